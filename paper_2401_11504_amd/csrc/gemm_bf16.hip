// bf16 MFMA GEMMs for the LoRA-adapted linear layers (gfx950, v_mfma_f32_32x32x16_bf16).
//
//  gemm_nt : C = alpha (A B^T + A2 B2^T) (+ R)      both operand pairs are K-contiguous.
//            Forward:  Y  = X W^T  + Hs B^T           (A2 = Hs = s X A^T, K2 = r)
//            Backward: dX = dY Wt^T + dH At^T          (Wt, At = transposed copies, K2 = r)
//            Low-rank: Hs = s X A^T, dH = s dY Bt^T    (N = r, split over K)
//            The low-rank term rides along as extra K tiles of the same accumulator, so the
//            frozen product and the LoRA correction are one pass over the output.
//  gemm_tn : C = alpha P^T Q, contraction over the token dimension (dA = dH^T X, dB = dY^T Hs),
//            fp32 output.  Operand tiles are transposed on their way into LDS.
//
// LDS tiles hold 64 contraction elements per row, padded to 72 so that the 16-byte fragment
// reads of 8 consecutive rows fall into distinct banks.
#include "kernels.h"
#include "tiles.h"

// ======================================================================== NT
template <int BM, int BN, int WM, int WN, bool PARTIAL>
__global__ __launch_bounds__(256) void gemm_nt_kernel(GemmNT p, int tiles_m, int tiles_n, int split_k) {
    extern __shared__ __align__(16) unsigned char smem[];
    bf16_t* sA = (bf16_t*)smem;       // [2][BM * LS]
    bf16_t* sB = sA + 2 * BM * LS;    // [2][BN * LS]
    constexpr int TM = BM / WM, TN = BN / WN, FM = TM / 32, FN = TN / 32;
    constexpr int CA = BM / 32, CB = BN / 32;  // 16-byte chunks per thread per tile
    static_assert(WM * WN == 4 && FM >= 1 && FN >= 1, "4 waves");

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave / WN, wn = wave % WN;
    const int l32 = lane & 31, g = lane >> 5;

    // XCD-aware tile order: consecutive workgroup ids go round-robin over the 8 XCDs, so give
    // XCD x the contiguous tile range [x * n/8, (x+1) * n/8): its CUs then share W columns in its L2.
    const int ntiles = tiles_m * tiles_n;
    int pid = blockIdx.x;
    if ((ntiles & 7) == 0) pid = (pid & 7) * (ntiles >> 3) + (pid >> 3);
    const int tile_m = pid % tiles_m, tile_n = pid / tiles_m;
    const int m0 = tile_m * BM, n0 = tile_n * BN;
    const int z = blockIdx.z, split = blockIdx.y;

    const bf16_t* A = p.A + (long)z * p.bA;
    const bf16_t* B = p.B + (long)z * p.bB;
    const bf16_t* A2 = p.A2 ? p.A2 + (long)z * p.bA2 : nullptr;
    const bf16_t* B2 = p.B2 ? p.B2 + (long)z * p.bB2 : nullptr;

    const int nk1 = (p.K + BK - 1) / BK, nk2 = (p.K2 + BK - 1) / BK;
    const int nk = nk1 + nk2;
    const int kt_begin = (int)((long)nk * split / split_k), kt_end = (int)((long)nk * (split + 1) / split_k);

    uint4 ra[CA], rb[CB];
    auto gload = [&](int kt) {
        const bf16_t *pa, *pb;
        long la, lb;
        int k0, kmax;
        if (kt < nk1) { pa = A; pb = B; la = p.lda; lb = p.ldb; k0 = kt * BK; kmax = p.K; }
        else { pa = A2; pb = B2; la = p.lda2; lb = p.ldb2; k0 = (kt - nk1) * BK; kmax = p.K2; }
#pragma unroll
        for (int i = 0; i < CA; ++i) {
            const int c = tid + 256 * i, row = c >> 3, kk = k0 + (c & 7) * 8;
            ra[i] = (m0 + row < p.M && kk < kmax) ? *(const uint4*)(pa + (long)(m0 + row) * la + kk)
                                                  : make_uint4(0, 0, 0, 0);
        }
#pragma unroll
        for (int i = 0; i < CB; ++i) {
            const int c = tid + 256 * i, row = c >> 3, kk = k0 + (c & 7) * 8;
            rb[i] = (n0 + row < p.N && kk < kmax) ? *(const uint4*)(pb + (long)(n0 + row) * lb + kk)
                                                  : make_uint4(0, 0, 0, 0);
        }
    };
    auto sstore = [&](int buf) {
        bf16_t* a = sA + buf * BM * LS;
        bf16_t* b = sB + buf * BN * LS;
#pragma unroll
        for (int i = 0; i < CA; ++i) {
            const int c = tid + 256 * i;
            *(uint4*)(a + (c >> 3) * LS + (c & 7) * 8) = ra[i];
        }
#pragma unroll
        for (int i = 0; i < CB; ++i) {
            const int c = tid + 256 * i;
            *(uint4*)(b + (c >> 3) * LS + (c & 7) * 8) = rb[i];
        }
    };

    f32x16_t acc[FM][FN];
#pragma unroll
    for (int i = 0; i < FM; ++i)
#pragma unroll
        for (int j = 0; j < FN; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;

    if (kt_begin < kt_end) {
        gload(kt_begin);
        sstore(0);
    }
    __syncthreads();
    for (int kt = kt_begin; kt < kt_end; ++kt) {
        const int buf = (kt - kt_begin) & 1;
        if (kt + 1 < kt_end) gload(kt + 1);
        const bf16_t* a = sA + buf * BM * LS + (wm * TM + l32) * LS + g * 8;
        const bf16_t* b = sB + buf * BN * LS + (wn * TN + l32) * LS + g * 8;
#pragma unroll
        for (int ks = 0; ks < BK / 16; ++ks) {
            bf16x8_t fa[FM], fb[FN];
#pragma unroll
            for (int i = 0; i < FM; ++i) fa[i] = *(const bf16x8_t*)(a + i * 32 * LS + ks * 16);
#pragma unroll
            for (int j = 0; j < FN; ++j) fb[j] = *(const bf16x8_t*)(b + j * 32 * LS + ks * 16);
#pragma unroll
            for (int i = 0; i < FM; ++i)
#pragma unroll
                for (int j = 0; j < FN; ++j) acc[i][j] = mfma32(fa[i], fb[j], acc[i][j]);
        }
        if (kt + 1 < kt_end) sstore(buf ^ 1);
        __syncthreads();
    }

    // epilogue: lane holds column l32 and rows 8*(v/4) + 4*g + v%4 of each 32x32 fragment
#pragma unroll
    for (int i = 0; i < FM; ++i)
#pragma unroll
        for (int j = 0; j < FN; ++j) {
            const int col = n0 + wn * TN + j * 32 + l32;
            if (col >= p.N) continue;
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int row = m0 + wm * TM + i * 32 + 8 * (v >> 2) + 4 * g + (v & 3);
                if (row >= p.M) continue;
                if (PARTIAL) {
                    p.partial[(((long)z * split_k + split) * p.M + row) * p.N + col] = acc[i][j][v];
                } else {
                    const long off = (long)z * p.bC + (long)row * p.ldc + col;
                    float val = p.alpha * acc[i][j][v];
                    if (p.c_f32) {
                        if (p.R) val += p.R[off];
                        ((float*)p.C)[off] = val;
                    } else {
                        ((bf16_t*)p.C)[off] = f32_to_bf16(val);
                    }
                }
            }
        }
}

// sum the split-K partials in a fixed order (deterministic), scale, add residual, convert
__global__ __launch_bounds__(256) void splitk_reduce_kernel(GemmNT p, int split_k) {
    const long mn = (long)p.M * p.N;
    const long idx = (long)blockIdx.x * blockDim.x + threadIdx.x;
    if (idx >= mn * p.batch) return;
    const int z = (int)(idx / mn);
    const long r = idx % mn;
    const int row = (int)(r / p.N), col = (int)(r % p.N);
    float s = 0.f;
    for (int k = 0; k < split_k; ++k) s += p.partial[((long)z * split_k + k) * mn + r];
    const long off = (long)z * p.bC + (long)row * p.ldc + col;
    float val = p.alpha * s;
    if (p.c_f32) {
        if (p.R) val += p.R[off];
        ((float*)p.C)[off] = val;
    } else {
        ((bf16_t*)p.C)[off] = f32_to_bf16(val);
    }
}

template <int BM, int BN, int WM, int WN>
static hipError_t run_nt(const GemmNT& g, int split_k, hipStream_t s) {
    const int tiles_m = cdiv(g.M, BM), tiles_n = cdiv(g.N, BN);
    const size_t lds = (size_t)2 * (BM + BN) * LS * sizeof(bf16_t);
    dim3 grid(tiles_m * tiles_n, split_k, g.batch);
    hipError_t e;
    if (split_k > 1) {
        auto kern = gemm_nt_kernel<BM, BN, WM, WN, true>;
        e = hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        if (e != hipSuccess) return e;
        kern<<<grid, 256, lds, s>>>(g, tiles_m, tiles_n, split_k);
        const long n = (long)g.M * g.N * g.batch;
        splitk_reduce_kernel<<<cdiv(n, 256), 256, 0, s>>>(g, split_k);
    } else {
        auto kern = gemm_nt_kernel<BM, BN, WM, WN, false>;
        e = hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        if (e != hipSuccess) return e;
        kern<<<grid, 256, lds, s>>>(g, tiles_m, tiles_n, 1);
    }
    return hipGetLastError();
}

hipError_t launch_gemm_nt(const GemmNT& g, hipStream_t s) {
    if (g.M <= 0 || g.N <= 0 || g.batch <= 0) return hipSuccess;
    if ((g.K & 7) || (g.K2 & 7) || (g.lda & 7) || (g.ldb & 7) || (g.lda2 & 7) || (g.ldb2 & 7)) return hipErrorInvalidValue;
    if ((g.bA & 7) || (g.bB & 7) || (g.bA2 & 7) || (g.bB2 & 7)) return hipErrorInvalidValue;
    if (!g.c_f32 && g.R) return hipErrorInvalidValue;
    const int nk = cdiv(g.K, BK) + cdiv(g.K2, BK);
    const long t128 = (long)cdiv(g.M, 128) * cdiv(g.N, 128) * g.batch;
    const long t64n = (long)cdiv(g.M, 128) * cdiv(g.N, 64) * g.batch;
    int split = g.split_k;
    if (g.N > 64 && t128 >= 200) {
        return run_nt<128, 128, 2, 2>(g, 1, s);
    }
    if (g.N > 64 && t64n >= 200) {
        return run_nt<128, 64, 2, 2>(g, 1, s);
    }
    // few output tiles: 64x64 tiles, and split the contraction when scratch is available
    const long t64 = (long)cdiv(g.M, 64) * cdiv(g.N, 64) * g.batch;
    if (split == 0) {
        split = 1;
        if (g.partial && t64 < 256) {
            split = (int)(512 / t64);
            if (split > nk / 4) split = nk / 4;
            if (split < 1) split = 1;
            while (split > 1 && (size_t)split * g.M * g.N * g.batch > g.partial_elems) --split;
        }
    }
    if (split > 1 && (!g.partial || (size_t)split * g.M * g.N * g.batch > g.partial_elems)) return hipErrorInvalidValue;
    if (split > nk) split = nk > 0 ? nk : 1;
    return run_nt<64, 64, 2, 2>(g, split, s);
}

// ======================================================================== TN
// Transposing store of a [64 t][64 i] operand tile: thread (tp, ic) holds rows t = 2tp, 2tp+1 and the
// 8 columns i = 8ic..8ic+7, and writes 8 dwords (t, t+1) pairs into the [i][t] LDS tile.  The 8-element
// t-chunk index is XORed with (i / 8) % 8 so that the 8 column groups of one row land in distinct banks.
__global__ __launch_bounds__(256) void gemm_tn_kernel(GemmTN p) {
    __shared__ __align__(16) bf16_t sP[64 * LS];
    __shared__ __align__(16) bf16_t sQ[64 * LS];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wi = wave >> 1, wj = wave & 1, l32 = lane & 31, g = lane >> 5;
    const int i0 = blockIdx.y * 64, j0 = blockIdx.x * 64, z = blockIdx.z;
    const bf16_t* P = p.P + (long)z * p.bP;
    const bf16_t* Q = p.Q + (long)z * p.bQ;
    const int tp = tid >> 3, ic = tid & 7;

    f32x16_t acc;
#pragma unroll
    for (int v = 0; v < 16; ++v) acc[v] = 0.f;

    auto ld = [&](const bf16_t* base, long ldx, int c0, int cmax, int t) -> uint4 {
        const int c = c0 + ic * 8;
        return (t < p.T && c < cmax) ? *(const uint4*)(base + (long)t * ldx + c) : make_uint4(0, 0, 0, 0);
    };
    const int nt = (p.T + 63) / 64;
    uint4 p0, p1, q0, q1;
    p0 = ld(P, p.ldp, i0, p.Mo, 2 * tp); p1 = ld(P, p.ldp, i0, p.Mo, 2 * tp + 1);
    q0 = ld(Q, p.ldq, j0, p.No, 2 * tp); q1 = ld(Q, p.ldq, j0, p.No, 2 * tp + 1);
    for (int it = 0; it < nt; ++it) {
        __syncthreads();
        store_transposed_pair(sP, ic * 8, 2 * tp, p0, p1);
        store_transposed_pair(sQ, ic * 8, 2 * tp, q0, q1);
        __syncthreads();
        if (it + 1 < nt) {
            const int t = (it + 1) * 64 + 2 * tp;
            p0 = ld(P, p.ldp, i0, p.Mo, t); p1 = ld(P, p.ldp, i0, p.Mo, t + 1);
            q0 = ld(Q, p.ldq, j0, p.No, t); q1 = ld(Q, p.ldq, j0, p.No, t + 1);
        }
        const int ri = wi * 32 + l32, rj = wj * 32 + l32;
#pragma unroll
        for (int ks = 0; ks < 4; ++ks) {
            bf16x8_t a = *(const bf16x8_t*)(sP + tn_off(ri, ks * 16 + g * 8));
            bf16x8_t b = *(const bf16x8_t*)(sQ + tn_off(rj, ks * 16 + g * 8));
            acc = mfma32(a, b, acc);
        }
    }
    const int col = j0 + wj * 32 + l32;
    if (col < p.No) {
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            const int row = i0 + wi * 32 + 8 * (v >> 2) + 4 * g + (v & 3);
            if (row < p.Mo) p.C[(long)z * p.bC + (long)row * p.ldc + col] = p.alpha * acc[v];
        }
    }
}

hipError_t launch_gemm_tn(const GemmTN& g, hipStream_t s) {
    if (g.Mo <= 0 || g.No <= 0 || g.batch <= 0) return hipSuccess;
    if ((g.ldp & 7) || (g.ldq & 7) || (g.Mo & 7) || (g.No & 7) || (g.bP & 7) || (g.bQ & 7)) return hipErrorInvalidValue;
    dim3 grid(cdiv(g.No, 64), cdiv(g.Mo, 64), g.batch);
    gemm_tn_kernel<<<grid, 256, 0, s>>>(g);
    return hipGetLastError();
}
