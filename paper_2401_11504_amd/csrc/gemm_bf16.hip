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
#include <type_traits>

// ======================================================================== NT
// Workgroup ids go round-robin over the 8 XCDs (each with its own L2).  XCD c therefore runs ids c, c + 8, ..: give
// it the contiguous tile range that starts after the ranges of XCDs 0 .. c-1 (the first n % 8 XCDs hold one tile
// more), so that the CUs of one XCD work on neighbouring tiles and share operand rows in their L2.
__device__ __forceinline__ int xcd_contiguous(int id, int n) {
    const int c = id & 7, q = n >> 3, rem = n & 7;
    return c * q + min(c, rem) + (id >> 3);
}

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
    pid = xcd_contiguous(pid, ntiles);
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


__global__ void splitk_reduce_kernel(GemmNT p, int split_k);

// ======================================================================== NT, direct-to-LDS pipeline
// Same contract as gemm_nt_kernel for K % 64 == 0 and K2 % 64 == 0.  Operand tiles go from global
// memory straight into LDS (global_load_lds_dwordx4: each lane's 16 bytes land at M0 + 16 * lane), so a
// ring of STAGES tiles is in flight without staging registers.  A tile row is 64 bf16 = 8 chunks of
// 16 bytes; chunk c of row r is kept at position c ^ ((r / 2) % 8), chosen by which global chunk each
// lane fetches.  The LDS serves 16 lanes x 16 bytes per clock from 64 banks, and two 128-byte rows span
// the 64 banks once, so 16 consecutive rows reading the same logical chunk must land on 8 distinct
// positions in the even rows and 8 in the odd rows: that is what the (r / 2) term gives.
// Rows beyond M / N are clamped to the last valid row: they only feed outputs that are never stored.
__device__ __forceinline__ void load_lds16(unsigned voff, const void* sbase, unsigned lds_addr) {
    // M0 carries the LDS destination: bound as a physical-register operand, so the compiler sets it and knows it is used
    asm volatile("global_load_lds_dwordx4 %0, %1" ::"v"(voff), "s"(sbase), "{m0}"(lds_addr) : "memory");
}
template <int N>
__device__ __forceinline__ void wait_vmcnt() {
    asm volatile("s_waitcnt vmcnt(%0)" ::"n"(N) : "memory");
}

// How a launch maps workgroup ids to tiles and contraction ranges, worked out on the host: the kernel's prologue is
// exposed time on every launch, and integer divisions by run-time values cost it dozens of scalar instructions each.
// q = n / d for the small n that occur here is umulhi(n, ceil(2^32 / d)) (exact while n * d < 2^32).
struct NtMap {
    int tiles_m, tiles_n;
    unsigned inv_tiles_m;    // ceil(2^32 / tiles_m)
    unsigned inv_n_split;    // ceil(2^32 / n_split)
    int xcd_split;           // 1: the XCD a workgroup runs on also fixes its split (n_split 2, 4 or 8 and tiles divide evenly)
    int xs_log2;             // log2 of the XCDs per split in that case
    int tiles_per_xs;        // tiles / XCDs per split
};
static NtMap make_nt_map(int tiles_m, int tiles_n, int n_split, int batch, bool splitk) {
    NtMap m;
    m.tiles_m = tiles_m;
    m.tiles_n = tiles_n;
    m.inv_tiles_m = (unsigned)((0x100000000ull + (unsigned)tiles_m - 1) / (unsigned)tiles_m);
    m.inv_n_split = (unsigned)((0x100000000ull + (unsigned)n_split - 1) / (unsigned)n_split);
    const int ntiles = tiles_m * tiles_n, xs = 8 / (n_split > 0 ? n_split : 1);
    m.xcd_split = splitk && batch == 1 && (n_split == 2 || n_split == 4 || n_split == 8) && ntiles % xs == 0;
    m.xs_log2 = xs == 4 ? 2 : xs == 2 ? 1 : 0;
    m.tiles_per_xs = m.xcd_split ? ntiles / xs : 0;
    return m;
}
__device__ __forceinline__ unsigned div_by(unsigned n, unsigned inv) { return inv == 0 ? n : __umulhi(n, inv); }   // inv == 0 encodes d = 1

template <int BM, int BN, int WM, int WN, int STAGES, int BKT = 64, bool SPLITK = false, int PIPE = 0>
__global__ __launch_bounds__(WM* WN * 64) void gemm_nt_dl_kernel(GemmNT p, NtMap map) {
    constexpr int NT = WM * WN * 64;
    constexpr int ROWS = BM + BN;
    constexpr int CPRW = BKT / 8;             // 16-byte chunks per tile row
    constexpr int RP = 256 / (BKT * 2);       // tile rows per 256 bytes of LDS (one pass over the 64 banks)
    constexpr int KS = BKT / 16;              // MFMA k-steps per tile
    constexpr int L = ROWS * CPRW / NT;       // 16-byte loads per thread per stage
    constexpr int LA = BM * CPRW / NT;        // the first LA of them fetch A rows
    constexpr int ROWB = BKT * 2;             // bytes per tile row
    constexpr int STAGE_BYTES = ROWS * ROWB;
    constexpr int TM = BM / WM, TN = BN / WN, FM = TM / 32, FN = TN / 32;
    static_assert((ROWS * CPRW) % NT == 0 && (BM * CPRW) % NT == 0 && FM >= 1 && FN >= 1 && STAGES >= 2, "tile shape");
    static_assert((STAGES - 2) * L <= 63, "vmcnt range");  // s_waitcnt vmcnt is a 6-bit field
    static_assert(BKT == 64 || BKT == 32, "tile depth");
    extern __shared__ __align__(16) unsigned char smem[];
    const unsigned lds0 = (unsigned)(size_t)smem;

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave / WN, wn = wave % WN;
    const int l32 = lane & 31, g = lane >> 5;

    // Workgroup ids go round-robin over the 8 XCDs (x fastest, then y), each with its own L2: XCD c gets a contiguous
    // range of tiles (m fastest), so that its CUs share weight rows.  With the contraction split 2, 4 or 8 ways the
    // XCD also fixes the split: XCD c works on split c / (8 / n_split) only, so an XCD fetches just its share of the
    // contraction range of the activations instead of all of it.
    const int tiles_m = map.tiles_m, tiles_n = map.tiles_n;
    const int ntiles = tiles_m * tiles_n;
    const int n_split = SPLITK ? (int)gridDim.y : 1;
    int pid = blockIdx.x, split = SPLITK ? (int)blockIdx.y : 0;
    if (SPLITK && map.xcd_split) {
        const int id = blockIdx.y * gridDim.x + blockIdx.x, c = id & 7, j = id >> 3;
        split = c >> map.xs_log2;
        pid = (c & ((1 << map.xs_log2) - 1)) * map.tiles_per_xs + j;
    } else {
        pid = xcd_contiguous(pid, ntiles);
    }
    const int tile_n = (int)div_by((unsigned)pid, map.inv_tiles_m), tile_m = pid - tile_n * tiles_m;
    const int m0 = tile_m * BM, n0 = tile_n * BN;
    const int z = blockIdx.z;

    const bf16_t* A = p.A + (long)z * p.bA;
    const bf16_t* B = p.B + (long)z * p.bB;
    const bf16_t* A2 = p.A2 ? p.A2 + (long)z * p.bA2 : nullptr;
    const bf16_t* B2 = p.B2 ? p.B2 + (long)z * p.bB2 : nullptr;
    const int nk1 = p.K / BKT, nk2 = p.K2 / BKT;
    // with SPLITK, n_split workgroups share one output tile: this one takes k-tiles [kt0, kt0 + nk)
    const int kt0 = SPLITK ? (int)div_by((unsigned)((nk1 + nk2) * split), map.inv_n_split) : 0;
    const int nk = (SPLITK ? (int)div_by((unsigned)((nk1 + nk2) * (split + 1)), map.inv_n_split) : nk1 + nk2) - kt0;

    // per-thread byte offsets of its L chunks, for the main and the low-rank operand pair
    unsigned vo1[L], vo2[L];
#pragma unroll
    for (int j = 0; j < L; ++j) {
        const int q = j * NT + tid, r = q / CPRW, c = (q % CPRW) ^ ((r / RP) % CPRW);
        // 32-bit arithmetic: the launcher only takes this path for operands below 2^30 elements
        if (j < LA) {
            const unsigned row = (unsigned)min(m0 + r, p.M - 1);
            vo1[j] = (row * (unsigned)p.lda + c * 8) * 2;
            vo2[j] = (row * (unsigned)p.lda2 + c * 8) * 2;
        } else {
            const unsigned row = (unsigned)min(n0 + r - BM, p.N - 1);
            vo1[j] = (row * (unsigned)p.ldb + c * 8) * 2;
            vo2[j] = (row * (unsigned)p.ldb2 + c * 8) * 2;
        }
    }
    auto issue = [&](int ktl) {
        const unsigned dst = __builtin_amdgcn_readfirstlane(lds0 + (ktl % STAGES) * STAGE_BYTES + wave * 1024);
        const int kt = kt0 + ktl;
        if (kt < nk1) {
            const bf16_t* ba = A + (long)kt * BKT;
            const bf16_t* bb = B + (long)kt * BKT;
#pragma unroll
            for (int j = 0; j < L; ++j) load_lds16(vo1[j], j < LA ? (const void*)ba : (const void*)bb, dst + j * NT * 16);
        } else {
            const bf16_t* ba = A2 + (long)(kt - nk1) * BKT;
            const bf16_t* bb = B2 + (long)(kt - nk1) * BKT;
#pragma unroll
            for (int j = 0; j < L; ++j) load_lds16(vo2[j], j < LA ? (const void*)ba : (const void*)bb, dst + j * NT * 16);
        }
    };

    f32x16_t acc[FM][FN];
#pragma unroll
    for (int i = 0; i < FM; ++i)
#pragma unroll
        for (int j = 0; j < FN; ++j) acc[i][j] = zero16();

    // fragment read offsets: row (w*T + l32) -> swizzle (l32 / RP) % CPRW; chunk (2 ks + g) ^ swizzle
    int coff[KS];
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) coff[ks] = (((2 * ks + g) ^ ((l32 / RP) % CPRW)) << 4);
    const int a_row = (wm * TM + l32) * ROWB, b_row = (BM + wn * TN + l32) * ROWB;

    if constexpr (PIPE != 0) {
        // One wave per SIMD: the matrix pipe only stays busy if the wave never waits, so inside the steady-state
        // loop nothing is issued in bursts.  Tile kt+STAGES-1 is fetched during iteration kt, its 16-byte
        // global->LDS loads spread evenly between the MFMAs (a burst of L loads would hold the wave at the address
        // unit for hundreds of clocks), and the fragments of the k-step PD steps ahead are read one per MFMA slot
        // while the current k-step's MFMAs run (PD = PIPE; with 64x64 wave tiles a k-step is only 128 clocks of
        // MFMA, less than an LDS round trip under load, hence PD = 2 there).  The loop body has no branches; the
        // last STAGES-1 tiles, which fetch nothing, run in a peeled tail.  The host only picks this path for
        // nk >= STAGES.
        constexpr int PD = PIPE, NSETS = PD == 1 ? 2 : 4, HS = KS - PD;   // hand-over happens before k-step HS
        static_assert(PD == 1 || (PD == 2 && KS == 4), "prefetch distance");
        static_assert(STAGES >= 3 && KS * FM * FN >= L && KS % NSETS == 0, "slots");
        constexpr int NMF = FM * FN, NRD = FM + FN, NSLOT = KS * NMF, RPS = (NRD + NMF - 1) / NMF;
        // load j of a tile goes into slot j * NSLOT / L; LBH = loads issued before the hand-over
        constexpr int LBH = (HS * NMF * L + NSLOT - 1) / NSLOT;
        const unsigned char* a_ptr = smem + a_row;
        const unsigned char* b_ptr = smem + b_row;
        bf16x8_t fa[NSETS][FM], fb[NSETS][FN];
        // one k-step: NMF MFMAs on fragment set ks % NSETS; the slot after MFMA e carries one fragment read of the
        // k-step PD ahead (RPS per slot until all NRD are issued); the tile's L DMA loads are spread evenly over its KS * NMF slots
        auto kstep = [&](auto loads_c, unsigned ext, auto reads_c, int ks, size_t rd_stage, int rd_ks,
                         const bf16_t* pa, const bf16_t* pb, unsigned dst) {
            constexpr bool LOADS = decltype(loads_c)::value, READS = decltype(reads_c)::value;
            const int cur = ks % NSETS, nxt = (ks + PD) % NSETS;
#pragma unroll
            for (int e = 0; e < NMF; ++e) {
                acc[e / FN][e % FN] = mfma32(fa[cur][e / FN], fb[cur][e % FN], acc[e / FN][e % FN]);
                if constexpr (READS) {
                    // RPS reads per slot, in the order A0, B0..B(FN-1), A1..: what that k-step's first MFMAs need first
#pragma unroll
                    for (int r = e * RPS; r < (e + 1) * RPS && r < NRD; ++r) {
                        if (r == 0) fa[nxt][0] = *(const bf16x8_t*)(a_ptr + rd_stage + coff[rd_ks]);
                        else if (r <= FN) fb[nxt][r - 1] = *(const bf16x8_t*)(b_ptr + rd_stage + (r - 1) * 32 * ROWB + coff[rd_ks]);
                        else fa[nxt][r - FN] = *(const bf16x8_t*)(a_ptr + rd_stage + (r - FN) * 32 * ROWB + coff[rd_ks]);
                    }
                }
                if constexpr (LOADS) {
                    const int gs = ks * NMF + e;          // slot number within the tile
                    const int j = (gs * L + NSLOT - 1) / NSLOT;   // first load with j * NSLOT / L >= gs
                    if (j < L && j * NSLOT / L == gs) {
                        // vo2 - vo1 is folded in arithmetically (ext is 0 or 1, wave-uniform): one loop body serves both pairs
                        load_lds16(vo1[j] + ext * vo2[j], j < LA ? (const void*)pa : (const void*)pb, dst + j * NT * 16);
                    }
                }
                __builtin_amdgcn_sched_barrier(0);
            }
        };
        // one tile; HW = loads that may still be outstanding at the hand-over so that tile kt+1 has landed
        auto tile = [&](auto loads_c, auto hw_c, auto last_c, int kt) {
            constexpr int HW = decltype(hw_c)::value;
            constexpr bool LAST = decltype(last_c)::value;
            const int tn = kt + STAGES - 1;
            const int ktn = kt0 + tn;
            const unsigned ext_c = ktn >= nk1 ? 1u : 0u;
            const bf16_t* pa = ext_c ? A2 + (long)(ktn - nk1) * BKT : A + (long)ktn * BKT;
            const bf16_t* pb = ext_c ? B2 + (long)(ktn - nk1) * BKT : B + (long)ktn * BKT;
            const unsigned dst = __builtin_amdgcn_readfirstlane(lds0 + (tn % STAGES) * STAGE_BYTES + wave * 1024);
            const size_t st_cur = (size_t)(kt % STAGES) * STAGE_BYTES, st_nxt = (size_t)((kt + 1) % STAGES) * STAGE_BYTES;
#pragma unroll
            for (int ks = 0; ks < KS; ++ks) {
                if (ks < HS) {
                    kstep(loads_c, ext_c, std::true_type{}, ks, st_cur, ks + PD, pa, pb, dst);
                } else if constexpr (!LAST) {
                    if (ks == HS) {
                        // hand-over: every wave's reads of this tile are complete (so its buffer may be refilled from
                        // the next iteration on) and tile kt+1 has landed for every wave
                        asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
                        wait_vmcnt<HW>();
                        __builtin_amdgcn_s_barrier();
                        asm volatile("" ::: "memory");
                    }
                    kstep(loads_c, ext_c, std::true_type{}, ks, st_nxt, ks + PD - KS, pa, pb, dst);
                } else {
                    kstep(std::false_type{}, 0u, std::false_type{}, ks, 0, 0, pa, pb, dst);
                }
            }
        };
#pragma unroll
        for (int s = 0; s < STAGES - 1; ++s) issue(s);
#pragma unroll
        for (int j = 0; j < L; ++j) vo2[j] -= vo1[j];
        wait_vmcnt<(STAGES - 2) * L>();
        __builtin_amdgcn_s_barrier();
        asm volatile("" ::: "memory");
#pragma unroll
        for (int ks = 0; ks < PD; ++ks) {
#pragma unroll
            for (int i = 0; i < FM; ++i) fa[ks][i] = *(const bf16x8_t*)(a_ptr + i * 32 * ROWB + coff[ks]);
#pragma unroll
            for (int j = 0; j < FN; ++j) fb[ks][j] = *(const bf16x8_t*)(b_ptr + j * 32 * ROWB + coff[ks]);
        }
        // at the hand-over of a steady-state tile, tile kt+2.. and the LBH loads of tile kt+STAGES-1 issued
        // so far may be outstanding
        constexpr int HW_STEADY = (STAGES - 3) * L + LBH;
        static_assert(HW_STEADY <= 63, "vmcnt range");
        using T_ = std::true_type; using F_ = std::false_type;
        int kt = 0;
        // (vo2 now holds the difference to vo1, see kstep)
        for (; kt + STAGES - 1 < nk; ++kt) tile(T_{}, std::integral_constant<int, HW_STEADY>{}, F_{}, kt);
        // tail: tiles nk-STAGES+1 .. nk-1 fetch nothing; with r tiles after this one, r-1 of them may be in flight
        auto tail = [&](auto self, auto r_c) -> void {
            constexpr int R = decltype(r_c)::value;
            if constexpr (R > 0) {
                tile(F_{}, std::integral_constant<int, (R - 1) * L>{}, F_{}, kt);
                ++kt;
                self(self, std::integral_constant<int, R - 1>{});
            } else {
                tile(F_{}, std::integral_constant<int, 0>{}, T_{}, kt);
            }
        };
        tail(tail, std::integral_constant<int, STAGES - 2>{});
    } else if constexpr (STAGES >= 3) {
#pragma unroll
        for (int s = 0; s < STAGES - 1; ++s)
            if (s < nk) issue(s);
        // Software pipeline: the fragments of k-step ks+1 are read while the MFMAs of ks run, and the
        // hand-over to the next tile (wait, barrier, next global loads, first fragments) happens before
        // the last k-step's MFMAs, so the matrix pipe never waits for LDS at a tile boundary.
        auto read_frags = [&](int stage, int ks, bf16x8_t* fa, bf16x8_t* fb) {
            const unsigned char* st = smem + stage * STAGE_BYTES;
#pragma unroll
            for (int i = 0; i < FM; ++i) fa[i] = *(const bf16x8_t*)(st + a_row + i * 32 * ROWB + coff[ks]);
#pragma unroll
            for (int j = 0; j < FN; ++j) fb[j] = *(const bf16x8_t*)(st + b_row + j * 32 * ROWB + coff[ks]);
        };
        if (STAGES - 2 < nk) wait_vmcnt<(STAGES - 2) * L>(); else wait_vmcnt<0>();
        __builtin_amdgcn_s_barrier();
        asm volatile("" ::: "memory");
        bf16x8_t fa[2][FM], fb[2][FN];
        read_frags(0, 0, fa[0], fb[0]);
        for (int kt = 0; kt < nk; ++kt) {
            const int stg = kt % STAGES;
#pragma unroll
            for (int ks = 0; ks < KS; ++ks) {
                const int cur = ks & 1, nxt = cur ^ 1;
                if (ks < KS - 1) {
                    read_frags(stg, ks + 1, fa[nxt], fb[nxt]);
                } else if (kt + 1 < nk) {
                    if (kt + STAGES - 2 < nk) wait_vmcnt<(STAGES - 3) * L>(); else wait_vmcnt<0>();
                    __builtin_amdgcn_s_barrier();
                    asm volatile("" ::: "memory");
                    if (kt + STAGES - 1 < nk) issue(kt + STAGES - 1);
                    read_frags((kt + 1) % STAGES, 0, fa[nxt], fb[nxt]);
                }
#pragma unroll
                for (int i = 0; i < FM; ++i)
#pragma unroll
                    for (int j = 0; j < FN; ++j) acc[i][j] = mfma32(fa[cur][i], fb[cur][j], acc[i][j]);
            }
        }
    } else {
#pragma unroll
        for (int s = 0; s < STAGES - 1; ++s)
            if (s < nk) issue(s);
        for (int kt = 0; kt < nk; ++kt) {
            // tile kt has landed once at most the loads of the STAGES-2 younger tiles are outstanding
            if (kt + STAGES - 2 < nk) wait_vmcnt<(STAGES - 2) * L>(); else wait_vmcnt<0>();
            __builtin_amdgcn_s_barrier();
            asm volatile("" ::: "memory");
            if (kt + STAGES - 1 < nk) issue(kt + STAGES - 1);   // into the buffer every wave finished reading last iteration
            const unsigned char* st = smem + (kt % STAGES) * STAGE_BYTES;
#pragma unroll
            for (int ks = 0; ks < KS; ++ks) {
                bf16x8_t fa[FM], fb[FN];
#pragma unroll
                for (int i = 0; i < FM; ++i) fa[i] = *(const bf16x8_t*)(st + a_row + i * 32 * ROWB + coff[ks]);
#pragma unroll
                for (int j = 0; j < FN; ++j) fb[j] = *(const bf16x8_t*)(st + b_row + j * 32 * ROWB + coff[ks]);
#pragma unroll
                for (int i = 0; i < FM; ++i)
#pragma unroll
                    for (int j = 0; j < FN; ++j) acc[i][j] = mfma32(fa[i], fb[j], acc[i][j]);
            }
        }
    }

    bool bf16_partials = false;
    if constexpr (SPLITK) bf16_partials = p.partial_bf16 != 0;
    if (SPLITK && !bf16_partials) {
        // each split stores its fp32 tile; splitk_reduce_kernel adds the splits in index order afterwards
        // (a second launch: device-wide fences inside a kernel cost a full L2 write-back on this chip)
        float* part = p.partial + ((long)z * n_split + split) * (long)p.M * p.N;
        if (m0 + BM <= p.M && n0 + BN <= p.N) {
            // a whole tile (workgroup-uniform): no bounds checks, one base address per lane
            float* base = part + (long)(m0 + wm * TM + 4 * g) * p.N + n0 + wn * TN + l32;
#pragma unroll
            for (int i = 0; i < FM; ++i)
#pragma unroll
                for (int j = 0; j < FN; ++j)
#pragma unroll
                    for (int v = 0; v < 16; ++v)
                        base[(long)(i * 32 + 8 * (v >> 2) + (v & 3)) * p.N + j * 32] = acc[i][j][v];
            return;
        }
#pragma unroll
        for (int i = 0; i < FM; ++i)
#pragma unroll
            for (int j = 0; j < FN; ++j) {
                const int col = n0 + wn * TN + j * 32 + l32;
                if (col >= p.N) continue;
#pragma unroll
                for (int v = 0; v < 16; ++v) {
                    const int row = m0 + wm * TM + i * 32 + 8 * (v >> 2) + 4 * g + (v & 3);
                    if (row < p.M) part[(long)row * p.N + col] = acc[i][j][v];
                }
            }
        return;
    }
    if (p.c_f32 && !bf16_partials) {
        // fp32 output (+ fp32 residual): half a wave already writes 128 contiguous bytes per row
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
                    const long off = (long)z * p.bC + (long)row * p.ldc + col;
                    float val = p.alpha * acc[i][j][v];
                    if (p.R) val += p.R[off];
                    ((float*)p.C)[off] = val;
                }
            }
    } else {
        // bf16 output: each wave turns 32-row slabs of its tile around in LDS so that a row leaves as
        // 16-byte pieces covering TN contiguous columns instead of 2-byte pieces
        constexpr int SLD = TN + 8;  // slab row stride in elements
        static_assert(WM * WN * 32 * SLD * 2 <= STAGES * STAGE_BYTES, "epilogue slab fits in the tile ring");
        __builtin_amdgcn_s_barrier();  // every wave is done reading operand tiles
        asm volatile("" ::: "memory");
        bf16_t* slab = (bf16_t*)smem + wave * 32 * SLD;
        // a split whose consumer adds the tiles up itself and asked for bf16 ones: the split's tile leaves the same
        // way, unscaled, into its [M, N] slice of the scratch
        bf16_t* Cb = bf16_partials ? (bf16_t*)p.partial + ((long)z * n_split + split) * (long)p.M * p.N
                                   : (bf16_t*)p.C + (long)z * p.bC;
        const long ldc = bf16_partials ? (long)p.N : p.ldc;
        const float alpha = bf16_partials ? 1.f : p.alpha;
        const bool vec_ok = bf16_partials ? ((p.N & 7) == 0 && (((size_t)p.partial & 15) == 0) && (((long)p.M * p.N) & 7) == 0)
                                          : ((p.ldc & 7) == 0) && ((p.bC & 7) == 0) && (((size_t)p.C & 15) == 0);
#pragma unroll
        for (int i = 0; i < FM; ++i) {
#pragma unroll
            for (int j = 0; j < FN; ++j)
#pragma unroll
                for (int v = 0; v < 16; ++v)
                    slab[(8 * (v >> 2) + 4 * g + (v & 3)) * SLD + j * 32 + l32] = f32_to_bf16(alpha * acc[i][j][v]);
            __builtin_amdgcn_wave_barrier();
            asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
            constexpr int CPR = TN / 8;  // 16-byte chunks per slab row
            if (vec_ok && m0 + BM <= p.M && n0 + BN <= p.N) {
                // a whole tile with aligned rows (workgroup-uniform): no bounds checks
                bf16_t* tile = Cb + (long)(m0 + wm * TM + i * 32) * ldc + n0 + wn * TN;
#pragma unroll
                for (int c = lane; c < 32 * CPR; c += 64) {
                    const int r = c / CPR, cc = (c % CPR) * 8;
                    *(uint4*)(tile + (long)r * ldc + cc) = *(const uint4*)(slab + r * SLD + cc);
                }
                __builtin_amdgcn_wave_barrier();
                asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
                continue;
            }
#pragma unroll
            for (int c = lane; c < 32 * CPR; c += 64) {
                const int r = c / CPR, cc = (c % CPR) * 8;
                const int row = m0 + wm * TM + i * 32 + r, col = n0 + wn * TN + cc;
                if (row >= p.M || col >= p.N) continue;
                const uint4 val = *(const uint4*)(slab + r * SLD + cc);
                bf16_t* dst = Cb + (long)row * ldc + col;
                if (vec_ok && col + 8 <= p.N) {
                    *(uint4*)dst = val;
                } else {
                    // (taken apart by shifts: a pointer into `val` would put it, and a scratch allocation, into memory)
                    const uint32_t w[4] = {val.x, val.y, val.z, val.w};
#pragma unroll
                    for (int x = 0; x < 8; ++x)
                        if (col + x < p.N) dst[x] = (bf16_t)(w[x >> 1] >> (16 * (x & 1)));
                }
            }
            __builtin_amdgcn_wave_barrier();
            asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
        }
    }
}

template <int BM, int BN, int WM, int WN, int STAGES, int BKT = 64, bool SPLITK = false, int PIPE = 0>
static hipError_t run_nt_dl(const GemmNT& g, hipStream_t s, int n_split = 1) {
    const int tiles_m = cdiv(g.M, BM), tiles_n = cdiv(g.N, BN);
    const size_t lds = (size_t)STAGES * (BM + BN) * BKT * 2;
    dim3 grid(tiles_m * tiles_n, SPLITK ? n_split : 1, g.batch);
    auto kern = gemm_nt_dl_kernel<BM, BN, WM, WN, STAGES, BKT, SPLITK, PIPE>;
    if constexpr (PIPE != 0) {  // the branch-free steady-state loop assumes every split has at least STAGES k-tiles
        const int nkt = g.K / BKT + g.K2 / BKT;
        if (nkt / n_split < STAGES) return run_nt_dl<BM, BN, WM, WN, STAGES, BKT, SPLITK, 0>(g, s, n_split);
    }
    hipError_t e = hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    if (e != hipSuccess) return e;
    GemmNT gk = g;
    if (!(SPLITK && g.deferred && BM >= 256)) gk.partial_bf16 = 0;   // bf16 partial tiles only where the reduce is left to the consumer
    kern<<<grid, WM * WN * 64, lds, s>>>(gk, make_nt_map(tiles_m, tiles_n, SPLITK ? n_split : 1, g.batch, SPLITK));
    if (SPLITK) {
        if (g.deferred && BM >= 256) {    // wide-output instance: the consumer adds the partial tiles up
            *g.deferred = n_split;
            return hipGetLastError();
        }
        const long n = (long)g.M * (g.N >> 2) * g.batch;
        splitk_reduce_kernel<<<cdiv(n, 256), 256, 0, s>>>(g, n_split);
    }
    return hipGetLastError();
}

// sum the split-K partials in a fixed order (deterministic), scale, add residual, convert.  One thread owns four
// consecutive columns; the partials are fetched eight splits at a time before they are added, so that the loads
// of a batch are all in flight together instead of one L2 round trip per split.
__global__ __launch_bounds__(256) void splitk_reduce_kernel(GemmNT p, int split_k) {
    const long mn = (long)p.M * p.N;
    const int n4 = p.N >> 2;                      // N % 4 == 0 (checked by the launcher)
    const long idx = (long)blockIdx.x * blockDim.x + threadIdx.x;
    if (idx >= (long)p.M * n4 * p.batch) return;
    const int z = (int)(idx / ((long)p.M * n4));
    const long q = idx % ((long)p.M * n4);
    const int row = (int)(q / n4), col = (int)(q % n4) * 4;
    const float* src = p.partial + (long)z * split_k * mn + (long)row * p.N + col;
    float4 s = make_float4(0.f, 0.f, 0.f, 0.f);
    int k = 0;
    for (; k + 8 <= split_k; k += 8) {
        float4 t[8];
#pragma unroll
        for (int j = 0; j < 8; ++j) t[j] = *(const float4*)(src + (long)(k + j) * mn);
#pragma unroll
        for (int j = 0; j < 8; ++j) { s.x += t[j].x; s.y += t[j].y; s.z += t[j].z; s.w += t[j].w; }
    }
    for (; k < split_k; ++k) {
        const float4 t = *(const float4*)(src + (long)k * mn);
        s.x += t.x; s.y += t.y; s.z += t.z; s.w += t.w;
    }
    const long off = (long)z * p.bC + (long)row * p.ldc + col;
    const float v[4] = {p.alpha * s.x, p.alpha * s.y, p.alpha * s.z, p.alpha * s.w};
    if (p.c_f32) {
#pragma unroll
        for (int e = 0; e < 4; ++e) ((float*)p.C)[off + e] = v[e] + (p.R ? p.R[off + e] : 0.f);
    } else {
#pragma unroll
        for (int e = 0; e < 4; ++e) ((bf16_t*)p.C)[off + e] = f32_to_bf16(v[e]);
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
        const long n = (long)g.M * (g.N >> 2) * g.batch;
        splitk_reduce_kernel<<<cdiv(n, 256), 256, 0, s>>>(g, split_k);
    } else {
        auto kern = gemm_nt_kernel<BM, BN, WM, WN, false>;
        e = hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        if (e != hipSuccess) return e;
        kern<<<grid, 256, lds, s>>>(g, tiles_m, tiles_n, 1);
    }
    return hipGetLastError();
}

// A many-tile GEMM whose tile count leaves the last round of workgroups poorly filled can be cheaper as two launches:
// columns [0, N1) (of every batch) as whole rounds of 256x256 tiles, the rest on its own with whatever tile suits it
// (gate|up at 1024 tokens: 688 tiles of 256x128 are 2.7 rounds and cost three; 256 tiles of 256x256 plus 176 of 256x128
// cost 12.2 + 7.0 instead of 3 x 7.0 in the units of the tile model below).  Returns N1, or 0 for one launch.
int gemm_nt_column_split(const GemmNT& g) {
    if (g.deferred || g.split_k > 1 || g.M <= 0 || g.N < 512 || g.batch <= 0) return 0;
    if ((g.K % BK) || (g.K2 % BK) || g.K <= 0) return 0;
    const long tm = (long)cdiv(g.M, 256) * g.batch;
    if (tm > 256 || 256 % tm) return 0;                       // a round of 256x256 tiles must be whole tile columns
    const long cols_round = 256 / tm * 256;
    if (tm * cdiv(g.N, 256) < 160) return 0;                  // few tiles: launch_gemm_nt has other choices there
    auto rounds = [](long t) { return (double)((t + 255) / 256); };
    auto one_launch = [&](long n) {                           // the many-tile model of launch_gemm_nt, per unit of K
        const double c256 = rounds(tm * cdiv(n, 256)) * 512.0 / 42.0, c128 = rounds(tm * cdiv(n, 128)) * 384.0 / 55.0;
        const double c192 = rounds(tm * cdiv(n, 192)) * 448.0 / 42.0;
        return c256 < c128 ? (c256 < c192 ? c256 : c192) : (c128 < c192 ? c128 : c192);
    };
    const double k_us = ((double)g.K + g.K2) * 2.0 / 1e3, second_launch_us = 6.0;
    double best = one_launch(g.N) * k_us;
    int n1 = 0;
    for (long c = cols_round; c + 128 <= g.N; c += cols_round) {
        const double cost = ((double)(c / cols_round) * 512.0 / 42.0 + one_launch(g.N - c)) * k_us + second_launch_us;
        if (cost < 0.97 * best) { best = cost; n1 = (int)c; }
    }
    return n1;
}

// the two launches of a column split: a = columns [0, N1), b = the rest; false (and nothing written) for one launch
bool gemm_nt_split_columns(const GemmNT& g, GemmNT* a, GemmNT* b) {
    const int n1 = gemm_nt_column_split(g);
    if (n1 <= 0) return false;
    *a = g;
    *b = g;
    a->N = n1;
    b->N = g.N - n1;
    b->B = g.B + (long)n1 * g.ldb;
    if (g.K2 > 0) b->B2 = g.B2 + (long)n1 * g.ldb2;
    b->C = (char*)g.C + (size_t)n1 * (g.c_f32 ? sizeof(float) : sizeof(bf16_t));
    if (g.R) b->R = g.R + n1;
    return true;
}

// The tile configurations the launcher can pick (every one is reachable from launch_gemm_nt; the kernel tests name the
// shape that lands on each).
enum NtConfig {
    NT_128x128,         // 128x128 tiles, BK 64, four-stage ring, interleaved loop: a few hundred tiles in all
    NT_256x128,         // 256x128 tiles, BK 64, three stages
    NT_256x128_SPLIT,   // the same with the contraction split 2..4 ways (partials reduced afterwards or by the consumer)
    NT_256x192,         // 256x192 tiles, BK 64, two stages: tile counts that 256x256 leaves a third of the CUs idle on
    NT_256x256,         // 256x256 tiles, BK 32, four stages
    NT_REG_128x128,     // register-staged fallbacks for contractions that are no multiple of 64 or operands beyond 1 Gi elements
    NT_REG_128x64,
    NT_SKINNY           // N <= 64 per batch or few tiles: 64x64 tiles, contraction split over up to 16 workgroups
};

// Measured on MI355X at M = 1024.  Every tile shape is limited by how fast a CU can pull operand bytes out of L2, so
// the largest tile that still gives every CU work wins.
static NtConfig choose_nt(const GemmNT& g, int* n_split) {
    *n_split = 1;
    const int nk = cdiv(g.K, BK) + cdiv(g.K2, BK);
    const long t128 = (long)cdiv(g.M, 128) * cdiv(g.N, 128) * g.batch;
    const long t64n = (long)cdiv(g.M, 128) * cdiv(g.N, 64) * g.batch;
    const bool dl_ok = (g.K % BK) == 0 && (g.K2 % BK) == 0 && g.K > 0 && g.N > 64 &&
                       (long)g.M * g.lda < (1L << 30) && (long)g.N * g.ldb < (1L << 30) &&
                       (long)g.M * g.lda2 < (1L << 30) && (long)g.N * g.ldb2 < (1L << 30);
    auto rounds = [](long t) { return (double)((t + 255) / 256); };
    if (dl_ok && t128 >= 128) {
        const long t256 = (long)cdiv(g.M, 256) * cdiv(g.N, 256) * g.batch;
        const long t256x128 = (long)cdiv(g.M, 256) * cdiv(g.N, 128) * g.batch;
        if (t256 < 160) {
            // Few 256x256 tiles: pick among 128x128 tiles, 256x128 tiles, and 256x128 tiles with the contraction split
            // 2..4 ways, by the operand bytes the busiest CU has to pull in (the loop is bound by that rate, about
            // 53 GB/s per CU, not by the matrix pipe): rounds of tiles x (BM + BN) x K x 2 bytes.  A split adds one
            // pass over its partials (written and read back at about 5 TB/s, plus a launch).  At M = 1024 this
            // picks the two-way split from K of about 10k on (measured: K 11008 -7 %, 12288 -13 %, 22016 -17 %,
            // 32000 -15 % against 128x128) and 128x128 below; at M = 2048 plain 256x128 tiles fill the chip.
            const double ktot = (double)g.K + g.K2, per_us = 53e3;
            double best = rounds(t128) * 256.0 * ktot * 2.0 / per_us;
            NtConfig cfg = NT_128x128;
            const double c28 = rounds(t256x128) * 384.0 * ktot * 2.0 / per_us;
            if (c28 < best) { best = c28; cfg = NT_256x128; }
            for (int sp = 2; sp <= 4; ++sp) {
                const size_t need = (size_t)sp * g.M * g.N * g.batch;
                if (!g.partial || need > g.partial_elems || (g.N & 3) || nk / sp < 8) continue;
                // the pass over the partials: a reduce launch that reads them and writes C, or, when the consumer
                // adds them up itself (g.deferred), only the extra bytes written here and read there
                const double pass = g.deferred ? (double)need * (g.partial_bf16 ? 2.0 : 4.0) / 5e6 : (double)need * 8.0 / 5e6 + 5.0;
                const double c = rounds(t256x128 * sp) * 384.0 * (ktot / sp) * 2.0 / per_us + pass;
                if (c < 0.97 * best) { best = c; cfg = NT_256x128_SPLIT; *n_split = sp; }
            }
            return cfg;
        }
        // Many tiles: the same byte count decides between 256x256 tiles (fewest bytes per flop, but only four
        // half-depth stages fit in LDS and the loop reaches about 42 GB/s per CU) and 256x128 tiles (55 GB/s per CU);
        // rounds of tiles x rows per tile / rate.  256x192 tiles when they land in fewer rounds (dx of the down
        // projection at 1024 tokens: 232 tiles, one round, against 172 of 256x256 that leave a third of the CUs
        // idle; measured -9 %).
        const double c256 = rounds(t256) * 512.0 / 42.0, c128 = rounds(t256x128) * 384.0 / 55.0;
        const long t256x192 = (long)cdiv(g.M, 256) * cdiv(g.N, 192) * g.batch;
        const double c192 = rounds(t256x192) * 448.0 / 42.0;
        if (c192 < c256 && c192 < c128) return NT_256x192;
        return c128 < c256 ? NT_256x128 : NT_256x256;
    }
    if (g.N > 64 && t128 >= 200) return NT_REG_128x128;
    if (g.N > 64 && t64n >= 200) return NT_REG_128x64;
    // few output tiles: 64x64 tiles, and split the contraction when scratch is available
    const long t64 = (long)cdiv(g.M, 64) * cdiv(g.N, 64) * g.batch;
    int split = g.split_k;
    if (split == 0) {
        split = 1;
        if (g.partial && t64 < 256) {
            split = (int)(512 / t64);
            if (split > nk / 4) split = nk / 4;   // at least four k-tiles per split
            if (split < 1) split = 1;
            while (split > 1 && (size_t)split * g.M * g.N * g.batch > g.partial_elems) --split;
        }
    }
    if (split > nk) split = nk > 0 ? nk : 1;
    if (g.N & 3) split = 1;   // the reduce kernel works on groups of four columns
    *n_split = split;
    return NT_SKINNY;
}

const char* gemm_nt_plan(const GemmNT& g, int* n_split) {
    int sp = 1;
    const NtConfig c = choose_nt(g, &sp);
    if (n_split) *n_split = sp;
    switch (c) {
        case NT_128x128: return "128x128";
        case NT_256x128: return "256x128";
        case NT_256x128_SPLIT: return "256x128-split";
        case NT_256x192: return "256x192";
        case NT_256x256: return "256x256";
        case NT_REG_128x128: return "reg-128x128";
        case NT_REG_128x64: return "reg-128x64";
        case NT_SKINNY: break;
    }
    const bool dl_small = (g.K % BK) == 0 && g.K2 == 0 && g.K > 0 && (long)g.M * g.lda < (1L << 30) &&
                          (long)g.N * g.ldb < (1L << 30);
    return dl_small ? (sp > 1 ? "64x64-split" : "64x64") : (sp > 1 ? "reg-64x64-split" : "reg-64x64");
}

hipError_t launch_gemm_nt(const GemmNT& g, hipStream_t s) {
    if (g.deferred) {
        *g.deferred = 0;
        if (g.batch != 1 || g.alpha != 1.f) return hipErrorInvalidValue;
    }
    if (g.M <= 0 || g.N <= 0 || g.batch <= 0) return hipSuccess;
    if ((g.K & 7) || (g.K2 & 7) || (g.lda & 7) || (g.ldb & 7) || (g.lda2 & 7) || (g.ldb2 & 7)) return hipErrorInvalidValue;
    if ((g.bA & 7) || (g.bB & 7) || (g.bA2 & 7) || (g.bB2 & 7)) return hipErrorInvalidValue;
    if (!g.c_f32 && g.R) return hipErrorInvalidValue;
    int split = 1;
    switch (choose_nt(g, &split)) {
        case NT_128x128: return run_nt_dl<128, 128, 2, 2, 4, 64, false, 1>(g, s);
        case NT_256x128: return run_nt_dl<256, 128, 4, 2, 3, 64, false, 1>(g, s);
        case NT_256x128_SPLIT: return run_nt_dl<256, 128, 4, 2, 3, 64, true, 1>(g, s, split);
        case NT_256x192: return run_nt_dl<256, 192, 4, 2, 2>(g, s);
        case NT_256x256: return run_nt_dl<256, 256, 4, 2, 4, 32, false, 1>(g, s);
        case NT_REG_128x128: return run_nt<128, 128, 2, 2>(g, 1, s);
        case NT_REG_128x64: return run_nt<128, 64, 2, 2>(g, 1, s);
        case NT_SKINNY: break;
    }
    if (split > 1 && (!g.partial || (size_t)split * g.M * g.N * g.batch > g.partial_elems)) return hipErrorInvalidValue;
    const bool dl_small = (g.K % BK) == 0 && g.K2 == 0 && g.K > 0 && (long)g.M * g.lda < (1L << 30) &&
                          (long)g.N * g.ldb < (1L << 30);
    if (dl_small) {
        if (split > 1) return run_nt_dl<64, 64, 2, 2, 4, 64, true>(g, s, split);
        return run_nt_dl<64, 64, 2, 2, 4>(g, s);
    }
    return run_nt<64, 64, 2, 2>(g, split, s);
}

// ======================================================================== TN
// One 64x64 output tile of P^T Q over the 64-token tiles [it0, it1).  The operand tiles stay in LDS as they lie in
// memory, [t][i] with the token index t as rows, and the matrix unit's operands (contraction over t) come out of the
// LDS transpose read of gfx950 (load_a_tr in tiles.h): no transposing stores, no bank conflicts.  Both operands use the
// same slot order, so the permutation that load_a_tr applies to the 16 contraction slots of a step cancels.  Two LDS
// buffers per operand (one barrier per token tile), the next tile's global loads issued a full tile ahead.  Thread
// (tp, ic) moves rows t = 2tp, 2tp+1 and the 8 columns i = 8ic..8ic+7.  Returns this wave's 32x32 accumulator.
__device__ __forceinline__ f32x16_t tn_tile(const bf16_t* P, long ldp, int Mo, const bf16_t* Q, long ldq, int No, int T,
                                            int i0, int j0, int it0, int it1) {
    constexpr int LD = LTR(64);
    __shared__ __align__(16) bf16_t sP[2][64 * LD];
    __shared__ __align__(16) bf16_t sQ[2][64 * LD];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wi = wave >> 1, wj = wave & 1;
    const int tp = tid >> 3, ic = tid & 7;
    const int tr_off = tr_lane_offset(lane, LD);
    f32x16_t acc = zero16();
    // byte offsets of this thread's two rows within a 64-token tile, computed once; a tile's address is wave-uniform,
    // and only a ragged last tile (or a ragged last column block) pays for per-element bounds checks
    const unsigned po = (unsigned)((2 * tp * ldp + i0 + ic * 8) * 2), qo = (unsigned)((2 * tp * ldq + j0 + ic * 8) * 2);
    const unsigned pstep = (unsigned)(ldp * 2), qstep = (unsigned)(ldq * 2);
    const bool pc = i0 + ic * 8 < Mo, qc = j0 + ic * 8 < No;
    const bool cols_full = i0 + 64 <= Mo && j0 + 64 <= No;
    typedef unsigned u32x4 __attribute__((ext_vector_type(4)));   // a plain vector value: stays in registers on every path
    u32x4 p0, p1, q0, q1;
    auto gload = [&](int it) {
        const char* pb = (const char*)(P + (long)it * 64 * ldp);
        const char* qb = (const char*)(Q + (long)it * 64 * ldq);
        if (cols_full && it * 64 + 64 <= T) {
            p0 = *(const u32x4*)(pb + po); p1 = *(const u32x4*)(pb + po + pstep);
            q0 = *(const u32x4*)(qb + qo); q1 = *(const u32x4*)(qb + qo + qstep);
        } else {
            const int t = it * 64 + 2 * tp;
            const u32x4 z = {0u, 0u, 0u, 0u};
            p0 = z; p1 = z; q0 = z; q1 = z;
            if (t < T && pc) p0 = *(const u32x4*)(pb + po);
            if (t + 1 < T && pc) p1 = *(const u32x4*)(pb + po + pstep);
            if (t < T && qc) q0 = *(const u32x4*)(qb + qo);
            if (t + 1 < T && qc) q1 = *(const u32x4*)(qb + qo + qstep);
        }
    };
    auto park = [&](int buf) {
        *(u32x4*)(sP[buf] + (2 * tp) * LD + ic * 8) = p0;
        *(u32x4*)(sP[buf] + (2 * tp + 1) * LD + ic * 8) = p1;
        *(u32x4*)(sQ[buf] + (2 * tp) * LD + ic * 8) = q0;
        *(u32x4*)(sQ[buf] + (2 * tp + 1) * LD + ic * 8) = q1;
    };
    if (it0 < it1) {
        gload(it0);
        park(0);
        if (it0 + 1 < it1) gload(it0 + 1);
    }
    __syncthreads();
    for (int it = it0; it < it1; ++it) {
        const int buf = (it - it0) & 1;
        // registers hold tile it+1: park it in the other buffer, then fetch tile it+2
        if (it + 1 < it1) {
            park(buf ^ 1);
            if (it + 2 < it1) gload(it + 2);
        }
#pragma unroll
        for (int ks = 0; ks < 4; ++ks) {
            const bf16x8_t a = load_a_tr(sP[buf], LD, tr_off, wi * 32, ks * 16);
            const bf16x8_t b = load_a_tr(sQ[buf], LD, tr_off, wj * 32, ks * 16);
            acc = mfma32(a, b, acc);
        }
        __syncthreads();
    }
    return acc;
}

__global__ __launch_bounds__(256) void gemm_tn_kernel(GemmTN p, int n_split) {
    // grid.y = Mo tiles x n_split: each split covers a contiguous token range; with n_split > 1 the splits are
    // stored as fp32 partials and added by tn_reduce_kernel.
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int wi = wave >> 1, wj = wave & 1, l32 = lane & 31, g = lane >> 5;
    const int tiles_i = (p.Mo + 63) / 64;
    const int ti = blockIdx.y % tiles_i, split = blockIdx.y / tiles_i;
    const int i0 = ti * 64, j0 = blockIdx.x * 64, z = blockIdx.z;
    const int nt_all = (p.T + 63) / 64;
    const int it0 = (int)((long)nt_all * split / n_split), it1 = (int)((long)nt_all * (split + 1) / n_split);
    const f32x16_t acc = tn_tile(p.P + (long)z * p.bP, p.ldp, p.Mo, p.Q + (long)z * p.bQ, p.ldq, p.No, p.T, i0, j0, it0, it1);
    const int col = j0 + wj * 32 + l32;
    if (n_split == 1) {
        if (col < p.No) {
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int row = i0 + wi * 32 + 8 * (v >> 2) + 4 * g + (v & 3);
                if (row < p.Mo) p.C[(long)z * p.bC + (long)row * p.ldc + col] = p.alpha * acc[v];
            }
        }
        return;
    }
    const long mn = (long)p.Mo * p.No;
    float* part = p.partial + ((long)z * n_split + split) * mn;
    if (col < p.No) {
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            const int row = i0 + wi * 32 + 8 * (v >> 2) + 4 * g + (v & 3);
            if (row < p.Mo) part[(long)row * p.No + col] = acc[v];
        }
    }
}

// Several independent P^T Q products over the same T tokens in one launch: workgroup b takes output tile
// b - tile0 of the problem whose tile range holds b.  Every tile runs over all tokens, so nothing is split or reduced.
__global__ __launch_bounds__(256) void gemm_tn_grouped_kernel(GemmTNGroup grp) {
    const int b = blockIdx.x;
    int k = 0;
    while (k + 1 < grp.n && b >= grp.p[k + 1].tile0) ++k;
    const TnProblem& q = grp.p[k];
    const int t = b - q.tile0, tiles_j = (q.No + 63) / 64;
    const int i0 = (t / tiles_j) * 64, j0 = (t % tiles_j) * 64;
    const f32x16_t acc = tn_tile(q.P, q.ldp, q.Mo, q.Q, q.ldq, q.No, grp.T, i0, j0, 0, (grp.T + 63) / 64);
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int wi = wave >> 1, wj = wave & 1, l32 = lane & 31, g = lane >> 5;
    const int col = j0 + wj * 32 + l32;
    bool bad = false;
    if (col < q.No) {
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            const int row = i0 + wi * 32 + 8 * (v >> 2) + 4 * g + (v & 3);
            if (row < q.Mo) {
                q.C[(long)row * q.ldc + col] = acc[v];
                bad |= !isfinite(acc[v]);
            }
        }
    }
    // a gradient that is not finite must not reach the optimizer: raise bit 1 of the update's flag (one vector atomic
    // per wave that saw one; never in a healthy update)
    if (grp.flag && __builtin_amdgcn_ballot_w64(bad) != 0 && lane == 0) atomicOr(grp.flag, 2);
}

// adds the token splits of gemm_tn_kernel in index order
__global__ __launch_bounds__(256) void tn_reduce_kernel(GemmTN p, int n_split) {
    const long mn = (long)p.Mo * p.No;
    const long idx = (long)blockIdx.x * blockDim.x + threadIdx.x;
    if (idx >= mn * p.batch) return;
    const int z = (int)(idx / mn);
    const long r = idx % mn;
    float sum = 0.f;
    for (int sp = 0; sp < n_split; ++sp) sum += p.partial[((long)z * n_split + sp) * mn + r];
    p.C[(long)z * p.bC + (r / p.No) * p.ldc + (r % p.No)] = p.alpha * sum;
}

hipError_t launch_gemm_tn(const GemmTN& g, hipStream_t s) {
    if (g.Mo <= 0 || g.No <= 0 || g.batch <= 0) return hipSuccess;
    if ((g.ldp & 7) || (g.ldq & 7) || (g.Mo & 7) || (g.No & 7) || (g.bP & 7) || (g.bQ & 7)) return hipErrorInvalidValue;
    const long tiles = (long)cdiv(g.No, 64) * cdiv(g.Mo, 64) * g.batch;
    int split = 1;
    if (g.partial && tiles < 512) {
        split = (int)(768 / tiles);
        const int max_split = cdiv(g.T, 64) / 2;   // at least two token tiles per split
        if (split > max_split) split = max_split;
        if (split > 8) split = 8;
        if (split < 1) split = 1;
        while (split > 1 && (size_t)split * g.Mo * g.No * g.batch > g.partial_elems) --split;
    }
    dim3 grid(cdiv(g.No, 64), cdiv(g.Mo, 64) * split, g.batch);
    gemm_tn_kernel<<<grid, 256, 0, s>>>(g, split);
    if (split > 1) {
        const long n = (long)g.Mo * g.No * g.batch;
        tn_reduce_kernel<<<cdiv(n, 256), 256, 0, s>>>(g, split);
    }
    return hipGetLastError();
}

hipError_t launch_gemm_tn_grouped(GemmTNGroup& g, hipStream_t s) {
    if (g.n <= 0 || g.T <= 0) return hipSuccess;
    if (g.n > TN_GROUP_MAX) return hipErrorInvalidValue;
    int tiles = 0;
    for (int k = 0; k < g.n; ++k) {
        TnProblem& q = g.p[k];
        if (q.Mo <= 0 || q.No <= 0 || (q.ldp & 7) || (q.ldq & 7) || (q.Mo & 7) || (q.No & 7)) return hipErrorInvalidValue;
        q.tile0 = tiles;
        tiles += cdiv(q.Mo, 64) * cdiv(q.No, 64);
    }
    gemm_tn_grouped_kernel<<<tiles, 256, 0, s>>>(g);
    return hipGetLastError();
}
