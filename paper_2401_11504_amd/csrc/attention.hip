// Causal self-attention within one chunk, forward and backward, on bf16 MFMA (gfx950).
//
// All three kernels work on the TRANSPOSED score tile where that keeps the softmax row in one lane:
//   forward / dQ :  S^T[u][t] = K[u] . Q[t]   -> a lane owns one query t (and its partner lane t too),
//                   so the running max, the row sum, lse[t] and delta[t] are per-lane scalars;
//                   O^T[d][t] += V^T[d][u] P^T[u][t]   and   dQ^T[d][t] += K^T[d][u] dS^T[u][t]
//                   reuse the score fragment directly as the B operand (see tiles.h); their A operands V^T, K^T (and
//                   dO^T, Q^T below) are never built: the tiles stay as they lie in memory and are read through the
//                   LDS transpose read of gfx950 (load_a_tr in tiles.h), which costs no bank conflicts and no
//                   transposing stores.
//   dK / dV      :  S[t][u] = Q[t] . K[u]     -> a lane owns one key u;
//                   dV^T[d][u] += dO^T[d][t] P[t][u],  dK^T[d][u] += Q^T[d][t] dS[t][u].
// P is never stored: the backward kernels rebuild it from the saved log-sum-exp.
// The two backward kernels write disjoint outputs, so no atomics are needed and results are
// bit-reproducible.
#include <type_traits>

#include "kernels.h"
#include "tiles.h"

#define NEG_BIG (-1.0e30f)

template <int DH>
struct AttnCfg {
    static constexpr int LSK = DH + 8;  // row stride of a [row][d] tile
    static constexpr int NKS = DH / 16; // MFMA steps over d
    static constexpr int ND = DH / 32;  // 32-wide d tiles
};

// Byte offsets, within a [64 rows][DH] tile of a matrix with row stride ld, of the 16-byte chunks this thread fetches
// (NT = threads that share the tile).  Computed once per kernel: the loop then adds them to a wave-uniform tile
// address, which costs no vector arithmetic per load.
template <int DH, int NT>
__device__ __forceinline__ void tile_chunk_offsets(long ld, unsigned* off, int tid = threadIdx.x) {
    constexpr int CH = DH / 8;  // chunks per row
#pragma unroll
    for (int i = 0; i < 8 * DH / NT; ++i) {
        const int c = tid + NT * i, row = c / CH, ch = c % CH;
        off[i] = (unsigned)((row * ld + ch * 8) * 2);
    }
}
// load the tile of rows r0 .. r0 + 63 (zero beyond T) into registers; r0 is wave-uniform, so only a ragged last tile
// pays for per-row checks
template <int DH, int NT>
__device__ __forceinline__ void load_tile_regs(const bf16_t* __restrict__ base, long ld, int r0, int T, const unsigned* off,
                                               uint4* regs, int tid = threadIdx.x) {
    constexpr int CH = DH / 8;
    const char* p = (const char*)(base + (long)r0 * ld);
    if (r0 + 64 <= T) {
#pragma unroll
        for (int i = 0; i < 8 * DH / NT; ++i) regs[i] = *(const uint4*)(p + off[i]);
    } else {
#pragma unroll
        for (int i = 0; i < 8 * DH / NT; ++i) {
            const int row = (tid + NT * i) / CH;
            regs[i] = (r0 + row < T) ? *(const uint4*)(p + off[i]) : make_uint4(0, 0, 0, 0);
        }
    }
}
template <int DH, int NT>
__device__ __forceinline__ void store_tile_normal(bf16_t* tile, const uint4* regs, int tid = threadIdx.x) {
    constexpr int CH = DH / 8;
#pragma unroll
    for (int i = 0; i < 8 * DH / NT; ++i) {
        const int c = tid + NT * i, row = c / CH, ch = c % CH;
        *(uint4*)(tile + row * AttnCfg<DH>::LSK + ch * 8) = regs[i];
    }
}
// the same with row stride LD (tiles that are read with the LDS transpose read, see load_a_tr)
template <int DH, int NT, int LD>
__device__ __forceinline__ void store_tile_ld(bf16_t* tile, const uint4* regs, int tid = threadIdx.x) {
    constexpr int CH = DH / 8;
#pragma unroll
    for (int i = 0; i < 8 * DH / NT; ++i) {
        const int c = tid + NT * i, row = c / CH, ch = c % CH;
        *(uint4*)(tile + row * LD + ch * 8) = regs[i];
    }
}
__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

// write a D fragment set holding X^T[d][row] (lane = row) as bf16 rows of X
template <int DH>
__device__ __forceinline__ void write_rows_from_dT(bf16_t* __restrict__ dst, const f32x16_t* acc, float mul, int g) {
#pragma unroll
    for (int dt = 0; dt < DH / 32; ++dt)
#pragma unroll
        for (int vq = 0; vq < 4; ++vq) {
            uint2 w;
            w.x = pack_bf16x2(acc[dt][4 * vq] * mul, acc[dt][4 * vq + 1] * mul);
            w.y = pack_bf16x2(acc[dt][4 * vq + 2] * mul, acc[dt][4 * vq + 3] * mul);
            *(uint2*)(dst + dt * 32 + 8 * vq + 4 * g) = w;
        }
}

// ======================================================================== forward
// KG key groups of NW waves each; a wave owns 32 queries, and the key tiles (64 keys) of the causal range are dealt
// out to the key groups in turn (group kg takes tiles kg, kg + KG, ..).  Every group keeps its own running max, row
// sum and output accumulator over its tiles and the groups are merged once at the end through LDS (the usual
// two-state softmax merge).  With KG = 2 a SIMD runs two waves, so one wave's softmax arithmetic overlaps the other's
// MFMAs; at T = 1024 with 32 heads there are otherwise only as many 32-query waves as the chip has SIMDs.
// K and V tiles are fetched one tile ahead into registers (the loads fly during the MFMAs of the current tile) and
// parked in the group's LDS buffers between two barriers.
template <int DH, int NW, int KG>
__global__ __launch_bounds__(NW * 64 * KG) void attn_fwd_kernel(const bf16_t* __restrict__ q, const bf16_t* __restrict__ k,
                                                                const bf16_t* __restrict__ v, long ldq, int T,
                                                                bf16_t* __restrict__ o, long ldo, float* __restrict__ lse,
                                                                float scale_log2e) {
    using C = AttnCfg<DH>;
    constexpr int NT = NW * 64, QB = NW * 32;
    constexpr int LDV = LTR(DH);
    constexpr int GROUP_ELEMS = 64 * C::LSK + 64 * LDV;          // bf16 elements of one group's K and V tiles
    extern __shared__ __align__(16) unsigned char smem_raw[];
    const int kg = __builtin_amdgcn_readfirstlane(threadIdx.x / NT);
    const int tid = threadIdx.x % NT, lane = tid & 63, wave = tid >> 6, l32 = lane & 31, g = lane >> 5;
    bf16_t* sK = (bf16_t*)smem_raw + kg * GROUP_ELEMS;
    bf16_t* sV = sK + 64 * C::LSK;
    const int tr_off = tr_lane_offset(lane, LDV);
    // Heaviest (latest) query blocks first; the second half of the heads takes the mirrored block, so that two
    // workgroups placed on one CU by round-robin dispatch (ids i and i + n/2 in dispatch order, x fastest) carry the
    // same total number of key tiles whichever CU they land on.
    // With more workgroups than CUs (several rounds) the order of dispatch decides the tail instead: every head's
    // heaviest block first, then every head's second heaviest, and so on (longest job first).
    const bool mirror = 2 * blockIdx.y >= gridDim.y + 1;
    int qb = mirror ? (int)blockIdx.x : (int)(gridDim.x - 1 - blockIdx.x);
    int head = blockIdx.y;
    if (gridDim.x * gridDim.y > 256) {
        const int idx = blockIdx.y * gridDim.x + blockIdx.x;   // position in dispatch order (x fastest)
        qb = (int)gridDim.x - 1 - idx / (int)gridDim.y;
        head = idx % (int)gridDim.y;
    }
    const int q0 = qb * QB, tq0 = q0 + 32 * wave, t_abs = tq0 + l32;
    const bf16_t* qh = q + (long)head * DH;
    const bf16_t* kh = k + (long)head * DH;
    const bf16_t* vh = v + (long)head * DH;

    bf16x8_t qf[C::NKS];
#pragma unroll
    for (int ks = 0; ks < C::NKS; ++ks) {
        uint4 r = (t_abs < T) ? *(const uint4*)(qh + (long)t_abs * ldq + ks * 16 + g * 8) : make_uint4(0, 0, 0, 0);
        qf[ks] = *(bf16x8_t*)&r;
    }
    f32x16_t oacc[C::ND];
#pragma unroll
    for (int dt = 0; dt < C::ND; ++dt) oacc[dt] = zero16();
    float m = NEG_BIG, lpart = 0.f;

    const int kend = min(q0 + QB, T);
    const int n_tiles = (kend + 63) / 64;
    const int n_iter = (n_tiles + KG - 1) / KG;   // a group's surplus tile lies wholly in the future and is skipped
    uint4 rk[8 * DH / NT], rv[8 * DH / NT];
    unsigned toff[8 * DH / NT];
    tile_chunk_offsets<DH, NT>(ldq, toff, tid);
    load_tile_regs<DH, NT>(kh, ldq, kg * 64, T, toff, rk, tid);
    load_tile_regs<DH, NT>(vh, ldq, kg * 64, T, toff, rv, tid);
    for (int it = 0; it < n_iter; ++it) {
        const int u0 = (it * KG + kg) * 64;
        __syncthreads();
        store_tile_normal<DH, NT>(sK, rk, tid);
        store_tile_ld<DH, NT, LDV>(sV, rv, tid);                 // V as it lies in memory: P V reads it transposed
        __syncthreads();
        if (it + 1 < n_iter) {
            load_tile_regs<DH, NT>(kh, ldq, u0 + 64 * KG, T, toff, rk, tid);
            load_tile_regs<DH, NT>(vh, ldq, u0 + 64 * KG, T, toff, rv, tid);
        }
        if (u0 > tq0 + 31) continue;  // wave-uniform: every key of this tile is in the future
        // both 32-key halves of the tile at once: two independent MFMA chains, one softmax update
        f32x16_t s0 = zero16(), s1 = zero16();
#pragma unroll
        for (int ks = 0; ks < C::NKS; ++ks) {
            const bf16x8_t a0 = *(const bf16x8_t*)(sK + l32 * C::LSK + ks * 16 + g * 8);
            const bf16x8_t a1 = *(const bf16x8_t*)(sK + (32 + l32) * C::LSK + ks * 16 + g * 8);
            s0 = mfma32(a0, qf[ks], s0);
            s1 = mfma32(a1, qf[ks], s1);
        }
        // the running max m is kept in units of the raw scores (the scale is positive, so it commutes with max) and
        // the scale is folded into the exponent's multiply-add: one instruction per score less
        float x[32];
        float mloc = NEG_BIG;
        if (u0 + 63 > tq0) {  // the tile touches the diagonal: causal mask
#pragma unroll
            for (int vv = 0; vv < 16; ++vv) {
                const int u = u0 + 8 * (vv >> 2) + 4 * g + (vv & 3);
                x[vv] = (u > t_abs) ? NEG_BIG : s0[vv];
                x[16 + vv] = (u + 32 > t_abs) ? NEG_BIG : s1[vv];
            }
        } else {
#pragma unroll
            for (int vv = 0; vv < 16; ++vv) {
                x[vv] = s0[vv];
                x[16 + vv] = s1[vv];
            }
        }
#pragma unroll
        for (int vv = 0; vv < 32; ++vv) mloc = fmaxf(mloc, x[vv]);
        mloc = fmaxf(mloc, __shfl_xor(mloc, 32, 64));
        const float m_new = fmaxf(m, mloc);
        const float alpha = fast_exp2((m - m_new) * scale_log2e);
        const float mb = m_new * scale_log2e;
        float psum = 0.f;
#pragma unroll
        for (int vv = 0; vv < 32; ++vv) {
            x[vv] = fast_exp2(fmaf(x[vv], scale_log2e, -mb));
            psum += x[vv];
        }
        lpart = lpart * alpha + psum;
        m = m_new;
        if (__builtin_amdgcn_ballot_w64(alpha != 1.f)) {  // skip the rescale once the running max has settled
#pragma unroll
            for (int dt = 0; dt < C::ND; ++dt)
#pragma unroll
                for (int vv = 0; vv < 16; ++vv) oacc[dt][vv] *= alpha;
        }
#pragma unroll
        for (int us = 0; us < 2; ++us)
#pragma unroll
            for (int h = 0; h < 2; ++h) {
                const bf16x8_t b = pack_b_from_d(x + 16 * us, h);
#pragma unroll
                for (int dt = 0; dt < C::ND; ++dt) {
                    const bf16x8_t a = load_a_tr(sV, LDV, tr_off, dt * 32, us * 32 + 16 * h);
                    oacc[dt] = mfma32(a, b, oacc[dt]);
                }
            }
    }
    if constexpr (KG > 1) {
        // merge the key groups into group 0: values of thread `tid` are kept NT apart (no bank conflicts)
        static_assert(KG == 2, "two key groups");
        float* mg = (float*)smem_raw;
        __syncthreads();                            // every group is done with its K / V tiles
        if (kg == 1) {
#pragma unroll
            for (int dt = 0; dt < C::ND; ++dt)
#pragma unroll
                for (int vv = 0; vv < 16; ++vv) mg[(dt * 16 + vv) * NT + tid] = oacc[dt][vv];
            mg[(C::ND * 16) * NT + tid] = m;
            mg[(C::ND * 16 + 1) * NT + tid] = lpart;
        }
        __syncthreads();
        if (kg == 1) return;
        const float m1 = mg[(C::ND * 16) * NT + tid], l1 = mg[(C::ND * 16 + 1) * NT + tid];
        const float mt = fmaxf(m, m1);
        const float a0 = fast_exp2((m - mt) * scale_log2e), a1 = fast_exp2((m1 - mt) * scale_log2e);
#pragma unroll
        for (int dt = 0; dt < C::ND; ++dt)
#pragma unroll
            for (int vv = 0; vv < 16; ++vv) oacc[dt][vv] = oacc[dt][vv] * a0 + mg[(dt * 16 + vv) * NT + tid] * a1;
        lpart = lpart * a0 + l1 * a1;
        m = mt;
    }
    const float ltot = lpart + __shfl_xor(lpart, 32, 64);
    if (t_abs < T) {
        write_rows_from_dT<DH>(o + (long)t_abs * ldo + (long)head * DH, oacc, 1.f / ltot, g);
        if (g == 0) lse[(long)head * T + t_abs] = (m * scale_log2e + log2f(ltot)) * 0.6931471805599453f;
    }
}

// Rotate the (d, d + DH/2) pairs of a transposed fragment set X^T[d][row] (lane = row at position `pos`) by the RoPE
// angle of that position, sign = -1 for the inverse rotation (the adjoint of the forward rotation): both members of a
// pair sit in the same lane and register index of fragments dt and dt + ND/2, so nothing crosses lanes.
template <int DH>
__device__ __forceinline__ void rope_rotate_dT(f32x16_t* acc, const float2* __restrict__ table, int pos, float sign, int g) {
    constexpr int ND = DH / 32, HALF = DH / 2;
    const float2* row = table + (long)pos * HALF;
#pragma unroll
    for (int dt = 0; dt < ND / 2; ++dt)
#pragma unroll
        for (int vv = 0; vv < 16; ++vv) {
            const int i = dt * 32 + 8 * (vv >> 2) + 4 * g + (vv & 3);
            const float2 cs = row[i];
            const float a = acc[dt][vv], b = acc[dt + ND / 2][vv], sn = cs.y * sign;
            acc[dt][vv] = a * cs.x - b * sn;
            acc[dt + ND / 2][vv] = b * cs.x + a * sn;
        }
}

// ======================================================================== backward: dQ
// Same shape as the forward kernel: KG key groups share the causal range tile by tile and their dQ partial sums are
// added through LDS at the end.  delta[t] = dO[t] . O[t] is read from memory (attn_delta_kernel wrote it for the dK/dV
// parts of the same launch); with a RoPE table the gradient is rotated back before it is stored, so no separate pass
// over dq is needed.
template <int DH, int NW, int KG>
__device__ __forceinline__ void attn_dq_block(
    const bf16_t* __restrict__ q, const bf16_t* __restrict__ k, const bf16_t* __restrict__ v,
    const bf16_t* __restrict__ d_o, const float* __restrict__ lse, const float* __restrict__ delta, long ldq, long ldo, int T,
    bf16_t* __restrict__ dq, float scale, const float2* __restrict__ rope, int qb, int head, unsigned char* smem_raw) {
    using C = AttnCfg<DH>;
    constexpr int NT = NW * 64, QB = NW * 32;
    constexpr int LDT = LTR(DH);
    constexpr int GROUP_ELEMS = 2 * 64 * C::LSK + 64 * LDT;
    const int kg = __builtin_amdgcn_readfirstlane(threadIdx.x / NT);
    const int tid = threadIdx.x % NT, lane = tid & 63, wave = tid >> 6, l32 = lane & 31, g = lane >> 5;
    bf16_t* sK = (bf16_t*)smem_raw + kg * GROUP_ELEMS;
    bf16_t* sV = sK + 64 * C::LSK;
    bf16_t* sK2 = sV + 64 * C::LSK;         // K once more, with the row stride of the LDS transpose read (dS K)
    const int tr_off = tr_lane_offset(lane, LDT);
    const int q0 = qb * QB, tq0 = q0 + 32 * wave, t_abs = tq0 + l32;
    const float scale_log2e = scale * 1.4426950408889634f;
    const bf16_t* qh = q + (long)head * DH;
    const bf16_t* kh = k + (long)head * DH;
    const bf16_t* vh = v + (long)head * DH;
    const bf16_t* doh = d_o + (long)head * DH;

    bf16x8_t qf[C::NKS], dof[C::NKS];
#pragma unroll
    for (int ks = 0; ks < C::NKS; ++ks) {
        uint4 r = (t_abs < T) ? *(const uint4*)(qh + (long)t_abs * ldq + ks * 16 + g * 8) : make_uint4(0, 0, 0, 0);
        qf[ks] = *(bf16x8_t*)&r;
        uint4 r2 = (t_abs < T) ? *(const uint4*)(doh + (long)t_abs * ldo + ks * 16 + g * 8) : make_uint4(0, 0, 0, 0);
        dof[ks] = *(bf16x8_t*)&r2;
    }
    const float dlt = (t_abs < T) ? delta[(long)head * T + t_abs] : 0.f;
    const float lse2 = (t_abs < T) ? lse[(long)head * T + t_abs] * 1.4426950408889634f : 1.0e30f;
    f32x16_t acc[C::ND];
#pragma unroll
    for (int dt = 0; dt < C::ND; ++dt) acc[dt] = zero16();

    const int kend = min(q0 + QB, T);
    const int n_tiles = (kend + 63) / 64;
    const int n_iter = (n_tiles + KG - 1) / KG;
    uint4 rk[8 * DH / NT], rv[8 * DH / NT];
    unsigned toff[8 * DH / NT];
    tile_chunk_offsets<DH, NT>(ldq, toff, tid);
    load_tile_regs<DH, NT>(kh, ldq, kg * 64, T, toff, rk, tid);
    load_tile_regs<DH, NT>(vh, ldq, kg * 64, T, toff, rv, tid);
    for (int it = 0; it < n_iter; ++it) {
        const int u0 = (it * KG + kg) * 64;
        __syncthreads();
        store_tile_normal<DH, NT>(sK, rk, tid);
        store_tile_ld<DH, NT, LDT>(sK2, rk, tid);
        store_tile_normal<DH, NT>(sV, rv, tid);
        __syncthreads();
        if (it + 1 < n_iter) {
            load_tile_regs<DH, NT>(kh, ldq, u0 + 64 * KG, T, toff, rk, tid);
            load_tile_regs<DH, NT>(vh, ldq, u0 + 64 * KG, T, toff, rv, tid);
        }
        if (u0 > tq0 + 31) continue;
        f32x16_t s0 = zero16(), s1 = zero16(), dp0 = zero16(), dp1 = zero16();
#pragma unroll
        for (int ks = 0; ks < C::NKS; ++ks) {
            const int o0 = l32 * C::LSK + ks * 16 + g * 8, o1 = o0 + 32 * C::LSK;
            s0 = mfma32(*(const bf16x8_t*)(sK + o0), qf[ks], s0);
            s1 = mfma32(*(const bf16x8_t*)(sK + o1), qf[ks], s1);
            dp0 = mfma32(*(const bf16x8_t*)(sV + o0), dof[ks], dp0);
            dp1 = mfma32(*(const bf16x8_t*)(sV + o1), dof[ks], dp1);
        }
        float ds[32];
        // only a tile on the diagonal needs the causal mask (wave-uniform); the others skip its compares
        auto probs = [&](auto masked) {
#pragma unroll
            for (int vv = 0; vv < 16; ++vv) {
                const int u = u0 + 8 * (vv >> 2) + 4 * g + (vv & 3);
                const float pe0 = fast_exp2(s0[vv] * scale_log2e - lse2);
                const float pe1 = fast_exp2(s1[vv] * scale_log2e - lse2);
                const float p0 = (decltype(masked)::value && u > t_abs) ? 0.f : pe0;
                const float p1 = (decltype(masked)::value && u + 32 > t_abs) ? 0.f : pe1;
                ds[vv] = p0 * (dp0[vv] - dlt);
                ds[16 + vv] = p1 * (dp1[vv] - dlt);
            }
        };
        if (u0 + 63 > tq0) probs(std::true_type{}); else probs(std::false_type{});
#pragma unroll
        for (int us = 0; us < 2; ++us)
#pragma unroll
            for (int h = 0; h < 2; ++h) {
                const bf16x8_t b = pack_b_from_d(ds + 16 * us, h);
#pragma unroll
                for (int dt = 0; dt < C::ND; ++dt) {
                    const bf16x8_t a = load_a_tr(sK2, LDT, tr_off, dt * 32, us * 32 + 16 * h);
                    acc[dt] = mfma32(a, b, acc[dt]);
                }
            }
    }
    if constexpr (KG > 1) {
        static_assert(KG == 2, "two key groups");
        float* mg = (float*)smem_raw;
        __syncthreads();
        if (kg == 1) {
#pragma unroll
            for (int dt = 0; dt < C::ND; ++dt)
#pragma unroll
                for (int vv = 0; vv < 16; ++vv) mg[(dt * 16 + vv) * NT + tid] = acc[dt][vv];
        }
        __syncthreads();
        if (kg == 1) return;
#pragma unroll
        for (int dt = 0; dt < C::ND; ++dt)
#pragma unroll
            for (int vv = 0; vv < 16; ++vv) acc[dt][vv] += mg[(dt * 16 + vv) * NT + tid];
    }
    if (t_abs < T) {
        if (rope) rope_rotate_dT<DH>(acc, rope, t_abs, -1.f, g);
        write_rows_from_dT<DH>(dq + (long)t_abs * ldq + (long)head * DH, acc, scale, g);
    }
}

// ======================================================================== backward: dK, dV
template <int DH, int NW>
__device__ __forceinline__ void attn_dkv_block(const bf16_t* __restrict__ q, const bf16_t* __restrict__ k,
                                               const bf16_t* __restrict__ v, const bf16_t* __restrict__ d_o,
                                               const float* __restrict__ lse, const float* __restrict__ delta, long ldq,
                                               long ldo, int T, bf16_t* __restrict__ dk, bf16_t* __restrict__ dv,
                                               float scale, const float2* __restrict__ rope, int kb, int head,
                                               unsigned char* smem) {
    using C = AttnCfg<DH>;
    constexpr int NT = NW * 64, KB = NW * 32;
    constexpr int LDT = LTR(DH);
    bf16_t* sQ = (bf16_t*)smem;             // [64][LSK]
    bf16_t* sdO = sQ + 64 * C::LSK;         // [64][LSK]
    bf16_t* sQ2 = sdO + 64 * C::LSK;        // [64][LDT]: Q and dO once more, with the row stride of the LDS transpose
    bf16_t* sdO2 = sQ2 + 64 * LDT;          // [64][LDT]  read (dS^T Q and P^T dO take them with the token index as contraction)
    float* sLse = (float*)(sdO2 + 64 * LDT); // [64]
    float* sDelta = sLse + 64;              // [64]
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, l32 = lane & 31, g = lane >> 5;
    const int tr_off = tr_lane_offset(lane, LDT);
    const int u0 = kb * KB, uw0 = u0 + 32 * wave, u_abs = uw0 + l32;
    const float scale_log2e = scale * 1.4426950408889634f;
    const bf16_t* qh = q + (long)head * DH;
    const bf16_t* kh = k + (long)head * DH;
    const bf16_t* vh = v + (long)head * DH;
    const bf16_t* doh = d_o + (long)head * DH;

    bf16x8_t kf[C::NKS], vf[C::NKS];
#pragma unroll
    for (int ks = 0; ks < C::NKS; ++ks) {
        uint4 r = (u_abs < T) ? *(const uint4*)(kh + (long)u_abs * ldq + ks * 16 + g * 8) : make_uint4(0, 0, 0, 0);
        kf[ks] = *(bf16x8_t*)&r;
        uint4 r2 = (u_abs < T) ? *(const uint4*)(vh + (long)u_abs * ldq + ks * 16 + g * 8) : make_uint4(0, 0, 0, 0);
        vf[ks] = *(bf16x8_t*)&r2;
    }
    f32x16_t dkacc[C::ND], dvacc[C::ND];
#pragma unroll
    for (int dt = 0; dt < C::ND; ++dt) { dkacc[dt] = zero16(); dvacc[dt] = zero16(); }

    const int n_tiles = (T + 63) / 64;
    const int tile0 = u0 / 64;
    uint4 rq[8 * DH / NT], rdo[8 * DH / NT];
    unsigned qoff[8 * DH / NT], dooff[8 * DH / NT];
    tile_chunk_offsets<DH, NT>(ldq, qoff);
    tile_chunk_offsets<DH, NT>(ldo, dooff);
    float lse_v = 0.f, dl_v = 0.f;
    auto fetch = [&](int tile) {
        const int t0 = tile * 64;
        load_tile_regs<DH, NT>(qh, ldq, t0, T, qoff, rq);
        load_tile_regs<DH, NT>(doh, ldo, t0, T, dooff, rdo);
        if (tid < 64) {
            const int t = t0 + tid;
            lse_v = (t < T) ? lse[(long)head * T + t] * 1.4426950408889634f : 1.0e30f;
            dl_v = (t < T) ? delta[(long)head * T + t] : 0.f;
        }
    };
    if (tile0 < n_tiles) fetch(tile0);
    for (int tile = tile0; tile < n_tiles; ++tile) {
        const int t0 = tile * 64;
        __syncthreads();
        store_tile_normal<DH, NT>(sQ, rq);
        store_tile_normal<DH, NT>(sdO, rdo);
        store_tile_ld<DH, NT, LDT>(sQ2, rq);
        store_tile_ld<DH, NT, LDT>(sdO2, rdo);
        if (tid < 64) { sLse[tid] = lse_v; sDelta[tid] = dl_v; }
        __syncthreads();
        if (tile + 1 < n_tiles) fetch(tile + 1);
#pragma unroll
        for (int ts = 0; ts < 2; ++ts) {
            const int tsub0 = t0 + ts * 32;
            if (tsub0 + 31 < uw0) continue;  // wave-uniform: every query of this sub-tile precedes every key
            f32x16_t sacc = zero16(), dpacc = zero16();
#pragma unroll
            for (int ks = 0; ks < C::NKS; ++ks) {
                bf16x8_t a = *(const bf16x8_t*)(sQ + (ts * 32 + l32) * C::LSK + ks * 16 + g * 8);
                sacc = mfma32(a, kf[ks], sacc);
                bf16x8_t b = *(const bf16x8_t*)(sdO + (ts * 32 + l32) * C::LSK + ks * 16 + g * 8);
                dpacc = mfma32(b, vf[ks], dpacc);
            }
            float p[16], ds[16];
            // only a sub-tile on the diagonal needs the causal mask (wave-uniform); the others skip its compares
            auto probs = [&](auto masked) {
#pragma unroll
                for (int vq = 0; vq < 4; ++vq) {
                    const int tl = ts * 32 + 8 * vq + 4 * g;
                    const float4 l4 = *(const float4*)(sLse + tl);
                    const float4 d4 = *(const float4*)(sDelta + tl);
                    const float ll[4] = {l4.x, l4.y, l4.z, l4.w}, dd[4] = {d4.x, d4.y, d4.z, d4.w};
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        const int vv = 4 * vq + e;
                        const int t = t0 + tl + e;
                        const float pe = fast_exp2(sacc[vv] * scale_log2e - ll[e]);
                        const float pv = (decltype(masked)::value && u_abs > t) ? 0.f : pe;
                        p[vv] = pv;
                        ds[vv] = pv * (dpacc[vv] - dd[e]);
                    }
                }
            };
            if (tsub0 < uw0 + 32) probs(std::true_type{}); else probs(std::false_type{});
#pragma unroll
            for (int h = 0; h < 2; ++h) {
                const bf16x8_t bp = pack_b_from_d(p, h);
                const bf16x8_t bs = pack_b_from_d(ds, h);
#pragma unroll
                for (int dt = 0; dt < C::ND; ++dt) {
                    const bf16x8_t a1 = load_a_tr(sdO2, LDT, tr_off, dt * 32, ts * 32 + 16 * h);
                    dvacc[dt] = mfma32(a1, bp, dvacc[dt]);
                    const bf16x8_t a2 = load_a_tr(sQ2, LDT, tr_off, dt * 32, ts * 32 + 16 * h);
                    dkacc[dt] = mfma32(a2, bs, dkacc[dt]);
                }
            }
        }
    }
    if (u_abs < T) {
        if (rope) rope_rotate_dT<DH>(dkacc, rope, u_abs, -1.f, g);   // linear, so it commutes with the scale below
        write_rows_from_dT<DH>(dk + (long)u_abs * ldq + (long)head * DH, dkacc, scale, g);
        write_rows_from_dT<DH>(dv + (long)u_abs * ldq + (long)head * DH, dvacc, 1.f, g);
    }
}

// ======================================================================== backward: both in one launch
// Every workgroup does ONE part -- the dK/dV of a key block (all query blocks from it on) or the dQ of a query block (all
// key blocks up to it) -- and the parts are handed out longest first: level j of the grid holds the dK/dV part of key
// block j and the dQ part of query block n - 1 - j of every head, which cost about the same, and levels run from the
// heaviest down.  As two launches each part list has an 8:1 causal imbalance between its workgroups and, at 1024
// tokens x 32 heads, exactly one workgroup per CU, so the chip waits for the longest one twice; in one launch a CU that
// finishes a light part picks up the next.  delta must already be in memory (the dK/dV parts read rows that other
// workgroups' dQ parts own).  grid = (n blocks, heads, 2).
template <int DH, int NW>
__global__ __launch_bounds__(NW * 64) void attn_bwd_fused_kernel(
    const bf16_t* __restrict__ q, const bf16_t* __restrict__ k, const bf16_t* __restrict__ v,
    const bf16_t* __restrict__ d_o, const float* __restrict__ lse, const float* __restrict__ delta, long ldq, long ldo,
    int T, bf16_t* __restrict__ dq, bf16_t* __restrict__ dk, bf16_t* __restrict__ dv, float scale,
    const float2* __restrict__ rope) {
    extern __shared__ __align__(16) unsigned char smem[];
    const int n = gridDim.x, heads = gridDim.y;
    const int idx = (blockIdx.z * heads + blockIdx.y) * n + blockIdx.x;   // position in dispatch order (x fastest)
    const int level = idx / (2 * heads), r = idx % (2 * heads), head = r % heads;
    if (r < heads) attn_dkv_block<DH, NW>(q, k, v, d_o, lse, delta, ldq, ldo, T, dk, dv, scale, rope, level, head, smem);
    else attn_dq_block<DH, NW, 1>(q, k, v, d_o, lse, delta, ldq, ldo, T, dq, scale, rope, n - 1 - level, head, smem);
}

// ======================================================================== launchers
// waves per workgroup (32 queries / keys each), fixed at build time.  Measured at T = 1024, 32 heads of 128:
// 4 waves beat 2 (a K/V tile is shared by more queries; the extra workgroups of 2 do not overlap enough).
#ifndef ATTN_NW
#define ATTN_NW 4
#endif

// key groups of the forward kernel (see attn_fwd_kernel)
#ifndef ATTN_KG
#define ATTN_KG 2
#endif

template <int DH, int NW, int KG>
static hipError_t run_fwd(dim3 grid, const bf16_t* q, const bf16_t* k, const bf16_t* v, long ldq, int T, bf16_t* o,
                          long ldo, float* lse, float sl2, hipStream_t s) {
    using C = AttnCfg<DH>;
    size_t lds = (size_t)KG * (64 * C::LSK + 64 * LTR(DH)) * sizeof(bf16_t);
    const size_t merge = KG > 1 ? (size_t)NW * 64 * (C::ND * 16 + 2) * sizeof(float) : 0;
    if (merge > lds) lds = merge;
    auto kern = attn_fwd_kernel<DH, NW, KG>;
    hipError_t e = hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    if (e != hipSuccess) return e;
    kern<<<grid, NW * 64 * KG, lds, s>>>(q, k, v, ldq, T, o, ldo, lse, sl2);
    return hipGetLastError();
}

hipError_t launch_attention_fwd(const bf16_t* q, const bf16_t* k, const bf16_t* v, long ldq, int T, int n_heads,
                                int d_head, bf16_t* o, long ldo, float* lse, hipStream_t s) {
    if (T <= 0 || n_heads <= 0) return hipSuccess;
    if ((ldq & 7) || (ldo & 7)) return hipErrorInvalidValue;
    const float sl2 = (1.f / sqrtf((float)d_head)) * 1.4426950408889634f;
    constexpr int NW = ATTN_NW, KG = ATTN_KG;
    dim3 grid(cdiv(T, NW * 32), n_heads);
    if (d_head == 128) return run_fwd<128, NW, KG>(grid, q, k, v, ldq, T, o, ldo, lse, sl2, s);
    if (d_head == 64) return run_fwd<64, NW, KG>(grid, q, k, v, ldq, T, o, ldo, lse, sl2, s);
    return hipErrorInvalidValue;
}

// delta[head][t] = dO[t, head, :] . O[t, head, :] on its own, for the one-launch backward, whose dK/dV parts cannot
// wait for the dQ parts of other workgroups to produce it: DH / 8 lanes per (t, head), 16 bytes each.
template <int DH>
__global__ __launch_bounds__(256) void attn_delta_kernel(const bf16_t* __restrict__ o, const bf16_t* __restrict__ d_o,
                                                         long ldo, int T, int n_heads, float* __restrict__ delta) {
    // grid: x over the heads of a token (256 / LPR heads per workgroup), y over tokens
    constexpr int LPR = DH / 8;
    const int head_raw = (int)(blockIdx.x * 256 + threadIdx.x) / LPR, sub = threadIdx.x % LPR;
    const bool live = head_raw < n_heads;
    const int head = live ? head_raw : 0;
    for (long t = blockIdx.y; t < T; t += gridDim.y) {
        float a[8], b[8], dot = 0.f;
        unpack8(*(const uint4*)(o + t * ldo + (long)head * DH + sub * 8), a);
        unpack8(*(const uint4*)(d_o + t * ldo + (long)head * DH + sub * 8), b);
#pragma unroll
        for (int e = 0; e < 8; ++e) dot += a[e] * b[e];
        for (int off = LPR >> 1; off > 0; off >>= 1) dot += __shfl_xor(dot, off, 64);
        if (live && sub == 0) delta[(long)head * T + t] = dot;
    }
}

// delta from its own small kernel, then one launch that holds every dK/dV and every dQ part, longest first.
template <int DH>
static hipError_t run_bwd(const bf16_t* q, const bf16_t* k, const bf16_t* v, const bf16_t* o, const bf16_t* d_o,
                          const float* lse, float* delta, long ldq, long ldo, int T, int n_heads, bf16_t* dq, bf16_t* dk,
                          bf16_t* dv, const float2* rope, hipStream_t s) {
    using C = AttnCfg<DH>;
    constexpr int NW = ATTN_NW;
    const float scale = 1.f / sqrtf((float)DH);
    dim3 grid(cdiv(T, NW * 32), n_heads, 2);
    const size_t lds_kv = (size_t)(2 * 64 * C::LSK + 2 * 64 * LTR(DH)) * sizeof(bf16_t) + 128 * sizeof(float);
    const dim3 dgrid(cdiv((long)n_heads * (DH / 8), 256), T < 65535 ? T : 65535);
    attn_delta_kernel<DH><<<dgrid, 256, 0, s>>>(o, d_o, ldo, T, n_heads, delta);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    const size_t lds_q = (size_t)(2 * 64 * C::LSK + 64 * LTR(DH)) * sizeof(bf16_t);
    const size_t lds = lds_q > lds_kv ? lds_q : lds_kv;
    auto kern = attn_bwd_fused_kernel<DH, NW>;
    e = hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    if (e != hipSuccess) return e;
    kern<<<grid, NW * 64, lds, s>>>(q, k, v, d_o, lse, delta, ldq, ldo, T, dq, dk, dv, scale, rope);
    return hipGetLastError();
}

// delta (fp32 [n_heads, T]) = rowsum(dO * O), workspace written here and read by the dK/dV part.  rope != null: q and k
// were rotated by RoPE (table of (cos, sin) per position and pair, positions 0 .. T-1) before the forward pass, and dq,
// dk come out as gradients with respect to the UNROTATED projections.
hipError_t launch_attention_bwd(const bf16_t* q, const bf16_t* k, const bf16_t* v, const bf16_t* o, const bf16_t* d_o,
                                const float* lse, long ldq, long ldo, int T, int n_heads, int d_head, bf16_t* dq,
                                bf16_t* dk, bf16_t* dv, float* delta, const float2* rope, hipStream_t s) {
    if (T <= 0 || n_heads <= 0) return hipSuccess;
    if ((ldq & 7) || (ldo & 7)) return hipErrorInvalidValue;
    if (d_head == 128) return run_bwd<128>(q, k, v, o, d_o, lse, delta, ldq, ldo, T, n_heads, dq, dk, dv, rope, s);
    if (d_head == 64) return run_bwd<64>(q, k, v, o, d_o, lse, delta, ldq, ldo, T, n_heads, dq, dk, dv, rope, s);
    return hipErrorInvalidValue;
}
