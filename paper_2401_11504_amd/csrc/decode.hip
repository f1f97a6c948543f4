// One-token kernels of the generation side of Algorithm 1 (greedy decoding with the temporary LoRA module and a
// key/value cache): matrix-vector products with the LoRA correction, attention of one query against the cache, and
// the greedy argmax.  All of them stream their operand once: at one token per step the decoder is bound by reading
// the 13.5 GB of frozen weights, not by arithmetic.
#include "kernels.h"

typedef unsigned gemv_vu4 __attribute__((ext_vector_type(4)));
// 16 bytes of a weight row.  Every byte of the matrix is read exactly once per token, so the loads are marked
// non-temporal: measured 5 % faster per token than ordinary loads (eight loads in flight instead of four, two or four
// rows per wave, or two waves per row were all slower or equal).
__device__ __forceinline__ uint4 load_w16(const bf16_t* p) {
    const gemv_vu4 v = __builtin_nontemporal_load((const gemv_vu4*)p);
    return make_uint4(v.x, v.y, v.z, v.w);
}

// ---------------------------------------------------------------- y = W x (+ s-scaled LoRA term) (+ residual)
// One wave per output row n: the row W[n, :] is read with 16-byte loads, 64 lanes wide; x sits in LDS.
// lora_h (fp32 [G * r], already scaled by s) and lora_b (bf16 [N, r]) add  sum_j B[n, j] h[(n / rows_per_group) r + j].
// Where x comes from (pre.mode): 0 a bf16 vector; 1 RMSNorm of an fp32 row, x = bf16(h rho gain); 2 SwiGLU of a
// gate|up row, x = bf16(silu(g) u).  Modes 1 and 2 do the work of the separate kernels in every workgroup (the
// vector is a few KB out of L2), and workgroup 0 stores x to pre.x_out for the launches that follow.
__global__ __launch_bounds__(256) void gemv_kernel(const bf16_t* __restrict__ W, long ldw, const bf16_t* __restrict__ x, int N,
                                                   int K, const bf16_t* __restrict__ lora_b, const float* __restrict__ lora_h,
                                                   int r, int rows_per_group, float alpha, const float* __restrict__ resid,
                                                   bf16_t* __restrict__ y_bf, float* __restrict__ y_f32, GemvPre pre,
                                                   int row_per_block) {
    extern __shared__ __align__(16) unsigned char smem[];
    __shared__ float red[16];
    bf16_t* sx = (bf16_t*)smem;
    if (pre.mode == 1) {
        float ss = 0.f;
        for (int i = threadIdx.x * 4; i < K; i += blockDim.x * 4) {
            const float4 v = *(const float4*)(pre.h + i);
            ss += v.x * v.x + v.y * v.y + v.z * v.z + v.w * v.w;
        }
        ss = block_sum(ss, red);
        const float rho = rsqrtf(ss / (float)K + pre.eps);
        for (int i = threadIdx.x * 4; i < K; i += blockDim.x * 4) {
            const float4 v = *(const float4*)(pre.h + i), w = *(const float4*)(pre.gain + i);
            uint2 o;
            o.x = pack_bf16x2(v.x * rho * w.x, v.y * rho * w.y);
            o.y = pack_bf16x2(v.z * rho * w.z, v.w * rho * w.w);
            *(uint2*)(sx + i) = o;
        }
    } else if (pre.mode == 2) {
        for (int i = threadIdx.x * 8; i < K; i += blockDim.x * 8) {
            float g[8], u[8], o[8];
            unpack8(*(const uint4*)(pre.gu + i), g);
            unpack8(*(const uint4*)(pre.gu + K + i), u);
#pragma unroll
            for (int e = 0; e < 8; ++e) o[e] = g[e] / (1.f + __expf(-g[e])) * u[e];
            *(uint4*)(sx + i) = pack8(o);
        }
    } else {
        for (int i = threadIdx.x * 8; i < K; i += blockDim.x * 8) *(uint4*)(sx + i) = *(const uint4*)(x + i);
    }
    __syncthreads();
    if (pre.x_out && blockIdx.x == 0)
        for (int i = threadIdx.x * 8; i < K; i += blockDim.x * 8) *(uint4*)(pre.x_out + i) = *(const uint4*)(sx + i);
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    if (row_per_block) {
        // few rows (the LoRA A factors): the whole workgroup shares one row, so that the row's loads are all in
        // flight at once instead of queued behind one wave
        const int n = blockIdx.x;
        const bf16_t* w = W + (long)n * ldw;
        float acc = 0.f;
        for (int k = threadIdx.x * 8; k < K; k += 2048) {
            float a[8], b[8];
            unpack8(*(const uint4*)(w + k), a);
            unpack8(*(const uint4*)(sx + k), b);
#pragma unroll
            for (int e = 0; e < 8; ++e) acc += a[e] * b[e];
        }
        if (lora_b) {
            const float* h = lora_h + (long)(n / rows_per_group) * r;
            const bf16_t* b = lora_b + (long)n * r;
            for (int j = threadIdx.x; j < r; j += 256) acc += bf16_to_f32(b[j]) * h[j];
        }
        acc = block_sum(acc, red);
        if (threadIdx.x == 0) {
            float v = alpha * acc;
            if (y_f32) y_f32[n] = v + (resid ? resid[n] : 0.f);
            else y_bf[n] = f32_to_bf16(v);
        }
        return;
    }
    const int n = blockIdx.x * 4 + wave;
    if (n >= N) return;
    const bf16_t* w = W + (long)n * ldw;
    float acc = 0.f;
    int k = lane * 8;
    for (; k + 3 * 512 < K; k += 4 * 512) {          // four 16-byte loads of the row in flight per lane
        uint4 wv[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) wv[u] = load_w16(w + k + u * 512);
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            float a[8], b[8];
            unpack8(wv[u], a);
            unpack8(*(const uint4*)(sx + k + u * 512), b);
#pragma unroll
            for (int e = 0; e < 8; ++e) acc += a[e] * b[e];
        }
    }
    for (; k < K; k += 512) {
        float a[8], b[8];
        unpack8(load_w16(w + k), a);
        unpack8(*(const uint4*)(sx + k), b);
#pragma unroll
        for (int e = 0; e < 8; ++e) acc += a[e] * b[e];
    }
    if (lora_b) {
        const float* h = lora_h + (long)(n / rows_per_group) * r;
        const bf16_t* b = lora_b + (long)n * r;
        for (int j = lane; j < r; j += 64) acc += bf16_to_f32(b[j]) * h[j];
    }
    acc = wave_sum(acc);
    if (lane == 0) {
        float v = alpha * acc;
        if (y_f32) y_f32[n] = v + (resid ? resid[n] : 0.f);
        else y_bf[n] = f32_to_bf16(v);
    }
}

hipError_t launch_gemv(const bf16_t* W, long ldw, const bf16_t* x, int N, int K, const bf16_t* lora_b, const float* lora_h,
                       int r, int rows_per_group, float alpha, const float* resid, bf16_t* y_bf, float* y_f32,
                       hipStream_t s, const GemvPre* pre) {
    if (N <= 0) return hipSuccess;
    if ((K & 7) || (ldw & 7) || K <= 0 || (size_t)K * 2 > 160 * 1024 || (!y_bf && !y_f32)) return hipErrorInvalidValue;
    GemvPre p = pre ? *pre : GemvPre{};
    if (p.mode < 0 || p.mode > 2 || (p.mode == 0 && !x) || (p.mode == 1 && (!p.h || !p.gain)) || (p.mode == 2 && !p.gu))
        return hipErrorInvalidValue;
    const size_t lds = (size_t)K * sizeof(bf16_t);
    hipError_t e = hipFuncSetAttribute((const void*)gemv_kernel, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    if (e != hipSuccess) return e;
    const int row_per_block = N <= 512;
    gemv_kernel<<<row_per_block ? N : cdiv(N, 4), 256, lds, s>>>(W, ldw, x, N, K, lora_b, lora_h, r,
                                                                 rows_per_group > 0 ? rows_per_group : N, alpha, resid, y_bf,
                                                                 y_f32, p, row_per_block);
    return hipGetLastError();
}

// ---------------------------------------------------------------- attention of one query against the cache
// q: the query row (already rotated); K, V: rows 0 .. n_keys-1 of the cache with row stride ld (the layout q|k|v of
// the chunk path, so the cache IS the forward pass's saved projections).  Scores and the softmax are fp32; the
// output row is written in bf16.
//
// attend_range: one head against nk consecutive keys, by one workgroup.  A key (or value) row of the head is
// d_head * 2 contiguous bytes, read by d_head / 8 adjacent lanes with one 16-byte load each, so a workgroup covers
// blockDim / (d_head / 8) keys per pass; four passes of loads are issued before the first is consumed (the loop is
// bound by load latency, not by bytes).  Returns the score maximum and the sum of exponentials; the unnormalised
// output sum_u exp(s_u - max) v_u is left in out_acc[0 .. d_head).
//
// rope_row != null: the query row and key row `new_key` of the range (the token being decoded; -1 if it lies in another
// range) are still unrotated.  They are rotated here with the (cos, sin) pairs of the token's position (RoPE pairs
// elements i and i + d_head / 2; both halves of a row are held by lanes of the same wave), rounded to bf16 as the
// separate kernel would have stored them, and the rotated key is written back to the cache for the tokens to come.
__device__ __forceinline__ void rope8(const float* mine, const float* other, const float2* __restrict__ rope_row,
                                      int sub, int lpk, float* out) {
    const bool first = sub < (lpk >> 1);
    const int i0 = (sub % (lpk >> 1)) * 8;
#pragma unroll
    for (int e = 0; e < 8; ++e) {
        const float2 cs = rope_row[i0 + e];
        const float a = first ? mine[e] : other[e], b = first ? other[e] : mine[e];   // a: first-half element of the pair
        out[e] = bf16_to_f32(f32_to_bf16(first ? a * cs.x - b * cs.y : b * cs.x + a * cs.y));
    }
}
__device__ __forceinline__ void attend_range(const bf16_t* __restrict__ qh, bf16_t* __restrict__ kh,
                                             const bf16_t* __restrict__ vh, long ld, int nk, int d_head, float scale,
                                             float* sp, float* part_buf, float* red, float& mx_out, float& sum_out,
                                             const float2* __restrict__ rope_row, int new_key) {
    const int tid = threadIdx.x, nthr = blockDim.x;
    const int lpk = d_head >> 3, sub = tid % lpk, kk = tid / lpk, kpp = nthr / lpk;   // lanes per key, keys per pass
    const int psub = sub ^ (lpk >> 1);                                                 // the lane holding the pair partners
    float qv[8];
    unpack8(*(const uint4*)(qh + sub * 8), qv);
    if (rope_row) {
        float other[8], rot[8];
        unpack8(*(const uint4*)(qh + psub * 8), other);
        rope8(qv, other, rope_row, sub, lpk, rot);
#pragma unroll
        for (int e = 0; e < 8; ++e) qv[e] = rot[e];
    }
    for (int u0 = 0; u0 < nk; u0 += 4 * kpp) {
        uint4 kr[4];
#pragma unroll
        for (int b = 0; b < 4; ++b) {
            const int u = u0 + b * kpp + kk;
            kr[b] = u < nk ? *(const uint4*)(kh + (long)u * ld + sub * 8) : make_uint4(0, 0, 0, 0);
        }
#pragma unroll
        for (int b = 0; b < 4; ++b) {
            const int u = u0 + b * kpp + kk;
            float a[8], sdot = 0.f;
            unpack8(kr[b], a);
            if (rope_row && u == new_key) {      // taken by the d_head / 8 lanes of one key, all in one wave
                float other[8], rot[8];
                unpack8(*(const uint4*)(kh + (long)u * ld + psub * 8), other);
                rope8(a, other, rope_row, sub, lpk, rot);
                *(uint4*)(kh + (long)u * ld + sub * 8) = pack8(rot);
#pragma unroll
                for (int e = 0; e < 8; ++e) a[e] = rot[e];
            }
#pragma unroll
            for (int e = 0; e < 8; ++e) sdot += a[e] * qv[e];
            for (int off = lpk >> 1; off > 0; off >>= 1) sdot += __shfl_xor(sdot, off, 64);
            if (u < nk && sub == 0) sp[u] = sdot * scale;
        }
    }
    __syncthreads();
    float mx = -1.0e30f;
    for (int u = tid; u < nk; u += nthr) mx = fmaxf(mx, sp[u]);
    mx = block_max(mx, red);
    float sum = 0.f;
    for (int u = tid; u < nk; u += nthr) {
        const float pr = __expf(sp[u] - mx);
        sp[u] = pr;
        sum += pr;
    }
    sum = block_sum(sum, red);
    __syncthreads();
    // lane group kk accumulates its keys' share of columns sub*8 .. sub*8+7; the groups are summed through LDS
    float acc[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
    for (int u0 = 0; u0 < nk; u0 += 4 * kpp) {
        uint4 vr[4];
#pragma unroll
        for (int b = 0; b < 4; ++b) {
            const int u = u0 + b * kpp + kk;
            vr[b] = u < nk ? *(const uint4*)(vh + (long)u * ld + sub * 8) : make_uint4(0, 0, 0, 0);
        }
#pragma unroll
        for (int b = 0; b < 4; ++b) {
            const int u = u0 + b * kpp + kk;
            const float pr = u < nk ? sp[u] : 0.f;
            float a[8];
            unpack8(vr[b], a);
#pragma unroll
            for (int e = 0; e < 8; ++e) acc[e] += pr * a[e];
        }
    }
#pragma unroll
    for (int e = 0; e < 8; ++e) part_buf[kk * d_head + sub * 8 + e] = acc[e];
    __syncthreads();
    if (tid < d_head) {
        float t = 0.f;
        for (int g = 0; g < kpp; ++g) t += part_buf[g * d_head + tid];
        part_buf[tid] = t;      // only entry [0][tid] is overwritten, by the thread that has just read column tid
    }
    mx_out = mx;
    sum_out = sum;
}

// LDS floats attend_range needs for nk keys with nthr threads
static size_t attend_lds_floats(int nk, int nthr, int d_head) {
    return (size_t)((nk + 3) & ~3) + (size_t)(nthr / (d_head / 8)) * d_head;
}

// One workgroup per head over the whole cache.
__global__ __launch_bounds__(1024) void attn_decode_kernel(const bf16_t* __restrict__ q, bf16_t* __restrict__ k,
                                                           const bf16_t* __restrict__ v, long ld, int n_keys, int d_head,
                                                           float scale, bf16_t* __restrict__ o,
                                                           const float2* __restrict__ rope_row) {
    extern __shared__ __align__(16) unsigned char smem[];
    float* sp = (float*)smem;
    float* part_buf = sp + ((n_keys + 3) & ~3);
    __shared__ float red[16];
    const int head = blockIdx.x;
    float mx, sum;
    attend_range(q + (long)head * d_head, k + (long)head * d_head, v + (long)head * d_head, ld, n_keys, d_head, scale, sp,
                 part_buf, red, mx, sum, rope_row, n_keys - 1);
    if ((int)threadIdx.x < d_head) o[(long)head * d_head + threadIdx.x] = f32_to_bf16(part_buf[threadIdx.x] / sum);
}

// Long windows: the keys are cut into n_split ranges, one workgroup per (head, range), so that the cache is read by
// hundreds of workgroups instead of one per head.  Each writes its unnormalised output, its score maximum and its
// sum of exponentials to ws[(head * n_split + range) * (d_head + 2)]; attn_decode_combine_kernel merges the ranges.
__global__ __launch_bounds__(256) void attn_decode_split_kernel(const bf16_t* __restrict__ q, bf16_t* __restrict__ k,
                                                                const bf16_t* __restrict__ v, long ld, int n_keys,
                                                                int d_head, float scale, int chunk,
                                                                float* __restrict__ ws,
                                                                const float2* __restrict__ rope_row) {
    extern __shared__ __align__(16) unsigned char smem[];
    float* sp = (float*)smem;
    float* part_buf = sp + ((chunk + 3) & ~3);
    __shared__ float red[16];
    const int head = blockIdx.x;
    const int k0 = blockIdx.y * chunk, nk = min(chunk, n_keys - k0);   // nk >= 1 by the launch geometry
    float mx, sum;
    const int new_key = n_keys - 1 - k0;                             // inside this range only for the last one
    attend_range(q + (long)head * d_head, k + (long)k0 * ld + (long)head * d_head, v + (long)k0 * ld + (long)head * d_head,
                 ld, nk, d_head, scale, sp, part_buf, red, mx, sum, rope_row, new_key < nk ? new_key : -1);
    float* out = ws + ((long)head * gridDim.y + blockIdx.y) * (d_head + 2);
    if ((int)threadIdx.x < d_head) out[threadIdx.x] = part_buf[threadIdx.x];
    if (threadIdx.x == 0) { out[d_head] = mx; out[d_head + 1] = sum; }
}

__global__ void attn_decode_combine_kernel(const float* __restrict__ ws, int n_split, int d_head, bf16_t* __restrict__ o) {
    const int head = blockIdx.x, c = threadIdx.x;
    const float* w = ws + (long)head * n_split * (d_head + 2);
    float M = -1.0e30f;
    for (int i = 0; i < n_split; ++i) M = fmaxf(M, w[i * (d_head + 2) + d_head]);
    float L = 0.f, acc = 0.f;
    for (int i = 0; i < n_split; ++i) {
        const float e = __expf(w[i * (d_head + 2) + d_head] - M);
        L += e * w[i * (d_head + 2) + d_head + 1];
        acc += e * w[i * (d_head + 2) + c];
    }
    o[(long)head * d_head + c] = f32_to_bf16(acc / L);
}

// ws (may be null): scratch of ws_elems floats for the split path; n_heads * n_split * (d_head + 2) of them are used.
// rope_row (may be null): (cos, sin) of the newest position for i = 0 .. d_head / 2 - 1.  With it q and key row
// n_keys - 1 are taken as unrotated, and the rotated key row is written back into k (k is then written, not only read).
hipError_t launch_attention_decode(const bf16_t* q, bf16_t* k, const bf16_t* v, long ld, int n_keys, int n_heads,
                                   int d_head, bf16_t* o, float* ws, size_t ws_elems, hipStream_t s,
                                   const float2* rope_row) {
    if (n_keys <= 0 || n_heads <= 0) return hipErrorInvalidValue;
    if ((d_head != 64 && d_head != 128) || (ld & 7)) return hipErrorInvalidValue;
    const float scale = 1.f / sqrtf((float)d_head);
    // ranges of at least 128 keys, at most ATTN_DECODE_MAX_SPLIT of them, as many as the scratch holds
    // (below about 400 keys one workgroup per head is as fast and saves the second launch)
    int n_split = ws && n_keys >= 384 ? min(cdiv(n_keys, 128), ATTN_DECODE_MAX_SPLIT) : 1;
    if (ws && (size_t)n_heads * n_split * (d_head + 2) > ws_elems) n_split = (int)(ws_elems / ((size_t)n_heads * (d_head + 2)));
    if (n_split >= 2) {
        const int chunk = cdiv(n_keys, n_split);
        n_split = cdiv(n_keys, chunk);            // no empty range
        const size_t lds = attend_lds_floats(chunk, 256, d_head) * sizeof(float);
        if (lds > 60 * 1024) return hipErrorInvalidValue;
        attn_decode_split_kernel<<<dim3(n_heads, n_split), 256, lds, s>>>(q, k, v, ld, n_keys, d_head, scale, chunk, ws,
                                                                          rope_row);
        hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
        attn_decode_combine_kernel<<<n_heads, d_head, 0, s>>>(ws, n_split, d_head, o);
        return hipGetLastError();
    }
    const int nthr = n_keys > 128 ? 1024 : 256;
    const size_t lds = attend_lds_floats(n_keys, nthr, d_head) * sizeof(float);
    if (lds > 150 * 1024) return hipErrorInvalidValue;
    hipError_t e = hipFuncSetAttribute((const void*)attn_decode_kernel, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    if (e != hipSuccess) return e;
    attn_decode_kernel<<<n_heads, nthr, lds, s>>>(q, k, v, ld, n_keys, d_head, scale, o, rope_row);
    return hipGetLastError();
}

// ---------------------------------------------------------------- greedy choice: index of the largest logit
// The lowest index wins among equal values.  One workgroup.
__global__ __launch_bounds__(1024) void argmax_kernel(const float* __restrict__ x, int n, int* __restrict__ out) {
    __shared__ float bv[16];
    __shared__ int bi[16];
    float best = -INFINITY;
    int idx = 0x7fffffff;
    for (int i = threadIdx.x; i < n; i += blockDim.x) {
        const float v = x[i];
        if (v > best || (v == best && i < idx)) { best = v; idx = i; }
    }
    for (int off = 32; off > 0; off >>= 1) {
        const float ov = __shfl_xor(best, off, 64);
        const int oi = __shfl_xor(idx, off, 64);
        if (ov > best || (ov == best && oi < idx)) { best = ov; idx = oi; }
    }
    const int w = threadIdx.x >> 6;
    if ((threadIdx.x & 63) == 0) { bv[w] = best; bi[w] = idx; }
    __syncthreads();
    if (threadIdx.x == 0) {
        for (int k = 1; k < (int)(blockDim.x >> 6); ++k)
            if (bv[k] > best || (bv[k] == best && bi[k] < idx)) { best = bv[k]; idx = bi[k]; }
        *out = idx;
    }
}

hipError_t launch_argmax(const float* x, int n, int* out, hipStream_t s) {
    if (n <= 0) return hipErrorInvalidValue;
    argmax_kernel<<<1, 1024, 0, s>>>(x, n, out);
    return hipGetLastError();
}
