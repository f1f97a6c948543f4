// One-token kernels of the generation side of Algorithm 1 (greedy decoding with the temporary LoRA module and a
// key/value cache): matrix-vector products with the LoRA correction, attention of one query against the cache, and
// the greedy argmax.  All of them stream their operand once: at one token per step the decoder is bound by reading
// the 13.5 GB of frozen weights, not by arithmetic.
#include "kernels.h"

// ---------------------------------------------------------------- y = W x (+ s-scaled LoRA term) (+ residual)
// One wave per output row n: the row W[n, :] is read with 16-byte loads, 64 lanes wide; x sits in LDS.
// lora_h (fp32 [G * r], already scaled by s) and lora_b (bf16 [N, r]) add  sum_j B[n, j] h[(n / rows_per_group) r + j].
__global__ __launch_bounds__(256) void gemv_kernel(const bf16_t* __restrict__ W, long ldw, const bf16_t* __restrict__ x, int N,
                                                   int K, const bf16_t* __restrict__ lora_b, const float* __restrict__ lora_h,
                                                   int r, int rows_per_group, float alpha, const float* __restrict__ resid,
                                                   bf16_t* __restrict__ y_bf, float* __restrict__ y_f32) {
    extern __shared__ __align__(16) unsigned char smem[];
    bf16_t* sx = (bf16_t*)smem;
    for (int i = threadIdx.x * 8; i < K; i += blockDim.x * 8) *(uint4*)(sx + i) = *(const uint4*)(x + i);
    __syncthreads();
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int n = blockIdx.x * 4 + wave;
    if (n >= N) return;
    const bf16_t* w = W + (long)n * ldw;
    float acc = 0.f;
    int k = lane * 8;
    for (; k + 3 * 512 < K; k += 4 * 512) {          // four 16-byte loads of the row in flight per lane
        uint4 wv[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) wv[u] = *(const uint4*)(w + k + u * 512);
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
        unpack8(*(const uint4*)(w + k), a);
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
                       hipStream_t s) {
    if (N <= 0) return hipSuccess;
    if ((K & 7) || (ldw & 7) || K <= 0 || (size_t)K * 2 > 160 * 1024 || (!y_bf && !y_f32)) return hipErrorInvalidValue;
    const size_t lds = (size_t)K * sizeof(bf16_t);
    hipError_t e = hipFuncSetAttribute((const void*)gemv_kernel, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    if (e != hipSuccess) return e;
    gemv_kernel<<<cdiv(N, 4), 256, lds, s>>>(W, ldw, x, N, K, lora_b, lora_h, r, rows_per_group > 0 ? rows_per_group : N,
                                             alpha, resid, y_bf, y_f32);
    return hipGetLastError();
}

// ---------------------------------------------------------------- attention of one query against the cache
// One workgroup per head.  q: the query row (already rotated); K, V: rows 0 .. n_keys-1 of the cache with row stride
// ld (the layout q|k|v of the chunk path, so the cache IS the forward pass's saved projections).  Scores and the
// softmax are fp32; the output row is written in bf16.
__global__ __launch_bounds__(1024) void attn_decode_kernel(const bf16_t* __restrict__ q, const bf16_t* __restrict__ k,
                                                           const bf16_t* __restrict__ v, long ld, int n_keys, int d_head,
                                                           float scale, bf16_t* __restrict__ o) {
    extern __shared__ __align__(16) unsigned char smem[];
    float* sp = (float*)smem;                 // [n_keys] scores, then probabilities
    float* part_buf = sp + ((n_keys + 3) & ~3);   // [parts][d_head] partial outputs
    __shared__ float red[16];
    const int head = blockIdx.x, tid = threadIdx.x, nthr = blockDim.x;
    const bf16_t* qh = q + (long)head * d_head;
    const bf16_t* kh = k + (long)head * d_head;
    const bf16_t* vh = v + (long)head * d_head;
    // scores: a key row (d_head * 2 bytes, contiguous) is read by d_head / 8 adjacent lanes, 16 bytes each
    const int lpk = d_head >> 3, sub = tid % lpk, kpp = nthr / lpk;   // lanes per key, keys per pass
    float qv[8];
    unpack8(*(const uint4*)(qh + sub * 8), qv);
    float mx = -1.0e30f;
    for (int u0 = 0; u0 < n_keys; u0 += kpp) {
        const int u = u0 + tid / lpk;
        float sdot = 0.f;
        if (u < n_keys) {
            float a[8];
            unpack8(*(const uint4*)(kh + (long)u * ld + sub * 8), a);
#pragma unroll
            for (int e = 0; e < 8; ++e) sdot += a[e] * qv[e];
        }
        for (int off = lpk >> 1; off > 0; off >>= 1) sdot += __shfl_xor(sdot, off, 64);
        if (u < n_keys && sub == 0) sp[u] = sdot * scale;
    }
    __syncthreads();
    for (int u = tid; u < n_keys; u += nthr) mx = fmaxf(mx, sp[u]);
    mx = block_max(mx, red);
    float sum = 0.f;
    for (int u = tid; u < n_keys; u += nthr) {
        const float p = __expf(sp[u] - mx);
        sp[u] = p;
        sum += p;
    }
    sum = block_sum(sum, red);
    __syncthreads();
    // thread (c, part): column c of the head over keys part, part + parts, .. (a V row is read by d_head adjacent lanes)
    const int parts = nthr / d_head, c = tid % d_head, part = tid / d_head;
    float acc = 0.f;
    for (int u = part; u < n_keys; u += parts) acc += sp[u] * bf16_to_f32(vh[(long)u * ld + c]);
    part_buf[part * d_head + c] = acc;
    __syncthreads();
    if (tid < d_head) {
        float t = 0.f;
        for (int pp = 0; pp < parts; ++pp) t += part_buf[pp * d_head + tid];
        o[(long)head * d_head + tid] = f32_to_bf16(t / sum);
    }
}

// Long windows: the keys are cut into n_split ranges, one workgroup per (head, range), so that the cache is read by
// hundreds of workgroups instead of one per head.  Each writes its unnormalised output, its score maximum and its
// sum of exponentials to ws[(head * n_split + range) * (d_head + 2)]; attn_decode_combine_kernel merges the ranges.
__global__ __launch_bounds__(256) void attn_decode_split_kernel(const bf16_t* __restrict__ q, const bf16_t* __restrict__ k,
                                                                const bf16_t* __restrict__ v, long ld, int n_keys,
                                                                int d_head, float scale, int chunk,
                                                                float* __restrict__ ws) {
    extern __shared__ __align__(16) unsigned char smem[];
    float* sp = (float*)smem;                     // [chunk] scores, then probabilities
    float* part_buf = sp + ((chunk + 3) & ~3);    // [parts][d_head]
    __shared__ float red[16];
    const int head = blockIdx.x, tid = threadIdx.x, nthr = blockDim.x;
    const int k0 = blockIdx.y * chunk, nk = min(chunk, n_keys - k0);   // nk >= 1 by the launch geometry
    const bf16_t* qh = q + (long)head * d_head;
    const bf16_t* kh = k + (long)k0 * ld + (long)head * d_head;
    const bf16_t* vh = v + (long)k0 * ld + (long)head * d_head;
    const int lpk = d_head >> 3, sub = tid % lpk, kpp = nthr / lpk;
    float qv[8];
    unpack8(*(const uint4*)(qh + sub * 8), qv);
    for (int u0 = 0; u0 < nk; u0 += kpp) {
        const int u = u0 + tid / lpk;
        float sdot = 0.f;
        if (u < nk) {
            float a[8];
            unpack8(*(const uint4*)(kh + (long)u * ld + sub * 8), a);
#pragma unroll
            for (int e = 0; e < 8; ++e) sdot += a[e] * qv[e];
        }
        for (int off = lpk >> 1; off > 0; off >>= 1) sdot += __shfl_xor(sdot, off, 64);
        if (u < nk && sub == 0) sp[u] = sdot * scale;
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
    const int parts = nthr / d_head, c = tid % d_head, part = tid / d_head;
    float acc = 0.f;
    for (int u = part; u < nk; u += parts) acc += sp[u] * bf16_to_f32(vh[(long)u * ld + c]);
    part_buf[part * d_head + c] = acc;
    __syncthreads();
    float* out = ws + ((long)head * gridDim.y + blockIdx.y) * (d_head + 2);
    if (tid < d_head) {
        float t = 0.f;
        for (int pp = 0; pp < parts; ++pp) t += part_buf[pp * d_head + tid];
        out[tid] = t;
    }
    if (tid == 0) { out[d_head] = mx; out[d_head + 1] = sum; }
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
hipError_t launch_attention_decode(const bf16_t* q, const bf16_t* k, const bf16_t* v, long ld, int n_keys, int n_heads,
                                   int d_head, bf16_t* o, float* ws, size_t ws_elems, hipStream_t s) {
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
        const int parts = 256 / d_head;
        const size_t lds = ((size_t)((chunk + 3) & ~3) + (size_t)parts * d_head) * sizeof(float);
        if (lds > 60 * 1024) return hipErrorInvalidValue;
        attn_decode_split_kernel<<<dim3(n_heads, n_split), 256, lds, s>>>(q, k, v, ld, n_keys, d_head, scale, chunk, ws);
        hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
        attn_decode_combine_kernel<<<n_heads, d_head, 0, s>>>(ws, n_split, d_head, o);
        return hipGetLastError();
    }
    const int nthr = n_keys > 128 ? 1024 : 256;
    const int parts = nthr / d_head;
    const size_t lds = ((size_t)((n_keys + 3) & ~3) + (size_t)parts * d_head) * sizeof(float);
    if (lds > 150 * 1024) return hipErrorInvalidValue;
    hipError_t e = hipFuncSetAttribute((const void*)attn_decode_kernel, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    if (e != hipSuccess) return e;
    attn_decode_kernel<<<n_heads, nthr, lds, s>>>(q, k, v, ld, n_keys, d_head, scale, o);
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
