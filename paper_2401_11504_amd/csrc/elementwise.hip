// Bandwidth-bound kernels of the Temp-Lora chunk update: RMSNorm, RoPE, SwiGLU,
// embedding gather, fused softmax cross-entropy, fused AdamW, and layout helpers.
// Every kernel streams its operands once with 16-byte accesses where the layout allows.
#include "kernels.h"

// ---------------------------------------------------------------- RMSNorm
// One block per token row.  y = h * rsqrt(mean(h^2) + eps) * g   (Llama2 decoder norm).
// With d <= 256 * 4 * NV the row stays in registers between the reduction and the output pass (NV float4 per
// thread); wider rows are read twice (NV = 0).
template <int NV>
__global__ __launch_bounds__(256) void rmsnorm_fwd_kernel(const float* h, const float* __restrict__ g,
                                                          int d, float eps, bf16_t* __restrict__ y,
                                                          const float* __restrict__ part, int n_part, long part_stride,
                                                          const float* resid, float* h_write) {
    __shared__ float red[16];
    const long row = blockIdx.x;
    // chunk i (four elements) of the row: read from h, or (part != null) assembled as the sum of the partial tiles a
    // split GEMM left behind plus the residual, which becomes the residual stream (h_write) on the way
    auto fetch = [&](int i) {
        if (!part) return ((const float4*)(h + row * d))[i];
        float4 t = resid ? *(const float4*)(resid + row * d + 4 * (long)i) : make_float4(0.f, 0.f, 0.f, 0.f);
        for (int k = 0; k < n_part; ++k) {
            const float4 q = *(const float4*)(part + (long)k * part_stride + row * d + 4 * (long)i);
            t.x += q.x; t.y += q.y; t.z += q.z; t.w += q.w;
        }
        *(float4*)(h_write + row * d + 4 * (long)i) = t;
        return t;
    };
    const float4* gp = (const float4*)g;
    uint2* yp = (uint2*)(y + row * d);
    const int n4 = d >> 2;
    float ss = 0.f;
    constexpr int NR = NV > 0 ? NV : 1;
    float4 xs[NR], ws[NR];
    if constexpr (NV > 0) {
#pragma unroll
        for (int j = 0; j < NV; ++j) {
            const int i = threadIdx.x + 256 * j;
            xs[j] = i < n4 ? fetch(i) : make_float4(0.f, 0.f, 0.f, 0.f);
            ws[j] = i < n4 ? gp[i] : make_float4(0.f, 0.f, 0.f, 0.f);   // the gain too: the output pass then only stores
            ss += xs[j].x * xs[j].x + xs[j].y * xs[j].y + xs[j].z * xs[j].z + xs[j].w * xs[j].w;
        }
    } else {
        for (int i = threadIdx.x; i < n4; i += blockDim.x) {
            const float4 x = fetch(i);
            ss += x.x * x.x + x.y * x.y + x.z * x.z + x.w * x.w;
        }
    }
    ss = block_sum(ss, red);
    const float rho = rsqrtf(ss / (float)d + eps);
    auto emit = [&](int i, const float4& x, const float4& w) {
        uint2 o;
        o.x = pack_bf16x2(x.x * rho * w.x, x.y * rho * w.y);
        o.y = pack_bf16x2(x.z * rho * w.z, x.w * rho * w.w);
        yp[i] = o;
    };
    if constexpr (NV > 0) {
#pragma unroll
        for (int j = 0; j < NV; ++j) {
            const int i = threadIdx.x + 256 * j;
            if (i < n4) emit(i, xs[j], ws[j]);
        }
    } else {
        const float4* hp = (const float4*)((part ? h_write : h) + row * d);   // each thread re-reads only what it wrote itself
        for (int i = threadIdx.x; i < n4; i += blockDim.x) emit(i, hp[i], gp[i]);
    }
}

// dh_out = dres + rho (g*dy) - h rho^3 mean(h g dy); gain is frozen, so no gain gradient.
// One workgroup per row.  With d <= 256 * 4 * NV the row is read once and kept in registers between the two
// reductions and the output pass (NV float4 per thread); wider rows take the two-pass form (NV = 0).
template <int NV>
__global__ __launch_bounds__(256) void rmsnorm_bwd_kernel(const bf16_t* __restrict__ dy, const float* __restrict__ h,
                                                          const float* __restrict__ g, const float* __restrict__ dres,
                                                          int d, float eps, float* __restrict__ dh_out,
                                                          bf16_t* __restrict__ dh_bf, const float* __restrict__ dy_part,
                                                          int n_part, long part_stride, int part_bf16) {
    __shared__ float red[32];
    const long row = blockIdx.x;
    // chunk i (four elements) of this row of dy: the bf16 array, or the sum of the partial arrays (fp32 or bf16)
    auto dy4 = [&](int i) {
        if (dy_part) {
            float4 t = make_float4(0.f, 0.f, 0.f, 0.f);
            for (int k = 0; k < n_part; ++k) {
                if (part_bf16) {
                    const uint2 r = *(const uint2*)((const bf16_t*)dy_part + (long)k * part_stride + row * d + 4 * (long)i);
                    t.x += bf16_to_f32(r.x & 0xffff); t.y += bf16_to_f32(r.x >> 16);
                    t.z += bf16_to_f32(r.y & 0xffff); t.w += bf16_to_f32(r.y >> 16);
                } else {
                    const float4 q = *(const float4*)(dy_part + (long)k * part_stride + row * d + 4 * (long)i);
                    t.x += q.x; t.y += q.y; t.z += q.z; t.w += q.w;
                }
            }
            return t;
        }
        const uint2 r = ((const uint2*)(dy + row * d))[i];
        return make_float4(bf16_to_f32(r.x & 0xffff), bf16_to_f32(r.x >> 16), bf16_to_f32(r.y & 0xffff),
                           bf16_to_f32(r.y >> 16));
    };
    const float4* hp = (const float4*)(h + row * d);
    const float4* gp = (const float4*)g;
    const float4* rp = dres ? (const float4*)(dres + row * d) : nullptr;
    float4* op = (float4*)(dh_out + row * d);
    uint2* bp = dh_bf ? (uint2*)(dh_bf + row * d) : nullptr;
    const int n4 = d >> 2;
    float ss = 0.f, dot = 0.f;
    constexpr int NR = NV > 0 ? NV : 1;
    float4 xs[NR], gd[NR], rs[NR];   // h, g * dy and the upstream residual gradient of this thread's chunks: everything the
                                     // output pass needs is fetched before the reduction, so that pass only stores
    if constexpr (NV > 0) {
#pragma unroll
        for (int j = 0; j < NV; ++j) {
            const int i = threadIdx.x + 256 * j;
            xs[j] = make_float4(0.f, 0.f, 0.f, 0.f);
            gd[j] = xs[j];
            rs[j] = xs[j];
            if (i < n4) {
                if (rp) rs[j] = rp[i];
                const float4 x = hp[i], w = gp[i], dv = dy4(i);
                xs[j] = x;
                gd[j] = make_float4(w.x * dv.x, w.y * dv.y, w.z * dv.z, w.w * dv.w);
                ss += x.x * x.x + x.y * x.y + x.z * x.z + x.w * x.w;
                dot += x.x * gd[j].x + x.y * gd[j].y + x.z * gd[j].z + x.w * gd[j].w;
            }
        }
    } else {
        for (int i = threadIdx.x; i < n4; i += blockDim.x) {
            const float4 x = hp[i], w = gp[i], dv = dy4(i);
            ss += x.x * x.x + x.y * x.y + x.z * x.z + x.w * x.w;
            dot += x.x * w.x * dv.x + x.y * w.y * dv.y + x.z * w.z * dv.z + x.w * w.w * dv.w;
        }
    }
    // both sums through one pair of barriers
    ss = wave_sum(ss);
    dot = wave_sum(dot);
    const int wv = threadIdx.x >> 6;
    if ((threadIdx.x & 63) == 0) { red[wv] = ss; red[4 + wv] = dot; }
    __syncthreads();
    ss = (red[0] + red[1]) + (red[2] + red[3]);
    dot = (red[4] + red[5]) + (red[6] + red[7]);
    const float rho = rsqrtf(ss / (float)d + eps);
    const float c = rho * rho * rho * (dot / (float)d);
    auto emit = [&](int i, const float4& x, const float4& wd, const float4& q) {
        float4 o = make_float4(rho * wd.x - x.x * c, rho * wd.y - x.y * c, rho * wd.z - x.z * c, rho * wd.w - x.w * c);
        o.x += q.x; o.y += q.y; o.z += q.z; o.w += q.w;
        op[i] = o;
        if (bp) {
            uint2 b;
            b.x = pack_bf16x2(o.x, o.y);
            b.y = pack_bf16x2(o.z, o.w);
            bp[i] = b;
        }
    };
    if constexpr (NV > 0) {
#pragma unroll
        for (int j = 0; j < NV; ++j) {
            const int i = threadIdx.x + 256 * j;
            if (i < n4) emit(i, xs[j], gd[j], rs[j]);
        }
    } else {
        for (int i = threadIdx.x; i < n4; i += blockDim.x) {
            const float4 x = hp[i], w = gp[i], dv = dy4(i);
            emit(i, x, make_float4(w.x * dv.x, w.y * dv.y, w.z * dv.z, w.w * dv.w),
                 rp ? rp[i] : make_float4(0.f, 0.f, 0.f, 0.f));
        }
    }
}

hipError_t launch_rmsnorm_fwd(const float* h, const float* g, int T, int d, float eps, bf16_t* y, hipStream_t s,
                              const float* part, int n_part, long part_stride, const float* resid, float* h_write) {
    if (T <= 0) return hipSuccess;
    if (part ? (n_part < 1 || (part_stride & 3) || !h_write) : !h) return hipErrorInvalidValue;
    if (d <= 4096) rmsnorm_fwd_kernel<4><<<T, 256, 0, s>>>(h, g, d, eps, y, part, n_part, part_stride, resid, h_write);
    else if (d <= 8192) rmsnorm_fwd_kernel<8><<<T, 256, 0, s>>>(h, g, d, eps, y, part, n_part, part_stride, resid, h_write);
    else rmsnorm_fwd_kernel<0><<<T, 256, 0, s>>>(h, g, d, eps, y, part, n_part, part_stride, resid, h_write);
    return hipGetLastError();
}
hipError_t launch_rmsnorm_bwd(const bf16_t* dy, const float* h, const float* g, const float* dres, int T, int d,
                              float eps, float* dh_out, bf16_t* dh_bf, hipStream_t s, const float* dy_part, int n_part,
                              long part_stride, int part_bf16) {
    if (T <= 0) return hipSuccess;
    if (dy_part ? (n_part < 1 || (part_stride & 3)) : !dy) return hipErrorInvalidValue;
    if (d <= 4096) rmsnorm_bwd_kernel<4><<<T, 256, 0, s>>>(dy, h, g, dres, d, eps, dh_out, dh_bf, dy_part, n_part, part_stride, part_bf16);
    else if (d <= 8192) rmsnorm_bwd_kernel<8><<<T, 256, 0, s>>>(dy, h, g, dres, d, eps, dh_out, dh_bf, dy_part, n_part, part_stride, part_bf16);
    else rmsnorm_bwd_kernel<0><<<T, 256, 0, s>>>(dy, h, g, dres, d, eps, dh_out, dh_bf, dy_part, n_part, part_stride, part_bf16);
    return hipGetLastError();
}

// ---------------------------------------------------------------- RoPE
// Pair (i, i + d_head/2) of every head rotated by pos * base^(-2i/d_head) (half-split pairing).
// table[pos * d_head/2 + i] = (cos, sin) in fp32, built in fp64; without a table the angle is formed in fp64 here.
__global__ void rope_table_kernel(float2* table, int n_pos, int half, double base) {
    const long idx = (long)blockIdx.x * blockDim.x + threadIdx.x;
    if (idx >= (long)n_pos * half) return;
    const int i = (int)(idx % half), p = (int)(idx / half);
    const double theta = pow(base, -2.0 * (double)i / (double)(2 * half));
    double sn, cs;
    sincos((double)p * theta, &sn, &cs);
    table[idx] = make_float2((float)cs, (float)sn);
}

__global__ __launch_bounds__(256) void rope_kernel(bf16_t* __restrict__ x, long ld, int T, int n_heads, int d_head,
                                                   double base, int pos0, float sign,
                                                   const float2* __restrict__ table) {
    const int half = d_head >> 1;
    const int per_row = n_heads * (half >> 1);  // two pairs per thread
    const long idx = (long)blockIdx.x * blockDim.x + threadIdx.x;
    if (idx >= (long)T * per_row) return;
    const int t = (int)(idx / per_row);
    const int rem = (int)(idx % per_row);
    const int hd = rem / (half >> 1);
    const int i = (rem % (half >> 1)) * 2;
    bf16_t* p = x + (long)t * ld + (long)hd * d_head + i;
    uint32_t lo = *(uint32_t*)p, hi = *(uint32_t*)(p + half);
    float c[2], sn[2];
#pragma unroll
    for (int e = 0; e < 2; ++e) {
        if (table) {
            float2 cs = table[(long)(pos0 + t) * half + i + e];
            c[e] = cs.x; sn[e] = cs.y;
        } else {
            double theta = pow(base, -2.0 * (double)(i + e) / (double)d_head);
            double sd, cd;
            sincos((double)(pos0 + t) * theta, &sd, &cd);
            c[e] = (float)cd; sn[e] = (float)sd;
        }
        sn[e] *= sign;
    }
    float a0 = bf16_to_f32(lo & 0xffff), a1 = bf16_to_f32(lo >> 16);
    float b0 = bf16_to_f32(hi & 0xffff), b1 = bf16_to_f32(hi >> 16);
    *(uint32_t*)p = pack_bf16x2(a0 * c[0] - b0 * sn[0], a1 * c[1] - b1 * sn[1]);
    *(uint32_t*)(p + half) = pack_bf16x2(b0 * c[0] + a0 * sn[0], b1 * c[1] + a1 * sn[1]);
}

// The same with a table and 16-byte accesses: a thread rotates eight neighbouring pairs (columns i .. i+7 of a head
// with columns i + half .. i + half + 7).
__global__ __launch_bounds__(256) void rope_table_vec_kernel(bf16_t* __restrict__ x, long ld, int T, int n_heads,
                                                             int d_head, int pos0, float sign,
                                                             const float2* __restrict__ table) {
    // grid: x over the (head, eight-pair chunk) items of a row, y over rows
    const int half = d_head >> 1, per_head = half >> 3;
    const unsigned rem = blockIdx.x * blockDim.x + threadIdx.x;
    if (rem >= (unsigned)(n_heads * per_head)) return;
    const unsigned hd = rem / (unsigned)per_head, i = (rem - hd * per_head) * 8;
    for (long t = blockIdx.y; t < T; t += gridDim.y) {
        bf16_t* p = x + t * ld + (long)hd * d_head + i;
        float a[8], b[8], lo[8], hi[8];
        unpack8(*(const uint4*)p, a);
        unpack8(*(const uint4*)(p + half), b);
        const float4* cs4 = (const float4*)(table + (pos0 + t) * half + i);   // (cos, sin) pairs, two per float4
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const float4 w = cs4[e];
            const float s0 = w.y * sign, s1 = w.w * sign;
            lo[2 * e] = a[2 * e] * w.x - b[2 * e] * s0;
            hi[2 * e] = b[2 * e] * w.x + a[2 * e] * s0;
            lo[2 * e + 1] = a[2 * e + 1] * w.z - b[2 * e + 1] * s1;
            hi[2 * e + 1] = b[2 * e + 1] * w.z + a[2 * e + 1] * s1;
        }
        *(uint4*)p = pack8(lo);
        *(uint4*)(p + half) = pack8(hi);
    }
}

hipError_t launch_rope_table(float2* table, int n_pos, int d_head, float base, hipStream_t s) {
    const long n = (long)n_pos * (d_head / 2);
    if (n <= 0) return hipSuccess;
    rope_table_kernel<<<cdiv(n, 256), 256, 0, s>>>(table, n_pos, d_head / 2, (double)base);
    return hipGetLastError();
}
hipError_t launch_rope(bf16_t* x, long ld, int T, int n_heads, int d_head, float base, int pos0, int sign,
                       const float2* table, hipStream_t s) {
    const long n = (long)T * n_heads * (d_head / 4);
    if (n <= 0) return hipSuccess;
    if (table && (d_head & 15) == 0 && (ld & 7) == 0 && ((size_t)x & 15) == 0) {
        const dim3 grid(cdiv((long)n_heads * (d_head / 16), 256), T < 65535 ? T : 65535);
        rope_table_vec_kernel<<<grid, 256, 0, s>>>(x, ld, T, n_heads, d_head, pos0, sign >= 0 ? 1.f : -1.f, table);
        return hipGetLastError();
    }
    rope_kernel<<<cdiv(n, 256), 256, 0, s>>>(x, ld, T, n_heads, d_head, (double)base, pos0, sign >= 0 ? 1.f : -1.f,
                                             table);
    return hipGetLastError();
}

// ---------------------------------------------------------------- SwiGLU
// gu [T, 2f] = [gate | up];  a = gate * sigmoid(gate) * up
__global__ __launch_bounds__(256) void swiglu_fwd_kernel(const bf16_t* __restrict__ gu, int T, int f,
                                                         bf16_t* __restrict__ a) {
    // grid: x over the eight-column chunks of a row, y over rows (no index division per thread)
    const int c = (blockIdx.x * blockDim.x + threadIdx.x) * 8;
    if (c >= f) return;
    for (long t = blockIdx.y; t < T; t += gridDim.y) {
        float g[8], u[8], o[8];
        unpack8(*(const uint4*)(gu + t * 2 * f + c), g);
        unpack8(*(const uint4*)(gu + t * 2 * f + f + c), u);
#pragma unroll
        for (int e = 0; e < 8; ++e) o[e] = g[e] * __builtin_amdgcn_rcpf(1.f + __expf(-g[e])) * u[e];   // 1 ulp reciprocal: the result is rounded to bf16
        *(uint4*)(a + t * f + c) = pack8(o);
    }
}

// dgate = da * up * sig * (1 + gate (1 - sig));  dup = da * gate * sig
__global__ __launch_bounds__(256) void swiglu_bwd_kernel(const bf16_t* __restrict__ da, const bf16_t* __restrict__ gu,
                                                         int T, int f, bf16_t* __restrict__ dgu) {
    const int c = (blockIdx.x * blockDim.x + threadIdx.x) * 8;
    if (c >= f) return;
    for (long t = blockIdx.y; t < T; t += gridDim.y) {
        float g[8], u[8], d[8], dg[8], du[8];
        unpack8(*(const uint4*)(gu + t * 2 * f + c), g);
        unpack8(*(const uint4*)(gu + t * 2 * f + f + c), u);
        unpack8(*(const uint4*)(da + t * f + c), d);
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            float sg = __builtin_amdgcn_rcpf(1.f + __expf(-g[e]));
            dg[e] = d[e] * u[e] * sg * (1.f + g[e] * (1.f - sg));
            du[e] = d[e] * g[e] * sg;
        }
        *(uint4*)(dgu + t * 2 * f + c) = pack8(dg);
        *(uint4*)(dgu + t * 2 * f + f + c) = pack8(du);
    }
}

hipError_t launch_swiglu_fwd(const bf16_t* gu, int T, int f, bf16_t* a, hipStream_t s) {
    const long n = (long)T * (f / 8);
    if (n <= 0) return hipSuccess;
    swiglu_fwd_kernel<<<dim3(cdiv(f / 8, 256), T < 65535 ? T : 65535), 256, 0, s>>>(gu, T, f, a);
    return hipGetLastError();
}
hipError_t launch_swiglu_bwd(const bf16_t* da, const bf16_t* gu, int T, int f, bf16_t* dgu, hipStream_t s) {
    const long n = (long)T * (f / 8);
    if (n <= 0) return hipSuccess;
    swiglu_bwd_kernel<<<dim3(cdiv(f / 8, 256), T < 65535 ? T : 65535), 256, 0, s>>>(da, gu, T, f, dgu);
    return hipGetLastError();
}

// ---------------------------------------------------------------- embedding / labels
__global__ __launch_bounds__(256) void embed_kernel(const bf16_t* __restrict__ E, const int* __restrict__ tok, int d,
                                                    float* __restrict__ h) {
    const long t = blockIdx.x;
    const bf16_t* src = E + (long)tok[t] * d;
    float* dst = h + t * d;
    for (int i = threadIdx.x * 8; i < d; i += blockDim.x * 8) {
        float f[8];
        unpack8(*(const uint4*)(src + i), f);
        *(float4*)(dst + i) = make_float4(f[0], f[1], f[2], f[3]);
        *(float4*)(dst + i + 4) = make_float4(f[4], f[5], f[6], f[7]);
    }
}
hipError_t launch_embed(const bf16_t* E, const int* tokens, int T, int d, float* h, hipStream_t s) {
    if (T <= 0) return hipSuccess;
    embed_kernel<<<T, 256, 0, s>>>(E, tokens, d, h);
    return hipGetLastError();
}

// label[t] = tok[t + 1]; the last position has no label (-1)
__global__ void labels_kernel(const int* __restrict__ tok, int T, int* __restrict__ labels) {
    const int t = blockIdx.x * blockDim.x + threadIdx.x;
    if (t < T) labels[t] = (t + 1 < T) ? tok[t + 1] : -1;
}
hipError_t launch_labels(const int* tokens, int T, int* labels, hipStream_t s) {
    if (T <= 0) return hipSuccess;
    labels_kernel<<<cdiv(T, 256), 256, 0, s>>>(tokens, T, labels);
    return hipGetLastError();
}

// ---------------------------------------------------------------- fused softmax cross-entropy
// One block per position.  Pass 1: online max / sum-exp over the vocabulary; pass 2 (targets only):
// dlogits = (softmax - onehot) / n_targets.  Non-target rows get nll = 0 and zero gradient.
__global__ __launch_bounds__(512) void cross_entropy_kernel(const float* __restrict__ logits,
                                                            const int* __restrict__ labels, int T, int V,
                                                            int first_target, float inv_n, float* __restrict__ nll,
                                                            bf16_t* __restrict__ dlogits, int row0) {
    __shared__ float red[16];
    const int t = blockIdx.x + row0;
    const float* z = logits + (long)t * V;
    bf16_t* dz = dlogits ? dlogits + (long)t * V : nullptr;
    const bool target = (t >= first_target) && (t < T - 1);
    if (!target) {
        if (threadIdx.x == 0) nll[t] = 0.f;
        if (dz) for (int i = threadIdx.x; i < V; i += blockDim.x) dz[i] = 0;
        return;
    }
    float m = -INFINITY, ssum = 0.f;
    for (int i = threadIdx.x; i < V; i += blockDim.x) {
        float x = z[i];
        if (x > m) { ssum *= __expf(m - x); m = x; }
        ssum += __expf(x - m);
    }
    const float M = block_max(m, red);
    ssum = block_sum(ssum * __expf(m - M), red);
    const float lse = M + logf(ssum);
    const int lab = labels[t];
    if (threadIdx.x == 0) nll[t] = lse - z[lab];
    if (dz) {
        for (int i = threadIdx.x; i < V; i += blockDim.x) {
            float p = __expf(z[i] - lse);
            if (i == lab) p -= 1.f;
            dz[i] = f32_to_bf16(p * inv_n);
        }
    }
}
// deterministic sum of nll over the call's positions (one block); flag (may be null) receives 0 if the sum is finite,
// 1 otherwise: the optimizer launches of the same update read it and leave the module untouched when it is set
__global__ __launch_bounds__(256) void nll_sum_kernel(const float* __restrict__ nll, int T, float* __restrict__ out,
                                                      int* __restrict__ flag) {
    __shared__ float red[16];
    float s = 0.f;
    for (int i = threadIdx.x; i < T; i += blockDim.x) s += nll[i];
    s = block_sum(s, red);
    if (threadIdx.x == 0) {
        out[0] = s;
        if (flag) flag[0] = isfinite(s) ? 0 : 1;
    }
}
// row0: rows below it are conditioning positions the caller knows carry no loss: their nll is set to 0 and their
// logits / dlogits rows are neither read nor written (the caller does not compute or use them).
hipError_t launch_cross_entropy(const float* logits, const int* labels, int T, int V, int first_target,
                                int n_targets, float* nll, bf16_t* dlogits, float* loss_sum, hipStream_t s, int row0,
                                int* flag) {
    if (T <= 0) return hipSuccess;
    if (row0 < 0 || row0 > first_target || row0 >= T) return hipErrorInvalidValue;
    if (row0 > 0) {
        hipError_t e = launch_fill_f32(nll, (size_t)row0, 0.f, s);
        if (e != hipSuccess) return e;
    }
    cross_entropy_kernel<<<T - row0, 512, 0, s>>>(logits, labels, T, V, first_target, 1.f / (float)n_targets, nll, dlogits,
                                                  row0);
    if (loss_sum) nll_sum_kernel<<<1, 256, 0, s>>>(nll, T, loss_sum, flag);
    return hipGetLastError();
}

// ---------------------------------------------------------------- fused AdamW
// Decoupled weight decay, bias correction, epsilon added after the corrected square root.
__global__ __launch_bounds__(256) void adamw_kernel(float* __restrict__ p, const float* __restrict__ g,
                                                    float* __restrict__ m, float* __restrict__ v,
                                                    bf16_t* __restrict__ shadow, size_t n4, size_t n, float lr,
                                                    float b1, float b2, float eps, float decay, float inv_bc1,
                                                    float inv_bc2, const int* __restrict__ skip_flag) {
    if (skip_flag && *skip_flag != 0) return;   // the update was found invalid (non-finite loss or gradient): change nothing
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    // two independent groups of four per trip: eight 16-byte loads are in flight before the first one is used
    for (size_t i0 = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i0 < n4; i0 += 2 * stride) {
        const size_t i1 = i0 + stride;
        const bool two = i1 < n4;
        const size_t ii[2] = {i0, two ? i1 : i0};
        float4 P[2], G[2], Mm[2], Vv[2];
#pragma unroll
        for (int k = 0; k < 2; ++k) {
            P[k] = ((float4*)p)[ii[k]]; G[k] = ((const float4*)g)[ii[k]];
            Mm[k] = ((float4*)m)[ii[k]]; Vv[k] = ((float4*)v)[ii[k]];
        }
#pragma unroll
        for (int k = 0; k < 2; ++k) {
            if (k == 1 && !two) break;
            float pp[4] = {P[k].x, P[k].y, P[k].z, P[k].w}, gg[4] = {G[k].x, G[k].y, G[k].z, G[k].w};
            float mm[4] = {Mm[k].x, Mm[k].y, Mm[k].z, Mm[k].w}, vv[4] = {Vv[k].x, Vv[k].y, Vv[k].z, Vv[k].w};
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                pp[e] *= decay;
                mm[e] = b1 * mm[e] + (1.f - b1) * gg[e];
                vv[e] = b2 * vv[e] + (1.f - b2) * gg[e] * gg[e];
                pp[e] -= lr * (mm[e] * inv_bc1) / (sqrtf(vv[e] * inv_bc2) + eps);
            }
            const size_t i = ii[k];
            ((float4*)p)[i] = make_float4(pp[0], pp[1], pp[2], pp[3]);
            ((float4*)m)[i] = make_float4(mm[0], mm[1], mm[2], mm[3]);
            ((float4*)v)[i] = make_float4(vv[0], vv[1], vv[2], vv[3]);
            if (shadow) {
                uint2 b;
                b.x = pack_bf16x2(pp[0], pp[1]);
                b.y = pack_bf16x2(pp[2], pp[3]);
                ((uint2*)shadow)[i] = b;
            }
        }
    }
    // tail (n not a multiple of 4)
    if (blockIdx.x == 0) {
        for (size_t i = n4 * 4 + threadIdx.x; i < n; i += blockDim.x) {
            float pp = p[i] * decay, gg = g[i];
            float mm = b1 * m[i] + (1.f - b1) * gg;
            float vv = b2 * v[i] + (1.f - b2) * gg * gg;
            pp -= lr * (mm * inv_bc1) / (sqrtf(vv * inv_bc2) + eps);
            p[i] = pp; m[i] = mm; v[i] = vv;
            if (shadow) shadow[i] = f32_to_bf16(pp);
        }
    }
}
hipError_t launch_adamw(float* p, const float* g, float* m, float* v, bf16_t* shadow, size_t n, long step, float lr,
                        float beta1, float beta2, float eps, float wd, hipStream_t s, const int* skip_flag) {
    if (n == 0) return hipSuccess;
    const double bc1 = 1.0 - pow((double)beta1, (double)step);
    const double bc2 = 1.0 - pow((double)beta2, (double)step);
    const size_t n4 = n / 4;
    size_t blocks = (n4 + 255) / 256;
    if (blocks > 256 * 16) blocks = 256 * 16;
    if (blocks < 1) blocks = 1;
    adamw_kernel<<<(unsigned)blocks, 256, 0, s>>>(p, g, m, v, shadow, n4, n, lr, beta1, beta2, eps, 1.f - lr * wd,
                                                  (float)(1.0 / bc1), (float)(1.0 / bc2), skip_flag);
    return hipGetLastError();
}

// ---------------------------------------------------------------- conversions / fills / init
__global__ void f32_to_bf16_kernel(const float* __restrict__ src, bf16_t* __restrict__ dst, size_t n) {
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += stride) dst[i] = f32_to_bf16(src[i]);
}
hipError_t launch_f32_to_bf16(const float* src, bf16_t* dst, size_t n, hipStream_t s) {
    if (n == 0) return hipSuccess;
    size_t blocks = (n + 255) / 256;
    if (blocks > 8192) blocks = 8192;
    f32_to_bf16_kernel<<<(unsigned)blocks, 256, 0, s>>>(src, dst, n);
    return hipGetLastError();
}
__global__ void fill_f32_kernel(float* __restrict__ p, size_t n, float v) {
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += stride) p[i] = v;
}
// n bf16 zeros (n a multiple of 2, p 4-byte aligned): a fill kernel rather than a memset node, so that the path stays
// capturable in a HIP graph
__global__ void zero_u32_kernel(uint32_t* __restrict__ p, size_t n) {
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += stride) p[i] = 0u;
}
hipError_t launch_fill_bf16_zero(bf16_t* p, size_t n, hipStream_t s) {
    if (n == 0) return hipSuccess;
    if ((n & 1) || ((size_t)p & 3)) return hipErrorInvalidValue;
    size_t blocks = (n / 2 + 255) / 256;
    if (blocks > 8192) blocks = 8192;
    zero_u32_kernel<<<(unsigned)blocks, 256, 0, s>>>((uint32_t*)p, n / 2);
    return hipGetLastError();
}
hipError_t launch_fill_f32(float* p, size_t n, float value, hipStream_t s) {
    if (n == 0) return hipSuccess;
    size_t blocks = (n + 255) / 256;
    if (blocks > 8192) blocks = 8192;
    fill_f32_kernel<<<(unsigned)blocks, 256, 0, s>>>(p, n, value);
    return hipGetLastError();
}

// Counter-based normal draws for the initial A factors: a 64-bit mix of (seed, stream, index)
// gives two uniforms, Box-Muller gives the value.  Element i depends only on (seed, stream, i).
__host__ __device__ __forceinline__ uint64_t mix64(uint64_t z) {
    z += 0x9E3779B97F4A7C15ull;
    z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
    z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
    return z ^ (z >> 31);
}
__global__ void init_normal_kernel(float* __restrict__ p, size_t n, float std, uint64_t seed, uint64_t stream_id) {
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += stride) {
        uint64_t r = mix64(mix64(seed ^ mix64(stream_id)) + i);
        float u1 = ((float)(uint32_t)(r >> 40) + 1.0f) * (1.0f / 16777217.0f);  // (0, 1)
        float u2 = (float)(uint32_t)((r >> 8) & 0xffffffu) * (1.0f / 16777216.0f);
        p[i] = std * sqrtf(-2.f * logf(u1)) * cosf(6.283185307179586f * u2);
    }
}
hipError_t launch_init_normal(float* p, size_t n, float std, uint64_t seed, uint64_t stream_id, hipStream_t s) {
    if (n == 0) return hipSuccess;
    size_t blocks = (n + 255) / 256;
    if (blocks > 8192) blocks = 8192;
    init_normal_kernel<<<(unsigned)blocks, 256, 0, s>>>(p, n, std, seed, stream_id);
    return hipGetLastError();
}

// ---------------------------------------------------------------- LoRA dropout (Section 3 "Setup": dropout = 0.05)
// Dropout sits on the input of the low-rank branch only: Y = X W^T + s (D o X) A^T B^T with D = 0 (dropped) or
// 1 / (1 - p) (kept).  One mask per projection group input (q|k|v share theirs, gate|up theirs).  The mask is a pure
// function of (seed, optimizer step, layer, group, element): element e = t * d_in + c is kept iff the upper 32 bits of
// mix64(key + e) are >= floor(p * 2^32), with key = mix64(seed ^ mix64(2^63 | step << 16 | layer << 3 | group)); the top
// bit keeps these streams apart from the ones that draw the initial A.
uint64_t dropout_key(uint64_t seed, int64_t step, int layer, int group) {
    const uint64_t stream_id = (1ull << 63) | ((uint64_t)step << 16) | ((uint64_t)layer << 3) | (uint64_t)group;
    return mix64(seed ^ mix64(stream_id));
}
uint32_t dropout_threshold(float p) {
    const double t = floor((double)p * 4294967296.0);
    return t <= 0.0 ? 0u : (t >= 4294967295.0 ? 4294967295u : (uint32_t)t);
}
__device__ __forceinline__ bool dropout_keep(uint64_t key, uint64_t e, uint32_t thr) {
    return (uint32_t)(mix64(key + e) >> 32) >= thr;
}
// y = D o x, eight elements per thread
__global__ __launch_bounds__(256) void dropout_fwd_kernel(const bf16_t* __restrict__ x, bf16_t* __restrict__ y, size_t n8,
                                                          uint64_t key, uint32_t thr, float scale) {
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n8; i += stride) {
        float v[8];
        unpack8(*(const uint4*)(x + i * 8), v);
#pragma unroll
        for (int e = 0; e < 8; ++e) v[e] = dropout_keep(key, i * 8 + e, thr) ? v[e] * scale : 0.f;
        *(uint4*)(y + i * 8) = pack8(v);
    }
}
// dx += D o z   (the low-rank branch's share of the input gradient)
__global__ __launch_bounds__(256) void dropout_add_kernel(bf16_t* __restrict__ dx, const float* __restrict__ z, size_t n8,
                                                          uint64_t key, uint32_t thr, float scale) {
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n8; i += stride) {
        float v[8];
        unpack8(*(const uint4*)(dx + i * 8), v);
        const float4 z0 = *(const float4*)(z + i * 8), z1 = *(const float4*)(z + i * 8 + 4);
        const float zz[8] = {z0.x, z0.y, z0.z, z0.w, z1.x, z1.y, z1.z, z1.w};
#pragma unroll
        for (int e = 0; e < 8; ++e)
            if (dropout_keep(key, i * 8 + e, thr)) v[e] += zz[e] * scale;
        *(uint4*)(dx + i * 8) = pack8(v);
    }
}
static unsigned dropout_blocks(size_t n8) {
    size_t b = (n8 + 255) / 256;
    return (unsigned)(b > 16384 ? 16384 : b);
}
hipError_t launch_dropout_fwd(const bf16_t* x, bf16_t* y, size_t n, uint64_t key, float p, hipStream_t s) {
    if (n == 0) return hipSuccess;
    if ((n & 7) || !(p >= 0.f && p < 1.f)) return hipErrorInvalidValue;
    dropout_fwd_kernel<<<dropout_blocks(n / 8), 256, 0, s>>>(x, y, n / 8, key, dropout_threshold(p), 1.f / (1.f - p));
    return hipGetLastError();
}
hipError_t launch_dropout_add(bf16_t* dx, const float* z, size_t n, uint64_t key, float p, hipStream_t s) {
    if (n == 0) return hipSuccess;
    if ((n & 7) || !(p >= 0.f && p < 1.f)) return hipErrorInvalidValue;
    dropout_add_kernel<<<dropout_blocks(n / 8), 256, 0, s>>>(dx, z, n / 8, key, dropout_threshold(p), 1.f / (1.f - p));
    return hipGetLastError();
}

// ---------------------------------------------------------------- transposes / copies
// 64x64 bf16 tiles through LDS.  With everything a multiple of 8 elements (every LoRA factor is) a thread moves 16-byte
// pieces on both sides of the turn; otherwise element by element.  tile: TR_TILE_ELEMS elements, 16-byte aligned.
constexpr int TR_LD = 72;                    // LDS row stride: 144 bytes, so that a row starts on a 16-byte boundary
constexpr int TR_TILE_ELEMS = 64 * TR_LD;
__device__ __forceinline__ void transpose_tile(const bf16_t* __restrict__ src, long lds, int rows, int cols,
                                               bf16_t* __restrict__ dst, long ldd, int tr, int tc, bf16_t* tile) {
    const int r0 = tr * 64, c0 = tc * 64;
    const bool vec = !((lds | ldd | rows | cols) & 7) && !(((size_t)src | (size_t)dst) & 15);
    if (vec) {
        for (int i = threadIdx.x; i < 64 * 8; i += blockDim.x) {
            const int r = i >> 3, c8 = (i & 7) * 8;
            uint4 v = make_uint4(0, 0, 0, 0);
            if (r0 + r < rows && c0 + c8 < cols) v = *(const uint4*)(src + (long)(r0 + r) * lds + c0 + c8);
            *(uint4*)(tile + r * TR_LD + c8) = v;
        }
        __syncthreads();
        for (int i = threadIdx.x; i < 64 * 8; i += blockDim.x) {
            const int c = i >> 3, r8 = (i & 7) * 8;
            if (c0 + c >= cols || r0 + r8 >= rows) continue;
            uint32_t w[4];
#pragma unroll
            for (int e = 0; e < 4; ++e)
                w[e] = (uint32_t)tile[(r8 + 2 * e) * TR_LD + c] | ((uint32_t)tile[(r8 + 2 * e + 1) * TR_LD + c] << 16);
            *(uint4*)(dst + (long)(c0 + c) * ldd + r0 + r8) = make_uint4(w[0], w[1], w[2], w[3]);
        }
        return;
    }
    for (int i = threadIdx.x; i < 64 * 64; i += blockDim.x) {
        const int r = i >> 6, c = i & 63;
        bf16_t v = 0;
        if (r0 + r < rows && c0 + c < cols) v = src[(long)(r0 + r) * lds + c0 + c];
        tile[r * TR_LD + c] = v;
    }
    __syncthreads();
    for (int i = threadIdx.x; i < 64 * 64; i += blockDim.x) {
        const int c = i >> 6, r = i & 63;
        if (r0 + r < rows && c0 + c < cols) dst[(long)(c0 + c) * ldd + r0 + r] = tile[r * TR_LD + c];
    }
}
__global__ __launch_bounds__(256) void transpose_kernel(const bf16_t* __restrict__ src, long lds, int rows, int cols,
                                                        bf16_t* __restrict__ dst, long ldd) {
    __shared__ __align__(16) bf16_t tile[TR_TILE_ELEMS];
    transpose_tile(src, lds, rows, cols, dst, ldd, blockIdx.y, blockIdx.x, tile);
}
hipError_t launch_transpose_bf16(const bf16_t* src, long lds, int rows, int cols, bf16_t* dst, long ldd,
                                 hipStream_t s) {
    if (rows <= 0 || cols <= 0) return hipSuccess;
    dim3 grid(cdiv(cols, 64), cdiv(rows, 64));
    transpose_kernel<<<grid, 256, 0, s>>>(src, lds, rows, cols, dst, ldd);
    return hipGetLastError();
}
__global__ __launch_bounds__(256) void transpose_table_kernel(const bf16_t* __restrict__ src_base,
                                                              bf16_t* __restrict__ dst_base,
                                                              const TransposeDesc* __restrict__ tab, int n_desc,
                                                              int tile_begin) {
    __shared__ __align__(16) bf16_t tile[TR_TILE_ELEMS];
    // binary search for the descriptor whose tile range holds this block
    int lo = 0, hi = n_desc - 1;
    const int b = blockIdx.x + tile_begin;
    while (lo < hi) {
        int mid = (lo + hi + 1) >> 1;
        if (tab[mid].tile0 <= b) lo = mid; else hi = mid - 1;
    }
    const TransposeDesc d = tab[lo];
    const int local = b - d.tile0;
    const int tiles_c = (d.cols + 63) >> 6;
    transpose_tile(src_base + d.src_off, d.lds, d.rows, d.cols, dst_base + d.dst_off, d.ldd, local / tiles_c,
                   local % tiles_c, tile);
}
// tiles [tile_begin, tile_begin + n_tiles) of the table's tile numbering
hipError_t launch_transpose_table(const bf16_t* src_base, bf16_t* dst_base, const TransposeDesc* table_dev,
                                  int n_desc, int n_tiles, hipStream_t s, int tile_begin) {
    if (n_desc <= 0 || n_tiles <= 0) return hipSuccess;
    transpose_table_kernel<<<n_tiles, 256, 0, s>>>(src_base, dst_base, table_dev, n_desc, tile_begin);
    return hipGetLastError();
}
__global__ void copy2d_kernel(const bf16_t* __restrict__ src, long lds, int rows, int cols8, bf16_t* __restrict__ dst,
                              long ldd) {
    const long idx = (long)blockIdx.x * blockDim.x + threadIdx.x;
    if (idx >= (long)rows * cols8) return;
    const long r = idx / cols8;
    const int c = (int)(idx % cols8) * 8;
    *(uint4*)(dst + r * ldd + c) = *(const uint4*)(src + r * lds + c);
}
hipError_t launch_copy2d_bf16(const bf16_t* src, long lds, int rows, int cols, bf16_t* dst, long ldd, hipStream_t s) {
    const long n = (long)rows * (cols / 8);
    if (n <= 0) return hipSuccess;
    copy2d_kernel<<<cdiv(n, 256), 256, 0, s>>>(src, lds, rows, cols / 8, dst, ldd);
    return hipGetLastError();
}
