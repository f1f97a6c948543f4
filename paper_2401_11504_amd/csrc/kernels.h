// Internal launch interface between the host orchestration and the gfx950 kernels.
#pragma once
#include "common.h"

// ---------------------------------------------------------------- GEMM (gemm_bf16.hip)
// C = alpha * (A B^T + A2 B2^T) (+ R), bf16 operands, fp32 accumulate (MFMA 32x32x16).
struct GemmNT {
    const bf16_t* A = nullptr;  long lda = 0;   // [M, K]
    const bf16_t* B = nullptr;  long ldb = 0;   // [N, K]
    int M = 0, N = 0, K = 0;
    const bf16_t* A2 = nullptr; long lda2 = 0;  // [M, K2]  (low-rank K-extension; may be null)
    const bf16_t* B2 = nullptr; long ldb2 = 0;  // [N, K2]
    int K2 = 0;
    float alpha = 1.f;
    const float* R = nullptr;                   // fp32 [M, N] residual (c_f32 only), row stride ldc
    void* C = nullptr;          long ldc = 0;   // bf16 or fp32 [M, N]
    int c_f32 = 0;
    int batch = 1;                              // grid.z; element offsets applied per batch index:
    long bA = 0, bB = 0, bA2 = 0, bB2 = 0, bC = 0;
    int split_k = 0;                            // 0 = choose; >1 needs `partial`
    float* partial = nullptr;                   // fp32 scratch, >= batch*split*M*N elements
    size_t partial_elems = 0;
    // If set (batch must be 1, alpha 1): when the launcher splits the contraction of a wide-output GEMM it leaves the
    // fp32 partial tiles in `partial` ([n_split][M][N]), does not write C (nor add R), and stores n_split here, so that
    // the consumer can add them up itself instead of a reduce pass; otherwise 0 is stored and C is written.
    int* deferred = nullptr;
    // With `deferred`: the partial tiles left for the consumer are bf16 (the same [n_split][M][N] layout over the same
    // scratch, half the bytes written here and read there; each partial is rounded once) instead of fp32.
    int partial_bf16 = 0;
};
hipError_t launch_gemm_nt(const GemmNT& g, hipStream_t s);
// name of the tile configuration launch_gemm_nt picks for g (a static string) and the contraction split it uses
const char* gemm_nt_plan(const GemmNT& g, int* n_split);
// N1 > 0: cheaper as two launches, columns [0, N1) and [N1, N) of every batch (see gemm_bf16.hip); 0: one launch
int gemm_nt_column_split(const GemmNT& g);
bool gemm_nt_split_columns(const GemmNT& g, GemmNT* a, GemmNT* b);   // the two launches, if N1 > 0

// C[Mo, No] (fp32) = alpha * P[T, Mo]^T Q[T, No]
struct GemmTN {
    const bf16_t* P = nullptr; long ldp = 0;
    const bf16_t* Q = nullptr; long ldq = 0;
    int T = 0, Mo = 0, No = 0;
    float alpha = 1.f;
    float* C = nullptr; long ldc = 0;
    int batch = 1;
    long bP = 0, bQ = 0, bC = 0;
    float* partial = nullptr;                   // optional scratch for splitting the token dimension
    size_t partial_elems = 0;
};
hipError_t launch_gemm_tn(const GemmTN& g, hipStream_t s);

// Up to TN_GROUP_MAX products C_k[Mo_k, No_k] (fp32) = P_k[T, Mo_k]^T Q_k[T, No_k] over the same T tokens in one
// launch (the dA and dB of every projection of a decoder layer).  tile0 is filled in by the launcher.
constexpr int TN_GROUP_MAX = 12;
struct TnProblem {
    const bf16_t* P = nullptr; const bf16_t* Q = nullptr; float* C = nullptr;
    long ldp = 0, ldq = 0, ldc = 0;
    int Mo = 0, No = 0, tile0 = 0, pad = 0;
};
struct GemmTNGroup {
    TnProblem p[TN_GROUP_MAX];
    int n = 0, T = 0;
    int* flag = nullptr;   // if set: bit 1 of *flag is raised when any product entry is not finite
    void add(const bf16_t* P, long ldp, int Mo, const bf16_t* Q, long ldq, int No, float* C, long ldc) {
        if (n < TN_GROUP_MAX) { TnProblem& q = p[n]; q.P = P; q.ldp = ldp; q.Mo = Mo; q.Q = Q; q.ldq = ldq; q.No = No; q.C = C; q.ldc = ldc; }
        ++n;
    }
};
hipError_t launch_gemm_tn_grouped(GemmTNGroup& g, hipStream_t s);

// fp32 reference-precision GEMM for the single-layer fp32 step: C = alpha * op(A) op(B) + beta * C
// ta/tb: 0 = as stored [rows, cols] row-major, 1 = transposed use.  (gemm_f32.hip)
hipError_t launch_sgemm(int ta, int tb, int M, int N, int K, float alpha, const float* A, int lda, const float* B,
                        int ldb, float beta, float* C, int ldc, hipStream_t s);

// ---------------------------------------------------------------- attention (attention.hip)
hipError_t launch_attention_fwd(const bf16_t* q, const bf16_t* k, const bf16_t* v, long ldq, int T, int n_heads,
                                int d_head, bf16_t* o, long ldo, float* lse, hipStream_t s);
hipError_t launch_attention_bwd(const bf16_t* q, const bf16_t* k, const bf16_t* v, const bf16_t* o, const bf16_t* d_o,
                                const float* lse, long ldq, long ldo, int T, int n_heads, int d_head, bf16_t* dq,
                                bf16_t* dk, bf16_t* dv, float* delta, const float2* rope, hipStream_t s);

// ---------------------------------------------------------------- elementwise / reductions (elementwise.hip)
// part != null: the input row is not read from h but formed as the sum of n_part fp32 arrays [T, d] lying part_stride
// elements apart plus resid (may be null), and written to h_write (the residual stream) on the way.
hipError_t launch_rmsnorm_fwd(const float* h, const float* g, int T, int d, float eps, bf16_t* y, hipStream_t s,
                              const float* part = nullptr, int n_part = 0, long part_stride = 0,
                              const float* resid = nullptr, float* h_write = nullptr);
// dy_part != null: dy is the sum of n_part fp32 arrays [T, d] that lie part_stride elements apart (the partial tiles a
// split GEMM left behind, see GemmNT::deferred); the bf16 dy is then not read.
hipError_t launch_rmsnorm_bwd(const bf16_t* dy, const float* h, const float* g, const float* dres, int T, int d,
                              float eps, float* dh_out, bf16_t* dh_bf, hipStream_t s, const float* dy_part = nullptr,
                              int n_part = 0, long part_stride = 0, int part_bf16 = 0);
hipError_t launch_rope(bf16_t* x, long ld, int T, int n_heads, int d_head, float base, int pos0, int sign,
                       const float2* table, hipStream_t s);
hipError_t launch_rope_table(float2* table, int n_pos, int d_head, float base, hipStream_t s);
hipError_t launch_swiglu_fwd(const bf16_t* gu, int T, int f, bf16_t* a, hipStream_t s);
hipError_t launch_swiglu_bwd(const bf16_t* da, const bf16_t* gu, int T, int f, bf16_t* dgu, hipStream_t s);
hipError_t launch_cross_entropy(const float* logits, const int* labels, int T, int V, int first_target,
                                int n_targets, float* nll, bf16_t* dlogits, float* loss_sum, hipStream_t s, int row0 = 0,
                                int* flag = nullptr);
hipError_t launch_adamw(float* p, const float* g, float* m, float* v, bf16_t* shadow, size_t n, long step, float lr,
                        float beta1, float beta2, float eps, float wd, hipStream_t s, const int* skip_flag = nullptr);
hipError_t launch_embed(const bf16_t* E, const int* tokens, int T, int d, float* h, hipStream_t s);
hipError_t launch_labels(const int* tokens, int T, int* labels, hipStream_t s);
hipError_t launch_f32_to_bf16(const float* src, bf16_t* dst, size_t n, hipStream_t s);
hipError_t launch_fill_f32(float* p, size_t n, float value, hipStream_t s);
hipError_t launch_fill_bf16_zero(bf16_t* p, size_t n, hipStream_t s);
hipError_t launch_init_normal(float* p, size_t n, float std, uint64_t seed, uint64_t stream_id, hipStream_t s);
// LoRA dropout: the mask is a function of (key, element index); key from (seed, optimizer step, layer, group)
uint64_t dropout_key(uint64_t seed, int64_t step, int layer, int group);
hipError_t launch_dropout_fwd(const bf16_t* x, bf16_t* y, size_t n, uint64_t key, float p, hipStream_t s);
hipError_t launch_dropout_add(bf16_t* dx, const float* z, size_t n, uint64_t key, float p, hipStream_t s);
// dst[c, r] = src[r, c] for a [rows, cols] bf16 matrix with row strides lds / ldd
hipError_t launch_transpose_bf16(const bf16_t* src, long lds, int rows, int cols, bf16_t* dst, long ldd,
                                 hipStream_t s);
// many transposes in one launch: descriptors live in device memory
struct TransposeDesc { long src_off, dst_off; int rows, cols, lds, ldd, tile0, pad; };
hipError_t launch_transpose_table(const bf16_t* src_base, bf16_t* dst_base, const TransposeDesc* table_dev,
                                  int n_desc, int n_tiles, hipStream_t s, int tile_begin = 0);
// copy rows [rows, cols] bf16 from src (stride lds) to dst (stride ldd)
hipError_t launch_copy2d_bf16(const bf16_t* src, long lds, int rows, int cols, bf16_t* dst, long ldd, hipStream_t s);

// ---------------------------------------------------------------- one-token decoding (decode.hip)
// y[N] = alpha * (W[N, K] x[K] + sum_j lora_b[n, j] lora_h[(n / rows_per_group) r + j]) (+ resid, fp32 output only)
// Where a matrix-vector product takes its input vector from (see gemv_kernel)
struct GemvPre {
    int mode = 0;                 // 0: x as given; 1: RMSNorm of h with gain; 2: SwiGLU of the gate|up row gu
    const float* h = nullptr;
    const float* gain = nullptr;
    float eps = 0.f;
    const bf16_t* gu = nullptr;
    bf16_t* x_out = nullptr;      // if set, workgroup 0 stores the input vector it formed
};
hipError_t launch_gemv(const bf16_t* W, long ldw, const bf16_t* x, int N, int K, const bf16_t* lora_b, const float* lora_h,
                       int r, int rows_per_group, float alpha, const float* resid, bf16_t* y_bf, float* y_f32,
                       hipStream_t s, const GemvPre* pre = nullptr);
// one query row against cache rows 0 .. n_keys-1 (row stride ld), per head
constexpr int ATTN_DECODE_MAX_SPLIT = 32;   // key ranges per head in the split decode-attention path
hipError_t launch_attention_decode(const bf16_t* q, bf16_t* k, const bf16_t* v, long ld, int n_keys, int n_heads,
                                   int d_head, bf16_t* o, float* ws, size_t ws_elems, hipStream_t s,
                                   const float2* rope_row = nullptr);
// index of the largest of n floats, lowest index among equals
hipError_t launch_argmax(const float* x, int n, int* out, hipStream_t s);
