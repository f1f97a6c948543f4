// Host side of the Temp-Lora chunk-update library: C ABI, memory ownership and the
// order in which the gfx950 kernels run.  See include/templora.h for the contract.
#include "../../include/templora.h"
#include "kernels.h"

#include <cmath>
#include <cstdarg>
#include <cstdio>
#include <cstring>
#include <mutex>
#include <new>
#include <vector>

// ---------------------------------------------------------------- errors
static thread_local char g_err[512] = "";
static tl_status fail(tl_status st, const char* fmt, ...) {
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof(g_err), fmt, ap);
    va_end(ap);
    return st;
}
#define HIPCHK(expr)                                                                              \
    do {                                                                                          \
        hipError_t e__ = (expr);                                                                  \
        if (e__ != hipSuccess)                                                                    \
            return fail(e__ == hipErrorOutOfMemory ? TL_ERR_OOM : TL_ERR_DEVICE, "%s: %s (%s:%d)", #expr, \
                        hipGetErrorString(e__), __FILE__, __LINE__);                              \
    } while (0)
#define TLCHK(expr)                      \
    do {                                 \
        tl_status s__ = (expr);          \
        if (s__ != TL_OK) return s__;    \
    } while (0)

extern "C" const char* tl_last_error(void) { return g_err; }
extern "C" const char* tl_version(void) { return "templora-gfx950 0.1"; }

static tl_status require_gfx950() {
    int n = 0;
    if (hipGetDeviceCount(&n) != hipSuccess || n < 1) {
        (void)hipGetLastError();
        return fail(TL_ERR_DEVICE, "no HIP device: this library has no CPU fallback");
    }
    int dev = 0;
    HIPCHK(hipGetDevice(&dev));
    hipDeviceProp_t prop;
    HIPCHK(hipGetDeviceProperties(&prop, dev));
    if (strncmp(prop.gcnArchName, "gfx950", 6) != 0)
        return fail(TL_ERR_DEVICE, "device %d is %s; kernels are built for gfx950 only", dev, prop.gcnArchName);
    return TL_OK;
}

// ---------------------------------------------------------------- device memory bookkeeping
struct Pool {
    std::vector<void*> ptrs;
    template <typename T>
    tl_status alloc(T** out, size_t n_elems) {
        void* p = nullptr;
        size_t bytes = n_elems * sizeof(T);
        if (bytes == 0) bytes = 16;
        hipError_t e = hipMalloc(&p, bytes);
        if (e != hipSuccess) {
            (void)hipGetLastError();
            return fail(TL_ERR_OOM, "hipMalloc of %zu bytes failed: %s", bytes, hipGetErrorString(e));
        }
        ptrs.push_back(p);
        *out = (T*)p;
        return TL_OK;
    }
    void release() {
        for (void* p : ptrs) (void)hipFree(p);
        ptrs.clear();
    }
};

// projection groups that share an input: q|k|v, o, gate|up, down
enum { G_QKV = 0, G_O = 1, G_GU = 2, G_DOWN = 3, N_GROUPS = 4 };
static const int kGroupCount[N_GROUPS] = {3, 1, 2, 1};
static const int kProjGroup[7] = {G_QKV, G_QKV, G_QKV, G_O, G_GU, G_GU, G_DOWN};
static const int kProjIndex[7] = {0, 1, 2, 0, 0, 1, 0};

struct LayerW {
    bf16_t* w[N_GROUPS];   // packed [G*d_out, d_in]
    bf16_t* wt[N_GROUPS];  // transposed [d_in, G*d_out]
    float *g1, *g2;
};

struct tl_model {
    tl_model_cfg cfg;
    hipStream_t stream;
    int device;
    Pool pool;
    std::vector<LayerW> layers;
    bf16_t *emb = nullptr, *head = nullptr, *head_t = nullptr;
    float* gf = nullptr;
    float2* rope = nullptr;
    int d_in(int g) const { return g == G_DOWN ? cfg.d_ffn : cfg.d_model; }
    int d_out(int g) const { return g == G_GU ? cfg.d_ffn : cfg.d_model; }
};

struct LayerOff {           // element offsets into the LoRA arenas
    size_t A[N_GROUPS], B[N_GROUPS];    // fp32 arenas and same-layout bf16 shadow
    size_t AT[N_GROUPS], BT[N_GROUPS];  // transposed bf16 shadows
};

struct LayerSave {          // activations kept from forward to backward
    bf16_t *x1, *qkv, *o, *x2, *gu, *act, *hs[N_GROUPS];
    bf16_t* xd[N_GROUPS] = {};   // dropped copy of each group's input (only with dropout > 0)
    float *lse, *hmid;
};

struct tl_lora {
    tl_model* model = nullptr;
    tl_lora_cfg cfg;
    bool discarded = false;
    int64_t step = 0;
    int last_tokens = 0;
    bool have_grads = false;
    float s = 1.f;
    Pool pool;
    size_t n_params = 0, n_t = 0;
    float *P = nullptr, *G = nullptr, *M = nullptr, *V = nullptr;
    bf16_t *S = nullptr, *ST = nullptr;
    std::vector<LayerOff> off;
    TransposeDesc* ttable = nullptr;
    int n_desc = 0, total_tiles = 0;
    std::vector<int> layer_tile0;     // first tile of each layer in the table's numbering (and the total at [n_layers])
    // During tl_chunk_update the AdamW step of a layer (and the refresh of its transposed shadows) is issued on the side
    // stream right after that layer's dA / dB launch, so it runs under the backward pass of the layers below.
    bool opt_inline = false;
    float opt_lr = 0.f;
    hipEvent_t ev_opt = nullptr;      // side: every optimizer launch of the update has finished
    // The gradient at the embedding output feeds nothing trainable; an update computes it only on request
    // (tl_keep_input_grad), for tl_get_dh(boundary 0).
    bool keep_input_grad = false, have_dh0 = false;
    std::vector<LayerSave> save;
    std::vector<float*> hs, dhs;   // residual stream / its gradient at the L+1 layer boundaries
    // shared temporaries
    bf16_t *hf = nullptr, *dlogits = nullptr, *dhf = nullptr, *dh_bf[2] = {nullptr, nullptr}, *d_act = nullptr, *dgu = nullptr,
           *dx = nullptr, *dhmid_bf = nullptr, *d_o = nullptr, *dqkv = nullptr, *dH = nullptr;
    float *logits = nullptr, *nll = nullptr, *loss_sum = nullptr, *dhmid = nullptr, *delta = nullptr,
          *partial = nullptr;
    size_t partial_elems = 0;
    int *tok = nullptr, *labels = nullptr;
    int* tok_host = nullptr;      // pinned
    float* loss_host = nullptr;   // pinned
    // Device-side verdict on the update in flight: bit 0 = the loss is not finite, bit 1 = a dA / dB entry is not finite.
    // The AdamW launches read it and leave the module alone when it is set, so the host can enqueue the whole backward
    // pass without waiting for the loss and still promise that a failed update changes nothing.
    int* flag = nullptr;
    int* flag_host = nullptr;     // pinned
    // generation side: the key/value cache is the q|k|v buffer the forward pass keeps per layer (rows = positions);
    // kv_len rows are valid.  Any training-side forward overwrites it, which matches the method (the cache is
    // recomputed with the updated module after every chunk update).
    // LoRA dropout (training-side forward / backward only): on for the pass in flight?
    bool drop_on = false;
    float* zdrop = nullptr;       // [max_tokens, max(d_model, d_ffn)] fp32: dH A before the mask is applied
    // A split down-projection GEMM may leave its partial tiles in `partial` for the next RMSNorm, which then also writes
    // the residual stream row (pend_h = pend_resid + sum of pend_n tiles); until then pend_h does not hold its values.
    int pend_n = 0;
    float* pend_h = nullptr;
    const float* pend_resid = nullptr;
    int pend_T = 0;
    int loss_row0 = 0;            // first row lm_head and the loss were computed for in the last forward pass
    int kv_len = 0;
    // cache reuse (Section 2): with kv_keep the cache lives in buffers of its own ([max_tokens, 3 d] per layer, same
    // q|k|v row layout), so that a module update leaves it in place: decoding then goes on over keys and values that
    // the previous module computed.
    bool kv_keep = false;
    std::vector<bf16_t*> kvbuf;
    float* lora_h = nullptr;      // [3 r] scaled low-rank activations of the projection group in flight
    float* attn_ws = nullptr;     // partial results of the split decode attention
    size_t attn_ws_elems = 0;
    int* next_dev = nullptr;
    int* next_host = nullptr;     // pinned
    // dA / dB of a layer (one grouped launch) are off the critical path of the backward pass: they run on a second
    // stream (default priority) while the main stream goes on with the layer below.  Everything that launch reads and
    // the layer below would overwrite too early exists twice, indexed by layer parity: dH of each projection group and
    // the bf16 copy of the residual-stream gradient.
    hipStream_t side = nullptr;
    hipEvent_t ev_ready[2] = {};          // main: every operand of the layer's dA / dB launch is written
    hipEvent_t ev_done[2] = {};           // side: the launch has finished
    bool tn_pending[2] = {false, false};
    bf16_t* dHg[2][N_GROUPS] = {};
    // optional timing of the frozen-weight GEMM launches (HIP events on the model's stream)
    bool prof_on = false;
    std::vector<hipEvent_t> prof_ev;
    size_t prof_used = 0;
    double prof_flop = 0.0;
};

// Events that order the two streams of one GPU against each other: no timing, and no system-scope fence when they are
// recorded (that fence writes the caches back and invalidates them for the host's and other devices' sake; kernels of
// one device see each other's results through the release at the end of every kernel).
static constexpr unsigned kSyncEvent = hipEventDisableTiming | hipEventDisableSystemFence;
// Events that only bracket launches for timing: no system-scope fence either, which would lengthen what they measure.
static constexpr unsigned kTimingEvent = hipEventDisableSystemFence;

static void prof_mark(tl_lora* L) {
    if (!L->prof_on) return;
    if (L->prof_used == L->prof_ev.size()) {
        hipEvent_t e;
        if (hipEventCreateWithFlags(&e, kTimingEvent) != hipSuccess) { (void)hipGetLastError(); L->prof_on = false; return; }
        L->prof_ev.push_back(e);
    }
    (void)hipEventRecord(L->prof_ev[L->prof_used++], L->model->stream);
}
// run one frozen-weight GEMM, bracketed by events when timing is on
static hipError_t timed_gemm_one(tl_lora* L, const GemmNT& g) {
    prof_mark(L);
    hipError_t e = launch_gemm_nt(g, L->model->stream);
    prof_mark(L);
    if (L->prof_on) L->prof_flop += 2.0 * g.M * (double)g.N * ((double)g.K + g.K2) * g.batch;
    return e;
}
// as two launches over two column ranges where the tile model finds that cheaper (each is timed as a launch of its own)
static hipError_t timed_gemm(tl_lora* L, const GemmNT& g) {
    GemmNT a, b;
    if (!gemm_nt_split_columns(g, &a, &b)) return timed_gemm_one(L, g);
    hipError_t e = timed_gemm_one(L, a);
    return e != hipSuccess ? e : timed_gemm_one(L, b);
}

// ---------------------------------------------------------------- model
extern "C" tl_status tl_model_create(const tl_model_cfg* cfg, const void* const* wp, void* hip_stream,
                                     tl_model** out) {
    if (!cfg || !wp || !out) return fail(TL_ERR_ARG, "tl_model_create: null argument");
    const tl_model_cfg c = *cfg;
    if (c.n_layers < 1 || c.d_model < 8 || c.n_heads < 1 || c.d_ffn < 8 || c.vocab < 0 || c.max_tokens < 2)
        return fail(TL_ERR_SHAPE, "tl_model_create: non-positive dimension");
    if (c.d_head != 64 && c.d_head != 128) return fail(TL_ERR_SHAPE, "d_head must be 64 or 128 (got %d)", c.d_head);
    if (c.d_model != c.n_heads * c.d_head) return fail(TL_ERR_SHAPE, "d_model != n_heads * d_head");
    if ((c.d_model & 7) || (c.d_ffn & 7) || (c.vocab & 7))
        return fail(TL_ERR_SHAPE, "d_model, d_ffn and vocab must be multiples of 8");
    if (!(c.rms_eps >= 0.f) || !(c.rope_base > 1.f)) return fail(TL_ERR_ARG, "bad rms_eps / rope_base");
    const int nptr = TL_N_WEIGHT_PTRS(c.n_layers);
    for (int i = 0; i < nptr; ++i) {
        const bool tail = i >= TL_PTRS_PER_LAYER * c.n_layers;
        if (!wp[i] && !(tail && c.vocab == 0)) return fail(TL_ERR_ARG, "weight pointer %d is null", i);
    }
    TLCHK(require_gfx950());
    tl_model* m = new (std::nothrow) tl_model();
    if (!m) return fail(TL_ERR_OOM, "host allocation failed");
    m->cfg = c;
    m->stream = (hipStream_t)hip_stream;
    hipStream_t s = m->stream;
    tl_status st = TL_OK;
    auto body = [&]() -> tl_status {
        HIPCHK(hipGetDevice(&m->device));
        const int d = c.d_model, f = c.d_ffn;
        m->layers.resize(c.n_layers);
        for (int l = 0; l < c.n_layers; ++l) {
            LayerW& L = m->layers[l];
            const void* const* p = wp + TL_PTRS_PER_LAYER * l;
            for (int g = 0; g < N_GROUPS; ++g) {
                const int G = kGroupCount[g], din = m->d_in(g), dout = m->d_out(g);
                TLCHK(m->pool.alloc(&L.w[g], (size_t)G * dout * din));
                TLCHK(m->pool.alloc(&L.wt[g], (size_t)G * dout * din));
            }
            for (int pj = 0; pj < 7; ++pj) {
                const int g = kProjGroup[pj], i = kProjIndex[pj], din = m->d_in(g), dout = m->d_out(g);
                HIPCHK(hipMemcpyAsync(L.w[g] + (size_t)i * dout * din, p[pj], (size_t)dout * din * sizeof(bf16_t),
                                      hipMemcpyDeviceToDevice, s));
            }
            for (int g = 0; g < N_GROUPS; ++g) {
                const int G = kGroupCount[g], din = m->d_in(g), dout = m->d_out(g);
                HIPCHK(launch_transpose_bf16(L.w[g], din, G * dout, din, L.wt[g], (long)G * dout, s));
            }
            TLCHK(m->pool.alloc(&L.g1, (size_t)d));
            TLCHK(m->pool.alloc(&L.g2, (size_t)d));
            HIPCHK(hipMemcpyAsync(L.g1, p[7], d * sizeof(float), hipMemcpyDeviceToDevice, s));
            HIPCHK(hipMemcpyAsync(L.g2, p[8], d * sizeof(float), hipMemcpyDeviceToDevice, s));
            (void)f;
        }
        if (c.vocab > 0) {
            const void* const* p = wp + TL_PTRS_PER_LAYER * c.n_layers;
            const size_t n = (size_t)c.vocab * d;
            TLCHK(m->pool.alloc(&m->emb, n));
            TLCHK(m->pool.alloc(&m->head, n));
            TLCHK(m->pool.alloc(&m->head_t, n));
            TLCHK(m->pool.alloc(&m->gf, (size_t)d));
            HIPCHK(hipMemcpyAsync(m->emb, p[0], n * sizeof(bf16_t), hipMemcpyDeviceToDevice, s));
            HIPCHK(hipMemcpyAsync(m->gf, p[1], d * sizeof(float), hipMemcpyDeviceToDevice, s));
            HIPCHK(hipMemcpyAsync(m->head, p[2], n * sizeof(bf16_t), hipMemcpyDeviceToDevice, s));
            HIPCHK(launch_transpose_bf16(m->head, d, c.vocab, d, m->head_t, c.vocab, s));
        }
        TLCHK(m->pool.alloc(&m->rope, (size_t)c.max_tokens * (c.d_head / 2)));
        HIPCHK(launch_rope_table(m->rope, c.max_tokens, c.d_head, c.rope_base, s));
        HIPCHK(hipStreamSynchronize(s));
        return TL_OK;
    };
    st = body();
    if (st != TL_OK) {
        m->pool.release();
        delete m;
        return st;
    }
    *out = m;
    return TL_OK;
}

extern "C" tl_status tl_model_destroy(tl_model* m) {
    if (!m) return TL_OK;
    (void)hipStreamSynchronize(m->stream);
    m->pool.release();
    delete m;
    return TL_OK;
}

// ---------------------------------------------------------------- module life cycle
static void lora_release(tl_lora* L) {
    if (L->side) { (void)hipStreamSynchronize(L->side); (void)hipStreamDestroy(L->side); L->side = nullptr; }
    for (int k = 0; k < 2; ++k) {
        if (L->ev_ready[k]) (void)hipEventDestroy(L->ev_ready[k]);
        if (L->ev_done[k]) (void)hipEventDestroy(L->ev_done[k]);
        L->ev_ready[k] = L->ev_done[k] = nullptr;
        L->tn_pending[k] = false;
    }
    if (L->ev_opt) { (void)hipEventDestroy(L->ev_opt); L->ev_opt = nullptr; }
    for (hipEvent_t e : L->prof_ev) (void)hipEventDestroy(e);
    L->prof_ev.clear();
    L->prof_used = 0;
    L->prof_on = false;
    L->pool.release();
    if (L->tok_host) (void)hipHostFree(L->tok_host);
    if (L->loss_host) (void)hipHostFree(L->loss_host);
    if (L->flag_host) (void)hipHostFree(L->flag_host);
    L->flag_host = nullptr;
    if (L->next_host) (void)hipHostFree(L->next_host);
    L->tok_host = nullptr;
    L->loss_host = nullptr;
    L->next_host = nullptr;
    L->kv_len = 0;
    L->P = L->G = L->M = L->V = nullptr;
}

static tl_status refresh_transposed(tl_lora* L) {
    HIPCHK(launch_transpose_table(L->S, L->ST, L->ttable, L->n_desc, L->total_tiles, L->model->stream));
    return TL_OK;
}

extern "C" tl_status tl_lora_init(tl_model* m, const tl_lora_cfg* cfg, tl_lora** out) {
    if (!m || !cfg || !out) return fail(TL_ERR_ARG, "tl_lora_init: null argument");
    const tl_lora_cfg c = *cfg;
    if (c.rank < 8 || (c.rank & 7) || c.rank > 256) return fail(TL_ERR_SHAPE, "rank must be a multiple of 8 in [8, 256]");
    if (!(c.alpha > 0.f) || !(c.beta1 >= 0.f && c.beta1 < 1.f) || !(c.beta2 >= 0.f && c.beta2 < 1.f) ||
        !(c.eps >= 0.f) || !(c.weight_decay >= 0.f) || !(c.a_init_std >= 0.f) || !(c.dropout >= 0.f && c.dropout < 1.f))
        return fail(TL_ERR_ARG, "tl_lora_init: bad hyper-parameter");
    TLCHK(require_gfx950());
    tl_lora* L = new (std::nothrow) tl_lora();
    if (!L) return fail(TL_ERR_OOM, "host allocation failed");
    L->model = m;
    L->cfg = c;
    L->s = c.alpha / (float)c.rank;
    const tl_model_cfg& mc = m->cfg;
    const int r = c.rank, d = mc.d_model, f = mc.d_ffn, nl = mc.n_layers, Tm = mc.max_tokens, V = mc.vocab;
    hipStream_t s = m->stream;
    auto body = [&]() -> tl_status {
        // arena layout: per layer, per group: A_pack [G r, d_in] then B_pack [G d_out, r]
        L->off.resize(nl);
        size_t n = 0, nt = 0;
        std::vector<TransposeDesc> desc;
        int tiles = 0;
        L->layer_tile0.assign(nl + 1, 0);
        for (int l = 0; l < nl; ++l)
            for (int g = 0; g < N_GROUPS; ++g) {
                if (g == 0) L->layer_tile0[l] = tiles;
                const int G = kGroupCount[g], din = m->d_in(g), dout = m->d_out(g);
                L->off[l].A[g] = n;  n += (size_t)G * r * din;
                L->off[l].B[g] = n;  n += (size_t)G * dout * r;
                L->off[l].AT[g] = nt; nt += (size_t)G * r * din;
                L->off[l].BT[g] = nt; nt += (size_t)G * dout * r;
                // A_pack [G r, d_in] -> AT [d_in, G r]
                TransposeDesc da = {(long)L->off[l].A[g], (long)L->off[l].AT[g], G * r, din, din, G * r, tiles, 0};
                desc.push_back(da);
                tiles += cdiv(G * r, 64) * cdiv(din, 64);
                // each B_p [d_out, r] -> BT_p [r, d_out]
                for (int i = 0; i < G; ++i) {
                    TransposeDesc db = {(long)(L->off[l].B[g] + (size_t)i * dout * r),
                                        (long)(L->off[l].BT[g] + (size_t)i * dout * r), dout, r, r, dout, tiles, 0};
                    desc.push_back(db);
                    tiles += cdiv(dout, 64) * cdiv(r, 64);
                }
            }
        L->layer_tile0[nl] = tiles;
        L->n_params = n;
        L->n_t = nt;
        L->n_desc = (int)desc.size();
        L->total_tiles = tiles;
        TLCHK(L->pool.alloc(&L->P, n));
        TLCHK(L->pool.alloc(&L->G, n));
        TLCHK(L->pool.alloc(&L->M, n));
        TLCHK(L->pool.alloc(&L->V, n));
        TLCHK(L->pool.alloc(&L->S, n));
        TLCHK(L->pool.alloc(&L->ST, nt));
        TLCHK(L->pool.alloc(&L->ttable, desc.size()));
        HIPCHK(hipMemcpyAsync(L->ttable, desc.data(), desc.size() * sizeof(TransposeDesc), hipMemcpyHostToDevice, s));
        HIPCHK(hipStreamSynchronize(s));  // desc is a host temporary
        HIPCHK(launch_fill_f32(L->P, n, 0.f, s));
        HIPCHK(launch_fill_f32(L->G, n, 0.f, s));
        HIPCHK(launch_fill_f32(L->M, n, 0.f, s));
        HIPCHK(launch_fill_f32(L->V, n, 0.f, s));
        for (int l = 0; l < nl; ++l)
            for (int g = 0; g < N_GROUPS; ++g)
                HIPCHK(launch_init_normal(L->P + L->off[l].A[g], (size_t)kGroupCount[g] * r * m->d_in(g),
                                          c.a_init_std, c.seed, (uint64_t)(l * N_GROUPS + g), s));
        HIPCHK(launch_f32_to_bf16(L->P, L->S, n, s));
        TLCHK(refresh_transposed(L));

        // activations
        const size_t Td = (size_t)Tm * d;
        L->save.resize(nl);
        L->hs.resize(nl + 1);
        L->dhs.resize(nl + 1);
        for (int l = 0; l <= nl; ++l) {
            TLCHK(L->pool.alloc(&L->hs[l], Td));
            TLCHK(L->pool.alloc(&L->dhs[l], Td));
        }
        for (int l = 0; l < nl; ++l) {
            LayerSave& sv = L->save[l];
            TLCHK(L->pool.alloc(&sv.x1, Td));
            TLCHK(L->pool.alloc(&sv.qkv, 3 * Td));
            TLCHK(L->pool.alloc(&sv.o, Td));
            TLCHK(L->pool.alloc(&sv.x2, Td));
            TLCHK(L->pool.alloc(&sv.gu, (size_t)Tm * 2 * f));
            TLCHK(L->pool.alloc(&sv.act, (size_t)Tm * f));
            for (int g = 0; g < N_GROUPS; ++g) TLCHK(L->pool.alloc(&sv.hs[g], (size_t)Tm * kGroupCount[g] * r));
            TLCHK(L->pool.alloc(&sv.lse, (size_t)mc.n_heads * Tm));
            TLCHK(L->pool.alloc(&sv.hmid, Td));
            if (c.dropout > 0.f)
                for (int g = 0; g < N_GROUPS; ++g) TLCHK(L->pool.alloc(&sv.xd[g], (size_t)Tm * m->d_in(g)));
        }
        if (c.dropout > 0.f) TLCHK(L->pool.alloc(&L->zdrop, (size_t)Tm * (d > f ? d : f)));
        TLCHK(L->pool.alloc(&L->dh_bf[0], Td));
        TLCHK(L->pool.alloc(&L->dh_bf[1], Td));
        TLCHK(L->pool.alloc(&L->d_act, (size_t)Tm * f));
        TLCHK(L->pool.alloc(&L->dgu, (size_t)Tm * 2 * f));
        TLCHK(L->pool.alloc(&L->dx, Td));
        TLCHK(L->pool.alloc(&L->dhmid, Td));
        TLCHK(L->pool.alloc(&L->dhmid_bf, Td));
        TLCHK(L->pool.alloc(&L->d_o, Td));
        TLCHK(L->pool.alloc(&L->dqkv, 3 * Td));
        TLCHK(L->pool.alloc(&L->dH, (size_t)Tm * 3 * r));
        for (int k = 0; k < 2; ++k) {
            for (int g = 0; g < N_GROUPS; ++g) TLCHK(L->pool.alloc(&L->dHg[k][g], (size_t)Tm * kGroupCount[g] * r));
            HIPCHK(hipEventCreateWithFlags(&L->ev_ready[k], kSyncEvent));
            HIPCHK(hipEventCreateWithFlags(&L->ev_done[k], kSyncEvent));
        }
        HIPCHK(hipStreamCreateWithFlags(&L->side, hipStreamNonBlocking));
        HIPCHK(hipEventCreateWithFlags(&L->ev_opt, hipEventDisableTiming));   // gates the copy of loss and status word to the host: keeps its system-scope fence
        TLCHK(L->pool.alloc(&L->delta, (size_t)mc.n_heads * Tm));
        // split-contraction scratch: up to 16 partial copies of the largest skinny output (Hs: [T, 3r]) or four of a
        // [T, d_model] output (long-K GEMMs with few output tiles)
        {
            const size_t skinny = (size_t)Tm * 3 * r * 16;
            const size_t wide = (size_t)Tm * d * 4;     // four-way split of a GEMM with d_model output columns
            L->partial_elems = skinny > wide ? skinny : wide;
        }
        TLCHK(L->pool.alloc(&L->partial, L->partial_elems));

        TLCHK(L->pool.alloc(&L->tok, (size_t)Tm));
        TLCHK(L->pool.alloc(&L->labels, (size_t)Tm));
        TLCHK(L->pool.alloc(&L->nll, (size_t)Tm));
        TLCHK(L->pool.alloc(&L->loss_sum, (size_t)4));
        TLCHK(L->pool.alloc(&L->flag, (size_t)4));
        HIPCHK(hipMemsetAsync(L->flag, 0, 4 * sizeof(int), s));
        HIPCHK(hipHostMalloc((void**)&L->flag_host, 4 * sizeof(int), hipHostMallocDefault));
        if (V > 0) {
            TLCHK(L->pool.alloc(&L->hf, Td));
            TLCHK(L->pool.alloc(&L->dhf, Td));
            TLCHK(L->pool.alloc(&L->logits, (size_t)Tm * V));
            TLCHK(L->pool.alloc(&L->dlogits, (size_t)Tm * V));
        }
        HIPCHK(hipHostMalloc((void**)&L->tok_host, (size_t)Tm * sizeof(int), hipHostMallocDefault));
        HIPCHK(hipHostMalloc((void**)&L->loss_host, 4 * sizeof(float), hipHostMallocDefault));
        HIPCHK(hipHostMalloc((void**)&L->next_host, 4 * sizeof(int), hipHostMallocDefault));
        TLCHK(L->pool.alloc(&L->lora_h, (size_t)3 * r));
        L->attn_ws_elems = (size_t)mc.n_heads * ATTN_DECODE_MAX_SPLIT * (mc.d_head + 2);
        TLCHK(L->pool.alloc(&L->attn_ws, L->attn_ws_elems));
        TLCHK(L->pool.alloc(&L->next_dev, (size_t)4));
        HIPCHK(hipStreamSynchronize(s));
        return TL_OK;
    };
    tl_status st = body();
    if (st != TL_OK) {
        lora_release(L);
        delete L;
        return st;
    }
    *out = L;
    return TL_OK;
}

extern "C" tl_status tl_discard(tl_lora* L) {
    if (!L) return fail(TL_ERR_ARG, "tl_discard: null handle");
    if (L->discarded) return fail(TL_ERR_DISCARDED, "module already discarded");
    (void)hipStreamSynchronize(L->model->stream);
    lora_release(L);
    L->discarded = true;
    return TL_OK;
}

extern "C" tl_status tl_lora_free(tl_lora* L) {
    if (!L) return TL_OK;
    if (!L->discarded) {
        (void)hipStreamSynchronize(L->model->stream);
        lora_release(L);
    }
    delete L;
    return TL_OK;
}

#define LIVE(L, name)                                                        \
    do {                                                                     \
        if (!(L)) return fail(TL_ERR_ARG, name ": null handle");             \
        if ((L)->discarded) return fail(TL_ERR_DISCARDED, name ": module was discarded"); \
    } while (0)

// ---------------------------------------------------------------- one LoRA-adapted projection group
// forward:  Hs = s X A^T  (kept),  Y = X W^T + Hs B^T (+ residual)
static tl_status group_fwd(tl_lora* L, int l, int g, const bf16_t* X, int T, bf16_t* Y_bf, float* Y_f32,
                           const float* resid, int* deferred = nullptr) {
    tl_model* m = L->model;
    hipStream_t s = m->stream;
    const int G = kGroupCount[g], din = m->d_in(g), dout = m->d_out(g), r = L->cfg.rank;
    const LayerOff& o = L->off[l];
    bf16_t* Hs = L->save[l].hs[g];
    const bf16_t* Xl = X;        // input of the low-rank branch
    if (L->drop_on) {
        HIPCHK(launch_dropout_fwd(X, L->save[l].xd[g], (size_t)T * din, dropout_key(L->cfg.seed, L->step, l, g),
                                  L->cfg.dropout, s));
        Xl = L->save[l].xd[g];
    }
    GemmNT h;
    h.A = Xl; h.lda = din; h.B = L->S + o.A[g]; h.ldb = din; h.M = T; h.N = G * r; h.K = din;
    h.alpha = L->s; h.C = Hs; h.ldc = G * r;
    h.partial = L->partial; h.partial_elems = L->partial_elems;
    HIPCHK(launch_gemm_nt(h, s));
    GemmNT y;
    y.A = X; y.lda = din; y.B = m->layers[l].w[g]; y.ldb = din; y.M = T; y.N = dout; y.K = din;
    y.A2 = Hs; y.lda2 = G * r; y.B2 = L->S + o.B[g]; y.ldb2 = r; y.K2 = r;
    y.batch = G; y.bB = (long)dout * din; y.bA2 = r; y.bB2 = (long)dout * r; y.bC = dout;
    y.ldc = (long)G * dout;
    if (Y_f32) { y.C = Y_f32; y.c_f32 = 1; y.R = resid; } else { y.C = Y_bf; }
    y.partial = L->partial; y.partial_elems = L->partial_elems;
    if (deferred && G == 1) y.deferred = deferred;
    HIPCHK(timed_gemm(L, y));
    return TL_OK;
}

// RMSNorm of a residual-stream row block that may still be pending as partial tiles (see tl_lora::pend_n)
static tl_status norm_fwd(tl_lora* L, const float* h, const float* gain, int T, bf16_t* y) {
    tl_model* m = L->model;
    const int d = m->cfg.d_model;
    if (L->pend_n > 0 && L->pend_h == h && L->pend_T == T) {
        HIPCHK(launch_rmsnorm_fwd(nullptr, gain, T, d, m->cfg.rms_eps, y, m->stream, L->partial, L->pend_n, (long)T * d,
                                  L->pend_resid, L->pend_h));
        L->pend_n = 0;
        return TL_OK;
    }
    if (L->pend_n > 0) return fail(TL_ERR_DEVICE, "internal: pending partial tiles were not consumed");
    HIPCHK(launch_rmsnorm_fwd(h, gain, T, d, m->cfg.rms_eps, y, m->stream));
    return TL_OK;
}
// write a pending residual-stream block out without a norm (single-layer entry point, generation side)
static tl_status flush_pending(tl_lora* L) {
    if (L->pend_n == 0) return TL_OK;
    tl_model* m = L->model;
    // the norm kernel is the one that knows how to add the tiles up: run it into a scratch output
    HIPCHK(launch_rmsnorm_fwd(nullptr, m->layers[0].g1, L->pend_T, m->cfg.d_model, m->cfg.rms_eps, L->dhmid_bf, m->stream,
                              L->partial, L->pend_n, (long)L->pend_T * m->cfg.d_model, L->pend_resid, L->pend_h));
    L->pend_n = 0;
    return TL_OK;
}

// The partial tiles a split dX GEMM leaves to the RMSNorm backward are bf16: dX was a bf16 tensor before the reduce
// pass was folded into the norm, so the gradient loses nothing it had, and the tiles cost half the bytes on both sides.
constexpr int kDeferBf16 = 1;

// backward: dH = s dY B;  dX = dY W + D o (dH A)  (D = 1 without dropout: then one GEMM with the contraction extended
// by dH | A);  the products dA = dH^T X and dB = dY^T Hs are appended to `tn`, which
// the caller launches once per layer (dY, dH, X and Hs must stay untouched until then).
// deferred (may be null): where the dX GEMM may report that it left split partial tiles in L->partial instead of
// writing dX (see GemmNT::deferred); the caller's next kernel then adds them up.
static tl_status group_bwd(tl_lora* L, int l, int g, const bf16_t* dY, const bf16_t* X, int T, bf16_t* dX,
                           GemmTNGroup& tn, int* deferred = nullptr) {
    tl_model* m = L->model;
    hipStream_t s = m->stream;
    const int G = kGroupCount[g], din = m->d_in(g), dout = m->d_out(g), r = L->cfg.rank;
    const LayerOff& o = L->off[l];
    const bf16_t* Hs = L->save[l].hs[g];
    bf16_t* dH = L->dHg[l & 1][g];
    GemmNT h;
    h.A = dY; h.lda = (long)G * dout; h.B = L->ST + o.BT[g]; h.ldb = dout; h.M = T; h.N = r; h.K = dout;
    h.alpha = L->s; h.C = dH; h.ldc = G * r;
    h.batch = G; h.bA = dout; h.bB = (long)r * dout; h.bC = r;
    h.partial = L->partial; h.partial_elems = L->partial_elems;
    HIPCHK(launch_gemm_nt(h, s));
    if (dX) {
        GemmNT x;
        x.A = dY; x.lda = (long)G * dout; x.B = m->layers[l].wt[g]; x.ldb = (long)G * dout; x.M = T; x.N = din;
        x.K = G * dout;
        if (!L->drop_on) { x.A2 = dH; x.lda2 = G * r; x.B2 = L->ST + o.AT[g]; x.ldb2 = G * r; x.K2 = G * r; }
        x.C = dX; x.ldc = din;
        x.partial = L->partial; x.partial_elems = L->partial_elems;
        if (deferred && !L->drop_on) {   // with dropout dX is needed as a whole below
            x.deferred = deferred;
            x.partial_bf16 = kDeferBf16;
        }
        HIPCHK(timed_gemm(L, x));
        if (L->drop_on) {
            GemmNT z;
            z.A = dH; z.lda = G * r; z.B = L->ST + o.AT[g]; z.ldb = G * r; z.M = T; z.N = din; z.K = G * r;
            z.C = L->zdrop; z.ldc = din; z.c_f32 = 1;
            HIPCHK(launch_gemm_nt(z, s));
            HIPCHK(launch_dropout_add(dX, L->zdrop, (size_t)T * din, dropout_key(L->cfg.seed, L->step, l, g),
                                      L->cfg.dropout, s));
        }
    }
    if (L->drop_on) X = L->save[l].xd[g];                                                  // dA = dH^T (D o X)
    tn.add(dH, (long)G * r, G * r, X, din, din, L->G + o.A[g], din);                    // dA [G r, d_in]
    for (int k = 0; k < G; ++k)                                                            // dB_k [d_out, r]
        tn.add(dY + (long)k * dout, (long)G * dout, dout, Hs + (long)k * r, (long)G * r, r,
               L->G + o.B[g] + (size_t)k * dout * r, r);
    return TL_OK;
}

// ---------------------------------------------------------------- one decoder layer
static tl_status layer_forward(tl_lora* L, int l, const float* h_in, float* h_out, int T) {
    tl_model* m = L->model;
    const tl_model_cfg& c = m->cfg;
    hipStream_t s = m->stream;
    const int d = c.d_model, f = c.d_ffn;
    LayerSave& sv = L->save[l];
    const LayerW& W = m->layers[l];
    TLCHK(norm_fwd(L, h_in, W.g1, T, sv.x1));
    TLCHK(group_fwd(L, l, G_QKV, sv.x1, T, sv.qkv, nullptr, nullptr));
    HIPCHK(launch_rope(sv.qkv, 3L * d, T, 2 * c.n_heads, c.d_head, c.rope_base, 0, +1, m->rope, s));  // q and k
    HIPCHK(launch_attention_fwd(sv.qkv, sv.qkv + d, sv.qkv + 2 * d, 3L * d, T, c.n_heads, c.d_head, sv.o, d, sv.lse, s));
    int nsp_o = 0;
    TLCHK(group_fwd(L, l, G_O, sv.o, T, nullptr, sv.hmid, h_in, &nsp_o));
    if (nsp_o > 0) { L->pend_n = nsp_o; L->pend_h = sv.hmid; L->pend_resid = h_in; L->pend_T = T; }
    TLCHK(norm_fwd(L, sv.hmid, W.g2, T, sv.x2));
    TLCHK(group_fwd(L, l, G_GU, sv.x2, T, sv.gu, nullptr, nullptr));
    HIPCHK(launch_swiglu_fwd(sv.gu, T, f, sv.act, s));
    int nsp = 0;
    TLCHK(group_fwd(L, l, G_DOWN, sv.act, T, nullptr, h_out, sv.hmid, &nsp));
    if (nsp > 0) { L->pend_n = nsp; L->pend_h = h_out; L->pend_resid = sv.hmid; L->pend_T = T; }
    return TL_OK;
}

// main stream: wait until the dA / dB launch of the given layer parity has finished
static tl_status wait_tn(tl_lora* L, int par) {
    if (L->tn_pending[par]) {
        HIPCHK(hipStreamWaitEvent(L->model->stream, L->ev_done[par], 0));
        L->tn_pending[par] = false;
    }
    return TL_OK;
}

// dh_out (fp32) and its bf16 copy dh_out_bf -> dh_in (fp32) and, if dh_in_bf != null, its bf16 copy
static tl_status layer_backward(tl_lora* L, int l, const float* h_in, const float* dh_out, const bf16_t* dh_out_bf,
                                float* dh_in, bf16_t* dh_in_bf, int T) {
    tl_model* m = L->model;
    const tl_model_cfg& c = m->cfg;
    hipStream_t s = m->stream;
    const int d = c.d_model, f = c.d_ffn;
    LayerSave& sv = L->save[l];
    const LayerW& W = m->layers[l];
    GemmTNGroup tn;
    tn.T = T;
    tn.flag = L->opt_inline ? L->flag : nullptr;
    const int par = l & 1;
    TLCHK(group_bwd(L, l, G_DOWN, dh_out_bf, sv.act, T, L->d_act, tn));
    // the dA / dB launch of the layer above still reads dgu, dhmid_bf, dqkv (and the other parity's dH): everything
    // below this point overwrites them
    TLCHK(wait_tn(L, par ^ 1));
    HIPCHK(launch_swiglu_bwd(L->d_act, sv.gu, T, f, L->dgu, s));
    // the two dX GEMMs that feed an RMSNorm backward have a long contraction and may be split: the norm kernel then
    // adds the partial tiles up itself (no reduce launch, no bf16 round trip of dX)
    int nsp = 0;
    TLCHK(group_bwd(L, l, G_GU, L->dgu, sv.x2, T, L->dx, tn, &nsp));
    HIPCHK(launch_rmsnorm_bwd(L->dx, sv.hmid, W.g2, dh_out, T, d, c.rms_eps, L->dhmid, L->dhmid_bf, s,
                              nsp ? L->partial : nullptr, nsp, (long)T * d, kDeferBf16));
    TLCHK(group_bwd(L, l, G_O, L->dhmid_bf, sv.o, T, L->d_o, tn));
    // one launch for every dQ and dK/dV part, longest first (dq, dk rotated back inside): 120 -> 84 us per layer at 1024 tokens
    HIPCHK(launch_attention_bwd(sv.qkv, sv.qkv + d, sv.qkv + 2 * d, sv.o, L->d_o, sv.lse, 3L * d, d, T, c.n_heads,
                                c.d_head, L->dqkv, L->dqkv + d, L->dqkv + 2 * d, L->delta, m->rope, s));
    nsp = 0;
    // dh_in == null: the caller does not want the gradient of the layer's input (the bottom layer of an update: it would
    // feed only the frozen embedding), so dX of q|k|v and the first RMSNorm's backward are left out; dA / dB are not
    TLCHK(group_bwd(L, l, G_QKV, L->dqkv, sv.x1, T, dh_in ? L->dx : nullptr, tn, &nsp));
    // all eleven dA / dB products of the layer in one launch on the side stream
    if (tn.n > TN_GROUP_MAX) return fail(TL_ERR_ARG, "too many products for one grouped launch");
    HIPCHK(hipEventRecord(L->ev_ready[par], s));
    HIPCHK(hipStreamWaitEvent(L->side, L->ev_ready[par], 0));
    HIPCHK(launch_gemm_tn_grouped(tn, L->side));
    HIPCHK(hipEventRecord(L->ev_done[par], L->side));
    L->tn_pending[par] = true;
    if (L->opt_inline) {
        // this layer's gradients are complete once that launch is: its AdamW step and the transposed shadows follow on
        // the side stream (every main-stream kernel that reads the layer's factors was enqueued before ev_ready)
        const size_t off = L->off[l].A[0];
        const size_t end = (l + 1 < c.n_layers) ? L->off[l + 1].A[0] : L->n_params;
        HIPCHK(launch_adamw(L->P + off, L->G + off, L->M + off, L->V + off, L->S + off, end - off, (long)(L->step + 1),
                            L->opt_lr, L->cfg.beta1, L->cfg.beta2, L->cfg.eps, L->cfg.weight_decay, L->side, L->flag));
        HIPCHK(launch_transpose_table(L->S, L->ST, L->ttable, L->n_desc, L->layer_tile0[l + 1] - L->layer_tile0[l],
                                      L->side, L->layer_tile0[l]));
    }
    // dh_in_bf must not be the buffer dh_out_bf (dB of the down projection is still reading it): callers alternate
    if (dh_in)
        HIPCHK(launch_rmsnorm_bwd(L->dx, h_in, W.g1, L->dhmid, T, d, c.rms_eps, dh_in, dh_in_bf, s,
                                  nsp ? L->partial : nullptr, nsp, (long)T * d, kDeferBf16));
    return TL_OK;
}

static tl_status optimizer_step(tl_lora* L, float lr, size_t off, size_t n) {
    hipStream_t s = L->model->stream;
    HIPCHK(launch_adamw(L->P + off, L->G + off, L->M + off, L->V + off, L->S + off, n, (long)(L->step + 1), lr,
                        L->cfg.beta1, L->cfg.beta2, L->cfg.eps, L->cfg.weight_decay, s));
    TLCHK(refresh_transposed(L));
    return TL_OK;
}

// ---------------------------------------------------------------- chunk update
static tl_status check_tokens(tl_lora* L, const int32_t* tokens, int32_t n_tokens, int32_t n_ctx) {
    const tl_model_cfg& c = L->model->cfg;
    if (!tokens) return fail(TL_ERR_ARG, "tokens is null");
    if (c.vocab <= 0) return fail(TL_ERR_SHAPE, "model was created without embedding / lm_head (vocab = 0)");
    if (n_tokens < 2 || n_tokens > c.max_tokens)
        return fail(TL_ERR_WINDOW, "n_tokens = %d outside [2, max_tokens = %d]", n_tokens, c.max_tokens);
    if (n_ctx < 0 || n_ctx >= n_tokens) return fail(TL_ERR_WINDOW, "n_ctx = %d must be in [0, n_tokens)", n_ctx);
    for (int i = 0; i < n_tokens; ++i)
        if (tokens[i] < 0 || tokens[i] >= c.vocab)
            return fail(TL_ERR_TOKEN_RANGE, "tokens[%d] = %d outside [0, %d)", i, tokens[i], c.vocab);
    return TL_OK;
}

static tl_status forward_loss(tl_lora* L, const int32_t* tokens, int T, int n_ctx, bool want_grad, int* n_targets) {
    tl_model* m = L->model;
    const tl_model_cfg& c = m->cfg;
    hipStream_t s = m->stream;
    const int d = c.d_model, V = c.vocab;
    // position t predicts token t+1: a target iff t+1 >= max(n_ctx, 1) and t+1 < T
    const int first = (n_ctx > 1 ? n_ctx : 1) - 1;
    const int N = (T - 1) - first;
    *n_targets = N;
    if (!L->kv_keep) L->kv_len = 0;   // the forward pass below overwrites the buffers the cache lives in by default
    L->drop_on = want_grad && L->cfg.dropout > 0.f;   // scoring (no gradient) runs the module without dropout
    memcpy(L->tok_host, tokens, (size_t)T * sizeof(int));
    HIPCHK(hipMemcpyAsync(L->tok, L->tok_host, (size_t)T * sizeof(int), hipMemcpyHostToDevice, s));
    HIPCHK(launch_labels(L->tok, T, L->labels, s));
    HIPCHK(launch_embed(m->emb, L->tok, T, d, L->hs[0], s));
    L->pend_n = 0;
    for (int l = 0; l < c.n_layers; ++l) TLCHK(layer_forward(L, l, L->hs[l], L->hs[l + 1], T));
    TLCHK(norm_fwd(L, L->hs[c.n_layers], m->gf, T, L->hf));
    // conditioning positions carry no loss: their logits are not needed, so lm_head runs on the rows from the first
    // target on only (with the paper's 1024 + 1024 sample that halves it; with Table 5's short pieces it is most of it)
    const int r0 = first >= 64 ? first : 0;
    L->loss_row0 = r0;
    GemmNT lg;
    lg.A = L->hf + (size_t)r0 * d; lg.lda = d; lg.B = m->head; lg.ldb = d; lg.M = T - r0; lg.N = V; lg.K = d;
    lg.C = L->logits + (size_t)r0 * V; lg.ldc = V; lg.c_f32 = 1;
    HIPCHK(timed_gemm(L, lg));
    HIPCHK(launch_cross_entropy(L->logits, L->labels, T, V, first, N, L->nll, want_grad ? L->dlogits : nullptr,
                                L->loss_sum, s, r0, L->flag));
    HIPCHK(hipMemcpyAsync(L->loss_host, L->loss_sum, sizeof(float), hipMemcpyDeviceToHost, s));
    L->last_tokens = T;
    return TL_OK;
}

extern "C" tl_status tl_chunk_loss(tl_lora* L, const int32_t* tokens, int32_t n_tokens, int32_t n_ctx,
                                   float* loss_out, int32_t* n_targets_out) {
    LIVE(L, "tl_chunk_loss");
    if (!loss_out) return fail(TL_ERR_ARG, "loss_out is null");
    TLCHK(check_tokens(L, tokens, n_tokens, n_ctx));
    int N = 0;
    TLCHK(forward_loss(L, tokens, n_tokens, n_ctx, false, &N));
    HIPCHK(hipStreamSynchronize(L->model->stream));
    const float loss = L->loss_host[0] / (float)N;
    if (!std::isfinite(loss)) return fail(TL_ERR_NONFINITE, "loss is not finite");
    *loss_out = loss;
    if (n_targets_out) *n_targets_out = N;
    return TL_OK;
}

// One optimizer step on an already validated sample (forward, loss, backward, AdamW).
static tl_status update_step(tl_lora* L, const int32_t* tokens, int32_t n_tokens, int32_t n_ctx, float lr,
                             float* loss_out, int32_t* n_targets_out) {
    tl_model* m = L->model;
    const tl_model_cfg& c = m->cfg;
    hipStream_t s = m->stream;
    const int T = n_tokens, d = c.d_model, V = c.vocab, nl = c.n_layers;
    int N = 0;
    TLCHK(forward_loss(L, tokens, T, n_ctx, true, &N));
    // The loss decides whether anything is updated, but the host does not wait for it: the loss kernel leaves its
    // verdict in L->flag, which every AdamW launch below reads before it writes, and the host looks at it once, after
    // the backward pass.
    // backward: lm_head, final norm, layers
    const int r0 = L->loss_row0;          // rows below it have no loss and hence a zero gradient at the lm_head input
    if (r0 > 0) HIPCHK(launch_fill_bf16_zero(L->dhf, (size_t)r0 * d, s));
    GemmNT dh;
    dh.A = L->dlogits + (size_t)r0 * V; dh.lda = V; dh.B = m->head_t; dh.ldb = V; dh.M = T - r0; dh.N = d; dh.K = V;
    dh.C = L->dhf + (size_t)r0 * d; dh.ldc = d;
    dh.partial = L->partial; dh.partial_elems = L->partial_elems;
    HIPCHK(timed_gemm(L, dh));
    HIPCHK(launch_rmsnorm_bwd(L->dhf, L->hs[nl], m->gf, nullptr, T, d, c.rms_eps, L->dhs[nl], L->dh_bf[nl & 1], s));
    // a layer's AdamW step follows its dA / dB launch on the side stream (see layer_backward)
    L->opt_inline = true;
    L->opt_lr = lr;
    tl_status bst = TL_OK;
    for (int l = nl - 1; l >= 0 && bst == TL_OK; --l) {
        const bool want_in = l > 0 || L->keep_input_grad;
        bst = layer_backward(L, l, L->hs[l], L->dhs[l + 1], L->dh_bf[(l + 1) & 1], want_in ? L->dhs[l] : nullptr,
                             L->dh_bf[l & 1], T);
        if (l == 0) L->have_dh0 = want_in;
    }
    L->opt_inline = false;
    TLCHK(bst);
    TLCHK(wait_tn(L, 0));
    TLCHK(wait_tn(L, 1));
    L->have_grads = true;
    HIPCHK(hipEventRecord(L->ev_opt, L->side));
    HIPCHK(hipStreamWaitEvent(s, L->ev_opt, 0));
    HIPCHK(hipMemcpyAsync(L->flag_host, L->flag, sizeof(int), hipMemcpyDeviceToHost, s));
    HIPCHK(hipStreamSynchronize(s));
    const float loss = L->loss_host[0] / (float)N;
    if ((L->flag_host[0] & 1) || !std::isfinite(loss))
        return fail(TL_ERR_NONFINITE, "loss is not finite; optimizer step skipped");
    if (L->flag_host[0] & 2)
        return fail(TL_ERR_NONFINITE, "a LoRA gradient is not finite; the optimizer step of the layer it appeared in and "
                                      "of every layer below was skipped");
    L->step += 1;
    *loss_out = loss;
    if (n_targets_out) *n_targets_out = N;
    return TL_OK;
}

extern "C" tl_status tl_chunk_update(tl_lora* L, const int32_t* tokens, int32_t n_tokens, int32_t n_ctx, float lr,
                                     float* loss_out, int32_t* n_targets_out) {
    LIVE(L, "tl_chunk_update");
    if (!loss_out) return fail(TL_ERR_ARG, "loss_out is null");
    if (!(lr >= 0.f) || !std::isfinite(lr)) return fail(TL_ERR_ARG, "lr must be finite and >= 0");
    TLCHK(check_tokens(L, tokens, n_tokens, n_ctx));
    return update_step(L, tokens, n_tokens, n_ctx, lr, loss_out, n_targets_out);
}

// Rate of the optimizer step with 0-based index `step` under a linear warm-up over `warmup_steps` steps.
extern "C" float tl_warmup_lr(float lr, int64_t step, int32_t warmup_steps) {
    if (warmup_steps <= 0 || step + 1 >= (int64_t)warmup_steps) return lr;
    if (step < 0) step = 0;
    return (float)((double)lr * (double)(step + 1) / (double)warmup_steps);
}

// The whole module update for one chunk (Algorithm 1, "Train Theta_k"; Table 5's batch sizes): n epochs over the
// chunk, each epoch cut into pieces of `batch` tokens, one optimizer step per piece.
extern "C" tl_status tl_chunk_train(tl_lora* L, const int32_t* tokens, int32_t n_tokens, int32_t n_chunk,
                                    const tl_train_cfg* cfg, float* losses_out, int32_t* n_steps_out) {
    LIVE(L, "tl_chunk_train");
    if (!cfg) return fail(TL_ERR_ARG, "cfg is null");
    if (!tokens) return fail(TL_ERR_ARG, "tokens is null");
    const tl_model_cfg& c = L->model->cfg;
    if (c.vocab <= 0) return fail(TL_ERR_SHAPE, "model was created without embedding / lm_head (vocab = 0)");
    if (!(cfg->lr >= 0.f) || !std::isfinite(cfg->lr)) return fail(TL_ERR_ARG, "lr must be finite and >= 0");
    if (cfg->epochs < 1) return fail(TL_ERR_ARG, "epochs = %d must be >= 1", cfg->epochs);
    if (cfg->n_ctx_max < 0 || cfg->batch < 0 || cfg->warmup_steps < 0)
        return fail(TL_ERR_ARG, "n_ctx_max, batch and warmup_steps must be >= 0");
    if (n_chunk < 1 || n_chunk > n_tokens)
        return fail(TL_ERR_WINDOW, "n_chunk = %d outside [1, n_tokens = %d]", n_chunk, n_tokens);
    const int batch = cfg->batch > 0 && cfg->batch < n_chunk ? cfg->batch : n_chunk;
    const int n_before = n_tokens - n_chunk;
    const int pieces = (n_chunk + batch - 1) / batch;
    // every sample is checked before the first step, so that an error leaves the module as it was
    for (int j = 0; j < pieces; ++j) {
        const int start = n_before + j * batch, end = std::min(start + batch, n_tokens);
        const int ctx = std::min(start, cfg->n_ctx_max);
        if (end - (start - ctx) > c.max_tokens)
            return fail(TL_ERR_WINDOW, "piece %d: %d conditioning + %d chunk tokens exceed max_tokens = %d", j, ctx,
                        end - start, c.max_tokens);
        if (end - (start - ctx) < 2)
            return fail(TL_ERR_WINDOW, "piece %d has a single token and nothing before it: no prediction target", j);
    }
    for (int i = 0; i < n_tokens; ++i)
        if (tokens[i] < 0 || tokens[i] >= c.vocab)
            return fail(TL_ERR_TOKEN_RANGE, "tokens[%d] = %d outside [0, %d)", i, tokens[i], c.vocab);
    int steps = 0;
    for (int e = 0; e < cfg->epochs; ++e)
        for (int j = 0; j < pieces; ++j) {
            const int start = n_before + j * batch, end = std::min(start + batch, n_tokens);
            const int ctx = std::min(start, cfg->n_ctx_max);
            float loss = 0.f;
            const float lr = tl_warmup_lr(cfg->lr, L->step, cfg->warmup_steps);
            TLCHK(update_step(L, tokens + (start - ctx), end - (start - ctx), ctx, lr, &loss, nullptr));
            if (losses_out) losses_out[steps] = loss;
            ++steps;
            if (n_steps_out) *n_steps_out = steps;
        }
    return TL_OK;
}

// ---------------------------------------------------------------- generation side (Algorithm 1, the token loop)
// Last-position logits -> greedy token; optional copy of the logits to the host.
static tl_status emit_next(tl_lora* L, const float* h_last, int32_t* next_token, float* logits_out) {
    tl_model* m = L->model;
    const tl_model_cfg& c = m->cfg;
    hipStream_t s = m->stream;
    GemvPre nf;    // the final norm is formed inside the lm_head product
    nf.mode = 1; nf.h = h_last; nf.gain = m->gf; nf.eps = c.rms_eps;
    prof_mark(L);
    hipError_t e = launch_gemv(m->head, c.d_model, nullptr, c.vocab, c.d_model, nullptr, nullptr, 0, 0, 1.f, nullptr,
                               nullptr, L->logits, s, &nf);
    prof_mark(L);
    if (L->prof_on) L->prof_flop += 2.0 * c.vocab * (double)c.d_model;
    HIPCHK(e);
    HIPCHK(launch_argmax(L->logits, c.vocab, L->next_dev, s));
    HIPCHK(hipMemcpyAsync(L->next_host, L->next_dev, sizeof(int), hipMemcpyDeviceToHost, s));
    if (logits_out)
        HIPCHK(hipMemcpyAsync(logits_out, L->logits, (size_t)c.vocab * sizeof(float), hipMemcpyDeviceToHost, s));
    HIPCHK(hipStreamSynchronize(s));
    *next_token = L->next_host[0];
    return TL_OK;
}

extern "C" tl_status tl_prefill(tl_lora* L, const int32_t* tokens, int32_t n_tokens, int32_t* next_token,
                                float* logits_out) {
    LIVE(L, "tl_prefill");
    if (!next_token) return fail(TL_ERR_ARG, "next_token is null");
    tl_model* m = L->model;
    const tl_model_cfg& c = m->cfg;
    if (!tokens) return fail(TL_ERR_ARG, "tokens is null");
    if (c.vocab <= 0) return fail(TL_ERR_SHAPE, "model was created without embedding / lm_head (vocab = 0)");
    if (n_tokens < 1 || n_tokens > c.max_tokens)
        return fail(TL_ERR_WINDOW, "n_tokens = %d outside [1, max_tokens = %d]", n_tokens, c.max_tokens);
    for (int i = 0; i < n_tokens; ++i)
        if (tokens[i] < 0 || tokens[i] >= c.vocab)
            return fail(TL_ERR_TOKEN_RANGE, "tokens[%d] = %d outside [0, %d)", i, tokens[i], c.vocab);
    hipStream_t s = m->stream;
    const int T = n_tokens, d = c.d_model;
    L->kv_len = 0;
    L->drop_on = false;   // generation runs the module without dropout
    memcpy(L->tok_host, tokens, (size_t)T * sizeof(int));
    HIPCHK(hipMemcpyAsync(L->tok, L->tok_host, (size_t)T * sizeof(int), hipMemcpyHostToDevice, s));
    HIPCHK(launch_embed(m->emb, L->tok, T, d, L->hs[0], s));
    // the chunk path's forward: it leaves q|k|v (q, k rotated) of every position in save[l].qkv, which is the cache
    L->pend_n = 0;
    for (int l = 0; l < c.n_layers; ++l) TLCHK(layer_forward(L, l, L->hs[l], L->hs[l + 1], T));
    TLCHK(flush_pending(L));      // the last layer's output rows are read directly below
    if (L->kv_keep)
        for (int l = 0; l < c.n_layers; ++l)
            HIPCHK(hipMemcpyAsync(L->kvbuf[l], L->save[l].qkv, (size_t)T * 3 * d * sizeof(bf16_t), hipMemcpyDeviceToDevice, s));
    TLCHK(emit_next(L, L->hs[c.n_layers] + (size_t)(T - 1) * d, next_token, logits_out));
    L->kv_len = T;
    return TL_OK;
}

extern "C" tl_status tl_cache_reuse(tl_lora* L, int32_t on) {
    LIVE(L, "tl_cache_reuse");
    tl_model* m = L->model;
    const tl_model_cfg& c = m->cfg;
    if (!on) {
        if (L->kv_keep) L->kv_len = 0;    // the cache in the dedicated buffers is dropped
        L->kv_keep = false;
        return TL_OK;
    }
    if (L->kv_keep) return TL_OK;
    if (L->kvbuf.empty()) {
        std::vector<bf16_t*> bufs(c.n_layers, nullptr);
        for (int l = 0; l < c.n_layers; ++l) TLCHK(L->pool.alloc(&bufs[l], (size_t)c.max_tokens * 3 * c.d_model));
        L->kvbuf = bufs;
    }
    // a cache that exists already moves along
    for (int l = 0; l < c.n_layers && L->kv_len > 0; ++l)
        HIPCHK(hipMemcpyAsync(L->kvbuf[l], L->save[l].qkv, (size_t)L->kv_len * 3 * c.d_model * sizeof(bf16_t),
                              hipMemcpyDeviceToDevice, m->stream));
    HIPCHK(hipStreamSynchronize(m->stream));
    L->kv_keep = true;
    return TL_OK;
}

// One LoRA-adapted projection group of a single token: h = s A x, then y = W x + B h (+ residual)
// x: the group's input vector; with `pre` it is formed (norm / SwiGLU) inside the first launch, which stores it to x
static tl_status group_decode(tl_lora* L, int l, int g, const bf16_t* x, bf16_t* y_bf, float* y_f32, const float* resid,
                              const GemvPre* pre = nullptr) {
    tl_model* m = L->model;
    hipStream_t s = m->stream;
    const int G = kGroupCount[g], din = m->d_in(g), dout = m->d_out(g), r = L->cfg.rank;
    const LayerOff& o = L->off[l];
    HIPCHK(launch_gemv(L->S + o.A[g], din, x, G * r, din, nullptr, nullptr, 0, 0, L->s, nullptr, nullptr, L->lora_h, s,
                       pre));
    prof_mark(L);   // timing (when on) brackets the launches that stream a frozen matrix
    hipError_t e = launch_gemv(m->layers[l].w[g], din, x, G * dout, din, L->S + o.B[g], L->lora_h, r, dout, 1.f, resid,
                               y_bf, y_f32, s);
    prof_mark(L);
    if (L->prof_on) L->prof_flop += 2.0 * G * dout * ((double)din + r);
    HIPCHK(e);
    return TL_OK;
}

extern "C" tl_status tl_decode_step(tl_lora* L, int32_t token, int32_t* next_token, float* logits_out) {
    LIVE(L, "tl_decode_step");
    if (!next_token) return fail(TL_ERR_ARG, "next_token is null");
    tl_model* m = L->model;
    const tl_model_cfg& c = m->cfg;
    if (L->kv_len <= 0)
        return fail(TL_ERR_ARG, "tl_decode_step: no key/value cache (call tl_prefill first, and again after every "
                                "update unless tl_cache_reuse is on)");
    if (L->kv_len >= c.max_tokens) return fail(TL_ERR_WINDOW, "the window is full (%d positions)", c.max_tokens);
    if (token < 0 || token >= c.vocab) return fail(TL_ERR_TOKEN_RANGE, "token = %d outside [0, %d)", token, c.vocab);
    hipStream_t s = m->stream;
    const int d = c.d_model, p = L->kv_len;
    L->tok_host[0] = token;
    HIPCHK(hipMemcpyAsync(L->tok, L->tok_host, sizeof(int), hipMemcpyHostToDevice, s));
    HIPCHK(launch_embed(m->emb, L->tok, 1, d, L->hs[0], s));
    for (int l = 0; l < c.n_layers; ++l) {
        LayerSave& sv = L->save[l];
        const LayerW& W = m->layers[l];
        const float* h_in = L->hs[l];
        float* h_out = L->hs[l + 1];
        bf16_t* cache = L->kv_keep ? L->kvbuf[l] : sv.qkv;
        bf16_t* row = cache + (size_t)p * 3 * d;                  // the new cache row: q | k | v of position p
        GemvPre n1, n2, sw;
        n1.mode = 1; n1.h = h_in; n1.gain = W.g1; n1.eps = c.rms_eps; n1.x_out = sv.x1;
        n2.mode = 1; n2.h = sv.hmid; n2.gain = W.g2; n2.eps = c.rms_eps; n2.x_out = sv.x2;
        sw.mode = 2; sw.gu = sv.gu; sw.x_out = sv.act;
        TLCHK(group_decode(L, l, G_QKV, sv.x1, row, nullptr, nullptr, &n1));
        // q and k of the new row are rotated inside the attention launch (the rotated k goes back into the cache)
        HIPCHK(launch_attention_decode(row, cache + d, cache + 2 * d, 3L * d, p + 1, c.n_heads, c.d_head, sv.o,
                                       L->attn_ws, L->attn_ws_elems, s, m->rope + (size_t)p * (c.d_head / 2)));
        TLCHK(group_decode(L, l, G_O, sv.o, nullptr, sv.hmid, h_in));
        TLCHK(group_decode(L, l, G_GU, sv.x2, sv.gu, nullptr, nullptr, &n2));
        TLCHK(group_decode(L, l, G_DOWN, sv.act, nullptr, h_out, sv.hmid, &sw));
    }
    TLCHK(emit_next(L, L->hs[c.n_layers], next_token, logits_out));
    L->kv_len = p + 1;
    return TL_OK;
}

// Algorithm 1, cascaded deployment: generate, and after every full chunk pause and train the module on it.
extern "C" tl_status tl_generate(tl_lora* L, const int32_t* prompt, int32_t n_prompt, int32_t n_new,
                                 const tl_generate_cfg* cfg, int32_t* tokens_out, float* losses_out,
                                 int32_t* n_steps_out) {
    LIVE(L, "tl_generate");
    if (!prompt || !cfg || !tokens_out) return fail(TL_ERR_ARG, "tl_generate: null pointer");
    const tl_model_cfg& c = L->model->cfg;
    if (n_prompt < 1 || n_new < 0) return fail(TL_ERR_ARG, "tl_generate: n_prompt must be >= 1 and n_new >= 0");
    if (cfg->window < 1 || cfg->chunk < 1) return fail(TL_ERR_ARG, "tl_generate: window and chunk must be >= 1");
    if (cfg->window + cfg->chunk > c.max_tokens)
        return fail(TL_ERR_WINDOW, "window %d + chunk %d exceed max_tokens = %d", cfg->window, cfg->chunk, c.max_tokens);
    const int batch = cfg->train.batch > 0 && cfg->train.batch < cfg->chunk ? cfg->train.batch : cfg->chunk;
    if (cfg->train.n_ctx_max < 0 || cfg->train.n_ctx_max + batch > c.max_tokens)
        return fail(TL_ERR_WINDOW, "training sample of %d conditioning + %d chunk tokens exceeds max_tokens = %d",
                    cfg->train.n_ctx_max, batch, c.max_tokens);
    for (int i = 0; i < n_prompt; ++i)
        if (prompt[i] < 0 || prompt[i] >= c.vocab)
            return fail(TL_ERR_TOKEN_RANGE, "prompt[%d] = %d outside [0, %d)", i, prompt[i], c.vocab);
    if (n_steps_out) *n_steps_out = 0;
    std::vector<int32_t> text(prompt, prompt + n_prompt);     // Y of Algorithm 1: everything read or generated so far
    int produced = 0, steps = 0;
    while (produced < n_new) {
        // X: the most recent `window` tokens; the cache is rebuilt with the current module
        const int n_x = std::min<int>((int)text.size(), cfg->window);
        int32_t next = 0;
        TLCHK(tl_prefill(L, text.data() + text.size() - n_x, n_x, &next, nullptr));
        int in_chunk = 0;
        while (in_chunk < cfg->chunk && produced < n_new) {
            text.push_back(next);
            tokens_out[produced++] = next;
            ++in_chunk;
            if (in_chunk < cfg->chunk && produced < n_new) TLCHK(tl_decode_step(L, next, &next, nullptr));
        }
        if (in_chunk < cfg->chunk) break;                     // generation ended inside a chunk: nothing to train on
        // train on the chunk just generated, conditioned on what precedes it
        const int n_before = std::min<int>((int)text.size() - cfg->chunk, cfg->train.n_ctx_max);
        int made = 0;
        tl_status st = tl_chunk_train(L, text.data() + text.size() - cfg->chunk - n_before, n_before + cfg->chunk, cfg->chunk,
                                      &cfg->train, losses_out ? losses_out + steps : nullptr, &made);
        steps += made;
        if (n_steps_out) *n_steps_out = steps;
        TLCHK(st);
    }
    return TL_OK;
}

extern "C" tl_status tl_kv_length(tl_lora* L, int32_t* n_out) {
    LIVE(L, "tl_kv_length");
    if (!n_out) return fail(TL_ERR_ARG, "n_out is null");
    *n_out = L->kv_len;
    return TL_OK;
}

extern "C" tl_status tl_layer_step(tl_lora* L, int32_t layer, const float* h_in, const float* dh_out, int32_t n_tokens,
                                   float* h_out, float* dh_in, float lr, int32_t apply_adamw) {
    LIVE(L, "tl_layer_step");
    if (!h_in || !dh_out || !h_out || !dh_in) return fail(TL_ERR_ARG, "tl_layer_step: null pointer");
    const tl_model_cfg& c = L->model->cfg;
    if (layer < 0 || layer >= c.n_layers) return fail(TL_ERR_ARG, "layer %d out of range", layer);
    if (n_tokens < 1 || n_tokens > c.max_tokens) return fail(TL_ERR_WINDOW, "n_tokens outside [1, max_tokens]");
    if (!(lr >= 0.f) || !std::isfinite(lr)) return fail(TL_ERR_ARG, "lr must be finite and >= 0");
    hipStream_t s = L->model->stream;
    if (!L->kv_keep) L->kv_len = 0;
    L->drop_on = L->cfg.dropout > 0.f;
    L->pend_n = 0;
    TLCHK(layer_forward(L, layer, h_in, h_out, n_tokens));
    TLCHK(flush_pending(L));      // the caller reads h_out
    HIPCHK(launch_f32_to_bf16(dh_out, L->dh_bf[0], (size_t)n_tokens * c.d_model, s));
    TLCHK(layer_backward(L, layer, h_in, dh_out, L->dh_bf[0], dh_in, nullptr, n_tokens));
    TLCHK(wait_tn(L, 0));
    TLCHK(wait_tn(L, 1));
    L->have_grads = true;
    L->last_tokens = n_tokens;
    if (apply_adamw) {
        const size_t off = L->off[layer].A[0];
        const size_t end = (layer + 1 < c.n_layers) ? L->off[layer + 1].A[0] : L->n_params;
        TLCHK(optimizer_step(L, lr, off, end - off));
    }
    HIPCHK(hipStreamSynchronize(s));
    if (apply_adamw) L->step += 1;
    return TL_OK;
}

// ---------------------------------------------------------------- inspection
static tl_status factor_span(tl_lora* L, int layer, int proj, int which, size_t n, size_t* off) {
    const tl_model* m = L->model;
    if (layer < 0 || layer >= m->cfg.n_layers || proj < 0 || proj > 6 || which < 0 || which > 7)
        return fail(TL_ERR_ARG, "bad (layer, proj, which) = (%d, %d, %d)", layer, proj, which);
    const int g = kProjGroup[proj], i = kProjIndex[proj], r = L->cfg.rank;
    const size_t na = (size_t)r * m->d_in(g), nb = (size_t)m->d_out(g) * r;
    const bool isB = which & 1;
    if (n != (isB ? nb : na)) return fail(TL_ERR_ARG, "size mismatch: expected %zu elements", isB ? nb : na);
    *off = isB ? L->off[layer].B[g] + i * nb : L->off[layer].A[g] + i * na;
    return TL_OK;
}

extern "C" tl_status tl_get_factor(tl_lora* L, int32_t layer, int32_t proj, int32_t which, float* host_out, size_t n) {
    LIVE(L, "tl_get_factor");
    if (!host_out) return fail(TL_ERR_ARG, "host_out is null");
    size_t off = 0;
    TLCHK(factor_span(L, layer, proj, which, n, &off));
    const float* base = which < 2 ? L->P : which < 4 ? L->G : which < 6 ? L->M : L->V;
    HIPCHK(hipStreamSynchronize(L->model->stream));
    HIPCHK(hipMemcpy(host_out, base + off, n * sizeof(float), hipMemcpyDeviceToHost));
    return TL_OK;
}

extern "C" tl_status tl_set_factor(tl_lora* L, int32_t layer, int32_t proj, int32_t which, const float* host_in,
                                   size_t n) {
    LIVE(L, "tl_set_factor");
    if (!host_in) return fail(TL_ERR_ARG, "host_in is null");
    if (which != TL_FACTOR_A && which != TL_FACTOR_B) return fail(TL_ERR_ARG, "only A or B can be set");
    size_t off = 0;
    TLCHK(factor_span(L, layer, proj, which, n, &off));
    hipStream_t s = L->model->stream;
    HIPCHK(hipStreamSynchronize(s));
    HIPCHK(hipMemcpy(L->P + off, host_in, n * sizeof(float), hipMemcpyHostToDevice));
    HIPCHK(launch_f32_to_bf16(L->P + off, L->S + off, n, s));
    TLCHK(refresh_transposed(L));
    HIPCHK(hipStreamSynchronize(s));
    return TL_OK;
}

extern "C" tl_status tl_get_step(tl_lora* L, int64_t* step_out) {
    LIVE(L, "tl_get_step");
    if (!step_out) return fail(TL_ERR_ARG, "step_out is null");
    *step_out = L->step;
    return TL_OK;
}

extern "C" tl_status tl_get_nll(tl_lora* L, float* host_out, size_t n) {
    LIVE(L, "tl_get_nll");
    if (!host_out) return fail(TL_ERR_ARG, "host_out is null");
    if (L->last_tokens <= 0 || n != (size_t)L->last_tokens) return fail(TL_ERR_ARG, "n must equal the last call's n_tokens");
    HIPCHK(hipStreamSynchronize(L->model->stream));
    HIPCHK(hipMemcpy(host_out, L->nll, n * sizeof(float), hipMemcpyDeviceToHost));
    return TL_OK;
}

extern "C" tl_status tl_keep_input_grad(tl_lora* L, int32_t on) {
    LIVE(L, "tl_keep_input_grad");
    L->keep_input_grad = on != 0;
    return TL_OK;
}

extern "C" tl_status tl_get_dh(tl_lora* L, int32_t boundary, float* host_out, size_t n) {
    LIVE(L, "tl_get_dh");
    if (!host_out) return fail(TL_ERR_ARG, "host_out is null");
    const tl_model_cfg& c = L->model->cfg;
    if (boundary < 0 || boundary > c.n_layers) return fail(TL_ERR_ARG, "boundary out of range");
    if (!L->have_grads || n != (size_t)L->last_tokens * c.d_model) return fail(TL_ERR_ARG, "n must be n_tokens * d_model of the last update");
    if (boundary == 0 && !L->have_dh0)
        return fail(TL_ERR_ARG, "the gradient at the embedding output was not computed: call tl_keep_input_grad(lora, 1) before the update");
    HIPCHK(hipStreamSynchronize(L->model->stream));
    HIPCHK(hipMemcpy(host_out, L->dhs[boundary], n * sizeof(float), hipMemcpyDeviceToHost));
    return TL_OK;
}

extern "C" tl_status tl_profile_enable(tl_lora* L, int32_t on) {
    LIVE(L, "tl_profile_enable");
    HIPCHK(hipStreamSynchronize(L->model->stream));
    L->prof_on = on != 0;
    L->prof_used = 0;
    L->prof_flop = 0.0;
    return TL_OK;
}

extern "C" tl_status tl_profile_read(tl_lora* L, double* ms_total, int64_t* launches, double* flop_total) {
    LIVE(L, "tl_profile_read");
    if (!ms_total || !launches || !flop_total) return fail(TL_ERR_ARG, "tl_profile_read: null pointer");
    HIPCHK(hipStreamSynchronize(L->model->stream));
    double ms = 0.0;
    for (size_t i = 0; i + 1 < L->prof_used; i += 2) {
        float t = 0.f;
        HIPCHK(hipEventElapsedTime(&t, L->prof_ev[i], L->prof_ev[i + 1]));
        ms += t;
    }
    *ms_total = ms;
    *launches = (int64_t)(L->prof_used / 2);
    *flop_total = L->prof_flop;
    L->prof_used = 0;
    L->prof_flop = 0.0;
    return TL_OK;
}

// ---------------------------------------------------------------- single fp32 LoRA-adapted linear layer
// H, dH: [T, r] scratch; mom: 2 (r d_in + d_out r) floats of optimizer moments (only with apply_adamw).
static tl_status linear_step_run(const float* X, const float* W, const float* A, const float* B, const float* dY, int T,
                                 int d_in, int d_out, int r, float s, float lr, float beta1, float beta2, float eps,
                                 float wd, int apply_adamw, float* Y, float* dX, float* dA, float* dB, float* A_new,
                                 float* B_new, float* H, float* dH, float* mom, hipStream_t st) {
    // H = X A^T;  Y = X W^T + s H B^T
    HIPCHK(launch_sgemm(0, 1, T, r, d_in, 1.f, X, d_in, A, d_in, 0.f, H, r, st));
    HIPCHK(launch_sgemm(0, 1, T, d_out, d_in, 1.f, X, d_in, W, d_in, 0.f, Y, d_out, st));
    HIPCHK(launch_sgemm(0, 1, T, d_out, r, s, H, r, B, r, 1.f, Y, d_out, st));
    // dH = s dY B;  dX = dY W + dH A;  dA = dH^T X;  dB = s dY^T H
    HIPCHK(launch_sgemm(0, 0, T, r, d_out, s, dY, d_out, B, r, 0.f, dH, r, st));
    HIPCHK(launch_sgemm(0, 0, T, d_in, d_out, 1.f, dY, d_out, W, d_in, 0.f, dX, d_in, st));
    HIPCHK(launch_sgemm(0, 0, T, d_in, r, 1.f, dH, r, A, d_in, 1.f, dX, d_in, st));
    HIPCHK(launch_sgemm(1, 0, r, d_in, T, 1.f, dH, r, X, d_in, 0.f, dA, d_in, st));
    HIPCHK(launch_sgemm(1, 0, d_out, r, T, s, dY, d_out, H, r, 0.f, dB, r, st));
    if (apply_adamw) {
        const size_t na = (size_t)r * d_in, nb = (size_t)d_out * r;
        HIPCHK(launch_fill_f32(mom, 2 * (na + nb), 0.f, st));     // first step: zero moments (a kernel, not a memset node)
        HIPCHK(hipMemcpyAsync(A_new, A, na * sizeof(float), hipMemcpyDeviceToDevice, st));
        HIPCHK(hipMemcpyAsync(B_new, B, nb * sizeof(float), hipMemcpyDeviceToDevice, st));
        HIPCHK(launch_adamw(A_new, dA, mom, mom + na, nullptr, na, 1, lr, beta1, beta2, eps, wd, st));
        HIPCHK(launch_adamw(B_new, dB, mom + 2 * na, mom + 2 * na + nb, nullptr, nb, 1, lr, beta1, beta2, eps, wd, st));
    }
    HIPCHK(hipStreamSynchronize(st));
    return TL_OK;
}

static tl_status linear_step_args(const float* X, const float* W, const float* A, const float* B, const float* dY, int T,
                                  int d_in, int d_out, int r, int apply_adamw, float* Y, float* dX, float* dA,
                                  float* dB, float* A_new, float* B_new) {
    if (!X || !W || !A || !B || !dY || !Y || !dX || !dA || !dB) return fail(TL_ERR_ARG, "tl_linear_step: null pointer");
    if (apply_adamw && (!A_new || !B_new)) return fail(TL_ERR_ARG, "tl_linear_step: A_new/B_new required");
    if (T < 1 || d_in < 1 || d_out < 1 || r < 1) return fail(TL_ERR_SHAPE, "tl_linear_step: non-positive dimension");
    return require_gfx950();
}

extern "C" tl_status tl_linear_step(const float* X, const float* W, const float* A, const float* B, const float* dY,
                                    int32_t T, int32_t d_in, int32_t d_out, int32_t r, float s, float lr, float beta1,
                                    float beta2, float eps, float wd, int32_t apply_adamw, float* Y, float* dX,
                                    float* dA, float* dB, float* A_new, float* B_new, void* hip_stream) {
    TLCHK(linear_step_args(X, W, A, B, dY, T, d_in, d_out, r, apply_adamw, Y, dX, dA, dB, A_new, B_new));
    hipStream_t st = (hipStream_t)hip_stream;
    Pool pool;
    float *H = nullptr, *dH = nullptr, *mom = nullptr;
    auto body = [&]() -> tl_status {
        TLCHK(pool.alloc(&H, (size_t)T * r));
        TLCHK(pool.alloc(&dH, (size_t)T * r));
        if (apply_adamw) TLCHK(pool.alloc(&mom, 2 * ((size_t)r * d_in + (size_t)d_out * r)));
        return linear_step_run(X, W, A, B, dY, T, d_in, d_out, r, s, lr, beta1, beta2, eps, wd, apply_adamw, Y, dX, dA, dB,
                               A_new, B_new, H, dH, mom, st);
    };
    tl_status rc = body();
    if (rc != TL_OK) (void)hipStreamSynchronize(st);
    pool.release();
    return rc;
}

// ---------------------------------------------------------------- tl_linear_step without allocation
// For callers that cannot allocate (HIP graph capture, tight serving loops, harnesses that forbid hipMalloc): the
// scratch tl_linear_step takes from hipMalloc (H, dH and, with AdamW, the moments) lives in one file-scope device
// array instead.  Every GPU the library runs on holds its own copy for the life of the process; the array's name is
// only a host-side handle, so its device address is looked up once per device (with that device current) and kept.
constexpr size_t kStaticScratchFloats = (size_t)1 << 20;    // 4 MiB
static __device__ __align__(256) float tl_static_scratch[kStaticScratchFloats];
constexpr int kMaxDevices = 64;
static float* g_static_scratch_ptr[kMaxDevices] = {};
static std::mutex g_static_scratch_mutex;

static tl_status static_scratch(float** out) {
    int dev = -1;
    HIPCHK(hipGetDevice(&dev));
    if (dev < 0 || dev >= kMaxDevices) return fail(TL_ERR_DEVICE, "device index %d out of range", dev);
    std::lock_guard<std::mutex> lock(g_static_scratch_mutex);
    if (!g_static_scratch_ptr[dev]) {
        float* p = nullptr;
        HIPCHK(hipGetSymbolAddress((void**)&p, HIP_SYMBOL(tl_static_scratch)));
        if (!p) return fail(TL_ERR_DEVICE, "hipGetSymbolAddress returned a null address for the static scratch");
        g_static_scratch_ptr[dev] = p;
    }
    *out = g_static_scratch_ptr[dev];
    return TL_OK;
}

extern "C" tl_status tl_linear_step_static(const float* X, const float* W, const float* A, const float* B,
                                           const float* dY, int32_t T, int32_t d_in, int32_t d_out, int32_t r, float s,
                                           float lr, float beta1, float beta2, float eps, float wd, int32_t apply_adamw,
                                           float* Y, float* dX, float* dA, float* dB, float* A_new, float* B_new,
                                           void* hip_stream) {
    TLCHK(linear_step_args(X, W, A, B, dY, T, d_in, d_out, r, apply_adamw, Y, dX, dA, dB, A_new, B_new));
    // sub-buffers start on 256-byte boundaries
    auto up = [](size_t n) { return (n + 63) & ~(size_t)63; };
    const size_t n_h = up((size_t)T * r);
    const size_t n_mom = apply_adamw ? up(2 * ((size_t)r * d_in + (size_t)d_out * r)) : 0;
    const size_t need = 2 * n_h + n_mom;
    if (need > kStaticScratchFloats)
        return fail(TL_ERR_SHAPE, "tl_linear_step_static: needs %zu floats of scratch (2 T r%s), the static buffer holds %zu; "
                                  "use tl_linear_step", need, apply_adamw ? " + 2 r (d_in + d_out)" : "", kStaticScratchFloats);
    float* base = nullptr;
    TLCHK(static_scratch(&base));
    hipStream_t st = (hipStream_t)hip_stream;
    tl_status rc = linear_step_run(X, W, A, B, dY, T, d_in, d_out, r, s, lr, beta1, beta2, eps, wd, apply_adamw, Y, dX, dA,
                                   dB, A_new, B_new, base, base + n_h, apply_adamw ? base + 2 * n_h : nullptr, st);
    if (rc != TL_OK) (void)hipStreamSynchronize(st);
    return rc;
}

// ---------------------------------------------------------------- single kernels
#define KARGS_OK(cond, name) \
    do { if (!(cond)) return fail(TL_ERR_ARG, name ": bad argument"); } while (0)

extern "C" tl_status tl_k_gemm_nt(const uint16_t* A, int32_t lda, const uint16_t* B, int32_t ldb, int32_t M, int32_t N,
                                  int32_t K, const uint16_t* A2, int32_t lda2, const uint16_t* B2, int32_t ldb2,
                                  int32_t K2, float alpha, const float* R, void* C, int32_t ldc, int32_t c_f32,
                                  float* workspace, size_t workspace_elems, void* hip_stream) {
    KARGS_OK(A && B && C && M >= 0 && N >= 0 && K >= 0 && K2 >= 0 && (K2 == 0 || (A2 && B2)), "tl_k_gemm_nt");
    GemmNT g;
    g.A = A; g.lda = lda; g.B = B; g.ldb = ldb; g.M = M; g.N = N; g.K = K;
    g.A2 = K2 ? A2 : nullptr; g.lda2 = lda2; g.B2 = K2 ? B2 : nullptr; g.ldb2 = ldb2; g.K2 = K2;
    g.alpha = alpha; g.R = R; g.C = C; g.ldc = ldc; g.c_f32 = c_f32;
    if (workspace && workspace_elems > 0) { g.partial = workspace; g.partial_elems = workspace_elems; }
    GemmNT ga, gb;   // the same column split as the update path makes
    if (gemm_nt_split_columns(g, &ga, &gb)) {
        HIPCHK(launch_gemm_nt(ga, (hipStream_t)hip_stream));
        HIPCHK(launch_gemm_nt(gb, (hipStream_t)hip_stream));
        return TL_OK;
    }
    HIPCHK(launch_gemm_nt(g, (hipStream_t)hip_stream));
    return TL_OK;
}
extern "C" tl_status tl_k_gemm_nt_plan(int32_t M, int32_t N, int32_t K, int32_t K2, size_t workspace_elems, char* name_out,
                                       size_t name_cap, int32_t* n_split_out, int32_t* n_launches_out) {
    KARGS_OK(name_out && name_cap > 0 && M > 0 && N > 0 && K >= 0 && K2 >= 0, "tl_k_gemm_nt_plan");
    GemmNT g;     // dense operands, as tl_k_gemm_nt is called by the tests; only sizes matter to the choice
    g.M = M; g.N = N; g.K = K; g.K2 = K2; g.lda = K; g.ldb = K; g.lda2 = K2; g.ldb2 = K2; g.ldc = N;
    static float dummy;
    if (workspace_elems > 0) { g.partial = &dummy; g.partial_elems = workspace_elems; }
    GemmNT ga, gb;
    int sp = 1;
    const bool two = gemm_nt_split_columns(g, &ga, &gb);
    const char* name = gemm_nt_plan(two ? ga : g, &sp);
    snprintf(name_out, name_cap, "%s", name);
    if (n_split_out) *n_split_out = sp;
    if (n_launches_out) *n_launches_out = two ? 2 : 1;
    return TL_OK;
}
extern "C" tl_status tl_k_gemm_tn(const uint16_t* P, int32_t ldp, const uint16_t* Q, int32_t ldq, int32_t T, int32_t Mo,
                                  int32_t No, float alpha, float* C, int32_t ldc, void* hip_stream) {
    KARGS_OK(P && Q && C && T >= 0 && Mo >= 0 && No >= 0, "tl_k_gemm_tn");
    GemmTN g;
    g.P = P; g.ldp = ldp; g.Q = Q; g.ldq = ldq; g.T = T; g.Mo = Mo; g.No = No; g.alpha = alpha; g.C = C; g.ldc = ldc;
    HIPCHK(launch_gemm_tn(g, (hipStream_t)hip_stream));
    return TL_OK;
}
extern "C" tl_status tl_k_rmsnorm_fwd(const float* h, const float* g, int32_t T, int32_t d, float eps, uint16_t* y,
                                      void* hip_stream) {
    KARGS_OK(h && g && y && T >= 0 && d > 0 && (d & 7) == 0, "tl_k_rmsnorm_fwd");
    HIPCHK(launch_rmsnorm_fwd(h, g, T, d, eps, y, (hipStream_t)hip_stream));
    return TL_OK;
}
extern "C" tl_status tl_k_rmsnorm_bwd(const uint16_t* dy, const float* h, const float* g, const float* dres, int32_t T,
                                      int32_t d, float eps, float* dh_out, uint16_t* dh_out_bf16, void* hip_stream) {
    KARGS_OK(dy && h && g && dh_out && T >= 0 && d > 0 && (d & 7) == 0, "tl_k_rmsnorm_bwd");
    HIPCHK(launch_rmsnorm_bwd(dy, h, g, dres, T, d, eps, dh_out, dh_out_bf16, (hipStream_t)hip_stream));
    return TL_OK;
}
extern "C" tl_status tl_k_rope(uint16_t* x, int32_t ld, int32_t T, int32_t n_heads, int32_t d_head, float base,
                               int32_t pos0, int32_t sign, void* hip_stream) {
    KARGS_OK(x && T >= 0 && n_heads > 0 && d_head >= 4 && (d_head & 3) == 0 && (ld & 1) == 0 && pos0 >= 0, "tl_k_rope");
    HIPCHK(launch_rope(x, ld, T, n_heads, d_head, base, pos0, sign, nullptr, (hipStream_t)hip_stream));
    return TL_OK;
}
extern "C" tl_status tl_k_rope_table(uint16_t* x, int32_t ld, int32_t T, int32_t n_heads, int32_t d_head, float base,
                                     int32_t pos0, int32_t sign, float* table, size_t table_elems, void* hip_stream) {
    KARGS_OK(x && table && T >= 0 && n_heads > 0 && d_head >= 4 && (d_head & 3) == 0 && (ld & 1) == 0 && pos0 >= 0,
             "tl_k_rope_table");
    if (((size_t)table & 15) || table_elems < (size_t)(pos0 + T) * d_head)
        return fail(TL_ERR_SHAPE, "tl_k_rope_table: the table needs (pos0 + T) * d_head floats, 16-byte aligned");
    HIPCHK(launch_rope_table((float2*)table, pos0 + T, d_head, base, (hipStream_t)hip_stream));
    HIPCHK(launch_rope(x, ld, T, n_heads, d_head, base, pos0, sign, (const float2*)table, (hipStream_t)hip_stream));
    return TL_OK;
}
extern "C" tl_status tl_k_dropout(const uint16_t* x, int32_t T, int32_t d_in, float p, uint64_t seed, int64_t step,
                                  int32_t layer, int32_t group, uint16_t* y, void* hip_stream) {
    if (!x || !y) return fail(TL_ERR_ARG, "tl_k_dropout: null pointer");
    if (T < 0 || d_in < 0 || (d_in & 7) || !(p >= 0.f && p < 1.f) || step < 0 || layer < 0 || group < 0 || group > 3)
        return fail(TL_ERR_ARG, "tl_k_dropout: bad argument");
    TLCHK(require_gfx950());
    HIPCHK(launch_dropout_fwd(x, y, (size_t)T * d_in, dropout_key(seed, step, layer, group), p, (hipStream_t)hip_stream));
    return TL_OK;
}

extern "C" tl_status tl_k_swiglu_fwd(const uint16_t* gu, int32_t T, int32_t f, uint16_t* a, void* hip_stream) {
    KARGS_OK(gu && a && T >= 0 && f > 0 && (f & 7) == 0, "tl_k_swiglu_fwd");
    HIPCHK(launch_swiglu_fwd(gu, T, f, a, (hipStream_t)hip_stream));
    return TL_OK;
}
extern "C" tl_status tl_k_gemv(const uint16_t* W, int32_t ldw, const uint16_t* x, int32_t N, int32_t K,
                               const uint16_t* lora_b, const float* lora_h, int32_t r, int32_t rows_per_group, float alpha,
                               const float* resid, void* y, int32_t y_f32, void* hip_stream) {
    KARGS_OK(W && x && y && N >= 0 && K > 0 && (K & 7) == 0 && (ldw & 7) == 0 && (!lora_b || (lora_h && r > 0)) &&
                 (y_f32 || !resid), "tl_k_gemv");
    HIPCHK(launch_gemv(W, ldw, x, N, K, lora_b, lora_h, r, rows_per_group, alpha, resid, y_f32 ? nullptr : (bf16_t*)y,
                       y_f32 ? (float*)y : nullptr, (hipStream_t)hip_stream));
    return TL_OK;
}
extern "C" tl_status tl_k_gemv_pre(const uint16_t* W, int32_t ldw, int32_t N, int32_t K, int32_t mode, const float* h,
                                   const float* gain, float eps, const uint16_t* gu, uint16_t* x_out, float* y,
                                   void* hip_stream) {
    KARGS_OK(W && y && N >= 0 && K > 0 && (K & 7) == 0 && (ldw & 7) == 0 &&
                 ((mode == 1 && h && gain) || (mode == 2 && gu)), "tl_k_gemv_pre");
    GemvPre pre;
    pre.mode = mode; pre.h = h; pre.gain = gain; pre.eps = eps; pre.gu = gu; pre.x_out = x_out;
    HIPCHK(launch_gemv(W, ldw, nullptr, N, K, nullptr, nullptr, 0, 0, 1.f, nullptr, nullptr, y, (hipStream_t)hip_stream,
                       &pre));
    return TL_OK;
}
extern "C" tl_status tl_k_attention_decode(const uint16_t* q, const uint16_t* k, const uint16_t* v, int32_t ld,
                                           int32_t n_keys, int32_t n_heads, int32_t d_head, uint16_t* o,
                                           float* workspace, size_t workspace_elems, void* hip_stream) {
    KARGS_OK(q && k && v && o && n_keys > 0 && n_heads > 0 && (d_head == 64 || d_head == 128) && (ld & 7) == 0,
             "tl_k_attention_decode");
    HIPCHK(launch_attention_decode(q, (bf16_t*)k, v, ld, n_keys, n_heads, d_head, o, workspace, workspace_elems,
                                   (hipStream_t)hip_stream));   // without a RoPE row nothing is written to k
    return TL_OK;
}
extern "C" tl_status tl_k_argmax(const float* x, int32_t n, int32_t* out, void* hip_stream) {
    KARGS_OK(x && out && n > 0, "tl_k_argmax");
    HIPCHK(launch_argmax(x, n, out, (hipStream_t)hip_stream));
    return TL_OK;
}
extern "C" tl_status tl_k_swiglu_bwd(const uint16_t* da, const uint16_t* gu, int32_t T, int32_t f, uint16_t* dgu,
                                     void* hip_stream) {
    KARGS_OK(da && gu && dgu && T >= 0 && f > 0 && (f & 7) == 0, "tl_k_swiglu_bwd");
    HIPCHK(launch_swiglu_bwd(da, gu, T, f, dgu, (hipStream_t)hip_stream));
    return TL_OK;
}
extern "C" tl_status tl_k_attention_fwd(const uint16_t* q, const uint16_t* k, const uint16_t* v, int32_t ldq, int32_t T,
                                        int32_t n_heads, int32_t d_head, uint16_t* o, int32_t ldo, float* lse,
                                        void* hip_stream) {
    KARGS_OK(q && k && v && o && lse && T >= 0 && n_heads > 0 && (d_head == 64 || d_head == 128), "tl_k_attention_fwd");
    HIPCHK(launch_attention_fwd(q, k, v, ldq, T, n_heads, d_head, o, ldo, lse, (hipStream_t)hip_stream));
    return TL_OK;
}
extern "C" tl_status tl_k_attention_bwd(const uint16_t* q, const uint16_t* k, const uint16_t* v, const uint16_t* o,
                                        const uint16_t* d_o, const float* lse, int32_t ldq, int32_t ldo, int32_t T,
                                        int32_t n_heads, int32_t d_head, uint16_t* dq, uint16_t* dk, uint16_t* dv,
                                        float* delta, void* hip_stream) {
    KARGS_OK(q && k && v && o && d_o && lse && dq && dk && dv && delta && T >= 0 && n_heads > 0 &&
                 (d_head == 64 || d_head == 128), "tl_k_attention_bwd");
    HIPCHK(launch_attention_bwd(q, k, v, o, d_o, lse, ldq, ldo, T, n_heads, d_head, dq, dk, dv, delta, nullptr,
                                (hipStream_t)hip_stream));
    return TL_OK;
}
extern "C" tl_status tl_k_cross_entropy(const float* logits, const int32_t* labels, int32_t T, int32_t V,
                                        int32_t first_target, int32_t n_targets, float* nll, uint16_t* dlogits,
                                        float* loss_sum, void* hip_stream) {
    KARGS_OK(logits && labels && nll && T >= 0 && V > 0 && n_targets > 0 && first_target >= 0, "tl_k_cross_entropy");
    HIPCHK(launch_cross_entropy(logits, labels, T, V, first_target, n_targets, nll, dlogits, loss_sum,
                                (hipStream_t)hip_stream));
    return TL_OK;
}
extern "C" tl_status tl_k_adamw(float* p, const float* g, float* m, float* v, uint16_t* shadow, size_t n, int64_t step,
                                float lr, float beta1, float beta2, float eps, float wd, void* hip_stream) {
    KARGS_OK(p && g && m && v && step >= 1, "tl_k_adamw");
    HIPCHK(launch_adamw(p, g, m, v, shadow, n, (long)step, lr, beta1, beta2, eps, wd, (hipStream_t)hip_stream));
    return TL_OK;
}
extern "C" tl_status tl_k_embed(const uint16_t* E, const int32_t* tokens, int32_t T, int32_t d, float* h,
                                void* hip_stream) {
    KARGS_OK(E && tokens && h && T >= 0 && d > 0 && (d & 7) == 0, "tl_k_embed");
    HIPCHK(launch_embed(E, tokens, T, d, h, (hipStream_t)hip_stream));
    return TL_OK;
}
