// Host side of the library: context, workspace layout, weight packing, and the launch schedule of prefill,
// decode step and commit.  No arithmetic of the method happens here; every step of the path is a kernel.
#include <math.h>
#include <stdarg.h>
#include <stdio.h>
#include <string.h>

#include <mutex>
#include <string>
#include <vector>

#include "internal.hpp"
#include "mfma.hpp"

using namespace sdlm;

// Partial-result scratch of sdlm_decode_step_static: split-k slabs, split-KV partial results and the LM head's
// per-vocabulary-block partials (fp32 mode: the logits when the caller does not ask for them).  One copy per GPU,
// held until the process ends; every context on a GPU shares it.  In host code this name is only a handle for
// hipGetSymbolAddress: the device address is looked up once per device and kept in g_static_scratch.
constexpr size_t STATIC_SCRATCH_BYTES = (size_t)32 << 20;
constexpr size_t STATIC_SLAB_BYTES = (size_t)16 << 20, STATIC_ATTN_BYTES = (size_t)12 << 20;
constexpr size_t STATIC_LM_BYTES = STATIC_SCRATCH_BYTES - STATIC_SLAB_BYTES - STATIC_ATTN_BYTES;
static __device__ __align__(256) unsigned char scratch[STATIC_SCRATCH_BYTES];

namespace {

constexpr int MAX_DEVICES = 64;
std::mutex g_static_mu;
void *g_static_scratch[MAX_DEVICES] = {};

// Device address of `scratch` on the current device (looked up on first use, with that device current).
hipError_t static_scratch_of_current_device(void **out)
{
    *out = nullptr;
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    if (dev < 0 || dev >= MAX_DEVICES) return hipErrorInvalidDevice;
    std::lock_guard<std::mutex> lock(g_static_mu);
    if (!g_static_scratch[dev]) {
        void *p = nullptr;
        e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess) return e;
        g_static_scratch[dev] = p;
    }
    *out = g_static_scratch[dev];
    return hipSuccess;
}

struct LayerW {
    void *attn_norm, *wqkv, *bqkv, *wo, *ffn_norm, *w_gate, *w_up, *w_down;   // w_gate: fused gate/up when packed
};

struct Layout {
    size_t total = 0;
    size_t embed, lm_head, final_norm, rope, pool, state_i32, meta_i32;
    std::vector<size_t> layer_off;   // start of each layer's weights
    size_t l_attn_norm, l_wqkv, l_bqkv, l_wo, l_ffn_norm, l_gate, l_up, l_down, l_size;   // offsets inside a layer
    size_t x, xn, qkv, q, att, act, xhat, logits, conf_rows, ids_rows, attn_part, slabs, lm_part;
    size_t slab_floats, attn_bytes;
    int verify_rows;
    int group_rows;
    size_t state_ints, meta_ints;
    int max_rows, max_groups, pages_per_seq, n_pages, pool_tiles, prefill_rows;
    size_t esz;
    bool mfma;
};

size_t align_up(size_t v, size_t a = 256) { return (v + a - 1) / a * a; }

bool validate(const sdlm_model_cfg *m, const sdlm_run_cfg *r, std::string *why)
{
    auto bad = [&](const char *s) { if (why) *why = s; return false; };
    if (!m || !r) return bad("null configuration");
    if (m->n_layers < 1 || m->hidden < 8 || m->ffn < 8 || m->vocab < 2) return bad("bad model sizes");
    if (m->hidden % 4 || m->hidden > 16384) return bad("hidden must be a multiple of 4, at most 16384");
    if (m->n_kv_heads < 1 || m->n_q_heads < 1 || m->n_q_heads % m->n_kv_heads) return bad("n_q_heads must be a multiple of n_kv_heads");
    if (m->head_dim != 32 && m->head_dim != 64 && m->head_dim != 96 && m->head_dim != 128) return bad("head_dim must be 32, 64, 96 or 128");
    if (m->dtype != 0 && m->dtype != 1) return bad("dtype must be 0 (fp32) or 1 (bf16)");
    if (m->mask_token_id < 0 || m->mask_token_id >= m->vocab) return bad("mask_token_id outside the vocabulary");
    if (m->block_causal != 0 && m->block_causal != 1) return bad("block_causal must be 0 or 1");
    if (r->max_batch < 1 || r->max_batch > 1024) return bad("max_batch must be 1..1024");
    if (r->block_D < 1 || r->block_D > MAX_D) return bad("block_D must be 1..16");
    if (r->page_size != PAGE) return bad("page_size must be 16");
    if (r->max_seq_len < r->block_D) return bad("max_seq_len too small");
    if (r->kv_layout != 0 && r->kv_layout != 1) return bad("kv_layout must be 0 or 1");
    if (r->kv_layout == 1 && r->n_pages < 1) return bad("paged layout needs n_pages >= 1");
    if (r->conf_fn != 0 && r->conf_fn != 1) return bad("conf_fn must be 0 or 1");
    if (r->accept_rule != 0 && r->accept_rule != 1) return bad("accept_rule must be 0 or 1");
    if (r->prefill_rows < 0) return bad("prefill_rows must be >= 0");
    return true;
}

void plan(const sdlm_model_cfg *m, const sdlm_run_cfg *r, Layout *L)
{
    const size_t e = m->dtype == 0 ? 4 : 2;
    const size_t h = m->hidden, F = m->ffn, V = m->vocab, d = m->head_dim;
    const size_t nq = (size_t)m->n_q_heads * d, nk = (size_t)m->n_kv_heads * d, nqkv = nq + 2 * nk;
    L->esz = e;
    L->mfma = mfma_supported(m);
    size_t o = 0;
    auto take = [&](size_t bytes) { size_t at = o; o = align_up(o + bytes); return at; };
    L->embed = take(V * h * e);
    L->lm_head = take(mfma_packed_elems(L->mfma, V, h) * e);
    L->final_norm = take(h * e);
    // one layer
    size_t lo = 0;
    auto ltake = [&](size_t bytes) { size_t at = lo; lo = align_up(lo + bytes); return at; };
    L->l_attn_norm = ltake(h * e);
    L->l_wqkv = ltake(mfma_packed_elems(L->mfma, nqkv, h) * e);
    L->l_bqkv = ltake(nqkv * e);
    L->l_wo = ltake(mfma_packed_elems(L->mfma, h, nq) * e);
    L->l_ffn_norm = ltake(h * e);
    if (L->mfma) {
        L->l_gate = ltake(mfma_packed_elems(true, 2 * mfma_pad_n(F), h) * e);   // gate and up interleaved by tile
        L->l_up = L->l_gate;
    } else {
        L->l_gate = ltake(F * h * e);
        L->l_up = ltake(F * h * e);
    }
    L->l_down = ltake(mfma_packed_elems(L->mfma, h, F) * e);
    L->l_size = lo;
    L->layer_off.resize(m->n_layers);
    for (int l = 0; l < m->n_layers; ++l) L->layer_off[l] = take(L->l_size);
    const int max_pos = r->max_seq_len + 2 * r->block_D;   // a verification input reaches position n + 2D - 3
    L->rope = take((size_t)max_pos * (d / 2) * sizeof(float2));
    L->pages_per_seq = (r->max_seq_len + PAGE - 1) / PAGE;
    L->n_pages = r->kv_layout == 0 ? r->max_batch * L->pages_per_seq : r->n_pages;
    L->pool_tiles = L->n_pages + r->max_batch * (r->block_D + 1);   // pages, then per sequence: the step's staging tile, one per verification input, one for their shared causal rows
    L->pool = take((size_t)m->n_layers * L->pool_tiles * m->n_kv_heads * 2 * PAGE * d * e);
    const int B = r->max_batch, D = r->block_D;
    int pre = r->prefill_rows > 0 ? r->prefill_rows : 4096;   // measured on the 7B shape: 2048 rows/pass 66k tokens/s, 4096 72k, 8192 73k
    L->prefill_rows = pre;
    L->verify_rows = B * verify_rows_per_seq(D, nullptr);
    L->max_rows = B * 2 * D > pre ? B * 2 * D : pre;
    if (L->verify_rows > L->max_rows) L->max_rows = L->verify_rows;
    L->max_rows = (L->max_rows + 63) / 64 * 64;
    L->max_groups = L->max_rows;   // worst case: every row its own group (prefill of many 1-token prompts)
    L->state_ints = (size_t)B * 3 + (size_t)B * D + (size_t)B * L->pages_per_seq + B + 4 + (size_t)B * D + B;
    L->state_i32 = take(L->state_ints * 4);
    L->meta_ints = (size_t)L->max_rows * 8 + (size_t)L->max_groups * 6 + (size_t)B * D + 4;
    L->meta_i32 = take(L->meta_ints * 4);
    const size_t R = L->max_rows;
    L->x = take(R * h * 4);
    L->xn = take(R * h * e);
    L->qkv = take(R * nqkv * 4);
    L->q = take(R * nq * e);
    L->att = take(R * nq * e);
    L->act = take(R * F * e);
    L->xhat = take((size_t)B * D * h * e);
    L->logits = take(L->mfma ? 256 : (size_t)B * D * V * 4);
    L->conf_rows = take((size_t)B * D * 4);
    L->ids_rows = take((size_t)B * D * 4);
    L->attn_bytes = L->mfma ? mfma_attn_scratch_bytes(m, r, L->max_rows) : 256;
    L->attn_part = take(L->attn_bytes);
    L->slab_floats = L->mfma ? ((size_t)16 << 20) : 64;                      // 64 MB of split-k slabs
    L->slabs = take(L->slab_floats * 4);
    L->lm_part = take(L->mfma ? mfma_lm_scratch_bytes(m->vocab, B * D) : 256);
    L->group_rows = L->mfma ? mfma_group_rows(m) : GROUP_ROWS;
    L->total = o;
}

struct Tap { int layer, which; void *dst; };

}  // namespace

struct sdlm_ctx {
    sdlm_model_cfg m;
    sdlm_run_cfg r;
    Layout L;
    hipStream_t stream;
    char *ws;
    std::string err;
    std::vector<LayerW> lw;
    void *embed, *lm_head, *final_norm;
    float2 *rope;
    char *pool;
    KvGeom kg;
    SeqState st;
    RowMeta rm;
    float *x, *qkv, *logits, *conf_rows;
    void *xn, *q, *att, *act, *xhat, *attn_part, *lm_part;
    float *slabs;
    int32_t *ids_rows;
    int batch = 0;
    int pend_slabs = 0;                  // split-k slabs of the last residual projection not yet added to x
    size_t pend_stride = 0;
    bool prefilled = false, stepped = false;
    bool committed = false;              // a commit has happened since the prefill: every sequence has >= 1 pending row
    std::vector<int32_t> n_ub;           // host upper bound of n_b
    std::vector<int32_t> n_host;         // landing buffer of refresh_lengths (sized once, so that a step allocates nothing)
    char *static_scratch = nullptr;      // this GPU's copy of the library-owned scratch array (sdlm_decode_step_static)
    std::string static_err;              // why static_scratch is missing
    bool no_events = false;              // a call that must not create HIP events is running
    std::vector<Tap> taps;
    // graph replay of the decode step (opt-in): the launch sequence of a step is fixed once the batch is, all sizes
    // that vary from step to step live in device memory
    bool graph_on = false;
    hipGraphExec_t graph_exec = nullptr;
    void *graph_key[4] = {nullptr, nullptr, nullptr, nullptr};   // the output pointers baked into the captured launches
    // profiling
    uint32_t prof = 0;                   // bit p: phase p is bracketed by events
    uint32_t prof_every = 1;             // ... on every prof_every-th launch of the phase
    uint32_t prof_seen[SDLM_N_PHASES] = {};
    std::vector<hipEvent_t> ev;          // pairs
    std::vector<int> ev_phase;
    size_t ev_used = 0;
    std::string info;
};

namespace {

int fail(sdlm_ctx *c, int code, const char *fmt, ...)
{
    char buf[512];
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(buf, sizeof buf, fmt, ap);
    va_end(ap);
    if (c) c->err = buf;
    return code;
}

#define HIPCHK(c, call)                                                                             \
    do {                                                                                            \
        hipError_t e_ = (call);                                                                     \
        if (e_ != hipSuccess) return fail(c, SDLM_EHIP, "%s: %s", #call, hipGetErrorString(e_));    \
    } while (0)

struct Phase {
    sdlm_ctx *c;
    size_t idx = (size_t)-1;
    Phase(sdlm_ctx *c_, int ph) : c(c_)
    {
        if (!((c->prof >> ph) & 1u) || c->no_events) return;
        if (c->prof_seen[ph]++ % c->prof_every != 0) return;
        if (c->ev_used + 2 > c->ev.size()) {
            hipEvent_t a, b;
            if (hipEventCreate(&a) != hipSuccess || hipEventCreate(&b) != hipSuccess) return;
            c->ev.push_back(a); c->ev.push_back(b);
            c->ev_phase.push_back(ph);
        }
        idx = c->ev_used;
        c->ev_phase[idx / 2] = ph;
        c->ev_used += 2;
        (void)hipEventRecord(c->ev[idx], c->stream);
    }
    ~Phase()
    {
        if (idx != (size_t)-1) (void)hipEventRecord(c->ev[idx + 1], c->stream);
    }
};

void run_taps(sdlm_ctx *c, int layer, int which, const void *src, size_t bytes)
{
    for (auto &t : c->taps)
        if (t.which == which && (which == 4 || t.layer == layer))
            (void)hipMemcpyAsync(t.dst, src, bytes, hipMemcpyDeviceToDevice, c->stream);
}

// The decoder layers over the rows described by c->rm.  `rows` bounds the launch grids (the device-side row
// count decides what is computed); `rows_sure` is a host-known lower bound of that count (it only steers launch shapes).
// `cache_only`: the pass only has to leave its rows' K/V in the cache (prefill): the last layer then ends after the K/V placement.
void run_layers(sdlm_ctx *c, int rows, int groups, int rows_sure, bool cache_only, bool two_staging = false)
{
    const sdlm_model_cfg &m = c->m;
    const int dt = m.dtype, h = m.hidden, F = m.ffn, d = m.head_dim;
    const int nq = m.n_q_heads * d, nk = m.n_kv_heads * d, nqkv = nq + 2 * nk;
    const size_t e = c->L.esz;
    hipStream_t s = c->stream;
    c->pend_slabs = 0;   // a fresh residual stream: nothing pending from an earlier pass
    { Phase p(c, SDLM_PH_ROWS); launch_embed(s, dt, c->x, c->embed, c->rm, rows, h, m.vocab); }
    for (int l = 0; l < m.n_layers; ++l) {
        const LayerW &w = c->lw[l];
        char *pool_l = c->pool + (size_t)l * c->kg.layer_stride * e;
        run_taps(c, l, 0, c->x, (size_t)rows * h * 4);
        { Phase p(c, SDLM_PH_NORM); launch_rmsnorm(s, dt, c->xn, c->x, w.attn_norm, h, m.rms_eps, nullptr, c->rm.counts, rows, rows_sure, c->slabs, c->pend_slabs, c->pend_stride); c->pend_slabs = 0; }
        if (c->L.mfma && qkv_rope_skinny_applies(&m, rows)) {
            Phase p(c, SDLM_PH_QKV);   // projection, rotation and K/V placement in one launch
            launch_qkv_rope_skinny(s, &m, c->xn, w.wqkv, m.has_qkv_bias ? w.bqkv : nullptr, c->rm.counts, rows, c->q, pool_l, c->kg, c->rm, c->st, c->rope);
        } else {
            int qkv_slabs = 1;
            {
                Phase p(c, SDLM_PH_QKV);
                GemmArgs a{c->xn, w.wqkv, nullptr, m.has_qkv_bias ? w.bqkv : nullptr, c->qkv, nullptr, c->rm.counts, rows, nqkv, h, 1.f, rows_sure};
                if (c->L.mfma) qkv_slabs = launch_gemm_mfma(s, EPI_STORE_F32, a, c->slabs, c->L.slab_floats, false); else launch_gemm_generic(s, dt, EPI_STORE_F32, a);
            }
            {
                Phase p(c, SDLM_PH_ROPE);
                launch_rope_scatter(s, dt, qkv_slabs > 1 ? c->slabs : c->qkv, qkv_slabs, (size_t)rows * nqkv, c->q, pool_l, c->kg, c->rm, c->st, c->rope, m.n_q_heads, rows, rows_sure);
            }
        }
        run_taps(c, l, 5, c->q, (size_t)rows * nq * e);
        if (cache_only && l == m.n_layers - 1 && c->taps.empty()) break;   // nothing downstream of the last layer's K/V is used
        bool merge = false;
        {
            Phase p(c, SDLM_PH_ATTN);
            if (c->L.mfma) merge = launch_attn_mfma(s, &c->m, c->r.max_seq_len, c->q, c->att, pool_l, c->kg, c->rm, c->st, c->r.block_D, groups, c->attn_part, c->L.attn_bytes, 0, two_staging);
            else launch_attn_generic(s, dt, c->q, c->att, pool_l, c->kg, c->rm, c->st, m.n_q_heads, rows);
        }
        if (merge) {
            Phase p(c, SDLM_PH_ATTN_MERGE);
            launch_attn_mfma(s, &c->m, c->r.max_seq_len, c->q, c->att, pool_l, c->kg, c->rm, c->st, c->r.block_D, groups, c->attn_part, c->L.attn_bytes, 1, two_staging);
        }
        run_taps(c, l, 1, c->att, (size_t)rows * nq * e);
        {
            Phase p(c, SDLM_PH_OPROJ);
            GemmArgs a{c->att, w.wo, nullptr, nullptr, c->x, nullptr, c->rm.counts, rows, h, nq, 1.f, rows_sure};
            if (c->L.mfma) {
                // the split-k partial sums of a residual projection are added by the next RMSNorm (unless a tap wants x now)
                int sp = launch_gemm_mfma(s, EPI_RESID, a, c->slabs, c->L.slab_floats, c->taps.empty());
                if (sp > 1 && c->taps.empty()) { c->pend_slabs = sp; c->pend_stride = (size_t)rows * h; }
            } else launch_gemm_generic(s, dt, EPI_RESID, a);
        }
        run_taps(c, l, 6, c->x, (size_t)rows * h * 4);
        { Phase p(c, SDLM_PH_NORM); launch_rmsnorm(s, dt, c->xn, c->x, w.ffn_norm, h, m.rms_eps, nullptr, c->rm.counts, rows, rows_sure, c->slabs, c->pend_slabs, c->pend_stride); c->pend_slabs = 0; }
        {
            Phase p(c, SDLM_PH_GATEUP);
            GemmArgs a{c->xn, w.w_gate, w.w_up, nullptr, nullptr, c->act, c->rm.counts, rows, F, h, 1.f, rows_sure};
            if (c->L.mfma) launch_gemm_mfma(s, EPI_SWIGLU, a, c->slabs, c->L.slab_floats, false); else launch_gemm_generic(s, dt, EPI_SWIGLU, a);
        }
        run_taps(c, l, 2, c->act, (size_t)rows * F * e);
        {
            Phase p(c, SDLM_PH_DOWN);
            GemmArgs a{c->act, w.w_down, nullptr, nullptr, c->x, nullptr, c->rm.counts, rows, h, F, 1.f, rows_sure};
            if (c->L.mfma) {
                // the split-k partial sums of a residual projection are added by the next RMSNorm (unless a tap wants x now)
                int sp = launch_gemm_mfma(s, EPI_RESID, a, c->slabs, c->L.slab_floats, c->taps.empty());
                if (sp > 1 && c->taps.empty()) { c->pend_slabs = sp; c->pend_stride = (size_t)rows * h; }
            } else launch_gemm_generic(s, dt, EPI_RESID, a);
        }
        run_taps(c, l, 3, c->x, (size_t)rows * h * 4);
    }
}

// Final RMSNorm of the rows listed in rm.blk_row, LM head, per-row arg-max and confidence (-> ids_rows, conf_rows).
void run_lm_head(sdlm_ctx *c, int lm_rows, float *logits)
{
    hipStream_t s = c->stream;
    const int dt = c->m.dtype, h = c->m.hidden, V = c->m.vocab;
    { Phase p(c, SDLM_PH_NORM); launch_rmsnorm(s, dt, c->xhat, c->x, c->final_norm, h, c->m.rms_eps, c->rm.blk_row, c->rm.counts + 2, lm_rows, lm_rows, c->slabs, c->pend_slabs, c->pend_stride); c->pend_slabs = 0; }
    run_taps(c, 0, 4, c->xhat, (size_t)lm_rows * h * c->L.esz);
    {
        Phase p(c, SDLM_PH_LMHEAD);
        if (c->L.mfma) {
            launch_lmhead_mfma(s, c->xhat, c->lm_head, c->rm.counts + 2, lm_rows, lm_rows, V, h, c->m.logit_scale, c->r.conf_fn, logits, c->lm_part,
                               c->ids_rows, c->conf_rows);
        } else {
            float *z = logits ? logits : c->logits;
            GemmArgs a{c->xhat, c->lm_head, nullptr, nullptr, z, nullptr, c->rm.counts + 2, lm_rows, V, h, c->m.logit_scale};
            launch_gemm_generic(s, dt, EPI_LOGITS, a);
            launch_lm_reduce(s, z, V, c->ids_rows, c->conf_rows, c->r.conf_fn, c->rm.counts + 2, lm_rows);
        }
    }
}

void drop_graph(sdlm_ctx *c)
{
    if (c->graph_exec) (void)hipGraphExecDestroy(c->graph_exec);
    c->graph_exec = nullptr;
}

int refresh_lengths(sdlm_ctx *c, int32_t *flags_out)
{
    std::vector<int32_t> &n = c->n_host;
    int32_t al[2];
    HIPCHK(c, hipMemcpyAsync(n.data(), c->st.n, sizeof(int32_t) * c->batch, hipMemcpyDeviceToHost, c->stream));
    HIPCHK(c, hipMemcpyAsync(al, c->st.alloc, sizeof al, hipMemcpyDeviceToHost, c->stream));
    HIPCHK(c, hipStreamSynchronize(c->stream));
    for (int b = 0; b < c->batch; ++b) c->n_ub[b] = n[b];
    if (flags_out) *flags_out = al[1];
    return SDLM_OK;
}

}  // namespace

extern "C" {

size_t sdlm_workspace_bytes(const sdlm_model_cfg *m, const sdlm_run_cfg *r)
{
    if (!validate(m, r, nullptr)) return 0;
    Layout L;
    plan(m, r, &L);
    return L.total;
}

int sdlm_create(const sdlm_model_cfg *m, const sdlm_run_cfg *r, void *workspace, size_t bytes, void *hip_stream, sdlm_ctx **out)
{
    if (!out) return SDLM_EINVAL;
    *out = nullptr;
    std::string why;
    sdlm_ctx *c = new sdlm_ctx();
    *out = c;   // returned even on failure so that sdlm_last_error can be read; destroy it in either case
    if (!validate(m, r, &why)) return fail(c, SDLM_EINVAL, "%s", why.c_str());
    c->m = *m; c->r = *r;
    plan(m, r, &c->L);
    const Layout &L = c->L;
    if (!workspace || ((uintptr_t)workspace & 255)) return fail(c, SDLM_EINVAL, "workspace must be a 256-byte aligned device pointer");
    if (bytes < L.total) return fail(c, SDLM_ECAPACITY, "workspace has %zu bytes, %zu needed", bytes, L.total);
    c->stream = (hipStream_t)hip_stream;
    c->ws = (char *)workspace;
    char *ws = c->ws;
    c->embed = ws + L.embed; c->lm_head = ws + L.lm_head; c->final_norm = ws + L.final_norm;
    c->lw.resize(m->n_layers);
    for (int l = 0; l < m->n_layers; ++l) {
        char *b = ws + L.layer_off[l];
        c->lw[l] = LayerW{b + L.l_attn_norm, b + L.l_wqkv, b + L.l_bqkv, b + L.l_wo, b + L.l_ffn_norm, b + L.l_gate, b + L.l_up, b + L.l_down};
    }
    c->rope = (float2 *)(ws + L.rope);
    c->pool = ws + L.pool;
    c->kg.n_kv_heads = m->n_kv_heads; c->kg.head_dim = m->head_dim; c->kg.pages_per_seq = L.pages_per_seq;
    c->kg.staging_base = L.n_pages;
    c->kg.layer_stride = (size_t)L.pool_tiles * m->n_kv_heads * 2 * PAGE * m->head_dim;
    const int B = r->max_batch, D = r->block_D;
    int32_t *si = (int32_t *)(ws + L.state_i32);
    c->st.n = si; si += B; c->st.c = si; si += B; c->st.last_tok = si; si += B;
    c->st.pend_tok = si; si += (size_t)B * D;
    c->st.page_table = si; si += (size_t)B * L.pages_per_seq;
    c->st.pages_backed = si; si += B;
    c->st.alloc = si; si += 4;
    c->st.last_ids = si; si += (size_t)B * D;
    c->st.last_count = si; si += B;
    int32_t *mi = (int32_t *)(ws + L.meta_i32);
    c->rm.tok = mi; mi += L.max_rows; c->rm.pos = mi; mi += L.max_rows; c->rm.seq = mi; mi += L.max_rows;
    c->rm.kind = mi; mi += L.max_rows; c->rm.lim = mi; mi += L.max_rows;
    c->rm.stg = mi; mi += L.max_rows; c->rm.smask = mi; mi += L.max_rows; c->rm.stg2 = mi; mi += L.max_rows;
    c->rm.grp_row0 = mi; mi += L.max_groups; c->rm.grp_n = mi; mi += L.max_groups; c->rm.grp_seq = mi; mi += L.max_groups;
    c->rm.grp_stg = mi; mi += L.max_groups; c->rm.grp_stg2 = mi; mi += L.max_groups; c->rm.grp_hint = mi; mi += L.max_groups;
    c->rm.blk_row = mi; mi += (size_t)B * D;
    c->rm.counts = mi; mi += 4;
    c->x = (float *)(ws + L.x); c->xn = ws + L.xn; c->qkv = (float *)(ws + L.qkv); c->q = ws + L.q; c->att = ws + L.att;
    c->act = ws + L.act; c->xhat = ws + L.xhat; c->logits = (float *)(ws + L.logits);
    c->conf_rows = (float *)(ws + L.conf_rows); c->ids_rows = (int32_t *)(ws + L.ids_rows);
    c->attn_part = ws + L.attn_part; c->slabs = (float *)(ws + L.slabs); c->lm_part = ws + L.lm_part;
    c->n_ub.assign(B, 0);
    c->n_host.assign(B, 0);
    {
        void *p = nullptr;
        hipError_t e = static_scratch_of_current_device(&p);
        if (e == hipSuccess) c->static_scratch = (char *)p;
        else c->static_err = std::string("hipGetSymbolAddress(scratch): ") + hipGetErrorString(e);
        (void)hipGetLastError();   // the step's other entry points do not depend on it
    }
    c->info = L.mfma ? "mfma-bf16" : (m->dtype == 0 ? "generic-fp32" : "generic-bf16");
    // rotary table: (cos, sin)(pos * theta^(-2i/d)), evaluated in double on the host
    const int half = m->head_dim / 2, max_pos = r->max_seq_len + 2 * D;
    std::vector<float2> tab((size_t)max_pos * half);
    for (int i = 0; i < half; ++i) {
        double w = pow((double)m->rope_theta, -2.0 * i / m->head_dim);
        for (int p = 0; p < max_pos; ++p) tab[(size_t)p * half + i] = make_float2((float)cos(p * w), (float)sin(p * w));
    }
    HIPCHK(c, hipMemcpyAsync(c->rope, tab.data(), tab.size() * sizeof(float2), hipMemcpyHostToDevice, c->stream));
    // The K/V pool starts at zero: masked keys contribute weight 0 to the weighted sum of values, and 0 times a stale
    // non-finite bit pattern would not be 0.  Slots are only ever overwritten with finite K/V afterwards.
    HIPCHK(c, hipMemsetAsync(c->pool, 0, (size_t)m->n_layers * c->kg.layer_stride * L.esz, c->stream));
    HIPCHK(c, hipMemsetAsync(ws + L.state_i32, 0, L.state_ints * 4, c->stream));
    HIPCHK(c, hipMemsetAsync(ws + L.meta_i32, 0, L.meta_ints * 4, c->stream));
    HIPCHK(c, hipStreamSynchronize(c->stream));
    return SDLM_OK;
}

int sdlm_init_weights(sdlm_ctx *c, const sdlm_weights *w, int32_t on_device)
{
    if (!c || !w) return SDLM_EINVAL;
    const sdlm_model_cfg &m = c->m;
    const size_t e = c->L.esz, h = m.hidden, F = m.ffn, V = m.vocab, d = m.head_dim;
    const size_t nq = m.n_q_heads * d, nk = m.n_kv_heads * d;
    const bool mf = c->L.mfma;
    hipMemcpyKind kind = on_device ? hipMemcpyDeviceToDevice : hipMemcpyHostToDevice;
    std::vector<void *> staged;   // device staging of host matrices that need repacking
    auto copy = [&](void *dst, const void *src, size_t bytes) -> hipError_t {
        return hipMemcpyAsync(dst, src, bytes, kind, c->stream);
    };
    // a [N,K] matrix (rows n0.. of the packed destination): plain copy, or tile repack for the matrix-core path
    auto put_matrix = [&](void *dst, const void *src, size_t N, size_t K, size_t dst_row0, size_t dst_rows, int interleave) -> int {
        if (!mf) {
            HIPCHK(c, copy((char *)dst + dst_row0 * K * e, src, N * K * e));
            return SDLM_OK;
        }
        const void *dsrc = src;
        if (!on_device) {
            void *tmp = nullptr;
            // host sources are staged in the activation area of the workspace, one matrix at a time
            size_t room = c->L.total - c->L.x;
            if (N * K * e > room) return fail(c, SDLM_ECAPACITY, "host-side weights need on_device staging space");
            tmp = c->ws + c->L.x;
            HIPCHK(c, hipMemcpyAsync(tmp, src, N * K * e, hipMemcpyHostToDevice, c->stream));
            dsrc = tmp;
        }
        launch_pack_mfma(c->stream, dst, dsrc, (int)N, (int)K, (int)dst_row0, (int)dst_rows, interleave);
        if (!on_device) HIPCHK(c, hipStreamSynchronize(c->stream));
        return SDLM_OK;
    };
    int rc;
    if (w->embed) HIPCHK(c, copy(c->embed, w->embed, V * h * e));
    if (w->lm_head && (rc = put_matrix(c->lm_head, w->lm_head, V, h, 0, V, 0))) return rc;
    if (w->final_norm) HIPCHK(c, copy(c->final_norm, w->final_norm, h * e));
    for (int l = 0; l < m.n_layers; ++l) {
        LayerW &lw = c->lw[l];
        auto get = [&](const void *const *arr) -> const void * { return arr ? arr[l] : nullptr; };
        if (get(w->attn_norm)) HIPCHK(c, copy(lw.attn_norm, get(w->attn_norm), h * e));
        if (get(w->ffn_norm)) HIPCHK(c, copy(lw.ffn_norm, get(w->ffn_norm), h * e));
        const size_t nqkv = nq + 2 * nk;
        if (get(w->wq) && (rc = put_matrix(lw.wqkv, get(w->wq), nq, h, 0, nqkv, 0))) return rc;
        if (get(w->wk) && (rc = put_matrix(lw.wqkv, get(w->wk), nk, h, nq, nqkv, 0))) return rc;
        if (get(w->wv) && (rc = put_matrix(lw.wqkv, get(w->wv), nk, h, nq + nk, nqkv, 0))) return rc;
        if (m.has_qkv_bias) {
            if (get(w->bq)) HIPCHK(c, copy(lw.bqkv, get(w->bq), nq * e));
            if (get(w->bk)) HIPCHK(c, copy((char *)lw.bqkv + nq * e, get(w->bk), nk * e));
            if (get(w->bv)) HIPCHK(c, copy((char *)lw.bqkv + (nq + nk) * e, get(w->bv), nk * e));
        }
        if (get(w->wo) && (rc = put_matrix(lw.wo, get(w->wo), h, nq, 0, h, 0))) return rc;
        if (mf) {
            if (get(w->w_gate) && (rc = put_matrix(lw.w_gate, get(w->w_gate), F, h, 0, 2 * mfma_pad_n(F), 1))) return rc;
            if (get(w->w_up) && (rc = put_matrix(lw.w_gate, get(w->w_up), F, h, 0, 2 * mfma_pad_n(F), 2))) return rc;
        } else {
            if (get(w->w_gate) && (rc = put_matrix(lw.w_gate, get(w->w_gate), F, h, 0, F, 0))) return rc;
            if (get(w->w_up) && (rc = put_matrix(lw.w_up, get(w->w_up), F, h, 0, F, 0))) return rc;
        }
        if (get(w->w_down) && (rc = put_matrix(lw.w_down, get(w->w_down), h, F, 0, h, 0))) return rc;
    }
    if (!on_device) HIPCHK(c, hipStreamSynchronize(c->stream));
    return SDLM_OK;
}

int sdlm_prefill(sdlm_ctx *c, int32_t batch, const int32_t *ids, const int32_t *offsets)
{
    if (!c || !ids || !offsets) return SDLM_EINVAL;
    const int D = c->r.block_D, pps = c->L.pages_per_seq;
    if (batch < 1 || batch > c->r.max_batch) return fail(c, SDLM_EINVAL, "batch %d outside 1..%d", batch, c->r.max_batch);
    long pages_needed = 0;
    for (int b = 0; b < batch; ++b) {
        int len = offsets[b + 1] - offsets[b];
        if (len < 1) return fail(c, SDLM_EINVAL, "prompt %d is empty", b);
        if (len + D > c->r.max_seq_len) return fail(c, SDLM_ECAPACITY, "prompt %d: %d tokens + a block of %d exceed max_seq_len %d", b, len, D, c->r.max_seq_len);
        for (int i = offsets[b]; i < offsets[b + 1]; ++i)
            if (ids[i] < 0 || ids[i] >= c->m.vocab) return fail(c, SDLM_EINVAL, "token id %d outside the vocabulary", ids[i]);
        pages_needed += (len + PAGE - 1) / PAGE;
    }
    if (c->r.kv_layout == 1 && pages_needed > c->L.n_pages)
        return fail(c, SDLM_ECAPACITY, "prompts need %ld pages, the pool has %d", pages_needed, c->L.n_pages);
    c->batch = batch;
    c->prefilled = false; c->stepped = false; c->committed = false;
    drop_graph(c);   // the batch size is baked into the captured launches
    // sequence state
    const int B = c->r.max_batch;
    std::vector<int32_t> n(B, 0), last(B, 0), table((size_t)B * pps, -1), backed(B, 0);
    int32_t next = 0;
    for (int b = 0; b < batch; ++b) {
        int len = offsets[b + 1] - offsets[b];
        n[b] = len; last[b] = ids[offsets[b + 1] - 1];
        c->n_ub[b] = len;
        if (c->r.kv_layout == 0) {
            for (int j = 0; j < pps; ++j) table[(size_t)b * pps + j] = b * pps + j;
            backed[b] = pps;
        } else {
            int np = (len + PAGE - 1) / PAGE;
            for (int j = 0; j < np; ++j) table[(size_t)b * pps + j] = next++;
            backed[b] = np;
        }
    }
    int32_t al[4] = {next, 0, 0, 0};
    hipStream_t s = c->stream;
    HIPCHK(c, hipMemcpyAsync(c->st.n, n.data(), B * 4, hipMemcpyHostToDevice, s));
    HIPCHK(c, hipMemcpyAsync(c->st.c, n.data(), B * 4, hipMemcpyHostToDevice, s));
    HIPCHK(c, hipMemcpyAsync(c->st.last_tok, last.data(), B * 4, hipMemcpyHostToDevice, s));
    HIPCHK(c, hipMemcpyAsync(c->st.page_table, table.data(), table.size() * 4, hipMemcpyHostToDevice, s));
    HIPCHK(c, hipMemcpyAsync(c->st.pages_backed, backed.data(), B * 4, hipMemcpyHostToDevice, s));
    HIPCHK(c, hipMemcpyAsync(c->st.alloc, al, sizeof al, hipMemcpyHostToDevice, s));
    HIPCHK(c, hipStreamSynchronize(s));
    // causal passes over the prompts, prefill_rows rows at a time
    const int cap = c->L.prefill_rows;
    std::vector<int32_t> tok, pos, seq, kind, lim, g0, gn, gs, gh;
    auto flush = [&]() -> int {
        if (tok.empty()) return SDLM_OK;
        int R = (int)tok.size();
        for (int r0 = 0; r0 < R;) {   // groups: runs of <= group_rows rows of one sequence
            int r1 = r0 + 1;
            while (r1 < R && r1 - r0 < c->L.group_rows && seq[r1] == seq[r0]) ++r1;
            g0.push_back(r0); gn.push_back(r1 - r0); gs.push_back(seq[r0]);
            r0 = r1;
        }
        int32_t counts[4] = {R, (int32_t)g0.size(), 0, c->L.mfma ? mfma_attn_chunk_floor(&c->m, c->r.max_seq_len, (int)g0.size(), c->L.attn_bytes) : 0};
        for (size_t g = 0; g < g0.size(); ++g)   // causal rows: the group's last row sees the most keys
            gh.push_back(attn_group_hint(lim[g0[g] + gn[g] - 1], gn[g], counts[3] > 0 ? counts[3] : 1));
        const std::vector<int32_t> none((size_t)R, -1), zero((size_t)R, 0);   // causal rows: no staging tile
        HIPCHK(c, hipMemcpyAsync(c->rm.stg, none.data(), R * 4, hipMemcpyHostToDevice, s));
        HIPCHK(c, hipMemcpyAsync(c->rm.stg2, none.data(), R * 4, hipMemcpyHostToDevice, s));
        HIPCHK(c, hipMemcpyAsync(c->rm.grp_stg2, none.data(), g0.size() * 4, hipMemcpyHostToDevice, s));
        HIPCHK(c, hipMemcpyAsync(c->rm.smask, zero.data(), R * 4, hipMemcpyHostToDevice, s));
        HIPCHK(c, hipMemcpyAsync(c->rm.grp_stg, none.data(), g0.size() * 4, hipMemcpyHostToDevice, s));
        HIPCHK(c, hipMemcpyAsync(c->rm.tok, tok.data(), R * 4, hipMemcpyHostToDevice, s));
        HIPCHK(c, hipMemcpyAsync(c->rm.pos, pos.data(), R * 4, hipMemcpyHostToDevice, s));
        HIPCHK(c, hipMemcpyAsync(c->rm.seq, seq.data(), R * 4, hipMemcpyHostToDevice, s));
        HIPCHK(c, hipMemcpyAsync(c->rm.kind, kind.data(), R * 4, hipMemcpyHostToDevice, s));
        HIPCHK(c, hipMemcpyAsync(c->rm.lim, lim.data(), R * 4, hipMemcpyHostToDevice, s));
        HIPCHK(c, hipMemcpyAsync(c->rm.grp_row0, g0.data(), g0.size() * 4, hipMemcpyHostToDevice, s));
        HIPCHK(c, hipMemcpyAsync(c->rm.grp_n, gn.data(), gn.size() * 4, hipMemcpyHostToDevice, s));
        HIPCHK(c, hipMemcpyAsync(c->rm.grp_seq, gs.data(), gs.size() * 4, hipMemcpyHostToDevice, s));
        HIPCHK(c, hipMemcpyAsync(c->rm.grp_hint, gh.data(), gh.size() * 4, hipMemcpyHostToDevice, s));
        HIPCHK(c, hipMemcpyAsync(c->rm.counts, counts, sizeof counts, hipMemcpyHostToDevice, s));
        run_layers(c, R, (int)g0.size(), R, true);
        HIPCHK(c, hipStreamSynchronize(s));   // the host vectors are reused
        tok.clear(); pos.clear(); seq.clear(); kind.clear(); lim.clear(); g0.clear(); gn.clear(); gs.clear(); gh.clear();
        return SDLM_OK;
    };
    for (int b = 0; b < batch; ++b)
        for (int i = offsets[b]; i < offsets[b + 1]; ++i) {
            int p = i - offsets[b];
            tok.push_back(ids[i]); pos.push_back(p); seq.push_back(b); kind.push_back(-1); lim.push_back(p + 1);
            if ((int)tok.size() == cap) { int rc = flush(); if (rc) return rc; }
        }
    int rc = flush();
    if (rc) return rc;
    HIPCHK(c, hipGetLastError());
    c->prefilled = true;
    return SDLM_OK;
}

static int decode_step_impl(sdlm_ctx *c, int32_t *ids, int32_t *count, float *conf, float *logits, bool eager_only)
{
    if (!c) return SDLM_EINVAL;
    if (!c->prefilled) return fail(c, SDLM_ESTATE, "decode_step before prefill");
    if (!ids || !count) return fail(c, SDLM_EINVAL, "ids and count outputs are required");
    const int B = c->batch, D = c->r.block_D;
    // A step may accept all D tokens, and the commit must then be able to hold n + D known tokens: the step is refused
    // unless n + D <= max_seq_len, so that no commit can run out of positions (or of page-table entries) on the device.
    bool tight = false;
    for (int b = 0; b < B; ++b) tight |= c->n_ub[b] + D > c->r.max_seq_len;
    if (tight) {
        int32_t flags = 0;
        int rc = refresh_lengths(c, &flags);
        if (rc) return rc;
        if (flags & 1) return fail(c, SDLM_ECAPACITY, "a sequence could not grow at the last commit: page pool exhausted");
        for (int b = 0; b < B; ++b)
            if (c->n_ub[b] + D > c->r.max_seq_len)
                return fail(c, SDLM_ECAPACITY, "sequence %d: %d tokens + a block of %d exceed max_seq_len %d", b, c->n_ub[b], D, c->r.max_seq_len);
    }
    hipStream_t s = c->stream;
    auto launch_all = [&]() {
        const int rows = B * 2 * D, groups = B * ((2 * D + c->L.group_rows - 1) / c->L.group_rows);
        const int cp_floor = c->L.mfma ? mfma_attn_chunk_floor(&c->m, c->r.max_seq_len, groups, c->L.attn_bytes) : 0;
        { Phase p(c, SDLM_PH_ROWS); launch_assemble_decode(s, c->st, c->rm, B, D, c->m.mask_token_id, c->L.group_rows, c->kg.staging_base, c->m.block_causal, c->m.n_kv_heads, cp_floor); }
        run_layers(c, rows, groups, B * (D + (c->committed ? 1 : 0)), false);   // after a commit every sequence has >= 1 pending row
        run_lm_head(c, B * D, logits);
        { Phase p(c, SDLM_PH_ACCEPT); launch_accept(s, c->st, c->ids_rows, c->conf_rows, B, D, c->r.tau, c->r.accept_rule, ids, count, conf); }
    };
    if (c->graph_on && c->prof == 0 && c->taps.empty() && !eager_only) {
        void *key[4] = {ids, count, conf, logits};
        if (!c->graph_exec || memcmp(key, c->graph_key, sizeof key) != 0) {
            drop_graph(c);
            hipGraph_t g = nullptr;
            HIPCHK(c, hipStreamBeginCapture(s, hipStreamCaptureModeThreadLocal));
            launch_all();
            hipError_t e1 = hipStreamEndCapture(s, &g);
            if (e1 != hipSuccess || !g) return fail(c, SDLM_EHIP, "graph capture of the decode step failed: %s", hipGetErrorString(e1));
            hipError_t e2 = hipGraphInstantiate(&c->graph_exec, g, nullptr, nullptr, 0);
            (void)hipGraphDestroy(g);
            if (e2 != hipSuccess) { c->graph_exec = nullptr; return fail(c, SDLM_EHIP, "hipGraphInstantiate: %s", hipGetErrorString(e2)); }
            memcpy(c->graph_key, key, sizeof key);
        }
        HIPCHK(c, hipGraphLaunch(c->graph_exec, s));
    } else {
        launch_all();
    }
    HIPCHK(c, hipGetLastError());
    c->stepped = true;
    return SDLM_OK;
}

int sdlm_decode_step(sdlm_ctx *c, int32_t *ids, int32_t *count, float *conf, float *logits)
{
    return decode_step_impl(c, ids, count, conf, logits, false);
}

int sdlm_decode_step_static(sdlm_ctx *c, int32_t *ids, int32_t *count, float *conf, float *logits)
{
    if (!c) return SDLM_EINVAL;
    if (!c->static_scratch) return fail(c, SDLM_EHIP, "the library's static scratch array is unavailable: %s", c->static_err.c_str());
    if (!c->prefilled) return fail(c, SDLM_ESTATE, "decode_step before prefill");
    // what must fit: the LM head's partials of batch x D rows (fp32 mode: their logits, unless the caller takes them)
    const size_t lm_rows = (size_t)c->batch * c->r.block_D;
    const size_t lm_need = c->L.mfma ? mfma_lm_scratch_bytes(c->m.vocab, (int)lm_rows) : (logits ? 0 : lm_rows * c->m.vocab * sizeof(float));
    if (lm_need > STATIC_LM_BYTES)
        return fail(c, SDLM_ECAPACITY, "sdlm_decode_step_static: batch %d x D %d x vocabulary %d needs %zu bytes of LM-head scratch, the static array has %zu",
                    c->batch, c->r.block_D, c->m.vocab, lm_need, STATIC_LM_BYTES);
    // Point the step's partial-result scratch at the static array for the duration of the launches (the kernels take
    // the addresses as arguments); split counts and KV chunking adapt to the room they are given.
    struct Saved { float *slabs; size_t slab_floats; void *attn_part; size_t attn_bytes; void *lm_part; float *logits; } sv =
        {c->slabs, c->L.slab_floats, c->attn_part, c->L.attn_bytes, c->lm_part, c->logits};
    char *base = c->static_scratch;
    c->slabs = (float *)base; c->L.slab_floats = c->L.mfma ? STATIC_SLAB_BYTES / sizeof(float) : sv.slab_floats;
    c->attn_part = base + STATIC_SLAB_BYTES; c->L.attn_bytes = STATIC_ATTN_BYTES;
    c->lm_part = base + STATIC_SLAB_BYTES + STATIC_ATTN_BYTES;
    c->logits = (float *)c->lm_part;
    c->no_events = true;
    const int rc = decode_step_impl(c, ids, count, conf, logits, true);
    c->no_events = false;
    c->slabs = sv.slabs; c->L.slab_floats = sv.slab_floats; c->attn_part = sv.attn_part; c->L.attn_bytes = sv.attn_bytes;
    c->lm_part = sv.lm_part; c->logits = sv.logits;
    return rc;
}

int sdlm_graph(sdlm_ctx *c, int32_t enable)
{
    if (!c) return SDLM_EINVAL;
    if (enable && c->stream == nullptr)
        return fail(c, SDLM_ESTATE, "graph replay needs a context created on a stream other than the null stream (it cannot be captured)");
    c->graph_on = enable != 0;
    if (!enable) drop_graph(c);
    return SDLM_OK;
}

int sdlm_verify_step(sdlm_ctx *c, int32_t rule, int32_t *ids_tilde, int32_t *count, float *logits)
{
    if (!c) return SDLM_EINVAL;
    if (!c->stepped) return fail(c, SDLM_ESTATE, "verify_step without a preceding decode_step");
    if (rule != 0 && rule != 1) return fail(c, SDLM_EINVAL, "verify rule %d is not 0 (agreeing prefix) or 1 (largest agreeing index)", rule);
    const int B = c->batch, D = c->r.block_D;
    hipStream_t s = c->stream;
    if (D >= 2) {
        // positions reach n + 2D - 3 <= max_seq_len + D - 3 (decode_step checked n + D <= max_seq_len): inside the rotary
        // table; no cache slot beyond n - 1 is touched
        bool shared;
        const int rows_seq = verify_rows_per_seq(D, &shared);
        const int rows = B * rows_seq;
        const int gr = c->L.group_rows;
        int groups = 0;
        groups = verify_groups_per_seq(D, gr);
        const int cp_floor = c->L.mfma ? mfma_attn_chunk_floor(&c->m, c->r.max_seq_len, B * groups, c->L.attn_bytes) : 0;
        { Phase p(c, SDLM_PH_ROWS); launch_assemble_verify(s, c->st, c->rm, B, D, c->m.mask_token_id, gr, c->kg.staging_base, c->m.block_causal, c->m.n_kv_heads, cp_floor); }
        run_layers(c, rows, B * groups, rows, false, !shared);
        run_lm_head(c, B * (D - 1), logits);
    }
    { Phase p(c, SDLM_PH_ACCEPT); launch_verify_accept(s, c->st, c->ids_rows, B, D, rule, ids_tilde, count); }
    HIPCHK(c, hipGetLastError());
    return SDLM_OK;
}

int sdlm_kv_commit(sdlm_ctx *c, const int32_t *ids_override, const int32_t *count_override)
{
    if (!c) return SDLM_EINVAL;
    if (!c->stepped) return fail(c, SDLM_ESTATE, "kv_commit without a preceding decode_step");
    if ((ids_override == nullptr) != (count_override == nullptr)) return fail(c, SDLM_EINVAL, "pass both overrides or neither");
    const int B = c->batch, D = c->r.block_D;
    if (c->r.kv_layout == 1) {
        auto pages = [&]() { long t = 0; for (int b = 0; b < B; ++b) t += (c->n_ub[b] + D + PAGE - 1) / PAGE; return t; };
        if (pages() > c->L.n_pages) {
            int rc = refresh_lengths(c, nullptr);
            if (rc) return rc;
            if (pages() > c->L.n_pages) return fail(c, SDLM_ECAPACITY, "page pool (%d pages) would be exhausted", c->L.n_pages);
        }
    }
    launch_commit(c->stream, c->st, B, D, ids_override, count_override, c->r.kv_layout, c->L.n_pages, c->L.pages_per_seq, c->m.vocab);
    HIPCHK(c, hipGetLastError());
    for (int b = 0; b < B; ++b) c->n_ub[b] += D;
    c->stepped = false;
    if (!c->committed) { c->committed = true; drop_graph(c); }   // the certain-row bound of the step's launches changes
    return SDLM_OK;
}

int sdlm_get_lengths(sdlm_ctx *c, int32_t *n, int32_t *cc)
{
    if (!c) return SDLM_EINVAL;
    if (c->batch < 1) return fail(c, SDLM_ESTATE, "no sequences");
    if (n) HIPCHK(c, hipMemcpyAsync(n, c->st.n, sizeof(int32_t) * c->batch, hipMemcpyDeviceToDevice, c->stream));
    if (cc) HIPCHK(c, hipMemcpyAsync(cc, c->st.c, sizeof(int32_t) * c->batch, hipMemcpyDeviceToDevice, c->stream));
    int32_t flags = 0;
    int rc = refresh_lengths(c, &flags);
    if (rc) return rc;
    if (flags) {
        int32_t zero = 0;
        HIPCHK(c, hipMemcpyAsync(c->st.alloc + 1, &zero, 4, hipMemcpyHostToDevice, c->stream));
        HIPCHK(c, hipStreamSynchronize(c->stream));
        if (flags & 1) return fail(c, SDLM_ECAPACITY, "a sequence could not grow: page pool or max_seq_len exhausted");
        if (flags & 4) return fail(c, SDLM_EINVAL, "an override token id outside the vocabulary was replaced by 0");
        return fail(c, SDLM_EINVAL, "an override count outside 1..D was clamped");
    }
    return SDLM_OK;
}

int sdlm_debug_tap(sdlm_ctx *c, int32_t layer, int32_t which, void *dst)
{
    if (!c) return SDLM_EINVAL;
    if (which < 0) { c->taps.clear(); return SDLM_OK; }
    if (which > 6 || !dst || (which != 4 && (layer < 0 || layer >= c->m.n_layers))) return fail(c, SDLM_EINVAL, "bad tap");
    c->taps.push_back(Tap{layer, which, dst});
    return SDLM_OK;
}

int sdlm_debug_rows(sdlm_ctx *c, int32_t *tok, int32_t *pos, int32_t *seq, int32_t *kind, int32_t *n_rows)
{
    if (!c) return SDLM_EINVAL;
    size_t bytes = (size_t)c->L.max_rows * 4;
    if (tok) HIPCHK(c, hipMemcpyAsync(tok, c->rm.tok, bytes, hipMemcpyDeviceToDevice, c->stream));
    if (pos) HIPCHK(c, hipMemcpyAsync(pos, c->rm.pos, bytes, hipMemcpyDeviceToDevice, c->stream));
    if (seq) HIPCHK(c, hipMemcpyAsync(seq, c->rm.seq, bytes, hipMemcpyDeviceToDevice, c->stream));
    if (kind) HIPCHK(c, hipMemcpyAsync(kind, c->rm.kind, bytes, hipMemcpyDeviceToDevice, c->stream));
    if (n_rows) HIPCHK(c, hipMemcpyAsync(n_rows, c->rm.counts, 4, hipMemcpyDeviceToDevice, c->stream));
    return SDLM_OK;
}

int sdlm_debug_read_kv(sdlm_ctx *c, int32_t layer, int32_t seq, int32_t kv_head, int32_t pos0, int32_t count, float *k_out, float *v_out)
{
    if (!c || !k_out || !v_out) return SDLM_EINVAL;
    if (layer < 0 || layer >= c->m.n_layers || seq < 0 || seq >= c->batch || kv_head < 0 || kv_head >= c->m.n_kv_heads || count < 1)
        return fail(c, SDLM_EINVAL, "read_kv arguments out of range");
    if (pos0 == -1) {
        if (count > c->r.block_D) return fail(c, SDLM_EINVAL, "the staging tile holds D entries");
    } else if (pos0 < 0 || pos0 + count > c->r.max_seq_len) {
        return fail(c, SDLM_EINVAL, "read_kv arguments out of range");
    } else if (c->r.kv_layout == 1) {   // positions must be backed: check against the exact lengths
        int rc = refresh_lengths(c, nullptr);
        if (rc) return rc;
        if (pos0 + count > c->n_ub[seq]) return fail(c, SDLM_EINVAL, "positions beyond the sequence");
    }
    const char *pool_l = c->pool + (size_t)layer * c->kg.layer_stride * c->L.esz;
    launch_read_kv(c->stream, c->m.dtype, pool_l, c->kg, c->st, seq, kv_head, pos0, count, k_out, v_out);
    HIPCHK(c, hipGetLastError());
    return SDLM_OK;
}

int sdlm_debug_gemm_plan(int32_t epilogue, int32_t rows, int32_t min_rows, int32_t n, int32_t k, int32_t *tile_rows, int32_t *tile_cols,
                         int32_t *splits)
{
    if (!tile_rows || !tile_cols || !splits || rows < 1 || n < 1 || k < 64 || k % 64 || epilogue < 0 || epilogue > 3) return SDLM_EINVAL;
    int mt, nt, sp, wv;
    mfma_gemm_plan(epilogue == 3 ? 4 : epilogue, rows, min_rows, n, k, (size_t)16 << 20, &mt, &nt, &sp, &wv);
    *tile_rows = 32 * mt; *tile_cols = 32 * nt * wv; *splits = sp;
    return SDLM_OK;
}

int32_t sdlm_max_rows(const sdlm_ctx *c) { return c ? c->L.max_rows : 0; }

int sdlm_profile(sdlm_ctx *c, int32_t enable)
{
    if (!c) return SDLM_EINVAL;
    c->prof = (uint32_t)enable;
    return SDLM_OK;
}

int sdlm_profile_every(sdlm_ctx *c, int32_t n)
{
    if (!c) return SDLM_EINVAL;
    if (n < 1) return fail(c, SDLM_EINVAL, "sdlm_profile_every: n must be at least 1 (got %d)", n);
    c->prof_every = (uint32_t)n;
    for (int p = 0; p < SDLM_N_PHASES; ++p) c->prof_seen[p] = 0;
    return SDLM_OK;
}

int sdlm_profile_read(sdlm_ctx *c, float *ms, int32_t *launches)
{
    if (!c || !ms || !launches) return SDLM_EINVAL;
    HIPCHK(c, hipStreamSynchronize(c->stream));
    for (int p = 0; p < SDLM_N_PHASES; ++p) { ms[p] = 0.f; launches[p] = 0; }
    for (size_t i = 0; i + 1 < c->ev_used; i += 2) {
        float t = 0.f;
        if (hipEventElapsedTime(&t, c->ev[i], c->ev[i + 1]) == hipSuccess) {
            ms[c->ev_phase[i / 2]] += t;
            launches[c->ev_phase[i / 2]] += 1;
        }
    }
    c->ev_used = 0;
    return SDLM_OK;
}

const char *sdlm_kernel_info(const sdlm_ctx *c) { return c ? c->info.c_str() : ""; }
const char *sdlm_last_error(const sdlm_ctx *c) { return c ? c->err.c_str() : "null context"; }

void sdlm_destroy(sdlm_ctx *c)
{
    if (!c) return;
    for (auto e : c->ev) (void)hipEventDestroy(e);
    drop_graph(c);
    delete c;
}

}  // extern "C"
