// libspd host side: context, workspace carving, launch sequencing, HIP-graph replay of the
// timestep, and the C ABI declared in spd.h.  No device memory is allocated here.
#include "spd_internal.h"

#include <cmath>
#include <cstddef>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <new>

namespace {

constexpr size_t ALIGN = 256;
inline size_t up(size_t x) { return (x + ALIGN - 1) / ALIGN * ALIGN; }

enum State { ST_CREATED = 0, ST_PREFILLED = 1, ST_STEPPING = 2 };

enum KClass { KC_SUPERPOSE, KC_QKV, KC_ATTN, KC_O, KC_GATEUP, KC_DOWN, KC_HEAD, KC_TOPK, KC_EXPAND, KC_FUSED, KC_NUCLEUS, KC_N };
const char *const KC_NAMES[KC_N] = {"superpose", "gemv_qkv", "attention", "gemv_o", "gemv_gateup",
                                    "gemv_down", "gemv_head", "topk_partial", "expand_prune", "fused_forward", "nucleus"};

struct Layout {
    size_t pf_h, pf_h1, pf_q, pf_xhi, pf_xlo, pf_uhi, pf_ulo, pf_rope;   // dense prefix pass arena (0 = none)
    size_t pf_ks_part, pf_ks_count, pf_ks_tiles;
    bool dense;
    size_t state, sync, layers_dev, prof, act, logits, part, counters, inv_freq, prefix, hist_tok, hist_par, pv, pi, pm, ps, pn, nuc_pb, nuc_count, nuc_hist, nuc_bk, kv, total;
    size_t kv_layer_bytes;   // K (or V) of one layer
    size_t arena_bytes;      // one activation arena
    int max_splits, n_part, per_part;
    ActLayout al;
};


const char *check_cfg(const spd_model_cfg *c) {
    if (!c) return "cfg is null";
    if (c->dtype != SPD_DTYPE_FP32 && c->dtype != SPD_DTYPE_BF16) return "dtype must be fp32 or bf16";
    if (c->kv_dtype != SPD_DTYPE_FP32 && c->kv_dtype != SPD_DTYPE_FP16) return "kv_dtype must be fp32 or fp16";
    if (c->kv_dtype == SPD_DTYPE_FP16 && c->dtype != SPD_DTYPE_BF16) return "an fp16 key/value cache needs bf16 weights";
    if (c->n_layers < 0 || c->d_model <= 0 || c->n_heads <= 0 || c->n_kv_heads <= 0 || c->d_ffn <= 0 || c->vocab <= 0)
        return "non-positive model dimension";
    if (c->d_model % c->n_heads) return "d_model must be a multiple of n_heads";
    if (c->n_heads % c->n_kv_heads) return "n_heads must be a multiple of n_kv_heads";
    const int vec = c->dtype == SPD_DTYPE_BF16 ? 8 : 4;
    const int dh = c->d_model / c->n_heads;
    if (dh % vec || dh > 256) return "d_head must be a multiple of the 16-byte vector width and <= 256";
    const int lpp = dh / 4;   // lanes per cached position (fp32 cache, 16-byte pieces)
    if (dh % 4 || lpp > 64 || (lpp & (lpp - 1))) return "d_head / 4 must be a power of two <= 64";
    if (c->d_model % vec || c->d_ffn % vec) return "d_model and d_ffn must be multiples of the 16-byte vector width";
    if (c->vocab % 2) return "vocab must be even";
    if (c->max_ctx < 2) return "max_ctx must be >= 2";
    if (c->k_max < 1 || c->k_max > SPD_K_MAX) return "k_max out of range";
    if (c->vocab < c->k_max) return "vocab smaller than k_max";
    if (c->vocab >= (1 << 20)) return "vocab must be below 2^20";   // the sampler counts entries in 20 bits of a histogram word
    if (!(c->rms_eps > 0.f) || !(c->rope_theta > 0.f)) return "rms_eps and rope_theta must be positive";
    const int widest = c->d_model > c->d_ffn ? c->d_model : c->d_ffn;
    if (spdk::gemv_lds_bytes(c->dtype, widest) > 160 * 1024 - 1024) return "d_model / d_ffn too large for the LDS staging";
    return nullptr;
}

Layout make_layout(const spd_model_cfg &c) {
    Layout L{};
    const int dh = c.d_model / c.n_heads;
    L.max_splits = (c.max_ctx + ATTN_CHUNK_MIN - 1) / ATTN_CHUNK_MIN;   // room for the smallest chunk
    L.n_part = (c.vocab + 1023) / 1024;
    if (L.n_part > TOPK_PART_MAX) L.n_part = TOPK_PART_MAX;
    L.per_part = (c.vocab + L.n_part - 1) / L.n_part;
    size_t o = 0;
    auto take = [&](size_t bytes) { size_t at = o; o += up(bytes); return at; };
    L.state = take(sizeof(DevState));
    L.sync = take((size_t)SYNC_WORDS * 4);
    L.layers_dev = take((size_t)(c.n_layers > 0 ? c.n_layers : 1) * sizeof(spd_layer_weights));
    L.prof = take((size_t)FUSED_PROF_BLOCKS * (size_t)(2 * (5 * c.n_layers + 2)) * 8);   // phase clocks per block
    {   // one address per produced vector (see ActLayout)
        const size_t vd = up((size_t)c.d_model * 4), vq = up((size_t)c.n_heads * dh * 4), vu = up((size_t)c.d_ffn * 4);
        L.al.h0 = 0;
        L.al.layer0 = vd;
        const size_t vk = up((size_t)c.n_kv_heads * dh * 4);
        L.al.q = 0; L.al.att = vq; L.al.h1 = 2 * vq; L.al.u = 2 * vq + vd; L.al.h2 = 2 * vq + vd + vu;
        L.al.kn = 2 * vq + 2 * vd + vu; L.al.vn = L.al.kn + vk;
        L.al.stride = 2 * vq + 2 * vd + vu + 2 * vk;
        L.arena_bytes = up(vd + (size_t)c.n_layers * L.al.stride);
        L.act = take(2 * L.arena_bytes);   // the fused kernel alternates between two arenas (see ACT_UNSET)
    }
    L.logits = take((size_t)c.vocab * 4);
    L.part = take((size_t)c.n_heads * L.max_splits * (dh + 2) * 4);
    L.counters = take((size_t)c.n_heads * ATTN_COUNTER_STRIDE * 4);
    L.inv_freq = take((size_t)(dh / 2) * 8);
    L.prefix = take((size_t)c.max_ctx * 4);
    L.hist_tok = take((size_t)c.max_ctx * SPD_K_MAX * 4);
    L.hist_par = take((size_t)c.max_ctx * SPD_K_MAX * 4);
    L.pv = take((size_t)L.n_part * SPD_K_MAX * 4);
    L.pi = take((size_t)L.n_part * SPD_K_MAX * 4);
    L.pm = take((size_t)L.n_part * 4);
    L.ps = take((size_t)L.n_part * 4);
    L.pn = take((size_t)L.n_part * 4);
    L.nuc_pb = take((size_t)c.vocab * 8);      // the nucleus sampler's per-entry scratch
    L.nuc_count = take(4);
    L.nuc_hist = take(2048 * 8);
    L.nuc_bk = take(32768 * 2);
    // dense prefix pass (matrix cores): bf16 weights, d_head <= 128, widths the tiles divide,
    // d_model within what its norm kernel keeps in registers
    L.dense = c.dtype == SPD_DTYPE_BF16 && dh <= 128 && c.d_model % 128 == 0 && c.d_model <= 8192 && c.d_ffn % 128 == 0 &&
              (c.n_heads * dh) % 128 == 0 && c.n_layers > 0;
    if (L.dense) {
        const size_t nq = (size_t)c.n_heads * dh, wide = nq > (size_t)c.d_model ? nq : (size_t)c.d_model;
        L.pf_h = take((size_t)PREFILL_CHUNK * c.d_model * 4);
        L.pf_h1 = take((size_t)PREFILL_CHUNK * c.d_model * 4);
        L.pf_q = take((size_t)PREFILL_CHUNK * nq * 4);
        L.pf_xhi = take((size_t)PREFILL_CHUNK * wide * 2);
        L.pf_xlo = take((size_t)PREFILL_CHUNK * wide * 2);
        L.pf_uhi = take((size_t)PREFILL_CHUNK * c.d_ffn * 2);
        L.pf_ulo = take((size_t)PREFILL_CHUNK * c.d_ffn * 2);
        L.pf_rope = take((size_t)PREFILL_CHUNK * (dh / 2) * 8);
        const size_t widest = std::max((size_t)(nq + 2 * c.n_kv_heads * dh), std::max((size_t)c.d_model, (size_t)c.d_ffn));
        L.pf_ks_tiles = (widest + 31) / 32;
        L.pf_ks_part = take(L.pf_ks_tiles * 2 * 2 * 16 * 64 * 4);
        L.pf_ks_count = take(L.pf_ks_tiles * 4);
    }
    L.kv_layer_bytes = up((size_t)c.n_kv_heads * c.max_ctx * dh * (c.kv_dtype == SPD_DTYPE_FP16 ? 2 : 4));
    L.kv = take(L.kv_layer_bytes * 2 * (size_t)c.n_layers);
    L.total = o;
    return L;
}

struct Timed { int cls; hipEvent_t a, b; };

}  // namespace

struct spd_ctx {
    spd_model_cfg cfg;
    std::vector<spd_layer_weights> layers;
    const void *embed, *final_norm, *lm_head;
    hipStream_t stream;
    int num_cu;
    Layout L;
    char *ws;
    NgramDev ng;
    bool have_ng;
    int state, pos, n_gen, k;
    std::vector<int32_t> text;   // committed tokens: the prefix, extended by spd_commit
    char *pinned;
    size_t pinned_bytes;
    bool use_graph, timing, use_fused, use_dense;
    int fused_blocks;   // grid of the fused forward kernel; 0 = not available for this shape
    hipGraphExec_t step_exec, prefill_exec, nucleus_exec;
    spd_decode_cfg step_dc;
    spd_sample_cfg nucleus_sc;
    std::vector<Timed> timed;
    std::vector<hipEvent_t> ev_pool;
    double kc_ms[KC_N];
    int64_t kc_n[KC_N];
    std::string err;

    DevState *st() const { return (DevState *)(ws + L.state); }
    template <typename T> T *at(size_t off) const { return (T *)(ws + off); }
    void *kcache(int l) const { return ws + L.kv + (size_t)(2 * l) * L.kv_layer_bytes; }
    void *vcache(int l) const { return ws + L.kv + (size_t)(2 * l + 1) * L.kv_layer_bytes; }
};

namespace {

int fail(spd_ctx *c, int code, const std::string &msg) {
    if (c) c->err = msg;
    return code;
}
int hipfail(spd_ctx *c, hipError_t e, const char *what) {
    return fail(c, SPD_EHIP, std::string(what) + ": " + hipGetErrorString(e));
}
#define HIPCHK(c, call)                                         \
    do {                                                        \
        hipError_t e_ = (call);                                 \
        if (e_ != hipSuccess) return hipfail((c), e_, #call);   \
    } while (0)

// Every entry point that copies the draft state back from the device passes the copy through
// here: a bounded wait of the persistent kernel that gave up (the grid was not co-resident)
// leaves `err` set, and whatever the launch produced after that is not a result.
int device_state_status(spd_ctx *c, const DevState *hs) {
    if (hs->err) return fail(c, SPD_EHIP, "device-wide barrier timed out (grid not co-resident)");
    return SPD_OK;
}
#define STATECHK(c, hs)                                          \
    do {                                                         \
        const int rc_ = device_state_status((c), (hs));          \
        if (rc_ != SPD_OK) return rc_;                           \
    } while (0)

// Launch helper: plain, or bracketed by an event pair when per-kernel timing is on.
template <typename F> hipError_t launch(spd_ctx *c, int cls, F f) {
    if (!c->timing) return f();
    hipEvent_t ev[2];
    for (int i = 0; i < 2; ++i) {
        if (!c->ev_pool.empty()) { ev[i] = c->ev_pool.back(); c->ev_pool.pop_back(); }
        else { hipError_t e = hipEventCreate(&ev[i]); if (e != hipSuccess) return e; }
    }
    hipError_t e = hipEventRecord(ev[0], c->stream);
    if (e == hipSuccess) e = f();
    if (e == hipSuccess) e = hipEventRecord(ev[1], c->stream);
    c->timed.push_back({cls, ev[0], ev[1]});
    return e;
}

hipError_t drain_timing(spd_ctx *c) {
    hipError_t e = hipStreamSynchronize(c->stream);
    for (auto &t : c->timed) {
        float ms = 0.f;
        if (e == hipSuccess) e = hipEventElapsedTime(&ms, t.a, t.b);
        c->kc_ms[t.cls] += ms;
        c->kc_n[t.cls] += 1;
        c->ev_pool.push_back(t.a);
        c->ev_pool.push_back(t.b);
    }
    c->timed.clear();
    return e;
}

// mode 0: the prefix token at the current position; mode 1: the superposed drafts.
hipError_t enqueue_forward(spd_ctx *c, int mode, int k, bool head) {
    const spd_model_cfg &m = c->cfg;
    const int dh = m.d_model / m.n_heads;
    const int nq = m.n_heads * dh, nkv = m.n_kv_heads * dh;
    hipError_t e;
    char *act = c->ws + c->L.act;
    const ActLayout &al = c->L.al;
    SuperposeArgs sa{c->embed, c->st(), c->at<int32_t>(c->L.prefix), al.h_in(act, 0), m.d_model, mode, k};
    if (c->use_fused && c->fused_blocks > 0) {
        FusedArgsHost f{};
        f.sup = sa;
        f.layers = c->at<spd_layer_weights>(c->L.layers_dev);
        f.final_norm = c->final_norm; f.lm_head = c->lm_head;
        f.act = act; f.arena_bytes = c->L.arena_bytes; f.al = al; f.logits = c->at<float>(c->L.logits);
        f.kv = c->ws + c->L.kv; f.kv_layer_bytes = c->L.kv_layer_bytes;
        f.part = c->at<float>(c->L.part); f.counters = c->at<int32_t>(c->L.counters);
        f.inv_freq = c->at<double>(c->L.inv_freq); f.prof = c->timing ? c->at<long long>(c->L.prof) : nullptr;
        f.sync = c->at<unsigned>(c->L.sync);
        f.n_layers = m.n_layers; f.d_model = m.d_model; f.n_heads = m.n_heads; f.n_kv_heads = m.n_kv_heads;
        f.d_ffn = m.d_ffn; f.vocab = m.vocab; f.cap_ctx = m.max_ctx; f.max_splits = c->L.max_splits;
        f.head = head ? 1 : 0; f.eps = m.rms_eps; f.kv_half = m.kv_dtype == SPD_DTYPE_FP16;
        return launch(c, KC_FUSED, [&] { return spdk::fused_forward(c->stream, m.dtype, f, c->fused_blocks); });
    }
    e = launch(c, KC_SUPERPOSE, [&] { return spdk::superpose(c->stream, m.dtype, sa); });
    if (e != hipSuccess) return e;
    for (int l = 0; l < m.n_layers; ++l) {
        const spd_layer_weights &w = c->layers[l];
        float *h = al.h_in(act, l), *q = al.vec(act, l, al.q), *att = al.vec(act, l, al.att);
        float *h1 = al.vec(act, l, al.h1), *u = al.vec(act, l, al.u), *h2 = al.vec(act, l, al.h2);
        GemvArgs g{};
        g.W = w.wqkv; g.gain = w.attn_norm; g.eps = m.rms_eps; g.x = h; g.y = q;
        g.rows = nq + 2 * nkv; g.cols = m.d_model;
        g.kcache = c->kcache(l); g.vcache = c->vcache(l); g.st = c->st();
        g.inv_freq = c->at<double>(c->L.inv_freq);
        g.n_q_rows = nq; g.n_kv_rows = nkv; g.d_head = dh; g.cap_ctx = m.max_ctx;
        g.kv_half = m.kv_dtype == SPD_DTYPE_FP16;
        e = launch(c, KC_QKV, [&] { return spdk::gemv(c->stream, m.dtype, EPI_QKV, g, c->num_cu); });
        if (e != hipSuccess) return e;
        AttnArgs a{q, c->kcache(l), c->vcache(l), att, c->at<float>(c->L.part), c->at<int32_t>(c->L.counters),
                   c->st(), 0, m.n_heads, m.n_kv_heads, dh, m.max_ctx, ATTN_CHUNK, c->L.max_splits};
        e = launch(c, KC_ATTN, [&] { return spdk::attention(c->stream, m.kv_dtype, a); });
        if (e != hipSuccess) return e;
        GemvArgs o{};
        o.W = w.wo; o.x = att; o.resid = h; o.y = h1; o.rows = m.d_model; o.cols = nq;
        e = launch(c, KC_O, [&] { return spdk::gemv(c->stream, m.dtype, EPI_RESID, o, c->num_cu); });
        if (e != hipSuccess) return e;
        GemvArgs f{};
        f.W = w.w_gate; f.W2 = w.w_up; f.gain = w.ffn_norm; f.eps = m.rms_eps; f.x = h1; f.y = u;
        f.rows = m.d_ffn; f.cols = m.d_model;
        e = launch(c, KC_GATEUP, [&] { return spdk::gemv(c->stream, m.dtype, EPI_SWIGLU, f, c->num_cu); });
        if (e != hipSuccess) return e;
        GemvArgs d{};
        d.W = w.w_down; d.x = u; d.resid = h1; d.y = h2; d.rows = m.d_model; d.cols = m.d_ffn;
        e = launch(c, KC_DOWN, [&] { return spdk::gemv(c->stream, m.dtype, EPI_RESID, d, c->num_cu); });
        if (e != hipSuccess) return e;
    }
    if (head) {
        GemvArgs g{};
        g.W = c->lm_head; g.gain = c->final_norm; g.eps = m.rms_eps; g.x = al.h_in(act, m.n_layers); g.y = c->at<float>(c->L.logits);
        g.rows = m.vocab; g.cols = m.d_model;
        e = launch(c, KC_HEAD, [&] { return spdk::gemv(c->stream, m.dtype, EPI_PLAIN, g, c->num_cu); });
        if (e != hipSuccess) return e;
    }
    return hipSuccess;
}

hipError_t enqueue_decide(spd_ctx *c, const spd_decode_cfg &dc, const float *logits, int first, int advance) {
    TopkArgs t{logits, c->cfg.vocab, dc.k, c->L.n_part, c->L.per_part, dc.tau,
               c->at<float>(c->L.pv), c->at<int32_t>(c->L.pi), c->at<float>(c->L.pm), c->at<float>(c->L.ps), c->at<float>(c->L.pn)};
    hipError_t e = launch(c, KC_TOPK, [&] { return spdk::topk_partial(c->stream, t); });
    if (e != hipSuccess) return e;
    ExpandArgs x{};
    x.st = c->st(); x.pv = t.pv; x.pi = t.pi; x.pm = t.pm; x.ps = t.ps; x.n_part = c->L.n_part;
    x.ng = c->ng;
    if (!c->have_ng) x.ng.slots = nullptr;
    x.k = dc.k; x.alpha = dc.alpha; x.tau = dc.tau; x.delta = dc.delta;
    x.first = first; x.advance = advance;
    x.hist_tok = c->at<int32_t>(c->L.hist_tok); x.hist_par = c->at<int32_t>(c->L.hist_par);
    x.max_gen = c->cfg.max_ctx;
    return launch(c, KC_EXPAND, [&] { return spdk::expand_prune(c->stream, x); });
}

// Post-forward part of one nucleus-sampling step: slice statistics, then the sampler.
hipError_t enqueue_sample(spd_ctx *c, const spd_sample_cfg &sc, const float *logits, int first, int advance) {
    TopkArgs t{logits, c->cfg.vocab, 1, c->L.n_part, c->L.per_part, sc.tau,
               c->at<float>(c->L.pv), c->at<int32_t>(c->L.pi), c->at<float>(c->L.pm), c->at<float>(c->L.ps), c->at<float>(c->L.pn)};
    hipError_t e = launch(c, KC_TOPK, [&] { return spdk::topk_partial(c->stream, t); });
    if (e != hipSuccess) return e;
    NucleusArgs n{};
    n.logits = logits; n.vocab = c->cfg.vocab; n.st = c->st(); n.pm = t.pm; n.ps = t.ps; n.pn = t.pn; n.n_part = c->L.n_part;
    n.per_part = c->L.per_part;
    n.sc_pb = c->at<unsigned long long>(c->L.nuc_pb);
    n.sc_count = c->at<unsigned>(c->L.nuc_count);
    n.sc_hist = c->at<unsigned long long>(c->L.nuc_hist);
    n.sc_bk = c->at<uint16_t>(c->L.nuc_bk);
    n.top_p = sc.top_p; n.tau = sc.tau; n.first = first; n.advance = advance;
    n.hist_tok = c->at<int32_t>(c->L.hist_tok); n.hist_par = c->at<int32_t>(c->L.hist_par);
    n.max_gen = c->cfg.max_ctx;
    return launch(c, KC_NUCLEUS, [&] { return spdk::nucleus(c->stream, n); });
}

// What the persistent forward kernel carries from launch to launch, back to its initial state:
// counters zero, every element of both activation arenas ACT_UNSET (and the chunk-arrival
// counters of the attention merge, which a launch that gave up on a wait may have left short
// of the count that resets them).
hipError_t reset_fused_state(spd_ctx *c) {
    hipError_t e = spdk::fill_i32(c->stream, c->at<int32_t>(c->L.sync), 0, SYNC_WORDS);
    if (e == hipSuccess) e = spdk::fill_i32(c->stream, c->at<int32_t>(c->L.counters), 0, c->cfg.n_heads * ATTN_COUNTER_STRIDE);
    if (e == hipSuccess) e = spdk::fill_i32(c->stream, c->at<int32_t>(c->L.act), (int32_t)ACT_UNSET, (int)(2 * c->L.arena_bytes / 4));
    return e;
}

void drop_graph(hipGraphExec_t &g) {
    if (g) { (void)hipGraphExecDestroy(g); g = nullptr; }
}

// Capture `body` on the ctx stream into an executable graph.
template <typename F> int capture(spd_ctx *c, hipGraphExec_t *out, F body) {
    hipGraph_t graph = nullptr;
    HIPCHK(c, hipStreamBeginCapture(c->stream, hipStreamCaptureModeRelaxed));
    hipError_t e = body();
    hipError_t e2 = hipStreamEndCapture(c->stream, &graph);
    if (e != hipSuccess) { if (graph) (void)hipGraphDestroy(graph); return hipfail(c, e, "launch during graph capture"); }
    if (e2 != hipSuccess) return hipfail(c, e2, "hipStreamEndCapture");
    e = hipGraphInstantiate(out, graph, nullptr, nullptr, 0);
    (void)hipGraphDestroy(graph);
    if (e != hipSuccess) return hipfail(c, e, "hipGraphInstantiate");
    return SPD_OK;
}

const char *check_dc(const spd_ctx *c, const spd_decode_cfg *dc) {
    if (!dc) return "decode cfg is null";
    if (dc->k < 1 || dc->k > c->cfg.k_max) return "k outside [1, k_max]";
    if (!(dc->alpha >= 0.f && dc->alpha <= 1.f)) return "alpha outside [0, 1]";
    if (!(dc->tau > 0.f)) return "tau must be positive";
    if (!(dc->delta > 0.f)) return "delta must be positive";
    if (dc->alpha != 0.f && !c->have_ng) return "alpha > 0 needs n-gram tables (spd_load_ngrams)";
    return nullptr;
}

constexpr int DENSE_PREFILL_MIN = 8;   // shorter prefixes go token by token

bool graphs_usable(const spd_ctx *c) { return c->use_graph && !c->timing && c->stream != nullptr; }

}  // namespace

// Shared by spd_op_attention and its variant on the library's static scratch.
namespace spdk {
int attention_args_status(int dtype, const float *q, const void *K, const void *V, const float *out, int n_heads,
                          int n_kv_heads, int d_head, int n_ctx, int cap_ctx) {
    if (!q || !K || !V || !out) return SPD_EINVAL;
    if (dtype != SPD_DTYPE_FP32 && dtype != SPD_DTYPE_BF16 && dtype != SPD_DTYPE_FP16) return SPD_EINVAL;
    const int vec = dtype == SPD_DTYPE_FP32 ? 4 : 8;
    if (n_heads <= 0 || n_kv_heads <= 0 || n_heads % n_kv_heads || d_head <= 0 || d_head % vec || d_head > 256) return SPD_EINVAL;
    const int lpp = d_head / vec;
    if (lpp > 64 || (lpp & (lpp - 1))) return SPD_EINVAL;
    if (n_ctx < 1 || n_ctx > cap_ctx) return SPD_EINVAL;
    return SPD_OK;
}

// `scratch`: DEVICE, 256-byte aligned, spd_op_attention_scratch_bytes() bytes: the heads'
// arrival counters (cleared here, by a fill kernel) followed by the chunks' partial results.
int attention_on_scratch(hipStream_t s, int dtype, const float *q, const void *K, const void *V, float *out,
                         void *scratch, int n_heads, int n_kv_heads, int d_head, int n_ctx, int cap_ctx) {
    int32_t *counters = (int32_t *)scratch;
    float *part = (float *)((char *)scratch + up((size_t)n_heads * ATTN_COUNTER_STRIDE * 4));
    if (fill_i32(s, counters, 0, n_heads * ATTN_COUNTER_STRIDE) != hipSuccess) return SPD_EHIP;
    AttnArgs a{q, K, V, out, part, counters, nullptr, n_ctx, n_heads, n_kv_heads, d_head, cap_ctx, ATTN_CHUNK,
               (cap_ctx + ATTN_CHUNK - 1) / ATTN_CHUNK};
    return attention(s, dtype, a) == hipSuccess ? SPD_OK : SPD_EHIP;
}
}  // namespace spdk

// =============================================================================== C ABI
extern "C" {

const char *spd_strerror(int s) {
    switch (s) {
        case SPD_OK: return "ok";
        case SPD_EINVAL: return "invalid argument";
        case SPD_ESTATE: return "call out of order";
        case SPD_ECTX_OVERFLOW: return "context would exceed max_ctx";
        case SPD_EWORKSPACE: return "workspace or table buffer too small or misaligned";
        case SPD_ETABLE: return "n-gram table rejected";
        case SPD_EHIP: return "HIP runtime error";
        default: return "unknown status";
    }
}

const char *spd_last_error(const spd_ctx *ctx) { return ctx ? ctx->err.c_str() : "ctx is null"; }

int spd_workspace_bytes(const spd_model_cfg *cfg, size_t *out_bytes) {
    if (!out_bytes || check_cfg(cfg)) return SPD_EINVAL;
    *out_bytes = make_layout(*cfg).total;
    return SPD_OK;
}

int spd_create(const spd_model_cfg *cfg, const spd_weight_ptrs *w, void *workspace, size_t workspace_bytes,
               void *hip_stream, spd_ctx **out) {
    if (!out) return SPD_EINVAL;
    *out = nullptr;
    if (check_cfg(cfg) || !w || !workspace) return SPD_EINVAL;
    if (!w->embed || !w->final_norm || !w->lm_head || (cfg->n_layers > 0 && !w->layers)) return SPD_EINVAL;
    auto misaligned = [](const void *p) { return ((uintptr_t)p & 15u) != 0; };
    if (misaligned(w->embed) || misaligned(w->final_norm) || misaligned(w->lm_head)) return SPD_EINVAL;
    for (int l = 0; l < cfg->n_layers; ++l) {
        const spd_layer_weights &lw = w->layers[l];
        const void *ps[7] = {lw.attn_norm, lw.wqkv, lw.wo, lw.ffn_norm, lw.w_gate, lw.w_up, lw.w_down};
        for (const void *p : ps)
            if (!p || misaligned(p)) return SPD_EINVAL;
    }
    const Layout L = make_layout(*cfg);
    if (((uintptr_t)workspace & (ALIGN - 1)) || workspace_bytes < L.total) return SPD_EWORKSPACE;

    spd_ctx *c = new (std::nothrow) spd_ctx();
    if (!c) return SPD_EINVAL;
    c->cfg = *cfg;
    c->layers.assign(w->layers, w->layers + cfg->n_layers);
    c->embed = w->embed; c->final_norm = w->final_norm; c->lm_head = w->lm_head;
    c->stream = (hipStream_t)hip_stream;
    c->L = L;
    c->ws = (char *)workspace;
    c->have_ng = false;
    std::memset(&c->ng, 0, sizeof(c->ng));
    c->state = ST_CREATED; c->pos = 0; c->n_gen = 0; c->k = 0;
    c->use_graph = true; c->timing = false; c->use_fused = true; c->fused_blocks = 0;
    c->use_dense = c->L.dense && spdk::prefill_init() == hipSuccess;
    c->step_exec = nullptr; c->prefill_exec = nullptr; c->nucleus_exec = nullptr;
    std::memset(&c->step_dc, 0, sizeof(c->step_dc));
    std::memset(c->kc_ms, 0, sizeof(c->kc_ms));
    std::memset(c->kc_n, 0, sizeof(c->kc_n));
    c->pinned = nullptr;

    int dev = 0;
    hipDeviceProp_t prop;
    hipError_t e = hipGetDevice(&dev);
    if (e == hipSuccess) e = hipGetDeviceProperties(&prop, dev);
    if (e == hipSuccess) e = spdk::init();
    c->pinned_bytes = up(sizeof(DevState)) + (size_t)cfg->max_ctx * (4 + 2 * SPD_K_MAX * 4) + (size_t)cfg->vocab * 4 +
                      up(2048) + (size_t)cfg->n_layers * sizeof(spd_layer_weights);
    if (e == hipSuccess) e = hipHostMalloc((void **)&c->pinned, c->pinned_bytes, hipHostMallocDefault);
    if (e != hipSuccess) { delete c; return SPD_EHIP; }
    c->num_cu = prop.multiProcessorCount;
    {   // the fused forward needs its whole grid resident at once: size it from the occupancy
        int per_cu = spdk::fused_max_blocks_per_cu(cfg->dtype, cfg->kv_dtype == SPD_DTYPE_FP16, cfg->d_model, cfg->d_ffn);
        if (per_cu > 1) per_cu = 1;
        c->fused_blocks = per_cu > 0 ? per_cu * c->num_cu : 0;
        if (c->fused_blocks > FUSED_MAX_BLOCKS) c->fused_blocks = 0;
        if (c->fused_blocks > 0 && (4 * cfg->d_model) / (3 * c->fused_blocks) + 4 > FUSED_MAX_EPI) c->fused_blocks = 0;   // residual slice per block (a quarter of the blocks may sit a phase out)
    }

    // rotary frequencies theta^(-2i/d_head) in double; zeroed state and attention counters
    const int dh = cfg->d_model / cfg->n_heads;
    double *f = (double *)c->pinned;
    for (int i = 0; i < dh / 2; ++i) f[i] = std::pow((double)cfg->rope_theta, -2.0 * i / dh);
    spd_layer_weights *hl = (spd_layer_weights *)(c->pinned + up((size_t)(dh / 2) * 8));
    for (int l = 0; l < cfg->n_layers; ++l) hl[l] = c->layers[l];
    e = hipMemcpyAsync(c->ws + L.inv_freq, f, (size_t)(dh / 2) * 8, hipMemcpyHostToDevice, c->stream);
    if (e == hipSuccess && cfg->n_layers > 0)
        e = hipMemcpyAsync(c->ws + L.layers_dev, hl, (size_t)cfg->n_layers * sizeof(spd_layer_weights),
                           hipMemcpyHostToDevice, c->stream);
    if (e == hipSuccess) e = spdk::fill_i32(c->stream, (int32_t *)c->st(), 0, sizeof(DevState) / 4);
    if (e == hipSuccess) e = spdk::fill_i32(c->stream, c->at<int32_t>(L.counters), 0, cfg->n_heads * ATTN_COUNTER_STRIDE);
    if (e == hipSuccess && L.dense) e = spdk::fill_i32(c->stream, c->at<int32_t>(L.pf_ks_count), 0, (int)L.pf_ks_tiles);
    if (e == hipSuccess) e = spdk::fill_i32(c->stream, c->at<int32_t>(L.nuc_count), 0, 1);
    if (e == hipSuccess) e = spdk::fill_i32(c->stream, c->at<int32_t>(L.nuc_hist), 0, 2048 * 2);
    if (e == hipSuccess) e = spdk::fill_i32(c->stream, c->at<int32_t>(L.nuc_bk), -1, 32768 / 2);   // 0xFFFF: no bucket
    if (e == hipSuccess) e = hipStreamSynchronize(c->stream);
    if (e != hipSuccess) { (void)hipHostFree(c->pinned); delete c; return SPD_EHIP; }
    *out = c;
    return SPD_OK;
}

void spd_destroy(spd_ctx *c) {
    if (!c) return;
    (void)hipStreamSynchronize(c->stream);
    drop_graph(c->step_exec);
    drop_graph(c->prefill_exec);
    drop_graph(c->nucleus_exec);
    for (auto &t : c->timed) { (void)hipEventDestroy(t.a); (void)hipEventDestroy(t.b); }
    for (auto &e : c->ev_pool) (void)hipEventDestroy(e);
    if (c->pinned) (void)hipHostFree(c->pinned);
    delete c;
}

int spd_ngram_table_bytes(const spd_ngram_host_tables *t, size_t *out_bytes) {
    if (!t || !out_bytes) return SPD_EINVAL;
    for (int o = 0; o < SPD_N_ORDERS; ++o)
        if (t->n_entries[o] < 0) return SPD_EINVAL;
    *out_bytes = up(ngram_capacity_for(t) * sizeof(NgramSlot));
    return SPD_OK;
}

int spd_load_ngrams(spd_ctx *c, const spd_ngram_host_tables *t, void *dev_buf, size_t dev_bytes) {
    if (!c) return SPD_EINVAL;
    if (!t || !dev_buf) return fail(c, SPD_EINVAL, "null tables or buffer");
    const uint64_t cap = ngram_capacity_for(t);
    if (((uintptr_t)dev_buf & (ALIGN - 1)) || dev_bytes < cap * sizeof(NgramSlot))
        return fail(c, SPD_EWORKSPACE, "n-gram device buffer too small or misaligned");
    NgramHostTable host;
    std::string err;
    const int rc = ngram_build(t, c->cfg.vocab, cap, host, err);
    if (rc != SPD_OK) return fail(c, rc, err);
    HIPCHK(c, hipStreamSynchronize(c->stream));
    HIPCHK(c, hipMemcpy(dev_buf, host.slots.data(), cap * sizeof(NgramSlot), hipMemcpyHostToDevice));
    c->ng.slots = (const NgramSlot *)dev_buf;
    c->ng.capacity = cap;
    c->ng.max_probe = host.max_probe;
    for (int o = 0; o < SPD_N_ORDERS; ++o) { c->ng.present[o] = host.present[o]; c->ng.lambda[o] = t->lambda[o]; }
    c->have_ng = true;
    drop_graph(c->step_exec);   // the captured step holds the old table by value
    return SPD_OK;
}

// The prefix pass over tokens p0 .. m-1 of c->text (cache positions 0 .. p0-1 are in place):
// stages the draft-state header and the token ids, fills the cache, keeps the logits of token
// m-1.  Dense (whole chunks on the matrix cores) where the model allows it.
static int run_prefix_pass(spd_ctx *c, int p0, int m) {
    if (c->timing) HIPCHK(c, drain_timing(c));
    HIPCHK(c, hipStreamSynchronize(c->stream));   // the pinned staging area may still be in flight
    DevState *hs = (DevState *)c->pinned;
    std::memset(hs, 0, sizeof(DevState));
    hs->pos = p0;
    for (int q = 0; q < SPD_TAIL; ++q) {
        const int src = m - SPD_TAIL + q;
        hs->prefix_tail[q] = src >= 0 ? c->text[src] : NG_PAD;
    }
    int32_t *hp = (int32_t *)(c->pinned + up(sizeof(DevState)));
    std::memcpy(hp, c->text.data() + p0, (size_t)(m - p0) * 4);
    HIPCHK(c, hipMemcpyAsync(c->st(), hs, sizeof(DevState), hipMemcpyHostToDevice, c->stream));
    // the persistent kernel's launch / layer counts and per-head counters run on from launch to
    // launch within a generation, and it expects both activation arenas unset
    HIPCHK(c, reset_fused_state(c));
    HIPCHK(c, hipMemcpyAsync(c->ws + c->L.prefix + (size_t)p0 * 4, hp, (size_t)(m - p0) * 4, hipMemcpyHostToDevice, c->stream));
    c->state = ST_CREATED;
    c->pos = p0; c->n_gen = 0; c->k = 0;
    const int n = m - p0;

    if (c->use_dense && n >= DENSE_PREFILL_MIN) {
        // whole chunks of prefix tokens on the matrix cores; the last token's final norm and
        // LM head go through the matrix-vector kernel
        const spd_model_cfg &mc = c->cfg;
        PrefillChunk pc{};
        pc.embed = c->embed; pc.prefix = c->at<int32_t>(c->L.prefix); pc.layers = c->layers.data();
        pc.n_layers = mc.n_layers; pc.d_model = mc.d_model; pc.n_heads = mc.n_heads; pc.n_kv_heads = mc.n_kv_heads;
        pc.d_ffn = mc.d_ffn; pc.cap_ctx = mc.max_ctx; pc.eps = mc.rms_eps; pc.num_cu = c->num_cu;
        pc.inv_freq = c->at<double>(c->L.inv_freq); pc.kv = c->ws + c->L.kv; pc.kv_layer_bytes = c->L.kv_layer_bytes; pc.kv_half = mc.kv_dtype == SPD_DTYPE_FP16;
        pc.h = c->at<float>(c->L.pf_h); pc.h1 = c->at<float>(c->L.pf_h1); pc.q = c->at<float>(c->L.pf_q);
        pc.xhi = c->at<uint16_t>(c->L.pf_xhi); pc.xlo = c->at<uint16_t>(c->L.pf_xlo);
        pc.uhi = c->at<uint16_t>(c->L.pf_uhi); pc.ulo = c->at<uint16_t>(c->L.pf_ulo);
        pc.rope = c->at<float2>(c->L.pf_rope);
        pc.ks_part = c->at<float>(c->L.pf_ks_part); pc.ks_count = c->at<int32_t>(c->L.pf_ks_count);
        int last_T = 0;
        for (int at = p0; at < m; at += PREFILL_CHUNK) {
            pc.p0 = at; pc.T = last_T = (m - at < PREFILL_CHUNK) ? m - at : PREFILL_CHUNK;
            HIPCHK(c, spdk::prefill_chunk(c->stream, pc));
        }
        GemvArgs g{};
        g.W = c->lm_head; g.gain = c->final_norm; g.eps = mc.rms_eps; g.x = pc.h + (size_t)(last_T - 1) * mc.d_model;
        g.y = c->at<float>(c->L.logits); g.rows = mc.vocab; g.cols = mc.d_model;
        HIPCHK(c, spdk::gemv(c->stream, mc.dtype, EPI_PLAIN, g, c->num_cu));
        HIPCHK(c, spdk::fill_i32(c->stream, &c->st()->pos, m, 1));
        c->pos = m;
        c->state = ST_PREFILLED;
        return SPD_OK;
    }
    auto one_token = [&]() -> hipError_t {
        hipError_t e = enqueue_forward(c, 0, 1, false);
        if (e == hipSuccess) e = spdk::advance(c->stream, c->st());
        return e;
    };
    if (graphs_usable(c) && n > 2) {
        if (!c->prefill_exec) {
            const int rc = capture(c, &c->prefill_exec, one_token);
            if (rc != SPD_OK) return rc;
        }
        for (int i = 0; i < n - 1; ++i) HIPCHK(c, hipGraphLaunch(c->prefill_exec, c->stream));
    } else {
        for (int i = 0; i < n - 1; ++i) HIPCHK(c, one_token());
    }
    HIPCHK(c, enqueue_forward(c, 0, 1, true));   // last prefix position: keep its logits
    HIPCHK(c, spdk::advance(c->stream, c->st()));
    c->pos = m;
    c->state = ST_PREFILLED;
    return SPD_OK;
}

int spd_prefill(spd_ctx *c, const int32_t *prefix, int32_t m) {
    if (!c) return SPD_EINVAL;
    if (!prefix) return fail(c, SPD_EINVAL, "prefix is null");
    if (m < 1) return fail(c, SPD_EINVAL, "prefix must hold at least one token");
    if (m >= c->cfg.max_ctx) return fail(c, SPD_ECTX_OVERFLOW, "prefix does not fit max_ctx");
    for (int i = 0; i < m; ++i)
        if (prefix[i] < 0 || prefix[i] >= c->cfg.vocab) return fail(c, SPD_EINVAL, "prefix token id outside [0, vocab)");
    c->text.assign(prefix, prefix + m);
    return run_prefix_pass(c, 0, m);
}

static int copy_step_outputs(spd_ctx *c, int k, int32_t *out_tok, int32_t *out_par, float *out_sc) {
    if (!out_tok && !out_par && !out_sc) return SPD_OK;
    DevState *hs = (DevState *)c->pinned;
    HIPCHK(c, hipMemcpyAsync(hs, c->st(), sizeof(DevState), hipMemcpyDeviceToHost, c->stream));
    if (c->timing) HIPCHK(c, drain_timing(c));
    HIPCHK(c, hipStreamSynchronize(c->stream));
    STATECHK(c, hs);
    for (int i = 0; i < k; ++i) {
        if (out_tok) out_tok[i] = hs->new_tok[i];
        if (out_par) out_par[i] = hs->new_parent[i];
        if (out_sc) out_sc[i] = hs->logscore[i];
    }
    return SPD_OK;
}

int spd_step(spd_ctx *c, const spd_decode_cfg *dc, int32_t *out_tok, int32_t *out_par, float *out_sc) {
    if (!c) return SPD_EINVAL;
    if (const char *why = check_dc(c, dc)) return fail(c, SPD_EINVAL, why);
    if (c->state == ST_CREATED) return fail(c, SPD_ESTATE, "spd_step before spd_prefill");
    if (c->state == ST_PREFILLED) {
        HIPCHK(c, enqueue_decide(c, *dc, c->at<float>(c->L.logits), 1, 0));
        c->state = ST_STEPPING;
        c->k = dc->k;
        c->n_gen = 1;
        return copy_step_outputs(c, dc->k, out_tok, out_par, out_sc);
    }
    if (dc->k != c->k) return fail(c, SPD_EINVAL, "k changed within a generation");
    if (c->pos + 1 > c->cfg.max_ctx) return fail(c, SPD_ECTX_OVERFLOW, "KV cache is full");
    if (c->n_gen >= c->cfg.max_ctx) return fail(c, SPD_ECTX_OVERFLOW, "token history is full");
    auto body = [&]() -> hipError_t {
        hipError_t e = enqueue_forward(c, 1, dc->k, true);
        if (e == hipSuccess) e = enqueue_decide(c, *dc, c->at<float>(c->L.logits), 0, 1);
        return e;
    };
    if (graphs_usable(c)) {
        if (c->step_exec && std::memcmp(&c->step_dc, dc, sizeof(*dc)) != 0) drop_graph(c->step_exec);
        if (!c->step_exec) {
            const int rc = capture(c, &c->step_exec, body);
            if (rc != SPD_OK) return rc;
            c->step_dc = *dc;
        }
        HIPCHK(c, hipGraphLaunch(c->step_exec, c->stream));
    } else {
        HIPCHK(c, body());
    }
    c->pos += 1;
    c->n_gen += 1;
    return copy_step_outputs(c, dc->k, out_tok, out_par, out_sc);
}

int spd_commit(spd_ctx *c, float u, int32_t *out_chosen, int32_t *out_tokens, int32_t cap, int32_t *out_n) {
    if (!c) return SPD_EINVAL;
    if (!(u >= 0.f && u < 1.f)) return fail(c, SPD_EINVAL, "the draw u must lie in [0, 1)");
    if (c->state != ST_STEPPING) return fail(c, SPD_ESTATE, "no drafts to commit: run spd_step or spd_nucleus_step first");
    const int k = c->k, n = c->n_gen, base = (int)c->text.size();
    if (base + n >= c->cfg.max_ctx) return fail(c, SPD_ECTX_OVERFLOW, "committed text does not fit max_ctx");
    if (out_tokens && cap < n) return fail(c, SPD_EINVAL, "token buffer too small");
    const size_t hist_bytes = (size_t)n * SPD_K_MAX * 4;
    DevState *hs = (DevState *)c->pinned;
    int32_t *ht = (int32_t *)(c->pinned + up(sizeof(DevState)));
    int32_t *hp = ht + (size_t)c->cfg.max_ctx * SPD_K_MAX;
    HIPCHK(c, hipMemcpyAsync(hs, c->st(), sizeof(DevState), hipMemcpyDeviceToHost, c->stream));
    HIPCHK(c, hipMemcpyAsync(ht, c->ws + c->L.hist_tok, hist_bytes, hipMemcpyDeviceToHost, c->stream));
    HIPCHK(c, hipMemcpyAsync(hp, c->ws + c->L.hist_par, hist_bytes, hipMemcpyDeviceToHost, c->stream));
    if (c->timing) HIPCHK(c, drain_timing(c));
    HIPCHK(c, hipStreamSynchronize(c->stream));
    STATECHK(c, hs);
    // sample draft i with its superposition weight (Eq. 2): inverse CDF over the rank order
    double total = 0.0;
    for (int i = 0; i < k; ++i) total += (double)hs->gamma[i];
    int chosen = k - 1;
    double cum = 0.0;
    for (int i = 0; i < k; ++i) {
        cum += (double)hs->gamma[i];
        if (cum > (double)u * total) { chosen = i; break; }
    }
    std::vector<int32_t> toks((size_t)n);
    int slot = chosen;
    for (int t = n - 1; t >= 0; --t) {   // walk the parent indices back from the last timestep
        toks[(size_t)t] = ht[(size_t)t * SPD_K_MAX + slot];
        const int par = hp[(size_t)t * SPD_K_MAX + slot];
        if (t > 0 && (par < 0 || par >= k)) return fail(c, SPD_EHIP, "corrupt parent index in the device history");
        if (t > 0) slot = par;
    }
    for (int t = 0; t < n; ++t)
        if (toks[(size_t)t] < 0 || toks[(size_t)t] >= c->cfg.vocab) return fail(c, SPD_EHIP, "corrupt token in the device history");
    if (out_chosen) *out_chosen = chosen;
    if (out_n) *out_n = n;
    if (out_tokens) std::memcpy(out_tokens, toks.data(), (size_t)n * 4);
    c->text.insert(c->text.end(), toks.begin(), toks.end());
    // One draft (a greedy or nucleus pass): the cache already holds exactly this text except for
    // its newest token.  k > 1: positions base .. hold keys/values of superposed inputs; redo them.
    const int p0 = (k == 1) ? base + n - 1 : base;
    return run_prefix_pass(c, p0, base + n);
}

static const char *check_sample(const spd_sample_cfg *sc, float u);

int spd_nucleus_step(spd_ctx *c, const spd_sample_cfg *sc, float u, int32_t *out_tok, float *out_logprob) {
    if (!c) return SPD_EINVAL;
    if (const char *why = check_sample(sc, u)) return fail(c, SPD_EINVAL, why);
    if (c->state == ST_CREATED) return fail(c, SPD_ESTATE, "spd_nucleus_step before spd_prefill");
    if (c->state == ST_STEPPING && c->k != 1) return fail(c, SPD_ESTATE, "a generation with k > 1 drafts is in progress");
    uint32_t bits;
    std::memcpy(&bits, &u, 4);
    HIPCHK(c, hipMemsetD32Async((hipDeviceptr_t)&c->st()->sample_u, (int)bits, 1, c->stream));
    if (c->state == ST_PREFILLED) {
        HIPCHK(c, enqueue_sample(c, *sc, c->at<float>(c->L.logits), 1, 0));
        c->state = ST_STEPPING;
        c->k = 1;
        c->n_gen = 1;
    } else {
        if (c->pos + 1 > c->cfg.max_ctx) return fail(c, SPD_ECTX_OVERFLOW, "KV cache is full");
        if (c->n_gen >= c->cfg.max_ctx) return fail(c, SPD_ECTX_OVERFLOW, "token history is full");
        auto body = [&]() -> hipError_t {
            hipError_t e = enqueue_forward(c, 1, 1, true);
            if (e == hipSuccess) e = enqueue_sample(c, *sc, c->at<float>(c->L.logits), 0, 1);
            return e;
        };
        if (graphs_usable(c)) {
            if (c->nucleus_exec && std::memcmp(&c->nucleus_sc, sc, sizeof(*sc)) != 0) drop_graph(c->nucleus_exec);
            if (!c->nucleus_exec) {
                const int rc = capture(c, &c->nucleus_exec, body);
                if (rc != SPD_OK) return rc;
                c->nucleus_sc = *sc;
            }
            HIPCHK(c, hipGraphLaunch(c->nucleus_exec, c->stream));
        } else {
            HIPCHK(c, body());
        }
        c->pos += 1;
        c->n_gen += 1;
    }
    if (!out_tok && !out_logprob) return SPD_OK;
    DevState *hs = (DevState *)c->pinned;
    HIPCHK(c, hipMemcpyAsync(hs, c->st(), sizeof(DevState), hipMemcpyDeviceToHost, c->stream));
    if (c->timing) HIPCHK(c, drain_timing(c));
    HIPCHK(c, hipStreamSynchronize(c->stream));
    STATECHK(c, hs);
    if (out_tok) *out_tok = hs->new_tok[0];
    if (out_logprob) *out_logprob = hs->top_logp[0];
    return SPD_OK;
}

static const char *check_sample(const spd_sample_cfg *sc, float u) {
    if (!sc) return "sample cfg is null";
    if (!(sc->top_p > 0.f && sc->top_p <= 1.f)) return "top_p outside (0, 1]";
    if (!(sc->tau > 0.f)) return "tau must be positive";
    if (!(u >= 0.f && u < 1.f)) return "the draw u must lie in [0, 1)";
    return nullptr;
}

int spd_nucleus_sample(spd_ctx *c, const spd_sample_cfg *sc, float u, const float *dev_logits, int32_t first) {
    if (!c) return SPD_EINVAL;
    if (const char *why = check_sample(sc, u)) return fail(c, SPD_EINVAL, why);
    if (!dev_logits) return fail(c, SPD_EINVAL, "logits pointer is null");
    if (c->state == ST_CREATED) return fail(c, SPD_ESTATE, "spd_nucleus_sample before spd_prefill");
    if (!first && (c->state != ST_STEPPING || c->k != 1)) return fail(c, SPD_ESTATE, "no nucleus pass is in progress");
    if (!first && c->n_gen >= c->cfg.max_ctx) return fail(c, SPD_ECTX_OVERFLOW, "token history is full");
    uint32_t bits;
    std::memcpy(&bits, &u, 4);
    HIPCHK(c, hipMemsetD32Async((hipDeviceptr_t)&c->st()->sample_u, (int)bits, 1, c->stream));
    HIPCHK(c, enqueue_sample(c, *sc, dev_logits, first ? 1 : 0, 0));
    if (first) { c->state = ST_STEPPING; c->k = 1; c->n_gen = 1; }
    else c->n_gen += 1;
    return SPD_OK;
}

int spd_get_nucleus_info(spd_ctx *c, int32_t *out_size, float *out_mass, float *out_sum_logprob) {
    if (!c) return SPD_EINVAL;
    if (c->state != ST_STEPPING || c->k != 1) return fail(c, SPD_ESTATE, "no nucleus step has run");
    DevState *hs = (DevState *)c->pinned;
    HIPCHK(c, hipMemcpyAsync(hs, c->st(), sizeof(DevState), hipMemcpyDeviceToHost, c->stream));
    HIPCHK(c, hipStreamSynchronize(c->stream));
    STATECHK(c, hs);
    if (out_size) *out_size = hs->nucleus_size;
    if (out_mass) *out_mass = hs->nucleus_mass;
    if (out_sum_logprob) *out_sum_logprob = hs->logscore[0];
    return SPD_OK;
}

int spd_generate(spd_ctx *c, const int32_t *prefix, int32_t m, const spd_decode_cfg *dc, int32_t n_tokens,
                 int32_t *out_drafts, float *out_sc) {
    if (!c) return SPD_EINVAL;
    if (const char *why = check_dc(c, dc)) return fail(c, SPD_EINVAL, why);
    if (n_tokens < 1) return fail(c, SPD_EINVAL, "n_tokens must be >= 1");
    if (!out_drafts) return fail(c, SPD_EINVAL, "out_drafts is null");
    if ((int64_t)m + n_tokens - 1 > c->cfg.max_ctx) return fail(c, SPD_ECTX_OVERFLOW, "prefix + generation exceeds max_ctx");
    int rc = spd_prefill(c, prefix, m);
    if (rc != SPD_OK) return rc;
    for (int t = 0; t < n_tokens; ++t) {
        rc = spd_step(c, dc, nullptr, nullptr, nullptr);
        if (rc != SPD_OK) return rc;
    }
    const int k = dc->k;
    const size_t hist_bytes = (size_t)n_tokens * SPD_K_MAX * 4;
    DevState *hs = (DevState *)c->pinned;
    int32_t *ht = (int32_t *)(c->pinned + up(sizeof(DevState)));
    int32_t *hp = ht + (size_t)c->cfg.max_ctx * SPD_K_MAX;
    HIPCHK(c, hipMemcpyAsync(hs, c->st(), sizeof(DevState), hipMemcpyDeviceToHost, c->stream));
    HIPCHK(c, hipMemcpyAsync(ht, c->ws + c->L.hist_tok, hist_bytes, hipMemcpyDeviceToHost, c->stream));
    HIPCHK(c, hipMemcpyAsync(hp, c->ws + c->L.hist_par, hist_bytes, hipMemcpyDeviceToHost, c->stream));
    if (c->timing) HIPCHK(c, drain_timing(c));
    HIPCHK(c, hipStreamSynchronize(c->stream));
    STATECHK(c, hs);
    for (int r = 0; r < k; ++r) {   // walk the parent indices back from the last timestep
        int slot = r;
        for (int t = n_tokens - 1; t >= 0; --t) {
            out_drafts[(size_t)r * n_tokens + t] = ht[(size_t)t * SPD_K_MAX + slot];
            const int par = hp[(size_t)t * SPD_K_MAX + slot];
            if (t > 0 && (par < 0 || par >= k)) return fail(c, SPD_EHIP, "corrupt parent index in the device history");
            slot = par;
        }
        if (out_sc) out_sc[r] = hs->logscore[r];
    }
    return SPD_OK;
}

int spd_get_state(spd_ctx *c, int32_t *out_k, int32_t *out_tails, float *out_sc, float *out_gamma) {
    if (!c) return SPD_EINVAL;
    if (c->state != ST_STEPPING) return fail(c, SPD_ESTATE, "no drafts yet: run the first spd_step");
    DevState *hs = (DevState *)c->pinned;
    HIPCHK(c, hipMemcpyAsync(hs, c->st(), sizeof(DevState), hipMemcpyDeviceToHost, c->stream));
    HIPCHK(c, hipStreamSynchronize(c->stream));
    STATECHK(c, hs);
    if (out_k) *out_k = c->k;
    for (int i = 0; i < c->k; ++i) {
        if (out_tails) std::memcpy(out_tails + i * SPD_TAIL, hs->tails[i], SPD_TAIL * 4);
        if (out_sc) out_sc[i] = hs->logscore[i];
        if (out_gamma) out_gamma[i] = hs->gamma[i];
    }
    return SPD_OK;
}

int spd_set_state(spd_ctx *c, int32_t k, const int32_t *tails, const float *sc) {
    if (!c) return SPD_EINVAL;
    if (c->state != ST_STEPPING) return fail(c, SPD_ESTATE, "no drafts yet: run the first spd_step");
    if (k != c->k || !tails || !sc) return fail(c, SPD_EINVAL, "k must match the generation; tails and logscores required");
    for (int i = 0; i < k; ++i) {
        if (tails[i * SPD_TAIL + SPD_TAIL - 1] < 0) return fail(c, SPD_EINVAL, "a draft's newest token is missing");
        for (int q = 0; q < SPD_TAIL; ++q)
            if (tails[i * SPD_TAIL + q] >= c->cfg.vocab) return fail(c, SPD_EINVAL, "tail token id >= vocab");
    }
    HIPCHK(c, hipStreamSynchronize(c->stream));
    DevState *hs = (DevState *)c->pinned;
    std::memset(hs, 0, sizeof(DevState));
    for (int i = 0; i < k; ++i) {
        std::memcpy(hs->tails[i], tails + i * SPD_TAIL, SPD_TAIL * 4);
        hs->logscore[i] = sc[i];
    }
    DevState *d = c->st();
    HIPCHK(c, hipMemcpyAsync(d->tails, hs->tails, sizeof(hs->tails), hipMemcpyHostToDevice, c->stream));
    HIPCHK(c, hipMemcpyAsync(d->logscore, hs->logscore, sizeof(hs->logscore), hipMemcpyHostToDevice, c->stream));
    HIPCHK(c, spdk::renorm(c->stream, d, k));
    HIPCHK(c, hipStreamSynchronize(c->stream));
    return SPD_OK;
}

int spd_read_logits(spd_ctx *c, float *out) {
    if (!c) return SPD_EINVAL;
    if (!out) return fail(c, SPD_EINVAL, "out is null");
    if (c->state == ST_CREATED) return fail(c, SPD_ESTATE, "no forward pass has run");
    float *stage = (float *)(c->pinned + c->pinned_bytes - (size_t)c->cfg.vocab * 4);
    HIPCHK(c, hipMemcpyAsync(stage, c->ws + c->L.logits, (size_t)c->cfg.vocab * 4, hipMemcpyDeviceToHost, c->stream));
    HIPCHK(c, hipStreamSynchronize(c->stream));
    std::memcpy(out, stage, (size_t)c->cfg.vocab * 4);
    return SPD_OK;
}

int spd_get_step_info(spd_ctx *c, int32_t *top_ids, float *top_logp, float *cs, int32_t *cv, float *cp) {
    if (!c) return SPD_EINVAL;
    if (c->state != ST_STEPPING) return fail(c, SPD_ESTATE, "no step has run");
    DevState *hs = (DevState *)c->pinned;
    HIPCHK(c, hipMemcpyAsync(hs, c->st(), sizeof(DevState), hipMemcpyDeviceToHost, c->stream));
    HIPCHK(c, hipStreamSynchronize(c->stream));
    STATECHK(c, hs);
    const int k = c->k;
    for (int i = 0; i < k; ++i) {
        if (top_ids) top_ids[i] = hs->top_ids[i];
        if (top_logp) top_logp[i] = hs->top_logp[i];
    }
    for (int e = 0; e < k * k; ++e) {
        if (cs) cs[e] = hs->cand_score[e];
        if (cv) cv[e] = hs->cand_valid[e];
        if (cp) cp[e] = hs->cand_png[e];
    }
    return SPD_OK;
}

int spd_expand_prune(spd_ctx *c, const spd_decode_cfg *dc, const float *dev_logits, int32_t first) {
    if (!c) return SPD_EINVAL;
    if (const char *why = check_dc(c, dc)) return fail(c, SPD_EINVAL, why);
    if (!dev_logits) return fail(c, SPD_EINVAL, "logits pointer is null");
    if (c->state == ST_CREATED) return fail(c, SPD_ESTATE, "spd_expand_prune before spd_prefill");
    if (first) {
        HIPCHK(c, enqueue_decide(c, *dc, dev_logits, 1, 0));
        c->state = ST_STEPPING; c->k = dc->k; c->n_gen = 1;
        return SPD_OK;
    }
    if (c->state != ST_STEPPING) return fail(c, SPD_ESTATE, "the first timestep has not run");
    if (dc->k != c->k) return fail(c, SPD_EINVAL, "k changed within a generation");
    if (c->n_gen >= c->cfg.max_ctx) return fail(c, SPD_ECTX_OVERFLOW, "token history is full");
    HIPCHK(c, enqueue_decide(c, *dc, dev_logits, 0, 0));
    c->n_gen += 1;
    return SPD_OK;
}

int spd_test_state_status(const int32_t *state_words, size_t n_words) {
    if (!state_words || n_words * 4 < sizeof(DevState)) return SPD_EINVAL;
    DevState hs;
    std::memcpy(&hs, state_words, sizeof(DevState));
    return device_state_status(nullptr, &hs);
}

int spd_test_state_layout(size_t *out_words, size_t *out_err_word) {
    if (!out_words || !out_err_word) return SPD_EINVAL;
    *out_words = (sizeof(DevState) + 3) / 4;
    *out_err_word = offsetof(DevState, err) / 4;
    return SPD_OK;
}

int spd_test_poke_err(spd_ctx *c, int32_t value) {
    if (!c) return SPD_EINVAL;
    HIPCHK(c, spdk::fill_i32(c->stream, &c->st()->err, value, 1));
    return SPD_OK;
}

int spd_position(const spd_ctx *c, int32_t *out_pos) {
    if (!c || !out_pos) return SPD_EINVAL;
    *out_pos = c->pos;
    return SPD_OK;
}

int spd_set_graph(spd_ctx *c, int32_t enable) {
    if (!c) return SPD_EINVAL;
    c->use_graph = enable != 0;
    return SPD_OK;
}

int spd_set_fused(spd_ctx *c, int32_t enable) {
    if (!c) return SPD_EINVAL;
    if (enable && c->fused_blocks == 0) return fail(c, SPD_EINVAL, "no fused forward kernel for this model shape");
    if ((enable != 0) != c->use_fused) {
        drop_graph(c->step_exec); drop_graph(c->prefill_exec); drop_graph(c->nucleus_exec);
        // the per-operator kernels leave plain values in the first arena: unset both again
        if (enable) HIPCHK(c, reset_fused_state(c));
    }
    c->use_fused = enable != 0;
    return SPD_OK;
}

int spd_set_dense_prefill(spd_ctx *c, int32_t enable) {
    if (!c) return SPD_EINVAL;
    if (enable && !c->L.dense) return fail(c, SPD_EINVAL, "no dense prefix pass for this model (bf16 weights, d_head <= 128, widths divisible by 128, d_model <= 8192)");
    c->use_dense = enable != 0;
    return SPD_OK;
}

int spd_get_dense_prefill(const spd_ctx *c, int32_t *out_enabled) {
    if (!c || !out_enabled) return SPD_EINVAL;
    *out_enabled = c->use_dense ? 1 : 0;
    return SPD_OK;
}

int spd_get_fused(const spd_ctx *c, int32_t *out_enabled) {
    if (!c || !out_enabled) return SPD_EINVAL;
    *out_enabled = (c->use_fused && c->fused_blocks > 0) ? 1 : 0;
    return SPD_OK;
}

int spd_set_kernel_timing(spd_ctx *c, int32_t enable) {
    if (!c) return SPD_EINVAL;
    if (c->timing && !enable) HIPCHK(c, drain_timing(c));
    c->timing = enable != 0;
    if (enable) { std::memset(c->kc_ms, 0, sizeof(c->kc_ms)); std::memset(c->kc_n, 0, sizeof(c->kc_n)); }
    return SPD_OK;
}

int spd_get_phase_clock(spd_ctx *c, int32_t cap, int64_t *out_stamps, int32_t *out_n, int32_t *out_blocks) {
    if (!c) return SPD_EINVAL;
    if (!out_stamps || !out_n || !out_blocks) return fail(c, SPD_EINVAL, "null output");
    const int n = 2 * (5 * c->cfg.n_layers + 2);
    if (c->fused_blocks <= 0) return fail(c, SPD_ESTATE, "no fused forward kernel for this model shape");
    const int nb = c->fused_blocks < FUSED_PROF_BLOCKS ? c->fused_blocks : FUSED_PROF_BLOCKS;
    if ((int64_t)cap < (int64_t)n * nb) return fail(c, SPD_EINVAL, "buffer too small for the phase stamps");
    HIPCHK(c, hipStreamSynchronize(c->stream));
    HIPCHK(c, hipMemcpy(out_stamps, c->ws + c->L.prof, (size_t)n * nb * 8, hipMemcpyDeviceToHost));
    *out_n = n;
    *out_blocks = nb;
    return SPD_OK;
}

int spd_get_kernel_timing(spd_ctx *c, int32_t cap, const char **names, float *ms, int64_t *launches, int32_t *out_n) {
    if (!c) return SPD_EINVAL;
    if (!out_n) return fail(c, SPD_EINVAL, "out_n is null");
    HIPCHK(c, drain_timing(c));
    int n = 0;
    for (int i = 0; i < KC_N && n < cap; ++i, ++n) {
        if (names) names[n] = KC_NAMES[i];
        if (ms) ms[n] = (float)c->kc_ms[i];
        if (launches) launches[n] = c->kc_n[i];
    }
    *out_n = n;
    return SPD_OK;
}

// ---- stand-alone operators
static int device_cus() {
    static int cus = 0;
    if (!cus) {
        int dev = 0;
        hipDeviceProp_t p;
        if (hipGetDevice(&dev) != hipSuccess || hipGetDeviceProperties(&p, dev) != hipSuccess) return -1;
        if (spdk::init() != hipSuccess) return -1;
        cus = p.multiProcessorCount;
    }
    return cus;
}

static bool op_shape_ok(int dtype, int rows, int cols) {
    if (dtype != SPD_DTYPE_FP32 && dtype != SPD_DTYPE_BF16) return false;
    const int vec = dtype == SPD_DTYPE_BF16 ? 8 : 4;
    return rows > 0 && cols > 0 && cols % vec == 0 && spdk::gemv_lds_bytes(dtype, cols) <= 160 * 1024 - 1024;
}

int spd_op_gemv(int32_t dtype, const void *W, const void *gain, float eps, const float *x, const float *resid,
                float *y, int32_t rows, int32_t cols, void *hip_stream) {
    if (!W || !x || !y || !op_shape_ok(dtype, rows, cols) || rows % 2) return SPD_EINVAL;
    const int cus = device_cus();
    if (cus < 0) return SPD_EHIP;
    GemvArgs g{};
    g.W = W; g.gain = gain; g.eps = eps; g.x = x; g.resid = resid; g.y = y; g.rows = rows; g.cols = cols;
    return spdk::gemv((hipStream_t)hip_stream, dtype, resid ? EPI_RESID : EPI_PLAIN, g, cus) == hipSuccess ? SPD_OK : SPD_EHIP;
}

int spd_op_swiglu(int32_t dtype, const void *Wg, const void *Wu, const void *gain, float eps, const float *x,
                  float *u, int32_t rows, int32_t cols, void *hip_stream) {
    if (!Wg || !Wu || !x || !u || !op_shape_ok(dtype, rows, cols)) return SPD_EINVAL;
    const int cus = device_cus();
    if (cus < 0) return SPD_EHIP;
    GemvArgs g{};
    g.W = Wg; g.W2 = Wu; g.gain = gain; g.eps = eps; g.x = x; g.y = u; g.rows = rows; g.cols = cols;
    return spdk::gemv((hipStream_t)hip_stream, dtype, EPI_SWIGLU, g, cus) == hipSuccess ? SPD_OK : SPD_EHIP;
}

size_t spd_op_attention_scratch_bytes(int32_t n_heads, int32_t d_head, int32_t cap_ctx) {
    if (n_heads <= 0 || d_head <= 0 || cap_ctx <= 0) return 0;
    const size_t splits = (size_t)(cap_ctx + ATTN_CHUNK - 1) / ATTN_CHUNK;
    return up((size_t)n_heads * ATTN_COUNTER_STRIDE * 4) + up((size_t)n_heads * splits * (d_head + 2) * 4);
}

int spd_op_attention(int32_t dtype, const float *q, const void *K, const void *V, float *out, void *scratch,
                     int32_t n_heads, int32_t n_kv_heads, int32_t d_head, int32_t n_ctx, int32_t cap_ctx,
                     void *hip_stream) {
    const int rc = spdk::attention_args_status(dtype, q, K, V, out, n_heads, n_kv_heads, d_head, n_ctx, cap_ctx);
    if (rc != SPD_OK) return rc;
    if (!scratch || ((uintptr_t)scratch & (ALIGN - 1))) return SPD_EINVAL;
    return spdk::attention_on_scratch((hipStream_t)hip_stream, dtype, q, K, V, out, scratch, n_heads, n_kv_heads,
                                      d_head, n_ctx, cap_ctx);
}

}  // extern "C"
