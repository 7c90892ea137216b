// Internal declarations shared by the host library and the HIP kernels of libspd.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "spd.h"

// ---------------------------------------------------------------- n-gram store (device)
// One open-addressing table (linear probing) for every order.  A slot holds up to six token
// ids, oldest first, and a 64-bit count:
//   count entry of order n : tok[0..n-1] >= 0, the rest NG_PAD
//   total entry of order n : tok[0..n-2] = context, tok[n-1] = NG_TOTAL, the rest NG_PAD;
//                            count = sum of the counts of all order-n entries with that context
//   empty slot             : tok[0] = NG_EMPTY
struct NgramSlot {
    int32_t tok[6];
    uint32_t cnt_lo, cnt_hi;
};
static_assert(sizeof(NgramSlot) == 32, "slot must be 32 bytes");
constexpr int32_t NG_PAD = -1;
constexpr int32_t NG_TOTAL = -2;
constexpr int32_t NG_EMPTY = -3;

struct NgramDev {
    const NgramSlot *slots;  // device
    uint64_t capacity;       // number of slots; home slot = mulhi64(hash, capacity)
    int32_t max_probe;       // longest displacement of any stored key
    int32_t present[SPD_N_ORDERS];
    float lambda[SPD_N_ORDERS];
};

// Home slot of a hash value: floor(h * capacity / 2^64).
__host__ __device__ inline uint64_t ngram_home(uint64_t h, uint64_t capacity) {
#if defined(__HIP_DEVICE_COMPILE__)
    return __umul64hi(h, capacity);
#else
    return (uint64_t)(((unsigned __int128)h * capacity) >> 64);
#endif
}

__host__ __device__ inline uint64_t ngram_hash(const int32_t *tok6) {
    uint64_t h = 0x9E3779B97F4A7C15ull;
    for (int i = 0; i < 6; ++i) {
        h ^= (uint64_t)(uint32_t)tok6[i];
        h *= 0xFF51AFD7ED558CCDull;
        h ^= h >> 29;
    }
    h *= 0xC4CEB9FE1A85EC53ull;
    h ^= h >> 32;
    return h;
}

// ---------------------------------------------------------------- draft state (device)
constexpr int SPD_KK = SPD_K_MAX * SPD_K_MAX;

struct DevState {
    int32_t pos;    // number of cached positions = position the next forward pass writes
    int32_t n_gen;  // tokens generated so far per draft
    int32_t k;
    int32_t err;
    int32_t prefix_tail[SPD_TAIL];        // last 5 prefix tokens, oldest first, NG_PAD-padded
    int32_t tails[SPD_K_MAX][SPD_TAIL];   // last 5 tokens of (prefix, draft i)
    float logscore[SPD_K_MAX];            // log p_i
    float gamma[SPD_K_MAX];               // Eq. 2 on the current scores
    float gamma_in[SPD_K_MAX];            // the weights the last superposed input used
    int32_t top_ids[SPD_K_MAX];           // KeepTopK of the last step
    float top_logp[SPD_K_MAX];
    int32_t new_tok[SPD_K_MAX];           // newest token / parent of each surviving draft
    int32_t new_parent[SPD_K_MAX];
    float cand_score[SPD_KK];             // option (i, j) at [i * k + j]
    int32_t cand_valid[SPD_KK];
    float cand_png[SPD_KK];
    float sample_u;                       // nucleus pass: the uniform draw of the next token (host-written)
    int32_t nucleus_size;                 // nucleus pass: size and mass of the last nucleus
    float nucleus_mass;
};

// ---------------------------------------------------------------- kernel launch arguments
enum GemvEpilogue { EPI_PLAIN = 0, EPI_RESID = 1, EPI_QKV = 2, EPI_SWIGLU = 3 };

struct GemvArgs {
    const void *W;       // [rows, cols]
    const void *W2;      // EPI_SWIGLU: the "up" matrix
    const void *gain;    // [cols] in weight dtype, or null: no RMS normalisation of x
    float eps;
    const float *x;      // [cols]
    const float *resid;  // EPI_RESID: may alias y
    float *y;            // EPI_PLAIN/RESID/SWIGLU: [rows]; EPI_QKV: q buffer [n_q_rows]
    int32_t rows, cols;
    // EPI_QKV
    void *kcache, *vcache;      // [n_kv_heads, cap_ctx, d_head], fp32 or (kv_half) fp16
    int32_t kv_half;
    const DevState *st;         // position
    const double *inv_freq;     // [d_head / 2]
    int32_t n_q_rows, n_kv_rows, d_head, cap_ctx;
    int32_t first_block;        // fused kernel: blocks below this index take no rows of this phase
    float *k_new, *v_new;       // fused kernel, EPI_QKV: [n_kv_rows] the new key and value rows also go here (see AttnArgs)
    int32_t chunk_span;         // fused kernel: the phase's units are cut into chunks of this many, every block owns a
                                // share of each chunk and walks them in order; 0 = one chunk
    long long twin;             // fused kernel: byte offset from y to the same vector in the other activation arena
                                // (every element stored to y is accompanied by ACT_UNSET stored there); 0 = none
};

constexpr int ATTN_COUNTER_STRIDE = 64;

struct AttnArgs {
    const float *q;   // [n_heads, d_head]
    const void *K, *V;
    float *out;       // [n_heads, d_head]
    float *part;      // [n_heads, max_splits, d_head + 2]
    int32_t *counters;  // [n_heads] x ATTN_COUNTER_STRIDE ints (one 256-byte line per head: the chunks' arrivals on different
                        // heads do not queue behind one another), zero between launches
    const DevState *st;  // n_ctx = st->pos + 1 when non-null
    int32_t n_ctx;       // used when st is null
    int32_t n_heads, n_kv_heads, d_head, cap_ctx, chunk, max_splits;
    long long out_twin;  // fused kernel: byte offset from out to its twin in the other activation arena; 0 = none
    const float *k_new, *v_new;  // fused kernel: [n_kv_heads, d_head] key and value rows of the newest position as the QKV phase
                                 // of this launch writes them (awaited as data, like q); null: everything is read from the cache
};

struct SuperposeArgs {
    const void *embed;
    DevState *st;
    const int32_t *prefix;  // mode 0: token = prefix[st->pos]
    float *h;
    int32_t d_model, mode, k;
    long long twin;         // fused kernel: byte offset from h to its twin in the other activation arena; 0 = none
};

struct TopkArgs {
    const float *logits;
    int32_t vocab, k, n_part, per_part;
    float tau;
    float *pv;    // [n_part, SPD_K_MAX]
    int32_t *pi;  // [n_part, SPD_K_MAX]
    float *pm, *ps;  // [n_part]: largest scaled logit of the slice, sum of exp(z - that)
    float *pn;       // [n_part]: smallest scaled logit of the slice
};

struct NucleusArgs {
    const float *logits;
    int32_t vocab;
    DevState *st;
    const float *pm, *ps, *pn;   // per-slice max, sum of exp and min of logit / tau (topk_partial)
    int32_t n_part, per_part;    // one block per slice of per_part entries
    unsigned long long *sc_pb;   // scratch, [vocab]: first-level bucket above the probability in 40-bit fixed point
    unsigned *sc_count;          // blocks that have finished their slice; zero between calls
    unsigned long long *sc_hist; // scratch, [2048]: entry count above probability mass per first-level bucket; zero between calls
    uint16_t *sc_bk;             // scratch, [32768]: first-level bucket per entry, 0xFFFF past the vocabulary (vocab <= 32768 only)
    float top_p, tau;
    int32_t first, advance;
    int32_t *hist_tok, *hist_par;
    int32_t max_gen;
};

struct ExpandArgs {
    DevState *st;
    const float *pv;
    const int32_t *pi;
    const float *pm, *ps;
    int32_t n_part;
    NgramDev ng;
    int32_t k;
    float alpha, tau, delta;
    int32_t first, advance;
    int32_t *hist_tok, *hist_par;  // [max_gen, SPD_K_MAX]
    int32_t max_gen;
};

// Activation vectors of one forward pass.  Every vector a phase produces has an address of
// its own (no buffer is written twice within a pass), so a consumer on another XCD can read
// it through its L2 without ever meeting a stale line: byte offsets from `base`.
struct ActLayout {
    size_t h0;                 // the input vector x~
    size_t layer0, stride;     // layer l's block starts at layer0 + l * stride
    size_t q, att, h1, u, h2;  // within a layer block: query, attention output, residual stream
                               // after attention, SwiGLU output, residual stream after the FFN
    size_t kn, vn;             // and the newest position's key and value rows
    __host__ __device__ __forceinline__ float *at(char *base, size_t off) const { return (float *)(base + off); }
    __host__ __device__ __forceinline__ float *h_in(char *base, int l) const { return l == 0 ? at(base, h0) : at(base, layer0 + (size_t)(l - 1) * stride + h2); }
    __host__ __device__ __forceinline__ float *vec(char *base, int l, size_t which) const { return at(base, layer0 + (size_t)l * stride + which); }
};

// The fused forward kernel synchronises through the activation vectors themselves: a vector
// element holds this bit pattern (a NaN no arithmetic produces) until its producer has stored
// it.  There are two activation arenas; a launch works in one (they alternate from launch to
// launch) and leaves every element of the other at ACT_UNSET for its successor.
constexpr uint32_t ACT_UNSET = 0xFFFFFFFFu;

// Arguments of the fused forward kernel (one persistent launch for the whole model).
struct FusedArgsHost {
    SuperposeArgs sup;
    const spd_layer_weights *layers;   // DEVICE array [n_layers]
    const void *final_norm, *lm_head;
    char *act;                         // arena 0; arena 1 starts arena_bytes later
    size_t arena_bytes;
    ActLayout al;
    float *logits;
    void *kv;
    size_t kv_layer_bytes;
    float *part;
    int32_t *counters;
    const double *inv_freq;
    long long *prof;                   // optional [blocks][2 * (5 n_layers + 2)] clock stamps
    unsigned *sync;                    // SYNC_WORDS words: the launch count
    int32_t n_layers, d_model, n_heads, n_kv_heads, d_ffn, vocab, cap_ctx, max_splits, head;
    int32_t kv_half;                   // the cache holds fp16 (bf16 models only), not fp32
    float eps;
};

// One chunk of the dense prefix pass (bf16 weights): T <= PREFILL_CHUNK prefix tokens at
// positions p0 .. p0 + T - 1.  Arena buffers are DEVICE, sized for PREFILL_CHUNK rows.
constexpr int PREFILL_CHUNK = 1024;
struct PrefillChunk {
    const void *embed;
    const int32_t *prefix;             // DEVICE token ids of the whole prefix
    const spd_layer_weights *layers;   // HOST array [n_layers]
    int32_t n_layers, d_model, n_heads, n_kv_heads, d_ffn, cap_ctx, p0, T, num_cu;
    float eps;
    const double *inv_freq;
    char *kv;
    size_t kv_layer_bytes;
    int32_t kv_half;                   // the cache holds fp16, not fp32
    float *h, *h1;                     // [PREFILL_CHUNK, d_model] residual stream (in / out) and after attention
    float *q;                          // [PREFILL_CHUNK, n_heads * d_head]
    uint16_t *xhi, *xlo;               // [PREFILL_CHUNK, max(d_model, n_heads * d_head)] bf16 pair
    uint16_t *uhi, *ulo;               // [PREFILL_CHUNK, d_ffn] bf16 pair
    float2 *rope;                      // [PREFILL_CHUNK, d_head / 2]
    float *ks_part;                    // [column tiles of the widest product, 2, 2, 16, 64]: partial tiles of the split-k kernel
    int32_t *ks_count;                 // [column tiles of the widest product], zero between launches
};

constexpr int FUSED_MAX_EPI = 512;     // residual values one block of the fused kernel stages per phase
constexpr int FUSED_PROF_BLOCKS = 512;  // blocks of the fused kernel whose phase clocks are kept
constexpr int FUSED_MAX_BLOCKS = 1024;                      // largest grid of the fused kernel
constexpr int SYNC_LAUNCH_WORD = 0;                         // launches of the fused kernel since the last reset (its parity picks the arena)
constexpr int SYNC_WORDS = 64;
constexpr int TOPK_PART_MAX = 128;
constexpr int ATTN_CHUNK = 128;        // cached positions per attention item (one kernel per operator; short contexts)
constexpr int ATTN_CHUNK_MIN = 64;    // the fused kernel picks the chunk per step within these bounds
constexpr int ATTN_CHUNK_MAX = 512;

namespace spdk {
hipError_t gemv(hipStream_t s, int dtype, int epi, const GemvArgs &a, int num_cu);
size_t gemv_lds_bytes(int dtype, int cols);
hipError_t attention(hipStream_t s, int dtype, const AttnArgs &a);
hipError_t superpose(hipStream_t s, int dtype, const SuperposeArgs &a);
hipError_t topk_partial(hipStream_t s, const TopkArgs &a);
hipError_t expand_prune(hipStream_t s, const ExpandArgs &a);
hipError_t nucleus(hipStream_t s, const NucleusArgs &a);
hipError_t prefill_chunk(hipStream_t s, const PrefillChunk &c);
hipError_t prefill_init();
hipError_t advance(hipStream_t s, DevState *st);
hipError_t renorm(hipStream_t s, DevState *st, int k);
hipError_t fill_i32(hipStream_t s, int32_t *p, int32_t v, int n);
// Fused forward: 0 if no instantiation serves this shape, else resident blocks per CU.
int fused_max_blocks_per_cu(int dtype, int kv_half, int d_model, int d_ffn);
hipError_t fused_forward(hipStream_t s, int dtype, const FusedArgsHost &a, int blocks);
hipError_t init();  // raise the dynamic-LDS limit of the kernels that need it
// stand-alone attention: argument check (an spd_status) and the launch on a given scratch buffer
int attention_args_status(int dtype, const float *q, const void *K, const void *V, const float *out, int n_heads,
                          int n_kv_heads, int d_head, int n_ctx, int cap_ctx);
int attention_on_scratch(hipStream_t s, int dtype, const float *q, const void *K, const void *V, float *out,
                         void *scratch, int n_heads, int n_kv_heads, int d_head, int n_ctx, int cap_ctx);
}  // namespace spdk

// ---------------------------------------------------------------- host-side table builder
#include <string>
#include <vector>
struct NgramHostTable {
    std::vector<NgramSlot> slots;
    int32_t max_probe = 0;
    int32_t present[SPD_N_ORDERS] = {0, 0, 0, 0, 0};
};
// Upper bound on the slots ngram_build will use for these entry counts.
uint64_t ngram_capacity_for(const spd_ngram_host_tables *t);
// Returns SPD_OK or SPD_ETABLE / SPD_EINVAL with a reason in `err`.
int ngram_build(const spd_ngram_host_tables *t, int32_t vocab, uint64_t capacity, NgramHostTable &out,
                std::string &err);
