// Nucleus (top-p) sampling of one token from the logits of a batch-1 forward pass: the
// comparison decoder of the paper's latency study (Section 4.3), k independent passes of which
// Superposed Decoding is timed against.  Section 2: keep the smallest set of most probable
// tokens whose cumulative probability reaches p, renormalise, sample.
//
// No sort: with the vocabulary ordered by probability (descending, lower id first among
// equals) both questions -- where does the nucleus end, which token does the draw u select by
// inverse CDF -- are "find the largest threshold t such that the probability mass of
// {tokens >= t} still reaches (exceeds) x", answered by bisection over the 32 bits of an
// order-preserving integer image of the scaled logit.  One block; every thread keeps its
// share of the vocabulary in registers; masses are summed in a fixed order.
#include "spd_device.h"

using namespace spdd;

namespace {

constexpr int SNT = 1024;     // threads
constexpr int ITEMS = 32;     // vocabulary entries per thread held in registers (vocab <= 32768)

// Order-preserving map float -> uint32 (larger float, larger key).
__device__ __forceinline__ uint32_t order_key(float z) {
    const uint32_t b = __float_as_uint(z);
    return (b & 0x80000000u) ? ~b : (b | 0x80000000u);
}

struct Share {                 // one thread's entries i = tid + j * SNT
    uint32_t key[ITEMS];
    float p[ITEMS];
};

// Mass of the entries whose key is >= t.  CACHED: from the registers; else recomputed.
template <bool CACHED>
__device__ __forceinline__ float mass_ge(const NucleusArgs &a, const Share &sh, float lse, uint32_t t, float *red) {
    float m = 0.f;
    if (CACHED) {
#pragma unroll
        for (int j = 0; j < ITEMS; ++j) m += sh.key[j] >= t ? sh.p[j] : 0.f;
    } else {
        for (int i = threadIdx.x; i < a.vocab; i += SNT) {
            const float z = __fdiv_rn(as_global(a.logits)[i], a.tau);
            if (order_key(z) >= t) m += expf(z - lse);
        }
    }
    return block_sum<SNT>(m, red);
}

// Largest t with mass(>= t) >= x (STRICT: > x).  mass(>= 0) is the whole vocabulary.
template <bool CACHED, bool STRICT>
__device__ __forceinline__ uint32_t threshold(const NucleusArgs &a, const Share &sh, float lse, float x, float *red) {
    uint32_t t = 0u;
    for (int bit = 31; bit >= 0; --bit) {
        const uint32_t cand = t | (1u << bit);
        const float m = mass_ge<CACHED>(a, sh, lse, cand, red);
        if (STRICT ? m > x : m >= x) t = cand;
    }
    return t;
}

// Number of entries with key == t, their (common) probability, and the smallest id > after among them.
template <bool CACHED>
__device__ __forceinline__ void ties(const NucleusArgs &a, const Share &sh, float lse, uint32_t t, int after,
                                     int &count, float &p_each, int &next_id, float *red, int *ired) {
    int c = 0, best = INT_MAX;
    float pe = 0.f;
    if (CACHED) {
#pragma unroll
        for (int j = 0; j < ITEMS; ++j) {
            const int i = threadIdx.x + j * SNT;
            if (i < a.vocab && sh.key[j] == t) { ++c; pe = sh.p[j]; if (i > after) best = min(best, i); }
        }
    } else {
        for (int i = threadIdx.x; i < a.vocab; i += SNT) {
            const float z = __fdiv_rn(as_global(a.logits)[i], a.tau);
            if (order_key(z) == t) { ++c; pe = expf(z - lse); if (i > after) best = min(best, i); }
        }
    }
    count = (int)(block_sum<SNT>((float)c, red) + 0.5f);
    p_each = block_max<SNT>(pe, red);
    // block-wide minimum of `best`
    const int lane = threadIdx.x & (WAVE - 1), w = threadIdx.x / WAVE;
#pragma unroll
    for (int o = WAVE / 2; o > 0; o >>= 1) best = min(best, __shfl_xor(best, o, WAVE));
    __syncthreads();
    if (lane == 0) ired[w] = best;
    __syncthreads();
    int r = ired[0];
    for (int q = 1; q < SNT / WAVE; ++q) r = min(r, ired[q]);
    next_id = r;
}

template <bool CACHED>
__global__ __launch_bounds__(SNT) void nucleus_kernel(const NucleusArgs a) {
    __shared__ float red[SNT / WAVE];
    __shared__ int ired[SNT / WAVE];
    __shared__ float s_lse;
    const int tid = threadIdx.x;
    global_ptr<DevState> st = as_global(a.st);
    if (tid == 0) {   // log-sum-exp of the scaled logits from the per-slice statistics
        float M = -INFINITY;
        for (int b = 0; b < a.n_part; ++b) M = fmaxf(M, as_global(a.pm)[b]);
        float S = 0.f;
        for (int b = 0; b < a.n_part; ++b) S += as_global(a.ps)[b] * expf(as_global(a.pm)[b] - M);
        s_lse = M + logf(S);
    }
    __syncthreads();
    const float lse = s_lse;
    Share sh;
    if (CACHED) {
#pragma unroll
        for (int j = 0; j < ITEMS; ++j) {
            const int i = tid + j * SNT;
            sh.key[j] = 0u; sh.p[j] = 0.f;
            if (i < a.vocab) {
                const float z = __fdiv_rn(as_global(a.logits)[i], a.tau);
                sh.key[j] = order_key(z);
                sh.p[j] = expf(z - lse);
            }
        }
    }
    // 1. the nucleus: keys > T entirely, of the keys == T the `need` lowest ids
    const uint32_t T = threshold<CACHED, false>(a, sh, lse, a.top_p, red);
    const float above_T = T == 0xFFFFFFFFu ? 0.f : mass_ge<CACHED>(a, sh, lse, T + 1u, red);
    int n_T, dummy;
    float p_T;
    ties<CACHED>(a, sh, lse, T, -1, n_T, p_T, dummy, red, ired);
    int need = 1;
    while (need < n_T && above_T + (float)need * p_T < a.top_p) ++need;
    const float mass = above_T + (float)need * p_T;
    // 2. the draw: first token, in that order, whose cumulative probability exceeds u * mass
    const float target = st->sample_u * mass;
    uint32_t S = threshold<CACHED, true>(a, sh, lse, target, red);
    if (S < T) S = T;                                   // (only rounding could take it below)
    const float above_S = S == 0xFFFFFFFFu ? 0.f : mass_ge<CACHED>(a, sh, lse, S + 1u, red);
    int n_S, tok;
    float p_S;
    ties<CACHED>(a, sh, lse, S, -1, n_S, p_S, tok, red, ired);
    int skip = p_S > 0.f ? (int)floorf(fmaxf(target - above_S, 0.f) / p_S) : 0;
    skip = min(skip, (S == T ? need : n_S) - 1);
    for (int r = 0; r < skip; ++r) ties<CACHED>(a, sh, lse, S, tok, n_S, p_S, tok, red, ired);
    // nucleus size = entries with key > T plus `need`
    float cnt = 0.f;
    if (CACHED) {
#pragma unroll
        for (int j = 0; j < ITEMS; ++j) cnt += (tid + j * SNT < a.vocab && sh.key[j] > T) ? 1.f : 0.f;
    } else {
        for (int i = tid; i < a.vocab; i += SNT) cnt += order_key(__fdiv_rn(as_global(a.logits)[i], a.tau)) > T ? 1.f : 0.f;
    }
    const int size = (int)(block_sum<SNT>(cnt, red) + 0.5f) + need;

    if (tid == 0) {   // the pass's state: one draft (k = 1, gamma = 1)
        const float logp = __fdiv_rn(as_global(a.logits)[tok], a.tau) - lse;
        int tail[SPD_TAIL];
        for (int q = 0; q < SPD_TAIL; ++q) tail[q] = a.first ? st->prefix_tail[q] : st->tails[0][q];
        for (int q = 0; q < SPD_TAIL - 1; ++q) st->tails[0][q] = tail[q + 1];
        st->tails[0][SPD_TAIL - 1] = tok;
        st->logscore[0] = a.first ? logp : st->logscore[0] + logp;
        st->gamma[0] = 1.f;
        st->new_tok[0] = tok;
        st->new_parent[0] = a.first ? -1 : 0;
        st->top_ids[0] = tok;
        st->top_logp[0] = logp;
        const int gen = a.first ? 0 : st->n_gen;
        if (gen < a.max_gen) { as_global(a.hist_tok)[(size_t)gen * SPD_K_MAX] = tok; as_global(a.hist_par)[(size_t)gen * SPD_K_MAX] = a.first ? -1 : 0; }
        st->nucleus_size = size;
        st->nucleus_mass = mass;
        st->k = 1;
        st->n_gen = gen + 1;
        if (a.advance) st->pos += 1;
    }
}

}  // namespace

namespace spdk {

hipError_t nucleus(hipStream_t s, const NucleusArgs &a) {
    if (a.vocab <= SNT * ITEMS) hipLaunchKernelGGL(nucleus_kernel<true>, dim3(1), dim3(SNT), 0, s, a);
    else hipLaunchKernelGGL(nucleus_kernel<false>, dim3(1), dim3(SNT), 0, s, a);
    return hipGetLastError();
}

}  // namespace spdk
