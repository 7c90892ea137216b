// Nucleus (top-p) sampling of one token from the logits of a batch-1 forward pass: the
// comparison decoder of the paper's latency study (Section 4.3), k independent passes of which
// Superposed Decoding is timed against.  Section 2: keep the smallest set of most probable
// tokens whose cumulative probability reaches p, renormalise, sample.
//
// No sort.  With the vocabulary ordered by (probability descending, id ascending) both
// questions -- where does the nucleus end, which token does the draw u select by inverse CDF --
// are "the first entry, in that order, whose cumulative probability reaches (exceeds) x".
// Every entry's probability is a 40-bit fixed-point integer, so that probability masses are
// sums of integers: exact, and the same in whatever order they are added (the histograms below
// are built with atomic adds); its 64-bit sort key, ascending in that order, is that integer,
// inverted, above the token id.
//
//   stage A (one block per slice of the vocabulary, all compute units in parallel): scaled
//     logit z, probability, and a bucket number that is linear in z between the largest and the
//     smallest z (2048 buckets), stored per entry; mass and count per bucket of the slice (LDS
//     atomics), added to the histogram in memory (one atomic per bucket the slice touches; sums
//     of integers: the same in any order); the last block to finish goes on alone;
//   stage B: that histogram (vocabularies beyond 32768 entries: built here from the entries'
//     words instead), prefix sums over the buckets, the bucket
//     in which the cumulative mass crosses x; should it hold more than a list's worth of
//     entries it is cut again by key range (2048 sub-buckets per round: at most a few rounds
//     even where thousands of entries tie); the bucket's entries are then ranked against one
//     another (all pairs) and the first one whose cumulative mass crosses x is the answer.
//   The first-level histogram serves both questions.
#include "spd_device.h"

using namespace spdd;

namespace {

constexpr int SNT = 1024;          // threads per block
constexpr int SNW = SNT / WAVE;
constexpr int NB = 2 * SNT;        // buckets per level: two per thread in the prefix sums
constexpr int LC = 256;            // entries that are ranked pairwise
constexpr int ID_BITS = 23;        // token ids in a key (vocab <= 2^23)
constexpr int ITEMS = 32;          // entries per thread that stage B keeps in registers (vocab <= 32768; else they are re-read)
constexpr float FX_ONE = 1099511627776.0f;   // 2^40: probability 1 in fixed point

// Ascending in (probability descending, id ascending); pf < 2^41.
__device__ __forceinline__ unsigned long long sort_key(unsigned long long pf, int id) {
    return (((1ull << 41) - 1ull - pf) << ID_BITS) | (unsigned long long)(unsigned)id;
}

// A sum over the wave that every lane gets (no LDS, no barrier).
__device__ __forceinline__ float wave_all_sum(float v) { return __int_as_float(__builtin_amdgcn_readlane(__float_as_int(wave_sum_last(v)), WAVE - 1)); }
__device__ __forceinline__ float wave_all_max(float v) { return __int_as_float(__builtin_amdgcn_readlane(__float_as_int(wave_max_last(v)), WAVE - 1)); }

struct Stage {                                  // LDS of stage B
    unsigned long long hm[2][NB + 1];          // [level 1 / deeper levels]: per bucket, entry count above mass (one atomic add per
                                                // entry); then the exclusive prefix sums of both (totals at NB)
    unsigned long long wm[SNW];                 // per-wave totals of the prefix sums
    unsigned long long lk[LC], lp[LC], lcum[LC];   // the list: key, probability, mass of the entries up to and including it
    unsigned lrank[LC];                         // entries of the list before it
    int lid[LC];
    unsigned long long kmin, kmax;
    int found, lastb, n_list, best;
    int r_id;                                   // result of a search: the entry, its cumulative mass, its position in the order
    unsigned long long r_mass, r_key;
    unsigned r_index;
    int is_last;
};

// A histogram word: entry count (20 bits: vocab <= 2^20... the sums of all masses stay below
// 2^41) above the mass.
constexpr int CNT_SHIFT = 44;
constexpr unsigned long long ONE_ENTRY = 1ull << CNT_SHIFT;
__device__ __forceinline__ unsigned long long mass_of(unsigned long long w) { return w & (ONE_ENTRY - 1ull); }
__device__ __forceinline__ unsigned count_of(unsigned long long w) { return (unsigned)(w >> CNT_SHIFT); }

// In place: hm (NB values) -> exclusive prefix sums, totals at index NB.
__device__ __forceinline__ void prefix_sums(Stage &s, int lv) {
    const int t = threadIdx.x, lane = t & (WAVE - 1), w = t / WAVE;
    const unsigned long long a0 = s.hm[lv][2 * t], a1 = s.hm[lv][2 * t + 1];
    unsigned long long m = a0 + a1;
#pragma unroll
    for (int o = 1; o < WAVE; o <<= 1) {        // inclusive scan over the wave
        const unsigned long long um = __shfl_up(m, o, WAVE);
        if (lane >= o) m += um;
    }
    if (lane == WAVE - 1) s.wm[w] = m;
    __syncthreads();
    unsigned long long pm = 0;
    for (int q = 0; q < w; ++q) pm += s.wm[q];
    const unsigned long long em = pm + m - (a0 + a1);
    s.hm[lv][2 * t] = em; s.hm[lv][2 * t + 1] = em + a0;
    if (t == SNT - 1) s.hm[lv][NB] = em + a0 + a1;
    __syncthreads();
}

// The bucket in which the cumulative mass first reaches x (STRICT: exceeds x), or, if the
// total does not get there, the last bucket that holds an entry.  Every thread gets it.
template <bool STRICT>
__device__ __forceinline__ int crossing(Stage &s, int lv, unsigned long long x) {
    const int t = threadIdx.x;
    if (t == 0) { s.found = -1; s.lastb = 0; }
    __syncthreads();
    int last = 0;
#pragma unroll
    for (int q = 0; q < 2; ++q) {
        const int b = 2 * t + q;
        const unsigned long long e = mass_of(s.hm[lv][b]), i = mass_of(s.hm[lv][b + 1]);
        if (STRICT ? (e <= x && i > x) : (e < x && i >= x)) s.found = b;     // one bucket at most
        if (count_of(s.hm[lv][b + 1]) > count_of(s.hm[lv][b])) last = b;
    }
    __syncthreads();
    if (s.found < 0) {   // (the same for every thread) nothing reaches x: one atomic per wave, not one per bucket on one address
        last = (int)wave_all_max((float)last);   // bucket numbers are exact in a float
        if ((t & (WAVE - 1)) == 0) atomicMax(&s.lastb, last);
        __syncthreads();
    }
    const int b = s.found >= 0 ? s.found : s.lastb;
    __syncthreads();
    return b;
}

// Per entry, written by stage A: one word with the first-level bucket above the probability
// (x 2^40).  Written through to memory and read back coherently (the writers sit behind other
// L2 caches; a device-wide fence would write back and invalidate whole caches -- tens of
// microseconds -- where this is 8 bytes per entry).
constexpr int PB_SHIFT = 48;
constexpr unsigned long long P_MASK = (1ull << PB_SHIFT) - 1ull;
constexpr unsigned long long NO_ENTRY = ~0ull;
__device__ __forceinline__ unsigned long long load_pb(const unsigned long long *pb, int i) {
    return __hip_atomic_load(as_global(pb) + i, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
// The entries i = tid, tid + SNT, ... that stage B walks several times.  The first walk reads
// their words, CH at a time (one dependent trip to memory per CH entries: these walks are
// chains of latencies, not bandwidth).  CACHED: it leaves the bucket numbers in registers, two
// per register, and the later walks -- which look for the entries of ONE bucket -- read only
// the words of those; otherwise every walk reads all words again.
constexpr int CH = 16;
template <bool CACHED>
struct Entries {
    const unsigned long long *pb;
    int vocab;
    unsigned bk[CACHED ? ITEMS / 2 : 1];
    // CACHED: entry c of this thread is token 8 (tid + SNT (c / 8)) + c % 8 -- its bucket numbers are
    // four 16-byte pieces of the per-entry bucket array (0xFFFF past the vocabulary)
    static __device__ __forceinline__ int entry(int c) { return CACHED ? 8 * ((int)threadIdx.x + (c / 8) * SNT) + (c % 8) : (int)threadIdx.x + c * SNT; }
    __device__ __forceinline__ void load_buckets(const uint16_t *ids) {
        static_assert(!CACHED || ITEMS == 32, "four pieces of eight bucket numbers");
        const __amdgpu_buffer_rsrc_t rs = __builtin_amdgcn_make_buffer_rsrc(const_cast<uint16_t *>(ids), 0, SNT * ITEMS * 2, 0x00020000);
#pragma unroll
        for (int r = 0; r < (CACHED ? 4 : 0); ++r) {
            const u32x4 v = coherent_load16(rs, 16u * (threadIdx.x + (unsigned)(r * SNT)));
            bk[4 * r] = v.x; bk[4 * r + 1] = v.y; bk[4 * r + 2] = v.z; bk[4 * r + 3] = v.w;
        }
    }
    // f(i, bucket of entry i, its probability) for every entry of this thread
    template <typename F>
    __device__ __forceinline__ void first_walk(F &&f) {
        const int rounds = CACHED ? ITEMS / CH : (vocab + SNT * CH - 1) / (SNT * CH);
#pragma unroll
        for (int r = 0; r < (CACHED ? ITEMS / CH : 1); ++r) {
            for (int rr = CACHED ? r : 0; rr < (CACHED ? r + 1 : rounds); ++rr) {
                unsigned long long w[CH];
#pragma unroll
                for (int c = 0; c < CH; ++c) {
                    const int i = threadIdx.x + (rr * CH + c) * SNT;
                    w[c] = i < vocab ? load_pb(pb, i) : NO_ENTRY;
                }
#pragma unroll
                for (int c = 0; c < CH; ++c) {
                    const int i = threadIdx.x + (rr * CH + c) * SNT;
                    const unsigned b = (unsigned)(w[c] >> PB_SHIFT);      // NO_ENTRY: 0xFFFF, no bucket
                    if (CACHED) {
                        if (c & 1) bk[(r * CH + c) / 2] |= b << 16;
                        else bk[(r * CH + c) / 2] = b;
                    }
                    if (w[c] != NO_ENTRY) f(i, (int)b, w[c] & P_MASK);
                }
            }
        }
    }
    // f(i, its probability) for every entry of this thread in bucket b1
    template <typename F>
    __device__ __forceinline__ void walk_bucket(int b1, F &&f) {
        if (CACHED) {
            static_assert(ITEMS <= 32, "one bit per entry");
            unsigned hits = 0u;
            const unsigned both = (unsigned)b1 | ((unsigned)b1 << 16);
#pragma unroll
            for (int r = 0; r < ITEMS / 2; ++r) {   // two bucket numbers per register
                const unsigned x = bk[r] ^ both;
                hits |= (unsigned)((x & 0xFFFFu) == 0u) << (2 * r);
                hits |= (unsigned)((x >> 16) == 0u) << (2 * r + 1);
            }
            while (hits) {   // (few: a bucket holds some dozens of the block's entries)
                const int c = __ffs(hits) - 1;
                hits &= hits - 1u;
                const int i = entry(c);
                f(i, load_pb(pb, i) & P_MASK);
            }
        } else {
            for (int i0 = threadIdx.x; i0 < vocab; i0 += SNT * CH) {
                unsigned long long w[CH];
#pragma unroll
                for (int c = 0; c < CH; ++c) {
                    const int i = i0 + c * SNT;
                    w[c] = i < vocab ? load_pb(pb, i) : NO_ENTRY;
                }
#pragma unroll
                for (int c = 0; c < CH; ++c)
                    if ((int)(w[c] >> PB_SHIFT) == b1) f(i0 + c * SNT, w[c] & P_MASK);
            }
        }
    }
};

// The first entry in the order whose cumulative mass reaches (STRICT: exceeds) x; the last
// entry if none does.  Level-1 prefix sums are in s.hm[0].  Result in s.r_*.
template <bool STRICT, bool CACHED>
__device__ __forceinline__ void search(Stage &s, Entries<CACHED> &en, unsigned long long x) {
    const int t = threadIdx.x;
    const int b1 = crossing<STRICT>(s, 0, x);
    unsigned long long base_m = mass_of(s.hm[0][b1]);
    unsigned base_c = count_of(s.hm[0][b1]);
    unsigned n = count_of(s.hm[0][b1 + 1]) - base_c;
    // the candidates: level-1 bucket b1, and within it the key range [klo, khi] once it has been cut
    unsigned long long klo = 0ull, khi = ~0ull;
    bool cut = false;
    while (n > (unsigned)LC) {
        if (!cut) {   // the key range of the bucket's entries
            if (t == 0) { s.kmin = ~0ull; s.kmax = 0ull; }
            __syncthreads();
            en.walk_bucket(b1, [&](int i, unsigned long long pf) {
                const unsigned long long k = sort_key(pf, i);
                atomicMin(&s.kmin, k);
                atomicMax(&s.kmax, k);
            });
            __syncthreads();
            klo = s.kmin; khi = s.kmax;
            cut = true;
        }
        const unsigned long long width = khi - klo;                 // > 0: more than one entry, keys are distinct
        const int bits = 64 - __clzll((long long)width);
        const int sh = bits > 11 ? bits - 11 : 0;                  // (k - klo) >> sh < 2048
        s.hm[1][2 * t] = 0ull; s.hm[1][2 * t + 1] = 0ull;
        __syncthreads();
        en.walk_bucket(b1, [&](int i, unsigned long long pf) {
            const unsigned long long k = sort_key(pf, i);
            if (k >= klo && k <= khi) {
                const int b2 = (int)((k - klo) >> sh);
                atomicAdd(&s.hm[1][b2], pf + ONE_ENTRY);
            }
        });
        __syncthreads();
        prefix_sums(s, 1);
        const int b2 = crossing<STRICT>(s, 1, x - base_m);          // (x >= base_m: the crossing lies in this range or beyond everything)
        base_m += mass_of(s.hm[1][b2]);
        base_c += count_of(s.hm[1][b2]);
        n = count_of(s.hm[1][b2 + 1]) - count_of(s.hm[1][b2]);
        const unsigned long long lo2 = klo + ((unsigned long long)b2 << sh);
        const unsigned long long hi2 = lo2 + ((1ull << sh) - 1ull);
        klo = lo2;
        khi = hi2 < khi ? hi2 : khi;
        __syncthreads();
    }
    // the candidates into the list (in any order: they are ranked below)
    if (t == 0) { s.n_list = 0; s.best = INT_MAX; }
    if (t < LC) { s.lrank[t] = 0u; s.lcum[t] = 0ull; }
    __syncthreads();
    en.walk_bucket(b1, [&](int i, unsigned long long pf) {
        const unsigned long long k = sort_key(pf, i);
        if (k >= klo && k <= khi) {
            const int at = atomicAdd(&s.n_list, 1);
            s.lk[at] = k; s.lp[at] = pf; s.lid[at] = i;
        }
    });
    __syncthreads();
    const int nl = s.n_list;   // == n
    {   // all pairs: entry i against one part of the list each; the shorter the list, the more parts
        const int slots = nl <= 32 ? 32 : nl <= 64 ? 64 : nl <= 128 ? 128 : LC;
        const int i = t % slots, part = t / slots;
        const int PARTS = SNT / slots;
        if (i < nl) {
            const unsigned long long ki = s.lk[i];
            unsigned cnt = 0u;
            unsigned long long mass = 0ull;
            for (int j = part; j < nl; j += PARTS) {
                const unsigned long long kj = s.lk[j];
                if (kj < ki) ++cnt;
                if (kj <= ki) mass += s.lp[j];
            }
            atomicAdd(&s.lrank[i], cnt);
            atomicAdd(&s.lcum[i], mass);
        }
    }
    __syncthreads();
    if (t < nl) {
        const unsigned long long tot = base_m + s.lcum[t];
        if (STRICT ? tot > x : tot >= x) atomicMin(&s.best, (int)s.lrank[t]);
    }
    __syncthreads();
    const int pick = s.best == INT_MAX ? nl - 1 : s.best;   // nothing reaches x: the last entry
    if (t < nl && (int)s.lrank[t] == pick) {
        s.r_id = s.lid[t]; s.r_key = s.lk[t];
        s.r_mass = base_m + s.lcum[t];
        s.r_index = base_c + (unsigned)pick;
    }
    __syncthreads();
}

template <bool CACHED>
__global__ __launch_bounds__(SNT) void nucleus_kernel(const NucleusArgs a) {
    __shared__ Stage s;
    const int tid = threadIdx.x, lane = tid & (WAVE - 1);
    global_ptr<DevState> st = as_global(a.st);
    // log-sum-exp, largest and smallest scaled logit from the per-slice statistics (every wave for itself)
    float M = -INFINITY, mn = INFINITY;
    for (int b = lane; b < a.n_part; b += WAVE) { M = fmaxf(M, as_global(a.pm)[b]); mn = fminf(mn, as_global(a.pn)[b]); }
    M = wave_all_max(M);
    mn = -wave_all_max(-mn);
    float S = 0.f;
    for (int b = lane; b < a.n_part; b += WAVE) S += as_global(a.ps)[b] * expf(as_global(a.pm)[b] - M);
    const float lse = M + logf(wave_all_sum(S));
    const float range = M - mn;
    const float scale = range > 0.f ? (float)NB / range : 0.f;

    // ---- stage A: this block's slice
    const int lo = blockIdx.x * a.per_part, hi = min(a.vocab, lo + a.per_part);
    if (CACHED) {   // the slice's histogram
        s.hm[1][2 * tid] = 0ull; s.hm[1][2 * tid + 1] = 0ull;
        __syncthreads();
    }
    for (int i = lo + tid; i < hi; i += SNT) {
        const float z = __fdiv_rn(as_global(a.logits)[i], a.tau);
        const float p = expf(z - lse);
        const float fb = (M - z) * scale;                          // monotonic in z; anything beyond lands in the last bucket
        const int b = fb < (float)(NB - 1) ? (int)fb : NB - 1;
        const unsigned long long pf = (unsigned long long)(p * FX_ONE);   // <= 2^40 (1 + a few ulp)
        const int bb = b < 0 ? 0 : b;
        __hip_atomic_store(as_global(a.sc_pb) + i, ((unsigned long long)bb << PB_SHIFT) | pf, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        if (CACHED) {
            __hip_atomic_store(as_global(a.sc_bk) + i, (uint16_t)bb, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            atomicAdd(&s.hm[1][bb], pf + ONE_ENTRY);
        }
    }
    if (CACHED) {
        __syncthreads();
#pragma unroll
        for (int q = 0; q < 2; ++q) {
            const unsigned long long w = s.hm[1][2 * tid + q];
            if (w) (void)__hip_atomic_fetch_add(as_global(a.sc_hist) + 2 * tid + q, w, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
    }
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");   // this wave's write-through stores have been acknowledged
    __syncthreads();
    if (tid == 0) s.is_last = (__hip_atomic_fetch_add(as_global(a.sc_count), 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) == (unsigned)(gridDim.x - 1));
    __syncthreads();
    if (!s.is_last) return;

    // ---- stage B: first-level histogram
    Entries<CACHED> en;
    en.pb = a.sc_pb; en.vocab = a.vocab;
    if constexpr (CACHED) {
        // the histogram all blocks have added to (left at zero for the next call), and this thread's bucket numbers
        {   // one 16-byte piece: this thread's two words
            const __amdgpu_buffer_rsrc_t hrs = __builtin_amdgcn_make_buffer_rsrc(a.sc_hist, 0, NB * 8, 0x00020000);
            const u32x4 v = coherent_load16(hrs, 16u * (unsigned)tid);
            en.load_buckets(a.sc_bk);
            s.hm[0][2 * tid] = ((unsigned long long)v.y << 32) | v.x;
            s.hm[0][2 * tid + 1] = ((unsigned long long)v.w << 32) | v.z;
        }
    } else {
        s.hm[0][2 * tid] = 0ull; s.hm[0][2 * tid + 1] = 0ull;
        __syncthreads();
        en.first_walk([&](int, int b, unsigned long long pf) {
            atomicAdd(&s.hm[0][b], pf + ONE_ENTRY);
        });
    }
    __syncthreads();
    prefix_sums(s, 0);

    // 1. the nucleus: the first entry whose cumulative probability reaches top_p, and all before it
    const unsigned long long x_p = (unsigned long long)((double)a.top_p * (double)FX_ONE);
    search<false, CACHED>(s, en, x_p);
    const unsigned long long mass_fx = s.r_mass, key_T = s.r_key;
    const unsigned size = s.r_index + 1u;
    const int id_T = s.r_id;
    __syncthreads();
    // 2. the draw: the first entry whose cumulative probability exceeds u * mass (within the nucleus)
    const unsigned long long x_u = (unsigned long long)((double)st->sample_u * (double)mass_fx);
    search<true, CACHED>(s, en, x_u);
    int tok = s.r_id;
    if (s.r_key > key_T) tok = id_T;   // (only rounding could take it past the nucleus)

    if (CACHED) {
        __hip_atomic_store(as_global(a.sc_hist) + 2 * tid, 0ull, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        __hip_atomic_store(as_global(a.sc_hist) + 2 * tid + 1, 0ull, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
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
        st->nucleus_size = (int)size;
        st->nucleus_mass = (float)((double)mass_fx / (double)FX_ONE);
        st->k = 1;
        st->n_gen = gen + 1;
        if (a.advance) st->pos += 1;
        __hip_atomic_store(as_global(a.sc_count), 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);   // for the next call
    }
}

}  // namespace

namespace spdk {

hipError_t nucleus(hipStream_t s, const NucleusArgs &a) {
    if (a.vocab <= SNT * ITEMS) hipLaunchKernelGGL(nucleus_kernel<true>, dim3(a.n_part), dim3(SNT), 0, s, a);
    else hipLaunchKernelGGL(nucleus_kernel<false>, dim3(a.n_part), dim3(SNT), 0, s, a);
    return hipGetLastError();
}

}  // namespace spdk
