// The whole transformer forward of one SPD timestep as ONE persistent kernel.
//
// Batch-1 decode is a chain of ~160 small matrix-vector products (7B shape: 33-180 MB each,
// 6-30 us at HBM speed), every one of which needs the complete output of its predecessor.
// Launching them one by one leaves HBM idle at every boundary, so here a grid that exactly
// fills the chip walks through all phases itself and meets at a device-wide barrier between
// phases.  The weights a block needs for its first tile of the NEXT phase do not depend on
// any activation, so they are requested before the barrier and are in flight while the block
// waits: the weight stream from HBM does not stop at phase boundaries.
//
// Phase GEMV ("row-contiguous"): the NW waves of a block read one matrix row side by side
// (wave w takes columns [(p*NW + w)*64*VEC, +64*VEC) of pass p), so the slice of x a lane
// multiplies with is fixed and lives in registers; a tile is U rows, partial sums meet in LDS.
#include "spd_device.h"

using namespace spdd;

namespace {

// One block per CU (few barrier participants).  With 512 threads: 8 waves that read one matrix
// row side by side and have 256 vector registers each, i.e. room for a 16 KB weight tile in
// flight per wave.  (1024 threads = two such row groups with half the registers.)
constexpr int FUSED_UA = 16;          // rows per tile where one pass covers a row
constexpr int FUSED_UO_EXTRA = 4;     // extra rows per tile of the O projection
constexpr int FUSED_QD = 12;          // 16-byte pieces per lane of the next tile requested while the block synchronises
constexpr int FUSED_SLICE = 3;        // of which this many go out per synchronisation step of wave 0
constexpr int FUSED_SLICE_WIDE = 4;   // the same for models whose d_model takes two block passes (measured: 3 costs the
                                      //   13B shape 0.3 % and the 70B shape 1 %, and gains the 7B shape 0.1...0.6 %)
constexpr int FUSED_ONE_CHUNK = 256;  // contexts up to this long are one attention item per head (no merge across blocks)
static_assert(FUSED_ONE_CHUNK <= ATTN_CHUNK_MAX, "one attention item must fit the score buffer");
constexpr int BAR_SLEEP_7B = 36;      // s_sleep units (64 cycles) between two polls of the barrier
constexpr int BAR_SLEEP_WIDE = 48;    // the same where d_ffn takes more than four block passes (the 70B shape: long
                                      //   phases, and 36 costs it 0.3 %; the 7B and 13B shapes gain 0.4 and 0.2 %)
constexpr int QKV_SLEEP = 1;          // the same between two polls of a head's arrival counter
constexpr int NT = 512;               // threads per block
constexpr int NW = 8;                 // waves side by side on one row
constexpr int MAX_U = 32;
constexpr int NG = NT / WAVE / NW;   // row groups per block
constexpr unsigned SPIN_LIMIT = 1u << 22;

constexpr int MAX_EPI = FUSED_MAX_EPI;   // residual values a block may need in one phase

struct FusedShared {
    float part[2][NG][MAX_U][NW]; // [buffer][row group][tile slot][wave]
    float epi[MAX_EPI];           // this block's slice of the residual, staged when the phase starts
    float2 rope[128];             // (cos, sin) of this step's position, all d_head / 2 <= 128 pairs
    float red[NT / WAVE];
    float sc[ATTN_CHUNK_MAX];
    int s_last;
    unsigned tick;                // bumped by thread 0 whenever it has issued a synchronisation step
    unsigned released;            // number of synchronisation points this block has been released from
};

// (volatile accesses must name the LDS address space, or they become generic-address
// instructions, which hold up the weight stream: see spd_device.h)
typedef volatile unsigned __attribute__((address_space(3))) *lds_flag_ptr;
__device__ __forceinline__ lds_flag_ptr lds_flag(unsigned *p) { return (lds_flag_ptr)p; }

// Thread 0 tells the other waves that one more of its memory operations is on its way.
__device__ __forceinline__ void tick_bump(FusedShared &sh) {
    asm volatile("" ::: "memory");
    lds_flag_ptr t = lds_flag(&sh.tick);
    *t = *t + 1;
    asm volatile("" ::: "memory");
}

// Device-wide barrier, two levels: blocks arrive on their group's counter (BAR_GROUP
// consecutive blocks per group, counters 256 bytes apart), the last arriver of a group bumps
// the top counter, everyone polls the top counter.  Same-address atomics serialise at the
// memory side (~14 ns each): a flat counter pays for 256 of them, a top counter fed by many
// small groups for the groups' bumps landing on the line everybody polls.  Measured per step
// at the 7B shape (256 blocks): groups of 8 / 16 / 32 / 64 / 96 / 128 / 256 blocks = +170 / +80 /
// +32 / +8 / 0 / +13 / +60 us with one top counter; with two copies of the top counter away
// from the group counters, two groups of 128 are 3 us per step ahead of 96 / 96 / 64 (one
// bump per copy fewer on the polled lines).  (One counter per group polled side by side by every block,
// without the top level, measured slower: the polls of 256 blocks on each of 8 addresses take
// longer than the extra hop.)  All counters increase monotonically and run on from launch to
// launch (the kernel continues from the count its predecessor left behind); the host zeroes
// them when a prefix pass begins.  Bounded: if the grid is not co-resident the wait gives up,
// raises *err, and every later wait returns at once, so the kernel always drains.
//
// Everything other blocks will read was stored with write-through (device-scope) stores and
// every storing wave has waited for its own stores (wait_stores) before getting here.
// ALL_WAVES_STORED: waves other than wave 0 stored too, so the block meets before it arrives.
// Wave 0 should have no weight loads outstanding when it gets here: memory operations of a
// wave return in order, so the arrival count and every poll would queue behind them.
//
// While thread 0 works through the barrier the other waves request the next phase's first
// tile a slice at a time, one slice behind each memory operation thread 0 issues (tick_bump):
// a compute unit serves its memory operations in order, so an arrival or a poll issued behind
// a whole tile of weight requests would wait for all of them, while a slice issued behind the
// poll delays nothing and keeps the weight stream going through the barrier.
template <bool ALL_WAVES_STORED, int SLEEP>
__device__ __forceinline__ void grid_barrier(unsigned *ctr, unsigned epoch, int *err, FusedShared &sh, unsigned seq) {
    if (ALL_WAVES_STORED) __syncthreads();
    if (threadIdx.x == 0) {
        const unsigned g = blockIdx.x / BAR_GROUP;
        const unsigned n_groups = (gridDim.x + BAR_GROUP - 1) / BAR_GROUP;
        const unsigned my_size = min((unsigned)BAR_GROUP, gridDim.x - g * BAR_GROUP);
        // The top counter exists BAR_TOPS times, kilobytes away from the group counters (the last
        // lines of the range reserved for groups): the last arriver of a group bumps every copy, a
        // block polls only its own.  Half the pollers per line, and no poll lands next to a line that
        // a group's arrivals are being added to: 1.1 % of a step against one top counter in the first line.
        unsigned *grp = ctr + 64 * (1 + g);
        unsigned *tops = ctr + 64 * (1 + BAR_MAX_GROUPS - BAR_TOPS), *top = tops + 64 * (blockIdx.x % BAR_TOPS);
        const unsigned old = __hip_atomic_fetch_add(as_global(grp), 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        tick_bump(sh);
        if (old + 1 == epoch * my_size) {
#pragma unroll
            for (int r = 0; r < BAR_TOPS; ++r)
                __hip_atomic_fetch_add(as_global(tops) + 64 * r, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
        unsigned spins = 0;
        while (true) {
            const unsigned seen = __hip_atomic_load(as_global(top), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            tick_bump(sh);
            if (seen >= epoch * n_groups) break;
            __builtin_amdgcn_s_sleep(SLEEP);
            ++spins;
            if ((spins & 255u) == 0 && __hip_atomic_load(as_global(err), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT)) break;
            if (spins > SPIN_LIMIT) {
                __hip_atomic_store(as_global(err), 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                break;
            }
        }
        *lds_flag(&sh.released) = seq;
    }
    __syncthreads();
}

// Values that are the same in every lane but were loaded from global memory would occupy
// vector registers; these move them to scalar registers.
__device__ __forceinline__ int uniform(int v) { return __builtin_amdgcn_readfirstlane(v); }
template <typename T> __device__ __forceinline__ T *uniform(T *p) {
    const uint64_t u = (uint64_t)p;
    const uint32_t lo = __builtin_amdgcn_readfirstlane((uint32_t)u), hi = __builtin_amdgcn_readfirstlane((uint32_t)(u >> 32));
    return (T *)(((uint64_t)hi << 32) | lo);
}
__device__ __forceinline__ spd_layer_weights uniform(const spd_layer_weights &w) {
    spd_layer_weights r;
    r.attn_norm = uniform(w.attn_norm); r.wqkv = uniform(w.wqkv); r.wo = uniform(w.wo);
    r.ffn_norm = uniform(w.ffn_norm); r.w_gate = uniform(w.w_gate); r.w_up = uniform(w.w_up);
    r.w_down = uniform(w.w_down);
    return r;
}

__device__ __forceinline__ GemvArgs uniform(const GemvArgs &a) {
    GemvArgs r = a;
    r.W = uniform(a.W); r.W2 = uniform(a.W2); r.gain = uniform(a.gain); r.x = uniform(a.x);
    r.resid = uniform(a.resid); r.y = uniform(a.y); r.rows = uniform(a.rows); r.cols = uniform(a.cols);
    r.kcache = uniform(a.kcache); r.vcache = uniform(a.vcache);
    r.n_q_rows = uniform(a.n_q_rows); r.n_kv_rows = uniform(a.n_kv_rows); r.d_head = uniform(a.d_head);
    r.cap_ctx = uniform(a.cap_ctx); r.first_block = uniform(a.first_block);
    return r;
}

__device__ __forceinline__ bool is_wave0() { return __builtin_amdgcn_readfirstlane((int)threadIdx.x) < WAVE; }

// Wait until this wave's stores have been acknowledged.  Called before the next phase's
// weights are requested, so it never waits for those.
__device__ __forceinline__ void wait_stores() { asm volatile("s_waitcnt vmcnt(0)" ::: "memory"); }

// Units [lo, hi) of n that block b of G owns (contiguous, balanced to within one unit); the
// first `skip` blocks own nothing.
__device__ __forceinline__ void block_range(int n, int b, int G, int &lo, int &hi, int skip = 0) {
    if (b < skip) { lo = hi = 0; return; }
    b -= skip; G -= skip;
    // n * (b + 1) stays below 2^32 for every supported shape (n <= 2^21 units, G <= 2^10 blocks)
    // (integer division runs on the vector unit: bring the uniform results back to scalars)
    lo = __builtin_amdgcn_readfirstlane((int)(((unsigned)n * (unsigned)b) / (unsigned)G));
    hi = __builtin_amdgcn_readfirstlane((int)(((unsigned)n * (unsigned)(b + 1)) / (unsigned)G));
}

// A phase keeps ONE tile of U rows x P passes (NS = U * P 16-byte pieces per lane) in
// registers.  The moment a piece has been multiplied in, its register is re-used for the same
// piece of the block's next tile, so a wave always has about NS loads in flight; after the
// last tile the first tile of the NEXT phase is requested, before the device-wide barrier.
// Loads are never predicated: a row past the block's range re-reads the last valid row (a
// cache hit), and a column past the row end lies outside the buffer descriptor, which
// describes one row (zeros come back, nothing is fetched); the inner loop has no branches.
template <typename WT, int P, int U, int EPI, int NBUF, int SL>
struct Gemv {
    static constexpr int VEC = Store<WT>::VEC;
    static constexpr int UT = U / 2;   // units per tile
    static constexpr int NS = U * P;
    static_assert(U % 2 == 0 && NS <= NBUF && U <= MAX_U, "tile does not fit the register window");
    static_assert(NG * UT <= WAVE, "the epilogue threads must all sit in wave 0");

    static __device__ __forceinline__ int n_units(const GemvArgs &a) { return EPI == EPI_SWIGLU ? a.rows : a.rows / 2; }

    // Byte offset of this lane's piece of pass p within a row.
    static __device__ __forceinline__ uint32_t col_offset(const GemvArgs &a, int p) {
        const int lane = threadIdx.x & (WAVE - 1), w = (threadIdx.x / WAVE) % NW;
        const int c = ((p * NW + w) * WAVE + lane) * VEC;
        return (uint32_t)c * (uint32_t)sizeof(WT);   // past the row end: the load returns zero
    }

    // Piece q = s * P + p of this wave's row group within the block tile starting at unit u0
    // (a block tile is NG * UT units) of a block whose range ends at u_end.
    static __device__ __forceinline__ u32x4 piece(const GemvArgs &a, int u0, int u_end, int q, const uint32_t (&coff)[P]) {
        const int s = q / P, p = q % P;
        const int g = __builtin_amdgcn_readfirstlane(threadIdx.x / (WAVE * NW));
        const int unit = min(u0 + g * UT + (EPI == EPI_SWIGLU ? (s % UT) : (s / 2)), u_end - 1);
        const uint32_t row_bytes = (uint32_t)a.cols * (uint32_t)sizeof(WT);
        const char *W = (const char *)(EPI == EPI_SWIGLU && s >= UT ? a.W2 : a.W);
        const int row = EPI == EPI_SWIGLU ? unit : 2 * unit + (s & 1);
        return stream_load16(row_resource(W + (size_t)row * row_bytes, row_bytes), coff[p]);
    }

    // The head of this block's first tile, pieces [0, QD), is requested before the phase
    // starts; the rest follows the load of x.
    static constexpr int QD = NS < FUSED_QD ? NS : FUSED_QD;
    static __device__ __forceinline__ void prefetch(const GemvArgs &a_in, u32x4 (&buf)[NBUF]) {
        const GemvArgs a = uniform(a_in);
        int lo, hi;
        block_range(n_units(a), blockIdx.x, gridDim.x, lo, hi, a.first_block);
        if (lo >= hi) return;
        uint32_t coff[P];
#pragma unroll
        for (int p = 0; p < P; ++p) coff[p] = col_offset(a, p);
#pragma unroll
        for (int q = 0; q < QD; ++q) buf[q] = piece(a, lo, hi, q, coff);
    }
    // The same while thread 0 runs barrier number `epoch`: SL pieces behind each
    // of its synchronisation steps, everything that is left once the block has been released.
    static __device__ __forceinline__ void prefetch_sliced(const GemvArgs &a_in, u32x4 (&buf)[NBUF], FusedShared &sh,
                                                           unsigned epoch) {
        const GemvArgs a = uniform(a_in);
        int lo, hi;
        block_range(n_units(a), blockIdx.x, gridDim.x, lo, hi, a.first_block);
        if (lo >= hi) return;
        uint32_t coff[P];
#pragma unroll
        for (int p = 0; p < P; ++p) coff[p] = col_offset(a, p);
        lds_flag_ptr tick = lds_flag(&sh.tick), released = lds_flag(&sh.released);
        unsigned seen = uniform((int)*tick);
#pragma unroll
        for (int q = 0; q < QD; ++q) {
            if (q % SL == 0) {
                unsigned now = seen;
                for (unsigned spins = 0; spins < SPIN_LIMIT; ++spins) {   // thread 0's own wait is bounded too
                    now = uniform((int)*tick);
                    if (now != seen || (unsigned)uniform((int)*released) >= epoch) break;
                    __builtin_amdgcn_s_sleep(1);
                }
                seen = now;
            }
            buf[q] = piece(a, lo, hi, q, coff);
        }
    }

    // One tile: U rows of this wave's row group against x, partial sums to LDS, the block
    // meets, the first NG * UT threads finish their units.  REFILL: every consumed register is
    // re-requested at once with the same piece of the block's next tile.
    template <bool REFILL>
    static __device__ __forceinline__ void tile(const GemvArgs &a, int u0, int lo, int hi, int pos,
                                                FusedShared &sh, u32x4 (&buf)[NBUF], const float (&xr)[P][VEC],
                                                const uint32_t (&coff)[P], int pb) {
        const int tid = threadIdx.x, lane = tid & (WAVE - 1), w = (tid / WAVE) % NW, g = tid / (WAVE * NW);
        const int eu = min(u0 + tid, hi - 1);
#pragma unroll
        for (int s = 0; s < U; ++s) {
            float acc = 0.f;
#pragma unroll
            for (int p = 0; p < P; ++p) {
                float f[VEC];
                Store<WT>::unpack(buf[s * P + p], f);
#pragma unroll
                for (int v = 0; v < VEC; ++v) acc = fmaf(f[v], xr[p][v], acc);
                if (REFILL) buf[s * P + p] = piece(a, u0 + NG * UT, hi, s * P + p, coff);
            }
            acc = wave_sum_last(acc);
            if (lane == WAVE - 1) sh.part[pb][g][s][w] = acc;
        }
        __syncthreads();
        if (tid < NG * UT && u0 + tid < hi) {   // unit u0 + tid: row group tid / UT, pair tid % UT
            const int eg = tid / UT, t = tid % UT;
            const int s0 = EPI == EPI_SWIGLU ? t : 2 * t;
            const int s1 = EPI == EPI_SWIGLU ? t + UT : 2 * t + 1;
            float r0 = 0.f, r1 = 0.f;
#pragma unroll
            for (int q = 0; q < NW; ++q) { r0 += sh.part[pb][eg][s0][q]; r1 += sh.part[pb][eg][s1][q]; }
            // what the epilogue needs beyond the sums sits in LDS: the tile loop holds no load
            // from global memory but the weights'
            if (EPI == EPI_RESID) {
                act_store<true>(a.y + 2 * eu, sh.epi[2 * (eu - lo)] + r0);
                act_store<true>(a.y + 2 * eu + 1, sh.epi[2 * (eu - lo) + 1] + r1);
            } else {
                const float2 cs = EPI == EPI_QKV ? sh.rope[((2 * eu) % a.d_head) / 2] : make_float2(1.f, 0.f);
                gemv_epilogue<WT, EPI, true, true>(a, eu, r0, r1, pos, cs);
            }
        }
        if (!REFILL && tid == 0) tick_bump(sh);   // the phase's last stores are on their way
    }

    // Runs the phase.  On entry `buf` holds this block's first tile; on return it holds the
    // block's first tile of phase Next (arguments `na`).
    template <typename Next>
    static __device__ __forceinline__ void run(const GemvArgs &a_in, const GemvArgs &na, int pos,
                                               FusedShared &sh, u32x4 (&buf)[NBUF], unsigned seq) {
        const GemvArgs a = uniform(a_in);   // keep every address ingredient in scalar registers
        const int tid = threadIdx.x, lane = tid & (WAVE - 1), w = (tid / WAVE) % NW, g = tid / (WAVE * NW);
        int lo, hi;
        block_range(n_units(a), blockIdx.x, gridDim.x, lo, hi, a.first_block);
        if (lo < hi) {
            // this lane's slice of x (RMS-normalised when a gain is given); the gain does not
            // depend on any activation, so its load goes out first
            float xr[P][VEC];
            uint32_t coff[P];
            u32x4 graw[P];
            float ss = 0.f;
#pragma unroll
            for (int p = 0; p < P; ++p) {
                coff[p] = col_offset(a, p);
                if (a.gain != nullptr)   // clamped: lanes past the row end must stay inside the gain vector
                    graw[p] = global_load16((const char *)a.gain + min(coff[p], (uint32_t)((a.cols - VEC) * sizeof(WT))));
            }
#pragma unroll
            for (int p = 0; p < P; ++p) {
                const int c = ((p * NW + w) * WAVE + lane) * VEC;
#pragma unroll
                for (int v = 0; v < VEC; v += 4) {
                    float4 t = make_float4(0.f, 0.f, 0.f, 0.f);
                    if (c < a.cols) t = global_load_float4(a.x + c + v);   // first read of a fresh address
                    xr[p][v] = t.x; xr[p][v + 1] = t.y; xr[p][v + 2] = t.z; xr[p][v + 3] = t.w;
                }
            }
            if (EPI == EPI_RESID) {   // this block's slice of the residual: 2 (hi - lo) <= MAX_EPI values
                for (int i = tid; i < 2 * (hi - lo); i += NT) sh.epi[i] = as_global(a.resid)[2 * lo + i];
            }
            if (QD < NS) {   // the rest of the first tile goes out behind x, which everything waits for
                asm volatile("" ::: "memory");
#pragma unroll
                for (int q = QD; q < NS; ++q) buf[q] = piece(a, lo, hi, q, coff);
            }
#pragma unroll
            for (int p = 0; p < P; ++p)
#pragma unroll
                for (int v = 0; v < VEC; ++v) ss += xr[p][v] * xr[p][v];
            if (a.gain != nullptr) {
                const float tot = block_sum<NT>(g == 0 ? ss : 0.f, sh.red);   // every group holds all of x
                const float rs = 1.0f / sqrtf(tot / (float)a.cols + a.eps);
#pragma unroll
                for (int p = 0; p < P; ++p) {
                    float gf[VEC];
                    Store<WT>::unpack(graw[p], gf);
#pragma unroll
                    for (int v = 0; v < VEC; ++v) xr[p][v] = xr[p][v] * rs * gf[v];   // x is 0 past the row end
                }
            }
            // All tiles but the last refill their registers unconditionally; the last one has
            // its own copy of the loop body.  (A refill under a branch makes the compiler wait
            // for every outstanding load at the loop's back edge: the stream would stop once
            // per tile.)
            int pb = 0, u0 = lo;
            for (; u0 + NG * UT < hi; u0 += NG * UT, pb ^= 1) tile<true>(a, u0, lo, hi, pos, sh, buf, xr, coff, pb);
            tile<false>(a, u0, lo, hi, pos, sh, buf, xr, coff, pb);
        }
        // Only wave 0 stored anything; the others request the next phase's first tile at once.
        // Wave 0 runs the device-wide barrier next and asks for its share after the release
        // (see grid_barrier).
        if (is_wave0()) wait_stores();
        else Next::prefetch_sliced(na, buf, sh, seq + 1);   // `seq` synchronisation points have been passed so far
    }
};

struct FusedArgs {
    SuperposeArgs sup;
    const spd_layer_weights *layers;   // device array [n_layers]
    const void *final_norm, *lm_head;
    char *act;
    ActLayout al;
    float *logits;
    void *kv;                          // layer l: K at kv + 2 l kv_layer_bytes, V one kv_layer_bytes later
    size_t kv_layer_bytes;
    float *part;
    int32_t *counters;
    const double *inv_freq;
    long long *prof;                   // optional: every block stamps wall_clock64() around every barrier
    unsigned *barrier;
    int32_t n_layers, d_model, n_heads, n_kv_heads, d_ffn, vocab, cap_ctx, max_splits, head;
    float eps;
};

template <int NBUF>
struct NoNext {
    static __device__ __forceinline__ void prefetch(const GemvArgs &, u32x4 (&)[NBUF]) {}
    static __device__ __forceinline__ void prefetch_sliced(const GemvArgs &, u32x4 (&)[NBUF], FusedShared &, unsigned) {}
};

__device__ __forceinline__ GemvArgs qkv_args(const FusedArgs &a, int l) {
    const int dh = a.d_model / a.n_heads;
    const int nq = a.n_heads * dh, nkv = a.n_kv_heads * dh;
    GemvArgs g{};
    const spd_layer_weights w = uniform(a.layers[l]);
    g.W = w.wqkv; g.gain = w.attn_norm; g.eps = a.eps; g.x = a.al.h_in(a.act, l); g.y = a.al.vec(a.act, l, a.al.q);
    g.rows = nq + 2 * nkv; g.cols = a.d_model;
    g.kcache = (char *)a.kv + (size_t)(2 * l) * a.kv_layer_bytes;
    g.vcache = (char *)a.kv + (size_t)(2 * l + 1) * a.kv_layer_bytes;
    g.inv_freq = a.inv_freq;
    g.n_q_rows = nq; g.n_kv_rows = nkv; g.d_head = dh; g.cap_ctx = a.cap_ctx;
    return g;
}

// After the QKV phase nothing but attention needs the new q, k and v, and attention for one
// head needs only that head's rows.  So instead of a device-wide barrier there is an arrival
// counter per key/value head that counts finished row pairs: a block adds, for every head, how
// many of its row pairs belong to the head's query, key or value rows (one lane of wave 0 per
// head, one atomic instruction), and a block about to run an attention item waits until the
// head's counter shows all of its row pairs.  Blocks without an item do not wait at all.  The
// counters run on from layer to layer and launch to launch like the barrier's.  Same rules as
// grid_barrier: the arriving wave has waited for its write-through stores; the wait is bounded.
__device__ __forceinline__ void qkv_arrive(unsigned *sync, const GemvArgs &q, FusedShared &sh, unsigned seq) {
    if (is_wave0()) {
        int lo, hi;
        block_range(q.rows / 2, blockIdx.x, gridDim.x, lo, hi, q.first_block);
        const int g = threadIdx.x, dh2 = q.d_head / 2, n_kv = q.n_kv_rows / q.d_head;
        const int tq = (q.n_q_rows / q.n_kv_rows) * dh2, kb = q.n_q_rows / 2, vb = (q.n_q_rows + q.n_kv_rows) / 2;
        auto overlap = [&](int a0, int a1) { return max(0, min(hi, a1) - max(lo, a0)); };
        const int mine = overlap(g * tq, (g + 1) * tq) + overlap(kb + g * dh2, kb + (g + 1) * dh2) + overlap(vb + g * dh2, vb + (g + 1) * dh2);
        if (g < n_kv && mine > 0)
            __hip_atomic_fetch_add(as_global(sync) + 64 * g, (unsigned)mine, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        if (threadIdx.x == 0) {
            tick_bump(sh);
            *lds_flag(&sh.released) = seq;
        }
    }
    __syncthreads();
}
__device__ __forceinline__ void qkv_wait(unsigned *sync, int kv_head, unsigned target, int *err) {
    if (threadIdx.x == 0) {
        unsigned spins = 0;
        while (__hip_atomic_load(as_global(sync) + 64 * kv_head, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) < target) {
            __builtin_amdgcn_s_sleep(QKV_SLEEP);
            ++spins;
            if ((spins & 255u) == 0 && __hip_atomic_load(as_global(err), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT)) break;
            if (spins > SPIN_LIMIT) {
                __hip_atomic_store(as_global(err), 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                break;
            }
        }
    }
    __syncthreads();
}

__device__ __forceinline__ GemvArgs head_args(const FusedArgs &a) {
    GemvArgs g{};
    g.W = a.lm_head; g.gain = a.final_norm; g.eps = a.eps; g.x = a.al.h_in(a.act, a.n_layers); g.y = a.logits;
    g.rows = a.vocab; g.cols = a.d_model;
    return g;
}

// PA / PB: passes a block needs to cover d_model / d_ffn columns.  Rows per tile follow from
// them so that a tile stays at about 16 pieces (16 bytes each) per lane.
constexpr int tile_rows(int passes) { return passes == 1 ? FUSED_UA : passes == 2 ? FUSED_UA / 2 : passes <= 4 ? 4 : 2; }

template <typename WT, int PA, int PB>
__global__ __launch_bounds__(NT) void fused_forward_kernel(const FusedArgs a) {
    constexpr int UA = tile_rows(PA), UB = tile_rows(PB);
    // The O projection is one tile per block; its tile is a little taller so that it still is
    // when the blocks busy with attention items leave their rows to the others.
    constexpr int UO = UA + FUSED_UO_EXTRA / PA;
    constexpr int NA = PA * UO;
    constexpr int NBUF = (NA > PB * UB) ? NA : PB * UB;
    constexpr int SL = PA == 1 ? FUSED_SLICE : FUSED_SLICE_WIDE;
    constexpr int BAR_SLEEP = PB > 4 ? BAR_SLEEP_WIDE : BAR_SLEEP_7B;
    using Qkv = Gemv<WT, PA, UA, EPI_QKV, NBUF, SL>;
    using Oproj = Gemv<WT, PA, UO, EPI_RESID, NBUF, SL>;
    using GateUp = Gemv<WT, PA, UA, EPI_SWIGLU, NBUF, SL>;
    using Down = Gemv<WT, PB, UB, EPI_RESID, NBUF, SL>;
    using Head = Gemv<WT, PA, UA, EPI_PLAIN, NBUF, SL>;
    __shared__ FusedShared sh;
    __shared__ __align__(16) float dyn[NT * Store<KvT>::VEC];

#define SPD_BARRIER(ALL_WAVES_STORED)                                        \
    do {                                                                     \
        if (prof && threadIdx.x == 0) as_global(prof)[2 * seq] = wall_clock64();      \
        grid_barrier<ALL_WAVES_STORED, BAR_SLEEP>(a.barrier, ++epoch, &st->err, sh, ++seq); \
        if (prof && threadIdx.x == 0) as_global(prof)[2 * seq - 1] = wall_clock64();  \
    } while (0)
    DevState *st = a.sup.st;
    long long *prof = (a.prof && blockIdx.x < FUSED_PROF_BLOCKS) ? a.prof + (size_t)blockIdx.x * (size_t)(2 * (5 * a.n_layers + 2)) : nullptr;
    const int pos = uniform(as_global(st)->pos);
    const int dh = a.d_model / a.n_heads;
    const int nq = a.n_heads * dh;
    // The barrier counters run on from launch to launch (the host zeroes them only when a prefix
    // pass begins): `epoch` continues from the number of barriers all earlier launches passed,
    // which block 0 leaves behind when it ends.  Every block has read it before it arrives at
    // this launch's first barrier, and block 0 cannot get past that barrier without them.
    const unsigned epoch0 = (unsigned)uniform((int)__hip_atomic_load(as_global(a.barrier) + BAR_EPOCH_WORD, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT));
    unsigned epoch = epoch0;
    unsigned seq = 0;   // synchronisation points passed in this launch (device-wide barriers and per-head arrivals)
    const unsigned layers0 = (unsigned)uniform((int)__hip_atomic_load(as_global(a.barrier) + BAR_LAYER_WORD, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT));
    unsigned *qkv_sync = a.barrier + QKV_SYNC_WORD0;
    const bool per_head = a.n_kv_heads <= QKV_SYNC_MAX;
    const unsigned head_units = (unsigned)((a.n_heads / a.n_kv_heads + 2) * (dh / 2));   // row pairs of one key/value head's q, k, v

    // phase 0: the input vector (Section 3.1, Eq. 1 and 2); every block keeps this position's
    // rotary table in LDS
    for (int c = blockIdx.x * NT + threadIdx.x; c < a.d_model; c += gridDim.x * NT)
        superpose_element<WT, true>(a.sup, c, pos);
    if (threadIdx.x < dh / 2) sh.rope[threadIdx.x] = rope_cos_sin(a.inv_freq, threadIdx.x, pos);
    wait_stores();
    u32x4 buf[NBUF];
    GemvArgs cur = a.n_layers > 0 ? qkv_args(a, 0) : head_args(a);
    if (threadIdx.x == 0) { sh.tick = 0; sh.released = 0; }
    __syncthreads();
    if (!is_wave0()) {   // (not sliced: before this barrier the whole block meets first)
        if (a.n_layers > 0) Qkv::prefetch(cur, buf);
        else if (a.head) Head::prefetch(cur, buf);
    }
    SPD_BARRIER(true);
    if (is_wave0()) {
        if (a.n_layers > 0) Qkv::prefetch(cur, buf);
        else if (a.head) Head::prefetch(cur, buf);
    }

    for (int l = 0; l < a.n_layers; ++l) {
        const spd_layer_weights w = uniform(a.layers[l]);
        GemvArgs o{};
        float *att = a.al.vec(a.act, l, a.al.att), *h1 = a.al.vec(a.act, l, a.al.h1);
        float *u = a.al.vec(a.act, l, a.al.u), *h2 = a.al.vec(a.act, l, a.al.h2);
        o.W = w.wo; o.x = att; o.resid = a.al.h_in(a.act, l); o.y = h1; o.rows = a.d_model; o.cols = nq;
        // Attention items: one per (query head, chunk of cached positions).  Up to
        // FUSED_ONE_CHUNK positions a head is ONE item (one or two batches of loads in one
        // block): a second batch costs about 2 us, merging chunks across blocks about 4 us (an
        // acknowledged store, an atomic and two dependent loads), but one compute unit's share
        // of the bandwidth makes a single block the slower choice past some 270 positions.
        // Longer contexts are cut so that every block gets an item if the chunk bounds allow.
        // While few blocks have an item those take no rows of the O projection: they would hold
        // everybody up fetching their tile after the attention.
        const int n_ctx = pos + 1;
        int chunk = FUSED_ONE_CHUNK;
        if (n_ctx > FUSED_ONE_CHUNK) {
            const int per_head = max(1, (int)gridDim.x / a.n_heads);
            chunk = ((n_ctx + per_head - 1) / per_head + 15) & ~15;
            chunk = min(ATTN_CHUNK_MAX, max(ATTN_CHUNK_MIN, chunk));
        }
        const int n_splits = (n_ctx + chunk - 1) / chunk;
        const int n_items = a.n_heads * n_splits;
        o.first_block = 4 * n_items <= (int)gridDim.x ? n_items : 0;
        Qkv::template run<Oproj>(cur, o, pos, sh, buf, seq);
        if (per_head) {   // no device-wide barrier here: see qkv_arrive
            if (prof && threadIdx.x == 0) as_global(prof)[2 * seq] = wall_clock64();
            qkv_arrive(qkv_sync, cur, sh, ++seq);
            if (prof && threadIdx.x == 0) as_global(prof)[2 * seq - 1] = wall_clock64();
        } else {
            SPD_BARRIER(false);
        }
        if (is_wave0()) Oproj::prefetch(o, buf);

        {   // attention over pos + 1 cached positions; the O-projection tile stays in flight
            AttnArgs t{cur.y, cur.kcache, cur.vcache, att, a.part, a.counters, nullptr, n_ctx,
                       a.n_heads, a.n_kv_heads, dh, a.cap_ctx, chunk, a.max_splits};
            const int group = a.n_heads / a.n_kv_heads;
            for (int item = blockIdx.x; item < n_items; item += gridDim.x) {
                const int h = item / n_splits;
                if (per_head) qkv_wait(qkv_sync, h / group, (layers0 + l + 1) * head_units, &st->err);
                attn_item<KvT, NT, true>(t, h / group, item % n_splits, n_ctx, sh.sc, sh.red, dyn, &sh.s_last,
                                         h % group, h % group + 1);
            }
            wait_stores();
        }
        SPD_BARRIER(true);

        GemvArgs f{};
        f.W = w.w_gate; f.W2 = w.w_up; f.gain = w.ffn_norm; f.eps = a.eps; f.x = h1; f.y = u;
        f.rows = a.d_ffn; f.cols = a.d_model;
        Oproj::template run<GateUp>(o, f, pos, sh, buf, seq);
        SPD_BARRIER(false);
        if (is_wave0()) GateUp::prefetch(f, buf);

        GemvArgs d{};
        d.W = w.w_down; d.x = u; d.resid = h1; d.y = h2; d.rows = a.d_model; d.cols = a.d_ffn;
        GateUp::template run<Down>(f, d, pos, sh, buf, seq);
        SPD_BARRIER(false);
        if (is_wave0()) Down::prefetch(d, buf);

        if (l + 1 < a.n_layers) {
            cur = qkv_args(a, l + 1);
            Down::template run<Qkv>(d, cur, pos, sh, buf, seq);
        } else if (a.head) {
            cur = head_args(a);
            Down::template run<Head>(d, cur, pos, sh, buf, seq);
        } else {
            Down::template run<NoNext<NBUF>>(d, d, pos, sh, buf, seq);
        }
        if (l + 1 < a.n_layers || a.head) SPD_BARRIER(false);
        if (is_wave0()) {
            if (l + 1 < a.n_layers) Qkv::prefetch(cur, buf);
            else if (a.head) Head::prefetch(cur, buf);
        }
    }
    if (a.head) Head::template run<NoNext<NBUF>>(cur, cur, pos, sh, buf, seq);
    if (prof && threadIdx.x == 0) as_global(prof)[2 * seq] = wall_clock64();
    if (blockIdx.x == 0 && threadIdx.x == 0) {
        __hip_atomic_store(as_global(a.barrier) + BAR_EPOCH_WORD, epoch, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        __hip_atomic_store(as_global(a.barrier) + BAR_LAYER_WORD, layers0 + (unsigned)a.n_layers, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
#undef SPD_BARRIER
}

template <typename WT, int PA, int PB> struct Variant {
    static hipError_t launch(hipStream_t s, const FusedArgs &a, int blocks) {
        hipLaunchKernelGGL((fused_forward_kernel<WT, PA, PB>), dim3(blocks), dim3(NT), 0, s, a);
        return hipGetLastError();
    }
    static int blocks_per_cu() {
        int n = 0;
        if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&n, (const void *)fused_forward_kernel<WT, PA, PB>, NT, 0) != hipSuccess) {
            (void)hipGetLastError();
            return 0;
        }
        return n;
    }
};

// The instantiations that exist: passes needed to cover d_model and d_ffn with NW waves
// (bf16: 4096 columns per pass).  (1,1) and (1,2): small models; (1,3): the Llama-2-7B shape;
// (2,4): 13B; (2,7): 70B.  Calls f(Variant<...>{}) for the one that serves the shape.
template <typename F>
bool with_variant(int dtype, int d_model, int d_ffn, F &&f) {
    const int vec = dtype == SPD_DTYPE_BF16 ? 8 : 4;
    const int span = NW * WAVE * vec;
    const int pa = (d_model + span - 1) / span, pb = (d_ffn + span - 1) / span;
    if (dtype == SPD_DTYPE_BF16) {
        if (pa == 1 && pb == 1) return f(Variant<bf16_t, 1, 1>{}), true;
        if (pa == 1 && pb == 2) return f(Variant<bf16_t, 1, 2>{}), true;
        if (pa == 1 && pb == 3) return f(Variant<bf16_t, 1, 3>{}), true;
        if (pa == 2 && pb == 4) return f(Variant<bf16_t, 2, 4>{}), true;
        if (pa == 2 && pb == 7) return f(Variant<bf16_t, 2, 7>{}), true;
    } else {
        if (pa == 1 && pb == 1) return f(Variant<float, 1, 1>{}), true;
        if (pa == 1 && pb == 2) return f(Variant<float, 1, 2>{}), true;
        if (pa == 1 && pb == 3) return f(Variant<float, 1, 3>{}), true;
    }
    return false;
}

}  // namespace

namespace spdk {

int fused_max_blocks_per_cu(int dtype, int d_model, int d_ffn) {
    int n = 0;
    with_variant(dtype, d_model, d_ffn, [&](auto v) { n = decltype(v)::blocks_per_cu(); });
    return n;
}

hipError_t fused_forward(hipStream_t s, int dtype, const FusedArgsHost &h, int blocks) {
    FusedArgs a{};
    a.sup = h.sup; a.layers = h.layers; a.final_norm = h.final_norm; a.lm_head = h.lm_head;
    a.act = h.act; a.al = h.al; a.logits = h.logits;
    a.kv = h.kv; a.kv_layer_bytes = h.kv_layer_bytes; a.part = h.part; a.counters = h.counters;
    a.inv_freq = h.inv_freq; a.prof = h.prof; a.barrier = h.barrier;
    a.n_layers = h.n_layers; a.d_model = h.d_model; a.n_heads = h.n_heads; a.n_kv_heads = h.n_kv_heads;
    a.d_ffn = h.d_ffn; a.vocab = h.vocab; a.cap_ctx = h.cap_ctx; a.max_splits = h.max_splits; a.head = h.head;
    a.eps = h.eps;
    hipError_t e = hipErrorInvalidValue;
    with_variant(dtype, h.d_model, h.d_ffn, [&](auto v) { e = decltype(v)::launch(s, a, blocks); });
    return e;
}

}  // namespace spdk
