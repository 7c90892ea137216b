// The whole transformer forward of one SPD timestep as ONE persistent kernel.
//
// Batch-1 decode is a chain of ~160 small matrix-vector products (7B shape: 33-180 MB each,
// 6-30 us at HBM speed), every one of which needs the complete output of its predecessor.
// Launching them one by one leaves HBM idle at every boundary, so here a grid that exactly
// fills the chip walks through all phases itself.  There is no device-wide barrier between
// phases: the activation vectors themselves say whether they are complete.  Every element of
// a vector holds ACT_UNSET (a NaN bit pattern no arithmetic produces) until its producer has
// stored it; a consumer loads the slice of the vector it needs, coherently, and loads again
// whatever still reads ACT_UNSET.  So between "the last producer stored" and "every consumer
// computes" lies one trip to memory, not the chain store acknowledged -> arrival counted ->
// release polled -> vector loaded, each link of which queues behind the compute unit's own
// outstanding weight requests (a compute unit serves its memory operations in order).
// (The query and the newest key and value rows are such vectors too: attention awaits its
// head's slices of them.)
// Two activation arenas alternate from launch to launch: whoever stores an element of this
// launch's arena stores ACT_UNSET to the same element of the other one, which the next launch
// finds unset throughout (the host sets both when a prefix pass begins).
//
// The weights a block needs for its first tile of the NEXT phase do not depend on any
// activation, so they are requested while the block waits for its input, a slice at a time
// between two looks at the input: the weight stream from HBM does not stop at phase boundaries.
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
constexpr int FUSED_QD = 20;          // 16-byte pieces per lane of a phase's first tile requested while its input is awaited
constexpr int FUSED_QD_ITEM = 4;      // of which this many are requested before an attention item (they stay in registers through it)
constexpr int FUSED_SLICE = 20;        // pieces that go out between two looks at the input
constexpr int FUSED_SLICE_GATE = 4;   // the first slice of the gate/up phase (its input follows the attention within a microsecond or two)
constexpr int FUSED_SLICE_WIDE = 4;   // the same for models whose d_model takes two block passes
// An fp16 cache is read 8 bytes (4 elements) per lane, like the fp32 one, while the context fits one batch of
// loads (160 positions), 16 bytes per lane beyond:
constexpr int FUSED_HALF_ROWS_ONE = 8;        // 16 bytes per lane: rows in flight per lane where a head is one item (256 positions per batch)
constexpr int FUSED_HALF_ROWS_CUT = 6;        // ... and where the context is cut into chunks (192 per batch: chunks of contexts up to 1536)
constexpr int FUSED_ONE_CHUNK_HALF = 512;     // FUSED_ONE_CHUNK for an fp16 cache: half the bytes per position
constexpr int FUSED_ONE_CHUNK = 256;  // contexts up to this long are one attention item per head (no merge across blocks)
static_assert(FUSED_ONE_CHUNK <= ATTN_CHUNK_MAX && FUSED_ONE_CHUNK_HALF <= ATTN_CHUNK_MAX, "one attention item must fit the score buffer");
constexpr int INPUT_SLEEP = 2;        // s_sleep units (64 cycles) between two looks at an input that is not complete yet
constexpr int NT = 512;               // threads per block
constexpr int NW = 8;                 // waves side by side on one row
constexpr int MAX_U = 32;
constexpr int MAX_SLOTS = 128;       // partial sums (rows x passes) a tile may leave in LDS per row group
constexpr int FUSED_UPM = 16;        // rows per tile (= pieces per lane in flight) of a pass-major phase
constexpr bool FUSED_PM_CACHED = true;    // a pass-major phase reads all passes of its input but the last through the L2
constexpr int NG = NT / WAVE / NW;   // row groups per block
constexpr unsigned SPIN_LIMIT = 1u << 22;

constexpr int MAX_EPI = FUSED_MAX_EPI;   // residual values a block may need in one phase

struct FusedShared {
    float part[2][NG][MAX_SLOTS][NW]; // [buffer][row group][tile slot][wave]
    float epi[MAX_EPI];           // this block's slice of the residual, staged when the phase starts
    float2 rope[128];             // (cos, sin) of this step's position, all d_head / 2 <= 128 pairs
    float red[NT / WAVE];
    float sc[ATTN_CHUNK_MAX];
    int s_last;
};

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
    r.cap_ctx = uniform(a.cap_ctx); r.first_block = uniform(a.first_block); r.chunk_span = uniform(a.chunk_span);
    r.k_new = uniform(a.k_new); r.v_new = uniform(a.v_new);
    return r;
}

__device__ __forceinline__ bool is_wave0() { return __builtin_amdgcn_readfirstlane((int)threadIdx.x) < WAVE; }

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

// What a phase leaves in the profile: stamp[2i] = the block has finished everything before
// synchronisation point i (its outputs are stored), stamp[2i+1] = it has what it needs to go on.
struct Prof {
    long long *p;
    __device__ __forceinline__ void done(unsigned point) const { if (p && threadIdx.x == 0) as_global(p)[2 * point] = wall_clock64(); }
    __device__ __forceinline__ void go(unsigned point) const { if (p && threadIdx.x == 0) as_global(p)[2 * point + 1] = wall_clock64(); }
};

// After the QKV phase nothing but attention needs the new q, k and v, and attention for one
// head needs only that head's rows.  Like every other vector they are awaited as data: the
// query in its activation vector, the newest key and value rows in two more (k_new, v_new;
// the cache gets them too, for the launches to come), each element unset until its producer has
// stored it.  A block with an attention item requests the cached rows of the earlier positions
// and then looks at its head's slices until they are complete; blocks without an item do not
// wait at all.
// The two finished dot products of row pair `unit` of the QKV matrix: rotary on q and k pairs
// (the arithmetic of gemv_epilogue, bit for bit), stores as above.
template <typename WT, typename KT>
__device__ __forceinline__ void qkv_store(const GemvArgs &a, int unit, float acc0, float acc1, int pos, float2 cs) {
    const int r0 = 2 * unit;
    if (r0 < a.n_q_rows + a.n_kv_rows) {
        const float c = cs.x, s = cs.y;
        const float e = __fsub_rn(__fmul_rn(acc0, c), __fmul_rn(acc1, s));
        const float o = __fadd_rn(__fmul_rn(acc0, s), __fmul_rn(acc1, c));
        if (r0 < a.n_q_rows) {
            act_store<true>(a.y + r0, e);
            act_store<true>(a.y + r0 + 1, o);
            if (a.twin) { twin_unset(a.y + r0, a.twin); twin_unset(a.y + r0 + 1, a.twin); }
        } else {
            const int rr = r0 - a.n_q_rows;
            const size_t at = ((size_t)(rr / a.d_head) * a.cap_ctx + pos) * a.d_head + rr % a.d_head;
            float ke = e, ko = o;   // (as the cache holds them: this step sees what later steps will read)
            kv_store_pair<true, sizeof(KT) == 2>(a.kcache, at, ke, ko);
            act_store<true>(a.k_new + rr, ke);
            act_store<true>(a.k_new + rr + 1, ko);
            if (a.twin) { twin_unset(a.k_new + rr, a.twin); twin_unset(a.k_new + rr + 1, a.twin); }
        }
    } else {
        const int rr = r0 - a.n_q_rows - a.n_kv_rows;
        const size_t at = ((size_t)(rr / a.d_head) * a.cap_ctx + pos) * a.d_head + rr % a.d_head;
        kv_store_pair<true, sizeof(KT) == 2>(a.vcache, at, acc0, acc1);
        act_store<true>(a.v_new + rr, acc0);
        act_store<true>(a.v_new + rr + 1, acc1);
        if (a.twin) { twin_unset(a.v_new + rr, a.twin); twin_unset(a.v_new + rr + 1, a.twin); }
    }
}

// Where a block stands in its walk through a phase: chunk j, of which it owns units [lo, hi),
// tile at unit u0.
struct Cursor { int j, lo, hi, u0; };

// The input vector of a phase as its lanes await it: raw 16-byte pieces (XP per column pass),
// which of them still read unset.
template <int P, int VEC>
struct LazyXT {
    static constexpr int XP = VEC / 4;
    static constexpr int PASS_COLS = NW * WAVE * VEC;
    __amdgpu_buffer_rsrc_t xres;
    int c0;                 // this lane's first column of pass 0
    u32x4 xv[P][XP];
    unsigned pend;          // bit p * XP + j: that piece is still missing
    static constexpr unsigned pass_mask(int p) { return ((1u << XP) - 1u) << (p * XP); }
    // Passes below CACHED_BELOW are read through the L2 (a producer finished them long ago:
    // a hit costs no trip across the chip; should a word still read unset, the line is stale
    // in this L2 from then on, which costs later looks a coherent retry and nothing else:
    // retries are always coherent).
    template <int CACHED_BELOW = 0>
    __device__ __forceinline__ void look(unsigned mask) {
#pragma unroll
        for (int p = 0; p < P; ++p) {
#pragma unroll
            for (int j = 0; j < XP; ++j)
                if (pend & mask & (1u << (p * XP + j)))
                    xv[p][j] = p < CACHED_BELOW ? cached_look16(xres, (uint32_t)(c0 + p * PASS_COLS + 4 * j) * 4u)
                                                : coherent_load16(xres, (uint32_t)(c0 + p * PASS_COLS + 4 * j) * 4u);
        }
    }
    __device__ __forceinline__ void judge(unsigned mask) {
#pragma unroll
        for (int p = 0; p < P; ++p)
#pragma unroll
            for (int j = 0; j < XP; ++j) {
                const u32x4 v = xv[p][j];
                if ((mask & (1u << (p * XP + j))) && v.x != ACT_UNSET && v.y != ACT_UNSET && v.z != ACT_UNSET && v.w != ACT_UNSET)
                    pend &= ~(1u << (p * XP + j));
            }
    }
    // Waits (bounded) until none of the pieces in `mask` is missing.  The answer to the last
    // look is judged outside the loop: inside it the compiler has to assume the look at the
    // loop's end and waits for EVERY outstanding load, the weight requests behind it included.
    __device__ __forceinline__ void await(unsigned mask, int *err) {
        if (__any((pend & mask) != 0)) judge(mask);
        for (unsigned spins = 0; __any((pend & mask) != 0); ++spins) {
            if (spins > SPIN_LIMIT || ((spins & 255u) == 255u && __hip_atomic_load(as_global(err), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT))) {
                // bounded: the grid is not co-resident (or a producer gave up): raise the flag and go on
                __hip_atomic_store(as_global(err), 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                break;
            }
            __builtin_amdgcn_s_sleep(INPUT_SLEEP);
            look(mask);
            judge(mask);
        }
    }
    __device__ __forceinline__ void take(int p, float (&xr)[P][VEC]) const {
#pragma unroll
        for (int j = 0; j < XP; ++j) {
            xr[p][4 * j] = __uint_as_float(xv[p][j].x); xr[p][4 * j + 1] = __uint_as_float(xv[p][j].y);
            xr[p][4 * j + 2] = __uint_as_float(xv[p][j].z); xr[p][4 * j + 3] = __uint_as_float(xv[p][j].w);
        }
    }
};

// What the predecessor phase sets up of a phase before its own last tile (see Gemv::tile, MODE
// 2): where the block starts and, for a pass-major phase, the look at the first pass of its
// input and the residual.
template <int P, int VEC>
struct PreT {
    Cursor cur;
    LazyXT<P, VEC> lx;
    float resid;  // this thread's element of the block's residual slice
    bool valid;   // the block owns units of this phase
};

// A phase keeps ONE tile of U rows x P passes (NS = U * P 16-byte pieces per lane) in
// registers.  The moment a piece has been multiplied in, its register is re-used for the same
// piece of the block's next tile, so a wave always has about NS loads in flight.
// Loads are never predicated: a row past the block's range re-reads the last valid row (a
// cache hit), and a column past the row end lies outside the buffer descriptor, which
// describes one row (zeros come back, nothing is fetched); the inner loop has no branches.
//
// Chunks (a.chunk_span > 0): the phase's units are cut into chunks of chunk_span units, every
// block owns a balanced range of EVERY chunk and walks chunk after chunk.  All blocks together
// therefore complete the output vector front to back, a chunk at a time, and a consumer that
// needs the vector a column pass at a time (below) finds its first passes long before the
// phase ends.
//
// PM ("pass-major", for a phase whose rows take P >= 2 column passes): a tile is U rows, walked
// pass by pass -- all U rows against pass 0 of x, then against pass 1, ... -- with U pieces per
// lane in flight (piece (p, s) is re-requested as (p + 1, s), the last pass as the next tile's
// pass 0).  Pass p of x is needed only when the walk gets there: the phase starts as soon as
// pass 0 is complete and looks at the later passes, a tile's pass ahead each, while it streams.
// With a producer that works in chunks of one pass width, only the last pass's chunk is still
// being written when the phase starts, and it is needed a tile's (P - 1) / P later.
template <typename WT, int P, int U, int EPI, int NBUF, int SL, bool PM = false, bool CHUNKS = false, int SL0 = SL, typename KT = float>
struct Gemv {
    static constexpr int VEC = Store<WT>::VEC;
    static constexpr int XP = VEC / 4;   // 16-byte pieces of x per pass and lane
    static constexpr int UT = U / 2;     // units per tile
    static constexpr int NS = PM ? U : U * P;   // pieces per lane in flight
    static constexpr int PASS_COLS = NW * WAVE * VEC;   // columns of a row the block covers per pass
    using LazyX = LazyXT<P, VEC>;
    using Pre = PreT<P, VEC>;
    static_assert(U % 2 == 0 && NS <= NBUF && U <= MAX_U && U * P <= MAX_SLOTS, "tile does not fit the register window");
    static_assert(NG * UT <= WAVE, "the epilogue threads must all sit in wave 0");
    static_assert(P * XP <= 32, "one bit per piece of x");
    static_assert(!PM || (P >= 2 && EPI == EPI_RESID), "pass-major tiles: several passes, no normalisation of x");

    static __device__ __forceinline__ int n_units(const GemvArgs &a) { return EPI == EPI_SWIGLU ? a.rows : a.rows / 2; }

    // Byte offset of this lane's piece of pass p within a row.
    static __device__ __forceinline__ uint32_t col_offset(const GemvArgs &a, int p) {
        const int lane = threadIdx.x & (WAVE - 1), w = (threadIdx.x / WAVE) % NW;
        const int c = ((p * NW + w) * WAVE + lane) * VEC;
        return (uint32_t)c * (uint32_t)sizeof(WT);   // past the row end: the load returns zero
    }

    static __device__ __forceinline__ int n_chunks(const GemvArgs &a) {
        return CHUNKS ? (n_units(a) + a.chunk_span - 1) / a.chunk_span : 1;
    }
    static __device__ __forceinline__ void chunk_range(const GemvArgs &a, int j, int &lo, int &hi) {
        const int n = n_units(a);
        const int base = CHUNKS ? j * a.chunk_span : 0;
        const int len = CHUNKS ? min(a.chunk_span, n - base) : n;
        block_range(len, blockIdx.x, gridDim.x, lo, hi, a.first_block);
        lo += base; hi += base;
    }
    // The block's first tile; false: the block owns no unit of this phase.
    static __device__ __forceinline__ bool first_tile(const GemvArgs &a, Cursor &c) {
        const int nc = n_chunks(a);
        for (c.j = 0; c.j < nc; ++c.j) {
            chunk_range(a, c.j, c.lo, c.hi);
            if (c.lo < c.hi) { c.u0 = c.lo; return true; }
        }
        return false;
    }
    // The tile after c; false: c is the block's last tile.
    static __device__ __forceinline__ bool next_tile(const GemvArgs &a, const Cursor &c, Cursor &n) {
        n = c;
        n.u0 += NG * UT;
        if (n.u0 < n.hi) return true;
        if (!CHUNKS) return false;
        const int nc = n_chunks(a);
        while (++n.j < nc) {
            chunk_range(a, n.j, n.lo, n.hi);
            if (n.lo < n.hi) { n.u0 = n.lo; return true; }
        }
        return false;
    }

    // Row slot s, pass p of this wave's row group within the block tile starting at unit u0
    // (a block tile is NG * UT units) of a chunk range that ends at u_end.
    static __device__ __forceinline__ u32x4 piece_sp(const GemvArgs &a, int u0, int u_end, int s, int p, const uint32_t (&coff)[P]) {
        const int g = __builtin_amdgcn_readfirstlane(threadIdx.x / (WAVE * NW));
        const int unit = min(u0 + g * UT + (EPI == EPI_SWIGLU ? (s % UT) : (s / 2)), u_end - 1);
        const uint32_t row_bytes = (uint32_t)a.cols * (uint32_t)sizeof(WT);
        const char *W = (const char *)(EPI == EPI_SWIGLU && s >= UT ? a.W2 : a.W);
        const int row = EPI == EPI_SWIGLU ? unit : 2 * unit + (s & 1);
        return stream_load16(row_resource(W + (size_t)row * row_bytes, row_bytes), coff[p]);
    }
    // Piece q of the tile in the order the registers hold it: row-major q = s * P + p; pass-major:
    // the U rows of pass 0.
    static __device__ __forceinline__ u32x4 piece(const GemvArgs &a, int u0, int u_end, int q, const uint32_t (&coff)[P]) {
        return PM ? piece_sp(a, u0, u_end, q, 0, coff) : piece_sp(a, u0, u_end, q / P, q % P, coff);
    }

    // Piece q of a tile for a predecessor phase that requests it (see tile, MODE 2): the lane's
    // column offset of pass 0 is the same in every phase, the other passes follow from it.
    static __device__ __forceinline__ u32x4 piece_for(const GemvArgs &a, int u0, int u_end, int q, uint32_t coff0) {
        uint32_t coff[P];
#pragma unroll
        for (int p = 0; p < P; ++p) coff[p] = coff0 + (uint32_t)p * (uint32_t)(PASS_COLS * sizeof(WT));
        return piece(a, u0, u_end, q, coff);
    }

    // The head of a block's first tile, pieces [0, QD), goes out while the input is awaited;
    // the rest follows once the input is there.
    static constexpr int QD = NS < FUSED_QD ? NS : FUSED_QD;

    // Requests pieces [0, QI) at once.  For a block that has other work to do (an attention
    // item) before it can look at this phase's input: run() is then told they are on their way.
    static constexpr int QI = NS < FUSED_QD_ITEM ? NS : FUSED_QD_ITEM;
    static __device__ __forceinline__ void prefetch(const GemvArgs &a_in, u32x4 (&buf)[NBUF]) {
        const GemvArgs a = uniform(a_in);
        Cursor c;
        if (!first_tile(a, c)) return;
        uint32_t coff[P];
#pragma unroll
        for (int p = 0; p < P; ++p) coff[p] = col_offset(a, p);
#pragma unroll
        for (int q = 0; q < QI; ++q) buf[q] = piece(a, c.u0, c.hi, q, coff);
    }

    // The block has met after a tile: the first NG * UT threads finish their units of the tile
    // at unit u0 (chunk range [lo, hi)); a unit's two sums are spread over NPART slots each.
    template <int NPART>
    static __device__ __forceinline__ void finish(const GemvArgs &a, int u0, int lo, int hi, int pos, FusedShared &sh, int pb) {
        const int tid = threadIdx.x;
        const int eu = min(u0 + tid, hi - 1);
        if (tid < NG * UT && u0 + tid < hi) {   // unit u0 + tid: row group tid / UT, pair tid % UT
            const int eg = tid / UT, t = tid % UT;
            const int s0 = EPI == EPI_SWIGLU ? t : 2 * t;
            const int s1 = EPI == EPI_SWIGLU ? t + UT : 2 * t + 1;
            float r0 = 0.f, r1 = 0.f;
#pragma unroll
            for (int p = 0; p < NPART; ++p) {
#pragma unroll
                for (int q = 0; q < NW; ++q) { r0 += sh.part[pb][eg][p * U + s0][q]; r1 += sh.part[pb][eg][p * U + s1][q]; }
            }
            // what the epilogue needs beyond the sums sits in LDS: the tile loop holds no load
            // from global memory but the weights'
            if (EPI == EPI_RESID) {
                act_store<true>(a.y + 2 * eu, sh.epi[2 * (eu - lo)] + r0);
                act_store<true>(a.y + 2 * eu + 1, sh.epi[2 * (eu - lo) + 1] + r1);
                if (a.twin) { twin_unset(a.y + 2 * eu, a.twin); twin_unset(a.y + 2 * eu + 1, a.twin); }
            } else if (EPI == EPI_QKV) {
                qkv_store<WT, KT>(a, eu, r0, r1, pos, sh.rope[((2 * eu) % a.d_head) / 2]);
            } else {
                gemv_epilogue<WT, EPI, true, true>(a, eu, r0, r1, pos);
                if (EPI == EPI_SWIGLU && a.twin) twin_unset(a.y + eu, a.twin);
            }
        }
    }

    // One tile: U rows of this wave's row group against x, partial sums to LDS, the block
    // meets, the first NG * UT threads finish their units.  Every consumed register is
    // re-requested at once -- MODE 1: with the same piece of the block's next tile (cursor n);
    // MODE 2 (the phase's last tile): the first NXQ registers with the same piece of the block's
    // first tile of the NEXT phase Nx (arguments na, cursor n) -- weights do not depend on
    // activations, and so the stream from HBM does not run dry at the phase boundary.  All of
    // the tile where Nx finds its input complete (gate/up -> down); elsewhere only its head:
    // whatever is requested here is in the compute unit's queue AHEAD of this tile's own stores
    // and of the next phase's look at its input, and the head is the part that has come back
    // by then.  MODE 0: not at all.
    template <int MODE, typename Nx, int NXQ = 0>
    static __device__ __forceinline__ void tile(const GemvArgs &a, const Cursor &c, const Cursor &n, int pos,
                                                FusedShared &sh, u32x4 (&buf)[NBUF], const float (&xr)[P][VEC],
                                                const uint32_t (&coff)[P], int pb, const GemvArgs &na) {
        const int tid = threadIdx.x, lane = tid & (WAVE - 1), w = (tid / WAVE) % NW, g = tid / (WAVE * NW);
        if constexpr (MODE == 2) {   // registers the next phase's tile has beyond this one's
#pragma unroll
            for (int q = NS; q < NXQ; ++q) buf[q] = Nx::piece_for(na, n.u0, n.hi, q, coff[0]);
        }
#pragma unroll
        for (int s = 0; s < U; ++s) {
            float acc = 0.f;
#pragma unroll
            for (int p = 0; p < P; ++p) {
                float f[VEC];
                Store<WT>::unpack(buf[s * P + p], f);
#pragma unroll
                for (int v = 0; v < VEC; ++v) acc = fmaf(f[v], xr[p][v], acc);
                if (MODE == 1) buf[s * P + p] = piece(a, n.u0, n.hi, s * P + p, coff);
                if constexpr (MODE == 2) { if (s * P + p < NXQ) buf[s * P + p] = Nx::piece_for(na, n.u0, n.hi, s * P + p, coff[0]); }
            }
            acc = wave_sum_last(acc);
            if (lane == WAVE - 1) sh.part[pb][g][s][w] = acc;
        }
        __syncthreads();
        finish<1>(a, c.u0, c.lo, c.hi, pos, sh, pb);
    }

    // Element threadIdx.x of the block's slice of the residual: 2 (hi - lo) <= MAX_EPI = NT values.
    // It has been complete for a whole phase; read coherently all the same.  (Phases with a
    // residual are not cut into chunks.)  Requested before anything else of the phase, so that
    // it does not come back behind the weight stream.
    static __device__ __forceinline__ float load_resid(const GemvArgs &a, const Cursor &c) {
        static_assert(MAX_EPI <= NT, "one residual element per thread");
        const int i = threadIdx.x;
        return (EPI == EPI_RESID && i < 2 * (c.hi - c.lo)) ? coherent_load(a.resid + 2 * c.lo + i) : 0.f;
    }
    static __device__ __forceinline__ void lazy_init(const GemvArgs &a, LazyX &lx) {
        const int lane = threadIdx.x & (WAVE - 1), w = (threadIdx.x / WAVE) % NW;
        lx.xres = __builtin_amdgcn_make_buffer_rsrc(const_cast<float *>(a.x), 0, a.cols * 4, 0x00020000);
        lx.c0 = (w * WAVE + lane) * VEC;
        lx.pend = 0;
#pragma unroll
        for (int p = 0; p < P; ++p) {
#pragma unroll
            for (int j = 0; j < XP; ++j) {
                lx.xv[p][j] = u32x4{0u, 0u, 0u, 0u};   // past the row end: x is 0, nothing to wait for
                if (lx.c0 + p * PASS_COLS < a.cols) lx.pend |= 1u << (p * XP + j);
            }
        }
    }
    // (a: scalar copies of the arguments)
    static __device__ __forceinline__ void early(const GemvArgs &a, Pre &pre) {
        pre.valid = first_tile(a, pre.cur);
        if (!PM || !pre.valid) return;
        lazy_init(a, pre.lx);
        pre.lx.template look<FUSED_PM_CACHED ? P - 1 : 0>(LazyX::pass_mask(0));
        pre.resid = load_resid(a, pre.cur);
    }

    // Called by the predecessor right behind its last tile (which requested this phase's first
    // tile): takes the first pass of x and stages the residual.  Done there, in straight-line
    // code behind the requests, because the compiler counts outstanding loads per path: after
    // the merge with the path that requested nothing it would wait for every one of them.
    static __device__ __forceinline__ void settle(const GemvArgs &a, Pre &pre, FusedShared &sh, int *err) {
        if (!PM) return;   // (others look at their input when they start)
        pre.lx.await(LazyX::pass_mask(0), err);
        stage_resid(a, pre.cur, pre.resid, sh, err);
    }
    // The block's slice of the residual goes to LDS for the epilogues (visible to them after
    // the tile's barrier; the last phase that read this buffer lies at least one barrier back).
    static __device__ __forceinline__ void stage_resid(const GemvArgs &a, const Cursor &c, float r, FusedShared &sh, int *err) {
        const int tid = threadIdx.x;
        if (EPI == EPI_RESID && tid < 2 * (c.hi - c.lo)) {
            for (unsigned spins = 0; __float_as_uint(r) == ACT_UNSET; ++spins) {   // (never taken unset)
                if (spins > SPIN_LIMIT || ((spins & 255u) == 255u && __hip_atomic_load(as_global(err), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT))) {
                    __hip_atomic_store(as_global(err), 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                    break;
                }
                __builtin_amdgcn_s_sleep(INPUT_SLEEP);
                r = coherent_load(a.resid + 2 * c.lo + tid);
            }
            sh.epi[tid] = r;
        }
    }

    // One pass-major tile.  `first`: the block's first tile of the phase, where passes 1 .. P-1 of
    // x are still to be taken: each is looked at when the pass before it begins, so the answer
    // comes back behind that pass's weight requests and is there when the pass is reached; only
    // a pass that is still incomplete then is waited for.
    template <int MODE, typename Nx, int NXQ = 0>
    static __device__ __forceinline__ void tile_pm(const GemvArgs &a, const Cursor &c, const Cursor &n, int pos,
                                                   FusedShared &sh, u32x4 (&buf)[NBUF], float (&xr)[P][VEC], LazyX &lx, bool first,
                                                   int *err, const uint32_t (&coff)[P], int pb, const GemvArgs &na) {
        const int tid = threadIdx.x, lane = tid & (WAVE - 1), w = (tid / WAVE) % NW, g = tid / (WAVE * NW);
#pragma unroll
        for (int p = 0; p < P; ++p) {
            if (first) {
                if (p > 0) {
                    lx.await(LazyX::pass_mask(p), err);
                    lx.take(p, xr);
                }
                if (p + 1 < P) lx.template look<FUSED_PM_CACHED ? P - 1 : 0>(LazyX::pass_mask(p + 1));
            }
#pragma unroll
            for (int s = 0; s < U; ++s) {
                float f[VEC];
                Store<WT>::unpack(buf[s], f);
                float acc = 0.f;
#pragma unroll
                for (int v = 0; v < VEC; ++v) acc = fmaf(f[v], xr[p][v], acc);
                if (p + 1 < P) buf[s] = piece_sp(a, c.u0, c.hi, s, p + 1, coff);
                else if (MODE == 1) buf[s] = piece_sp(a, n.u0, n.hi, s, 0, coff);
                else if constexpr (MODE == 2) { if (s < NXQ) buf[s] = Nx::piece_for(na, n.u0, n.hi, s, coff[0]); }
                acc = wave_sum_last(acc);
                if (lane == WAVE - 1) sh.part[pb][g][p * U + s][w] = acc;
                }
        }
        __syncthreads();
        finish<P>(a, c.u0, c.lo, c.hi, pos, sh, pb);
    }

    // Runs the phase.  `ahead`: pieces [0, QI) of the block's first tile are in `buf` already
    // (prefetch); the others up to QD are requested here, a slice of SL between two looks at x.
    // `pb` (which of the two partial-sum buffers the next tile uses) runs on from phase to
    // phase: wave 0 may still be finishing the previous phase's last tile from the other one.
    // Nx, na_in, NXQ > 0: the phase that follows and how many pieces of its first tile this
    // phase's last tile requests (if `hand`), with `npre` left for its run(); AH > 0: this phase was set up
    // that way by its predecessor (`pre`), pieces [0, AH) of its first tile are on their way (a
    // pass-major phase: all of the tile, first pass of the input taken, residual staged).
    template <typename Nx, int NXQ, int AH>
    static __device__ __forceinline__ void run(const GemvArgs &a_in, int pos, FusedShared &sh, u32x4 (&buf)[NBUF],
                                               int &pb, bool ahead, int *err, const Prof &prof, unsigned point,
                                               const GemvArgs &na_in, bool hand, typename Nx::Pre *npre, Pre *pre) {
        constexpr bool PRE = PM && AH > 0;
        static_assert(!PM || AH == 0 || AH == NS, "a pass-major phase is handed over whole");
        static_assert(AH <= QD, "what is on its way is part of what goes out during the wait");
        const GemvArgs a = uniform(a_in);   // keep every address ingredient in scalar registers
        const int tid = threadIdx.x, lane = tid & (WAVE - 1), w = (tid / WAVE) % NW, g = tid / (WAVE * NW);
        Cursor cur;
        if (AH > 0) {
            if (!pre->valid) { prof.go(point); return; }
            cur = pre->cur;
        } else if (!first_tile(a, cur)) {
            if constexpr (NXQ > 0) {   // no unit of this phase: the next phase's first tile is requested at once
                const GemvArgs na = uniform(na_in);
                npre->valid = false;
                if (hand) Nx::early(na, *npre);
                if (npre->valid) {
                    const uint32_t coff0 = col_offset(a, 0);
#pragma unroll
                    for (int q = 0; q < NXQ; ++q) buf[q] = Nx::piece_for(na, npre->cur.u0, npre->cur.hi, q, coff0);
                    __syncthreads();   // (as run() has it before the residual is staged)
                    Nx::settle(na, *npre, sh, err);
                }
            }
            prof.go(point);
            return;
        }
        float rres = 0.f;
        if (EPI == EPI_RESID && !PRE) rres = load_resid(a, cur);
        // this lane's slice of x (RMS-normalised when a gain is given); the gain does not
        // depend on any activation, so its load goes out first
        uint32_t coff[P];
        u32x4 graw[P];
#pragma unroll
        for (int p = 0; p < P; ++p) {
            coff[p] = col_offset(a, p);
            if (a.gain != nullptr)   // clamped: lanes past the row end must stay inside the gain vector
                graw[p] = global_load16((const char *)a.gain + min(coff[p], (uint32_t)((a.cols - VEC) * sizeof(WT))));
        }
        // x: every 16-byte piece is loaded until none of its four words reads ACT_UNSET
        LazyX lx;
        if (PRE) lx = pre->lx;
        else lazy_init(a, lx);
        // what must be complete before the first tile can start: all of x, or its first pass
        constexpr unsigned NEED = PM ? LazyX::pass_mask(0) : ~0u;
        if (!PRE) {
            lx.template look<PM && FUSED_PM_CACHED ? P - 1 : 0>(NEED);
            // (SL0 pieces first, then SL at a time: an input that arrives soon after the phase
            // starts is seen by the look behind a short first slice)
#pragma unroll
            for (int q0 = 0; q0 < QD; q0 += (q0 == 0 ? SL0 : SL)) {
#pragma unroll
                for (int q = q0; q < q0 + (q0 == 0 ? SL0 : SL) && q < QD; ++q)
                    if (q >= AH && (q >= QI || !ahead)) buf[q] = piece(a, cur.u0, cur.hi, q, coff);
                if (__any((lx.pend & NEED) != 0)) {   // the look before this slice has come back: whatever is
                    lx.judge(NEED);          // still missing is asked for again, behind the slice
                    if (__any((lx.pend & NEED) != 0)) lx.look(NEED);
                }
            }
        }
        if (!PRE) lx.await(NEED, err);
        prof.go(point);
        if (!PRE && QD < NS) {   // the rest of the first tile
#pragma unroll
            for (int q = QD; q < NS; ++q) buf[q] = piece(a, cur.u0, cur.hi, q, coff);
        }
        float xr[P][VEC];
        if (PM) {
            lx.take(0, xr);
        } else {
#pragma unroll
            for (int p = 0; p < P; ++p) lx.take(p, xr);
        }
        if (EPI == EPI_RESID && !PRE) {
            __syncthreads();   // wave 0 may still be in the epilogue of the last phase that staged a slice
            stage_resid(a, cur, rres, sh, err);
        }
        if (!PM && a.gain != nullptr) {
            float ss = 0.f;
#pragma unroll
            for (int p = 0; p < P; ++p)
#pragma unroll
                for (int v = 0; v < VEC; ++v) ss += xr[p][v] * xr[p][v];
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
        Cursor nxt;
        bool first = true;
        for (; next_tile(a, cur, nxt); cur = nxt, pb ^= 1, first = false) {
            if constexpr (PM) tile_pm<1, Nx>(a, cur, nxt, pos, sh, buf, xr, lx, first, err, coff, pb, a);
            else tile<1, Nx>(a, cur, nxt, pos, sh, buf, xr, coff, pb, a);
        }
        bool handed = false;
        if constexpr (NXQ > 0) {
            const GemvArgs na = uniform(na_in);
            npre->valid = false;
            if (hand) Nx::early(na, *npre);
            if (npre->valid) {
                if constexpr (PM) tile_pm<2, Nx, NXQ>(a, cur, npre->cur, pos, sh, buf, xr, lx, first, err, coff, pb, na);
                else tile<2, Nx, NXQ>(a, cur, npre->cur, pos, sh, buf, xr, coff, pb, na);
                Nx::settle(na, *npre, sh, err);
                handed = true;
            }
        }
        if (!handed) {
            if constexpr (PM) tile_pm<0, Nx>(a, cur, cur, pos, sh, buf, xr, lx, first, err, coff, pb, a);
            else tile<0, Nx>(a, cur, cur, pos, sh, buf, xr, coff, pb, a);
        }
        pb ^= 1;
    }
};

struct FusedArgs {
    SuperposeArgs sup;
    const spd_layer_weights *layers;   // device array [n_layers]
    const void *final_norm, *lm_head;
    char *act;                         // arena 0; arena 1 starts arena_bytes later
    size_t arena_bytes;
    ActLayout al;
    float *logits;
    void *kv;                          // layer l: K at kv + 2 l kv_layer_bytes, V one kv_layer_bytes later
    size_t kv_layer_bytes;
    float *part;
    int32_t *counters;
    const double *inv_freq;
    long long *prof;                   // optional: every block stamps wall_clock64() around every synchronisation point
    unsigned *sync;
    int32_t n_layers, d_model, n_heads, n_kv_heads, d_ffn, vocab, cap_ctx, max_splits, head, kv_half;
    float eps;
};

__device__ __forceinline__ GemvArgs qkv_args(const FusedArgs &a, char *act, int l) {
    const int dh = a.d_model / a.n_heads;
    const int nq = a.n_heads * dh, nkv = a.n_kv_heads * dh;
    GemvArgs g{};
    const spd_layer_weights w = uniform(a.layers[l]);
    g.W = w.wqkv; g.gain = w.attn_norm; g.eps = a.eps; g.x = a.al.h_in(act, l); g.y = a.al.vec(act, l, a.al.q);
    g.rows = nq + 2 * nkv; g.cols = a.d_model;
    g.kcache = (char *)a.kv + (size_t)(2 * l) * a.kv_layer_bytes;
    g.vcache = (char *)a.kv + (size_t)(2 * l + 1) * a.kv_layer_bytes;
    g.inv_freq = a.inv_freq;
    g.n_q_rows = nq; g.n_kv_rows = nkv; g.d_head = dh; g.cap_ctx = a.cap_ctx;
    g.k_new = a.al.vec(act, l, a.al.kn); g.v_new = a.al.vec(act, l, a.al.vn);
    return g;
}

__device__ __forceinline__ GemvArgs head_args(const FusedArgs &a, char *act) {
    GemvArgs g{};
    g.W = a.lm_head; g.gain = a.final_norm; g.eps = a.eps; g.x = a.al.h_in(act, a.n_layers); g.y = a.logits;
    g.rows = a.vocab; g.cols = a.d_model;
    return g;
}

// PA / PB: passes a block needs to cover d_model / d_ffn columns.  Rows per tile follow from
// them so that a tile stays at about 16 pieces (16 bytes each) per lane.
constexpr int tile_rows(int passes) { return passes == 1 ? FUSED_UA : passes == 2 ? FUSED_UA / 2 : passes <= 4 ? 4 : 2; }

// KT: element type of the key/value cache (float, or half_t for a bf16 model that asked for it).
template <typename WT, typename KT, int PA, int PB>
__global__ __launch_bounds__(NT) void fused_forward_kernel(const FusedArgs a) {
    constexpr int UA = tile_rows(PA), UB = tile_rows(PB);
    // The O projection is one tile per block; its tile is a little taller so that it still is
    // when the blocks busy with attention items leave their rows to the others.
    constexpr int UO = UA + FUSED_UO_EXTRA / PA;
    constexpr int NA = PA * UO;
    // The down projection walks its tiles pass by pass, and the gate/up phase before it works in
    // chunks of one such pass, where d_model is one block pass wide and d_ffn several.
    constexpr bool PMD = PB >= 2 && PB <= 4;
    // (rows per tile: 16, or 20 where a block's 20 rows -- the 13B shape -- would otherwise spill into a second tile)
    constexpr int UPM = (PA == 2 && PB == 4) ? 20 : FUSED_UPM;
    constexpr int ND = PMD ? UPM : PB * UB;
    constexpr int NBUF = (NA > ND) ? NA : ND;
    constexpr int SL = PA == 1 ? FUSED_SLICE : FUSED_SLICE_WIDE;
    using Qkv = Gemv<WT, PA, UA, EPI_QKV, NBUF, SL, false, false, SL, KT>;
    using Oproj = Gemv<WT, PA, UO, EPI_RESID, NBUF, SL>;
    using GateUp = Gemv<WT, PA, UA, EPI_SWIGLU, NBUF, SL, false, PMD, FUSED_SLICE_GATE < SL ? FUSED_SLICE_GATE : SL>;
    using Down = Gemv<WT, PB, PMD ? UPM : UB, EPI_RESID, NBUF, SL, PMD>;
    using Head = Gemv<WT, PA, UA, EPI_PLAIN, NBUF, SL>;
    __shared__ FusedShared sh;
    __shared__ __align__(16) float dyn[NT * Store<KT>::VEC];

    DevState *st = a.sup.st;
    int *err = &st->err;
    const Prof prof{(a.prof && blockIdx.x < FUSED_PROF_BLOCKS) ? a.prof + (size_t)blockIdx.x * (size_t)(2 * (5 * a.n_layers + 2)) : nullptr};
    const int pos = uniform(as_global(st)->pos);
    const int dh = a.d_model / a.n_heads;
    const int nq = a.n_heads * dh;
    // The arenas alternate from launch to launch: block 0 leaves the number of launches behind
    // when it ends.
    const unsigned launch0 = (unsigned)uniform((int)__hip_atomic_load(as_global(a.sync) + SYNC_LAUNCH_WORD, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT));
    char *act = a.act + (size_t)(launch0 & 1u) * a.arena_bytes;
    const long long twin = (launch0 & 1u) ? -(long long)a.arena_bytes : (long long)a.arena_bytes;
    unsigned point = 0;   // synchronisation points passed: one after the input phase, five per layer
    int pb = 0;

    // phase 0: the input vector (Section 3.1, Eq. 1 and 2); every block keeps this position's
    // rotary table in LDS
    {
        SuperposeArgs sup = a.sup;
        sup.h = a.al.h_in(act, 0);
        sup.twin = twin;
        for (int c = blockIdx.x * NT + threadIdx.x; c < a.d_model; c += gridDim.x * NT)
            superpose_element<WT, true>(sup, c, pos);
    }
    if (threadIdx.x < dh / 2) sh.rope[threadIdx.x] = rope_cos_sin(a.inv_freq, threadIdx.x, pos);
    u32x4 buf[NBUF];
    prof.done(point);

    for (int l = 0; l < a.n_layers; ++l) {
        const spd_layer_weights w = uniform(a.layers[l]);
        float *q = a.al.vec(act, l, a.al.q), *att = a.al.vec(act, l, a.al.att), *h1 = a.al.vec(act, l, a.al.h1);
        float *u = a.al.vec(act, l, a.al.u), *h2 = a.al.vec(act, l, a.al.h2);
        GemvArgs cur = qkv_args(a, act, l);
        cur.twin = twin;
        Qkv::template run<Qkv, 0, 0>(cur, pos, sh, buf, pb, false, err, prof, point++, cur, false, nullptr, nullptr);
        prof.done(point);
        prof.go(point++);   // (nobody waits here: attention awaits its head's q, k, v as data)

        // Attention items: one per (query head, chunk of cached positions).  Up to
        // FUSED_ONE_CHUNK positions a head is ONE item (one or two batches of loads in one
        // block): a second batch costs about 2 us, merging chunks across blocks about 4 us (an
        // acknowledged store, an atomic and two dependent loads), but one compute unit's share
        // of the bandwidth makes a single block the slower choice past some 270 positions.
        // Longer contexts are cut so that every block gets an item if the chunk bounds allow.
        // While few blocks have an item those take no rows of the O projection: they would hold
        // everybody up fetching their tile after the attention.
        GemvArgs o{};
        o.W = w.wo; o.x = att; o.resid = a.al.h_in(act, l); o.y = h1; o.rows = a.d_model; o.cols = nq; o.twin = twin;
        const int n_ctx = pos + 1;
        constexpr int ONE_CHUNK = sizeof(KT) == 2 ? FUSED_ONE_CHUNK_HALF : FUSED_ONE_CHUNK;
        int chunk = ONE_CHUNK;
        if (n_ctx > ONE_CHUNK) {
            const int per_head = max(1, (int)gridDim.x / a.n_heads);
            chunk = ((n_ctx + per_head - 1) / per_head + 15) & ~15;
            chunk = min(ATTN_CHUNK_MAX, max(ATTN_CHUNK_MIN, chunk));
        }
        const int n_splits = (n_ctx + chunk - 1) / chunk;
        const int n_items = a.n_heads * n_splits;
        o.first_block = 4 * n_items <= (int)gridDim.x ? n_items : 0;
        const bool has_item = (int)blockIdx.x < n_items;
        if (has_item) {   // attention over pos + 1 cached positions with the head of the O-projection tile in flight
            Oproj::prefetch(o, buf);
            AttnArgs t{q, cur.kcache, cur.vcache, att, a.part, a.counters, nullptr, n_ctx,
                       a.n_heads, a.n_kv_heads, dh, a.cap_ctx, chunk, a.max_splits, twin, cur.k_new, cur.v_new};
            const int group = a.n_heads / a.n_kv_heads;
            for (int item = blockIdx.x; item < n_items; item += gridDim.x) {
                const int h = item / n_splits;
                // (the 13B class holds a 20-row pass-major tile in registers through the other phases and
                // spills with the full set: its items keep fewer cached rows in flight)
                constexpr bool TIGHT = PA == 2 && PMD;
                constexpr int R4 = TIGHT ? 8 : 10, R8_ONE = TIGHT ? 6 : FUSED_HALF_ROWS_ONE, R8_CUT = TIGHT ? 5 : FUSED_HALF_ROWS_CUT;
                if constexpr (sizeof(KT) == 2) {
                    if (n_ctx <= 16 * R4)   // one batch of 8-byte pieces
                        attn_item<half4_t, NT, true, R4>(t, h / group, item % n_splits, n_ctx, sh.sc, sh.red, dyn, &sh.s_last,
                                                         h % group, h % group + 1, err);
                    else if (n_splits == 1)
                        attn_item<half_t, NT, true, R8_ONE>(t, h / group, item % n_splits, n_ctx, sh.sc, sh.red, dyn, &sh.s_last,
                                                            h % group, h % group + 1, err);
                    else
                        attn_item<half_t, NT, true, R8_CUT>(t, h / group, item % n_splits, n_ctx, sh.sc, sh.red, dyn, &sh.s_last,
                                                            h % group, h % group + 1, err);
                } else {
                    attn_item<KT, NT, true, R4>(t, h / group, item % n_splits, n_ctx, sh.sc, sh.red, dyn, &sh.s_last,
                                                h % group, h % group + 1, err);
                }
            }
        }
        prof.done(point);
        Oproj::template run<Oproj, 0, 0>(o, pos, sh, buf, pb, has_item, err, prof, point++, o, false, nullptr, nullptr);
        prof.done(point);

        GemvArgs f{};
        f.W = w.w_gate; f.W2 = w.w_up; f.gain = w.ffn_norm; f.eps = a.eps; f.x = h1; f.y = u;
        f.rows = a.d_ffn; f.cols = a.d_model; f.twin = twin;
        f.chunk_span = PMD ? Down::PASS_COLS : 0;   // the chunks of u are the column passes of the down projection
        GemvArgs d{};
        d.W = w.w_down; d.x = u; d.resid = h1; d.y = h2; d.rows = a.d_model; d.cols = a.d_ffn; d.twin = twin;
        if constexpr (PMD) {
            // the last gate/up tile requests the first tile of the down projection, whose first
            // pass of input (the first chunk of u) has been complete since early in this phase
            typename Down::Pre dpre;
            GateUp::template run<Down, Down::NS, 0>(f, pos, sh, buf, pb, false, err, prof, point++, d, true, &dpre, nullptr);
            prof.done(point);
            Down::template run<Down, 0, Down::NS>(d, pos, sh, buf, pb, false, err, prof, point++, d, false, nullptr, &dpre);
        } else {
            GateUp::template run<GateUp, 0, 0>(f, pos, sh, buf, pb, false, err, prof, point++, f, false, nullptr, nullptr);
            prof.done(point);
            Down::template run<Down, 0, 0>(d, pos, sh, buf, pb, false, err, prof, point++, d, false, nullptr, nullptr);
        }
        prof.done(point);
    }
    if (a.head) Head::template run<Head, 0, 0>(head_args(a, act), pos, sh, buf, pb, false, err, prof, point, head_args(a, act), false, nullptr, nullptr);
    if (prof.p && threadIdx.x == 0) as_global(prof.p)[2 * (point + 1)] = wall_clock64();
    if (blockIdx.x == 0 && threadIdx.x == 0) {
        __hip_atomic_store(as_global(a.sync) + SYNC_LAUNCH_WORD, launch0 + 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
}

template <typename WT, typename KT, int PA, int PB> struct Variant {
    static hipError_t launch(hipStream_t s, const FusedArgs &a, int blocks) {
        hipLaunchKernelGGL((fused_forward_kernel<WT, KT, PA, PB>), dim3(blocks), dim3(NT), 0, s, a);
        return hipGetLastError();
    }
    static int blocks_per_cu() {
        int n = 0;
        if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&n, (const void *)fused_forward_kernel<WT, KT, PA, PB>, NT, 0) != hipSuccess) {
            (void)hipGetLastError();
            return 0;
        }
        return n;
    }
};

// The instantiations that exist: passes needed to cover d_model and d_ffn with NW waves
// (bf16: 4096 columns per pass).  (1,1) and (1,2): small models; (1,3): the Llama-2-7B shape;
// (2,4): 13B; (2,7): 70B.  Calls f(Variant<...>{}) for the one that serves the shape.
// The cache is fp32, or fp16 for a bf16 model that asked for it.
template <typename F>
bool with_variant(int dtype, int kv_half, int d_model, int d_ffn, F &&f) {
    const int vec = dtype == SPD_DTYPE_BF16 ? 8 : 4;
    const int span = NW * WAVE * vec;
    const int pa = (d_model + span - 1) / span, pb = (d_ffn + span - 1) / span;
    if (dtype == SPD_DTYPE_BF16 && kv_half) {
        if (pa == 1 && pb == 1) return f(Variant<bf16_t, half_t, 1, 1>{}), true;
        if (pa == 1 && pb == 2) return f(Variant<bf16_t, half_t, 1, 2>{}), true;
        if (pa == 1 && pb == 3) return f(Variant<bf16_t, half_t, 1, 3>{}), true;
        if (pa == 2 && pb == 4) return f(Variant<bf16_t, half_t, 2, 4>{}), true;
        if (pa == 2 && pb == 7) return f(Variant<bf16_t, half_t, 2, 7>{}), true;
    } else if (dtype == SPD_DTYPE_BF16) {
        if (pa == 1 && pb == 1) return f(Variant<bf16_t, float, 1, 1>{}), true;
        if (pa == 1 && pb == 2) return f(Variant<bf16_t, float, 1, 2>{}), true;
        if (pa == 1 && pb == 3) return f(Variant<bf16_t, float, 1, 3>{}), true;
        if (pa == 2 && pb == 4) return f(Variant<bf16_t, float, 2, 4>{}), true;
        if (pa == 2 && pb == 7) return f(Variant<bf16_t, float, 2, 7>{}), true;
    } else if (!kv_half) {
        if (pa == 1 && pb == 1) return f(Variant<float, float, 1, 1>{}), true;
        if (pa == 1 && pb == 2) return f(Variant<float, float, 1, 2>{}), true;
        if (pa == 1 && pb == 3) return f(Variant<float, float, 1, 3>{}), true;
    }
    return false;
}

}  // namespace

namespace spdk {

int fused_max_blocks_per_cu(int dtype, int kv_half, int d_model, int d_ffn) {
    int n = 0;
    with_variant(dtype, kv_half, d_model, d_ffn, [&](auto v) { n = decltype(v)::blocks_per_cu(); });
    return n;
}

hipError_t fused_forward(hipStream_t s, int dtype, const FusedArgsHost &h, int blocks) {
    FusedArgs a{};
    a.sup = h.sup; a.layers = h.layers; a.final_norm = h.final_norm; a.lm_head = h.lm_head;
    a.act = h.act; a.arena_bytes = h.arena_bytes; a.al = h.al; a.logits = h.logits;
    a.kv = h.kv; a.kv_layer_bytes = h.kv_layer_bytes; a.part = h.part; a.counters = h.counters;
    a.inv_freq = h.inv_freq; a.prof = h.prof; a.sync = h.sync;
    a.n_layers = h.n_layers; a.d_model = h.d_model; a.n_heads = h.n_heads; a.n_kv_heads = h.n_kv_heads;
    a.d_ffn = h.d_ffn; a.vocab = h.vocab; a.cap_ctx = h.cap_ctx; a.max_splits = h.max_splits; a.head = h.head;
    a.eps = h.eps; a.kv_half = h.kv_half;
    hipError_t e = hipErrorInvalidValue;
    with_variant(dtype, h.kv_half, h.d_model, h.d_ffn, [&](auto v) { e = decltype(v)::launch(s, a, blocks); });
    return e;
}

}  // namespace spdk
