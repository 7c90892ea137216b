// Dense prefix pass: the first-timestep forward over the prefix M (Section 3, "First
// Timestep") for a whole chunk of prefix tokens at once, so that the weights are read once per
// chunk instead of once per token.  Here the work IS a dense contraction, [tokens, d] x
// [rows, d]^T, and runs on the matrix cores (v_mfma_f32_32x32x16_bf16).
//
// Precision: the step path multiplies bf16 weights with fp32 activations.  To stay within
// rounding of it, an activation x is fed as two bf16 terms, hi = bf16(x) and lo = bf16(x - hi)
// (16 mantissa bits together), and W x = W hi + W lo is two matrix-core products into the same
// fp32 accumulator.  Feeding bf16(x) alone costs about 2e-2 of the logit scale over 32 layers.
//
// Operands need no transposition: with W row-major [rows, d] and activations [tokens, d], both
// MFMA operands are "row index in the lane, 8 consecutive k in the register", i.e. plain
// 16-byte pieces.  The k-index assignment inside a 64-wide k step is permuted (each half of the
// wave owns 32 consecutive k) so that a lane's four weight loads of a step are 64 contiguous
// bytes.
#include "spd_device.h"

using namespace spdd;

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

namespace {

// One element of the key/value cache (fp32, or fp16 rounded to nearest even).
__device__ __forceinline__ void kv_put(void *cache, int kv_half, size_t at, float v) {
    if (kv_half) Store<half_t>::store1(cache, at, v);
    else as_global((float *)cache)[at] = v;
}

constexpr int KSTEP = 64;         // k per pipeline step (4 MFMAs of k = 16)

__device__ __forceinline__ uint16_t bf16_rn(float v) {
    uint32_t u = __float_as_uint(v);
    u += 0x7FFFu + ((u >> 16) & 1u);
    return (uint16_t)(u >> 16);
}
__device__ __forceinline__ float bf16_f(uint16_t b) { return __uint_as_float((uint32_t)b << 16); }
// x = hi + lo up to 2^-17 |x|
__device__ __forceinline__ void split_store(uint16_t *hi, uint16_t *lo, size_t at, float x) {
    const uint16_t h = bf16_rn(x);
    as_global(hi)[at] = h;
    as_global(lo)[at] = bf16_rn(x - bf16_f(h));
}

// Where element (token t, feature k) of a [T, K] activation operand lives.  Row-major for the
// LDS-tiled GEMM; for the split-k GEMM of short chunks the operand is stored the way the matrix
// cores take it, so that every load of a wave is 1 KB contiguous: 32-token tile, then 64-wide
// k step, then the step's four 16-wide products j, then the lane (token t % 32 in lanes
// 0..31 for the step's first 32 k, in lanes 32..63 for the other 32), then 8 consecutive k.
__device__ __forceinline__ size_t act_at(bool tiled, int t, int k, int K) {
    if (!tiled) return (size_t)t * K + k;
    const int kk = k % KSTEP;
    return ((((size_t)(t / 32) * (K / KSTEP) + k / KSTEP) * 4 + (kk % 32) / 8) * WAVE + (t % 32) + 32 * (kk / 32)) * 8 + k % 8;
}

// ------------------------------------------------------------------ token rows, norms, rotary table
__global__ __launch_bounds__(256) void embed_rows_kernel(const uint16_t *embed, const int32_t *prefix, int p0, int T,
                                                         int d, float *H) {
    const int t = blockIdx.x;
    const int tok = as_global(prefix)[p0 + t];
    for (int c = threadIdx.x; c < d; c += 256) as_global(H)[(size_t)t * d + c] = bf16_f(as_global(embed)[(size_t)tok * d + c]);
}

// xn = x * rsqrt(mean x^2 + eps) * gain, written as the (hi, lo) pair.  One block per token; a
// thread keeps its runs of 8 consecutive features in registers (one read of the row) and
// writes each run as one 16-byte store per half (8 consecutive k are contiguous in both layouts).
constexpr int NORM_RUNS = 4;      // runs per thread: d_model <= 256 * 8 * NORM_RUNS

__global__ __launch_bounds__(256) void rmsnorm_split_kernel(const float *H, const uint16_t *gain, float eps, int d,
                                                            uint16_t *hi, uint16_t *lo, bool tiled) {
    __shared__ float red[256 / WAVE];
    const int t = blockIdx.x;
    const float *x = H + (size_t)t * d;
    float v[NORM_RUNS][8];
    float ss = 0.f;
#pragma unroll
    for (int i = 0; i < NORM_RUNS; ++i) {
        const int c = 8 * (threadIdx.x + 256 * i);
        if (c < d) {
            const float4 a = global_load_float4(x + c), b = global_load_float4(x + c + 4);
            v[i][0] = a.x; v[i][1] = a.y; v[i][2] = a.z; v[i][3] = a.w; v[i][4] = b.x; v[i][5] = b.y; v[i][6] = b.z; v[i][7] = b.w;
#pragma unroll
            for (int e = 0; e < 8; ++e) ss += v[i][e] * v[i][e];
        }
    }
    const float tot = block_sum<256>(ss, red);
    const float rs = 1.0f / sqrtf(tot / (float)d + eps);
#pragma unroll
    for (int i = 0; i < NORM_RUNS; ++i) {
        const int c = 8 * (threadIdx.x + 256 * i);
        if (c < d) {
            const u32x4 g = global_load16(gain + c);
            uint32_t h[4], l[4];
#pragma unroll
            for (int e = 0; e < 8; e += 2) {
                const uint32_t gw = e < 2 ? g.x : e < 4 ? g.y : e < 6 ? g.z : g.w;
                const float y0 = v[i][e] * rs * __uint_as_float(gw << 16), y1 = v[i][e + 1] * rs * __uint_as_float(gw & 0xFFFF0000u);
                const uint16_t h0 = bf16_rn(y0), h1 = bf16_rn(y1);
                h[e / 2] = (uint32_t)h0 | ((uint32_t)h1 << 16);
                l[e / 2] = (uint32_t)bf16_rn(y0 - bf16_f(h0)) | ((uint32_t)bf16_rn(y1 - bf16_f(h1)) << 16);
            }
            const size_t at = act_at(tiled, t, c, d);
            *(u32x4 __attribute__((address_space(1))) *)(hi + at) = u32x4{h[0], h[1], h[2], h[3]};
            *(u32x4 __attribute__((address_space(1))) *)(lo + at) = u32x4{l[0], l[1], l[2], l[3]};
        }
    }
}

// (cos, sin) of (p0 + t) * theta^(-2i/d_head), in double as everywhere else
__global__ void rope_table_kernel(const double *inv_freq, int p0, int T, int half, float2 *table) {
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= T * half) return;
    const float2 cs = rope_cos_sin(inv_freq, i % half, p0 + i / half);
    table[i] = cs;
}

// ------------------------------------------------------------------ GEMM on the matrix cores
enum { PE_RESID = 0, PE_QKV = 1, PE_SWIGLU = 2 };

struct PrefillGemmArgs {
    const uint16_t *xhi, *xlo;   // [T_pad, K] bf16 pair
    const uint16_t *W, *W2;      // [N, K] bf16; W2: the "up" matrix (PE_SWIGLU)
    int32_t T, N, K;
    // PE_RESID
    const float *resid;          // [T, N]
    float *out;                  // [T, N]
    // PE_QKV
    float *q;                    // [T, n_q_rows]
    void *kcache, *vcache;       // [n_kv_heads, cap_ctx, d_head] fp32, or fp16 (kv_half)
    int32_t kv_half;
    const float2 *rope;          // [T, d_head / 2]
    int32_t n_q_rows, n_kv_rows, d_head, cap_ctx, p0;
    // PE_SWIGLU
    uint16_t *uhi, *ulo;         // [T_pad, N]
    bool tiled;                  // layout of xhi / xlo and of uhi / ulo: see act_at
    int32_t t_tiles, n_tiles;    // tiled kernel: token tiles and column tiles of the launch
    float *ks_part;              // split-k kernel, k range halved between two blocks: their partial tiles
    int32_t *ks_count;           //   and one arrival count per tile (zero between launches)
};

// Block: one token tile (32 * TT tokens) and one column tile (32 * NWV columns);
// wave w owns columns [32 w, 32 w + 32) of it, all TT token tiles.  Per k step of 64:
//   * the activation tile (hi and lo, 32 TT rows x 64 k) is brought in ONCE per block through
//     LDS (every wave needs all of it; fetched per wave it saturates the L2),
//   * each wave fetches its 32 weight rows' 64 k coalesced (one load = 8 rows x 128 bytes) and turns
//     them into the operand layout (row in the lane) through a wave-private LDS tile; fetched in
//     that layout directly, every load touches 32 cache lines and the address path saturates,
//   * 8 TT (x 2 for gate and up) matrix-core products per wave.
// Both are double-buffered: the loads of step s + 1 are in flight during the products of
// step s.  Token rows past T are computed and dropped.
constexpr int A_ROW = KSTEP * 2 + 16;    // bytes per LDS row: 64 bf16 + 16 (rows 4 banks apart: conflict-free)

template <int EPI, int TT, int NWV>
__global__ __launch_bounds__(64 * NWV) void prefill_gemm_kernel(const PrefillGemmArgs a) {
    constexpr int NMAT = EPI == PE_SWIGLU ? 2 : 1;
    constexpr int NTH = 64 * NWV;
    constexpr int ROWS = 32 * TT;
    constexpr int PIECES = ROWS * 8;                       // 16-byte pieces of one (hi or lo) tile
    constexpr int PER_THREAD = (PIECES + NTH - 1) / NTH;   // staged per thread, per half
    extern __shared__ __align__(16) char a_lds[];          // [2 buffers][hi, lo][ROWS][A_ROW]
    const int tid = threadIdx.x, lane = tid & (WAVE - 1), w = tid / WAVE;
    // Workgroups go to the 8 XCDs round-robin and each XCD has its own L2: all token tiles of a
    // column tile are placed on one XCD, so a weight tile is fetched into one L2 only (the
    // activations, an order of magnitude smaller, are what every L2 holds).
    const int xcd = blockIdx.x % 8, slot_in_xcd = blockIdx.x / 8;
    const int tile_y = (slot_in_xcd / a.t_tiles) * 8 + xcd, tile_x = slot_in_xcd % a.t_tiles;
    if (tile_y >= a.n_tiles) return;
    const int t0 = tile_x * ROWS;
    f32x16 acc[NMAT][TT];
#pragma unroll
    for (int mt = 0; mt < NMAT; ++mt)
#pragma unroll
        for (int tt = 0; tt < TT; ++tt)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[mt][tt][r] = 0.f;

    // pieces on their way to LDS: two steps are in flight (one step's products are shorter than a
    // trip to memory), in two register slots
    u32x4 stage_hi[2][PER_THREAD], stage_lo[2][PER_THREAD], ws[2][NMAT][4];
    // weights, fetch side: load i of a step takes rows 8 i + lane / 8 of the wave's 32, piece lane % 8.
    // Addresses are a wave-uniform base (matrix + k offset, scalar registers) plus a 32-bit byte
    // offset per lane, computed once.
    uint32_t w_off[4], x_off[PER_THREAD];
#pragma unroll
    for (int i = 0; i < 4; ++i)
        w_off[i] = ((uint32_t)min(tile_y * (32 * NWV) + 32 * w + 8 * i + lane / 8, a.N - 1) * (uint32_t)a.K + 8 * (lane % 8)) * 2u;   // (ragged last tile: re-reads the last row)
#pragma unroll
    for (int i = 0; i < PER_THREAD; ++i) {
        const int p = min(tid + NTH * i, PIECES - 1);
        x_off[i] = ((uint32_t)(t0 + p / 8) * (uint32_t)a.K + 8 * (p % 8)) * 2u;
    }
    char *w_tile = a_lds + (size_t)2 * 2 * ROWS * A_ROW + (size_t)w * (NMAT * 32 * A_ROW);   // wave-private
    const int w_put = (lane / 8) * A_ROW + (lane % 8) * 16;           // + (mt * 32 + 8 i) * A_ROW
    const int w_get = (lane % 32) * A_ROW + (lane / 32) * 64;         // + mt * 32 * A_ROW + 16 j
    auto lds_at = [&](int buf, int half, int row, int piece) -> char * {
        return a_lds + (size_t)((buf * 2 + half) * ROWS + row) * A_ROW + piece * 16;
    };
#define FETCH_A(slot, k0)                                                                                      \
    _Pragma("unroll") for (int i = 0; i < PER_THREAD; ++i) {                                              \
        stage_hi[slot][i] = global_load16(a.xhi + (k0), x_off[i]);                                        \
        stage_lo[slot][i] = global_load16(a.xlo + (k0), x_off[i]);                                        \
    }
#define FETCH_W(slot, k0)                                                                                      \
    _Pragma("unroll") for (int i = 0; i < 4; ++i) {                                                       \
        ws[slot][0][i] = stream_load16(a.W + (k0), w_off[i]);                                             \
        if (NMAT == 2) ws[slot][1][i] = stream_load16(a.W2 + (k0), w_off[i]);                             \
    }
#define STORE_A(buf, slot)                                                                                   \
    _Pragma("unroll") for (int i = 0; i < PER_THREAD; ++i) {                                              \
        const int p = tid + NTH * i;                                                                      \
        if (PIECES % NTH == 0 || p < PIECES) {                                                            \
            *(u32x4 *)lds_at(buf, 0, p / 8, p % 8) = stage_hi[slot][i];                                     \
            *(u32x4 *)lds_at(buf, 1, p / 8, p % 8) = stage_lo[slot][i];                                     \
        }                                                                                                 \
    }
#define STORE_W(slot)                                                                                  \
    _Pragma("unroll") for (int mt = 0; mt < NMAT; ++mt)                                                   \
        _Pragma("unroll") for (int i = 0; i < 4; ++i)                                                     \
            *(u32x4 *)(w_tile + w_put + (mt * 32 + 8 * i) * A_ROW) = ws[slot][mt][i];
#define PRODUCTS(buf)                                                                                    \
    _Pragma("unroll") for (int j = 0; j < 4; ++j) {                                                       \
        bf16x8 wv[NMAT];                                                                                  \
        _Pragma("unroll") for (int mt = 0; mt < NMAT; ++mt)                                               \
            wv[mt] = __builtin_bit_cast(bf16x8, *(const u32x4 *)(w_tile + w_get + mt * 32 * A_ROW + 16 * j)); \
        _Pragma("unroll") for (int tt = 0; tt < TT; ++tt) {                                               \
            const bf16x8 xh = __builtin_bit_cast(bf16x8, *(const u32x4 *)lds_at(buf, 0, 32 * tt + lane % 32, 4 * (lane / 32) + j)); \
            const bf16x8 xl = __builtin_bit_cast(bf16x8, *(const u32x4 *)lds_at(buf, 1, 32 * tt + lane % 32, 4 * (lane / 32) + j)); \
            _Pragma("unroll") for (int mt = 0; mt < NMAT; ++mt) {                                         \
                acc[mt][tt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(xh, wv[mt], acc[mt][tt], 0, 0, 0); \
                acc[mt][tt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(xl, wv[mt], acc[mt][tt], 0, 0, 0); \
            }                                                                                             \
        }                                                                                                 \
    }

    // K is a multiple of two steps (the host checks): the loop body has no branch, and the
    // scheduling barriers keep the compiler from sinking a step's loads down to their first use.
    // The weight tile is private to its wave and the LDS serves a wave's accesses in order: the
    // tile of the next step is written behind the reads of this one without a barrier.
    const int k_last = a.K - KSTEP;
    FETCH_A(0, 0) FETCH_W(0, 0)
    FETCH_A(1, KSTEP) FETCH_W(1, KSTEP)
    STORE_A(0, 0) STORE_W(0)
    __syncthreads();
    for (int k0 = 0; k0 < a.K; k0 += 2 * KSTEP) {
        // LDS buffer 0 holds step k0, slot 1 (in flight) step k0 + 1; slot 0 is free
        FETCH_A(0, min(k0 + 2 * KSTEP, k_last)) FETCH_W(0, min(k0 + 2 * KSTEP, k_last))
        __builtin_amdgcn_sched_barrier(0);
        PRODUCTS(0)
        __builtin_amdgcn_sched_barrier(0);
        STORE_A(1, 1) STORE_W(1)
        __syncthreads();
        FETCH_A(1, min(k0 + 3 * KSTEP, k_last)) FETCH_W(1, min(k0 + 3 * KSTEP, k_last))
        __builtin_amdgcn_sched_barrier(0);
        PRODUCTS(1)
        __builtin_amdgcn_sched_barrier(0);
        STORE_A(0, 0) STORE_W(0)
        __syncthreads();
    }
#undef STORE_W
#undef FETCH_A
#undef FETCH_W
#undef STORE_A
#undef PRODUCTS

    // C layout: lane -> column nc = tile + lane % 32; register r -> token 8 (r / 4) + 4 (lane / 32) + r % 4
    const int nc = tile_y * (32 * NWV) + 32 * w + lane % 32;
#pragma unroll
    for (int tt = 0; tt < TT; ++tt)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            const int t = t0 + 32 * tt + 8 * (r / 4) + 4 * (lane / 32) + (r % 4);
            const float v = acc[0][tt][r];
            if (EPI == PE_QKV) {
                // rotary on (even, odd) column pairs: the partner sits in the neighbouring lane
                const float other = dpp_move<0xB1, 0xF>(v, 0.f);
                if (t < a.T && nc < a.N) {
                    if (nc < a.n_q_rows + a.n_kv_rows) {
                        const size_t ri = 2 * ((size_t)t * (a.d_head / 2) + (nc % a.d_head) / 2);
                        const float2 cs = make_float2(as_global((const float *)a.rope)[ri], as_global((const float *)a.rope)[ri + 1]);
                        const float rot = (nc & 1) ? __fadd_rn(__fmul_rn(other, cs.y), __fmul_rn(v, cs.x))
                                                   : __fsub_rn(__fmul_rn(v, cs.x), __fmul_rn(other, cs.y));
                        if (nc < a.n_q_rows) as_global(a.q)[(size_t)t * a.n_q_rows + nc] = rot;
                        else {
                            const int rr = nc - a.n_q_rows;
                            kv_put(a.kcache, a.kv_half, ((size_t)(rr / a.d_head) * a.cap_ctx + a.p0 + t) * a.d_head + rr % a.d_head, rot);
                        }
                    } else {
                        const int rr = nc - a.n_q_rows - a.n_kv_rows;
                        kv_put(a.vcache, a.kv_half, ((size_t)(rr / a.d_head) * a.cap_ctx + a.p0 + t) * a.d_head + rr % a.d_head, v);
                    }
                }
            } else if (t < a.T && nc < a.N) {
                if (EPI == PE_RESID) {
                    as_global(a.out)[(size_t)t * a.N + nc] = as_global(a.resid)[(size_t)t * a.N + nc] + v;
                } else {   // PE_SWIGLU: gate in acc[0], up in acc[1]
                    const float up = acc[NMAT - 1][tt][r];
                    split_store(a.uhi, a.ulo, (size_t)t * a.N + nc, v / (1.0f + expf(-v)) * up);
                }
            }
        }
}

// ------------------------------------------------------------------ few tokens: split-k GEMM
// With at most a few dozen tokens the product is bound by streaming the weights, and the tiling
// above leaves most of the chip idle (few blocks, one k sweep each).  Here a block owns 32
// weight rows and one 32-token tile, and its NWV waves split the k range between them: wave w
// takes the 64-wide k steps w, w + NWV, ...  No operand is shared between the waves:
//   * the weights are fetched coalesced (a wave's load = 8 rows x 128 bytes) and turned into
//     the matrix-core layout (row in the lane) through a wave-private LDS tile -- fetched in
//     that layout directly, every load touches 32 cache lines and the address path, not the
//     HBM, is the bound;
//   * the activations are stored in the matrix-core layout by their producers (act_at) and go
//     straight into registers, 1 KB contiguous per load, out of the L2.
// The waves' partial accumulators are summed through LDS in wave order (a fixed order: results
// do not vary from run to run), and the epilogue runs on the sums: wave w finishes accumulator
// registers w, w + NWV, ...
constexpr int W_ROW = KSTEP * 2 + 16;    // bytes per LDS row of the weight tile (as A_ROW)

// KS = 2: two blocks share a tile, each with half of the k steps (twice the blocks: the 128
// column tiles of a 4096-row matrix then fill 256 compute units, and 344 tiles spread more
// evenly); the block that finishes second adds the other's partial tile (a sum of two terms:
// the same whichever is second) and runs the epilogue.
template <int EPI, int NWV, int KS>
__global__ __launch_bounds__(64 * NWV) void prefill_skinny_kernel(const PrefillGemmArgs a) {
    constexpr int NMAT = EPI == PE_SWIGLU ? 2 : 1;
    constexpr int TILE = NMAT * 32 * W_ROW;                // one wave's weight tile(s)
    constexpr int NWE = NWV * KS;                          // waves that share the tile's k range
    constexpr int RPW = 16 / NWV;                          // accumulator registers a wave finishes
    extern __shared__ __align__(16) char a_lds[];          // weight tiles [NWV][TILE]; then float [NWV][NMAT][16][64]
    __shared__ int ks_second;
    float *red = (float *)a_lds;
    const int tid = threadIdx.x, lane = tid & (WAVE - 1), w = tid / WAVE;
    // Block order (KS = 1, several token tiles): workgroups go to the 8 XCDs round-robin, so the
    // token tiles of a column tile are 8 apart in the linear index: same XCD, started together,
    // and the second one finds the weight tile in that XCD's L2.
    const int n_col = (a.N + 31) / 32;
    const int grp = blockIdx.x / (8 * a.t_tiles), rem = blockIdx.x % (8 * a.t_tiles);
    const int ty = KS == 1 ? rem / 8 : 0;
    const int col_tile = KS == 1 ? grp * 8 + rem % 8 : (int)blockIdx.x / KS;
    const int half = KS == 1 ? 0 : (int)blockIdx.x % KS, we = w + NWV * half;
    if (col_tile >= n_col) return;
    const int t0 = ty * 32;
    const int S = a.K / KSTEP;
    const int n_w = we < S ? (S - we + NWE - 1) / NWE : 0;           // k steps of this wave
    f32x16 acc[NMAT];
#pragma unroll
    for (int mt = 0; mt < NMAT; ++mt)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[mt][r] = 0.f;

    // fetch side: load i of a step takes rows 8 i + lane / 8, 16-byte piece lane % 8
    size_t w_row[4];
#pragma unroll
    for (int i = 0; i < 4; ++i)
        w_row[i] = (size_t)min(col_tile * 32 + 8 * i + lane / 8, a.N - 1) * a.K + 8 * (lane % 8);   // (ragged last tile: re-reads the last row)
    char *tile = a_lds + (size_t)w * TILE;
    const int put = (lane / 8) * W_ROW + (lane % 8) * 16;            // + (mt * 32 + 8 i) * W_ROW
    const int get = (lane % 32) * W_ROW + (lane / 32) * 64;          // + mt * 32 * W_ROW + 16 j
    // Activations: one descriptor per half over this token tile's region (act_at order: step, j,
    // lane, 8 k).  Lanes whose token does not exist get an offset past the extent: zeros come
    // back and nothing is fetched, so a tile with few tokens costs few cache lines per load.
    const uint32_t tile_bytes = (uint32_t)S * (4 * WAVE * 8) * 2u;
    const __amdgpu_buffer_rsrc_t xh_rsrc = row_resource(a.xhi + (size_t)ty * S * (4 * WAVE * 8), tile_bytes);
    const __amdgpu_buffer_rsrc_t xl_rsrc = row_resource(a.xlo + (size_t)ty * S * (4 * WAVE * 8), tile_bytes);
    const bool token_exists = t0 + lane % 32 < a.T;
    const uint32_t x_lane = token_exists ? (uint32_t)lane * 16u : 0xFFFFFFF0u - 4u * (WAVE * 16u);   // (+ 3 j pieces stays past the extent, no wrap)

    u32x4 stage[2][NMAT][4], xh[2][4], xl[2][4];
#define FETCH_W(slot, i_)                                                                                \
    {                                                                                                     \
        const int k0 = KSTEP * min(we + NWE * (i_), S - 1);                                               \
        _Pragma("unroll") for (int i = 0; i < 4; ++i) {                                                   \
            stage[slot][0][i] = stream_load16(a.W + w_row[i] + k0);                                       \
            if (NMAT == 2) stage[slot][1][i] = stream_load16(a.W2 + w_row[i] + k0);                       \
        }                                                                                                 \
    }
#define FETCH_X(slot, i_)                                                                                \
    {                                                                                                     \
        const uint32_t at = (token_exists ? (uint32_t)min(we + NWE * (i_), S - 1) * (4 * WAVE * 16u) : 0u) + x_lane; \
        _Pragma("unroll") for (int j = 0; j < 4; ++j) {                                                   \
            xh[slot][j] = buffer_load16(xh_rsrc, at + j * (WAVE * 16u));                                  \
            xl[slot][j] = buffer_load16(xl_rsrc, at + j * (WAVE * 16u));                                  \
        }                                                                                                 \
    }
    // Step i: its weights (asked for two steps ago) go through the LDS tile; then the requests
    // of the coming steps -- activations of step i + 1 first, weights of step i + 2 behind them,
    // since a wave's loads complete in the order they were issued and the next step must not
    // have to wait for weights it does not need yet -- and the products of step i.
#define STEP(slot, i_)                                                                                   \
    {                                                                                                     \
        _Pragma("unroll") for (int mt = 0; mt < NMAT; ++mt)                                               \
            _Pragma("unroll") for (int i = 0; i < 4; ++i)                                                 \
                *(u32x4 *)(tile + put + (mt * 32 + 8 * i) * W_ROW) = stage[slot][mt][i];                  \
        __builtin_amdgcn_sched_barrier(0);                                                                \
        FETCH_X(1 - slot, (i_) + 1)                                                                       \
        FETCH_W(slot, (i_) + 2)                                                                           \
        __builtin_amdgcn_sched_barrier(0);                                                                \
        _Pragma("unroll") for (int j = 0; j < 4; ++j)                                                     \
            _Pragma("unroll") for (int mt = 0; mt < NMAT; ++mt) {                                         \
                const bf16x8 wv = __builtin_bit_cast(bf16x8, *(const u32x4 *)(tile + get + mt * 32 * W_ROW + 16 * j)); \
                acc[mt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, xh[slot][j]), wv, acc[mt], 0, 0, 0); \
                acc[mt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, xl[slot][j]), wv, acc[mt], 0, 0, 0); \
            }                                                                                             \
        __builtin_amdgcn_sched_barrier(0);                                                                \
    }
    // The tile is private to the wave and the LDS serves a wave's accesses in order: no barrier
    // inside the loop.  Loads are unconditional (clamped to the last step); a step past the
    // wave's share is skipped as a whole on a wave-uniform condition.
    FETCH_W(0, 0)
    FETCH_X(0, 0)
    FETCH_W(1, 1)
    for (int i = 0; i < n_w; i += 2) {
        STEP(0, i)
        if (i + 1 < n_w) STEP(1, i + 1)
    }
#undef FETCH_W
#undef FETCH_X
#undef STEP

    __syncthreads();                                       // every wave is done with its weight tile
#pragma unroll
    for (int mt = 0; mt < NMAT; ++mt)
#pragma unroll
        for (int r = 0; r < 16; ++r) red[((w * NMAT + mt) * 16 + r) * WAVE + lane] = acc[mt][r];
    __syncthreads();

    // C layout: lane -> column nc = tile + lane % 32; register r -> token 8 (r / 4) + 4 (lane / 32) + r % 4
    const int nc = col_tile * 32 + lane % 32;
    float sums[RPW][NMAT];
#pragma unroll
    for (int ri = 0; ri < RPW; ++ri)
#pragma unroll
        for (int mt = 0; mt < NMAT; ++mt) {
            sums[ri][mt] = 0.f;
            for (int ww = 0; ww < NWV; ++ww) sums[ri][mt] += red[((ww * NMAT + mt) * 16 + w + NWV * ri) * WAVE + lane];
        }
    if (KS == 2) {
        const size_t tile_lin = (size_t)col_tile;   // (KS = 2 runs with one token tile)
        float *mine = a.ks_part + ((tile_lin * 2 + half) * NMAT) * (16 * WAVE);
        const float *other = a.ks_part + ((tile_lin * 2 + (1 - half)) * NMAT) * (16 * WAVE);
#pragma unroll
        for (int ri = 0; ri < RPW; ++ri)
#pragma unroll
            for (int mt = 0; mt < NMAT; ++mt) act_store<true>(mine + (mt * 16 + w + NWV * ri) * WAVE + lane, sums[ri][mt]);
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");       // write-through stores acknowledged
        __syncthreads();
        if (tid == 0) {
            const int old = __hip_atomic_fetch_add(as_global(a.ks_count) + tile_lin, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            ks_second = old;
            if (old == 1) __hip_atomic_store(as_global(a.ks_count) + tile_lin, 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
        __syncthreads();
        if (!ks_second) return;
#pragma unroll
        for (int ri = 0; ri < RPW; ++ri)
#pragma unroll
            for (int mt = 0; mt < NMAT; ++mt) sums[ri][mt] += coherent_load(other + (mt * 16 + w + NWV * ri) * WAVE + lane);
    }
#pragma unroll
    for (int ri = 0; ri < RPW; ++ri) {
        const int r = w + NWV * ri;
        float sum[NMAT];
#pragma unroll
        for (int mt = 0; mt < NMAT; ++mt) sum[mt] = sums[ri][mt];
        const int t = t0 + 8 * (r / 4) + 4 * (lane / 32) + (r % 4);
        const float v = sum[0];
        if (EPI == PE_QKV) {
            const float other = dpp_move<0xB1, 0xF>(v, 0.f);   // rotary partner: the neighbouring column
            if (t < a.T && nc < a.N) {
                if (nc < a.n_q_rows + a.n_kv_rows) {
                    const size_t ri = 2 * ((size_t)t * (a.d_head / 2) + (nc % a.d_head) / 2);
                    const float cs_x = as_global((const float *)a.rope)[ri], cs_y = as_global((const float *)a.rope)[ri + 1];
                    const float rot = (nc & 1) ? __fadd_rn(__fmul_rn(other, cs_y), __fmul_rn(v, cs_x))
                                               : __fsub_rn(__fmul_rn(v, cs_x), __fmul_rn(other, cs_y));
                    if (nc < a.n_q_rows) as_global(a.q)[(size_t)t * a.n_q_rows + nc] = rot;
                    else {
                        const int rr = nc - a.n_q_rows;
                        kv_put(a.kcache, a.kv_half, ((size_t)(rr / a.d_head) * a.cap_ctx + a.p0 + t) * a.d_head + rr % a.d_head, rot);
                    }
                } else {
                    const int rr = nc - a.n_q_rows - a.n_kv_rows;
                    kv_put(a.vcache, a.kv_half, ((size_t)(rr / a.d_head) * a.cap_ctx + a.p0 + t) * a.d_head + rr % a.d_head, v);
                }
            }
        } else if (t < a.T && nc < a.N) {
            if (EPI == PE_RESID) {
                as_global(a.out)[(size_t)t * a.N + nc] = as_global(a.resid)[(size_t)t * a.N + nc] + v;
            } else {   // PE_SWIGLU: gate in sum[0], up in sum[1]
                const float up = sum[NMAT - 1];
                split_store(a.uhi, a.ulo, act_at(true, t, nc, a.N), v / (1.0f + expf(-v)) * up);
            }
        }
    }
}

// ------------------------------------------------------------------ causal attention over the chunk
// Four (two) consecutive elements of the key/value cache, element type KT, from element `at`.
template <typename KT> __device__ __forceinline__ float4 kv_load4(const void *base, size_t at);
template <> __device__ __forceinline__ float4 kv_load4<float>(const void *base, size_t at) { return global_load_float4((const float *)base + at); }
template <> __device__ __forceinline__ float4 kv_load4<half_t>(const void *base, size_t at) {
    typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
    typedef _Float16 h2 __attribute__((ext_vector_type(2)));
    const u32x2 w = *(const u32x2 __attribute__((address_space(1))) *)((const uint16_t *)base + at);
    const uint32_t x = w.x, y = w.y;   // (bit casts of copies, not of the vector's elements)
    const h2 lo = __builtin_bit_cast(h2, x), hi = __builtin_bit_cast(h2, y);
    return make_float4((float)lo.x, (float)lo.y, (float)hi.x, (float)hi.y);
}
template <typename KT> __device__ __forceinline__ float2 kv_load2(const void *base, size_t at);
template <> __device__ __forceinline__ float2 kv_load2<float>(const void *base, size_t at) {
    return make_float2(as_global((const float *)base)[at], as_global((const float *)base)[at + 1]);
}
template <> __device__ __forceinline__ float2 kv_load2<half_t>(const void *base, size_t at) {
    typedef _Float16 h2 __attribute__((ext_vector_type(2)));
    const uint32_t x = *(const uint32_t __attribute__((address_space(1))) *)((const uint16_t *)base + at);
    const h2 v = __builtin_bit_cast(h2, x);
    return make_float2((float)v.x, (float)v.y);
}
// One block: one query head, AQ queries of the chunk; keys / values streamed through LDS in
// chunks of AK cached positions (cache elements of type KT, widened on load), online softmax.  Output as the (hi, lo) pair.
constexpr int ANT = 256, AQ = 32, AK = 64;

struct PrefillAttnArgs {
    const float *q;               // [T, n_heads * d_head]
    const void *kcache, *vcache;  // [n_kv_heads, cap_ctx, d_head] in the kernel's KT
    uint16_t *ohi, *olo;          // [T_pad, n_heads * d_head]
    int32_t T, p0, n_heads, n_kv_heads, d_head, cap_ctx;
    bool tiled;                   // layout of ohi / olo: see act_at
};

template <typename KT>
__global__ __launch_bounds__(ANT) void prefill_attn_kernel(const PrefillAttnArgs a) {
    extern __shared__ __align__(16) float lds[];
    // row strides: 16-byte aligned, and consecutive rows 4 banks apart (no conflicts for the
    // 8 rows the 8 threads of a query read side by side)
    const int dh = a.d_head, ldk = dh + 4, lds_s = AK + 1;
    float *Qs = lds;                       // [AQ][dh + 4]
    float *Ks = Qs + AQ * ldk;             // [AK][dh + 4]
    float *Vs = Ks + AK * ldk;             // [AK][dh]
    float *Ss = Vs + AK * dh;              // [AQ][AK + 1]
    const int tid = threadIdx.x;
    const int h = blockIdx.y, g = h / (a.n_heads / a.n_kv_heads);
    const int q0 = blockIdx.x * AQ;
    const int nqd = a.n_heads * dh, dh4 = dh / 4;
    const float scale = 1.0f / sqrtf((float)dh);
    for (int e = tid; e < AQ * dh4; e += ANT) {
        const int i = e / dh4, c = 4 * (e % dh4), t = q0 + i;
        float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
        if (t < a.T) v = global_load_float4(a.q + (size_t)t * nqd + (size_t)h * dh + c);
        *(float4 *)(Qs + i * ldk + c) = v;
    }
    const int qi = tid / 8, sub = tid % 8;          // this thread's query, and its share of keys / dims
    const int qpos = a.p0 + q0 + qi;                // cached positions 0 .. qpos are visible
    float m = -INFINITY, l = 0.f;
    float4 acc[4];                                  // dims 4 (sub + 8 g4) .. + 3, g4 = 0 .. 3 (d_head <= 128)
#pragma unroll
    for (int g4 = 0; g4 < 4; ++g4) acc[g4] = make_float4(0.f, 0.f, 0.f, 0.f);
    const int last = min(a.p0 + q0 + AQ - 1, a.p0 + a.T - 1);   // last position any query of the tile sees
    const size_t head_at = (size_t)g * a.cap_ctx * dh;
    for (int c0 = 0; c0 <= last; c0 += AK) {
        __syncthreads();
        for (int e = tid; e < AK * dh4; e += ANT) {
            const int j = e / dh4, c = 4 * (e % dh4), pos = c0 + j;
            float4 kv = make_float4(0.f, 0.f, 0.f, 0.f), vv = kv;
            if (pos <= last) {
                kv = kv_load4<KT>(a.kcache, head_at + (size_t)pos * dh + c);
                vv = kv_load4<KT>(a.vcache, head_at + (size_t)pos * dh + c);
            }
            *(float4 *)(Ks + j * ldk + c) = kv;
            *(float4 *)(Vs + j * dh + c) = vv;
        }
        __syncthreads();
        // scores of query qi with keys sub + 8 jj
        float s[8], cmax = -INFINITY;
#pragma unroll
        for (int jj = 0; jj < 8; ++jj) s[jj] = 0.f;
        for (int d = 0; d < dh; d += 4) {
            const float4 qv = *(const float4 *)(Qs + qi * ldk + d);
#pragma unroll
            for (int jj = 0; jj < 8; ++jj) {
                const float4 kv = *(const float4 *)(Ks + (sub + 8 * jj) * ldk + d);
                s[jj] = fmaf(qv.x, kv.x, s[jj]); s[jj] = fmaf(qv.y, kv.y, s[jj]);
                s[jj] = fmaf(qv.z, kv.z, s[jj]); s[jj] = fmaf(qv.w, kv.w, s[jj]);
            }
        }
#pragma unroll
        for (int jj = 0; jj < 8; ++jj) {
            const int pos = c0 + sub + 8 * jj;
            s[jj] = pos <= qpos ? s[jj] * scale : -INFINITY;
            cmax = fmaxf(cmax, s[jj]);
        }
        // the 8 threads of a query sit in consecutive lanes
        cmax = fmaxf(cmax, __shfl_xor(cmax, 1, WAVE));
        cmax = fmaxf(cmax, __shfl_xor(cmax, 2, WAVE));
        cmax = fmaxf(cmax, __shfl_xor(cmax, 4, WAVE));
        const float m_new = fmaxf(m, cmax);
        float psum = 0.f;
#pragma unroll
        for (int jj = 0; jj < 8; ++jj) {
            const float p = m_new == -INFINITY ? 0.f : expf(s[jj] - m_new);
            Ss[qi * lds_s + sub + 8 * jj] = p;
            psum += p;
        }
        psum += __shfl_xor(psum, 1, WAVE);
        psum += __shfl_xor(psum, 2, WAVE);
        psum += __shfl_xor(psum, 4, WAVE);
        const float corr = m == -INFINITY ? 0.f : expf(m - m_new);
        l = l * corr + psum;
        m = m_new;
        __syncthreads();
#pragma unroll
        for (int g4 = 0; g4 < 4; ++g4) { acc[g4].x *= corr; acc[g4].y *= corr; acc[g4].z *= corr; acc[g4].w *= corr; }
        for (int j = 0; j < AK; ++j) {
            const float p = Ss[qi * lds_s + j];
#pragma unroll
            for (int g4 = 0; g4 < 4; ++g4)
                if (4 * (sub + 8 * g4) < dh) {
                    const float4 v = *(const float4 *)(Vs + j * dh + 4 * (sub + 8 * g4));
                    acc[g4].x = fmaf(p, v.x, acc[g4].x); acc[g4].y = fmaf(p, v.y, acc[g4].y);
                    acc[g4].z = fmaf(p, v.z, acc[g4].z); acc[g4].w = fmaf(p, v.w, acc[g4].w);
                }
        }
    }
    const int t = q0 + qi;
    if (t < a.T) {
#pragma unroll
        for (int g4 = 0; g4 < 4; ++g4)
            if (4 * (sub + 8 * g4) < dh) {
                const size_t at = act_at(a.tiled, t, h * dh + 4 * (sub + 8 * g4), nqd);   // 4 consecutive k share a run of 8
                split_store(a.ohi, a.olo, at, acc[g4].x / l); split_store(a.ohi, a.olo, at + 1, acc[g4].y / l);
                split_store(a.ohi, a.olo, at + 2, acc[g4].z / l); split_store(a.ohi, a.olo, at + 3, acc[g4].w / l);
            }
    }
}

// The same attention on the matrix cores, in fp32 (v_mfma_f32_32x32x2_f32: exact fp32 products,
// as on the step path), for d_head 64 and 128.  One block: 32 queries of one head; its four
// waves share the cached positions between them (wave w takes the 32-key tiles w, w + 4, ...),
// each flash-style (running maximum and sum per query), and their partial results are merged
// through LDS at the end.  Both products are formed transposed, so that a query lives in a
// lane from start to end:
//   S^T [key, query] = K [key, d] Q^T [d, query]      -- d_head / 2 products
//   O^T [d, query]  += V^T [d, key] P^T [key, query]  -- 16 products per 32 features d; tile dt holds
//                                                        features {(d_head / 32) rho + dt}, so that a lane
//                                                        reads a key's values as one 16-byte piece
// The accumulator layout (lane = column, register r = row 8 (r / 4) + 4 (lane / 32) + r % 4)
// of S^T is, register by register, the operand layout the second product wants for P^T when
// its k index (step i, lane half h) stands for key 8 (i / 4) + 4 h + i % 4: the probabilities
// never leave their registers.  For the first product k index (i, h) stands for feature
// (d_head / 2) h + i, so a lane reads half a row of K as contiguous 16-byte pieces.
// Q sits in LDS in operand order; K and V come straight from the cache into the same registers,
// one after the other, which keeps a wave under half the register file: two waves share a
// SIMD and one computes while the other waits for its loads.
template <int DH, typename KT>
__global__ __launch_bounds__(256, 2) void prefill_attn_mfma_kernel(const PrefillAttnArgs a) {
    constexpr int HALF = DH / 2, NT = DH / 32, NWV = 4;
    constexpr int SLOT = (2 + 16 * NT) * WAVE;               // one wave's partial result: m, sum, O^T
    __shared__ float q_lds[HALF * WAVE];
    __shared__ float merge[2 * SLOT];
    const int lane = threadIdx.x & (WAVE - 1), w = threadIdx.x / WAVE, h = lane / 32, c = lane % 32;
    // Workgroups go to the 8 XCDs round-robin: all query tiles of a head are placed on one XCD (its
    // L2 then holds that head's keys and values once), the tiles that see the most keys first.
    const int q_tiles = (a.T + 31) / 32;
    const int xcd = blockIdx.x % 8, slot_in_xcd = blockIdx.x / 8;
    const int head = (slot_in_xcd / q_tiles) * 8 + xcd;
    if (head >= a.n_heads) return;
    const int kvh = head / (a.n_heads / a.n_kv_heads);
    const int q0 = (q_tiles - 1 - slot_in_xcd % q_tiles) * 32;
    const int nqd = a.n_heads * DH;
    const float scale = 1.0f / sqrtf((float)DH);
    if (w == 0) {   // this lane's operand values of Q: query q0 + c (clamped), features HALF h + i
        const float *qrow = a.q + (size_t)min(q0 + c, a.T - 1) * nqd + (size_t)head * DH + HALF * h;
#pragma unroll
        for (int i = 0; i < HALF; i += 4) {
            const float4 v = global_load_float4(qrow + i);
            q_lds[(i + 0) * WAVE + lane] = v.x; q_lds[(i + 1) * WAVE + lane] = v.y;
            q_lds[(i + 2) * WAVE + lane] = v.z; q_lds[(i + 3) * WAVE + lane] = v.w;
        }
    }
    const size_t head_at = (size_t)kvh * a.cap_ctx * DH;
    const int qpos = a.p0 + q0 + c;                          // cached positions 0 .. qpos are visible to this lane's query
    const int last_key = a.p0 + min(q0 + 31, a.T - 1);       // last position any query of the tile sees
    float m = -INFINITY, lsum = 0.f;
    f32x16 o[NT];
#pragma unroll
    for (int dt = 0; dt < NT; ++dt)
#pragma unroll
        for (int r = 0; r < 16; ++r) o[dt][r] = 0.f;
    __syncthreads();                                         // Q is in place

    for (int k0 = 32 * w; k0 <= last_key; k0 += 32 * NWV) {
        f32x16 st;
#pragma unroll
        for (int r = 0; r < 16; ++r) st[r] = 0.f;
        {
            float kreg[HALF];
            const size_t krow = head_at + (size_t)min(k0 + c, last_key) * DH + HALF * h;
#pragma unroll
            for (int i = 0; i < HALF; i += 4) {
                const float4 v = kv_load4<KT>(a.kcache, krow + i);
                kreg[i] = v.x; kreg[i + 1] = v.y; kreg[i + 2] = v.z; kreg[i + 3] = v.w;
            }
#pragma unroll
            for (int i = 0; i < HALF; ++i) st = __builtin_amdgcn_mfma_f32_32x32x2f32(kreg[i], q_lds[i * WAVE + lane], st, 0, 0, 0);
        }
        __builtin_amdgcn_sched_barrier(0);
        // V of this tile: requested once K's registers are free (a second wave on the same
        // SIMD covers the wait), in flight during the softmax
        float vreg[NT][16];
#pragma unroll
        for (int i = 0; i < 16; ++i) {   // one 16-byte piece per key: features NT c .. NT c + NT - 1, one for each product tile
            const size_t vrow = head_at + (size_t)min(k0 + 8 * (i / 4) + 4 * h + i % 4, last_key) * DH + NT * c;
            if (NT == 4) {
                const float4 v = kv_load4<KT>(a.vcache, vrow);
                vreg[0][i] = v.x; vreg[1][i] = v.y; vreg[2][i] = v.z; vreg[3 % NT][i] = v.w;
            } else {
                const float2 v = kv_load2<KT>(a.vcache, vrow);
                vreg[0][i] = v.x; vreg[1 % NT][i] = v.y;
            }
        }
        __builtin_amdgcn_sched_barrier(0);
        float mx = m;
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            const int key = k0 + 8 * (r / 4) + 4 * h + r % 4;
            st[r] = key <= qpos ? st[r] * scale : -INFINITY;
            mx = fmaxf(mx, st[r]);
        }
        mx = fmaxf(mx, __shfl_xor(mx, 32));                  // the other half of the keys
        // a query that sees none of this tile's keys and none before it: keep exp() away from inf - inf
        const float ref = mx == -INFINITY ? 0.f : mx;
        const float alpha = expf(m - ref);
        float psum = 0.f;
#pragma unroll
        for (int r = 0; r < 16; ++r) { st[r] = expf(st[r] - ref); psum += st[r]; }
        lsum = lsum * alpha + psum;
        m = mx;
#pragma unroll
        for (int dt = 0; dt < NT; ++dt) {
#pragma unroll
            for (int r = 0; r < 16; ++r) o[dt][r] *= alpha;
#pragma unroll
            for (int i = 0; i < 16; ++i) o[dt] = __builtin_amdgcn_mfma_f32_32x32x2f32(vreg[dt][i], st[i], o[dt], 0, 0, 0);
        }
        __builtin_amdgcn_sched_barrier(0);
    }

    // merge: waves 2, 3 -> waves 0, 1; wave 1 -> wave 0.  Wave 0 holds key 0, visible to every
    // query, so the merged maximum is finite.
    auto put = [&](int slot) {
        float *b = merge + slot * SLOT;
        b[lane] = m; b[WAVE + lane] = lsum;
#pragma unroll
        for (int dt = 0; dt < NT; ++dt)
#pragma unroll
            for (int r = 0; r < 16; ++r) b[(2 + 16 * dt + r) * WAVE + lane] = o[dt][r];
    };
    auto take = [&](int slot) {
        const float *b = merge + slot * SLOT;
        const float m2 = b[lane], mt = fmaxf(m, m2);
        const float ref = mt == -INFINITY ? 0.f : mt;
        const float f1 = expf(m - ref), f2 = expf(m2 - ref);
        lsum = lsum * f1 + b[WAVE + lane] * f2;
#pragma unroll
        for (int dt = 0; dt < NT; ++dt)
#pragma unroll
            for (int r = 0; r < 16; ++r) o[dt][r] = o[dt][r] * f1 + b[(2 + 16 * dt + r) * WAVE + lane] * f2;
        m = mt;
    };
    if (w >= 2) put(w - 2);
    __syncthreads();
    if (w < 2) take(w);
    __syncthreads();
    if (w == 1) put(0);
    __syncthreads();
    if (w != 0) return;
    take(0);
    lsum += __shfl_xor(lsum, 32);
    const int t = q0 + c;
    if (t < a.T) {
        const float inv = 1.0f / lsum;
#pragma unroll
        for (int r = 0; r < 16; ++r) {                       // row rho of product tile dt is feature NT rho + dt
            const size_t at = act_at(a.tiled, t, head * DH + NT * (8 * (r / 4) + 4 * h + r % 4), nqd);
#pragma unroll
            for (int dt = 0; dt < NT; ++dt) split_store(a.ohi, a.olo, at + dt, o[dt][r] * inv);
        }
    }
}

}  // namespace

namespace spdk {

size_t prefill_attn_lds(int d_head) { return (size_t)(AQ * (d_head + 4) + AK * (d_head + 4) + AK * d_head + AQ * (AK + 1)) * sizeof(float); }

// Launch with the widest column tile that still gives every compute unit a block.
constexpr int GEMM_TT = 2;
constexpr int SWIGLU_TT = 2;  // the same for gate and up side by side

static size_t skinny_lds(int nmat, int nwv) {
    const size_t tiles = (size_t)nwv * nmat * 32 * W_ROW, red = (size_t)nwv * nmat * 16 * 64 * sizeof(float);
    return tiles > red ? tiles : red;
}
constexpr int SKINNY_MAX_T = 96;      // up to here the split-k kernel is the faster one

template <int EPI, int TT>
static void launch_gemm(hipStream_t s, const PrefillGemmArgs &g, int num_cu) {
    if (g.tiled) {
        // one 32-token tile: halve the k range between two blocks (more, smaller blocks balance better)
        PrefillGemmArgs a = g;
        a.t_tiles = (g.T + 31) / 32;
        const int n_col = (g.N + 31) / 32;
        if (a.t_tiles == 1 && g.ks_part != nullptr)
            hipLaunchKernelGGL((prefill_skinny_kernel<EPI, 8, 2>), dim3(2 * n_col), dim3(512), skinny_lds(EPI == PE_SWIGLU ? 2 : 1, 8), s, a);
        else
            hipLaunchKernelGGL((prefill_skinny_kernel<EPI, 8, 1>), dim3(((n_col + 7) / 8) * 8 * a.t_tiles), dim3(512), skinny_lds(EPI == PE_SWIGLU ? 2 : 1, 8), s, a);
        return;
    }
    const int t_tiles = (g.T + 32 * TT - 1) / (32 * TT);
    const int nmat = EPI == PE_SWIGLU ? 2 : 1;
    auto lds_of = [&](int nwv) { return (size_t)(2 * 2 * (32 * TT) + nwv * nmat * 32) * A_ROW; };
    auto blocks = [&](int nwv) { return t_tiles * ((g.N + 32 * nwv - 1) / (32 * nwv)); };
    PrefillGemmArgs a = g;
    a.t_tiles = t_tiles;
    auto launch = [&](auto kernel, int nwv) {
        a.n_tiles = (g.N + 32 * nwv - 1) / (32 * nwv);
        hipLaunchKernelGGL(kernel, dim3(t_tiles * ((a.n_tiles + 7) / 8) * 8), dim3(64 * nwv), lds_of(nwv), s, a);
    };
    if (blocks(4) >= num_cu) launch(prefill_gemm_kernel<EPI, TT, 4>, 4);
    else if (blocks(2) >= num_cu) launch(prefill_gemm_kernel<EPI, TT, 2>, 2);
    else launch(prefill_gemm_kernel<EPI, TT, 1>, 1);
}

hipError_t prefill_init() {
    hipError_t e = hipFuncSetAttribute((const void *)prefill_attn_kernel<float>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)prefill_attn_lds(128));
    if (e == hipSuccess) e = hipFuncSetAttribute((const void *)prefill_attn_kernel<half_t>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)prefill_attn_lds(128));
    const int big = (2 * 2 * 128 + 4 * 2 * 32) * A_ROW;     // at least what any instantiation asks for
#define SPD_LDS(K, B) if (e == hipSuccess) e = hipFuncSetAttribute((const void *)(K), hipFuncAttributeMaxDynamicSharedMemorySize, B)
    SPD_LDS((prefill_gemm_kernel<PE_QKV, GEMM_TT, 4>), big); SPD_LDS((prefill_gemm_kernel<PE_QKV, GEMM_TT, 2>), big); SPD_LDS((prefill_gemm_kernel<PE_QKV, GEMM_TT, 1>), big);
    SPD_LDS((prefill_gemm_kernel<PE_RESID, GEMM_TT, 4>), big); SPD_LDS((prefill_gemm_kernel<PE_RESID, GEMM_TT, 2>), big); SPD_LDS((prefill_gemm_kernel<PE_RESID, GEMM_TT, 1>), big);
    SPD_LDS((prefill_gemm_kernel<PE_SWIGLU, SWIGLU_TT, 4>), big); SPD_LDS((prefill_gemm_kernel<PE_SWIGLU, SWIGLU_TT, 2>), big); SPD_LDS((prefill_gemm_kernel<PE_SWIGLU, SWIGLU_TT, 1>), big);
    SPD_LDS((prefill_skinny_kernel<PE_QKV, 8, 1>), (int)skinny_lds(1, 8)); SPD_LDS((prefill_skinny_kernel<PE_QKV, 8, 2>), (int)skinny_lds(1, 8));
    SPD_LDS((prefill_skinny_kernel<PE_RESID, 8, 1>), (int)skinny_lds(1, 8)); SPD_LDS((prefill_skinny_kernel<PE_RESID, 8, 2>), (int)skinny_lds(1, 8));
    SPD_LDS((prefill_skinny_kernel<PE_SWIGLU, 8, 1>), (int)skinny_lds(2, 8)); SPD_LDS((prefill_skinny_kernel<PE_SWIGLU, 8, 2>), (int)skinny_lds(2, 8));
#undef SPD_LDS
    return e;
}

// One chunk of T prefix tokens at positions p0 .. p0 + T - 1 through the whole stack.  On
// return (stream order) A.h holds the residual stream after the last layer and the caches are
// extended; the caller finishes the last token (final norm + LM head).
hipError_t prefill_chunk(hipStream_t s, const PrefillChunk &c) {
    const int T = c.T, d = c.d_model, dh = d / c.n_heads, nq = c.n_heads * dh, nkv = c.n_kv_heads * dh;
    hipLaunchKernelGGL(embed_rows_kernel, dim3(T), dim3(256), 0, s, (const uint16_t *)c.embed, c.prefix, c.p0, T, d, c.h);
    hipLaunchKernelGGL(rope_table_kernel, dim3((T * (dh / 2) + 255) / 256), dim3(256), 0, s, c.inv_freq, c.p0, T, dh / 2, c.rope);
    float *h = c.h, *h1 = c.h1;
    const bool tiled = T <= SKINNY_MAX_T;      // short chunk: split-k GEMMs, operands in their layout
    for (int l = 0; l < c.n_layers; ++l) {
        const spd_layer_weights &w = c.layers[l];
        hipLaunchKernelGGL(rmsnorm_split_kernel, dim3(T), dim3(256), 0, s, h, (const uint16_t *)w.attn_norm, c.eps, d, c.xhi, c.xlo, tiled);
        PrefillGemmArgs g{};
        g.xhi = c.xhi; g.xlo = c.xlo; g.W = (const uint16_t *)w.wqkv; g.T = T; g.N = nq + 2 * nkv; g.K = d;
        g.q = c.q; g.kcache = c.kv + (size_t)(2 * l) * c.kv_layer_bytes;
        g.vcache = c.kv + (size_t)(2 * l + 1) * c.kv_layer_bytes; g.kv_half = c.kv_half;
        g.tiled = tiled; g.ks_part = c.ks_part; g.ks_count = c.ks_count; g.rope = c.rope; g.n_q_rows = nq; g.n_kv_rows = nkv; g.d_head = dh; g.cap_ctx = c.cap_ctx; g.p0 = c.p0;
        launch_gemm<PE_QKV, GEMM_TT>(s, g, c.num_cu);

        PrefillAttnArgs at{c.q, g.kcache, g.vcache, c.xhi, c.xlo, T, c.p0, c.n_heads, c.n_kv_heads, dh, c.cap_ctx, tiled};
        const dim3 mfma_grid(((T + 31) / 32) * ((c.n_heads + 7) / 8) * 8), plain_grid((T + AQ - 1) / AQ, c.n_heads);
        if (c.kv_half) {
            if (dh == 128) hipLaunchKernelGGL((prefill_attn_mfma_kernel<128, half_t>), mfma_grid, dim3(256), 0, s, at);
            else if (dh == 64) hipLaunchKernelGGL((prefill_attn_mfma_kernel<64, half_t>), mfma_grid, dim3(256), 0, s, at);
            else hipLaunchKernelGGL(prefill_attn_kernel<half_t>, plain_grid, dim3(ANT), prefill_attn_lds(dh), s, at);
        } else {
            if (dh == 128) hipLaunchKernelGGL((prefill_attn_mfma_kernel<128, float>), mfma_grid, dim3(256), 0, s, at);
            else if (dh == 64) hipLaunchKernelGGL((prefill_attn_mfma_kernel<64, float>), mfma_grid, dim3(256), 0, s, at);
            else hipLaunchKernelGGL(prefill_attn_kernel<float>, plain_grid, dim3(ANT), prefill_attn_lds(dh), s, at);
        }

        PrefillGemmArgs o{};
        o.xhi = c.xhi; o.xlo = c.xlo; o.W = (const uint16_t *)w.wo; o.T = T; o.N = d; o.K = nq; o.resid = h; o.out = h1; o.tiled = tiled; o.ks_part = c.ks_part; o.ks_count = c.ks_count;
        launch_gemm<PE_RESID, GEMM_TT>(s, o, c.num_cu);

        hipLaunchKernelGGL(rmsnorm_split_kernel, dim3(T), dim3(256), 0, s, h1, (const uint16_t *)w.ffn_norm, c.eps, d, c.xhi, c.xlo, tiled);
        PrefillGemmArgs f{};
        f.xhi = c.xhi; f.xlo = c.xlo; f.W = (const uint16_t *)w.w_gate; f.W2 = (const uint16_t *)w.w_up; f.T = T; f.N = c.d_ffn; f.K = d;
        f.uhi = c.uhi; f.ulo = c.ulo; f.tiled = tiled; f.ks_part = c.ks_part; f.ks_count = c.ks_count;
        launch_gemm<PE_SWIGLU, SWIGLU_TT>(s, f, c.num_cu);

        PrefillGemmArgs dn{};
        dn.xhi = c.uhi; dn.xlo = c.ulo; dn.W = (const uint16_t *)w.w_down; dn.T = T; dn.N = d; dn.K = c.d_ffn; dn.resid = h1; dn.out = h; dn.tiled = tiled; dn.ks_part = c.ks_part; dn.ks_count = c.ks_count;
        launch_gemm<PE_RESID, GEMM_TT>(s, dn, c.num_cu);
    }
    return hipGetLastError();
}

}  // namespace spdk
