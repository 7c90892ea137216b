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
// Operands need no LDS staging: with W row-major [rows, d] and activations [tokens, d], both
// MFMA operands are "row index in the lane, 8 consecutive k in the register", i.e. plain
// 16-byte loads.  The k-index assignment inside a 64-wide k step is permuted (each half of the
// wave owns 32 consecutive k) so that a lane's four loads of a step are 64 contiguous bytes.
#include "spd_device.h"

using namespace spdd;

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

namespace {

constexpr int GNT = 256;          // threads per GEMM block: 4 waves, each 32 columns of a 128-column tile
constexpr int G_NB = 128;         // columns (weight rows) per block
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

// ------------------------------------------------------------------ token rows, norms, rotary table
__global__ __launch_bounds__(256) void embed_rows_kernel(const uint16_t *embed, const int32_t *prefix, int p0, int T,
                                                         int d, float *H) {
    const int t = blockIdx.x;
    const int tok = as_global(prefix)[p0 + t];
    for (int c = threadIdx.x; c < d; c += 256) as_global(H)[(size_t)t * d + c] = bf16_f(as_global(embed)[(size_t)tok * d + c]);
}

// xn = x * rsqrt(mean x^2 + eps) * gain, written as the (hi, lo) pair
__global__ __launch_bounds__(256) void rmsnorm_split_kernel(const float *H, const uint16_t *gain, float eps, int d,
                                                            uint16_t *hi, uint16_t *lo) {
    __shared__ float red[256 / WAVE];
    const int t = blockIdx.x;
    const float *x = H + (size_t)t * d;
    float ss = 0.f;
    for (int c = threadIdx.x; c < d; c += 256) { const float v = as_global(x)[c]; ss += v * v; }
    const float tot = block_sum<256>(ss, red);
    const float rs = 1.0f / sqrtf(tot / (float)d + eps);
    for (int c = threadIdx.x; c < d; c += 256)
        split_store(hi, lo, (size_t)t * d + c, as_global(x)[c] * rs * bf16_f(as_global(gain)[c]));
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
    float *kcache, *vcache;      // [n_kv_heads, cap_ctx, d_head] fp32
    const float2 *rope;          // [T, d_head / 2]
    int32_t n_q_rows, n_kv_rows, d_head, cap_ctx, p0;
    // PE_SWIGLU
    uint16_t *uhi, *ulo;         // [T_pad, N]
};

template <int NMAT>
struct Frags {                    // one k step: 4 pieces of 8 k each
    u32x4 a_hi[2][4], a_lo[2][4]; // two token tiles
    u32x4 b[NMAT][4];
};

template <int TT, int NMAT>
__device__ __forceinline__ void load_step(const PrefillGemmArgs &a, Frags<NMAT> &f, int t0, int n, int k0, int lane) {
    const size_t koff = (size_t)k0 + 32 * (lane / 32);
#pragma unroll
    for (int tt = 0; tt < TT; ++tt) {
        const size_t row = (size_t)(t0 + 32 * tt + lane % 32) * a.K + koff;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            f.a_hi[tt][j] = global_load16(a.xhi + row + 8 * j);
            f.a_lo[tt][j] = global_load16(a.xlo + row + 8 * j);
        }
    }
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        f.b[0][j] = stream_load16(a.W + (size_t)n * a.K + koff + 8 * j);
        if (NMAT == 2) f.b[1][j] = stream_load16(a.W2 + (size_t)n * a.K + koff + 8 * j);
    }
}

template <int TT, int NMAT>
__device__ __forceinline__ void mma_step(const Frags<NMAT> &f, f32x16 (&acc)[NMAT][2]) {
#pragma unroll
    for (int j = 0; j < 4; ++j)
#pragma unroll
        for (int mt = 0; mt < NMAT; ++mt) {
            const bf16x8 b = __builtin_bit_cast(bf16x8, f.b[mt][j]);
#pragma unroll
            for (int tt = 0; tt < TT; ++tt) {
                acc[mt][tt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, f.a_hi[tt][j]), b, acc[mt][tt], 0, 0, 0);
                acc[mt][tt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, f.a_lo[tt][j]), b, acc[mt][tt], 0, 0, 0);
            }
        }
}

// Block: token tile blockIdx.x (32 * TT tokens), column tile blockIdx.y (128 columns); wave w
// owns columns [32 w, 32 w + 32) of it.  Token rows past T are computed and dropped.
template <int EPI, int TT>
__global__ __launch_bounds__(GNT, 2) void prefill_gemm_kernel(const PrefillGemmArgs a) {
    constexpr int NMAT = EPI == PE_SWIGLU ? 2 : 1;
    const int lane = threadIdx.x & (WAVE - 1), w = threadIdx.x / WAVE;
    const int t0 = blockIdx.x * 32 * TT;
    const int n = blockIdx.y * G_NB + 32 * w + lane % 32;      // this lane's weight row (load side)
    const int nl = min(n, a.N - 1);                              // (a ragged last tile re-reads the last row)
    f32x16 acc[NMAT][2];
#pragma unroll
    for (int mt = 0; mt < NMAT; ++mt)
#pragma unroll
        for (int tt = 0; tt < 2; ++tt)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[mt][tt][r] = 0.f;
    // Two steps in flight.  K is a multiple of two steps (the host checks), so the loop body has
    // no branch at all: a load or a product under a branch makes the compiler wait for
    // everything outstanding.  Past the end the last step is simply requested again.
    Frags<NMAT> f0, f1;
    const int k_last = a.K - KSTEP;
    load_step<TT, NMAT>(a, f0, t0, nl, 0, lane);
    for (int k0 = 0; k0 < a.K; k0 += 2 * KSTEP) {
        // (the scheduling barriers keep the compiler from sinking a step's loads down to their
        // first use, which would put a memory latency in front of every product)
        load_step<TT, NMAT>(a, f1, t0, nl, k0 + KSTEP, lane);
        __builtin_amdgcn_sched_barrier(0);
        mma_step<TT, NMAT>(f0, acc);
        __builtin_amdgcn_sched_barrier(0);
        load_step<TT, NMAT>(a, f0, t0, nl, min(k0 + 2 * KSTEP, k_last), lane);
        __builtin_amdgcn_sched_barrier(0);
        mma_step<TT, NMAT>(f1, acc);
        __builtin_amdgcn_sched_barrier(0);
    }

    // C layout: lane -> column nc = tile + lane % 32; register r -> token 8 (r / 4) + 4 (lane / 32) + r % 4
    const int nc = blockIdx.y * G_NB + 32 * w + lane % 32;
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
                            as_global(a.kcache)[((size_t)(rr / a.d_head) * a.cap_ctx + a.p0 + t) * a.d_head + rr % a.d_head] = rot;
                        }
                    } else {
                        const int rr = nc - a.n_q_rows - a.n_kv_rows;
                        as_global(a.vcache)[((size_t)(rr / a.d_head) * a.cap_ctx + a.p0 + t) * a.d_head + rr % a.d_head] = v;
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

// ------------------------------------------------------------------ causal attention over the chunk
// One block: one query head, AQ queries of the chunk; keys / values streamed through LDS in
// chunks of AK cached positions (fp32 cache), online softmax.  Output as the (hi, lo) pair.
constexpr int ANT = 256, AQ = 32, AK = 64;

struct PrefillAttnArgs {
    const float *q;               // [T, n_heads * d_head]
    const float *kcache, *vcache; // [n_kv_heads, cap_ctx, d_head]
    uint16_t *ohi, *olo;          // [T_pad, n_heads * d_head]
    int32_t T, p0, n_heads, n_kv_heads, d_head, cap_ctx;
};

__global__ __launch_bounds__(ANT) void prefill_attn_kernel(const PrefillAttnArgs a) {
    extern __shared__ float lds[];
    const int dh = a.d_head, ldk = dh + 1, lds_s = AK + 1;   // (odd row strides: no LDS bank conflicts)
    float *Qs = lds;                       // [AQ][dh + 1]
    float *Ks = Qs + AQ * ldk;             // [AK][dh + 1]
    float *Vs = Ks + AK * ldk;             // [AK][dh]
    float *Ss = Vs + AK * dh;              // [AQ][AK + 1]
    const int tid = threadIdx.x;
    const int h = blockIdx.y, g = h / (a.n_heads / a.n_kv_heads);
    const int q0 = blockIdx.x * AQ;
    const int nqd = a.n_heads * dh;
    const float scale = 1.0f / sqrtf((float)dh);
    for (int e = tid; e < AQ * dh; e += ANT) {
        const int i = e / dh, t = q0 + i;
        Qs[i * ldk + e % dh] = t < a.T ? as_global(a.q)[(size_t)t * nqd + (size_t)h * dh + e % dh] : 0.f;
    }
    const int qi = tid / 8, sub = tid % 8;          // this thread's query, and its share of keys / dims
    const int qpos = a.p0 + q0 + qi;                // cached positions 0 .. qpos are visible
    float m = -INFINITY, l = 0.f, acc[16];          // dims sub + 8 dd (d_head <= 128)
#pragma unroll
    for (int dd = 0; dd < 16; ++dd) acc[dd] = 0.f;
    const int last = min(a.p0 + q0 + AQ - 1, a.p0 + a.T - 1);   // last position any query of the tile sees
    const float *Kg = a.kcache + (size_t)g * a.cap_ctx * dh, *Vg = a.vcache + (size_t)g * a.cap_ctx * dh;
    for (int c0 = 0; c0 <= last; c0 += AK) {
        __syncthreads();
        for (int e = tid; e < AK * dh; e += ANT) {
            const int j = e / dh, d = e % dh, pos = c0 + j;
            const bool ok = pos <= last;
            Ks[j * ldk + d] = ok ? as_global(Kg)[(size_t)pos * dh + d] : 0.f;
            Vs[j * dh + d] = ok ? as_global(Vg)[(size_t)pos * dh + d] : 0.f;
        }
        __syncthreads();
        // scores of query qi with keys sub + 8 jj
        float s[8], cmax = -INFINITY;
#pragma unroll
        for (int jj = 0; jj < 8; ++jj) s[jj] = 0.f;
        for (int d = 0; d < dh; ++d) {
            const float qv = Qs[qi * ldk + d];
#pragma unroll
            for (int jj = 0; jj < 8; ++jj) s[jj] = fmaf(qv, Ks[(sub + 8 * jj) * ldk + d], s[jj]);
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
        const float m_new = fmaxf(m, cmax);          // finite: position c0 <= qpos whenever this chunk matters
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
        for (int dd = 0; dd < 16; ++dd) acc[dd] *= corr;
        for (int j = 0; j < AK; ++j) {
            const float p = Ss[qi * lds_s + j];
#pragma unroll
            for (int dd = 0; dd < 16; ++dd)
                if (sub + 8 * dd < dh) acc[dd] = fmaf(p, Vs[j * dh + sub + 8 * dd], acc[dd]);
        }
    }
    const int t = q0 + qi;
    if (t < a.T) {
#pragma unroll
        for (int dd = 0; dd < 16; ++dd)
            if (sub + 8 * dd < dh) split_store(a.ohi, a.olo, (size_t)t * nqd + (size_t)h * dh + sub + 8 * dd, acc[dd] / l);
    }
}

}  // namespace

namespace spdk {

size_t prefill_attn_lds(int d_head) { return (size_t)(AQ * (d_head + 1) + AK * (d_head + 1) + AK * d_head + AQ * (AK + 1)) * sizeof(float); }

hipError_t prefill_init() {
    return hipFuncSetAttribute((const void *)prefill_attn_kernel, hipFuncAttributeMaxDynamicSharedMemorySize, (int)prefill_attn_lds(128));
}

// One chunk of T prefix tokens at positions p0 .. p0 + T - 1 through the whole stack.  On
// return (stream order) A.h holds the residual stream after the last layer and the caches are
// extended; the caller finishes the last token (final norm + LM head).
hipError_t prefill_chunk(hipStream_t s, const PrefillChunk &c) {
    const int T = c.T, d = c.d_model, dh = d / c.n_heads, nq = c.n_heads * dh, nkv = c.n_kv_heads * dh;
    const int tt2 = (T + 63) / 64, tt1 = (T + 31) / 32;
    hipLaunchKernelGGL(embed_rows_kernel, dim3(T), dim3(256), 0, s, (const uint16_t *)c.embed, c.prefix, c.p0, T, d, c.h);
    hipLaunchKernelGGL(rope_table_kernel, dim3((T * (dh / 2) + 255) / 256), dim3(256), 0, s, c.inv_freq, c.p0, T, dh / 2, c.rope);
    float *h = c.h, *h1 = c.h1;
    for (int l = 0; l < c.n_layers; ++l) {
        const spd_layer_weights &w = c.layers[l];
        hipLaunchKernelGGL(rmsnorm_split_kernel, dim3(T), dim3(256), 0, s, h, (const uint16_t *)w.attn_norm, c.eps, d, c.xhi, c.xlo);
        PrefillGemmArgs g{};
        g.xhi = c.xhi; g.xlo = c.xlo; g.W = (const uint16_t *)w.wqkv; g.T = T; g.N = nq + 2 * nkv; g.K = d;
        g.q = c.q; g.kcache = (float *)(c.kv + (size_t)(2 * l) * c.kv_layer_bytes);
        g.vcache = (float *)(c.kv + (size_t)(2 * l + 1) * c.kv_layer_bytes);
        g.rope = c.rope; g.n_q_rows = nq; g.n_kv_rows = nkv; g.d_head = dh; g.cap_ctx = c.cap_ctx; g.p0 = c.p0;
        hipLaunchKernelGGL((prefill_gemm_kernel<PE_QKV, 2>), dim3(tt2, (g.N + G_NB - 1) / G_NB), dim3(GNT), 0, s, g);

        PrefillAttnArgs at{c.q, g.kcache, g.vcache, c.xhi, c.xlo, T, c.p0, c.n_heads, c.n_kv_heads, dh, c.cap_ctx};
        hipLaunchKernelGGL(prefill_attn_kernel, dim3((T + AQ - 1) / AQ, c.n_heads), dim3(ANT), prefill_attn_lds(dh), s, at);

        PrefillGemmArgs o{};
        o.xhi = c.xhi; o.xlo = c.xlo; o.W = (const uint16_t *)w.wo; o.T = T; o.N = d; o.K = nq; o.resid = h; o.out = h1;
        hipLaunchKernelGGL((prefill_gemm_kernel<PE_RESID, 2>), dim3(tt2, (o.N + G_NB - 1) / G_NB), dim3(GNT), 0, s, o);

        hipLaunchKernelGGL(rmsnorm_split_kernel, dim3(T), dim3(256), 0, s, h1, (const uint16_t *)w.ffn_norm, c.eps, d, c.xhi, c.xlo);
        PrefillGemmArgs f{};
        f.xhi = c.xhi; f.xlo = c.xlo; f.W = (const uint16_t *)w.w_gate; f.W2 = (const uint16_t *)w.w_up; f.T = T; f.N = c.d_ffn; f.K = d;
        f.uhi = c.uhi; f.ulo = c.ulo;
        hipLaunchKernelGGL((prefill_gemm_kernel<PE_SWIGLU, 1>), dim3(tt1, (f.N + G_NB - 1) / G_NB), dim3(GNT), 0, s, f);

        PrefillGemmArgs dn{};
        dn.xhi = c.uhi; dn.xlo = c.ulo; dn.W = (const uint16_t *)w.w_down; dn.T = T; dn.N = d; dn.K = c.d_ffn; dn.resid = h1; dn.out = h;
        hipLaunchKernelGGL((prefill_gemm_kernel<PE_RESID, 2>), dim3(tt2, (dn.N + G_NB - 1) / G_NB), dim3(GNT), 0, s, dn);
    }
    return hipGetLastError();
}

}  // namespace spdk
