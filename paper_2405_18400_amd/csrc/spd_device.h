// Device-side helpers shared by the HIP kernels of libspd (gfx950, wave64).
#pragma once
#include "spd_internal.h"

#include <climits>
#include <cmath>

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

namespace spdd {

constexpr int WAVE = 64;

// ------------------------------------------------------------------ storage types
struct bf16_t { uint16_t b; };

struct half_t { uint16_t b; };   // IEEE binary16 (key/value cache of bf16 models, if asked for)
struct half4_t { uint16_t b; };

template <typename T> struct Store;
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
template <> struct Store<float> {
    static constexpr int VEC = 4;  // elements per 16-byte load
    typedef u32x4 piece_t;
    static __device__ __forceinline__ void unpack(const u32x4 v, float *f) {
        f[0] = __uint_as_float(v.x); f[1] = __uint_as_float(v.y);
        f[2] = __uint_as_float(v.z); f[3] = __uint_as_float(v.w);
    }
    static __device__ __forceinline__ float load1(const void *p, size_t i) { return ((const float __attribute__((address_space(1))) *)p)[i]; }
    static __device__ __forceinline__ void store1(void *p, size_t i, float v) { ((float __attribute__((address_space(1))) *)p)[i] = v; }
    static __device__ __forceinline__ void store1_coherent(void *p, size_t i, float v) {
        __hip_atomic_store((float __attribute__((address_space(1))) *)p + i, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
};
template <> struct Store<bf16_t> {
    static constexpr int VEC = 8;
    typedef u32x4 piece_t;
    static __device__ __forceinline__ void unpack(const u32x4 v, float *f) {
        f[0] = __uint_as_float(v.x << 16); f[1] = __uint_as_float(v.x & 0xFFFF0000u);
        f[2] = __uint_as_float(v.y << 16); f[3] = __uint_as_float(v.y & 0xFFFF0000u);
        f[4] = __uint_as_float(v.z << 16); f[5] = __uint_as_float(v.z & 0xFFFF0000u);
        f[6] = __uint_as_float(v.w << 16); f[7] = __uint_as_float(v.w & 0xFFFF0000u);
    }
    static __device__ __forceinline__ float load1(const void *p, size_t i) {
        return __uint_as_float((uint32_t)((const uint16_t __attribute__((address_space(1))) *)p)[i] << 16);
    }
    static __device__ __forceinline__ void store1(void *p, size_t i, float v) {
        uint32_t u = __float_as_uint(v);               // round to nearest even
        u += 0x7FFFu + ((u >> 16) & 1u);
        ((uint16_t __attribute__((address_space(1))) *)p)[i] = (uint16_t)(u >> 16);
    }
    static __device__ __forceinline__ void store1_coherent(void *p, size_t i, float v) {
        uint32_t u = __float_as_uint(v);
        u += 0x7FFFu + ((u >> 16) & 1u);
        __hip_atomic_store((uint16_t __attribute__((address_space(1))) *)p + i, (uint16_t)(u >> 16), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
};

template <> struct Store<half_t> {
    static constexpr int VEC = 8;
    typedef u32x4 piece_t;
    typedef _Float16 h2 __attribute__((ext_vector_type(2)));
    static __device__ __forceinline__ void unpack(const u32x4 v, float *f) {
        // (bit casts of copies: cast straight from a vector's element, every one reads element 0)
        const uint32_t x = v.x, y = v.y, z = v.z, w = v.w;
        const h2 a = __builtin_bit_cast(h2, x), b = __builtin_bit_cast(h2, y);
        const h2 c = __builtin_bit_cast(h2, z), d = __builtin_bit_cast(h2, w);
        f[0] = (float)a.x; f[1] = (float)a.y; f[2] = (float)b.x; f[3] = (float)b.y;
        f[4] = (float)c.x; f[5] = (float)c.y; f[6] = (float)d.x; f[7] = (float)d.y;
    }
    static __device__ __forceinline__ uint16_t bits(float v) { return __builtin_bit_cast(uint16_t, (_Float16)v); }   // round to nearest even
    static __device__ __forceinline__ float load1(const void *p, size_t i) {
        return (float)__builtin_bit_cast(_Float16, ((const uint16_t __attribute__((address_space(1))) *)p)[i]);
    }
    static __device__ __forceinline__ void store1(void *p, size_t i, float v) {
        ((uint16_t __attribute__((address_space(1))) *)p)[i] = bits(v);
    }
    static __device__ __forceinline__ void store1_coherent(void *p, size_t i, float v) {
        __hip_atomic_store((uint16_t __attribute__((address_space(1))) *)p + i, bits(v), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
};

// The same cache read four elements (8 bytes) per lane: the lane layout of an fp32 cache.
template <> struct Store<half4_t> {
    static constexpr int VEC = 4;
    typedef u32x2 piece_t;
    typedef _Float16 h2 __attribute__((ext_vector_type(2)));
    static __device__ __forceinline__ void unpack(const u32x2 v, float *f) {
        const uint32_t x = v.x, y = v.y;
        const h2 a = __builtin_bit_cast(h2, x), b = __builtin_bit_cast(h2, y);
        f[0] = (float)a.x; f[1] = (float)a.y; f[2] = (float)b.x; f[3] = (float)b.y;
    }
};

// Pointers that reach a kernel inside structures or through memory are "generic" to the
// compiler, and generic loads are slower than global ones here in a way that matters: they
// also count as LDS traffic, so every LDS wait would drain the weight stream.  Everything
// this library reads in bulk is global memory, and says so.
template <typename T> using global_ptr = T __attribute__((address_space(1))) *;
template <typename T> __device__ __forceinline__ global_ptr<T> as_global(T *p) { return (global_ptr<T>)p; }
typedef const u32x4 __attribute__((address_space(1))) *global_u32x4_ptr;
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef const f32x4 __attribute__((address_space(1))) *global_f32x4_ptr;

// Weight rows are streamed with raw buffer loads: a row is described by a resource descriptor
// in scalar registers (built with scalar arithmetic from the row's address) and only the
// lane's column offset sits in a vector register -- no 64-bit per-lane address arithmetic.
// The descriptor's extent is ONE ROW, so a lane whose columns lie past the row end gets zeros
// back and causes no memory traffic.
__device__ __forceinline__ __amdgpu_buffer_rsrc_t row_resource(const void *row, uint32_t row_bytes) {
    return __builtin_amdgcn_make_buffer_rsrc(const_cast<void *>(row), 0, (int)row_bytes, 0x00020000);
}
__device__ __forceinline__ u32x4 stream_load16(__amdgpu_buffer_rsrc_t row, uint32_t lane_offset) {
    return __builtin_amdgcn_raw_buffer_load_b128(row, (int)lane_offset, 0, 2);   // 2 = non-temporal
}
// Cached 16-byte load through a descriptor: a lane whose offset lies past the extent gets zeros.
__device__ __forceinline__ u32x4 buffer_load16(__amdgpu_buffer_rsrc_t rsrc, uint32_t lane_offset) {
    return __builtin_amdgcn_raw_buffer_load_b128(rsrc, (int)lane_offset, 0, 0);
}

typedef const char __attribute__((address_space(1))) *global_char_ptr;

__device__ __forceinline__ u32x4 stream_load16(const void *p) {
    return __builtin_nontemporal_load((global_u32x4_ptr)p);   // weights are read once per step
}
// Same, from a wave-uniform base plus a per-lane 32-bit byte offset: written so that the
// load can take the base from scalar registers and only the offset from a vector register.
__device__ __forceinline__ u32x4 stream_load16(const void *uniform_base, uint32_t lane_offset) {
    const global_char_ptr b = (global_char_ptr)uniform_base;
    return __builtin_nontemporal_load((global_u32x4_ptr)(b + lane_offset));
}
__device__ __forceinline__ u32x4 global_load16(const void *p) { return *(global_u32x4_ptr)p; }
// One lane's piece of a cached row (16 bytes, or 8 for half4_t).
template <typename KT> __device__ __forceinline__ typename Store<KT>::piece_t kv_piece(const void *p) {
    return *(const typename Store<KT>::piece_t __attribute__((address_space(1))) *)p;
}
__device__ __forceinline__ u32x4 global_load16(const void *uniform_base, uint32_t lane_offset) {
    return *(global_u32x4_ptr)((global_char_ptr)uniform_base + lane_offset);
}
__device__ __forceinline__ float4 global_load_float4(const float *p) {
    const f32x4 v = *(global_f32x4_ptr)p;
    return make_float4(v.x, v.y, v.z, v.w);
}

// Read data another workgroup (possibly on another XCD, behind another L2) wrote and
// published with a device-scope fence.
__device__ __forceinline__ float coherent_load(const float *p) {
    return __hip_atomic_load(as_global(p), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// Activation traffic between workgroups.  COH = true (the persistent kernel): stores are
// written through to memory (device-scope relaxed atomic stores, the `sc1` form) and every
// produced vector has an address nothing read earlier in the launch, so consumers on other
// XCDs use ordinary loads: their L2 cannot hold a stale copy, and after the first miss the
// vector is served from that L2.  No L2 write-back or invalidate is ever needed.  The few
// places that re-read an address within a launch (attention partials) use act_load<true>.
// COH = false (one kernel per operator): ordinary accesses; the kernel boundary orders them.
template <bool COH> __device__ __forceinline__ float act_load(const float *p) {
    if (COH) return __hip_atomic_load(as_global(p), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    return *as_global(p);
}
template <bool COH> __device__ __forceinline__ void act_store(float *p, float v) {
    if (COH) __hip_atomic_store(as_global(p), v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    else *as_global(p) = v;
}

// 16 bytes of another workgroup's output, read coherently at device scope (the form a
// device-scope atomic load takes, four words wide).  The compiler barrier keeps it where it is
// written: a look at memory that another workgroup is writing must not be hoisted or merged.
__device__ __forceinline__ u32x4 coherent_load16(__amdgpu_buffer_rsrc_t rsrc, uint32_t byte_offset) {
    asm volatile("" ::: "memory");
    return __builtin_amdgcn_raw_buffer_load_b128(rsrc, (int)byte_offset, 0, 16);   // 16 = sc1: device scope
}
// The same look through the L2 (no scope bits): for data whose producer finished long ago.
__device__ __forceinline__ u32x4 cached_look16(__amdgpu_buffer_rsrc_t rsrc, uint32_t byte_offset) {
    asm volatile("" ::: "memory");
    return __builtin_amdgcn_raw_buffer_load_b128(rsrc, (int)byte_offset, 0, 0);
}
// The twin of an activation element in the other arena (see ACT_UNSET).
__device__ __forceinline__ float *twin_of(float *p, long long twin) { return (float *)((char *)p + twin); }
__device__ __forceinline__ void twin_unset(float *p, long long twin) {
    __hip_atomic_store((global_ptr<uint32_t>)twin_of(p, twin), ACT_UNSET, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
    for (int o = WAVE / 2; o > 0; o >>= 1) v += __shfl_xor(v, o, WAVE);
    return v;
}
__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
    for (int o = WAVE / 2; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, WAVE));
    return v;
}
// The same reductions on the vector unit's own lane-crossing paths (quad permutes, mirrors
// within a row of 16 lanes, row broadcasts) instead of six dependent trips through the LDS
// crossbar: a fraction of the latency.  The result is complete in lane 63 ONLY.
template <int CTRL, int ROW_MASK>
__device__ __forceinline__ float dpp_move(float v, float identity) {
    return __int_as_float(__builtin_amdgcn_update_dpp(__float_as_int(identity), __float_as_int(v), CTRL, ROW_MASK, 0xF, false));
}
__device__ __forceinline__ float wave_sum_last(float v) {
    v += dpp_move<0xB1, 0xF>(v, 0.f);    // quad_perm [1,0,3,2]
    v += dpp_move<0x4E, 0xF>(v, 0.f);    // quad_perm [2,3,0,1]
    v += dpp_move<0x141, 0xF>(v, 0.f);   // row_half_mirror
    v += dpp_move<0x140, 0xF>(v, 0.f);   // row_mirror: every lane holds its row's sum
    v += dpp_move<0x142, 0xA>(v, 0.f);   // row_bcast15 into rows 1 and 3
    v += dpp_move<0x143, 0xC>(v, 0.f);   // row_bcast31 into rows 2 and 3
    return v;
}
__device__ __forceinline__ float wave_max_last(float v) {
    v = fmaxf(v, dpp_move<0xB1, 0xF>(v, -INFINITY));
    v = fmaxf(v, dpp_move<0x4E, 0xF>(v, -INFINITY));
    v = fmaxf(v, dpp_move<0x141, 0xF>(v, -INFINITY));
    v = fmaxf(v, dpp_move<0x140, 0xF>(v, -INFINITY));
    v = fmaxf(v, dpp_move<0x142, 0xA>(v, -INFINITY));
    v = fmaxf(v, dpp_move<0x143, 0xC>(v, -INFINITY));
    return v;
}
// Sum over the block in a fixed order; every thread gets the result. `red` has NT/64 floats.
template <int NT>
__device__ __forceinline__ float block_sum(float v, float *red) {
    constexpr int NWAVE = NT / WAVE;
    v = wave_sum_last(v);
    __syncthreads();
    if ((threadIdx.x & (WAVE - 1)) == WAVE - 1) red[threadIdx.x / WAVE] = v;
    __syncthreads();
    float t = 0.f;
#pragma unroll
    for (int w = 0; w < NWAVE; ++w) t += red[w];
    return t;
}
template <int NT>
__device__ __forceinline__ float block_max(float v, float *red) {
    constexpr int NWAVE = NT / WAVE;
    v = wave_max_last(v);
    __syncthreads();
    if ((threadIdx.x & (WAVE - 1)) == WAVE - 1) red[threadIdx.x / WAVE] = v;
    __syncthreads();
    float t = red[0];
#pragma unroll
    for (int w = 1; w < NWAVE; ++w) t = fmaxf(t, red[w]);
    return t;
}


// The key/value cache holds fp32 by default whatever the weight type: rounding cached keys and
// values to bf16 alone costs about 2e-2 of the logit scale over 32 layers, the whole error
// budget.  A bf16 model may ask for an fp16 cache (11 significant bits: an eighth of that
// error, half the bytes of the fp32 cache per cached position).
// Two adjacent elements (at, at + 1; at is even) of a cache row, as the cache stores them;
// returns through e, o the values a later read of the cache will see.
template <bool COH, bool HALF>
__device__ __forceinline__ void kv_store_pair(void *cache, size_t at, float &e, float &o) {
    if (HALF) {
        const uint32_t w = (uint32_t)Store<half_t>::bits(e) | ((uint32_t)Store<half_t>::bits(o) << 16);
        global_ptr<uint32_t> p = (global_ptr<uint32_t>)((global_ptr<uint16_t>)cache + at);
        if (COH) __hip_atomic_store(p, w, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        else *p = w;
        e = (float)__builtin_bit_cast(_Float16, (uint16_t)(w & 0xFFFFu));
        o = (float)__builtin_bit_cast(_Float16, (uint16_t)(w >> 16));
    } else {
        if (COH) { Store<float>::store1_coherent(cache, at, e); Store<float>::store1_coherent(cache, at + 1, o); }
        else { Store<float>::store1(cache, at, e); Store<float>::store1(cache, at + 1, o); }
    }
}

// ------------------------------------------------------------------ GEMV epilogues
// What happens to the two finished dot products of one work unit (a row pair, or for
// EPI_SWIGLU row `unit` of the gate and of the up matrix).
// cos/sin of pos * theta^(-2i/d_head), computed in double as the reference does.
__device__ __forceinline__ float2 rope_cos_sin(const double *inv_freq, int i, int pos) {
    const double ang = (double)pos * as_global(inv_freq)[i];
    return make_float2((float)cos(ang), (float)sin(ang));
}

// ROPE_GIVEN: the caller supplies (cos, sin) of this unit's rotary angle in `given` instead
// of having the angle evaluated on the spot.
template <typename WT, int EPI, bool ROPE_GIVEN = false, bool COH = false>
__device__ __forceinline__ void gemv_epilogue(const GemvArgs &a, int unit, float acc0, float acc1, int pos,
                                              float2 given = make_float2(1.f, 0.f)) {
    if (EPI == EPI_PLAIN) {
        act_store<COH>(a.y + 2 * unit, acc0);
        act_store<COH>(a.y + 2 * unit + 1, acc1);
    } else if (EPI == EPI_RESID) {
        act_store<COH>(a.y + 2 * unit, as_global(a.resid)[2 * unit] + acc0);
        act_store<COH>(a.y + 2 * unit + 1, as_global(a.resid)[2 * unit + 1] + acc1);
    } else if (EPI == EPI_SWIGLU) {
        act_store<COH>(a.y + unit, acc0 / (1.0f + expf(-acc0)) * acc1);
    } else {  // EPI_QKV: rotary on q and k pairs, append k and v to the cache
        const int r0 = 2 * unit;
        if (r0 < a.n_q_rows + a.n_kv_rows) {
            const int i = (r0 % a.d_head) / 2;
            const float2 cs = ROPE_GIVEN ? given : rope_cos_sin(a.inv_freq, i, pos);
            const float c = cs.x, s = cs.y;
            const float e = __fsub_rn(__fmul_rn(acc0, c), __fmul_rn(acc1, s));
            const float o = __fadd_rn(__fmul_rn(acc0, s), __fmul_rn(acc1, c));
            if (r0 < a.n_q_rows) {
                act_store<COH>(a.y + r0, e);
                act_store<COH>(a.y + r0 + 1, o);
            } else {
                const int rr = r0 - a.n_q_rows;
                const size_t at = ((size_t)(rr / a.d_head) * a.cap_ctx + pos) * a.d_head + rr % a.d_head;
                float ke = e, ko = o;
                if (a.kv_half) kv_store_pair<COH, true>(a.kcache, at, ke, ko);
                else kv_store_pair<COH, false>(a.kcache, at, ke, ko);
            }
        } else {
            const int rr = r0 - a.n_q_rows - a.n_kv_rows;
            const size_t at = ((size_t)(rr / a.d_head) * a.cap_ctx + pos) * a.d_head + rr % a.d_head;
            if (a.kv_half) kv_store_pair<COH, true>(a.vcache, at, acc0, acc1);
            else kv_store_pair<COH, false>(a.vcache, at, acc0, acc1);
        }
    }
}

// ------------------------------------------------------------------ single-query attention
// One work item = (key/value head g, context chunk s) handled by a block of NT threads.  The
// query heads [hq0, hq1) of those sharing head g are served from the chunk, one after another.  Chunks are merged by whichever block
// finishes last for a head, walking the partial results in chunk order (deterministic).
// LDS: sc[a.chunk], red[NT/64], dyn[NT * VEC] floats, one int.
// COH: outputs are written through; partial results of other chunks are re-read coherently.
// Sum over groups of LPP consecutive lanes (LPP a power of two), complete in the LAST lane of
// each group: lane-crossing moves of the vector unit instead of LDS permutes.
__device__ __forceinline__ float group_sum_last(float v, int lpp) {
    if (lpp >= 2) v += dpp_move<0xB1, 0xF>(v, 0.f);
    if (lpp >= 4) v += dpp_move<0x4E, 0xF>(v, 0.f);
    if (lpp >= 8) v += dpp_move<0x141, 0xF>(v, 0.f);
    if (lpp >= 16) v += dpp_move<0x140, 0xF>(v, 0.f);
    if (lpp >= 32) v += dpp_move<0x142, 0xA>(v, 0.f);
    if (lpp >= 64) v += dpp_move<0x143, 0xC>(v, 0.f);
    return v;
}

// The same for N values at once, step by step: the N independent lane-crossing moves of a step sit
// between two (wave-uniform) branches and overlap, where N calls of group_sum_last run as N chains.
template <int N>
__device__ __forceinline__ void group_sums_last(float (&v)[N], int lpp) {
    if (lpp >= 2) {
#pragma unroll
        for (int i = 0; i < N; ++i) v[i] += dpp_move<0xB1, 0xF>(v[i], 0.f);
    }
    if (lpp >= 4) {
#pragma unroll
        for (int i = 0; i < N; ++i) v[i] += dpp_move<0x4E, 0xF>(v[i], 0.f);
    }
    if (lpp >= 8) {
#pragma unroll
        for (int i = 0; i < N; ++i) v[i] += dpp_move<0x141, 0xF>(v[i], 0.f);
    }
    if (lpp >= 16) {
#pragma unroll
        for (int i = 0; i < N; ++i) v[i] += dpp_move<0x140, 0xF>(v[i], 0.f);
    }
    if (lpp >= 32) {
#pragma unroll
        for (int i = 0; i < N; ++i) v[i] += dpp_move<0x142, 0xA>(v[i], 0.f);
    }
    if (lpp >= 64) {
#pragma unroll
        for (int i = 0; i < N; ++i) v[i] += dpp_move<0x143, 0xC>(v[i], 0.f);
    }
}

// a.k_new / a.v_new (the persistent kernel): the newest position's key and value rows are not
// read from the cache but from activation vectors [n_kv_heads * d_head] that the QKV phase of
// this very launch is writing, and so is the query: all three are awaited as data (looked at
// coherently until no word reads ACT_UNSET; bounded, the error word is raised past the limit)
// -- after the cached rows of the earlier positions have been requested, so that the wait and
// that fetch overlap.  The newest position is handled by the first lanes of wave 0.
// ROWS: cached rows a lane keeps in flight per batch of loads (0: 10); every row of a batch costs
// its arithmetic whether the chunk reaches it or not.
template <typename KT, int NT, bool COH = false, int ROWS = 0>
__device__ __forceinline__ void attn_item(const AttnArgs &a, int g, int s, int n_ctx, float *sc, float *red,
                                          float *dyn, int *s_last, int hq0 = 0, int hq1 = INT_MAX, int *err = nullptr) {
    constexpr int VEC = Store<KT>::VEC;
    constexpr int NWAVE = NT / WAVE;
    int tid = threadIdx.x;
    // (the persistent kernel calls this once per layer: without this the compiler computes every
    // thread-dependent address below once, before the layer loop, and keeps some thirty vector
    // registers occupied through all the other phases)
    if (COH) asm volatile("" : "+v"(tid));
    const int lane = tid & (WAVE - 1), wid = tid / WAVE;
    const int dh = a.d_head;
    const int LPP = dh / VEC;             // lanes per cached position
    const int PPW = WAVE / LPP;           // positions per wave per iteration
    const int PPB = PPW * NWAVE;
    const int sub = lane / LPP, li = lane % LPP;
    const int t0 = s * a.chunk;
    const int t1 = min(n_ctx, t0 + a.chunk);
    const bool awaited = COH && a.k_new != nullptr;              // q (and the newest k, v) are awaited as data
    const bool has_new = awaited && t1 == n_ctx && t1 > t0;      // this chunk ends with the newest position
    const int t1c = has_new ? t1 - 1 : t1;                       // cached rows: [t0, t1c)
    const bool new_lanes = has_new && wid == 0 && sub == 0;      // the lanes that handle the newest position
    const int n_splits = (n_ctx + a.chunk - 1) / a.chunk;
    const int group = a.n_heads / a.n_kv_heads;
    const float scale = 1.0f / sqrtf((float)dh);
    const char *Kg = (const char *)a.K + (size_t)g * a.cap_ctx * dh * sizeof(KT);
    const char *Vg = (const char *)a.V + (size_t)g * a.cap_ctx * dh * sizeof(KT);

    // Cached rows are requested ATTN_BATCH at a time per lane (10: one batch covers a chunk of up to
    // 160 positions, which is what contexts up to 1280 give on 256 blocks and 32 heads; 12 spills
    // registers in the persistent kernel), and the first batch of value
    // rows together with the keys: this phase is a chain of memory latencies, not bandwidth.
    constexpr int ATTN_BATCH = ROWS ? ROWS : 10;
    const int tbase = t0 + wid * PPW + sub;
    // query heads [hq0, hq1) of the group that shares key/value head g
    for (int hq = hq0; hq < min(hq1, group); ++hq) {
        const int h = g * group + hq;
        float qv[VEC];
        float lmax = -INFINITY;
        typedef typename Store<KT>::piece_t piece_t;
        piece_t vb[ATTN_BATCH], kb[ATTN_BATCH];
        auto first_batch = [&]() {
#pragma unroll
            for (int i = 0; i < ATTN_BATCH; ++i) {
                const int t = tbase + i * PPB;
                kb[i] = (piece_t)(0u);
                if (t < t1c) kb[i] = kv_piece<KT>(Kg + ((size_t)t * dh + li * VEC) * sizeof(KT));
            }
#pragma unroll
            for (int i = 0; i < ATTN_BATCH; ++i) {
                const int t = tbase + i * PPB;
                vb[i] = (piece_t)(0u);
                if (t < t1c) vb[i] = kv_piece<KT>(Vg + ((size_t)t * dh + li * VEC) * sizeof(KT));
            }
        };
        float knew[VEC], vnew[VEC];
        if (awaited) {
            // the awaited vectors are fp32: a lane's VEC elements are NP pieces of 16 bytes
            constexpr int NP = VEC / 4;
            // the looks go out together (one trip, not three); whatever is incomplete is looked at again
            const __amdgpu_buffer_rsrc_t qrs = __builtin_amdgcn_make_buffer_rsrc(const_cast<float *>(a.q), 0, a.n_heads * dh * 4, 0x00020000);
            const __amdgpu_buffer_rsrc_t krs = __builtin_amdgcn_make_buffer_rsrc(const_cast<float *>(a.k_new), 0, a.n_kv_heads * dh * 4, 0x00020000);
            const __amdgpu_buffer_rsrc_t vrs = __builtin_amdgcn_make_buffer_rsrc(const_cast<float *>(a.v_new), 0, a.n_kv_heads * dh * 4, 0x00020000);
            const uint32_t qat = (uint32_t)(h * dh + li * VEC) * 4u, kat = (uint32_t)(g * dh + li * VEC) * 4u;
            auto unset = [](const u32x4 v) { return v.x == ACT_UNSET || v.y == ACT_UNSET || v.z == ACT_UNSET || v.w == ACT_UNSET; };
            // a first look, then the first batch of cached keys and values right behind it (they are needed
            // whatever the look says; a look that has to be repeated comes back behind them)
            u32x4 qraw[NP], kr[NP], vr[NP];
#pragma unroll
            for (int p = 0; p < NP; ++p) {
                qraw[p] = coherent_load16(qrs, qat + 16u * p);
                kr[p] = u32x4{0u, 0u, 0u, 0u}; vr[p] = u32x4{0u, 0u, 0u, 0u};
                if (new_lanes) { kr[p] = coherent_load16(krs, kat + 16u * p); vr[p] = coherent_load16(vrs, kat + 16u * p); }
            }
            first_batch();
            auto any_unset = [&]() {
                bool r = false;
#pragma unroll
                for (int p = 0; p < NP; ++p) r = r || unset(qraw[p]) || unset(kr[p]) || unset(vr[p]);
                return r;
            };
            for (unsigned spins = 0; any_unset(); ++spins) {
                if (spins > (1u << 22) || ((spins & 255u) == 255u && __hip_atomic_load(as_global(err), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT))) {
                    __hip_atomic_store(as_global(err), 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);   // bounded: give up, the host reports it
                    break;
                }
                __builtin_amdgcn_s_sleep(1);
#pragma unroll
                for (int p = 0; p < NP; ++p) {
                    if (unset(qraw[p])) qraw[p] = coherent_load16(qrs, qat + 16u * p);
                    if (unset(kr[p])) kr[p] = coherent_load16(krs, kat + 16u * p);
                    if (unset(vr[p])) vr[p] = coherent_load16(vrs, kat + 16u * p);
                }
            }
#pragma unroll
            for (int p = 0; p < NP; ++p) {
                qv[4 * p] = __uint_as_float(qraw[p].x); qv[4 * p + 1] = __uint_as_float(qraw[p].y);
                qv[4 * p + 2] = __uint_as_float(qraw[p].z); qv[4 * p + 3] = __uint_as_float(qraw[p].w);
                if (new_lanes) {
                    knew[4 * p] = __uint_as_float(kr[p].x); knew[4 * p + 1] = __uint_as_float(kr[p].y);
                    knew[4 * p + 2] = __uint_as_float(kr[p].z); knew[4 * p + 3] = __uint_as_float(kr[p].w);
                    vnew[4 * p] = __uint_as_float(vr[p].x); vnew[4 * p + 1] = __uint_as_float(vr[p].y);
                    vnew[4 * p + 2] = __uint_as_float(vr[p].z); vnew[4 * p + 3] = __uint_as_float(vr[p].w);
                }
            }
        } else {
            first_batch();
#pragma unroll
            for (int v = 0; v < VEC; ++v) qv[v] = as_global(a.q)[(size_t)h * dh + li * VEC + v];
        }
        for (int b0 = tbase; b0 - sub < t1c; b0 += ATTN_BATCH * PPB) {   // b0 - sub is wave-uniform
            if (b0 != tbase) {
#pragma unroll
                for (int i = 0; i < ATTN_BATCH; ++i) {
                    const int t = b0 + i * PPB;
                    kb[i] = (piece_t)(0u);
                    if (t < t1c) kb[i] = kv_piece<KT>(Kg + ((size_t)t * dh + li * VEC) * sizeof(KT));
                }
            }
            // all rows' dot products first, without a branch between them (their chains of dependent
            // operations interleave), then the stores
            float dd[ATTN_BATCH];
#pragma unroll
            for (int i = 0; i < ATTN_BATCH; ++i) {
                float kf[VEC];
                Store<KT>::unpack(kb[i], kf);
                float d = 0.f;
#pragma unroll
                for (int v = 0; v < VEC; ++v) d = fmaf(kf[v], qv[v], d);
                dd[i] = d;
            }
            group_sums_last<ATTN_BATCH>(dd, LPP);   // complete in each group's last lane
#pragma unroll
            for (int i = 0; i < ATTN_BATCH; ++i) dd[i] *= scale;
            if (li == LPP - 1) {
#pragma unroll
                for (int i = 0; i < ATTN_BATCH; ++i) {
                    const int t = b0 + i * PPB;
                    if (t < t1c) {
                        sc[t - t0] = dd[i];
                        lmax = fmaxf(lmax, dd[i]);
                    }
                }
            }
        }
        if (has_new && wid == 0) {   // (whole wave: the lane-crossing sum needs every lane's turn)
            float d = 0.f;
            if (new_lanes) {
#pragma unroll
                for (int v = 0; v < VEC; ++v) d = fmaf(knew[v], qv[v], d);
            }
            d = group_sum_last(d, LPP) * scale;
            if (new_lanes && li == LPP - 1) {
                sc[t1c - t0] = d;
                lmax = fmaxf(lmax, d);
            }
        }
        const float m = block_max<NT>(lmax, red);   // includes a barrier after the sc writes
        float lsum = 0.f;
        for (int t = tid; t < t1 - t0; t += NT) {
            const float p = expf(sc[t] - m);
            sc[t] = p;
            lsum += p;
        }
        const float l = block_sum<NT>(lsum, red);
        float acc[VEC];
#pragma unroll
        for (int v = 0; v < VEC; ++v) acc[v] = 0.f;
        for (int b0 = tbase; b0 < t1c; b0 += ATTN_BATCH * PPB) {
            if (b0 != tbase) {
#pragma unroll
                for (int i = 0; i < ATTN_BATCH; ++i) {
                    const int t = b0 + i * PPB;
                    vb[i] = (piece_t)(0u);
                    if (t < t1c) vb[i] = kv_piece<KT>(Vg + ((size_t)t * dh + li * VEC) * sizeof(KT));
                }
            }
#pragma unroll
            for (int i = 0; i < ATTN_BATCH; ++i) {   // (no branch: a row past the chunk holds zeros and gets weight 0)
                const int t = b0 + i * PPB;
                const bool row = t < t1c;
                float vf[VEC];
                Store<KT>::unpack(vb[i], vf);
                const float ps = sc[row ? t - t0 : 0];
                const float p = row ? ps : 0.f;
#pragma unroll
                for (int v = 0; v < VEC; ++v) acc[v] = fmaf(p, vf[v], acc[v]);
            }
        }
        if (new_lanes) {
            const float p = sc[t1c - t0];
#pragma unroll
            for (int v = 0; v < VEC; ++v) acc[v] = fmaf(p, vnew[v], acc[v]);
        }
        // the lane groups of a wave hold partial sums for the same features: add them across the wave
        // (ascending distance, a fixed order), then the waves' sums through LDS
#pragma unroll
        for (int d = 1; d < WAVE; d <<= 1) {
            if (d >= LPP) {
#pragma unroll
                for (int v = 0; v < VEC; ++v) acc[v] += __shfl_xor(acc[v], d, WAVE);
            }
        }
        if (sub == 0) {
#pragma unroll
            for (int v = 0; v < VEC; ++v) dyn[(size_t)wid * dh + li * VEC + v] = acc[v];
        }
        __syncthreads();
        float o = 0.f;
        if (tid < dh) {
#pragma unroll
            for (int r = 0; r < NWAVE; ++r) o += dyn[(size_t)r * dh + tid];
        }
        if (n_splits == 1) {
            if (tid < dh) {
                act_store<COH>(a.out + (size_t)h * dh + tid, o / l);
                if (COH && a.out_twin) twin_unset(a.out + (size_t)h * dh + tid, a.out_twin);
            }
        } else {
            float *pp = a.part + ((size_t)h * a.max_splits + s) * (dh + 2);
            if (tid < dh) act_store<COH>(pp + 2 + tid, o);
            if (tid == 0) { act_store<COH>(pp, m); act_store<COH>(pp + 1, l); }
            if (COH) asm volatile("s_waitcnt vmcnt(0)" ::: "memory");   // write-through stores acknowledged
            else __threadfence();
            __syncthreads();
            if (tid == 0) {
                const int old = __hip_atomic_fetch_add(as_global(a.counters) + (size_t)h * ATTN_COUNTER_STRIDE, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                *s_last = (old == n_splits - 1);
            }
            __syncthreads();
            if (*s_last) {
                if (!COH) __threadfence();
                const float *ph = a.part + (size_t)h * a.max_splits * (dh + 2);
                float L = 0.f, O = 0.f;
                if (n_splits <= min(a.chunk, NT)) {
                    // every chunk's (max, sum) at once, one thread each; weights via LDS; then
                    // the partial outputs eight chunks at a time.  Sums run in chunk order.
                    float mq = -INFINITY, lq = 0.f;
                    if (tid < n_splits) {
                        mq = coherent_load(ph + (size_t)tid * (dh + 2));
                        lq = coherent_load(ph + (size_t)tid * (dh + 2) + 1);
                    }
                    const float M = block_max<NT>(mq, red);
                    if (tid < n_splits) {
                        const float w = expf(mq - M);
                        sc[tid] = w;
                        dyn[tid] = w * lq;
                    }
                    __syncthreads();
                    for (int q = 0; q < n_splits; ++q) L += dyn[q];
                    if (tid < dh) {
                        for (int q0 = 0; q0 < n_splits; q0 += 8) {
                            float pv[8];
#pragma unroll
                            for (int j = 0; j < 8; ++j)
                                pv[j] = coherent_load(ph + (size_t)min(q0 + j, n_splits - 1) * (dh + 2) + 2 + tid);
#pragma unroll
                            for (int j = 0; j < 8; ++j)
                                if (q0 + j < n_splits) O += sc[q0 + j] * pv[j];
                        }
                    }
                } else {
                    float M = -INFINITY;
                    for (int q = 0; q < n_splits; ++q) M = fmaxf(M, coherent_load(ph + (size_t)q * (dh + 2)));
                    for (int q = 0; q < n_splits; ++q) {
                        const float *pq = ph + (size_t)q * (dh + 2);
                        const float w = expf(coherent_load(pq) - M);
                        L += w * coherent_load(pq + 1);
                        if (tid < dh) O += w * coherent_load(pq + 2 + tid);
                    }
                }
                if (tid < dh) {
                    act_store<COH>(a.out + (size_t)h * dh + tid, O / L);
                    if (COH && a.out_twin) twin_unset(a.out + (size_t)h * dh + tid, a.out_twin);
                }
                // (written through: the next user of this counter may sit behind another L2)
                if (tid == 0) __hip_atomic_store(as_global(a.counters) + (size_t)h * ATTN_COUNTER_STRIDE, 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            }
        }
        __syncthreads();   // sc / dyn / s_last are reused by the next query head or item
    }
}

// ------------------------------------------------------------------ superposed embedding
// Section 3.1: gamma_i = p_i / sum_j p_j (from log p_i), x~ = sum_i gamma_i z_i, element c.
// mode 0 feeds a prefix token's own embedding (gamma = 1) during the prefix pass.
template <typename WT, bool COH = false>
__device__ __forceinline__ void superpose_element(const SuperposeArgs &a, int c, int pos) {
    if (COH && a.twin && c < a.d_model) twin_unset(a.h + c, a.twin);
    if (a.mode == 0) {
        const int tok = as_global(a.prefix)[pos];
        if (c < a.d_model) act_store<COH>(a.h + c, Store<WT>::load1(a.embed, (size_t)tok * a.d_model + c));
        return;
    }
    const int k = a.k;
    float mx = -INFINITY;
    for (int i = 0; i < k; ++i) mx = fmaxf(mx, as_global(a.st)->logscore[i]);
    float sum = 0.f;
    for (int i = 0; i < k; ++i) sum += expf(as_global(a.st)->logscore[i] - mx);
    float acc = 0.f;
    for (int i = 0; i < k; ++i) {
        const float gi = expf(as_global(a.st)->logscore[i] - mx) / sum;
        if (c < a.d_model) {
            const int tok = as_global(a.st)->tails[i][SPD_TAIL - 1];
            acc = __fadd_rn(acc, __fmul_rn(gi, Store<WT>::load1(a.embed, (size_t)tok * a.d_model + c)));
        }
        if (c == 0) as_global(a.st)->gamma_in[i] = gi;
    }
    if (c < a.d_model) act_store<COH>(a.h + c, acc);
}

}  // namespace spdd
