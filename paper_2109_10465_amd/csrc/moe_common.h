// Shared device/host helpers for the MoE kernels (gfx950, wave64).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include "../../include/moe_hip.h"

#define MOE_WAVE 64

typedef uint16_t bf16_t;  // bfloat16 bit pattern

// ---- bf16 <-> fp32 ---------------------------------------------------------
__device__ __forceinline__ float bf16_to_f32(bf16_t v) {
    return __uint_as_float(((uint32_t)v) << 16);
}
// round to nearest, ties to even (finite inputs; NaN stays NaN)
__device__ __forceinline__ bf16_t f32_to_bf16(float f) {
    uint32_t u = __float_as_uint(f);
    if ((u & 0x7fffffffu) > 0x7f800000u) return (bf16_t)((u >> 16) | 0x40u);
    u += 0x7fffu + ((u >> 16) & 1u);
    return (bf16_t)(u >> 16);
}
// two fp32 -> packed bf16 pair (v_cvt_pk_bf16_f32, round to nearest even)
typedef __bf16 bf16x2_hw_t __attribute__((ext_vector_type(2)));
typedef float f32x2_hw_t __attribute__((ext_vector_type(2)));
__device__ __forceinline__ uint32_t pack_bf16x2(float lo, float hi) {
    const f32x2_hw_t v = {lo, hi};
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2_hw_t));
}

// element-type generic scalar load/store through fp32
template <typename T> __device__ __forceinline__ float ld_f32(const T* p);
template <> __device__ __forceinline__ float ld_f32<float>(const float* p) { return *p; }
template <> __device__ __forceinline__ float ld_f32<bf16_t>(const bf16_t* p) { return bf16_to_f32(*p); }
template <typename T> __device__ __forceinline__ void st_f32(T* p, float v);
template <> __device__ __forceinline__ void st_f32<float>(float* p, float v) { *p = v; }
template <> __device__ __forceinline__ void st_f32<bf16_t>(bf16_t* p, float v) { *p = f32_to_bf16(v); }

// A 16-byte chunk of activations: 4 floats or 8 bf16, widened to fp32 lanes.
template <typename T> struct Chunk;
template <> struct Chunk<float> {
    static constexpr int N = 4;
    __device__ static __forceinline__ void load(const float* p, float (&v)[4]) {
        float4 q = *reinterpret_cast<const float4*>(p);
        v[0] = q.x; v[1] = q.y; v[2] = q.z; v[3] = q.w;
    }
    __device__ static __forceinline__ void store(float* p, const float (&v)[4]) {
        *reinterpret_cast<float4*>(p) = make_float4(v[0], v[1], v[2], v[3]);
    }
};
template <> struct Chunk<bf16_t> {
    static constexpr int N = 8;
    __device__ static __forceinline__ void load(const bf16_t* p, float (&v)[8]) {
        uint4 q = *reinterpret_cast<const uint4*>(p);
        uint32_t w[4] = {q.x, q.y, q.z, q.w};
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            v[2 * i] = __uint_as_float(w[i] << 16);
            v[2 * i + 1] = __uint_as_float(w[i] & 0xffff0000u);
        }
    }
    __device__ static __forceinline__ void store(bf16_t* p, const float (&v)[8]) {
        uint4 q;
        q.x = pack_bf16x2(v[0], v[1]); q.y = pack_bf16x2(v[2], v[3]);
        q.z = pack_bf16x2(v[4], v[5]); q.w = pack_bf16x2(v[6], v[7]);
        *reinterpret_cast<uint4*>(p) = q;
    }
};

// 4 consecutive elements of one row as the activation type (8 or 16 bytes)
template <typename T> struct Vec4io;
template <> struct Vec4io<float> {
    typedef float4 raw;
    __device__ static __forceinline__ raw zero() { return make_float4(0.f, 0.f, 0.f, 0.f); }
    __device__ static __forceinline__ raw pack(const float (&v)[4]) { return make_float4(v[0], v[1], v[2], v[3]); }
    __device__ static __forceinline__ void unpack(raw q, float (&v)[4]) { v[0] = q.x; v[1] = q.y; v[2] = q.z; v[3] = q.w; }
};
template <> struct Vec4io<bf16_t> {
    typedef uint2 raw;
    __device__ static __forceinline__ raw zero() { return make_uint2(0u, 0u); }
    __device__ static __forceinline__ raw pack(const float (&v)[4]) {
        return make_uint2(pack_bf16x2(v[0], v[1]), pack_bf16x2(v[2], v[3]));
    }
    __device__ static __forceinline__ void unpack(raw q, float (&v)[4]) {
        v[0] = __uint_as_float(q.x << 16); v[1] = __uint_as_float(q.x & 0xffff0000u);
        v[2] = __uint_as_float(q.y << 16); v[3] = __uint_as_float(q.y & 0xffff0000u);
    }
};

// ---- raw buffer access: the descriptor's range check replaces per-lane branches ----
// Loads beyond `bytes` return 0 and stores beyond it are dropped, so a guard is
// folded into the offset (BUF_OOB for "not this lane") and the code stays branch free.
typedef unsigned int u32x2_buf_t __attribute__((ext_vector_type(2)));
typedef unsigned int u32x4_buf_t __attribute__((ext_vector_type(4)));
#define BUF_OOB 0x80000000u   // beyond every descriptor built here (ranges stay below 2 GiB)
__device__ __forceinline__ __amdgpu_buffer_rsrc_t buf_rsrc(const void* p, size_t bytes) {
    const uint32_t n = bytes < 0x7fffffffull ? (uint32_t)bytes : 0x7fffffffu;
    return __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(p), 0, (int)n, 0x00020000);
}
__device__ __forceinline__ float buf_load_f32(__amdgpu_buffer_rsrc_t r, uint32_t off) {
    return __uint_as_float(__builtin_amdgcn_raw_buffer_load_b32(r, off, 0, 0));
}
// 16 bytes of activations at byte offset off, widened to fp32
template <typename T> struct BufChunk;
template <> struct BufChunk<float> {
    static constexpr int N = 4;
    __device__ static __forceinline__ void load(__amdgpu_buffer_rsrc_t r, uint32_t off, float (&v)[4]) {
        const u32x4_buf_t q = __builtin_amdgcn_raw_buffer_load_b128(r, off, 0, 0);
#pragma unroll
        for (int i = 0; i < 4; ++i) v[i] = __uint_as_float(q[i]);
    }
    __device__ static __forceinline__ void store(__amdgpu_buffer_rsrc_t r, uint32_t off, const float (&v)[4]) {
        const u32x4_buf_t q = {__float_as_uint(v[0]), __float_as_uint(v[1]), __float_as_uint(v[2]), __float_as_uint(v[3])};
        __builtin_amdgcn_raw_buffer_store_b128(q, r, off, 0, 0);
    }
};
template <> struct BufChunk<bf16_t> {
    static constexpr int N = 8;
    __device__ static __forceinline__ void store(__amdgpu_buffer_rsrc_t r, uint32_t off, const float (&v)[8]) {
        const u32x4_buf_t q = {pack_bf16x2(v[0], v[1]), pack_bf16x2(v[2], v[3]), pack_bf16x2(v[4], v[5]),
                               pack_bf16x2(v[6], v[7])};
        __builtin_amdgcn_raw_buffer_store_b128(q, r, off, 0, 0);
    }
    __device__ static __forceinline__ void load(__amdgpu_buffer_rsrc_t r, uint32_t off, float (&v)[8]) {
        const u32x4_buf_t q = __builtin_amdgcn_raw_buffer_load_b128(r, off, 0, 0);
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            v[2 * i] = __uint_as_float(q[i] << 16);
            v[2 * i + 1] = __uint_as_float(q[i] & 0xffff0000u);
        }
    }
};

// ---- loads that write LDS directly, and the counters that track them ----------------
// Raw buffer descriptor (4 SGPRs) over `bytes` bytes at p: loads beyond the
// range return 0 (and, for loads into LDS, store 0).
__device__ __forceinline__ u32x4_buf_t make_desc(const void* p, uint32_t bytes) {
    const uint64_t a = (uint64_t)p;
    u32x4_buf_t d;
    d[0] = (uint32_t)a;
    d[1] = (uint32_t)(a >> 32) & 0xffffu;
    d[2] = bytes;
    d[3] = 0x00020000u;
    return d;
}
// One wavefront-wide 16-byte-per-lane load from a raw buffer straight into LDS:
// lane l's 16 bytes land at LDS byte address lds_base + 16*l (lds_base is wave
// uniform and travels in M0).  Written as asm so that the compiler does not
// serialise every later LDS read behind the load; completion is tracked by
// hand with s_waitcnt vmcnt.  M0 is a reserved register for the
// compiler: it never keeps a value live in it across other code but writes it
// immediately before each instruction of its own that reads it, so overwriting
// it here is safe (naming it as a clobber is rejected as "reserved").
__device__ __forceinline__ void load_to_lds(u32x4_buf_t desc, uint32_t voff, uint32_t lds_base) {
    asm volatile("s_mov_b32 m0, %0\n\tbuffer_load_dwordx4 %1, %2, 0 offen lds"
                 :: "s"(lds_base), "v"(voff), "s"(desc) : "memory");
}
// s_waitcnt vmcnt(N) only (gfx9 encoding: vmcnt[3:0] in bits 3:0, vmcnt[5:4] in 15:14)
template <int N> __device__ __forceinline__ void wait_vmcnt() {
    __builtin_amdgcn_s_waitcnt((N & 0xf) | ((N >> 4) << 14) | (0x7 << 4) | (0xf << 8));
}

// the same, and every LDS operation of this wave has completed as well
template <int N> __device__ __forceinline__ void wait_vmcnt_lgkm0() {
    __builtin_amdgcn_s_waitcnt((N & 0xf) | ((N >> 4) << 14) | (0x7 << 4));
}

// ---- fp32 operands on the bf16 matrix pipe ------------------------------------------
// w = hi + mid + lo exactly, each part holding 8 significant bits cut off by
// truncation (3 x 8 = the whole fp32 significand).  A product of a bf16 value with
// each part is exact in fp32, so three bf16 MFMAs with fp32 accumulation multiply a
// bf16 operand by an fp32 operand without loss; dropping `lo` leaves 16 bits.
typedef __bf16 bf16x8_hw_t __attribute__((ext_vector_type(8)));
__device__ __forceinline__ void split3_bf16(const float (&w)[8], bf16x8_hw_t& hi, bf16x8_hw_t& mid, bf16x8_hw_t& lo) {
    u32x4_buf_t qh, qm, ql;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const float a = w[2 * i], b = w[2 * i + 1];
        const uint32_t ah = __float_as_uint(a) & 0xffff0000u, bh = __float_as_uint(b) & 0xffff0000u;
        const float a1 = a - __uint_as_float(ah), b1 = b - __uint_as_float(bh);
        const uint32_t am = __float_as_uint(a1) & 0xffff0000u, bm = __float_as_uint(b1) & 0xffff0000u;
        const float a2 = a1 - __uint_as_float(am), b2 = b1 - __uint_as_float(bm);
        qh[i] = (ah >> 16) | bh;
        qm[i] = (am >> 16) | bm;
        ql[i] = (__float_as_uint(a2) >> 16) | (__float_as_uint(b2) & 0xffff0000u);
    }
    hi = __builtin_bit_cast(bf16x8_hw_t, qh);
    mid = __builtin_bit_cast(bf16x8_hw_t, qm);
    lo = __builtin_bit_cast(bf16x8_hw_t, ql);
}

// w ~ hi + lo with both parts rounded to nearest: |w - hi - lo| <= 2^-16 |w|
__device__ __forceinline__ void split2_bf16(const float (&w)[8], bf16x8_hw_t& hi, bf16x8_hw_t& lo) {
    u32x4_buf_t qh, ql;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const uint32_t ph = pack_bf16x2(w[2 * i], w[2 * i + 1]);
        ql[i] = pack_bf16x2(w[2 * i] - __uint_as_float(ph << 16), w[2 * i + 1] - __uint_as_float(ph & 0xffff0000u));
        qh[i] = ph;
    }
    hi = __builtin_bit_cast(bf16x8_hw_t, qh);
    lo = __builtin_bit_cast(bf16x8_hw_t, ql);
}

template <typename T> struct Vec4buf;
template <> struct Vec4buf<float> {
    __device__ static __forceinline__ float4 load(__amdgpu_buffer_rsrc_t r, uint32_t off) {
        const u32x4_buf_t q = __builtin_amdgcn_raw_buffer_load_b128(r, off, 0, 0);
        return make_float4(__uint_as_float(q[0]), __uint_as_float(q[1]), __uint_as_float(q[2]), __uint_as_float(q[3]));
    }
    __device__ static __forceinline__ void store(__amdgpu_buffer_rsrc_t r, uint32_t off, float4 v) {
        u32x4_buf_t q = {__float_as_uint(v.x), __float_as_uint(v.y), __float_as_uint(v.z), __float_as_uint(v.w)};
        __builtin_amdgcn_raw_buffer_store_b128(q, r, off, 0, 0);
    }
};
template <> struct Vec4buf<bf16_t> {
    __device__ static __forceinline__ uint2 load(__amdgpu_buffer_rsrc_t r, uint32_t off) {
        const u32x2_buf_t q = __builtin_amdgcn_raw_buffer_load_b64(r, off, 0, 0);
        return make_uint2(q[0], q[1]);
    }
    __device__ static __forceinline__ void store(__amdgpu_buffer_rsrc_t r, uint32_t off, uint2 v) {
        u32x2_buf_t q = {v.x, v.y};
        __builtin_amdgcn_raw_buffer_store_b64(q, r, off, 0, 0);
    }
};

// ---- seeded noise: Philox4x32 with 10 rounds (Salmon et al., SC 2011) --------------
// Element i of a tensor uses word i % 4 of the block with counter
// (i/4 low word, i/4 high word, stream, 0) and key (seed low word, seed high word).
#define MOE_STREAM_JITTER 1u
#define MOE_STREAM_DROPOUT 2u
__device__ __forceinline__ void philox4x32_10(uint32_t c0, uint32_t c1, uint32_t c2, uint32_t c3,
                                              uint32_t k0, uint32_t k1, uint32_t (&out)[4]) {
#pragma unroll
    for (int i = 0; i < 10; ++i) {
        const uint32_t hi0 = __umulhi(0xD2511F53u, c0), lo0 = 0xD2511F53u * c0;
        const uint32_t hi1 = __umulhi(0xCD9E8D57u, c2), lo1 = 0xCD9E8D57u * c2;
        c0 = hi1 ^ c1 ^ k0; c1 = lo1;
        c2 = hi0 ^ c3 ^ k1; c3 = lo0;
        k0 += 0x9E3779B9u; k1 += 0xBB67AE85u;
    }
    out[0] = c0; out[1] = c1; out[2] = c2; out[3] = c3;
}
// words of the 4 consecutive elements that start at element index `first` (a multiple of 4)
__device__ __forceinline__ void noise_words(size_t first, uint32_t stream, uint64_t seed, uint32_t (&w)[4]) {
    const size_t blk = first >> 2;
    philox4x32_10((uint32_t)blk, (uint32_t)(blk >> 32), stream, 0u, (uint32_t)seed, (uint32_t)(seed >> 32), w);
}
// Gate jitter (Sec. 5.1): v[j] *= 1 + eps (2 u_j - 1), u_j = word_j / 2^32, for the N
// consecutive elements (N = 4, 8 or 16) starting at element index `first`
template <int N>
__device__ __forceinline__ void jitter_scale(float (&v)[N], size_t first, float eps, uint64_t seed) {
    const float a = eps * 4.656612873077393e-10f, b = 1.0f - eps;    // 2 eps / 2^32
#pragma unroll
    for (int q = 0; q < N / 4; ++q) {
        uint32_t w[4];
        noise_words(first + 4 * q, MOE_STREAM_JITTER, seed, w);
#pragma unroll
        for (int j = 0; j < 4; ++j) v[4 * q + j] *= fmaf(a, (float)w[j], b);
    }
}

// ---- wave64 reductions (butterfly: every lane ends with the same bits) ------
__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, MOE_WAVE);
    return v;
}
__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, MOE_WAVE));
    return v;
}
__device__ __forceinline__ int wave_sum_i(int v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, MOE_WAVE);
    return v;
}

// ---- host-side helpers -------------------------------------------------------
static inline size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }
static inline int ceil_div(int a, int b) { return (a + b - 1) / b; }
static inline size_t elem_bytes(int dtype) { return dtype == MOE_BF16 ? 2 : 4; }

// Validates the shape limits documented in moe_hip.h.
static inline int check_shape(const moe_shape* s) {
    // every entry point starts here: an error that an earlier, unrelated HIP call left behind is
    // dropped now, so that launch_status() at the end reports this call's launches only
    (void)hipGetLastError();
    if (!s) return MOE_ERR_NULL;
    if (s->dtype != MOE_F32 && s->dtype != MOE_BF16) return MOE_ERR_DTYPE;
    if (s->act != MOE_RELU && s->act != MOE_GELU) return MOE_ERR_DTYPE;
    if (s->T < 1 || s->d_model < 1 || s->d_ff < 1 || s->E < 1 || s->capacity < 1) return MOE_ERR_SHAPE;
    if (s->k < 1 || s->k > 2 || s->E < s->k || s->E > 256) return MOE_ERR_SHAPE;
    if (s->d_model % 8 || s->d_ff % 8) return MOE_ERR_SHAPE;
    if ((int64_t)s->T * s->k >= (1 << 30) || (int64_t)s->E * s->capacity >= (1 << 30)) return MOE_ERR_SHAPE;
    return MOE_OK;
}
// A kernel that uses more than 64 KB of the CU's 160 KB LDS has to opt in, once per kernel
// instance and device (`done` is that instance's bit mask over device ids).
static inline bool lds_opt_in(const void* kern, size_t smem, unsigned long long* done) {
    if (smem <= 64 * 1024) return true;
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return false;
    if (__atomic_load_n(done, __ATOMIC_ACQUIRE) >> dev & 1ull) return true;
    if (hipFuncSetAttribute(kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem) != hipSuccess) {
        (void)hipGetLastError();
        return false;
    }
    __atomic_fetch_or(done, 1ull << dev, __ATOMIC_RELEASE);
    return true;
}

static inline int launch_status() { return hipGetLastError() == hipSuccess ? MOE_OK : MOE_ERR_LAUNCH; }

// Workspace layouts (bytes), shared by moe_workspace_bytes and the entry points.
size_t route_ws_bytes(const moe_shape* s);
size_t ffn_bwd_ws_bytes(const moe_shape* s);
size_t gate_logits_bwd_ws_bytes(const moe_shape* s);
size_t aux_loss_ws_bytes(const moe_shape* s);
