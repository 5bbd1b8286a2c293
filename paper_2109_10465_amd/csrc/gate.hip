// Gate projection and the gate's backward (Sec. 3.2: one gate matrix column per
// expert; Sec. 5.1: top-1 / top-2 gating).  Results have fp32 accuracy: fp32
// activations run on the fp32 matrix pipe; bf16 activations run on the bf16 pipe
// with every fp32 operand split into bf16 parts whose products are exact in fp32.
// Reductions run in a fixed order so results are bit-reproducible.
#include "moe_common.h"

// ---------------------------------------------------------------------------
// logits[T,E] = x[T,d] * Wg[d,E] (+ bias)   on the matrix pipe
// Workgroup: 32 tokens x all experts, 8 waves that split the reduction over d.
// v_mfma_f32_32x32x2_f32: lane (r = l%32, h = l/32) supplies A[token r][k] and
// B[k][expert r] for ONE k per instruction.  The order of a reduction is free,
// so a lane's 8 consecutive x values (one 16-byte load for bf16) serve 8
// instructions: in a 16-deep block, instruction s uses k = 8h + s.
// v_mfma_f32_32x32x16_bf16 takes exactly those 8 values per lane in one step.
// Wg (L2 resident) is read as 128-byte rows.  All loads of a group of blocks are in
// flight before the first MFMA; other waves cover the latency.  The 8 partial
// tiles are added in wave order through LDS, so the result is reproducible.
// ---------------------------------------------------------------------------
#define GLM_KSPLIT 8
typedef float glm_f32x16 __attribute__((ext_vector_type(16)));

template <typename T>
__device__ __forceinline__ void load8(__amdgpu_buffer_rsrc_t rs, uint32_t off, float (&v)[8]);
template <>
__device__ __forceinline__ void load8<bf16_t>(__amdgpu_buffer_rsrc_t rs, uint32_t off, float (&v)[8]) {
    BufChunk<bf16_t>::load(rs, off, v);
}
template <>
__device__ __forceinline__ void load8<float>(__amdgpu_buffer_rsrc_t rs, uint32_t off, float (&v)[8]) {
    float lo[4], hi[4];
    BufChunk<float>::load(rs, off, lo);
    BufChunk<float>::load(rs, off == BUF_OOB ? BUF_OOB : off + 16, hi);
#pragma unroll
    for (int i = 0; i < 4; ++i) { v[i] = lo[i]; v[4 + i] = hi[i]; }
}

// TT = 32-token tiles per workgroup: with more than 32 experts every workgroup reads all of
// Wg (E * d * 4 bytes, from L2) once, so two token tiles share each of its fragments.
template <typename T, int NB, bool JIT, int TT>   // JIT: gate jitter on (a separate instance keeps the plain one lean)
__global__ __launch_bounds__(64 * GLM_KSPLIT, NB == 1 ? 4 : 2) void gate_logits_kernel(
    int Tn, int d, int E, const T* __restrict__ x, const float* __restrict__ Wg,
    const float* __restrict__ bias, float* __restrict__ logits, float jitter_eps, uint64_t seed) {
    constexpr int GRP = NB <= 2 && TT == 1 ? 8 : 4;   // 16-deep blocks whose loads are in flight together
    __shared__ float red[GLM_KSPLIT][32][33];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int r = lane & 31, h = lane >> 5;
    const int t0 = blockIdx.x * 32 * TT;
    const int rows_here = min(32 * TT, Tn - t0);
    const __amdgpu_buffer_rsrc_t rs_x = buf_rsrc(x + (size_t)t0 * d, (size_t)rows_here * d * sizeof(T));
    const __amdgpu_buffer_rsrc_t rs_w = buf_rsrc(Wg, (size_t)d * E * 4);
    const int nblk = (d + 15) / 16;
    const int per_wave = (nblk + GLM_KSPLIT - 1) / GLM_KSPLIT;
    const int b_lo = wave * per_wave, b_hi = min(nblk, b_lo + per_wave);
    glm_f32x16 acc[TT][NB];
#pragma unroll
    for (int tt = 0; tt < TT; ++tt)
#pragma unroll
        for (int nb = 0; nb < NB; ++nb)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[tt][nb][v] = 0.0f;
    // bf16 activations (no jitter): x goes to the bf16 matrix pipe as loaded and Wg as
    // three bf16 parts that add up to it exactly, so the fp32 result is kept at a
    // fraction of the fp32 pipe's time (one 32x32x16 step per part instead of eight 32x32x2)
    constexpr bool SPLIT = sizeof(T) == 2 && !JIT;
    for (int b0 = b_lo; b0 < b_hi; b0 += GRP) {
        float a[SPLIT ? 1 : TT][SPLIT ? 1 : GRP][8];
        u32x4_buf_t araw[SPLIT ? TT : 1][SPLIT ? GRP : 1];
#pragma unroll
        for (int tt = 0; tt < TT; ++tt)
#pragma unroll
            for (int u = 0; u < GRP; ++u) {
                const int k = (b0 + u) * 16 + 8 * h;
                const bool ok = b0 + u < b_hi && k < d;     // rows beyond T fall outside rs_x
                const uint32_t off = ok ? (uint32_t)(((tt * 32 + r) * d + k) * sizeof(T)) : BUF_OOB;
                if constexpr (SPLIT) araw[tt][u] = __builtin_amdgcn_raw_buffer_load_b128(rs_x, off, 0, 0);
                else load8<T>(rs_x, off, a[tt][u]);
            }
        if constexpr (JIT) {   // the gate sees x * noise
#pragma unroll
            for (int tt = 0; tt < TT; ++tt)
#pragma unroll
                for (int u = 0; u < GRP; ++u)
                    jitter_scale<8>(a[tt][u], (size_t)(t0 + tt * 32 + r) * d + (b0 + u) * 16 + 8 * h, jitter_eps, seed);
        }
#pragma unroll
        for (int nb = 0; nb < NB; ++nb) {
            float bw[GRP][8];
            const bool col_ok = nb * 32 + r < E;
#pragma unroll
            for (int u = 0; u < GRP; ++u)
#pragma unroll
                for (int s_ = 0; s_ < 8; ++s_) {
                    const int k = (b0 + u) * 16 + 8 * h + s_;   // rows beyond d fall outside rs_w
                    const bool ok = col_ok && b0 + u < b_hi;
                    bw[u][s_] = buf_load_f32(rs_w, ok ? (uint32_t)((k * E + nb * 32 + r) * 4) : BUF_OOB);
                }
#pragma unroll
            for (int u = 0; u < GRP; ++u) {
                if constexpr (SPLIT) {
                    bf16x8_hw_t w_hi, w_mid, w_lo;
                    split3_bf16(bw[u], w_hi, w_mid, w_lo);
#pragma unroll
                    for (int tt = 0; tt < TT; ++tt) {
                        const bf16x8_hw_t xa = __builtin_bit_cast(bf16x8_hw_t, araw[tt][u]);
                        acc[tt][nb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(xa, w_lo, acc[tt][nb], 0, 0, 0);
                        acc[tt][nb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(xa, w_mid, acc[tt][nb], 0, 0, 0);
                        acc[tt][nb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(xa, w_hi, acc[tt][nb], 0, 0, 0);
                    }
                } else {
#pragma unroll
                    for (int tt = 0; tt < TT; ++tt)
#pragma unroll
                        for (int s_ = 0; s_ < 8; ++s_)
                            acc[tt][nb] = __builtin_amdgcn_mfma_f32_32x32x2f32(a[tt][u][s_], bw[u][s_], acc[tt][nb], 0, 0, 0);
                }
            }
        }
    }
    // accumulator element v of lane l: expert column l%32, token row 8*(v/4) + 4*(l/32) + v%4
#pragma unroll
    for (int tt = 0; tt < TT; ++tt)
#pragma unroll
        for (int nb = 0; nb < NB; ++nb) {
            if (tt + nb) __syncthreads();
#pragma unroll
            for (int v = 0; v < 16; ++v) red[wave][8 * (v >> 2) + 4 * h + (v & 3)][r] = acc[tt][nb][v];
            __syncthreads();
#pragma unroll
            for (int o = threadIdx.x; o < 32 * 32; o += 64 * GLM_KSPLIT) {
                const int m = tt * 32 + (o >> 5), n = o & 31, e = nb * 32 + n;
                float sum = 0.0f;
#pragma unroll
                for (int w = 0; w < GLM_KSPLIT; ++w) sum += red[w][o >> 5][n];
                if (m < rows_here && e < E) logits[(size_t)(t0 + m) * E + e] = sum + (bias ? bias[e] : 0.0f);
            }
        }
}

// ---------------------------------------------------------------------------
// The same product for bf16 activations and 33..128 experts (E % 4 == 0, no
// jitter), tiled like a GEMM: with that many experts the gate matrix (d x E fp32)
// is the larger operand of a token tile, and splitting it into bf16 parts costs
// about as much vector-ALU time as the product costs matrix-pipe time, so both must
// be done once per workgroup, not once per wave or per 32 tokens, and side by side.
// Workgroup: 32*TT tokens x all experts, reduction in 64-deep slabs through a
// two-stage LDS ring, 12 waves in two roles (two producers and one consumer per SIMD,
// so the splitting of one slab runs under the MFMAs of the previous one):
//   producers (waves 0-7) move a slab global -> registers -> LDS.  x: rows of 128
//       bytes, 16-byte pieces XOR-swizzled so that a fragment read (32 rows x 16
//       bytes) touches every bank once.  Wg: a thread loads rows 4kg..4kg+3 of expert
//       quad 4q..4q+3 (16-byte loads, a wave instruction = two whole 512-byte rows),
//       splits the 16 values exactly into three bf16 parts and writes them where
//       the MFMA wants them: operand j (j = 0..3) stands for the experts 4r+j,
//       r = tile column, so the four values of a load go to four operands and the
//       four rows to four consecutive reduction entries of one lane: 8-byte LDS
//       writes, contiguous over the wave; an operand is read back as 1 KB, 16
//       bytes per lane.  The registers of two slabs are in flight (loads are
//       issued two iterations before their values are used).
//   consumers (waves 8-11) multiply: wave 8+j takes operand j over the whole slab
//       for all TT token tiles (a B fragment serves TT MFMAs per part).
// One barrier per slab.  At the end the tiles go through LDS and a thread stores
// 4 consecutive experts of a token as 16 bytes.
// ---------------------------------------------------------------------------
#define GLL_BK 64
#define GLL_PRODUCERS 512                 // threads in the producer role (8 waves)
#define GLL_THREADS (GLL_PRODUCERS + 256) // + one consumer wave per SIMD
#define GLL_LDO 132                       // floats per token row of the output stage
template <int TT>
struct GllSmem {
    static constexpr int XB = TT * 32 * GLL_BK * 2;         // x slab
    static constexpr int WB = 4 * (GLL_BK / 16) * 3 * 1024; // 4 operands x 4 steps x 3 parts x 1 KB
    static constexpr int STAGE = XB + WB;
    static constexpr int OUT = TT * 32 * GLL_LDO * 4;
    static constexpr int BYTES = 2 * STAGE > OUT ? 2 * STAGE : OUT;
};

template <int TT>
__global__ __launch_bounds__(GLL_THREADS, 1) void gate_logits_lds_kernel(
    int Tn, int d, int E, const bf16_t* __restrict__ x, const float* __restrict__ Wg,
    const float* __restrict__ bias, float* __restrict__ logits) {
    typedef GllSmem<TT> SM;
    extern __shared__ __align__(16) unsigned char gll_smem[];
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int t0 = blockIdx.x * 32 * TT;
    const int rows_here = min(32 * TT, Tn - t0);
    const int nslab = (d + GLL_BK - 1) / GLL_BK;
    // every LDS operation of this wave is complete, then the workgroup meets; loads into
    // registers stay in flight across it (a __syncthreads() would wait for them too)
    auto lds_barrier = [] { asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory"); };

    glm_f32x16 acc[TT];
    if (wave < GLL_PRODUCERS / 64) {
        // descriptors in scalar registers for the hand-issued loads (ranges below 4 GiB by the shape limits)
        u32x4_buf_t rs_x = make_desc(x + (size_t)t0 * d, (uint32_t)((size_t)rows_here * d * 2));
        u32x4_buf_t rs_w = make_desc(Wg, (uint32_t)((size_t)d * E * 4));
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            rs_x[i] = __builtin_amdgcn_readfirstlane(rs_x[i]);
            rs_w[i] = __builtin_amdgcn_readfirstlane(rs_w[i]);
        }
        constexpr int XPT = TT * 32 * 8 / GLL_PRODUCERS;    // 16-byte pieces of x per thread and slab
        struct Regs { u32x4_buf_t xr[XPT]; u32x4_buf_t wr[4]; };
        // x: piece p = row*8 + c of the slab; LDS position of piece c in its row: c ^ ((row/2)%8)
        uint32_t xoff[XPT], xdst[XPT];
        int xcol[XPT];
#pragma unroll
        for (int i = 0; i < XPT; ++i) {
            const int p = threadIdx.x + i * GLL_PRODUCERS;
            const int row = p >> 3, c = p & 7;
            xoff[i] = (uint32_t)((row * d + c * 8) * 2);   // rows beyond T lie beyond the descriptor
            xcol[i] = c * 8;
            xdst[i] = (uint32_t)((row * 8 + (c ^ ((row >> 1) & 7))) * 16);
        }
        // Wg: this thread's quad of experts and its group of four rows of a slab
        const int q = threadIdx.x & 31, kg0 = threadIdx.x >> 5;
        const bool q_ok = 4 * q < E;                        // E % 4 == 0: a quad is inside or beyond
        // The loads are issued by hand and their completion is awaited by hand (land): three
        // slabs are in flight per thread, and the wait counts the compiler derives for loads
        // that cross a loop's back edge drain all of them.  Every slab issues the same number
        // of loads (slabs beyond d read zeros), so "two younger slabs" is a constant count.
        constexpr int LOADS = 4 + XPT;
        auto issue1 = [](u32x4_buf_t rs, uint32_t off) {
            u32x4_buf_t v;
            asm volatile("buffer_load_dwordx4 %0, %1, %2, 0 offen" : "=v"(v) : "v"(off), "s"(rs) : "memory");
            return v;
        };
        // Workgroups start at different slabs and wrap around: in step they would all read the
        // same 128-byte column of their rows, addresses a row pitch apart, i.e. a fraction of the
        // memory channels at any one time.
        const int rot = blockIdx.x % nslab;
        auto load_slab = [&](int s, Regs& g) {
            const int sr = s + rot - (s + rot >= nslab ? nslab : 0);
            const int k0 = s < nslab ? sr * GLL_BK : d;     // slabs beyond the last read zeros
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const int k = k0 + 4 * kg0 + i;
                g.wr[i] = issue1(rs_w, (q_ok & (k < d)) ? (uint32_t)((k * E + 4 * q) * 4) : BUF_OOB);
            }
#pragma unroll
            for (int i = 0; i < XPT; ++i)
                g.xr[i] = issue1(rs_x, (xcol[i] + k0 < d) ? xoff[i] + (uint32_t)(k0 * 2) : BUF_OOB);
        };
        // waits until at most 2 * LOADS loads are outstanding: slab g has landed; the asm "modifies"
        // the registers so that no use of them can be scheduled above it
        auto land = [&](Regs& g) {
            if constexpr (XPT == 2)
                asm volatile("s_waitcnt vmcnt(%6)" : "+v"(g.wr[0]), "+v"(g.wr[1]), "+v"(g.wr[2]), "+v"(g.wr[3]),
                             "+v"(g.xr[0]), "+v"(g.xr[XPT - 1]) : "n"(2 * LOADS) : "memory");
            else
                asm volatile("s_waitcnt vmcnt(%5)" : "+v"(g.wr[0]), "+v"(g.wr[1]), "+v"(g.wr[2]), "+v"(g.wr[3]),
                             "+v"(g.xr[0]) : "n"(2 * LOADS) : "memory");
        };
        // rows 4kg..4kg+3 are reduction entries 4*(kg%2) .. +3 of lane q + 32*((kg/2)%2) in step kg/4
        const uint32_t wdst = (uint32_t)(((kg0 >> 2) * 3) * 1024 + (q + 32 * ((kg0 >> 1) & 1)) * 16 + (kg0 & 1) * 8);
        auto store_slab = [&](const Regs& g, int stage) {
            unsigned char* sx = gll_smem + stage * SM::STAGE;
#pragma unroll
            for (int i = 0; i < XPT; ++i) *reinterpret_cast<u32x4_buf_t*>(sx + xdst[i]) = g.xr[i];
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                uint32_t ph[4], pm[4], pl[4];
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    const float w = __uint_as_float(g.wr[i][j]);
                    ph[i] = __float_as_uint(w) & 0xffff0000u;
                    const float w1 = w - __uint_as_float(ph[i]);
                    pm[i] = __float_as_uint(w1) & 0xffff0000u;
                    pl[i] = __float_as_uint(w1 - __uint_as_float(pm[i]));
                }
                unsigned char* dst = sx + SM::XB + wdst + j * (GLL_BK / 16) * 3 * 1024;
                // the high halves of two words, the earlier reduction entry in the low half
                constexpr uint32_t HH = 0x07060302u;
                *reinterpret_cast<uint2*>(dst) =
                    make_uint2(__builtin_amdgcn_perm(ph[1], ph[0], HH), __builtin_amdgcn_perm(ph[3], ph[2], HH));
                *reinterpret_cast<uint2*>(dst + 1024) =
                    make_uint2(__builtin_amdgcn_perm(pm[1], pm[0], HH), __builtin_amdgcn_perm(pm[3], pm[2], HH));
                *reinterpret_cast<uint2*>(dst + 2048) =
                    make_uint2(__builtin_amdgcn_perm(pl[1], pl[0], HH), __builtin_amdgcn_perm(pl[3], pl[2], HH));
            }
        };
        static_assert(XPT == 1 || XPT == 2, "land() names every register of a slab");
        Regs g0, g1, g2;
        load_slab(0, g0);
        load_slab(1, g1);
        load_slab(2, g2);
        land(g0);
        store_slab(g0, 0);
        load_slab(3, g0);
        lds_barrier();                   // slab 0 is staged
        // step n (the consumers multiply slab n): stage slab n+1, request slab n+4
        auto step = [&](int n, Regs& g) {
            land(g);
            store_slab(g, (n + 1) & 1);  // that stage was last read before the previous barrier
            load_slab(n + 4, g);
            lds_barrier();
        };
        for (int s = 0;; s += 3) {
            step(s, g1);
            if (s + 1 >= nslab) break;
            step(s + 1, g2);
            if (s + 2 >= nslab) break;
            step(s + 2, g0);
            if (s + 3 >= nslab) break;
        }
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");   // nothing may land in a register that is reused below
    } else {
        const int r = lane & 31, h = lane >> 5;
        const int jw = wave - GLL_PRODUCERS / 64;
#pragma unroll
        for (int tt = 0; tt < TT; ++tt)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[tt][v] = 0.0f;
        auto compute = [&](int stage) {
            const unsigned char* sx = gll_smem + stage * SM::STAGE;
            const unsigned char* sw = sx + SM::XB + jw * (GLL_BK / 16) * 3 * 1024 + lane * 16;
#pragma unroll
            for (int ks = 0; ks < GLL_BK / 16; ++ks) {
                const bf16x8_hw_t w_hi = *reinterpret_cast<const bf16x8_hw_t*>(sw + (ks * 3 + 0) * 1024);
                const bf16x8_hw_t w_mid = *reinterpret_cast<const bf16x8_hw_t*>(sw + (ks * 3 + 1) * 1024);
                const bf16x8_hw_t w_lo = *reinterpret_cast<const bf16x8_hw_t*>(sw + (ks * 3 + 2) * 1024);
                bf16x8_hw_t xa[TT];
#pragma unroll
                for (int tt = 0; tt < TT; ++tt) {
                    const int row = tt * 32 + r;
                    xa[tt] = *reinterpret_cast<const bf16x8_hw_t*>(sx + (row * 8 + ((2 * ks + h) ^ ((row >> 1) & 7))) * 16);
                }
#pragma unroll
                for (int tt = 0; tt < TT; ++tt) acc[tt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(xa[tt], w_lo, acc[tt], 0, 0, 0);
#pragma unroll
                for (int tt = 0; tt < TT; ++tt) acc[tt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(xa[tt], w_mid, acc[tt], 0, 0, 0);
#pragma unroll
                for (int tt = 0; tt < TT; ++tt) acc[tt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(xa[tt], w_hi, acc[tt], 0, 0, 0);
            }
        };
        lds_barrier();
        for (int s = 0; s < nslab; s += 2) {
            compute(0);
            lds_barrier();
            if (s + 1 >= nslab) break;
            compute(1);
            lds_barrier();
        }
        // accumulator element v of lane l: expert 4*(l%32) + jw, token row 8*(v/4) + 4*(l/32) + v%4
        float* out = reinterpret_cast<float*>(gll_smem);
#pragma unroll
        for (int tt = 0; tt < TT; ++tt)
#pragma unroll
            for (int v = 0; v < 16; ++v)
                out[(tt * 32 + 8 * (v >> 2) + 4 * h + (v & 3)) * GLL_LDO + 4 * r + jw] = acc[tt][v];
    }
    __syncthreads();
    if (threadIdx.x < 512) {
        const int q = threadIdx.x & 31, m0 = threadIdx.x >> 5;
        const bool q_ok = 4 * q < E;
        const float* o0 = reinterpret_cast<const float*>(gll_smem);
        float4 b4 = make_float4(0.0f, 0.0f, 0.0f, 0.0f);
        if (bias && q_ok) b4 = *reinterpret_cast<const float4*>(bias + 4 * q);
#pragma unroll
        for (int i = 0; i < TT * 32 * 32 / 512; ++i) {
            const int m = m0 + 16 * i;                      // token row; q = expert quad
            const float4 a = *reinterpret_cast<const float4*>(o0 + m * GLL_LDO + 4 * q);
            if (m < rows_here && q_ok)
                *reinterpret_cast<float4*>(logits + (size_t)(t0 + m) * E + 4 * q) =
                    make_float4(a.x + b4.x, a.y + b4.y, a.z + b4.z, a.w + b4.w);
        }
    }
}

template <int TT>
static bool launch_gate_logits_lds(const moe_shape* s, const void* x, const float* Wg, const float* bias,
                                   float* logits, hipStream_t st) {
    static unsigned long long opted = 0;
    if (!lds_opt_in((const void*)gate_logits_lds_kernel<TT>, GllSmem<TT>::BYTES, &opted)) return false;
    gate_logits_lds_kernel<TT><<<ceil_div(s->T, 32 * TT), GLL_THREADS, GllSmem<TT>::BYTES, st>>>(
        s->T, s->d_model, s->E, (const bf16_t*)x, Wg, bias, logits);
    return true;
}

template <typename T>
static bool launch_gate_logits(const moe_shape* s, const void* x, const float* Wg, const float* bias,
                               float* logits, float eps, uint64_t seed, hipStream_t st) {
    if constexpr (sizeof(T) == 2) {
        // bias rows are read as 16 bytes: the pointer must be 16-byte aligned like every tensor here
        if (eps == 0.0f && s->E > 32 && s->E <= 128 && s->E % 4 == 0 && ((uintptr_t)logits & 15) == 0 &&
            ((uintptr_t)bias & 15) == 0 && ((uintptr_t)Wg & 15) == 0) {
            // 128 tokens per workgroup when that still gives most compute units a workgroup
            if (ceil_div(s->T, 128) >= 192) return launch_gate_logits_lds<4>(s, x, Wg, bias, logits, st);
            return launch_gate_logits_lds<2>(s, x, Wg, bias, logits, st);
        }
    }
    // two token tiles per workgroup on the bf16 matrix path with more than 32 experts
#define GLM(NB, JIT, TT) gate_logits_kernel<T, NB, JIT, TT><<<ceil_div(s->T, 32 * TT), 64 * GLM_KSPLIT, 0, st>>>( \
    s->T, s->d_model, s->E, (const T*)x, Wg, bias, logits, eps, seed)
    constexpr int TT2 = sizeof(T) == 2 ? 2 : 1;
    if (eps != 0.0f) {
        if (s->E <= 32) GLM(1, true, 1); else if (s->E <= 64) GLM(2, true, 1);
        else if (s->E <= 128) GLM(4, true, 1); else GLM(8, true, 1);
    } else {
#ifndef MOE_GATE_TT32
#define MOE_GATE_TT32 2   // two 32-token tiles share each Wg fragment (measured: 15.7 -> 14.2 us at T = 16384, E = 32; four: slower)
#endif
        constexpr int TT32 = sizeof(T) == 2 ? MOE_GATE_TT32 : 1;
        if (s->E <= 32) GLM(1, false, TT32); else if (s->E <= 64) GLM(2, false, TT2);
        else if (s->E <= 128) GLM(4, false, TT2); else GLM(8, false, 1);
    }
#undef GLM
    return true;
}

static int gate_logits_impl(const moe_shape* shape, const void* x, const float* Wg,
                            const float* bias_or_null, float eps, uint64_t seed, float* logits, void* stream) {
    int rc = check_shape(shape);
    if (rc) return rc;
    if (!x || !Wg || !logits) return MOE_ERR_NULL;
    if (!(eps >= 0.0f && eps < 1.0f)) return MOE_ERR_SHAPE;
    const bool ok = shape->dtype == MOE_BF16
        ? launch_gate_logits<bf16_t>(shape, x, Wg, bias_or_null, logits, eps, seed, (hipStream_t)stream)
        : launch_gate_logits<float>(shape, x, Wg, bias_or_null, logits, eps, seed, (hipStream_t)stream);
    return ok ? launch_status() : MOE_ERR_LAUNCH;
}

extern "C" int moe_gate_logits(const moe_shape* shape, const void* x, const float* Wg,
                               const float* bias_or_null, float* logits, void* stream) {
    return gate_logits_impl(shape, x, Wg, bias_or_null, 0.0f, 0, logits, stream);
}

extern "C" int moe_gate_logits_jitter(const moe_shape* shape, const void* x, const float* Wg,
                                      const float* bias_or_null, float jitter_eps, uint64_t seed,
                                      float* logits, void* stream) {
    return gate_logits_impl(shape, x, Wg, bias_or_null, jitter_eps, seed, logits, stream);
}

// ---------------------------------------------------------------------------
// dlogits from dgate_w (derivative of the gate weights and the softmax)
// ---------------------------------------------------------------------------
template <int V>   // V consecutive experts of one token per thread (V = 4 needs E % 4 == 0)
__global__ __launch_bounds__(256) void gate_bwd_kernel(
    int Tn, int E, int k, const float* __restrict__ dgate_w, const float* __restrict__ probs,
    const int32_t* __restrict__ expert_idx, const int32_t* __restrict__ slot,
    float* __restrict__ dlogits) {
    const size_t idx = ((size_t)blockIdx.x * 256 + threadIdx.x) * V;
    if (idx >= (size_t)Tn * E) return;
    const int t = (int)(idx / E), e = (int)(idx - (size_t)t * E);
    const float* pr = probs + (size_t)t * E;
    float pe[V];
    if constexpr (V == 4) {
        const float4 q = *reinterpret_cast<const float4*>(pr + e);
        pe[0] = q.x; pe[1] = q.y; pe[2] = q.z; pe[3] = q.w;
    } else {
        pe[0] = pr[e];
    }
    float dp0 = 0.0f, dp1 = 0.0f, sum = 0.0f;
    int e0, e1 = -1;
    if (k == 1) {
        e0 = expert_idx[t];
        dp0 = slot[t] >= 0 ? dgate_w[t] : 0.0f;
        sum = pr[e0] * dp0;
    } else {
        e0 = expert_idx[2 * t];
        e1 = expert_idx[2 * t + 1];
        const float dg0 = slot[2 * t] >= 0 ? dgate_w[2 * t] : 0.0f;
        const float dg1 = slot[2 * t + 1] >= 0 ? dgate_w[2 * t + 1] : 0.0f;
        const float p0 = pr[e0], p1 = pr[e1];
        const float S = p0 + p1;
        dp0 = p1 * (dg0 - dg1) / (S * S);
        dp1 = p0 * (dg1 - dg0) / (S * S);
        sum = p0 * dp0 + p1 * dp1;
    }
    float out[V];
#pragma unroll
    for (int i = 0; i < V; ++i) {
        const float dp_e = e + i == e0 ? dp0 : (e + i == e1 ? dp1 : 0.0f);
        out[i] = pe[i] * (dp_e - sum);
    }
    if constexpr (V == 4) *reinterpret_cast<float4*>(dlogits + idx) = make_float4(out[0], out[1], out[2], out[3]);
    else dlogits[idx] = out[0];
}

extern "C" int moe_gate_bwd(const moe_shape* shape, const float* dgate_w, const float* probs,
                            const int32_t* expert_idx, const int32_t* slot, float* dlogits,
                            void* stream) {
    int rc = check_shape(shape);
    if (rc) return rc;
    if (!dgate_w || !probs || !expert_idx || !slot || !dlogits) return MOE_ERR_NULL;
    const size_t n = (size_t)shape->T * shape->E;
    if (shape->E % 4 == 0)
        gate_bwd_kernel<4><<<(unsigned)((n / 4 + 255) / 256), 256, 0, (hipStream_t)stream>>>(
            shape->T, shape->E, shape->k, dgate_w, probs, expert_idx, slot, dlogits);
    else
        gate_bwd_kernel<1><<<(unsigned)((n + 255) / 256), 256, 0, (hipStream_t)stream>>>(
            shape->T, shape->E, shape->k, dgate_w, probs, expert_idx, slot, dlogits);
    return launch_status();
}

// ---------------------------------------------------------------------------
// dWg[d,E] = x^T dlogits   on the matrix pipe: partial sums over token
// chunks, then an ordered sum over the chunks.
// Workgroup: 256 columns of d x 32 experts x one chunk of tokens, 4 waves that
// split the chunk's tokens.  The reduction runs over tokens, two per MFMA (one
// per lane half).  A lane loads 8 consecutive columns of its token (16 bytes for
// bf16) and feeds them to 8 MFMAs: in MFMA c, tile row m stands for column
// i0 + 8m + c, so the 8 accumulator tiles cover 256 columns and every load is a
// contiguous 512-byte piece of a token row.  B = the token's dlogits row.
// ---------------------------------------------------------------------------
#define GW_COLS 256
#define GW_WAVES 4

static inline int gw_chunks(const moe_shape* s) {
    // enough workgroups to fill the chip twice, at least 256 tokens per chunk
    int want = ceil_div(512, ceil_div(s->d_model, GW_COLS) * ceil_div(s->E, 32));
    int maxc = ceil_div(s->T, 256);
    int n = want < maxc ? want : maxc;
    // one chunk's rows of x are addressed with 32-bit byte offsets: keep it below 1 GiB
    const int minc = (int)(((size_t)s->T * s->d_model * 4 + ((size_t)1 << 30) - 1) >> 30);
    if (n < minc) n = minc;
    return n < 1 ? 1 : n;
}
// tokens per chunk: a multiple of 2 tokens per wave
static inline int gw_chunk_tokens(const moe_shape* s) {
    return ceil_div(ceil_div(s->T, gw_chunks(s)), 2 * GW_WAVES) * 2 * GW_WAVES;
}
size_t gate_logits_bwd_ws_bytes(const moe_shape* s) {
    return align_up((size_t)ceil_div(s->T, gw_chunk_tokens(s)) * s->d_model * s->E * 4, 256);
}

#ifndef GW_MINB
#define GW_MINB 2
#endif
template <typename T, bool JIT>
__global__ __launch_bounds__(64 * GW_WAVES, JIT ? 1 : GW_MINB) void gate_dwg_partial_kernel(
    int Tn, int d, int E, int tok_per_chunk, const T* __restrict__ x,
    const float* __restrict__ dlogits, float* __restrict__ partial, float jitter_eps, uint64_t seed) {
    extern __shared__ __align__(16) float gw_red[];      // [2][256 columns][32 experts]
    constexpr int GRP = 4;                               // token pairs whose loads are in flight together (x2 buffers)
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int r = lane & 31, h = lane >> 5;
    const int bx = blockIdx.x, by = blockIdx.y, bz = blockIdx.z;
    const int i0 = bx * GW_COLS, e0 = bz * 32;
    const int tbeg = by * tok_per_chunk;
    const int tend = min(Tn, tbeg + tok_per_chunk);
    const int per_wave = tok_per_chunk / GW_WAVES;
    const int w_lo = tbeg + wave * per_wave, w_hi = min(tend, w_lo + per_wave);
    const int nrows = max(tend - tbeg, 0);
    const __amdgpu_buffer_rsrc_t rs_x = buf_rsrc(x + (size_t)tbeg * d, (size_t)nrows * d * sizeof(T));
    const __amdgpu_buffer_rsrc_t rs_d = buf_rsrc(dlogits + (size_t)tbeg * E, (size_t)nrows * E * 4);
    const int col = i0 + 8 * r;
    const bool col_ok = col < d, e_ok = e0 + r < E;      // d % 8 == 0: 8 columns are inside or wholly beyond
    glm_f32x16 acc[8];
#pragma unroll
    for (int c = 0; c < 8; ++c)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[c][v] = 0.0f;
    if constexpr (sizeof(T) == 2 && !JIT) {
        // bf16 activations on the bf16 matrix pipe (32x32x16: a lane supplies 8 consecutive
        // k = tokens).  A lane loads 8 columns x 8 tokens (one 16-byte load per token),
        // transposes the 8x8 block in registers (one byte permute per packed pair) into the
        // 8 operands "column 8r+c of tokens 8h..8h+7", and multiplies each with dlogits split
        // exactly into three bf16 parts: 24 steps of 32 cycles per 16 tokens instead of 64 of 64.
        auto fetch16 = [&](int t, u32x4_buf_t (&fx)[8], float (&fd)[8]) {
#pragma unroll
            for (int s_ = 0; s_ < 8; ++s_) {
                const int tok = t + 8 * h + s_;
                const bool ok = tok < w_hi;              // the next wave's tokens are not ours
                fx[s_] = __builtin_amdgcn_raw_buffer_load_b128(
                    rs_x, ok && col_ok ? (uint32_t)(((tok - tbeg) * d + col) * sizeof(T)) : BUF_OOB, 0, 0);
                fd[s_] = buf_load_f32(rs_d, ok && e_ok ? (uint32_t)(((tok - tbeg) * E + e0 + r) * 4) : BUF_OOB);
            }
        };
        auto multiply16 = [&](const u32x4_buf_t (&fx)[8], const float (&fd)[8]) {
            bf16x8_hw_t d_hi, d_mid, d_lo;
            split3_bf16(fd, d_hi, d_mid, d_lo);
#pragma unroll
            for (int c = 0; c < 8; ++c) {
                u32x4_buf_t q;
#pragma unroll
                for (int w = 0; w < 4; ++w)   // tokens 2w (low half) and 2w+1 (high half) at column c
                    q[w] = __builtin_amdgcn_perm(fx[2 * w + 1][c >> 1], fx[2 * w][c >> 1],
                                                 (c & 1) ? 0x07060302u : 0x05040100u);
                const bf16x8_hw_t xa = __builtin_bit_cast(bf16x8_hw_t, q);
                acc[c] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(xa, d_lo, acc[c], 0, 0, 0);
                acc[c] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(xa, d_mid, acc[c], 0, 0, 0);
                acc[c] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(xa, d_hi, acc[c], 0, 0, 0);
            }
        };
        // two register buffers: the loads of the next 16 tokens travel under this group's MFMAs
        // (more requests in flight only queue up: the first data then arrives later)
        u32x4_buf_t xa0[8], xa1[8];
        float dl0[8], dl1[8];
        fetch16(w_lo, xa0, dl0);
        for (int t = w_lo; t < w_hi; t += 32) {
            fetch16(t + 16, xa1, dl1);       // beyond w_hi: every lane reads zeros, harmless
            multiply16(xa0, dl0);
            fetch16(t + 32, xa0, dl0);
            multiply16(xa1, dl1);
        }
    } else {
    // two register buffers: the loads of the next group travel under this group's MFMAs
    float a[2][GRP][8], b[2][GRP];
    auto fetch = [&](int t, float (&fa)[GRP][8], float (&fb)[GRP]) {
#pragma unroll
        for (int u = 0; u < GRP; ++u) {
            const int tok = t + 2 * u + h;
            const bool ok = tok < w_hi;                  // the next wave's tokens are not ours
            load8<T>(rs_x, ok && col_ok ? (uint32_t)(((tok - tbeg) * d + col) * sizeof(T)) : BUF_OOB, fa[u]);
            fb[u] = buf_load_f32(rs_d, ok && e_ok ? (uint32_t)(((tok - tbeg) * E + e0 + r) * 4) : BUF_OOB);
        }
    };
    auto multiply = [&](int t, float (&fa)[GRP][8], const float (&fb)[GRP]) {
        if constexpr (JIT) {   // dWg = (x * noise)^T dlogits
#pragma unroll
            for (int u = 0; u < GRP; ++u)
                jitter_scale<8>(fa[u], (size_t)(t + 2 * u + h) * d + col, jitter_eps, seed);
        }
#pragma unroll
        for (int u = 0; u < GRP; ++u)
#pragma unroll
            for (int c = 0; c < 8; ++c) acc[c] = __builtin_amdgcn_mfma_f32_32x32x2f32(fa[u][c], fb[u], acc[c], 0, 0, 0);
    };
    fetch(w_lo, a[0], b[0]);
    for (int t = w_lo; t < w_hi; t += 4 * GRP) {
        fetch(t + 2 * GRP, a[1], b[1]);      // beyond w_hi: every lane reads zeros, harmless
        multiply(t, a[0], b[0]);
        fetch(t + 4 * GRP, a[0], b[0]);
        multiply(t + 2 * GRP, a[1], b[1]);
    }
    }
    // accumulator v of tile c, lane l: column i0 + 8*(8*(v/4) + 4*(l/32) + v%4) + c, expert e0 + l%32
    // The four waves' tiles are added as (w0 + w2) + (w1 + w3) through two staged tiles (64 KB, so
    // that two workgroups share a compute unit): waves 2, 3 stage theirs, waves 0, 1 add their own
    // in place, every thread then adds the two sums.  A fixed order: reproducible.
    static_assert(GW_WAVES == 4, "the reduction below pairs wave w with wave w + 2");
    if (wave >= 2) {
#pragma unroll
        for (int c = 0; c < 8; ++c)
#pragma unroll
            for (int v = 0; v < 16; ++v)
                gw_red[((wave - 2) * GW_COLS + 8 * (8 * (v >> 2) + 4 * h + (v & 3)) + c) * 32 + r] = acc[c][v];
    }
    __syncthreads();
    if (wave < 2) {
#pragma unroll
        for (int c = 0; c < 8; ++c) {
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                float* p = &gw_red[(wave * GW_COLS + 8 * (8 * (v >> 2) + 4 * h + (v & 3)) + c) * 32 + r];
                *p = acc[c][v] + *p;
            }
            __builtin_amdgcn_sched_barrier(0);           // one tile's 16 reads at a time
        }
    }
    __syncthreads();
    // 4 experts per thread and pass; every LDS read of the loop is issued before the first add
    constexpr int NPASS = GW_COLS * 32 / 4 / (64 * GW_WAVES);
    constexpr int NSUM = 2;
    float4 part[NPASS][NSUM];
#pragma unroll
    for (int q = 0; q < NPASS; ++q)
#pragma unroll
        for (int w = 0; w < NSUM; ++w)
            part[q][w] = *reinterpret_cast<const float4*>(
                &gw_red[(size_t)(w * GW_COLS) * 32 + (size_t)(q * 64 * GW_WAVES + threadIdx.x) * 4]);
    const bool e_vec = (E & 3) == 0;
#pragma unroll
    for (int q = 0; q < NPASS; ++q) {
        const int o = (q * 64 * GW_WAVES + threadIdx.x) * 4;
        const int il = o >> 5, e = o & 31;
        float4 sum = part[q][0];
#pragma unroll
        for (int w = 1; w < NSUM; ++w) {
            sum.x += part[q][w].x; sum.y += part[q][w].y; sum.z += part[q][w].z; sum.w += part[q][w].w;
        }
        if (i0 + il < d) {
            float* dst = partial + ((size_t)by * d + i0 + il) * E + e0 + e;
            if (e_vec && e0 + e + 3 < E) {
                *reinterpret_cast<float4*>(dst) = sum;
            } else {
                const float v4[4] = {sum.x, sum.y, sum.z, sum.w};
#pragma unroll
                for (int j = 0; j < 4; ++j)
                    if (e0 + e + j < E) dst[j] = v4[j];
            }
        }
    }
}

__global__ __launch_bounds__(256) void gate_dwg_reduce_kernel(int n, int nchunk,
                                                              const float* __restrict__ partial,
                                                              float* __restrict__ dWg) {
    const int idx = blockIdx.x * 256 + threadIdx.x;
    if (idx >= n) return;
    float s = 0.0f;
    int c = 0;
    for (; c + 8 <= nchunk; c += 8) {   // 8 independent loads in flight, added in chunk order
        float v[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) v[u] = partial[(size_t)(c + u) * n + idx];
#pragma unroll
        for (int u = 0; u < 8; ++u) s += v[u];
    }
    for (; c < nchunk; ++c) s += partial[(size_t)c * n + idx];
    dWg[idx] = s;
}

// ---------------------------------------------------------------------------
// dx[t,:] (+)= dlogits[t,:] * Wg^T   on the matrix pipe
// Workgroup: 32 tokens, 4 waves; wave w takes the 64-column passes w, w+4, ...
// of d (two 32x32 tiles, D[token][column]).  A = dlogits rows (token, all
// experts), B = Wg rows (column i, all experts): both are contiguous along the
// reduction, so a lane half reads its 16 experts of a 32-expert block as 64
// contiguous bytes (instruction s uses expert 16h+s).  For bf16 activations the
// result needs 8 bits only: both operands go to the bf16 matrix pipe as hi + lo
// pairs (three 32x32x16 steps per 16 experts instead of sixteen 32x32x2 ones,
// relative error 2^-15).  The tiles leave through a
// wave-private LDS stage so that global accesses run along the row: 16 bytes per
// lane, a whole 64-column row piece (128 or 256 bytes) per group of lanes.
// GATHER: dx is not read; the value the product is added to is dispatch's
// backward, the sum of the token's kept rows of dxd [E, C, d] (row slot[t,j] of
// expert expert_idx[t,j]; slot < 0: dropped), fetched here so that this
// intermediate never goes through memory.
// ---------------------------------------------------------------------------
template <bool VEC, int N>
__device__ __forceinline__ void load_row_f32(__amdgpu_buffer_rsrc_t rs, int row_elems, int e0, int E, float (&v)[N]) {
    // N consecutive fp32 of one row starting at element e0 of the row (row_elems = row * E)
    if constexpr (VEC) {
#pragma unroll
        for (int c = 0; c < N / 4; ++c) {
            float q[4];
            BufChunk<float>::load(rs, e0 + 4 * c < E ? (uint32_t)((row_elems + e0 + 4 * c) * 4) : BUF_OOB, q);
#pragma unroll
            for (int j = 0; j < 4; ++j) v[4 * c + j] = q[j];
        }
    } else {
#pragma unroll
        for (int j = 0; j < N; ++j)
            v[j] = buf_load_f32(rs, e0 + j < E ? (uint32_t)((row_elems + e0 + j) * 4) : BUF_OOB);
    }
}

#define GDX_WAVES 4
#define GDX_COLS 64     // columns per wave pass

template <typename T, int EB, bool VEC, bool GATHER>   // EB = 32-expert blocks (E <= 32*EB); VEC: E % 4 == 0
__global__ __launch_bounds__(64 * GDX_WAVES) void gate_dx_kernel(int Tn, int d, int E, int k, int C,
                                                                 const float* __restrict__ dlogits,
                                                                 const float* __restrict__ Wg,
                                                                 const T* __restrict__ dxd,
                                                                 const int32_t* __restrict__ expert_idx,
                                                                 const int32_t* __restrict__ slot,
                                                                 T* __restrict__ dx, float jitter_eps, uint64_t seed) {
    constexpr bool HOIST = EB <= 2;      // dlogits fragments stay in registers across passes
    constexpr int LD = GDX_COLS + 4;     // floats per staged row (16-byte aligned, rows 4 apart on other banks)
    constexpr int CN = Chunk<T>::N;      // elements per 16-byte piece
    constexpr int LPR = GDX_COLS / CN;   // lanes per staged row
    constexpr int RPI = 64 / LPR;        // rows per wave instruction
    constexpr int NIT = 32 / RPI;        // row pieces per lane and pass
    __shared__ __align__(16) float stage[GDX_WAVES][32][LD];
    __shared__ int s_row[2][32];         // row of dxd behind each of the token's choices (-1: dropped)
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int r = lane & 31, h = lane >> 5;
    const int t0 = blockIdx.x * 32;
    const int rows_here = min(32, Tn - t0);
    const __amdgpu_buffer_rsrc_t rs_dl = buf_rsrc(dlogits + (size_t)t0 * E, (size_t)rows_here * E * 4);
    const __amdgpu_buffer_rsrc_t rs_w = buf_rsrc(Wg, (size_t)d * E * 4);
    const __amdgpu_buffer_rsrc_t rs_dx = buf_rsrc(dx + (size_t)t0 * d, (size_t)rows_here * d * sizeof(T));
    if constexpr (GATHER) {
        if (threadIdx.x < 64) {
            const int t = t0 + r;
            int row = -1;
            if (t < Tn && h < k) {
                const int sl = slot[(size_t)t * k + h];
                if (sl >= 0) row = expert_idx[(size_t)t * k + h] * C + sl;
            }
            s_row[h][r] = row;
        }
        __syncthreads();
    }
    constexpr bool SPLIT = sizeof(T) == 2;
    float afr[(HOIST && !SPLIT) ? EB : 1][16];
    bf16x8_hw_t a_hi[(HOIST && SPLIT) ? EB : 1][2], a_lo[(HOIST && SPLIT) ? EB : 1][2];
    auto load_a = [&](int eb, int to) {   // the token row's fragments of expert block eb (rows beyond T read zeros)
        if constexpr (SPLIT) {
#pragma unroll
            for (int ks = 0; ks < 2; ++ks) {
                float w8[8];
                load_row_f32<VEC, 8>(rs_dl, r * E, eb * 32 + ks * 16 + 8 * h, E, w8);
                split2_bf16(w8, a_hi[to][ks], a_lo[to][ks]);
            }
        } else {
            load_row_f32<VEC, 16>(rs_dl, r * E, eb * 32 + 16 * h, E, afr[to]);
        }
    };
    if constexpr (HOIST) {
#pragma unroll
        for (int eb = 0; eb < EB; ++eb) load_a(eb, eb);
    }
    const int er = lane / LPR, ec = (lane - er * LPR) * CN;
    float(*st)[LD] = stage[wave];
    // What the product is added to does not depend on it: the 16-byte pieces of a
    // pass are requested one pass ahead and stay packed until they are used.
    constexpr int NSRC = GATHER ? 2 : 1;
    int grow[NSRC][NIT];                 // GATHER: row of dxd per choice (-1: dropped)
    if constexpr (GATHER) {
#pragma unroll
        for (int it = 0; it < NIT; ++it) {
            grow[0][it] = s_row[0][er + it * RPI];
            grow[1][it] = k == 2 ? s_row[1][er + it * RPI] : -1;
        }
    }
    auto request = [&](int i0, u32x4_buf_t (&q)[NSRC][NIT]) {
        const int col = i0 + ec;
        const bool ok = col < d;         // d % 8 == 0: a piece is inside the row or wholly beyond it
#pragma unroll
        for (int it = 0; it < NIT; ++it) {
            if constexpr (GATHER) {
                // a dropped choice (or a piece beyond d) reads a valid address and is masked
                // out afterwards: every load is unconditional and inside the tensor
                q[0][it] = *reinterpret_cast<const u32x4_buf_t*>(dxd + (size_t)max(grow[0][it], 0) * d + (ok ? col : 0));
                if (k == 2)   // uniform
                    q[1][it] = *reinterpret_cast<const u32x4_buf_t*>(dxd + (size_t)max(grow[1][it], 0) * d + (ok ? col : 0));
            } else {
                q[0][it] = __builtin_amdgcn_raw_buffer_load_b128(
                    rs_dx, ok ? (uint32_t)(((er + it * RPI) * d + col) * sizeof(T)) : BUF_OOB, 0, 0);
            }
        }
    };
    auto widen = [](u32x4_buf_t q, float (&v)[CN]) {
        if constexpr (sizeof(T) == 2) {
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                v[2 * i] = __uint_as_float(q[i] << 16);
                v[2 * i + 1] = __uint_as_float(q[i] & 0xffff0000u);
            }
        } else {
#pragma unroll
            for (int i = 0; i < 4; ++i) v[i] = __uint_as_float(q[i]);
        }
    };
    u32x4_buf_t now[NSRC][NIT] = {}, ahead[NSRC][NIT] = {};
    request(wave * GDX_COLS, now);
    for (int i0 = wave * GDX_COLS; i0 < d; i0 += GDX_WAVES * GDX_COLS) {
        const int col = i0 + ec;
        const bool col_ok = col < d;
        const int i0n = i0 + GDX_WAVES * GDX_COLS;
        glm_f32x16 acc[2];
#pragma unroll
        for (int c = 0; c < 2; ++c)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[c][v] = 0.0f;
#pragma unroll
        for (int eb = 0; eb < EB; ++eb) {
            if constexpr (!HOIST) load_a(eb, 0);
            const int ai = HOIST ? eb : 0;
            // Wg (L2 resident) first, then the next pass's pieces: loads return in the
            // order they were issued, and the MFMAs below must not wait for memory
            float wfr[2][16];
#pragma unroll
            for (int c = 0; c < 2; ++c) {   // rows beyond d fall outside rs_w
                const int wrow = (i0 + 32 * c + r) * E;
                if constexpr (SPLIT) {      // experts 8h.. and 16 + 8h.. of the block (k = 8h + s per 16-deep step)
                    float lo8[8], hi8[8];
                    load_row_f32<VEC, 8>(rs_w, wrow, eb * 32 + 8 * h, E, lo8);
                    load_row_f32<VEC, 8>(rs_w, wrow, eb * 32 + 16 + 8 * h, E, hi8);
#pragma unroll
                    for (int j = 0; j < 8; ++j) { wfr[c][j] = lo8[j]; wfr[c][8 + j] = hi8[j]; }
                } else {
                    load_row_f32<VEC, 16>(rs_w, wrow, eb * 32 + 16 * h, E, wfr[c]);
                }
            }
            if (eb == EB - 1 && i0n < d) request(i0n, ahead);    // uniform
#pragma unroll
            for (int c = 0; c < 2; ++c) {
                if constexpr (SPLIT) {
#pragma unroll
                    for (int ks = 0; ks < 2; ++ks) {
                        float w8[8];
                        bf16x8_hw_t b_hi, b_lo;
#pragma unroll
                        for (int j = 0; j < 8; ++j) w8[j] = wfr[c][8 * ks + j];
                        split2_bf16(w8, b_hi, b_lo);
                        acc[c] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a_lo[ai][ks], b_hi, acc[c], 0, 0, 0);
                        acc[c] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a_hi[ai][ks], b_lo, acc[c], 0, 0, 0);
                        acc[c] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a_hi[ai][ks], b_hi, acc[c], 0, 0, 0);
                    }
                } else {
#pragma unroll
                    for (int s_ = 0; s_ < 16; ++s_)
                        acc[c] = __builtin_amdgcn_mfma_f32_32x32x2f32(afr[ai][s_], wfr[c][s_], acc[c], 0, 0, 0);
                }
            }
        }
        // accumulator element v of lane l: column l%32, token row 8*(v/4) + 4*(l/32) + v%4
#pragma unroll
        for (int c = 0; c < 2; ++c)
#pragma unroll
            for (int v = 0; v < 16; ++v) st[8 * (v >> 2) + 4 * h + (v & 3)][32 * c + r] = acc[c][v];
        // LDS operations of a wave execute in order: the row pieces read below are complete
#pragma unroll
        for (int it = 0; it < NIT; ++it) {
            const int m = er + it * RPI;
            float inc[CN];
#pragma unroll
            for (int q = 0; q < CN / 4; ++q) {
                const float4 w4 = *reinterpret_cast<const float4*>(&st[m][ec + 4 * q]);
                inc[4 * q] = w4.x; inc[4 * q + 1] = w4.y; inc[4 * q + 2] = w4.z; inc[4 * q + 3] = w4.w;
            }
            if (jitter_eps != 0.0f)     // the gate saw x * noise: d/dx carries the factor (uniform branch)
                jitter_scale<CN>(inc, (size_t)(t0 + m) * d + col, jitter_eps, seed);
            float add[CN];
            widen(now[0][it], add);
            if constexpr (GATHER) {
                float add1[CN];
                widen(now[1][it], add1);
#pragma unroll
                for (int j = 0; j < CN; ++j)
                    inc[j] += (grow[0][it] >= 0 ? add[j] : 0.0f) + (grow[1][it] >= 0 ? add1[j] : 0.0f);
            } else {
#pragma unroll
                for (int j = 0; j < CN; ++j) inc[j] += add[j];
            }
            // stores beyond T or d are dropped by the range check
            BufChunk<T>::store(rs_dx, col_ok ? (uint32_t)((m * d + col) * sizeof(T)) : BUF_OOB, inc);
        }
#pragma unroll
        for (int q = 0; q < NSRC; ++q)
#pragma unroll
            for (int it = 0; it < NIT; ++it) now[q][it] = ahead[q][it];
    }
}

// ---------------------------------------------------------------------------
// The same update for bf16 activations and 33..128 experts (E % 4 == 0, no
// jitter).  With that many experts the 32-token kernel above reads and splits the
// whole gate matrix once per 32 tokens, which costs several times the product
// itself.  Here a workgroup owns 128 tokens: their dlogits rows are split once
// (hi + lo) and stay in LDS as ready MFMA operands for the workgroup's lifetime;
// each of the 8 waves then walks 64-column passes of d on its own, no barrier:
// per 16 experts it loads its columns' gate rows (32 contiguous bytes per lane, the
// B operand as it lies in memory), splits them once and uses them for all four
// token tiles (12 MFMAs per split), so the vector ALU and the L2 see a quarter of
// the work per token.  The tiles leave through the wave-private LDS stage as above.
// ---------------------------------------------------------------------------
#define GDW_KS 8                          // 16-expert steps held in LDS (E <= 128)
template <int TT, int NW>                 // 32-token tiles and waves per workgroup
struct GdwSmem {
    static constexpr int A_BYTES = TT * GDW_KS * 2 * 1024;                // [tile][step][hi, lo] 1 KB operands
    static constexpr int STAGE_LD = GDX_COLS + 4;
    static constexpr int STAGE_BYTES = NW * 32 * STAGE_LD * 4;
    static constexpr int ROW_BYTES = 2 * TT * 32 * 4;
    static constexpr int BYTES = A_BYTES + STAGE_BYTES + ROW_BYTES;
};

template <int NSRC_G, int TT, int NW>   // NSRC_G: 0 = add to dx in place; 1, 2 = gather the token's k kept rows of dxd
__global__ __launch_bounds__(64 * NW, TT == 2 ? 2 : 1) void gate_dx_wide_kernel(
    int Tn, int d, int E, int k, int C, const float* __restrict__ dlogits, const float* __restrict__ Wg,
    const bf16_t* __restrict__ dxd, const int32_t* __restrict__ expert_idx, const int32_t* __restrict__ slot,
    bf16_t* __restrict__ dx) {
    typedef GdwSmem<TT, NW> SM;
    constexpr int NT = 64 * NW;
    constexpr bool GATHER = NSRC_G > 0;
    extern __shared__ __align__(16) unsigned char gdw_smem[];
    unsigned char* s_a = gdw_smem;
    float(*stage)[SM::STAGE_LD] =
        reinterpret_cast<float(*)[SM::STAGE_LD]>(gdw_smem + SM::A_BYTES) + (threadIdx.x >> 6) * 32;
    int* s_row = reinterpret_cast<int*>(gdw_smem + SM::A_BYTES + SM::STAGE_BYTES);   // [2][32*TT]
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int r = lane & 31, h = lane >> 5;
    const int t0 = blockIdx.x * 32 * TT;
    const int rows_here = min(32 * TT, Tn - t0);
    const int nks = (E + 15) / 16;
    const __amdgpu_buffer_rsrc_t rs_dl = buf_rsrc(dlogits + (size_t)t0 * E, (size_t)rows_here * E * 4);
    const __amdgpu_buffer_rsrc_t rs_w = buf_rsrc(Wg, (size_t)d * E * 4);
    const __amdgpu_buffer_rsrc_t rs_dx = buf_rsrc(dx + (size_t)t0 * d, (size_t)rows_here * d * 2);
    // 8 consecutive fp32 of a row (two 16-byte loads; E % 4 == 0: a quad is inside the row or beyond it)
    auto load8_row = [&](__amdgpu_buffer_rsrc_t rs, int row_elems, int e0, float (&v)[8]) {
#pragma unroll
        for (int c = 0; c < 2; ++c) {
            const u32x4_buf_t q = __builtin_amdgcn_raw_buffer_load_b128(
                rs, e0 + 4 * c < E ? (uint32_t)((row_elems + e0 + 4 * c) * 4) : BUF_OOB, 0, 0);
#pragma unroll
            for (int j = 0; j < 4; ++j) v[4 * c + j] = __uint_as_float(q[j]);
        }
    };
    // the workgroup's dlogits rows as MFMA operands: lane (r, h) of operand (tile, step) holds
    // experts 16*step + 8h .. +7 of token 32*tile + r
#pragma unroll
    for (int i = 0; i < TT * GDW_KS * 64 / NT; ++i) {
        const int it = threadIdx.x + i * NT;
        const int l = it & 63, f = it >> 6;                 // f = tile*8 + step
        const int ks = f & (GDW_KS - 1), tok = (f >> 3) * 32 + (l & 31);
        float w8[8];
        load8_row(rs_dl, tok * E, 16 * ks + 8 * (l >> 5), w8);   // rows beyond T read zeros
        bf16x8_hw_t a_hi, a_lo;
        split2_bf16(w8, a_hi, a_lo);
        *reinterpret_cast<bf16x8_hw_t*>(s_a + (f * 2) * 1024 + l * 16) = a_hi;
        *reinterpret_cast<bf16x8_hw_t*>(s_a + (f * 2 + 1) * 1024 + l * 16) = a_lo;
    }
    if constexpr (GATHER) {
        for (int i = threadIdx.x; i < 2 * TT * 32; i += NT) {
            const int j = i / (TT * 32), tl = i - j * (TT * 32), t = t0 + tl;
            int row = -1;
            if (t < Tn && j < k) {
                const int sl = slot[(size_t)t * k + j];
                if (sl >= 0) row = expert_idx[(size_t)t * k + j] * C + sl;
            }
            s_row[i] = row;
        }
    }
    __syncthreads();

    constexpr int LPR = GDX_COLS / 8;    // lanes per staged row (16-byte pieces of 8 bf16)
    constexpr int RPI = 64 / LPR;        // rows per wave instruction
    constexpr int NIT = 32 / RPI;        // row pieces per lane and tile
    constexpr int NSRC = GATHER ? NSRC_G : 1;
    const int er = lane / LPR, ec = (lane - er * LPR) * 8;
    const int npass = (d + GDX_COLS - 1) / GDX_COLS;
    for (int p = wave; p < npass; p += NW) {
        const int i0 = p * GDX_COLS;
        const int col = i0 + ec;
        const bool col_ok = col < d;     // d % 8 == 0: a piece is inside the row or wholly beyond it
        // What the product is added to (the token's kept rows of dxd, or dx itself), per tile.
        u32x4_buf_t src[TT][NSRC][NIT];
        uint32_t kept[TT];               // bit q*NIT + it: that piece counts (a dropped choice reads row 0 and is masked out)
        auto request = [&](int tt) {
            kept[tt] = 0;
#pragma unroll
            for (int it = 0; it < NIT; ++it) {
                const int m = tt * 32 + er + it * RPI;
                if constexpr (GATHER) {
#pragma unroll
                    for (int q = 0; q < NSRC; ++q) {
                        const int row = s_row[q * TT * 32 + m];
                        kept[tt] |= (row >= 0 ? 1u : 0u) << (q * NIT + it);
                        src[tt][q][it] = *reinterpret_cast<const u32x4_buf_t*>(
                            dxd + (size_t)max(row, 0) * d + (col_ok ? col : 0));
                    }
                } else {
                    kept[tt] = ~0u;
                    src[tt][0][it] = __builtin_amdgcn_raw_buffer_load_b128(
                        rs_dx, col_ok ? (uint32_t)((m * d + col) * 2) : BUF_OOB, 0, 0);
                }
            }
        };
        request(0);                      // before the products of the pass: in flight under them
        glm_f32x16 acc[TT][2];
#pragma unroll
        for (int tt = 0; tt < TT; ++tt)
#pragma unroll
            for (int c = 0; c < 2; ++c)
#pragma unroll
                for (int v = 0; v < 16; ++v) acc[tt][c][v] = 0.0f;
        // Gate rows are requested for two 16-expert steps at a time: the 128-byte line that holds
        // experts 32j .. 32j+31 of a column is then touched by four back-to-back instructions and
        // fetched from L2 once (a step apart, the other waves' lines have displaced it from L1).
#pragma unroll
        for (int kp = 0; kp < GDW_KS / 2; ++kp) {
            if (2 * kp < nks) {                             // uniform
                float w8[2][2][8];
#pragma unroll
                for (int u = 0; u < 2; ++u)
#pragma unroll
                    for (int c = 0; c < 2; ++c)             // rows beyond d fall outside rs_w, experts beyond E read zeros
                        load8_row(rs_w, (i0 + 32 * c + r) * E, 16 * (2 * kp + u) + 8 * h, w8[u][c]);
#pragma unroll
                for (int u = 0; u < 2; ++u) {
                    const int ks = 2 * kp + u;
                    bf16x8_hw_t b_hi[2], b_lo[2];
#pragma unroll
                    for (int c = 0; c < 2; ++c) split2_bf16(w8[u][c], b_hi[c], b_lo[c]);
                    bf16x8_hw_t a_hi[TT], a_lo[TT];
#pragma unroll
                    for (int tt = 0; tt < TT; ++tt) {
                        const unsigned char* pa = s_a + ((tt * GDW_KS + ks) * 2) * 1024 + lane * 16;
                        a_hi[tt] = *reinterpret_cast<const bf16x8_hw_t*>(pa);
                        a_lo[tt] = *reinterpret_cast<const bf16x8_hw_t*>(pa + 1024);
                    }
                    // the three partial products of a tile are far apart: no MFMA waits for its predecessor
#pragma unroll
                    for (int tt = 0; tt < TT; ++tt)
#pragma unroll
                        for (int c = 0; c < 2; ++c)
                            acc[tt][c] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a_lo[tt], b_hi[c], acc[tt][c], 0, 0, 0);
#pragma unroll
                    for (int tt = 0; tt < TT; ++tt)
#pragma unroll
                        for (int c = 0; c < 2; ++c)
                            acc[tt][c] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a_hi[tt], b_lo[c], acc[tt][c], 0, 0, 0);
#pragma unroll
                    for (int tt = 0; tt < TT; ++tt)
#pragma unroll
                        for (int c = 0; c < 2; ++c)
                            acc[tt][c] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a_hi[tt], b_hi[c], acc[tt][c], 0, 0, 0);
                }
            }
        }
        // the other tiles' sources as registers come free, each well before its use
        request(1);
        if constexpr (TT > 2) request(2);
#pragma unroll
        for (int tt = 0; tt < TT; ++tt) {
            if (tt >= 1 && tt + 2 < TT) request(tt + 2);
            // accumulator element v of lane l: column l%32, token row 8*(v/4) + 4*(l/32) + v%4
#pragma unroll
            for (int c = 0; c < 2; ++c)
#pragma unroll
                for (int v = 0; v < 16; ++v) stage[8 * (v >> 2) + 4 * h + (v & 3)][32 * c + r] = acc[tt][c][v];
            // LDS operations of a wave execute in order: the row pieces read below are complete
#pragma unroll
            for (int it = 0; it < NIT; ++it) {
                const int ml = er + it * RPI;
                float inc[8];
#pragma unroll
                for (int q = 0; q < 2; ++q) {
                    const float4 w4 = *reinterpret_cast<const float4*>(&stage[ml][ec + 4 * q]);
                    inc[4 * q] = w4.x; inc[4 * q + 1] = w4.y; inc[4 * q + 2] = w4.z; inc[4 * q + 3] = w4.w;
                }
#pragma unroll
                for (int q = 0; q < NSRC; ++q) {
                    const bool on = (kept[tt] >> (q * NIT + it)) & 1u;
#pragma unroll
                    for (int j = 0; j < 4; ++j) {
                        inc[2 * j] += on ? __uint_as_float(src[tt][q][it][j] << 16) : 0.0f;
                        inc[2 * j + 1] += on ? __uint_as_float(src[tt][q][it][j] & 0xffff0000u) : 0.0f;
                    }
                }
                // stores beyond T or d are dropped by the range check
                BufChunk<bf16_t>::store(rs_dx, col_ok ? (uint32_t)(((tt * 32 + ml) * d + col) * 2) : BUF_OOB, inc);
            }
        }
    }
}

#ifndef GDW_TT
#define GDW_TT 4
#define GDW_NW 8
#endif
template <typename T>
static bool launch_gate_logits_bwd(const moe_shape* s, const void* x, const float* Wg,
                                   const float* dlogits, float* dWg, void* dx, const void* dxd,
                                   const int32_t* expert_idx, const int32_t* slot, float* partial, float eps,
                                   uint64_t seed, hipStream_t st) {
    const int tpc = gw_chunk_tokens(s);
    const int nch_used = ceil_div(s->T, tpc);
    dim3 grid(ceil_div(s->d_model, GW_COLS), nch_used, ceil_div(s->E, 32));
    constexpr size_t red_bytes = (size_t)2 * GW_COLS * 32 * sizeof(float);   // two staged tiles: 64 KB
    static unsigned long long opted_w[2] = {0, 0};
    if (eps != 0.0f) {
        if (!lds_opt_in((const void*)gate_dwg_partial_kernel<T, true>, red_bytes, &opted_w[1])) return false;
        gate_dwg_partial_kernel<T, true><<<grid, 64 * GW_WAVES, red_bytes, st>>>(s->T, s->d_model, s->E, tpc,
                                                                              (const T*)x, dlogits, partial, eps, seed);
    } else {
        if (!lds_opt_in((const void*)gate_dwg_partial_kernel<T, false>, red_bytes, &opted_w[0])) return false;
        gate_dwg_partial_kernel<T, false><<<grid, 64 * GW_WAVES, red_bytes, st>>>(s->T, s->d_model, s->E, tpc,
                                                                               (const T*)x, dlogits, partial, eps, seed);
    }
    const int n = s->d_model * s->E;
    gate_dwg_reduce_kernel<<<ceil_div(n, 256), 256, 0, st>>>(n, nch_used, partial, dWg);
    if (dx && sizeof(T) == 2 && eps == 0.0f && s->E > 32 && s->E <= 16 * GDW_KS && s->E % 4 == 0 &&
        ceil_div(s->T, 32 * GDW_TT) >= 192) {
        // 128 tokens per workgroup once that still gives most compute units a workgroup
        typedef GdwSmem<GDW_TT, GDW_NW> SM;
        static unsigned long long opted_x[3] = {0, 0, 0};
        const int grid_w = ceil_div(s->T, 32 * GDW_TT);
#define GDWL(NS, DXD, EI, SL) do { \
    if (!lds_opt_in((const void*)gate_dx_wide_kernel<NS, GDW_TT, GDW_NW>, SM::BYTES, &opted_x[NS])) return false; \
    gate_dx_wide_kernel<NS, GDW_TT, GDW_NW><<<grid_w, 64 * GDW_NW, SM::BYTES, st>>>( \
        s->T, s->d_model, s->E, s->k, s->capacity, dlogits, Wg, DXD, EI, SL, (bf16_t*)dx); } while (0)
        if (!dxd) GDWL(0, nullptr, nullptr, nullptr);
        else if (s->k == 1) GDWL(1, (const bf16_t*)dxd, expert_idx, slot);
        else GDWL(2, (const bf16_t*)dxd, expert_idx, slot);
#undef GDWL
    } else if (dx) {
        const int grid_dx = ceil_div(s->T, 32);
#define GDX(EB, VEC, GA) gate_dx_kernel<T, EB, VEC, GA><<<grid_dx, 64 * GDX_WAVES, 0, st>>>( \
    s->T, s->d_model, s->E, s->k, s->capacity, dlogits, Wg, (const T*)dxd, expert_idx, slot, (T*)dx, eps, seed)
#define GDXE(VEC, GA) do { if (s->E <= 32) GDX(1, VEC, GA); else if (s->E <= 64) GDX(2, VEC, GA); \
                           else if (s->E <= 128) GDX(4, VEC, GA); else GDX(8, VEC, GA); } while (0)
        if (dxd) { if (s->E % 4 == 0) GDXE(true, true); else GDXE(false, true); }
        else     { if (s->E % 4 == 0) GDXE(true, false); else GDXE(false, false); }
#undef GDXE
#undef GDX
    }
    return true;
}

static int gate_logits_bwd_impl(const moe_shape* shape, const void* x, const float* Wg, const float* dlogits,
                                float eps, uint64_t seed, float* dWg, void* dx_accum, const void* dxd,
                                const int32_t* expert_idx, const int32_t* slot, void* ws, size_t ws_bytes,
                                void* stream) {
    int rc = check_shape(shape);
    if (rc) return rc;
    if (!x || !Wg || !dlogits || !dWg) return MOE_ERR_NULL;
    if (!(eps >= 0.0f && eps < 1.0f)) return MOE_ERR_SHAPE;
    if (!ws || ((uintptr_t)ws & 255) || ws_bytes < gate_logits_bwd_ws_bytes(shape)) return MOE_ERR_WORKSPACE;
    const bool ok = shape->dtype == MOE_BF16
        ? launch_gate_logits_bwd<bf16_t>(shape, x, Wg, dlogits, dWg, dx_accum, dxd, expert_idx, slot, (float*)ws, eps, seed, (hipStream_t)stream)
        : launch_gate_logits_bwd<float>(shape, x, Wg, dlogits, dWg, dx_accum, dxd, expert_idx, slot, (float*)ws, eps, seed, (hipStream_t)stream);
    return ok ? launch_status() : MOE_ERR_LAUNCH;
}

extern "C" int moe_gate_logits_bwd(const moe_shape* shape, const void* x, const float* Wg,
                                   const float* dlogits, float* dWg, void* dx_accum, void* ws,
                                   size_t ws_bytes, void* stream) {
    return gate_logits_bwd_impl(shape, x, Wg, dlogits, 0.0f, 0, dWg, dx_accum, nullptr, nullptr, nullptr, ws, ws_bytes, stream);
}

extern "C" int moe_gate_logits_bwd_jitter(const moe_shape* shape, const void* x, const float* Wg,
                                          const float* dlogits, float jitter_eps, uint64_t seed,
                                          float* dWg, void* dx_accum, void* ws, size_t ws_bytes,
                                          void* stream) {
    return gate_logits_bwd_impl(shape, x, Wg, dlogits, jitter_eps, seed, dWg, dx_accum, nullptr, nullptr, nullptr, ws, ws_bytes, stream);
}

extern "C" int moe_dispatch_gate_logits_bwd(const moe_shape* shape, const void* x, const float* Wg,
                                            const float* dlogits, const void* dxd, const int32_t* expert_idx,
                                            const int32_t* slot, float jitter_eps, uint64_t seed, float* dWg,
                                            void* dx, void* ws, size_t ws_bytes, void* stream) {
    if (!dxd || !expert_idx || !slot || !dx) return MOE_ERR_NULL;
    return gate_logits_bwd_impl(shape, x, Wg, dlogits, jitter_eps, seed, dWg, dx, dxd, expert_idx, slot, ws, ws_bytes,
                                stream);
}
