// Grouped expert GEMMs on the MFMA matrix cores: the per-expert feed-forward
// block d_model -> d_ff -> d_model, forward and backward (Sec. 4.2 "Model
// details"; Sec. 2.3: these matmuls are where the layer's time goes).
//
// One kernel template serves the six contractions.  Per expert e with
// n_e = expert_count[e] rows in use:
//   forward   z = xd W1        (rows x d)(d x f)     epilogue: h = act(z), a = act'(z)
//             yd = h W2        (rows x f)(f x d)
//   backward  dz = (dyd W2^T) .* a
//             dxd = dz W1^T
//             dW2 = h^T dyd    (f x rows)(rows x d)  fp32 output, K = rows
//             dW1 = xd^T dz    (d x rows)(rows x f)
// Each operand is described as a (row index r, reduction index k) array that is
// either k-contiguous in memory (KC) or r-contiguous (!KC); no transposed copy
// of any tensor is ever materialised.
//
// Structure of a workgroup (4 waves, 2 x 2):
//   * owns a BM x BN output tile of one expert; workgroup ids are remapped so
//     that consecutive tiles of one expert land on the same XCD and share its L2;
//   * streams BK-deep slabs of both operands with 16-byte buffer loads that
//     write straight into LDS (no register staging), NSTAGE-1 slabs ahead of
//     the one being multiplied, so HBM/L2 latency is covered by several slabs
//     of MFMA work; the buffer range check supplies the zero fill for rows
//     >= n_e (no branches in the loop); LDS tiles are unpadded and XOR-swizzled
//     in 16-byte units so that fragment reads are bank-conflict free;
//   * each wave accumulates (BM/2) x (BN/2) in 32x32 MFMA tiles
//     (bf16: v_mfma_f32_32x32x16_bf16, fp32: v_mfma_f32_32x32x2_f32); !KC bf16
//     operands are read from LDS with the transposing ds_read_b64_tr_b16;
//   * the epilogue passes the accumulators through LDS so that every global
//     store is a full 8/16-byte vector along the row; the activation and its
//     derivative are evaluated once, in the forward epilogue (code kept in a
//     rolled loop), and the backward epilogue only multiplies by the saved
//     derivative, which it fetched into registers before the main loop.
#include "moe_common.h"

// bf16 tile shape (tuning knobs; the defaults are the shipped configuration)
#ifndef MOE_GEMM_BM
#define MOE_GEMM_BM 256
#endif
#ifndef MOE_GEMM_BN
#define MOE_GEMM_BN 256
#endif
#ifndef MOE_GEMM_BK
#define MOE_GEMM_BK 32
#endif

typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef float f32x16_t __attribute__((ext_vector_type(16)));
typedef unsigned int u32x4_t __attribute__((ext_vector_type(4)));
typedef short s16x4_t __attribute__((ext_vector_type(4)));
typedef short s16x8_t __attribute__((ext_vector_type(8)));
typedef __attribute__((address_space(3))) s16x4_t lds_s16x4_t;

enum { EPI_STORE = 0, EPI_H_DACT = 1, EPI_MUL = 2, EPI_F32 = 3 };

struct GemmArgs {
    const void* A; const void* B;
    void* out0; void* out1; const void* aux;
    const int32_t* expert_count;
    long long strideA, strideB, strideO;  // elements per expert
    int lda, ldb, ldo;
    int M, N, K;      // extents; the one bounded by expert_count is an upper limit
    int var_k;        // 0: rows (M) bounded by expert_count; 1: K bounded by it
    int tiles_m, tiles_n, total_tiles, tiles_per_xcd;
};

template <typename T> struct Mma;
template <> struct Mma<bf16_t> {
    static constexpr int FE = 8;      // elements per lane per operand
    static constexpr int KSTEP = 16;  // reduction depth of one MFMA
    typedef bf16x8_t frag;
    __device__ static __forceinline__ f32x16_t mma(frag a, frag b, f32x16_t c) {
        return __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0);
    }
};
template <> struct Mma<float> {
    static constexpr int FE = 1;
    static constexpr int KSTEP = 2;
    typedef float frag;
    __device__ static __forceinline__ f32x16_t mma(frag a, frag b, f32x16_t c) {
        return __builtin_amdgcn_mfma_f32_32x32x2f32(a, b, c, 0, 0, 0);
    }
};

// Raw buffer descriptor (4 SGPRs) over `bytes` bytes at p: loads beyond the
// range return 0 (and, for loads into LDS, store 0).
__device__ __forceinline__ u32x4_t make_desc(const void* p, uint32_t bytes) {
    const uint64_t a = (uint64_t)p;
    u32x4_t d;
    d[0] = (uint32_t)a;
    d[1] = (uint32_t)(a >> 32) & 0xffffu;
    d[2] = bytes;
    d[3] = 0x00020000u;
    return d;
}
#define OOB_OFFSET 0x80000000u  // beyond any descriptor this kernel builds (slices < 2 GiB)

// One wavefront-wide 16-byte-per-lane load from a raw buffer straight into LDS:
// lane l's 16 bytes land at LDS byte address lds_base + 16*l (lds_base is wave
// uniform and travels in M0).  Written as asm so that the compiler does not
// serialise every later LDS read behind the load; completion is tracked by
// hand with vmcnt (see the main loop).
__device__ __forceinline__ void load_to_lds(u32x4_t desc, uint32_t voff, uint32_t lds_base) {
#ifndef MOE_DMA_MODE
#define MOE_DMA_MODE 0
#endif
#if MOE_DMA_MODE == 1
#define MOE_DMA_MODS " nt"
#elif MOE_DMA_MODE == 2
#define MOE_DMA_MODS " sc1"
#elif MOE_DMA_MODE == 3
#define MOE_DMA_MODS " sc0"
#elif MOE_DMA_MODE == 4
#define MOE_DMA_MODS " sc0 sc1"
#else
#define MOE_DMA_MODS ""
#endif
    asm volatile("s_mov_b32 m0, %0\n\tbuffer_load_dwordx4 %1, %2, 0 offen" MOE_DMA_MODS " lds"
                 :: "s"(lds_base), "v"(voff), "s"(desc) : "memory");
}
// s_waitcnt vmcnt(N) only (gfx9 encoding: vmcnt[3:0] in bits 3:0, vmcnt[5:4] in 15:14)
template <int N> __device__ __forceinline__ void wait_vmcnt() {
    __builtin_amdgcn_s_waitcnt((N & 0xf) | ((N >> 4) << 14) | (0x7 << 4) | (0xf << 8));
}

// LDS tile of one operand: BR rows (r) x BK reduction entries, unpadded, as
// 16-byte slots; slot p is filled by thread p % 256 in its (p / 256)-th load.
//   KC : LDS row = r (BK entries),  slot = r*CPR + (chunk ^ swz(r))
//   !KC: LDS row = k (BR entries),  slot = k*CPR + (chunk ^ swz(k))
// swz: KC  -> consecutive rows that share a 256-byte bank window get distinct
//             chunk positions (16-byte fragment reads of 16 rows hit 64 banks);
//      !KC -> rows k, k+1, k+2, k+3 are shifted by 64 bytes each (the
//             transposing 8-byte reads of 4 rows x 64 bytes hit 64 banks).
template <typename T, int BR, int BK, bool KC> struct Tile {
    static constexpr int CN = 16 / (int)sizeof(T);           // elements per slot
    static constexpr int CPR = (KC ? BK : BR) / CN;          // slots per LDS row
    static constexpr int ROWS = KC ? BR : BK;
    static constexpr int SLOTS = ROWS * CPR;
    static constexpr int PER_THREAD = SLOTS / 256;
    static constexpr int BYTES = SLOTS * 16;
    static constexpr int WIN = CPR >= 16 ? 1 : 16 / CPR;     // rows per 256-byte window
    static_assert(SLOTS % 256 == 0, "tile must be a multiple of 256 slots");
    static_assert((CPR & (CPR - 1)) == 0, "slots per row must be a power of two");

    __device__ static __forceinline__ int swz(int row) {
        return KC ? (row / WIN) & (CPR - 1) : ((row & 3) << 2) & (CPR - 1);
    }

    // Per-thread load plan: byte offset of each of its slots at reduction offset 0
    // (OOB_OFFSET where the non-linear guard already fails) and, for KC, the
    // reduction column of the slot (its guard depends on the slab).
    struct Plan { uint32_t voff[PER_THREAD]; int kcol[PER_THREAD]; };
    __device__ static __forceinline__ void plan(Plan& pl, int ld, int r0, int r_lim) {
#pragma unroll
        for (int i = 0; i < PER_THREAD; ++i) {
            const int p = threadIdx.x + i * 256;
            const int row = p / CPR, c = (p % CPR) ^ swz(row);
            if (KC) {
                pl.voff[i] = (uint32_t)((r0 + row) * ld + c * CN) * (uint32_t)sizeof(T);
                pl.kcol[i] = c * CN;
            } else {
                const int r = r0 + c * CN;
                pl.voff[i] = r < r_lim ? (uint32_t)(row * ld + r) * (uint32_t)sizeof(T) : OOB_OFFSET;
                pl.kcol[i] = 0;
            }
        }
    }
    // Descriptor range = the linear guard: KC rows < r_lim, !KC reduction rows < k_lim.
    __device__ static __forceinline__ u32x4_t desc(const T* g, int ld, int r_lim, int k_lim) {
        return make_desc(g, (uint32_t)(KC ? r_lim : k_lim) * (uint32_t)ld * (uint32_t)sizeof(T));
    }
    // Issue this thread's loads of the slab at reduction offset k0 into the stage at lds_base.
    __device__ static __forceinline__ void issue(const Plan& pl, u32x4_t ds, int ld, int k0, int k_lim,
                                                 uint32_t lds_base) {
        const uint32_t kstep = (uint32_t)(KC ? k0 : k0 * ld) * (uint32_t)sizeof(T);
        const uint32_t wave_base = lds_base + (threadIdx.x >> 6) * 1024;
#pragma unroll
        for (int i = 0; i < PER_THREAD; ++i) {
            uint32_t off = pl.voff[i] + kstep;
            if (KC) off = pl.kcol[i] + k0 < k_lim ? off : OOB_OFFSET;
            load_to_lds(ds, off, __builtin_amdgcn_readfirstlane(wave_base + i * 4096));
        }
    }
    // LDS -> MFMA operand for the 32 tile rows rbase..rbase+31 (this lane: row
    // rbase + lane%32), reduction step ks; lane group g = lane/32 holds the
    // reduction entries ks*KSTEP + FE*g .. + FE-1.
    __device__ static __forceinline__ typename Mma<T>::frag frag(const unsigned char* s, int rbase, int ks, int lane) {
        constexpr int FE = Mma<T>::FE;
        const int g = lane >> 5, l32 = lane & 31;
        const int k = ks * Mma<T>::KSTEP + FE * g;
        if constexpr (sizeof(T) == 2) {
            if constexpr (KC) {
                const int row = rbase + l32;
                const int slot = row * CPR + ((k / CN) ^ swz(row));
                return __builtin_bit_cast(bf16x8_t, *reinterpret_cast<const u32x4_t*>(s + slot * 16));
            } else {
                // ds_read_b64_tr_b16: within 16 lanes, lane s supplies the address of 4
                // consecutive r at reduction row (s/4); lane l receives, for its own
                // r = 4*(l/4)+(l%4) of those 16, the entries of 4 consecutive rows.
                const int sl = lane & 15;
                const int kr = k + (sl >> 2);
                const int col = rbase + (l32 & 16) + 4 * (sl & 3);
                const int slot = kr * CPR + ((col / CN) ^ swz(kr));
                const unsigned char* p = s + slot * 16 + (col % CN) * 2;
                const s16x4_t lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4_t*)p);
                const s16x4_t hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4_t*)(p + 4 * CPR * 16));
                const s16x8_t v = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
                return __builtin_bit_cast(bf16x8_t, v);
            }
        } else {
            if constexpr (KC) {
                const int row = rbase + l32;
                const int slot = row * CPR + ((k / CN) ^ swz(row));
                return *reinterpret_cast<const float*>(s + slot * 16 + (k % CN) * 4);
            } else {
                const int col = rbase + l32;
                const int slot = k * CPR + ((col / CN) ^ swz(k));
                return *reinterpret_cast<const float*>(s + slot * 16 + (col % CN) * 4);
            }
        }
    }
};

// ---- activation in the forward epilogue ---------------------------------------
// h = act(z) and a = act'(z) together.  fp32 tensors use the accurate erff/expf;
// bf16 tensors (8 mantissa bits) share one exponential between the normal
// density and a 5-term rational erfc (absolute error < 2e-7).
template <bool FAST, int ACT>
__device__ __forceinline__ void act_both(float z, float& h, float& a) {
    if constexpr (ACT == MOE_RELU) {
        h = fmaxf(z, 0.0f);
        a = z > 0.0f ? 1.0f : 0.0f;
        return;
    }
    float cdf, zpdf;
    if constexpr (!FAST) {
        cdf = 0.5f * (1.0f + erff(z * 0.70710678118654752440f));
        zpdf = z * 0.39894228040143267794f * expf(-0.5f * z * z);
    } else {
        const float ex = __builtin_amdgcn_exp2f(z * z * -0.72134752044448170368f);  // exp(-z^2/2)
        const float t = __builtin_amdgcn_rcpf(fmaf(0.23164189f, fabsf(z), 1.0f));    // 0.3275911/sqrt(2)
        float poly = fmaf(0.5307027145f, t, -0.7265760135f);                         // coefficients / 2
        poly = fmaf(poly, t, 0.7107068705f);
        poly = fmaf(poly, t, -0.142248368f);
        poly = fmaf(poly, t, 0.127414796f);
        const float q = poly * t * ex;  // (1 - erf(|z|/sqrt 2)) / 2
        cdf = z >= 0.0f ? 1.0f - q : q;
        zpdf = z * 0.39894228040143267794f * ex;
    }
    h = z * cdf;
    a = cdf + zpdf;
}

// One row vector of the output tile: o = element offset, v = 4 accumulators,
// aux = the 4 saved derivatives (EPI_MUL only).
template <typename T, int EPI, int ACT>
__device__ __forceinline__ void epilogue4(const GemmArgs& p, size_t o, float (&v)[4],
                                          typename Vec4io<T>::raw aux) {
    typedef typename Vec4io<T>::raw raw;
    if constexpr (EPI == EPI_STORE) {
        *reinterpret_cast<raw*>((T*)p.out0 + o) = Vec4io<T>::pack(v);
    } else if constexpr (EPI == EPI_H_DACT) {
        float h[4], a[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) act_both<sizeof(T) == 2, ACT>(v[i], h[i], a[i]);
        *reinterpret_cast<raw*>((T*)p.out0 + o) = Vec4io<T>::pack(a);
        *reinterpret_cast<raw*>((T*)p.out1 + o) = Vec4io<T>::pack(h);
    } else if constexpr (EPI == EPI_MUL) {
        float a[4];
        Vec4io<T>::unpack(aux, a);
#pragma unroll
        for (int i = 0; i < 4; ++i) v[i] *= a[i];
        *reinterpret_cast<raw*>((T*)p.out0 + o) = Vec4io<T>::pack(v);
    } else {
        *reinterpret_cast<float4*>((float*)p.out0 + o) = make_float4(v[0], v[1], v[2], v[3]);
    }
}

#ifndef MOE_GEMM_LDS_KB
#define MOE_GEMM_LDS_KB 144
#endif
#define GEMM_LDS_BUDGET (MOE_GEMM_LDS_KB * 1024)  // LDS one workgroup may take (CU: 160 KB)

template <typename T, int BM, int BN, int BK, bool A_KC, bool B_KC>
struct GemmSmem {
    typedef Tile<T, BM, BK, A_KC> TA;
    typedef Tile<T, BN, BK, B_KC> TB;
    static constexpr int STAGE = TA::BYTES + TB::BYTES;
    // LDS ring: 1 slab being multiplied + NSTAGE-1 in flight
    static constexpr int NSTAGE = 4 * STAGE <= GEMM_LDS_BUDGET ? 4 : 3 * STAGE <= GEMM_LDS_BUDGET ? 3 : 2;
    static constexpr int EPI_LD = BN / 2 + 8;  // floats per staged row (4 rows apart -> other bank half)
    static constexpr size_t OPERANDS = (size_t)NSTAGE * STAGE;
    static constexpr size_t EPILOGUE = 4 * 32 * (size_t)EPI_LD * sizeof(float);
    static constexpr size_t BYTES = OPERANDS > EPILOGUE ? OPERANDS : EPILOGUE;
    static constexpr int LOADS = TA::PER_THREAD + TB::PER_THREAD;  // per thread per slab
    static_assert((NSTAGE - 1) * LOADS < 64, "vmcnt is a 6-bit counter");
    static_assert(NSTAGE >= 3, "the loop refills a stage while the next slab is already resident");
    static_assert((BK / Mma<T>::KSTEP) % 2 == 0, "fragment double buffering needs an even number of k-steps");
};

template <typename T, int BM, int BN, int BK, bool A_KC, bool B_KC, int EPI, int ACT>
__global__ __launch_bounds__(256) void grouped_gemm_kernel(const GemmArgs p) {
    typedef GemmSmem<T, BM, BN, BK, A_KC, B_KC> SM;
    typedef typename SM::TA TA;
    typedef typename SM::TB TB;
    constexpr int TM = BM / 64, TN = BN / 64;  // 32x32 MFMA tiles per wave (2x2 waves)
    constexpr int KS = BK / Mma<T>::KSTEP;
    constexpr int NS = SM::NSTAGE;
    extern __shared__ __align__(16) unsigned char smem_raw[];

    // XCD-aware tile order: workgroup ids are dealt round-robin to the 8 XCDs, so
    // give each XCD one contiguous run of logical tiles (= whole experts).
    const int bid = blockIdx.x;
#ifdef MOE_DEBUG_NOREMAP
    const int logical = bid;
#else
    const int logical = (bid & 7) * p.tiles_per_xcd + (bid >> 3);
#endif
    if (logical >= p.total_tiles) return;
    const int per_e = p.tiles_m * p.tiles_n;
    const int e = logical / per_e;
    const int rem = logical - e * per_e;
    const int tm = rem / p.tiles_n, tn = rem - tm * p.tiles_n;
    const int n_e = p.expert_count[e];
    const int m0 = tm * BM, n0 = tn * BN;
    const int m_lim = p.var_k ? p.M : n_e;
    const int k_lim = p.var_k ? n_e : p.K;
    if (m0 >= m_lim) return;

    const u32x4_t dsA = TA::desc((const T*)p.A + (size_t)e * p.strideA, p.lda, m_lim, k_lim);
    const u32x4_t dsB = TB::desc((const T*)p.B + (size_t)e * p.strideB, p.ldb, p.N, k_lim);
    typename TA::Plan planA;
    typename TB::Plan planB;
    TA::plan(planA, p.lda, m0, m_lim);
    TB::plan(planB, p.ldb, n0, p.N);
    const uint32_t lds0 = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) unsigned char*)smem_raw;

    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int wm = wave >> 1, wn = wave & 1;

    f32x16_t acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.0f;

    // epilogue geometry: the wave's (BM/2) x (BN/2) sub-tile goes out in strips of
    // 32 rows; a lane owns 4 consecutive columns of RPI-strided rows
    constexpr int ELD = SM::EPI_LD;
    constexpr int WCOLS = BN / 2;
    constexpr int LPR = WCOLS / 4;                // lanes per staged row
    constexpr int RPI = 64 / LPR;                 // rows per wave instruction
    constexpr int NIT = 32 / RPI;
    const int er = lane / LPR, ec = (lane - er * LPR) * 4;
    const size_t obase = (size_t)e * p.strideO;
    const int ncol = n0 + wn * WCOLS + ec;
    // EPI_MUL: the saved derivative does not depend on the product, so it is
    // fetched now and rides in registers through the main loop
    typename Vec4io<T>::raw aux[EPI == EPI_MUL ? TM : 1][EPI == EPI_MUL ? NIT : 1];
    if constexpr (EPI == EPI_MUL) {
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int it = 0; it < NIT; ++it) {
                const int m = m0 + wm * (BM / 2) + i * 32 + er + it * RPI;
                aux[i][it] = (m < m_lim && ncol < p.N)
                    ? *reinterpret_cast<const typename Vec4io<T>::raw*>((const T*)p.aux + obase + (size_t)m * p.ldo + ncol)
                    : Vec4io<T>::zero();
            }
    }

    const int nk = (k_lim + BK - 1) / BK;
    // prologue: slabs 0 .. NS-2 into stages 0 .. NS-2 (slabs past the end read zeros)
#pragma unroll
    for (int s = 0; s < NS - 1; ++s) {
        TA::issue(planA, dsA, p.lda, s * BK, k_lim, lds0 + s * SM::STAGE);
        TB::issue(planB, dsB, p.ldb, s * BK, k_lim, lds0 + s * SM::STAGE + TA::BYTES);
    }
    // slab 0 has landed once at most the NS-2 younger slabs are outstanding
    wait_vmcnt<(NS - 2) * SM::LOADS>();
    __syncthreads();
    typename Mma<T>::frag fa[2][TM], fb[2][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i) fa[0][i] = TA::frag(smem_raw, wm * (BM / 2) + i * 32, 0, lane);
#pragma unroll
    for (int j = 0; j < TN; ++j) fb[0][j] = TB::frag(smem_raw + TA::BYTES, wn * (BN / 2) + j * 32, 0, lane);
    int stage = 0;
    for (int kt = 0; kt < nk; ++kt) {
        const unsigned char* a_s = smem_raw + stage * SM::STAGE;
        const unsigned char* b_s = a_s + TA::BYTES;
        const int next = stage == NS - 1 ? 0 : stage + 1;
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
            const int c = ks & 1, n = c ^ 1;   // KS is even: slab kt+1 starts in buffer 0 again
            if (ks + 1 < KS) {
#pragma unroll
                for (int i = 0; i < TM; ++i) fa[n][i] = TA::frag(a_s, wm * (BM / 2) + i * 32, ks + 1, lane);
#pragma unroll
                for (int j = 0; j < TN; ++j) fb[n][j] = TB::frag(b_s, wn * (BN / 2) + j * 32, ks + 1, lane);
            } else {
                // Before the last k-step of slab kt: slab kt+1 has landed once at most
                // the NS-3 younger slabs are outstanding.  After the barrier every wave
                // is past slab kt-1, so its stage is refilled with slab kt+NS-1, and the
                // first fragments of slab kt+1 are fetched under this slab's last MFMAs.
                wait_vmcnt<(NS - 3) * SM::LOADS>();
                __syncthreads();
#ifndef MOE_DEBUG_NOLOAD
                const int fill = stage == 0 ? NS - 1 : stage - 1;
                TA::issue(planA, dsA, p.lda, (kt + NS - 1) * BK, k_lim, lds0 + fill * SM::STAGE);
                TB::issue(planB, dsB, p.ldb, (kt + NS - 1) * BK, k_lim, lds0 + fill * SM::STAGE + TA::BYTES);
#endif
                const unsigned char* a_n = smem_raw + next * SM::STAGE;
#pragma unroll
                for (int i = 0; i < TM; ++i) fa[n][i] = TA::frag(a_n, wm * (BM / 2) + i * 32, 0, lane);
#pragma unroll
                for (int j = 0; j < TN; ++j) fb[n][j] = TB::frag(a_n + TA::BYTES, wn * (BN / 2) + j * 32, 0, lane);
            }
#pragma unroll
            for (int i = 0; i < TM; ++i)
#pragma unroll
                for (int j = 0; j < TN; ++j) acc[i][j] = Mma<T>::mma(fa[c][i], fb[c][j], acc[i][j]);
        }
        stage = next;
    }
    // drain the loads still in flight (they target LDS that the epilogue reuses)
    wait_vmcnt<0>();
    __syncthreads();

    // ---- epilogue: accumulators -> wave-private LDS strip -> row vectors -------
    // accumulator element v of lane l in a 32x32 tile: column l%32,
    // row 8*(v/4) + 4*(l/32) + v%4
    float* strip = reinterpret_cast<float*>(smem_raw) + wave * 32 * ELD;
    const int l32 = lane & 31, g = lane >> 5;
#pragma unroll
    for (int i = 0; i < TM; ++i) {
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v)
                strip[(8 * (v >> 2) + 4 * g + (v & 3)) * ELD + j * 32 + l32] = acc[i][j][v];
        const int mrow0 = m0 + wm * (BM / 2) + i * 32 + er;
        if constexpr (EPI == EPI_H_DACT) {
#pragma unroll 2
            for (int it = 0; it < NIT; ++it) {  // (almost) rolled: few copies of the activation code
                const float4 q = *reinterpret_cast<const float4*>(strip + (er + it * RPI) * ELD + ec);
                float v[4] = {q.x, q.y, q.z, q.w};
                const int m = mrow0 + it * RPI;
                if (m < m_lim && ncol < p.N)
                    epilogue4<T, EPI, ACT>(p, obase + (size_t)m * p.ldo + ncol, v, Vec4io<T>::zero());
            }
        } else {
#pragma unroll
            for (int it = 0; it < NIT; ++it) {
                const float4 q = *reinterpret_cast<const float4*>(strip + (er + it * RPI) * ELD + ec);
                float v[4] = {q.x, q.y, q.z, q.w};
                const int m = mrow0 + it * RPI;
                if (m < m_lim && ncol < p.N)
                    epilogue4<T, EPI, ACT>(p, obase + (size_t)m * p.ldo + ncol, v, aux[EPI == EPI_MUL ? i : 0][EPI == EPI_MUL ? it : 0]);
            }
        }
    }
}

template <typename T, int BM, int BN, int BK, bool A_KC, bool B_KC, int EPI, int ACT = 0>
static void launch_gemm(GemmArgs p, int E, hipStream_t st) {
    typedef GemmSmem<T, BM, BN, BK, A_KC, B_KC> SM;
    p.tiles_m = ceil_div(p.M, BM);
    p.tiles_n = ceil_div(p.N, BN);
    p.total_tiles = E * p.tiles_m * p.tiles_n;
    p.tiles_per_xcd = ceil_div(p.total_tiles, 8);
    const size_t smem = SM::BYTES;
    auto kern = grouped_gemm_kernel<T, BM, BN, BK, A_KC, B_KC, EPI, ACT>;
    if (smem > 64 * 1024) {
        // opt in (once per kernel instance) to more than 64 KB of the CU's 160 KB LDS
        static const hipError_t attr = hipFuncSetAttribute(
            (const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
        (void)attr;
    }
    kern<<<p.tiles_per_xcd * 8, 256, smem, st>>>(p);
}

size_t ffn_bwd_ws_bytes(const moe_shape* s) {
    return align_up((size_t)s->E * s->capacity * s->d_ff * elem_bytes(s->dtype), 256);
}

// Per-expert operand slices are addressed with 32-bit byte offsets.
static int check_slice_limits(const moe_shape* s) {
    const long long big = (long long)(s->d_model > s->d_ff ? s->d_model : s->d_ff);
    if (((long long)s->capacity + 512) * big * 4 >= (1ll << 31) || (long long)s->d_model * s->d_ff * 4 >= (1ll << 31))
        return MOE_ERR_SHAPE;
    return MOE_OK;
}

template <typename T, int BM, int BN, int BK>
static void ffn_fwd(const moe_shape* s, const void* xd, const int32_t* cnt, const void* W1,
                    const void* W2, void* h, void* a, void* yd, hipStream_t st) {
    const int E = s->E, C = s->capacity, d = s->d_model, f = s->d_ff;
    GemmArgs p = {};
    p.expert_count = cnt; p.var_k = 0;
    // z = xd W1 (not stored);  h = act(z), a = act'(z)
    p.A = xd; p.lda = d; p.strideA = (long long)C * d;
    p.B = W1; p.ldb = f; p.strideB = (long long)d * f;
    p.out0 = a; p.out1 = h; p.ldo = f; p.strideO = (long long)C * f;
    p.M = C; p.N = f; p.K = d;
    if (s->act == MOE_RELU) launch_gemm<T, BM, BN, BK, true, false, EPI_H_DACT, MOE_RELU>(p, E, st);
    else launch_gemm<T, BM, BN, BK, true, false, EPI_H_DACT, MOE_GELU>(p, E, st);
    // yd = h W2
    p.A = h; p.lda = f; p.strideA = (long long)C * f;
    p.B = W2; p.ldb = d; p.strideB = (long long)f * d;
    p.out0 = yd; p.out1 = nullptr; p.ldo = d; p.strideO = (long long)C * d;
    p.M = C; p.N = d; p.K = f;
    launch_gemm<T, BM, BN, BK, true, false, EPI_STORE>(p, E, st);
}

template <typename T, int BM, int BN, int BK>
static void ffn_bwd(const moe_shape* s, const void* dyd, const void* xd, const void* h,
                    const void* a, const int32_t* cnt, const void* W1, const void* W2, void* dxd,
                    float* dW1, float* dW2, void* dz, hipStream_t st) {
    const int E = s->E, C = s->capacity, d = s->d_model, f = s->d_ff;
    GemmArgs p = {};
    p.expert_count = cnt;
    // dz = (dyd W2^T) .* a:  B(r = n in f, k in d) = W2[n*d + k]
    p.var_k = 0;
    p.A = dyd; p.lda = d; p.strideA = (long long)C * d;
    p.B = W2; p.ldb = d; p.strideB = (long long)f * d;
    p.out0 = dz; p.aux = a; p.ldo = f; p.strideO = (long long)C * f;
    p.M = C; p.N = f; p.K = d;
    launch_gemm<T, BM, BN, BK, true, true, EPI_MUL>(p, E, st);
    // dxd = dz W1^T:  B(r = n in d, k in f) = W1[n*f + k]
    p.A = dz; p.lda = f; p.strideA = (long long)C * f;
    p.B = W1; p.ldb = f; p.strideB = (long long)d * f;
    p.out0 = dxd; p.aux = nullptr; p.ldo = d; p.strideO = (long long)C * d;
    p.M = C; p.N = d; p.K = f;
    launch_gemm<T, BM, BN, BK, true, true, EPI_STORE>(p, E, st);
    // dW2[f,d] = h^T dyd:  A(r = m in f, k = row) = h[k*f + m], B(r = n in d, k) = dyd[k*d + n]
    p.var_k = 1;
    p.A = h; p.lda = f; p.strideA = (long long)C * f;
    p.B = dyd; p.ldb = d; p.strideB = (long long)C * d;
    p.out0 = dW2; p.ldo = d; p.strideO = (long long)f * d;
    p.M = f; p.N = d; p.K = C;
    launch_gemm<T, BM, BN, BK, false, false, EPI_F32>(p, E, st);
    // dW1[d,f] = xd^T dz
    p.A = xd; p.lda = d; p.strideA = (long long)C * d;
    p.B = dz; p.ldb = f; p.strideB = (long long)C * f;
    p.out0 = dW1; p.ldo = f; p.strideO = (long long)d * f;
    p.M = d; p.N = f; p.K = C;
    launch_gemm<T, BM, BN, BK, false, false, EPI_F32>(p, E, st);
}

extern "C" int moe_expert_ffn_fwd(const moe_shape* shape, const void* xd,
                                  const int32_t* expert_count, const void* W1, const void* W2,
                                  void* h_saved, void* dact_saved, void* yd, void* stream) {
    int rc = check_shape(shape);
    if (rc) return rc;
    if ((rc = check_slice_limits(shape))) return rc;
    if (!xd || !expert_count || !W1 || !W2 || !h_saved || !dact_saved || !yd) return MOE_ERR_NULL;
    hipStream_t st = (hipStream_t)stream;
    if (shape->dtype == MOE_BF16)
        ffn_fwd<bf16_t, MOE_GEMM_BM, MOE_GEMM_BN, MOE_GEMM_BK>(shape, xd, expert_count, W1, W2, h_saved, dact_saved, yd, st);
    else
        ffn_fwd<float, 128, 128, 16>(shape, xd, expert_count, W1, W2, h_saved, dact_saved, yd, st);
    return launch_status();
}

extern "C" int moe_expert_ffn_bwd(const moe_shape* shape, const void* dyd, const void* xd,
                                  const void* h_saved, const void* dact_saved,
                                  const int32_t* expert_count, const void* W1, const void* W2,
                                  void* dxd, float* dW1, float* dW2, void* ws, size_t ws_bytes,
                                  void* stream) {
    int rc = check_shape(shape);
    if (rc) return rc;
    if ((rc = check_slice_limits(shape))) return rc;
    if (!dyd || !xd || !h_saved || !dact_saved || !expert_count || !W1 || !W2 || !dxd || !dW1 || !dW2)
        return MOE_ERR_NULL;
    if (!ws || ((uintptr_t)ws & 255) || ws_bytes < ffn_bwd_ws_bytes(shape)) return MOE_ERR_WORKSPACE;
    hipStream_t st = (hipStream_t)stream;
    if (shape->dtype == MOE_BF16)
        ffn_bwd<bf16_t, MOE_GEMM_BM, MOE_GEMM_BN, MOE_GEMM_BK>(shape, dyd, xd, h_saved, dact_saved, expert_count, W1, W2, dxd, dW1, dW2, ws, st);
    else
        ffn_bwd<float, 128, 128, 16>(shape, dyd, xd, h_saved, dact_saved, expert_count, W1, W2, dxd, dW1, dW2, ws, st);
    return launch_status();
}
