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
// Structure of a workgroup (bf16: 8 waves, 2 x 4, two per SIMD; fp32: 4 waves, 2 x 2;
// one persistent workgroup per CU):
//   * walks BM x BN output tiles.  Only tiles that hold rows exist; the expert-major
//     tile sequence is dealt block-cyclically, a block of as many consecutive tiles
//     as an XCD has workgroups going to one XCD (workgroup w runs on XCD w % 8), so
//     the tiles an XCD works on at one time are neighbours and share operand panels
//     in its L2, every workgroup gets the same number of tiles up to one, and a
//     heavily loaded expert is spread over all XCDs.  The slabs of all tiles of a
//     workgroup form one stream through the LDS ring: the next tile's first slabs
//     arrive under the current tile's epilogue;
//   * streams BK-deep slabs of both operands with 16-byte buffer loads that write
//     straight into LDS (no register staging).  bf16: BK = 64 (a k-contiguous operand
//     is fetched in 128-byte row pieces), two 64 KB stages.  The B half of a stage is
//     released early: a wave holds few B fragments, so it reads those of all four
//     k-steps during the slab's first step and the half is refilled three k-steps
//     before the A half - requests are in flight nearly all the time instead of in
//     one burst per slab, and B has 1.75 slab periods to arrive.  The slab's offset
//     is applied to the buffer descriptor (scalar work); the descriptor's range check
//     supplies the zero fill for rows >= n_e, so the loop has no branches.  LDS tiles
//     are unpadded and XOR-swizzled in 16-byte units (fragment reads are free of bank
//     conflicts);
//   * each wave accumulates (BM/2) x (BN/NWN) in 32x32 MFMA tiles
//     (bf16: v_mfma_f32_32x32x16_bf16, fp32: v_mfma_f32_32x32x2_f32); !KC bf16
//     operands are read from LDS with the transposing ds_read_b64_tr_b16.  A wave
//     issues strictly in order and an MFMA holds it for the MFMA's 32 cycles, so the
//     matrix pipe is kept busy by the SIMD's other wave; loads and fragment reads are
//     dealt evenly over the MFMA slots for that reason;
//   * the epilogue passes the accumulators through LDS so that every global
//     store is a full 8/16-byte vector along the row; the activation and its
//     derivative are evaluated once, in the forward epilogue (code kept in a
//     rolled loop), and the backward epilogue only multiplies by the saved
//     derivative, which it fetched into registers before the main loop;
//   * the backward's four products run as two launches of two independent products
//     each (dz with dW2, dxd with dW1): a workgroup walks its tiles of the first,
//     then of the second.
#include <math.h>
#include "moe_common.h"

// bf16 tile shape (tuning knobs; the defaults are the shipped configuration)
#ifndef MOE_GEMM_BM
#define MOE_GEMM_BM 256
#endif
#ifndef MOE_GEMM_BN
#define MOE_GEMM_BN 256
#endif
#ifndef MOE_GEMM_BK
#define MOE_GEMM_BK 64
#endif

typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef float f32x16_t __attribute__((ext_vector_type(16)));
typedef unsigned int u32x4_t __attribute__((ext_vector_type(4)));
typedef short s16x4_t __attribute__((ext_vector_type(4)));
typedef short s16x8_t __attribute__((ext_vector_type(8)));
typedef __attribute__((address_space(3))) s16x4_t lds_s16x4_t;

enum { EPI_STORE = 0, EPI_H_DACT = 1, EPI_MUL = 2, EPI_F32 = 3, EPI_H = 4 };   // EPI_H: activation only (forward-only use)

struct GemmArgs {
    const void* A; const void* B;
    void* out0; void* out1; const void* aux;
    const int32_t* expert_count;
    long long strideA, strideB, strideO;  // elements per expert
    int lda, ldb, ldo;
    int M, N, K;      // extents; the one bounded by expert_count is an upper limit
    int var_k;        // 0: rows (M) bounded by expert_count; 1: K bounded by it
    int tiles_m, tiles_n, E;
    // expert dropout in the activation epilogue (drop_thr = 0: off): an element is dropped when its
    // noise word < drop_thr, kept ones are scaled by drop_scale = 1 / (1 - p)
    uint32_t drop_thr;
    float drop_scale;
    uint64_t seed;
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

#define OOB_OFFSET 0x80000000u  // beyond any descriptor this kernel builds (slices < 2 GiB)

// LDS tile of one operand: BR rows (r) x BK reduction entries, unpadded, as
// 16-byte slots; slot p is filled by thread p % NT in its (p / NT)-th load.
//   KC : LDS row = r (BK entries),  slot = r*CPR + (chunk ^ swz(r))
//   !KC: LDS row = k (BR entries),  slot = k*CPR + (chunk ^ swz(k))
// swz: KC  -> consecutive rows that share a 256-byte bank window get distinct
//             chunk positions (16-byte fragment reads of 16 rows hit 64 banks);
//      !KC -> rows k, k+1, k+2, k+3 are shifted by 64 bytes each (the
//             transposing 8-byte reads of 4 rows x 64 bytes hit 64 banks).
template <typename T, int BR, int BK, bool KC, int NT> struct Tile {
    static constexpr int CN = 16 / (int)sizeof(T);           // elements per slot
    static constexpr int CPR = (KC ? BK : BR) / CN;          // slots per LDS row
    static constexpr int ROWS = KC ? BR : BK;
    static constexpr int SLOTS = ROWS * CPR;
    static constexpr int PER_THREAD = SLOTS / NT;
    static constexpr int BYTES = SLOTS * 16;
    static constexpr int WIN = CPR >= 16 ? 1 : 16 / CPR;     // rows per 256-byte window
    static_assert(SLOTS % NT == 0, "tile must be a multiple of the workgroup size in slots");
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
            const int p = threadIdx.x + i * NT;
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
    // Byte shift of the slab at reduction offset k0 inside the operand; it is applied to the
    // descriptor (scalar work, once per slab), not to every lane's offset.
    __device__ static __forceinline__ uint32_t slab_shift(int ld, int k0) {
        return (uint32_t)(KC ? k0 : k0 * ld) * (uint32_t)sizeof(T);
    }
    // The descriptor of one slab: base moved to the slab's first reduction entry.  For an
    // r-contiguous operand the range shrinks by the same amount, so that "reduction row < k_lim"
    // stays the descriptor's range check; for a k-contiguous operand the range (rows < r_lim)
    // is kept - every in-range row stays inside the tensor as long as the slab does.
    __device__ static __forceinline__ u32x4_t slab_desc(u32x4_t d, uint32_t shift) {
        const uint64_t base = ((uint64_t)(d[1] & 0xffffu) << 32 | d[0]) + shift;
        d[0] = (uint32_t)base;
        d[1] = (d[1] & 0xffff0000u) | (uint32_t)(base >> 32);
        if (!KC) d[2] = d[2] > shift ? d[2] - shift : 0u;
        return d;
    }
    // The i-th of this thread's loads of the slab whose descriptor is ds, into the stage at lds_base.
    // KG: the reduction length is not a multiple of BK, so a k-contiguous operand needs a per-lane
    // guard in its last slab (an r-contiguous one never does: the descriptor's range is that guard).
    template <bool KG>
    __device__ static __forceinline__ void issue_one(const Plan& pl, u32x4_t ds, int k0, int k_lim, uint32_t lds_base, int i) {
        const uint32_t wave_base = lds_base + (threadIdx.x >> 6) * 1024;
        uint32_t off = pl.voff[i];
        if (KC && KG) off = pl.kcol[i] + k0 < k_lim ? off : OOB_OFFSET;
        load_to_lds(ds, off, __builtin_amdgcn_readfirstlane(wave_base + i * NT * 16));
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
// h = act(z) and a = act'(z) together.  fp32 tensors use the accurate erff/expf.
// bf16 tensors (8 significant bits) use the three-term rational erfc of Abramowitz &
// Stegun 7.1.25 (absolute error of the normal cdf below 1.1e-5, i.e. 1/350 of a bf16
// rounding step at 1) with one exponential shared with the density and all scale
// factors folded into the constants: this epilogue is bound by vector-ALU issue
// (two transcendentals at quarter rate plus 13 other instructions per element).
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
        // phi(z) = exp2(-z^2 log2(e)/2 - log2 sqrt(2 pi));  t = 1 / (1 + 0.47047 |z| / sqrt 2)
        const float pdf = __builtin_amdgcn_exp2f(fmaf(z * z, -0.72134752044448170368f, -1.32574806473615920f));
        const float t = __builtin_amdgcn_rcpf(fmaf(0.33267252734483500f, fabsf(z), 1.0f));
        // Phi(-|z|) = erfc(|z|/sqrt 2)/2 = phi(z) t (b1 + b2 t + b3 t^2), b = sqrt(pi/2) (0.3480242, -0.0958798, 0.7478556)
        const float q = t * fmaf(fmaf(0.93729799615056560f, t, -0.12016750882298269f), t, 0.43618364998791710f) * pdf;
        cdf = z >= 0.0f ? 1.0f - q : q;
        zpdf = z * pdf;
    }
    h = z * cdf;
    a = cdf + zpdf;
}

// Output of one tile: raw buffer descriptors over the expert's rows in use, so that
// rows >= m_lim fall outside the range and their stores are dropped (no branches).
struct TileOut {
    __amdgpu_buffer_rsrc_t o0, o1, ax;
};

// One row vector of the output tile: off = byte offset inside the expert's output
// (BUF_OOB for a column beyond N), o = element index in the whole tensor (for the
// dropout noise), v = 4 accumulators, aux = the 4 saved derivatives (EPI_MUL only).
template <typename T, int EPI, int ACT>
__device__ __forceinline__ void epilogue4(const GemmArgs& p, const TileOut& to, uint32_t off, size_t o,
                                          float (&v)[4], typename Vec4io<T>::raw aux) {
    if constexpr (EPI == EPI_STORE) {
        Vec4buf<T>::store(to.o0, off, Vec4io<T>::pack(v));
    } else if constexpr (EPI == EPI_H_DACT) {
        float h[4], a[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) act_both<sizeof(T) == 2, ACT>(v[i], h[i], a[i]);
        if (p.drop_thr) {   // expert dropout (Sec. 5.4): o is the element index in [E, C, d_ff], a multiple of 4
            uint32_t w[4];
            noise_words(o, MOE_STREAM_DROPOUT, p.seed, w);
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const float sc = w[i] >= p.drop_thr ? p.drop_scale : 0.0f;
                h[i] *= sc;     // the mask rides in the saved derivative too, so the
                a[i] *= sc;     // backward needs no knowledge of it
            }
        }
        Vec4buf<T>::store(to.o0, off, Vec4io<T>::pack(a));
        Vec4buf<T>::store(to.o1, off, Vec4io<T>::pack(h));
    } else if constexpr (EPI == EPI_H) {
        float h[4], a[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) act_both<sizeof(T) == 2, ACT>(v[i], h[i], a[i]);   // the derivative is dead code here
        Vec4buf<T>::store(to.o0, off, Vec4io<T>::pack(h));
    } else if constexpr (EPI == EPI_MUL) {
        float a[4];
        Vec4io<T>::unpack(aux, a);
#pragma unroll
        for (int i = 0; i < 4; ++i) v[i] *= a[i];
        Vec4buf<T>::store(to.o0, off, Vec4io<T>::pack(v));
    } else {
        Vec4buf<float>::store(to.o0, off, make_float4(v[0], v[1], v[2], v[3]));
    }
}

// NWN = wavefronts along N (2 or 4); always 2 along M.
template <typename T, int BM, int BN, int BK, bool A_KC, bool B_KC, int NWN>
struct GemmSmem {
    static constexpr int NT = 128 * NWN;        // threads per workgroup
    typedef Tile<T, BM, BK, A_KC, NT> TA;
    typedef Tile<T, BN, BK, B_KC, NT> TB;
    static constexpr int STAGE = TA::BYTES + TB::BYTES;
#ifndef MOE_GEMM_NS
#define MOE_GEMM_NS 0
#endif
    // LDS ring: 1 slab being multiplied + NSTAGE-1 in flight (as many as fit beside the epilogue strips)
    static constexpr int NSTAGE = MOE_GEMM_NS ? MOE_GEMM_NS : (STAGE > 48 * 1024 ? 2 : (STAGE > 32 * 1024 ? 3 : 4));
    static constexpr int EPI_LD = BN / NWN + 8; // floats per staged epilogue row (4 rows apart -> other bank half)
    static constexpr int EPI_ROWS = 8;          // one accumulator register quad of both lane halves
    static constexpr size_t RING = (size_t)NSTAGE * STAGE;
    static constexpr size_t EPILOGUE = 2 * NWN * EPI_ROWS * (size_t)EPI_LD * sizeof(float);  // wave-private strips
    static constexpr size_t BYTES = RING + EPILOGUE;   // the epilogue never touches the ring
    static constexpr int LOADS = TA::PER_THREAD + TB::PER_THREAD;  // per thread per slab
    static_assert(NSTAGE * LOADS < 64, "vmcnt is a 6-bit counter");
    static_assert((BK / Mma<T>::KSTEP) % 2 == 0, "fragment double buffering needs an even number of k-steps");
    static_assert(BYTES + 4096 <= 160 * 1024, "LDS of one CU (the tile-walk table follows)");
};

// The walk of one workgroup over its tiles.  Only tiles that hold rows exist:
// expert e has ceil(n_e / BM) row tiles (all of them if the expert count is the
// reduction length: an empty expert's weight gradient is still written, as zeros).
// A table in LDS holds the running number of tiles per expert.  The tile
// sequence (expert-major) is dealt block-cyclically: with S workgroups per XCD
// (workgroup w serves XCD w % 8: ids are dealt round-robin to the XCDs), block b
// of S consecutive tiles goes to XCD b % 8, one tile per workgroup.  The tiles an
// XCD works on at one time are neighbours and share operand panels in its L2;
// every workgroup gets the same number of tiles up to one; and the tiles of a
// heavily loaded expert (long reductions in the weight-gradient GEMMs) are spread
// over all workgroups instead of piling up on one XCD.
#define WALK_BAND 4                     // row tiles per band of the walk inside an expert
#define WALK_SLOTS 257                  // experts + 1
#define WALK_BYTES (WALK_SLOTS * 4 + 12)
template <int BM, int BN>
struct TileWalk {
    const int* tp;          // LDS: tiles before expert e (tp[256] = all tiles)
    int t, t_end, step;
    int e, m0, n0, m_lim, k_lim;   // current tile

    // Fills the table (wave 0; 4 experts per lane) and synchronises the workgroup.
    __device__ static __forceinline__ void build(const GemmArgs& p, unsigned char* lds) {
        int* tpw = reinterpret_cast<int*>(lds);
        if (threadIdx.x < 64) {
            const int lane = threadIdx.x;
            int a[4];
            int sa = 0;
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const int ex = 4 * lane + i;
                int n = ex < p.E ? p.expert_count[ex] : 0;
                n = max(0, min(n, p.var_k ? p.K : p.M));
                const int tm = ex >= p.E ? 0 : (p.var_k ? p.tiles_m : (n + BM - 1) / BM);
                a[i] = tm * p.tiles_n;
                sa += a[i];
            }
            int ia = sa;
#pragma unroll
            for (int o = 1; o < 64; o <<= 1) {
                const int va = __shfl_up(ia, o, MOE_WAVE);
                if (lane >= o) ia += va;
            }
            int ea = ia - sa;
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                tpw[4 * lane + i] = ea;
                ea += a[i];
            }
            if (lane == 63) tpw[256] = ea;
        }
        __syncthreads();
    }
    __device__ __forceinline__ void start(const GemmArgs& p, const unsigned char* lds) {
        tp = reinterpret_cast<const int*>(lds);
        const int S = gridDim.x >> 3;
        step = 8 * S;
        t = (int)(blockIdx.x & 7) * S + (int)(blockIdx.x >> 3) - step;
        t_end = __builtin_amdgcn_readfirstlane(tp[256]);
        e = 0;
    }
    // moves to the workgroup's next tile; false when the walk is over
    __device__ __forceinline__ bool next(const GemmArgs& p) {
        t += step;
        if (t >= t_end) return false;
        while (t >= tp[e + 1]) ++e;          // t < tp[256]: stops at an expert that has tiles
        // everything here is the same in every lane; keep it in scalar registers
        e = __builtin_amdgcn_readfirstlane(e);
        const int first = __builtin_amdgcn_readfirstlane(tp[e]);
        const int count = __builtin_amdgcn_readfirstlane(tp[e + 1]) - first;
        const int rem = t - first;
        const int tm_e = count / p.tiles_n;   // row tiles of this expert
        // Inside an expert the tiles are taken band by band: a band is WALK_BAND row tiles high
        // and all column tiles wide, and inside it the row tile varies fastest.  A run of 32
        // consecutive tiles (what one XCD works on at a time) is then a 4 x 8 block that shares
        // 4 + 8 operand panels in the XCD's L2, whatever the expert's size (one row tile per
        // column tile, or the reverse, would fetch 32 + 1 panels for the same 32 tiles).
        int tm, tn;
        {
            const int band = rem / (WALK_BAND * p.tiles_n);
            const int r = rem - band * WALK_BAND * p.tiles_n;
            const int rows = min(WALK_BAND, tm_e - band * WALK_BAND);   // the last band may be lower
            tn = r / rows;
            tm = band * WALK_BAND + (r - tn * rows);
        }
        const int n_e = max(0, min(p.expert_count[e], p.var_k ? p.K : p.M));
        m0 = tm * BM; n0 = tn * BN;
        m_lim = p.var_k ? p.M : n_e;
        k_lim = p.var_k ? n_e : p.K;
        return true;
    }
};

// Persistent workgroups: each walks its tiles and treats the slabs of all of
// them as one stream through the LDS ring, so the first slabs of the next tile
// are already resident when the epilogue of the current one ends, and no
// workgroup launch or cold first load sits between two tiles.
template <typename T, int BM, int BN, int BK, bool A_KC, bool B_KC, int EPI, int ACT, int NWN, bool KG>
__device__ __forceinline__ void gemm_body(const GemmArgs& p) {
    typedef GemmSmem<T, BM, BN, BK, A_KC, B_KC, NWN> SM;
    typedef typename SM::TA TA;
    typedef typename SM::TB TB;
    typedef typename Vec4io<T>::raw raw;
    constexpr int TM = BM / 64, TN = BN / (32 * NWN);  // 32x32 MFMA tiles per wave (2 x NWN waves)
    constexpr int KS = BK / Mma<T>::KSTEP;
    constexpr int NS = SM::NSTAGE;
    extern __shared__ __align__(16) unsigned char smem_raw[];
    const uint32_t lds0 = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) unsigned char*)smem_raw;

    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int wm = wave / NWN, wn = wave % NWN;
    const int l32 = lane & 31, g = lane >> 5;

    // epilogue geometry: the wave's (BM/2) x (BN/2) sub-tile leaves in strips of 8
    // rows; a lane owns 4 consecutive columns of RPI-strided rows
    constexpr int ELD = SM::EPI_LD;
    constexpr int WCOLS = BN / NWN;
    constexpr int LPR = WCOLS / 4;                // lanes per staged row
    constexpr int RPI = 64 / LPR;                 // rows per wave instruction
    constexpr int NIT = SM::EPI_ROWS / RPI;       // row vectors per lane per strip
    static_assert(NIT >= 1, "strip narrower than a wavefront");
    const int er = lane / LPR, ec = (lane - er * LPR) * 4;
    float* strip = reinterpret_cast<float*>(smem_raw + SM::RING) + wave * SM::EPI_ROWS * ELD;

    // ---- producer: the stream of slabs of all tiles of this workgroup ---------
    unsigned char* walk_lds = smem_raw + SM::BYTES;
    TileWalk<BM, BN>::build(p, walk_lds);
    TileWalk<BM, BN> pw;       // tile whose slabs are being requested
    pw.start(p, walk_lds);
    bool p_more = pw.next(p);
    int p_kt = 0, p_nk = 0;
    u32x4_t dsA = {0, 0, 0, 0}, dsB = {0, 0, 0, 0};
    typename TA::Plan planA;
    typename TB::Plan planB;
    auto producer_setup = [&]() {
        dsA = TA::desc((const T*)p.A + (size_t)pw.e * p.strideA, p.lda, pw.m_lim, pw.k_lim);
        dsB = TB::desc((const T*)p.B + (size_t)pw.e * p.strideB, p.ldb, p.N, pw.k_lim);
        TA::plan(planA, p.lda, pw.m0, pw.m_lim);
        TB::plan(planB, p.ldb, pw.n0, p.N);
        p_kt = 0;
        p_nk = (pw.k_lim + BK - 1) / BK;
    };
    if (p_more) producer_setup();
    // requests the next slab of the stream into ring stage `st`; past the end of
    // the stream it requests out-of-range loads (zeros) so that every slab counts
    // the same number of loads in vmcnt
    // The request of a slab is split in two so that, inside the main loop, its
    // loads can be issued one at a time between MFMAs (a burst of all of them fills
    // the address FIFO of the memory pipe and stalls the wave's instruction issue).
    int pk0 = 0, pkl = 0;
    uint32_t plds = 0;
    u32x4_t pua = {0, 0, 0, 0}, pub = {0, 0, 0, 0};
    auto produce_prepare = [&](int st) {
        while (p_more && p_kt >= p_nk) {
            p_more = pw.next(p);
            if (p_more) producer_setup();
        }
        pk0 = p_more ? p_kt * BK : 0;
        pkl = p_more ? pw.k_lim : 0;              // k_lim 0: every guard fails, nothing is read
        if (!p_more) { dsA[2] = 0; dsB[2] = 0; }  // empty range: every load returns zeros
        const u32x4_t sdA = TA::slab_desc(dsA, TA::slab_shift(p.lda, pk0)), sdB = TB::slab_desc(dsB, TB::slab_shift(p.ldb, pk0));
        // the descriptors are wave-uniform by construction; say so to the compiler
        // (they must sit in scalar registers for the load instruction)
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            pua[i] = __builtin_amdgcn_readfirstlane(sdA[i]);
            pub[i] = __builtin_amdgcn_readfirstlane(sdB[i]);
        }
        plds = lds0 + st * SM::STAGE;
        ++p_kt;
    };
    auto produce_issue = [&](int i) {   // load i of the prepared slab (i < SM::LOADS; A's loads come first)
        if (i < TA::PER_THREAD) TA::template issue_one<KG>(planA, pua, pk0, pkl, plds, i);
        else TB::template issue_one<KG>(planB, pub, pk0, pkl, plds + TA::BYTES, i - TA::PER_THREAD);
    };
    auto produce = [&](int st) {
        produce_prepare(st);
#pragma unroll
        for (int i = 0; i < SM::LOADS; ++i) produce_issue(i);
    };

    // ---- consumer ---------------------------------------------------------------
    TileWalk<BM, BN> cw;
    cw.start(p, walk_lds);
    if (!cw.next(p)) return;       // nothing to do for this workgroup (uniform)
#pragma unroll
    for (int s = 0; s < NS; ++s) produce(s);
    // slab 0 of the stream has landed once at most the NS-1 younger slabs are outstanding
    wait_vmcnt<(NS - 1) * SM::LOADS>();
    __syncthreads();
#ifndef MOE_GEMM_BEARLY
#define MOE_GEMM_BEARLY 1
#endif
    // Two-stage ring with four k-steps per slab (the bf16 tiles): the B half of a stage is released
    // early.  A wave needs few B fragments (TN per k-step), so it reads those of all four k-steps
    // during the slab's first step; one barrier later nobody reads the B half again and it is
    // refilled three k-steps before the A half.  The two halves of a slab are then requested at
    // different times, there is (almost) always a request in flight, and B has 1.75 slab periods
    // to arrive instead of one.
    // (not in the instance whose epilogue keeps saved-derivative rows in registers through the
    // main loop: the extra fragment registers would spill there)
#ifndef MOE_GEMM_DZ_BEARLY
#define MOE_GEMM_DZ_BEARLY 0
#endif
    constexpr bool BEARLY = MOE_GEMM_BEARLY && NS == 2 && KS == 4 && (EPI != EPI_MUL || MOE_GEMM_DZ_BEARLY);
    typename Mma<T>::frag fa[2][TM], fb[BEARLY ? KS : 2][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i) fa[0][i] = TA::frag(smem_raw, wm * (BM / 2) + i * 32, 0, lane);
#pragma unroll
    for (int j = 0; j < TN; ++j) fb[0][j] = TB::frag(smem_raw + TA::BYTES, wn * WCOLS + j * 32, 0, lane);
    int stage = 0;

    bool more = true;
    while (more) {
        const int nk = (cw.k_lim + BK - 1) / BK;
        const size_t obase = (size_t)cw.e * p.strideO;
        const int ncol = cw.n0 + wn * WCOLS + ec;
        const int mrow = cw.m0 + wm * (BM / 2) + er;
        const int m_lim = cw.m_lim;

        // EPI_MUL: the saved derivative does not depend on the product.  The rows of
        // the first two 32-row blocks are requested now and ride in registers through
        // the main loop; the later blocks are requested while earlier ones are written.
#ifndef MOE_GEMM_AUXB
#define MOE_GEMM_AUXB 2
#endif
        constexpr int AUXB = EPI == EPI_MUL ? (TM < MOE_GEMM_AUXB ? TM : MOE_GEMM_AUXB) : 1;
        raw aux[AUXB][EPI == EPI_MUL ? 4 : 1][EPI == EPI_MUL ? NIT : 1];
        constexpr uint32_t OSZ = EPI == EPI_F32 ? 4u : (uint32_t)sizeof(T);   // bytes per output element
        const size_t obytes = (size_t)m_lim * p.ldo * OSZ;                    // the expert's rows in use
        TileOut to;
        to.o0 = buf_rsrc((const char*)p.out0 + obase * OSZ, obytes);
        to.o1 = buf_rsrc(EPI == EPI_H_DACT ? (const char*)p.out1 + obase * OSZ : nullptr, EPI == EPI_H_DACT ? obytes : 0);
        to.ax = buf_rsrc(EPI == EPI_MUL ? (const char*)p.aux + obase * OSZ : nullptr, EPI == EPI_MUL ? obytes : 0);
        const bool col_ok = ncol < p.N;
        // byte offset of this lane's row vector in row m of the expert's output; a row
        // >= m_lim lies beyond the descriptor's range by itself
        auto out_off = [&](int m) { return col_ok ? (uint32_t)(((size_t)m * p.ldo + ncol) * OSZ) : BUF_OOB; };
        auto fetch_aux = [&](int buf, int i) {
#pragma unroll
            for (int q = 0; q < 4; ++q)
#pragma unroll
                for (int it = 0; it < NIT; ++it)
                    aux[buf][q][it] = Vec4buf<T>::load(to.ax, out_off(mrow + i * 32 + q * 8 + it * RPI));
        };
        if constexpr (EPI == EPI_MUL) {
            if (nk == 0) {
#pragma unroll
                for (int i = 0; i < AUXB; ++i) fetch_aux(i, i);
            }
        }

        f32x16_t acc[TM][TN];
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int j = 0; j < TN; ++j)
#pragma unroll
                for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.0f;

        for (int kt = 0; kt < nk; ++kt) {
            const unsigned char* a_s = smem_raw + stage * SM::STAGE;
            const unsigned char* b_s = a_s + TA::BYTES;
            const int next = stage == NS - 1 ? 0 : stage + 1;
            if constexpr (BEARLY) {
                constexpr int NMMA = TM * TN;
                static_assert(TM + TN <= NMMA && TB::PER_THREAD <= NMMA && TA::PER_THREAD <= NMMA, "one request per MFMA slot");
                // ---- k-step 0: MFMAs on (fa[0], fb[0]); A fragments of step 1 and B fragments of steps 1..3
#pragma unroll
                for (int i = 0; i < TM; ++i) fa[1][i] = TA::frag(a_s, wm * (BM / 2) + i * 32, 1, lane);
#pragma unroll
                for (int ks = 1; ks < KS; ++ks)
#pragma unroll
                    for (int j = 0; j < TN; ++j) fb[ks][j] = TB::frag(b_s, wn * WCOLS + j * 32, ks, lane);
#pragma unroll
                for (int i = 0; i < TM; ++i)
#pragma unroll
                    for (int j = 0; j < TN; ++j) acc[i][j] = Mma<T>::mma(fa[0][i], fb[0][j], acc[i][j]);
#pragma unroll
                for (int q = 0; q < NMMA; ++q) {
                    __builtin_amdgcn_sched_group_barrier(0x100, 3, 0);   // LDS reads
                    __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);   // one MFMA
                }
                __builtin_amdgcn_sched_barrier(0);
                // every B fragment of this slab is in registers once this wave's LDS reads have
                // returned; when all waves are here the B half of the stage is refilled
                wait_vmcnt_lgkm0<63>();
                __builtin_amdgcn_s_barrier();
                asm volatile("" ::: "memory");
                produce_prepare(stage);
                // ---- k-step 1: MFMAs on (fa[1], fb[1]); B requests; A fragments of step 2
                // (a wave issues its instructions strictly one after another, an MFMA holding it for the
                // MFMA's 32 cycles: only the other wave of the SIMD can fill the matrix pipe meanwhile.  The
                // requests and fragment reads are therefore dealt evenly over the MFMA slots - a long run of
                // them in one place leaves the pipe idle whenever both waves are in such a run.)
#pragma unroll
                for (int q = 0; q < NMMA; ++q) {
                    constexpr int LSTEP = NMMA / TB::PER_THREAD >= 1 ? NMMA / TB::PER_THREAD : 1;   // a request every LSTEP slots
                    if (q % LSTEP == 0 && q / LSTEP < TB::PER_THREAD) produce_issue(TA::PER_THREAD + q / LSTEP);
                    if (NMMA >= 2 * TM ? (q % 2 == 1 && q / 2 < TM) : q < TM) {
                        const int i = NMMA >= 2 * TM ? q / 2 : q;
                        fa[0][i] = TA::frag(a_s, wm * (BM / 2) + i * 32, 2, lane);
                    }
                    acc[q / TN][q % TN] = Mma<T>::mma(fa[1][q / TN], fb[1][q % TN], acc[q / TN][q % TN]);
                    __builtin_amdgcn_sched_barrier(0);
                }
                // ---- k-step 2: MFMAs on (fa[0], fb[2]); A fragments of step 3
#pragma unroll
                for (int q = 0; q < NMMA; ++q) {
                    if (NMMA >= 2 * TM ? (q % 2 == 0 && q / 2 < TM) : q < TM) {
                        const int i = NMMA >= 2 * TM ? q / 2 : q;
                        fa[1][i] = TA::frag(a_s, wm * (BM / 2) + i * 32, 3, lane);
                    }
                    acc[q / TN][q % TN] = Mma<T>::mma(fa[0][q / TN], fb[2][q % TN], acc[q / TN][q % TN]);
                    __builtin_amdgcn_sched_barrier(0);
                }
                // ---- k-step 3: the next slab (requested a slab period ago for A, 1.75 for B) has
                // landed once only the B requests of this slab's step 1 are outstanding (loads complete
                // in order; anything else that is younger only makes the wait longer); every A
                // fragment of this slab is in registers, so the A half is refilled; the next
                // slab's first fragments are fetched under the MFMAs on (fa[1], fb[3])
                wait_vmcnt_lgkm0<TB::PER_THREAD>();
                __builtin_amdgcn_s_barrier();
                asm volatile("" ::: "memory");
                if constexpr (EPI == EPI_MUL) {
                    if (kt == 0) {
#pragma unroll
                        for (int i = 0; i < AUXB; ++i) fetch_aux(i, i);
                    }
                }
                const unsigned char* a_n = smem_raw + next * SM::STAGE;
#pragma unroll
                for (int q = 0; q < NMMA; ++q) {
                    constexpr int LSTEP = NMMA / TA::PER_THREAD >= 1 ? NMMA / TA::PER_THREAD : 1;
                    if (q % LSTEP == 0 && q / LSTEP < TA::PER_THREAD) produce_issue(q / LSTEP);
                    if (NMMA >= 2 * TM) {
                        // odd slots: one A fragment each; the B fragments (needed first) ride with the first ones
                        if (q % 2 == 1) {
                            const int i = q / 2;
                            if (i < TM) fa[0][i] = TA::frag(a_n, wm * (BM / 2) + i * 32, 0, lane);
                            if (i < TN) fb[0][i] = TB::frag(a_n + TA::BYTES, wn * WCOLS + i * 32, 0, lane);
                        }
                    } else {
                        if (q < TM) fa[0][q] = TA::frag(a_n, wm * (BM / 2) + q * 32, 0, lane);
                        else if (q < TM + TN) fb[0][q - TM] = TB::frag(a_n + TA::BYTES, wn * WCOLS + (q - TM) * 32, 0, lane);
                    }
                    acc[q / TN][q % TN] = Mma<T>::mma(fa[1][q / TN], fb[3][q % TN], acc[q / TN][q % TN]);
                    __builtin_amdgcn_sched_barrier(0);
                }
                stage = next;
                continue;
            }
#pragma unroll
            for (int ks = 0; ks < KS; ++ks) {
                const int c = ks & 1, n = c ^ 1;   // KS is even: every slab starts in buffer 0
                if (ks + 1 < KS) {
#pragma unroll
                    for (int i = 0; i < TM; ++i) fa[n][i] = TA::frag(a_s, wm * (BM / 2) + i * 32, ks + 1, lane);
#pragma unroll
                    for (int j = 0; j < TN; ++j) fb[n][j] = TB::frag(b_s, wn * WCOLS + j * 32, ks + 1, lane);
                } else {
                    // Before the last k-step of a slab: its fragments are already in
                    // registers (requested one step ago; the wait below covers them), so once
                    // every wave is here nobody reads this stage again and it is refilled at
                    // once with the slab NS positions down the stream.  The next slab (this
                    // tile's or the next tile's first) has landed once at most the NS-2
                    // younger ones are outstanding; its first fragments are fetched under
                    // this slab's last MFMAs.
                    wait_vmcnt_lgkm0<(NS - 2) * SM::LOADS>();
                    __builtin_amdgcn_s_barrier();
                    asm volatile("" ::: "memory");
                    if constexpr (EPI == EPI_MUL) {
                        // requested right after a wait, a whole slab period before the next one:
                        // every wait of the loop is for all outstanding loads, these included
                        if (kt == 0) {
#pragma unroll
                            for (int i = 0; i < AUXB; ++i) fetch_aux(i, i);
                        }
                    }
                    produce_prepare(stage);
                    const unsigned char* a_n = smem_raw + next * SM::STAGE;
                    // hand-laid schedule of the last step: per MFMA one slab request and one
                    // fragment read of the next slab
                    constexpr int NMMA = TM * TN, LPM = (SM::LOADS + NMMA - 1) / NMMA;
#pragma unroll
                    for (int q = 0; q < NMMA; ++q) {
#pragma unroll
                        for (int u = 0; u < LPM; ++u)
                            if (q * LPM + u < SM::LOADS) produce_issue(q * LPM + u);
                        if (q < TM) fa[n][q] = TA::frag(a_n, wm * (BM / 2) + q * 32, 0, lane);
                        else if (q < TM + TN) fb[n][q - TM] = TB::frag(a_n + TA::BYTES, wn * WCOLS + (q - TM) * 32, 0, lane);
                        acc[q / TN][q % TN] = Mma<T>::mma(fa[c][q / TN], fb[c][q % TN], acc[q / TN][q % TN]);
                        __builtin_amdgcn_sched_barrier(0);
                    }
                    static_assert(TM + TN <= NMMA, "one fragment read per MFMA slot");
                    continue;
                }
#pragma unroll
                for (int i = 0; i < TM; ++i)
#pragma unroll
                    for (int j = 0; j < TN; ++j) acc[i][j] = Mma<T>::mma(fa[c][i], fb[c][j], acc[i][j]);
                // issue order: the fragment reads of the next k-step go out under the
                // first MFMAs of this one, so a full step of matrix work covers their latency
#pragma unroll
                for (int q = 0; q < TM * TN; ++q) {
                    __builtin_amdgcn_sched_group_barrier(0x100, 2, 0);   // LDS reads
                    __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);   // one MFMA
                }
                __builtin_amdgcn_sched_barrier(0);   // no MFMA drifts into the next step
            }
            stage = next;
        }

        // ---- epilogue: accumulators -> wave-private LDS strip -> row vectors --------
        // accumulator element v of lane l in a 32x32 tile: column l%32,
        // row 8*(v/4) + 4*(l/32) + v%4; strip s = (i, q) = (s/4, s%4) holds rows i*32 + 8q .. +7.
        // LDS operations of a wave execute in order, so strip s+1 is written and read
        // back (into the other register set) before the vectors of strip s are used:
        // the LDS round trip of every strip hides behind the previous strip's work.
        constexpr int NSTRIP = 4 * TM;
        auto write_strip = [&](int s_) {
            const int i = s_ >> 2, q = s_ & 3;
#pragma unroll
            for (int j = 0; j < TN; ++j)
#pragma unroll
                for (int r = 0; r < 4; ++r) strip[(4 * g + r) * ELD + j * 32 + l32] = acc[i][j][4 * q + r];
        };
        auto read_strip = [&](float4 (&w)[NIT]) {
#pragma unroll
            for (int it = 0; it < NIT; ++it) w[it] = *reinterpret_cast<const float4*>(strip + (er + it * RPI) * ELD + ec);
        };
        constexpr bool ROLLED = EPI == EPI_H_DACT || EPI == EPI_H;   // long per-vector code: kept in a rolled loop
        float4 w[ROLLED ? 1 : 2][NIT];
        write_strip(0);
        if constexpr (!ROLLED) read_strip(w[0]);
#pragma unroll
        for (int s_ = 0; s_ < NSTRIP; ++s_) {
            const int i = s_ >> 2, q = s_ & 3;
            const int m_strip = mrow + i * 32 + q * 8;
            if constexpr (ROLLED) {
                // one copy of the activation code per strip; the next vector is read from
                // LDS before the current one is worked on (carried in registers, no arrays)
                float4 cur = *reinterpret_cast<const float4*>(strip + er * ELD + ec);
#pragma unroll 1
                for (int it = 0; it < NIT; ++it) {
                    const int itn = it + 1 < NIT ? it + 1 : it;
                    const float4 nxt = *reinterpret_cast<const float4*>(strip + (er + itn * RPI) * ELD + ec);
                    float v[4] = {cur.x, cur.y, cur.z, cur.w};
                    const int m = m_strip + it * RPI;
                    epilogue4<T, EPI, ACT>(p, to, out_off(m), obase + (size_t)m * p.ldo + ncol, v, Vec4io<T>::zero());
                    cur = nxt;
                }
                if (s_ + 1 < NSTRIP) write_strip(s_ + 1);
            } else {
                if (s_ + 1 < NSTRIP) {
                    write_strip(s_ + 1);
                    read_strip(w[(s_ + 1) & 1]);
                }
#pragma unroll
                for (int it = 0; it < NIT; ++it) {
                    const float4 x4 = w[s_ & 1][it];
                    float v[4] = {x4.x, x4.y, x4.z, x4.w};
                    const int m = m_strip + it * RPI;
                    epilogue4<T, EPI, ACT>(p, to, out_off(m), 0, v,
                                           aux[EPI == EPI_MUL ? i % AUXB : 0][EPI == EPI_MUL ? q : 0][EPI == EPI_MUL ? it : 0]);
                }
            }
            if constexpr (EPI == EPI_MUL) {
                if (q == 3 && i + AUXB < TM) fetch_aux(i % AUXB, i + AUXB);   // the buffer just used is free again
            }
        }
        more = cw.next(p);
    }
    // the zero-fill loads requested past the end of the stream target this
    // workgroup's LDS: wait for them before the workgroup retires
    wait_vmcnt<0>();
}

template <typename T, int BM, int BN, int BK, bool A_KC, bool B_KC, int EPI, int ACT, int NWN, bool KG>
__global__ __launch_bounds__(128 * NWN, 2) void grouped_gemm_kernel(const GemmArgs p) {   // two waves per SIMD: at most 256 registers
    gemm_body<T, BM, BN, BK, A_KC, B_KC, EPI, ACT, NWN, KG>(p);
}

// Two independent grouped GEMMs in one launch: every workgroup walks its tiles of the
// first, then its tiles of the second.  Nothing is synchronised between workgroups (the
// two products must not depend on each other), so a workgroup that is done with the first
// starts the second at once: one launch, one ramp-up and one tail instead of two, and the
// workgroups drift apart, which spreads the store bursts of their epilogues.
template <typename T, int BM, int BN, int BK, bool A1, bool B1, int EPI1, bool A2, bool B2, int EPI2, int NWN, bool KG>
__global__ __launch_bounds__(128 * NWN, 2) void grouped_gemm_pair_kernel(const GemmArgs p1, const GemmArgs p2) {
    gemm_body<T, BM, BN, BK, A1, B1, EPI1, 0, NWN, KG>(p1);
    __syncthreads();      // every wave is done with the ring and the tile table of the first product
    gemm_body<T, BM, BN, BK, A2, B2, EPI2, 0, NWN, KG>(p2);
}

// Number of compute units of the current device (looked up once per device).
static int num_cus() {
    static int cached[64];
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return 256;
    int n = __atomic_load_n(&cached[dev], __ATOMIC_RELAXED);
    if (n == 0) {
        int v = 0;
        n = (hipDeviceGetAttribute(&v, hipDeviceAttributeMultiprocessorCount, dev) == hipSuccess && v > 0) ? v : 256;
        __atomic_store_n(&cached[dev], n, __ATOMIC_RELAXED);
    }
    return n;
}

#ifndef MOE_GEMM_NWN
#define MOE_GEMM_NWN 4
#endif
// one persistent workgroup per CU (its LDS footprint allows no second one), in groups of 8 so
// that every XCD gets the same number; never more than there could be tiles
static int gemm_grid(long long tiles) {
    const long long most = (tiles + 7) / 8;
    int per_xcd = num_cus() / 8;
    if (per_xcd < 1) per_xcd = 1;
    if (per_xcd > most) per_xcd = (int)most;
    return per_xcd * 8;
}

template <typename T, int BM, int BN, int BK, bool A_KC, bool B_KC, int EPI, int ACT = 0>
static bool launch_gemm(GemmArgs p, int E, hipStream_t st) {
    constexpr int NWN = sizeof(T) == 2 ? MOE_GEMM_NWN : 2;
    typedef GemmSmem<T, BM, BN, BK, A_KC, B_KC, NWN> SM;
    p.tiles_m = ceil_div(p.M, BM);
    p.tiles_n = ceil_div(p.N, BN);
    p.E = E;
    const size_t smem = SM::BYTES + WALK_BYTES;
    const int grid = gemm_grid((long long)E * p.tiles_m * p.tiles_n);
    // a k-contiguous operand whose reduction length is not a multiple of BK needs the guarded instance
    const bool kg = (A_KC || B_KC) && !p.var_k && p.K % BK != 0;
    static unsigned long long opted[2] = {0, 0};
    if (kg) {
        auto kern = grouped_gemm_kernel<T, BM, BN, BK, A_KC, B_KC, EPI, ACT, NWN, true>;
        if (!lds_opt_in((const void*)kern, smem, &opted[1])) return false;
        kern<<<grid, SM::NT, smem, st>>>(p);
    } else {
        auto kern = grouped_gemm_kernel<T, BM, BN, BK, A_KC, B_KC, EPI, ACT, NWN, false>;
        if (!lds_opt_in((const void*)kern, smem, &opted[0])) return false;
        kern<<<grid, SM::NT, smem, st>>>(p);
    }
    return true;
}

template <typename T, int BM, int BN, int BK, bool A1, bool B1, int EPI1, bool A2, bool B2, int EPI2>
static bool launch_gemm_pair(GemmArgs p1, GemmArgs p2, int E, hipStream_t st) {
    constexpr int NWN = sizeof(T) == 2 ? MOE_GEMM_NWN : 2;
    typedef GemmSmem<T, BM, BN, BK, A1, B1, NWN> SM1;
    typedef GemmSmem<T, BM, BN, BK, A2, B2, NWN> SM2;
    static_assert(SM1::NT == SM2::NT, "one workgroup shape");
    p1.tiles_m = ceil_div(p1.M, BM); p1.tiles_n = ceil_div(p1.N, BN); p1.E = E;
    p2.tiles_m = ceil_div(p2.M, BM); p2.tiles_n = ceil_div(p2.N, BN); p2.E = E;
    const size_t smem = (SM1::BYTES > SM2::BYTES ? SM1::BYTES : SM2::BYTES) + WALK_BYTES;
    const long long t1 = (long long)E * p1.tiles_m * p1.tiles_n, t2 = (long long)E * p2.tiles_m * p2.tiles_n;
    const int grid = gemm_grid(t1 > t2 ? t1 : t2);
    const bool kg = ((A1 || B1) && !p1.var_k && p1.K % BK != 0) || ((A2 || B2) && !p2.var_k && p2.K % BK != 0);
    static unsigned long long opted[2] = {0, 0};
    if (kg) {
        auto kern = grouped_gemm_pair_kernel<T, BM, BN, BK, A1, B1, EPI1, A2, B2, EPI2, NWN, true>;
        if (!lds_opt_in((const void*)kern, smem, &opted[1])) return false;
        kern<<<grid, SM1::NT, smem, st>>>(p1, p2);
    } else {
        auto kern = grouped_gemm_pair_kernel<T, BM, BN, BK, A1, B1, EPI1, A2, B2, EPI2, NWN, false>;
        if (!lds_opt_in((const void*)kern, smem, &opted[0])) return false;
        kern<<<grid, SM1::NT, smem, st>>>(p1, p2);
    }
    return true;
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
static bool ffn_fwd(const moe_shape* s, const void* xd, const int32_t* cnt, const void* W1,
                    const void* W2, void* h, void* a, void* yd, float drop_p, uint64_t seed, hipStream_t st) {
    const int E = s->E, C = s->capacity, d = s->d_model, f = s->d_ff;
    GemmArgs p = {};
    p.expert_count = cnt; p.var_k = 0;
    if (drop_p > 0.0f) {
        p.drop_thr = (uint32_t)floor((double)drop_p * 4294967296.0);
        p.drop_scale = (float)(1.0 / (1.0 - (double)drop_p));
        p.seed = seed;
    }
    // z = xd W1 (not stored);  h = act(z), a = act'(z)
    p.A = xd; p.lda = d; p.strideA = (long long)C * d;
    p.B = W1; p.ldb = f; p.strideB = (long long)d * f;
    p.out0 = a; p.out1 = h; p.ldo = f; p.strideO = (long long)C * f;
    p.M = C; p.N = f; p.K = d;
    bool ok;
    if (!a) {   // forward-only: the derivative is neither computed nor stored
        p.out0 = h; p.out1 = nullptr;
        if (s->act == MOE_RELU) ok = launch_gemm<T, BM, BN, BK, true, false, EPI_H, MOE_RELU>(p, E, st);
        else ok = launch_gemm<T, BM, BN, BK, true, false, EPI_H, MOE_GELU>(p, E, st);
    } else if (s->act == MOE_RELU) ok = launch_gemm<T, BM, BN, BK, true, false, EPI_H_DACT, MOE_RELU>(p, E, st);
    else ok = launch_gemm<T, BM, BN, BK, true, false, EPI_H_DACT, MOE_GELU>(p, E, st);
    if (!ok) return false;
    // yd = h W2
    p.A = h; p.lda = f; p.strideA = (long long)C * f;
    p.B = W2; p.ldb = d; p.strideB = (long long)f * d;
    p.out0 = yd; p.out1 = nullptr; p.ldo = d; p.strideO = (long long)C * d;
    p.M = C; p.N = d; p.K = f;
    p.drop_thr = 0;
    return launch_gemm<T, BM, BN, BK, true, false, EPI_STORE>(p, E, st);
}

template <typename T, int BM, int BN, int BK>
static bool ffn_bwd(const moe_shape* s, const void* dyd, const void* xd, const void* h,
                    const void* a, const int32_t* cnt, const void* W1, const void* W2, void* dxd,
                    float* dW1, float* dW2, void* dz, hipStream_t st) {
    const int E = s->E, C = s->capacity, d = s->d_model, f = s->d_ff;
    // Four products in two launches.  dW2 needs only h and dyd, so it shares a launch with dz;
    // dxd and dW1 both need dz and share the second one.
    GemmArgs p = {}, q = {};
    p.expert_count = q.expert_count = cnt;
    // dz = (dyd W2^T) .* a:  B(r = n in f, k in d) = W2[n*d + k]
    p.var_k = 0;
    p.A = dyd; p.lda = d; p.strideA = (long long)C * d;
    p.B = W2; p.ldb = d; p.strideB = (long long)f * d;
    p.out0 = dz; p.aux = a; p.ldo = f; p.strideO = (long long)C * f;
    p.M = C; p.N = f; p.K = d;
    // dW2[f,d] = h^T dyd:  A(r = m in f, k = row) = h[k*f + m], B(r = n in d, k) = dyd[k*d + n]
    q.var_k = 1;
    q.A = h; q.lda = f; q.strideA = (long long)C * f;
    q.B = dyd; q.ldb = d; q.strideB = (long long)C * d;
    q.out0 = dW2; q.ldo = d; q.strideO = (long long)f * d;
    q.M = f; q.N = d; q.K = C;
    if (!launch_gemm_pair<T, BM, BN, BK, true, true, EPI_MUL, false, false, EPI_F32>(p, q, E, st)) return false;
    // dxd = dz W1^T:  B(r = n in d, k in f) = W1[n*f + k]
    p.A = dz; p.lda = f; p.strideA = (long long)C * f;
    p.B = W1; p.ldb = f; p.strideB = (long long)d * f;
    p.out0 = dxd; p.aux = nullptr; p.ldo = d; p.strideO = (long long)C * d;
    p.M = C; p.N = d; p.K = f;
    // dW1[d,f] = xd^T dz
    q.A = xd; q.lda = d; q.strideA = (long long)C * d;
    q.B = dz; q.ldb = f; q.strideB = (long long)C * f;
    q.out0 = dW1; q.ldo = f; q.strideO = (long long)d * f;
    q.M = d; q.N = f; q.K = C;
    return launch_gemm_pair<T, BM, BN, BK, true, true, EPI_STORE, false, false, EPI_F32>(p, q, E, st);
}

static int ffn_fwd_impl(const moe_shape* shape, const void* xd, const int32_t* expert_count,
                        const void* W1, const void* W2, float drop_p, uint64_t seed, void* h_saved,
                        void* dact_saved, void* yd, void* stream) {
    int rc = check_shape(shape);
    if (rc) return rc;
    if ((rc = check_slice_limits(shape))) return rc;
    if (!xd || !expert_count || !W1 || !W2 || !h_saved || !yd) return MOE_ERR_NULL;   // dact_saved may be NULL
    if (!(drop_p >= 0.0f && drop_p < 1.0f)) return MOE_ERR_SHAPE;
    if (drop_p > 0.0f && !dact_saved) return MOE_ERR_NULL;      // dropout is a training feature
    if (drop_p > 0.0f && floor((double)drop_p * 4294967296.0) < 1.0) drop_p = 0.0f;   // below one part in 2^32
    hipStream_t st = (hipStream_t)stream;
    const bool ok = shape->dtype == MOE_BF16
        ? ffn_fwd<bf16_t, MOE_GEMM_BM, MOE_GEMM_BN, MOE_GEMM_BK>(shape, xd, expert_count, W1, W2, h_saved, dact_saved, yd, drop_p, seed, st)
        : ffn_fwd<float, 128, 128, 16>(shape, xd, expert_count, W1, W2, h_saved, dact_saved, yd, drop_p, seed, st);
    return ok ? launch_status() : MOE_ERR_LAUNCH;
}

extern "C" int moe_expert_ffn_fwd(const moe_shape* shape, const void* xd,
                                  const int32_t* expert_count, const void* W1, const void* W2,
                                  void* h_saved, void* dact_saved, void* yd, void* stream) {
    return ffn_fwd_impl(shape, xd, expert_count, W1, W2, 0.0f, 0, h_saved, dact_saved, yd, stream);
}

extern "C" int moe_expert_ffn_fwd_dropout(const moe_shape* shape, const void* xd,
                                          const int32_t* expert_count, const void* W1, const void* W2,
                                          float drop_p, uint64_t seed, void* h_saved, void* dact_saved,
                                          void* yd, void* stream) {
    return ffn_fwd_impl(shape, xd, expert_count, W1, W2, drop_p, seed, h_saved, dact_saved, yd, stream);
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
    const bool ok = shape->dtype == MOE_BF16
        ? ffn_bwd<bf16_t, MOE_GEMM_BM, MOE_GEMM_BN, MOE_GEMM_BK>(shape, dyd, xd, h_saved, dact_saved, expert_count, W1, W2, dxd, dW1, dW2, ws, st)
        : ffn_bwd<float, 128, 128, 16>(shape, dyd, xd, h_saved, dact_saved, expert_count, W1, W2, dxd, dW1, dW2, ws, st);
    return ok ? launch_status() : MOE_ERR_LAUNCH;
}
