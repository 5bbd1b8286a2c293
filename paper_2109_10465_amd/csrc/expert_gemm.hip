// Grouped expert GEMMs on the MFMA matrix cores: the per-expert feed-forward
// block d_model -> d_ff -> d_model, forward and backward (Sec. 4.2 "Model
// details"; Sec. 2.3: these matmuls are where the layer's time goes).
//
// One kernel template serves the six contractions.  Per expert e with
// n_e = expert_count[e] rows in use:
//   forward   z = xd W1        (rows x d)(d x f)     epilogue: z, h = act(z)
//             yd = h W2        (rows x f)(f x d)
//   backward  dz = (dyd W2^T) .* act'(z)
//             dxd = dz W1^T
//             dW2 = h^T dyd    (f x rows)(rows x d)  fp32 output, K = rows
//             dW1 = xd^T dz    (d x rows)(rows x f)
// Each operand is described as a (row index r, reduction index k) array that is
// either k-contiguous in memory (KC) or r-contiguous (!KC); no transposed copy
// of any tensor is ever materialised.  A workgroup of 4 waves owns a BM x BN
// output tile, stages BK-deep slabs of both operands through double-buffered
// LDS with 16-byte loads, and each wave accumulates (BM/2) x (BN/2) in 32x32
// MFMA tiles (bf16: v_mfma_f32_32x32x16_bf16; fp32: v_mfma_f32_32x32x2_f32).
// Workgroup ids are remapped so that consecutive tiles of one expert land on
// the same XCD and share its L2.
#include "moe_common.h"

typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef float f32x16_t __attribute__((ext_vector_type(16)));

enum { EPI_STORE = 0, EPI_Z_H = 1, EPI_DZ = 2, EPI_F32 = 3 };

struct GemmArgs {
    const void* A; const void* B;
    void* out0; void* out1; const void* aux;
    const int32_t* expert_count;
    long long strideA, strideB, strideO;  // elements per expert
    int lda, ldb, ldo;
    int M, N, K;      // extents; the one bounded by expert_count is an upper limit
    int var_k;        // 0: rows (M) bounded by expert_count; 1: K bounded by it
    int act;
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

// LDS tile of one operand: BR rows (r) x BK reduction entries.
//   KC : element (r,k) at [r*LD + k],  LD = BK + PAD
//   !KC: element (r,k) at [k*LD + r],  LD = BR + PAD
template <typename T, int BR, int BK, bool KC> struct Tile {
    static constexpr int CN = 16 / (int)sizeof(T);  // elements per 16-byte chunk
    static constexpr int PAD = CN;
    static constexpr int LD = (KC ? BK : BR) + PAD;
    static constexpr int ROWS = KC ? BR : BK;        // LDS rows
    static constexpr int CPR = (KC ? BK : BR) / CN;  // chunks per LDS row
    static constexpr int CHUNKS = ROWS * CPR;
    static constexpr int PER_THREAD = (CHUNKS + 255) / 256;
    static constexpr int ELEMS = ROWS * LD;

    // global -> registers (zero fill outside [r_lim) x [k_lim))
    __device__ static __forceinline__ void fetch(uint4 (&reg)[PER_THREAD], const T* __restrict__ g,
                                                 int ld, int r0, int k0, int r_lim, int k_lim) {
#pragma unroll
        for (int i = 0; i < PER_THREAD; ++i) {
            const int c = threadIdx.x + i * 256;
            const int row = c / CPR, col = (c - row * CPR) * CN;
            const int r = KC ? r0 + row : r0 + col;
            const int k = KC ? k0 + col : k0 + row;
            uint4 v = make_uint4(0, 0, 0, 0);
            if ((CHUNKS % 256 == 0 || c < CHUNKS) && r < r_lim && k < k_lim) {
                const size_t off = KC ? (size_t)r * ld + k : (size_t)k * ld + r;
                v = *reinterpret_cast<const uint4*>(g + off);
            }
            reg[i] = v;
        }
    }
    // registers -> LDS
    __device__ static __forceinline__ void commit(const uint4 (&reg)[PER_THREAD], T* s) {
#pragma unroll
        for (int i = 0; i < PER_THREAD; ++i) {
            const int c = threadIdx.x + i * 256;
            const int row = c / CPR, col = (c - row * CPR) * CN;
            if (CHUNKS % 256 == 0 || c < CHUNKS) *reinterpret_cast<uint4*>(s + row * LD + col) = reg[i];
        }
    }
    // LDS -> MFMA operand: row r of the tile, reduction step ks
    __device__ static __forceinline__ typename Mma<T>::frag frag(const T* s, int r, int ks, int g) {
        constexpr int FE = Mma<T>::FE;
        const int k = ks * Mma<T>::KSTEP + FE * g;
        if constexpr (sizeof(T) == 2) {
            if constexpr (KC) {
                return __builtin_bit_cast(bf16x8_t, *reinterpret_cast<const uint4*>(s + r * LD + k));
            } else {
                uint32_t w[4];
#pragma unroll
                for (int i = 0; i < 4; ++i)
                    w[i] = (uint32_t)s[(k + 2 * i) * LD + r] | ((uint32_t)s[(k + 2 * i + 1) * LD + r] << 16);
                return __builtin_bit_cast(bf16x8_t, make_uint4(w[0], w[1], w[2], w[3]));
            }
        } else {
            return KC ? s[r * LD + k] : s[k * LD + r];
        }
    }
};

template <typename T, int EPI>
__device__ __forceinline__ void epilogue_store(const GemmArgs& p, size_t o, float v) {
    if constexpr (EPI == EPI_STORE) {
        st_f32<T>((T*)p.out0 + o, v);
    } else if constexpr (EPI == EPI_Z_H) {
        st_f32<T>((T*)p.out0 + o, v);
        st_f32<T>((T*)p.out1 + o, act_fwd(v, p.act));
    } else if constexpr (EPI == EPI_DZ) {
        const float z = ld_f32<T>((const T*)p.aux + o);
        st_f32<T>((T*)p.out0 + o, v * act_bwd(z, p.act));
    } else {
        ((float*)p.out0)[o] = v;
    }
}

template <typename T, int BM, int BN, int BK, bool A_KC, bool B_KC, int EPI>
__global__ __launch_bounds__(256) void grouped_gemm_kernel(const GemmArgs p) {
    typedef Tile<T, BM, BK, A_KC> TA;
    typedef Tile<T, BN, BK, B_KC> TB;
    constexpr int TM = BM / 64, TN = BN / 64;  // 32x32 MFMA tiles per wave (2x2 waves)
    constexpr int KS = BK / Mma<T>::KSTEP;
    extern __shared__ __align__(16) unsigned char smem_raw[];
    T* sA = reinterpret_cast<T*>(smem_raw);
    T* sB = sA + 2 * TA::ELEMS;

    // XCD-aware tile order: workgroup ids are dealt round-robin to the 8 XCDs, so
    // give each XCD one contiguous run of logical tiles (= whole experts).
    const int bid = blockIdx.x;
    const int logical = (bid & 7) * p.tiles_per_xcd + (bid >> 3);
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

    const T* gA = (const T*)p.A + (size_t)e * p.strideA;
    const T* gB = (const T*)p.B + (size_t)e * p.strideB;

    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int wm = wave >> 1, wn = wave & 1;
    const int l32 = lane & 31, g = lane >> 5;

    f32x16_t acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.0f;

    uint4 ra[TA::PER_THREAD], rb[TB::PER_THREAD];
    const int nk = (k_lim + BK - 1) / BK;
    if (nk > 0) {
        TA::fetch(ra, gA, p.lda, m0, 0, m_lim, k_lim);
        TB::fetch(rb, gB, p.ldb, n0, 0, p.N, k_lim);
        TA::commit(ra, sA);
        TB::commit(rb, sB);
    }
    __syncthreads();
    for (int kt = 0; kt < nk; ++kt) {
        const int cur = kt & 1;
        const bool more = kt + 1 < nk;
        if (more) {
            TA::fetch(ra, gA, p.lda, m0, (kt + 1) * BK, m_lim, k_lim);
            TB::fetch(rb, gB, p.ldb, n0, (kt + 1) * BK, p.N, k_lim);
        }
        const T* a_s = sA + cur * TA::ELEMS;
        const T* b_s = sB + cur * TB::ELEMS;
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
            typename Mma<T>::frag fa[TM], fb[TN];
#pragma unroll
            for (int i = 0; i < TM; ++i) fa[i] = TA::frag(a_s, wm * (BM / 2) + i * 32 + l32, ks, g);
#pragma unroll
            for (int j = 0; j < TN; ++j) fb[j] = TB::frag(b_s, wn * (BN / 2) + j * 32 + l32, ks, g);
#pragma unroll
            for (int i = 0; i < TM; ++i)
#pragma unroll
                for (int j = 0; j < TN; ++j) acc[i][j] = Mma<T>::mma(fa[i], fb[j], acc[i][j]);
        }
        if (more) {
            TA::commit(ra, sA + (cur ^ 1) * TA::ELEMS);
            TB::commit(rb, sB + (cur ^ 1) * TB::ELEMS);
        }
        __syncthreads();
    }

    // accumulator element v of lane l in a 32x32 tile: column l%32,
    // row 8*(v/4) + 4*(l/32) + v%4
    const size_t obase = (size_t)e * p.strideO;
#pragma unroll
    for (int i = 0; i < TM; ++i) {
#pragma unroll
        for (int j = 0; j < TN; ++j) {
            const int n = n0 + wn * (BN / 2) + j * 32 + l32;
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int m = m0 + wm * (BM / 2) + i * 32 + 8 * (v >> 2) + 4 * g + (v & 3);
                if (m < m_lim && n < p.N) epilogue_store<T, EPI>(p, obase + (size_t)m * p.ldo + n, acc[i][j][v]);
            }
        }
    }
}

template <typename T, int BM, int BN, int BK, bool A_KC, bool B_KC, int EPI>
static void launch_gemm(GemmArgs p, int E, hipStream_t st) {
    typedef Tile<T, BM, BK, A_KC> TA;
    typedef Tile<T, BN, BK, B_KC> TB;
    p.tiles_m = ceil_div(p.M, BM);
    p.tiles_n = ceil_div(p.N, BN);
    p.total_tiles = E * p.tiles_m * p.tiles_n;
    p.tiles_per_xcd = ceil_div(p.total_tiles, 8);
    const size_t smem = 2 * (size_t)(TA::ELEMS + TB::ELEMS) * sizeof(T);
    grouped_gemm_kernel<T, BM, BN, BK, A_KC, B_KC, EPI><<<p.tiles_per_xcd * 8, 256, smem, st>>>(p);
}

size_t ffn_bwd_ws_bytes(const moe_shape* s) {
    return align_up((size_t)s->E * s->capacity * s->d_ff * elem_bytes(s->dtype), 256);
}

template <typename T, int BM, int BN, int BK>
static void ffn_fwd(const moe_shape* s, const void* xd, const int32_t* cnt, const void* W1,
                    const void* W2, void* z, void* h, void* yd, hipStream_t st) {
    const int E = s->E, C = s->capacity, d = s->d_model, f = s->d_ff;
    GemmArgs p = {};
    p.expert_count = cnt; p.act = s->act; p.var_k = 0;
    // z = xd W1, h = act(z)
    p.A = xd; p.lda = d; p.strideA = (long long)C * d;
    p.B = W1; p.ldb = f; p.strideB = (long long)d * f;
    p.out0 = z; p.out1 = h; p.ldo = f; p.strideO = (long long)C * f;
    p.M = C; p.N = f; p.K = d;
    launch_gemm<T, BM, BN, BK, true, false, EPI_Z_H>(p, E, st);
    // yd = h W2
    p.A = h; p.lda = f; p.strideA = (long long)C * f;
    p.B = W2; p.ldb = d; p.strideB = (long long)f * d;
    p.out0 = yd; p.out1 = nullptr; p.ldo = d; p.strideO = (long long)C * d;
    p.M = C; p.N = d; p.K = f;
    launch_gemm<T, BM, BN, BK, true, false, EPI_STORE>(p, E, st);
}

template <typename T, int BM, int BN, int BK>
static void ffn_bwd(const moe_shape* s, const void* dyd, const void* xd, const void* z,
                    const void* h, const int32_t* cnt, const void* W1, const void* W2, void* dxd,
                    float* dW1, float* dW2, void* dz, hipStream_t st) {
    const int E = s->E, C = s->capacity, d = s->d_model, f = s->d_ff;
    GemmArgs p = {};
    p.expert_count = cnt; p.act = s->act;
    // dz = (dyd W2^T) .* act'(z):  B(r = n in f, k in d) = W2[n*d + k]
    p.var_k = 0;
    p.A = dyd; p.lda = d; p.strideA = (long long)C * d;
    p.B = W2; p.ldb = d; p.strideB = (long long)f * d;
    p.out0 = dz; p.aux = z; p.ldo = f; p.strideO = (long long)C * f;
    p.M = C; p.N = f; p.K = d;
    launch_gemm<T, BM, BN, BK, true, true, EPI_DZ>(p, E, st);
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
                                  void* z_saved, void* h_saved, void* yd, void* stream) {
    int rc = check_shape(shape);
    if (rc) return rc;
    if (!xd || !expert_count || !W1 || !W2 || !z_saved || !h_saved || !yd) return MOE_ERR_NULL;
    hipStream_t st = (hipStream_t)stream;
    if (shape->dtype == MOE_BF16)
        ffn_fwd<bf16_t, 128, 128, 32>(shape, xd, expert_count, W1, W2, z_saved, h_saved, yd, st);
    else
        ffn_fwd<float, 128, 128, 16>(shape, xd, expert_count, W1, W2, z_saved, h_saved, yd, st);
    return launch_status();
}

extern "C" int moe_expert_ffn_bwd(const moe_shape* shape, const void* dyd, const void* xd,
                                  const void* z_saved, const void* h_saved,
                                  const int32_t* expert_count, const void* W1, const void* W2,
                                  void* dxd, float* dW1, float* dW2, void* ws, size_t ws_bytes,
                                  void* stream) {
    int rc = check_shape(shape);
    if (rc) return rc;
    if (!dyd || !xd || !z_saved || !h_saved || !expert_count || !W1 || !W2 || !dxd || !dW1 || !dW2)
        return MOE_ERR_NULL;
    if (!ws || ((uintptr_t)ws & 255) || ws_bytes < ffn_bwd_ws_bytes(shape)) return MOE_ERR_WORKSPACE;
    hipStream_t st = (hipStream_t)stream;
    if (shape->dtype == MOE_BF16)
        ffn_bwd<bf16_t, 128, 128, 32>(shape, dyd, xd, z_saved, h_saved, expert_count, W1, W2, dxd, dW1, dW2, ws, st);
    else
        ffn_bwd<float, 128, 128, 16>(shape, dyd, xd, z_saved, h_saved, expert_count, W1, W2, dxd, dW1, dW2, ws, st);
    return launch_status();
}
