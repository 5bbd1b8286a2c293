// Gate projection and the gate's backward (Sec. 3.2: one gate matrix column per
// expert; Sec. 5.1: top-1 / top-2 gating).  All math in fp32; reductions run in
// a fixed order so results are bit-reproducible.
#include "moe_common.h"

// ---------------------------------------------------------------------------
// logits[T,E] = x[T,d] * Wg[d,E] (+ bias)   on the fp32 matrix pipe
// Workgroup: 32 tokens x all experts, 8 waves that split the reduction over d.
// v_mfma_f32_32x32x2_f32: lane (r = l%32, h = l/32) supplies A[token r][k] and
// B[k][expert r] for ONE k per instruction.  The order of a reduction is free,
// so a lane's 8 consecutive x values (one 16-byte load for bf16) serve 8
// instructions: in a 16-deep block, instruction s uses k = 8h + s.  Wg (L2
// resident) is read as 128-byte rows.  All loads of a group of blocks are in
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

template <typename T, int NB, bool JIT>   // JIT: gate jitter on (a separate instance keeps the plain one lean)
__global__ __launch_bounds__(64 * GLM_KSPLIT, NB == 1 ? 4 : 2) void gate_logits_kernel(
    int Tn, int d, int E, const T* __restrict__ x, const float* __restrict__ Wg,
    const float* __restrict__ bias, float* __restrict__ logits, float jitter_eps, uint64_t seed) {
    constexpr int GRP = NB <= 2 ? 8 : 4;   // 16-deep blocks whose loads are in flight together
    __shared__ float red[GLM_KSPLIT][32][33];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int r = lane & 31, h = lane >> 5;
    const int t0 = blockIdx.x * 32;
    const int rows_here = min(32, Tn - t0);
    const __amdgpu_buffer_rsrc_t rs_x = buf_rsrc(x + (size_t)t0 * d, (size_t)rows_here * d * sizeof(T));
    const __amdgpu_buffer_rsrc_t rs_w = buf_rsrc(Wg, (size_t)d * E * 4);
    const int nblk = (d + 15) / 16;
    const int per_wave = (nblk + GLM_KSPLIT - 1) / GLM_KSPLIT;
    const int b_lo = wave * per_wave, b_hi = min(nblk, b_lo + per_wave);
    glm_f32x16 acc[NB];
#pragma unroll
    for (int nb = 0; nb < NB; ++nb)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[nb][v] = 0.0f;
    // bf16 activations (no jitter): x goes to the bf16 matrix pipe as loaded and Wg as
    // three bf16 parts that add up to it exactly, so the fp32 result is kept at a
    // fraction of the fp32 pipe's time (one 32x32x16 step per part instead of eight 32x32x2)
    constexpr bool SPLIT = sizeof(T) == 2 && !JIT;
    for (int b0 = b_lo; b0 < b_hi; b0 += GRP) {
        float a[SPLIT ? 1 : GRP][8];
        u32x4_buf_t araw[SPLIT ? GRP : 1];
#pragma unroll
        for (int u = 0; u < GRP; ++u) {
            const int k = (b0 + u) * 16 + 8 * h;
            const bool ok = b0 + u < b_hi && k < d;     // rows beyond T fall outside rs_x
            const uint32_t off = ok ? (uint32_t)((r * d + k) * sizeof(T)) : BUF_OOB;
            if constexpr (SPLIT) araw[u] = __builtin_amdgcn_raw_buffer_load_b128(rs_x, off, 0, 0);
            else load8<T>(rs_x, off, a[u]);
        }
        if constexpr (JIT) {   // the gate sees x * noise
#pragma unroll
            for (int u = 0; u < GRP; ++u)
                jitter_scale<8>(a[u], (size_t)(t0 + r) * d + (b0 + u) * 16 + 8 * h, jitter_eps, seed);
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
                    const bf16x8_hw_t xa = __builtin_bit_cast(bf16x8_hw_t, araw[u]);
                    acc[nb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(xa, w_lo, acc[nb], 0, 0, 0);
                    acc[nb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(xa, w_mid, acc[nb], 0, 0, 0);
                    acc[nb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(xa, w_hi, acc[nb], 0, 0, 0);
                } else {
#pragma unroll
                    for (int s_ = 0; s_ < 8; ++s_)
                        acc[nb] = __builtin_amdgcn_mfma_f32_32x32x2f32(a[u][s_], bw[u][s_], acc[nb], 0, 0, 0);
                }
            }
        }
    }
    // accumulator element v of lane l: expert column l%32, token row 8*(v/4) + 4*(l/32) + v%4
#pragma unroll
    for (int nb = 0; nb < NB; ++nb) {
        if (nb) __syncthreads();
#pragma unroll
        for (int v = 0; v < 16; ++v) red[wave][8 * (v >> 2) + 4 * h + (v & 3)][r] = acc[nb][v];
        __syncthreads();
#pragma unroll
        for (int o = threadIdx.x; o < 32 * 32; o += 64 * GLM_KSPLIT) {
            const int m = o >> 5, n = o & 31, e = nb * 32 + n;
            float sum = 0.0f;
#pragma unroll
            for (int w = 0; w < GLM_KSPLIT; ++w) sum += red[w][m][n];
            if (m < rows_here && e < E) logits[(size_t)(t0 + m) * E + e] = sum + (bias ? bias[e] : 0.0f);
        }
    }
}

template <typename T>
static void launch_gate_logits(const moe_shape* s, const void* x, const float* Wg, const float* bias,
                               float* logits, float eps, uint64_t seed, hipStream_t st) {
    const int grid = ceil_div(s->T, 32);
#define GLM(NB, JIT) gate_logits_kernel<T, NB, JIT><<<grid, 64 * GLM_KSPLIT, 0, st>>>(s->T, s->d_model, s->E, (const T*)x, Wg, bias, logits, eps, seed)
#define GLME(JIT) do { if (s->E <= 32) GLM(1, JIT); else if (s->E <= 64) GLM(2, JIT); \
                       else if (s->E <= 128) GLM(4, JIT); else GLM(8, JIT); } while (0)
    if (eps != 0.0f) GLME(true); else GLME(false);
#undef GLME
#undef GLM
}

static int gate_logits_impl(const moe_shape* shape, const void* x, const float* Wg,
                            const float* bias_or_null, float eps, uint64_t seed, float* logits, void* stream) {
    int rc = check_shape(shape);
    if (rc) return rc;
    if (!x || !Wg || !logits) return MOE_ERR_NULL;
    if (!(eps >= 0.0f && eps < 1.0f)) return MOE_ERR_SHAPE;
    if (shape->dtype == MOE_BF16) launch_gate_logits<bf16_t>(shape, x, Wg, bias_or_null, logits, eps, seed, (hipStream_t)stream);
    else launch_gate_logits<float>(shape, x, Wg, bias_or_null, logits, eps, seed, (hipStream_t)stream);
    return launch_status();
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
__global__ __launch_bounds__(256) void gate_bwd_kernel(
    int Tn, int E, int k, const float* __restrict__ dgate_w, const float* __restrict__ probs,
    const int32_t* __restrict__ expert_idx, const int32_t* __restrict__ slot,
    float* __restrict__ dlogits) {
    const size_t idx = (size_t)blockIdx.x * 256 + threadIdx.x;
    if (idx >= (size_t)Tn * E) return;
    const int t = (int)(idx / E), e = (int)(idx - (size_t)t * E);
    const float* pr = probs + (size_t)t * E;
    float dp_e = 0.0f, sum = 0.0f;
    if (k == 1) {
        const int e0 = expert_idx[t];
        const float dg0 = slot[t] >= 0 ? dgate_w[t] : 0.0f;
        sum = pr[e0] * dg0;
        if (e == e0) dp_e = dg0;
    } else {
        const int e0 = expert_idx[2 * t], e1 = expert_idx[2 * t + 1];
        const float dg0 = slot[2 * t] >= 0 ? dgate_w[2 * t] : 0.0f;
        const float dg1 = slot[2 * t + 1] >= 0 ? dgate_w[2 * t + 1] : 0.0f;
        const float p0 = pr[e0], p1 = pr[e1];
        const float S = p0 + p1;
        const float dp0 = p1 * (dg0 - dg1) / (S * S);
        const float dp1 = p0 * (dg1 - dg0) / (S * S);
        sum = p0 * dp0 + p1 * dp1;
        if (e == e0) dp_e = dp0;
        if (e == e1) dp_e = dp1;
    }
    dlogits[idx] = pr[e] * (dp_e - sum);
}

extern "C" int moe_gate_bwd(const moe_shape* shape, const float* dgate_w, const float* probs,
                            const int32_t* expert_idx, const int32_t* slot, float* dlogits,
                            void* stream) {
    int rc = check_shape(shape);
    if (rc) return rc;
    if (!dgate_w || !probs || !expert_idx || !slot || !dlogits) return MOE_ERR_NULL;
    const size_t n = (size_t)shape->T * shape->E;
    gate_bwd_kernel<<<(unsigned)((n + 255) / 256), 256, 0, (hipStream_t)stream>>>(
        shape->T, shape->E, shape->k, dgate_w, probs, expert_idx, slot, dlogits);
    return launch_status();
}

// ---------------------------------------------------------------------------
// dWg[d,E] = x^T dlogits   on the fp32 matrix pipe: partial sums over token
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

template <typename T, bool JIT>
__global__ __launch_bounds__(64 * GW_WAVES) void gate_dwg_partial_kernel(
    int Tn, int d, int E, int tok_per_chunk, const T* __restrict__ x,
    const float* __restrict__ dlogits, float* __restrict__ partial, float jitter_eps, uint64_t seed) {
    extern __shared__ __align__(16) float gw_red[];      // [wave][256 columns][32 experts]
    constexpr int GRP = 4;                               // token pairs whose loads are in flight together (x2 buffers)
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int r = lane & 31, h = lane >> 5;
    const int i0 = blockIdx.x * GW_COLS, e0 = blockIdx.z * 32;
    const int tbeg = blockIdx.y * tok_per_chunk;
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
    // accumulator v of tile c, lane l: column i0 + 8*(8*(v/4) + 4*(l/32) + v%4) + c, expert e0 + l%32
#pragma unroll
    for (int c = 0; c < 8; ++c)
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            const int m = 8 * (v >> 2) + 4 * h + (v & 3);
            gw_red[(wave * GW_COLS + 8 * m + c) * 32 + r] = acc[c][v];
        }
    __syncthreads();
    for (int o = threadIdx.x; o < GW_COLS * 32; o += 64 * GW_WAVES) {
        const int il = o >> 5, e = o & 31;
        float sum = 0.0f;
#pragma unroll
        for (int w = 0; w < GW_WAVES; ++w) sum += gw_red[(w * GW_COLS + il) * 32 + e];
        if (i0 + il < d && e0 + e < E) partial[((size_t)blockIdx.y * d + i0 + il) * E + e0 + e] = sum;
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
// dx[t,:] += dlogits[t,:] * Wg^T   on the fp32 matrix pipe
// Workgroup: 32 tokens, 8 waves; wave w takes the 32-column blocks w, w+8, ...
// of d.  The product is formed transposed, D[column][token], so that a lane's
// accumulators (4 consecutive rows of D at 4 places) are 4 consecutive columns of
// ONE token row (16 consecutive ones after a permutation of the tile's rows): dx
// is updated in place with 16-byte accesses and no LDS.
// A = Wg rows (column i, all experts), B = dlogits rows (token, all experts):
// both are contiguous along the reduction, so a lane half reads its 16 experts
// of a 32-expert block as 64 contiguous bytes (instruction s uses expert 16h+s).
// ---------------------------------------------------------------------------
template <bool VEC>
__device__ __forceinline__ void load16(__amdgpu_buffer_rsrc_t rs, int row_elems, int e0, int E, float (&v)[16]) {
    // 16 consecutive fp32 of one row starting at element e0 of the row (row_elems = row * E)
    if constexpr (VEC) {
#pragma unroll
        for (int c = 0; c < 4; ++c) {
            float q[4];
            BufChunk<float>::load(rs, e0 + 4 * c < E ? (uint32_t)((row_elems + e0 + 4 * c) * 4) : BUF_OOB, q);
#pragma unroll
            for (int j = 0; j < 4; ++j) v[4 * c + j] = q[j];
        }
    } else {
#pragma unroll
        for (int j = 0; j < 16; ++j)
            v[j] = buf_load_f32(rs, e0 + j < E ? (uint32_t)((row_elems + e0 + j) * 4) : BUF_OOB);
    }
}

template <typename T, int EB, bool VEC>   // EB = 32-expert blocks (E <= 32*EB); VEC: E % 4 == 0
__global__ __launch_bounds__(512) void gate_dx_kernel(int Tn, int d, int E,
                                                      const float* __restrict__ dlogits,
                                                      const float* __restrict__ Wg,
                                                      T* __restrict__ dx, float jitter_eps, uint64_t seed) {
    constexpr bool HOIST = EB <= 2;      // dlogits fragments stay in registers across column blocks
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int r = lane & 31, h = lane >> 5;
    const int t0 = blockIdx.x * 32;
    const int rows_here = min(32, Tn - t0);
    const __amdgpu_buffer_rsrc_t rs_dl = buf_rsrc(dlogits + (size_t)t0 * E, (size_t)rows_here * E * 4);
    const __amdgpu_buffer_rsrc_t rs_w = buf_rsrc(Wg, (size_t)d * E * 4);
    const __amdgpu_buffer_rsrc_t rs_dx = buf_rsrc(dx + (size_t)t0 * d, (size_t)rows_here * d * sizeof(T));
    float bfr[HOIST ? EB : 1][16];
    if constexpr (HOIST) {
#pragma unroll
        for (int eb = 0; eb < EB; ++eb) load16<VEC>(rs_dl, r * E, eb * 32 + 16 * h, E, bfr[eb]);   // rows beyond T read zeros
    }
    const int ncb = (d + 31) / 32;
    // Row m of the product tile stands for column i0 + pi(m) of the block, with
    // pi(8q + 4h' + j) = 16h' + 4q + j: a lane's accumulator v (row 8(v/4) + 4h + v%4)
    // is then column i0 + 16h + v, i.e. 16 CONSECUTIVE columns of its token row.
    const int a_col = 16 * ((r >> 2) & 1) + 4 * (r >> 3) + (r & 3);   // pi(r): the Wg row this lane supplies
    constexpr int CN = BufChunk<T>::N, NCH = 16 / CN;                 // 16-byte pieces of the lane's 16 columns
    for (int cb = wave; cb < ncb; cb += 8) {
        const int i0 = cb * 32;
        const int c0 = i0 + 16 * h;
        float cur[NCH][CN];
#pragma unroll
        for (int q = 0; q < NCH; ++q)   // d % 8 == 0: a piece is inside the row or wholly beyond it
            BufChunk<T>::load(rs_dx, c0 + q * CN < d ? (uint32_t)((r * d + c0 + q * CN) * sizeof(T)) : BUF_OOB, cur[q]);
        glm_f32x16 acc;
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[v] = 0.0f;
#pragma unroll
        for (int eb = 0; eb < EB; ++eb) {
            float afr[16];
            load16<VEC>(rs_w, (i0 + a_col) * E, eb * 32 + 16 * h, E, afr);   // rows beyond d fall outside rs_w
            if constexpr (!HOIST) load16<VEC>(rs_dl, r * E, eb * 32 + 16 * h, E, bfr[0]);
#pragma unroll
            for (int s_ = 0; s_ < 16; ++s_)
                acc = __builtin_amdgcn_mfma_f32_32x32x2f32(afr[s_], bfr[HOIST ? eb : 0][s_], acc, 0, 0, 0);
        }
        float inc[16];
#pragma unroll
        for (int v = 0; v < 16; ++v) inc[v] = acc[v];
        if (jitter_eps != 0.0f)     // the gate saw x * noise: d/dx carries the factor (uniform branch)
            jitter_scale<16>(inc, (size_t)(t0 + r) * d + c0, jitter_eps, seed);
#pragma unroll
        for (int q = 0; q < NCH; ++q) {   // stores beyond T or d are dropped by the range check
#pragma unroll
            for (int j = 0; j < CN; ++j) cur[q][j] += inc[q * CN + j];
            BufChunk<T>::store(rs_dx, c0 + q * CN < d ? (uint32_t)((r * d + c0 + q * CN) * sizeof(T)) : BUF_OOB, cur[q]);
        }
    }
}

template <typename T>
static void launch_gate_logits_bwd(const moe_shape* s, const void* x, const float* Wg,
                                   const float* dlogits, float* dWg, void* dx, float* partial,
                                   float eps, uint64_t seed, hipStream_t st) {
    const int tpc = gw_chunk_tokens(s);
    const int nch_used = ceil_div(s->T, tpc);
    dim3 grid(ceil_div(s->d_model, GW_COLS), nch_used, ceil_div(s->E, 32));
    constexpr size_t red_bytes = (size_t)GW_WAVES * GW_COLS * 32 * sizeof(float);   // 128 KB: opt in beyond 64 KB
    static const hipError_t attr0 = hipFuncSetAttribute(
        (const void*)gate_dwg_partial_kernel<T, false>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)red_bytes);
    static const hipError_t attr1 = hipFuncSetAttribute(
        (const void*)gate_dwg_partial_kernel<T, true>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)red_bytes);
    (void)attr0; (void)attr1;
    if (eps != 0.0f)
        gate_dwg_partial_kernel<T, true><<<grid, 64 * GW_WAVES, red_bytes, st>>>(s->T, s->d_model, s->E, tpc,
                                                                              (const T*)x, dlogits, partial, eps, seed);
    else
        gate_dwg_partial_kernel<T, false><<<grid, 64 * GW_WAVES, red_bytes, st>>>(s->T, s->d_model, s->E, tpc,
                                                                               (const T*)x, dlogits, partial, eps, seed);
    const int n = s->d_model * s->E;
    gate_dwg_reduce_kernel<<<ceil_div(n, 256), 256, 0, st>>>(n, nch_used, partial, dWg);
    if (dx) {
        const int grid_dx = ceil_div(s->T, 32);
#define GDX(EB, VEC) gate_dx_kernel<T, EB, VEC><<<grid_dx, 512, 0, st>>>(s->T, s->d_model, s->E, dlogits, Wg, (T*)dx, eps, seed)
#define GDXE(VEC) do { if (s->E <= 32) GDX(1, VEC); else if (s->E <= 64) GDX(2, VEC); \
                       else if (s->E <= 128) GDX(4, VEC); else GDX(8, VEC); } while (0)
        if (s->E % 4 == 0) GDXE(true); else GDXE(false);
#undef GDXE
#undef GDX
    }
}

static int gate_logits_bwd_impl(const moe_shape* shape, const void* x, const float* Wg, const float* dlogits,
                                float eps, uint64_t seed, float* dWg, void* dx_accum, void* ws,
                                size_t ws_bytes, void* stream) {
    int rc = check_shape(shape);
    if (rc) return rc;
    if (!x || !Wg || !dlogits || !dWg) return MOE_ERR_NULL;
    if (!(eps >= 0.0f && eps < 1.0f)) return MOE_ERR_SHAPE;
    if (!ws || ((uintptr_t)ws & 255) || ws_bytes < gate_logits_bwd_ws_bytes(shape)) return MOE_ERR_WORKSPACE;
    if (shape->dtype == MOE_BF16)
        launch_gate_logits_bwd<bf16_t>(shape, x, Wg, dlogits, dWg, dx_accum, (float*)ws, eps, seed, (hipStream_t)stream);
    else
        launch_gate_logits_bwd<float>(shape, x, Wg, dlogits, dWg, dx_accum, (float*)ws, eps, seed, (hipStream_t)stream);
    return launch_status();
}

extern "C" int moe_gate_logits_bwd(const moe_shape* shape, const void* x, const float* Wg,
                                   const float* dlogits, float* dWg, void* dx_accum, void* ws,
                                   size_t ws_bytes, void* stream) {
    return gate_logits_bwd_impl(shape, x, Wg, dlogits, 0.0f, 0, dWg, dx_accum, ws, ws_bytes, stream);
}

extern "C" int moe_gate_logits_bwd_jitter(const moe_shape* shape, const void* x, const float* Wg,
                                          const float* dlogits, float jitter_eps, uint64_t seed,
                                          float* dWg, void* dx_accum, void* ws, size_t ws_bytes,
                                          void* stream) {
    return gate_logits_bwd_impl(shape, x, Wg, dlogits, jitter_eps, seed, dWg, dx_accum, ws, ws_bytes, stream);
}
