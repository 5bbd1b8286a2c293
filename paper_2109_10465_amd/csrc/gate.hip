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

template <typename T, int NB>
__global__ __launch_bounds__(64 * GLM_KSPLIT) void gate_logits_kernel(
    int Tn, int d, int E, const T* __restrict__ x, const float* __restrict__ Wg,
    const float* __restrict__ bias, float* __restrict__ logits) {
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
    for (int b0 = b_lo; b0 < b_hi; b0 += GRP) {
        float a[GRP][8];
#pragma unroll
        for (int u = 0; u < GRP; ++u) {
            const int k = (b0 + u) * 16 + 8 * h;
            const bool ok = b0 + u < b_hi && k < d;     // rows beyond T fall outside rs_x
            load8<T>(rs_x, ok ? (uint32_t)((r * d + k) * sizeof(T)) : BUF_OOB, a[u]);
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
            for (int u = 0; u < GRP; ++u)
#pragma unroll
                for (int s_ = 0; s_ < 8; ++s_)
                    acc[nb] = __builtin_amdgcn_mfma_f32_32x32x2f32(a[u][s_], bw[u][s_], acc[nb], 0, 0, 0);
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
                               float* logits, hipStream_t st) {
    const int grid = ceil_div(s->T, 32);
#define GLM(NB) gate_logits_kernel<T, NB><<<grid, 64 * GLM_KSPLIT, 0, st>>>(s->T, s->d_model, s->E, (const T*)x, Wg, bias, logits)
    if (s->E <= 32) GLM(1); else if (s->E <= 64) GLM(2); else if (s->E <= 128) GLM(4); else GLM(8);
#undef GLM
}

extern "C" int moe_gate_logits(const moe_shape* shape, const void* x, const float* Wg,
                               const float* bias_or_null, float* logits, void* stream) {
    int rc = check_shape(shape);
    if (rc) return rc;
    if (!x || !Wg || !logits) return MOE_ERR_NULL;
    if (shape->dtype == MOE_BF16) launch_gate_logits<bf16_t>(shape, x, Wg, bias_or_null, logits, (hipStream_t)stream);
    else launch_gate_logits<float>(shape, x, Wg, bias_or_null, logits, (hipStream_t)stream);
    return launch_status();
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
// dWg[d,E] = x^T dlogits : partial sums over token chunks, then an ordered sum
// ---------------------------------------------------------------------------
#define GW_DT 64   // d columns per workgroup
#define GW_TT 64   // tokens per LDS slab

static inline int gw_chunks(const moe_shape* s) {
    // enough workgroups to fill the chip, at least 256 tokens per chunk
    int want = ceil_div(1024, ceil_div(s->d_model, GW_DT));
    int maxc = ceil_div(s->T, 256);
    int n = want < maxc ? want : maxc;
    // one chunk's rows of x are addressed with 32-bit byte offsets: keep it below 1 GiB
    const int minc = (int)(((size_t)s->T * s->d_model * 4 + ((size_t)1 << 30) - 1) >> 30);
    if (n < minc) n = minc;
    return n < 1 ? 1 : n;
}
size_t gate_logits_bwd_ws_bytes(const moe_shape* s) {
    return align_up((size_t)gw_chunks(s) * s->d_model * s->E * 4, 256);
}

// Workgroup: 64 columns of d x one chunk of tokens; experts in passes of 32.
// Thread (ti,te) owns a 4-column x 2-expert register tile.
template <typename T>
__global__ __launch_bounds__(256) void gate_dwg_partial_kernel(
    int Tn, int d, int E, int tok_per_chunk, const T* __restrict__ x,
    const float* __restrict__ dlogits, float* __restrict__ partial) {
    __shared__ __align__(16) float xs[GW_TT][GW_DT];
    __shared__ __align__(16) float dls[GW_TT][32];
    const int tid = threadIdx.x, ti = tid & 15, te = tid >> 4;
    const int i0 = blockIdx.x * GW_DT;
    const int tbeg = blockIdx.y * tok_per_chunk;
    const int tend = min(Tn, tbeg + tok_per_chunk);
    constexpr int CN = Chunk<T>::N, CPR = GW_DT / CN;
    const int nrows = max(tend - tbeg, 0);
    const __amdgpu_buffer_rsrc_t rs_x = buf_rsrc(x + (size_t)tbeg * d, (size_t)nrows * d * sizeof(T));
    const __amdgpu_buffer_rsrc_t rs_d = buf_rsrc(dlogits + (size_t)tbeg * E, (size_t)nrows * E * 4);
    constexpr int XPT = GW_TT * CPR / 256 > 0 ? GW_TT * CPR / 256 : 1;
    constexpr int DPT = GW_TT * 32 / 256;
    for (int e0 = 0; e0 < E; e0 += 32) {
        float acc[4][2] = {{0.f, 0.f}, {0.f, 0.f}, {0.f, 0.f}, {0.f, 0.f}};
        float xr[XPT][CN], dr[DPT];
        auto fetch = [&](int ts) {   // branch free: out-of-range lanes read zeros
#pragma unroll
            for (int j = 0; j < XPT; ++j) {
                const int c = tid + j * 256, r = c / CPR, cc = c - r * CPR;
                const bool ok = c < GW_TT * CPR && i0 + cc * CN < d;   // rows beyond tend fall outside rs_x
                BufChunk<T>::load(rs_x, ok ? (uint32_t)(((ts - tbeg + r) * d + i0 + cc * CN) * sizeof(T)) : BUF_OOB, xr[j]);
            }
#pragma unroll
            for (int j = 0; j < DPT; ++j) {
                const int c = tid + j * 256, r = c >> 5, e = c & 31;
                const bool ok = e0 + e < E;
                dr[j] = buf_load_f32(rs_d, ok ? (uint32_t)(((ts - tbeg + r) * E + e0 + e) * 4) : BUF_OOB);
            }
        };
        fetch(tbeg);
        for (int ts = tbeg; ts < tend; ts += GW_TT) {
            __syncthreads();
#pragma unroll
            for (int j = 0; j < XPT; ++j) {
                const int c = tid + j * 256, r = c / CPR, cc = c - r * CPR;
                if (c < GW_TT * CPR) {
#pragma unroll
                    for (int q = 0; q < CN; ++q) xs[r][cc * CN + q] = xr[j][q];
                }
            }
#pragma unroll
            for (int j = 0; j < DPT; ++j) {
                const int c = tid + j * 256;
                dls[c >> 5][c & 31] = dr[j];
            }
            __syncthreads();
            if (ts + GW_TT < tend) fetch(ts + GW_TT);
            for (int tb = 0; tb < GW_TT; tb += 8) {   // 16 LDS reads in flight, then 64 FMAs
                float4 xv[8];
                float2 dv[8];
#pragma unroll
                for (int u = 0; u < 8; ++u) {
                    xv[u] = *reinterpret_cast<const float4*>(&xs[tb + u][ti * 4]);
                    dv[u] = *reinterpret_cast<const float2*>(&dls[tb + u][te * 2]);
                }
#pragma unroll
                for (int u = 0; u < 8; ++u) {
                    acc[0][0] = fmaf(xv[u].x, dv[u].x, acc[0][0]); acc[0][1] = fmaf(xv[u].x, dv[u].y, acc[0][1]);
                    acc[1][0] = fmaf(xv[u].y, dv[u].x, acc[1][0]); acc[1][1] = fmaf(xv[u].y, dv[u].y, acc[1][1]);
                    acc[2][0] = fmaf(xv[u].z, dv[u].x, acc[2][0]); acc[2][1] = fmaf(xv[u].z, dv[u].y, acc[2][1]);
                    acc[3][0] = fmaf(xv[u].w, dv[u].x, acc[3][0]); acc[3][1] = fmaf(xv[u].w, dv[u].y, acc[3][1]);
                }
            }
        }
#pragma unroll
        for (int a = 0; a < 4; ++a) {
            const int i = i0 + ti * 4 + a;
            if (i >= d) continue;
            float* out = partial + ((size_t)blockIdx.y * d + i) * E;
#pragma unroll
            for (int b = 0; b < 2; ++b)
                if (e0 + te * 2 + b < E) out[e0 + te * 2 + b] = acc[a][b];
        }
    }
}

__global__ __launch_bounds__(256) void gate_dwg_reduce_kernel(int n, int nchunk,
                                                              const float* __restrict__ partial,
                                                              float* __restrict__ dWg) {
    const int idx = blockIdx.x * 256 + threadIdx.x;
    if (idx >= n) return;
    float s = 0.0f;
    for (int c = 0; c < nchunk; ++c) s += partial[(size_t)c * n + idx];
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
                                                      T* __restrict__ dx) {
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
#pragma unroll
        for (int q = 0; q < NCH; ++q) {   // stores beyond T or d are dropped by the range check
#pragma unroll
            for (int j = 0; j < CN; ++j) cur[q][j] += acc[q * CN + j];
            BufChunk<T>::store(rs_dx, c0 + q * CN < d ? (uint32_t)((r * d + c0 + q * CN) * sizeof(T)) : BUF_OOB, cur[q]);
        }
    }
}

template <typename T>
static void launch_gate_logits_bwd(const moe_shape* s, const void* x, const float* Wg,
                                   const float* dlogits, float* dWg, void* dx, float* partial,
                                   hipStream_t st) {
    const int nch = gw_chunks(s);
    const int tpc = ceil_div(ceil_div(s->T, nch), GW_TT) * GW_TT;
    const int nch_used = ceil_div(s->T, tpc);
    dim3 grid(ceil_div(s->d_model, GW_DT), nch_used);
    gate_dwg_partial_kernel<T><<<grid, 256, 0, st>>>(s->T, s->d_model, s->E, tpc, (const T*)x, dlogits, partial);
    const int n = s->d_model * s->E;
    gate_dwg_reduce_kernel<<<ceil_div(n, 256), 256, 0, st>>>(n, nch_used, partial, dWg);
    if (dx) {
        const int grid_dx = ceil_div(s->T, 32);
#define GDX(EB, VEC) gate_dx_kernel<T, EB, VEC><<<grid_dx, 512, 0, st>>>(s->T, s->d_model, s->E, dlogits, Wg, (T*)dx)
#define GDXE(VEC) do { if (s->E <= 32) GDX(1, VEC); else if (s->E <= 64) GDX(2, VEC); \
                       else if (s->E <= 128) GDX(4, VEC); else GDX(8, VEC); } while (0)
        if (s->E % 4 == 0) GDXE(true); else GDXE(false);
#undef GDXE
#undef GDX
    }
}

extern "C" int moe_gate_logits_bwd(const moe_shape* shape, const void* x, const float* Wg,
                                   const float* dlogits, float* dWg, void* dx_accum, void* ws,
                                   size_t ws_bytes, void* stream) {
    int rc = check_shape(shape);
    if (rc) return rc;
    if (!x || !Wg || !dlogits || !dWg) return MOE_ERR_NULL;
    if (!ws || ((uintptr_t)ws & 255) || ws_bytes < gate_logits_bwd_ws_bytes(shape)) return MOE_ERR_WORKSPACE;
    if (shape->dtype == MOE_BF16)
        launch_gate_logits_bwd<bf16_t>(shape, x, Wg, dlogits, dWg, dx_accum, (float*)ws, (hipStream_t)stream);
    else
        launch_gate_logits_bwd<float>(shape, x, Wg, dlogits, dWg, dx_accum, (float*)ws, (hipStream_t)stream);
    return launch_status();
}
