// Gate projection and the gate's backward (Sec. 3.2: one gate matrix column per
// expert; Sec. 5.1: top-1 / top-2 gating).  All math in fp32; reductions run in
// a fixed order so results are bit-reproducible.
#include "moe_common.h"

// ---------------------------------------------------------------------------
// logits[T,E] = x[T,d] * Wg[d,E] (+ bias)
// Workgroup: 64 tokens x all experts; thread (ty,tx) owns 4 tokens x NE
// consecutive experts; x and Wg are staged through LDS in slabs of DK columns.
// ---------------------------------------------------------------------------
#define GL_TB 64
#define GL_DK 32

template <typename T, int NE>
__global__ __launch_bounds__(256) void gate_logits_kernel(
    int Tn, int d, int E, const T* __restrict__ x, const float* __restrict__ Wg,
    const float* __restrict__ bias, float* __restrict__ logits) {
    constexpr int EP = 16 * NE;
    __shared__ float xs[GL_TB][GL_DK + 1];
    __shared__ float ws[GL_DK][EP];
    const int tid = threadIdx.x, ty = tid >> 4, tx = tid & 15;
    const int t0 = blockIdx.x * GL_TB;
    float acc[4][NE];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int a = 0; a < NE; ++a) acc[i][a] = 0.0f;
    constexpr int CN = Chunk<T>::N;           // elements per 16-byte chunk
    constexpr int CPR = GL_DK / CN;           // chunks per token row of the slab
    for (int k0 = 0; k0 < d; k0 += GL_DK) {
        for (int c = tid; c < GL_TB * CPR; c += 256) {
            const int r = c / CPR, cc = c - r * CPR;
            float v[CN];
#pragma unroll
            for (int i = 0; i < CN; ++i) v[i] = 0.0f;
            if (t0 + r < Tn && k0 + cc * CN < d) Chunk<T>::load(x + (size_t)(t0 + r) * d + k0 + cc * CN, v);
#pragma unroll
            for (int i = 0; i < CN; ++i) xs[r][cc * CN + i] = v[i];
        }
        for (int c = tid; c < GL_DK * EP; c += 256) {
            const int r = c / EP, e = c - r * EP;
            ws[r][e] = (k0 + r < d && e < E) ? Wg[(size_t)(k0 + r) * E + e] : 0.0f;
        }
        __syncthreads();
#pragma unroll 4
        for (int kk = 0; kk < GL_DK; ++kk) {
            float w[NE];
#pragma unroll
            for (int a = 0; a < NE; ++a) w[a] = ws[kk][tx * NE + a];
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const float xv = xs[ty * 4 + i][kk];
#pragma unroll
                for (int a = 0; a < NE; ++a) acc[i][a] = fmaf(xv, w[a], acc[i][a]);
            }
        }
        __syncthreads();
    }
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int t = t0 + ty * 4 + i;
        if (t >= Tn) continue;
#pragma unroll
        for (int a = 0; a < NE; ++a) {
            const int e = tx * NE + a;
            if (e < E) logits[(size_t)t * E + e] = acc[i][a] + (bias ? bias[e] : 0.0f);
        }
    }
}

template <typename T>
static void launch_gate_logits(const moe_shape* s, const void* x, const float* Wg, const float* bias,
                               float* logits, hipStream_t st) {
    const int grid = ceil_div(s->T, GL_TB);
    const int ne = ceil_div(s->E, 16);
#define GL(NE) gate_logits_kernel<T, NE><<<grid, 256, 0, st>>>(s->T, s->d_model, s->E, (const T*)x, Wg, bias, logits)
    if (ne <= 1) GL(1); else if (ne <= 2) GL(2); else if (ne <= 4) GL(4); else if (ne <= 8) GL(8); else GL(16);
#undef GL
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
#define GW_TT 32   // tokens per LDS slab

static inline int gw_chunks(const moe_shape* s) {
    // enough workgroups to fill the chip, at least 256 tokens per chunk
    int want = ceil_div(1024, ceil_div(s->d_model, GW_DT));
    int maxc = ceil_div(s->T, 256);
    int n = want < maxc ? want : maxc;
    return n < 1 ? 1 : n;
}
size_t gate_logits_bwd_ws_bytes(const moe_shape* s) {
    return align_up((size_t)gw_chunks(s) * s->d_model * s->E * 4, 256);
}

template <typename T, int NE>  // thread owns experts eg*NE .. eg*NE+NE-1, eg = tid/64
__global__ __launch_bounds__(256) void gate_dwg_partial_kernel(
    int Tn, int d, int E, int tok_per_chunk, const T* __restrict__ x,
    const float* __restrict__ dlogits, float* __restrict__ partial) {
    constexpr int EP = 4 * NE;
    __shared__ float xs[GW_TT][GW_DT];
    __shared__ float dls[GW_TT][EP];
    const int tid = threadIdx.x, i = tid & 63, eg = tid >> 6;
    const int i0 = blockIdx.x * GW_DT;
    const int tbeg = blockIdx.y * tok_per_chunk;
    const int tend = min(Tn, tbeg + tok_per_chunk);
    float acc[NE];
#pragma unroll
    for (int a = 0; a < NE; ++a) acc[a] = 0.0f;
    constexpr int CN = Chunk<T>::N, CPR = GW_DT / CN;
    for (int ts = tbeg; ts < tend; ts += GW_TT) {
        for (int c = tid; c < GW_TT * CPR; c += 256) {
            const int r = c / CPR, cc = c - r * CPR;
            float v[CN];
#pragma unroll
            for (int q = 0; q < CN; ++q) v[q] = 0.0f;
            if (ts + r < tend && i0 + cc * CN < d) Chunk<T>::load(x + (size_t)(ts + r) * d + i0 + cc * CN, v);
#pragma unroll
            for (int q = 0; q < CN; ++q) xs[r][cc * CN + q] = v[q];
        }
        for (int c = tid; c < GW_TT * EP; c += 256) {
            const int r = c / EP, e = c - r * EP;
            dls[r][e] = (ts + r < tend && e < E) ? dlogits[(size_t)(ts + r) * E + e] : 0.0f;
        }
        __syncthreads();
#pragma unroll 4
        for (int tt = 0; tt < GW_TT; ++tt) {
            const float xv = xs[tt][i];
#pragma unroll
            for (int a = 0; a < NE; ++a) acc[a] = fmaf(xv, dls[tt][eg * NE + a], acc[a]);
        }
        __syncthreads();
    }
    if (i0 + i < d) {
        float* out = partial + ((size_t)blockIdx.y * d + i0 + i) * E;
#pragma unroll
        for (int a = 0; a < NE; ++a)
            if (eg * NE + a < E) out[eg * NE + a] = acc[a];
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
// dx[t,:] += dlogits[t,:] * Wg^T
// Workgroup: 32 tokens; loops over 64-column slabs of d; thread (i, tg) owns
// column i of the slab for 8 tokens.
// ---------------------------------------------------------------------------
#define GX_TB 32

template <typename T>
__global__ __launch_bounds__(256) void gate_dx_kernel(int Tn, int d, int E,
                                                      const float* __restrict__ dlogits,
                                                      const float* __restrict__ Wg,
                                                      T* __restrict__ dx) {
    extern __shared__ float smem[];
    float* dls = smem;                 // [GX_TB][E]
    float* wgs = smem + GX_TB * E;     // [64 columns][64 experts + 1]
    const int tid = threadIdx.x, i = tid & 63, tg = tid >> 6;
    const int t0 = blockIdx.x * GX_TB;
    for (int c = tid; c < GX_TB * E; c += 256) {
        const int r = c / E;
        dls[c] = t0 + r < Tn ? dlogits[(size_t)t0 * E + c] : 0.0f;
    }
    for (int i0 = 0; i0 < d; i0 += 64) {
        float acc[8];
#pragma unroll
        for (int a = 0; a < 8; ++a) acc[a] = 0.0f;
        for (int e0 = 0; e0 < E; e0 += 64) {
            const int ne = min(64, E - e0);
            __syncthreads();
            for (int c = tid; c < 64 * ne; c += 256) {
                const int r = c / ne, e = c - r * ne;
                wgs[r * 65 + e] = i0 + r < d ? Wg[(size_t)(i0 + r) * E + e0 + e] : 0.0f;
            }
            __syncthreads();
            for (int e = 0; e < ne; ++e) {
                const float w = wgs[i * 65 + e];
#pragma unroll
                for (int a = 0; a < 8; ++a) acc[a] = fmaf(dls[(tg * 8 + a) * E + e0 + e], w, acc[a]);
            }
        }
        if (i0 + i < d) {
#pragma unroll
            for (int a = 0; a < 8; ++a) {
                const int t = t0 + tg * 8 + a;
                if (t < Tn) {
                    T* p = dx + (size_t)t * d + i0 + i;
                    st_f32<T>(p, ld_f32<T>(p) + acc[a]);
                }
            }
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
    const int ne = ceil_div(s->E, 4);
#define GW(NE) gate_dwg_partial_kernel<T, NE><<<grid, 256, 0, st>>>(s->T, s->d_model, s->E, tpc, (const T*)x, dlogits, partial)
    if (ne <= 1) GW(1); else if (ne <= 2) GW(2); else if (ne <= 4) GW(4); else if (ne <= 8) GW(8);
    else if (ne <= 16) GW(16); else if (ne <= 32) GW(32); else GW(64);
#undef GW
    const int n = s->d_model * s->E;
    gate_dwg_reduce_kernel<<<ceil_div(n, 256), 256, 0, st>>>(n, nch_used, partial, dWg);
    if (dx) {
        const size_t smem = ((size_t)GX_TB * s->E + 64 * 65) * 4;
        gate_dx_kernel<T><<<ceil_div(s->T, GX_TB), 256, smem, st>>>(s->T, s->d_model, s->E, dlogits, Wg, (T*)dx);
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
