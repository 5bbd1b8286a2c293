// Balancing auxiliary loss of the gate and the gate backward that carries its
// gradient (Sec. 5.1, "MoE setting": a balancing loss, times 0.01, is added to
// the training loss; Switch / GShard form):
//     f[e] = (tokens whose first choice is e) / T,   P[e] = mean_t p[t,e],
//     L = E * sum_e f[e] * P[e].
// All sums run in a fixed order (per-thread strided rows, then row groups, then
// chunks of tokens), so the loss and its gradient are bit-reproducible.
#include "moe_common.h"

// Tokens per workgroup of the partial-sum kernel: 64 for small batches (enough
// workgroups to spread over the chip), more for large ones so that there are
// never more than 1024 chunks.
static inline int aux_chunk_tokens(const moe_shape* s) {
    const int c = ceil_div(ceil_div(s->T, 1024), 64) * 64;
    return c < 64 ? 64 : c;
}
static inline int aux_chunks(const moe_shape* s) { return ceil_div(s->T, aux_chunk_tokens(s)); }
size_t aux_loss_ws_bytes(const moe_shape* s) {
    return align_up((size_t)aux_chunks(s) * s->E * 8, 256);   // float sums + int32 counts per chunk
}

static inline int pow2_at_least(int v) {
    int p = 1;
    while (p < v) p <<= 1;
    return p;
}

// Workgroup: one chunk of tokens.  Thread (g, e) with e = tid % EP sums column e
// over rows g, g+RS, g+2RS, ... of the chunk (EP = E rounded up to a power of
// two, RS = 256 / EP row groups), 8 independent loads at a time; the row groups
// are then added in order.  First choices are counted with integer LDS atomics.
__global__ __launch_bounds__(256) void aux_partial_kernel(
    int T, int E, int k, int EP, int chunk, const float* __restrict__ probs,
    const int32_t* __restrict__ expert_idx, float* __restrict__ part_sum, int32_t* __restrict__ part_cnt) {
    __shared__ float s_sum[256];
    __shared__ int32_t s_cnt[256];
    const int tid = threadIdx.x;
    const int e = tid & (EP - 1), g = tid / EP, RS = 256 / EP;
    const int t0 = blockIdx.x * chunk;
    const int rows = min(chunk, T - t0);
    s_cnt[tid] = 0;
    float acc = 0.0f;
    if (e < E) {
        for (int r0 = g; r0 < rows; r0 += 8 * RS) {
            float v[8];
#pragma unroll
            for (int u = 0; u < 8; ++u) {
                const int r = r0 + u * RS;
                v[u] = r < rows ? probs[(size_t)(t0 + r) * E + e] : 0.0f;
            }
#pragma unroll
            for (int u = 0; u < 8; ++u) acc += v[u];
        }
    }
    s_sum[tid] = acc;
    __syncthreads();
    for (int r = tid; r < rows; r += 256) {
        const int e0 = expert_idx[(size_t)(t0 + r) * k];
        if ((unsigned)e0 < (unsigned)E) atomicAdd(&s_cnt[e0], 1);   // ids outside [0,E) are not counted
    }
    __syncthreads();
    if (tid < E) {
        float s = 0.0f;
        for (int q = 0; q < RS; ++q) s += s_sum[q * EP + tid];
        part_sum[(size_t)blockIdx.x * E + tid] = s;
        part_cnt[(size_t)blockIdx.x * E + tid] = s_cnt[tid];
    }
}

// One workgroup: thread (g, e) adds the partials of chunks g, g+RS, ... of expert
// e (8 independent loads at a time); the groups are then added in order.
__global__ __launch_bounds__(256) void aux_final_kernel(
    int T, int E, int EP, int nchunk, const float* __restrict__ part_sum,
    const int32_t* __restrict__ part_cnt, float* __restrict__ first_frac, float* __restrict__ mean_prob,
    float* __restrict__ loss) {
    __shared__ float s_sum[256];
    __shared__ int32_t s_cnt[256];
    __shared__ float s_prod[256];
    const int tid = threadIdx.x;
    const int e = tid & (EP - 1), g = tid / EP, RS = 256 / EP;
    float acc = 0.0f;
    int cnt = 0;
    if (e < E) {
        for (int q0 = g; q0 < nchunk; q0 += 8 * RS) {
            float v[8];
            int c[8];
#pragma unroll
            for (int u = 0; u < 8; ++u) {
                const int q = q0 + u * RS;
                v[u] = q < nchunk ? part_sum[(size_t)q * E + e] : 0.0f;
                c[u] = q < nchunk ? part_cnt[(size_t)q * E + e] : 0;
            }
#pragma unroll
            for (int u = 0; u < 8; ++u) { acc += v[u]; cnt += c[u]; }
        }
    }
    s_sum[tid] = acc;
    s_cnt[tid] = cnt;
    __syncthreads();
    float prod = 0.0f;
    if (tid < E) {
        float s = 0.0f;
        int c = 0;
        for (int q = 0; q < RS; ++q) { s += s_sum[q * EP + tid]; c += s_cnt[q * EP + tid]; }
        const float f = (float)c / (float)T, P = s / (float)T;
        first_frac[tid] = f;
        mean_prob[tid] = P;
        prod = f * P;
    }
    s_prod[tid] = prod;
    __syncthreads();
    if (tid == 0) {
        float L = 0.0f;
        for (int q = 0; q < E; ++q) L += s_prod[q];
        loss[0] = (float)E * L;
    }
}

extern "C" int moe_aux_loss(const moe_shape* shape, const float* probs, const int32_t* expert_idx,
                            float* first_frac, float* mean_prob, float* loss, void* ws,
                            size_t ws_bytes, void* stream) {
    int rc = check_shape(shape);
    if (rc) return rc;
    if (!probs || !expert_idx || !first_frac || !mean_prob || !loss) return MOE_ERR_NULL;
    if (!ws || ((uintptr_t)ws & 255) || ws_bytes < aux_loss_ws_bytes(shape)) return MOE_ERR_WORKSPACE;
    hipStream_t st = (hipStream_t)stream;
    const int nchunk = aux_chunks(shape);
    float* part_sum = (float*)ws;
    int32_t* part_cnt = (int32_t*)(part_sum + (size_t)nchunk * shape->E);
    const int EP = pow2_at_least(shape->E);
    aux_partial_kernel<<<nchunk, 256, 0, st>>>(shape->T, shape->E, shape->k, EP, aux_chunk_tokens(shape), probs,
                                               expert_idx, part_sum, part_cnt);
    aux_final_kernel<<<1, 256, 0, st>>>(shape->T, shape->E, EP, nchunk, part_sum, part_cnt, first_frac,
                                        mean_prob, loss);
    return launch_status();
}

// ---------------------------------------------------------------------------
// Gate backward with the balancing term:  dp[t,e] = (gate-weight term) + c f[e],
// c = aux_coef * E / T, for every token, then the softmax backward.
// LPT lanes share one token, 4 consecutive experts per lane (4*LPT >= E); the
// row sum sum_e p[t,e] f[e] is a butterfly over those lanes (same order for
// every token, so results do not depend on the launch).
// ---------------------------------------------------------------------------
template <int LPT>
__global__ __launch_bounds__(256) void gate_bwd_aux_kernel(
    int T, int E, int k, float c, const float* __restrict__ dgate_w, const float* __restrict__ probs,
    const int32_t* __restrict__ expert_idx, const int32_t* __restrict__ slot,
    const float* __restrict__ first_frac, float* __restrict__ dlogits) {
    const int gl = threadIdx.x % LPT;
    const int t = blockIdx.x * (256 / LPT) + threadIdx.x / LPT;
    const bool valid = t < T;       // uniform within a token's lane group
    const int e4 = gl * 4;
    const bool vec = (E & 3) == 0;
    float p[4] = {0.f, 0.f, 0.f, 0.f}, f[4] = {0.f, 0.f, 0.f, 0.f};
    if (valid) {
        const float* row = probs + (size_t)t * E;
        if (vec) {
            if (e4 < E) {
                const float4 q = *reinterpret_cast<const float4*>(row + e4);
                p[0] = q.x; p[1] = q.y; p[2] = q.z; p[3] = q.w;
                const float4 r = *reinterpret_cast<const float4*>(first_frac + e4);
                f[0] = r.x; f[1] = r.y; f[2] = r.z; f[3] = r.w;
            }
        } else {
#pragma unroll
            for (int i = 0; i < 4; ++i)
                if (e4 + i < E) { p[i] = row[e4 + i]; f[i] = first_frac[e4 + i]; }
        }
    }
    // the gate-weight term touches the one or two chosen experts only
    int e0 = -1, e1 = -1;
    float dp0 = 0.0f, dp1 = 0.0f, sum = 0.0f;
    if (valid) {
        const float* pr = probs + (size_t)t * E;
        if (k == 1) {
            e0 = expert_idx[t];
            dp0 = slot[t] >= 0 ? dgate_w[t] : 0.0f;
            sum = pr[e0] * dp0;
        } else {
            e0 = expert_idx[2 * t]; e1 = expert_idx[2 * t + 1];
            const float dg0 = slot[2 * t] >= 0 ? dgate_w[2 * t] : 0.0f;
            const float dg1 = slot[2 * t + 1] >= 0 ? dgate_w[2 * t + 1] : 0.0f;
            const float p0 = pr[e0], p1 = pr[e1];
            const float S = p0 + p1;
            dp0 = p1 * (dg0 - dg1) / (S * S);
            dp1 = p0 * (dg1 - dg0) / (S * S);
            sum = p0 * dp0 + p1 * dp1;
        }
    }
    float part = 0.0f;
#pragma unroll
    for (int i = 0; i < 4; ++i) part = fmaf(p[i], f[i], part);
#pragma unroll
    for (int o = LPT / 2; o > 0; o >>= 1) part += __shfl_xor(part, o, MOE_WAVE);
    const float total = sum + c * part;       // sum_e' p[t,e'] dp[t,e']
    if (!valid) return;
    float out[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int e = e4 + i;
        float dp = c * f[i];
        if (e == e0) dp += dp0;
        if (e == e1) dp += dp1;
        out[i] = p[i] * (dp - total);
    }
    float* dl = dlogits + (size_t)t * E;
    if (vec) {
        if (e4 < E) *reinterpret_cast<float4*>(dl + e4) = make_float4(out[0], out[1], out[2], out[3]);
    } else {
#pragma unroll
        for (int i = 0; i < 4; ++i)
            if (e4 + i < E) dl[e4 + i] = out[i];
    }
}

extern "C" int moe_gate_bwd_aux(const moe_shape* shape, const float* dgate_w, const float* probs,
                                const int32_t* expert_idx, const int32_t* slot,
                                const float* first_frac, float aux_coef, float* dlogits, void* stream) {
    int rc = check_shape(shape);
    if (rc) return rc;
    if (!dgate_w || !probs || !expert_idx || !slot || !first_frac || !dlogits) return MOE_ERR_NULL;
    hipStream_t st = (hipStream_t)stream;
    const int T = shape->T, E = shape->E, k = shape->k;
    const float c = aux_coef * (float)E / (float)T;
#define GBA(LPT) gate_bwd_aux_kernel<LPT><<<ceil_div(T, 256 / LPT), 256, 0, st>>>( \
        T, E, k, c, dgate_w, probs, expert_idx, slot, first_frac, dlogits)
    if (E <= 4) GBA(1); else if (E <= 8) GBA(2); else if (E <= 16) GBA(4); else if (E <= 32) GBA(8);
    else if (E <= 64) GBA(16); else if (E <= 128) GBA(32); else GBA(64);
#undef GBA
    return launch_status();
}

// ---------------------------------------------------------------------------
// Expert utilisation (Sec. 3.3: experts are ranked for pruning by how many
// tokens were routed to each of them over a validation set).
// ---------------------------------------------------------------------------
__global__ __launch_bounds__(256) void utilisation_kernel(int E, const int32_t* __restrict__ counts,
                                                          long long* __restrict__ accum) {
    const int e = threadIdx.x;
    if (e < E) accum[e] += (long long)counts[e];
}

extern "C" int moe_utilisation_accumulate(const moe_shape* shape, const int32_t* counts,
                                          int64_t* accum, void* stream) {
    int rc = check_shape(shape);
    if (rc) return rc;
    if (!counts || !accum) return MOE_ERR_NULL;
    utilisation_kernel<<<1, 256, 0, (hipStream_t)stream>>>(shape->E, counts, (long long*)accum);
    return launch_status();
}
