// Dispatch into per-expert capacity buffers and the gate-weighted combine
// (Sec. 3.1: fixed-shape per-expert buffers; dropped tokens get a zero output
// row).  Pure HBM traffic: every row moves as 16-byte vectors, one wavefront
// per row, fp32 math, no atomics (each output row has exactly one writer).
#include "moe_common.h"

#ifndef ROWS_PER_WG
#define ROWS_PER_WG 4  // one wave per row, 4 waves per workgroup
#endif

// xd[e,s,:] = x[slot_src[e,s]/k, :]   for s < expert_count[e]
template <typename T>
__global__ __launch_bounds__(64 * ROWS_PER_WG) void dispatch_kernel(int d, int k, int C, int n_rows, int n_cand,
                                                       const T* __restrict__ x,
                                                       const int32_t* __restrict__ slot_src,
                                                       const int32_t* __restrict__ expert_count,
                                                       T* __restrict__ xd) {
    const int lane = threadIdx.x & 63;
    const int row = blockIdx.x * ROWS_PER_WG + (threadIdx.x >> 6);
    if (row >= n_rows) return;
    const int e = row / C, s = row - e * C;
    if (s >= expert_count[e]) return;
    // a slot in use always names a candidate; the check only matters when the routing was
    // fed non-finite keys (two candidates can then share a rank and leave a slot unwritten)
    const int cand = slot_src[row];
    if ((unsigned)cand >= (unsigned)n_cand) return;
    const int t = cand / k;
    const uint4* src = reinterpret_cast<const uint4*>(x + (size_t)t * d);
    uint4* dst = reinterpret_cast<uint4*>(xd + (size_t)row * d);
    const int nvec = d * (int)sizeof(T) / 16;
    for (int v = lane; v < nvec; v += 64) dst[v] = src[v];
}

// The same copy, token-major: one wave per token reads x[t,:] once and writes it to the
// slot of each kept choice (the slot-major kernel above reads a token's row once per
// kept choice).  xd[expert_idx[t,j], slot[t,j], :] = x[t,:] for slot[t,j] >= 0.
template <typename T>
__global__ __launch_bounds__(64 * ROWS_PER_WG) void dispatch_tokens_kernel(int Tn, int d, int k, int E, int C,
                                                                           const T* __restrict__ x,
                                                                           const int32_t* __restrict__ expert_idx,
                                                                           const int32_t* __restrict__ slot,
                                                                           T* __restrict__ xd) {
    const int lane = threadIdx.x & 63;
    const int t = blockIdx.x * ROWS_PER_WG + (threadIdx.x >> 6);
    if (t >= Tn) return;
    uint4* dst[2] = {nullptr, nullptr};
    for (int j = 0; j < k; ++j) {
        const int s = slot[(size_t)t * k + j];
        const int e = expert_idx[(size_t)t * k + j];
        // ids and slots come from the routing call; anything else is skipped, never dereferenced
        if (s >= 0 && s < C && (unsigned)e < (unsigned)E) dst[j] = reinterpret_cast<uint4*>(xd + ((size_t)e * C + s) * d);
    }
    if (!dst[0] && !dst[1]) return;      // fully dropped token: nothing to copy, x[t] is not read
    const uint4* src = reinterpret_cast<const uint4*>(x + (size_t)t * d);
    const int nvec = d * (int)sizeof(T) / 16;
    for (int v = lane; v < nvec; v += 64) {
        const uint4 q = src[v];
        if (dst[0]) dst[0][v] = q;
        if (dst[1]) dst[1][v] = q;
    }
}

// y[t,:] = sum_j [slot>=0] g_j * yd[e_j, slot_j, :]
template <typename T>
__global__ __launch_bounds__(64 * ROWS_PER_WG) void combine_fwd_kernel(int Tn, int d, int k, int C,
                                                          const T* __restrict__ yd,
                                                          const int32_t* __restrict__ expert_idx,
                                                          const int32_t* __restrict__ slot,
                                                          const float* __restrict__ gate_w,
                                                          T* __restrict__ y) {
    constexpr int CN = Chunk<T>::N;
    const int lane = threadIdx.x & 63;
    const int t = blockIdx.x * ROWS_PER_WG + (threadIdx.x >> 6);
    if (t >= Tn) return;
    const T* src[2] = {nullptr, nullptr};
    float g[2] = {0.0f, 0.0f};
    for (int j = 0; j < k; ++j) {
        const int s = slot[(size_t)t * k + j];
        if (s >= 0) {
            src[j] = yd + ((size_t)expert_idx[(size_t)t * k + j] * C + s) * d;
            g[j] = gate_w ? gate_w[(size_t)t * k + j] : 1.0f;
        }
    }
    const int nvec = d / CN;
    for (int v = lane; v < nvec; v += 64) {
        float acc[CN];
#pragma unroll
        for (int i = 0; i < CN; ++i) acc[i] = 0.0f;
#pragma unroll
        for (int j = 0; j < 2; ++j) {
            if (src[j]) {
                float a[CN];
                Chunk<T>::load(src[j] + (size_t)v * CN, a);
#pragma unroll
                for (int i = 0; i < CN; ++i) acc[i] = fmaf(g[j], a[i], acc[i]);
            }
        }
        Chunk<T>::store(y + (size_t)t * d + (size_t)v * CN, acc);
    }
}

// dyd[e,s,:] = g_j * dy[t,:];  dgate_w[t,j] = <dy[t,:], yd[e,s,:]>
template <typename T>
__global__ __launch_bounds__(64 * ROWS_PER_WG) void combine_bwd_kernel(int Tn, int d, int k, int C,
                                                          const T* __restrict__ dy,
                                                          const T* __restrict__ yd,
                                                          const int32_t* __restrict__ expert_idx,
                                                          const int32_t* __restrict__ slot,
                                                          const float* __restrict__ gate_w,
                                                          T* __restrict__ dyd,
                                                          float* __restrict__ dgate_w) {
    constexpr int CN = Chunk<T>::N;
    const int lane = threadIdx.x & 63;
    const int t = blockIdx.x * ROWS_PER_WG + (threadIdx.x >> 6);
    if (t >= Tn) return;
    size_t off[2] = {0, 0};
    bool kept[2] = {false, false};
    float g[2] = {0.0f, 0.0f}, dot[2] = {0.0f, 0.0f};
    for (int j = 0; j < k; ++j) {
        const int s = slot[(size_t)t * k + j];
        if (s >= 0) {
            kept[j] = true;
            off[j] = ((size_t)expert_idx[(size_t)t * k + j] * C + s) * d;
            g[j] = gate_w[(size_t)t * k + j];
        }
    }
    if (kept[0] || kept[1]) {
        const int nvec = d / CN;
        for (int v = lane; v < nvec; v += 64) {
            float a[CN];
            Chunk<T>::load(dy + (size_t)t * d + (size_t)v * CN, a);
#pragma unroll
            for (int j = 0; j < 2; ++j) {
                if (kept[j]) {
                    float b[CN], o[CN];
                    Chunk<T>::load(yd + off[j] + (size_t)v * CN, b);
#pragma unroll
                    for (int i = 0; i < CN; ++i) {
                        dot[j] = fmaf(a[i], b[i], dot[j]);
                        o[i] = g[j] * a[i];
                    }
                    Chunk<T>::store(dyd + off[j] + (size_t)v * CN, o);
                }
            }
        }
    }
    for (int j = 0; j < k; ++j) {
        const float tot = wave_sum(dot[j]);
        if (lane == 0) dgate_w[(size_t)t * k + j] = kept[j] ? tot : 0.0f;
    }
}

extern "C" int moe_dispatch(const moe_shape* shape, const void* x, const int32_t* slot_src,
                            const int32_t* expert_count, void* xd, void* stream) {
    int rc = check_shape(shape);
    if (rc) return rc;
    if (!x || !slot_src || !expert_count || !xd) return MOE_ERR_NULL;
    const int n_rows = shape->E * shape->capacity;
    const int grid = ceil_div(n_rows, ROWS_PER_WG);
    hipStream_t st = (hipStream_t)stream;
    if (shape->dtype == MOE_BF16)
        dispatch_kernel<bf16_t><<<grid, 64 * ROWS_PER_WG, 0, st>>>(shape->d_model, shape->k, shape->capacity, n_rows, shape->T * shape->k,
                                                      (const bf16_t*)x, slot_src, expert_count, (bf16_t*)xd);
    else
        dispatch_kernel<float><<<grid, 64 * ROWS_PER_WG, 0, st>>>(shape->d_model, shape->k, shape->capacity, n_rows, shape->T * shape->k,
                                                     (const float*)x, slot_src, expert_count, (float*)xd);
    return launch_status();
}

extern "C" int moe_dispatch_tokens(const moe_shape* shape, const void* x, const int32_t* expert_idx,
                                   const int32_t* slot, void* xd, void* stream) {
    int rc = check_shape(shape);
    if (rc) return rc;
    if (!x || !expert_idx || !slot || !xd) return MOE_ERR_NULL;
    const int grid = ceil_div(shape->T, ROWS_PER_WG);
    hipStream_t st = (hipStream_t)stream;
    if (shape->dtype == MOE_BF16)
        dispatch_tokens_kernel<bf16_t><<<grid, 64 * ROWS_PER_WG, 0, st>>>(shape->T, shape->d_model, shape->k, shape->E, shape->capacity,
                                                                 (const bf16_t*)x, expert_idx, slot, (bf16_t*)xd);
    else
        dispatch_tokens_kernel<float><<<grid, 64 * ROWS_PER_WG, 0, st>>>(shape->T, shape->d_model, shape->k, shape->E, shape->capacity,
                                                                (const float*)x, expert_idx, slot, (float*)xd);
    return launch_status();
}

extern "C" int moe_combine_fwd(const moe_shape* shape, const void* yd, const int32_t* expert_idx,
                               const int32_t* slot, const float* gate_w_or_null, void* y,
                               void* stream) {
    int rc = check_shape(shape);
    if (rc) return rc;
    if (!yd || !expert_idx || !slot || !y) return MOE_ERR_NULL;
    const int grid = ceil_div(shape->T, ROWS_PER_WG);
    hipStream_t st = (hipStream_t)stream;
    if (shape->dtype == MOE_BF16)
        combine_fwd_kernel<bf16_t><<<grid, 64 * ROWS_PER_WG, 0, st>>>(shape->T, shape->d_model, shape->k, shape->capacity,
                                                         (const bf16_t*)yd, expert_idx, slot, gate_w_or_null, (bf16_t*)y);
    else
        combine_fwd_kernel<float><<<grid, 64 * ROWS_PER_WG, 0, st>>>(shape->T, shape->d_model, shape->k, shape->capacity,
                                                        (const float*)yd, expert_idx, slot, gate_w_or_null, (float*)y);
    return launch_status();
}

extern "C" int moe_combine_bwd(const moe_shape* shape, const void* dy, const void* yd,
                               const int32_t* expert_idx, const int32_t* slot, const float* gate_w,
                               void* dyd, float* dgate_w, void* stream) {
    int rc = check_shape(shape);
    if (rc) return rc;
    if (!dy || !yd || !expert_idx || !slot || !gate_w || !dyd || !dgate_w) return MOE_ERR_NULL;
    const int grid = ceil_div(shape->T, ROWS_PER_WG);
    hipStream_t st = (hipStream_t)stream;
    if (shape->dtype == MOE_BF16)
        combine_bwd_kernel<bf16_t><<<grid, 64 * ROWS_PER_WG, 0, st>>>(shape->T, shape->d_model, shape->k, shape->capacity,
                                                         (const bf16_t*)dy, (const bf16_t*)yd, expert_idx, slot, gate_w,
                                                         (bf16_t*)dyd, dgate_w);
    else
        combine_bwd_kernel<float><<<grid, 64 * ROWS_PER_WG, 0, st>>>(shape->T, shape->d_model, shape->k, shape->capacity,
                                                        (const float*)dy, (const float*)yd, expert_idx, slot, gate_w,
                                                        (float*)dyd, dgate_w);
    return launch_status();
}
