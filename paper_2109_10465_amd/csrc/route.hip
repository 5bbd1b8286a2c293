// moe_gate_route: softmax / top-k gate and the capacity assignment with
// Random-Token-Selection priority (Sec. 5.1 "MoE setting", Sec. 3.1).
//
// Four kernels on one stream, all integer-exact and free of float atomics:
//   1. gate_topk     one wave per token: softmax, top-k, gate weights; per
//                    64-token chunk a histogram of (expert, choice) segments.
//   2. route_scan    one workgroup: exclusive prefix of the histograms over
//                    chunks, segment offsets, expert_demand / expert_count.
//   3. route_place   stable counting-sort placement: every candidate (t,j) is
//                    written into its (expert, choice) segment in token order.
//   4. route_rank    rank inside a segment by counting the candidates that
//                    precede it in (key descending, token ascending) order,
//                    LDS-tiled; slot = rank (+ first-choice demand for j = 1).
// Total work is O(T*E + sum over segments n^2 / 1), bounded by the single-expert
// worst case; typical balanced routing makes step 4 a few microseconds.
#include "moe_common.h"

#define CHUNK 64        // tokens per histogram chunk (= per gate_topk workgroup)
#define RANK_TILE 256   // candidates per route_rank workgroup

struct RouteWs {
    int32_t* hist;        // [nchunk][k*E] -> exclusive prefix over chunks
    int32_t* seg_start;   // [k*E+1] segment seg = e*k+j starts here in seg_tok/seg_key
    int32_t* tile_start;  // [k*E+1] prefix of ceil(n_seg / RANK_TILE)
    int32_t* seg_tok;     // [T*k]
    float* seg_key;       // [T*k]
};

static inline int n_chunks(const moe_shape* s) { return ceil_div(s->T, CHUNK); }

size_t route_ws_bytes(const moe_shape* s) {
    const size_t kE = (size_t)s->k * s->E, Tk = (size_t)s->T * s->k;
    return align_up((size_t)n_chunks(s) * kE * 4, 256) + 2 * align_up((kE + 1) * 4, 256) +
           2 * align_up(Tk * 4, 256);
}

static RouteWs carve(const moe_shape* s, void* ws) {
    const size_t kE = (size_t)s->k * s->E, Tk = (size_t)s->T * s->k;
    char* p = (char*)ws;
    RouteWs r;
    r.hist = (int32_t*)p;       p += align_up((size_t)n_chunks(s) * kE * 4, 256);
    r.seg_start = (int32_t*)p;  p += align_up((kE + 1) * 4, 256);
    r.tile_start = (int32_t*)p; p += align_up((kE + 1) * 4, 256);
    r.seg_tok = (int32_t*)p;    p += align_up(Tk * 4, 256);
    r.seg_key = (float*)p;
    return r;
}

// ---------------------------------------------------------------------------
// 1. gate: softmax, top-k (largest logits, ties -> smaller id), gate weights
// ---------------------------------------------------------------------------
__device__ __forceinline__ void argmax_reduce(float& v, int& i) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) {
        const float ov = __shfl_xor(v, o, MOE_WAVE);
        const int oi = __shfl_xor(i, o, MOE_WAVE);
        if (ov > v || (ov == v && oi < i)) { v = ov; i = oi; }
    }
}

template <int NI>  // experts per lane: E <= 64*NI
__global__ __launch_bounds__(256) void gate_topk_kernel(
    int T, int E, int k, const float* __restrict__ logits, float* __restrict__ probs,
    int32_t* __restrict__ expert_idx, float* __restrict__ gate_w, int32_t* __restrict__ hist) {
    __shared__ int32_t s_hist[512];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int kE = k * E;
    for (int i = threadIdx.x; i < kE; i += 256) s_hist[i] = 0;
    __syncthreads();
    const int t0 = blockIdx.x * CHUNK + wave * (CHUNK / 4);
    for (int tt = 0; tt < CHUNK / 4; ++tt) {
        const int t = t0 + tt;
        if (t >= T) break;  // uniform per wave
        float l[NI];
#pragma unroll
        for (int i = 0; i < NI; ++i) {
            const int e = lane + 64 * i;
            l[i] = e < E ? logits[(size_t)t * E + e] : -INFINITY;
        }
        // first choice
        float bv = -INFINITY;
        int bi = 0x7fffffff;
#pragma unroll
        for (int i = 0; i < NI; ++i)
            if (lane + 64 * i < E && (l[i] > bv || bi == 0x7fffffff)) { bv = l[i]; bi = lane + 64 * i; }
        argmax_reduce(bv, bi);
        const int e0 = bi;
        const float mx = bv;
        // second choice: same reduction with e0 masked out
        int e1 = -1;
        if (k == 2) {
            float cv = -INFINITY;
            int ci = 0x7fffffff;
#pragma unroll
            for (int i = 0; i < NI; ++i) {
                const int e = lane + 64 * i;
                if (e < E && e != e0 && (l[i] > cv || ci == 0x7fffffff)) { cv = l[i]; ci = e; }
            }
            argmax_reduce(cv, ci);
            e1 = ci;
        }
        // softmax
        float ex[NI], part = 0.0f;
#pragma unroll
        for (int i = 0; i < NI; ++i) {
            ex[i] = lane + 64 * i < E ? expf(l[i] - mx) : 0.0f;
            part += ex[i];
        }
        const float sum = wave_sum(part);
        float p[NI];
#pragma unroll
        for (int i = 0; i < NI; ++i) {
            p[i] = ex[i] / sum;
            if (lane + 64 * i < E) probs[(size_t)t * E + lane + 64 * i] = p[i];
        }
        // probabilities of the chosen experts, broadcast from their owner lanes
        float p0 = 0.0f, p1 = 0.0f;
#pragma unroll
        for (int i = 0; i < NI; ++i) {
            const float a = __shfl(p[i], e0 & 63, MOE_WAVE);
            if ((e0 >> 6) == i) p0 = a;
            if (k == 2) {
                const float b = __shfl(p[i], e1 & 63, MOE_WAVE);
                if ((e1 >> 6) == i) p1 = b;
            }
        }
        if (lane == 0) {
            if (k == 1) {
                expert_idx[t] = e0;
                gate_w[t] = p0;
                atomicAdd(&s_hist[e0], 1);
            } else {
                const float S = p0 + p1;
                expert_idx[2 * t] = e0;
                expert_idx[2 * t + 1] = e1;
                gate_w[2 * t] = p0 / S;
                gate_w[2 * t + 1] = p1 / S;
                atomicAdd(&s_hist[e0 * 2], 1);
                atomicAdd(&s_hist[e1 * 2 + 1], 1);
            }
        }
    }
    __syncthreads();
    for (int i = threadIdx.x; i < kE; i += 256) hist[(size_t)blockIdx.x * kE + i] = s_hist[i];
}

// ---------------------------------------------------------------------------
// 2. scan over chunks per segment, then over segments
// ---------------------------------------------------------------------------
__device__ __forceinline__ int wave_incl_scan(int v, int lane) {
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) {
        const int u = __shfl_up(v, o, MOE_WAVE);
        if (lane >= o) v += u;
    }
    return v;
}

__global__ __launch_bounds__(1024) void route_scan_kernel(
    int E, int k, int C, int nchunk, int32_t* __restrict__ hist, int32_t* __restrict__ seg_start,
    int32_t* __restrict__ tile_start, int32_t* __restrict__ expert_count,
    int32_t* __restrict__ expert_demand) {
    __shared__ int32_t s_total[512];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int kE = k * E;
    for (int seg = wave; seg < kE; seg += 16) {
        int running = 0;
        for (int c0 = 0; c0 < nchunk; c0 += 64) {
            const int c = c0 + lane;
            const int v = c < nchunk ? hist[(size_t)c * kE + seg] : 0;
            const int incl = wave_incl_scan(v, lane);
            if (c < nchunk) hist[(size_t)c * kE + seg] = running + incl - v;
            running += __shfl(incl, 63, MOE_WAVE);
        }
        if (lane == 0) s_total[seg] = running;
    }
    __syncthreads();
    if (wave == 0) {
        int run_pos = 0, run_tile = 0;
        for (int s0 = 0; s0 < kE; s0 += 64) {
            const int seg = s0 + lane;
            const int n = seg < kE ? s_total[seg] : 0;
            const int nt = (n + RANK_TILE - 1) / RANK_TILE;
            const int ip = wave_incl_scan(n, lane), it = wave_incl_scan(nt, lane);
            if (seg < kE) {
                seg_start[seg] = run_pos + ip - n;
                tile_start[seg] = run_tile + it - nt;
            }
            run_pos += __shfl(ip, 63, MOE_WAVE);
            run_tile += __shfl(it, 63, MOE_WAVE);
        }
        if (lane == 0) {
            seg_start[kE] = run_pos;
            tile_start[kE] = run_tile;
        }
        for (int e = lane; e < E; e += 64) {
            int dem = s_total[e * k];
            if (k == 2) dem += s_total[e * k + 1];
            expert_demand[e] = dem;
            expert_count[e] = dem < C ? dem : C;
        }
    }
}

// ---------------------------------------------------------------------------
// 3. stable placement of candidates into their segments (token order kept)
// ---------------------------------------------------------------------------
__global__ __launch_bounds__(256) void route_place_kernel(
    int T, int E, int k, const int32_t* __restrict__ expert_idx, const float* __restrict__ keys,
    const int32_t* __restrict__ hist, const int32_t* __restrict__ seg_start,
    int32_t* __restrict__ seg_tok, float* __restrict__ seg_key) {
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int chunk = blockIdx.x * 4 + wave;
    const int t = chunk * CHUNK + lane;
    const bool valid = t < T;
    const int kE = k * E;
    const float key = (valid && keys) ? keys[t] : 0.0f;
    for (int j = 0; j < k; ++j) {
        const int e = valid ? expert_idx[(size_t)t * k + j] : -1;
        unsigned long long todo = __ballot(valid);
        int rank = 0;
        while (todo) {  // one round per distinct expert among the 64 tokens
            const int leader = __ffsll((long long)todo) - 1;
            const int ev = __shfl(e, leader, MOE_WAVE);
            const unsigned long long same = __ballot(valid && e == ev);
            if (valid && e == ev) rank = __popcll(same & ((1ull << lane) - 1ull));
            todo &= ~same;
        }
        if (valid) {
            const int seg = e * k + j;
            const int pos = seg_start[seg] + hist[(size_t)chunk * kE + seg] + rank;
            seg_tok[pos] = t;
            seg_key[pos] = key;
        }
    }
}

// ---------------------------------------------------------------------------
// 4. rank inside the segment, slots, slot_src
// ---------------------------------------------------------------------------
__global__ __launch_bounds__(RANK_TILE) void route_rank_kernel(
    int E, int k, int C, int has_keys, const int32_t* __restrict__ seg_start,
    const int32_t* __restrict__ tile_start, const int32_t* __restrict__ seg_tok,
    const float* __restrict__ seg_key, int32_t* __restrict__ slot, int32_t* __restrict__ slot_src) {
    __shared__ float s_key[RANK_TILE];
    const int kE = k * E;
    const int tid = threadIdx.x;
    const int b = blockIdx.x;
    if (b < tile_start[kE]) {
        // segment owning tile b: the last seg with tile_start[seg] <= b
        int lo = 0, hi = kE - 1;
        while (lo < hi) {
            const int mid = (lo + hi + 1) >> 1;
            if (tile_start[mid] <= b) lo = mid; else hi = mid - 1;
        }
        const int seg = lo;
        const int s0 = seg_start[seg], s1 = seg_start[seg + 1];
        const int own0 = s0 + (b - tile_start[seg]) * RANK_TILE;
        const int p = own0 + tid;
        const bool valid = p < s1;
        int cnt = p - s0;  // position priority: candidates are stored in token order
        if (has_keys) {
            const float mine = valid ? seg_key[p] : 0.0f;
            cnt = 0;
            for (int q0 = s0; q0 < s1; q0 += RANK_TILE) {
                __syncthreads();
                s_key[tid] = q0 + tid < s1 ? seg_key[q0 + tid] : -INFINITY;
                __syncthreads();
                if (q0 < own0) {          // earlier tokens: equal keys precede
#pragma unroll 8
                    for (int i = 0; i < RANK_TILE; ++i) cnt += s_key[i] >= mine;
                } else if (q0 > own0) {   // later tokens: only strictly larger keys precede
#pragma unroll 8
                    for (int i = 0; i < RANK_TILE; ++i) cnt += s_key[i] > mine;
                } else {
#pragma unroll 8
                    for (int i = 0; i < RANK_TILE; ++i)
                        cnt += (s_key[i] > mine) || (s_key[i] == mine && i < tid);
                }
            }
        }
        if (valid) {
            const int e = seg / k, j = seg - e * k;
            const int base = j == 1 ? s0 - seg_start[seg - 1] : 0;  // first choices go first
            const int rank = base + cnt;
            const int cand = seg_tok[p] * k + j;
            slot[cand] = rank < C ? rank : -1;
            if (rank < C) slot_src[(size_t)e * C + rank] = cand;
        }
    }
    // unused slots
    const int total = E * C;
    for (int idx = b * RANK_TILE + tid; idx < total; idx += gridDim.x * RANK_TILE) {
        const int e = idx / C, s = idx - e * C;
        const int dem = seg_start[(e + 1) * k] - seg_start[e * k];
        if (s >= dem) slot_src[idx] = -1;
    }
}

extern "C" int moe_gate_route(const moe_shape* shape, const float* logits,
                              const float* rts_keys_or_null, float* probs, int32_t* expert_idx,
                              float* gate_w, int32_t* slot, int32_t* expert_count,
                              int32_t* expert_demand, int32_t* slot_src, void* ws, size_t ws_bytes,
                              void* stream) {
    int rc = check_shape(shape);
    if (rc) return rc;
    if (!logits || !probs || !expert_idx || !gate_w || !slot || !expert_count || !expert_demand ||
        !slot_src)
        return MOE_ERR_NULL;
    if (!ws || ((uintptr_t)ws & 255) || ws_bytes < route_ws_bytes(shape)) return MOE_ERR_WORKSPACE;
    hipStream_t st = (hipStream_t)stream;
    const int T = shape->T, E = shape->E, k = shape->k, C = shape->capacity;
    const RouteWs r = carve(shape, ws);
    const int nchunk = n_chunks(shape);
    const int ni = ceil_div(E, 64);
#define GATE(NI) gate_topk_kernel<NI><<<nchunk, 256, 0, st>>>(T, E, k, logits, probs, expert_idx, gate_w, r.hist)
    if (ni == 1) GATE(1); else if (ni == 2) GATE(2); else if (ni == 3) GATE(3); else GATE(4);
#undef GATE
    route_scan_kernel<<<1, 1024, 0, st>>>(E, k, C, nchunk, r.hist, r.seg_start, r.tile_start,
                                          expert_count, expert_demand);
    route_place_kernel<<<ceil_div(nchunk, 4), 256, 0, st>>>(T, E, k, expert_idx, rts_keys_or_null,
                                                            r.hist, r.seg_start, r.seg_tok, r.seg_key);
    const int ntile_max = ceil_div(T * k, RANK_TILE) + k * E;
    route_rank_kernel<<<ntile_max, RANK_TILE, 0, st>>>(E, k, C, rts_keys_or_null != nullptr,
                                                       r.seg_start, r.tile_start, r.seg_tok,
                                                       r.seg_key, slot, slot_src);
    return launch_status();
}
