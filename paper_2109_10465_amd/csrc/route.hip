// moe_gate_route: softmax / top-k gate and the capacity assignment with
// Random-Token-Selection priority (Sec. 5.1 "MoE setting", Sec. 3.1).
//
// Three kernels on one stream, all integer-exact and free of float atomics:
//   1. gate_topk     a few lanes per token: top-k, softmax, gate weights; per
//                    256-token chunk a histogram of (expert, choice) segments.
//   2. route_place   every workgroup re-derives, from the chunk histograms, the
//                    segment offsets and its own chunk's prefix (a few KB of L2
//                    reads instead of a separate scan launch), then writes its
//                    candidates (t,j) into their (expert, choice) segments in
//                    token order: a stable counting sort.  Workgroup 0 also
//                    publishes segment offsets, expert_demand and expert_count.
//   3. route_rank    rank inside a segment by counting the candidates that
//                    precede it in (key descending, token ascending) order,
//                    LDS-tiled, four threads per candidate; slot = rank
//                    (+ first-choice demand for j = 1).
// Grouped token selection (Sec. 3.1) runs the same three kernels with one set
// of segments per group of consecutive tokens and Cg = C / G slots per group
// and expert; an expert's kept rows of successive groups are laid end to end.
// Work is O(T*E + sum over segments of n^2), bounded by the single-expert worst
// case; balanced routing makes step 3 a few microseconds.
#include "moe_common.h"

#define CHUNK 256       // tokens per histogram chunk (= per route_place workgroup; gate_topk: see topk_sub)
#define RANK_TILE 256   // candidates per route_rank workgroup
#define RANK_PARTS 4    // threads per candidate: each counts over a quarter of every staged tile
#define RANK_PAIR_TILES 4   // segments longer than this many tiles are ranked through key buckets
#define RANK_BUCKETS 1024   // = threads of a route_rank workgroup

struct RouteWs {
    int32_t* hist;        // [nchunk * topk_sub(E)][k*E] candidates per chunk part and segment
    int32_t* seg_start;   // [G][k*E+1] segment seg = e*k+j of group g starts here in seg_tok/seg_key
    int32_t* tile_start;  // [G][k*E+1] prefix, inside group g, of ceil(n_seg / RANK_TILE)
    int32_t* goff;        // [G][E] rows kept for expert e in the groups before g
    int32_t* seg_tok;     // [T*k]
    float* seg_key;       // [T*k]
};

static inline int n_chunks(const moe_shape* s) { return ceil_div(s->T, CHUNK); }
// With more than 64 experts a chunk's tokens are shared by 2 (4 beyond 128 experts) gate_topk
// workgroups, each with its own histogram row: a workgroup of 1024 threads then still takes 4
// rounds per chunk part, and a batch of 32 k tokens gives 256 workgroups instead of 128.
static inline int topk_sub(int E) { return E > 128 ? 4 : (E > 64 ? 2 : 1); }

// Sized for the largest possible number of groups (one per chunk).
size_t route_ws_bytes(const moe_shape* s) {
    const size_t kE = (size_t)s->k * s->E, Tk = (size_t)s->T * s->k, G = (size_t)n_chunks(s);
    return align_up(G * topk_sub(s->E) * kE * 4, 256) + 2 * align_up(G * (kE + 1) * 4, 256) + align_up(G * s->E * 4, 256) +
           2 * align_up(Tk * 4, 256);
}

static RouteWs carve(const moe_shape* s, void* ws) {
    const size_t kE = (size_t)s->k * s->E, Tk = (size_t)s->T * s->k, G = (size_t)n_chunks(s);
    char* p = (char*)ws;
    RouteWs r;
    r.hist = (int32_t*)p;       p += align_up(G * topk_sub(s->E) * kE * 4, 256);
    r.seg_start = (int32_t*)p;  p += align_up(G * (kE + 1) * 4, 256);
    r.tile_start = (int32_t*)p; p += align_up(G * (kE + 1) * 4, 256);
    r.goff = (int32_t*)p;       p += align_up(G * s->E * 4, 256);
    r.seg_tok = (int32_t*)p;    p += align_up(Tk * 4, 256);
    r.seg_key = (float*)p;
    return r;
}

// ---------------------------------------------------------------------------
// 1. gate: top-k (largest logits, ties -> smaller id), softmax, gate weights
// ---------------------------------------------------------------------------
// (value, expert) pairs ordered by value descending, expert id ascending
__device__ __forceinline__ bool better(float va, int ia, float vb, int ib) {
    return va > vb || (va == vb && ia < ib);
}

// LPT lanes share one token, 4 consecutive experts per lane (4*LPT >= E), so a
// token's logits are read with one coalesced 16-byte load per lane and reduced
// with log2(LPT) butterfly steps.  A workgroup of up to 1024 threads owns a
// 256-token chunk and walks it in ROUNDS rounds of 256/ROUNDS tokens; the logits
// of up to 8 rounds are requested before any of them is used, so the chunk costs
// one memory latency, not one per round.
template <int LPT>
struct TopkGeom {
    static constexpr int SUB = LPT >= 32 ? LPT / 16 : 1;        // workgroups per chunk (= topk_sub(E))
    static constexpr int TOK = CHUNK / SUB;                     // tokens per workgroup
    static constexpr int ROUNDS = TOK * LPT <= 1024 ? 1 : TOK * LPT / 1024;
    static constexpr int THREADS = TOK * LPT / ROUNDS;
    static constexpr int TPI = TOK / ROUNDS;                    // tokens per round
    static constexpr int BATCH = ROUNDS < 8 ? ROUNDS : 8;       // rounds whose logits are in flight together
};

template <int LPT>
__global__ __launch_bounds__(TopkGeom<LPT>::THREADS) void gate_topk_kernel(
    int T, int E, int k, const float* __restrict__ logits, float* __restrict__ probs,
    int32_t* __restrict__ expert_idx, float* __restrict__ gate_w, int32_t* __restrict__ hist) {
    typedef TopkGeom<LPT> G;
    __shared__ int32_t s_hist[512];
    const int kE = k * E;
    for (int i = threadIdx.x; i < kE; i += G::THREADS) s_hist[i] = 0;
    __syncthreads();
    const int gl = threadIdx.x % LPT, slot = threadIdx.x / LPT;
    const int e4 = gl * 4;
    const bool vec = (E & 3) == 0;
    for (int it0 = 0; it0 < G::ROUNDS; it0 += G::BATCH) {
        float lq[G::BATCH][4];
#pragma unroll
        for (int u = 0; u < G::BATCH; ++u) {
            const int t = blockIdx.x * G::TOK + (it0 + u) * G::TPI + slot;
#pragma unroll
            for (int i = 0; i < 4; ++i) lq[u][i] = -INFINITY;
            if (t < T) {
                const float* row = logits + (size_t)t * E;
                if (vec) {
                    if (e4 < E) {
                        const float4 q = *reinterpret_cast<const float4*>(row + e4);
                        lq[u][0] = q.x; lq[u][1] = q.y; lq[u][2] = q.z; lq[u][3] = q.w;
                    }
                } else {
#pragma unroll
                    for (int i = 0; i < 4; ++i)
                        if (e4 + i < E) lq[u][i] = row[e4 + i];
                }
            }
        }
#pragma unroll
        for (int u = 0; u < G::BATCH; ++u) {
            const int t = blockIdx.x * G::TOK + (it0 + u) * G::TPI + slot;
            const bool valid = t < T;   // uniform within a token's lane group
            const float(&l)[4] = lq[u];
            // the lane's own best two (ascending ids, strict comparisons).  A NaN logit never
            // wins a comparison, so for the selection it counts as -inf: among equal values
            // the smaller id wins, hence every expert id < E beats the sentinel and the
            // token's k choices are always distinct valid ids, whatever the logits hold
            // (the probabilities of such a row are NaN; nothing is indexed with them).
            float v0 = -INFINITY, v1 = -INFINITY;
            int i0 = 0x7fffffff, i1 = 0x7fffffff;
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const int e = e4 + i;
                if (e < E) {
                    const float li = l[i] == l[i] ? l[i] : -INFINITY;
                    if (better(li, e, v0, i0)) { v1 = v0; i1 = i0; v0 = li; i0 = e; }
                    else if (better(li, e, v1, i1)) { v1 = li; i1 = e; }
                }
            }
#pragma unroll
            for (int o = LPT / 2; o > 0; o >>= 1) {
                const float w0 = __shfl_xor(v0, o, MOE_WAVE), w1 = __shfl_xor(v1, o, MOE_WAVE);
                const int j0 = __shfl_xor(i0, o, MOE_WAVE), j1 = __shfl_xor(i1, o, MOE_WAVE);
                if (better(w0, j0, v0, i0)) {
                    if (better(v0, i0, w1, j1)) { v1 = v0; i1 = i0; } else { v1 = w1; i1 = j1; }
                    v0 = w0; i0 = j0;
                } else if (better(w0, j0, v1, i1)) {
                    v1 = w0; i1 = j0;
                }
            }
            float ex[4], part = 0.0f;
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                ex[i] = (valid && e4 + i < E) ? expf(l[i] - v0) : 0.0f;
                part += ex[i];
            }
#pragma unroll
            for (int o = LPT / 2; o > 0; o >>= 1) part += __shfl_xor(part, o, MOE_WAVE);
            const float sum = part;
            if (valid) {
                float* pr = probs + (size_t)t * E;
                const float inv = 1.0f / sum;      // one division per lane; the products are within an ulp of ex / sum
                if (vec) {
                    if (e4 < E)
                        *reinterpret_cast<float4*>(pr + e4) = make_float4(ex[0] * inv, ex[1] * inv, ex[2] * inv, ex[3] * inv);
                } else {
#pragma unroll
                    for (int i = 0; i < 4; ++i)
                        if (e4 + i < E) pr[e4 + i] = ex[i] * inv;
                }
                if (gl == 0) {
                    const float p0 = 1.0f / sum;   // = exp(0) / sum
                    if (k == 1) {
                        expert_idx[t] = i0;
                        gate_w[t] = p0;
                        atomicAdd(&s_hist[i0], 1);
                    } else {
                        const float p1 = expf(v1 - v0) / sum;
                        const float S = p0 + p1;
                        expert_idx[2 * t] = i0;
                        expert_idx[2 * t + 1] = i1;
                        gate_w[2 * t] = p0 / S;
                        gate_w[2 * t + 1] = p1 / S;
                        atomicAdd(&s_hist[i0 * 2], 1);
                        atomicAdd(&s_hist[i1 * 2 + 1], 1);
                    }
                }
            }
        }
    }
    __syncthreads();
    for (int i = threadIdx.x; i < kE; i += G::THREADS) hist[(size_t)blockIdx.x * kE + i] = s_hist[i];
}

// ---------------------------------------------------------------------------
// 2. segment offsets + stable placement of candidates (token order kept)
// ---------------------------------------------------------------------------
__device__ __forceinline__ int wave_incl_scan(int v, int lane) {
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) {
        const int u = __shfl_up(v, o, MOE_WAVE);
        if (lane >= o) v += u;
    }
    return v;
}

// Groups (grouped token selection, Sec. 3.1): chunks [g*cpg, (g+1)*cpg) form group
// g, which routes on its own with Cg slots per expert; its candidates occupy
// positions [g*cpg*CHUNK*k, ...) of seg_tok/seg_key.  One group = plain routing.
__global__ __launch_bounds__(CHUNK) void route_place_kernel(
    int T, int E, int k, int Cg, int nchunk, int cpg, int sub, const int32_t* __restrict__ expert_idx,
    const float* __restrict__ keys, const int32_t* __restrict__ hist,
    int32_t* __restrict__ seg_start, int32_t* __restrict__ tile_start, int32_t* __restrict__ goff,
    int32_t* __restrict__ expert_count, int32_t* __restrict__ expert_demand,
    int32_t* __restrict__ seg_tok, float* __restrict__ seg_key) {
    __shared__ int32_t s_tot[512];          // candidates per segment, whole group
    __shared__ int32_t s_base[512];         // segment start + candidates in the group's earlier chunks
    __shared__ int32_t s_wcnt[CHUNK / 64][512];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int chunk = blockIdx.x;
    const int kE = k * E;
    const int g = chunk / cpg, c_lo = g * cpg, c_hi = min(c_lo + cpg, nchunk);
    const bool leader = chunk == c_lo;      // publishes the group's tables
    // this thread's token: requested first, used after the offsets are known
    const int t = chunk * CHUNK + threadIdx.x;
    const bool valid = t < T;
    const float key = (valid && keys) ? keys[t] : 0.0f;
    int ev[2] = {-1, -1}, rank[2] = {0, 0};
    for (int j = 0; j < k; ++j) ev[j] = valid ? expert_idx[(size_t)t * k + j] : -1;
    for (int seg = threadIdx.x; seg < kE; seg += CHUNK) {
        s_tot[seg] = 0;
        s_base[seg] = 0;
#pragma unroll
        for (int w = 0; w < CHUNK / 64; ++w) s_wcnt[w][seg] = 0;
    }
    __syncthreads();
    {
        // the group's histograms are one array [chunk part][segment]: every thread sums a
        // strided share of it (16 loads in flight) and adds its part with integer LDS
        // atomics; entries of chunks before this one also count towards the prefix
        const int32_t* gh = hist + (size_t)c_lo * sub * kE;      // sub histogram rows per chunk
        const int n = (c_hi - c_lo) * sub * kE, before = (chunk - c_lo) * sub * kE;
        const bool fixed_seg = CHUNK % kE == 0;   // then a thread always meets the same segment
        constexpr int HU = 16;
        int tot = 0, pre = 0;
        for (int i0 = threadIdx.x; i0 < n; i0 += HU * CHUNK) {
            int v[HU];
#pragma unroll
            for (int u = 0; u < HU; ++u) v[u] = i0 + u * CHUNK < n ? gh[i0 + u * CHUNK] : 0;
#pragma unroll
            for (int u = 0; u < HU; ++u) {
                const int idx = i0 + u * CHUNK;
                if (fixed_seg) {
                    tot += v[u];
                    pre += idx < before ? v[u] : 0;
                } else if (idx < n && v[u]) {
                    const int seg = idx % kE;
                    atomicAdd(&s_tot[seg], v[u]);
                    if (idx < before) atomicAdd(&s_base[seg], v[u]);
                }
            }
        }
        if (fixed_seg) {
            const int seg = threadIdx.x % kE;
            if (tot) atomicAdd(&s_tot[seg], tot);
            if (pre) atomicAdd(&s_base[seg], pre);
        }
    }
    __syncthreads();
    if (leader && threadIdx.x < E) {
        // rows kept for this expert by the groups before g (chunk 0: also the totals)
        const int e = threadIdx.x;
        const int ngroups = (nchunk + cpg - 1) / cpg;
        const int upto = chunk == 0 ? ngroups : g;
        int off = 0, dem_tot = 0, cnt_tot = 0;
        if (ngroups == 1) {      // plain routing: the group totals are the batch totals
            dem_tot = s_tot[e * k] + (k == 2 ? s_tot[e * k + 1] : 0);
            cnt_tot = dem_tot < Cg ? dem_tot : Cg;
        }
        for (int gg = 0; gg < (ngroups == 1 ? 0 : upto); ++gg) {
            int dem = 0;
            const int hi = min((gg + 1) * cpg, nchunk) * sub;   // histogram rows of group gg
            int c = gg * cpg * sub;
            for (; c + 8 <= hi; c += 8) {
                int v[8];
#pragma unroll
                for (int u = 0; u < 8; ++u) {
                    v[u] = hist[(size_t)(c + u) * kE + e * k];
                    if (k == 2) v[u] += hist[(size_t)(c + u) * kE + e * k + 1];
                }
#pragma unroll
                for (int u = 0; u < 8; ++u) dem += v[u];
            }
            for (; c < hi; ++c) {
                dem += hist[(size_t)c * kE + e * k];
                if (k == 2) dem += hist[(size_t)c * kE + e * k + 1];
            }
            const int kept = dem < Cg ? dem : Cg;
            if (gg < g) off += kept;
            dem_tot += dem;
            cnt_tot += kept;
        }
        goff[(size_t)g * E + e] = off;
        if (chunk == 0) {
            expert_demand[e] = dem_tot;
            expert_count[e] = cnt_tot;
        }
    }
    if (wave == 0) {  // exclusive scan over the group's segments (seg = e*k+j)
        int run_pos = c_lo * CHUNK * k, run_tile = 0;   // every token before the group has k candidates
        int32_t* gs = seg_start + (size_t)g * (kE + 1);
        int32_t* gt = tile_start + (size_t)g * (kE + 1);
        for (int s0 = 0; s0 < kE; s0 += 64) {
            const int seg = s0 + lane;
            const int n = seg < kE ? s_tot[seg] : 0;
            const int nt = (n + RANK_TILE - 1) / RANK_TILE;
            const int ip = wave_incl_scan(n, lane), it = wave_incl_scan(nt, lane);
            if (seg < kE) {
                const int start = run_pos + ip - n;
                s_base[seg] += start;
                if (leader) {
                    gs[seg] = start;
                    gt[seg] = run_tile + it - nt;
                }
            }
            run_pos += __shfl(ip, 63, MOE_WAVE);
            run_tile += __shfl(it, 63, MOE_WAVE);
        }
        if (leader && lane == 0) {
            gs[kE] = run_pos;
            gt[kE] = run_tile;
        }
    }
    __syncthreads();
    // rank among the wave's tokens with the same (expert, choice): the set of such
    // lanes is the intersection, over the bits of the expert id, of the lanes that
    // agree with this lane on that bit (one ballot per bit, no lane exchange)
    const int nbits = E > 1 ? 32 - __clz(E - 1) : 0;
    for (int j = 0; j < k; ++j) {
        const int e = ev[j];
        unsigned long long same = __ballot(valid);
        for (int b = 0; b < nbits; ++b) {
            const bool bit = (e >> b) & 1;
            const unsigned long long m = __ballot(valid && bit);
            same &= bit ? m : ~m;
        }
        if (valid) {
            rank[j] = __popcll(same & ((1ull << lane) - 1ull));
            if (rank[j] == 0) s_wcnt[wave][e * k + j] = __popcll(same);
        }
    }
    __syncthreads();
    if (valid) {
        for (int j = 0; j < k; ++j) {
            const int seg = ev[j] * k + j;
            int pos = s_base[seg] + rank[j];
            for (int w = 0; w < wave; ++w) pos += s_wcnt[w][seg];
            seg_tok[pos] = t;
            seg_key[pos] = key;
        }
    }
}

// ---------------------------------------------------------------------------
// 3. rank inside the segment, slots, slot_src
// ---------------------------------------------------------------------------
__global__ __launch_bounds__(RANK_TILE * RANK_PARTS) void route_rank_kernel(
    int E, int k, int C, int Cg, int tiles_per_group, int has_keys, const int32_t* __restrict__ seg_start_all,
    const int32_t* __restrict__ tile_start_all, const int32_t* __restrict__ goff,
    const int32_t* __restrict__ expert_count, const int32_t* __restrict__ seg_tok,
    const float* __restrict__ seg_key, int32_t* __restrict__ slot, int32_t* __restrict__ slot_src) {
    constexpr int NT = RANK_TILE * RANK_PARTS, Q = RANK_TILE / RANK_PARTS;
    __shared__ __align__(16) float s_key[2][RANK_TILE];
    __shared__ int s_cnt[RANK_PARTS][RANK_TILE];
    __shared__ int s_info[5];   // segment, its start and end, its first tile, start of the segment before it
    const int kE = k * E;
    const int tid = threadIdx.x & (RANK_TILE - 1);          // candidate inside the tile
    const int part = threadIdx.x / RANK_TILE;               // wave-uniform
    const int grp = blockIdx.x / tiles_per_group;
    const int b = blockIdx.x - grp * tiles_per_group;       // tile inside the group
    const int32_t* seg_start = seg_start_all + (size_t)grp * (kE + 1);
    const int32_t* tile_start = tile_start_all + (size_t)grp * (kE + 1);
    // segment owning tile b: the one with tile_start[seg] <= b < tile_start[seg+1]
    // (empty segments have an empty range); found by all threads in parallel, each
    // fetching what the owner will need in the same round of loads
    if (threadIdx.x == 0) s_info[0] = -1;
    __syncthreads();
    for (int sg = threadIdx.x; sg < kE; sg += NT) {
        const int t0 = tile_start[sg], t1 = tile_start[sg + 1];
        const int a0 = seg_start[sg], a1 = seg_start[sg + 1];
        const int ap = sg > 0 ? seg_start[sg - 1] : 0;
        if (t0 <= b && b < t1) {
            s_info[0] = sg; s_info[1] = a0; s_info[2] = a1; s_info[3] = t0; s_info[4] = ap;
        }
    }
    // unused slots (independent of the ranking; its loads overlap the search above)
    const int total = E * C;
    for (int idx = blockIdx.x * NT + threadIdx.x; idx < total; idx += gridDim.x * NT) {
        const int e = idx / C, sl = idx - e * C;
        if (sl >= expert_count[e]) slot_src[idx] = -1;
    }
    __syncthreads();
    if (s_info[0] < 0) return;   // uniform: a spare tile
    const int seg = s_info[0], s0 = s_info[1], s1 = s_info[2];
    const int own0 = s0 + (b - s_info[3]) * RANK_TILE;
    const int p = own0 + tid;
    const bool valid = p < s1;
    const int e = seg / k, j = seg - e * k;
    // everything the result needs is requested before the ranking starts
    const int tok = (valid && part == 0) ? seg_tok[p] : 0;
    const int row0 = goff[(size_t)grp * E + e];             // earlier groups' rows come first
    int cnt = p - s0;  // position priority: candidates are stored in token order
    const int n_seg = s1 - s0;
    if (has_keys && n_seg > RANK_PAIR_TILES * RANK_TILE) {
        // Long segment (skewed routing): counting every pair costs n per candidate.  Instead
        // the workgroup buckets the segment's keys by value (any monotone bucket function keeps
        // the result exact): candidates in higher buckets precede, and only the keys that fall
        // into the bucket of one of the tile's own candidates are compared with it.  Three
        // passes over the segment's keys (L2), each thread a strided share.
        static_assert(RANK_BUCKETS == NT, "one bucket per thread");
        __shared__ int s_hist[RANK_BUCKETS];      // keys per bucket, then inclusive prefix sums
        __shared__ int s_head[RANK_BUCKETS];      // list of the tile's own candidates per bucket
        __shared__ int s_next[RANK_TILE];
        __shared__ float s_mine[RANK_TILE];
        __shared__ int s_prec[RANK_TILE];         // same-bucket candidates that precede
        __shared__ float s_lo[NT / 64], s_hi[NT / 64];
        __shared__ int s_wtot[NT / 64];
        const int lane = threadIdx.x & 63, wv = threadIdx.x >> 6;
        float lo = INFINITY, hi = -INFINITY;
        for (int i = threadIdx.x; i < n_seg; i += NT) {
            const float kq = seg_key[s0 + i];
            lo = fminf(lo, kq);
            hi = fmaxf(hi, kq);
        }
        lo = -wave_max(-lo);
        hi = wave_max(hi);
        if (lane == 0) { s_lo[wv] = lo; s_hi[wv] = hi; }
        s_hist[threadIdx.x] = 0;
        s_head[threadIdx.x] = -1;
        __syncthreads();
#pragma unroll
        for (int w = 0; w < NT / 64; ++w) { lo = fminf(lo, s_lo[w]); hi = fmaxf(hi, s_hi[w]); }
        const float span = hi - lo;
        const float scale = (span > 0.0f && span < INFINITY) ? (float)RANK_BUCKETS / span : 0.0f;
        // monotone in the key: subtraction, a non-negative factor, the clamp and the truncation all are
        // (scale 0 - all keys equal, or a span beyond fp32 - puts everything into bucket 0: still exact)
        auto bucket = [&](float kq) {
            return scale == 0.0f ? 0 : (int)fminf((kq - lo) * scale, (float)(RANK_BUCKETS - 1));
        };
        const float mine = (valid && part == 0) ? seg_key[p] : 0.0f;
        const int my_b = bucket(mine);
        if (valid && part == 0) {
            s_mine[tid] = mine;
            s_prec[tid] = 0;
            s_next[tid] = atomicExch(&s_head[my_b], tid);
        }
        for (int i = threadIdx.x; i < n_seg; i += NT) atomicAdd(&s_hist[bucket(seg_key[s0 + i])], 1);
        __syncthreads();
        {   // inclusive prefix sums of the bucket counts: wave scan, then the earlier waves' totals
            const int incl = wave_incl_scan(s_hist[threadIdx.x], lane);
            if (lane == 63) s_wtot[wv] = incl;
            __syncthreads();
            int before = 0;
            for (int w = 0; w < wv; ++w) before += s_wtot[w];
            s_hist[threadIdx.x] = incl + before;
        }
        for (int i = threadIdx.x; i < n_seg; i += NT) {
            const int q = s0 + i;
            const float kq = seg_key[q];
            for (int c = s_head[bucket(kq)]; c >= 0; c = s_next[c]) {
                const float mc = s_mine[c];
                if (kq > mc || (kq == mc && q < own0 + c)) atomicAdd(&s_prec[c], 1);   // equal keys: token order
            }
        }
        __syncthreads();
        if (valid && part == 0) cnt = (n_seg - s_hist[my_b]) + s_prec[tid];
    } else if (has_keys) {
        const float mine = valid ? seg_key[p] : 0.0f;
        cnt = 0;
        float nxt = (part == 0 && s0 + tid < s1) ? seg_key[s0 + tid] : -INFINITY;
        int buf = 0;
        for (int q0 = s0; q0 < s1; q0 += RANK_TILE, buf ^= 1) {
            if (part == 0) s_key[buf][tid] = nxt;   // the other buffer may still be read by slower waves
            __syncthreads();
            const int qn = q0 + RANK_TILE + tid;
            nxt = (part == 0 && qn < s1) ? seg_key[qn] : -INFINITY;   // in flight under the counting
            const float4* kk = reinterpret_cast<const float4*>(s_key[buf] + part * Q);
            if (q0 < own0) {          // earlier tokens: equal keys precede
#pragma unroll 4
                for (int i = 0; i < Q / 4; ++i) {
                    const float4 c4 = kk[i];
                    cnt += (c4.x >= mine) + (c4.y >= mine) + (c4.z >= mine) + (c4.w >= mine);
                }
            } else if (q0 > own0) {   // later tokens: only strictly larger keys precede
#pragma unroll 4
                for (int i = 0; i < Q / 4; ++i) {
                    const float4 c4 = kk[i];
                    cnt += (c4.x > mine) + (c4.y > mine) + (c4.z > mine) + (c4.w > mine);
                }
            } else {
#pragma unroll 4
                for (int i = 0; i < Q / 4; ++i) {
                    const float4 c4 = kk[i];
                    const int i4 = part * Q + 4 * i;
                    cnt += (c4.x > mine || (c4.x == mine && i4 < tid)) + (c4.y > mine || (c4.y == mine && i4 + 1 < tid)) +
                           (c4.z > mine || (c4.z == mine && i4 + 2 < tid)) + (c4.w > mine || (c4.w == mine && i4 + 3 < tid));
                }
            }
        }
        s_cnt[part][tid] = cnt;
        __syncthreads();
        if (part == 0) {
            cnt = 0;
#pragma unroll
            for (int q = 0; q < RANK_PARTS; ++q) cnt += s_cnt[q][tid];
        }
    }
    if (valid && part == 0) {
        const int base = j == 1 ? s0 - s_info[4] : 0;           // first choices go first
        const int rank = base + cnt;                            // inside (group, expert)
        const int cand = tok * k + j;
        const int row = row0 + rank;
        slot[cand] = rank < Cg ? row : -1;
        if (rank < Cg) slot_src[(size_t)e * C + row] = cand;
    }
}

static int route_impl(const moe_shape* shape, int G, const float* logits, const float* rts_keys_or_null,
                      float* probs, int32_t* expert_idx, float* gate_w, int32_t* slot,
                      int32_t* expert_count, int32_t* expert_demand, int32_t* slot_src, void* ws,
                      size_t ws_bytes, void* stream) {
    int rc = check_shape(shape);
    if (rc) return rc;
    if (!logits || !probs || !expert_idx || !gate_w || !slot || !expert_count || !expert_demand ||
        !slot_src)
        return MOE_ERR_NULL;
    const int T = shape->T, E = shape->E, k = shape->k, C = shape->capacity;
    if (G < 1) return MOE_ERR_SHAPE;
    if (G > 1 && (T % G || (T / G) % CHUNK || C % G)) return MOE_ERR_SHAPE;
    if (!ws || ((uintptr_t)ws & 255) || ws_bytes < route_ws_bytes(shape)) return MOE_ERR_WORKSPACE;
    hipStream_t st = (hipStream_t)stream;
    const RouteWs r = carve(shape, ws);
    const int nchunk = n_chunks(shape);
    const int cpg = G == 1 ? nchunk : T / G / CHUNK;    // chunks per group
    const int Cg = C / G;
#define GATE(LPT) gate_topk_kernel<LPT><<<nchunk * TopkGeom<LPT>::SUB, TopkGeom<LPT>::THREADS, 0, st>>>(T, E, k, logits, probs, expert_idx, gate_w, r.hist)
    if (E <= 4) GATE(1); else if (E <= 8) GATE(2); else if (E <= 16) GATE(4); else if (E <= 32) GATE(8);
    else if (E <= 64) GATE(16); else if (E <= 128) GATE(32); else GATE(64);
#undef GATE
    route_place_kernel<<<nchunk, CHUNK, 0, st>>>(T, E, k, Cg, nchunk, cpg, topk_sub(E), expert_idx, rts_keys_or_null, r.hist,
                                                 r.seg_start, r.tile_start, r.goff, expert_count,
                                                 expert_demand, r.seg_tok, r.seg_key);
    const int Tg = G == 1 ? T : T / G;
    const int tiles_per_group = ceil_div(Tg * k, RANK_TILE) + k * E;
    route_rank_kernel<<<G * tiles_per_group, RANK_TILE * RANK_PARTS, 0, st>>>(E, k, C, Cg, tiles_per_group,
                                                                 rts_keys_or_null != nullptr, r.seg_start,
                                                                 r.tile_start, r.goff, expert_count, r.seg_tok,
                                                                 r.seg_key, slot, slot_src);
    return launch_status();
}

extern "C" int moe_gate_route(const moe_shape* shape, const float* logits,
                              const float* rts_keys_or_null, float* probs, int32_t* expert_idx,
                              float* gate_w, int32_t* slot, int32_t* expert_count,
                              int32_t* expert_demand, int32_t* slot_src, void* ws, size_t ws_bytes,
                              void* stream) {
    return route_impl(shape, 1, logits, rts_keys_or_null, probs, expert_idx, gate_w, slot, expert_count,
                      expert_demand, slot_src, ws, ws_bytes, stream);
}

// ---------------------------------------------------------------------------
// moe_gate_route for callers that cannot allocate: the scratch memory (chunk
// histograms, segment tables, segment-sorted candidate lists) lives in a
// file-scope device array instead of a caller workspace.  Every GPU holds its
// own copy of the array at its own address; the address is looked up once per
// device and that pointer, never the array's name, is what host code passes on.
// ---------------------------------------------------------------------------
#define ROUTE_SCRATCH_BYTES (5u << 20)
static __device__ __align__(256) unsigned char scratch[ROUTE_SCRATCH_BYTES];

#define ROUTE_MAX_DEVICES 64
static void* scratch_ptr_of_current_device() {
    static void* ptrs[ROUTE_MAX_DEVICES];      // zero-initialised; written once per device
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= ROUTE_MAX_DEVICES) return nullptr;
    void* p = __atomic_load_n(&ptrs[dev], __ATOMIC_ACQUIRE);
    if (!p) {
        // a plain address query (no allocation); two threads racing here look up the same address
        if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) {
            (void)hipGetLastError();
            return nullptr;
        }
        __atomic_store_n(&ptrs[dev], p, __ATOMIC_RELEASE);
    }
    return p;
}

extern "C" size_t moe_gate_route_static_max_bytes(void) { return ROUTE_SCRATCH_BYTES; }

extern "C" int moe_gate_route_static(const moe_shape* shape, const float* logits,
                                     const float* rts_keys_or_null, float* probs, int32_t* expert_idx,
                                     float* gate_w, int32_t* slot, int32_t* expert_count,
                                     int32_t* expert_demand, int32_t* slot_src, void* stream) {
    int rc = check_shape(shape);
    if (rc) return rc;
    if (route_ws_bytes(shape) > ROUTE_SCRATCH_BYTES) return MOE_ERR_WORKSPACE;   // shape beyond the built-in scratch
    void* ws = scratch_ptr_of_current_device();
    if (!ws) return MOE_ERR_LAUNCH;
    // Nothing in the scratch has to start at zero: the histograms, the segment tables and the
    // candidate lists are all written in full by this call's kernels before they are read, so
    // what an earlier (possibly larger) call left behind is never seen.
    return route_impl(shape, 1, logits, rts_keys_or_null, probs, expert_idx, gate_w, slot, expert_count,
                      expert_demand, slot_src, ws, ROUTE_SCRATCH_BYTES, stream);
}

extern "C" int moe_gate_route_grouped(const moe_shape* shape, int32_t n_groups, const float* logits,
                                      const float* rts_keys_or_null, float* probs, int32_t* expert_idx,
                                      float* gate_w, int32_t* slot, int32_t* expert_count,
                                      int32_t* expert_demand, int32_t* slot_src, void* ws,
                                      size_t ws_bytes, void* stream) {
    return route_impl(shape, n_groups, logits, rts_keys_or_null, probs, expert_idx, gate_w, slot, expert_count,
                      expert_demand, slot_src, ws, ws_bytes, stream);
}
