// Measurement aid, not a step of the layer: the rate of the bf16 matrix pipe with
// register-resident operands, so that a benchmark can print what this chip
// sustains next to the published peak the roofline is quoted against.
#include "moe_common.h"
#include "../../include/moe_bench_aid.h"

typedef float mb_f32x16 __attribute__((ext_vector_type(16)));

// Every wave issues `iters` rounds of 8 independent v_mfma_f32_32x32x16_bf16 (8
// accumulator tiles: the pipe never waits for a result).  Operands: small seeded
// pseudo-random values, or all-equal ones (random = 0): the clock the chip holds
// under matrix load depends on how many bits toggle.
__global__ __launch_bounds__(256) void mfma_rate_kernel(int iters, int random, float* __restrict__ out) {
    mb_f32x16 acc[8];
#pragma unroll
    for (int i = 0; i < 8; ++i)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[i][v] = 0.0f;
    float fa[2][8], fb[2][8];
    uint32_t r = threadIdx.x * 2654435761u + blockIdx.x * 40503u + 12345u;
#pragma unroll
    for (int q = 0; q < 2; ++q)
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            r = r * 1664525u + 1013904223u;
            fa[q][i] = random ? ((int)((r >> 8) % 2001u) - 1000) * 1e-3f : 0.5f;
            r = r * 1664525u + 1013904223u;
            fb[q][i] = random ? ((int)((r >> 8) % 2001u) - 1000) * 1e-3f : 1.0f;
        }
    bf16x8_hw_t a[2], b[2], unused;
#pragma unroll
    for (int q = 0; q < 2; ++q) {
        split2_bf16(fa[q], a[q], unused);
        split2_bf16(fb[q], b[q], unused);
    }
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int i = 0; i < 8; ++i) acc[i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[i & 1], b[i & 1], acc[i], 0, 0, 0);
    }
    float s = 0.0f;
#pragma unroll
    for (int i = 0; i < 8; ++i)
#pragma unroll
        for (int v = 0; v < 16; ++v) s += acc[i][v];
    out[(size_t)blockIdx.x * blockDim.x + threadIdx.x] = s;
}

extern "C" int moe_microbench_mfma_bf16(int32_t n_workgroups, int32_t iters, int32_t random_operands, float* out,
                                        void* stream) {
    if (!out) return MOE_ERR_NULL;
    if (n_workgroups < 1 || n_workgroups > 65536 || iters < 1) return MOE_ERR_SHAPE;
    mfma_rate_kernel<<<n_workgroups, 256, 0, (hipStream_t)stream>>>(iters, random_operands, out);
    return launch_status();
}
