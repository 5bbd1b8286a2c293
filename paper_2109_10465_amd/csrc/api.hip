// Host-only entry points of the C ABI: capacity rule, workspace size, status names.
#include <math.h>
#include "moe_common.h"

extern "C" const char* moe_status_string(int status) {
    switch (status) {
        case MOE_OK: return "ok";
        case MOE_ERR_NULL: return "a required pointer is NULL";
        case MOE_ERR_SHAPE: return "shape outside the supported limits";
        case MOE_ERR_DTYPE: return "unknown dtype or activation";
        case MOE_ERR_WORKSPACE: return "workspace NULL, misaligned or too small";
        case MOE_ERR_LAUNCH: return "the HIP runtime refused a kernel launch";
        default: return "unknown status";
    }
}

// Slots per expert: max(1, ceil(k * cf * T / E))  (Sec. 5.1 capacity factor).
extern "C" int32_t moe_capacity(int32_t T, int32_t E, int32_t k, double capacity_factor) {
    if (T < 1 || E < 1 || k < 1 || k > 2 || !(capacity_factor > 0.0)) return -1;
    const double c = ceil((double)k * capacity_factor * (double)T / (double)E);
    if (c >= 2147483647.0) return -1;
    return c < 1.0 ? 1 : (int32_t)c;
}

extern "C" size_t moe_workspace_bytes(const moe_shape* shape) {
    if (check_shape(shape) != MOE_OK) return 0;
    size_t n = route_ws_bytes(shape);
    const size_t b = ffn_bwd_ws_bytes(shape), c = gate_logits_bwd_ws_bytes(shape);
    if (b > n) n = b;
    if (c > n) n = c;
    const size_t a = aux_loss_ws_bytes(shape);
    if (a > n) n = a;
    return n;
}
