// tw_tree_verify_attn_static: tree verification for callers that can neither allocate device
// memory nor own a workspace.  The scratch that a split launch needs (arrival counters and the
// partial results of the pieces) lives in a file-scope device array; every GPU the library runs on
// holds its own copy of it until the process ends.
#include "twig_internal.h"

namespace {

// One copy per device.  In host code this name is only a handle for hipGetSymbolAddress; the
// device address it stands for is looked up once per device and kept in g_scratch.
static __device__ __align__(256) unsigned char scratch[TW_STATIC_SCRATCH_BYTES];

constexpr int kMaxDevices = 64;
std::atomic<void*> g_scratch[kMaxDevices];

// Device address of the current device's copy of the array.
hipError_t scratch_address(void** out) {
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    if (dev >= 0 && dev < kMaxDevices) {
        void* p = g_scratch[dev].load(std::memory_order_acquire);
        if (p) {
            *out = p;
            return hipSuccess;
        }
    }
    void* p = nullptr;
    e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
    if (e != hipSuccess) return e;
    if (!p) return hipErrorInvalidSymbol;
    if (dev >= 0 && dev < kMaxDevices) g_scratch[dev].store(p, std::memory_order_release);
    *out = p;
    return hipSuccess;
}

}  // namespace

extern "C" int32_t tw_tree_verify_attn_static(const void* q, const tw_kv_view* k, const tw_kv_view* v,
                                              const int32_t* ctx_len, int32_t max_ctx_len, const int32_t* parent,
                                              const int32_t* n_nodes, int32_t T_max, int32_t B, float scale, void* out,
                                              int32_t out_dtype, void* stream) {
    // the size check needs the head count; everything else is validated by the call below
    if (!k || k->H <= 0 || k->d_h <= 0 || B < 0 || T_max < 1 || max_ctx_len < 0) return TW_ERR_INVALID_ARG;
    if (T_max > TW_MAX_TREE || (int64_t)max_ctx_len + T_max > (1ll << 30)) return TW_ERR_UNSUPPORTED;
    const size_t need = tw_workspace_bytes(TW_CALL_TREE_VERIFY_ATTN, B, T_max, k->H, k->d_h, max_ctx_len + T_max);
    if (need > TW_STATIC_SCRATCH_BYTES) return TW_ERR_WORKSPACE;
    void* ws = nullptr;
    if (need > 0 && scratch_address(&ws) != hipSuccess) return TW_ERR_LAUNCH;
    return tw_tree_verify_attn(q, k, v, ctx_len, max_ctx_len, parent, n_nodes, T_max, B, scale, out, out_dtype, ws,
                               need > 0 ? (size_t)TW_STATIC_SCRATCH_BYTES : 0, stream);
}
