// agq_gemm_w4a8_static: agq_gemm_w4a8 for callers that cannot allocate device memory (code under HIP graph
// capture, serving loops, harnesses that forbid hipMalloc).  The workspace of the tiled path (the activation
// codes in operand order and, behind them, the int32 partial tiles of a K split) is a fixed array in the
// library's own device image instead of a caller buffer.
#include <hip/hip_runtime.h>
#include <mutex>

#include "../../include/agq.h"
#include "agq_internal.h"

namespace {

// One copy per GPU the library runs on, held until the process ends.  In host code this name is only a handle
// for hipGetSymbolAddress: the kernels receive the address that call returns for the current device.
static __device__ __align__(256) unsigned char scratch[AGQ_STATIC_WORKSPACE_BYTES];

constexpr int kMaxDevices = 64;
void *g_scratch_ptr[kMaxDevices];   // device address of `scratch` on each GPU, looked up on first use
std::mutex g_scratch_mu;

int scratch_of_current_device(void **out) {
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return AGQ_EHIP;
    std::lock_guard<std::mutex> lock(g_scratch_mu);
    if (!g_scratch_ptr[dev]) {
        void *p = nullptr;
        if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) return AGQ_EHIP;
        g_scratch_ptr[dev] = p;
    }
    *out = g_scratch_ptr[dev];
    return AGQ_OK;
}

}  // namespace

extern "C" int agq_gemm_w4a8_static(const void *x, int x_kind, int64_t M, int64_t K, int64_t ldx, int e, int zp,
                                    const void *w_packed, const void *w_scale_f16, int64_t N, void *y_f16, int64_t ldy,
                                    int32_t *acc_out, void *stream) {
    const agq_proj one = {w_packed, w_scale_f16, N, y_f16, ldy, acc_out};
    // every argument error, a size beyond the array included, is reported before the first HIP call
    // (the stand-in address is only compared against NULL and checked for alignment)
    void *ws = reinterpret_cast<void *>(static_cast<uintptr_t>(256));
    int st = agq_gemm_w4_run(8, x, x_kind, M, K, ldx, e, zp, &one, 1, ws, AGQ_STATIC_WORKSPACE_BYTES, stream, true);
    if (st != AGQ_OK || M == 0) return st;
    st = scratch_of_current_device(&ws);
    if (st != AGQ_OK) return st;
    // Nothing in the array has to start at zero: the pre-pass writes every code (padding rows of the last token
    // tile included) and every partial tile is stored whole before the reduction reads it.
    return agq_gemm_w4_run(8, x, x_kind, M, K, ldx, e, zp, &one, 1, ws, AGQ_STATIC_WORKSPACE_BYTES, stream, false);
}
