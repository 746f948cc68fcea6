// Measurement aid for bench.py, built as its own small library (libagq_probe.so): not part of the product and
// not linked into libagq.so.  Two kernels that bound what one launch of a weight-streaming kernel can reach on
// the device at hand: a plain read of a buffer with the access pattern of the decode kernels (one coalesced
// 16-byte load per lane and KiB, every load of a workgroup requested before the first is used), and an empty
// kernel (the cost of a launch inside a replayed graph).
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace {

typedef unsigned int probe_u4 __attribute__((ext_vector_type(4)));
constexpr int kLoads = 4;        // 16-byte loads in flight per lane
constexpr int kThreads = 512;    // 32 KiB per workgroup: the weights of one 16-channel tile at K = 4096

__global__ __launch_bounds__(kThreads) void probe_read_kernel(const probe_u4 *src, size_t n16, uint32_t *sink) {
    const size_t base = (size_t)blockIdx.x * (kThreads * kLoads) + threadIdx.x;
    probe_u4 v[kLoads];
#pragma unroll
    for (int i = 0; i < kLoads; ++i) {
        const size_t at = base + (size_t)i * kThreads;
        v[i] = src[at < n16 ? at : n16 - 1];
    }
    uint32_t acc = 0;
#pragma unroll
    for (int i = 0; i < kLoads; ++i) acc ^= v[i][0] ^ v[i][1] ^ v[i][2] ^ v[i][3];
    // every lane's loads are needed by a store the compiler cannot rule out (it happens for one bit pattern)
    if (acc == 0x9e3779b9u) sink[threadIdx.x & 63] = acc;
}

__global__ void probe_empty_kernel() {}

// The int8 matrix instruction of the tiled kernel with no memory traffic at all: every lane loads four pairs of
// operand registers once (4 x 16 bytes each from `a` and `b`, the same 16 KiB for every workgroup) and then issues
// `reps` rounds of four independent 32 x 32 x 32 MFMAs, every one with another pair than the one before it, as in a
// GEMM.  What this measures is the rate the matrix cores sustain for given operand VALUES (the instruction stream
// is the same for all of them).
typedef int probe_v4i __attribute__((ext_vector_type(4)));
typedef int probe_v16i __attribute__((ext_vector_type(16)));

__global__ __launch_bounds__(256) void probe_mfma_kernel(const probe_v4i *a, const probe_v4i *b, int reps, uint32_t *sink) {
    probe_v4i av[4], bv[4];
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        av[j] = a[j * 256 + threadIdx.x];
        bv[j] = b[j * 256 + threadIdx.x];
    }
    probe_v16i acc[4];
#pragma unroll
    for (int j = 0; j < 4; ++j)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[j][r] = 0;
    for (int it = 0; it < reps; it += 4) {
#pragma unroll
        for (int u = 0; u < 4; ++u)
#pragma unroll
            for (int j = 0; j < 4; ++j)
                acc[j] = __builtin_amdgcn_mfma_i32_32x32x32_i8(av[j], bv[(j + u) & 3], acc[j], 0, 0, 0);
    }
    uint32_t x = 0;
#pragma unroll
    for (int j = 0; j < 4; ++j)
#pragma unroll
        for (int r = 0; r < 16; ++r) x ^= (uint32_t)acc[j][r];
    if (x == 0x9e3779b9u) sink[threadIdx.x & 63] = x;   // never, but the compiler cannot rule it out
}

}  // namespace

// src: device buffer of `bytes` bytes (a multiple of 16, at least 16), 16-byte aligned; sink: device, 256 bytes.
extern "C" int agq_probe_read(const void *src, size_t bytes, void *sink, void *stream) {
    if (!src || !sink || bytes < 16 || (bytes % 16) != 0) return -1;
    const size_t n16 = bytes / 16;
    const size_t per_wg = (size_t)kThreads * kLoads;
    probe_read_kernel<<<(unsigned)((n16 + per_wg - 1) / per_wg), kThreads, 0, (hipStream_t)stream>>>(
        (const probe_u4 *)src, n16, (uint32_t *)sink);
    return hipGetLastError() == hipSuccess ? 0 : -3;
}

extern "C" int agq_probe_empty(void *stream) {
    probe_empty_kernel<<<1, 64, 0, (hipStream_t)stream>>>();
    return hipGetLastError() == hipSuccess ? 0 : -3;
}

// `a`, `b`: 16 KiB each (4 x 256 lanes x 16 bytes of int8 operand values, device memory); `workgroups` of 256
// threads (four wavefronts, one per SIMD of a CU); `reps` (a multiple of four) rounds of four MFMAs per wavefront
// = 8 x 32^3 x reps operations each.
extern "C" int agq_probe_mfma_i8(const void *a, const void *b, int workgroups, int reps, void *sink, void *stream) {
    if (!a || !b || !sink || workgroups < 1 || reps < 4 || (reps & 3)) return -1;
    probe_mfma_kernel<<<(unsigned)workgroups, 256, 0, (hipStream_t)stream>>>((const probe_v4i *)a, (const probe_v4i *)b,
                                                                            reps, (uint32_t *)sink);
    return hipGetLastError() == hipSuccess ? 0 : -3;
}
