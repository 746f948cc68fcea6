// The fp16 operators that Section 4.2's pipeline leaves unquantized, for a LLaMA
// block: RMS normalisation (optionally fused with the residual addition and the
// row gather that follows token pruning), the rotary embedding fused with Eq.2 for
// q, k and v, SwiGLU, and the residual addition.  Each takes fp16 tensors and
// returns fp16 (or Eq.2 codes); the arithmetic in between is float64 with one
// rounding to fp16 at the end, so that a result does not depend on the order of a
// reduction or on the exponential's implementation beyond the last bit of a double.
// All of them stream their operands once: they are bound by HBM.
#include "agq_device.h"
#include "agq_internal.h"

namespace {

// float64 -> fp16, round to nearest even in ONE step.  The hardware converts
// f64 -> f32 and f32 -> f16; rounding twice to nearest can differ from rounding
// once, so the first step is turned into round-to-odd (truncate, then set the last
// bit when anything was cut off), after which the second rounding is exact: 24
// bits keep two more than the 11 of the target.
__device__ __forceinline__ __half f64_to_f16(double d) {
    float f = (float)d;
    const double back = (double)f;
    if (back != d && fabsf(f) <= 3.0e38f) {   // inexact and not overflowed (NaN compares false)
        uint32_t u = __float_as_uint(f);
        if (fabs(back) > fabs(d)) u -= 1;     // nearest went away from zero: step back to the truncation
        f = __uint_as_float(u | 1u);
    }
    return __float2half_rn(f);
}
__device__ __forceinline__ double h2d(uint16_t h) { return (double)__half2float(__ushort_as_half(h)); }
__device__ __forceinline__ uint16_t d2h(double d) { return __half_as_ushort(f64_to_f16(d)); }

struct Half8 {
    uint16_t v[8];
};
static_assert(sizeof(Half8) == 16, "eight fp16 are one 16-byte access");
__device__ __forceinline__ Half8 load8(const void *p) { return __builtin_bit_cast(Half8, *reinterpret_cast<const uint4 *>(p)); }
__device__ __forceinline__ void store8(void *p, const Half8 &h) { *reinterpret_cast<uint4 *>(p) = __builtin_bit_cast(uint4, h); }

constexpr int kNormThreads = 256;
constexpr int kNormCache = 4;   // rows up to 4 * 256 * 8 = 8192 elements stay in registers between the two passes

// y[r,:] = x1[r,:] * g / sqrt(mean(x1[r,:]^2) + eps), x1 = x (ADD == false) or
// fp16(res[idx[r],:] + x[r,:]) (ADD == true, x1 also written out, with the positions
// of the surviving rows).
template <bool ADD>
__global__ __launch_bounds__(kNormThreads) void rmsnorm_kernel(const uint16_t *__restrict__ x, const uint16_t *__restrict__ res,
                                                              const int32_t *__restrict__ idx, const uint16_t *__restrict__ g,
                                                              uint16_t *__restrict__ x1_out, uint16_t *__restrict__ y, int d,
                                                              double eps, const int32_t *__restrict__ pos,
                                                              int32_t *__restrict__ pos_out, int32_t *__restrict__ idx_out) {
    const int r = blockIdx.x, tid = threadIdx.x;
    const int src = (ADD && idx) ? idx[r] : r;
    const uint16_t *xr = x + (size_t)r * d;
    const uint16_t *rr = ADD ? res + (size_t)src * d : nullptr;
    if (ADD && tid == 0) {
        if (pos_out) pos_out[r] = pos[src];
        if (idx_out) idx_out[r] = src;
    }
    Half8 cache[kNormCache];
    double ss = 0.0;
    const int nchunk = d >> 3;
#pragma unroll
    for (int it = 0; it < kNormCache; ++it) {
        const int c = tid + it * kNormThreads;
        if (c < nchunk) {
            Half8 h = load8(xr + c * 8);
            if (ADD) {
                const Half8 b = load8(rr + c * 8);
#pragma unroll
                for (int i = 0; i < 8; ++i) h.v[i] = d2h(h2d(b.v[i]) + h2d(h.v[i]));
                store8(x1_out + (size_t)r * d + c * 8, h);
            }
            cache[it] = h;
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                const double v = h2d(h.v[i]);
                ss += v * v;
            }
        }
    }
    for (int c = tid + kNormCache * kNormThreads; c < nchunk; c += kNormThreads) {   // rows wider than the cache
        Half8 h = load8(xr + c * 8);
        if (ADD) {
            const Half8 b = load8(rr + c * 8);
#pragma unroll
            for (int i = 0; i < 8; ++i) h.v[i] = d2h(h2d(b.v[i]) + h2d(h.v[i]));
            store8(x1_out + (size_t)r * d + c * 8, h);
        }
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            const double v = h2d(h.v[i]);
            ss += v * v;
        }
    }
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) ss += __shfl_xor(ss, o);
    __shared__ double part[kNormThreads / 64];
    if ((tid & 63) == 0) part[tid >> 6] = ss;
    __syncthreads();
    double tot = 0.0;
#pragma unroll
    for (int w = 0; w < kNormThreads / 64; ++w) tot += part[w];
    const double inv = 1.0 / sqrt(tot / (double)d + eps);
    const uint16_t *src1 = ADD ? x1_out + (size_t)r * d : xr;   // this thread re-reads only what it wrote itself
#pragma unroll
    for (int it = 0; it < kNormCache; ++it) {
        const int c = tid + it * kNormThreads;
        if (c < nchunk) {
            const Half8 gg = load8(g + c * 8);
            Half8 o;
#pragma unroll
            for (int i = 0; i < 8; ++i) o.v[i] = d2h((h2d(cache[it].v[i]) * h2d(gg.v[i])) * inv);
            store8(y + (size_t)r * d + c * 8, o);
        }
    }
    for (int c = tid + kNormCache * kNormThreads; c < nchunk; c += kNormThreads) {
        const Half8 h = load8(src1 + c * 8), gg = load8(g + c * 8);
        Half8 o;
#pragma unroll
        for (int i = 0; i < 8; ++i) o.v[i] = d2h((h2d(h.v[i]) * h2d(gg.v[i])) * inv);
        store8(y + (size_t)r * d + c * 8, o);
    }
}

// Eq.2 on one fp16 value, signed 8-bit grid, step 2^e (inv = 2^-e): the product is
// exact in fp32, the rounding is to nearest even.
__device__ __forceinline__ uint32_t quant8_1(uint16_t h, float inv) {
    const float r = rintf(__half2float(__ushort_as_half(h)) * inv);
    return (uint32_t)(int)fminf(fmaxf(r, -128.0f), 127.0f) & 0xFFu;
}
__device__ __forceinline__ uint2 quant8_8(const Half8 &h, float inv) {
    uint2 o;
    o.x = quant8_1(h.v[0], inv) | (quant8_1(h.v[1], inv) << 8) | (quant8_1(h.v[2], inv) << 16) | (quant8_1(h.v[3], inv) << 24);
    o.y = quant8_1(h.v[4], inv) | (quant8_1(h.v[5], inv) << 8) | (quant8_1(h.v[6], inv) << 16) | (quant8_1(h.v[7], inv) << 24);
    return o;
}

struct RopeArgs {
    const uint16_t *src[3];   // q, k, v: fp16 [S, H*D]
    int8_t *dst_q[3];         // int8 [H, S_pad, D]            (QUANT)
    uint16_t *dst_h[2];       // rotated q, k: fp16 [S, H*D]   (!QUANT)
    float inv[3];             // 2^-e of q, k, v
    const int32_t *pos;
    const float *cos_t, *sin_t;   // float32 [P, D/2]
    int S, S_pad, H, D, P;
    int32_t *zero;            // optional int32 [S_pad] cleared on the way (the importance score accumulates)
};

// blockIdx.x = token row (0 .. S_pad-1), blockIdx.y = tensor (0 q, 1 k, 2 v).  A work
// item is eight pairs (i, i + D/2) of one head: two 16-byte loads, rotation by the
// angles of (pos[row], i) for q and k, then either Eq.2 and the head-major int8 store
// or the rotated fp16 values (the calibration pass needs those).
template <bool QUANT>
__global__ __launch_bounds__(256) void rope_kernel(const RopeArgs a) {
    const int row = blockIdx.x, t = blockIdx.y;
    const int D = a.D, Dh = D >> 1, per_head = D >> 4;
    const int items = a.H * per_head;
    const bool pad = row >= a.S;
    if (QUANT && a.zero && t == 0 && threadIdx.x == 0) a.zero[row] = 0;
    const int p = pad ? 0 : min(max(a.pos[row], 0), a.P - 1);   // a position outside the table is clamped into it
    // selects instead of indexing with t: the argument record stays in scalar registers
    const uint16_t *src = (t == 0 ? a.src[0] : t == 1 ? a.src[1] : a.src[2]) + (size_t)row * a.H * D;
    const float inv = t == 0 ? a.inv[0] : t == 1 ? a.inv[1] : a.inv[2];
    for (int it = threadIdx.x; it < items; it += 256) {
        const int head = it / per_head, j = (it - head * per_head) * 8;
        uint2 qlo = make_uint2(0u, 0u), qhi = make_uint2(0u, 0u);
        if (!pad) {
            Half8 lo = load8(src + head * D + j), hi = load8(src + head * D + Dh + j);
            if (t < 2) {
                const float4 c0 = *reinterpret_cast<const float4 *>(a.cos_t + (size_t)p * Dh + j);
                const float4 c1 = *reinterpret_cast<const float4 *>(a.cos_t + (size_t)p * Dh + j + 4);
                const float4 s0 = *reinterpret_cast<const float4 *>(a.sin_t + (size_t)p * Dh + j);
                const float4 s1 = *reinterpret_cast<const float4 *>(a.sin_t + (size_t)p * Dh + j + 4);
                const float cs[8] = {c0.x, c0.y, c0.z, c0.w, c1.x, c1.y, c1.z, c1.w};
                const float sn[8] = {s0.x, s0.y, s0.z, s0.w, s1.x, s1.y, s1.z, s1.w};
#pragma unroll
                for (int i = 0; i < 8; ++i) {
                    const double l = h2d(lo.v[i]), h = h2d(hi.v[i]), c = (double)cs[i], s = (double)sn[i];
                    lo.v[i] = d2h(l * c - h * s);
                    hi.v[i] = d2h(h * c + l * s);
                }
            }
            if (!QUANT) {
                if (t < 2) {
                    uint16_t *dh = (t == 0 ? a.dst_h[0] : a.dst_h[1]) + (size_t)row * a.H * D + head * D;
                    store8(dh + j, lo);
                    store8(dh + Dh + j, hi);
                }
                continue;
            }
            qlo = quant8_8(lo, inv);
            qhi = quant8_8(hi, inv);
        }
        if (QUANT) {
            int8_t *dst = (t == 0 ? a.dst_q[0] : t == 1 ? a.dst_q[1] : a.dst_q[2]) + ((size_t)head * a.S_pad + row) * D;
            *reinterpret_cast<uint2 *>(dst + j) = qlo;
            *reinterpret_cast<uint2 *>(dst + Dh + j) = qhi;
        }
    }
}

// a = silu(gate) * up, eight values per thread
__global__ __launch_bounds__(256) void swiglu_kernel(const uint16_t *__restrict__ gate, const uint16_t *__restrict__ up,
                                                     uint16_t *__restrict__ out, size_t nchunk) {
    const size_t c = (size_t)blockIdx.x * 256 + threadIdx.x;
    if (c >= nchunk) return;
    const Half8 g = load8(gate + c * 8), u = load8(up + c * 8);
    Half8 o;
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        const double z = h2d(g.v[i]);
        o.v[i] = d2h(z / (1.0 + exp(-z)) * h2d(u.v[i]));
    }
    store8(out + c * 8, o);
}

__global__ __launch_bounds__(256) void add_kernel(const uint16_t *__restrict__ a, const uint16_t *__restrict__ b,
                                                  uint16_t *__restrict__ out, size_t nchunk) {
    const size_t c = (size_t)blockIdx.x * 256 + threadIdx.x;
    if (c >= nchunk) return;
    const Half8 x = load8(a + c * 8), y = load8(b + c * 8);
    Half8 o;
#pragma unroll
    for (int i = 0; i < 8; ++i) o.v[i] = d2h(h2d(x.v[i]) + h2d(y.v[i]));
    store8(out + c * 8, o);
}

}  // namespace

int agq_launch_rmsnorm(const void *x, const void *res, const int32_t *idx, const void *g, void *x1_out, void *y, int64_t rows,
                       int64_t d, double eps, const int32_t *pos, int32_t *pos_out, int32_t *idx_out, void *stream) {
    if (rows == 0) return 0;
    hipStream_t st = (hipStream_t)stream;
    if (res)
        rmsnorm_kernel<true><<<(unsigned)rows, kNormThreads, 0, st>>>((const uint16_t *)x, (const uint16_t *)res, idx,
                                                                      (const uint16_t *)g, (uint16_t *)x1_out, (uint16_t *)y,
                                                                      (int)d, eps, pos, pos_out, idx_out);
    else
        rmsnorm_kernel<false><<<(unsigned)rows, kNormThreads, 0, st>>>((const uint16_t *)x, nullptr, nullptr, (const uint16_t *)g,
                                                                       nullptr, (uint16_t *)y, (int)d, eps, nullptr, nullptr,
                                                                       nullptr);
    return (int)hipGetLastError();
}

int agq_launch_rope(const void *q, const void *k, const void *v, int64_t S, int64_t S_pad, int64_t H, int64_t D,
                    const int32_t *pos, const float *cos_t, const float *sin_t, int64_t P, int e_q, int e_k, int e_v,
                    int8_t *q_q, int8_t *k_q, int8_t *v_q, void *q_rot, void *k_rot, int32_t *zero, void *stream) {
    if (q_q ? S_pad == 0 : S == 0) return 0;   // with S == 0 the padding rows are still cleared
    RopeArgs a;
    a.src[0] = (const uint16_t *)q; a.src[1] = (const uint16_t *)k; a.src[2] = (const uint16_t *)v;
    a.dst_q[0] = q_q; a.dst_q[1] = k_q; a.dst_q[2] = v_q;
    a.dst_h[0] = (uint16_t *)q_rot; a.dst_h[1] = (uint16_t *)k_rot;
    a.inv[0] = ldexpf(1.0f, -e_q); a.inv[1] = ldexpf(1.0f, -e_k); a.inv[2] = ldexpf(1.0f, -e_v);
    a.pos = pos; a.cos_t = cos_t; a.sin_t = sin_t;
    a.S = (int)S; a.S_pad = (int)S_pad; a.H = (int)H; a.D = (int)D; a.P = (int)P;
    a.zero = zero;
    hipStream_t st = (hipStream_t)stream;
    if (q_q)
        rope_kernel<true><<<dim3((unsigned)S_pad, 3), 256, 0, st>>>(a);
    else
        rope_kernel<false><<<dim3((unsigned)S, 2), 256, 0, st>>>(a);
    return (int)hipGetLastError();
}

int agq_launch_swiglu(const void *gate, const void *up, void *out, int64_t n, void *stream) {
    if (n == 0) return 0;
    const size_t nchunk = (size_t)n / 8;
    swiglu_kernel<<<(unsigned)((nchunk + 255) / 256), 256, 0, (hipStream_t)stream>>>((const uint16_t *)gate, (const uint16_t *)up,
                                                                                   (uint16_t *)out, nchunk);
    return (int)hipGetLastError();
}

int agq_launch_add(const void *a, const void *b, void *out, int64_t n, void *stream) {
    if (n == 0) return 0;
    const size_t nchunk = (size_t)n / 8;
    add_kernel<<<(unsigned)((nchunk + 255) / 256), 256, 0, (hipStream_t)stream>>>((const uint16_t *)a, (const uint16_t *)b,
                                                                                (uint16_t *)out, nchunk);
    return (int)hipGetLastError();
}

// blocking read of a few device words (calibration only)
int agq_read_i32(const int32_t *dev, int32_t *host, int n, void *stream) {
    hipError_t e = hipMemcpyAsync(host, dev, (size_t)n * sizeof(int32_t), hipMemcpyDeviceToHost, (hipStream_t)stream);
    if (e != hipSuccess) return (int)e;
    return (int)hipStreamSynchronize((hipStream_t)stream);
}
