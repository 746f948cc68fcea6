// Activation quantizer (Eq.2), power-of-two calibration, and the 4-bit weight
// blob (pack / unpack).  All of these are bandwidth-trivial helper kernels:
// 16-byte loads per lane, no LDS.
#include "agq_device.h"
#include "agq_internal.h"

#include <math.h>

namespace {

constexpr int kThreads = 256;

// ------------------------------------------------------------------ calibrate

__global__ void calib_init_kernel(int32_t *e_dev) { *e_dev = 0; }

// max over the tensor of the fp16 magnitude bits (sign cleared); the bit
// patterns of non-negative fp16 order like unsigned integers
__global__ __launch_bounds__(kThreads) void calib_absmax_kernel(const __half *__restrict__ x, int64_t M,
                                                                 int64_t K8, int64_t ldx, uint32_t *amax_bits) {
    uint32_t m = 0;
    const int64_t total = M * K8;
    for (int64_t i = (int64_t)blockIdx.x * kThreads + threadIdx.x; i < total; i += (int64_t)gridDim.x * kThreads) {
        const int64_t r = i / K8, c = i - r * K8;
        const uint4 v = *reinterpret_cast<const uint4 *>(x + r * ldx + c * 8);
        const uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const uint32_t a = w[j] & 0x7FFF7FFFu;
            m = max(m, max(a & 0xFFFFu, a >> 16));
        }
    }
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) m = max(m, (uint32_t)__shfl_xor((int)m, off));
    if ((threadIdx.x & 63) == 0 && m) atomicMax(amax_bits, m);
}

// smallest e with amax <= qmax * 2^e, by the predicate itself
__global__ void calib_final_kernel(int32_t *e_dev, int qmax) {
    const uint32_t bits = (uint32_t)*e_dev;
    int e = 0;
    if (bits != 0) {
        const float amax = bits >= 0x7C00u ? 65536.0f : __half2float(__ushort_as_half((unsigned short)bits));
        e = -64;
        while (amax > ldexpf((float)qmax, e)) ++e;
    }
    *e_dev = e;
}

// ------------------------------------------------------------------ quantize

// one lane = eight consecutive k of one row.  out_bits = 8: one byte per code;
// out_bits = 4: two codes per byte, low nibble = even k.
template <int OUT_BITS>
__global__ __launch_bounds__(kThreads) void quantize_kernel(const __half *__restrict__ x, int64_t M, int64_t K8,
                                                             int64_t ldx, AgqQuant q, uint8_t *__restrict__ out,
                                                             int64_t ld_out_bytes) {
    const int64_t i = (int64_t)blockIdx.x * kThreads + threadIdx.x;
    if (i >= M * K8) return;
    const int64_t r = i / K8, c = i - r * K8;
    const uint4 v = *reinterpret_cast<const uint4 *>(x + r * ldx + c * 8);
    const uint2 b = agq_quant8<true>(v, q);
    if (OUT_BITS == 8) {
        *reinterpret_cast<uint2 *>(out + r * ld_out_bytes + c * 8) = b;
    } else {
        // bytes k0..k3 in b.x, k4..k7 in b.y -> nibbles
        uint32_t lo = b.x & 0x0F0F0F0Fu, hi = b.y & 0x0F0F0F0Fu;
        uint32_t n0 = (lo & 0xF) | ((lo >> 4) & 0xF0) | ((lo >> 8) & 0xF00) | ((lo >> 12) & 0xF000);
        uint32_t n1 = (hi & 0xF) | ((hi >> 4) & 0xF0) | ((hi >> 8) & 0xF00) | ((hi >> 12) & 0xF000);
        *reinterpret_cast<uint32_t *>(out + r * ld_out_bytes + c * 4) = n0 | (n1 << 16);
    }
}

// ------------------------------------------------------------------ activation tiles for the MFMA kernel
//
// The tiled GEMM reads its activation codes from a private int8 copy laid out in
// MFMA operand order, so that its global-to-LDS copies are contiguous 1 KiB runs
// and its fragment reads are linear.  For every 128-token tile and every K step
// of 128 there is one 16 KiB stage [i (4)][t (4)][lane (64)][16 bytes]: i = which
// 32-token tile, t = which k-block of 32, lane = 32 (k-half of 16) + token % 32,
// the 16 bytes = 16 consecutive k.  One workgroup produces the 4 KiB of one
// (32-token tile, K step): coalesced row-major loads, Eq.2 (or a plain copy /
// nibble widening for pre-quantized input), a transpose through LDS, and a
// linear 16-byte-per-lane store.  Rows past M are written as zeros.
enum { PRE_F16 = 0, PRE_I8 = 1, PRE_I4 = 2 };

template <int MODE>
__global__ __launch_bounds__(kThreads) void prepack_act_kernel(const void *__restrict__ x, int64_t M, int64_t KT,
                                                                int64_t ldx, AgqQuant q, uint32_t flip,
                                                                uint4 *__restrict__ out) {
    __shared__ uint4 tile[256];                       // 4 KiB in operand order
    const int tid = threadIdx.x;
    const int64_t kt = blockIdx.x, mt = blockIdx.y;  // K step, 32-token tile
    const int r = tid >> 3, c = tid & 7;              // token row in the tile, 16-wide k segment
    const int64_t m = mt * 32 + r;
    uint4 codes = make_uint4(0, 0, 0, 0);
    if (m < M) {
        const int64_t k0 = kt * 128 + c * 16;
        // `flip` is non-zero for the unsigned grid: stored codes q become q - 2^(b-1)
        if (MODE == PRE_F16) {
            const __half *xp = reinterpret_cast<const __half *>(x) + m * ldx + k0;
            const uint2 lo = agq_quant8<true>(*reinterpret_cast<const uint4 *>(xp), q);
            const uint2 hi = agq_quant8<true>(*reinterpret_cast<const uint4 *>(xp + 8), q);
            codes = make_uint4(lo.x, lo.y, hi.x, hi.y);
        } else if (MODE == PRE_I8) {
            codes = *reinterpret_cast<const uint4 *>(reinterpret_cast<const int8_t *>(x) + m * ldx + k0);
            codes.x ^= flip;
            codes.y ^= flip;
            codes.z ^= flip;
            codes.w ^= flip;
        } else {
            const uint2 v = *reinterpret_cast<const uint2 *>(reinterpret_cast<const uint8_t *>(x) + m * (ldx >> 1) + (k0 >> 1));
            const uint32_t w[2] = {v.x ^ flip, v.y ^ flip};
            uint32_t o[4];
#pragma unroll
            for (int j = 0; j < 2; ++j)
#pragma unroll
                for (int h = 0; h < 2; ++h) {
                    const uint32_t four = (w[j] >> (16 * h)) & 0xFFFFu;
                    uint32_t r4 = 0;
#pragma unroll
                    for (int t = 0; t < 4; ++t) {
                        const int code = (int)((four >> (4 * t)) & 0xF);
                        r4 |= (uint32_t)(((code ^ 8) - 8) & 0xFF) << (8 * t);
                    }
                    o[2 * j + h] = r4;
                }
            codes = make_uint4(o[0], o[1], o[2], o[3]);
        }
    }
    tile[(c >> 1) * 64 + (c & 1) * 32 + r] = codes;   // k-block c >> 1, lane 32 (c & 1) + r
    __syncthreads();
    // stage of (128-token tile mt >> 2, step kt); this workgroup owns chunks 4 (mt & 3) .. + 3
    out[(((mt >> 2) * KT + kt) * 16 + (mt & 3) * 4) * 64 + tid] = tile[tid];
}

// ------------------------------------------------------------------ weight blob
//
// The blob is an array of 1 KiB chunks, chunk (nt, kt) at index nt * KT + kt,
// nt = 16-row tile of output channels, kt = 128-wide tile of K.  Inside a chunk
// lane l of a wavefront owns bytes [16 l, 16 l + 16): output channel
// n = 16 nt + (l & 15), k-group g = l >> 4.  Byte j of word d of that lane holds
//   low  nibble: W[n, 128 kt +      16 g + 4 d + j]   (MFMA step 0)
//   high nibble: W[n, 128 kt + 64 + 16 g + 4 d + j]   (MFMA step 1)
// so that one coalesced 16-byte load per lane feeds two 16x16x64 int8 MFMAs
// whose other operand is 16 consecutive activation codes.  Rows are padded with
// zero weights up to a multiple of 256.

__global__ __launch_bounds__(kThreads) void pack_kernel(const int8_t *__restrict__ wq, int64_t N, int64_t K,
                                                         int64_t KT, int64_t total_words, uint32_t *__restrict__ blob,
                                                         int32_t *bad) {
    const int64_t i = (int64_t)blockIdx.x * kThreads + threadIdx.x;
    if (i >= total_words) return;
    const int64_t chunk = i >> 8;
    const int within = (int)(i & 255), lane = within >> 2, d = within & 3;
    const int64_t nt = chunk / KT, kt = chunk - nt * KT;
    const int64_t n = nt * 16 + (lane & 15);
    uint32_t word = 0;
    int nbad = 0;
    if (n < N) {
        const int64_t k0 = kt * 128 + (lane >> 4) * 16 + 4 * d;
        const uint32_t lo = *reinterpret_cast<const uint32_t *>(wq + n * K + k0);
        const uint32_t hi = *reinterpret_cast<const uint32_t *>(wq + n * K + k0 + 64);
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            int a = (int)(int8_t)(lo >> (8 * j)), b = (int)(int8_t)(hi >> (8 * j));
            const int as = min(max(a, -8), 7), bs = min(max(b, -8), 7);
            nbad += (as != a) + (bs != b);
            word |= (uint32_t)((as & 0xF) | ((bs & 0xF) << 4)) << (8 * j);
        }
    }
    blob[i] = word;
    if (nbad && bad) atomicAdd(bad, nbad);
}

__global__ __launch_bounds__(kThreads) void unpack_kernel(const uint32_t *__restrict__ blob, int64_t N, int64_t K,
                                                           int64_t KT, int8_t *__restrict__ wq) {
    const int64_t i = (int64_t)blockIdx.x * kThreads + threadIdx.x;  // one lane = 4 consecutive k of one row
    const int64_t K4 = K >> 2;
    if (i >= N * K4) return;
    const int64_t n = i / K4, k0 = (i - n * K4) * 4;
    const int64_t kt = k0 >> 7;
    const int rem = (int)(k0 & 127), s = rem >> 6, g = (rem & 63) >> 4, d = (rem & 15) >> 2;
    const int lane = g * 16 + (int)(n & 15);
    const uint32_t word = blob[(((n >> 4) * KT + kt) * 64 + lane) * 4 + d];
    uint32_t o = 0;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        const int code = (int)((word >> (8 * j + 4 * s)) & 0xF);
        o |= (uint32_t)(((code ^ 8) - 8) & 0xFF) << (8 * j);
    }
    *reinterpret_cast<uint32_t *>(wq + n * K + k0) = o;
}

// Sum of the (saturated) 4-bit weights of every output channel, padded channels 0:
// the term the asymmetric activation grid needs, one wavefront per channel.
__global__ __launch_bounds__(64) void wsum_kernel(const int8_t *__restrict__ wq, int64_t N, int64_t K,
                                                   int32_t *__restrict__ wsum) {
    const int64_t n = blockIdx.x;
    int sum = 0;
    if (n < N) {
        const uint32_t *row = reinterpret_cast<const uint32_t *>(wq + n * K);
        for (int64_t i = threadIdx.x; i < (K >> 2); i += 64) {
            const uint32_t w = row[i];
#pragma unroll
            for (int j = 0; j < 4; ++j) sum += min(max((int)(int8_t)(w >> (8 * j)), -8), 7);
        }
    }
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) sum += __shfl_down(sum, off);
    if (threadIdx.x == 0) wsum[n] = sum;
}

inline int64_t blocks_for(int64_t n) { return (n + kThreads - 1) / kThreads; }

}  // namespace

AgqQuant agq_make_quant(int bits, int e, int zp) {
    const int lo = zp == 0 ? -(1 << (bits - 1)) : 0;
    const int hi = zp == 0 ? (1 << (bits - 1)) - 1 : (1 << bits) - 1;
    AgqQuant q;
    q.scale = ldexpf(1.0f, -e);
    q.lo = AGQ_MAGIC + (float)(lo - zp);
    q.hi = AGQ_MAGIC + (float)(hi - zp);
    q.zp = zp;
    q.h_scale2 = q.h_lo2 = q.h_hi2 = q.h_zp2 = 0;   // the packed fp16 form serves the GEMM prologues only
    return q;
}

// Quantizer of the GEMM prologues: codes on the signed grid [-2^(b-1), 2^(b-1)-1]
// that the int8 MFMA takes.  zp == 0: Eq.1's signed grid as it is.  zp > 0: Eq.2's
// unsigned code minus 2^(b-1), i.e. the signed grid with zero point zp - 2^(b-1).
AgqQuant agq_make_quant_signed(int bits, int e, int zp) {
    const int lo = -(1 << (bits - 1)), hi = (1 << (bits - 1)) - 1;
    const int off = zp ? zp - (1 << (bits - 1)) : 0;
    AgqQuant q;
    q.scale = ldexpf(1.0f, -e);
    q.lo = AGQ_MAGIC + (float)(lo - off);
    q.hi = AGQ_MAGIC + (float)(hi - off);
    q.zp = off;
    // fp16 images: 2^-e has exponent field 15 - e, a normal number for 1 <= 15 - e <= 30;
    // the bounds carry the rounding constant 1536: integers in [1281, 1790], exact in fp16
    auto pair = [](uint32_t h) { return h | (h << 16); };
    const int field = 15 - e;
    q.h_scale2 = (field >= 1 && field <= 30) ? pair((uint32_t)field << 10) : 0u;
    q.h_lo2 = pair((uint32_t)__half_as_ushort(__float2half((float)(1536 + lo - off))));
    q.h_hi2 = pair((uint32_t)__half_as_ushort(__float2half((float)(1536 + hi - off))));
    q.h_zp2 = pair((uint32_t)(off & 0xFF));
    return q;
}

int agq_launch_calibrate(const void *x, int64_t M, int64_t K, int64_t ldx, int bits, int32_t *e_dev, void *stream) {
    hipStream_t st = (hipStream_t)stream;
    calib_init_kernel<<<1, 1, 0, st>>>(e_dev);
    const int64_t total = M * (K / 8);
    if (total > 0) {
        const int64_t nb = blocks_for(total);
        calib_absmax_kernel<<<(unsigned)(nb < 2048 ? nb : 2048), kThreads, 0, st>>>((const __half *)x, M, K / 8, ldx,
                                                                                   (uint32_t *)e_dev);
    }
    calib_final_kernel<<<1, 1, 0, st>>>(e_dev, (1 << (bits - 1)) - 1);
    return (int)hipGetLastError();
}

int agq_launch_quantize(const void *x, int64_t M, int64_t K, int64_t ldx, int bits, int e, int zp, void *out,
                        int64_t ld_out_bytes, int out_bits, void *stream) {
    const int64_t total = M * (K / 8);
    if (total == 0) return 0;
    const AgqQuant q = agq_make_quant(bits, e, zp);
    hipStream_t st = (hipStream_t)stream;
    if (out_bits == 8)
        quantize_kernel<8><<<(unsigned)blocks_for(total), kThreads, 0, st>>>((const __half *)x, M, K / 8, ldx, q,
                                                                             (uint8_t *)out, ld_out_bytes);
    else
        quantize_kernel<4><<<(unsigned)blocks_for(total), kThreads, 0, st>>>((const __half *)x, M, K / 8, ldx, q,
                                                                             (uint8_t *)out, ld_out_bytes);
    return (int)hipGetLastError();
}

int agq_launch_prepack_act(const void *x, int x_kind, int bits, int64_t M, int64_t K, int64_t ldx, int e, int zp,
                           void *out, void *stream) {
    const AgqQuant q = agq_make_quant_signed(bits, e, zp);
    const uint32_t flip = zp ? (bits == 8 ? 0x80808080u : 0x88888888u) : 0u;
    const int64_t KT = K / 128;
    const dim3 grid((unsigned)KT, (unsigned)(((M + 127) / 128) * 4));
    hipStream_t st = (hipStream_t)stream;
    if (x_kind == 0)
        prepack_act_kernel<PRE_F16><<<grid, kThreads, 0, st>>>(x, M, KT, ldx, q, flip, (uint4 *)out);
    else if (bits == 8)
        prepack_act_kernel<PRE_I8><<<grid, kThreads, 0, st>>>(x, M, KT, ldx, q, flip, (uint4 *)out);
    else
        prepack_act_kernel<PRE_I4><<<grid, kThreads, 0, st>>>(x, M, KT, ldx, q, flip, (uint4 *)out);
    return (int)hipGetLastError();
}

int agq_launch_pack(const int8_t *wq, int64_t N, int64_t K, void *packed, int32_t *bad, void *stream) {
    const int64_t KT = agq_k_tiles(K);
    const int64_t total_words = agq_n_tiles_padded(N) * KT * 256;
    pack_kernel<<<(unsigned)blocks_for(total_words), kThreads, 0, (hipStream_t)stream>>>(wq, N, K, KT, total_words,
                                                                                         (uint32_t *)packed, bad);
    wsum_kernel<<<(unsigned)(agq_n_tiles_padded(N) * 16), 64, 0, (hipStream_t)stream>>>(
        wq, N, K, const_cast<int32_t *>(agq_blob_wsum(packed, N, K)));
    return (int)hipGetLastError();
}

int agq_launch_unpack(const void *packed, int64_t N, int64_t K, int8_t *wq, void *stream) {
    const int64_t total = N * (K / 4);
    unpack_kernel<<<(unsigned)blocks_for(total), kThreads, 0, (hipStream_t)stream>>>((const uint32_t *)packed, N, K,
                                                                                     agq_k_tiles(K), wq);
    return (int)hipGetLastError();
}
