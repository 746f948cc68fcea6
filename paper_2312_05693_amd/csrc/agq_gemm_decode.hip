// Weight-streaming kernel of the quantized linear layer for a few tokens
// (M <= 16): the decode regime, bound by the HBM read of the 4-bit weights.
//
// One workgroup owns one 16-row tile of output channels and the whole K, so no
// partial sums ever leave the CU: its wavefronts split K, each streams its own
// contiguous run of 1 KiB weight chunks with one coalesced 16-byte load per
// lane, and a single LDS reduction joins them before the fused dequantisation.
// Eq.2 runs as a prologue: a wavefront quantizes exactly the slice of the
// activation it multiplies (M x 128 values per chunk) into a private LDS
// region laid out in MFMA operand order; rows beyond M are never written or
// read back into a stored result, because each MFMA output row depends on the
// matching operand row only.
#include "agq_device.h"
#include "agq_internal.h"

AgqQuant agq_make_quant(int bits, int e, int zp);

namespace {

constexpr int kGroup = 2;        // weight chunks (k-tiles of 128) per pipeline step
constexpr int kMaxWaves = 16;

struct DecodeArgs {
    const void *x;
    int64_t ldx;      // elements (fp16 / int8) or codes (nibbles)
    int M, N, K, KT;
    int kt_per_wave;
    AgqQuant q;
    const uint4 *blob;
    const __half *sw;
    __half *y;
    int64_t ldy;
    int32_t *acc_out;
    float scale_e;    // 2^e
};

enum { XK_F16 = 0, XK_I8 = 1, XK_I4 = 2 };

template <int XK>
__global__ __launch_bounds__(1024) void gemm_decode_kernel(const DecodeArgs a) {
    extern __shared__ __align__(16) unsigned char smem[];
    const int lane = threadIdx.x & 63;
    const int wave = threadIdx.x >> 6;
    const int nwaves = blockDim.x >> 6;
    const int nt = blockIdx.x;

    // LDS: per wave kGroup x 2 KiB of operand-ordered codes; the reduction
    // buffer reuses the same bytes once every wavefront has left its main loop
    uint4 *stage = reinterpret_cast<uint4 *>(smem) + wave * (kGroup * 128);
    agq_v4i *red = reinterpret_cast<agq_v4i *>(smem);

    const int kb = wave * a.kt_per_wave;
    const int ke = min(kb + a.kt_per_wave, a.KT);
    const uint4 *wptr = a.blob + ((int64_t)nt * a.KT) * 64 + lane;

    agq_v4i acc = {0, 0, 0, 0};
    const uint4 zero4 = make_uint4(0, 0, 0, 0);

    uint4 wc[kGroup], wn[kGroup];
#pragma unroll
    for (int i = 0; i < kGroup; ++i) wc[i] = (kb + i < ke) ? wptr[(int64_t)(kb + i) * 64] : zero4;

    const int arow = min(lane & 15, a.M - 1);   // operand row of this lane, clamped into the tensor
    const int ag = lane >> 4;

    for (int kt = kb; kt < ke; kt += kGroup) {
#pragma unroll
        for (int i = 0; i < kGroup; ++i) wn[i] = (kt + kGroup + i < ke) ? wptr[(int64_t)(kt + kGroup + i) * 64] : zero4;

        agq_v4i a0[kGroup], a1[kGroup];
        if (XK == XK_F16) {
            // Eq.2 on the M x (kGroup*128) slice: lane = 8 consecutive k of one row
            const __half *xh = reinterpret_cast<const __half *>(a.x);
            const int c = lane & 15, rr = lane >> 4;
            uint4 xv[kGroup][4];
#pragma unroll
            for (int i = 0; i < kGroup; ++i)
#pragma unroll
                for (int it = 0; it < 4; ++it) {
                    const int m = it * 4 + rr;
                    if (m < a.M && kt + i < ke)
                        xv[i][it] = *reinterpret_cast<const uint4 *>(xh + (int64_t)m * a.ldx + (int64_t)(kt + i) * 128 + c * 8);
                }
            const int s = c >> 3, g = (c & 7) >> 1, hf = c & 1;
#pragma unroll
            for (int i = 0; i < kGroup; ++i)
#pragma unroll
                for (int it = 0; it < 4; ++it) {
                    const int m = it * 4 + rr;
                    if (m < a.M && kt + i < ke) {
                        const uint2 b = agq_quant8(xv[i][it], a.q);
                        uint2 *dst = reinterpret_cast<uint2 *>(stage + i * 128 + s * 64 + g * 16 + m) + hf;
                        *dst = b;
                    }
                }
            // same wavefront wrote and reads: LDS keeps program order per wave
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
            __builtin_amdgcn_wave_barrier();
            __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
#pragma unroll
            for (int i = 0; i < kGroup; ++i) {
                const uint4 v0 = stage[i * 128 + lane], v1 = stage[i * 128 + 64 + lane];
                a0[i] = agq_v4i{(int)v0.x, (int)v0.y, (int)v0.z, (int)v0.w};
                a1[i] = agq_v4i{(int)v1.x, (int)v1.y, (int)v1.z, (int)v1.w};
            }
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
            __builtin_amdgcn_wave_barrier();
        } else if (XK == XK_I8) {
            const int8_t *xq = reinterpret_cast<const int8_t *>(a.x) + (int64_t)arow * a.ldx + ag * 16;
#pragma unroll
            for (int i = 0; i < kGroup; ++i) {
                uint4 v0 = zero4, v1 = zero4;
                if (kt + i < ke) {
                    v0 = *reinterpret_cast<const uint4 *>(xq + (int64_t)(kt + i) * 128);
                    v1 = *reinterpret_cast<const uint4 *>(xq + (int64_t)(kt + i) * 128 + 64);
                }
                a0[i] = agq_v4i{(int)v0.x, (int)v0.y, (int)v0.z, (int)v0.w};
                a1[i] = agq_v4i{(int)v1.x, (int)v1.y, (int)v1.z, (int)v1.w};
            }
        } else {
            // nibble codes, low nibble = even k: widen to 16 * code in k order
            const uint8_t *xq = reinterpret_cast<const uint8_t *>(a.x) + (int64_t)arow * (a.ldx >> 1) + ag * 8;
#pragma unroll
            for (int i = 0; i < kGroup; ++i) {
                uint2 p0 = make_uint2(0, 0), p1 = make_uint2(0, 0);
                if (kt + i < ke) {
                    p0 = *reinterpret_cast<const uint2 *>(xq + (int64_t)(kt + i) * 64);
                    p1 = *reinterpret_cast<const uint2 *>(xq + (int64_t)(kt + i) * 64 + 32);
                }
                const uint32_t pw[4] = {p0.x, p0.y, p1.x, p1.y};
                uint32_t o[8];
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    const uint32_t ev = (pw[j] << 4) & 0xF0F0F0F0u, od = pw[j] & 0xF0F0F0F0u;
                    o[2 * j] = __builtin_amdgcn_perm(od, ev, 0x05010400u);
                    o[2 * j + 1] = __builtin_amdgcn_perm(od, ev, 0x07030602u);
                }
                a0[i] = agq_v4i{(int)o[0], (int)o[1], (int)o[2], (int)o[3]};
                a1[i] = agq_v4i{(int)o[4], (int)o[5], (int)o[6], (int)o[7]};
            }
        }

#pragma unroll
        for (int i = 0; i < kGroup; ++i) {
            agq_v4i b0, b1;
            agq_unpack_w(wc[i], b0, b1);
            acc = __builtin_amdgcn_mfma_i32_16x16x64_i8(a0[i], b0, acc, 0, 0, 0);
            acc = __builtin_amdgcn_mfma_i32_16x16x64_i8(a1[i], b1, acc, 0, 0, 0);
        }
#pragma unroll
        for (int i = 0; i < kGroup; ++i) wc[i] = wn[i];
    }

    // join the K-slices of the wavefronts, then dequantize (fused epilogue)
    __syncthreads();
    red[wave * 64 + lane] = acc;
    __syncthreads();
    const int shift = AGQ_W_SHIFT + (XK == XK_I4 ? 4 : 0);
    const int *redi = reinterpret_cast<const int *>(red);
    for (int o = threadIdx.x; o < 256; o += blockDim.x) {
        const int l = o & 63, r = o >> 6;
        int sum = 0;
        for (int w = 0; w < nwaves; ++w) sum += redi[(w * 64 + l) * 4 + r];
        const int m = 4 * (l >> 4) + r;
        const int n = nt * 16 + (l & 15);
        if (m < a.M && n < a.N) {
            const int v = sum >> shift;   // exact: every term carries the factor
            if (a.acc_out) a.acc_out[(int64_t)m * a.N + n] = v;
            a.y[(int64_t)m * a.ldy + n] = agq_dequant(v, a.scale_e * __half2float(a.sw[n]));
        }
    }
}

}  // namespace

int agq_launch_gemm_decode(const void *x, int x_kind, int bits, int64_t M, int64_t K, int64_t ldx, int e,
                           const void *w_packed, const void *sw, int64_t N, void *y, int64_t ldy, int32_t *acc_out,
                           void *stream) {
    DecodeArgs a;
    a.x = x;
    a.ldx = ldx;
    a.M = (int)M;
    a.N = (int)N;
    a.K = (int)K;
    a.KT = (int)agq_k_tiles(K);
    a.q = agq_make_quant(bits, e, 0);
    a.blob = (const uint4 *)w_packed;
    a.sw = (const __half *)sw;
    a.y = (__half *)y;
    a.ldy = ldy;
    a.acc_out = acc_out;
    a.scale_e = ldexpf(1.0f, e);
    int waves = 1;
    while (waves < kMaxWaves && waves * kGroup < a.KT) waves *= 2;
    a.kt_per_wave = (a.KT + waves - 1) / waves;
    const unsigned grid = (unsigned)((N + 15) / 16);
    const size_t lds = (size_t)waves * kGroup * 2048;   // >= waves * 1 KiB of reduction buffer
    hipStream_t st = (hipStream_t)stream;
    if (x_kind == 0)
        gemm_decode_kernel<XK_F16><<<grid, waves * 64, lds, st>>>(a);
    else if (bits == 8)
        gemm_decode_kernel<XK_I8><<<grid, waves * 64, lds, st>>>(a);
    else
        gemm_decode_kernel<XK_I4><<<grid, waves * 64, lds, st>>>(a);
    return (int)hipGetLastError();
}
