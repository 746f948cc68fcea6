// Weight-streaming kernel of the quantized linear layer for a few tokens
// (M <= 16): the decode regime, bound by the HBM read of the 4-bit weights.
//
// One workgroup owns one 16-row tile of output channels and the whole K, so no
// partial sum ever leaves the CU.  Its wavefronts split K: each streams KPW
// consecutive 1 KiB weight chunks (one coalesced 16-byte load per lane and
// chunk), all issued before anything else so that the HBM latency is paid once
// and overlaps the prologue.  Small workgroups with few registers keep several
// of them resident per CU: the chip holds every chunk of a LLaMA-sized matrix
// in flight at once, which is what a 10-20 MB read needs to approach HBM rate.
//
// Eq.2 runs as a prologue while the weights fly: a wavefront quantizes exactly
// the slice of the activation it multiplies (M x 128 values per chunk) into a
// private LDS region laid out in MFMA operand order.  Rows beyond M are never
// written, and never reach a stored result, because an MFMA output row depends
// on the matching operand row only.  A single LDS reduction joins the
// wavefronts before the fused per-channel dequantisation.
#include "../../include/agq.h"
#include "agq_device.h"
#include "agq_internal.h"

AgqQuant agq_make_quant(int bits, int e, int zp);

namespace {

// Up to kMaxProj projections that read the same activation (q/k/v, gate/up) run
// as one launch: workgroup b serves 16-channel tile b - tile_start[p] of the
// projection p whose tile range contains b.
constexpr int kMaxProj = AGQ_MAX_PROJ;

struct DecodeArgs {
    const void *x;
    int64_t ldx;      // elements (fp16 / int8) or codes (nibbles)
    int M, KT, count;
    AgqQuant q;
    float scale_e;    // 2^e
    int tile_start[kMaxProj + 1];
    int N[kMaxProj];
    const uint4 *blob[kMaxProj];
    const __half *sw[kMaxProj];
    __half *y[kMaxProj];
    int64_t ldy[kMaxProj];
    int32_t *acc_out[kMaxProj];
};

enum { XK_F16 = 0, XK_I8 = 1, XK_I4 = 2 };

typedef unsigned int agq_u4 __attribute__((ext_vector_type(4)));
typedef unsigned int agq_u2 __attribute__((ext_vector_type(2)));

// eight fp16 -> eight int8 codes (signed grid), k ascending
__device__ __forceinline__ agq_u2 quant8v(const agq_u4 &h, const AgqQuant &q) {
    uint32_t c[8];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const uint32_t two = h[i];           // copy out first: a vector element is not addressable
        const float2 f = __half22float2(__builtin_bit_cast(__half2, two));
        c[2 * i] = agq_quant1(f.x, q);
        c[2 * i + 1] = agq_quant1(f.y, q);
    }
    return agq_u2{agq_pack4(c[0], c[1], c[2], c[3]), agq_pack4(c[4], c[5], c[6], c[7])};
}

// XK: what x holds; KPW: weight chunks per wavefront and pass over K;
// MP: passes of four token rows the Eq.2 prologue makes (M <= 4 MP).
template <int XK, int KPW, int MP>
__global__ __launch_bounds__(KPW == 8 ? 1024 : 512, KPW == 8 ? 4 : (MP == 1 ? 6 : 5)) void gemm_decode_kernel(const DecodeArgs a) {
    extern __shared__ __align__(16) unsigned char smem[];
    const int lane = threadIdx.x & 63;
    const int wave = threadIdx.x >> 6;
    const int nwaves = blockDim.x >> 6;
    int pj = 0;   // which projection this workgroup serves (uniform)
    while (pj + 1 < a.count && (int)blockIdx.x >= a.tile_start[pj + 1]) ++pj;
    const int nt = blockIdx.x - a.tile_start[pj];
    const int KT = a.KT;
    const int pN = a.N[pj];
    const __half *psw = a.sw[pj];
    const agq_u4 *wptr = reinterpret_cast<const agq_u4 *>(a.blob[pj]) + ((int64_t)nt * KT) * 64 + lane;

    agq_v4i acc0 = {0, 0, 0, 0}, acc1 = {0, 0, 0, 0};
    agq_u4 *stage = reinterpret_cast<agq_u4 *>(smem) + wave * 128;   // 2 KiB per wavefront
    const int arow = min(lane & 15, a.M - 1);   // operand row of this lane, clamped into the tensor
    const int ag = lane >> 4;
    uint32_t sw_bits = 0;                       // raw fp16 scale of this thread's output channel

    for (int kb = wave * KPW; kb < KT; kb += nwaves * KPW) {
        // The activation slice is requested first and the weight chunks right after:
        // loads return in order, so the prologue can start as soon as the (L2-hot)
        // activation arrives while the weights are still on their way from HBM.
        // Chunk indices are clamped into the tensors: a chunk past the end is
        // loaded again and its weights are zeroed.  With many token rows the
        // activation is fetched HB chunks at a time to bound the registers.
        constexpr int HB = XK != XK_F16 ? KPW : (8 / MP < KPW ? 8 / MP : KPW);
        const int c16 = lane & 15, rr = lane >> 4;
        agq_u4 xv[XK == XK_F16 ? HB : 1][XK == XK_F16 ? MP : 1];
        agq_v4i fa0[XK == XK_F16 ? 1 : KPW], fa1[XK == XK_F16 ? 1 : KPW];
        auto load_x = [&](int i0) {
#pragma unroll
            for (int i = 0; i < HB; ++i) {
                const int64_t kc = min(kb + i0 + i, KT - 1);
                const __half *xh = reinterpret_cast<const __half *>(a.x) + kc * 128 + c16 * 8;
#pragma unroll
                for (int it = 0; it < MP; ++it)
                    xv[i][it] = *reinterpret_cast<const agq_u4 *>(xh + (int64_t)min(it * 4 + rr, a.M - 1) * a.ldx);
            }
        };
        if (XK == XK_F16) {
            load_x(0);
        } else {
#pragma unroll
            for (int i = 0; i < KPW; ++i) {
                const int64_t kc = min(kb + i, KT - 1);
                if (XK == XK_I8) {
                    const int8_t *xq = reinterpret_cast<const int8_t *>(a.x) + (int64_t)arow * a.ldx + ag * 16 + kc * 128;
                    fa0[i] = __builtin_bit_cast(agq_v4i, *reinterpret_cast<const agq_u4 *>(xq));
                    fa1[i] = __builtin_bit_cast(agq_v4i, *reinterpret_cast<const agq_u4 *>(xq + 64));
                } else {
                    // nibble codes, low nibble = even k: widen to 16 * code in k order
                    const uint8_t *xq = reinterpret_cast<const uint8_t *>(a.x) + (int64_t)arow * (a.ldx >> 1) + ag * 8 + kc * 64;
                    const agq_u2 p0 = *reinterpret_cast<const agq_u2 *>(xq);
                    const agq_u2 p1 = *reinterpret_cast<const agq_u2 *>(xq + 32);
                    const uint32_t pw[4] = {p0.x, p0.y, p1.x, p1.y};
                    uint32_t o[8];
#pragma unroll
                    for (int j = 0; j < 4; ++j) {
                        const uint32_t ev = (pw[j] << 4) & 0xF0F0F0F0u, od = pw[j] & 0xF0F0F0F0u;
                        o[2 * j] = __builtin_amdgcn_perm(od, ev, 0x05010400u);
                        o[2 * j + 1] = __builtin_amdgcn_perm(od, ev, 0x07030602u);
                    }
                    fa0[i] = agq_v4i{(int)o[0], (int)o[1], (int)o[2], (int)o[3]};
                    fa1[i] = agq_v4i{(int)o[4], (int)o[5], (int)o[6], (int)o[7]};
                }
            }
        }
        asm volatile("" ::: "memory");   // keep the activation loads ahead of the weight loads
        agq_u4 w[KPW];
#pragma unroll
        for (int i = 0; i < KPW; ++i) w[i] = wptr[(int64_t)min(kb + i, KT - 1) * 64];
        if (kb == wave * KPW && threadIdx.x < 256) {
            const int n = min(nt * 16 + (lane & 15), pN - 1);
            sw_bits = reinterpret_cast<const uint16_t *>(psw)[n];
        }
        asm volatile("" ::: "memory");

#pragma unroll
        for (int i = 0; i < KPW; ++i) {
            const bool valid = kb + i < KT;            // wave-uniform
            agq_v4i a0, a1;
            if (XK == XK_F16) {
                if (i > 0 && i % HB == 0) load_x(i);
                // Eq.2 on the M x 128 slice of this chunk: lane = 8 consecutive k of one
                // row, four rows per pass; rows were clamped for the load and are
                // masked for the LDS store
                const int s = c16 >> 3, g = (c16 & 7) >> 1, hf = c16 & 1;
#pragma unroll
                for (int it = 0; it < MP; ++it) {
                    const int m = it * 4 + rr;
                    const agq_u2 codes = quant8v(xv[i % HB][it], a.q);
                    if (m < a.M) reinterpret_cast<agq_u2 *>(stage + s * 64 + g * 16 + m)[hf] = codes;
                }
                // the same wavefront wrote and now reads: LDS keeps program order per wave
                __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
                __builtin_amdgcn_wave_barrier();
                __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
                a0 = __builtin_bit_cast(agq_v4i, stage[lane]);
                a1 = __builtin_bit_cast(agq_v4i, stage[64 + lane]);
                __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
                __builtin_amdgcn_wave_barrier();
            } else {
                a0 = fa0[i];
                a1 = fa1[i];
            }
            const agq_u4 wv = valid ? w[i] : agq_u4{0u, 0u, 0u, 0u};
            const agq_v4i b0 = __builtin_bit_cast(agq_v4i, (wv << 4) & 0xF0F0F0F0u);
            const agq_v4i b1 = __builtin_bit_cast(agq_v4i, wv & 0xF0F0F0F0u);
            acc0 = __builtin_amdgcn_mfma_i32_16x16x64_i8(a0, b0, acc0, 0, 0, 0);
            acc1 = __builtin_amdgcn_mfma_i32_16x16x64_i8(a1, b1, acc1, 0, 0, 0);
        }
    }

    // join the K-slices of the wavefronts, then dequantize (fused epilogue).
    // Partial sums are stored [wave][register][lane] so that both the write and
    // the read below are conflict-free.
    __syncthreads();   // every wavefront has left its staging region
    int *red = reinterpret_cast<int *>(smem);
    const agq_v4i acc = acc0 + acc1;
#pragma unroll
    for (int r = 0; r < 4; ++r) red[(wave * 4 + r) * 64 + lane] = acc[r];
    __syncthreads();
    const int shift = AGQ_W_SHIFT + (XK == XK_I4 ? 4 : 0);
    for (int o = threadIdx.x; o < 256; o += blockDim.x) {
        const int l = o & 63, r = o >> 6;
        const int m = 4 * (l >> 4) + r;
        const int n = nt * 16 + (l & 15);
        if (m < a.M && n < pN) {
            int sum = 0;
            for (int w = 0; w < nwaves; ++w) sum += red[(w * 4 + r) * 64 + l];
            const int v = sum >> shift;   // exact: every term carries the factor
            if (a.acc_out[pj]) a.acc_out[pj][(int64_t)m * pN + n] = v;
            const uint32_t sb = blockDim.x >= 256 ? sw_bits : (uint32_t) reinterpret_cast<const uint16_t *>(psw)[n];
            a.y[pj][(int64_t)m * a.ldy[pj] + n] = agq_dequant(v, a.scale_e * __half2float(__ushort_as_half((unsigned short)sb)));
        }
    }
}

template <int XK, int MP>
int launch_xk(const DecodeArgs &a, int kpw, unsigned grid, int waves, size_t lds, hipStream_t st) {
    switch (kpw) {
        case 1: gemm_decode_kernel<XK, 1, MP><<<grid, waves * 64, lds, st>>>(a); break;
        case 2: gemm_decode_kernel<XK, 2, MP><<<grid, waves * 64, lds, st>>>(a); break;
        case 4: gemm_decode_kernel<XK, 4, MP><<<grid, waves * 64, lds, st>>>(a); break;
        default: gemm_decode_kernel<XK, 8, MP><<<grid, waves * 64, lds, st>>>(a); break;
    }
    return (int)hipGetLastError();
}

}  // namespace

int agq_launch_gemm_decode(const void *x, int x_kind, int bits, int64_t M, int64_t K, int64_t ldx, int e,
                           const agq_proj *projs, int count, void *stream) {
    DecodeArgs a;
    a.x = x;
    a.ldx = ldx;
    a.M = (int)M;
    a.KT = (int)agq_k_tiles(K);
    a.count = count;
    a.q = agq_make_quant(bits, e, 0);
    a.scale_e = ldexpf(1.0f, e);
    int tiles = 0;
    for (int p = 0; p < kMaxProj; ++p) {
        const agq_proj &pr = projs[p < count ? p : count - 1];
        a.tile_start[p] = tiles;
        if (p < count) tiles += (int)((pr.N + 15) / 16);
        a.N[p] = (int)pr.N;
        a.blob[p] = (const uint4 *)pr.w_packed;
        a.sw[p] = (const __half *)pr.w_scale_f16;
        a.y[p] = (__half *)pr.y_f16;
        a.ldy[p] = pr.ldy;
        a.acc_out[p] = pr.acc_out;
    }
    a.tile_start[kMaxProj] = tiles;
    for (int p = count; p <= kMaxProj; ++p) a.tile_start[p] = tiles;
    // chunks per wavefront: the smallest of 1, 2, 4, 8 that needs at most 8
    // wavefronts (16 for the largest); very long K loops inside the kernel
    int kpw = 1;
    while (kpw < 8 && (a.KT + kpw - 1) / kpw > 8) kpw *= 2;
    int waves = (a.KT + kpw - 1) / kpw;
    if (waves > 16) waves = 16;
    const unsigned grid = (unsigned)tiles;
    const size_t lds = (size_t)waves * 2048;   // staging; reused as waves * 1 KiB of partial sums
    hipStream_t st = (hipStream_t)stream;
    if (x_kind == 0) {
        if (M <= 4) return launch_xk<XK_F16, 1>(a, kpw, grid, waves, lds, st);
        if (M <= 8) return launch_xk<XK_F16, 2>(a, kpw, grid, waves, lds, st);
        return launch_xk<XK_F16, 4>(a, kpw, grid, waves, lds, st);
    }
    if (bits == 8) return launch_xk<XK_I8, 1>(a, kpw, grid, waves, lds, st);
    return launch_xk<XK_I4, 1>(a, kpw, grid, waves, lds, st);
}
