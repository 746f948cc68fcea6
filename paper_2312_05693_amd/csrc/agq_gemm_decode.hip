// Weight-streaming kernel of the quantized linear layer for a few tokens
// (M <= 16): the decode regime, bound by the HBM read of the 4-bit weights.
//
// One workgroup owns one 16-row tile of output channels and the whole K, so no
// partial sum ever leaves the CU.  Its wavefronts split K: each streams KPW
// consecutive 1 KiB weight chunks (one coalesced 16-byte load per lane and
// chunk), all requested up front so that the HBM latency is paid once and
// overlaps the prologue: the chip holds every chunk of a LLaMA-sized matrix in
// flight at once, which is what a 10-20 MB read needs to approach HBM rate.
// The kernel is a chain of latencies (arguments, load issue through the CU's one
// address unit, activation from L2, LDS staging, weights, reduction, store), and
// what is tuned here is the length of that chain: one round of scalar loads,
// as few vector-memory instructions as the bytes allow, one LDS round trip.
//
// Eq.2 runs as a prologue while the weights fly: a wavefront quantizes exactly
// the slice of the activation it multiplies (M x 128 values per chunk, packed
// fp16 arithmetic) into a private LDS region laid out in MFMA operand order.
// Rows beyond M are never written, and never reach a stored result, because an
// MFMA output row depends on the matching operand row only.  A single LDS
// reduction joins the wavefronts before the fused per-channel dequantisation.
#include "../../include/agq.h"
#include "agq_device.h"
#include "agq_internal.h"

#include <mutex>

AgqQuant agq_make_quant_signed(int bits, int e, int zp);

namespace {

// Up to kMaxProj projections that read the same activation (q/k/v, gate/up) run
// as one launch: workgroup b serves 16-channel tile b - tile_start[p] of the
// projection p whose tile range contains b.
constexpr int kMaxProj = AGQ_MAX_PROJ;

// One projection as a workgroup holds it once it knows which one it serves.
struct DecodeProj {
    const uint4 *blob;
    const __half *sw;
    __half *y;
    int32_t *acc_out;
    int ldy, N;
};

// The kernel arguments.  What a workgroup needs before that load comes first and packed, so that a few
// wide scalar loads (one round trip) bring it in; the output pointers, needed
// only for the store, follow as one array per field.
struct DecodeArgs {
    const void *x;
    int64_t ldx;      // elements (fp16 / int8) or codes (nibbles)
    int M, KT, count;
    float scale_e;    // 2^e
    int tile_start[kMaxProj + 1];   // entries from `count` on hold the total
    int waves;                      // wavefronts per workgroup (= blockDim.x / 64, without a trip to the dispatch packet)
    int corr;                       // unsigned grid: acc += corr * sum_k w[n,k]; 0 on the signed grid
    uint32_t flip;                  // unsigned grid, codes given: xor that turns q into q - 2^(b-1); else 0
    const uint4 *blob4[kMaxProj];   // per projection: weight blob, channel scales, width
    const __half *sw4[kMaxProj];
    int N4[kMaxProj];
    AgqQuant q;
    __half *y4[kMaxProj];
    int32_t *acc4[kMaxProj];
    int ldy4[kMaxProj];
    int n_extra;   // TRIP blob: extra chunks in front of the KT main chunks of every tile; else 0
    // Never read.  With the record at 368 or 384 bytes every launch of a replayed graph
    // measured 0.1-0.15 us shorter than at 256, 400 or 408 bytes (same instructions; the
    // cause is in how the runtime lays consecutive argument records out, not in the kernel).
    int reserved[31];
};
static_assert(sizeof(DecodeArgs) == 384, "see the note on `reserved`");

__device__ __forceinline__ DecodeProj load_proj(const DecodeArgs &a, int pj) {
    DecodeProj pr;
    pr.blob = a.blob4[pj];
    pr.sw = a.sw4[pj];
    pr.y = a.y4[pj];
    pr.acc_out = a.acc4[pj];
    pr.ldy = a.ldy4[pj];
    pr.N = a.N4[pj];
    return pr;
}

// Per-channel weight sums at the end of a blob (after the padded nibble tiles);
// read on the unsigned grid only.
__device__ __forceinline__ const int32_t *blob_wsum(const uint4 *blob, int N, int KT) {
    return reinterpret_cast<const int32_t *>(blob + (int64_t)((N + 255) / 256) * 16 * KT * 64);
}

// Which projection a tile belongs to, and its index inside it, without a loop of
// dependent loads: the three inner boundaries are compared at once.
__device__ __forceinline__ int find_proj(const DecodeArgs &a, int tile, int &nt) {
    const int t1 = a.tile_start[1], t2 = a.tile_start[2], t3 = a.tile_start[3];
    const int pj = (tile >= t1) + (tile >= t2) + (tile >= t3);
    nt = tile - (pj == 0 ? 0 : (pj == 1 ? t1 : (pj == 2 ? t2 : t3)));
    return pj;
}

// ONE: fp16 with a single token row; Z: fp16 on the unsigned grid (a zero point is added to every code)
// T: fp16 with a TRIP blob (Section 4.4): one more wavefront multiplies the extra chunks
enum { XK_F16 = 0, XK_I8 = 1, XK_I4 = 2, XK_F16_ONE = 3, XK_F16_Z = 4, XK_F16_ONE_Z = 5,
       XK_F16_T = 6, XK_F16_ONE_T = 7, XK_F16_TZ = 8 };

typedef unsigned int agq_u4 __attribute__((ext_vector_type(4)));
typedef unsigned int agq_u2 __attribute__((ext_vector_type(2)));

// eight fp16 -> eight int8 codes (signed grid), k ascending
template <bool ZP>
__device__ __forceinline__ agq_u2 quant8v(const agq_u4 &h, const AgqQuant &q) {
    if (q.h_scale2 != 0) {       // uniform: the packed fp16 quantizer covers every usual exponent
        const uint32_t h0 = h[0], h1 = h[1], h2 = h[2], h3 = h[3];
        const uint2 c = agq_quant8h<ZP>(h0, h1, h2, h3, q);
        return agq_u2{c.x, c.y};
    }
    uint32_t c[8];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const uint32_t two = h[i];           // copy out first: a vector element is not addressable
        const float2 f = __half22float2(__builtin_bit_cast(__half2, two));
        c[2 * i] = agq_quant1(f.x, q) + (ZP ? (uint32_t)q.zp : 0u);
        c[2 * i + 1] = agq_quant1(f.y, q) + (ZP ? (uint32_t)q.zp : 0u);
    }
    return agq_u2{agq_pack4(c[0], c[1], c[2], c[3]), agq_pack4(c[4], c[5], c[6], c[7])};
}

// XK: what x holds; KPW: weight chunks per wavefront and pass over K;
// MP: passes of four token rows the Eq.2 prologue makes (M <= 4 MP).
// (The second launch bound, wavefronts per SIMD the compiler has to leave room for: the one-row instantiation
// with four chunks per wavefront otherwise takes 70 registers, i.e. three of its eight-wavefront workgroups per
// CU instead of four; with 62 the gate/up launch of LLaMA-7B went from 10.4 to 10.1 us, the others stayed.)
template <int XK, int KPW, int MP, bool RG = false>
__global__ __launch_bounds__(1024, (XK == XK_F16_ONE && KPW == 4 && MP == 1 && !RG) ? 8 : 1) void gemm_decode_kernel(const DecodeArgs a) {
    extern __shared__ __align__(16) unsigned char smem[];
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int nwaves = a.waves;
    // RG: more than sixteen token rows, sixteen per workgroup; blockIdx.y picks the group
    const int row0 = RG ? 16 * (int)blockIdx.y : 0;
    const int Mloc = RG ? min(16, a.M - row0) : a.M;
    const void *const xbase = RG ? static_cast<const void *>(reinterpret_cast<const __half *>(a.x) + (int64_t)row0 * a.ldx) : a.x;
    constexpr bool TRIP = XK == XK_F16_T || XK == XK_F16_ONE_T || XK == XK_F16_TZ;
    constexpr bool F16 = XK == XK_F16 || XK == XK_F16_ONE || XK == XK_F16_Z || XK == XK_F16_ONE_Z || TRIP;
    constexpr bool ONE = XK == XK_F16_ONE || XK == XK_F16_ONE_Z || XK == XK_F16_ONE_T;   // one row: a lane's 16 bytes are its own chunk's, four chunks per load
    constexpr bool ZP = XK == XK_F16_Z || XK == XK_F16_ONE_Z || XK == XK_F16_TZ;         // fp16 input on the unsigned grid
    // Everything the first vector loads depend on is requested in one round of
    // scalar loads; the weight pointer, scale pointer and width of this workgroup's
    // projection are picked by scalar selects instead of a second, dependent round
    // (~500 cycles).  The rest of the record is fetched now and used at the store.
    const int KT = a.KT;
    const int t1 = a.tile_start[1], t2 = a.tile_start[2], t3 = a.tile_start[3];
    const uint4 *bl0 = a.blob4[0], *bl1 = a.blob4[1], *bl2 = a.blob4[2], *bl3 = a.blob4[3];
    const __half *sc0 = a.sw4[0], *sc1 = a.sw4[1], *sc2 = a.sw4[2], *sc3 = a.sw4[3];
    const int n0 = a.N4[0], n1 = a.N4[1], n2 = a.N4[2], n3 = a.N4[3];
    asm volatile("" ::"s"(a.x), "s"(a.ldx), "s"(a.M), "s"(KT), "s"(nwaves), "s"(t1), "s"(t2), "s"(t3), "s"(a.scale_e), "s"(bl0),
                 "s"(bl1), "s"(bl2), "s"(bl3), "s"(sc0), "s"(sc1), "s"(sc2), "s"(sc3), "s"(n0), "s"(n1), "s"(n2), "s"(n3),
                 "s"(a.q.scale), "s"(a.q.lo), "s"(a.q.hi), "s"(a.q.h_scale2), "s"(a.q.h_lo2), "s"(a.q.h_hi2),
                 "s"(ZP ? a.q.h_zp2 : 0u), "s"(F16 ? 0u : a.flip), "s"(a.corr), "s"(TRIP ? a.n_extra : 0));
    int corr_keep = 0;
    if (!(F16 && !ZP)) asm volatile("v_mov_b32 %0, %1" : "=v"(corr_keep) : "s"(a.corr));
    int nt;
    const int pj = find_proj(a, blockIdx.x, nt);   // which projection this workgroup serves (uniform)
    // RG: a workgroup serves two neighbouring channel tiles of its projection with the same quantized rows (the
    // activation, which every workgroup reads in full, is most of such a launch's traffic); tile_start counts pairs
    if (RG) nt *= 2;
    __half *const py = a.y4[pj];
    int32_t *const pacc = a.acc4[pj];
    const int pldy = a.ldy4[pj];
    const int pN = pj == 0 ? n0 : (pj == 1 ? n1 : (pj == 2 ? n2 : n3));
    const __half *psw = pj == 0 ? sc0 : (pj == 1 ? sc1 : (pj == 2 ? sc2 : sc3));
    const uint4 *pblob = pj == 0 ? bl0 : (pj == 1 ? bl1 : (pj == 2 ? bl2 : bl3));
    // TRIP: the last wavefront serves the extra chunks (channels with a factor), the
    // others the KT main chunks that follow them in every tile of the blob
    const int n_extra = TRIP ? a.n_extra : 0;
    const int KTall = KT + n_extra;
    const int nmain = TRIP ? nwaves - 1 : nwaves;
    const agq_u4 *wptr = reinterpret_cast<const agq_u4 *>(pblob) + ((int64_t)nt * KTall + n_extra) * 64 + lane;
    const bool second = RG && (nt + 1) * 16 < pN;                     // the pair's second tile exists (uniform)
    const agq_u4 *wptr2 = second ? wptr + (int64_t)KTall * 64 : wptr;

    agq_v4i acc0 = {0, 0, 0, 0}, acc1 = {0, 0, 0, 0};
    agq_v4i acc2 = {0, 0, 0, 0}, acc3 = {0, 0, 0, 0};                 // second tile (RG)
    // Staging of the quantized activation: one region per chunk of a batch, in MFMA
    // operand order [k-half s][k-group g][row m] x 16 bytes with only the R = 4 MP
    // rows the prologue writes (operand rows beyond R alias lower rows; they never
    // reach a stored result).  A batch is HB chunks: all of them are written, then
    // all operands are read back, so the LDS round trip is paid once per batch.
    constexpr int R = 4 * MP;
    constexpr int HB = !F16 ? KPW : (8 / MP < KPW ? 8 / MP : KPW);
    constexpr int NX = ONE ? (HB + 3) / 4 : HB;                       // activation loads per batch and row pass
    constexpr int kRegion = 8 * R;                                     // 16-byte pieces per chunk
    agq_u4 *stage = reinterpret_cast<agq_u4 *>(smem) + wave * (HB * kRegion);
    const int arow = min(lane & 15, Mloc - 1);   // operand row of this lane, clamped into the tensor
    const int ag = lane >> 4;
    const int srow = (lane & 15) & (R - 1);     // staged row this lane's operand comes from
    uint32_t sw_bits = 0;                       // raw fp16 scale of this thread's output channel

    for (int kb = (TRIP && wave == nmain) ? KT : wave * KPW; kb < KT; kb += nmain * KPW) {
        // The activation slice is requested first and the weight chunks right after:
        // loads return in order, so the prologue can start as soon as the (L2-hot)
        // activation arrives while the weights are still on their way from HBM.
        // Chunk indices are clamped into the tensors: a chunk past the end is
        // loaded again and its weights are zeroed.  With many token rows the
        // activation is fetched HB chunks at a time to bound the registers.
        const int c16 = lane & 15, rr = lane >> 4;
        agq_u4 xv[F16 ? NX : 1][F16 ? MP : 1];
        agq_v4i fa0[F16 ? HB : KPW], fa1[F16 ? HB : KPW];
        auto load_x = [&](int i0) {
#pragma unroll
            for (int i = 0; i < NX; ++i) {
                if (ONE) {   // lane = (chunk 4 i + rr of the batch, eight k): one row only
                    const int64_t kc = min(kb + i0 + 4 * i + rr, KT - 1);
                    xv[i][0] = *reinterpret_cast<const agq_u4 *>(reinterpret_cast<const __half *>(xbase) + kc * 128 + c16 * 8);
                    continue;
                }
                const int64_t kc = min(kb + i0 + i, KT - 1);
                const __half *xh = reinterpret_cast<const __half *>(xbase) + kc * 128 + c16 * 8;
#pragma unroll
                for (int it = 0; it < MP; ++it)
                    xv[i][it] = *reinterpret_cast<const agq_u4 *>(xh + (int64_t)min(it * 4 + rr, Mloc - 1) * a.ldx);
            }
        };
        if (F16) {
            load_x(0);
        } else {
#pragma unroll
            for (int i = 0; i < KPW; ++i) {
                const int64_t kc = min(kb + i, KT - 1);
                if (XK == XK_I8) {
                    const int8_t *xq = reinterpret_cast<const int8_t *>(xbase) + (int64_t)arow * a.ldx + ag * 16 + kc * 128;
                    fa0[i] = __builtin_bit_cast(agq_v4i, *reinterpret_cast<const agq_u4 *>(xq) ^ a.flip);
                    fa1[i] = __builtin_bit_cast(agq_v4i, *reinterpret_cast<const agq_u4 *>(xq + 64) ^ a.flip);
                } else {
                    // nibble codes, low nibble = even k: widen to 16 * code in k order
                    const uint8_t *xq = reinterpret_cast<const uint8_t *>(xbase) + (int64_t)arow * (a.ldx >> 1) + ag * 8 + kc * 64;
                    const agq_u2 p0 = *reinterpret_cast<const agq_u2 *>(xq);
                    const agq_u2 p1 = *reinterpret_cast<const agq_u2 *>(xq + 32);
                    const uint32_t pw[4] = {p0.x ^ a.flip, p0.y ^ a.flip, p1.x ^ a.flip, p1.y ^ a.flip};
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
        agq_u4 w[KPW], w2[RG ? KPW : 1];
#pragma unroll
        for (int i = 0; i < KPW; ++i) w[i] = wptr[(int64_t)min(kb + i, KT - 1) * 64];
        if (RG) {
#pragma unroll
            for (int i = 0; i < KPW; ++i) w2[i] = wptr2[(int64_t)min(kb + i, KT - 1) * 64];
        }
        if (kb == wave * KPW && threadIdx.x < (RG ? 512 : 256)) {
            // the scale of the first output this thread will store (RG: threads 256.. store the second tile)
            const int n = min((nt + (RG ? (int)(threadIdx.x >> 8) : 0)) * 16 + (lane & 15), pN - 1);
            sw_bits = reinterpret_cast<const uint16_t *>(psw)[n];
        }
        asm volatile("" ::: "memory");

#pragma unroll
        for (int b0 = 0; b0 < KPW; b0 += HB) {
            if (F16) {
                if (b0 > 0) load_x(b0);
                // Eq.2 on the M x 128 slice of each chunk: lane = 8 consecutive k of one
                // row, four rows per pass; rows were clamped for the load and are
                // masked for the LDS store
                const int s = c16 >> 3, g = (c16 & 7) >> 1, hf = c16 & 1;
#pragma unroll
                for (int i = 0; i < NX; ++i)
#pragma unroll
                    for (int it = 0; it < MP; ++it) {
                        const agq_u2 codes = quant8v<ZP>(xv[i][it], a.q);
                        if (ONE) {
                            const int ch = 4 * i + rr;   // chunk of the batch, row 0
                            if (ch < HB) reinterpret_cast<agq_u2 *>(stage + ch * kRegion + (s * 4 + g) * R)[hf] = codes;
                        } else {
                            const int m = it * 4 + rr;
                            if (m < Mloc) reinterpret_cast<agq_u2 *>(stage + i * kRegion + (s * 4 + g) * R + m)[hf] = codes;
                        }
                    }
                // the same wavefront wrote and now reads: LDS keeps program order per wave
                __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
                __builtin_amdgcn_wave_barrier();
                __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
#pragma unroll
                for (int i = 0; i < HB; ++i) {
                    fa0[i] = __builtin_bit_cast(agq_v4i, stage[i * kRegion + ag * R + srow]);
                    fa1[i] = __builtin_bit_cast(agq_v4i, stage[i * kRegion + (4 + ag) * R + srow]);
                }
                __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
                __builtin_amdgcn_wave_barrier();
            }
#pragma unroll
            for (int i = 0; i < HB; ++i) {
                const bool valid = kb + b0 + i < KT;            // wave-uniform
                const agq_v4i a0 = fa0[F16 ? i : b0 + i], a1 = fa1[F16 ? i : b0 + i];
                const agq_u4 wv = valid ? w[b0 + i] : agq_u4{0u, 0u, 0u, 0u};
                const agq_v4i b0v = __builtin_bit_cast(agq_v4i, (wv << 4) & 0xF0F0F0F0u);
                const agq_v4i b1v = __builtin_bit_cast(agq_v4i, wv & 0xF0F0F0F0u);
                acc0 = __builtin_amdgcn_mfma_i32_16x16x64_i8(a0, b0v, acc0, 0, 0, 0);
                acc1 = __builtin_amdgcn_mfma_i32_16x16x64_i8(a1, b1v, acc1, 0, 0, 0);
                if (RG) {
                    const agq_u4 wv2 = valid ? w2[b0 + i] : agq_u4{0u, 0u, 0u, 0u};
                    const agq_v4i b2v = __builtin_bit_cast(agq_v4i, (wv2 << 4) & 0xF0F0F0F0u);
                    const agq_v4i b3v = __builtin_bit_cast(agq_v4i, wv2 & 0xF0F0F0F0u);
                    acc2 = __builtin_amdgcn_mfma_i32_16x16x64_i8(a0, b2v, acc2, 0, 0, 0);
                    acc3 = __builtin_amdgcn_mfma_i32_16x16x64_i8(a1, b3v, acc3, 0, 0, 0);
                }
            }
        }
    }

    if (TRIP && wave == nmain) {
        // Extra chunks: slot j of chunk c is input channel idx[c * 128 + j], quantized with
        // the step 2^(e + factor of the chunk) (Eq.5); the chunk's partial product is
        // shifted left by its factor (Section 4.4: the factor sits on the weight row).
        // Same lane roles and staging as the main prologue (lane = eight slots of one
        // row, four rows per pass), with a gather instead of a 16-byte load.  Two chunks
        // at a time: their factors, indices and weights are requested in one round, the
        // gathered activations in a second one.
        const int32_t *meta = blob_wsum(pblob, pN, KTall) + ((pN + 255) / 256) * 256;
        const int32_t *idx = meta + 32;
        const agq_u4 *wx = reinterpret_cast<const agq_u4 *>(pblob) + ((int64_t)nt * KTall) * 64 + lane;
        const __half *xh = reinterpret_cast<const __half *>(xbase);
        const int c16 = lane & 15, rr = lane >> 4;
        const int s = c16 >> 3, g = (c16 & 7) >> 1, hf = c16 & 1;
        const int metav = meta[c16];                    // the factors of all (at most 16) chunks
        for (int c0 = 0; c0 < n_extra; c0 += 2) {
            int4 ia[2][2];
            agq_u4 wv[2];
#pragma unroll
            for (int u = 0; u < 2; ++u) {
                const int cc = min(c0 + u, n_extra - 1);
                const int4 *ip = reinterpret_cast<const int4 *>(idx + cc * 128 + c16 * 8);
                ia[u][0] = ip[0];
                ia[u][1] = ip[1];
                wv[u] = wx[(int64_t)cc * 64];
            }
            __half xg[2][MP][8];
#pragma unroll
            for (int u = 0; u < 2; ++u) {
                const int kk[8] = {ia[u][0].x, ia[u][0].y, ia[u][0].z, ia[u][0].w,
                                   ia[u][1].x, ia[u][1].y, ia[u][1].z, ia[u][1].w};
#pragma unroll
                for (int it = 0; it < MP; ++it) {
                    const __half *xr = xh + (int64_t)min(it * 4 + rr, Mloc - 1) * a.ldx;
#pragma unroll
                    for (int j = 0; j < 8; ++j) xg[u][it][j] = xr[max(kk[j], 0)];   // an unused slot (-1) meets zero weights
                }
            }
#pragma unroll
            for (int u = 0; u < 2; ++u) {
                if (c0 + u >= n_extra) break;
                const int factor = __builtin_amdgcn_readlane(metav, c0 + u);
                AgqQuant qe = a.q;
                qe.scale = ldexpf(a.q.scale, -factor);
#pragma unroll
                for (int it = 0; it < MP; ++it) {
                    uint32_t b[8];
#pragma unroll
                    for (int j = 0; j < 8; ++j) b[j] = agq_quant1(__half2float(xg[u][it][j]), qe) + (uint32_t)qe.zp;
                    const agq_u2 codes = {agq_pack4(b[0], b[1], b[2], b[3]), agq_pack4(b[4], b[5], b[6], b[7])};
                    const int m = it * 4 + rr;
                    if (m < Mloc) reinterpret_cast<agq_u2 *>(stage + (s * 4 + g) * R + m)[hf] = codes;
                }
                __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
                __builtin_amdgcn_wave_barrier();
                __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
                const agq_v4i a0 = __builtin_bit_cast(agq_v4i, stage[ag * R + srow]);
                const agq_v4i a1 = __builtin_bit_cast(agq_v4i, stage[(4 + ag) * R + srow]);
                __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
                __builtin_amdgcn_wave_barrier();
                const agq_v4i b0v = __builtin_bit_cast(agq_v4i, (wv[u] << 4) & 0xF0F0F0F0u);
                const agq_v4i b1v = __builtin_bit_cast(agq_v4i, wv[u] & 0xF0F0F0F0u);
                const agq_v4i zero = {0, 0, 0, 0};
                const agq_v4i t0 = __builtin_amdgcn_mfma_i32_16x16x64_i8(a0, b0v, zero, 0, 0, 0);
                const agq_v4i t1 = __builtin_amdgcn_mfma_i32_16x16x64_i8(a1, b1v, zero, 0, 0, 0);
                acc0 += (t0 + t1) << factor;
            }
        }
    }

    // join the K-slices of the wavefronts, then dequantize (fused epilogue).
    // Partial sums are stored [wave][register][lane] so that both the write and
    // the read below are conflict-free.
    // fp16 input on the signed grid has no correction term: nothing of it is compiled.  Otherwise the factor waits
    // in a vector register: a scalar register would be given up during the weight stream and the argument fetched
    // again here, a memory round trip on the tail of the launch.
    const int corr = (F16 && !ZP) ? 0 : __builtin_amdgcn_readfirstlane(corr_keep);
    // (behind the staging regions, so that a wavefront need not wait for the others to leave theirs)
    constexpr int kStageBytes = F16 ? HB * kRegion * 16 : 0;
    int *red = reinterpret_cast<int *>(smem + nwaves * kStageBytes);
    const agq_v4i acc = acc0 + acc1;
#pragma unroll
    for (int r = 0; r < 4; ++r) red[(wave * 4 + r) * 64 + lane] = acc[r];
    if (RG) {   // the second tile's sums behind the first's
        const agq_v4i accb = acc2 + acc3;
#pragma unroll
        for (int r = 0; r < 4; ++r) red[((nwaves + wave) * 4 + r) * 64 + lane] = accb[r];
    }
    __syncthreads();
    const int shift = AGQ_W_SHIFT + (XK == XK_I4 ? 4 : 0);
    for (int o = threadIdx.x; o < (RG ? 512 : 256); o += nwaves * 64) {
        const int tsel = RG ? o >> 8 : 0;            // which tile of the pair
        const int l = o & 63, r = (o >> 6) & 3;
        const int m = 4 * (l >> 4) + r;
        const int n = (nt + tsel) * 16 + (l & 15);
        if (m < Mloc && n < pN) {
            int sum = 0;
            for (int w = 0; w < nwaves; ++w) sum += red[((tsel * nwaves + w) * 4 + r) * 64 + l];
            int v = sum >> shift;   // exact: every term carries the factor
            if (corr) v += corr * blob_wsum(pblob, pN, KTall)[n];
            if (pacc) pacc[(int64_t)(row0 + m) * pN + n] = v;
            const bool have = RG ? o == (int)threadIdx.x : nmain >= 4;   // prefetched above
            const uint32_t sb = have ? sw_bits : (uint32_t) reinterpret_cast<const uint16_t *>(psw)[n];
            py[(int64_t)(row0 + m) * pldy + n] = agq_dequant(v, a.scale_e * __half2float(__ushort_as_half((unsigned short)sb)));
        }
    }
}

// Workgroup barrier that orders LDS traffic only.  __syncthreads() also waits for every outstanding global load
// of the wavefront, i.e. for weight chunks that were requested ahead on purpose.
__device__ __forceinline__ void lds_barrier() { asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory"); }

// Variant for 5..16 token rows of fp16 input when a CU serves two or more channel
// tiles and K <= 8192.  With that many rows the activation is no longer small:
// every workgroup that covers the whole K reads all of it from L2 (M x K x 2
// bytes, times the number of workgroups: several times the weight bytes) and
// quantizes all of it.  Here one workgroup of sixteen wavefronts per CU does
// that once, with K split over the wavefronts for EVERY tile of the workgroup.
// A wavefront owns KPW chunks of K: it loads and quantizes (Eq.2) only that
// slice of the activation, once, keeps the MFMA operands of the slice in
// registers, and multiplies them with its slice of each of the workgroup's
// tiles, TL of them in flight: their weight chunks are requested at the start
// (the first `kPre` tiles ahead of the quantization, the rest right behind it),
// so the CU's memory queue holds the weight stream from the first microsecond
// on and nothing in the kernel waits on anything but its own oldest load.  The
// partial sums of a round of TL tiles go to LDS (the wavefront's staging area,
// reused), the workgroup meets, and wavefront b finishes tile b of the round.
// Everything between the loads and their uses is straight-line code with the
// same loads on every path (tiles past the end request one line of the last
// tile), which keeps the compiler's wait counts exact: where two paths with
// different numbers of outstanding loads meet, it waits for the larger number
// to drain, which is how a look-ahead written with `if (more tiles)` around its
// loads ends up waiting for the look-ahead itself.
//
// KPW: chunks of K per wavefront (16 KPW >= KT); MP: passes of four rows (M <= 4 MP);
// TL: tiles a workgroup holds at a time (its tiles are blockIdx.x + gridDim.x j, j = 0, 1, ...);
// MULTI: more than TL tiles per workgroup, in rounds of TL: a slot is requested again, for the next round,
// as soon as it has been multiplied, and the workgroup meets twice per round (the operands stay in registers).
constexpr int kSliceMaxKT = 64;

template <int KPW, int MP, int TL, bool ZP, bool MULTI>
__global__ __launch_bounds__(1024) void gemm_decode_slice_kernel(const DecodeArgs a, int total_tiles) {
    extern __shared__ __align__(16) unsigned char smem[];
    constexpr int kPre = TL >= 4 ? 2 : 1;
    // a wavefront's own LDS: first the operand staging of its slice (2 KiB per chunk), then its partial sums (1 KiB per tile)
    constexpr int kWaveInts = (KPW * 2048 > TL * 1024 ? KPW * 2048 : TL * 1024) / 4;
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int KT = a.KT;
    // every argument in scalar registers up front (one round of scalar loads), picked by comparisons later:
    // an indexed read of the argument record would be a dependent load in the middle of the kernel
    const int t1 = a.tile_start[1], t2 = a.tile_start[2], t3 = a.tile_start[3];
    const uint4 *bl0 = a.blob4[0], *bl1 = a.blob4[1], *bl2 = a.blob4[2], *bl3 = a.blob4[3];
    const __half *sc0 = a.sw4[0], *sc1 = a.sw4[1], *sc2 = a.sw4[2], *sc3 = a.sw4[3];
    const int n0 = a.N4[0], n1 = a.N4[1], n2 = a.N4[2], n3 = a.N4[3];
    __half *const y0 = a.y4[0], *const y1 = a.y4[1], *const y2 = a.y4[2], *const y3 = a.y4[3];
    int32_t *const ac0 = a.acc4[0], *const ac1 = a.acc4[1], *const ac2 = a.acc4[2], *const ac3 = a.acc4[3];
    const int ld0 = a.ldy4[0], ld1 = a.ldy4[1], ld2 = a.ldy4[2], ld3 = a.ldy4[3];
    asm volatile("" ::"s"(a.x), "s"(a.ldx), "s"(a.M), "s"(KT), "s"(t1), "s"(t2), "s"(t3), "s"(a.scale_e), "s"(bl0),
                 "s"(bl1), "s"(bl2), "s"(bl3), "s"(sc0), "s"(sc1), "s"(sc2), "s"(sc3), "s"(n0), "s"(n1), "s"(n2), "s"(n3),
                 "s"(a.q.h_scale2), "s"(a.q.h_lo2), "s"(a.q.h_hi2), "s"(ZP ? a.q.h_zp2 : 0u), "s"(ZP ? a.corr : 0));
    asm volatile("" ::"s"(y0), "s"(y1), "s"(y2), "s"(y3), "s"(ac0), "s"(ac1), "s"(ac2), "s"(ac3), "s"(ld0), "s"(ld1),
                 "s"(ld2), "s"(ld3));
    int *const mine = reinterpret_cast<int *>(smem) + wave * kWaveInts;
    agq_u4 *const stage = reinterpret_cast<agq_u4 *>(mine);
    const int G = (int)gridDim.x;
    const int first = (int)blockIdx.x;
    const int my_tiles = (total_tiles - first + G - 1) / G;   // at least one; at most TL unless MULTI
    // (macros, not lambdas: a lambda that selects among the captured values makes them addressable,
    // and the argument record and these locals then live in scratch memory)
#define AGQ_SLICE_PROJ(tile, pj, nt)                                                                       \
    const int pj = __builtin_amdgcn_readfirstlane(((tile) >= t1) + ((tile) >= t2) + ((tile) >= t3));       \
    const int nt = (tile) - (pj == 0 ? 0 : (pj == 1 ? +t1 : (pj == 2 ? +t2 : +t3)))
#define AGQ_SLICE_PICK(pj, v0, v1, v2, v3) (pj == 0 ? +(v0) : (pj == 1 ? +(v1) : (pj == 2 ? +(v2) : +(v3))))
    const int kb = wave * KPW;
    const int c16 = lane & 15, rr = lane >> 4;
    const int s = c16 >> 3, g = (c16 & 7) >> 1, hf = c16 & 1;

    // the channel scales of the tile this wavefront will finish (tile `wave` of the workgroup's first TL): lane l
    // holds channel l & 15.  Kept as the 16 bits that were loaded: widening it here would wait for it here.
    const int tile_f = first + G * min(wave, my_tiles - 1);
    AGQ_SLICE_PROJ(tile_f, pj_f, nt_f);
    const int pN_f = AGQ_SLICE_PICK(pj_f, n0, n1, n2, n3);
    const unsigned short sw_u =
        reinterpret_cast<const uint16_t *>(AGQ_SLICE_PICK(pj_f, sc0, sc1, sc2, sc3))[min(nt_f * 16 + c16, pN_f - 1)];

    // the activation slice: unit = (chunk, pass of four rows), lane = eight consecutive k of one row
    agq_u4 xv[KPW][MP];
#pragma unroll
    for (int i = 0; i < KPW; ++i)
#pragma unroll
        for (int it = 0; it < MP; ++it) {
            const __half *xh = reinterpret_cast<const __half *>(a.x) + (int64_t)min(kb + i, KT - 1) * 128 + c16 * 8;
            xv[i][it] = *reinterpret_cast<const agq_u4 *>(xh + (int64_t)min(it * 4 + rr, a.M - 1) * a.ldx);
        }
    // the weight chunks of tile b; past the workgroup's last tile: the same number of loads, all lanes on one line
    agq_u4 ring[TL][KPW];
#define AGQ_SLICE_ISSUE(b, idx)                                                                                       \
    do {                                                                                                              \
        const bool real = (idx) < my_tiles;                                                                           \
        const int tile_i = first + G * (real ? (idx) : my_tiles - 1);                                                 \
        AGQ_SLICE_PROJ(tile_i, pj_i, nt_i);                                                                           \
        const uint4 *const blob_i = AGQ_SLICE_PICK(pj_i, bl0, bl1, bl2, bl3);                                         \
        const agq_u4 *p_i = reinterpret_cast<const agq_u4 *>(blob_i) + ((int64_t)nt_i * KT) * 64 + (real ? lane : 0); \
        const int stride_i = real ? 64 : 0;                                                                           \
        _Pragma("unroll") for (int i = 0; i < KPW; ++i) ring[b][i] = p_i[(int64_t)min(kb + i, KT - 1) * stride_i];    \
    } while (0)
#pragma unroll
    for (int b = 0; b < kPre; ++b) AGQ_SLICE_ISSUE(b, b);

    // Eq.2 on the slice, into the staging area in MFMA operand order; rows past M repeat the last row (never stored)
#pragma unroll
    for (int i = 0; i < KPW; ++i)
#pragma unroll
        for (int it = 0; it < MP; ++it) {
            const agq_u2 codes = quant8v<ZP>(xv[i][it], a.q);
            reinterpret_cast<agq_u2 *>(stage + i * 128 + s * 64 + g * 16 + it * 4 + rr)[hf] = codes;
        }
    // the same wavefront wrote and now reads: LDS keeps program order per wave
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
    agq_v4i fa0[KPW], fa1[KPW];
#pragma unroll
    for (int i = 0; i < KPW; ++i) {
        fa0[i] = __builtin_bit_cast(agq_v4i, stage[i * 128 + lane]);
        fa1[i] = __builtin_bit_cast(agq_v4i, stage[i * 128 + 64 + lane]);
    }
    asm volatile("" ::"v"(fa0[0]), "v"(fa1[0]));   // read before the rest of the requests, which can stall at issue
#pragma unroll
    for (int b = kPre; b < TL; ++b) AGQ_SLICE_ISSUE(b, b);

    // this wavefront's slice of the tile in slot b, times the activation slice, into its partial-sum area
#define AGQ_SLICE_TILE(b)                                                                                   \
    do {                                                                                                    \
        agq_v4i acc0 = {0, 0, 0, 0}, acc1 = {0, 0, 0, 0};                                                   \
        _Pragma("unroll") for (int i = 0; i < KPW; ++i) {                                                   \
            const agq_u4 wv = kb + i < KT ? ring[b][i] : agq_u4{0u, 0u, 0u, 0u};                            \
            const agq_v4i b0 = __builtin_bit_cast(agq_v4i, (wv << 4) & 0xF0F0F0F0u);                        \
            const agq_v4i b1 = __builtin_bit_cast(agq_v4i, wv & 0xF0F0F0F0u);                               \
            acc0 = __builtin_amdgcn_mfma_i32_16x16x64_i8(fa0[i], b0, acc0, 0, 0, 0);                        \
            acc1 = __builtin_amdgcn_mfma_i32_16x16x64_i8(fa1[i], b1, acc1, 0, 0, 0);                        \
        }                                                                                                   \
        const agq_v4i acc = acc0 + acc1;                                                                    \
        _Pragma("unroll") for (int r = 0; r < 4; ++r) mine[(b) * 256 + r * 64 + lane] = acc[r];             \
    } while (0)
    // Wavefront w < TL finishes tile base + w of the workgroup (slot w of the round): lane l takes the four
    // channels 4 (l & 3) .. + 3 of row l >> 2; in the accumulator layout row m sits in register m & 3 of the
    // lanes 16 (m >> 2) + channel, so four neighbouring channels are one 16-byte read.  MULTI: the next
    // round's weight chunks are in registers already, so four reads in flight, not sixteen.
#define AGQ_SLICE_FINISH(base, swv)                                                                                        \
    do {                                                                                                                   \
        if (wave < TL && (base) + wave < my_tiles) {                                                                       \
            const int tile_e = first + G * ((base) + wave);                                                                \
            AGQ_SLICE_PROJ(tile_e, pj_e, nt_e);                                                                            \
            const int pN_e = AGQ_SLICE_PICK(pj_e, n0, n1, n2, n3);                                                         \
            const int *rb = reinterpret_cast<const int *>(smem) + wave * 256;                                              \
            const int m = lane >> 2, c0 = (lane & 3) * 4;                                                                  \
            const int lsrc = 16 * (m >> 2) + c0, r = m & 3;                                                                \
            agq_v4i sum = {0, 0, 0, 0};                                                                                    \
            _Pragma("unroll") for (int w = 0; w < 16; ++w) {                                                               \
                sum += *reinterpret_cast<const agq_v4i *>(rb + w * kWaveInts + r * 64 + lsrc);                             \
                if (MULTI && (w & 3) == 3) asm volatile("" : "+v"(sum)::"memory");                                         \
            }                                                                                                              \
            const int n = nt_e * 16 + c0;                                                                                  \
            uint32_t h[4];                                                                                                 \
            int v4[4];                                                                                                     \
            _Pragma("unroll") for (int i = 0; i < 4; ++i) {                                                                \
                int v = sum[i] >> AGQ_W_SHIFT; /* exact: every term carries the factor */                                  \
                if (ZP)                                                                                                    \
                    v += a.corr * blob_wsum(AGQ_SLICE_PICK(pj_e, bl0, bl1, bl2, bl3), pN_e, KT)[min(n + i, pN_e - 1)];     \
                v4[i] = v;                                                                                                 \
                const unsigned short sb = (unsigned short)__shfl((int)(swv), c0 + i); /* channel c0 + i: lane c0 + i */    \
                h[i] = __half_as_ushort(agq_dequant(v, a.scale_e * __half2float(__ushort_as_half(sb))));                   \
            }                                                                                                              \
            int32_t *const pacc = AGQ_SLICE_PICK(pj_e, ac0, ac1, ac2, ac3);                                                \
            __half *const py = AGQ_SLICE_PICK(pj_e, y0, y1, y2, y3);                                                       \
            const int pldy = AGQ_SLICE_PICK(pj_e, ld0, ld1, ld2, ld3);                                                     \
            if (m < a.M) {                                                                                                 \
                if (n + 3 < pN_e && (pldy & 3) == 0 && (reinterpret_cast<uintptr_t>(py) & 7) == 0) {                       \
                    *reinterpret_cast<uint2 *>(py + (int64_t)m * pldy + n) =                                               \
                        make_uint2(h[0] | (h[1] << 16), h[2] | (h[3] << 16));                                              \
                } else {                                                                                                   \
                    for (int i = 0; i < 4 && n + i < pN_e; ++i)                                                            \
                        py[(int64_t)m * pldy + n + i] = __ushort_as_half((unsigned short)h[i]);                            \
                }                                                                                                          \
                if (pacc)                                                                                                  \
                    for (int i = 0; i < 4 && n + i < pN_e; ++i) pacc[(int64_t)m * pN_e + n + i] = v4[i];                   \
            }                                                                                                              \
        }                                                                                                                  \
    } while (0)

    int base = 0;
    unsigned short sw_cur = sw_u;
    if (MULTI) {
        // Full rounds, no way out of the middle of one: the same loads on every path, so the waits stay exact
        // across the loop.  A slot is requested again, for the next round, right behind its product; the scales
        // for the next round's epilogue a round ahead (by every wavefront: those that finish no tile read the
        // scales of the workgroup's last tile).
        for (; base + TL <= my_tiles; base += TL) {
            const int tile_n = first + G * min(base + TL + wave, my_tiles - 1);
            AGQ_SLICE_PROJ(tile_n, pj_n, nt_n);
            const int pN_n = AGQ_SLICE_PICK(pj_n, n0, n1, n2, n3);
            const unsigned short sw_nxt =
                reinterpret_cast<const uint16_t *>(AGQ_SLICE_PICK(pj_n, sc0, sc1, sc2, sc3))[min(nt_n * 16 + c16, pN_n - 1)];
#pragma unroll
            for (int b = 0; b < TL; ++b) {
                AGQ_SLICE_TILE(b);
                AGQ_SLICE_ISSUE(b, base + TL + b);
            }
            lds_barrier();
            AGQ_SLICE_FINISH(base, sw_cur);
            lds_barrier();   // the partial sums are read before the next round overwrites them
            sw_cur = sw_nxt;
        }
    }
    // The last round (the only one unless MULTI): up to TL tiles.  The loop is left, not skipped through: with a
    // skip the compiler would have to assume, at every later tile, the path on which fewer loads are outstanding,
    // and wait for more than the tile's own chunks.
#pragma unroll
    for (int b = 0; b < TL; ++b) {
        if (base + b >= my_tiles) goto tiles_done;
        AGQ_SLICE_TILE(b);
    }
tiles_done:
    lds_barrier();
    AGQ_SLICE_FINISH(base, sw_cur);
#undef AGQ_SLICE_TILE
#undef AGQ_SLICE_FINISH
#undef AGQ_SLICE_ISSUE
#undef AGQ_SLICE_PROJ
#undef AGQ_SLICE_PICK
}

// One token row, fp16 input on the signed grid, no matrix core and no LDS staging: the vector-ALU form of the
// product (what the 4-bit multiplier of the paper's appendix stands for on this chip).  A lane owns the 32 weights
// of one output channel that its 16 bytes of a chunk hold, loads the 32 activation values they meet (the sixteen
// lanes of a k group read the same addresses, which the memory pipeline merges), applies Eq.2 to them in registers
// and multiplies with v_dot4_i32_i8 (8-bit activations: the nibbles widened to 16 w as in the other kernels) or
// v_dot8_i32_i4 (4-bit activations: code nibbles paired up in the weights' own order, no widening at all).  The four
// k groups of a channel are joined by two lane shuffles, the wavefronts by one small LDS reduction.
template <int BITS, int KPW>
__global__ __launch_bounds__(1024) void gemm_decode_dot_kernel(const DecodeArgs a) {
    __shared__ int red[16 * 16];   // [wavefront][channel]
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int nwaves = a.waves;
    const int KT = a.KT;
    int nt;
    const int pj = find_proj(a, blockIdx.x, nt);
    const DecodeProj pr = load_proj(a, pj);
    const agq_u4 *wptr = reinterpret_cast<const agq_u4 *>(pr.blob) + (int64_t)nt * KT * 64 + lane;
    const int g = lane >> 4;
    const __half *xg = reinterpret_cast<const __half *>(a.x) + 16 * g;
    int acc = 0;
    for (int kb = wave * KPW; kb < KT; kb += nwaves * KPW) {
        agq_u4 w[KPW];
#pragma unroll
        for (int i = 0; i < KPW; ++i) w[i] = wptr[(int64_t)min(kb + i, KT - 1) * 64];
        constexpr int XB = KPW < 2 ? KPW : 2;          // chunks of activation in registers at a time
#pragma unroll
        for (int i0 = 0; i0 < KPW; i0 += XB) {
            agq_u4 xv[XB][4];
#pragma unroll
            for (int i = 0; i < XB; ++i) {
                const __half *xh = xg + (int64_t)min(kb + i0 + i, KT - 1) * 128;
                xv[i][0] = *reinterpret_cast<const agq_u4 *>(xh);        // k = 16 g + 0..7 of the chunk
                xv[i][1] = *reinterpret_cast<const agq_u4 *>(xh + 8);    //     16 g + 8..15
                xv[i][2] = *reinterpret_cast<const agq_u4 *>(xh + 64);   //     64 + 16 g + 0..7
                xv[i][3] = *reinterpret_cast<const agq_u4 *>(xh + 72);   //     64 + 16 g + 8..15
            }
#pragma unroll
            for (int i = 0; i < XB; ++i) {
                const bool valid = kb + i0 + i < KT;                      // wave-uniform
                const agq_u2 c0 = quant8v<false>(xv[i][0], a.q), c1 = quant8v<false>(xv[i][1], a.q);
                const agq_u2 c2 = quant8v<false>(xv[i][2], a.q), c3 = quant8v<false>(xv[i][3], a.q);
                const uint32_t lo[4] = {c0.x, c0.y, c1.x, c1.y}, hi[4] = {c2.x, c2.y, c3.x, c3.y};
                const agq_u4 wv = valid ? w[i0 + i] : agq_u4{0u, 0u, 0u, 0u};
#pragma unroll
                for (int d = 0; d < 4; ++d) {
                    if (BITS == 8) {
                        acc = __builtin_amdgcn_sdot4((int)lo[d], (int)((wv[d] << 4) & 0xF0F0F0F0u), acc, false);
                        acc = __builtin_amdgcn_sdot4((int)hi[d], (int)(wv[d] & 0xF0F0F0F0u), acc, false);
                    } else {
                        // byte j of the weight word: low nibble k = 4 d + j, high nibble k = 64 + 4 d + j
                        const uint32_t pair = (lo[d] & 0x0F0F0F0Fu) | ((hi[d] << 4) & 0xF0F0F0F0u);
                        acc = __builtin_amdgcn_sdot8((int)pair, (int)wv[d], acc, false);
                    }
                }
            }
        }
    }
    acc += __shfl_xor(acc, 16);
    acc += __shfl_xor(acc, 32);
    if (lane < 16) red[wave * 16 + lane] = acc;
    __syncthreads();
    if (threadIdx.x < 16) {
        const int n = nt * 16 + lane;
        if (n < pr.N) {
            int sum = 0;
            for (int wv = 0; wv < nwaves; ++wv) sum += red[wv * 16 + lane];
            const int v = BITS == 8 ? sum >> AGQ_W_SHIFT : sum;   // exact: the widened weights carry the factor
            if (pr.acc_out) pr.acc_out[n] = v;
            pr.y[n] = agq_dequant(v, a.scale_e * __half2float(pr.sw[n]));
        }
    }
}

template <int BITS>
int launch_dot(const DecodeArgs &a, int kpw, unsigned grid, int waves, hipStream_t st) {
    switch (kpw) {
        case 1: gemm_decode_dot_kernel<BITS, 1><<<grid, waves * 64, 0, st>>>(a); break;
        case 2: gemm_decode_dot_kernel<BITS, 2><<<grid, waves * 64, 0, st>>>(a); break;
        case 4: gemm_decode_dot_kernel<BITS, 4><<<grid, waves * 64, 0, st>>>(a); break;
        default: gemm_decode_dot_kernel<BITS, 8><<<grid, waves * 64, 0, st>>>(a); break;
    }
    return (int)hipGetLastError();
}

// More than 48 KiB of dynamic LDS needs the limit of the kernel raised: a host-side setting per device and
// kernel, not a stream operation.  Every instantiation is raised once per device, on the first weight-streaming
// launch of any shape made with that device current (so a caller never meets it in the middle of a run).
template <int KPW, int TL, bool ZP>
hipError_t raise_slice_lds() {
    hipError_t err = hipSuccess;
    const void *const kernels[4] = {reinterpret_cast<const void *>(gemm_decode_slice_kernel<KPW, 2, TL, ZP, false>),
                                    reinterpret_cast<const void *>(gemm_decode_slice_kernel<KPW, 4, TL, ZP, false>),
                                    reinterpret_cast<const void *>(gemm_decode_slice_kernel<KPW, 2, TL, ZP, true>),
                                    reinterpret_cast<const void *>(gemm_decode_slice_kernel<KPW, 4, TL, ZP, true>)};
    for (int i = 0; i < 4 && err == hipSuccess; ++i)
        err = hipFuncSetAttribute(kernels[i], hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024 - 512);
    return err;
}

constexpr int kMaxDevices = 64;
std::once_flag g_lds_once[kMaxDevices];
hipError_t g_lds_err[kMaxDevices];

int ensure_lds_limits() {
    int device = 0;
    if (hipGetDevice(&device) != hipSuccess) return (int)hipGetLastError();
    if (device < 0 || device >= kMaxDevices) return (int)hipErrorInvalidDevice;
    std::call_once(g_lds_once[device], [device] {
        hipError_t err = raise_slice_lds<1, 6, false>();
        if (err == hipSuccess) err = raise_slice_lds<2, 6, false>();
        if (err == hipSuccess) err = raise_slice_lds<3, 6, false>();
        if (err == hipSuccess) err = raise_slice_lds<4, 3, false>();
        if (err == hipSuccess) err = raise_slice_lds<1, 6, true>();
        if (err == hipSuccess) err = raise_slice_lds<2, 6, true>();
        if (err == hipSuccess) err = raise_slice_lds<3, 6, true>();
        if (err == hipSuccess) err = raise_slice_lds<4, 3, true>();
        g_lds_err[device] = err;
    });
    return (int)g_lds_err[device];
}

// chunks of K per wavefront -> tiles a workgroup can hold (registers: TL x KPW weight chunks per lane)
constexpr int slice_tiles(int kpw) { return kpw <= 3 ? 6 : 3; }

template <int KPW, bool ZP>
int launch_slice_kpw(const DecodeArgs &a, int tiles, hipStream_t st) {
    constexpr int TL = slice_tiles(KPW);
    constexpr size_t lds = 16 * (size_t)(KPW * 2048 > TL * 1024 ? KPW * 2048 : TL * 1024);
    if (tiles <= 256 * TL) {
        if (a.M <= 8) gemm_decode_slice_kernel<KPW, 2, TL, ZP, false><<<256, 1024, lds, st>>>(a, tiles);
        else gemm_decode_slice_kernel<KPW, 4, TL, ZP, false><<<256, 1024, lds, st>>>(a, tiles);
    } else {
        if (a.M <= 8) gemm_decode_slice_kernel<KPW, 2, TL, ZP, true><<<256, 1024, lds, st>>>(a, tiles);
        else gemm_decode_slice_kernel<KPW, 4, TL, ZP, true><<<256, 1024, lds, st>>>(a, tiles);
    }
    return (int)hipGetLastError();
}

template <bool ZP>
int launch_slice(const DecodeArgs &a, int kpw, int tiles, hipStream_t st) {
    switch (kpw) {
        case 1: return launch_slice_kpw<1, ZP>(a, tiles, st);
        case 2: return launch_slice_kpw<2, ZP>(a, tiles, st);
        case 3: return launch_slice_kpw<3, ZP>(a, tiles, st);
        default: return launch_slice_kpw<4, ZP>(a, tiles, st);
    }
}

// more than sixteen rows: sixteen per workgroup, grid.y row groups (fp16 input, four passes of four rows)
template <int XK>
int launch_rg(const DecodeArgs &a, int kpw, unsigned grid, unsigned groups, int waves, size_t lds, hipStream_t st) {
    const dim3 g(grid, groups);
    switch (kpw) {
        case 1: gemm_decode_kernel<XK, 1, 4, true><<<g, waves * 64, lds, st>>>(a); break;
        case 2: gemm_decode_kernel<XK, 2, 4, true><<<g, waves * 64, lds, st>>>(a); break;
        case 4: gemm_decode_kernel<XK, 4, 4, true><<<g, waves * 64, lds, st>>>(a); break;
        default: gemm_decode_kernel<XK, 8, 4, true><<<g, waves * 64, lds, st>>>(a); break;
    }
    return (int)hipGetLastError();
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

int agq_launch_gemm_decode(const void *x, int x_kind, int bits, int64_t M, int64_t K, int64_t ldx, int e, int zp,
                           const agq_proj *projs, int count, int n_extra, void *stream) {
    if (const int err = ensure_lds_limits()) return err;
    DecodeArgs a = {};
    a.x = x;
    a.ldx = ldx;
    a.M = (int)M;
    a.KT = (int)agq_k_tiles(K);
    a.count = count;
    a.waves = 0;
    a.q = agq_make_quant_signed(bits, e, zp);
    a.corr = agq_zp_corr(bits, zp);
    a.flip = zp ? (bits == 8 ? 0x80808080u : 0x88888888u) : 0u;
    a.scale_e = ldexpf(1.0f, e);
    a.n_extra = n_extra > 0 ? n_extra : 0;
    const bool trip = n_extra >= 0;
    int tiles = 0;
    for (int p = 0; p < kMaxProj; ++p) {
        const agq_proj &pr = projs[p < count ? p : count - 1];
        a.tile_start[p] = tiles;
        // row groups (more than sixteen rows): a workgroup serves a pair of tiles
        if (p < count) tiles += M > AGQ_DECODE_MAX_M ? (int)((pr.N + 31) / 32) : (int)((pr.N + 15) / 16);
        a.blob4[p] = (const uint4 *)pr.w_packed;
        a.sw4[p] = (const __half *)pr.w_scale_f16;
        a.N4[p] = (int)pr.N;
        a.y4[p] = (__half *)pr.y_f16;
        a.acc4[p] = pr.acc_out;
        a.ldy4[p] = (int)pr.ldy;
    }
    a.tile_start[kMaxProj] = tiles;
    for (int p = count; p <= kMaxProj; ++p) a.tile_start[p] = tiles;
    // chunks per wavefront: the smallest of 1, 2, 4, 8 that needs at most 8
    // wavefronts (16 for the largest); very long K loops inside the kernel
    int kpw = 1;
    while (kpw < 8 && (a.KT + kpw - 1) / kpw > 8) kpw *= 2;
    int waves = (a.KT + kpw - 1) / kpw;
    if (waves > 16) waves = 16;
    if (x_kind == 0 && ((M > 4 && tiles <= 256) || a.KT > 64)) {
        // Several token rows with one workgroup per CU, or a long K: the Eq.2 prologue
        // weighs more, so spread it over as many wavefronts as a workgroup holds (K in
        // rounds when it is very long).  Measured: faster than eight fatter wavefronts
        // in exactly these cases; with several workgroups per CU and K <= 8192 the
        // smaller workgroups win.
        kpw = 1;
        while (kpw < 4 && (a.KT + kpw - 1) / kpw > 16) kpw *= 2;
        waves = (a.KT + kpw - 1) / kpw;
        if (waves > 16) waves = 16;
    }
    if (M > AGQ_DECODE_MAX_M && kpw == 8) {
        // row groups keep two tiles' weight chunks in registers: four chunks per wavefront at most
        kpw = 4;
        waves = (a.KT + kpw - 1) / kpw;
        if (waves > 16) waves = 16;
    }
    if (trip) {
        // one more wavefront for the extra chunks: at most 15 for the main ones
        if (waves > 15) {
            kpw = 1;
            while (kpw < 8 && (a.KT + kpw - 1) / kpw > 15) kpw *= 2;
            waves = (a.KT + kpw - 1) / kpw;
            if (waves > 15) waves = 15;
        }
        waves += 1;
    }
    const unsigned grid = (unsigned)tiles;
    a.waves = waves;
    // staging: per wavefront HB chunks x (8 x 4 MP) 16-byte pieces (see the kernel)
    const int mp = M <= 4 ? 1 : (M <= 8 ? 2 : 4);
    const int hb = x_kind != 0 ? kpw : (8 / mp < kpw ? 8 / mp : kpw);
    const size_t per_wave = x_kind != 0 ? 0 : (size_t)hb * 8 * 4 * mp * 16;
    // behind the staging regions: one KiB of partial sums per wavefront and channel tile
    const size_t lds = (size_t)waves * (per_wave + (M > AGQ_DECODE_MAX_M ? 2048 : 1024));
    hipStream_t st = (hipStream_t)stream;
    if (x_kind == AGQ_X_F16_DOT)   // the caller's choice (checked there: one row, signed grid, plain blobs)
        return bits == 8 ? launch_dot<8>(a, kpw, grid, waves, st) : launch_dot<4>(a, kpw, grid, waves, st);
    if (M > AGQ_DECODE_MAX_M) {   // row groups (the caller has checked: fp16 input, plain blobs)
        const unsigned groups = (unsigned)((M + 15) / 16);
        if (zp) return launch_rg<XK_F16_Z>(a, kpw, grid, groups, waves, lds, st);
        return launch_rg<XK_F16>(a, kpw, grid, groups, waves, lds, st);
    }
    if (trip) {
        if (zp) {
            if (M <= 4) return launch_xk<XK_F16_TZ, 1>(a, kpw, grid, waves, lds, st);
            if (M <= 8) return launch_xk<XK_F16_TZ, 2>(a, kpw, grid, waves, lds, st);
            return launch_xk<XK_F16_TZ, 4>(a, kpw, grid, waves, lds, st);
        }
        if (M == 1) return launch_xk<XK_F16_ONE_T, 1>(a, kpw, grid, waves, lds, st);
        if (M <= 4) return launch_xk<XK_F16_T, 1>(a, kpw, grid, waves, lds, st);
        if (M <= 8) return launch_xk<XK_F16_T, 2>(a, kpw, grid, waves, lds, st);
        return launch_xk<XK_F16_T, 4>(a, kpw, grid, waves, lds, st);
    }
    // K split over the wavefronts of one workgroup per CU, up to six of its tiles in flight at once: from nine
    // rows on whenever a CU has more than one tile, at five to eight rows from three tiles per CU on (eight rows,
    // K = 4096, q/k/v: 8.1 against 10.1 us for one workgroup per tile; at two tiles per CU the two are level);
    // in rounds when a CU has more tiles than a workgroup holds.  Measured at sixteen rows against the kernel
    // this one replaced (the whole quantized activation in LDS, the tiles one after another with two meetings per
    // tile): K = 4096 q/k/v 10.2 -> 9.3 us, gate/up 14.2 -> 13.2; K = 5120, N = 27648: 21.9 -> 20.0; K = 8192,
    // N = 28672: 30.4 -> 26.1.  Below five rows the per-tile prologue, which overlaps better with the weight
    // stream, is faster (four rows, q/k/v: 7.4 against 8.6 us).
    if (x_kind == 0 && a.KT <= kSliceMaxKT && M > 4) {
        const int skpw = (a.KT + 15) / 16;
        if (tiles > (M > 8 ? 256 : 512))
            return zp ? launch_slice<true>(a, skpw, tiles, st) : launch_slice<false>(a, skpw, tiles, st);
    }
    if (x_kind == 0) {
        if (zp) {
            if (M == 1) return launch_xk<XK_F16_ONE_Z, 1>(a, kpw, grid, waves, lds, st);
            if (M <= 4) return launch_xk<XK_F16_Z, 1>(a, kpw, grid, waves, lds, st);
            if (M <= 8) return launch_xk<XK_F16_Z, 2>(a, kpw, grid, waves, lds, st);
            return launch_xk<XK_F16_Z, 4>(a, kpw, grid, waves, lds, st);
        }
        if (M == 1) return launch_xk<XK_F16_ONE, 1>(a, kpw, grid, waves, lds, st);
        if (M <= 4) return launch_xk<XK_F16, 1>(a, kpw, grid, waves, lds, st);
        if (M <= 8) return launch_xk<XK_F16, 2>(a, kpw, grid, waves, lds, st);
        return launch_xk<XK_F16, 4>(a, kpw, grid, waves, lds, st);
    }
    if (bits == 8) return launch_xk<XK_I8, 1>(a, kpw, grid, waves, lds, st);
    return launch_xk<XK_I4, 1>(a, kpw, grid, waves, lds, st);
}
