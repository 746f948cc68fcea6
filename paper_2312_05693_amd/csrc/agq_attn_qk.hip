// Attention from quantized Q and K in one kernel: integer Q K^T on the int8
// matrix cores (Section 4.2 lists QK among the quantized products), softmax in
// floating point (Section 3.3: non-linear operators stay in floating point),
// Eq.3 (Section 4.1) on the probabilities, the product with the int8 value
// matrix, and the importance of every token on the quantized map (Section 4.3).
// The probabilities never exist in memory.
//
//   s[i,j] = sum_d q[i,d] k[j,d]                         (int32, exact)
//   t[i,j] = -log2 softmax_j(s 2^(e_q+e_k) / sqrt(D)) = L[i] - kappa s[i,j],
//            kappa = 2^(e_q+e_k) log2(e) / sqrt(D),  L[i] = log2 sum_j 2^(kappa s[i,j])
//   c[i,j] = CLIP(round(t), 0, qmax),   o[i,:] = 2^(e_v-qmax) sum_j 2^(qmax-c[i,j]) v[j,:]
//
// Two passes over the key tiles of a 128-row block: the first keeps a running
// maximum and sum per row (L), the second recomputes the scores, turns them
// into the weights 2^(qmax-c) and multiplies.  L and t are evaluated in fp32
// (hardware exp2 / log2), so a code can differ from a float64 evaluation where t
// lies within ~1e-5 of a rounding boundary; everything after the codes is exact.
//
// Scores are computed transposed, S^T = K Q^T, with the 32x32x32 int8 MFMA: a lane
// then holds, for its query (column l & 31), the keys 8 q + 4 g + r (g = l >> 5,
// register 4 q + r) of a 32-key sub-tile - which is already the layout of the
// first operand of the 32x32x16 fp16 MFMA if its sixteen k slots are dealt to keys
// in that order (slot 8 g + 4 q' + r of step u <-> key 16 u + 8 q' + 4 g + r).  The
// V tile in LDS is written in that slot order, so no shuffle is needed between
// the two products.
#include "agq_device.h"
#include "agq_internal.h"

#include <math.h>

#include <type_traits>

typedef _Float16 agq_v8h __attribute__((ext_vector_type(8)));
typedef _Float16 agq_v2h __attribute__((ext_vector_type(2)));
typedef float agq_v16f __attribute__((ext_vector_type(16)));
typedef int agq_v16i __attribute__((ext_vector_type(16)));
typedef uint32_t agq_u4 __attribute__((ext_vector_type(4)));

namespace {

constexpr int kQRows = 128;     // query rows per workgroup (32 per wavefront)
constexpr int kKeys = 64;       // keys per tile: two 32-key sub-tiles
constexpr int kVRow = 144;      // bytes per channel row of the V tile: 64 key slots in fp16 + 16 of padding

struct QkArgs {
    const int8_t *q, *k, *v;   // [H,S,D] each
    __half *o;                 // [S, H*D]
    uint8_t *codes;            // [H,S,S/2] or null
    int32_t *score;            // [S] or null (accumulated with atomics: the caller zeroes it)
    int H, S;
    int causal, qmax;
    float kappa;               // 2^(e_q+e_k) log2(e) / sqrt(D)
    float out_scale;           // 2^(e_v - qmax)
    int ncu;
};

// DT = D / 32: int8 MFMA steps per score tile and 32-channel blocks of the output
template <int DT, bool CODES>
__global__ __launch_bounds__(256, 3) void qk_log2_attn_kernel(const QkArgs a) {
    constexpr int D = DT * 32, DQ = D / 4;
    constexpr int kKRow = D + 16;                                // bytes per key row of the K tile (padded)
    __shared__ __align__(16) uint8_t kt[kKeys * kKRow];          // one K tile: three workgroups fit a CU
    __shared__ __align__(16) uint8_t vt[2][D * kVRow];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int S = a.S, H = a.H;
    const int nb = S / kQRows;

    // workgroup -> (head, row block); causal blocks ranked by length and dealt so that
    // the workgroups a CU receives together carry equal work (see the other attention kernel)
    int rank = (int)blockIdx.x;
    if (a.causal) {
        const int run = rank / a.ncu, base = run * a.ncu;
        if (run & 1) rank = base + min(a.ncu, (int)gridDim.x - base) - 1 - (rank - base);
    }
    const int h = rank % H;
    const int b = a.causal ? nb - 1 - rank / H : rank / H;
    const int q0 = b * kQRows;
    const int r0 = q0 + wave * 32;
    const int row = r0 + (lane & 31);                            // this lane's query
    const int g = lane >> 5;
    const int nt = (a.causal ? q0 + kQRows : S) / kKeys;         // key tiles of the block
    const int wave_last = a.causal ? r0 + 31 : S - 1;            // tiles starting past this are dead for the wavefront
    const int wave_lim = a.causal ? r0 : S - 1;                  // a sub-tile reaching past this needs the mask

    const int8_t *qh = a.q + (int64_t)h * S * D;
    const int8_t *kh = a.k + (int64_t)h * S * D;
    const int8_t *vh = a.v + (int64_t)h * S * D;

    // Q: second operand of S^T = K Q^T (column = query l & 31, sixteen d of k-group g per step)
    agq_v4i qf[DT];
#pragma unroll
    for (int s = 0; s < DT; ++s) qf[s] = *reinterpret_cast<const agq_v4i *>(qh + (int64_t)row * D + 32 * s + 16 * g);

    // K tile: 64 keys x D bytes; thread = (key tid >> 2, quarter tid & 3 of the row)
    constexpr int KL = D / 64;                                   // 16-byte loads per thread
    agq_u4 kraw[KL];
    const int kkey = threadIdx.x >> 2, kpart = threadIdx.x & 3;
    auto load_k = [&](int t) {
#pragma unroll
        for (int i = 0; i < KL; ++i)
            kraw[i] = *reinterpret_cast<const agq_u4 *>(kh + (int64_t)(t * kKeys + kkey) * D + (kpart * KL + i) * 16);
    };
    auto store_k = [&](uint8_t *buf) {
#pragma unroll
        for (int i = 0; i < KL; ++i) *reinterpret_cast<agq_u4 *>(buf + kkey * kKRow + (kpart * KL + i) * 16) = kraw[i];
    };

    // V tile: int8 [key][d] -> fp16 [d][slot] in LDS.  A thread unit is (chunk of eight
    // slots, four channels); the eight slots of chunk ch = 4 sub + 2 u + g' hold the keys
    // 32 sub + 16 u + 8 (i >> 2) + 4 g' + (i & 3), i = 0..7 (see the header).
    uint32_t vraw[8];
    const bool vu_ok = (int)threadIdx.x < 8 * DQ;
    const int vu_c = threadIdx.x % DQ, vu_ch = vu_ok ? threadIdx.x / DQ : 0;
    auto load_v = [&](int t) {
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            const int key = t * kKeys + 32 * (vu_ch >> 2) + 16 * ((vu_ch >> 1) & 1) + 8 * (i >> 2) + 4 * (vu_ch & 1) + (i & 3);
            vraw[i] = *reinterpret_cast<const uint32_t *>(vh + (int64_t)key * D + 4 * vu_c);
        }
    };
    auto store_v = [&](uint8_t *buf) {
        const agq_v2h bias = {(_Float16)1152.0f, (_Float16)1152.0f};
        uint32_t x[8];
#pragma unroll
        for (int i = 0; i < 8; ++i) x[i] = vraw[i] ^ 0x80808080u;            // bytes v + 128
#pragma unroll
        for (int bb = 0; bb < 4; ++bb) {
            // halves 0x64uu = 1024 + (v + 128) of slots 2 i and 2 i + 1 of channel 4 c + bb
            const uint32_t sel = 0x0C000C00u | (uint32_t)bb | ((uint32_t)(4 + bb) << 16);
            agq_u4 out;
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const uint32_t w = __builtin_amdgcn_perm(x[2 * i + 1], x[2 * i], sel) | 0x64006400u;
                out[i] = __builtin_bit_cast(uint32_t, __builtin_bit_cast(agq_v2h, w) - bias);
            }
            if (vu_ok) *reinterpret_cast<agq_u4 *>(buf + (bb * DQ + vu_c) * kVRow + (vu_ch << 4)) = out;
        }
    };

    // scores of a 32-key sub-tile, transposed: register 4 q + r = key 8 q + 4 g + r, this lane's query
    auto scores = [&](const uint8_t *kbuf, int sub) {
        agq_v16i acc;
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[r] = 0;
#pragma unroll
        for (int s = 0; s < DT; ++s) {
            const agq_v4i kf = *reinterpret_cast<const agq_v4i *>(kbuf + (32 * sub + (lane & 31)) * kKRow + 32 * s + 16 * g);
            acc = __builtin_amdgcn_mfma_i32_32x32x32_i8(kf, qf[s], acc, 0, 0, 0);
        }
        return acc;
    };

    // both sub-tiles of a tile at once: two independent accumulation chains
    auto scores2 = [&](const uint8_t *kbuf, agq_v16i &acc0, agq_v16i &acc1) {
#pragma unroll
        for (int r = 0; r < 16; ++r) acc0[r] = acc1[r] = 0;
#pragma unroll
        for (int s = 0; s < DT; ++s) {
            const agq_v4i k0f = *reinterpret_cast<const agq_v4i *>(kbuf + (lane & 31) * kKRow + 32 * s + 16 * g);
            const agq_v4i k1f = *reinterpret_cast<const agq_v4i *>(kbuf + (32 + (lane & 31)) * kKRow + 32 * s + 16 * g);
            acc0 = __builtin_amdgcn_mfma_i32_32x32x32_i8(k0f, qf[s], acc0, 0, 0, 0);
            acc1 = __builtin_amdgcn_mfma_i32_32x32x32_i8(k1f, qf[s], acc1, 0, 0, 0);
        }
    };

    // ---- pass 1: per row the maximum score M (an integer) and sum_j 2^(kappa (s_j - M)).
    // Differences of scores are exact integers, so the only roundings are the product
    // with kappa and the exponential.
    constexpr int kMasked = -(1 << 30);                          // stands for -infinity (|s| < 2^23)
    int run_m = kMasked;
    float run_s = 0.f;
    auto stats = [&](agq_v16i acc, int kb, auto masked_tag) {
        constexpr bool MASKED = decltype(masked_tag)::value;
        if (MASKED) {                                            // diagonal sub-tile: keys past the query do not count
#pragma unroll
            for (int r = 0; r < 16; ++r)
                if (kb + 8 * (r >> 2) + 4 * g + (r & 3) > row) acc[r] = kMasked;
        }
        int mx = acc[0];
#pragma unroll
        for (int r = 1; r < 16; ++r) mx = max(mx, acc[r]);
        const int nm = max(run_m, mx);
        float add = 0.f;
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            const float term = __builtin_amdgcn_exp2f(a.kappa * (float)(acc[r] - nm));
            add += (MASKED && acc[r] == kMasked) ? 0.f : term;
        }
        // nothing counted so far (run_m == kMasked) means run_s == 0: the factor does not matter
        run_s = run_s * __builtin_amdgcn_exp2f(a.kappa * (float)(run_m - nm)) + add;
        run_m = nm;
    };
    load_k(0);
    for (int t = 0; t < nt; ++t) {
        uint8_t *kbuf = (t & 1) ? vt[0] : kt;                    // the V buffers are idle in this pass: two K tiles, one barrier
        store_k(kbuf);
        if (t + 1 < nt) load_k(t + 1);
        __syncthreads();
        const int k0 = t * kKeys;
        if (k0 > wave_last) continue;                            // wave-uniform; the barrier above was joined
        if (k0 + kKeys - 1 <= wave_lim) {
            // whole tile live for every row of the wavefront: 32 scores per lane, one rescale
            agq_v16i acc0, acc1;
            scores2(kbuf, acc0, acc1);
            int mx = max(acc0[0], acc1[0]);
#pragma unroll
            for (int r = 1; r < 16; ++r) mx = max(mx, max(acc0[r], acc1[r]));
            const int nm = max(run_m, mx);
            // kappa s - kappa M with one rounding of the product (|kappa s| stays far below 2^10,
            // so the difference is good to ~1e-5: enough for a sum of 2^x)
            const float nmf = -a.kappa * (float)nm;
            float add0 = 0.f, add1 = 0.f;
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                add0 += __builtin_amdgcn_exp2f(fmaf(a.kappa, (float)acc0[r], nmf));
                add1 += __builtin_amdgcn_exp2f(fmaf(a.kappa, (float)acc1[r], nmf));
            }
            run_s = run_s * __builtin_amdgcn_exp2f(a.kappa * (float)(run_m - nm)) + (add0 + add1);
            run_m = nm;
            continue;
        }
#pragma unroll
        for (int sub = 0; sub < 2; ++sub) {
            const int kb = k0 + 32 * sub;
            if (kb > wave_last) continue;
            const agq_v16i acc = scores(kbuf, sub);
            if (kb + 31 > wave_lim) stats(acc, kb, std::true_type{});
            else stats(acc, kb, std::false_type{});
        }
    }
    // the two lanes of a query (k-groups 0 and 1) join their halves; every row has its own key, so M is a real score
    const int om = __shfl_xor(run_m, 32);
    const float os = __shfl_xor(run_s, 32);
    const int M = max(run_m, om);
    // (a half with nothing counted has sum 0, whatever its factor)
    const float tot = run_s * __builtin_amdgcn_exp2f(a.kappa * (float)(run_m - M)) +
                      os * __builtin_amdgcn_exp2f(a.kappa * (float)(om - M));
    // -log2 p = t = kappa (M - s) + log2(tot).  The weight 2^(qmax - c) has the fp16 exponent field
    // 15 + qmax - c = round(15 + qmax - t) clamped to [15, 15 + qmax]: one fused multiply-add gives
    // 15 + qmax - t, adding 1.5 * 2^23 rounds it to an integer (ties to even: a tie has measure
    // zero and lies inside the evaluation error anyway) that sits in the low bits of the pattern.
    const float c2 = (float)(15 + a.qmax) - __builtin_amdgcn_logf(tot) - a.kappa * (float)M;   // v_log_f32: base 2

    // ---- pass 2: codes, weights, product with V
    // four accumulators: block n holds the channels 4 c + n (c = column l & 31 < D / 4)
    agq_v16f acc_o[4];
#pragma unroll
    for (int n = 0; n < 4; ++n)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc_o[n][r] = 0.f;
    const int bslot = min(lane & 31, DQ - 1);
    const uint32_t wtop = 15u + (uint32_t)a.qmax;                // exponent field of the weight of code 0
    const float elo = AGQ_MAGIC + 15.0f, ehi = AGQ_MAGIC + (float)(15 + a.qmax);

    auto weights = [&](const agq_v16i &acc, int kb, const uint8_t *vbuf, int sub, auto masked_tag) {
        constexpr bool MASKED = decltype(masked_tag)::value;
        uint32_t ex[16];       // bit patterns whose low byte is the exponent field of the weight (0 = weight 0)
        uint32_t cw[4] = {0, 0, 0, 0};                           // codes of keys 8 q + 4 g + r, r = 0..3, as nibbles
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            const float ef = __builtin_amdgcn_fmed3f(fmaf(a.kappa, (float)acc[r], c2) + AGQ_MAGIC, elo, ehi);
            uint32_t e = __float_as_uint(ef);                    // 0x4B400000 + exponent field
            if (MASKED && kb + 8 * (r >> 2) + 4 * g + (r & 3) > row) e = 0;
            ex[r] = e;
            if (CODES) cw[r >> 2] |= ((e & 0xFFu) ? wtop - (e & 0xFFu) : (uint32_t)a.qmax) << (4 * (r & 3));
            // importance on the quantized map: the weight of the first key (always live)
            if (r == 0 && a.score && kb == 0 && g == 0) atomicAdd(&a.score[row], 1 << ((int)(e & 0xFFu) - 15));
        }
        if (CODES) {
#pragma unroll
            for (int q = 0; q < 4; ++q)
                *reinterpret_cast<uint16_t *>(a.codes + ((int64_t)h * S + row) * (S >> 1) + ((kb + 8 * q + 4 * g) >> 1)) =
                    (uint16_t)cw[q];
        }
#pragma unroll
        for (int u = 0; u < 2; ++u) {
            // first operand: slots 8 g .. 8 g + 7 of step u = registers 8 u .. 8 u + 7, as fp16 bit patterns
            agq_u4 wq;
#pragma unroll
            for (int j = 0; j < 4; ++j)   // the shifts drop everything above the low byte's five bits
                wq[j] = ((ex[8 * u + 2 * j + 1] << 16) | ex[8 * u + 2 * j]) << 10;
            const agq_v8h af = __builtin_bit_cast(agq_v8h, wq);
            const int chunk = 4 * sub + 2 * u + g;
#pragma unroll
            for (int n = 0; n < 4; ++n) {
                const agq_v8h bf = *reinterpret_cast<const agq_v8h *>(vbuf + (n * DQ + bslot) * kVRow + (chunk << 4));
                acc_o[n] = __builtin_amdgcn_mfma_f32_32x32x16_f16(af, bf, acc_o[n], 0, 0, 0);
            }
        }
    };

    __syncthreads();                                             // pass 1 is done with the K tile
    load_k(0);
    load_v(0);
    for (int t = 0; t < nt; ++t) {
        uint8_t *vbuf = vt[t & 1];
        if (t > 0) __syncthreads();                              // everyone is done with the previous K tile
        store_k(kt);
        store_v(vbuf);
        if (t + 1 < nt) {
            load_k(t + 1);
            load_v(t + 1);
        }
        __syncthreads();
        const int k0 = t * kKeys;
        if (k0 > wave_last) continue;                            // wave-uniform; the barriers above were joined
        if (k0 + kKeys - 1 <= wave_lim) {                        // whole tile live: both sub-tiles' scores first
            agq_v16i acc0, acc1;
            scores2(kt, acc0, acc1);
            weights(acc0, k0, vbuf, 0, std::false_type{});
            weights(acc1, k0 + 32, vbuf, 1, std::false_type{});
            continue;
        }
#pragma unroll
        for (int sub = 0; sub < 2; ++sub) {
            const int kb = k0 + 32 * sub;
            if (kb > wave_last) continue;
            const agq_v16i acc = scores(kt, sub);
            if (kb + 31 > wave_lim) weights(acc, kb, vbuf, sub, std::true_type{});
            else weights(acc, kb, vbuf, sub, std::false_type{});
        }
    }

    // code map right of the last sub-tile this wavefront multiplied: all qmax
    if (CODES && a.causal) {
        const uint32_t fill = 0x11111111u * (uint32_t)a.qmax;
        uint8_t *dst = a.codes + ((int64_t)h * S + row) * (S >> 1);
        const int done = (wave_last / 32 + 1) * 32;             // first key past the wavefront's last sub-tile
        for (int k = done + g * 8; k < S; k += 16) *reinterpret_cast<uint32_t *>(dst + (k >> 1)) = fill;
    }

    // accumulator register 4 q + r holds query row 8 q + 4 g + r of the wavefront,
    // channel 4 c + n in block n: four consecutive channels per lane and row
    const int c = lane & 31;
#pragma unroll
    for (int q = 0; q < 4; ++q)
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            const int orow = r0 + 8 * q + 4 * g + r;
            __half hv[4];
#pragma unroll
            for (int n = 0; n < 4; ++n) hv[n] = __float2half_rn(acc_o[n][4 * q + r] * a.out_scale);
            if (c < DQ)
                *reinterpret_cast<uint2 *>(a.o + (int64_t)orow * ((int64_t)H * D) + (int64_t)h * D + 4 * c) =
                    *reinterpret_cast<const uint2 *>(hv);
        }
}

}  // namespace

int agq_launch_qk_log2_attn(const int8_t *q, const int8_t *k, const int8_t *v, int64_t H, int64_t S, int64_t D, int causal,
                            int qmax, int e_q, int e_k, int e_v, void *o, void *codes, int32_t *score, void *stream) {
    QkArgs a;
    a.q = q;
    a.k = k;
    a.v = v;
    a.o = (__half *)o;
    a.codes = (uint8_t *)codes;
    a.score = score;
    a.H = (int)H;
    a.S = (int)S;
    a.causal = causal;
    a.qmax = qmax;
    a.kappa = (float)(ldexp(1.0, e_q + e_k) * 1.4426950408889634 / sqrt((double)D));
    a.out_scale = ldexpf(1.0f, e_v - qmax);
    static int ncu_of[64] = {0};
    int device = 0;
    if (hipGetDevice(&device) != hipSuccess) return (int)hipGetLastError();
    int ncu = (device >= 0 && device < 64) ? ncu_of[device] : 0;
    if (ncu == 0) {
        if (hipDeviceGetAttribute(&ncu, hipDeviceAttributeMultiprocessorCount, device) != hipSuccess || ncu < 1) ncu = 256;
        if (device >= 0 && device < 64) ncu_of[device] = ncu;
    }
    a.ncu = ncu;
    hipStream_t st = (hipStream_t)stream;
    const unsigned grid = (unsigned)((S / kQRows) * H);
    if (D == 128) {
        if (codes) qk_log2_attn_kernel<4, true><<<grid, 256, 0, st>>>(a);
        else qk_log2_attn_kernel<4, false><<<grid, 256, 0, st>>>(a);
    } else {
        if (codes) qk_log2_attn_kernel<2, true><<<grid, 256, 0, st>>>(a);
        else qk_log2_attn_kernel<2, false><<<grid, 256, 0, st>>>(a);
    }
    return (int)hipGetLastError();
}
