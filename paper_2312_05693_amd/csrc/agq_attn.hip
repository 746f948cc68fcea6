// Log2-quantized softmax probabilities times the int8 value matrix, the
// start-token importance score, and token pruning.
//
// Eq.3 (Section 4.1) on a probability p = 2^E (1 + f) needs no logarithm:
// round(-log2 p) = -E when 1 + f < sqrt(2) and -E - 1 otherwise, and
// -log2 p is never half-way between integers for a rational p.  On fp16 bit
// patterns h (normal numbers) this is 15 - ((h + 599) >> 10): 1 + 425/1024 is
// the first mantissa above sqrt(2), and adding 1024 - 425 carries into the
// exponent field exactly from there on.  Subnormals (h < 1024, value h * 2^-24)
// round to 14 from h = 725 on, else to 15 or more.
//
// The product uses the fp16 MFMA with fp32 accumulation on the integers
// 2^(qmax - c) and v: every term and every partial sum is an integer below
// 2^24 for softmax rows, so the result is exact in any order.
#include "agq_device.h"
#include "agq_internal.h"

#include <type_traits>

typedef _Float16 agq_v8h __attribute__((ext_vector_type(8)));
typedef _Float16 agq_v2h __attribute__((ext_vector_type(2)));
typedef unsigned short agq_v2us __attribute__((ext_vector_type(2)));
typedef float agq_v16f __attribute__((ext_vector_type(16)));
typedef uint32_t agq_u4 __attribute__((ext_vector_type(4)));

namespace {

constexpr int kQRows = 128;     // query rows per workgroup (32 per wavefront)
constexpr int kKeys = 64;       // keys per tile: four MFMA steps of 16
constexpr int kVRow = 144;      // bytes per channel row of the V tile in LDS: 64 keys in fp16 + 16 of padding
constexpr int kMaxD = 256;

struct AttnArgs {
    const uint16_t *p;   // fp16 bits [H,S,S]
    const int8_t *v;     // [H,S,D]
    __half *o;           // [S, H*D]
    uint8_t *codes;      // [H,S,S/2] or null
    int32_t *score;      // [S] or null
    int H, S, D;
    int causal, qmax;
    float out_scale;     // 2^(e_v - qmax)
    int ncu;             // compute units of the device (ordering of the causal row blocks)
};

// Two probabilities (packed fp16) -> two weights 2^(qmax - c) as packed fp16 bit
// patterns.  Scaling by 2^10 first makes every non-zero input a normal number, so
// one formula covers subnormals: with e = (bits(1024 p) + 599) >> 10 the code is
// c = min(25 - e, qmax) and the weight's exponent field 15 + max(e - (25 - qmax), 0).
// kmin = (25 - qmax) << 10 and kadd = (qmax - 10) << 10, both replicated per half
// (kadd in wrap-around arithmetic: no half ever borrows from the other).
__device__ __forceinline__ uint32_t log2_weight2(uint32_t p2, uint32_t kmin, uint32_t kadd) {
    const agq_v2h x = __builtin_bit_cast(agq_v2h, p2) * agq_v2h{(_Float16)1024.0f, (_Float16)1024.0f};
    uint32_t u = (__builtin_bit_cast(uint32_t, x) + 0x02570257u) & 0xFC00FC00u;
    agq_v2us e = __builtin_bit_cast(agq_v2us, u);
    e = __builtin_elementwise_min(__builtin_elementwise_max(e, __builtin_bit_cast(agq_v2us, kmin)),
                                  agq_v2us{25u << 10, 25u << 10});
    return __builtin_bit_cast(uint32_t, e) + kadd;
}

// Byte offset of the 16-byte piece (eight keys in fp16) `chunk` of row `slot`
// inside the LDS tile; rows are padded to 144 bytes so that sixteen lanes
// reading the same chunk of consecutive rows hit sixteen different bank groups.
__device__ __forceinline__ int vt_offset(int slot, int chunk) { return slot * kVRow + (chunk << 4); }

// One workgroup = 128 query rows of one head; wavefront w owns rows 32 w .. 32 w + 31
// as the A operand of the 32x32x16 fp16 MFMA (lane: row l & 31, eight keys of
// k-group l >> 5).  Inside a 64-key tile the keys are dealt to the MFMA steps so
// that a lane's four steps cover 32 consecutive keys (64 contiguous bytes of its
// row): step t of k-group g uses keys 32 g + 8 t .. + 7, for both operands.
// V tile: int8 [key][d] -> fp16 [d][key] in LDS, once per workgroup and tile.  A
// thread unit is (eight keys, four channels): eight dword loads, a byte
// transpose by v_perm that puts each byte u = v + 128 under 0x64 (the fp16
// pattern of 1024 + u), minus 1152, four 16-byte LDS writes.  Channel d sits in
// row (d & 3) * D/4 + (d >> 2), so the conversion writes and the MFMA reads both
// walk consecutive rows, and a lane ends up with four consecutive channels of
// its query rows.
// P runs two tiles ahead in registers, V one tile ahead; V loads are issued
// before the P loads so that waiting for V leaves the P loads in flight.
template <int CB, bool CODES>
__global__ __launch_bounds__(256, CB == 1 ? 3 : 1) void log2_attn_kernel(const AttnArgs a) {
    constexpr int NBUF = CB == 1 ? 2 : 1;
    __shared__ __align__(16) uint8_t vt[NBUF][CB * 128 * kVRow];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int S = a.S, D = a.D, H = a.H, DQ = D >> 2;
    const int nb = (S + kQRows - 1) / kQRows;

    // workgroup -> (head, row block).  Causal: blocks ranked by length, longest first.
    // All workgroups of a launch are resident at once when there are at most three
    // per CU, and the dispatcher hands workgroup i and workgroup i + (number of CUs)
    // to the same CU; every second run of that many workgroups therefore takes its
    // blocks in ascending order, so that a CU's long first block is paired with a
    // short second one and the CUs finish together (loads of 19-24 instead of 14-30
    // units at H = 40, S = 2048).
    int rank = (int)blockIdx.x;
    if (a.causal) {
        const int run = rank / a.ncu, base = run * a.ncu;
        if (run & 1) rank = base + min(a.ncu, (int)gridDim.x - base) - 1 - (rank - base);
    }
    const int h = rank % H;
    const int b = a.causal ? nb - 1 - rank / H : rank / H;
    const int q0 = b * kQRows;
    const int r0 = q0 + wave * 32;                        // first row of this wavefront
    const int row = r0 + (lane & 31);
    const int g = lane >> 5;
    const int last_key = a.causal ? min(q0 + kQRows, S) : S;
    const int nt = (last_key + kKeys - 1) / kKeys;
    // Step t of this workgroup handles tile (t + rot) mod nt.  Workgroups that run
    // side by side would otherwise all read the same column window of their rows
    // at the same time; with a row pitch that is a power of two those addresses
    // fall on few memory channels.
    const int rot = (int)((blockIdx.x * 11u) % (unsigned)nt);
    auto tile_of = [&](int t) {
        int kt = min(t, nt - 1) + rot;
        return kt >= nt ? kt - nt : kt;
    };
    const int lim = a.causal ? row : S - 1;               // last key this row uses
    const int wave_lim = a.causal ? r0 : S - 1;           // a tile reaching past this needs the mask
    const int wave_last = a.causal ? r0 + 31 : S - 1;     // tiles starting past this are dead for the wavefront

    const uint32_t kmin = ((uint32_t)(25 - a.qmax) << 10) * 0x00010001u;
    const uint32_t kadd = (uint32_t)((a.qmax - 10) * 1024) * 0x00010001u;
    const uint32_t ctop = ((uint32_t)(15 + a.qmax) << 10) * 0x00010001u;
    const uint32_t cdead = ((uint32_t)a.qmax << 10) * 0x00010001u;

    // Addresses are a uniform base plus a 32-bit per-lane byte offset (one head of
    // P is below 4 GiB: S <= 32768).
    const uint8_t *phead = reinterpret_cast<const uint8_t *>(a.p + (int64_t)h * S * S);
    const uint32_t prow_off = (uint32_t)min(row, S - 1) * (uint32_t)S * 2u;
    // V conversion units of this thread: (eight keys kg, four channels 4 c .. 4 c + 3)
    uint32_t vraw[CB][8];
    int vu_c[CB], vu_kg[CB];
    bool vu_ok[CB];
#pragma unroll
    for (int u = 0; u < CB; ++u) {
        const int unit = threadIdx.x + 256 * u;
        vu_ok[u] = unit < 8 * DQ;
        vu_c[u] = unit % DQ;
        vu_kg[u] = vu_ok[u] ? unit / DQ : 0;
    }
    const int8_t *vh = a.v + (int64_t)h * S * D;
    auto load_v = [&](int t) {
        const int k0 = tile_of(t) * kKeys;
#pragma unroll
        for (int u = 0; u < CB; ++u)
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                const int key = min(k0 + 8 * vu_kg[u] + i, S - 1);   // keys past S get weight 0
                vraw[u][i] = *reinterpret_cast<const uint32_t *>(vh + (uint32_t)(key * D + 4 * vu_c[u]));
            }
    };
    auto store_v = [&](uint8_t *buf) {
        const agq_v2h bias = {(_Float16)1152.0f, (_Float16)1152.0f};
#pragma unroll
        for (int u = 0; u < CB; ++u) {
            uint32_t x[8];
#pragma unroll
            for (int i = 0; i < 8; ++i) x[i] = vraw[u][i] ^ 0x80808080u;     // bytes v + 128
#pragma unroll
            for (int bb = 0; bb < 4; ++bb) {
                // halves 0x64uu = 1024 + (v + 128) of keys 2 i and 2 i + 1 of channel 4 c + bb
                const uint32_t sel = 0x0C000C00u | (uint32_t)bb | ((uint32_t)(4 + bb) << 16);
                agq_u4 out;
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    const uint32_t w = __builtin_amdgcn_perm(x[2 * i + 1], x[2 * i], sel) | 0x64006400u;
                    out[i] = __builtin_bit_cast(uint32_t, __builtin_bit_cast(agq_v2h, w) - bias);
                }
                if (vu_ok[u]) *reinterpret_cast<agq_u4 *>(buf + vt_offset(bb * DQ + vu_c[u], vu_kg[u])) = out;
            }
        }
    };
    // four 16-byte pieces of this lane's row: keys k0 + 32 g + 8 t .. + 7
    auto load_p = [&](agq_u4 (&dst)[4], int t) {
        int tt = tile_of(t);
        if (tt * kKeys > wave_last) tt = 0;               // dead tile: re-read a line that is already cached
#pragma unroll
        for (int st = 0; st < 4; ++st) {
            const uint32_t kc = (uint32_t)min(tt * kKeys + 32 * g + 8 * st, S - 8);
            dst[st] = *reinterpret_cast<const agq_u4 *>(phead + (prow_off + kc * 2u));
        }
    };

    agq_v16f acc[4][CB];
#pragma unroll
    for (int n = 0; n < 4; ++n)
#pragma unroll
        for (int cb = 0; cb < CB; ++cb)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[n][cb][r] = 0.f;

    __shared__ int ssum[kQRows];
    if (a.score && threadIdx.x < kQRows) ssum[threadIdx.x] = 0;   // made visible by the main loop's barriers

    int bslot[CB];                                          // LDS row of this lane's B operand, n = 0
#pragma unroll
    for (int cb = 0; cb < CB; ++cb) bslot[cb] = min(cb * 32 + (lane & 31), DQ - 1);

    // MASKED: the tile reaches past the last key of some row (diagonal tiles of the
    // causal case, the ragged last tile); dead keys get weight 0 and code qmax.
    auto multiply = [&](const agq_u4 (&pc)[4], int k0, const uint8_t *buf, auto masked_tag) {
        constexpr bool MASKED = decltype(masked_tag)::value;
#pragma unroll
        for (int st = 0; st < 4; ++st) {
            const int kc = k0 + 32 * g + 8 * st;
            const int nl = lim - kc + 1;                   // live keys of this piece (may be <= 0 or >= 8)
            uint32_t wv[4];
            uint32_t cw = 0;
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                uint32_t u = log2_weight2(pc[st][j], kmin, kadd);
                uint32_t m = 0xFFFFFFFFu;
                if (MASKED) {
                    const int lv = nl - 2 * j;
                    m = lv >= 2 ? 0xFFFFFFFFu : (lv == 1 ? 0x0000FFFFu : 0u);
                    u &= m;
                }
                if (CODES) {
                    uint32_t c10 = ctop - u;               // code << 10 per half (dead: above qmax, fixed below)
                    if (MASKED) c10 = (c10 & m) | (cdead & ~m);
                    cw |= (((c10 >> 10) | (c10 >> 22)) & 0xFFu) << (8 * j);
                }
                wv[j] = u;
            }
            if (CODES) {
                if (row < S && kc < S)
                    *reinterpret_cast<uint32_t *>(a.codes + ((int64_t)h * S + row) * (S >> 1) + (kc >> 1)) = cw;
            }
            const agq_u4 wq = {wv[0], wv[1], wv[2], wv[3]};
            const agq_v8h af = __builtin_bit_cast(agq_v8h, wq);
#pragma unroll
            for (int n = 0; n < 4; ++n)
#pragma unroll
                for (int cb = 0; cb < CB; ++cb) {
                    const int slot = n * DQ + bslot[cb];
                    const agq_v8h bf = *reinterpret_cast<const agq_v8h *>(buf + vt_offset(slot, 4 * g + st));
                    acc[n][cb] = __builtin_amdgcn_mfma_f32_32x32x16_f16(af, bf, acc[n][cb], 0, 0, 0);
                }
        }
    };
    auto compute = [&](const agq_u4 (&pc)[4], int t, const uint8_t *buf) {
        const int k0 = tile_of(t) * kKeys;
        if (k0 > wave_last) return;
        if (k0 + kKeys - 1 > wave_lim) multiply(pc, k0, buf, std::true_type{});
        else multiply(pc, k0, buf, std::false_type{});
    };

    // tile t: V(t) registers -> LDS, issue V(t+1) then P(t+2), barrier, multiply
    auto tile = [&](const agq_u4 (&pc)[4], agq_u4 (&pfar)[4], int t, bool more_v, bool more_p) {
        uint8_t *buf = vt[NBUF == 2 ? (t & 1) : 0];
        if (NBUF == 1) __syncthreads();                     // everyone is done reading the only buffer
        store_v(buf);
        if (more_v) load_v(t + 1);
        if (more_p) load_p(pfar, t + 2);
        __syncthreads();
        compute(pc, t, buf);
    };

    // The steady-state loop always runs three whole tiles, so every path around
    // its back edge has consumed the same register sets; the last one or two
    // tiles follow outside it.
    agq_u4 p0[4], p1[4], p2[4];
    load_v(0);
    load_p(p0, 0);
    load_p(p1, 1);
    int t = 0;
    for (; t + 3 <= nt; t += 3) {
        tile(p0, p2, t, true, true);
        tile(p1, p0, t + 1, true, true);
        tile(p2, p1, t + 2, true, true);
    }
    if (t < nt) {
        const bool two = t + 2 == nt;                       // uniform over the workgroup
        tile(p0, p2, t, true, false);
        if (two) tile(p1, p0, t + 1, false, false);
    }

    // code map right of the last tile this wavefront multiplied: all qmax
    if (CODES && a.causal && row < S) {
        const uint32_t fill = 0x11111111u * (uint32_t)a.qmax;
        uint8_t *dst = a.codes + ((int64_t)h * S + row) * (S >> 1);
        const int done = min(nt, wave_last / kKeys + 1);
        for (int k = done * kKeys + g * 8; k < S; k += 16) *reinterpret_cast<uint32_t *>(dst + (k >> 1)) = fill;
    }

    // accumulator register 4 q + r holds query row 8 q + 4 g + r of the wavefront,
    // channel 4 c + n in tile n: four consecutive channels per lane and row
#pragma unroll
    for (int cb = 0; cb < CB; ++cb) {
        const int c = cb * 32 + (lane & 31);
#pragma unroll
        for (int q = 0; q < 4; ++q)
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                const int orow = r0 + 8 * q + 4 * g + r;
                __half hv[4];
#pragma unroll
                for (int n = 0; n < 4; ++n) hv[n] = __float2half_rn(acc[n][cb][4 * q + r] * a.out_scale);
                if (orow < S && c < DQ)
                    *reinterpret_cast<uint2 *>(a.o + (int64_t)orow * ((int64_t)H * D) + (int64_t)h * D + 4 * c) =
                        *reinterpret_cast<const uint2 *>(hv);
            }
    }

    // Importance of a token = attention it pays to the first token, summed over
    // heads as exact integers p * 2^24 (Section 4.3).  The 128 rows of a row block
    // are dealt to the H workgroups that share it; each loads its rows' first
    // column from every head (one value per thread) and sums them in LDS.
    if (a.score) {
        const int rows_per = (kQRows + H - 1) / H;
        const int j = threadIdx.x / H, hh = threadIdx.x - j * H;
        const int i = q0 + h * rows_per + j;
        if (j < rows_per && h * rows_per + j < kQRows && i < S)
            atomicAdd(&ssum[j], (int)(__half2float(__ushort_as_half(a.p[((int64_t)hh * S + i) * S])) * 16777216.0f));
        __syncthreads();
        const int io = q0 + h * rows_per + (int)threadIdx.x;
        if ((int)threadIdx.x < rows_per && h * rows_per + (int)threadIdx.x < kQRows && io < S)
            a.score[io] = ssum[threadIdx.x];
    }
}

// ------------------------------------------------------------------ pruning

constexpr int kSelThreads = 1024;
constexpr int kSelMaxS = 8192;
constexpr int kSelPer = kSelMaxS / kSelThreads;   // tokens per thread, kept in registers

// Survivors of Eq.4: the n_keep tokens with the largest score, equal scores to
// the lower index, written in ascending order.  One workgroup, no sort:
//   1. radix select (four 8-bit digits, LDS histograms) finds the score T of the
//      n_keep-th largest token and how many tokens with exactly that score
//      still fit (`need`);
//   2. a token survives if its score is above T, or equals T and fewer than
//      `need` equal-scored tokens precede it;
//   3. wavefront-shuffle prefix sums give the tie ordinals and output positions.
// Thread t owns the contiguous tokens [t * per, t * per + per).
__global__ __launch_bounds__(kSelThreads) void prune_select_kernel(const int32_t *__restrict__ score, int S, int n_keep,
                                                                    int32_t *__restrict__ idx_out) {
    __shared__ int hist[256];
    __shared__ int wave_tot[kSelThreads / 64];
    __shared__ unsigned sel_prefix;
    __shared__ int sel_k;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int per = (S + kSelThreads - 1) / kSelThreads;
    const int lo = threadIdx.x * per;
    unsigned key[kSelPer];     // order-preserving unsigned image of the signed score
#pragma unroll
    for (int e = 0; e < kSelPer; ++e)
        key[e] = (e < per && lo + e < S) ? ((unsigned)score[lo + e] ^ 0x80000000u) : 0u;
    auto live = [&](int e) { return e < per && lo + e < S; };

    unsigned prefix = 0, himask = 0;
    int k = n_keep;            // the k-th largest among the tokens matching `prefix`
    for (int shift = 24; shift >= 0; shift -= 8) {
        if (threadIdx.x < 256) hist[threadIdx.x] = 0;
        __syncthreads();
#pragma unroll
        for (int e = 0; e < kSelPer; ++e)
            if (live(e) && (key[e] & himask) == prefix) atomicAdd(&hist[(key[e] >> shift) & 255], 1);
        __syncthreads();
        if (wave == 0) {
            // lane l owns digits 4l .. 4l+3; suffix sums from the top digit down
            const int c0 = hist[4 * lane], c1 = hist[4 * lane + 1], c2 = hist[4 * lane + 2], c3 = hist[4 * lane + 3];
            const int mine4 = c0 + c1 + c2 + c3;
            int above = mine4;                       // inclusive suffix sum over lanes >= l
#pragma unroll
            for (int off = 1; off < 64; off <<= 1) {
                const int v = __shfl_down(above, off);
                if (lane + off < 64) above += v;
            }
            const int higher = above - mine4;        // tokens in digits owned by higher lanes
            if (higher < k && k <= above) {          // the k-th largest falls into this lane's digits
                int rem = k - higher, d = 3;
                const int c[4] = {c0, c1, c2, c3};
                while (rem > c[d]) {
                    rem -= c[d];
                    --d;
                }
                sel_prefix = prefix | ((unsigned)(4 * lane + d) << shift);
                sel_k = rem;
            }
        }
        __syncthreads();
        prefix = sel_prefix;
        k = sel_k;
        himask |= 0xFFu << shift;
    }
    // prefix = image of T; k = number of tokens with score T that survive
    int ties = 0;
#pragma unroll
    for (int e = 0; e < kSelPer; ++e) ties += live(e) && key[e] == prefix;
    auto excl_scan = [&](int v) {                    // exclusive prefix over the workgroup
        int incl = v;
#pragma unroll
        for (int off = 1; off < 64; off <<= 1) {
            const int u = __shfl_up(incl, off);
            if (lane >= off) incl += u;
        }
        __syncthreads();                             // wave_tot is reused between the two scans
        if (lane == 63) wave_tot[wave] = incl;
        __syncthreads();
        int base = 0;
        for (int w = 0; w < wave; ++w) base += wave_tot[w];
        return base + incl - v;
    };
    int tie_ord = excl_scan(ties);
    unsigned keepmask = 0;
    int mine = 0;
#pragma unroll
    for (int e = 0; e < kSelPer; ++e) {
        if (!live(e)) continue;
        bool keep = key[e] > prefix;
        if (key[e] == prefix) keep = tie_ord++ < k;
        if (keep) {
            keepmask |= 1u << e;
            ++mine;
        }
    }
    int pos = excl_scan(mine);
#pragma unroll
    for (int e = 0; e < kSelPer; ++e)
        if (keepmask >> e & 1) idx_out[pos++] = lo + e;
}

__global__ __launch_bounds__(256) void gather_rows_kernel(const uint4 *__restrict__ x, const int32_t *__restrict__ idx,
                                                           int64_t d8, uint4 *__restrict__ out) {
    const int64_t src = idx[blockIdx.x];
    for (int64_t c = threadIdx.x; c < d8; c += blockDim.x) out[(int64_t)blockIdx.x * d8 + c] = x[src * d8 + c];
}

}  // namespace

int agq_launch_log2_attn(const void *p, int64_t H, int64_t S, int64_t D, int causal, int qmax, const int8_t *vq,
                         int e_v, void *o, void *codes, int32_t *score, void *stream) {
    AttnArgs a;
    a.p = (const uint16_t *)p;
    a.v = vq;
    a.o = (__half *)o;
    a.codes = (uint8_t *)codes;
    a.score = score;
    a.H = (int)H;
    a.S = (int)S;
    a.D = (int)D;
    a.causal = causal;
    a.qmax = qmax;
    a.out_scale = ldexpf(1.0f, e_v - qmax);
    // number of compute units of the current device, asked once per device
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
    const unsigned grid = (unsigned)(((S + kQRows - 1) / kQRows) * H);
    if (D <= 128) {
        if (codes) log2_attn_kernel<1, true><<<grid, 256, 0, st>>>(a);
        else log2_attn_kernel<1, false><<<grid, 256, 0, st>>>(a);
    } else {
        if (codes) log2_attn_kernel<2, true><<<grid, 256, 0, st>>>(a);
        else log2_attn_kernel<2, false><<<grid, 256, 0, st>>>(a);
    }
    return (int)hipGetLastError();
}

int agq_launch_prune(const int32_t *score, int64_t S, int64_t n_keep, const void *x, int64_t d, int32_t *idx,
                     void *x_out, void *stream) {
    hipStream_t st = (hipStream_t)stream;
    prune_select_kernel<<<1, kSelThreads, 0, st>>>(score, (int)S, (int)n_keep, idx);
    gather_rows_kernel<<<(unsigned)n_keep, 256, 0, st>>>((const uint4 *)x, idx, d / 8, (uint4 *)x_out);
    return (int)hipGetLastError();
}
