// Tiled int8-MFMA kernel of the quantized linear layer for many tokens (the
// prefill regime, bound by the matrix cores).
//
// Workgroup tile 128 (tokens) x 128 (output channels), K step 128, four
// wavefronts as 2 (tokens) x 2 (channels): each owns 64 x 64 as 2 x 2 MFMA tiles
// of 32 x 32 (v_mfma_i32_32x32x32_i8, 64 accumulator registers per lane).  Two
// workgroups share a CU, one wavefront of each per SIMD: a workgroup barrier (one
// per K step), a prologue or an epilogue stalls only one of the two wavefronts
// that feed a matrix core.  The 32 x 32 x 32 form is used because back-to-back
// 16 x 16 x 64 MFMAs of one wavefront keep the matrix core only 55 % busy.
// Two variants serve calls with few tiles: 64-token tiles (NI == 1) and a split of
// K over workgroups (SPLIT), both described at the kernel.
//
//   activation codes: int8, already laid out in MFMA operand order by the
//     pre-pass (16 KiB per 128-token tile and K step, see agq_quant.hip), copied
//     HBM/L2 -> LDS by direct global-to-LDS loads (no registers in between,
//     contiguous 1 KiB per instruction), three stages deep.  A fragment read is
//     one conflict-free ds_read_b128 at lane * 16.
//   weights: the packed 4-bit blob is copied the same way (16 bytes per lane,
//     512-byte contiguous runs); a wavefront reads its 64 channels back once per
//     step and widens them to int8 in registers: three bit operations per eight
//     weights.  The nibbles cross HBM, L2 and LDS at half the bytes of int8.  A
//     lane addresses the blob's 16-row chunks so that it receives the operand
//     of a 32-row MFMA: low nibbles feed k-block t, high nibbles k-block t + 2.
//   No load in the main loop returns to registers, so the only waits on vector
//   memory are the ones written here: loads return in order, every step issues
//   four per wavefront, and a step waits until at most the four of the step two
//   ahead are still in flight (copies start three steps ahead; the fragments of the
//   step being multiplied are already in registers, so three stages suffice).
//
// The weight fragment is the MFMA's first operand and the activation the second:
// a lane then holds four consecutive output channels of one token.  The
// epilogue dequantizes in registers, transposes through LDS (free by then) and
// stores whole 128-byte rows, 16 bytes per lane.
#include "../../include/agq.h"
#include "agq_device.h"
#include "agq_internal.h"

typedef unsigned int agq_u4 __attribute__((ext_vector_type(4)));
typedef int agq_v16i __attribute__((ext_vector_type(16)));

namespace {

constexpr int BM = 128, BN = 128, BK = 128;
constexpr int kThreads = 256;
constexpr int kBand = 4;                  // token tiles per band of the tile walk
constexpr int kAChunks = (BM / 32) * 4;   // 16 chunks of 1 KiB per stage
constexpr int kBChunks = BN / 16;         // 8 chunks of 1 KiB per stage
constexpr int kABytes = kAChunks * 1024;
constexpr int kStageBytes = (kAChunks + kBChunks) * 1024;   // 24 KiB
constexpr int kStages = 3;
constexpr int kCopies = (kAChunks + kBChunks) * 64 / kThreads;   // 6 copies per wavefront and step
constexpr int kOutStride = 144;           // bytes per row of a wavefront's 64 x 64 fp16 output tile in LDS

constexpr int kMaxProj = 4;   // == AGQ_MAX_PROJ of the public header

// Up to four projections of the same activation share a launch (q/k/v, gate/up): one
// grid covers the tiles of all of them, which fills the chip where a single projection
// has too few tiles and saves the gaps between launches.
struct TiledArgs {
    const agq_u4 *xt;    // activation codes in operand order (pre-pass output)
    int M, K, KT;
    int tiles_m;
    int tile_start[kMaxProj + 1];   // first workgroup of every projection; [count..] = the grid size
    int N4[kMaxProj];
    int tiles_n4[kMaxProj];
    const agq_u4 *blob4[kMaxProj];
    const __half *sw4[kMaxProj];
    __half *y4[kMaxProj];
    int64_t ldy4[kMaxProj];
    int32_t *acc4[kMaxProj];
    const int32_t *wsum4[kMaxProj];   // per-channel weight sums (end of every blob)
    float scale_e;
    int corr;               // unsigned activation grid: acc += corr * wsum[n]; 0 on the signed grid
    // TRIP blob: the first n_extra steps are the extra chunks of the channels with a factor;
    // trip_shift[kt] (device) is the left shift of the running accumulators after step kt
    int n_extra;
    const int32_t *trip_shift;
    // K split over `splits` workgroups per tile (few tiles, long K), steps_per_split K steps each: they
    // leave int32 partial tiles in `part`, which a second kernel adds up and dequantizes
    int splits, steps_per_split, tiles_all;
    int32_t *part;       // [tile][split][16][256 threads][4]
};

// TRIP: the blob and the activation stages carry extra steps in front, ordered by
// descending factor; after the last step of a factor the accumulators are shifted
// left by the difference to the next factor (Horner), so that at the end every
// extra step has been multiplied by 2^factor (Section 4.4) - exact in int32.
//
// SPLIT: with fewer tiles than the chip has workgroup slots and a long K, a tile's K steps are shared
// out over several workgroups.  Each stores its int32 accumulators as a partial tile and is done;
// split_reduce_kernel, launched behind it, adds the partial tiles up and runs the epilogue.  (One
// kernel in which the last workgroup to arrive at a tile adds the others' partial tiles was measured
// slower than no split at all: it has to read them in dependent rounds through device-scope loads,
// or with cache-wide write-backs and invalidations around them.  A lone workgroup on a CU is not
// short of copies in flight either: six stages instead of three changed nothing, its sixteen
// MFMAs per wavefront and step, about 60 cycles apart in this loop, are the step time.)  An int32 sum does not depend on
// its order, so the result is the unsplit kernel's bit for bit.
//
// NI: 32-token MFMA tiles per wavefront.  2: the 128-token workgroup tile described above.  1: a 64-token
// tile (each wavefront 32 x 64, half of the MFMAs per step for two thirds of the operand bytes), for grids
// whose 128-token tiles would leave the last round of workgroups mostly empty.
template <bool TRIP, bool SPLIT, int NI = 2>
__global__ __launch_bounds__(kThreads, 2) void gemm_tiled_kernel(const TiledArgs a) {
    static_assert(NI == 2 || (NI == 1 && !SPLIT), "the partial tiles of a K split are laid out for 128 tokens");
    constexpr int BMT = NI * 64;                 // tokens per workgroup tile
    constexpr int kAChunksT = NI * 8;            // activation chunks of 1 KiB per stage
    constexpr int kABytesT = kAChunksT * 1024;
    constexpr int kStageT = kABytesT + kBChunks * 1024;      // 24 KiB (16 KiB for NI == 1)
    constexpr int kNA = NI * 2;                  // activation copies per wavefront and step
    constexpr int kCopiesT = kNA + 2;
    // Three pipeline stages; the epilogue reuses the first 36 KiB.
    __shared__ __align__(16) unsigned char lds[kStages * kStageT];
    unsigned char *const stage0 = lds, *const stage1 = lds + kStageT, *const stage2 = lds + 2 * kStageT;
    const int lane = threadIdx.x & 63;
    const int wave = threadIdx.x >> 6;
    const int wm = wave >> 1, wn = wave & 1;

    // XCD-aware tile order.  Consecutive workgroup ids land on different XCDs
    // (round-robin over 8), each with its own L2, so first give every XCD a
    // contiguous run of logical tile ids; then walk the tile grid in bands of
    // kBand token tiles, column by column, so that a run covers a compact
    // rectangle and re-reads as little of either operand as possible.
    const int nblk = gridDim.x;
    int bid = blockIdx.x;
    if ((nblk & 7) == 0) bid = (bid & 7) * (nblk >> 3) + (bid >> 3);
    // SPLIT: workgroups with the same K slice are neighbours (they share activation stages)
    const int split = SPLIT ? bid / a.tiles_all : 0;
    if (SPLIT) bid -= split * a.tiles_all;
    const int tile_id = bid;
    // which projection this workgroup serves: scalar compares and selects (an index into the
    // argument record would move it to memory)
    const int pj = (bid >= a.tile_start[1]) + (bid >= a.tile_start[2]) + (bid >= a.tile_start[3]);
    auto pick = [pj](auto v0, auto v1, auto v2, auto v3) { return pj == 0 ? v0 : (pj == 1 ? v1 : (pj == 2 ? v2 : v3)); };
    bid -= pick(0, a.tile_start[1], a.tile_start[2], a.tile_start[3]);
    const int pN = pick(a.N4[0], a.N4[1], a.N4[2], a.N4[3]);
    const int ptiles_n = pick(a.tiles_n4[0], a.tiles_n4[1], a.tiles_n4[2], a.tiles_n4[3]);
    const agq_u4 *const pblob = pick(a.blob4[0], a.blob4[1], a.blob4[2], a.blob4[3]);
    const __half *const psw = pick(a.sw4[0], a.sw4[1], a.sw4[2], a.sw4[3]);
    __half *const py = pick(a.y4[0], a.y4[1], a.y4[2], a.y4[3]);
    const int64_t pldy = pick(a.ldy4[0], a.ldy4[1], a.ldy4[2], a.ldy4[3]);
    int32_t *const pacc = pick(a.acc4[0], a.acc4[1], a.acc4[2], a.acc4[3]);
    const int32_t *const pwsum = pick(a.wsum4[0], a.wsum4[1], a.wsum4[2], a.wsum4[3]);
    const int band = bid / (kBand * ptiles_n);
    const int rows = min(kBand, a.tiles_m - band * kBand);
    const int within = bid - band * kBand * ptiles_n;
    const int tn = within / rows, tm = band * kBand + within - tn * rows;
    const int m0 = tm * BMT, n0 = tn * BN;
    const int KTfull = a.KT;
    const int kbeg = SPLIT ? split * a.steps_per_split : 0;
    const int KT = SPLIT ? min(a.steps_per_split, KTfull - kbeg) : KTfull;   // steps of this workgroup

    // Copies of this wavefront per step: activation chunks 4 wave .. 4 wave + 3 of
    // the 16 KiB stage, and weight chunks 2 wave, 2 wave + 1.  Weight chunk c
    // serves channel group c >> 2 (64 channels), 32-channel tile (c >> 1) & 1,
    // k-blocks t = c & 1 (low nibbles) and t + 2 (high nibbles): channel l & 31
    // of the tile lives in the blob's 16-row chunk (l & 31) >> 4 at blob lane
    // (2 t + (l >> 5)) * 16 + (l & 15).
    // (NI == 1: the 64-token tile tm is half tm & 1 of the 128-token tile tm >> 1 of the pre-pass: eight
    // consecutive chunks of every stage, two per wavefront)
    const agq_u4 *asrc = a.xt + (((int64_t)(NI == 2 ? tm : tm >> 1) * KTfull + kbeg) * 16 + (NI == 2 ? 0 : (tm & 1) * 8) + wave * kNA) * 64 + lane;
    const agq_u4 *bsrc[2];
#pragma unroll
    for (int p = 0; p < 2; ++p) {
        const int c = wave * 2 + p, grp = c >> 2, j = (c >> 1) & 1, t = c & 1;
        const int chunk_row = n0 / 16 + grp * 4 + j * 2 + ((lane & 31) >> 4);
        bsrc[p] = pblob + ((int64_t)chunk_row * KTfull + kbeg) * 64 + (2 * t + (lane >> 5)) * 16 + (lane & 15);
    }
    // LDS byte address (wave-uniform, kept in a scalar register) of this
    // wavefront's first activation chunk in stage 0
    const uint32_t lds_base = __builtin_amdgcn_readfirstlane(
        (uint32_t)(uintptr_t)(const __attribute__((address_space(3))) unsigned char *)lds);
    const uint32_t wave_u = __builtin_amdgcn_readfirstlane((uint32_t)wave);
    auto copy_piece = [&](int p, int kt, unsigned char *st) {
        if (kt >= KT) return;               // nothing to fetch past the last step (uniform)
        const int k = kt;
        const uint32_t dst = lds_base + (uint32_t)(st - lds);
        if (p < kNA)
            lds_dma16(asrc + ((int64_t)k * 16 + p) * 64, dst + (wave_u * kNA + p) * 1024);
        else
            lds_dma16(bsrc[p - kNA] + (int64_t)k * 64, dst + kABytesT + (wave_u * 2 + (p - kNA)) * 1024);
    };

    // per-channel scales of this lane's output columns, fetched early
    // (accumulator register 4 q + r of tile j: channel 32 j + 8 q + 4 (lane >> 5) + r)
    const int ncol = n0 + wn * 64 + (lane >> 5) * 4;
    uint2 swp[2][4];
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const int n = ncol + j * 32 + q * 8;
            // channels past N are never stored: clamp their addresses into the array
            const uint16_t *sp = reinterpret_cast<const uint16_t *>(psw);
            if ((pN & 3) == 0) {
                swp[j][q] = *reinterpret_cast<const uint2 *>(sp + min(n, pN - 4));   // 8-byte aligned: n % 4 == 0
            } else {
                uint32_t h[4];
                for (int r = 0; r < 4; ++r) h[r] = sp[min(n + r, pN - 1)];
                swp[j][q] = make_uint2(h[0] | (h[1] << 16), h[2] | (h[3] << 16));
            }
        }

    agq_v16i acc[NI][2];
#pragma unroll
    for (int i = 0; i < NI; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0;

    // Fragments of a whole step live in registers: eight activation fragments
    // (index i * 4 + t: 32-token tile i, k-block t) and four packed weight pieces.
    // Two such sets alternate: while one is multiplied, the other is filled from
    // the next step's LDS stage, so no MFMA ever waits for an LDS read it issued
    // a few instructions earlier.
    agq_u4 xa0[NI * 4], b0[4], xa1[NI * 4], b1[4];

    // One K step, software-pipelined by hand.  A wavefront issues in order and an
    // MFMA blocks the next MFMA while the matrix core is busy, but LDS reads,
    // copies and bit operations slip in between: every pair of MFMAs is followed
    // by LDS reads for the next step (twelve per step), and the six copies of the
    // step three ahead are spread over the step.
    auto step = [&](int kt, const unsigned char *nxt, unsigned char *fill, const agq_u4 (&xc)[NI * 4], const agq_u4 (&bc)[4],
                    agq_u4 (&xn)[NI * 4], agq_u4 (&bn)[4]) {
        const agq_u4 *sn = reinterpret_cast<const agq_u4 *>(nxt) + lane;
#pragma unroll
        for (int t = 0; t < 4; ++t) {
            agq_v4i wb[2];
#pragma unroll
            for (int j = 0; j < 2; ++j) {
                const agq_u4 p = bc[j * 2 + (t & 1)];
                const agq_u4 w = t < 2 ? ((p << 4) & 0xF0F0F0F0u) : (p & 0xF0F0F0F0u);
                wb[j] = __builtin_bit_cast(agq_v4i, w);
            }
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int i = 0; i < NI; ++i) {
                const agq_v4i x = __builtin_bit_cast(agq_v4i, xc[i * 4 + t]);
                acc[i][0] = __builtin_amdgcn_mfma_i32_32x32x32_i8(wb[0], x, acc[i][0], 0, 0, 0);
                acc[i][1] = __builtin_amdgcn_mfma_i32_32x32x32_i8(wb[1], x, acc[i][1], 0, 0, 0);
                __builtin_amdgcn_sched_barrier(0);
                const int mi = wm * NI + i;   // 32-token tile of the stage
                xn[i * 4 + t] = sn[(mi * 4 + t) * 64];
                if (i == NI - 1) bn[t] = sn[(kAChunksT + wn * 4 + t) * 64];
                if (NI * t + i < kCopiesT) copy_piece(NI * t + i, kt + 3, fill);
                __builtin_amdgcn_sched_barrier(0);
            }
        }
    };

    auto shift_acc = [&](int sh) {          // uniform
        if (sh == 0) return;
#pragma unroll
        for (int i = 0; i < NI; ++i)
#pragma unroll
            for (int j = 0; j < 2; ++j)
#pragma unroll
                for (int r = 0; r < 16; ++r) acc[i][j][r] <<= sh;
    };

#pragma unroll
    for (int p = 0; p < kCopiesT; ++p) copy_piece(p, 0, stage0);
#pragma unroll
    for (int p = 0; p < kCopiesT; ++p) copy_piece(p, 1, stage1);
#pragma unroll
    for (int p = 0; p < kCopiesT; ++p) copy_piece(p, 2, stage2);
    static_assert(kCopiesT == 6 || kCopiesT == 4, "the vmcnt immediates below count the copies of one and two steps");
    if (KT < 3)
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    else if (kCopiesT == 6)
        asm volatile("s_waitcnt vmcnt(12)" ::: "memory");   // step 0 has landed
    else
        asm volatile("s_waitcnt vmcnt(8)" ::: "memory");
    __syncthreads();
    {
        const agq_u4 *s0 = reinterpret_cast<const agq_u4 *>(stage0) + lane;
#pragma unroll
        for (int i = 0; i < NI; ++i)
#pragma unroll
            for (int t = 0; t < 4; ++t) xa0[i * 4 + t] = s0[((wm * NI + i) * 4 + t) * 64];
#pragma unroll
        for (int j = 0; j < 4; ++j) b0[j] = s0[(kAChunksT + wn * 4 + j) * 64];
    }
    // Every step kt: wait until this wavefront's copies of step kt+1 have landed
    // (loads return in order, each step issues kCopiesT, so only those of step
    // kt+2, if there is one, may still fly), meet the others (everybody's copies of step kt+1 are
    // in LDS, and everybody has read step kt's fragments out of the stage that is
    // refilled next), then multiply step kt while copying step kt+3.
#define AGQ_STEP(KT_, NXT, FILL, XC, BC, XN, BN)                             \
    if ((KT_) < KT) {                                                        \
        if ((KT_) + 2 >= KT)                                                 \
            asm volatile("s_waitcnt vmcnt(0)" ::: "memory");                 \
        else if (kCopiesT == 6)                                              \
            asm volatile("s_waitcnt vmcnt(6)" ::: "memory");                 \
        else                                                                 \
            asm volatile("s_waitcnt vmcnt(4)" ::: "memory");                 \
        __syncthreads();                                                     \
        step((KT_), NXT, FILL, XC, BC, XN, BN);                              \
        if (TRIP && split == 0 && (KT_) < a.n_extra) shift_acc(a.trip_shift[(KT_)]); \
    }
    for (int kt = 0; kt < KT; kt += 6) {      // stage of step kt is kt % 3, register set kt % 2
        AGQ_STEP(kt, stage1, stage0, xa0, b0, xa1, b1)
        AGQ_STEP(kt + 1, stage2, stage1, xa1, b1, xa0, b0)
        AGQ_STEP(kt + 2, stage0, stage2, xa0, b0, xa1, b1)
        AGQ_STEP(kt + 3, stage1, stage0, xa1, b1, xa0, b0)
        AGQ_STEP(kt + 4, stage2, stage1, xa0, b0, xa1, b1)
        AGQ_STEP(kt + 5, stage0, stage2, xa1, b1, xa0, b0)
    }
#undef AGQ_STEP
    __syncthreads();                                   // every wavefront is done with the stages

    if (SPLIT) {
        // accumulator piece c = (i * 2 + j) * 4 + q of thread t at [c][t]: 16 bytes per lane, contiguous
        int4 *const mine = reinterpret_cast<int4 *>(a.part) + ((int64_t)tile_id * a.splits + split) * (16 * kThreads) + threadIdx.x;
#pragma unroll
        for (int i = 0; i < NI; ++i) {
            if (m0 + wm * 64 + i * 32 >= a.M) continue;   // no token in these 32 rows: nobody reads them (uniform)
#pragma unroll
            for (int j = 0; j < 2; ++j)
#pragma unroll
                for (int q = 0; q < 4; ++q)
                    mine[((i * 2 + j) * 4 + q) * kThreads] =
                        make_int4(acc[i][j][4 * q], acc[i][j][4 * q + 1], acc[i][j][4 * q + 2], acc[i][j][4 * q + 3]);
        }
        return;
    }

    // Fused epilogue.  Drop the factor 16 of the widened weights, dequantize with
    // 2^e * sw[n] in registers, then transpose through LDS: a lane holds four
    // consecutive channels of one token (8 bytes), the store wants eight lanes
    // per 128-byte row.  Each wavefront uses a private 64 x 144-byte region.
    const int mrow = m0 + wm * (NI * 32) + (lane & 31);
    if (a.corr) {
        // unsigned activation grid: add corr * sum_k w[n,k], times the 16 the
        // accumulators still carry (|16 acc| <= 16 * 255 * 8 * K < 2^31 for K <= 65536)
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const int4 ws = *reinterpret_cast<const int4 *>(pwsum + ncol + j * 32 + q * 8);   // padded to 256 channels
                const int t[4] = {ws.x, ws.y, ws.z, ws.w};
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    const int add = (a.corr * t[r]) << AGQ_W_SHIFT;
#pragma unroll
                    for (int i = 0; i < NI; ++i) acc[i][j][4 * q + r] += add;
                }
            }
    }
    if (pacc) {   // exact accumulators for parity checks (plain stores)
#pragma unroll
        for (int i = 0; i < NI; ++i)
#pragma unroll
            for (int j = 0; j < 2; ++j)
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const int m = mrow + i * 32, n = ncol + j * 32 + (r >> 2) * 8 + (r & 3);
                    if (m < a.M && n < pN) pacc[(int64_t)m * pN + n] = acc[i][j][r] >> AGQ_W_SHIFT;
                }
    }
    unsigned char *obuf = lds + wave * (64 * kOutStride);   // 9 KiB per wavefront, 36 KiB in all
#pragma unroll
    for (int i = 0; i < NI; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const float g0 = a.scale_e * __half2float(__ushort_as_half((unsigned short)(swp[j][q].x & 0xFFFF)));
                const float g1 = a.scale_e * __half2float(__ushort_as_half((unsigned short)(swp[j][q].x >> 16)));
                const float g2 = a.scale_e * __half2float(__ushort_as_half((unsigned short)(swp[j][q].y & 0xFFFF)));
                const float g3 = a.scale_e * __half2float(__ushort_as_half((unsigned short)(swp[j][q].y >> 16)));
                const __half h0 = agq_dequant(acc[i][j][4 * q] >> AGQ_W_SHIFT, g0);
                const __half h1 = agq_dequant(acc[i][j][4 * q + 1] >> AGQ_W_SHIFT, g1);
                const __half h2 = agq_dequant(acc[i][j][4 * q + 2] >> AGQ_W_SHIFT, g2);
                const __half h3 = agq_dequant(acc[i][j][4 * q + 3] >> AGQ_W_SHIFT, g3);
                uint2 pk;
                pk.x = (uint32_t)__half_as_ushort(h0) | ((uint32_t)__half_as_ushort(h1) << 16);
                pk.y = (uint32_t)__half_as_ushort(h2) | ((uint32_t)__half_as_ushort(h3) << 16);
                const int row = i * 32 + (lane & 31), col = j * 32 + q * 8 + (lane >> 5) * 4;
                *reinterpret_cast<uint2 *>(obuf + row * kOutStride + col * 2) = pk;
            }
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
    const int nbase = n0 + wn * 64 + (lane & 7) * 8;          // eight channels per lane
    const bool vec_ok = (pldy & 7) == 0 && nbase + 7 < pN;
#pragma unroll
    for (int it = 0; it < NI * 4; ++it) {
        const int row = it * 8 + (lane >> 3);
        const int m = m0 + wm * (NI * 32) + row;
        if (m >= a.M || nbase >= pN) continue;
        const uint4 v = *reinterpret_cast<const uint4 *>(obuf + row * kOutStride + (lane & 7) * 16);
        __half *yp = py + (int64_t)m * pldy + nbase;
        if (vec_ok) {
            *reinterpret_cast<uint4 *>(yp) = v;
        } else {
            const uint32_t w[4] = {v.x, v.y, v.z, v.w};
            for (int c = 0; c < 8 && nbase + c < pN; ++c)
                yp[c] = __ushort_as_half((unsigned short)(w[c >> 1] >> (16 * (c & 1))));
        }
    }
}

// Second kernel of a K split: workgroup (tile, piece c) adds the `splits` partial copies of accumulator piece c of
// every thread of the tile's workgroups (same thread numbering, same tile walk as above) and runs the same
// epilogue arithmetic on the sums; a thread owns four consecutive channels of one token.
__global__ __launch_bounds__(kThreads) void split_reduce_kernel(const TiledArgs a) {
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int wm = wave >> 1, wn = wave & 1;
    const int tile_id = blockIdx.x >> 4, c = blockIdx.x & 15;
    const int i = c >> 3, j = (c >> 2) & 1, q = c & 3;
    int bid = tile_id;
    const int pj = (bid >= a.tile_start[1]) + (bid >= a.tile_start[2]) + (bid >= a.tile_start[3]);
    auto pick = [pj](auto v0, auto v1, auto v2, auto v3) { return pj == 0 ? v0 : (pj == 1 ? v1 : (pj == 2 ? v2 : v3)); };
    bid -= pick(0, a.tile_start[1], a.tile_start[2], a.tile_start[3]);
    const int pN = pick(a.N4[0], a.N4[1], a.N4[2], a.N4[3]);
    const int ptiles_n = pick(a.tiles_n4[0], a.tiles_n4[1], a.tiles_n4[2], a.tiles_n4[3]);
    const uint16_t *const psw = reinterpret_cast<const uint16_t *>(pick(a.sw4[0], a.sw4[1], a.sw4[2], a.sw4[3]));
    __half *const py = pick(a.y4[0], a.y4[1], a.y4[2], a.y4[3]);
    const int64_t pldy = pick(a.ldy4[0], a.ldy4[1], a.ldy4[2], a.ldy4[3]);
    int32_t *const pacc = pick(a.acc4[0], a.acc4[1], a.acc4[2], a.acc4[3]);
    const int32_t *const pwsum = pick(a.wsum4[0], a.wsum4[1], a.wsum4[2], a.wsum4[3]);
    const int band = bid / (kBand * ptiles_n);
    const int rows = min(kBand, a.tiles_m - band * kBand);
    const int within = bid - band * kBand * ptiles_n;
    const int tn = within / rows, tm = band * kBand + within - tn * rows;
    const int m = tm * BM + wm * 64 + i * 32 + (lane & 31);
    const int n = tn * BN + wn * 64 + j * 32 + q * 8 + (lane >> 5) * 4;

    if (m >= a.M || n >= pN) return;
    const int4 *src = reinterpret_cast<const int4 *>(a.part) + ((int64_t)tile_id * a.splits * 16 + c) * kThreads + threadIdx.x;
    int sum[4] = {0, 0, 0, 0};
#pragma unroll 4
    for (int s = 0; s < a.splits; ++s) {
        const int4 v = src[(int64_t)s * (16 * kThreads)];
        sum[0] += v.x;
        sum[1] += v.y;
        sum[2] += v.z;
        sum[3] += v.w;
    }
    uint32_t h[4];
#pragma unroll
    for (int r = 0; r < 4; ++r) {
        const int nn = min(n + r, pN - 1);   // channels past N are not stored
        if (a.corr) sum[r] += (a.corr * pwsum[nn]) << AGQ_W_SHIFT;
        const int v = sum[r] >> AGQ_W_SHIFT;
        if (pacc && n + r < pN) pacc[(int64_t)m * pN + n + r] = v;
        h[r] = __half_as_ushort(agq_dequant(v, a.scale_e * __half2float(__ushort_as_half((unsigned short)psw[nn]))));
    }
    __half *yp = py + (int64_t)m * pldy + n;
    if ((pldy & 3) == 0 && n + 3 < pN) {
        *reinterpret_cast<uint2 *>(yp) = make_uint2(h[0] | (h[1] << 16), h[2] | (h[3] << 16));
    } else {
        for (int r = 0; r < 4 && n + r < pN; ++r) yp[r] = __ushort_as_half((unsigned short)h[r]);
    }
}

}  // namespace

int agq_launch_gemm_tiled(const void *x_tiles, int64_t M, int64_t K, int e, int corr, const struct agq_proj *projs, int count,
                          int n_extra, void *split_ws, bool half_tiles, void *stream) {
    TiledArgs a = {};
    a.xt = (const agq_u4 *)x_tiles;
    a.M = (int)M;
    a.K = (int)K;
    a.KT = (int)agq_k_tiles(K);
    a.tiles_m = (int)((M + BM - 1) / BM);
    if (half_tiles) a.tiles_m = (int)((M + 63) / 64);
    a.scale_e = ldexpf(1.0f, e);
    a.corr = corr;
    a.n_extra = 0;
    a.trip_shift = nullptr;
    int tiles = 0;
    for (int p = 0; p < kMaxProj; ++p) {
        const agq_proj &pr = projs[p < count ? p : count - 1];
        a.tile_start[p] = tiles;
        a.N4[p] = (int)pr.N;
        a.tiles_n4[p] = (int)((pr.N + BN - 1) / BN);
        if (p < count) tiles += a.tiles_m * a.tiles_n4[p];
        a.blob4[p] = (const agq_u4 *)pr.w_packed;
        a.sw4[p] = (const __half *)pr.w_scale_f16;
        a.y4[p] = (__half *)pr.y_f16;
        a.ldy4[p] = pr.ldy;
        a.acc4[p] = pr.acc_out;
        a.wsum4[p] = n_extra >= 0 ? (const int32_t *)((const char *)pr.w_packed + agq_trip_layout(pr.N, K, n_extra).wsum_off)
                                  : agq_blob_wsum(pr.w_packed, pr.N, K);
    }
    for (int p = count; p <= kMaxProj; ++p) a.tile_start[p] = tiles;
    const unsigned grid = (unsigned)tiles;
    hipStream_t st = (hipStream_t)stream;
    if (n_extra >= 0) {
        // every blob of the call was packed with the same factors: the shift table of the first serves all
        const AgqTripLayout L = agq_trip_layout(projs[0].N, K, n_extra);
        a.KT = (int)L.KTall;
        a.n_extra = n_extra;
        a.trip_shift = (const int32_t *)((const char *)projs[0].w_packed + L.meta_off) + 16;
    }
    if (split_ws && !half_tiles) {
        // the extra steps and their shifts stay together in the first slice
        const AgqSplitPlan plan = agq_tiled_split_plan(M, tiles / a.tiles_m, a.KT, true, n_extra >= 0 ? n_extra : 0);
        if (plan.splits > 1) {
            a.splits = plan.splits;
            a.steps_per_split = plan.steps;
            a.tiles_all = tiles;
            a.part = (int32_t *)split_ws;
            if (n_extra >= 0)
                gemm_tiled_kernel<true, true><<<grid * (unsigned)plan.splits, kThreads, 0, st>>>(a);
            else
                gemm_tiled_kernel<false, true><<<grid * (unsigned)plan.splits, kThreads, 0, st>>>(a);
            split_reduce_kernel<<<grid * 16, kThreads, 0, st>>>(a);
            return (int)hipGetLastError();
        }
    }
    if (half_tiles) {
        if (n_extra >= 0)
            gemm_tiled_kernel<true, false, 1><<<grid, kThreads, 0, st>>>(a);
        else
            gemm_tiled_kernel<false, false, 1><<<grid, kThreads, 0, st>>>(a);
    } else if (n_extra >= 0) {
        gemm_tiled_kernel<true, false><<<grid, kThreads, 0, st>>>(a);
    } else {
        gemm_tiled_kernel<false, false><<<grid, kThreads, 0, st>>>(a);
    }
    return (int)hipGetLastError();
}
