// Tiled int8-MFMA kernel of the quantized linear layer for many tokens (the
// prefill regime, bound by the matrix cores).
//
// Workgroup tile 128 (tokens) x 256 (output channels), K step 128, four
// wavefronts side by side along the channels: each owns 128 x 64 as 4 x 2 MFMA
// tiles of 32 x 32 (v_mfma_i32_32x32x32_i8, 128 accumulator registers per lane).
// The 32 x 32 x 32 form is used because one wavefront per SIMD keeps the matrix
// core above 90 % busy with it, against 55 % with back-to-back 16 x 16 x 64.
//
//   activation codes: int8, copied HBM/L2 -> LDS by the wavefronts' direct
//     global-to-LDS loads (no registers in between), four stages deep.  One
//     copy instruction moves 8 token rows x 128 bytes (whole cache lines), so
//     a stage is the row-major 128 x 128 tile; the 16-byte segments of a row
//     are stored XOR-swizzled with the row number, so that the MFMA fragment
//     read - 32 rows, same k - spreads over all LDS banks (conflict-free
//     ds_read_b128).  All four wavefronts read the whole stage.
//   weights: each wavefront copies its own 64 channels of the packed 4-bit blob
//     the same way (16 bytes per lane, 512-byte contiguous runs) into a private
//     4 KiB of the stage, reads them back once and widens them to int8 in
//     registers: three bit operations per eight weights.  The nibbles cross HBM,
//     L2 and LDS at half the bytes of int8.  A lane addresses the blob's 16-row
//     chunks so that it receives the operand of a 32-row MFMA: low nibbles feed
//     k-block t, high nibbles k-block t + 2.
//   No load in the main loop returns to registers, so the only waits on vector
//   memory are the ones written here: loads return in order, every step issues
//   eight per wavefront, and a step waits until at most the sixteen of the two
//   steps ahead are still in flight (prefetch distance three).
//
// The weight fragment is the MFMA's first operand and the activation the second:
// a lane then holds four consecutive output channels of one token, which makes
// the fp16 store 8 bytes per lane.
#include "agq_device.h"
#include "agq_internal.h"

typedef unsigned int agq_u4 __attribute__((ext_vector_type(4)));
typedef int agq_v16i __attribute__((ext_vector_type(16)));

namespace {

constexpr int BM = 128, BN = 256, BK = 128;
constexpr int kThreads = 256;
constexpr int kBand = 4;                  // token tiles per band of the tile walk
constexpr int kStages = 4;                // LDS stages of activation codes
constexpr int kAChunks = (BM / 32) * 4;   // 16 chunks of 1 KiB per stage
constexpr int kBChunks = BN / 16;         // 16 chunks of 1 KiB per stage (4 per wavefront)
constexpr int kABytes = kAChunks * 1024;
constexpr int kStageBytes = (kAChunks + kBChunks) * 1024;

struct TiledArgs {
    const int8_t *xq;
    int64_t ldq;
    int M, N, K, KT;
    int tiles_m, tiles_n;
    const agq_u4 *blob;
    const __half *sw;
    __half *y;
    int64_t ldy;
    int32_t *acc_out;
    float scale_e;
};

// Direct global-to-LDS copy: lane i's 16 bytes land at lds_chunk + 16 i (the LDS
// address is wave-uniform and travels in M0).  Issued as inline assembly on
// purpose: the compiler, seeing such a copy, drains every outstanding load
// (vmcnt(0)) before any later LDS read, which would cancel the prefetch distance;
// here the kernel waits for exactly the copies it needs (see the step macro).
__device__ __forceinline__ void lds_dma16(const void *gsrc, const unsigned char *lds_chunk) {
    const uint32_t lds_addr = __builtin_amdgcn_readfirstlane(
        (uint32_t)(uintptr_t)(const __attribute__((address_space(3))) unsigned char *)lds_chunk);
    asm volatile("s_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, off"
                 :
                 : "v"(gsrc), "s"(lds_addr)
                 : "memory", "m0");
}

__global__ __launch_bounds__(kThreads) void gemm_tiled_kernel(const TiledArgs a) {
    // One LDS array per pipeline stage: distinct objects let the compiler prove
    // that a copy into one stage cannot alias the fragment reads of another, so
    // it does not drain every outstanding copy before each read.
    __shared__ __align__(16) unsigned char stage0[kStageBytes];
    __shared__ __align__(16) unsigned char stage1[kStageBytes];
    __shared__ __align__(16) unsigned char stage2[kStageBytes];
    __shared__ __align__(16) unsigned char stage3[kStageBytes];
    const int lane = threadIdx.x & 63;
    const int wave = threadIdx.x >> 6;

    // XCD-aware tile order.  Consecutive workgroup ids land on different XCDs
    // (round-robin over 8), each with its own L2, so first give every XCD a
    // contiguous run of logical tile ids; then walk the tile grid in bands of
    // kBand token tiles, column by column, so that a run covers a compact
    // rectangle and re-reads as little of either operand as possible.
    const int nblk = gridDim.x;
    int bid = blockIdx.x;
    if ((nblk & 7) == 0) bid = (bid & 7) * (nblk >> 3) + (bid >> 3);
    const int band = bid / (kBand * a.tiles_n);
    const int rows = min(kBand, a.tiles_m - band * kBand);
    const int within = bid - band * kBand * a.tiles_n;
    const int tn = within / rows, tm = band * kBand + within - tn * rows;
    const int m0 = tm * BM, n0 = tn * BN;

    // activation source of this lane for the four copies its wavefront issues per
    // stage: copy c moves token rows 8 c .. 8 c + 7 of the tile.  LDS slot
    // (row, p) - 16-byte units, p = lane & 7 - receives segment p ^ (row & 7).
    const int8_t *asrc[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int r = (wave * 4 + i) * 8 + (lane >> 3);
        const int row = min(m0 + r, a.M - 1);   // clamp: rows past M are never stored
        asrc[i] = a.xq + (int64_t)row * a.ldq + (((lane & 7) ^ (r & 7)) << 4);
    }
    // weight source: load (j, t) serves the wavefront's 32-channel tile j and
    // k-blocks t (low nibbles) and t + 2 (high nibbles).  Channel l & 31 lives in
    // the blob's 16-row chunk (l & 31) >> 4 at blob lane (2 t + (l >> 5)) * 16 + (l & 15).
    const agq_u4 *bsrc[4];
#pragma unroll
    for (int jt = 0; jt < 4; ++jt) {
        const int j = jt >> 1, t = jt & 1;
        const int chunk_row = n0 / 16 + wave * 4 + j * 2 + ((lane & 31) >> 4);
        bsrc[jt] = a.blob + ((int64_t)chunk_row * a.KT) * 64 + (2 * t + (lane >> 5)) * 16 + (lane & 15);
    }

    const int KT = a.KT;
    auto issue = [&](int kt, unsigned char *st) {
        const int k = min(kt, KT - 1);      // past the end: reload the last step (harmless, keeps counts uniform)
        const unsigned char *stage = st + wave * 4096;
#pragma unroll
        for (int i = 0; i < 4; ++i) lds_dma16(asrc[i] + (int64_t)k * BK, stage + i * 1024);
#pragma unroll
        for (int j = 0; j < 4; ++j) lds_dma16(bsrc[j] + (int64_t)k * 64, stage + kABytes + j * 1024);
    };

    agq_v16i acc[4][2];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0;

    // One K step: the activation fragments of k-block t+1 are requested from LDS
    // before the eight MFMAs of k-block t are issued, so the matrix core never
    // waits for an LDS round trip inside a step (the four wavefronts of a
    // workgroup run in lockstep and would otherwise all stall together).
    auto compute = [&](const unsigned char *st) {
        const agq_u4 *stage = reinterpret_cast<const agq_u4 *>(st) + lane;
        // fragment (token tile i, k-block t): row 32 i + (lane & 31), segment 2 t + (lane >> 5), swizzled
        const agq_u4 *arow = reinterpret_cast<const agq_u4 *>(st) + (lane & 31) * 8;
        const int sw7 = lane & 7, g = lane >> 5;
        agq_u4 bset[4], xa[4], xn[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) xa[i] = arow[i * 256 + (g ^ sw7)];
#pragma unroll
        for (int j = 0; j < 4; ++j) bset[j] = stage[(kAChunks + wave * 4 + j) * 64];
#pragma unroll
        for (int t = 0; t < 4; ++t) {
            if (t < 3) {
#pragma unroll
                for (int i = 0; i < 4; ++i) xn[i] = arow[i * 256 + ((2 * (t + 1) + g) ^ sw7)];
            }
            __builtin_amdgcn_sched_barrier(0);
            agq_v4i wb[2];
#pragma unroll
            for (int j = 0; j < 2; ++j) {
                const agq_u4 p = bset[j * 2 + (t & 1)];
                const agq_u4 w = t < 2 ? ((p << 4) & 0xF0F0F0F0u) : (p & 0xF0F0F0F0u);
                wb[j] = __builtin_bit_cast(agq_v4i, w);
            }
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const agq_v4i x = __builtin_bit_cast(agq_v4i, xa[i]);
#pragma unroll
                for (int j = 0; j < 2; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_i32_32x32x32_i8(wb[j], x, acc[i][j], 0, 0, 0);
            }
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int i = 0; i < 4; ++i) xa[i] = xn[i];
        }
    };

    issue(0, stage0);
    issue(1, stage1);
    issue(2, stage2);
    // Every step kt: wait until this wavefront's copies of step kt have landed (the
    // sixteen of steps kt+1 and kt+2 may still fly), meet the others (their copies
    // of step kt are in LDS too, and everybody has left step kt-1, whose LDS stage
    // is refilled next), start the copies of step kt+3, multiply step kt.
#define AGQ_STEP(KT_, ST, ST3)                                               \
    if ((KT_) < KT) {                                                        \
        asm volatile("s_waitcnt vmcnt(16)" ::: "memory");                    \
        __syncthreads();                                                     \
        issue((KT_) + 3, ST3);                                               \
        compute(ST);                                                         \
    }
    for (int kt = 0; kt < KT; kt += 4) {      // stage of step kt is kt % 4
        AGQ_STEP(kt, stage0, stage3)
        AGQ_STEP(kt + 1, stage1, stage0)
        AGQ_STEP(kt + 2, stage2, stage1)
        AGQ_STEP(kt + 3, stage3, stage2)
    }
#undef AGQ_STEP
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");   // drain the trailing reloads before the LDS goes away

    // fused epilogue: drop the factor 16 of the widened weights, dequantize with
    // 2^e * sw[n], store four consecutive channels per lane.  Accumulator
    // register 4 q + r of lane l is channel 8 q + 4 (l >> 5) + r of the 32-channel
    // tile, token l & 31 of the 32-token tile.
    const int mrow = m0 + (lane & 31);
    const int ncol = n0 + wave * 64 + (lane >> 5) * 4;
    const bool vec_ok = (a.ldy & 3) == 0;
#pragma unroll
    for (int j = 0; j < 2; ++j) {
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const int n = ncol + j * 32 + q * 8;
            if (n >= a.N) continue;
            const bool full = n + 3 < a.N;
            const float g0 = a.scale_e * __half2float(a.sw[n]);
            const float g1 = n + 1 < a.N ? a.scale_e * __half2float(a.sw[n + 1]) : 0.0f;
            const float g2 = n + 2 < a.N ? a.scale_e * __half2float(a.sw[n + 2]) : 0.0f;
            const float g3 = n + 3 < a.N ? a.scale_e * __half2float(a.sw[n + 3]) : 0.0f;
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const int m = mrow + i * 32;
                if (m >= a.M) continue;
                const int v0 = acc[i][j][4 * q] >> AGQ_W_SHIFT, v1 = acc[i][j][4 * q + 1] >> AGQ_W_SHIFT;
                const int v2 = acc[i][j][4 * q + 2] >> AGQ_W_SHIFT, v3 = acc[i][j][4 * q + 3] >> AGQ_W_SHIFT;
                const __half h0 = agq_dequant(v0, g0), h1 = agq_dequant(v1, g1);
                const __half h2 = agq_dequant(v2, g2), h3 = agq_dequant(v3, g3);
                __half *yp = a.y + (int64_t)m * a.ldy + n;
                if (full && vec_ok) {
                    uint2 pk;
                    pk.x = (uint32_t)__half_as_ushort(h0) | ((uint32_t)__half_as_ushort(h1) << 16);
                    pk.y = (uint32_t)__half_as_ushort(h2) | ((uint32_t)__half_as_ushort(h3) << 16);
                    *reinterpret_cast<uint2 *>(yp) = pk;
                } else {
                    yp[0] = h0;
                    if (n + 1 < a.N) yp[1] = h1;
                    if (n + 2 < a.N) yp[2] = h2;
                    if (n + 3 < a.N) yp[3] = h3;
                }
                if (a.acc_out) {
                    int32_t *ap = a.acc_out + (int64_t)m * a.N + n;
                    ap[0] = v0;
                    if (n + 1 < a.N) ap[1] = v1;
                    if (n + 2 < a.N) ap[2] = v2;
                    if (n + 3 < a.N) ap[3] = v3;
                }
            }
        }
    }
}

}  // namespace

int agq_launch_gemm_tiled(const int8_t *xq, int64_t ldq, int64_t M, int64_t K, int e, const void *w_packed,
                          const void *sw, int64_t N, void *y, int64_t ldy, int32_t *acc_out, void *stream) {
    TiledArgs a;
    a.xq = xq;
    a.ldq = ldq;
    a.M = (int)M;
    a.N = (int)N;
    a.K = (int)K;
    a.KT = (int)agq_k_tiles(K);
    a.tiles_m = (int)((M + BM - 1) / BM);
    a.tiles_n = (int)((N + BN - 1) / BN);
    a.blob = (const agq_u4 *)w_packed;
    a.sw = (const __half *)sw;
    a.y = (__half *)y;
    a.ldy = ldy;
    a.acc_out = acc_out;
    a.scale_e = ldexpf(1.0f, e);
    gemm_tiled_kernel<<<(unsigned)(a.tiles_m * a.tiles_n), kThreads, 0, (hipStream_t)stream>>>(a);
    return (int)hipGetLastError();
}
