// Tiled int8-MFMA kernel of the quantized linear layer for many tokens (the
// prefill regime, bound by the matrix cores).
//
// Workgroup tile 128 (tokens) x 256 (output channels), K step 128, four
// wavefronts side by side along the channels: each owns 128 x 64 as 8 x 4 MFMA
// tiles of 16 x 16 (v_mfma_i32_16x16x64_i8, 128 accumulator registers per lane).
//
//   activation codes: int8, copied HBM/L2 -> LDS by the wavefronts' direct
//     global-to-LDS loads (no registers in between), three stages deep.  A
//     stage is 16 chunks of 1 KiB, chunk (m-tile, step), laid out in MFMA operand
//     order - lane l = row l & 15, 16 consecutive k from 64 step + 16 (l >> 4) -
//     so that a fragment read is one conflict-free ds_read_b128 at lane * 16.
//     All four wavefronts read the whole stage.
//   weights: each wavefront streams its own 64 channels of the packed 4-bit blob
//     straight into registers (one coalesced 16-byte load per lane and 1 KiB
//     chunk, two K steps ahead) and widens them to int8 there: three bit
//     operations per eight weights.  The nibbles never touch LDS and cross HBM
//     and L2 at half the bytes of int8.
//
// The weight fragment is the MFMA's first operand and the activation the second:
// a lane then holds four consecutive output channels of one token, which makes
// the fp16 store 8 bytes per lane.
#include "agq_device.h"
#include "agq_internal.h"

typedef unsigned int agq_u4 __attribute__((ext_vector_type(4)));

namespace {

constexpr int BM = 128, BN = 256, BK = 128;
constexpr int kThreads = 256;
constexpr int kBand = 4;                  // token tiles per band of the tile walk
constexpr int kStages = 3;                // LDS stages of activation codes
constexpr int kAChunks = (BM / 16) * 2;   // 16 chunks of 1 KiB per stage
constexpr int kStageBytes = kAChunks * 1024;

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

// s_waitcnt immediate for "at most n vector-memory operations outstanding"
// (gfx9 encoding: vmcnt in bits 3:0 and 15:14, expcnt 6:4 and lgkmcnt 11:8 left open)
constexpr int vmcnt_imm(int n) { return (n & 15) | ((n >> 4) << 14) | (7 << 4) | (15 << 8); }

__device__ __forceinline__ void lds_dma16(const void *gsrc, void *lds_chunk) {
    // lane i's 16 bytes land at lds_chunk + 16 i (the LDS address is wave-uniform)
    __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void *)gsrc,
                                     (__attribute__((address_space(3))) void *)lds_chunk, 16, 0, 0);
}

__global__ __launch_bounds__(kThreads, 2) void gemm_tiled_kernel(const TiledArgs a) {
    extern __shared__ __align__(16) unsigned char smem[];
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

    // activation source of this lane for the four chunks its wavefront copies per stage
    const int8_t *asrc[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int c = wave * 4 + i, mt = c >> 1, s = c & 1;
        const int row = min(m0 + mt * 16 + (lane & 15), a.M - 1);   // clamp: rows past M are never stored
        asrc[i] = a.xq + (int64_t)row * a.ldq + s * 64 + (lane >> 4) * 16;
    }
    // weight source: this wavefront's four 16-channel tiles
    const agq_u4 *bsrc[4];
#pragma unroll
    for (int j = 0; j < 4; ++j) bsrc[j] = a.blob + ((int64_t)(n0 / 16 + wave * 4 + j) * a.KT) * 64 + lane;

    const int KT = a.KT;
    auto issue = [&](int kt, int st, agq_u4 (&bset)[4]) {
        const int k = min(kt, KT - 1);      // past the end: reload the last step (harmless, keeps counts uniform)
#pragma unroll
        for (int j = 0; j < 4; ++j) bset[j] = bsrc[j][(int64_t)k * 64];
        unsigned char *stage = smem + st * kStageBytes + wave * 4096;
#pragma unroll
        for (int i = 0; i < 4; ++i) lds_dma16(asrc[i] + (int64_t)k * BK, stage + i * 1024);
    };

    agq_v4i acc[8][4];
#pragma unroll
    for (int i = 0; i < 8; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) acc[i][j] = agq_v4i{0, 0, 0, 0};

    auto compute = [&](int st, const agq_u4 (&bset)[4]) {
        const agq_u4 *stage = reinterpret_cast<const agq_u4 *>(smem + st * kStageBytes) + lane;
#pragma unroll
        for (int s = 0; s < 2; ++s) {
            agq_v4i wb[4];
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const agq_u4 p = bset[j];
                const agq_u4 w = s == 0 ? ((p << 4) & 0xF0F0F0F0u) : (p & 0xF0F0F0F0u);
                wb[j] = __builtin_bit_cast(agq_v4i, w);
            }
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                const agq_v4i xa = __builtin_bit_cast(agq_v4i, stage[(i * 2 + s) * 64]);
#pragma unroll
                for (int j = 0; j < 4; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_i32_16x16x64_i8(wb[j], xa, acc[i][j], 0, 0, 0);
            }
        }
    };

    agq_u4 b0[4], b1[4], b2[4];
    issue(0, 0, b0);
    issue(1, 1, b1);
    // Every step: wait until this wavefront's loads of step kt have landed (the
    // eight loads of step kt+1 may still fly), meet the others (their copies of
    // step kt are in LDS, and everybody has left step kt-1, whose LDS stage is
    // the one refilled next), start the loads of step kt+2, multiply step kt.
#define AGQ_STEP(KT_, ST, CUR, ST2, NXT2)                   \
    if ((KT_) < KT) {                                       \
        __builtin_amdgcn_s_waitcnt(vmcnt_imm(8));           \
        __syncthreads();                                    \
        issue((KT_) + 2, ST2, NXT2);                        \
        compute(ST, CUR);                                   \
    }
    for (int kt = 0; kt < KT; kt += 3) {      // stage of step kt is kt % 3
        AGQ_STEP(kt, 0, b0, 2, b2)
        AGQ_STEP(kt + 1, 1, b1, 0, b0)
        AGQ_STEP(kt + 2, 2, b2, 1, b1)
    }
#undef AGQ_STEP
    __builtin_amdgcn_s_waitcnt(vmcnt_imm(0));   // drain the trailing reloads before the LDS goes away

    // fused epilogue: drop the factor 16 of the widened weights, dequantize with
    // 2^e * sw[n], store four consecutive channels per lane
    const int mrow = m0 + (lane & 15);
    const int ncol = n0 + wave * 64 + (lane >> 4) * 4;
    const bool vec_ok = (a.ldy & 3) == 0;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        const int n = ncol + j * 16;
        if (n >= a.N) continue;
        const bool full = n + 3 < a.N;
        float g0 = a.scale_e * __half2float(a.sw[n]);
        float g1 = n + 1 < a.N ? a.scale_e * __half2float(a.sw[n + 1]) : 0.0f;
        float g2 = n + 2 < a.N ? a.scale_e * __half2float(a.sw[n + 2]) : 0.0f;
        float g3 = n + 3 < a.N ? a.scale_e * __half2float(a.sw[n + 3]) : 0.0f;
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            const int m = mrow + i * 16;
            if (m >= a.M) continue;
            const int v0 = acc[i][j].x >> AGQ_W_SHIFT, v1 = acc[i][j].y >> AGQ_W_SHIFT;
            const int v2 = acc[i][j].z >> AGQ_W_SHIFT, v3 = acc[i][j].w >> AGQ_W_SHIFT;
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
    const size_t lds = (size_t)kStages * kStageBytes;   // 48 KiB
    gemm_tiled_kernel<<<(unsigned)(a.tiles_m * a.tiles_n), kThreads, lds, (hipStream_t)stream>>>(a);
    return (int)hipGetLastError();
}
