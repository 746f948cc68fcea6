// Tiled int8-MFMA kernel of the quantized linear layer for many tokens (the
// prefill regime, bound by the matrix cores).
//
// Workgroup tile 128 (tokens) x 256 (output channels), K step 128, four
// wavefronts in a 2 x 2 arrangement, each owning 64 x 128 as 4 x 8 MFMA tiles of
// 16 x 16 (v_mfma_i32_16x16x64_i8, 128 accumulator registers per lane).
// Both operands are staged in LDS in MFMA operand order, so every fragment read
// is one conflict-free ds_read_b128 at lane * 16:
//   activation codes: chunk (m-tile, step) of 1 KiB, lane l = row l & 15,
//                     16 consecutive k starting at 64 step + 16 (l >> 4);
//   weights: the blob's own 1 KiB chunks, still 4-bit; a wavefront widens them
//            to int8 in registers (three bit operations per eight weights), so
//            the nibbles cross HBM, L2 and LDS at half the bytes of int8.
// The weight fragment is the MFMA's first operand and the activation the second:
// a lane then holds four consecutive output channels of one token, which makes
// the fp16 store 8 bytes per lane.
#include "agq_device.h"
#include "agq_internal.h"

namespace {

constexpr int BM = 128, BN = 256, BK = 128;
constexpr int kThreads = 256;
constexpr int kBand = 4;                  // token tiles per band of the tile walk
constexpr int kAChunks = (BM / 16) * 2;   // 16 chunks of 1 KiB per stage
constexpr int kBChunks = BN / 16;         // 16 chunks of 1 KiB per stage
constexpr int kStageBytes = (kAChunks + kBChunks) * 1024;

struct TiledArgs {
    const int8_t *xq;
    int64_t ldq;
    int M, N, K, KT;
    int tiles_m, tiles_n;
    const uint4 *blob;
    const __half *sw;
    __half *y;
    int64_t ldy;
    int32_t *acc_out;
    float scale_e;
};

__global__ __launch_bounds__(kThreads, 2) void gemm_tiled_kernel(const TiledArgs a) {
    extern __shared__ __align__(16) unsigned char smem[];
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
    const int band = bid / (kBand * a.tiles_n);
    const int rows = min(kBand, a.tiles_m - band * kBand);
    const int within = bid - band * kBand * a.tiles_n;
    const int tn = within / rows, tm = band * kBand + within - tn * rows;
    const int m0 = tm * BM, n0 = tn * BN;

    // global sources of this lane's staging loads: wave w moves A chunks 4w..4w+3
    // and B chunks 4w..4w+3 of every stage
    const int8_t *asrc[4];
    const uint4 *bsrc[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int c = wave * 4 + i, mt = c >> 1, s = c & 1;
        const int row = min(m0 + mt * 16 + (lane & 15), a.M - 1);
        asrc[i] = a.xq + (int64_t)row * a.ldq + s * 64 + (lane >> 4) * 16;
        bsrc[i] = a.blob + ((int64_t)(n0 / 16 + c) * a.KT) * 64 + lane;
    }
    uint4 *lds = reinterpret_cast<uint4 *>(smem);
    auto stage_a = [&](int buf, int chunk) { return lds + buf * (kStageBytes / 16) + chunk * 64; };
    auto stage_b = [&](int buf, int chunk) { return lds + buf * (kStageBytes / 16) + (kAChunks + chunk) * 64; };

    agq_v4i acc[4][8];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 8; ++j) acc[i][j] = agq_v4i{0, 0, 0, 0};

    uint4 ra[4], rb[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        ra[i] = *reinterpret_cast<const uint4 *>(asrc[i]);
        rb[i] = bsrc[i][0];
    }
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        stage_a(0, wave * 4 + i)[lane] = ra[i];
        stage_b(0, wave * 4 + i)[lane] = rb[i];
    }
    __syncthreads();

    for (int kt = 0; kt < a.KT; ++kt) {
        const int buf = kt & 1;
        const bool more = kt + 1 < a.KT;
        if (more) {
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                ra[i] = *reinterpret_cast<const uint4 *>(asrc[i] + (int64_t)(kt + 1) * BK);
                rb[i] = bsrc[i][(int64_t)(kt + 1) * 64];
            }
        }

        uint4 bp[8];
#pragma unroll
        for (int j = 0; j < 8; ++j) bp[j] = stage_b(buf, wn * 8 + j)[lane];
#pragma unroll
        for (int s = 0; s < 2; ++s) {
            agq_v4i xa[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const uint4 v = stage_a(buf, (wm * 4 + i) * 2 + s)[lane];
                xa[i] = agq_v4i{(int)v.x, (int)v.y, (int)v.z, (int)v.w};
            }
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                agq_v4i b0, b1;
                agq_unpack_w(bp[j], b0, b1);
                const agq_v4i wb = s == 0 ? b0 : b1;
#pragma unroll
                for (int i = 0; i < 4; ++i)
                    acc[i][j] = __builtin_amdgcn_mfma_i32_16x16x64_i8(wb, xa[i], acc[i][j], 0, 0, 0);
            }
        }

        if (more) {
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                stage_a(buf ^ 1, wave * 4 + i)[lane] = ra[i];
                stage_b(buf ^ 1, wave * 4 + i)[lane] = rb[i];
            }
        }
        __syncthreads();
    }

    // fused epilogue: drop the factor 16 of the widened weights, dequantize with
    // 2^e * sw[n], store four consecutive channels per lane
    const int mrow = m0 + wm * 64 + (lane & 15);
    const int ncol = n0 + wn * 128 + (lane >> 4) * 4;
#pragma unroll
    for (int j = 0; j < 8; ++j) {
        const int n = ncol + j * 16;
        if (n >= a.N) continue;
        float g[4];
#pragma unroll
        for (int r = 0; r < 4; ++r) g[r] = n + r < a.N ? a.scale_e * __half2float(a.sw[n + r]) : 0.0f;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int m = mrow + i * 16;
            if (m >= a.M) continue;
            const int v[4] = {acc[i][j].x >> AGQ_W_SHIFT, acc[i][j].y >> AGQ_W_SHIFT, acc[i][j].z >> AGQ_W_SHIFT,
                              acc[i][j].w >> AGQ_W_SHIFT};
            __half h[4];
#pragma unroll
            for (int r = 0; r < 4; ++r) h[r] = agq_dequant(v[r], g[r]);
            if (n + 3 < a.N && (a.ldy & 3) == 0) {
                *reinterpret_cast<uint2 *>(a.y + (int64_t)m * a.ldy + n) = *reinterpret_cast<const uint2 *>(h);
            } else {
                for (int r = 0; r < 4 && n + r < a.N; ++r) a.y[(int64_t)m * a.ldy + n + r] = h[r];
            }
            if (a.acc_out) {
                for (int r = 0; r < 4 && n + r < a.N; ++r) a.acc_out[(int64_t)m * a.N + n + r] = v[r];
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
    a.blob = (const uint4 *)w_packed;
    a.sw = (const __half *)sw;
    a.y = (__half *)y;
    a.ldy = ldy;
    a.acc_out = acc_out;
    a.scale_e = ldexpf(1.0f, e);
    const size_t lds = 2 * (size_t)kStageBytes;   // 64 KiB: two workgroups fit a CU
    gemm_tiled_kernel<<<(unsigned)(a.tiles_m * a.tiles_n), kThreads, lds, (hipStream_t)stream>>>(a);
    return (int)hipGetLastError();
}
