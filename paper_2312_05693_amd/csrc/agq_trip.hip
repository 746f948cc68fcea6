// agq - TRIP: per-channel power-of-two factors on top of the layer-wise
// activation step (Section 4.3, Eq.5-8) and the weight blob that carries them
// into the matrix product (Section 4.4, efficient TRIP matrix multiplication).
//
// Eq.5 quantizes input channel k with the step 2^(e + alpha[k]); Section 4.4 moves
// the factor onto row k of the weights: acc = sum_k (q_k - zp) 2^alpha[k] w[n,k].
// A 4-bit weight times 2^alpha no longer fits four bits, and the int8 operand of
// the matrix instruction has no room for q 2^alpha either, so the channels with
// alpha > 0 (the outlier channels, a small minority) are taken out of the main
// product: their weights are zero in the main chunks of the blob, and they come
// back as extra 128-wide chunks, one factor per chunk, whose partial product is
// shifted left by that factor in the int32 accumulator (exact).  The activation
// side gathers those channels by an index table stored with the blob.
#include <hip/hip_runtime.h>
#include <hip/hip_fp16.h>

#include <vector>

#include "agq_device.h"
#include "agq_internal.h"

namespace {

constexpr int kThreads = 256;
constexpr int kSearchThreads = 64;   // channels per workgroup of the factor search (one wavefront per factor)
inline int64_t blocks_for(int64_t n) { return (n + kThreads - 1) / kThreads; }

// ------------------------------------------------------------------ Eq.8
//
// One thread per (channel, factor): wavefront a of a workgroup handles factor a for
// 64 channels, walks the tokens in order and keeps the squared error of quantizing
// (Eq.5, clip included) and dequantizing its channel with that factor, in float64:
// every residual is exact, each square and each addition rounds once, so the sums
// (and with them the argmin) are the same on any machine that adds in token
// order.  Equal errors keep the smaller factor.
__global__ __launch_bounds__(kSearchThreads * 5) void trip_search_kernel(const __half *__restrict__ x, int64_t M,
                                                                          int64_t K, int64_t ldx, int e, double lo,
                                                                          double hi, int kmax,
                                                                          int8_t *__restrict__ alpha) {
#pragma clang fp contract(off)
    __shared__ double errs[5][kSearchThreads];
    const int a = threadIdx.y;                                   // factor of this wavefront (blockDim.y = kmax + 1)
    const int64_t c = min((int64_t)blockIdx.x * kSearchThreads + threadIdx.x, K - 1);
    const double inv = ldexp(1.0, -(e + a)), step = ldexp(1.0, e + a);
    double err = 0.0;
    // tokens are fetched sixteen at a time (the loads do not depend on the sum), and added in order
    constexpr int kAhead = 16;
    for (int64_t m0 = 0; m0 < M; m0 += kAhead) {
        __half xv[kAhead];
#pragma unroll
        for (int i = 0; i < kAhead; ++i) xv[i] = x[min(m0 + i, M - 1) * ldx + c];
#pragma unroll
        for (int i = 0; i < kAhead; ++i) {
            if (m0 + i >= M) break;
            const double v = (double)__half2float(xv[i]);
            // lo, hi are the grid bounds minus the zero point: CLIP(round + zp) - zp
            const double q = fmin(fmax(rint(v * inv), lo), hi);
            const double r = v - q * step;
            const double sq = r * r;
            err = err + sq;
        }
    }
    errs[a][threadIdx.x] = err;
    __syncthreads();
    if (a == 0 && (int64_t)blockIdx.x * kSearchThreads + threadIdx.x < K) {
        int best = 0;
        double best_err = errs[0][threadIdx.x];
        for (int b = 1; b <= kmax; ++b)
            if (errs[b][threadIdx.x] < best_err) {
                best = b;
                best_err = errs[b][threadIdx.x];
            }
        alpha[c] = (int8_t)best;
    }
}

// ------------------------------------------------------------------ blob
//
// Same chunk format as the plain blob (see the packer of the plain blob): chunk
// (nt, c) at index nt * KTall + c; c < E are the extra chunks, c >= E the main
// chunk c - E.  Slot j of a chunk is the j-th k position of its 128.
__global__ __launch_bounds__(kThreads) void pack_trip_kernel(const int8_t *__restrict__ wq, int64_t N, int64_t K,
                                                              int64_t KTall, int E, const int32_t *__restrict__ idx,
                                                              const int8_t *__restrict__ alpha, int64_t total_words,
                                                              uint32_t *__restrict__ blob, int32_t *bad) {
    const int64_t i = (int64_t)blockIdx.x * kThreads + threadIdx.x;
    if (i >= total_words) return;
    const int64_t chunk = i >> 8;
    const int within = (int)(i & 255), lane = within >> 2, d = within & 3;
    const int64_t nt = chunk / KTall, c = chunk - nt * KTall;
    const int64_t n = nt * 16 + (lane & 15);
    uint32_t word = 0;
    int nbad = 0;
    if (n < N) {
        const int j0 = (lane >> 4) * 16 + 4 * d;   // slots j0 .. j0+3 (low nibbles) and 64 + j0 .. (high nibbles)
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            int a = 0, b = 0;
            if (c < E) {
                const int ka = idx[c * 128 + j0 + j], kb = idx[c * 128 + 64 + j0 + j];
                if (ka >= 0) a = wq[n * K + ka];
                if (kb >= 0) b = wq[n * K + kb];
                // saturation of these values is counted where the main chunks meet them
                a = min(max(a, -8), 7);
                b = min(max(b, -8), 7);
            } else {
                const int64_t ka = (c - E) * 128 + j0 + j, kb = ka + 64;
                a = wq[n * K + ka];
                b = wq[n * K + kb];
                const int as = min(max(a, -8), 7), bs = min(max(b, -8), 7);
                nbad += (as != a) + (bs != b);
                a = alpha[ka] ? 0 : as;
                b = alpha[kb] ? 0 : bs;
            }
            word |= (uint32_t)((a & 0xF) | ((b & 0xF) << 4)) << (8 * j);
        }
    }
    blob[i] = word;
    if (nbad && bad) atomicAdd(bad, nbad);
}

// sum_k 2^alpha[k] * (saturated) w[n,k] per output channel, padded channels 0
__global__ __launch_bounds__(64) void wsum_trip_kernel(const int8_t *__restrict__ wq, int64_t N, int64_t K,
                                                        const int8_t *__restrict__ alpha, int32_t *__restrict__ wsum) {
    const int64_t n = blockIdx.x;
    int sum = 0;
    if (n < N)
        for (int64_t k = threadIdx.x; k < K; k += 64) sum += min(max((int)wq[n * K + k], -8), 7) << alpha[k];
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) sum += __shfl_down(sum, off);
    if (threadIdx.x == 0) wsum[n] = sum;
}

__device__ __forceinline__ int nibble_of(const uint32_t *blob, int64_t n, int64_t chunk_index, int slot) {
    const int s = slot >> 6, g = (slot & 63) >> 4, d = (slot & 15) >> 2, j = slot & 3;
    const int lane = g * 16 + (int)(n & 15);
    const uint32_t word = blob[(chunk_index * 64 + lane) * 4 + d];
    const int code = (int)((word >> (8 * j + 4 * s)) & 0xF);
    return (code ^ 8) - 8;
}

// main chunks give the channels with factor 0, the extra chunks the others
__global__ __launch_bounds__(kThreads) void unpack_trip_kernel(const uint32_t *__restrict__ blob, int64_t N, int64_t K,
                                                                int64_t KTall, int E, const int32_t *__restrict__ idx,
                                                                const int8_t *__restrict__ alpha,
                                                                int8_t *__restrict__ wq) {
    const int64_t i = (int64_t)blockIdx.x * kThreads + threadIdx.x;
    const int64_t main_items = N * K, extra_items = N * (int64_t)E * 128;
    if (i < main_items) {
        const int64_t n = i / K, k = i - n * K;
        if (alpha[k] == 0) wq[i] = (int8_t)nibble_of(blob, n, (n >> 4) * KTall + E + (k >> 7), (int)(k & 127));
    } else if (i < main_items + extra_items) {
        const int64_t r = i - main_items;
        const int64_t n = r / (E * 128);
        const int slot = (int)(r - n * (E * 128));
        const int k = idx[slot];
        if (k >= 0) wq[n * K + k] = (int8_t)nibble_of(blob, n, (n >> 4) * KTall + (slot >> 7), slot & 127);
    }
}

// ------------------------------------------------------------------ activation pre-pass (many tokens)
//
// As the plain pre-pass (Eq.2 into 16 KiB stages in MFMA operand order), with
// E more K steps in front: step c < E gathers the channels idx[c * 128 ..] and
// quantizes them with the step 2^(e + factor of chunk c) (Eq.5).
__global__ __launch_bounds__(kThreads) void prepack_trip_kernel(const __half *__restrict__ x, int64_t M, int64_t KTall,
                                                                 int E, int64_t ldx, AgqQuant q,
                                                                 const int32_t *__restrict__ meta,
                                                                 const int32_t *__restrict__ idx,
                                                                 uint4 *__restrict__ out) {
    __shared__ uint4 tile[256];                       // 4 KiB in operand order
    const int tid = threadIdx.x;
    const int64_t kt = blockIdx.x, mt = blockIdx.y;  // K step, 32-token tile
    const int r = tid >> 3, c = tid & 7;              // token row in the tile, 16-wide k segment
    const int64_t m = mt * 32 + r;
    uint4 codes = make_uint4(0, 0, 0, 0);
    if (m < M) {
        if (kt >= E) {
            const __half *xp = x + m * ldx + (kt - E) * 128 + c * 16;
            const uint2 lo = agq_quant8<true>(*reinterpret_cast<const uint4 *>(xp), q);
            const uint2 hi = agq_quant8<true>(*reinterpret_cast<const uint4 *>(xp + 8), q);
            codes = make_uint4(lo.x, lo.y, hi.x, hi.y);
        } else {
            AgqQuant qe = q;
            qe.scale = ldexpf(q.scale, -meta[kt]);
            const int32_t *ip = idx + kt * 128 + c * 16;
            uint32_t b[16];
#pragma unroll
            for (int j = 0; j < 16; ++j) {
                const int k = max(ip[j], 0);           // an unused slot meets zero weights
                b[j] = agq_quant1(__half2float(x[m * ldx + k]), qe) + (uint32_t)qe.zp;
            }
            codes = make_uint4(agq_pack4(b[0], b[1], b[2], b[3]), agq_pack4(b[4], b[5], b[6], b[7]),
                               agq_pack4(b[8], b[9], b[10], b[11]), agq_pack4(b[12], b[13], b[14], b[15]));
        }
    }
    tile[(c >> 1) * 64 + (c & 1) * 32 + r] = codes;   // k-block c >> 1, lane 32 (c & 1) + r
    __syncthreads();
    out[(((mt >> 2) * KTall + kt) * 16 + (mt & 3) * 4) * 64 + tid] = tile[tid];
}

}  // namespace

AgqQuant agq_make_quant_signed(int bits, int e, int zp);

int agq_launch_trip_search(const void *x, int64_t M, int64_t K, int64_t ldx, int bits, int e, int zp, int kmax,
                           int8_t *alpha, void *stream) {
    const int lo = zp ? 0 : -(1 << (bits - 1)), hi = zp ? (1 << bits) - 1 : (1 << (bits - 1)) - 1;
    trip_search_kernel<<<(unsigned)((K + kSearchThreads - 1) / kSearchThreads), dim3(kSearchThreads, kmax + 1), 0,
                         (hipStream_t)stream>>>(
        (const __half *)x, M, K, ldx, e, (double)(lo - zp), (double)(hi - zp), kmax, alpha);
    return (int)hipGetLastError();
}

// Extra chunks needed by a set of factors: per factor 4, 3, 2, 1 the channels that carry it,
// rounded up to whole chunks.  -1: a factor outside 0..4, or more than AGQ_TRIP_MAX_E chunks.
int agq_trip_count_extra(const int8_t *alpha_host, int64_t K) {
    int64_t count[5] = {0, 0, 0, 0, 0};
    for (int64_t k = 0; k < K; ++k) {
        if (alpha_host[k] < 0 || alpha_host[k] > 4) return -1;
        ++count[alpha_host[k]];
    }
    int64_t E = 0;
    for (int a = 1; a <= 4; ++a) E += (count[a] + 127) / 128;
    return E > AGQ_TRIP_MAX_E ? -1 : (int)E;
}

int agq_launch_pack_trip(const int8_t *wq, int64_t N, int64_t K, const int8_t *alpha_host, void *packed, int32_t *bad,
                         void *stream) {
    const int E = agq_trip_count_extra(alpha_host, K);
    if (E < 0) return (int)hipErrorInvalidValue;
    const AgqTripLayout L = agq_trip_layout(N, K, E);
    // tables: chunks by descending factor, channels in ascending order inside a factor
    std::vector<int32_t> table(32 + (size_t)E * 128, -1);
    int32_t *meta = table.data(), *idx = table.data() + 32;
    for (int i = 0; i < 32; ++i) meta[i] = 0;
    int c = 0;
    for (int a = 4; a >= 1; --a) {
        int fill = 128;   // slots used in the current chunk
        for (int64_t k = 0; k < K; ++k) {
            if (alpha_host[k] != a) continue;
            if (fill == 128) {
                meta[c++] = a;
                fill = 0;
            }
            idx[(c - 1) * 128 + fill++] = (int32_t)k;
        }
    }
    for (int i = 0; i < E; ++i) meta[16 + i] = meta[i] - (i + 1 < E ? meta[i + 1] : 0);
    hipStream_t st = (hipStream_t)stream;
    char *base = (char *)packed;
    // the tables are small and this call is set-up work: copy, then wait, so that the host
    // buffers may go away
    if (hipMemcpyAsync(base + L.meta_off, table.data(), table.size() * 4, hipMemcpyHostToDevice, st) != hipSuccess)
        return (int)hipGetLastError();
    if (hipMemcpyAsync(base + L.alpha_off, alpha_host, (size_t)K, hipMemcpyHostToDevice, st) != hipSuccess)
        return (int)hipGetLastError();
    if (hipStreamSynchronize(st) != hipSuccess) return (int)hipGetLastError();
    const int64_t total_words = agq_n_tiles_padded(N) * L.KTall * 256;
    pack_trip_kernel<<<(unsigned)blocks_for(total_words), kThreads, 0, st>>>(
        wq, N, K, L.KTall, E, (const int32_t *)(base + L.idx_off), (const int8_t *)(base + L.alpha_off), total_words,
        (uint32_t *)packed, bad);
    wsum_trip_kernel<<<(unsigned)L.Npad, 64, 0, st>>>(wq, N, K, (const int8_t *)(base + L.alpha_off),
                                                      (int32_t *)(base + L.wsum_off));
    return (int)hipGetLastError();
}

int agq_launch_unpack_trip(const void *packed, int64_t N, int64_t K, int n_extra, int8_t *wq, void *stream) {
    const AgqTripLayout L = agq_trip_layout(N, K, n_extra);
    const char *base = (const char *)packed;
    const int64_t items = N * K + N * (int64_t)n_extra * 128;
    unpack_trip_kernel<<<(unsigned)blocks_for(items), kThreads, 0, (hipStream_t)stream>>>(
        (const uint32_t *)packed, N, K, L.KTall, n_extra, (const int32_t *)(base + L.idx_off),
        (const int8_t *)(base + L.alpha_off), wq);
    return (int)hipGetLastError();
}

int agq_launch_prepack_trip(const void *x, int bits, int64_t M, int64_t K, int64_t ldx, int e, int zp,
                            const void *packed, int64_t N, int n_extra, void *out, void *stream) {
    const AgqTripLayout L = agq_trip_layout(N, K, n_extra);
    const char *base = (const char *)packed;
    const AgqQuant q = agq_make_quant_signed(bits, e, zp);
    const dim3 grid((unsigned)L.KTall, (unsigned)(((M + 127) / 128) * 4));
    prepack_trip_kernel<<<grid, kThreads, 0, (hipStream_t)stream>>>((const __half *)x, M, L.KTall, n_extra, ldx, q,
                                                                     (const int32_t *)(base + L.meta_off),
                                                                     (const int32_t *)(base + L.idx_off), (uint4 *)out);
    return (int)hipGetLastError();
}
