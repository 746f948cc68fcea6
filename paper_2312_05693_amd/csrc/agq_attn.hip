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

typedef _Float16 agq_v8h __attribute__((ext_vector_type(8)));
typedef float agq_v4f __attribute__((ext_vector_type(4)));

namespace {

constexpr int kQRows = 64;      // query rows per workgroup (16 per wavefront)
constexpr int kKeys = 64;       // keys per step
constexpr int kVPad = kKeys + 8;  // row stride of the transposed V tile in halves (144 B: conflict-free 16-byte reads)
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
};

// Eq.3 code of one fp16 bit pattern in [0, 1]
__device__ __forceinline__ int log2_code(uint32_t h, int qmax) {
    int c = 15 - (int)((h + 599u) >> 10);
    if (h < 1024u) c = h >= 725u ? 14 : 15;
    return max(min(c, qmax), 0);
}

__global__ __launch_bounds__(256) void log2_attn_kernel(const AttnArgs a) {
    __shared__ __align__(16) _Float16 vt[kMaxD * kVPad];   // V tile, transposed: [d][key]
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int h = blockIdx.y;
    const int q0 = blockIdx.x * kQRows;
    const int S = a.S, D = a.D;
    const int ntile = D >> 4;

    const int row = q0 + wave * 16 + (lane & 15);       // query row of this lane's P fragment
    const int rowc = min(row, S - 1);
    const int g = lane >> 4;
    const uint16_t *prow = a.p + ((int64_t)h * S + rowc) * S;
    const int8_t *vh = a.v + (int64_t)h * S * D;
    const int last_key = a.causal ? min(q0 + kQRows, S) : S;   // keys needed by this workgroup
    const int row_limit = a.causal ? row : S - 1;               // last key this row may use

    agq_v4f acc[kMaxD / 16];
#pragma unroll
    for (int j = 0; j < kMaxD / 16; ++j) acc[j] = agq_v4f{0.f, 0.f, 0.f, 0.f};

    for (int k0 = 0; k0 < last_key; k0 += kKeys) {
        __syncthreads();   // previous tile fully consumed
        // V tile: 16 channels of one key per lane, int8 -> fp16, scattered transposed
        for (int idx = threadIdx.x; idx < kKeys * (D >> 4); idx += blockDim.x) {
            const int key = idx / (D >> 4), dq = idx - key * (D >> 4);
            uint4 raw = make_uint4(0, 0, 0, 0);
            if (k0 + key < S) raw = *reinterpret_cast<const uint4 *>(vh + (int64_t)(k0 + key) * D + dq * 16);
            const uint32_t w[4] = {raw.x, raw.y, raw.z, raw.w};
#pragma unroll
            for (int b = 0; b < 16; ++b) {
                const int val = (int)(int8_t)(w[b >> 2] >> (8 * (b & 3)));
                vt[(dq * 16 + b) * kVPad + key] = (_Float16)val;
            }
        }
        __syncthreads();

        // P fragment: 16 consecutive keys of one row per lane, two MFMA steps of 8
        uint4 praw[2];
        const int kbase = k0 + g * 16;
#pragma unroll
        for (int t = 0; t < 2; ++t) {
            praw[t] = make_uint4(0, 0, 0, 0);
            if (kbase + t * 8 < S) praw[t] = *reinterpret_cast<const uint4 *>(prow + kbase + t * 8);
        }
        agq_v8h pf[2];
        uint32_t codes[4];
#pragma unroll
        for (int t = 0; t < 2; ++t) {
            const uint32_t w[4] = {praw[t].x, praw[t].y, praw[t].z, praw[t].w};
            uint32_t cw = 0;
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                const uint32_t hb = (w[i >> 1] >> (16 * (i & 1))) & 0xFFFFu;
                const int key = kbase + t * 8 + i;
                const int c = log2_code(hb, a.qmax);
                const bool live = key <= row_limit && key < S;
                // 2^(qmax - c) as fp16: exponent field 15 + qmax - c; dead entries are 0
                const uint16_t bits = live ? (uint16_t)((15 + a.qmax - c) << 10) : (uint16_t)0;
                pf[t][i] = __builtin_bit_cast(_Float16, bits);
                cw |= (uint32_t)(live ? c : a.qmax) << (4 * i);
            }
            codes[t] = cw;
        }
        if (a.codes && row < S && kbase < S) {
            uint8_t *dst = a.codes + ((int64_t)h * S + row) * (S >> 1) + (kbase >> 1);
            *reinterpret_cast<uint32_t *>(dst) = codes[0];
            if (kbase + 8 < S) *reinterpret_cast<uint32_t *>(dst + 4) = codes[1];
        }

#pragma unroll
        for (int t = 0; t < 2; ++t) {
#pragma unroll
            for (int j = 0; j < kMaxD / 16; ++j) {
                if (j < ntile) {
                    const agq_v8h vf = *reinterpret_cast<const agq_v8h *>(&vt[(j * 16 + (lane & 15)) * kVPad + g * 16 + t * 8]);
                    acc[j] = __builtin_amdgcn_mfma_f32_16x16x32_f16(vf, pf[t], acc[j], 0, 0, 0);
                }
            }
        }
    }

    // entries of the code map to the right of the last tile this workgroup visited
    if (a.codes && a.causal && row < S) {
        const uint32_t fill = 0x11111111u * (uint32_t)a.qmax;
        uint8_t *dst = a.codes + ((int64_t)h * S + row) * (S >> 1);
        const int start = ((last_key + kKeys - 1) / kKeys) * kKeys;
        for (int k = start + g * 8; k < S; k += 32) *reinterpret_cast<uint32_t *>(dst + (k >> 1)) = fill;
    }

    // lane holds four consecutive channels (4 g + r) of query row (lane & 15)
    if (row < S) {
#pragma unroll
        for (int j = 0; j < kMaxD / 16; ++j) {
            if (j < ntile) {
                __half hv[4];
#pragma unroll
                for (int r = 0; r < 4; ++r) hv[r] = __float2half_rn(acc[j][r] * a.out_scale);
                *reinterpret_cast<uint2 *>(a.o + (int64_t)row * ((int64_t)a.H * D) + (int64_t)h * D + j * 16 + g * 4) =
                    *reinterpret_cast<const uint2 *>(hv);
            }
        }
    }

    // importance of a token = attention it pays to the first token, summed over
    // heads as exact integers p * 2^24 (Section 4.3)
    if (a.score && h == 0 && threadIdx.x < kQRows) {
        const int i = q0 + threadIdx.x;
        if (i < S) {
            int sum = 0;
            for (int hh = 0; hh < a.H; ++hh) {
                const uint16_t hb = a.p[((int64_t)hh * S + i) * S];
                sum += (int)(__half2float(__ushort_as_half(hb)) * 16777216.0f);
            }
            a.score[i] = sum;
        }
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
    dim3 grid((unsigned)((S + kQRows - 1) / kQRows), (unsigned)H);
    log2_attn_kernel<<<grid, 256, 0, (hipStream_t)stream>>>(a);
    return (int)hipGetLastError();
}

int agq_launch_prune(const int32_t *score, int64_t S, int64_t n_keep, const void *x, int64_t d, int32_t *idx,
                     void *x_out, void *stream) {
    hipStream_t st = (hipStream_t)stream;
    prune_select_kernel<<<1, kSelThreads, 0, st>>>(score, (int)S, (int)n_keep, idx);
    gather_rows_kernel<<<(unsigned)n_keep, 256, 0, st>>>((const uint4 *)x, idx, d / 8, (uint4 *)x_out);
    return (int)hipGetLastError();
}
