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

// keep[i] = fewer than n_keep tokens beat token i (higher score, or equal score
// and lower index); survivors are written in ascending order
__global__ __launch_bounds__(kSelThreads) void prune_select_kernel(const int32_t *__restrict__ score, int S, int n_keep,
                                                                    int32_t *__restrict__ idx_out) {
    extern __shared__ int sc[];          // S scores, then kSelThreads scan cells
    int *cnt = sc + S;
    for (int i = threadIdx.x; i < S; i += kSelThreads) sc[i] = score[i];
    __syncthreads();
    const int per = (S + kSelThreads - 1) / kSelThreads;
    const int lo = threadIdx.x * per, hi = min(lo + per, S);
    unsigned long long keepmask = 0;     // per <= 16 for S <= 16384
    int mine = 0;
    for (int i = lo; i < hi; ++i) {
        const int si = sc[i];
        int rank = 0;
        for (int j = 0; j < S; ++j) {
            const int sj = sc[j];
            rank += (sj > si) || (sj == si && j < i);
        }
        if (rank < n_keep) {
            keepmask |= 1ull << (i - lo);
            ++mine;
        }
    }
    cnt[threadIdx.x] = mine;
    __syncthreads();
    for (int off = 1; off < kSelThreads; off <<= 1) {
        const int v = threadIdx.x >= off ? cnt[threadIdx.x - off] : 0;
        __syncthreads();
        cnt[threadIdx.x] += v;
        __syncthreads();
    }
    int pos = cnt[threadIdx.x] - mine;
    for (int i = lo; i < hi; ++i)
        if (keepmask >> (i - lo) & 1) idx_out[pos++] = i;
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
    const size_t lds = ((size_t)S + kSelThreads) * sizeof(int);
    hipError_t err = hipFuncSetAttribute((const void *)prune_select_kernel, hipFuncAttributeMaxDynamicSharedMemorySize,
                                         (int)lds);
    if (err != hipSuccess) return (int)err;
    prune_select_kernel<<<1, kSelThreads, lds, st>>>(score, (int)S, (int)n_keep, idx);
    gather_rows_kernel<<<(unsigned)n_keep, 256, 0, st>>>((const uint4 *)x, idx, d / 8, (uint4 *)x_out);
    return (int)hipGetLastError();
}
