// Host-side launcher prototypes; every launcher returns hipError_t as int.
#pragma once
#include <stddef.h>
#include <stdint.h>

// geometry of the packed weight blob (see the packer in agq_quant.hip)
static inline int64_t agq_n_tiles_padded(int64_t N) { return ((N + 255) / 256) * 16; }  // 16-row tiles, padded to 256 rows
static inline int64_t agq_k_tiles(int64_t K) { return K / 128; }
// The blob ends with one int32 per (padded) output channel: the sum of its weights, which the
// asymmetric grid's correction term needs.
static inline size_t agq_blob_nibble_bytes(int64_t N, int64_t K) {
    return (size_t)agq_n_tiles_padded(N) * (size_t)agq_k_tiles(K) * 1024;
}
static inline const int32_t *agq_blob_wsum(const void *packed, int64_t N, int64_t K) {
    return (const int32_t *)((const char *)packed + agq_blob_nibble_bytes(N, K));
}

// ---- TRIP blob (Section 4.4, efficient TRIP matrix multiplication).  The input channels whose
// factor alpha is > 0 are served by E extra 128-wide chunks placed in front of the K/128 main
// chunks of every 16-channel tile (their weights are zero in the main chunks): a chunk holds
// channels of one factor only, chunks are ordered by descending factor.  After the nibbles:
//   int32 wsum[Npad]      sum_k 2^alpha[k] w[n,k]
//   int32 meta[32]        meta[c] = factor of extra chunk c; meta[16 + c] = left shift of the
//                         running accumulator after chunk c (Horner: factor minus the next
//                         chunk's factor, the main chunks counting as factor 0)
//   int32 idx[E * 128]    input channel of every slot of the extra chunks, -1 = unused slot
//   int8  alpha[K]        the factors (read by the packer and by unpack)
#define AGQ_TRIP_MAX_E 16   // == AGQ_TRIP_MAX_EXTRA of the public header
struct AgqTripLayout {
    int64_t KT, KTall, Npad;
    size_t nibble_bytes, wsum_off, meta_off, idx_off, alpha_off, total;
};
static inline AgqTripLayout agq_trip_layout(int64_t N, int64_t K, int E) {
    AgqTripLayout L;
    L.KT = agq_k_tiles(K);
    L.KTall = L.KT + E;
    L.Npad = agq_n_tiles_padded(N) * 16;
    L.nibble_bytes = (size_t)agq_n_tiles_padded(N) * (size_t)L.KTall * 1024;
    L.wsum_off = L.nibble_bytes;
    L.meta_off = L.wsum_off + (size_t)L.Npad * 4;
    L.idx_off = L.meta_off + 32 * 4;
    L.alpha_off = L.idx_off + (size_t)E * 128 * 4;
    L.total = L.alpha_off + (size_t)((K + 15) / 16) * 16;
    return L;
}

// tokens up to which the weight-streaming kernel is used
#define AGQ_DECODE_MAX_M 16
// ... and beyond that, sixteen rows per workgroup (grid.y row groups): every row group reads the weights again
// (from L2 after the first), so this pays while those reads stay small.  Measured on MI355X against the pre-pass
// plus the tiled kernel, which needs hundreds of 128 x 128 tiles to fill the chip and walks K serially: the
// row-group launch takes about 3.5 us + 0.36 us per MB read, the other path about 6.6 us + 3.7 us per 1000 of K
// (768 x 768 at 128 rows: 4.5 against 9.7 us; 4096 x 4096 at 64 rows: 16.7 against 22.2 us).
#define AGQ_ROW_GROUP_MAX_M 256
static inline bool agq_decode_row_groups(int x_kind, int64_t M, int64_t K, int64_t n_sum) {
    return x_kind == 0 && M > AGQ_DECODE_MAX_M && M <= AGQ_ROW_GROUP_MAX_M &&
           ((M + 15) / 16) * (K * n_sum / 2) <= 6000000 + 10200 * K;
}

int agq_launch_calibrate(const void *x, int64_t M, int64_t K, int64_t ldx, int bits, int32_t *e_dev, void *stream);
int agq_launch_quantize(const void *x, int64_t M, int64_t K, int64_t ldx, int bits, int e, int zp,
                        void *out, int64_t ld_out_bytes, int out_bits, void *stream);
int agq_launch_prepack_act(const void *x, int x_kind, int bits, int64_t M, int64_t K, int64_t ldx, int e, int zp,
                           void *out, void *stream);
int agq_launch_pack(const int8_t *wq, int64_t N, int64_t K, void *packed, int32_t *bad, void *stream);
int agq_launch_unpack(const void *packed, int64_t N, int64_t K, int8_t *wq, void *stream);
struct agq_proj;
// n_extra >= 0 with TRIP blobs (all packed with the same factors, fp16 input); -1 for plain blobs
int agq_launch_gemm_decode(const void *x, int x_kind, int bits, int64_t M, int64_t K, int64_t ldx, int e, int zp,
                           const struct agq_proj *projs, int count, int n_extra, void *stream);
// K counts the main chunks only; with TRIP blobs (all packed with the same factors) x_tiles and the blobs hold
// n_extra more steps in front.  The `count` projections of the activation run as one launch.
int agq_launch_gemm_tiled(const void *x_tiles, int64_t M, int64_t K, int e, int corr, const struct agq_proj *projs, int count,
                          int n_extra, void *stream);
int agq_launch_trip_search(const void *x, int64_t M, int64_t K, int64_t ldx, int bits, int e, int zp, int kmax,
                           int8_t *alpha, void *stream);
int agq_trip_count_extra(const int8_t *alpha_host, int64_t K);   // number of extra chunks, -1 = bad factors or too many
int agq_launch_pack_trip(const int8_t *wq, int64_t N, int64_t K, const int8_t *alpha_host, void *packed, int32_t *bad,
                         void *stream);
int agq_launch_unpack_trip(const void *packed, int64_t N, int64_t K, int n_extra, int8_t *wq, void *stream);
int agq_launch_prepack_trip(const void *x, int bits, int64_t M, int64_t K, int64_t ldx, int e, int zp,
                            const void *packed, int64_t N, int n_extra, void *out, void *stream);
// Eq.2's unsigned grid (zp > 0) inside the GEMMs: codes travel as q - 2^(b-1) (signed, what the
// int8 MFMA takes) and sum_k (q - zp) w = sum_k (q - 2^(b-1)) w + corr * sum_k w.
static inline int agq_zp_corr(int bits, int zp) { return zp ? (1 << (bits - 1)) - zp : 0; }
int agq_launch_log2_attn(const void *p, int64_t H, int64_t S, int64_t D, int causal, int qmax,
                         const int8_t *vq, int e_v, void *o, void *codes, int32_t *score, void *stream);
int agq_launch_qk_log2_attn(const int8_t *q, const int8_t *k, const int8_t *v, int64_t H, int64_t S, int64_t D, int causal,
                            int qmax, int e_q, int e_k, int e_v, void *o, void *codes, int32_t *score, void *stream);
int agq_launch_prune(const int32_t *score, int64_t S, int64_t n_keep, const void *x, int64_t d,
                     int32_t *idx, void *x_out, void *stream);

// ---- fp16 operators of a block (agq_block.hip)
// res != NULL: x1 = fp16(res[idx ? idx[r] : r] + x[r]) is written to x1_out and normalised; pos_out / idx_out
// (optional) receive pos[...] and the source row of every output row
int agq_launch_rmsnorm(const void *x, const void *res, const int32_t *idx, const void *g, void *x1_out, void *y, int64_t rows,
                       int64_t d, double eps, const int32_t *pos, int32_t *pos_out, int32_t *idx_out, void *stream);
// q_q != NULL: rotate q and k, Eq.2 on q, k, v, int8 [H,S_pad,D] out (and zero[0..S_pad) = 0 when given);
// q_q == NULL: rotated fp16 q, k to q_rot, k_rot
int agq_launch_rope(const void *q, const void *k, const void *v, int64_t S, int64_t S_pad, int64_t H, int64_t D,
                    const int32_t *pos, const float *cos_t, const float *sin_t, int64_t P, int e_q, int e_k, int e_v,
                    int8_t *q_q, int8_t *k_q, int8_t *v_q, void *q_rot, void *k_rot, int32_t *zero, void *stream);
int agq_launch_swiglu(const void *gate, const void *up, void *out, int64_t n, void *stream);
int agq_launch_add(const void *a, const void *b, void *out, int64_t n, void *stream);
int agq_read_i32(const int32_t *dev, int32_t *host, int n, void *stream);
