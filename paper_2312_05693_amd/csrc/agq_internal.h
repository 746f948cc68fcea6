// Host-side launcher prototypes; every launcher returns hipError_t as int.
#pragma once
#include <stddef.h>
#include <stdint.h>

// geometry of the packed weight blob (see agq_pack.hip)
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

// tokens up to which the weight-streaming kernel is used
#define AGQ_DECODE_MAX_M 16

int agq_launch_calibrate(const void *x, int64_t M, int64_t K, int64_t ldx, int bits, int32_t *e_dev, void *stream);
int agq_launch_quantize(const void *x, int64_t M, int64_t K, int64_t ldx, int bits, int e, int zp,
                        void *out, int64_t ld_out_bytes, int out_bits, void *stream);
int agq_launch_prepack_act(const void *x, int x_kind, int bits, int64_t M, int64_t K, int64_t ldx, int e, int zp,
                           void *out, void *stream);
int agq_launch_pack(const int8_t *wq, int64_t N, int64_t K, void *packed, int32_t *bad, void *stream);
int agq_launch_unpack(const void *packed, int64_t N, int64_t K, int8_t *wq, void *stream);
struct agq_proj;
int agq_launch_gemm_decode(const void *x, int x_kind, int bits, int64_t M, int64_t K, int64_t ldx, int e, int zp,
                           const struct agq_proj *projs, int count, void *stream);
int agq_launch_gemm_tiled(const void *x_tiles, int64_t M, int64_t K, int e, int corr,
                          const void *w_packed, const void *sw, int64_t N, void *y, int64_t ldy,
                          int32_t *acc_out, void *stream);
// Eq.2's unsigned grid (zp > 0) inside the GEMMs: codes travel as q - 2^(b-1) (signed, what the
// int8 MFMA takes) and sum_k (q - zp) w = sum_k (q - 2^(b-1)) w + corr * sum_k w.
static inline int agq_zp_corr(int bits, int zp) { return zp ? (1 << (bits - 1)) - zp : 0; }
int agq_launch_log2_attn(const void *p, int64_t H, int64_t S, int64_t D, int causal, int qmax,
                         const int8_t *vq, int e_v, void *o, void *codes, int32_t *score, void *stream);
int agq_launch_prune(const int32_t *score, int64_t S, int64_t n_keep, const void *x, int64_t d,
                     int32_t *idx, void *x_out, void *stream);
