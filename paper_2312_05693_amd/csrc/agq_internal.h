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
// K split of the tiled kernel.  A workgroup that has its CU (or its half of one) to itself takes about 470 ns per
// K step (twice the time of its MFMAs: a single wavefront per SIMD cannot cover its own waits), however few
// workgroups the launch has: with few 128 x 128 tiles and a long K most CUs idle while a few walk K.  Then `splits` workgroups share a tile's K steps (at least four each,
// at most one workgroup per CU in all) and leave int32 partial tiles behind the activation codes in the workspace,
// which a second kernel adds up.  That costs about 2 us for the launch and 0.45 us per MB of partial tiles
// (written, read back); the plan is the split count with the smallest sum under this model (all measured on
// MI355X).  M tokens, tiles_n = 128-wide column tiles of all projections of the call, KT = K steps (TRIP
// blobs: the extra steps in front included, all of which stay in the first slice: min_steps of them).
// splits == 1: no split, bytes == 0.
struct AgqSplitPlan {
    int splits, steps;
    size_t bytes;
    int64_t cost_ns;   // the model's time for the chosen plan (GEMM launches only)
};
static inline AgqSplitPlan agq_tiled_split_plan(int64_t M, int64_t tiles_n, int64_t KT, bool may_split, int min_steps = 0) {
    const int64_t tiles = ((M + 127) / 128) * tiles_n;
    AgqSplitPlan p = {1, (int)KT, 0, KT * 470 * (tiles > 256 ? (tiles + 255) / 256 : 1)};
    if (!may_split || tiles < 1 || tiles * 2 > 256 || KT < 8) return p;
    const int64_t part_bytes = ((M + 31) / 32) * 32 * tiles_n * 512;   // per split: rows that hold tokens x columns x 4
    for (int64_t s = 2; s <= KT / 4 && s * tiles <= 256; ++s) {
        const int64_t steps = (KT + s - 1) / s;
        if ((KT + steps - 1) / steps != s || steps < min_steps) continue;   // the same steps with fewer workgroups exist
        const int64_t cost = steps * 470 + 2000 + part_bytes * s * 450 / 1000000;
        if (cost < p.cost_ns) {
            p.cost_ns = cost;
            p.splits = (int)s;
            p.steps = (int)steps;
        }
    }
    if (p.splits > 1) p.bytes = (size_t)tiles * p.splits * (128 * 128 * 4);
    return p;
}

// 64-token tiles instead of 128-token ones in the tiled kernel: twice the workgroups, each with half of the MFMAs
// per K step for two thirds of the operand bytes.  At full load that is 15-20 % slower (measured), but while the
// 128-token tiles number 128 or fewer every workgroup still has a CU to itself, and its step takes about 370 ns
// instead of 470: used when that beats the plan above (4096 x 4096 at 256..512 rows: 19.4..21.6 against
// 23.0..25.2 us; with a long K the split wins: 11008 -> 4096 at 128 rows 22.7 against 43.1 us).
static inline bool agq_tiled_half_tiles(int64_t M, int64_t tiles_n, int64_t KT, int64_t plan_cost_ns) {
    return ((M + 127) / 128) * tiles_n <= 128 && KT * 370 < plan_cost_ns;
}

// Between 17 and 256 rows of fp16 input the weight-streaming kernel can run with sixteen rows and two channel
// tiles per workgroup (grid.y row groups): every row group reads the weights again (from L2 after the first),
// about 3 us + 0.24 us per MB read in all, more when the workgroups fill the last round of 256 CUs badly.  The
// other path is the layout pre-pass plus the tiled kernel: about 8 us around the plan's time above.  Measured
// (row groups against tiles): 4096 x 4096 at 32 / 64 / 96 / 128 rows 6.4 / 11.0 / 15.6 / 19.6 against 13.4 /
// 14.7 / 16.2 / 17.5 us; 4096 -> 11008 at 48 / 64 rows 18.3 / 21.7 against 19.8 / 19.9 us; 768 x 768 at 128
// rows 4.1 against 8.2 us.  wg_pairs: tile pairs (32 channels) of all projections; tiled_ns: the cost of the
// plan the call would run instead.  (Four tiles per workgroup instead of two were measured too: the same at best,
// and 50 % slower on the widest layer, where the registers no longer hold the weight chunks.)
#define AGQ_ROW_GROUP_MAX_M 256
static inline bool agq_decode_row_groups(int x_kind, int64_t M, int64_t K, int64_t n_sum, int64_t wg_pairs,
                                         int64_t tiled_ns) {
    if (x_kind != 0 || M <= AGQ_DECODE_MAX_M || M > AGQ_ROW_GROUP_MAX_M) return false;
    const int64_t groups = (M + 15) / 16, wgs = groups * wg_pairs;
    int64_t read_ns = groups * (K * n_sum / 2) * 240 / 1000000;
    if (wgs < 768) read_ns = read_ns * ((wgs + 255) / 256 * 256) / wgs;   // a short last round costs a whole one
    return 3000 + read_ns <= 8000 + tiled_ns;
}

int agq_launch_calibrate(const void *x, int64_t M, int64_t K, int64_t ldx, int bits, int32_t *e_dev, void *stream);
int agq_launch_quantize(const void *x, int64_t M, int64_t K, int64_t ldx, int bits, int e, int zp,
                        void *out, int64_t ld_out_bytes, int out_bits, void *stream);
int agq_launch_prepack_act(const void *x, int x_kind, int bits, int64_t M, int64_t K, int64_t ldx, int e, int zp,
                           void *out, void *stream);
int agq_launch_pack(const int8_t *wq, int64_t N, int64_t K, void *packed, int32_t *bad, void *stream);
int agq_launch_unpack(const void *packed, int64_t N, int64_t K, int8_t *wq, void *stream);
struct agq_proj;
// The linear layer behind every agq_gemm_w4a* call of the public header (argument checks, choice of kernel,
// launches); returns an agq_status.  check_only: the host-side argument checks alone.
int agq_gemm_w4_run(int bits, const void *x, int x_kind, int64_t M, int64_t K, int64_t ldx, int e, int zp,
                    const struct agq_proj *projs, int count, void *workspace, size_t workspace_bytes, void *stream,
                    bool check_only);
// n_extra >= 0 with TRIP blobs (all packed with the same factors, fp16 input); -1 for plain blobs
int agq_launch_gemm_decode(const void *x, int x_kind, int bits, int64_t M, int64_t K, int64_t ldx, int e, int zp,
                           const struct agq_proj *projs, int count, int n_extra, void *stream);
// K counts the main chunks only; with TRIP blobs (all packed with the same factors) x_tiles and the blobs hold
// n_extra more steps in front.  The `count` projections of the activation run as one launch.
// split_ws != NULL: room for the partial tiles agq_tiled_split_plan describes for this call's tiles (the call
// is split).  half_tiles: 64-token tiles (never together with split_ws).
int agq_launch_gemm_tiled(const void *x_tiles, int64_t M, int64_t K, int e, int corr, const struct agq_proj *projs, int count,
                          int n_extra, void *split_ws, bool half_tiles, void *stream);
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
