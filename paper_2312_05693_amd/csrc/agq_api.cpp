// The C ABI of include/agq.h: argument checks on the host (before any HIP
// call), then dispatch to the kernel launchers.
#include "../../include/agq.h"
#include "agq_internal.h"

#define AGQ_VERSION 1

namespace {

inline bool aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15) == 0; }
inline bool bits_ok(int bits) { return bits == 4 || bits == 8; }
inline bool e_ok(int e) { return e >= AGQ_E_MIN && e <= AGQ_E_MAX; }
inline int hip_status(int err) { return err == 0 ? AGQ_OK : AGQ_EHIP; }
constexpr int64_t kMaxDim = (int64_t)1 << 30;
constexpr int64_t kMaxAttnS = 32768;   // one head of P stays below 4 GiB: 32-bit offsets inside the kernel

// int8 codes in operand order, tokens padded to the 128-row tile (a multiple of 16 KiB)
inline size_t codes_bytes(int64_t M, int64_t K) { return (size_t)((M + 127) / 128) * 128 * (size_t)K; }

}  // namespace

// The linear layer behind every agq_gemm_w4a* call.  check_only: run the argument checks (host only) and return.
int agq_gemm_w4_run(int bits, const void *x, int x_kind, int64_t M, int64_t K, int64_t ldx, int e, int zp,
                    const agq_proj *projs, int count, void *workspace, size_t workspace_bytes, void *stream,
                    bool check_only) {
    if (M < 0 || M > kMaxDim || K < 128 || K > 65536 || (K % 128) != 0) return AGQ_EINVAL;
    if (x_kind != AGQ_X_F16 && x_kind != AGQ_X_Q && x_kind != AGQ_X_F16_DOT) return AGQ_EINVAL;
    if (x_kind == AGQ_X_F16_DOT && (M > 1 || zp != 0)) return AGQ_EINVAL;   // the vector-ALU form: one row, signed grid
    if (!e_ok(e) || zp < 0 || zp > (1 << bits) - 1 || ldx < K) return AGQ_EINVAL;
    if (x_kind != AGQ_X_Q && (ldx % 8) != 0) return AGQ_EINVAL;
    if (x_kind == AGQ_X_Q && (ldx % (bits == 8 ? 16 : 32)) != 0) return AGQ_EINVAL;
    if (!projs || count < 1 || count > AGQ_MAX_PROJ) return AGQ_EINVAL;
    int64_t tiles = 0, n_sum = 0;
    for (int p = 0; p < count; ++p) {
        if (projs[p].N < 1 || projs[p].N > kMaxDim || projs[p].ldy < projs[p].N || projs[p].ldy > kMaxDim)
            return AGQ_EINVAL;
        tiles += (projs[p].N + 15) / 16;
        n_sum += projs[p].N;
    }
    if (tiles > kMaxDim) return AGQ_EINVAL;
    // the tiled kernel's grid: 128 x 128 tiles of all projections
    if (((M + 127) / 128) * ((n_sum + 127) / 128 + count) > kMaxDim) return AGQ_EINVAL;
    if (M == 0) return AGQ_OK;
    if (!x || !aligned16(x)) return AGQ_EINVAL;
    for (int p = 0; p < count; ++p) {
        if (!projs[p].w_packed || !projs[p].w_scale_f16 || !projs[p].y_f16) return AGQ_EINVAL;
        if (!aligned16(projs[p].w_packed) || !aligned16(projs[p].w_scale_f16) || !aligned16(projs[p].y_f16))
            return AGQ_EINVAL;
    }
    const size_t need = M <= AGQ_DECODE_MAX_M ? 0 : codes_bytes(M, K);
    if (need > 0) {
        if (!workspace || !aligned16(workspace)) return AGQ_EINVAL;
        if (workspace_bytes < need) return AGQ_ESIZE;
    }
    if (check_only) return AGQ_OK;
    // With few tiles and a long K the tiled kernel splits the tiles' K steps over workgroups, if the
    // caller's workspace has the room for the partial tiles behind the codes.
    int64_t tiles_n = 0, wg_pairs = 0;
    for (int p = 0; p < count; ++p) {
        tiles_n += (projs[p].N + 127) / 128;
        wg_pairs += (projs[p].N + 31) / 32;
    }
    AgqSplitPlan plan = agq_tiled_split_plan(M, tiles_n, K / 128, true);
    if (workspace_bytes < need + plan.bytes) plan = agq_tiled_split_plan(M, tiles_n, K / 128, false);
    const bool half_tiles = agq_tiled_half_tiles(M, tiles_n, K / 128, plan.cost_ns);
    const int64_t tiled_ns = half_tiles ? K / 128 * 370 : plan.cost_ns;
    if (M <= AGQ_DECODE_MAX_M || agq_decode_row_groups(x_kind, M, K, n_sum, wg_pairs, tiled_ns))
        return hip_status(agq_launch_gemm_decode(x, x_kind, bits, M, K, ldx, e, zp, projs, count, -1, stream));

    // many tokens: lay the codes out in MFMA operand order once (quantizing on the
    // way when x is fp16), then run the tiled kernel for all projections on that copy
    void *const split_ws = plan.splits > 1 && !half_tiles ? static_cast<char *>(workspace) + codes_bytes(M, K) : nullptr;
    if (agq_launch_prepack_act(x, x_kind, bits, M, K, ldx, e, zp, workspace, stream)) return AGQ_EHIP;
    return hip_status(
        agq_launch_gemm_tiled(workspace, M, K, e, agq_zp_corr(bits, zp), projs, count, -1, split_ws, half_tiles, stream));
}

namespace {

int gemm_w4_multi(int bits, const void *x, int x_kind, int64_t M, int64_t K, int64_t ldx, int e, int zp,
                  const agq_proj *projs, int count, void *workspace, size_t workspace_bytes, void *stream) {
    return agq_gemm_w4_run(bits, x, x_kind, M, K, ldx, e, zp, projs, count, workspace, workspace_bytes, stream, false);
}

int gemm_w4(int bits, const void *x, int x_kind, int64_t M, int64_t K, int64_t ldx, int e, int zp,
            const void *w_packed, const void *sw, int64_t N, void *y, int64_t ldy, int32_t *acc_out,
            void *workspace, size_t workspace_bytes, void *stream) {
    const agq_proj one = {w_packed, sw, N, y, ldy, acc_out};
    return gemm_w4_multi(bits, x, x_kind, M, K, ldx, e, zp, &one, 1, workspace, workspace_bytes, stream);
}

constexpr int64_t kTripMaxK = 32768;   // extra chunks included, every partial sum stays inside int32

inline bool trip_dims_ok(int64_t N, int64_t K, int n_extra) {
    return N >= 1 && N <= kMaxDim && K >= 128 && K <= kTripMaxK && (K % 128) == 0 && n_extra >= 0 &&
           n_extra <= AGQ_TRIP_MAX_EXTRA;
}

// The TRIP layer for `count` projections of one activation (their blobs packed with the same factors): one
// gathered pre-pass and one launch.
int gemm_w4_trip_multi(int bits, const void *x, int64_t M, int64_t K, int64_t ldx, int e, int zp, const agq_proj *projs,
                       int count, int n_extra, void *workspace, size_t workspace_bytes, void *stream) {
    if (!projs || count < 1 || count > AGQ_MAX_PROJ) return AGQ_EINVAL;
    int64_t n_sum = 0;
    for (int p = 0; p < count; ++p) {
        if (M < 0 || M > kMaxDim || !trip_dims_ok(projs[p].N, K, n_extra)) return AGQ_EINVAL;
        if (projs[p].ldy < projs[p].N || projs[p].ldy > kMaxDim) return AGQ_EINVAL;
        n_sum += projs[p].N;
    }
    if (!e_ok(e) || zp < 0 || zp > (1 << bits) - 1 || ldx < K || (ldx % 8) != 0) return AGQ_EINVAL;
    if (((M + 127) / 128) * ((n_sum + 127) / 128 + count) > kMaxDim) return AGQ_EINVAL;
    if (M == 0) return AGQ_OK;
    if (!x || !aligned16(x)) return AGQ_EINVAL;
    for (int p = 0; p < count; ++p) {
        if (!projs[p].w_packed || !projs[p].w_scale_f16 || !projs[p].y_f16) return AGQ_EINVAL;
        if (!aligned16(projs[p].w_packed) || !aligned16(projs[p].w_scale_f16) || !aligned16(projs[p].y_f16))
            return AGQ_EINVAL;
    }
    const size_t need = M <= AGQ_DECODE_MAX_M ? 0 : codes_bytes(M, K + 128 * (int64_t)n_extra);
    if (need > 0) {
        if (!workspace || !aligned16(workspace)) return AGQ_EINVAL;
        if (workspace_bytes < need) return AGQ_ESIZE;
    }
    if (M <= AGQ_DECODE_MAX_M)
        return hip_status(agq_launch_gemm_decode(x, AGQ_X_F16, bits, M, K, ldx, e, zp, projs, count, n_extra, stream));
    if (agq_launch_prepack_trip(x, bits, M, K, ldx, e, zp, projs[0].w_packed, projs[0].N, n_extra, workspace, stream))
        return AGQ_EHIP;
    // few tiles and a long K: K split over workgroups when the workspace has the room (as for plain blobs)
    int64_t tiles_n = 0;
    for (int p = 0; p < count; ++p) tiles_n += (projs[p].N + 127) / 128;
    AgqSplitPlan plan = agq_tiled_split_plan(M, tiles_n, K / 128 + n_extra, true, n_extra);
    if (workspace_bytes < need + plan.bytes) plan = agq_tiled_split_plan(M, tiles_n, K / 128 + n_extra, false);
    const bool half_tiles = agq_tiled_half_tiles(M, tiles_n, K / 128 + n_extra, plan.cost_ns);
    void *const split_ws = plan.splits > 1 && !half_tiles ? static_cast<char *>(workspace) + need : nullptr;
    return hip_status(agq_launch_gemm_tiled(workspace, M, K, e, agq_zp_corr(bits, zp), projs, count, n_extra, split_ws,
                                            half_tiles, stream));
}

int gemm_w4_trip(int bits, const void *x, int64_t M, int64_t K, int64_t ldx, int e, int zp, const void *w_packed,
                 int n_extra, const void *sw, int64_t N, void *y, int64_t ldy, int32_t *acc_out, void *workspace,
                 size_t workspace_bytes, void *stream) {
    const agq_proj one = {w_packed, sw, N, y, ldy, acc_out};
    return gemm_w4_trip_multi(bits, x, M, K, ldx, e, zp, &one, 1, n_extra, workspace, workspace_bytes, stream);
}

}  // namespace

extern "C" {

const char *agq_status_string(int status) {
    switch (status) {
        case AGQ_OK: return "ok";
        case AGQ_EINVAL: return "invalid argument";
        case AGQ_ESIZE: return "workspace too small";
        case AGQ_EHIP: return "HIP launch failed";
        case AGQ_ETIMEOUT: return "a wait inside the kernel timed out";
        default: return "unknown status";
    }
}

int agq_version(void) { return AGQ_VERSION; }

int agq_calibrate_act_exp(const void *x_f16, int64_t M, int64_t K, int64_t ldx, int bits, int32_t *e_dev,
                          void *stream) {
    if (M < 0 || K < 0 || M > kMaxDim || K > kMaxDim || !bits_ok(bits) || !e_dev) return AGQ_EINVAL;
    if ((K % 8) != 0 || ldx < K || (ldx % 8) != 0) return AGQ_EINVAL;
    if (M * K > 0 && (!x_f16 || !aligned16(x_f16))) return AGQ_EINVAL;
    return hip_status(agq_launch_calibrate(x_f16, M, K, ldx, bits, e_dev, stream));
}

int agq_quantize_act(const void *x_f16, int64_t M, int64_t K, int64_t ldx, int bits, int e, int zp, void *xq_out,
                     void *stream) {
    if (M < 0 || K < 0 || M > kMaxDim || K > kMaxDim || !bits_ok(bits) || !e_ok(e)) return AGQ_EINVAL;
    if (zp < 0 || zp > (1 << bits) - 1) return AGQ_EINVAL;
    if ((K % 8) != 0 || ldx < K || (ldx % 8) != 0) return AGQ_EINVAL;
    if (M * K == 0) return AGQ_OK;
    if (!x_f16 || !xq_out || !aligned16(x_f16) || !aligned16(xq_out)) return AGQ_EINVAL;
    const int64_t ld_out = bits == 8 ? K : K / 2;
    return hip_status(agq_launch_quantize(x_f16, M, K, ldx, bits, e, zp, xq_out, ld_out, bits, stream));
}

size_t agq_pack_w4_bytes(int64_t N, int64_t K) {
    if (N < 1 || N > kMaxDim || K < 128 || K > 65536 || (K % 128) != 0) return 0;
    return agq_blob_nibble_bytes(N, K) + (size_t)agq_n_tiles_padded(N) * 16 * sizeof(int32_t);
}

int agq_pack_w4(const int8_t *wq, int64_t N, int64_t K, void *packed, int32_t *bad_count_dev, void *stream) {
    if (agq_pack_w4_bytes(N, K) == 0 || !wq || !packed) return AGQ_EINVAL;
    if (!aligned16(wq) || !aligned16(packed)) return AGQ_EINVAL;
    return hip_status(agq_launch_pack(wq, N, K, packed, bad_count_dev, stream));
}

int agq_unpack_w4(const void *packed, int64_t N, int64_t K, int8_t *wq_out, void *stream) {
    if (agq_pack_w4_bytes(N, K) == 0 || !wq_out || !packed) return AGQ_EINVAL;
    if (!aligned16(wq_out) || !aligned16(packed)) return AGQ_EINVAL;
    return hip_status(agq_launch_unpack(packed, N, K, wq_out, stream));
}

size_t agq_gemm_workspace_bytes(int64_t M, int64_t N, int64_t K) {
    if (M <= AGQ_DECODE_MAX_M || K < 1) return 0;
    // the codes, plus the partial tiles of a K split when the call has few tiles (+ 3: a call with up to
    // four projections whose widths add up to N has at most three more column tiles than one of width N)
    const int64_t tiles_n = N > 0 ? (N + 127) / 128 : 0;
    size_t split = 0;
    for (int64_t t = tiles_n; t <= tiles_n + 3 && t > 0; ++t) {
        const AgqSplitPlan plan = agq_tiled_split_plan(M, t, K / 128, true);
        if (plan.bytes > split) split = plan.bytes;
    }
    return codes_bytes(M, K) + split;
}

int agq_trip_search(const void *x_f16, int64_t M, int64_t K, int64_t ldx, int bits, int e, int zp, int kmax,
                    int8_t *alpha_dev, void *stream) {
    if (M < 0 || K < 0 || M > kMaxDim || K > kMaxDim || !bits_ok(bits)) return AGQ_EINVAL;
    if (kmax < 0 || kmax > AGQ_TRIP_MAX_FACTOR || e < AGQ_E_MIN || e + kmax > AGQ_E_MAX) return AGQ_EINVAL;
    if (zp < 0 || zp > (1 << bits) - 1 || ldx < K) return AGQ_EINVAL;
    if (K == 0) return AGQ_OK;
    if (!alpha_dev || (M > 0 && !x_f16)) return AGQ_EINVAL;
    return hip_status(agq_launch_trip_search(x_f16, M, K, ldx, bits, e, zp, kmax, alpha_dev, stream));
}

int agq_trip_extra_chunks(const int8_t *alpha_host, int64_t K) {
    if (!alpha_host || K < 128 || K > kTripMaxK || (K % 128) != 0) return AGQ_EINVAL;
    const int E = agq_trip_count_extra(alpha_host, K);
    return E < 0 ? AGQ_EINVAL : E;
}

size_t agq_pack_w4_trip_bytes(int64_t N, int64_t K, int n_extra) {
    if (!trip_dims_ok(N, K, n_extra)) return 0;
    return agq_trip_layout(N, K, n_extra).total;
}

int agq_pack_w4_trip(const int8_t *wq, int64_t N, int64_t K, const int8_t *alpha_host, void *packed,
                     int32_t *bad_count_dev, void *stream) {
    if (!alpha_host || !wq || !packed || !aligned16(wq) || !aligned16(packed)) return AGQ_EINVAL;
    if (!trip_dims_ok(N, K, 0) || agq_trip_count_extra(alpha_host, K) < 0) return AGQ_EINVAL;
    return hip_status(agq_launch_pack_trip(wq, N, K, alpha_host, packed, bad_count_dev, stream));
}

int agq_unpack_w4_trip(const void *packed, int64_t N, int64_t K, int n_extra, int8_t *wq_out, void *stream) {
    if (!trip_dims_ok(N, K, n_extra) || !wq_out || !packed) return AGQ_EINVAL;
    if (!aligned16(wq_out) || !aligned16(packed)) return AGQ_EINVAL;
    return hip_status(agq_launch_unpack_trip(packed, N, K, n_extra, wq_out, stream));
}

size_t agq_gemm_trip_workspace_bytes(int64_t M, int64_t N, int64_t K, int n_extra) {
    if (M <= AGQ_DECODE_MAX_M || K < 1 || n_extra < 0) return 0;
    const int64_t tiles_n = N > 0 ? (N + 127) / 128 : 0;
    size_t split = 0;
    for (int64_t t = tiles_n; t <= tiles_n + 3 && t > 0; ++t) {
        const AgqSplitPlan plan = agq_tiled_split_plan(M, t, K / 128 + n_extra, true, n_extra);
        if (plan.bytes > split) split = plan.bytes;
    }
    return codes_bytes(M, K + 128 * (int64_t)n_extra) + split;
}

int agq_gemm_w4a8_trip(const void *x_f16, int64_t M, int64_t K, int64_t ldx, int e, int zp, const void *w_packed,
                       int n_extra, const void *w_scale_f16, int64_t N, void *y_f16, int64_t ldy, int32_t *acc_out,
                       void *workspace, size_t workspace_bytes, void *stream) {
    return gemm_w4_trip(8, x_f16, M, K, ldx, e, zp, w_packed, n_extra, w_scale_f16, N, y_f16, ldy, acc_out, workspace,
                        workspace_bytes, stream);
}

int agq_gemm_w4a8_trip_multi(const void *x_f16, int64_t M, int64_t K, int64_t ldx, int e, int zp, const agq_proj *projs,
                             int count, int n_extra, void *workspace, size_t workspace_bytes, void *stream) {
    return gemm_w4_trip_multi(8, x_f16, M, K, ldx, e, zp, projs, count, n_extra, workspace, workspace_bytes, stream);
}

int agq_gemm_w4a4_trip_multi(const void *x_f16, int64_t M, int64_t K, int64_t ldx, int e, int zp, const agq_proj *projs,
                             int count, int n_extra, void *workspace, size_t workspace_bytes, void *stream) {
    return gemm_w4_trip_multi(4, x_f16, M, K, ldx, e, zp, projs, count, n_extra, workspace, workspace_bytes, stream);
}

int agq_gemm_w4a4_trip(const void *x_f16, int64_t M, int64_t K, int64_t ldx, int e, int zp, const void *w_packed,
                       int n_extra, const void *w_scale_f16, int64_t N, void *y_f16, int64_t ldy, int32_t *acc_out,
                       void *workspace, size_t workspace_bytes, void *stream) {
    return gemm_w4_trip(4, x_f16, M, K, ldx, e, zp, w_packed, n_extra, w_scale_f16, N, y_f16, ldy, acc_out, workspace,
                        workspace_bytes, stream);
}

int agq_gemm_w4a8(const void *x, int x_kind, int64_t M, int64_t K, int64_t ldx, int e, int zp, const void *w_packed,
                  const void *w_scale_f16, int64_t N, void *y_f16, int64_t ldy, int32_t *acc_out, void *workspace,
                  size_t workspace_bytes, void *stream) {
    return gemm_w4(8, x, x_kind, M, K, ldx, e, zp, w_packed, w_scale_f16, N, y_f16, ldy, acc_out, workspace,
                   workspace_bytes, stream);
}

int agq_gemm_w4a4(const void *x, int x_kind, int64_t M, int64_t K, int64_t ldx, int e, int zp, const void *w_packed,
                  const void *w_scale_f16, int64_t N, void *y_f16, int64_t ldy, int32_t *acc_out, void *workspace,
                  size_t workspace_bytes, void *stream) {
    return gemm_w4(4, x, x_kind, M, K, ldx, e, zp, w_packed, w_scale_f16, N, y_f16, ldy, acc_out, workspace,
                   workspace_bytes, stream);
}

int agq_gemm_w4a8_multi(const void *x, int x_kind, int64_t M, int64_t K, int64_t ldx, int e, int zp,
                        const agq_proj *projs, int count, void *workspace, size_t workspace_bytes, void *stream) {
    return gemm_w4_multi(8, x, x_kind, M, K, ldx, e, zp, projs, count, workspace, workspace_bytes, stream);
}

int agq_gemm_w4a4_multi(const void *x, int x_kind, int64_t M, int64_t K, int64_t ldx, int e, int zp,
                        const agq_proj *projs, int count, void *workspace, size_t workspace_bytes, void *stream) {
    return gemm_w4_multi(4, x, x_kind, M, K, ldx, e, zp, projs, count, workspace, workspace_bytes, stream);
}

int agq_log2_quant_softmax(const void *p_f16, int64_t H, int64_t S, int64_t D, int causal, int qmax,
                           const int8_t *v_q, int e_v, void *o_f16, void *codes_out, int32_t *score_out,
                           void *stream) {
    if (H < 1 || H > 65535 || S < 8 || S > kMaxAttnS || (S % 8) != 0 || D < 16 || D > 256 || (D % 16) != 0)
        return AGQ_EINVAL;
    if (qmax != 15 && qmax != 7) return AGQ_EINVAL;
    if (!e_ok(e_v) || !p_f16 || !v_q || !o_f16) return AGQ_EINVAL;
    if (score_out && H > 127) return AGQ_EINVAL;
    if (!aligned16(p_f16) || !aligned16(v_q) || !aligned16(o_f16)) return AGQ_EINVAL;
    if (codes_out && !aligned16(codes_out)) return AGQ_EINVAL;
    return hip_status(agq_launch_log2_attn(p_f16, H, S, D, causal != 0, qmax, v_q, e_v, o_f16, codes_out, score_out,
                                           stream));
}

int agq_qk_log2_softmax(const int8_t *q_q, const int8_t *k_q, int64_t H, int64_t S, int64_t D, int causal, int qmax,
                        int e_q, int e_k, const int8_t *v_q, int e_v, void *o_f16, void *codes_out, int32_t *score_out,
                        void *stream) {
    if (H < 1 || H > 65535 || S < 128 || S > kMaxAttnS || (S % 128) != 0 || (D != 64 && D != 128)) return AGQ_EINVAL;
    if (qmax != 15 && qmax != 7) return AGQ_EINVAL;
    if (!e_ok(e_q) || !e_ok(e_k) || !e_ok(e_v) || !q_q || !k_q || !v_q || !o_f16) return AGQ_EINVAL;
    if (!aligned16(q_q) || !aligned16(k_q) || !aligned16(v_q) || !aligned16(o_f16)) return AGQ_EINVAL;
    if (codes_out && !aligned16(codes_out)) return AGQ_EINVAL;
    return hip_status(agq_launch_qk_log2_attn(q_q, k_q, v_q, H, S, D, causal != 0, qmax, e_q, e_k, e_v, o_f16, codes_out,
                                              score_out, stream));
}

int agq_prune_tokens(const int32_t *score, int64_t S, int64_t n_keep, const void *x_f16, int64_t d,
                     int32_t *idx_out, void *x_out_f16, void *stream) {
    if (S < 1 || S > 8192 || n_keep < 0 || n_keep > S || d < 8 || d > kMaxDim || (d % 8) != 0) return AGQ_EINVAL;
    if (!score || !x_f16) return AGQ_EINVAL;
    if (n_keep == 0) return AGQ_OK;
    if (!idx_out || !x_out_f16 || !aligned16(x_f16) || !aligned16(x_out_f16)) return AGQ_EINVAL;
    return hip_status(agq_launch_prune(score, S, n_keep, x_f16, d, idx_out, x_out_f16, stream));
}

}  // extern "C"
