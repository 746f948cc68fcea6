// One block of the quantized pipeline (Section 4.2, Figure 3) with token pruning
// after attention (Section 4.3) and the schedule of Eq.9: host-side sequencing of
// the library's own entry points and of the fp16 operators of agq_block.hip.
#include <math.h>

#include "../../include/agq.h"
#include "agq_internal.h"

namespace {

inline bool aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15) == 0; }
inline size_t up256(size_t v) { return (v + 255) & ~(size_t)255; }
constexpr int64_t kMaxTokens = 8192;        // agq_prune_tokens' limit (calls that prune)
constexpr int64_t kMaxAttnTokens = 32768;   // the attention call's limit (calls that keep every token)
constexpr int64_t kMaxWidth = 65536;   // the GEMMs' limit on K
constexpr int64_t kMaxTripWidth = 32768;   // and with TRIP blobs

bool dims_ok(const agq_block *b) {
    if (!b || b->H < 1 || b->d < 128 || b->d > kMaxWidth || b->F < 128 || b->F > kMaxWidth) return false;
    if ((b->d % 128) != 0 || (b->F % 128) != 0 || (b->d % b->H) != 0) return false;
    const int64_t D = b->d / b->H;
    if (D != 64 && D != 128) return false;
    if (b->H > 127) return false;   // the importance score sums H terms of 2^qmax in int32 with room to spare
    if (b->qmax != 15 && b->qmax != 7) return false;
    if (b->bits_attn_out != 4 && b->bits_attn_out != 8) return false;
    const int trips[4] = {b->trip_attn_in, b->trip_attn_out, b->trip_mlp_in, b->trip_mlp_act};
    for (int t : trips) {
        if (t < -1 || t > AGQ_TRIP_MAX_EXTRA) return false;
        if (t >= 0 && (b->d > kMaxTripWidth || b->F > kMaxTripWidth)) return false;
    }
    return b->rms_eps >= 0.0 && b->rms_eps == b->rms_eps;
}

// scratch of the projections that read an activation [M,K] (plain or TRIP blobs)
size_t site_ws(int64_t M, int64_t N, int64_t K, int n_extra) {
    return n_extra >= 0 ? agq_gemm_trip_workspace_bytes(M, N, K, n_extra) : agq_gemm_workspace_bytes(M, N, K);
}

int layout_of(const agq_block *b, int64_t S, int64_t n_keep, agq_block_layout *L) {
    if (!dims_ok(b) || !L || S < 1 || n_keep < 1 || n_keep > S) return AGQ_EINVAL;
    if (S > (n_keep < S ? kMaxTokens : kMaxAttnTokens)) return AGQ_EINVAL;
    const size_t d = (size_t)b->d, F = (size_t)b->F, s = (size_t)S, k = (size_t)n_keep;
    const size_t sp = (s + 127) / 128 * 128;
    L->S_pad = (int64_t)sp;
    size_t off = 0;
    auto take = [&off](size_t bytes) { const size_t at = off; off += up256(bytes); return at; };
    L->h1 = take(s * d * 2);
    L->q = take(s * d * 2);
    L->k = take(s * d * 2);
    L->v = take(s * d * 2);
    L->q_q = take(sp * d);
    L->k_q = take(sp * d);
    L->v_q = take(sp * d);
    L->o = take(sp * d * 2);
    L->score = take(sp * 4);
    L->idx = take(k * 4);
    L->o_kept = n_keep == S ? L->o : take(k * d * 2);
    L->attn_out = take(k * d * 2);
    L->x1 = take(k * d * 2);
    L->h2 = take(k * d * 2);
    L->gate = take(k * F * 2);
    L->up = take(k * F * 2);
    L->act = take(k * F * 2);
    L->down = take(k * d * 2);
    L->q_rot = take(s * d * 2);
    L->k_rot = take(s * d * 2);
    // N: the widths of the projections of one call added up (q, k, v; gate, up)
    const size_t need[4] = {site_ws(S, 3 * b->d, b->d, b->trip_attn_in), site_ws(n_keep, b->d, b->d, b->trip_attn_out),
                            site_ws(n_keep, 2 * b->F, b->d, b->trip_mlp_in), site_ws(n_keep, b->d, b->F, b->trip_mlp_act)};
    size_t ws = 0;
    for (size_t n : need) ws = ws > n ? ws : n;
    L->gemm_ws = take(ws + 16);   // a few words behind the GEMM scratch hold calibration results
    L->total = off;
    return AGQ_OK;
}

#define AGQ_TRY(call)                    \
    do {                                 \
        const int st_ = (call);          \
        if (st_ != AGQ_OK) return st_;   \
    } while (0)
#define AGQ_TRY_HIP(call)                \
    do {                                 \
        if ((call) != 0) return AGQ_EHIP; \
    } while (0)

// The projections `projs` of one activation x [M,K] (fp16, contiguous) through the multi-projection calls: one
// quantizer pass and one launch, with plain blobs or with TRIP blobs packed with the same factors.
int site_gemm(int bits, const void *x, int64_t M, int64_t K, int e, int n_extra, const agq_proj *projs, int count, void *gws,
              size_t gws_bytes, void *stream) {
    if (n_extra < 0)
        return bits == 8 ? agq_gemm_w4a8_multi(x, AGQ_X_F16, M, K, K, e, 0, projs, count, gws, gws_bytes, stream)
                         : agq_gemm_w4a4_multi(x, AGQ_X_F16, M, K, K, e, 0, projs, count, gws, gws_bytes, stream);
    return bits == 8 ? agq_gemm_w4a8_trip_multi(x, M, K, K, e, 0, projs, count, n_extra, gws, gws_bytes, stream)
                     : agq_gemm_w4a4_trip_multi(x, M, K, K, e, 0, projs, count, n_extra, gws, gws_bytes, stream);
}

// exps: the exponents to use, updated in place when `calibrate` is set
int run(const agq_block *b, int *exps, bool calibrate, const void *x, const int32_t *pos, const float *cos_t,
        const float *sin_t, int64_t P, int64_t S, int64_t n_keep, void *x_out, int32_t *pos_out, void *workspace,
        size_t workspace_bytes, void *stream) {
    agq_block_layout L;
    AGQ_TRY(layout_of(b, S, n_keep, &L));
    if (!x || !pos || !cos_t || !sin_t || !x_out || !workspace || P < 1 || P > ((int64_t)1 << 30)) return AGQ_EINVAL;
    if (!aligned16(x) || !aligned16(cos_t) || !aligned16(sin_t) || !aligned16(x_out) ||
        (reinterpret_cast<uintptr_t>(workspace) & 255) != 0)
        return AGQ_EINVAL;
    const void *ptrs[] = {b->g_attn_f16, b->g_mlp_f16, b->w_q, b->w_k, b->w_v, b->w_o, b->w_gate, b->w_up, b->w_down,
                          b->s_q, b->s_k, b->s_v, b->s_o, b->s_gate, b->s_up, b->s_down};
    for (const void *p : ptrs)
        if (!p || !aligned16(p)) return AGQ_EINVAL;
    if (!calibrate)
        for (int i = 0; i < 7; ++i)
            if (exps[i] < AGQ_E_MIN || exps[i] > AGQ_E_MAX) return AGQ_EINVAL;
    if (calibrate && (b->trip_attn_in >= 0 || b->trip_attn_out >= 0 || b->trip_mlp_in >= 0 || b->trip_mlp_act >= 0))
        return AGQ_EINVAL;   // the calibration pass runs on plain blobs; factors are searched on its tensors afterwards
    if (workspace_bytes < L.total) return AGQ_ESIZE;

    char *ws = static_cast<char *>(workspace);
    auto at = [ws](size_t off) { return static_cast<void *>(ws + off); };
    const int64_t d = b->d, H = b->H, F = b->F, D = d / H;
    void *gws = at(L.gemm_ws);
    const size_t gws_bytes = L.total - L.gemm_ws - 16;
    int32_t *e_dev = reinterpret_cast<int32_t *>(ws + L.total - 16);
    enum { E_ATTN_IN, E_Q, E_K, E_V, E_ATTN_OUT, E_MLP_IN, E_MLP_ACT };
    // the exponent of quantizer `which` for the fp16 tensor t [rows, cols]
    auto exp_for = [&](int which, const void *t, int64_t rows, int64_t cols, int bits) -> int {
        if (!calibrate) return AGQ_OK;
        AGQ_TRY(agq_calibrate_act_exp(t, rows, cols, cols, bits, e_dev, stream));
        int32_t e = 0;
        AGQ_TRY_HIP(agq_read_i32(e_dev, &e, 1, stream));
        exps[which] = e < AGQ_E_MIN ? AGQ_E_MIN : e > AGQ_E_MAX ? AGQ_E_MAX : e;
        return AGQ_OK;
    };

    // attention half
    AGQ_TRY_HIP(agq_launch_rmsnorm(x, nullptr, nullptr, b->g_attn_f16, nullptr, at(L.h1), S, d, b->rms_eps, nullptr, nullptr,
                                   nullptr, stream));
    AGQ_TRY(exp_for(E_ATTN_IN, at(L.h1), S, d, 8));
    const agq_proj qkv[3] = {{b->w_q, b->s_q, d, at(L.q), d, nullptr},
                             {b->w_k, b->s_k, d, at(L.k), d, nullptr},
                             {b->w_v, b->s_v, d, at(L.v), d, nullptr}};
    AGQ_TRY(site_gemm(8, at(L.h1), S, d, exps[E_ATTN_IN], b->trip_attn_in, qkv, 3, gws, gws_bytes, stream));
    if (calibrate) {
        AGQ_TRY_HIP(agq_launch_rope(at(L.q), at(L.k), at(L.v), S, L.S_pad, H, D, pos, cos_t, sin_t, P, 0, 0, 0, nullptr,
                                    nullptr, nullptr, at(L.q_rot), at(L.k_rot), nullptr, stream));
        AGQ_TRY(exp_for(E_Q, at(L.q_rot), S, d, 8));
        AGQ_TRY(exp_for(E_K, at(L.k_rot), S, d, 8));
        AGQ_TRY(exp_for(E_V, at(L.v), S, d, 8));
    }
    int8_t *q_q = static_cast<int8_t *>(at(L.q_q)), *k_q = static_cast<int8_t *>(at(L.k_q)),
           *v_q = static_cast<int8_t *>(at(L.v_q));
    int32_t *score = static_cast<int32_t *>(at(L.score));   // accumulated by the attention call: cleared by the kernel before it
    AGQ_TRY_HIP(agq_launch_rope(at(L.q), at(L.k), at(L.v), S, L.S_pad, H, D, pos, cos_t, sin_t, P, exps[E_Q], exps[E_K],
                                exps[E_V], q_q, k_q, v_q, nullptr, nullptr, score, stream));
    AGQ_TRY(agq_qk_log2_softmax(q_q, k_q, H, L.S_pad, D, 1, b->qmax, exps[E_Q], exps[E_K], v_q, exps[E_V], at(L.o), nullptr,
                                score, stream));

    // pruning (Eq.4) and the projection after attention on the surviving rows
    int32_t *idx = static_cast<int32_t *>(at(L.idx));
    const bool pruned = n_keep < S;
    if (pruned) AGQ_TRY(agq_prune_tokens(score, S, n_keep, at(L.o), d, idx, at(L.o_kept), stream));
    AGQ_TRY(exp_for(E_ATTN_OUT, at(L.o_kept), n_keep, d, b->bits_attn_out));
    const agq_proj op = {b->w_o, b->s_o, d, at(L.attn_out), d, nullptr};
    AGQ_TRY(site_gemm(b->bits_attn_out, at(L.o_kept), n_keep, d, exps[E_ATTN_OUT], b->trip_attn_out, &op, 1, gws, gws_bytes,
                      stream));

    // MLP half: x1 = x[idx] + attn_out, h2 = RMSNorm(x1)
    AGQ_TRY_HIP(agq_launch_rmsnorm(at(L.attn_out), x, pruned ? idx : nullptr, b->g_mlp_f16, at(L.x1), at(L.h2), n_keep, d,
                                   b->rms_eps, pos, pos_out, pruned ? nullptr : idx, stream));
    AGQ_TRY(exp_for(E_MLP_IN, at(L.h2), n_keep, d, 8));
    const agq_proj gu[2] = {{b->w_gate, b->s_gate, F, at(L.gate), F, nullptr}, {b->w_up, b->s_up, F, at(L.up), F, nullptr}};
    AGQ_TRY(site_gemm(8, at(L.h2), n_keep, d, exps[E_MLP_IN], b->trip_mlp_in, gu, 2, gws, gws_bytes, stream));
    AGQ_TRY_HIP(agq_launch_swiglu(at(L.gate), at(L.up), at(L.act), n_keep * F, stream));
    AGQ_TRY(exp_for(E_MLP_ACT, at(L.act), n_keep, F, 8));
    const agq_proj dp = {b->w_down, b->s_down, d, at(L.down), d, nullptr};
    AGQ_TRY(site_gemm(8, at(L.act), n_keep, F, exps[E_MLP_ACT], b->trip_mlp_act, &dp, 1, gws, gws_bytes, stream));
    AGQ_TRY_HIP(agq_launch_add(at(L.x1), at(L.down), x_out, n_keep * d, stream));
    return AGQ_OK;
}

}  // namespace

extern "C" {

int agq_rmsnorm(const void *x_f16, const void *res_f16, const int32_t *idx, const void *g_f16, int64_t rows, int64_t d,
                double eps, void *sum_out_f16, void *y_f16, void *stream) {
    if (rows < 0 || rows > ((int64_t)1 << 30) || d < 8 || d > kMaxWidth || (d % 8) != 0) return AGQ_EINVAL;
    if (!(eps >= 0.0) || (idx && !res_f16)) return AGQ_EINVAL;
    if (rows == 0) return AGQ_OK;
    if (!x_f16 || !g_f16 || !y_f16 || (res_f16 && !sum_out_f16)) return AGQ_EINVAL;
    if (!aligned16(x_f16) || !aligned16(g_f16) || !aligned16(y_f16) || !aligned16(res_f16) || !aligned16(sum_out_f16))
        return AGQ_EINVAL;
    return agq_launch_rmsnorm(x_f16, res_f16, idx, g_f16, sum_out_f16, y_f16, rows, d, eps, nullptr, nullptr, nullptr,
                              stream) ? AGQ_EHIP : AGQ_OK;
}

int agq_rope_quantize(const void *q_f16, const void *k_f16, const void *v_f16, int64_t S, int64_t H, int64_t D,
                      const int32_t *pos, const float *rope_cos, const float *rope_sin, int64_t P, int e_q, int e_k,
                      int e_v, int64_t S_pad, int8_t *q_q, int8_t *k_q, int8_t *v_q, void *stream) {
    if (S < 0 || S_pad < S || S_pad > ((int64_t)1 << 20) || H < 1 || H > 65535 || D < 16 || D > 1024 || (D % 16) != 0)
        return AGQ_EINVAL;
    if (P < 1 || P > ((int64_t)1 << 30)) return AGQ_EINVAL;
    const int es[3] = {e_q, e_k, e_v};
    for (int e : es)
        if (e < AGQ_E_MIN || e > AGQ_E_MAX) return AGQ_EINVAL;
    if (S_pad == 0) return AGQ_OK;
    const void *ptrs[] = {q_f16, k_f16, v_f16, rope_cos, rope_sin, q_q, k_q, v_q};
    for (const void *p : ptrs)
        if (!p || !aligned16(p)) return AGQ_EINVAL;
    if (!pos) return AGQ_EINVAL;
    return agq_launch_rope(q_f16, k_f16, v_f16, S, S_pad, H, D, pos, rope_cos, rope_sin, P, e_q, e_k, e_v, q_q, k_q, v_q,
                           nullptr, nullptr, nullptr, stream) ? AGQ_EHIP : AGQ_OK;
}

static int elementwise_ok(const void *a, const void *b, const void *out, int64_t n) {
    if (n < 0 || n > ((int64_t)1 << 40) || (n % 8) != 0) return AGQ_EINVAL;
    if (n == 0) return AGQ_OK;
    if (!a || !b || !out || !aligned16(a) || !aligned16(b) || !aligned16(out)) return AGQ_EINVAL;
    return AGQ_OK;
}

int agq_swiglu(const void *gate_f16, const void *up_f16, void *out_f16, int64_t n, void *stream) {
    AGQ_TRY(elementwise_ok(gate_f16, up_f16, out_f16, n));
    return agq_launch_swiglu(gate_f16, up_f16, out_f16, n, stream) ? AGQ_EHIP : AGQ_OK;
}

int agq_residual_add(const void *a_f16, const void *b_f16, void *out_f16, int64_t n, void *stream) {
    AGQ_TRY(elementwise_ok(a_f16, b_f16, out_f16, n));
    return agq_launch_add(a_f16, b_f16, out_f16, n, stream) ? AGQ_EHIP : AGQ_OK;
}

int agq_block_layout_of(const agq_block *blk, int64_t S, int64_t n_keep, agq_block_layout *out) {
    return layout_of(blk, S, n_keep, out);
}

int agq_block_forward(const agq_block *blk, const void *x_f16, const int32_t *pos, const float *rope_cos,
                      const float *rope_sin, int64_t P, int64_t S, int64_t n_keep, void *x_out_f16, int32_t *pos_out,
                      void *workspace, size_t workspace_bytes, void *stream) {
    if (!blk) return AGQ_EINVAL;
    int exps[7] = {blk->e_attn_in, blk->e_q, blk->e_k, blk->e_v, blk->e_attn_out, blk->e_mlp_in, blk->e_mlp_act};
    return run(blk, exps, false, x_f16, pos, rope_cos, rope_sin, P, S, n_keep, x_out_f16, pos_out, workspace,
               workspace_bytes, stream);
}

int agq_block_calibrate(agq_block *blk, const void *x_f16, const int32_t *pos, const float *rope_cos,
                        const float *rope_sin, int64_t P, int64_t S, int64_t n_keep, void *x_out_f16, int32_t *pos_out,
                        void *workspace, size_t workspace_bytes, void *stream) {
    if (!blk) return AGQ_EINVAL;
    int exps[7] = {0, 0, 0, 0, 0, 0, 0};
    const int st = run(blk, exps, true, x_f16, pos, rope_cos, rope_sin, P, S, n_keep, x_out_f16, pos_out, workspace,
                       workspace_bytes, stream);
    if (st != AGQ_OK) return st;
    blk->e_attn_in = exps[0]; blk->e_q = exps[1]; blk->e_k = exps[2]; blk->e_v = exps[3];
    blk->e_attn_out = exps[4]; blk->e_mlp_in = exps[5]; blk->e_mlp_act = exps[6];
    return AGQ_OK;
}

namespace {

// layout of a stack's workspace: two token buffers and two position buffers (ping-pong between blocks), then
// the largest block workspace
struct StackLayout {
    size_t xa, xb, pa, pb, blk, total;
};

int stack_layout(const agq_block *blocks, int n_blocks, int64_t S, const int64_t *keep, StackLayout *out) {
    if (!blocks || !keep || !out || n_blocks < 1 || n_blocks > 4096 || S < 1) return AGQ_EINVAL;
    size_t blk_max = 0;
    int64_t in = S;
    for (int l = 0; l < n_blocks; ++l) {
        if (blocks[l].d != blocks[0].d) return AGQ_EINVAL;
        agq_block_layout L;
        AGQ_TRY(layout_of(&blocks[l], in, keep[l], &L));   // checks 1 <= keep[l] <= in and the block itself
        blk_max = blk_max > L.total ? blk_max : L.total;
        in = keep[l];
    }
    const size_t xbytes = up256((size_t)keep[0] * (size_t)blocks[0].d * 2), pbytes = up256((size_t)keep[0] * 4);
    out->xa = 0;
    out->xb = xbytes;
    out->pa = 2 * xbytes;
    out->pb = 2 * xbytes + pbytes;
    out->blk = 2 * xbytes + 2 * pbytes;
    out->total = out->blk + blk_max;
    return AGQ_OK;
}

}  // namespace

size_t agq_stack_workspace_bytes(const agq_block *blocks, int n_blocks, int64_t S, const int64_t *keep) {
    StackLayout L;
    return stack_layout(blocks, n_blocks, S, keep, &L) == AGQ_OK ? L.total : 0;
}

int agq_stack_forward(const agq_block *blocks, int n_blocks, const int64_t *keep, const void *x_f16, const int32_t *pos,
                      const float *rope_cos, const float *rope_sin, int64_t P, int64_t S, void *x_out_f16,
                      int32_t *pos_out, void *workspace, size_t workspace_bytes, void *stream) {
    StackLayout L;
    AGQ_TRY(stack_layout(blocks, n_blocks, S, keep, &L));
    if (!workspace || (reinterpret_cast<uintptr_t>(workspace) & 255) != 0) return AGQ_EINVAL;
    if (workspace_bytes < L.total) return AGQ_ESIZE;
    char *ws = static_cast<char *>(workspace);
    // every block is validated before the first launch: a bad descriptor must not leave half a stack enqueued
    {
        int64_t in = S;
        for (int l = 0; l < n_blocks; ++l) {
            const agq_block &b = blocks[l];
            const void *ptrs[] = {b.g_attn_f16, b.g_mlp_f16, b.w_q, b.w_k, b.w_v, b.w_o, b.w_gate, b.w_up, b.w_down,
                                  b.s_q, b.s_k, b.s_v, b.s_o, b.s_gate, b.s_up, b.s_down};
            for (const void *p : ptrs)
                if (!p || !aligned16(p)) return AGQ_EINVAL;
            const int es[7] = {b.e_attn_in, b.e_q, b.e_k, b.e_v, b.e_attn_out, b.e_mlp_in, b.e_mlp_act};
            for (int e : es)
                if (e < AGQ_E_MIN || e > AGQ_E_MAX) return AGQ_EINVAL;
            in = keep[l];
        }
        (void)in;
        if (!x_f16 || !pos || !rope_cos || !rope_sin || !x_out_f16 || P < 1 || P > ((int64_t)1 << 30)) return AGQ_EINVAL;
        if (!aligned16(x_f16) || !aligned16(rope_cos) || !aligned16(rope_sin) || !aligned16(x_out_f16)) return AGQ_EINVAL;
    }
    const void *xin = x_f16;
    const int32_t *pin = pos;
    int64_t in = S;
    for (int l = 0; l < n_blocks; ++l) {
        const bool last = l == n_blocks - 1;
        void *xo = last ? x_out_f16 : static_cast<void *>(ws + ((l & 1) ? L.xb : L.xa));
        int32_t *po = last ? pos_out : reinterpret_cast<int32_t *>(ws + ((l & 1) ? L.pb : L.pa));
        int exps[7] = {blocks[l].e_attn_in, blocks[l].e_q, blocks[l].e_k, blocks[l].e_v, blocks[l].e_attn_out,
                       blocks[l].e_mlp_in, blocks[l].e_mlp_act};
        AGQ_TRY(run(&blocks[l], exps, false, xin, pin, rope_cos, rope_sin, P, in, keep[l], xo, po, ws + L.blk,
                    L.total - L.blk, stream));
        xin = xo;
        pin = po;
        in = keep[l];
    }
    return AGQ_OK;
}

int agq_cascade_keep(int64_t S, double beta, int m, int64_t *keep_out) {
    if (S < 0 || S > ((int64_t)1 << 40) || !(beta >= 0.0) || !(beta < 1.0) || m < 1 || m > 1024 || !keep_out)
        return AGQ_EINVAL;
    const double gamma = 1.0 - pow(1.0 - beta, 1.0 / (double)m);
    int64_t keep = S;
    for (int i = 0; i < m; ++i) {
        keep -= (int64_t)floor((double)keep * gamma);
        keep_out[i] = keep;
    }
    return AGQ_OK;
}

}  // extern "C"
