/* agq - the W4A8 / W4A4 quantized linear layer of Agile-Quant (arxiv 2312.05693)
 * and its log2-quantized softmax x V path, as HIP kernels for gfx950 (MI355X).
 *
 * C ABI.  Conventions that hold for every call unless a comment says otherwise:
 *   - every tensor pointer is a DEVICE pointer owned by the caller; the library
 *     allocates nothing and keeps no tensor state between calls.  What it does
 *     keep, per process and device, are facts looked up once: the device's number
 *     of compute units, a raised LDS limit of its own kernels, and the address of
 *     agq_gemm_w4a8_static's array.  Each is set up, thread-safely, by the first
 *     call that needs it on that device;
 *   - tensors are row-major, leading dimensions are in elements;
 *   - work is enqueued asynchronously on `stream` (a hipStream_t passed as
 *     void*, NULL = the default stream); the caller synchronises;
 *   - the return value is an agq_status: 0 on success, negative on error.
 *     Argument errors (AGQ_EINVAL, AGQ_ESIZE) are found on the host before any
 *     HIP call is made; AGQ_EHIP reports a failed launch.  Nothing is printed,
 *     thrown or aborted;
 *   - fp16 inputs must not hold NaN (a NaN yields an unspecified code inside
 *     the grid); +-Inf saturate.
 */
#ifndef AGQ_H
#define AGQ_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

enum agq_status {
    AGQ_OK = 0,
    AGQ_EINVAL = -1, /* bad argument (null pointer, size, granularity, range) */
    AGQ_ESIZE = -2,  /* workspace too small                                    */
    AGQ_EHIP = -3,   /* the HIP runtime refused a launch                       */
    AGQ_ETIMEOUT = -4 /* agq_gemm_chain_status: a wait inside a chain launch ran
                         out of time (see there)                                */
};

/* what `x` of the GEMM calls holds */
enum agq_x_kind {
    AGQ_X_F16 = 0, /* fp16 [M,K]; Eq.2 is applied inside the call            */
    AGQ_X_Q = 1,   /* codes written by agq_quantize_act with the same
                      bits / e / zp: int8 [M,K] (8 bit) or nibbles [M,K/2]   */
    AGQ_X_F16_DOT = 2 /* as AGQ_X_F16, for M == 1 and zp == 0 only: the product runs
                      on the vector ALU (v_dot4_i32_i8 / v_dot8_i32_i4, the
                      chip's counterpart of the paper's 4-bit multiplier,
                      Section 4.4 and the appendix) with Eq.2 applied in
                      registers, no LDS staging and no matrix core.  Same
                      results bit for bit; which form is faster is a
                      measurement (the library itself never picks this one).
                      Not accepted by the _trip and chain calls.             */
};

/* range of the activation exponent e (scale s = 2^e) accepted everywhere */
#define AGQ_E_MIN (-40)
#define AGQ_E_MAX 40

const char *agq_status_string(int status);
int agq_version(void);

/* Layer-wise power-of-two activation scale (Section 4.4: all channels share one
 * set of quantization parameters; the scale is read as a power of two).
 * Writes to *e_dev (device int32) the smallest e with max|x| <= qmax * 2^e,
 * qmax = 2^(bits-1)-1; 0 for an all-zero tensor; +-Inf/NaN count as 2^16.
 * x_f16: fp16 [M,K], ldx >= K.  bits in {4,8}.  M*K may be 0 (e = 0).        */
int agq_calibrate_act_exp(const void *x_f16, int64_t M, int64_t K, int64_t ldx,
                          int bits, int32_t *e_dev, void *stream);

/* Uniform quantizer, Section 4.1 Eq.2, with s = 2^e and round-half-to-even:
 *   q = CLIP(round(x / 2^e) + zp, lo, hi)
 * zp == 0 selects the signed grid of Eq.1, [-2^(b-1), 2^(b-1)-1]; zp > 0 the
 * unsigned grid [0, 2^b-1] of Eq.2 as printed.  bits in {4,8}.
 * x_f16 : fp16 [M,K], ldx >= K, ldx % 8 == 0, 16-byte aligned; K % 8 == 0.
 * xq_out: bits=8: one byte per code, [M,K] contiguous (int8, or uint8 if zp>0);
 *         bits=4: two codes per byte, [M,K/2] contiguous, low nibble = even k,
 *         signed codes in two's complement.
 * M == 0 is a no-op.                                                          */
int agq_quantize_act(const void *x_f16, int64_t M, int64_t K, int64_t ldx,
                     int bits, int e, int zp, void *xq_out, void *stream);

/* 4-bit weight storage (Section 4.4 stores two 4-bit weights per byte).  The
 * order of nibbles inside `packed` is private to the library: it is laid out
 * for 64-lane coalesced loads and the int8 MFMA operand order, followed by the
 * sum of each output channel's weights (used by the unsigned activation grid).
 * Only agq_unpack_w4(agq_pack_w4(W)) == W is contractual.
 * wq     : int8 [N,K], K contiguous, values in [-8,7]; K % 128 == 0, N >= 1.
 *          Values outside [-8,7] are saturated and counted into *bad_count_dev
 *          (device int32, may be NULL; the caller zeroes it and reads it after
 *          synchronising).
 * packed : agq_pack_w4_bytes(N,K) bytes, 16-byte aligned (0 = invalid N,K).   */
size_t agq_pack_w4_bytes(int64_t N, int64_t K);
int agq_pack_w4(const int8_t *wq, int64_t N, int64_t K, void *packed,
                int32_t *bad_count_dev, void *stream);
int agq_unpack_w4(const void *packed, int64_t N, int64_t K, int8_t *wq_out,
                  void *stream);

/* The quantized linear layer (Sections 4.2 and 4.4): the activation on the
 * b-bit grid of Eq.2 with the layer-wise scale 2^e, times the 4-bit weights,
 * accumulated in int32, dequantized per output channel:
 *   acc[m,n] = sum_k (q[m,k] - zp) * Wq[n,k]       (int32, exact)
 *   y[m,n]   = fp16( float(acc[m,n]) * (2^e * sw[n]) )
 * agq_gemm_w4a8 uses b = 8, agq_gemm_w4a4 b = 4 (codes widened to int8 for the
 * MFMA; CDNA4 has no 4-bit matrix instruction).
 * x        : see agq_x_kind.  fp16: ldx % 8 == 0; codes: ldx in code units,
 *            ldx % 16 == 0 (8 bit) or ldx % 32 == 0 (4 bit); 16-byte aligned.
 *            w_packed, w_scale_f16 and y_f16 are 16-byte aligned too.
 * zp       : 0 = the signed grid of Eq.1 (the measured configuration); 1 .. 2^b-1 =
 *            the unsigned grid of Eq.2 with that zero point.  Inside the kernels
 *            the unsigned code travels as q - 2^(b-1), which the int8 matrix
 *            instruction takes, and sum_k (q - zp) w = sum_k (q - 2^(b-1)) w +
 *            (2^(b-1) - zp) * sum_k w, the last sum precomputed by agq_pack_w4.
 * w_packed : output of agq_pack_w4 for [N,K].   w_scale_f16: fp16 [N].
 * y_f16    : fp16 [M,N], ldy >= N.   acc_out: optional int32 [M,N] contiguous
 *            copy of the accumulators (NULL to skip).
 * workspace: agq_gemm_workspace_bytes(M,N,K) bytes, 16-byte aligned, may be
 *            NULL when that is 0.  Holds the quantized activation when M is
 *            large enough for the tiled kernel, and behind it, when the call
 *            has few output tiles and a long K, the int32 partial tiles of a
 *            split of K over workgroups; contents are scratch.  A workspace of
 *            agq_gemm_workspace_bytes(M,0,K) bytes (the activation only) is
 *            accepted too: K is then not split, which costs time where it
 *            applies and changes no result; a smaller one is AGQ_ESIZE.
 * K % 128 == 0, K <= 65536 (keeps every partial sum inside int32), M >= 0.
 * Which kernel runs is the library's choice and does not change a result: up to 16
 * rows the weight-streaming kernel; 17..256 rows of fp16 input the same kernel with
 * sixteen rows (and two channel tiles) per workgroup while re-reading the weights per row group is cheaper
 * than the tiled path (a measured rule on the sizes); else the layout pre-pass and
 * the tiled kernel; while the call has at most 128 tiles of 128 x 128 either with K
 * split over workgroups (a long K, and the workspace has the room) or with 64-token
 * tiles, whichever a measured cost model puts first.
 * Graph capture: the calls enqueue kernels only and may be captured.  (The first
 * weight-streaming call on a device also raises the LDS limit of the library's
 * kernels there: a host-side setting, not a stream operation, made once per
 * device whatever the shape of that first call.)                              */
size_t agq_gemm_workspace_bytes(int64_t M, int64_t N, int64_t K);
int agq_gemm_w4a8(const void *x, int x_kind, int64_t M, int64_t K, int64_t ldx,
                  int e, int zp, const void *w_packed, const void *w_scale_f16,
                  int64_t N, void *y_f16, int64_t ldy, int32_t *acc_out,
                  void *workspace, size_t workspace_bytes, void *stream);
int agq_gemm_w4a4(const void *x, int x_kind, int64_t M, int64_t K, int64_t ldx,
                  int e, int zp, const void *w_packed, const void *w_scale_f16,
                  int64_t N, void *y_f16, int64_t ldy, int32_t *acc_out,
                  void *workspace, size_t workspace_bytes, void *stream);

/* For callers that cannot allocate device memory (code under HIP graph capture,
 * tight serving loops, harnesses that forbid hipMalloc): agq_gemm_w4a8 without the
 * workspace arguments.  The quantized activation of the tiled path, and the partial
 * tiles of a K split behind it, live in a fixed array of
 * AGQ_STATIC_WORKSPACE_BYTES inside the library's device image (one copy on every
 * GPU the library is used on, held until the process ends); the call makes no
 * hipMalloc / hipFree and calls no allocating routine.  The array's address is
 * looked up once per device, on the first call made with that device current.
 * Same arguments, checks, kernels and results as agq_gemm_w4a8.  A call whose
 * activation codes alone (M rounded up to 128, times K bytes; nothing for M <= 16)
 * exceed the array returns AGQ_ESIZE before any HIP call; every configuration up
 * to 2048 x 11008 fits.  When the codes fit but the partial tiles do not, K is
 * not split (slower for few output tiles, same result).
 * All calls on one GPU share the array: two calls that overlap in time on one GPU
 * (different streams or threads) race and give wrong results; calls on one stream
 * are safe.  Nothing in the array needs clearing between calls.                */
#define AGQ_STATIC_WORKSPACE_BYTES ((size_t)32 << 20)
int agq_gemm_w4a8_static(const void *x, int x_kind, int64_t M, int64_t K, int64_t ldx,
                         int e, int zp, const void *w_packed, const void *w_scale_f16,
                         int64_t N, void *y_f16, int64_t ldy, int32_t *acc_out,
                         void *stream);

/* Several projections of the same activation in one call (q/k/v, gate/up of a
 * transformer block; Section 4.2's pipeline quantizes such an activation once).
 * Same computation as `count` calls of agq_gemm_w4a8 / agq_gemm_w4a4 with the
 * same x, M, K, e: Eq.2 (or the layout pre-pass) runs once, and all projections
 * run as one kernel launch: what a launch-bound decode step needs, and for many
 * rows one grid over the tiles of all projections fills the chip better.  projs: HOST array of `count` descriptors (1 <= count <=
 * AGQ_MAX_PROJ), read before the call returns.  workspace:
 * agq_gemm_workspace_bytes(M, N, K) with N = the widths of the projections added
 * up (any smaller N down to 0 is accepted, see above).  Other arguments and errors as
 * for the single calls.                                                       */
#define AGQ_MAX_PROJ 4
typedef struct agq_proj {
    const void *w_packed;    /* agq_pack_w4 output for [N,K]            */
    const void *w_scale_f16; /* fp16 [N]                                */
    int64_t N;
    void *y_f16;             /* fp16 [M,N]                              */
    int64_t ldy;
    int32_t *acc_out;        /* optional int32 [M,N] contiguous, or NULL */
} agq_proj;
int agq_gemm_w4a8_multi(const void *x, int x_kind, int64_t M, int64_t K, int64_t ldx,
                        int e, int zp, const agq_proj *projs, int count,
                        void *workspace, size_t workspace_bytes, void *stream);
int agq_gemm_w4a4_multi(const void *x, int x_kind, int64_t M, int64_t K, int64_t ldx,
                        int e, int zp, const agq_proj *projs, int count,
                        void *workspace, size_t workspace_bytes, void *stream);

/* A chain of linear layers for a few tokens in ONE kernel launch: the decode
 * regime, where a step of the model is a sequence of layers that each read
 * 8-45 MB of 4-bit weights once (Section 3.3: the matrix products are the
 * workload; Section 4.4: layer-wise activation parameters, so every stage has its
 * own static exponent).  Stage s computes what agq_gemm_w4a8_multi /
 * agq_gemm_w4a4_multi computes (zp = 0, fp16 input, Eq.2 inside, per-channel
 * dequantization, fp16 outputs written to the caller's tensors), on
 *   - a caller tensor x_f16 [M,K] (ldx % 8 == 0, 16-byte aligned), or
 *   - x_f16 == NULL: the fp16 output of projection `src_proj` of stage s-1, whose
 *     width must equal this stage's K (never allowed for stage 0).
 * Results are those of the single calls, bit for bit.  One persistent workgroup
 * per compute unit walks through the stages; the weights of the next stage are
 * requested while the outputs of the current one travel between the compute
 * units (through records in the workspace that carry their own epoch), which a
 * launch per layer cannot do.
 *
 * M: 1..AGQ_CHAIN_MAX_M.  Per stage: K % 128 == 0, 128 <= K <= 16384; bits 8 or 4;
 * 1 <= count <= AGQ_MAX_PROJ; every N % 16 == 0, ldy even; pointers as for
 * agq_gemm_w4a8 (acc_out, if given, 8-byte aligned).  n_stages <=
 * AGQ_CHAIN_MAX_STAGES.  stages is a HOST array.
 *
 * agq_gemm_chain_prepare: checks everything on the host, then writes the stage
 * table and zeroes the records in `workspace` (agq_gemm_chain_workspace_bytes,
 * 0 = invalid arguments; 256-byte aligned) and WAITS for `stream`: set-up work,
 * not capturable.  The pointers inside the stages are baked into the workspace.
 * agq_gemm_chain_run: enqueues the one kernel on a prepared workspace; allocates
 * nothing and may be captured and replayed any number of times.  Runs of one
 * workspace must not overlap in time, and the device must not be busy with other
 * kernels of comparable length while a chain runs: the workgroups wait for each
 * other, so all of them have to be resident at once (one per compute unit).
 * Every wait inside the kernel is bounded (20 ms): if one runs out, all workgroups
 * leave, outputs are incomplete, and the workspace is marked; later runs on it
 * return at once.  agq_gemm_chain_status waits for `stream` and returns AGQ_OK or
 * AGQ_ETIMEOUT for the runs so far; after a time-out prepare the workspace again. */
#define AGQ_CHAIN_MAX_M 4
#define AGQ_CHAIN_MAX_STAGES 1024
typedef struct agq_chain_stage {
    const void *x_f16;          /* caller input, or NULL: output of the stage before */
    int64_t ldx;                /* elements; ignored when x_f16 == NULL               */
    int src_proj;               /* which projection of stage s-1 (x_f16 == NULL)      */
    int bits;                   /* activation grid: 8 or 4                            */
    int e;                      /* activation scale 2^e of this stage                 */
    int64_t K;
    int count;
    agq_proj projs[AGQ_MAX_PROJ];
} agq_chain_stage;
size_t agq_gemm_chain_workspace_bytes(const agq_chain_stage *stages, int n_stages, int64_t M);
int agq_gemm_chain_prepare(const agq_chain_stage *stages, int n_stages, int64_t M,
                           void *workspace, size_t workspace_bytes, void *stream);
int agq_gemm_chain_run(void *workspace, void *stream);
int agq_gemm_chain_status(const void *workspace, void *stream);

/* TRIP: per-channel power-of-two factors on top of the layer-wise step
 * (Section 4.3, Eq.5-8) and the matrix product that carries them on the weight
 * rows (Section 4.4, "efficient TRIP matrix multiplication").
 *
 * Eq.5 quantizes input channel k with the step 2^(e + alpha[k]), alpha[k] in
 * 0..AGQ_TRIP_MAX_FACTOR, grid and rounding as in Eq.2:
 *   q[m,k]   = CLIP(round(x[m,k] / 2^(e + alpha[k])) + zp, lo, hi)
 *   acc[m,n] = sum_k (q[m,k] - zp) * 2^alpha[k] * Wq[n,k]      (int32, exact)
 *   y[m,n]   = fp16( float(acc[m,n]) * (2^e * sw[n]) )
 * e is the base (finest) step: Eq.6 is read as the layer-wise step divided by
 * 2^kmax, i.e. e = agq_calibrate_act_exp's result minus kmax.
 *
 * agq_trip_search (Eq.8): alpha[k] = the factor in 0..kmax with the smallest
 * squared error || x[:,k] - dequant(quant(x[:,k])) ||^2 over the M tokens, the
 * quantizer being Eq.5 with its clip; equal errors give the smaller factor.
 * Errors are summed in float64 in token order, so the result is reproducible
 * bit for bit.  x_f16: fp16 [M,K], ldx >= K; alpha_dev: device int8 [K].
 * M == 0 gives all zeros.  A calibration-time call, not tuned for speed.
 *
 * The weight blob for a set of factors: channels with alpha > 0 are served by
 * extra 128-wide chunks (at most AGQ_TRIP_MAX_EXTRA of them, each holding
 * channels of one factor), the other channels by the ordinary chunks.
 * alpha_host is a HOST array int8 [K] (copy agq_trip_search's result back: packing
 * is set-up work).  agq_trip_extra_chunks returns the number of extra chunks
 * (>= 0) these factors need, or AGQ_EINVAL (a factor outside 0..4, more chunks
 * than the maximum, bad K).  agq_pack_w4_trip_bytes(N, K, n_extra) is the blob
 * size (0 = invalid arguments).  agq_pack_w4_trip copies small tables to the
 * device and WAITS for `stream` before it launches its kernels (not capturable).
 * agq_unpack_w4_trip(agq_pack_w4_trip(W)) == W (after saturation to [-8,7]).
 * K % 128 == 0, K <= 32768 (keeps every partial sum inside int32).
 *
 * agq_gemm_w4a8_trip / agq_gemm_w4a4_trip: the layer above with b = 8 / 4.
 * x_f16 is fp16 [M,K] (ldx % 8 == 0, 16-byte aligned): the quantizer runs inside
 * the call.  n_extra: as returned by agq_trip_extra_chunks for the factors the
 * blob was packed with.  workspace: agq_gemm_trip_workspace_bytes(M,N,K,n_extra)
 * (with N = 0: the activation alone, accepted too, as for agq_gemm_w4a8).
 * Other arguments, alignment and errors as for agq_gemm_w4a8.                 */
#define AGQ_TRIP_MAX_FACTOR 4
#define AGQ_TRIP_MAX_EXTRA 16
int agq_trip_search(const void *x_f16, int64_t M, int64_t K, int64_t ldx, int bits,
                    int e, int zp, int kmax, int8_t *alpha_dev, void *stream);
int agq_trip_extra_chunks(const int8_t *alpha_host, int64_t K);
size_t agq_pack_w4_trip_bytes(int64_t N, int64_t K, int n_extra);
int agq_pack_w4_trip(const int8_t *wq, int64_t N, int64_t K, const int8_t *alpha_host,
                     void *packed, int32_t *bad_count_dev, void *stream);
int agq_unpack_w4_trip(const void *packed, int64_t N, int64_t K, int n_extra,
                       int8_t *wq_out, void *stream);
size_t agq_gemm_trip_workspace_bytes(int64_t M, int64_t N, int64_t K, int n_extra);
int agq_gemm_w4a8_trip(const void *x_f16, int64_t M, int64_t K, int64_t ldx, int e, int zp,
                       const void *w_packed, int n_extra, const void *w_scale_f16,
                       int64_t N, void *y_f16, int64_t ldy, int32_t *acc_out,
                       void *workspace, size_t workspace_bytes, void *stream);
int agq_gemm_w4a4_trip(const void *x_f16, int64_t M, int64_t K, int64_t ldx, int e, int zp,
                       const void *w_packed, int n_extra, const void *w_scale_f16,
                       int64_t N, void *y_f16, int64_t ldy, int32_t *acc_out,
                       void *workspace, size_t workspace_bytes, void *stream);
/* Several projections of one activation with TRIP (the factors belong to the
 * activation, so q/k/v or gate/up share them): every blob packed with the same
 * factors, n_extra theirs.  One quantize-and-gather pass, one launch.  projs as for
 * agq_gemm_w4a8_multi; workspace: agq_gemm_trip_workspace_bytes(M, N, K, n_extra)
 * with N = the widths added up.                                                  */
int agq_gemm_w4a8_trip_multi(const void *x_f16, int64_t M, int64_t K, int64_t ldx, int e, int zp,
                             const agq_proj *projs, int count, int n_extra, void *workspace,
                             size_t workspace_bytes, void *stream);
int agq_gemm_w4a4_trip_multi(const void *x_f16, int64_t M, int64_t K, int64_t ldx, int e, int zp,
                             const agq_proj *projs, int count, int n_extra, void *workspace,
                             size_t workspace_bytes, void *stream);

/* Log2 quantizer on softmax probabilities (Section 4.1 Eq.3 with max|X| = 1,
 * used for the softmax output per Section 5.1) fused with the product with the
 * int8 value matrix, plus the token importance of Section 4.3 (attention paid
 * to the first token):
 *   c[h,i,j]  = CLIP(round(-log2 p[h,i,j]), 0, qmax)            (p = 0 -> qmax)
 *   o[i,h*D+d]= fp16( 2^(e_v-qmax) * sum_j 2^(qmax-c[h,i,j]) * v_q[h,j,d] )
 *   score[i]  = sum_h p[h,i,0] * 2^24                           (exact integer)
 * p_f16   : fp16 [H,S,S] in [0,1], row i = query i; causal != 0 reads j <= i only.
 * qmax    : 15 (all four bits carry magnitude) or 7 (Eq.3's 2^(b-1)-1, b = 4).
 * v_q     : int8 [H,S,D], scale 2^e_v;  D % 16 == 0, D <= 256;  S % 8 == 0,
 *           S <= 32768.
 * o_f16   : fp16 [S, H*D].   codes_out: optional [H,S,S/2] bytes, two codes per
 *           byte, low nibble = even j, entries above the diagonal carry qmax.
 * score_out: optional int32 [S]; needs H <= 127.
 * Precondition: rows are softmax outputs (values in [0,1], sum <= ~1), which
 * keeps the integer sum below 2^24; a value above 1 gives an unspecified
 * result, and arbitrary inputs may lose low bits.                           */
int agq_log2_quant_softmax(const void *p_f16, int64_t H, int64_t S, int64_t D,
                           int causal, int qmax, const int8_t *v_q, int e_v,
                           void *o_f16, void *codes_out, int32_t *score_out,
                           void *stream);

/* Attention from quantized Q and K in one call: the integer product Q K^T
 * (Section 4.2 lists QK among the quantized products), softmax in floating point
 * (Section 3.3), Eq.3 on the probabilities, the product with the int8 value
 * matrix, and the token importance of Section 4.3 read on the quantized map.
 * The probabilities are never written to memory.
 *   s[h,i,j]  = sum_d q_q[h,i,d] * k_q[h,j,d]                    (int32, exact)
 *   p[h,i,:]  = softmax_j( s * 2^(e_q+e_k) / sqrt(D) )           (j <= i if causal)
 *   c[h,i,j]  = CLIP(round(-log2 p[h,i,j]), 0, qmax)
 *   o[i,h*D+d]= fp16( 2^(e_v-qmax) * sum_j 2^(qmax-c[h,i,j]) * v_q[h,j,d] )
 *   score[i] += sum_h 2^(qmax - c[h,i,0])
 * -log2 p is evaluated in fp32 as log2(sum_j 2^(kappa s_j)) - kappa s with the
 * hardware's exp2 / log2: a code may differ from an exact evaluation where
 * -log2 p lies within about 1e-5 of a rounding boundary; o and score follow
 * exactly from the codes.
 * q_q, k_q, v_q : int8 [H,S,D] on the signed grid of Eq.2 with scales 2^e_q,
 *           2^e_k, 2^e_v.  D = 64 or 128; S % 128 == 0, S <= 32768.
 * qmax    : 15 or 7.   o_f16: fp16 [S, H*D].
 * codes_out : optional [H,S,S/2] bytes as for agq_log2_quant_softmax.
 * score_out : optional int32 [S], ACCUMULATED with atomic adds: the caller
 *           zeroes it before the call.
 * All pointers 16-byte aligned.                                               */
int agq_qk_log2_softmax(const int8_t *q_q, const int8_t *k_q, int64_t H, int64_t S,
                        int64_t D, int causal, int qmax, int e_q, int e_k,
                        const int8_t *v_q, int e_v, void *o_f16, void *codes_out,
                        int32_t *score_out, void *stream);

/* Token pruning, Section 4.3 Eq.4: keep the n_keep tokens with the largest
 * score (equal scores: lower index first), in their original order.
 * score  : int32 [S], S <= 8192.   x_f16: fp16 [S,d] contiguous, d % 8 == 0.
 * idx_out: int32 [n_keep] ascending.  x_out_f16: fp16 [n_keep,d].
 * 0 <= n_keep <= S.                                                           */
int agq_prune_tokens(const int32_t *score, int64_t S, int64_t n_keep,
                     const void *x_f16, int64_t d, int32_t *idx_out,
                     void *x_out_f16, void *stream);

/* One block of the quantized model: the activation quantization pipeline of
 * Section 4.2 (Figure 3: every matrix product takes quantized operands, the
 * non-linear operators in between stay in fp16) with the activation-aware token
 * pruning of Section 4.3 right after attention, for a LLaMA block (RMSNorm,
 * rotary embedding, SwiGLU).  With x fp16 [S,d], positions pos[S]:
 *   h1        = RMSNorm(x; g_attn)
 *   q,k,v     = W4A8(h1)        one Eq.2 pass (step 2^e_attn_in) serves all three
 *   Q,K,V     = Eq.2 to int8 of rope(q), rope(k), v   (steps 2^e_q, 2^e_k, 2^e_v)
 *   o, score  = agq_qk_log2_softmax(Q, K, V), causal
 *   idx       = the n_keep tokens with the largest score (agq_prune_tokens' rule)
 *   x1        = x[idx] + W4A8-or-W4A4(o[idx])           (step 2^e_attn_out;
 *               Section 4.2 allows 4-bit activations after self-attention)
 *   h2        = RMSNorm(x1; g_mlp)
 *   a         = silu(gate) * up,  gate, up = W4A8(h2)   (one Eq.2 pass, 2^e_mlp_in)
 *   x_out     = x1 + W4A8(a)                            (step 2^e_mlp_act)
 * RMSNorm: y = x g / sqrt(mean(x^2) + rms_eps).  rope: inside a head of width D the
 * pair (i, i + D/2) is rotated by the angle whose cosine and sine are
 * rope_cos[pos, i], rope_sin[pos, i].  Every fp16 operator computes in float64 and
 * rounds once to fp16.  All activation grids are signed (zp = 0).
 *
 * d = H*D with D = 64 or 128; d % 128 == 0, F % 128 == 0; 1 <= n_keep <= S
 * (n_keep == S: nothing is pruned); S <= 8192 when tokens are pruned, else
 * S <= 32768.  Eq.9's cascade is a sequence of such calls whose n_keep follow
 * agq_cascade_keep (agq_stack_forward runs such a sequence in one call).
 * All pointers are device pointers, 16-byte aligned; weights are agq_pack_w4 blobs
 * ([d,d] for q, k, v, o; [F,d] for gate, up; [d,F] for down) with fp16 scales.   */
typedef struct agq_block {
    int64_t d, H, F;
    int qmax;               /* 15 or 7, as for agq_qk_log2_softmax                */
    int bits_attn_out;      /* 4 or 8: activation grid of the projection after attention */
    double rms_eps;
    const void *g_attn_f16, *g_mlp_f16;                /* fp16 [d]               */
    const void *w_q, *w_k, *w_v, *w_o, *w_gate, *w_up, *w_down;
    const void *s_q, *s_k, *s_v, *s_o, *s_gate, *s_up, *s_down;
    /* static exponents of the seven quantizers (post-training calibration)       */
    int e_attn_in, e_q, e_k, e_v, e_attn_out, e_mlp_in, e_mlp_act;
    /* TRIP (Section 4.3) at the four activations that feed projections: -1 = the
     * projections of that activation are agq_pack_w4 blobs and Eq.2 is used; n >= 0 =
     * they are agq_pack_w4_trip blobs, all packed with the same factors, n =
     * agq_trip_extra_chunks of those factors, and the site's exponent is Eq.6's base
     * step.  (attn_in: q, k, v; attn_out: o; mlp_in: gate, up; mlp_act: down.)
     * Needs d, F <= 32768.  Factors come from agq_trip_search on the site's tensor of
     * a calibration pass (h1, o_kept, h2, act in the workspace).                  */
    int trip_attn_in, trip_attn_out, trip_mlp_in, trip_mlp_act;
} agq_block;

/* Where every intermediate tensor of a call lives inside the workspace (byte
 * offsets; fp16 unless noted).  Shapes: h1, q, k, v [S,d]; q_q, k_q, v_q int8
 * [H,S_pad,D] (rows from S on are zero); o [S_pad,d]; score int32 [S_pad]; idx int32
 * [n_keep]; o_kept, attn_out, x1, h2, down [n_keep,d] (o_kept == o when nothing is
 * pruned); gate, up, act [n_keep,F]; q_rot, k_rot [S,d] (written by
 * agq_block_calibrate only).  total = the workspace size a call needs.           */
typedef struct agq_block_layout {
    int64_t S_pad;          /* S rounded up to a multiple of 128                   */
    size_t h1, q, k, v, q_q, k_q, v_q, o, score, idx, o_kept, attn_out, x1, h2, gate, up, act, down, q_rot, k_rot,
        gemm_ws, total;
} agq_block_layout;
int agq_block_layout_of(const agq_block *blk, int64_t S, int64_t n_keep, agq_block_layout *out);

/* The fp16 operators of the block as calls of their own (Section 4.2 keeps them in
 * fp16; other block shapes can be wired from these and the products above).  Each
 * computes in float64 and rounds once to fp16.  fp16 tensors are contiguous
 * (leading dimension = row width) and 16-byte aligned.
 *
 * agq_rmsnorm: y[r,:] = t[r,:] * g / sqrt(mean(t[r,:]^2) + eps).  res_f16 == NULL:
 * t = x.  Otherwise t[r,:] = fp16(res[idx[r],:] + x[r,:]) (idx == NULL: row r
 * itself), also written to sum_out_f16 [rows,d]: the residual addition, and the row
 * gather after pruning, fused into the normalisation that follows them.
 * d % 8 == 0, d <= 65536; idx values must be valid rows of res.
 *
 * agq_rope_quantize: rotary embedding of q and k (pairs (i, i + D/2) of every head,
 * angle tables float32 [P, D/2] read at row pos[t], positions clamped into the
 * table), then Eq.2 to int8 (signed grid, steps 2^e_q, 2^e_k, 2^e_v) of the rotated
 * q, k and of v, written per head: int8 [H, S_pad, D] with zero rows from S on
 * (S_pad >= S; agq_qk_log2_softmax wants a multiple of 128).  q, k, v: fp16
 * [S, H*D]; D % 16 == 0.
 *
 * agq_swiglu: out = silu(gate) * up, silu(z) = z / (1 + exp(-z)); n elements,
 * n % 8 == 0.   agq_residual_add: out = fp16(a + b); n % 8 == 0.                  */
int agq_rmsnorm(const void *x_f16, const void *res_f16, const int32_t *idx, const void *g_f16,
                int64_t rows, int64_t d, double eps, void *sum_out_f16, void *y_f16, void *stream);
int agq_rope_quantize(const void *q_f16, const void *k_f16, const void *v_f16, int64_t S, int64_t H,
                      int64_t D, const int32_t *pos, const float *rope_cos, const float *rope_sin,
                      int64_t P, int e_q, int e_k, int e_v, int64_t S_pad, int8_t *q_q, int8_t *k_q,
                      int8_t *v_q, void *stream);
int agq_swiglu(const void *gate_f16, const void *up_f16, void *out_f16, int64_t n, void *stream);
int agq_residual_add(const void *a_f16, const void *b_f16, void *out_f16, int64_t n, void *stream);

/* x_f16 [S,d]; pos int32 [S], every value in [0, P); rope_cos, rope_sin float32
 * [P, D/2] (a position outside the table is clamped into it).  x_out_f16
 * [n_keep,d]; pos_out int32 [n_keep] = pos[idx] (may be NULL).  workspace: `total`
 * bytes of agq_block_layout_of, 256-byte aligned.  Enqueues kernels only.        */
int agq_block_forward(const agq_block *blk, const void *x_f16, const int32_t *pos, const float *rope_cos,
                      const float *rope_sin, int64_t P, int64_t S, int64_t n_keep, void *x_out_f16,
                      int32_t *pos_out, void *workspace, size_t workspace_bytes, void *stream);

/* The same pass with every exponent derived on the way from this input
 * (agq_calibrate_act_exp on the tensor each quantizer reads) and written back to
 * *blk: the post-training calibration step.  Waits for `stream` several times; not
 * capturable.  All four trip_* fields must be -1 (plain blobs).                   */
int agq_block_calibrate(agq_block *blk, const void *x_f16, const int32_t *pos, const float *rope_cos,
                        const float *rope_sin, int64_t P, int64_t S, int64_t n_keep, void *x_out_f16,
                        int32_t *pos_out, void *workspace, size_t workspace_bytes, void *stream);

/* A stack of blocks with the cascade pruning of Section 5.2: block l receives the
 * tokens block l-1 kept and keeps keep[l] of them (keep[l] equal to what it
 * receives: that block prunes nothing); Eq.9's schedule prunes in m of the blocks
 * with the counts of agq_cascade_keep.  blocks: HOST array of n_blocks descriptors
 * with the same d (read before the call returns); keep: HOST int64 [n_blocks],
 * non-increasing, keep[0] <= S.  x_out_f16 [keep[n_blocks-1], d]; pos_out as for a
 * block.  workspace: agq_stack_workspace_bytes (0 = invalid arguments), 256-byte
 * aligned; after the call it holds the intermediates of the last block only.
 * Enqueues kernels only.  Same result as n_blocks calls of agq_block_forward.    */
size_t agq_stack_workspace_bytes(const agq_block *blocks, int n_blocks, int64_t S, const int64_t *keep);
int agq_stack_forward(const agq_block *blocks, int n_blocks, const int64_t *keep, const void *x_f16,
                      const int32_t *pos, const float *rope_cos, const float *rope_sin, int64_t P,
                      int64_t S, void *x_out_f16, int32_t *pos_out, void *workspace,
                      size_t workspace_bytes, void *stream);

/* Section 5.2, Eq.9: m pruning stages share the progressive ratio
 * gamma = 1 - (1 - beta)^(1/m), so that a fraction beta is gone after the last one;
 * a stage that receives S tokens keeps S - floor(S * gamma).  keep_out (HOST int64
 * [m]) receives the tokens left after each stage.  0 <= beta < 1, 1 <= m <= 1024.  */
int agq_cascade_keep(int64_t S, double beta, int m, int64_t *keep_out);

#ifdef __cplusplus
}
#endif
#endif /* AGQ_H */
