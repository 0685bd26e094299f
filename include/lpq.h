/*
 * lpq.h -- C ABI of the MI355X (gfx950) mixed-precision quantized-linear library.
 *
 * The library runs the decoder-layer linears (QKV, out-proj, FC1, FC2) of an LLM pipeline
 * stage whose layers each carry their own weight bitwidth, as in LLM-PQ (arXiv 2403.01136):
 *   - Sec. 4.3, problem statement: a stage is a run of consecutive layers i, each with a
 *     bitwidth b_i from BITs = {3, 4, 8, 16}; it is run at a prefill micro-batch (eta
 *     prompts of s tokens, M = eta * s rows) and at a decode micro-batch (xi rows).
 *   - Sec. 2.4: quantise code = round((w - q) / s), s = (w_max - w_min) / (2^b - 1),
 *     dequantise w~ = s * code + q.  Sec. 4.2: the symmetric scaling factor
 *     max(|w_max|, |w_min|) / (2^(b-1) - 1) used by the per-row 8-bit scheme.
 *   - Sec. 4.1: a quantised weight occupies (#weights) * bit / 8 bytes (dense packing).
 *
 * Conventions that hold for every entry point
 *   - All data pointers are DEVICE pointers (HIP global memory on the current device) unless
 *     the argument is a descriptor struct, which is read on the HOST during the call.
 *   - The library allocates nothing the caller sees.  The caller owns every buffer and keeps
 *     it alive until the work enqueued on `hip_stream` has completed.  Split-K partial sums
 *     live in an internal per-device workspace; every call on a device shares it, so calls that
 *     compute (linears, attention, the indicator) must not overlap on one device: enqueue them on
 *     one stream, or order the streams with events.  The workspace grows on demand by allocating a
 *     larger block; a block that has been handed to a kernel is never freed before the process ends
 *     (queued work and captured graphs may hold its address), so growth costs memory, not safety.
 *     lpq_workspace_reserve sizes it once, after which no call on that device allocates.
 *   - `hip_stream` is a hipStream_t passed as void* (NULL = the default stream).  Calls
 *     enqueue work and return without synchronising.
 *   - Calls record only kernel launches (and, for the loader, copies) on `hip_stream`, so they can be
 *     captured in a HIP graph once an eager call of the same shape has run (the internal workspace is
 *     allocated, and kernel attributes are set, on first use -- not things a capture may contain).
 *     A captured graph keeps the workspace address it was recorded with; that block stays allocated,
 *     but eager calls that needed a larger block have moved on to another one, so a replay and an
 *     eager call may then run concurrently without sharing partial sums -- they are still ordered
 *     by the caller as above.
 *   - Arguments are validated on the host before the first HIP call; on any error nothing is
 *     launched and no buffer is touched.  No exceptions, no errno, no global error state.
 *   - fp16 is IEEE binary16.  x is [M][K], y is [M][N], both dense row-major, 16-byte
 *     aligned; y is overwritten.  A linear computes y[m][n] = sum_k x[m][k] * w~[n][k]
 *     (+ bias[n]) with fp32 accumulation and one final round-to-nearest-even to fp16.
 *
 * Storage format of a quantised weight W [N][K] (K contiguous); N % 64 == 0, K % 128 == 0
 *   A block is 64 rows x 128 columns (one quantisation group per row); blocks are stored in
 *   order rb * (K/128) + kt, so the blocks of one 64-row band are one contiguous byte stream.
 *   A block holds four 16-row tiles back to back; tile t holds rows 64*rb + 4*r + t (r = 0..15).
 *   Inside a tile, lane = 16*kq + r (kq = 0..3) owns the 32 codes of its row at block columns
 *   32*j + 8*kq + e (j = 0..3, e = 0..7), numbered c = 8*j + e -- the operand layout of one
 *   wavefront's four v_mfma_f32_16x16x32_f16 steps; a lane's four tiles are four consecutive rows.
 *     bits 4:  1024-byte tile; 16 B per lane at 16*lane; little-endian u32 word j; code e at bit
 *              4*(e/2) + 16*(e%2) of word j (even e in the low half-word, odd e in the high).
 *     bits 3:  768-byte tile (dense, not padded to 4 bits); 12 B per lane at 12*lane; three LE
 *              u32 words.  Pair P = c/2, half h = c%2.  P < 15: word P/5, bits 16*h + 3*(P%5) .. +2.
 *              P == 15: bit i of the code is bit 16*h + 15 of word i.
 *     bits 8:  2048-byte tile; 32 B per lane as two 16-byte pieces; piece p (j = 2p, 2p+1) at
 *              1024*p + 16*lane; byte 8*(j%2) + e.  Unsigned for LPQ_ASYM_GROUP, two's
 *              complement in [-127, 127] for LPQ_SYM_CHANNEL.
 *     bits 16: 4096-byte tile of the unchanged fp16 weights; 64 B per lane as four 16-byte pieces,
 *              piece j at 1024*j + 16*lane, element e at byte 2*e.
 *   scales, zeros: fp16 [K/128][N], group-major (index g*N + n) for LPQ_ASYM_GROUP; scales fp16
 *   [N] and no zeros for LPQ_SYM_CHANNEL; neither for LPQ_FP16.  "zero" is the group minimum, a
 *   floating offset.
 */
#ifndef LPQ_H
#define LPQ_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    LPQ_OK = 0,
    LPQ_ERR_NULL = 1,        /* a required pointer is NULL                                   */
    LPQ_ERR_BITS = 2,        /* bits not in {3, 4, 8, 16}                                    */
    LPQ_ERR_SCHEME = 3,      /* unknown scheme, or bits / scheme / group_size do not match   */
    LPQ_ERR_SHAPE = 4,       /* K % 128, N % 64, K, N, M or n_layers out of range; bad plan  */
    LPQ_ERR_ALIGN = 5,       /* a data pointer is not 16-byte aligned                        */
    LPQ_ERR_BUFSIZE = 6,     /* a caller's buffer is too small, or workspace could not grow  */
    LPQ_ERR_DEVICE = 7,      /* a HIP call failed                                            */
    LPQ_ERR_UNSUPPORTED = 8  /* valid request the library does not implement                 */
} lpq_status;

typedef enum {
    LPQ_FP16 = 0,         /* bits = 16: weights used unchanged (Sec. 4.3, BITs contains 16)   */
    LPQ_ASYM_GROUP = 1,   /* bits in {3,4,8}: per (row, 128 columns) scale and zero = minimum
                             (Sec. 2.4; asymmetric scaling factor of Sec. 4.2)                */
    LPQ_SYM_CHANNEL = 2   /* bits = 8: per-row scale, signed codes, no zero (symmetric scaling
                             factor of Sec. 4.2)                                              */
} lpq_scheme;

/* Shape and quantisation of one linear's weight.  group_size must be 128 for LPQ_ASYM_GROUP
 * and 0 (or 128, ignored) otherwise. */
typedef struct {
    int32_t bits;        /* 3, 4, 8 or 16 */
    int32_t scheme;      /* lpq_scheme    */
    int32_t group_size;
    int32_t K;           /* input features, % 128 == 0  */
    int32_t N;           /* output features, % 64 == 0  */
} lpq_qdesc;

/* One quantised weight: descriptor + caller-owned device buffers sized by lpq_packed_sizes.
 * zeros is ignored unless scheme == LPQ_ASYM_GROUP; scales is ignored for LPQ_FP16.
 * bias: optional fp16 [N] (NULL = none). */
typedef struct {
    lpq_qdesc d;
    void *codes;
    void *scales;
    void *zeros;
    const void *bias;
} lpq_qweight;

/* The four linears of one decoder layer (Sec. 4.1: 4*h1^2 + 2*h1*h2 weights per layer). */
typedef struct {
    lpq_qweight qkv, out, fc1, fc2;
} lpq_layer;

/* Per-layer inputs and outputs of lpq_stage_linears.  The four linears of a layer are
 * independent here: each reads its own x and writes its own y (attention, activation,
 * normalisation and residual, which connect them in a model, are outside this library). */
typedef struct {
    const void *x_qkv, *x_out, *x_fc1, *x_fc2;   /* fp16 [M][K of that linear] */
    void *y_qkv, *y_out, *y_fc1, *y_fc2;         /* fp16 [M][N of that linear] */
} lpq_layer_io;

typedef enum { LPQ_PREFILL = 0, LPQ_DECODE = 1 } lpq_phase;

/* What a linear does to acc + bias before its one rounding to fp16 (used by the decoder layer). */
typedef enum { LPQ_ACT_NONE = 0, LPQ_ACT_RELU = 1, LPQ_ACT_GELU_TANH = 2 } lpq_activation;
typedef struct {
    int32_t activation;      /* lpq_activation, applied to acc + bias                               */
    const void *residual;    /* device fp16 [M][N] added after the activation, or NULL              */
} lpq_epilogue;

/* Bytes of the three packed buffers of a weight (Sec. 4.1: codes = K*N*bits/8, dense).
 * Host-only, touches no device.  Errors: NULL, BITS, SCHEME, SHAPE. */
lpq_status lpq_packed_sizes(const lpq_qdesc *desc, size_t *code_bytes, size_t *scale_bytes, size_t *zero_bytes);

/* Round-to-nearest quantiser + bit-packer (Sec. 2.4, Sec. 4.2; the on-GPU step of the
 * on-the-fly quantised loader of Sec. 5).
 *   w_fp16: device, fp16 [N][K] row-major, 16-byte aligned, read only.
 *   out:    host struct; out->d must equal *desc; out->codes / scales / zeros are device
 *           buffers of at least the sizes lpq_packed_sizes reports; they are overwritten.
 * Results are bit-exact functions of w (fp32 IEEE arithmetic, round-half-even):
 *   LPQ_ASYM_GROUP  scale = fp16((max - min) / (2^b - 1)) (1.0 if that is zero),
 *                   zero = min, code = clamp(rint((w - zero) / scale), 0, 2^b - 1)
 *   LPQ_SYM_CHANNEL scale = fp16(max|w| / 127) (1.0 if zero), code = clamp(rint(w / scale), +-127)
 *   LPQ_FP16        codes = the fp16 values of w, unchanged, in tile order.
 * Weights must be finite.  Errors: NULL, BITS, SCHEME, SHAPE, ALIGN, DEVICE. */
lpq_status lpq_quantize_pack(const void *w_fp16, const lpq_qdesc *desc, lpq_qweight *out, void *hip_stream);

/* The same quantiser on a window of rows: rows [row0, row0 + n_rows) of the weight that `desc` describes,
 * read from a device buffer that holds just those rows ([n_rows][K] fp16).  row0 and n_rows are multiples
 * of 64 (the storage format's row blocks; n_rows may be 0).  Writes only those rows' codes, scales and
 * zeros in `out`, so a weight can be quantised piecewise, in any order, as its rows arrive.
 * Errors: as lpq_quantize_pack; SHAPE also for a window that is not on 64-row boundaries or leaves W. */
lpq_status lpq_quantize_pack_rows(const void *w_rows_fp16, const lpq_qdesc *desc, int32_t row0, int32_t n_rows,
                                  lpq_qweight *out, void *hip_stream);

/* On-the-fly quantised loading of one module's weight from HOST memory (Sec. 5, "On-The-Fly Quantizer":
 * module-level weights quantised on the GPU as they arrive, so that the fp16 weight is never resident on
 * the device as a whole).
 *   w_fp16_host: HOST pointer, fp16 [N][K] row-major, 16-byte aligned.  Pinned memory gives asynchronous
 *                copies at the link's rate; pageable memory works but is staged by the runtime.
 *   staging:     device buffer of staging_bytes, caller-owned, 16-byte aligned; it receives one band of rows
 *                at a time (as many 64-row blocks as fit), which is then quantised into its place in `out`.
 *                LPQ_ERR_BUFSIZE if it cannot hold 64 rows (64 * K * 2 bytes).
 *   out:         as for lpq_quantize_pack; the result is bit-identical to it.
 * Copies and quantiser alternate on `hip_stream` (the quantiser is some thirty times faster than the host
 * link, so the link stays busy); when the work queued on it has completed, `out` is ready and the host
 * buffer and the staging buffer are free again.  The call itself returns without synchronising when the
 * host memory is pinned.
 * Errors: NULL, BITS, SCHEME, SHAPE, ALIGN, BUFSIZE, DEVICE. */
lpq_status lpq_load_quantize_pack(const void *w_fp16_host, const lpq_qdesc *desc, lpq_qweight *out, void *staging,
                                  size_t staging_bytes, void *hip_stream);

/* One quantised linear at a prefill micro-batch (Sec. 4.3: M = eta * s tokens): weight tiles
 * are dequantised in registers to fp16 and multiplied on the matrix cores.
 *   w: host struct with device buffers;  x: device fp16 [M][K];  y: device fp16 [M][N].
 * Correct for every M >= 1.  Errors: NULL, BITS, SCHEME, SHAPE (M < 1), ALIGN, DEVICE. */
lpq_status lpq_qlinear_prefill(const lpq_qweight *w, const void *x, int32_t M, void *y, void *hip_stream);

/* The same function at a decode micro-batch (Sec. 4.3: M = xi rows, one token per sequence):
 * packed weights are streamed once from HBM and unpacked in registers.  Correct for every
 * M >= 1 (rows are processed 64 at a time).  Errors as for lpq_qlinear_prefill, plus BUFSIZE, and UNSUPPORTED
 * for K >= 2^23 (the decode kernels' descriptors keep K / 128 in 16 bits). */
lpq_status lpq_qlinear_decode(const lpq_qweight *w, const void *x, int32_t M, void *y, void *hip_stream);

/* One linear with a fused epilogue: y = fp16(act(x . w~^T + bias) + residual), one rounding.  `phase`
 * picks the kernel family as in lpq_stage_linears.  ep may be NULL (= lpq_qlinear_prefill / _decode).
 * residual may alias y (each element is read before it is written, by the same thread).
 * Errors: as the plain calls; UNSUPPORTED for an unknown activation. */
lpq_status lpq_qlinear_fused(const lpq_qweight *w, const void *x, int32_t M, void *y, const lpq_epilogue *ep,
                             lpq_phase phase, void *hip_stream);

/* All 4 * n_layers linears of a stage, each layer at its own bitwidth (Sec. 4.3: stage
 * latency is the sum over its layers of the per-layer latency at that layer's precision).
 *   layers: host array [n_layers];  io: host array [n_layers] of device pointers.
 *   phase:  LPQ_PREFILL or LPQ_DECODE selects the kernel family; M as above.
 * In the decode phase a stage of up to twelve layers is one grouped launch (with a short kernel that prepares the
 * activations in front and a fix-up pass behind); a longer stage takes one such launch per twelve layers or fewer.
 * Errors: as above; nothing is launched unless every layer validates. */
lpq_status lpq_stage_linears(const lpq_layer *layers, int32_t n_layers, lpq_phase phase, int32_t M,
                             const lpq_layer_io *io, void *hip_stream);

/* lpq_stage_linears for callers that cannot allocate device memory while they run: code under HIP graph capture,
 * tight serving loops, harnesses that forbid hipMalloc.  Same arguments, same kernels and the same results, but the
 * fp32 partial tiles and the prepared activations of the launches live in a static 128 MiB array inside the library
 * (one copy per device, held until the process ends) instead of the growing workspace, and the call never allocates or
 * frees.  That array covers a decode-phase call of any number of rows (64 MiB of partial tiles per pass of 64 rows; up to
 * 16 rows 16 MiB and, for 3-bit linears, 2 bytes per token row and column of the launch's activations: ten
 * BLOOM-176B-shaped layers at 16 rows take 31 MiB), and a prefill-phase call none of whose launches is
 * split over K (stage-wide launches are not); a call that would need more returns LPQ_ERR_BUFSIZE and launches nothing
 * further.  All calls on a device share the array, which keeps the last call's contents (nothing in it has to
 * start at zero: every partial tile read was written by the same call); calls that overlap on one device race.
 * Errors: as lpq_stage_linears, plus BUFSIZE as above. */
lpq_status lpq_stage_linears_noalloc(const lpq_layer *layers, int32_t n_layers, lpq_phase phase, int32_t M,
                                     const lpq_layer_io *io, void *hip_stream);

/* ---- The rest of the decoder layer (beyond the hot path of the four linears) -------------------------
 * The published pre-LayerNorm decoder block of the paper's models, with the KV cache reserved for
 * max_seq = s + n positions per sequence (Sec. 4.1, "KV Storage Modeling"; Sec. 5):
 *   h1 = LN1(x); qkv = h1 . Wqkv^T; append K, V at positions pos0 .. pos0+T-1; a = attention(q, cache);
 *   x1 = x + a . Wout^T; h2 = LN2(x1); f = act(h2 . Wfc1^T); y = x1 + f . Wfc2^T
 * with every operator's output rounded once to fp16.  Token rows are ordered [sequence][token]:
 * M = n_seqs * T rows, T = 1 in the decode phase; all sequences of a call are at the same position pos0.
 * Caches (device, fp16, caller-owned, one pair per layer): k_cache [batch][n_heads][max_seq][head_dim],
 * vt_cache [batch][n_heads][head_dim][max_seq] (V transposed: a feature's positions are contiguous). */
typedef struct {
    int32_t n_heads, head_dim;   /* hidden size = n_heads * head_dim; head_dim is 64 or 128                */
    int32_t max_seq;             /* cache positions per sequence, a multiple of 64                         */
    int32_t activation;          /* lpq_activation of the feed-forward block                               */
    float ln_eps;
} lpq_layer_cfg;

typedef struct {
    const void *ln1_gamma, *ln1_beta, *ln2_gamma, *ln2_beta;   /* device fp16 [hidden]                     */
    void *k_cache, *vt_cache;                                  /* device fp16, layouts above               */
    const float *alibi_slopes;   /* device fp32 [n_heads]: score += slope * (key position - query position), or NULL */
} lpq_layer_state;

/* y[m][:] = (x[m][:] - mean) / sqrt(var + eps) * gamma + beta per row (biased variance), fp32 statistics.
 * x, y: device fp16 [M][hidden]; hidden % 8 == 0, hidden <= 16384.  Errors: NULL, SHAPE, ALIGN, DEVICE. */
lpq_status lpq_layernorm(const void *x, const void *gamma, const void *beta, float eps, int32_t M, int32_t hidden, void *y,
                         void *hip_stream);

/* Copy the K and V parts of qkv (device fp16 [n_seqs * T][3 * hidden]; per token q | k | v, heads of
 * head_dim each) into the caches at positions pos0 .. pos0 + T - 1 of sequences 0 .. n_seqs - 1.
 * Errors: NULL, SHAPE (head_dim, max_seq, pos0 + T > max_seq, counts < 1), ALIGN, DEVICE. */
lpq_status lpq_kv_append(const void *qkv, const lpq_layer_cfg *cfg, const lpq_layer_state *st, int32_t n_seqs, int32_t T,
                         int32_t pos0, void *hip_stream);

/* Causal attention of the T new tokens of each sequence over cache positions 0 .. pos0 + t:
 * out = softmax(q . k / sqrt(head_dim) + alibi) . v per head, heads concatenated; queries are the q part of
 * qkv; the caches must already hold positions < pos0 + T (lpq_kv_append).  out: device fp16 [n_seqs * T][hidden].
 * T = 1 streams the cache once (split over positions when there are few sequences, partial results in the
 * library's workspace); T > 1 runs on the matrix cores.  Errors: as lpq_kv_append, plus BUFSIZE. */
lpq_status lpq_attention(const void *qkv, const lpq_layer_cfg *cfg, const lpq_layer_state *st, int32_t n_seqs, int32_t T,
                         int32_t pos0, void *out, void *hip_stream);

/* Bytes of workspace lpq_decoder_layer needs for M = n_seqs * T token rows (0 on a bad argument). */
size_t lpq_decoder_layer_workspace(const lpq_layer *layer, const lpq_layer_cfg *cfg, int32_t M);

/* One decoder layer: x, y device fp16 [n_seqs * T][hidden] (y may be x); `layer` holds the four quantised
 * linears (their K, N must match hidden and the feed-forward size; biases optional); `workspace` is a
 * caller-owned device buffer of at least lpq_decoder_layer_workspace bytes, 16-byte aligned.  `phase`
 * picks the linears' kernel family; attention follows T.  Updates the caches at pos0 .. pos0 + T - 1.
 * Errors: NULL, BITS, SCHEME, SHAPE, ALIGN, BUFSIZE, DEVICE, UNSUPPORTED (activation). */
lpq_status lpq_decoder_layer(const lpq_layer *layer, const lpq_layer_cfg *cfg, const lpq_layer_state *st, lpq_phase phase,
                             int32_t n_seqs, int32_t T, int32_t pos0, const void *x, void *y, void *workspace,
                             size_t workspace_bytes, void *hip_stream);

/* Variance indicator of one linear operator (Sec. 4.2, Theorem 1 and Eq. 3): the estimated extra output
 * variance D_W * S_W(b)^2 * G(X) under b-bit weight quantisation, G(X) = Var[X] / 4 (deterministic rounding,
 * stochastic = 0) or (E[X]^2 + Var[X]) / 6 (stochastic = 1), E and Var over all elements of X.  A layer's
 * indicator omega_{i,b} is the sum of its operators' values.
 *   w_fp16: device fp16 [N][K] (the unquantised weight; K % 128 == 0);  x: device fp16 [M][K].
 *   omega:  device double[8], written asynchronously:
 *           [0..2] bits 3, 4, 8 with the quantiser's granularity: sum over (row, 128-column) groups of
 *                  128 * ((max - min) / (2^b - 1))^2;   [3] symmetric 8-bit, a scale per row;
 *           [4..6] bits 3, 4, 8 as printed in the paper: one scaling factor for the whole matrix, D_W = N * K;
 *           [7]    symmetric 8-bit, one scaling factor for the whole matrix.
 * Scaling factors are not rounded to fp16.  Uses the library's per-device workspace.
 * Errors: NULL, SHAPE (K % 128, counts < 1), ALIGN, BUFSIZE, DEVICE. */
lpq_status lpq_variance_indicator(const void *w_fp16, int32_t K, int32_t N, const void *x, int32_t M, int32_t stochastic,
                                  double *omega, void *hip_stream);

/* ---- The assigner's cost models and bitwidth-transfer heuristic (Sec. 4.1, Sec. 4.3): host code only -------------
 * Every pointer below is a HOST pointer, nothing touches a device, nothing is asynchronous.  These calls close the
 * loop from the measured decoder-layer latencies back to the plan (layers per stage, bitwidth per layer) that the
 * kernels above serve. */

/* Shape of a model for the memory cost model (Table 2 notation). */
typedef struct lpq_model_shape {
    int64_t h1, h2;        /* hidden size, feed-forward size                                         */
    int64_t vocab, d_t;    /* vocabulary size, word-embedding width                                  */
    int64_t pos;           /* max position embeddings                                                */
    int32_t rmsnorm, pad;  /* 1: RMSNorm (4 h1 bytes of norm weights per layer), 0: LayerNorm (6 h1) */
} lpq_model_shape;

/* Memory cost model (Sec. 4.1), bytes as doubles (negative on a bad argument):
 * embeddings + LM head in fp16: (vocab d_t + pos d_t + [2 h1 d_t if h1 != d_t] + vocab d_t) * 2;
 * one decoder layer at `bit` bits: (4 h1^2 + 2 h1 h2) * bit / 8 + the norm term;
 * KV cache of one layer for v requests of s + n positions: 2 v (s + n) h1 * bit_kv / 8. */
double lpq_mem_embedding_bytes(const lpq_model_shape *m);
double lpq_mem_layer_bytes(const lpq_model_shape *m, int32_t bit);
double lpq_mem_kv_bytes(const lpq_model_shape *m, int64_t v, int64_t s, int64_t n, int32_t bit_kv);

/* Latency cost model (Sec. 4.1): least-squares fit of one decoder layer's time, per phase and precision.
 *   LPQ_PREFILL: t ~ c0 + c1 v + c2 s + c3 v s + c4 v s^2          (len = prompt length s;  5 coefficients)
 *   LPQ_DECODE:  t ~ c0 + c1 v + c2 v (t+s) + c3 (t+s)             (len = cached positions; 4 coefficients)
 * v, len, t: n_samples values each.  Solved by Householder QR on scaled columns.
 * Errors: NULL, SHAPE (fewer samples than coefficients, or samples that do not determine them), UNSUPPORTED (phase). */
lpq_status lpq_latency_fit(lpq_phase phase, int32_t n_samples, const double *v, const double *len, const double *t,
                           double *coef);
lpq_status lpq_latency_predict(lpq_phase phase, const double *coef, int32_t n, const double *v, const double *len,
                               double *t_out);

/* The assignment program of Sec. 4.3 (Eq. 1 and its constraints) for L layers of one shape on N pipeline devices.
 * A plan is counts[N] (consecutive layers per stage, each >= 1, summing to L) and choice[L] (index into bits). */
typedef struct lpq_plan_problem {
    int32_t L, N, n_bits, pad;
    const int32_t *bits;      /* [n_bits] allowed bitwidths                                                     */
    const double *omega;      /* [L][n_bits] variance indicator of layer i at bits[k]                           */
    const double *lat_pre;    /* [N][n_bits] seconds of one layer at bits[k] on device j, prefill micro-batch   */
    const double *lat_dec;    /* [N][n_bits] the same for one decode step at the mean context s + n / 2         */
    const double *mem;        /* [n_bits] bytes a layer at bits[k] reserves (weights + its KV cache)            */
    const double *cap;        /* [N] bytes device j offers to layers (temporary memory already taken off)       */
    const double *comm_pre;   /* [N] seconds of stage j's prefill send P_pre / f_j, or NULL for none            */
    const double *comm_dec;   /* [N] the same for decode, or NULL                                               */
    double emb;               /* bytes of embeddings the first device also holds                                */
    double theta;             /* weight of the quality term                                                     */
    int32_t B, eta, xi, n;    /* global batch, prefill and decode micro-batch, tokens to generate               */
} lpq_plan_problem;

/* Eq. (1): (ceil(B/eta) - 1) Tmax_pre + (ceil(B/xi) - 1)(n - 1) Tmax_dec + T_pre + T_dec + theta * sum omega, with
 * Tmax the largest stage time or send time of the phase; only the quality term if with_latency == 0.
 * *obj = +infinity for a plan that is malformed or exceeds a device's memory.  Errors: NULL, SHAPE. */
lpq_status lpq_plan_objective(const lpq_plan_problem *p, const int32_t *counts, const int32_t *choice, int32_t with_latency,
                              double *obj);

/* "adabits" (Sec. 4.3, Algorithm 2's starting point): the program without its latency terms, solved exactly by
 * dynamic programming over stages and per-stage bitwidth counts.  Writes a plan of least theta * sum omega under the
 * memory constraints; *obj = +infinity (plan untouched) if none exists.  Among equal plans any may be returned.
 * Errors: NULL, SHAPE (L < N, n_bits > 4, sizes < 1), BUFSIZE (tables would exceed 1 GiB). */
lpq_status lpq_plan_adabits(const lpq_plan_problem *p, int32_t *counts, int32_t *choice, double *obj);

/* Bitwidth transfer (Sec. 4.3, Algorithm 2) from the plan in counts / choice (in and out).  Each round ranks the
 * stages by ceil(B/eta) T_pre,j + ((ceil(B/xi) - 1)(n - 1) + 1) T_dec,j, takes the slowest as the straggler, tries
 * with every other stage (fastest first) every rule (b_st, b_pi, nums = max(1, b_pi / b_st)), b_st != b_pi in bits
 * order -- the straggler hands nums layers of b_st bits over and takes one of b_pi bits back, layer windows shift
 * accordingly, each stage gives its bitwidths to the layers that lose least -- and applies the exchange with the
 * strictly lowest Eq. (1) value if that is below the current one; it ends when a round finds none.
 * *obj = the final Eq. (1) value, *rounds = exchanges applied.  Errors: NULL, SHAPE (malformed start plan). */
lpq_status lpq_plan_bitwidth_transfer(const lpq_plan_problem *p, int32_t *counts, int32_t *choice, double *obj,
                                      int32_t *rounds);

/* ---- The library's per-device workspace and dispatch routing -------------------------------------------------- */

/* Growth policy of the workspace, as a pure function (host only, touches no device): a call that needs `need_bytes`
 * when the current block has `have_bytes` reuses the block (*alloc_bytes = 0) or allocates a new one of *alloc_bytes
 * (need + 25 %, at least 8 MiB) and retires the old one without freeing it; with a reservation in force
 * (reserved != 0) a larger need is LPQ_ERR_BUFSIZE instead.  Errors: NULL, BUFSIZE. */
lpq_status lpq_workspace_policy(size_t have_bytes, int32_t reserved, size_t need_bytes, size_t *alloc_bytes);

/* Make the current device's workspace at least `bytes` large now (one allocation, unless it already is) and forbid
 * later growth on this device: from here on no call allocates, and a call that would need more returns
 * LPQ_ERR_BUFSIZE.  For callers that capture graphs or must not allocate while serving.  Errors: DEVICE, BUFSIZE. */
lpq_status lpq_workspace_reserve(size_t bytes);

/* Bytes of the current device's workspace block (0 before first use). */
size_t lpq_workspace_bytes(void);

/* Routing of decode launches, process-wide, for tests that must reach either kernel family with small shapes:
 * a launch that streams at most rows_max_mib MiB of codes (default 192) takes the kernel that gives a group of
 * 16-row tiles a workgroup, others the even-share kernel; rows_tiles = 2..5 forces that group size (0 = the
 * library's choice).  Negative values restore the defaults.  Errors: SHAPE. */
lpq_status lpq_set_decode_routing(int32_t rows_max_mib, int32_t rows_tiles);

/* Test helper, not on the hot path: w_fp32[n][k] = scale * code + zero (fp32 multiply, then
 * fp32 add; the fp16 weight itself for LPQ_FP16) read back from the packed buffers.
 *   w_fp32: device float [N][K].  Errors: NULL, BITS, SCHEME, SHAPE, ALIGN, DEVICE. */
lpq_status lpq_unpack_dequant(const lpq_qweight *w, void *w_fp32, void *hip_stream);

/* Static string for a status code (never NULL). */
const char *lpq_status_str(lpq_status status);

#ifdef __cplusplus
}
#endif
#endif /* LPQ_H */
