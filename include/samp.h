/*
 * samp.h - C ABI of the MI355X (gfx950) self-adaptive mixed-precision encoder.
 *
 * The library runs the encoder hot path of SAMP (arXiv 2209.09130, Section 3.2):
 * a stack of BERT-style post-LayerNorm Transformer layers in which, per layer,
 * the attention block (MHA: QKV GEMM, softmax attention, attention-output GEMM)
 * and the feed-forward block (FFN: FFN1 GEMM + GELU, FFN2 GEMM) each run either
 * in FP16 or with post-training-quantised INT8 GEMMs.  "Fully-Quant" is both
 * blocks INT8, "Quant-FFN-Only" is INT8 FFN with FP16 MHA (Section 3.2); the
 * per-layer choice of either block is the mixed-precision configuration of
 * Section 3.2 / Table 1.  Inside a quantised block every tensor between kernels
 * is int8; dequantise + bias + residual + LayerNorm + quantise are one kernel;
 * the softmax output is quantised (Section 4.2, Appendix B); the last kernel of
 * a layer emits floating point when its consumer is not quantised.
 *
 * Conventions
 *   - All `dev` pointers are device memory of the current HIP device, owned by
 *     the caller, 16-byte aligned unless a stricter alignment is stated.  `host`
 *     pointers are ordinary host memory.  The library never allocates or frees
 *     device memory; it owns only the host-side encoder handle.
 *   - fp16 = IEEE binary16 stored as uint16_t; matrices are row-major; weight
 *     matrices are [out, in] (K contiguous).
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).
 *     Entry points that launch kernels are asynchronous on that stream and do
 *     not synchronise, except samp_encoder_create and samp_encoder_calibrate,
 *     which return after their work is complete.
 *   - Every function returning int returns SAMP_OK (0) or a negative samp_status;
 *     samp_last_error() then describes the failure.  No exception or abort
 *     crosses this boundary.  Arguments are checked on the host before any
 *     kernel is launched.
 *   - Threads: an encoder handle is used by one thread at a time (a forward
 *     updates its graph cache and event pool); different handles, and the step
 *     entry points, may be used from different threads.  samp_last_error() is
 *     per thread.  An encoder owns a few HIP streams and events for its batch
 *     groups and graph capture; samp_encoder_destroy releases them.
 *   - Quantiser (Appendix B: multiply by a scale, round, symmetric 8-bit range):
 *     code = clamp(round_half_even(x * (1/s)), -127, 127), where the step s is
 *     absmax/127 from a min-max calibration (Table 2 caption) and 1/s is formed
 *     once in binary32.  Weights use one step per output channel.
 */
#ifndef SAMP_H
#define SAMP_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define SAMP_API __attribute__((visibility("default")))

typedef struct samp_encoder samp_encoder_t;

/* per-layer precision: bit 0 = MHA block INT8, bit 1 = FFN block INT8 (Section 3.2, Table 1).
 * SAMP_P_UNSIGNED, valid only together with bit 0, stores the softmax output of that layer as
 * unsigned codes rne(P / s_p) in [0, 255] instead of the symmetric [-127, 127], whose negative
 * half a softmax never uses (the loss Section 4.2 and Appendix B describe); the caller then
 * passes the step s_p = absmax(P) / 255 in samp_layer_scales_t.
 * SAMP_P_FP16, valid only together with bit 0 and not with SAMP_P_UNSIGNED, is the other remedy:
 * the softmax output of that layer is rounded to binary16 instead of being put on an 8-bit grid
 * and multiplies the integer V codes, ctx = rne(fl32(sum P16 V) * s_v / s_ctx); the sum is
 * evaluated exactly (integer digit planes of P16 * 2^24 on the matrix cores); s_p is not used.   */
enum { SAMP_FP16 = 0, SAMP_MHA_INT8 = 1, SAMP_FFN_INT8 = 2, SAMP_FULL_INT8 = 3, SAMP_P_UNSIGNED = 4, SAMP_P_FP16 = 8 };

enum {
    SAMP_OK = 0,
    SAMP_ERR_ARG = -1,    /* null pointer, negative size, unknown mode, wrong encoder kind        */
    SAMP_ERR_SHAPE = -2,  /* shape outside the supported set or above max_batch / max_seq         */
    SAMP_ERR_SPACE = -3,  /* arena / workspace too small or misaligned (256 bytes)                */
    SAMP_ERR_HIP = -4,    /* a HIP call failed                                                    */
    SAMP_ERR_SCALE = -5   /* a scale needed by an INT8 block is not finite, not positive or out of range */
};

/* Supported shapes: head size hidden/heads == 64; hidden % 128 == 0; ffn % 128 == 0;
 * hidden <= 2048; 1 <= max_seq <= SAMP_MAX_SEQ; 1 <= max_batch <= SAMP_MAX_BATCH.  Up to 512 tokens a sequence's
 * attention scores stay in registers; longer sequences take a three-sweep attention kernel that
 * recomputes them (same results, about half the rate per token pair).  Row counts are 32-bit:
 * max_batch * max_seq <= SAMP_MAX_TOKENS.                                                         */
#define SAMP_MAX_SEQ 4096
#define SAMP_MAX_TOKENS (1 << 24)
#define SAMP_MAX_BATCH 8192
typedef struct {
    int32_t layers, hidden, heads, ffn, max_batch, max_seq;
    float ln_eps;
} samp_config_t;

/* One layer's parameters, HOST pointers, copied during samp_encoder_create.
 * w_qkv [3H,H]: rows 0..H-1 = Q, H..2H-1 = K, 2H..3H-1 = V; head h owns 64 consecutive rows of each.
 * w_o [H,H], w_ffn1 [F,H], w_ffn2 [H,F]; biases and LayerNorm vectors are binary32.               */
typedef struct {
    const uint16_t *w_qkv, *w_o, *w_ffn1, *w_ffn2;
    const float *b_qkv, *b_o, *b_ffn1, *b_ffn2, *ln1_g, *ln1_b, *ln2_g, *ln2_b;
} samp_layer_weights_t;

/* Per-tensor activation steps (absmax/127) of one layer, fixed after calibration (Appendix B):
 * x = layer input, q k v = projections incl. bias, p = softmax output, ctx = P.V,
 * attn_out = attention-output GEMM before its bias, ffn_in = first LayerNorm's output,
 * ffn_mid = GELU output, ffn_out = FFN2 GEMM before its bias.  Only the steps of INT8 blocks are
 * read: x..attn_out if the MHA block is INT8 (x also when this layer's input must be quantised by
 * its producer), ffn_in..ffn_out if the FFN block is INT8.                                        */
typedef struct {
    float x, q, k, v, p, ctx, attn_out, ffn_in, ffn_mid, ffn_out;
} samp_layer_scales_t;

/* ---- encoder ---------------------------------------------------------------------------------- */

/* Bytes of device memory samp_encoder_create needs for the packed weights of this configuration
 * (includes a staging area used only during create).  0 on invalid arguments.                     */
SAMP_API size_t samp_encoder_arena_bytes(const samp_config_t *cfg, const uint8_t *modes /* host [layers] */);

/* Builds an encoder.  Weights of INT8 blocks are quantised on the device per output channel
 * (s_w = absmax/127, code = rne(w / s_w)); epilogue multipliers are folded in binary64 and rounded
 * once to binary32.  `scales` (host [layers]) may be NULL only if every mode is SAMP_FP16.
 * `dev_arena` (dev, 256-byte aligned, >= samp_encoder_arena_bytes) must outlive the encoder; the
 * host arrays may be released when the call returns.  Synchronises `stream` before returning.     */
SAMP_API int samp_encoder_create(const samp_config_t *cfg, const uint8_t *modes,
                                 const samp_layer_weights_t *weights /* host [layers] */,
                                 const samp_layer_scales_t *scales /* host [layers] or NULL */,
                                 void *dev_arena, size_t arena_bytes, void *stream, samp_encoder_t **out);

/* Workspace bytes a forward of batch B and padded length S needs.  0 on invalid arguments.        */
SAMP_API size_t samp_encoder_workspace_bytes(const samp_encoder_t *enc, int32_t B, int32_t S);

/* One forward pass (Section 3.2).  hidden: dev fp16 [B,S,H].  mask: dev int32 [B,S], 1 = token,
 * right-padded (a sequence's tokens form a prefix, at least one token), or NULL = every sequence
 * has S tokens.  With a mask, padding is removed on entry (only valid tokens are computed) and
 * restored on exit: padded rows of `out` are written as zeros and never influence valid rows.
 * The mask is device memory and a forward never synchronises, so its contents are not checked: a
 * sequence whose mask row is all zero takes part in nothing (no packed rows, no attention work) and
 * all S rows of its output are zeros; a mask that is not a prefix is read as its number of ones.
 * out: dev fp16 [B,S,H], must not alias hidden.  workspace: dev, 256-byte aligned,
 * >= samp_encoder_workspace_bytes(enc,B,S); calls sharing a workspace must be stream-ordered.     */
SAMP_API int samp_encoder_forward(samp_encoder_t *enc, const void *hidden, const int32_t *mask, int32_t B, int32_t S,
                                  void *out, void *workspace, size_t workspace_bytes, void *stream);

/* samp_encoder_forward for callers that cannot allocate (code under HIP graph capture, tight serving loops,
 * harnesses that forbid hipMalloc): the same kernels, run as ONE group with plain launches on `stream`, with the
 * workspace in an array that is part of the library's device image (SAMP_NOALLOC_SCRATCH_BYTES per GPU, held
 * until the process ends) instead of a caller-provided buffer.  The call allocates nothing on host or device,
 * creates no stream, event or graph, and does not synchronise; the array's device address is looked up on the
 * first call per device.  SAMP_ERR_SPACE if B x S needs more workspace than the array holds (BERT-base: up to
 * about 1700 tokens; use samp_encoder_forward beyond).  All calls on one GPU share the array: calls that may
 * overlap in time (different streams, different encoders) race on it -- keep them stream-ordered.  Nothing in
 * the array needs to start at zero (every buffer in it is written before it is read within a call).
 * Not available while samp_encoder_profile timing is on.                                            */
#define SAMP_NOALLOC_SCRATCH_BYTES (32 << 20)
SAMP_API int samp_encoder_forward_noalloc(samp_encoder_t *enc, const void *hidden, const int32_t *mask, int32_t B, int32_t S,
                                          void *out, void *stream);

/* Embedding module in front of the encoder (Section 3.1: the token, segment and position embeddings
 * are summed in ONE kernel; BERT's embedding ends with a LayerNorm, which is part of it; Section 3.2:
 * when layer 0's attention block is INT8 the kernel hands int8 to the encoder directly, quantising
 * its binary32 LayerNorm value with layer 0's input step).  z = (tok[id] + seg[sid]) + pos[s] in
 * binary32, s = position inside the sequence.  All pointers are device memory, 16-byte aligned,
 * owned by the caller: tables fp16 row-major [rows, hidden], gamma / beta float [hidden].  Ids
 * outside their table are clamped into it.  Padding bytes of the struct must be zero (memset it). */
typedef struct {
    const void *token_table, *segment_table, *position_table;
    const float *gamma, *beta;
    int32_t vocab, segments, positions;   /* rows of the three tables; positions >= S */
    float ln_eps;
} samp_embedding_t;

/* samp_encoder_forward starting from ids: token_ids, segment_ids dev int32 [B,S] (segment_ids may be
 * NULL = segment 0); ids at padded positions are ignored.  Everything else as samp_encoder_forward.
 * The embedding's pointers and sizes become part of the recorded graph of this argument set.      */
SAMP_API int samp_encoder_forward_ids(samp_encoder_t *enc, const samp_embedding_t *emb, const int32_t *token_ids,
                                      const int32_t *segment_ids, const int32_t *mask, int32_t B, int32_t S, void *out,
                                      void *workspace, size_t workspace_bytes, void *stream);

/* Sequences are independent (all scales are static, Appendix B), so a forward may cut a batch
 * into up to 4 groups of sequences that run concurrently on streams owned by the encoder, forked
 * from and joined back into the caller's stream; results do not depend on the split.  groups = 0
 * (default) chooses by size (two groups from 2560 token rows on), 1 disables the split, 2..4 force it. */
SAMP_API int samp_encoder_set_groups(samp_encoder_t *enc, int32_t groups);

/* Section 3.2 hands the QKV GEMM's requantised int8 output straight to the attention; for sequences of at
 * most 256 tokens one kernel can do both per (sequence, head), so that q, k, v never reach memory and a layer
 * has one launch less (INT8 blocks with int8 softmax codes, signed or unsigned, and FP16 blocks outside calibration).
 * mode 0 (default): used where it measured faster (at least 128 (sequence, head) pairs per launch; INT8 blocks
 * up to 128 tokens, FP16 blocks up to 256); 1: never; 2: whenever the shape allows.  The context is the same
 * bytes either way.                                                                                       */
SAMP_API int samp_encoder_set_qkv_fusion(samp_encoder_t *enc, int32_t mode);

/* A forward is a few hundred short kernels, so by default the library records them once per distinct
 * argument set (pointers, B, S) into a HIP graph -- on the second call with those arguments, on a
 * stream of its own -- and replays that graph on the caller's stream afterwards.  enabled = 0 keeps
 * plain launches: choose that when the caller's stream is itself under graph capture (the plain
 * launches, events and side streams of a forward are capturable; a nested capture is not attempted).
 * Timing via samp_encoder_profile always uses plain launches.                                      */
SAMP_API int samp_encoder_set_graph(samp_encoder_t *enc, int32_t enabled);

/* Min-max calibration (Table 2 caption; Appendix B): runs the all-FP16 encoder `enc` (every mode
 * must be SAMP_FP16) on a calibration batch and returns, per layer, absmax/127 of the ten tensors
 * of samp_layer_scales_t.  Same argument rules as samp_encoder_forward; no output tensor.
 * scales_out: host [layers].  Synchronises `stream` before returning.                             */
SAMP_API int samp_encoder_calibrate(samp_encoder_t *enc, const void *hidden, const int32_t *mask, int32_t B, int32_t S,
                                    void *workspace, size_t workspace_bytes, void *stream,
                                    samp_layer_scales_t *scales_out);

/* Releases the host handle (device memory stays with the caller).  NULL is accepted.              */
SAMP_API int samp_encoder_destroy(samp_encoder_t *enc);

/* Kernel timing for benchmarks.  which = one of SAMP_PROF_*; the chosen kernel's launches inside
 * subsequent forwards get start/stop events attached to the dispatch itself; while timing is on,
 * forwards use plain launches and run their sequence groups one after another on the caller's
 * stream, so every timed launch has the device to itself.  SAMP_PROF_OFF stops.
 * samp_encoder_profile_read synchronises the events recorded so far, returns their mean duration
 * in milliseconds and their number, and clears them.                                             */
enum { SAMP_PROF_OFF = 0, SAMP_PROF_QKV = 1, SAMP_PROF_ATTN = 2, SAMP_PROF_ATTN_OUT = 3, SAMP_PROF_LN1 = 4,
       SAMP_PROF_FFN1 = 5, SAMP_PROF_FFN2 = 6, SAMP_PROF_LN2 = 7, SAMP_PROF_ENTRY = 8,
       SAMP_PROF_QKV_ATTN = 9 /* the QKV GEMM and attention in one kernel, where a forward uses it */ };
SAMP_API int samp_encoder_profile(samp_encoder_t *enc, int which);
SAMP_API int samp_encoder_profile_read(samp_encoder_t *enc, double *mean_ms, int64_t *launches);

/* Measured ceilings of the GPU the library runs on, for the benchmark's report next to the published peaks.
 * samp_probe_mfma_rate: operations per second (2 per multiply-add) of the matrix instruction the INT8 (fp16 = 0)
 * or FP16 (fp16 != 0) GEMMs are built from, issued from registers by every SIMD with no memory traffic; operands
 * all equal (random_operands = 0) or pseudo-random (the clock under matrix load depends on how many bits toggle).
 * dev_sink: 4 bytes of device memory.  samp_probe_copy_rate: bytes per second (read + written) of a plain device
 * copy of `bytes` bytes, repeated `reps` times.  samp_probe_feed_rate: bytes per second that the blocks of a
 * rows x N GEMM with 128 x 128 tiles pull into LDS when they only stream their operand stages (direct loads, 3-deep
 * ring of 128-byte stages, no matrix instruction): the operand-feed ceiling of the GEMM main loops.  operands: dev
 * buffer of at least (rows + N) * kbytes bytes (contents irrelevant); rows, N, kbytes multiples of 128.
 * All three synchronise `stream`.                                                                    */
SAMP_API int samp_probe_mfma_rate(int32_t fp16, int32_t random_operands, int32_t iters, void *dev_sink, void *stream,
                                  double *ops_per_s);
SAMP_API int samp_probe_copy_rate(const void *src, void *dst, size_t bytes, int32_t reps, void *stream, double *bytes_per_s);
SAMP_API int samp_probe_feed_rate(const void *operands, size_t bytes, int32_t rows, int32_t N, int32_t kbytes, int32_t reps,
                                  void *dev_sink, void *stream, double *bytes_per_s);

/* Thread-local description of the last failure on this thread ("" if none).                       */
SAMP_API const char *samp_last_error(void);

/* ---- choosing the per-layer modes (host functions, no GPU work) -------------------------------- */

/* Accuracy-Decay-Aware allocator (Section 3.2, Algorithm 1).  accuracy[i], latency[i], i = 0..n-1,
 * describe the settings of one mode in order of increasing number of quantised layers; setting 0
 * is all-FP16.  Latency is a time (Table 2's speedups enter as 1/speedup); both arrays are host
 * memory, finite, n in [1, 64].  Walking the settings in order, the recommended one moves to i
 * when dr = (A_i - A_rec) / (L_i - L_rec) is negative or smaller than every rate accepted before;
 * where L_i == L_rec the sign of the accuracy change decides (gain: accept, loss: reject, none:
 * skip).  *setting_out receives the index of the recommended setting.                            */
SAMP_API int samp_allocate_decay_aware(const double *accuracy, const double *latency, int32_t n, int32_t *setting_out);

/* Threshold rules (Appendix A) over the same arrays.  max_latency not NaN: the most accurate
 * setting with latency <= max_latency.  Else min_accuracy not NaN: the fastest setting with
 * accuracy >= min_accuracy.  Else up to five settings i >= 1 ranked by speedup over accuracy loss,
 * (L_0 / L_i) / (A_0 - A_i), settings that lose nothing first (by speedup).  Ties keep the setting
 * with the smaller index.  settings_out: host [capacity]; *count_out = number written (0 if no
 * setting qualifies).                                                                             */
SAMP_API int samp_recommend(const double *accuracy, const double *latency, int32_t n, double max_latency,
                            double min_accuracy, int32_t *settings_out, int32_t capacity, int32_t *count_out);

/* Downstream target (Section 3.1, "Downstream Target"): text classification on the first token of
 * every sequence of the encoder output.  logits[b, c] = W_c . tanh(W_p . hidden[b, 0, :] + b_p) + b_c
 * with binary32 accumulation.  hidden dev fp16 [B,S,H]; w_pool dev fp16 [H,H], w_cls dev fp16
 * [classes,H] (row = output channel, 16-byte aligned); b_pool, b_cls dev float; logits dev float
 * [B, classes].  H % 8 == 0, H <= 4096.                                                           */
SAMP_API int samp_classify(const uint16_t *hidden, int32_t B, int32_t S, int32_t H, const uint16_t *w_pool,
                           const float *b_pool, const uint16_t *w_cls, const float *b_cls, int32_t classes,
                           float *logits, void *stream);

/* Code-usage statistic of any int8 tensor (Appendix B compares the softmax codes with the codes of
 * the attention output): ADDS to hist[256] (dev uint64, zeroed by the caller; index = the code as
 * an unsigned byte) the number of occurrences of each code among codes[0..n).                     */
SAMP_API int samp_code_histogram(const int8_t *codes, size_t n, uint64_t *hist, void *stream);

/* Tuning aid: force the tile configuration of every GEMM launched afterwards by this process:
 * 0: 128x128 tile with 64-byte K stages, 1: 128x128 with 128-byte stages, 2: 64 tokens x 128 channels
 * (32x32 .. 64x64 per wave); the large tiles with double-buffered operand fragments, 3: 256x256 with two
 * 128-byte stages, 4: 128 tokens x 256 channels, 5: 256 tokens x 128 channels, 6: 128x192, 7: 256x256 with
 * four 64-byte stages (64x96 .. 128x128 per wave); or -1 (default) to choose by problem shape (which may
 * also take 64x96 tiles).  1..7 need operand rows that are multiples of 128 bytes (else 0 is taken), 3..7 a
 * channel count that is a multiple of their tile width (else the default choice is taken).  Results do not
 * depend on it for INT8; FP16 sums are formed in the same order in all of them.                      */
SAMP_API int samp_set_gemm_config(int32_t config);

/* ---- single steps of the path (what the encoder is made of; used by the parity tests) --------- */

/* INT8 GEMM with int32 accumulation (Section 3.2): C[M,N] = A[M,K] . W[N,K]^T, exact.
 * A, W dev int8, C dev int32.  N % 128 == 0, K % 64 == 0, M >= 1.                                 */
SAMP_API int samp_gemm_i8_i32(const int8_t *A, const int8_t *W, int32_t *C, int32_t M, int32_t N, int32_t K, void *stream);

/* INT8 GEMM + requantising epilogue: out = clamp(rne(fmaf(float(acc), m[n], b[n]))) as int8.
 * m, b dev float [N]; b may be NULL (zero).  Used for QKV (bias folded), attention-output, FFN2.  */
SAMP_API int samp_gemm_i8_requant(const int8_t *A, const int8_t *W, const float *m, const float *b, int8_t *out,
                                  int32_t M, int32_t N, int32_t K, void *stream);

/* Threshold table of the FFN1 epilogue for one output step (host function, no GPU work).  The code
 * rne(GELU(y) / s_out) is a step function of the binary32 number y alone; the table cuts the y axis
 * into uniform bins that hold at most one step each and stores, per bin, the binary32 number at which
 * the code changes and the codes on either side, found by bisection with the binary64 definition
 * below.  bin(y) = low mantissa bits of clamp(fmaf(y, rate, offset), 2^23, t_max); entry i is two
 * 32-bit words { Y_i, lo | hi << 8 }; code = y >= Y_i ? hi : lo.  host_entries: host memory of at
 * least SAMP_GELU_TABLE_BYTES, of which the first 8 * bins bytes are written (copy those to the
 * device).  SAMP_ERR_SCALE if the step would need more bins than the table holds.                  */
#define SAMP_GELU_TABLE_BYTES 16384
typedef struct { float rate, offset, t_max; int32_t bins; } samp_gelu_table_t;
SAMP_API int samp_gelu_table_build(float s_out, samp_gelu_table_t *table, void *host_entries, size_t entries_bytes);

/* INT8 GEMM + dequantise + bias + GELU + quantise (FFN1): y = fmaf(float(acc), m[n], bias[n]);
 * g = 0.5 y (1 + erf(y / sqrt 2)) in binary64, rounded once; out = clamp(rne(g * (1/s_out))).
 * table / table_entries: both NULL (GELU is evaluated per element: a certified binary32 form, and
 * binary64 where a rounding tie is near), or the description samp_gelu_table_build wrote for this
 * s_out and a dev copy of its entries, 8-byte aligned: the epilogue then looks the code up (same
 * results, a third of the vector work).  The encoder builds and uses such a table per layer.        */
SAMP_API int samp_gemm_i8_gelu_quant(const int8_t *A, const int8_t *W, const float *m, const float *bias, float s_out,
                                     const samp_gelu_table_t *table, const void *table_entries, int8_t *out, int32_t M,
                                     int32_t N, int32_t K, void *stream);

/* FP16 GEMM, binary32 accumulation: out = fp16(act(A . W^T + bias)); bias dev float [N] or NULL;
 * gelu != 0 applies GELU.  N % 128 == 0, K % 32 == 0.                                             */
SAMP_API int samp_gemm_f16(const uint16_t *A, const uint16_t *W, const float *bias, int32_t gelu, uint16_t *out,
                           int32_t M, int32_t N, int32_t K, void *stream);

/* Softmax attention over packed rows.  qkv: dev [T,3H] (int8 or fp16), columns [0,H) Q, [H,2H) K,
 * [2H,3H) V.  cu_seqlens: dev int32 [B+1], sequence b owns rows cu[b]..cu[b+1); max_len >= every
 * length, <= SAMP_MAX_SEQ.  cu_seqlens NULL: B sequences of exactly max_len rows each (T = B max_len).  INT8 flavour (Section 4.2 / Appendix B: quantised softmax output):
 * score = float(q.k) * (s_q s_k / 8); P = softmax; p_kind 0: Pq = rne(P / s_p) clamped to
 * [-127, 127]; p_kind 1: clamped to [0, 255]; ctx = rne(float(Pq.V) * s_p s_v / s_ctx).
 * p_kind 2: P is rounded to binary16 instead, ctx = rne(fl32(sum P16 V) * s_v / s_ctx), s_p is
 * ignored and p_hist must be NULL.
 * p_hist: NULL, or dev uint64 [256] to which the kernel ADDS the number of times each code byte
 * (index = the code as an unsigned byte) occurs among the softmax codes of valid query/key pairs
 * (the caller zeroes it): the code-usage statistic of Appendix B.
 * s_q * s_k / 8 must not exceed 256 (SAMP_ERR_SCALE; samp_encoder_create applies the same bound to
 * every INT8 attention block): beyond it a softmax is an argmax and the scores leave the range the
 * exponential is evaluated on.                                                                     */
SAMP_API int samp_attention_i8(const int8_t *qkv, const int32_t *cu_seqlens, int32_t B, int32_t max_len, int32_t hidden,
                               int32_t heads, float s_q, float s_k, float s_v, float s_p, float s_ctx, int32_t p_kind,
                               int8_t *ctx, uint64_t *p_hist, void *stream);
/* QKV GEMM, its requantisation and the INT8 attention (p_kind 0 or 1) of sequences of at most 256 tokens in one kernel
 * (Section 3.2: the same two steps, the q, k, v codes staying on chip): x dev int8 [T,hidden] packed rows,
 * w_qkv dev int8 [3 hidden, hidden] (rows [0,H) Q, [H,2H) K, [2H,3H) V), m and b dev float [3 hidden] as in
 * samp_gemm_i8_requant (b NULL = zeros); cu_seqlens, B, max_len <= 256, scales and ctx as in samp_attention_i8.
 * ctx equals samp_gemm_i8_requant followed by samp_attention_i8 byte for byte.                              */
SAMP_API int samp_qkv_attention_i8(const int8_t *x, const int8_t *w_qkv, const float *m, const float *b,
                                   const int32_t *cu_seqlens, int32_t B, int32_t max_len, int32_t hidden, int32_t heads,
                                   float s_q, float s_k, float s_v, float s_p, float s_ctx, int32_t p_kind, int8_t *ctx,
                                   void *stream);
/* The FP16 counterpart: out = samp_gemm_f16(x, w_qkv, bias, no GELU) followed by samp_attention_f16, in one kernel,
 * byte for byte.  x dev fp16 [T,hidden], w_qkv dev fp16 [3 hidden, hidden], bias dev float [3 hidden] or NULL.  */
SAMP_API int samp_qkv_attention_f16(const uint16_t *x, const uint16_t *w_qkv, const float *bias, const int32_t *cu_seqlens,
                                    int32_t B, int32_t max_len, int32_t hidden, int32_t heads, uint16_t *ctx, void *stream);
SAMP_API int samp_attention_f16(const uint16_t *qkv, const int32_t *cu_seqlens, int32_t B, int32_t max_len, int32_t hidden,
                                int32_t heads, uint16_t *ctx, void *stream);

/* The fused step of Section 3.2: z = deq(in) + bias + deq(res); y = LayerNorm(z; gamma, beta, eps);
 * out = quantised y (int8, step s_out) or fp16 y.  in/res/out: dev [M,H], int8 when the matching
 * *_i8 flag is set (then s_in / s_res / s_out are their steps), else fp16.  H % 16 == 0, H <= 2048. */
SAMP_API int samp_add_ln(const void *in, int32_t in_i8, float s_in, const float *bias, const void *res, int32_t res_i8,
                         float s_res, const float *gamma, const float *beta, float eps, void *out, int32_t out_i8,
                         float s_out, int32_t M, int32_t H, void *stream);

/* The decision step of the FFN1 epilogue on its own: codes[i] = clamp(rne(GELU(y[i]) / s_out)) for a
 * dev binary32 vector y of n elements; GELU in its exact-erf form.  fast (dev float [n], may be NULL)
 * receives the kernel's fast-path GELU values, whose error bound the tests verify.                 */
SAMP_API int samp_gelu_quant(const float *y, int64_t n, float s_out, int8_t *codes, float *fast, void *stream);

/* The entry quantiser on its own (Section 3.2: the producer of a quantised block's input emits INT8):
 * out[i] = clamp(rne(float(x[i]) * (1/s_x)), -127, 127) for a dev fp16 vector of n elements, n % 8 == 0;
 * x 16-byte aligned, out 8-byte aligned.  (With a mask, samp_pack_rows does the same while packing.) */
SAMP_API int samp_quantize_f16_i8(const uint16_t *x, int64_t n, float s_x, int8_t *out, void *stream);

/* Per-output-channel weight quantisation: W dev fp16 [N,K] -> Wq dev int8 [N,K], s_w dev float [N]. */
SAMP_API int samp_quantize_weight(const uint16_t *W, int32_t N, int32_t K, int8_t *Wq, float *s_w, void *stream);

/* The Embedding kernel on its own (see samp_embedding_t): out dev [B*S, H], fp16 (out_i8 == 0) or
 * int8 codes with step s_out, row b*S+s = LayerNorm(tok + seg + pos[s]).  H % 16 == 0, H <= 2048.  */
SAMP_API int samp_embed_ln(const samp_embedding_t *emb, const int32_t *token_ids, const int32_t *segment_ids, int32_t B,
                           int32_t S, int32_t H, void *out, int32_t out_i8, float s_out, void *stream);

/* Padding removal on entry (variable-length batches): packs the valid rows of hidden [B,S,H] (fp16)
 * into packed [T,H] as fp16 (s_x <= 0) or int8 codes with step s_x; writes cu_seqlens [B+1] and
 * row_map [B*S] (row_map[t] = b*S+s of packed row t).  mask as in samp_encoder_forward, not NULL.  */
SAMP_API int samp_pack_rows(const uint16_t *hidden, const int32_t *mask, int32_t B, int32_t S, int32_t H, float s_x,
                            void *packed, int32_t *cu_seqlens, int32_t *row_map, void *stream);

#ifdef __cplusplus
}
#endif
#endif /* SAMP_H */
