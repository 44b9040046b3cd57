/*
 * specsteer.h -- C ABI of the MI355X (gfx950) verify-and-recover block of
 * SpecSteer's Draft-Verify-Recover protocol.
 *
 * One call processes one drafted block for a batch of B independent
 * sequences (Algorithm 1, phase 2, the ratio test, and phase 3, the
 * recovery step):
 *
 *   for each sequence b, for t = 0 .. K_b-1 (stop at the first rejection):
 *       alpha_t = min(1, P_LLM(y_t) / (lambda * P_SLM^-(y_t)))          (Eq. 7)
 *       accept iff uniforms[b][t] <= alpha_t                            (Alg. 1)
 *   n_b = index of the first rejected position, or K_b if none
 *   h_rec = h_LLM + beta * (h_SLM^+ - h_SLM^-)   at row n_b            (Eq. 8)
 *   next_token ~ Softmax(h_rec / T), drawn by inverse CDF in vocabulary-index
 *       order from uniforms[b][k_max]: the first j whose inclusive cumulative
 *       probability exceeds the uniform (the sampling step of Algorithm 1, phase 3).
 *
 * P_x = Softmax(h_x / T) over the full vocabulary.  The paper has no
 * temperature (T = 1 is the paper); T > 0 divides all three logit tensors.
 * When every draft token is accepted (n_b == K_b) the same recovery
 * distribution, taken at the row after the last draft token, yields a bonus
 * token; the paper's loop simply re-drafts there.
 *
 * Logit layout: three tensors G (h_LLM), S_ctx (h_SLM^+), S_noctx (h_SLM^-),
 * each [B, k_max+1, V], vocabulary contiguous.  Row t is the next-token
 * distribution after the prefix plus draft tokens 0..t-1, so row t scores
 * draft[b][t] and row K_b is the bonus row.  Rows t > K_b, draft slots
 * t >= K_b and S_ctx rows other than n_b are never read.
 *
 * Pointers marked "device" must be dereferenceable by the GPU the call runs
 * on; "host" pointers are read on the CPU during the call.  No entry point
 * takes ownership of, allocates or frees any memory; none synchronises the
 * stream.  All work is enqueued on the given stream and the outputs are
 * complete when the stream reaches the end of that work.
 */
#ifndef SPECSTEER_H
#define SPECSTEER_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    SS_OK = 0,
    SS_ERR_NULL = 1,      /* a required pointer is NULL                               */
    SS_ERR_SHAPE = 2,     /* batch < 0, k_max < 0, vocab < 1 or above the limits      */
    SS_ERR_DTYPE = 3,     /* dtype is not an ss_dtype                                 */
    SS_ERR_PARAM = 4,     /* lambda, beta, temperature or flags out of range          */
    SS_ERR_STRIDE = 5,    /* strides overlap rows or are negative, or a logit pointer is off its element size */
    SS_ERR_WORKSPACE = 6, /* workspace NULL, misaligned or smaller than required      */
    SS_ERR_DEVICE = 7     /* a HIP call failed (launch error); see hipGetLastError    */
} ss_status;

typedef enum { SS_F32 = 0, SS_BF16 = 1 } ss_dtype;

#define SS_MAX_K 1024        /* largest k_max                                          */
#define SS_MAX_VOCAB (1 << 20)

typedef struct {
    int32_t batch;       /* B >= 0 (0 is a no-op)                                              */
    int32_t k_max;       /* padded draft length, 0..SS_MAX_K; logits hold k_max+1 rows         */
    int32_t vocab;       /* V, 1..SS_MAX_VOCAB                                                 */
    int32_t dtype;       /* ss_dtype of all three logit tensors                                */
    int64_t stride_b;    /* element stride between sequences; 0 => (k_max+1)*stride_t          */
    int64_t stride_t;    /* element stride between rows;      0 => vocab. Vocab stride is 1.   */
    float lambda;        /* verification threshold of Eq. 7; finite, > 0. Paper default 0.5    */
    float beta;          /* steering-recovery strength of Eq. 8; finite. Paper default 1.0     */
    float temperature;   /* T; finite, > 0. 1.0 reproduces the paper                           */
    uint32_t flags;      /* 0 or a combination of the SS_FLAG_ bits below; any other bit is an error */
} ss_params;

/*
 * Greedy decoding, the decoding setting stated in the paper's implementation-details appendix: the
 * ratio test of Eq. 7 is unchanged, but the correction / bonus token is the mode of the recovery
 * distribution, argmax_v of Eq. 8's h_rec(v) (lowest index on ties), instead of a draw;
 * uniforms[b][k_max] is not read.  h_rec is evaluated for this purpose as
 * h_LLM + beta * (h_SLM^+ - h_SLM^-) in double precision with no fused multiply-add.
 */
#define SS_FLAG_GREEDY 1u

/*
 * Algorithm 1 leaves its loop at the first rejection, so the rows of the later positions of a
 * rejected sequence never need scoring.  On large batches the block therefore scores the first
 * quarter of the positions for every sequence, applies the ratio test to them, and scores the
 * remaining positions only for the sequences that have not been rejected yet.  The outputs are
 * the same; only draft_logprobs (which asks for every position) forces the one-pass schedule.
 * SS_FLAG_FULL_ROWS forces it too: every valid row of G and S_noctx is then read.
 */
#define SS_FLAG_FULL_ROWS 2u

/*
 * Number of leading positions per sequence that the first row pass of specsteer_verify_block
 * scores for these params (host call).  Equal to k_max when the block is verified in one pass
 * (small batches, k_max < 4, SS_FLAG_FULL_ROWS; a non-NULL draft_logprobs has the same effect at
 * call time).  Returns -1 for invalid params.
 */
int specsteer_first_window(const ss_params *params);

/*
 * Bytes of device scratch specsteer_verify_block needs for these params
 * (depends on batch, k_max, vocab and dtype only).  Returns 0 if params is
 * NULL or its shape fields are invalid.  Host call, no GPU work.
 */
size_t specsteer_workspace_bytes(const ss_params *params);

/*
 * The block (Algorithm 1 phases 2-3, Eq. 7, Eq. 8; see the top of this file).
 *
 *   G, S_ctx, S_noctx  device, [B, k_max+1, V] logits of params->dtype.  With beta == 0 the
 *                      recovery distribution is Softmax(G/T) and S_ctx is not read.  Pointers
 *                      need element alignment only (SS_ERR_STRIDE otherwise) and any V works;
 *                      rows that start on 16-byte boundaries (base pointers 16-byte aligned,
 *                      strides multiples of 16 bytes) stream fastest, others cost about a
 *                      third more.
 *   draft              device, [B, k_max] int32 token ids; slots t >= K_b ignored.
 *                      May be NULL when k_max == 0.
 *   draft_len          device, [B] int32 K_b, or NULL meaning K_b = k_max for all b.
 *   uniforms           device, [B, k_max+1] fp32 in [0,1): column t < K_b drives
 *                      acceptance test t, column k_max drives the sampled token.
 *   params             host.
 *   accepted_len       device, [B] out: n_b in [0, K_b].
 *   next_token         device, [B] out: the correction token (n_b < K_b) or the
 *                      bonus token (n_b == K_b).
 *   next_token_logprob device, [B] out, or NULL: log Softmax(h_rec/T)[next_token].
 *   recovery_logprobs  device, [B, V] fp32 out, or NULL: log Softmax(h_rec/T) at row n_b.
 *   draft_logprobs     device, [B, k_max, 2] fp32 out, or NULL:
 *                      (log P_LLM(y_t), log P_SLM^-(y_t)) for every t < K_b
 *                      (also past the first rejection); 0 in padded slots.
 *   workspace          device scratch, 256-byte aligned, at least
 *                      specsteer_workspace_bytes(params) bytes; contents need no
 *                      initialisation and are garbage afterwards.  Calls that
 *                      may overlap in time need distinct workspaces.
 *   stream             a hipStream_t passed as void*; NULL is the default stream.
 *
 * Errors.  Argument errors are detected on the host before anything is
 * enqueued and leave every output untouched.  Data errors that only the GPU
 * can see -- draft_len[b] outside [0, k_max], or draft[b][t] outside [0, V)
 * for some t < K_b -- mark that sequence alone: accepted_len[b] =
 * next_token[b] = -1, next_token_logprob[b] and its draft_logprobs are NaN, its
 * recovery_logprobs row is left unwritten; no out-of-range address is ever
 * formed.  Masked tokens: a logit of -inf in G gives that token probability zero
 * (rejected if drafted, never drawn or picked); -inf in BOTH S_ctx and S_noctx at
 * a token means the specialist has nothing to say about it, and its steering term
 * in Eq. 8 is taken as 0 (not inf - inf), so a vocabulary mask shared by the three
 * models is handled.  Anything else non-finite on rows that are read (NaN, +inf,
 * -inf in only one of the specialist's rows) is unspecified but never faults.
 */
ss_status specsteer_verify_block(const void *G, const void *S_ctx, const void *S_noctx,
                                 const int32_t *draft, const int32_t *draft_len,
                                 const float *uniforms, const ss_params *params,
                                 int32_t *accepted_len, int32_t *next_token,
                                 float *next_token_logprob, float *recovery_logprobs,
                                 float *draft_logprobs, void *workspace, size_t workspace_bytes,
                                 void *stream);

/*
 * specsteer_verify_block for callers that cannot allocate device memory or hand over a workspace:
 * code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same
 * operation, arguments, outputs and errors as specsteer_verify_block, but the scratch is a
 * SS_STATIC_SCRATCH_BYTES array inside the library (one copy on every GPU the library runs on,
 * held until the process ends) and the call allocates nothing, on the host or on the device.
 * A block whose specsteer_workspace_bytes(params) exceeds SS_STATIC_SCRATCH_BYTES is refused
 * with SS_ERR_WORKSPACE before anything is enqueued (use specsteer_verify_block with a workspace
 * of your own then).  The address of the array is looked up on the first call on each device;
 * make that first call outside any stream capture.  Every call on one GPU shares that GPU's
 * array and nothing in it survives a call, so two calls that may overlap in time on one GPU
 * (two streams, two host threads) race: serialise them, or give all but one a workspace.
 */
#define SS_STATIC_SCRATCH_BYTES (8u << 20)
ss_status specsteer_verify_block_static(const void *G, const void *S_ctx, const void *S_noctx,
                                        const int32_t *draft, const int32_t *draft_len,
                                        const float *uniforms, const ss_params *params,
                                        int32_t *accepted_len, int32_t *next_token,
                                        float *next_token_logprob, float *recovery_logprobs,
                                        float *draft_logprobs, void *stream);

/*
 * Benchmark variant of specsteer_verify_block (same operation: Algorithm 1 phases 2-3,
 * Eq. 7, Eq. 8; same arguments, same outputs, same errors).  It brackets each kernel with
 * HIP events recorded on `stream`, WAITS for the last one, and writes the elapsed
 * milliseconds of each stage to the host array stage_ms[SS_NUM_STAGES]:
 *   [SS_STAGE_ROW_PASS1] log-sum-exp pass over G and S_noctx, positions [0, first window),
 *   [SS_STAGE_VERDICT]   ratio test on those positions (0 in the one-pass schedule),
 *   [SS_STAGE_ROW_PASS2] log-sum-exp pass over the remaining positions of the sequences still in
 *                        play (0 in the one-pass schedule),
 *   [SS_STAGE_RECOVER]   ratio test, first rejection, recovery distribution, sampling and the
 *                        optional log-prob rows.
 * Creates and destroys its events inside the call, so it is not for latency-critical use.
 */
#define SS_STAGE_ROW_PASS1 0
#define SS_STAGE_VERDICT 1
#define SS_STAGE_ROW_PASS2 2
#define SS_STAGE_RECOVER 3
#define SS_NUM_STAGES 4
ss_status specsteer_verify_block_timed(const void *G, const void *S_ctx, const void *S_noctx,
                                       const int32_t *draft, const int32_t *draft_len,
                                       const float *uniforms, const ss_params *params,
                                       int32_t *accepted_len, int32_t *next_token,
                                       float *next_token_logprob, float *recovery_logprobs,
                                       float *draft_logprobs, void *workspace,
                                       size_t workspace_bytes, void *stream, float *stage_ms);

/*
 * Deployment split of the recovery step (the paper's appendix on system deployment, its
 * downlink step): the cloud holds h_LLM and h_SLM^-, the edge holds h_SLM^+, and on a rejection only a
 * sparse top-k vector travels down.
 *
 * specsteer_cloud_topk -- cloud side.  For every sequence b, at row row[b] of G and S_noctx:
 *     h_cloud(v) = h_LLM(v) - beta * h_SLM^-(v)          (the non-private part of Eq. 8)
 * evaluated in double as one rounded product and one rounded difference, and its topk largest
 * entries written in order of decreasing h_cloud, ties by increasing token id:
 *   out_index  device, [B, topk] int32 token ids; -1 in slots beyond the vocabulary (V < topk)
 *   out_value  device, [B, topk] fp32  h_cloud of those tokens rounded to fp32; -inf in unused slots
 *   row        device, [B] int32 in [0, k_max] (normally accepted_len of specsteer_verify_block);
 *              a negative or too large entry marks a flagged sequence: all ids -1, values -inf.
 * Uses batch, k_max, vocab, dtype, strides, beta of params (host); 1 <= topk <= SS_MAX_TOPK
 * (the paper uses 32).  No workspace.  Argument errors as for specsteer_verify_block.
 *
 * specsteer_edge_resample -- edge side.  For every sequence, on the payload entries j:
 *     h_rec(j) = value[j] + beta * h_SLM^+(index[j])     (Eq. 8 restricted to the payload)
 * in double; tokens outside the payload have probability zero (the paper does not say; nothing
 * else can be computed from the payload); next_token is drawn from Softmax(h_rec / T) over the
 * payload by inverse CDF in payload order from uniform[b] (first j whose inclusive cumulative
 * probability exceeds it), or is the first maximum of h_rec with SS_FLAG_GREEDY (uniform may
 * then be NULL).  next_token_logprob (optional) is the log-probability under that k-way softmax.
 *   index, value  device, [B, topk] as written by specsteer_cloud_topk
 *   S_ctx         device, [B, k_max+1, V] logits of params->dtype; only the payload's tokens are read
 *   row, uniform  device, [B]
 *   next_token    device, [B] out; -1 (and NaN log-prob) for a flagged sequence or an empty payload
 * Uses batch, k_max, vocab, dtype, strides, beta, temperature, flags of params.
 */
#define SS_MAX_TOPK 64
ss_status specsteer_cloud_topk(const void *G, const void *S_noctx, const int32_t *row,
                               const ss_params *params, int32_t topk, int32_t *out_index,
                               float *out_value, void *stream);
ss_status specsteer_edge_resample(const int32_t *index, const float *value, const void *S_ctx,
                                  const int32_t *row, const float *uniform,
                                  const ss_params *params, int32_t topk, int32_t *next_token,
                                  float *next_token_logprob, void *stream);

/* Static, human-readable name of an ss_status value. */
const char *specsteer_status_string(int status);

/* Library version: major * 10000 + minor * 100 + patch. */
int specsteer_version(void);

#ifdef __cplusplus
}
#endif
#endif /* SPECSTEER_H */
