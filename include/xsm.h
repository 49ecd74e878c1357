/*
 * xsm.h - C ABI of the MI355X (gfx950) multi-head speculative decoding step.
 *
 * The library runs the inference-time hot path of XSpecMesh (arXiv 2507.23777):
 *   - the backbone decoder forward over each sequence's last accepted token plus
 *     K drafted candidates against its key-value cache, causal inside the draft
 *     block (Sec. 4.1 first paragraph, Sec. 4.2, Alg. 1 "forward with causal mask"),
 *   - the backbone distribution p^(0) = softmax(W^(0) h) (Eq. 3),
 *   - K decoding heads on the same final hidden state, head d predicting the
 *     token d+1 positions ahead (Eq. 4): the MLP head of Table 3 rows B/C,
 *     r = h + SiLU(W_d h + b_d) with logits through the shared unembedding, or
 *     the cross-attention head of rows D/E with its own unembedding W^(d),
 *   - verification: accept candidates until the first one that fails the
 *     criterion, resample K+1 tokens at the first rejected position
 *     (Sec. 4.2, Fig. 3, Alg. 1 inner loop and resample line),
 *   - cache rollback by length only (implied by Alg. 1 "s <- s*").
 * K is the paper's D.  R = K+1 rows enter the backbone per sequence and step.
 *
 * Conventions
 *   - Pointers named h_* are HOST pointers, d_* are DEVICE pointers.  Members of
 *     xsm_batch are device pointers unless stated.
 *   - The caller owns every device buffer and the stream.  The library allocates
 *     no device memory, never synchronises the stream inside a step, and keeps
 *     no per-sequence state of its own: cache lengths and draft blocks live in
 *     caller-visible device buffers.
 *   - All functions returning int return XSM_OK (0) or a negative xsm_status.
 *     On an argument error nothing is enqueued.  xsm_last_error() gives a text.
 *   - Problems only the device can see (a cache length beyond capacity, a token
 *     id outside the vocabulary, a slot out of range) never trap: the sequence is
 *     skipped for that step, n_accepted[b] = 0, and a bit is set in flags[b].
 *   - Calls on one context must not overlap in time (one stream at a time).
 */
#ifndef XSM_H
#define XSM_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define XSM_API __attribute__((visibility("default")))

typedef struct xsm_ctx xsm_ctx;              /* opaque, host-side */
typedef void* xsm_stream;                    /* a hipStream_t */

typedef enum {
  XSM_OK = 0,
  XSM_EINVAL = -1,      /* bad argument or configuration */
  XSM_ECAPACITY = -2,   /* kv_len_bound + rows per step exceeds max_ctx, or too many sequences */
  XSM_ESTATE = -3,      /* buffers not bound / weights not loaded */
  XSM_EHIP = -4,        /* a HIP runtime call failed */
  XSM_EDEVICE = -5      /* a device-side wait timed out (see xsm_check_device) */
} xsm_status;

enum { XSM_F32 = 0, XSM_BF16 = 1 };
/* Decoding-head architecture (Eq. 4; Table 3).  MLP: r = g + SiLU(W_k g + b_k), logits through
 * the shared unembedding.  CA: one multi-head cross-attention of the final hidden state g over the
 * n_cond condition tokens (keys/values W_kv,k c cached by xsm_prefill, no mask, no rotary
 * embedding, scale 1/sqrt(head_dim)), r = g + W_o,k attn(W_q,k g), logits through the head's own
 * unembedding W^(k); needs n_cond > 0. */
enum { XSM_HEAD_MLP = 0, XSM_HEAD_CA = 1 };

/* Model and capacity.  Pre-RMSNorm decoder, multi-head attention with rotary
 * embedding (pair (i, i+head_dim/2), angle pos*theta^(-2i/head_dim)), FFN
 * W2*gelu_erf(W1*x), no projection biases, untied embedding / unembedding.
 * n_heads*head_dim must equal d_model; n_draft + 1 <= 16. */
typedef struct {
  int32_t n_layers, d_model, n_heads, head_dim, d_ffn, vocab;
  int32_t n_draft;                /* K: decoding heads = candidates per step */
  int32_t max_batch;              /* cache slots = max sequences per call */
  int32_t max_ctx;                /* cache positions per slot (prefix + generated + K+1) */
  int32_t n_cond;                 /* cross-attention condition tokens per sequence, 0 = none */
  int32_t dtype;                  /* XSM_F32 | XSM_BF16: storage of weights, cache, embeddings */
  float rope_theta, rms_eps;
  int32_t head_kind;              /* XSM_HEAD_MLP | XSM_HEAD_CA */
} xsm_config;

/* Acceptance criterion and sampling rule (Sec. 5.4 "Verification criterion";
 * appendix "Independent Sampling"). */
enum { XSM_VERIFY_GREEDY = 0, XSM_VERIFY_TOPK = 1, XSM_VERIFY_THRESHOLD = 2 };
typedef struct {
  int32_t mode;          /* GREEDY: candidate == argmax p^(0) (top-K_a with K_a = 1);
                            TOPK: candidate among the top_ka largest logits, equal logits
                            ordered by lower index; THRESHOLD: softmax(z/T)[x] > delta, strict */
  int32_t top_ka;
  float delta;
  float temperature;     /* T > 0, used by THRESHOLD and by categorical sampling */
  int32_t sample;        /* 0: argmax (lowest index among equal maxima); 1: categorical over the
                            full vocabulary by inverse CDF in ascending token order, weights
                            exp((z - max z)/T), uniform u = (x0 >> 8) * 2^-24 with
                            x = Philox4x32-10(counter = (position, head, slot, 0), key = seed);
                            2: top-K_s probability-tree sampling of the K head tokens (appendix
                            "Sampling strategies"): level d = the top_ks most probable tokens of
                            softmax(z_d/T) (equal ones by lower index) with their probabilities as
                            edge weights, paths whose weight falls below pts_prune are cut, one
                            surviving path is drawn in proportion to its weight by inverse CDF in
                            depth-first order with one uniform (head coordinate 254); no survivor:
                            every head's most probable token.  The backbone token is drawn as
                            under 1.  Needs 1 <= top_ks <= 4 and top_ks^K <= 4096. */
  uint64_t seed;
  int32_t top_ks;        /* K_s (sample == 2) */
  float pts_prune;       /* path-weight cut-off (sample == 2); the paper uses 1e-5 */
} xsm_verify_params;

/* flags[b] bits */
enum {
  XSM_FLAG_NEAR_TIE = 1u,     /* some decision of this step was close to flipping: an argmax or
                                 rank-boundary logit margin <= 1e-2, T |ln(p / delta)| <= 1e-2 under
                                 the threshold criterion (the logit change that would flip it),
                                 a draw's uniform within 2e-5 (of the total
                                 weight) of an inverse-CDF edge, or a probability-tree path within
                                 1e-4 (relative) of the cut-off */
  XSM_FLAG_BAD_LEN = 2u,      /* kv_len[b] < 0 or kv_len[b] + rows > max_ctx or > kv_len_bound */
  XSM_FLAG_BAD_TOKEN = 4u,    /* a block token outside [0, vocab) */
  XSM_FLAG_BAD_SLOT = 8u,     /* slot[b] outside [0, max_batch) */
  XSM_FLAG_DEVICE_TIMEOUT = 16u /* a bounded device-side wait of the single-launch step gave up, in
                                 this step or an earlier one: the sequence produced nothing
                                 (n_accepted[b] = 0, block / kv_len / out_tokens untouched); see
                                 xsm_check_device */
};

/* One call's worth of sequences.  R = n_draft + 1 for xsm_spec_step, 1 for
 * xsm_plain_step.  block[b][0] is the last accepted token (not yet cached) at
 * absolute position kv_len[b]; block[b][1..] are the candidates. */
typedef struct {
  int32_t n_seq;               /* host value, 1..max_batch */
  int32_t kv_len_bound;        /* host value: upper bound of all kv_len[b] on entry */
  const int32_t* slot;         /* [n_seq] cache slot of each sequence (distinct) */
  int32_t* kv_len;             /* [n_seq] in/out: cached positions; += n_accepted */
  int32_t* block;              /* [n_seq][R] in: draft block; out: next draft block */
  int32_t* out_tokens;         /* [n_seq][R] out: accepted tokens, first n_accepted[b] valid */
  int32_t* n_accepted;         /* [n_seq] out: 1..R (0 if the sequence was skipped) */
  uint32_t* flags;             /* [n_seq] out */
  float* logits_dbg;           /* optional [n_seq][R][vocab]: backbone logits, NULL in production */
  float* head_logits_dbg;      /* optional [n_seq][K][vocab]: head logits at the accepted row */
} xsm_batch;

/* Validate cfg and create a context.  No device work. */
XSM_API int xsm_create(const xsm_config* cfg, xsm_ctx** out);
XSM_API void xsm_destroy(xsm_ctx* ctx);
XSM_API const char* xsm_last_error(const xsm_ctx* ctx);      /* ctx may be NULL: creation errors */

/* Sizes of the three caller-allocated device buffers (256-byte aligned). */
XSM_API size_t xsm_weights_bytes(const xsm_ctx* ctx);        /* weights in library layout + tables */
XSM_API size_t xsm_kv_bytes(const xsm_ctx* ctx);             /* self- and cross-attention caches */
XSM_API size_t xsm_workspace_bytes(const xsm_ctx* ctx);      /* per-step activations and partials */
XSM_API size_t xsm_canonical_weight_elems(const xsm_ctx* ctx); /* elements in the canonical weight file */
/* Bind the three buffers (device pointers, owned by the caller, alive until xsm_destroy).  Call
 * with the buffers' device current: the device's compute-unit count is read here (the
 * single-launch step needs 256 units, one per workgroup; smaller devices and partitions take the
 * per-stage kernels).  XSM_EINVAL on a null or misaligned pointer. */
XSM_API int xsm_bind(xsm_ctx* ctx, void* d_weights, void* d_kv, void* d_workspace);

/* Upload the model (Sec. 4.1: the backbone's decoder blocks and W^(0) of Eq. 3; Sec. 4.2, Eq. 4: the D
 * decoding heads).  h_canonical: host array of n_elems elements of cfg.dtype
 * (bf16 bit patterns or float), all matrices [out][in] row-major, in this order:
 * E[V][d]; per layer g1[d], Wqkv[3d][d] (q rows, k rows, v rows), Wo[d][d],
 * (if n_cond: gc[d], Wcq[d][d], Wckv[2d][d], Wco[d][d]), g2[d], W1[F][d], W2[d][F];
 * gf[d]; WU[V][d]; per head Wh[d][d], bh[d] (XSM_HEAD_MLP) or Wq[d][d], Wkv[2d][d] (key rows,
 * value rows), Wo[d][d], WU_k[V][d] (XSM_HEAD_CA).  Copies to the device, re-lays the
 * matrices for the kernels and builds the rotary table, all on `stream`; the host
 * array may be reused once the stream has been synchronised. */
XSM_API int xsm_load_weights(xsm_ctx* ctx, const void* h_canonical, size_t n_elems, xsm_stream stream);

/* Condition prefill (Sec. 4.1: generation is conditioned on c, and the decoder attends to the
 * cached x_0..x_{s-1}; Alg. 1 starts from that state): run the backbone over P prefix embeddings
 * per sequence (used directly as layer-0 hidden states at positions 0..P-1, full causal mask)
 * filling the cache of slot h_slot[i]; with n_cond > 0 also project the condition tokens to every
 * layer's cross-attention keys/values (and to the cross-attention heads' own, Eq. 4).
 * d_prefix_emb: [n_seq][P][d] of cfg.dtype (may be NULL when P == 0); d_cond:
 * [n_seq][n_cond][d] of cfg.dtype (NULL when n_cond == 0).  Cache lengths belong to the caller
 * (xsm_batch.kv_len is a caller-owned device array the library only reads and advances in a
 * step): the prefill writes cache positions 0..P-1 and no length, and the caller sets
 * kv_len[b] = P for these sequences before their first step.  h_slot is a host array, read
 * before the call returns.  Enqueues on `stream`, does not synchronise. */
XSM_API int xsm_prefill(xsm_ctx* ctx, int32_t n_seq, const int32_t* h_slot, const void* d_prefix_emb,
                int32_t P, const void* d_cond, xsm_stream stream);

/* One speculative step (one iteration of Alg. 1's outer loop) for every sequence
 * of the batch: accepted tokens, their count, the next draft block and the new
 * cache length are written to the batch's device arrays.  A step only enqueues
 * kernels on `stream` (no allocation, copy, memset or synchronisation), and its
 * state between calls (lengths, blocks, the step epoch) lives on the device, so
 * a caller may capture it in a HIP graph after one eager call; the graph then
 * repeats the call with the n_seq, kv_len_bound, parameters and options of the
 * capture. */
XSM_API int xsm_spec_step(xsm_ctx* ctx, const xsm_batch* batch, const xsm_verify_params* vp,
                  xsm_stream stream);

/* Next-token decoding (the non-speculative comparison, Table 3 row A): block is
 * [n_seq][1], one token is sampled from p^(0) and written to out_tokens / block. */
XSM_API int xsm_plain_step(xsm_ctx* ctx, const xsm_batch* batch, const xsm_verify_params* vp,
                   xsm_stream stream);

/* xsm_spec_step for callers that cannot allocate device memory or be handed a workspace: code
 * under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same
 * arguments, same outputs (the per-stage kernels of xsm_spec_step, same arithmetic in the same
 * order), but the step's activations, partial products and arrival counters live in a scratch
 * array that is part of the library image (64 MiB of device memory per GPU, held from the time
 * the library is loaded until the process ends) instead of the bound workspace, which this
 * call neither reads nor writes.  Weights and cache are the bound buffers (xsm_bind looks the
 * array's address up for its device; call with that device current).  The call allocates
 * nothing, copies nothing and does not synchronise; it enqueues kernels only.
 * XSM_ECAPACITY when the configuration's steps need more than the 64 MiB (the need grows with
 * max_batch: 6 MB for a 24-layer d = 1024 model at max_batch 1, 45 MB at max_batch 16 with K = 6,
 * 72 MB at max_batch 32 with K = 8, which is refused; then use xsm_spec_step).  Every call on a GPU, from any context, shares that GPU's one array, which
 * keeps the last call's contents (the call clears what must start at zero): calls that overlap
 * in time on one GPU race, so order them on one stream or with events. */
XSM_API int xsm_spec_step_static(xsm_ctx* ctx, const xsm_batch* batch, const xsm_verify_params* vp,
                                 xsm_stream stream);

/* Options.  XSM_OPT_SINGLE_LAUNCH (default 1): when a step has at most 16 block rows in total,
 * the model shape is supported and the device has 256 compute units, run the whole step (backbone,
 * heads, unembedding, verification under any criterion, draws under any sampling rule, emit) as
 * one persistent kernel instead of one kernel per stage; 0 forces the per-stage kernels.  XSM_OPT_ATTN_SPLITS (tuning aid, default 0 = automatic): key-range slices per
 * (sequence, head) of the attention kernel / stage (the single-launch step takes the largest power
 * of two not above it).  XSM_OPT_PREFILL_ROWS (tuning aid, default 0 = as many as the workspace
 * holds, 8192): upper limit of the rows (sequences x positions) one prefill pass takes. */
enum { XSM_OPT_SINGLE_LAUNCH = 1, XSM_OPT_TIMELINE = 2, XSM_OPT_ATTN_SPLITS = 3, XSM_OPT_PREFILL_ROWS = 4 };
XSM_API int xsm_set_option(xsm_ctx* ctx, int32_t option, int32_t value);

/* Tuning aid.  With XSM_OPT_TIMELINE = 1 every workgroup of the single-launch step stamps the
 * device's 100 MHz clock at its stage boundaries; this copies the stamps of the last step to
 * h_out as [256 workgroups][n_layers*16 + 8] words (synchronises the device). */
XSM_API int xsm_debug_timeline(xsm_ctx* ctx, uint64_t* h_out, size_t n_words);

/* Synchronises the device and reports whether a bounded device-side wait of the
 * single-launch step gave up since the last call (XSM_EDEVICE, reported once).  The step in
 * which that happened, and every single-launch step enqueued after it, wrote n_accepted[b] = 0
 * and XSM_FLAG_DEVICE_TIMEOUT for the sequences it could not finish and left their block,
 * kv_len and out_tokens untouched, so a caller that reads a step's outputs sees the failure
 * without this call.  After the report this context's steps run on the per-stage kernels
 * (until weights are loaded again): repeat the lost step.  XSM_OK otherwise. */
XSM_API int xsm_check_device(xsm_ctx* ctx);

/* Test only, synchronous: set the single-launch step's device-side error word as a timed-out
 * wait would (no wait is made to spin), so that the failure path above can be exercised. */
XSM_API int xsm_debug_inject_device_error(xsm_ctx* ctx, uint32_t code);

/* Test/bench only, synchronous (they synchronise the device): copy cache rows of
 * one layer/slot to or from a host float array [n_heads][n_pos][head_dim].
 * which: 0 keys, 1 values, 2 cross-attention keys, 3 cross-attention values. */
XSM_API int xsm_debug_kv_export(xsm_ctx* ctx, int32_t layer, int32_t which, int32_t slot, int32_t pos0,
                        int32_t n_pos, float* h_out);
XSM_API int xsm_debug_kv_import(xsm_ctx* ctx, int32_t layer, int32_t which, int32_t slot, int32_t pos0,
                        int32_t n_pos, const float* h_in);

/* Test only, synchronous: copy every layer's cache contents (self- and cross-attention) of
 * slot src to slot dst, device to device. */
XSM_API int xsm_debug_kv_clone(xsm_ctx* ctx, int32_t src_slot, int32_t dst_slot);

/* Benchmark only: per-kernel timing with HIP events recorded on the launch stream around
 * every kernel the library enqueues (process-wide switch, off by default; adds two event
 * records per launch).  xsm_debug_trace_report synchronises the device, writes one text line
 * "kernel_class count total_ms" per class into h_buf (NUL-terminated, at most cap bytes),
 * clears the records and returns the number of classes (negative on a HIP error). */
XSM_API void xsm_debug_trace_enable(int on);
XSM_API int xsm_debug_trace_report(char* h_buf, size_t cap);

#ifdef __cplusplus
}
#endif
#endif /* XSM_H */
