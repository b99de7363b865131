/*
 * eh.h -- C ABI of libeh: early-exit head evaluation and DSSD greedy
 * verification on one AMD MI355X (gfx950).
 *
 * Method: arXiv 2407.21082, "Accelerating Large Language Model Inference with
 * Dynamic Self-Speculative Decoding".  Section numbers below refer to it.
 *
 * General conventions
 *   - Every entry point returns an eh_status and never throws or aborts.
 *     Argument errors are detected on the host before anything is launched.
 *   - "device" pointers are HIP device memory on the context's device; "host"
 *     pointers are ordinary process memory.  The library never takes ownership
 *     of a caller buffer.  Inputs and outputs of an asynchronous call must stay
 *     alive and untouched until the stream has passed the call.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).
 *     All work of a call is enqueued on it; calls do not synchronise the host.
 *   - A context serialises its calls: it owns one workspace, so two calls on
 *     the same context must be ordered on the same stream (or by the caller).
 *   - A row whose hidden state contains NaN or Inf has NaN statistics (every
 *     logit is NaN) and argmax / token / target -1; it never passes the exit test
 *     and so leaves at the last head.  This is defined behaviour, not an error.
 *     Weights, gamma and beta must be finite.
 *   - Two kinds of call run a persistent kernel whose workgroups wait for each
 *     other, one workgroup per compute unit: every call with at most 16 rows (heads
 *     without a bias vector, d up to 2048 for bf16 / 1024 for fp32), and eh_cascade
 *     and dssd_verify with up to 256 rows that the first kind does not serve (bf16
 *     heads without a bias vector: 17 to 256 rows, and fewer at d above 2048).  The
 *     stream must have the device to itself while such a call runs (no other kernel
 *     holding compute units on another stream or from another context).  eh_create
 *     checks that the grids fit the empty device.  Every wait is bounded
 *     (eh_set_spin_limit); a call that gives up sets a flag that eh_check reports
 *     and clears, rows it did not finish read -1 / NaN, and the context stays usable.
 *     Such a launch also carries a tag (and, for dssd_verify, a choice of control
 *     block) that the host advances with every call, so these calls must be made
 *     anew each time: recording one into a HIP graph and replaying the graph is not
 *     supported.  eh_eval, eh_eval_heads, eh_eval_heads_metrics and eh_exit_decide
 *     with more than 16 rows, and eh_eval_noalloc with any number, carry no such state.
 */
#ifndef EH_H_
#define EH_H_

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct eh_ctx eh_ctx; /* opaque, owned by the library */

typedef enum {
  EH_OK = 0,
  EH_ERR_NULL = 1,      /* a required pointer is NULL                        */
  EH_ERR_SHAPE = 2,     /* a size is non-positive or inconsistent            */
  EH_ERR_DTYPE = 3,     /* unsupported dtype combination                     */
  EH_ERR_RANGE = 4,     /* index (head, n_rows, k ...) outside its range     */
  EH_ERR_HIP = 5,       /* a HIP runtime call failed (see eh_last_error)     */
  EH_ERR_WORKSPACE = 6  /* request exceeds the workspace sized at creation   */
} eh_status;

typedef enum { EH_F32 = 0, EH_BF16 = 1 } eh_dtype;

/*
 * Description of a stack of exit heads (Section 3.1 "Early exit heads",
 * Section 3.2: each head has the structure of the model's final classification
 * head; here LayerNorm(gamma, beta, eps) followed by a d -> V linear map).
 * Head n_heads-1 stands for the full model's own head: it always answers.
 *
 * W[l]      device, [V, d] row-major, dtype w_dtype.  Copied (re-tiled into the
 *           matrix-core operand order) at creation; the caller may free it
 *           after eh_create returns.
 * gamma[l], beta[l]   device, [d] float.  Copied at creation.
 * bias      NULL, or n_heads device pointers [V] float added to the logits.
 * tau       host, [n_heads] float, thresholds in nats (Section 3.4.1); the last
 *           entry is ignored.  Copied.
 * w_dtype must equal h_dtype.  In EH_BF16 mode the LayerNorm output is rounded
 * to bf16 (nearest even) before the projection; products are exact and sums
 * are accumulated in fp32.
 */
typedef struct {
  int32_t d;         /* hidden size, > 0                                       */
  int32_t V;         /* vocabulary size, > 0                                   */
  int32_t n_heads;   /* >= 1, includes the final head                          */
  int32_t max_rows;  /* largest n_rows any call will pass, >= 1                */
  int32_t w_dtype;   /* eh_dtype of W                                          */
  int32_t h_dtype;   /* eh_dtype of hidden states                              */
  float ln_eps;      /* LayerNorm epsilon (> 0; 1e-5 for the Pythia family)    */
  int32_t device;    /* HIP device ordinal                                     */
  const void* const* W;
  const float* const* gamma;
  const float* const* beta;
  const float* const* bias;
  const float* tau;
} eh_config;

/* Creates a context on cfg->device (made current for the call and restored).
 * The caller must have finished writing the weight buffers; the copies are
 * complete when the call returns.  *out is NULL on error. */
eh_status eh_create(const eh_config* cfg, eh_ctx** out);

/* Frees everything the context owns.  Synchronises the device first. */
eh_status eh_destroy(eh_ctx* ctx);

/*
 * One head on a set of rows (Sections 3.2 and 3.4.1): for each row, LayerNorm,
 * projection to V logits, and the entropy H = -sum p log p (nats), the
 * log-sum-exp and the argmax (lowest index on ties) of the softmax over the
 * logits.  The logits are never written to memory.
 *
 * head          0 <= head < n_heads
 * h             device, rows of d elements (h_dtype); row r starts at element
 *               r * h_row_stride (h_row_stride >= d)
 * row_idx       device [n_rows] or NULL.  If given, output position p reads
 *               input row row_idx[p] (gather after compaction); else row p.
 * n_rows_dev    device int32 or NULL.  If given, the number of live rows is
 *               read from it on the device (0 <= *n_rows_dev <= n_rows) and
 *               output positions beyond it are left untouched.
 * n_rows        host upper bound on rows, 0 <= n_rows <= max_rows (0 = no-op)
 * H, lse, argmax  device [n_rows] outputs (float, float, int32); any may be
 *               NULL.  Indexed by output position p.
 */
eh_status eh_eval(eh_ctx* ctx, int32_t head, const void* h, int64_t h_row_stride,
                  const int32_t* row_idx, const int32_t* n_rows_dev, int32_t n_rows,
                  float* H, float* lse, int32_t* argmax, void* stream);

/*
 * eh_eval for callers that cannot allocate or free device memory around the call: code
 * under HIP graph capture, tight serving loops, harnesses that forbid allocation.  Same
 * arguments, same results (the same kernels, at any row count: this call does not use the
 * persistent kernel), but the call's workspace -- the normalised activations and the partial
 * statistics of the workgroups -- is a 16 MiB array that is part of the library's image on
 * each GPU, not memory of the context, and the call performs no allocation of any kind.
 *
 * n_rows        0 <= n_rows, not bounded by max_rows but by the array: EH_ERR_WORKSPACE if
 *               (ceil32(n_rows) / 16 + 32) * ceil(d / k) KiB + 10 KiB * ceil32(n_rows)
 *               exceeds 16 MiB (k = 32 for bf16, 16 for fp32): up to 1024 rows at d = 2048 bf16, 896 at
 *               d = 2560.
 * Every call on a GPU, from any context, shares that GPU's array and finds the last call's
 * contents in it (nothing in it has to start at zero): calls that overlap in time on one GPU
 * race, so order them on one stream or by events.
 */
eh_status eh_eval_noalloc(eh_ctx* ctx, int32_t head, const void* h, int64_t h_row_stride,
                          const int32_t* row_idx, const int32_t* n_rows_dev, int32_t n_rows,
                          float* H, float* lse, int32_t* argmax, void* stream);

/*
 * Several heads on the same positions in one call (Section 3.4.1, "Calibration of
 * Confidence Thresholds": the confidence of every head is needed at every token of
 * the calibration set).  Same results as eh_eval for heads head0 .. head0 +
 * n_heads_eval - 1, but the LayerNorm of all heads runs as one launch and so do
 * their projections (bf16 heads, more than 16 rows) and the final merge, which
 * takes about 15 us per head off a 512-row batch.
 *
 * h_layers      device; head head0 + l reads row r at element
 *               l * layer_stride + r * row_stride
 * n_rows        0 <= n_rows <= max_rows (0 = no-op)
 * H, lse, argmax  device [n_heads_eval, n_rows] outputs, row-major; any may be NULL
 * The first call (and any later call with more heads) allocates a workspace of
 * n_heads_eval * (max_rows * d * element size + 10 KiB * max_rows) bytes that the
 * context keeps until eh_destroy, and synchronises the device to do so.
 */
eh_status eh_eval_heads(eh_ctx* ctx, int32_t head0, int32_t n_heads_eval, const void* h_layers,
                        int64_t layer_stride, int64_t row_stride, int32_t n_rows, float* H,
                        float* lse, int32_t* argmax, void* stream);

/*
 * eh_eval_heads plus the two other confidence metrics of Section 3.4.1
 * ("Calibration of Confidence Thresholds": maximum probability and the difference
 * between the two largest probabilities, "breaking ties"), for comparing them
 * with the entropy on a calibration set.  bf16 heads without a bias vector only
 * (EH_ERR_DTYPE otherwise); any 1 <= n_rows <= max_rows.
 *
 * max_prob, margin   device [n_heads_eval, n_rows] float, either may be NULL:
 *               max_j p_j, and the largest minus the second largest probability
 *               (0 on a tie at the top; the largest probability itself if V = 1)
 * Everything else as in eh_eval_heads.
 */
eh_status eh_eval_heads_metrics(eh_ctx* ctx, int32_t head0, int32_t n_heads_eval, const void* h_layers,
                                int64_t layer_stride, int64_t row_stride, int32_t n_rows, float* H,
                                float* lse, int32_t* argmax, float* max_prob, float* margin,
                                void* stream);

/*
 * Exit rule for one head (Section 3.4.2; entropy form of Section 4.3.1,
 * "Drafting phase") followed by compaction of the rows that go on.
 *
 * Position p (p < live rows) describes row r = row_idx ? row_idx[p] : p.
 * If H[p] < tau[head], or head == n_heads-1, the row exits here:
 * exit_layer[r] = head, token[r] = argmax[p].  Otherwise r is appended to
 * active_idx_out, which keeps the input order (stable), and the number of
 * survivors is written to *n_active_out.
 *
 * H, argmax          device [n_rows], outputs of eh_eval for the same positions
 * exit_layer, token  device, indexed by row r, in-out (caller initialises to -1)
 * active_idx_out     device [n_rows]; may alias nothing else
 * n_active_out       device int32
 */
eh_status eh_exit_decide(eh_ctx* ctx, int32_t head, const float* H, const int32_t* argmax,
                         const int32_t* row_idx, const int32_t* n_rows_dev, int32_t n_rows,
                         int32_t* exit_layer, int32_t* token, int32_t* active_idx_out,
                         int32_t* n_active_out, void* stream);

/*
 * Whole dynamic-exit cascade for n_rows independent rows (Section 3.4.2): heads
 * 0..n_heads-1 in order, each evaluated only on the rows that have not exited,
 * with no host synchronisation between heads.  Equivalent to calling eh_eval
 * and eh_exit_decide per head with the active list carried on the device.
 *
 * h_layers      device; head l reads row r at element
 *               l * layer_stride + r * row_stride
 * exit_layer, token   device [n_rows] outputs (need no initialisation)
 * H_out         NULL or device [n_heads, n_rows] float: entropy of every
 *               evaluated (head, row); entries never evaluated are set to NaN
 * n_evals_out   NULL or device int64: incremented by the number of
 *               (row, head) evaluations performed
 */
eh_status eh_cascade(eh_ctx* ctx, const void* h_layers, int64_t layer_stride,
                     int64_t row_stride, int32_t n_rows, int32_t* exit_layer,
                     int32_t* token, float* H_out, int64_t* n_evals_out, void* stream);

/*
 * DSSD greedy verification (Section 4.3.1, "Verification phase").
 *
 * f_final    device [B, k+1, d] (h_dtype, contiguous): the full model's final
 *            hidden state at the position preceding draft token j (j < k) and
 *            after the last draft token (j = k)
 * draft      device [B, k] int32 drafted tokens
 * draft_len  device [B] int32 (0 <= draft_len[b] <= k) or NULL (= k)
 * accepted   device [B]: length of the longest prefix with
 *            draft[b, j] == target[b, j], bounded by draft_len[b]
 * next_token device [B]: target[b, accepted[b]] -- the full-model token that
 *            replaces the first mismatch, or the bonus token
 * target     NULL or device [B, k+1]: the final head's argmax at every position
 * Requires B * (k+1) <= max_rows.  Uses head n_heads-1.
 */
eh_status dssd_verify(eh_ctx* ctx, const void* f_final, const int32_t* draft,
                      const int32_t* draft_len, int32_t B, int32_t k, int32_t* accepted,
                      int32_t* next_token, int32_t* target, void* stream);

/*
 * DSSD drafting phase (Section 4.3.1, "Drafting phase") for one sequence, without a
 * host round trip: position after position the exit heads are tried from the
 * shallowest to the deepest and the first with H < tau drafts its token, which is
 * appended to the draft buffer; drafting stops when the buffer holds `limit` tokens
 * (EH_DRAFT_LIMIT), right after an end-of-sequence token was appended
 * (EH_DRAFT_EOS), at a position where no exit head is confident (EH_DRAFT_FALLBACK:
 * nothing is appended, the last head's -- the model's own -- prediction there is
 * reported), or when the positions run out (EH_DRAFT_EXHAUSTED).  The hidden
 * states of every position are supplied by the caller (the backbone is not part of
 * this library; in a real decoder position t depends on the token drafted at t-1,
 * so a caller drafts with n_positions = 1 per backbone step, or with as many
 * positions as its backbone has produced).  Once drafting has stopped the
 * remaining launches of the call return at once on the device.
 *
 * h_positions   device; position t, head l: d elements (h_dtype) at element
 *               t * pos_stride + l * layer_stride
 * n_positions   positions available, >= 0; limit  buffer size, >= 0
 * eos_token     token id that ends the draft (pass -1 for none)
 * draft         device [limit] int32: the drafted tokens (first *draft_len valid)
 * draft_len     device int32
 * exit_layers   device [limit] int32: the head that drafted each token, -1 beyond
 * stop_reason, fallback_token   device int32, nullable; fallback_token is -1 unless
 *               the reason is EH_DRAFT_FALLBACK
 * n_evals_out   NULL or device int64, incremented by the (position, head)
 *               evaluations performed
 * Needs one of the single-launch cascade kernels (heads without a bias vector; fp32
 * heads up to d = 1024); EH_ERR_DTYPE otherwise.
 */
enum { EH_DRAFT_LIMIT = 0, EH_DRAFT_EOS = 1, EH_DRAFT_FALLBACK = 2, EH_DRAFT_EXHAUSTED = 3 };
eh_status dssd_draft(eh_ctx* ctx, const void* h_positions, int64_t pos_stride, int64_t layer_stride,
                     int32_t n_positions, int32_t limit, int32_t eos_token, int32_t* draft,
                     int32_t* draft_len, int32_t* exit_layers, int32_t* stop_reason,
                     int32_t* fallback_token, int64_t* n_evals_out, void* stream);

/*
 * Verification bookkeeping (Section 4.3.1, "Verification phase"; the acceptance
 * rate and the discarded tokens of Section 4.3.2): adds a batch of B verification
 * rounds to five running counters on the device,
 *   counters[0] += B                       rounds
 *   counters[1] += sum_b len_b             tokens drafted
 *   counters[2] += sum_b accepted_b        tokens committed from the drafts
 *   counters[3] += sum_b (len_b - accepted_b)   tokens drafted for nothing
 *   counters[4] += sum_b sum_{j < len_b} exit_layers[b, j]   (0 if exit_layers is NULL)
 * so that counters[2] / counters[1] is the acceptance rate, counters[2] /
 * counters[0] the mean accepted tokens per round and counters[4] / counters[1] the
 * mean exit head during drafting.  The caller zeroes the counters to start.
 *
 * draft_len    NULL (every round drafted k tokens) or device [B] int32, clamped to [0, k]
 * accepted     device [B] int32 (dssd_verify's output), clamped to [0, len_b]
 * exit_layers  NULL or device [B, k] int32 (row-major), read only below len_b
 * counters     device [5] int64
 */
enum { EH_TALLY_ROUNDS = 0, EH_TALLY_DRAFTED = 1, EH_TALLY_ACCEPTED = 2, EH_TALLY_WASTED = 3,
       EH_TALLY_LAYER_SUM = 4, EH_TALLY_COUNT = 5 };
eh_status dssd_tally(eh_ctx* ctx, const int32_t* draft_len, const int32_t* accepted, int32_t B, int32_t k,
                     const int32_t* exit_layers, int64_t* counters, void* stream);

/*
 * The training objectives of Section 3.3 ("Losses") for one exit head on a sequence
 * of n_rows tokens, forward only, without materialising either distribution: the
 * head (LayerNorm + projection on h_head) and the model's own head (the context's
 * last head, on h_model) are projected together and, per token t,
 *   kl[t] = sum_v y_hat_v log(y_hat_v / f_v)    y_hat = softmax(head), f = softmax(model)
 *   ce[t] = -log y_hat_{labels[t]}              (NaN without labels or for a label outside [0, V))
 * are accumulated on the fly;  loss[0] = L_CE = mean ce, loss[1] = L_KL = mean kl,
 * loss[2] = L_hyb = alpha * L_CE + (1 - alpha) * L_KL.
 *
 * h_head, h_model   device, n_rows rows of d elements (h_dtype), row strides in elements
 * labels            NULL or device [n_rows] int32
 * kl, ce            NULL or device [n_rows] float
 * loss              device [3] float
 * bf16 heads without a bias vector only (EH_ERR_DTYPE otherwise); 1 <= n_rows <= max_rows.
 * The first call allocates its workspace in the context (and synchronises the device).
 */
eh_status eh_head_losses(eh_ctx* ctx, int32_t head, const void* h_head, int64_t row_stride_head,
                         const void* h_model, int64_t row_stride_model, const int32_t* labels,
                         int32_t n_rows, float alpha, float* kl, float* ce, float* loss, void* stream);

/*
 * Threshold calibration of one head (Section 3.4.1, "Calibration of Confidence
 * Thresholds"), entropy as the confidence metric: the M calibration tokens are
 * ordered by ascending confidence (descending entropy); for a level epsilon the
 * threshold is the entropy of the first token in that order such that, among all
 * tokens at least as confident, the proportion whose prediction equals the
 * model's (eq. (2)) is at least epsilon.  Tokens with equal entropy are taken as
 * a whole; NaN entropies are ignored; if no token qualifies tau = -inf (the head
 * never exits).  The value returned is the paper's tau, to be used as
 * "exit if H <= tau"; eh_exit_decide tests H < tau, so pass nextafterf(tau, +inf)
 * there to let the boundary token exit as well.
 *
 * H            device [M] float, e.g. one row of eh_eval_heads' output
 * pred, ref    device [M] int32: the head's and the full model's argmax
 * M            0 <= M < 2^31
 * eps          host [n_eps] double, each in [0, 1]; 0 <= n_eps <= 64
 * tau_out      device [n_eps] float
 * n_exit_out   NULL or device [n_eps] int64: tokens with H <= tau
 * The call waits for `stream` before it returns: it finds the thresholds by counting
 * the tokens into bins in three levels, keeping at each level only the bins that can
 * still hold an answer, and reads one word back to learn whether its tables of kept
 * bins were large enough.  They are unless the proportion stays within a hair of a
 * level over a wide range of thresholds (or M > 2^27); the call then sorts all tokens
 * instead.  The results are the same either way, and are complete in tau_out and
 * n_exit_out when the call returns.  Uses about 5.2 * M bytes + 8 MiB of scratch
 * memory (20 * M when it sorts) that the context keeps until eh_destroy; a call that
 * needs more than any before grows it, which synchronises the device.
 */
eh_status eh_calibrate(eh_ctx* ctx, const float* H, const int32_t* pred, const int32_t* ref, int64_t M,
                       const double* eps, int32_t n_eps, float* tau_out, int64_t* n_exit_out,
                       void* stream);

/*
 * Waits for `stream` and reports failures that only the device can see: the
 * persistent kernels (calls with at most 16 rows; eh_cascade and dssd_verify with up
 * to 256 rows) wait for other workgroups with a bounded spin, and a call that gave
 * up sets a flag in the context.
 * Returns EH_ERR_HIP if the flag is set (or if the synchronisation fails) and
 * clears it: outputs of rows the failed call did not finish hold -1 (exit_layer,
 * token, argmax) or NaN (H, lse), later calls run normally.
 */
eh_status eh_check(eh_ctx* ctx, void* stream);

/*
 * Bound of the persistent kernels' waits (the cascade of Section 3.4.2 and the
 * verification of Section 4.3.1 at up to 256 rows): the number of polls of another
 * workgroup's record or counter after which a workgroup gives up (each poll is followed by a short sleep; the default, 2^22, is several
 * seconds).  polls >= 0; 0 makes a workgroup give up at its first unanswered poll,
 * which is how the failure path is tested without hanging anything.
 */
eh_status eh_set_spin_limit(eh_ctx* ctx, int32_t polls);

/* Message describing the last error on this context (or, with ctx == NULL, the
 * last eh_create failure of the calling thread).  Never NULL.  The string is
 * owned by the library and valid until the next call on the same context. */
const char* eh_last_error(const eh_ctx* ctx);

/* Library version, e.g. "libeh 0.1 (gfx950)". Static string. */
const char* eh_version(void);

#ifdef __cplusplus
}
#endif
#endif /* EH_H_ */
