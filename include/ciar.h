/*
 * ciar.h -- C ABI of the MI355X (gfx950) implementation of CIAR's per-position hot path.
 *
 * For every drafted image-token position (a "row") the library streams the V-wide centre
 * ("draft") logit row, and for verification also the cloud ("target") logit row, once from
 * HBM and computes
 *
 *   quantify : softmax statistics, the InterFuse probability interval [p^l, p^u], the widths'
 *              Total Ambiguity Omega, Confidence Disparity Sigma and score U = Omega * Sigma,
 *              and the "send to the cloud" flag U > tau
 *   verify   : the speculative accept / reject test of each drafted token against the target
 *              distribution, the residual resample of rejected tokens, and per window of K
 *              drafted tokens the accepted prefix length and the replacement token
 *
 * C99; no C++ types and no exceptions cross this boundary.
 *
 * Conventions for every entry point
 *   - Every tensor pointer is a DEVICE pointer owned by the caller; `params` is a HOST pointer
 *     and is read before the call returns.  The library allocates nothing, frees nothing and
 *     never synchronises: kernels are enqueued on `hip_stream` (a hipStream_t, NULL = the
 *     default stream) and outputs are valid once the caller has synchronised that stream.
 *   - `workspace` is device scratch of at least ciar_workspace_bytes(N, params) bytes, 16-byte
 *     aligned, owned by the caller.  It carries the per-row statistics, the words in which the
 *     rows of a window that spans workgroups meet, and per-row results the caller did not ask for
 *     but a later kernel or a window output needs.  Its contents need no initialisation (the window
 *     words carry a per-launch tag; everything else is written before it is read) and are
 *     garbage afterwards; calls that overlap in time on one device must not share a workspace.
 *   - Logits: row-major [N, row_stride] with V <= row_stride, element type `dtype`
 *     (float32, or bfloat16 widened exactly to float32 on load).  Base pointers and
 *     row_stride * sizeof(element) must be multiples of 16 bytes, and the buffer must be
 *     readable up to (N-1)*row_stride + roundup(V, 16 bytes / sizeof(element)) elements.
 *     Values must be finite or -inf (-inf = masked token: probability 0, width 0, still
 *     counted in V); every row needs at least one finite logit.  NaN / +inf is a violated
 *     precondition and gives unspecified numbers (never a fault).
 *   - 0 <= draft_ids[i] < V and uniforms in [0, 1) are preconditions (ids are clamped into
 *     range on the device so a bad id cannot fault).
 *   - Output pointers may be NULL to skip that output, where stated.
 *   - HIP keeps a last-error state per host thread.  An entry point that launches kernels reads and resets it
 *     before its first launch (so that an error left by an earlier, unrelated call is not reported as this
 *     call's) and after each launch.
 *   - Return value: a ciar_status.  On any error nothing has been launched and
 *     ciar_last_error() describes the problem.  N == 0 is valid and launches nothing.
 *   - Supported vocabulary: 1 <= V <= 32768 (float32) or 65536 (bfloat16).
 */
#ifndef CIAR_H
#define CIAR_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum ciar_dtype { CIAR_F32 = 0, CIAR_BF16 = 1 } ciar_dtype;

typedef enum ciar_status {
    CIAR_OK = 0,
    CIAR_EINVAL = -1,        /* NULL / out-of-range argument                      */
    CIAR_EALIGN = -2,        /* pointer or row stride not 16-byte aligned         */
    CIAR_EWORKSPACE = -3,    /* workspace missing or too small                    */
    CIAR_EUNSUPPORTED = -4,  /* vocabulary or dtype outside the supported range   */
    CIAR_EHIP = -5           /* the HIP runtime reported an error at launch       */
} ciar_status;

/*
 * Parameters of the pass.  Fill with ciar_params_default() and override.
 *
 * Radius.  The paper's logit radius is the Softplus output of a trained head (Sec. 3.2.1,
 * Inter-Head equation: r_t = Softplus(Linear_radius(h_t))).  Token i of a row has the radius
 *   r_i = min(kappa * rho_i, radius_max),
 *   rho_i = 1                          scalar mode: the call's `radius` argument is NULL
 *         = Softplus(radius[row, i])   tensor mode: `radius` is the raw output of the radius half of
 *                                      the Interval Head, laid out like draft_logits (same dtype,
 *                                      same row_stride, same alignment rules; any finite value)
 *   kappa = radius_scale               if radius_scale >= 0 (1 = the head as the paper writes it)
 *         = sqrt(2) * erfinv(confidence) otherwise (two-sided standard-normal quantile of the
 *           "interval confidence" gamma in (0,1): 0.8 -> 1.2816, 0.9 -> 1.6449, 0.95 -> 1.9600).
 * radius_max is the clamp the paper applies without naming a value (App. "Proof of Interval
 * Validity", last paragraph).  Accepted range [0, 16] (CIAR_EINVAL outside it): at radius 16 the bounds of a
 * token are its probability with the odds scaled by e^16 = 8.9e6 either way.  Beyond that the bounds of the top
 * token of a nearly one-hot row are quotients of e^-r and 1 - x_max: its width is (1 - x_max) / e^-r with
 * 1 - x_max known to 4e-15 from fp32 exponentials, which stops meeting the library's 1e-7 absolute accuracy
 * at e^-r = 4e-8.
 */
typedef struct ciar_params {
    uint32_t struct_size;   /* sizeof(ciar_params); checked                                        */
    int32_t  vocab;         /* V                                                                   */
    int32_t  dtype;         /* ciar_dtype of the logit tensors                                     */
    int32_t  window;        /* K >= 1: drafted tokens per cloud verification (Algorithm 1)         */
    int64_t  row_stride;    /* elements between consecutive rows                                   */
    float    confidence;    /* gamma, used when radius_scale < 0                                   */
    float    radius_scale;  /* kappa override, < 0 = derive from confidence                        */
    float    radius_max;    /* clamp on the radius, in [0, 16], default 10                         */
    float    tau;           /* threshold on U, default 0.30 (Algorithm 1; Sec. 4 threshold study)  */
    float    lower_cap;     /* 0.99 (normalisation equations of the validity appendix)             */
    float    upper_cap;     /* 1.01                                                                */
    int32_t  normalize;     /* 1 = apply the caps (the paper), 0 = raw InterFuse                   */
    int32_t  reserved;      /* must be 0                                                           */
} ciar_params;

/* Writes the defaults (confidence 0.9, radius_scale -1, radius_max 10, tau 0.30, caps 0.99 / 1.01,
 * normalize 1, window 8, dtype float32, vocab 0, row_stride 0).  `p` is a host pointer. */
void ciar_params_default(ciar_params* p);

/*
 * Host only (no GPU work): the polynomial the kernels use for the interval width of small probabilities at
 * this call's scalar radius r = min(kappa, radius_max), a = e^r, b = e^-r (App. "Proof of Interval Validity":
 * the InterFuse bounds as functions of the probability x).  For x <= *x_max
 *   (p^u - p^l) / ((a - b) x) = (1 - x) / ((1 + (a-1) x)(1 - (1-b) x)) = 1 + x (c[0] + c[1] x + c[2] x^2 + c[3] x^3)
 * to 2e-8 relative.  *x_max < 0: the kernels use no polynomial at this radius.  Exposed so that the fit can be
 * checked without a GPU.  `coef` (4 floats) and `x_max` are host pointers.  Returns CIAR_OK or CIAR_EINVAL.
 */
int ciar_width_polynomial(const ciar_params* params, float* coef, float* x_max);

/*
 * Bytes of device workspace ciar_quantify / ciar_verify / ciar_quantify_verify need for N rows
 * (113 bytes per row, rounded up).  Always a multiple of 256; returns 0 for N <= 0.
 */
size_t ciar_workspace_bytes(int64_t N, const ciar_params* params);

/*
 * Uncertainty quantifier (Sec. 3.2.1 "Device-Side Uncertainty Quantification"; Eq.
 * uncertainty_score; App. "Proof of Interval Validity"; threshold test of Algorithm 1).
 *
 *   draft_logits [N, row_stride]   in   centre logits c
 *   radius       [N, row_stride]   in   raw radius tensor (tensor mode), or NULL (scalar mode)
 *   draft_ids    [N] int32         in   token whose interval is reported; NULL = the arg-max token
 *   p_lo, p_mid, p_hi [N] float    out  p^l_x, softmax(c)_x, p^u_x of that token (after the caps)
 *   omega, sigma, score [N] float  out  Omega = sum of widths, Sigma = population std of widths, U
 *   flags        [N] uint8         out  1 = U > tau (uncertain: send to the cloud), 0 = accept locally
 * Any output may be NULL; at least one must be given.
 */
int ciar_quantify(const void* draft_logits, const void* radius, const int32_t* draft_ids, int64_t N,
                  const ciar_params* params,
                  float* p_lo, float* p_mid, float* p_hi,
                  float* omega, float* sigma, float* score, uint8_t* flags,
                  void* workspace, size_t workspace_bytes, void* hip_stream);

/*
 * Cloud-side verification of drafted tokens (Algorithm 1, "Cloud verification" and the resample /
 * advance steps that follow it).  The paper states the step as speculative decoding without
 * writing the test; this is the standard rule: with p = softmax(draft row), q = softmax(target row)
 * and x the drafted token, accept iff u_accept < min(1, q_x / p_x) (evaluated in the log domain);
 * on rejection draw from (q - p)^+ / ||(q - p)^+||_1 by inverse CDF in token order with u_resample:
 * the smallest j whose inclusive running sum exceeds u_resample * R.
 *
 *   draft_logits, target_logits [N, row_stride]  in
 *   draft_ids  [N] int32, u_accept [N] float, u_resample [N] float   in
 *   accept          [N] uint8   out  1 = accepted                              (may be NULL)
 *   row_resample_id [N] int32   out  residual sample of a rejected row, -1 if accepted (may be NULL)
 *   accept_len      [W] int32   out  leading accepted rows of window w = rows [wK, min((w+1)K, N)),
 *                                    W = ceil(N / K)                            (may be NULL)
 *   resampled_id    [W] int32   out  row_resample_id of the window's first rejected row, -1 if the
 *                                    whole window was accepted                  (may be NULL)
 * At least one output must be given.
 */
int ciar_verify(const void* draft_logits, const void* target_logits, const int32_t* draft_ids,
                const float* u_accept, const float* u_resample, int64_t N,
                const ciar_params* params,
                uint8_t* accept, int32_t* row_resample_id,
                int32_t* accept_len, int32_t* resampled_id,
                void* workspace, size_t workspace_bytes, void* hip_stream);

/*
 * Fused quantify + verify: both rows are read from HBM exactly once and nothing V-wide is written.
 * Arguments and semantics are the union of ciar_quantify (with draft_ids required) and ciar_verify.
 * In tensor mode the radius rows are read once as well (three V-wide rows per position).
 */
int ciar_quantify_verify(const void* draft_logits, const void* radius, const void* target_logits,
                         const int32_t* draft_ids, const float* u_accept, const float* u_resample,
                         int64_t N, const ciar_params* params,
                         float* p_lo, float* p_mid, float* p_hi,
                         float* omega, float* sigma, float* score, uint8_t* flags,
                         uint8_t* accept, int32_t* row_resample_id,
                         int32_t* accept_len, int32_t* resampled_id,
                         void* workspace, size_t workspace_bytes, void* hip_stream);

/*
 * ciar_quantify_verify for callers that cannot allocate device memory or hand over a workspace: code under HIP
 * graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments, semantics, kernels and
 * results as ciar_quantify_verify, without `workspace` / `workspace_bytes`: the per-row statistics, the list of
 * rejected rows and the per-row results the caller did not ask for live in a buffer that is part of the library's
 * device image (ciar_workspace_bytes(CIAR_STATIC_MAX_ROWS) = 3.53 MiB on every GPU the library runs on, held
 * until the process ends).  The call allocates and frees nothing.
 *   - N > CIAR_STATIC_MAX_ROWS returns CIAR_EWORKSPACE and launches nothing.
 *   - Every call on a GPU uses that GPU's one buffer: calls that overlap in time on one GPU (different streams,
 *     different host threads) race on it.  Calls on one stream, or otherwise ordered, are safe; the buffer needs
 *     no clearing between calls (its counters carry the tag of the launch that uses them, see `workspace` above).
 *   - The first call on a device looks the buffer's address up (hipGetSymbolAddress) with that device current.
 */
#define CIAR_STATIC_MAX_ROWS 32768
int ciar_quantify_verify_static(const void* draft_logits, const void* radius, const void* target_logits,
                                const int32_t* draft_ids, const float* u_accept, const float* u_resample,
                                int64_t N, const ciar_params* params,
                                float* p_lo, float* p_mid, float* p_hi,
                                float* omega, float* sigma, float* score, uint8_t* flags,
                                uint8_t* accept, int32_t* row_resample_id,
                                int32_t* accept_len, int32_t* resampled_id, void* hip_stream);

/*
 * The two stages of the calls above, on their own, for callers that want to time them or to put
 * other work between them.  ciar_quantify, ciar_verify and ciar_quantify_verify are exactly
 * ciar_stream_rows followed by ciar_finish_rows (same kernels, same launch configuration).  Both take the
 * argument list of ciar_quantify_verify and must be given the same arguments: target_logits = NULL with
 * no verify output is a quantify-only call, no quantify output a verify-only call (radius must be NULL).
 *
 * ciar_stream_rows   the streaming kernel: reads every logit row once from HBM and writes every per-row output:
 *                    the quantifier's (p_lo ... flags) and, with a verifier row, the accept bits.  For float32
 *                    logits (V <= 32768) under a scalar or tensor radius that is not very wide it also makes the
 *                    residual draws of the rejected rows, from the registers that still hold both rows, and
 *                    writes the window outputs; the call is then this one launch.  (Calls whose flat rows need the
 *                    fp64 pass launch that behind it, see the radius notes above.)
 * ciar_finish_rows   what remains, if anything: for bfloat16 logits and very wide radii the residual
 *                    draws of the rejected rows (their rows are read again), and the window outputs where neither
 *                    kernel could write them (windows longer than 255 rows that span workgroups).
 */
int ciar_stream_rows(const void* draft_logits, const void* radius, const void* target_logits,
                     const int32_t* draft_ids,
                     const float* u_accept, const float* u_resample, int64_t N, const ciar_params* params,
                     float* p_lo, float* p_mid, float* p_hi,
                     float* omega, float* sigma, float* score, uint8_t* flags,
                     uint8_t* accept, int32_t* row_resample_id,
                     int32_t* accept_len, int32_t* resampled_id,
                     void* workspace, size_t workspace_bytes, void* hip_stream);

/*
 * Measurement aid: ciar_stream_rows whose streaming-kernel dispatch records two HIP events (hipEvent_t handles,
 * created by the caller with timing enabled, host pointers; both required) at the kernel's start and at its end,
 * so that hipEventElapsedTime(start, stop) is the kernel's own duration without the dispatch latency that an
 * event pair recorded around the call also spans.  N = 0 launches nothing and records nothing.
 */
int ciar_stream_rows_timed(const void* draft_logits, const void* radius, const void* target_logits,
                           const int32_t* draft_ids,
                           const float* u_accept, const float* u_resample, int64_t N, const ciar_params* params,
                           float* p_lo, float* p_mid, float* p_hi,
                           float* omega, float* sigma, float* score, uint8_t* flags,
                           uint8_t* accept, int32_t* row_resample_id,
                           int32_t* accept_len, int32_t* resampled_id,
                           void* workspace, size_t workspace_bytes, void* hip_stream,
                           void* start_event, void* stop_event);

int ciar_finish_rows(const void* draft_logits, const void* radius, const void* target_logits,
                     const int32_t* draft_ids,
                     const float* u_accept, const float* u_resample, int64_t N, const ciar_params* params,
                     float* p_lo, float* p_mid, float* p_hi,
                     float* omega, float* sigma, float* score, uint8_t* flags,
                     uint8_t* accept, int32_t* row_resample_id,
                     int32_t* accept_len, int32_t* resampled_id,
                     void* workspace, size_t workspace_bytes, void* hip_stream);

/*
 * Several Interval Heads (Sec. 4, ablation on the Inter-Head: heads trained under different seeds,
 * aggregated by "Voting" or "Ensemble"; the paper names the two strategies without formulas, the
 * readings are stated here).
 *
 *   draft_heads  [heads, N, row_stride]  in   centre logits of head h at draft_heads + h * head_stride
 *                                             elements; head_stride * sizeof(element) a multiple of 16
 *   radius_heads same layout, or NULL    in   raw radius tensors (tensor mode), one per head
 *   draft_ids    [N] int32, or NULL      in   reported token (NULL: the arg-max token, see below)
 *   strategy = CIAR_VOTING    every head runs ciar_quantify on its own; flags [N] is the strict majority of
 *                             the heads' flags (2 * votes > heads).  p_lo ... score are per head,
 *                             [heads, N]; head_flags [heads, N] uint8 (may be NULL) are the heads' own
 *                             flags; a NULL draft_ids reports each head's own arg-max token.
 *   strategy = CIAR_ENSEMBLE  the heads' curves are averaged token by token (p^l_i = mean_h p^l_{h,i}, the
 *                             same for the centre probabilities and p^u, every head after its own
 *                             0.99 / 1.01 scaling), and Omega, Sigma, U, the flag and the reported
 *                             token's interval come from the averaged curves.  All outputs are [N];
 *                             head_flags is not written; a NULL draft_ids reports the arg-max token of
 *                             the averaged centre distribution.
 * Any output may be NULL; at least one must be given.  1 <= heads <= 8.  workspace: at least
 * ciar_multihead_workspace_bytes(N, heads, params) bytes, rules as above.  Every head's rows are
 * streamed once (Voting) or twice (Ensemble: the second sweep forms the token-wise averages once
 * every head's partition sum and caps are known).
 */
enum { CIAR_VOTING = 0, CIAR_ENSEMBLE = 1 };

size_t ciar_multihead_workspace_bytes(int64_t N, int32_t heads, const ciar_params* params);

int ciar_quantify_multihead(const void* draft_heads, const void* radius_heads, int32_t heads, int64_t head_stride,
                            const int32_t* draft_ids, int64_t N, const ciar_params* params, int32_t strategy,
                            float* p_lo, float* p_mid, float* p_hi,
                            float* omega, float* sigma, float* score,
                            uint8_t* flags, uint8_t* head_flags,
                            void* workspace, size_t workspace_bytes, void* hip_stream);

/*
 * Forward value of the Inter-DRO training loss (Sec. 3.2.3 "Interval-enhanced Distributionally Robust
 * Training": the anchor, DRO and alignment equations).  No gradients.
 *
 *   center_logits [N, row_stride]   in   centre logits c of the Interval Head
 *   radius        [N, row_stride]   in   raw radius tensor, or NULL (scalar radius; radius rules as above)
 *   cloud_logits  [N, row_stride]   in   the cloud model's logits o_cloud
 * With p_mid = softmax(c), p_up = softmax(c + r), p_lo = softmax(c - r), p_cloud = softmax(o_cloud):
 *   L1(p) = ||p - p_cloud||_1,  CE(p) = - sum_i p_cloud,i ln p_i,  KL = KL(p_cloud || p_mid)
 *   (a token with p_cloud,i = 0, e.g. a -inf cloud logit, contributes nothing to CE and KL).
 *   row_terms [7, N] float  out  rows of L1(p_mid), L1(p_up), L1(p_lo), CE(p_mid), CE(p_up), CE(p_lo), KL
 *   weights   [N]    float  out  w_n = exp(alpha CE_n(p_lo)) / sum_k exp(alpha CE_k(p_lo))   (may be NULL)
 *   losses    [5]    float  out  centre, upper, lower, DRO, total                             (may be NULL)
 *       centre = mean_n(lambda_v L1(p_mid) + lambda_p CE(p_mid) + lambda_beta KL)
 *       upper  = mean_n(lambda_v L1(p_up) + lambda_p CE(p_up)),  lower likewise with p_lo
 *       DRO    = sum_n w_n CE_n(p_lo),  total = centre + upper + lower + DRO
 * The paper prints no batch reduction for the anchor and alignment terms: the mean over the N rows is this
 * library's reading; lambda_v, lambda_p, lambda_beta and alpha are not given in the paper and have no defaults.
 * No workspace.  Same pointer, alignment, stream and error rules as ciar_quantify.
 */
int ciar_interdro_loss(const void* center_logits, const void* radius, const void* cloud_logits, int64_t N,
                       const ciar_params* params, float lambda_v, float lambda_p, float lambda_beta, float alpha,
                       float* row_terms, float* weights, float* losses, void* hip_stream);

/*
 * Measurement aid, not a step of the method: a plain streaming read of the rows the hot path reads
 * (the "read both rows and sum" ceiling a memory-bound pass is held against).  Every logit of
 * draft_logits [N, row_stride] and, unless NULL, target_logits is loaded once with 16-byte loads and
 * added up as floats; padding between rows is not counted.
 *   row_sum [N] fp32  out  sum of the row's V draft logits (plus its V target logits)
 * params supplies vocab, dtype and row_stride (validated as for the other calls).  Same pointer,
 * alignment, stream and error rules as ciar_quantify; no workspace.
 */
int ciar_read_rows(const void* draft_logits, const void* target_logits, int64_t N, const ciar_params* params,
                   float* row_sum, void* hip_stream);

/* The same with the kernel's dispatch recording two HIP events at its start and end (see ciar_stream_rows_timed). */
int ciar_read_rows_timed(const void* draft_logits, const void* target_logits, int64_t N, const ciar_params* params,
                         float* row_sum, void* hip_stream, void* start_event, void* stop_event);

/*
 * The Interval Head as a producer (Sec. 3.2.1, "Interval Head Architecture": the head's output dimension is
 * 2 |V|; c_t = Linear_center(h_t), r_t = Softplus(Linear_radius(h_t)), then InterFuse and the score).
 * The two linear maps run as one bf16 contraction on the matrix cores with fp32 accumulation:
 *   logits[n, j] = sum_k hidden[n, k] * weight[j, k] + bias[j],   j in [0, 2V)
 * columns [0, V) are the centre logits, columns [V, 2V) the raw radius (before Softplus).
 *
 *   hidden     [N, hidden_dim] bf16   in   hidden states, rows contiguous (row stride hidden_dim)
 *   weight     [2V, hidden_dim] bf16  in   row j = the weights of output column j (centre rows first)
 *   bias       [2V] float             in   or NULL (no bias)
 * The logits are produced in fp32, so params->dtype must be CIAR_F32; params->row_stride is the row stride of the
 * produced logit rows.  Supported shapes: vocab a multiple of 128, hidden_dim a multiple of 64 (CIAR_EUNSUPPORTED
 * otherwise); hidden and weight 16-byte aligned.
 *
 * ciar_interhead_logits writes the two logit tensors, centre and radius [N, row_stride] float each (both
 * required), and nothing else; no workspace.
 *
 * ciar_interhead_quantify keeps them in the workspace and runs ciar_quantify in tensor-radius mode on them
 * (radius_scale 1 is the head as the paper writes it); draft_ids and the outputs are ciar_quantify's.  Its
 * workspace is ciar_interhead_workspace_bytes(N, params) = the two logit tensors + ciar_workspace_bytes.
 */
size_t ciar_interhead_workspace_bytes(int64_t N, const ciar_params* params);
int ciar_interhead_logits(const void* hidden, const void* weight, const float* bias, int32_t hidden_dim, int64_t N,
                          const ciar_params* params, float* centre, float* radius, void* hip_stream);
int ciar_interhead_quantify(const void* hidden, const void* weight, const float* bias, int32_t hidden_dim,
                            const int32_t* draft_ids, int64_t N, const ciar_params* params,
                            float* p_lo, float* p_mid, float* p_hi,
                            float* omega, float* sigma, float* score, uint8_t* flags,
                            void* workspace, size_t workspace_bytes, void* hip_stream);

/* ciar_interhead_logits with the contraction kernel's dispatch recording two HIP events at its start and end
 * (see ciar_stream_rows_timed). */
int ciar_interhead_logits_timed(const void* hidden, const void* weight, const float* bias, int32_t hidden_dim,
                                int64_t N, const ciar_params* params, float* centre, float* radius,
                                void* hip_stream, void* start_event, void* stop_event);

/*
 * Window epilogue on its own (the last step of ciar_verify / ciar_quantify_verify, which run it when
 * a window output is requested): from the per-row results of N rows,
 *   accept_len[w]   = number of leading rows with accept != 0 in window w = rows [wK, min((w+1)K, N))
 *   resampled_id[w] = row_resample_id of the first row with accept == 0 in the window, -1 if none
 * (Algorithm 1: the verified prefix of a drafted window and the token that replaces the first
 * rejected one).  accept [N] uint8 and row_resample_id [N] int32 are inputs; either output may be
 * NULL, not both; row_resample_id may be NULL when resampled_id is.  Only params->window is read.
 */
int ciar_window_epilogue(const uint8_t* accept, const int32_t* row_resample_id, int64_t N,
                         const ciar_params* params, int32_t* accept_len, int32_t* resampled_id,
                         void* hip_stream);

/*
 * Test / debugging export of the dense curves: p_lo, p_mid, p_hi as [N, V] float32 each, densely
 * packed (row stride V), computed with the same per-token arithmetic as ciar_quantify.  Writes
 * 3*N*V floats; not part of the hot path.  Any of the three may be NULL.  radius as for ciar_quantify.
 */
int ciar_dense_intervals(const void* draft_logits, const void* radius, int64_t N, const ciar_params* params,
                         float* p_lo, float* p_mid, float* p_hi, void* hip_stream);

/* Message for the last non-OK status returned on the calling thread; never NULL. */
const char* ciar_last_error(void);

/* "major.minor.patch" of the library. */
const char* ciar_version(void);

#ifdef __cplusplus
}
#endif
#endif /* CIAR_H */
