/*
 * libulorl -- the per-token core of the UloRL reinforcement-learning objective
 * (arxiv 2507.19766) for AMD MI355X (gfx950), behind a plain C ABI.
 *
 * From the policy's vocabulary logits the forward call computes, per token row,
 * the log-softmax statistics, the chosen-token log-prob and the entropy; then the
 * importance ratio against the behaviour policy of the token's segment (SAIS) or
 * the pseudo-on-policy ratio (POIS), the clipped policy-gradient term, the dynamic
 * mask of well-mastered positive tokens (MPTs) with its entropy gate, and the
 * token-mean loss.  The backward call streams the logits once more and writes
 * d loss / d logits.
 *
 * Conventions common to every entry point
 *   - All array arguments are DEVICE pointers (HIP global memory on the current
 *     device) unless marked HOST.  The library never allocates, frees or copies
 *     device memory, and never synchronises: every call only enqueues kernels on
 *     the HIP stream passed in (`hip_stream` is a hipStream_t; NULL = default
 *     stream) and returns.  Buffers must stay alive until the stream has drained.
 *   - The return value is a ulorl_status; nothing throws or aborts.  Argument
 *     errors are detected on the host before anything is launched.  Errors that
 *     only the device can see (token id outside [0, V), a non-finite logit,
 *     malformed cu_seqlens) never fault: the offending row contributes zero to
 *     the loss and gets a zero gradient, and a bit is raised in counters[3].
 *   - Results are bitwise reproducible from run to run (no floating-point atomics;
 *     every cross-row sum has a fixed order).
 *   - Rows are packed without padding: response i owns rows cu_seqlens[i] ..
 *     cu_seqlens[i+1]-1.
 */
#ifndef ULORL_H
#define ULORL_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    ULORL_OK = 0,
    ULORL_ERR_NULL = -1,      /* a required pointer is NULL                          */
    ULORL_ERR_SHAPE = -2,     /* N, V, R, stride or chunk out of range               */
    ULORL_ERR_DTYPE = -3,     /* unknown storage type                                */
    ULORL_ERR_ALIGN = -4,     /* logits base or row stride not 16-byte aligned       */
    ULORL_ERR_PARAM = -5,     /* eps < 0, tau outside (0,1], unknown mode, ...       */
    ULORL_ERR_WORKSPACE = -6, /* workspace missing, misaligned or too small          */
    ULORL_ERR_HIP = -7,       /* a kernel launch was rejected by the runtime         */
    ULORL_ERR_TOO_LARGE = -8  /* ulorl_token_loss_fwd_bwd_static: the problem needs more scratch
                                 memory than the library's static array holds          */
} ulorl_status;

/* Storage type of logits / dlogits. */
typedef enum { ULORL_F32 = 0, ULORL_BF16 = 1 } ulorl_dtype;

/* Importance-sampling mode (Sec. 3.1.2).
 *   SAIS: r_t = exp(logp_t - old_logp_t); old_logp_t is the log-prob recorded by the
 *         policy that generated the segment f(t) the token belongs to (Eq. "sais").
 *   POIS: every segment's behaviour policy is replaced by the latest one, which with
 *         one update per rollout step equals the current policy: r_t = 1 in value,
 *         d r_t / d logp_t = 1, nothing is ever clipped.  old_logp is not read.      */
typedef enum { ULORL_IS_SAIS = 0, ULORL_IS_POIS = 1 } ulorl_is_mode;

/* When MPTs are masked (Sec. 3.2.2).  The equation of I_msk gates per response on
 * the response's mean token entropy; the prose around it speaks of the entropy of the
 * model as a whole, offered as GLOBAL (token-mean entropy over the whole call).  ALWAYS is the
 * static "Masking MPTs" experiment of Sec. 3.2.1; NEVER gives the DAPO objective
 * (Eq. 7) unchanged.                                                                */
typedef enum {
    ULORL_GATE_PER_RESPONSE = 0,
    ULORL_GATE_GLOBAL = 1,
    ULORL_GATE_ALWAYS = 2,
    ULORL_GATE_NEVER = 3
} ulorl_gate_mode;

/* Bits of the device status word counters[3]. */
enum {
    ULORL_STATUS_BAD_TOKEN = 1,     /* a token id outside [0, V)                      */
    ULORL_STATUS_NONFINITE = 2,     /* a row whose softmax statistics are not finite  */
    ULORL_STATUS_BAD_CU = 4,        /* cu_seqlens not 0 = cu[0] <= ... <= cu[R] = N   */
    ULORL_STATUS_SYNC = 8           /* one-call path only, informational: a workgroup waited in vain
                                       (seconds; never observed) for the others that share its row.
                                       It then wrote nothing; the call's repair pass finished its
                                       part of the row from the intact logits, so every result is
                                       complete and identical to a call without the bit.         */
};

/* HOST struct of scalar parameters. */
typedef struct ulorl_params {
    float eps_low;        /* clip range [1 - eps_low, 1 + eps_high] (Eq. 7; Sec. 3.2.2 uses one eps) */
    float eps_high;
    float tau;            /* MPT probability threshold, 0.99 in Sec. 4.1; in (0, 1]  */
    float sigma;          /* target entropy in nats, 0.2 in Sec. 4.1                  */
    int32_t is_mode;      /* ulorl_is_mode                                            */
    int32_t gate_mode;    /* ulorl_gate_mode                                          */
    int32_t seg_len;      /* > 0: segment id f(t) = offset in response / seg_len;
                             0: ids are taken from segment_ids[] (or all 0)          */
    int32_t reserved;     /* must be 0                                                */
    double denominator;   /* <= 0: D = N, the token count of the call (the 1/sum|o_i|
                             of Sec. 3.2.2 counts masked tokens too); > 0: use this D,
                             e.g. the global count when a batch is split over calls   */
} ulorl_params;

/* HOST struct of launch options, passed per call; NULL selects the defaults.  Nothing in the
 * library keeps state between calls, so concurrent calls from several threads are safe as long as
 * their buffers are distinct.  Workspace sizes never depend on these options. */
enum {
    ULORL_LAUNCH_PER_ROW = 1,       /* row statistics and the one-call path by ONE looping workgroup
                                       per row instead of several cooperating ones: the kernels the
                                       library takes by itself for rows beyond 64 pieces
                                       (1.9 M bf16 logits).  Slower on long rows (16.3 ms against
                                       12.9 ms at 131072 x 151936); results differ from the default
                                       by the summation order of the row statistics only.        */
    ULORL_LAUNCH_DENSE_ROWS = 2     /* lm_head backward: run every row through the three products.  By
                                       default only the rows with a non-zero coefficient are (they are
                                       gathered in order first): masked, clipped and flagged tokens
                                       then cost nothing, which is most of the positive tokens when the
                                       MPT mask is active.  d_hidden is the same either way; d_W
                                       differs by the rounding of fp32 sums whose zero terms are left
                                       out.                                                      */
};
typedef struct ulorl_launch {
    uint32_t flags;       /* ULORL_LAUNCH_* bits                                                  */
    int32_t sync_spins;   /* one-call path: polls (about 0.25 us each) a workgroup waits for the
                             others of its row before it leaves its part to the repair pass
                             (ULORL_STATUS_SYNC); 0: the default 2^24; a tiny value lets a test
                             exercise that pass                                                  */
    int32_t gemm_tile;    /* lm_head variant: 0 = 256 x 256 x 64 block tile, eight waves, tiles
                             copied global -> LDS directly (default); 1 = 128 x 128 x 64, four
                             waves, for products with fewer than a few hundred large tiles      */
    int32_t gemm_group_m; /* lm_head variant: block tiles along M that an XCD walks before it moves
                             along N (its L2 then re-serves their operand rows); 0 = default 4;
                             1..64                                                               */
    int32_t reserved[4];  /* must be 0                                                            */
} ulorl_launch;

/* HOST struct of DEVICE pointers: per-segment training-dynamics diagnostics, optional output of
 * the forward calls (NULL: not wanted).  Produced in the same pass as the token terms, from the
 * values already in registers.  Fields as in ulorl_segment_diagnostics below, which computes the
 * same numbers (bit for bit) from the stored outputs of a forward call. */
typedef struct ulorl_segment_stats {
    int32_t K;            /* segment ids 0 .. K-1 are counted; 1 <= K <= 1024                     */
    int32_t reserved;     /* must be 0                                                            */
    int64_t *count;       /* [K]                                                                  */
    double *ratio_sum;    /* [K]                                                                  */
    float *ratio_max;     /* [K]                                                                  */
    int64_t *clipped;     /* [K]                                                                  */
    double *kl_sum;       /* [K]                                                                  */
    double *ent_sum;      /* [K]                                                                  */
    int64_t *masked;      /* [K]                                                                  */
    int64_t *out_of_range;/* [1], may be NULL                                                     */
    void *workspace;      /* ulorl_segment_diagnostics_workspace_bytes(N, K) bytes, 256-aligned   */
    size_t workspace_bytes;
} ulorl_segment_stats;

/* Library version: major * 10000 + minor * 100 + patch. */
int32_t ulorl_version(void);

/* Static string for a status code (HOST pointer, never NULL). */
const char *ulorl_status_string(int32_t status);

/* Bytes of device workspace ulorl_token_loss_fwd / _fwd_bwd need for N rows of V logits
 * in R responses (0 if an argument is out of range).  The workspace holds per-response
 * entropy sums, per-block partial sums, nine bytes per row and 16 bytes per row and
 * per piece of the row (61440 bytes of a long row); its contents need not be preserved
 * between calls.  The size depends on N, V and R only.                              */
size_t ulorl_token_loss_workspace_bytes(int64_t N, int64_t V, int32_t R);

/*
 * Forward: log-softmax statistics -> ratio -> clipped term -> MPT mask -> loss.
 *
 *   logits        [N, V] row-major, element type dt, row t at logits + t*row_stride
 *                 elements; base and row_stride*sizeof(element) multiples of 16 bytes;
 *                 row_stride >= V.  V need not be a multiple of the vector width.
 *                 1 <= N <= 32768 * 65535 rows, 1 <= V < 2^31.
 *   token_ids     [N] chosen token o_t of each row, in [0, V).
 *                 DOMAIN: every logit must be finite.  A row holding +-infinity or not-a-number
 *                 -- this includes -infinity used to mask vocabulary entries, which a softmax
 *                 defined by limits would take as probability 0 -- is outside the domain: it is
 *                 reported (ULORL_STATUS_NONFINITE), contributes zero to the loss and gets a
 *                 zero gradient.  Callers that mask vocabulary entries pass a large negative
 *                 finite value (e.g. -1e30, exactly representable in bf16 as 0xF149) instead.
 *   cu_seqlens    [R+1] response boundaries, cu[0] = 0, cu[R] = N, non-decreasing.
 *   segment_ids   [N] segment id f(t) per token, or NULL (then p->seg_len rules).
 *                 The ids do not enter the loss (old_logp is already per token); they
 *                 are validated/derived and returned in segment_out.
 *   old_logp      [N] log pi_old_{f(t)}(o_t): behaviour-policy log-prob recorded when
 *                 the token's segment was generated.  May be NULL iff POIS.
 *   advantages    [N] advantage A_t of each token (a response's value broadcast over
 *                 its tokens).  A token is "positive" iff A_t > 0 (reward 1 in a mixed
 *                 group, Sec. 3.3).  NULL selects the STATS-ONLY pass: only lse, logp
 *                 and entropy are written (this is how a caller records old_logp).
 *   p             HOST parameters.
 * Outputs (all DEVICE; [N] float unless noted; any of segment_out, ratio, mpt_mask,
 * resp_entropy, resp_gate, counters may be NULL):
 *   loss          [1]  -(1/D) sum_t (1 - I_t) min(r_t A_t, clip(r_t) A_t)   (Sec. 3.2.2, loss = -J)
 *   logp          log pi_theta(o_t) = z[t, o_t] - lse_t                     (Eq. 6 numerator)
 *   entropy       H_t = - sum_j p_j ln p_j over the vocabulary, nats         (inner sum of H-bar)
 *   lse           log-sum-exp of the row (saved for the backward pass)
 *   gcoef         d loss / d logp_t = -(1/D)(1 - I_t)[r A <= clip(r) A] r_t A_t  (saved for backward)
 *   mpt_mask      [N] uint8  I_t = gate(response of t) and A_t > 0 and p_t >= tau   (Eq. MPTS, I_msk)
 *   ratio         r_t
 *   segment_out   [N] int32 f(t)
 *   resp_entropy  [R] float  H-bar_i, mean token entropy over all tokens of response i
 *   resp_gate     [R] uint8  1 if MPTs of response i are masked
 *   counters      [4] int64: masked tokens, tokens on the clipped (gradient-free) branch,
 *                 positive tokens, status word (ULORL_STATUS_* bits)
 *   seg_stats     HOST, may be NULL: per-segment diagnostics wanted as a by-product (ignored by
 *                 the stats-only pass).
 *   workspace     >= ulorl_token_loss_workspace_bytes(N, V, R) bytes, 256-byte aligned.  The
 *                 stats-only pass works without one (NULL); given one (sized with any R >= 1)
 *                 it forms the statistics by pieces of rows, which is faster and gives the
 *                 same bits as ulorl_token_loss_fwd_bwd.
 *   launch        HOST, may be NULL: launch options.
 */
int32_t ulorl_token_loss_fwd(
    const void *logits, int32_t dt, int64_t N, int64_t V, int64_t row_stride,
    const int32_t *token_ids, const int32_t *cu_seqlens, int32_t R,
    const int32_t *segment_ids, const float *old_logp, const float *advantages,
    const ulorl_params *p,
    float *loss, float *logp, float *entropy, float *lse, float *gcoef,
    uint8_t *mpt_mask, float *ratio, int32_t *segment_out,
    float *resp_entropy, uint8_t *resp_gate, int64_t *counters,
    const ulorl_segment_stats *seg_stats,
    void *workspace, size_t workspace_bytes, const ulorl_launch *launch, void *hip_stream);

/*
 * Backward: dlogits[t, j] = grad_out * gcoef[t] * ( [j == token_ids[t]] - exp(logits[t, j] - lse[t]) )
 * (chain rule through the log-softmax; the mask is a constant).  Rows with gcoef[t] == 0
 * (masked, clipped, zero advantage, or flagged invalid) are written as zeros without being
 * read.  dlogits has the type and row stride of logits and MAY BE THE SAME BUFFER as logits
 * (every 16-byte piece is read and then overwritten by the same thread).  Values are
 * rounded to the storage type with round-to-nearest-even.
 *   lse, gcoef    [N] as produced by the forward call on the same logits.
 *   grad_out      HOST scalar, upstream d(objective)/d(loss), usually 1.
 */
int32_t ulorl_token_loss_bwd(
    const void *logits, int32_t dt, int64_t N, int64_t V, int64_t row_stride,
    const int32_t *token_ids, const float *lse, const float *gcoef, float grad_out,
    void *dlogits, void *hip_stream);

/*
 * Fused forward + backward in one call: same inputs, outputs and conventions as
 * ulorl_token_loss_fwd (advantages must not be NULL) plus grad_out and dlogits as in
 * ulorl_token_loss_bwd (dlogits MAY BE logits).  A row is shared by a few workgroups that keep
 * their pieces in registers and exchange the pieces' softmax statistics through the workspace,
 * so every logit is read once and every gradient written once: HBM sees one read and one write
 * per row instead of two reads and a write.  A row's gradient can be formed at once unless it
 * waits for the entropy gate of Sec. 3.2.2: under the PER_RESPONSE and GLOBAL gates the members
 * of the MPT set (A_t > 0, p_t >= tau) are finished by a second, filtered backward launch after
 * the gate is known.  Results are bit-identical with ulorl_token_loss_fwd (given a workspace)
 * followed by ulorl_token_loss_bwd: both form a row's statistics from the same pieces in the same
 * order (under ULORL_LAUNCH_PER_ROW both calls take their one-workgroup-per-row kernels, again
 * bit-identical with each other).
 * The workgroups of a row wait for each other with a bounded wait.  One whose wait expires writes
 * nothing -- in place its part of the logits stays intact -- and marks its part; a repair pass at
 * the end of the call (two small launches that return at once when nothing is marked) forms the
 * row's statistics from the published pieces and writes the missing parts, so an expired wait
 * costs time, never data: see ULORL_STATUS_SYNC.
 */
int32_t ulorl_token_loss_fwd_bwd(
    const void *logits, int32_t dt, int64_t N, int64_t V, int64_t row_stride,
    const int32_t *token_ids, const int32_t *cu_seqlens, int32_t R,
    const int32_t *segment_ids, const float *old_logp, const float *advantages,
    const ulorl_params *p, float grad_out,
    float *loss, float *logp, float *entropy, float *lse, float *gcoef,
    uint8_t *mpt_mask, float *ratio, int32_t *segment_out,
    float *resp_entropy, uint8_t *resp_gate, int64_t *counters,
    const ulorl_segment_stats *seg_stats,
    void *dlogits, void *workspace, size_t workspace_bytes, const ulorl_launch *launch, void *hip_stream);

/*
 * ulorl_token_loss_fwd_bwd for callers that cannot allocate device memory or pass a workspace:
 * code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same
 * arguments, results (bit for bit) and conventions as ulorl_token_loss_fwd_bwd, without the
 * workspace: the scratch memory is a static device array inside the library,
 * ulorl_static_scratch_bytes() = 32 MiB per GPU, held from library load until the process ends.
 * The call allocates and frees nothing.
 *   - Returns ULORL_ERR_TOO_LARGE when ulorl_token_loss_workspace_bytes(N, V, R) exceeds the
 *     array (131072 rows of 151936 bf16 logits need 10.7 MB; 198004 rows 16.1 MB).
 *   - Every call on a GPU uses that GPU's one array: calls that overlap in time on one GPU (two
 *     streams, two threads) race and give wrong results; calls on one stream are safe back to
 *     back (what must start at zero is cleared by the call itself).
 *   - ulorl_init() resolves the array's address for the current device (hipGetSymbolAddress, once
 *     per device); call it at set-up, outside any stream capture.  Without it the first
 *     ulorl_token_loss_fwd_bwd_static call on a device does so.
 */
int32_t ulorl_init(void);
size_t ulorl_static_scratch_bytes(void);
int32_t ulorl_token_loss_fwd_bwd_static(
    const void *logits, int32_t dt, int64_t N, int64_t V, int64_t row_stride,
    const int32_t *token_ids, const int32_t *cu_seqlens, int32_t R,
    const int32_t *segment_ids, const float *old_logp, const float *advantages,
    const ulorl_params *p, float grad_out,
    float *loss, float *logp, float *entropy, float *lse, float *gcoef,
    uint8_t *mpt_mask, float *ratio, int32_t *segment_out,
    float *resp_entropy, uint8_t *resp_gate, int64_t *counters,
    const ulorl_segment_stats *seg_stats,
    void *dlogits, const ulorl_launch *launch, void *hip_stream);

/* ------------------------------------------------------------------------------------------
 * lm_head variant: the logits are hidden . W and are never materialised.
 *
 *   hidden        [N, Hd] bf16 row-major (Hd contiguous), 16-byte aligned
 *   W             [Hd, V] bf16 row-major (V contiguous), 16-byte aligned: output projection
 *   Hd, V         multiples of 8 (16-byte rows); Hd <= 2^20
 *   N             at most 2^22 - 256 token rows per call (N is a leading dimension of GEMM
 *                 operands in the backward pass; larger batches are split by the caller)
 *   vocab_chunk   multiple of 64, at most 2^22 - 256; the backward pass materialises dlogits one chunk of this many
 *                 vocabulary columns at a time ([N, vocab_chunk] bf16, twice) in the workspace
 * Logits are formed tile by tile with bf16 MFMA and fp32 accumulation and consumed in registers.
 * Everything else (token ids, cu_seqlens, old_logp, advantages, parameters, per-token and
 * per-response outputs, counters, status bits) is exactly as in ulorl_token_loss_fwd, including
 * the stats-only pass selected by advantages == NULL (only lse, logp and entropy are written;
 * the workspace is still needed, sized with any R >= 1).
 *
 * The workspace (ulorl_lmhead_workspace_bytes, 256-byte aligned) holds W^T, hidden^T, two pairs of
 * dlogits chunk buffers (each chunk in both orientations; one chunk's gradient products read theirs
 * while the next chunk's are written: 4 x N x vocab_chunk x 2 bytes), an fp32 accumulator for
 * dHidden, the gathered live rows of hidden with their index maps and the token-loss workspace;
 * nothing in it needs to survive between the forward and the backward call.
 */
size_t ulorl_lmhead_workspace_bytes(int64_t N, int64_t Hd, int64_t V, int32_t R, int32_t vocab_chunk);

int32_t ulorl_lmhead_token_loss_fwd(
    const void *hidden, const void *W, int64_t N, int64_t Hd, int64_t V, int32_t vocab_chunk,
    const int32_t *token_ids, const int32_t *cu_seqlens, int32_t R,
    const int32_t *segment_ids, const float *old_logp, const float *advantages,
    const ulorl_params *p,
    float *loss, float *logp, float *entropy, float *lse, float *gcoef,
    uint8_t *mpt_mask, float *ratio, int32_t *segment_out,
    float *resp_entropy, uint8_t *resp_gate, int64_t *counters,
    const ulorl_segment_stats *seg_stats,
    void *workspace, size_t workspace_bytes, const ulorl_launch *launch, void *hip_stream);

/*
 * Backward of the lm_head variant.  With dz[t, v] = grad_out * gcoef[t] * ([v == token_ids[t]]
 * - exp(z[t, v] - lse[t])) recomputed chunk by chunk (rounded to bf16 as the GEMM operand):
 *   d_hidden [N, Hd] bf16 = dz . W^T      (fp32 accumulation over the whole vocabulary)
 *   d_W      [Hd, V] bf16 = hidden^T . dz (fp32 accumulation over all rows, rounded once)
 * lse and gcoef are those the forward call produced.
 */
int32_t ulorl_lmhead_token_loss_bwd(
    const void *hidden, const void *W, int64_t N, int64_t Hd, int64_t V, int32_t vocab_chunk,
    const int32_t *token_ids, const float *lse, const float *gcoef, float grad_out,
    void *d_hidden, void *d_W, void *workspace, size_t workspace_bytes, const ulorl_launch *launch,
    void *hip_stream);

/*
 * The tiled bf16 MFMA product the lm_head variant is built from, on its own:
 * C[m, n] = sum_k A[m, k] * B[n, k], A [M, K] and B [N, K] bf16 row-major with leading
 * dimensions lda, ldb (multiples of 8, at most 2^22 elements, 16-byte aligned bases), C fp32
 * [M, N] with leading dimension ldc.  K must be a multiple of 8.
 */
int32_t ulorl_gemm_tn_bf16(const void *A, int64_t lda, const void *B, int64_t ldb,
                           int64_t M, int64_t N, int64_t K, float *C, int64_t ldc,
                           const ulorl_launch *launch, void *hip_stream);

/* ------------------------------------------------------------------------------------------
 * The step before the token loss: group-relative advantages (Eq. 4) with the dynamic-sampling
 * constraint of Eq. 7 and the overlong punishment of Sec. 3.5.  Responses come in consecutive
 * groups of group_size (the G samples of one prompt); R must be a multiple of group_size.
 *   rewards      [R]  outcome reward of each response, {0, 1} in the paper (Sec. 3.3)
 *   truncated    [R]  uint8, non-zero if the response hit the global length limit: its reward
 *                     counts as 0 (Sec. 3.5).  May be NULL.
 *   eps          added to the group's standard deviation (Eq. 4 has none; 0 is allowed)
 *   unbiased     0: population standard deviation (divide by G); 1: divide by G - 1
 * Outputs:
 *   resp_adv     [R]  A_i = (r_i - mean_g) / (std_g + eps), or 0 for every response of a group in
 *                     which all or none of the answers are correct (such groups are dropped)
 *   group_keep   [R / group_size] uint8, may be NULL
 *   token_adv    [N]  A_i broadcast over the tokens of response i: the `advantages` input of the
 *                     token-loss calls
 *   kept_tokens  [1]  int64, tokens in kept groups: the denominator 1 / sum |o_i| of the filtered
 *                     batch (pass it as ulorl_params.denominator).  May be NULL.
 */
int32_t ulorl_advantage_prep(
    const float *rewards, const uint8_t *truncated, const int32_t *cu_seqlens, int32_t R,
    int32_t group_size, int64_t N, float eps, int32_t unbiased,
    float *resp_adv, uint8_t *group_keep, float *token_adv, int64_t *kept_tokens, void *hip_stream);

/* ------------------------------------------------------------------------------------------
 * One rollout step of training with segment rollouts (Algorithm 1, Sec. 3.1.1): after the decoder
 * has produced at most seg_len further tokens for each of the B samples in flight (samples carried
 * over from the unfinished pool, or new prompts with prev_len = 0), sort them into the two pools.
 * The three ways a decode ends:
 *   the end-of-sequence token was produced          -> state 1, experience pool
 *   the global maximum length max_len is reached     -> state 2 (truncated), experience pool
 *   the segment is full, max_len not reached          -> state 0, unfinished pool (decode on next step)
 * (an end token exactly at max_len is a normal end).  A sample whose numbers fit none of these
 * (fewer than seg_len new tokens without a reason, more than the segment or max_len allow, an end
 * flag with no new token) is counted in counts[4], clamped into range and kept unfinished.
 *   prev_len, new_len  [B] int32   tokens decoded before / in this step
 *   hit_eos            [B] uint8
 * Outputs (sample order is preserved inside each pool):
 *   state [B] uint8, total_len [B] = prev_len + new_len, segments [B] = segments spanned so far
 *   unfinished_idx [B]   first counts[0] entries: indices of the samples to decode further
 *   experience_idx [B]   first counts[1] entries: indices of the samples that go to training
 *   exp_cu_seqlens [B+1] first counts[1]+1 entries: prefix sums of their total lengths, i.e. the
 *                        cu_seqlens of the packed training batch (token t of it belongs to
 *                        segment offset / seg_len, the seg_len rule of ulorl_params)
 *   exp_truncated  [B]   first counts[1] entries: 1 where the sample was cut at max_len -- the
 *                        `truncated` input of ulorl_advantage_prep (Sec. 3.5)
 *   counts [5] int64     unfinished, experience, truncated, experience tokens, inconsistent samples
 * B * max_len must fit in int32 (offsets of the packed batch).  One workgroup; no workspace.
 */
int32_t ulorl_segment_pool_step(
    int32_t B, const int32_t *prev_len, const int32_t *new_len, const uint8_t *hit_eos,
    int32_t seg_len, int32_t max_len,
    uint8_t *state, int32_t *total_len, int32_t *segments, int32_t *unfinished_idx,
    int32_t *experience_idx, int32_t *exp_cu_seqlens, uint8_t *exp_truncated, int64_t *counts,
    void *hip_stream);

/*
 * Training-dynamics diagnostics per segment id, from the outputs of a forward call: the
 * quantities behind the comparison of the importance-sampling schemes in Sec. 3.1.2 (how far the
 * ratio of older segments has drifted, how much of each segment is clipped) and the entropy
 * curves of Sec. 3.2.  For every k in [0, K):
 *   count[k]      int64   tokens with segment id k
 *   ratio_sum[k]  double  sum of r_t            ratio_max[k]  float   largest r_t
 *   clipped[k]    int64   tokens on the clipped, gradient-free branch of the min
 *   kl_sum[k]     double  sum of (old_logp_t - logp_t): sampled estimate of KL(pi_old || pi_theta) * count
 *   ent_sum[k]    double  sum of token entropies
 *   masked[k]     int64   tokens removed by the MPT mask
 * out_of_range [1] int64 (may be NULL) counts tokens whose id is outside [0, K); they are ignored.
 * old_logp may be NULL (POIS): kl_sum is then 0.  Sums are fixed-order fp64: bitwise reproducible.
 * K <= 1024.  The workspace size comes from ulorl_segment_diagnostics_workspace_bytes.
 * The forward calls produce the same numbers as a by-product when given a ulorl_segment_stats.
 */
size_t ulorl_segment_diagnostics_workspace_bytes(int64_t N, int32_t K);

int32_t ulorl_segment_diagnostics(
    int64_t N, int32_t K, const int32_t *segment_ids, const float *ratio, const float *logp,
    const float *old_logp, const float *entropy, const uint8_t *mpt_mask, const float *advantages,
    float eps_low, float eps_high,
    int64_t *count, double *ratio_sum, float *ratio_max, int64_t *clipped, double *kl_sum,
    double *ent_sum, int64_t *masked, int64_t *out_of_range,
    void *workspace, size_t workspace_bytes, void *hip_stream);

#ifdef __cplusplus
}
#endif
#endif /* ULORL_H */
