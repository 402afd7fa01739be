/*
 * semicrf.h - C ABI of the MI355X (gfx950) streaming semi-Markov CRF library.
 *
 * The library computes, for a batch of sequences, the log-partition function
 * logZ of a semi-Markov CRF whose edge potential is the three-term form of the
 * paper's Eq. 4 (centred content score from prefix sums, duration bias,
 * transition), and the exact gradients of sum_b w_b*logZ_b with respect to the
 * emissions, the duration bias and the transition matrix (the expected
 * sufficient statistics of the paper's "Gradient Formulas" section).  Edge
 * potentials are never stored; working memory beyond the O(T*C) prefix arrays
 * is a K-deep ring per sequence plus checkpoints every `ckpt_interval`
 * positions (Algorithm 1 / Algorithm 3).
 *
 * Conventions common to every entry point
 *   - Every array pointer is a DEVICE pointer owned by the caller, except where
 *     "host" is stated.  The library allocates nothing and frees nothing; all
 *     scratch comes from the caller's `workspace`.
 *   - Work is enqueued on `stream` (a hipStream_t passed as void*; NULL is the
 *     default stream).  No entry point synchronises with the host.
 *   - Return value: SEMICRF_OK or a negative semicrf_status.  On any error no
 *     kernel has been launched and the outputs are untouched.
 *   - Layouts are row-major with the label index fastest:
 *       emis   [B,T,C]  float   raw emissions f(t,c); rows t >= lengths[b] are never read
 *       lengths[B]      int32   true lengths L_b, clamped on the device to [0,T]; NULL = all T
 *       trans  [C,C]    float   trans[c_src*C + c_dst]         (source label first)
 *       dur    [K,C]    float   dur[(k-1)*C + c], k = 1..K     (durations are 1-based)
 *   - Positions t in 0..T are boundaries between tokens; a segment [s,s+k)
 *     covers tokens s..s+k-1 and its content score is S[s+k,c]-S[s,c]
 *     ("Indexing conventions").  alpha_0(c) = 0 for every label, so the first
 *     segment pays LSE over the source label of trans[.,c]; there is no end
 *     term: logZ = LSE_c alpha_L(c).  K may exceed T.  An empty sequence
 *     (L_b = 0) has logZ = ln C and zero gradients.
 *   - Supported sizes: 1 <= C <= 256, and K*C small enough for the ring, the
 *     duration table and the per-interval accumulators to fit the 160 KB LDS of
 *     one compute unit (see semicrf_workspace_bytes, which reports
 *     SEMICRF_EUNSUPPORTED otherwise); T <= 2^30 and B*(T+1)*C <= 2e10.
 */
#ifndef SEMICRF_H
#define SEMICRF_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    SEMICRF_OK = 0,
    SEMICRF_EINVAL = -1,       /* bad size, null required pointer, negative interval */
    SEMICRF_EWORKSPACE = -2,   /* workspace_bytes too small or workspace misaligned (256 B) */
    SEMICRF_EUNSUPPORTED = -3, /* (K,C) does not fit the LDS budget of the kernels, or T / B*T*C beyond the stated limits */
    SEMICRF_ELAUNCH = -4       /* a HIP call or kernel launch reported an error */
} semicrf_status;

/* flags bit 0: subtract the per-sequence emission baseline nu[b,c] before the
 * prefix sum (Eq. 1).  Without it S is the raw prefix sum. */
#define SEMICRF_CENTER 1u
/* flags bit 1: run the forward scan of Algorithm 1 and the backward scan of Algorithm 3
 * strictly sequentially.  By default both are run chunk-parallel: every checkpoint interval
 * is scanned as an independent task that first warms its ring up over the max(1.5K,32)
 * positions before the interval (max(8K,64) in a second attempt for what the first did not
 * verify), starting from the state of a sequence that begins there.
 * The state each task reaches at its end is then compared, entry by entry and up to the
 * common scale factor, with the warmed-up state its neighbour started from; a (sequence,
 * direction) is accepted only if every one of its boundaries agrees to 1e-10 (relative),
 * which bounds the deviation from the sequential scan by 2e-10 per boundary crossed.  A
 * rejected (sequence, direction) is rescanned sequentially inside the same call, so the
 * results are those of the sequential scan either way; only the time differs.
 * semicrf_scan_report tells which happened. */
#define SEMICRF_SEQUENTIAL_SCAN 2u
/* flags bits 2, 3: storage type of `emis`.  With one of them set the `emis` argument of every
 * entry point addresses 2-byte elements, IEEE half precision or bfloat16, in the same [B,T,C]
 * layout (pass the pointer cast to const float*); they are widened exactly on load and
 * everything downstream is unchanged (all outputs stay float).  Setting both is invalid. */
#define SEMICRF_EMIS_F16 4u
#define SEMICRF_EMIS_BF16 8u
/* flags bit 4: run the chunk-parallel scans of semicrf_logz_fwd / semicrf_fwd_bwd (and their _boundary forms)
 * on the matrix cores where the sizes allow (17 <= C <= 24, K <= 64, checkpoint interval a multiple of 32,
 * B*(T+1)*C < 2^27): sixteen checkpoint intervals advance in lock step as the columns of
 * v_mfma_f64_16x16x4_f64 products (window: [16 positions] x [4 source positions] x [16 intervals] per label,
 * transition: [16 labels] x [4 labels] x [16 intervals] per position).  Checkpoints, verification and results
 * are those of the default one-wave-per-interval kernel (the acceptance test is the same); only the time
 * differs.  Off by default: measured slower than the default kernel on MI355X (a lone wave per SIMD issues its
 * per-position bookkeeping too slowly); kept as the measured alternative.  Ignored where the sizes do not allow it. */
#define SEMICRF_MATRIX_SCAN 16u
/* flags bits 5, 6: where semicrf_fwd_bwd takes the expected statistics of the "Gradient Formulas" section from.
 * Default (neither bit): from the stored rows of both scans (the backward scan tasks keep their rows like the
 * forward ones, and no recurrence is run a third time) wherever the chunk-parallel scans apply, every interval has
 * its row slot and no boundary term is an input or output of the call; otherwise, and for the sequences whose
 * scans were not accepted, from Algorithm 3's per-interval recurrence.  SEMICRF_MARGINALS_ROWS states the default
 * (want_grad = 1 or 3), SEMICRF_MARGINALS_INTERVAL asks for the per-interval recurrence everywhere (want_grad = 2
 * suffices: one O(T*C) row array less).  Setting both is invalid.  The results agree to the rounding of the
 * outputs. */
#define SEMICRF_MARGINALS_ROWS 32u
#define SEMICRF_MARGINALS_INTERVAL 64u
/* flags bit 8 (semicrf_logz_fwd, semicrf_fwd_bwd and their _boundary / _profiled / _static forms): the
 * low-memory plan.  With ckpt_interval = 0 the interval is the spacing of Algorithm 1, ceil(sqrt(T*K)) rounded
 * up to a multiple of 8, instead of the one that fills the chip, and the interval stage keeps 8 row buffers of
 * ckpt_interval positions per sequence instead of one per interval: it recomputes each interval's forward rows
 * from the checkpoint (the body of Algorithm 3) instead of taking them from the forward scan.  Everything
 * beyond the O(T*C) prefix arrays then grows like sqrt(T*K)*C per sequence: the paper's memory bound.  The
 * results are the same up to rounding; the call is several times slower.  The workspace must have been sized
 * with want_grad + 8 (8 forward only, 9 gradients); not combinable with SEMICRF_MARGINALS_ROWS. */
#define SEMICRF_LOW_MEMORY 256u
/* flags bits 9 and 10: the chunk-parallel scan tasks run with two waves each (one runs the positions' dependent
 * chains, one adds up the older window entries a block ahead) / with one wave each.  By default the library takes
 * two waves where the window is deep or the label set large (more than 32 durations per lane, or C > 32), where
 * that is the faster form.  Same results up to rounding; both at once are refused. */
#define SEMICRF_TWO_WAVE_SCAN 512u
#define SEMICRF_ONE_WAVE_SCAN 1024u
/* flags bit 7 (semicrf_viterbi only): trace back by pointer doubling over all nodes, the route otherwise taken
 * only when an interval's nodes do not fit in LDS.  Same back-pointers, same path; for tests of that route. */
#define SEMICRF_VITERBI_GLOBAL_TRACE 128u
/* flags bits 16..31: first warm-up length of the chunk-parallel scans, in positions (0 = the default, max(1.5K, 32);
 * the long second warm-up is four times this).  A length too short for the input costs time, never accuracy:
 * what does not verify is repaired or rescanned.  Tests use it to force those routes. */
#define SEMICRF_WARMUP(n) ((unsigned)(n) << 16)

int semicrf_version(void);

/* Host only.  Text for a status code; the pointer is static storage. */
const char *semicrf_strerror(int status);

/*
 * Host only, pure.  Bytes of device workspace the calls below need for these
 * sizes.  ckpt_interval = 0 selects the automatic interval: the multiple of 8 within
 * [max(8, K/2), sqrt(T*K)] (the upper end is the spacing of Algorithm 1) that minimises
 * the modelled time of the (sequence, interval) tasks, which run in rounds of about one
 * task per SIMD of the chip; roughly ceil(B*T/1024) when the K-deep window is small.
 * want_grad = 0 sizes for semicrf_logz_fwd / semicrf_cum_scores only; 1 for semicrf_fwd_bwd with the default
 * choice of marginal route (row slots for both scans); 2 for semicrf_fwd_bwd with SEMICRF_MARGINALS_INTERVAL
 * (the smallest); 3 is the same as 1.  A workspace sized with 1 serves every gradient call.
 * Add 8 for calls with SEMICRF_LOW_MEMORY (8 forward only, 9 or 10 gradients): another layout, for those
 * calls only.  `bytes` is a host pointer.
 */
int semicrf_workspace_bytes(int B, int T, int K, int C, int ckpt_interval, int want_grad,
                            size_t *bytes);

/*
 * Host only, pure.  The checkpoint interval (the Delta of Algorithm 1) the calls below
 * use for these sizes: ckpt_interval itself (clamped to T) when positive, else the
 * automatic choice described above.  `interval` is a host pointer.
 * semicrf_ckpt_interval_low_memory: the same for calls with SEMICRF_LOW_MEMORY.
 */
int semicrf_ckpt_interval(int B, int T, int K, int C, int ckpt_interval, int *interval);
int semicrf_ckpt_interval_low_memory(int B, int T, int K, int C, int ckpt_interval, int *interval);

/*
 * Eq. 1 and Eq. 2: per-sequence baseline and centred prefix sums.
 *   cum [B,T+1,C] double: cum[b,0,c] = 0, cum[b,t,c] = sum_{u<t} (emis[b,u,c] - nu[b,c])
 *   for t <= L_b; rows t > L_b are written as 0.
 * Workspace: as for want_grad = 0 with K = 1.
 */
int semicrf_cum_scores(const float *emis, const int32_t *lengths, int B, int T, int C,
                       unsigned flags, void *workspace, size_t workspace_bytes,
                       double *cum, void *stream);

/*
 * Algorithm 1 (streaming forward scan): logz[b] = log partition function of
 * sequence b.  logz [B] float.  The result does not depend on ckpt_interval (beyond
 * rounding order and the 1e-10 acceptance bound of the chunk-parallel scan).
 */
int semicrf_logz_fwd(const float *emis, const int32_t *lengths, const float *trans,
                     const float *dur, int B, int T, int K, int C, int ckpt_interval,
                     unsigned flags, void *workspace, size_t workspace_bytes,
                     float *logz, void *stream);

/*
 * Algorithm 1 + Algorithm 3 (forward scan, checkpointed backward pass) and the
 * gradient formulas.
 *   grad_logz [B] float or NULL: upstream weights w_b = dLoss/dlogZ_b (NULL = ones)
 * Outputs (all fully overwritten):
 *   logz       [B]     float
 *   grad_emis  [B,T,C] float  w_b * d logZ_b / d emis[b,u,c]; with SEMICRF_CENTER this
 *                             includes the Jacobian of the baseline subtraction; rows
 *                             u >= L_b are 0.  (Also used as scratch during the call.)
 *   grad_trans [C,C]   float  sum_b w_b * sum_{t,k} mu_b(t,k,c,c')   at [c'*C + c]
 *   grad_dur   [K,C]   float  sum_b w_b * sum_{t,c'} mu_b(t,k,c,c')  at [(k-1)*C + c]
 *   pos_marg   [B,T,C] float or NULL: posterior P(token u has label c), which is the
 *                             gradient of logZ_b w.r.t. the centred emission; rows
 *                             u >= L_b are 0.
 * For K >= 128 (when every checkpoint interval has a buffer slot of its own) the chunk-parallel
 * backward scan keeps its per-position rows as the forward scan does, and the expected
 * statistics of the "Gradient Formulas" section are formed as position-local products of the
 * two sets of rows instead of by a third recurrence per interval; sequences whose scans were
 * not both accepted take Algorithm 3's per-interval pass.  The results are the same to the
 * rounding of the outputs.  SEMICRF_MARGINALS_ROWS / SEMICRF_MARGINALS_INTERVAL select one route.
 */
int semicrf_fwd_bwd(const float *emis, const int32_t *lengths, const float *trans,
                    const float *dur, const float *grad_logz, int B, int T, int K, int C,
                    int ckpt_interval, unsigned flags, void *workspace, size_t workspace_bytes,
                    float *logz, float *grad_emis, float *grad_trans, float *grad_dur,
                    float *pos_marg, void *stream);

/*
 * For callers that cannot allocate device memory or pass a workspace: code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc.  semicrf_fwd_bwd with the
 * workspace taken from a static array in the library's device image instead of an argument:
 * SEMICRF_STATIC_WORKSPACE_BYTES per GPU, held by every GPU the library runs on until the process
 * ends.  The call allocates and frees nothing (no hipMalloc, hipFree or allocating library
 * routine); the first call on a device looks the array's address up once.  Inputs, outputs,
 * results and errors are those of semicrf_fwd_bwd; sizes whose semicrf_workspace_bytes(B, T, K, C,
 * ckpt_interval, want_grad) exceeds the limit return SEMICRF_EWORKSPACE before anything is launched
 * (want_grad as the flags ask: 1, 2 with SEMICRF_MARGINALS_INTERVAL, plus 8 with SEMICRF_LOW_MEMORY).
 * All calls on one GPU share that GPU's array: calls that may overlap in time on one GPU (two
 * streams, two host threads) race on it and must be serialised by the caller.  Nothing in the
 * array has to survive between calls and nothing in it is assumed zero: every call writes what
 * it later reads.  The device that is current when the call is made must be the stream's.
 */
#define SEMICRF_STATIC_WORKSPACE_BYTES (64u << 20)
int semicrf_fwd_bwd_static(const float *emis, const int32_t *lengths, const float *trans,
                           const float *dur, const float *grad_logz, int B, int T, int K, int C,
                           int ckpt_interval, unsigned flags, float *logz, float *grad_emis,
                           float *grad_trans, float *grad_dur, float *pos_marg, void *stream);

/*
 * The full edge potential of Eq. 4: the three terms above plus the optional boundary terms
 * of the "Boundary Projections" section and the scalar sequence boundaries of the appendix on
 * boundary handling.  A segment [s, s+k) with label c additionally scores
 *     proj_start[b, s, c] + proj_end[b, s+k-1, c]
 * (first and last TOKEN of the segment), plus pi_start[c] if s = 0 and pi_end[c] if
 * s+k = L_b (the scalars are added to the projections at token 0 / token L_b-1).
 *   proj_start, proj_end [B,T,C] float or NULL (= zeros); rows u >= L_b are never read
 *   pi_start, pi_end     [C]     float or NULL (= zeros)
 * With all four NULL these calls are semicrf_logz_fwd / semicrf_fwd_bwd.  Additional
 * outputs of the gradient call, each optional (NULL = not wanted), fully overwritten:
 *   grad_proj_start [B,T,C] float  w_b * P(a segment with label c starts at token u); rows u >= L_b are 0
 *   grad_proj_end   [B,T,C] float  w_b * P(a segment with label c ends with token u);  rows u >= L_b are 0
 *   grad_pi_start   [C]     float  sum_b w_b * P(first segment of b has label c)
 *   grad_pi_end     [C]     float  sum_b w_b * P(last segment of b has label c)
 *   bdy_post        [B,T+1] float  P(a segment boundary falls at position t): 1 at t = 0 and
 *                                  t = L_b, 0 for t > L_b (the boundary posterior of the paper's
 *                                  analysis; independent of grad_logz)
 * The score range bound of the header comment includes max|proj_start| + max|proj_end| + the
 * scalars.  Everything else as for semicrf_logz_fwd / semicrf_fwd_bwd.
 */
int semicrf_logz_fwd_boundary(const float *emis, const int32_t *lengths, const float *trans,
                              const float *dur, const float *proj_start, const float *proj_end,
                              const float *pi_start, const float *pi_end, int B, int T, int K, int C,
                              int ckpt_interval, unsigned flags, void *workspace, size_t workspace_bytes,
                              float *logz, void *stream);

int semicrf_fwd_bwd_boundary(const float *emis, const int32_t *lengths, const float *trans,
                             const float *dur, const float *grad_logz, const float *proj_start,
                             const float *proj_end, const float *pi_start, const float *pi_end, int B, int T,
                             int K, int C, int ckpt_interval, unsigned flags, void *workspace,
                             size_t workspace_bytes, float *logz, float *grad_emis, float *grad_trans,
                             float *grad_dur, float *pos_marg, float *grad_proj_start, float *grad_proj_end,
                             float *grad_pi_start, float *grad_pi_end, float *bdy_post, void *stream);

/*
 * Viterbi decode (the max-semiring counterpart of Algorithm 1; the paper's inference path):
 * the best-scoring segmentation under the edge potential of Eq. 4, boundary terms included
 * (each of the four may be NULL).  Same conventions as the sum: every initial label has score
 * 0, so the first segment pays max_c' trans[c',c]; no end term.
 *   score  [B]   float  score of the best segmentation (0 for an empty sequence)
 *   labels [B,T] int32  label of the segment that covers token u; -1 for u >= L_b
 *   starts [B,T] int32  1 on the first token of every segment, else 0 (0 for u >= L_b)
 *   nseg   [B]   int32  number of segments
 * Among equally good segmentations the last segment's label is the smallest, and going
 * backwards each segment takes the smallest duration, then the smallest predecessor label,
 * among the maximisers; since sums are rounded, "equally good" means equal in fp64.
 * Supported sizes: C <= 64 and K <= 64 * (64 / (C rounded up to 8/16/32/64)).  Workspace:
 * semicrf_viterbi_workspace_bytes (O(T*C): prefix arrays plus two doubles and four
 * integers per position and label).
 * The forward recurrence runs chunk-parallel like the sums: every checkpoint interval is
 * scanned on its own after a warm-up from the state of a sequence that begins there.  Best
 * paths that have merged give states equal up to one additive constant, so each interval
 * boundary is checked entry by entry (-inf entries must coincide) after removing that
 * constant, to 1e-12 relative to the larger of the entry and the prefix sums of Eq. 2 there
 * (the entries are differences of prefix sums, so that is the scale of their rounding); the
 * constants are chained in a fixed order.  Intervals whose start did not agree are scanned
 * once more after a longer warm-up; a sequence with a boundary that still does not agree
 * is rescanned sequentially inside the same call, and SEMICRF_SEQUENTIAL_SCAN forces that.
 * semicrf_scan_report with ckpt_interval = 0 and want_grad = 0 on this workspace reports
 * the outcome in column 0.  The trace-back (back-pointers of every node, pointer jumping
 * inside each interval, pointer doubling across intervals, one store per token) is parallel
 * either way.
 */
int semicrf_viterbi_workspace_bytes(int B, int T, int K, int C, size_t *bytes);

int semicrf_viterbi(const float *emis, const int32_t *lengths, const float *trans, const float *dur,
                    const float *proj_start, const float *proj_end, const float *pi_start,
                    const float *pi_end, int B, int T, int K, int C, unsigned flags, void *workspace,
                    size_t workspace_bytes, float *score, int32_t *labels, int32_t *starts, int32_t *nseg,
                    void *stream);

/*
 * Duration-dependent transitions: one transition matrix per duration, the generality whose
 * gradient the paper's gradient-workspace section allocates (a transition gradient with a
 * duration index).  The edge potential is that of Eq. 4 with trans3[k-1,c',c] in place of
 * trans[c',c]:
 *     psi(t,k,c,c') = S[t,c] - S[t-k,c] + dur[k-1,c] + trans3[k-1,c',c]      (no boundary terms)
 *   trans3      [K,C,C] float  trans3[((k-1)*C + c_src)*C + c_dst]
 *   grad_trans3 [K,C,C] float  sum_b w_b * sum_t mu_b(t,k,c,c')  at [((k-1)*C + c')*C + c]
 *   grad_dur    [K,C]   float  its sum over the source label (dur and trans3 enter together)
 * Everything else (emis, lengths, dur, grad_logz, flags, logz, grad_emis, pos_marg, stream,
 * errors) as for semicrf_logz_fwd / semicrf_fwd_bwd.  The transition no longer factors out
 * of the sum over durations, so a position costs K*C*C multiply-adds per recurrence.
 * Supported sizes: C <= 32, K <= 8 * floor(1024 / C) and C*C * ceil(K/64) <= 1024 (one label
 * pair per thread, at most 64 durations per thread in the backward recurrence);
 * SEMICRF_EUNSUPPORTED otherwise.  Workspace: semicrf_durtrans_workspace_bytes (that of
 * semicrf_workspace_bytes plus the K*C*C table, four O(T*C) arrays of stored messages and up
 * to 256 partial gradient tables).  semicrf_scan_report applies to this workspace too.
 */
int semicrf_durtrans_workspace_bytes(int B, int T, int K, int C, int ckpt_interval, int want_grad,
                                     size_t *bytes);

/* Host only, pure.  The checkpoint interval these calls use: ckpt_interval (clamped to T) when
 * positive, else their own automatic choice (tasks here are workgroups, not single waves: the
 * multiple of 8, at least max(8, K/2), that minimises rounds * (warm-up + interval)).  Pass it
 * as ckpt_interval to semicrf_scan_report. */
int semicrf_durtrans_ckpt_interval(int B, int T, int K, int C, int ckpt_interval, int *interval);

int semicrf_logz_fwd_durtrans(const float *emis, const int32_t *lengths, const float *trans3,
                              const float *dur, int B, int T, int K, int C, int ckpt_interval,
                              unsigned flags, void *workspace, size_t workspace_bytes, float *logz,
                              void *stream);

int semicrf_fwd_bwd_durtrans(const float *emis, const int32_t *lengths, const float *trans3,
                             const float *dur, const float *grad_logz, int B, int T, int K, int C,
                             int ckpt_interval, unsigned flags, void *workspace, size_t workspace_bytes,
                             float *logz, float *grad_emis, float *grad_trans3, float *grad_dur,
                             float *pos_marg, void *stream);

/*
 * The two entropies of the paper's boundary-entropy paragraph, from outputs of the calls above
 * (device pointers; needs no workspace):
 *   h_pos [B] float or NULL: mean over the L_b tokens of -sum_c pos_marg[b,u,c] ln pos_marg[b,u,c]
 *   h_bdy [B] float or NULL: -sum_{u<L_b} ph_u ln ph_u with ph_u = bdy_post[b,u] / sum_{u'<L_b} bdy_post[b,u']
 *                            (a segment starts at token u iff a boundary falls at position u); ln L_b at K = 1
 * pos_marg [B,T,C] is needed for h_pos, bdy_post [B,T+1] for h_bdy; at least one output must be
 * given.  Empty sequences give 0.
 */
int semicrf_entropies(const float *pos_marg, const float *bdy_post, const int32_t *lengths, int B, int T,
                      int C, float *h_pos, float *h_bdy, void *stream);

/*
 * Measurement aid: semicrf_fwd_bwd with five caller-owned HIP events recorded on
 * `stream`: stage_events[0] before the first kernel and stage_events[1..4] after
 * each of the four stages
 *   1 prefix sums (Eq. 1-2 kernels),
 *   2 the two scans (Algorithm 1 and the beta recurrence of Algorithm 3; chunk-parallel with verification,
 *     repair and the sequential fallback),
 *   3 per-interval recompute + marginals (Algorithm 3 body),
 *   4 fixed-order reductions of the gradient formulas.
 * stage_events is a HOST array of 5 hipEvent_t handles created by the caller
 * with timing enabled; the library neither creates, waits on nor destroys them
 * (the caller synchronises and calls hipEventElapsedTime).  Results are
 * identical to semicrf_fwd_bwd.
 */
int semicrf_fwd_bwd_profiled(const float *emis, const int32_t *lengths, const float *trans,
                             const float *dur, const float *grad_logz, int B, int T, int K, int C,
                             int ckpt_interval, unsigned flags, void *workspace,
                             size_t workspace_bytes, float *logz, float *grad_emis,
                             float *grad_trans, float *grad_dur, float *pos_marg, void *stream,
                             void *const *stage_events);

/*
 * Diagnostics of the scans of the LAST semicrf_logz_fwd / semicrf_fwd_bwd call that used
 * this workspace with these sizes (same B, T, K, C, ckpt_interval and want_grad: they
 * locate the fields in the workspace).  Enqueued on `stream` after that call.
 *   accepted [B,2] int32 device, or NULL: [b,0] forward scan (Algorithm 1), [b,1] backward
 *             scan (Algorithm 3): > 0 = the chunk-parallel result was verified and used:
 *             1 at the first attempt, 2 after the intervals whose start had disagreed were
 *             rerun from the state their neighbour reached, 3 after the long warm-up;
 *             0 = the sequential scan computed it (flag SEMICRF_SEQUENTIAL_SCAN, sizes the
 *             chunk-parallel kernels do not cover, a direction that call did not run, or
 *             a boundary that did not agree).
 *   mismatch [B,2] double device, or NULL: largest relative disagreement over the chunk
 *             boundaries of that scan; -1 where the chunk-parallel scan was not attempted.
 * At least one of the two must be given.
 */
int semicrf_scan_report(const void *workspace, size_t workspace_bytes, int B, int T, int K, int C,
                        int ckpt_interval, int want_grad, int32_t *accepted, double *mismatch,
                        void *stream);

/*
 * Per-sequence results the LAST semicrf_logz_fwd / semicrf_fwd_bwd call (or their _boundary forms) left in
 * this workspace; sizes and want_grad as for semicrf_scan_report.  Enqueued on `stream` after that call.
 *   range_exceeded [B] int32 device, or NULL: 1 if the scores of sequence b exceed the range the scaled
 *             recurrences are built for: with r = max|f - nu| + max(0, max dur) + max(0, max trans) + ln(K*C)
 *             (or the same with the minima; boundary terms added), one position may change the messages by
 *             e^r, and r must stay below 300 nats so that a product of two scaled factors stays inside the
 *             double range (Eq. 2 is what keeps f - nu small).  logZ and the gradients of such a sequence may
 *             be inf or NaN; nothing else is affected.  0 otherwise.
 *   logz64 [B] double device, or NULL: logZ_b as the forward scan computed it, before rounding to float
 *             (at T = 100 000 a float holds logZ to about 0.03 absolute).
 * At least one of the two must be given.
 */
int semicrf_seq_report(const void *workspace, size_t workspace_bytes, int B, int T, int K, int C,
                       int ckpt_interval, int want_grad, int32_t *range_exceeded, double *logz64, void *stream);

#ifdef __cplusplus
}
#endif
#endif /* SEMICRF_H */
