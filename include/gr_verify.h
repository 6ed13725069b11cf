/*
 * gr_verify.h -- C ABI of the MI355X Global Resolution verifier.
 *
 * The library computes, for a batch of B decode positions, the optimal multi-draft
 * verification distribution of "Global Resolution: Optimal Multi-Draft Speculative
 * Sampling via Convex Minimization" (Thomas & Pal) for n i.i.d. drafts from one draft
 * distribution q (optionally top-k restricted) against a target distribution p:
 *
 *   gr_solve   Alg. 1 lines 1-2 and both truncated convex programs:
 *              top-k support (App. "Top-k Sampling for the Relaxed OTLP"), the order by
 *              decreasing q/p and H*, alpha* = 1 + psi(H*) (Thm 3.1, Sec. 5.1), the outer
 *              targets p_i (Thm 6.2, Lemma 6.3), the softmax weights that minimise
 *              Theta_T (Thm 6.5) and Phi_T (Thm 6.4, solved per block of the outer system).
 *   gr_accept_sweep  alpha* alone over a grid of top-k sizes and draft counts (Thm 3.1, Sec. 5.1).
 *   gr_verify  the transport slice pi(.|drafts) (Eq. "cases" / Eq. "approx-c") and one
 *              inverse-CDF draw from it (App. A, multi-draft procedure, step 3).
 *   gr_solve_verify, gr_solve_logits_verify  the two steps in one call.
 *
 * Conventions
 *   - every pointer argument except `out`, `cfg` and host-side scalars is a DEVICE pointer
 *     owned by the caller; the library never frees or keeps them beyond what is stated;
 *   - all work is enqueued on `hip_stream` (a hipStream_t passed as void*; NULL = the
 *     default stream); gr_solve, gr_accept_sweep, gr_verify and the inspection calls neither
 *     allocate nor synchronise with the host (gr_create / gr_destroy allocate and free, and
 *     gr_profile_read waits for its events);
 *   - return value 0 = success, negative = call-level error (see GR_E*).  Argument and state errors
 *     (GR_EINVAL, GR_ESTATE, GR_EUNSUPPORTED) are found before anything is enqueued; GR_EHIP reports
 *     a failed launch, possibly after earlier kernels of the same call were enqueued: the handle then
 *     holds no policy (GR_ESTATE until the next successful gr_solve).  Per-row conditions never fail a
 *     call, they set status[b].
 *   - calls on one handle must not overlap in time (the handle owns scratch and the
 *     policy of the last gr_solve).
 */
#ifndef GR_VERIFY_H
#define GR_VERIFY_H

#ifdef __cplusplus
extern "C" {
#endif

typedef struct gr_handle_s* gr_handle;

/* call-level errors */
#define GR_OK            0
#define GR_EINVAL       (-1)   /* bad shape / parameter, or beyond the handle's capacity */
#define GR_ENOMEM       (-2)   /* device allocation failed */
#define GR_ESTATE       (-3)   /* gr_verify / gr_policy_* before a successful gr_solve */
#define GR_EHIP         (-4)   /* a HIP runtime call failed */
#define GR_EUNSUPPORTED (-5)   /* V >= 2^24 with a support above GR_MAX_SUPPORT; dense export of such a policy */
#define GR_ECAPACITY    (-6)   /* more rows than the fixed scratch of gr_accept_sweep_noalloc holds */

/* per-row status written by gr_solve */
#define GR_ROW_OK         0
#define GR_ROW_TRUNC_CAP  1    /* a program needed more than max_T variables (App. "Truncated Solver Details") */
#define GR_ROW_ITER_CAP   2    /* iteration cap reached before the gradient criterion (same appendix) */
#define GR_ROW_BAD        3    /* NaN / negative entry, or a row sum further than 1e-3 from 1 */

#define GR_MAX_SUPPORT  256    /* largest top-k support (|V_0|) the LDS-resident path holds */
#define GR_MAX_T        128    /* largest number of variables of one convex program */
#define GR_MAX_N         16    /* largest number of drafts */

typedef struct {
    int    max_iter;   /* cap on the evaluations of the routed masses of ONE convex program (App. "Truncated Solver
                          Details": iteration cap of the minimiser); <= 0 selects 1000 */
    int    max_T;      /* cap on the variables of one program; <= 0 or > GR_MAX_T selects GR_MAX_T */
    double rel_tol;    /* stop when every routed mass is within this relative distance of its
                          target (this implies Alg. 1's  ||grad||_1 <= 5*tol); <= 0 selects 1e-8, an order
                          above the error of the quadrature behind the routed masses */
    int    flags;      /* 0, or GR_FLAG_PROFILE */
    double tail_mass;  /* nucleus (top-p) cut of the draft (Sec. 5.1: top-p/k sampling of the draft restricts the
                          domain; App. A): the support is the fewest tokens by decreasing q (ties: lower token id)
                          whose running sum reaches (1 - tail_mass) of the row's q mass, cut further to the top k
                          when a top-k is given; drafts must then be drawn from q renormalised over that support.
                          As an approximation of the uncut draft it moves alpha* and the coupling by at most
                          n * tail_mass.  0: no cut; must lie in [0, 1).  Rows given as logits do not take it
                          (gr_solve_logits on such a handle returns GR_EUNSUPPORTED) */
} gr_config;

#define GR_FLAG_PROFILE 1      /* record HIP events around every kernel launch (see gr_profile_read) */

/* Create a handle able to serve up to max_B rows of up to max_V tokens, supports (top-k sizes, App. "Top-k
 * Sampling for the Relaxed OTLP") of up to max_k tokens (max_k <= 0 or >= max_V: whole rows, no top-k) and
 * up to max_n drafts (1..GR_MAX_N).  cfg may be NULL.
 * Device memory held by the handle until gr_destroy: about 150 KB per row (candidate keys, the policy
 * object of GR_MAX_SUPPORT entries, the Jacobian scratch of the solver's Newton fallback) plus 8 bytes per
 * 256 tokens and row; when max_k exceeds GR_MAX_SUPPORT, also 128 bytes per token of max_V and row (supports
 * that large are ordered, scanned and kept in HBM; max_V must then stay below 2^24, otherwise
 * GR_EUNSUPPORTED).  GR_ENOMEM if it cannot be allocated. */
int gr_create(gr_handle* out, int max_B, int max_V, int max_k, int max_n, const gr_config* cfg);
int gr_destroy(gr_handle h);

/*
 * p, q        [B, V] float32 row-major, each row a distribution (q before top-k).
 * n           number of i.i.d. drafts per row, 1..max_n of the handle.
 * k           top-k applied to q (ties: lower token id); k <= 0 or k >= V means none.
 *             A support above GR_MAX_SUPPORT (no top-k on a larger V, or a larger top-k) needs a handle
 *             created with max_k at least that large (GR_EINVAL otherwise): it lives in the handle's
 *             HBM workspace.
 * tol         the paper's error threshold tau (Alg. 1), >= 0: truncation sets are the fewest
 *             tokens by decreasing q with gamma_T <= tol (inner) / epsilon_T <= tol (outer).
 * accept_prob [B] float32 out: alpha* (Thm 3.1).       status [B] int32 out: GR_ROW_*.
 * The per-row policy stays inside the handle until the next gr_solve.
 */
int gr_solve(gr_handle h, const float* p, const float* q, int n, int k, float tol,
             int B, int V, float* accept_prob, int* status, void* hip_stream);

/*
 * gr_solve for rows given as logits (App. A, first paragraph: temperature and top-k sampling only change how p
 * and q are computed from the models' logits; Sec. 5.1 for the order): p = softmax(target_logits / T),
 * q = softmax(draft_logits / T) with one temperature per row, never written to memory.  One pass over both
 * rows keeps the k largest draft logits (they are the k largest q; ties: lower token id) and the target's
 * softmax normaliser (online, in float64); the supports' p and q are float64 exponentials, and every order the method needs is decided on the logits
 * themselves: decreasing q/p is decreasing (draft - target) logit, exact for float32 logits.
 *
 * target_logits, draft_logits [B, V] float32 row-major, finite (a NaN or infinite entry gives GR_ROW_BAD).
 * temperature [B] float32, positive and finite (GR_ROW_BAD otherwise): the target's, and the draft's too when
 *             draft_temperature is NULL.
 * draft_temperature [B] float32 or NULL: the draft's own temperature (the paper's temperature study cools the target
 *             and leaves the draft at 1).  q/p is then proportional to exp(d / Td - t / Tt); its order is taken on that
 *             value in float64 (two rounded products, one subtraction).
 * k           top-k on the draft, as in gr_solve (a support above GR_MAX_SUPPORT runs on the HBM-resident path, where
 *             the orders are sorts on the draft logit and on draft minus target logit, and needs a handle created
 *             with max_k at least that large).  A handle with tail_mass > 0 gives GR_EUNSUPPORTED.
 * Everything else as gr_solve.  target_logits and temperature must stay valid until the last gr_verify /
 * gr_policy_slice on this solve: they stand in for the p row there.
 */
int gr_solve_logits(gr_handle h, const float* target_logits, const float* draft_logits, const float* temperature,
                    const float* draft_temperature, int n, int k, float tol, int B, int V, float* accept_prob,
                    int* status, void* hip_stream);

/*
 * Acceptance-only sweep: alpha*(k, n) = 1 + min_H psi(H) (Thm 3.1; by the order of decreasing q/p
 * and the best prefix, Sec. 5.1) for every top-k size in ks and every number of i.i.d. drafts in ns,
 * from one streaming pass over p and q: the quantity of the paper's acceptance-versus-(k, n) study
 * (Sec. 7, first experiment; top-k as in App. "Top-k Sampling for the Relaxed OTLP").  No convex
 * program runs.
 * p, q        [B, V] float32 device arrays, as for gr_solve.
 * ks          HOST array of nk top-k sizes, 1 <= nk <= GR_SWEEP_MAX_K; k <= 0 or k >= V means no top-k.  When every
 *             k is at most GR_MAX_SUPPORT the grid is served from one streaming pass; otherwise (the study runs k
 *             up to the whole vocabulary) the handle must have been created with max_k at least the largest
 *             (GR_EINVAL otherwise) and the whole grid runs on the HBM-resident ordering: one sort by q/p, one
 *             by q, masked prefix scans.
 * ns          HOST array of nn draft counts, 1 <= nn <= GR_SWEEP_MAX_N, each 1..GR_SWEEP_MAX_DRAFTS.
 * accept_prob [B, nk, nn] float32 device out (NaN for a bad row).   status [B] int32 device out:
 *             GR_ROW_OK or GR_ROW_BAD.
 * Overwrites the handle's selection scratch: the policy of an earlier gr_solve is gone
 * (gr_verify returns GR_ESTATE until the next gr_solve).
 */
#define GR_SWEEP_MAX_K        8
#define GR_SWEEP_MAX_N       16
#define GR_SWEEP_MAX_DRAFTS  64
int gr_accept_sweep(gr_handle h, const float* p, const float* q, const int* ks, int nk, const int* ns, int nn,
                    int B, int V, float* accept_prob, int* status, void* hip_stream);

/*
 * gr_accept_sweep for callers that cannot allocate device memory or create a handle: code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments, outputs and arithmetic as
 * gr_accept_sweep, without the handle, for top-k sizes of 1..GR_MAX_SUPPORT (GR_EINVAL beyond: the HBM-resident
 * ordering lives in a handle's workspace); the selection scratch (candidate keys and partial sums, 16.2 KB per row)
 * is a fixed array in the library's device image, so B is limited to GR_NOALLOC_MAX_B rows (GR_ECAPACITY
 * beyond; 4.2 MB per GPU, held until the process ends).  The call allocates nothing, frees nothing and does
 * not synchronise.  The array's address on the current device is looked up on the first call on that device
 * (and by any gr_create on it): make that first call outside a graph capture.  Every call on a GPU uses
 * that GPU's one array: calls that overlap in time on one GPU race, whatever their streams.  Nothing in the
 * array needs clearing between calls (every entry a call reads was written by that call).
 */
#define GR_NOALLOC_MAX_B 256
int gr_accept_sweep_noalloc(const float* p, const float* q, const int* ks, int nk, const int* ns, int nn,
                            int B, int V, float* accept_prob, int* status, void* hip_stream);

/*
 * drafts   [B, n] int32 token ids drawn from the top-k renormalised q rows.
 * uniforms [B] float32 in [0, 1): one uniform per row.
 * token    [B] int32 out: x0 ~ pi(.|drafts); inverse-CDF entry order = distinct drafts in
 *          order of first appearance, then all other tokens by ascending id.
 * accepted [B] uint8 out: 1 iff token is one of the row's drafts.
 * Rows whose status is not GR_ROW_OK draw from p itself (the valid fallback transport of
 * App. "Multi-Step Experiments").  A draft outside the support gives token -1, accepted 0.
 * p must be the array passed to the last gr_solve and still hold the same values.
 */
int gr_verify(gr_handle h, const int* drafts, const float* uniforms,
              int* token, unsigned char* accepted, void* hip_stream);

/*
 * gr_solve followed by gr_verify as one call, for callers that hold the drafts when they ask for the solve (the
 * verification step of Sec. 3.1: the drafts are drawn before the verifier runs).  Arguments, outputs, order of the
 * sampled tokens and error codes are those of the two calls (all device pointers; drafts [B, n], uniforms [B]); the
 * results are identical to theirs.  With a support of at most GR_MAX_SUPPORT tokens the workgroup that solved a row
 * verifies it in the same launch, as soon as the row's policy is written, so that the verification of the rows that
 * finish early hides behind the rows that still iterate; larger supports run the two steps one after the other.  The
 * handle keeps the policy as after gr_solve (gr_verify, gr_policy_* may follow).
 */
int gr_solve_verify(gr_handle h, const float* p, const float* q, int n, int k, float tol, int B, int V,
                    const int* drafts, const float* uniforms, float* accept_prob, int* status,
                    int* token, unsigned char* accepted, void* hip_stream);

/* The same for rows given as logits: gr_solve_logits followed by gr_verify as one call (arguments of the two). */
int gr_solve_logits_verify(gr_handle h, const float* target_logits, const float* draft_logits, const float* temperature,
                           const float* draft_temperature, int n, int k, float tol, int B, int V,
                           const int* drafts, const float* uniforms, float* accept_prob, int* status,
                           int* token, unsigned char* accepted, void* hip_stream);

/* Test / inspection entry points --------------------------------------------------- */

/*
 * Multi-step verification over a tree of draft paths (App. "Multi-Step Experiments": K i.i.d. paths of length L
 * are drafted autoregressively from the draft model; the verifier advances from the root with n = the number of
 * drafted continuations of the current node until it lands off the tree; a row whose solve fails is sampled from p).
 * For each of S sequences and each level, sequences are grouped by n; every group is gathered, solved with
 * gr_solve(n) and sampled with gr_verify, and the paths that drew the emitted token go on to the next level.
 *
 * p, q       DEVICE [S, K, L, V] float32: the target / draft distribution after the first l tokens of path a of
 *            sequence s (paths with equal prefixes must carry equal rows; level 0 is the same row for all paths).
 * temperature HOST [S] float32 or NULL.  Not NULL: p and q hold the models' logits and every level is solved with
 *            gr_solve_logits at the sequence's temperature.
 * paths      HOST [S, K, L] int32 drafted tokens (path a's token l drawn from the top-k renormalised q row (s, a, l)).
 * uniforms   HOST [S, L] float32 in [0, 1), one per level.
 * k, tol     as in gr_solve.  K <= max_n and S <= max_B of the handle.
 * out_tokens HOST [S, L] int32: the tokens emitted, -1 beyond the last.  out_len [S]: how many (the walk emits one
 *            token per level visited; no bonus token after a fully accepted tree).  out_accepted [S]: how many of
 *            them were drafts.  out_fallbacks [S] or NULL: levels whose row had a status other than GR_ROW_OK.
 * The first call allocates staging for max_B rows of max_V tokens (8 max_V bytes per row; GR_ENOMEM); every call
 * synchronises the stream once per level and group, and leaves the handle without a policy (GR_ESTATE for a
 * gr_verify that follows).
 */
int gr_tree_walk(gr_handle h, const float* p, const float* q, const float* temperature, const int* paths,
                 const float* uniforms, int S, int K, int L, int V, int k, float tol,
                 int* out_tokens, int* out_len, int* out_accepted, int* out_fallbacks, void* hip_stream);

/* Dense slice of the transport for the drafted tuple, normalised by pdraft(drafts) (Eq. "cases" with
 * the residual lift of Eq. (3); Eq. "approx-c" when truncated; Alg. 1 "return normalized C"):
 * pi [B, V] float32 out = pi(.|drafts);  accept_given_drafts [B] float32 out = sum of pi over the row's
 * distinct drafts.  drafts [B, n] int32 with B, n of the last gr_solve. */
int gr_policy_slice(gr_handle h, const int* drafts, float* pi, float* accept_given_drafts,
                    void* hip_stream);

/* Per-row policy object, each array [B, GR_MAX_SUPPORT] (entries beyond support[b] are
 * unspecified): order = token ids by decreasing q/p (Sec. 5.1); block = 0 for H* (Thm 3.1), b >= 1 for the
 * b-th outer block (ranks between two consecutive suffix-minimum records of psi, Lemma 6.3);
 * weight = e^{alpha_i}, the softmax parameters of Thm 6.5 (inside H*) / Thm 6.4 (outside), float64;
 * rho = p(i) - p_i, the outer residuals of Thm 6.2, float64.  The weights of a row whose status is not GR_ROW_OK
 * are unspecified (such a row is sampled from p).
 * support, h_size, iterations: [B] int32.  Any pointer may be NULL. */
int gr_policy_export(gr_handle h, int* order, int* block, double* weight, double* rho,
                     int* support, int* h_size, int* iterations, void* hip_stream);

/* One row of the policy object (Thm 6.2 residuals, Thm 6.4 / 6.5 weights, as above), the first `count`
 * ranks (count <= the row's support): the same arrays as gr_policy_export.  This is the only export of a policy over a support above
 * GR_MAX_SUPPORT, whose rows hold up to V entries.  Device pointers, any may be NULL. */
int gr_policy_export_row(gr_handle h, int row, int count, int* order, int* block, double* weight,
                         double* rho, void* hip_stream);

/* Work done by the last gr_solve, per row ([B] device arrays, either may be NULL):
 * evaluations = calls of the routed-mass evaluator (one per fixed-point or Newton step, plus
 * the finite-difference columns of a Newton Jacobian); node_tokens = sum over those calls of
 * (quadrature nodes x active tokens of the program), the unit in which the arithmetic of the
 * generating-function evaluator of Sec. 6.3's objectives is counted: one call costs about
 * 4 n^2 floating-point operations per (node, token) pair. */
int gr_solve_stats(gr_handle h, int* evaluations, double* node_tokens, void* hip_stream);

/* Measurement hook (handles created with GR_FLAG_PROFILE): average duration in milliseconds of
 * the streaming selection kernel, the per-row solve kernel (both launched by gr_solve) and the
 * verification kernel, over the gr_solve + gr_verify pairs issued since the last read (at most
 * 512 are kept), from HIP events recorded on the caller's stream.  Waits for the last of them.
 * With a support above GR_MAX_SUPPORT, select_ms covers the ordering, scan and truncation kernels
 * in HBM and solve_ms the kernel that runs the convex programs.
 * All four outputs are HOST pointers. */
int gr_profile_read(gr_handle h, double* select_ms, double* solve_ms, double* verify_ms, int* steps);

/* Measurement hook: record the events of GR_FLAG_PROFILE only on every stride-th gr_solve (and the gr_verify that
 * follows it), so that a timed loop is not slowed by five event records per step.  stride >= 1 (GR_EINVAL);
 * GR_ESTATE on a handle created without GR_FLAG_PROFILE.  The count starts again with the next gr_solve. */
int gr_profile_stride(gr_handle h, int stride);

const char* gr_strerror(int code);

#ifdef __cplusplus
}
#endif
#endif /* GR_VERIFY_H */
