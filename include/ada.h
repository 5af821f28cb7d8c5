/*
 * ada.h -- C ABI of libada: Gram-threshold representative-token selection and the
 * cascade step on one AMD MI355X (gfx950).
 *
 * Conventions for every call
 *   - X is a DEVICE pointer to a row-major T x d activation matrix (row t = hidden
 *     state of token t, Section 2.1 of the paper) with leading dimension ld >= d,
 *     counted in elements.  dtype says how elements are stored (ada_dtype).
 *   - All output buffers and the workspace are DEVICE memory owned by the caller.
 *     The library allocates no device memory and keeps no state between calls; the
 *     only state between layers is the index set R^(l), which the caller carries
 *     (Algorithm 1, "Require").
 *   - stream is a hipStream_t passed as void* (NULL = the default stream).  Calls
 *     only enqueue work; outputs are valid once the caller has synchronised the
 *     stream.  Two calls that share a workspace must be ordered on one stream.
 *   - The return value is an ada_status.  Everything the host can check (null
 *     pointers, shapes, tau, workspace size, dtype) is reported synchronously and
 *     nothing is enqueued in that case.  A bad inherited index list is found on the
 *     device and reported in counts[3] (see ada_cascade_step).
 *   - Non-finite inputs are outside the contract.
 */
#ifndef ADA_H
#define ADA_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    ADA_OK = 0,
    ADA_ERR_NULL = 1,      /* a required pointer is NULL */
    ADA_ERR_SHAPE = 2,     /* T < 1, d < 1, ld < d, r < 1, r > T, L < 1, T too large */
    ADA_ERR_TAU = 3,       /* tau outside the open interval (0,1) (Definition "Gram threshold") */
    ADA_ERR_INDEX = 4,     /* inherited indices not strictly ascending / out of range (device-detected) */
    ADA_ERR_WORKSPACE = 5, /* workspace smaller than ada_workspace_bytes(T) or misaligned */
    ADA_ERR_DEVICE = 6,    /* a HIP call failed */
    ADA_ERR_DTYPE = 7      /* unknown ada_dtype */
} ada_status;

typedef enum {
    ADA_F32 = 0, /* IEEE binary32 elements; products and sums in fp32 */
    ADA_BF16 = 1 /* bfloat16 elements; exact products, fp32 accumulation */
} ada_dtype;

/* flags */
#define ADA_FLAG_CROSS_EARLIER_ONLY 1u /* cascade: compare a non-representative t only with valid
                                          representatives s < t (the form the proof of the superset
                                          proposition uses) instead of all of them (Algorithm 1, step 8) */

#define ADA_FLAG_TWO_PASS 2u           /* cascade: run the r x r Gram and the cross-Gram as separate launches instead of
                                          the one-launch form.  Same results (sets, counts, gram_ops, gamma) */

#define ADA_FLAG_RESIDENT_PASS 4u      /* ada_cascade_layers: run the cascade layers (up to 64 per launch) in ONE launch whose
                                          workgroups stay resident and hand the set from layer to layer through device memory,
                                          instead of one launch per layer.  Same results.  It needs every CU of the device for
                                          itself (one workgroup per CU must be resident at once) and rows in whole, aligned
                                          128-byte chunks; otherwise the flag is ignored.  The wait between layers is bounded:
                                          if it runs out, the kernel ends and the unfinished layers report ADA_ERR_DEVICE in
                                          their counts (initialise the workspace again after that) */

#define ADA_FLAG_ATTN_CAUSAL 8u        /* ada_attention_compressed: a representative attends only to members of R that are
                                          not later than itself in the sequence (eq. (1) prints no mask; the decoder-only
                                          models of Section 6 have one) */

#define ADA_FLAG_GREEDY_COVER 16u       /* ada_select_full: the greedy covering of Section 2.5 instead of the Definition: token t
                                          is a representative iff no earlier REPRESENTATIVE s has |G_st| >= 1 - tau^2 (the
                                          Definition compares with all earlier tokens; the two differ exactly on chains
                                          a ~ b ~ c with a not ~ c).  The decisions are sequential in t: the Gram tiles leave one
                                          bit per pair s < t, and one workgroup resolves them in token order.  T <= 16384.
                                          The gamma output is still the Definition's (max over ALL earlier tokens) */

#define ADA_MAX_T (1 << 20)
#define ADA_MAX_BATCH 4096

/* Human-readable name of a status code (static storage). */
const char* ada_status_string(int status);

/* Bytes of device workspace a call with this T needs (256-byte aligned base required). */
size_t ada_workspace_bytes(int T);

/*
 * Zero-fills a workspace (one small kernel on the stream).  A workspace must be zero-filled once, by this call or
 * by any memset, before its first use; every library call leaves it ready for the next one (it holds counters that
 * the last workgroup of a launch resets).  If a call is abandoned part-way (device error), initialise it again.
 * Calls that share a workspace must not overlap in time.
 */
int ada_workspace_init(void* ws, size_t ws_bytes, void* stream);

/*
 * Full ("independent") selection -- Definition "Gram threshold" (Section 2.2):
 *   gamma_t = max_{s<t} |G_st|,  G = Xhat Xhat^T with Xhat the row-normalised X (Section 2.1);
 *   token t is representative iff gamma_t < 1 - tau^2.  A zero row has all cosines 0.
 * Outputs
 *   mask  [T] uint8   1 = representative                                   (required)
 *   idx   [T] int32   the representatives' token ids, ascending; first *count entries valid (may be NULL)
 *   count [4] int32   {r, r, 0, 0}: same layout as ada_cascade_step's counts so that it can be
 *                     handed on as r_dev of the next layer                 (required)
 *   gamma [T] float   gamma_t                                              (may be NULL)
 */
int ada_select_full(const void* X, int T, int d, int64_t ld, int dtype, float tau,
                    uint8_t* mask, int32_t* idx, int32_t* count, float* gamma,
                    void* ws, size_t ws_bytes, void* stream, unsigned flags);

/*
 * One cascade step -- Algorithm 1 (Section 4.1) on X = X^(l+1):
 *   validate the inherited set R^(l) with the r x r Gram among its rows
 *   (gamma^rep_s = max over inherited s' < s, R_valid = {gamma^rep < 1 - tau^2}),
 *   test every other token against R_valid with the (T-r) x r_valid cross-Gram
 *   (gamma^cross_t, R_new = {gamma^cross < 1 - tau^2}), return R_valid u R_new.
 * Inputs
 *   prev_idx  device int32, strictly ascending token ids of R^(l)
 *   r         number of valid entries in prev_idx if r_dev is NULL; otherwise an upper bound on it
 *             (the capacity of prev_idx, at most T)
 *   r_dev     optional device int32 holding |R^(l)| (e.g. counts[0] of the previous step), so that
 *             layers can be chained without a host round trip
 * Outputs
 *   idx      [T] int32  R^(l+1), ascending
 *   adds     [T] int32  R_new, ascending
 *   removes  [r] int32  R^(l) \ R_valid, ascending
 *   counts   [4] int32  {|R^(l+1)|, |adds|, |removes|, status}; status is ADA_OK or ADA_ERR_INDEX /
 *                       ADA_ERR_SHAPE for a bad prev_idx / r_dev, in which case the sizes are 0
 *   gram_ops [1] uint64 r^2 + (T-r) * r_valid Gram entries (eq. (6) counts T*r, which is the same
 *                       when nothing is removed; one operation = one Gram entry as in Table 6)  (may be NULL)
 *   gamma    [T] float  (may be NULL) Algorithm 1's maxima: gamma^rep (step 4) for an inherited token, gamma^cross (step 8,
 *                       over the VALID representatives) for any other, 0 where the maximum is empty.  (With
 *                       ADA_FLAG_CROSS_EARLIER_ONLY only earlier representatives enter either maximum.)  In the one-launch
 *                       form validity is known only after the products, so asking for gamma adds a small second launch
 *                       that recomputes the tokens whose nearest inherited representative was removed; sets and counts
 *                       never depend on it.
 * The one-launch form is used for T <= 16384; larger T always takes the two-launch form.
 * Output buffers must not overlap the inputs (prev_idx in particular: idx is written while prev_idx is still read).
 */
int ada_cascade_step(const void* X, int T, int d, int64_t ld, int dtype, float tau,
                     const int32_t* prev_idx, int r, const int32_t* r_dev,
                     int32_t* idx, int32_t* adds, int32_t* removes, int32_t* counts,
                     uint64_t* gram_ops, float* gamma,
                     void* ws, size_t ws_bytes, void* stream, unsigned flags);

/*
 * ada_cascade_step for callers that cannot allocate device memory: code under HIP graph capture, tight serving
 * loops, harnesses that forbid allocation.  Same arguments, outputs, flags and results as ada_cascade_step, without a
 * workspace: the step's scratch memory (row maxima, hit table, counters; about 2.2 MB) is an array in the library's
 * own image, one copy per GPU for the life of the process.  The call allocates nothing and frees nothing.
 *   T <= ADA_STATIC_MAX_T, else ADA_ERR_SHAPE (nothing is enqueued).
 * Every call on a GPU uses that GPU's one array: calls that overlap in time on one GPU (different streams, or threads)
 * race and must be ordered by the caller.  What must start at zero is cleared at the start of each call (by a small
 * kernel, so the call can be captured), whatever an earlier call left behind.
 */
#define ADA_STATIC_MAX_T 4096
int ada_cascade_step_static(const void* X, int T, int d, int64_t ld, int dtype, float tau,
                            const int32_t* prev_idx, int r, const int32_t* r_dev,
                            int32_t* idx, int32_t* adds, int32_t* removes, int32_t* counts,
                            uint64_t* gram_ops, float* gamma, void* stream, unsigned flags);

/*
 * Nearest-representative assignment -- Section 2.3 ("Attention on the representative set"): a token outside R
 * takes the attention output of the member s* of R that maximises |G_{t s*}|.  The maximum runs over the whole
 * set handed in (earlier and later tokens alike); a member of R is its own representative.  One launch: the
 * T x r products on the cascade step's tile engine with an arg-max epilogue.
 * Inputs
 *   idx    device int32, strictly ascending token ids of R (the idx output of ada_select_full or ada_cascade_step)
 *   r      number of entries if r_dev is NULL, otherwise an upper bound (capacity of idx, at most T)
 *   r_dev  optional device int32 holding |R| (e.g. counts[0] of the call that produced idx)
 * Outputs
 *   assign [T] int32  token id of s*(t); t itself for t in R.  Among representatives whose |cosine| to t is equal
 *                     in the fp32 arithmetic of the kernel the smallest token id is taken.
 *   corr   [T] float  |G_{t s*(t)}|, 1 for t in R                                     (may be NULL)
 *   info   [4] int32  {T - r (tokens represented by another token), 0, 0, status}; status is ADA_OK, or
 *                     ADA_ERR_INDEX / ADA_ERR_SHAPE for a bad idx / r_dev, and then assign / corr hold no result
 * Errors the host can see (null pointers, shapes, workspace) are returned before anything is enqueued.
 */
int ada_assign_nearest(const void* X, int T, int d, int64_t ld, int dtype,
                       const int32_t* idx, int r, const int32_t* r_dev,
                       int32_t* assign, float* corr, int32_t* info,
                       void* ws, size_t ws_bytes, void* stream, unsigned flags);

/*
 * Attention on the representative set -- eq. (1) (Section 2.3): per head,
 *   O_R = softmax(Q_R K_R^T / sqrt(d_h)) V_R      on the r representative rows (r x r instead of T x T),
 * and every token takes the output row of its representative: out[t] = O_R[position of assign[t] in R].
 * Inputs
 *   Q, K, V  device, row-major T x (H * d_h), heads side by side, leading dimension ld (elements), dtype as for X;
 *            base pointers and rows 16-byte aligned; d_h in {64, 128, 256} for bf16, {64, 128} for fp32
 *   idx, r, r_dev   the set R as for ada_assign_nearest
 *   assign   [T] int32, the representative of every token (the output of ada_assign_nearest for the same R)
 * Outputs
 *   out   [T x (H * d_h)] float, leading dimension ld_out (elements), any alignment (a 16-byte aligned base with
 *         ld_out a multiple of 4 lets the bf16 kernel store whole rows per instruction)
 *   info  [4] int32  {|R|, 0, 0, status}; status is ADA_OK, or ADA_ERR_INDEX (idx not strictly ascending / out of
 *                    range, or an assign entry that is not a member of R) / ADA_ERR_SHAPE (bad r_dev), and then out
 *                    is not written
 * Scores and weights are fp32 (a per-row reference close to the running maximum subtracted, so no weight exceeds
 * 2^10); bf16 weights enter the second product as hi + lo pairs.
 * ADA_FLAG_ATTN_CAUSAL masks later members of R.  Two launches (positions and validation, attention).
 */
int ada_attention_compressed(const void* Q, const void* K, const void* V, int T, int H, int d_h, int64_t ld, int dtype,
                             const int32_t* idx, int r, const int32_t* r_dev, const int32_t* assign,
                             float* out, int64_t ld_out, int32_t* info,
                             void* ws, size_t ws_bytes, void* stream, unsigned flags);

/*
 * The layer loop of Section 4.1: full selection at layer 0, Algorithm 1 at layers 1..L-1, each
 * step inheriting the previous step's set on the device (no host synchronisation inside).
 *   X_layers     HOST array of L device pointers, one T x d matrix per layer
 *   idx_all      device [L*T] int32   row l = R^(l) ascending
 *   counts_all   device [L*4] int32   row l as in ada_cascade_step (layer 0: {r, r, 0, 0})
 *   gram_ops_all device [L]   uint64  layer 0: T*T
 *   adds_all / removes_all  device [L*T] int32 each, or NULL to skip reporting them
 */
int ada_cascade_layers(const void* const* X_layers, int L, int T, int d, int64_t ld, int dtype, float tau,
                       int32_t* idx_all, int32_t* counts_all, uint64_t* gram_ops_all,
                       int32_t* adds_all, int32_t* removes_all,
                       void* ws, size_t ws_bytes, void* stream, unsigned flags);

/*
 * The same layer loop for B independent sequences at once (Section 8.4 suggests keeping selection work in flight next to other
 * work; here the selection work of several sequences is in flight together).  Sequence b runs exactly what ada_cascade_layers runs, on streams[b]; the
 * chains are issued layer by layer across the batch, so that while one sequence's set update runs on a single CU the
 * other sequences' tiles fill the rest of the device.
 *   X_layers     HOST array of B*L device pointers, sequence-major: X_layers[b*L + l]
 *   idx_all, counts_all, gram_ops_all, adds_all, removes_all   as for ada_cascade_layers, B blocks of L rows
 *   ws           B workspaces back to back, ada_workspace_bytes(T) apart, each initialised; ws_bytes >= B times that
 *   streams      HOST array of B HIP streams (default priority), or NULL: all chains one after the other on `stream`.
 *                Chains on the same stream run in order; distinct streams may overlap
 *   stream       the caller's stream: the chains start after the work enqueued on it before this call, and work
 *                enqueued on it after this call starts after all chains (events; no host synchronisation)
 * ADA_FLAG_RESIDENT_PASS is ignored (that form needs the whole device for one sequence).  B <= ADA_MAX_BATCH.
 */
int ada_cascade_layers_batched(const void* const* X_layers, int B, int L, int T, int d, int64_t ld, int dtype, float tau,
                               int32_t* idx_all, int32_t* counts_all, uint64_t* gram_ops_all,
                               int32_t* adds_all, int32_t* removes_all,
                               void* ws, size_t ws_bytes, void* const* streams, void* stream, unsigned flags);

/*
 * Several independent selection problems of one shape that live in ONE allocation, served by one launch per cascade
 * step: the h heads of a T x (h * d_h) matrix for the per-head cascade of Section 8.5 (a representative set per head,
 * cost h x T r_h d_h), or sequences stacked in one [G][T][ld] tensor.  Group g's matrix starts x_gstride elements
 * after group g-1's and has the common T, d (= d_h for heads), ld and dtype.
 */
typedef struct {
    int G;                  /* number of groups, 1 .. ADA_MAX_BATCH */
    int64_t x_gstride;      /* elements between consecutive groups' X (>= d): d_h for heads side by side, T * ld for
                               stacked sequences */
    int64_t list_gstride;   /* int32 elements between consecutive groups in prev_idx, idx, adds, removes (>= T) */
    int64_t counts_gstride; /* int32 elements between consecutive groups in counts, and in r_dev if given (>= 4) */
    int64_t ops_gstride;    /* elements between consecutive groups in gram_ops (>= 1) */
} ada_groups;

/*
 * Algorithm 1 for every group at once.  Arguments as for ada_cascade_step (the pointers are group 0's; r bounds every
 * group's inherited count, r_dev[g * counts_gstride] is group g's actual count); every group writes its own idx,
 * adds, removes, counts[4] and gram_ops.  There is no gamma output.
 *   ws   G workspaces back to back, ada_workspace_bytes(T) apart, each initialised
 * For T <= 16384 and without ADA_FLAG_TWO_PASS all groups share one launch (the chip's workgroups are divided among
 * the groups; a group's last workgroup updates that group's set); otherwise the groups run one after the other.
 */
int ada_cascade_step_grouped(const ada_groups* groups, const void* X, int T, int d, int64_t ld, int dtype, float tau,
                             const int32_t* prev_idx, int r, const int32_t* r_dev,
                             int32_t* idx, int32_t* adds, int32_t* removes, int32_t* counts, uint64_t* gram_ops,
                             void* ws, size_t ws_bytes, void* stream, unsigned flags);

/*
 * The full selection (Definition "Gram threshold") of every group, in the launches one problem takes (up to T = 4096
 * one: the Gram tiles sum the norms from their own operands and their last workgroup updates the set; beyond that, or
 * for rows that are not bf16 in whole aligned 128-byte chunks, a norm launch, the tiles and, beyond T = 4096, an
 * update launch).
 *   mask    [G][T] uint8, or NULL
 *   idx     group g's representatives at idx + g * list_gstride, ascending     (required)
 *   counts  group g's {r, r, 0, 0} at counts + g * counts_gstride               (required)
 *   ws      G workspaces back to back (as for ada_cascade_step_grouped)
 */
int ada_select_full_grouped(const ada_groups* groups, const void* X, int T, int d, int64_t ld, int dtype, float tau,
                            uint8_t* mask, int32_t* idx, int32_t* counts,
                            void* ws, size_t ws_bytes, void* stream, unsigned flags);

/*
 * The layer loop for G groups: full selection of every group at layer 0, then one grouped cascade step per layer.
 *   X_layers   HOST array of L device pointers (group 0's matrix of each layer)
 *   outputs    as for ada_cascade_layers_batched with B = G: idx_all [G][L][T], counts_all [G][L][4], ...
 * Only groups->G and groups->x_gstride are read (the other strides follow from the output layout).
 */
int ada_cascade_layers_grouped(const ada_groups* groups, const void* const* X_layers, int L, int T, int d, int64_t ld,
                               int dtype, float tau, int32_t* idx_all, int32_t* counts_all, uint64_t* gram_ops_all,
                               int32_t* adds_all, int32_t* removes_all,
                               void* ws, size_t ws_bytes, void* stream, unsigned flags);

/*
 * Selection pipelined against attention (Section 8.4): for every layer l, the selection (full at layer 0,
 * Algorithm 1 afterwards) runs on stream_sel; the layer's nearest-representative assignment (Section 2.3) and
 * its attention on the representative set (eq. (1)) run on stream_attn and wait only for that layer's set.  The
 * selection of layer l+1 needs nothing from the attention of layer l, so the two overlap.
 *   X_layers, Q_layers, K_layers, V_layers   HOST arrays of L device pointers: T x (H * d_h) matrices, leading
 *                dimension ld, dtype as usual; the alignment rules of ada_attention_compressed apply to Q, K, V
 *   idx_all, counts_all, gram_ops_all        as for ada_cascade_layers
 *   assign_all   device [L*T] int32          row l: the representative of every token at layer l
 *   info_all     device [L*8] int32          row l: info of ada_assign_nearest, then info of ada_attention_compressed
 *   out_layers   HOST array of L device pointers: T x (H * d_h) float outputs, leading dimension ld_out
 *   ws           TWO workspaces back to back (ws_bytes >= 2 * ada_workspace_bytes(T)), both initialised: the two
 *                streams work at the same time
 *   stream_sel, stream_attn   HIP streams of default priority; NULL = `stream` (with both NULL, or both the same
 *                stream, the layers run strictly one step after the other)
 *   stream       the caller's stream: the pipeline starts after the work enqueued on it before the call; work
 *                enqueued on it afterwards waits for the whole pipeline (events, no host synchronisation)
 * flags: ADA_FLAG_CROSS_EARLIER_ONLY, ADA_FLAG_TWO_PASS (selection), ADA_FLAG_ATTN_CAUSAL (attention).
 */
int ada_pipeline_layers(const void* const* X_layers, const void* const* Q_layers, const void* const* K_layers,
                        const void* const* V_layers, int L, int T, int H, int d_h, int64_t ld, int dtype, float tau,
                        int32_t* idx_all, int32_t* counts_all, uint64_t* gram_ops_all, int32_t* assign_all,
                        int32_t* info_all, float* const* out_layers, int64_t ld_out,
                        void* ws, size_t ws_bytes, void* stream_sel, void* stream_attn, void* stream, unsigned flags);

/*
 * A threshold that follows the turnover (Section 8.1 gives only the direction of the adjustment -- tighten where the
 * set is stable, loosen where it changes -- and no formula).  The rule used here:
 *   eta^(l)   = (adds + removes) / |R^(l-1)|            the turnover of the step just made (eq. (8))
 *   tau^(l+1) = clip(tau^(l) + kappa * (eta_target - eta^(l)), tau_min, tau_max)
 * A larger tau is a tighter threshold (1 - tau^2 falls: fewer representatives).  Layers 0 and 1 use tau0.  A step the
 * device rejects (bad list) leaves tau unchanged.  Evaluated on the device in IEEE double, one rounding per operation.
 */
typedef struct {
    double kappa;       /* gain; 0 keeps tau fixed */
    double eta_target;  /* turnover at which tau stays where it is */
    double tau_min;     /* 0 < tau_min <= tau0 <= tau_max < 1 */
    double tau_max;
} ada_tau_control;

/*
 * ada_cascade_layers with the threshold adapted between layers on the device (no host synchronisation).
 *   tau_all  device [L] double   the tau each layer used
 *   thr_all  device [L] float    1 - tau^2 as the kernels compared with it
 * Other arguments and outputs as for ada_cascade_layers.  T <= 16384; ADA_FLAG_TWO_PASS and
 * ADA_FLAG_RESIDENT_PASS are not available (ADA_ERR_SHAPE / ignored).  ADA_ERR_TAU for bounds that are not
 * 0 < tau_min <= tau0 <= tau_max < 1 or for a NaN gain / target.
 */
int ada_cascade_layers_adaptive(const void* const* X_layers, int L, int T, int d, int64_t ld, int dtype, float tau0,
                                const ada_tau_control* ctl, int32_t* idx_all, int32_t* counts_all,
                                uint64_t* gram_ops_all, int32_t* adds_all, int32_t* removes_all,
                                double* tau_all, float* thr_all,
                                void* ws, size_t ws_bytes, void* stream, unsigned flags);

/*
 * Which tile shape a one-launch cascade step takes when `workgroups` workgroups share its tiles (the CU count for a
 * single problem; that divided by the number of groups for a grouped call) and the rows come in whole aligned
 * 128-byte chunks of bf16: 0 = 64 x 64, 1 = 64 representatives x 128 tokens, 2 = 128 x 128, 3 = 128 representatives x
 * 256 tokens; -1 for arguments out of range.
 * Host only (no device is touched): the same function the kernel evaluates with the set size it finds.
 */
int ada_plan_tile_shape(int r, int T, int d, int workgroups);

/*
 * How ada_select_full cuts the lower triangle of the T x T Gram into work units when it runs its direct-to-LDS kernel
 * (bf16 rows in whole aligned 64-byte pieces, T >= 1536, no greedy covering) on `workgroups` workgroups (the CU count
 * for one problem): 0 = 128 x 128 units everywhere; 1 = 256 x 256 units off the diagonal, 128 x 128 on it (T > 4096);
 * 2 = 64 x 128 units off the diagonal of 128-blocks and one unit per diagonal block (T <= 4096, d a multiple of 64,
 * where 128 x 128 units would leave CUs idle); -1 for arguments outside that kernel's range.
 * Host only (no device is touched): the choice the launch makes.
 */
int ada_plan_full_units(int T, int d, int workgroups);

/*
 * |A n B| and |A u B| of two representative sets given as uint8 masks [T] (device), for the
 * Jaccard index of eq. (3).  out: device int32 [2] = {intersection, union}.
 */
int ada_set_overlap(const uint8_t* mask_a, const uint8_t* mask_b, int T, int32_t* out, void* stream);

/*
 * Host-side bookkeeping from the per-layer counts of ada_cascade_layers (HOST arrays in, HOST out):
 *   jaccard[l]  = |R^(l-1) n R^(l)| / |R^(l-1) u R^(l)| = (r_prev - removes) / (r_prev + adds)   (eq. (3))
 *   turnover[l] = (adds + removes) / r_prev                                                     (eq. (8))
 *   *savings    = 1 - sum_l gram_ops[l] / (L * T^2)                                             (Table 6)
 * jaccard[0] and turnover[0] are set to 0 (no step at layer 0).  Any output pointer may be NULL.
 */
int ada_cascade_report(int L, int T, const int32_t* counts_all, const uint64_t* gram_ops_all,
                       double* jaccard, double* turnover, double* savings);

/*
 * Measurement aid (not part of the method).  While enabled, every kernel the library launches is bracketed by
 * two HIP events recorded on the stream it is launched on.  ada_profile_collect waits for them and returns,
 * per kernel class, the summed elapsed milliseconds and the number of launches since the last collect
 * (HOST arrays of ADA_K_COUNT entries), then forgets them.  Event pairs include the launch gap in front of the
 * kernel, so these figures are upper bounds of the durations a kernel trace reports.
 */
enum { ADA_K_NORM_PREP = 0, ADA_K_GRAM_FULL = 1, ADA_K_GRAM_REP = 2, ADA_K_GRAM_CROSS = 3, ADA_K_UPDATE = 4,
       ADA_K_CASCADE_FUSED = 5, ADA_K_MFMA_PROBE = 6, ADA_K_ASSIGN = 7, ADA_K_ATTN = 8, ADA_K_COUNT = 9 };
int ada_profile_enable(int on);
int ada_profile_collect(double* ms_sum, int* launches);
/* A plain device-to-device copy kernel (bytes: multiple of 16, both pointers 16-byte aligned): it reads and writes
 * exactly `bytes`, which is what hardware traffic counters of the library's kernels are scaled against. */
int ada_profile_copy_probe(void* dst, const void* src, size_t bytes, void* stream);
/* A kernel that does nothing but bf16 matrix instructions (the 32x32x16 form the Gram kernels use) on pseudo-random
 * operands held in registers: `workgroups` workgroups of four wavefronts, each wavefront issuing 16 * iters
 * independent instructions of 32768 flops.  Timed through ada_profile_collect (class ADA_K_MFMA_PROBE) it gives the
 * matrix rate this device sustains on realistic data, which sits below the published peak when the clock is
 * power-limited; the Gram kernels' fractions are reported against both.  sink: device, >= workgroups floats
 * (written only in a case that does not occur; keeps the arithmetic alive).  Returns ADA_ERR_SHAPE for
 * workgroups < 1, iters < 1 or more than 2^20 of either. */
int ada_profile_mfma_probe(int workgroups, int iters, float* sink, void* stream);

/*
 * Development switches (environment variables; not part of the interface).  They force code paths that the library
 * otherwise chooses by shape, for tests and measurements, and are read only when ADA_DEV_SWITCHES=1 is set as well:
 *   ADA_GRAM=tile|dma0|dma1|dma2  full selection: register-staged tiles / direct-to-LDS kernel with 128-row, 256-row or
 *                                 64 x 128 units
 *   ADA_TILE=64|128               register-staged Gram tile size
 *   ADA_KGROUPS=1|2               K-groups of the 64 x 64 one-launch cascade tile
 *   ADA_CASCADE_TILE=64|64x128|128|256x128   tile shape of the one-launch cascade step
 *   ADA_NO_DMA=1                  operands through registers instead of straight into LDS
 *   ADA_ATTN=lds                  the first attention kernel
 *   ADA_SPIN_LIMIT=n              bound of the resident pass's wait between layers (polls)
 */

#ifdef __cplusplus
}
#endif
#endif /* ADA_H */
