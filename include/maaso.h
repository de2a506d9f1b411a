/* maaso.h - C ABI of the MI355X scoring path of MaaSO's placer and distributor.
 *
 * The library evaluates the profiler's performance model for every (candidate deployment, request,
 * instance) triple, checks the request's deadlines, and reduces the result either to a chosen
 * instance per request (distributor) or to an SLO-satisfaction ratio per candidate (placer).
 * All kernels are HIP for gfx950; there is no CPU fallback: without a GPU every compute entry point
 * returns MAASO_E_HIP.
 *
 * Conventions
 *   - Every function returns 0 (MAASO_OK) or a negative maaso_status.  Nothing throws, aborts or
 *     prints.  maaso_strerror() names a status.
 *   - "HOST" pointers are read during the call and may be freed afterwards.  "DEVICE" pointers are
 *     caller-owned device memory (for example torch tensors) on the context's device; the library
 *     never frees or reallocates them.  The only memory the library owns is the context (device
 *     copies of the tables, a workspace, a status word).
 *   - Compute calls (maaso_score_assign, maaso_score_assign_selected, maaso_placement_sweep,
 *     maaso_placement_sweep_noalloc, maaso_placement_score, maaso_placement_score_sets,
 *     maaso_split_by_slo, maaso_ins_deploy_select, maaso_resource_partition,
 *     maaso_resource_partition_requests, maaso_batch_size_prune) are asynchronous on the given HIP
 *     stream (NULL = the default stream).  They allocate nothing, free nothing and do no
 *     host synchronisation: the context's workspace is sized at maaso_profile_tables_load
 *     (MAASO_DEFAULT_WORKSPACE_BYTES, enough for 65,536 candidates of 32 instance slots) and
 *     changed only by maaso_ctx_reserve; a call whose shape needs more is refused with
 *     MAASO_E_WORKSPACE before anything is launched.  Outputs are valid once the stream has been
 *     synchronised.  The calls that do synchronise are the set-up and read-back calls:
 *     maaso_profile_tables_load, maaso_profile_fit, maaso_ctx_reserve, maaso_ctx_destroy,
 *     maaso_ctx_device_status, maaso_ctx_kernel_elapsed, maaso_ctx_sweep_evaluated.
 *   - A context serves one call at a time.  Its workspace and accumulators are shared by its calls:
 *     calls issued on one stream are ordered by that stream; a call issued on another stream than
 *     the context's previous call is ordered behind it by the library (an event recorded on the
 *     previous stream, awaited by the new one - no host wait; if the previous stream has been
 *     destroyed meanwhile the device is synchronised instead).  A second thread entering while a
 *     call's host part is running gets MAASO_E_BUSY.  For calls that should overlap on the GPU use
 *     one context per stream.
 *   - Time is counted in ticks of 2^-20 s where integers are used (arrival_ticks, q_ticks).
 *   - Arithmetic is IEEE-754 binary32, round to nearest even, one rounding per operation (fused
 *     multiply-add where the model has one), so results do not depend on the launch configuration.
 */
#ifndef MAASO_H
#define MAASO_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  MAASO_OK = 0,
  MAASO_E_INVALID_ARG = -1, /* NULL where a pointer is required, n_cand != 1 for the distributor, ... */
  MAASO_E_SHAPE = -2,       /* a size beyond MAASO_MAX_* or beyond what fits the LDS staging         */
  MAASO_E_TABLE = -3,       /* non-finite or non-positive table entry / deadline outside [2^-20,2^20] */
  MAASO_E_HIP = -4,         /* a HIP runtime call failed (no device, launch failure, ...)             */
  MAASO_E_NOMEM = -5,       /* host or device allocation failed                                       */
  MAASO_E_TIMEOUT = -6,     /* reported by maaso_ctx_device_status: an inter-window wait gave up      */
  MAASO_E_WORKSPACE = -7,   /* the call's shape needs a larger workspace: maaso_ctx_reserve first     */
  MAASO_E_BUSY = -8,        /* another thread is inside a call on this context                        */
  MAASO_E_RESIDENCY = -9    /* the windowed distributor's blocks cannot all be resident at once        */
} maaso_status;

#define MAASO_MAX_INSTANCES 256u   /* i_pad: instance slots per candidate                      */
#define MAASO_MAX_SLO 16u          /* K: SLO classes                                            */
#define MAASO_MAX_TABLE_CELLS 2048u /* n_tp * (b_cap + 1): cells per profile table (LDS-resident) */
#define MAASO_MAX_REQUESTS 2147483648u /* R: requests per call                                  */
#define MAASO_MAX_LEN 16777215u    /* prompt_len / out_len: exactly representable in binary32   */
#define MAASO_MAX_GPUS 4096u       /* |G|: GPUs of a (sub-)cluster in the placer's outer algorithms */
#define MAASO_MAX_REQUEST_SETS 4u  /* request sets scored by one maaso_placement_score_sets call   */
#define MAASO_DEFAULT_WORKSPACE_BYTES (64u << 20) /* workspace a context is loaded with            */
#define MAASO_COUNT_INCOMPLETE (1ull << 63) /* set in n_satisfied by a windowed call that gave up  */

/* bits of the device status word (maaso_ctx_device_status) */
#define MAASO_DEV_BAD_CLASS 1u     /* a request with slo_class >= n_slo was skipped (never satisfied) */
#define MAASO_DEV_BAD_INSTANCE 2u  /* an instance with tp_idx >= n_tp or max_batch outside 1..b_cap was
                                      treated as absent */
#define MAASO_DEV_WAIT_TIMEOUT 4u  /* the windowed distributor's inter-window wait exceeded its spin
                                      limit.  Of that call: chosen / slack / latencies are written
                                      for the windows scored before it gave up and untouched after,
                                      n_satisfied has MAASO_COUNT_INCOMPLETE set, occ and q_ticks are
                                      left as they were given */

#define MAASO_DEV_BAD_CHAIN 8u     /* chain_offsets of maaso_ins_deploy_select not non-decreasing
                                      within [0, n_cand]; that chain was ignored */

typedef struct maaso_ctx maaso_ctx; /* opaque */

/* Profile tables and SLO classes.  HOST pointers, copied at load.
 *
 * The profiler's throughput-decay function F(M,P,B,W) depends on the strategy P and on min(B,W)
 * (Sec. IV-B, Eq. 1), so a profile is tabulated per (strategy row t, effective batch b), b = 1..b_cap.
 * Row-major [n_tp][b_cap+1]; column 0 is never read and may hold anything.
 *   prefill_a + prefill_p * prompt_len = prefill seconds;  tbt = seconds per output token (= 1/F).
 * An SLO class k carries a first-token deadline d_ttft[k] and a between-token deadline d_tbt[k]; the
 * end-to-end deadline of a request is d_ttft + out_len * d_tbt (normalised deadline, Sec. III-C). */
typedef struct {
  uint32_t n_tp;             /* T >= 1                                                   */
  uint32_t b_cap;            /* >= 1; T * (b_cap + 1) <= MAASO_MAX_TABLE_CELLS           */
  const uint32_t* tp_degree; /* [T] GPUs per instance N(P); may be NULL, but then
                                maaso_ins_deploy_select is refused                       */
  const float* prefill_a;    /* [T*(b_cap+1)] seconds, > 0 and finite for b >= 1         */
  const float* prefill_p;    /* [T*(b_cap+1)] seconds per prompt token, > 0, finite      */
  const float* tbt;          /* [T*(b_cap+1)] seconds per output token, > 0, finite      */
  uint32_t n_slo;            /* K, 1..MAASO_MAX_SLO                                      */
  const float* d_ttft;       /* [K] seconds, within [2^-20, 2^20]                        */
  const float* d_tbt;        /* [K] seconds, within [2^-20, 2^20]                        */
} maaso_profile_desc;

/* Profiler (Sec. IV-B): least-squares fit of the throughput-decay function of Eq. 1,
 *   F(w) = T0 * (1 - delta * log(eps + w)),  w = min(B, W),
 * to measured samples, one fit per parallelism strategy, and the per-token latency table the scoring
 * reads: tbt[t][b] = 1 / F_t(b), b = 1..b_cap (column 0 = NaN), ready for maaso_profile_desc.tbt.
 * All pointers are HOST memory; the call copies in, runs on `device`, copies out and synchronises.
 *   offsets [n_tp+1]: the samples of strategy t are [offsets[t], offsets[t+1]) (at least 3 each);
 *   level [N]: w of a sample, >= 1;  thr [N]: its measured throughput in tokens/s, > 0;
 *   eps is searched in [eps_lo, eps_hi], 0 < eps_lo < eps_hi;
 *   params [n_tp][4] (binary64): T0, delta, eps, residual sum of squares;  tbt [n_tp*(b_cap+1)].
 * For a fixed eps the fit is a straight line in log(eps + w) with a closed-form solution; eps itself is
 * found by a nested grid search on log(eps) (256 points, shrinking to the best point's neighbours,
 * 10 levels).  Binary64 arithmetic throughout; the table is rounded once to binary32.
 * Errors: INVALID_ARG, SHAPE (table too large for the scoring kernels), TABLE (a sample out of range,
 * fewer than 3 samples for a strategy, T0 <= 0 or F(b) <= 0 for some b <= b_cap: params and tbt are
 * still written, NaN where undefined), HIP, NOMEM. */
int maaso_profile_fit(int device, uint32_t n_tp, const uint32_t* offsets, const float* level,
                      const float* thr, uint32_t b_cap, float eps_lo, float eps_hi, double* params,
                      float* tbt);

/* Validates and copies the tables to `device` (a HIP device ordinal) and creates a context.
 * Profiles are the placer's and distributor's input F(.) (Alg. 1 and Alg. 2, "Model profiles").
 * Errors: INVALID_ARG (NULL), SHAPE, TABLE, HIP, NOMEM.  On error *out_ctx is set to NULL. */
int maaso_profile_tables_load(const maaso_profile_desc* desc, int device, maaso_ctx** out_ctx);

/* Frees the context and everything it owns.  NULL is allowed.  Synchronises the device. */
void maaso_ctx_destroy(maaso_ctx* ctx);

/* Sizes the context's workspace so that no later compute call with at most max_cand candidates of
 * i_pad instance slots and max_req requests is refused with MAASO_E_WORKSPACE, whatever launch shape
 * it takes (set the launch-shape knobs before reserving: more blocks per queue need more).  The
 * workspace holds, for the static sweep, the prompt lengths bucketed by class (4*K*R bytes), one
 * 16-byte record per instance slot and the work-queue heads; 12 KiB for the windowed distributor;
 * 4 bytes per 1024 requests for maaso_split_by_slo.  The windowed sweep, the scores and the static
 * distributor use none.  Never shrinks.  A set-up call: it synchronises the device and reallocates
 * when the workspace has to grow.  Errors: INVALID_ARG, SHAPE, HIP, NOMEM, BUSY. */
int maaso_ctx_reserve(maaso_ctx* ctx, uint32_t max_cand, uint32_t i_pad, uint32_t max_req);

/* Bytes of workspace the context holds and how many times it has been allocated since (and
 * including) maaso_profile_tables_load - a compute call never changes either.  Either pointer may be
 * NULL.  Errors: INVALID_ARG. */
int maaso_ctx_workspace(maaso_ctx* ctx, uint64_t* bytes, uint32_t* allocations);

/* Synchronises the context's device, returns the MAASO_DEV_* bits raised by kernels since the last
 * call in *bits (may be NULL) and clears them.  Returns MAASO_E_TIMEOUT if MAASO_DEV_WAIT_TIMEOUT is
 * among them, MAASO_E_INVALID_ARG if another bit is, else MAASO_OK. */
int maaso_ctx_device_status(maaso_ctx* ctx, uint32_t* bits);

const char* maaso_strerror(int status);

/* Performance knobs; they never change a result.  0 selects the library's own choice.
 *   sweep_requests_per_lane: requests a lane of the sweep kernel keeps in registers (0, 2, 4, 8, 16);
 *     a block of the sweep owns 256 times as many requests of one SLO class;
 *   sweep_group: candidates per work item of the sweep kernel (clamped to what fits its LDS lists);
 *   sweep_blocks_per_queue: persistent blocks serving each (request tile, XCD) work queue;
 *   window_blocks: blocks of the windowed distributor's persistent kernel (at most one per compute
 *   unit is used).  Left at 0, windows of up to four requests are distributed by a single wavefront
 *   instead (no device-wide barrier per window); a value keeps the persistent kernel for them too.
 * Errors: INVALID_ARG. */
int maaso_ctx_set_launch_shape(maaso_ctx* ctx, uint32_t sweep_requests_per_lane, uint32_t sweep_group,
                               uint32_t sweep_blocks_per_queue, uint32_t window_blocks);

/* Number of polls after which a block of the windowed distributor stops waiting for the other
 * blocks at a window boundary, raises MAASO_DEV_WAIT_TIMEOUT and leaves the kernel (all other blocks
 * then leave too; the call's outputs are incomplete).  The default, 2^22, is seconds of waiting.
 * Errors: INVALID_ARG. */
int maaso_ctx_set_wait_limit(maaso_ctx* ctx, uint32_t polls);

/* How the windowed distributor's persistent kernel is launched.  enable != 0 (the default where the
 * device supports it): cooperatively - the runtime guarantees that all blocks are resident together
 * or refuses the launch.  0: as an ordinary grid, after the host has checked with the occupancy query
 * that the device can hold all blocks at once; other work on the device can then still keep blocks
 * from starting, which the bounded wait turns into MAASO_E_TIMEOUT.  For tools that cannot follow
 * cooperative launches (rocprofv3 crashed at process exit after one).  Errors: INVALID_ARG, HIP. */
int maaso_ctx_set_cooperative(maaso_ctx* ctx, int enable);

/* Instrumentation.  With timing enabled, each compute call records a pair of HIP events on its
 * stream directly around its dominant kernel (the sweep kernel of maaso_placement_sweep and of
 * maaso_placement_score, the scoring kernel of maaso_score_assign), for up to 256 calls.  maaso_ctx_kernel_elapsed waits for the
 * recorded events, returns the sum of the kernel durations in milliseconds and their number, and
 * starts a new series.  Enabling allocates the events once; no other call is affected.
 * Errors: INVALID_ARG, HIP. */
int maaso_ctx_kernel_timing(maaso_ctx* ctx, int enable);
int maaso_ctx_kernel_elapsed(maaso_ctx* ctx, float* total_ms, uint32_t* launches);
/* The same series launch by launch, in the order issued: durations_ms [cap] (HOST) receives the
 * first min(cap, recorded) durations in milliseconds, *launches their number; starts a new series.
 * (Shows, for instance, whether the device's clock was still rising during a short series.) */
int maaso_ctx_kernel_durations(maaso_ctx* ctx, float* durations_ms, uint32_t cap, uint32_t* launches);

/* What the chip sustains for the sweep's instruction mix.  Runs, on `device`, a kernel that is nothing
 * but the sweep's inner instruction sequence in a loop (8 wavefronts per SIMD, no memory access) and
 * returns the vector lane operations per second it reaches - the practical ceiling for the sweep on
 * this device, next to the nominal peak that roofline fractions are quoted against.
 *   pattern 0: two fma + one three-input minimum per request (a pair of records without queue wait),
 *   1: the same with the wait's two adds, 2: pattern 0 unrolled four times, 3: compares that write a
 *   lane mask, 4: fma with a scalar-register operand.
 * trips: loop trips; the kernel runs three times and the last run is reported, and only runs of some
 * tens of milliseconds (65,536 trips) see the device at its sustained clock.  *instructions_per_trip
 * (may be NULL) receives the vector instructions of one trip.  A set-up style call: it allocates,
 * synchronises and frees.
 * Errors: INVALID_ARG, HIP, NOMEM. */
int maaso_probe_valu(int device, uint32_t pattern, uint32_t trips, double* lane_ops_per_s,
                     uint32_t* instructions_per_trip);

/* Where the windowed distributor's time goes.  With profiling enabled, a maaso_score_assign call that
 * runs the persistent windowed kernel (window > 4, policy 0, no latency outputs) has block 0 sum the
 * shader clock cycles it spends, per window, on: [0] evaluating the instances' profiles for the
 * window's state, [1] scoring its share of the window's requests, [2] exchanging the admitted load
 * with the other blocks (device-wide barrier included), [3] advancing the state; [4] is the whole
 * window loop, [5] the number of windows.  maaso_ctx_window_phases synchronises the device and returns
 * the six figures of the context's most recent such call (zeros if there was none).  Results of the
 * call are unchanged; its kernel is a few per cent slower.  Errors: INVALID_ARG, HIP. */
int maaso_ctx_window_profile(maaso_ctx* ctx, int enable);
int maaso_ctx_window_phases(maaso_ctx* ctx, uint64_t cycles[6]);

/* Synchronises the device and returns how many (request, instance) pairs the context's most recent
 * maaso_placement_sweep evaluated in its latency loop, i.e. the valid triples minus those whose
 * instance already fails the between-token deadline of the request's class (they are settled per
 * (class, instance) and never reach the loop).  *pairs_without_wait (may be NULL) receives how many
 * of them belong to an instance whose queue wait is exactly zero: for those the sweep leaves the
 * addition of the wait out (0 + x = x), so they cost it less.  Both 0 if no sweep has run.
 * Errors: INVALID_ARG, HIP. */
int maaso_ctx_sweep_evaluated(maaso_ctx* ctx, uint64_t* pairs, uint64_t* pairs_without_wait);

/* Requests as structure-of-arrays streams (Sec. IV-C: a request r decodes S_r tokens before its
 * deadline; Sec. V-A: arrivals over time).  DEVICE pointers, read only. */
typedef struct {
  uint32_t n_req;                /* R, 0..MAASO_MAX_REQUESTS                                      */
  const uint32_t* prompt_len;    /* [R] tokens, <= MAASO_MAX_LEN                                  */
  const uint32_t* out_len;       /* [R] tokens, <= MAASO_MAX_LEN                                  */
  const uint8_t* slo_class;      /* [R] < n_slo                                                   */
  const uint32_t* arrival_ticks; /* [R] non-decreasing; read only when window > 0, else may be NULL */
} maaso_requests;

/* Candidate deployments: n_cand rows of i_pad instance slots, row-major [n_cand][i_pad]; the valid
 * instances of candidate c are the slots j < n_inst[c].  An instance is configured by its strategy
 * and inference batch size (P_i, B_i) and carries its live workload level W_i (Sec. IV-C) and the
 * prefill work already queued on it (the pending time of Sec. III-C).  DEVICE pointers. */
typedef struct {
  uint32_t n_cand;           /* C >= 1                                                      */
  uint32_t i_pad;            /* 1..MAASO_MAX_INSTANCES                                      */
  const uint32_t* n_inst;    /* [C] <= i_pad; 0 is allowed (nothing can be served)          */
  const uint8_t* tp_idx;     /* [C*i_pad] row of the profile tables, < n_tp                 */
  const uint16_t* max_batch; /* [C*i_pad] B_j, 1..b_cap                                     */
  int32_t* occ;              /* [C*i_pad] W_j >= 0: requests on the instance; written only by
                                maaso_score_assign with window > 0                           */
  uint64_t* q_ticks;         /* [C*i_pad] queued prefill time in ticks; written as occ is    */
} maaso_placements;

typedef struct {
  float s_bar;       /* E[S_r] > 0: expected output length, used for the slot wait of an instance past
                        its batch cap and for the fluid drain between windows (Eq. 2)             */
  float pen_kappa;   /* >= 0: per-token latency is scaled by 1 + kappa * max(4w - 3B, 0) / B, i.e. it
                        grows linearly once the batch is more than 75 % full; 0 disables           */
  uint32_t tbt_mode; /* 0: profile row at the effective batch w = min(B, W + 1) (Eq. 1);
                        1: worst case w = B (the distributor's conservative estimate, Sec. IV-F)   */
  uint32_t window;   /* 0: every request is scored against the state as given (static);
                        n > 0: requests are taken n at a time and the state advances in between    */
  uint32_t policy;   /* which instance a request is given (Sec. IV-F step 2):
                        0: the one with the largest slack (lowest index on ties);
                        1: among the instances able to meet its SLO (slack >= 0) the one with the
                           shortest request queue - fewest requests W_j on it at the start of the
                           window - lowest index on ties; the paper's wording.  With no capable
                           instance the request is blocked either way and the largest-slack instance
                           is reported.  The static sweep's counts do not depend on it.          */
} maaso_params;

/* Per-request outputs of the distributor.  DEVICE pointers; any of them may be NULL (not written),
 * except that at least n_satisfied or chosen must be given. */
typedef struct {
  int32_t* chosen;       /* [R] instance with the largest slack, lowest index on ties; -1 iff the
                            placement has no valid instance                                     */
  float* slack;          /* [R] its slack = min of the three relative margins; the request is
                            admitted iff slack >= 0; -inf iff chosen == -1                       */
  float* ttft;           /* [R] first-token latency on the chosen instance (NaN iff none)       */
  float* tbt;            /* [R] between-token latency of the chosen instance (NaN iff none)     */
  float* e2e;            /* [R] end-to-end latency on the chosen instance (NaN iff none)        */
  uint64_t* n_satisfied; /* [1] number of admitted requests                                     */
} maaso_assign_out;

/* Distributor: instance assignment and overflow protection (Sec. IV-F, steps 2 and 3) for one
 * placement (pl->n_cand must be 1).  For each request and each valid instance j:
 *   prefill = p_j*L + a_j (fused);  ttft = wait_j + prefill;  e2e = S*tbt_j + ttft (fused);
 *   margins (D - latency) / D against the TTFT, TBT and end-to-end deadlines;  slack = their min
 * (L_r = L_q + L_d against the deadline, Eq. 2 and Eq. 3).  The request goes to the instance of
 * largest slack (prm->policy == 0; with policy 1 to the capable instance with the shortest queue, see
 * maaso_params) and is admitted iff that instance's slack is >= 0 (equality counts, Eq. 3), else
 * blocked.
 * With window > 0 the state (occ, q_ticks) is advanced after every window from the admitted
 * requests: occupancy and queued prefill ticks are added, the queue drains by the arrival time that
 * passed, and min(W,B) * elapsed / (s_bar * tbt_j) requests complete; blocked requests add no load.
 * After the last window the load is added and nothing drains.  window >= R behaves as one window.
 * Windows of more than four requests run in one persistent kernel whose blocks meet at a device-wide
 * barrier after every window, so all of them must be resident together: the kernel is launched
 * cooperatively, which the runtime either guarantees or refuses (MAASO_E_RESIDENCY, nothing ran).
 * Errors: INVALID_ARG, SHAPE, WORKSPACE, RESIDENCY, BUSY, HIP - all detected on the host. */
int maaso_score_assign(maaso_ctx* ctx, const maaso_placements* pl, const maaso_requests* rq,
                       const maaso_params* prm, const maaso_assign_out* out, void* hip_stream);

/* The same distributor on one row of a multi-candidate placement, the row index being read on the
 * DEVICE when the kernel starts: cand [1] is typically the best_cand output of maaso_placement_sweep
 * or maaso_placement_score issued just before on the same stream, so that placing and distributing
 * need no host round trip in between.  pl may hold any number of candidates; only row *cand is read
 * (and, with window > 0, written).  *cand >= pl->n_cand raises MAASO_DEV_BAD_INSTANCE and the call
 * behaves as for a placement without instances.  Errors as maaso_score_assign. */
int maaso_score_assign_selected(maaso_ctx* ctx, const maaso_placements* pl, const uint32_t* cand,
                                const maaso_requests* rq, const maaso_params* prm,
                                const maaso_assign_out* out, void* hip_stream);

/* Placer: SLO-satisfaction count and ratio of every candidate deployment against the whole request
 * set, and the best candidate - the evaluation of Phi_S^n(I', R_x) that Alg. 1 performs for each
 * candidate deployment I' (Eq. 3, Eq. 6).
 *   prm->window == 0 (static): a request counts for candidate c iff some valid instance of c has
 *     slack >= 0 against the state as given (the same triple arithmetic as maaso_score_assign).
 *   prm->window  > 0 (capacity-aware): every candidate is run through the windowed distributor of
 *     maaso_score_assign on its own copy of its instance state, so admitted requests load the
 *     instances and later windows see it (the stand-in for the paper's virtual-slot simulator,
 *     Sec. V-A); the count is the number of admitted requests.  rq->arrival_ticks is required.
 * Outputs, DEVICE pointers: sat_count [C] (required), sat_ratio [C] = count / R (0 when R == 0; may
 * be NULL), best_cand [1] = lowest index among the largest counts (may be NULL).
 * The placements are not written in either form.
 * Errors: INVALID_ARG, SHAPE, WORKSPACE (static form), BUSY, HIP. */
int maaso_placement_sweep(maaso_ctx* ctx, const maaso_placements* pl, const maaso_requests* rq,
                          const maaso_params* prm, uint32_t* sat_count, float* sat_ratio,
                          uint32_t* best_cand, void* hip_stream);

/* For callers that cannot allocate device memory while they call (code under HIP graph capture, tight
 * serving loops, harnesses that forbid it): maaso_placement_sweep with the same arguments, results
 * and errors, whose static form (prm->window == 0) keeps its intermediate data - the class-bucketed
 * prompt lengths, one staged 16-byte record per instance slot, the work-queue heads - in a device
 * array of MAASO_NOALLOC_SCRATCH_BYTES that is part of the library image (every GPU the library runs
 * on holds its own copy until the process ends).  The call contains no hipMalloc, hipFree or other
 * allocating routine and no host synchronisation.  A shape that needs more - about
 * 4*K*R + 16*C*i_pad bytes plus 20 bytes per launched block - is refused with MAASO_E_SHAPE before
 * anything is launched.  (The capacity-aware form, window > 0, uses no scratch and is passed through.)
 * All calls on one GPU share that GPU's array, whatever the context: calls that overlap in time on
 * one GPU race on it - order them on one stream or with events.  Everything in the array that must
 * start at zero is cleared by the call's own first launch. */
#define MAASO_NOALLOC_SCRATCH_BYTES (8u << 20)
int maaso_placement_sweep_noalloc(maaso_ctx* ctx, const maaso_placements* pl, const maaso_requests* rq,
                                  const maaso_params* prm, uint32_t* sat_count, float* sat_ratio,
                                  uint32_t* best_cand, void* hip_stream);

/* Weights and thresholds of the composite serving score (Sec. IV-D, Eq. 6): alpha prioritises SLO
 * satisfaction (the paper uses 4, and 10 in its ablation), beta in [0,1] balances throughput against
 * latency (0.3), gamma_t > 0 is the throughput that normalises to 1 (tokens/s), gamma_l > 0 the
 * largest acceptable queuing latency (seconds). */
typedef struct {
  float alpha, beta, gamma_t, gamma_l;
} maaso_score_weights;

/* Per-candidate outputs of maaso_placement_score.  DEVICE pointers, [C] each; sat_count and score
 * are required, the others may be NULL.  best_cand [1] (may be NULL): lowest index among the largest
 * scores. */
typedef struct {
  uint32_t* sat_count; /* admitted requests                                              */
  float* phi_s;        /* Phi_S^n = sat_count / R (0 when R == 0)                        */
  float* phi_t;        /* Phi_T: sum of 1 / tbt_j over the instances that served a request */
  float* phi_l;        /* Phi_L: mean queue wait of the admitted requests, seconds       */
  float* score;        /* Phi                                                            */
  uint32_t* best_cand;
} maaso_score_out;

/* Placer objective: the composite serving score Phi(I', R_x) of every candidate deployment
 * (Sec. IV-D, Eq. 6-8; the quantity Alg. 1 compares).  Each candidate is run through the distributor
 * of maaso_score_assign - against the state as given when prm->window == 0, window by window on a
 * copy of its state when prm->window > 0 (rq->arrival_ticks required) - and
 *   Phi = alpha * Phi_S^n + beta * min(Phi_T, gamma_t) / gamma_t + (1 - beta) * max(gamma_l - Phi_L, 0) / gamma_l
 * with Phi_S^n the admitted fraction (Eq. 3), Phi_T the sum, in index order, of 1 / tbt_j over the
 * instances that served at least one request (tbt_j as staged for the first window; Eq. 4) and Phi_L
 * the mean over the admitted requests of their instance's queue wait at admission, taken from the
 * exact integer sum of the waits in ticks (Eq. 5).  Every float operation is a single binary32
 * operation in a fixed order, so the result does not depend on scheduling.
 * The placements are not written.  Errors: INVALID_ARG, SHAPE, HIP. */
int maaso_placement_score(maaso_ctx* ctx, const maaso_placements* pl, const maaso_requests* rq,
                          const maaso_params* prm, const maaso_score_weights* wts,
                          const maaso_score_out* out, void* hip_stream);

/* maaso_placement_score of the same candidates against n_sets (1..MAASO_MAX_REQUEST_SETS) request
 * sets at once: rq[k] is scored into out[k], HOST arrays of n_sets elements each, exactly as a call of
 * maaso_placement_score per set would - every set starts from the state as given in pl.  Alg. 2
 * (Sec. IV-E) needs the score of every candidate deployment against R_t, against R_l and, for its
 * homogeneous fallback, against all of R; the runs are independent, so one launch carries them all
 * and the device stays filled while the longest of them finishes.  No two sets may share an output
 * array.  Errors: INVALID_ARG, SHAPE, HIP. */
int maaso_placement_score_sets(maaso_ctx* ctx, const maaso_placements* pl, uint32_t n_sets,
                               const maaso_requests* rq, const maaso_params* prm,
                               const maaso_score_weights* wts, const maaso_score_out* out,
                               void* hip_stream);

/* Alg. 2, first step (Sec. IV-E: the requests are categorised by SLO into a strict set R_t and a
 * relaxed set R_l).  Classes whose bit is set in tight_classes form R_t.  The four request streams
 * are rewritten into the *_out arrays (DEVICE, [R] each): R_t first, R_l from index *n_tight on, both
 * in their original (arrival) order; *n_tight (DEVICE, [1]) receives |R_t|.  arrival_ticks_out is
 * required when rq->arrival_ticks is given and ignored otherwise.  Outputs must not alias inputs.
 * A request with slo_class >= n_slo raises MAASO_DEV_BAD_CLASS and stays with R_l.
 * Errors: INVALID_ARG, SHAPE, WORKSPACE, BUSY, HIP. */
int maaso_split_by_slo(maaso_ctx* ctx, const maaso_requests* rq, uint32_t tight_classes,
                       uint32_t* prompt_len_out, uint32_t* out_len_out, uint8_t* slo_class_out,
                       uint32_t* arrival_ticks_out, uint32_t* n_tight, void* hip_stream);

/* Alg. 1's bookkeeping (Sec. IV-E) over deployments that have already been scored, e.g. by
 * maaso_placement_score: phi_star[k] (DEVICE, [n_gpus+1]) is the best score among the accepted
 * deployments occupying exactly k GPUs (k = sum of tp_degree over the candidate's instances),
 * cand_star[k] its candidate index; 0 and -1 where there is none.
 *   chain_offsets == NULL: every candidate with a score > 0 that fits into n_gpus GPUs is accepted.
 *   chain_offsets (DEVICE, [n_chains+1], non-decreasing, last <= n_cand): chain i is the growth path
 *   of one configuration (P_i, B_i) - candidate chain_offsets[i] + m is the deployment after m + 1
 *   additions.  A candidate is accepted when all before it in its chain are, it fits, and its score
 *   is strictly larger than its predecessor's (0 before the first): Alg. 1 keeps an addition only if
 *   the score improves and otherwise stops growing that configuration (with one model the rejected
 *   model saturates the model set).  Scoring a whole chain at once and cutting it here gives what the
 *   sequential loop gives, because the loop's next deployment never depends on a rejected one.
 * Ties between configurations go to the lowest candidate index (Alg. 1 replaces an entry only on a
 * strictly larger score).  Only pl->n_cand, i_pad, n_inst and tp_idx are read.
 * Errors: INVALID_ARG (also: profile loaded without tp_degree), SHAPE, HIP. */
int maaso_ins_deploy_select(maaso_ctx* ctx, const maaso_placements* pl, const float* score,
                            const uint32_t* chain_offsets, uint32_t n_chains, uint32_t n_gpus,
                            float* phi_star, int32_t* cand_star, void* hip_stream);

/* Alg. 2's scan over the GPU partitions (Sec. IV-E).  phi_t_star / phi_l_star (DEVICE, [n_gpus+1]) are
 * Alg. 1's score lists for R_t and R_l.  The relaxed sub-cluster is tried at g_l = 1 .. G'_l GPUs,
 * G'_l = floor(|R_l| * |G| / |R|) (n_req_l, n_req: HOST scalars; 0 when n_req == 0), the strict one
 * takes g_t = n_gpus - g_l, and the partition with the largest phi_t_star[g_t] + phi_l_star[g_l]
 * (smallest g_l on ties) is chosen if that sum is strictly larger than the starting value: the largest
 * entry of phi_h_star (Alg. 1 on all requests and all GPUs, the homogeneous fallback; lowest GPU
 * count on ties), or 0 when phi_h_star is NULL.
 * partition (DEVICE, [6]): g_t, g_l, heterogeneous (1: a partition was chosen, 0: the fallback
 * stands, then g_t = k_h and g_l = 0), k_h (GPUs of the homogeneous deployment, 0 if none),
 * cand_t, cand_l (entries of cand_t_star[g_t] / cand_l_star[g_l], or cand_h_star[k_h] and -1 for
 * the fallback; -1 as 0xffffffff; the cand arrays may be NULL).  phi_opt (DEVICE, [1]): the score
 * that stands.  Errors: INVALID_ARG, SHAPE, HIP. */
int maaso_resource_partition(maaso_ctx* ctx, uint32_t n_gpus, const float* phi_t_star,
                             const float* phi_l_star, const float* phi_h_star,
                             const int32_t* cand_t_star, const int32_t* cand_l_star,
                             const int32_t* cand_h_star, uint64_t n_req_l, uint64_t n_req,
                             uint32_t* partition, float* phi_opt, void* hip_stream);

/* Batch-size pruning ahead of Alg. 1 (Sec. IV-E, "Inference Batch Size Pruning": for each
 * parallelism configuration only the batch sizes with a Pareto-optimal trade-off between latency
 * and SLO satisfaction are retained).  The candidates [group_offsets[g], group_offsets[g+1]) are the
 * batch sizes of configuration g, each already evaluated on the request set - for example as a
 * single-instance deployment by maaso_placement_score, with sat_count its admitted requests and
 * latency its Phi_L.  keep[c] (DEVICE, [n_cand]) becomes 0 when candidate c meets no request's SLO
 * (sat_count[c] == 0: the batch sizes too high to meet any deadline under load) or when another
 * candidate j of its group has sat_count[j] >= sat_count[c] and latency[j] <= latency[c] with one of
 * the two strict (the batch sizes too low: more latency, no more requests served), else 1; equal
 * candidates keep each other.  n_kept[g] (DEVICE, [n_groups]) counts the retained candidates of
 * group g.  group_offsets (DEVICE, [n_groups+1]) must be non-decreasing with its last entry at most
 * n_cand; a group that is not raises MAASO_DEV_BAD_CHAIN, gets n_kept 0 and leaves keep untouched.
 * Candidates outside every group are not written.  Errors: INVALID_ARG, SHAPE, BUSY, HIP. */
int maaso_batch_size_prune(maaso_ctx* ctx, uint32_t n_cand, const uint32_t* group_offsets,
                           uint32_t n_groups, const uint32_t* sat_count, const float* latency,
                           uint8_t* keep, uint32_t* n_kept, void* hip_stream);

/* Arrays that maaso_resource_partition_requests works in and reports through: all DEVICE,
 * caller-owned, distinct from each other and from the inputs.  R = rq->n_req, C = pl->n_cand. */
typedef struct {
  uint32_t* prompt_len_split;    /* [R] the request streams after the split: R_t first, then R_l */
  uint32_t* out_len_split;       /* [R]                                                           */
  uint8_t* slo_class_split;      /* [R]                                                           */
  uint32_t* arrival_ticks_split; /* [R]; required when rq->arrival_ticks is given                 */
  uint32_t* n_tight;             /* [1] |R_t|                                                     */
  uint32_t* sat_t;               /* [C] admitted requests of R_t per deployment                   */
  uint32_t* sat_l;               /* [C] ... of R_l                                                */
  uint32_t* sat_h;               /* [C] ... of all of R; required with score_h                    */
  float* score_t;                /* [C] Phi(I', R_t)                                              */
  float* score_l;                /* [C] Phi(I', R_l)                                              */
  float* score_h;                /* [C] Phi(I', R), or NULL: no homogeneous fallback              */
  float* phi_t_star;             /* [n_gpus+1] Alg. 1's lists, as maaso_ins_deploy_select writes  */
  float* phi_l_star;             /* [n_gpus+1]                                                    */
  float* phi_h_star;             /* [n_gpus+1]; required with score_h                             */
  int32_t* cand_t_star;          /* [n_gpus+1]                                                    */
  int32_t* cand_l_star;          /* [n_gpus+1]                                                    */
  int32_t* cand_h_star;          /* [n_gpus+1]; required with score_h                             */
  uint32_t* partition;           /* [6] as maaso_resource_partition writes it                     */
  float* phi_opt;                /* [1]                                                           */
} maaso_partition_work;

/* Alg. 2 from requests to partition in one call (Sec. IV-E): maaso_split_by_slo of rq by
 * tight_classes; the composite score of every deployment in pl against R_t, against R_l and - when
 * wk->score_h is given - against all of R, in one launch as maaso_placement_score_sets makes it;
 * maaso_ins_deploy_select over the growth chains (chain_offsets, n_chains: as there) for each of the
 * score lists; the scan of maaso_resource_partition with G'_l = floor(|R_l| * |G| / |R|).  |R_t| never
 * leaves the device: the scoring kernels and the scan read it from wk->n_tight, so the call enqueues
 * its launches and returns without waiting for any of them, and every result is what the five
 * calls in sequence would have written.  Nothing is allocated; the placements are not written.
 * Errors: INVALID_ARG, SHAPE, WORKSPACE, BUSY, HIP. */
int maaso_resource_partition_requests(maaso_ctx* ctx, const maaso_placements* pl,
                                      const uint32_t* chain_offsets, uint32_t n_chains,
                                      uint32_t n_gpus, const maaso_requests* rq,
                                      uint32_t tight_classes, const maaso_params* prm,
                                      const maaso_score_weights* wts,
                                      const maaso_partition_work* wk, void* hip_stream);

#ifdef __cplusplus
}
#endif
#endif /* MAASO_H */
