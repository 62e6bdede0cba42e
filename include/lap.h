/*
 * lap.h -- C ABI of liblap, the lifetime-aware pool planner for MI355X (gfx950).
 *
 * Offline planning for one training iteration's variable trace (arXiv
 * 1903.06631, Sections II-IV): every variable has a size and a fixed logical
 * time at which it is allocated and freed (Section III-A).  Three calls:
 *
 *   lap_load_profile  memory load per step and its peak (Section II, Def. 2
 *                     and Def. 4; Eq. 1: the peak is the weighted clique
 *                     number, a lower bound on any pool's footprint, Eq. 2).
 *   lap_plan_pool     SmartPool placement (Section III-C): variables taken in
 *                     a heuristic order, each put at the lowest address that
 *                     none of its already-placed, time-overlapping neighbours
 *                     uses (first-fit), or in the smallest hole between them
 *                     that fits (best-fit); many orders evaluated in parallel
 *                     and the smallest footprint kept.
 *   lap_score_swaps   AutoSwap candidate filter and priority scores (Section
 *                     IV-A, IV-B): DOA, AOA, WDOA, and the drop of the peak
 *                     load when the variable is away for its idle gap.
 *   lap_schedule_swaps  the swap-out / swap-in plan of Section IV-E and the load under it.
 *   lap_simulate_swaps  that plan replayed under a memory-load limit: the time a tight limit costs.
 *   lap_evaluate_weights  many weight vectors of the aggregated score (Section IV-C), each
 *                     walked to a limit and replayed: the overhead every vector would cause.
 *   lap_detect_iteration  finds one iteration in a recorded request stream (Section V).
 *   lap_select_swaps  AutoSwap selection (Section IV-D): candidates taken in
 *                     priority order until the peak load is within a limit,
 *                     for several scores (SWDOA of Section IV-B (iv) among
 *                     them) and limits at once; load_min of Section VI-B1.
 *
 * Conventions
 *   - Lifetimes are half-open: variable i is live during steps
 *     alloc[i] .. free[i]-1, with 0 <= alloc < free <= n_steps.  A variable
 *     freed at step t and one allocated at step t do not coexist.
 *   - Two variables are neighbours (edge of the interval graph of Section
 *     III-B) iff alloc_i < free_j && alloc_j < free_i.
 *   - gap_lo[i] <= gap_hi[i] are the two consecutive accesses (Section IV-B)
 *     that bound the variable's idle gap; NULL,NULL means alloc and free-1.
 *   - step_ns[t] is the compute time of step t in ns; NULL means 1 ms each.
 *
 * Memory and ownership
 *   - Every pointer inside lap_trace and every output / workspace pointer is
 *     a DEVICE pointer owned by the caller.  The library never allocates or
 *     frees device memory.  The lap_trace struct itself and every array marked
 *     "host" (orderings, score kinds, limits, weights, prefix lengths) are HOST
 *     memory; they are read before the call returns and reach the device inside
 *     kernel arguments, so the caller may reuse them at once and no call waits
 *     for such a copy.
 *   - Work is enqueued on the given HIP stream (a hipStream_t passed as
 *     void*; NULL = the default stream) and the call returns without waiting.
 *     Outputs, including the scalar ones, are valid once the stream has been
 *     synchronised.  lap_validate_trace is the exception: it waits.
 *   - ws must hold at least lap_workspace_bytes(...) bytes, 256-byte aligned.
 *     Two calls may run concurrently only on distinct workspaces.
 *
 * Errors: every call returns LAP_OK (0) or a negative code.  Argument errors
 * are detected on the host before anything is enqueued.  Trace-content errors
 * (LAP_E_TRACE, LAP_E_RANGE) are reported by lap_validate_trace only; the
 * other calls assume a valid trace.
 */
#ifndef LAP_H
#define LAP_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

enum {
    LAP_OK = 0,
    LAP_E_NULL = -1,       /* a required pointer is NULL (or only one of gap_lo/gap_hi given) */
    LAP_E_SIZE = -2,       /* n_vars, n_steps or B is 0, or a size exceeds the supported maximum */
    LAP_E_WORKSPACE = -3,  /* ws is NULL, misaligned or smaller than lap_workspace_bytes() */
    LAP_E_ORDERING = -4,   /* unknown ordering / score kind / fit, NULL explicit permutation, non-finite weight */
    LAP_E_LINK = -5,       /* link_GBps <= 0, not finite, or rounds to 0 bytes per microsecond */
    LAP_E_TRACE = -6,      /* size 0, alloc >= free, free > n_steps, gap outside [alloc, free-1], step_ns 0 */
    LAP_E_RANGE = -7,      /* sum of sizes >= 2^63, a size >= 2^53, sum of step_ns >= 2^53, max size * n_steps >= 2^64 */
    LAP_E_HIP = -8         /* a HIP runtime call or kernel launch failed */
};

/* One training iteration's variable trace (Section III-A), structure of arrays. */
typedef struct {
    uint32_t n_vars;          /* N > 0 */
    uint32_t n_steps;         /* T > 0 */
    const uint64_t *size;     /* [N] bytes, > 0 */
    const uint32_t *alloc;    /* [N] first live step */
    const uint32_t *free_;    /* [N] one past the last live step */
    const uint32_t *gap_lo;   /* [N] or NULL */
    const uint32_t *gap_hi;   /* [N] or NULL (both or neither) */
    const uint64_t *step_ns;  /* [T] or NULL */
} lap_trace;

/* Placement orders.  Ties in a key keep ascending variable index.
 *   SIZE_DESC   the paper's order: largest variable first (Section III-C)
 *   LIFE_DESC   longest lifetime (free - alloc) first
 *   AREA_DESC   largest size * lifetime first
 *   ALLOC_ASC   arrival order, what an online pool would see
 *   SEEDED      ascending splitmix64 output of (seed + (i+1) * 0x9E3779B97F4A7C15)
 *   EXPLICIT    seed holds a device pointer to a u32[N] permutation
 *               (placement rank -> variable index).  An array that is not a
 *               permutation of 0..N-1 is replaced by the identity order.
 *   CLASS_SEEDED  seeded shuffle inside size classes: class = floor(log2 size), larger
 *               classes first, ascending SEEDED key within a class -- random orders that
 *               stay close to the paper's largest-first order */
enum {
    LAP_ORD_SIZE_DESC = 0,
    LAP_ORD_LIFE_DESC = 1,
    LAP_ORD_AREA_DESC = 2,
    LAP_ORD_ALLOC_ASC = 3,
    LAP_ORD_SEEDED = 4,
    LAP_ORD_EXPLICIT = 5,
    LAP_ORD_CLASS_SEEDED = 6
};

/* Where a variable goes among the holes between its neighbours' blocks (Section III-C).
 *   FIT_FIRST  the lowest hole that is large enough (lowest feasible offset)
 *   FIT_BEST   the smallest hole that is large enough, the lowest of equally small ones (the
 *              paper's default).  A hole is a free range below the neighbours' highest end.
 * With both, a variable that fits no hole goes above the neighbours' highest end.
 * Cost: first-fit stops at the first hole that fits, best-fit looks at every one.  On traces whose
 * lifetimes are short (a transformer-shaped trace of 200 000 variables) best-fit takes 1.5 times as
 * long as first-fit; on dense interval graphs (tens of thousands of variables that mostly live
 * together) a variable can have thousands of fitting holes and best-fit takes minutes per ordering. */
enum { LAP_FIT_FIRST = 0, LAP_FIT_BEST = 1 };

typedef struct {
    uint32_t kind;  /* LAP_ORD_* */
    uint32_t fit;   /* LAP_FIT_*; zero-initialised descriptors plan first-fit */
    uint64_t seed;
} lap_ordering;

enum {
    LAP_WS_LOAD_PROFILE = 0,
    LAP_WS_PLAN_POOL = 1,
    LAP_WS_SCORE_SWAPS = 2,
    LAP_WS_VALIDATE = 3,
    LAP_WS_SELECT_SWAPS = 4,
    LAP_WS_DETECT_ITERATION = 5,  /* n_vars = number of requests */
    LAP_WS_SCHEDULE_SWAPS = 6,
    LAP_WS_SIMULATE_SWAPS = 7,    /* B = number of runs Q */
    LAP_WS_EVALUATE_WEIGHTS = 8   /* B = number of weight vectors W */
};

/* Bytes of workspace the given call needs.  B is the number of orderings for PLAN_POOL, the
 * number of score kinds for SELECT_SWAPS, and ignored otherwise.  Returns 0 for an unknown
 * call id. */
size_t lap_workspace_bytes(int which_call, uint32_t n_vars, uint32_t n_steps, uint32_t B);

/* Section II Def. 2 / Def. 4, Eq. 1.
 *   load   [T]  out: load[t] = sum of size[i] over variables live at step t
 *   peak   [1]  out: max_t load[t]
 *   t_peak [1]  out: earliest step where the peak occurs */
int lap_load_profile(const lap_trace *trace, uint64_t *load, uint64_t *peak, uint32_t *t_peak,
                     void *ws, size_t ws_bytes, void *hip_stream);

/* lap_load_profile for callers that cannot allocate device memory and have no workspace to pass
 * (code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc): same
 * arguments without ws, same kernels, same results.  The scratch (the difference array, 8 bytes
 * per step) is a fixed array inside the library's code object, (LAP_STATIC_MAX_STEPS + 1) * 8 bytes
 * = 8 MiB per GPU, held until the process ends; the call allocates nothing and frees nothing.
 *   - n_steps > LAP_STATIC_MAX_STEPS returns LAP_E_SIZE (and says so on stderr) before anything
 *     is enqueued; n_vars is not limited.
 *   - The first call on each device looks up the array's address on that device (no allocation, but
 *     a runtime query: make that first call outside a graph capture); later calls only launch.
 *   - All calls on one GPU share that GPU's array, whatever their stream: calls that overlap in
 *     time on one GPU race.  Order them on one stream or with events.  The array keeps the last
 *     call's contents; the kernels clear the part they use before they use it. */
#define LAP_STATIC_MAX_STEPS (1u << 20)
int lap_load_profile_static(const lap_trace *trace, uint64_t *load, uint64_t *peak, uint32_t *t_peak,
                            void *hip_stream);

/* Section III-C, for B orderings (each with its own fit policy) at once.
 *   ords           [B] host
 *   best_offsets   [N]   out: byte offset of every variable under the best ordering
 *   best_footprint [1]   out: pool size of the best ordering (max offset + size)
 *   best_ordering  [1]   out: index of the smallest footprint, lowest index on ties
 *   footprints     [B]   out or NULL
 *   all_offsets    [B*N] out or NULL: offsets under every ordering, ordering-major */
int lap_plan_pool(const lap_trace *trace, const lap_ordering *ords, uint32_t B,
                  uint64_t *best_offsets, uint64_t *best_footprint, uint32_t *best_ordering,
                  uint64_t *footprints, uint64_t *all_offsets,
                  void *ws, size_t ws_bytes, void *hip_stream);

/* Section IV-A / IV-B.  link_GBps is the host link in 10^9 bytes per second,
 * rounded to an integer number of bytes per microsecond; one transfer of
 * `size` bytes takes ceil(size*1000 / bytes_per_us) ns in either direction.
 *   load      [T] from lap_load_profile, or NULL to compute it here
 *   candidate [N] out: 1 iff size >= min_bytes, alloc <= t_peak < free, gap_hi > gap_lo
 *   doa_ns    [N] out: time between the two accesses minus both transfers (may be < 0)
 *   aoa       [N] out: doa*size if doa >= 0 else doa/size, one binary64 operation
 *   wdoa      [N] out: sum of load over the idle steps gap_lo+1 .. gap_hi-1
 *   peak_cut  [N] out: peak minus the peak of the load curve with the variable
 *                 removed from the whole steps between swap-out end and swap-in start
 * Variables with gap_hi == gap_lo get 0 in every output. */
int lap_score_swaps(const lap_trace *trace, double link_GBps, uint64_t min_bytes,
                    const uint64_t *load,
                    uint8_t *candidate, int64_t *doa_ns, double *aoa, uint64_t *wdoa, uint64_t *peak_cut,
                    void *ws, size_t ws_bytes, void *hip_stream);

/* Priority scores a selection can walk by (Section IV-B). */
enum { LAP_PS_DOA = 0, LAP_PS_AOA = 1, LAP_PS_WDOA = 2, LAP_PS_SWDOA = 3, LAP_PS_PEAK_CUT = 4,
       LAP_PS_CUSTOM = 5 /* internal: lap_evaluate_weights */ };

/* Section IV-D, for K priority scores and L load limits at once.  The candidates of
 * Section IV-A are put in priority order, highest score first, equal scores by ascending
 * variable index, and added to the swap list one by one; an added variable leaves the load
 * curve on the whole steps between the end of its swap-out and the start of its swap-in
 * (none if its DOA is negative).  A limit is served by the shortest prefix of the order whose
 * remaining peak is <= the limit, or by all candidates when the limit is out of reach.
 * LAP_PS_SWDOA (Section IV-B iv) builds its order as it goes: the next variable is the one
 * with the largest WDOA measured on the curve already reduced by the earlier picks.
 *   load, link_GBps, min_bytes   as for lap_score_swaps
 *   score_kinds [K] host, K <= 64          limits [L] host, L <= 1024 (L may be 0)
 *   order      [K*N]     out: order[k*N + j] = j-th variable of kind k's order, j < n_cand;
 *                             the rest of each row is left untouched
 *   rank       [K*N]     out or NULL: position of a variable in the order, 0xFFFFFFFF if not a candidate
 *   peaks      [K*(N+1)] out: peaks[k*(N+1) + j] = peak load after the first j additions, j <= n_cand
 *   n_cand     [1]       out: number of candidates
 *   n_selected [K*L]     out: variables selected for each limit
 *   peak_after [K*L]     out: peak load reached for each limit
 *   load_min   [1]       out: Section VI-B1, the peak of the curve with every candidate away on
 *                             all its idle steps gap_lo+1 .. gap_hi-1 (transfers not hidden)
 * The walk is sequential: one workgroup per score kind, about n_cand * (n_cand + T) / 1024
 * steps of work each. */
int lap_select_swaps(const lap_trace *trace, double link_GBps, uint64_t min_bytes, const uint64_t *load,
                     const uint32_t *score_kinds, uint32_t K, const uint64_t *limits, uint32_t L,
                     uint32_t *order, uint32_t *rank, uint64_t *peaks, uint32_t *n_cand,
                     uint32_t *n_selected, uint64_t *peak_after, uint64_t *load_min,
                     void *ws, size_t ws_bytes, void *hip_stream);

/* Section IV-E, the plan before any stall: the selected variables' swap-outs run one after the
 * other on one stream in ascending order of their access (ties: variable index), each as soon as
 * the access is over (end of step gap_lo) and the stream is free; their swap-ins run one after the
 * other on a second stream in the order of the next accesses, each as late as possible such that
 * it is done when its access begins (start of step gap_hi) and the swap-in after it can start on
 * time.  Times are ns from the start of the iteration; a swap-in time is negative when that
 * stream is overbooked.
 *   load       [T] from lap_load_profile, or NULL to compute it here
 *   swap_list  [k] device: distinct variable indices (for example a prefix of an order of
 *              lap_select_swaps); k may be 0
 *   out_start, out_end, in_start, in_end [k] out, by list position
 *   load_sched [T] out: load with every listed variable away on the whole steps between the end
 *              of its swap-out and the start of its swap-in
 *   peak_sched [1] out: its maximum
 *   late_ns    [1] out: sum of max(0, out_end - in_start), transfer time the plan cannot hide
 * The stalls that a tight limit forces on top of this plan are not modelled. */
int lap_schedule_swaps(const lap_trace *trace, double link_GBps, const uint64_t *load,
                       const uint32_t *swap_list, uint32_t k,
                       int64_t *out_start, int64_t *out_end, int64_t *in_start, int64_t *in_end,
                       uint64_t *load_sched, uint64_t *peak_sched, uint64_t *late_ns,
                       void *ws, size_t ws_bytes, void *hip_stream);

/* Section IV-E under a memory-load limit: one iteration replayed as a discrete-event machine, Q
 * runs at once.  Run q swaps the first prefix_len[q] variables of swap_list (those with an idle
 * gap) under limits[q] bytes.
 *   compute   runs the steps in order; a step starts when the one before it has ended, every swapped
 *             variable accessed at that step (gap_hi) is back, and -- if the step allocates -- resident
 *             bytes + the bytes it allocates <= limit (the delayed Malloc)
 *   swap-out  one stream, ascending (gap_lo, index); issued when step gap_lo ends
 *   swap-in   a second stream, ascending (gap_hi, index); issued when compute reaches the step boundary
 *             at or before its start in the plan of lap_schedule_swaps for these variables (not before
 *             boundary gap_lo+1); starts when issued, the stream is free, its own swap-out has ended
 *             and resident + size <= limit
 *   resident  + at a step's start (its allocations) and a swap-in's start; - at a step's end (its frees)
 *             and a swap-out's end
 *   one instant: ends first, then starts in the order swap-out, step, swap-in.  If nothing runs and the
 *   next step cannot start, the limit is overridden once (counted in forced) for the step's allocations,
 *   else for the swap-in at the head of its stream.
 * swap_list [k_max] device, distinct indices; prefix_len, limits [Q] host, Q <= 4096.
 * Outputs [Q] device: total_ns (end of the last step), overhead_ns = total - sum of step_ns,
 * peak_resident (largest resident value), forced. */
int lap_simulate_swaps(const lap_trace *trace, double link_GBps, const uint32_t *swap_list, uint32_t k_max,
                       const uint32_t *prefix_len, const uint64_t *limits, uint32_t Q,
                       uint64_t *total_ns, uint64_t *overhead_ns, uint64_t *peak_resident, uint32_t *forced,
                       void *ws, size_t ws_bytes, void *hip_stream);

/* Section IV-C, Eq. 3: the aggregated priority score BO = a*AOA + b*DOA + c*WDOA + d*SWDOA, whose
 * weights are tuned against the communication overhead of the schedule it leads to.  This call
 * evaluates W weight vectors at once; the optimiser that proposes them is the caller's.
 *   weights [W*4] host, rows (a, b, c, d), finite, W <= 64.  They apply to the RAW scores:
 *           standardising a score is an affine map, so for the induced order it only rescales
 *           that score's weight (fold 1/sigma into it).
 *   SWDOA_i = the WDOA variable i had on the reduced curve when the SWDOA walk picked it.
 *   BO is one binary64 expression, ((a*AOA + b*DOA) + c*WDOA) + d*SWDOA, not contracted.
 * For every vector: candidates in descending BO (ties: lower index) are selected until the peak
 * load is <= limit (lap_select_swaps), and that selection is replayed under the limit
 * (lap_simulate_swaps).
 *   order      [W*N] out: row w = the vector's priority order (first n_cand entries)
 *   n_cand [1], n_selected [W], peak_after [W], overhead_ns [W], forced [W] out
 *   best   [1] out: the vector with the least overhead_ns, the lowest index among equals
 *   swdoa  [N] out: the SWDOA values (0 for non-candidates) */
int lap_evaluate_weights(const lap_trace *trace, double link_GBps, uint64_t min_bytes, const uint64_t *load,
                         const double *weights, uint32_t W, uint64_t limit,
                         uint32_t *order, uint32_t *n_cand, uint32_t *n_selected, uint64_t *peak_after,
                         uint64_t *overhead_ns, uint32_t *forced, uint32_t *best, uint64_t *swdoa,
                         void *ws, size_t ws_bytes, void *hip_stream);

/* Section V: the requests of the first iterations are recorded in a list, and an iteration has
 * been seen once the list ends with two equal consecutive subsequences; that subsequence is one
 * iteration's operations.
 *   tokens [n_requests] device: one 64-bit value per recorded request (operation kind and size,
 *                       whatever the caller folds in; not the address, which changes between
 *                       iterations)
 *   min_period >= 1     shortest iteration the caller accepts (guards against a short repeat
 *                       inside an iteration that happens to end the list)
 *   period [1] device   out: the smallest p >= min_period with tokens[M-2p+i] == tokens[M-p+i]
 *                       for all i < p, or 0 if there is none; the iteration is tokens[M-p .. M) */
int lap_detect_iteration(const uint64_t *tokens, uint32_t n_requests, uint32_t min_period, uint32_t *period,
                         void *ws, size_t ws_bytes, void *hip_stream);

/* Checks the trace content on the device, waits for the stream, and returns
 * LAP_OK, LAP_E_TRACE or LAP_E_RANGE. */
int lap_validate_trace(const lap_trace *trace, void *ws, size_t ws_bytes, void *hip_stream);

const char *lap_status_string(int status);

/* Tuning knobs, process-wide and not thread safe: set them before the calls they affect.
 *   LAP_OPT_SEG_MIN_VARS  lap_plan_pool has three ways to keep track of free addresses and picks
 *       one per trace on the device: per-step free lists when the lifetimes are short (their sum
 *       is at most 6 N), else, for first-fit orderings, free lists per time segment when the
 *       trace has at least this many variables (default 32768) and the workspace has room for
 *       them, else a sweep over the sorted list of placed blocks.  All three give the same
 *       offsets.  0 = segment lists whenever they apply.
 *   LAP_OPT_SEG_TRIAL_PERCENT  whether the segment lists pay also depends on how their searches
 *       converge (two to three rounds on traces with nested lifetimes, as a training iteration
 *       has; six to eight with lifetimes at random, where the sweep is faster).  Before they are
 *       used, one workgroup places the first 2048 variables of the first first-fit ordering with
 *       them and counts the rounds of the multi-step variables; above this many rounds per
 *       variable, times 100 (default 250), the sweep places the trace.  0 = no trial.
 * Returns LAP_E_ORDERING for an unknown option or value. */
enum { LAP_OPT_SEG_MIN_VARS = 0, LAP_OPT_SEG_TRIAL_PERCENT = 1 };
int lap_set_option(int option, uint64_t value);

/* Optional kernel timing for benchmarks, per calling thread.  When a thread has enabled it, each of
 * its calls brackets its dominant kernel with HIP events on the caller's stream; after the stream is
 * synchronised lap_profile_last_ms, called by the same thread, returns that kernel's duration in ms
 * (negative if none was recorded).  LAP_K_PLACE covers every placement kernel a lap_plan_pool call
 * launches (those that do not apply to the trace or to an ordering's policy return at once).  The
 * event records do not belong inside a graph capture: leave the timing off there. */
enum { LAP_K_LOAD_SCATTER = 0, LAP_K_PLACE = 1, LAP_K_SCORE = 2, LAP_K_SORT = 3, LAP_K_SELECT = 4, LAP_K_COUNT = 5 };
int lap_profile_enable(int on);
float lap_profile_last_ms(int kernel_id);
/* How long the placement kernel worked on every ordering of the last lap_plan_pool call that used
 * this workspace with these n_vars, n_steps and B (always recorded, by the device's constant-rate
 * timer): the launch ends with its slowest ordering.  Waits for the stream.
 *   ms_host [B] HOST out */
int lap_profile_ordering_ms(uint32_t n_vars, uint32_t n_steps, uint32_t B, const void *ws, size_t ws_bytes,
                            void *hip_stream, float *ms_host);

/* The placement orders of the last lap_plan_pool call that used this workspace with these n_vars,
 * n_steps and B (Section III-C: the heuristic order in which the variables are placed; kinds and
 * tie rule as documented at lap_ordering): orders[b * n_vars + r] = the variable that ordering b
 * placed r-th.  A device-to-device copy enqueued on the stream; the call does not wait.  What it
 * returns before any lap_plan_pool call on the workspace, or after another call has used it, is
 * unspecified (but never read or written out of bounds).
 *   orders [B * n_vars] DEVICE out, caller-owned
 * Errors: LAP_E_NULL, LAP_E_SIZE (a zero count), LAP_E_WORKSPACE, LAP_E_HIP. */
int lap_plan_pool_orders(uint32_t n_vars, uint32_t n_steps, uint32_t B, const void *ws, size_t ws_bytes,
                         void *hip_stream, uint32_t *orders);

#ifdef __cplusplus
}
#endif
#endif /* LAP_H */
