// Host-side launch wrappers of the liblap kernels (one per kernel family).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace lap {

// candidate segment widths of the segment kernel: 2^PLAN_SEG_SHIFT0 .. 2^(PLAN_SEG_SHIFT0 + PLAN_SEG_CAND - 1) steps
constexpr uint32_t PLAN_SEG_SHIFT0 = 2, PLAN_SEG_CAND = 9;
// list entries of the segment kernel's pool per ordering and variable (the pool is shared: an
// ordering that needs more leaves fewer slots)
constexpr uint32_t PLAN_SEG_BUDGET = 27;

// Per-call facts about the trace, computed on the device before placement.
struct PlanHeader {
    unsigned long long or_sizes;   // bitwise OR of all sizes
    unsigned long long sum_sizes;  // sum of all sizes (bytes)
    uint32_t n_multi;              // variables that live for more than one step
    uint32_t shift;                // log2 of the offset granule: ctz(or_sizes)
    uint32_t fast;                 // 1: sum_sizes >> shift fits 32 bits -> packed 32-bit path
    uint32_t mode1;                // 1: per-step lists are in use (sum of lifetimes <= PLAN_CL * N)
    uint32_t part[2];              // placement workgroups that have started, per fit policy
    uint32_t progress[2];          // their progress, in units of 512 ranks, summed
    // segment lists (place_seg.hip), used when per-step lists are not and the pool has room
    uint32_t mode2;                // 1: the segment kernel places this trace
    uint32_t seg_shift;            // log2 of the segment width in steps
    uint32_t seg_K;                // number of segments
    uint32_t seg_slots;            // orderings that have room in the list pool at once
    unsigned long long seg_need;   // list entries one ordering needs
    unsigned long long seg_tot[PLAN_SEG_CAND];   // per candidate width: blocks entered into lists, summed over the variables
    uint32_t seg_trial_rounds;     // trial run: search rounds of its multi-step variables, summed
    uint32_t seg_trial_vars;       // ... and how many those were
    uint32_t seg_next;             // next ordering to hand to a workgroup of the segment kernel
    uint32_t seg_pad;
};
constexpr uint32_t PLAN_CL = 6;

hipError_t launch_fill_u64(uint64_t *p, size_t n, uint64_t v, hipStream_t st);
// copies n_words 32-bit words of HOST memory to the device through kernel arguments (the host
// array is read before the call returns; nothing waits)
hipError_t launch_put_words(void *dst, const void *host_src, size_t n_words, hipStream_t st);
hipError_t launch_delta(uint32_t n, uint32_t T, const uint64_t *size, const uint32_t *alloc, const uint32_t *free_,
                        uint64_t *delta, hipStream_t st);
hipError_t launch_scan_peak(uint32_t T, uint64_t *delta, uint64_t *load, uint64_t *peak, uint32_t *t_peak,
                            hipStream_t st);
hipError_t launch_validate(uint32_t n, uint32_t T, const uint64_t *size, const uint32_t *alloc, const uint32_t *free_,
                           const uint32_t *gap_lo, const uint32_t *gap_hi, const uint64_t *step_ns, uint64_t *out8,
                           hipStream_t st);

hipError_t launch_sort_perm(uint32_t n, uint32_t B, const uint64_t *size, const uint32_t *alloc, const uint32_t *free_,
                            const uint32_t *kinds, const uint64_t *seeds, uint32_t *perm, uint32_t *tmp,
                            bool any_explicit, hipStream_t st);
hipError_t launch_plan_prep(uint32_t n, uint32_t T, uint32_t B, const uint64_t *size, const uint32_t *alloc,
                            const uint32_t *free_, uint32_t *cntd, uint32_t *lstart, PlanHeader *hdr, void *vrec,
                            uint64_t seg_pool_entries, uint64_t seg_min_vars, hipStream_t st);
hipError_t launch_seg_prep(uint32_t n, uint32_t T, uint32_t B, const uint32_t *alloc, const uint32_t *free_,
                           PlanHeader *hdr, uint32_t *cnt, uint32_t *lst, uint32_t dir_cap, uint64_t pool_entries,
                           hipStream_t st);
// trial_b: ordering whose first ranks are placed ahead of time to see how the searches go (negative:
// no trial); trial_percent: rounds per multi-step variable, times 100, above which the sweep is kept
hipError_t launch_seg_trial(uint32_t n, uint32_t T, uint32_t B, const uint32_t *perm, const uint32_t *fits,
                            int trial_b, uint32_t trial_percent, PlanHeader *hdr, const void *vrec, const uint32_t *lst,
                            uint64_t *pool, uint32_t *lens, uint32_t dir_cap, uint64_t *offs, uint64_t *fps,
                            uint64_t *ticks, hipStream_t st);
hipError_t launch_place_seg(uint32_t n, uint32_t T, uint32_t B, const uint32_t *perm, const uint32_t *fits,
                            bool any_first, PlanHeader *hdr, const void *vrec, const uint32_t *lst,
                            uint64_t *pool, uint32_t *lens, uint32_t dir_cap, uint64_t *offs, uint64_t *fps,
                            uint64_t *ticks, hipStream_t st);
hipError_t launch_place_fast(uint32_t n, uint32_t T, uint32_t B, const uint64_t *size, const uint32_t *alloc,
                             const uint32_t *free_, const uint32_t *perm, const uint32_t *fits, bool any_first,
                             bool any_best, PlanHeader *hdr, const void *vrec,
                             const uint32_t *lstart, uint64_t *m_oe, uint64_t *m_life, uint64_t *m_oe2,
                             uint64_t *m_life2, uint64_t *r_oe, uint64_t *r_life, uint64_t *r_oe2,
                             uint64_t *r_life2, uint64_t *L, uint64_t capL,
                             uint32_t *l_ns, uint32_t *l_nu, uint64_t *offs, uint64_t *fps, uint64_t *ticks,
                             hipStream_t st);
constexpr uint32_t PLAN_REC = 4096;   // entries of the sorted "recent" list per ordering
hipError_t launch_place_wide(uint32_t n, uint32_t B, const uint64_t *size, const uint32_t *alloc,
                             const uint32_t *free_, const uint32_t *perm, const uint32_t *fits,
                             const PlanHeader *hdr, uint64_t *m_off,
                             uint64_t *m_end, uint64_t *m_life, uint64_t *offs, uint64_t *fps, uint64_t *ticks,
                             hipStream_t st);
hipError_t launch_select(uint32_t n, uint32_t B, const uint64_t *fps, const uint64_t *offs_rank, const uint32_t *perm,
                         uint64_t *best_fp, uint32_t *best_idx, uint64_t *best_offsets, uint64_t *all_offsets,
                         hipStream_t st);

hipError_t launch_swap_prefix(uint32_t T, const uint64_t *load, const uint64_t *step_ns, uint64_t *C, uint64_t *S,
                              uint64_t *PM, uint64_t *SM, uint64_t *peak, uint32_t *t_peak, hipStream_t st);
hipError_t launch_sparse_table(uint32_t T, const uint64_t *load, uint64_t *table, uint32_t levels, hipStream_t st);
hipError_t launch_score(uint32_t n, uint32_t T, const uint64_t *size, const uint32_t *alloc, const uint32_t *free_,
                        const uint32_t *gap_lo, const uint32_t *gap_hi, uint64_t bpus, uint64_t min_bytes,
                        const uint64_t *load, const uint64_t *C, const uint64_t *S, const uint64_t *PM,
                        const uint64_t *SM, const uint64_t *table, const uint64_t *peak, const uint32_t *t_peak,
                        uint8_t *cand, int64_t *doa, double *aoa, uint64_t *wdoa, uint64_t *cut, uint32_t *win_lo,
                        uint32_t *win_hi, hipStream_t st);

// Selection of swap variables (select_swaps.hip).  All pointers are device memory.
struct SelectArgs {
    uint32_t n, T, K, L;
    const uint64_t *size;
    const uint32_t *gap_lo, *gap_hi, *alloc, *free_;
    const uint64_t *load;
    const uint8_t *cand;
    const int64_t *doa;
    const double *aoa;
    const uint64_t *wdoa, *cut;
    const uint32_t *win_lo, *win_hi;
    uint32_t *nc;              // [1] number of candidates (device counter)
    uint32_t *cidx;            // [n] candidate slot -> variable
    uint32_t *c_ilo, *c_ihi;   // [n] idle steps [ilo, ihi) of the candidate in a slot
    uint64_t *dmin;            // [T+1] difference array of the load removed for load_min
    const uint32_t *kinds;     // [K]
    const uint64_t *limits;    // [L]
    uint64_t *r_score;         // [K][n] current score of every slot
    uint32_t *r_var;           // [K][n] variable of the slot, 0xFFFFFFFF once taken
    uint64_t *l_cur;           // [K][T] current load curve
    uint32_t *order, *rank;    // [K][n] outputs (rank may be null)
    uint64_t *peaks;           // [K][n+1]
    uint32_t *n_cand;          // [1]
    uint32_t *n_selected;      // [K][L]
    uint64_t *peak_after;      // [K][L]
    uint64_t *load_min;        // [1]
    const double *custom;      // [K][n] score of kind 5 (custom), row = position in kinds; else null
    uint64_t *pick_wdoa;       // [n] or null: for a SWDOA walk, the score a variable had when it was picked
};
// gather = build the candidate slots and load_min first (once per trace and candidate filter)
hipError_t launch_select_swaps(const SelectArgs &a, bool gather, hipStream_t st);
hipError_t launch_weighted_scores(uint32_t n, uint32_t W, const double *weights, const double *aoa, const int64_t *doa,
                                  const uint64_t *wdoa, const uint64_t *swdoa, double *bo, hipStream_t st);
hipError_t launch_argmin_u64(uint32_t n, const uint64_t *v, uint32_t *best, hipStream_t st);

hipError_t launch_schedule_swaps(uint32_t n, uint32_t T, uint32_t k, const uint64_t *size, const uint32_t *step_lo,
                                 const uint32_t *step_hi, uint32_t hi_minus, const uint64_t *C,
                                 const uint32_t *perm_lo, const uint32_t *perm_hi, uint32_t *posmap,
                                 const uint32_t *list, uint64_t bpus, int64_t *out_start, int64_t *out_end,
                                 int64_t *in_start, int64_t *in_end, uint64_t *diff, uint64_t *late,
                                 const uint64_t *load, uint64_t *load_sched, uint64_t *peak, hipStream_t st);

hipError_t launch_simulate_swaps(uint32_t n, uint32_t T, uint32_t Q, uint32_t kmax, const uint64_t *size,
                                 const uint32_t *alloc, const uint32_t *free_, const uint32_t *step_lo,
                                 const uint32_t *step_hi, uint32_t hi_minus, const uint64_t *C, uint64_t *need,
                                 uint64_t *rel, const uint32_t *list, const uint32_t *perm_lo,
                                 const uint32_t *perm_hi, const uint32_t *posmap, uint32_t *jobs_lo,
                                 uint32_t *jobs_hi, uint32_t *m, const uint32_t *prefix, const uint64_t *limits,
                                 uint32_t *kb, uint8_t *out_done, uint64_t bpus, uint64_t *total_ns,
                                 uint64_t *overhead_ns, uint64_t *peak_resident, uint32_t *forced, hipStream_t st,
                                 uint32_t n_lists = 1, const uint32_t *n_listed = nullptr);
hipError_t launch_sched_mark(uint32_t n, uint32_t k, const uint32_t *list, uint32_t *posmap, hipStream_t st);

hipError_t launch_detect_iteration(const uint64_t *tokens, uint32_t M, uint32_t min_period, uint64_t *P,
                                   uint32_t *period, hipStream_t st);

}  // namespace lap
