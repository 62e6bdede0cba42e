// extern "C" entry points of liblap: argument checks, workspace carving, launches.
#include <math.h>
#include <stdio.h>
#include <string.h>

#include <algorithm>
#include <mutex>
#include <vector>

#include "../../include/lap.h"
#include "lap_kernels.h"

namespace {

constexpr size_t ALIGN = 256;
inline size_t up(size_t x) { return (x + ALIGN - 1) / ALIGN * ALIGN; }

struct Carver {
    char *base;
    size_t used = 0;
    explicit Carver(void *p) : base((char *)p) {}
    template <class T> T *take(size_t count)
    {
        T *r = (T *)(base + used);
        used += up(count * sizeof(T));
        return r;
    }
};

inline uint32_t table_levels(uint32_t T)
{
    uint32_t lv = 1;
    while ((1ull << lv) <= T) ++lv;
    return lv;                       // floor(log2 T) + 1
}

size_t ws_load(uint32_t T) { return up(((size_t)T + 1) * 8); }

// entries of the per-step lists of one ordering: PLAN_CL per variable, a whole number of 128-byte lines
inline uint64_t plan_list_cap(uint32_t n) { return ((uint64_t)n * lap::PLAN_CL + 15) & ~15ull; }

// block lists of the placement kernels: the 64-bit path needs off/end/life per ordering, the
// packed 32-bit path a packed main list with lifetimes, the per-step lists and their counters
// entries of the segment kernel's list pool (all orderings together), and of its list directory
inline size_t seg_pool_entries(uint32_t n, uint32_t B) { return (size_t)B * n * lap::PLAN_SEG_BUDGET; }
inline size_t seg_dir_cap(uint32_t T) { return (size_t)T + 2 * (((size_t)T >> lap::PLAN_SEG_SHIFT0) + 1) + 1; }

size_t ws_plan_lists(uint32_t n, uint32_t T, uint32_t B)
{
    const size_t bn = (size_t)B * n;
    const size_t wide = 3 * up(bn * 8);
    const size_t fast = 4 * up(bn * 8) + 4 * up((size_t)B * lap::PLAN_REC * 8) + up((size_t)B * plan_list_cap(n) * 8) +
                        up((size_t)B * T * 4) + up((size_t)B * T * 8);       // per-step lists: sorted counts; unsorted counts and top holes
    const size_t seg = up(seg_pool_entries(n, B) * 8);
    return std::max(wide, std::max(fast, seg));
}

size_t ws_plan(uint32_t n, uint32_t T, uint32_t B)
{
    const size_t bn = (size_t)B * n;
    return up(sizeof(lap::PlanHeader)) + 2 * up(((size_t)T + 2) * 4)   // header, step counts, list starts
           + 2 * up((size_t)B * 4) + 2 * up((size_t)B * 8)            // kinds, fit policies, seeds, durations
           + 2 * up(bn * 4)                                            // perm, sort scratch
           + up((size_t)B * 8)                                         // footprints
           + up((size_t)n * 16)                                        // packed variable records
           + up(bn * 8)                                                // offsets of every ordering
           + 2 * up((seg_dir_cap(T) + 2) * 4)                          // segment lists: blocks per list, list starts
           + up((size_t)B * seg_dir_cap(T) * 8)                        // and their lengths and topmost ranges, per slot
           + ws_plan_lists(n, T, B);
}

size_t ws_score(uint32_t T)
{
    const size_t t1 = (size_t)T + 1;
    return up((size_t)T * 8) + up(t1 * 8)              // load, delta
           + 4 * up(t1 * 8)                            // C, S, PM, SM
           + up((size_t)table_levels(T) * T * 8)       // range-max table
           + 2 * ALIGN;                                // peak, t_peak
}

size_t ws_validate() { return up(8 * 8); }

constexpr uint32_t SELECT_MAX_LIMITS = 1024;
constexpr uint32_t SELECT_MAX_KINDS = 64;

size_t ws_schedule(uint32_t n, uint32_t T)
{
    const size_t t1 = (size_t)T + 1, N = n;
    return up((size_t)T * 8) + 6 * up(t1 * 8)          // load, delta, C, S, PM, SM, diff  (diff counted below)
           + up(t1 * 8) + 2 * ALIGN                    // diff; peak, t_peak
           + 4 * up(N * 4) + 2 * ALIGN;                // posmap, perm_lo, perm_hi, sort scratch; kinds, seeds
}

constexpr uint32_t SIM_MAX_RUNS = 4096;

size_t ws_simulate(uint32_t n, uint32_t T, uint32_t Q)
{
    const size_t t1 = (size_t)T + 1, N = n;
    return up((size_t)T * 8) + 5 * up(t1 * 8) + 2 * ALIGN          // load, delta, C, S, PM, SM; peak, t_peak
           + 2 * up((size_t)T * 8)                                 // bytes allocated / freed per step
           + 6 * up(N * 4) + 3 * ALIGN                             // posmap, perm x2, sort scratch, jobs x2; kinds, seeds, m
           + up((size_t)SIM_MAX_RUNS * 4) + up((size_t)SIM_MAX_RUNS * 8)   // prefix lengths, limits
           + (size_t)Q * (up(N * 4) + up(N));                      // per run: issue boundaries, swap-out flags
}

size_t ws_select(uint32_t n, uint32_t T, uint32_t K);

size_t ws_weights(uint32_t n, uint32_t T, uint32_t W)
{
    const size_t N = n, w = W;
    return ws_select(n, T, 0) + up(SELECT_MAX_KINDS * 8) + up(SELECT_MAX_KINDS * 32) + ALIGN
           + up(w * N * 8) + up(w * N * 4) + up(w * T * 8) + up(w * (N + 1) * 8) + up(w * N * 8)   // walk state, peaks, scores
           + 2 * up((size_t)T * 8) + 3 * up(N * 4) + 2 * ALIGN                                      // steps, perms
           + up((w * N + 1) * 4) + 2 * up(w * N * 4) + up(w * 4) + up(w * N * 4) + up(w * N)        // replay state
           + 2 * up(w * 8);
}

size_t ws_select(uint32_t n, uint32_t T, uint32_t K)
{
    const size_t N = n;
    return ws_score(T) + up(N) + 4 * up(N * 8) + 2 * up(N * 4)      // scores and away windows of every variable
           + 3 * up(N * 4) + up(((size_t)T + 1) * 8) + ALIGN          // candidate slots, load_min differences, counter
           + up((size_t)SELECT_MAX_KINDS * 4) + up((size_t)SELECT_MAX_LIMITS * 8)
           + (size_t)K * (up(N * 8) + up(N * 4) + up((size_t)T * 8)); // per kind: slot scores, slot variables, curve
}

int check_trace_args(const lap_trace *tr)
{
    if (!tr) return LAP_E_NULL;
    if (!tr->size || !tr->alloc || !tr->free_) return LAP_E_NULL;
    if ((tr->gap_lo == nullptr) != (tr->gap_hi == nullptr)) return LAP_E_NULL;
    if (tr->n_vars == 0 || tr->n_steps == 0) return LAP_E_SIZE;
    if (tr->n_steps == 0xFFFFFFFFu) return LAP_E_SIZE;   // n_steps + 1 bins must fit 32 bits
    return LAP_OK;
}

int check_ws(void *ws, size_t have, size_t need)
{
    if (!ws || ((uintptr_t)ws % ALIGN) != 0 || have < need) return LAP_E_WORKSPACE;
    return LAP_OK;
}

// lap_set_option(LAP_OPT_SEG_MIN_VARS): variables from which on the segment lists are used
uint64_t g_seg_min_vars = 32768;
// lap_set_option(LAP_OPT_SEG_TRIAL_PERCENT): search rounds per multi-step variable (times 100) in the
// trial run above which the segment lists are not used; 0 = no trial
uint64_t g_seg_trial_percent = 250;

// kernel timing is per calling thread: each thread that enables it gets events of its own
thread_local bool g_prof = false;
thread_local hipEvent_t g_ev[LAP_K_COUNT][2];
thread_local bool g_ev_made[LAP_K_COUNT];
thread_local bool g_ev_used[LAP_K_COUNT];

struct ProfScope {
    int id;
    hipStream_t st;
    bool on;
    ProfScope(int id_, hipStream_t st_) : id(id_), st(st_), on(g_prof)
    {
        if (!on) return;
        if (!g_ev_made[id]) {
            if (hipEventCreate(&g_ev[id][0]) != hipSuccess || hipEventCreate(&g_ev[id][1]) != hipSuccess) {
                on = false;
                return;
            }
            g_ev_made[id] = true;
        }
        (void)hipEventRecord(g_ev[id][0], st);
    }
    ~ProfScope()
    {
        if (!on) return;
        (void)hipEventRecord(g_ev[id][1], st);
        g_ev_used[id] = true;
    }
};

// a failing HIP call is reported on stderr (with the runtime's message) and as LAP_E_HIP
#define LAP_HIP(expr)                                                                          \
    do {                                                                                       \
        const hipError_t lap_e_ = (expr);                                                      \
        if (lap_e_ != hipSuccess) {                                                            \
            fprintf(stderr, "liblap: %s failed: %s\n", #expr, hipGetErrorString(lap_e_));      \
            return LAP_E_HIP;                                                                  \
        }                                                                                      \
    } while (0)

int load_profile_impl(const lap_trace *tr, uint64_t *load, uint64_t *peak, uint32_t *t_peak, uint64_t *delta,
                      hipStream_t st)
{
    const uint32_t n = tr->n_vars, T = tr->n_steps;
    LAP_HIP(lap::launch_fill_u64(delta, (size_t)T + 1, 0, st));
    {
        ProfScope p(LAP_K_LOAD_SCATTER, st);
        LAP_HIP(lap::launch_delta(n, T, tr->size, tr->alloc, tr->free_, delta, st));
    }
    LAP_HIP(lap::launch_scan_peak(T, delta, load, peak, t_peak, st));
    return LAP_OK;
}

// Scratch of lap_load_profile_static: the difference array of the largest supported time line.
// One copy per GPU, held from module load to process end.  In host code the name only stands
// for the symbol; its device address comes from hipGetSymbolAddress, once per device.
constexpr uint32_t STATIC_MAX_STEPS = LAP_STATIC_MAX_STEPS;
constexpr size_t STATIC_SCRATCH_BYTES = ((size_t)STATIC_MAX_STEPS + 1) * 8;
static __device__ __align__(256) unsigned char scratch[(STATIC_SCRATCH_BYTES + 255) / 256 * 256];

constexpr int MAX_DEVICES = 64;
std::mutex g_scratch_mu;
void *g_scratch_ptr[MAX_DEVICES];      // per device: address of its copy of `scratch`, null until asked for

// address of the current device's copy of the scratch array (no allocation: the array is part of
// the loaded code object)
int static_scratch(void **out)
{
    int dev = -1;
    LAP_HIP(hipGetDevice(&dev));
    if (dev < 0 || dev >= MAX_DEVICES) return LAP_E_HIP;
    std::lock_guard<std::mutex> lock(g_scratch_mu);
    if (!g_scratch_ptr[dev]) {
        void *p = nullptr;
        LAP_HIP(hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)));
        if (!p) return LAP_E_HIP;
        g_scratch_ptr[dev] = p;
    }
    *out = g_scratch_ptr[dev];
    return LAP_OK;
}

}  // namespace

extern "C" {

size_t lap_workspace_bytes(int which, uint32_t n_vars, uint32_t n_steps, uint32_t B)
{
    switch (which) {
    case LAP_WS_LOAD_PROFILE: return ws_load(n_steps);
    case LAP_WS_PLAN_POOL: return ws_plan(n_vars, n_steps, B);
    case LAP_WS_SCORE_SWAPS: return ws_score(n_steps);
    case LAP_WS_VALIDATE: return ws_validate();
    case LAP_WS_SELECT_SWAPS: return ws_select(n_vars, n_steps, B);
    case LAP_WS_DETECT_ITERATION: return up(((size_t)n_vars + 1) * 8);
    case LAP_WS_SCHEDULE_SWAPS: return ws_schedule(n_vars, n_steps);
    case LAP_WS_SIMULATE_SWAPS: return ws_simulate(n_vars, n_steps, B);
    case LAP_WS_EVALUATE_WEIGHTS: return ws_weights(n_vars, n_steps, B);
    default: return 0;
    }
}

const char *lap_status_string(int s)
{
    switch (s) {
    case LAP_OK: return "ok";
    case LAP_E_NULL: return "null pointer argument";
    case LAP_E_SIZE: return "zero or unsupported size";
    case LAP_E_WORKSPACE: return "workspace missing, misaligned or too small";
    case LAP_E_ORDERING: return "bad ordering descriptor or score kind";
    case LAP_E_LINK: return "bad link bandwidth";
    case LAP_E_TRACE: return "invalid trace content";
    case LAP_E_RANGE: return "trace values out of the supported range";
    case LAP_E_HIP: return "HIP runtime error";
    default: return "unknown status";
    }
}

int lap_set_option(int option, uint64_t value)
{
    if (option == LAP_OPT_SEG_MIN_VARS) g_seg_min_vars = value;
    else if (option == LAP_OPT_SEG_TRIAL_PERCENT && value <= 0xFFFFFFFFull) g_seg_trial_percent = value;
    else return LAP_E_ORDERING;
    return LAP_OK;
}

int lap_profile_enable(int on)
{
    g_prof = on != 0;
    for (int i = 0; i < LAP_K_COUNT; ++i) g_ev_used[i] = false;
    return LAP_OK;
}

int lap_profile_ordering_ms(uint32_t n_vars, uint32_t n_steps, uint32_t B, const void *ws, size_t ws_bytes,
                            void *hip_stream, float *ms_host)
{
    if (!ms_host) return LAP_E_NULL;
    if (n_vars == 0 || n_steps == 0 || B == 0) return LAP_E_SIZE;
    const int rc = check_ws(const_cast<void *>(ws), ws_bytes, ws_plan(n_vars, n_steps, B));
    if (rc) return rc;
    // same steps as lap_plan_pool takes to its `ticks` region
    Carver c(const_cast<void *>(ws));
    c.take<lap::PlanHeader>(1);
    c.take<uint32_t>((size_t)n_steps + 2);
    c.take<uint32_t>((size_t)n_steps + 2);
    c.take<uint32_t>(B);
    c.take<uint32_t>(B);
    c.take<uint64_t>(B);
    const uint64_t *ticks = c.take<uint64_t>(B);
    std::vector<uint64_t> h(B);
    hipStream_t st = (hipStream_t)hip_stream;
    LAP_HIP(hipMemcpyAsync(h.data(), ticks, (size_t)B * 8, hipMemcpyDeviceToHost, st));
    LAP_HIP(hipStreamSynchronize(st));
    int dev = 0, khz = 0;
    LAP_HIP(hipGetDevice(&dev));
    LAP_HIP(hipDeviceGetAttribute(&khz, hipDeviceAttributeWallClockRate, dev));
    if (khz <= 0) return LAP_E_HIP;
    for (uint32_t b = 0; b < B; ++b) ms_host[b] = (float)((double)h[b] / (double)khz);
    return LAP_OK;
}

int lap_plan_pool_orders(uint32_t n_vars, uint32_t n_steps, uint32_t B, const void *ws, size_t ws_bytes,
                         void *hip_stream, uint32_t *orders)
{
    if (!orders) return LAP_E_NULL;
    if (n_vars == 0 || n_steps == 0 || B == 0) return LAP_E_SIZE;
    const int rc = check_ws(const_cast<void *>(ws), ws_bytes, ws_plan(n_vars, n_steps, B));
    if (rc) return rc;
    // same steps as lap_plan_pool takes to its `perm` region
    Carver c(const_cast<void *>(ws));
    c.take<lap::PlanHeader>(1);
    c.take<uint32_t>((size_t)n_steps + 2);
    c.take<uint32_t>((size_t)n_steps + 2);
    c.take<uint32_t>(B);
    c.take<uint32_t>(B);
    c.take<uint64_t>(B);
    c.take<uint64_t>(B);
    const uint32_t *perm = c.take<uint32_t>((size_t)B * n_vars);
    LAP_HIP(hipMemcpyAsync(orders, perm, (size_t)B * n_vars * 4, hipMemcpyDeviceToDevice, (hipStream_t)hip_stream));
    return LAP_OK;
}

float lap_profile_last_ms(int id)
{
    if (id < 0 || id >= LAP_K_COUNT || !g_ev_used[id]) return -1.0f;
    float ms = -1.0f;
    if (hipEventElapsedTime(&ms, g_ev[id][0], g_ev[id][1]) != hipSuccess) return -1.0f;
    return ms;
}

int lap_load_profile(const lap_trace *tr, uint64_t *load, uint64_t *peak, uint32_t *t_peak, void *ws,
                     size_t ws_bytes, void *hip_stream)
{
    int rc = check_trace_args(tr);
    if (rc) return rc;
    if (!load || !peak || !t_peak) return LAP_E_NULL;
    rc = check_ws(ws, ws_bytes, ws_load(tr->n_steps));
    if (rc) return rc;
    Carver c(ws);
    uint64_t *delta = c.take<uint64_t>((size_t)tr->n_steps + 1);
    return load_profile_impl(tr, load, peak, t_peak, delta, (hipStream_t)hip_stream);
}

int lap_load_profile_static(const lap_trace *tr, uint64_t *load, uint64_t *peak, uint32_t *t_peak, void *hip_stream)
{
    int rc = check_trace_args(tr);
    if (rc) return rc;
    if (!load || !peak || !t_peak) return LAP_E_NULL;
    if (tr->n_steps > STATIC_MAX_STEPS) {
        fprintf(stderr, "liblap: lap_load_profile_static: n_steps = %u exceeds LAP_STATIC_MAX_STEPS = %u; "
                        "use lap_load_profile with a workspace\n", tr->n_steps, STATIC_MAX_STEPS);
        return LAP_E_SIZE;
    }
    void *p = nullptr;
    rc = static_scratch(&p);
    if (rc) return rc;
    // same kernels as lap_load_profile; they clear the part of the array they use first
    return load_profile_impl(tr, load, peak, t_peak, (uint64_t *)p, (hipStream_t)hip_stream);
}

int lap_plan_pool(const lap_trace *tr, const lap_ordering *ords, uint32_t B, uint64_t *best_offsets,
                  uint64_t *best_footprint, uint32_t *best_ordering, uint64_t *footprints, uint64_t *all_offsets,
                  void *ws, size_t ws_bytes, void *hip_stream)
{
    int rc = check_trace_args(tr);
    if (rc) return rc;
    if (!ords || !best_offsets || !best_footprint || !best_ordering) return LAP_E_NULL;
    if (B == 0) return LAP_E_SIZE;
    bool any_explicit = false, any_best = false, any_first = false;
    for (uint32_t b = 0; b < B; ++b) {
        any_explicit |= ords[b].kind == LAP_ORD_EXPLICIT;
        if (ords[b].kind > LAP_ORD_CLASS_SEEDED) return LAP_E_ORDERING;
        if (ords[b].kind == LAP_ORD_EXPLICIT && ords[b].seed == 0) return LAP_E_ORDERING;
        if (ords[b].fit > LAP_FIT_BEST) return LAP_E_ORDERING;
        any_best |= ords[b].fit == LAP_FIT_BEST;
        any_first |= ords[b].fit == LAP_FIT_FIRST;
    }
    const uint32_t n = tr->n_vars, T = tr->n_steps;
    if ((uint64_t)n * lap::PLAN_CL >= (1ull << 32)) return LAP_E_SIZE;
    rc = check_ws(ws, ws_bytes, ws_plan(n, T, B));
    if (rc) return rc;
    hipStream_t st = (hipStream_t)hip_stream;
    const size_t bn = (size_t)B * n;
    Carver c(ws);
    lap::PlanHeader *hdr = c.take<lap::PlanHeader>(1);
    uint32_t *cntd = c.take<uint32_t>((size_t)T + 2);
    uint32_t *lstart = c.take<uint32_t>((size_t)T + 2);
    uint32_t *kinds = c.take<uint32_t>(B);
    uint32_t *fits = c.take<uint32_t>(B);
    uint64_t *seeds = c.take<uint64_t>(B);
    uint64_t *ticks = c.take<uint64_t>(B);          // (lap_profile_ordering_ms finds them by the same steps)
    uint32_t *perm = c.take<uint32_t>(bn);          // (lap_plan_pool_orders likewise)
    uint32_t *tmp = c.take<uint32_t>(bn);
    uint64_t *fps_ws = c.take<uint64_t>(B);
    uint64_t *vrec = c.take<uint64_t>((size_t)n * 2);
    uint64_t *offs_ws = c.take<uint64_t>(bn);
    const size_t dir_cap = seg_dir_cap(T);
    uint32_t *seg_cnt = c.take<uint32_t>(dir_cap + 2);
    uint32_t *seg_lst = c.take<uint32_t>(dir_cap + 2);
    uint32_t *seg_len = c.take<uint32_t>((size_t)B * dir_cap * 2);   // per slot: dir_cap lengths, then dir_cap topmost ranges
    // the placement kernels run one after the other and none needs another's lists: they share one region
    uint64_t *seg_pool = (uint64_t *)((char *)ws + c.used);
    Carver cw((char *)ws + c.used), cf((char *)ws + c.used);
    uint64_t *m_off = cw.take<uint64_t>(bn);
    uint64_t *m_end = cw.take<uint64_t>(bn);
    uint64_t *m_life = cw.take<uint64_t>(bn);
    uint64_t *f_oe = cf.take<uint64_t>(bn);
    uint64_t *f_life = cf.take<uint64_t>(bn);
    uint64_t *f_oe2 = cf.take<uint64_t>(bn);
    uint64_t *f_life2 = cf.take<uint64_t>(bn);
    uint64_t *f_roe = cf.take<uint64_t>((size_t)B * lap::PLAN_REC);
    uint64_t *f_rlife = cf.take<uint64_t>((size_t)B * lap::PLAN_REC);
    uint64_t *f_roe2 = cf.take<uint64_t>((size_t)B * lap::PLAN_REC);
    uint64_t *f_rlife2 = cf.take<uint64_t>((size_t)B * lap::PLAN_REC);
    const uint64_t capL = plan_list_cap(n);
    uint64_t *f_L = cf.take<uint64_t>((size_t)B * capL);
    uint32_t *l_ns = cf.take<uint32_t>((size_t)B * T);
    uint32_t *l_nu = cf.take<uint32_t>((size_t)B * T * 2);     // [B][T] unsorted counts, then [B][T] starts of the top holes

    // The descriptors are split into three arrays; they reach the device inside kernel arguments,
    // so nothing on the host has to outlive this call and nothing waits.
    {
        std::vector<uint32_t> hk(B), hf(B);
        std::vector<uint64_t> hs(B);
        for (uint32_t b = 0; b < B; ++b) { hk[b] = ords[b].kind; hf[b] = ords[b].fit; hs[b] = ords[b].seed; }
        LAP_HIP(lap::launch_put_words(kinds, hk.data(), B, st));
        LAP_HIP(lap::launch_put_words(fits, hf.data(), B, st));
        LAP_HIP(lap::launch_put_words(seeds, hs.data(), (size_t)B * 2, st));
    }

    uint64_t *fps = footprints ? footprints : fps_ws;
    uint64_t *offs = offs_ws;       // in rank order; the outputs are un-permuted from it
    {
        ProfScope p(LAP_K_SORT, st);
        LAP_HIP(lap::launch_sort_perm(n, B, tr->size, tr->alloc, tr->free_, kinds, seeds, perm, tmp, any_explicit, st));
    }
    static_assert(sizeof(lap::PlanHeader) % 8 == 0, "header is cleared in 64-bit words");
    LAP_HIP(lap::launch_fill_u64((uint64_t *)hdr, sizeof(lap::PlanHeader) / 8, 0, st));
    LAP_HIP(lap::launch_fill_u64((uint64_t *)cntd, ((size_t)T + 2) / 2, 0, st));
    LAP_HIP(lap::launch_plan_prep(n, T, B, tr->size, tr->alloc, tr->free_, cntd, lstart, hdr, vrec,
                                  seg_pool_entries(n, B), g_seg_min_vars, st));
    LAP_HIP(lap::launch_seg_prep(n, T, B, tr->alloc, tr->free_, hdr, seg_cnt, seg_lst, (uint32_t)dir_cap,
                                 seg_pool_entries(n, B), st));
    // per-step entry counts start at zero (cleared as 64-bit words, the regions are padded)
    LAP_HIP(lap::launch_fill_u64((uint64_t *)l_ns, ((size_t)B * T + 1) / 2, 0, st));
    LAP_HIP(lap::launch_fill_u64((uint64_t *)l_nu, (size_t)B * T, 0, st));
    {
        int trial_b = -1;                   // the first first-fit ordering shows how the segment lists' searches go
        for (uint32_t b = 0; b < B && trial_b < 0; ++b)
            if (ords[b].fit == LAP_FIT_FIRST) trial_b = (int)b;
        ProfScope p(LAP_K_PLACE, st);
        LAP_HIP(lap::launch_seg_trial(n, T, B, perm, fits, trial_b, (uint32_t)g_seg_trial_percent, hdr, vrec, seg_lst,
                                      seg_pool, seg_len, (uint32_t)dir_cap, offs, fps, ticks, st));
        LAP_HIP(lap::launch_place_fast(n, T, B, tr->size, tr->alloc, tr->free_, perm, fits, any_first, any_best, hdr, vrec,
                                       lstart, f_oe, f_life, f_oe2,
                                       f_life2, f_roe, f_rlife, f_roe2, f_rlife2, f_L, capL, l_ns, l_nu, offs, fps, ticks, st));
        LAP_HIP(lap::launch_place_wide(n, B, tr->size, tr->alloc, tr->free_, perm, fits, hdr, m_off, m_end, m_life, offs,
                                       fps, ticks, st));
        LAP_HIP(lap::launch_place_seg(n, T, B, perm, fits, any_first, hdr, vrec, seg_lst, seg_pool, seg_len,
                                      (uint32_t)dir_cap, offs, fps, ticks, st));
    }
    LAP_HIP(lap::launch_select(n, B, fps, offs, perm, best_footprint, best_ordering, best_offsets, all_offsets, st));
    return LAP_OK;
}

int lap_score_swaps(const lap_trace *tr, double link_GBps, uint64_t min_bytes, const uint64_t *load,
                    uint8_t *candidate, int64_t *doa_ns, double *aoa, uint64_t *wdoa, uint64_t *peak_cut, void *ws,
                    size_t ws_bytes, void *hip_stream)
{
    int rc = check_trace_args(tr);
    if (rc) return rc;
    if (!candidate || !doa_ns || !aoa || !wdoa || !peak_cut) return LAP_E_NULL;
    if (!(link_GBps > 0.0) || !isfinite(link_GBps) || link_GBps * 1000.0 >= 9.0e18) return LAP_E_LINK;
    const long long bpus = llround(link_GBps * 1000.0);
    if (bpus <= 0) return LAP_E_LINK;
    const uint32_t n = tr->n_vars, T = tr->n_steps;
    rc = check_ws(ws, ws_bytes, ws_score(T));
    if (rc) return rc;
    hipStream_t st = (hipStream_t)hip_stream;
    const size_t t1 = (size_t)T + 1;
    Carver c(ws);
    uint64_t *load_ws = c.take<uint64_t>(T);
    uint64_t *delta = c.take<uint64_t>(t1);
    uint64_t *C = c.take<uint64_t>(t1);
    uint64_t *S = c.take<uint64_t>(t1);
    uint64_t *PM = c.take<uint64_t>(t1);
    uint64_t *SM = c.take<uint64_t>(t1);
    const uint32_t levels = table_levels(T);
    uint64_t *table = c.take<uint64_t>((size_t)levels * T);
    uint64_t *peak = c.take<uint64_t>(1);
    uint32_t *t_peak = c.take<uint32_t>(1);

    if (!load) {
        rc = load_profile_impl(tr, load_ws, peak, t_peak, delta, st);
        if (rc) return rc;
        load = load_ws;
    }
    LAP_HIP(lap::launch_swap_prefix(T, load, tr->step_ns, C, S, PM, SM, peak, t_peak, st));
    LAP_HIP(lap::launch_sparse_table(T, load, table, levels, st));
    {
        ProfScope p(LAP_K_SCORE, st);
        LAP_HIP(lap::launch_score(n, T, tr->size, tr->alloc, tr->free_, tr->gap_lo, tr->gap_hi, (uint64_t)bpus,
                                  min_bytes, load, C, S, PM, SM, table, peak, t_peak, candidate, doa_ns, aoa, wdoa,
                                  peak_cut, nullptr, nullptr, st));
    }
    return LAP_OK;
}

int lap_select_swaps(const lap_trace *tr, double link_GBps, uint64_t min_bytes, const uint64_t *load,
                     const uint32_t *score_kinds, uint32_t K, const uint64_t *limits, uint32_t L, uint32_t *order,
                     uint32_t *rank, uint64_t *peaks, uint32_t *n_cand, uint32_t *n_selected, uint64_t *peak_after,
                     uint64_t *load_min, void *ws, size_t ws_bytes, void *hip_stream)
{
    int rc = check_trace_args(tr);
    if (rc) return rc;
    if (!score_kinds || !order || !peaks || !n_cand || !load_min) return LAP_E_NULL;
    if (L && (!limits || !n_selected || !peak_after)) return LAP_E_NULL;
    if (K == 0 || K > SELECT_MAX_KINDS || L > SELECT_MAX_LIMITS) return LAP_E_SIZE;
    for (uint32_t k = 0; k < K; ++k)
        if (score_kinds[k] > LAP_PS_PEAK_CUT) return LAP_E_ORDERING;   // the custom kind is internal
    if (!(link_GBps > 0.0) || !isfinite(link_GBps) || link_GBps * 1000.0 >= 9.0e18) return LAP_E_LINK;
    const long long bpus = llround(link_GBps * 1000.0);
    if (bpus <= 0) return LAP_E_LINK;
    const uint32_t n = tr->n_vars, T = tr->n_steps;
    rc = check_ws(ws, ws_bytes, ws_select(n, T, K));
    if (rc) return rc;
    hipStream_t st = (hipStream_t)hip_stream;
    const size_t t1 = (size_t)T + 1;
    Carver c(ws);
    uint64_t *load_ws = c.take<uint64_t>(T);
    uint64_t *delta = c.take<uint64_t>(t1);
    uint64_t *C = c.take<uint64_t>(t1);
    uint64_t *S = c.take<uint64_t>(t1);
    uint64_t *PM = c.take<uint64_t>(t1);
    uint64_t *SM = c.take<uint64_t>(t1);
    const uint32_t levels = table_levels(T);
    uint64_t *table = c.take<uint64_t>((size_t)levels * T);
    uint64_t *peak = c.take<uint64_t>(1);
    uint32_t *t_peak = c.take<uint32_t>(1);
    uint8_t *cand = c.take<uint8_t>(n);
    int64_t *doa = c.take<int64_t>(n);
    double *aoa = c.take<double>(n);
    uint64_t *wdoa = c.take<uint64_t>(n);
    uint64_t *cut = c.take<uint64_t>(n);
    uint32_t *win_lo = c.take<uint32_t>(n);
    uint32_t *win_hi = c.take<uint32_t>(n);
    uint32_t *cidx = c.take<uint32_t>(n);
    uint32_t *c_ilo = c.take<uint32_t>(n);
    uint32_t *c_ihi = c.take<uint32_t>(n);
    uint64_t *dmin = c.take<uint64_t>(t1);
    uint32_t *nc = c.take<uint32_t>(1);
    uint32_t *d_kinds = c.take<uint32_t>(SELECT_MAX_KINDS);
    uint64_t *d_limits = c.take<uint64_t>(SELECT_MAX_LIMITS);
    uint64_t *r_score = c.take<uint64_t>(0);
    c.used += (size_t)K * up((size_t)n * 8);
    uint32_t *r_var = c.take<uint32_t>(0);
    c.used += (size_t)K * up((size_t)n * 4);
    uint64_t *l_cur = c.take<uint64_t>(0);
    c.used += (size_t)K * up((size_t)T * 8);

    LAP_HIP(lap::launch_put_words(d_kinds, score_kinds, K, st));
    if (L) LAP_HIP(lap::launch_put_words(d_limits, limits, (size_t)L * 2, st));

    if (!load) {
        rc = load_profile_impl(tr, load_ws, peak, t_peak, delta, st);
        if (rc) return rc;
        load = load_ws;
    }
    LAP_HIP(lap::launch_swap_prefix(T, load, tr->step_ns, C, S, PM, SM, peak, t_peak, st));
    LAP_HIP(lap::launch_sparse_table(T, load, table, levels, st));
    LAP_HIP(lap::launch_score(n, T, tr->size, tr->alloc, tr->free_, tr->gap_lo, tr->gap_hi, (uint64_t)bpus, min_bytes,
                              load, C, S, PM, SM, table, peak, t_peak, cand, doa, aoa, wdoa, cut, win_lo, win_hi, st));
    LAP_HIP(lap::launch_fill_u64(dmin, t1, 0, st));
    LAP_HIP(lap::launch_fill_u64((uint64_t *)nc, 1, 0, st));
    lap::SelectArgs a;
    a.n = n; a.T = T; a.K = K; a.L = L;
    a.size = tr->size; a.gap_lo = tr->gap_lo; a.gap_hi = tr->gap_hi; a.alloc = tr->alloc; a.free_ = tr->free_;
    a.load = load; a.cand = cand; a.doa = doa; a.aoa = aoa; a.wdoa = wdoa; a.cut = cut;
    a.win_lo = win_lo; a.win_hi = win_hi; a.nc = nc; a.cidx = cidx; a.c_ilo = c_ilo; a.c_ihi = c_ihi; a.dmin = dmin;
    a.kinds = d_kinds; a.limits = d_limits;
    // per-kind regions are laid out with the kind as the slowest index and a stride of n (or T) elements
    a.r_score = r_score; a.r_var = r_var; a.l_cur = l_cur;
    a.order = order; a.rank = rank; a.peaks = peaks; a.n_cand = n_cand; a.n_selected = n_selected;
    a.peak_after = peak_after; a.load_min = load_min;
    a.custom = nullptr; a.pick_wdoa = nullptr;
    {
        ProfScope p(LAP_K_SELECT, st);
        LAP_HIP(lap::launch_select_swaps(a, true, st));
    }
    return LAP_OK;
}

int lap_evaluate_weights(const lap_trace *tr, double link_GBps, uint64_t min_bytes, const uint64_t *load,
                         const double *weights, uint32_t W, uint64_t limit, uint32_t *order, uint32_t *n_cand,
                         uint32_t *n_selected, uint64_t *peak_after, uint64_t *overhead_ns, uint32_t *forced,
                         uint32_t *best, uint64_t *swdoa, void *ws, size_t ws_bytes, void *hip_stream)
{
    int rc = check_trace_args(tr);
    if (rc) return rc;
    if (!weights || !order || !n_cand || !n_selected || !peak_after || !overhead_ns || !forced || !best || !swdoa)
        return LAP_E_NULL;
    if (W == 0 || W > SELECT_MAX_KINDS) return LAP_E_SIZE;
    for (uint32_t i = 0; i < 4 * W; ++i)
        if (!isfinite(weights[i])) return LAP_E_ORDERING;
    if (!(link_GBps > 0.0) || !isfinite(link_GBps) || link_GBps * 1000.0 >= 9.0e18) return LAP_E_LINK;
    const long long bpus = llround(link_GBps * 1000.0);
    if (bpus <= 0) return LAP_E_LINK;
    const uint32_t n = tr->n_vars, T = tr->n_steps;
    rc = check_ws(ws, ws_bytes, ws_weights(n, T, W));
    if (rc) return rc;
    hipStream_t st = (hipStream_t)hip_stream;
    const size_t t1 = (size_t)T + 1, N = n;
    Carver c(ws);
    uint64_t *load_ws = c.take<uint64_t>(T);
    uint64_t *delta = c.take<uint64_t>(t1);
    uint64_t *C = c.take<uint64_t>(t1);
    uint64_t *S = c.take<uint64_t>(t1);
    uint64_t *PM = c.take<uint64_t>(t1);
    uint64_t *SM = c.take<uint64_t>(t1);
    const uint32_t levels = table_levels(T);
    uint64_t *table = c.take<uint64_t>((size_t)levels * T);
    uint64_t *peak = c.take<uint64_t>(1);
    uint32_t *t_peak = c.take<uint32_t>(1);
    uint8_t *cand = c.take<uint8_t>(n);
    int64_t *doa = c.take<int64_t>(n);
    double *aoa = c.take<double>(n);
    uint64_t *wdoa = c.take<uint64_t>(n);
    uint64_t *cut = c.take<uint64_t>(n);
    uint32_t *win_lo = c.take<uint32_t>(n);
    uint32_t *win_hi = c.take<uint32_t>(n);
    uint32_t *cidx = c.take<uint32_t>(n);
    uint32_t *c_ilo = c.take<uint32_t>(n);
    uint32_t *c_ihi = c.take<uint32_t>(n);
    uint64_t *dmin = c.take<uint64_t>(t1);
    uint32_t *nc = c.take<uint32_t>(1);
    uint32_t *d_kinds = c.take<uint32_t>(SELECT_MAX_KINDS);
    uint64_t *d_limits = c.take<uint64_t>(SELECT_MAX_KINDS);
    double *d_weights = c.take<double>((size_t)SELECT_MAX_KINDS * 4);
    uint64_t *load_min = c.take<uint64_t>(1);
    uint64_t *r_score = c.take<uint64_t>((size_t)W * N);
    uint32_t *r_var = c.take<uint32_t>((size_t)W * N);
    uint64_t *l_cur = c.take<uint64_t>((size_t)W * T);
    uint64_t *peaks = c.take<uint64_t>((size_t)W * (N + 1));
    double *bo = c.take<double>((size_t)W * N);
    uint64_t *need = c.take<uint64_t>(T);
    uint64_t *rel = c.take<uint64_t>(T);
    uint32_t *perm_lo = c.take<uint32_t>(n);
    uint32_t *perm_hi = c.take<uint32_t>(n);
    uint32_t *tmp = c.take<uint32_t>(n);
    uint32_t *s_kind = c.take<uint32_t>(1);
    uint64_t *s_seed = c.take<uint64_t>(1);
    uint32_t *posmap = c.take<uint32_t>((size_t)W * N + 1);
    uint32_t *jobs_lo = c.take<uint32_t>((size_t)W * N);
    uint32_t *jobs_hi = c.take<uint32_t>((size_t)W * N);
    uint32_t *m = c.take<uint32_t>(W);
    uint32_t *kb = c.take<uint32_t>((size_t)W * N);
    uint8_t *out_done = c.take<uint8_t>((size_t)W * N);
    uint64_t *total_ns = c.take<uint64_t>(W);
    uint64_t *peak_res = c.take<uint64_t>(W);

    const std::vector<uint32_t> hk(W, (uint32_t)LAP_PS_CUSTOM);
    if (!load) {
        rc = load_profile_impl(tr, load_ws, peak, t_peak, delta, st);
        if (rc) return rc;
        load = load_ws;
    }
    LAP_HIP(lap::launch_swap_prefix(T, load, tr->step_ns, C, S, PM, SM, peak, t_peak, st));
    LAP_HIP(lap::launch_sparse_table(T, load, table, levels, st));
    LAP_HIP(lap::launch_score(n, T, tr->size, tr->alloc, tr->free_, tr->gap_lo, tr->gap_hi, (uint64_t)bpus, min_bytes,
                              load, C, S, PM, SM, table, peak, t_peak, cand, doa, aoa, wdoa, cut, win_lo, win_hi, st));
    LAP_HIP(lap::launch_fill_u64(dmin, t1, 0, st));
    LAP_HIP(lap::launch_fill_u64((uint64_t *)nc, 1, 0, st));
    LAP_HIP(lap::launch_fill_u64(swdoa, n, 0, st));
    LAP_HIP(lap::launch_fill_u64(d_limits, W, limit, st));
    lap::SelectArgs a;
    a.n = n; a.T = T; a.K = 1; a.L = 0;
    a.size = tr->size; a.gap_lo = tr->gap_lo; a.gap_hi = tr->gap_hi; a.alloc = tr->alloc; a.free_ = tr->free_;
    a.load = load; a.cand = cand; a.doa = doa; a.aoa = aoa; a.wdoa = wdoa; a.cut = cut;
    a.win_lo = win_lo; a.win_hi = win_hi; a.nc = nc; a.cidx = cidx; a.c_ilo = c_ilo; a.c_ihi = c_ihi; a.dmin = dmin;
    a.kinds = d_kinds; a.limits = d_limits;
    a.r_score = r_score; a.r_var = r_var; a.l_cur = l_cur;
    a.order = order; a.rank = nullptr; a.peaks = peaks; a.n_cand = n_cand; a.n_selected = n_selected;
    a.peak_after = peak_after; a.load_min = load_min;
    a.custom = nullptr; a.pick_wdoa = swdoa;
    // 1. the SWDOA walk, once: the value every candidate is picked at
    const uint32_t h_swdoa = LAP_PS_SWDOA;
    LAP_HIP(lap::launch_put_words(d_kinds, &h_swdoa, 1, st));
    LAP_HIP(lap::launch_select_swaps(a, true, st));
    // 2. the aggregated score of every weight vector, 3. its walk down to the limit
    LAP_HIP(lap::launch_put_words(d_weights, weights, (size_t)W * 8, st));
    LAP_HIP(lap::launch_weighted_scores(n, W, d_weights, aoa, doa, wdoa, swdoa, bo, st));
    LAP_HIP(lap::launch_put_words(d_kinds, hk.data(), W, st));
    a.K = W; a.L = 1; a.custom = bo; a.pick_wdoa = nullptr;
    {
        ProfScope p(LAP_K_SELECT, st);
        LAP_HIP(lap::launch_select_swaps(a, false, st));
    }
    // 4. every selection replayed under the limit, 5. the vector that loses the least time
    const uint32_t h_kind = LAP_ORD_ALLOC_ASC;
    LAP_HIP(lap::launch_put_words(s_kind, &h_kind, 1, st));
    LAP_HIP(lap::launch_fill_u64(s_seed, 1, 0, st));
    const uint32_t *step_lo = tr->gap_lo ? tr->gap_lo : tr->alloc;
    const uint32_t *step_hi = tr->gap_hi ? tr->gap_hi : tr->free_;
    LAP_HIP(lap::launch_sort_perm(n, 1, tr->size, step_lo, tr->free_, s_kind, s_seed, perm_lo, tmp, false, st));
    LAP_HIP(lap::launch_sort_perm(n, 1, tr->size, step_hi, tr->free_, s_kind, s_seed, perm_hi, tmp, false, st));
    LAP_HIP(lap::launch_fill_u64((uint64_t *)posmap, ((size_t)W * N + 1) / 2, ~0ull, st));
    LAP_HIP(lap::launch_fill_u64(need, T, 0, st));
    LAP_HIP(lap::launch_fill_u64(rel, T, 0, st));
    LAP_HIP(lap::launch_simulate_swaps(n, T, W, n, tr->size, tr->alloc, tr->free_, step_lo, step_hi,
                                       tr->gap_hi ? 0u : 1u, C, need, rel, order, perm_lo, perm_hi, posmap, jobs_lo,
                                       jobs_hi, m, n_selected, d_limits, kb, out_done, (uint64_t)bpus, total_ns,
                                       overhead_ns, peak_res, forced, st, W, n_cand));
    LAP_HIP(lap::launch_argmin_u64(W, overhead_ns, best, st));
    return LAP_OK;
}

int lap_schedule_swaps(const lap_trace *tr, double link_GBps, const uint64_t *load, const uint32_t *swap_list,
                       uint32_t k, int64_t *out_start, int64_t *out_end, int64_t *in_start, int64_t *in_end,
                       uint64_t *load_sched, uint64_t *peak_sched, uint64_t *late_ns, void *ws, size_t ws_bytes,
                       void *hip_stream)
{
    int rc = check_trace_args(tr);
    if (rc) return rc;
    if (!load_sched || !peak_sched || !late_ns) return LAP_E_NULL;
    if (k && (!swap_list || !out_start || !out_end || !in_start || !in_end)) return LAP_E_NULL;
    if (k > tr->n_vars) return LAP_E_SIZE;
    if (!(link_GBps > 0.0) || !isfinite(link_GBps) || link_GBps * 1000.0 >= 9.0e18) return LAP_E_LINK;
    const long long bpus = llround(link_GBps * 1000.0);
    if (bpus <= 0) return LAP_E_LINK;
    const uint32_t n = tr->n_vars, T = tr->n_steps;
    rc = check_ws(ws, ws_bytes, ws_schedule(n, T));
    if (rc) return rc;
    hipStream_t st = (hipStream_t)hip_stream;
    const size_t t1 = (size_t)T + 1;
    Carver c(ws);
    uint64_t *load_ws = c.take<uint64_t>(T);
    uint64_t *delta = c.take<uint64_t>(t1);
    uint64_t *C = c.take<uint64_t>(t1);
    uint64_t *S = c.take<uint64_t>(t1);
    uint64_t *PM = c.take<uint64_t>(t1);
    uint64_t *SM = c.take<uint64_t>(t1);
    uint64_t *diff = c.take<uint64_t>(t1);
    uint64_t *peak = c.take<uint64_t>(1);
    uint32_t *t_peak = c.take<uint32_t>(1);
    uint32_t *posmap = c.take<uint32_t>(n);
    uint32_t *perm_lo = c.take<uint32_t>(n);
    uint32_t *perm_hi = c.take<uint32_t>(n);
    uint32_t *tmp = c.take<uint32_t>(n);
    uint32_t *kinds = c.take<uint32_t>(1);
    uint64_t *seeds = c.take<uint64_t>(1);

    if (!load) {
        rc = load_profile_impl(tr, load_ws, peak, t_peak, delta, st);
        if (rc) return rc;
        load = load_ws;
    }
    LAP_HIP(lap::launch_swap_prefix(T, load, tr->step_ns, C, S, PM, SM, peak, t_peak, st));
    // all variables by (first access, index) and by (next access, index): the ascending-step sort of
    // the placement orders, fed with the access steps
    const uint32_t h_kind = LAP_ORD_ALLOC_ASC;
    LAP_HIP(lap::launch_put_words(kinds, &h_kind, 1, st));
    LAP_HIP(lap::launch_fill_u64(seeds, 1, 0, st));
    const uint32_t *step_lo = tr->gap_lo ? tr->gap_lo : tr->alloc;
    const uint32_t *step_hi = tr->gap_hi ? tr->gap_hi : tr->free_;
    LAP_HIP(lap::launch_sort_perm(n, 1, tr->size, step_lo, tr->free_, kinds, seeds, perm_lo, tmp, false, st));
    LAP_HIP(lap::launch_sort_perm(n, 1, tr->size, step_hi, tr->free_, kinds, seeds, perm_hi, tmp, false, st));
    LAP_HIP(lap::launch_fill_u64((uint64_t *)posmap, ((size_t)n + 1) / 2, ~0ull, st));
    LAP_HIP(lap::launch_fill_u64(diff, t1, 0, st));
    LAP_HIP(lap::launch_fill_u64(late_ns, 1, 0, st));
    LAP_HIP(lap::launch_schedule_swaps(n, T, k, tr->size, step_lo, step_hi, tr->gap_hi ? 0u : 1u, C, perm_lo, perm_hi,
                                       posmap, swap_list, (uint64_t)bpus, out_start, out_end, in_start, in_end, diff,
                                       late_ns, load, load_sched, peak_sched, st));
    return LAP_OK;
}

int lap_simulate_swaps(const lap_trace *tr, double link_GBps, const uint32_t *swap_list, uint32_t k_max,
                       const uint32_t *prefix_len, const uint64_t *limits, uint32_t Q, uint64_t *total_ns,
                       uint64_t *overhead_ns, uint64_t *peak_resident, uint32_t *forced, void *ws, size_t ws_bytes,
                       void *hip_stream)
{
    int rc = check_trace_args(tr);
    if (rc) return rc;
    if (!prefix_len || !limits || !total_ns || !overhead_ns || !peak_resident || !forced) return LAP_E_NULL;
    if (k_max && !swap_list) return LAP_E_NULL;
    if (Q == 0 || Q > SIM_MAX_RUNS || k_max > tr->n_vars) return LAP_E_SIZE;
    for (uint32_t q = 0; q < Q; ++q)
        if (prefix_len[q] > k_max) return LAP_E_SIZE;
    if (!(link_GBps > 0.0) || !isfinite(link_GBps) || link_GBps * 1000.0 >= 9.0e18) return LAP_E_LINK;
    const long long bpus = llround(link_GBps * 1000.0);
    if (bpus <= 0) return LAP_E_LINK;
    const uint32_t n = tr->n_vars, T = tr->n_steps;
    rc = check_ws(ws, ws_bytes, ws_simulate(n, T, Q));
    if (rc) return rc;
    hipStream_t st = (hipStream_t)hip_stream;
    const size_t t1 = (size_t)T + 1;
    Carver c(ws);
    uint64_t *load_ws = c.take<uint64_t>(T);
    uint64_t *delta = c.take<uint64_t>(t1);
    uint64_t *C = c.take<uint64_t>(t1);
    uint64_t *S = c.take<uint64_t>(t1);
    uint64_t *PM = c.take<uint64_t>(t1);
    uint64_t *SM = c.take<uint64_t>(t1);
    uint64_t *peak = c.take<uint64_t>(1);
    uint32_t *t_peak = c.take<uint32_t>(1);
    uint64_t *need = c.take<uint64_t>(T);
    uint64_t *rel = c.take<uint64_t>(T);
    uint32_t *posmap = c.take<uint32_t>(n);
    uint32_t *perm_lo = c.take<uint32_t>(n);
    uint32_t *perm_hi = c.take<uint32_t>(n);
    uint32_t *tmp = c.take<uint32_t>(n);
    uint32_t *jobs_lo = c.take<uint32_t>(n);
    uint32_t *jobs_hi = c.take<uint32_t>(n);
    uint32_t *kinds = c.take<uint32_t>(1);
    uint64_t *seeds = c.take<uint64_t>(1);
    uint32_t *m = c.take<uint32_t>(1);
    uint32_t *d_prefix = c.take<uint32_t>(SIM_MAX_RUNS);
    uint64_t *d_limits = c.take<uint64_t>(SIM_MAX_RUNS);
    uint32_t *kb = c.take<uint32_t>(0);
    c.used += (size_t)Q * up((size_t)n * 4);
    uint8_t *out_done = c.take<uint8_t>(0);
    c.used += (size_t)Q * up((size_t)n);

    LAP_HIP(lap::launch_put_words(d_prefix, prefix_len, Q, st));
    LAP_HIP(lap::launch_put_words(d_limits, limits, (size_t)Q * 2, st));
    // the step start times come from the same prefix kernel as the scores (it needs a load curve)
    rc = load_profile_impl(tr, load_ws, peak, t_peak, delta, st);
    if (rc) return rc;
    LAP_HIP(lap::launch_swap_prefix(T, load_ws, tr->step_ns, C, S, PM, SM, peak, t_peak, st));
    const uint32_t h_kind = LAP_ORD_ALLOC_ASC;
    LAP_HIP(lap::launch_put_words(kinds, &h_kind, 1, st));
    LAP_HIP(lap::launch_fill_u64(seeds, 1, 0, st));
    const uint32_t *step_lo = tr->gap_lo ? tr->gap_lo : tr->alloc;
    const uint32_t *step_hi = tr->gap_hi ? tr->gap_hi : tr->free_;
    LAP_HIP(lap::launch_sort_perm(n, 1, tr->size, step_lo, tr->free_, kinds, seeds, perm_lo, tmp, false, st));
    LAP_HIP(lap::launch_sort_perm(n, 1, tr->size, step_hi, tr->free_, kinds, seeds, perm_hi, tmp, false, st));
    LAP_HIP(lap::launch_fill_u64((uint64_t *)posmap, ((size_t)n + 1) / 2, ~0ull, st));
    LAP_HIP(lap::launch_sched_mark(n, k_max, swap_list, posmap, st));
    LAP_HIP(lap::launch_fill_u64(need, T, 0, st));
    LAP_HIP(lap::launch_fill_u64(rel, T, 0, st));
    // the per-run regions use a stride of n entries
    LAP_HIP(lap::launch_simulate_swaps(n, T, Q, n, tr->size, tr->alloc, tr->free_, step_lo, step_hi,
                                       tr->gap_hi ? 0u : 1u, C, need, rel, swap_list, perm_lo, perm_hi, posmap,
                                       jobs_lo, jobs_hi, m, d_prefix, d_limits, kb, out_done, (uint64_t)bpus,
                                       total_ns, overhead_ns, peak_resident, forced, st));
    return LAP_OK;
}

int lap_detect_iteration(const uint64_t *tokens, uint32_t n_requests, uint32_t min_period, uint32_t *period,
                         void *ws, size_t ws_bytes, void *hip_stream)
{
    if (!tokens || !period) return LAP_E_NULL;
    if (n_requests == 0 || n_requests == 0xFFFFFFFFu || min_period == 0) return LAP_E_SIZE;
    const int rc = check_ws(ws, ws_bytes, up(((size_t)n_requests + 1) * 8));
    if (rc) return rc;
    LAP_HIP(lap::launch_detect_iteration(tokens, n_requests, min_period, (uint64_t *)ws, period,
                                         (hipStream_t)hip_stream));
    return LAP_OK;
}

int lap_validate_trace(const lap_trace *tr, void *ws, size_t ws_bytes, void *hip_stream)
{
    int rc = check_trace_args(tr);
    if (rc) return rc;
    rc = check_ws(ws, ws_bytes, ws_validate());
    if (rc) return rc;
    hipStream_t st = (hipStream_t)hip_stream;
    uint64_t *out = (uint64_t *)ws;
    LAP_HIP(lap::launch_fill_u64(out, 8, 0, st));
    LAP_HIP(lap::launch_validate(tr->n_vars, tr->n_steps, tr->size, tr->alloc, tr->free_, tr->gap_lo, tr->gap_hi,
                                 tr->step_ns, out, st));
    uint64_t h[8];
    LAP_HIP(hipMemcpyAsync(h, out, sizeof(h), hipMemcpyDeviceToHost, st));
    LAP_HIP(hipStreamSynchronize(st));
    if (h[0]) return LAP_E_TRACE;
    if (h[1]) return LAP_E_RANGE;
    const unsigned __int128 sum = ((unsigned __int128)h[3] << 32) + h[2];
    if (sum >= ((unsigned __int128)1 << 63)) return LAP_E_RANGE;
    if (h[4] > UINT64_MAX / tr->n_steps) return LAP_E_RANGE;
    unsigned __int128 ns = tr->step_ns ? (((unsigned __int128)h[6] << 32) + h[5])
                                       : (unsigned __int128)tr->n_steps * 1000000u;
    if (ns >= ((unsigned __int128)1 << 53)) return LAP_E_RANGE;
    return LAP_OK;
}

}  // extern "C"
