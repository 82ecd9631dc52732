// Host side of the C ABI declared in include/monta.h: argument validation,
// workspace layout, launch shapes, the slice pipeline and event profiling.
// Everything that touches data runs in the kernels of monta_kernels.hpp.
#include "monta.h"

#include <hip/hip_runtime.h>

#include <algorithm>
#include <atomic>
#include <cstdlib>
#include <cmath>
#include <cstring>
#include <mutex>
#include <vector>

#include "monta_kernels.hpp"
#include "monta_planner.hpp"

namespace {

using namespace monta;


thread_local int g_last_hip = 0;
std::atomic<int> g_pipeline_mode{-1};  // -1: chosen from the bytes one slice moves
std::atomic<int> g_plan_mode{-1};      // -1: per-workgroup rebuild when the histogram table is small; 0: always ticketed scan
std::atomic<int> g_cache_policy{-1};   // -1: chosen from the working-set size

// The process-wide switches as one entry point saw them when it was called: every decision of that call, and of
// the internal steps it is made of, uses this snapshot, so a switch flipped by another thread takes effect at
// the next call and never in the middle of one.
struct Modes {
    int pipeline, plan, cache;
};
Modes snapshot_modes() { return {g_pipeline_mode.load(), g_plan_mode.load(), g_cache_policy.load()}; }

#define HIP_TRY(expr)                          \
    do {                                       \
        hipError_t e__ = (expr);               \
        if (e__ != hipSuccess) {               \
            g_last_hip = (int)e__;             \
            (void)hipGetLastError();           \
            return MONTA_ERR_HIP;              \
        }                                      \
    } while (0)

inline int64_t align_up(int64_t v, int64_t a) { return (v + a - 1) / a * a; }

int pow2ceil(int v)
{
    int p = 1;
    while (p < v) p <<= 1;
    return p;
}

constexpr size_t kRouteLdsBudget = 120 * 1024;

struct Geometry {
    Shape s;
    Modes modes;
    int64_t max_rows;
    int64_t row_bytes;
    size_t route_lds;
    int route_threads;   // workgroup size of the route kernel: TB * lanes per token
    int plan_threads;    // workgroup size of the positions kernels: one lane per token
};

// Per-expert capacity: C = min(T, ceil(cf*T*k/E)), cf = 0 meaning "no drop".
int64_t capacity_of(const monta_cfg *c)
{
    if (c->capacity_factor <= 0.f) return c->tokens;
    double v = std::ceil((double)c->capacity_factor * (double)c->tokens * (double)c->top_k / (double)c->experts);
    if (v > (double)c->tokens) return c->tokens;
    return (int64_t)v;
}

// lanes that share one token in the route kernel: each lane should still scan at least 8 experts
int route_lanes_per_token(int TB, int E)
{
    int rl = 1;
    while (rl < 8 && E / (2 * rl) >= 8 && TB * 2 * rl <= 1024) rl *= 2;
    return rl;
}

size_t route_lds_bytes(int TB, int E, int k)
{
    const int NW = TB > kWave ? TB / kWave : 1;
    const int stride = route_row_stride(E, route_lanes_per_token(TB, E));
    size_t b = ((size_t)TB * stride * 4 + (size_t)TB * k * 4 + 7) & ~(size_t)7;    // logits tile, selections
    return b + (size_t)E * NW * 8 + (size_t)TB * k * 8 + (size_t)TB * 8;            // bit masks, weights, denominators
}

int validate(const monta_cfg *c, Geometry *g)
{
    if (!c) return MONTA_ERR_NULL;
    g->modes = snapshot_modes();
    if (c->tokens < 1 || c->hidden < 1 || c->experts < 1 || c->top_k < 1 || c->ep < 1 || c->tp < 1 || c->slices < 1)
        return MONTA_ERR_INVALID;
    if (c->dtype != MONTA_FP32 && c->dtype != MONTA_BF16) return MONTA_ERR_INVALID;
    if (c->renorm != 0 && c->renorm != 1) return MONTA_ERR_INVALID;
    if (c->padded != 0 && c->padded != 1) return MONTA_ERR_INVALID;
    if (c->top_k > c->experts) return MONTA_ERR_INVALID;
    if (c->experts % c->ep != 0) return MONTA_ERR_INVALID;
    if (!(c->capacity_factor >= 0.f) || !std::isfinite(c->capacity_factor)) return MONTA_ERR_INVALID;
    const int64_t U = (int64_t)c->slices * c->tp;
    if (c->tokens % U != 0) return MONTA_ERR_INVALID;
    const int64_t row = (int64_t)c->hidden * (c->dtype == MONTA_FP32 ? 4 : 2);
    if (row % 16 != 0) return MONTA_ERR_INVALID;
    if (c->experts > 256 || c->top_k > 32) return MONTA_ERR_UNSUPPORTED;
    if (c->tokens * (int64_t)c->top_k > 0x7fffffffLL) return MONTA_ERR_UNSUPPORTED;
    if (row / 16 > 0x7fffffffLL || U * c->experts > 0x7fffffffLL) return MONTA_ERR_UNSUPPORTED;

    Shape &s = g->s;
    s.T = (int32_t)c->tokens;
    s.E = c->experts;
    s.k = c->top_k;
    s.ep = c->ep;
    s.tp = c->tp;
    s.S = c->slices;
    s.U = (int32_t)U;
    s.Tu = (int32_t)(c->tokens / U);
    s.C = (int32_t)capacity_of(c);
    s.renorm = c->renorm;
    s.vpr = (int32_t)(row / 16);
    const int lpr_max = kMoverThreads;
    s.lpr = pow2ceil(s.vpr) < lpr_max ? pow2ceil(s.vpr) : lpr_max;
    // route workgroup: as many tokens as fit the LDS budget (gfx950 gives a workgroup up to 160 KiB),
    // at most 256, no more than a unit needs
    int TB = 256;
    while (TB > 32 && (route_lds_bytes(TB, s.E, s.k) > kRouteLdsBudget || TB / 2 >= s.Tu)) TB >>= 1;
    if (route_lds_bytes(TB, s.E, s.k) > kRouteLdsBudget) return MONTA_ERR_UNSUPPORTED;
    s.TB = TB;
    s.bpu = (s.Tu + TB - 1) / TB;
    const int64_t nb = (int64_t)s.bpu * U;
    if (nb * s.E > 0x7fffffffLL) return MONTA_ERR_UNSUPPORTED;
    s.num_blocks = (int32_t)nb;
    // the per-workgroup rebuild of the scans reads num_blocks*E counters in every workgroup
    s.fast_plan = (g->modes.plan != 0 && nb * s.E <= 65536) ? 1 : 0;
    g->route_lds = route_lds_bytes(TB, s.E, s.k);
    g->plan_threads = TB < kWave ? kWave : TB;
    const int rl = route_lanes_per_token(TB, s.E);
    s.rl = rl;
    g->route_threads = TB * rl < kWave ? kWave : TB * rl;
    const int64_t tk = c->tokens * (int64_t)c->top_k, ec = (int64_t)c->experts * s.C;
    if (c->padded && ec > 0x7fffffffLL) return MONTA_ERR_UNSUPPORTED;
    s.padded = c->padded;
    g->max_rows = c->padded ? ec : (tk < ec ? tk : ec);
    s.max_rows = (int32_t)g->max_rows;
    {
        // Measured on MI355X (256 MB memory-side cache): a producer's cacheable stores pay when the
        // consumer kernel reads them back soon; beyond the cache everything but the pack stores streams.
        const int pol = g->modes.cache;
        const int64_t touched = (2 * c->tokens + 2 * g->max_rows) * row;   // x + out + STAGE + FINAL
        if (pol >= 0) s.cache = pol;
        else if (touched <= (512ll << 20)) s.cache = NT_REG_LD | NT_COMB_LD | NT_COMB_ST;
        else if (touched <= (1024ll << 20)) s.cache = NT_REG_LD | NT_REG_ST | NT_COMB_LD | NT_COMB_ST;
        else s.cache = NT_PACK_LD | NT_REG_LD | NT_REG_ST | NT_COMB_LD | NT_COMB_ST;
    }
    g->row_bytes = row;
    return MONTA_OK;
}

void fill_layout(const Geometry &g, monta_ws_layout *L)
{
    const Shape &s = g.s;
    int64_t off = 0;
    auto take = [&](int64_t ints) {
        int64_t o = off;
        off = align_up(off + ints * 4, 256);
        return o;
    };
    L->max_rows = g.max_rows;
    L->capacity = s.C;
    L->units = s.U;
    L->tokens_per_unit = s.Tu;
    L->block_tokens = s.TB;
    L->num_blocks = s.num_blocks;
    L->off_meta = take(META_SLOTS);
    L->off_counts = take(s.E);
    L->off_kept = take(s.E);
    L->off_offsets = take(s.E + 1);
    L->off_n = take((int64_t)s.U * s.E);
    L->off_stage_off = take((int64_t)s.U * s.E);
    L->off_unit_base = take((int64_t)s.U * s.E);
    L->off_send_rows = take((int64_t)s.U * s.ep);
    L->off_unit_rows = take((int64_t)s.U + 1);
    L->off_pos_final = take((int64_t)s.T * s.k);
    L->off_pos_stage = take((int64_t)s.T * s.k);
    L->off_row_map = take(g.max_rows);
    L->off_block_counts = take((int64_t)s.num_blocks * s.E);
    L->off_block_base = take((int64_t)s.num_blocks * s.E);
    L->off_local_rank = take((int64_t)s.T * s.k);
    L->off_kept_prefix = take(s.E + 1);
    L->ws_bytes = off;
}

PlanPtrs plan_ptrs(const Geometry &g, const void *ws)
{
    monta_ws_layout L;
    fill_layout(g, &L);
    char *b = const_cast<char *>(static_cast<const char *>(ws));
    auto at = [&](int64_t o) { return reinterpret_cast<int32_t *>(b + o); };
    PlanPtrs p;
    p.meta = at(L.off_meta);
    p.counts = at(L.off_counts);
    p.kept = at(L.off_kept);
    p.offsets = at(L.off_offsets);
    p.n = at(L.off_n);
    p.stage_off = at(L.off_stage_off);
    p.unit_base = at(L.off_unit_base);
    p.send_rows = at(L.off_send_rows);
    p.unit_rows = at(L.off_unit_rows);
    p.pos_final = at(L.off_pos_final);
    p.pos_stage = at(L.off_pos_stage);
    p.row_map = at(L.off_row_map);
    p.block_counts = at(L.off_block_counts);
    p.block_base = at(L.off_block_base);
    p.local_rank = at(L.off_local_rank);
    p.kept_prefix = at(L.off_kept_prefix);
    return p;
}

inline bool misaligned(const void *p, uintptr_t a) { return (reinterpret_cast<uintptr_t>(p) & (a - 1)) != 0; }

// ------------------------------------------------------------- profiling
//
// One event is recorded after every kernel launch, on the launching stream.  A
// kernel's duration is the time from the previous such event on the same stream
// (the end of the previous kernel) to its own event, so consecutive kernels are
// timed back to back without a second marker between them; the first kernel of a
// chain, or one that follows a cross-stream wait, gets a start event of its own.

struct ProfRec {
    int kid;
    hipEvent_t a, b;
};
std::mutex g_prof_mu;
std::atomic<int> g_prof_on{0};
std::vector<ProfRec> g_prof_recs;
std::vector<hipEvent_t> g_prof_events;                        // everything created, destroyed when drained
std::vector<std::pair<hipStream_t, hipEvent_t>> g_prof_last;  // last end event per stream
double g_prof_ms[MONTA_K_COUNT] = {0};
int64_t g_prof_n[MONTA_K_COUNT] = {0};

void prof_break_chain(hipStream_t st)
{
    if (!g_prof_on.load()) return;
    std::lock_guard<std::mutex> lk(g_prof_mu);
    for (auto &pr : g_prof_last)
        if (pr.first == st) pr.second = nullptr;
}

struct ProfScope {
    hipStream_t st;
    int kid;
    hipEvent_t a = nullptr;
    bool on;
    ProfScope(int kid_, hipStream_t st_) : st(st_), kid(kid_), on(g_prof_on.load() != 0)
    {
        if (!on) return;
        std::lock_guard<std::mutex> lk(g_prof_mu);
        for (auto &pr : g_prof_last)
            if (pr.first == st) a = pr.second;
        if (!a) {
            if (hipEventCreate(&a) != hipSuccess) {
                on = false;
                a = nullptr;
                return;
            }
            g_prof_events.push_back(a);
            (void)hipEventRecord(a, st);
        }
    }
    ~ProfScope()
    {
        if (!on) return;
        hipEvent_t b = nullptr;
        if (hipEventCreate(&b) != hipSuccess) return;
        (void)hipEventRecord(b, st);
        std::lock_guard<std::mutex> lk(g_prof_mu);
        g_prof_events.push_back(b);
        g_prof_recs.push_back({kid, a, b});
        bool found = false;
        for (auto &pr : g_prof_last)
            if (pr.first == st) {
                pr.second = b;
                found = true;
            }
        if (!found) g_prof_last.push_back({st, b});
    }
};

int prof_drain()
{
    std::lock_guard<std::mutex> lk(g_prof_mu);
    int rc = MONTA_OK;
    for (auto &r : g_prof_recs) {
        float ms = 0.f;
        hipError_t e = hipEventSynchronize(r.b);
        if (e == hipSuccess) e = hipEventElapsedTime(&ms, r.a, r.b);
        if (e == hipSuccess) {
            g_prof_ms[r.kid] += ms;
            g_prof_n[r.kid] += 1;
        } else {
            g_last_hip = (int)e;
            rc = MONTA_ERR_HIP;
        }
    }
    for (hipEvent_t ev : g_prof_events) (void)hipEventDestroy(ev);
    g_prof_events.clear();
    g_prof_recs.clear();
    g_prof_last.clear();
    return rc;
}

// ------------------------------------------------- side stream for mode 0

struct DevState {
    std::mutex mu;              // held while a call enqueues work that uses the side stream or the events
    hipStream_t side = nullptr;
    std::vector<hipEvent_t> ev;
    hipEvent_t done = nullptr;
};
std::mutex g_dev_mu;
DevState g_dev[64];

int dev_state(int nslices, DevState **out)
{
    int dev = 0;
    HIP_TRY(hipGetDevice(&dev));
    if (dev < 0 || dev >= 64) return MONTA_ERR_UNSUPPORTED;
    std::lock_guard<std::mutex> lk(g_dev_mu);
    DevState &d = g_dev[dev];
    if (!d.side) HIP_TRY(hipStreamCreateWithFlags(&d.side, hipStreamNonBlocking));
    if (!d.done) HIP_TRY(hipEventCreateWithFlags(&d.done, hipEventDisableTiming));
    while ((int)d.ev.size() < nslices) {
        hipEvent_t e;
        HIP_TRY(hipEventCreateWithFlags(&e, hipEventDisableTiming));
        d.ev.push_back(e);
    }
    *out = &d;
    return MONTA_OK;
}

// ------------------------------------------------------------ launch shapes

constexpr int kMaxMoverGrid = 1 << 16;
constexpr int kResidentMoverWgs = 2048;         // mover workgroups the chip holds at once: 256 CUs x 8
constexpr int64_t kGroupBytes = 256ll << 20;   // a launch group's share of STAGE: the size of the memory-side cache

int mover_grid(const Shape &s, int64_t rows)
{
    const int rows_per_wg = kMoverThreads / s.lpr;
    int64_t g = (rows + rows_per_wg - 1) / rows_per_wg;
    if (g < 1) g = 1;
    if (g > kMaxMoverGrid) g = kMaxMoverGrid;
    return (int)g;
}

// The row count of a slice is only known on the device; the grid is sized from the host-side bound.
// With capacity drops most of those workgroups would find nothing to do, and an idle workgroup still
// costs dispatch time (measured on the largest workload, 55 % of the pairs dropped: a cap of 65536 workgroups
// makes the step 4 % longer than 32768, 16384 is another 0.5 % shorter, 8192 is slower again), so the grid stops
// at 16384 workgroups and the kernel strides over the rest.
constexpr int kMaxRegatherGrid = 16384;
int regather_grid(const Shape &s, int64_t rows_bound)
{
    const int g = mover_grid(s, rows_bound);
    return g < kMaxRegatherGrid ? g : kMaxRegatherGrid;
}

int64_t slice_rows_bound(const Geometry &g, int nslices_covered)
{
    int64_t r = (int64_t)g.s.tp * g.s.Tu * nslices_covered * g.s.k;
    return r < g.max_rows ? r : g.max_rows;
}

// The launch helpers below take a range of slices [j0, j1).
int launch_pack(const Geometry &g, const PlanPtrs &p, const void *x, void *stage, int j0, int j1, hipStream_t st)
{
    const Shape &s = g.s;
    const int per_slice = s.tp * s.Tu;
    const int t0 = j0 * per_slice, nt = (j1 - j0) * per_slice;
    ProfScope ps(MONTA_K_PACK, st);
    hipLaunchKernelGGL(pack_kernel, dim3(mover_grid(s, nt)), dim3(kMoverThreads), 0, st,
                       static_cast<const u32x4 *>(x), static_cast<u32x4 *>(stage), p, s, t0, nt);
    HIP_TRY(hipGetLastError());
    return MONTA_OK;
}

int launch_regather(const Geometry &g, const PlanPtrs &p, const void *stage, void *fin, int j0, int j1, hipStream_t st)
{
    const Shape &s = g.s;
    const int64_t bound = slice_rows_bound(g, j1 - j0);
    ProfScope ps(MONTA_K_REGATHER, st);
    hipLaunchKernelGGL(regather_kernel, dim3(regather_grid(s, bound)), dim3(kMoverThreads), 0, st,
                       static_cast<const u32x4 *>(stage), static_cast<u32x4 *>(fin), p, s, j0 * s.tp, j1 * s.tp);
    HIP_TRY(hipGetLastError());
    return MONTA_OK;
}

// packs slices [pj0, pj1) and regathers slices [rj0, rj1) in disjoint workgroups of one grid
int launch_pack_regather(const Geometry &g, const PlanPtrs &p, const void *x, void *stage, void *fin, int pj0, int pj1,
                         int rj0, int rj1, hipStream_t st)
{
    const Shape &s = g.s;
    const int per_slice = s.tp * s.Tu;
    const int n_pack = mover_grid(s, (pj1 - pj0) * per_slice);
    const int n_reg = regather_grid(s, slice_rows_bound(g, rj1 - rj0));
    ProfScope ps(MONTA_K_PACK_REGATHER, st);
    hipLaunchKernelGGL(pack_regather_kernel, dim3(n_pack + n_reg), dim3(kMoverThreads), 0, st,
                       static_cast<const u32x4 *>(x), static_cast<u32x4 *>(stage), static_cast<u32x4 *>(fin), p, s,
                       pj0 * per_slice, (pj1 - pj0) * per_slice, rj0 * s.tp, rj1 * s.tp, n_pack);
    HIP_TRY(hipGetLastError());
    return MONTA_OK;
}

int check_act_ptrs(const void *a, const void *b)
{
    if (!a || !b) return MONTA_ERR_NULL;
    if (misaligned(a, 16) || misaligned(b, 16)) return MONTA_ERR_ALIGN;
    return MONTA_OK;
}

// Dynamic LDS above the default limit has to be asked for once per kernel and device.
struct LdsOptIn {
    std::atomic<int> done[64];
};

int opt_in_lds(const void *kernel, int bytes, LdsOptIn &state)
{
    int dev = 0;
    HIP_TRY(hipGetDevice(&dev));
    if (dev < 0 || dev >= 64) return MONTA_ERR_UNSUPPORTED;
    if (!state.done[dev].load()) {
        HIP_TRY(hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize, bytes));
        state.done[dev].store(1);
    }
    return MONTA_OK;
}

template <int MT, int NT, int KS, bool DEEP, bool SPLIT = false>
int launch_gate(const u32x4 *x, const u32x4 *w, float *logits, int64_t T, int H, int E, hipStream_t st)
{
    using G = GateTile<MT, NT, KS>;
    static LdsOptIn lds_opt_in;
    if (int rc = opt_in_lds(reinterpret_cast<const void *>(gate_bf16_kernel<MT, NT, KS, DEEP, SPLIT>),
                            (int)G::lds_bytes(32 * NT, !SPLIT), lds_opt_in))
        return rc;
    const unsigned grid = (unsigned)((T + G::kTokens - 1) / G::kTokens);
    hipLaunchKernelGGL((gate_bf16_kernel<MT, NT, KS, DEEP, SPLIT>), dim3(grid), dim3(kGateThreads), G::lds_bytes(E, !SPLIT), st, x, w, logits,
                       T, H, E);
    return MONTA_OK;
}

template <int NCH, int THREADS, int MAXCHUNK>
int launch_gate_small(const u32x4 *x, const u32x4 *w, float *logits, int64_t T, int H, int E, int wgs_per_cu,
                      hipStream_t st)
{
    static LdsOptIn lds_opt_in;
    if (int rc = opt_in_lds(reinterpret_cast<const void *>(gate_small_kernel<NCH, THREADS, MAXCHUNK>),
                            (int)gate_small_lds_bytes(MAXCHUNK, THREADS), lds_opt_in))
        return rc;
    static std::atomic<int> cus{0};
    if (!cus.load()) {
        int dev = 0, n = 0;
        HIP_TRY(hipGetDevice(&dev));
        HIP_TRY(hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev));
        cus.store(n > 0 ? n : 256);
    }
    const int64_t ngroups = (T + kGateSmallTokens - 1) / kGateSmallTokens;
    const int64_t resident = (int64_t)wgs_per_cu * cus.load();
    const unsigned grid = (unsigned)(ngroups < resident ? ngroups : resident);
    hipLaunchKernelGGL((gate_small_kernel<NCH, THREADS, MAXCHUNK>), dim3(grid), dim3(THREADS),
                       gate_small_lds_bytes(H / NCH, THREADS), st, x, w, logits, T, H, E, ngroups);
    return MONTA_OK;
}

// The whole-row kernel for at most 8 experts; returns 1 if the shape does not fit it.  Measured on MI355X: tiles
// of 8 rows x 4 KiB serve rows of up to 8 KiB best (a workgroup then sees more, smaller tiles and starts
// sooner), tiles of 8 rows x 8 KiB longer rows; more than one workgroup per CU only repeats the weight set-up.
int launch_gate_small_any(const u32x4 *x, const u32x4 *w, float *logits, int64_t T, int H, int E, hipStream_t st)
{
    if (E > kGateSmallExperts) return 1;
    if (H <= 2048 && H % 64 == 0) return launch_gate_small<1, 512, 2048>(x, w, logits, T, H, E, 1, st);
    if (H <= 4096 && H % 128 == 0) return launch_gate_small<2, 512, 2048>(x, w, logits, T, H, E, 1, st);
    if (H <= 4096 && H % 64 == 0) return launch_gate_small<1, 512, 4096>(x, w, logits, T, H, E, 1, st);
    if (H <= 8192 && H % 128 == 0) return launch_gate_small<2, 512, 4096>(x, w, logits, T, H, E, 1, st);
    return 1;
}

template <bool RAGGED_LAST>
int launch_expert_dtl_t(const void *x_final, const void *w_exp, void *y, const ExpertArgs &a, unsigned grid, hipStream_t st)
{
    static LdsOptIn lds_opt_in;
    if (int rc = opt_in_lds(reinterpret_cast<const void *>(expert_dtl_kernel<RAGGED_LAST>), kDtlLdsBytes, lds_opt_in)) return rc;
    hipLaunchKernelGGL(expert_dtl_kernel<RAGGED_LAST>, dim3(grid), dim3(kDtlThreads), kDtlLdsBytes, st,
                       static_cast<const u32x4 *>(x_final), static_cast<const u32x4 *>(w_exp),
                       static_cast<unsigned short *>(y), a);
    return MONTA_OK;
}

int launch_expert_dtl(const void *x_final, const void *w_exp, void *y, ExpertArgs a, int64_t rows_bound, hipStream_t st)
{
    const int64_t row_tiles = (rows_bound + kDtlBM - 1) / kDtlBM + a.E;      // each expert may end in a ragged tile
    const int64_t nct = (a.N + kDtlBN - 1) / kDtlBN;
    // whole blocks of 256 workgroups: the kernel hands out tile numbers in such blocks, 32 per XCD
    const int64_t grid = (row_tiles * nct + 32 * kXcds - 1) / (32 * kXcds) * (32 * kXcds);
    if (grid > 0x7fffffff) return MONTA_ERR_UNSUPPORTED;
    a.reserved = 0;
    // The segments' ragged last tiles go to the end of the numbering (and skip their empty blocks) only when there
    // are few of them, at most one round of 256 workgroups: measured on MI355X, 2-2.5 % faster with 8 and with 2
    // experts, 2.4 % slower with 64 experts of 28 column tiles, whose ragged tiles then lose their panel's L2 reuse.
    if ((int64_t)a.E * nct <= 256) return launch_expert_dtl_t<true>(x_final, w_exp, y, a, (unsigned)grid, st);
    return launch_expert_dtl_t<false>(x_final, w_exp, y, a, (unsigned)grid, st);
}

template <int BM, int BN, int WM, int WN>
int launch_expert(const void *x_final, const void *w_exp, void *y, ExpertArgs a, int64_t rows_bound, hipStream_t st)
{
    using G = ExpertTile<BM, BN, WM, WN>;
    static LdsOptIn lds_opt_in;
    if (int rc = opt_in_lds(reinterpret_cast<const void *>(expert_bf16_kernel<BM, BN, WM, WN>), G::kLdsBytes, lds_opt_in))
        return rc;
    const int64_t row_tiles = (rows_bound + BM - 1) / BM + a.E;      // each expert may end in a ragged tile
    const int64_t nct = (a.N + BN - 1) / BN;
    constexpr int64_t block = 32 * G::kWgsPerCu * kXcds;            // the kernel numbers its tiles in such blocks
    const int64_t grid8 = (row_tiles * nct + block - 1) / block * block;
    if (grid8 > 0x7fffffff) return MONTA_ERR_UNSUPPORTED;
    a.reserved = 0;
    hipLaunchKernelGGL((expert_bf16_kernel<BM, BN, WM, WN>), dim3((unsigned)grid8), dim3(G::kThreads), G::kLdsBytes, st,
                       static_cast<const u32x4 *>(x_final), static_cast<const u32x4 *>(w_exp),
                       static_cast<unsigned short *>(y), a);
    return MONTA_OK;
}

int launch_route(const Geometry &g, const PlanPtrs &p, const float *logits, int32_t *topk_idx, float *gates,
                 hipStream_t st)
{
    static LdsOptIn lds_opt_in;
    if (g.route_lds > 48 * 1024)
        if (int rc = opt_in_lds(reinterpret_cast<const void *>(route_plan_kernel), (int)kRouteLdsBudget, lds_opt_in)) return rc;
    ProfScope ps(MONTA_K_ROUTE, st);
    hipLaunchKernelGGL(route_plan_kernel, dim3(g.s.num_blocks), dim3(g.route_threads), g.route_lds, st, logits,
                       topk_idx, gates, p, g.s);
    HIP_TRY(hipGetLastError());
    return MONTA_OK;
}

int check_ws(const void *ws)
{
    if (!ws) return MONTA_ERR_NULL;
    if (misaligned(ws, 16)) return MONTA_ERR_ALIGN;
    return MONTA_OK;
}

int check_route_ptrs(const float *logits, const int32_t *topk_idx, const float *gates, const void *ws)
{
    if (!logits || !topk_idx || !gates) return MONTA_ERR_NULL;
    if (misaligned(logits, 4) || misaligned(topk_idx, 4) || misaligned(gates, 4)) return MONTA_ERR_ALIGN;
    return check_ws(ws);
}

int check_expert_args(const monta_cfg *cfg, const Geometry &g, const void *x_final, const void *w_exp, int32_t out_features,
                      const void *y, const void *ws, int slice)
{
    if (!x_final || !w_exp || !y || !ws) return MONTA_ERR_NULL;
    if (misaligned(x_final, 16) || misaligned(w_exp, 16) || misaligned(y, 16) || misaligned(ws, 16)) return MONTA_ERR_ALIGN;
    const int bpe = cfg->dtype == MONTA_BF16 ? 2 : 4;
    if (out_features < 1 || ((int64_t)out_features * bpe) % 16 != 0) return MONTA_ERR_INVALID;
    if (slice < -1 || slice >= g.s.S) return MONTA_ERR_INVALID;
    if (x_final == y) return MONTA_ERR_INVALID;
    return MONTA_OK;
}

int launch_expert_layer(const monta_cfg *cfg, const Geometry &g, const void *x_final, const void *w_exp, int32_t out_features,
                        void *y, const void *ws, int slice, hipStream_t st)
{
    const Shape &s = g.s;
    int rc = MONTA_OK;
    PlanPtrs p = plan_ptrs(g, const_cast<void *>(ws));
    ExpertArgs a;
    a.E = s.E;
    a.H = cfg->hidden;
    a.N = out_features;
    a.max_rows = s.max_rows;
    // rows of expert e: its whole kept segment [offsets[e], offsets[e] + kept[e]), or the part of it filled by the
    // slice's units, which starts at unit_base[first unit of the slice][e] and ends where the next slice's starts
    a.lo = slice < 0 ? p.offsets : p.unit_base + (int64_t)slice * s.tp * s.E;
    if (slice >= 0 && slice + 1 < s.S) {
        a.hi_base = p.unit_base + (int64_t)(slice + 1) * s.tp * s.E;
        a.hi_len = nullptr;
    } else {
        a.hi_base = p.offsets;
        a.hi_len = p.kept;
    }
    // worst case of the rows in play: every pair of the slice's tokens kept
    int64_t rows_bound = slice < 0 ? (int64_t)s.max_rows : std::min<int64_t>(s.max_rows, (int64_t)(s.T / s.S) * s.k);
    ProfScope ps(MONTA_K_EXPERT, st);
    if (cfg->dtype == MONTA_BF16) {
        // whole 64-element steps and segments long enough for 256-row tiles: the direct-to-LDS kernel
        if (cfg->hidden % 64 == 0 && rows_bound / s.E >= 256)
            rc = launch_expert_dtl(x_final, w_exp, y, a, rows_bound, st);
        else
            rc = launch_expert<128, 256, 2, 2>(x_final, w_exp, y, a, rows_bound, st);
        if (rc) return rc;
    } else {
        a.reserved = 0;
        const int64_t blocks = ((int64_t)s.max_rows * out_features + 255) / 256;
        if (blocks > 0x7fffffff) return MONTA_ERR_UNSUPPORTED;
        hipLaunchKernelGGL(expert_f32_kernel, dim3((unsigned)blocks), dim3(256), 0, st, static_cast<const float *>(x_final),
                           static_cast<const float *>(w_exp), static_cast<float *>(y), a);
    }
    HIP_TRY(hipGetLastError());
    return MONTA_OK;
}

// How one call runs the slice pipeline: the realisation (0, 1 or 2) and how many consecutive slices one launch
// covers.  An explicit mode keeps one slice per launch.  The default (-1) chooses from the sizes, as the paper's
// planner chooses its chunk count from the traffic (section "Network-traffic-aware"): measured on MI355X,
//  - a launch boundary costs a few microseconds of idle memory system, so slices that move only tens of
//    megabytes are grouped until a launch's share of STAGE reaches 256 MiB (the size of the memory-side cache:
//    what the pack writes is still there when the regather reads it); a problem that fits one group runs as
//    plan + pack of everything, then one regather;
//  - co-scheduling pack(j) with regather(j-1) in one grid saves a boundary per slice, which decides it while
//    a group's copies take a few tens of microseconds; once they take hundreds, two plain kernels run faster
//    than the mixed grid (the regather alone reaches 6.6-7.0 TB/s, the mixed grid 6.2-6.7).
struct PipePlan {
    int mode;
    int first;      // slices in the first launch group
    int spg;        // slices in every later group
};

// Can the kernel that finishes the plan also pack (plan_pack_kernel)?  It needs a histogram table small enough to
// rebuild in every pack workgroup and token groups that never straddle two route workgroups.
bool plan_pack_shape_ok(const Geometry &g)
{
    const Shape &s = g.s;
    const int rows_per_wg = kMoverThreads / s.lpr;
    return s.fast_plan && (int64_t)s.num_blocks * s.E <= 2048 && s.Tu % s.TB == 0 && rows_per_wg <= s.TB &&
           kMoverThreads >= s.TB;
}

PipePlan pipeline_plan(const Geometry &g)
{
    if (g.modes.pipeline >= 0) return {g.modes.pipeline, 1, 1};
    const int S = g.s.S;
    const int64_t slice_bytes = slice_rows_bound(g, 1) * g.row_bytes;      // what one slice may put into STAGE
    if (slice_bytes >= kGroupBytes) return {2, 1, 1};
    int spg = (int)(kGroupBytes / slice_bytes);
    if (spg > S) spg = S;
    int groups = (S + spg - 1) / spg;
    spg = (S + groups - 1) / groups;                                       // even groups
    if (groups > 1) return {spg * slice_bytes >= kGroupBytes * 3 / 4 ? 2 : 1, spg, spg};
    // Everything fits one group.  The pack workgroups of the fused plan-and-pack kernel each rebuild the plan's
    // scans before their first store; with one round of them resident on the chip that hides behind the row
    // reads, with several rounds it is paid every round (measured: 8192 of them pack 192 MiB at 5.0 TB/s, the
    // plain pack at 6.3).  So the first launch takes about one round of workgroups (whole slices), the rest
    // of the slices form the second group: plan + pack(first), pack(rest) with regather(first), regather(rest).
    if (!plan_pack_shape_ok(g) || S == 1) return {1, S, S};
    const int64_t round_tokens = (int64_t)kResidentMoverWgs * (kMoverThreads / g.s.lpr);
    int first = (int)(round_tokens / ((int64_t)g.s.tp * g.s.Tu));
    if (first < 1) first = 1;
    if (first >= S) first = S - 1;
    return {1, first, S - first};
}

int route_impl(const Geometry &g, const float *logits, int32_t *topk_idx, float *gates, void *ws, hipStream_t st)
{
    const Shape &s = g.s;
    PlanPtrs p = plan_ptrs(g, ws);
    if (int rc = launch_route(g, p, logits, topk_idx, gates, st)) return rc;
    ProfScope ps(MONTA_K_POSITIONS, st);
    if (s.fast_plan)
        hipLaunchKernelGGL(plan_positions_kernel, dim3(s.num_blocks), dim3(g.plan_threads), 0, st, topk_idx, p, s);
    else
        hipLaunchKernelGGL(positions_kernel, dim3((s.T + 255) / 256), dim3(256), 0, st, topk_idx, p, s);
    HIP_TRY(hipGetLastError());
    return MONTA_OK;
}

// the pipeline from group `first` on (group 0 may have been packed already by the kernel that finishes the plan)
int pipeline_impl(const Geometry &g, const PipePlan &pp, const void *x, void *stage, void *final_, const void *ws,
                  bool group0_packed, hipStream_t st)
{
    int rc = MONTA_OK;
    const PlanPtrs p = plan_ptrs(g, ws);
    const int S = g.s.S;
    const int first = pp.first < S ? pp.first : S, spg = pp.spg;
    auto lo = [&](int gi) { return gi == 0 ? 0 : first + (gi - 1) * spg; };
    auto hi = [&](int gi) { const int h = first + gi * spg; return h < S ? h : S; };
    const int G = 1 + (S - first + spg - 1) / spg;
    if (pp.mode == 2) {
        for (int gi = 0; gi < G; ++gi) {
            if (!(gi == 0 && group0_packed))
                if ((rc = launch_pack(g, p, x, stage, lo(gi), hi(gi), st))) return rc;
            if ((rc = launch_regather(g, p, stage, final_, lo(gi), hi(gi), st))) return rc;
        }
        return MONTA_OK;
    }
    if (pp.mode == 1) {
        if (!group0_packed)
            if ((rc = launch_pack(g, p, x, stage, lo(0), hi(0), st))) return rc;
        for (int gi = 1; gi < G; ++gi)
            if ((rc = launch_pack_regather(g, p, x, stage, final_, lo(gi), hi(gi), lo(gi - 1), hi(gi - 1), st))) return rc;
        return launch_regather(g, p, stage, final_, lo(G - 1), hi(G - 1), st);
    }
    // mode 0: packs on the caller's stream, regathers on the side stream, one event per slice.  The side stream
    // and its events are shared by every caller on this device: the whole enqueue holds the device's lock, so
    // that each wait pairs with the record made just before it (a wait refers to the event's latest record at
    // the time the wait is enqueued; what another call records later does not change it).
    DevState *d = nullptr;
    if ((rc = dev_state(G, &d))) return rc;
    std::lock_guard<std::mutex> lk(d->mu);
    for (int gi = 0; gi < G; ++gi) {
        if (!(gi == 0 && group0_packed))
            if ((rc = launch_pack(g, p, x, stage, lo(gi), hi(gi), st))) return rc;
        HIP_TRY(hipEventRecord(d->ev[gi], st));
        HIP_TRY(hipStreamWaitEvent(d->side, d->ev[gi], 0));
        prof_break_chain(d->side);
        if ((rc = launch_regather(g, p, stage, final_, lo(gi), hi(gi), d->side))) return rc;
    }
    HIP_TRY(hipEventRecord(d->done, d->side));
    HIP_TRY(hipStreamWaitEvent(st, d->done, 0));
    prof_break_chain(st);
    return MONTA_OK;
}

int dispatch_regather_impl(const Geometry &g, const void *x, void *stage, void *final_, const void *ws, hipStream_t st)
{
    return pipeline_impl(g, pipeline_plan(g), x, stage, final_, ws, false, st);
}

// Does monta_route_dispatch_regather finish the plan and pack the first launch group in one grid?  An explicit
// mode 0 or 2 keeps the plain sequence of kernels.
bool plan_pack_fused(const Geometry &g, const PipePlan &pp)
{
    return pp.mode != 0 && (pp.mode == 1 || g.modes.pipeline < 0) && plan_pack_shape_ok(g);
}

int route_dispatch_regather_impl(const Geometry &g, const float *logits, const void *x, int32_t *topk_idx, float *gates,
                                 void *stage, void *final_, void *ws, hipStream_t st)
{
    int rc = MONTA_OK;
    const Shape &s = g.s;
    const PipePlan pp = pipeline_plan(g);
    const int rows_per_wg = kMoverThreads / s.lpr;
    if (!plan_pack_fused(g, pp)) {
        if ((rc = route_impl(g, logits, topk_idx, gates, ws, st))) return rc;
        return pipeline_impl(g, pp, x, stage, final_, ws, false, st);
    }
    PlanPtrs p = plan_ptrs(g, ws);
    if ((rc = launch_route(g, p, logits, topk_idx, gates, st))) return rc;
    {
        const int nt = (pp.first < s.S ? pp.first : s.S) * s.tp * s.Tu;      // tokens of the first group
        const int n_pack = (nt + rows_per_wg - 1) / rows_per_wg;           // one token group per workgroup, no striding
        ProfScope ps(MONTA_K_PLAN_PACK, st);
        hipLaunchKernelGGL(plan_pack_kernel, dim3(s.num_blocks + n_pack), dim3(kMoverThreads), 0, st, topk_idx,
                           static_cast<const u32x4 *>(x), static_cast<u32x4 *>(stage), p, s, 0, nt, s.num_blocks);
        HIP_TRY(hipGetLastError());
    }
    return pipeline_impl(g, pp, x, stage, final_, ws, true, st);
}

int combine_impl(const Geometry &g, int dtype, const void *y, const float *gates, void *out, const void *ws, hipStream_t st)
{
    const Shape &s = g.s;
    const PlanPtrs p = plan_ptrs(g, ws);
    ProfScope ps(MONTA_K_COMBINE, st);
    const dim3 grid(mover_grid(s, s.T)), block(kMoverThreads);
    const bool wide = s.vpr > 2 * s.lpr;   // more than two vectors per lane: 4 per pass
    const u32x4 *yv = static_cast<const u32x4 *>(y);
    u32x4 *ov = static_cast<u32x4 *>(out);
    // With three or more choices per token the software-pipelined form wins (measured on MI355X, 65536 tokens of
    // 14 KiB, top-8 with drops: 802 -> 707 us); with one or two there is nothing to pipeline and its extra
    // registers cost 2-4 %.  It needs the token's k positions to fit the lanes that share its row.
    if (s.k >= 3 && s.k <= s.lpr) {
        if (dtype == MONTA_BF16) {
            if (wide) hipLaunchKernelGGL((combine_pf_kernel<true, 4>), grid, block, 0, st, yv, gates, ov, p, s);
            else hipLaunchKernelGGL((combine_pf_kernel<true, 2>), grid, block, 0, st, yv, gates, ov, p, s);
        } else {
            if (wide) hipLaunchKernelGGL((combine_pf_kernel<false, 4>), grid, block, 0, st, yv, gates, ov, p, s);
            else hipLaunchKernelGGL((combine_pf_kernel<false, 2>), grid, block, 0, st, yv, gates, ov, p, s);
        }
        HIP_TRY(hipGetLastError());
        return MONTA_OK;
    }
    if (dtype == MONTA_BF16) {
        if (wide) hipLaunchKernelGGL((combine_kernel<true, 4>), grid, block, 0, st, yv, gates, ov, p, s);
        else hipLaunchKernelGGL((combine_kernel<true, 2>), grid, block, 0, st, yv, gates, ov, p, s);
    } else {
        if (wide) hipLaunchKernelGGL((combine_kernel<false, 4>), grid, block, 0, st, yv, gates, ov, p, s);
        else hipLaunchKernelGGL((combine_kernel<false, 2>), grid, block, 0, st, yv, gates, ov, p, s);
    }
    HIP_TRY(hipGetLastError());
    return MONTA_OK;
}

}  // namespace

extern "C" {

int monta_workspace_bytes(const monta_cfg *cfg, size_t *ws_bytes, int64_t *max_rows)
{
    if (!ws_bytes || !max_rows) return MONTA_ERR_NULL;
    Geometry g;
    int rc = validate(cfg, &g);
    if (rc) return rc;
    monta_ws_layout L;
    fill_layout(g, &L);
    *ws_bytes = (size_t)L.ws_bytes;
    *max_rows = L.max_rows;
    return MONTA_OK;
}

int monta_ws_layout_query(const monta_cfg *cfg, monta_ws_layout *layout)
{
    if (!layout) return MONTA_ERR_NULL;
    Geometry g;
    int rc = validate(cfg, &g);
    if (rc) return rc;
    fill_layout(g, layout);
    return MONTA_OK;
}

int monta_ws_init(const monta_cfg *cfg, void *ws, void *stream)
{
    Geometry g;
    int rc = validate(cfg, &g);
    if (rc) return rc;
    if ((rc = check_ws(ws))) return rc;
    PlanPtrs p = plan_ptrs(g, ws);
    hipLaunchKernelGGL(ws_init_kernel, dim3(1), dim3(kWave), 0, static_cast<hipStream_t>(stream), p.meta);
    HIP_TRY(hipGetLastError());
    return MONTA_OK;
}

int monta_gate(const monta_cfg *cfg, const void *x, const void *w_gate, float *logits, void *stream)
{
    Geometry g;
    int rc = validate(cfg, &g);
    if (rc) return rc;
    if (!x || !w_gate || !logits) return MONTA_ERR_NULL;
    if (misaligned(x, 16) || misaligned(w_gate, 16) || misaligned(logits, 4)) return MONTA_ERR_ALIGN;
    const Shape &s = g.s;
    const int64_t T = s.T;
    const int H = cfg->hidden, E = s.E;
    hipStream_t st = static_cast<hipStream_t>(stream);
    ProfScope ps(MONTA_K_GATE, st);
    if (cfg->dtype == MONTA_BF16) {
        // validate() guarantees H % 8 == 0 (rows are whole 16-byte vectors) and E <= 256 (at most 8 tiles).
        // Few token tiles: one workgroup per CU with a deep step; many: shallower steps, several workgroups per CU.
        const int64_t tiles32 = (T + 31) / 32;
        const u32x4 *xv = static_cast<const u32x4 *>(x), *wv = static_cast<const u32x4 *>(w_gate);
        rc = launch_gate_small_any(xv, wv, logits, T, H, E, st);
        if (rc <= 0) {
            if (rc) return rc;
        }
        else if (E <= 32)
            rc = tiles32 >= 512 ? launch_gate<1, 1, 512, true>(xv, wv, logits, T, H, E, st)
                                : launch_gate<1, 1, 1024, true>(xv, wv, logits, T, H, E, st);
        // More experts: with at least one 128-token workgroup per CU, every wave owns whole output tiles (W_g is
        // re-read once per 128 tokens instead of once per 32-64, and the small tiles let 3 workgroups share a CU);
        // with fewer tokens, 32-token workgroups with the k-slices dealt to the waves keep the chip filled.
        else if (E <= 64)
            rc = tiles32 >= 1024 ? launch_gate<4, 2, 128, false, true>(xv, wv, logits, T, H, E, st)
                                 : launch_gate<1, 2, 512, true>(xv, wv, logits, T, H, E, st);
        else if (E <= 128)
            rc = tiles32 >= 1024 ? launch_gate<4, 4, 64, false, true>(xv, wv, logits, T, H, E, st)
                                 : launch_gate<1, 4, 256, true>(xv, wv, logits, T, H, E, st);
        else
            rc = tiles32 >= 1024 ? launch_gate<4, 8, 64, false, true>(xv, wv, logits, T, H, E, st)
                                 : launch_gate<1, 8, 128, false>(xv, wv, logits, T, H, E, st);
        if (rc) return rc;
    } else {
        hipLaunchKernelGGL(gate_f32_kernel, dim3((unsigned)((T + 3) / 4)), dim3(256), 0, st,
                           static_cast<const float4 *>(x), static_cast<const float4 *>(w_gate), logits, T, H, E);
    }
    HIP_TRY(hipGetLastError());
    return MONTA_OK;
}

int monta_expert_linear(const monta_cfg *cfg, const void *x_final, const void *w_exp, int32_t out_features, void *y,
                        const void *ws, int slice, void *stream)
{
    Geometry g;
    int rc = validate(cfg, &g);
    if (rc) return rc;
    if ((rc = check_expert_args(cfg, g, x_final, w_exp, out_features, y, ws, slice))) return rc;
    return launch_expert_layer(cfg, g, x_final, w_exp, out_features, y, ws, slice, static_cast<hipStream_t>(stream));
}

int monta_route_dispatch_expert(const monta_cfg *cfg, const float *logits, const void *x, int32_t *topk_idx, float *gates,
                                void *stage, void *final_, const void *w_exp, int32_t out_features, void *y, void *ws,
                                int overlap, void *stream)
{
    Geometry g;
    int rc = validate(cfg, &g);
    if (rc) return rc;
    if ((rc = check_route_ptrs(logits, topk_idx, gates, ws))) return rc;
    if ((rc = check_act_ptrs(x, stage))) return rc;
    if ((rc = check_act_ptrs(stage, final_))) return rc;
    if (stage == final_ || y == stage || y == x) return MONTA_ERR_INVALID;
    if ((rc = check_expert_args(cfg, g, final_, w_exp, out_features, y, ws, -1))) return rc;
    if (overlap != 0 && overlap != 1) return MONTA_ERR_INVALID;
    hipStream_t st = static_cast<hipStream_t>(stream);
    if (!overlap) {
        if ((rc = route_dispatch_regather_impl(g, logits, x, topk_idx, gates, stage, final_, ws, st))) return rc;
        return launch_expert_layer(cfg, g, final_, w_exp, out_features, y, ws, -1, st);
    }
    // Overlapped: the slice pipeline of pipeline mode 1 on the caller's stream, an event behind the kernel that
    // completes a slice's rows of FINAL, and that slice's expert layer on the side stream: the matrix cores work
    // on slice j while the movers stream slice j+1.
    const int S = g.s.S;
    DevState *d = nullptr;
    if ((rc = dev_state(S, &d))) return rc;
    std::lock_guard<std::mutex> lk(d->mu);      // the side stream and its events are shared per device
    if ((rc = route_impl(g, logits, topk_idx, gates, ws, st))) return rc;
    const PlanPtrs p = plan_ptrs(g, ws);
    if ((rc = launch_pack(g, p, x, stage, 0, 1, st))) return rc;
    for (int j = 0; j < S; ++j) {
        rc = j + 1 < S ? launch_pack_regather(g, p, x, stage, final_, j + 1, j + 2, j, j + 1, st)      // pack(j+1) and regather(j)
                       : launch_regather(g, p, stage, final_, j, j + 1, st);
        if (rc) return rc;
        HIP_TRY(hipEventRecord(d->ev[j], st));
        HIP_TRY(hipStreamWaitEvent(d->side, d->ev[j], 0));
        prof_break_chain(d->side);
        if ((rc = launch_expert_layer(cfg, g, final_, w_exp, out_features, y, ws, j, d->side))) return rc;
    }
    HIP_TRY(hipEventRecord(d->done, d->side));
    HIP_TRY(hipStreamWaitEvent(st, d->done, 0));
    prof_break_chain(st);
    return MONTA_OK;
}

int monta_route(const monta_cfg *cfg, const float *logits, int32_t *topk_idx, float *gates, void *ws, void *stream)
{
    Geometry g;
    int rc = validate(cfg, &g);
    if (rc) return rc;
    if ((rc = check_route_ptrs(logits, topk_idx, gates, ws))) return rc;
    return route_impl(g, logits, topk_idx, gates, ws, static_cast<hipStream_t>(stream));
}

int monta_route_dispatch_regather(const monta_cfg *cfg, const float *logits, const void *x, int32_t *topk_idx,
                                  float *gates, void *stage, void *final_, void *ws, void *stream)
{
    Geometry g;
    int rc = validate(cfg, &g);
    if (rc) return rc;
    if ((rc = check_route_ptrs(logits, topk_idx, gates, ws))) return rc;
    if ((rc = check_act_ptrs(x, stage))) return rc;
    if ((rc = check_act_ptrs(stage, final_))) return rc;
    if (stage == final_) return MONTA_ERR_INVALID;
    return route_dispatch_regather_impl(g, logits, x, topk_idx, gates, stage, final_, ws, static_cast<hipStream_t>(stream));
}

int monta_dispatch(const monta_cfg *cfg, const void *x, void *stage, const void *ws, int slice, void *stream)
{
    Geometry g;
    int rc = validate(cfg, &g);
    if (rc) return rc;
    if (slice < -1 || slice >= cfg->slices) return MONTA_ERR_INVALID;
    if ((rc = check_act_ptrs(x, stage))) return rc;
    if ((rc = check_ws(ws))) return rc;
    return launch_pack(g, plan_ptrs(g, ws), x, stage, slice < 0 ? 0 : slice, slice < 0 ? g.s.S : slice + 1,
                       static_cast<hipStream_t>(stream));
}

int monta_regather(const monta_cfg *cfg, const void *stage, void *final_, const void *ws, int slice, void *stream)
{
    Geometry g;
    int rc = validate(cfg, &g);
    if (rc) return rc;
    if (slice < -1 || slice >= cfg->slices) return MONTA_ERR_INVALID;
    if ((rc = check_act_ptrs(stage, final_))) return rc;
    if (stage == final_) return MONTA_ERR_INVALID;
    if ((rc = check_ws(ws))) return rc;
    return launch_regather(g, plan_ptrs(g, ws), stage, final_, slice < 0 ? 0 : slice, slice < 0 ? g.s.S : slice + 1,
                           static_cast<hipStream_t>(stream));
}

int monta_dispatch_regather(const monta_cfg *cfg, const void *x, void *stage, void *final_, const void *ws,
                            void *stream)
{
    Geometry g;
    int rc = validate(cfg, &g);
    if (rc) return rc;
    if ((rc = check_act_ptrs(x, stage))) return rc;
    if ((rc = check_act_ptrs(stage, final_))) return rc;
    if (stage == final_) return MONTA_ERR_INVALID;
    if ((rc = check_ws(ws))) return rc;
    return dispatch_regather_impl(g, x, stage, final_, ws, static_cast<hipStream_t>(stream));
}

int monta_combine(const monta_cfg *cfg, const void *y, const float *gates, void *out, const void *ws, void *stream)
{
    Geometry g;
    int rc = validate(cfg, &g);
    if (rc) return rc;
    if (!gates) return MONTA_ERR_NULL;
    if (misaligned(gates, 4)) return MONTA_ERR_ALIGN;
    if ((rc = check_act_ptrs(y, out))) return rc;
    if (y == out) return MONTA_ERR_INVALID;
    if ((rc = check_ws(ws))) return rc;
    return combine_impl(g, cfg->dtype, y, gates, out, ws, static_cast<hipStream_t>(stream));
}

namespace {

int allgather_grid(const Geometry &g, int nslices)
{
    const int64_t vecs = slice_rows_bound(g, nslices) * g.s.vpr;
    int64_t wg = (vecs + (int64_t)kMoverThreads * kVecInFlight - 1) / ((int64_t)kMoverThreads * kVecInFlight);
    if (wg < 1) wg = 1;
    if (wg > 32768) wg = 32768;
    return (int)wg;
}

int launch_allgather(const Geometry &g, const PlanPtrs &p, const void *stage, void *gathered, int j0, int j1, hipStream_t st)
{
    const Shape &s = g.s;
    ProfScope ps(MONTA_K_ALLGATHER, st);
    hipLaunchKernelGGL(allgather_kernel, dim3((unsigned)allgather_grid(g, j1 - j0)), dim3(kMoverThreads), 0, st,
                       static_cast<const u32x4 *>(stage), static_cast<u32x4 *>(gathered), p, s, j0 * s.tp, j1 * s.tp);
    HIP_TRY(hipGetLastError());
    return MONTA_OK;
}

}  // namespace

int monta_allgather(const monta_cfg *cfg, const void *stage, void *gathered, const void *ws, int slice, void *stream)
{
    Geometry g;
    int rc = validate(cfg, &g);
    if (rc) return rc;
    if (slice < -1 || slice >= cfg->slices) return MONTA_ERR_INVALID;
    if ((rc = check_act_ptrs(stage, gathered))) return rc;
    if (stage == gathered) return MONTA_ERR_INVALID;
    if ((rc = check_ws(ws))) return rc;
    return launch_allgather(g, plan_ptrs(g, ws), stage, gathered, slice < 0 ? 0 : slice, slice < 0 ? g.s.S : slice + 1,
                            static_cast<hipStream_t>(stream));
}

int monta_allgather_regather(const monta_cfg *cfg, const void *stage, void *gathered, void *final_, const void *ws,
                             int schedule, void *stream)
{
    Geometry g;
    int rc = validate(cfg, &g);
    if (rc) return rc;
    if (schedule < 0 || schedule > 2) return MONTA_ERR_INVALID;
    if ((rc = check_act_ptrs(stage, gathered))) return rc;
    if ((rc = check_act_ptrs(gathered, final_))) return rc;
    if (stage == gathered || gathered == final_ || stage == final_) return MONTA_ERR_INVALID;
    if ((rc = check_ws(ws))) return rc;
    const Shape &s = g.s;
    const PlanPtrs p = plan_ptrs(g, ws);
    hipStream_t st = static_cast<hipStream_t>(stream);
    const int S = s.S;
    if (schedule == 0) {            // chunk by chunk, gather then copy: no overlap
        for (int j = 0; j < S; ++j) {
            if ((rc = launch_allgather(g, p, stage, gathered, j, j + 1, st))) return rc;
            if ((rc = launch_regather(g, p, gathered, final_, j, j + 1, st))) return rc;
        }
        return MONTA_OK;
    }
    if (schedule == 1) {            // launch j gathers chunk j and, in disjoint workgroups, copies chunk j-1
        if ((rc = launch_allgather(g, p, stage, gathered, 0, 1, st))) return rc;
        for (int j = 1; j < S; ++j) {
            const int n_gather = allgather_grid(g, 1), n_copy = regather_grid(s, slice_rows_bound(g, 1));
            ProfScope ps(MONTA_K_ALLGATHER_REGATHER, st);
            hipLaunchKernelGGL(allgather_regather_kernel, dim3(n_gather + n_copy), dim3(kMoverThreads), 0, st,
                               static_cast<const u32x4 *>(stage), static_cast<u32x4 *>(gathered), static_cast<u32x4 *>(final_),
                               p, s, j * s.tp, (j + 1) * s.tp, (j - 1) * s.tp, j * s.tp, n_gather);
            HIP_TRY(hipGetLastError());
        }
        return launch_regather(g, p, gathered, final_, S - 1, S, st);
    }
    // schedule 2: the paper's stream picture: gathers on the caller's stream, copies on the library's side stream
    // (default priority), one event per chunk, joined back into the caller's stream
    DevState *d = nullptr;
    if ((rc = dev_state(S, &d))) return rc;
    std::lock_guard<std::mutex> lk(d->mu);
    for (int j = 0; j < S; ++j) {
        if ((rc = launch_allgather(g, p, stage, gathered, j, j + 1, st))) return rc;
        HIP_TRY(hipEventRecord(d->ev[j], st));
        HIP_TRY(hipStreamWaitEvent(d->side, d->ev[j], 0));
        prof_break_chain(d->side);
        if ((rc = launch_regather(g, p, gathered, final_, j, j + 1, d->side))) return rc;
    }
    HIP_TRY(hipEventRecord(d->done, d->side));
    HIP_TRY(hipStreamWaitEvent(st, d->done, 0));
    prof_break_chain(st);
    return MONTA_OK;
}

// mirrored return path -------------------------------------------------------------------------

int monta_unregather(const monta_cfg *cfg, const void *y, void *y_stage, const void *ws, int slice, void *stream)
{
    Geometry g;
    int rc = validate(cfg, &g);
    if (rc) return rc;
    if (slice < -1 || slice >= cfg->slices) return MONTA_ERR_INVALID;
    if ((rc = check_act_ptrs(y, y_stage))) return rc;
    if (y == y_stage) return MONTA_ERR_INVALID;
    if ((rc = check_ws(ws))) return rc;
    const Shape &s = g.s;
    const PlanPtrs p = plan_ptrs(g, ws);
    hipStream_t st = static_cast<hipStream_t>(stream);
    const int u0 = slice < 0 ? 0 : slice * s.tp;
    const int u1 = slice < 0 ? s.U : (slice + 1) * s.tp;
    ProfScope ps(MONTA_K_UNREGATHER, st);
    hipLaunchKernelGGL(unregather_kernel, dim3(regather_grid(s, slice_rows_bound(g, slice < 0 ? s.S : 1))),
                       dim3(kMoverThreads), 0, st, static_cast<const u32x4 *>(y), static_cast<u32x4 *>(y_stage), p, s,
                       u0, u1);
    HIP_TRY(hipGetLastError());
    return MONTA_OK;
}

namespace {

// launches unregather(units [u0,u1)) and / or combine of tokens [t0, t0+nt) from the unit-major layout
int launch_unregather_combine(const Geometry &g, const PlanPtrs &p, int dtype, const void *y, void *y_stage,
                              const float *gates, void *out, int u0, int u1, int t0, int nt, hipStream_t st)
{
    Shape s = g.s;
    // the rows fetched back are read exactly once by the staged combine: stream them unless the caller set a policy
    if (g.modes.cache < 0) s.cache |= NT_COMB_LD;
    const int n_unreg = u0 < u1 ? regather_grid(s, slice_rows_bound(g, (u1 - u0) / s.tp)) : 0;
    const int n_comb = nt > 0 ? mover_grid(s, nt) : 0;
    if (n_unreg + n_comb == 0) return MONTA_OK;
    const bool wide = s.vpr > 2 * s.lpr;
    const u32x4 *yv = static_cast<const u32x4 *>(y);
    u32x4 *sv = static_cast<u32x4 *>(y_stage), *ov = static_cast<u32x4 *>(out);
    const dim3 grid(n_unreg + n_comb), block(kMoverThreads);
    ProfScope ps(n_unreg && n_comb ? MONTA_K_UNREGATHER_COMBINE : (n_unreg ? MONTA_K_UNREGATHER : MONTA_K_COMBINE), st);
    const bool pf = s.k >= 3 && s.k <= s.lpr;       // as in monta_combine
#define MONTA_LAUNCH_UC(BF, NV_, PF_)                                                                                    \
    hipLaunchKernelGGL((unregather_combine_kernel<BF, NV_, PF_>), grid, block, 0, st, yv, sv, gates, ov, p, s, u0, u1, t0, \
                       nt, n_unreg)
    if (dtype == MONTA_BF16) {
        if (pf) { if (wide) MONTA_LAUNCH_UC(true, 4, true); else MONTA_LAUNCH_UC(true, 2, true); }
        else { if (wide) MONTA_LAUNCH_UC(true, 4, false); else MONTA_LAUNCH_UC(true, 2, false); }
    } else {
        if (pf) { if (wide) MONTA_LAUNCH_UC(false, 4, true); else MONTA_LAUNCH_UC(false, 2, true); }
        else { if (wide) MONTA_LAUNCH_UC(false, 4, false); else MONTA_LAUNCH_UC(false, 2, false); }
    }
#undef MONTA_LAUNCH_UC
    HIP_TRY(hipGetLastError());
    return MONTA_OK;
}

int check_staged_combine(const monta_cfg *cfg, Geometry *g, const void *y_stage, const float *gates, void *out,
                         const void *ws)
{
    int rc = validate(cfg, g);
    if (rc) return rc;
    if (!gates) return MONTA_ERR_NULL;
    if (misaligned(gates, 4)) return MONTA_ERR_ALIGN;
    if ((rc = check_act_ptrs(y_stage, out))) return rc;
    if (y_stage == out) return MONTA_ERR_INVALID;
    return check_ws(ws);
}

}  // namespace

int monta_combine_staged(const monta_cfg *cfg, const void *y_stage, const float *gates, void *out, const void *ws,
                         int slice, void *stream)
{
    Geometry g;
    int rc = check_staged_combine(cfg, &g, y_stage, gates, out, ws);
    if (rc) return rc;
    if (slice < -1 || slice >= cfg->slices) return MONTA_ERR_INVALID;
    const Shape &s = g.s;
    const int per_slice = s.tp * s.Tu;
    const int t0 = slice < 0 ? 0 : slice * per_slice, nt = slice < 0 ? s.T : per_slice;
    return launch_unregather_combine(g, plan_ptrs(g, ws), cfg->dtype, y_stage, const_cast<void *>(y_stage), gates, out,
                                     0, 0, t0, nt, static_cast<hipStream_t>(stream));
}

int monta_unregather_combine(const monta_cfg *cfg, const void *y, void *y_stage, const float *gates, void *out,
                             const void *ws, void *stream)
{
    Geometry g;
    int rc = check_staged_combine(cfg, &g, y_stage, gates, out, ws);
    if (rc) return rc;
    if ((rc = check_act_ptrs(y, y_stage))) return rc;
    if (y == y_stage || y == out) return MONTA_ERR_INVALID;
    const Shape &s = g.s;
    const PlanPtrs p = plan_ptrs(g, ws);
    hipStream_t st = static_cast<hipStream_t>(stream);
    const int per_slice = s.tp * s.Tu;
    // Launch grouping as in the forward pipeline, by the same measurements: with an explicit pipeline mode launch j
    // fetches slice j back and, in disjoint workgroups of the same grid, combines the tokens of slice j-1; by
    // default consecutive slices are grouped until a group's rows reach 256 MiB, and a group that large (or a
    // problem that is one group) runs as two plain kernels, fetch then combine.
    int spg = 1;
    bool serial = false;
    if (g.modes.pipeline < 0) {
        const int64_t slice_bytes = slice_rows_bound(g, 1) * g.row_bytes;
        if (slice_bytes >= kGroupBytes) serial = true;
        else {
            spg = (int)(kGroupBytes / slice_bytes);
            if (spg > s.S) spg = s.S;
            const int groups = (s.S + spg - 1) / spg;
            spg = (s.S + groups - 1) / groups;
            serial = groups == 1 || spg * slice_bytes >= kGroupBytes * 3 / 4;
        }
    } else {
        serial = g.modes.pipeline == 2;
    }
    const int G = (s.S + spg - 1) / spg;
    auto lo = [&](int gi) { return gi * spg; };
    auto hi = [&](int gi) { return (gi + 1) * spg < s.S ? (gi + 1) * spg : s.S; };
    if (serial) {
        for (int gi = 0; gi < G; ++gi) {
            if ((rc = launch_unregather_combine(g, p, cfg->dtype, y, y_stage, gates, out, lo(gi) * s.tp, hi(gi) * s.tp, 0, 0, st)))
                return rc;
            if ((rc = launch_unregather_combine(g, p, cfg->dtype, y, y_stage, gates, out, 0, 0, lo(gi) * per_slice,
                                                (hi(gi) - lo(gi)) * per_slice, st)))
                return rc;
        }
        return MONTA_OK;
    }
    for (int gi = 0; gi <= G; ++gi) {
        const int u0 = gi < G ? lo(gi) * s.tp : 0, u1 = gi < G ? hi(gi) * s.tp : 0;
        const int t0 = gi > 0 ? lo(gi - 1) * per_slice : 0, nt = gi > 0 ? (hi(gi - 1) - lo(gi - 1)) * per_slice : 0;
        if ((rc = launch_unregather_combine(g, p, cfg->dtype, y, y_stage, gates, out, u0, u1, t0, nt, st))) return rc;
    }
    return MONTA_OK;
}

// ---- one entry point that allocates nothing -------------------------------------------------------
//
// The plan tables of the whole step live in a file-scope device array instead of a caller workspace.
// In host code the array's name is only a stand-in for the symbol: the device address is looked up once
// per device (every GPU holds its own copy at its own address) and only that address is ever handed to
// kernels.

constexpr size_t kStaticScratchBytes = 16u << 20;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

namespace {

std::mutex g_scratch_mu;
void *g_scratch_ptr[64] = {nullptr};

int static_scratch(void **out)
{
    int dev = 0;
    HIP_TRY(hipGetDevice(&dev));
    if (dev < 0 || dev >= 64) return MONTA_ERR_UNSUPPORTED;
    std::lock_guard<std::mutex> lk(g_scratch_mu);
    if (!g_scratch_ptr[dev]) {
        void *ptr = nullptr;
        HIP_TRY(hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)));      // the current device's copy of the array
        if (!ptr) return MONTA_ERR_HIP;
        g_scratch_ptr[dev] = ptr;
    }
    *out = g_scratch_ptr[dev];
    return MONTA_OK;
}

}  // namespace

int monta_route_dispatch_combine_static(const monta_cfg *cfg, const float *logits, const void *x, int32_t *topk_idx,
                                        float *gates, void *stage, void *final_, void *out, void *stream)
{
    Geometry g;
    int rc = validate(cfg, &g);
    if (rc) return rc;
    if (!logits || !topk_idx || !gates) return MONTA_ERR_NULL;
    if (misaligned(logits, 4) || misaligned(topk_idx, 4) || misaligned(gates, 4)) return MONTA_ERR_ALIGN;
    if ((rc = check_act_ptrs(x, stage))) return rc;
    if ((rc = check_act_ptrs(final_, out))) return rc;
    if (stage == final_ || final_ == out || stage == out || x == out) return MONTA_ERR_INVALID;
    monta_ws_layout L;
    fill_layout(g, &L);
    if ((size_t)L.ws_bytes > kStaticScratchBytes) return MONTA_ERR_TOO_LARGE;
    // event profiling creates events per launch and the two-stream pipeline creates a stream: neither belongs
    // in a call that must not allocate
    if (g_prof_on.load()) return MONTA_ERR_INVALID;
    if (g.modes.pipeline == 0) g.modes.pipeline = -1;      // pipeline_plan() then never answers 0
    void *ws = nullptr;
    if ((rc = static_scratch(&ws))) return rc;
    hipStream_t st = static_cast<hipStream_t>(stream);
    // the array keeps the previous call's contents (possibly of another shape): put the counters back to zero
    hipLaunchKernelGGL(ws_init_kernel, dim3(1), dim3(kWave), 0, st, plan_ptrs(g, ws).meta);
    HIP_TRY(hipGetLastError());
    if ((rc = route_dispatch_regather_impl(g, logits, x, topk_idx, gates, stage, final_, ws, st))) return rc;
    return combine_impl(g, cfg->dtype, final_, gates, out, ws, st);
}

int monta_pipeline_query(const monta_cfg *cfg, int32_t *mode, int32_t *first_slices, int32_t *slices_per_launch,
                         int32_t *plan_fused)
{
    if (!mode || !first_slices || !slices_per_launch || !plan_fused) return MONTA_ERR_NULL;
    Geometry g;
    int rc = validate(cfg, &g);
    if (rc) return rc;
    const PipePlan pp = pipeline_plan(g);
    *mode = pp.mode;
    *first_slices = pp.first < g.s.S ? pp.first : g.s.S;
    *slices_per_launch = pp.spg;
    *plan_fused = plan_pack_fused(g, pp) ? 1 : 0;
    return MONTA_OK;
}

int monta_set_pipeline_mode(int mode)
{
    if (mode < -1 || mode > 2) return MONTA_ERR_INVALID;
    g_pipeline_mode.store(mode);
    return MONTA_OK;
}

int monta_get_pipeline_mode(void) { return g_pipeline_mode.load(); }

int monta_set_plan_mode(int mode)
{
    if (mode != -1 && mode != 0) return MONTA_ERR_INVALID;
    g_plan_mode.store(mode);
    return MONTA_OK;
}

int monta_get_plan_mode(void) { return g_plan_mode.load(); }

int monta_set_cache_policy(int policy)
{
    if (policy < -1 || policy > 63) return MONTA_ERR_INVALID;
    g_cache_policy.store(policy);
    return MONTA_OK;
}

int monta_get_cache_policy(void) { return g_cache_policy.load(); }

int monta_copy(void *dst, const void *src, size_t bytes, void *stream)
{
    if (!dst || !src) return MONTA_ERR_NULL;
    if (bytes == 0 || bytes % 16 != 0) return MONTA_ERR_INVALID;
    if (misaligned(dst, 16) || misaligned(src, 16)) return MONTA_ERR_ALIGN;
    const size_t nvec = bytes / 16;
    size_t wg = (nvec + (size_t)kMoverThreads * kVecInFlight - 1) / ((size_t)kMoverThreads * kVecInFlight);
    if (wg > (size_t)kMaxMoverGrid) wg = kMaxMoverGrid;
    hipStream_t st = static_cast<hipStream_t>(stream);
    ProfScope ps(MONTA_K_COPY, st);
    hipLaunchKernelGGL(copy_kernel, dim3((unsigned)wg), dim3(kMoverThreads), 0, st, static_cast<const u32x4 *>(src),
                       static_cast<u32x4 *>(dst), nvec);
    HIP_TRY(hipGetLastError());
    return MONTA_OK;
}

int monta_profile_enable(int on)
{
    g_prof_on.store(on ? 1 : 0);
    std::lock_guard<std::mutex> lk(g_prof_mu);
    for (auto &pr : g_prof_last) pr.second = nullptr;     // work enqueued while disabled must not be timed
    return MONTA_OK;
}

int monta_profile_reset(void)
{
    int rc = prof_drain();
    std::lock_guard<std::mutex> lk(g_prof_mu);
    for (int i = 0; i < MONTA_K_COUNT; ++i) {
        g_prof_ms[i] = 0.0;
        g_prof_n[i] = 0;
    }
    return rc;
}

int monta_profile_read(int kernel_id, double *total_ms, int64_t *launches)
{
    if (!total_ms || !launches) return MONTA_ERR_NULL;
    if (kernel_id < 0 || kernel_id >= MONTA_K_COUNT) return MONTA_ERR_INVALID;
    int rc = prof_drain();
    std::lock_guard<std::mutex> lk(g_prof_mu);
    *total_ms = g_prof_ms[kernel_id];
    *launches = g_prof_n[kernel_id];
    return rc;
}

const char *monta_strerror(int code)
{
    switch (code) {
        case MONTA_OK: return "ok";
        case MONTA_ERR_INVALID: return "invalid argument (size, flag or slice violates the preconditions)";
        case MONTA_ERR_UNSUPPORTED: return "shape outside the library's limits";
        case MONTA_ERR_NULL: return "required pointer is NULL";
        case MONTA_ERR_HIP: return "HIP runtime call failed (see monta_last_hip_error)";
        case MONTA_ERR_ALIGN: return "pointer is not aligned as required";
        case MONTA_ERR_TOO_LARGE: return "problem needs more plan-table space than the library's static scratch array holds (16 MiB)";
        default: return "unknown monta status";
    }
}

int monta_last_hip_error(void) { return g_last_hip; }

int monta_shutdown(void)
{
    int rc = prof_drain();
    std::lock_guard<std::mutex> lk(g_dev_mu);
    int cur = 0;
    HIP_TRY(hipGetDevice(&cur));
    for (int dev = 0; dev < 64; ++dev) {
        DevState &d = g_dev[dev];
        if (!d.side && !d.done && d.ev.empty()) continue;
        std::lock_guard<std::mutex> dl(d.mu);
        HIP_TRY(hipSetDevice(dev));
        if (d.side) {
            HIP_TRY(hipStreamSynchronize(d.side));
            HIP_TRY(hipStreamDestroy(d.side));
            d.side = nullptr;
        }
        for (hipEvent_t e : d.ev) HIP_TRY(hipEventDestroy(e));
        d.ev.clear();
        if (d.done) {
            HIP_TRY(hipEventDestroy(d.done));
            d.done = nullptr;
        }
    }
    HIP_TRY(hipSetDevice(cur));
    return rc;
}

}  // extern "C"
