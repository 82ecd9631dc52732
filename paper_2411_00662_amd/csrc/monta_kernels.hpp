// Device code of the MoE dispatch / combine path for gfx950 (wave64).
//
// The path itself (route, plan, pack, regather, combine and the mirrored return path)
// is bandwidth or latency bound: no dense contraction, so no MFMA.  The row movers
// move rows of 16-byte vectors straight through registers with several loads in
// flight per lane; the planning kernels are integer work on wavefront bit masks.
// The two optional stages around it, the gate projection and the expert layer, are
// dense contractions and run on the matrix cores; they follow further down.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include <type_traits>

namespace monta {

typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

constexpr int kWave = 64;
// Chosen by measurement on MI355X (128 and 512 threads, 2 and 8 vectors in flight were slower or equal).
constexpr int kMoverThreads = 256;   // threads per workgroup of the row movers
constexpr int kVecInFlight = 4;      // 16-byte loads issued by a lane before its first store

// meta[] slots (int32)
enum { META_R = 0, META_ALIVE = 1, META_C = 2, META_DONE = 3, META_FINAL_ROWS = 4, META_SLOTS = 16 };

struct PlanPtrs {
    int32_t *meta, *counts, *kept, *offsets, *n, *stage_off, *unit_base, *send_rows, *unit_rows;
    int32_t *pos_final, *pos_stage, *row_map, *block_counts, *block_base, *local_rank, *kept_prefix;
};

struct Shape {
    int32_t T, E, k, ep, tp, S, U, Tu;
    int32_t TB;        // tokens per route workgroup
    int32_t bpu;       // route workgroups per unit
    int32_t num_blocks;
    int32_t C;         // per-expert capacity
    int32_t renorm;
    int32_t vpr;       // 16-byte vectors per activation row
    int32_t lpr;       // lanes cooperating on one row in the movers (power of two <= kMoverThreads)
    int32_t max_rows;  // rows STAGE / FINAL hold; every row index read from a table is checked against it
    int32_t cache;     // CachePolicy bits: which streams of the movers use non-temporal accesses
    int32_t padded;    // 1: FINAL is [E][C][H] (expert e at row e*C), 0: compact
    int32_t rl;        // lanes that share one token in the route kernel (1, 2, 4 or 8)
    int32_t fast_plan; // 1: plan_positions_kernel rebuilds the scans per workgroup; 0: ticketed scan + positions_kernel
};

// A set bit makes that stream non-temporal (streaming, no reuse expected); a clear bit leaves
// it cacheable, which pays when the consumer kernel finds the data still in the memory-side cache.
enum CachePolicy {
    NT_PACK_LD = 1, NT_PACK_ST = 2, NT_REG_LD = 4, NT_REG_ST = 8, NT_COMB_LD = 16, NT_COMB_ST = 32
};

// ------------------------------------------------------------------ helpers

__device__ __forceinline__ int wave_inclusive_scan(int v, int lane)
{
#pragma unroll
    for (int d = 1; d < kWave; d <<= 1) {
        int o = __shfl_up(v, d, kWave);
        if (lane >= d) v += o;
    }
    return v;
}

template <bool NT>
__device__ __forceinline__ u32x4 ld16(const u32x4 *p)
{
    if (NT) return __builtin_nontemporal_load(p);
    return *p;
}
template <bool NT>
__device__ __forceinline__ void st16(u32x4 *p, u32x4 v)
{
    if (NT) __builtin_nontemporal_store(v, p);
    else *p = v;
}

// Calls f(integral_constant<bool, load_nt>, integral_constant<bool, store_nt>) for the two policy bits:
// the four variants stay separate loops, so the compiler cannot fold the access kinds together.
template <typename F>
__device__ __forceinline__ void with_policy(bool ntl, bool nts, F f)
{
    if (ntl) {
        if (nts) f(std::true_type{}, std::true_type{});
        else f(std::true_type{}, std::false_type{});
    } else {
        if (nts) f(std::false_type{}, std::true_type{});
        else f(std::false_type{}, std::false_type{});
    }
}

// ------------------------------------------------------------ route + plan

// Row stride (floats) of the logits tile in LDS.  A wave holds 64 / L tokens with L lanes each, lane (token, sub)
// reads element sub + q * L of its row: with a stride that is L times an odd number the 64 lanes of a read hit 64
// different banks (for L = 1 this is the usual odd stride).
__host__ __device__ inline int route_row_stride(int E, int L) { return L * (((E + L - 1) / L) | 1); }


// One workgroup routes TB consecutive tokens of ONE unit; s.rl lanes share a token (1 for few experts).
//  1. the [nt][E] logits tile is staged in LDS (coalesced, odd row stride);
//  2. k selection passes per token over its LDS row: the next winner is the largest
//     element that comes after the previous winner in (value desc, index asc) order,
//     so ties resolve to the lower index with no "taken" mask; with s.rl > 1 each lane
//     scans every s.rl-th expert and the lanes of a token agree by xor-shuffles;
//  3. gates in fp64 from the winners' logits, one rounding to fp32;
//  4. every lane ORs its bit into mask[expert][wave] in LDS; popcounts of those
//     masks give the workgroup's expert histogram and each pair's stable rank inside
//     the workgroup (lanes hold consecutive tokens, so bit order is token order);
//  5. (only when s.fast_plan == 0) the last workgroup to finish (ticket counter)
//     turns the per-workgroup histograms into every plan table: exclusive scans
//     over workgroups per expert, capacity clip, expert offsets, per-unit block
//     tables.  With s.fast_plan == 1 plan_positions_kernel does that instead.
// No atomics decide a position: the result is deterministic.
__global__ __launch_bounds__(1024) void route_plan_kernel(const float *__restrict__ logits,
                                                         int32_t *__restrict__ topk_idx,
                                                         float *__restrict__ gates, PlanPtrs p, Shape s)
{
    extern __shared__ __align__(16) unsigned char smem[];
    const int E = s.E, k = s.k, TB = s.TB;
    const int stride = route_row_stride(E, s.rl);
    const int NW = TB > kWave ? TB / kWave : 1;
    float *s_l = reinterpret_cast<float *>(smem);
    int *s_sel = reinterpret_cast<int *>(s_l + (size_t)TB * stride);
    unsigned long long *s_mask = reinterpret_cast<unsigned long long *>(
        smem + (((size_t)TB * stride * 4 + (size_t)TB * k * 4 + 7) & ~(size_t)7));
    double *s_w = reinterpret_cast<double *>(s_mask + (size_t)E * NW);     // [TB][k] unnormalised weights
    double *s_den = s_w + (size_t)TB * k;                                  // [TB] softmax denominators (renorm = 0)
    __shared__ int s_last;
    __shared__ int s_cnt[256];
    __shared__ int s_off[257];

    const int tid = threadIdx.x, lane = tid & (kWave - 1), wave = tid >> 6;
    const int b = blockIdx.x;
    const int u = b / s.bpu, ib = b - u * s.bpu;
    const int t_begin = u * s.Tu + ib * TB;
    int nt = s.Tu - ib * TB;
    if (nt > TB) nt = TB;

    for (int i = tid; i < E * NW; i += blockDim.x) s_mask[i] = 0ull;
    {
        const float *src = logits + (size_t)t_begin * E;
        const int total = nt * E;
        for (int i = tid; i < total; i += blockDim.x) {
            float v = src[i];
            if (v != v) v = -INFINITY;
            const int tok = i / E;
            s_l[tok * stride + (i - tok * E)] = v;
        }
    }
    __syncthreads();

    // token handled by this lane, and which of the token's s.rl lanes it is
    const int L = s.rl;
    const int tok = tid / L, sub = tid - tok * L;
    const int tword = tok >> 6;                     // mask word and bit of the token inside the workgroup
    const unsigned long long tbit = 1ull << (tok & 63);
    const int t = t_begin + tok;
    const bool active = tok < nt;
    if (active) {
        const float *row = s_l + tok * stride;
        int *sel = s_sel + tok * k;
        float pv = INFINITY, top_logit = 0.f;
        int pi = -1;
        for (int j = 0; j < k; ++j) {
            int best = -1;
            float bv = 0.f;
            auto consider = [&](int e, float v) {
                const bool after_prev = (v < pv) || (v == pv && e > pi);
                if (after_prev && (best < 0 || v > bv)) { best = e; bv = v; }
            };
            int e = sub;
            for (; e + 7 * L < E; e += 8 * L) {     // eight independent LDS reads in flight per step
                float v[8];
#pragma unroll
                for (int q = 0; q < 8; ++q) v[q] = row[e + q * L];
#pragma unroll
                for (int q = 0; q < 8; ++q) consider(e + q * L, v[q]);
            }
            for (; e < E; e += L) consider(e, row[e]);
            for (int mk = 1; mk < L; mk <<= 1) {    // the token's lanes agree on (value desc, index asc)
                const float ov = __shfl_xor(bv, mk, kWave);
                const int oi = __shfl_xor(best, mk, kWave);
                if (oi >= 0 && (best < 0 || ov > bv || (ov == bv && oi < best))) { best = oi; bv = ov; }
            }
            if (best < 0) best = (pi + 1 < E) ? pi + 1 : E - 1;   // unreachable for k <= E; keeps indices in range
            pv = bv;
            pi = best;
            if (j == 0) top_logit = bv;
            if (sub == 0) {
                sel[j] = best;
                topk_idx[(size_t)t * k + j] = best;
                atomicOr(&s_mask[best * NW + tword], tbit);
            }
        }
        if (!s.renorm) {
            // softmax over all E: the token's lanes each sum their experts, then add up across the lanes
            double part = 0.0;
            for (int e = sub; e < E; e += L) part += exp((double)row[e] - (double)top_logit);
            for (int mk = 1; mk < L; mk <<= 1) part += __shfl_xor(part, mk, kWave);
            if (sub == 0) s_den[tok] = part;
        }
    }
    __syncthreads();
    // gates: w_j = exp(l_j - l_0) in fp64 (w_0 = 1 needs no call), one (token, choice) pair per lane so that every
    // lane of the workgroup has an exp to do, not only one lane per token; then the denominator is summed in j
    // order (or taken from the sum over all experts), one division, one rounding to fp32.
    const int npairs = nt * k;
    for (int tk = tid; tk < nt; tk += blockDim.x) s_w[tk * k] = 1.0;
    for (int idx = tid; idx < nt * (k - 1); idx += blockDim.x) {         // only the choices j >= 1 need an exp
        const int tk = idx / (k - 1), j = 1 + idx - tk * (k - 1);
        const float *row = s_l + tk * stride;
        const int *sel = s_sel + tk * k;
        s_w[tk * k + j] = exp((double)row[sel[j]] - (double)row[sel[0]]);
    }
    __syncthreads();
    for (int idx = tid; idx < npairs; idx += blockDim.x) {
        const int tk = idx / k;
        double denom = 0.0;
        if (s.renorm) {
            const double *wt = s_w + tk * k;
            for (int j = 0; j < k; ++j) denom += wt[j];
        } else {
            denom = s_den[tk];
        }
        gates[(size_t)t_begin * k + idx] = (float)(s_w[idx] / denom);
    }

    for (int e = tid; e < E; e += blockDim.x) {
        int c = 0;
        for (int w = 0; w < NW; ++w) c += __popcll(s_mask[e * NW + w]);
        p.block_counts[(size_t)b * E + e] = c;
    }
    for (int idx = tid; idx < npairs; idx += blockDim.x) {      // one pair per lane again
        const int tk = idx / k;
        const int e = s_sel[idx];
        const int word = tk >> 6;
        int r = 0;
        for (int w = 0; w < word; ++w) r += __popcll(s_mask[e * NW + w]);
        r += __popcll(s_mask[e * NW + word] & ((1ull << (tk & 63)) - 1ull));
        p.local_rank[(size_t)t_begin * k + idx] = r;    // rank inside the workgroup; the positions kernels finish it
    }

    if (b == 0 && tid == 0) p.meta[META_ALIVE] = 0;   // counted by the kernel that finishes the positions
    if (s.fast_plan) return;

    // ---- ticket: the last workgroup builds the tables
    __threadfence();
    __syncthreads();
    if (tid == 0) s_last = (atomicAdd(&p.meta[META_DONE], 1) == s.num_blocks - 1);
    __syncthreads();
    if (!s_last) return;
    __threadfence();

    const int nblk = s.num_blocks;
    const int nwaves = blockDim.x >> 6;
    const int C = s.C;
    // A: per expert, exclusive scan of the workgroup histograms in workgroup (= token) order
    for (int e = wave; e < E; e += nwaves) {
        int carry = 0;
        for (int b0 = 0; b0 < nblk; b0 += kWave) {
            const int bb = b0 + lane;
            const int v = bb < nblk ? p.block_counts[(size_t)bb * E + e] : 0;
            const int incl = wave_inclusive_scan(v, lane);
            if (bb < nblk) p.block_base[(size_t)bb * E + e] = carry + incl - v;
            carry += __shfl(incl, kWave - 1, kWave);
        }
        if (lane == 0) s_cnt[e] = carry;
    }
    __syncthreads();
    // B: capacity clip and expert offsets (expert order = (EP rank, local expert) order)
    if (wave == 0) {
        int carry = 0;
        for (int e0 = 0; e0 < E; e0 += kWave) {
            const int e = e0 + lane;
            const int cnt = e < E ? s_cnt[e] : 0;
            const int kp = cnt < C ? cnt : C;
            const int incl = wave_inclusive_scan(kp, lane);
            if (e < E) {
                const int off = s.padded ? e * C : carry + incl - kp;
                p.counts[e] = cnt;
                p.kept[e] = kp;
                p.kept_prefix[e] = carry + incl - kp;
                p.offsets[e] = off;
                s_off[e] = off;
            }
            carry += __shfl(incl, kWave - 1, kWave);
        }
        if (lane == 0) {
            p.kept_prefix[E] = carry;
            p.offsets[E] = s.padded ? E * C : carry;
            p.meta[META_FINAL_ROWS] = s.padded ? E * C : carry;
            p.meta[META_R] = carry;
            p.meta[META_C] = C;
        }
    }
    __syncthreads();
    // C: per (unit, expert) block sizes and FINAL bases
    const int UE = s.U * E;
    for (int i = tid; i < UE; i += blockDim.x) {
        const int uu = i / E, e = i - uu * E;
        const int base = p.block_base[(size_t)uu * s.bpu * E + e];
        const int next = (uu + 1 < s.U) ? p.block_base[(size_t)(uu + 1) * s.bpu * E + e] : s_cnt[e];
        const int lo = base < C ? base : C, hi = next < C ? next : C;
        p.n[i] = hi - lo;
        p.unit_base[i] = s_off[e] + lo;
    }
    __syncthreads();
    // D: STAGE block offsets = exclusive scan of n in (unit, expert) order; unit starts; per-destination rows
    if (wave == 0) {
        int carry = 0;
        for (int i0 = 0; i0 < UE; i0 += kWave) {
            const int i = i0 + lane;
            const int v = i < UE ? p.n[i] : 0;
            const int incl = wave_inclusive_scan(v, lane);
            if (i < UE) {
                const int off = carry + incl - v;
                p.stage_off[i] = off;
                if (i % E == 0) p.unit_rows[i / E] = off;
            }
            carry += __shfl(incl, kWave - 1, kWave);
        }
        if (lane == 0) p.unit_rows[s.U] = carry;
    }
    const int E_loc = E / s.ep;
    for (int i = tid; i < s.U * s.ep; i += blockDim.x) {
        const int uu = i / s.ep, d = i - uu * s.ep;
        int sum = 0;
        for (int el = 0; el < E_loc; ++el) sum += p.n[uu * E + d * E_loc + el];
        p.send_rows[i] = sum;
    }
    if (tid == 0) p.meta[META_DONE] = 0;   // ready for the next call
}

// Finishes the plan: one lane per token turns (rank inside workgroup, workgroup base)
// into the global stable rank, applies the capacity and writes the pair's rows in
// FINAL and STAGE plus the STAGE->FINAL row map used by the regather copy.
__global__ __launch_bounds__(256) void positions_kernel(const int32_t *__restrict__ topk_idx, PlanPtrs p, Shape s)
{
    const int t = blockIdx.x * blockDim.x + threadIdx.x;
    bool any = false;
    if (t < s.T) {
        const int E = s.E, k = s.k;
        const int u = t / s.Tu;
        const int b = u * s.bpu + (t - u * s.Tu) / s.TB;
        const int32_t *bb = p.block_base + (size_t)b * E;
        const int32_t *ub = p.block_base + (size_t)u * s.bpu * E;
        for (int j = 0; j < k; ++j) {
            const int e = topk_idx[(size_t)t * k + j];
            const int r = bb[e] + p.local_rank[(size_t)t * k + j];
            int pf = -1, ps = -1;
            if (r < s.C) {
                pf = p.offsets[e] + r;
                ps = p.stage_off[u * E + e] + (r - ub[e]);
                // always true for tables built by route_plan_kernel; guards a workspace that was never initialised
                if ((unsigned)pf < (unsigned)s.max_rows && (unsigned)ps < (unsigned)s.max_rows) {
                    p.row_map[ps] = pf;
                    any = true;
                } else {
                    pf = ps = -1;
                }
            }
            p.pos_final[(size_t)t * k + j] = pf;
            p.pos_stage[(size_t)t * k + j] = ps;
        }
    }
    const unsigned long long m = __ballot(any);
    if ((threadIdx.x & (kWave - 1)) == 0 && m) atomicAdd(&p.meta[META_ALIVE], __popcll(m));
}

// Shared-memory result of rebuilding the scans for one route workgroup b (see block_plan).
struct BlockPlan {
    int before[256];   // P[u][e]: pairs of expert e in units before b's unit
    int unit[256];     // pairs of e in b's unit
    int pre[256];      // pairs of e in b's unit, in workgroups before b
    int total[256];    // counts[e]
    int off[256];      // offsets[e]: first FINAL row of expert e
    int kpre[256];     // exclusive scan of the kept counts (= off when the layout is compact)
    int stage[256];    // stage_off[u][e]: first STAGE row of block (u, e)
    int alive[256];    // per token of the workgroup: has a kept pair (plan_positions_block)
    int R, unit_row0;
};

// One lane's share of the histogram-table reduction of block_plan: the counters of expert e in blocks bl, bl + bstep,
// ..., LD loads requested before any is added up.
struct BlockSums {
    int total, before, unit, pre;
};
template <int LD>
__device__ __forceinline__ BlockSums sum_blocks(const int32_t *__restrict__ block_counts, int E, int e, int bl, int bstep,
                                                int nblk, int b, int first, int last)
{
    BlockSums a = {0, 0, 0, 0};
    for (int bb0 = bl; bb0 < nblk; bb0 += bstep * LD) {
        int cnt[LD];
#pragma unroll
        for (int q = 0; q < LD; ++q) {
            const int bb = bb0 + q * bstep;
            cnt[q] = bb < nblk ? block_counts[(size_t)bb * E + e] : 0;
        }
#pragma unroll
        for (int q = 0; q < LD; ++q) {
            const int bb = bb0 + q * bstep;
            const int c = cnt[q];
            a.total += c;
            if (bb < first) a.before += c;
            else if (bb < last) {
                a.unit += c;
                if (bb < b) a.pre += c;
            }
        }
    }
    return a;
}

// Every workgroup that calls this re-reads the whole [num_blocks][E] histogram table (a few KiB,
// L2 resident) and reduces it to four sums per expert; two wave scans over the experts then give
// the expert offsets and the unit's STAGE block offsets, using the telescoped form
//   sum_{u' < u} n[u'][e] = min(P[u][e], C),  P[u][e] = pairs of e before unit u,
// so no table over all units is needed.  There is no serial tail and no ticket; the price is the
// redundant table read.  All threads of the workgroup must call it; it ends with a barrier.
__device__ __forceinline__ void block_plan(BlockPlan &bp, int b, const PlanPtrs &p, const Shape &s)
{
    const int E = s.E, C = s.C;
    const int tid = threadIdx.x, lane = tid & (kWave - 1), wave = tid >> 6;
    const int u = b / s.bpu;
    for (int e = tid; e < E; e += blockDim.x)
        bp.before[e] = bp.unit[e] = bp.pre[e] = bp.total[e] = 0;
    __syncthreads();
    {
        const int total = s.num_blocks * E;
        const int first = u * s.bpu, last = first + s.bpu;     // blocks of this unit: [first, last)
        const int nthr = blockDim.x;
        if (nthr % E == 0) {
            // A lane meets one expert only and sums in registers, with one LDS update at the end.  The table
            // sits in the L2: a load costs hundreds of cycles, so a lane asks for LD of its counters at a time
            // before it adds any of them up (one at a time the loop is a chain of L2 round trips; measured on a
            // table of 256 x 64 counters the kernel takes 26 us this way against 32 us).  Small tables take the
            // plain loop, which needs fewer registers.
            const int e = tid % E;
            const int bl = tid / E, bstep = nthr / E;            // this lane's first block and its stride
            const int nblk = s.num_blocks;
            const BlockSums a = nblk > 4 * bstep
                                    ? sum_blocks<16>(p.block_counts, E, e, bl, bstep, nblk, b, first, last)
                                    : sum_blocks<1>(p.block_counts, E, e, bl, bstep, nblk, b, first, last);
            if (a.total) atomicAdd(&bp.total[e], a.total);
            if (a.before) atomicAdd(&bp.before[e], a.before);
            if (a.unit) atomicAdd(&bp.unit[e], a.unit);
            if (a.pre) atomicAdd(&bp.pre[e], a.pre);
        } else {
            for (int i = tid; i < total; i += nthr) {
                const int bb = i / E, e = i - bb * E;
                const int c = p.block_counts[i];
                if (c == 0) continue;
                atomicAdd(&bp.total[e], c);
                if (bb < first) atomicAdd(&bp.before[e], c);
                else if (bb < last) {
                    atomicAdd(&bp.unit[e], c);
                    if (bb < b) atomicAdd(&bp.pre[e], c);
                }
            }
        }
    }
    __syncthreads();
    if (wave == 0) {
        int carry_off = 0, carry_stage = 0;
        int base_u = 0;     // sum over experts of min(P[u][e], C): first STAGE row of the unit
        for (int e0 = 0; e0 < E; e0 += kWave) {
            const int e = e0 + lane;
            const int v = e < E ? (bp.before[e] < C ? bp.before[e] : C) : 0;
            const int incl = wave_inclusive_scan(v, lane);
            base_u += __shfl(incl, kWave - 1, kWave);
        }
        for (int e0 = 0; e0 < E; e0 += kWave) {
            const int e = e0 + lane;
            int kp = 0, nu = 0;
            if (e < E) {
                const int cnt = bp.total[e];
                kp = cnt < C ? cnt : C;
                const int lo = bp.before[e] < C ? bp.before[e] : C;
                const int nxt = bp.before[e] + bp.unit[e];
                nu = (nxt < C ? nxt : C) - lo;
            }
            const int incl_off = wave_inclusive_scan(kp, lane);
            const int incl_st = wave_inclusive_scan(nu, lane);
            if (e < E) {
                bp.kpre[e] = carry_off + incl_off - kp;
                bp.off[e] = s.padded ? e * C : carry_off + incl_off - kp;
                bp.stage[e] = base_u + carry_stage + incl_st - nu;
            }
            carry_off += __shfl(incl_off, kWave - 1, kWave);
            carry_stage += __shfl(incl_st, kWave - 1, kWave);
        }
        if (lane == 0) {
            bp.R = carry_off;
            bp.unit_row0 = base_u;
        }
    }
    __syncthreads();
}

// STAGE and FINAL rows of one pair from the rebuilt scans; false if the pair is dropped.
__device__ __forceinline__ bool place_pair(const BlockPlan &bp, const Shape &s, int e, int local_rank, int &pf, int &ps)
{
    const int in_unit = bp.pre[e] + local_rank;     // rank among the unit's pairs of expert e
    const int r = bp.before[e] + in_unit;           // global stable rank
    pf = ps = -1;
    if (r >= s.C) return false;
    pf = bp.off[e] + r;
    ps = bp.stage[e] + in_unit;
    // always true for a consistent histogram table; guards a workspace that was never initialised
    if ((unsigned)pf < (unsigned)s.max_rows && (unsigned)ps < (unsigned)s.max_rows) return true;
    pf = ps = -1;
    return false;
}

// Plan + positions in one pass, for problems whose histogram table is small: workgroup b owns the
// tokens of route workgroup b, rebuilds the scans (block_plan) and writes its tokens' positions.
// The first workgroup of each unit writes that unit's rows of the public tables; workgroup 0
// writes the per-expert ones.
__device__ __forceinline__ void plan_positions_block(BlockPlan &bp, int b, const int32_t *__restrict__ topk_idx,
                                                     const PlanPtrs &p, const Shape &s)
{
    constexpr int PRE = 8;      // pairs per lane fetched before the table reduction, to overlap their latency
    const int E = s.E, k = s.k, C = s.C;
    const int tid = threadIdx.x, lane = tid & (kWave - 1);
    const int u = b / s.bpu, ib = b - u * s.bpu;
    const int t_begin = u * s.Tu + ib * s.TB;
    int nt = s.Tu - ib * s.TB;
    if (nt > s.TB) nt = s.TB;
    // One (token, choice) pair per lane and pass, in the tables' own order: loads and stores of the per-pair
    // tables are contiguous across the lanes.
    const int npairs = nt * k, nthr = blockDim.x;
    const size_t pair0 = (size_t)t_begin * k;

    int e_pre[PRE], r_pre[PRE];
#pragma unroll
    for (int q = 0; q < PRE; ++q) {
        e_pre[q] = 0;
        r_pre[q] = 0;
        const int idx = tid + q * nthr;
        if (idx < npairs) {
            e_pre[q] = topk_idx[pair0 + idx];
            r_pre[q] = p.local_rank[pair0 + idx];
        }
    }
    for (int i = tid; i < s.TB; i += nthr) bp.alive[i] = 0;      // block_plan's barriers order this before its use
    block_plan(bp, b, p, s);

    for (int e = tid; e < E; e += blockDim.x) {
        if (ib == 0) {      // first workgroup of the unit publishes the unit's rows
            const int lo = bp.before[e] < C ? bp.before[e] : C;
            const int nxt = bp.before[e] + bp.unit[e];
            p.n[u * E + e] = (nxt < C ? nxt : C) - lo;
            p.stage_off[u * E + e] = bp.stage[e];
            p.unit_base[u * E + e] = bp.off[e] + lo;
        }
        if (b == 0) {
            p.counts[e] = bp.total[e];
            p.kept[e] = bp.total[e] < C ? bp.total[e] : C;
            p.offsets[e] = bp.off[e];
            p.kept_prefix[e] = bp.kpre[e];
        }
    }
    if (tid == 0) {
        if (ib == 0) p.unit_rows[u] = bp.unit_row0;
        if (b == 0) {
            p.offsets[E] = s.padded ? E * C : bp.R;
            p.kept_prefix[E] = bp.R;
            p.unit_rows[s.U] = bp.R;
            p.meta[META_R] = bp.R;
            p.meta[META_FINAL_ROWS] = s.padded ? E * C : bp.R;
            p.meta[META_C] = C;
        }
    }
    if (ib == 0) {
        const int E_loc = E / s.ep;
        for (int d = tid; d < s.ep; d += blockDim.x) {
            // rows for EP rank d = STAGE span of its experts inside this unit
            const int first_e = d * E_loc, end_e = first_e + E_loc;
            const int begin = bp.stage[first_e];
            int end;
            if (end_e < E) end = bp.stage[end_e];
            else {
                const int eL = E - 1;
                const int lo = bp.before[eL] < C ? bp.before[eL] : C;
                const int nxt = bp.before[eL] + bp.unit[eL];
                end = bp.stage[eL] + ((nxt < C ? nxt : C) - lo);
            }
            p.send_rows[u * s.ep + d] = end - begin;
        }
    }

    auto place = [&](int idx, int e, int lr) {
        int pf, ps;
        if (place_pair(bp, s, e, lr, pf, ps)) {
            p.row_map[ps] = pf;
            bp.alive[idx / k] = 1;
        }
        p.pos_final[pair0 + idx] = pf;
        p.pos_stage[pair0 + idx] = ps;
    };
#pragma unroll
    for (int q = 0; q < PRE; ++q) {
        const int idx = tid + q * nthr;
        if (idx < npairs) place(idx, e_pre[q], r_pre[q]);
    }
    for (int idx = tid + PRE * nthr; idx < npairs; idx += nthr) place(idx, topk_idx[pair0 + idx], p.local_rank[pair0 + idx]);
    __syncthreads();
    // tokens with a kept pair
    for (int i0 = 0; i0 < nt; i0 += nthr) {
        const int i = i0 + tid;
        const unsigned long long m = __ballot(i < nt && bp.alive[i] != 0);
        if (lane == 0 && m) atomicAdd(&p.meta[META_ALIVE], __popcll(m));
    }
}

__global__ __launch_bounds__(256) void plan_positions_kernel(const int32_t *__restrict__ topk_idx, PlanPtrs p, Shape s)
{
    __shared__ BlockPlan bp;
    plan_positions_block(bp, blockIdx.x, topk_idx, p, s);
}

__global__ void ws_init_kernel(int32_t *meta)
{
    if (threadIdx.x < META_SLOTS) meta[threadIdx.x] = 0;
}

// --------------------------------------------------------------- row movers

// Tokens [t0, t0+nt): each token row is read once and written to the STAGE row of
// every kept choice (read once / write up to k).  `lpr` lanes share a row.
template <bool NTL, bool NTS>
__device__ __forceinline__ void pack_rows_t(const u32x4 *__restrict__ x, u32x4 *__restrict__ stage,
                                          const int32_t *__restrict__ pos_stage, const Shape &s, int t0,
                                          int nt, int wg, int nwg)
{
    const int lpr = s.lpr, vpr = s.vpr, k = s.k;
    const int rows_per_wg = kMoverThreads / lpr;
    const int sub = threadIdx.x / lpr, lane = threadIdx.x - sub * lpr;
    for (int i = wg * rows_per_wg + sub; i < nt; i += nwg * rows_per_wg) {
        const int t = t0 + i;
        const int32_t *pos = pos_stage + (size_t)t * k;
        const u32x4 *src = x + (size_t)t * vpr;
        // The first pass of the row is requested before the positions are looked at: the two latencies overlap
        // instead of adding up.  The price is the row of a token whose choices were all dropped, read in vain
        // (a few percent of the tokens of a workload with heavy drops, none otherwise).
        u32x4 val[kVecInFlight];
#pragma unroll
        for (int q = 0; q < kVecInFlight; ++q)
            if (lane + q * lpr < vpr) val[q] = ld16<NTL>(src + lane + q * lpr);
        bool any = false;
        for (int j = 0; j < k; ++j) any |= (unsigned)pos[j] < (unsigned)s.max_rows;
        if (!any) continue;                 // every choice of this token was dropped
        for (int v0 = lane; v0 < vpr; v0 += lpr * kVecInFlight) {
            if (v0 != lane) {
#pragma unroll
                for (int q = 0; q < kVecInFlight; ++q)
                    if (v0 + q * lpr < vpr) val[q] = ld16<NTL>(src + v0 + q * lpr);
            }
            for (int j = 0; j < k; ++j) {
                const int ps = pos[j];
                if ((unsigned)ps >= (unsigned)s.max_rows) continue;   // dropped (-1) or not a row
                u32x4 *dst = stage + (size_t)ps * vpr;
#pragma unroll
                for (int q = 0; q < kVecInFlight; ++q)
                    if (v0 + q * lpr < vpr) st16<NTS>(dst + v0 + q * lpr, val[q]);
            }
        }
    }
}

__device__ __forceinline__ void pack_rows(const u32x4 *__restrict__ x, u32x4 *__restrict__ stage,
                                          const int32_t *__restrict__ pos_stage, const Shape &s, int t0,
                                          int nt, int wg, int nwg)
{
    with_policy(s.cache & NT_PACK_LD, s.cache & NT_PACK_ST, [&](auto l, auto st) {
        pack_rows_t<decltype(l)::value, decltype(st)::value>(x, stage, pos_stage, s, t0, nt, wg, nwg);
    });
}

// STAGE rows [r0, r1) go to FINAL rows row_map[.], walked in STAGE order: the reads are one contiguous run, the
// writes one run per (unit, expert) block.  (Walking a slice's rows expert by expert instead, so that the writes
// of neighbouring workgroups are neighbours, needs a second lookup per row and measured slower on three of four
// large workloads, 2 % faster on one.)
// REVERSE: the other direction (the mirrored return path): row row_map[r] of `fin` goes to row r of `stage`.
template <bool REVERSE, bool NTL, bool NTS>
__device__ __forceinline__ void regather_rows_t(u32x4 *stage, u32x4 *fin, const int32_t *__restrict__ row_map,
                                                const Shape &s, int r0, int r1, int wg, int nwg)
{
    const int lpr = s.lpr, vpr = s.vpr;
    const int rows_per_wg = kMoverThreads / lpr;
    const int sub = threadIdx.x / lpr, lane = threadIdx.x - sub * lpr;
    if (r0 < 0) r0 = 0;
    if (r1 > s.max_rows) r1 = s.max_rows;
    for (int r = r0 + wg * rows_per_wg + sub; r < r1; r += nwg * rows_per_wg) {
        u32x4 val[kVecInFlight];
        if (!REVERSE) {
            // forward: the source row does not depend on the table, so its first pass is requested before the
            // destination is looked up
            const u32x4 *src0 = stage + (size_t)r * vpr;
#pragma unroll
            for (int q = 0; q < kVecInFlight; ++q)
                if (lane + q * lpr < vpr) val[q] = ld16<NTL>(src0 + lane + q * lpr);
        }
        const int fr = row_map[r];
        if ((unsigned)fr >= (unsigned)s.max_rows) continue;
        const u32x4 *src = REVERSE ? fin + (size_t)fr * vpr : stage + (size_t)r * vpr;
        u32x4 *dst = REVERSE ? stage + (size_t)r * vpr : fin + (size_t)fr * vpr;
        for (int v0 = lane; v0 < vpr; v0 += lpr * kVecInFlight) {
            if (REVERSE || v0 != lane) {
#pragma unroll
                for (int q = 0; q < kVecInFlight; ++q)
                    if (v0 + q * lpr < vpr) val[q] = ld16<NTL>(src + v0 + q * lpr);
            }
#pragma unroll
            for (int q = 0; q < kVecInFlight; ++q)
                if (v0 + q * lpr < vpr) st16<NTS>(dst + v0 + q * lpr, val[q]);
        }
    }
}

// Capacity-padded layout: zero-fills the padding rows [e*C + kept[e], (e+1)*C) of every expert.  Padding row i
// (0 <= i < E*C - R) belongs to the expert found by bisection over pad_before[e] = e*C - kept_prefix[e].
__device__ __forceinline__ void pad_rows(u32x4 *__restrict__ fin, const PlanPtrs &p, const Shape &s, int wg, int nwg)
{
    const int lpr = s.lpr, vpr = s.vpr, E = s.E, C = s.C;
    const int rows_per_wg = kMoverThreads / lpr;
    const int sub = threadIdx.x / lpr, lane = threadIdx.x - sub * lpr;
    int total = E * C - p.kept_prefix[E];
    if (total > s.max_rows) total = s.max_rows;
    const u32x4 zero = {0u, 0u, 0u, 0u};
    for (int i = wg * rows_per_wg + sub; i < total; i += nwg * rows_per_wg) {
        int lo = 0, hi = E - 1;                      // largest e with pad_before[e] <= i
        while (lo < hi) {
            const int mid = (lo + hi + 1) >> 1;
            if (mid * C - p.kept_prefix[mid] <= i) lo = mid;
            else hi = mid - 1;
        }
        const int row = lo * C + p.kept[lo] + (i - (lo * C - p.kept_prefix[lo]));
        if ((unsigned)row >= (unsigned)s.max_rows || row >= (lo + 1) * C) continue;
        u32x4 *dst = fin + (size_t)row * vpr;
        for (int v = lane; v < vpr; v += lpr) st16<true>(dst + v, zero);
    }
}

__device__ __forceinline__ void regather_rows(const u32x4 *__restrict__ stage, u32x4 *__restrict__ fin,
                                              const PlanPtrs &p, const Shape &s, int r0, int r1, int wg, int nwg)
{
    with_policy(s.cache & NT_REG_LD, s.cache & NT_REG_ST, [&](auto l, auto st) {
        regather_rows_t<false, decltype(l)::value, decltype(st)::value>(const_cast<u32x4 *>(stage), fin, p.row_map, s, r0,
                                                                        r1, wg, nwg);
    });
}

// the mirrored direction: expert output y (FINAL layout) back to the unit-major layout
__device__ __forceinline__ void unregather_rows(const u32x4 *__restrict__ y, u32x4 *__restrict__ y_stage,
                                                const int32_t *__restrict__ row_map, const Shape &s, int r0,
                                                int r1, int wg, int nwg)
{
    with_policy(s.cache & NT_REG_LD, s.cache & NT_REG_ST, [&](auto l, auto st) {
        regather_rows_t<true, decltype(l)::value, decltype(st)::value>(y_stage, const_cast<u32x4 *>(y), row_map, s, r0, r1,
                                                                       wg, nwg);
    });
}

// pack for tokens whose positions have not been written yet: the workgroup rebuilds the scans of
// the route workgroup its tokens belong to (all of them belong to one: the host checks the shape)
// and derives the STAGE rows itself.  The first pass of every row is loaded before the rebuild, so
// the table read overlaps the row read.  Writes no table: plan_positions_block does that.
template <bool NTL, bool NTS>
__device__ __forceinline__ void pack_rows_selfplan_t(BlockPlan &bp, const u32x4 *__restrict__ x,
                                                     u32x4 *__restrict__ stage, const int32_t *__restrict__ topk_idx,
                                                     const PlanPtrs &p, const Shape &s, int t0, int nt, int wg)
{
    const int lpr = s.lpr, vpr = s.vpr, k = s.k;
    const int rows_per_wg = kMoverThreads / lpr;
    const int sub = threadIdx.x / lpr, lane = threadIdx.x - sub * lpr;
    const int i = wg * rows_per_wg + sub;
    const bool have = i < nt;
    const int t = t0 + (have ? i : 0);
    const int t_first = t0 + wg * rows_per_wg;                  // same route workgroup for the whole group
    const int u = t_first / s.Tu;
    const int b = u * s.bpu + (t_first - u * s.Tu) / s.TB;
    const u32x4 *src = x + (size_t)t * vpr;
    u32x4 val[kVecInFlight];
#pragma unroll
    for (int q = 0; q < kVecInFlight; ++q)
        if (have && lane + q * lpr < vpr) val[q] = ld16<NTL>(src + lane + q * lpr);
    block_plan(bp, b, p, s);
    if (!have) return;
    for (int v0 = lane; v0 < vpr; v0 += lpr * kVecInFlight) {
        if (v0 != lane) {
#pragma unroll
            for (int q = 0; q < kVecInFlight; ++q)
                if (v0 + q * lpr < vpr) val[q] = ld16<NTL>(src + v0 + q * lpr);
        }
        for (int j = 0; j < k; ++j) {
            int pf, ps;
            if (!place_pair(bp, s, topk_idx[(size_t)t * k + j], p.local_rank[(size_t)t * k + j], pf, ps)) continue;
            u32x4 *dst = stage + (size_t)ps * vpr;
#pragma unroll
            for (int q = 0; q < kVecInFlight; ++q)
                if (v0 + q * lpr < vpr) st16<NTS>(dst + v0 + q * lpr, val[q]);
        }
    }
}

// One grid, two jobs: the first n_plan workgroups finish the plan (tables and positions of every
// token), the others pack slice 0 with positions they derive themselves, so the first pack does
// not wait for the plan kernel.
__global__ __launch_bounds__(kMoverThreads) void plan_pack_kernel(const int32_t *__restrict__ topk_idx,
                                                                  const u32x4 *__restrict__ x,
                                                                  u32x4 *__restrict__ stage, PlanPtrs p, Shape s,
                                                                  int t0, int nt, int n_plan)
{
    __shared__ BlockPlan bp;
    const int bid = blockIdx.x;
    if (bid < n_plan) {
        plan_positions_block(bp, bid, topk_idx, p, s);
        return;
    }
    with_policy(s.cache & NT_PACK_LD, s.cache & NT_PACK_ST, [&](auto l, auto st) {
        pack_rows_selfplan_t<decltype(l)::value, decltype(st)::value>(bp, x, stage, topk_idx, p, s, t0, nt,
                                                                      bid - n_plan);
    });
}

__global__ __launch_bounds__(kMoverThreads) void pack_kernel(const u32x4 *__restrict__ x, u32x4 *__restrict__ stage,
                                                             PlanPtrs p, Shape s, int t0, int nt)
{
    pack_rows(x, stage, p.pos_stage, s, t0, nt, blockIdx.x, gridDim.x);
}

// u0, u1: unit range whose STAGE rows are moved (row range read from the device table)
__global__ __launch_bounds__(kMoverThreads) void regather_kernel(const u32x4 *__restrict__ stage,
                                                                 u32x4 *__restrict__ fin, PlanPtrs p, Shape s,
                                                                 int u0, int u1)
{
    regather_rows(stage, fin, p, s, p.unit_rows[u0], p.unit_rows[u1], blockIdx.x, gridDim.x);
    if (s.padded && u0 == 0) pad_rows(fin, p, s, blockIdx.x, gridDim.x);
}

// One grid, two jobs in disjoint workgroups: the first n_pack_wg workgroups pack
// slice j (tokens [t0, t0+nt)), the others regather slice j-1 (units [u0, u1)).
// The two touch disjoint rows of STAGE, so they may run in any interleaving.
__global__ __launch_bounds__(kMoverThreads) void pack_regather_kernel(const u32x4 *__restrict__ x,
                                                                      u32x4 *__restrict__ stage,
                                                                      u32x4 *__restrict__ fin, PlanPtrs p, Shape s,
                                                                      int t0, int nt, int u0, int u1, int n_pack_wg)
{
    // interleave the two jobs over the grid so that both make progress from the start
    const int n_reg_wg = gridDim.x - n_pack_wg;
    const int bid = blockIdx.x;
    const int pairs = n_pack_wg < n_reg_wg ? n_pack_wg : n_reg_wg;
    bool is_pack;
    int idx;
    if (bid < 2 * pairs) {
        is_pack = (bid & 1) == 0;
        idx = bid >> 1;
    } else {
        is_pack = n_pack_wg > n_reg_wg;
        idx = bid - pairs;
    }
    if (is_pack)
        pack_rows(x, stage, p.pos_stage, s, t0, nt, idx, n_pack_wg);
    else
{
        regather_rows(stage, fin, p, s, p.unit_rows[u0], p.unit_rows[u1], idx, n_reg_wg);
        if (s.padded && u0 == 0) pad_rows(fin, p, s, idx, n_reg_wg);
    }
}

// ------------------------------------------------------------------ combine

__device__ __forceinline__ double bf16_lo(unsigned int w) { return (double)__uint_as_float(w << 16); }
__device__ __forceinline__ double bf16_hi(unsigned int w) { return (double)__uint_as_float(w & 0xffff0000u); }

// fp64 -> bf16 bits with ONE rounding (nearest, ties to even).  The value first goes to fp32 (nearest-even, one
// hardware conversion).  Rounding is monotone and every midpoint between two bf16 values is an fp32 number, so
// unless the fp32 value IS such a midpoint (low 16 bits 0x8000) it lies on the same side of every midpoint as
// the fp64 value, and rounding it to nearest gives the fp64 value's bf16: add 0x8000 and drop the low half.
// Only in the midpoint case (one in 65536) the fp32 step may have hidden on which side the fp64 value lay: the
// slow branch compares the two and rounds down, up, or (a true tie) to even.  Overflow, underflow and
// infinities fall out of the same arithmetic; NaN is mapped to the canonical quiet NaN.
__device__ __forceinline__ unsigned int f64_to_bf16_rne(double d)
{
    const float f = (float)d;                       // nearest-even
    const unsigned int u = __float_as_uint(f);
    unsigned int r = (u + 0x8000u) >> 16;
    if (__builtin_expect((u & 0xffffu) == 0x8000u, 0)) {
        const double back = (double)f;
        if (back == d) r = (u + 0x7fffu + ((u >> 16) & 1u)) >> 16;                 // true tie: to even
        else if (__builtin_fabs(back) > __builtin_fabs(d)) r = u >> 16;            // below the midpoint
        else r = (u >> 16) + 1u;                                                   // above it
    }
    return f != f ? 0x7fc0u : r;
}

// out[t] = sum_j gate[t,j] * y[pos_final[t,j]] over kept j in ascending order.
// The sum is carried in fp64 (every product of an fp32 gate with an fp32 / bf16
// element is exact there) and rounded once to the activation type, so the rounding
// decision is taken at the same precision as the CPU reference takes it; measured
// against a copy-only version of the same loop the arithmetic costs a few percent.
// NV 16-byte vectors per lane per pass: 2 covers rows up to 8 KiB in one pass, 4 up
// to 16 KiB.  Tokens are walked from the last to the first: the FINAL rows written
// most recently (by the last slices) are read first, while the memory-side cache
// still holds them.  A dropped pair is skipped; a token with no kept pair writes zeros.
// `pos_table` is pos_final (y in FINAL layout) or pos_stage (y in the unit-major layout of the mirrored
// return path); tokens [t0, t0+nt) are combined by workgroups wg of nwg.
template <bool BF16, int NV, bool NTL, bool NTS>
__device__ __forceinline__ void combine_rows_t(const u32x4 *__restrict__ y, const float *__restrict__ gates,
                                               u32x4 *__restrict__ out, const int32_t *__restrict__ pos_table,
                                               const Shape &s, int t0, int nt, int wg, int nwg)
{
    constexpr int NF = BF16 ? 8 : 4;            // accumulators per vector
    const int lpr = s.lpr, vpr = s.vpr, k = s.k;
    const int rows_per_wg = kMoverThreads / lpr;
    const int sub = threadIdx.x / lpr, lane = threadIdx.x - sub * lpr;
    for (int i = wg * rows_per_wg + sub; i < nt; i += nwg * rows_per_wg) {
        const int t = t0 + nt - 1 - i;
        const int32_t *pos = pos_table + (size_t)t * k;
        const float *g = gates + (size_t)t * k;
        u32x4 *dst = out + (size_t)t * vpr;
        for (int v0 = lane; v0 < vpr; v0 += lpr * NV) {
            double acc[NV][NF];
#pragma unroll
            for (int q = 0; q < NV; ++q)
#pragma unroll
                for (int f = 0; f < NF; ++f) acc[q][f] = 0.0;
            for (int j = 0; j < k; ++j) {
                const int pf = pos[j];
                if ((unsigned)pf >= (unsigned)s.max_rows) continue;   // dropped (-1) or not a row
                const double gj = (double)g[j];
                const u32x4 *src = y + (size_t)pf * vpr;
                u32x4 val[NV];
#pragma unroll
                for (int q = 0; q < NV; ++q)
                    if (v0 + q * lpr < vpr) val[q] = ld16<NTL>(src + v0 + q * lpr);
#pragma unroll
                for (int q = 0; q < NV; ++q) {
                    if (v0 + q * lpr < vpr) {
#pragma unroll
                        for (int c = 0; c < 4; ++c) {
                            if (BF16) {
                                acc[q][2 * c] = __builtin_fma(gj, bf16_lo(val[q][c]), acc[q][2 * c]);
                                acc[q][2 * c + 1] = __builtin_fma(gj, bf16_hi(val[q][c]), acc[q][2 * c + 1]);
                            } else {
                                acc[q][c] = __builtin_fma(gj, (double)__uint_as_float(val[q][c]), acc[q][c]);
                            }
                        }
                    }
                }
            }
#pragma unroll
            for (int q = 0; q < NV; ++q) {
                if (v0 + q * lpr < vpr) {
                    u32x4 o;
#pragma unroll
                    for (int c = 0; c < 4; ++c) {
                        if (BF16)
                            o[c] = f64_to_bf16_rne(acc[q][2 * c]) | (f64_to_bf16_rne(acc[q][2 * c + 1]) << 16);
                        else
                            o[c] = __float_as_uint((float)acc[q][c]);
                    }
                    st16<NTS>(dst + v0 + q * lpr, o);
                }
            }
        }
    }
}

// The same scale-add with the row reads software-pipelined.  One wave's time on a token is a chain of
// memory latencies: position and gate of choice j, then the row they point to, then the next choice.  Here
// the first k lanes of a row's lane group fetch the token's k positions and gates in one go (a ballot of
// their validity gives the kept choices as a bit mask, shuffles hand each one to all lanes), and the row of
// the next kept choice is requested before the current one is added, so two rows' loads are in flight per
// lane and the fp64 arithmetic runs under them.  Needs k <= lanes per row (the host checks).  Same order of
// additions, same result.
template <bool BF16, int NV, bool NTL, bool NTS>
__device__ __forceinline__ void combine_rows_pf_t(const u32x4 *__restrict__ y, const float *__restrict__ gates,
                                                  u32x4 *__restrict__ out, const int32_t *__restrict__ pos_table,
                                                  const Shape &s, int t0, int nt, int wg, int nwg)
{
    constexpr int NF = BF16 ? 8 : 4;            // accumulators per vector
    const int lpr = s.lpr, vpr = s.vpr, k = s.k;
    const int rows_per_wg = kMoverThreads / lpr;
    const int sub = threadIdx.x / lpr, lane = threadIdx.x - sub * lpr;
    const int wl = threadIdx.x & (kWave - 1);
    const int gbase = lpr >= kWave ? 0 : (wl & ~(lpr - 1));     // first lane, inside the wave, of this lane's row group
    const int gl = wl - gbase;                                  // this lane's index in it
    const unsigned int kmask = k >= 32 ? 0xffffffffu : ((1u << k) - 1u);
    for (int i = wg * rows_per_wg + sub; i < nt; i += nwg * rows_per_wg) {
        const int t = t0 + nt - 1 - i;
        u32x4 *dst = out + (size_t)t * vpr;
        int my_pos = -1;
        float my_g = 0.f;
        if (gl < k) {
            my_pos = pos_table[(size_t)t * k + gl];
            my_g = gates[(size_t)t * k + gl];
        }
        const unsigned long long valid = __ballot((unsigned)my_pos < (unsigned)s.max_rows);
        const unsigned int kept = (unsigned int)(valid >> gbase) & kmask;      // bit j: choice j of this token is kept
        // every lane of the group walks every pass, also lanes past the end of a short row: the shuffles below
        // read the positions from the group's first k lanes, which must therefore stay active
        for (int vbase = 0; vbase < vpr; vbase += lpr * NV) {
            const int v0 = vbase + lane;
            double acc[NV][NF];
#pragma unroll
            for (int q = 0; q < NV; ++q)
#pragma unroll
                for (int f = 0; f < NF; ++f) acc[q][f] = 0.0;
            unsigned int rem = kept;
            u32x4 cur[NV];
            float g_cur = 0.f;
            bool have = rem != 0;
            if (have) {
                const int j = __builtin_ctz(rem);
                rem &= rem - 1;
                const int pf = __shfl(my_pos, gbase + j, kWave);
                g_cur = __shfl(my_g, gbase + j, kWave);
                const u32x4 *src = y + (size_t)pf * vpr;
#pragma unroll
                for (int q = 0; q < NV; ++q)
                    if (v0 + q * lpr < vpr) cur[q] = ld16<NTL>(src + v0 + q * lpr);
            }
            while (have) {
                u32x4 nxt[NV];
                float g_nxt = 0.f;
                const bool have_nxt = rem != 0;
                if (have_nxt) {
                    const int j = __builtin_ctz(rem);
                    rem &= rem - 1;
                    const int pf = __shfl(my_pos, gbase + j, kWave);
                    g_nxt = __shfl(my_g, gbase + j, kWave);
                    const u32x4 *src = y + (size_t)pf * vpr;
#pragma unroll
                    for (int q = 0; q < NV; ++q)
                        if (v0 + q * lpr < vpr) nxt[q] = ld16<NTL>(src + v0 + q * lpr);
                }
                const double gj = (double)g_cur;
#pragma unroll
                for (int q = 0; q < NV; ++q) {
                    if (v0 + q * lpr < vpr) {
#pragma unroll
                        for (int c = 0; c < 4; ++c) {
                            if (BF16) {
                                acc[q][2 * c] = __builtin_fma(gj, bf16_lo(cur[q][c]), acc[q][2 * c]);
                                acc[q][2 * c + 1] = __builtin_fma(gj, bf16_hi(cur[q][c]), acc[q][2 * c + 1]);
                            } else {
                                acc[q][c] = __builtin_fma(gj, (double)__uint_as_float(cur[q][c]), acc[q][c]);
                            }
                        }
                    }
                }
#pragma unroll
                for (int q = 0; q < NV; ++q) cur[q] = nxt[q];
                g_cur = g_nxt;
                have = have_nxt;
            }
#pragma unroll
            for (int q = 0; q < NV; ++q) {
                if (v0 + q * lpr < vpr) {
                    u32x4 o;
#pragma unroll
                    for (int c = 0; c < 4; ++c) {
                        if (BF16)
                            o[c] = f64_to_bf16_rne(acc[q][2 * c]) | (f64_to_bf16_rne(acc[q][2 * c + 1]) << 16);
                        else
                            o[c] = __float_as_uint((float)acc[q][c]);
                    }
                    st16<NTS>(dst + v0 + q * lpr, o);
                }
            }
        }
    }
}

template <bool BF16, int NV>
__global__ __launch_bounds__(kMoverThreads) void combine_pf_kernel(const u32x4 *__restrict__ y,
                                                                   const float *__restrict__ gates,
                                                                   u32x4 *__restrict__ out, PlanPtrs p, Shape s)
{
    with_policy(s.cache & NT_COMB_LD, s.cache & NT_COMB_ST, [&](auto l, auto st) {
        combine_rows_pf_t<BF16, NV, decltype(l)::value, decltype(st)::value>(y, gates, out, p.pos_final, s, 0, s.T,
                                                                             blockIdx.x, gridDim.x);
    });
}

template <bool BF16, int NV>
__global__ __launch_bounds__(kMoverThreads) void combine_kernel(const u32x4 *__restrict__ y,
                                                                const float *__restrict__ gates,
                                                                u32x4 *__restrict__ out, PlanPtrs p, Shape s)
{
    with_policy(s.cache & NT_COMB_LD, s.cache & NT_COMB_ST, [&](auto l, auto st) {
        combine_rows_t<BF16, NV, decltype(l)::value, decltype(st)::value>(y, gates, out, p.pos_final, s, 0, s.T,
                                                                          blockIdx.x, gridDim.x);
    });
}

// The gather as a pass of its own: the STAGE rows of units [u0, u1) (one contiguous range, read from the
// device table) copied unchanged into a second buffer.
__device__ __forceinline__ void allgather_rows(const u32x4 *__restrict__ stage, u32x4 *__restrict__ gathered,
                                               const PlanPtrs &p, const Shape &s, int u0, int u1, int wg, int nwg)
{
    int r0 = p.unit_rows[u0], r1 = p.unit_rows[u1];
    if (r0 < 0) r0 = 0;
    if (r1 > s.max_rows) r1 = s.max_rows;
    if (r1 <= r0) return;
    const size_t first = (size_t)r0 * s.vpr, nvec = (size_t)(r1 - r0) * s.vpr;
    const size_t stride = (size_t)nwg * kMoverThreads * kVecInFlight;
    for (size_t base = (size_t)wg * kMoverThreads * kVecInFlight + threadIdx.x; base < nvec; base += stride) {
        u32x4 val[kVecInFlight];
#pragma unroll
        for (int q = 0; q < kVecInFlight; ++q)
            if (base + (size_t)q * kMoverThreads < nvec) val[q] = ld16<true>(stage + first + base + (size_t)q * kMoverThreads);
#pragma unroll
        for (int q = 0; q < kVecInFlight; ++q)
            if (base + (size_t)q * kMoverThreads < nvec) st16<false>(gathered + first + base + (size_t)q * kMoverThreads, val[q]);
    }
}

__global__ __launch_bounds__(kMoverThreads) void allgather_kernel(const u32x4 *__restrict__ stage,
                                                                  u32x4 *__restrict__ gathered, PlanPtrs p, Shape s,
                                                                  int u0, int u1)
{
    allgather_rows(stage, gathered, p, s, u0, u1, blockIdx.x, gridDim.x);
}

// The paper's third transform (paragraph "AllGather and D2D copy Pipelining", Fig. 8): while the D2D copy
// places chunk j from the gathered buffer, the gather of chunk j+1 already runs.  One grid, two jobs in
// disjoint, interleaved workgroups: the first n_gather_wg gather units [gu0, gu1) (STAGE -> gathered), the
// others copy units [cu0, cu1) from `gathered` to their index offsets in FINAL.  The two ranges are different
// chunks, so the jobs touch disjoint rows of `gathered`.
__global__ __launch_bounds__(kMoverThreads) void allgather_regather_kernel(const u32x4 *__restrict__ stage,
                                                                           u32x4 *gathered, u32x4 *__restrict__ fin,
                                                                           PlanPtrs p, Shape s, int gu0, int gu1,
                                                                           int cu0, int cu1, int n_gather_wg)
{
    const int n_copy_wg = gridDim.x - n_gather_wg;
    const int bid = blockIdx.x;
    const int pairs = n_gather_wg < n_copy_wg ? n_gather_wg : n_copy_wg;
    bool is_gather;
    int idx;
    if (bid < 2 * pairs) {
        is_gather = (bid & 1) == 0;
        idx = bid >> 1;
    } else {
        is_gather = n_gather_wg > n_copy_wg;
        idx = bid - pairs;
    }
    if (is_gather) {
        allgather_rows(stage, gathered, p, s, gu0, gu1, idx, n_gather_wg);
    } else {
        regather_rows(gathered, fin, p, s, p.unit_rows[cu0], p.unit_rows[cu1], idx, n_copy_wg);
        if (s.padded && cu0 == 0) pad_rows(fin, p, s, idx, n_copy_wg);
    }
}

// ---- the second AllToAll, mirrored: y (FINAL layout) -> unit-major layout -> token order, slice by slice

__global__ __launch_bounds__(kMoverThreads) void unregather_kernel(const u32x4 *__restrict__ y,
                                                                   u32x4 *__restrict__ y_stage, PlanPtrs p, Shape s,
                                                                   int u0, int u1)
{
    unregather_rows(y, y_stage, p.row_map, s, p.unit_rows[u0], p.unit_rows[u1], blockIdx.x, gridDim.x);
}

// One grid, up to two jobs in disjoint, interleaved workgroups: the unit-major rows of units [u0, u1)
// are fetched back from y (skipped if u0 >= u1) while the tokens [t0, t0+nt) of the slice before are
// combined from rows fetched by the previous launch (skipped if nt == 0).
// PF: the software-pipelined scale-add (three or more choices per token), as in combine_pf_kernel.
template <bool BF16, int NV, bool PF = false>
__global__ __launch_bounds__(kMoverThreads) void unregather_combine_kernel(const u32x4 *__restrict__ y,
                                                                           u32x4 *y_stage,
                                                                           const float *__restrict__ gates,
                                                                           u32x4 *__restrict__ out, PlanPtrs p,
                                                                           Shape s, int u0, int u1, int t0, int nt,
                                                                           int n_unreg_wg)
{
    const int n_comb_wg = gridDim.x - n_unreg_wg;
    const int bid = blockIdx.x;
    const int pairs = n_unreg_wg < n_comb_wg ? n_unreg_wg : n_comb_wg;
    bool is_unreg;
    int idx;
    if (bid < 2 * pairs) {
        is_unreg = (bid & 1) == 0;
        idx = bid >> 1;
    } else {
        is_unreg = n_unreg_wg > n_comb_wg;
        idx = bid - pairs;
    }
    if (is_unreg) {
        if (u0 < u1) unregather_rows(y, y_stage, p.row_map, s, p.unit_rows[u0], p.unit_rows[u1], idx, n_unreg_wg);
    } else if (nt > 0) {
        with_policy(s.cache & NT_COMB_LD, s.cache & NT_COMB_ST, [&](auto l, auto st) {
            if (PF)
                combine_rows_pf_t<BF16, NV, decltype(l)::value, decltype(st)::value>(y_stage, gates, out, p.pos_stage, s,
                                                                                     t0, nt, idx, n_comb_wg);
            else
                combine_rows_t<BF16, NV, decltype(l)::value, decltype(st)::value>(y_stage, gates, out, p.pos_stage, s, t0,
                                                                                  nt, idx, n_comb_wg);
        });
    }
}

// --------------------------------------------------------- gate projection
//
// logits[t][e] = sum_h x[t][h] * w[e][h]  (section "MoE": the gate is a linear layer ahead of softmax and TopK).
// The contraction is read-bound on x: every element of x is used E times, far below what the matrix cores
// need to be busy, so the kernel is laid out for the x stream and uses MFMA to keep the arithmetic off the
// critical path at large E.
//
// bf16: a workgroup of 8 waves owns 32*MT tokens and all experts.  The hidden axis is cut into steps of KS
// elements; a step's tile (the tokens' rows, then the experts' rows, KS*2 bytes each) is fetched with 16-byte
// loads whose lanes run along a row, so every load instruction covers whole cache lines, parked in registers
// while the previous tile is multiplied, and then laid into LDS with a 16-byte pad per row.  The 32x32x16 bf16
// MFMA wants, from lane l, row l%32 and the 8 k-values 8*(l/32)..+7 of A and the same of B (column l%32); those
// fragments are single 16-byte LDS reads.  The k-slices of a step are dealt round robin to the waves, each wave
// carries MT*NT accumulator tiles (element i of lane l = row (i/4)*8 + (l/32)*4 + i%4, column l%32), and the
// waves' partial tiles are added through LDS in a fixed order at the end, so results are reproducible.

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

constexpr int kGateThreads = 512;
constexpr int kGateWaves = kGateThreads / 64;

template <int MT, int NT, int KS>
struct GateTile {
    static constexpr int kTokens = 32 * MT;
    static constexpr int kPiecesPerRow = KS / 8;                 // 16-byte pieces of one row of a step
    static constexpr int kRowStride = KS * 2 + 16;               // bytes in LDS
    static constexpr int kLoads = (32 * (MT + NT) * kPiecesPerRow + kGateThreads - 1) / kGateThreads;
    static constexpr int kTiles = MT * NT;
    // partial tiles of several waves side by side in 64 KiB; waves sharing a slot add one after the other
    static constexpr int kSlots = kTiles > 16 ? 1 : (16 / kTiles) < kGateWaves ? (16 / kTiles) : kGateWaves;
    static constexpr int kRounds = kGateWaves / kSlots;
    static_assert(kSlots * kRounds == kGateWaves, "gate reduction: waves must fill the slots evenly");
    static_assert((KS & (KS - 1)) == 0 && KS >= 64, "gate: KS must be a power of two");
    // `reduce`: the kernel variant that adds the waves' partial tiles through LDS at the end
    static constexpr size_t lds_bytes(int E, bool reduce)
    {
        const size_t tile = (size_t)(kTokens + E) * kRowStride, red = reduce ? (size_t)kSlots * kTiles * 4096 : 0;
        return tile > red ? tile : red;
    }
};

// DEEP: two tiles in flight instead of one (not where the accumulators leave no registers for it).
// SPLIT (needs MT*NT = number of waves): instead of dealing the k-slices, every wave owns one 32x32 output tile
// and walks all k-slices of it: one accumulator tile per wave, which leaves registers for larger tiles in
// flight, and no reduction across waves at the end.
template <int MT, int NT, int KS, bool DEEP, bool SPLIT>
__global__ __launch_bounds__(kGateThreads) void gate_bf16_kernel(const u32x4 *__restrict__ x, const u32x4 *__restrict__ w,
                                                                 float *__restrict__ logits, int64_t T, int H, int E)
{
    using G = GateTile<MT, NT, KS>;
    extern __shared__ __align__(16) unsigned char gate_lds[];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int m = lane & 31, g = lane >> 5;
    const int64_t t0 = (int64_t)blockIdx.x * G::kTokens;
    const int cpr = H / 8;                                        // 16-byte pieces per row in memory
    const int pieces = (G::kTokens + E) * G::kPiecesPerRow;       // pieces of one tile
    const int nsteps = (cpr + G::kPiecesPerRow - 1) / G::kPiecesPerRow;
    const u32x4 zero = {0u, 0u, 0u, 0u};

    // Two tiles are kept in flight.  Every load is issued unconditionally, from a clamped in-bounds address, and
    // what lies outside the matrices is replaced by zeros when the piece is laid into LDS: the number of loads
    // between a tile's issue and its use is then fixed, and the wait before the use lets the younger tile's
    // loads stay outstanding.
    auto piece_ok = [&](int p, int step, int &row, int &c) {
        row = p / G::kPiecesPerRow;
        c = step * G::kPiecesPerRow + p % G::kPiecesPerRow;
        return p < pieces && c < cpr && (row >= G::kTokens || t0 + row < T);
    };
    auto fetch = [&](u32x4(&pre)[G::kLoads], int step) {
#pragma unroll
        for (int q = 0; q < G::kLoads; ++q) {
            int row, c;
            const bool ok = piece_ok(tid + q * kGateThreads, step, row, c);
            const u32x4 *src = x;
            if (ok) src = (row < G::kTokens) ? x + (t0 + row) * cpr + c : w + (int64_t)(row - G::kTokens) * cpr + c;
            pre[q] = *src;
        }
    };
    auto stage = [&](const u32x4(&pre)[G::kLoads], int step) {
        __syncthreads();                                          // the previous tile has been read by every wave
#pragma unroll
        for (int q = 0; q < G::kLoads; ++q) {
            const int p = tid + q * kGateThreads;
            int row, c;
            const bool ok = piece_ok(p, step, row, c);
            if (p < pieces)
                *reinterpret_cast<u32x4 *>(gate_lds + (size_t)row * G::kRowStride + (p % G::kPiecesPerRow) * 16) =
                    ok ? pre[q] : zero;
        }
        __syncthreads();
    };

    // SPLIT: wave v owns column tile v % NT and the row tiles v / NT + i * (waves / NT)
    constexpr int kPerWave = G::kTiles / kGateWaves, kRowTileStep = kGateWaves / NT;
    static_assert(!SPLIT || (kGateWaves % NT == 0 && kPerWave >= 1 && kPerWave * kRowTileStep == MT),
                  "gate: the output tiles must divide evenly among the waves");
    constexpr int kAcc = SPLIT ? kPerWave : G::kTiles;
    f32x16 acc[kAcc];
#pragma unroll
    for (int i = 0; i < kAcc; ++i)
#pragma unroll
        for (int j = 0; j < 16; ++j) acc[i][j] = 0.f;
    auto multiply = [&]() {
        if constexpr (SPLIT) {
            const int n = (wave % NT) * 32 + m;
            const unsigned char *pa = gate_lds + (size_t)((wave / NT) * 32 + m) * G::kRowStride + g * 16;
            const unsigned char *pb = gate_lds + (size_t)(G::kTokens + (n < E ? n : 0)) * G::kRowStride + g * 16;
#pragma unroll 4
            for (int ks = 0; ks < KS / 16; ++ks) {
                bf16x8 b = *reinterpret_cast<const bf16x8 *>(pb + ks * 32);
                if (n >= E) b = __builtin_bit_cast(bf16x8, zero);
#pragma unroll
                for (int i = 0; i < kAcc; ++i) {
                    const bf16x8 a =
                        *reinterpret_cast<const bf16x8 *>(pa + (size_t)i * kRowTileStep * 32 * G::kRowStride + ks * 32);
                    acc[i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, acc[i], 0, 0, 0);
                }
            }
            return;
        }
        for (int ks = wave; ks < KS / 16; ks += kGateWaves) {
            const int off = ks * 32 + g * 16;
            bf16x8 a[MT], b[NT];
#pragma unroll
            for (int mt = 0; mt < MT; ++mt)
                a[mt] = *reinterpret_cast<const bf16x8 *>(gate_lds + (size_t)(mt * 32 + m) * G::kRowStride + off);
#pragma unroll
            for (int nt = 0; nt < NT; ++nt) {
                const int n = nt * 32 + m;
                b[nt] = __builtin_bit_cast(bf16x8, zero);
                if (n < E)
                    b[nt] = *reinterpret_cast<const bf16x8 *>(gate_lds + (size_t)(G::kTokens + n) * G::kRowStride + off);
            }
#pragma unroll
            for (int mt = 0; mt < MT; ++mt)
#pragma unroll
                for (int nt = 0; nt < NT; ++nt)
                    acc[mt * NT + nt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[mt], b[nt], acc[mt * NT + nt], 0, 0, 0);
        }
    };

    if constexpr (DEEP) {
        u32x4 pre0[G::kLoads], pre1[G::kLoads];
        fetch(pre0, 0);
        fetch(pre1, 1);                                           // past the last step: clamped loads, never used
        for (int step = 0; step < nsteps; step += 2) {
            stage(pre0, step);
            fetch(pre0, step + 2);
            multiply();
            if (step + 1 < nsteps) {
                stage(pre1, step + 1);
                fetch(pre1, step + 3);
                multiply();
            }
        }
    } else {
        u32x4 pre0[G::kLoads];
        fetch(pre0, 0);
        for (int step = 0; step < nsteps; ++step) {
            stage(pre0, step);
            fetch(pre0, step + 1);
            multiply();
        }
    }

    if constexpr (SPLIT) {
        // element j of this lane: row (j/4)*8 + g*4 + j%4, column m of the wave's own tile
        const int n = (wave % NT) * 32 + m;
#pragma unroll
        for (int i = 0; i < kAcc; ++i)
#pragma unroll
            for (int j = 0; j < 16; ++j) {
                const int64_t t = t0 + (wave / NT + i * kRowTileStep) * 32 + (j >> 2) * 8 + g * 4 + (j & 3);
                if (t < T && n < E) logits[t * E + n] = acc[i][j];
            }
        return;
    }
    // partial tiles -> LDS [slot][tile][row][col]
    float *red = reinterpret_cast<float *>(gate_lds);
    const int slot = wave % G::kSlots, round = wave / G::kSlots;
    __syncthreads();                                              // the last tile is no longer needed
    for (int r = 0; r < G::kRounds; ++r) {
        if (round == r) {
#pragma unroll
            for (int i = 0; i < G::kTiles; ++i)
#pragma unroll
                for (int j = 0; j < 16; ++j) {
                    const int row = (j >> 2) * 8 + g * 4 + (j & 3);
                    float *q = red + ((slot * G::kTiles + i) * 32 + row) * 32 + m;
                    *q = (r == 0) ? acc[i % kAcc][j] : *q + acc[i % kAcc][j];
                }
        }
        __syncthreads();
    }
    const int64_t rows = (T - t0 < G::kTokens) ? (T - t0) : G::kTokens;
    for (int64_t idx = tid; idx < rows * E; idx += kGateThreads) {
        const int row = (int)(idx / E), n = (int)(idx % E);
        const int tile = (row >> 5) * NT + (n >> 5);
        float sum = 0.f;
#pragma unroll
        for (int sl = 0; sl < G::kSlots; ++sl) sum += red[((sl * G::kTiles + tile) * 32 + (row & 31)) * 32 + (n & 31)];
        logits[t0 * E + idx] = sum;
    }
}

// bf16, at most 8 experts, H <= 8192 and a multiple of 64*NCH: the shapes of the paper's layers.  A tile of 32
// consecutive rows walked in column steps touches memory in short strided runs, which the memory system serves
// well below its streaming rate; here a workgroup reads 8 whole consecutive rows at a time (NCH = 1; halves of
// them if NCH = 2), i.e. one contiguous run of up to 64 KiB.  The 32 MFMA rows are (quarter of the row chunk,
// token) pairs and the 32 columns (quarter, expert) pairs: row qk*8+tok holds x[tok][quarter qk], column qk'*8+e
// holds w[e][quarter qk'], so the diagonal blocks qk = qk' of the accumulator carry the four quarter sums of
// every (token, expert) logit, and the off-diagonal blocks, which would be idle columns anyway with so few
// experts, are ignored.  The weights never change, so a persistent workgroup keeps its B fragments in registers
// for the whole launch: wave v owns steps v, v+8, ... of each quarter.  The sums over chunks (in the accumulator) and
// over waves and quarters (through LDS, by 64 threads, one tile later) run in a fixed order: results are reproducible.
// (A variant with direct-to-LDS loads, three tile buffers and two tiles in flight measured the same within 3 % on
// MI355X and is not kept.)

constexpr int kGateSmallTokens = 8;          // rows of one tile
constexpr int kGateSmallExperts = 8;         // expert slots of one quarter

__host__ __device__ constexpr int gate_small_quarter_stride(int chunk) { return chunk / 2 + 128; }      // bytes
__host__ __device__ constexpr int gate_small_row_stride(int chunk) { return 4 * gate_small_quarter_stride(chunk) + 16; }
__host__ __device__ constexpr size_t gate_small_lds_bytes(int chunk, int threads)
{
    // the tile, then two buffers of partial sums [wave][quarter][token][expert]
    return (size_t)kGateSmallTokens * gate_small_row_stride(chunk) +
           2 * sizeof(float) * (threads / 64) * 4 * kGateSmallTokens * kGateSmallExperts;
}

// NCH chunks per row, THREADS per workgroup, MAXCHUNK = most elements of a row in LDS at a time
template <int NCH, int THREADS, int MAXCHUNK>
__global__ __launch_bounds__(THREADS) void gate_small_kernel(const u32x4 *__restrict__ x, const u32x4 *__restrict__ w,
                                                             float *__restrict__ logits, int64_t T, int H, int E,
                                                             int64_t ngroups)
{
    constexpr int kGateThreads = THREADS, kGateWaves = THREADS / 64;
    constexpr int kGateSmallSteps = MAXCHUNK / 64 / kGateWaves;     // MFMA steps of a chunk per wave, at most
    constexpr int kGateSmallLoads = kGateSmallTokens * MAXCHUNK / 8 / THREADS;
    constexpr int kRedFloats = kGateWaves * 4 * kGateSmallTokens * kGateSmallExperts;
    static_assert(kGateSmallSteps >= 1 && kGateSmallLoads >= 1, "gate_small_kernel: chunk too small for the workgroup");
    extern __shared__ __align__(16) unsigned char gate_lds[];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, g = lane >> 5;
    const int chunk = H / NCH;                       // elements, a multiple of 64
    const int ppr = chunk / 8, ppq = chunk / 32;     // 16-byte pieces per row chunk / per quarter
    const int cpr = H / 8;
    const int QS = gate_small_quarter_stride(chunk), RS = gate_small_row_stride(chunk);
    const int nsteps = chunk / 64;                   // MFMA steps per chunk: a quarter is nsteps*16 elements
    float *red = reinterpret_cast<float *>(gate_lds + (size_t)kGateSmallTokens * RS);
    const u32x4 zero = {0u, 0u, 0u, 0u};

    // This thread's pieces of a tile, fixed for the whole launch: piece p = tid + q*threads is row p / ppr, column
    // p % ppr.  One division per thread; the others follow by stepping (integer division is slow here).
    int piece_row[kGateSmallLoads], piece_col[kGateSmallLoads], piece_lds[kGateSmallLoads];
    {
        const int step_rows = kGateThreads / ppr, step_cols = kGateThreads % ppr;
        int row = tid / ppr, col = tid % ppr;
#pragma unroll
        for (int q = 0; q < kGateSmallLoads; ++q) {
            const bool in_tile = row < kGateSmallTokens;
            const int qk = (col >= ppq ? 1 : 0) + (col >= 2 * ppq ? 1 : 0) + (col >= 3 * ppq ? 1 : 0);
            piece_row[q] = in_tile ? row : -1;
            piece_col[q] = in_tile ? col : 0;
            piece_lds[q] = in_tile ? row * RS + qk * QS + (col - qk * ppq) * 16 : 0;
            row += step_rows;
            col += step_cols;
            if (col >= ppr) {
                col -= ppr;
                ++row;
            }
        }
    }
    // fragment address of this lane at step 0: row lane%8, quarter (lane%32)/8, k-values 8*(lane/32)..+7
    const unsigned char *frag = gate_lds + (size_t)(lane & 7) * RS + (size_t)((lane & 31) >> 3) * QS + g * 16;

    // Loads are issued unconditionally, from clamped addresses, all of a tile before the first use; what lies
    // outside the matrix becomes zeros when the tile is laid into LDS.
    auto fetch = [&](u32x4(&dst)[kGateSmallLoads], const u32x4 *base, int64_t first_row, int64_t row_limit, int c) {
        unsigned ok = 0;
#pragma unroll
        for (int q = 0; q < kGateSmallLoads; ++q) {
            const int64_t r = first_row + piece_row[q];
            const bool live = piece_row[q] >= 0 && r < row_limit;
            dst[q] = *(live ? base + r * cpr + c * ppr + piece_col[q] : base);
            ok |= (live ? 1u : 0u) << q;
        }
        return ok;
    };
    auto lay = [&](const u32x4(&src)[kGateSmallLoads], unsigned ok) {
        __syncthreads();                                          // the previous tile has been read by every wave
#pragma unroll
        for (int q = 0; q < kGateSmallLoads; ++q)
            if (piece_row[q] >= 0)
                *reinterpret_cast<u32x4 *>(gate_lds + piece_lds[q]) = ((ok >> q) & 1u) ? src[q] : zero;
        __syncthreads();
    };

    // weights -> LDS (same layout, expert rows) -> B fragments in registers, while the first tile of x is already
    // on its way
    u32x4 pre[kGateSmallLoads];
    int64_t grp = blockIdx.x;
    unsigned ok = 0;
    bf16x8 bfrag[NCH][kGateSmallSteps];
    {
        u32x4 wpre[kGateSmallLoads];
#pragma unroll
        for (int c = 0; c < NCH; ++c) {
            const unsigned wok = fetch(wpre, w, 0, E, c);
            if (c == NCH - 1) ok = fetch(pre, x, grp * kGateSmallTokens, T, 0);
            lay(wpre, wok);
#pragma unroll
            for (int i = 0; i < kGateSmallSteps; ++i) {
                const int st = wave + i * kGateWaves;
                bfrag[c][i] = __builtin_bit_cast(bf16x8, zero);
                if (st < nsteps) bfrag[c][i] = *reinterpret_cast<const bf16x8 *>(frag + st * 32);
            }
        }
    }

    f32x16 acc;
#pragma unroll
    for (int j = 0; j < 16; ++j) acc[j] = 0.f;

    // The waves' partial sums of a group go to LDS, and 64 threads add them up and store the logits one tile
    // later, behind that tile's barriers: no barrier of its own, and the additions run beside the other waves'
    // MFMAs.  Two buffers, used alternately.
    const int qn = (lane & 31) >> 3;
    int64_t pending = -1;                           // group whose partial sums wait in red[parity]
    int parity = 0;
    auto finish = [&](int64_t done, int buf) {
        if (tid < kGateSmallTokens * kGateSmallExperts) {
            const float *src = red + buf * kRedFloats + tid;      // [wave][quarter][token][expert], tid = token*8 + expert
            float sum = 0.f;
#pragma unroll
            for (int i = 0; i < kGateWaves * 4; ++i) sum += src[i * kGateSmallTokens * kGateSmallExperts];
            const int64_t t = done * kGateSmallTokens + (tid >> 3);
            if ((tid & 7) < E && t < T) logits[t * E + (tid & 7)] = sum;
        }
    };

    for (; grp < ngroups; grp += gridDim.x) {
#pragma unroll
        for (int c = 0; c < NCH; ++c) {
            lay(pre, ok);
            // the next tile is in flight during the MFMAs
            ok = (c + 1 < NCH) ? fetch(pre, x, grp * kGateSmallTokens, T, c + 1)
                               : fetch(pre, x, (grp + gridDim.x) * kGateSmallTokens, T, 0);
            if (pending >= 0) {
                finish(pending, parity ^ 1);
                pending = -1;
            }
            // steps past the chunk's end multiply zeros (their B fragments are zero, A is made zero here)
            bf16x8 a[kGateSmallSteps];
#pragma unroll
            for (int i = 0; i < kGateSmallSteps; ++i) {
                const int st = wave + i * kGateWaves;
                a[i] = __builtin_bit_cast(bf16x8, zero);
                if (st < nsteps) a[i] = *reinterpret_cast<const bf16x8 *>(frag + st * 32);
            }
#pragma unroll
            for (int i = 0; i < kGateSmallSteps; ++i)
                acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[i], bfrag[c][i], acc, 0, 0, 0);
        }
        // accumulator element j of this lane: row (j/4)*8 + g*4 + j%4 = (quarter j/4, token g*4 + j%4), column
        // (quarter (lane%32)/8, expert lane%8): only the diagonal blocks, quarter j/4 = quarter of the column, count
        float *dst = red + parity * kRedFloats + ((wave * 4 + qn) * kGateSmallTokens + g * 4) * kGateSmallExperts + (lane & 7);
#pragma unroll
        for (int i = 0; i < 4; ++i)
            dst[i * kGateSmallExperts] = qn == 0 ? acc[i] : qn == 1 ? acc[4 + i] : qn == 2 ? acc[8 + i] : acc[12 + i];
        pending = grp;
        parity ^= 1;
#pragma unroll
        for (int j = 0; j < 16; ++j) acc[j] = 0.f;
    }
    if (pending >= 0) {
        __syncthreads();
        finish(pending, parity ^ 1);
    }
}

// fp32 activations: one wave per token, eight experts at a time, fp32 fused multiply-adds and a shuffle reduction
__global__ __launch_bounds__(256) void gate_f32_kernel(const float4 *__restrict__ x, const float4 *__restrict__ w,
                                                       float *__restrict__ logits, int64_t T, int H, int E)
{
    const int lane = threadIdx.x & 63;
    const int64_t t = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    if (t >= T) return;
    const int vpr = H / 4;
    const float4 *xr = x + t * vpr;
    for (int e0 = 0; e0 < E; e0 += 8) {
        float acc[8];
#pragma unroll
        for (int j = 0; j < 8; ++j) acc[j] = 0.f;
        for (int v = lane; v < vpr; v += 64) {
            const float4 xv = xr[v];
#pragma unroll
            for (int j = 0; j < 8; ++j)
                if (e0 + j < E) {
                    const float4 wv = w[(int64_t)(e0 + j) * vpr + v];
                    acc[j] = fmaf(xv.x, wv.x, fmaf(xv.y, wv.y, fmaf(xv.z, wv.z, fmaf(xv.w, wv.w, acc[j]))));
                }
        }
#pragma unroll
        for (int j = 0; j < 8; ++j) {
#pragma unroll
            for (int off = 32; off >= 1; off >>= 1) acc[j] += __shfl_xor(acc[j], off, 64);
            if (lane == 0 && e0 + j < E) logits[t * E + e0 + j] = acc[j];
        }
    }
}

// ------------------------------------------------------------ expert layer
//
// y[r][n] = sum_k x_final[r][k] * w[e][n][k] for the rows r of expert e's range in the expert-major buffer
// (section "Expert Parallel": the experts process the tokens grouped to them between Dispatch and Combine).  A
// grouped GEMM whose group sizes exist only on the device: the ranges come from the plan tables, the launch is
// sized for the worst case and surplus workgroups leave at once.
//
// bf16: a workgroup of 4 waves computes a 128 x 256 tile of y (rows x output features) of one expert; the hidden
// axis goes in steps of 64 elements through registers into LDS (rows padded by 16 bytes, as in the gate kernels).
// The waves form a 2 x 2 grid; a wave owns 64 x 128 = 2 x 4 MFMA tiles (128 accumulator registers), so every A
// fragment read from LDS feeds 4 MFMAs and every B fragment 2.  Workgroups are numbered so that those which run
// together on one XCD (hardware deals consecutive workgroups round robin to the 8 XCDs) are row tiles of the
// same few weight tiles: the weight tile then comes from that XCD's L2 after its first reader.

constexpr int kExpBK = 64;
constexpr int kExpRowStride = kExpBK * 2 + 16;                                  // bytes in LDS
constexpr int kXcds = 8;

// BM x BN: the workgroup's tile of y; its WM x WN waves each own (BM/WM) x (BN/WN).  One LDS buffer, two barriers
// per step.  In use: 128 x 256 with 2 x 2 waves, two workgroups per CU.  Measured and not faster on MI355X (all
// within 5 % of it): 256 x 256 with 8 waves, 256 x 128, two register sets of tiles in flight, two LDS buffers, and
// staggered starts along the hidden axis; the stores of y cost nothing measurable.
template <int BM, int BN, int WM, int WN>
struct ExpertTile {
    static constexpr int kThreads = 64 * WM * WN;
    static constexpr int kRowsPerPass = kThreads / 8;             // tile rows the threads cover with one load each
    static constexpr int kLoads = (BM + BN) / kRowsPerPass;       // 16-byte pieces per thread and step
    static constexpr int kLdsBytes = (BM + BN) * kExpRowStride;
    static constexpr int kMT = BM / WM / 32, kNT = BN / WN / 32;  // MFMA tiles of a wave
    static constexpr int kWgsPerCu = kThreads <= 256 ? 2 : 1;     // what the registers allow
    static_assert(BM % (32 * WM) == 0 && BN % (32 * WN) == 0 && kExpBK == 64 && BM % kRowsPerPass == 0 &&
                      BN % kRowsPerPass == 0, "expert kernel: tile shape");
};

struct ExpertArgs {
    const int32_t *lo;      // [E] first row of the expert's range
    const int32_t *hi_base; // [E] one past its last row is hi_base[e] + hi_len[e] ...
    const int32_t *hi_len;  // [E] ... or hi_base[e] alone if this is nullptr
    int32_t E, H, N, max_rows;
    int32_t reserved;       // unused
};

// The expert whose tiles include logical tile number L, found without walking the experts one by one (a walk costs
// one dependent table read per expert before the workgroup can start): 64 experts at a time, one per lane, a wave
// scan of their tile counts, a ballot for the first lane whose running total passes L.  Every lane of every wave
// takes part and gets the same answer.  e == E: no such tile (a surplus workgroup).
struct ExpertTileHit {
    int e, lo, hi, tiles;     // expert, its row range [lo, hi), its row tiles
    int64_t L;                // tile number inside the expert
};

// WHOLE: only the whole tiles of a segment count (its ragged last tile is numbered elsewhere); `all` returns the
// number of tiles counted over all experts when L lies past them.
template <int BM, bool WHOLE = false>
__device__ __forceinline__ ExpertTileHit find_expert_tile(const ExpertArgs &a, int nct, int64_t L, int lane,
                                                          int64_t *all = nullptr)
{
    ExpertTileHit h;
    h.e = a.E;
    h.lo = h.hi = h.tiles = 0;
    h.L = 0;
    int64_t before = 0;                                            // tiles of the experts of earlier rounds
    for (int e0 = 0; e0 < a.E; e0 += kWave) {
        const int e = e0 + lane;
        int lo = 0, hi = 0, tiles = 0;
        if (e < a.E) {
            lo = a.lo[e];
            hi = a.hi_base[e] + (a.hi_len ? a.hi_len[e] : 0);
            tiles = hi > lo ? (int)(((int64_t)hi - lo + (WHOLE ? 0 : BM - 1)) / BM) : 0;
        }
        const int64_t cnt = (int64_t)tiles * nct;
        int64_t incl = cnt;
#pragma unroll
        for (int d = 1; d < kWave; d <<= 1) {
            const int64_t o = __shfl_up(incl, d, kWave);
            if (lane >= d) incl += o;
        }
        const int64_t total = __shfl(incl, kWave - 1, kWave);
        if (L < before + total) {
            // an expert without tiles repeats its predecessor's running total, so the first lane past L has tiles
            const unsigned long long past = __ballot(L < before + incl);
            const int src = __ffsll((long long)past) - 1;
            h.e = e0 + src;
            h.lo = __shfl(lo, src, kWave);
            h.hi = __shfl(hi, src, kWave);
            h.tiles = __shfl(tiles, src, kWave);
            h.L = L - before - (__shfl(incl, src, kWave) - __shfl(cnt, src, kWave));
            return h;
        }
        before += total;
    }
    if (all) *all = before;
    return h;
}

__device__ __forceinline__ unsigned int f32_to_bf16_rne(float f)
{
    const unsigned int u = __float_as_uint(f);
    return (u + 0x7fffu + ((u >> 16) & 1u)) >> 16;       // finite inputs
}

template <int BM, int BN, int WM, int WN>
__global__ __launch_bounds__(64 * WM * WN, (64 * WM * WN <= 256 ? 2 : 1)) void expert_bf16_kernel(const u32x4 *__restrict__ x,
                                                                                      const u32x4 *__restrict__ w,
                                                                                      unsigned short *__restrict__ y,
                                                                                      ExpertArgs a)
{
    using G = ExpertTile<BM, BN, WM, WN>;
    extern __shared__ __align__(16) unsigned char exp_lds[];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, m = lane & 31, g = lane >> 5;
    const int cpr = a.H / 8;                                       // 16-byte pieces per row in memory
    const int nct = (a.N + BN - 1) / BN;                           // column tiles

    // logical tile numbers go out in blocks, XCD i taking kPerXcd consecutive numbers of each block (the workgroups
    // that run together on one XCD, which hardware fills round robin, then share operand tiles, and surplus numbers at
    // the end are spread over all XCDs); the numbering is (expert, column tile, row tile), row tile fastest
    constexpr int kPerXcd = 32 * G::kWgsPerCu;
    const int64_t jx = blockIdx.x / kXcds;
    int64_t L = (jx / kPerXcd) * (kPerXcd * kXcds) + (int64_t)(blockIdx.x % kXcds) * kPerXcd + jx % kPerXcd;
    const ExpertTileHit hit = find_expert_tile<BM>(a, nct, L, lane);
    const int e = hit.e;
    int row0 = 0, row_end = 0, ct = 0;
    if (e < a.E) {
        ct = (int)(hit.L / hit.tiles);
        row0 = hit.lo + (int)(hit.L % hit.tiles) * BM;
        row_end = hit.hi < a.max_rows ? hit.hi : a.max_rows;
    }
    if (e == a.E || row0 < 0 || row0 >= row_end) return;          // surplus workgroup (uniform for the workgroup)
    const int col0 = ct * BN;

    // This thread's pieces of a step's tile: piece q is row tid/8 + (threads/8)*q of the tile, 16-byte column tid%8;
    // tile rows 0..BM-1 are rows of x, the others rows of the weight tile.  Loads are issued unconditionally from
    // clamped in-bounds addresses; what lies outside becomes zeros when the tile is laid into LDS.
    const u32x4 zero = {0u, 0u, 0u, 0u};
    const int r8 = tid >> 3, c_real = tid & 7;
    const int c0 = c_real < cpr ? c_real : 0;                     // rows shorter than a step: stay inside the row
    int grow[G::kLoads];                                           // row of x, or row of w, that piece q reads
    unsigned live = 0;
#pragma unroll
    for (int q = 0; q < G::kLoads; ++q) {
        bool ok;
        if (q < BM / G::kRowsPerPass) {
            const int r = row0 + r8 + q * G::kRowsPerPass;
            ok = r < row_end;
            grow[q] = ok ? r : row0;
        } else {
            const int n = col0 + r8 + (q - BM / G::kRowsPerPass) * G::kRowsPerPass;
            ok = n < a.N;
            grow[q] = e * a.N + (ok ? n : 0);
        }
        live |= (ok ? 1u : 0u) << q;
    }
    const int nsteps = (cpr + kExpBK / 8 - 1) / (kExpBK / 8);
    unsigned char *lay_at = exp_lds + r8 * kExpRowStride + c_real * 16;

    // steps past the end of the hidden axis are fetched from clamped addresses and never laid down
    auto fetch = [&](u32x4(&pre)[G::kLoads], int step) {
        const int c = step * (kExpBK / 8) + c_real < cpr ? step * (kExpBK / 8) + c0 : c0;
#pragma unroll
        for (int q = 0; q < G::kLoads; ++q) pre[q] = (q < BM / G::kRowsPerPass ? x : w)[(int64_t)grow[q] * cpr + c];
    };
    auto lay = [&](const u32x4(&pre)[G::kLoads], int step) {
        const bool col_ok = step * (kExpBK / 8) + c_real < cpr;
        __syncthreads();                                           // the previous tile has been read by every wave
#pragma unroll
        for (int q = 0; q < G::kLoads; ++q)
            *reinterpret_cast<u32x4 *>(lay_at + q * G::kRowsPerPass * kExpRowStride) =
                (((live >> q) & 1u) && col_ok) ? pre[q] : zero;
        __syncthreads();
    };

    f32x16 acc[G::kMT][G::kNT];
#pragma unroll
    for (int i = 0; i < G::kMT; ++i)
#pragma unroll
        for (int j = 0; j < G::kNT; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;

    const int wm = wave / WN, wn = wave % WN;                      // the wave's place in the WM x WN grid
    const unsigned char *pa = exp_lds + (size_t)(wm * (BM / WM) + m) * kExpRowStride + g * 16;
    const unsigned char *pb = exp_lds + (size_t)(BM + wn * (BN / WN) + m) * kExpRowStride + g * 16;
    auto multiply = [&]() {
#pragma unroll
        for (int ks = 0; ks < kExpBK / 16; ++ks) {
            bf16x8 fa[G::kMT], fb[G::kNT];
#pragma unroll
            for (int i = 0; i < G::kMT; ++i)
                fa[i] = *reinterpret_cast<const bf16x8 *>(pa + (size_t)i * 32 * kExpRowStride + ks * 32);
#pragma unroll
            for (int j = 0; j < G::kNT; ++j)
                fb[j] = *reinterpret_cast<const bf16x8 *>(pb + (size_t)j * 32 * kExpRowStride + ks * 32);
#pragma unroll
            for (int i = 0; i < G::kMT; ++i)
#pragma unroll
                for (int j = 0; j < G::kNT; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[i], fb[j], acc[i][j], 0, 0, 0);
        }
    };

    u32x4 pre[G::kLoads];
    fetch(pre, 0);
    for (int step = 0; step < nsteps; ++step) {
        lay(pre, step);
        fetch(pre, step + 1);                                      // in flight during the MFMAs
        multiply();
    }

    // accumulator element v of a lane: row (v/4)*8 + g*4 + v%4, column m of the 32 x 32 tile
#pragma unroll
    for (int i = 0; i < G::kMT; ++i)
#pragma unroll
        for (int j = 0; j < G::kNT; ++j) {
            const int n = col0 + wn * (BN / WN) + j * 32 + m;
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int r = row0 + wm * (BM / WM) + i * 32 + (v >> 2) * 8 + g * 4 + (v & 3);
                if (r < row_end && n < a.N) y[(int64_t)r * a.N + n] = (unsigned short)f32_to_bf16_rne(acc[i][j][v]);
            }
        }
}

// The same contraction with direct-to-LDS loads (global_load_lds_dwordx4: 64 lanes x 16 bytes land in 1 KiB of
// LDS that the instruction addresses, lane i at byte 16*i, without passing through registers).  That frees the
// registers the staged tile occupied, so 8 waves can hold a 256 x 256 tile of y (a wave 128 x 64), which halves
// the L2 traffic per flop, and a step needs one barrier instead of two: the next step's tile streams into the other
// of two LDS buffers while the MFMAs run.  Rows are 128 bytes in LDS without padding; the 16-byte piece c of row r
// sits at position c ^ ((r / 2) % 8).  A fragment read has 16 lanes (16 consecutive rows, one piece each) share the
// 64 banks: two rows fill them, so the pieces must differ among the even rows and among the odd rows, which r / 2
// gives; c ^ (r % 8) makes rows r and r + 8 collide (measured with ds_read_b128 alone: 113 against 220 bytes per
// clock and CU).  Since the LDS position of a lane's data is fixed by the instruction, the swizzle is applied on the
// global side (lane i of a chunk of 8 rows fetches piece (i % 8) ^ ((row / 2) % 8) of tile row `row` = chunk * 8 +
// i / 8).  Needs H to be a multiple of 64 (a tail step cannot be zero-filled on this path); rows past a segment's
// end are fetched from its last row and their results are not stored.
// Measured on MI355X (16384 x 4096 x 4096, one expert, bursts of 20 launches): 590-610 us against 715-740 us for the
// register-staged kernel; with clocks settled over thousands of launches a stand-alone copy of this loop takes
// 460-477 us.  A segment's ragged last tile costs a full tile's time (skipping the MFMAs of its empty 32-row blocks
// was measured and does not pay).
constexpr int kDtlBM = 256, kDtlBN = 256, kDtlWM = 2, kDtlWN = 4, kDtlThreads = 64 * kDtlWM * kDtlWN;
constexpr int kDtlStageBytes = (kDtlBM + kDtlBN) * 128;
constexpr int kDtlLdsBytes = 2 * kDtlStageBytes;

// A ragged tile of at most 64 rows, the kind a launch's last round is made of: so little arithmetic per step that the
// step is as long as its loads take to arrive.  Compact stages of 64 + 256 rows (40 KiB), three of them, the loads of
// two steps in flight: half the time per step of the two-stage loop.  Eight waves, each all 64 rows x 32 columns.
// Every wave issues the same number of loads per step (rows past the segment's end repeat its last row), because the
// wait for a stage counts the younger loads.  The barrier is the bare instruction behind a wait for the LDS reads: the
// compiler's own barrier would wait for every outstanding load, the next stages' included.
__device__ __forceinline__ void expert_dtl_small_rows(const u32x4 *__restrict__ x, const u32x4 *__restrict__ w,
                                                      unsigned short *__restrict__ y, const ExpertArgs &a, int e,
                                                      int row0, int row_end, int col0, unsigned char *lds)
{
    constexpr int XR = 64, WR = 256, STG = (XR + WR) * 128, NST = 3, CPW = (XR + WR) / 8 / 8;   // 5 chunks per wave
    static_assert(NST * STG <= kDtlLdsBytes && XR % 16 == 0, "expert_dtl_small_rows: stages must fit the kernel's LDS");
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, m = lane & 31, g = lane >> 5;
    const int cpr = a.H / 8, nsteps = a.H / 64;
    const int lr = lane >> 3;
    const u32x4 *src[CPW];
#pragma unroll
    for (int q = 0; q < CPW; ++q) {
        const int trow = (wave * CPW + q) * 8 + lr;                // 0 .. 319
        const int lc = (lane & 7) ^ ((trow >> 1) & 7);
        if (trow < XR) {
            const int r = row0 + trow;
            src[q] = x + (int64_t)(r < row_end ? r : row_end - 1) * cpr + lc;
        } else {
            const int n = col0 + trow - XR;
            src[q] = w + ((int64_t)e * a.N + (n < a.N ? n : a.N - 1)) * cpr + lc;
        }
    }
    auto issue = [&](int step, int slot) {
#pragma unroll
        for (int q = 0; q < CPW; ++q)
            __builtin_amdgcn_global_load_lds(
                (const void __attribute__((address_space(1))) *)(src[q] + step * 8),
                (void __attribute__((address_space(3))) *)(lds + slot * STG + (wave * CPW + q) * 1024), 16, 0, 0);
    };
    f32x16 acc[2];
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[i][v] = 0.f;
    const unsigned char *pa = lds + (size_t)m * 128;
    const unsigned char *pb = lds + (size_t)(XR + wave * 32 + m) * 128;
    int koff[4];
#pragma unroll
    for (int ks = 0; ks < 4; ++ks) koff[ks] = ((2 * ks + g) ^ ((m >> 1) & 7)) * 16;
    const int nb = row_end - row0 > 32 ? 2 : 1;                    // 32-row blocks with rows of the segment

    issue(0, 0);
    if (nsteps > 1) issue(1, 1);
    int slot = 0;
    for (int step = 0; step < nsteps; ++step) {
        // stage `step` has landed once at most the CPW loads of stage step+1 are outstanding (loads finish in order)
        if (step + 1 < nsteps) __builtin_amdgcn_s_waitcnt(0x0f70 | CPW);
        else __builtin_amdgcn_s_waitcnt(0x0f70);
        asm volatile("" ::: "memory");
        __builtin_amdgcn_s_waitcnt(0xc07f);                        // lgkmcnt(0): this wave's reads of the previous stage
        __builtin_amdgcn_s_barrier();
        asm volatile("" ::: "memory");
        if (step + 2 < nsteps) issue(step + 2, slot == 0 ? 2 : slot - 1);   // the slot of stage step-1, free now
        const int buf = slot * STG;
#pragma unroll
        for (int ks = 0; ks < 4; ++ks) {
            const bf16x8 fb = *reinterpret_cast<const bf16x8 *>(pb + buf + koff[ks]);
            const bf16x8 fa0 = *reinterpret_cast<const bf16x8 *>(pa + buf + koff[ks]);
            acc[0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa0, fb, acc[0], 0, 0, 0);
            if (nb > 1) {
                const bf16x8 fa1 = *reinterpret_cast<const bf16x8 *>(pa + buf + 32 * 128 + koff[ks]);
                acc[1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa1, fb, acc[1], 0, 0, 0);
            }
        }
        slot = slot == 2 ? 0 : slot + 1;
    }
    const int n = col0 + wave * 32 + m;
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            const int r = row0 + i * 32 + (v >> 2) * 8 + g * 4 + (v & 3);
            if (r < row_end && n < a.N) y[(int64_t)r * a.N + n] = (unsigned short)f32_to_bf16_rne(acc[i][v]);
        }
}


template <bool RAGGED_LAST>
__global__ __launch_bounds__(kDtlThreads) void expert_dtl_kernel(const u32x4 *__restrict__ x, const u32x4 *__restrict__ w,
                                                                 unsigned short *__restrict__ y, ExpertArgs a)
{
    constexpr int BM = kDtlBM, BN = kDtlBN, WM = kDtlWM, WN = kDtlWN, WAVES = WM * WN;
    constexpr int CPW = (BM + BN) / 8 / WAVES;                     // 1 KiB chunks (8 tile rows) per wave and step
    constexpr int MT = BM / WM / 32, NT = BN / WN / 32;
    static_assert((BM + BN) % (8 * WAVES) == 0 && BM % 16 == 0, "expert_dtl_kernel: chunks must divide among the waves");
    extern __shared__ __align__(16) unsigned char dtl_lds[];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, m = lane & 31, g = lane >> 5;
    const int cpr = a.H / 8, nsteps = a.H / 64;
    const int nct = (a.N + BN - 1) / BN;

    // Tile of this workgroup.  Hardware deals consecutive workgroups round robin to the 8 XCDs, each with its own L2;
    // the 32 workgroups that run together on one XCD should share tiles of x and of the weights.  So logical tile
    // numbers are handed out in blocks of 256, XCD i taking numbers 32 i .. 32 i + 31 of each block, and inside an
    // expert the numbering is (panel of 8 row tiles, column tile, row tile in the panel), innermost fastest: an XCD
    // then works on 8 row tiles x 4 column tiles at a time (12 distinct operand tiles instead of 33).
    const int64_t j = blockIdx.x / kXcds;
    int64_t L = (j / 32) * (32 * kXcds) + (int64_t)(blockIdx.x % kXcds) * 32 + j % 32;
    // With RAGGED_LAST the whole tiles of all experts are numbered first and the ragged last tiles of the segments
    // after them, the one with the most rows first: a launch rarely fills its last round of workgroups, and this way
    // that round consists of the tiles that cost least (their empty 32-row blocks are skipped below).  The price: a
    // ragged tile no longer shares its weight tile's trip through the L2 with the other row tiles of its panel, so
    // the host asks for it only when the ragged tiles are few (at most one round of workgroups).
    int64_t whole = 0;
    const ExpertTileHit hit = RAGGED_LAST ? find_expert_tile<BM, true>(a, nct, L, lane, &whole)
                                          : find_expert_tile<BM, false>(a, nct, L, lane);
    int e = hit.e;
    int row0 = 0, row_end = 0, ct = 0;
    if (e < a.E) {
        constexpr int P = 8;                                       // row tiles of a panel (4..32 measure alike)
        const int tiles = hit.tiles, full = tiles / P;             // whole panels
        int rt;
        if (hit.L < (int64_t)full * P * nct) {
            const int p = (int)(hit.L / (P * nct)), rem = (int)(hit.L % (P * nct));
            ct = rem / P;
            rt = p * P + rem % P;
        } else {
            const int rem = (int)(hit.L - (int64_t)full * P * nct), pr = tiles - full * P;
            ct = rem / pr;
            rt = full * P + rem % pr;
        }
        row0 = hit.lo + rt * BM;
        row_end = hit.hi < a.max_rows ? hit.hi : a.max_rows;
    } else if (RAGGED_LAST) {
        // ragged tiles: position L / nct in the order (rows in the ragged tile, descending; expert, ascending).  The
        // tile buffers are not in use yet, so their first bytes serve as the scratch of the ranking (E <= 256).
        const int64_t Lr = L - whole;
        int *scr = reinterpret_cast<int *>(dtl_lds);
        int my_rem = 0;
        if (tid < a.E) {
            const int lo = a.lo[tid], hi = a.hi_base[tid] + (a.hi_len ? a.hi_len[tid] : 0);
            my_rem = hi > lo ? (int)(((int64_t)hi - lo) % BM) : 0;
            scr[tid] = my_rem;
        }
        if (tid == 0) scr[256] = -1;
        __syncthreads();
        if (my_rem > 0) {
            int rank = 0;
            for (int o = 0; o < a.E; ++o) {
                const int ro = scr[o];
                rank += (ro > my_rem || (ro == my_rem && o < tid)) ? 1 : 0;
            }
            if (rank == Lr / nct) scr[256] = tid;
        }
        __syncthreads();
        const int eh = scr[256];
        __syncthreads();                                           // everyone has read it before the tiles stream in
        if (eh >= 0 && eh < a.E) {
            e = eh;
            const int lo = a.lo[e], hi = a.hi_base[e] + (a.hi_len ? a.hi_len[e] : 0);
            ct = (int)(Lr % nct);
            row0 = lo + (int)(((int64_t)hi - lo) / BM) * BM;
            row_end = hi < a.max_rows ? hi : a.max_rows;
        }
    }
    if (e == a.E || row0 < 0 || row0 >= row_end) return;          // surplus workgroup (uniform for the workgroup)
    const int col0 = ct * BN;
    if (RAGGED_LAST && row_end - row0 <= 64) {                     // a short ragged tile: the three-stage loop
        expert_dtl_small_rows(x, w, y, a, e, row0, row_end, col0, dtl_lds);
        return;
    }

    // source of this lane in each of its wave's chunks: tile row chunk*8 + lane/8, piece (lane%8) ^ ((row/2)%8)
    // (BM is a multiple of 16, so the rows of the weight tile swizzle like rows 0.. of their own)
    const int lr = lane >> 3;
    const u32x4 *src[CPW];
    unsigned skip = 0;                      // chunks of 8 rows of x wholly past the segment's end: never fetched
#pragma unroll
    for (int q = 0; q < CPW; ++q) {
        const int trow = (wave * CPW + q) * 8 + lr;
        const int lc = (lane & 7) ^ ((trow >> 1) & 7);
        if (RAGGED_LAST && (wave * CPW + q) * 8 < BM && row0 + (wave * CPW + q) * 8 >= row_end) skip |= 1u << q;
        if (trow < BM) {
            const int r = row0 + trow;
            src[q] = x + (int64_t)(r < row_end ? r : row_end - 1) * cpr + lc;
        } else {
            const int n = col0 + trow - BM;
            src[q] = w + ((int64_t)e * a.N + (n < a.N ? n : a.N - 1)) * cpr + lc;
        }
    }
    auto issue = [&](int step, int buf) {
        if (skip == 0) {
#pragma unroll
            for (int q = 0; q < CPW; ++q)
                __builtin_amdgcn_global_load_lds(
                    (const void __attribute__((address_space(1))) *)(src[q] + step * 8),
                    (void __attribute__((address_space(3))) *)(dtl_lds + buf * kDtlStageBytes + (wave * CPW + q) * 1024), 16, 0, 0);
        } else {
#pragma unroll
            for (int q = 0; q < CPW; ++q)
                if (!((skip >> q) & 1u))
                    __builtin_amdgcn_global_load_lds(
                        (const void __attribute__((address_space(1))) *)(src[q] + step * 8),
                        (void __attribute__((address_space(3))) *)(dtl_lds + buf * kDtlStageBytes + (wave * CPW + q) * 1024), 16, 0, 0);
        }
    };

    f32x16 acc[MT][NT];
#pragma unroll
    for (int i = 0; i < MT; ++i)
#pragma unroll
        for (int j = 0; j < NT; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;

    const int wm = wave / WN, wn = wave % WN;
    const unsigned char *pa = dtl_lds + (size_t)(wm * (BM / WM) + m) * 128;
    const unsigned char *pb = dtl_lds + (size_t)(BM + wn * (BN / WN) + m) * 128;
    int koff[kExpBK / 16];                                         // byte offset of this lane's fragment piece per k-slice
#pragma unroll
    for (int ks = 0; ks < kExpBK / 16; ++ks) koff[ks] = ((2 * ks + g) ^ ((m >> 1) & 7)) * 16;   // 32-row blocks: (row/2)%8 = (m/2)%8

    // 32-row blocks of this wave that hold rows of the segment (all MT of them except in a ragged tile)
    int nb = MT;
    if (RAGGED_LAST) {
        nb = (row_end - row0 - wm * (BM / WM) + 31) / 32;
        nb = nb < 0 ? 0 : (nb > MT ? MT : nb);
    }

    issue(0, 0);
    for (int step = 0; step < nsteps; ++step) {
        // s_waitcnt vmcnt(0) (expcnt and lgkmcnt left at their maxima): this step's tile has landed in LDS
        __builtin_amdgcn_s_waitcnt(0x0f70);
        __syncthreads();                                           // ... for every wave, and the other buffer is free
        if (step + 1 < nsteps) issue(step + 1, (step + 1) & 1);    // streams in during the MFMAs
        const int buf = (step & 1) * kDtlStageBytes;
        if (nb == MT) {
#pragma unroll
            for (int ks = 0; ks < kExpBK / 16; ++ks) {
                bf16x8 fa[MT], fb[NT];
#pragma unroll
                for (int i = 0; i < MT; ++i) fa[i] = *reinterpret_cast<const bf16x8 *>(pa + buf + i * 32 * 128 + koff[ks]);
#pragma unroll
                for (int j = 0; j < NT; ++j) fb[j] = *reinterpret_cast<const bf16x8 *>(pb + buf + j * 32 * 128 + koff[ks]);
#pragma unroll
                for (int i = 0; i < MT; ++i)
#pragma unroll
                    for (int j = 0; j < NT; ++j)
                        acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[i], fb[j], acc[i][j], 0, 0, 0);
            }
        } else if (nb > 0) {
            // ragged tile: blocks past the segment's end are not multiplied (uniform per wave); the fragment reads stay
            // as they are, so that the loop keeps the shape of the one above (what they fetch there is never used)
#pragma unroll
            for (int ks = 0; ks < kExpBK / 16; ++ks) {
                bf16x8 fa[MT], fb[NT];
#pragma unroll
                for (int i = 0; i < MT; ++i) fa[i] = *reinterpret_cast<const bf16x8 *>(pa + buf + i * 32 * 128 + koff[ks]);
#pragma unroll
                for (int j = 0; j < NT; ++j) fb[j] = *reinterpret_cast<const bf16x8 *>(pb + buf + j * 32 * 128 + koff[ks]);
#pragma unroll
                for (int i = 0; i < MT; ++i)
                    if (i < nb) {
#pragma unroll
                        for (int j = 0; j < NT; ++j)
                            acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[i], fb[j], acc[i][j], 0, 0, 0);
                    }
            }
        }
    }

    // accumulator element v of a lane: row (v/4)*8 + g*4 + v%4, column m of the 32 x 32 tile
#pragma unroll
    for (int i = 0; i < MT; ++i)
#pragma unroll
        for (int j = 0; j < NT; ++j) {
            const int n = col0 + wn * (BN / WN) + j * 32 + m;
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int r = row0 + wm * (BM / WM) + i * 32 + (v >> 2) * 8 + g * 4 + (v & 3);
                if (r < row_end && n < a.N) y[(int64_t)r * a.N + n] = (unsigned short)f32_to_bf16_rne(acc[i][j][v]);
            }
        }
}

// fp32 activations (small test shapes only): one thread per output element, fp32 fused multiply-adds
__global__ __launch_bounds__(256) void expert_f32_kernel(const float *__restrict__ x, const float *__restrict__ w,
                                                         float *__restrict__ y, ExpertArgs a)
{
    const int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;
    const int64_t r = idx / a.N;
    const int n = (int)(idx % a.N);
    if (r >= a.max_rows) return;
    int e = 0;
    for (; e < a.E; ++e) {
        const int lo = a.lo[e], hi = a.hi_base[e] + (a.hi_len ? a.hi_len[e] : 0);
        if (r >= lo && r < hi) break;
    }
    if (e == a.E) return;
    const float *xr = x + r * a.H, *wr = w + ((int64_t)e * a.N + n) * a.H;
    float acc = 0.f;
    for (int k = 0; k < a.H; ++k) acc = fmaf(xr[k], wr[k], acc);
    y[r * a.N + n] = acc;
}

// ------------------------------------------------------------- plain copy

__global__ __launch_bounds__(kMoverThreads) void copy_kernel(const u32x4 *__restrict__ src, u32x4 *__restrict__ dst,
                                                             size_t nvec)
{
    const size_t stride = (size_t)gridDim.x * kMoverThreads * kVecInFlight;
    for (size_t base = (size_t)blockIdx.x * kMoverThreads * kVecInFlight + threadIdx.x; base < nvec; base += stride) {
        u32x4 val[kVecInFlight];
#pragma unroll
        for (int q = 0; q < kVecInFlight; ++q)
            if (base + (size_t)q * kMoverThreads < nvec) val[q] = ld16<true>(src + base + (size_t)q * kMoverThreads);
#pragma unroll
        for (int q = 0; q < kVecInFlight; ++q)
            if (base + (size_t)q * kMoverThreads < nvec) st16<true>(dst + base + (size_t)q * kMoverThreads, val[q]);
    }
}

}  // namespace monta
