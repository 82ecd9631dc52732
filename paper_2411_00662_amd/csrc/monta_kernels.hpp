// Device code of the MoE dispatch / combine path for gfx950 (wave64).
//
// Everything here is bandwidth or latency bound; there is no dense contraction
// on the path, so no MFMA.  The row movers (pack, regather, combine) move rows of
// 16-byte vectors straight through registers with several loads in flight per
// lane; the planning kernels are integer work on wavefront bit masks.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace monta {

typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

constexpr int kWave = 64;
constexpr int kMoverThreads = 256;   // threads per workgroup of the row movers
constexpr int kVecInFlight = 4;      // 16-byte loads issued by a lane before its first store

// meta[] slots (int32)
enum { META_R = 0, META_ALIVE = 1, META_C = 2, META_DONE = 3, META_SLOTS = 16 };

struct PlanPtrs {
    int32_t *meta, *counts, *kept, *offsets, *n, *stage_off, *unit_base, *send_rows, *unit_rows;
    int32_t *pos_final, *pos_stage, *row_map, *block_counts, *block_base;
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

__device__ __forceinline__ u32x4 ld16(const u32x4 *p) { return __builtin_nontemporal_load(p); }
__device__ __forceinline__ void st16(u32x4 *p, u32x4 v) { __builtin_nontemporal_store(v, p); }

// ------------------------------------------------------------ route + plan

// One workgroup routes TB consecutive tokens of ONE unit, one token per lane.
//  1. the [nt][E] logits tile is staged in LDS (coalesced, odd row stride);
//  2. k selection passes per token over its LDS row: the next winner is the largest
//     element that comes after the previous winner in (value desc, index asc) order,
//     so ties resolve to the lower index with no "taken" mask;
//  3. gates in fp64 from the winners' logits, one rounding to fp32;
//  4. every lane ORs its bit into mask[expert][wave] in LDS; popcounts of those
//     masks give the workgroup's expert histogram and each pair's stable rank inside
//     the workgroup (lanes hold consecutive tokens, so bit order is token order);
//  5. the last workgroup to finish (ticket counter) turns the per-workgroup
//     histograms into every plan table: exclusive scans over workgroups per
//     expert, capacity clip, expert offsets, per-unit block tables.
// No atomics decide a position: the result is deterministic.
__global__ __launch_bounds__(256) void route_plan_kernel(const float *__restrict__ logits,
                                                         int32_t *__restrict__ topk_idx,
                                                         float *__restrict__ gates, PlanPtrs p, Shape s)
{
    extern __shared__ __align__(16) unsigned char smem[];
    const int E = s.E, k = s.k, TB = s.TB;
    const int stride = E | 1;
    const int NW = TB > kWave ? TB / kWave : 1;
    float *s_l = reinterpret_cast<float *>(smem);
    int *s_sel = reinterpret_cast<int *>(s_l + (size_t)TB * stride);
    unsigned long long *s_mask = reinterpret_cast<unsigned long long *>(
        smem + (((size_t)TB * stride * 4 + (size_t)TB * k * 4 + 7) & ~(size_t)7));
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

    const int t = t_begin + tid;
    const bool active = tid < nt;
    if (active) {
        const float *row = s_l + tid * stride;
        int *sel = s_sel + tid * k;
        float pv = INFINITY;
        int pi = -1;
        for (int j = 0; j < k; ++j) {
            int best = -1;
            float bv = 0.f;
            for (int e = 0; e < E; ++e) {
                const float v = row[e];
                const bool after_prev = (v < pv) || (v == pv && e > pi);
                if (after_prev && (best < 0 || v > bv)) { best = e; bv = v; }
            }
            if (best < 0) best = (pi + 1 < E) ? pi + 1 : E - 1;   // unreachable for k <= E; keeps indices in range
            sel[j] = best;
            topk_idx[(size_t)t * k + j] = best;
            pv = bv;
            pi = best;
            atomicOr(&s_mask[best * NW + wave], 1ull << lane);
        }
        const double top = (double)row[sel[0]];
        double denom = 0.0;
        if (s.renorm) {
            for (int j = 0; j < k; ++j) denom += exp((double)row[sel[j]] - top);
        } else {
            for (int e = 0; e < E; ++e) denom += exp((double)row[e] - top);
        }
        for (int j = 0; j < k; ++j)
            gates[(size_t)t * k + j] = (float)(exp((double)row[sel[j]] - top) / denom);
    }
    __syncthreads();

    for (int e = tid; e < E; e += blockDim.x) {
        int c = 0;
        for (int w = 0; w < NW; ++w) c += __popcll(s_mask[e * NW + w]);
        p.block_counts[(size_t)b * E + e] = c;
    }
    if (active) {
        const unsigned long long below = (1ull << lane) - 1ull;
        for (int j = 0; j < k; ++j) {
            const int e = s_sel[tid * k + j];
            int r = 0;
            for (int w = 0; w < wave; ++w) r += __popcll(s_mask[e * NW + w]);
            r += __popcll(s_mask[e * NW + wave] & below);
            p.pos_final[(size_t)t * k + j] = r;     // rank inside the workgroup; finished by positions_kernel
        }
    }

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
                p.counts[e] = cnt;
                p.kept[e] = kp;
                p.offsets[e] = carry + incl - kp;
                s_off[e] = carry + incl - kp;
            }
            carry += __shfl(incl, kWave - 1, kWave);
        }
        if (lane == 0) {
            p.offsets[E] = carry;
            p.meta[META_R] = carry;
            p.meta[META_C] = C;
            p.meta[META_ALIVE] = 0;
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
            const int r = bb[e] + p.pos_final[(size_t)t * k + j];
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

__global__ void ws_init_kernel(int32_t *meta)
{
    if (threadIdx.x < META_SLOTS) meta[threadIdx.x] = 0;
}

// --------------------------------------------------------------- row movers

// Tokens [t0, t0+nt): each token row is read once and written to the STAGE row of
// every kept choice (read once / write up to k).  `lpr` lanes share a row.
__device__ __forceinline__ void pack_rows(const u32x4 *__restrict__ x, u32x4 *__restrict__ stage,
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
        for (int v0 = lane; v0 < vpr; v0 += lpr * kVecInFlight) {
            u32x4 val[kVecInFlight];
#pragma unroll
            for (int q = 0; q < kVecInFlight; ++q)
                if (v0 + q * lpr < vpr) val[q] = ld16(src + v0 + q * lpr);
            for (int j = 0; j < k; ++j) {
                const int ps = pos[j];
                if ((unsigned)ps >= (unsigned)s.max_rows) continue;   // dropped (-1) or not a row
                u32x4 *dst = stage + (size_t)ps * vpr;
#pragma unroll
                for (int q = 0; q < kVecInFlight; ++q)
                    if (v0 + q * lpr < vpr) st16(dst + v0 + q * lpr, val[q]);
            }
        }
    }
}

// STAGE rows [r0, r1) go to FINAL rows row_map[.]
__device__ __forceinline__ void regather_rows(const u32x4 *__restrict__ stage, u32x4 *__restrict__ fin,
                                              const int32_t *__restrict__ row_map, const Shape &s, int r0,
                                              int r1, int wg, int nwg)
{
    const int lpr = s.lpr, vpr = s.vpr;
    const int rows_per_wg = kMoverThreads / lpr;
    const int sub = threadIdx.x / lpr, lane = threadIdx.x - sub * lpr;
    if (r0 < 0) r0 = 0;
    if (r1 > s.max_rows) r1 = s.max_rows;
    for (int r = r0 + wg * rows_per_wg + sub; r < r1; r += nwg * rows_per_wg) {
        const int fr = row_map[r];
        if ((unsigned)fr >= (unsigned)s.max_rows) continue;
        const u32x4 *src = stage + (size_t)r * vpr;
        u32x4 *dst = fin + (size_t)fr * vpr;
        for (int v0 = lane; v0 < vpr; v0 += lpr * kVecInFlight) {
            u32x4 val[kVecInFlight];
#pragma unroll
            for (int q = 0; q < kVecInFlight; ++q)
                if (v0 + q * lpr < vpr) val[q] = ld16(src + v0 + q * lpr);
#pragma unroll
            for (int q = 0; q < kVecInFlight; ++q)
                if (v0 + q * lpr < vpr) st16(dst + v0 + q * lpr, val[q]);
        }
    }
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
    regather_rows(stage, fin, p.row_map, s, p.unit_rows[u0], p.unit_rows[u1], blockIdx.x, gridDim.x);
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
        regather_rows(stage, fin, p.row_map, s, p.unit_rows[u0], p.unit_rows[u1], idx, n_reg_wg);
}

// ------------------------------------------------------------------ combine

__device__ __forceinline__ double bf16_lo(unsigned int w) { return (double)__uint_as_float(w << 16); }
__device__ __forceinline__ double bf16_hi(unsigned int w) { return (double)__uint_as_float(w & 0xffff0000u); }

// fp64 -> bf16 bits, one rounding, nearest with ties to even, straight from the
// fp64 bit pattern (a detour through fp32 would round twice).
__device__ __forceinline__ unsigned int f64_to_bf16_rne(double d)
{
    const unsigned long long u = (unsigned long long)__double_as_longlong(d);
    const unsigned int sign = (unsigned int)(u >> 48) & 0x8000u;
    const int ex = (int)((u >> 52) & 0x7ff);
    const unsigned long long mant = u & 0x000fffffffffffffull;
    if (ex == 0x7ff) return sign | (mant ? 0x7fc0u : 0x7f80u);
    const int ef = ex - 1023 + 127;                 // biased exponent of the bf16 / fp32 format
    if (ef >= 255) return sign | 0x7f80u;
    if (ef <= 0) {
        // below the smallest normal: fixed spacing 2^-133; the scaling is exact
        const double q = __builtin_rint(__builtin_fabs(d) * 0x1p133);
        return sign | (unsigned int)q;              // q <= 128; 128 is the smallest normal
    }
    unsigned int r = ((unsigned int)ef << 7) | (unsigned int)(mant >> 45);
    const unsigned long long rem = mant & ((1ull << 45) - 1ull), half = 1ull << 44;
    r += (rem > half || (rem == half && (r & 1u))) ? 1u : 0u;   // a carry walks into the exponent, up to inf
    return sign | r;
}

// out[t] = sum_j gate[t,j] * y[pos_final[t,j]] over kept j in ascending order.
// The sum is carried in fp64 (every product of an fp32 gate with an fp32 / bf16
// element is exact there) and rounded once to the activation type, so the rounding
// decision is taken at the same precision as the CPU reference takes it.  fp64 FMA
// throughput is far above what the HBM stream of this kernel can feed.
// A dropped pair is skipped; a token with no kept pair writes zeros.
template <bool BF16>
__global__ __launch_bounds__(kMoverThreads) void combine_kernel(const u32x4 *__restrict__ y,
                                                                const float *__restrict__ gates,
                                                                u32x4 *__restrict__ out, PlanPtrs p, Shape s)
{
    constexpr int NV = 2;                       // 16-byte vectors per lane per pass
    constexpr int NF = BF16 ? 8 : 4;            // accumulators per vector
    const int lpr = s.lpr, vpr = s.vpr, k = s.k;
    const int rows_per_wg = kMoverThreads / lpr;
    const int sub = threadIdx.x / lpr, lane = threadIdx.x - sub * lpr;
    for (int t = blockIdx.x * rows_per_wg + sub; t < s.T; t += gridDim.x * rows_per_wg) {
        const int32_t *pos = p.pos_final + (size_t)t * k;
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
                    if (v0 + q * lpr < vpr) val[q] = ld16(src + v0 + q * lpr);
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
                    st16(dst + v0 + q * lpr, o);
                }
            }
        }
    }
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
            if (base + (size_t)q * kMoverThreads < nvec) val[q] = ld16(src + base + (size_t)q * kMoverThreads);
#pragma unroll
        for (int q = 0; q < kVecInFlight; ++q)
            if (base + (size_t)q * kMoverThreads < nvec) st16(dst + base + (size_t)q * kMoverThreads, val[q]);
    }
}

}  // namespace monta
