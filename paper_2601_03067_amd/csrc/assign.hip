// a3: thresholded arg-max assignment (Algorithm 1: "indices where sim(row) > thr", read as one target per right
// block: the left row with the largest cosine, lowest row on exact ties, strict '>').
//
// The other reading of the same line (rule KVFUSE_RULE_FIRST_ROW) follows the row loop literally: the first left row
// whose cosine is > thr takes the block.  It uses the same candidate lists: a listed row whose screened cosine is
// above thr + 2*band certainly qualifies, an unlisted one certainly does not, and only listed rows below the first
// certain one need the fp64 re-check, in ascending row order.
//
// Three kernels per height:
//   screen   one thread per right block.  The MFMA screen has left a short candidate list per column.  A column
//            with no candidate cannot fuse.  A column whose best candidate is clear of the threshold and of every
//            other candidate by more than 2*band is decided from the screen.  Everything else goes to a list.
//   refine   one wavefront per listed column: re-evaluation in fp64 on the stored values (wave-wide dot products
//            in a fixed lane order, so identical blocks give identical cosines and the lowest-row rule applies to
//            them exactly as on a CPU).
//   finalize one workgroup per (group, node): members grouped by target in ascending right index (CSR), evicted
//            blocks entered in the remap table, targets to rebuild appended to the merge work list, and the node's
//            surviving set cat(left, non-fused right in order) compacted in place for the parent node.
#include <algorithm>

#include "common.h"

namespace kvfuse {

__device__ __forceinline__ int find_node(const int32_t *__restrict__ base, int n_nodes, int idx)
{
    int lo = 0, hi = n_nodes;   // largest k with base[k] <= idx
    while (hi - lo > 1) {
        const int mid = (lo + hi) >> 1;
        if (base[mid] <= idx)
            lo = mid;
        else
            hi = mid;
    }
    return lo;
}

template <typename T>
__device__ __forceinline__ double cosine_f64(const T *__restrict__ pool_g, int r, const double *__restrict__ norm_g,
                                             int a, int b, int lane)
{
    const double na = norm_g[a], nb = norm_g[b];
    const uint4 *pa = reinterpret_cast<const uint4 *>(pool_g + (int64_t)a * r);
    const uint4 *pb = reinterpret_cast<const uint4 *>(pool_g + (int64_t)b * r);
    const int chunks = r / Elem<T>::PER16;
    double dot = 0.0;
    for (int c = lane; c < chunks; c += 64) {
        double x[Elem<T>::PER16], y[Elem<T>::PER16];
        Elem<T>::widen(pa[c], x);
        Elem<T>::widen(pb[c], y);
#pragma unroll
        for (int i = 0; i < Elem<T>::PER16; ++i)
            dot = fma(x[i], y[i], dot);
    }
    dot = wave_sum(dot);
    return (na == 0.0 || nb == 0.0) ? 0.0 : dot / (na * nb);
}

// The same cosine with the right block already in registers (raw 16-byte chunks, chunk c of this lane = chunk
// lane + 64 * c of the block): the re-check evaluates many left rows against one right block, and re-reading that
// block for every row doubled the traffic through L2.  Same order of operations as cosine_f64, so the two give
// bit-identical results.
template <typename T, int CPL>
__device__ __forceinline__ double cosine_f64_reg(const T *__restrict__ pool_g, int r, const double *__restrict__ norm_g,
                                                 int a, const uint4 *braw, double nb, int lane)
{
    const double na = norm_g[a];
    const uint4 *pa = reinterpret_cast<const uint4 *>(pool_g + (int64_t)a * r);
    const int chunks = r / Elem<T>::PER16;
    uint4 araw[CPL];
#pragma unroll
    for (int c = 0; c < CPL; ++c)
        araw[c] = pa[min(lane + 64 * c, chunks - 1)];
    double dot = 0.0;
#pragma unroll
    for (int c = 0; c < CPL; ++c) {
        if (lane + 64 * c < chunks) {
            double x[Elem<T>::PER16], y[Elem<T>::PER16];
            Elem<T>::widen(araw[c], x);
            Elem<T>::widen(braw[c], y);
#pragma unroll
            for (int i = 0; i < Elem<T>::PER16; ++i)
                dot = fma(x[i], y[i], dot);
        }
    }
    dot = wave_sum(dot);
    return (na == 0.0 || nb == 0.0) ? 0.0 : dot / (na * nb);
}

// KW such cosines side by side (rows a[0 .. n), n the same in every lane): the blocks of all rows are on their way
// together and the chains of fused multiply-adds are independent of each other, where one row after the other left a
// wavefront waiting on one load and one chain at a time.  Each cosine is built by the operations of cosine_f64_reg in
// their order, so the values are bit-identical to it.
template <typename T, int CPL, int KW>
__device__ __forceinline__ void cosines_f64_reg(const T *__restrict__ pool_g, int r, const double *__restrict__ norm_g,
                                                const int (&a)[KW], int n, const uint4 *braw, double nb, int lane, double (&cs)[KW])
{
    const int chunks = r / Elem<T>::PER16;
    uint4 araw[KW][CPL];
    double na[KW], dot[KW];
#pragma unroll
    for (int k = 0; k < KW; ++k) {
        dot[k] = 0.0;
        na[k] = 0.0;
        if (k < n) {
            na[k] = norm_g[a[k]];
            const uint4 *pa = reinterpret_cast<const uint4 *>(pool_g + (int64_t)a[k] * r);
#pragma unroll
            for (int c = 0; c < CPL; ++c)
                araw[k][c] = pa[min(lane + 64 * c, chunks - 1)];
        }
    }
#pragma unroll
    for (int c = 0; c < CPL; ++c) {
        if (lane + 64 * c < chunks) {
            double y[Elem<T>::PER16];
            Elem<T>::widen(braw[c], y);
#pragma unroll
            for (int k = 0; k < KW; ++k) {
                if (k < n) {
                    double x[Elem<T>::PER16];
                    Elem<T>::widen(araw[k][c], x);
#pragma unroll
                    for (int i = 0; i < Elem<T>::PER16; ++i)
                        dot[k] = fma(x[i], y[i], dot[k]);
                }
            }
        }
    }
#pragma unroll
    for (int k = 0; k < KW; ++k) {
        cs[k] = 0.0;
        if (k < n) {
            dot[k] = wave_sum(dot[k]);
            cs[k] = (na[k] == 0.0 || nb == 0.0) ? 0.0 : dot[k] / (na[k] * nb);
        }
    }
}

__global__ void assign_reset_kernel(WorkDesc w, int height)
{
    w.n_active[height] = 0;   // the finalize kernel appends to this list
    w.n_refine[height] = 0;   // the screen kernel appends to this one
}

// One THREAD per right block: everything the screen settles on its own (no candidate; or one candidate clear of the
// threshold and of all others by more than 2 * band).  Columns it cannot settle go to the re-check list.
// bound != 0: the listed values are not cosines but heads of upper bounds (prefix screen, fp8 screen): they settle nothing except
// "no candidate, no fusion", so every listed column goes to the re-check, which then evaluates all its candidates.
// bound == 2: the listed values are products of the fp8 copies: cosines to within band + err_a + err_b + err_a err_b, a
// radius that differs from candidate to candidate (q8_err holds err per block).  The same two-sided reasoning then works
// with an interval per candidate: a row is certain when its lower end clears thr + band, and it is the arg-max when its
// lower end lies above the upper end of every other listed row.
// The decision for column `id`; valid = the column exists, recheck = it goes to the list, else result is its assignment.
__device__ __forceinline__ void screen_column(const WorkDesc &w, const HeightDesc &h, double thr, double band, int rule, int bound,
                                              int P, int64_t id, bool &valid, bool &recheck_out, int &result_out, int64_t &cidx_out,
                                              int &node_out)
{
    const int g = (int)(id / h.total_r_cap);
    const int c = (int)(id - (int64_t)g * h.total_r_cap);
    const int node = find_node(h.r_base, h.n_nodes, c);
    const int j = c - h.r_base[node];
    const int ml = w.set_cnt[(int64_t)g * w.n_slots + h.l_slot[node]];
    const int mr = w.set_cnt[(int64_t)g * w.n_slots + h.r_slot[node]];
    if (j >= mr)
        return;
    valid = true;
    const int64_t cidx = (int64_t)g * w.r_stride + c;
    const int cnt = ml > 0 ? w.cand_cnt[cidx] : 0;
    int result = -1;
    bool recheck = cnt > w.cand_cap || ((bound == 1 || bound == 3) && cnt > 0);
    if (cnt > 0 && !recheck && bound == 2) {
        const float *qe = w.q8.err + (int64_t)g * P;
        const int32_t *l_ids = w.set_ids + (int64_t)g * w.n + h.l_off[node];
        const double eb = (double)qe[w.set_ids[(int64_t)g * w.n + h.r_off[node] + j]];
        auto radius = [&](int row) {
            const double ea = (double)qe[l_ids[row]];
            return band + ea + eb + ea * eb;
        };
        if (rule == KVFUSE_RULE_FIRST_ROW) {
            int i_def = 0x7FFFFFFF;
            for (int k = 0; k < cnt; ++k) {
                const int row = w.cand_idx[cidx * w.cand_cap + k];
                if ((double)w.cand_val[cidx * w.cand_cap + k] - radius(row) > thr + band)
                    i_def = min(i_def, row);
            }
            bool open = false;
            for (int k = 0; k < cnt; ++k) {
                const int row = w.cand_idx[cidx * w.cand_cap + k];
                open |= row < i_def && !((double)w.cand_val[cidx * w.cand_cap + k] - radius(row) > thr + band);
            }
            if (open || i_def == 0x7FFFFFFF)
                recheck = true;
            else
                result = i_def;
        } else {
            double lo_max = -INFINITY;
            int kmax = -1;
            for (int k = 0; k < cnt; ++k) {
                const double lo = (double)w.cand_val[cidx * w.cand_cap + k] - radius(w.cand_idx[cidx * w.cand_cap + k]);
                if (lo > lo_max) {
                    lo_max = lo;
                    kmax = k;
                }
            }
            bool alone = lo_max > thr + band;
            for (int k = 0; k < cnt; ++k)
                if (k != kmax)
                    alone &= (double)w.cand_val[cidx * w.cand_cap + k] + radius(w.cand_idx[cidx * w.cand_cap + k]) < lo_max;
            if (alone)
                result = w.cand_idx[cidx * w.cand_cap + kmax];
            else
                recheck = true;
        }
    } else if (cnt > 0 && !recheck && rule == KVFUSE_RULE_FIRST_ROW) {
        // lowest row that certainly clears the threshold; open = some undecided row comes before it
        int i_def = 0x7FFFFFFF;
        for (int k = 0; k < cnt; ++k)
            if ((double)w.cand_val[cidx * w.cand_cap + k] > thr + 2.0 * band)
                i_def = min(i_def, w.cand_idx[cidx * w.cand_cap + k]);
        bool open = false;
        for (int k = 0; k < cnt; ++k)
            open |= !((double)w.cand_val[cidx * w.cand_cap + k] > thr + 2.0 * band) &&
                    w.cand_idx[cidx * w.cand_cap + k] < i_def;
        if (open)
            recheck = true;
        else
            result = i_def;      // every list entry is either certain or open, so i_def is a row here
    } else if (cnt > 0 && !recheck) {
        float smax = -INFINITY;
        int imax = -1;
        for (int k = 0; k < cnt; ++k) {
            const float cv = w.cand_val[cidx * w.cand_cap + k];
            if (cv > smax) {
                smax = cv;
                imax = w.cand_idx[cidx * w.cand_cap + k];
            }
        }
        int contenders = 0;
        for (int k = 0; k < cnt; ++k)
            contenders += (double)w.cand_val[cidx * w.cand_cap + k] >= (double)smax - 2.0 * band;
        if (contenders == 1 && (double)smax > thr + 2.0 * band)
            result = imax;
        else
            recheck = true;
    }
    recheck_out = recheck;
    result_out = result;
    cidx_out = cidx;
    node_out = node;
}

__global__ __launch_bounds__(256) void assign_screen_kernel(WorkDesc w, HeightDesc h, int height, double thr, double band,
                                                            int rule, int bound, int P)
{
    __shared__ int wave_cnt[4];
    __shared__ int wg_base;
    const int64_t id = (int64_t)blockIdx.x * 256 + threadIdx.x;
    bool valid = false, recheck = false;
    int result = -1, node = 0;
    int64_t cidx = 0;
    if (id < (int64_t)w.G * h.total_r_cap)
        screen_column(w, h, thr, band, rule, bound, P, id, valid, recheck, result, cidx, node);
    // List entries are (column, node): the re-check need not search for the node again.  One atomic per workgroup, not
    // per column: with a screen whose listed values settle nothing every fusing column of a height lands in the list, and
    // that many atomics on one counter would take longer than everything else in this kernel.
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const unsigned long long listed = __ballot(valid && recheck);
    if (lane == 0)
        wave_cnt[wave] = __popcll(listed);
    __syncthreads();
    if (threadIdx.x == 0) {
        const int total = wave_cnt[0] + wave_cnt[1] + wave_cnt[2] + wave_cnt[3];
        wg_base = total > 0 ? atomicAdd(&w.n_refine[height], total) : 0;
    }
    __syncthreads();
    if (valid) {
        if (recheck) {
            int slot = wg_base + __popcll(listed & ((1ull << lane) - 1ull));
            for (int q = 0; q < wave; ++q)
                slot += wave_cnt[q];
            reinterpret_cast<int2 *>(w.refine)[slot] = make_int2((int32_t)cidx, node);
        } else {
            w.assign[cidx] = result;
        }
    }
}

// One WAVEFRONT per listed column: fp64 cosines of the contenders (or of the whole column when the candidate list
// overflowed), strict '>' against thr, lowest row on exact ties.
// CPL = 16-byte chunks of a block per lane when the right block is kept in registers (blocks up to 8 KiB), 0 = blocks
// too long for that: both operands are streamed.
template <typename T, int CPL>
__global__ __launch_bounds__(256) void assign_refine_kernel(PoolDesc pool, WorkDesc w, HeightDesc h, int height, double thr,
                                                            double band, int rule, int bound)
{
    constexpr int KW = CPL >= 8 ? 2 : 4;       // left rows multiplied side by side (cosines_f64_reg); two for the longest blocks, whose registers are full
    const int lane = threadIdx.x & 63;
    const int n_items = w.n_refine[height];
    const int n_waves = gridDim.x * 4;
    for (int it = blockIdx.x * 4 + (threadIdx.x >> 6); it < n_items; it += n_waves) {
        const int2 item = reinterpret_cast<const int2 *>(w.refine)[it];
        if (item.x < 0)         // settled by assign_q8_fill_kernel
            continue;
        const int64_t cidx = item.x;
        const int node = item.y;
        const int g = (int)(cidx / w.r_stride);
        const int c = (int)(cidx - (int64_t)g * w.r_stride);
        const int j = c - h.r_base[node];
        const int ml = w.set_cnt[(int64_t)g * w.n_slots + h.l_slot[node]];
        const int32_t *l_ids = w.set_ids + (int64_t)g * w.n + h.l_off[node];
        const int b = w.set_ids[(int64_t)g * w.n + h.r_off[node] + j];
        const T *pool_g = (const T *)pool.k + (int64_t)g * pool.P * pool.r;
        const double *norm_g = pool.norm_k + (int64_t)g * pool.P;
        const int cnt = w.cand_cnt[cidx];
        uint4 braw[CPL > 0 ? CPL : 1];
        double nb = 0.0;
        if constexpr (CPL > 0) {
            const uint4 *pb = reinterpret_cast<const uint4 *>(pool_g + (int64_t)b * pool.r);
            const int chunks = pool.r / Elem<T>::PER16;
#pragma unroll
            for (int q = 0; q < CPL; ++q)
                braw[q] = pb[min(lane + 64 * q, chunks - 1)];
            nb = norm_g[b];
        }
        auto cosine = [&](int a) __attribute__((always_inline)) {
            if constexpr (CPL > 0)
                return cosine_f64_reg<T, CPL>(pool_g, pool.r, norm_g, a, braw, nb, lane);
            else
                return cosine_f64<T>(pool_g, pool.r, norm_g, a, b, lane);
        };
        // radius of a listed value around the cosine: band, or (fp8 screen) band + the two copies' errors; per lane, for
        // the candidate that lane holds
        auto radius = [&](int row) __attribute__((always_inline)) {
            if (bound < 2)
                return band;
            const float *qe = w.q8.err + (int64_t)g * pool.P;
            const double ea = (double)qe[l_ids[row]], eb = (double)qe[b];
            return band + ea + eb + ea * eb;
        };
        double bv = -INFINITY;
        int bi = 0x7FFFFFFF;
        if (rule == KVFUSE_RULE_FIRST_ROW) {
            // bv ends as the cosine that decided the column: the taker's, or the largest one seen when no row takes it
            int win = -1;
            if (cnt <= w.cand_cap) {
                int ci = 0x7FFFFFFF;
                float cv = -INFINITY;
                if (lane < cnt) {
                    ci = w.cand_idx[cidx * w.cand_cap + lane];
                    cv = w.cand_val[cidx * w.cand_cap + lane];
                }
                const bool certain = bound >= 2 ? (lane < cnt && (double)cv - radius(ci) > thr + band)
                                                : (!bound && lane < cnt && (double)cv > thr + 2.0 * band);
                int i_def = certain ? ci : 0x7FFFFFFF;
#pragma unroll
                for (int off = 32; off >= 1; off >>= 1)
                    i_def = min(i_def, __shfl_xor(i_def, off, 64));
                unsigned long long open = __ballot(lane < cnt && !certain && ci < i_def);
                if constexpr (CPL > 0) {
                    while (open && win < 0) {
                        int rows[KW], a[KW], n = 0;
#pragma unroll
                        for (int k = 0; k < KW; ++k) {      // the lowest open rows come first
                            int i = ((open >> lane) & 1ull) ? ci : 0x7FFFFFFF;
#pragma unroll
                            for (int off = 32; off >= 1; off >>= 1)
                                i = min(i, __shfl_xor(i, off, 64));
                            const bool on = open != 0ull;
                            open &= ~__ballot(ci == i);
                            rows[k] = i;
                            a[k] = on ? l_ids[i] : 0;
                            n += on;
                        }
                        double cs[KW];
                        cosines_f64_reg<T, CPL, KW>(pool_g, pool.r, norm_g, a, n, braw, nb, lane, cs);
#pragma unroll
                        for (int k = 0; k < KW; ++k) {
                            if (k < n && win < 0) {
                                if (cs[k] > thr) {
                                    win = rows[k];
                                    bv = cs[k];
                                } else {
                                    bv = fmax(bv, cs[k]);
                                }
                            }
                        }
                    }
                } else {
                while (open) {
                    int i = ((open >> lane) & 1ull) ? ci : 0x7FFFFFFF;     // the lowest open row comes first
#pragma unroll
                    for (int off = 32; off >= 1; off >>= 1)
                        i = min(i, __shfl_xor(i, off, 64));
                    open &= ~__ballot(ci == i);
                    const double cs = cosine(l_ids[i]);
                    if (cs > thr) {
                        win = i;
                        bv = cs;
                        break;
                    }
                    bv = fmax(bv, cs);
                }
                }
                if (win < 0 && i_def != 0x7FFFFFFF) {
                    win = i_def;
                    bv = INFINITY;      // certain rows are more than band above thr
                }
            } else if constexpr (CPL > 0) {
                for (int i0 = 0; i0 < ml && win < 0; i0 += KW) {
                    const int n = min(KW, ml - i0);
                    int a[KW];
#pragma unroll
                    for (int k = 0; k < KW; ++k)
                        a[k] = l_ids[min(i0 + k, ml - 1)];
                    double cs[KW];
                    cosines_f64_reg<T, CPL, KW>(pool_g, pool.r, norm_g, a, n, braw, nb, lane, cs);
#pragma unroll
                    for (int k = 0; k < KW; ++k) {
                        if (k < n && win < 0) {
                            if (cs[k] > thr) {
                                win = i0 + k;
                                bv = cs[k];
                            } else {
                                bv = fmax(bv, cs[k]);
                            }
                        }
                    }
                }
            } else {
                for (int i = 0; i < ml; ++i) {
                    const double cs = cosine(l_ids[i]);
                    if (cs > thr) {
                        win = i;
                        bv = cs;
                        break;
                    }
                    bv = fmax(bv, cs);
                }
            }
            bi = win;                   // no taker: every cosine seen was <= thr, so the store below writes -1
        } else if (cnt <= w.cand_cap) {
            int ci = 0x7FFFFFFF;
            float cv = -INFINITY;
            if (lane < cnt) {
                ci = w.cand_idx[cidx * w.cand_cap + lane];
                cv = w.cand_val[cidx * w.cand_cap + lane];
            }
            float smax = cv;
#pragma unroll
            for (int off = 32; off >= 1; off >>= 1)
                smax = fmaxf(smax, __shfl_xor(smax, off, 64));
            unsigned long long mask;
            if (bound >= 2) {       // contenders: upper end not below the largest lower end
                const double rad = lane < cnt ? radius(ci) : 0.0;
                double lo = lane < cnt ? (double)cv - rad : -INFINITY;
#pragma unroll
                for (int off = 32; off >= 1; off >>= 1)
                    lo = fmax(lo, __shfl_xor(lo, off, 64));
                mask = __ballot(lane < cnt && (double)cv + rad >= lo);
            } else {
                mask = __ballot(lane < cnt && (bound || (double)cv >= (double)smax - 2.0 * band));
            }
            if constexpr (CPL > 0) {
                // Every contender costs one block read that nothing else shares, so the chain "row -> physical id ->
                // block -> dot product" is what a column waits for.  The ids of all contenders are fetched at once (one
                // per lane), and KW contenders are multiplied side by side.
                const int pid = lane < cnt ? l_ids[ci] : 0;
                while (mask) {
                    int src[KW], a[KW], n = 0;
#pragma unroll
                    for (int k = 0; k < KW; ++k) {
                        const bool on = mask != 0ull;
                        src[k] = on ? __ffsll((long long)mask) - 1 : 0;
                        if (on)
                            mask &= mask - 1;
                        a[k] = __shfl(pid, src[k], 64);
                        n += on;
                    }
                    double cs[KW];
                    cosines_f64_reg<T, CPL, KW>(pool_g, pool.r, norm_g, a, n, braw, nb, lane, cs);
#pragma unroll
                    for (int k = 0; k < KW; ++k) {
                        const int i = __shfl(ci, src[k], 64);
                        if (k < n && (cs[k] > bv || (cs[k] == bv && i < bi))) {
                            bv = cs[k];
                            bi = i;
                        }
                    }
                }
            } else {
                while (mask) {
                    const int src = __ffsll((long long)mask) - 1;
                    mask &= mask - 1;
                    const int i = __shfl(ci, src, 64);
                    const double cs = cosine(l_ids[i]);
                    if (cs > bv || (cs == bv && i < bi)) {
                        bv = cs;
                        bi = i;
                    }
                }
            }
        } else {
            // more screen candidates than slots: rescan the whole column (ascending rows, strict '>')
            if constexpr (CPL > 0) {
                for (int i0 = 0; i0 < ml; i0 += KW) {
                    const int n = min(KW, ml - i0);
                    int a[KW];
#pragma unroll
                    for (int k = 0; k < KW; ++k)
                        a[k] = l_ids[min(i0 + k, ml - 1)];
                    double cs[KW];
                    cosines_f64_reg<T, CPL, KW>(pool_g, pool.r, norm_g, a, n, braw, nb, lane, cs);
#pragma unroll
                    for (int k = 0; k < KW; ++k) {
                        if (k < n && cs[k] > bv) {
                            bv = cs[k];
                            bi = i0 + k;
                        }
                    }
                }
            } else {
                for (int i = 0; i < ml; ++i) {
                    const double cs = cosine(l_ids[i]);
                    if (cs > bv) {
                        bv = cs;
                        bi = i;
                    }
                }
            }
        }
        if (lane == 0) {
            w.assign[cidx] = (bv > thr && bi != 0x7FFFFFFF) ? bi : -1;
            int32_t *cn = w.counters + (int64_t)g * 8;
            if (fabs(bv - thr) <= band)
                atomicAdd(&cn[1], 1);
            atomicAdd(&cn[2], 1);
            if (cnt > w.cand_cap)
                atomicAdd(&cn[3], 1);
        }
    }
}

// 16 e4m3 bytes times 16 e4m3 bytes, accumulated in binary32 (every product is exact).
__device__ __forceinline__ float dot16_e4m3(const uint4 &a, const uint4 &b, float acc)
{
    typedef float floatx2 __attribute__((ext_vector_type(2)));
    const uint32_t wa[4] = {a.x, a.y, a.z, a.w}, wb[4] = {b.x, b.y, b.z, b.w};
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const floatx2 a0 = __builtin_amdgcn_cvt_pk_f32_fp8((int)wa[i], false), a1 = __builtin_amdgcn_cvt_pk_f32_fp8((int)wa[i], true);
        const floatx2 b0 = __builtin_amdgcn_cvt_pk_f32_fp8((int)wb[i], false), b1 = __builtin_amdgcn_cvt_pk_f32_fp8((int)wb[i], true);
        acc = fmaf(a0.x, b0.x, acc);
        acc = fmaf(a0.y, b0.y, acc);
        acc = fmaf(a1.x, b1.x, acc);
        acc = fmaf(a1.y, b1.y, acc);
    }
    return acc;
}

// Both screens on (bound == 3): the similarity step has listed heads of upper bounds over a prefix of the fp8 copies, which
// settle nothing.  One WAVEFRONT per listed column multiplies the whole copies of its candidates (r bytes each instead of
// the pool's r elements, binary32 arithmetic) and writes the results back into the list: from here on a listed value is a
// cosine to within band + err_a + err_b + err_a err_b, as with the fp8 screen alone.  Columns that these intervals settle
// (one row whose lower end clears thr + band and every other row's upper end; or no row whose upper end reaches
// thr - band; the row-order rule accordingly) are assigned here and struck from the list; the rest goes on to the fp64
// re-check with the new values.
__global__ __launch_bounds__(256) void assign_q8_fill_kernel(PoolDesc pool, WorkDesc w, HeightDesc h, int height, double thr,
                                                             double band, int rule)
{
    // A column's data hangs on a chain of dependent loads (list entry -> candidate count and column -> candidate row ->
    // physical id -> the copies).  A wavefront therefore takes kBatch list entries at a time and walks the chains of all of
    // them side by side, one entry per lane, before it multiplies their copies one entry after the other.
    constexpr int kBatch = 16;
    const int lane = threadIdx.x & 63;
    const int n_items = w.n_refine[height];
    const int n_waves = gridDim.x * 4;
    const int ch = pool.r / 16;
    for (int base = (blockIdx.x * 4 + (threadIdx.x >> 6)) * kBatch; base < n_items; base += n_waves * kBatch) {
        // ---- one list entry per lane: everything up to the first candidate's physical id
        int64_t m_cidx = -1;
        int m_node = 0, m_cnt = 0, m_g = 0, m_b = 0, m_ci0 = 0x7FFFFFFF, m_pid0 = 0;
        float m_eb = 0.0f, m_ea0 = 0.0f;
        if (lane < kBatch && base + lane < n_items) {
            const int2 item = reinterpret_cast<const int2 *>(w.refine)[base + lane];
            m_cidx = item.x;
            m_node = item.y;
            m_cnt = w.cand_cnt[m_cidx];
            m_g = (int)(m_cidx / w.r_stride);
            const int c = (int)(m_cidx - (int64_t)m_g * w.r_stride);
            m_b = w.set_ids[(int64_t)m_g * w.n + h.r_off[m_node] + (c - h.r_base[m_node])];
            m_ci0 = w.cand_idx[m_cidx * w.cand_cap];
            m_pid0 = w.set_ids[(int64_t)m_g * w.n + h.l_off[m_node] + m_ci0];
            m_eb = w.q8.err[(int64_t)m_g * pool.P + m_b];
            m_ea0 = w.q8.err[(int64_t)m_g * pool.P + m_pid0];
        }
        const int n_here = min(kBatch, n_items - base);
        for (int t = 0; t < n_here; ++t) {
            const int64_t cidx = __shfl(m_cidx, t, 64);
            const int node = __shfl(m_node, t, 64);
            const int cnt = __shfl(m_cnt, t, 64);
            if (cnt > w.cand_cap)           // overflowed list: the re-check rescans the whole column
                continue;
            const int g = __shfl(m_g, t, 64);
            const int b = __shfl(m_b, t, 64);
            const double eb = (double)__shfl(m_eb, t, 64);
            const int32_t *l_ids = w.set_ids + (int64_t)g * w.n + h.l_off[node];
            const uint8_t *q8_g = w.q8.k + (int64_t)g * pool.P * pool.r;
            const float *qe = w.q8.err + (int64_t)g * pool.P;
            const float *qs = w.q8.scale + (int64_t)g * pool.P;
            const float *qa = w.q8.alpha + (int64_t)g * pool.P;
            const float sb = qs[b], ab = qa[b];
            const uint4 *pb = reinterpret_cast<const uint4 *>(q8_g + (int64_t)b * pool.r);
            // candidates one per lane; the first one is already known
            const int ci0 = __shfl(m_ci0, t, 64), pid0 = __shfl(m_pid0, t, 64);
            const float ea0 = __shfl(m_ea0, t, 64);
            int ci = 0x7FFFFFFF, pid = 0;
            double ea = 0.0;
            float sa = 0.0f, aa = 0.0f;
            if (lane == 0) {
                ci = ci0;
                pid = pid0;
                ea = (double)ea0;
            } else if (lane < cnt) {
                ci = w.cand_idx[cidx * w.cand_cap + lane];
                pid = l_ids[ci];
                ea = (double)qe[pid];
            }
            if (lane < cnt) {
                sa = qs[pid];
                aa = qa[pid];
            }
            float cv = -INFINITY;
            for (int k = 0; k < cnt; ++k) {
                const uint4 *pa = reinterpret_cast<const uint4 *>(q8_g + (int64_t)__shfl(pid, k, 64) * pool.r);
                float dot = 0.0f;
                for (int q = lane; q < ch; q += 64)
                    dot = dot16_e4m3(pa[q], pb[q], dot);
#pragma unroll
                for (int off = 32; off >= 1; off >>= 1)
                    dot += __shfl_xor(dot, off, 64);
                if (lane == k)
                    cv = fmaf(dot * sa, sb, aa * ab);
            }
            double lo = -INFINITY, hi = -INFINITY;
            if (lane < cnt) {
                w.cand_val[cidx * w.cand_cap + lane] = cv;
                const double rad = band + ea + eb + ea * eb;
                lo = (double)cv - rad;
                hi = (double)cv + rad;
            }
            bool settled = false;
            int result = -1;
            if (rule == KVFUSE_RULE_FIRST_ROW) {
                const bool certain = lane < cnt && lo > thr + band;
                int i_def = certain ? ci : 0x7FFFFFFF;
#pragma unroll
                for (int off = 32; off >= 1; off >>= 1)
                    i_def = min(i_def, __shfl_xor(i_def, off, 64));
                const unsigned long long open = __ballot(lane < cnt && !certain && ci < i_def && !(hi < thr - band));
                settled = open == 0ull;
                result = i_def == 0x7FFFFFFF ? -1 : i_def;
            } else {
                double lo_max = lo, hi_max = hi;
#pragma unroll
                for (int off = 32; off >= 1; off >>= 1) {
                    lo_max = fmax(lo_max, __shfl_xor(lo_max, off, 64));
                    hi_max = fmax(hi_max, __shfl_xor(hi_max, off, 64));
                }
                const unsigned long long cont = __ballot(lane < cnt && hi >= lo_max);
                if (hi_max < thr - band) {
                    settled = true;
                } else if (__popcll(cont) == 1 && lo_max > thr + band) {
                    settled = true;
                    result = __shfl(ci, __ffsll((long long)cont) - 1, 64);
                }
            }
            if (settled && lane == 0) {
                w.assign[cidx] = result;
                reinterpret_cast<int2 *>(w.refine)[base + t] = make_int2(-1, node);
            }
        }
    }
}

__device__ __forceinline__ int ld_relaxed(const int32_t *p)
{
    return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

__global__ __launch_bounds__(256) void assign_finalize_kernel(int P, TableDesc tab, WorkDesc w, HeightDesc h, int height)
{
    __shared__ int64_t lds4[4];
    __shared__ int lds_base;
    const int g = blockIdx.x / h.n_nodes;
    const int node = blockIdx.x - g * h.n_nodes;
    const int tid = threadIdx.x;
    const int ml = w.set_cnt[(int64_t)g * w.n_slots + h.l_slot[node]];
    const int mr = w.set_cnt[(int64_t)g * w.n_slots + h.r_slot[node]];
    int32_t *l_ids = w.set_ids + (int64_t)g * w.n + h.l_off[node];
    int32_t *r_ids = w.set_ids + (int64_t)g * w.n + h.r_off[node];
    const int32_t *assign = w.assign + (int64_t)g * w.r_stride + h.r_base[node];
    int32_t *members = w.seg_members + (int64_t)g * w.r_stride + h.r_base[node];
    int32_t *seg_cnt = w.seg_cnt + (int64_t)g * w.l_stride + h.l_base[node];
    int32_t *seg_ptr = w.seg_ptr + (int64_t)g * w.l_stride + h.l_base[node];
    int32_t *seg_slot = w.seg_slot + (int64_t)g * w.l_stride + h.l_base[node];

    // 1. members per target
    for (int i = tid; i < ml; i += 256)
        seg_cnt[i] = 0;
    __syncthreads();
    for (int j = tid; j < mr; j += 256) {
        const int a = assign[j];
        if (a >= 0)
            atomicAdd(&seg_cnt[a], 1);
    }
    __syncthreads();

    // 2. segment offsets (exclusive scan) and the merge work list.  The node's targets get consecutive slots of the
    // height's list: they are counted first, so that one atomic reserves them all (a reservation per 256 rows cost a
    // round trip to memory each).
    int n_targets = 0;
    for (int i = tid; i < ml; i += 256)
        n_targets += ld_relaxed(&seg_cnt[i]) > 0;
    {
        int64_t total;
        (void)block_exscan_256((int64_t)n_targets, lds4, total);
        if (tid == 0)
            lds_base = total > 0 ? atomicAdd(&w.n_active[height], (int)total) : 0;
        __syncthreads();
    }
    const int slot_base = lds_base;
    int64_t run = 0;
    int slots = 0;
    for (int i0 = 0; i0 < ml; i0 += 256) {
        const int i = i0 + tid;
        const int cnt = i < ml ? ld_relaxed(&seg_cnt[i]) : 0;
        int64_t total;
        const int64_t pre = block_exscan_256(((int64_t)(cnt > 0) << 40) | (int64_t)cnt, lds4, total);
        if (i < ml) {
            const int start = (int)(run + (pre & 0xFFFFFFFFFFll));
            seg_ptr[i] = start;
            if (cnt > 0)
                seg_slot[i] = slot_base + slots + (int)(pre >> 40);
        }
        run += total & 0xFFFFFFFFFFll;
        slots += (int)(total >> 40);
        __syncthreads();
    }

    // 3. scatter right indices into their segments (seg_ptr runs on to the segment end), then order each segment
    for (int j = tid; j < mr; j += 256) {
        const int a = assign[j];
        if (a >= 0)
            members[atomicAdd(&seg_ptr[a], 1)] = j;
    }
    __syncthreads();
    for (int i = tid; i < ml; i += 256) {
        const int cnt = ld_relaxed(&seg_cnt[i]);
        if (cnt > 1) {
            const int start = ld_relaxed(&seg_ptr[i]) - cnt;
            for (int x = 1; x < cnt; ++x) {
                const int key = members[start + x];
                int y = x - 1;
                while (y >= 0) {
                    const int m = members[start + y];
                    if (m <= key)
                        break;
                    members[start + y + 1] = m;
                    --y;
                }
                members[start + y + 1] = key;
            }
        }
    }
    __syncthreads();
    // right index -> physical id, before the right set is compacted away
    for (int k = tid; k < (int)run; k += 256)
        members[k] = r_ids[members[k]];
    __syncthreads();
    // work-list records: target, count, member list and the first two members themselves
    for (int i = tid; i < ml; i += 256) {
        const int cnt = ld_relaxed(&seg_cnt[i]);
        if (cnt > 0) {
            const int start = ld_relaxed(&seg_ptr[i]) - cnt;
            const int a = l_ids[i];
            int4 *rec = w.active + 2 * (int64_t)seg_slot[i];
            rec[0] = make_int4(g, a, cnt, (int)((int64_t)g * w.r_stride + h.r_base[node] + start));
            rec[1] = make_int4(members[start], cnt > 1 ? members[start + 1] : a, 0, 0);
        }
    }

    // 4. remap of evicted blocks and in-place compaction of the survivors behind the left set
    int kept = 0;
    for (int j0 = 0; j0 < mr; j0 += 256) {
        const int j = j0 + tid;
        int id = -1, a = -1;
        if (j < mr) {
            id = r_ids[j];
            a = assign[j];
        }
        int64_t total;
        const int64_t pre = block_exscan_256((j < mr && a < 0) ? 1 : 0, lds4, total);   // barriers inside: all ids are read
        if (j < mr) {
            if (a >= 0)
                tab.remap[(int64_t)g * P + id] = l_ids[a];
            else
                l_ids[ml + kept + (int)pre] = id;
        }
        kept += (int)total;
        __syncthreads();
    }
    if (tid == 0) {
        w.set_cnt[(int64_t)g * w.n_slots + h.out_slot[node]] = ml + kept;
        if (mr - kept > 0)
            atomicAdd(&w.counters[(int64_t)g * 8 + 0], mr - kept);
    }
}

void launch_assign(hipStream_t s, const PoolDesc &pool, const TableDesc &tab, const WorkDesc &w, const HeightDesc &h,
                   int height, double thr, double band, int rule)
{
    const int64_t cols = (int64_t)w.G * h.total_r_cap;
    assign_reset_kernel<<<1, 1, 0, s>>>(w, height);
    if (cols > 0) {
        // 1: the listed values are upper bounds only (prefix screen); 2: cosines within a per-pair radius (fp8 screen);
        // 3: both screens: upper bounds that assign_q8_fill_kernel turns into the values of 2
        const bool prefix = w.screen_prefix > 0 && w.screen_prefix < pool.r;
        const int bound = prefix ? (w.q8.k ? 3 : 1) : (w.q8.k ? 2 : 0);
        assign_screen_kernel<<<(unsigned)((cols + 255) / 256), 256, 0, s>>>(w, h, height, thr, band, rule, bound, pool.P);
        if (bound == 3) {
            const unsigned fgrid = (unsigned)std::min<int64_t>((cols + 63) / 64, resident_workgroups(assign_q8_fill_kernel));
            assign_q8_fill_kernel<<<fgrid, 256, 0, s>>>(pool, w, h, height, thr, band, rule);
        }
        unsigned rgrid = 0;
        const int cpl = (pool.r / (pool.dtype == KVFUSE_BF16 ? 8 : 4) + 63) / 64;     // 16-byte chunks per lane
        // a persistent grid: exactly as many workgroups as the GPU holds at once (a workgroup that had to wait for a
        // free slot would start its share of the list when the others are nearly done)
#define KVF_REFINE(T, C)                                                                                         \
    do {                                                                                                         \
        rgrid = (unsigned)std::min<int64_t>((cols + 3) / 4, resident_workgroups(assign_refine_kernel<T, C>));    \
        assign_refine_kernel<T, C><<<rgrid, 256, 0, s>>>(pool, w, h, height, thr, band, rule, bound);                   \
    } while (0)
        if (pool.dtype == KVFUSE_BF16) {
            if (cpl <= 1) KVF_REFINE(bf16_t, 1);
            else if (cpl <= 2) KVF_REFINE(bf16_t, 2);
            else if (cpl <= 4) KVF_REFINE(bf16_t, 4);
            else if (cpl <= 8) KVF_REFINE(bf16_t, 8);
            else KVF_REFINE(bf16_t, 0);
        } else {
            if (cpl <= 1) KVF_REFINE(float, 1);
            else if (cpl <= 2) KVF_REFINE(float, 2);
            else if (cpl <= 4) KVF_REFINE(float, 4);
            else if (cpl <= 8) KVF_REFINE(float, 8);
            else KVF_REFINE(float, 0);
        }
#undef KVF_REFINE
    }
    if (w.G * h.n_nodes > 0)
        assign_finalize_kernel<<<(unsigned)(w.G * h.n_nodes), 256, 0, s>>>(pool.P, tab, w, h, height);
}

}  // namespace kvfuse
