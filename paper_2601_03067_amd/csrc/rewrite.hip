// a5: block-table rewrite (Algorithm 1: "evict fused blocks", "update block-table"; results section: the runner
// hands the scheduler the updated tables so that it can free unused blocks and raise reference counts).
//
// Integer gather/scatter, HBM-bound and small: one pass over the table follows the remap chain of each entry to
// its surviving block and recounts references; a second pass refreshes the per-logical scales; a per-group pass
// lists the freed ids in ascending order.
#include "common.h"

namespace kvfuse {

__global__ void rewrite_clear_kernel(int32_t *__restrict__ refcount, int64_t total)
{
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < total)
        refcount[i] = 0;
}

__global__ void rewrite_chase_kernel(TableDesc tab, int G, int P)
{
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= (int64_t)G * tab.n)
        return;
    const int64_t gp = (i / tab.n) * P;
    int p = tab.bt[i];
    if (p < 0 || p >= P)
        return;
    // A block fused at one height can be fused again higher up: follow the chain.  Its length is at most the
    // number of heights; the bound only guards against a malformed (cyclic) remap table.
    for (int hop = 0; hop < 64; ++hop) {
        const int q = tab.remap[gp + p];
        if (q < 0 || q >= P || q == p)
            break;
        p = q;
    }
    tab.bt[i] = p;
    atomicAdd(&tab.refcount[gp + p], 1);
}

__global__ void rewrite_scale_kernel(TableDesc tab, int G, int P, const double *__restrict__ norm_k,
                                     const double *__restrict__ norm_v)
{
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= (int64_t)G * tab.n)
        return;
    const int64_t gp = (i / tab.n) * P;
    const int p = tab.bt[i];
    if (p < 0 || p >= P)
        return;
    if (tab.refcount[gp + p] <= 1) {      // never fused: the entry still is its own raw block
        tab.scale_k[i] = 1.0f;
        tab.scale_v[i] = 1.0f;
        return;
    }
    const double nk = norm_k[gp + p], nv = norm_v[gp + p];
    tab.scale_k[i] = nk == 0.0 ? 0.0f : (float)(tab.orig_norm_k[i] / nk);
    tab.scale_v[i] = nv == 0.0 ? 0.0f : (float)(tab.orig_norm_v[i] / nv);
}

// One workgroup per group: freed ids (blocks that were fused away) in ascending order, and the live count.
__global__ __launch_bounds__(256) void rewrite_free_kernel(TableDesc tab, int P, int32_t *__restrict__ free_list,
                                                          int32_t *__restrict__ n_free, int32_t *__restrict__ n_phys)
{
    __shared__ int wave_tot[4];
    const int g = blockIdx.x, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int64_t gp = (int64_t)g * P;
    int freed = 0, live = 0;
    for (int p0 = 0; p0 < P; p0 += 256) {
        const int p = p0 + tid;
        const bool is_free = p < P && tab.remap[gp + p] >= 0;
        const bool is_live = p < P && tab.refcount[gp + p] > 0;
        const unsigned long long mf = __ballot(is_free);
        const unsigned long long ml = __ballot(is_live);
        __syncthreads();
        if (lane == 0)
            wave_tot[wave] = __popcll(mf);
        __syncthreads();
        int pre = 0, tot = 0;
        for (int k = 0; k < 4; ++k) {
            if (k < wave)
                pre += wave_tot[k];
            tot += wave_tot[k];
        }
        if (is_free && free_list)
            free_list[gp + freed + pre + __popcll(mf & ((1ull << lane) - 1ull))] = p;
        freed += tot;
        live += __popcll(ml);
    }
    // live counts are per wave: add them up
    __syncthreads();
    if (lane == 0)
        wave_tot[wave] = live;
    __syncthreads();
    if (tid == 0) {
        if (n_free)
            n_free[g] = freed;
        if (n_phys)
            n_phys[g] = wave_tot[0] + wave_tot[1] + wave_tot[2] + wave_tot[3];
    }
}

void launch_rewrite(hipStream_t s, const PoolDesc &pool, const TableDesc &tab, int32_t *free_list, int32_t *n_free,
                    int32_t *n_phys)
{
    const int64_t nb = (int64_t)pool.G * pool.P;
    const int64_t ne = (int64_t)pool.G * tab.n;
    if (nb > 0)
        rewrite_clear_kernel<<<(unsigned)((nb + 255) / 256), 256, 0, s>>>(tab.refcount, nb);
    if (ne > 0) {
        rewrite_chase_kernel<<<(unsigned)((ne + 255) / 256), 256, 0, s>>>(tab, pool.G, pool.P);
        rewrite_scale_kernel<<<(unsigned)((ne + 255) / 256), 256, 0, s>>>(tab, pool.G, pool.P, pool.norm_k, pool.norm_v);
    }
    if (pool.G > 0 && (free_list || n_free || n_phys))
        rewrite_free_kernel<<<(unsigned)pool.G, 256, 0, s>>>(tab, pool.P, free_list, n_free, n_phys);
}

}  // namespace kvfuse
