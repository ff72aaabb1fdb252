// a1: block norms and table initialisation (method section: every block vector keeps its norm; leaf step of
// Algorithm 1).  Pure HBM stream: every K and V byte is read once; one wavefront per block, 16-byte loads,
// fp64 accumulation in a fixed order so that identical blocks get bit-identical norms.
#include <algorithm>

#include "common.h"

namespace kvfuse {

template <typename T>
__global__ __launch_bounds__(256) void block_norms_kernel(const T *__restrict__ kpool, const T *__restrict__ vpool,
                                                          int64_t n_blocks, int r, double *__restrict__ norm_k,
                                                          double *__restrict__ norm_v, float *__restrict__ inv_norm_k,
                                                          float *__restrict__ rem, int prefix_chunks)
{
    const int lane = threadIdx.x & 63;
    const int64_t w = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);   // wave index over 2 * n_blocks
    if (w >= 2 * n_blocks)
        return;
    const bool is_v = w >= n_blocks;
    const int64_t b = is_v ? w - n_blocks : w;
    const uint4 *src = reinterpret_cast<const uint4 *>((is_v ? vpool : kpool) + b * (int64_t)r);
    const int chunks = r / Elem<T>::PER16;
    // st: the squares beyond the prefix of the prefix screen, summed on their own (rem = |tail| / |block|, see
    // prefix_tails_kernel); the norm's own sum keeps its order
    const bool want_tail = rem != nullptr && !is_v;
    double ss = 0.0, st = 0.0;
    for (int c = lane; c < chunks; c += 64) {
        const uint4 raw = src[c];
        double x[Elem<T>::PER16];
        Elem<T>::widen(raw, x);
#pragma unroll
        for (int i = 0; i < Elem<T>::PER16; ++i)
            ss = fma(x[i], x[i], ss);
        if (want_tail && c >= prefix_chunks) {
#pragma unroll
            for (int i = 0; i < Elem<T>::PER16; ++i)
                st = fma(x[i], x[i], st);
        }
    }
    ss = wave_sum(ss);
    if (want_tail)
        st = wave_sum(st);
    if (lane == 0) {
        const double nrm = sqrt(ss);
        if (is_v) {
            norm_v[b] = nrm;
        } else {
            norm_k[b] = nrm;
            inv_norm_k[b] = nrm > 0.0 ? (float)(1.0 / nrm) : 0.0f;
            if (want_tail)
                rem[b] = tail_share(st, nrm);
        }
    }
}

__global__ void table_clear_kernel(int32_t *__restrict__ refcount, int32_t *__restrict__ remap, int64_t total)
{
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < total) {
        refcount[i] = 0;
        remap[i] = -1;
    }
}

__global__ void table_init_kernel(TableDesc tab, int G, int P, const double *__restrict__ norm_k,
                                  const double *__restrict__ norm_v)
{
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= (int64_t)G * tab.n)
        return;
    const int g = (int)(i / tab.n);
    const int p = tab.bt[i];
    if (p < 0 || p >= P) {       // invalid id: leave a poisoned entry rather than touch memory out of range
        tab.orig_norm_k[i] = 0.0;
        tab.orig_norm_v[i] = 0.0;
        tab.scale_k[i] = 0.0f;
        tab.scale_v[i] = 0.0f;
        return;
    }
    tab.orig_norm_k[i] = norm_k[(int64_t)g * P + p];
    tab.orig_norm_v[i] = norm_v[(int64_t)g * P + p];
    tab.scale_k[i] = 1.0f;
    tab.scale_v[i] = 1.0f;
    atomicAdd(&tab.refcount[(int64_t)g * P + p], 1);
}

void launch_block_norms(hipStream_t s, const PoolDesc &pool, const TableDesc &tab, float *rem, int prefix)
{
    const int pchunks = prefix / (pool.dtype == KVFUSE_BF16 ? 8 : 4);
    const int64_t nb = (int64_t)pool.G * pool.P;
    const unsigned grid = (unsigned)((2 * nb + 3) / 4);
    if (nb > 0) {
        if (pool.dtype == KVFUSE_BF16)
            block_norms_kernel<bf16_t><<<grid, 256, 0, s>>>((const bf16_t *)pool.k, (const bf16_t *)pool.v, nb, pool.r,
                                                            pool.norm_k, pool.norm_v, pool.inv_norm_k, rem, pchunks);
        else
            block_norms_kernel<float><<<grid, 256, 0, s>>>((const float *)pool.k, (const float *)pool.v, nb, pool.r,
                                                           pool.norm_k, pool.norm_v, pool.inv_norm_k, rem, pchunks);
        table_clear_kernel<<<(unsigned)((nb + 255) / 256), 256, 0, s>>>(tab.refcount, tab.remap, nb);
    }
    const int64_t ne = (int64_t)pool.G * tab.n;
    if (ne > 0)
        table_init_kernel<<<(unsigned)((ne + 255) / 256), 256, 0, s>>>(tab, pool.G, pool.P, pool.norm_k, pool.norm_v);
}

// Leaf sets = physical ids of the leaves' logical entries, each leaf at the region the plan gave it (leaf_src maps
// a set position back to its logical entry).  An id outside [0, P) (a caller error) is clamped so that no later
// kernel can read out of range, and counted in counters[g][4].
__global__ void leaf_sets_kernel(WorkDesc w, int P, const int32_t *__restrict__ bt, const int32_t *__restrict__ slot_init)
{
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    const int64_t ne = (int64_t)w.G * w.n;
    if (i < (int64_t)w.G * 8)
        w.counters[i] = 0;
    if (i < ne) {
        const int64_t g = i / w.n;
        const int src = w.leaf_src[i - g * w.n];
        int p = src >= 0 ? bt[g * w.n + src] : 0;
        if (p < 0 || p >= P)
            p = p < 0 ? 0 : P - 1;
        w.set_ids[i] = p;
    }
    const int64_t ns = (int64_t)w.G * w.n_slots;
    if (i < ns)
        w.set_cnt[i] = slot_init[i % w.n_slots];
}

// Caller errors that the tree cannot work with are counted per group: ids outside [0, P) in counters[g][4], and entries
// whose block is also held by another entry in counters[g][5] (Algorithm 1 starts from unshared blocks: a shared block
// would sit in several sets of one height and be rewritten by one node while another reads it).  refcount is the
// count the norm pass has just taken.
__global__ void check_ids_kernel(WorkDesc w, int P, const int32_t *__restrict__ bt, const int32_t *__restrict__ refcount)
{
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < (int64_t)w.G * w.n) {
        const int p = bt[i];
        const int64_t g = i / w.n;
        if (p < 0 || p >= P)
            atomicAdd(&w.counters[g * 8 + 4], 1);
        else if (refcount[g * P + p] > 1)
            atomicAdd(&w.counters[g * 8 + 5], 1);
    }
}

void launch_leaf_sets(hipStream_t s, const WorkDesc &w, const TableDesc &tab, int P, const int32_t *slot_init)
{
    int64_t total = (int64_t)w.G * w.n;
    const int64_t ns = (int64_t)w.G * w.n_slots;
    if (ns > total)
        total = ns;
    if ((int64_t)w.G * 8 > total)
        total = (int64_t)w.G * 8;
    if (total > 0)
        leaf_sets_kernel<<<(unsigned)((total + 255) / 256), 256, 0, s>>>(w, P, tab.bt, slot_init);
    if ((int64_t)w.G * w.n > 0)
        check_ids_kernel<<<(unsigned)(((int64_t)w.G * w.n + 255) / 256), 256, 0, s>>>(w, P, tab.bt, tab.refcount);
}

// Prefix screen (similarity.hip): rem[b] = |tail of block b| / |block b| for the key blocks, where the tail is everything
// beyond the first `prefix` elements.  The norm pass and the merge step write it along with the norms (tail_share in
// common.h); this kernel does the same for a caller who runs the steps one by one (kvfuse_leaf_sets): fp64 sum of the
// tail squares against the stored norm, one wavefront per block.
template <typename T>
__global__ __launch_bounds__(256) void prefix_tails_kernel(const T *__restrict__ k, const double *__restrict__ norm_k, int64_t n_blocks,
                                                           int r, int prefix, float *__restrict__ rem)
{
    const int lane = threadIdx.x & 63;
    const int64_t stride = (int64_t)gridDim.x * 4;
    for (int64_t b = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6); b < n_blocks; b += stride) {
        const uint4 *p = reinterpret_cast<const uint4 *>(k + b * r);
        const int chunks = r / Elem<T>::PER16;
        double st = 0.0;
        for (int c = prefix / Elem<T>::PER16 + lane; c < chunks; c += 64) {
            double x[Elem<T>::PER16];
            Elem<T>::widen(p[c], x);
#pragma unroll
            for (int e = 0; e < Elem<T>::PER16; ++e)
                st = fma(x[e], x[e], st);
        }
        st = wave_sum(st);
        if (lane == 0)
            rem[b] = tail_share(st, norm_k[b]);
    }
}

void launch_prefix_tails(hipStream_t s, const PoolDesc &pool, const WorkDesc &w)
{
    if (w.screen_prefix <= 0 || !w.rem_k)
        return;
    const int64_t nb = (int64_t)pool.G * pool.P;
    if (nb <= 0)
        return;
    const unsigned grid = (unsigned)std::min<int64_t>((nb + 3) / 4, 256 * 16);
    if (pool.dtype == KVFUSE_BF16)
        prefix_tails_kernel<bf16_t><<<grid, 256, 0, s>>>((const bf16_t *)pool.k, pool.norm_k, nb, pool.r, w.screen_prefix, w.rem_k);
    else
        prefix_tails_kernel<float><<<grid, 256, 0, s>>>((const float *)pool.k, pool.norm_k, nb, pool.r, w.screen_prefix, w.rem_k);
}

}  // namespace kvfuse
