// a1: block norms and table initialisation (method section: every block vector keeps its norm; leaf step of
// Algorithm 1).  Pure HBM stream: every K and V byte is read once; one wavefront per block, 16-byte loads,
// fp64 accumulation in a fixed order so that identical blocks get bit-identical norms.
#include <algorithm>

#include "common.h"

namespace kvfuse {

// fp8 screen (similarity.hip): the e4m3 copy of a key block, q = e4m3(x / |x| * kQ8Scale) element by element, and the
// error it really has, err = | x / |x| - decode(q) / kQ8Scale | as a Euclidean norm in fp64, rounded up with a margin.
// The similarity kernel adds err(a) + err(b) + err(a) err(b) to the product of two copies, which bounds their cosine from
// above whatever the conversion did (the decode used here is the hardware's, the one the matrix cores apply).  One
// wavefront per block.  A block of norm 0 becomes zeros with err 0 (its cosines are 0 by definition).
template <typename T>
__device__ __forceinline__ void quantise_block(const T *__restrict__ src, double nrm, uint8_t *__restrict__ dst,
                                               float *__restrict__ err_out, int r, int lane)
{
    constexpr int PER = Elem<T>::PER16;
    const int chunks = r / PER;
    const double inv = nrm > 0.0 ? 1.0 / nrm : 0.0;
    const float mf = (float)((double)kQ8Scale * inv);
    const uint4 *p = reinterpret_cast<const uint4 *>(src);
    double se = 0.0;
    for (int c = lane; c < chunks; c += 64)
        quantise_chunk<T>(p[c], inv, mf, dst + (size_t)c * PER, se);
    se = wave_sum(se);
    if (lane == 0)
        *err_out = quantise_error(se, nrm);
}

// KEEP > 0 (fp8 screen on, blocks of at most 64 * KEEP chunks): the wavefront of a key block holds the block in registers,
// so the one-byte copy, which needs the norm first, costs no second read.
template <typename T, int KEEP>
__global__ __launch_bounds__(256) void block_norms_kernel(const T *__restrict__ kpool, const T *__restrict__ vpool,
                                                          int64_t n_blocks, int r, double *__restrict__ norm_k,
                                                          double *__restrict__ norm_v, float *__restrict__ inv_norm_k,
                                                          float *__restrict__ rem, int prefix_chunks, uint8_t *__restrict__ q8,
                                                          float *__restrict__ q8_err)
{
    constexpr int PER = Elem<T>::PER16;
    const int lane = threadIdx.x & 63;
    const int64_t w = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);   // wave index over 2 * n_blocks
    if (w >= 2 * n_blocks)
        return;
    const bool is_v = w >= n_blocks;
    const int64_t b = is_v ? w - n_blocks : w;
    const uint4 *src = reinterpret_cast<const uint4 *>((is_v ? vpool : kpool) + b * (int64_t)r);
    const int chunks = r / PER;
    // st: the squares beyond the prefix of the prefix screen, summed on their own (rem = |tail| / |block|, see
    // prefix_tails_kernel); the norm's own sum keeps its order
    const bool want_tail = rem != nullptr && !is_v;
    double ss = 0.0, st = 0.0;
    uint4 keep[KEEP > 0 ? KEEP : 1];
    if (KEEP > 0 && !is_v) {
#pragma unroll
        for (int q = 0; q < KEEP; ++q)
            keep[q] = src[min(lane + 64 * q, chunks - 1)];
#pragma unroll
        for (int q = 0; q < KEEP; ++q) {
            const int c = lane + 64 * q;
            if (c < chunks) {
                double x[PER];
                Elem<T>::widen(keep[q], x);
#pragma unroll
                for (int i = 0; i < PER; ++i)
                    ss = fma(x[i], x[i], ss);
                if (want_tail && c >= prefix_chunks) {
#pragma unroll
                    for (int i = 0; i < PER; ++i)
                        st = fma(x[i], x[i], st);
                }
            }
        }
    } else {
        for (int c = lane; c < chunks; c += 64) {
            const uint4 raw = src[c];
            double x[PER];
            Elem<T>::widen(raw, x);
#pragma unroll
            for (int i = 0; i < PER; ++i)
                ss = fma(x[i], x[i], ss);
            if (want_tail && c >= prefix_chunks) {
#pragma unroll
                for (int i = 0; i < PER; ++i)
                    st = fma(x[i], x[i], st);
            }
        }
    }
    ss = wave_sum(ss);
    if (want_tail)
        st = wave_sum(st);
    const double nrm = sqrt(ss);
    if (lane == 0) {
        if (is_v) {
            norm_v[b] = nrm;
        } else {
            norm_k[b] = nrm;
            inv_norm_k[b] = nrm > 0.0 ? (float)(1.0 / nrm) : 0.0f;
            if (want_tail)
                rem[b] = tail_share(st, nrm);
        }
    }
    // fp8 screen: the one-byte copy of the key block (from the registers, or for long blocks in a second walk while the
    // block is still in the cache)
    if (q8 != nullptr && !is_v) {
        if constexpr (KEEP > 0) {
            const double inv = nrm > 0.0 ? 1.0 / nrm : 0.0;
            const float mf = (float)((double)kQ8Scale * inv);
            double se = 0.0;
#pragma unroll
            for (int q = 0; q < KEEP; ++q) {
                const int c = lane + 64 * q;
                if (c < chunks)
                    quantise_chunk<T>(keep[q], inv, mf, q8 + b * (int64_t)r + (size_t)c * PER, se);
            }
            se = wave_sum(se);
            if (lane == 0)
                q8_err[b] = quantise_error(se, nrm);
        } else {
            quantise_block<T>((const T *)kpool + b * (int64_t)r, nrm, q8 + b * (int64_t)r, q8_err + b, r, lane);
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

void launch_block_norms(hipStream_t s, const PoolDesc &pool, const TableDesc &tab, float *rem, int prefix, uint8_t *q8, float *q8_err)
{
    const int pchunks = prefix / (pool.dtype == KVFUSE_BF16 ? 8 : 4);
    const int64_t nb = (int64_t)pool.G * pool.P;
    const unsigned grid = (unsigned)((2 * nb + 3) / 4);
    if (nb > 0) {
        const int chunks = pool.r / (pool.dtype == KVFUSE_BF16 ? 8 : 4);
        const int keep = !q8 ? 0 : (chunks <= 256 ? 4 : (chunks <= 512 ? 8 : 0));
#define KVF_NORMS(T, KEEP)                                                                                              \
    block_norms_kernel<T, KEEP><<<grid, 256, 0, s>>>((const T *)pool.k, (const T *)pool.v, nb, pool.r, pool.norm_k, pool.norm_v, \
                                                     pool.inv_norm_k, rem, pchunks, q8, q8_err)
        if (pool.dtype == KVFUSE_BF16) {
            if (keep == 4) KVF_NORMS(bf16_t, 4);
            else if (keep == 8) KVF_NORMS(bf16_t, 8);
            else KVF_NORMS(bf16_t, 0);
        } else {
            if (keep == 4) KVF_NORMS(float, 4);
            else if (keep == 8) KVF_NORMS(float, 8);
            else KVF_NORMS(float, 0);
        }
#undef KVF_NORMS
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

template <typename T>
__global__ __launch_bounds__(256) void quantise_all_kernel(const T *__restrict__ k, const double *__restrict__ norm_k, int64_t n_blocks,
                                                           int r, uint8_t *__restrict__ q8, float *__restrict__ q8_err)
{
    const int64_t b = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    if (b < n_blocks)
        quantise_block<T>(k + b * r, norm_k[b], q8 + b * r, q8_err + b, r, threadIdx.x & 63);
}

// The targets that the merge step of this height has rebuilt (the work list of the assignment step).
template <typename T>
__global__ __launch_bounds__(256) void quantise_targets_kernel(PoolDesc pool, WorkDesc w, int height)
{
    const int n_act = w.n_active[height];
    const int stride = gridDim.x * 4;
    for (int t = blockIdx.x * 4 + (threadIdx.x >> 6); t < n_act; t += stride) {
        const int4 rec = w.active[2 * (int64_t)t];
        const int64_t b = (int64_t)rec.x * pool.P + rec.y;
        quantise_block<T>((const T *)pool.k + b * pool.r, pool.norm_k[b], w.q8_k + b * pool.r, w.q8_err + b, pool.r, threadIdx.x & 63);
    }
}

void launch_quantise_all(hipStream_t s, const PoolDesc &pool, const WorkDesc &w)
{
    const int64_t nb = (int64_t)pool.G * pool.P;
    if (!w.q8_k || nb <= 0)
        return;
    const unsigned grid = (unsigned)((nb + 3) / 4);
    if (pool.dtype == KVFUSE_BF16)
        quantise_all_kernel<bf16_t><<<grid, 256, 0, s>>>((const bf16_t *)pool.k, pool.norm_k, nb, pool.r, w.q8_k, w.q8_err);
    else
        quantise_all_kernel<float><<<grid, 256, 0, s>>>((const float *)pool.k, pool.norm_k, nb, pool.r, w.q8_k, w.q8_err);
}

void launch_quantise_targets(hipStream_t s, const PoolDesc &pool, const WorkDesc &w, int height)
{
    if (!w.q8_k || (int64_t)w.G * w.l_stride <= 0)
        return;
    const unsigned grid = (unsigned)std::min<int64_t>(((int64_t)w.G * w.l_stride + 3) / 4, 256 * 8);
    if (pool.dtype == KVFUSE_BF16)
        quantise_targets_kernel<bf16_t><<<grid, 256, 0, s>>>(pool, w, height);
    else
        quantise_targets_kernel<float><<<grid, 256, 0, s>>>(pool, w, height);
}

}  // namespace kvfuse
