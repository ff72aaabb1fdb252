// a1: block norms and table initialisation (method section: every block vector keeps its norm; leaf step of
// Algorithm 1).  Pure HBM stream: every K and V byte is read once; one wavefront per block, 16-byte loads,
// fp64 accumulation in a fixed order so that identical blocks get bit-identical norms.
#include <algorithm>

#include "common.h"

namespace kvfuse {

// fp8 screen (similarity.hip): the one-byte copy of a key block and what goes with it (Q8Desc in common.h).  With
// u = x / |x|: alpha = <m, u> rounded to binary32 (0 without a direction m), u_c = u - alpha m, the copy holds
// e4m3(u_c * kQ8Scale / |u_c|) element by element, and err bounds what the similarity kernel's value
// <copy_a, copy_b> scale_a scale_b + alpha_a alpha_b can miss of the cosine: the Euclidean distance between u_c and the
// decoded copy (measured on the bytes written, with the hardware's own decode, the one the matrix cores apply), plus a
// margin for the binary32 arithmetic of the measurement and for what the rounding of alpha and of m's norm take from
// the identity <u, v> = <u_c, v_c> + alpha_u alpha_v (quantise_error in common.h), rounded up.  Taking the
// common direction out first matters when unrelated blocks share one: the copies then spend their eight bits on what
// tells the blocks apart.  One wavefront per block.  A block of norm 0 becomes zeros with err 0 (its cosines are 0 by
// definition).
template <typename T>
__device__ __forceinline__ void quantise_block(const T *__restrict__ src, double nrm, const float *__restrict__ dir_g,
                                               uint8_t *__restrict__ dst, float *__restrict__ err_out, float *__restrict__ scale_out,
                                               float *__restrict__ alpha_out, int r, int lane)
{
    constexpr int PER = Elem<T>::PER16;
    const int chunks = r / PER;
    const uint4 *p = reinterpret_cast<const uint4 *>(src);
    double sm = 0.0;
    if (dir_g) {
        for (int c = lane; c < chunks; c += 64)
            q8_dir_dot_chunk<T>(p[c], dir_g, c * PER, sm);
        sm = wave_sum(sm);
    }
    const Q8Block blk = q8_block(nrm, dir_g != nullptr, sm);
    float se32 = 0.0f;
    for (int c = lane; c < chunks; c += 64)
        quantise_chunk<T>(p[c], dir_g, c * PER, blk, dst + (size_t)c * PER, se32);
    const double se = wave_sum((double)se32);
    if (lane == 0) {
        *err_out = quantise_error(se, blk, nrm);
        *scale_out = (float)blk.scale;
        *alpha_out = nrm > 0.0 ? (float)blk.alpha : 0.0f;
    }
}

// KEEP > 0 (fp8 screen on, blocks of at most 64 * KEEP chunks): the wavefront of a key block holds the block in registers,
// so the one-byte copy, which needs the norm first, costs no second read.
template <typename T, int KEEP>
__global__ __launch_bounds__(256) void block_norms_kernel(const T *__restrict__ kpool, const T *__restrict__ vpool,
                                                          int64_t n_blocks, int r, double *__restrict__ norm_k,
                                                          double *__restrict__ norm_v, float *__restrict__ inv_norm_k,
                                                          float *__restrict__ rem, int prefix_chunks, Q8Desc q8, int P)
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
    double ss = 0.0, st = 0.0, sm = 0.0;
    const float *dir_g = (KEEP > 0 && !is_v && q8.dir) ? q8.dir + (b / P) * (int64_t)r : nullptr;
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
                if (dir_g)
                    q8_dir_dot_chunk<T>(keep[q], dir_g, c * PER, sm);
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
    if (q8.k != nullptr && !is_v) {
        if constexpr (KEEP > 0) {
            if (dir_g)
                sm = wave_sum(sm);
            const Q8Block blk = q8_block(nrm, dir_g != nullptr, sm);
            float se32 = 0.0f;
#pragma unroll
            for (int q = 0; q < KEEP; ++q) {
                const int c = lane + 64 * q;
                if (c < chunks)
                    quantise_chunk<T>(keep[q], dir_g, c * PER, blk, q8.k + b * (int64_t)r + (size_t)c * PER, se32);
            }
            const double se = wave_sum((double)se32);
            if (lane == 0) {
                q8.err[b] = quantise_error(se, blk, nrm);
                q8.scale[b] = (float)blk.scale;
                q8.alpha[b] = nrm > 0.0 ? (float)blk.alpha : 0.0f;
            }
        } else {
            quantise_block<T>((const T *)kpool + b * (int64_t)r, nrm, q8.dir ? q8.dir + (b / P) * (int64_t)r : nullptr,
                              q8.k + b * (int64_t)r, q8.err + b, q8.scale + b, q8.alpha + b, r, lane);
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

void launch_block_norms(hipStream_t s, const PoolDesc &pool, const TableDesc &tab, float *rem, int prefix, const Q8Desc *q8p)
{
    Q8Desc q8 = {};
    if (q8p)
        q8 = *q8p;
    const int pchunks = prefix / (pool.dtype == KVFUSE_BF16 ? 8 : 4);
    const int64_t nb = (int64_t)pool.G * pool.P;
    const unsigned grid = (unsigned)((2 * nb + 3) / 4);
    if (nb > 0) {
        const int chunks = pool.r / (pool.dtype == KVFUSE_BF16 ? 8 : 4);
        const int keep = !q8.k ? 0 : (chunks <= 256 ? 4 : (chunks <= 512 ? 8 : 0));
#define KVF_NORMS(T, KEEP)                                                                                              \
    block_norms_kernel<T, KEEP><<<grid, 256, 0, s>>>((const T *)pool.k, (const T *)pool.v, nb, pool.r, pool.norm_k, pool.norm_v, \
                                                     pool.inv_norm_k, rem, pchunks, q8, pool.P)
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

// Caller errors that the tree cannot work with are counted per group: ids outside [0, P) in counters[g][4], entries
// whose block is also held by another entry in counters[g][5] (Algorithm 1 starts from unshared blocks: a shared block
// would sit in several sets of one height and be rewritten by one node while another reads it), and in counters[g][6]
// key blocks whose norm is not finite or, unless zero, outside [2^-40, 2^40]: the similarity screen multiplies the
// stored values in binary32, where products of such blocks underflow or overflow, so that a pair could be missed.
// refcount is the count the norm pass has just taken.
__global__ void check_ids_kernel(WorkDesc w, int P, const int32_t *__restrict__ bt, const int32_t *__restrict__ refcount,
                                 const double *__restrict__ norm_k)
{
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < (int64_t)w.G * w.n) {
        const int p = bt[i];
        const int64_t g = i / w.n;
        if (p < 0 || p >= P) {
            atomicAdd(&w.counters[g * 8 + 4], 1);
        } else {
            if (refcount[g * P + p] > 1)
                atomicAdd(&w.counters[g * 8 + 5], 1);
            const double nk = norm_k[g * P + p];
            if (nk != 0.0 && !(nk >= 0x1p-40 && nk <= 0x1p40))
                atomicAdd(&w.counters[g * 8 + 6], 1);
        }
    }
}

void launch_leaf_sets(hipStream_t s, const WorkDesc &w, const TableDesc &tab, int P, const int32_t *slot_init, const double *norm_k)
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
        check_ids_kernel<<<(unsigned)(((int64_t)w.G * w.n + 255) / 256), 256, 0, s>>>(w, P, tab.bt, tab.refcount, norm_k);
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
                                                           int P, int r, Q8Desc q8)
{
    const int64_t b = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    if (b < n_blocks)
        quantise_block<T>(k + b * r, norm_k[b], q8.dir ? q8.dir + (b / P) * (int64_t)r : nullptr, q8.k + b * r, q8.err + b,
                          q8.scale + b, q8.alpha + b, r, threadIdx.x & 63);
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
        quantise_block<T>((const T *)pool.k + b * pool.r, pool.norm_k[b], w.q8.dir ? w.q8.dir + (int64_t)rec.x * pool.r : nullptr,
                          w.q8.k + b * pool.r, w.q8.err + b, w.q8.scale + b, w.q8.alpha + b, pool.r, threadIdx.x & 63);
    }
}

// The direction that the key blocks of a group are centred on: the normalised sum of up to 64 unit key blocks taken at
// even steps through the group's pool (fp64, one workgroup per group, every element of the sum owned by one thread).
// Any vector serves, the bound of the screen holds for all of them; this one follows the mean of the keys, which is
// the direction that unrelated blocks of real caches share.  A zero sum gives a zero direction (no centring).
template <typename T>
__global__ __launch_bounds__(256) void centre_direction_kernel(const T *__restrict__ k, int P, int r, float *__restrict__ dir)
{
    constexpr int PER = Elem<T>::PER16;
    extern __shared__ double acc[];          // [r]
    __shared__ double red[4];
    const int g = blockIdx.x, tid = threadIdx.x;
    const int chunks = r / PER;
    const T *kg = k + (int64_t)g * P * r;
    for (int e = tid; e < r; e += 256)
        acc[e] = 0.0;
    const int n_s = P < 64 ? P : 64;
    for (int s = 0; s < n_s; ++s) {
        const uint4 *x = reinterpret_cast<const uint4 *>(kg + ((int64_t)s * P / n_s) * r);
        double ss = 0.0;
        for (int c = tid; c < chunks; c += 256) {
            double v[PER];
            Elem<T>::widen(x[c], v);
#pragma unroll
            for (int i = 0; i < PER; ++i)
                ss = fma(v[i], v[i], ss);
        }
        __syncthreads();
        ss = block_sum_256(ss, red);
        const double inv = ss > 0.0 ? 1.0 / sqrt(ss) : 0.0;
        for (int c = tid; c < chunks; c += 256) {
            double v[PER];
            Elem<T>::widen(x[c], v);
#pragma unroll
            for (int i = 0; i < PER; ++i)
                acc[c * PER + i] = fma(v[i], inv, acc[c * PER + i]);
        }
    }
    double nn = 0.0;
    for (int c = tid; c < chunks; c += 256)
#pragma unroll
        for (int i = 0; i < PER; ++i)
            nn = fma(acc[c * PER + i], acc[c * PER + i], nn);
    __syncthreads();
    nn = block_sum_256(nn, red);
    const double invn = nn > 0.0 ? 1.0 / sqrt(nn) : 0.0;
    for (int c = tid; c < chunks; c += 256)
#pragma unroll
        for (int i = 0; i < PER; ++i)
            dir[(int64_t)g * r + c * PER + i] = (float)(acc[c * PER + i] * invn);
}

void launch_centre_direction(hipStream_t s, const PoolDesc &pool, const WorkDesc &w)
{
    if (!w.q8.k || !w.q8.dir || pool.G <= 0 || pool.P <= 0)
        return;
    const size_t lds = (size_t)pool.r * sizeof(double);
    if (pool.dtype == KVFUSE_BF16)
        centre_direction_kernel<bf16_t><<<pool.G, 256, lds, s>>>((const bf16_t *)pool.k, pool.P, pool.r, w.q8.dir);
    else
        centre_direction_kernel<float><<<pool.G, 256, lds, s>>>((const float *)pool.k, pool.P, pool.r, w.q8.dir);
}

void launch_quantise_all(hipStream_t s, const PoolDesc &pool, const WorkDesc &w)
{
    const int64_t nb = (int64_t)pool.G * pool.P;
    if (!w.q8.k || nb <= 0)
        return;
    const unsigned grid = (unsigned)((nb + 3) / 4);
    if (pool.dtype == KVFUSE_BF16)
        quantise_all_kernel<bf16_t><<<grid, 256, 0, s>>>((const bf16_t *)pool.k, pool.norm_k, nb, pool.P, pool.r, w.q8);
    else
        quantise_all_kernel<float><<<grid, 256, 0, s>>>((const float *)pool.k, pool.norm_k, nb, pool.P, pool.r, w.q8);
}

void launch_quantise_targets(hipStream_t s, const PoolDesc &pool, const WorkDesc &w, int height)
{
    if (!w.q8.k || (int64_t)w.G * w.l_stride <= 0)
        return;
    const unsigned grid = (unsigned)std::min<int64_t>(((int64_t)w.G * w.l_stride + 3) / 4, 256 * 8);
    if (pool.dtype == KVFUSE_BF16)
        quantise_targets_kernel<bf16_t><<<grid, 256, 0, s>>>(pool, w, height);
    else
        quantise_targets_kernel<float><<<grid, 256, 0, s>>>(pool, w, height);
}

}  // namespace kvfuse
