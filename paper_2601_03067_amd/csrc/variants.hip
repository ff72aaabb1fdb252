// Variants of the method beside the main path.
//
//   - Order of the requests (remark after Algorithm 1): requests with fewer blocks are better placed on the left of
//     the tree.  Host side only: a stable sort of the units (of the leaves, when there is one unit) by block count.
//   - The two ways the results section evaluates a fused cache.  The first copies the fused, rescaled cache back into
//     every fused block and frees nothing: every logical block gets its own block back, holding
//     scale * representative rounded to the pool type, so that an attention kernel that knows nothing of fusion
//     sees what the fused cache stands for.  The second fuses and frees blocks without rescaling: it keeps the
//     fused table and drops the per-block scales.
#include "common.h"

#include <algorithm>
#include <numeric>

namespace kvfuse {

template <typename T> struct Requant;
template <> struct Requant<bf16_t> {
    // 8 bfloat16 values times a binary32 scale: the product is exact in fp64, so this is one rounding
    __device__ static __forceinline__ uint4 run(const uint4 &raw, double s)
    {
        double x[8];
        Elem<bf16_t>::widen(raw, x);
        uint32_t o[4];
#pragma unroll
        for (int i = 0; i < 4; ++i)
            o[i] = f64_to_bf16_fast(x[2 * i] * s) | (f64_to_bf16_fast(x[2 * i + 1] * s) << 16);
        return make_uint4(o[0], o[1], o[2], o[3]);
    }
};
template <> struct Requant<float> {
    __device__ static __forceinline__ uint4 run(const uint4 &raw, double s)
    {
        double x[4];
        Elem<float>::widen(raw, x);
        return make_uint4(__float_as_uint((float)(x[0] * s)), __float_as_uint((float)(x[1] * s)),
                          __float_as_uint((float)(x[2] * s)), __float_as_uint((float)(x[3] * s)));
    }
};

// One workgroup per logical entry (g, x).  Phase 0 serves the entries whose own block was evicted: it is dead, no
// table entry points at it, so it can be written while the representatives are still being read.  Phase 1 then
// rescales, in place, the blocks that hold a representative themselves (every thread rewrites only the 16 bytes it
// has read).  Entries with an id outside [0, P) in either table are left alone.
template <typename T>
__global__ __launch_bounds__(256) void replicate_kernel(PoolDesc pool, TableDesc tab, const int32_t *__restrict__ orig_bt,
                                                        int phase)
{
    const int64_t e = blockIdx.x;
    const int g = (int)(e / tab.n);
    const int src = tab.bt[e], dst = orig_bt[e];
    if (src < 0 || src >= pool.P || dst < 0 || dst >= pool.P)
        return;
    const bool holder = src == dst;
    if (holder != (phase == 1))
        return;
    const float sk = tab.scale_k[e], sv = tab.scale_v[e];
    const int chunks = pool.r / Elem<T>::PER16;
    const int64_t so = ((int64_t)g * pool.P + src) * (int64_t)pool.r, dk = ((int64_t)g * pool.P + dst) * (int64_t)pool.r;
    if (!(holder && sk == 1.0f)) {
        const uint4 *s = reinterpret_cast<const uint4 *>((const T *)pool.k + so);
        uint4 *d = reinterpret_cast<uint4 *>((T *)pool.k + dk);
        for (int c = threadIdx.x; c < chunks; c += 256)
            d[c] = Requant<T>::run(s[c], (double)sk);
    }
    if (!(holder && sv == 1.0f)) {
        const uint4 *s = reinterpret_cast<const uint4 *>((const T *)pool.v + so);
        uint4 *d = reinterpret_cast<uint4 *>((T *)pool.v + dk);
        for (int c = threadIdx.x; c < chunks; c += 256)
            d[c] = Requant<T>::run(s[c], (double)sv);
    }
}

__global__ void restore_table_kernel(TableDesc tab, const int32_t *__restrict__ orig_bt, int64_t total)
{
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < total)
        tab.bt[i] = orig_bt[i];
}

__global__ void unit_scales_kernel(TableDesc tab, int64_t total)
{
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < total) {
        tab.scale_k[i] = 1.0f;
        tab.scale_v[i] = 1.0f;
    }
}

}  // namespace kvfuse

using namespace kvfuse;

extern "C" {

int kvfuse_tree_spec_shortest_first(const kvfuse_tree_spec *spec, int32_t *leaf_start, int32_t *leaf_count,
                                    int32_t *unit_leaf_ptr, int32_t *order)
{
    if (!spec || spec->n_leaves < 0 || spec->n_units < 0 || (spec->n_leaves > 0 && (!spec->leaf_start || !spec->leaf_count)) ||
        (spec->n_units > 0 && !spec->unit_leaf_ptr) || (spec->n_leaves > 0 && (!leaf_start || !leaf_count)) || !unit_leaf_ptr)
        return KVFUSE_EINVAL;
    if (spec->n_units == 0) {
        if (spec->n_leaves != 0)
            return KVFUSE_EINVAL;       // leaves without units
        unit_leaf_ptr[0] = 0;
        return KVFUSE_OK;
    }
    if (spec->unit_leaf_ptr[0] != 0 || spec->unit_leaf_ptr[spec->n_units] != spec->n_leaves)
        return KVFUSE_EINVAL;
    for (int u = 0; u < spec->n_units; ++u)
        if (spec->unit_leaf_ptr[u + 1] < spec->unit_leaf_ptr[u])
            return KVFUSE_EINVAL;
    if (spec->n_units == 1) {
        // one request: its chunks are what the tree is built over
        std::vector<int> idx((size_t)spec->n_leaves);
        std::iota(idx.begin(), idx.end(), 0);
        std::stable_sort(idx.begin(), idx.end(),
                         [&](int a, int b) { return spec->leaf_count[a] < spec->leaf_count[b]; });
        std::vector<int32_t> ls((size_t)spec->n_leaves), lc((size_t)spec->n_leaves);
        for (int k = 0; k < spec->n_leaves; ++k) {
            ls[(size_t)k] = spec->leaf_start[idx[(size_t)k]];
            lc[(size_t)k] = spec->leaf_count[idx[(size_t)k]];
        }
        for (int k = 0; k < spec->n_leaves; ++k) {
            leaf_start[k] = ls[(size_t)k];
            leaf_count[k] = lc[(size_t)k];
            if (order)
                order[k] = idx[(size_t)k];
        }
        unit_leaf_ptr[0] = 0;
        unit_leaf_ptr[1] = spec->n_leaves;
        return KVFUSE_OK;
    }
    std::vector<int64_t> blocks((size_t)spec->n_units, 0);
    for (int u = 0; u < spec->n_units; ++u)
        for (int l = spec->unit_leaf_ptr[u]; l < spec->unit_leaf_ptr[u + 1]; ++l)
            blocks[(size_t)u] += spec->leaf_count[l];
    std::vector<int> idx((size_t)spec->n_units);
    std::iota(idx.begin(), idx.end(), 0);
    std::stable_sort(idx.begin(), idx.end(), [&](int a, int b) { return blocks[(size_t)a] < blocks[(size_t)b]; });
    // the inputs may alias the outputs: gather into temporaries first
    std::vector<int32_t> ls, lc, up(1, 0);
    for (int k = 0; k < spec->n_units; ++k) {
        const int u = idx[(size_t)k];
        for (int l = spec->unit_leaf_ptr[u]; l < spec->unit_leaf_ptr[u + 1]; ++l) {
            ls.push_back(spec->leaf_start[l]);
            lc.push_back(spec->leaf_count[l]);
        }
        up.push_back((int32_t)ls.size());
    }
    for (size_t l = 0; l < ls.size(); ++l) {
        leaf_start[l] = ls[l];
        leaf_count[l] = lc[l];
    }
    for (int k = 0; k <= spec->n_units; ++k)
        unit_leaf_ptr[k] = up[(size_t)k];
    if (order)
        for (int k = 0; k < spec->n_units; ++k)
            order[k] = idx[(size_t)k];
    return KVFUSE_OK;
}

static int check_eval_args(kvfuse_ctx *ctx, const kvfuse_pool *pool, const kvfuse_table *table, const char *what)
{
    Ctx *c = &ctx->c;
    if (!pool || !pool->k || !pool->v || !pool->norm_k || !pool->norm_v || !pool->inv_norm_k || !table || !table->bt ||
        !table->scale_k || !table->scale_v || !table->orig_norm_k || !table->orig_norm_v || !table->refcount || !table->remap)
        return fail(c, KVFUSE_EINVAL, std::string(what) + ": null pointer");
    if (pool->G <= 0 || pool->P <= 0 || pool->t <= 0 || pool->d <= 0 || table->n < 0)
        return fail(c, KVFUSE_EINVAL, std::string(what) + ": non-positive size");
    if (pool->dtype != KVFUSE_BF16 && pool->dtype != KVFUSE_F32)
        return fail(c, KVFUSE_ESHAPE, std::string(what) + ": dtype must be KVFUSE_BF16 or KVFUSE_F32");
    const int64_t bytes = (int64_t)pool->t * pool->d * (pool->dtype == KVFUSE_BF16 ? 2 : 4);
    if (bytes % 128 != 0 || bytes > 32768)
        return fail(c, KVFUSE_ESHAPE, std::string(what) + ": t*d*sizeof(element) must be a multiple of 128 bytes and at most 32 KiB");
    if ((int64_t)pool->G * std::max(table->n, 1) >= (1ll << 31))
        return fail(c, KVFUSE_ESHAPE, std::string(what) + ": G * n must fit in 31 bits");
    return KVFUSE_OK;
}

int kvfuse_replicate_rescaled(kvfuse_ctx *ctx, const kvfuse_pool *pool, const kvfuse_table *table, const int32_t *orig_bt)
{
    if (!ctx)
        return KVFUSE_EINVAL;
    Ctx *c = &ctx->c;
    const int rc = check_eval_args(ctx, pool, table, "replicate");
    if (rc)
        return rc;
    if (!orig_bt)
        return fail(c, KVFUSE_EINVAL, "replicate: null original table");
    const PoolDesc pd = to_desc(*pool);
    const TableDesc td = to_desc(*table);
    const int64_t total = (int64_t)pool->G * table->n;
    if (total > 0) {
        for (int phase = 0; phase < 2; ++phase) {
            if (pool->dtype == KVFUSE_BF16)
                replicate_kernel<bf16_t><<<(unsigned)total, 256, 0, c->stream>>>(pd, td, orig_bt, phase);
            else
                replicate_kernel<float><<<(unsigned)total, 256, 0, c->stream>>>(pd, td, orig_bt, phase);
        }
        restore_table_kernel<<<(unsigned)((total + 255) / 256), 256, 0, c->stream>>>(td, orig_bt, total);
    }
    // norms of the rewritten blocks, unit scales, one reference per block, nothing evicted
    launch_block_norms(c->stream, pd, td);
    KVF_HIP(c, hipGetLastError());
    return KVFUSE_OK;
}

int kvfuse_drop_rescale(kvfuse_ctx *ctx, const kvfuse_pool *pool, const kvfuse_table *table)
{
    if (!ctx)
        return KVFUSE_EINVAL;
    Ctx *c = &ctx->c;
    const int rc = check_eval_args(ctx, pool, table, "drop rescale");
    if (rc)
        return rc;
    const int64_t total = (int64_t)pool->G * table->n;
    if (total > 0)
        unit_scales_kernel<<<(unsigned)((total + 255) / 256), 256, 0, c->stream>>>(to_desc(*table), total);
    KVF_HIP(c, hipGetLastError());
    return KVFUSE_OK;
}

}  // extern "C"
