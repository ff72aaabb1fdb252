// Host side of the kvfuse C ABI: contexts, Algorithm 1's recursion tree cut into heights (a6), workspace layout,
// argument checks and the stage sequencing of the whole pipeline.  No device memory is allocated here.
#include <algorithm>
#include <climits>
#include <cmath>
#include <cstdint>
#include <cstring>
#include <new>
#include <utility>

#include "common.h"

namespace kvfuse {

int fail(Ctx *c, int code, const std::string &msg)
{
    if (c)
        c->err = msg;
    return code;
}

// ---- Algorithm 1's recursion as a tree --------------------------------------------------------------------

struct Node {
    int left = -1, right = -1;   // children (node indices) or -1 for a leaf
    int off = 0;                 // start of the node's region in a set_ids row
    int src = 0;                 // leaves: first logical entry of the leaf
    int cap = 0;                 // size of the surviving set if nothing fuses
    int height = 0;
};

struct HostHeight {
    std::vector<int32_t> l_off, r_off, l_slot, r_slot, out_slot, l_cap, r_cap, l_base, r_base;
    int item_cap = 0;                                          // most similarity work items of one group
    bool big = false;
    std::vector<int64_t> s_base;
    HeightDesc dev;
};

struct Plan {
    Ctx *ctx = nullptr;
    PoolDesc pool;
    TableDesc tab;
    WorkDesc work;
    std::vector<Node> nodes;
    std::vector<HostHeight> heights;
    int32_t *slot_init = nullptr;   // device [n_slots]
    int max_r = 0, max_l = 0;
    std::vector<uint8_t> group_enable_host;   // copy of the group mask for the statistics; empty = all groups
    int assign_rule = KVFUSE_RULE_ARGMAX;
    float *q8_dir_mem = nullptr;    // fp8 screen with centring asked for: the caller's [G][r] floats for the directions

    // The copies are centred only where that pays and fits: not together with the prefix screen (a block's share of the
    // common direction differs between prefix and tail) and not for blocks whose direction kernel would need more than
    // 64 KiB of LDS.
    void refresh_q8_dir() { work.q8.dir = (work.q8.k && q8_dir_mem && work.screen_prefix == 0 && pool.r <= 8192) ? q8_dir_mem : nullptr; }
};

// Similarity tile shapes (must match the two kernel instantiations): big 256 x 256, small 128 x 128.
constexpr int kBigM = 256, kBigN = 256, kSmallM = 128, kSmallN = 128;
constexpr int kMaxHeights = 64;

struct TreeBuilder {
    const kvfuse_tree_spec *spec;
    std::vector<Node> nodes;
    int next_off = 0;   // set regions are handed out in the order the recursion meets the leaves, whatever their
                        // logical positions: the region of an inner node is then its children's, left then right

    int leaf(int l)
    {
        Node n;
        n.off = next_off;
        n.src = spec->leaf_start[l];
        n.cap = spec->leaf_count[l];
        next_off += n.cap;
        nodes.push_back(n);
        return (int)nodes.size() - 1;
    }
    int join(int a, int b)
    {
        Node n;
        n.left = a;
        n.right = b;
        n.off = nodes[a].off;
        n.cap = nodes[a].cap + nodes[b].cap;
        n.height = 1 + std::max(nodes[a].height, nodes[b].height);
        nodes.push_back(n);
        return (int)nodes.size() - 1;
    }
    // FastFusion over leaves [lo, hi): split at len / 2, left half first
    int over_leaves(int lo, int hi)
    {
        if (hi - lo == 1)
            return leaf(lo);
        const int mid = lo + (hi - lo) / 2;
        const int a = over_leaves(lo, mid);
        const int b = over_leaves(mid, hi);
        return join(a, b);
    }
    int empty_leaf()
    {
        Node n;
        n.off = next_off;
        n.cap = 0;
        nodes.push_back(n);
        return (int)nodes.size() - 1;
    }
    // FastFusion over units [lo, hi); a unit with several leaves is fused over its own leaves first
    int over_units(int lo, int hi)
    {
        if (hi - lo == 1) {
            const int a = spec->unit_leaf_ptr[lo], b = spec->unit_leaf_ptr[lo + 1];
            if (a == b)
                return empty_leaf();
            return over_leaves(a, b);
        }
        const int mid = lo + (hi - lo) / 2;
        const int a = over_units(lo, mid);
        const int b = over_units(mid, hi);
        return join(a, b);
    }
};

static int check_spec(Ctx *ctx, int n, const kvfuse_tree_spec *s)
{
    if (!s || s->n_leaves < 0 || s->n_units < 0 || (s->n_leaves > 0 && (!s->leaf_start || !s->leaf_count)) ||
        (s->n_units > 0 && !s->unit_leaf_ptr))
        return fail(ctx, KVFUSE_EINVAL, "tree spec: null or negative field");
    std::vector<std::pair<int64_t, int64_t>> runs;   // (start, end) of the non-empty leaves
    for (int l = 0; l < s->n_leaves; ++l) {
        if (s->leaf_count[l] < 0 || s->leaf_start[l] < 0 || (int64_t)s->leaf_start[l] + s->leaf_count[l] > n)
            return fail(ctx, KVFUSE_EINVAL, "tree spec: leaves must lie inside the table");
        if (s->leaf_count[l] > 0)
            runs.emplace_back(s->leaf_start[l], (int64_t)s->leaf_start[l] + s->leaf_count[l]);
    }
    std::sort(runs.begin(), runs.end());
    for (size_t k = 1; k < runs.size(); ++k)
        if (runs[k].first < runs[k - 1].second)
            return fail(ctx, KVFUSE_EINVAL, "tree spec: leaves must not overlap");
    if (s->n_units > 0) {
        if (s->unit_leaf_ptr[0] != 0 || s->unit_leaf_ptr[s->n_units] != s->n_leaves)
            return fail(ctx, KVFUSE_EINVAL, "tree spec: unit_leaf_ptr must run from 0 to n_leaves");
        for (int u = 0; u < s->n_units; ++u)
            if (s->unit_leaf_ptr[u + 1] < s->unit_leaf_ptr[u])
                return fail(ctx, KVFUSE_EINVAL, "tree spec: unit_leaf_ptr must be non-decreasing");
    } else if (s->n_leaves > 0) {
        return fail(ctx, KVFUSE_EINVAL, "tree spec: leaves without units");
    }
    return KVFUSE_OK;
}

static void build_tree(const kvfuse_tree_spec *s, std::vector<Node> &nodes)
{
    TreeBuilder tb{s, {}};
    if (s->n_units == 1) {
        const int lo = s->unit_leaf_ptr[0], hi = s->unit_leaf_ptr[1];
        const int step = s->group_size > 0 ? s->group_size : std::max(hi - lo, 1);
        for (int a = lo; a < hi; a += step)
            tb.over_leaves(a, std::min(a + step, hi));
    } else if (s->n_units > 1) {
        const int step = s->group_size > 0 ? s->group_size : s->n_units;
        for (int a = 0; a < s->n_units; a += step)
            tb.over_units(a, std::min(a + step, s->n_units));
    }
    nodes.swap(tb.nodes);
}

static void build_heights(const std::vector<Node> &nodes, std::vector<HostHeight> &hs)
{
    int max_h = 0;
    for (const Node &n : nodes)
        max_h = std::max(max_h, n.height);
    hs.assign(max_h, HostHeight());
    for (int k = 0; k < (int)nodes.size(); ++k) {
        const Node &n = nodes[k];
        if (n.left < 0)
            continue;
        HostHeight &h = hs[n.height - 1];
        h.l_off.push_back(nodes[n.left].off);
        h.r_off.push_back(nodes[n.right].off);
        h.l_slot.push_back(n.left);
        h.r_slot.push_back(n.right);
        h.out_slot.push_back(k);
        h.l_cap.push_back(nodes[n.left].cap);
        h.r_cap.push_back(nodes[n.right].cap);
    }
    for (HostHeight &h : hs) {
        const int nn = (int)h.l_off.size();
        h.l_base.assign(nn + 1, 0);
        h.r_base.assign(nn + 1, 0);
        h.s_base.assign(nn + 1, 0);
        for (int k = 0; k < nn; ++k) {
            h.l_base[k + 1] = h.l_base[k] + h.l_cap[k];
            h.r_base[k + 1] = h.r_base[k] + h.r_cap[k];
            h.s_base[k + 1] = h.s_base[k] + (int64_t)h.l_cap[k] * h.r_cap[k];
        }
        // Tile shape: big tiles when the typical node (weighted by its work) is at least one big tile in both
        // directions; small tiles waste less padding on the low heights.
        double wsum = 0.0, wmin = 0.0;
        for (int k = 0; k < nn; ++k) {
            const double wk = (double)h.l_cap[k] * h.r_cap[k];
            wsum += wk;
            wmin += wk * std::min(h.l_cap[k], h.r_cap[k]);
        }
        h.big = wsum > 0.0 && wmin / wsum >= 256.0;
        const int bm = h.big ? kBigM : kSmallM, bn = h.big ? kBigN : kSmallN;
        // Room for the similarity work items of one group.  The items themselves are laid out on the device from the
        // sets' current sizes (similarity.hip); a node whose left set spans a row tiles and whose right set c panels has
        // c * ceil(a / min(ceil(a / 4), 4)) of them, which for a up to A is at most c * (A < 4 ? A : max(4, ceil(A / 4))).
        int64_t cap = 0;
        for (int k = 0; k < nn; ++k) {
            const int n_cp = (h.r_cap[k] + bn - 1) / bn;
            const int n_rtile = (h.l_cap[k] + bm - 1) / bm;
            cap += (int64_t)n_cp * (n_rtile < 4 ? n_rtile : std::max(4, (n_rtile + 3) / 4));
        }
        h.item_cap = (int)std::min<int64_t>(cap, INT32_MAX);
    }
}

static size_t align256(size_t x) { return (x + 255) & ~(size_t)255; }

// Walks the workspace layout; with base == nullptr it only measures.
struct Carver {
    char *base;
    size_t off = 0;
    template <typename T> T *take(size_t count)
    {
        T *p = base ? reinterpret_cast<T *>(base + off) : nullptr;
        off = align256(off + count * sizeof(T));
        return p;
    }
};

static void carve(Carver &cv, int G, int n, int n_slots, int max_r, int max_l, int cand_cap,
                  std::vector<HostHeight> &hs, WorkDesc &w, int32_t *&slot_init)
{
    w.G = G; w.n = n; w.n_slots = n_slots; w.r_stride = std::max(max_r, 1); w.l_stride = std::max(max_l, 1);
    w.cand_cap = cand_cap;
    const size_t R = (size_t)G * w.r_stride, L = (size_t)G * w.l_stride;
    w.set_ids = cv.take<int32_t>((size_t)G * n);
    w.set_cnt = cv.take<int32_t>((size_t)G * n_slots);
    w.assign = cv.take<int32_t>(R);
    w.best_packed = cv.take<unsigned long long>(R);
    w.cand_cnt = cv.take<int32_t>(R);
    w.cand_idx = cv.take<int32_t>(R * cand_cap);
    w.cand_val = cv.take<float>(R * cand_cap);
    w.seg_cnt = cv.take<int32_t>(L);
    w.seg_ptr = cv.take<int32_t>(L);
    w.seg_members = cv.take<int32_t>(R);
    w.active = cv.take<int4>(2 * L);
    w.seg_slot = cv.take<int32_t>(L);
    w.n_active = cv.take<int32_t>(kMaxHeights);
    w.refine = cv.take<int32_t>(2 * R);
    w.n_refine = cv.take<int32_t>(kMaxHeights);
    w.counters = cv.take<int32_t>((size_t)G * 8);
    w.group_enable = nullptr;
    w.leaf_src = cv.take<int32_t>((size_t)std::max(n, 1));
    w.rem_k = nullptr;
    w.screen_prefix = 0;
    w.q8 = Q8Desc{};
    slot_init = cv.take<int32_t>(n_slots);
    {
        size_t items = 1, nodes = 1;
        for (const HostHeight &h : hs) {
            items = std::max(items, (size_t)h.item_cap);
            nodes = std::max(nodes, h.l_off.size());
        }
        w.dyn_stride = (int32_t)(nodes + 1);
        w.dyn_items = cv.take<int4>((size_t)G * items);
        w.dyn_base = cv.take<int32_t>((size_t)G * w.dyn_stride);
        w.dyn_count = cv.take<int32_t>((size_t)G);
    }
    for (HostHeight &h : hs) {
        const size_t nn = h.l_off.size();
        HeightDesc &d = h.dev;
        d.n_nodes = (int)nn;
        d.total_l_cap = h.l_base[nn];
        d.total_r_cap = h.r_base[nn];
        d.total_s = h.s_base[nn];
        d.use_big_tiles = h.big;
        d.item_cap = h.item_cap;
        d.l_off = cv.take<int32_t>(nn);
        d.r_off = cv.take<int32_t>(nn);
        d.l_slot = cv.take<int32_t>(nn);
        d.r_slot = cv.take<int32_t>(nn);
        d.out_slot = cv.take<int32_t>(nn);
        d.l_cap = cv.take<int32_t>(nn);
        d.r_cap = cv.take<int32_t>(nn);
        d.l_base = cv.take<int32_t>(nn + 1);
        d.r_base = cv.take<int32_t>(nn + 1);
        d.s_base = cv.take<int64_t>(nn + 1);
    }
}

static void plan_extents(const std::vector<HostHeight> &hs, int &max_r, int &max_l)
{
    max_r = max_l = 0;
    for (const HostHeight &h : hs) {
        max_r = std::max(max_r, (int)h.r_base.back());
        max_l = std::max(max_l, (int)h.l_base.back());
    }
}

static int check_pool(Ctx *ctx, const kvfuse_pool *p)
{
    if (!p || !p->k || !p->v || !p->norm_k || !p->norm_v || !p->inv_norm_k)
        return fail(ctx, KVFUSE_EINVAL, "pool: null pointer");
    if (p->G <= 0 || p->P <= 0 || p->t <= 0 || p->d <= 0)
        return fail(ctx, KVFUSE_EINVAL, "pool: non-positive size");
    if (p->dtype != KVFUSE_BF16 && p->dtype != KVFUSE_F32)
        return fail(ctx, KVFUSE_ESHAPE, "pool: dtype must be KVFUSE_BF16 or KVFUSE_F32");
    const int64_t r = (int64_t)p->t * p->d;
    const int64_t bytes = r * (p->dtype == KVFUSE_BF16 ? 2 : 4);
    if (bytes % 128 != 0 || bytes > 32768)
        return fail(ctx, KVFUSE_ESHAPE, "pool: t*d*sizeof(element) must be a multiple of 128 bytes and at most 32 KiB");
    return KVFUSE_OK;
}

static int check_table(Ctx *ctx, const kvfuse_table *t)
{
    if (!t || t->n < 0 || !t->bt || !t->scale_k || !t->scale_v || !t->orig_norm_k || !t->orig_norm_v || !t->refcount ||
        !t->remap)
        return fail(ctx, KVFUSE_EINVAL, "table: null pointer or negative n");
    return KVFUSE_OK;
}

template <typename T> static hipError_t upload(hipStream_t s, const T *dst, const std::vector<T> &src)
{
    if (src.empty())
        return hipSuccess;
    return hipMemcpyAsync(const_cast<T *>(dst), src.data(), src.size() * sizeof(T), hipMemcpyHostToDevice, s);
}

}  // namespace kvfuse

using namespace kvfuse;

struct kvfuse_plan {
    Plan p;
};

extern "C" {

int kvfuse_create(kvfuse_ctx **out, int device, void *hip_stream)
{
    if (!out)
        return KVFUSE_EINVAL;
    *out = nullptr;
    int count = 0;
    if (hipGetDeviceCount(&count) != hipSuccess || device < 0 || device >= count)
        return KVFUSE_EHIP;
    kvfuse_ctx *x = new (std::nothrow) kvfuse_ctx();
    if (!x)
        return KVFUSE_ENOMEM;
    x->c.device = device;
    x->c.stream = (hipStream_t)hip_stream;
    *out = x;
    return KVFUSE_OK;
}

int kvfuse_destroy(kvfuse_ctx *ctx)
{
    if (!ctx)
        return KVFUSE_OK;
    if (ctx->c.ev_ready)
        for (hipEvent_t &e : ctx->c.ev)
            (void)hipEventDestroy(e);
    if (ctx->c.aux) {
        (void)hipStreamSynchronize(ctx->c.aux);
        (void)hipEventDestroy(ctx->c.fork);
        (void)hipEventDestroy(ctx->c.join);
        (void)hipStreamDestroy(ctx->c.aux);
    }
    delete ctx;
    return KVFUSE_OK;
}

const char *kvfuse_last_error(const kvfuse_ctx *ctx) { return ctx ? ctx->c.err.c_str() : "null context"; }

int kvfuse_workspace_bytes(int32_t G, int32_t n, const kvfuse_tree_spec *spec, int32_t cand_cap, size_t *bytes)
{
    if (!bytes || G <= 0 || n < 0 || cand_cap < 1 || cand_cap > 64)
        return KVFUSE_EINVAL;
    const int rc = check_spec(nullptr, n, spec);
    if (rc)
        return rc;
    std::vector<Node> nodes;
    build_tree(spec, nodes);
    std::vector<HostHeight> hs;
    build_heights(nodes, hs);
    if ((int)hs.size() > kMaxHeights)
        return KVFUSE_ESHAPE;
    int max_r, max_l;
    plan_extents(hs, max_r, max_l);
    Carver cv{nullptr};
    WorkDesc w;
    int32_t *si;
    carve(cv, G, n, std::max((int)nodes.size(), 1), max_r, max_l, cand_cap, hs, w, si);
    *bytes = cv.off + 256;
    return KVFUSE_OK;
}

int kvfuse_plan_create(kvfuse_ctx *ctx, const kvfuse_pool *pool, const kvfuse_table *table, const kvfuse_tree_spec *spec,
                       int32_t cand_cap, void *workspace, size_t workspace_bytes, kvfuse_plan **out)
{
    if (!ctx || !out)
        return KVFUSE_EINVAL;
    *out = nullptr;
    Ctx *c = &ctx->c;
    int rc;
    if ((rc = check_pool(c, pool)) || (rc = check_table(c, table)) || (rc = check_spec(c, table->n, spec)))
        return rc;
    if (cand_cap < 1 || cand_cap > 64)
        return fail(c, KVFUSE_EINVAL, "cand_cap must be in [1, 64]");
    if (!workspace || ((uintptr_t)workspace & 255))
        return fail(c, KVFUSE_EINVAL, "workspace must be non-null and 256-byte aligned");
    if ((int64_t)pool->G * std::max(table->n, 1) >= (1ll << 31))
        return fail(c, KVFUSE_ESHAPE, "G * n must fit in 31 bits");
    kvfuse_plan *pl = new (std::nothrow) kvfuse_plan();
    if (!pl)
        return fail(c, KVFUSE_ENOMEM, "host allocation failed");
    Plan &p = pl->p;
    p.ctx = c;
    p.pool = to_desc(*pool);
    p.tab = to_desc(*table);
    build_tree(spec, p.nodes);
    build_heights(p.nodes, p.heights);
    if ((int)p.heights.size() > kMaxHeights) {
        delete pl;
        return fail(c, KVFUSE_ESHAPE, "tree deeper than 64 heights");
    }
    plan_extents(p.heights, p.max_r, p.max_l);
    const int n_slots = std::max((int)p.nodes.size(), 1);
    Carver cv{(char *)workspace};
    carve(cv, pool->G, table->n, n_slots, p.max_r, p.max_l, cand_cap, p.heights, p.work, p.slot_init);
    if (cv.off > workspace_bytes) {
        delete pl;
        return fail(c, KVFUSE_ENOMEM, "workspace too small: need " + std::to_string(cv.off) + " bytes");
    }
    // upload the static tables
    std::vector<int32_t> init(n_slots, 0);
    for (size_t k = 0; k < p.nodes.size(); ++k)
        init[k] = p.nodes[k].left < 0 ? p.nodes[k].cap : 0;
    hipError_t e = upload(c->stream, p.slot_init, init);
    // position in a set_ids row -> logical entry it is filled from (-1: not part of any leaf)
    std::vector<int32_t> leaf_src((size_t)std::max(table->n, 1), -1);
    for (const Node &nd : p.nodes)
        if (nd.left < 0)
            for (int i = 0; i < nd.cap; ++i)
                leaf_src[(size_t)nd.off + i] = nd.src + i;
    if (e == hipSuccess) e = upload(c->stream, p.work.leaf_src, leaf_src);
    for (HostHeight &h : p.heights) {
        const HeightDesc &d = h.dev;
        if (e == hipSuccess) e = upload(c->stream, d.l_off, h.l_off);
        if (e == hipSuccess) e = upload(c->stream, d.r_off, h.r_off);
        if (e == hipSuccess) e = upload(c->stream, d.l_slot, h.l_slot);
        if (e == hipSuccess) e = upload(c->stream, d.r_slot, h.r_slot);
        if (e == hipSuccess) e = upload(c->stream, d.out_slot, h.out_slot);
        if (e == hipSuccess) e = upload(c->stream, d.l_cap, h.l_cap);
        if (e == hipSuccess) e = upload(c->stream, d.r_cap, h.r_cap);
        if (e == hipSuccess) e = upload(c->stream, d.l_base, h.l_base);
        if (e == hipSuccess) e = upload(c->stream, d.r_base, h.r_base);
        if (e == hipSuccess) e = upload(c->stream, d.s_base, h.s_base);
    }
    if (e == hipSuccess)
        e = hipStreamSynchronize(c->stream);   // the host vectors may now be reused or freed
    if (e != hipSuccess) {
        delete pl;
        return fail(c, KVFUSE_EHIP, std::string("plan upload: ") + hipGetErrorString(e));
    }
    *out = pl;
    return KVFUSE_OK;
}

int kvfuse_plan_destroy(kvfuse_plan *plan)
{
    delete plan;
    return KVFUSE_OK;
}

int kvfuse_plan_heights(const kvfuse_plan *plan, int32_t *n_heights)
{
    if (!plan || !n_heights)
        return KVFUSE_EINVAL;
    *n_heights = (int32_t)plan->p.heights.size();
    return KVFUSE_OK;
}

int kvfuse_plan_view(const kvfuse_plan *plan, int32_t height, kvfuse_height_view *v)
{
    if (!plan || !v || height < 0 || height >= (int)plan->p.heights.size())
        return KVFUSE_EINVAL;
    const HeightDesc &d = plan->p.heights[height].dev;
    const WorkDesc &w = plan->p.work;
    v->n_nodes = d.n_nodes; v->total_l_cap = d.total_l_cap; v->total_r_cap = d.total_r_cap; v->cand_cap = w.cand_cap;
    v->total_s = d.total_s;
    v->l_off = d.l_off; v->r_off = d.r_off; v->l_slot = d.l_slot; v->r_slot = d.r_slot; v->out_slot = d.out_slot;
    v->l_cap = d.l_cap; v->r_cap = d.r_cap; v->l_base = d.l_base; v->r_base = d.r_base; v->s_base = d.s_base;
    v->set_ids = w.set_ids; v->set_cnt = w.set_cnt; v->assign = w.assign; v->best_packed = w.best_packed;
    v->cand_cnt = w.cand_cnt;
    v->n_slots = w.n_slots; v->r_stride = w.r_stride; v->l_stride = w.l_stride; v->reserved = 0;
    return KVFUSE_OK;
}

int kvfuse_block_norms(kvfuse_ctx *ctx, const kvfuse_pool *pool, const kvfuse_table *table)
{
    if (!ctx)
        return KVFUSE_EINVAL;
    int rc;
    if ((rc = check_pool(&ctx->c, pool)) || (rc = check_table(&ctx->c, table)))
        return rc;
    launch_block_norms(ctx->c.stream, to_desc(*pool), to_desc(*table));
    KVF_HIP(&ctx->c, hipGetLastError());
    return KVFUSE_OK;
}

int kvfuse_leaf_sets(kvfuse_ctx *ctx, kvfuse_plan *plan)
{
    if (!ctx || !plan)
        return KVFUSE_EINVAL;
    launch_leaf_sets(ctx->c.stream, plan->p.work, plan->p.tab, plan->p.pool.P, plan->p.slot_init, plan->p.pool.norm_k);
    launch_prefix_tails(ctx->c.stream, plan->p.pool, plan->p.work);          // no-op unless the prefix screen is on
    launch_centre_direction(ctx->c.stream, plan->p.pool, plan->p.work);      // no-ops unless the fp8 screen is on
    launch_quantise_all(ctx->c.stream, plan->p.pool, plan->p.work);
    KVF_HIP(&ctx->c, hipGetLastError());
    return KVFUSE_OK;
}

static int check_step(kvfuse_ctx *ctx, kvfuse_plan *plan, int height, double thr, double band, bool need_band)
{
    if (!ctx || !plan)
        return KVFUSE_EINVAL;
    if (height < 0 || height >= (int)plan->p.heights.size())
        return fail(&ctx->c, KVFUSE_EINVAL, "height out of range");
    if (need_band) {
        if (!(band >= std::ldexp((double)plan->p.pool.r, -22)) || !std::isfinite(thr))
            return fail(&ctx->c, KVFUSE_EINVAL, "band must be >= r * 2^-22 and thr finite");
    }
    return KVFUSE_OK;
}

int kvfuse_similarity(kvfuse_ctx *ctx, kvfuse_plan *plan, int32_t height, double thr, double band, float *dense_s)
{
    const int rc = check_step(ctx, plan, height, thr, band, true);
    if (rc)
        return rc;
    // candidate floor thr - 2*band, nudged down so that float rounding can only admit more candidates
    const float floor_f = std::nextafterf((float)(thr - 2.0 * band), -INFINITY);
    launch_similarity(ctx->c.stream, plan->p.pool, plan->p.work, plan->p.heights[height].dev, floor_f, dense_s);
    KVF_HIP(&ctx->c, hipGetLastError());
    return KVFUSE_OK;
}

int kvfuse_assign(kvfuse_ctx *ctx, kvfuse_plan *plan, int32_t height, double thr, double band)
{
    const int rc = check_step(ctx, plan, height, thr, band, true);
    if (rc)
        return rc;
    launch_assign(ctx->c.stream, plan->p.pool, plan->p.tab, plan->p.work, plan->p.heights[height].dev, height, thr, band,
                  plan->p.assign_rule);
    KVF_HIP(&ctx->c, hipGetLastError());
    return KVFUSE_OK;
}

int kvfuse_merge(kvfuse_ctx *ctx, kvfuse_plan *plan, int32_t height)
{
    const int rc = check_step(ctx, plan, height, 0.0, 0.0, false);
    if (rc)
        return rc;
    launch_merge(ctx->c.stream, plan->p.pool, plan->p.work, plan->p.heights[height].dev, height);
    KVF_HIP(&ctx->c, hipGetLastError());
    return KVFUSE_OK;
}

int kvfuse_rewrite_block_table(kvfuse_ctx *ctx, const kvfuse_pool *pool, const kvfuse_table *table, int32_t *free_list,
                               int32_t *n_free, int32_t *n_phys)
{
    if (!ctx)
        return KVFUSE_EINVAL;
    int rc;
    if ((rc = check_pool(&ctx->c, pool)) || (rc = check_table(&ctx->c, table)))
        return rc;
    launch_rewrite(ctx->c.stream, to_desc(*pool), to_desc(*table), free_list, n_free, n_phys);
    KVF_HIP(&ctx->c, hipGetLastError());
    return KVFUSE_OK;
}

int kvfuse_fuse_tree(kvfuse_ctx *ctx, kvfuse_plan *plan, double thr, double band, int32_t *free_list, int32_t *n_free,
                     int32_t *n_phys, kvfuse_stats *stats, int32_t want_timing)
{
    if (!ctx || !plan)
        return KVFUSE_EINVAL;
    Ctx *c = &ctx->c;
    Plan &p = plan->p;
    if (!(band >= std::ldexp((double)p.pool.r, -22)) || !std::isfinite(thr))
        return fail(c, KVFUSE_EINVAL, "band must be >= r * 2^-22 and thr finite");
    const bool timing = stats && want_timing;
    const int nh = (int)p.heights.size();
    // events: 0 start, 1 after norms + leaf sets, then per stage accumulation through pairs
    std::vector<hipEvent_t> evs;
    auto mark = [&]() -> hipError_t {
        if (!timing)
            return hipSuccess;
        hipEvent_t e;
        hipError_t rc = hipEventCreate(&e);
        if (rc != hipSuccess)
            return rc;
        evs.push_back(e);
        return hipEventRecord(e, c->stream);
    };
    auto cleanup = [&]() {
        for (hipEvent_t e : evs)
            (void)hipEventDestroy(e);
    };
#define KVF_TRY(expr)                                                                            \
    do {                                                                                         \
        hipError_t e__ = (expr);                                                                 \
        if (e__ != hipSuccess) {                                                                 \
            cleanup();                                                                           \
            return fail(c, KVFUSE_EHIP, std::string(#expr) + ": " + hipGetErrorString(e__));     \
        }                                                                                        \
    } while (0)

    const float floor_f = std::nextafterf((float)(thr - 2.0 * band), -INFINITY);
    KVF_TRY(mark());
    launch_centre_direction(c->stream, p.pool, p.work);                      // no-op unless the fp8 copies are centred
    launch_block_norms(c->stream, p.pool, p.tab, p.work.screen_prefix > 0 ? p.work.rem_k : nullptr, p.work.screen_prefix,
                       p.work.q8.k ? &p.work.q8 : nullptr);
    launch_leaf_sets(c->stream, p.work, p.tab, p.pool.P, p.slot_init, p.pool.norm_k);
    KVF_TRY(mark());
    for (int hgt = 0; hgt < nh; ++hgt) {
        const HeightDesc &d = p.heights[hgt].dev;
        launch_similarity(c->stream, p.pool, p.work, d, floor_f, nullptr);
        KVF_TRY(mark());
        launch_assign(c->stream, p.pool, p.tab, p.work, d, hgt, thr, band, p.assign_rule);
        KVF_TRY(mark());
        launch_merge(c->stream, p.pool, p.work, d, hgt);
        KVF_TRY(mark());
    }
    launch_rewrite(c->stream, p.pool, p.tab, free_list, n_free, n_phys);
    KVF_TRY(mark());
    KVF_TRY(hipGetLastError());
    if (!stats)
        return KVFUSE_OK;

    KVF_TRY(hipStreamSynchronize(c->stream));
    std::memset(stats, 0, sizeof(*stats));
    stats->n_heights = nh;
    if (timing) {
        auto ms = [&](int a, int b) {
            float t = 0.f;
            (void)hipEventElapsedTime(&t, evs[a], evs[b]);
            return t;
        };
        stats->ms_norms = ms(0, 1);
        for (int hgt = 0; hgt < nh; ++hgt) {
            stats->ms_similarity += ms(1 + 3 * hgt, 2 + 3 * hgt);
            stats->ms_assign += ms(2 + 3 * hgt, 3 + 3 * hgt);
            stats->ms_merge += ms(3 + 3 * hgt, 4 + 3 * hgt);
        }
        stats->ms_rewrite = ms(1 + 3 * nh, 2 + 3 * nh);
        stats->ms_total = ms(0, 2 + 3 * nh);
    }
    cleanup();
    evs.clear();
    // counters and set sizes (small) come back to the host; the similarity flop count uses the actual set sizes
    const WorkDesc &w = p.work;
    std::vector<int32_t> counters((size_t)w.G * 8), cnt((size_t)w.G * w.n_slots);
    KVF_TRY(hipMemcpy(counters.data(), w.counters, counters.size() * 4, hipMemcpyDeviceToHost));
    KVF_TRY(hipMemcpy(cnt.data(), w.set_cnt, cnt.size() * 4, hipMemcpyDeviceToHost));
    if (nh > 0) {
        std::vector<int32_t> n_act((size_t)nh);
        KVF_TRY(hipMemcpy(n_act.data(), w.n_active, (size_t)nh * 4, hipMemcpyDeviceToHost));
        int64_t targets = 0;
        for (int32_t x : n_act)
            targets += x;
        stats->merge_targets = (int32_t)std::min<int64_t>(targets, INT32_MAX);
    }
    int64_t invalid = 0, shared = 0, out_of_range = 0;
    for (int g = 0; g < w.G; ++g) {
        const bool on = p.group_enable_host.empty() || p.group_enable_host[(size_t)g] != 0;
        stats->fused += counters[(size_t)g * 8 + 0];
        stats->near_threshold += counters[(size_t)g * 8 + 1];
        stats->refined += counters[(size_t)g * 8 + 2];
        stats->cand_overflow += counters[(size_t)g * 8 + 3];
        invalid += counters[(size_t)g * 8 + 4];
        shared += counters[(size_t)g * 8 + 5];
        out_of_range += counters[(size_t)g * 8 + 6];
        for (const Node &nd : p.nodes)
            if (nd.left >= 0 && on)
                stats->sim_flops += 2.0 * (double)cnt[(size_t)g * w.n_slots + nd.left] *
                                    (double)cnt[(size_t)g * w.n_slots + nd.right] * (double)p.pool.r;
    }
    stats->logical_blocks = (int64_t)w.G * w.n;
    stats->physical_blocks = stats->logical_blocks - stats->fused;
    stats->compression_ratio = stats->physical_blocks > 0 ? (double)stats->logical_blocks / (double)stats->physical_blocks : 0.0;
    if (invalid)
        return fail(c, KVFUSE_EINVAL, "block table holds " + std::to_string(invalid) + " ids outside [0, P)");
    if (shared)
        return fail(c, KVFUSE_EINVAL, "block table is not injective on entry: " + std::to_string(shared) +
                                          " entries point at a block that another entry of their group holds as well "
                                          "(a table that was fused before, or a prefix cache); the result is undefined");
    if (out_of_range)
        return fail(c, KVFUSE_EINVAL, std::to_string(out_of_range) + " key blocks have a norm that is not finite or lies outside "
                                          "[2^-40, 2^40]: products of such blocks leave binary32's range in the similarity screen "
                                          "and pairs could be missed; rescale the cache");
    return KVFUSE_OK;
#undef KVF_TRY
}

int kvfuse_plan_group_counters(kvfuse_ctx *ctx, const kvfuse_plan *plan, int32_t *out, int32_t n_groups)
{
    if (!ctx)
        return KVFUSE_EINVAL;
    Ctx *c = &ctx->c;
    if (!plan || !out)
        return fail(c, KVFUSE_EINVAL, "group counters: null plan or output");
    const WorkDesc &w = plan->p.work;
    if (n_groups != w.G)
        return fail(c, KVFUSE_EINVAL, "group counters: n_groups must be the plan's number of groups");
    std::vector<int32_t> raw((size_t)w.G * 8);
    KVF_HIP(c, hipStreamSynchronize(c->stream));
    KVF_HIP(c, hipMemcpy(raw.data(), w.counters, raw.size() * sizeof(int32_t), hipMemcpyDeviceToHost));
    for (int g = 0; g < w.G; ++g)
        for (int k = 0; k < 4; ++k)
            out[(size_t)g * 4 + k] = raw[(size_t)g * 8 + k];
    return KVFUSE_OK;
}

int kvfuse_plan_set_group_mask(kvfuse_ctx *ctx, kvfuse_plan *plan, const uint8_t *enable)
{
    if (!ctx)
        return KVFUSE_EINVAL;
    Ctx *c = &ctx->c;
    if (!plan)
        return fail(c, KVFUSE_EINVAL, "group mask: null plan");
    Plan &p = plan->p;
    p.group_enable_host.clear();
    p.work.group_enable = enable;
    if (enable && p.work.G > 0) {
        p.group_enable_host.resize((size_t)p.work.G);
        KVF_HIP(c, hipStreamSynchronize(c->stream));
        KVF_HIP(c, hipMemcpy(p.group_enable_host.data(), enable, (size_t)p.work.G, hipMemcpyDeviceToHost));
    }
    return KVFUSE_OK;
}

int kvfuse_plan_set_screen_prefix(kvfuse_ctx *ctx, kvfuse_plan *plan, int32_t prefix_elements, float *tail_share)
{
    if (!ctx)
        return KVFUSE_EINVAL;
    if (!plan)
        return fail(&ctx->c, KVFUSE_EINVAL, "screen prefix: null plan");
    Plan &p = plan->p;
    if (prefix_elements == 0) {
        p.work.screen_prefix = 0;
        p.work.rem_k = nullptr;
        p.refresh_q8_dir();
        return KVFUSE_OK;
    }
    // elements of one 64-byte K slice of what the screen multiplies: the pool, or its one-byte copy
    const int per_slice = p.work.q8.k ? 64 : (p.pool.dtype == KVFUSE_BF16 ? 32 : 16);
    if (prefix_elements < 0 || prefix_elements >= p.pool.r || prefix_elements % per_slice != 0 || prefix_elements / per_slice < 2)
        return fail(&ctx->c, KVFUSE_EINVAL, "screen prefix: must be 0, or at least 128 bytes, a multiple of 64 bytes (of the pool, "
                                            "or of its one-byte copy when the fp8 screen is on) and shorter than a block");
    if (!tail_share)
        return fail(&ctx->c, KVFUSE_EINVAL, "screen prefix: needs a device array of G * P floats");
    p.work.screen_prefix = prefix_elements;
    p.work.rem_k = tail_share;
    p.refresh_q8_dir();
    return KVFUSE_OK;
}

int kvfuse_plan_set_screen_fp8(kvfuse_ctx *ctx, kvfuse_plan *plan, void *k8, size_t k8_bytes, float *k8_side, size_t k8_side_floats,
                               int32_t centre)
{
    if (!ctx)
        return KVFUSE_EINVAL;
    if (!plan)
        return fail(&ctx->c, KVFUSE_EINVAL, "fp8 screen: null plan");
    Plan &p = plan->p;
    if (!k8 && !k8_side) {
        p.work.q8 = Q8Desc{};
        p.q8_dir_mem = nullptr;
        return KVFUSE_OK;
    }
    if (!k8 || !k8_side)
        return fail(&ctx->c, KVFUSE_EINVAL, "fp8 screen: needs G * P * t * d bytes and 3 * G * P + G * t * d floats of device "
                                            "memory (or two nulls to switch it off)");
    if (p.pool.r % 64 != 0 || p.pool.r < 128)
        return fail(&ctx->c, KVFUSE_EINVAL, "fp8 screen: blocks must have a multiple of 64 and at least 128 elements");
    if (p.work.screen_prefix > 0 && (p.work.screen_prefix % 64 != 0 || p.work.screen_prefix < 128))
        return fail(&ctx->c, KVFUSE_EINVAL, "fp8 screen: the screen prefix in force is not a multiple of 64 elements of at least 128");
    const size_t gp = (size_t)p.pool.G * p.pool.P;
    if (k8_bytes < gp * (size_t)p.pool.r || k8_side_floats < 3 * gp + (size_t)p.pool.G * p.pool.r)
        return fail(&ctx->c, KVFUSE_EINVAL, "fp8 screen: arrays too small: need G * P * t * d bytes and 3 * G * P + G * t * d floats");
    p.work.q8.k = static_cast<uint8_t *>(k8);
    p.work.q8.err = k8_side;
    p.work.q8.scale = k8_side + gp;
    p.work.q8.alpha = k8_side + 2 * gp;
    p.q8_dir_mem = centre ? k8_side + 3 * gp : nullptr;
    p.refresh_q8_dir();
    return KVFUSE_OK;
}

int kvfuse_plan_set_assign_rule(kvfuse_ctx *ctx, kvfuse_plan *plan, int32_t rule)
{
    if (!ctx)
        return KVFUSE_EINVAL;
    if (!plan)
        return fail(&ctx->c, KVFUSE_EINVAL, "assign rule: null plan");
    if (rule != KVFUSE_RULE_ARGMAX && rule != KVFUSE_RULE_FIRST_ROW)
        return fail(&ctx->c, KVFUSE_EINVAL, "assign rule: must be KVFUSE_RULE_ARGMAX or KVFUSE_RULE_FIRST_ROW");
    plan->p.assign_rule = rule;
    return KVFUSE_OK;
}

int kvfuse_decode_workspace_bytes(int32_t n_layers, int32_t B, int32_t Hq, int32_t kv_heads, int32_t d, int32_t max_blocks,
                                  size_t *bytes)
{
    if (!bytes || n_layers < 0 || B < 0 || Hq <= 0 || kv_heads <= 0 || d <= 0 || max_blocks < 0)
        return KVFUSE_EINVAL;
    *bytes = decode_workspace_bytes(n_layers, B, Hq, kv_heads, d, max_blocks);
    return KVFUSE_OK;
}

static int decode_entry(kvfuse_ctx *ctx, const kvfuse_pool *pool, const kvfuse_table *table, int32_t kv_heads,
                        int32_t layer_begin, int32_t n_layers, const void *q, const int32_t *req_start, const int32_t *ctx_len,
                        int32_t B, int32_t Hq, int32_t max_blocks, float sm_scale, void *workspace, size_t workspace_bytes,
                        float *out, bool all_heads)
{
    if (!ctx)
        return KVFUSE_EINVAL;
    Ctx *c = &ctx->c;
    if (B == 0 || n_layers == 0)
        return KVFUSE_OK;       // nothing to compute; the (empty) arrays may be null
    if (!pool || !pool->k || !pool->v || !table || !table->bt || !table->scale_k || !table->scale_v || !q || !req_start ||
        !ctx_len || !out)
        return fail(c, KVFUSE_EINVAL, "decode: null pointer");
    const int64_t groups_per_layer = all_heads ? 1 : kv_heads;
    if (kv_heads <= 0 || Hq <= 0 || Hq % kv_heads != 0 || Hq / kv_heads > 16 || B < 0 || n_layers < 0 || layer_begin < 0 ||
        max_blocks < 0 || (int64_t)(layer_begin + n_layers) * groups_per_layer > pool->G)
        return fail(c, KVFUSE_EINVAL, "decode: head counts or layer range do not fit the pool");
    if (pool->dtype != KVFUSE_BF16 && pool->dtype != KVFUSE_F32)
        return fail(c, KVFUSE_ESHAPE, "decode: dtype must be KVFUSE_BF16 or KVFUSE_F32");
    if (all_heads && pool->d % kv_heads != 0)
        return fail(c, KVFUSE_ESHAPE, "decode (all-head blocks): pool.d must be kv_heads times the head size");
    const int head_dim = all_heads ? pool->d / kv_heads : pool->d;
    if ((head_dim != 64 && head_dim != 128) || pool->t % 16 != 0 || pool->t <= 0)
        return fail(c, KVFUSE_ESHAPE, "decode: needs a head size of 64 or 128 and t a multiple of 16");
    if (B * (int64_t)kv_heads > 65535 || n_layers > 65535)
        return fail(c, KVFUSE_ESHAPE, "decode: B * kv_heads and n_layers must be <= 65535 per call");
    const int rc = launch_decode(c->stream, to_desc(*pool), to_desc(*table), kv_heads, layer_begin, n_layers, q, req_start,
                                 ctx_len, B, Hq, max_blocks, sm_scale, workspace, workspace_bytes, out, all_heads);
    if (rc)
        return fail(c, rc, "decode: workspace too small");
    KVF_HIP(c, hipGetLastError());
    return KVFUSE_OK;
}

int kvfuse_paged_decode_attn(kvfuse_ctx *ctx, const kvfuse_pool *pool, const kvfuse_table *table, int32_t kv_heads,
                             int32_t layer_begin, int32_t n_layers, const void *q, const int32_t *req_start,
                             const int32_t *ctx_len, int32_t B, int32_t Hq, int32_t max_blocks, float sm_scale,
                             void *workspace, size_t workspace_bytes, float *out)
{
    return decode_entry(ctx, pool, table, kv_heads, layer_begin, n_layers, q, req_start, ctx_len, B, Hq, max_blocks, sm_scale,
                        workspace, workspace_bytes, out, false);
}

int kvfuse_paged_decode_attn_all_heads(kvfuse_ctx *ctx, const kvfuse_pool *pool, const kvfuse_table *table, int32_t kv_heads,
                                       int32_t layer_begin, int32_t n_layers, const void *q, const int32_t *req_start,
                                       const int32_t *ctx_len, int32_t B, int32_t Hq, int32_t max_blocks, float sm_scale,
                                       void *workspace, size_t workspace_bytes, float *out)
{
    return decode_entry(ctx, pool, table, kv_heads, layer_begin, n_layers, q, req_start, ctx_len, B, Hq, max_blocks, sm_scale,
                        workspace, workspace_bytes, out, true);
}

}  // extern "C"
