// Chunked-prefill attention over a fused cache with reuse of the work on fused blocks (motivation section: with
// chunked prefill, any softmax-attention computation that involves a fused block can be reused for the later
// instances of that block, and the result is the merge, with rescaling, of the fused part and the unique part).
//
// One request (Chunks Fast-Fusion is per request).  The queries are a run of tokens [q_begin, q_end) of one chunk
// that starts at token chunk_begin; the query at position pos sees the tokens 0 .. pos of the request through the
// block table: logical block x is scale_k[x] * K[bt[x]], scale_v[x] * V[bt[x]].
//
// What is reused.  Every logical block that ends before the chunk is visible to every query of the chunk.  Among
// those, the logical blocks that point at the same stored block p differ only by their two scale factors, so
//     logits of instance i   = scale_k[x_i] * (Q K_p^T)          -- one matrix product Q K_p^T for all instances
//     their weighted values  = (sum_i scale_v[x_i] P_i) V_p      -- one matrix product with V_p
// The host plan lists, per group, the distinct stored blocks of that part of the context with their instances'
// scale pairs; only the exponentials are taken per instance.  The blocks of the chunk itself (the unique part:
// blocks of one leaf never fuse with each other, and they need the causal mask) are walked one by one from the
// table.  With reuse switched off the plan lists every logical block as its own entry, which gives the baseline
// the reuse is measured against.
//
// Kernel: a workgroup of 4 wavefronts takes 4 x (16 / rep) consecutive query positions of one KV head; a wavefront
// owns (16 / rep) positions x rep query heads = the 16 rows of an MFMA tile and walks all blocks itself, so no
// partial states are exchanged.  Logits by v_mfma_f32_16x16x32_bf16 (K fragments straight from global memory),
// online softmax in fp32, P.V by v_mfma_f32_16x16x16_bf16 after transposing each 16 x 16 piece of V through one
// MFMA against the identity, probabilities split into a bfloat16 head and remainder -- the same arithmetic as the
// shared-block decode kernel.  bfloat16 pools only.
#include "common.h"

#include <algorithm>
#include <new>
#include <vector>

namespace kvfuse {

typedef float floatx4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef short short4v __attribute__((ext_vector_type(4)));

struct PEntry {          // 16 bytes
    int32_t phys, inst_off, inst_cnt, pad;
};

struct PrefillArgs {
    const void *kpool, *vpool;
    const int32_t *bt;
    const float *scale_k, *scale_v;
    const void *q;
    const PEntry *entries;
    const float2 *inst;              // (scale_k, scale_v) of every instance
    const int32_t *entry_begin;      // [groups of the plan + 1]
    float *out;                      // [n_layers][Nq][Hq][D]
    int32_t P, n, t, kv_heads, layer_begin, Hq, rep, rep_pad, npw;
    int32_t req_start, q_begin, q_end, chunk_begin;
    float sm_scale;
};

template <int D>
__global__ __launch_bounds__(256, 4) void prefill_attn_kernel(PrefillArgs A)
{
    typedef bf16_t T;
    constexpr int NF = D / 32;             // 16-byte fragments per lane (a lane owns a quarter of a token row)
    constexpr int NT = 2 * NF;             // 16-column accumulator tiles

    __shared__ __attribute__((aligned(16))) float c_lds[4][16];   // per wave: a per-row factor on its way to the accumulator layout

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int kvh = blockIdx.y, li = blockIdx.z;
    const int gi = li * A.kv_heads + kvh;                        // group index within the plan
    const int g = (A.layer_begin + li) * A.kv_heads + kvh;
    const int64_t r = (int64_t)A.t * D;
    const T *kg = (const T *)A.kpool + (int64_t)g * A.P * r;
    const T *vg = (const T *)A.vpool + (int64_t)g * A.P * r;
    const int32_t *btg = A.bt + (int64_t)g * A.n;
    const float *skg = A.scale_k + (int64_t)g * A.n;
    const float *svg = A.scale_v + (int64_t)g * A.n;

    const int head = lane & 15, tg = lane >> 4;      // logits / P: row, token group;  K and V loads: token, row quarter
    const int pos_first = A.q_begin + ((int)blockIdx.x * 4 + wave) * A.npw;    // first query position of this wavefront
    if (pos_first >= A.q_end)
        return;                                       // no barrier below: a whole wavefront may leave
    const int pos_last = min(A.q_end - 1, pos_first + A.npw - 1);
    const int rs = head / A.rep_pad, hh = head - rs * A.rep_pad;
    const bool row_used = pos_first + rs <= pos_last && hh < A.rep;
    const int my_pos = min(pos_first + rs, pos_last);             // unused rows mask like the wavefront's last position

    uint4 qf[NF];
    {
        const int64_t qi = (int64_t)li * (A.q_end - A.q_begin) + (my_pos - A.q_begin);
        const T *qrow = (const T *)A.q + (qi * A.Hq + (int64_t)kvh * A.rep + (row_used ? hh : 0)) * D + tg * (D / 4);
#pragma unroll
        for (int f = 0; f < NF; ++f)
            qf[f] = row_used ? reinterpret_cast<const uint4 *>(qrow)[f] : make_uint4(0, 0, 0, 0);
    }
    short4v ident;                                    // identity as a B operand: I[k = 4 * tg + i][n = head]
#pragma unroll
    for (int i = 0; i < 4; ++i)
        ident[i] = (4 * tg + i == head) ? (short)0x3F80 : (short)0;

    float m_run = -INFINITY, l_run = 0.0f;
    floatx4 o[NT];
#pragma unroll
    for (int nt = 0; nt < NT; ++nt)
        o[nt] = floatx4{0.0f, 0.0f, 0.0f, 0.0f};

    // One 16-token piece of a stored block: logits once, then every instance's probabilities, then one P.V.
    //   n_inst instances with scale pairs inst_ptr[0 .. n_inst);  tok_base = absolute position of the piece's first
    //   token for the causal test (a very negative value for pieces that are visible to everybody)
    auto piece = [&](const T *kblk, const T *vblk, int sub, const float2 *inst_ptr, int n_inst, int tok_base, int n_valid)
        __attribute__((always_inline)) {
        const uint4 *krow = reinterpret_cast<const uint4 *>(kblk + (int64_t)(sub + head) * D + tg * (D / 4));
        const uint4 *vrow = reinterpret_cast<const uint4 *>(vblk + (int64_t)(sub + head) * D + tg * (D / 4));
        uint4 kf[NF], vf[NF];
#pragma unroll
        for (int f = 0; f < NF; ++f)
            kf[f] = krow[f];
#pragma unroll
        for (int f = 0; f < NF; ++f)
            vf[f] = vrow[f];
        floatx4 z = {0.0f, 0.0f, 0.0f, 0.0f};
#pragma unroll
        for (int f = 0; f < NF; ++f)
            z = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, kf[f]), __builtin_bit_cast(bf16x8, qf[f]), z, 0, 0, 0);
        // which of this lane's 4 tokens its row may see
        bool vis[4];
#pragma unroll
        for (int v = 0; v < 4; ++v)
            vis[v] = tok_base + 4 * tg + v <= my_pos && 4 * tg + v < n_valid;
        // block maximum over all instances
        float bmax = -INFINITY;
        for (int i = 0; i < n_inst; ++i) {
            const float zs = A.sm_scale * inst_ptr[i].x;
#pragma unroll
            for (int v = 0; v < 4; ++v)
                bmax = fmaxf(bmax, vis[v] ? z[v] * zs : -INFINITY);
        }
        bmax = fmaxf(bmax, __shfl_xor(bmax, 16, 64));
        bmax = fmaxf(bmax, __shfl_xor(bmax, 32, 64));
        const float m_new = fmaxf(m_run, bmax);
        const float corr = m_new == -INFINITY ? 1.0f : __expf(m_run - m_new);     // 0 on the first visible piece
        float psum = 0.0f;
        float pw[4] = {0.0f, 0.0f, 0.0f, 0.0f};
        for (int i = 0; i < n_inst; ++i) {
            const float2 sc = inst_ptr[i];
            const float zs = A.sm_scale * sc.x;
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                const float pr = vis[v] ? __expf(z[v] * zs - m_new) : 0.0f;
                psum += pr;
                pw[v] = fmaf(pr, sc.y, pw[v]);
            }
        }
        psum += __shfl_xor(psum, 16, 64);
        psum += __shfl_xor(psum, 32, 64);
        l_run = l_run * corr + psum;
        m_run = m_new;
        short4v p_hi, p_lo;
#pragma unroll
        for (int v = 0; v < 4; ++v) {
            const uint32_t hb = __float_as_uint(pw[v]) & 0xFFFF0000u;            // bfloat16 head (truncated)
            const float rest = pw[v] - __uint_as_float(hb);                       // exact
            p_hi[v] = (short)(hb >> 16);
            p_lo[v] = (short)((__float_as_uint(rest) + 0x8000u) >> 16);           // bfloat16 remainder (rounded)
        }
        if (tg == 0)
            c_lds[wave][head] = corr;
        __builtin_amdgcn_wave_barrier();
        const float4 c4 = *reinterpret_cast<const float4 *>(&c_lds[wave][4 * tg]);   // rows 4 * tg .. + 3 of every tile
#pragma unroll
        for (int nt = 0; nt < NT; ++nt) {
            o[nt][0] *= c4.x; o[nt][1] *= c4.y; o[nt][2] *= c4.z; o[nt][3] *= c4.w;
        }
        // V rows that no row of this wavefront may see can hold anything (the tail of the last block): zero them
        if (tok_base + head > pos_last || head >= n_valid) {
#pragma unroll
            for (int f = 0; f < NF; ++f)
                vf[f] = make_uint4(0, 0, 0, 0);
        }
#pragma unroll
        for (int f = 0; f < NF; ++f) {
#pragma unroll
            for (int hs = 0; hs < 2; ++hs) {
                const uint32_t w0 = hs ? vf[f].z : vf[f].x, w1 = hs ? vf[f].w : vf[f].y;
                short4v va;
                va[0] = (short)(w0 & 0xFFFFu); va[1] = (short)(w0 >> 16);
                va[2] = (short)(w1 & 0xFFFFu); va[3] = (short)(w1 >> 16);
                const floatx4 vt = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(va, ident, floatx4{0.0f, 0.0f, 0.0f, 0.0f}, 0, 0, 0);
                short4v vb;
#pragma unroll
                for (int i = 0; i < 4; ++i)
                    vb[i] = (short)(__float_as_uint(vt[i]) >> 16);
                o[2 * f + hs] = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(p_hi, vb, o[2 * f + hs], 0, 0, 0);
                o[2 * f + hs] = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(p_lo, vb, o[2 * f + hs], 0, 0, 0);
            }
        }
        __builtin_amdgcn_wave_barrier();
    };

    // ---- the part before the chunk: distinct stored blocks with their instances, visible to every query
    {
        const int e0 = A.entry_begin[gi], e1 = A.entry_begin[gi + 1];
        for (int e = e0; e < e1; ++e) {
            const PEntry en = A.entries[e];
            const T *kblk = kg + (int64_t)en.phys * r;
            const T *vblk = vg + (int64_t)en.phys * r;
            for (int sub = 0; sub < A.t; sub += 16)
                piece(kblk, vblk, sub, A.inst + en.inst_off, en.inst_cnt, -(1 << 30), 16);
        }
    }
    // ---- the chunk itself, block by block with the causal mask
    {
        const int xb0 = A.chunk_begin / A.t, xb1 = pos_last / A.t;
        for (int xb = xb0; xb <= xb1; ++xb) {
            const int x = A.req_start + xb;
            const int phys = btg[x];
            const float2 sc = make_float2(skg[x], svg[x]);
            const T *kblk = kg + (int64_t)phys * r;
            const T *vblk = vg + (int64_t)phys * r;
            for (int sub = 0; sub < A.t; sub += 16) {
                if (xb * A.t + sub > pos_last)
                    break;
                piece(kblk, vblk, sub, &sc, 1, xb * A.t + sub, 16);
            }
        }
    }

    // ---- normalise and store: this lane holds o[row 4 * tg + i][column slot head] of every tile
    if (tg == 0)
        c_lds[wave][head] = l_run > 0.0f ? 1.0f / l_run : 0.0f;
    __builtin_amdgcn_wave_barrier();
    const float4 inv4 = *reinterpret_cast<const float4 *>(&c_lds[wave][4 * tg]);
    const float inv[4] = {inv4.x, inv4.y, inv4.z, inv4.w};
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int row = 4 * tg + i;
        const int rrs = row / A.rep_pad, rhh = row - rrs * A.rep_pad;
        if (pos_first + rrs > pos_last || rhh >= A.rep)
            continue;
        const int64_t qi = (int64_t)li * (A.q_end - A.q_begin) + (pos_first + rrs - A.q_begin);
        float *dst = A.out + (qi * A.Hq + (int64_t)kvh * A.rep + rhh) * D;
#pragma unroll
        for (int f = 0; f < NF; ++f)
#pragma unroll
            for (int hs = 0; hs < 2; ++hs)
                dst[(D / 4) * (head >> 2) + 8 * f + 4 * hs + (head & 3)] = o[2 * f + hs][i] * inv[i];
    }
}

static int pad_pow2_p(int rep)
{
    int p = 1;
    while (p < rep)
        p <<= 1;
    return p;
}

}  // namespace kvfuse

using namespace kvfuse;

struct kvfuse_prefill_plan {
    int32_t dtype = 0, P = 0, n = 0, t = 0, d = 0, G = 0;
    int32_t kv_heads = 0, layer_begin = 0, n_layers = 0, Hq = 0, rep = 0, rep_pad = 0, npw = 1;
    int32_t req_start = 0, q_begin = 0, q_end = 0, chunk_begin = 0;
    std::vector<PEntry> entries;
    std::vector<float2> inst;
    std::vector<int32_t> entry_begin;
    kvfuse_prefill_plan_info info = {};
    size_t off_entries = 0, off_inst = 0, off_begin = 0, bytes = 0;
    char *dev = nullptr;
};

static size_t up256p(size_t x) { return (x + 255) & ~(size_t)255; }

extern "C" {

int kvfuse_prefill_plan_build(kvfuse_ctx *ctx, const kvfuse_pool *pool, const kvfuse_table *table, int32_t kv_heads,
                              int32_t layer_begin, int32_t n_layers, int32_t req_start, int32_t chunk_begin, int32_t q_begin,
                              int32_t q_end, int32_t Hq, int32_t reuse, kvfuse_prefill_plan **plan,
                              kvfuse_prefill_plan_info *info)
{
    if (!ctx)
        return KVFUSE_EINVAL;
    Ctx *c = &ctx->c;
    if (!plan)
        return fail(c, KVFUSE_EINVAL, "prefill plan: null output");
    *plan = nullptr;
    if (!pool || !table || !table->bt || !table->scale_k || !table->scale_v)
        return fail(c, KVFUSE_EINVAL, "prefill plan: null pointer");
    if (pool->dtype != KVFUSE_BF16)
        return fail(c, KVFUSE_ESHAPE, "prefill: bfloat16 pools only");
    if ((pool->d != 64 && pool->d != 128) || pool->t % 16 != 0 || pool->t <= 0)
        return fail(c, KVFUSE_ESHAPE, "prefill: needs d in {64, 128} and t a multiple of 16");
    if (kv_heads <= 0 || Hq <= 0 || Hq % kv_heads != 0 || Hq / kv_heads > 16 || n_layers < 0 || layer_begin < 0 ||
        (int64_t)(layer_begin + n_layers) * kv_heads > pool->G)
        return fail(c, KVFUSE_EINVAL, "prefill plan: head counts or layer range do not fit the pool");
    const int t = pool->t, n = table->n;
    if (req_start < 0 || chunk_begin < 0 || chunk_begin % t != 0 || q_begin < chunk_begin || q_end < q_begin ||
        (int64_t)req_start + ((int64_t)q_end + t - 1) / t > n)
        return fail(c, KVFUSE_EINVAL, "prefill plan: need 0 <= chunk_begin (a multiple of t) <= q_begin <= q_end and the "
                                      "request's blocks inside the table");
    if (kv_heads > 65535 || n_layers > 65535)
        return fail(c, KVFUSE_ESHAPE, "prefill plan: kv_heads and n_layers must be <= 65535 per call");
    kvfuse_prefill_plan *pl = new (std::nothrow) kvfuse_prefill_plan();
    if (!pl)
        return fail(c, KVFUSE_ENOMEM, "prefill plan: out of host memory");
    pl->dtype = pool->dtype; pl->P = pool->P; pl->n = n; pl->t = t; pl->d = pool->d; pl->G = pool->G;
    pl->kv_heads = kv_heads; pl->layer_begin = layer_begin; pl->n_layers = n_layers; pl->Hq = Hq;
    pl->rep = Hq / kv_heads;
    pl->rep_pad = pad_pow2_p(pl->rep);
    pl->npw = 16 / pl->rep_pad;
    pl->req_start = req_start; pl->q_begin = q_begin; pl->q_end = q_end; pl->chunk_begin = chunk_begin;

    const int Gsel = n_layers * kv_heads;
    const int nb_pre = chunk_begin / t;                 // logical blocks that end before the chunk
    std::vector<int32_t> bt((size_t)Gsel * nb_pre);
    std::vector<float> sk((size_t)Gsel * nb_pre), sv((size_t)Gsel * nb_pre);
    if (!bt.empty()) {
        hipError_t e = hipStreamSynchronize(c->stream);
        const int64_t g0 = (int64_t)layer_begin * kv_heads;
        if (e == hipSuccess)
            e = hipMemcpy2D(bt.data(), (size_t)nb_pre * 4, table->bt + g0 * n + req_start, (size_t)n * 4, (size_t)nb_pre * 4,
                            (size_t)Gsel, hipMemcpyDeviceToHost);
        if (e == hipSuccess)
            e = hipMemcpy2D(sk.data(), (size_t)nb_pre * 4, table->scale_k + g0 * n + req_start, (size_t)n * 4,
                            (size_t)nb_pre * 4, (size_t)Gsel, hipMemcpyDeviceToHost);
        if (e == hipSuccess)
            e = hipMemcpy2D(sv.data(), (size_t)nb_pre * 4, table->scale_v + g0 * n + req_start, (size_t)n * 4,
                            (size_t)nb_pre * 4, (size_t)Gsel, hipMemcpyDeviceToHost);
        if (e != hipSuccess) {
            delete pl;
            return fail(c, KVFUSE_EHIP, std::string("prefill plan: reading the table: ") + hipGetErrorString(e));
        }
    }
    kvfuse_prefill_plan_info &I = pl->info;
    pl->entry_begin.assign((size_t)Gsel + 1, 0);
    std::vector<std::pair<int32_t, int32_t>> order((size_t)nb_pre);      // (stored block, logical index)
    for (int gi = 0; gi < Gsel; ++gi) {
        const int32_t *b = bt.data() + (size_t)gi * nb_pre;
        for (int x = 0; x < nb_pre; ++x) {
            if (b[x] < 0 || b[x] >= pool->P) {
                delete pl;
                return fail(c, KVFUSE_EINVAL, "prefill plan: the table holds a physical id outside the pool");
            }
            order[(size_t)x] = std::make_pair(reuse ? b[x] : x, (int32_t)x);
        }
        std::sort(order.begin(), order.end());
        for (size_t s = 0; s < order.size();) {
            size_t e = s + 1;
            while (e < order.size() && order[e].first == order[s].first)
                ++e;
            PEntry en;
            en.phys = b[order[s].second];
            en.inst_off = (int32_t)pl->inst.size();
            en.inst_cnt = (int32_t)(e - s);
            en.pad = 0;
            for (size_t k = s; k < e; ++k)
                pl->inst.push_back(make_float2(sk[(size_t)gi * nb_pre + order[k].second], sv[(size_t)gi * nb_pre + order[k].second]));
            pl->entries.push_back(en);
            s = e;
        }
        pl->entry_begin[(size_t)gi + 1] = (int32_t)pl->entries.size();
        I.logical_blocks_before_chunk += nb_pre;
        if (pl->inst.size() > (size_t)0x7FFFFFF0) {
            delete pl;
            return fail(c, KVFUSE_ESHAPE, "prefill plan: more than 2^31 instances; plan fewer layers per call");
        }
    }
    I.stored_blocks_before_chunk = (int64_t)pl->entries.size();
    size_t off = 0;
    pl->off_entries = off;
    off = up256p(off + pl->entries.size() * sizeof(PEntry));
    pl->off_inst = off;
    off = up256p(off + pl->inst.size() * sizeof(float2));
    pl->off_begin = off;
    off = up256p(off + pl->entry_begin.size() * sizeof(int32_t));
    pl->bytes = off + 256;
    I.device_bytes = (int64_t)pl->bytes;
    if (info)
        *info = I;
    *plan = pl;
    return KVFUSE_OK;
}

int kvfuse_prefill_plan_upload(kvfuse_ctx *ctx, kvfuse_prefill_plan *plan, void *workspace, size_t workspace_bytes)
{
    if (!ctx)
        return KVFUSE_EINVAL;
    Ctx *c = &ctx->c;
    if (!plan || !workspace)
        return fail(c, KVFUSE_EINVAL, "prefill plan upload: null pointer");
    if (workspace_bytes < plan->bytes)
        return fail(c, KVFUSE_ENOMEM, "prefill plan upload: workspace smaller than info.device_bytes");
    if ((reinterpret_cast<uintptr_t>(workspace) & 255) != 0)
        return fail(c, KVFUSE_EINVAL, "prefill plan upload: workspace must be 256-byte aligned");
    char *dev = static_cast<char *>(workspace);
    if (!plan->entries.empty())
        KVF_HIP(c, hipMemcpyAsync(dev + plan->off_entries, plan->entries.data(), plan->entries.size() * sizeof(PEntry),
                                  hipMemcpyHostToDevice, c->stream));
    if (!plan->inst.empty())
        KVF_HIP(c, hipMemcpyAsync(dev + plan->off_inst, plan->inst.data(), plan->inst.size() * sizeof(float2),
                                  hipMemcpyHostToDevice, c->stream));
    KVF_HIP(c, hipMemcpyAsync(dev + plan->off_begin, plan->entry_begin.data(), plan->entry_begin.size() * sizeof(int32_t),
                              hipMemcpyHostToDevice, c->stream));
    KVF_HIP(c, hipStreamSynchronize(c->stream));
    plan->dev = dev;
    return KVFUSE_OK;
}

int kvfuse_prefill_plan_destroy(kvfuse_prefill_plan *plan)
{
    delete plan;
    return KVFUSE_OK;
}

int kvfuse_prefill_attn(kvfuse_ctx *ctx, const kvfuse_pool *pool, const kvfuse_table *table, const kvfuse_prefill_plan *plan,
                        const void *q, float sm_scale, float *out)
{
    if (!ctx)
        return KVFUSE_EINVAL;
    Ctx *c = &ctx->c;
    if (!pool || !pool->k || !pool->v || !table || !table->bt || !table->scale_k || !table->scale_v || !plan || !q || !out)
        return fail(c, KVFUSE_EINVAL, "prefill: null pointer");
    if (!plan->dev)
        return fail(c, KVFUSE_EINVAL, "prefill: the plan has not been uploaded");
    if (pool->dtype != plan->dtype || pool->P != plan->P || pool->t != plan->t || pool->d != plan->d || pool->G != plan->G ||
        table->n != plan->n)
        return fail(c, KVFUSE_EINVAL, "prefill: pool or table shape differs from the one the plan was built for");
    const int nq = plan->q_end - plan->q_begin;
    if (nq <= 0 || plan->n_layers == 0)
        return KVFUSE_OK;
    PrefillArgs A;
    A.kpool = pool->k; A.vpool = pool->v; A.bt = table->bt; A.scale_k = table->scale_k; A.scale_v = table->scale_v; A.q = q;
    A.entries = reinterpret_cast<const PEntry *>(plan->dev + plan->off_entries);
    A.inst = reinterpret_cast<const float2 *>(plan->dev + plan->off_inst);
    A.entry_begin = reinterpret_cast<const int32_t *>(plan->dev + plan->off_begin);
    A.out = out;
    A.P = pool->P; A.n = table->n; A.t = pool->t; A.kv_heads = plan->kv_heads; A.layer_begin = plan->layer_begin;
    A.Hq = plan->Hq; A.rep = plan->rep; A.rep_pad = plan->rep_pad; A.npw = plan->npw;
    A.req_start = plan->req_start; A.q_begin = plan->q_begin; A.q_end = plan->q_end; A.chunk_begin = plan->chunk_begin;
    A.sm_scale = sm_scale;
    const int per_wg = 4 * plan->npw;
    const dim3 grid((unsigned)((nq + per_wg - 1) / per_wg), (unsigned)plan->kv_heads, (unsigned)plan->n_layers);
    if (pool->d == 128)
        prefill_attn_kernel<128><<<grid, 256, 0, c->stream>>>(A);
    else
        prefill_attn_kernel<64><<<grid, 256, 0, c->stream>>>(A);
    KVF_HIP(c, hipGetLastError());
    return KVFUSE_OK;
}

}  // extern "C"
