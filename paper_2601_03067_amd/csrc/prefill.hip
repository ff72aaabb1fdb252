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
// Kernel: a workgroup of 4 wavefronts takes 4 x (32 / rep) consecutive query positions of one KV head; a wavefront
// owns (32 / rep) positions x rep query heads = 32 query rows.  The context is walked in tiles of 32 tokens (two
// 16-token pieces, each from one stored block with its own instance list) that the workgroup stages in LDS, double
// buffered, so every K and V byte is fetched once per workgroup.
//   logits^T = K Q^T with v_mfma_f32_32x32x16_bf16: K rows are the A operand as they lie in LDS, the query fragments
//   (B operand) stay in registers.  In the accumulator layout a lane then owns ONE query and 16 of the 32 tokens, so
//   the online softmax (per instance: exponentials of the scaled logits, weights summed with the value scales) is
//   lane-local up to one exchange with lane ^ 32, and so is every rescaling of the output.
//   out^T += V^T P^T: the weights of a lane are already a B operand (the order of the tokens inside the summation
//   index is free as long as both operands agree); V^T fragments come from the row-major V tile through the LDS
//   transpose read ds_read_b64_tr_b16 (16 lanes x 4 values: lane i receives element i & 3 of the rows that lanes
//   i >> 2, 4 + (i >> 2), 8 + (i >> 2), 12 + (i >> 2) point at -- so when source lane s points at 4 consecutive head
//   elements 4 (s & 3) .. of token (s >> 2), lane i ends up with head element i of 4 consecutive tokens).
//   Weights are split into a bfloat16 head and remainder (two MFMAs) as in the decode kernels.
// bfloat16 pools only.
#include "common.h"

#include <algorithm>
#include <new>
#include <vector>

namespace kvfuse {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));

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

typedef float floatx16 __attribute__((ext_vector_type(16)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));

// One 16-token piece of the context: where its K and V rows are, whose scale pairs apply, and the absolute
// position of its first token for the causal test (very negative = visible to every query).
struct PPiece {
    const bf16_t *k, *v;
    const float2 *ip;       // instance list, or null: the single pair below
    float2 single;
    int n_inst;             // 0 = no such piece (past the end of the walk)
    int tok_base;
};

template <int D>
__global__ __launch_bounds__(256, 2) void prefill_attn_kernel(PrefillArgs A)
{
    typedef bf16_t T;
    constexpr int KS = D / 16;                 // MFMA steps along the head dimension for the logits
    constexpr int DT = D / 32;                 // 32-row tiles of out^T
    constexpr int KSTR = D * 2 + 16;           // bytes per token row of the K tile (pad: conflict-free 16-byte row reads)
    constexpr int VSTR = D * 2 + 64;           // bytes per token row of the V tile (pad: conflict-free transpose reads)
    constexpr int RCH = D / 8;                 // 16-byte chunks per token row
    constexpr int LPT = 32 * RCH / 256;        // chunks per thread, per tensor and tile (2 for D = 128, 1 for D = 64)

    __shared__ __attribute__((aligned(16))) char k_lds[2][32 * KSTR];
    __shared__ __attribute__((aligned(16))) char v_lds[2][32 * VSTR];

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

    // rows of this wavefront: lane & 31 = query row, lane >> 5 = which half of the tokens / head elements it holds
    const int qrow = lane & 31, h2 = lane >> 5;
    const int wg_first = A.q_begin + (int)blockIdx.x * 4 * A.npw;
    const int pos_last_wg = min(A.q_end - 1, wg_first + 4 * A.npw - 1);
    const int pos_first = wg_first + wave * A.npw;                // may lie past the end: such a wavefront only helps loading
    const bool wave_live = pos_first < A.q_end;
    const int pos_last = min(A.q_end - 1, pos_first + A.npw - 1);
    const int rs = qrow / A.rep_pad, hh = qrow - rs * A.rep_pad;
    const bool row_used = wave_live && pos_first + rs <= pos_last && hh < A.rep;
    const int my_pos = wave_live ? min(pos_first + rs, pos_last) : A.q_end - 1;   // unused rows mask like a real one

    uint4 qf[KS];                                     // B operand of step ks: head elements 16 ks + 8 h2 .. + 7 of the row
    {
        const int64_t qi = (int64_t)li * (A.q_end - A.q_begin) + (my_pos - A.q_begin);
        const T *qp = (const T *)A.q + (qi * A.Hq + (int64_t)kvh * A.rep + (row_used ? hh : 0)) * D + 8 * h2;
#pragma unroll
        for (int ks = 0; ks < KS; ++ks)
            qf[ks] = row_used ? *reinterpret_cast<const uint4 *>(qp + 16 * ks) : make_uint4(0, 0, 0, 0);
    }

    // ---- the walk: pieces of the part before the chunk (distinct stored blocks with their instances), then the
    //      chunk's own blocks up to the last position of this workgroup
    const int ppb = A.t / 16;                                     // pieces per block
    const int e0 = A.entry_begin[gi], e1 = A.entry_begin[gi + 1];
    const int n_pre = (e1 - e0) * ppb;
    const int n_pieces = n_pre + (pos_last_wg - A.chunk_begin) / 16 + 1;
    const int n_tiles = (n_pieces + 1) / 2;
    auto piece_at = [&](int p) __attribute__((always_inline)) {
        PPiece pc;
        pc.k = kg; pc.v = vg; pc.ip = nullptr; pc.single = make_float2(0.0f, 0.0f); pc.n_inst = 0; pc.tok_base = 0;
        if (p < n_pre) {
            const PEntry en = A.entries[e0 + p / ppb];
            const int sub = (p % ppb) * 16;
            pc.k = kg + (int64_t)en.phys * r + (int64_t)sub * D;
            pc.v = vg + (int64_t)en.phys * r + (int64_t)sub * D;
            pc.ip = A.inst + en.inst_off;
            pc.n_inst = en.inst_cnt;
            pc.tok_base = -(1 << 30);
        } else if (p < n_pieces) {
            const int cp = p - n_pre;
            const int tok = A.chunk_begin + cp * 16;
            const int x = A.req_start + tok / A.t;
            const int phys = min(max(btg[x], 0), A.P - 1);      // a bad id in the table must not leave the pool
            const int sub = tok % A.t;
            pc.k = kg + (int64_t)phys * r + (int64_t)sub * D;
            pc.v = vg + (int64_t)phys * r + (int64_t)sub * D;
            pc.single = make_float2(skg[x], svg[x]);
            pc.n_inst = 1;
            pc.tok_base = tok;
        }
        return pc;
    };

    // global -> registers -> LDS, LPT chunks per thread and tensor: chunk c of a tile = token c / RCH, row chunk c % RCH
    // two register sets: the tile after next is already on its way while the next one waits to be written to LDS
    uint4 kr0[LPT], vr0[LPT], kr1[LPT], vr1[LPT];
    auto fetch = [&](int ti, uint4 (&kreg)[LPT], uint4 (&vreg)[LPT]) __attribute__((always_inline)) {
#pragma unroll
        for (int u = 0; u < LPT; ++u) {
            const int c = tid + 256 * u;
            const int tok = c / RCH, rc = c % RCH;                // token 0 .. 31 of the tile
            const PPiece pc = piece_at(2 * ti + (tok >> 4));
            const bool ok = pc.n_inst > 0;
            // values of tokens that no query of this workgroup may see can be anything (tail of the last block): zero
            const bool v_ok = ok && pc.tok_base + (tok & 15) <= pos_last_wg;
            const int64_t off = (int64_t)(tok & 15) * D + rc * 8;
            kreg[u] = ok ? *reinterpret_cast<const uint4 *>(pc.k + off) : make_uint4(0, 0, 0, 0);
            vreg[u] = v_ok ? *reinterpret_cast<const uint4 *>(pc.v + off) : make_uint4(0, 0, 0, 0);
        }
    };
    auto stash = [&](int buf, const uint4 (&kreg)[LPT], const uint4 (&vreg)[LPT]) __attribute__((always_inline)) {
#pragma unroll
        for (int u = 0; u < LPT; ++u) {
            const int c = tid + 256 * u;
            const int tok = c / RCH, rc = c % RCH;
            *reinterpret_cast<uint4 *>(&k_lds[buf][tok * KSTR + rc * 16]) = kreg[u];
            *reinterpret_cast<uint4 *>(&v_lds[buf][tok * VSTR + rc * 16]) = vreg[u];
        }
    };

    float m_run = -INFINITY, l_run = 0.0f;       // running maximum in base-2 units, running sum
    floatx16 o[DT];
#pragma unroll
    for (int dt = 0; dt < DT; ++dt)
#pragma unroll
        for (int i = 0; i < 16; ++i)
            o[dt][i] = 0.0f;

    // this lane's addresses inside a tile: K row for the logits, V patch for the transpose reads
    const int k_off = qrow * KSTR + h2 * 16;
    const int l16 = lane & 15;
    const int v_off = (4 * h2 + (l16 >> 2)) * VSTR + (16 * ((lane >> 4) & 1) + 4 * (l16 & 3)) * 2;

    auto compute = [&](int ti, int buf) __attribute__((always_inline)) {
        if (wave_live) {
            // ---- logits^T of the tile: 32 tokens x 32 query rows
            floatx16 z;
#pragma unroll
            for (int i = 0; i < 16; ++i)
                z[i] = 0.0f;
#pragma unroll
            for (int ks = 0; ks < KS; ++ks) {
                const uint4 ka = *reinterpret_cast<const uint4 *>(&k_lds[buf][k_off + ks * 32]);
                z = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, ka), __builtin_bit_cast(bf16x8, qf[ks]), z, 0, 0, 0);
            }
            // accumulator i of this lane: token 8 (i / 4) + 4 h2 + i % 4 of the tile, i.e. piece i / 8
            const PPiece pc0 = piece_at(2 * ti), pc1 = piece_at(2 * ti + 1);
            // everything below works in base 2: exp(x) = exp2(x * log2(e)), and v_exp_f32 is an exp2
            constexpr float LOG2E = 1.4426950408889634f;
            float bmax, m_new, corr, psum = 0.0f;
            float pw[16];
#pragma unroll
            for (int i = 0; i < 16; ++i)
                pw[i] = 0.0f;
            // The common tile: both pieces lie before the chunk (visible to every query) and stand for one logical
            // block each.  No masks and no instance loops: the kernel is bound by instruction issue, and this is
            // where most of its instructions went.
            const bool plain = pc0.tok_base < 0 && pc1.tok_base < 0 && pc0.n_inst == 1 && pc1.n_inst == 1;
            if (__builtin_amdgcn_readfirstlane((int)plain)) {
                const float2 s0 = pc0.ip[0], s1 = pc1.ip[0];
                const float zs0 = A.sm_scale * LOG2E * s0.x, zs1 = A.sm_scale * LOG2E * s1.x;
                float t[16];
#pragma unroll
                for (int i = 0; i < 16; ++i)
                    t[i] = z[i] * (i < 8 ? zs0 : zs1);
                bmax = fmaxf(fmaxf(fmaxf(fmaxf(t[0], t[1]), fmaxf(t[2], t[3])), fmaxf(fmaxf(t[4], t[5]), fmaxf(t[6], t[7]))),
                             fmaxf(fmaxf(fmaxf(t[8], t[9]), fmaxf(t[10], t[11])), fmaxf(fmaxf(t[12], t[13]), fmaxf(t[14], t[15]))));
                bmax = fmaxf(bmax, __shfl_xor(bmax, 32, 64));
                m_new = fmaxf(m_run, bmax);
                corr = __builtin_amdgcn_exp2f(m_run - m_new);          // m_new is finite here; 0 on the very first tile
#pragma unroll
                for (int i = 0; i < 16; ++i) {
                    const float pr = __builtin_amdgcn_exp2f(t[i] - m_new);
                    psum += pr;
                    pw[i] = pr * (i < 8 ? s0.y : s1.y);
                }
            } else if (__builtin_amdgcn_readfirstlane((int)(pc0.tok_base < 0 && pc1.tok_base < 0 && pc1.n_inst > 0))) {
                // both pieces before the chunk, several logical blocks behind at least one of them: instance loops, no masks
                bmax = -INFINITY;
#pragma unroll
                for (int half = 0; half < 2; ++half) {
                    const PPiece &pc = half ? pc1 : pc0;
                    const int ni = __builtin_amdgcn_readfirstlane(pc.n_inst);
                    for (int q = 0; q < ni; ++q) {
                        const float zs = A.sm_scale * LOG2E * pc.ip[q].x;
#pragma unroll
                        for (int i = 8 * half; i < 8 * half + 8; ++i)
                            bmax = fmaxf(bmax, z[i] * zs);
                    }
                }
                bmax = fmaxf(bmax, __shfl_xor(bmax, 32, 64));
                m_new = fmaxf(m_run, bmax);
                corr = __builtin_amdgcn_exp2f(m_run - m_new);
#pragma unroll
                for (int half = 0; half < 2; ++half) {
                    const PPiece &pc = half ? pc1 : pc0;
                    const int ni = __builtin_amdgcn_readfirstlane(pc.n_inst);
                    for (int q = 0; q < ni; ++q) {
                        const float2 sc = pc.ip[q];
                        const float zs = A.sm_scale * LOG2E * sc.x;
#pragma unroll
                        for (int i = 8 * half; i < 8 * half + 8; ++i) {
                            const float pr = __builtin_amdgcn_exp2f(fmaf(z[i], zs, -m_new));
                            psum += pr;
                            pw[i] = fmaf(pr, sc.y, pw[i]);
                        }
                    }
                }
            } else {
                // pieces before the chunk are visible to every query: no masks in that (common) case
                const bool masked = pc0.tok_base >= 0 || pc1.tok_base >= 0 || pc1.n_inst == 0;
                bool vis[16];
#pragma unroll
                for (int i = 0; i < 16; ++i) {
                    const int tp = 8 * ((i >> 2) & 1) + 4 * h2 + (i & 3);
                    const PPiece &pc = i < 8 ? pc0 : pc1;
                    vis[i] = !masked || (pc.n_inst > 0 && pc.tok_base + tp <= my_pos);
                }
                bmax = -INFINITY;
#pragma unroll
                for (int half = 0; half < 2; ++half) {
                    const PPiece &pc = half ? pc1 : pc0;
                    for (int q = 0; q < pc.n_inst; ++q) {
                        const float zs = A.sm_scale * LOG2E * (pc.ip ? pc.ip[q].x : pc.single.x);
#pragma unroll
                        for (int i = 8 * half; i < 8 * half + 8; ++i)
                            bmax = fmaxf(bmax, vis[i] ? z[i] * zs : -INFINITY);
                    }
                }
                bmax = fmaxf(bmax, __shfl_xor(bmax, 32, 64));
                m_new = fmaxf(m_run, bmax);
                corr = m_new == -INFINITY ? 1.0f : __builtin_amdgcn_exp2f(m_run - m_new);   // 0 on the first visible tile
#pragma unroll
                for (int half = 0; half < 2; ++half) {
                    const PPiece &pc = half ? pc1 : pc0;
                    for (int q = 0; q < pc.n_inst; ++q) {
                        const float2 sc = pc.ip ? pc.ip[q] : pc.single;
                        const float zs = A.sm_scale * LOG2E * sc.x;
#pragma unroll
                        for (int i = 8 * half; i < 8 * half + 8; ++i) {
                            const float pr = vis[i] ? __builtin_amdgcn_exp2f(fmaf(z[i], zs, -m_new)) : 0.0f;
                            psum += pr;
                            pw[i] = fmaf(pr, sc.y, pw[i]);
                        }
                    }
                }
            }
            psum += __shfl_xor(psum, 32, 64);
            l_run = l_run * corr + psum;
            m_run = m_new;
            if (__builtin_amdgcn_ballot_w64(corr != 1.0f)) {
#pragma unroll
                for (int dt = 0; dt < DT; ++dt)
#pragma unroll
                    for (int i = 0; i < 16; ++i)
                        o[dt][i] *= corr;
            }
            // weights as B operands: the 8 values of MFMA jj are accumulators 8 jj .. 8 jj + 7, as a bfloat16 head
            // (nearest) plus the bfloat16 of what is left
            bf16x8 p_hi[2], p_lo[2];
#pragma unroll
            for (int jj = 0; jj < 2; ++jj)
#pragma unroll
                for (int e = 0; e < 8; ++e) {
                    const float w = pw[8 * jj + e];
                    const __bf16 hb = (__bf16)w;
                    p_hi[jj][e] = hb;
                    p_lo[jj][e] = (__bf16)(w - (float)hb);
                }
            // ---- out^T += V^T P^T
#pragma unroll
            for (int jj = 0; jj < 2; ++jj) {
#pragma unroll
                for (int dt = 0; dt < DT; ++dt) {
                    const char *vp = &v_lds[buf][v_off + (16 * jj) * VSTR + dt * 64];
                    const bf16x4 t0 = __builtin_amdgcn_ds_read_tr16_b64_v4bf16(
                        (__attribute__((address_space(3))) bf16x4 *)(vp));
                    const bf16x4 t1 = __builtin_amdgcn_ds_read_tr16_b64_v4bf16(
                        (__attribute__((address_space(3))) bf16x4 *)(vp + 8 * VSTR));
                    const bf16x8 va = __builtin_shufflevector(t0, t1, 0, 1, 2, 3, 4, 5, 6, 7);
                    o[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(va, p_hi[jj], o[dt], 0, 0, 0);
                    o[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(va, p_lo[jj], o[dt], 0, 0, 0);
                }
            }
        }
    };

    fetch(0, kr0, vr0);
    if (n_tiles > 1)
        fetch(1, kr1, vr1);
    stash(0, kr0, vr0);
    __syncthreads();
    for (int ti = 0; ti < n_tiles; ti += 2) {
        // tile ti is in buffer 0, tile ti + 1 in register set 1
        if (ti + 2 < n_tiles)
            fetch(ti + 2, kr0, vr0);
        compute(ti, 0);
        if (ti + 1 < n_tiles)
            stash(1, kr1, vr1);
        __syncthreads();
        if (ti + 1 >= n_tiles)
            break;
        // tile ti + 1 is in buffer 1, tile ti + 2 in register set 0
        if (ti + 3 < n_tiles)
            fetch(ti + 3, kr1, vr1);
        compute(ti + 1, 1);
        if (ti + 2 < n_tiles)
            stash(0, kr0, vr0);
        __syncthreads();
    }

    // ---- normalise and store: this lane holds out[row qrow][head element 32 dt + 8 (i / 4) + 4 h2 + i % 4]
    if (row_used) {
        const float inv = l_run > 0.0f ? 1.0f / l_run : 0.0f;
        const int64_t qi = (int64_t)li * (A.q_end - A.q_begin) + (pos_first + rs - A.q_begin);
        float *dst = A.out + (qi * A.Hq + (int64_t)kvh * A.rep + hh) * D + 4 * h2;
#pragma unroll
        for (int dt = 0; dt < DT; ++dt)
#pragma unroll
            for (int g4 = 0; g4 < 4; ++g4)
                *reinterpret_cast<float4 *>(dst + 32 * dt + 8 * g4) =
                    make_float4(o[dt][4 * g4] * inv, o[dt][4 * g4 + 1] * inv, o[dt][4 * g4 + 2] * inv, o[dt][4 * g4 + 3] * inv);
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
    pl->npw = 32 / pl->rep_pad;
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
