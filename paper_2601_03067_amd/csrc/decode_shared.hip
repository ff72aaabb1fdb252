// Shared-block decode attention: the attention of the paged decode step (analysis section: logits q . k / sqrt(d),
// softmax, weighted values), organised around the blocks that fusion made common to several requests.
//
// Motivation section: a fused representation lets one matrix-matrix product replace several matrix-vector
// products, and the result for a request is the merge (with rescaling) of the attention over its fused part and
// over its unique part; Algorithm 1 marks shared blocks for this purpose.
//
// Host side (the decode plan).  Per group, full blocks are grouped by physical id; physical blocks referenced by
// exactly the same set of requests (each at most once) form a cluster.  A cluster with enough blocks becomes work
// items (tile of up to NREQ requests) x (chunk of its blocks); the NREQ x rep query heads of a tile fill the rows
// of the 16-row MFMA tile that the per-request kernel leaves mostly empty, so a cluster block is read once per
// tile.  Everything else (unshared blocks, small clusters, partial last blocks) becomes per-request items.  Every
// (item, request) pair owns one slot of partial softmax state; a last kernel merges a request's slots.
//
// Device side.  One kernel, templated on the number of rows it carries through P.V (ROWS = rep for per-request
// items, NREQ x rep for cluster items): same structure as the per-request decode kernel -- logits on the MFMA units
// from K fragments loaded straight from global memory, online softmax in fp32, P.V on the vector ALU -- except that
// the block list comes from the plan and the scale factors of a block are per row (they belong to the logical
// entry of the row's request).
#include "common.h"

#include <algorithm>
#include <map>
#include <new>
#include <vector>

namespace kvfuse {

typedef float floatx4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));

constexpr int kMaxTileReq = 4;        // requests per cluster tile (entries carry that many logical indices)
constexpr int kClusterChunk = 32;     // blocks per cluster work item, about

struct DItem {            // 64 bytes
    int32_t li, kvh, nreq, entry_off, entry_cnt, pad0, pad1, pad2;
    int32_t req[kMaxTileReq];
    int32_t slot[kMaxTileReq];
};
struct DEntry {           // 32 bytes
    int32_t phys, ntok;
    int32_t x[kMaxTileReq];   // logical entry of the block in each request of the tile (unused ones repeat x[0])
    int32_t pad0, pad1;
};
static_assert(sizeof(DItem) == 64 && sizeof(DEntry) == 32, "plan records are read as 16-byte vectors");

struct SharedArgs {
    const void *kpool, *vpool;
    const float *scale_k, *scale_v;
    const void *q;
    const DItem *items;
    const DEntry *entries;
    const int32_t *slot_begin;   // [tuples + 1]
    float *part;                 // [slots][rep_pad][D + 2] : o, then m, l
    float *out;                  // [n_layers][B][Hq][D]
    int32_t P, n, t, kv_heads, layer_begin, B, Hq, rep, rep_pad;
    float sm_scale;
};

template <typename T> struct SQkMma;
template <> struct SQkMma<bf16_t> {
    __device__ static __forceinline__ void run(const uint4 &a, const uint4 &b, floatx4 &c)
    {
        c = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, a), __builtin_bit_cast(bf16x8, b), c, 0, 0, 0);
    }
};
template <> struct SQkMma<float> {
    __device__ static __forceinline__ void run(const uint4 &a, const uint4 &b, floatx4 &c)
    {
        c = __builtin_amdgcn_mfma_f32_16x16x4f32(__uint_as_float(a.x), __uint_as_float(b.x), c, 0, 0, 0);
        c = __builtin_amdgcn_mfma_f32_16x16x4f32(__uint_as_float(a.y), __uint_as_float(b.y), c, 0, 0, 0);
        c = __builtin_amdgcn_mfma_f32_16x16x4f32(__uint_as_float(a.z), __uint_as_float(b.z), c, 0, 0, 0);
        c = __builtin_amdgcn_mfma_f32_16x16x4f32(__uint_as_float(a.w), __uint_as_float(b.w), c, 0, 0, 0);
    }
};

template <typename T> struct SToF32;
template <> struct SToF32<bf16_t> {
    __device__ static __forceinline__ void run(const uint4 &raw, float *o)
    {
        o[0] = __uint_as_float(raw.x << 16); o[1] = __uint_as_float(raw.x & 0xFFFF0000u);
        o[2] = __uint_as_float(raw.y << 16); o[3] = __uint_as_float(raw.y & 0xFFFF0000u);
        o[4] = __uint_as_float(raw.z << 16); o[5] = __uint_as_float(raw.z & 0xFFFF0000u);
        o[6] = __uint_as_float(raw.w << 16); o[7] = __uint_as_float(raw.w & 0xFFFF0000u);
    }
};
template <> struct SToF32<float> {
    __device__ static __forceinline__ void run(const uint4 &raw, float *o)
    {
        o[0] = __uint_as_float(raw.x); o[1] = __uint_as_float(raw.y);
        o[2] = __uint_as_float(raw.z); o[3] = __uint_as_float(raw.w);
    }
};

// One workgroup per plan item; its 4 wavefronts walk the item's blocks round-robin.  Row `head` (0..15) of the MFMA
// tile belongs to request slot head / rep_pad of the item and query head head % rep_pad of the KV head's group.
// With 16 rows two wavefronts share a block: both compute its logits and softmax state, each carries half of the
// rows through P.V (64 instead of 128 accumulators per lane, so that three workgroups fit a compute unit).
template <typename T, int D, int ROWS>
__global__ __launch_bounds__(256) void decode_items_kernel(SharedArgs A, int item_base)
{
    constexpr int RSPLIT = ROWS == 16 ? 2 : 1;     // wavefronts per block
    constexpr int NSTREAM = 4 / RSPLIT;            // blocks in flight per workgroup
    constexpr int RPW = ROWS / RSPLIT;             // rows a wavefront carries through P.V
    constexpr int PER = Elem<T>::PER16;
    constexpr int NF = D / (4 * PER);      // 16-byte K fragments per lane (a lane owns a quarter of a token row)
    constexpr int LPR = D / PER;           // lanes per V row
    constexpr int RPP = 64 / LPR;          // V rows per pass
    constexpr int NPASS = 16 / RPP;

    __shared__ __attribute__((aligned(16))) float p_lds[4][16][16];     // per wave: probability * scale_v, [token][row]
    __shared__ float c_lds[4][16];         // per wave: rescale factor per row
    __shared__ float w_m[4][16], w_l[4][16];
    __shared__ float w_o[4][RPW][D];

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int stream = wave / RSPLIT, row0 = (wave % RSPLIT) * RPW;
    const DItem item = A.items[item_base + blockIdx.x];
    const int li = item.li, kvh = item.kvh, nreq = item.nreq;
    const int g = (A.layer_begin + li) * A.kv_heads + kvh;
    const int64_t r = (int64_t)A.t * D;
    const T *kg = (const T *)A.kpool + (int64_t)g * A.P * r;
    const T *vg = (const T *)A.vpool + (int64_t)g * A.P * r;
    const float *skg = A.scale_k + (int64_t)g * A.n;
    const float *svg = A.scale_v + (int64_t)g * A.n;

    // logits roles: lane = (row, token group); K fragment roles: lane = (token, row quarter)
    const int head = lane & 15, tg = lane >> 4;
    const int ktok = lane & 15, kq = lane >> 4;
    // P.V roles: lane = (column slice, row within pass)
    const int dl = lane % LPR, tr = lane / LPR;
    // the request slot and query head of this lane's row; rows beyond the item's requests or the group's heads
    // carry a zero query and the scales of slot 0 (finite everywhere, never stored)
    const int rs_raw = head / A.rep_pad, hh = head - rs_raw * A.rep_pad;
    const bool row_used = rs_raw < nreq && hh < A.rep && head < ROWS;
    const int rs = row_used ? rs_raw : 0;
    const int my_req = rs == 0 ? item.req[0] : (rs == 1 ? item.req[1] : (rs == 2 ? item.req[2] : item.req[3]));

    uint4 qf[NF];
    {
        const T *qrow = (const T *)A.q + (((int64_t)li * A.B + my_req) * A.Hq + (int64_t)kvh * A.rep + (row_used ? hh : 0)) * D + kq * (D / 4);
#pragma unroll
        for (int f = 0; f < NF; ++f)
            qf[f] = row_used ? reinterpret_cast<const uint4 *>(qrow)[f] : make_uint4(0, 0, 0, 0);
    }

    float m_run = -INFINITY, l_run = 0.0f;
    float o[RPW][PER];
#pragma unroll
    for (int h = 0; h < RPW; ++h)
#pragma unroll
        for (int e = 0; e < PER; ++e)
            o[h][e] = 0.0f;

    for (int eb = stream; eb < item.entry_cnt; eb += NSTREAM) {
        const DEntry ent = A.entries[item.entry_off + eb];
        const int phys = ent.phys, ntok = ent.ntok;
        const int x = rs == 0 ? ent.x[0] : (rs == 1 ? ent.x[1] : (rs == 2 ? ent.x[2] : ent.x[3]));
        const float zs = A.sm_scale * skg[x];
        const float sv = svg[x];
        const T *kblk = kg + (int64_t)phys * r;
        const T *vblk = vg + (int64_t)phys * r;
        for (int sub = 0; sub < A.t; sub += 16) {
            if (sub >= ntok)
                break;
            // ---- logits: 16 tokens x 16 rows
            floatx4 z = {0.0f, 0.0f, 0.0f, 0.0f};
            const uint4 *krow = reinterpret_cast<const uint4 *>(kblk + (int64_t)(sub + ktok) * D + kq * (D / 4));
            uint4 kf[NF];
#pragma unroll
            for (int f = 0; f < NF; ++f)
                kf[f] = krow[f];
            uint4 vf[NPASS];
#pragma unroll
            for (int ps = 0; ps < NPASS; ++ps)
                vf[ps] = reinterpret_cast<const uint4 *>(vblk + (int64_t)(sub + ps * RPP + tr) * D)[dl];
#pragma unroll
            for (int f = 0; f < NF; ++f)
                SQkMma<T>::run(kf[f], qf[f], z);
            // ---- online softmax for this lane's row over its 4 tokens, then over the 4 token groups
            const int tok0 = sub + tg * 4;
            float zz[4];
            float bmax = -INFINITY;
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                zz[v] = (tok0 + v < ntok) ? z[v] * zs : -INFINITY;
                bmax = fmaxf(bmax, zz[v]);
            }
            bmax = fmaxf(bmax, __shfl_xor(bmax, 16, 64));
            bmax = fmaxf(bmax, __shfl_xor(bmax, 32, 64));
            const float m_new = fmaxf(m_run, bmax);
            const float corr = __expf(m_run - m_new);      // 0 on the first block (m_run = -inf)
            float psum = 0.0f;
            float pv[4];
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                const float pr = __expf(zz[v] - m_new);
                psum += pr;
                pv[v] = pr * sv;
            }
            psum += __shfl_xor(psum, 16, 64);
            psum += __shfl_xor(psum, 32, 64);
            l_run = l_run * corr + psum;
            m_run = m_new;
#pragma unroll
            for (int v = 0; v < 4; ++v)
                p_lds[wave][tg * 4 + v][head] = pv[v];
            if (tg == 0)
                c_lds[wave][head] = corr;
            __builtin_amdgcn_wave_barrier();
            // ---- P.V: this lane's column slice, rows tr, tr + RPP, ...
            float cf[RPW];
#pragma unroll
            for (int h = 0; h < RPW; ++h)
                cf[h] = c_lds[wave][row0 + h];
#pragma unroll
            for (int h = 0; h < RPW; ++h)
#pragma unroll
                for (int e = 0; e < PER; ++e)
                    o[h][e] *= cf[h];
#pragma unroll
            for (int ps = 0; ps < NPASS; ++ps) {
                float vv[PER];
                SToF32<T>::run(vf[ps], vv);
                const int tok = ps * RPP + tr;
                if (sub + tok >= ntok) {             // rows past the context may hold anything, even NaN
#pragma unroll
                    for (int e = 0; e < PER; ++e)
                        vv[e] = 0.0f;
                }
                if constexpr (RPW % 4 == 0) {        // four rows' probabilities per LDS read
#pragma unroll
                    for (int h4 = 0; h4 < RPW; h4 += 4) {
                        const float4 pw4 = *reinterpret_cast<const float4 *>(&p_lds[wave][tok][row0 + h4]);
                        const float pw[4] = {pw4.x, pw4.y, pw4.z, pw4.w};
#pragma unroll
                        for (int hq = 0; hq < 4; ++hq)
#pragma unroll
                            for (int e = 0; e < PER; ++e)
                                o[h4 + hq][e] = fmaf(pw[hq], vv[e], o[h4 + hq][e]);
                    }
                } else {
#pragma unroll
                    for (int h = 0; h < RPW; ++h) {
                        const float pw = p_lds[wave][tok][row0 + h];
#pragma unroll
                        for (int e = 0; e < PER; ++e)
                            o[h][e] = fmaf(pw, vv[e], o[h][e]);
                    }
                }
            }
            __builtin_amdgcn_wave_barrier();
        }
    }

    // ---- reduce o over the rows of a pass (lanes with the same column slice), publish the wave's state
#pragma unroll
    for (int off = LPR; off < 64; off <<= 1)
#pragma unroll
        for (int h = 0; h < RPW; ++h)
#pragma unroll
            for (int e = 0; e < PER; ++e)
                o[h][e] += __shfl_xor(o[h][e], off, 64);
    if (tr == 0) {
#pragma unroll
        for (int h = 0; h < RPW; ++h)
#pragma unroll
            for (int e = 0; e < PER; ++e)
                w_o[wave][h][dl * PER + e] = o[h][e];
    }
    if (tg == 0) {
        w_m[wave][head] = m_run;
        w_l[wave][head] = l_run;
    }
    __syncthreads();

    for (int idx = tid; idx < ROWS * D; idx += 256) {
        const int h = idx / D, e = idx - h * D;
        const int hs = h / A.rep_pad, hq = h - hs * A.rep_pad;
        if (hs >= nreq || hq >= A.rep)
            continue;
        // the wavefronts that carried row h: one per block stream
        const int wsel = h / RPW, hl = h - wsel * RPW;
        float M = -INFINITY;
#pragma unroll
        for (int st = 0; st < NSTREAM; ++st)
            M = fmaxf(M, w_m[st * RSPLIT + wsel][h]);
        float L = 0.0f, O = 0.0f;
#pragma unroll
        for (int st = 0; st < NSTREAM; ++st) {
            const int wv = st * RSPLIT + wsel;
            const float f = w_m[wv][h] == -INFINITY ? 0.0f : __expf(w_m[wv][h] - M);
            L += w_l[wv][h] * f;
            O += w_o[wv][hl][e] * f;
        }
        const int slot = hs == 0 ? item.slot[0] : (hs == 1 ? item.slot[1] : (hs == 2 ? item.slot[2] : item.slot[3]));
        float *pp = A.part + ((int64_t)slot * A.rep_pad + hq) * (D + 2);
        pp[e] = O;
        if (e == 0) {
            pp[D] = M;
            pp[D + 1] = L;
        }
    }
}

// bfloat16 pools: the same work item with P.V on the MFMA units as well.  The logits tile S[token][row] comes out of
// the first MFMA with each lane holding (row = lane % 16, tokens 4 * (lane / 16) .. + 3): exactly the A-operand
// layout of v_mfma_f32_16x16x16_bf16 for P[row][token].  V's layout ([token][d], d contiguous) is the wrong way
// round for the B operand (which wants 4 consecutive tokens of one column per lane), so every 16 x 16 piece of V
// first goes through one MFMA against the identity: its fp32 result (exact, the inputs are bfloat16) arrives with
// (tokens 4 * (lane / 16) .. + 3, column lane % 16) per lane, i.e. transposed into the B layout.  Probabilities are
// split into a bfloat16 head and a bfloat16 remainder (two MFMAs), which keeps them to 16 bits of mantissa.
// The 16 columns of a piece are those that the lanes' 16-byte loads deliver together, not 16 consecutive ones:
// piece (f, hs), slot n holds column 32 * (n / 4) + 8 * f + 4 * hs + n % 4 (for D = 128; D / 4 instead of 32 in
// general); the mapping is undone when the accumulators are written out.
typedef short short4v __attribute__((ext_vector_type(4)));

template <int D>
__global__ __launch_bounds__(256, 4) void decode_items_mfma_kernel(SharedArgs A, int item_base)
{
    typedef bf16_t T;
    constexpr int NF = D / 32;             // 16-byte fragments per lane (a lane owns a quarter of a token row)
    constexpr int NT = 2 * NF;             // 16-column accumulator tiles

    __shared__ __attribute__((aligned(16))) float c_lds[4][16];   // per wave: rescale factor per row
    __shared__ float w_m[4][16], w_l[4][16];
    __shared__ float w_o[4][16][D];

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const DItem item = A.items[item_base + blockIdx.x];
    const int li = item.li, kvh = item.kvh, nreq = item.nreq;
    const int g = (A.layer_begin + li) * A.kv_heads + kvh;
    const int64_t r = (int64_t)A.t * D;
    const T *kg = (const T *)A.kpool + (int64_t)g * A.P * r;
    const T *vg = (const T *)A.vpool + (int64_t)g * A.P * r;
    const float *skg = A.scale_k + (int64_t)g * A.n;
    const float *svg = A.scale_v + (int64_t)g * A.n;

    const int head = lane & 15, tg = lane >> 4;      // logits / P: row, token group;  K and V loads: token, row quarter
    const int rs_raw = head / A.rep_pad, hh = head - rs_raw * A.rep_pad;
    const bool row_used = rs_raw < nreq && hh < A.rep;
    const int rs = row_used ? rs_raw : 0;
    const int my_req = rs == 0 ? item.req[0] : (rs == 1 ? item.req[1] : (rs == 2 ? item.req[2] : item.req[3]));

    uint4 qf[NF];
    {
        const T *qrow = (const T *)A.q + (((int64_t)li * A.B + my_req) * A.Hq + (int64_t)kvh * A.rep + (row_used ? hh : 0)) * D + tg * (D / 4);
#pragma unroll
        for (int f = 0; f < NF; ++f)
            qf[f] = row_used ? reinterpret_cast<const uint4 *>(qrow)[f] : make_uint4(0, 0, 0, 0);
    }
    // identity as a B operand: this lane holds I[k = 4 * tg + i][n = head]
    short4v ident;
#pragma unroll
    for (int i = 0; i < 4; ++i)
        ident[i] = (4 * tg + i == head) ? (short)0x3F80 : (short)0;

    float m_run = -INFINITY, l_run = 0.0f;
    floatx4 o[NT];
#pragma unroll
    for (int nt = 0; nt < NT; ++nt)
        o[nt] = floatx4{0.0f, 0.0f, 0.0f, 0.0f};

    for (int eb = wave; eb < item.entry_cnt; eb += 4) {
        const DEntry ent = A.entries[item.entry_off + eb];
        const int phys = ent.phys, ntok = ent.ntok;
        const int x = rs == 0 ? ent.x[0] : (rs == 1 ? ent.x[1] : (rs == 2 ? ent.x[2] : ent.x[3]));
        const float zs = A.sm_scale * skg[x];
        const float sv = svg[x];
        const T *kblk = kg + (int64_t)phys * r;
        const T *vblk = vg + (int64_t)phys * r;
        for (int sub = 0; sub < A.t; sub += 16) {
            if (sub >= ntok)
                break;
            const uint4 *krow = reinterpret_cast<const uint4 *>(kblk + (int64_t)(sub + head) * D + tg * (D / 4));
            const uint4 *vrow = reinterpret_cast<const uint4 *>(vblk + (int64_t)(sub + head) * D + tg * (D / 4));
            uint4 kf[NF], vf[NF];
#pragma unroll
            for (int f = 0; f < NF; ++f)
                kf[f] = krow[f];
#pragma unroll
            for (int f = 0; f < NF; ++f)
                vf[f] = vrow[f];
            // ---- logits: 16 tokens x 16 rows
            floatx4 z = {0.0f, 0.0f, 0.0f, 0.0f};
#pragma unroll
            for (int f = 0; f < NF; ++f)
                z = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, kf[f]), __builtin_bit_cast(bf16x8, qf[f]), z, 0, 0, 0);
            // ---- online softmax for this lane's row over its 4 tokens, then over the 4 token groups
            const int tok0 = sub + tg * 4;
            float zz[4];
            float bmax = -INFINITY;
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                zz[v] = (tok0 + v < ntok) ? z[v] * zs : -INFINITY;
                bmax = fmaxf(bmax, zz[v]);
            }
            bmax = fmaxf(bmax, __shfl_xor(bmax, 16, 64));
            bmax = fmaxf(bmax, __shfl_xor(bmax, 32, 64));
            const float m_new = fmaxf(m_run, bmax);
            const float corr = __expf(m_run - m_new);      // 0 on the first block (m_run = -inf)
            float psum = 0.0f;
            short4v p_hi, p_lo;
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                const float pr = __expf(zz[v] - m_new);
                psum += pr;
                const float pw = pr * sv;
                const uint32_t hb = __float_as_uint(pw) & 0xFFFF0000u;           // bfloat16 head (truncated)
                const float rest = pw - __uint_as_float(hb);                      // exact
                p_hi[v] = (short)(hb >> 16);
                p_lo[v] = (short)((__float_as_uint(rest) + 0x8000u) >> 16);       // bfloat16 remainder (rounded)
            }
            psum += __shfl_xor(psum, 16, 64);
            psum += __shfl_xor(psum, 32, 64);
            l_run = l_run * corr + psum;
            m_run = m_new;
            if (tg == 0)
                c_lds[wave][head] = corr;
            __builtin_amdgcn_wave_barrier();
            // ---- rescale the accumulators: this lane holds rows 4 * tg .. + 3 of every tile
            const float4 c4 = *reinterpret_cast<const float4 *>(&c_lds[wave][4 * tg]);
#pragma unroll
            for (int nt = 0; nt < NT; ++nt) {
                o[nt][0] *= c4.x; o[nt][1] *= c4.y; o[nt][2] *= c4.z; o[nt][3] *= c4.w;
            }
            // ---- P.V.  V rows past the context may hold anything, even NaN: this lane's row is token `head`
            if (sub + head >= ntok) {
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
        }
    }

    // ---- publish the wave's state: this lane holds o[row 4 * tg + i][column slot head] of every tile
#pragma unroll
    for (int f = 0; f < NF; ++f)
#pragma unroll
        for (int hs = 0; hs < 2; ++hs) {
            const int col = (D / 4) * (head >> 2) + 8 * f + 4 * hs + (head & 3);
#pragma unroll
            for (int i = 0; i < 4; ++i)
                w_o[wave][4 * tg + i][col] = o[2 * f + hs][i];
        }
    if (tg == 0) {
        w_m[wave][head] = m_run;
        w_l[wave][head] = l_run;
    }
    __syncthreads();

    for (int idx = tid; idx < 16 * D; idx += 256) {
        const int h = idx / D, e = idx - h * D;
        const int hs = h / A.rep_pad, hq = h - hs * A.rep_pad;
        if (hs >= nreq || hq >= A.rep)
            continue;
        float M = fmaxf(fmaxf(w_m[0][h], w_m[1][h]), fmaxf(w_m[2][h], w_m[3][h]));
        float L = 0.0f, O = 0.0f;
#pragma unroll
        for (int wv = 0; wv < 4; ++wv) {
            const float f = w_m[wv][h] == -INFINITY ? 0.0f : __expf(w_m[wv][h] - M);
            L += w_l[wv][h] * f;
            O += w_o[wv][h][e] * f;
        }
        const int slot = hs == 0 ? item.slot[0] : (hs == 1 ? item.slot[1] : (hs == 2 ? item.slot[2] : item.slot[3]));
        float *pp = A.part + ((int64_t)slot * A.rep_pad + hq) * (D + 2);
        pp[e] = O;
        if (e == 0) {
            pp[D] = M;
            pp[D + 1] = L;
        }
    }
}

// Merge of a request's partial states: one workgroup per (layer, request, KV head).
template <int D>
__global__ __launch_bounds__(256) void decode_shared_combine_kernel(SharedArgs A)
{
    const int64_t tuple = blockIdx.x;
    const int kvh = (int)(tuple % A.kv_heads);
    const int64_t lb = tuple / A.kv_heads;       // li * B + b
    const int s0 = A.slot_begin[tuple], s1 = A.slot_begin[tuple + 1];
    for (int idx = threadIdx.x; idx < A.rep * D; idx += 256) {
        const int h = idx / D, e = idx - h * D;
        float M = -INFINITY;
        for (int s = s0; s < s1; ++s)
            M = fmaxf(M, A.part[((int64_t)s * A.rep_pad + h) * (D + 2) + D]);
        float L = 0.0f, O = 0.0f;
        for (int s = s0; s < s1; ++s) {
            const float *pp = A.part + ((int64_t)s * A.rep_pad + h) * (D + 2);
            const float f = pp[D] == -INFINITY ? 0.0f : __expf(pp[D] - M);
            L += pp[D + 1] * f;
            O += pp[e] * f;
        }
        A.out[(lb * A.Hq + (int64_t)kvh * A.rep + h) * D + e] = L > 0.0f ? O / L : 0.0f;
    }
}

static int pad_pow2(int rep)
{
    int p = 1;
    while (p < rep)
        p <<= 1;
    return p;
}

template <typename T, int D>
static void launch_items(hipStream_t s, const SharedArgs &A, int rows, int item_base, int n_items)
{
    if (n_items <= 0)
        return;
    switch (rows) {
    case 1: decode_items_kernel<T, D, 1><<<n_items, 256, 0, s>>>(A, item_base); break;
    case 2: decode_items_kernel<T, D, 2><<<n_items, 256, 0, s>>>(A, item_base); break;
    case 4: decode_items_kernel<T, D, 4><<<n_items, 256, 0, s>>>(A, item_base); break;
    case 8: decode_items_kernel<T, D, 8><<<n_items, 256, 0, s>>>(A, item_base); break;
    default: decode_items_kernel<T, D, 16><<<n_items, 256, 0, s>>>(A, item_base); break;
    }
}

}  // namespace kvfuse

using namespace kvfuse;

struct kvfuse_decode_plan {
    // parameters the plan was built for
    int32_t dtype = 0, P = 0, n = 0, t = 0, d = 0, G = 0;
    int32_t kv_heads = 0, layer_begin = 0, n_layers = 0, B = 0, Hq = 0, rep = 0, rep_pad = 0, nreq_max = 1;
    // host tables
    std::vector<DItem> items_cluster, items_residual;
    std::vector<DEntry> entries;
    std::vector<int32_t> slot_begin;
    int64_t total_slots = 0;
    kvfuse_decode_plan_info info = {};
    // device placement
    size_t off_items = 0, off_entries = 0, off_slots = 0, off_part = 0, bytes = 0;
    char *dev = nullptr;
};

static size_t up256(size_t x) { return (x + 255) & ~(size_t)255; }

namespace {

struct Inst {
    int32_t p, b, x;
};

int residual_splits(int64_t tuples, int blocks)
{
    int64_t ns = tuples > 0 ? (2048 + tuples - 1) / tuples : 1;
    const int cap = (blocks + 7) / 8;
    if (ns > cap)
        ns = cap;
    if (ns > 64)
        ns = 64;
    if (ns < 1)
        ns = 1;
    return (int)ns;
}

}  // namespace

extern "C" {

int kvfuse_shared_decode_plan_build(kvfuse_ctx *ctx, const kvfuse_pool *pool, const kvfuse_table *table, int32_t kv_heads,
                                    int32_t layer_begin, int32_t n_layers, const int32_t *req_start, const int32_t *ctx_len,
                                    int32_t B, int32_t Hq, int32_t min_cluster_blocks, kvfuse_decode_plan **plan,
                                    kvfuse_decode_plan_info *info)
{
    if (!ctx)
        return KVFUSE_EINVAL;
    Ctx *c = &ctx->c;
    if (!plan)
        return fail(c, KVFUSE_EINVAL, "decode plan: null output");
    *plan = nullptr;
    if (!pool || !table || !table->bt || !req_start || !ctx_len)
        return fail(c, KVFUSE_EINVAL, "decode plan: null pointer");
    if (kv_heads <= 0 || Hq <= 0 || Hq % kv_heads != 0 || Hq / kv_heads > 16 || B < 0 || n_layers < 0 || layer_begin < 0 ||
        (int64_t)(layer_begin + n_layers) * kv_heads > pool->G || min_cluster_blocks < 1)
        return fail(c, KVFUSE_EINVAL, "decode plan: head counts, layer range or min_cluster_blocks out of range");
    if (pool->dtype != KVFUSE_BF16 && pool->dtype != KVFUSE_F32)
        return fail(c, KVFUSE_ESHAPE, "decode plan: dtype must be KVFUSE_BF16 or KVFUSE_F32");
    if ((pool->d != 64 && pool->d != 128) || pool->t % 16 != 0 || pool->t <= 0)
        return fail(c, KVFUSE_ESHAPE, "decode plan: needs d in {64, 128} and t a multiple of 16");
    const int n = table->n, t = pool->t;
    int max_blocks = 0;
    for (int b = 0; b < B; ++b) {
        if (ctx_len[b] < 0 || req_start[b] < 0)
            return fail(c, KVFUSE_EINVAL, "decode plan: negative request start or context length");
        const int nb = (ctx_len[b] + t - 1) / t;
        if ((int64_t)req_start[b] + nb > n)
            return fail(c, KVFUSE_EINVAL, "decode plan: a request's blocks run past the table");
        max_blocks = std::max(max_blocks, nb);
    }
    kvfuse_decode_plan *pl = new (std::nothrow) kvfuse_decode_plan();
    if (!pl)
        return fail(c, KVFUSE_ENOMEM, "decode plan: out of host memory");
    pl->dtype = pool->dtype; pl->P = pool->P; pl->n = n; pl->t = t; pl->d = pool->d; pl->G = pool->G;
    pl->kv_heads = kv_heads; pl->layer_begin = layer_begin; pl->n_layers = n_layers; pl->B = B; pl->Hq = Hq;
    pl->rep = Hq / kv_heads;
    pl->rep_pad = pad_pow2(pl->rep);
    pl->nreq_max = std::max(1, std::min(kMaxTileReq, 16 / pl->rep_pad));

    const int Gsel = n_layers * kv_heads;
    const int64_t tuples = (int64_t)n_layers * B * kv_heads;
    std::vector<int32_t> bt((size_t)Gsel * n);
    if (!bt.empty()) {
        hipError_t e = hipStreamSynchronize(c->stream);
        if (e == hipSuccess)
            e = hipMemcpy(bt.data(), table->bt + (int64_t)layer_begin * kv_heads * n, bt.size() * sizeof(int32_t),
                          hipMemcpyDeviceToHost);
        if (e != hipSuccess) {
            delete pl;
            return fail(c, KVFUSE_EHIP, std::string("decode plan: reading the table: ") + hipGetErrorString(e));
        }
    }
    std::vector<int32_t> slot_count((size_t)tuples, 0);
    std::vector<Inst> inst;
    std::vector<uint8_t> covered((size_t)n);
    const int nsplit_res = residual_splits(tuples, max_blocks);
    kvfuse_decode_plan_info &I = pl->info;

    auto take_slot = [&](DItem &it, int rs, int li, int b, int kvh) {
        const int64_t tuple = ((int64_t)li * B + b) * kv_heads + kvh;
        it.slot[rs] = slot_count[(size_t)tuple]++;      // local index for now; made absolute below
    };

    for (int gi = 0; gi < Gsel; ++gi) {
        const int li = gi / kv_heads, kvh = gi % kv_heads;
        const int32_t *btg = bt.data() + (size_t)gi * n;
        inst.clear();
        std::fill(covered.begin(), covered.end(), 0);
        for (int b = 0; b < B; ++b) {
            const int nb = (ctx_len[b] + t - 1) / t;
            for (int j = 0; j < nb; ++j) {
                const int x = req_start[b] + j;
                const int p = btg[x];
                if (p < 0 || p >= pool->P) {
                    delete pl;
                    return fail(c, KVFUSE_EINVAL, "decode plan: the table holds a physical id outside the pool");
                }
                ++I.logical_blocks;
                if ((int64_t)(j + 1) * t <= ctx_len[b])
                    inst.push_back(Inst{p, b, x});
            }
        }
        std::sort(inst.begin(), inst.end(), [](const Inst &a, const Inst &b2) {
            return a.p != b2.p ? a.p < b2.p : (a.b != b2.b ? a.b < b2.b : a.x < b2.x);
        });
        // physical blocks used by >= 2 requests, each once, keyed by the set of requests
        std::map<std::vector<int32_t>, std::vector<int32_t>> by_set;    // request set -> starts of runs in inst
        std::vector<int32_t> key;
        for (size_t s = 0; s < inst.size();) {
            size_t e = s + 1;
            while (e < inst.size() && inst[e].p == inst[s].p)
                ++e;
            if (e - s >= 2) {
                bool distinct = true;
                for (size_t k = s + 1; k < e; ++k)
                    distinct = distinct && inst[k].b != inst[k - 1].b;
                if (distinct) {
                    key.clear();
                    for (size_t k = s; k < e; ++k)
                        key.push_back(inst[k].b);
                    by_set[key].push_back((int32_t)s);
                }
            }
            s = e;
        }
        for (const auto &kv : by_set) {
            const std::vector<int32_t> &reqs = kv.first;
            const std::vector<int32_t> &runs = kv.second;
            const int nb = (int)runs.size(), k = (int)reqs.size();
            if (nb < min_cluster_blocks)
                continue;
            ++I.clusters;
            I.shared_instances += (int64_t)nb * k;
            const int nchunk = std::max(1, (nb + kClusterChunk / 2) / kClusterChunk);
            for (int s0 = 0; s0 < k; s0 += pl->nreq_max) {
                const int nr = std::min(pl->nreq_max, k - s0);
                for (int ch = 0; ch < nchunk; ++ch) {
                    const int lo = (int)((int64_t)nb * ch / nchunk), hi = (int)((int64_t)nb * (ch + 1) / nchunk);
                    if (hi <= lo)
                        continue;
                    DItem it = {};
                    it.li = li; it.kvh = kvh; it.nreq = nr;
                    it.entry_off = (int32_t)pl->entries.size();
                    it.entry_cnt = hi - lo;
                    for (int rs = 0; rs < kMaxTileReq; ++rs)
                        it.req[rs] = reqs[(size_t)(s0 + std::min(rs, nr - 1))];
                    for (int rs = 0; rs < nr; ++rs)
                        take_slot(it, rs, li, reqs[(size_t)(s0 + rs)], kvh);
                    for (int q = lo; q < hi; ++q) {
                        DEntry en = {};
                        const int32_t run = runs[(size_t)q];
                        en.phys = inst[(size_t)run].p;
                        en.ntok = t;
                        for (int rs = 0; rs < kMaxTileReq; ++rs)
                            en.x[rs] = inst[(size_t)(run + s0 + std::min(rs, nr - 1))].x;
                        pl->entries.push_back(en);
                    }
                    I.cluster_block_reads += hi - lo;
                    pl->items_cluster.push_back(it);
                }
            }
            for (int32_t run : runs)
                for (int q = 0; q < k; ++q)
                    covered[(size_t)inst[(size_t)(run + q)].x] = 1;
        }
        // what is left of every request
        for (int b = 0; b < B; ++b) {
            const int nb = (ctx_len[b] + t - 1) / t;
            int nres = 0;
            for (int j = 0; j < nb; ++j)
                nres += covered[(size_t)(req_start[b] + j)] ? 0 : 1;
            if (nres == 0)
                continue;
            const int nsp = std::min(nsplit_res, nres);
            int j = 0;
            for (int sp = 0; sp < nsp; ++sp) {
                const int want = (int)((int64_t)nres * (sp + 1) / nsp) - (int)((int64_t)nres * sp / nsp);
                DItem it = {};
                it.li = li; it.kvh = kvh; it.nreq = 1;
                it.entry_off = (int32_t)pl->entries.size();
                for (int rs = 0; rs < kMaxTileReq; ++rs)
                    it.req[rs] = b;
                take_slot(it, 0, li, b, kvh);
                int got = 0;
                while (got < want && j < nb) {
                    const int x = req_start[b] + j;
                    if (!covered[(size_t)x]) {
                        DEntry en = {};
                        en.phys = btg[x];
                        en.ntok = std::min(t, ctx_len[b] - j * t);
                        for (int rs = 0; rs < kMaxTileReq; ++rs)
                            en.x[rs] = x;
                        pl->entries.push_back(en);
                        ++got;
                    }
                    ++j;
                }
                it.entry_cnt = got;
                I.residual_block_reads += got;
                pl->items_residual.push_back(it);
            }
        }
        if (pl->entries.size() > (size_t)0x7FFFFFF0) {
            delete pl;
            return fail(c, KVFUSE_ESHAPE, "decode plan: more than 2^31 block entries; plan fewer layers per call");
        }
    }
    // absolute slot numbers: a tuple's slots are consecutive
    pl->slot_begin.assign((size_t)tuples + 1, 0);
    for (int64_t tp = 0; tp < tuples; ++tp)
        pl->slot_begin[(size_t)tp + 1] = pl->slot_begin[(size_t)tp] + slot_count[(size_t)tp];
    pl->total_slots = tuples > 0 ? pl->slot_begin[(size_t)tuples] : 0;
    auto make_absolute = [&](std::vector<DItem> &v) {
        for (DItem &it : v)
            for (int rs = 0; rs < it.nreq; ++rs) {
                const int64_t tuple = ((int64_t)it.li * B + it.req[rs]) * kv_heads + it.kvh;
                it.slot[rs] += pl->slot_begin[(size_t)tuple];
            }
    };
    make_absolute(pl->items_cluster);
    make_absolute(pl->items_residual);
    I.items_cluster = (int64_t)pl->items_cluster.size();
    I.items_residual = (int64_t)pl->items_residual.size();
    // device layout
    size_t off = 0;
    pl->off_items = off;
    off = up256(off + (pl->items_cluster.size() + pl->items_residual.size()) * sizeof(DItem));
    pl->off_entries = off;
    off = up256(off + pl->entries.size() * sizeof(DEntry));
    pl->off_slots = off;
    off = up256(off + pl->slot_begin.size() * sizeof(int32_t));
    pl->off_part = off;
    off = up256(off + (size_t)pl->total_slots * pl->rep_pad * (pl->d + 2) * sizeof(float));
    pl->bytes = off + 256;
    I.device_bytes = (int64_t)pl->bytes;
    if (info)
        *info = I;
    *plan = pl;
    return KVFUSE_OK;
}

int kvfuse_shared_decode_plan_upload(kvfuse_ctx *ctx, kvfuse_decode_plan *plan, void *workspace, size_t workspace_bytes)
{
    if (!ctx)
        return KVFUSE_EINVAL;
    Ctx *c = &ctx->c;
    if (!plan || !workspace)
        return fail(c, KVFUSE_EINVAL, "decode plan upload: null pointer");
    if (workspace_bytes < plan->bytes)
        return fail(c, KVFUSE_ENOMEM, "decode plan upload: workspace smaller than info.device_bytes");
    if ((reinterpret_cast<uintptr_t>(workspace) & 255) != 0)
        return fail(c, KVFUSE_EINVAL, "decode plan upload: workspace must be 256-byte aligned");
    char *dev = static_cast<char *>(workspace);
    const size_t nc = plan->items_cluster.size(), nr = plan->items_residual.size();
    if (nc)
        KVF_HIP(c, hipMemcpyAsync(dev + plan->off_items, plan->items_cluster.data(), nc * sizeof(DItem), hipMemcpyHostToDevice, c->stream));
    if (nr)
        KVF_HIP(c, hipMemcpyAsync(dev + plan->off_items + nc * sizeof(DItem), plan->items_residual.data(), nr * sizeof(DItem),
                                  hipMemcpyHostToDevice, c->stream));
    if (!plan->entries.empty())
        KVF_HIP(c, hipMemcpyAsync(dev + plan->off_entries, plan->entries.data(), plan->entries.size() * sizeof(DEntry),
                                  hipMemcpyHostToDevice, c->stream));
    KVF_HIP(c, hipMemcpyAsync(dev + plan->off_slots, plan->slot_begin.data(), plan->slot_begin.size() * sizeof(int32_t),
                              hipMemcpyHostToDevice, c->stream));
    KVF_HIP(c, hipStreamSynchronize(c->stream));      // the host vectors may go away after this call
    plan->dev = dev;
    return KVFUSE_OK;
}

int kvfuse_shared_decode_plan_destroy(kvfuse_decode_plan *plan)
{
    delete plan;
    return KVFUSE_OK;
}

int kvfuse_paged_decode_attn_shared(kvfuse_ctx *ctx, const kvfuse_pool *pool, const kvfuse_table *table,
                                    const kvfuse_decode_plan *plan, const void *q, float sm_scale, float *out)
{
    if (!ctx)
        return KVFUSE_EINVAL;
    Ctx *c = &ctx->c;
    if (!pool || !pool->k || !pool->v || !table || !table->scale_k || !table->scale_v || !plan || !q || !out)
        return fail(c, KVFUSE_EINVAL, "shared decode: null pointer");
    if (!plan->dev)
        return fail(c, KVFUSE_EINVAL, "shared decode: the plan has not been uploaded");
    if (pool->dtype != plan->dtype || pool->P != plan->P || pool->t != plan->t || pool->d != plan->d || pool->G != plan->G ||
        table->n != plan->n)
        return fail(c, KVFUSE_EINVAL, "shared decode: pool or table shape differs from the one the plan was built for");
    const int64_t tuples = (int64_t)plan->n_layers * plan->B * plan->kv_heads;
    if (tuples == 0)
        return KVFUSE_OK;
    if (tuples > 0x7FFFFFFF)
        return fail(c, KVFUSE_ESHAPE, "shared decode: too many (layer, request, head) tuples for one call");
    SharedArgs A;
    A.kpool = pool->k; A.vpool = pool->v; A.scale_k = table->scale_k; A.scale_v = table->scale_v; A.q = q;
    A.items = reinterpret_cast<const DItem *>(plan->dev + plan->off_items);
    A.entries = reinterpret_cast<const DEntry *>(plan->dev + plan->off_entries);
    A.slot_begin = reinterpret_cast<const int32_t *>(plan->dev + plan->off_slots);
    A.part = reinterpret_cast<float *>(plan->dev + plan->off_part);
    A.out = out;
    A.P = pool->P; A.n = table->n; A.t = pool->t; A.kv_heads = plan->kv_heads; A.layer_begin = plan->layer_begin;
    A.B = plan->B; A.Hq = plan->Hq; A.rep = plan->rep; A.rep_pad = plan->rep_pad;
    A.sm_scale = sm_scale;
    const int nc = (int)plan->items_cluster.size(), nr = (int)plan->items_residual.size();
    const int rows_cluster = plan->nreq_max * plan->rep_pad, rows_residual = plan->rep_pad;
    // The cluster pass is bound by the vector ALU, the per-request pass by HBM: they run side by side, the cluster
    // pass on the context's second stream, and meet again before the merge.
    const bool fork = nc > 0 && nr > 0;
    if (fork) {
        if (!c->aux) {
            hipStream_t st = nullptr;
            hipEvent_t e0 = nullptr, e1 = nullptr;
            KVF_HIP(c, hipSetDevice(c->device));
            KVF_HIP(c, hipStreamCreateWithFlags(&st, hipStreamNonBlocking));
            hipError_t er = hipEventCreateWithFlags(&e0, hipEventDisableTiming);
            if (er == hipSuccess)
                er = hipEventCreateWithFlags(&e1, hipEventDisableTiming);
            if (er != hipSuccess) {
                if (e0)
                    (void)hipEventDestroy(e0);
                (void)hipStreamDestroy(st);
                KVF_HIP(c, er);
            }
            c->aux = st; c->fork = e0; c->join = e1;
        }
        KVF_HIP(c, hipEventRecord(c->fork, c->stream));
        KVF_HIP(c, hipStreamWaitEvent(c->aux, c->fork, 0));
    }
    hipStream_t cs = fork ? c->aux : c->stream;
#define KVF_SHARED_LAUNCH(T, D)                                                        \
    do {                                                                               \
        launch_items<T, D>(cs, A, rows_cluster, 0, nc);                                \
        launch_items<T, D>(c->stream, A, rows_residual, nc, nr);                       \
        if (fork) {                                                                    \
            (void)hipEventRecord(c->join, c->aux);                                     \
            (void)hipStreamWaitEvent(c->stream, c->join, 0);                           \
        }                                                                              \
        decode_shared_combine_kernel<D><<<(unsigned)tuples, 256, 0, c->stream>>>(A);   \
    } while (0)
    if (pool->dtype == KVFUSE_BF16) {
#define KVF_SHARED_LAUNCH_MFMA(D)                                                                   \
    do {                                                                                            \
        if (nc > 0)                                                                                 \
            decode_items_mfma_kernel<D><<<nc, 256, 0, cs>>>(A, 0);                                  \
        if (nr > 0)                                                                                 \
            decode_items_mfma_kernel<D><<<nr, 256, 0, c->stream>>>(A, nc);                          \
        if (fork) {                                                                                 \
            (void)hipEventRecord(c->join, c->aux);                                                  \
            (void)hipStreamWaitEvent(c->stream, c->join, 0);                                        \
        }                                                                                           \
        decode_shared_combine_kernel<D><<<(unsigned)tuples, 256, 0, c->stream>>>(A);                \
    } while (0)
        if (pool->d == 128) KVF_SHARED_LAUNCH_MFMA(128);
        else KVF_SHARED_LAUNCH_MFMA(64);
#undef KVF_SHARED_LAUNCH_MFMA
    } else {
        if (pool->d == 128) KVF_SHARED_LAUNCH(float, 128);
        else KVF_SHARED_LAUNCH(float, 64);
    }
#undef KVF_SHARED_LAUNCH
    KVF_HIP(c, hipGetLastError());
    return KVFUSE_OK;
}

}  // extern "C"
