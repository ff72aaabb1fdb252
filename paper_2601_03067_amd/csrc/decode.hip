// a7: paged decode attention through the fused block table (motivation section: after encoding, several logical
// blocks share one stored representation that the block table points at; method section: one unit vector plus a
// norm per logical block; analysis section: logits z_t = q . k_t / sqrt(d)).
//
// Logical block x of group g is scale_k[x] * K[bt[x]] / scale_v[x] * V[bt[x]].  Bandwidth-bound: every K and V byte
// of the context is read once.  One workgroup per (layer, request, KV head, split); its 4 wavefronts walk the
// blocks of the split round-robin.  All query heads of the KV head (GQA group, up to 16) are processed together:
//   logits  16 tokens x 16 heads per MFMA group (v_mfma_f32_16x16x32_bf16, or 16x16x4_f32 for f32 pools), K
//           fragments loaded straight from global memory (each lane owns a quarter of a token row),
//   softmax online, fp32, per head (state replicated over the 4 lanes that hold a head's 16 tokens),
//   P.V     on the vector ALU with lanes owning 16-byte column slices of V rows (V's layout would need a transpose
//           to feed the MFMA k-dimension); probabilities pass through a per-wave LDS tile.
// Partial states of the 4 wavefronts are merged in LDS; with several splits a second kernel merges the splits.
#include <mutex>

#include "common.h"

namespace kvfuse {

typedef float floatx4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));

template <typename T> struct QkMma;
template <> struct QkMma<bf16_t> {
    __device__ static __forceinline__ void run(const uint4 &a, const uint4 &b, floatx4 &c)
    {
        c = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, a), __builtin_bit_cast(bf16x8, b), c, 0, 0, 0);
    }
};
template <> struct QkMma<float> {
    __device__ static __forceinline__ void run(const uint4 &a, const uint4 &b, floatx4 &c)
    {
        c = __builtin_amdgcn_mfma_f32_16x16x4f32(__uint_as_float(a.x), __uint_as_float(b.x), c, 0, 0, 0);
        c = __builtin_amdgcn_mfma_f32_16x16x4f32(__uint_as_float(a.y), __uint_as_float(b.y), c, 0, 0, 0);
        c = __builtin_amdgcn_mfma_f32_16x16x4f32(__uint_as_float(a.z), __uint_as_float(b.z), c, 0, 0, 0);
        c = __builtin_amdgcn_mfma_f32_16x16x4f32(__uint_as_float(a.w), __uint_as_float(b.w), c, 0, 0, 0);
    }
};

template <typename T> struct ToF32;
template <> struct ToF32<bf16_t> {
    __device__ static __forceinline__ void run(const uint4 &raw, float *o)
    {
        o[0] = __uint_as_float(raw.x << 16); o[1] = __uint_as_float(raw.x & 0xFFFF0000u);
        o[2] = __uint_as_float(raw.y << 16); o[3] = __uint_as_float(raw.y & 0xFFFF0000u);
        o[4] = __uint_as_float(raw.z << 16); o[5] = __uint_as_float(raw.z & 0xFFFF0000u);
        o[6] = __uint_as_float(raw.w << 16); o[7] = __uint_as_float(raw.w & 0xFFFF0000u);
    }
};
template <> struct ToF32<float> {
    __device__ static __forceinline__ void run(const uint4 &raw, float *o)
    {
        o[0] = __uint_as_float(raw.x); o[1] = __uint_as_float(raw.y);
        o[2] = __uint_as_float(raw.z); o[3] = __uint_as_float(raw.w);
    }
};

struct DecodeArgs {
    const void *kpool, *vpool;
    const int32_t *bt;
    const float *scale_k, *scale_v;
    const void *q;
    const int32_t *req_start, *ctx_len;
    float *part;   // [tuples][nsplit][REP][D + 2] : o, then m, l
    float *out;    // [n_layers][B][Hq][D]
    int32_t P, n, t, kv_heads, layer_begin, B, Hq, rep, nsplit, blocks_per_split;
    int32_t gstride;   // groups between consecutive layers of the pool and the table: kv_heads, or 1 with all-head blocks
    float sm_scale;
};

// AH = all-head blocks (method section: one vector per block over all KV heads, one table per layer): the pool is
// [layers][P][t][kv_heads][D], so the tokens of a block lie kv_heads * D elements apart, the KV head selects a
// D-element slice of each token row, and all KV heads of a layer share one block table and one scale per entry.
template <typename T, int D, int REP, bool AH>
__global__ __launch_bounds__(256) void decode_kernel(DecodeArgs A)
{
    constexpr int PER = Elem<T>::PER16;
    constexpr int NF = D / (4 * PER);      // 16-byte K fragments per lane (a lane owns a quarter of a token row)
    constexpr int LPR = D / PER;           // lanes per V row
    constexpr int RPP = 64 / LPR;          // V rows per pass
    constexpr int NPASS = 16 / RPP;

    __shared__ float p_lds[4][16][16];     // per wave: probability * scale_v, [token][head]
    __shared__ float c_lds[4][16];         // per wave: rescale factor per head
    __shared__ float w_m[4][16], w_l[4][16];
    __shared__ float w_o[4][REP][D];

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int split = blockIdx.x;
    const int b = blockIdx.y / A.kv_heads;
    const int kvh = blockIdx.y - b * A.kv_heads;
    const int li = blockIdx.z;
    const int g = AH ? A.layer_begin + li : (A.layer_begin + li) * A.kv_heads + kvh;
    const int64_t row = AH ? (int64_t)A.kv_heads * D : (int64_t)D;      // elements from one token of a block to the next
    const int ctx = A.ctx_len[b];
    const int nb = (ctx + A.t - 1) / A.t;
    const int blk_lo = split * A.blocks_per_split;
    const int blk_hi = min(nb, blk_lo + A.blocks_per_split);
    const int x0 = A.req_start[b];
    const int64_t r = (int64_t)A.t * row;
    const T *kg = (const T *)A.kpool + (int64_t)g * A.P * r + (AH ? kvh * D : 0);
    const T *vg = (const T *)A.vpool + (int64_t)g * A.P * r + (AH ? kvh * D : 0);
    const int32_t *btg = A.bt + (int64_t)g * A.n;
    const float *skg = A.scale_k + (int64_t)g * A.n;
    const float *svg = A.scale_v + (int64_t)g * A.n;

    // logits roles: lane = (head, token group); K fragment roles: lane = (token, row quarter)
    const int head = lane & 15, tg = lane >> 4;
    const int ktok = lane & 15, kq = lane >> 4;
    // P.V roles: lane = (column slice, row within pass)
    const int dl = lane % LPR, tr = lane / LPR;

    uint4 qf[NF];
    {
        const T *qrow = (const T *)A.q + (((int64_t)li * A.B + b) * A.Hq + (int64_t)kvh * A.rep + head) * D + kq * (D / 4);
#pragma unroll
        for (int f = 0; f < NF; ++f)
            qf[f] = head < A.rep ? reinterpret_cast<const uint4 *>(qrow)[f] : make_uint4(0, 0, 0, 0);
    }

    float m_run = -INFINITY, l_run = 0.0f;
    float o[REP][PER];
#pragma unroll
    for (int h = 0; h < REP; ++h)
#pragma unroll
        for (int e = 0; e < PER; ++e)
            o[h][e] = 0.0f;

    for (int xb = blk_lo + wave; xb < blk_hi; xb += 4) {
        const int x = x0 + xb;
        const int phys = btg[x];
        const float zs = A.sm_scale * skg[x];
        const float sv = svg[x];
        const T *kblk = kg + (int64_t)phys * r;
        const T *vblk = vg + (int64_t)phys * r;
        for (int sub = 0; sub < A.t; sub += 16) {
            // ---- logits: 16 tokens x 16 heads
            floatx4 z = {0.0f, 0.0f, 0.0f, 0.0f};
            const uint4 *krow = reinterpret_cast<const uint4 *>(kblk + (int64_t)(sub + ktok) * row + kq * (D / 4));
            uint4 kf[NF];
#pragma unroll
            for (int f = 0; f < NF; ++f)
                kf[f] = krow[f];
            // V rows of this sub-block, issued early so that they overlap the softmax
            uint4 vf[NPASS];
#pragma unroll
            for (int ps = 0; ps < NPASS; ++ps)
                vf[ps] = reinterpret_cast<const uint4 *>(vblk + (int64_t)(sub + ps * RPP + tr) * row)[dl];
#pragma unroll
            for (int f = 0; f < NF; ++f)
                QkMma<T>::run(kf[f], qf[f], z);
            // ---- online softmax for this lane's head over its 4 tokens, then over the 4 token groups
            const int tok0 = xb * A.t + sub + tg * 4;
            float zz[4];
            float bmax = -INFINITY;
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                zz[v] = (tok0 + v < ctx) ? z[v] * zs : -INFINITY;
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
            float cf[REP];
#pragma unroll
            for (int h = 0; h < REP; ++h)
                cf[h] = c_lds[wave][h];
#pragma unroll
            for (int h = 0; h < REP; ++h)
#pragma unroll
                for (int e = 0; e < PER; ++e)
                    o[h][e] *= cf[h];
#pragma unroll
            for (int ps = 0; ps < NPASS; ++ps) {
                float vv[PER];
                ToF32<T>::run(vf[ps], vv);
                const int tok = ps * RPP + tr;
                if (xb * A.t + sub + tok >= ctx) {   // rows past the context may hold anything, even NaN
#pragma unroll
                    for (int e = 0; e < PER; ++e)
                        vv[e] = 0.0f;
                }
#pragma unroll
                for (int h = 0; h < REP; ++h) {
                    const float pw = p_lds[wave][tok][h];
#pragma unroll
                    for (int e = 0; e < PER; ++e)
                        o[h][e] = fmaf(pw, vv[e], o[h][e]);
                }
            }
            __builtin_amdgcn_wave_barrier();
        }
    }

    // ---- reduce o over the rows of a pass (lanes with the same column slice), publish the wave's state
#pragma unroll
    for (int off = LPR; off < 64; off <<= 1)
#pragma unroll
        for (int h = 0; h < REP; ++h)
#pragma unroll
            for (int e = 0; e < PER; ++e)
                o[h][e] += __shfl_xor(o[h][e], off, 64);
    if (tr == 0) {
#pragma unroll
        for (int h = 0; h < REP; ++h)
#pragma unroll
            for (int e = 0; e < PER; ++e)
                w_o[wave][h][dl * PER + e] = o[h][e];
    }
    if (tg == 0) {
        w_m[wave][head] = m_run;
        w_l[wave][head] = l_run;
    }
    __syncthreads();

    const int64_t tuple = ((int64_t)li * A.B + b) * A.kv_heads + kvh;
    for (int idx = tid; idx < REP * D; idx += 256) {
        const int h = idx / D, e = idx - h * D;
        if (h >= A.rep)
            continue;
        float M = fmaxf(fmaxf(w_m[0][h], w_m[1][h]), fmaxf(w_m[2][h], w_m[3][h]));
        float L = 0.0f, O = 0.0f;
#pragma unroll
        for (int wv = 0; wv < 4; ++wv) {
            const float f = w_m[wv][h] == -INFINITY ? 0.0f : __expf(w_m[wv][h] - M);
            L += w_l[wv][h] * f;
            O += w_o[wv][h][e] * f;
        }
        if (A.nsplit == 1) {
            A.out[(((int64_t)li * A.B + b) * A.Hq + (int64_t)kvh * A.rep + h) * D + e] = L > 0.0f ? O / L : 0.0f;
        } else {
            float *pp = A.part + ((tuple * A.nsplit + split) * REP + h) * (D + 2);
            pp[e] = O;
            if (e == 0) {
                pp[D] = M;
                pp[D + 1] = L;
            }
        }
    }
}

template <int D, int REP>
__global__ __launch_bounds__(256) void decode_combine_kernel(DecodeArgs A)
{
    const int b = blockIdx.y / A.kv_heads;
    const int kvh = blockIdx.y - b * A.kv_heads;
    const int li = blockIdx.z;
    const int64_t tuple = ((int64_t)li * A.B + b) * A.kv_heads + kvh;
    for (int idx = threadIdx.x; idx < REP * D; idx += 256) {
        const int h = idx / D, e = idx - h * D;
        if (h >= A.rep)
            continue;
        float M = -INFINITY;
        for (int s = 0; s < A.nsplit; ++s)
            M = fmaxf(M, A.part[((tuple * A.nsplit + s) * REP + h) * (D + 2) + D]);
        float L = 0.0f, O = 0.0f;
        for (int s = 0; s < A.nsplit; ++s) {
            const float *pp = A.part + ((tuple * A.nsplit + s) * REP + h) * (D + 2);
            const float f = pp[D] == -INFINITY ? 0.0f : __expf(pp[D] - M);
            L += pp[D + 1] * f;
            O += pp[e] * f;
        }
        A.out[(((int64_t)li * A.B + b) * A.Hq + (int64_t)kvh * A.rep + h) * D + e] = L > 0.0f ? O / L : 0.0f;
    }
}

static int pick_rep(int rep)
{
    int p = 1;
    while (p < rep)
        p <<= 1;
    return p;
}

static int pick_nsplit(int64_t tuples, int max_blocks)
{
    int64_t ns = tuples > 0 ? (2048 + tuples - 1) / tuples : 1;
    const int cap = (max_blocks + 7) / 8;
    if (ns > cap)
        ns = cap;
    if (ns > 64)
        ns = 64;
    if (ns < 1)
        ns = 1;
    return (int)ns;
}

size_t decode_workspace_bytes(int n_layers, int B, int Hq, int kv_heads, int d, int max_blocks)
{
    const int64_t tuples = (int64_t)n_layers * B * kv_heads;
    const int ns = pick_nsplit(tuples, max_blocks);
    if (ns == 1)
        return 256;
    const int rep = pick_rep(Hq / (kv_heads > 0 ? kv_heads : 1));
    return (size_t)(tuples * ns * rep * (d + 2)) * sizeof(float) + 256;
}

template <typename T, int D>
static void launch_decode_t(hipStream_t s, const DecodeArgs &A, int n_layers, int rep_pad)
{
    const dim3 grid((unsigned)A.nsplit, (unsigned)(A.B * A.kv_heads), (unsigned)n_layers);
    const dim3 cgrid(1, (unsigned)(A.B * A.kv_heads), (unsigned)n_layers);
#define KVF_DEC(R)                                                    \
    do {                                                              \
        if (A.gstride == 1 && A.kv_heads > 1)                         \
            decode_kernel<T, D, R, true><<<grid, 256, 0, s>>>(A);     \
        else                                                          \
            decode_kernel<T, D, R, false><<<grid, 256, 0, s>>>(A);    \
        if (A.nsplit > 1)                                             \
            decode_combine_kernel<D, R><<<cgrid, 256, 0, s>>>(A);     \
    } while (0)
    switch (rep_pad) {
    case 1: KVF_DEC(1); break;
    case 2: KVF_DEC(2); break;
    case 4: KVF_DEC(4); break;
    case 8: KVF_DEC(8); break;
    default: KVF_DEC(16); break;
    }
#undef KVF_DEC
}

int launch_decode(hipStream_t s, const PoolDesc &pool, const TableDesc &tab, int kv_heads, int layer_begin, int n_layers,
                  const void *q, const int32_t *req_start, const int32_t *ctx_len, int B, int Hq, int max_blocks,
                  float sm_scale, void *workspace, size_t workspace_bytes, float *out, bool all_heads)
{
    const int head_dim = all_heads ? pool.d / kv_heads : pool.d;
    DecodeArgs A;
    A.kpool = pool.k; A.vpool = pool.v; A.bt = tab.bt; A.scale_k = tab.scale_k; A.scale_v = tab.scale_v;
    A.q = q; A.req_start = req_start; A.ctx_len = ctx_len; A.out = out;
    A.P = pool.P; A.n = tab.n; A.t = pool.t; A.kv_heads = kv_heads; A.layer_begin = layer_begin; A.B = B; A.Hq = Hq;
    A.rep = Hq / kv_heads;
    A.gstride = all_heads ? 1 : kv_heads;
    A.sm_scale = sm_scale;
    const int64_t tuples = (int64_t)n_layers * B * kv_heads;
    A.nsplit = pick_nsplit(tuples, max_blocks);
    A.blocks_per_split = (max_blocks + A.nsplit - 1) / A.nsplit;
    if (A.blocks_per_split < 1)
        A.blocks_per_split = 1;
    A.part = (float *)workspace;
    if (A.nsplit > 1 && workspace_bytes < decode_workspace_bytes(n_layers, B, Hq, kv_heads, head_dim, max_blocks))
        return KVFUSE_ENOMEM;
    if (tuples == 0)
        return KVFUSE_OK;
    const int rep_pad = pick_rep(A.rep);
    if (pool.dtype == KVFUSE_BF16) {
        if (head_dim == 128) launch_decode_t<bf16_t, 128>(s, A, n_layers, rep_pad);
        else launch_decode_t<bf16_t, 64>(s, A, n_layers, rep_pad);
    } else {
        if (head_dim == 128) launch_decode_t<float, 128>(s, A, n_layers, rep_pad);
        else launch_decode_t<float, 64>(s, A, n_layers, rep_pad);
    }
    return KVFUSE_OK;
}

}  // namespace kvfuse

// ---- the same decode step for callers that cannot allocate -------------------------------------------------
//
// The split-KV partial states (the only device memory the decode kernels use besides their inputs and outputs) live in
// a static device array instead of a caller workspace.  Each GPU that loads the library holds its own copy of the
// array, at its own address, until the process ends; `scratch` below is only the host-side handle of the symbol, so
// host code never passes it to a kernel: the device address is looked up once per device and used from then on.
static __device__ __align__(256) unsigned char scratch[KVFUSE_DECODE_STATIC_SCRATCH_BYTES];

namespace kvfuse {
namespace {

constexpr size_t kStaticScratchBytes = KVFUSE_DECODE_STATIC_SCRATCH_BYTES;
constexpr int kMaxDevices = 64;
std::mutex scratch_mutex;
void *scratch_ptr[kMaxDevices] = {};

// Device address of this device's copy of the array; looked up with that device current, kept afterwards.
hipError_t static_scratch(int device, void **out)
{
    std::lock_guard<std::mutex> lock(scratch_mutex);
    if (!scratch_ptr[device]) {
        int cur = -1;
        hipError_t e = hipGetDevice(&cur);
        if (e != hipSuccess)
            return e;
        if (cur != device && (e = hipSetDevice(device)) != hipSuccess)
            return e;
        void *p = nullptr;
        e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (cur != device)
            (void)hipSetDevice(cur);
        if (e != hipSuccess)
            return e;
        scratch_ptr[device] = p;
    }
    *out = scratch_ptr[device];
    return hipSuccess;
}

}  // namespace

}  // namespace kvfuse

extern "C" int kvfuse_paged_decode_attn_static(kvfuse_ctx *ctx, const kvfuse_pool *pool, const kvfuse_table *table,
                                               int32_t kv_heads, int32_t layer_begin, int32_t n_layers, const void *q,
                                               const int32_t *req_start, const int32_t *ctx_len, int32_t B, int32_t Hq,
                                               int32_t max_blocks, float sm_scale, float *out)
{
    using namespace kvfuse;
    if (!ctx)
        return KVFUSE_EINVAL;
    Ctx *c = &ctx->c;
    if (B == 0 || n_layers == 0)
        return KVFUSE_OK;
    if (c->device < 0 || c->device >= kMaxDevices)
        return fail(c, KVFUSE_EINVAL, "decode (static scratch): device index beyond 63");
    if (!pool || B < 0 || n_layers < 0 || Hq <= 0 || kv_heads <= 0 || max_blocks < 0)
        return fail(c, KVFUSE_EINVAL, "decode (static scratch): null pool or negative size");
    const size_t need = decode_workspace_bytes(n_layers, B, Hq, kv_heads, pool->d, max_blocks);
    if (need > kStaticScratchBytes)
        return fail(c, KVFUSE_ENOMEM, "decode (static scratch): this call needs " + std::to_string(need) +
                                          " bytes of split-KV state, the static array holds " +
                                          std::to_string(kStaticScratchBytes) + "; use kvfuse_paged_decode_attn with a workspace");
    void *ptr = nullptr;
    KVF_HIP(c, static_scratch(c->device, &ptr));
    // every partial state a call reads was written by that same call (empty splits write a neutral state), so
    // nothing has to be cleared between calls
    return kvfuse_paged_decode_attn(ctx, pool, table, kv_heads, layer_begin, n_layers, q, req_start, ctx_len, B, Hq, max_blocks,
                                    sm_scale, ptr, kStaticScratchBytes, out);
}
