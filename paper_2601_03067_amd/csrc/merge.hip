// a4: build the fused representative of every target chosen at this height (Algorithm 1:
// k_l(row) <- normalize(k_l(row) + sum_{i in idx_fused} k_r(i)), and the same for v with the same indices).
//
// Operands are the current unit representatives, i.e. stored block / its stored norm.  HBM-bound: a target with m
// members reads 1 + m blocks and writes one, for K and for V; blocks that are not fused are never touched.  One
// or two wavefronts per (target, tensor) -- a persistent grid strides over the work list left by the assignment
// step -- with 16-byte coalesced loads, the loads of the target and of its first members issued together, the whole
// block held in registers as fp64 and two fixed-order reductions (length of the sum, norm of the rounded result).
// Blocks too long for two wavefronts' registers take the workgroup-per-target kernel.
// Unit vectors are formed by multiplying with the fp64 reciprocal of the norm (within one fp64 ulp of a
// division); the result is rounded once, from fp64, to the pool dtype.
#include "common.h"

namespace kvfuse {

template <typename T> struct Store16;
template <> struct Store16<bf16_t> {
    // Eight fp64 values -> bfloat16, nearest even straight from fp64.  The common case is branch free: round to
    // binary32 (nearest even), then to bfloat16 (nearest even); the two roundings agree with the direct one unless
    // the binary32 value sits exactly on a bfloat16 rounding boundary or is zero / subnormal / non-finite.  Those
    // cases (a few per million elements) send all eight values through the exact integer routine.
    __device__ static __forceinline__ uint4 pack(const double *u, double *back)
    {
        uint32_t h[8];
        bool special = false;
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            const uint32_t b = __float_as_uint((float)u[i]);
            const uint32_t ex = (b >> 23) & 0xFFu;
            special |= ex == 0u || ex == 0xFFu || (b & 0xFFFFu) == 0x8000u;
            h[i] = (b + 0x7FFFu + ((b >> 16) & 1u)) >> 16;
        }
        if (special) {
#pragma unroll
            for (int i = 0; i < 8; ++i)
                h[i] = f64_to_bf16_rne(u[i]);
        }
#pragma unroll
        for (int i = 0; i < 8; ++i)
            back[i] = (double)__uint_as_float(h[i] << 16);
        return make_uint4(h[0] | (h[1] << 16), h[2] | (h[3] << 16), h[4] | (h[5] << 16), h[6] | (h[7] << 16));
    }
};
template <> struct Store16<float> {
    __device__ static __forceinline__ uint4 pack(const double *u, double *back)
    {
        uint32_t h[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const float f = (float)u[i];   // v_cvt_f32_f64: round to nearest even
            h[i] = __float_as_uint(f);
            back[i] = (double)f;
        }
        return make_uint4(h[0], h[1], h[2], h[3]);
    }
};

__device__ __forceinline__ int find_base(const int32_t *__restrict__ base, int n_nodes, int idx)
{
    int lo = 0, hi = n_nodes;
    while (hi - lo > 1) {
        const int mid = (lo + hi) >> 1;
        if (base[mid] <= idx)
            lo = mid;
        else
            hi = mid;
    }
    return lo;
}

// GW wavefronts per (target, tensor) item, 4 / GW items per workgroup; CPT = 16-byte chunks per thread.  With GW = 1
// there are no barriers at all; with GW = 2 each thread holds half as much and more items are in flight per CU.
// Q8 (fp8 screen on): the rebuilt key block's one-byte copy and its error are written here as well, from the rounded
// values this kernel has just stored.
template <typename T, int CPT, int GW, bool Q8>
__global__ __launch_bounds__(256, 3) void merge_group_kernel(PoolDesc pool, WorkDesc w, HeightDesc h, int height)
{
    constexpr int PER = Elem<T>::PER16;
    constexpr int GT = 64 * GW;          // threads per item
    constexpr int GPW = 4 / GW;          // items per workgroup
    __shared__ double red[GPW][GW];
    const int grp = __builtin_amdgcn_readfirstlane(threadIdx.x / GT);     // wave-uniform
    const int tg = threadIdx.x % GT;
    const int wv = tg >> 6;
    const int chunks = pool.r / PER;
    const int n_items = 2 * w.n_active[height];
    const int stride = gridDim.x * GPW;
    const int n_iter = (n_items + stride - 1) / stride;      // same for every thread of the workgroup (barriers below)
    // the record of the next item is fetched while the current one is being worked on
    int4 nrec0 = make_int4(0, 0, 0, 0), nrec1 = make_int4(0, 0, 0, 0);
    {
        const int it = blockIdx.x * GPW + grp;
        if (it < n_items) {
            nrec0 = w.active[2 * (int64_t)(it >> 1)];
            nrec1 = w.active[2 * (int64_t)(it >> 1) + 1];
        }
    }
    for (int k = 0; k < n_iter; ++k) {
        const int it = k * stride + blockIdx.x * GPW + grp;
        const bool live = it < n_items;
        const int kv = it & 1;
        // an item belongs to whole wavefronts, so its record is the same in every lane: keep it in scalar registers
        const int g = __builtin_amdgcn_readfirstlane(nrec0.x);
        const int a = __builtin_amdgcn_readfirstlane(nrec0.y);
        const int cnt = live ? __builtin_amdgcn_readfirstlane(nrec0.z) : 0;
        const int32_t *members = w.seg_members + __builtin_amdgcn_readfirstlane(nrec0.w);
        const int m1 = __builtin_amdgcn_readfirstlane(nrec1.x), m2 = __builtin_amdgcn_readfirstlane(nrec1.y);
        T *pool_g = (T *)(kv ? pool.v : pool.k) + (int64_t)g * pool.P * pool.r;
        double *norm_g = (kv ? pool.norm_v : pool.norm_k) + (int64_t)g * pool.P;

        // the target and the first two members are fetched together; further members (rare) follow one by one.
        // Loads are unconditional (a lane past the end of the block re-reads its last chunk, an item past the end of
        // the list reads block 0) and the surplus is masked afterwards: no divergent control flow around memory.
        const int b1 = cnt > 0 ? m1 : a;
        const int b2 = cnt > 1 ? m2 : a;
        const uint4 *sa = reinterpret_cast<const uint4 *>(pool_g + (int64_t)a * pool.r);
        const uint4 *s1 = reinterpret_cast<const uint4 *>(pool_g + (int64_t)b1 * pool.r);
        const uint4 *s2 = reinterpret_cast<const uint4 *>(pool_g + (int64_t)b2 * pool.r);
        uint4 xa[CPT], x1[CPT], x2[CPT];
#pragma unroll
        for (int c = 0; c < CPT; ++c) {
            const int ch = min(tg + GT * c, chunks - 1);
            xa[c] = sa[ch];
            x1[c] = s1[ch];
            x2[c] = s2[ch];
        }
        const double na = norm_g[a], n1 = norm_g[b1], n2 = norm_g[b2];
        {
            const int nit = it + stride;
            if (nit < n_items) {
                nrec0 = w.active[2 * (int64_t)(nit >> 1)];
                nrec1 = w.active[2 * (int64_t)(nit >> 1) + 1];
            }
        }
        const double ia = na == 0.0 ? 0.0 : 1.0 / na;
        const double i1 = (cnt > 0 && n1 != 0.0) ? 1.0 / n1 : 0.0;
        const double i2 = (cnt > 1 && n2 != 0.0) ? 1.0 / n2 : 0.0;
        double acc[CPT][PER];
#pragma unroll
        for (int c = 0; c < CPT; ++c) {
            double ya[PER], y1[PER], y2[PER];
            Elem<T>::widen(xa[c], ya);
            Elem<T>::widen(x1[c], y1);
            Elem<T>::widen(x2[c], y2);
            const bool in = live && tg + GT * c < chunks;
#pragma unroll
            for (int e = 0; e < PER; ++e)
                acc[c][e] = in ? fma(y2[e], i2, fma(y1[e], i1, ya[e] * ia)) : 0.0;
        }
        for (int m = 2; m < cnt; ++m) {
            const int b = members[m];
            const double nb = norm_g[b];
            const double ib = nb == 0.0 ? 0.0 : 1.0 / nb;
            const uint4 *sb = reinterpret_cast<const uint4 *>(pool_g + (int64_t)b * pool.r);
#pragma unroll
            for (int c = 0; c < CPT; ++c) {
                const int ch = tg + GT * c;
                double y[PER];
                Elem<T>::widen(ch < chunks ? sb[ch] : make_uint4(0, 0, 0, 0), y);
#pragma unroll
                for (int e = 0; e < PER; ++e)
                    acc[c][e] = fma(y[e], ib, acc[c][e]);
            }
        }
        double ss = 0.0;
#pragma unroll
        for (int c = 0; c < CPT; ++c)
#pragma unroll
            for (int e = 0; e < PER; ++e)
                ss = fma(acc[c][e], acc[c][e], ss);
        ss = wave_sum(ss);
        if constexpr (GW > 1) {      // fixed-order sum over the item's wavefronts
            if ((tg & 63) == 0)
                red[grp][wv] = ss;
            __syncthreads();
            ss = 0.0;
#pragma unroll
            for (int q = 0; q < GW; ++q)
                ss += red[grp][q];
            __syncthreads();
        }
        const double len = sqrt(ss);
        const double il = len == 0.0 ? 0.0 : 1.0 / len;
        uint4 *dst = reinterpret_cast<uint4 *>(pool_g + (int64_t)a * pool.r);
        // ss2t: the squares of the new key block beyond the prefix of the prefix screen, for its tail share
        const bool want_tail = w.rem_k != nullptr && w.screen_prefix > 0;     // uniform over the launch
        const int prefix_chunks = w.screen_prefix / PER;
        double ss2 = 0.0, ss2t = 0.0;
        uint4 outp[Q8 ? CPT : 1];
#pragma unroll
        for (int c = 0; c < CPT; ++c) {
            const int ch = tg + GT * c;
            double u[PER], back[PER];
#pragma unroll
            for (int e = 0; e < PER; ++e)
                u[e] = acc[c][e] * il;
            const uint4 packed_out = Store16<T>::pack(u, back);
            if constexpr (Q8)
                outp[c] = packed_out;
            if (live && ch < chunks) {
                dst[ch] = packed_out;
#pragma unroll
                for (int e = 0; e < PER; ++e)
                    ss2 = fma(back[e], back[e], ss2);
                if (want_tail && ch >= prefix_chunks) {
#pragma unroll
                    for (int e = 0; e < PER; ++e)
                        ss2t = fma(back[e], back[e], ss2t);
                }
            }
        }
        ss2 = wave_sum(ss2);
        if (want_tail)
            ss2t = wave_sum(ss2t);
        if constexpr (GW > 1) {
            if ((tg & 63) == 0)
                red[grp][wv] = ss2;
            __syncthreads();
            ss2 = 0.0;
#pragma unroll
            for (int q = 0; q < GW; ++q)
                ss2 += red[grp][q];
            __syncthreads();
            if (want_tail) {
                if ((tg & 63) == 0)
                    red[grp][wv] = ss2t;
                __syncthreads();
                ss2t = 0.0;
#pragma unroll
                for (int q = 0; q < GW; ++q)
                    ss2t += red[grp][q];
                __syncthreads();
            }
        }
        const double nrm = sqrt(ss2);
        if (live && tg == 0) {
            norm_g[a] = nrm;
            if (kv == 0) {
                pool.inv_norm_k[(int64_t)g * pool.P + a] = nrm > 0.0 ? (float)(1.0 / nrm) : 0.0f;
                if (want_tail)
                    w.rem_k[(int64_t)g * pool.P + a] = tail_share(ss2t, nrm);
            }
        }
        if constexpr (Q8) {
            auto group_sum = [&](double v) {
                v = wave_sum(v);
                if constexpr (GW > 1) {
                    if ((tg & 63) == 0)
                        red[grp][wv] = v;
                    __syncthreads();
                    v = 0.0;
#pragma unroll
                    for (int q = 0; q < GW; ++q)
                        v += red[grp][q];
                    __syncthreads();
                }
                return v;
            };
            const bool doq = live && kv == 0;               // uniform over the item's wavefronts
            const bool centred = w.q8.dir != nullptr;       // uniform over the launch
            const float *dir_g = (doq && centred) ? w.q8.dir + (int64_t)g * pool.r : nullptr;
            double sm = 0.0;
            if (centred) {
                if (doq) {
#pragma unroll
                    for (int c = 0; c < CPT; ++c) {
                        const int ch = tg + GT * c;
                        if (ch < chunks)
                            q8_dir_dot_chunk<T>(outp[c], dir_g, ch * PER, sm);
                    }
                }
                sm = group_sum(sm);
            }
            const Q8Block blk = q8_block(nrm, centred, sm);
            float se32 = 0.0f;
            if (doq) {
                uint8_t *q = w.q8.k + ((int64_t)g * pool.P + a) * pool.r;
#pragma unroll
                for (int c = 0; c < CPT; ++c) {
                    const int ch = tg + GT * c;
                    if (ch < chunks)
                        quantise_chunk<T>(outp[c], dir_g, ch * PER, blk, q + (size_t)ch * PER, se32);
                }
            }
            const double se = group_sum((double)se32);
            if (doq && tg == 0) {
                const int64_t b = (int64_t)g * pool.P + a;
                w.q8.err[b] = quantise_error(se, blk, nrm);
                w.q8.scale[b] = (float)blk.scale;
                w.q8.alpha[b] = nrm > 0.0 ? (float)blk.alpha : 0.0f;
            }
        }
    }
}

// Workgroup per target: for blocks longer than one wavefront can hold in registers.
template <typename T, int MAXC>
__global__ __launch_bounds__(256) void merge_kernel(PoolDesc pool, WorkDesc w, HeightDesc h, int height)
{
    constexpr int PER = Elem<T>::PER16;
    __shared__ double red[4];
    const int tid = threadIdx.x;
    const int chunks = pool.r / PER;
    const int n_act = w.n_active[height];
    for (int t = blockIdx.x; t < n_act; t += gridDim.x) {
        const int4 rec = w.active[2 * (int64_t)t];
        const int g = rec.x;
        const int a = rec.y;
        const int cnt = rec.z;
        const int32_t *members = w.seg_members + rec.w;

        for (int kv = 0; kv < 2; ++kv) {
            T *pool_g = (T *)(kv ? pool.v : pool.k) + (int64_t)g * pool.P * pool.r;
            double *norm_g = (kv ? pool.norm_v : pool.norm_k) + (int64_t)g * pool.P;
            double acc[MAXC][PER];
#pragma unroll
            for (int c = 0; c < MAXC; ++c)
#pragma unroll
                for (int e = 0; e < PER; ++e)
                    acc[c][e] = 0.0;
            for (int m = -1; m < cnt; ++m) {
                const int b = m < 0 ? a : members[m];
                const double nb = norm_g[b];
                if (nb == 0.0)
                    continue;   // a zero block has the zero vector as direction
                const uint4 *src = reinterpret_cast<const uint4 *>(pool_g + (int64_t)b * pool.r);
#pragma unroll
                for (int c = 0; c < MAXC; ++c) {
                    const int ch = tid + 256 * c;
                    if (ch < chunks) {
                        double x[PER];
                        Elem<T>::widen(src[ch], x);
#pragma unroll
                        for (int e = 0; e < PER; ++e)
                            acc[c][e] = fma(x[e], 1.0 / nb, acc[c][e]);
                    }
                }
            }
            double ss = 0.0;
#pragma unroll
            for (int c = 0; c < MAXC; ++c)
#pragma unroll
                for (int e = 0; e < PER; ++e)
                    ss = fma(acc[c][e], acc[c][e], ss);
            const double len = sqrt(block_sum_256(ss, red));
            uint4 *dst = reinterpret_cast<uint4 *>(pool_g + (int64_t)a * pool.r);
            const bool want_tail = w.rem_k != nullptr && w.screen_prefix > 0 && kv == 0;     // uniform over the workgroup
            const int prefix_chunks = w.screen_prefix / PER;
            double ss2 = 0.0, ss2t = 0.0;
#pragma unroll
            for (int c = 0; c < MAXC; ++c) {
                const int ch = tid + 256 * c;
                if (ch < chunks) {
                    double u[PER], back[PER];
#pragma unroll
                    for (int e = 0; e < PER; ++e)
                        u[e] = len == 0.0 ? 0.0 : acc[c][e] * (1.0 / len);
                    dst[ch] = Store16<T>::pack(u, back);
#pragma unroll
                    for (int e = 0; e < PER; ++e)
                        ss2 = fma(back[e], back[e], ss2);
                    if (want_tail && ch >= prefix_chunks) {
#pragma unroll
                        for (int e = 0; e < PER; ++e)
                            ss2t = fma(back[e], back[e], ss2t);
                    }
                }
            }
            const double nrm = sqrt(block_sum_256(ss2, red));
            double tail2 = 0.0;
            if (want_tail)
                tail2 = block_sum_256(ss2t, red);
            if (tid == 0) {
                norm_g[a] = nrm;
                if (kv == 0) {
                    pool.inv_norm_k[(int64_t)g * pool.P + a] = nrm > 0.0 ? (float)(1.0 / nrm) : 0.0f;
                    if (want_tail)
                        w.rem_k[(int64_t)g * pool.P + a] = tail_share(tail2, nrm);
                }
            }
        }
    }
}

void launch_merge(hipStream_t s, const PoolDesc &pool, const WorkDesc &w, const HeightDesc &h, int height)
{
    if ((int64_t)w.G * h.total_l_cap <= 0)
        return;
    int64_t want = (int64_t)w.G * h.total_l_cap;
    const unsigned grid = (unsigned)(want < 256 * 16 ? want : 256 * 16);
    const int per = pool.dtype == KVFUSE_BF16 ? 8 : 4;
    const int chunks = pool.r / per;
    const int maxc = (chunks + 255) / 256;
    const int cpl = (chunks + 63) / 64;
    if (cpl <= 8) {
        const unsigned wgrid = (unsigned)(want < 256 * 16 ? (want + 1) / 2 + 1 : 256 * 16);
        // up to 4 chunks per lane (bfloat16) one wavefront holds the block and no barrier is needed; longer blocks
        // and binary32 blocks of 4 chunks per lane are split over two wavefronts
#define KVF_MERGE_G(T, C, W)                                                          \
    do {                                                                              \
        if (w.q8.k)                                                                  \
            merge_group_kernel<T, C, W, true><<<wgrid, 256, 0, s>>>(pool, w, h, height);  \
        else                                                                          \
            merge_group_kernel<T, C, W, false><<<wgrid, 256, 0, s>>>(pool, w, h, height); \
    } while (0)
        if (pool.dtype == KVFUSE_BF16) {
            if (cpl <= 1) KVF_MERGE_G(bf16_t, 1, 1);
            else if (cpl <= 2) KVF_MERGE_G(bf16_t, 2, 1);
            else if (cpl <= 4) KVF_MERGE_G(bf16_t, 4, 1);
            else KVF_MERGE_G(bf16_t, 4, 2);
        } else {
            if (cpl <= 1) KVF_MERGE_G(float, 1, 1);
            else if (cpl <= 2) KVF_MERGE_G(float, 2, 1);
            else if (cpl <= 4) KVF_MERGE_G(float, 2, 2);
            else KVF_MERGE_G(float, 4, 2);
        }
#undef KVF_MERGE_G
        return;
    }
#define KVF_MERGE(T, C) merge_kernel<T, C><<<grid, 256, 0, s>>>(pool, w, h, height)
    if (pool.dtype == KVFUSE_BF16) {
        if (maxc <= 1) KVF_MERGE(bf16_t, 1);
        else if (maxc <= 2) KVF_MERGE(bf16_t, 2);
        else if (maxc <= 4) KVF_MERGE(bf16_t, 4);
        else KVF_MERGE(bf16_t, 8);
    } else {
        if (maxc <= 1) KVF_MERGE(float, 1);
        else if (maxc <= 2) KVF_MERGE(float, 2);
        else if (maxc <= 4) KVF_MERGE(float, 4);
        else KVF_MERGE(float, 8);
    }
#undef KVF_MERGE
    launch_quantise_targets(s, pool, w, height);        // no-op unless the fp8 screen is on
}

}  // namespace kvfuse
