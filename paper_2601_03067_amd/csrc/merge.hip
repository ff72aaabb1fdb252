// a4: build the fused representative of every target chosen at this height (Algorithm 1:
// k_l(row) <- normalize(k_l(row) + sum_{i in idx_fused} k_r(i)), and the same for v with the same indices).
//
// Operands are the current unit representatives, i.e. stored block / its stored norm.  HBM-bound: a target with m
// members reads 1 + m blocks and writes one, for K and for V; blocks that are not fused are never touched.  One
// workgroup per target (a persistent grid strides over the work list left by the assignment step), 16-byte
// coalesced loads, the whole block held in registers as fp64, two fixed-order workgroup reductions (length of the
// sum, norm of the rounded result).  The result is rounded once, from fp64, to the pool dtype.
#include "common.h"

namespace kvfuse {

template <typename T> struct Store16;
template <> struct Store16<bf16_t> {
    __device__ static __forceinline__ uint4 pack(const double *u, double *back)
    {
        uint32_t h[8];
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            h[i] = f64_to_bf16_rne(u[i]);
            back[i] = (double)__uint_as_float(h[i] << 16);
        }
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

template <typename T, int MAXC>
__global__ __launch_bounds__(256) void merge_kernel(PoolDesc pool, WorkDesc w, HeightDesc h, int height)
{
    constexpr int PER = Elem<T>::PER16;
    __shared__ double red[4];
    const int tid = threadIdx.x;
    const int chunks = pool.r / PER;
    const int n_act = w.n_active[height];
    for (int t = blockIdx.x; t < n_act; t += gridDim.x) {
        const int packed = w.active[t];
        const int g = packed / w.l_stride;
        const int ti = packed - g * w.l_stride;
        const int node = find_base(h.l_base, h.n_nodes, ti);
        const int i = ti - h.l_base[node];
        const int a = w.set_ids[(int64_t)g * w.n + h.l_off[node] + i];
        const int cnt = w.seg_cnt[(int64_t)g * w.l_stride + ti];
        const int start = w.seg_ptr[(int64_t)g * w.l_stride + ti] - cnt;
        const int32_t *members = w.seg_members + (int64_t)g * w.r_stride + h.r_base[node] + start;

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
                            acc[c][e] += x[e] / nb;
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
            double ss2 = 0.0;
#pragma unroll
            for (int c = 0; c < MAXC; ++c) {
                const int ch = tid + 256 * c;
                if (ch < chunks) {
                    double u[PER], back[PER];
#pragma unroll
                    for (int e = 0; e < PER; ++e)
                        u[e] = len == 0.0 ? 0.0 : acc[c][e] / len;
                    dst[ch] = Store16<T>::pack(u, back);
#pragma unroll
                    for (int e = 0; e < PER; ++e)
                        ss2 = fma(back[e], back[e], ss2);
                }
            }
            const double nrm = sqrt(block_sum_256(ss2, red));
            if (tid == 0) {
                norm_g[a] = nrm;
                if (kv == 0)
                    pool.inv_norm_k[(int64_t)g * pool.P + a] = nrm > 0.0 ? (float)(1.0 / nrm) : 0.0f;
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
#define KVF_MERGE(T, C) merge_kernel<T, C><<<grid, 256, 0, s>>>(pool, w, h, height)
    if (pool.dtype == KVFUSE_BF16) {
        if (maxc <= 1) KVF_MERGE(bf16_t, 1);
        else if (maxc <= 2) KVF_MERGE(bf16_t, 2);
        else KVF_MERGE(bf16_t, 4);
    } else {
        if (maxc <= 1) KVF_MERGE(float, 1);
        else if (maxc <= 2) KVF_MERGE(float, 2);
        else if (maxc <= 4) KVF_MERGE(float, 4);
        else KVF_MERGE(float, 8);
    }
#undef KVF_MERGE
}

}  // namespace kvfuse
