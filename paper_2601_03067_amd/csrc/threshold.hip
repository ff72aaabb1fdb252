// Statistics for threshold control (analysis section: per-layer similarity moments mu_l, sigma_l^2 feed the Poisson
// exceedance rate Lambda_l(u) = n (1 - Phi((u - mu_l) / sigma_l)), the compression corollary and the probability of a
// layer that fuses nothing; method section, remark on self-adjusting thresholds).
//
// The data-parallel part is the sampling: cosines of a caller-drawn list of logical block pairs, the same list
// for every group, read through the block table like every other step.  HBM-bound: two blocks per pair.  The
// moments are a fixed-order reduction, so they do not depend on scheduling.
#include "common.h"

#include <cmath>

namespace kvfuse {

// one wavefront per (group, pair)
template <typename T>
__global__ __launch_bounds__(256) void pair_cosines_kernel(const T *__restrict__ kpool, const double *__restrict__ norm_k,
                                                           const int32_t *__restrict__ bt, const int32_t *__restrict__ pairs,
                                                           int G, int P, int n, int r, int n_pairs, double *__restrict__ cos_out)
{
    const int lane = threadIdx.x & 63;
    const int64_t w = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    if (w >= (int64_t)G * n_pairs)
        return;
    const int g = (int)(w / n_pairs);
    const int q = (int)(w - (int64_t)g * n_pairs);
    const int xi = min(max(pairs[2 * q], 0), n - 1), xj = min(max(pairs[2 * q + 1], 0), n - 1);
    const int pi = min(max(bt[(int64_t)g * n + xi], 0), P - 1), pj = min(max(bt[(int64_t)g * n + xj], 0), P - 1);
    const uint4 *a = reinterpret_cast<const uint4 *>(kpool + ((int64_t)g * P + pi) * r);
    const uint4 *b = reinterpret_cast<const uint4 *>(kpool + ((int64_t)g * P + pj) * r);
    const int chunks = r / Elem<T>::PER16;
    double dot = 0.0;
    for (int c = lane; c < chunks; c += 64) {
        double x[Elem<T>::PER16], y[Elem<T>::PER16];
        Elem<T>::widen(a[c], x);
        Elem<T>::widen(b[c], y);
#pragma unroll
        for (int i = 0; i < Elem<T>::PER16; ++i)
            dot = fma(x[i], y[i], dot);
    }
    dot = wave_sum(dot);
    if (lane == 0) {
        const double na = norm_k[(int64_t)g * P + pi], nb = norm_k[(int64_t)g * P + pj];
        cos_out[w] = (na > 0.0 && nb > 0.0) ? dot / (na * nb) : 0.0;
    }
}

// one workgroup per group: mean and population variance of its n_pairs cosines
__global__ __launch_bounds__(256) void cosine_moments_kernel(const double *__restrict__ cos_in, int n_pairs,
                                                             double *__restrict__ moments)
{
    __shared__ double red[4];
    const int g = blockIdx.x;
    const double *x = cos_in + (int64_t)g * n_pairs;
    double s1 = 0.0, s2 = 0.0;
    for (int q = threadIdx.x; q < n_pairs; q += 256) {
        const double v = x[q];
        s1 += v;
        s2 = fma(v, v, s2);
    }
    s1 = block_sum_256(s1, red);
    s2 = block_sum_256(s2, red);
    if (threadIdx.x == 0) {
        const double mu = n_pairs > 0 ? s1 / n_pairs : 0.0;
        const double var = n_pairs > 0 ? s2 / n_pairs - mu * mu : 0.0;
        moments[2 * g] = mu;
        moments[2 * g + 1] = var > 0.0 ? var : 0.0;
    }
}

void launch_pair_cosines(hipStream_t s, const PoolDesc &pool, const TableDesc &tab, const int32_t *pairs, int n_pairs,
                         double *cos_out)
{
    const int64_t waves = (int64_t)pool.G * n_pairs;
    if (waves <= 0)
        return;
    const unsigned grid = (unsigned)((waves + 3) / 4);
    if (pool.dtype == KVFUSE_BF16)
        pair_cosines_kernel<bf16_t><<<grid, 256, 0, s>>>((const bf16_t *)pool.k, pool.norm_k, tab.bt, pairs, pool.G, pool.P,
                                                          tab.n, pool.r, n_pairs, cos_out);
    else
        pair_cosines_kernel<float><<<grid, 256, 0, s>>>((const float *)pool.k, pool.norm_k, tab.bt, pairs, pool.G, pool.P,
                                                         tab.n, pool.r, n_pairs, cos_out);
}

void launch_cosine_moments(hipStream_t s, const double *cos_in, int G, int n_pairs, double *moments)
{
    if (G > 0)
        cosine_moments_kernel<<<G, 256, 0, s>>>(cos_in, n_pairs, moments);
}

// upper tail of the standard normal
static double normal_tail(double z) { return 0.5 * std::erfc(z / std::sqrt(2.0)); }

}  // namespace kvfuse

using namespace kvfuse;

extern "C" {

int kvfuse_pair_cosines(kvfuse_ctx *ctx, const kvfuse_pool *pool, const kvfuse_table *table, const int32_t *pairs,
                        int32_t n_pairs, double *cos_out)
{
    if (!ctx)
        return KVFUSE_EINVAL;
    Ctx *c = &ctx->c;
    if (!pool || !pool->k || !pool->norm_k || !table || !table->bt || !pairs || !cos_out || n_pairs < 0)
        return fail(c, KVFUSE_EINVAL, "pair cosines: null pointer or negative count");
    if (pool->dtype != KVFUSE_BF16 && pool->dtype != KVFUSE_F32)
        return fail(c, KVFUSE_ESHAPE, "pair cosines: dtype must be KVFUSE_BF16 or KVFUSE_F32");
    const int64_t bytes = (int64_t)pool->t * pool->d * (pool->dtype == KVFUSE_BF16 ? 2 : 4);
    if (bytes <= 0 || bytes % 16 != 0)
        return fail(c, KVFUSE_ESHAPE, "pair cosines: a block must be a multiple of 16 bytes");
    if ((int64_t)pool->G * n_pairs > (int64_t)4 * 0x7FFFFFFF)
        return fail(c, KVFUSE_ESHAPE, "pair cosines: too many (group, pair) items for one call");
    if (table->n <= 0 || pool->P <= 0)
        return KVFUSE_OK;
    launch_pair_cosines(c->stream, to_desc(*pool), to_desc(*table), pairs, n_pairs, cos_out);
    KVF_HIP(c, hipGetLastError());
    return KVFUSE_OK;
}

int kvfuse_cosine_moments(kvfuse_ctx *ctx, const double *cos_in, int32_t G, int32_t n_pairs, double *moments)
{
    if (!ctx)
        return KVFUSE_EINVAL;
    Ctx *c = &ctx->c;
    if (!cos_in || !moments || G < 0 || n_pairs < 0)
        return fail(c, KVFUSE_EINVAL, "cosine moments: null pointer or negative count");
    launch_cosine_moments(c->stream, cos_in, G, n_pairs, moments);
    KVF_HIP(c, hipGetLastError());
    return KVFUSE_OK;
}

double kvfuse_exceedance_rate(double n, double mu, double sigma, double u)
{
    if (!(sigma > 0.0))
        return mu > u ? n : 0.0;
    return n * normal_tail((u - mu) / sigma);
}

double kvfuse_threshold_for_rate(double n, double mu, double sigma, double rate)
{
    if (!(n > 0.0) || !(rate > 0.0) || !(rate < n) || !(sigma > 0.0))
        return std::nan("");
    // normal_tail is strictly decreasing: bisection on z in [-40, 40] to the last bit
    const double p = rate / n;
    double lo = -40.0, hi = 40.0;
    for (int it = 0; it < 200 && hi - lo > 0.0; ++it) {
        const double mid = 0.5 * (lo + hi);
        if (mid == lo || mid == hi)
            break;
        if (normal_tail(mid) > p)
            lo = mid;
        else
            hi = mid;
    }
    return mu + sigma * 0.5 * (lo + hi);
}

int kvfuse_predict_compression(const double *rates, int32_t n_layers, double blocks_per_layer, double *compression_ratio,
                               double *p_no_fusion)
{
    if (!rates || n_layers <= 0 || !(blocks_per_layer > 0.0) || !compression_ratio)
        return KVFUSE_EINVAL;
    double sum = 0.0;
    for (int l = 0; l < n_layers; ++l) {
        sum += rates[l];
        if (p_no_fusion)
            p_no_fusion[l] = std::exp(-rates[l]);
    }
    const double total = (double)n_layers * blocks_per_layer;
    *compression_ratio = total / (total - sum);
    return KVFUSE_OK;
}

double kvfuse_threshold_feedback(double thr, double observed_cr, double target_cr, double gain, double lo, double hi)
{
    const double next = thr + gain * (observed_cr - target_cr) / target_cr;
    return next < lo ? lo : (next > hi ? hi : next);
}

}  // extern "C"
