// a2: similarity of every left block with every right block of a tree node (Algorithm 1: sim <- k_l k_r^T on
// unit vectors, keys only), as a gathered, grouped NT GEMM on the MFMA units.
//
// Rows of both operands are whole KV blocks addressed by physical id, so every gathered row is one contiguous
// r-element run.  A workgroup owns one panel of BN right blocks of one (group, node) and streams all tiles of
// BM left blocks past it; the cosine matrix is never written (unless a dense buffer is asked for): the epilogue
// multiplies the fp32 accumulators by the two inverse norms, keeps the column maximum and appends every entry
// above the candidate floor to the column's candidate list.  Because one workgroup sees all rows of its columns,
// no float atomics and no cross-workgroup reduction are needed.
//
// Tiling: 256 threads = 4 wavefronts in a 2 x 2 arrangement, 64 x 64 outputs per wavefront = 2 x 2 MFMA tiles of
// 32 x 32 (v_mfma_f32_32x32x16_bf16, or 4 x v_mfma_f32_32x32x2_f32 per 16-byte fragment for f32 pools).  K is
// walked in 128-byte slices per row, double buffered in LDS with a 16-byte-chunk XOR swizzle (chunk ^ (row & 7))
// so that both the 16-byte stores and the MFMA fragment reads are bank-conflict free.
#include "common.h"

namespace kvfuse {

typedef float floatx16 __attribute__((ext_vector_type(16)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));

constexpr int BM = 128;
constexpr int BN = 128;

template <typename T> struct Mma;
template <> struct Mma<bf16_t> {
    __device__ static __forceinline__ void run(const uint4 &a, const uint4 &b, floatx16 &c)
    {
        c = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a), __builtin_bit_cast(bf16x8, b), c, 0, 0, 0);
    }
};
template <> struct Mma<float> {
    // One 16-byte fragment holds 4 consecutive floats of a row; lane halves hold different chunks.  Element e of
    // both operands pairs up, which is a valid k-assignment because A and B use the same one.
    __device__ static __forceinline__ void run(const uint4 &a, const uint4 &b, floatx16 &c)
    {
        c = __builtin_amdgcn_mfma_f32_32x32x2f32(__uint_as_float(a.x), __uint_as_float(b.x), c, 0, 0, 0);
        c = __builtin_amdgcn_mfma_f32_32x32x2f32(__uint_as_float(a.y), __uint_as_float(b.y), c, 0, 0, 0);
        c = __builtin_amdgcn_mfma_f32_32x32x2f32(__uint_as_float(a.z), __uint_as_float(b.z), c, 0, 0, 0);
        c = __builtin_amdgcn_mfma_f32_32x32x2f32(__uint_as_float(a.w), __uint_as_float(b.w), c, 0, 0, 0);
    }
};

template <typename T>
__global__ __launch_bounds__(256, 2) void similarity_kernel(PoolDesc pool, WorkDesc w, HeightDesc h, float thr_floor,
                                                            float *__restrict__ dense_s)
{
    __shared__ uint4 lds_a[2][BM * 8];
    __shared__ uint4 lds_b[2][BN * 8];
    __shared__ float lds_invl[BM];
    __shared__ int lds_cnt[BN];
    __shared__ float red_val[2][BN];
    __shared__ int red_idx[2][BN];

    // Consecutive hardware workgroup ids go to different XCDs; renumber so that the panels of one (group, node),
    // which all read the same left rows, land on one XCD and share its L2.
    const int per_xcd = gridDim.x >> 3;
    const int v = (blockIdx.x & 7) * per_xcd + (blockIdx.x >> 3);
    if (v >= w.G * h.n_panels)
        return;
    const int g = v / h.n_panels;
    const int panel = v - g * h.n_panels;
    const int node = h.panel_node[panel];
    const int col0 = h.panel_col0[panel];
    const int ml = w.set_cnt[(int64_t)g * w.n_slots + h.l_slot[node]];
    const int mr = w.set_cnt[(int64_t)g * w.n_slots + h.r_slot[node]];
    if (col0 >= mr)
        return;
    const int32_t *l_ids = w.set_ids + (int64_t)g * w.n + h.l_off[node];
    const int32_t *r_ids = w.set_ids + (int64_t)g * w.n + h.r_off[node];
    const int64_t cbase = (int64_t)g * w.r_stride + h.r_base[node];

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = tid >> 6;
    const int wm = wave >> 1, wn = wave & 1;
    const int64_t row_bytes = (int64_t)pool.r * sizeof(T);
    const int nk = (int)(row_bytes >> 7);                 // 128-byte slices per row
    const int n_rt = (ml + BM - 1) / BM;
    const int total_it = n_rt * nk;
    const char *kbase = (const char *)pool.k + (int64_t)g * pool.P * row_bytes;

    // global -> LDS mapping: 8 threads cover the 128-byte slice of one row, 32 rows per pass, 4 passes
    const int ld_c = tid & 7;
    const int ld_r = tid >> 3;
    const char *pb[4];
    const char *pa[4];
#pragma unroll
    for (int p = 0; p < 4; ++p) {
        int col = col0 + ld_r + 32 * p;
        col = col < mr ? col : mr - 1;
        pb[p] = kbase + (int64_t)r_ids[col] * row_bytes + ld_c * 16;
        pa[p] = kbase;
    }
    auto set_pa = [&](int rt) {
#pragma unroll
        for (int p = 0; p < 4; ++p) {
            int row = rt * BM + ld_r + 32 * p;
            row = row < ml ? row : ml - 1;
            pa[p] = kbase + (int64_t)l_ids[row] * row_bytes + ld_c * 16;
        }
    };
    int pf_rt = 0, pf_kt = 0;
    uint4 ra[4], rb[4];
    auto load_tile = [&]() {
#pragma unroll
        for (int p = 0; p < 4; ++p) {
            ra[p] = *reinterpret_cast<const uint4 *>(pa[p] + (int64_t)pf_kt * 128);
            rb[p] = *reinterpret_cast<const uint4 *>(pb[p] + (int64_t)pf_kt * 128);
        }
        if (++pf_kt == nk) {
            pf_kt = 0;
            if (++pf_rt < n_rt)
                set_pa(pf_rt);
        }
    };
    auto store_tile = [&](int buf) {
#pragma unroll
        for (int p = 0; p < 4; ++p) {
            const int row = ld_r + 32 * p;
            const int slot = row * 8 + (ld_c ^ (row & 7));
            lds_a[buf][slot] = ra[p];
            lds_b[buf][slot] = rb[p];
        }
    };

    if (tid < BN)
        lds_cnt[tid] = 0;

    // per-lane state of the epilogue: lane holds column (lane & 31) of each of its two N tiles
    const int half = lane >> 5;
    float inv_r[2];
    float best[2] = {-INFINITY, -INFINITY};
    int best_i[2] = {0x7FFFFFFF, 0x7FFFFFFF};
#pragma unroll
    for (int nt = 0; nt < 2; ++nt) {
        const int col = col0 + wn * 64 + nt * 32 + (lane & 31);
        inv_r[nt] = col < mr ? pool.inv_norm_k[(int64_t)g * pool.P + r_ids[col]] : 0.0f;
    }

    floatx16 acc[2][2];
#pragma unroll
    for (int mt = 0; mt < 2; ++mt)
#pragma unroll
        for (int nt = 0; nt < 2; ++nt)
#pragma unroll
            for (int e = 0; e < 16; ++e)
                acc[mt][nt][e] = 0.0f;

    if (total_it > 0) {
        set_pa(0);
        load_tile();
        store_tile(0);
    }
    __syncthreads();

    for (int it = 0; it < total_it; ++it) {
        const int cur = it & 1;
        const int kt = it % nk;
        const int rt = it / nk;
        const bool more = it + 1 < total_it;
        if (kt == 0 && tid < BM) {
            const int row = rt * BM + tid;
            lds_invl[tid] = row < ml ? pool.inv_norm_k[(int64_t)g * pool.P + l_ids[row]] : 0.0f;
        }
        if (more)
            load_tile();
#pragma unroll
        for (int s = 0; s < 4; ++s) {
            uint4 fa[2], fb[2];
            const int chunk = 2 * s + half;
#pragma unroll
            for (int mt = 0; mt < 2; ++mt) {
                const int row = wm * 64 + mt * 32 + (lane & 31);
                fa[mt] = lds_a[cur][row * 8 + (chunk ^ (row & 7))];
            }
#pragma unroll
            for (int nt = 0; nt < 2; ++nt) {
                const int row = wn * 64 + nt * 32 + (lane & 31);
                fb[nt] = lds_b[cur][row * 8 + (chunk ^ (row & 7))];
            }
#pragma unroll
            for (int mt = 0; mt < 2; ++mt)
#pragma unroll
                for (int nt = 0; nt < 2; ++nt)
                    Mma<T>::run(fa[mt], fb[nt], acc[mt][nt]);
        }
        if (more)
            store_tile(cur ^ 1);
        if (kt == nk - 1) {
            __syncthreads();   // lds_invl of this row tile is visible even when nk == 1
#pragma unroll
            for (int nt = 0; nt < 2; ++nt) {
                const int cl = wn * 64 + nt * 32 + (lane & 31);   // column within the panel
                const int col = col0 + cl;
#pragma unroll
                for (int mt = 0; mt < 2; ++mt) {
#pragma unroll
                    for (int e = 0; e < 16; ++e) {
                        const int rl = wm * 64 + mt * 32 + (e >> 2) * 8 + half * 4 + (e & 3);
                        const int row = rt * BM + rl;
                        const float s = acc[mt][nt][e] * lds_invl[rl] * inv_r[nt];
                        acc[mt][nt][e] = 0.0f;
                        if (row < ml && col < mr) {
                            if (dense_s)
                                dense_s[(int64_t)g * h.total_s + h.s_base[node] + (int64_t)row * h.r_cap[node] + col] = s;
                            if (s > thr_floor) {
                                const int slot = atomicAdd(&lds_cnt[cl], 1);
                                if (slot < w.cand_cap) {
                                    w.cand_idx[(cbase + col) * w.cand_cap + slot] = row;
                                    w.cand_val[(cbase + col) * w.cand_cap + slot] = s;
                                }
                            }
                            if (s > best[nt]) {
                                best[nt] = s;
                                best_i[nt] = row;
                            }
                        }
                    }
                }
            }
        }
        __syncthreads();
    }

    // column maxima: the two lane halves hold different rows of the same column, then the two wavefronts with
    // the same wn; ties go to the lower row.
#pragma unroll
    for (int nt = 0; nt < 2; ++nt) {
        const float ov = __shfl_xor(best[nt], 32, 64);
        const int oi = __shfl_xor(best_i[nt], 32, 64);
        if (ov > best[nt] || (ov == best[nt] && oi < best_i[nt])) {
            best[nt] = ov;
            best_i[nt] = oi;
        }
        if (half == 0) {
            red_val[wm][wn * 64 + nt * 32 + lane] = best[nt];
            red_idx[wm][wn * 64 + nt * 32 + lane] = best_i[nt];
        }
    }
    __syncthreads();
    if (tid < BN && col0 + tid < mr) {
        float bv = red_val[0][tid];
        int bi = red_idx[0][tid];
        if (red_val[1][tid] > bv || (red_val[1][tid] == bv && red_idx[1][tid] < bi)) {
            bv = red_val[1][tid];
            bi = red_idx[1][tid];
        }
        w.best_sim[cbase + col0 + tid] = bv;
        w.best_idx[cbase + col0 + tid] = ml > 0 ? bi : -1;
        w.cand_cnt[cbase + col0 + tid] = lds_cnt[tid];
    }
}

void launch_similarity(hipStream_t s, const PoolDesc &pool, const WorkDesc &w, const HeightDesc &h, float thr_floor,
                       float *dense_s)
{
    const int64_t total = (int64_t)w.G * h.n_panels;
    if (total <= 0)
        return;
    const unsigned grid = (unsigned)(((total + 7) / 8) * 8);
    if (pool.dtype == KVFUSE_BF16)
        similarity_kernel<bf16_t><<<grid, 256, 0, s>>>(pool, w, h, thr_floor, dense_s);
    else
        similarity_kernel<float><<<grid, 256, 0, s>>>(pool, w, h, thr_floor, dense_s);
}

}  // namespace kvfuse
