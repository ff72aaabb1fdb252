// a2: similarity of every left block with every right block of a tree node (Algorithm 1: sim <- k_l k_r^T on
// unit vectors, keys only), as a gathered, grouped NT GEMM on the MFMA units.
//
// Rows of both operands are whole KV blocks addressed by physical id, so every gathered row is one contiguous
// r-element run.  The cosine matrix is never written (unless a dense buffer is asked for): the epilogue multiplies
// the fp32 accumulators by the two inverse norms, keeps the column maximum and appends every entry above the
// candidate floor to the column's candidate list.
//
// Work decomposition.  A work item is (group, node, panel of BN right blocks, chunk of up to RT tiles of BM left
// blocks); one workgroup per item.  Items are numbered so that consecutive ones form a 2-D patch of one node
// (8 panels x several chunks), and hardware workgroup ids are renumbered so that each XCD walks a contiguous range
// of items: the workgroups resident on one XCD then share both their left tiles and their right panels through
// that XCD's L2 instead of each streaming a private panel from HBM.  Column results of different chunks meet in
// global memory through integer atomics only (64-bit max of (ordered cosine, inverted row), 32-bit slot counters),
// so the outcome does not depend on scheduling.
//
// Tiling.  WM x WN wavefronts, each TM x TN MFMA tiles of 32 x 32 (v_mfma_f32_32x32x16_bf16, or 4 x
// v_mfma_f32_32x32x2_f32 per 16-byte fragment for f32 pools).  K is walked in 128-byte slices per row, double
// buffered in LDS with a 16-byte-chunk XOR swizzle (chunk ^ ((row >> 1) & 7)): the LDS has 64 four-byte banks, so
// two 128-byte rows make one sweep over the banks, and with this swizzle both the 16-byte stores (16 lanes = 2 rows x
// 8 chunks) and the MFMA fragment reads (16 lanes = 16 rows, one chunk) touch every bank exactly once.  Global loads of the next slice are in flight during the MFMAs.
#include "common.h"

namespace kvfuse {

typedef float floatx16 __attribute__((ext_vector_type(16)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));

template <typename T> struct Mma;
template <> struct Mma<bf16_t> {
    __device__ static __forceinline__ floatx16 run(const uint4 a, const uint4 b, floatx16 c)
    {
        return __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a), __builtin_bit_cast(bf16x8, b), c, 0, 0, 0);
    }
};
template <> struct Mma<float> {
    // One 16-byte fragment holds 4 consecutive floats of a row; lane halves hold different chunks.  Element e of
    // both operands pairs up, which is a valid k-assignment because A and B use the same one.
    __device__ static __forceinline__ floatx16 run(const uint4 a, const uint4 b, floatx16 c)
    {
        c = __builtin_amdgcn_mfma_f32_32x32x2f32(__uint_as_float(a.x), __uint_as_float(b.x), c, 0, 0, 0);
        c = __builtin_amdgcn_mfma_f32_32x32x2f32(__uint_as_float(a.y), __uint_as_float(b.y), c, 0, 0, 0);
        c = __builtin_amdgcn_mfma_f32_32x32x2f32(__uint_as_float(a.z), __uint_as_float(b.z), c, 0, 0, 0);
        c = __builtin_amdgcn_mfma_f32_32x32x2f32(__uint_as_float(a.w), __uint_as_float(b.w), c, 0, 0, 0);
        return c;
    }
};

// (cosine, row) packed so that an unsigned 64-bit max picks the larger cosine and, on equal cosines, the lower row.
__device__ __forceinline__ unsigned long long pack_best(float s, int row)
{
    const uint32_t b = __float_as_uint(s);
    const uint32_t ord = (b & 0x80000000u) ? ~b : (b | 0x80000000u);
    return ((unsigned long long)ord << 32) | (unsigned long long)(0xFFFFFFFFu - (uint32_t)row);
}

struct SimArgs {
    int32_t G, n, n_slots, r_stride, cand_cap, P, n_items;
    int32_t row_bytes;             // bytes of one block row
    float thr_floor;
    int64_t total_s;
};

template <typename T, int WM, int WN, int TM, int TN>
__global__ __launch_bounds__(64 * WM * WN) void similarity_kernel(
    SimArgs A, const char *__restrict__ kpool, const float *__restrict__ inv_norm, const int32_t *__restrict__ set_ids,
    const int32_t *__restrict__ set_cnt, const int32_t *__restrict__ item_node, const int32_t *__restrict__ item_col0,
    const int32_t *__restrict__ item_row0, const int32_t *__restrict__ item_rows, const int32_t *__restrict__ l_off,
    const int32_t *__restrict__ r_off, const int32_t *__restrict__ l_slot, const int32_t *__restrict__ r_slot,
    const int32_t *__restrict__ r_base, const int32_t *__restrict__ r_cap, const int64_t *__restrict__ s_base,
    unsigned long long *__restrict__ best_packed, int32_t *__restrict__ cand_cnt, int32_t *__restrict__ cand_idx,
    float *__restrict__ cand_val, float *__restrict__ dense_s)
{
    constexpr int NT = 64 * WM * WN;
    constexpr int BM = WM * TM * 32;
    constexpr int BN = WN * TN * 32;
    constexpr int LA = BM * 8 / NT;   // 16-byte chunks of the left tile per thread and K slice
    constexpr int LB = BN * 8 / NT;
    constexpr int RPP = NT / 8;       // rows covered by one pass of the loaders
    static_assert(LA == 4 && LB == 4, "the loaders below are written out for 4 + 4 chunks per thread");

    __shared__ uint4 lds_a[2][BM * 8];
    __shared__ uint4 lds_b[2][BN * 8];
    __shared__ float lds_invl[BM];

    // hardware workgroup id -> item: XCD x (ids congruent x mod 8) walks items [x * per_xcd, (x + 1) * per_xcd)
    const int per_xcd = gridDim.x >> 3;
    const long long v = (long long)(blockIdx.x & 7) * per_xcd + (blockIdx.x >> 3);
    if (v >= (long long)A.G * A.n_items)
        return;
    const int g = (int)(v / A.n_items);
    const int item = (int)(v - (long long)g * A.n_items);
    const int node = item_node[item];
    const int col0 = item_col0[item];
    const int row0 = item_row0[item];
    const int ml = set_cnt[(int64_t)g * A.n_slots + l_slot[node]];
    const int mr = set_cnt[(int64_t)g * A.n_slots + r_slot[node]];
    if (col0 >= mr || row0 >= ml)
        return;
    const int row_end = min(ml, row0 + item_rows[item]);
    const int32_t *__restrict__ l_ids = set_ids + (int64_t)g * A.n + l_off[node];
    const int32_t *__restrict__ r_ids = set_ids + (int64_t)g * A.n + r_off[node];
    const int64_t cbase = (int64_t)g * A.r_stride + r_base[node];

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = tid >> 6;
    const int wm = wave / WN, wn = wave % WN;
    const int half = lane >> 5;
    const int64_t row_bytes = A.row_bytes;
    const int nk = A.row_bytes >> 7;                          // 128-byte slices per row
    const int n_rt = (row_end - row0 + BM - 1) / BM;
    const int total_it = n_rt * nk;
    const char *__restrict__ kg = kpool + (int64_t)g * A.P * row_bytes;
    const float *__restrict__ inv_g = inv_norm + (int64_t)g * A.P;

    // loaders: 8 consecutive threads cover the 128-byte slice of one row
    const int ld_c = tid & 7;
    const int ld_r = tid >> 3;
    // The staging registers are named scalars, not arrays: an array that is written under one `if` and read under
    // another is left in scratch memory by the compiler, which doubles the memory traffic of the kernel.
#define KVF_COL_PTR(P) (kg + (int64_t)r_ids[min(col0 + ld_r + RPP * (P), mr - 1)] * row_bytes + ld_c * 16)
#define KVF_ROW_PTR(RT, P) (kg + (int64_t)l_ids[min(row0 + (RT) * BM + ld_r + RPP * (P), row_end - 1)] * row_bytes + ld_c * 16)
#define KVF_LD(PTR, KO) (*reinterpret_cast<const uint4 *>((PTR) + (KO)))
#define KVF_SLOT(P) ((ld_r + RPP * (P)) * 8 + (ld_c ^ (((ld_r + RPP * (P)) >> 1) & 7)))
    const char *pb0 = KVF_COL_PTR(0), *pb1 = KVF_COL_PTR(1), *pb2 = KVF_COL_PTR(2), *pb3 = KVF_COL_PTR(3);
    const char *pa0 = KVF_ROW_PTR(0, 0), *pa1 = KVF_ROW_PTR(0, 1), *pa2 = KVF_ROW_PTR(0, 2), *pa3 = KVF_ROW_PTR(0, 3);
    const int sl0 = KVF_SLOT(0), sl1 = KVF_SLOT(1), sl2 = KVF_SLOT(2), sl3 = KVF_SLOT(3);

    // per-lane epilogue state: the lane holds column (lane & 31) of each of its TN tiles
    float inv_r[TN], best[TN];
    int best_i[TN];
#pragma unroll
    for (int nt = 0; nt < TN; ++nt) {
        const int col = col0 + (wn * TN + nt) * 32 + (lane & 31);
        inv_r[nt] = col < mr ? inv_g[r_ids[col]] : 0.0f;
        best[nt] = -INFINITY;
        best_i[nt] = 0x7FFFFFFF;
    }

    floatx16 acc[TM][TN];
#pragma unroll
    for (int mt = 0; mt < TM; ++mt)
#pragma unroll
        for (int nt = 0; nt < TN; ++nt)
#pragma unroll
            for (int e = 0; e < 16; ++e)
                acc[mt][nt][e] = 0.0f;

    int pf_kt = 1, pf_rt = 0;
    // first slice
    uint4 ra0 = KVF_LD(pa0, 0), ra1 = KVF_LD(pa1, 0), ra2 = KVF_LD(pa2, 0), ra3 = KVF_LD(pa3, 0);
    uint4 rb0 = KVF_LD(pb0, 0), rb1 = KVF_LD(pb1, 0), rb2 = KVF_LD(pb2, 0), rb3 = KVF_LD(pb3, 0);
    if (pf_kt == nk) {
        pf_kt = 0;
        pf_rt = 1;
    }
    lds_a[0][sl0] = ra0; lds_a[0][sl1] = ra1; lds_a[0][sl2] = ra2; lds_a[0][sl3] = ra3;
    lds_b[0][sl0] = rb0; lds_b[0][sl1] = rb1; lds_b[0][sl2] = rb2; lds_b[0][sl3] = rb3;
    __syncthreads();

    for (int it = 0; it < total_it; ++it) {
        const int cur = it & 1;
        const int kt = it % nk;
        const int rt = it / nk;
        const bool more = it + 1 < total_it;
        if (kt == 0) {
            for (int x = tid; x < BM; x += NT) {
                const int row = row0 + rt * BM + x;
                lds_invl[x] = row < row_end ? inv_g[l_ids[row]] : 0.0f;
            }
        }
        if (more) {
            if (pf_kt == 0) {      // the prefetch enters a new tile of left rows
                pa0 = KVF_ROW_PTR(pf_rt, 0); pa1 = KVF_ROW_PTR(pf_rt, 1); pa2 = KVF_ROW_PTR(pf_rt, 2); pa3 = KVF_ROW_PTR(pf_rt, 3);
            }
            const int64_t ko = (int64_t)pf_kt * 128;
            ra0 = KVF_LD(pa0, ko); ra1 = KVF_LD(pa1, ko); ra2 = KVF_LD(pa2, ko); ra3 = KVF_LD(pa3, ko);
            rb0 = KVF_LD(pb0, ko); rb1 = KVF_LD(pb1, ko); rb2 = KVF_LD(pb2, ko); rb3 = KVF_LD(pb3, ko);
            if (++pf_kt == nk) {
                pf_kt = 0;
                ++pf_rt;
            }
        }
        const uint4 *__restrict__ la = lds_a[cur];
        const uint4 *__restrict__ lb = lds_b[cur];
#pragma unroll
        for (int s = 0; s < 4; ++s) {
            uint4 fa[TM], fb[TN];
            const int chunk = 2 * s + half;
#pragma unroll
            for (int mt = 0; mt < TM; ++mt) {
                const int row = (wm * TM + mt) * 32 + (lane & 31);
                fa[mt] = la[row * 8 + (chunk ^ ((row >> 1) & 7))];
            }
#pragma unroll
            for (int nt = 0; nt < TN; ++nt) {
                const int row = (wn * TN + nt) * 32 + (lane & 31);
                fb[nt] = lb[row * 8 + (chunk ^ ((row >> 1) & 7))];
            }
#pragma unroll
            for (int mt = 0; mt < TM; ++mt)
#pragma unroll
                for (int nt = 0; nt < TN; ++nt)
                    acc[mt][nt] = Mma<T>::run(fa[mt], fb[nt], acc[mt][nt]);
        }
        if (more) {
            uint4 *__restrict__ na = lds_a[cur ^ 1];
            uint4 *__restrict__ nb = lds_b[cur ^ 1];
            na[sl0] = ra0; na[sl1] = ra1; na[sl2] = ra2; na[sl3] = ra3;
            nb[sl0] = rb0; nb[sl1] = rb1; nb[sl2] = rb2; nb[sl3] = rb3;
        }
        if (kt == nk - 1) {
            __syncthreads();   // lds_invl of this row tile is visible even when nk == 1
#pragma unroll
            for (int nt = 0; nt < TN; ++nt) {
                const int col = col0 + (wn * TN + nt) * 32 + (lane & 31);
#pragma unroll
                for (int mt = 0; mt < TM; ++mt) {
#pragma unroll
                    for (int e = 0; e < 16; ++e) {
                        const int rl = (wm * TM + mt) * 32 + (e >> 2) * 8 + half * 4 + (e & 3);
                        const int row = row0 + rt * BM + rl;
                        const float s = acc[mt][nt][e] * lds_invl[rl] * inv_r[nt];
                        acc[mt][nt][e] = 0.0f;
                        if (row < row_end && col < mr) {
                            if (dense_s)
                                dense_s[(int64_t)g * A.total_s + s_base[node] + (int64_t)row * r_cap[node] + col] = s;
                            if (s > A.thr_floor) {
                                const int slot = atomicAdd(&cand_cnt[cbase + col], 1);
                                if (slot < A.cand_cap) {
                                    cand_idx[(cbase + col) * A.cand_cap + slot] = row;
                                    cand_val[(cbase + col) * A.cand_cap + slot] = s;
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

    // column maxima of this item: lane halves hold different rows of a column; all chunks of a panel and all
    // wavefront rows meet in the packed 64-bit maximum
#pragma unroll
    for (int nt = 0; nt < TN; ++nt) {
        const int col = col0 + (wn * TN + nt) * 32 + (lane & 31);
        const float ov = __shfl_xor(best[nt], 32, 64);
        const int oi = __shfl_xor(best_i[nt], 32, 64);
        if (ov > best[nt] || (ov == best[nt] && oi < best_i[nt])) {
            best[nt] = ov;
            best_i[nt] = oi;
        }
        if (half == 0 && col < mr && best_i[nt] != 0x7FFFFFFF)
            atomicMax(&best_packed[cbase + col], pack_best(best[nt], best_i[nt]));
    }
}

__global__ void similarity_clear_kernel(unsigned long long *__restrict__ best_packed, int32_t *__restrict__ cand_cnt,
                                        int64_t total)
{
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < total) {
        best_packed[i] = 0ull;
        cand_cnt[i] = 0;
    }
}

template <typename T, int WM, int WN, int TM, int TN>
static void launch_cfg(hipStream_t s, const PoolDesc &pool, const WorkDesc &w, const HeightDesc &h, const TileTable &tt,
                       float thr_floor, float *dense_s)
{
    const int64_t total = (int64_t)w.G * tt.n_items;
    if (total <= 0)
        return;
    SimArgs A;
    A.G = w.G; A.n = w.n; A.n_slots = w.n_slots; A.r_stride = w.r_stride; A.cand_cap = w.cand_cap; A.P = pool.P;
    A.n_items = tt.n_items;
    A.row_bytes = pool.r * (int)sizeof(T);
    A.thr_floor = thr_floor;
    A.total_s = h.total_s;
    const unsigned grid = (unsigned)(((total + 7) / 8) * 8);
    similarity_kernel<T, WM, WN, TM, TN><<<grid, 64 * WM * WN, 0, s>>>(
        A, (const char *)pool.k, pool.inv_norm_k, w.set_ids, w.set_cnt, tt.node, tt.col0, tt.row0, tt.rows, h.l_off, h.r_off,
        h.l_slot, h.r_slot, h.r_base, h.r_cap, h.s_base, w.best_packed, w.cand_cnt, w.cand_idx, w.cand_val, dense_s);
}

void launch_similarity(hipStream_t s, const PoolDesc &pool, const WorkDesc &w, const HeightDesc &h, float thr_floor,
                       float *dense_s)
{
    const int64_t cols = (int64_t)w.G * w.r_stride;
    if (cols > 0)
        similarity_clear_kernel<<<(unsigned)((cols + 255) / 256), 256, 0, s>>>(w.best_packed, w.cand_cnt, cols);
    const bool big = h.use_big_tiles;
    if (pool.dtype == KVFUSE_BF16) {
        if (big)
            launch_cfg<bf16_t, 4, 2, 2, 4>(s, pool, w, h, h.big, thr_floor, dense_s);
        else
            launch_cfg<bf16_t, 2, 2, 2, 2>(s, pool, w, h, h.small, thr_floor, dense_s);
    } else {
        if (big)
            launch_cfg<float, 4, 2, 2, 4>(s, pool, w, h, h.big, thr_floor, dense_s);
        else
            launch_cfg<float, 2, 2, 2, 2>(s, pool, w, h, h.small, thr_floor, dense_s);
    }
}

}  // namespace kvfuse
