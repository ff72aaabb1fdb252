// a2: similarity of every left block with every right block of a tree node (Algorithm 1: sim <- k_l k_r^T on
// unit vectors, keys only), as a gathered, grouped NT GEMM on the MFMA units.
//
// Rows of both operands are whole KV blocks addressed by physical id, so every gathered row is one contiguous
// r-element run.  The cosine matrix is never written (unless a dense buffer is asked for): the epilogue multiplies
// the fp32 accumulators by the two inverse norms, keeps the column maximum and appends every entry above the
// candidate floor to the column's candidate list.
//
// Work decomposition.  A work item is (group, node, panel of BN right blocks, chunk of up to 4 tiles of BM left
// blocks); one workgroup per item.  Items are numbered so that consecutive ones form a 2-D patch of one node
// (8 panels x several chunks), and hardware workgroup ids are renumbered so that each XCD walks a contiguous range
// of items: the workgroups resident on one XCD then share both their left tiles and their right panels through
// that XCD's L2 instead of each streaming a private panel from HBM.  Column results of different chunks meet in
// global memory through integer atomics only (64-bit max of (ordered cosine, inverted row), 32-bit slot counters),
// so the outcome does not depend on scheduling.
//
// Tiling.  WM x 2 wavefronts, each 2 x TN MFMA tiles of 32 x 32 (v_mfma_f32_32x32x16_bf16, or 4 x
// v_mfma_f32_32x32x2_f32 per 16-byte fragment for f32 pools): 256 x 256 with 8 wavefronts, or 128 x 128 with 4 for
// nodes whose sets are smaller than that.  The MFMA tiles of a wavefront are not adjacent: tile (mt, nt) of every
// wavefront lies in the same 128-row band and 64-column band of the workgroup tile, so on a ragged tile (set sizes
// are data dependent and rarely multiples of 256) all wavefronts drop the same MFMA tiles and finish together.
//
// K is walked in 64-byte slices per row.  A ring of four LDS stages (each BM left + BN right rows x 64 bytes) is
// filled by global_load_lds_dwordx4: the data never passes through registers, so three slices can be on their way
// while one is being multiplied, with no staging registers at all.  Every wavefront issues four such loads per
// slice (1 KB each: 16 rows x 64 bytes).  A load writes LDS at (wave-uniform base + lane * 16), so the XOR swizzle
// that keeps the fragment reads conflict-free (the LDS has 64 four-byte banks) is applied on the global side: lane L
// covers row L / 4 and fetches logical 16-byte chunk (L & 3) ^ ((row >> 2) & 3) of that row's slice.
//
// Fragment reads are ds_read_b128 in inline assembly.  The compiler cannot tell that they never touch a stage
// that is still being filled and would otherwise wait for every outstanding global -> LDS load before each LDS
// read.  Each read's destination registers are handed to the following wait statement as in/out operands, which
// is what orders the MFMAs behind the wait.  Fragments are double buffered (one set per 32-byte half slice).
//
// Iteration j (slice j in stage j & 3):   read set1 <- slice j, second half;  MFMAs on set0 + the 2 right-panel loads
// of slice j + 3;  wait set1;  wait until only this wavefront's last 8 loads are outstanding;  BARRIER;  read set0 <-
// slice j + 1, first half;  MFMAs on set1 + the 2 left-tile loads of slice j + 4 into stage j & 3.
// The one barrier of an iteration sits where two things become true at once: every wavefront holds slice j in
// registers, so stage j & 3 may be overwritten, and every wavefront's loads of slice j + 1 have landed, so it may be
// read.  A load therefore has two to three iterations to arrive (its data is first touched right after the barrier
// of the iteration before its slice), which covers an L2 miss that goes out to memory; with the barrier at the end of
// the iteration the same ring gave it one to two.
#include <type_traits>

#include "common.h"

namespace kvfuse {

typedef float floatx16 __attribute__((ext_vector_type(16)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));


// (cosine, row) packed so that an unsigned 64-bit max picks the larger cosine and, on equal cosines, the lower row.
__device__ __forceinline__ unsigned long long pack_best(float s, int row)
{
    const uint32_t b = __float_as_uint(s);
    const uint32_t ord = (b & 0x80000000u) ? ~b : (b | 0x80000000u);
    return ((unsigned long long)ord << 32) | (unsigned long long)(0xFFFFFFFFu - (uint32_t)row);
}

// Rare path of the epilogue: append (row, cosine) to the
// candidate list of a column; the count is exact even when the list is full.
__device__ __forceinline__ void emit_candidate(int32_t *__restrict__ cand_cnt, int32_t *__restrict__ cand_idx,
                                                         float *__restrict__ cand_val, int64_t column, int cap, int row, float s)
{
    const int slot = atomicAdd(&cand_cnt[column], 1);
    if (slot < cap) {
        cand_idx[column * cap + slot] = row;
        cand_val[column * cap + slot] = s;
    }
}

struct SimArgs {
    int32_t G, n, n_slots, r_stride, cand_cap, P, n_items;
    int32_t row_bytes;             // bytes of one block row
    int32_t nk_screen;             // 64-byte slices of a row that are multiplied: all of them, or a prefix (see PREFIX)
    float thr_floor;
    int64_t total_s;
};

typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

template <typename T> struct MmaV;
template <> struct MmaV<bf16_t> {
    __device__ static __forceinline__ floatx16 run(const u32x4 a, const u32x4 b, floatx16 c)
    {
        return __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a), __builtin_bit_cast(bf16x8, b), c, 0, 0, 0);
    }
};
template <> struct MmaV<float> {
    __device__ static __forceinline__ floatx16 run(const u32x4 a, const u32x4 b, floatx16 c)
    {
        c = __builtin_amdgcn_mfma_f32_32x32x2f32(__uint_as_float(a.x), __uint_as_float(b.x), c, 0, 0, 0);
        c = __builtin_amdgcn_mfma_f32_32x32x2f32(__uint_as_float(a.y), __uint_as_float(b.y), c, 0, 0, 0);
        c = __builtin_amdgcn_mfma_f32_32x32x2f32(__uint_as_float(a.z), __uint_as_float(b.z), c, 0, 0, 0);
        c = __builtin_amdgcn_mfma_f32_32x32x2f32(__uint_as_float(a.w), __uint_as_float(b.w), c, 0, 0, 0);
        return c;
    }
};

// One 64-byte K slice of the fp8 copies in a single instruction: v_mfma_f32_32x32x64_f8f6f4 with both operands e4m3
// (twice the rate of the 16-wide instructions).  A lane supplies 32 bytes per operand, here as two 16-byte fragments;
// any assignment of a row's 64 bytes to (lane half, byte) works as long as both operands use the same one.
typedef int intx8 __attribute__((ext_vector_type(8)));
__device__ __forceinline__ floatx16 mma_q8(const u32x4 al, const u32x4 ah, const u32x4 bl, const u32x4 bh, floatx16 c)
{
    const intx8 a = {(int)al.x, (int)al.y, (int)al.z, (int)al.w, (int)ah.x, (int)ah.y, (int)ah.z, (int)ah.w};
    const intx8 b = {(int)bl.x, (int)bl.y, (int)bl.z, (int)bl.w, (int)bh.x, (int)bh.y, (int)bh.z, (int)bh.w};
    return __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(a, b, c, 0, 0, 0, 0, 0, 0);
}

constexpr int kRingRowTiles = 4;   // most row tiles of one work item (the host's tile table keeps to it)

// BIG: 256 x 256 tile, 8 wavefronts of 64 x 128, one workgroup per compute unit.  Otherwise 128 x 128, 4 wavefronts
// of 64 x 64 and a 64 KB ring, two workgroups per compute unit: for nodes whose sets are smaller than a big tile.
// PREFIX: only the first nk_screen slices of every row are multiplied, and a pair becomes a candidate when an upper
// bound of its cosine clears the floor: cos(a, b) <= <a_head, b_head> / (|a| |b|) + rem_a * rem_b, where rem_x is the
// share of |x| that lies beyond the prefix (Cauchy-Schwarz on the tails; `rem` holds it per block, rounded up).  On
// caches whose unrelated blocks are spread over the whole block length a quarter of the row settles almost every pair;
// every candidate is then evaluated in full in fp64 by the assignment step, so the decisions are the same.
// T = fp8_t (fp8 screen): kpool holds the one-byte copies of the key blocks and q8 what goes with them (Q8Desc in
// common.h): for two blocks the kernel's value <copy_a, copy_b> scale_a scale_b + alpha_a alpha_b is within
// err_a + err_b + err_a err_b of their cosine, so the value plus that is an upper bound of the cosine, listed when it
// clears the floor and evaluated in full by the assignment step like a prefix-screen candidate.  The two bounds add up
// when both shortcuts are on.
template <typename T, bool BIG, bool DENSE, bool PREFIX>
__global__ __launch_bounds__(BIG ? 512 : 256, BIG ? 1 : 2) void similarity_ring_kernel(
    SimArgs A, const char *__restrict__ kpool, const float *__restrict__ inv_norm, const int32_t *__restrict__ set_ids,
    const int32_t *__restrict__ set_cnt, const int4 *__restrict__ dyn_items, const int32_t *__restrict__ dyn_count,
    const int32_t *__restrict__ l_off,
    const int32_t *__restrict__ r_off, const int32_t *__restrict__ l_slot, const int32_t *__restrict__ r_slot,
    const int32_t *__restrict__ r_base, const int32_t *__restrict__ r_cap, const int64_t *__restrict__ s_base,
    unsigned long long *__restrict__ best_packed, int32_t *__restrict__ cand_cnt, int32_t *__restrict__ cand_idx,
    float *__restrict__ cand_val, float *__restrict__ dense_s, const uint8_t *__restrict__ group_enable,
    const float *__restrict__ rem, const Q8Desc q8)
{
    static_assert(!(DENSE && PREFIX), "the dense matrix is the full-length product");
    constexpr bool Q8 = std::is_same<T, fp8_t>::value;
    constexpr int WN = 2, TM = 2, TN = BIG ? 4 : 2, NT = BIG ? 512 : 256, BM = BIG ? 256 : 128, BN = BM;
    constexpr int WM = NT / 64 / WN;          // wavefronts along the rows
    // MFMA tile (mt, nt) of wavefront (wm, wn) covers rows mt * WM * 32 + wm * 32 .. + 31 and columns
    // nt * WN * 32 + wn * 32 .. + 31 of the workgroup tile: the tiles of one index are spread over all wavefronts, so
    // when the valid part of a ragged tile ends early every wavefront can drop the same MFMA tiles and the whole
    // workgroup gets shorter, not just some of its wavefronts.
    constexpr int MT_STRIDE = WM * 32, NT_STRIDE = WN * 32;
    constexpr int HALF = BM / 2;              // rows one pass of the loaders covers (16 per wavefront)
    constexpr int STAGE = (BM + BN) * 64;
    constexpr int B_REGION = BM * 64;
    constexpr int RT = kRingRowTiles;

    __shared__ __attribute__((aligned(1024))) char ring[4 * STAGE];
    __shared__ float lds_invl[RT * BM];      // inverse norms of all left rows of the item; NaN past the end
    __shared__ float lds_invr[BN];
    __shared__ float lds_tcol[BN];
    __shared__ __attribute__((aligned(16))) float lds_reml[PREFIX ? RT * BM : 1];     // PREFIX: tail share of the left rows
    __shared__ float lds_tcolb[PREFIX ? BN : 1];         // PREFIX: tail share of the right blocks / their inverse norm
    __shared__ __attribute__((aligned(16))) float lds_errl[Q8 ? RT * BM : 1];        // Q8: copy error of the left rows
    __shared__ float lds_c1[Q8 ? BN : 1];                // Q8: (1 + copy error of the right block) / its scale
    __shared__ __attribute__((aligned(16))) float lds_all[Q8 ? RT * BM : 1];         // Q8: alpha of the left rows
    __shared__ float lds_alr[Q8 ? BN : 1];               // Q8: alpha of the right blocks
    __shared__ float lds_alrs[Q8 ? BN : 1];              // Q8: the same / the block's scale
    // Largest values over each group of 32 left rows (the rows of one MFMA tile): inverse norm, and what the screens
    // subtract from the floor.  With them one test settles a whole 32 x 32 tile that holds no candidate.
    __shared__ float lds_g_inv[RT * BM / 32];
    __shared__ float lds_g_err[Q8 ? RT * BM / 32 : 1];
    __shared__ float lds_g_al[Q8 ? RT * BM / 32 : 1];
    __shared__ float lds_g_rem[PREFIX ? RT * BM / 32 : 1];
    // The column maximum (best_packed) is a diagnostic: the assignment step works from the candidate lists alone.  It
    // is kept only in the instantiation that also writes the dense matrix; in the production one it cost four of
    // the six vector instructions per accumulator in the epilogue, during which the MFMA units of the CU idle.
    constexpr bool BEST = DENSE && !Q8;      // (no room in LDS for it next to the fp8 screen's arrays)
    __shared__ uint32_t lds_bkey[BEST ? TN : 1][BEST ? NT : 1];
    __shared__ int lds_brt[BEST ? TN : 1][BEST ? NT : 1];
    constexpr int MAXC = (BIG || !Q8) ? 512 : 256;      // (two small fp8 workgroups must fit one compute unit's LDS)
    __shared__ int lds_ncand;
    __shared__ int lds_cand_row[MAXC];
    __shared__ int lds_cand_col[MAXC];
    __shared__ float lds_cand_val[MAXC];

    const int per_xcd = gridDim.x >> 3;
    const long long v = (long long)(blockIdx.x & 7) * per_xcd + (blockIdx.x >> 3);
    if (v >= (long long)A.G * A.n_items)
        return;
    const int g = (int)(v / A.n_items);
    if (group_enable && !group_enable[g])      // a switched-off group keeps empty candidate lists: nothing fuses
        return;
    const int item = (int)(v - (long long)g * A.n_items);
    if (item >= dyn_count[g])
        return;
    const int4 it_rec = dyn_items[(int64_t)g * A.n_items + item];
    const int node = it_rec.x;
    const int col0 = it_rec.y;
    const int row0 = it_rec.z;
    const int ml = set_cnt[(int64_t)g * A.n_slots + l_slot[node]];
    const int mr = set_cnt[(int64_t)g * A.n_slots + r_slot[node]];
    if (col0 >= mr || row0 >= ml)
        return;
    const int row_end = min(ml, row0 + min(it_rec.w, RT * BM));
    const int32_t *__restrict__ l_ids = set_ids + (int64_t)g * A.n + l_off[node];
    const int32_t *__restrict__ r_ids = set_ids + (int64_t)g * A.n + r_off[node];
    const int64_t cbase = (int64_t)g * A.r_stride + r_base[node];

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm = wave / WN, wn = wave % WN;
    const int half = lane >> 5;
    const int64_t row_bytes = A.row_bytes;
    const int nk = A.nk_screen;                               // 64-byte slices walked per row
    const int n_rt = (row_end - row0 + BM - 1) / BM;
    const char *__restrict__ kg = kpool + (int64_t)g * A.P * row_bytes;
    const float *__restrict__ inv_g = inv_norm + (int64_t)g * A.P;

    // ---- global -> LDS loaders: this lane's row within a half tile and its (swizzled) chunk
    const int ld_row = wave * 16 + (lane >> 2);
    const int ld_chunk = ((lane & 3) ^ ((lane >> 4) & 3)) * 16;
#define KVF_LID(t, i) l_ids[min(row0 + (t) * BM + (i) * HALF + ld_row, row_end - 1)]
    const int ia00 = KVF_LID(0, 0), ia01 = KVF_LID(0, 1);
    const int ia10 = KVF_LID(1, 0), ia11 = KVF_LID(1, 1);
    const int ia20 = KVF_LID(2, 0), ia21 = KVF_LID(2, 1);
    const int ia30 = KVF_LID(3, 0), ia31 = KVF_LID(3, 1);
#undef KVF_LID
    const char *pa0 = kg + (int64_t)ia00 * row_bytes + ld_chunk;
    const char *pa1 = kg + (int64_t)ia01 * row_bytes + ld_chunk;
    const char *pb0 = kg + (int64_t)r_ids[min(col0 + ld_row, mr - 1)] * row_bytes + ld_chunk;
    const char *pb1 = kg + (int64_t)r_ids[min(col0 + HALF + ld_row, mr - 1)] * row_bytes + ld_chunk;
    const int dma_a0 = wave * 16 * 64;                          // LDS byte offsets of this wavefront's four 1 KB pieces
    const int dma_a1 = dma_a0 + HALF * 64;
    const int dma_b0 = B_REGION + dma_a0;
    const int dma_b1 = B_REGION + dma_a1;
#define KVF_DMA(PTR, OFF)                                                                                          \
    __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void *)(PTR),                        \
                                     (__attribute__((address_space(3))) void *)(ring + (OFF)), 16, 0, 0)

    // ---- fragment read addresses (LDS byte addresses)
    const uint32_t ring_addr = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) char *)ring;
    const int l31 = lane & 31;
    const uint32_t frag = (uint32_t)(l31 * 64 + ((half ^ ((l31 >> 2) & 3)) * 16));   // first half; second half = ^ 32
    const uint32_t fa_lo = ring_addr + wm * (32 * 64) + frag;
    const uint32_t fb_lo = ring_addr + B_REGION + wn * (32 * 64) + frag;
    const uint32_t fa_hi = fa_lo ^ 32u;
    const uint32_t fb_hi = fb_lo ^ 32u;
#define KVF_DS_READ(DST, ADDR, IMM) asm volatile("ds_read_b128 %0, %1 offset:%2" : "=v"(DST) : "v"(ADDR), "n"(IMM))
#define KVF_WAIT_SET(S)                                                                                            \
    do {                                                                                                           \
        if constexpr (TN > 2)                                                                                      \
            asm volatile("s_waitcnt lgkmcnt(0)"                                                                   \
                         : "+v"(fa0_##S), "+v"(fa1_##S), "+v"(fb0_##S), "+v"(fb1_##S), "+v"(fb2_##S), "+v"(fb3_##S)); \
        else                                                                                                       \
            asm volatile("s_waitcnt lgkmcnt(0)" : "+v"(fa0_##S), "+v"(fa1_##S), "+v"(fb0_##S), "+v"(fb1_##S));     \
    } while (0)
    // The dense-output instantiation (tests only) is short of registers in its epilogue; it waits for each set
    // right away so that no register is ever moved or spilled while its data is still on the way.
#define KVF_READ_SET(S, ADDR_A, ADDR_B)          \
    KVF_DS_READ(fa0_##S, ADDR_A, 0);             \
    KVF_DS_READ(fb0_##S, ADDR_B, 0);             \
    KVF_DS_READ(fa1_##S, ADDR_A, MT_STRIDE * 64); \
    KVF_DS_READ(fb1_##S, ADDR_B, NT_STRIDE * 64); \
    if constexpr (TN > 2) {                      \
        KVF_DS_READ(fb2_##S, ADDR_B, 2 * NT_STRIDE * 64); \
        KVF_DS_READ(fb3_##S, ADDR_B, 3 * NT_STRIDE * 64); \
    }                                            \
    if constexpr (DENSE) { KVF_WAIT_SET(S); }
#define KVF_MMA(S, MT, NTI) acc[MT][NTI] = MmaV<T>::run(fa##MT##_##S, fb##NTI##_##S, acc[MT][NTI]);
    // column tiles 2 and 3 exist only in the big configuration
#define KVF_MMA_HI(S, MT, NTI) if constexpr (TN > 2) { acc[MT][TN > 2 ? NTI : 0] = MmaV<T>::run(fa##MT##_##S, fb##NTI##_##S, acc[MT][TN > 2 ? NTI : 0]); }
    u32x4 fa0_0, fa1_0, fb0_0, fb1_0, fb2_0, fb3_0;
    u32x4 fa0_1, fa1_1, fb0_1, fb1_1, fb2_1, fb3_1;
    // fp8 screen: one MFMA takes a whole 64-byte slice of a row, so the two fragment sets are split by tile instead of
    // by K.  Set 0 = left tile 0 and the first half of the right tiles (p0, p1), set 1 = left tile 1 and the second half
    // (q0, q1), each as a low and a high 16-byte fragment.  MFMA groups of a slice: G1 = tile 0 x p (set 0 only),
    // G2 = tile 0 x q and tile 1 x p (both sets), G3 = tile 1 x q (set 1 only); set 1 is read under G1, the next slice's
    // set 0 under G3, and the barrier sits between G2 and G3 where the other loop has it.
    u32x4 za0l, za0h, zp0l, zp0h, zp1l, zp1h;
    u32x4 za1l, za1h, zq0l, zq0h, zq1l, zq1h;
#define KVF_Q8_WAIT_SET0()                                                                                         \
    do {                                                                                                           \
        if constexpr (TN > 2)                                                                                      \
            asm volatile("s_waitcnt lgkmcnt(0)" : "+v"(za0l), "+v"(za0h), "+v"(zp0l), "+v"(zp0h), "+v"(zp1l), "+v"(zp1h)); \
        else                                                                                                       \
            asm volatile("s_waitcnt lgkmcnt(0)" : "+v"(za0l), "+v"(za0h), "+v"(zp0l), "+v"(zp0h));                 \
    } while (0)
#define KVF_Q8_WAIT_SET1()                                                                                         \
    do {                                                                                                           \
        if constexpr (TN > 2)                                                                                      \
            asm volatile("s_waitcnt lgkmcnt(0)" : "+v"(za1l), "+v"(za1h), "+v"(zq0l), "+v"(zq0h), "+v"(zq1l), "+v"(zq1h)); \
        else                                                                                                       \
            asm volatile("s_waitcnt lgkmcnt(0)" : "+v"(za1l), "+v"(za1h), "+v"(zq0l), "+v"(zq0h));                 \
    } while (0)
#define KVF_Q8_READ_SET0(OFF)                                      \
    KVF_DS_READ(za0l, fa_lo + (OFF), 0);                           \
    KVF_DS_READ(zp0l, fb_lo + (OFF), 0);                           \
    KVF_DS_READ(za0h, fa_hi + (OFF), 0);                           \
    KVF_DS_READ(zp0h, fb_hi + (OFF), 0);                           \
    if constexpr (TN > 2) {                                        \
        KVF_DS_READ(zp1l, fb_lo + (OFF), NT_STRIDE * 64);          \
        KVF_DS_READ(zp1h, fb_hi + (OFF), NT_STRIDE * 64);          \
    }                                                              \
    if constexpr (DENSE) { KVF_Q8_WAIT_SET0(); }
#define KVF_Q8_READ_SET1(OFF)                                      \
    KVF_DS_READ(za1l, fa_lo + (OFF), MT_STRIDE * 64);              \
    KVF_DS_READ(zq0l, fb_lo + (OFF), (TN / 2) * NT_STRIDE * 64);   \
    KVF_DS_READ(za1h, fa_hi + (OFF), MT_STRIDE * 64);              \
    KVF_DS_READ(zq0h, fb_hi + (OFF), (TN / 2) * NT_STRIDE * 64);   \
    if constexpr (TN > 2) {                                        \
        KVF_DS_READ(zq1l, fb_lo + (OFF), (TN / 2 + 1) * NT_STRIDE * 64); \
        KVF_DS_READ(zq1h, fb_hi + (OFF), (TN / 2 + 1) * NT_STRIDE * 64); \
    }                                                              \
    if constexpr (DENSE) { KVF_Q8_WAIT_SET1(); }
    // tile (MT, NTI) from the fragments A (za0 / za1) and B (zp0, zp1, zq0, zq1); tiles of index 1 within a set exist only
    // in the big configuration
#define KVF_Q8_MMA(MT, NTI, A, B) acc[MT][NTI] = mma_q8(A##l, A##h, B##l, B##h, acc[MT][NTI]);
#define KVF_Q8_MMA_HI(MT, NTI, A, B) if constexpr (TN > 2) { acc[MT][TN > 2 ? NTI : 0] = mma_q8(A##l, A##h, B##l, B##h, acc[MT][TN > 2 ? NTI : 0]); }

    // ---- epilogue state
    constexpr uint32_t CODE_MASK = TM * 16 - 1;
    for (int x = tid; x < BN; x += NT) {
        const int col = col0 + x;
        if constexpr (Q8) {
            // The "inverse norm" of a copy is its scale (positive for every block).  The test of a pair,
            //   acc scale_l scale_r + alpha_l alpha_r > floor - err_r - err_l (1 + err_r) [- rem_l rem_r],
            // is taken with everything that belongs to the column divided by scale_r beforehand.
            const int64_t id = (int64_t)g * A.P + r_ids[min(col, mr - 1)];
            const bool ok = col < mr;
            const float eb = ok ? q8.err[id] : 0.0f;
            const float ir = q8.scale[id];
            const float ar = ok ? q8.alpha[id] : 0.0f;
            lds_invr[x] = ok ? ir : 0.0f;
            lds_tcol[x] = ok ? (A.thr_floor - eb) / ir : INFINITY;
            lds_c1[x] = ok ? (1.0f + eb) / ir : 0.0f;
            lds_alr[x] = ar;
            lds_alrs[x] = ar / ir;
            if constexpr (PREFIX)
                lds_tcolb[x] = ok ? rem[id] / ir : 0.0f;
        } else {
            const float ir = col < mr ? inv_g[r_ids[col]] : 0.0f;
            lds_invr[x] = ir;
            lds_tcol[x] = col >= mr ? INFINITY : (ir > 0.0f ? A.thr_floor / ir : (A.thr_floor < 0.0f ? -INFINITY : INFINITY));
            if constexpr (PREFIX)
                lds_tcolb[x] = (col < mr && ir > 0.0f) ? rem[(int64_t)g * A.P + r_ids[col]] / ir : 0.0f;
        }
    }
    static_assert((RT * BM) % NT == 0, "every wavefront takes whole groups of 32 rows");
    for (int x = tid; x < RT * BM; x += NT) {
        const int row = row0 + x;
        float g_inv = 0.0f, g_err = 0.0f, g_al = 0.0f, g_rem = 0.0f;
        if constexpr (Q8) {
            const int64_t id = (int64_t)g * A.P + l_ids[min(row, row_end - 1)];
            if (row < row_end) {
                g_inv = q8.scale[id];
                g_err = q8.err[id];
                g_al = q8.alpha[id];
            }
            lds_invl[x] = row < row_end ? g_inv : __uint_as_float(0x7FC00000u);
            lds_errl[x] = g_err;
            lds_all[x] = g_al;
            g_al = fabsf(g_al);
        } else {
            if (row < row_end)
                g_inv = inv_g[l_ids[row]];
            lds_invl[x] = row < row_end ? g_inv : __uint_as_float(0x7FC00000u);
        }
        if constexpr (PREFIX) {
            if (row < row_end)
                g_rem = rem[(int64_t)g * A.P + l_ids[row]];
            lds_reml[x] = g_rem;
        }
        // maxima over the 32 rows that this half of the wavefront holds
#pragma unroll
        for (int off = 16; off >= 1; off >>= 1) {
            g_inv = fmaxf(g_inv, __shfl_xor(g_inv, off, 64));
            if constexpr (Q8) {
                g_err = fmaxf(g_err, __shfl_xor(g_err, off, 64));
                g_al = fmaxf(g_al, __shfl_xor(g_al, off, 64));
            }
            if constexpr (PREFIX)
                g_rem = fmaxf(g_rem, __shfl_xor(g_rem, off, 64));
        }
        if ((x & 31) == 0) {
            lds_g_inv[x >> 5] = g_inv;
            if constexpr (Q8) {
                lds_g_err[x >> 5] = g_err;
                lds_g_al[x >> 5] = g_al;
            }
            if constexpr (PREFIX)
                lds_g_rem[x >> 5] = g_rem;
        }
    }
    if constexpr (BEST) {
#pragma unroll
        for (int nt = 0; nt < TN; ++nt) {
            lds_bkey[nt][tid] = 0u;
            lds_brt[nt][tid] = 0;
        }
    }
    if (tid == 0)
        lds_ncand = 0;

    floatx16 acc[TM][TN];
#pragma unroll
    for (int mt = 0; mt < TM; ++mt)
#pragma unroll
        for (int nt = 0; nt < TN; ++nt)
#pragma unroll
            for (int e = 0; e < 16; ++e)
                acc[mt][nt][e] = 0.0f;

    // ---- prologue: slices 0, 1, 2 on their way; 0 and 1 landed and visible before the first iteration
    // The A (left) part of a slice is issued half an iteration before its B (right) part, so each part walks the
    // slices with its own counters.  Past the last slice of the last row tile both keep loading rows that exist (the
    // ids of the last row tile, the panel from its start), and those loads are only waited for, never read.
    int pf_kt_a = 0, pf_rt_a = 0, pf_kt_b = 0;
#define KVF_DMA_ADVANCE_A()                                                                                        \
    do {                                                                                                           \
        pa0 += 64; pa1 += 64;                                                                                      \
        if (++pf_kt_a == nk) {                                                                                     \
            pf_kt_a = 0;                                                                                           \
            ++pf_rt_a;                                                                                             \
            const int na0 = pf_rt_a == 1 ? ia10 : (pf_rt_a == 2 ? ia20 : ia30);                                    \
            const int na1 = pf_rt_a == 1 ? ia11 : (pf_rt_a == 2 ? ia21 : ia31);                                    \
            pa0 = kg + (int64_t)na0 * row_bytes + ld_chunk;                                                        \
            pa1 = kg + (int64_t)na1 * row_bytes + ld_chunk;                                                        \
        }                                                                                                          \
    } while (0)
#define KVF_DMA_ADVANCE_B()                                                                                        \
    do {                                                                                                           \
        pb0 += 64; pb1 += 64;                                                                                      \
        if (++pf_kt_b == nk) {                                                                                     \
            pf_kt_b = 0;                                                                                           \
            pb0 -= (int64_t)nk * 64;                                                                               \
            pb1 -= (int64_t)nk * 64;                                                                               \
        }                                                                                                          \
    } while (0)
#pragma unroll 1
    for (int p = 0; p < 3; ++p) {
        const int so = p * STAGE;
        KVF_DMA(pa0, so + dma_a0);
        KVF_DMA(pa1, so + dma_a1);
        KVF_DMA(pb0, so + dma_b0);
        KVF_DMA(pb1, so + dma_b1);
        KVF_DMA_ADVANCE_A();
        KVF_DMA_ADVANCE_B();
    }
    KVF_DMA(pa0, 3 * STAGE + dma_a0);       // the A part of slice 3; its B part follows in the first iteration
    KVF_DMA(pa1, 3 * STAGE + dma_a1);
    KVF_DMA_ADVANCE_A();
    asm volatile("s_waitcnt vmcnt(10)" ::: "memory");     // slice 0 has landed
    __syncthreads();
    if constexpr (Q8) {
        KVF_Q8_READ_SET0(0u)
        KVF_Q8_WAIT_SET0();
    } else {
        KVF_READ_SET(0, fa_lo, fb_lo)
        KVF_WAIT_SET(0);     // nothing but the loop body below runs while fragment reads are on their way
    }

    // One K slice.  M and MH stand for the MFMA statements: the plain ones, or the ones that test whether their
    // tile lies inside the valid part of a ragged workgroup tile.
#define KVF_SLICE(M, MH)                                                                                           \
    do {                                                                                                           \
        const uint32_t cur = (uint32_t)(it & 3) * STAGE;                                                           \
        const uint32_t nxt = (uint32_t)((it + 1) & 3) * STAGE;                                                     \
        const int dst_b = ((it + 3) & 3) * STAGE;                                                                  \
        const int dst_a = (it & 3) * STAGE;                                                                        \
        const uint32_t ra1 = fa_hi + cur, rb1 = fb_hi + cur, ra0 = fa_lo + nxt, rb0 = fb_lo + nxt;                 \
        KVF_WAIT_SET(0);                                                                                           \
        KVF_READ_SET(1, ra1, rb1)                                                                                  \
        __builtin_amdgcn_sched_barrier(0);                                                                         \
        M(0, 0, 0) M(0, 1, 0)                                                                                      \
        __builtin_amdgcn_sched_barrier(0);                                                                         \
        KVF_DMA(pb0, dst_b + dma_b0);                                                                              \
        __builtin_amdgcn_sched_barrier(0);                                                                         \
        M(0, 0, 1) M(0, 1, 1) MH(0, 0, 2) MH(0, 1, 2)                                                              \
        __builtin_amdgcn_sched_barrier(0);                                                                         \
        KVF_DMA(pb1, dst_b + dma_b1);                                                                              \
        __builtin_amdgcn_sched_barrier(0);                                                                         \
        MH(0, 0, 3) MH(0, 1, 3)                                                                                    \
        __builtin_amdgcn_sched_barrier(0);                                                                         \
        KVF_DMA_ADVANCE_B();                                                                                       \
        KVF_WAIT_SET(1);                                                                                           \
        /* Slice it is now in registers in every wavefront that passes the barrier, so its stage is free; and all   \
           but the last 8 loads of this wavefront (slices it + 2 and it + 3) have landed, so slice it + 1 is there. */ \
        asm volatile("s_waitcnt vmcnt(8)\n\ts_barrier" ::: "memory");                                             \
        KVF_READ_SET(0, ra0, rb0)                                                                                  \
        __builtin_amdgcn_sched_barrier(0);                                                                         \
        M(1, 0, 0) M(1, 1, 0)                                                                                      \
        __builtin_amdgcn_sched_barrier(0);                                                                         \
        KVF_DMA(pa0, dst_a + dma_a0);                                                                              \
        __builtin_amdgcn_sched_barrier(0);                                                                         \
        M(1, 0, 1) M(1, 1, 1) MH(1, 0, 2) MH(1, 1, 2)                                                              \
        __builtin_amdgcn_sched_barrier(0);                                                                         \
        KVF_DMA(pa1, dst_a + dma_a1);                                                                              \
        __builtin_amdgcn_sched_barrier(0);                                                                         \
        MH(1, 0, 3) MH(1, 1, 3)                                                                                    \
        __builtin_amdgcn_sched_barrier(0);                                                                         \
        KVF_DMA_ADVANCE_A();                                                                                       \
    } while (0)
    // MFMA tiles that lie wholly outside the valid part are dropped (their accumulators stay zero, which the epilogue
    // treats like any entry below the candidate floor).  Fragment reads and loads stay as they are: every wavefront
    // keeps issuing four loads per slice, which is what the vmcnt arithmetic counts on (leaving out the loads of
    // a wholly invalid half tile as well, with waits that count what was issued, measured slower: the tests and
    // wait variants cost more than the loads).
    const int vcols = mr - col0;
    const bool act_n[4] = {true, vcols > NT_STRIDE, vcols > 2 * NT_STRIDE, vcols > 3 * NT_STRIDE};
#define KVF_MMA_IF(S, MT, NTI) if ((MT == 0 || act_m1) && act_n[NTI]) { KVF_MMA(S, MT, NTI) }
#define KVF_MMA_HI_IF(S, MT, NTI) if ((MT == 0 || act_m1) && act_n[NTI]) { KVF_MMA_HI(S, MT, NTI) }

#define KVF_Q8_MMA_IF(MT, NTI, A, B) if ((MT == 0 || act_m1) && act_n[NTI]) { KVF_Q8_MMA(MT, NTI, A, B) }
#define KVF_Q8_MMA_HI_IF(MT, NTI, A, B) if ((MT == 0 || act_m1) && act_n[TN > 2 ? NTI : 0]) { KVF_Q8_MMA_HI(MT, NTI, A, B) }
    // One K slice of the fp8 screen (same ring, same loads, same barrier as KVF_SLICE).
#define KVF_Q8_SLICE(M, MH)                                                                                        \
    do {                                                                                                           \
        const uint32_t cur = (uint32_t)(it & 3) * STAGE;                                                           \
        const uint32_t nxt = (uint32_t)((it + 1) & 3) * STAGE;                                                     \
        const int dst_b = ((it + 3) & 3) * STAGE;                                                                  \
        const int dst_a = (it & 3) * STAGE;                                                                        \
        KVF_Q8_WAIT_SET0();                                                                                        \
        KVF_Q8_READ_SET1(cur)                                                                                      \
        __builtin_amdgcn_sched_barrier(0);                                                                         \
        M(0, 0, za0, zp0)                                                                                          \
        __builtin_amdgcn_sched_barrier(0);                                                                         \
        KVF_DMA(pb0, dst_b + dma_b0);                                                                              \
        __builtin_amdgcn_sched_barrier(0);                                                                         \
        MH(0, 1, za0, zp1)                                                                                         \
        __builtin_amdgcn_sched_barrier(0);                                                                         \
        KVF_DMA(pb1, dst_b + dma_b1);                                                                              \
        __builtin_amdgcn_sched_barrier(0);                                                                         \
        KVF_DMA_ADVANCE_B();                                                                                       \
        KVF_Q8_WAIT_SET1();                                                                                        \
        M(0, TN / 2, za0, zq0) MH(0, TN / 2 + 1, za0, zq1) M(1, 0, za1, zp0) MH(1, 1, za1, zp1)                    \
        __builtin_amdgcn_sched_barrier(0);                                                                         \
        /* every wavefront that passes the barrier holds slice it in registers, and its loads of slice it + 1 have  \
           landed (all but the last 8 loads of this wavefront, slices it + 2 and it + 3) */                          \
        asm volatile("s_waitcnt vmcnt(8)\n\ts_barrier" ::: "memory");                                             \
        KVF_Q8_READ_SET0(nxt)                                                                                      \
        __builtin_amdgcn_sched_barrier(0);                                                                         \
        M(1, TN / 2, za1, zq0)                                                                                     \
        __builtin_amdgcn_sched_barrier(0);                                                                         \
        KVF_DMA(pa0, dst_a + dma_a0);                                                                              \
        __builtin_amdgcn_sched_barrier(0);                                                                         \
        MH(1, TN / 2 + 1, za1, zq1)                                                                                \
        __builtin_amdgcn_sched_barrier(0);                                                                         \
        KVF_DMA(pa1, dst_a + dma_a1);                                                                              \
        __builtin_amdgcn_sched_barrier(0);                                                                         \
        KVF_DMA_ADVANCE_A();                                                                                       \
    } while (0)

    int it = 0;
    for (int rt = 0; rt < n_rt; ++rt) {
        const bool act_m1 = row_end - (row0 + rt * BM) > MT_STRIDE;
        if constexpr (Q8) {
            if (act_m1 && act_n[TN - 1]) {
#pragma unroll 1
                for (int kt = 0; kt < nk; ++kt, ++it)
                    KVF_Q8_SLICE(KVF_Q8_MMA, KVF_Q8_MMA_HI);
            } else {
#pragma unroll 1
                for (int kt = 0; kt < nk; ++kt, ++it)
                    KVF_Q8_SLICE(KVF_Q8_MMA_IF, KVF_Q8_MMA_HI_IF);
            }
            KVF_Q8_WAIT_SET0();
        } else {
            if (act_m1 && act_n[TN - 1]) {
#pragma unroll 1
                for (int kt = 0; kt < nk; ++kt, ++it)
                    KVF_SLICE(KVF_MMA, KVF_MMA_HI);
            } else {
#pragma unroll 1
                for (int kt = 0; kt < nk; ++kt, ++it)
                    KVF_SLICE(KVF_MMA_IF, KVF_MMA_HI_IF);
            }
            // the prefetched fragments of the next row tile's first slice must be in their registers before anything
            // else may touch them
            KVF_WAIT_SET(0);
        }

        // ---- epilogue of row tile rt
        {
            uint32_t kmax[TN];
            float tcol[TN], tcolb[TN], c1[TN], alrs[TN];
#pragma unroll
            for (int nt = 0; nt < TN; ++nt) {
                kmax[nt] = 0u;
                tcol[nt] = lds_tcol[nt * NT_STRIDE + wn * 32 + (lane & 31)];
                tcolb[nt] = PREFIX ? lds_tcolb[nt * NT_STRIDE + wn * 32 + (lane & 31)] : 0.0f;
                c1[nt] = Q8 ? lds_c1[nt * NT_STRIDE + wn * 32 + (lane & 31)] : 0.0f;
                alrs[nt] = Q8 ? lds_alrs[nt * NT_STRIDE + wn * 32 + (lane & 31)] : 0.0f;
            }
#pragma unroll
            for (int mt = 0; mt < TM; ++mt) {
                // One test per 32 x 32 tile first: no entry of this lane's column can clear its floor if the largest
                // accumulator (or 0) times the largest inverse norm of the 32 rows stays below the floor lowered by
                // the largest corrections of the 32 rows.  Candidates are rare, so this is all most tiles cost.
                bool look[TN];
                bool any_look = false;
                {
                    const int grp = (rt * BM + mt * MT_STRIDE + wm * 32) >> 5;
                    const float gi = lds_g_inv[grp];
                    const float ge = Q8 ? lds_g_err[grp] : 0.0f, ga = Q8 ? lds_g_al[grp] : 0.0f;
                    const float gr = PREFIX ? lds_g_rem[grp] : 0.0f;
#pragma unroll
                    for (int nt = 0; nt < TN; ++nt) {
                        float mx = 0.0f;
#pragma unroll
                        for (int e = 0; e < 16; e += 2)
                            mx = fmaxf(fmaxf(acc[mt][nt][e], acc[mt][nt][e + 1]), mx);
                        float low = tcol[nt];
                        if constexpr (Q8) {
                            low = fmaf(-ge, c1[nt], low);
                            low = fmaf(-ga, fabsf(alrs[nt]), low);
                        }
                        if constexpr (PREFIX)
                            low = fmaf(-gr, tcolb[nt], low);
                        // (the binary32 roundings of this line and of the exact test differ by parts in 10^7; the factor
                        // covers them, and the floor sits a whole band below anything that has to be listed)
                        look[nt] = DENSE || !(mx * gi * (1.0f + 1e-6f) < low);      // (the diagnostic instance looks at everything)
                        any_look |= look[nt];
                    }
                }
                if (any_look) {
#pragma unroll
                for (int eg = 0; eg < 4; ++eg) {
                    const int rl0 = mt * MT_STRIDE + wm * 32 + eg * 8 + half * 4;
                    const float4 il4 = *reinterpret_cast<const float4 *>(&lds_invl[rt * BM + rl0]);
                    const float il[4] = {il4.x, il4.y, il4.z, il4.w};
                    float rl[4] = {0.0f, 0.0f, 0.0f, 0.0f};
                    if constexpr (PREFIX) {
                        const float4 rl4 = *reinterpret_cast<const float4 *>(&lds_reml[rt * BM + rl0]);
                        rl[0] = rl4.x; rl[1] = rl4.y; rl[2] = rl4.z; rl[3] = rl4.w;
                    }
                    float el[4] = {0.0f, 0.0f, 0.0f, 0.0f}, al[4] = {0.0f, 0.0f, 0.0f, 0.0f};
                    if constexpr (Q8) {
                        const float4 el4 = *reinterpret_cast<const float4 *>(&lds_errl[rt * BM + rl0]);
                        el[0] = el4.x; el[1] = el4.y; el[2] = el4.z; el[3] = el4.w;
                        const float4 al4 = *reinterpret_cast<const float4 *>(&lds_all[rt * BM + rl0]);
                        al[0] = al4.x; al[1] = al4.y; al[2] = al4.z; al[3] = al4.w;
                    }
#pragma unroll
                    for (int nt = 0; nt < TN; ++nt) {
                        if (!look[nt])
                            continue;
                        float t[4], lim[4];
                        bool hit = false;
#pragma unroll
                        for (int q = 0; q < 4; ++q) {
                            t[q] = acc[mt][nt][eg * 4 + q] * il[q];
                            // the floor of this pair, lowered by what the unseen tails could add at most (rem is rounded up with a
                            // margin far above the rounding of this line)
                            lim[q] = tcol[nt];
                            if constexpr (Q8) {         // the copies' errors: - err_a (1 + err_b); - err_b is in tcol;
                                lim[q] = fmaf(-el[q], c1[nt], lim[q]);      // and the part of the cosine that lies along
                                lim[q] = fmaf(-al[q], alrs[nt], lim[q]);    // the common direction moves over to this side
                            }
                            if constexpr (PREFIX)
                                lim[q] = fmaf(-rl[q], tcolb[nt], lim[q]);
                            hit |= t[q] > lim[q];
                            if constexpr (BEST) {
                                const uint32_t key = (__float_as_uint(fmaxf(t[q], 0.0f)) & ~CODE_MASK) |
                                                     (CODE_MASK - (uint32_t)(mt * 16 + eg * 4 + q));
                                kmax[nt] = max(kmax[nt], key);
                            }
                        }
                        if (hit) {      // rare: an entry clears the candidate floor
                            const int cl = nt * NT_STRIDE + wn * 32 + (lane & 31);
#pragma unroll
                            for (int q = 0; q < 4; ++q)
                                if (t[q] > lim[q]) {
                                    const int row = row0 + rt * BM + rl0 + q;
                                    float sv = t[q] * lds_invr[cl];
                                    if constexpr (Q8)
                                        sv = fmaf(al[q], lds_alr[cl], sv);
                                    const int k = atomicAdd(&lds_ncand, 1);
                                    if (k < MAXC) {
                                        lds_cand_row[k] = row;
                                        lds_cand_col[k] = cl;
                                        lds_cand_val[k] = sv;
                                    } else {
                                        emit_candidate(cand_cnt, cand_idx, cand_val, cbase + col0 + cl, A.cand_cap, row, sv);
                                    }
                                }
                        }
                    }
                }
                }
                __builtin_amdgcn_sched_barrier(0);
            }
            if constexpr (DENSE) {
#pragma unroll
                for (int mt = 0; mt < TM; ++mt)
#pragma unroll
                    for (int nt = 0; nt < TN; ++nt)
#pragma unroll
                        for (int e = 0; e < 16; ++e) {
                            const int rl = mt * MT_STRIDE + wm * 32 + (e >> 2) * 8 + half * 4 + (e & 3);
                            const int row = row0 + rt * BM + rl;
                            const int col = col0 + nt * NT_STRIDE + wn * 32 + (lane & 31);
                            if (row < row_end && col < mr) {
                                float sv = acc[mt][nt][e] * lds_invl[rt * BM + rl] * lds_invr[nt * NT_STRIDE + wn * 32 + (lane & 31)];
                                if constexpr (Q8)
                                    sv = fmaf(lds_all[rt * BM + rl], lds_alr[nt * NT_STRIDE + wn * 32 + (lane & 31)], sv);
                                dense_s[(int64_t)g * A.total_s + s_base[node] + (int64_t)row * r_cap[node] + col] = sv;
                            }
                        }
            }
#pragma unroll
            for (int nt = 0; nt < TN; ++nt) {
                if constexpr (BEST) {
                    if (kmax[nt] > lds_bkey[nt][tid]) {
                        lds_bkey[nt][tid] = kmax[nt];
                        lds_brt[nt][tid] = rt;
                    }
                }
#pragma unroll
                for (int mt = 0; mt < TM; ++mt)
#pragma unroll
                    for (int e = 0; e < 16; ++e)
                        acc[mt][nt][e] = 0.0f;
            }
        }
    }
    // loads past the last slice are still on their way into the ring; nothing may leave before they land
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __syncthreads();

    {
        const int nc = min(lds_ncand, MAXC);
        for (int k = tid; k < nc; k += NT)
            emit_candidate(cand_cnt, cand_idx, cand_val, cbase + col0 + lds_cand_col[k], A.cand_cap, lds_cand_row[k],
                           lds_cand_val[k]);
    }
    if constexpr (BEST) {
#pragma unroll
        for (int nt = 0; nt < TN; ++nt) {
            const int col = col0 + nt * NT_STRIDE + wn * 32 + (lane & 31);
            const uint32_t bkey = lds_bkey[nt][tid];
            const int code = (int)(CODE_MASK - (bkey & CODE_MASK));
            const int row = min(row_end - 1, row0 + lds_brt[nt][tid] * BM + (code >> 4) * MT_STRIDE + wm * 32 + ((code & 15) >> 2) * 8 + half * 4 + (code & 3));
            unsigned long long pk = bkey ? pack_best(__uint_as_float(bkey & ~CODE_MASK) * lds_invr[nt * NT_STRIDE + wn * 32 + (lane & 31)], row) : 0ull;
            const unsigned long long other = __shfl_xor(pk, 32, 64);
            pk = other > pk ? other : pk;
            if (half == 0 && col < mr && pk)
                atomicMax(&best_packed[cbase + col], pk);
        }
    }
#undef KVF_DMA
#undef KVF_DS_READ
#undef KVF_READ_SET
#undef KVF_WAIT_SET
#undef KVF_MMA
#undef KVF_MMA_HI
#undef KVF_DMA_ADVANCE_A
#undef KVF_DMA_ADVANCE_B
#undef KVF_SLICE
#undef KVF_MMA_IF
#undef KVF_MMA_HI_IF
#undef KVF_Q8_WAIT_SET0
#undef KVF_Q8_WAIT_SET1
#undef KVF_Q8_READ_SET0
#undef KVF_Q8_READ_SET1
#undef KVF_Q8_MMA
#undef KVF_Q8_MMA_HI
#undef KVF_Q8_MMA_IF
#undef KVF_Q8_MMA_HI_IF
#undef KVF_Q8_SLICE
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

// The work items of a height, laid out from the sizes the sets have NOW (they shrink as blocks fuse; the plan only knows
// their capacities).  An item covers one panel of BN right blocks x up to 4 row tiles of BM left blocks of a node: a node
// with c panels and a row tiles is cut into row chunks of rt = min(ceil(a / 4), 4) tiles, and its items are ordered in
// patches of 8 panels x all row chunks, row chunk by row chunk within a patch.  The 32 workgroups that an XCD runs at a
// time are then one patch (or what is left of a node and the start of the next): they start together, do equal work,
// and share 8 panels and at most 4 row chunks in that XCD's L2.  Laid out from the capacities instead, a third of the
// items of an upper height had nothing to do, ended at once and let the patches of an XCD drift apart.
__device__ __forceinline__ int items_of_node(int ml, int mr, int bm, int bn, int &n_cp, int &rt, int &n_rc)
{
    n_cp = (mr + bn - 1) / bn;
    const int n_rtile = (ml + bm - 1) / bm;
    rt = min((n_rtile + 3) / 4, 4);

    n_rc = rt > 0 ? (n_rtile + rt - 1) / rt : 0;
    return n_cp * n_rc;
}

// First item of every node of a group (exclusive scan over the nodes) and the group's number of items.
__global__ __launch_bounds__(256) void items_count_kernel(WorkDesc w, HeightDesc h, int bm, int bn)
{
    __shared__ int64_t lds4[4];
    const int g = blockIdx.x, tid = threadIdx.x;
    int32_t *base = w.dyn_base + (int64_t)g * w.dyn_stride;
    int64_t run = 0;
    for (int k0 = 0; k0 < h.n_nodes; k0 += 256) {
        const int k = k0 + tid;
        int c = 0;
        if (k < h.n_nodes) {
            int n_cp, rt, n_rc;
            c = items_of_node(w.set_cnt[(int64_t)g * w.n_slots + h.l_slot[k]], w.set_cnt[(int64_t)g * w.n_slots + h.r_slot[k]], bm, bn,
                              n_cp, rt, n_rc);
        }
        int64_t total;
        const int64_t pre = block_exscan_256((int64_t)c, lds4, total);
        if (k < h.n_nodes)
            base[k] = (int)min(run + pre, (int64_t)h.item_cap);
        run += total;
        __syncthreads();
    }
    if (tid == 0) {
        base[h.n_nodes] = (int)min(run, (int64_t)h.item_cap);
        w.dyn_count[g] = (int)min(run, (int64_t)h.item_cap);      // (never more than the room: see the plan's bound)
    }
}

// One thread per item slot: which node it falls into, and which panel and row chunk of that node it is.
__global__ __launch_bounds__(256) void items_fill_kernel(WorkDesc w, HeightDesc h, int bm, int bn)
{
    const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (i >= (int64_t)w.G * h.item_cap)
        return;
    const int g = (int)(i / h.item_cap);
    const int item = (int)(i - (int64_t)g * h.item_cap);
    if (item >= w.dyn_count[g])
        return;
    const int32_t *base = w.dyn_base + (int64_t)g * w.dyn_stride;
    int lo = 0, hi = h.n_nodes;             // the last node whose first item is <= item (empty nodes share a first item
    while (hi - lo > 1) {                   // with their successor and are skipped by taking the last)
        const int mid = (lo + hi) >> 1;
        if (base[mid] <= item)
            lo = mid;
        else
            hi = mid;
    }
    const int k = lo;
    int n_cp, rt, n_rc;
    (void)items_of_node(w.set_cnt[(int64_t)g * w.n_slots + h.l_slot[k]], w.set_cnt[(int64_t)g * w.n_slots + h.r_slot[k]], bm, bn, n_cp,
                        rt, n_rc);
    const int local = item - base[k];
    const int patch = local / (8 * n_rc);
    const int within = local - patch * 8 * n_rc;
    const int np = min(8, n_cp - 8 * patch);
    const int rc = within / np;
    const int cp = 8 * patch + within - rc * np;
    w.dyn_items[(int64_t)g * h.item_cap + item] = make_int4(k, cp * bn, rc * rt * bm, rt * bm);
}

template <typename T, bool BIG>
static void launch_ring(hipStream_t s, const PoolDesc &pool, const WorkDesc &w, const HeightDesc &h, float thr_floor, float *dense_s)
{
    const int64_t total = (int64_t)w.G * h.item_cap;
    if (total <= 0)
        return;
    {
        const int bm = BIG ? 256 : 128;
        items_count_kernel<<<w.G, 256, 0, s>>>(w, h, bm, bm);
        items_fill_kernel<<<(unsigned)((total + 255) / 256), 256, 0, s>>>(w, h, bm, bm);
    }
    SimArgs A;
    A.G = w.G; A.n = w.n; A.n_slots = w.n_slots; A.r_stride = w.r_stride; A.cand_cap = w.cand_cap; A.P = pool.P;
    A.n_items = h.item_cap;
    A.row_bytes = pool.r * (int)sizeof(T);
    const bool prefix = !dense_s && w.screen_prefix > 0 && w.screen_prefix < pool.r;
    const char *kpool = std::is_same<T, fp8_t>::value ? (const char *)w.q8.k : (const char *)pool.k;
    A.nk_screen = (prefix ? w.screen_prefix * (int)sizeof(T) : A.row_bytes) >> 6;
    A.thr_floor = thr_floor;
    A.total_s = h.total_s;
    const unsigned grid = (unsigned)(((total + 7) / 8) * 8);
#define KVF_SIM_LAUNCH(D, PF)                                                                                          \
    similarity_ring_kernel<T, BIG, D, PF><<<grid, BIG ? 512 : 256, 0, s>>>(                                                             \
        A, kpool, pool.inv_norm_k, w.set_ids, w.set_cnt, w.dyn_items, w.dyn_count, h.l_off, h.r_off, \
        h.l_slot, h.r_slot, h.r_base, h.r_cap, h.s_base, w.best_packed, w.cand_cnt, w.cand_idx, w.cand_val, dense_s,           \
        w.group_enable, w.rem_k, w.q8)
    if (dense_s)
        KVF_SIM_LAUNCH(true, false);
    else if (prefix)
        KVF_SIM_LAUNCH(false, true);
    else
        KVF_SIM_LAUNCH(false, false);
#undef KVF_SIM_LAUNCH
}


void launch_similarity(hipStream_t s, const PoolDesc &pool, const WorkDesc &w, const HeightDesc &h, float thr_floor,
                       float *dense_s)
{
    const int64_t cols = (int64_t)w.G * w.r_stride;
    if (cols > 0)
        similarity_clear_kernel<<<(unsigned)((cols + 255) / 256), 256, 0, s>>>(w.best_packed, w.cand_cnt, cols);
    const bool big = h.use_big_tiles;
    if (w.q8.k) {
        if (big)
            launch_ring<fp8_t, true>(s, pool, w, h, thr_floor, dense_s);
        else
            launch_ring<fp8_t, false>(s, pool, w, h, thr_floor, dense_s);
    } else if (pool.dtype == KVFUSE_BF16) {
        if (big)
            launch_ring<bf16_t, true>(s, pool, w, h, thr_floor, dense_s);
        else
            launch_ring<bf16_t, false>(s, pool, w, h, thr_floor, dense_s);
    } else {
        if (big)
            launch_ring<float, true>(s, pool, w, h, thr_floor, dense_s);
        else
            launch_ring<float, false>(s, pool, w, h, thr_floor, dense_s);
    }
}

}  // namespace kvfuse
