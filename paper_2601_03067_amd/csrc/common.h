// Internal declarations shared by the kvfuse HIP sources (gfx950 only).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include <string>
#include <vector>

#include "../../include/kvfuse.h"

namespace kvfuse {

// ---------------------------------------------------------------------------------------------------
// host side
// ---------------------------------------------------------------------------------------------------

struct Ctx {
    int device = 0;
    hipStream_t stream = nullptr;
    std::string err;
    hipEvent_t ev[16] = {};
    bool ev_ready = false;
    // second stream (default priority) and fork / join events for launches that may overlap; made on first use
    hipStream_t aux = nullptr;
    hipEvent_t fork = nullptr, join = nullptr;
};

int fail(Ctx *c, int code, const std::string &msg);

#define KVF_HIP(ctx, expr)                                                                        \
    do {                                                                                          \
        hipError_t e__ = (expr);                                                                  \
        if (e__ != hipSuccess)                                                                    \
            return ::kvfuse::fail((ctx), KVFUSE_EHIP, std::string(#expr) + ": " + hipGetErrorString(e__)); \
    } while (0)

}  // namespace kvfuse

// the opaque context of the C ABI
struct kvfuse_ctx {
    kvfuse::Ctx c;
};

namespace kvfuse {

// Tables of one tree height, all device pointers into the plan workspace (identical for every group).
struct HeightDesc {
    int32_t n_nodes;
    int32_t total_l_cap, total_r_cap;
    const int32_t *l_off, *r_off, *l_slot, *r_slot, *out_slot, *l_cap, *r_cap;
    const int32_t *l_base, *r_base;   // [n_nodes + 1] prefix sums of the capacities
    const int64_t *s_base;            // [n_nodes + 1] prefix sums of l_cap * r_cap
    int32_t item_cap;                 // most similarity work items one group can have at this height (see similarity.hip)
    bool use_big_tiles;
    int64_t total_s;
};

// fp8 screen.  With u = block / |block| and, when a direction m of the group is given, u_c = u - alpha m (alpha the
// binary32 value stored here; without a direction alpha = 0 and u_c = u):
//   k      [G][P][r]  e4m3(u_c * kQ8Scale / |u_c|), one byte per element
//   scale  [G][P]     |u_c| / kQ8Scale: decoded bytes * scale reconstruct u_c
//   alpha  [G][P]
//   err    [G][P]     |u_c - decoded bytes * scale| + what the exact identity <u, v> = <u_c, v_c> + alpha_u alpha_v loses
//                     because m is not exactly unit and alpha is rounded, rounded up: for two blocks
//                     |<u, v> - (<copy_u, copy_v> scale_u scale_v + alpha_u alpha_v)| <= err_u + err_v + err_u err_v
//   dir    [G][r]     m, or null
struct Q8Desc {
    uint8_t *k;
    float *err, *scale, *alpha, *dir;
};

// Group-strided work arrays of a plan (device).
struct WorkDesc {
    int32_t G, n, n_slots, r_stride, l_stride, cand_cap;
    int32_t *set_ids;    // [G][n]
    int32_t *set_cnt;    // [G][n_slots]
    int32_t *assign;     // [G][r_stride]
    unsigned long long *best_packed;   // [G][r_stride] (ordered cosine << 32) | (0xFFFFFFFF - row); 0 = none
    int32_t *cand_cnt;   // [G][r_stride]
    int32_t *cand_idx;   // [G][r_stride][cand_cap]
    float *cand_val;     // [G][r_stride][cand_cap]
    int32_t *seg_cnt;    // [G][l_stride]
    int32_t *seg_ptr;    // [G][l_stride]
    int32_t *seg_members;// [G][r_stride]
    int4 *active;        // [G * l_stride][2] merge work list, 32 bytes per target: (group, target's physical id,
                         // member count, index of the first member in seg_members), (physical ids of the first
                         // two members, unused, unused) -- the merge kernel starts its block loads straight from it
    int32_t *seg_slot;   // [G][l_stride] position of a target in the work list
    int32_t *n_active;   // [max_heights]
    int32_t *refine;     // [G * r_stride][2] columns that need the fp64 re-check: (g * r_stride + c, node)
    int32_t *n_refine;   // [max_heights]
    int32_t *counters;   // [G][8]: 0 fused, 1 near-threshold, 2 refined, 3 candidate overflow, 4 invalid ids, 5 entries of shared blocks
    const uint8_t *group_enable;   // [G] or null: groups with 0 are skipped by the similarity step (nothing fuses)
    int32_t *leaf_src;   // [n] position in a set_ids row -> logical entry the leaf step fills it from, -1 = none
    float *rem_k;        // [G][P] prefix screen: share of each key block's norm that lies beyond the prefix, rounded up
    int32_t screen_prefix;   // elements of every block the similarity screen multiplies; 0 = the whole block
    // similarity work items of the current height, built on the device from the sets' sizes (similarity.hip):
    int4 *dyn_items;     // [G][item_cap of the height] node, first column, first row, rows
    int32_t *dyn_base;   // [G][dyn_stride] first item of every node, and the total
    int32_t *dyn_count;  // [G]
    int32_t dyn_stride;
    Q8Desc q8;           // fp8 screen: the one-byte copies of the key blocks and what goes with them; q8.k null = off
};

// fp8 screen: unit key vectors are multiplied by this before conversion to e4m3 (largest finite value 448), which puts
// the elements of a typical block (around r^-1/2) in the middle of the format's normal range.
constexpr float kQ8Scale = 256.0f;

struct PoolDesc {
    void *k, *v;
    int32_t dtype, G, P, r, t, d;
    double *norm_k, *norm_v;
    float *inv_norm_k;
};

struct TableDesc {
    int32_t n;
    int32_t *bt;
    float *scale_k, *scale_v;
    double *orig_norm_k, *orig_norm_v;
    int32_t *refcount, *remap;
};

static inline PoolDesc to_desc(const kvfuse_pool &p)
{
    return PoolDesc{p.k, p.v, p.dtype, p.G, p.P, p.t * p.d, p.t, p.d, p.norm_k, p.norm_v, p.inv_norm_k};
}
static inline TableDesc to_desc(const kvfuse_table &t)
{
    return TableDesc{t.n, t.bt, t.scale_k, t.scale_v, t.orig_norm_k, t.orig_norm_v, t.refcount, t.remap};
}

// Workgroups of `threads` threads of `kernel` that the current device holds at once: the size of a persistent grid
// (a workgroup that had to wait for a free slot would start its share of the work when the others are nearly done).
// Asked once per kernel.
template <typename K> static int resident_workgroups(K kernel, int threads = 256)
{
    static int cached = 0;
    if (cached <= 0) {
        int per_cu = 0, dev = 0, cus = 0;
        if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, kernel, threads, 0) != hipSuccess || per_cu <= 0)
            per_cu = 2;
        if (hipGetDevice(&dev) != hipSuccess || hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess ||
            cus <= 0)
            cus = 256;
        cached = per_cu * cus;
    }
    return cached;
}

// launchers, one per source file
void launch_block_norms(hipStream_t s, const PoolDesc &pool, const TableDesc &tab, float *rem = nullptr, int prefix = 0,
                        const Q8Desc *q8 = nullptr);
// fp8 screen: the direction of every group that its key blocks are centred on (no-op unless one is asked for)
void launch_centre_direction(hipStream_t s, const PoolDesc &pool, const WorkDesc &w);
void launch_leaf_sets(hipStream_t s, const WorkDesc &w, const TableDesc &tab, int P, const int32_t *slot_init, const double *norm_k);
void launch_similarity(hipStream_t s, const PoolDesc &pool, const WorkDesc &w, const HeightDesc &h, float thr_floor,
                       float *dense_s);
void launch_assign(hipStream_t s, const PoolDesc &pool, const TableDesc &tab, const WorkDesc &w, const HeightDesc &h,
                   int height, double thr, double band, int rule);
void launch_merge(hipStream_t s, const PoolDesc &pool, const WorkDesc &w, const HeightDesc &h, int height);
// prefix screen: tail shares of all key blocks (for callers that run the steps one by one)
void launch_prefix_tails(hipStream_t s, const PoolDesc &pool, const WorkDesc &w);
// fp8 screen: the e4m3 copy and its error for all key blocks, and for the targets the merge step of a height rebuilt
void launch_quantise_all(hipStream_t s, const PoolDesc &pool, const WorkDesc &w);
void launch_quantise_targets(hipStream_t s, const PoolDesc &pool, const WorkDesc &w, int height);
void launch_rewrite(hipStream_t s, const PoolDesc &pool, const TableDesc &tab, int32_t *free_list, int32_t *n_free,
                    int32_t *n_phys);
size_t decode_workspace_bytes(int n_layers, int B, int Hq, int kv_heads, int d, int max_blocks);
int launch_decode(hipStream_t s, const PoolDesc &pool, const TableDesc &tab, int kv_heads, int layer_begin, int n_layers,
                  const void *q, const int32_t *req_start, const int32_t *ctx_len, int B, int Hq, int max_blocks,
                  float sm_scale, void *workspace, size_t workspace_bytes, float *out, bool all_heads = false);

// threshold statistics (threshold.hip)
void launch_pair_cosines(hipStream_t s, const PoolDesc &pool, const TableDesc &tab, const int32_t *pairs, int n_pairs,
                         double *cos_out);
void launch_cosine_moments(hipStream_t s, const double *cos_in, int G, int n_pairs, double *moments);

// ---------------------------------------------------------------------------------------------------
// device side
// ---------------------------------------------------------------------------------------------------
#if defined(__HIPCC__)

typedef uint16_t bf16_t;   // raw bfloat16 bits
struct fp8_t { uint8_t bits; };   // element type of the fp8 screen copy (OCP e4m3)

__device__ __forceinline__ float bf16_to_f32(uint32_t bits16) { return __uint_as_float(bits16 << 16); }

// 16 bytes of pool data widened to fp64: 8 bfloat16 or 4 float values.
template <typename T> struct Elem;
template <> struct Elem<bf16_t> {
    static constexpr int PER16 = 8;
    __device__ static __forceinline__ void widen(const uint4 &raw, double *out)
    {
        const uint32_t w[4] = {raw.x, raw.y, raw.z, raw.w};
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            out[2 * i] = (double)__uint_as_float(w[i] << 16);
            out[2 * i + 1] = (double)__uint_as_float(w[i] & 0xFFFF0000u);
        }
    }
};
template <> struct Elem<float> {
    static constexpr int PER16 = 4;
    __device__ static __forceinline__ void widen(const uint4 &raw, double *out)
    {
        out[0] = (double)__uint_as_float(raw.x);
        out[1] = (double)__uint_as_float(raw.y);
        out[2] = (double)__uint_as_float(raw.z);
        out[3] = (double)__uint_as_float(raw.w);
    }
};

// Sum over the 64 lanes of a wavefront in a fixed butterfly order; every lane gets the result.
__device__ __forceinline__ double wave_sum(double x)
{
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1)
        x += __shfl_xor(x, off, 64);
    return x;
}

// Sum over a 256-thread workgroup in a fixed order (wave butterflies, then waves 0..3 left to right).
__device__ __forceinline__ double block_sum_256(double x, double *lds4)
{
    x = wave_sum(x);
    __syncthreads();
    if ((threadIdx.x & 63) == 0)
        lds4[threadIdx.x >> 6] = x;
    __syncthreads();
    return ((lds4[0] + lds4[1]) + lds4[2]) + lds4[3];
}

// Exclusive scan of one int64 per thread over a 256-thread workgroup; returns the exclusive prefix and the total.
__device__ __forceinline__ int64_t block_exscan_256(int64_t x, int64_t *lds4, int64_t &total)
{
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    int64_t inc = x;
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) {
        const int64_t y = __shfl_up(inc, off, 64);
        if (lane >= off)
            inc += y;
    }
    __syncthreads();
    if (lane == 63)
        lds4[wave] = inc;
    __syncthreads();
    int64_t pre = 0;
    for (int k = 0; k < wave; ++k)
        pre += lds4[k];
    total = lds4[0] + lds4[1] + lds4[2] + lds4[3];
    return pre + inc - x;
}

// Prefix screen: share of a block's norm that lies beyond the prefix, from the sum of the tail squares and the norm,
// rounded up to float with an absolute margin (the similarity kernel multiplies two of these into an upper bound).
__device__ __forceinline__ float tail_share(double tail_squares, double norm)
{
    return norm > 0.0 ? __double2float_ru(fmin(sqrt(fmax(tail_squares, 0.0)) / norm, 1.0) + 1e-6) : 0.0f;
}

// fp8 screen: the parameters of one block's copy.  With u_c,i = x_i / |x| - alpha m_i and `scale` the binary32 value
// stored as the block's scale, the byte of element i is e4m3(t_i), t_i = x_i * a - b * m_i in binary32 with
// a = 1 / (|x| scale) and b = alpha / scale, so that decoded byte * scale reconstructs u_c,i.  `wide` marks a block
// whose norm is so small that a leaves binary32's range: its copy is zeros with a vacuous error.
struct Q8Block {
    float a, b;
    double alpha, scale;
    bool wide;
};

// 16 bytes of pool data as binary32 (exact for both pool types).
template <typename T> __device__ __forceinline__ void widen_f32(const uint4 &raw, float *out);
template <> __device__ __forceinline__ void widen_f32<bf16_t>(const uint4 &raw, float *out)
{
    const uint32_t w[4] = {raw.x, raw.y, raw.z, raw.w};
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        out[2 * i] = __uint_as_float(w[i] << 16);
        out[2 * i + 1] = __uint_as_float(w[i] & 0xFFFF0000u);
    }
}
template <> __device__ __forceinline__ void widen_f32<float>(const uint4 &raw, float *out)
{
    out[0] = __uint_as_float(raw.x);
    out[1] = __uint_as_float(raw.y);
    out[2] = __uint_as_float(raw.z);
    out[3] = __uint_as_float(raw.w);
}

// <m, x> over one 16-byte piece of a block (PER16 elements from element offset e0), in fp64: alpha must be <m, u> to
// binary32 rounding for the identity behind the centred copies to hold as closely as quantise_error assumes.
template <typename T>
__device__ __forceinline__ void q8_dir_dot_chunk(const uint4 &raw, const float *__restrict__ dir_g, int e0, double &sm)
{
    constexpr int PER = Elem<T>::PER16;
    float x[PER];
    widen_f32<T>(raw, x);
#pragma unroll
    for (int i = 0; i < PER / 4; ++i) {
        const float4 f = *reinterpret_cast<const float4 *>(dir_g + e0 + 4 * i);
        sm = fma((double)f.x, (double)x[4 * i], sm);
        sm = fma((double)f.y, (double)x[4 * i + 1], sm);
        sm = fma((double)f.z, (double)x[4 * i + 2], sm);
        sm = fma((double)f.w, (double)x[4 * i + 3], sm);
    }
}

// One piece to e4m3 (the hardware's nearest-even conversion) and, in se, the squared distance between t and the bytes
// decoded with the hardware's own conversion, in units of the scale.  All in binary32: t_i * scale differs from the
// exact u_c,i by at most 2^-24 (|x_i| / |x| + 2 |alpha m_i| + |u_c,i|) (the roundings of a, b, b * m_i and the
// multiply-add), 2.4e-7 over a block in the Euclidean norm; quantise_error's margin covers it.
template <typename T>
__device__ __forceinline__ void quantise_chunk(const uint4 &raw, const float *__restrict__ dir_g, int e0, const Q8Block &p,
                                               uint8_t *__restrict__ dst, float &se)
{
    constexpr int PER = Elem<T>::PER16;
    float x[PER], t[PER];
    widen_f32<T>(raw, x);
    if (dir_g) {
#pragma unroll
        for (int i = 0; i < PER / 4; ++i) {
            const float4 f = *reinterpret_cast<const float4 *>(dir_g + e0 + 4 * i);
            t[4 * i] = fmaf(x[4 * i], p.a, -(p.b * f.x));
            t[4 * i + 1] = fmaf(x[4 * i + 1], p.a, -(p.b * f.y));
            t[4 * i + 2] = fmaf(x[4 * i + 2], p.a, -(p.b * f.z));
            t[4 * i + 3] = fmaf(x[4 * i + 3], p.a, -(p.b * f.w));
        }
    } else {
#pragma unroll
        for (int i = 0; i < PER; ++i)
            t[i] = x[i] * p.a;
    }
    uint32_t w[PER / 4];
#pragma unroll
    for (int i = 0; i < PER / 4; ++i) {
        int packed = __builtin_amdgcn_cvt_pk_fp8_f32(t[4 * i], t[4 * i + 1], 0, false);
        packed = __builtin_amdgcn_cvt_pk_fp8_f32(t[4 * i + 2], t[4 * i + 3], packed, true);
        w[i] = (uint32_t)packed;
        const float d0 = t[4 * i] - __builtin_amdgcn_cvt_f32_fp8(packed, 0);
        const float d1 = t[4 * i + 1] - __builtin_amdgcn_cvt_f32_fp8(packed, 1);
        const float d2 = t[4 * i + 2] - __builtin_amdgcn_cvt_f32_fp8(packed, 2);
        const float d3 = t[4 * i + 3] - __builtin_amdgcn_cvt_f32_fp8(packed, 3);
        se = fmaf(d0, d0, se);
        se = fmaf(d1, d1, se);
        se = fmaf(d2, d2, se);
        se = fmaf(d3, d3, se);
    }
    if constexpr (PER == 8) {
        __builtin_nontemporal_store(w[0], reinterpret_cast<uint32_t *>(dst));
        __builtin_nontemporal_store(w[1], reinterpret_cast<uint32_t *>(dst) + 1);
    } else {
        __builtin_nontemporal_store(w[0], reinterpret_cast<uint32_t *>(dst));
    }
}

// The copy's parameters from the block's norm and, with a direction m, dot_m = <m, x> (all lanes pass the same values).
// Without a direction the copy holds the unit vector itself.  With one, alpha is <m, u> rounded to binary32 and the
// copy is scaled by an estimate of |u_c| from |u_c|^2 = 1 - 2 alpha <m, u> + alpha^2 |m|^2 with |m| taken as 1.  The
// estimate only sets the gain: the copy's error is measured with the scale actually stored.  It must not be so low
// that an element leaves e4m3's range (448 against the 256 aimed at): m is the binary32 rounding of an fp64 unit vector,
// so | |m|^2 - 1 | < 2^-22 and the estimate of |u_c|^2 is off by less than 3e-7; with the floor of 1e-6 the true value
// is below 1.3 times the estimate and the largest element below 256 * 1.15.
__device__ __forceinline__ Q8Block q8_block(double nrm, bool centred, double dot_m)
{
    Q8Block p;
    const double inv = nrm > 0.0 ? 1.0 / nrm : 0.0;
    p.alpha = 0.0;
    p.scale = (double)(1.0f / kQ8Scale);
    if (centred) {
        const double a = dot_m * inv;
        p.alpha = (double)(float)a;
        const double c = sqrt(fmax(fma(p.alpha, p.alpha - 2.0 * a, 1.0), 1e-6));
        p.scale = (double)(float)(c / (double)kQ8Scale);
    }
    const double a_wide = inv / p.scale;
    p.wide = !(a_wide < 1e37);
    p.a = p.wide ? 0.0f : (float)a_wide;
    p.b = p.wide ? 0.0f : (float)(p.alpha / p.scale);
    return p;
}

// The stored error of a copy from the sum over the block of quantise_chunk's se.  On top of the measured distance
// sqrt(se) * scale (the factor 1 + 1e-5 covers the binary32 sums) the margin covers: what binary32 loses in
// quantise_chunk (2.4e-7); the identity behind the centred copies, <u, v> = <u_c, v_c> + alpha_u alpha_v, which holds
// exactly for a unit m and alpha = <m, u> while the stored m and alpha are binary32 roundings of these, so that
// <m, u_c> and |m|^2 - 1 are below 2^-21 each and the identity is off by less than
// (|alpha_u| + |alpha_v| + |alpha_u alpha_v|) 2^-21 < 1.5e-6 for a pair, 0.75e-6 for each of its blocks; and the binary32
// arithmetic of the similarity kernel's test (a few 1e-7).  A block whose copy could not be written (Q8Block::wide)
// gets an error that makes every bound vacuous: all its pairs are then evaluated in fp64.
__device__ __forceinline__ float quantise_error(double se, const Q8Block &p, double nrm)
{
    if (p.wide)
        return nrm > 0.0 ? 2.0f : 0.0f;
    return nrm > 0.0 ? __double2float_ru(sqrt(se) * p.scale * (1.0 + 1e-5) + 3e-6) : 0.0f;
}

// Nearest-even rounding of a finite double straight to bfloat16 bits (no intermediate binary32 rounding).
__device__ __forceinline__ uint32_t f64_to_bf16_rne(double x)
{
    const uint64_t b = (uint64_t)__double_as_longlong(x);
    const uint32_t sign = (uint32_t)(b >> 63) << 15;
    const int ex = (int)((b >> 52) & 0x7FF);
    const uint64_t mant = b & 0xFFFFFFFFFFFFFull;
    if (ex == 0x7FF)
        return sign | 0x7F80u | (mant ? 0x40u : 0u);
    if (ex == 0)
        return sign;                         // double subnormals are far below the bfloat16 range
    const int e = ex - 1023 + 127;           // biased bfloat16 exponent
    if (e >= 255)
        return sign | 0x7F80u;
    const uint64_t sig = mant | (1ull << 52);
    int shift = 45;                          // 52 - 7 mantissa bits
    uint32_t base;
    if (e >= 1) {
        base = ((uint32_t)e << 7) - 128u;    // exponent field, the implicit one of sig is added back below
    } else {
        shift += 1 - e;
        base = 0u;
        if (shift > 54)
            return sign;
    }
    const uint64_t q = sig >> shift;
    const uint64_t rem = sig & ((1ull << shift) - 1ull);
    const uint64_t half = 1ull << (shift - 1);
    uint32_t out = base + (uint32_t)q;
    if (rem > half || (rem == half && (q & 1ull)))
        out += 1u;                            // a carry runs into the exponent field, which is what rounding up needs
    if (out >= 0x7F80u)
        out = 0x7F80u;
    return sign | out;
}

// Same result as f64_to_bf16_rne for finite inputs in the binary32 normal range, with one fp64 instruction: round
// to binary32 first (nearest even).  Every bfloat16 rounding boundary is a binary32 number and that rounding is
// monotonic, so unless the binary32 value sits exactly on a boundary it lies on the same side of it as x and the
// second rounding is safe; on a boundary the comparison with x itself decides (equal = a true tie, to even).
__device__ __forceinline__ uint32_t f64_to_bf16_fast(double x)
{
    const float f = (float)x;
    const uint32_t b = __float_as_uint(f);
    const uint32_t ex = (b >> 23) & 0xFFu;
    if (ex == 0u || ex == 0xFFu)
        return f64_to_bf16_rne(x);            // zero, subnormal, infinity, NaN: the exact path
    uint32_t up;
    if ((b & 0xFFFFu) == 0x8000u) {
        const double fd = (double)f;
        const bool away = fabs(x) > fabs(fd);
        const bool tie = x == fd;
        up = (away || (tie && ((b >> 16) & 1u))) ? 1u : 0u;
    } else {
        up = (b >> 15) & 1u;
    }
    return (b >> 16) + up;
}

#endif // __HIPCC__

}  // namespace kvfuse
