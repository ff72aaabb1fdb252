// Machine probes (libkvfuse_probe.so): what the MFMA units and the HBM sustain on this GPU, measured with the same
// instructions the hot path uses.  A library of its own for benchmarks; the product library neither contains nor
// calls any of this.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <string>

#include "../../include/kvfuse_probe.h"

namespace kvfuse_probe {

typedef float floatx16 __attribute__((ext_vector_type(16)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));

// Every wavefront issues independent v_mfma_f32_32x32x16_bf16 on operands that stay in registers: eight
// accumulators (as in the similarity kernel), two wavefronts per SIMD, no memory traffic inside the loop.
__global__ __launch_bounds__(512, 1) void probe_mfma_kernel(const uint4 *__restrict__ operands, int iters, float *__restrict__ sink)
{
    const int tid = threadIdx.x;
    uint4 a[4], b[4];
#pragma unroll
    for (int q = 0; q < 4; ++q) {
        a[q] = operands[(tid * 4 + q) & 4095];
        b[q] = operands[(tid * 4 + q + 2048) & 4095];
    }
    floatx16 acc[8];
#pragma unroll
    for (int x = 0; x < 8; ++x)
#pragma unroll
        for (int e = 0; e < 16; ++e)
            acc[x][e] = 0.0f;
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int s = 0; s < 4; ++s)
#pragma unroll
            for (int x = 0; x < 8; ++x)
                acc[x] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a[(x + s) & 3]),
                                                                 __builtin_bit_cast(bf16x8, b[(x * 3 + s) & 3]), acc[x], 0, 0, 0);
    }
    float s = 0.0f;
#pragma unroll
    for (int x = 0; x < 8; ++x)
#pragma unroll
        for (int e = 0; e < 16; ++e)
            s += acc[x][e];
    if (s == 12345.678f)      // keeps the accumulators alive without a store in the common case
        sink[0] = s;
}

// The same with the fp8 instruction of the fp8 screen, v_mfma_f32_32x32x64_f8f6f4 on two e4m3 operands (32 bytes per lane
// and operand): eight accumulators, operands in registers.
typedef int intx8 __attribute__((ext_vector_type(8)));
__global__ __launch_bounds__(512, 1) void probe_mfma_fp8_kernel(const uint4 *__restrict__ operands, int iters, float *__restrict__ sink)
{
    const int tid = threadIdx.x;
    uint4 a[8], b[8];
#pragma unroll
    for (int q = 0; q < 8; ++q) {
        a[q] = operands[(tid * 8 + q) & 4095];
        b[q] = operands[(tid * 8 + q + 2048) & 4095];
    }
    floatx16 acc[8];
#pragma unroll
    for (int x = 0; x < 8; ++x)
#pragma unroll
        for (int e = 0; e < 16; ++e)
            acc[x][e] = 0.0f;
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int s = 0; s < 4; ++s)
#pragma unroll
            for (int x = 0; x < 8; ++x) {
                const uint4 a0 = a[(x + s) & 3], a1 = a[4 + ((x + s) & 3)];
                const uint4 b0 = b[(x * 3 + s) & 3], b1 = b[4 + ((x * 3 + s) & 3)];
                const intx8 av = {(int)a0.x, (int)a0.y, (int)a0.z, (int)a0.w, (int)a1.x, (int)a1.y, (int)a1.z, (int)a1.w};
                const intx8 bv = {(int)b0.x, (int)b0.y, (int)b0.z, (int)b0.w, (int)b1.x, (int)b1.y, (int)b1.z, (int)b1.w};
                acc[x] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(av, bv, acc[x], 0, 0, 0, 0, 0, 0);
            }
    }
    float s = 0.0f;
#pragma unroll
    for (int x = 0; x < 8; ++x)
#pragma unroll
        for (int e = 0; e < 16; ++e)
            s += acc[x][e];
    if (s == 12345.678f)
        sink[0] = s;
}

// fp8 operands: e4m3 ones (0x38), or pseudo-random values with exponents within two binades of 1, random mantissa and sign
__global__ void probe_fill_fp8_kernel(uint4 *__restrict__ operands, int random_operands)
{
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= 4096)
        return;
    uint32_t w[4];
    uint32_t st = 0x9E3779B9u * (uint32_t)(i + 1);
#pragma unroll
    for (int k = 0; k < 4; ++k) {
        uint32_t v = 0x38383838u;
        if (random_operands) {
            v = 0u;
            for (int by = 0; by < 4; ++by) {
                st = st * 1664525u + 1013904223u;
                const uint32_t e = 5u + ((st >> 12) & 3u), m = (st >> 8) & 7u, sg = (st >> 20) & 1u;
                v |= ((sg << 7) | (e << 3) | m) << (8 * by);
            }
        }
        w[k] = v;
    }
    operands[i] = make_uint4(w[0], w[1], w[2], w[3]);
}

__global__ void probe_fill_kernel(uint4 *__restrict__ operands, int random_operands)
{
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= 4096)
        return;
    uint32_t w[4];
    uint32_t st = 0x9E3779B9u * (uint32_t)(i + 1);
#pragma unroll
    for (int k = 0; k < 4; ++k) {
        uint32_t v = 0x3F803F80u;                      // two bfloat16 ones
        if (random_operands) {
            // two bfloat16 values with random sign and mantissa and exponents within a few binades of 1
            st = st * 1664525u + 1013904223u;
            const uint32_t lo = 0x3E00u + ((st >> 8) & 0x1FFu) + ((st >> 20) & 1u) * 0x8000u;
            st = st * 1664525u + 1013904223u;
            const uint32_t hi = 0x3E00u + ((st >> 8) & 0x1FFu) + ((st >> 20) & 1u) * 0x8000u;
            v = lo | (hi << 16);
        }
        w[k] = v;
    }
    operands[i] = make_uint4(w[0], w[1], w[2], w[3]);
}

// One 16-byte chunk per lane and one workgroup per 4 KB, no loop: the hardware hands workgroups out in address order, so
// the chunks in flight at any time form one dense, advancing window of the buffer.  On this machine that is the fastest
// way to copy (about 6.2 TB/s read + written); a persistent grid that strides through the buffer with several loads in
// flight per lane reaches 5.1 - 5.7 TB/s, because slower workgroups fall behind and the window frays.
__global__ __launch_bounds__(256) void probe_copy_kernel(const uint4 *__restrict__ src, uint4 *__restrict__ dst, size_t n16)
{
    const size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
    if (i < n16)
        dst[i] = src[i];
}

// The similarity kernel's inner loop without its gather, its ragged tiles and its epilogue: 8 wavefronts, each
// 2 x 4 MFMA tiles per 256 x 256 x 32-element slice, fragments read from LDS one half slice ahead, one barrier per
// slice and, if LOADS, 32 KB of global -> LDS loads per slice from a 4 MB window (L2 resident).  LDS holds real
// (caller-supplied) bfloat16 data, because the rate depends on how the operand bits toggle.
template <bool LOADS>
__global__ __launch_bounds__(512, 1) void probe_tile_loop_kernel(const char *__restrict__ src, int iters, float *__restrict__ sink)
{
    __shared__ uint4 lds[2 * 2048 + 2048];     // two 32 KB operand stages + a 32 KB landing zone for the loads
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    for (int i = tid; i < 4096; i += 512)
        lds[i] = reinterpret_cast<const uint4 *>(src)[((size_t)blockIdx.x * 4096 + i) & 262143];
    __syncthreads();
    floatx16 acc[2][4];
#pragma unroll
    for (int a = 0; a < 2; ++a)
#pragma unroll
        for (int b = 0; b < 4; ++b)
#pragma unroll
            for (int e = 0; e < 16; ++e)
                acc[a][b][e] = 0.0f;
    uint4 fa[2][2], fb[2][4];
    auto rd = [&](int set, int stage) __attribute__((always_inline)) {
#pragma unroll
        for (int a = 0; a < 2; ++a)
            fa[set][a] = lds[(stage & 1) * 2048 + ((wave * 7 + a * 64 + lane) & 2047)];
#pragma unroll
        for (int b = 0; b < 4; ++b)
            fb[set][b] = lds[(stage & 1) * 2048 + ((wave * 13 + b * 64 + 1024 + lane) & 2047)];
    };
    rd(0, 0);
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int s = 0; s < 2; ++s) {
            rd(s ^ 1, it + s + 1);                                  // fragments of the next half slice
#pragma unroll
            for (int a = 0; a < 2; ++a)
#pragma unroll
                for (int b = 0; b < 4; ++b) {
                    acc[a][b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, fa[s][a]),
                                                                       __builtin_bit_cast(bf16x8, fb[s][b]), acc[a][b], 0, 0, 0);
                    if (LOADS && b == 1)                            // four 1 KB loads per wavefront and slice
                        __builtin_amdgcn_global_load_lds(
                            (const __attribute__((address_space(1))) void *)(src + ((size_t)((((blockIdx.x * 8 + wave) * 8 + ((it * 4 + s * 2 + a) & 7)) & 4095) * 64 + lane)) * 16),
                            (__attribute__((address_space(3))) void *)(lds + 4096 + (s * 2 + a) * 512 + wave * 64), 16, 0, 0);
                }
        }
        if (LOADS)
            asm volatile("s_waitcnt vmcnt(4)" ::: "memory");
        asm volatile("s_barrier" ::: "memory");
    }
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    float s = 0.0f;
#pragma unroll
    for (int a = 0; a < 2; ++a)
#pragma unroll
        for (int b = 0; b < 4; ++b)
#pragma unroll
            for (int e = 0; e < 16; ++e)
                s += acc[a][b][e];
    if (s == 12345.678f)
        sink[0] = s;
}

void launch_probe_tile_loop(hipStream_t s, const void *src, int with_loads, int workgroups, int iters, float *sink)
{
    if (with_loads)
        probe_tile_loop_kernel<true><<<workgroups, 512, 0, s>>>(static_cast<const char *>(src), iters, sink);
    else
        probe_tile_loop_kernel<false><<<workgroups, 512, 0, s>>>(static_cast<const char *>(src), iters, sink);
}

// The merge step's access pattern without its arithmetic: one wavefront per item reads two blocks of block_bytes
// (a target and, `gap` blocks further on, a member) and writes the first one back.  Items walk the buffer in
// stripes of 2 * gap blocks, the first `per_stripe` blocks of each stripe being targets.
__global__ __launch_bounds__(256) void probe_rmw_kernel(uint4 *__restrict__ buf, int n_items, int chunks, int gap, int per_stripe)
{
    const int lane = threadIdx.x & 63;
    const int n_waves = gridDim.x * 4;
    for (int it = blockIdx.x * 4 + (threadIdx.x >> 6); it < n_items; it += n_waves) {
        const size_t a = ((size_t)(it / per_stripe) * 2 * gap + it % per_stripe) * chunks, b = a + (size_t)gap * chunks;
        for (int c0 = 0; c0 < chunks; c0 += 256) {
            uint4 xa[4], xb[4];
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const int c = min(c0 + lane + 64 * q, chunks - 1);
                xa[q] = buf[a + c];
                xb[q] = buf[b + c];
            }
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const int c = c0 + lane + 64 * q;
                if (c < chunks)
                    buf[a + c] = make_uint4(xa[q].x ^ xb[q].x, xa[q].y ^ xb[q].y, xa[q].z ^ xb[q].z, xa[q].w ^ xb[q].w);
            }
        }
    }
}

void launch_probe_rmw(hipStream_t s, void *buf, int n_items, int block_bytes, int gap, int per_stripe)
{
    if (n_items > 0)
        probe_rmw_kernel<<<4096, 256, 0, s>>>(reinterpret_cast<uint4 *>(buf), n_items, block_bytes / 16, gap, per_stripe);
}

void launch_probe_fill(hipStream_t s, void *operands, int random_operands)
{
    probe_fill_kernel<<<16, 256, 0, s>>>(reinterpret_cast<uint4 *>(operands), random_operands);
}
void launch_probe_mfma(hipStream_t s, const void *operands, int workgroups, int iters, float *sink)
{
    probe_mfma_kernel<<<workgroups, 512, 0, s>>>(reinterpret_cast<const uint4 *>(operands), iters, sink);
}
void launch_probe_fill_fp8(hipStream_t s, void *operands, int random_operands)
{
    probe_fill_fp8_kernel<<<16, 256, 0, s>>>(reinterpret_cast<uint4 *>(operands), random_operands);
}
void launch_probe_mfma_fp8(hipStream_t s, const void *operands, int workgroups, int iters, float *sink)
{
    probe_mfma_fp8_kernel<<<workgroups, 512, 0, s>>>(reinterpret_cast<const uint4 *>(operands), iters, sink);
}
void launch_probe_copy(hipStream_t s, const void *src, void *dst, size_t bytes)
{
    const size_t n16 = bytes / 16;
    if (n16 == 0)
        return;
    probe_copy_kernel<<<(unsigned)((n16 + 255) / 256), 256, 0, s>>>(reinterpret_cast<const uint4 *>(src),
                                                                    reinterpret_cast<uint4 *>(dst), n16);
}


static thread_local std::string last_error;

static int fail(int code, const std::string &msg)
{
    last_error = msg;
    return code;
}

#define PROBE_HIP(expr)                                                                                  \
    do {                                                                                                 \
        hipError_t e__ = (expr);                                                                         \
        if (e__ != hipSuccess)                                                                           \
            return fail(KVFUSE_PROBE_EHIP, std::string(#expr) + ": " + hipGetErrorString(e__));          \
    } while (0)

}  // namespace kvfuse_probe

using namespace kvfuse_probe;

extern "C" {

const char *kvfuse_probe_last_error(void) { return last_error.c_str(); }

static int probe_mfma(void *hip_stream, int32_t random_operands, void *scratch, size_t scratch_bytes, double *tflops, bool fp8)
{
    hipStream_t stream = (hipStream_t)hip_stream;
    if (!scratch || !tflops || scratch_bytes < (size_t)KVFUSE_PROBE_SCRATCH_BYTES)
        return fail(KVFUSE_PROBE_EINVAL, "probe: needs a device scratch buffer of KVFUSE_PROBE_SCRATCH_BYTES and an output");
    int device = 0;
    PROBE_HIP(hipGetDevice(&device));
    hipDeviceProp_t prop;
    PROBE_HIP(hipGetDeviceProperties(&prop, device));
    const int wgs = prop.multiProcessorCount * 4;      // four rounds of one 8-wavefront workgroup per compute unit
    const int iters = 2000;
    float *sink = reinterpret_cast<float *>(static_cast<char *>(scratch) + 65536);
    hipEvent_t e0, e1;
    PROBE_HIP(hipEventCreate(&e0));
    PROBE_HIP(hipEventCreate(&e1));
    auto run = [&](int n) {
        if (fp8)
            launch_probe_mfma_fp8(stream, scratch, wgs, n, sink);
        else
            launch_probe_mfma(stream, scratch, wgs, n, sink);
    };
    if (fp8)
        launch_probe_fill_fp8(stream, scratch, random_operands);
    else
        launch_probe_fill(stream, scratch, random_operands);
    run(iters / 10);     // warm-up
    hipError_t err = hipEventRecord(e0, stream);
    run(iters);
    if (err == hipSuccess)
        err = hipEventRecord(e1, stream);
    if (err == hipSuccess)
        err = hipEventSynchronize(e1);
    float ms = 0.0f;
    if (err == hipSuccess)
        err = hipEventElapsedTime(&ms, e0, e1);
    (void)hipEventDestroy(e0);
    (void)hipEventDestroy(e1);
    PROBE_HIP(err);
    PROBE_HIP(hipGetLastError());
    // per wavefront and iteration: 32 MFMAs of 2 * 32 * 32 * 16 flops (bfloat16) or 2 * 32 * 32 * 64 (fp8)
    *tflops = ms > 0.0f ? (double)wgs * 8.0 * iters * 32.0 * (fp8 ? 131072.0 : 32768.0) / (ms * 1e-3) / 1e12 : 0.0;
    return KVFUSE_PROBE_OK;
}

int kvfuse_probe_mfma_bf16(void *hip_stream, int32_t random_operands, void *scratch, size_t scratch_bytes, double *tflops)
{
    return probe_mfma(hip_stream, random_operands, scratch, scratch_bytes, tflops, false);
}

int kvfuse_probe_mfma_fp8(void *hip_stream, int32_t random_operands, void *scratch, size_t scratch_bytes, double *tflops)
{
    return probe_mfma(hip_stream, random_operands, scratch, scratch_bytes, tflops, true);
}

int kvfuse_probe_copy(void *hip_stream, const void *src, void *dst, size_t bytes, int32_t repeats, double *gbps)
{
    hipStream_t stream = (hipStream_t)hip_stream;
    if (!src || !dst || !gbps || bytes < 16 || repeats <= 0 || bytes / 4096 >= 0x7FFFFFFFull)
        return fail(KVFUSE_PROBE_EINVAL, "probe: null pointer, fewer than 16 bytes, 8 TiB or more, or no repeats");
    hipEvent_t e0, e1;
    PROBE_HIP(hipEventCreate(&e0));
    PROBE_HIP(hipEventCreate(&e1));
    launch_probe_copy(stream, src, dst, bytes);                      // warm-up
    hipError_t err = hipEventRecord(e0, stream);
    for (int i = 0; i < repeats; ++i)
        launch_probe_copy(stream, src, dst, bytes);
    if (err == hipSuccess)
        err = hipEventRecord(e1, stream);
    if (err == hipSuccess)
        err = hipEventSynchronize(e1);
    float ms = 0.0f;
    if (err == hipSuccess)
        err = hipEventElapsedTime(&ms, e0, e1);
    (void)hipEventDestroy(e0);
    (void)hipEventDestroy(e1);
    PROBE_HIP(err);
    PROBE_HIP(hipGetLastError());
    *gbps = ms > 0.0f ? 2.0 * (double)(bytes / 16 * 16) * repeats / (ms * 1e-3) / 1e9 : 0.0;
    return KVFUSE_PROBE_OK;
}

int kvfuse_probe_tile_loop_bf16(void *hip_stream, const void *src, size_t src_bytes, int32_t with_loads, float *sink,
                                double *tflops)
{
    hipStream_t stream = (hipStream_t)hip_stream;
    if (!src || !sink || !tflops || src_bytes < ((size_t)4 << 20))
        return fail(KVFUSE_PROBE_EINVAL, "probe: needs 4 MiB of bfloat16 data to read, a device word to write and an output");
    int device = 0;
    PROBE_HIP(hipGetDevice(&device));
    hipDeviceProp_t prop;
    PROBE_HIP(hipGetDeviceProperties(&prop, device));
    const int wgs = prop.multiProcessorCount * 4;
    const int iters = 4000;
    hipEvent_t e0, e1;
    PROBE_HIP(hipEventCreate(&e0));
    PROBE_HIP(hipEventCreate(&e1));
    launch_probe_tile_loop(stream, src, with_loads, wgs, iters / 10, sink);      // warm-up
    hipError_t err = hipEventRecord(e0, stream);
    launch_probe_tile_loop(stream, src, with_loads, wgs, iters, sink);
    if (err == hipSuccess)
        err = hipEventRecord(e1, stream);
    if (err == hipSuccess)
        err = hipEventSynchronize(e1);
    float ms = 0.0f;
    if (err == hipSuccess)
        err = hipEventElapsedTime(&ms, e0, e1);
    (void)hipEventDestroy(e0);
    (void)hipEventDestroy(e1);
    PROBE_HIP(err);
    PROBE_HIP(hipGetLastError());
    *tflops = ms > 0.0f ? (double)wgs * iters * 2.0 * 256.0 * 256.0 * 32.0 / (ms * 1e-3) / 1e12 : 0.0;
    return KVFUSE_PROBE_OK;
}

int kvfuse_probe_read2_write1(void *hip_stream, void *buf, size_t bytes, int32_t block_bytes, int32_t repeats, double *gbps)
{
    hipStream_t stream = (hipStream_t)hip_stream;
    if (!buf || !gbps || block_bytes < 16 || block_bytes % 16 != 0 || repeats <= 0)
        return fail(KVFUSE_PROBE_EINVAL, "probe: null pointer, block size not a positive multiple of 16 bytes, or no repeats");
    // stripes of 256 blocks: the first 32 are targets, their members lie 128 blocks further on (the distance between
    // the same block of two neighbouring requests in the bench workload)
    const int gap = 128, per_stripe = 32;
    const size_t stripes = bytes / ((size_t)2 * gap * block_bytes);
    if (stripes == 0 || stripes * per_stripe > (size_t)INT32_MAX)
        return fail(KVFUSE_PROBE_EINVAL, "probe: buffer smaller than one stripe of 256 blocks, or too large");
    const int n_items = (int)(stripes * per_stripe);
    hipEvent_t e0, e1;
    PROBE_HIP(hipEventCreate(&e0));
    PROBE_HIP(hipEventCreate(&e1));
    launch_probe_rmw(stream, buf, n_items, block_bytes, gap, per_stripe);          // warm-up
    hipError_t err = hipEventRecord(e0, stream);
    for (int i = 0; i < repeats; ++i)
        launch_probe_rmw(stream, buf, n_items, block_bytes, gap, per_stripe);
    if (err == hipSuccess)
        err = hipEventRecord(e1, stream);
    if (err == hipSuccess)
        err = hipEventSynchronize(e1);
    float ms = 0.0f;
    if (err == hipSuccess)
        err = hipEventElapsedTime(&ms, e0, e1);
    (void)hipEventDestroy(e0);
    (void)hipEventDestroy(e1);
    PROBE_HIP(err);
    PROBE_HIP(hipGetLastError());
    *gbps = ms > 0.0f ? 3.0 * (double)block_bytes * n_items * repeats / (ms * 1e-3) / 1e9 : 0.0;
    return KVFUSE_PROBE_OK;
}

}  // extern "C"
