/*
 * kvfuse_probe.h -- C ABI of the machine probes (libkvfuse_probe.so).
 *
 * Measurement aids for benchmarks: what the matrix units and the memory system of the GPU at hand sustain, measured
 * with the instructions and access patterns the Fast Fusion hot path uses, so that its kernels can be held against
 * the machine and not only against data-sheet peaks.  This is a library of its own: nothing in libkvfuse.so calls it
 * and it is no part of the method's interface (kvfuse.h).
 *
 * Conventions: plain C; every call returns 0 on success, KVFUSE_PROBE_EINVAL for a bad argument or
 * KVFUSE_PROBE_EHIP for a HIP runtime error (text from kvfuse_probe_last_error, per calling thread).  Device
 * pointers are owned by the caller; nothing is allocated.  hip_stream is a hipStream_t (NULL = default stream); every
 * probe enqueues its kernels there and waits for them before it returns.
 */
#ifndef KVFUSE_PROBE_H
#define KVFUSE_PROBE_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

enum { KVFUSE_PROBE_OK = 0, KVFUSE_PROBE_EINVAL = 1, KVFUSE_PROBE_EHIP = 5 };

#define KVFUSE_PROBE_SCRATCH_BYTES 65792

const char *kvfuse_probe_last_error(void);

/* Sustained rate of the bfloat16 MFMA instruction the similarity step uses (Algorithm 1's product sim <- k_l k_r^T runs
 * on it), over the whole GPU, with operands in registers and no memory traffic: the compute ceiling the similarity
 * kernel can be held against besides the nominal peak.  random_operands = 0 multiplies a constant pattern,
 * 1 multiplies pseudo-random values, which is what real caches look like to the multipliers -- the chip lowers
 * its clock under that load, so the two differ.  scratch: device, >= KVFUSE_PROBE_SCRATCH_BYTES, overwritten.
 * tflops: host.  About 50 - 100 ms. */
int kvfuse_probe_mfma_bf16(void *hip_stream, int32_t random_operands, void *scratch, size_t scratch_bytes, double *tflops);

/* The same for the fp8 instruction of the opt-in fp8 screen (v_mfma_f32_32x32x64_f8f6f4 on two e4m3 operands), whose
 * nominal dense peak is twice the bfloat16 one.  Same arguments. */
int kvfuse_probe_mfma_fp8(void *hip_stream, int32_t random_operands, void *scratch, size_t scratch_bytes, double *tflops);

/* Rate of a plain device copy kernel (one 16-byte chunk per lane, one workgroup per 4 KB, workgroups handed out in
 * address order), read + write bytes per second: the HBM ceiling for one read per write.  src, dst: device, bytes each
 * (below 8 TiB), not overlapping; gbps: host. */
int kvfuse_probe_copy(void *hip_stream, const void *src, void *dst, size_t bytes, int32_t repeats, double *gbps);

/* Rate of the similarity kernel's inner loop without its gather, ragged tiles and epilogue: per compute unit 8
 * wavefronts of 2 x 4 MFMA tiles per 256 x 256 x 32-element slice, fragments read from LDS one half slice ahead, a
 * barrier per slice and, if with_loads, 32 KB of global -> LDS loads per slice from an L2-resident 4 MiB window of
 * src.  The LDS operands are taken from src, so pass data like the cache's (the rate depends on how the operand bits
 * toggle).  This is the ceiling of the kernel's tile organisation on a given machine, between the register-fed MFMA
 * probe and the kernel itself.  src: device, >= 4 MiB, read only; sink: device, one float; tflops: host.  About
 * 30 ms. */
int kvfuse_probe_tile_loop_bf16(void *hip_stream, const void *src, size_t src_bytes, int32_t with_loads, float *sink,
                                double *tflops);

/* Rate of the merge step's access pattern without its arithmetic: one wavefront per item reads two blocks of
 * block_bytes (a target and a member 128 blocks further on) and writes the first one back; bytes read + written per
 * second.  This is the ceiling the merge step (two reads per write, Algorithm 1's fusion line) can be held against on a
 * given machine.  buf: device, bytes >= 256 * block_bytes, overwritten; gbps: host. */
int kvfuse_probe_read2_write1(void *hip_stream, void *buf, size_t bytes, int32_t block_bytes, int32_t repeats, double *gbps);

#ifdef __cplusplus
}
#endif
#endif /* KVFUSE_PROBE_H */
