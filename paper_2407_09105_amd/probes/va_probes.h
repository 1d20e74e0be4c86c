/*
 * va_probes.h -- C ABI of libva_probes.so: measurement aids of the benchmark.  They are no part of
 * the attention method and are not exported by libvarlen_attn.so; bench.py loads them to print what
 * this GPU sustains beside the published peaks.  All pointers are device memory unless marked host;
 * kernels are enqueued on `stream` (hipStream_t as void*), nothing is allocated or synchronised.
 */
#ifndef VA_PROBES_H
#define VA_PROBES_H
#include <stdint.h>
#ifdef __cplusplus
extern "C" {
#endif

enum { VAP_OK = 0, VAP_ERR_NULL = 1, VAP_ERR_ARG = 2, VAP_ERR_UNSUPPORTED = 3, VAP_ERR_HIP = 5 };

/*
 * Enqueue a kernel that issues nothing but bf16 32x32x16 matrix instructions on every SIMD,
 * `iters` (1 .. 2^24) rounds of 16 per wave.  The caller times it with events on `stream`;
 * *flops (host, may be NULL) receives the floating-point operations the launch performs.
 * sink: >= 64 floats, normally left untouched.
 */
int vap_probe_mfma(float *sink, int32_t iters, double *flops /* host, out */, void *stream);

/*
 * The same matrix instructions in the company they keep in the attention kernels.  operands: 64 KB
 * of 16-bit values with the bit patterns of real inputs (e.g. N(0,1) rounded to bf16), which the
 * kernel stages in LDS and multiplies (the rate a power-limited GPU sustains depends on how many
 * operand bits toggle).  Per 16 matrix instructions a wave also issues `lds_reads` 1 KB fragment
 * reads from LDS and `valu_groups` groups of {fma, exp2, max, add}, all independent of the matrix
 * instructions, 2 waves per SIMD.  Supported (lds_reads, valu_groups): (0,0), (8,0), (16,0),
 * (16,24) - the forward kernel's mix -, (16,12) and (8,16); others: VAP_ERR_UNSUPPORTED.
 * clocks (2 x uint64, may be NULL) receives the shader-clock ticks and the 100 MHz wall-clock ticks
 * of one wave's loop: their ratio is the clock the GPU held under that load.
 */
int vap_probe_mix(const void *operands, int32_t lds_reads, int32_t valu_groups, float *sink,
                  uint64_t *clocks /* out */, int32_t iters, double *flops /* host, out */, void *stream);

#ifdef __cplusplus
}
#endif
#endif /* VA_PROBES_H */
