/*
 * dlprobe.h -- measurement aids of the MI355X convolution + loss library.
 *
 * Not part of the computation: two of the simplest possible kernels that show,
 * in the same process and on the same box as a benchmark run, what the matrix
 * units and the memory system deliver when nothing else is in the way.  The
 * benchmark prints their results next to the kernels' own figures; reported
 * roofline fractions keep the published peaks as denominators.
 *
 * Pointers marked "device" are caller-owned device memory; nothing is
 * allocated, work is enqueued on `hip_stream` (a hipStream_t as void*) and the
 * call returns at once.  Return value: 0 = ok, 1 = null pointer, 2 = bad
 * argument, 7 = the HIP runtime refused the launch.
 */
#ifndef DLPROBE_H
#define DLPROBE_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

enum { DL_PROBE_SINK_FLOATS = 1024 * 256 };

/* Register-resident loop of independent matrix instructions, no memory traffic:
 * 1024 workgroups of 4 wavefronts, each wavefront issuing `iters` rounds of
 * 262144 FLOP (shape 0: 8 x v_mfma_f32_32x32x16_f16, shape 1: 16 x
 * v_mfma_f32_16x16x32_f16, 16 independent accumulators either way).
 * operands 0: constants (1.0 and 0.5 in every element); 1: values distributed
 * like the benchmark's (|N(0,1)| activations against N(0, 0.03) filters), drawn
 * per lane in the kernel.  The chip is power-limited, so the two differ.
 * sink: device float[DL_PROBE_SINK_FLOATS] (receives the sums, so that nothing is
 * optimised away); clocks: device uint64[2], receives the ticks of the 100 MHz
 * wall clock and the shader-clock cycles that one wavefront spent in the loop
 * (their ratio is the clock the loop ran at).  *flop: host, the FLOPs issued. */
int dl_probe_mfma(int32_t shape, int32_t operands, int32_t iters, float *sink, uint64_t *clocks, double *flop,
                  void *hip_stream);

/* Streaming kernels over `bytes` bytes (a multiple of 3072), 16 bytes per lane,
 * whole 1 KB rows per wavefront, non-temporal, 1024 workgroups:
 *   mode 0: read src;  mode 1: copy src -> dst;  mode 2: write dst;
 *   mode 3: the loss kernel's traffic without its arithmetic: read src, read
 *           bytes/6 of aux (the label bytes), write dst: 13 bytes moved per 6
 *           bytes of src.
 * src, dst: device, 16-byte aligned, `bytes` each (either may be null where the
 * mode does not touch it); aux: device, bytes/6, mode 3 only; sink: device
 * uint32[1]. */
int dl_probe_stream(int32_t mode, const void *src, const void *aux, void *dst, int64_t bytes, uint32_t *sink,
                    void *hip_stream);

#ifdef __cplusplus
}
#endif
#endif /* DLPROBE_H */
