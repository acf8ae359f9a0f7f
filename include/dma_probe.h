/*
 * dma_probe.h -- C ABI of libdma_probe.so: roofline yardsticks measured on the device at hand.
 *
 * Not operations of the paper and not part of the attention library (libdma_hip.so, dma.h): the
 * benchmark uses them to report what this GPU reaches next to the published peaks.
 *   dma_probe_mfma  n_workgroups workgroups of 8 waves run `iters` rounds of 8 independent
 *                   32x32x16 bf16 MFMA chains from registers: n_workgroups * 8 * iters * 8 * 32768 flops.
 *                   sink: DEVICE buffer of n_workgroups * 512 floats (receives sums; contents are
 *                   of no interest).
 *   dma_probe_copy  plain streaming copy of `bytes` (a multiple of 16) from src to dst (DEVICE,
 *                   16-byte aligned).
 * Both enqueue one kernel on `stream` (a hipStream_t as void*, NULL = default stream) and return
 * without synchronising; the caller times them with events.  Return value: 0, or the dma_status of
 * dma.h (DMA_EINVAL for a bad argument, before any launch; DMA_EHIP if the launch failed).  The
 * caller owns the buffers; nothing is allocated or kept.
 */
#ifndef DMA_PROBE_H_
#define DMA_PROBE_H_

#include <stddef.h>

#ifdef __cplusplus
extern "C" {
#endif

int dma_probe_mfma(float* sink, int n_workgroups, int iters, void* stream);
int dma_probe_copy(const void* src, void* dst, size_t bytes, void* stream);

#ifdef __cplusplus
}
#endif

#endif /* DMA_PROBE_H_ */
