#include "common.h"
namespace dma {
int launch_bwd(const Ptrs&, const void*, const void*, const void*, const void*, const void*, const float*,
               const float*, const int32_t*, const int32_t*, void*, void*, void*, float*, char*, hipStream_t) {
  return DMA_EUNSUPPORTED;
}
}  // namespace dma
