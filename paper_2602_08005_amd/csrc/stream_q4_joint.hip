// Streaming-kernel variants: one stream of 4-bit token-wise latents (all ranks).
#include "stream_kernel.h"

namespace dkv {

hipError_t stream_q4_joint(const DecodeParams& P, dim3 grid, size_t lds, hipStream_t st) {
  return P.sel_pages ? dispatch_stream<8, true, true, true>(P, grid, lds, st)
                     : dispatch_stream<8, true, false, true>(P, grid, lds, st);
}

}  // namespace dkv
