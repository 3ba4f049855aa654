// bf16 MFMA matrix products (placeholder until the tiled kernels land: reports
// every shape as unsupported so the plain FMA path is used).
#include "kernels.hpp"

namespace gpts {

bool gemm_mfma_supported(int, int, int, int) { return false; }
hipError_t gemm_mfma(int, int, int, int, const void*, const void*, void*, const GemmEpilogue&,
                     hipStream_t) {
  return hipErrorNotSupported;
}

}  // namespace gpts
