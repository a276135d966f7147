// Matrix-core product, instantiation: binary layer x 1-bit activations, integer part D.
#include "apb_binary_mfma_kernel.h"

namespace apb {

int launch_mfma_d_1bit(const mfma_detail::MfmaParams& p, int N, hipStream_t s) {
    return mfma_detail::launch_best_tile<1, 1, mfma_detail::kIntD>(p, N, s);
}

}  // namespace apb
