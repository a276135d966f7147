// Matrix-core product, instantiation: binary layer x 2-bit activations, integer part D.
#include "apb_binary_mfma_kernel.h"

namespace apb {

int launch_mfma_d_2bit(const mfma_detail::MfmaParams& p, int N, hipStream_t s) {
    return mfma_detail::launch_best_tile<1, 2, mfma_detail::kIntD>(p, N, s);
}

}  // namespace apb
