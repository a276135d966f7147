// Matrix-core product, instantiation: 2-bit weights x 2-bit activations, integer result D22.
#include "apb_binary_mfma_kernel.h"

namespace apb {

int launch_mfma_22_int(const mfma_detail::MfmaParams& p, int N, hipStream_t s) {
    return mfma_detail::launch_best_tile<2, 2, mfma_detail::kInt22>(p, N, s);
}

}  // namespace apb
