// Matrix-core path: convolution instantiations with 4 packed words per lane and load.
#include "bnn_mfma_kernel.h"

namespace bnn {

int launch_mfma_conv_v4(const uint32_t* A, const uint32_t* B, const Geom& g, const Epi& e, hipStream_t s) {
    return mfma::launch_shape<4, true, false>(A, B, g, e, s);
}

}  // namespace bnn
