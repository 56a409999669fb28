// Matrix-core path: convolution instantiations with one packed word per lane and load
// (channel counts that are not a multiple of 128; odd word counts take the guarded variant).
#include "bnn_mfma_kernel.h"

namespace bnn {

int launch_mfma_conv_v1(const uint32_t* A, const uint32_t* B, const Geom& g, const Epi& e, hipStream_t s) {
    if (g.tw % 2 == 0) return mfma::launch_shape<1, true, false>(A, B, g, e, s);
    return mfma::launch_shape<1, true, true>(A, B, g, e, s);
}

}  // namespace bnn
