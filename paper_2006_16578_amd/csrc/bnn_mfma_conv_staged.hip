// Matrix-core path: LDS-staged convolution instantiations (16-byte pixels and multiples; 8-byte
// pixels, i.e. 64 channels).
#include "bnn_mfma_staged.h"

namespace bnn {

namespace {

template <int U>
int launch_u(const uint32_t* A, const uint32_t* B, const Geom& g, const Epi& e, hipStream_t s) {
    switch (mfma::pick_tile(g, &e)) {
        case 0: return mfma::launch_staged_tile<mfma::TileBig, U, true>(A, B, g, e, s);
        case 1:
            if constexpr (U == 16) return mfma::launch_staged_tile<mfma::TileTall, 16, true>(A, B, g, e, s);
            else return BNN_ERR_UNSUPPORTED;     // not dispatched: see staged_ok()
        default: return mfma::launch_staged_tile<mfma::TileMid, U, true>(A, B, g, e, s);
    }
}

}  // namespace

int launch_mfma_conv_staged(const uint32_t* A, const uint32_t* B, const Geom& g, const Epi& e, hipStream_t s) {
    if (g.tw == 2) return launch_u<8>(A, B, g, e, s);
    return launch_u<16>(A, B, g, e, s);
}

}  // namespace bnn
