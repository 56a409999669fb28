// Matrix-core path, dispatch and the BMM instantiations (the kernel is in bnn_mfma_kernel.h).
#include "bnn_mfma_kernel.h"

namespace bnn {

int launch_mfma(const uint32_t* A, const uint32_t* B, const Geom& g, const Epi& e, hipStream_t s) {
    if (!g.conv) {
        // tw is a multiple of 4 words; a chunk is 8 words, so an odd number of 4-word groups
        // leaves the upper half-wave without data in the last chunk -> guarded variant
        if (g.tw % 8 == 0) return mfma::launch_shape<4, false, false>(A, B, g, e, s);
        return mfma::launch_shape<4, false, true>(A, B, g, e, s);
    }
    if (g.tw % 8 == 0) return launch_mfma_conv_v4(A, B, g, e, s);
    if (g.tw % 4 == 0) return launch_mfma_conv_v2(A, B, g, e, s);
    return launch_mfma_conv_v1(A, B, g, e, s);
}

const char* describe_mfma(const Geom& g) {
    switch (mfma::pick_tile(g)) {
        case 0: return g.conv ? "mfma_fp4_conv_wg256x128" : "mfma_fp4_bmm_wg256x128";
        case 1: return g.conv ? "mfma_fp4_conv_wg512x64" : "mfma_fp4_bmm_wg512x64";
        case 2: return g.conv ? "mfma_fp4_conv_wg128x128" : "mfma_fp4_bmm_wg128x128";
        default: return g.conv ? "mfma_fp4_conv_wg64x64" : "mfma_fp4_bmm_wg64x64";
    }
}

}  // namespace bnn
