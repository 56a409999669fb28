// Matrix-core path: dispatch and the BMM instantiations (kernels are in bnn_mfma_kernel.h and
// bnn_mfma_staged.h).
#include "bnn_mfma_staged.h"

namespace bnn {

namespace {

// The LDS-staged kernel covers every BMM (rows are padded to 128 bits) and the convolutions whose
// pixels are 8 bytes or a multiple of 16 bytes with -1 padding; the smallest tile, exclude
// padding and other channel counts use the direct kernel.
bool staged_ok(const Geom& g, int tile) {
    if (tile == 3) return false;
    if (!g.conv) return true;
    if (tile == 1 && g.tw == 2) return false;    // 512 loader rows of 8-byte pixels: too many registers
    return mfma::conv_stages_through_lds(g);
}

}  // namespace

int launch_mfma(const uint32_t* A, const uint32_t* B, const Geom& g, const Epi& e, hipStream_t s) {
    if (mfma_skinny_takes(g)) return launch_mfma_skinny(A, B, g, e, s);
    const int tile = mfma::pick_tile(g, &e);
    if (tile == 0 && mfma_wide_takes(g, e)) return launch_mfma_wide(A, B, g, e, s);
    if (!g.conv) {
        if (!g.b_tiled && staged_ok(g, tile)) {
            switch (tile) {
                case 0: return mfma::launch_staged_tile<mfma::TileBig, 16, false>(A, B, g, e, s);
                case 1: return mfma::launch_staged_tile<mfma::TileTall, 16, false>(A, B, g, e, s);
                default: return mfma::launch_staged_tile<mfma::TileMid, 16, false>(A, B, g, e, s);
            }
        }
        // tw is a multiple of 4 words; a chunk is 8 words, so an odd number of 4-word groups
        // leaves the upper half-wave without data in the last chunk -> guarded variant
        if (!mfma::offsets_fit(g)) {     // leading dimensions beyond the direct kernel's 32-bit offsets
            if (g.b_tiled) return BNN_ERR_UNSUPPORTED;
            return mfma::launch_staged_tile<mfma::TileMid, 16, false>(A, B, g, e, s);
        }
        if (g.tw % 8 == 0) return mfma::launch_shape<4, false, false>(A, B, g, e, s);
        return mfma::launch_shape<4, false, true>(A, B, g, e, s);
    }
    if (mfma_conv_patch_takes(g, e)) return launch_mfma_conv_patch(A, B, g, e, s);
    // (blocked 16-bit sums are implemented by the direct kernels only)
    if (!e.sums_tiled && staged_ok(g, tile)) return launch_mfma_conv_staged(A, B, g, e, s);
    if (!mfma::offsets_fit(g)) return BNN_ERR_UNSUPPORTED;
    if (g.tw % 8 == 0) return launch_mfma_conv_v4(A, B, g, e, s);
    if (g.tw % 4 == 0) return launch_mfma_conv_v2(A, B, g, e, s);
    return launch_mfma_conv_v1(A, B, g, e, s);
}

const char* describe_mfma(const Geom& g, bool int32_out) {
    if (mfma_skinny_takes(g)) return describe_mfma_skinny(g);
    static int32_t some_output;
    static uint32_t some_bits;
    Epi e = {};                                   // the choice only asks which outputs there are, never touches them
    e.out = int32_out ? &some_output : nullptr;
    e.bits = int32_out ? nullptr : &some_bits;
    e.ldbits_w = (g.cols + 31) / 32;
    const int tile = mfma::pick_tile(g, &e);
    if (tile == 0 && mfma_wide_takes(g, e)) return "mfma_fp4_bmm_xlds_wg256x256";
    if (mfma_conv_patch_takes(g, e)) return describe_mfma_conv_patch(g);
    const bool st = !g.b_tiled && staged_ok(g, tile);
    switch (tile) {
        case 0: return g.conv ? (st ? "mfma_fp4_conv_lds_wg256x128" : "mfma_fp4_conv_wg256x128")
                              : (st ? "mfma_fp4_bmm_lds_wg256x128" : "mfma_fp4_bmm_wg256x128");
        case 1: return g.conv ? (st ? "mfma_fp4_conv_lds_wg512x64" : "mfma_fp4_conv_wg512x64")
                              : (st ? "mfma_fp4_bmm_lds_wg512x64" : "mfma_fp4_bmm_wg512x64");
        case 2: return g.conv ? (st ? "mfma_fp4_conv_lds_wg128x128" : "mfma_fp4_conv_wg128x128")
                              : (st ? "mfma_fp4_bmm_lds_wg128x128" : "mfma_fp4_bmm_wg128x128");
        default: return g.conv ? "mfma_fp4_conv_wg64x64" : "mfma_fp4_bmm_wg64x64";
    }
}

}  // namespace bnn
