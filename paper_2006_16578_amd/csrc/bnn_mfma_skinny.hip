// Matrix-core path for skinny matrix products (at most 128 rows of A: fully-connected layers at small batch).
//
// Such a product is bound by streaming the weights: M = 8, K = N = 4096 is 2 MB of B for 0.13 G bit-products.
// The tiled kernels give it one workgroup per 64 x 64 outputs, each walking all of K serially -- 64 workgroups on
// 256 compute units, a handful of loads in flight each.  Here a workgroup owns 32 output columns and ALL rows, and
// its waves (eight for up to 32 rows, else four) split K between them (the occupancy argument of Sec. 5.2, Design-1, turned around: with few rows
// the parallelism has to come from K and N).  Every wave requests all of its share of B and A up front (four
// 256-bit chunks in flight per lane), multiplies, and leaves its partial 32 x 32 sums in LDS; after one barrier
// wave i adds the partials of row tile i and runs the ordinary epilogue (threshold -> packed bits, or int32).
// N / 32 workgroups, each with its whole 16 KB of weights in flight at once.
#include "bnn_mfma_kernel.h"

namespace bnn {
namespace {

using mfma::v16f;
using mfma::v8i;

constexpr int DEPTH = 4;      // chunks (256 bits of K per row) a wave keeps in flight

// WAVES: 8 for a single row tile (the partial sums of 8 waves are 32 KB of LDS), 4 otherwise
template <int MT, int WAVES>
__global__ __launch_bounds__(64 * WAVES) void mfma_skinny_kernel(const uint32_t* __restrict__ A, const uint32_t* __restrict__ B,
                                                                 Geom g, Epi e) {
    __shared__ float part[WAVES][MT][16][64];
    const int lane = threadIdx.x & 63, l32 = lane & 31, half = lane >> 5;
    const int wave = threadIdx.x >> 6;
    const int n0 = (int)blockIdx.x * 32;

    uint32_t c2;
    asm volatile("v_mov_b32 %0, 0x22222222" : "=v"(c2));

    const uint32_t* ap[MT];
#pragma unroll
    for (int i = 0; i < MT; ++i) ap[i] = A + (long long)min((long long)(32 * i + l32), g.rows - 1) * g.lda_w + half * 4;
    const uint32_t* bp = B + (long long)min(n0 + l32, g.cols - 1) * g.ldb_w + half * 4;

    v16f acc[MT];
#pragma unroll
    for (int i = 0; i < MT; ++i)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[i][r] = 0.f;

    // chunk c covers words 8c .. 8c+7 of a row (lower half-wave the first four, upper the last four); wave w
    // takes chunks w, w + 4, ...  tw is a multiple of 4, so only the upper half of the last chunk can lie past
    // the row's end: it is read from the row's start instead and masked to zero bits when multiplied.
    const int T = (g.tw + 7) / 8;
    const int mine = (T - wave + WAVES - 1) / WAVES;
    uint4 ra[DEPTH][MT], rb[DEPTH];
    uint32_t keep[DEPTH];
    auto request = [&](int buf, int t) {
        if (t < mine) {
            const int wo = (wave + WAVES * t) * 8;
            const bool ok = wo + half * 4 < g.tw;
            const int off = ok ? wo : -half * 4;
            rb[buf] = *reinterpret_cast<const uint4*>(bp + off);
#pragma unroll
            for (int i = 0; i < MT; ++i) ra[buf][i] = *reinterpret_cast<const uint4*>(ap[i] + off);
            keep[buf] = ok ? 0xFFFFFFFFu : 0u;
        }
    };
    auto multiply = [&](int buf) {
        const uint32_t km = keep[buf];
        const uint32_t bw[4] = {rb[buf].x & km, rb[buf].y & km, rb[buf].z & km, rb[buf].w & km};
#pragma unroll
        for (int v = 0; v < 4; ++v) {
            const v8i eb = mfma::expand_fp4(bw[v], c2);
#pragma unroll
            for (int i = 0; i < MT; ++i) {
                const uint4 a4 = ra[buf][i];
                const uint32_t aw = (v == 0 ? a4.x : v == 1 ? a4.y : v == 2 ? a4.z : a4.w) & km;
                acc[i] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(mfma::expand_fp4(aw, c2), eb, acc[i], 4, 4, 0, 0, 0, 0);
            }
        }
    };
#pragma unroll
    for (int d = 0; d < DEPTH; ++d) request(d, d);
    for (int t = 0; t < mine; t += DEPTH) {
#pragma unroll
        for (int d = 0; d < DEPTH; ++d) {
            if (t + d < mine) multiply(d);
            request(d, t + d + DEPTH);
        }
    }

#pragma unroll
    for (int i = 0; i < MT; ++i)
#pragma unroll
        for (int r = 0; r < 16; ++r) part[wave][i][r][lane] = acc[i][r];
    __syncthreads();
    if (wave < MT) {                      // wave i finishes row tile i
        v16f sum[1][1];
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            float v = 0.f;                // exact: every partial is an integer below 2^24 in magnitude
#pragma unroll
            for (int w = 0; w < WAVES; ++w) v += part[w][wave][r][lane];
            sum[0][0][r] = v;
        }
        // every chunk multiplied 256 bit positions per row; those past K are 0 bits in both operands (+1 each)
        mfma::epilogue<1, 1, false, false>(sum, 32LL * wave, n0, lane, g, e, T * 256 - g.bits_tap, 0);
    }
}

}  // namespace

bool mfma_skinny_takes(const Geom& g) { return !g.conv && !g.b_tiled && g.rows <= 128; }

const char* describe_mfma_skinny(const Geom& g) {
    return g.rows <= 32 ? "mfma_fp4_bmm_skinny_m32" : g.rows <= 64 ? "mfma_fp4_bmm_skinny_m64" : "mfma_fp4_bmm_skinny_m128";
}

int launch_mfma_skinny(const uint32_t* A, const uint32_t* B, const Geom& g, const Epi& e, hipStream_t s) {
    const int col_span = (e.bits != nullptr) ? max(g.cols, e.ldbits_w * 32) : g.cols;
    const dim3 grid((unsigned)cdiv(col_span, 32));
    if (g.rows <= 32) hipLaunchKernelGGL((mfma_skinny_kernel<1, 8>), grid, dim3(64 * 8), 0, s, A, B, g, e);
    else if (g.rows <= 64) hipLaunchKernelGGL((mfma_skinny_kernel<2, 4>), grid, dim3(64 * 4), 0, s, A, B, g, e);
    else hipLaunchKernelGGL((mfma_skinny_kernel<4, 4>), grid, dim3(64 * 4), 0, s, A, B, g, e);
    return check_launch();
}

}  // namespace bnn
