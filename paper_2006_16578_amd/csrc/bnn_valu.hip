// XOR + popcount path on the vector ALUs: Eq. 2 of the paper taken literally,
//   v = n - 2 * popc(a xor b),
// with v_xor_b32 + v_bcnt_u32_b32 (popcount with fused accumulate): two VALU instructions per
// 32 bit-MACs per lane.
//
// Mapping (wave64): one lane owns one output row (an A row of a BMM, an output pixel of a
// convolution) and keeps 32 running popcounts for 32 consecutive output columns.  The 32 B rows
// (filters) a wave needs are the same for all its lanes, so their words are fetched through the
// scalar cache and enter v_xor as SGPR operands; only the lane's own A words use vector loads.
// The four waves of a workgroup share the same 64 rows and cover 128 columns.
#include "bnn_internal.h"

namespace bnn {

namespace {

template <int VW> struct WordVec;
template <> struct WordVec<1> { typedef uint32_t type; };
template <> struct WordVec<2> { typedef uint2 type; };
template <> struct WordVec<4> { typedef uint4 type; };

template <int VW>
__device__ __forceinline__ void load_words(const uint32_t* p, uint32_t (&a)[VW]) {
    typename WordVec<VW>::type v = *reinterpret_cast<const typename WordVec<VW>::type*>(p);
    if constexpr (VW == 1) { a[0] = v; }
    else if constexpr (VW == 2) { a[0] = v.x; a[1] = v.y; }
    else { a[0] = v.x; a[1] = v.y; a[2] = v.z; a[3] = v.w; }
}

template <int VW, bool CONV, bool EXCL>
__global__ __launch_bounds__(256) void valu_kernel(const uint32_t* __restrict__ A,
                                                   const uint32_t* __restrict__ B, Geom g, Epi e) {
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
    const long long row_raw = (long long)blockIdx.x * 64 + lane;
    const bool row_ok = row_raw < g.rows;
    const long long row = row_ok ? row_raw : g.rows - 1;
    const int col0 = ((int)blockIdx.y * 4 + wave) * 32;

    if (col0 >= g.cols) {   // only the zero pad words of a packed output live here
        if (e.bits != nullptr && (col0 >> 5) < e.ldbits_w && row_ok)
            e.bits[row * e.ldbits_w + (col0 >> 5)] = 0u;
        return;
    }

    int y0 = 0, x0 = 0;
    long long img_pix = 0;
    if (CONV) {
        const int pq = g.P * g.Q;
        const int n = (int)(row / pq);
        const int rem = (int)(row - (long long)n * pq);
        const int p = rem / g.Q, q = rem - p * g.Q;
        y0 = p * g.stride - g.pad;
        x0 = q * g.stride - g.pad;
        img_pix = (long long)n * g.H * g.W;
    }

    uint32_t acc[32];
#pragma unroll
    for (int j = 0; j < 32; ++j) acc[j] = 0u;
    int nvalid = 0;

    for (int tap = 0; tap < g.taps; ++tap) {
        const uint32_t* ap;
        bool inside = true;
        if (CONV) {
            const int r = tap / g.k, s = tap - r * g.k;
            const int y = y0 + r, x = x0 + s;
            inside = (unsigned)y < (unsigned)g.H && (unsigned)x < (unsigned)g.W;
            const long long pix = img_pix + (inside ? (long long)y * g.W + x : 0);
            ap = A + pix * g.lda_w;
        } else {
            ap = A + row * g.lda_w;
        }
        nvalid += inside ? 1 : 0;
        const uint32_t keep = inside ? 0xFFFFFFFFu : 0u;
        const long long btap = (long long)tap * g.tw;
        for (int w = 0; w < g.tw; w += VW) {
            uint32_t a[VW];
            load_words<VW>(ap + w, a);
            if (CONV) {
#pragma unroll
                for (int v = 0; v < VW; ++v) a[v] &= keep;   // out-of-frame pixel: all bits 0 (= -1)
            }
#pragma unroll
            for (int j = 0; j < 32; ++j) {
                const int col = min(col0 + j, g.cols - 1);           // uniform: scalar loads
                const uint32_t* bp = B + (long long)col * g.ldb_w + btap + w;
                uint32_t b[VW];
                load_words<VW>(bp, b);
#pragma unroll
                for (int v = 0; v < VW; ++v) {
                    uint32_t x = a[v] ^ b[v];
                    if (EXCL) x &= keep;                             // excluded tap adds nothing
                    acc[j] += __builtin_popcount(x);
                }
            }
        }
    }

    int nbits2 = 0;
    if (CONV && g.A2 != nullptr) {      // fused 1x1 shortcut convolution of a second tensor, always in frame
        const int pq = g.P * g.Q;
        const int n = (int)(row / pq);
        const int rem = (int)(row - (long long)n * pq);
        const int p = rem / g.Q, q = rem - p * g.Q;
        const uint32_t* a2 = g.A2 + (((long long)n * g.H2 + p * g.stride2) * g.W2 + q * g.stride2) * g.cw2;
        for (int w = 0; w < g.cw2; ++w) {
            const uint32_t a = a2[w];
#pragma unroll
            for (int j = 0; j < 32; ++j) {
                const int col = min(col0 + j, g.cols - 1);
                acc[j] += __builtin_popcount(a ^ g.B2[(long long)col * g.cw2 + w]);
            }
        }
        nbits2 = g.bits2;
    }
    // v = n - 2 * popc  (Eq. 2); n counts only in-frame taps in exclude mode (Sec. 5.3)
    const int nbits = (EXCL ? nvalid : g.taps) * g.bits_tap + nbits2;
    if (!row_ok) return;
    const long long obase = row * (long long)e.ldc;
    uint32_t word = 0u;
#pragma unroll
    for (int j = 0; j < 32; ++j) {
        const int col = col0 + j;
        if (col < g.cols) {
            int v = nbits - 2 * (int)acc[j];
            if (e.resid != nullptr) v += e.resid[obase + col];
            else if (e.resid16 != nullptr) v += (int)e.resid16[e.sums_tiled ? sums16_index(row, col, e.ldc) : obase + col];
            else if (e.resid_bits != nullptr)
                v += ((e.resid_bits[row * (long long)e.ld_resid_bits_w + (col >> 5)] >> (col & 31)) & 1u) ? 1 : -1;
            if (e.out != nullptr) e.out[obase + col] = e.out_f32 ? __float_as_int((float)v) : v;
            if (e.out16 != nullptr) e.out16[e.sums_tiled ? sums16_index(row, col, e.ldc) : obase + col] = (int16_t)v;
            if (e.thr != nullptr && v >= e.thr[col]) word |= (1u << j);
        }
    }
    if (e.bits != nullptr) e.bits[row * e.ldbits_w + (col0 >> 5)] = word;
}

template <int VW, bool CONV>
int launch_vw(const uint32_t* A, const uint32_t* B, const Geom& g, const Epi& e, hipStream_t s) {
    const int col_span = (e.bits != nullptr) ? max(g.cols, e.ldbits_w * 32) : g.cols;
    dim3 grid((unsigned)cdiv(g.rows, 64), (unsigned)cdiv(col_span, 128));
    if (g.excl) hipLaunchKernelGGL((valu_kernel<VW, CONV, true>), grid, dim3(256), 0, s, A, B, g, e);
    else        hipLaunchKernelGGL((valu_kernel<VW, CONV, false>), grid, dim3(256), 0, s, A, B, g, e);
    return check_launch();
}

}  // namespace

int launch_valu(const uint32_t* A, const uint32_t* B, const Geom& g, const Epi& e, hipStream_t s) {
    if (!g.conv) return launch_vw<4, false>(A, B, g, e, s);     // tw is a multiple of 4 by contract
    if (g.tw % 4 == 0) return launch_vw<4, true>(A, B, g, e, s);
    if (g.tw % 2 == 0) return launch_vw<2, true>(A, B, g, e, s);
    return launch_vw<1, true>(A, B, g, e, s);
}

const char* describe_valu(const Geom& g) { return g.conv ? "valu_xor_popc_conv" : "valu_xor_popc_bmm"; }

}  // namespace bnn
