// Internal declarations shared by the translation units of libbnn (not part of the ABI).
#ifndef BNN_INTERNAL_H
#define BNN_INTERNAL_H

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "../../include/bnn.h"

namespace bnn {

// Division of 0 <= n < 2^31 by a runtime constant d >= 1 without a divide: one 32x32 high multiply
// and a shift (m == 0 marks a power of two: shift only).  For d not a power of two, with
// L = ceil(log2 d): sh = L - 1, m = floor(2^(32+sh) / d) + 1 < 2^32, and mulhi(n, m) >> sh == n / d
// for every n < 2^31 (the excess of m over the exact reciprocal contributes less than 1/d).
struct FastDiv {
    uint32_t m;
    int sh;
};
inline FastDiv make_fastdiv(uint32_t d) {
    FastDiv f;
    int L = 0;
    while ((1ull << L) < d) ++L;
    if ((1ull << L) == d) { f.m = 0u; f.sh = L; return f; }
    f.sh = L - 1;
    f.m = (uint32_t)(((1ull << (32 + f.sh)) / d) + 1ull);
    return f;
}
__host__ __device__ inline int fast_div(int n, const FastDiv& f) {
#if defined(__HIP_DEVICE_COMPILE__)
    return f.m == 0u ? (n >> f.sh) : (int)(__umulhi((uint32_t)n, f.m) >> f.sh);
#else
    return f.m == 0u ? (n >> f.sh) : (int)((((unsigned long long)(uint32_t)n * f.m) >> 32) >> f.sh);
#endif
}

// One +1/-1 contraction seen as an implicit GEMM: `rows` output rows (A rows of a BMM, output
// pixels n*P*Q of a convolution) by `cols` output columns (B rows / output channels), contracted
// over `taps` windows of `tw` packed words each.
struct Geom {
    long long rows;
    int cols;
    int conv;        // 0: BMM (taps = 1), 1: convolution
    int taps;        // k*k
    int tw;          // words per tap that are read: BMM ceil(K/32) rounded up to 4; conv cw = ceil(C/32)
    int bits_tap;    // logical bits per tap: K (BMM) or C (conv)
    int lda_w;       // BMM: words between A rows.  conv: words between pixels (= cw)
    int ldb_w;       // words between B rows (BMM: ldb_w, conv: k*k*cw)
    // convolution geometry (Sec. 5.3)
    int H, W, P, Q, k, stride, pad;
    FastDiv div_pq, div_q;   // divisions by P*Q and by Q (row -> image, pixel row, pixel column); rows < 2^31
    int kinv;        // ceil(65536 / k): tap / k == (tap * kinv) >> 16 for every tap < k*k + 64 (checked for k <= 42; k <= 32 accepted)
    int excl;        // 1: out-of-frame taps contribute nothing; 0: they count as -1
    int b_tiled;     // BMM only: B is stored in tiles of 32 rows x 16 bytes (bnn_tile_b), ldb_w words per row as before
    // Optional second source, accumulated into the same sums: a 1x1 convolution (no padding) of
    // a second packed tensor A2 [N][H2][W2][cw2] sampled at (p*stride2, q*stride2) with filters
    // B2 [cols][cw2] -- the binarized downsample shortcut of a residual block, fused so that its
    // int32 output never exists in memory.  A2 == nullptr: none.
    const uint32_t* A2;
    const uint32_t* B2;
    int H2, W2, cw2, stride2, bits2;
};

// What happens to each finished sum v[row][col] (all pointers may be null except as noted).
struct Epi {
    int32_t* out;          // out[row*ldc + col] = v (+ residual)
    const int32_t* resid;  // residual[row*ldc + col], added before the threshold (Sec. 6.1)
    const uint32_t* resid_bits;  // alternative residual: +1/-1 of bit col of resid_bits[row*ld_resid_bits_w + col/32]
    int ld_resid_bits_w;
    // 16-bit storage of the same int32 values (row stride ldc), used by the layer chain when the
    // sums provably fit: the arithmetic stays int32, only the bytes in memory are halved
    const int16_t* resid16;
    int16_t* out16;
    // 1: resid16 / out16 are stored in blocks of 32 rows x 32 columns (ldc a multiple of 32, rows padded to 32),
    // each block in the order the matrix cores hand out a 32x32 accumulator (sums16_index): a lane's 16 values
    // are 32 contiguous bytes, so the residual moves as two 16-byte accesses per lane instead of sixteen
    // 2-byte ones.  The tensor is private to the layer chain, which produces and consumes it with these kernels;
    // which element a lane's register holds is private to the kernel that writes a block (the 3x3 patch kernel keeps
    // 16 channels of one pixel per lane, the others one channel of 16 pixels).  That is safe because a block's sums
    // are only ever read by the second convolution of the next identity block: the same geometry and epilogue kind,
    // hence the same kernel choice.
    int sums_tiled;
    int ldc;               // elements between rows of out / resid
    int out_f32;           // 1: `out` receives the sums converted to fp32 (exact: |v| < 2^24) instead of int32
    const int32_t* thr;    // thr[col]: bit = (v >= thr[col])
    uint32_t* bits;        // bits[row*ldbits_w + col/32]
    int ldbits_w;          // words between rows of bits; words beyond ceil(cols/32) are zeroed
};

// Position of element (row, col) of a blocked 16-bit sum tensor (Epi::sums_tiled).  Inside a block, lane
// l = col % 32 + 32 * ((row / 4) % 2) of a wave holds the element in accumulator register
// r = 4 * ((row % 32) / 8) + row % 4, and the block stores lane after lane, 16 registers each.
__host__ __device__ inline long long sums16_index(long long row, int col, int ldc) {
    const int rl = (int)(row & 31);
    const int lane = (col & 31) + 32 * ((rl >> 2) & 1);
    const int r = 4 * (rl >> 3) + (rl & 3);
    return ((row >> 5) * (long long)(ldc >> 5) + (col >> 5)) * 1024 + lane * 16 + r;
}

// A chain of binarized layers for the whole-network persistent kernel.  The layer table lives in device memory
// (a ResNet-18-shaped chain has 16 layers of 256 bytes: more than a kernel argument block holds).
constexpr int PERSIST_MAX_LAYERS = 48;
struct PersistLayer {
    const uint32_t* A;
    const uint32_t* B;
    Geom g;
    Epi e;
    int gx, gy;            // 64 x 64 output tiles
    int variant;           // 0: matrix product; 1 + persist_conv_variant(): 3x3 convolution, see bnn_persistent.hip
};
struct PersistNet {
    int nlayers;
    const PersistLayer* layers;    // device memory, nlayers entries
    const uint8_t* in_u8;  // optional input layer: [in_rows][in_cols] 8-bit values -> in_bits [in_rows][in_ldw], bit = (x >= in_thr)
    uint32_t* in_bits;
    long long in_rows;
    int in_cols, in_thr, in_ldw;
};
// Index of the kernel's convolution form for this geometry, or -1 if the persistent kernel has none (it carries the
// fully unrolled 3x3 forms for 64, 128, 256 and 512 channels only).
int persist_conv_variant(const Geom& g);
// max_tiles: the largest tile count of the chain's layers (sizes the grid); max_grid: upper bound for the grid (the cost
// of a device-wide barrier grows with the number of workgroups).
int launch_persist_chain(const PersistNet& net, int max_tiles, int max_grid, unsigned* ctr, int sync, int spin_limit,
                         hipStream_t s);

int launch_valu(const uint32_t* A, const uint32_t* B, const Geom& g, const Epi& e, hipStream_t s);
int launch_mfma(const uint32_t* A, const uint32_t* B, const Geom& g, const Epi& e, hipStream_t s);
// Skinny matrix products (at most 128 rows): workgroups of 32 columns x all rows whose waves split K.
bool mfma_skinny_takes(const Geom& g);
const char* describe_mfma_skinny(const Geom& g);
int launch_mfma_skinny(const uint32_t* A, const uint32_t* B, const Geom& g, const Epi& e, hipStream_t s);
// Large matrix products: 256 x 256 workgroup tiles whose operands are expanded once, on their way into LDS.
bool mfma_wide_takes(const Geom& g, const Epi& e);
int launch_mfma_wide(const uint32_t* A, const uint32_t* B, const Geom& g, const Epi& e, hipStream_t s);
int launch_mfma_wide_panels(const uint32_t* A, const uint32_t* B, const Geom& g, const Epi& e, hipStream_t s);
// 3x3 stride-1 pad-1 convolutions with at most 128 channels in and out: filters resident in LDS, wave-private input patches.
bool mfma_conv_patch_takes(const Geom& g, const Epi& e);
const char* describe_mfma_conv_patch(const Geom& g);
int launch_mfma_conv_patch(const uint32_t* A, const uint32_t* B, const Geom& g, const Epi& e, hipStream_t s);
int launch_mfma_conv_staged(const uint32_t* A, const uint32_t* B, const Geom& g, const Epi& e, hipStream_t s);
int launch_mfma_conv_v4(const uint32_t* A, const uint32_t* B, const Geom& g, const Epi& e, hipStream_t s);
int launch_mfma_conv_v2(const uint32_t* A, const uint32_t* B, const Geom& g, const Epi& e, hipStream_t s);
int launch_mfma_conv_v1(const uint32_t* A, const uint32_t* B, const Geom& g, const Epi& e, hipStream_t s);
// Name of the kernel variant launch_mfma / launch_valu would pick for this geometry.
const char* describe_mfma(const Geom& g, bool int32_out = false);
const char* describe_valu(const Geom& g);

int launch_threshold_pack(const int32_t* X, const int32_t* thr, uint32_t* bits, long long rows, int cols,
                          int ldx, int ldb_w, hipStream_t s);
int launch_pack_u8(const uint8_t* x, int thr, uint32_t* bits, long long rows, int cols, int ldb_w, hipStream_t s);
int launch_sign_pack_f32(const float* x, uint32_t* bits, long long rows, int cols, int ldx, int ldb_w, hipStream_t s);
int launch_tile_b(const uint32_t* B, uint32_t* Bt, int N, int ldb_w, hipStream_t s);
int launch_panels_from_rows(const uint32_t* X, uint32_t* Xp, long long rows, int K, int ldx_w, hipStream_t s);
int launch_rows_from_panels(const uint32_t* Xp, uint32_t* X, long long rows, int K, int ldx_w, hipStream_t s);
int launch_probe_stride(const uint32_t* buf, long long* cycles, int stride_bytes, int rows, int iters, int dependent, hipStream_t s);
int launch_probe_pipeline(int which, void* buf, size_t buf_bytes, int iters, double* work, hipStream_t s);
int launch_pack_f32(const float* x, const float* thr, uint32_t* bits, long long rows, int cols, int ldb_w, hipStream_t s);
int launch_unpack_i32(const uint32_t* bits, int32_t* out, long long rows, int cols, int ldb_w, int ldo, hipStream_t s);
int launch_maxpool_or(const uint32_t* in, uint32_t* out, int N, int H, int W, int C, int win, int stride, hipStream_t s);
int launch_conv_f32_thr(const float* x, const float* w, const float* thr, float* y, uint32_t* bits,
                        int N, int H, int W, int C, int O, int k, int stride, int pad, hipStream_t s);
size_t bwn_workspace_bytes(int C, int O, int k);
size_t conv_f32_split_workspace_bytes(int C, int O, int k);
int launch_conv_f32_split_thr(const float* x, const float* w, const float* thr, float* y, uint32_t* bits,
                              int N, int H, int W, int C, int O, int k, int stride, int pad, int products,
                              void* workspace, size_t workspace_bytes, hipStream_t s);
int launch_bwn_conv_thr(const float* x, const uint32_t* wbits, const float* thr, float* y, uint32_t* bits,
                        int N, int H, int W, int C, int O, int k, int stride, int pad, void* workspace,
                        size_t workspace_bytes, hipStream_t s);
int launch_head_f32(const uint32_t* bits, const float* w, float* y, int32_t* pooled, int N, int HW, int C, int J,
                    hipStream_t s);

inline int check_launch() {
    return hipGetLastError() == hipSuccess ? BNN_OK : BNN_ERR_DEVICE;
}

inline long long cdiv(long long a, long long b) { return (a + b - 1) / b; }

}  // namespace bnn
#endif
