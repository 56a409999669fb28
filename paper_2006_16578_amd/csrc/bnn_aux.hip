// Thin boundary kernels: stand-alone threshold / pack / unpack (Sec. 6.1 thrd, Eq. 1) and the
// full-precision first convolution and pooled last FC of a network whose inner layers are
// binarized (Sec. 6.1).  None of these is on the bit-matrix hot path; they are kept simple and
// coalesced.
#include "bnn_internal.h"

namespace bnn {

namespace {

// One wave per 64 columns: lane c tests its element, the 64-bit ballot is two packed words.
template <typename T, typename TH, bool SCALAR_THR>
__global__ __launch_bounds__(256) void pack_kernel(const T* __restrict__ x, const TH* __restrict__ thr, TH thr0,
                                                   uint32_t* __restrict__ bits, long long rows, int cols,
                                                   int ldx, int ldb_w) {
    const int lane = threadIdx.x & 63;
    const long long row = (long long)blockIdx.x * 4 + (threadIdx.x >> 6);
    if (row >= rows) return;                         // whole wave leaves together
    const T* xr = x + row * (long long)ldx;
    uint32_t* br = bits + row * (long long)ldb_w;
    const int nw2 = (ldb_w + 1) / 2;                 // 64-bit groups to write, pad words included
    for (int g = 0; g < nw2; ++g) {
        const int c = g * 64 + lane;
        bool pred = false;
        if (c < cols) {
            const TH t = SCALAR_THR ? thr0 : thr[c];
            pred = (TH)xr[c] >= t;
        }
        const unsigned long long ball = __builtin_amdgcn_ballot_w64(pred);
        if (lane == 0) br[2 * g] = (uint32_t)ball;
        if (lane == 1 && 2 * g + 1 < ldb_w) br[2 * g + 1] = (uint32_t)(ball >> 32);
    }
}

__global__ __launch_bounds__(256) void unpack_kernel(const uint32_t* __restrict__ bits, int32_t* __restrict__ out,
                                                     long long rows, int cols, int ldb_w, int ldo) {
    const long long row = blockIdx.y;
    for (long long r = row; r < rows; r += gridDim.y) {
        for (int c = blockIdx.x * blockDim.x + threadIdx.x; c < cols; c += gridDim.x * blockDim.x) {
            const uint32_t w = bits[r * ldb_w + (c >> 5)];
            out[r * ldo + c] = ((w >> (c & 31)) & 1u) ? 1 : -1;
        }
    }
}

// First layer: fp32 convolution with zero padding, then per-channel threshold -> bits, as an
// implicit GEMM on the fp32 matrix cores (v_mfma_f32_32x32x2_f32): rows are output pixels,
// columns output channels, and K runs over the k filter rows times the k*C contiguous floats of
// one filter row -- contiguous in the NHWC input as well, so lane l of a wave reads element
// 2*t + l/32 of the row segment of pixel l%32 with no index arithmetic beyond one bounds test.
// A wave owns 2 x 2 accumulator tiles (64 pixels x 64 channels), a workgroup 256 pixels.
typedef float v16f_aux __attribute__((ext_vector_type(16)));
extern "C" __device__ int bnn_aux_writelane_i32(int val, int lane, int old) __asm("llvm.amdgcn.writelane.i32");

constexpr int STEM_MT = 2, STEM_NT = 2;

__global__ __launch_bounds__(256) void conv_f32_kernel(const float* __restrict__ x, const float* __restrict__ w,
                                                       const float* __restrict__ thr, float* __restrict__ y,
                                                       uint32_t* __restrict__ bits, int N, int H, int W, int C,
                                                       int O, int k, int stride, int pad, int P, int Q) {
    const int lane = threadIdx.x & 63, l32 = lane & 31, half = lane >> 5, wave = threadIdx.x >> 6;
    const long long npix = (long long)N * P * Q;
    const long long m0 = ((long long)blockIdx.x * 4 + wave) * (STEM_MT * 32);
    const int n0 = (int)blockIdx.y * (STEM_NT * 32);
    if (m0 >= npix) return;                                  // uniform per wave
    const int seg = k * C;                                   // floats in one filter row
    const int steps = (seg + 1) / 2;
    const int rowlen = W * C;

    const float* xrow[STEM_MT];     // start of input row y0 of this lane's pixel
    int xoff[STEM_MT], ytop[STEM_MT];
#pragma unroll
    for (int i = 0; i < STEM_MT; ++i) {
        long long pix = m0 + 32 * i + l32;
        if (pix > npix - 1) pix = npix - 1;
        const int n = (int)(pix / (P * Q));
        const int rem = (int)(pix - (long long)n * P * Q);
        const int p = rem / Q, q = rem - p * Q;
        ytop[i] = p * stride - pad;
        xoff[i] = (q * stride - pad) * C;
        xrow[i] = x + (long long)n * H * rowlen;
    }
    const float* wrow[STEM_NT];
#pragma unroll
    for (int j = 0; j < STEM_NT; ++j) wrow[j] = w + (long long)min(n0 + 32 * j + l32, O - 1) * k * seg;

    v16f_aux acc[STEM_MT][STEM_NT];
#pragma unroll
    for (int i = 0; i < STEM_MT; ++i)
#pragma unroll
        for (int j = 0; j < STEM_NT; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

    for (int r = 0; r < k; ++r) {
        for (int t = 0; t < steps; ++t) {
            const int e = 2 * t + half;
            const bool eok = e < seg;
            float a[STEM_MT], b[STEM_NT];
#pragma unroll
            for (int i = 0; i < STEM_MT; ++i) {
                const int yy = ytop[i] + r;
                const int xe = xoff[i] + e;
                const bool ok = eok && (unsigned)yy < (unsigned)H && (unsigned)xe < (unsigned)rowlen;
                const float v = xrow[i][ok ? (long long)yy * rowlen + xe : 0];
                a[i] = ok ? v : 0.f;                         // zero padding
            }
#pragma unroll
            for (int j = 0; j < STEM_NT; ++j) {
                const float v = wrow[j][eok ? r * seg + e : 0];
                b[j] = eok ? v : 0.f;
            }
#pragma unroll
            for (int i = 0; i < STEM_MT; ++i)
#pragma unroll
                for (int j = 0; j < STEM_NT; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(a[i], b[j], acc[i][j], 0, 0, 0);
        }
    }

    float th[STEM_NT];
    bool cok[STEM_NT];
#pragma unroll
    for (int j = 0; j < STEM_NT; ++j) {
        const int col = n0 + 32 * j + l32;
        cok[j] = col < O;
        th[j] = (bits != nullptr && cok[j]) ? thr[col] : __builtin_inff();
    }
    const int ow = (O + 31) / 32;
#pragma unroll
    for (int i = 0; i < STEM_MT; ++i) {
        const long long rbase = m0 + 32 * i;
        if (rbase >= npix) break;
        uint32_t wout[STEM_NT];
#pragma unroll
        for (int j = 0; j < STEM_NT; ++j) wout[j] = 0u;
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            const int lo_row = 8 * (r >> 2) + (r & 3);
            const long long row = rbase + lo_row + 4 * half;
#pragma unroll
            for (int j = 0; j < STEM_NT; ++j) {
                const float v = acc[i][j][r];
                if (y != nullptr && row < npix && cok[j]) y[row * O + n0 + 32 * j + l32] = v;
                if (bits != nullptr) {
                    const unsigned long long ball = __builtin_amdgcn_ballot_w64(v >= th[j]);
                    wout[j] = (uint32_t)bnn_aux_writelane_i32((int)(uint32_t)ball, lo_row, (int)wout[j]);
                    wout[j] = (uint32_t)bnn_aux_writelane_i32((int)(uint32_t)(ball >> 32), lo_row + 4, (int)wout[j]);
                }
            }
        }
        const long long row = rbase + lane;
        if (bits != nullptr && lane < 32 && row < npix) {
#pragma unroll
            for (int j = 0; j < STEM_NT; ++j) {
                const int wi = (n0 >> 5) + j;
                if (wi < ow) bits[row * ow + wi] = wout[j];
            }
        }
    }
}

// Head: exact integer sum-pool of +1/-1 over HW positions, then fp32 FC.  A workgroup handles
// HEAD_IMGS images and HEAD_OUTS output rows.  Pooling: a thread owns one packed word (32
// channels) of one image and counts set bits per channel over the HW positions, 4 channels at a
// time in the bytes of one register (HW <= 255); the sum of +1/-1 is 2 * count - HW.  FC: a wave
// per output row, lanes stride over channels, butterfly reduction.
constexpr int HEAD_IMGS = 4;
constexpr int HEAD_OUTS = 128;
constexpr int HEAD_MAXC = 1024;

__global__ __launch_bounds__(256) void head_kernel(const uint32_t* __restrict__ bits, const float* __restrict__ w,
                                                   float* __restrict__ y, int32_t* __restrict__ pooled_out,
                                                   int N, int HW, int C, int J) {
    __shared__ float pooled[HEAD_IMGS][HEAD_MAXC];
    const int n0 = blockIdx.x * HEAD_IMGS;
    const int j0 = blockIdx.y * HEAD_OUTS;
    const int cw = (C + 31) / 32;
    const float inv = (float)HW;
    for (int idx = threadIdx.x; idx < HEAD_IMGS * cw; idx += blockDim.x) {
        const int im = idx / cw, wi = idx - im * cw;
        const int n = n0 + im;
        uint32_t cnt[8];                       // cnt[q] byte b = number of set bits of channel 4*q... see below
#pragma unroll
        for (int q = 0; q < 8; ++q) cnt[q] = 0u;
        if (n < N) {
            const uint32_t* b = bits + (long long)n * HW * cw + wi;
            for (int i = 0; i < HW; ++i) {
                const uint32_t v = b[(long long)i * cw];
                // bit (q + 8*t) of v is added to byte t of cnt[q]
#pragma unroll
                for (int q = 0; q < 8; ++q) cnt[q] += (v >> q) & 0x01010101u;
            }
        }
#pragma unroll
        for (int q = 0; q < 8; ++q)
#pragma unroll
            for (int t = 0; t < 4; ++t) {
                const int c = wi * 32 + q + 8 * t;
                if (c < C) {
                    const int s = (n < N) ? 2 * (int)((cnt[q] >> (8 * t)) & 0xFFu) - HW : 0;
                    if (pooled_out != nullptr && blockIdx.y == 0 && n < N) pooled_out[(long long)n * C + c] = s;
                    pooled[im][c] = (float)s / inv;
                }
            }
    }
    __syncthreads();
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    for (int j = j0 + wave; j < min(j0 + HEAD_OUTS, J); j += 4) {
        float part[HEAD_IMGS];
#pragma unroll
        for (int im = 0; im < HEAD_IMGS; ++im) part[im] = 0.f;
        for (int c = lane; c < C; c += 64) {
            const float wv = w[(long long)j * C + c];
#pragma unroll
            for (int im = 0; im < HEAD_IMGS; ++im) part[im] = fmaf(pooled[im][c], wv, part[im]);
        }
#pragma unroll
        for (int im = 0; im < HEAD_IMGS; ++im) {
            float v = part[im];
            for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off, 64);
            if (lane == 0 && n0 + im < N) y[(long long)(n0 + im) * J + j] = v;
        }
    }
}

}  // namespace

int launch_threshold_pack(const int32_t* X, const int32_t* thr, uint32_t* bits, long long rows, int cols,
                          int ldx, int ldb_w, hipStream_t s) {
    hipLaunchKernelGGL((pack_kernel<int32_t, int32_t, false>), dim3((unsigned)cdiv(rows, 4)), dim3(256), 0, s,
                       X, thr, 0, bits, rows, cols, ldx, ldb_w);
    return check_launch();
}

int launch_pack_u8(const uint8_t* x, int thr, uint32_t* bits, long long rows, int cols, int ldb_w, hipStream_t s) {
    hipLaunchKernelGGL((pack_kernel<uint8_t, int32_t, true>), dim3((unsigned)cdiv(rows, 4)), dim3(256), 0, s,
                       x, (const int32_t*)nullptr, thr, bits, rows, cols, cols, ldb_w);
    return check_launch();
}

int launch_pack_f32(const float* x, const float* thr, uint32_t* bits, long long rows, int cols, int ldb_w, hipStream_t s) {
    hipLaunchKernelGGL((pack_kernel<float, float, false>), dim3((unsigned)cdiv(rows, 4)), dim3(256), 0, s,
                       x, thr, 0.f, bits, rows, cols, cols, ldb_w);
    return check_launch();
}

int launch_unpack_i32(const uint32_t* bits, int32_t* out, long long rows, int cols, int ldb_w, int ldo, hipStream_t s) {
    dim3 grid((unsigned)min((long long)cdiv(cols, 256), 64LL), (unsigned)min(rows, 65535LL));
    hipLaunchKernelGGL(unpack_kernel, grid, dim3(256), 0, s, bits, out, rows, cols, ldb_w, ldo);
    return check_launch();
}

int launch_conv_f32_thr(const float* x, const float* w, const float* thr, float* y, uint32_t* bits,
                        int N, int H, int W, int C, int O, int k, int stride, int pad, hipStream_t s) {
    const int P = (H + 2 * pad - k) / stride + 1, Q = (W + 2 * pad - k) / stride + 1;
    const long long npix = (long long)N * P * Q;
    dim3 grid((unsigned)cdiv(npix, 4 * STEM_MT * 32), (unsigned)cdiv(O, STEM_NT * 32));
    hipLaunchKernelGGL(conv_f32_kernel, grid, dim3(256), 0, s, x, w, thr, y, bits, N, H, W, C, O, k, stride, pad, P, Q);
    return check_launch();
}

int launch_head_f32(const uint32_t* bits, const float* w, float* y, int32_t* pooled, int N, int HW, int C, int J,
                    hipStream_t s) {
    if (C > HEAD_MAXC || HW > 255) return BNN_ERR_UNSUPPORTED;
    hipLaunchKernelGGL(head_kernel, dim3((unsigned)cdiv(N, HEAD_IMGS), (unsigned)cdiv(J, HEAD_OUTS)), dim3(256), 0, s, bits, w, y,
                       pooled, N, HW, C, J);
    return check_launch();
}

}  // namespace bnn
