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

// First layer: fp32 convolution, zero padding, then per-channel threshold -> bits.
// One lane per output pixel, one wave per group of 16 output channels (weights of a wave are
// uniform and come through the scalar cache); the 4 waves of a workgroup cover 64 channels of the
// same 64 pixels.  Weights are read in the caller's [O][k][k][C] order.
__global__ __launch_bounds__(256) void conv_f32_kernel(const float* __restrict__ x, const float* __restrict__ w,
                                                       const float* __restrict__ thr, float* __restrict__ y,
                                                       uint32_t* __restrict__ bits, int N, int H, int W, int C,
                                                       int O, int k, int stride, int pad, int P, int Q) {
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
    const long long npix = (long long)N * P * Q;
    const long long pix_raw = (long long)blockIdx.x * 64 + lane;
    const bool pix_ok = pix_raw < npix;
    const long long pix = pix_ok ? pix_raw : npix - 1;
    const int o0 = ((int)blockIdx.y * 4 + wave) * 16;
    if (o0 >= O) return;
    const int n = (int)(pix / (P * Q));
    const int rem = (int)(pix - (long long)n * P * Q);
    const int p = rem / Q, q = rem - p * Q;
    const int y0 = p * stride - pad, x0 = q * stride - pad;
    float acc[16];
#pragma unroll
    for (int j = 0; j < 16; ++j) acc[j] = 0.f;
    const int kkc = k * k * C;
    for (int r = 0; r < k; ++r) {
        for (int s = 0; s < k; ++s) {
            const int yy = y0 + r, xx = x0 + s;
            const bool inside = (unsigned)yy < (unsigned)H && (unsigned)xx < (unsigned)W;
            const float* xp = x + (((long long)n * H + (inside ? yy : 0)) * W + (inside ? xx : 0)) * C;
            const float* wp = w + (r * k + s) * C;
            for (int c = 0; c < C; ++c) {
                const float xv = inside ? xp[c] : 0.f;
#pragma unroll
                for (int j = 0; j < 16; ++j) {
                    const int o = min(o0 + j, O - 1);
                    acc[j] = fmaf(xv, wp[(long long)o * kkc + c], acc[j]);
                }
            }
        }
    }
    if (!pix_ok) return;
    uint32_t word = 0u;
#pragma unroll
    for (int j = 0; j < 16; ++j) {
        const int o = o0 + j;
        if (o < O) {
            if (y != nullptr) y[pix * O + o] = acc[j];
            if (bits != nullptr && acc[j] >= thr[o]) word |= (1u << j);
        }
    }
    if (bits != nullptr) {
        // 16 channels = one half word; the two halves of a word are written by different waves
        uint16_t* hb = reinterpret_cast<uint16_t*>(bits + pix * (long long)((O + 31) / 32));
        hb[o0 >> 4] = (uint16_t)word;
    }
}

// When O is not a multiple of 32 the upper half word of the last word may belong to no wave.
__global__ void conv_f32_padfix_kernel(uint32_t* bits, long long npix, int O) {
    const long long pix = (long long)blockIdx.x * blockDim.x + threadIdx.x;
    if (pix >= npix) return;
    uint16_t* hb = reinterpret_cast<uint16_t*>(bits + pix * (long long)((O + 31) / 32));
    hb[((O + 31) / 32) * 2 - 1] = 0;
}

// Head: exact integer sum-pool of +1/-1 over HW positions, then fp32 FC.  One workgroup handles
// IMGS images so that each weight row is read once per IMGS images; one wave per output row j,
// lanes stride over channels, wave reduction at the end.
constexpr int HEAD_IMGS = 8;
constexpr int HEAD_MAXC = 1024;

__global__ __launch_bounds__(256) void head_kernel(const uint32_t* __restrict__ bits, const float* __restrict__ w,
                                                   float* __restrict__ y, int32_t* __restrict__ pooled_out,
                                                   int N, int HW, int C, int J) {
    __shared__ float pooled[HEAD_IMGS][HEAD_MAXC];
    const int n0 = blockIdx.x * HEAD_IMGS;
    const int cw = (C + 31) / 32;
    const float inv = (float)HW;
    for (int idx = threadIdx.x; idx < HEAD_IMGS * C; idx += blockDim.x) {
        const int im = idx / C, c = idx - im * C;
        const int n = n0 + im;
        int s = 0;
        if (n < N) {
            const uint32_t* b = bits + (long long)n * HW * cw + (c >> 5);
            for (int i = 0; i < HW; ++i) s += ((b[(long long)i * cw] >> (c & 31)) & 1u) ? 1 : -1;
            if (pooled_out != nullptr) pooled_out[(long long)n * C + c] = s;
        }
        pooled[im][c] = (float)s / inv;
    }
    __syncthreads();
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    for (int j = wave; j < J; j += 4) {
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
    dim3 grid((unsigned)cdiv(npix, 64), (unsigned)cdiv(O, 64));
    hipLaunchKernelGGL(conv_f32_kernel, grid, dim3(256), 0, s, x, w, thr, y, bits, N, H, W, C, O, k, stride, pad, P, Q);
    int rc = check_launch();
    if (rc == BNN_OK && bits != nullptr && (O % 32) != 0 && (O % 32) <= 16) {
        hipLaunchKernelGGL(conv_f32_padfix_kernel, dim3((unsigned)cdiv(npix, 256)), dim3(256), 0, s, bits, npix, O);
        rc = check_launch();
    }
    return rc;
}

int launch_head_f32(const uint32_t* bits, const float* w, float* y, int32_t* pooled, int N, int HW, int C, int J,
                    hipStream_t s) {
    if (C > HEAD_MAXC) return BNN_ERR_UNSUPPORTED;
    hipLaunchKernelGGL(head_kernel, dim3((unsigned)cdiv(N, HEAD_IMGS)), dim3(256), 0, s, bits, w, y, pooled, N, HW, C, J);
    return check_launch();
}

}  // namespace bnn
