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

// Re-tiles a packed operand for the matrix-core fragment loads (the idea of the paper's FSB format, Sec. 5.1,
// with this chip's tile): rows are grouped by 32; a group stores, for every 16-byte step along K, the 16 bytes
// of its 32 rows back to back.  Unit (16 bytes) u of row r goes to ((r / 32) * units_per_row + u) * 32 + r % 32.
// Rows past N in the last group are written as zeros.  One thread per destination unit.
__global__ __launch_bounds__(256) void tile_b_kernel(const uint4* __restrict__ B, uint4* __restrict__ Bt, int N, int upr,
                                                     long long nunits) {
    const long long d = (long long)blockIdx.x * 256 + threadIdx.x;
    if (d >= nunits) return;
    const int r32 = (int)(d & 31);
    const long long gu = d >> 5;
    const long long grp = gu / upr;
    const int u = (int)(gu - grp * upr);
    const long long row = grp * 32 + r32;
    Bt[d] = row < N ? B[row * upr + u] : make_uint4(0u, 0u, 0u, 0u);
}

// K-panel layout (the fixed-stride idea of Sec. 5.1 with this chip's sizes): K is cut into panels of 256 bits and panel p
// stores its 32 bytes of every row back to back, so 16-byte unit u of row r sits at unit ((u / 2) * rows + r) * 2 + u % 2.
// The last panel is filled up with 0 bits.  One thread per destination unit, both directions.
__global__ __launch_bounds__(256) void panels_from_rows_kernel(const uint32_t* __restrict__ X, uint4* __restrict__ Xp, long long rows,
                                                               int K, int ldx_w, long long nunits) {
    const long long d = (long long)blockIdx.x * 256 + threadIdx.x;
    if (d >= nunits) return;
    const long long t = d >> 1;
    const long long panel = t / rows;
    const long long r = t - panel * rows;
    const int w0 = (int)(panel * 8 + 4 * (d & 1));
    uint32_t w[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int left = K - 32 * (w0 + i);          // logical bits from this word on
        const uint32_t v = left > 0 ? X[r * ldx_w + w0 + i] : 0u;
        w[i] = left >= 32 ? v : left > 0 ? v & (0xFFFFFFFFu >> (32 - left)) : 0u;
    }
    Xp[d] = make_uint4(w[0], w[1], w[2], w[3]);
}

__global__ __launch_bounds__(256) void rows_from_panels_kernel(const uint4* __restrict__ Xp, uint4* __restrict__ X, long long rows,
                                                               int npanels, int upr, long long nunits) {
    const long long d = (long long)blockIdx.x * 256 + threadIdx.x;
    if (d >= nunits) return;
    const long long r = d / upr;
    const int u = (int)(d - r * upr);
    X[d] = (u >> 1) < npanels ? Xp[((long long)(u >> 1) * rows + r) * 2 + (u & 1)] : make_uint4(0u, 0u, 0u, 0u);
}

// Load-latency probe in the manner of the paper's Sec. 4.1 (latency of a tile load against the row stride):
// one wave repeatedly loads the operand fragment of one MFMA -- lane l reads 16 bytes of row l % 32 at byte
// offset 16 * (l / 32) -- from rows `stride` bytes apart, walking along K.  dependent = 1 chains each address
// on the previous load's data (pure latency), 0 issues them back to back (throughput of one wave).
// cycles[0] = ticks of the shader cycle counter for `iters` loads, cycles[1] = a checksum that keeps the loads alive.
__global__ __launch_bounds__(64) void probe_stride_kernel(const uint32_t* __restrict__ buf, long long* __restrict__ cycles,
                                                          int stride_bytes, int rows, int iters, int dependent) {
    const int lane = threadIdx.x;
    const int r = lane & 31, half = lane >> 5;
    const int steps = stride_bytes / 32;                     // fragment positions along a row (32 bytes each)
    const char* base = reinterpret_cast<const char*>(buf) + (long long)r * stride_bytes + half * 16;
    unsigned sum = 0;
    int step = 0, row0 = 0;
    auto advance = [&]() {
        if (++step >= steps) { step = 0; row0 += 32; if (row0 + 32 > rows) row0 = 0; }
    };
    const long long t0 = __builtin_readcyclecounter();
    if (dependent) {
        for (int it = 0; it < iters; ++it) {
            const uint4 v = *reinterpret_cast<const uint4*>(base + (long long)row0 * stride_bytes + step * 32);
            sum += v.y ^ v.z ^ v.w;
            step += (int)v.x;                                // the buffer holds zeros: a data dependence, same addresses
            advance();
        }
    } else {
        for (int it = 0; it < iters; it += 8) {              // eight loads in flight
            uint4 v[8];
#pragma unroll
            for (int u = 0; u < 8; ++u) {
                v[u] = *reinterpret_cast<const uint4*>(base + (long long)row0 * stride_bytes + step * 32);
                advance();
            }
#pragma unroll
            for (int u = 0; u < 8; ++u) sum += v[u].x ^ v[u].y ^ v[u].z ^ v[u].w;
        }
    }
    const long long t1 = __builtin_readcyclecounter();
    if (lane == 0) cycles[0] = t1 - t0;
    if (sum == 0x12345u && lane == 1) cycles[1] = sum;
}

// Max-pooling of +1/-1 activations after the threshold = bitwise OR of the packed words of the
// window (Sec. 6.1).  One thread per output word.
__global__ __launch_bounds__(256) void maxpool_or_kernel(const uint32_t* __restrict__ in, uint32_t* __restrict__ out,
                                                         long long nwords_out, int H, int W, int cw, int P, int Q,
                                                         int win, int stride) {
    const long long idx = (long long)blockIdx.x * blockDim.x + threadIdx.x;
    if (idx >= nwords_out) return;
    const int wi = (int)(idx % cw);
    long long pix = idx / cw;
    const int q = (int)(pix % Q); pix /= Q;
    const int p = (int)(pix % P);
    const long long n = pix / P;
    const uint32_t* base = in + ((n * H + (long long)p * stride) * W + (long long)q * stride) * cw + wi;
    uint32_t v = 0u;
    for (int r = 0; r < win; ++r)
        for (int t = 0; t < win; ++t) v |= base[((long long)r * W + t) * cw];
    out[idx] = v;
}

// First layer: fp32 convolution with zero padding, then per-channel threshold -> bits, as an
// implicit GEMM on the fp32 matrix cores (v_mfma_f32_32x32x2_f32): rows are output pixels,
// columns output channels, and K runs over the k filter rows times the k*C contiguous floats of
// one filter row, which are contiguous in the NHWC input as well.  That segment is cut in blocks
// of 24 floats; in a block the lower half-wave takes floats 0..11 and the upper one 12..23 (any
// pairing of K indices is fine as long as both operands use it), so every lane reads a run of 12
// consecutive floats with three 16-byte loads, a whole block ahead of the MFMAs that use it.
// The 64 x k*k*C weights of the workgroup live in LDS.  A wave owns 2 x 2 accumulator tiles
// (64 pixels x 64 channels), a workgroup 256 pixels.
typedef float v16f_aux __attribute__((ext_vector_type(16)));
typedef float float4_u __attribute__((ext_vector_type(4), aligned(4)));
extern "C" __device__ int bnn_aux_writelane_i32(int val, int lane, int old) __asm("llvm.amdgcn.writelane.i32");

constexpr int STEM_MT = 2, STEM_NT = 2, STEM_RUN = 12;

__global__ __launch_bounds__(256) void conv_f32_kernel(const float* __restrict__ x, const float* __restrict__ w,
                                                       const float* __restrict__ thr, float* __restrict__ y,
                                                       uint32_t* __restrict__ bits, int N, int H, int W, int C,
                                                       int O, int k, int stride, int pad, int P, int Q) {
    const int lane = threadIdx.x & 63, l32 = lane & 31, half = lane >> 5, wave = threadIdx.x >> 6;
    const long long npix = (long long)N * P * Q;
    const int n0 = (int)blockIdx.y * (STEM_NT * 32);
    const int seg = k * C;                                   // floats in one filter row
    const int nblk = (seg + 2 * STEM_RUN - 1) / (2 * STEM_RUN);
    const int rowlen = W * C;
    const long long total = (long long)N * H * rowlen;       // floats in x

    // weights of this workgroup's 64 output channels -> LDS (row stride odd: 32 channels, 32 banks)
    extern __shared__ float wlds[];
    const int kkc = k * seg;
    const int wstride = kkc | 1;
    {
        // 8 independent loads in flight per thread; channels past O repeat the last valid floats
        // (their results are dropped)
        const long long wbase = (long long)n0 * kkc, wlast = (long long)O * kkc - 1;
        const int nelem = STEM_NT * 32 * kkc;
        for (int base = 0; base < nelem; base += 8 * 256) {
            float tmp[8];
#pragma unroll
            for (int u = 0; u < 8; ++u) {
                const int idx = base + u * 256 + (int)threadIdx.x;
                tmp[u] = w[min(wbase + min(idx, nelem - 1), wlast)];
            }
#pragma unroll
            for (int u = 0; u < 8; ++u) {
                const int idx = base + u * 256 + (int)threadIdx.x;
                if (idx < nelem) {
                    const int c = idx / kkc;
                    wlds[c * wstride + (idx - c * kkc)] = tmp[u];
                }
            }
        }
        // the slack after the last row is read (times an A value of 0) by padded K indices: keep it finite
        if (threadIdx.x < 2 * STEM_RUN) wlds[STEM_NT * 32 * wstride + threadIdx.x] = 0.f;
        if (wstride > kkc && threadIdx.x < STEM_NT * 32) wlds[threadIdx.x * wstride + kkc] = 0.f;   // row pad
    }
    __syncthreads();

    const long long m0 = ((long long)blockIdx.x * 4 + wave) * (STEM_MT * 32);
    if (m0 >= npix) return;                                  // uniform per wave, after the barrier

    long long xbase[STEM_MT];       // float index of input row 0 of this lane's image
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
        xbase[i] = (long long)n * H * rowlen;
    }

    v16f_aux acc[STEM_MT][STEM_NT];
#pragma unroll
    for (int i = 0; i < STEM_MT; ++i)
#pragma unroll
        for (int j = 0; j < STEM_NT; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

    // Loads the run of floats of filter row r, block blk, for every A fragment; positions that are
    // padding (outside the image) become 0.  A block covers bl <= 24 floats of the segment, split
    // evenly: the lower half-wave takes the first hs = ceil(bl/2), the upper one the rest.
    auto fetch = [&](int r, int blk, float (&run)[STEM_MT][STEM_RUN]) {
        const int bl = min(2 * STEM_RUN, seg - blk * (2 * STEM_RUN));
        const int hs = (bl + 1) >> 1;
        const int e0 = blk * (2 * STEM_RUN) + half * hs;             // first float of this lane's run
        const int cnt = half ? bl - hs : hs;                         // floats of the run that exist
#pragma unroll
        for (int i = 0; i < STEM_MT; ++i) {
            const int yy = ytop[i] + r;
            const bool yok = (unsigned)yy < (unsigned)H;
            const long long start = xbase[i] + (long long)(yok ? yy : 0) * rowlen + xoff[i] + e0;
            if (start >= 0 && start + STEM_RUN <= total) {           // the whole run lies inside the tensor
                const float4_u v0 = *reinterpret_cast<const float4_u*>(x + start);
                const float4_u v1 = *reinterpret_cast<const float4_u*>(x + start + 4);
                const float4_u v2 = *reinterpret_cast<const float4_u*>(x + start + 8);
#pragma unroll
                for (int t = 0; t < 4; ++t) { run[i][t] = v0[t]; run[i][4 + t] = v1[t]; run[i][8 + t] = v2[t]; }
            } else {                                                 // first / last pixels of the tensor
#pragma unroll
                for (int t = 0; t < STEM_RUN; ++t) {
                    const long long idx = start + t;
                    run[i][t] = (idx >= 0 && idx < total) ? x[idx] : 0.f;
                }
            }
            // zero padding; skipped when every lane of the wave has its whole run inside the image
            const int xs = xoff[i] + e0;
            const bool inside = yok && xs >= 0 && xs + cnt <= rowlen && cnt == hs;
            if (__builtin_amdgcn_ballot_w64(inside) != ~0ull) {
#pragma unroll
                for (int t = 0; t < STEM_RUN; ++t) {
                    const bool ok = yok && t < cnt && (unsigned)(xs + t) < (unsigned)rowlen;
                    run[i][t] = ok ? run[i][t] : 0.f;
                }
            }
        }
    };

    // Weights come from LDS unmasked: where a K index is padding the A value is 0.
    auto multiply = [&](int r, int blk, const float (&run)[STEM_MT][STEM_RUN]) {
        const int bl = min(2 * STEM_RUN, seg - blk * (2 * STEM_RUN));
        const int hs = (bl + 1) >> 1;                                // K-steps of this block (uniform)
        const float* wp[STEM_NT];
#pragma unroll
        for (int j = 0; j < STEM_NT; ++j) wp[j] = wlds + (32 * j + l32) * wstride + r * seg + blk * (2 * STEM_RUN) + half * hs;
#pragma unroll
        for (int t = 0; t < STEM_RUN; ++t) {
            if (t < hs) {
                float b[STEM_NT];
#pragma unroll
                for (int j = 0; j < STEM_NT; ++j) b[j] = wp[j][t];
#pragma unroll
                for (int i = 0; i < STEM_MT; ++i)
#pragma unroll
                    for (int j = 0; j < STEM_NT; ++j)
                        acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(run[i][t], b[j], acc[i][j], 0, 0, 0);
            }
        }
    };

    const int total_blocks = k * nblk;
    float run0[STEM_MT][STEM_RUN], run1[STEM_MT][STEM_RUN];
    fetch(0, 0, run0);
    int r = 0, blk = 0;
    for (int it = 0; it < total_blocks; it += 2) {
        int r1 = r, b1 = blk + 1;
        if (b1 == nblk) { b1 = 0; ++r1; }
        if (it + 1 < total_blocks) fetch(r1, b1, run1);
        multiply(r, blk, run0);
        if (it + 1 < total_blocks) {
            int r2 = r1, b2 = b1 + 1;
            if (b2 == nblk) { b2 = 0; ++r2; }
            if (it + 2 < total_blocks) fetch(r2, b2, run0);
            multiply(r1, b1, run1);
            r = r2; blk = b2;
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

// Head: exact integer sum-pool of +1/-1 over HW positions, then fp32 FC.  A workgroup handles HEAD_IMGS images
// and HEAD_OUTS output rows.  Pooling: a thread owns one packed word (32 channels) of one image and counts set
// bits per channel over the HW positions, 4 channels at a time in the bytes of one register (HW <= 255); the sum
// of +1/-1 is 2 * count - HW.  FC: the pooled values and the weight rows of the workgroup are staged in LDS,
// channel-major ([c][image] and [c][output], rows padded by one float against bank conflicts), and thread
// (image, output) walks the channels: no cross-lane reduction.
constexpr int HEAD_IMGS = 16;
constexpr int HEAD_OUTS = 16;
constexpr int HEAD_MAXC = 1024;
constexpr int HEAD_LD = 17;                              // floats per channel row in LDS (16 + 1 pad)

__global__ __launch_bounds__(256) void head_kernel(const uint32_t* __restrict__ bits, const float* __restrict__ w,
                                                   float* __restrict__ y, int32_t* __restrict__ pooled_out,
                                                   int N, int HW, int C, int J) {
    extern __shared__ float head_lds[];
    float* pooled = head_lds;                            // [C][HEAD_LD]: pooled[c][image]
    float* wt = head_lds + (size_t)C * HEAD_LD;          // [C][HEAD_LD]: wt[c][output]
    const int n0 = blockIdx.x * HEAD_IMGS;
    const int j0 = blockIdx.y * HEAD_OUTS;
    const int cw = (C + 31) / 32;
    const float inv = (float)HW;
    // weight rows of this workgroup, transposed into LDS (coalesced reads along c), eight loads in flight per thread
    {
        const int total = HEAD_OUTS * C;
        for (int base = 0; base < total; base += 8 * 256) {
            float tmp[8];
#pragma unroll
            for (int u = 0; u < 8; ++u) {
                const int idx = base + u * 256 + (int)threadIdx.x;
                const int jj = idx / C, c = idx - jj * C;
                tmp[u] = (idx < total && j0 + jj < J) ? w[(long long)(j0 + jj) * C + c] : 0.f;
            }
#pragma unroll
            for (int u = 0; u < 8; ++u) {
                const int idx = base + u * 256 + (int)threadIdx.x;
                const int jj = idx / C, c = idx - jj * C;
                if (idx < total) wt[c * HEAD_LD + jj] = tmp[u];
            }
        }
    }
    for (int idx = threadIdx.x; idx < HEAD_IMGS * cw; idx += blockDim.x) {
        const int im = idx / cw, wi = idx - im * cw;
        const int n = n0 + im;
        uint32_t cnt[8];                       // byte t of cnt[q] = number of set bits of channel q + 8*t of this word
#pragma unroll
        for (int q = 0; q < 8; ++q) cnt[q] = 0u;
        if (n < N) {
            const uint32_t* b = bits + (long long)n * HW * cw + wi;
            for (int i0 = 0; i0 < HW; i0 += 16) {           // 16 independent loads in flight
                uint32_t v[16];
#pragma unroll
                for (int u = 0; u < 16; ++u) v[u] = (i0 + u < HW) ? b[(long long)(i0 + u) * cw] : 0u;
#pragma unroll
                for (int u = 0; u < 16; ++u)
#pragma unroll
                    for (int q = 0; q < 8; ++q) cnt[q] += (v[u] >> q) & 0x01010101u;
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
                    pooled[c * HEAD_LD + im] = (float)s / inv;
                }
            }
    }
    __syncthreads();
    // thread -> (image, output); four independent partial sums shorten the dependent chain
    const int im = threadIdx.x & (HEAD_IMGS - 1), jj = threadIdx.x / HEAD_IMGS;
    float p0 = 0.f, p1 = 0.f, p2 = 0.f, p3 = 0.f;
    int c = 0;
    for (; c + 4 <= C; c += 4) {
        p0 = fmaf(pooled[(c + 0) * HEAD_LD + im], wt[(c + 0) * HEAD_LD + jj], p0);
        p1 = fmaf(pooled[(c + 1) * HEAD_LD + im], wt[(c + 1) * HEAD_LD + jj], p1);
        p2 = fmaf(pooled[(c + 2) * HEAD_LD + im], wt[(c + 2) * HEAD_LD + jj], p2);
        p3 = fmaf(pooled[(c + 3) * HEAD_LD + im], wt[(c + 3) * HEAD_LD + jj], p3);
    }
    for (; c < C; ++c) p0 = fmaf(pooled[c * HEAD_LD + im], wt[c * HEAD_LD + jj], p0);
    if (n0 + im < N && j0 + jj < J) y[(long long)(n0 + im) * J + j0 + jj] = (p0 + p1) + (p2 + p3);
}

// The same head as two kernels, for callers that give it a place for the pooled sums: the pooling runs once per
// image instead of once per (image group, output group) workgroup, and the FC runs on the matrix cores.
// Pooling: four adjacent lanes share one packed word (32 channels) of one image, each counting every fourth
// position (set bits per channel, 4 channels at a time in the bytes of one register: HW <= 255); the four partial
// counts meet through lane exchanges, and lane t of the four writes channels q + 8 t.
__global__ __launch_bounds__(256) void head_pool_kernel(const uint32_t* __restrict__ bits, int32_t* __restrict__ pooled_out,
                                                        int N, int HW, int C) {
    const int cw = (C + 31) / 32;
    const long long idx = (long long)blockIdx.x * blockDim.x + threadIdx.x;
    const long long item = idx >> 2;
    const int part = (int)(idx & 3);
    const bool live = item < (long long)N * cw;            // whole groups of four lanes are live or not
    const int n = live ? (int)(item / cw) : 0, wi = live ? (int)(item - (long long)n * cw) : 0;
    uint32_t cnt[8];
#pragma unroll
    for (int q = 0; q < 8; ++q) cnt[q] = 0u;
    const uint32_t* b = bits + (long long)n * HW * cw + wi;
    for (int i0 = part; i0 < HW; i0 += 64) {               // 16 independent loads in flight
        uint32_t v[16];
#pragma unroll
        for (int u = 0; u < 16; ++u) v[u] = (live && i0 + 4 * u < HW) ? b[(long long)(i0 + 4 * u) * cw] : 0u;
#pragma unroll
        for (int u = 0; u < 16; ++u)
#pragma unroll
            for (int q = 0; q < 8; ++q) cnt[q] += (v[u] >> q) & 0x01010101u;
    }
#pragma unroll
    for (int q = 0; q < 8; ++q) {
        cnt[q] += (uint32_t)__shfl_xor((int)cnt[q], 1);
        cnt[q] += (uint32_t)__shfl_xor((int)cnt[q], 2);
    }
    if (!live) return;
#pragma unroll
    for (int q = 0; q < 8; ++q) {
        const int c = wi * 32 + q + 8 * part;
        if (c < C) pooled_out[(long long)n * C + c] = 2 * (int)((cnt[q] >> (8 * part)) & 0xFFu) - HW;
    }
}

// FC on the pooled sums with the fp32 matrix instruction (exact fp32 products, fp32 accumulation): a workgroup
// computes 32 images x 32 outputs, its eight waves taking every eighth step of 8 channels; lane l holds image /
// output l % 32 and channels 4 * (l / 32) .. + 3 of the step, one MFMA per channel pair.  The eight partial tiles meet
// in LDS; the division by HW is applied once, to the finished sum.  VEC: C is a multiple of 4 (16-byte loads).
// (Eight waves: at 512 channels every wave has all of its loads in flight at once -- one memory round trip; a lane's
// loads go to 32 different rows, so what a wave can have in flight is what bounds this kernel.)
typedef float fc_v16f __attribute__((ext_vector_type(16)));
constexpr int FC_STEPS = 8;                     // steps (of 8 channels) a wave requests before it multiplies them
constexpr int FC_WAVES = 8;

template <bool VEC>
__global__ __launch_bounds__(64 * FC_WAVES) void head_fc_kernel(const int32_t* __restrict__ pooled, const float* __restrict__ w,
                                                                float* __restrict__ y, int N, int HW, int C, int J) {
    __shared__ float red[FC_WAVES][16 * 64];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int l32 = lane & 31, half = lane >> 5;
    const int n0 = blockIdx.x * 32, j0 = blockIdx.y * 32;
    const bool nok = n0 + l32 < N, jok = j0 + l32 < J;
    const int32_t* prow = pooled + (long long)min(n0 + l32, N - 1) * C;
    const float* wrow = w + (long long)min(j0 + l32, J - 1) * C;
    fc_v16f acc;
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[r] = 0.f;
    const int steps = (C + 7) / 8;
    for (int s0 = wave; s0 < steps; s0 += FC_WAVES * FC_STEPS) {
        float a[FC_STEPS][4], b[FC_STEPS][4];
#pragma unroll
        for (int u = 0; u < FC_STEPS; ++u) {
            const int c = 8 * (s0 + FC_WAVES * u) + 4 * half;
            if (VEC) {
                const bool ok = c < C;                      // C % 4 == 0: the four channels are in range together
                const int4 pa = (ok && nok) ? *reinterpret_cast<const int4*>(prow + c) : make_int4(0, 0, 0, 0);
                const float4 wb = (ok && jok) ? *reinterpret_cast<const float4*>(wrow + c) : make_float4(0.f, 0.f, 0.f, 0.f);
                a[u][0] = (float)pa.x; a[u][1] = (float)pa.y; a[u][2] = (float)pa.z; a[u][3] = (float)pa.w;
                b[u][0] = wb.x; b[u][1] = wb.y; b[u][2] = wb.z; b[u][3] = wb.w;
            } else {
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    a[u][q] = (c + q < C && nok) ? (float)prow[c + q] : 0.f;
                    b[u][q] = (c + q < C && jok) ? wrow[c + q] : 0.f;
                }
            }
        }
#pragma unroll
        for (int u = 0; u < FC_STEPS; ++u)
#pragma unroll
            for (int q = 0; q < 4; ++q) acc = __builtin_amdgcn_mfma_f32_32x32x2f32(a[u][q], b[u][q], acc, 0, 0, 0);
    }
#pragma unroll
    for (int r = 0; r < 16; ++r) red[wave][r * 64 + lane] = acc[r];
    __syncthreads();
    // thread (wave, lane) finishes accumulator registers 2 * wave, 2 * wave + 1 of lane (register r: row 8 * (r / 4) +
    // 4 * half + r % 4)
    const float inv = (float)HW;
#pragma unroll
    for (int q = 0; q < 16 / FC_WAVES; ++q) {
        const int r = (16 / FC_WAVES) * wave + q;
        float sum = 0.f;
#pragma unroll
        for (int wv = 0; wv < FC_WAVES; ++wv) sum += red[wv][r * 64 + lane];
        const int row = n0 + 8 * (r >> 2) + 4 * half + (r & 3), col = j0 + l32;
        if (row < N && col < J) y[(long long)row * J + col] = sum / inv;
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

// Binarization by sign (Eq. 1: x >= 0 -> +1) of a row-major fp32 matrix with row stride ldx.
int launch_sign_pack_f32(const float* x, uint32_t* bits, long long rows, int cols, int ldx, int ldb_w, hipStream_t s) {
    hipLaunchKernelGGL((pack_kernel<float, float, true>), dim3((unsigned)cdiv(rows, 4)), dim3(256), 0, s,
                       x, nullptr, 0.f, bits, rows, cols, ldx, ldb_w);
    return check_launch();
}

int launch_tile_b(const uint32_t* B, uint32_t* Bt, int N, int ldb_w, hipStream_t s) {
    const int upr = ldb_w / 4;
    const long long nunits = cdiv(N, 32) * 32 * (long long)upr;
    hipLaunchKernelGGL(tile_b_kernel, dim3((unsigned)cdiv(nunits, 256)), dim3(256), 0, s, reinterpret_cast<const uint4*>(B),
                       reinterpret_cast<uint4*>(Bt), N, upr, nunits);
    return check_launch();
}

int launch_panels_from_rows(const uint32_t* X, uint32_t* Xp, long long rows, int K, int ldx_w, hipStream_t s) {
    const long long nunits = cdiv(K, 256) * rows * 2;
    hipLaunchKernelGGL(panels_from_rows_kernel, dim3((unsigned)cdiv(nunits, 256)), dim3(256), 0, s, X, reinterpret_cast<uint4*>(Xp),
                       rows, K, ldx_w, nunits);
    return check_launch();
}

int launch_rows_from_panels(const uint32_t* Xp, uint32_t* X, long long rows, int K, int ldx_w, hipStream_t s) {
    const int upr = ldx_w / 4;
    const long long nunits = rows * upr;
    hipLaunchKernelGGL(rows_from_panels_kernel, dim3((unsigned)cdiv(nunits, 256)), dim3(256), 0, s,
                       reinterpret_cast<const uint4*>(Xp), reinterpret_cast<uint4*>(X), rows, (int)cdiv(K, 256), upr, nunits);
    return check_launch();
}

int launch_probe_stride(const uint32_t* buf, long long* cycles, int stride_bytes, int rows, int iters, int dependent,
                        hipStream_t s) {
    hipLaunchKernelGGL(probe_stride_kernel, dim3(1), dim3(64), 0, s, buf, cycles, stride_bytes, rows, iters, dependent);
    return check_launch();
}

int launch_unpack_i32(const uint32_t* bits, int32_t* out, long long rows, int cols, int ldb_w, int ldo, hipStream_t s) {
    dim3 grid((unsigned)min((long long)cdiv(cols, 256), 64LL), (unsigned)min(rows, 65535LL));
    hipLaunchKernelGGL(unpack_kernel, grid, dim3(256), 0, s, bits, out, rows, cols, ldb_w, ldo);
    return check_launch();
}

int launch_maxpool_or(const uint32_t* in, uint32_t* out, int N, int H, int W, int C, int win, int stride, hipStream_t s) {
    const int P = (H - win) / stride + 1, Q = (W - win) / stride + 1, cw = (C + 31) / 32;
    const long long n = (long long)N * P * Q * cw;
    hipLaunchKernelGGL(maxpool_or_kernel, dim3((unsigned)cdiv(n, 256)), dim3(256), 0, s, in, out, n, H, W, cw, P, Q, win, stride);
    return check_launch();
}

int launch_conv_f32_thr(const float* x, const float* w, const float* thr, float* y, uint32_t* bits,
                        int N, int H, int W, int C, int O, int k, int stride, int pad, hipStream_t s) {
    const int P = (H + 2 * pad - k) / stride + 1, Q = (W + 2 * pad - k) / stride + 1;
    const long long npix = (long long)N * P * Q;
    dim3 grid((unsigned)cdiv(npix, 4 * STEM_MT * 32), (unsigned)cdiv(O, STEM_NT * 32));
    // + slack: the unmasked weight reads of a padded K index may run a few floats past the last row
    const size_t lds_bytes = ((size_t)STEM_NT * 32 * ((k * k * C) | 1) + 2 * STEM_RUN) * sizeof(float);
    if (lds_bytes > 160 * 1024) return BNN_ERR_UNSUPPORTED;  // more than ~630 filter taps*channels per output
    if (lds_bytes > 64 * 1024) {
        static const hipError_t attr = hipFuncSetAttribute(reinterpret_cast<const void*>(&conv_f32_kernel),
                                                           hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
        if (attr != hipSuccess) return BNN_ERR_DEVICE;
    }
    hipLaunchKernelGGL(conv_f32_kernel, grid, dim3(256), lds_bytes, s, x, w, thr, y, bits, N, H, W, C, O, k, stride, pad, P,
                       Q);
    return check_launch();
}

int launch_head_f32(const uint32_t* bits, const float* w, float* y, int32_t* pooled, int N, int HW, int C, int J,
                    hipStream_t s) {
    if (C > HEAD_MAXC || HW > 255) return BNN_ERR_UNSUPPORTED;
    if (pooled != nullptr) {
        const long long lanes = 4LL * N * ((C + 31) / 32);
        hipLaunchKernelGGL(head_pool_kernel, dim3((unsigned)cdiv(lanes, 256)), dim3(256), 0, s, bits, pooled, N, HW, C);
        const dim3 grid((unsigned)cdiv(N, 32), (unsigned)cdiv(J, 32));
        const bool vec = C % 4 == 0 && ((reinterpret_cast<uintptr_t>(w) | reinterpret_cast<uintptr_t>(pooled)) & 15u) == 0;
        if (vec) hipLaunchKernelGGL(head_fc_kernel<true>, grid, dim3(64 * FC_WAVES), 0, s, pooled, w, y, N, HW, C, J);
        else hipLaunchKernelGGL(head_fc_kernel<false>, grid, dim3(64 * FC_WAVES), 0, s, pooled, w, y, N, HW, C, J);
        return check_launch();
    }
    const size_t lds_bytes = (size_t)2 * C * HEAD_LD * sizeof(float);
    if (lds_bytes > 64 * 1024) {
        static const hipError_t attr = hipFuncSetAttribute(reinterpret_cast<const void*>(&head_kernel),
                                                           hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
        if (attr != hipSuccess) return BNN_ERR_DEVICE;
    }
    hipLaunchKernelGGL(head_kernel, dim3((unsigned)cdiv(N, HEAD_IMGS), (unsigned)cdiv(J, HEAD_OUTS)), dim3(256), lds_bytes, s, bits,
                       w, y, pooled, N, HW, C, J);
    return check_launch();
}

}  // namespace bnn
