// First layer with binarized weights (paper Sec. 6.1, "BWN"): real-valued NHWC input, one bit per
// weight, out[n][p][q][o] = sum over the window of (+x if the weight bit is 1, -x if it is 0), zero
// padding, then the fused threshold -> packed bits.
//
// gfx950 design.  The paper adds or subtracts element by element on the scalar cores because Turing's
// bit tensor cores cannot take a real-valued operand.  Here the layer runs on the bf16 matrix cores
// (16x the fp32 MFMA rate) without giving up fp32 inputs: every fp32 input value is split exactly into
// three bf16 terms x = h + m + l (8 significant bits each), the +1/-1 weights are exact in bf16, so each
// product is exact and the sum is accumulated in fp32 by v_mfma_f32_32x32x16_bf16 -- the same result, up
// to the order of the fp32 additions, as an fp32 multiply-accumulate.
//
// Implicit GEMM: a GEMM row is an output pixel, a column an output channel.  K is covered by "runs" of
// 8 consecutive elements of one filter row (the k*C values of a filter row are contiguous in NHWC): a lane
// supplies the 8 K-slots of its half-wave for one MFMA from one run.  K-slots that would count an element
// twice or that hold no element get weight 0, so the input side needs no mask for them.  A small kernel
// first expands the weight bits into bf16 in fragment order [channel tile][run][channel][8 x bf16]
// (caller's workspace); every workgroup copies its channel tile to LDS with plain 16-byte loads and reads
// one 16-byte unit per MFMA operand.
//
// Two kernels:
//  * LDS-staged (default).  A workgroup owns a rectangle of output pixels of one image.  It loads the
//    input patch under that rectangle once with coalesced loads, splits every value once, and keeps the
//    three bf16 planes in LDS ([plane][patch row][pixel][Cp], Cp = C padded so that a pixel step is a
//    multiple of 8 bytes).  The K loop then only reads LDS (two 8-byte reads per operand) and issues MFMAs;
//    zero padding is written at staging time.  This removes the k*k/stride^2-fold re-splitting and
//    re-masking of the same input value by neighbouring output pixels that bounds the direct kernel.
//  * Direct (fallback when patch + weights exceed LDS).  Every lane loads its runs straight from global
//    memory two K-steps ahead and splits them in registers.
#include <type_traits>

#include "bnn_internal.h"

namespace bnn {
namespace {

typedef float v16f_bwn __attribute__((ext_vector_type(16)));
typedef __bf16 v8bf_bwn __attribute__((ext_vector_type(8)));
typedef float float4_ub __attribute__((ext_vector_type(4), aligned(4)));
typedef float float2_ub __attribute__((ext_vector_type(2), aligned(4)));
extern "C" __device__ int bnn_bwn_writelane_i32(int val, int lane, int old) __asm("llvm.amdgcn.writelane.i32");

struct Split3 {
    uint4 h, m, l;      // 8 bf16 each: x = h + m + l exactly
};

// Exact three-way split of 8 floats into bf16 terms, packed two per register (element 2p in the low half).
__device__ __forceinline__ Split3 split3(const float (&x)[8]) {
    Split3 s;
    uint32_t hw[4], mw[4], lw[4];
#pragma unroll
    for (int p = 0; p < 4; ++p) {
        const float x0 = x[2 * p], x1 = x[2 * p + 1];
        const uint32_t u0 = __float_as_uint(x0), u1 = __float_as_uint(x1);
        hw[p] = __builtin_amdgcn_perm(u1, u0, 0x07060302u);                 // upper halves = truncation to bf16
        const float r0 = x0 - __uint_as_float(u0 & 0xffff0000u);            // exact: at most 16 significant bits left
        const float r1 = x1 - __uint_as_float(u1 & 0xffff0000u);
        const uint32_t v0 = __float_as_uint(r0), v1 = __float_as_uint(r1);
        mw[p] = __builtin_amdgcn_perm(v1, v0, 0x07060302u);
        const float l0 = r0 - __uint_as_float(v0 & 0xffff0000u);            // exact: at most 8 significant bits left
        const float l1 = r1 - __uint_as_float(v1 & 0xffff0000u);
        lw[p] = __builtin_amdgcn_perm(__float_as_uint(l1), __float_as_uint(l0), 0x07060302u);
    }
    s.h = make_uint4(hw[0], hw[1], hw[2], hw[3]);
    s.m = make_uint4(mw[0], mw[1], mw[2], mw[3]);
    s.l = make_uint4(lw[0], lw[1], lw[2], lw[3]);
    return s;
}

// Expands weight bits to bf16 +1.0 / -1.0 / 0: one thread per 16-byte unit (8 K-slots of one run of one
// channel).  wexp [col_tiles][2 * nsteps][cols] units.  A filter row is seg = k*Cp slots (channel c of tap t at
// slot t*Cp + c, channels >= C are padding); run j of a row starts at slot 8*j, or, with `moveback`, the last
// run is moved back to end at seg and the slots it shares with the run before get weight 0.
__global__ __launch_bounds__(256) void bwn_expand_kernel(const uint32_t* __restrict__ wbits, uint4* __restrict__ wexp, int C, int Cp,
                                                         int O, int k, int cols, int moveback, int nsteps, int nunits) {
    const int u = (int)(blockIdx.x * 256 + threadIdx.x);
    if (u >= nunits) return;
    const int seg = k * Cp, rpr = (seg + 7) >> 3, nruns = k * rpr;      // nsteps >= ceil(nruns / 2); the rest is zero
    const int last0 = seg >= 8 ? seg - 8 : 0, cw = (C + 31) >> 5;
    const int per_tile = 2 * nsteps * cols;
    const int tile = u / per_tile, v = u - tile * per_tile;
    const int rho = v / cols, col = v - rho * cols;
    const int o = tile * cols + col;
    uint32_t pk[4] = {0u, 0u, 0u, 0u};
    if (rho < nruns && o < O) {
        const int r = rho / rpr, j = rho - r * rpr;
        const int e0 = moveback ? min(8 * j, last0) : 8 * j;
        int t = e0 / Cp, c = e0 - t * Cp;
        const uint32_t* wrow = wbits + ((long long)o * k + r) * k * cw;
#pragma unroll
        for (int s = 0; s < 8; ++s) {
            const int e = e0 + s;
            uint32_t val = 0u;
            if (e < seg && e >= 8 * j && c < C) {
                const uint32_t b = (wrow[t * cw + (c >> 5)] >> (c & 31)) & 1u;
                val = b ? 0x3F80u : 0xBF80u;
            }
            pk[s >> 1] |= val << (16 * (s & 1));
            if (++c == Cp) { c = 0; ++t; }
        }
    }
    wexp[u] = make_uint4(pk[0], pk[1], pk[2], pk[3]);
}

// Same layout for real-valued weights w [O][k][k][C]: each weight is split exactly into three bf16 terms
// (as the input values are) and the three terms go to three planes, wexp [col_tiles][3][2 * nsteps][cols] units.
__global__ __launch_bounds__(256) void conv_f32_expand_kernel(const float* __restrict__ w, uint4* __restrict__ wexp, int C, int O,
                                                              int k, int cols, int nsteps, int nunits, int moveback) {
    const int u = (int)(blockIdx.x * 256 + threadIdx.x);
    if (u >= nunits) return;
    const int seg = k * C, rpr = (seg + 7) >> 3, nruns = k * rpr;
    const int last0 = seg >= 8 ? seg - 8 : 0;
    const int per_plane = 2 * nsteps * cols;
    const int tile = u / (3 * per_plane), v3 = u - tile * (3 * per_plane);
    const int plane = v3 / per_plane, v = v3 - plane * per_plane;
    const int rho = v / cols, col = v - rho * cols;
    const int o = tile * cols + col;
    uint32_t pk[4] = {0u, 0u, 0u, 0u};
    if (rho < nruns && o < O) {
        const int r = rho / rpr, j = rho - r * rpr;
        const int e0 = moveback ? min(8 * j, last0) : 8 * j;
        const float* wrow = w + ((long long)o * k + r) * seg;        // the k*C weights of filter row r are contiguous
        float xs[8];
#pragma unroll
        for (int s = 0; s < 8; ++s) xs[s] = wrow[min(e0 + s, seg - 1)];     // all eight loads in flight at once; masked below
#pragma unroll
        for (int s = 0; s < 8; ++s) {
            const int e = e0 + s;
            uint32_t val = 0u;
            if (e < seg && e >= 8 * j) {
                const float x0 = xs[s];
                const uint32_t a = __float_as_uint(x0);
                const float r1 = x0 - __uint_as_float(a & 0xffff0000u);
                const uint32_t b = __float_as_uint(r1);
                const float r2 = r1 - __uint_as_float(b & 0xffff0000u);
                val = (plane == 0 ? a : plane == 1 ? b : __float_as_uint(r2)) >> 16;
            }
            pk[s >> 1] |= val << (16 * (s & 1));
        }
    }
    wexp[u] = make_uint4(pk[0], pk[1], pk[2], pk[3]);
}

// ------------------------------------------------------------------------------------------ LDS-staged
struct BwnTile {            // geometry of the LDS-staged kernel, computed on the host
    int H, W, C, Cp, O, stride, pad, P, Q, k;
    int FQ, FP;             // a 32-pixel fragment is FP rows x FQ columns of output pixels (FP * FQ = 32)
    int TP;                 // output rows per workgroup (= WAVES * MT * FP); its columns are one fragment wide
    int tiles_p, tiles_q;
    int PR;                 // patch rows
    int PC, PCC;            // patch pixels per row; bf16 elements of a patch row that hold data (PC * Cp)
    int pitch;              // bytes between patch rows of a plane: multiple of 8, >= 2 * PCC + 16
    int rpr, nsteps;        // runs per filter row, MFMA K-steps
    int wbytes;             // bytes of expanded weights in LDS (patch planes follow)
    FastDiv div_tiles, div_tq, div_row, div_cp, div_fq, div_pc;
};

// CIN: input channels known at compile time (3: colour images), 0: any.  WANT_Y: also store the fp32 sums.
// At least two waves per SIMD are requested so that the register budget is 256: the accumulators then stay in
// ordinary VGPRs and the epilogue compares them in place (with 512 registers allowed the compiler parks them in
// AGPRs and copies every one back before the compare).
template <int MT, int NT, int WAVES, int CIN, bool WANT_Y>
__global__ __launch_bounds__(WAVES * 64, 8 / WAVES) void bwn_staged_kernel(const float* __restrict__ x, const uint4* __restrict__ wexp,
                                                                const float* __restrict__ thr, float* __restrict__ y,
                                                                uint32_t* __restrict__ bits, BwnTile g) {
    constexpr int COLS = NT * 32, NTHR = WAVES * 64;
    extern __shared__ uint4 smem[];
    uint4* wlds = smem;                                               // [2 * nsteps][COLS] units of 8 bf16
    char* patch = reinterpret_cast<char*>(smem) + g.wbytes;           // [3 planes][PR][pitch bytes]
    const int tid = (int)threadIdx.x;
    const int lane = tid & 63, l32 = lane & 31, half = lane >> 5, wave = tid >> 6;
    const int n0 = (int)blockIdx.y * COLS;
    const int plane = g.PR * g.pitch;

    // workgroup -> image, tile row, tile column
    const int blk = (int)blockIdx.x;
    const int n = fast_div(blk, g.div_tiles);
    const int trem = blk - n * (g.tiles_p * g.tiles_q);
    const int tp = fast_div(trem, g.div_tq), tq = trem - tp * g.tiles_q;
    const int p0 = tp * g.TP, q0 = tq * g.FQ;
    const int y0 = p0 * g.stride - g.pad, x0 = q0 * g.stride - g.pad;

    {   // expanded weights of this channel tile -> LDS
        const int nunits = 2 * g.nsteps * COLS;
        const uint4* src = wexp + (long long)blockIdx.y * nunits;
        for (int base = 0; base < nunits; base += 4 * NTHR) {
            uint4 tmp[4];
#pragma unroll
            for (int q = 0; q < 4; ++q) tmp[q] = src[min(base + q * NTHR + tid, nunits - 1)];
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const int u = base + q * NTHR + tid;
                if (u < nunits) wlds[u] = tmp[q];
            }
        }
    }
    {   // input patch -> three bf16 planes; out-of-image positions, padding channels and row slack become 0
        const float* ximg = x + (long long)n * g.H * g.W * g.C;
        auto put = [&](int off, float v) {                            // exact three-way split of one value
            const uint32_t a = __float_as_uint(v);
            const float r1 = v - __uint_as_float(a & 0xffff0000u);
            const uint32_t b = __float_as_uint(r1);
            const float r2 = r1 - __uint_as_float(b & 0xffff0000u);  // fits bf16
            *reinterpret_cast<unsigned short*>(patch + off) = (unsigned short)(a >> 16);
            *reinterpret_cast<unsigned short*>(patch + plane + off) = (unsigned short)(b >> 16);
            *reinterpret_cast<unsigned short*>(patch + 2 * plane + off) = (unsigned short)(__float_as_uint(r2) >> 16);
        };
        if (CIN == 3) {
            // one patch pixel per thread and pass, four passes in flight
            const int npx = g.PR * g.PC;
            for (int base = 0; base < npx; base += 4 * NTHR) {
                float v[4][3];
                int off[4];
#pragma unroll
                for (int u = 0; u < 4; ++u) {
                    const int e = base + u * NTHR + tid;
                    const int r = fast_div(e, g.div_pc), px = e - r * g.PC;
                    const int yy = y0 + r, xx = x0 + px;
                    const bool ok = e < npx && (unsigned)yy < (unsigned)g.H && (unsigned)xx < (unsigned)g.W;
                    v[u][0] = v[u][1] = v[u][2] = 0.f;
                    if (ok) {
                        const float* src = ximg + ((long long)yy * g.W + xx) * 3;
                        v[u][0] = src[0]; v[u][1] = src[1]; v[u][2] = src[2];
                    }
                    off[u] = e < npx ? r * g.pitch + px * g.Cp * 2 : -1;
                }
#pragma unroll
                for (int u = 0; u < 4; ++u) {
                    if (off[u] < 0) continue;
                    put(off[u], v[u][0]); put(off[u] + 2, v[u][1]); put(off[u] + 4, v[u][2]);
                    if (g.Cp == 4) put(off[u] + 6, 0.f);
                }
            }
            // slack behind the last pixel of every row
            const int slack = (g.pitch - 2 * g.PCC) >> 1;
            for (int e = tid; e < g.PR * slack; e += NTHR) {
                const int r = e / slack, i2 = e - r * slack;
                put(r * g.pitch + 2 * (g.PCC + i2), 0.f);
            }
        } else {
            const int epr = g.pitch >> 1;                             // bf16 slots per patch row
            const int total = g.PR * epr;
            for (int base = 0; base < total; base += 4 * NTHR) {
                float v[4];
                int off[4];
#pragma unroll
                for (int u = 0; u < 4; ++u) {
                    const int e = base + u * NTHR + tid;
                    const int r = fast_div(e, g.div_row);
                    const int rem = e - r * epr;
                    const int px = fast_div(rem, g.div_cp), c = rem - px * g.Cp;
                    const int yy = y0 + r, xx = x0 + px;
                    const bool ok = e < total && rem < g.PCC && c < g.C && (unsigned)yy < (unsigned)g.H && (unsigned)xx < (unsigned)g.W;
                    v[u] = 0.f;
                    if (ok) v[u] = ximg[((long long)yy * g.W + xx) * g.C + c];
                    off[u] = e < total ? r * g.pitch + rem * 2 : -1;
                }
#pragma unroll
                for (int u = 0; u < 4; ++u)
                    if (off[u] >= 0) put(off[u], v[u]);
            }
        }
    }
    __syncthreads();

    // fragment i of this wave: output rows p0 + (wave*MT + i)*FP + dp, column q0 + dq
    const int dp = fast_div(l32, g.div_fq), dq = l32 - dp * g.FQ;
    if (p0 + wave * MT * g.FP >= g.P) return;                         // nothing of this wave is inside the image
    int abase[MT];
#pragma unroll
    for (int i = 0; i < MT; ++i) abase[i] = (((wave * MT + i) * g.FP + dp) * g.stride) * g.pitch + dq * g.stride * g.Cp * 2;

    v16f_bwn acc[MT][NT];

    // this lane's run index is 2*step + half; (rr, jj) = (filter row, run within the row).  A run index past
    // the last one (odd run count, upper half-wave) re-reads the last run against zero weights.
    int rr = half / g.rpr, jj = half - rr * g.rpr;
    auto advance = [&]() {
        jj += 2;
        while (jj >= g.rpr) { jj -= g.rpr; ++rr; }
        if (rr >= g.k) { rr = g.k - 1; jj = g.rpr - 1; }
    };
    if (rr >= g.k) { rr = g.k - 1; jj = g.rpr - 1; }
    auto load_a = [&](uint4 (&a)[MT][3]) {
        const int off = rr * g.pitch + jj * 16;
#pragma unroll
        for (int i = 0; i < MT; ++i)
#pragma unroll
            for (int pl = 0; pl < 3; ++pl) {
                const char* src = patch + pl * plane + abase[i] + off;
                const uint2 lo = *reinterpret_cast<const uint2*>(src);
                const uint2 hi = *reinterpret_cast<const uint2*>(src + 8);
                a[i][pl] = make_uint4(lo.x, lo.y, hi.x, hi.y);
            }
    };
    auto load_b = [&](int step, uint4 (&b)[NT]) {
#pragma unroll
        for (int j = 0; j < NT; ++j) b[j] = wlds[(2 * step + half) * COLS + 32 * j + l32];
    };
    auto multiply = [&](const uint4 (&a)[MT][3], const uint4 (&b)[NT], auto first) {
        const v16f_bwn zero = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int pl = 2; pl >= 0; --pl)                               // smallest terms first
#pragma unroll
            for (int i = 0; i < MT; ++i)
#pragma unroll
                for (int j = 0; j < NT; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(v8bf_bwn, a[i][pl]),
                                                                         __builtin_bit_cast(v8bf_bwn, b[j]),
                                                                         (decltype(first)::value && pl == 2) ? zero : acc[i][j], 0, 0, 0);
    };

    // the first K-step starts the accumulators from a constant 0 (no register clearing)
    uint4 a0[MT][3], a1[MT][3], b0[NT], b1[NT];
    load_a(a0); load_b(0, b0);
    if (g.nsteps > 1) { advance(); load_a(a1); load_b(1, b1); }
    multiply(a0, b0, std::true_type{});
    for (int step = 1; step < g.nsteps; step += 2) {
        if (step + 1 < g.nsteps) { advance(); load_a(a0); load_b(step + 1, b0); }
        multiply(a1, b1, std::false_type{});
        if (step + 1 < g.nsteps) {
            if (step + 2 < g.nsteps) { advance(); load_a(a1); load_b(step + 2, b1); }
            multiply(a0, b0, std::false_type{});
        }
    }

    float th[NT];
    bool cok[NT];
#pragma unroll
    for (int j = 0; j < NT; ++j) {
        const int col = n0 + 32 * j + l32;
        cok[j] = col < g.O;
        th[j] = ((!WANT_Y || bits != nullptr) && cok[j]) ? thr[col] : __builtin_inff();
    }
    const int ow = (g.O + 31) / 32;
    const long long img_pix = (long long)n * g.P * g.Q;
#pragma unroll
    for (int i = 0; i < MT; ++i) {
        const int frow0 = p0 + (wave * MT + i) * g.FP;                // first output row of the fragment
        if (frow0 >= g.P) break;
        uint32_t wout[NT];
#pragma unroll
        for (int j = 0; j < NT; ++j) wout[j] = 0u;
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            const int lo_row = 8 * (r >> 2) + (r & 3);
#pragma unroll
            for (int j = 0; j < NT; ++j) {
                const float v = acc[i][j][r];
                if (WANT_Y) {
                    const int m = lo_row + 4 * half;                  // fragment row of this register in this lane
                    const int mp = fast_div(m, g.div_fq), mq = m - mp * g.FQ;
                    if (frow0 + mp < g.P && q0 + mq < g.Q && cok[j])
                        y[(img_pix + (long long)(frow0 + mp) * g.Q + q0 + mq) * g.O + n0 + 32 * j + l32] = v;
                }
                if (!WANT_Y || bits != nullptr) {       // without the fp32 output the bits are always wanted
                    const unsigned long long ball = __builtin_amdgcn_ballot_w64(v >= th[j]);
                    wout[j] = (uint32_t)bnn_bwn_writelane_i32((int)(uint32_t)ball, lo_row, (int)wout[j]);
                    wout[j] = (uint32_t)bnn_bwn_writelane_i32((int)(uint32_t)(ball >> 32), lo_row + 4, (int)wout[j]);
                }
            }
        }
        // lane m < 32 holds the packed words of fragment row m = output pixel (frow0 + dp, q0 + dq)
        if ((!WANT_Y || bits != nullptr) && lane < 32 && frow0 + dp < g.P && q0 + dq < g.Q) {
            const long long pix = img_pix + (long long)(frow0 + dp) * g.Q + q0 + dq;
#pragma unroll
            for (int j = 0; j < NT; ++j) {
                const int wi = (n0 >> 5) + j;
                if (wi < ow) bits[pix * ow + wi] = wout[j];
            }
        }
    }
}

// ------------------------------------------------------------------------------------------ direct
// MT x NT accumulator tiles of 32x32 per wave, WAVES waves per workgroup (they share the weights in LDS); the
// workgroup covers NT*32 output channels and is persistent: its waves stride over the groups of MT*32 output pixels.
// NPL: weight planes -- 1: +1/-1 weights (one bf16 value each); 3: real-valued weights split into three bf16 terms.
// TERMS (NPL == 3): 9 -- every input-term x weight-term product is formed, so each product x * w is exact here too;
// 6 -- without the three smallest (middle x low, low x middle, low x low), which together lie below 2^-23 of the
// product: as accurate as rounding each product to fp32, two thirds of the matrix work.
template <int MT, int NT, int WAVES, int NPL, int TERMS = 3 * NPL>
__global__ __launch_bounds__(WAVES * 64) void bwn_conv_kernel(const float* __restrict__ x, const uint4* __restrict__ wexp,
                                                       const float* __restrict__ thr, float* __restrict__ y,
                                                       uint32_t* __restrict__ bits, int N, int H, int W, int C, int O,
                                                       int k, int stride, int pad, int P, int Q, FastDiv div_pq, FastDiv div_q) {
    constexpr int COLS = NT * 32, NTHR = WAVES * 64;
    const int lane = threadIdx.x & 63, l32 = lane & 31, half = lane >> 5, wave = threadIdx.x >> 6;
    const int npix = N * P * Q;
    const int n0 = (int)blockIdx.y * COLS;
    const int seg = k * C;                                   // floats in one filter row
    const int rpr = (seg + 7) >> 3;                          // runs per filter row
    const int nruns = k * rpr;
    // one MFMA K-step takes two runs (one per half-wave); the step count is rounded up to a multiple of 3 (the
    // depth of the prefetch rotation), the added steps multiply by zero weights
    const int nreal = (nruns + 1) / 2;                       // steps that hold data
    const int nsteps = (nreal + 2) / 3 * 3;
    const int last0 = seg >= 8 ? seg - 8 : 0;                // first float of the last run of a filter row
    const int rowlen = W * C;
    const long long total = (long long)N * H * rowlen;       // floats in x

    // ---- expanded weights of this workgroup's channel tile -> LDS
    extern __shared__ uint4 wlds[];                          // [NPL][2 * nsteps][COLS] units of 8 bf16
    {
        const int nunits = NPL * 2 * nsteps * COLS;
        const uint4* src = wexp + (long long)blockIdx.y * nunits;
        for (int base = 0; base < nunits; base += 4 * NTHR) {
            uint4 tmp[4];
#pragma unroll
            for (int q = 0; q < 4; ++q) tmp[q] = src[min(base + q * NTHR + (int)threadIdx.x, nunits - 1)];
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const int u = base + q * NTHR + (int)threadIdx.x;
                if (u < nunits) wlds[u] = tmp[q];
            }
        }
    }
    __syncthreads();

    float th[NT];
    bool cok[NT];
#pragma unroll
    for (int j = 0; j < NT; ++j) {
        const int col = n0 + 32 * j + l32;
        cok[j] = col < O;
        th[j] = (bits != nullptr && cok[j]) ? thr[col] : __builtin_inff();
    }
    const int ow = (O + 31) / 32;

    // the workgroups stay for the whole kernel (one per CU: the weights are copied once); the waves stride over
    // the groups of MT*32 output pixels
    for (long long grp = (long long)blockIdx.x * WAVES + wave; grp * (MT * 32) < npix; grp += (long long)gridDim.x * WAVES) {
        const int m0 = (int)(grp * (MT * 32));

        long long xbase[MT];        // float index of input row 0 of this lane's image
        int xoff[MT], ytop[MT];
#pragma unroll
        for (int i = 0; i < MT; ++i) {
            const int pix = min(m0 + 32 * i + l32, npix - 1);
            const int n = fast_div(pix, div_pq);
            const int rem = pix - n * (P * Q);
            const int p = fast_div(rem, div_q), q = rem - p * Q;
            ytop[i] = p * stride - pad;
            xoff[i] = (q * stride - pad) * C;
            xbase[i] = (long long)n * H * rowlen;
        }

        v16f_bwn acc[MT][NT];
#pragma unroll
        for (int i = 0; i < MT; ++i)
#pragma unroll
            for (int j = 0; j < NT; ++j)
#pragma unroll
                for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

        struct Run {                // one prefetched K-step: the values, their in-image range, where they start
            float v[MT][8];
            int rng[MT];
            long long start[MT];
        };

        // Loads this lane's run (filter row r, floats [e0, e0+8) of the row's segment) for every A fragment and
        // records which of the 8 positions lie inside the image as the range [lo, hi) (packed lo | hi << 8).
        // The zero padding itself is applied when the run is consumed, so that nothing waits on the loads here,
        // and there is no branch: a run that would leave the tensor (only at its very first and last pixels) is
        // loaded from offset 0 instead, flagged (bit 16), and re-read element by element when it is consumed.
        auto fetch = [&](int r, int e0, Run& q) {
            const int cnt = min(8, seg - e0);                // floats of the run inside the segment
#pragma unroll
            for (int i = 0; i < MT; ++i) {
                const int yy = ytop[i] + r;
                const bool yok = (unsigned)yy < (unsigned)H;
                const long long start = xbase[i] + (long long)(yok ? yy : 0) * rowlen + xoff[i] + e0;
                const bool inb = start >= 0 && start + 8 <= total;
                const float* src = x + (inb ? start : 0);
                const float4_ub v0 = *reinterpret_cast<const float4_ub*>(src);
                const float4_ub v1 = *reinterpret_cast<const float4_ub*>(src + 4);
#pragma unroll
                for (int t = 0; t < 4; ++t) { q.v[i][t] = v0[t]; q.v[i][4 + t] = v1[t]; }
                const int xs = xoff[i] + e0;
                const int lo = max(0, -xs), hi = yok ? max(min(cnt, rowlen - xs), 0) : 0;
                q.rng[i] = lo | (hi << 8) | (inb ? 0 : 1 << 16);
                q.start[i] = start;
            }
        };

        auto multiply = [&](int step, Run& q) {
            uint4 b[NPL][NT];
#pragma unroll
            for (int pw = 0; pw < NPL; ++pw)
#pragma unroll
                for (int j = 0; j < NT; ++j) b[pw][j] = wlds[(pw * 2 * nsteps + 2 * step + half) * COLS + 32 * j + l32];
#pragma unroll
            for (int i = 0; i < MT; ++i) {
                // zero padding; skipped when every lane of the wave has its whole run inside the image
                if (__builtin_amdgcn_ballot_w64(q.rng[i] == (8 << 8)) != ~0ull) {
                    if (__builtin_amdgcn_ballot_w64((q.rng[i] >> 16) != 0) != 0ull) {
#pragma unroll
                        for (int t = 0; t < 8; ++t) {
                            const long long idx = q.start[i] + t;
                            if ((q.rng[i] >> 16) != 0) q.v[i][t] = (idx >= 0 && idx < total) ? x[idx < 0 ? 0 : (idx < total ? idx : 0)] : 0.f;
                        }
                    }
                    const int lo = q.rng[i] & 255, hi = (q.rng[i] >> 8) & 255;
#pragma unroll
                    for (int t = 0; t < 8; ++t) q.v[i][t] = (t >= lo && t < hi) ? q.v[i][t] : 0.f;
                }
                const Split3 s = split3(q.v[i]);
                const uint4 xs[3] = {s.h, s.m, s.l};
                // smallest terms first: (input term, weight term) pairs in order of decreasing index sum
#pragma unroll
                for (int sum = (TERMS == 3 * NPL ? 2 + (NPL - 1) : 2); sum >= 0; --sum)
#pragma unroll
                    for (int px = 2; px >= 0; --px) {
                        const int pw = sum - px;
                        if (pw < 0 || pw >= NPL) continue;
#pragma unroll
                        for (int j = 0; j < NT; ++j)
                            acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(v8bf_bwn, xs[px]),
                                                                                 __builtin_bit_cast(v8bf_bwn, b[pw][j]), acc[i][j], 0, 0, 0);
                    }
            }
        };

        // this lane's run index advances by 2 per step; (rr, jj) = (filter row, run within the row).  A run
        // index past the last one (odd run count, upper half-wave) repeats the last run against zero weights.
        int rr = half / rpr, jj = half - rr * rpr;
        auto advance = [&]() {
            jj += 2;
            while (jj >= rpr) { jj -= rpr; ++rr; }
        };
        auto run_e0 = [&]() { return min(8 * jj, last0); };
        auto clamp_last = [&]() {
            if (rr >= k) { rr = k - 1; jj = rpr - 1; }
        };

        // three run buffers: the loads of step s + 2 are issued before the MFMAs of step s.  Fetches are
        // unconditional (past the end they repeat the last run) so that the number of loads in flight at every
        // wait is the same on every path.
        Run run0, run1, run2;
        auto next = [&](Run& q) {
            advance(); clamp_last(); fetch(rr, run_e0(), q);
        };
        clamp_last();
        fetch(rr, run_e0(), run0);
        next(run1);
        for (int step = 0; step < nsteps; step += 3) {
            next(run2);
            multiply(step, run0);
            next(run0);
            if (step + 1 < nreal) multiply(step + 1, run1);     // the padding steps of the last round only fetch
            next(run1);
            if (step + 2 < nreal) multiply(step + 2, run2);
        }

#pragma unroll
        for (int i = 0; i < MT; ++i) {
            const int rbase = m0 + 32 * i;
            if (rbase >= npix) break;
            uint32_t wout[NT];
#pragma unroll
            for (int j = 0; j < NT; ++j) wout[j] = 0u;
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int lo_row = 8 * (r >> 2) + (r & 3);
                const int row = rbase + lo_row + 4 * half;
#pragma unroll
                for (int j = 0; j < NT; ++j) {
                    const float v = acc[i][j][r];
                    if (y != nullptr && row < npix && cok[j]) y[(long long)row * O + n0 + 32 * j + l32] = v;
                    if (bits != nullptr) {
                        const unsigned long long ball = __builtin_amdgcn_ballot_w64(v >= th[j]);
                        wout[j] = (uint32_t)bnn_bwn_writelane_i32((int)(uint32_t)ball, lo_row, (int)wout[j]);
                        wout[j] = (uint32_t)bnn_bwn_writelane_i32((int)(uint32_t)(ball >> 32), lo_row + 4, (int)wout[j]);
                    }
                }
            }
            const int row = rbase + lane;
            if (bits != nullptr && lane < 32 && row < npix) {
#pragma unroll
                for (int j = 0; j < NT; ++j) {
                    const int wi = (n0 >> 5) + j;
                    if (wi < ow) bits[(long long)row * ow + wi] = wout[j];
                }
            }
        }
    }
}

template <int MT, int NT, int WAVES, int NPL, int TERMS = 3 * NPL>
int launch_bwn_direct(const float* x, const void* weights, const float* thr, float* y, uint32_t* bits, int N, int H, int W,
                      int C, int O, int k, int stride, int pad, int P, int Q, void* workspace, size_t workspace_bytes,
                      hipStream_t s) {
    constexpr int COLS = NT * 32;
    const long long npix = (long long)N * P * Q;
    const int seg = k * C, nruns = k * ((seg + 7) / 8), nsteps = ((nruns + 1) / 2 + 2) / 3 * 3;
    const int col_tiles = (int)cdiv(O, COLS);
    const size_t lds_bytes = (size_t)NPL * 2 * nsteps * COLS * 16;
    if (lds_bytes > 160 * 1024) return BNN_ERR_UNSUPPORTED;
    if (workspace_bytes < lds_bytes * col_tiles) return BNN_ERR_WORKSPACE;
    if (lds_bytes > 64 * 1024) {
        static const hipError_t attr = hipFuncSetAttribute(reinterpret_cast<const void*>(&bwn_conv_kernel<MT, NT, WAVES, NPL, TERMS>),
                                                           hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
        if (attr != hipSuccess) return BNN_ERR_DEVICE;
    }
    uint4* wexp = static_cast<uint4*>(workspace);
    const int nunits = col_tiles * NPL * 2 * nsteps * COLS;
    if (NPL == 1)
        hipLaunchKernelGGL(bwn_expand_kernel, dim3((unsigned)cdiv(nunits, 256)), dim3(256), 0, s, static_cast<const uint32_t*>(weights),
                           wexp, C, C, O, k, COLS, 1, nsteps, nunits);
    else
        hipLaunchKernelGGL(conv_f32_expand_kernel, dim3((unsigned)cdiv(nunits, 256)), dim3(256), 0, s,
                           static_cast<const float*>(weights), wexp, C, O, k, COLS, nsteps, nunits, 1);
    // one workgroup per CU (registers allow no more), resident for the whole call
    const long long groups = cdiv(npix, MT * 32);
    static int cus = 0;
    if (cus == 0) {
        int dev = 0;
        if (hipGetDevice(&dev) != hipSuccess || hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess ||
            cus < 1)
            return BNN_ERR_DEVICE;
    }
    const long long wgs = min(cdiv(groups, WAVES), (long long)max(1, cus / col_tiles));
    dim3 grid((unsigned)wgs, (unsigned)col_tiles);
    hipLaunchKernelGGL((bwn_conv_kernel<MT, NT, WAVES, NPL, TERMS>), grid, dim3(WAVES * 64), lds_bytes, s, x, wexp, thr, y, bits, N, H, W, C, O, k, stride,
                       pad, P, Q, make_fastdiv(P * Q), make_fastdiv(Q));
    return check_launch();
}

// Channels per pixel in the LDS patch: the smallest Cp >= C for which a pixel step (stride * Cp bf16) is a
// multiple of 8 bytes, so that every operand read is 8-byte aligned.
int staged_cp(int C, int stride) {
    const int m = stride % 4 == 0 ? 1 : (stride % 2 == 0 ? 2 : 4);
    return (C + m - 1) / m * m;
}

constexpr size_t LDS_MAX = 160 * 1024;

// Fills the geometry for an MT x NT x WAVES configuration; false if weights + patch do not fit LDS.
bool staged_geom(int MT, int NT, int WAVES, int N, int H, int W, int C, int O, int k, int stride, int pad, int P, int Q,
                 BwnTile* g, size_t* lds_bytes) {
    g->H = H; g->W = W; g->C = C; g->Cp = staged_cp(C, stride); g->O = O; g->stride = stride; g->pad = pad; g->P = P; g->Q = Q; g->k = k;
    g->FQ = Q >= 24 ? 32 : (Q >= 12 ? 16 : 8);
    g->FP = 32 / g->FQ;
    g->TP = WAVES * MT * g->FP;
    g->tiles_p = (int)cdiv(P, g->TP); g->tiles_q = (int)cdiv(Q, g->FQ);
    g->PR = (g->TP - 1) * stride + k;
    const long long pcc = ((long long)(g->FQ - 1) * stride + k) * g->Cp;
    const long long pitch = (2 * pcc + 16 + 7) / 8 * 8;
    const long long seg = (long long)k * g->Cp;
    g->rpr = (int)((seg + 7) / 8);
    const long long nruns = (long long)k * g->rpr;
    g->nsteps = (int)((nruns + 1) / 2);
    const long long wbytes = 2LL * g->nsteps * NT * 32 * 16;
    const long long total = wbytes + 3LL * g->PR * pitch;
    if (total > (long long)LDS_MAX || (long long)N * g->tiles_p * g->tiles_q >= (1LL << 31)) return false;
    g->PC = (g->FQ - 1) * stride + k; g->PCC = (int)pcc; g->pitch = (int)pitch; g->wbytes = (int)wbytes;
    g->div_pc = make_fastdiv((uint32_t)g->PC);
    g->div_tiles = make_fastdiv((uint32_t)(g->tiles_p * g->tiles_q)); g->div_tq = make_fastdiv((uint32_t)g->tiles_q);
    g->div_row = make_fastdiv((uint32_t)(pitch / 2)); g->div_cp = make_fastdiv((uint32_t)g->Cp); g->div_fq = make_fastdiv((uint32_t)g->FQ);
    *lds_bytes = (size_t)total;
    return true;
}

template <int MT, int NT, int WAVES, int CIN, bool WANT_Y>
int launch_bwn_staged_v(const float* x, const uint32_t* wbits, const float* thr, float* y, uint32_t* bits, int N, int C, int O,
                      int k, const BwnTile& g, size_t lds_bytes, void* workspace, size_t workspace_bytes, hipStream_t s) {
    constexpr int COLS = NT * 32;
    const int col_tiles = (int)cdiv(O, COLS);
    if (workspace_bytes < (size_t)g.wbytes * col_tiles) return BNN_ERR_WORKSPACE;
    if (lds_bytes > 64 * 1024) {
        static const hipError_t attr = hipFuncSetAttribute(reinterpret_cast<const void*>(&bwn_staged_kernel<MT, NT, WAVES, CIN, WANT_Y>),
                                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)LDS_MAX);
        if (attr != hipSuccess) return BNN_ERR_DEVICE;
    }
    uint4* wexp = static_cast<uint4*>(workspace);
    const int nunits = col_tiles * 2 * g.nsteps * COLS;
    hipLaunchKernelGGL(bwn_expand_kernel, dim3((unsigned)cdiv(nunits, 256)), dim3(256), 0, s, wbits, wexp, C, g.Cp, O, k, COLS, 0,
                       g.nsteps, nunits);
    dim3 grid((unsigned)(N * g.tiles_p * g.tiles_q), (unsigned)col_tiles);
    hipLaunchKernelGGL((bwn_staged_kernel<MT, NT, WAVES, CIN, WANT_Y>), grid, dim3(WAVES * 64), lds_bytes, s, x, wexp, thr, y, bits, g);
    return check_launch();
}

template <int MT, int NT, int WAVES>
int launch_bwn_staged(const float* x, const uint32_t* wbits, const float* thr, float* y, uint32_t* bits, int N, int C, int O,
                      int k, const BwnTile& g, size_t lds_bytes, void* workspace, size_t workspace_bytes, hipStream_t s) {
    // the fp32 sums are a test / debugging output: only the generic-channel variant carries them
    if (y != nullptr)
        return launch_bwn_staged_v<MT, NT, WAVES, 0, true>(x, wbits, thr, y, bits, N, C, O, k, g, lds_bytes, workspace, workspace_bytes, s);
    if (C == 3)
        return launch_bwn_staged_v<MT, NT, WAVES, 3, false>(x, wbits, thr, y, bits, N, C, O, k, g, lds_bytes, workspace, workspace_bytes, s);
    return launch_bwn_staged_v<MT, NT, WAVES, 0, false>(x, wbits, thr, y, bits, N, C, O, k, g, lds_bytes, workspace, workspace_bytes, s);
}

}  // namespace

// Upper bound over every kernel configuration: 128-channel tiles, channels padded by at most 3.
size_t bwn_workspace_bytes(int C, int O, int k) {
    const long long seg = (long long)k * (C + 3), nruns = k * ((seg + 7) / 8), nsteps = ((nruns + 1) / 2 + 2) / 3 * 3;
    return (size_t)(cdiv(O, 128) * 128 * 2 * nsteps * 16);
}

bool try_bwn_wave(const float* x, const uint32_t* wbits, const float* thr, float* y, uint32_t* bits, int N, int H, int W, int C, int O,
                  int k, int stride, int pad, int P, int Q, void* workspace, size_t workspace_bytes, hipStream_t s, int* rc);

int launch_bwn_conv_thr(const float* x, const uint32_t* wbits, const float* thr, float* y, uint32_t* bits, int N, int H, int W,
                        int C, int O, int k, int stride, int pad, void* workspace, size_t workspace_bytes, hipStream_t s) {
    const int P = (H + 2 * pad - k) / stride + 1, Q = (W + 2 * pad - k) / stride + 1;
    int wave_rc = BNN_OK;
    if (try_bwn_wave(x, wbits, thr, y, bits, N, H, W, C, O, k, stride, pad, P, Q, workspace, workspace_bytes, s, &wave_rc))
        return wave_rc;                        // wave-private patches in LDS for the filter geometries that kernel is built for
    BwnTile g;
    size_t lds = 0;
    // LDS-staged kernel with small workgroups while several of them fit a CU side by side (one loads its
    // patch while another multiplies); otherwise the direct kernel, eight waves sharing one copy of the weights.
    constexpr size_t SIDE_BY_SIDE = 64 * 1024;
    if (O > 64 && staged_geom(1, 4, 4, N, H, W, C, O, k, stride, pad, P, Q, &g, &lds) && lds <= SIDE_BY_SIDE)
        return launch_bwn_staged<1, 4, 4>(x, wbits, thr, y, bits, N, C, O, k, g, lds, workspace, workspace_bytes, s);
    if (staged_geom(2, 2, 4, N, H, W, C, O, k, stride, pad, P, Q, &g, &lds) && lds <= SIDE_BY_SIDE)
        return launch_bwn_staged<2, 2, 4>(x, wbits, thr, y, bits, N, C, O, k, g, lds, workspace, workspace_bytes, s);
    if (staged_geom(1, 2, 4, N, H, W, C, O, k, stride, pad, P, Q, &g, &lds) && lds <= SIDE_BY_SIDE)
        return launch_bwn_staged<1, 2, 4>(x, wbits, thr, y, bits, N, C, O, k, g, lds, workspace, workspace_bytes, s);
    if (O <= 64) return launch_bwn_direct<2, 2, 8, 1>(x, wbits, thr, y, bits, N, H, W, C, O, k, stride, pad, P, Q, workspace, workspace_bytes, s);
    return launch_bwn_direct<1, 4, 8, 1>(x, wbits, thr, y, bits, N, H, W, C, O, k, stride, pad, P, Q, workspace, workspace_bytes, s);
}

// ------------------------------------------------------------------------------------------ wave-private patches
// Real-valued first layer (three weight planes) for one filter geometry fixed at compile time (the 7x7 stride-4 stem
// of 3-channel images): every wave on its own.  A wave owns a rectangle of FP x FQ = 32 output pixels, keeps the input
// patch under it in a private slice of LDS as three bf16 planes, and walks the K loop from LDS only: with the geometry
// known, every LDS address of the loop is a lane base plus an immediate, so a K-step is twelve MFMAs, twelve LDS reads
// and one vector instruction (the direct kernel above issues ten vector instructions per MFMA for loading, masking
// and splitting its runs).  The patch of the wave's NEXT rectangle is requested from global memory before the K loop
// (coalesced 8-byte loads into registers, one scalar address per patch row) and is split and written to LDS after the
// epilogue, so the only memory wait a wave sees is one it has had a whole rectangle of MFMA work to cover; the eight
// waves of a workgroup share nothing but the weights (copied to LDS once: the workgroups are persistent) and drift
// apart, so that on every SIMD one wave stages while the other multiplies.  No barrier after the weights are in.
// WAVES_: waves per workgroup (what fits LDS beside the weights); WPL_: weight planes -- 3 for real-valued weights (split
// like the inputs), 1 for binarized weights (+1.0 / -1.0 are exact in bf16).
template <int KS_, int STRIDE_, int CIN_, int FP_, int FQ_, int WAVES_ = 8, int WPL_ = 3>
struct WaveGeom {
    static constexpr int KS = KS_, STRIDE = STRIDE_, CIN = CIN_, FP = FP_, FQ = FQ_, WPL = WPL_;
    static constexpr int PR = (FP - 1) * STRIDE + KS;                        // patch rows
    static constexpr int ROW_ELEMS = ((FQ - 1) * STRIDE + KS) * CIN;         // input values of a patch row
    static constexpr int SEG = KS * CIN;                                     // values of one filter row
    static constexpr int RPR = (SEG + 7) / 8;                                // runs of 8 per filter row
    static constexpr int NRUNS = KS * RPR;
    static constexpr int NSTEPS = (NRUNS + 1) / 2;                           // MFMA K-steps (two runs each)
    static constexpr int REACH = (FQ - 1) * STRIDE * CIN + 8 * RPR;          // farthest element a run reads from a patch row, + 1
    static constexpr int PITCH = (2 * (REACH > ROW_ELEMS ? REACH : ROW_ELEMS) + 7) / 8 * 8;    // bytes between patch rows
    static constexpr int PAIRS = PITCH / 4;                                  // 2-element units written per patch row (data + zeroed slack)
    static constexpr int PLANE = PR * PITCH;                                 // bytes of one bf16 plane of a patch
    static constexpr int WUNITS = NRUNS * 64;                                // 16-byte units of one weight plane in LDS
    static constexpr int WAVES = WAVES_;
    static constexpr size_t LDS = (size_t)WPL * WUNITS * 16 + (size_t)WAVES * 3 * PLANE;
    static_assert(FP * FQ == 32 && PAIRS <= 64 && (STRIDE * CIN * 2) % 8 == 0, "one lane per pair; 8-byte aligned runs");
};

template <int N, class F, int I = 0>
__device__ __forceinline__ void static_for(F&& f) {
    if constexpr (I < N) {
        f(std::integral_constant<int, I>{});
        static_for<N, F, I + 1>(static_cast<F&&>(f));
    }
}

struct WaveArgs {
    int N, H, W, O, pad, P, Q;
    int tiles_p, tiles_q;
    int ntiles;              // N * tiles_p * tiles_q
    FastDiv div_tiles, div_tq;
};

template <class G, int TERMS, bool WANT_Y>
__global__ __launch_bounds__(G::WAVES * 64, 1) void conv_f32_wave_kernel(const float* __restrict__ x, const void* __restrict__ wv,
                                                                        const float* __restrict__ thr, float* __restrict__ y,
                                                                        uint32_t* __restrict__ bits, WaveArgs g) {
    constexpr int NT = 2, COLS = 64;
    constexpr bool BWN = G::WPL == 1;                                  // wv: weight bits [O][k][k][1 word] instead of floats [O][k][k][C]
    static_assert(G::WPL == 3 || (G::WPL == 1 && G::CIN <= 32 && TERMS == 3), "three planes of real weights or one of +-1");
    extern __shared__ uint4 smem[];
    uint4* wlds = smem;                                                // [weight planes][NRUNS][64 columns] units of 8 bf16
    const int tid = (int)threadIdx.x;
    const int lane = tid & 63, l32 = lane & 31, half = lane >> 5;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);        // scalar: everything derived from the rectangle index stays scalar
    char* patch = reinterpret_cast<char*>(smem) + G::WPL * G::WUNITS * 16 + wave * (3 * G::PLANE);     // this wave's three planes
    const int n0 = (int)blockIdx.y * COLS;

    float th[NT];
    bool cok[NT];
#pragma unroll
    for (int j = 0; j < NT; ++j) {
        const int col = n0 + 32 * j + l32;
        cok[j] = col < g.O;
        th[j] = ((!WANT_Y || bits != nullptr) && cok[j]) ? thr[col] : __builtin_inff();
    }
    const int ow = (g.O + 31) / 32;

    // this lane's output pixel inside a rectangle; where its runs start in a patch plane; its column in a weight plane,
    // the upper half-wave one run further (its run index is 2 * step + 1)
    // (rows vary fastest over the lanes: with 4 rows of 864 bytes and pixels 24 bytes apart, the sixteen 8-byte reads
    // LDS serves together then fall on sixteen different bank pairs)
    const int dp = l32 % G::FP, dq = l32 / G::FP;
    const char* abase = patch + dp * (G::STRIDE * G::PITCH) + dq * (G::STRIDE * G::CIN * 2);
    const char* bbase = reinterpret_cast<const char*>(wlds + l32) + half * (COLS * 16);
    const int rowlen = g.W * G::CIN;                                 // values per image row (H * W * C < 2^31: checked on the host)

    // ---- patch prefetch: lane l holds elements 2l, 2l + 1 of every patch row.  A pair may hang over the left or right
    // edge of the image row by one element (the padding is not a multiple of 2 elements): it is then loaded one element
    // further in, and stage() picks the element that is image data.
    float2_ub pre[G::PR];
    auto tile_origin = [&](int t, int& n, int& p0, int& q0) {
        n = fast_div(t, g.div_tiles);
        const int rem = t - n * (g.tiles_p * g.tiles_q);
        const int tp = fast_div(rem, g.div_tq);
        p0 = tp * G::FP;
        q0 = (rem - tp * g.tiles_q) * G::FQ;
    };
    auto request = [&](int t) {                // issues the loads of rectangle t's patch; nothing waits here
        int n, p0, q0;
        tile_origin(t, n, p0, q0);
        const int y0 = p0 * G::STRIDE - g.pad;
        const int e0 = (q0 * G::STRIDE - g.pad) * G::CIN + 2 * lane;                // first element of this lane's pair in the image row
        const uint32_t lane_bytes = (uint32_t)min(max(e0, 0), rowlen - 2) * 4u;          // rowlen >= 2 (checked on the host)
        const float* img = x + (long long)n * g.H * rowlen;                             // uniform
#pragma unroll
        for (int r = 0; r < G::PR; ++r) {
            const int yy = min(max(y0 + r, 0), g.H - 1);                                // uniform: rows outside the image are zeroed in stage()
            const char* rowp = reinterpret_cast<const char*>(img + yy * rowlen);        // uniform: scalar base + lane offset
            pre[r] = *reinterpret_cast<const float2_ub*>(rowp + lane_bytes);            // 8 bytes, 4-byte aligned
        }
    };
    auto stage = [&](int t) {                  // splits the prefetched patch of rectangle t into the wave's three planes
        int n, p0, q0;
        tile_origin(t, n, p0, q0);
        const int y0 = p0 * G::STRIDE - g.pad;
        const int e0 = (q0 * G::STRIDE - g.pad) * G::CIN + 2 * lane;
        const bool shifted = min(max(e0, 0), rowlen - 2) != e0;
        // element validity as bit masks: inside the image row and inside the patch row's data (beyond it the row's slack
        // is zeroed); rows above / below the image are zeroed through a wave-uniform mask -- no branch in the loop
        const uint32_t m0 = (e0 >= 0 && e0 < rowlen && 2 * lane < G::ROW_ELEMS) ? 0xFFFFFFFFu : 0u;
        const uint32_t m1 = (e0 + 1 >= 0 && e0 + 1 < rowlen && 2 * lane + 1 < G::ROW_ELEMS) ? 0xFFFFFFFFu : 0u;
        static_assert(2 * (G::PAIRS - 1) >= G::ROW_ELEMS, "the last pair is slack: the lanes past it repeat its stores of zeros");
        char* dst = patch + 4 * min(lane, G::PAIRS - 1);
#pragma unroll
        for (int r = 0; r < G::PR; ++r) {
            const uint32_t ym = (unsigned)(y0 + r) < (unsigned)g.H ? 0xFFFFFFFFu : 0u;     // uniform
            // shifted by one element: the left-edge pair holds its second element first, the right-edge pair its first element second
            const uint32_t ua = __float_as_uint(shifted ? pre[r][1] : pre[r][0]) & m0 & ym;
            const uint32_t ub = __float_as_uint(shifted ? pre[r][0] : pre[r][1]) & m1 & ym;
            const float a = __uint_as_float(ua), b = __uint_as_float(ub);
            const float ra = a - __uint_as_float(ua & 0xffff0000u), rb = b - __uint_as_float(ub & 0xffff0000u);
            const uint32_t va = __float_as_uint(ra), vb = __float_as_uint(rb);
            const float la = ra - __uint_as_float(va & 0xffff0000u), lb = rb - __uint_as_float(vb & 0xffff0000u);
            *reinterpret_cast<uint32_t*>(dst + r * G::PITCH) = __builtin_amdgcn_perm(ub, ua, 0x07060302u);
            *reinterpret_cast<uint32_t*>(dst + r * G::PITCH + G::PLANE) = __builtin_amdgcn_perm(vb, va, 0x07060302u);
            *reinterpret_cast<uint32_t*>(dst + r * G::PITCH + 2 * G::PLANE) =
                __builtin_amdgcn_perm(__float_as_uint(lb), __float_as_uint(la), 0x07060302u);
        }
    };

    // Rectangle of this wave in round r: whole rounds give a workgroup's waves consecutive rectangles; the last, partial
    // round is dealt across the workgroups (wave 0 of each first), so that no compute unit runs a full extra round.
    const int step = (int)gridDim.x * G::WAVES;
    const int whole = g.ntiles / step;
    auto tile_of = [&](int r) {
        if (r < whole) return r * step + (int)blockIdx.x * G::WAVES + wave;
        return r == whole ? whole * step + wave * (int)gridDim.x + (int)blockIdx.x : g.ntiles;   // past the last round: no rectangle
    };
    int t = tile_of(0);
    if (t < g.ntiles) request(t);              // the first patch is on its way while the weights are staged
    if constexpr (!BWN) {   // weights of this channel tile -> LDS, split on the way (w [O][k][k][C]; a run is 8 consecutive values of one filter
        // row, zero past the row's end; column = output channel): unit (plane, run, column) of wlds.  Every load is issued
        // before the first split; pairs past the end repeat the last one and store nothing.
        constexpr int PER = (G::WUNITS + G::WAVES * 64 - 1) / (G::WAVES * 64);
        float xs[PER][8];
#pragma unroll
        for (int i = 0; i < PER; ++i) {
            const int p = min(tid + i * G::WAVES * 64, G::WUNITS - 1);
            const int rho = p >> 6, o = min(n0 + (p & 63), g.O - 1);
            const int r = rho / G::RPR, j = rho - r * G::RPR;
            const float* wrow = static_cast<const float*>(wv) + ((long long)o * G::KS + r) * G::SEG;
#pragma unroll
            for (int e = 0; e < 8; ++e) xs[i][e] = wrow[min(8 * j + e, G::SEG - 1)];
        }
#pragma unroll
        for (int i = 0; i < PER; ++i) {
            const int p = tid + i * G::WAVES * 64;
            const int rho = min(p, G::WUNITS - 1) >> 6;
            const int j = rho % G::RPR;
            const bool col_ok = n0 + (p & 63) < g.O;
            uint32_t hi[4] = {0u, 0u, 0u, 0u}, mid[4] = {0u, 0u, 0u, 0u}, lo[4] = {0u, 0u, 0u, 0u};
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                const float x0 = (col_ok && 8 * j + e < G::SEG) ? xs[i][e] : 0.f;
                const uint32_t a = __float_as_uint(x0);
                const float r1 = x0 - __uint_as_float(a & 0xffff0000u);
                const uint32_t b = __float_as_uint(r1);
                const float r2 = r1 - __uint_as_float(b & 0xffff0000u);
                hi[e >> 1] |= (a >> 16) << (16 * (e & 1));
                mid[e >> 1] |= (b >> 16) << (16 * (e & 1));
                lo[e >> 1] |= (__float_as_uint(r2) >> 16) << (16 * (e & 1));
            }
            if (p < G::WUNITS) {
                wlds[p] = make_uint4(hi[0], hi[1], hi[2], hi[3]);
                wlds[G::WUNITS + p] = make_uint4(mid[0], mid[1], mid[2], mid[3]);
                wlds[2 * G::WUNITS + p] = make_uint4(lo[0], lo[1], lo[2], lo[3]);
            }
        }
    }
    if constexpr (BWN) {    // weight bits of this channel tile -> LDS as bf16 +1.0 / -1.0 (0 past a filter row's end and past
        // the last channel): a run of 8 values lies in at most 8 / C + 2 tap words, all of them requested before the first is used
        const uint32_t* wbits = static_cast<const uint32_t*>(wv);
        constexpr int PER = (G::WUNITS + G::WAVES * 64 - 1) / (G::WAVES * 64), TW = 8 / G::CIN + 2;
        uint32_t tw[PER][TW];
#pragma unroll
        for (int i = 0; i < PER; ++i) {
            const int p = min(tid + i * G::WAVES * 64, G::WUNITS - 1);
            const int rho = p >> 6, o = min(n0 + (p & 63), g.O - 1);
            const int r = rho / G::RPR, j = rho - r * G::RPR;
            const uint32_t* wrow = wbits + ((long long)o * G::KS + r) * G::KS;          // one word per tap
            const int t0 = (8 * j) / G::CIN;
#pragma unroll
            for (int q = 0; q < TW; ++q) tw[i][q] = wrow[min(t0 + q, G::KS - 1)];
        }
#pragma unroll
        for (int i = 0; i < PER; ++i) {
            const int p = tid + i * G::WAVES * 64;
            const int rho = min(p, G::WUNITS - 1) >> 6;
            const int j = rho % G::RPR;
            const bool col_ok = n0 + (p & 63) < g.O;
            const int t0 = (8 * j) / G::CIN;
            uint32_t pk[4] = {0u, 0u, 0u, 0u};
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                const int el = 8 * j + e, t = el / G::CIN, c = el - t * G::CIN;
                uint32_t word = 0u;
#pragma unroll
                for (int q = 0; q < TW; ++q) word = (t - t0 == q) ? tw[i][q] : word;
                const uint32_t val = !(col_ok && el < G::SEG) ? 0u : ((word >> c) & 1u) ? 0x3F80u : 0xBF80u;
                pk[e >> 1] |= val << (16 * (e & 1));
            }
            if (p < G::WUNITS) wlds[p] = make_uint4(pk[0], pk[1], pk[2], pk[3]);
        }
    }
    if (t < g.ntiles) stage(t);
    __syncthreads();                                                   // the only barrier: the weights are in place
    for (int r = 0; t < g.ntiles; ++r) {
        const int t_next = tile_of(r + 1);
        const bool more = t_next < g.ntiles;
        if (more) request(t_next);

        // ---- K loop, unrolled in full: run index of this lane = 2 * step + half; every offset is a compile-time constant
        v16f_bwn acc[NT];
#pragma unroll
        for (int j = 0; j < NT; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[j][r] = 0.f;
        // two operand sets: the LDS reads of step st + 1 are issued before the MFMAs of step st
        uint4 oa[2][3], ob[2][G::WPL][NT];
        auto fetch = [&](auto st_tag) {
            constexpr int st = decltype(st_tag)::value;
            constexpr int rho0 = 2 * st, rho1 = 2 * st + 1;
            constexpr bool upper_real = rho1 < G::NRUNS;               // false only in the last step of an odd run count
            constexpr int off0 = (rho0 / G::RPR) * G::PITCH + (rho0 % G::RPR) * 16;
            constexpr int off1 = upper_real ? (rho1 / G::RPR) * G::PITCH + (rho1 % G::RPR) * 16 : off0;
            const char* asrc = abase + (half ? off1 : off0);           // one vector instruction: the offsets are constants
            // the upper half-wave's weights: one run further (built into bbase); a run that does not exist re-reads the
            // lower one's slot and multiplies zeroed inputs
            const char* bsrc = upper_real ? bbase + rho0 * (COLS * 16) : bbase - half * (COLS * 16) + rho0 * (COLS * 16);
#pragma unroll
            for (int pl = 0; pl < 3; ++pl) {
                const uint2 lo = *reinterpret_cast<const uint2*>(asrc + pl * G::PLANE);
                const uint2 hi = *reinterpret_cast<const uint2*>(asrc + pl * G::PLANE + 8);
                oa[st & 1][pl] = make_uint4(lo.x, lo.y, hi.x, hi.y);
                if (pl < G::WPL)
#pragma unroll
                    for (int j = 0; j < NT; ++j)
                        ob[st & 1][pl][j] = *reinterpret_cast<const uint4*>(bsrc + pl * (G::WUNITS * 16) + j * (32 * 16));
            }
        };
        auto multiply = [&](auto st_tag) {
            constexpr int st = decltype(st_tag)::value;
            if (2 * st + 1 >= G::NRUNS && half) {
#pragma unroll
                for (int pl = 0; pl < 3; ++pl) oa[st & 1][pl] = make_uint4(0u, 0u, 0u, 0u);
            }
            // smallest terms first: (input term, weight term) pairs in order of decreasing index sum
#pragma unroll
            for (int sum = (TERMS == 9 ? 4 : 2); sum >= 0; --sum)
#pragma unroll
                for (int px = 2; px >= 0; --px) {
                    const int pw = sum - px;
                    if (pw < 0 || pw >= G::WPL) continue;
#pragma unroll
                    for (int j = 0; j < NT; ++j)
                        acc[j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(v8bf_bwn, oa[st & 1][px]),
                                                                         __builtin_bit_cast(v8bf_bwn, ob[st & 1][pw][j]), acc[j], 0, 0, 0);
                }
        };
        fetch(std::integral_constant<int, 0>{});
        __builtin_amdgcn_sched_barrier(0);
        static_for<G::NSTEPS>([&](auto st_tag) {
            constexpr int st = decltype(st_tag)::value;
            if constexpr (st + 1 < G::NSTEPS) fetch(std::integral_constant<int, st + 1>{});
            multiply(st_tag);
            // Left alone, the compiler sinks every LDS read to just before the MFMA that uses it (fewer live registers) and
            // the wave then waits out the LDS latency a dozen times per step: keep the reads of the next step between this
            // step's MFMAs, one each, and let nothing cross a step boundary.
#pragma unroll
            for (int q = 0; q < TERMS * NT; ++q) {
                __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
                __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
            }
            __builtin_amdgcn_sched_barrier(0);
        });

        // ---- epilogue: threshold -> packed bits (and / or the fp32 sums)
        int n, p0, q0;
        tile_origin(t, n, p0, q0);
        const long long img_pix = (long long)n * g.P * g.Q;
        uint32_t wout[NT];
#pragma unroll
        for (int j = 0; j < NT; ++j) wout[j] = 0u;
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            const int lo_row = 8 * (r >> 2) + (r & 3);
#pragma unroll
            for (int j = 0; j < NT; ++j) {
                const float v = acc[j][r];
                if (WANT_Y) {
                    const int m = lo_row + 4 * half;                   // rectangle pixel of this register in this lane
                    const int mp = m % G::FP, mq = m / G::FP;
                    if (p0 + mp < g.P && q0 + mq < g.Q && cok[j])
                        y[(img_pix + (long long)(p0 + mp) * g.Q + q0 + mq) * g.O + n0 + 32 * j + l32] = v;
                }
                if (!WANT_Y || bits != nullptr) {
                    const unsigned long long ball = __builtin_amdgcn_ballot_w64(v >= th[j]);
                    wout[j] = (uint32_t)bnn_bwn_writelane_i32((int)(uint32_t)ball, lo_row, (int)wout[j]);
                    wout[j] = (uint32_t)bnn_bwn_writelane_i32((int)(uint32_t)(ball >> 32), lo_row + 4, (int)wout[j]);
                }
            }
        }
        if ((!WANT_Y || bits != nullptr) && lane < 32 && p0 + dp < g.P && q0 + dq < g.Q) {
            const long long pix = img_pix + (long long)(p0 + dp) * g.Q + q0 + dq;
#pragma unroll
            for (int j = 0; j < NT; ++j) {
                const int wi = (n0 >> 5) + j;
                if (wi < ow) bits[pix * ow + wi] = wout[j];
            }
        }
        if (more) stage(t_next);               // every read of this rectangle's patch has been consumed by its MFMAs
        t = t_next;
    }
}

template <class G, int TERMS, bool WANT_Y>
int launch_conv_f32_wave_v(const float* x, const void* w, const float* thr, float* y, uint32_t* bits, int N, int H, int W, int O,
                           int pad, int P, int Q, void* workspace, size_t workspace_bytes, hipStream_t s) {
    const int col_tiles = (int)cdiv(O, 64);
    WaveArgs g;
    g.N = N; g.H = H; g.W = W; g.O = O; g.pad = pad; g.P = P; g.Q = Q;
    g.tiles_p = (int)cdiv(P, G::FP); g.tiles_q = (int)cdiv(Q, G::FQ);
    g.ntiles = N * g.tiles_p * g.tiles_q;
    g.div_tiles = make_fastdiv((uint32_t)(g.tiles_p * g.tiles_q));
    g.div_tq = make_fastdiv((uint32_t)g.tiles_q);
    // This kernel splits the weights itself while it stages them; the workspace the entry point asks for (the other
    // first-layer kernels keep their expanded weights there) is checked all the same, so that the call's contract does
    // not depend on which kernel serves a shape.
    if (workspace == nullptr || workspace_bytes < (size_t)G::WPL * 2 * G::NSTEPS * 64 * 16 * col_tiles) return BNN_ERR_WORKSPACE;
    static const hipError_t attr = hipFuncSetAttribute(reinterpret_cast<const void*>(&conv_f32_wave_kernel<G, TERMS, WANT_Y>),
                                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)LDS_MAX);
    if (attr != hipSuccess) return BNN_ERR_DEVICE;
    int dev = 0, cus = 0;
    if (hipGetDevice(&dev) != hipSuccess || hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus < 1)
        return BNN_ERR_DEVICE;
    const long long wgs = min(cdiv(g.ntiles, G::WAVES), (long long)max(1, cus / col_tiles));
    hipLaunchKernelGGL((conv_f32_wave_kernel<G, TERMS, WANT_Y>), dim3((unsigned)wgs, (unsigned)col_tiles), dim3(G::WAVES * 64), G::LDS, s, x,
                       w, thr, y, bits, g);
    return check_launch();
}

// The geometries the wave-private kernel is built for.  true: launched (rc receives the status).
bool try_conv_f32_wave(const float* x, const float* w, const float* thr, float* y, uint32_t* bits, int N, int H, int W, int C, int O,
                       int k, int stride, int pad, int P, int Q, int products, void* workspace, size_t workspace_bytes, hipStream_t s,
                       int* rc) {
    if (!(k == 7 && stride == 4 && C == 3)) return false;
    if ((long long)W * C < 2 || (long long)H * W * C >= (1LL << 31)) return false;
    constexpr int FP = 4, FQ = 8;
    typedef WaveGeom<7, 4, 3, FP, FQ> G;
    static_assert(G::LDS <= LDS_MAX, "weights and eight patches fit LDS");
    if ((long long)N * cdiv(P, FP) * cdiv(Q, FQ) >= (1LL << 31) - 65536) return false;
    if (y != nullptr)
        *rc = products == 6 ? launch_conv_f32_wave_v<G, 6, true>(x, w, thr, y, bits, N, H, W, O, pad, P, Q, workspace, workspace_bytes, s)
                            : launch_conv_f32_wave_v<G, 9, true>(x, w, thr, y, bits, N, H, W, O, pad, P, Q, workspace, workspace_bytes, s);
    else
        *rc = products == 6 ? launch_conv_f32_wave_v<G, 6, false>(x, w, thr, y, bits, N, H, W, O, pad, P, Q, workspace, workspace_bytes, s)
                            : launch_conv_f32_wave_v<G, 9, false>(x, w, thr, y, bits, N, H, W, O, pad, P, Q, workspace, workspace_bytes, s);
    return true;
}

// Binarized weights on the wave-private kernel: the 11x11 stride-4 first layer of 3-channel images (one weight plane,
// three term products; six waves: a patch is 23 rows).  true: launched (rc receives the status).
bool try_bwn_wave(const float* x, const uint32_t* wbits, const float* thr, float* y, uint32_t* bits, int N, int H, int W, int C, int O,
                  int k, int stride, int pad, int P, int Q, void* workspace, size_t workspace_bytes, hipStream_t s, int* rc) {
    if (!(k == 11 && stride == 4 && C == 3)) return false;
    if ((long long)W * C < 2 || (long long)H * W * C >= (1LL << 31)) return false;
    constexpr int FP = 4, FQ = 8;
    typedef WaveGeom<11, 4, 3, FP, FQ, 6, 1> G;
    static_assert(G::LDS <= LDS_MAX, "weights and six patches fit LDS");
    const long long tiles = (long long)N * cdiv(P, FP) * cdiv(Q, FQ);
    if (tiles >= (1LL << 31) - 65536) return false;
    if (tiles < 4096) return false;            // small batches: the LDS-staged and direct kernels (more workgroups, shorter prologue)
    *rc = y != nullptr ? launch_conv_f32_wave_v<G, 3, true>(x, wbits, thr, y, bits, N, H, W, O, pad, P, Q, workspace, workspace_bytes, s)
                       : launch_conv_f32_wave_v<G, 3, false>(x, wbits, thr, y, bits, N, H, W, O, pad, P, Q, workspace, workspace_bytes, s);
    return true;
}

// Real-valued weights on the same kernel: three weight planes, nine exact products per element pair.
size_t conv_f32_split_workspace_bytes(int C, int O, int k) {
    const long long seg = (long long)k * C, nruns = k * ((seg + 7) / 8), nsteps = ((nruns + 1) / 2 + 2) / 3 * 3;
    return (size_t)(cdiv(O, 64) * 64 * 3 * 2 * nsteps * 16);
}

int launch_conv_f32_split_thr(const float* x, const float* w, const float* thr, float* y, uint32_t* bits, int N, int H, int W,
                              int C, int O, int k, int stride, int pad, int products, void* workspace, size_t workspace_bytes,
                              hipStream_t s) {
    const int P = (H + 2 * pad - k) / stride + 1, Q = (W + 2 * pad - k) / stride + 1;
    int rc = BNN_OK;
    if (try_conv_f32_wave(x, w, thr, y, bits, N, H, W, C, O, k, stride, pad, P, Q, products, workspace, workspace_bytes, s, &rc))
        return rc;                             // wave-private patches in LDS for the filter geometries that kernel is built for
    if (products == 6)
        return launch_bwn_direct<2, 2, 8, 3, 6>(x, w, thr, y, bits, N, H, W, C, O, k, stride, pad, P, Q, workspace, workspace_bytes, s);
    return launch_bwn_direct<2, 2, 8, 3>(x, w, thr, y, bits, N, H, W, C, O, k, stride, pad, P, Q, workspace, workspace_bytes, s);
}

}  // namespace bnn
