// Matrix-core path, LDS-staged variant (kernel template).
//
// Same arithmetic as bnn_mfma_kernel.h (fp4 expansion in registers, 32x32x64 MFMA, same epilogue),
// but the packed operands reach the waves through LDS instead of straight from L2:
//   - the workgroup loads a K-slab of 512 bits of all its A rows and B rows with 16-byte loads in
//     which four consecutive lanes cover 64 contiguous bytes of one row (four times fewer distinct
//     cache lines per load instruction than the per-fragment gather of the direct kernel, and rows
//     shared by two waves are fetched once);
//   - slabs are double-buffered in LDS; the global loads of slab s+2 are in flight, in registers,
//     while slab s is being multiplied, so a full slab of MFMA work hides the memory latency;
//   - LDS layout per slab: [granule 0..3][row] of 16-byte units, rows padded by 2 units.  A wave
//     reading fragment rows l%32 of one granule reads 32 consecutive units (conflict-free); the
//     pad of 2 makes the transposing writes (4 granules x 16 rows per wave instruction) hit
//     distinct bank groups as well.
// One barrier per slab.  Out-of-frame taps of a convolution load zero words (-1 padding); the
// exclude-padding mode and channel counts other than 64 or a multiple of 128 stay on the direct
// kernel.
#ifndef BNN_MFMA_STAGED_H
#define BNN_MFMA_STAGED_H

#include <type_traits>

#include "bnn_mfma_kernel.h"

namespace bnn {
namespace mfma {

// U: bytes per global load instruction and lane: 16, or 8 when a pixel has only 8 bytes (C = 64).
template <class TL, int U, bool CONV>
__global__ __launch_bounds__(256, TL::MINB) void mfma_staged_kernel(const uint32_t* __restrict__ A,
                                                                    const uint32_t* __restrict__ B, Geom g, Epi e,
                                                                    int gx, int gy) {
    constexpr int MT = TL::MT, NT = TL::NT;
    constexpr int ROWS = TL::ROWS, COLS = TL::COLS;
    constexpr int RA = ROWS + 2, RB = COLS + 2;          // padded row counts, in 16-byte units
    constexpr int STAGE = 4 * (RA + RB);                 // units per slab
    constexpr int LA = ROWS / 64, LB = (COLS + 63) / 64; // granules each thread moves per slab
    extern __shared__ uint4 lds[];                       // 2 * STAGE units, sized at launch
    // BMM on the large tiles: the registers left beside 128 accumulators suffice without spilling
    if constexpr (!CONV && TL::MINB <= 2) accumulators_in_agprs();

    int bx, by;
    if (!tile_coords(gx, gy, bx, by)) return;            // uniform for the workgroup
    const int tid = threadIdx.x;
    const int lane = tid & 63, l32 = lane & 31, half = lane >> 5, wave = tid >> 6;
    const int wm = wave / TL::WN, wn = wave % TL::WN;
    const long long m_base = (long long)bx * ROWS;
    const int n_base = by * COLS;

    uint32_t c2;
    asm volatile("v_mov_b32 %0, 0x22222222" : "=v"(c2));

    // ---- loader: thread -> granule g4 of rows r4 + 64*q ---------------------------------------
    const int g4 = tid & 3, r4 = tid >> 2;
    const uint32_t* ap[LA];
    int ay0[LA], ax0[LA];
#pragma unroll
    for (int q = 0; q < LA; ++q) {
        long long row = m_base + r4 + 64 * q;
        if (row > g.rows - 1) row = g.rows - 1;          // clamp: loads stay in bounds, results are dropped
        if (CONV) {
            const int n = fast_div((int)row, g.div_pq);
            const int rem = (int)row - n * (g.P * g.Q);
            const int p = fast_div(rem, g.div_q), qq = rem - p * g.Q;
            ay0[q] = p * g.stride - g.pad;
            ax0[q] = qq * g.stride - g.pad;
            ap[q] = A + (long long)n * g.H * g.W * g.lda_w;
        } else {
            ay0[q] = 0; ax0[q] = 0;
            ap[q] = A + row * g.lda_w;
        }
    }
    const uint32_t* bp[LB];
#pragma unroll
    for (int q = 0; q < LB; ++q) {
        const int col = min(n_base + r4 + 64 * q, g.cols - 1);
        bp[q] = B + (long long)col * g.ldb_w;
    }
    const int kwords = g.taps * g.tw;                    // packed words in one B row / one A row of the GEMM
    const int nslabs = (kwords + 15) / 16;

    uint4 sa[LA], sb[LB];                                // staging registers: one slab in flight

    auto load_slab = [&](int s) {
        const int wq = (s * 4 + g4) * 4;                 // first word of this thread's granule in the K order
        if (!CONV) {
            const bool ok = wq < kwords;
#pragma unroll
            for (int q = 0; q < LA; ++q) {
                sa[q] = *reinterpret_cast<const uint4*>(ap[q] + (ok ? wq : 0));
                if (!ok) sa[q] = make_uint4(0u, 0u, 0u, 0u);
            }
#pragma unroll
            for (int q = 0; q < LB; ++q) {
                sb[q] = *reinterpret_cast<const uint4*>(bp[q] + (ok ? wq : 0));
                if (!ok) sb[q] = make_uint4(0u, 0u, 0u, 0u);
            }
        } else if (U == 16) {
            // tap and offset of this granule without a vector division: the slab's first word is
            // wave-uniform (scalar division), the lane adds at most 12 words and wraps a few times
            const int w0 = s * 16;
            int tap = w0 / g.tw, off = w0 - tap * g.tw + g4 * 4;  // tw is a multiple of 4 here
#pragma unroll
            for (int it = 0; it < 3; ++it)
                if (off >= g.tw) { off -= g.tw; ++tap; }
            const bool ok = wq < kwords;
            const int r = (tap * g.kinv) >> 16, sx = tap - r * g.k;
#pragma unroll
            for (int q = 0; q < LA; ++q) {
                const int y = ay0[q] + r, x = ax0[q] + sx;
                const bool in = ok && (unsigned)y < (unsigned)g.H && (unsigned)x < (unsigned)g.W;
                sa[q] = *reinterpret_cast<const uint4*>(ap[q] + (in ? (y * g.W + x) * g.lda_w + off : 0));
                if (!in) sa[q] = make_uint4(0u, 0u, 0u, 0u);       // out of frame: all -1; past the end: pad
            }
#pragma unroll
            for (int q = 0; q < LB; ++q) {
                sb[q] = *reinterpret_cast<const uint4*>(bp[q] + (ok ? wq : 0));
                if (!ok) sb[q] = make_uint4(0u, 0u, 0u, 0u);
            }
        } else {                                         // U == 8: two words per pixel, a granule spans two taps
            uint2 lo[LA], hi[LA];
#pragma unroll
            for (int h = 0; h < 2; ++h) {
                const int tap = (wq >> 1) + h;
                const bool ok = tap < g.taps;
                const int r = (tap * g.kinv) >> 16, sx = tap - r * g.k;
#pragma unroll
                for (int q = 0; q < LA; ++q) {
                    const int y = ay0[q] + r, x = ax0[q] + sx;
                    const bool in = ok && (unsigned)y < (unsigned)g.H && (unsigned)x < (unsigned)g.W;
                    uint2 v = *reinterpret_cast<const uint2*>(ap[q] + (in ? (y * g.W + x) * 2 : 0));
                    if (!in) v = make_uint2(0u, 0u);
                    if (h == 0) lo[q] = v; else hi[q] = v;
                }
            }
#pragma unroll
            for (int q = 0; q < LA; ++q) sa[q] = make_uint4(lo[q].x, lo[q].y, hi[q].x, hi[q].y);
#pragma unroll
            for (int q = 0; q < LB; ++q) {
                const bool ok0 = wq < kwords, ok1 = wq + 2 < kwords;
                uint2 v0 = *reinterpret_cast<const uint2*>(bp[q] + (ok0 ? wq : 0));
                uint2 v1 = *reinterpret_cast<const uint2*>(bp[q] + (ok1 ? wq + 2 : 0));
                if (!ok0) v0 = make_uint2(0u, 0u);
                if (!ok1) v1 = make_uint2(0u, 0u);
                sb[q] = make_uint4(v0.x, v0.y, v1.x, v1.y);
            }
        }
    };

    auto store_slab = [&](int buf) {
        uint4* base = lds + buf * STAGE;
#pragma unroll
        for (int q = 0; q < LA; ++q) base[g4 * RA + r4 + 64 * q] = sa[q];
#pragma unroll
        for (int q = 0; q < LB; ++q)
            if (r4 + 64 * q < COLS) base[4 * RA + g4 * RB + r4 + 64 * q] = sb[q];
    };

    v16f acc[MT][NT];
#pragma unroll
    for (int i = 0; i < MT; ++i)
#pragma unroll
        for (int j = 0; j < NT; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

    // Multiplies the slab in buffer `buf`.  FULL: all 8 K-steps; otherwise the K range ends inside
    // this slab and only the first `steps[c]` K-steps of chunk c hold data (wave-uniform).
    auto compute_slab = [&](int buf, auto full, int steps0, int steps1) {
        constexpr bool FULL = decltype(full)::value;
        const uint4* base = lds + buf * STAGE;
#pragma unroll
        for (int c = 0; c < 2; ++c) {                    // the two 256-bit chunks of the slab
            const int nst = c == 0 ? steps0 : steps1;
            if (!FULL && nst == 0) continue;
            const int gq = 2 * c + half;
            uint4 fa[MT], fb[NT];
#pragma unroll
            for (int i = 0; i < MT; ++i) fa[i] = base[gq * RA + wm * (MT * 32) + 32 * i + l32];
#pragma unroll
            for (int j = 0; j < NT; ++j) fb[j] = base[4 * RA + gq * RB + wn * (NT * 32) + 32 * j + l32];
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                if (!FULL && v >= nst) break;
                v8i ea[MT], eb[NT];
#pragma unroll
                for (int i = 0; i < MT; ++i) {
                    const uint32_t w = v == 0 ? fa[i].x : v == 1 ? fa[i].y : v == 2 ? fa[i].z : fa[i].w;
                    ea[i] = expand_fp4(w, c2);
                }
#pragma unroll
                for (int j = 0; j < NT; ++j) {
                    const uint32_t w = v == 0 ? fb[j].x : v == 1 ? fb[j].y : v == 2 ? fb[j].z : fb[j].w;
                    eb[j] = expand_fp4(w, c2);
                }
#pragma unroll
                for (int i = 0; i < MT; ++i)
#pragma unroll
                    for (int j = 0; j < NT; ++j)
                        acc[i][j] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(
                            ea[i], eb[j], acc[i][j], 4 /*A: E2M1*/, 4 /*B: E2M1*/, 0, 0, 0, 0);
                if constexpr (FULL) {
                    // ask the scheduler for an even mix: each MFMA followed by its share of the next K-step's
                    // expansion (vector ALU), so that the matrix pipe and the vector ALU run side by side
#pragma unroll
                    for (int q = 0; q < MT * NT; ++q) {
                        __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);                                  // one MFMA
                        __builtin_amdgcn_sched_group_barrier(0x002, (MT + NT) * 7 / (MT * NT), 0);          // VALU
                    }
                }
            }
        }
    };

    // K-steps of the last slab that hold data: chunk c covers words 8c .. 8c+7 of the slab, its
    // K-step v the words 8c+v (lower half-wave) and 8c+4+v (upper half-wave).
    const int wl = kwords - (nslabs - 1) * 16;           // valid words in the last slab, 1..16
    const int last0 = min(4, wl), last1 = min(4, max(0, wl - 8));
    const bool last_full = (last0 == 4 && last1 == 4);

    load_slab(0);
    store_slab(0);
    if (nslabs > 1) load_slab(1);
    __syncthreads();
    const int nfull = last_full ? nslabs : nslabs - 1;   // the hot loop only sees complete slabs
    for (int s = 0; s < nfull; ++s) {
        const int buf = s & 1;
        compute_slab(buf, std::true_type{}, 4, 4);
        if (s + 1 < nslabs) {
            store_slab(buf ^ 1);                         // slab s+1: loaded one iteration ago
            if (s + 2 < nslabs) load_slab(s + 2);
        }
        __syncthreads();
    }
    if (!last_full) compute_slab((nslabs - 1) & 1, std::false_type{}, last0, last1);

    const long long m0 = m_base + (long long)wm * (MT * 32);
    const int n0 = n_base + wn * (NT * 32);
    // bit positions multiplied in all: 64 per K-step
    const int processed = (nslabs - 1) * 512 + (last0 + last1) * 64;
    int corr2 = 0;
    if (CONV && g.A2 != nullptr) corr2 = extra_source<MT, NT>(acc, g, m0, n0, lane, c2) - g.bits2;
    Epi es = e;
    es.sums_tiled = 0;          // blocked 16-bit sums go to the direct kernel (launch_mfma): that code is left out here
    epilogue<MT, NT, CONV, false>(acc, m0, n0, lane, g, es, processed - g.taps * g.bits_tap + corr2, 0);
}

template <class TL, int U, bool CONV>
int launch_staged_tile(const uint32_t* A, const uint32_t* B, const Geom& g, const Epi& e, hipStream_t s) {
    const int col_span = (e.bits != nullptr) ? max(g.cols, e.ldbits_w * 32) : g.cols;
    const int gx = (int)cdiv(g.rows, TL::ROWS), gy = (int)cdiv(col_span, TL::COLS);
    const unsigned nwg = (unsigned)(cdiv((long long)gx * gy, 8) * 8);
    constexpr size_t lds_bytes = 2 * 4 * (TL::ROWS + 2 + TL::COLS + 2) * 16;
    static const hipError_t attr = hipFuncSetAttribute(reinterpret_cast<const void*>(&mfma_staged_kernel<TL, U, CONV>),
                                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds_bytes);
    if (attr != hipSuccess) return BNN_ERR_DEVICE;
    hipLaunchKernelGGL((mfma_staged_kernel<TL, U, CONV>), dim3(nwg), dim3(256), lds_bytes, s, A, B, g, e, gx, gy);
    return check_launch();
}

}  // namespace mfma
}  // namespace bnn
#endif
