// Matrix-core path (kernel template; included by the translation units that instantiate it): +1/-1 products on the CDNA4 MFMA units.
//
// gfx950 has no 1-bit matrix type.  Its densest one is the 4-bit float E2M1 of
// v_mfma_f32_32x32x64_f8f6f4, in which +1.0 is 0b0010 and -1.0 is 0b1010.  A packed word of 32
// bits becomes the 32 four-bit operands one lane feeds to that instruction with seven VALU
// operations: nibble i of output register j is 0x2 | (bit(4i+j) << 3).  This maps bit 1 to -1.0
// and bit 0 to +1.0 in BOTH operands, which leaves every product, hence the dot product of
// Eq. 2, unchanged ((-a)(-b) = ab) and saves inverting the word.  Which bit lands in which K
// slot of the instruction does not matter as long as both operands use the same rule.
// Products are +-1 and are accumulated in fp32, exact while |sum| < 2^24 (K <= 2^20 here).
//
// Operand delivery: in the 32x32x64 shape lane l supplies row (l % 32) and the 32 K-values of
// K-group (l / 32) -- exactly one packed word.  This file holds the DIRECT kernel: fragments are read
// straight from global memory / L2 into registers, 4 to 16 bytes per lane and request, through a ring
// of up to 8 chunk buffers that are all requested before the first multiply (the layers of a network
// have short K: their time is memory latency and instruction issue, not the matrix pipe).  The
// LDS-staged kernel for long K is in bnn_mfma_staged.h and shares the epilogue below.
//
// Tiling: a workgroup is 4 waves, a wave owns MT x NT accumulator tiles of 32 x 32: 256 x 128 per
// workgroup (waves 2 x 2, 4 x 2 tiles each), 512 x 64, 128 x 128 or 64 x 64 (see Tile below).
//
// Epilogue: in the 32x32 accumulator layout register r of lane l holds row 8*(r/4) + 4*(l/32)
// + r%4, column l%32.  A threshold compare of one register therefore yields, as a 64-bit wave
// ballot, the packed output words of two rows; they are collected with v_writelane so that lane
// m ends up with the word of row m.  int32 sums never go to memory unless asked for.
#ifndef BNN_MFMA_KERNEL_H
#define BNN_MFMA_KERNEL_H
#include <limits.h>

#include "bnn_internal.h"

namespace bnn {
namespace mfma {

typedef int v8i __attribute__((ext_vector_type(8)));
typedef float v16f __attribute__((ext_vector_type(16)));

template <int V> struct WordVec;
template <> struct WordVec<1> { typedef uint32_t type; };
template <> struct WordVec<2> { typedef uint2 type; };
template <> struct WordVec<4> { typedef uint4 type; };

template <int V>
__device__ __forceinline__ void load_words(const uint32_t* p, uint32_t (&a)[V]) {
    typename WordVec<V>::type v = *reinterpret_cast<const typename WordVec<V>::type*>(p);
    if constexpr (V == 1) { a[0] = v; }
    else if constexpr (V == 2) { a[0] = v.x; a[1] = v.y; }
    else { a[0] = v.x; a[1] = v.y; a[2] = v.z; a[3] = v.w; }
}

// 32 packed bits -> 32 E2M1 values in 4 registers (the upper 4 of the 8-register operand are
// ignored by the instruction for 4-bit formats).  c2 holds 0x22222222 in a VGPR so that each
// output needs one shift and one v_and_or_b32.
__device__ __forceinline__ v8i expand_fp4(uint32_t w, uint32_t c2) {
    v8i r;
    r[0] = (int)(((w << 3) & 0x88888888u) | c2);
    r[1] = (int)(((w << 2) & 0x88888888u) | c2);
    r[2] = (int)(((w << 1) & 0x88888888u) | c2);
    r[3] = (int)((w & 0x88888888u) | c2);
    r[4] = 0; r[5] = 0; r[6] = 0; r[7] = 0;
    return r;
}

// A lane's 32 bytes of a blocked 16-bit residual read ahead of the main loop (passed by value, so that it stays
// in registers).
struct Fetched {
    uint4 lo, hi;
    bool valid;
};

// v_writelane_b32 through the compiler's own intrinsic (clang has no builtin for it), so that the
// wait states the hardware needs between a VALU compare that writes an SGPR pair and the
// v_writelane that reads it are inserted by the compiler: hand-written asm reads a stale value.
extern "C" __device__ int bnn_llvm_writelane_i32(int val, int lane, int old) __asm("llvm.amdgcn.writelane.i32");

// Returns `old` with the value of lane `lane` replaced by the wave-uniform `val`.
__device__ __forceinline__ uint32_t write_lane(uint32_t val, int lane, uint32_t old) {
    return (uint32_t)bnn_llvm_writelane_i32((int)val, lane, (int)old);
}

// Makes the compiler keep the MFMA accumulators in the accumulation registers (AGPRs).  When a kernel's
// register budget is 256 or less (two or more waves per SIMD) the compiler otherwise puts them in ordinary
// VGPRs, and the accumulator reads and writes of every MFMA then compete with the vector ALU for the VGPR
// ports: the same expansion + MFMA loop runs at 5.4 PFLOP/s with VGPR accumulators and at 6.4 with AGPR ones.
// An (empty) inline-asm result in an AGPR is what tells the compiler that the function uses AGPRs at all.
__device__ __forceinline__ void accumulators_in_agprs() {
    int hint;
    asm volatile("; accumulators in AGPRs" : "=a"(hint));
}

// Workgroup shape: WM x WN waves, each owning MT x NT accumulator tiles of 32 x 32; MINB is the
// number of workgroups per CU the register allocation is sized for.
template <int MT_, int NT_, int WM_, int WN_, int MINB_>
struct Tile {
    static constexpr int MT = MT_, NT = NT_, WM = WM_, WN = WN_, MINB = MINB_;
    static constexpr int ROWS = WM_ * MT_ * 32, COLS = WN_ * NT_ * 32;
};
typedef Tile<4, 2, 2, 2, 2> TileBig;    // 256 x 128
typedef Tile<4, 2, 4, 1, 2> TileTall;   // 512 x 64   (at most 64 output columns)
typedef Tile<2, 2, 2, 2, 3> TileMid;    // 128 x 128
typedef Tile<1, 1, 2, 2, 4> TileSmall;  // 64 x 64

// Workgroup id -> tile coordinates.  Consecutive workgroup ids are dealt round-robin to the 8
// XCDs, each with its own L2: give every XCD one contiguous range of tiles, and inside a range
// walk groups of 8 row tiles for each column tile, so that the workgroups resident on an XCD at
// the same time share A rows and B rows in that L2.
__device__ __forceinline__ bool tile_coords(int gx, int gy, int& bx, int& by) {
    const int total = gx * gy;
    const int per_xcd = (total + 7) / 8;
    const int id = (int)blockIdx.x;
    const int t = (id & 7) * per_xcd + (id >> 3);
    if (t >= total) return false;
    constexpr int GM = 8;
    const int span = GM * gy;
    const int group = t / span;
    const int first = group * GM;
    const int gsz = min(gx - first, GM);
    const int in = t - group * span;
    by = in / gsz;
    bx = first + (in - by * gsz);
    return true;
}

// Generic epilogue body: optional residual (int32 tensor or +1/-1 from packed bits), optional int32
// store, optional threshold + pack.
template <int MT, int NT, bool CONV, bool EXCL, bool HAS_RESID>
__device__ __forceinline__ void epilogue_generic(v16f (&acc)[MT][NT], const long long m0, const int n0, const int lane,
                                                 const Geom& g, const Epi& e, const int corr_all, const int pad_tap,
                                                 const int (&thi)[NT], const bool (&cok)[NT], const bool row_corr,
                                                 const Fetched fetched) {
    const int l32 = lane & 31;
    const int half = lane >> 5;
    const bool tiled16 = CONV && e.sums_tiled != 0;              // blocked 16-bit sums (uniform; the layer chain's convolutions)
#pragma unroll
    for (int i = 0; i < MT; ++i) {
        uint32_t wout[NT];
#pragma unroll
        for (int j = 0; j < NT; ++j) wout[j] = 0u;
        const long long rbase = m0 + 32 * i;
        if (rbase >= g.rows) break;                              // uniform per wave
        // Residual of this 32-row slab: every load is issued before the first store, so the
        // memory latency is paid once per slab and not once per element.  (sum_out may alias
        // residual_in: each element is still read before the same thread writes it.)
        int rv[16][NT];
        if (HAS_RESID && tiled16 && e.resid16 != nullptr) {
            // a lane's 16 values of a 32x32 block are 32 contiguous bytes (sums16_index)
#pragma unroll
            for (int j = 0; j < NT; ++j) {
                uint4 lo = make_uint4(0u, 0u, 0u, 0u), hi = lo;
                if (fetched.valid) {                                     // MT == NT == 1: read before the main loop
                    lo = fetched.lo; hi = fetched.hi;
                } else if (n0 + 32 * j < g.cols) {
                    const uint4* src = reinterpret_cast<const uint4*>(
                        e.resid16 + ((rbase >> 5) * (long long)(e.ldc >> 5) + ((n0 >> 5) + j)) * 1024 + lane * 16);
                    lo = src[0]; hi = src[1];
                }
                const uint32_t w[8] = {lo.x, lo.y, lo.z, lo.w, hi.x, hi.y, hi.z, hi.w};
#pragma unroll
                for (int r = 0; r < 16; ++r) rv[r][j] = (r & 1) ? ((int)w[r >> 1] >> 16) : (int)(short)(w[r >> 1] & 0xffffu);
            }
        } else if (HAS_RESID && e.resid == nullptr && e.resid16 == nullptr) {
            // +1/-1 taken from a packed tensor (first residual of a chain): lane t of the lower half reads the
            // word of row rbase + t once; every row's word then comes from that lane
#pragma unroll
            for (int j = 0; j < NT; ++j) {
                const long long rrow = min(rbase + l32, g.rows - 1);
                const int wi = min((n0 >> 5) + j, e.ld_resid_bits_w - 1);
                const uint32_t mine = e.resid_bits[rrow * (long long)e.ld_resid_bits_w + wi];
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const int lo_row = 8 * (r >> 2) + (r & 3);
                    const uint32_t w0 = (uint32_t)__builtin_amdgcn_readlane((int)mine, lo_row);
                    const uint32_t w1 = (uint32_t)__builtin_amdgcn_readlane((int)mine, lo_row + 4);
                    rv[r][j] = (((half ? w1 : w0) >> l32) & 1u) ? 1 : -1;
                }
            }
        } else if (HAS_RESID) {
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const long long row = rbase + 8 * (r >> 2) + 4 * half + (r & 3);
                const bool rok = row < g.rows;
#pragma unroll
                for (int j = 0; j < NT; ++j) {
                    const int col = n0 + 32 * j + l32;
                    rv[r][j] = 0;
                    if (rok && cok[j]) {
                        if (e.resid != nullptr) {
                            rv[r][j] = e.resid[row * (long long)e.ldc + col];
                        } else {
                            rv[r][j] = (int)e.resid16[row * (long long)e.ldc + col];
                        }
                    }
                }
            }
        } else {
#pragma unroll
            for (int r = 0; r < 16; ++r)
#pragma unroll
                for (int j = 0; j < NT; ++j) rv[r][j] = 0;
        }
        uint32_t pk[NT][8];                                      // blocked 16-bit sums: two values per word
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            const int rloc = 8 * (r >> 2) + 4 * half + (r & 3);
            const long long row = rbase + rloc;
            const bool rok = row < g.rows;
            int corr = corr_all;
            if (row_corr) {
                const int rr = (int)(rok ? row : g.rows - 1);
                const int rem = rr - fast_div(rr, g.div_pq) * (g.P * g.Q);
                const int p = fast_div(rem, g.div_q), q = rem - p * g.Q;
                const int ylo = p * g.stride - g.pad, xlo = q * g.stride - g.pad;
                const int vy = min(ylo + g.k, g.H) - max(ylo, 0);
                const int vx = min(xlo + g.k, g.W) - max(xlo, 0);
                // pad positions of the in-frame taps, plus what is not per tap (the fused second source's pad positions)
                corr = vy * vx * pad_tap + (corr_all - g.taps * pad_tap);
            }
#pragma unroll
            for (int j = 0; j < NT; ++j) {
                const int col = n0 + 32 * j + l32;
                const int v = (int)acc[i][j][r] - corr + (HAS_RESID ? rv[r][j] : 0);
                if (e.out != nullptr && rok && cok[j]) e.out[row * (long long)e.ldc + col] = e.out_f32 ? __float_as_int((float)v) : v;
                if (e.out16 != nullptr) {
                    if (tiled16) {
                        if (r & 1) pk[j][r >> 1] |= (uint32_t)v << 16;
                        else pk[j][r >> 1] = (uint32_t)v & 0xffffu;
                    } else if (rok && cok[j]) {
                        e.out16[row * (long long)e.ldc + col] = (int16_t)v;
                    }
                }
                if (e.bits != nullptr) {
                    const unsigned long long ball = __builtin_amdgcn_ballot_w64(v >= thi[j]);
                    const int lo_row = 8 * (r >> 2) + (r & 3);
                    wout[j] = write_lane((uint32_t)ball, lo_row, wout[j]);
                    wout[j] = write_lane((uint32_t)(ball >> 32), lo_row + 4, wout[j]);
                }
            }
        }
        if (e.out16 != nullptr && tiled16) {
#pragma unroll
            for (int j = 0; j < NT; ++j) {
                if (n0 + 32 * j < g.cols) {      // whole blocks: cols is a multiple of 32, rows are padded to 32
                    uint4* dst = reinterpret_cast<uint4*>(
                        e.out16 + ((rbase >> 5) * (long long)(e.ldc >> 5) + ((n0 >> 5) + j)) * 1024 + lane * 16);
                    dst[0] = make_uint4(pk[j][0], pk[j][1], pk[j][2], pk[j][3]);
                    dst[1] = make_uint4(pk[j][4], pk[j][5], pk[j][6], pk[j][7]);
                }
            }
        }
        if (e.bits != nullptr && lane < 32) {
            const long long row = rbase + lane;
            if (row < g.rows) {
#pragma unroll
                for (int j = 0; j < NT; ++j) {
                    const int wi = (n0 >> 5) + j;
                    if (wi < e.ldbits_w) e.bits[row * e.ldbits_w + wi] = wout[j];
                }
            }
        }
    }
}

// Epilogue of a residual layer inside a layer chain: blocked 16-bit sums in and / or out (or the +1/-1 of packed
// bits as the residual), threshold -> bits.  Straight-line code in fp32, where the accumulators already are:
// every value is an integer below 2^24 in magnitude, so the arithmetic is exact.  No pixel-dependent correction.
typedef short v2s __attribute__((ext_vector_type(2)));

template <int MT, int NT>
__device__ __forceinline__ void epilogue_chain(v16f (&acc)[MT][NT], const long long m0, const int n0, const int lane,
                                               const Geom& g, const Epi& e, const int corr_all, const int (&thi)[NT],
                                               const bool (&cok)[NT], const Fetched fetched) {
    const int l32 = lane & 31;
    const float corr = (float)corr_all;
    float thf[NT];                                           // acc + residual >= threshold + correction
#pragma unroll
    for (int j = 0; j < NT; ++j) thf[j] = cok[j] ? (float)thi[j] + corr : __builtin_inff();
#pragma unroll
    for (int i = 0; i < MT; ++i) {
        const long long rbase = m0 + 32 * i;
        if (rbase >= g.rows) break;                              // uniform per wave
        uint32_t wout[NT];
#pragma unroll
        for (int j = 0; j < NT; ++j) {
            wout[j] = 0u;
            const bool cblk = n0 + 32 * j < g.cols;              // uniform: whole blocks (cols is a multiple of 32)
            const long long blk = ((rbase >> 5) * (long long)(e.ldc >> 5) + ((n0 >> 5) + j)) * 1024 + lane * 16;
            float rv[16];
            if (e.resid16 != nullptr) {
                // a lane's 16 values of a 32x32 block are 32 contiguous bytes (sums16_index)
                uint4 lo = make_uint4(0u, 0u, 0u, 0u), hi = lo;
                if (fetched.valid) {                             // MT == NT == 1: read before the main loop
                    lo = fetched.lo; hi = fetched.hi;
                } else if (cblk) {
                    const uint4* src = reinterpret_cast<const uint4*>(e.resid16 + blk);
                    lo = src[0]; hi = src[1];
                }
                const uint32_t w[8] = {lo.x, lo.y, lo.z, lo.w, hi.x, hi.y, hi.z, hi.w};
#pragma unroll
                for (int r = 0; r < 16; ++r)
                    rv[r] = (float)((r & 1) ? ((int)w[r >> 1] >> 16) : (int)(short)(w[r >> 1] & 0xffffu));
            } else if (e.resid_bits != nullptr) {
                // +1/-1 taken from a packed tensor (first residual of a chain): lane t of the lower half reads the
                // (inverted) word of row rbase + t once; rows R and R + 4 then sit in one 64-bit scalar, which each
                // lane shifts so that its column's bit of its own row becomes the sign of 1.0
                const long long rrow = min(rbase + l32, g.rows - 1);
                const int wi = min((n0 >> 5) + j, e.ld_resid_bits_w - 1);
                const uint32_t mine = ~e.resid_bits[rrow * (long long)e.ld_resid_bits_w + wi];
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const int lo_row = 8 * (r >> 2) + (r & 3);
                    const unsigned long long both =
                        ((unsigned long long)(uint32_t)__builtin_amdgcn_readlane((int)mine, lo_row + 4) << 32) |
                        (uint32_t)__builtin_amdgcn_readlane((int)mine, lo_row);
                    const uint32_t top = (uint32_t)((both << (63 - lane)) >> 32);
                    rv[r] = __uint_as_float((top & 0x80000000u) | 0x3f800000u);
                }
            } else {
#pragma unroll
                for (int r = 0; r < 16; ++r) rv[r] = 0.f;
            }
            int vs[16];
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const float sum = acc[i][j][r] + rv[r];
                vs[r] = (int)(sum - corr);
                const unsigned long long ball = __builtin_amdgcn_ballot_w64(sum >= thf[j]);
                const int lo_row = 8 * (r >> 2) + (r & 3);
                wout[j] = write_lane((uint32_t)ball, lo_row, wout[j]);
                wout[j] = write_lane((uint32_t)(ball >> 32), lo_row + 4, wout[j]);
            }
            if (e.out16 != nullptr && cblk) {
                uint32_t pk[8];
#pragma unroll
                for (int q = 0; q < 8; ++q) {
                    const v2s two = __builtin_amdgcn_cvt_pk_i16(vs[2 * q], vs[2 * q + 1]);
                    pk[q] = (uint32_t)(uint16_t)two[0] | ((uint32_t)(uint16_t)two[1] << 16);
                }
                uint4* dst = reinterpret_cast<uint4*>(e.out16 + blk);
                dst[0] = make_uint4(pk[0], pk[1], pk[2], pk[3]);
                dst[1] = make_uint4(pk[4], pk[5], pk[6], pk[7]);
            }
        }
        if (lane < 32) {
            const long long row = rbase + lane;
            if (row < g.rows) {
#pragma unroll
                for (int j = 0; j < NT; ++j) {
                    const int wi = (n0 >> 5) + j;
                    if (wi < e.ldbits_w) e.bits[row * e.ldbits_w + wi] = wout[j];
                }
            }
        }
    }
}

// Which epilogue a call needs (uniform; also evaluated on the host by kernels that are compiled per kind).
enum { EPI_BITS = 0, EPI_CHAIN = 1, EPI_SUMS = 2, EPI_GENERIC = 3 };
__host__ __device__ inline int epilogue_kind(const Epi& e, const bool conv, const bool row_corr) {
    const bool no_resid = e.resid == nullptr && e.resid16 == nullptr && e.resid_bits == nullptr;
    if (e.bits != nullptr && e.out == nullptr && e.out16 == nullptr && no_resid && !row_corr) return EPI_BITS;
    if (conv && e.sums_tiled != 0 && e.bits != nullptr && e.out == nullptr && e.resid == nullptr && !row_corr) return EPI_CHAIN;
    if (e.out != nullptr && e.bits == nullptr && e.out16 == nullptr && no_resid && !row_corr) return EPI_SUMS;
    return EPI_GENERIC;
}

// Threshold of this lane's column in each column tile; INT_MAX (never reached) outside the matrix.
template <int NT>
__device__ __forceinline__ void column_thresholds(int (&thi)[NT], bool (&cok)[NT], const int n0, const int l32, const Geom& g,
                                                  const Epi& e) {
#pragma unroll
    for (int j = 0; j < NT; ++j) {
        const int col = n0 + 32 * j + l32;
        cok[j] = col < g.cols;
        thi[j] = (e.bits != nullptr && cok[j]) ? e.thr[col] : INT_MAX;
    }
}

// Bits only: compare the fp32 accumulators (exact integers) against the threshold shifted by the pad correction;
// one v_cmp per accumulator register gives two packed words.
// PANELS: the packed output is laid out in panels of 8 words (word wi of row `row` at ((wi / 8) * rows + row) * 8 + wi % 8).
template <int MT, int NT, bool PANELS = false>
__device__ __forceinline__ void epilogue_bits(v16f (&acc)[MT][NT], const long long m0, const int n0, const int lane,
                                              const Geom& g, const Epi& e, const int corr_all, const int (&thi)[NT],
                                              const bool (&cok)[NT]) {
    float thf[NT];
#pragma unroll
    for (int j = 0; j < NT; ++j) thf[j] = cok[j] ? (float)thi[j] + (float)corr_all : __builtin_inff();
#pragma unroll
    for (int i = 0; i < MT; ++i) {
        const long long rbase = m0 + 32 * i;
        if (rbase >= g.rows) break;                          // uniform per wave
        uint32_t wout[NT];
#pragma unroll
        for (int j = 0; j < NT; ++j) wout[j] = 0u;
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            const int lo_row = 8 * (r >> 2) + (r & 3);
#pragma unroll
            for (int j = 0; j < NT; ++j) {
                const unsigned long long ball = __builtin_amdgcn_ballot_w64(acc[i][j][r] >= thf[j]);
                wout[j] = write_lane((uint32_t)ball, lo_row, wout[j]);
                wout[j] = write_lane((uint32_t)(ball >> 32), lo_row + 4, wout[j]);
            }
        }
        const long long row = rbase + lane;
        if (lane < 32 && row < g.rows) {
#pragma unroll
            for (int j = 0; j < NT; ++j) {
                const int wi = (n0 >> 5) + j;
                if (wi < e.ldbits_w) e.bits[PANELS ? ((wi >> 3) * g.rows + row) * 8 + (wi & 7) : row * e.ldbits_w + wi] = wout[j];
            }
        }
    }
}

// Sums only (int32, or the same values as fp32): blocks of 32 x 32 that lie inside the matrix are stored without
// per-element tests, from a scalar base per accumulator register (its row) plus one 32-bit offset per lane (its
// column and half) -- no vector address arithmetic; the edge blocks test every element.
template <int MT, int NT>
__device__ __forceinline__ void epilogue_sums(v16f (&acc)[MT][NT], const long long m0, const int n0, const int lane,
                                              const Geom& g, const Epi& e, const int corr_all) {
    const int l32 = lane & 31;
    const int half = lane >> 5;
    const long long m0u = ((long long)__builtin_amdgcn_readfirstlane((int)(m0 >> 32)) << 32) |
                          (uint32_t)__builtin_amdgcn_readfirstlane((int)m0);          // wave-uniform, made scalar
    const int n0u = __builtin_amdgcn_readfirstlane(n0);
    const float corrf = (float)corr_all;
#pragma unroll
    for (int i = 0; i < MT; ++i) {
        const long long rbase = m0u + 32 * i;
        if (rbase >= g.rows) break;
        const bool rows_in = rbase + 32 <= g.rows;
#pragma unroll
        for (int j = 0; j < NT; ++j) {
            const int cbase = n0u + 32 * j;
            const uint32_t lane_off = (uint32_t)((4 * half * e.ldc + l32) * 4);
            if (rows_in && cbase + 32 <= g.cols) {
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    char* row_base = reinterpret_cast<char*>(e.out + (rbase + 8 * (r >> 2) + (r & 3)) * (long long)e.ldc + cbase);
                    const float v = acc[i][j][r] - corrf;            // exact: integers below 2^24
                    *reinterpret_cast<int32_t*>(row_base + (size_t)lane_off) = e.out_f32 ? __float_as_int(v) : (int)v;
                }
            } else {
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const long long row = rbase + 8 * (r >> 2) + 4 * half + (r & 3);
                    const int col = cbase + l32;
                    const float v = acc[i][j][r] - corrf;
                    if (row < g.rows && col < g.cols)
                        e.out[row * (long long)e.ldc + col] = e.out_f32 ? __float_as_int(v) : (int)v;
                }
            }
        }
    }
}

// Epilogue shared by the matrix-core kernels.  acc holds, as exact integers in fp32, the sums
// over every processed bit position; positions beyond the logical width are 0 bits in both
// operands and have contributed (+1)(+1) = +1 each: corr_all of them per output (in exclude mode
// only in-frame taps did: pad_tap per in-frame tap).  Then: optional residual add and int32
// store, threshold compare, and packing through wave ballots.
template <int MT, int NT, bool CONV, bool EXCL>
__device__ __forceinline__ void epilogue(v16f (&acc)[MT][NT], const long long m0, const int n0, const int lane,
                                         const Geom& g, const Epi& e, const int corr_all, const int pad_tap,
                                         const Fetched fetched = Fetched{make_uint4(0u, 0u, 0u, 0u), make_uint4(0u, 0u, 0u, 0u), false}) {
    const bool row_corr = EXCL && CONV && pad_tap != 0;      // correction depends on the pixel
    int thi[NT];
    bool cok[NT];
    column_thresholds<NT>(thi, cok, n0, lane & 31, g, e);
    switch (epilogue_kind(e, CONV, row_corr)) {
        case EPI_BITS: epilogue_bits<MT, NT>(acc, m0, n0, lane, g, e, corr_all, thi, cok); return;
        case EPI_CHAIN: epilogue_chain<MT, NT>(acc, m0, n0, lane, g, e, corr_all, thi, cok, fetched); return;
        case EPI_SUMS: epilogue_sums<MT, NT>(acc, m0, n0, lane, g, e, corr_all); return;
        default: break;
    }
    if (e.resid != nullptr || e.resid16 != nullptr || e.resid_bits != nullptr)
        epilogue_generic<MT, NT, CONV, EXCL, true>(acc, m0, n0, lane, g, e, corr_all, pad_tap, thi, cok, row_corr, fetched);
    else
        epilogue_generic<MT, NT, CONV, EXCL, false>(acc, m0, n0, lane, g, e, corr_all, pad_tap, thi, cok, row_corr, fetched);
}

// The optional second source of a Geom (fused 1x1 downsample shortcut): a handful of K-steps read
// straight from global memory.  Returns the number of bit positions it multiplied.  SWAP: the filters are the MFMA's
// row operand (accumulators hold 16 channels of one pixel per lane instead of one channel of 16 pixels).
template <int MT, int NT, bool SWAP = false>
__device__ __forceinline__ int extra_source(v16f (&acc)[MT][NT], const Geom& g, const long long m0, const int n0,
                                            const int lane, const uint32_t c2) {
    const int l32 = lane & 31;
    const int half = lane >> 5;
    const uint32_t* ar[MT];
    const uint32_t* br[NT];
#pragma unroll
    for (int i = 0; i < MT; ++i) {
        long long row = m0 + 32 * i + l32;
        if (row > g.rows - 1) row = g.rows - 1;
        const int n = fast_div((int)row, g.div_pq);
        const int rem = (int)row - n * (g.P * g.Q);
        const int p = fast_div(rem, g.div_q), q = rem - p * g.Q;
        ar[i] = g.A2 + (((long long)n * g.H2 + p * g.stride2) * g.W2 + q * g.stride2) * g.cw2;
    }
#pragma unroll
    for (int j = 0; j < NT; ++j) br[j] = g.B2 + (long long)min(n0 + 32 * j + l32, g.cols - 1) * g.cw2;
    const int steps = (g.cw2 + 1) / 2;
    for (int ks = 0; ks < steps; ++ks) {
        const int wo = 2 * ks + half;
        const bool ok = wo < g.cw2;
        v8i ea[MT], eb[NT];
#pragma unroll
        for (int i = 0; i < MT; ++i) { const uint32_t w = ar[i][ok ? wo : 0]; ea[i] = expand_fp4(ok ? w : 0u, c2); }
#pragma unroll
        for (int j = 0; j < NT; ++j) { const uint32_t w = br[j][ok ? wo : 0]; eb[j] = expand_fp4(ok ? w : 0u, c2); }
#pragma unroll
        for (int i = 0; i < MT; ++i)
#pragma unroll
            for (int j = 0; j < NT; ++j)
                acc[i][j] = SWAP ? __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(eb[j], ea[i], acc[i][j], 4, 4, 0, 0, 0, 0)
                                 : __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(ea[i], eb[j], acc[i][j], 4, 4, 0, 0, 0, 0);
    }
    return steps * 64;
}

// V: words each lane loads per fragment and chunk (a chunk is 2*V words = V MFMA K-steps);
// CONV: rows are output pixels gathered through the filter window; EXCL: out-of-frame taps
// contribute nothing; GUARD: the last chunk of a tap may run past tw.
// One workgroup tile (bx, by) of the product: everything from the operand loads to the epilogue.
// CPT3 > 0: a 3x3 window whose taps are exactly CPT3 chunks each (tw == CPT3 * 2 * V): the loop over the 9 * CPT3
// chunks is unrolled in full, so that tap and chunk indices are compile-time constants and a request is a handful of
// instructions (the layers of a network are short: their time is instruction issue, not the matrix cores).
template <class TL, int V, bool CONV, bool EXCL, bool GUARD, int CPT3 = 0>
__device__ __forceinline__ void mfma_tile(const uint32_t* __restrict__ A, const uint32_t* __restrict__ B, const Geom& g,
                                          const Epi& e, const int bx, const int by) {
    constexpr int MT = TL::MT, NT = TL::NT;
    const int lane = threadIdx.x & 63;
    const int l32 = lane & 31;
    const int half = lane >> 5;
    const int wave = threadIdx.x >> 6;
    const long long m0 = ((long long)bx * TL::WM + (wave / TL::WN)) * (MT * 32);
    const int n0 = (by * TL::WN + (wave % TL::WN)) * (NT * 32);

    uint32_t c2;
    asm volatile("v_mov_b32 %0, 0x22222222" : "=v"(c2));

    // Addresses are a uniform base (scalar registers) plus a 32-bit byte offset per lane: the base moves with the
    // tap and the chunk, the lane's part is fixed per row, so a request costs no 64-bit vector arithmetic.  The
    // bases belong to the workgroup tile (its first row's image, its first column), which keeps every offset
    // non-negative and below 2^31 (checked on the host: offsets_fit).
    const long long m0_wg = (long long)bx * TL::ROWS;               // < g.rows
    const int n0_wg = min(by * TL::COLS, ((g.cols - 1) >> 5) << 5);
    int n_first = 0;
    if (CONV) n_first = fast_div((int)m0_wg, g.div_pq);
    const uint32_t* Abase = CONV ? A + (long long)n_first * g.H * g.W * g.lda_w : A + m0_wg * g.lda_w;
    const uint32_t* Bbase = B + (long long)n0_wg * g.ldb_w;

    uint32_t aoff[MT];             // bytes from Abase to the row's pixel (y0, x0) (BMM: to the row), plus the half-wave's words
    int y0[MT], x0[MT];
#pragma unroll
    for (int i = 0; i < MT; ++i) {
        long long row = m0 + 32 * i + l32;
        if (row > g.rows - 1) row = g.rows - 1;          // clamp: loads stay in bounds, results are dropped
        if (CONV) {
            const int n = fast_div((int)row, g.div_pq);
            const int rem = (int)row - n * (g.P * g.Q);
            const int p = fast_div(rem, g.div_q), q = rem - p * g.Q;
            y0[i] = p * g.stride - g.pad;
            x0[i] = q * g.stride - g.pad;
            aoff[i] = (uint32_t)(((((n - n_first) * g.H + y0[i]) * g.W + x0[i]) * g.lda_w + half * V) * 4);
        } else {
            y0[i] = 0; x0[i] = 0;
            aoff[i] = (uint32_t)(((int)(row - m0_wg) * g.lda_w + half * V) * 4);
        }
    }
    uint32_t boff[NT];             // bytes from Bbase to the column's row of B, plus the half-wave's words
#pragma unroll
    for (int j = 0; j < NT; ++j) {
        const int col = min(n0 + 32 * j + l32, g.cols - 1);
        // tiled B: rows are grouped by 32; a group stores, for each 16-byte step along K, its 32 rows' 16 bytes
        // back to back, so the 32 lanes of a fragment load read 512 contiguous bytes
        boff[j] = g.b_tiled ? (uint32_t)((((col >> 5) - (n0_wg >> 5)) * g.ldb_w * 32 + (col & 31) * 4 + half * V * 32) * 4)
                            : (uint32_t)(((col - n0_wg) * g.ldb_w + half * V) * 4);
    }
    const int bmul = g.b_tiled ? 32 : 1;                // words between consecutive 4-word groups of a row, / 4

    // One-block wave tiles read their blocked 16-bit residual now, so that its latency passes behind the main
    // loop: these are the layers with short K, where a wave otherwise waits for it after its last MFMA.
    // (requested after the first chunks: the memory counter retires in order, and the residual comes from HBM
    // while the operands mostly come from L2)
    Fetched fetched = {make_uint4(0u, 0u, 0u, 0u), make_uint4(0u, 0u, 0u, 0u), false};
    auto fetch_residual = [&]() {
        if (MT * NT == 1 && e.sums_tiled != 0 && e.resid16 != nullptr) {
            fetched.valid = true;
            if (m0 < g.rows && n0 < g.cols) {
                const uint4* src = reinterpret_cast<const uint4*>(
                    e.resid16 + ((m0 >> 5) * (long long)(e.ldc >> 5) + (n0 >> 5)) * 1024 + lane * 16);
                fetched.lo = src[0]; fetched.hi = src[1];
            }
        }
    };

    v16f acc[MT][NT];
#pragma unroll
    for (int i = 0; i < MT; ++i)
#pragma unroll
        for (int j = 0; j < NT; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

    const int cpt = CPT3 > 0 ? CPT3 : (g.tw + 2 * V - 1) / (2 * V);   // chunks per tap
    const int T = g.taps * cpt;                     // chunks in all

    // Chunks in flight: as many as about 48 registers hold (at least 2, at most 8; the unrolled 3x3 form keeps no
    // masks per chunk and goes up to all of its chunks).  The short-K layers of a network run a handful of chunks
    // per wave, so the wave's time is the memory latency times the number of times it waits: with D chunks
    // requested ahead it waits about T / D times instead of T.
    constexpr int DWANT = 48 / ((MT + NT) * V + ((CONV && CPT3 == 0) ? MT : 0));
    constexpr int DMAX = CPT3 > 0 ? 9 * CPT3 : 8;
    constexpr int D = DWANT < 2 ? 2 : (DWANT > DMAX ? DMAX : DWANT);
    uint32_t ra[D][MT][V], rb[D][NT][V];

    // Multiplies the chunk in buffer `buf`; am[i]: 0 for an out-of-frame tap, bm: 0 for words past the row's end,
    // else all ones.  The masks are applied here, not when the chunk is loaded, so that a request does not have
    // to wait for its own data.
    auto multiply = [&](int buf, const uint32_t (&am)[MT], uint32_t bm) {
#pragma unroll
        for (int v = 0; v < V; ++v) {
            v8i fa[MT], fb[NT];
#pragma unroll
            for (int i = 0; i < MT; ++i) {
                // an out-of-frame tap is 0 bits (-1 padding) or, with excluded padding, fp4 zeros
                uint32_t w = ra[buf][i][v];
                if (CONV) w &= am[i];
                if (GUARD) w &= bm;
                fa[i] = expand_fp4(w, c2);
                if (EXCL) {
                    const int keep = (int)am[i];
                    fa[i][0] &= keep; fa[i][1] &= keep; fa[i][2] &= keep; fa[i][3] &= keep;
                }
            }
#pragma unroll
            for (int j = 0; j < NT; ++j) fb[j] = expand_fp4(GUARD ? (rb[buf][j][v] & bm) : rb[buf][j][v], c2);
#pragma unroll
            for (int i = 0; i < MT; ++i)
#pragma unroll
                for (int j = 0; j < NT; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(
                        fa[i], fb[j], acc[i][j], 4 /*A: E2M1*/, 4 /*B: E2M1*/, 0, 0, 0, 0);
        }
    };

    if constexpr (CPT3 > 0) {
        // bit t of vm[i]: tap t = 3 r + s of row i is in frame
        uint32_t vm[MT];
#pragma unroll
        for (int i = 0; i < MT; ++i) {
            uint32_t cm = 0u;
#pragma unroll
            for (int d = 0; d < 3; ++d) cm |= ((unsigned)(x0[i] + d) < (unsigned)g.W) ? (1u << d) : 0u;
            vm[i] = 0u;
#pragma unroll
            for (int d = 0; d < 3; ++d) vm[i] |= ((unsigned)(y0[i] + d) < (unsigned)g.H) ? (cm << (3 * d)) : 0u;
        }
        const uint32_t safe = (uint32_t)(half * V * 4);      // an out-of-frame tap reads the image's first pixel
        const uint32_t row_bytes = (uint32_t)(g.W * g.lda_w * 4), pix_bytes = (uint32_t)(g.lda_w * 4);
        auto request3 = [&](int buf, int q) {                // q: chunk index, a constant after unrolling
            const int tt = q / CPT3, cc = q % CPT3, r = tt / 3, s = tt % 3;
            const char* abase = reinterpret_cast<const char*>(Abase + cc * 2 * V);
            const uint32_t tapoff = (uint32_t)r * row_bytes + (uint32_t)s * pix_bytes;
#pragma unroll
            for (int i = 0; i < MT; ++i) {
                const uint32_t in = (uint32_t)__builtin_amdgcn_sbfe((int)vm[i], tt, 1);     // all ones or 0
                const uint32_t off = ((aoff[i] + tapoff) & in) | (safe & ~in);
                load_words<V>(reinterpret_cast<const uint32_t*>(abase + (size_t)off), ra[buf][i]);
            }
            const char* bbase = reinterpret_cast<const char*>(Bbase + (tt * g.tw + cc * 2 * V) * bmul);
#pragma unroll
            for (int j = 0; j < NT; ++j)
                load_words<V>(reinterpret_cast<const uint32_t*>(bbase + (size_t)boff[j]), rb[buf][j]);
        };
        constexpr int T3 = 9 * CPT3;
#pragma unroll
        for (int q = 0; q < D; ++q) request3(q, q);
        fetch_residual();
#pragma unroll
        for (int q = 0; q < T3; ++q) {
            uint32_t am[MT];
#pragma unroll
            for (int i = 0; i < MT; ++i) am[i] = (uint32_t)__builtin_amdgcn_sbfe((int)vm[i], q / CPT3, 1);
            multiply(q % D, am, 0xFFFFFFFFu);
            if (q + D < T3) request3(q % D, q + D);
        }
    } else {
        uint32_t amask[D][MT], bmask[D];

        // Loads chunk cc of tap tt into buffer `buf`.
        auto load_chunk = [&](int buf, int tt, int cc) {
            const int wo = cc * 2 * V;                  // first word of the chunk inside the tap (uniform)
            const bool wok = !GUARD || (wo + half * V < g.tw);     // tw is a multiple of V
            // GUARD: the chunk's word offset is added per lane, and lanes past the row's end re-read word 0 of the tap
            const uint32_t lane_wo = !GUARD ? 0u : (wok ? (uint32_t)(wo * 4) : (uint32_t)(-(half * V * 4)));
            int r = 0, s = 0;
            if (CONV) { r = (tt * g.kinv) >> 16; s = tt - r * g.k; }
            const char* abase = reinterpret_cast<const char*>(Abase + (GUARD ? 0 : wo));
            const uint32_t tapoff = CONV ? (uint32_t)((r * g.W + s) * g.lda_w * 4) : 0u;
#pragma unroll
            for (int i = 0; i < MT; ++i) {
                uint32_t off = aoff[i] + tapoff;
                bool ok = true;
                if (CONV) {
                    const int y = y0[i] + r, x = x0[i] + s;
                    ok = (unsigned)y < (unsigned)g.H && (unsigned)x < (unsigned)g.W;
                    off = ok ? off : (uint32_t)(half * V * 4);      // an out-of-frame tap reads the image's first pixel
                }
                load_words<V>(reinterpret_cast<const uint32_t*>(abase + (size_t)(off + lane_wo)), ra[buf][i]);
                amask[buf][i] = ok ? 0xFFFFFFFFu : 0u;
            }
            const char* bbase = reinterpret_cast<const char*>(Bbase + (tt * g.tw + (GUARD ? 0 : wo)) * bmul);
#pragma unroll
            for (int j = 0; j < NT; ++j)
                load_words<V>(reinterpret_cast<const uint32_t*>(bbase + (size_t)(boff[j] + lane_wo * (uint32_t)bmul)),
                              rb[buf][j]);
            bmask[buf] = wok ? 0xFFFFFFFFu : 0u;
        };

        int lt = 0, lc = 0, issued = 0;             // tap, chunk of the tap and index of the next chunk to request
        auto request = [&](int buf) {
            if (issued < T) load_chunk(buf, lt, lc);
            ++issued;
            if (++lc == cpt) { lc = 0; ++lt; }
        };
#pragma unroll
        for (int d = 0; d < D; ++d) request(d);
        fetch_residual();
        for (int t = 0; t < T; t += D) {
            // unrolled by D so that the ring buffer indices are compile-time constants
#pragma unroll
            for (int d = 0; d < D; ++d) {
                if (t + d < T) multiply(d, amask[d], bmask[d]);
                request(d);
            }
        }
    }

    // Every processed bit position beyond the logical width is a 0 bit in both operands.
    const int pad_tap = cpt * 2 * V * 32 - g.bits_tap;
    int corr2 = 0;
    if (CONV && g.A2 != nullptr) corr2 = extra_source<MT, NT>(acc, g, m0, n0, lane, c2) - g.bits2;
    epilogue<MT, NT, CONV, EXCL>(acc, m0, n0, lane, g, e, g.taps * pad_tap + corr2, pad_tap, fetched);
}

template <class TL, int V, bool CONV, bool EXCL, bool GUARD, int CPT3 = 0>
__global__ __launch_bounds__(256, TL::MINB) void mfma_kernel(const uint32_t* __restrict__ A,
                                                             const uint32_t* __restrict__ B, Geom g, Epi e,
                                                             int gx, int gy) {
    int bx, by;
    if (!tile_coords(gx, gy, bx, by)) return;          // uniform for the workgroup
    mfma_tile<TL, V, CONV, EXCL, GUARD, CPT3>(A, B, g, e, bx, by);
}

template <class TL, int V, bool EXCL, int CPT3>
int launch_tile_3x3(const uint32_t* A, const uint32_t* B, const Geom& g, const Epi& e, int gx, int gy, unsigned nwg,
                    hipStream_t s) {
    hipLaunchKernelGGL((mfma_kernel<TL, V, true, EXCL, false, CPT3>), dim3(nwg), dim3(256), 0, s, A, B, g, e, gx, gy);
    return check_launch();
}

template <class TL, int V, bool CONV, bool GUARD>
int launch_tile(const uint32_t* A, const uint32_t* B, const Geom& g, const Epi& e, hipStream_t s) {
    const int col_span = (e.bits != nullptr) ? max(g.cols, e.ldbits_w * 32) : g.cols;
    const int gx = (int)cdiv(g.rows, TL::ROWS), gy = (int)cdiv(col_span, TL::COLS);
    const unsigned nwg = (unsigned)(cdiv((long long)gx * gy, 8) * 8);
    if constexpr (CONV && !GUARD) {
        // 3x3 windows of one or two chunks per tap (C = 64 V, 128 V): the unrolled form
        if (g.k == 3 && g.taps == 9 && (g.tw == 2 * V || (V == 4 && g.tw == 4 * V))) {
            if (g.tw == 2 * V) return g.excl ? launch_tile_3x3<TL, V, true, 1>(A, B, g, e, gx, gy, nwg, s)
                                             : launch_tile_3x3<TL, V, false, 1>(A, B, g, e, gx, gy, nwg, s);
            if constexpr (V == 4)        // (narrower loads are only chosen for tw not a multiple of 8)
                return g.excl ? launch_tile_3x3<TL, V, true, 2>(A, B, g, e, gx, gy, nwg, s)
                              : launch_tile_3x3<TL, V, false, 2>(A, B, g, e, gx, gy, nwg, s);
        }
    }
    if (CONV && g.excl)
        hipLaunchKernelGGL((mfma_kernel<TL, V, CONV, CONV, GUARD>), dim3(nwg), dim3(256), 0, s, A, B, g, e, gx, gy);
    else
        hipLaunchKernelGGL((mfma_kernel<TL, V, CONV, false, GUARD>), dim3(nwg), dim3(256), 0, s, A, B, g, e, gx, gy);
    return check_launch();
}

// Convolutions that the LDS-staged kernel takes (on any tile but the smallest): -1 padding, whole-word pixels of
// 8 bytes or a multiple of 16 bytes, and a long K.  How long was measured in same-run comparisons (VGG and ResNet
// shapes, the 64x64 sweep): pixels of a multiple of 32 bytes feed the direct kernel with 16-byte loads, and it wins
// up to K = 10240 bits (with few slabs it has less fixed cost per workgroup); narrower pixels make it use 8- or
// 4-byte loads, and the staged kernel wins from K = 4096 bits.
inline bool conv_stages_through_lds(const Geom& g) {
    if (!g.conv || g.excl || g.bits_tap != g.tw * 32 || !(g.tw % 4 == 0 || g.tw == 2)) return false;
    return g.taps * g.tw >= (g.tw % 8 == 0 ? 320 : 128);
}

// 0: TileBig, 1: TileTall, 2: TileMid, 3: TileSmall.  The largest tile that still gives the 256
// CUs (two workgroups each for the big tiles) enough workgroups -- unless a matrix product moves full-precision
// sums and K is short: then the call is bound by that traffic (2.5 P MAC/s against 4.5 TB/s: below about 500 bits
// of K per byte moved per output), and the small tile, with four times the resident workgroups, overlaps the waits
// for it with the matrix work of others.  Convolutions never take the small tile for that reason: measured by
// same-run comparison on the ResNet shapes, the big tiles win with row-major int32 sums (wider stores) and with
// the blocked 16-bit sums of a layer chain alike, since a small-tile wave expands one word per operand for every
// MFMA and the big ones a fraction of that.
inline int pick_tile(const Geom& g, const Epi* e = nullptr) {
    if (e != nullptr && !g.conv) {
        const int bytes = 4 * (e->resid != nullptr) + 4 * (e->out != nullptr);
        if (bytes > 0 && (long long)g.taps * g.bits_tap < 500LL * bytes &&
            cdiv(g.rows, TileSmall::ROWS) * cdiv(g.cols, TileSmall::COLS) >= 2048)
            return 3;
    }
    if (g.cols <= 64) return (cdiv(g.rows, TileTall::ROWS) >= 256) ? 1 : 3;
    // the LDS-staged convolution kernel does better on the 128x128 tile until the 256x128 one has about four
    // workgroups per CU slot (measured on the 14x14x256 ResNet layer and the 64x64 sweep); the others from 1.5
    const long long big_min = conv_stages_through_lds(g) ? 2048 : 384;
    if (cdiv(g.rows, TileBig::ROWS) * cdiv(g.cols, TileBig::COLS) >= big_min) return 0;
    if (cdiv(g.rows, TileMid::ROWS) * cdiv(g.cols, TileMid::COLS) >= 256) return 2;
    return 3;
}

// The direct kernel addresses a workgroup tile's operands with 32-bit byte offsets from the tile's first row /
// image and first column: 512 rows of A and 160 rows of B must span less than 2 GiB (leading dimensions below
// 2^20 and 2^21 words), and so must the images that up to 512 consecutive output pixels touch.
inline bool offsets_fit(const Geom& g) {
    if (!g.conv) return g.lda_w < (1 << 20) && g.ldb_w < (1 << 21);
    const long long images = (TileTall::ROWS - 1) / ((long long)g.P * g.Q) + 2;
    return images * g.H * g.W * g.lda_w * 4 < (1LL << 31);
}

template <int V, bool CONV, bool GUARD>
int launch_shape(const uint32_t* A, const uint32_t* B, const Geom& g, const Epi& e, hipStream_t s) {
    switch (pick_tile(g, &e)) {
        case 0: return launch_tile<TileBig, V, CONV, GUARD>(A, B, g, e, s);
        case 1: return launch_tile<TileTall, V, CONV, GUARD>(A, B, g, e, s);
        case 2: return launch_tile<TileMid, V, CONV, GUARD>(A, B, g, e, s);
        default: return launch_tile<TileSmall, V, CONV, GUARD>(A, B, g, e, s);
    }
}

}  // namespace mfma
}  // namespace bnn
#endif
