// Matrix-core path for 3x3 convolutions with pad 1 (stride 1; stride 2 for 64 -> 128 channels) with few channels on
// both sides: the filters stay in LDS as finished E2M1 operands for the whole launch, and every wave keeps the input
// patch of its 64 output pixels there, expanded once for all nine taps.
//
// Why.  The short-K layers of a network (Sec. 6: C = O = 64 or 128) give each accumulator 9 or 18 MFMAs.  In the
// direct kernel a wave expands its own fragments for every tap (7 vector instructions per packed word, each
// activation word 9 times over, plus the tap's address and frame test): 13 to 37 vector instructions per MFMA
// measured on the ResNet-18 layers, the matrix cores 12-26 % busy.  A 3x3 window with stride 1 reads, for
// consecutive output pixels, consecutive input pixels at nine fixed offsets.  So a wave copies the input pixels its
// 64 outputs touch into LDS once (global -> registers -> expand -> two 16-byte LDS writes per word) and then reads
// every tap's fragment with one ds_read_b128 at a constant offset from a per-lane base: no vector arithmetic in the
// K loop at all.
//
// Halo-sharing coordinates.  Padding must not cost tests in the K loop either, so the patch lives in padded
// coordinates: input pixel (n, y, x) sits at  PL = (n (H+1) + y + 1)(W+1) + x + 1.  Column 0 of every padded row
// and row 0 of every padded image hold the padding value, and because the row pitch is W+1 (not W+2) the cell right
// of a row's last pixel IS the next row's column 0, the row below an image's last row IS the next image's row 0.
// Tap (r, s) of the output pixel at PL reads PL + (r-1)(W+1) + (s-1).  64 consecutive output pixels span
// 63 + (row crossings) + (W+1)(image crossings) cells, plus one padded row and one cell on either side.
//
// A patch is private to its wave (two planes of 16-byte units, one per half of a 64-channel slab, so that a
// fragment read is 32 consecutive units per half-wave: conflict-free): no barrier after the filters are in place,
// waves drift apart, and one wave's epilogue overlaps another's MFMAs.  The words of the next tile are requested
// before the current tile's last K-steps, so global latency is not waited for either.
#include "bnn_mfma_kernel.h"

namespace bnn {
namespace {

using mfma::v16f;
using mfma::v8i;

constexpr int MT = 2;            // a wave tile is 64 output pixels x all output channels
// patch positions per lane whose words are requested one tile ahead (a stride-2 tile spans twice the cells)
constexpr int pre_positions(int stride) { return stride == 2 ? 8 : 4; }

struct PatchArgs {
    int wp1, hp1;                // W + 1, H + 1
    int magic_wp1, magic_hp1, magic_q, magic_p;      // ceil(2^20 / d) for d = W + 1, H + 1, Q, P
    int images;                  // N
    int plane;                   // 16-byte units per plane of a wave's patch: 64 * pp
    int pp;                      // patch positions per lane
    int ntiles;                  // wave tiles
    uint32_t pad_keep;           // -1 padding: all ones (a padding cell is the expansion of 0 bits); excluded padding: 0 (fp4 zeros)
};

__device__ __forceinline__ uint4 expand_unit(uint32_t w, uint32_t c2) {
    return make_uint4(((w << 3) & 0x88888888u) | c2, ((w << 2) & 0x88888888u) | c2, ((w << 1) & 0x88888888u) | c2,
                      (w & 0x88888888u) | c2);
}

__device__ __forceinline__ v8i as_operand(const uint4& u) {
    v8i r;
    r[0] = (int)u.x; r[1] = (int)u.y; r[2] = (int)u.z; r[3] = (int)u.w;
    r[4] = 0; r[5] = 0; r[6] = 0; r[7] = 0;         // the upper half is not read for 4-bit formats
    return r;
}

// 16 sign bits of a lane's registers (bit r = register r = channel 8a + 4 half + b, r = 4a + b) -> that lane pair's
// packed word of 32 channels with a 1 where the value is NOT negative; both half-waves end up with the whole word.
__device__ __forceinline__ uint32_t word_from_signs(uint32_t m, int half) {
    m = (m | (m << 8)) & 0x00FF00FFu;                // nibble a -> byte a
    m = (m | (m << 4)) & 0x0F0F0F0Fu;
    m <<= 4 * half;                                  // this half-wave's channels of each byte
    const auto both = __builtin_amdgcn_permlane32_swap(m, m, false, false);      // meet the other half-wave
    return ~(both[0] | both[1]);
}

// Epilogue of a residual layer inside a layer chain with swapped operand roles: a lane holds 16 channels of one pixel,
// accumulators started at 0.5 - threshold (`start`: LDS, [column tile][half-wave][register]).  Blocked 16-bit sums in
// and / or out (a lane's 16 values are 32 contiguous bytes of the block, in this kernel's own order), or the +1/-1 of
// packed bits as the residual: each lane reads the word of its own pixel, and a register's channel is a compile-time
// bit position once the word is shifted by the half-wave's 4.  corr: what the second source added beyond its logical
// width.  fp32 throughout: half-integers below 2^23, exact.
template <int MT>
__device__ __forceinline__ void epilogue_chain_swapped(v16f (&acc)[MT][2], const long long m0, const int n0, const int lane,
                                                       const Geom& g, const Epi& e, const float* start, const int corr) {
    const int l32 = lane & 31, half = lane >> 5;
#pragma unroll
    for (int i = 0; i < MT; ++i) {
        const long long rbase = m0 + 32 * i;
        if (rbase >= g.rows) break;                              // uniform per wave
        uint32_t wout[2];
#pragma unroll
        for (int j = 0; j < 2; ++j) {
            const bool cblk = n0 + 32 * j < g.cols;              // uniform: whole blocks (cols is a multiple of 32)
            const long long blk = ((rbase >> 5) * (long long)(e.ldc >> 5) + ((n0 >> 5) + j)) * 1024 + lane * 16;
            float rv[16];
            if (e.resid16 != nullptr) {
                uint4 lo = make_uint4(0u, 0u, 0u, 0u), hi = lo;
                if (cblk) {
                    const uint4* src = reinterpret_cast<const uint4*>(e.resid16 + blk);
                    lo = src[0]; hi = src[1];
                }
                const uint32_t w[8] = {lo.x, lo.y, lo.z, lo.w, hi.x, hi.y, hi.z, hi.w};
#pragma unroll
                for (int r = 0; r < 16; ++r)
                    rv[r] = (float)((r & 1) ? ((int)w[r >> 1] >> 16) : (int)(short)(w[r >> 1] & 0xffffu));
            } else if (e.resid_bits != nullptr) {
                const long long rrow = min(rbase + l32, g.rows - 1);
                const int wi = min((n0 >> 5) + j, e.ld_resid_bits_w - 1);
                const uint32_t y = ~e.resid_bits[rrow * (long long)e.ld_resid_bits_w + wi] >> (4 * half);
#pragma unroll
                for (int r = 0; r < 16; ++r) {                   // bit 1 -> +1.0, bit 0 -> -1.0
                    const int c = 8 * (r >> 2) + (r & 3);
                    rv[r] = __uint_as_float(((y << (31 - c)) & 0x80000000u) | 0x3f800000u);
                }
            } else {
#pragma unroll
                for (int r = 0; r < 16; ++r) rv[r] = 0.f;
            }
            if (corr != 0) {                                     // uniform: bit positions past the second source's width
                const float corrf = (float)corr;
#pragma unroll
                for (int r = 0; r < 16; ++r) rv[r] -= corrf;
            }
            const float4* sv = reinterpret_cast<const float4*>(start + ((((n0 >> 5) + j) * 2 + half) * 16));
            float st[16];
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const float4 v = sv[q];
                st[4 * q] = v.x; st[4 * q + 1] = v.y; st[4 * q + 2] = v.z; st[4 * q + 3] = v.w;
            }
            uint32_t m = 0u;
            int vs[16];
#pragma unroll
            for (int r = 15; r >= 0; --r) {
                const float sum = acc[i][j][r] + rv[r];
                m = __builtin_amdgcn_alignbit(m, __float_as_uint(sum), 31);
                vs[r] = (int)(sum - st[r]);                      // the integer sum itself
            }
            if (e.out16 != nullptr && cblk) {
                uint32_t pk[8];
#pragma unroll
                for (int q = 0; q < 8; ++q) {
                    const mfma::v2s two = __builtin_amdgcn_cvt_pk_i16(vs[2 * q], vs[2 * q + 1]);
                    pk[q] = (uint32_t)(uint16_t)two[0] | ((uint32_t)(uint16_t)two[1] << 16);
                }
                uint4* dst = reinterpret_cast<uint4*>(e.out16 + blk);
                dst[0] = make_uint4(pk[0], pk[1], pk[2], pk[3]);
                dst[1] = make_uint4(pk[4], pk[5], pk[6], pk[7]);
            }
            wout[j] = word_from_signs(m, half);
        }
        const long long row = rbase + lane;
        if (lane < 32 && row < g.rows) {
#pragma unroll
            for (int j = 0; j < 2; ++j) {
                const int wi = (n0 >> 5) + j;
                if (wi < e.ldbits_w) e.bits[row * e.ldbits_w + wi] = wout[j];
            }
        }
    }
}

// NT: 32-column accumulator tiles per wave (all output channels); CW: packed words per pixel (C / 32); KIND: the
// epilogue the call needs (mfma::epilogue_kind), compiled in alone to keep the register count of the tile loop low.
// S: stride (1 or 2).  With stride 2 the output pixel (p, q) is centred on the input pixel (2p, 2q): the same padded
// coordinates, a lane's base twice as far from the tile's first pixel, the same nine offsets.
template <int NT, int CW, int WAVES, int KIND, int S = 1>
__global__ __launch_bounds__(64 * WAVES, 1) void conv_patch_kernel(const uint32_t* __restrict__ A,
                                                                   const uint32_t* __restrict__ B, Geom g, Epi e,
                                                                   PatchArgs pa) {
    extern __shared__ uint4 lds[];
    constexpr int COLSP = NT * 32;
    constexpr int CG = CW / 2;                       // 64-channel slabs
    constexpr int PRE = pre_positions(S);

    const int tid = threadIdx.x, lane = tid & 63, l32 = lane & 31, half = lane >> 5;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    uint32_t c2;
    asm volatile("v_mov_b32 %0, 0x22222222" : "=v"(c2));

    uint4* const filt = lds;                                         // [tap][word][column]
    uint4* const patch = lds + 9 * CW * COLSP + wave * 2 * pa.plane; // [half of the slab][cell]
    // bits kind: start values of the accumulators, [column tile][half-wave][register] (see SWAPPED below)
    // (eight copies, one unit more than a copy apart: the eight lanes LDS serves together read eight different units --
    // sixteen lanes reading ONE 16-byte unit are not a broadcast but a conflict)
    constexpr int START_PITCH = NT * 2 * 16 + 4;
    float* const start_all = reinterpret_cast<float*>(lds + 9 * CW * COLSP + WAVES * 2 * pa.plane);
    const float* const start = start_all + (l32 & 7) * START_PITCH;
    const char* const Ab = reinterpret_cast<const char*>(A);

    // A tile's first output pixel (wave-uniform; scalar arithmetic).  Everything a lane needs is then a small
    // offset from it, and small numbers divide with one 24-bit multiply (full rate; 32-bit multiplies are not):
    // x / d == (x * ceil(2^20 / d)) >> 20 whenever x * d <= 2^20, which the host checks for every use below.
    struct First { int n, p, q; };
    auto first_pixel = [&](int T) {
        const int m0 = 64 * T;
        First f;
        f.n = fast_div(m0, g.div_pq);
        const int rem = m0 - f.n * (g.P * g.Q);
        f.p = fast_div(rem, g.div_q);
        f.q = rem - f.p * g.Q;
        return f;
    };
    auto small_div = [](int x, int magic) { return (int)(__umul24((uint32_t)x, (uint32_t)magic) >> 20); };
    // byte offset of the input pixel at the patch's cell j (0 and in = false for a padding cell).  The patch starts
    // one padded row and one cell before the first pixel's centre: at padded row S f.p of image f.n, column S f.q.
    auto locate = [&](const First& f, int j, bool& in) {
        const int x = S * f.q + j;
        const int drow = small_div(x, pa.magic_wp1), xp = x - __mul24(drow, pa.wp1);
        const int yl = S * f.p + drow;
        const int dimg = small_div(yl, pa.magic_hp1), yp = yl - __mul24(dimg, pa.hp1);
        const int n = f.n + dimg;
        in = xp > 0 && yp > 0 && n < pa.images;
        const int pix = __mul24(__mul24(n, g.H) + yp - 1, g.W) + xp - 1;
        return in ? (uint32_t)pix * (uint32_t)(CW * 4) : 0u;
    };

    uint32_t pre[PRE][CW];
    uint32_t pre_in = 0u;                            // bit pp: position pp is an input pixel
    auto request = [&](int T) {
        const First f = first_pixel(T);
        pre_in = 0u;
#pragma unroll
        for (int pp = 0; pp < PRE; ++pp) {
            if (pp < pa.pp) {                        // uniform
                bool in;
                const uint32_t off = locate(f, lane + 64 * pp, in);
                mfma::load_words<CW>(reinterpret_cast<const uint32_t*>(Ab + (size_t)off), pre[pp]);
                pre_in |= in ? (1u << pp) : 0u;
            }
        }
    };
    // expands two words of a cell into the wave's patch; keep: all ones for an input pixel, 0 for a padding cell,
    // which becomes the expansion of 0 bits (-1 padding) or fp4 zeros (excluded padding: nothing is added)
    auto put = [&](int cell_rel, uint32_t w0, uint32_t w1, uint32_t keep) {
        const uint32_t c2v = c2 & (keep | pa.pad_keep);
        patch[cell_rel] = expand_unit(w0 & keep, c2v);
        patch[pa.plane + cell_rel] = expand_unit(w1 & keep, c2v);
    };
    auto stage = [&](const First& f, int cg) {
#pragma unroll
        for (int pp = 0; pp < PRE; ++pp) {
            if (pp < pa.pp) {
                const uint32_t keep = (uint32_t)__builtin_amdgcn_sbfe((int)pre_in, pp, 1);
                put(lane + 64 * pp, pre[pp][2 * cg], pre[pp][2 * cg + 1], keep);
            }
        }
        for (int pp = PRE; pp < pa.pp; ++pp) {       // wide images: the rest of the patch, read now
            bool in;
            const uint32_t off = locate(f, lane + 64 * pp, in);
            const uint2 w = *reinterpret_cast<const uint2*>(Ab + (size_t)off + 8 * cg);
            put(lane + 64 * pp, w.x, w.y, in ? 0xFFFFFFFFu : 0u);
        }
    };

    // Tile order.  In a full round every wave of the launch takes one tile, neighbouring tiles (whose patches
    // overlap) on the waves of one workgroup.  The tiles left for the last, partial round are dealt across the
    // workgroups first, so that every compute unit gets its share of them instead of some running a full extra
    // round while the others idle.
    const int per_round = (int)gridDim.x * WAVES;
    const int full_rounds = pa.ntiles / per_round;
    const int my_turns = full_rounds + ((full_rounds * per_round + wave * (int)gridDim.x + (int)blockIdx.x) < pa.ntiles ? 1 : 0);
    auto tile_of = [&](int turn) {
        return turn < full_rounds ? turn * per_round + (int)blockIdx.x * WAVES + wave
                                  : full_rounds * per_round + wave * (int)gridDim.x + (int)blockIdx.x;
    };
    if (my_turns > 0) request(tile_of(0));

    // The filters: every packed word expanded once per workgroup, [tap][word][column] so that a fragment read is
    // 32 consecutive units per half-wave.  A thread takes (tap, column) items, consecutive lanes consecutive columns:
    // their 16-byte LDS writes then fall on consecutive units (with consecutive taps of one column per lane they were
    // a whole plane apart, all eight lanes LDS serves together on the same banks: 4500 conflict cycles per compute
    // unit, 2 us, for 128 -> 128 channels).  One 8- or 16-byte load per item, all of them requested before the first
    // is expanded (every workgroup of the launch reads these same few KB at the same moment; loads waited for one by
    // one made this prologue longer than the tiles of a small layer).
    {
        constexpr int ITEMS = 9 * COLSP, PER = (ITEMS + 64 * WAVES - 1) / (64 * WAVES);
        uint32_t fw[PER][CW];
#pragma unroll
        for (int it = 0; it < PER; ++it) {
            const int item = tid + it * 64 * WAVES, tap = item / COLSP, col = item - COLSP * tap;
            const bool ok = item < ITEMS && col < g.cols;
            mfma::load_words<CW>(B + (ok ? (long long)col * g.ldb_w + tap * CW : 0), fw[it]);
        }
#pragma unroll
        for (int it = 0; it < PER; ++it) {
            const int item = tid + it * 64 * WAVES, tap = item / COLSP, col = item - COLSP * tap;
            if (item < ITEMS) {
                const uint32_t keep = col < g.cols ? 0xFFFFFFFFu : 0u;      // columns past the last: 0 bits
#pragma unroll
                for (int w = 0; w < CW; ++w) filt[(tap * CW + w) * COLSP + col] = expand_unit(fw[it][w] & keep, c2);
            }
        }
    }
    // Bits kind: the operand roles are swapped (filters as the MFMA's row operand), so that a lane ends up with 16
    // output channels of ONE pixel and can pack its own bits: every accumulator starts at 0.5 - threshold of its
    // channel (exact: thresholds are clamped to +-2^20, beyond every reachable sum, and partial sums stay half-integers
    // below 2^23), the output bit is then "not the sign bit", and 16 v_alignbit collect a lane's 16 signs -- against
    // a compare, a wait state and two lane writes per register when a lane holds one channel of 16 pixels.  Channels
    // past the last start at -infinity: their bits stay 0.
    constexpr bool SWAPPED = KIND != mfma::EPI_SUMS;
    if (SWAPPED && tid < COLSP) {
        const int col = tid, jt = col >> 5, c = col & 31;
        const int reg = 4 * (c >> 3) + (c & 3), hf = (c >> 2) & 1;     // channel 8a + 4 hf + b of a tile: register 4a + b
        float v = -__builtin_inff();
        if (col < g.cols) {
            const int lim = 1 << 20;                 // beyond every reachable sum (K <= 1152 here, residual sums are 16-bit)
            v = 0.5f - (float)max(-lim, min(lim, e.thr[col]));
        }
#pragma unroll
        for (int cp = 0; cp < 8; ++cp) start_all[cp * START_PITCH + (jt * 2 + hf) * 16 + reg] = v;
    }
    __syncthreads();

    // this lane's thresholds, read once for all tiles (a load inside the tile loop would make every epilogue start
    // with a full wait on global memory, the next tile's words included)
    int thi[NT / 2][2];
    bool cok[NT / 2][2];
#pragma unroll
    for (int h = 0; h < NT / 2; ++h) mfma::column_thresholds<2>(thi[h], cok[h], 64 * h, l32, g, e);

    for (int turn = 0; turn < my_turns; ++turn) {
        const int T = tile_of(turn);
        const long long m0 = 64LL * T;
        const First f = first_pixel(T);
        const int last_rel = (int)min(63LL, g.rows - 1 - m0);            // clamp: results past the last row are dropped
        int abase[MT];                               // unit of tap (0, 0) of this lane's pixel, in its half's plane
#pragma unroll
        for (int i = 0; i < MT; ++i) {
            const int lq = f.q + min(32 * i + l32, last_rel);
            const int dp = small_div(lq, pa.magic_q), q = lq - __mul24(dp, g.Q);
            const int lp = f.p + dp;
            const int dn = small_div(lp, pa.magic_p), p = lp - __mul24(dn, g.P);
            // cells between this pixel and the tile's first: whole padded rows, then columns
            abase[i] = half * pa.plane + __mul24(__mul24(dn, pa.hp1) + S * (p - f.p), pa.wp1) + S * (q - f.q);
        }

        v16f acc[NT / 2][MT][2];                     // [64-column half][row tile][column tile]: the epilogue runs per half
#pragma unroll
        for (int h = 0; h < NT / 2; ++h)
#pragma unroll
            for (int i = 0; i < MT; ++i)
#pragma unroll
                for (int j = 0; j < 2; ++j) {
                    if constexpr (SWAPPED) {         // 0.5 - threshold of the register's channel, straight from LDS
                        const float4* sv = reinterpret_cast<const float4*>(start + ((2 * h + j) * 2 + half) * 16);
#pragma unroll
                        for (int q = 0; q < 4; ++q) {
                            const float4 v = sv[q];
                            acc[h][i][j][4 * q] = v.x; acc[h][i][j][4 * q + 1] = v.y;
                            acc[h][i][j][4 * q + 2] = v.z; acc[h][i][j][4 * q + 3] = v.w;
                        }
                    } else {
#pragma unroll
                        for (int r = 0; r < 16; ++r) acc[h][i][j][r] = 0.f;
                    }
                }

        // K loop: nine taps per 64-channel slab.  The fragments of tap t + 1 are requested before the MFMAs of tap
        // t (two register sets), and the scheduler is told to spread those reads between the MFMAs, so that the
        // matrix pipe does not wait for LDS between taps (a wave is often alone in its K loop: its SIMD mates are
        // in their epilogues).
        uint4 fa[2][MT], fb[2][NT];
        auto read_tap = [&](int cg, int t, int slot) {
            const int r = t / 3, s3 = t % 3;
#pragma unroll
            for (int i = 0; i < MT; ++i) fa[slot][i] = patch[abase[i] + r * pa.wp1 + s3];
#pragma unroll
            for (int j = 0; j < NT; ++j) fb[slot][j] = filt[((t * CW) + 2 * cg) * COLSP + half * COLSP + 32 * j + l32];
        };
#pragma unroll
        for (int cg = 0; cg < CG; ++cg) {
            stage(f, cg);
            if (cg == CG - 1 && turn + 1 < my_turns) request(tile_of(turn + 1));
            read_tap(cg, 0, 0);
#pragma unroll
            for (int t = 0; t < 9; ++t) {
                if (t + 1 < 9) read_tap(cg, t + 1, (t + 1) & 1);
#pragma unroll
                for (int i = 0; i < MT; ++i)
#pragma unroll
                    for (int j = 0; j < NT; ++j)
                        acc[j / 2][i][j % 2] = SWAPPED
                            ? __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(as_operand(fb[t & 1][j]), as_operand(fa[t & 1][i]),
                                                                             acc[j / 2][i][j % 2], 4, 4, 0, 0, 0, 0)
                            : __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(as_operand(fa[t & 1][i]), as_operand(fb[t & 1][j]),
                                                                             acc[j / 2][i][j % 2], 4 /*A: E2M1*/, 4 /*B: E2M1*/, 0, 0, 0, 0);
                if (t + 1 < 9) {
#pragma unroll
                    for (int q = 0; q < MT * NT; ++q) {
                        __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);                       // one MFMA
                        if (q < MT + NT) __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);      // one LDS read
                    }
                }
                __builtin_amdgcn_sched_barrier(0);
            }
        }

#pragma unroll
        for (int h = 0; h < NT / 2; ++h) {
            int corr2 = 0;                           // no bit position beyond the logical width was multiplied here
            if (g.A2 != nullptr) corr2 = mfma::extra_source<MT, 2, SWAPPED>(acc[h], g, m0, 64 * h, lane, c2) - g.bits2;
            if constexpr (KIND == mfma::EPI_BITS) {
                // lane (pixel l32, half): register r = 4a + b holds channel 8a + 4 half + b of column tile 2h + j
#pragma unroll
                for (int i = 0; i < MT; ++i) {
                    uint32_t wout[2];
#pragma unroll
                    for (int j = 0; j < 2; ++j) {
                        uint32_t m = 0u;             // bit r: sign of register r
#pragma unroll
                        for (int r = 15; r >= 0; --r) m = __builtin_amdgcn_alignbit(m, __float_as_uint(acc[h][i][j][r]), 31);
                        wout[j] = word_from_signs(m, half);
                    }
                    const long long row = m0 + 32 * i + lane;
                    if (lane < 32 && row < g.rows) {
#pragma unroll
                        for (int j = 0; j < 2; ++j)
                            if (2 * h + j < e.ldbits_w) e.bits[row * e.ldbits_w + 2 * h + j] = wout[j];
                    }
                }
            } else if constexpr (KIND == mfma::EPI_CHAIN) {
                if (e.resid16 == nullptr && e.resid_bits != nullptr) {
                    // A first residual taken from packed bits (+1 / -1 per pixel and channel) goes through the matrix
                    // pipe: one more K-step whose "filter" is the identity -- -1.0 where the K slot is the column's own
                    // channel (a 1 bit expands to -1.0, so the product is +1), 0.0 elsewhere -- against the expanded word
                    // of the pixel.  Two MFMAs per row tile instead of three vector instructions per accumulator register.
                    v8i ident[2], px[MT];
#pragma unroll
                    for (int j = 0; j < 2; ++j) {
                        const uint4 u = expand_unit(j == half ? 1u << l32 : 0u, 0u);       // 0x8 in the one nibble of bit l32
                        ident[j] = as_operand(make_uint4(u.x | (u.x >> 2), u.y | (u.y >> 2), u.z | (u.z >> 2), u.w | (u.w >> 2)));
                    }
#pragma unroll
                    for (int i = 0; i < MT; ++i) {
                        const long long rrow = min(m0 + 32 * i + l32, g.rows - 1);
                        const int wi = min(2 * h + half, e.ld_resid_bits_w - 1);
                        px[i] = mfma::expand_fp4(e.resid_bits[rrow * (long long)e.ld_resid_bits_w + wi], c2);
                    }
#pragma unroll
                    for (int i = 0; i < MT; ++i)
#pragma unroll
                        for (int j = 0; j < 2; ++j)
                            acc[h][i][j] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(ident[j], px[i], acc[h][i][j], 4, 4, 0, 0, 0, 0);
                    Epi e2 = e;
                    e2.resid_bits = nullptr;
                    epilogue_chain_swapped<MT>(acc[h], m0, 64 * h, lane, g, e2, start, corr2);
                } else
                    epilogue_chain_swapped<MT>(acc[h], m0, 64 * h, lane, g, e, start, corr2);
            } else
                mfma::epilogue_sums<MT, 2>(acc[h], m0, 64 * h, lane, g, e, corr2);
        }
    }
}

// Waves per workgroup: what the registers allow (three per SIMD with 64-column tiles, two with 128-column tiles).
constexpr int waves_for(int nt, int kind) { (void)kind; return nt == 2 ? 12 : 8; }
// stride 2, 64 -> 128 channels: a patch is twice as long, seven of them fit beside the filters
constexpr int WAVES_STRIDE2 = 7;

struct PatchPlan {
    bool ok;
    int nt, cw, waves, kind;
    PatchArgs pa;
    size_t lds_bytes;
};

PatchPlan plan_patch(const Geom& g, const Epi& e) {
    PatchPlan pl = {};
    if (!g.conv || g.b_tiled || g.k != 3 || (g.stride != 1 && g.stride != 2) || g.pad != 1 || g.taps != 9) return pl;
    if ((g.tw != 2 && g.tw != 4) || g.bits_tap != g.tw * 32 || g.lda_w != g.tw) return pl;
    const int S = g.stride;
    if (g.cols > 128 || g.P != (g.H - 1) / S + 1 || g.Q != (g.W - 1) / S + 1) return pl;
    pl.kind = mfma::epilogue_kind(e, true, false);
    if (pl.kind == mfma::EPI_GENERIC) return pl;                     // (row-major residuals: the direct kernels)
    if (pl.kind == mfma::EPI_BITS && g.A2 != nullptr) return pl;     // (the bits-only form has no second source)
    pl.nt = g.cols <= 64 ? 2 : 4;
    pl.cw = g.tw;
    // stride 2: built for 64 -> 128 channels, bits out (the first convolution of a block that halves the image)
    if (S == 2 && (pl.nt != 4 || pl.cw != 2 || pl.kind != mfma::EPI_BITS)) return pl;
    pl.waves = S == 2 ? WAVES_STRIDE2 : waves_for(pl.nt, pl.kind);
    if (e.bits != nullptr && e.ldbits_w > pl.nt) return pl;          // words beyond the tile would stay unwritten
    const long long images = g.rows / ((long long)g.P * g.Q);
    // Cells a tile of 64 consecutive output pixels can span.  From one output pixel to the next the centre moves S cells;
    // a row change adds S (W + 1 - Q) cells to that, an image change the padded rows between the last window row of one
    // image and the first of the next; then two padded rows and three cells for the last pixel's window.
    const int row_x = 63 / g.Q + 1, img_x = 63 / (g.P * g.Q) + 1;
    const int row_extra = S * (g.W + 1 - g.Q);
    const int img_extra = max(0, (g.H + 1 - S * (g.P - 1)) * (g.W + 1) - S * g.Q - row_extra);
    const int cells = 63 * S + row_x * row_extra + img_x * img_extra + 2 * (g.W + 1) + 3;
    const int pp = (cells + 63) / 64;
    if (pp > 16) return pl;
    if ((images * (g.H + 1) + 2) * (g.W + 1) + 64LL * pp >= (1LL << 31)) return pl;          // cell numbers fit an int
    if (images * g.H * g.W * g.tw * 4 >= (1LL << 32)) return pl;                              // 32-bit byte offsets
    pl.lds_bytes = ((size_t)9 * pl.cw * pl.nt * 32 + (size_t)pl.waves * 2 * 64 * pp) * 16 + (size_t)8 * (pl.nt * 2 * 16 + 4) * 4;
    if (pl.lds_bytes > 160 * 1024) return pl;
    const long long ntiles = cdiv(g.rows, 64);
    // Measured against the direct kernels on 56x56x64->64, 28x28 / 64x64x128->128 and 56x56x64->128 (stride 2) layers
    // over batch sizes (GPU time per call, microseconds, patch / direct): 64 columns 3.9 / 3.6 at 196 tiles, 3.9 / 4.5 at
    // 392, 4.0 / 5.9 at 784; 128 columns 6.8 / 7.5 at 784, 7.7 / 7.6 at 1024, 9.3 / 11.2 at 1568; stride 2 5.3 / 4.6 at
    // 196, 5.5 / 6.2 at 392, 5.7 / 7.6 at 784.
    if (ntiles < (pl.nt == 2 || S == 2 ? 384 : 768)) return pl;
    pl.pa.wp1 = g.W + 1; pl.pa.hp1 = g.H + 1;
    // the small divisions of the kernel (x / d with one 24-bit multiply) are exact for x * d <= 2^20
    const long long lim = 1LL << 20;
    if ((S * g.Q + 64LL * pp) * (g.W + 1) > lim || (S * g.P + 64LL * pp / (g.W + 1) + 2) * (g.H + 1) > lim) return pl;
    if ((g.Q + 63LL) * g.Q > lim || (g.P + 63LL / g.Q + 2) * g.P > lim || images * g.H >= (1LL << 24)) return pl;
    auto magic = [](int d) { return (int)(((1LL << 20) + d - 1) / d); };
    pl.pa.magic_wp1 = magic(g.W + 1); pl.pa.magic_hp1 = magic(g.H + 1);
    pl.pa.magic_q = magic(g.Q); pl.pa.magic_p = magic(g.P);
    pl.pa.images = (int)images;
    pl.pa.plane = 64 * pp; pl.pa.pp = pp;
    pl.pa.ntiles = (int)ntiles;
    pl.pa.pad_keep = g.excl ? 0u : 0xFFFFFFFFu;
    pl.ok = true;
    return pl;
}

template <int NT, int CW, int WAVES, int KIND, int S = 1>
int launch_patch_kind(const uint32_t* A, const uint32_t* B, const Geom& g, const Epi& e, const PatchPlan& pl, hipStream_t s) {
    static const hipError_t attr = hipFuncSetAttribute(reinterpret_cast<const void*>(&conv_patch_kernel<NT, CW, WAVES, KIND, S>),
                                                       hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
    if (attr != hipSuccess) return BNN_ERR_DEVICE;
    const unsigned nwg = (unsigned)min(256, pl.pa.ntiles);   // one workgroup per compute unit; few tiles: spread over all of them
    hipLaunchKernelGGL((conv_patch_kernel<NT, CW, WAVES, KIND, S>), dim3(nwg), dim3(64 * WAVES), pl.lds_bytes, s, A, B, g, e, pl.pa);
    return check_launch();
}

template <int NT, int CW>
int launch_patch(const uint32_t* A, const uint32_t* B, const Geom& g, const Epi& e, const PatchPlan& pl, hipStream_t s) {
    switch (pl.kind) {
        case mfma::EPI_BITS:
            return launch_patch_kind<NT, CW, waves_for(NT, mfma::EPI_BITS), mfma::EPI_BITS>(A, B, g, e, pl, s);
        case mfma::EPI_CHAIN:
            return launch_patch_kind<NT, CW, waves_for(NT, mfma::EPI_CHAIN), mfma::EPI_CHAIN>(A, B, g, e, pl, s);
        default:
            return launch_patch_kind<NT, CW, waves_for(NT, mfma::EPI_SUMS), mfma::EPI_SUMS>(A, B, g, e, pl, s);
    }
}

}  // namespace

bool mfma_conv_patch_takes(const Geom& g, const Epi& e) { return plan_patch(g, e).ok; }

const char* describe_mfma_conv_patch(const Geom& g) {
    if (g.stride == 2) return "mfma_fp4_conv3x3s2_patch_wave64x128";
    return g.cols <= 64 ? "mfma_fp4_conv3x3_patch_wave64x64" : "mfma_fp4_conv3x3_patch_wave64x128";
}

int launch_mfma_conv_patch(const uint32_t* A, const uint32_t* B, const Geom& g, const Epi& e, hipStream_t s) {
    const PatchPlan pl = plan_patch(g, e);
    if (!pl.ok) return BNN_ERR_UNSUPPORTED;
    if (g.stride == 2) return launch_patch_kind<4, 2, WAVES_STRIDE2, mfma::EPI_BITS, 2>(A, B, g, e, pl, s);
    if (pl.nt == 2) return pl.cw == 2 ? launch_patch<2, 2>(A, B, g, e, pl, s) : launch_patch<2, 4>(A, B, g, e, pl, s);
    return pl.cw == 2 ? launch_patch<4, 2>(A, B, g, e, pl, s) : launch_patch<4, 4>(A, B, g, e, pl, s);
}

}  // namespace bnn
