// Matrix-core path for large matrix products: the row operand is expanded to E2M1 ONCE per workgroup, on its way
// into LDS, and the waves read finished MFMA operands; the column operand travels through LDS packed and every wave
// expands its own two column fragments a K-step ahead.
//
// Why.  In the LDS-staged kernel of bnn_mfma_staged.h every wave expands the packed words of its own fragments:
// 42 vector-ALU instructions for the 8 MFMAs of a K-step, each MFMA waiting on registers a vector instruction has
// just written.  Measured on this chip with register-resident loops (bnn_probe_pipeline and variants): MFMAs
// alone 8.6-9.3 PFLOP/s, with that dependent expansion 5.8-6.2, with the same number of INDEPENDENT vector
// instructions 7.4, with operands arriving from LDS and 14 independent vector instructions per K-step 7.2.
// So what costs is vector work that feeds the matrix pipe directly, and how much of it there is per MFMA.
// Here a workgroup of 8 waves owns a 256 x 256 tile (a wave: 128 x 64, 4 x 2 accumulators, as before).  A row
// fragment is shared by 4 waves: it is expanded once, by the thread that fetched it from global memory, and read
// from LDS as a finished operand.  Expanding the column operand the same way (a first version of this kernel) put
// eight 1 KB LDS instructions beside every eight MFMAs of a wave: counters showed the LDS pipe busy 71 % of the time at
// 8.2 cycles per instruction (128 bytes per cycle), i.e. LDS time equal to MFMA time at full matrix rate.  A column
// fragment is shared by only 2 waves, so it is the one to take out of LDS: its packed words are written once (one
// 16-byte unit per thread and slab instead of four) and each wave expands the two fragments of its next K-step
// itself -- 14 dependent vector instructions per K-step, a third of the staged kernel's, for 22 % fewer LDS
// instructions.  LDS pipe 53 % busy, MFMA 70 -> 74 % of the busy cycles, n = 16384: 5.80 -> 6.02 P binary op/s.
// One workgroup per compute unit (its two waves per SIMD hide each other's waits).
//
// LDS layout per buffer (41 KB, two buffers): A [word 0..7 of the slab][row 0..255 (+1 pad)] of 16-byte units (one
// unit = one packed word expanded = the four operand registers of one lane); B [plane 0..1][row 0..255 (+4 pad)],
// one unit = the four packed words a half-wave needs from that row (K-step v of a slab multiplies word v + 4 * half
// in both operands, so those four words are contiguous in global memory and in LDS).  16-byte LDS accesses are
// served eight lanes at a time, conflict-free when those eight units are distinct modulo 8 (128 bytes of banks): a
// fragment read is 32 consecutive units per half-wave; a loader wave writes, per instruction, words w and w + 4 of
// 32 consecutive rows (even and odd lanes), and the odd word pitch puts those 4 units apart modulo 8
// (measured: SQ_LDS_BANK_CONFLICT 1.7e7 cycles per launch at n = 8192 with a pitch of 258, none with 257).
#include <type_traits>

#include "bnn_mfma_kernel.h"

namespace bnn {
namespace {

using mfma::v16f;
using mfma::v8i;

constexpr int TILE = 256;                 // rows and columns of the workgroup tile
constexpr int WS = TILE + 1;              // units between consecutive words of a slab: odd (see the layout note)
constexpr int WIDE_THREADS = 512;
constexpr int MT = 4, NT = 2;             // accumulator tiles per wave: 128 x 64
constexpr int WM = 2, WN = 4;             // waves per workgroup tile
static_assert(WM * MT * 32 == TILE && WN * NT * 32 == TILE && WM * WN * 64 == WIDE_THREADS, "wave grid covers the tile");

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

constexpr int BP = TILE + 4;                        // units between the two planes of packed B
constexpr int A_UNITS = 8 * WS;
constexpr int BUF_UNITS = A_UNITS + 2 * BP;         // A expanded: 8 words x 257 units; B packed: 2 planes of 4 words per row

// PANELS: both operands (and the packed output, if there is one) are in the K-panel layout of bnn.h -- panel p holds
// words 8p .. 8p+7 of every row back to back -- so that a loader wave's 16-byte loads of one slab cover 1 KB of
// contiguous memory (8 lines of 128 bytes) instead of 32 bytes in each of 32 lines.
template <bool PANELS>
__global__ __launch_bounds__(WIDE_THREADS, 1) void mfma_wide_kernel(const uint32_t* __restrict__ A, const uint32_t* __restrict__ B,
                                                                         Geom g, Epi e, int gx, int gy) {
    extern __shared__ uint4 lds[];                  // 2 * BUF_UNITS
    mfma::accumulators_in_agprs();
    int bx, by;
    if (!mfma::tile_coords(gx, gy, bx, by)) return;
    const int tid = threadIdx.x;
    const int lane = tid & 63, l32 = lane & 31, half = lane >> 5, wave = tid >> 6;
    const int wm = wave / WN, wn = wave % WN;
    const long long m_base = (long long)bx * TILE;
    const int n_base = by * TILE;

    uint32_t c2;
    asm volatile("v_mov_b32 %0, 0x22222222" : "=v"(c2));

    // loader: thread -> row tid / 2 of A and of B, words 4 * (tid % 2) .. + 3 of every slab.  K-step v of a slab multiplies
    // word v of the lower half-wave's four words and word v of the upper one's: word v + 4 * half, in both operands.
    const int lrow = tid >> 1, lpart = tid & 1;
    const uint32_t* ap = A + min(m_base + lrow, g.rows - 1) * (long long)(PANELS ? 8 : g.lda_w) + 4 * lpart;
    const uint32_t* bp = B + (long long)min(n_base + lrow, g.cols - 1) * (PANELS ? 8 : g.ldb_w) + 4 * lpart;
    const int kwords = g.tw;                        // PANELS: a multiple of 8 (whole panels, pad bits 0)
    const int nslabs = (kwords + 7) / 8;
    const long long a_slab = PANELS ? g.rows * 8 : 8, b_slab = PANELS ? (long long)g.cols * 8 : 8;   // words from slab to slab

    uint4 ga, gb;
    // a slab part past the end of K (row-major operands only) reads the start of the row instead: a valid address,
    // and the store masks it
    auto slab_offset = [&](int s, long long step) { return (PANELS || s * 8 + 4 * lpart < kwords) ? s * step : (long long)(-4 * lpart); };
    auto load_a = [&](int s) { ga = *reinterpret_cast<const uint4*>(ap + slab_offset(s, a_slab)); };
    auto load_b = [&](int s) { gb = *reinterpret_cast<const uint4*>(bp + slab_offset(s, b_slab)); };
    auto store_a = [&](int buf, int s, auto masked) {
        const uint32_t keep = (!decltype(masked)::value || s * 8 + 4 * lpart < kwords) ? 0xFFFFFFFFu : 0u;
        uint4* base = lds + buf * BUF_UNITS + (4 * lpart) * WS + lrow;
        base[0] = expand_unit(ga.x & keep, c2); base[WS] = expand_unit(ga.y & keep, c2);
        base[2 * WS] = expand_unit(ga.z & keep, c2); base[3 * WS] = expand_unit(ga.w & keep, c2);
    };
    auto store_b = [&](int buf, int s, auto masked) {
        const uint32_t keep = (!decltype(masked)::value || s * 8 + 4 * lpart < kwords) ? 0xFFFFFFFFu : 0u;
        lds[buf * BUF_UNITS + A_UNITS + lpart * BP + lrow] = make_uint4(gb.x & keep, gb.y & keep, gb.z & keep, gb.w & keep);
    };

    v16f acc[MT][NT];
#pragma unroll
    for (int i = 0; i < MT; ++i)
#pragma unroll
        for (int j = 0; j < NT; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

    const int a_unit = 4 * half * WS + wm * (MT * 32) + l32;
    const int b_unit = A_UNITS + half * BP + wn * (NT * 32) + l32;
    uint4 fa[2][MT], fb[2][NT], bq[NT];
    auto read_a = [&](int buf, int v, int slot) {
        const uint4* base = lds + buf * BUF_UNITS + v * WS;
#pragma unroll
        for (int i = 0; i < MT; ++i) fa[slot][i] = base[a_unit + 32 * i];
    };
    auto read_bq = [&](int buf) {
#pragma unroll
        for (int j = 0; j < NT; ++j) bq[j] = lds[buf * BUF_UNITS + b_unit + 32 * j];
    };
    auto expand_b = [&](int v, int slot) {
#pragma unroll
        for (int j = 0; j < NT; ++j) {
            const uint32_t w = v == 0 ? bq[j].x : v == 1 ? bq[j].y : v == 2 ? bq[j].z : bq[j].w;
            fb[slot][j] = expand_unit(w, c2);
        }
    };
    auto multiply = [&](int slot) {
#pragma unroll
        for (int i = 0; i < MT; ++i)
#pragma unroll
            for (int j = 0; j < NT; ++j)
                acc[i][j] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(as_operand(fa[slot][i]), as_operand(fb[slot][j]),
                                                                            acc[i][j], 4, 4, 0, 0, 0, 0);
    };

    // One slab: four K-steps from buffer s & 1.  A fragments and the expansion of this wave's B fragments run one K-step
    // ahead.  MORE: the next slab (held in ga / gb) is stored into the other buffer during K-steps 1 and 2 and the registers
    // are refilled from global memory with the slab after it right behind (clamped to the last slab: a redundant load, no
    // branch); the ONE barrier of the slab follows K-step 2 -- by then every wave has read all of this slab's LDS data
    // (its last fragments were requested before K-step 2's MFMAs and the barrier waits for them) and has written its
    // share of the next -- and K-step 3 fetches the next slab's packed B words and first A fragments.
    auto slab = [&](int s, auto more, auto masked) {
        constexpr bool MORE = decltype(more)::value;
        const int buf = s & 1;
        const int s2 = min(s + 2, nslabs - 1);
#pragma unroll
        for (int v = 0; v < 4; ++v) {
            if (v < 3) { read_a(buf, v + 1, (v + 1) & 1); expand_b(v + 1, (v + 1) & 1); }
            if (MORE && v == 3) { read_a(buf ^ 1, 0, 0); read_bq(buf ^ 1); expand_b(0, 0); }
            // the packed B words again rather than carried over the loop edge: with them live across the edge (or with this
            // read unconditional) the compiler spills 400-600 registers in this loop
            if (v == 0 && s > 0) read_bq(buf);
            if (MORE && v == 1) { store_a(buf ^ 1, s + 1, masked); load_a(s2); }
            if (MORE && v == 2) { store_b(buf ^ 1, s + 1, masked); load_b(s2); }
            multiply(v & 1);
#pragma unroll
            for (int q = 0; q < MT * NT; ++q) {
                __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);   // an even mix for the scheduler: MFMA, vector ALU, LDS; the global load last
                __builtin_amdgcn_sched_group_barrier(0x002, 5, 0);
                __builtin_amdgcn_sched_group_barrier(0x080, 1, 0);
                if (MORE && (v == 1 || v == 2) && q == MT * NT - 1) __builtin_amdgcn_sched_group_barrier(0x020, 1, 0);
            }
            __builtin_amdgcn_sched_barrier(0);
            if (MORE && v == 2) __syncthreads();
        }
    };

    load_a(0); load_b(0);
    store_a(0, 0, std::true_type{}); store_b(0, 0, std::true_type{});
    load_a(min(1, nslabs - 1)); load_b(min(1, nslabs - 1));
    __syncthreads();
    read_a(0, 0, 0); read_bq(0); expand_b(0, 0);
    // only the last slab can be half-filled: the stores of every other slab need no mask
    for (int s = 0; s + 2 < nslabs; ++s) slab(s, std::true_type{}, std::false_type{});
    if (nslabs > 1) slab(nslabs - 2, std::true_type{}, std::true_type{});
    slab(nslabs - 1, std::false_type{}, std::false_type{});

    const long long m0 = m_base + (long long)wm * (MT * 32);
    const int n0 = n_base + wn * (NT * 32);
    const int corr_all = nslabs * 256 - g.bits_tap;
    if constexpr (PANELS) {
        if (e.bits != nullptr) {                    // uniform
            int thi[NT];
            bool cok[NT];
            mfma::column_thresholds<NT>(thi, cok, n0, l32, g, e);
            mfma::epilogue_bits<MT, NT, true>(acc, m0, n0, lane, g, e, corr_all, thi, cok);
            return;
        }
    }
    mfma::epilogue<MT, NT, false, false>(acc, m0, n0, lane, g, e, corr_all, 0);
}


}  // namespace

// Large products only: the 256 x 256 tiles must fill the chip (one workgroup per compute unit), and K must be long
// enough for the slab pipeline to matter.
bool mfma_wide_takes(const Geom& g, const Epi& e) {
    if (g.conv || g.b_tiled || g.tw < 32) return false;
    const int col_span = (e.bits != nullptr) ? max(g.cols, e.ldbits_w * 32) : g.cols;
    return cdiv(g.rows, TILE) * cdiv(col_span, TILE) >= 240;
}

template <bool PANELS>
static int launch_wide(const uint32_t* A, const uint32_t* B, const Geom& g, const Epi& e, hipStream_t s) {
    const int col_span = (e.bits != nullptr) ? max(g.cols, e.ldbits_w * 32) : g.cols;
    const int gx = (int)cdiv(g.rows, TILE), gy = (int)cdiv(col_span, TILE);
    const unsigned nwg = (unsigned)(cdiv((long long)gx * gy, 8) * 8);
    constexpr size_t lds_bytes = (size_t)2 * BUF_UNITS * 16;
    static const hipError_t attr = hipFuncSetAttribute(reinterpret_cast<const void*>(&mfma_wide_kernel<PANELS>),
                                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds_bytes);
    if (attr != hipSuccess) return BNN_ERR_DEVICE;
    hipLaunchKernelGGL(mfma_wide_kernel<PANELS>, dim3(nwg), dim3(WIDE_THREADS), lds_bytes, s, A, B, g, e, gx, gy);
    return check_launch();
}

int launch_mfma_wide(const uint32_t* A, const uint32_t* B, const Geom& g, const Epi& e, hipStream_t s) {
    return launch_wide<false>(A, B, g, e, s);
}

// Operands in K panels (g.tw a multiple of 8, lda_w / ldb_w unused); e.bits, if set, receives panels too
// (e.ldbits_w = 8 * number of output panels).  Any shape; the tile is sized for large ones.
int launch_mfma_wide_panels(const uint32_t* A, const uint32_t* B, const Geom& g, const Epi& e, hipStream_t s) {
    if (g.conv || g.b_tiled || (g.tw & 7) || g.rows >= (1LL << 31)) return BNN_ERR_UNSUPPORTED;
    if (e.bits != nullptr && (e.out != nullptr || e.out16 != nullptr || e.resid != nullptr || e.resid16 != nullptr ||
                              e.resid_bits != nullptr || (e.ldbits_w & 7)))
        return BNN_ERR_UNSUPPORTED;
    return launch_wide<true>(A, B, g, e, s);
}

}  // namespace bnn
