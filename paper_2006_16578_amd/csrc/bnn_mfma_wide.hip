// Matrix-core path for large matrix products: operands are expanded to E2M1 ONCE per workgroup, on their way
// into LDS, and the waves read finished MFMA operands.
//
// Why.  In the LDS-staged kernel of bnn_mfma_staged.h every wave expands the packed words of its own fragments:
// 42 vector-ALU instructions for the 8 MFMAs of a K-step, each MFMA waiting on registers a vector instruction has
// just written.  Measured on this chip with register-resident loops (bnn_probe_pipeline and variants): MFMAs
// alone 8.6-9.3 PFLOP/s, with that dependent expansion 5.8-6.2, with the same number of INDEPENDENT vector
// instructions 7.4, with operands arriving from LDS and 14 independent vector instructions per K-step 7.2.
// So what costs is vector work that feeds the matrix pipe directly, and how much of it there is per MFMA.
// Here a workgroup of 8 waves owns a 256 x 256 tile (a wave: 128 x 64, 4 x 2 accumulators, as before); a row
// fragment is shared by 4 waves and a column fragment by 2, and it is expanded once, by the thread that fetched
// it from global memory: 14 vector instructions and two 16-byte LDS writes per wave and K-step instead of 42,
// none of them on the MFMAs' critical path.  The price is LDS: an expanded slab of 256 bits of K is 64 KB for the
// tile, two buffers 128 KB, one workgroup per compute unit (its two waves per SIMD hide each other's waits).
//
// LDS layout per buffer: [operand A, B][word 0..7 of the slab][row 0..255 (+1 pad)] of 16-byte units (one unit =
// one packed word expanded = the four operand registers of one lane).  16-byte LDS accesses are served eight
// lanes at a time, conflict-free when those eight units are distinct modulo 8 (128 bytes of banks): a fragment
// read is 32 consecutive units per half-wave; a loader wave writes, per instruction, words w and w + 4 of 32
// consecutive rows (even and odd lanes), and the odd word pitch puts those 4 units apart modulo 8
// (measured: SQ_LDS_BANK_CONFLICT 1.7e7 cycles per launch at n = 8192 with a pitch of 258, none with 257).
#include <type_traits>

#include "bnn_mfma_kernel.h"

namespace bnn {
namespace {

using mfma::v16f;
using mfma::v8i;

constexpr int TILE = 256;                 // rows and columns of the workgroup tile
constexpr int WS = TILE + 1;              // units between consecutive words of a slab: odd (see the layout note)
constexpr int SLAB_UNITS = 2 * 8 * WS;    // A and B, 8 words each
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

__global__ __launch_bounds__(WIDE_THREADS, 1) void mfma_wide_kernel(const uint32_t* __restrict__ A, const uint32_t* __restrict__ B,
                                                                    Geom g, Epi e, int gx, int gy) {
    extern __shared__ uint4 lds[];                  // 2 * SLAB_UNITS
    mfma::accumulators_in_agprs();
    int bx, by;
    if (!mfma::tile_coords(gx, gy, bx, by)) return; // uniform for the workgroup
    const int tid = threadIdx.x;
    const int lane = tid & 63, l32 = lane & 31, half = lane >> 5, wave = tid >> 6;
    const int wm = wave / WN, wn = wave % WN;
    const long long m_base = (long long)bx * TILE;
    const int n_base = by * TILE;

    uint32_t c2;
    asm volatile("v_mov_b32 %0, 0x22222222" : "=v"(c2));

    // loader: thread -> row tid / 2 of A and of B, words 4 * (tid % 2) .. + 3 of every slab
    const int lrow = tid >> 1, lpart = tid & 1;
    const uint32_t* ap = A + min(m_base + lrow, g.rows - 1) * (long long)g.lda_w + 4 * lpart;   // clamp: results are dropped
    const uint32_t* bp = B + (long long)min(n_base + lrow, g.cols - 1) * g.ldb_w + 4 * lpart;
    const int kwords = g.tw;                          // multiple of 4
    const int nslabs = (kwords + 7) / 8;

    // The next slab's words on their way from global memory: ga (A row) is expanded during the second K-step of a
    // slab and reloaded right behind, gb (B row) during the third: each load has most of a slab to arrive, with
    // one register set.
    uint4 ga, gb;
    uint32_t gkeep = 0xFFFFFFFFu;                     // 0: the words lie past the row's end and count as zero words
    // past the row's end (upper half of a last, half-filled slab): the row's first words are read instead and
    // masked to zero words -- 0 bits in both operands -- when they are expanded; no branch, nothing waits here
    auto slab_offset = [&](int s) { return s * 8 + 4 * lpart < kwords ? s * 8 : -4 * lpart; };
    auto load_a = [&](int s) { ga = *reinterpret_cast<const uint4*>(ap + slab_offset(s)); };
    auto load_b = [&](int s) { gb = *reinterpret_cast<const uint4*>(bp + slab_offset(s)); };
    // expands the held A (or B) words of slab s into buffer `buf`
    auto store_a = [&](int buf, int s) {
        const uint32_t keep = s * 8 + 4 * lpart < kwords ? 0xFFFFFFFFu : 0u;
        uint4* base = lds + buf * SLAB_UNITS + (4 * lpart) * WS + lrow;
        base[0] = expand_unit(ga.x & keep, c2); base[WS] = expand_unit(ga.y & keep, c2);
        base[2 * WS] = expand_unit(ga.z & keep, c2); base[3 * WS] = expand_unit(ga.w & keep, c2);
    };
    auto store_b = [&](int buf, int s) {
        const uint32_t keep = s * 8 + 4 * lpart < kwords ? 0xFFFFFFFFu : 0u;
        uint4* base = lds + buf * SLAB_UNITS + (8 + 4 * lpart) * WS + lrow;
        base[0] = expand_unit(gb.x & keep, c2); base[WS] = expand_unit(gb.y & keep, c2);
        base[2 * WS] = expand_unit(gb.z & keep, c2); base[3 * WS] = expand_unit(gb.w & keep, c2);
    };
    (void)gkeep;

    v16f acc[MT][NT];
#pragma unroll
    for (int i = 0; i < MT; ++i)
#pragma unroll
        for (int j = 0; j < NT; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

    // fragment of K-step v: word 2v + half of rows wm*128 + 32i + l32 (A) / wn*64 + 32j + l32 (B)
    const int a_unit = half * WS + wm * (MT * 32) + l32;
    const int b_unit = 8 * WS + half * WS + wn * (NT * 32) + l32;
    uint4 fa[2][MT], fb[2][NT];
    auto read_frags = [&](int buf, int v, int slot) {
        const uint4* base = lds + buf * SLAB_UNITS + 2 * v * WS;
#pragma unroll
        for (int i = 0; i < MT; ++i) fa[slot][i] = base[a_unit + 32 * i];
#pragma unroll
        for (int j = 0; j < NT; ++j) fb[slot][j] = base[b_unit + 32 * j];
    };
    auto multiply = [&](int slot) {
#pragma unroll
        for (int i = 0; i < MT; ++i)
#pragma unroll
            for (int j = 0; j < NT; ++j)
                acc[i][j] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(as_operand(fa[slot][i]), as_operand(fb[slot][j]),
                                                                            acc[i][j], 4 /*A: E2M1*/, 4 /*B: E2M1*/, 0, 0, 0, 0);
    };

    // One slab: four K-steps from buffer `buf`, whose first fragments are already in registers.  MORE: the next
    // slab (held in ga / gb) is expanded into the other buffer during the first two K-steps, the registers are
    // refilled from global memory with the slab after it as soon as they are free (clamped to the last slab: a
    // redundant load, no branch),
    // and the ONE barrier of the slab comes after the third K-step.  At that point every wave has read all of this
    // slab (its last fragments were requested before the third K-step's MFMAs and the barrier waits for them), so
    // this buffer may be overwritten from the next slab on; and every wave has written its share of the next slab,
    // so its first fragments are requested during the fourth K-step and no wave starts a slab waiting for LDS.
    auto slab = [&](int s, auto more) {
        constexpr bool MORE = decltype(more)::value;
        const int buf = s & 1;
        const int s2 = min(s + 2, nslabs - 1);
#pragma unroll
        for (int v = 0; v < 4; ++v) {
            if (v < 3) read_frags(buf, v + 1, (v + 1) & 1);
            if (MORE && v == 3) read_frags(buf ^ 1, 0, 0);
            if (MORE && v == 1) { store_a(buf ^ 1, s + 1); load_a(s2); }
            if (MORE && v == 2) { store_b(buf ^ 1, s + 1); load_b(s2); }
            multiply(v & 1);
#pragma unroll
            for (int q = 0; q < MT * NT; ++q) {     // an even mix for the scheduler: MFMA, vector ALU, LDS; the global load last
                __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
                __builtin_amdgcn_sched_group_barrier(0x002, 4, 0);
                __builtin_amdgcn_sched_group_barrier(0x080, 2, 0);
                if (MORE && (v == 1 || v == 2) && q == MT * NT - 1) __builtin_amdgcn_sched_group_barrier(0x020, 1, 0);
            }
            __builtin_amdgcn_sched_barrier(0);      // nothing moves between K-steps: the expansions stay late, the loads early
            if (MORE && v == 2) __syncthreads();
        }
    };

    load_a(0); load_b(0);
    store_a(0, 0); store_b(0, 0);
    load_a(min(1, nslabs - 1)); load_b(min(1, nslabs - 1));
    __syncthreads();
    read_frags(0, 0, 0);
    for (int s = 0; s + 1 < nslabs; ++s) slab(s, std::true_type{});
    slab(nslabs - 1, std::false_type{});

    const long long m0 = m_base + (long long)wm * (MT * 32);
    const int n0 = n_base + wn * (NT * 32);
    // every slab multiplied 256 bit positions per row; those past K are 0 bits in both operands (+1 each)
    mfma::epilogue<MT, NT, false, false>(acc, m0, n0, lane, g, e, nslabs * 256 - g.bits_tap, 0);
}

}  // namespace

// Large products only: the 256 x 256 tiles must fill the chip (one workgroup per compute unit), and K must be long
// enough for the slab pipeline to matter.
bool mfma_wide_takes(const Geom& g, const Epi& e) {
    if (g.conv || g.b_tiled || g.tw < 32) return false;
    const int col_span = (e.bits != nullptr) ? max(g.cols, e.ldbits_w * 32) : g.cols;
    return cdiv(g.rows, TILE) * cdiv(col_span, TILE) >= 240;
}

int launch_mfma_wide(const uint32_t* A, const uint32_t* B, const Geom& g, const Epi& e, hipStream_t s) {
    const int col_span = (e.bits != nullptr) ? max(g.cols, e.ldbits_w * 32) : g.cols;
    const int gx = (int)cdiv(g.rows, TILE), gy = (int)cdiv(col_span, TILE);
    const unsigned nwg = (unsigned)(cdiv((long long)gx * gy, 8) * 8);
    constexpr size_t lds_bytes = (size_t)2 * SLAB_UNITS * 16;
    static const hipError_t attr = hipFuncSetAttribute(reinterpret_cast<const void*>(&mfma_wide_kernel),
                                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds_bytes);
    if (attr != hipSuccess) return BNN_ERR_DEVICE;
    hipLaunchKernelGGL(mfma_wide_kernel, dim3(nwg), dim3(WIDE_THREADS), lds_bytes, s, A, B, g, e, gx, gy);
    return check_launch();
}

}  // namespace bnn
