// Whole-network persistent kernel for chains of binarized layers -- fully-connected layers, 3x3 convolutions and the
// two convolutions of residual blocks (paper Sec. 6.2: every layer is a device function inside one kernel, a
// device-wide barrier separates consecutive layers).
//
// One launch; the grid is at most what the chip holds at once (occupancy x compute units), so on an otherwise
// idle device every workgroup is resident for the whole kernel, and if other work holds compute units the
// remaining workgroups start as soon as that work ends.  (A cooperative launch would have the runtime check
// the same bound, but costs about 25 us more per call here.)  Per layer the workgroups stride over that layer's 64x64 output tiles with the
// same matrix-core tile routine the per-layer kernels use, then meet at a barrier: a release fence, one
// atomic increment of a counter in device memory, a bounded spin on that counter, an acquire fence.  The
// fences are device scope, which on this chip writes back and invalidates the per-XCD L2, so bits written
// by a workgroup on one XCD are seen by workgroups on another.  If a spin ever exceeds its bound the
// workgroup raises an abort flag that releases every other waiter, and all waves leave the kernel: the
// grid always drains.
#include "bnn_internal.h"
#include "bnn_mfma_kernel.h"

namespace bnn {
namespace {

typedef mfma::TileSmall PTile;

__device__ __forceinline__ bool grid_barrier(unsigned* ctr, unsigned* abort_flag, unsigned target, int spin_limit) {
    __shared__ int ok_sh;
    __syncthreads();                                   // every wave of the workgroup has issued its stores
    if (threadIdx.x == 0) {
        int ok = 1;
        __threadfence();                               // release: this workgroup's stores, device scope
        __hip_atomic_fetch_add(ctr, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        int spins = 0;
        // relaxed polls: an acquiring load would invalidate the caches on every iteration
        while (__hip_atomic_load(ctr, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) < target) {
            if (++spins > spin_limit || __hip_atomic_load(abort_flag, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) != 0u) {
                __hip_atomic_store(abort_flag, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                ok = 0;
                break;
            }
            __builtin_amdgcn_s_sleep(4);
        }
        __threadfence();                               // acquire: later loads see the other workgroups' stores
        ok_sh = ok;
    }
    __syncthreads();
    return ok_sh != 0;
}

template <int V, bool EXCL, int CPT3>
__device__ __forceinline__ void conv_tile(const PersistLayer& L, int bx, int by) {
    mfma::mfma_tile<PTile, V, true, EXCL, false, CPT3>(L.A, L.B, L.g, L.e, bx, by);
}

__global__ __launch_bounds__(256, 3) void persist_chain_kernel(PersistNet net, const PersistLayer* __restrict__ layers,
                                                                         unsigned* ctr, int spin_limit, int sync) {
    const unsigned nwg = gridDim.x;
    unsigned phase = 0;
    if (net.in_u8 != nullptr) {                        // input layer: 8-bit pixels -> bits, one wave per row
        const int lane = threadIdx.x & 63;
        const int nw2 = (net.in_ldw + 1) / 2;
        for (long long row = (long long)blockIdx.x * 4 + (threadIdx.x >> 6); row < net.in_rows; row += (long long)nwg * 4) {
            const uint8_t* xr = net.in_u8 + row * net.in_cols;
            uint32_t* br = net.in_bits + row * net.in_ldw;
            for (int g = 0; g < nw2; ++g) {
                const int c = g * 64 + lane;
                const bool pred = c < net.in_cols && (int)xr[c] >= net.in_thr;
                const unsigned long long ball = __builtin_amdgcn_ballot_w64(pred);
                if (lane == 0) br[2 * g] = (uint32_t)ball;
                if (lane == 1 && 2 * g + 1 < net.in_ldw) br[2 * g + 1] = (uint32_t)(ball >> 32);
            }
        }
        ++phase;
        if (sync && !grid_barrier(ctr, ctr + 1, phase * nwg, spin_limit)) return;
    }
    for (int l = 0; l < net.nlayers; ++l) {
        const PersistLayer& L = layers[l];
        const int total = L.gx * L.gy;
        for (int t = (int)blockIdx.x; t < total; t += (int)nwg) {
            const int by = t / L.gx, bx = t - by * L.gx;
            switch (L.variant) {                       // uniform
                case 0: mfma::mfma_tile<PTile, 4, false, false, true>(L.A, L.B, L.g, L.e, bx, by); break;
                case 1: conv_tile<1, false, 1>(L, bx, by); break;     // 64 channels
                case 2: conv_tile<1, true, 1>(L, bx, by); break;
                case 3: conv_tile<2, false, 1>(L, bx, by); break;     // 128
                case 4: conv_tile<2, true, 1>(L, bx, by); break;
                case 5: conv_tile<4, false, 1>(L, bx, by); break;     // 256
                case 6: conv_tile<4, true, 1>(L, bx, by); break;
                case 7: conv_tile<4, false, 2>(L, bx, by); break;     // 512
                default: conv_tile<4, true, 2>(L, bx, by); break;
            }
        }
        if (l + 1 < net.nlayers) {
            ++phase;
            if (sync && !grid_barrier(ctr, ctr + 1, phase * nwg, spin_limit)) return;
        }
    }
}

__global__ void persist_clear_kernel(unsigned* ctr) {
    if (threadIdx.x < 2) ctr[threadIdx.x] = 0u;
}

}  // namespace

int persist_conv_variant(const Geom& g) {
    if (!g.conv || g.k != 3 || g.taps != 9 || g.bits_tap != g.tw * 32 || g.lda_w != g.tw || !mfma::offsets_fit(g)) return -1;
    int form;
    switch (g.tw) {
        case 2: form = 0; break;
        case 4: form = 1; break;
        case 8: form = 2; break;
        case 16: form = 3; break;
        default: return -1;
    }
    return 2 * form + (g.excl ? 1 : 0);
}

// ctr: two words of device memory (barrier counter, abort flag).  sync == 0 skips the barriers: the results
// are then undefined; it exists to time the cost of the barriers alone.  spin_limit: polls (each an s_sleep and
// one device-scope load, about a microsecond) before a waiter gives up.
int launch_persist_chain(const PersistNet& net, int max_tiles, int max_grid, unsigned* ctr, int sync, int spin_limit,
                         hipStream_t s) {
    // workgroups the current device holds at once (queried per call: the property belongs to the device)
    int dev = 0, cus = 0, per_cu = 0;
    if (hipGetDevice(&dev) != hipSuccess) return BNN_ERR_DEVICE;
    if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess) return BNN_ERR_DEVICE;
    if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, reinterpret_cast<const void*>(&persist_chain_kernel), 256, 0) !=
        hipSuccess)
        return BNN_ERR_DEVICE;
    if (cus < 1 || per_cu < 1) return BNN_ERR_DEVICE;
    const int max_wg = cus * per_cu;
    int want = max(1, max_tiles);
    if (net.in_u8 != nullptr) {
        const long long row_groups = cdiv(net.in_rows, 4);
        want = max(want, row_groups < (1 << 20) ? (int)row_groups : (1 << 20));
    }
    const int grid = min(min(want, max_wg), max(1, max_grid));
    hipLaunchKernelGGL(persist_clear_kernel, dim3(1), dim3(64), 0, s, ctr);
    hipLaunchKernelGGL(persist_chain_kernel, dim3((unsigned)grid), dim3(256), 0, s, net, net.layers, ctr, spin_limit, sync);
    return check_launch();
}

}  // namespace bnn
