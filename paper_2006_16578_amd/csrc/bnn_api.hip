// C ABI of libbnn: argument validation, shape bookkeeping and kernel dispatch.
#include <string.h>

#include <algorithm>
#include <mutex>
#include <new>
#include <vector>

#include "bnn_internal.h"

using namespace bnn;

namespace {

inline bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }
inline int words(int nbits) { return (nbits + 31) / 32; }
inline int round4(int v) { return (v + 3) / 4 * 4; }

// While a persistent forward collects a chain, a layer's contraction is recorded here instead of launched.
thread_local std::vector<PersistLayer>* capture_sink = nullptr;

int dispatch(const uint32_t* A, const uint32_t* B, const Geom& g, const Epi& e, int path, hipStream_t s) {
    if (capture_sink != nullptr) {
        if (capture_sink->size() >= (size_t)PERSIST_MAX_LAYERS || g.b_tiled) return BNN_ERR_UNSUPPORTED;
        PersistLayer P = {};
        P.A = A; P.B = B; P.g = g; P.e = e;
        if (g.conv) {
            const int v = persist_conv_variant(g);
            if (v < 0) return BNN_ERR_UNSUPPORTED;
            P.variant = 1 + v;
        } else {
            if (g.lda_w >= (1 << 20) || g.ldb_w >= (1 << 21)) return BNN_ERR_UNSUPPORTED;
            P.variant = 0;
        }
        const int col_span = (e.bits != nullptr) ? std::max(g.cols, e.ldbits_w * 32) : g.cols;   // pad words are written too
        P.gx = (int)cdiv(g.rows, 64); P.gy = (int)cdiv(col_span, 64);
        capture_sink->push_back(P);
        return BNN_OK;
    }
    switch (path) {
        case BNN_PATH_VALU: return launch_valu(A, B, g, e, s);
        case BNN_PATH_MFMA: return launch_mfma(A, B, g, e, s);
        case BNN_PATH_AUTO: {
            // the matrix cores for everything they take; a shape beyond their kernels' 32-bit offsets (nothing has
            // been enqueued then) goes to the vector-ALU kernel, which addresses with 64 bits
            const int rc = launch_mfma(A, B, g, e, s);
            return rc == BNN_ERR_UNSUPPORTED ? launch_valu(A, B, g, e, s) : rc;
        }
        default: return BNN_ERR_INVALID_ARG;
    }
}

Geom bmm_geom(int M, int N, int K, int lda_w, int ldb_w) {
    Geom g = {};
    g.rows = M; g.cols = N; g.conv = 0; g.taps = 1; g.tw = round4(words(K)); g.bits_tap = K;
    g.lda_w = lda_w; g.ldb_w = ldb_w;
    g.H = g.W = g.P = g.Q = g.k = g.stride = 1; g.pad = 0; g.excl = 0; g.kinv = 65536;
    g.div_pq = make_fastdiv(1u); g.div_q = make_fastdiv(1u);
    return g;
}

int bmm_common(const uint32_t* A, const uint32_t* B, int32_t* C, const int32_t* thr, uint32_t* Cbits,
               int M, int N, int K, int lda_w, int ldb_w, int ldc, int ldcb_w, int path, void* stream, bool out_f32 = false,
               bool b_tiled = false) {
    if (!A || !B || M < 1 || N < 1 || K < 1) return BNN_ERR_INVALID_ARG;
    if (!C && !Cbits) return BNN_ERR_INVALID_ARG;
    if (Cbits && !thr) return BNN_ERR_INVALID_ARG;
    if (K > BNN_MAX_K) return BNN_ERR_UNSUPPORTED;
    const int kw4 = round4(words(K));
    if (lda_w < kw4 || ldb_w < kw4) return BNN_ERR_INVALID_ARG;
    if ((lda_w & 3) || (ldb_w & 3) || !aligned16(A) || !aligned16(B)) return BNN_ERR_ALIGNMENT;
    if (C && (ldc < N || !aligned16(C))) return ldc < N ? BNN_ERR_INVALID_ARG : BNN_ERR_ALIGNMENT;
    if (Cbits && (ldcb_w < words(N) || !aligned16(Cbits))) return ldcb_w < words(N) ? BNN_ERR_INVALID_ARG : BNN_ERR_ALIGNMENT;
    if (thr && !aligned16(thr)) return BNN_ERR_ALIGNMENT;
    Geom g = bmm_geom(M, N, K, lda_w, ldb_w);
    g.b_tiled = b_tiled ? 1 : 0;
    if (b_tiled && path == BNN_PATH_VALU) return BNN_ERR_UNSUPPORTED;
    Epi e = {};
    e.out = C; e.resid = nullptr; e.ldc = ldc; e.thr = thr; e.bits = Cbits; e.ldbits_w = ldcb_w; e.out_f32 = out_f32 ? 1 : 0;
    return dispatch(A, B, g, e, path, static_cast<hipStream_t>(stream));
}

int conv_shape(int N, int H, int W, int C, int O, int k, int stride, int pad, int pad_mode, int* P, int* Q) {
    if (N < 1 || H < 1 || W < 1 || C < 1 || O < 1 || k < 1 || stride < 1 || pad < 0) return BNN_ERR_INVALID_ARG;
    if (pad_mode != BNN_PAD_MINUS_ONE && pad_mode != BNN_PAD_EXCLUDE) return BNN_ERR_INVALID_ARG;
    if (H + 2 * pad < k || W + 2 * pad < k) return BNN_ERR_INVALID_ARG;
    if (pad >= k || k > 32) return BNN_ERR_UNSUPPORTED;    // a window entirely out of frame; tap index arithmetic
    if ((long long)k * k * C > BNN_MAX_K) return BNN_ERR_UNSUPPORTED;
    *P = (H + 2 * pad - k) / stride + 1;
    *Q = (W + 2 * pad - k) / stride + 1;
    if ((long long)N * *P * *Q * O > (1LL << 40) || (long long)N * *P * *Q >= (1LL << 31)) return BNN_ERR_UNSUPPORTED;
    return BNN_OK;
}

// resid_bits (internal, used by the layer chain): a packed [N][P][Q][ceil(O/32)] tensor whose +1/-1
// values are the residual, instead of an int32 tensor.
int bconv_common(const uint32_t* in, const uint32_t* filt, int32_t* out, const int32_t* resid,
                 const int32_t* thr, uint32_t* bits, int N, int H, int W, int C, int O, int k, int stride,
                 int pad, int pad_mode, int path, void* stream, const uint32_t* resid_bits = nullptr,
                 const uint32_t* x2 = nullptr, const uint32_t* filt2 = nullptr, int H2 = 0, int W2 = 0, int C2 = 0,
                 int stride2 = 1, bool sums16 = false, bool out_f32 = false) {
    if (!in || !filt) return BNN_ERR_INVALID_ARG;
    if (!out && !bits) return BNN_ERR_INVALID_ARG;
    if (bits && !thr) return BNN_ERR_INVALID_ARG;
    int P, Q;
    int rc = conv_shape(N, H, W, C, O, k, stride, pad, pad_mode, &P, &Q);
    if (rc != BNN_OK) return rc;
    if (!aligned16(in) || !aligned16(filt) || (out && !aligned16(out)) || (resid && !aligned16(resid)) ||
        (bits && !aligned16(bits)) || (thr && !aligned16(thr)))
        return BNN_ERR_ALIGNMENT;
    const int cw = words(C);
    Geom g = {};
    g.rows = (long long)N * P * Q; g.cols = O; g.conv = 1; g.taps = k * k; g.tw = cw; g.bits_tap = C;
    g.lda_w = cw; g.ldb_w = k * k * cw;
    g.H = H; g.W = W; g.P = P; g.Q = Q; g.k = k; g.stride = stride; g.pad = pad; g.kinv = (65536 + k - 1) / k;
    g.div_pq = make_fastdiv((uint32_t)(P * Q)); g.div_q = make_fastdiv((uint32_t)Q);
    g.excl = (pad_mode == BNN_PAD_EXCLUDE) ? 1 : 0;
    if (x2 != nullptr) {    // fused 1x1 shortcut convolution (internal callers only; shapes already checked)
        if (!filt2 || C2 < 1 || stride2 < 1 || (P - 1) * stride2 >= H2 || (Q - 1) * stride2 >= W2) return BNN_ERR_INVALID_ARG;
        g.A2 = x2; g.B2 = filt2; g.H2 = H2; g.W2 = W2; g.cw2 = words(C2); g.stride2 = stride2; g.bits2 = C2;
    }
    Epi e = {};
    e.out = out; e.resid = resid; e.ldc = O; e.thr = thr; e.bits = bits; e.ldbits_w = words(O); e.out_f32 = out_f32 ? 1 : 0;
    e.resid_bits = resid ? nullptr : resid_bits; e.ld_resid_bits_w = words(O);
    if (sums16) {       // internal callers: out / resid point at 16-bit storage of the same values
        e.out16 = reinterpret_cast<int16_t*>(out); e.out = nullptr;
        e.resid16 = reinterpret_cast<const int16_t*>(resid); e.resid = nullptr;
        e.sums_tiled = (O % 32 == 0) ? 1 : 0;      // the buffers hold 32 rows more than the tensor (plan())
    }
    return dispatch(in, filt, g, e, path, static_cast<hipStream_t>(stream));
}

}  // namespace

// ------------------------------------------------------------------------------------------ net
struct bnn_net {
    enum Kind { IN_U8, IN_BITS, IN_CONV_F32, FC, CONV, POOL, BLOCK, HEAD };
    struct Layer {
        Kind kind;
        const void* w0 = nullptr; const void* w1 = nullptr; const void* w2 = nullptr;   // weights
        const void* t0 = nullptr; const void* t1 = nullptr;                              // thresholds
        int a = 0, b = 0, c = 0, d = 0, k = 0, stride = 0, pad = 0, pad_mode = 0, thr_u8 = 0;
        // filled by plan(): spatial size and channels of the output, where its bits live
        int H = 1, W = 1, C = 0;
        size_t bits_off = 0; int words_per_row = 0; long long rows_per_image = 1;
        long long sum_bound = 0;      // BLOCK: largest |S| this block can produce
        bool bwn = false;             // IN_CONV_F32: w0 holds weight bits (first layer with binarized weights)
    };
    std::vector<Layer> layers;
    // results of the last forward, for bnn_net_layer_bits
    const char* last_ws = nullptr; int last_batch = 0;
    const unsigned* last_persist_sync = nullptr;   // barrier counter and abort flag of the last persistent forward
    // layer table of the last persistent forward as uploaded, and where: an identical table is not uploaded again
    std::vector<PersistLayer> persist_uploaded;
    const void* persist_uploaded_at = nullptr;
};

namespace {

inline size_t align256(size_t v) { return (v + 255) / 256 * 256; }

// Walks the layer list for `batch` inputs, assigning workspace offsets.  Layout: every layer's
// output bits get their own slot (they are small: 1 bit per activation), int32 residuals use
// three rotating slots sized for the largest residual tensor.
struct Plan {
    bool sums16 = false;     // every block sum fits 16 bits: residuals are stored as int16
    size_t total = 0;
    size_t resid_off[3] = {0, 0, 0};
    size_t resid_bytes = 0;
    size_t bwn_off = 0, bwn_bytes = 0;   // expanded first-layer weights (first layer with binarized weights only)
    size_t sync_off = 0;                 // barrier counter and abort flag of the persistent kernel
    size_t table_off = 0;                // layer table of the persistent kernel
    size_t pool_off = 0;                 // pooled sums [batch][C] int32 of a HEAD layer
    int rc = BNN_OK;
};

Plan plan(bnn_net* net, int batch) {
    Plan pl;
    size_t off = 0;
    int H = 1, W = 1, C = 0;
    size_t max_resid = 0;
    bool have_resid = false;
    size_t head_pool_bytes = 0;
    long long chain_bound = 1, max_bound = 0;     // |running residual| <= chain_bound
    for (size_t i = 0; i < net->layers.size(); ++i) {
        bnn_net::Layer& L = net->layers[i];
        if ((i == 0) != (L.kind == bnn_net::IN_U8 || L.kind == bnn_net::IN_BITS || L.kind == bnn_net::IN_CONV_F32)) {
            pl.rc = BNN_ERR_INVALID_ARG; return pl;
        }
        switch (L.kind) {
            case bnn_net::IN_U8: case bnn_net::IN_BITS:
                H = W = 1; C = L.a; L.words_per_row = round4(words(C)); break;
            case bnn_net::IN_CONV_F32:
                H = (L.a + 2 * L.pad - L.k) / L.stride + 1; W = (L.b + 2 * L.pad - L.k) / L.stride + 1; C = L.d;
                L.words_per_row = words(C); break;
            case bnn_net::FC:
                if (H * W * words(C) * 32 != H * W * C && H * W != 1) { pl.rc = BNN_ERR_UNSUPPORTED; return pl; }
                if (H * W * C != L.a) { pl.rc = BNN_ERR_INVALID_ARG; return pl; }
                // the flattened activation is the A operand as it lies in memory: its row stride (H*W pixels of
                // words(C) words for a spatial producer) must satisfy the BMM's 128-bit row alignment
                if (i > 0 && net->layers[i - 1].kind != bnn_net::FC && net->layers[i - 1].kind != bnn_net::IN_U8 &&
                    net->layers[i - 1].kind != bnn_net::IN_BITS && (H * W * words(C)) % 4 != 0) {
                    pl.rc = BNN_ERR_UNSUPPORTED; return pl;
                }
                H = W = 1; C = L.b; L.words_per_row = round4(words(C)); break;
            case bnn_net::CONV:
                if (C != L.a) { pl.rc = BNN_ERR_INVALID_ARG; return pl; }
                H = (H + 2 * L.pad - L.k) / L.stride + 1; W = (W + 2 * L.pad - L.k) / L.stride + 1; C = L.b;
                L.words_per_row = words(C); break;
            case bnn_net::POOL:
                if (H < L.k || W < L.k) { pl.rc = BNN_ERR_INVALID_ARG; return pl; }
                H = (H - L.k) / L.stride + 1; W = (W - L.k) / L.stride + 1;
                L.words_per_row = words(C); break;
            case bnn_net::BLOCK:
                if (C != L.a) { pl.rc = BNN_ERR_INVALID_ARG; return pl; }
                if (!L.w2 && (L.stride != 1 || L.a != L.b)) { pl.rc = BNN_ERR_INVALID_ARG; return pl; }
                H = (H + 2 - 3) / L.stride + 1; W = (W + 2 - 3) / L.stride + 1; C = L.b;
                L.words_per_row = words(C);
                have_resid = true;
                // |S| <= |conv3x3(h)| + |shortcut|: 9*cout + (cin for a 1x1 downsample, else the running bound,
                // which restarts at 1 (+1/-1 input bits) at the head of a chain)
                if (L.w2) chain_bound = L.a;
                else if (i == 0 || net->layers[i - 1].kind != bnn_net::BLOCK) chain_bound = 1;
                chain_bound += 9LL * L.b;
                L.sum_bound = chain_bound;
                max_bound = max(max_bound, chain_bound);
                break;
            case bnn_net::HEAD:
                if (i + 1 != net->layers.size()) { pl.rc = BNN_ERR_INVALID_ARG; return pl; }
                head_pool_bytes = align256((size_t)batch * C * 4);
                L.words_per_row = 0; break;
        }
        if (H < 1 || W < 1) { pl.rc = BNN_ERR_INVALID_ARG; return pl; }
        L.H = H; L.W = W; L.C = C; L.rows_per_image = (long long)H * W;
        if (L.kind == bnn_net::HEAD || (L.kind == bnn_net::FC && L.t0 == nullptr)) {
            if (i + 1 != net->layers.size()) { pl.rc = BNN_ERR_INVALID_ARG; return pl; }
            continue;
        }
        L.bits_off = off;
        size_t bytes = (size_t)batch * H * W * L.words_per_row * 4;
        if (L.kind == bnn_net::BLOCK) bytes = 2 * align256(bytes);   // hidden bits h of the block, then (aligned) its output
        off += align256(bytes);
        if (L.kind == bnn_net::BLOCK || L.kind == bnn_net::IN_CONV_F32 || L.kind == bnn_net::CONV)
            max_resid = max(max_resid, ((size_t)batch * H * W + 32) * C * 4);   // + 32 rows: blocked 16-bit sums pad rows
    }
    pl.sums16 = have_resid && max_bound <= 32767;
    if (have_resid) {
        pl.resid_bytes = align256(max_resid);
        for (int r = 0; r < 3; ++r) { pl.resid_off[r] = off; off += pl.resid_bytes; }
    }
    if (net->layers[0].kind == bnn_net::IN_CONV_F32) {
        const bnn_net::Layer& L0 = net->layers[0];
        pl.bwn_off = off;
        pl.bwn_bytes = L0.bwn ? bwn_workspace_bytes(L0.c, L0.d, L0.k) : conv_f32_split_workspace_bytes(L0.c, L0.d, L0.k);
        off += align256(pl.bwn_bytes);
    }
    pl.sync_off = off; off += 256;
    pl.table_off = off; off += align256(sizeof(PersistLayer) * PERSIST_MAX_LAYERS);
    pl.pool_off = off; off += head_pool_bytes;
    pl.total = off;
    return pl;
}

}  // namespace

extern "C" {

const char* bnn_status_string(int status) {
    switch (status) {
        case BNN_OK: return "ok";
        case BNN_ERR_INVALID_ARG: return "invalid argument";
        case BNN_ERR_ALIGNMENT: return "pointer or leading dimension not aligned";
        case BNN_ERR_UNSUPPORTED: return "unsupported size or configuration";
        case BNN_ERR_DEVICE: return "HIP launch failure";
        case BNN_ERR_WORKSPACE: return "workspace missing or too small";
        default: return "unknown status";
    }
}

int bnn_version(void) { return 100; }

const char* bnn_bmm_kernel_name(int M, int N, int K, int path) {
    return bnn_bmm_kernel_name_out(M, N, K, path, BNN_OUT_BITS);
}
const char* bnn_bconv_kernel_name(int N, int H, int W, int C, int O, int k, int stride, int pad, int path) {
    return bnn_bconv_kernel_name_out(N, H, W, C, O, k, stride, pad, path, BNN_OUT_BITS);
}
const char* bnn_bmm_kernel_name_out(int M, int N, int K, int path, int out_kind) {
    if (M < 1 || N < 1 || K < 1 || K > BNN_MAX_K || (out_kind != BNN_OUT_BITS && out_kind != BNN_OUT_INT32)) return "invalid";
    Geom g = {};
    g.rows = M; g.cols = N; g.conv = 0; g.taps = 1; g.tw = round4(words(K)); g.bits_tap = K;
    return path == BNN_PATH_VALU ? describe_valu(g) : describe_mfma(g, out_kind == BNN_OUT_INT32);
}
const char* bnn_bconv_kernel_name_out(int N, int H, int W, int C, int O, int k, int stride, int pad, int path,
                                      int out_kind) {
    int P, Q;
    if (out_kind != BNN_OUT_BITS && out_kind != BNN_OUT_INT32) return "invalid";
    if (conv_shape(N, H, W, C, O, k, stride, pad, BNN_PAD_MINUS_ONE, &P, &Q) != BNN_OK) return "invalid";
    Geom g = {};
    g.rows = (long long)N * P * Q; g.cols = O; g.conv = 1; g.taps = k * k; g.tw = words(C); g.bits_tap = C;
    g.H = H; g.W = W; g.P = P; g.Q = Q; g.k = k; g.stride = stride; g.pad = pad; g.lda_w = g.tw; g.ldb_w = k * k * g.tw;
    return path == BNN_PATH_VALU ? describe_valu(g) : describe_mfma(g, out_kind == BNN_OUT_INT32);
}

int bnn_bmm(const uint32_t* A, const uint32_t* B, int32_t* C, int M, int N, int K, int lda_w, int ldb_w, int ldc,
            void* stream) {
    return bnn_bmm_ex(A, B, C, M, N, K, lda_w, ldb_w, ldc, BNN_PATH_AUTO, stream);
}
int bnn_bmm_ex(const uint32_t* A, const uint32_t* B, int32_t* C, int M, int N, int K, int lda_w, int ldb_w, int ldc,
               int path, void* stream) {
    if (!C) return BNN_ERR_INVALID_ARG;
    return bmm_common(A, B, C, nullptr, nullptr, M, N, K, lda_w, ldb_w, ldc, 0, path, stream);
}
int bnn_bmm_thr(const uint32_t* A, const uint32_t* B, const int32_t* thr, uint32_t* Cbits, int M, int N, int K,
                int lda_w, int ldb_w, int ldcb_w, void* stream) {
    return bnn_bmm_thr_ex(A, B, thr, Cbits, M, N, K, lda_w, ldb_w, ldcb_w, BNN_PATH_AUTO, stream);
}
int bnn_bmm_thr_ex(const uint32_t* A, const uint32_t* B, const int32_t* thr, uint32_t* Cbits, int M, int N, int K,
                   int lda_w, int ldb_w, int ldcb_w, int path, void* stream) {
    if (!Cbits || !thr) return BNN_ERR_INVALID_ARG;
    return bmm_common(A, B, nullptr, thr, Cbits, M, N, K, lda_w, ldb_w, 0, ldcb_w, path, stream);
}

int bnn_bconv(const uint32_t* in, const uint32_t* filt, int32_t* out, int N, int H, int W, int C, int O, int k,
              int stride, int pad, int pad_mode, void* stream) {
    return bnn_bconv_ex(in, filt, out, N, H, W, C, O, k, stride, pad, pad_mode, BNN_PATH_AUTO, stream);
}
int bnn_bconv_ex(const uint32_t* in, const uint32_t* filt, int32_t* out, int N, int H, int W, int C, int O, int k,
                 int stride, int pad, int pad_mode, int path, void* stream) {
    if (!out) return BNN_ERR_INVALID_ARG;
    return bconv_common(in, filt, out, nullptr, nullptr, nullptr, N, H, W, C, O, k, stride, pad, pad_mode, path, stream);
}
int bnn_bconv_thr(const uint32_t* in, const uint32_t* filt, const int32_t* residual_in, int32_t* sum_out,
                  const int32_t* thr, uint32_t* out_bits, int N, int H, int W, int C, int O, int k, int stride,
                  int pad, int pad_mode, void* stream) {
    return bnn_bconv_thr_ex(in, filt, residual_in, sum_out, thr, out_bits, N, H, W, C, O, k, stride, pad, pad_mode,
                            BNN_PATH_AUTO, stream);
}
int bnn_bconv_thr_ex(const uint32_t* in, const uint32_t* filt, const int32_t* residual_in, int32_t* sum_out,
                     const int32_t* thr, uint32_t* out_bits, int N, int H, int W, int C, int O, int k, int stride,
                     int pad, int pad_mode, int path, void* stream) {
    if (!out_bits || !thr) return BNN_ERR_INVALID_ARG;
    return bconv_common(in, filt, sum_out, residual_in, thr, out_bits, N, H, W, C, O, k, stride, pad, pad_mode, path,
                        stream);
}

int bnn_threshold_pack(const int32_t* X, const int32_t* thr, uint32_t* bits, int64_t rows, int cols, int ldx,
                       int ldb_w, void* stream) {
    if (!X || !thr || !bits || rows < 1 || cols < 1 || ldx < cols || ldb_w < words(cols)) return BNN_ERR_INVALID_ARG;
    if (rows > (1LL << 33)) return BNN_ERR_UNSUPPORTED;
    return launch_threshold_pack(X, thr, bits, rows, cols, ldx, ldb_w, static_cast<hipStream_t>(stream));
}
int bnn_pack_u8(const uint8_t* x, int thr, uint32_t* bits, int64_t rows, int cols, int ldb_w, void* stream) {
    if (!x || !bits || rows < 1 || cols < 1 || ldb_w < words(cols)) return BNN_ERR_INVALID_ARG;
    if (rows > (1LL << 33)) return BNN_ERR_UNSUPPORTED;
    return launch_pack_u8(x, thr, bits, rows, cols, ldb_w, static_cast<hipStream_t>(stream));
}
int bnn_pack_f32(const float* x, const float* thr, uint32_t* bits, int64_t rows, int cols, int ldb_w, void* stream) {
    if (!x || !thr || !bits || rows < 1 || cols < 1 || ldb_w < words(cols)) return BNN_ERR_INVALID_ARG;
    if (rows > (1LL << 33)) return BNN_ERR_UNSUPPORTED;
    return launch_pack_f32(x, thr, bits, rows, cols, ldb_w, static_cast<hipStream_t>(stream));
}
int bnn_tile_b(const uint32_t* B, uint32_t* B_tiled, int N, int K, int ldb_w, void* stream) {
    if (!B || !B_tiled || N < 1 || K < 1 || ldb_w < round4(words(K))) return BNN_ERR_INVALID_ARG;
    if ((ldb_w & 3) || !aligned16(B) || !aligned16(B_tiled)) return BNN_ERR_ALIGNMENT;
    return launch_tile_b(B, B_tiled, N, ldb_w, static_cast<hipStream_t>(stream));
}
int bnn_bmm_tiled(const uint32_t* A, const uint32_t* B_tiled, int32_t* C, int M, int N, int K, int lda_w, int ldb_w, int ldc,
                  void* stream) {
    if (!C) return BNN_ERR_INVALID_ARG;
    return bmm_common(A, B_tiled, C, nullptr, nullptr, M, N, K, lda_w, ldb_w, ldc, 0, BNN_PATH_MFMA, stream, false, true);
}
int bnn_bmm_thr_tiled(const uint32_t* A, const uint32_t* B_tiled, const int32_t* thr, uint32_t* Cbits, int M, int N, int K,
                      int lda_w, int ldb_w, int ldcb_w, void* stream) {
    if (!Cbits || !thr) return BNN_ERR_INVALID_ARG;
    return bmm_common(A, B_tiled, nullptr, thr, Cbits, M, N, K, lda_w, ldb_w, 0, ldcb_w, BNN_PATH_MFMA, stream, false, true);
}
int bnn_panels_from_rows(const uint32_t* X, uint32_t* Xp, int64_t rows, int K, int ldx_w, void* stream) {
    if (!X || !Xp || rows < 1 || K < 1 || ldx_w < words(K)) return BNN_ERR_INVALID_ARG;
    if (K > BNN_MAX_K || rows >= (1LL << 31)) return BNN_ERR_UNSUPPORTED;
    if (!aligned16(Xp)) return BNN_ERR_ALIGNMENT;
    return launch_panels_from_rows(X, Xp, rows, K, ldx_w, static_cast<hipStream_t>(stream));
}
int bnn_rows_from_panels(const uint32_t* Xp, uint32_t* X, int64_t rows, int K, int ldx_w, void* stream) {
    if (!X || !Xp || rows < 1 || K < 1 || ldx_w < words(K)) return BNN_ERR_INVALID_ARG;
    if (K > BNN_MAX_K || rows >= (1LL << 31)) return BNN_ERR_UNSUPPORTED;
    if ((ldx_w & 3) || !aligned16(Xp) || !aligned16(X)) return BNN_ERR_ALIGNMENT;
    return launch_rows_from_panels(Xp, X, rows, K, ldx_w, static_cast<hipStream_t>(stream));
}
static int bmm_panels_common(const uint32_t* Ap, const uint32_t* Bp, int32_t* C, const int32_t* thr, uint32_t* Cbits_p, int M, int N,
                             int K, int ldc, void* stream) {
    if (!Ap || !Bp || M < 1 || N < 1 || K < 1) return BNN_ERR_INVALID_ARG;
    if (K > BNN_MAX_K) return BNN_ERR_UNSUPPORTED;
    if (!aligned16(Ap) || !aligned16(Bp)) return BNN_ERR_ALIGNMENT;
    if (C && (ldc < N || !aligned16(C))) return ldc < N ? BNN_ERR_INVALID_ARG : BNN_ERR_ALIGNMENT;
    if (Cbits_p && (!aligned16(Cbits_p) || !aligned16(thr))) return BNN_ERR_ALIGNMENT;
    const int kw8 = (words(K) + 7) / 8 * 8;
    Geom g = bmm_geom(M, N, K, kw8, kw8);
    g.tw = kw8;
    Epi e = {};
    e.out = C; e.ldc = ldc; e.thr = thr; e.bits = Cbits_p; e.ldbits_w = (words(N) + 7) / 8 * 8;
    return launch_mfma_wide_panels(Ap, Bp, g, e, static_cast<hipStream_t>(stream));
}
int bnn_bmm_panels(const uint32_t* Ap, const uint32_t* Bp, int32_t* C, int M, int N, int K, int ldc, void* stream) {
    if (!C) return BNN_ERR_INVALID_ARG;
    return bmm_panels_common(Ap, Bp, C, nullptr, nullptr, M, N, K, ldc, stream);
}
int bnn_bmm_thr_panels(const uint32_t* Ap, const uint32_t* Bp, const int32_t* thr, uint32_t* Cbits_p, int M, int N, int K,
                       void* stream) {
    if (!Cbits_p || !thr) return BNN_ERR_INVALID_ARG;
    return bmm_panels_common(Ap, Bp, nullptr, thr, Cbits_p, M, N, K, 0, stream);
}
int bnn_probe_load_stride(const uint32_t* zeros, int64_t* cycles, int stride_bytes, int rows, int iters, int dependent,
                          void* stream) {
    if (!zeros || !cycles || stride_bytes < 32 || (stride_bytes & 15) || rows < 32 || iters < 1) return BNN_ERR_INVALID_ARG;
    return launch_probe_stride(zeros, reinterpret_cast<long long*>(cycles), stride_bytes, rows, iters, dependent ? 1 : 0,
                               static_cast<hipStream_t>(stream));
}

int bnn_probe_pipeline(int which, void* buf, size_t buf_bytes, int iters, double* work_per_launch, void* stream) {
    if (!buf || !work_per_launch) return BNN_ERR_INVALID_ARG;
    if (reinterpret_cast<uintptr_t>(buf) & 255u) return BNN_ERR_ALIGNMENT;
    return launch_probe_pipeline(which, buf, buf_bytes, iters, work_per_launch, static_cast<hipStream_t>(stream));
}

int bnn_sign_pack_f32(const float* x, uint32_t* bits, int64_t rows, int cols, int ldx, int ldb_w, void* stream) {
    if (!x || !bits || rows < 1 || cols < 1 || ldx < cols || ldb_w < words(cols)) return BNN_ERR_INVALID_ARG;
    if (rows > (1LL << 33)) return BNN_ERR_UNSUPPORTED;
    return launch_sign_pack_f32(x, bits, rows, cols, ldx, ldb_w, static_cast<hipStream_t>(stream));
}

size_t bnn_bmm_general_workspace_bytes(int M, int N, int K) {
    if (M < 1 || N < 1 || K < 1 || K > BNN_MAX_K) return 0;
    const size_t ldw = (size_t)round4(words(K));
    return align256((size_t)M * ldw * 4) + align256((size_t)N * ldw * 4);
}
int bnn_bmm_general_f32(const float* A, const float* B, float* C, int M, int N, int K, int lda, int ldb, int ldc,
                        void* workspace, size_t workspace_bytes, void* stream) {
    if (!A || !B || !C || M < 1 || N < 1 || K < 1 || lda < K || ldb < K || ldc < N) return BNN_ERR_INVALID_ARG;
    if (K > BNN_MAX_K) return BNN_ERR_UNSUPPORTED;
    if (!workspace || workspace_bytes < bnn_bmm_general_workspace_bytes(M, N, K)) return BNN_ERR_WORKSPACE;
    if ((reinterpret_cast<uintptr_t>(workspace) & 255u) || !aligned16(C)) return BNN_ERR_ALIGNMENT;
    const int ldw = round4(words(K));
    uint32_t* Ab = static_cast<uint32_t*>(workspace);
    uint32_t* Bb = reinterpret_cast<uint32_t*>(static_cast<char*>(workspace) + align256((size_t)M * ldw * 4));
    hipStream_t s = static_cast<hipStream_t>(stream);
    int rc = launch_sign_pack_f32(A, Ab, M, K, lda, ldw, s);
    if (rc != BNN_OK) return rc;
    rc = launch_sign_pack_f32(B, Bb, N, K, ldb, ldw, s);
    if (rc != BNN_OK) return rc;
    return bmm_common(Ab, Bb, reinterpret_cast<int32_t*>(C), nullptr, nullptr, M, N, K, ldw, ldw, ldc, 0, BNN_PATH_AUTO, stream, true);
}

size_t bnn_bconv_general_workspace_bytes(int N, int H, int W, int C, int O, int k) {
    if (N < 1 || H < 1 || W < 1 || C < 1 || O < 1 || k < 1) return 0;
    const size_t cw = (size_t)words(C);
    return align256((size_t)N * H * W * cw * 4) + align256((size_t)O * k * k * cw * 4);
}
int bnn_bconv_general_f32(const float* in, const float* filt, float* out, int N, int H, int W, int C, int O, int k, int stride,
                          int pad, int pad_mode, void* workspace, size_t workspace_bytes, void* stream) {
    int P, Q;
    if (!in || !filt || !out) return BNN_ERR_INVALID_ARG;
    const int rc0 = conv_shape(N, H, W, C, O, k, stride, pad, pad_mode, &P, &Q);
    if (rc0 != BNN_OK) return rc0;
    if (!workspace || workspace_bytes < bnn_bconv_general_workspace_bytes(N, H, W, C, O, k)) return BNN_ERR_WORKSPACE;
    if ((reinterpret_cast<uintptr_t>(workspace) & 255u) || !aligned16(out)) return BNN_ERR_ALIGNMENT;
    const int cw = words(C);
    uint32_t* xb = static_cast<uint32_t*>(workspace);
    uint32_t* fb = reinterpret_cast<uint32_t*>(static_cast<char*>(workspace) + align256((size_t)N * H * W * cw * 4));
    hipStream_t s = static_cast<hipStream_t>(stream);
    int rc = launch_sign_pack_f32(in, xb, (long long)N * H * W, C, C, cw, s);
    if (rc != BNN_OK) return rc;
    rc = launch_sign_pack_f32(filt, fb, (long long)O * k * k, C, C, cw, s);
    if (rc != BNN_OK) return rc;
    return bconv_common(xb, fb, reinterpret_cast<int32_t*>(out), nullptr, nullptr, nullptr, N, H, W, C, O, k, stride, pad, pad_mode,
                        BNN_PATH_AUTO, stream, nullptr, nullptr, nullptr, 0, 0, 0, 1, false, true);
}

int bnn_unpack_i32(const uint32_t* bits, int32_t* out, int64_t rows, int cols, int ldb_w, int ldo, void* stream) {
    if (!bits || !out || rows < 1 || cols < 1 || ldb_w < words(cols) || ldo < cols) return BNN_ERR_INVALID_ARG;
    return launch_unpack_i32(bits, out, rows, cols, ldb_w, ldo, static_cast<hipStream_t>(stream));
}

int bnn_maxpool_or(const uint32_t* in, uint32_t* out, int N, int H, int W, int C, int win, int stride, void* stream) {
    if (!in || !out || N < 1 || H < 1 || W < 1 || C < 1 || win < 1 || stride < 1 || win > H || win > W)
        return BNN_ERR_INVALID_ARG;
    return launch_maxpool_or(in, out, N, H, W, C, win, stride, static_cast<hipStream_t>(stream));
}

int bnn_conv_f32_thr(const float* x, const float* w, const float* thr, float* y_f32, uint32_t* bits, int N, int H,
                     int W, int C, int O, int k, int stride, int pad, void* stream) {
    if (!x || !w || (!y_f32 && !bits) || (bits && !thr)) return BNN_ERR_INVALID_ARG;
    if (N < 1 || H < 1 || W < 1 || C < 1 || O < 1 || k < 1 || stride < 1 || pad < 0) return BNN_ERR_INVALID_ARG;
    if (H + 2 * pad < k || W + 2 * pad < k) return BNN_ERR_INVALID_ARG;
    return launch_conv_f32_thr(x, w, thr, y_f32, bits, N, H, W, C, O, k, stride, pad, static_cast<hipStream_t>(stream));
}
size_t bnn_conv_f32_split_workspace_bytes(int C, int O, int k) {
    if (C < 1 || O < 1 || k < 1 || (long long)k * C > (1 << 16)) return 0;
    return conv_f32_split_workspace_bytes(C, O, k);
}
int bnn_conv_f32_split_thr(const float* x, const float* w, const float* thr, float* y_f32, uint32_t* bits, int N, int H,
                           int W, int C, int O, int k, int stride, int pad, void* workspace, size_t workspace_bytes,
                           void* stream) {
    return bnn_conv_f32_split_thr_ex(x, w, thr, y_f32, bits, N, H, W, C, O, k, stride, pad, 9, workspace, workspace_bytes,
                                     stream);
}
int bnn_conv_f32_split_thr_ex(const float* x, const float* w, const float* thr, float* y_f32, uint32_t* bits, int N, int H,
                              int W, int C, int O, int k, int stride, int pad, int products, void* workspace,
                              size_t workspace_bytes, void* stream) {
    if (!x || !w || (!y_f32 && !bits) || (bits && !thr) || (products != 6 && products != 9)) return BNN_ERR_INVALID_ARG;
    if (N < 1 || H < 1 || W < 1 || C < 1 || O < 1 || k < 1 || stride < 1 || pad < 0) return BNN_ERR_INVALID_ARG;
    if (H + 2 * pad < k || W + 2 * pad < k) return BNN_ERR_INVALID_ARG;
    const long long P = (H + 2 * pad - k) / stride + 1, Q = (W + 2 * pad - k) / stride + 1;
    if ((long long)N * P * Q >= (1LL << 31) || (long long)k * C > (1 << 16) || (long long)W * C >= (1LL << 30))
        return BNN_ERR_UNSUPPORTED;
    if (!workspace) return BNN_ERR_WORKSPACE;
    if (!aligned16(workspace)) return BNN_ERR_ALIGNMENT;
    return launch_conv_f32_split_thr(x, w, thr, y_f32, bits, N, H, W, C, O, k, stride, pad, products, workspace,
                                     workspace_bytes, static_cast<hipStream_t>(stream));
}
size_t bnn_bwn_workspace_bytes(int C, int O, int k) {
    if (C < 1 || O < 1 || k < 1 || (long long)k * C > (1 << 16)) return 0;
    return bwn_workspace_bytes(C, O, k);
}
int bnn_bwn_conv_thr(const float* x, const uint32_t* wbits, const float* thr, float* y_f32, uint32_t* bits, int N, int H,
                     int W, int C, int O, int k, int stride, int pad, void* workspace, size_t workspace_bytes, void* stream) {
    if (!x || !wbits || (!y_f32 && !bits) || (bits && !thr)) return BNN_ERR_INVALID_ARG;
    if (N < 1 || H < 1 || W < 1 || C < 1 || O < 1 || k < 1 || stride < 1 || pad < 0) return BNN_ERR_INVALID_ARG;
    if (H + 2 * pad < k || W + 2 * pad < k) return BNN_ERR_INVALID_ARG;
    const long long P = (H + 2 * pad - k) / stride + 1, Q = (W + 2 * pad - k) / stride + 1;
    if ((long long)N * P * Q >= (1LL << 31) || (long long)k * C > (1 << 16) || (long long)W * C >= (1LL << 30))
        return BNN_ERR_UNSUPPORTED;
    if (!workspace) return BNN_ERR_WORKSPACE;
    if (!aligned16(workspace)) return BNN_ERR_ALIGNMENT;
    return launch_bwn_conv_thr(x, wbits, thr, y_f32, bits, N, H, W, C, O, k, stride, pad, workspace, workspace_bytes,
                               static_cast<hipStream_t>(stream));
}
int bnn_head_f32(const uint32_t* bits, const float* w, float* y, int32_t* pooled_out, int N, int HW, int C, int J,
                 void* stream) {
    if (!bits || !w || !y || N < 1 || HW < 1 || C < 1 || J < 1) return BNN_ERR_INVALID_ARG;
    return launch_head_f32(bits, w, y, pooled_out, N, HW, C, J, static_cast<hipStream_t>(stream));
}

// ---- layer-chained forward ------------------------------------------------------------------
int bnn_net_create(bnn_net** net) {
    if (!net) return BNN_ERR_INVALID_ARG;
    *net = new (std::nothrow) bnn_net();
    return *net ? BNN_OK : BNN_ERR_INVALID_ARG;
}
int bnn_net_destroy(bnn_net* net) {
    delete net;
    return BNN_OK;
}
int bnn_net_input_u8(bnn_net* net, int cols, int thr) {
    if (!net || cols < 1 || !net->layers.empty()) return BNN_ERR_INVALID_ARG;
    bnn_net::Layer L; L.kind = bnn_net::IN_U8; L.a = cols; L.thr_u8 = thr;
    net->layers.push_back(L);
    return BNN_OK;
}
int bnn_net_input_bits(bnn_net* net, int cols) {
    if (!net || cols < 1 || !net->layers.empty()) return BNN_ERR_INVALID_ARG;
    bnn_net::Layer L; L.kind = bnn_net::IN_BITS; L.a = cols;
    net->layers.push_back(L);
    return BNN_OK;
}
int bnn_net_input_conv_f32(bnn_net* net, const float* w, const float* thr, int H, int W, int C, int O, int k,
                           int stride, int pad) {
    if (!net || !w || !thr || !net->layers.empty()) return BNN_ERR_INVALID_ARG;
    if (H < 1 || W < 1 || C < 1 || O < 1 || k < 1 || stride < 1 || pad < 0 || H + 2 * pad < k || W + 2 * pad < k)
        return BNN_ERR_INVALID_ARG;
    bnn_net::Layer L; L.kind = bnn_net::IN_CONV_F32; L.w0 = w; L.t0 = thr;
    L.a = H; L.b = W; L.c = C; L.d = O; L.k = k; L.stride = stride; L.pad = pad;
    net->layers.push_back(L);
    return BNN_OK;
}
int bnn_net_input_bwn_f32(bnn_net* net, const uint32_t* wbits, const float* thr, int H, int W, int C, int O, int k,
                          int stride, int pad) {
    const int rc = bnn_net_input_conv_f32(net, reinterpret_cast<const float*>(wbits), thr, H, W, C, O, k, stride, pad);
    if (rc == BNN_OK) net->layers.back().bwn = true;
    return rc;
}
int bnn_net_add_fc(bnn_net* net, const uint32_t* W, const int32_t* thr, int K, int N) {
    if (!net || !W || K < 1 || N < 1 || net->layers.empty()) return BNN_ERR_INVALID_ARG;
    if (K > BNN_MAX_K) return BNN_ERR_UNSUPPORTED;
    if (!aligned16(W) || (thr && !aligned16(thr))) return BNN_ERR_ALIGNMENT;
    bnn_net::Layer L; L.kind = bnn_net::FC; L.w0 = W; L.t0 = thr; L.a = K; L.b = N;
    net->layers.push_back(L);
    return BNN_OK;
}
int bnn_net_add_conv(bnn_net* net, const uint32_t* filt, const int32_t* thr, int C, int O, int k, int stride, int pad,
                     int pad_mode) {
    if (!net || !filt || !thr || net->layers.empty()) return BNN_ERR_INVALID_ARG;
    int P, Q;
    int rc = conv_shape(1, k, k, C, O, k, stride, pad, pad_mode, &P, &Q);
    if (rc != BNN_OK) return rc;
    if (!aligned16(filt) || !aligned16(thr)) return BNN_ERR_ALIGNMENT;
    bnn_net::Layer L; L.kind = bnn_net::CONV; L.w0 = filt; L.t0 = thr; L.a = C; L.b = O; L.k = k; L.stride = stride;
    L.pad = pad; L.pad_mode = pad_mode;
    net->layers.push_back(L);
    return BNN_OK;
}
int bnn_net_add_pool(bnn_net* net, int win, int stride) {
    if (!net || win < 1 || stride < 1 || net->layers.empty()) return BNN_ERR_INVALID_ARG;
    bnn_net::Layer L; L.kind = bnn_net::POOL; L.k = win; L.stride = stride;
    net->layers.push_back(L);
    return BNN_OK;
}
int bnn_net_add_block(bnn_net* net, const uint32_t* W1, const int32_t* thr1, const uint32_t* W2, const int32_t* thr2,
                      const uint32_t* Wd, int cin, int cout, int stride, int pad_mode) {
    if (!net || !W1 || !thr1 || !W2 || !thr2 || net->layers.empty()) return BNN_ERR_INVALID_ARG;
    if (cin < 1 || cout < 1 || stride < 1) return BNN_ERR_INVALID_ARG;
    if (pad_mode != BNN_PAD_MINUS_ONE && pad_mode != BNN_PAD_EXCLUDE) return BNN_ERR_INVALID_ARG;
    if (!Wd && (stride != 1 || cin != cout)) return BNN_ERR_INVALID_ARG;
    if (!aligned16(W1) || !aligned16(W2) || !aligned16(thr1) || !aligned16(thr2) || (Wd && !aligned16(Wd)))
        return BNN_ERR_ALIGNMENT;
    bnn_net::Layer L; L.kind = bnn_net::BLOCK; L.w0 = W1; L.t0 = thr1; L.w1 = W2; L.t1 = thr2; L.w2 = Wd;
    L.a = cin; L.b = cout; L.stride = stride; L.pad_mode = pad_mode;
    net->layers.push_back(L);
    return BNN_OK;
}
int bnn_net_add_head_f32(bnn_net* net, const float* w, int J) {
    if (!net || !w || J < 1 || net->layers.empty()) return BNN_ERR_INVALID_ARG;
    bnn_net::Layer L; L.kind = bnn_net::HEAD; L.w0 = w; L.a = J;
    net->layers.push_back(L);
    return BNN_OK;
}

int bnn_net_workspace_bytes(const bnn_net* net, int batch, size_t* bytes) {
    if (!net || !bytes || batch < 1 || net->layers.empty()) return BNN_ERR_INVALID_ARG;
    Plan pl = plan(const_cast<bnn_net*>(net), batch);
    if (pl.rc != BNN_OK) return pl.rc;
    *bytes = pl.total;
    return BNN_OK;
}

namespace {

// State of a persistent forward: the run of layers collected so far and how to launch it.
struct PersistCtx {
    bnn_net* net;
    char* ws;
    const Plan* pl;
    int sync, spin_limit, max_grid;
    hipStream_t stream;
    PersistNet pn = {};
    std::vector<PersistLayer> segment;
    size_t table_used = 0;          // entries of the table region already taken by earlier runs of this forward
    std::vector<PersistLayer> table; // what the table region holds after this forward

    int flush() {
        if (segment.empty() && pn.in_u8 == nullptr) return BNN_OK;
        if (table_used + segment.size() > (size_t)PERSIST_MAX_LAYERS) return BNN_ERR_UNSUPPORTED;
        PersistLayer* dev = reinterpret_cast<PersistLayer*>(ws + pl->table_off) + table_used;
        // upload the run's layer table unless the same bytes are already there (repeated forwards of one net)
        const bool same = net->persist_uploaded_at == ws + pl->table_off &&
                          net->persist_uploaded.size() >= table_used + segment.size() &&
                          (segment.empty() || memcmp(net->persist_uploaded.data() + table_used, segment.data(),
                                                     segment.size() * sizeof(PersistLayer)) == 0);
        if (!same && !segment.empty()) {
            if (hipMemcpyAsync(dev, segment.data(), segment.size() * sizeof(PersistLayer), hipMemcpyHostToDevice, stream) !=
                hipSuccess)
                return BNN_ERR_DEVICE;
            if (hipStreamSynchronize(stream) != hipSuccess) return BNN_ERR_DEVICE;   // the host copy may go away
        }
        int max_tiles = 1;
        for (const PersistLayer& P : segment) max_tiles = std::max(max_tiles, P.gx * P.gy);
        pn.nlayers = (int)segment.size();
        pn.layers = dev;
        const int rc = launch_persist_chain(pn, max_tiles, max_grid, reinterpret_cast<unsigned*>(ws + pl->sync_off), sync,
                                            spin_limit, stream);
        table.insert(table.end(), segment.begin(), segment.end());
        table_used += segment.size();
        segment.clear();
        pn = PersistNet{};
        return rc;
    }
};

int forward_impl(bnn_net* net, const void* input, void* output, int batch, char* ws, const Plan& pl, int path, void* stream,
                 PersistCtx* pc) {
    const uint32_t* cur = nullptr;      // bits of the current activation
    int curH = 1, curW = 1, curC = 0, cur_ld = 0;
    int32_t* R = nullptr;               // running int32 residual (same shape as cur), or null
    int rslot = 0;
    for (size_t i = 0; i < net->layers.size(); ++i) {
        const bnn_net::Layer& L = net->layers[i];
        uint32_t* obits = reinterpret_cast<uint32_t*>(ws + L.bits_off);
        int rc = BNN_OK;
        // persistent forward: contractions are collected (dispatch() records them while capture_sink is set) and run
        // as one kernel per unbroken run of FC / CONV / BLOCK layers; every other layer first lets that kernel go
        const bool contraction = L.kind == bnn_net::FC || L.kind == bnn_net::CONV || L.kind == bnn_net::BLOCK;
        if (pc != nullptr) {
            if (!contraction && !(i == 0 && L.kind == bnn_net::IN_U8)) {
                rc = pc->flush();
                if (rc != BNN_OK) return rc;
            }
            capture_sink = contraction ? &pc->segment : nullptr;
        }
        switch (L.kind) {
            case bnn_net::IN_U8:
                if (pc != nullptr) {                 // done inside the persistent kernel, ahead of its first layer
                    pc->pn.in_u8 = static_cast<const uint8_t*>(input); pc->pn.in_bits = obits;
                    pc->pn.in_rows = batch; pc->pn.in_cols = L.a; pc->pn.in_thr = L.thr_u8; pc->pn.in_ldw = L.words_per_row;
                    break;
                }
                rc = bnn_pack_u8(static_cast<const uint8_t*>(input), L.thr_u8, obits, batch, L.a, L.words_per_row, stream);
                break;
            case bnn_net::IN_BITS:
                if (!aligned16(input)) return BNN_ERR_ALIGNMENT;
                obits = const_cast<uint32_t*>(static_cast<const uint32_t*>(input));   // used in place
                break;
            case bnn_net::IN_CONV_F32:
                rc = L.bwn ? bnn_bwn_conv_thr(static_cast<const float*>(input), static_cast<const uint32_t*>(L.w0),
                                              static_cast<const float*>(L.t0), nullptr, obits, batch, L.a, L.b, L.c, L.d, L.k,
                                              L.stride, L.pad, ws + pl.bwn_off, pl.bwn_bytes, stream)
                           : bnn_conv_f32_split_thr_ex(static_cast<const float*>(input), static_cast<const float*>(L.w0),
                                                       static_cast<const float*>(L.t0), nullptr, obits, batch, L.a, L.b, L.c,
                                                       L.d, L.k, L.stride, L.pad, 6, ws + pl.bwn_off, pl.bwn_bytes, stream);
                if (!L.bwn && rc == BNN_ERR_UNSUPPORTED)       // filter bank too large for the split kernel
                    rc = bnn_conv_f32_thr(static_cast<const float*>(input), static_cast<const float*>(L.w0),
                                          static_cast<const float*>(L.t0), nullptr, obits, batch, L.a, L.b, L.c, L.d, L.k,
                                          L.stride, L.pad, stream);
                R = nullptr;
                break;
            case bnn_net::FC: {
                const long long K = (long long)curH * curW * curC;
                // a [batch][H][W][cw] tensor with C a multiple of 32 is already a [batch][K/32] matrix
                const int lda = (curH * curW == 1) ? cur_ld : curH * curW * cur_ld;
                if (L.t0) {
                    rc = bnn_bmm_thr_ex(cur, static_cast<const uint32_t*>(L.w0), static_cast<const int32_t*>(L.t0), obits,
                                        batch, L.b, (int)K, lda, round4(words((int)K)), L.words_per_row, path, stream);
                } else {
                    if (!output) return BNN_ERR_INVALID_ARG;
                    rc = bnn_bmm_ex(cur, static_cast<const uint32_t*>(L.w0), static_cast<int32_t*>(output), batch, L.b,
                                    (int)K, lda, round4(words((int)K)), L.b, path, stream);
                }
                R = nullptr;
                break;
            }
            case bnn_net::CONV:
                rc = bnn_bconv_thr_ex(cur, static_cast<const uint32_t*>(L.w0), nullptr, nullptr,
                                      static_cast<const int32_t*>(L.t0), obits, batch, curH, curW, curC, L.b, L.k,
                                      L.stride, L.pad, L.pad_mode, path, stream);
                R = nullptr;
                break;
            case bnn_net::POOL:
                rc = bnn_maxpool_or(cur, obits, batch, curH, curW, curC, L.k, L.stride, stream);
                R = nullptr;
                break;
            case bnn_net::BLOCK: {
                uint32_t* hbits = obits;                                     // first half of the slot
                uint32_t* ybits = obits + align256((size_t)batch * L.H * L.W * L.words_per_row * 4) / 4;
                int32_t* Rnew = reinterpret_cast<int32_t*>(ws + pl.resid_off[(rslot + 1) % 3]);
                // the block's sum is kept only if the next layer is a block that adds it back
                const bool keep_sum = (i + 1 < net->layers.size()) && net->layers[i + 1].kind == bnn_net::BLOCK &&
                                      net->layers[i + 1].w2 == nullptr;
                const int32_t* shortcut = nullptr;
                const uint32_t* shortcut_bits = nullptr;
                const uint32_t* x2 = nullptr;
                if (L.w2) {     // 1x1 binarized downsample of the block input: fused into the second conv
                    x2 = cur;
                } else if (R) {
                    shortcut = R;
                } else {        // first block of a chain: the residual is the +1/-1 values of its input bits
                    shortcut_bits = cur;
                }
                rc = bnn_bconv_thr_ex(cur, static_cast<const uint32_t*>(L.w0), nullptr, nullptr,
                                      static_cast<const int32_t*>(L.t0), hbits, batch, curH, curW, curC, L.b, 3,
                                      L.stride, 1, L.pad_mode, path, stream);
                if (rc != BNN_OK) { capture_sink = nullptr; return rc; }
                rc = bconv_common(hbits, static_cast<const uint32_t*>(L.w1), keep_sum ? Rnew : nullptr, shortcut,
                                  static_cast<const int32_t*>(L.t1), ybits, batch, L.H, L.W, L.b, L.b, 3, 1, 1,
                                  L.pad_mode, path, stream, shortcut_bits, x2, static_cast<const uint32_t*>(L.w2), curH, curW,
                                  curC, L.stride, pl.sums16);
                R = keep_sum ? Rnew : nullptr; rslot = (rslot + 1) % 3;
                obits = ybits;
                break;
            }
            case bnn_net::HEAD:
                if (!output) return BNN_ERR_INVALID_ARG;
                rc = bnn_head_f32(cur, static_cast<const float*>(L.w0), static_cast<float*>(output),
                                  reinterpret_cast<int32_t*>(ws + pl.pool_off), batch,
                                  curH * curW, curC, L.a, stream);
                break;
        }
        capture_sink = nullptr;
        if (rc != BNN_OK) return rc;
        cur = obits; curH = L.H; curW = L.W; curC = L.C; cur_ld = L.words_per_row;
    }
    if (pc != nullptr) return pc->flush();
    return BNN_OK;
}

}  // namespace

int bnn_net_forward(bnn_net* net, const void* input, void* output, int batch, void* workspace, size_t workspace_bytes,
                    int path, void* stream) {
    if (!net || !input || batch < 1 || net->layers.empty()) return BNN_ERR_INVALID_ARG;
    Plan pl = plan(net, batch);
    if (pl.rc != BNN_OK) return pl.rc;
    if (pl.total > 0 && (!workspace || workspace_bytes < pl.total)) return BNN_ERR_WORKSPACE;
    if (reinterpret_cast<uintptr_t>(workspace) & 255u) return BNN_ERR_ALIGNMENT;
    char* ws = static_cast<char*>(workspace);
    net->last_ws = ws; net->last_batch = batch;
    return forward_impl(net, input, output, batch, ws, pl, path, stream, nullptr);
}

int bnn_net_forward_persistent(bnn_net* net, const void* input, void* output, int batch, void* workspace,
                               size_t workspace_bytes, int flags, void* stream) {
    if (!net || !input || !output || batch < 1 || net->layers.size() < 2) return BNN_ERR_INVALID_ARG;
    const int grid_cap = (flags >> 8) & 0xFFFF;
    if (flags & ~(BNN_PERSIST_NO_SYNC | BNN_PERSIST_GIVE_UP_AT_ONCE | (0xFFFF << 8))) return BNN_ERR_INVALID_ARG;
    bool any_contraction = false, any_conv = false;
    for (size_t i = 0; i < net->layers.size(); ++i) {
        const bnn_net::Kind kd = net->layers[i].kind;
        if (kd == bnn_net::FC || kd == bnn_net::CONV || kd == bnn_net::BLOCK) any_contraction = true;
        if (kd == bnn_net::CONV || kd == bnn_net::BLOCK) any_conv = true;
    }
    if (!any_contraction) return BNN_ERR_UNSUPPORTED;
    Plan pl = plan(net, batch);
    if (pl.rc != BNN_OK) return pl.rc;
    if (!workspace || workspace_bytes < pl.total) return BNN_ERR_WORKSPACE;
    if (reinterpret_cast<uintptr_t>(workspace) & 255u) return BNN_ERR_ALIGNMENT;
    char* ws = static_cast<char*>(workspace);
    net->last_ws = ws; net->last_batch = batch;

    PersistCtx pc;
    pc.net = net; pc.ws = ws; pc.pl = &pl;
    pc.sync = (flags & BNN_PERSIST_NO_SYNC) ? 0 : 1;
    // a waiter polls about once a microsecond: 2^17 polls are a few tenths of a second
    pc.spin_limit = (flags & BNN_PERSIST_GIVE_UP_AT_ONCE) ? 0 : (1 << 17);
    // a device-wide barrier costs more the more workgroups meet at it (measured: about 2 us with 16, 18 us with
    // 256); a convolution chain has many layers with few tiles each, so its grid is kept small unless the caller
    // asks otherwise
    pc.max_grid = grid_cap > 0 ? grid_cap : (any_conv ? 128 : (1 << 20));
    pc.stream = static_cast<hipStream_t>(stream);
    net->last_persist_sync = reinterpret_cast<const unsigned*>(ws + pl.sync_off);
    const int rc = forward_impl(net, input, output, batch, ws, pl, BNN_PATH_MFMA, stream, &pc);
    capture_sink = nullptr;
    if (rc == BNN_OK) {
        net->persist_uploaded = pc.table;
        net->persist_uploaded_at = ws + pl.table_off;
    } else {
        net->persist_uploaded.clear();
        net->persist_uploaded_at = nullptr;
    }
    return rc;
}

int bnn_net_persistent_status(bnn_net* net, int* aborted, void* stream) {
    if (!net || !aborted) return BNN_ERR_INVALID_ARG;
    if (!net->last_persist_sync) return BNN_ERR_WORKSPACE;          // no persistent forward has been enqueued
    unsigned flag = 0u;
    hipStream_t s = static_cast<hipStream_t>(stream);
    if (hipMemcpyAsync(&flag, net->last_persist_sync + 1, sizeof(flag), hipMemcpyDeviceToHost, s) != hipSuccess)
        return BNN_ERR_DEVICE;
    if (hipStreamSynchronize(s) != hipSuccess) return BNN_ERR_DEVICE;
    *aborted = flag != 0u ? 1 : 0;
    return BNN_OK;
}

// ---- forward for callers that cannot allocate -----------------------------------------------
// The workspace of bnn_net_forward_static: one fixed array per GPU in the library's code object (every GPU the
// library runs on holds its own copy, at its own address, until the process ends).  In host code `scratch` is
// only a handle for hipGetSymbolAddress; the device address is looked up once per device and kept here.
static __device__ __align__(256) unsigned char scratch[BNN_STATIC_WORKSPACE_BYTES];

namespace {
constexpr int kMaxDevices = 64;
std::mutex scratch_mutex;
void* scratch_ptr[kMaxDevices] = {};

int static_workspace(void** out) {
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess) return BNN_ERR_DEVICE;
    if (dev < 0 || dev >= kMaxDevices) return BNN_ERR_UNSUPPORTED;
    std::lock_guard<std::mutex> lock(scratch_mutex);
    if (scratch_ptr[dev] == nullptr) {
        void* p = nullptr;
        if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || p == nullptr) return BNN_ERR_DEVICE;
        scratch_ptr[dev] = p;
    }
    *out = scratch_ptr[dev];
    return BNN_OK;
}
}  // namespace

int bnn_static_workspace_init(void) {
    void* p = nullptr;
    return static_workspace(&p);
}

int bnn_net_forward_static(bnn_net* net, const void* input, void* output, int batch, int path, void* stream) {
    if (!net || !input || batch < 1 || net->layers.empty()) return BNN_ERR_INVALID_ARG;
    Plan pl = plan(net, batch);
    if (pl.rc != BNN_OK) return pl.rc;
    if (pl.total > (size_t)BNN_STATIC_WORKSPACE_BYTES) return BNN_ERR_WORKSPACE;   // this net at this batch needs more
    void* ws = nullptr;
    const int rc = static_workspace(&ws);
    if (rc != BNN_OK) return rc;
    return bnn_net_forward(net, input, output, batch, ws, (size_t)BNN_STATIC_WORKSPACE_BYTES, path, stream);
}

int bnn_net_layer_bits(const bnn_net* net, int layer, const uint32_t** bits, int64_t* rows, int* words_per_row) {
    if (!net || !bits || !rows || !words_per_row || layer < 0 || layer >= (int)net->layers.size()) return BNN_ERR_INVALID_ARG;
    if (!net->last_ws) return BNN_ERR_WORKSPACE;
    const bnn_net::Layer& L = net->layers[layer];
    if (L.kind == bnn_net::HEAD || L.kind == bnn_net::IN_BITS || (L.kind == bnn_net::FC && !L.t0)) return BNN_ERR_INVALID_ARG;
    const uint32_t* p = reinterpret_cast<const uint32_t*>(net->last_ws + L.bits_off);
    const long long r = (long long)net->last_batch * L.H * L.W;
    if (L.kind == bnn_net::BLOCK) p += align256((size_t)r * L.words_per_row * 4) / 4;    // the block's output bits
    *bits = p; *rows = r; *words_per_row = L.words_per_row;
    return BNN_OK;
}

}  // extern "C"
