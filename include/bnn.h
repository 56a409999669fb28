/*
 * bnn.h -- C ABI of libbnn: binarized fully-connected and convolution layers on packed +1/-1
 * bits for AMD MI355X (gfx950), after "Accelerating Binarized Neural Networks via
 * Bit-Tensor-Cores in Turing GPUs" (arXiv 2006.16578).
 *
 * Conventions common to every call
 * --------------------------------
 *  - Bits: bit 1 denotes +1, bit 0 denotes -1 (Sec. 5.2, text of Eq. 2).  Element k of a packed
 *    vector is bit (k % 32), counted from the least significant bit, of 32-bit word (k / 32).
 *    Rows of packed matrices are `ld*_w` words apart.  Bits beyond the logical length of a row
 *    ("pad bits"), up to the next multiple of 128 bits, MUST be 0 in every input; every output
 *    this library writes has its pad bits, up to the leading dimension, written as 0.
 *  - Pointers: every data pointer is a DEVICE pointer owned by the caller.  The library never
 *    allocates, frees or synchronises; a call only enqueues kernels on `stream`
 *    (a hipStream_t passed as void*; NULL is the default stream) and returns.
 *    Inputs must not overlap outputs.
 *  - Alignment: packed-bit and int32 base pointers must be 16-byte aligned, leading dimensions of
 *    packed BMM operands (`lda_w`, `ldb_w`) must be multiples of 4 words.
 *  - Return value: BNN_OK or a negative bnn_status; nothing is enqueued when an error is returned
 *    (except BNN_ERR_DEVICE, which reports a failed launch).  No exceptions, no global state.
 *  - Exactness: all binarized arithmetic is integer and exact.  K (or k*k*C for a convolution)
 *    must not exceed BNN_MAX_K.
 */
#ifndef BNN_H
#define BNN_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum bnn_status {
    BNN_OK = 0,
    BNN_ERR_INVALID_ARG = -1,   /* null pointer, non-positive size, window larger than padded image ... */
    BNN_ERR_ALIGNMENT = -2,     /* pointer not 16-byte aligned or leading dimension not a multiple of 4 words */
    BNN_ERR_UNSUPPORTED = -3,   /* valid request outside what the kernels implement (e.g. K > BNN_MAX_K) */
    BNN_ERR_DEVICE = -4,        /* the HIP runtime reported a launch failure */
    BNN_ERR_WORKSPACE = -5      /* workspace too small / missing */
} bnn_status;

/* How an out-of-frame input position enters a convolution (Sec. 5.3). */
#define BNN_PAD_MINUS_ONE 0  /* it counts as -1 (a 0 bit) */
#define BNN_PAD_EXCLUDE 1    /* its taps contribute nothing: the paper's "exclude" amendment */

/* Which arithmetic pipeline computes the +1/-1 products.  CDNA4 has no 1-bit matrix type, so the
 * library has two: XOR + popcount on the vector ALUs (Eq. 2 literally), and the matrix cores fed
 * with +1/-1 expanded on the fly to 4-bit floats (exact: products are +-1, sums stay below 2^24).
 * BNN_PATH_AUTO takes the matrix cores (the faster pipeline for every shape measured) and falls back to the
 * vector-ALU kernel for operands beyond the matrix-core kernels' 32-bit addressing range. */
#define BNN_PATH_AUTO 0
#define BNN_PATH_VALU 1
#define BNN_PATH_MFMA 2

#define BNN_MAX_K (1 << 20)

const char* bnn_status_string(int status);
int bnn_version(void);
/* Name of the kernel variant (path and wave tile) the library launches for a BMM / BConv of this
 * shape, for profiles and reports; a static string, "invalid" for shapes the calls reject. */
const char* bnn_bmm_kernel_name(int M, int N, int K, int path);
const char* bnn_bconv_kernel_name(int N, int H, int W, int C, int O, int k, int stride, int pad, int path);
/* The same for a given output: the two calls above describe the fused threshold -> bits calls
 * (BNN_OUT_BITS); with BNN_OUT_INT32 they describe bnn_bmm / bnn_bconv, whose full-precision output
 * can make the library choose a smaller wave tile. */
#define BNN_OUT_BITS 0
#define BNN_OUT_INT32 1
const char* bnn_bmm_kernel_name_out(int M, int N, int K, int path, int out_kind);
const char* bnn_bconv_kernel_name_out(int N, int H, int W, int C, int O, int k, int stride, int pad, int path,
                                      int out_kind);

/* ------------------------------------------------------------------------------------------
 * BMM (Sec. 5.2, Eq. 2): C[i][j] = sum_{k<K} a[i][k] * b[j][k] = K - 2 * popc(A_i xor B_j).
 *   A  [M][lda_w]  packed along K (row-major bit matrix)
 *   B  [N][ldb_w]  packed along K (the column-major K x N operand of Sec. 3.3: N rows of K bits)
 *   C  [M][ldc]    int32
 * M, N, K >= 1; lda_w, ldb_w >= ceil(K/32) rounded up to a multiple of 4; ldc >= N.
 * ---------------------------------------------------------------------------------------- */
int bnn_bmm(const uint32_t* A, const uint32_t* B, int32_t* C,
            int M, int N, int K, int lda_w, int ldb_w, int ldc, void* stream);
int bnn_bmm_ex(const uint32_t* A, const uint32_t* B, int32_t* C,
               int M, int N, int K, int lda_w, int ldb_w, int ldc, int path, void* stream);

/* BMM with the threshold of Sec. 6.1 applied in the epilogue, so that the int32 matrix is never
 * stored (the bit-in / bit-out form of Sec. 5.2): Cbits[i] bit j = (C[i][j] >= thr[j]).
 *   thr   [N] int32;  Cbits [M][ldcb_w], ldcb_w >= ceil(N/32); pad bits up to ldcb_w*32 are 0,
 *   so Cbits is directly the A operand of the next layer. */
int bnn_bmm_thr(const uint32_t* A, const uint32_t* B, const int32_t* thr, uint32_t* Cbits,
                int M, int N, int K, int lda_w, int ldb_w, int ldcb_w, void* stream);
int bnn_bmm_thr_ex(const uint32_t* A, const uint32_t* B, const int32_t* thr, uint32_t* Cbits,
                   int M, int N, int K, int lda_w, int ldb_w, int ldcb_w, int path, void* stream);

/* ------------------------------------------------------------------------------------------
 * BConv (Sec. 5.3, Eq. 3): cross-correlation, no filter flip,
 *   out[n][p][q][o] = sum_{r,s<k} sum_{c<C} x(n, p*stride-pad+r, q*stride-pad+s, c) * f[o][r][s][c]
 *   in    [N][H][W][cw]   packed along C, cw = ceil(C/32), pixels contiguous (NHWC)
 *   filt  [O][k][k][cw]   packed along C
 *   out   [N][P][Q][O]    int32,  P = (H + 2*pad - k)/stride + 1, Q likewise
 * pad_mode says what an out-of-frame x is (see BNN_PAD_*).  k*k*C <= BNN_MAX_K, k <= 32, pad < k.
 * The images that 512 consecutive output pixels touch must hold less than 2 GiB of packed input
 * ((511 / (P*Q) + 2) * H*W*cw*4 bytes), else BNN_ERR_UNSUPPORTED on the matrix-core path.
 * ---------------------------------------------------------------------------------------- */
int bnn_bconv(const uint32_t* in, const uint32_t* filt, int32_t* out,
              int N, int H, int W, int C, int O, int k, int stride, int pad, int pad_mode, void* stream);
int bnn_bconv_ex(const uint32_t* in, const uint32_t* filt, int32_t* out,
                 int N, int H, int W, int C, int O, int k, int stride, int pad, int pad_mode,
                 int path, void* stream);

/* BConv with fused epilogue: S = conv + residual_in (if given); sum_out = S (if given);
 * out_bits bit o = (S >= thr[o]).  The residual is the full-precision shortcut of Sec. 6.1 kept
 * as int32 and added before the threshold.
 *   residual_in [N][P][Q][O] int32 or NULL;  sum_out [N][P][Q][O] int32 or NULL (may alias
 *   residual_in: each element is read then written by the same thread);
 *   thr [O] int32;  out_bits [N][P][Q][ow], ow = ceil(O/32), pad bits 0. */
int bnn_bconv_thr(const uint32_t* in, const uint32_t* filt,
                  const int32_t* residual_in, int32_t* sum_out,
                  const int32_t* thr, uint32_t* out_bits,
                  int N, int H, int W, int C, int O, int k, int stride, int pad, int pad_mode, void* stream);
int bnn_bconv_thr_ex(const uint32_t* in, const uint32_t* filt,
                     const int32_t* residual_in, int32_t* sum_out,
                     const int32_t* thr, uint32_t* out_bits,
                     int N, int H, int W, int C, int O, int k, int stride, int pad, int pad_mode,
                     int path, void* stream);

/* ------------------------------------------------------------------------------------------
 * Stand-alone threshold and (un)packing (Sec. 6.1 thrd; Eq. 1 with sign(0) = +1).
 * ---------------------------------------------------------------------------------------- */
/* bits[r] bit c = (X[r][c] >= thr[c]);  X [rows][ldx] int32, bits [rows][ldb_w]. */
int bnn_threshold_pack(const int32_t* X, const int32_t* thr, uint32_t* bits,
                       int64_t rows, int cols, int ldx, int ldb_w, void* stream);
/* bits[r] bit c = (x[r][c] >= thr);  x [rows][cols] uint8 (8-bit input pixels). */
int bnn_pack_u8(const uint8_t* x, int thr, uint32_t* bits, int64_t rows, int cols, int ldb_w, void* stream);
/* bits[r] bit c = (x[r][c] >= thr[c]);  x [rows][cols] fp32, thr [cols] fp32. */
int bnn_pack_f32(const float* x, const float* thr, uint32_t* bits, int64_t rows, int cols, int ldb_w, void* stream);
/* Pre-tiled weight operand, in the spirit of the paper's FSB format (Sec. 5.1: store the operand in the order the
 * matrix unit's tile loads consume it), with this chip's tile: rows are grouped by 32, and a group stores, for
 * every 16-byte step along K, the 16 bytes of its 32 rows back to back, so that the 32 lanes of an MFMA fragment
 * load read 512 contiguous bytes.  16-byte unit u of row r moves to unit ((r/32) * (ldb_w/4) + u) * 32 + r % 32.
 *   bnn_tile_b: B [N][ldb_w] -> B_tiled, ceil(N/32)*32 * ldb_w words (rows past N are zeros); ldb_w % 4 == 0.
 *   bnn_bmm_tiled / bnn_bmm_thr_tiled: as bnn_bmm / bnn_bmm_thr with B given in that format (matrix-core path,
 *   operands read straight from L2 without LDS staging). */
int bnn_tile_b(const uint32_t* B, uint32_t* B_tiled, int N, int K, int ldb_w, void* stream);
int bnn_bmm_tiled(const uint32_t* A, const uint32_t* B_tiled, int32_t* C, int M, int N, int K,
                  int lda_w, int ldb_w, int ldc, void* stream);
int bnn_bmm_thr_tiled(const uint32_t* A, const uint32_t* B_tiled, const int32_t* thr, uint32_t* Cbits, int M, int N, int K,
                      int lda_w, int ldb_w, int ldcb_w, void* stream);
/* K-panel operand layout for large products: the fixed-stride idea of the paper's format (Sec. 5.1: a storage order in
 * which every tile load walks memory with one small constant stride) with this chip's sizes.  K is cut into panels of
 * 256 bits and panel p stores its 8 words of every row back to back: word w of row r sits at word
 * ((w / 8) * rows + r) * 8 + w % 8.  A matrix of `rows` rows and K bits takes ceil(K / 256) * rows * 8 words; the bits
 * past K in the last panel are 0.  A 16-byte load per lane then covers whole 128-byte lines (a slab of 256 bits of
 * 32 rows is 1 KB of contiguous memory), where the row-major layout gives a load instruction 32 bytes in each of 32
 * lines; the large-product kernel runs 6 % faster on it.
 *   bnn_panels_from_rows: X [rows][ldx_w] -> Xp (ldx_w >= ceil(K/32); bits past K in X are ignored).
 *   bnn_rows_from_panels: Xp -> X [rows][ldx_w] (ldx_w >= ceil(K/32), ldx_w % 4 == 0; words past the panels are zeroed).
 *   bnn_bmm_panels:      C [M][ldc] int32 = A x B^T as bnn_bmm (Eq. 2), A and B given in panels (M resp. N rows).
 *   bnn_bmm_thr_panels:  the fused threshold of bnn_bmm_thr; the output bits are written IN PANELS
 *                        (ceil(N / 256) * M * 8 words, bits past N are 0): the operand A of the next product.
 * All pointers device, 16-byte aligned.  Matrix-core path, 256 x 256 tiles: meant for products of thousands of rows and
 * columns (any shape is computed correctly).  rows < 2^31. */
int bnn_panels_from_rows(const uint32_t* X, uint32_t* Xp, int64_t rows, int K, int ldx_w, void* stream);
int bnn_rows_from_panels(const uint32_t* Xp, uint32_t* X, int64_t rows, int K, int ldx_w, void* stream);
int bnn_bmm_panels(const uint32_t* Ap, const uint32_t* Bp, int32_t* C, int M, int N, int K, int ldc, void* stream);
int bnn_bmm_thr_panels(const uint32_t* Ap, const uint32_t* Bp, const int32_t* thr, uint32_t* Cbits_p, int M, int N, int K,
                       void* stream);
/* Diagnostic, after the load-latency microbenchmark of Sec. 4.1: ONE wave loads `iters` MFMA operand fragments
 * (lane l: 16 bytes of row l % 32 at byte 16 * (l / 32)) from a zero-filled buffer of `rows` rows that are
 * `stride_bytes` apart (multiple of 16, >= 32; the buffer holds rows * stride_bytes bytes), walking along the rows.
 * dependent != 0 chains every address on the previous load (latency), 0 issues them back to back.
 * cycles[0] receives the elapsed ticks of the shader cycle counter, cycles[1] is scratch. */
int bnn_probe_load_stride(const uint32_t* zeros, int64_t* cycles, int stride_bytes, int rows, int iters, int dependent,
                          void* stream);

/* Diagnostic, after the method of Sec. 4 (measure the machine's ceilings by microbenchmark and design against
 * those): ONE kernel that keeps a single pipeline busy, operands resident in registers where the pipeline allows.
 * The caller times the launch (events on `stream`) and divides *work_per_launch by the elapsed time.
 *   which                        work unit   what runs
 *   BNN_PROBE_MFMA_FP4           flop        v_mfma_f32_32x32x64_f8f6f4 on E2M1 operands alone (8 accumulators per wave)
 *   BNN_PROBE_MFMA_FP4_EXPAND    flop        the BMM kernel's inner loop without memory: per K-step 6 packed words
 *                                            expanded to E2M1 (7 vector-ALU instructions each) feeding 8 MFMAs
 *   BNN_PROBE_MFMA_I8            op          v_mfma_i32_32x32x32_i8 alone (the +1/-1-as-int8 alternative)
 *   BNN_PROBE_MFMA_BF16          flop        v_mfma_f32_32x32x16_bf16 alone (first layer with real-valued input)
 *   BNN_PROBE_VALU_XOR_POPC      binary op   v_xor_b32 + v_bcnt_u32_b32 (Eq. 2 literally), 2 ops per bit product
 *   BNN_PROBE_LDS_READ           byte        ds_read_b128, conflict-free
 *   BNN_PROBE_HBM_READ / _WRITE  byte        streams buf with 16-byte accesses (use a buffer larger than the caches)
 *   BNN_PROBE_HBM_COPY           byte        first half of buf -> second half; counts bytes read + written
 * buf: device scratch, 256-byte aligned; the compute and LDS probes write one word per thread into it (at least
 * 2 MiB), the memory probes stream all buf_bytes of it.  iters: loop trips per wave (compute and LDS probes).
 * 2 workgroups of 256 threads per compute unit (compute, LDS), 8 per compute unit (memory). */
#define BNN_PROBE_MFMA_FP4 0
#define BNN_PROBE_MFMA_FP4_EXPAND 1
#define BNN_PROBE_MFMA_I8 2
#define BNN_PROBE_MFMA_BF16 3
#define BNN_PROBE_VALU_XOR_POPC 4
#define BNN_PROBE_LDS_READ 5
#define BNN_PROBE_HBM_READ 6
#define BNN_PROBE_HBM_WRITE 7
#define BNN_PROBE_HBM_COPY 8
int bnn_probe_pipeline(int which, void* buf, size_t buf_bytes, int iters, double* work_per_launch, void* stream);

/* Binarization by sign (Eq. 1): bit = (x >= 0).  x [rows][ldx] fp32 -> bits [rows][ldb_w] (pad bits and pad words 0). */
int bnn_sign_pack_f32(const float* x, uint32_t* bits, int64_t rows, int cols, int ldx, int ldb_w, void* stream);

/* The "general" forms of Sec. 7.2 / 7.3: real-valued operands in, real-valued result out.  Both operands are
 * binarized by sign (Eq. 1) into the caller's workspace, multiplied as +1/-1 values (Eq. 2 / Eq. 3), and the
 * integer sums are stored as fp32 (exact: every sum is below 2^24).
 *   BMM:   A [M][lda], B [N][ldb] (the K x N operand stored column by column), C [M][ldc] fp32.
 *   BConv: in [N][H][W][C], filt [O][k][k][C], out [N][P][Q][O] fp32; padding as in bnn_bconv.
 *   workspace: device scratch of at least bnn_*_general_workspace_bytes(...) bytes, 256-byte aligned; it holds the
 *   packed operands and is not needed after the call.  C / out 16-byte aligned. */
size_t bnn_bmm_general_workspace_bytes(int M, int N, int K);
int bnn_bmm_general_f32(const float* A, const float* B, float* C, int M, int N, int K, int lda, int ldb, int ldc,
                        void* workspace, size_t workspace_bytes, void* stream);
size_t bnn_bconv_general_workspace_bytes(int N, int H, int W, int C, int O, int k);
int bnn_bconv_general_f32(const float* in, const float* filt, float* out, int N, int H, int W, int C, int O, int k,
                          int stride, int pad, int pad_mode, void* workspace, size_t workspace_bytes, void* stream);

/* out[r][c] = +1 / -1 as int32 from bits [rows][ldb_w]; out [rows][ldo] (e.g. to seed an int32
 * residual tensor from a bit tensor). */
int bnn_unpack_i32(const uint32_t* bits, int32_t* out, int64_t rows, int cols, int ldb_w, int ldo, void* stream);

/* Max-pooling of packed +1/-1 activations: behind the threshold the maximum over a window is the
 * bitwise OR of the packed words (Sec. 6.1).  in [N][H][W][cw] -> out [N][P][Q][cw],
 * P = (H - win)/stride + 1, Q likewise (no padding; partial windows are dropped).  win <= H, W. */
int bnn_maxpool_or(const uint32_t* in, uint32_t* out, int N, int H, int W, int C, int win, int stride, void* stream);

/* ------------------------------------------------------------------------------------------
 * Full-precision end layers of a network whose inner layers are binarized (Sec. 6.1: the first
 * layer keeps full-precision input).  fp32 arithmetic, not bit-exact: 1e-4 relative.
 * ---------------------------------------------------------------------------------------- */
/* y = conv(x, w) with zero padding; bits = (y >= thr[o]).
 *   x [N][H][W][C] fp32, w [O][k][k][C] fp32, thr [O] fp32,
 *   y_f32 [N][P][Q][O] fp32 or NULL, bits [N][P][Q][ceil(O/32)] or NULL (not both NULL). */
int bnn_conv_f32_thr(const float* x, const float* w, const float* thr, float* y_f32, uint32_t* bits,
                     int N, int H, int W, int C, int O, int k, int stride, int pad, void* stream);
/* The same layer on the bf16 matrix cores: every input value and every weight is split exactly into three bf16
 * terms and all nine term products are accumulated in fp32, so each product x*w is exact and only the fp32
 * additions round (at least as accurate as an fp32 multiply-add chain; same 1e-4 contract).  Needs
 *   workspace: device scratch of at least bnn_conv_f32_split_workspace_bytes(C, O, k) bytes, 16-byte aligned
 *   (it receives the split weights in matrix-core operand order; not needed after the call);
 * N*P*Q < 2^31; finite inputs.  BNN_ERR_UNSUPPORTED when the split filter bank of 64 output channels does not
 * fit LDS (k*ceil(k*C/8) above about 50): use bnn_conv_f32_thr then. */
size_t bnn_conv_f32_split_workspace_bytes(int C, int O, int k);
int bnn_conv_f32_split_thr(const float* x, const float* w, const float* thr, float* y_f32, uint32_t* bits,
                           int N, int H, int W, int C, int O, int k, int stride, int pad,
                           void* workspace, size_t workspace_bytes, void* stream);
/* products = 9: as above.  products = 6: without the three smallest term products (middle x low, low x middle,
 * low x low), which together are below 2^-23 of x*w: each product is then as accurate as one rounded to fp32, for
 * two thirds of the matrix work.  The layer chain (bnn_net_forward) uses 6. */
int bnn_conv_f32_split_thr_ex(const float* x, const float* w, const float* thr, float* y_f32, uint32_t* bits,
                              int N, int H, int W, int C, int O, int k, int stride, int pad, int products,
                              void* workspace, size_t workspace_bytes, void* stream);
/* First layer with binarized weights only (Sec. 6.1, "BWN"): the input stays real-valued, each weight is one
 * bit that decides whether the input element is added (bit 1) or subtracted (bit 0); zero padding;
 * bits = (y >= thr[o]).  fp32 accumulation (every product is exact), 1e-4 relative like the layer above.
 *   x [N][H][W][C] fp32 (finite values), wbits [O][k][k][ceil(C/32)] packed along C (pad bits 0), thr [O] fp32,
 *   y_f32 [N][P][Q][O] fp32 or NULL, bits [N][P][Q][ceil(O/32)] or NULL (not both NULL).
 *   workspace: device scratch of at least bnn_bwn_workspace_bytes(C, O, k) bytes, 16-byte aligned (it receives
 *   the weights expanded to bf16 in matrix-core operand order; contents are not needed after the call).
 *   N*P*Q < 2^31.  k*ceil(k*C/8) above about 80 (64 output channels: 160) does not fit LDS: BNN_ERR_UNSUPPORTED. */
size_t bnn_bwn_workspace_bytes(int C, int O, int k);
int bnn_bwn_conv_thr(const float* x, const uint32_t* wbits, const float* thr, float* y_f32, uint32_t* bits,
                     int N, int H, int W, int C, int O, int k, int stride, int pad,
                     void* workspace, size_t workspace_bytes, void* stream);
/* pooled[n][c] = sum over HW positions of the +1/-1 value of channel c (exact integer);
 * y[n][j] = sum_c (pooled[n][c] / HW) * w[j][c].
 *   bits [N][HW][ceil(C/32)], w [J][C] fp32, y [N][J] fp32, pooled_out [N][C] int32 or NULL.
 *   HW <= 255 and C <= 1024, else BNN_ERR_UNSUPPORTED.  With pooled_out the call runs as two kernels (pooling once
 *   per image, then the FC on the pooled sums), which is the faster form for more than a few images. */
int bnn_head_f32(const uint32_t* bits, const float* w, float* y, int32_t* pooled_out,
                 int N, int HW, int C, int J, void* stream);

/* ------------------------------------------------------------------------------------------
 * Layer-chained forward (Sec. 6.1 order thrd -> bconv/bmm -> thrd ...; Sec. 6.2).  A net is a
 * host-side list of layers; bnn_net_forward enqueues one fused kernel per layer on `stream`,
 * the packed output bits of a layer being directly the operand of the next.
 * Weight and threshold pointers are device pointers BORROWED for the lifetime of the net.
 * The net object itself is host memory owned by the library (create/destroy).
 * ---------------------------------------------------------------------------------------- */
typedef struct bnn_net bnn_net;

int bnn_net_create(bnn_net** net);
int bnn_net_destroy(bnn_net* net);
/* Input layers (exactly one, first). */
int bnn_net_input_u8(bnn_net* net, int cols, int thr);                       /* [batch][cols] uint8 -> bits */
int bnn_net_input_bits(bnn_net* net, int cols);                             /* [batch][ld_w] packed bits, ld_w = ceil(cols/32) rounded up to 4 */
int bnn_net_input_conv_f32(bnn_net* net, const float* w, const float* thr, /* [batch][H][W][C] fp32 -> stem conv -> bits */
                           int H, int W, int C, int O, int k, int stride, int pad);
int bnn_net_input_bwn_f32(bnn_net* net, const uint32_t* wbits, const float* thr, /* same, weights as bits (bnn_bwn_conv_thr) */
                          int H, int W, int C, int O, int k, int stride, int pad);
/* Binarized fully-connected layer, W [N][ldw_w] with ldw_w = ceil(K/32) rounded up to 4.
 * thr != NULL: output bits; thr == NULL: int32 scores [batch][N] (only as the last layer). */
int bnn_net_add_fc(bnn_net* net, const uint32_t* W, const int32_t* thr, int K, int N);
/* Binarized convolution + threshold. */
int bnn_net_add_conv(bnn_net* net, const uint32_t* filt, const int32_t* thr,
                     int C, int O, int k, int stride, int pad, int pad_mode);
/* Max-pooling (OR) of the current packed activation. */
int bnn_net_add_pool(bnn_net* net, int win, int stride);
/* Residual basic block: h = thr1(conv3x3(x, W1, stride, pad 1)); S = conv3x3(h, W2, 1, pad 1) + shortcut;
 * y = (S >= thr2); the running residual becomes S.  shortcut = running residual when Wd == NULL
 * (needs stride 1, cin == cout; the first such block of a chain uses the +1/-1 values of its input
 * bits), else conv1x1(x, Wd [cout][1][1][ceil(cin/32)], stride, pad 0), which is computed inside the
 * second convolution's kernel as extra terms of the same sums. */
int bnn_net_add_block(bnn_net* net, const uint32_t* W1, const int32_t* thr1,
                      const uint32_t* W2, const int32_t* thr2, const uint32_t* Wd,
                      int cin, int cout, int stride, int pad_mode);
/* Head: sum-pool over all positions + fp32 FC, w [J][C]; output fp32 [batch][J]. */
int bnn_net_add_head_f32(bnn_net* net, const float* w, int J);
/* Device workspace the forward needs for `batch` inputs (activations, residuals). */
int bnn_net_workspace_bytes(const bnn_net* net, int batch, size_t* bytes);
/* input: as declared by the input layer; output: int32 scores or fp32 logits of the last layer.
 * workspace: device memory of at least bnn_net_workspace_bytes(), 256-byte aligned. */
int bnn_net_forward(bnn_net* net, const void* input, void* output, int batch,
                    void* workspace, size_t workspace_bytes, int path, void* stream);
/* bnn_net_forward for callers that cannot allocate device memory -- code under HIP graph capture, tight serving
 * loops, harnesses that forbid hipMalloc: the workspace is a fixed buffer of BNN_STATIC_WORKSPACE_BYTES that
 * lives in the library's code object, one copy per GPU, held until the process ends.  The call (and
 * bnn_static_workspace_init) calls no hipMalloc / hipFree or other allocating routine; inputs, output and weights
 * are still the caller's.  Same kernels, arguments and results as bnn_net_forward.
 *   BNN_ERR_WORKSPACE when bnn_net_workspace_bytes(net, batch) exceeds BNN_STATIC_WORKSPACE_BYTES (nothing is
 *   enqueued): e.g. the 784-1024-1024-1024-10 MLP fits up to batch 65536, the ResNet-18-shaped network up to batch 12.
 * Every call on a GPU uses that GPU's one buffer, which keeps the previous call's contents (nothing in it needs
 * clearing: each forward writes what it reads): calls that OVERLAP on one GPU -- two streams, two threads -- race;
 * calls on one stream are ordered and safe.  bnn_net_layer_bits afterwards points into that buffer.
 * bnn_static_workspace_init looks up the buffer's address for the current device; call it once per device at
 * set-up (outside any graph capture).  bnn_net_forward_static does the same on its first call on a device if
 * it has not been done. */
#define BNN_STATIC_WORKSPACE_BYTES (32u << 20)
int bnn_static_workspace_init(void);
int bnn_net_forward_static(bnn_net* net, const void* input, void* output, int batch, int path, void* stream);
/* The same forward with every unbroken run of fully-connected layers, 3x3 convolutions and residual blocks as ONE
 * kernel launch (Sec. 6.2: every layer a device function of one kernel, a device-wide barrier between layers).
 * An MLP (u8 or bits input, FC layers) is one launch in all; a ResNet-shaped net runs its first layer and its head
 * as the ordinary kernels and all blocks in one launch between them; a pooling layer ends a run.  Supported inside
 * a run: FC layers, and 3x3 convolutions (also those of residual blocks, any stride, both paddings) of 64, 128, 256
 * or 512 input channels; at most 48 such layers per forward; anything else returns BNN_ERR_UNSUPPORTED (use
 * bnn_net_forward).  Same arguments, workspace and results as bnn_net_forward.  The layer table of a run travels
 * through the workspace: the first forward of a net at a given batch and workspace uploads it and WAITS for the
 * stream once; later forwards with the same arguments enqueue only.  The grid never exceeds what the device holds at
 * once; a barrier that is not reached by all workgroups within a few tenths of a second (other work holding the
 * compute units) makes every workgroup leave the kernel: the output is then undefined and
 * bnn_net_persistent_status reports it.  Calls that overlap on one device must use different workspaces.
 * flags: 0, or a combination of
 *   BNN_PERSIST_NO_SYNC          skip the barriers -- the results are then UNDEFINED; it exists only to measure
 *                                what the barriers cost;
 *   BNN_PERSIST_GIVE_UP_AT_ONCE  a workgroup that finds a barrier not yet complete gives up at its first poll
 *                                (every workgroup still leaves the kernel normally) -- results UNDEFINED; it
 *                                exists to exercise the time-out path and its status report;
 *   BNN_PERSIST_GRID_CAP(n)      at most n workgroups (1 .. 65535; a barrier costs more the more workgroups meet at
 *                                it).  Default: 128 for nets with convolutions, the device's capacity otherwise. */
#define BNN_PERSIST_NO_SYNC 1
#define BNN_PERSIST_GIVE_UP_AT_ONCE 2
#define BNN_PERSIST_GRID_CAP(n) (((n) & 0xFFFF) << 8)
int bnn_net_forward_persistent(bnn_net* net, const void* input, void* output, int batch,
                               void* workspace, size_t workspace_bytes, int flags, void* stream);
/* Whether the LAST bnn_net_forward_persistent of this net gave up at a barrier: *aborted = 1 (its output is
 * undefined), else 0.  `stream` must be the stream of that forward, its workspace must still be allocated.
 * This is the one call of the library that waits for the device (it synchronises `stream`).
 * BNN_ERR_WORKSPACE when the net has not run a persistent forward. */
int bnn_net_persistent_status(bnn_net* net, int* aborted, void* stream);
/* After a forward: device pointer (inside the workspace) and shape of the packed bits produced by
 * layer `layer` (0 = input layer), for layer-by-layer checking.  words_per_row receives the row
 * length in words, rows the number of rows (batch, or batch*P*Q). */
int bnn_net_layer_bits(const bnn_net* net, int layer, const uint32_t** bits, int64_t* rows, int* words_per_row);

#ifdef __cplusplus
}
#endif
#endif /* BNN_H */
