/*
 * bnn_oracle.c -- CPU oracle for the binarized FC / convolution path (BTC-BNN paper).
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, plain statement of what the GPU library
 * must compute.  It shares no code, header, table or helper with the HIP path, and nothing in
 * the product path may call it: only tests/, __graft_entry__.smoke() and bench.py's
 * cpu_baseline leg load it.
 *
 * Two tiers:
 *   tier 0 ("orc_*")  -- the definition itself: operands are unpacked to +1/-1 held as int8
 *                        and multiplied in naive nested loops.  No xor, no popcount.
 *   tier 1 ("orc1_*") -- the method's formula, Eq. 2 of the paper: n - 2*popc(a xor b) on
 *                        packed 64-bit chunks.  It exists only so that full-size outputs can be
 *                        produced in reasonable time; tests require it to equal tier 0 wherever
 *                        tier 0 runs.
 *
 * Bit convention (paper Sec. 5.2, text around Eq. 2: bit 1 denotes +1, bit 0 denotes -1).
 * Element k of a packed vector lives in word k/32 at bit k%32 counted from the least
 * significant bit (the paper does not fix an in-word order; LSB-first is this build's reading).
 * Pad bits (beyond the logical length, up to the leading dimension) are required to be 0 in
 * inputs and are written as 0 in outputs.
 *
 * Every function returns 0 on success, 1 on allocation failure, 2 on a bad argument.
 * Every function here is pinned by tests/test_oracle_*.py (brute force, closed forms,
 * worked examples, numpy / torch library cross-checks): none is "parity unpinned".
 */
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

/* ---------------------------------------------------------------------------------------
 * O1. unpack: value(k) = +1 if bit k is set else -1            (Sec. 5.2, Eq. 1 and Eq. 2)
 * ------------------------------------------------------------------------------------- */
static inline int bit_at(const uint32_t* row, int64_t k) {
    return (int)((row[k >> 5] >> (k & 31)) & 1u);
}

/* bits [rows][ldw] -> out [rows][cols] of int8 in {+1,-1} */
int orc_unpack_pm1(const uint32_t* bits, int64_t rows, int64_t cols, int64_t ldw, int8_t* out) {
    if (!bits || !out || rows < 0 || cols < 0 || ldw * 32 < cols) return 2;
    for (int64_t r = 0; r < rows; ++r)
        for (int64_t k = 0; k < cols; ++k)
            out[r * cols + k] = bit_at(bits + r * ldw, k) ? 1 : -1;
    return 0;
}

/* ---------------------------------------------------------------------------------------
 * O2. BMM: C[i][j] = sum_k a[i][k] * b[j][k] over +1/-1 values.
 * This is the plain dot product that Eq. 2 rewrites as n - 2*popc(a xor b).  B is given as N
 * rows of K bits, i.e. the column-major K x N operand of Sec. 3.3.
 * ------------------------------------------------------------------------------------- */
int orc_bmm(const uint32_t* A, const uint32_t* B, int32_t* C,
            int64_t M, int64_t N, int64_t K, int64_t lda_w, int64_t ldb_w, int64_t ldc) {
    if (!A || !B || !C || M < 0 || N < 0 || K < 0 || ldc < N) return 2;
    int8_t* a = (int8_t*)malloc((size_t)(M * K + 1));
    int8_t* b = (int8_t*)malloc((size_t)(N * K + 1));
    if (!a || !b) { free(a); free(b); return 1; }
    int rc = orc_unpack_pm1(A, M, K, lda_w, a);
    if (!rc) rc = orc_unpack_pm1(B, N, K, ldb_w, b);
    if (rc) { free(a); free(b); return rc; }
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < M; ++i)
        for (int64_t j = 0; j < N; ++j) {
            int32_t s = 0;
            for (int64_t k = 0; k < K; ++k) s += (int32_t)a[i * K + k] * (int32_t)b[j * K + k];
            C[i * ldc + j] = s;
        }
    free(a); free(b);
    return 0;
}

/* A slab of rows [row0, row0+rows) of the same product, for sampled checks at sizes where the
 * full tier-0 product would take too long.  C_slab is [rows][N] with leading dimension N. */
int orc_bmm_rows(const uint32_t* A, const uint32_t* B, int32_t* C_slab,
                 int64_t row0, int64_t rows, int64_t N, int64_t K, int64_t lda_w, int64_t ldb_w) {
    if (row0 < 0 || rows < 0) return 2;
    return orc_bmm(A + row0 * lda_w, B, C_slab, rows, N, K, lda_w, ldb_w, N);
}

/* ---------------------------------------------------------------------------------------
 * O3. BConv: cross-correlation (no filter flip, Sec. 5.3) of an NHWC +1/-1 image with
 * O filters of k x k x C:
 *   out[n][p][q][o] = sum_{r,s,c} x(n, p*stride-pad+r, q*stride-pad+s, c) * f[o][r][s][c]
 * An out-of-frame x is -1 when pad_mode == 0 (the benchmark configuration's convention) and
 * contributes nothing (x = 0) when pad_mode == 1, which is what the paper's "exclude"
 * amendment in Sec. 5.3 (C*KH*KW - exclude*C - 2*acc) evaluates to.
 * in [N][H][W][cw], filt [O][k][k][cw], cw = ceil(C/32); out [N][P][Q][O] int32.
 * ------------------------------------------------------------------------------------- */
int orc_bconv(const uint32_t* in, const uint32_t* filt, int32_t* out,
              int64_t N, int64_t H, int64_t W, int64_t C, int64_t O,
              int64_t k, int64_t stride, int64_t pad, int pad_mode) {
    if (!in || !filt || !out || N < 0 || H <= 0 || W <= 0 || C <= 0 || O <= 0 || k <= 0 ||
        stride <= 0 || pad < 0 || (pad_mode != 0 && pad_mode != 1)) return 2;
    if (H + 2 * pad < k || W + 2 * pad < k) return 2;
    const int64_t cw = (C + 31) / 32;
    const int64_t P = (H + 2 * pad - k) / stride + 1;
    const int64_t Q = (W + 2 * pad - k) / stride + 1;
    int8_t* x = (int8_t*)malloc((size_t)(N * H * W * C + 1));
    int8_t* f = (int8_t*)malloc((size_t)(O * k * k * C + 1));
    if (!x || !f) { free(x); free(f); return 1; }
    int rc = orc_unpack_pm1(in, N * H * W, C, cw, x);
    if (!rc) rc = orc_unpack_pm1(filt, O * k * k, C, cw, f);
    if (rc) { free(x); free(f); return rc; }
    const int oob = (pad_mode == 0) ? -1 : 0;
#pragma omp parallel for collapse(2) schedule(static)
    for (int64_t n = 0; n < N; ++n)
        for (int64_t p = 0; p < P; ++p)
            for (int64_t q = 0; q < Q; ++q)
                for (int64_t o = 0; o < O; ++o) {
                    int32_t s = 0;
                    for (int64_t r = 0; r < k; ++r)
                        for (int64_t t = 0; t < k; ++t) {
                            const int64_t y = p * stride - pad + r;
                            const int64_t xx = q * stride - pad + t;
                            const int inside = (y >= 0 && y < H && xx >= 0 && xx < W);
                            const int8_t* fv = f + ((o * k + r) * k + t) * C;
                            if (inside) {
                                const int8_t* xv = x + ((n * H + y) * W + xx) * C;
                                for (int64_t c = 0; c < C; ++c) s += (int32_t)xv[c] * (int32_t)fv[c];
                            } else {
                                for (int64_t c = 0; c < C; ++c) s += oob * (int32_t)fv[c];
                            }
                        }
                    out[((n * P + p) * Q + q) * O + o] = s;
                }
    free(x); free(f);
    return 0;
}

/* The same convolution for images [n0, n0+n_cnt) only; out_slab is [n_cnt][P][Q][O]. */
int orc_bconv_images(const uint32_t* in, const uint32_t* filt, int32_t* out_slab,
                     int64_t n0, int64_t n_cnt, int64_t H, int64_t W, int64_t C, int64_t O,
                     int64_t k, int64_t stride, int64_t pad, int pad_mode) {
    if (n0 < 0 || n_cnt < 0) return 2;
    const int64_t cw = (C + 31) / 32;
    return orc_bconv(in + n0 * H * W * cw, filt, out_slab, n_cnt, H, W, C, O, k, stride, pad, pad_mode);
}

/* ---------------------------------------------------------------------------------------
 * O4. threshold: bit = (v >= tau[col]), i.e. the sign of v - tau under Eq. 1 (x >= 0 -> +1);
 * batch-norm followed by the next layer's sign collapses to this comparison (Sec. 6.1).
 * X [rows][ldx] int32, tau [cols] -> bits [rows][ldb_w], pad bits 0.
 * ------------------------------------------------------------------------------------- */
int orc_threshold_pack(const int32_t* X, const int32_t* tau, uint32_t* bits,
                       int64_t rows, int64_t cols, int64_t ldx, int64_t ldb_w) {
    if (!X || !tau || !bits || rows < 0 || cols < 0 || ldx < cols || ldb_w * 32 < cols) return 2;
    for (int64_t r = 0; r < rows; ++r) {
        uint32_t* w = bits + r * ldb_w;
        for (int64_t i = 0; i < ldb_w; ++i) w[i] = 0u;
        for (int64_t c = 0; c < cols; ++c)
            if (X[r * ldx + c] >= tau[c]) w[c >> 5] |= (1u << (c & 31));
    }
    return 0;
}

/* 8-bit pixels to bits with one scalar threshold: bit = (pixel >= thr)   (Eq. 1 on x - thr) */
int orc_pack_u8(const uint8_t* x, int thr, uint32_t* bits, int64_t rows, int64_t cols, int64_t ldb_w) {
    if (!x || !bits || rows < 0 || cols < 0 || ldb_w * 32 < cols) return 2;
    for (int64_t r = 0; r < rows; ++r) {
        uint32_t* w = bits + r * ldb_w;
        for (int64_t i = 0; i < ldb_w; ++i) w[i] = 0u;
        for (int64_t c = 0; c < cols; ++c)
            if ((int)x[r * cols + c] >= thr) w[c >> 5] |= (1u << (c & 31));
    }
    return 0;
}

/* fp32 values to bits with a per-column fp32 threshold: bit = (x >= tau[col]) */
int orc_pack_f32(const float* x, const float* tau, uint32_t* bits, int64_t rows, int64_t cols, int64_t ldb_w) {
    if (!x || !tau || !bits || rows < 0 || cols < 0 || ldb_w * 32 < cols) return 2;
    for (int64_t r = 0; r < rows; ++r) {
        uint32_t* w = bits + r * ldb_w;
        for (int64_t i = 0; i < ldb_w; ++i) w[i] = 0u;
        for (int64_t c = 0; c < cols; ++c)
            if (x[r * cols + c] >= tau[c]) w[c >> 5] |= (1u << (c & 31));
    }
    return 0;
}

/* ---------------------------------------------------------------------------------------
 * Max-pooling of +1/-1 activations (Sec. 6.1: for inference the pooling is moved behind the
 * threshold, where the maximum of +1/-1 values is the logical OR of their bits).  Here it is the
 * definition: the maximum over the window of the unpacked values, then re-packed.
 * in [N][H][W][cw] -> out [N][P][Q][cw], P = (H - win)/stride + 1 (no padding, partial windows dropped).
 * ------------------------------------------------------------------------------------- */
int orc_maxpool_pm1(const uint32_t* in, uint32_t* out, int64_t N, int64_t H, int64_t W, int64_t C,
                    int64_t win, int64_t stride) {
    if (!in || !out || N < 0 || H <= 0 || W <= 0 || C <= 0 || win <= 0 || stride <= 0 || H < win || W < win) return 2;
    const int64_t cw = (C + 31) / 32;
    const int64_t P = (H - win) / stride + 1, Q = (W - win) / stride + 1;
    for (int64_t n = 0; n < N; ++n)
        for (int64_t p = 0; p < P; ++p)
            for (int64_t q = 0; q < Q; ++q) {
                uint32_t* o = out + ((n * P + p) * Q + q) * cw;
                for (int64_t i = 0; i < cw; ++i) o[i] = 0u;
                for (int64_t c = 0; c < C; ++c) {
                    int best = -1;
                    for (int64_t r = 0; r < win; ++r)
                        for (int64_t t = 0; t < win; ++t) {
                            const int v = bit_at(in + ((n * H + p * stride + r) * W + q * stride + t) * cw, c) ? 1 : -1;
                            if (v > best) best = v;
                        }
                    if (best > 0) o[c >> 5] |= (1u << (c & 31));
                }
            }
    return 0;
}

/* ---------------------------------------------------------------------------------------
 * Full-precision first and last layers of the ResNet-18-shaped network (Sec. 6.1: the first
 * layer is not binarized).  Accumulated in double, rounded to fp32 once.
 * ------------------------------------------------------------------------------------- */

/* x [N][H][W][C] fp32 (zero padding), w [O][k][k][C] fp32 -> y [N][P][Q][O] fp32 */
int orc_conv_f32(const float* x, const float* w, float* y,
                 int64_t N, int64_t H, int64_t W, int64_t C, int64_t O,
                 int64_t k, int64_t stride, int64_t pad) {
    if (!x || !w || !y || N < 0 || H <= 0 || W <= 0 || C <= 0 || O <= 0 || k <= 0 || stride <= 0 || pad < 0) return 2;
    const int64_t P = (H + 2 * pad - k) / stride + 1;
    const int64_t Q = (W + 2 * pad - k) / stride + 1;
#pragma omp parallel for collapse(2) schedule(static)
    for (int64_t n = 0; n < N; ++n)
        for (int64_t p = 0; p < P; ++p)
            for (int64_t q = 0; q < Q; ++q)
                for (int64_t o = 0; o < O; ++o) {
                    double s = 0.0;
                    for (int64_t r = 0; r < k; ++r)
                        for (int64_t t = 0; t < k; ++t) {
                            const int64_t yy = p * stride - pad + r;
                            const int64_t xx = q * stride - pad + t;
                            if (yy < 0 || yy >= H || xx < 0 || xx >= W) continue;
                            const float* xv = x + ((n * H + yy) * W + xx) * C;
                            const float* wv = w + ((o * k + r) * k + t) * C;
                            for (int64_t c = 0; c < C; ++c) s += (double)xv[c] * (double)wv[c];
                        }
                    y[((n * P + p) * Q + q) * O + o] = (float)s;
                }
    return 0;
}

/* First layer with binarized weights only (Sec. 6.1, "BWN"): the input stays real-valued, every weight
 * is one bit, and the bit decides whether the input element is added (bit 1, +1) or subtracted (bit 0,
 * -1).  x [N][H][W][C] fp32, out-of-frame positions contribute nothing (zero padding of a real-valued
 * image); wbits [O][k][k][cw] packed along C; y [N][P][Q][O] fp32, accumulated in double. */
int orc_bwn_conv_f32(const float* x, const uint32_t* wbits, float* y,
                     int64_t N, int64_t H, int64_t W, int64_t C, int64_t O,
                     int64_t k, int64_t stride, int64_t pad) {
    if (!x || !wbits || !y || N < 0 || H <= 0 || W <= 0 || C <= 0 || O <= 0 || k <= 0 || stride <= 0 || pad < 0) return 2;
    const int64_t P = (H + 2 * pad - k) / stride + 1;
    const int64_t Q = (W + 2 * pad - k) / stride + 1;
    const int64_t cw = (C + 31) / 32;
#pragma omp parallel for collapse(2) schedule(static)
    for (int64_t n = 0; n < N; ++n)
        for (int64_t p = 0; p < P; ++p)
            for (int64_t q = 0; q < Q; ++q)
                for (int64_t o = 0; o < O; ++o) {
                    double s = 0.0;
                    for (int64_t r = 0; r < k; ++r)
                        for (int64_t t = 0; t < k; ++t) {
                            const int64_t yy = p * stride - pad + r;
                            const int64_t xx = q * stride - pad + t;
                            if (yy < 0 || yy >= H || xx < 0 || xx >= W) continue;
                            const float* xv = x + ((n * H + yy) * W + xx) * C;
                            const uint32_t* wv = wbits + ((o * k + r) * k + t) * cw;
                            for (int64_t c = 0; c < C; ++c) {
                                if (bit_at(wv, c)) s += (double)xv[c];
                                else s -= (double)xv[c];
                            }
                        }
                    y[((n * P + p) * Q + q) * O + o] = (float)s;
                }
    return 0;
}

/* Sum of +1/-1 over the HW positions of each channel: bits [N][HW][cw] -> pooled [N][C] int32 */
int orc_sumpool_pm1(const uint32_t* bits, int32_t* pooled, int64_t N, int64_t HW, int64_t C) {
    if (!bits || !pooled || N < 0 || HW <= 0 || C <= 0) return 2;
    const int64_t cw = (C + 31) / 32;
    for (int64_t n = 0; n < N; ++n)
        for (int64_t c = 0; c < C; ++c) {
            int32_t s = 0;
            for (int64_t i = 0; i < HW; ++i) s += bit_at(bits + (n * HW + i) * cw, c) ? 1 : -1;
            pooled[n * C + c] = s;
        }
    return 0;
}

/* y[n][j] = sum_c (pooled[n][c] / div) * w[j][c]; the division is one fp32 operation per
 * element (as the GPU head does), the dot product is accumulated in double. */
int orc_head_fc_f32(const int32_t* pooled, const float* w, float* y,
                    int64_t N, int64_t C, int64_t J, float div) {
    if (!pooled || !w || !y || N < 0 || C <= 0 || J <= 0 || div == 0.0f) return 2;
#pragma omp parallel for schedule(static)
    for (int64_t n = 0; n < N; ++n)
        for (int64_t j = 0; j < J; ++j) {
            double s = 0.0;
            for (int64_t c = 0; c < C; ++c) {
                const float a = (float)pooled[n * C + c] / div;
                s += (double)a * (double)w[j * C + c];
            }
            y[n * J + j] = (float)s;
        }
    return 0;
}

/* =======================================================================================
 * Tier 1: Eq. 2 on packed words, v = n - 2*popc(a xor b).  Pad bits are 0 in both operands,
 * so they xor to 0 and the true n is used.  Scalar C, 64 bits at a time.
 * ===================================================================================== */
static inline int64_t xor_popc_row(const uint32_t* a, const uint32_t* b, int64_t nwords) {
    int64_t acc = 0;
    int64_t w = 0;
    for (; w + 2 <= nwords; w += 2) {
        uint64_t x, y;
        memcpy(&x, a + w, 8);
        memcpy(&y, b + w, 8);
        acc += __builtin_popcountll(x ^ y);
    }
    if (w < nwords) acc += __builtin_popcount(a[w] ^ b[w]);
    return acc;
}

int orc1_bmm(const uint32_t* A, const uint32_t* B, int32_t* C,
             int64_t M, int64_t N, int64_t K, int64_t lda_w, int64_t ldb_w, int64_t ldc) {
    if (!A || !B || !C || M < 0 || N < 0 || K < 0 || ldc < N) return 2;
    const int64_t kw = (K + 31) / 32;
    if (lda_w < kw || ldb_w < kw) return 2;
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < M; ++i)
        for (int64_t j = 0; j < N; ++j)
            C[i * ldc + j] = (int32_t)(K - 2 * xor_popc_row(A + i * lda_w, B + j * ldb_w, kw));
    return 0;
}

int orc1_bconv(const uint32_t* in, const uint32_t* filt, int32_t* out,
               int64_t N, int64_t H, int64_t W, int64_t C, int64_t O,
               int64_t k, int64_t stride, int64_t pad, int pad_mode) {
    if (!in || !filt || !out || N < 0 || H <= 0 || W <= 0 || C <= 0 || O <= 0 || k <= 0 ||
        stride <= 0 || pad < 0 || (pad_mode != 0 && pad_mode != 1)) return 2;
    if (H + 2 * pad < k || W + 2 * pad < k) return 2;
    const int64_t cw = (C + 31) / 32;
    const int64_t P = (H + 2 * pad - k) / stride + 1;
    const int64_t Q = (W + 2 * pad - k) / stride + 1;
    uint32_t* zeros = (uint32_t*)calloc((size_t)cw, sizeof(uint32_t));   /* a pixel of all -1 */
    if (!zeros) return 1;
#pragma omp parallel for collapse(2) schedule(static)
    for (int64_t n = 0; n < N; ++n)
        for (int64_t p = 0; p < P; ++p)
            for (int64_t q = 0; q < Q; ++q)
                for (int64_t o = 0; o < O; ++o) {
                    int64_t len = 0, acc = 0;     /* len: number of +1/-1 products summed */
                    for (int64_t r = 0; r < k; ++r)
                        for (int64_t t = 0; t < k; ++t) {
                            const int64_t y = p * stride - pad + r;
                            const int64_t xx = q * stride - pad + t;
                            const uint32_t* fv = filt + ((o * k + r) * k + t) * cw;
                            if (y >= 0 && y < H && xx >= 0 && xx < W) {
                                acc += xor_popc_row(in + ((n * H + y) * W + xx) * cw, fv, cw);
                                len += C;
                            } else if (pad_mode == 0) {
                                acc += xor_popc_row(zeros, fv, cw);
                                len += C;
                            }
                        }
                    out[((n * P + p) * Q + q) * O + o] = (int32_t)(len - 2 * acc);
                }
    free(zeros);
    return 0;
}
