/*
 * CPU oracle for direct sparse convolution -- TEST INFRASTRUCTURE ONLY.
 *
 * Plain, slow, obviously-correct C written from the paper's section "Convolution operation using a
 * sparse operation on GPGPU" (CSR weights per output channel, column indices pre-stretched to
 * offsets into the padded NCHW input, every row padded to one common non-zero count, Algorithm 3's
 * gather-multiply-accumulate).  It shares no code with the HIP library and must never be called
 * from the product path: only the tests, the smoke check and the benchmark's cpu_baseline leg use
 * it.  Floating-point paths accumulate in double; integer paths accumulate in int32.
 *
 * Two independent definitions live here:
 *   oracle_dense_conv_*   the textbook direct convolution (cross-correlation, zero padding), which
 *                         the sparse method must reproduce because it only skips zero products;
 *   the four steps of the sparse method, one function per step, in the paper's order:
 *     1. oracle_unify_rows_*   pad every CSR row to N_nz = max row length with explicit zeros
 *     2. oracle_stretch        column index (c,r,s) -> flat offset lambda into one padded sample
 *     3. oracle_pad_input_*    materialise the zero-padded input
 *     4. oracle_gather_mac_*   Y[b,d,p,q] = sum_j theta[d,j] * Xp[b*X_size + base(p,q) + lambda[d,j]]
 *   plus oracle_decode_codebook (4-bit index -> centroid) for the non-linear quantisation variant.
 *
 * The only concession to run time is an OpenMP "parallel for" over independent (sample, channel)
 * pairs; there is no blocking, fusion or reordering of the arithmetic.
 */
#include <stdint.h>
#include <stddef.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

int oracle_num_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/* ---------------------------------------------------------------------------------------------
 * Ground truth: direct dense convolution, seven nested loops.
 * x  [N][C][H][W], wt [D][C][R][S], y [N][D][P][Q];  P = (H+2ph-R)/sh+1, Q = (W+2pw-S)/sw+1.
 * Out-of-image taps contribute zero (zero padding); no kernel flip (cross-correlation).
 * ------------------------------------------------------------------------------------------- */
#define DENSE_CONV(NAME, T, ACC)                                                                  \
void NAME(const T* x, const T* wt, T* y, int N, int C, int H, int W, int D, int R, int S,         \
          int sh, int sw, int ph, int pw)                                                         \
{                                                                                                 \
    const int P = (H + 2 * ph - R) / sh + 1;                                                      \
    const int Q = (W + 2 * pw - S) / sw + 1;                                                      \
    _Pragma("omp parallel for collapse(2) schedule(static)")                                      \
    for (int b = 0; b < N; ++b)                                                                   \
        for (int d = 0; d < D; ++d)                                                               \
            for (int p = 0; p < P; ++p)                                                           \
                for (int q = 0; q < Q; ++q) {                                                     \
                    ACC acc = 0;                                                                  \
                    for (int c = 0; c < C; ++c)                                                   \
                        for (int r = 0; r < R; ++r)                                               \
                            for (int s = 0; s < S; ++s) {                                         \
                                const int ih = p * sh + r - ph;                                   \
                                const int iw = q * sw + s - pw;                                   \
                                if (ih < 0 || ih >= H || iw < 0 || iw >= W) continue;             \
                                acc += wt[(((size_t)d * C + c) * R + r) * S + s] *                \
                                       x[(((size_t)b * C + c) * H + ih) * W + iw];                \
                            }                                                                     \
                    y[(((size_t)b * D + d) * P + p) * Q + q] = (T)acc;                            \
                }                                                                                 \
}
DENSE_CONV(oracle_dense_conv_f64, double, double)
DENSE_CONV(oracle_dense_conv_i32, int32_t, int32_t)

/* ---------------------------------------------------------------------------------------------
 * Step 1.  Unified non-zero count (the paper's "standardised sparse level").
 * N_nz is the longest row; shorter rows get explicit zero-valued entries "marked non-zero".
 * The paper does not say which column a filler entry carries: we repeat the row's last real
 * column (column 0 for an empty row), which is always a legal position.
 * ------------------------------------------------------------------------------------------- */
int oracle_unified_nnz(const int32_t* rowptr, int D)
{
    int n = 0;
    for (int d = 0; d < D; ++d) {
        const int len = rowptr[d + 1] - rowptr[d];
        if (len > n) n = len;
    }
    return n;
}

#define UNIFY_ROWS(NAME, T)                                                                       \
void NAME(const int32_t* rowptr, const int32_t* colidx, const T* values, int D, int n,            \
          int32_t* col_out, T* val_out)                                                           \
{                                                                                                 \
    for (int d = 0; d < D; ++d) {                                                                 \
        const int beg = rowptr[d], len = rowptr[d + 1] - rowptr[d];                               \
        for (int j = 0; j < n; ++j) {                                                             \
            if (j < len) {                                                                        \
                col_out[(size_t)d * n + j] = colidx[beg + j];                                     \
                val_out[(size_t)d * n + j] = values[beg + j];                                     \
            } else {                                                                              \
                col_out[(size_t)d * n + j] = len > 0 ? colidx[beg + len - 1] : 0;                 \
                val_out[(size_t)d * n + j] = 0;                                                   \
            }                                                                                     \
        }                                                                                         \
    }                                                                                             \
}
UNIFY_ROWS(oracle_unify_rows_f64, double)
UNIFY_ROWS(oracle_unify_rows_i32, int32_t)

/* ---------------------------------------------------------------------------------------------
 * Step 2.  Stretch the column indices.  A column of the D x (C*R*S) weight matrix names filter
 * tap (c, r, s); its pre-computed input offset is the distance, inside one padded sample of
 * C planes of Hp x Wp, from the top-left corner of an output pixel's receptive field to that tap.
 * ------------------------------------------------------------------------------------------- */
void oracle_stretch(const int32_t* col, size_t count, int R, int S, int Hp, int Wp, int64_t* lambda)
{
    for (size_t i = 0; i < count; ++i) {
        const int c = col[i] / (R * S);
        const int r = (col[i] % (R * S)) / S;
        const int s = col[i] % S;
        lambda[i] = ((int64_t)c * Hp + r) * Wp + s;
    }
}

/* ---------------------------------------------------------------------------------------------
 * Step 3.  Physically zero-padded input, xp [N][C][Hp][Wp] (the paper lists its inputs with the
 * padding already included, e.g. 226 x 226 for a 224 x 224 image under a 3 x 3 filter).
 * ------------------------------------------------------------------------------------------- */
#define PAD_INPUT(NAME, T)                                                                        \
void NAME(const T* x, int N, int C, int H, int W, int ph, int pw, T* xp)                          \
{                                                                                                 \
    const int Hp = H + 2 * ph, Wp = W + 2 * pw;                                                   \
    memset(xp, 0, (size_t)N * C * Hp * Wp * sizeof(T));                                           \
    for (size_t bc = 0; bc < (size_t)N * C; ++bc)                                                 \
        for (int h = 0; h < H; ++h)                                                               \
            for (int w = 0; w < W; ++w)                                                           \
                xp[(bc * Hp + h + ph) * Wp + w + pw] = x[(bc * H + h) * W + w];                   \
}
PAD_INPUT(oracle_pad_input_f64, double)
PAD_INPUT(oracle_pad_input_i32, int32_t)

/* ---------------------------------------------------------------------------------------------
 * Step 4.  Algorithm 3's arithmetic, one output value at a time: the base address of output
 * pixel (p, q) in the padded sample is p*s_h*Wp + q*s_w; every stored entry j adds
 * theta[d][j] * Xp[b*X_size + base + lambda[d][j]], j ascending, into one accumulator that is
 * written once after the last entry.
 * ------------------------------------------------------------------------------------------- */
#define GATHER_MAC(NAME, T, ACC)                                                                  \
void NAME(const T* xp, const T* theta, const int64_t* lambda, T* y, int N, int64_t X_size,        \
          int D, int n, int P, int Q, int sh, int sw, int Wp)                                     \
{                                                                                                 \
    _Pragma("omp parallel for collapse(2) schedule(static)")                                      \
    for (int b = 0; b < N; ++b)                                                                   \
        for (int d = 0; d < D; ++d)                                                               \
            for (int p = 0; p < P; ++p)                                                           \
                for (int q = 0; q < Q; ++q) {                                                     \
                    const int64_t base = (int64_t)b * X_size + (int64_t)p * sh * Wp + (int64_t)q * sw; \
                    ACC acc = 0;                                                                  \
                    for (int j = 0; j < n; ++j)                                                   \
                        acc += theta[(size_t)d * n + j] * xp[base + lambda[(size_t)d * n + j]];   \
                    y[(((size_t)b * D + d) * P + p) * Q + q] = (T)acc;                            \
                }                                                                                 \
}
GATHER_MAC(oracle_gather_mac_f64, double, double)
GATHER_MAC(oracle_gather_mac_i32, int32_t, int32_t)

/* ---------------------------------------------------------------------------------------------
 * Non-linear (clustered) quantisation: a stored weight is the index of its centroid; the forward
 * pass maps each index back to the (already bit-width-reduced) centroid value.
 * ------------------------------------------------------------------------------------------- */
void oracle_decode_codebook(const uint8_t* idx, size_t count, const int32_t* codebook, int32_t* out)
{
    for (size_t i = 0; i < count; ++i) out[i] = codebook[idx[i]];
}

/* the same with centroids kept in a floating-point format (sixteen-bit in the paper's 4b/16b runs) */
void oracle_decode_codebook_f64(const uint8_t* idx, size_t count, const double* codebook, double* out)
{
    for (size_t i = 0; i < count; ++i) out[i] = codebook[idx[i]];
}
