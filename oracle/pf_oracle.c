/*
 * pf_oracle.c -- TEST INFRASTRUCTURE, not part of the product.
 *
 * A plain, slow, unfused CPU evaluator for the operators a memory-intensive chain is made of.  Every
 * function reads complete fp64 tensors and writes a complete fp64 tensor: one call per operator, one
 * full intermediate per call, row-major nested loops, nothing fused, tiled or reordered.  The fused HIP
 * kernels of the library must reproduce what a chain of these calls produces, because the method only
 * removes data movement between operators and never changes their arithmetic (paper section 5.1,
 * gOperator merging: a write followed by a read of the same slice collapses; section 5.2: the rules do
 * not lower the theoretical memory performance and keep the program's meaning).
 *
 * The paper defines none of the operators by formula; it names the four basic kinds -- element-wise,
 * broadcast, reduce, transpose (section 6, GIR-Graph generation) -- and composite examples (SiLU =
 * sigmoid then multiply).  Each function below therefore states the textbook definition it implements.
 * Composite operators are written as the sequence of basic steps, each step with its own full buffer.
 *
 * Only tests, the smoke check and the benchmark's CPU-baseline leg may call this file.  It shares no
 * code, header, table or constant with the HIP library.
 *
 * Pins (tests/test_oracle_pins.py): closed forms, invariants, brute-force tiny cases and library
 * routines for every function here; none is "parity unpinned".
 *
 * Threading: loops over independent rows / groups / elements carry an OpenMP pragma so the benchmark can
 * time the same code on one core and on all cores (orc_set_threads).  The arithmetic per row is
 * sequential and identical for any thread count.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

#define ORC_OK 0
#define ORC_BAD_ARG 1
#define ORC_NOMEM 2

/* binary element-wise operator codes */
enum { ORC_ADD = 0, ORC_SUB = 1, ORC_MUL = 2, ORC_DIV = 3, ORC_MAX = 4, ORC_MIN = 5 };
/* unary element-wise operator codes */
enum { ORC_SCALE = 0, ORC_ADDC = 1, ORC_NEG = 2, ORC_RELU = 3, ORC_SIGMOID = 4, ORC_SILU = 5,
       ORC_GELU_ERF = 6, ORC_TANH = 7, ORC_EXP = 8, ORC_RSQRT = 9 };
/* reductions over the last dimension */
enum { ORC_RSUM = 0, ORC_RMAX = 1, ORC_RMEAN = 2 };

int orc_set_threads(int n)
{
#ifdef _OPENMP
    if (n < 1) n = 1;
    omp_set_num_threads(n);
    return n;
#else
    (void)n;
    return 1;
#endif
}

int orc_max_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/*
 * Element-wise binary operator with broadcast (basic kinds "element-wise" + "broadcast").
 * a has na elements, b has nb elements, the result has n = max(na, nb) elements; the smaller operand's
 * shape equals the trailing dimensions of the larger one, so in row-major order its element for flat
 * index k is k mod (its size).  out[k] = a[k mod na] (op) b[k mod nb]; operand order is kept, so SUB is
 * a - b and DIV is a / b.  MAX / MIN propagate NaN like fmax / fmin do not: a NaN operand gives NaN.
 */
int orc_ew_binary(int op, const double *a, int64_t na, const double *b, int64_t nb, double *out)
{
    if (na <= 0 || nb <= 0) return ORC_BAD_ARG;
    int64_t n = na > nb ? na : nb;
    if (n % na != 0 || n % nb != 0) return ORC_BAD_ARG;
    if (op < ORC_ADD || op > ORC_MIN) return ORC_BAD_ARG;
#pragma omp parallel for schedule(static)
    for (int64_t k = 0; k < n; ++k) {
        double x = a[k % na], y = b[k % nb], r;
        switch (op) {
        case ORC_ADD: r = x + y; break;
        case ORC_SUB: r = x - y; break;
        case ORC_MUL: r = x * y; break;
        case ORC_DIV: r = x / y; break;
        case ORC_MAX: r = (isnan(x) || isnan(y)) ? NAN : (x > y ? x : y); break;
        default:      r = (isnan(x) || isnan(y)) ? NAN : (x < y ? x : y); break;
        }
        out[k] = r;
    }
    return ORC_OK;
}

/*
 * Element-wise unary operator ("element-wise": arithmetic and activations).
 *   SCALE    x * alpha            ADDC  x + alpha          NEG   -x
 *   RELU     max(x, 0)            SIGMOID 1 / (1 + e^-x)   SILU  x * sigmoid(x)   (section 6: SiLU is a
 *            sigmoid followed by a multiply; here it is evaluated exactly so, with a full buffer for the
 *            sigmoid, in orc_silu_decomposed below; this entry computes the same product per element)
 *   GELU_ERF x/2 * (1 + erf(x / sqrt 2))   TANH  tanh x    EXP  e^x     RSQRT  1 / sqrt x
 */
int orc_ew_unary(int op, const double *x, int64_t n, double alpha, double *out)
{
    if (n <= 0) return ORC_BAD_ARG;
    if (op < ORC_SCALE || op > ORC_RSQRT) return ORC_BAD_ARG;
#pragma omp parallel for schedule(static)
    for (int64_t k = 0; k < n; ++k) {
        double v = x[k], r;
        switch (op) {
        case ORC_SCALE:    r = v * alpha; break;
        case ORC_ADDC:     r = v + alpha; break;
        case ORC_NEG:      r = -v; break;
        case ORC_RELU:     r = isnan(v) ? NAN : (v > 0.0 ? v : 0.0); break;
        case ORC_SIGMOID:  r = 1.0 / (1.0 + exp(-v)); break;
        case ORC_SILU:     r = v * (1.0 / (1.0 + exp(-v))); break;
        case ORC_GELU_ERF: r = 0.5 * v * (1.0 + erf(v / sqrt(2.0))); break;
        case ORC_TANH:     r = tanh(v); break;
        case ORC_EXP:      r = exp(v); break;
        default:           r = 1.0 / sqrt(v); break;
        }
        out[k] = r;
    }
    return ORC_OK;
}

/*
 * Causal mask on the last two dimensions (i = row, j = column): positions with j > i become -infinity,
 * all others keep their value.  x is [outer, si, sj].
 */
int orc_causal_mask(const double *x, int64_t outer, int64_t si, int64_t sj, double *out)
{
    if (outer <= 0 || si <= 0 || sj <= 0) return ORC_BAD_ARG;
#pragma omp parallel for schedule(static)
    for (int64_t o = 0; o < outer; ++o)
        for (int64_t i = 0; i < si; ++i)
            for (int64_t j = 0; j < sj; ++j) {
                int64_t k = (o * si + i) * sj + j;
                out[k] = (j > i) ? -INFINITY : x[k];
            }
    return ORC_OK;
}

/*
 * Reduction over the last dimension (basic kind "reduce"), keeping that dimension with extent 1:
 * x is [rows, n], out is [rows].  SUM and MEAN add left to right; MAX returns NaN if the row holds one.
 */
int orc_reduce_last(int op, const double *x, int64_t rows, int64_t n, double *out)
{
    if (rows <= 0 || n <= 0) return ORC_BAD_ARG;
    if (op < ORC_RSUM || op > ORC_RMEAN) return ORC_BAD_ARG;
#pragma omp parallel for schedule(static)
    for (int64_t r = 0; r < rows; ++r) {
        const double *p = x + r * n;
        double acc;
        if (op == ORC_RMAX) {
            acc = p[0];
            for (int64_t j = 1; j < n; ++j) {
                if (isnan(p[j]) || isnan(acc)) acc = NAN;
                else if (p[j] > acc) acc = p[j];
            }
        } else {
            acc = 0.0;
            for (int64_t j = 0; j < n; ++j) acc += p[j];
            if (op == ORC_RMEAN) acc /= (double)n;
        }
        out[r] = acc;
    }
    return ORC_OK;
}

/*
 * Broadcast of a per-row value back over the last dimension combined with an element-wise operator:
 * out[r, j] = x[r, j] (op) v[r].  This is the "broadcast" basic kind in the direction a reduction needs.
 */
int orc_row_broadcast_binary(int op, const double *x, int64_t rows, int64_t n, const double *v, double *out)
{
    if (rows <= 0 || n <= 0) return ORC_BAD_ARG;
    if (op < ORC_ADD || op > ORC_DIV) return ORC_BAD_ARG;
#pragma omp parallel for schedule(static)
    for (int64_t r = 0; r < rows; ++r)
        for (int64_t j = 0; j < n; ++j) {
            double a = x[r * n + j], b = v[r], o;
            switch (op) {
            case ORC_ADD: o = a + b; break;
            case ORC_SUB: o = a - b; break;
            case ORC_MUL: o = a * b; break;
            default:      o = a / b; break;
            }
            out[r * n + j] = o;
        }
    return ORC_OK;
}

/*
 * The three operators of an attention layer that generates one token against cached keys and values
 * (paper section 8, the GPT-2 case study): with a sequence length of one, both matrix products of the
 * layer are matrix-vector products, and the cache grows by one row through a concatenation.
 *
 * concat_rows: y[o, 0..t-1, :] = x[o, :, :]; y[o, t, :] = r[o, :]     (x: [outer, t, d], r: [outer, d])
 */
int orc_concat_rows(const double *x, int64_t outer, int64_t t, int64_t d, const double *r, double *out)
{
    if (outer <= 0 || t < 0 || d <= 0) return ORC_BAD_ARG;
    for (int64_t o = 0; o < outer; ++o) {
        for (int64_t j = 0; j < t; ++j)
            for (int64_t c = 0; c < d; ++c) out[(o * (t + 1) + j) * d + c] = x[(o * t + j) * d + c];
        for (int64_t c = 0; c < d; ++c) out[(o * (t + 1) + t) * d + c] = r[o * d + c];
    }
    return ORC_OK;
}

/* matvec: y[o, j] = sum_c a[o, j, c] * x[o, c]      (a: [outer, t, d], x: [outer, d]) -- contracts the last axis */
int orc_matvec(const double *a, int64_t outer, int64_t t, int64_t d, const double *x, double *out)
{
    if (outer <= 0 || t <= 0 || d <= 0) return ORC_BAD_ARG;
#pragma omp parallel for schedule(static)
    for (int64_t o = 0; o < outer; ++o)
        for (int64_t j = 0; j < t; ++j) {
            double acc = 0.0;
            for (int64_t c = 0; c < d; ++c) acc += a[(o * t + j) * d + c] * x[o * d + c];
            out[o * t + j] = acc;
        }
    return ORC_OK;
}

/* vecmat: y[o, c] = sum_j p[o, j] * a[o, j, c]      (p: [outer, t], a: [outer, t, d]) -- contracts the row axis */
int orc_vecmat(const double *p, int64_t outer, int64_t t, int64_t d, const double *a, double *out)
{
    if (outer <= 0 || t <= 0 || d <= 0) return ORC_BAD_ARG;
#pragma omp parallel for schedule(static)
    for (int64_t o = 0; o < outer; ++o)
        for (int64_t c = 0; c < d; ++c) {
            double acc = 0.0;
            for (int64_t j = 0; j < t; ++j) acc += p[o * t + j] * a[(o * t + j) * d + c];
            out[o * d + c] = acc;
        }
    return ORC_OK;
}

/*
 * Softmax over the last dimension, as the sequence of basic operators it consists of:
 *   m = reduce-max(x); d = x - m; e = exp(d); s = reduce-sum(e); y = e / s.
 * exp(-inf) = 0, so masked positions come out as exactly 0; a row that is -inf everywhere gives
 * (-inf) - (-inf) = NaN in every position, which is what the definition says.
 */
int orc_softmax_last(const double *x, int64_t rows, int64_t n, double *out)
{
    if (rows <= 0 || n <= 0) return ORC_BAD_ARG;
    size_t total = (size_t)rows * (size_t)n;
    double *m = (double *)malloc(sizeof(double) * (size_t)rows);
    double *s = (double *)malloc(sizeof(double) * (size_t)rows);
    double *d = (double *)malloc(sizeof(double) * total);
    double *e = (double *)malloc(sizeof(double) * total);
    int rc = ORC_NOMEM;
    if (m && s && d && e) {
        rc = orc_reduce_last(ORC_RMAX, x, rows, n, m);
        if (!rc) rc = orc_row_broadcast_binary(ORC_SUB, x, rows, n, m, d);
        if (!rc) rc = orc_ew_unary(ORC_EXP, d, (int64_t)total, 0.0, e);
        if (!rc) rc = orc_reduce_last(ORC_RSUM, e, rows, n, s);
        if (!rc) rc = orc_row_broadcast_binary(ORC_DIV, e, rows, n, s, out);
    }
    free(m); free(s); free(d); free(e);
    return rc;
}

/*
 * LayerNorm over the last dimension with affine parameters:
 *   mu = mean(x); c = x - mu; var = mean(c * c)   (biased: divided by n, two passes)
 *   y = c / sqrt(var + eps) * gamma + beta,  gamma and beta indexed by the position in the row.
 * gamma or beta may be NULL, meaning 1 and 0.
 */
int orc_layernorm_last(const double *x, int64_t rows, int64_t n, const double *gamma, const double *beta,
                       double eps, double *out)
{
    if (rows <= 0 || n <= 0) return ORC_BAD_ARG;
    size_t total = (size_t)rows * (size_t)n;
    double *mu = (double *)malloc(sizeof(double) * (size_t)rows);
    double *var = (double *)malloc(sizeof(double) * (size_t)rows);
    double *c = (double *)malloc(sizeof(double) * total);
    double *c2 = (double *)malloc(sizeof(double) * total);
    int rc = ORC_NOMEM;
    if (mu && var && c && c2) {
        rc = orc_reduce_last(ORC_RMEAN, x, rows, n, mu);
        if (!rc) rc = orc_row_broadcast_binary(ORC_SUB, x, rows, n, mu, c);
        if (!rc) rc = orc_ew_binary(ORC_MUL, c, (int64_t)total, c, (int64_t)total, c2);
        if (!rc) rc = orc_reduce_last(ORC_RMEAN, c2, rows, n, var);
        if (!rc) {
#pragma omp parallel for schedule(static)
            for (int64_t r = 0; r < rows; ++r) {
                double denom = sqrt(var[r] + eps);
                for (int64_t j = 0; j < n; ++j) {
                    double y = c[r * n + j] / denom;
                    if (gamma) y *= gamma[j];
                    if (beta) y += beta[j];
                    out[r * n + j] = y;
                }
            }
        }
    }
    free(mu); free(var); free(c); free(c2);
    return rc;
}

/*
 * RMSNorm over the last dimension: y = x / sqrt(mean(x * x) + eps) * gamma.
 */
int orc_rmsnorm_last(const double *x, int64_t rows, int64_t n, const double *gamma, double eps, double *out)
{
    if (rows <= 0 || n <= 0) return ORC_BAD_ARG;
    size_t total = (size_t)rows * (size_t)n;
    double *ms = (double *)malloc(sizeof(double) * (size_t)rows);
    double *x2 = (double *)malloc(sizeof(double) * total);
    int rc = ORC_NOMEM;
    if (ms && x2) {
        rc = orc_ew_binary(ORC_MUL, x, (int64_t)total, x, (int64_t)total, x2);
        if (!rc) rc = orc_reduce_last(ORC_RMEAN, x2, rows, n, ms);
        if (!rc) {
#pragma omp parallel for schedule(static)
            for (int64_t r = 0; r < rows; ++r) {
                double denom = sqrt(ms[r] + eps);
                for (int64_t j = 0; j < n; ++j) {
                    double y = x[r * n + j] / denom;
                    if (gamma) y *= gamma[j];
                    out[r * n + j] = y;
                }
            }
        }
    }
    free(ms); free(x2);
    return rc;
}

/*
 * GroupNorm on a channels-last tensor x[nb, hw, c] with g groups of c/g consecutive channels:
 * for every sample s and group q the statistics run over all hw positions and the group's channels,
 *   mu = mean, var = mean((x - mu)^2)  (biased, two passes),
 *   y[s, p, ch] = (x - mu) / sqrt(var + eps) * gamma[ch] + beta[ch].
 */
int orc_groupnorm_nhwc(const double *x, int64_t nb, int64_t hw, int64_t c, int64_t g, const double *gamma,
                       const double *beta, double eps, double *out)
{
    if (nb <= 0 || hw <= 0 || c <= 0 || g <= 0 || c % g != 0) return ORC_BAD_ARG;
    int64_t cpg = c / g;
    double cnt = (double)hw * (double)cpg;
#pragma omp parallel for schedule(static) collapse(2)
    for (int64_t s = 0; s < nb; ++s)
        for (int64_t q = 0; q < g; ++q) {
            double sum = 0.0;
            for (int64_t p = 0; p < hw; ++p)
                for (int64_t k = 0; k < cpg; ++k) sum += x[(s * hw + p) * c + q * cpg + k];
            double mu = sum / cnt;
            double ss = 0.0;
            for (int64_t p = 0; p < hw; ++p)
                for (int64_t k = 0; k < cpg; ++k) {
                    double d = x[(s * hw + p) * c + q * cpg + k] - mu;
                    ss += d * d;
                }
            double denom = sqrt(ss / cnt + eps);
            for (int64_t p = 0; p < hw; ++p)
                for (int64_t k = 0; k < cpg; ++k) {
                    int64_t ch = q * cpg + k;
                    int64_t idx = (s * hw + p) * c + ch;
                    double y = (x[idx] - mu) / denom;
                    if (gamma) y *= gamma[ch];
                    if (beta) y += beta[ch];
                    out[idx] = y;
                }
        }
    return ORC_OK;
}

/*
 * Permutation of dimensions (basic kind "transpose"): out has shape[perm[0]], shape[perm[1]], ... and
 * out[j0, j1, ...] = x[i0, i1, ...] with i[perm[k]] = j[k].  The element is copied as `esize` raw bytes,
 * so the same routine serves fp64 values (esize 8) and the bit patterns of 16- and 32-bit storage
 * types (esize 2 or 4) for the bit-exact layout checks.
 */
int orc_permute_bytes(const void *x, int32_t rank, const int64_t *shape, const int32_t *perm, int32_t esize,
                      void *out)
{
    if (rank < 1 || rank > 8 || esize < 1) return ORC_BAD_ARG;
    int seen[8] = {0};
    int64_t in_stride[8], out_shape[8], total = 1;
    for (int k = 0; k < rank; ++k) {
        if (perm[k] < 0 || perm[k] >= rank || seen[perm[k]] || shape[k] <= 0) return ORC_BAD_ARG;
        seen[perm[k]] = 1;
    }
    in_stride[rank - 1] = 1;
    for (int k = rank - 2; k >= 0; --k) in_stride[k] = in_stride[k + 1] * shape[k + 1];
    for (int k = 0; k < rank; ++k) { out_shape[k] = shape[perm[k]]; total *= shape[k]; }
    const char *src = (const char *)x;
    char *dst = (char *)out;
#pragma omp parallel for schedule(static)
    for (int64_t o = 0; o < total; ++o) {
        int64_t rem = o, src_idx = 0;
        for (int k = rank - 1; k >= 0; --k) {
            int64_t j = rem % out_shape[k];
            rem /= out_shape[k];
            src_idx += j * in_stride[perm[k]];
        }
        memcpy(dst + o * esize, src + src_idx * esize, (size_t)esize);
    }
    return ORC_OK;
}

/*
 * Concatenation and slicing along one axis (data movement only; the ShuffleNet fragment
 * concat -> channel shuffle -> split of section 2 is made of these, a reshape and a permutation).
 * Elements are moved as `esize` raw bytes.
 *
 * concat: out[..., 0..la-1, ...] = a, out[..., la..la+lb-1, ...] = b along `axis`; all other extents equal.
 */
int orc_concat_bytes(const void *a, const void *b, int32_t rank, const int64_t *shape_a, const int64_t *shape_b,
                     int32_t axis, int32_t esize, void *out)
{
    if (rank < 1 || rank > 8 || axis < 0 || axis >= rank || esize < 1) return ORC_BAD_ARG;
    int64_t outer = 1, inner = 1;
    for (int k = 0; k < rank; ++k) {
        if (shape_a[k] <= 0 || shape_b[k] <= 0) return ORC_BAD_ARG;
        if (k != axis && shape_a[k] != shape_b[k]) return ORC_BAD_ARG;
        if (k < axis) outer *= shape_a[k];
        if (k > axis) inner *= shape_a[k];
    }
    const int64_t la = shape_a[axis] * inner, lb = shape_b[axis] * inner;
    const char *pa = (const char *)a, *pb = (const char *)b;
    char *po = (char *)out;
    for (int64_t o = 0; o < outer; ++o) {
        for (int64_t i = 0; i < la; ++i) memcpy(po + (o * (la + lb) + i) * esize, pa + (o * la + i) * esize, (size_t)esize);
        for (int64_t i = 0; i < lb; ++i) memcpy(po + (o * (la + lb) + la + i) * esize, pb + (o * lb + i) * esize, (size_t)esize);
    }
    return ORC_OK;
}

/* slice: out[..., j, ...] = x[..., start + j, ...] for 0 <= j < length along `axis` */
int orc_slice_bytes(const void *x, int32_t rank, const int64_t *shape, int32_t axis, int64_t start, int64_t length,
                    int32_t esize, void *out)
{
    if (rank < 1 || rank > 8 || axis < 0 || axis >= rank || esize < 1) return ORC_BAD_ARG;
    int64_t outer = 1, inner = 1;
    for (int k = 0; k < rank; ++k) {
        if (shape[k] <= 0) return ORC_BAD_ARG;
        if (k < axis) outer *= shape[k];
        if (k > axis) inner *= shape[k];
    }
    if (start < 0 || length < 1 || start + length > shape[axis]) return ORC_BAD_ARG;
    const char *px = (const char *)x;
    char *po = (char *)out;
    for (int64_t o = 0; o < outer; ++o)
        for (int64_t j = 0; j < length; ++j)
            for (int64_t i = 0; i < inner; ++i)
                memcpy(po + ((o * length + j) * inner + i) * esize,
                       px + ((o * shape[axis] + start + j) * inner + i) * esize, (size_t)esize);
    return ORC_OK;
}

/*
 * Depthwise convolution on a channels-last tensor, the memory-intensive convolution of the paper's
 * EfficientNet fragment (section 6, preprocessing of the computation graph), in the usual DNN sense
 * (cross-correlation), zero padding of kh/2 rows and kw/2 columns on every side, odd kernel extents, the
 * same stride s >= 1 along both axes (that network's blocks use 1 and 2):
 *   y[n, i, j, c] = sum_{a < kh, b < kw} w[a, b, c] * x[n, i*s + a - kh/2, j*s + b - kw/2, c]
 * with x taken as 0 outside [0, h) x [0, w), for i < (h - 1)/s + 1, j < (w - 1)/s + 1 (stride 1 keeps the
 * spatial size).   x: [n, h, w, c], w: [kh, kw, c], y: [n, (h - 1)/s + 1, (w - 1)/s + 1, c].
 */
int orc_dwconv2d_nhwc(const double *x, int64_t n, int64_t h, int64_t w, int64_t c, const double *wgt, int64_t kh,
                      int64_t kw, int64_t stride, double *out)
{
    if (n <= 0 || h <= 0 || w <= 0 || c <= 0 || kh < 1 || kw < 1 || kh % 2 == 0 || kw % 2 == 0 || stride < 1) return ORC_BAD_ARG;
    const int64_t oh = (h - 1) / stride + 1, ow = (w - 1) / stride + 1;
#pragma omp parallel for schedule(static) collapse(2)
    for (int64_t b = 0; b < n; ++b)
        for (int64_t i = 0; i < oh; ++i)
            for (int64_t j = 0; j < ow; ++j)
                for (int64_t ch = 0; ch < c; ++ch) {
                    double acc = 0.0;
                    for (int64_t a = 0; a < kh; ++a)
                        for (int64_t q = 0; q < kw; ++q) {
                            const int64_t ii = i * stride + a - kh / 2, jj = j * stride + q - kw / 2;
                            if (ii < 0 || ii >= h || jj < 0 || jj >= w) continue;
                            acc += wgt[(a * kw + q) * c + ch] * x[((b * h + ii) * w + jj) * c + ch];
                        }
                    out[((b * oh + i) * ow + j) * c + ch] = acc;
                }
    return ORC_OK;
}
