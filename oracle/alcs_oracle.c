/*
 * CPU oracle for the SIMD-structured sparse convolution of arXiv 2109.00170 (ALCS).
 *
 * THIS IS TEST INFRASTRUCTURE, NOT THE PRODUCT.  It is a plain, slow, obviously
 * correct statement of what the hot path computes, written from the paper, and it
 * shares no code, header, table or helper with the HIP library.  Only the tests,
 * the smoke check and the benchmark's cpu_baseline leg may call it.
 *
 * What is defined where (all in Section 3.2 of the paper):
 *   - grouping of V adjacent output channels whose zero pattern is shared
 *     (Section 3.2.1)                                  -> oracle_densify
 *   - the convolution sum O(n,h,w) = sum_c sum_r sum_s W(n,c,r,s) I(c,h+r,w+s)
 *     (unnumbered equation of Section 3.2.2, "Overview")-> oracle_conv, oracle_conv_at
 *   - the grouped-CSR storage format: per filter group the number of kept
 *     columns, their column offsets and their V-vectors of values
 *     (Section 3.2.2, "Storage format")                 -> oracle_pack, oracle_unpack
 *   - the multiplication of the grouped-CSR matrix W* with the patch matrix I*
 *     (Section 3.2.2, "Overview" and "Efficient multiplication computation")
 *                                                       -> oracle_im2col, oracle_conv_csr
 *   - the element-wise layers after a convolution (ReLU, ReLU6, shortcut addition),
 *     the "other layers" behind the constant tau of Section 3.3, Eq. (2), folded into
 *     the convolution                                   -> oracle_conv_fused
 *   - the depthwise 3x3 layer that precedes every pointwise convolution of the
 *     MobileNet the paper prunes (Section 4; one filter per channel, the conv
 *     equation of Section 3.2.2 with the sum over c reduced to the channel itself),
 *     with its bias and activation                      -> oracle_depthwise
 *   - the latency model of Section 3.3: a layer's run time as a piecewise-linear
 *     function of its number of non-zero weights, Eqs. (4)-(6), and the network's
 *     run time as tau plus the sum over layers, Eq. (2)
 *                                 -> oracle_latency_estimate, oracle_network_latency
 *
 * Extensions beyond the paper's equation, taken from the library's problem
 * statement: a batch of N independent images, zero padding pad=(k-1)/2, a stride,
 * and an optional per-channel bias.  Cross-correlation (no kernel flip).
 *
 * Pins (see tests/test_oracle_*.py): the storage-format example the paper spells
 * out in prose, pack/unpack round trip, brute force on tiny inputs, a library
 * convolution at sparsity 0, all-bias output at sparsity 100 %, linearity in X,
 * identity/impulse inputs that make every sum a single term.
 * The paper prints no output tensor of its kernel, so numeric outputs of the
 * paper's own implementation are "parity unpinned"; only the definition pins values.
 *
 * Floating point: every sum is accumulated in double and rounded to float once.
 */
#include <stddef.h>
#include <stdint.h>
#include <string.h>

#ifdef _OPENMP
#include <omp.h>
#endif

#define ORACLE_OK 0
#define ORACLE_BAD_ARG (-1)

static int out_size(int in, int k, int stride) {
    int pad = (k - 1) / 2;
    return (in + 2 * pad - k) / stride + 1;
}

static int n_groups(int Cout, int V) { return (Cout + V - 1) / V; }

int oracle_out_size(int in, int k, int stride) { return out_size(in, k, stride); }

/* Section 3.2.1: output channel o belongs to group o / V; the mask holds one
 * keep/drop flag per (group, c, r, s).  A dropped block contributes nothing even
 * if W is non-zero there; a kept block is used as is, even if it holds zeros.
 * mask == NULL keeps everything. */
int oracle_densify(const float *W, const uint8_t *mask, int Cout, int Cin, int k, int V,
                   float *Wd) {
    if (!W || !Wd || Cout <= 0 || Cin <= 0 || k <= 0 || V <= 0) return ORACLE_BAD_ARG;
    size_t K = (size_t)Cin * k * k;
    for (int o = 0; o < Cout; ++o) {
        int g = o / V;
        for (size_t col = 0; col < K; ++col) {
            int keep = mask ? (mask[(size_t)g * K + col] != 0) : 1;
            Wd[(size_t)o * K + col] = keep ? W[(size_t)o * K + col] : 0.0f;
        }
    }
    return ORACLE_OK;
}

/* One output element by the defining sum, in the order c, r, s, in double. */
static double conv_point_d(const float *Wd, const float *X, const float *bias, int Cin, int H,
                           int Wi, int k, int stride, int n, int o, int ho, int wo) {
    int pad = (k - 1) / 2;
    double acc = 0.0;
    for (int c = 0; c < Cin; ++c)
        for (int r = 0; r < k; ++r)
            for (int s = 0; s < k; ++s) {
                float w = Wd[(((size_t)o * Cin + c) * k + r) * k + s];
                if (w == 0.0f) continue; /* adds nothing for finite inputs */
                int hi = ho * stride + r - pad;
                int wi = wo * stride + s - pad;
                if (hi < 0 || hi >= H || wi < 0 || wi >= Wi) continue; /* zero padding */
                acc += (double)w * (double)X[(((size_t)n * Cin + c) * H + hi) * Wi + wi];
            }
    if (bias) acc += (double)bias[o];
    return acc;
}

static float conv_point(const float *Wd, const float *X, const float *bias, int Cin, int H,
                        int Wi, int k, int stride, int n, int o, int ho, int wo) {
    return (float)conv_point_d(Wd, X, bias, Cin, H, Wi, k, stride, n, o, ho, wo);
}

/* The convolution equation of Section 3.2.2 on the densified weights:
 * seven nested loops n, o, ho, wo, c, r, s.  Threads only split the (n, o) pairs. */
int oracle_conv(const float *Wd, const float *X, const float *bias, float *Y, int N, int Cin,
                int Cout, int H, int Wi, int k, int stride, int nthreads) {
    if (!Wd || !X || !Y || N < 0 || Cin <= 0 || Cout <= 0 || H <= 0 || Wi <= 0) return ORACLE_BAD_ARG;
    if (k <= 0 || (k % 2) == 0 || stride <= 0) return ORACLE_BAD_ARG;
    int Ho = out_size(H, k, stride), Wo = out_size(Wi, k, stride);
    if (Ho <= 0 || Wo <= 0) return ORACLE_BAD_ARG;
    long long pairs = (long long)N * Cout;
#ifdef _OPENMP
    if (nthreads <= 0) nthreads = omp_get_max_threads();
#pragma omp parallel for schedule(dynamic, 1) num_threads(nthreads)
#endif
    for (long long no = 0; no < pairs; ++no) {
        int n = (int)(no / Cout), o = (int)(no % Cout);
        for (int ho = 0; ho < Ho; ++ho)
            for (int wo = 0; wo < Wo; ++wo)
                Y[(((size_t)n * Cout + o) * Ho + ho) * Wo + wo] =
                    conv_point(Wd, X, bias, Cin, H, Wi, k, stride, n, o, ho, wo);
    }
    (void)nthreads;
    return ORACLE_OK;
}

/* The convolution with the element-wise layers that follow it folded in:
 *   Y = act(conv(X) + bias + R),  act in {identity, max(.,0), min(max(.,0),6)},
 * R an optional tensor of Y's shape (a shortcut connection).  These are the "other
 * layers (e.g. ReLU layers ...)" whose latency Section 3.3, Eq. (2) of the paper books
 * as the constant tau; folding them into the convolution's epilogue removes their pass
 * over Y.  Sum, bias and R are added in double, the activation is applied in double,
 * and the result is rounded to float once.  R may be Y itself (element-wise in place). */
int oracle_conv_fused(const float *Wd, const float *X, const float *bias, const float *R, float *Y,
                      int N, int Cin, int Cout, int H, int Wi, int k, int stride, int act,
                      int nthreads) {
    if (!Wd || !X || !Y || N < 0 || Cin <= 0 || Cout <= 0 || H <= 0 || Wi <= 0) return ORACLE_BAD_ARG;
    if (k <= 0 || (k % 2) == 0 || stride <= 0 || act < 0 || act > 2) return ORACLE_BAD_ARG;
    int Ho = out_size(H, k, stride), Wo = out_size(Wi, k, stride);
    if (Ho <= 0 || Wo <= 0) return ORACLE_BAD_ARG;
    long long pairs = (long long)N * Cout;
#ifdef _OPENMP
    if (nthreads <= 0) nthreads = omp_get_max_threads();
#pragma omp parallel for schedule(dynamic, 1) num_threads(nthreads)
#endif
    for (long long no = 0; no < pairs; ++no) {
        int n = (int)(no / Cout), o = (int)(no % Cout);
        for (int ho = 0; ho < Ho; ++ho)
            for (int wo = 0; wo < Wo; ++wo) {
                size_t at = (((size_t)n * Cout + o) * Ho + ho) * Wo + wo;
                double v = conv_point_d(Wd, X, bias, Cin, H, Wi, k, stride, n, o, ho, wo);
                if (R) v += (double)R[at];
                if (act >= 1 && v < 0.0) v = 0.0;
                if (act == 2 && v > 6.0) v = 6.0;
                Y[at] = (float)v;
            }
    }
    (void)nthreads;
    return ORACLE_OK;
}

/* Depthwise convolution: channel c of the output sees only channel c of the input,
 *   Z(c,h,w) = act(b(c) + sum_r sum_s D(c,r,s) I(c, h*stride + r - pad, w*stride + s - pad)),
 * the convolution equation of Section 3.2.2 without the sum over input channels; zero
 * padding pad = (k-1)/2, no kernel flip.  D is [C,k,k].  Sum in double, one rounding.
 * It is the layer in front of each pointwise convolution of the MobileNet of Section 4. */
int oracle_depthwise(const float *D, const float *X, const float *bias, float *Z, int N, int C,
                     int H, int Wi, int k, int stride, int act) {
    if (!D || !X || !Z || N < 0 || C <= 0 || H <= 0 || Wi <= 0) return ORACLE_BAD_ARG;
    if (k <= 0 || (k % 2) == 0 || stride <= 0 || act < 0 || act > 2) return ORACLE_BAD_ARG;
    int Ho = out_size(H, k, stride), Wo = out_size(Wi, k, stride);
    if (Ho <= 0 || Wo <= 0) return ORACLE_BAD_ARG;
    int pad = (k - 1) / 2;
    for (int n = 0; n < N; ++n)
        for (int c = 0; c < C; ++c)
            for (int ho = 0; ho < Ho; ++ho)
                for (int wo = 0; wo < Wo; ++wo) {
                    double v = bias ? (double)bias[c] : 0.0;
                    for (int r = 0; r < k; ++r)
                        for (int q = 0; q < k; ++q) {
                            int hi = ho * stride + r - pad, wi = wo * stride + q - pad;
                            if (hi < 0 || hi >= H || wi < 0 || wi >= Wi) continue;
                            v += (double)D[((size_t)c * k + r) * k + q] *
                                 (double)X[(((size_t)n * C + c) * H + hi) * Wi + wi];
                        }
                    if (act >= 1 && v < 0.0) v = 0.0;
                    if (act == 2 && v > 6.0) v = 6.0;
                    Z[(((size_t)n * C + c) * Ho + ho) * Wo + wo] = (float)v;
                }
    return ORACLE_OK;
}

/* The same sum for a list of flat indices into Y[N,Cout,Ho,Wo]; lets a test check
 * sampled elements of a full-size layer one by one. */
int oracle_conv_at(const float *Wd, const float *X, const float *bias, int N, int Cin, int Cout,
                   int H, int Wi, int k, int stride, const int64_t *flat_idx, int64_t n_idx,
                   float *out) {
    if (!Wd || !X || !out || (!flat_idx && n_idx > 0)) return ORACLE_BAD_ARG;
    if (k <= 0 || (k % 2) == 0 || stride <= 0) return ORACLE_BAD_ARG;
    int Ho = out_size(H, k, stride), Wo = out_size(Wi, k, stride);
    int64_t total = (int64_t)N * Cout * Ho * Wo;
    for (int64_t i = 0; i < n_idx; ++i) {
        int64_t f = flat_idx[i];
        if (f < 0 || f >= total) return ORACLE_BAD_ARG;
        int wo = (int)(f % Wo); f /= Wo;
        int ho = (int)(f % Ho); f /= Ho;
        int o = (int)(f % Cout); f /= Cout;
        int n = (int)f;
        out[i] = conv_point(Wd, X, bias, Cin, H, Wi, k, stride, n, o, ho, wo);
    }
    return ORACLE_OK;
}

/* Number of kept blocks = total length of col_idx. */
int64_t oracle_pack_count(const uint8_t *mask, int Cout, int Cin, int k, int V) {
    if (Cout <= 0 || Cin <= 0 || k <= 0 || V <= 0) return ORACLE_BAD_ARG;
    int64_t G = n_groups(Cout, V), K = (int64_t)Cin * k * k;
    if (!mask) return G * K;
    int64_t t = 0;
    for (int64_t i = 0; i < G * K; ++i) t += mask[i] != 0;
    return t;
}

/* Grouped CSR of Section 3.2.2 ("Storage format").  For every group, in ascending
 * order of the flattened column col = (c*k + r)*k + s of the stretched filter:
 * a kept column adds its offset (the number of columns in front of it, i.e. its
 * absolute 0-based position) and its V values, top row first.  row_ptr is the
 * running total of the per-group counts, so count_g = row_ptr[g+1] - row_ptr[g].
 * Rows of a ragged last group that lie beyond Cout are stored as +0.0f. */
int oracle_pack(const float *W, const uint8_t *mask, int Cout, int Cin, int k, int V,
                int32_t *row_ptr, int32_t *col_idx, float *vals) {
    if (!W || !row_ptr || Cout <= 0 || Cin <= 0 || k <= 0 || V <= 0) return ORACLE_BAD_ARG;
    int G = n_groups(Cout, V);
    int64_t K = (int64_t)Cin * k * k;
    int64_t t = 0;
    row_ptr[0] = 0;
    for (int g = 0; g < G; ++g) {
        for (int64_t col = 0; col < K; ++col) {
            int keep = mask ? (mask[(int64_t)g * K + col] != 0) : 1;
            if (!keep) continue;
            col_idx[t] = (int32_t)col;
            for (int v = 0; v < V; ++v) {
                int o = g * V + v;
                vals[t * V + v] = (o < Cout) ? W[(int64_t)o * K + col] : 0.0f;
            }
            ++t;
        }
        row_ptr[g + 1] = (int32_t)t;
    }
    return ORACLE_OK;
}

/* Inverse of oracle_pack: scatter the stored V-vectors back into a dense
 * [Cout, Cin*k*k] matrix that is zero everywhere else. */
int oracle_unpack(const int32_t *row_ptr, const int32_t *col_idx, const float *vals, int Cout,
                  int Cin, int k, int V, float *Wd) {
    if (!row_ptr || !Wd || Cout <= 0 || Cin <= 0 || k <= 0 || V <= 0) return ORACLE_BAD_ARG;
    int G = n_groups(Cout, V);
    int64_t K = (int64_t)Cin * k * k;
    memset(Wd, 0, sizeof(float) * (size_t)Cout * (size_t)K);
    for (int g = 0; g < G; ++g)
        for (int32_t t = row_ptr[g]; t < row_ptr[g + 1]; ++t) {
            int32_t col = col_idx[t];
            if (col < 0 || col >= K) return ORACLE_BAD_ARG;
            for (int v = 0; v < V; ++v) {
                int o = g * V + v;
                if (o < Cout) Wd[(int64_t)o * K + col] = vals[(int64_t)t * V + v];
            }
        }
    return ORACLE_OK;
}

/* The patch matrix I* of Section 3.2.2 for one image: row col = (c*k + r)*k + s,
 * column p = ho*Wo + wo, entry = the input value that filter position (c,r,s)
 * meets at output location (ho,wo), 0 where the window hangs over the border. */
int oracle_im2col(const float *X1, int Cin, int H, int Wi, int k, int stride, float *Istar) {
    if (!X1 || !Istar || (k % 2) == 0) return ORACLE_BAD_ARG;
    int pad = (k - 1) / 2;
    int Ho = out_size(H, k, stride), Wo = out_size(Wi, k, stride);
    int64_t P = (int64_t)Ho * Wo;
    for (int c = 0; c < Cin; ++c)
        for (int r = 0; r < k; ++r)
            for (int s = 0; s < k; ++s) {
                int64_t col = ((int64_t)c * k + r) * k + s;
                for (int ho = 0; ho < Ho; ++ho)
                    for (int wo = 0; wo < Wo; ++wo) {
                        int hi = ho * stride + r - pad, wi = wo * stride + s - pad;
                        float x = 0.0f;
                        if (hi >= 0 && hi < H && wi >= 0 && wi < Wi)
                            x = X1[((int64_t)c * H + hi) * Wi + wi];
                        Istar[col * P + (int64_t)ho * Wo + wo] = x;
                    }
            }
    return ORACLE_OK;
}

/* Second, independently organised evaluator that walks the paper's algorithm:
 * build I* explicitly, then for every filter group run as many iterations as the
 * group has kept columns; each iteration takes the column's V-vector of weights
 * and the row of I* its offset names, and accumulates their outer product
 * (Section 3.2.2, "Efficient multiplication computation").  Used by the tests to
 * cross-check oracle_conv on small cases; `scratch` must hold Cin*k*k*Ho*Wo
 * floats and `accbuf` V*Ho*Wo doubles. */
int oracle_conv_csr(const int32_t *row_ptr, const int32_t *col_idx, const float *vals,
                    const float *X, const float *bias, float *Y, int N, int Cin, int Cout, int H,
                    int Wi, int k, int stride, int V, float *scratch, double *accbuf) {
    if (!row_ptr || !X || !Y || !scratch || !accbuf) return ORACLE_BAD_ARG;
    int G = n_groups(Cout, V);
    int Ho = out_size(H, k, stride), Wo = out_size(Wi, k, stride);
    int64_t P = (int64_t)Ho * Wo;
    for (int n = 0; n < N; ++n) {
        int rc = oracle_im2col(X + (int64_t)n * Cin * H * Wi, Cin, H, Wi, k, stride, scratch);
        if (rc) return rc;
        for (int g = 0; g < G; ++g) {
            for (int64_t i = 0; i < (int64_t)V * P; ++i) accbuf[i] = 0.0;
            int32_t count = row_ptr[g + 1] - row_ptr[g];
            for (int32_t j = 0; j < count; ++j) {
                const float *wcol = vals + ((int64_t)row_ptr[g] + j) * V;
                const float *irow = scratch + (int64_t)col_idx[row_ptr[g] + j] * P;
                for (int v = 0; v < V; ++v)
                    for (int64_t p = 0; p < P; ++p)
                        accbuf[v * P + p] += (double)wcol[v] * (double)irow[p];
            }
            for (int v = 0; v < V; ++v) {
                int o = g * V + v;
                if (o >= Cout) continue;
                for (int64_t p = 0; p < P; ++p) {
                    double a = accbuf[v * P + p] + (bias ? (double)bias[o] : 0.0);
                    Y[((int64_t)n * Cout + o) * P + p] = (float)a;
                }
            }
        }
    }
    return ORACLE_OK;
}

/* Section 3.3, Eqs. (4)-(6).  k[0] < k[1] < ... < k[n-1] are the numbers of non-zero
 * weights at which the layer was timed and t[i] the run time measured at k[i].  The
 * estimate for s non-zero weights starts from t[0] and adds, for every interval i whose
 * left end s has reached (delta_i = 1), the slope alpha_i of that interval times the part
 * of the interval that lies below s.  Written term by term as the equation states it. */
double oracle_latency_estimate(const double *k, const double *t, int n, double s) {
    double est = t[0];
    for (int i = 0; i + 1 < n; ++i) {
        const double delta = s >= k[i] ? 1.0 : 0.0;                      /* Eq. (5) */
        const double alpha = (t[i + 1] - t[i]) / (k[i + 1] - k[i]);      /* Eq. (6) */
        const double whole = k[i + 1] - k[i], part = s - k[i];
        est += delta * alpha * (whole < part ? whole : part);            /* Eq. (4) */
    }
    return est;
}

/* Section 3.3, Eq. (2): tau plus the estimates of the L layers.  Layer l owns the n[l]
 * knots that start at k[first[l]], t[first[l]] (first[l] = n[0] + ... + n[l-1]) and has
 * s[l] non-zero weights. */
double oracle_network_latency(double tau, const double *k, const double *t, const int *n, int L,
                              const double *s) {
    double total = tau;
    int first = 0;
    for (int l = 0; l < L; ++l) {
        total += oracle_latency_estimate(k + first, t + first, n[l], s[l]);
        first += n[l];
    }
    return total;
}

int oracle_max_threads(void) {
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}
