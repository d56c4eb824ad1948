/*
 * PEQA oracle -- TEST INFRASTRUCTURE ONLY.
 *
 * A plain, slow, obviously-correct CPU statement of what the PEQA quantized
 * linear layer computes (arXiv 2305.14152).  It exists so that the GPU library
 * can be checked against something that shares no code with it.  Nothing in the
 * product path may include, link or call this file; only the tests, the smoke
 * check and the benchmark's cpu_baseline leg do.
 *
 * Every floating-point result is computed in fp64 from the exact input bits,
 * with one exception that is part of the definition: the quantizer (Eq. 1)
 * decides integer codes, so its arithmetic is fixed to IEEE fp32 with one
 * correctly rounded operation per step (compile with -ffp-contract=off and
 * without fast-math).  There is no blocking, fusion or reordering beyond the
 * definitions.  `#pragma omp parallel for` on an outermost independent loop
 * is the only concession to run time.
 *
 * Notation (paper Sec. 3.2): W0 in R^{N x K} (paper's n x m), b bits,
 * codes Q in {0..2^b-1}, zero-point z0, scale s0, frozen integer matrix
 * Wbar = Q - z0, trainable ds, effective scale s = s0 + ds.
 * Group-wise variant (paper Sec. 4.2, paragraph "Group-wise Quantization", Table 5): one (s, z)
 * per output channel per contiguous group of g input features; g = 0 means
 * one group spanning all K (per-channel).
 */
#include <math.h>
#include <stddef.h>
#include <stdint.h>
#include <string.h>

#ifdef _OPENMP
#include <omp.h>
#endif

int oracle_max_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

static int groups_of(int K, int group) { return group > 0 ? K / group : 1; }
static int gsize_of(int K, int group) { return group > 0 ? group : K; }

static int check_layout(int N, int K, int bits, int group)
{
    if (N <= 0 || K <= 0) return 2;
    if (bits != 3 && bits != 4) return 3;
    if (N % 8 != 0 || K % 8 != 0) return 2;
    if (group < 0) return 4;
    if (group > 0 && (K % group != 0 || group % 8 != 0)) return 4;
    return 0;
}

/* bf16 bit pattern -> the real number it denotes (exact). */
static double bf16_to_double(uint16_t h)
{
    uint32_t u = (uint32_t)h << 16;
    float f;
    memcpy(&f, &u, sizeof f);
    return (double)f;
}

/* ------------------------------------------------------------------------
 * Eq. 1: round-to-nearest asymmetric uniform quantizer, min-max range.
 *
 * For each output channel i and group g of input features:
 *   xmin = min(min_k w, 0), xmax = max(max_k w, 0)   (range widened to hold 0
 *                                   so that the zero-point is a storable code)
 *   s0 = (xmax - xmin) / (2^b - 1)
 *   z0 = rint(-xmin / s0)
 *   Q  = clamp(rint(w / s0) + z0, 0, 2^b - 1)
 * rint = round half to even.  If s0 evaluates to zero (all-zero group, or a
 * range so small that the quotient underflows) the group is degenerate:
 * s0 = 1, z0 = 0.
 * All of xmax - xmin, / qmax, -xmin / s0 and w / s0 are single fp32 operations.
 * Outputs: codes[N*K] (row-major, one byte per code), s0[N*G], z0[N*G].
 * ---------------------------------------------------------------------- */
int oracle_quantize(const float *W0, int N, int K, int bits, int group,
                    uint8_t *codes, float *s0, uint8_t *z0)
{
    int rc = check_layout(N, K, bits, group);
    if (rc) return rc;
    const int G = groups_of(K, group), gs = gsize_of(K, group);
    const int qmax = (1 << bits) - 1;
#pragma omp parallel for schedule(static)
    for (int i = 0; i < N; ++i) {
        for (int g = 0; g < G; ++g) {
            const float *w = W0 + (size_t)i * K + (size_t)g * gs;
            float xmin = 0.0f, xmax = 0.0f;
            for (int k = 0; k < gs; ++k) {
                if (w[k] < xmin) xmin = w[k];
                if (w[k] > xmax) xmax = w[k];
            }
            volatile float range = xmax - xmin;
            volatile float s = range / (float)qmax;
            int z;
            if (!(s > 0.0f)) {
                s = 1.0f;
                z = 0;
            } else {
                volatile float zr = -xmin / s;
                z = (int)rintf(zr);
                if (z < 0) z = 0;
                if (z > qmax) z = qmax;
            }
            s0[(size_t)i * G + g] = s;
            z0[(size_t)i * G + g] = (uint8_t)z;
            for (int k = 0; k < gs; ++k) {
                volatile float t = w[k] / s;
                int q = (int)rintf(t) + z;
                if (q < 0) q = 0;
                if (q > qmax) q = qmax;
                codes[(size_t)i * K + (size_t)g * gs + k] = (uint8_t)q;
            }
        }
    }
    return 0;
}

/* Sec. 3.2 wants s0, z0 initialised so that the Frobenius norm of W0 - What0 is smallest, but gives
 * no procedure (the experiments use plain round-to-nearest).  The usual procedure is a grid search over
 * clipped ranges, which is what this function states: for every (channel, group) and every
 * ratio r_j = 1 - j * step, step = (1 - min_ratio) / (n_ratios - 1), j = 0 .. n_ratios - 1
 * (r_0 = 1 is Eq. 1 as it stands):
 *   lo = r_j * xmin,  hi = r_j * xmax,  s = (hi - lo) / (2^b - 1),  z = rint(-lo / s),
 *   Q = clamp(rint(w / s) + z, 0, 2^b - 1)            (the degenerate rule as in Eq. 1)
 *   err_j = sum_k (w - s * (Q - z))^2
 * and the candidate with the smallest err_j (the first of equal ones) is kept.
 * Every step that decides a code is one fp32 operation, as in oracle_quantize; the residual
 * w - s * (Q - z) is formed in fp32 (one multiply, one subtract), squared and summed in fp64.
 * choice[N*G] (may be NULL) receives the index j that was kept. */
int oracle_quantize_search(const float *W0, int N, int K, int bits, int group,
                           int n_ratios, float min_ratio,
                           uint8_t *codes, float *s0, uint8_t *z0, int *choice)
{
    int rc = check_layout(N, K, bits, group);
    if (rc) return rc;
    if (n_ratios < 1 || !(min_ratio > 0.0f) || min_ratio > 1.0f) return 5;
    const int G = groups_of(K, group), gs = gsize_of(K, group);
    const int qmax = (1 << bits) - 1;
    volatile float span = 1.0f - min_ratio;
    volatile float step = n_ratios > 1 ? span / (float)(n_ratios - 1) : 0.0f;
#pragma omp parallel for schedule(static)
    for (int i = 0; i < N; ++i) {
        for (int g = 0; g < G; ++g) {
            const float *w = W0 + (size_t)i * K + (size_t)g * gs;
            float xmin = 0.0f, xmax = 0.0f;
            for (int k = 0; k < gs; ++k) {
                if (w[k] < xmin) xmin = w[k];
                if (w[k] > xmax) xmax = w[k];
            }
            double best_err = 0.0;
            float best_s = 1.0f;
            int best_z = 0, best_j = -1;
            for (int j = 0; j < n_ratios; ++j) {
                volatile float jf = (float)j * step;
                volatile float r = 1.0f - jf;
                volatile float lo = r * xmin;
                volatile float hi = r * xmax;
                volatile float range = hi - lo;
                volatile float s = range / (float)qmax;
                int z;
                if (!(s > 0.0f)) {
                    s = 1.0f;
                    z = 0;
                } else {
                    volatile float zr = -lo / s;
                    z = (int)rintf(zr);
                    if (z < 0) z = 0;
                    if (z > qmax) z = qmax;
                }
                double err = 0.0;
                for (int k = 0; k < gs; ++k) {
                    volatile float t = w[k] / s;
                    int q = (int)rintf(t) + z;
                    if (q < 0) q = 0;
                    if (q > qmax) q = qmax;
                    volatile float back = s * (float)(q - z);
                    volatile float d = w[k] - back;
                    err += (double)d * (double)d;
                }
                if (best_j < 0 || err < best_err) {
                    best_err = err; best_s = s; best_z = z; best_j = j;
                }
            }
            s0[(size_t)i * G + g] = best_s;
            z0[(size_t)i * G + g] = (uint8_t)best_z;
            if (choice) choice[(size_t)i * G + g] = best_j;
            for (int k = 0; k < gs; ++k) {
                volatile float t = w[k] / best_s;
                int q = (int)rintf(t) + best_z;
                if (q < 0) q = 0;
                if (q > qmax) q = qmax;
                codes[(size_t)i * K + (size_t)g * gs + k] = (uint8_t)q;
            }
        }
    }
    return 0;
}

/* The same quantizer evaluated in fp64 throughout: a sanity shadow of the
 * fp32 definition above (not a parity criterion).  s0 is returned as double. */
int oracle_quantize_f64(const float *W0, int N, int K, int bits, int group,
                        uint8_t *codes, double *s0, uint8_t *z0, double *frac)
{
    int rc = check_layout(N, K, bits, group);
    if (rc) return rc;
    const int G = groups_of(K, group), gs = gsize_of(K, group);
    const int qmax = (1 << bits) - 1;
    for (int i = 0; i < N; ++i) {
        for (int g = 0; g < G; ++g) {
            const float *w = W0 + (size_t)i * K + (size_t)g * gs;
            double xmin = 0.0, xmax = 0.0;
            for (int k = 0; k < gs; ++k) {
                if (w[k] < xmin) xmin = w[k];
                if (w[k] > xmax) xmax = w[k];
            }
            double s = (xmax - xmin) / (double)qmax;
            int z;
            if (!(s > 0.0)) { s = 1.0; z = 0; }
            else {
                z = (int)rint(-xmin / s);
                if (z < 0) z = 0;
                if (z > qmax) z = qmax;
            }
            s0[(size_t)i * G + g] = s;
            z0[(size_t)i * G + g] = (uint8_t)z;
            for (int k = 0; k < gs; ++k) {
                double t = (double)w[k] / s;
                int q = (int)rint(t) + z;
                if (q < 0) q = 0;
                if (q > qmax) q = qmax;
                size_t idx = (size_t)i * K + (size_t)g * gs + k;
                codes[idx] = (uint8_t)q;
                if (frac) frac[idx] = fabs(fabs(t - floor(t)) - 0.5); /* distance to a rounding tie */
            }
        }
    }
    return 0;
}

/* ------------------------------------------------------------------------
 * Dense b-bit storage of the codes (Sec. 3.3 "b-bit integer matrix"; Table 4's
 * model sizes fix the density at exactly b bits per weight).
 *
 * The paper does not say where each bit lives, so the placement is this
 * library's own, stated here as a closed-form map (i, k, bit) -> (word, bit):
 *
 * The N x K code matrix is cut into 8 x 8 blocks (8 output channels x 8 input
 * features), each owning 2*b consecutive 32-bit words.  Blocks are stored tile
 * by tile: a tile is 128 channels x 32 features = 16 x 4 blocks; tiles run
 * along the input features first, then down the channels, and inside a tile
 * the blocks run along the features first as well.  So block (ib, kb) =
 * (i/8, k/8) has number
 *     ((ib/16) * (K/32) + kb/4) * 64 + (ib%16) * 4 + kb%4
 * and starts at word number * 2*b.  (Packing therefore needs N % 128 == 0 and
 * K % 32 == 0.)  Inside a block, r = i%8, c = k%8.
 *
 *  b = 4: word r of the block holds channel r; feature c sits in nibble
 *         p = c/2 + 4*(c%2), i.e. bits [4p, 4p+4).  (Even features fill the low
 *         half-word, odd features the high half-word.)
 *
 *  b = 3: channels come in partner pairs (2*rho, 2*rho+1), features in pairs
 *         (2*pr, 2*pr+1).  u = 4*rho + pr in 0..15 numbers the (channel pair,
 *         feature pair) cells.  Parity par = r%2 picks the word of a word pair,
 *         half = c%2 picks the half-word:
 *           u < 15 : word 2*(u/5) + par, bits [16*half + 3*(u%5), +3)
 *           u = 15 : bit t of the code is bit 15 + 16*half of word 2*t + par
 *         (the one spare bit of every half-word collects the last cell).
 * ---------------------------------------------------------------------- */
size_t oracle_packed_words(int N, int K, int bits)
{
    return (size_t)N * (size_t)K * (size_t)bits / 32u;
}

int oracle_bit_location(int K, int bits, int i, int k, int t,
                        size_t *word, int *bit)
{
    const int ib = i / 8, kb = k / 8;
    const size_t tile = (size_t)(ib / 16) * (size_t)(K / 32) + (size_t)(kb / 4);
    const size_t blk = tile * 64 + (size_t)((ib % 16) * 4 + kb % 4);
    const int r = i % 8, c = k % 8;
    if (bits == 4) {
        const int p = c / 2 + 4 * (c % 2);
        *word = blk * 8 + (size_t)r;
        *bit = 4 * p + t;
        return 0;
    }
    if (bits == 3) {
        const int rho = r / 2, par = r % 2, pr = c / 2, half = c % 2;
        const int u = 4 * rho + pr;
        if (u < 15) {
            *word = blk * 6 + (size_t)(2 * (u / 5) + par);
            *bit = 16 * half + 3 * (u % 5) + t;
        } else {
            *word = blk * 6 + (size_t)(2 * t + par);
            *bit = 15 + 16 * half;
        }
        return 0;
    }
    return 3;
}

int oracle_pack(const uint8_t *codes, int N, int K, int bits, uint32_t *words)
{
    int rc = check_layout(N, K, bits, 0);
    if (rc) return rc;
    if (N % 128 != 0 || K % 32 != 0) return 2;
    memset(words, 0, oracle_packed_words(N, K, bits) * sizeof(uint32_t));
    for (int i = 0; i < N; ++i)
        for (int k = 0; k < K; ++k) {
            const unsigned q = codes[(size_t)i * K + k];
            if (q >> bits) return 3; /* code out of range for b bits */
            for (int t = 0; t < bits; ++t) {
                size_t w; int pos;
                oracle_bit_location(K, bits, i, k, t, &w, &pos);
                if ((q >> t) & 1u) words[w] |= (uint32_t)1u << pos;
            }
        }
    return 0;
}

int oracle_unpack(const uint32_t *words, int N, int K, int bits, uint8_t *codes)
{
    int rc = check_layout(N, K, bits, 0);
    if (rc) return rc;
    if (N % 128 != 0 || K % 32 != 0) return 2;
    for (int i = 0; i < N; ++i)
        for (int k = 0; k < K; ++k) {
            unsigned q = 0;
            for (int t = 0; t < bits; ++t) {
                size_t w; int pos;
                oracle_bit_location(K, bits, i, k, t, &w, &pos);
                q |= ((words[w] >> pos) & 1u) << t;
            }
            codes[(size_t)i * K + k] = (uint8_t)q;
        }
    return 0;
}

/* Eq. 2: What[i,k] = (s0 + ds)[i,g(k)] * (Q[i,k] - z0[i,g(k)]), fp64.
 * s = s0 + ds is formed in fp32 (both are fp32 parameters), then widened.
 * ds may be NULL (= 0). */
int oracle_dequant(const uint8_t *codes, const float *s0, const float *ds,
                   const uint8_t *z0, int N, int K, int group, double *What)
{
    const int G = groups_of(K, group), gs = gsize_of(K, group);
    for (int i = 0; i < N; ++i)
        for (int k = 0; k < K; ++k) {
            const size_t sg = (size_t)i * G + k / gs;
            volatile float s = ds ? s0[sg] + ds[sg] : s0[sg];
            What[(size_t)i * K + k] =
                (double)s * ((double)codes[(size_t)i * K + k] - (double)z0[sg]);
        }
    return 0;
}

/* Forward of Eq. 2:  Y[t,i] = sum_k X[t,k] * s[i,g(k)] * (Q[i,k] - z0[i,g(k)]).
 * X is bf16 (bit patterns), Y is fp64 [T,N]. */
int oracle_fwd(const uint8_t *codes, const float *s0, const float *ds,
               const uint8_t *z0, const uint16_t *X, int T, int N, int K,
               int group, double *Y)
{
    const int G = groups_of(K, group), gs = gsize_of(K, group);
#pragma omp parallel for schedule(static)
    for (int i = 0; i < N; ++i) {
        for (int t = 0; t < T; ++t) {
            double acc = 0.0;
            for (int k = 0; k < K; ++k) {
                const size_t sg = (size_t)i * G + k / gs;
                volatile float sf = ds ? s0[sg] + ds[sg] : s0[sg];
                const double w = (double)sf *
                    ((double)codes[(size_t)i * K + k] - (double)z0[sg]);
                acc += bf16_to_double(X[(size_t)t * K + k]) * w;
            }
            Y[(size_t)t * N + i] = acc;
        }
    }
    return 0;
}

/* Backward of Eq. 2 by the chain rule (the paper trains only the scales and
 * leaves the formulas implicit):
 *   dX[t,k]   = sum_i dY[t,i] * s[i,g(k)] * (Q[i,k] - z0[i,g(k)])
 *   dds[i,g]  = sum_t dY[t,i] * sum_{k in g} X[t,k] * (Q[i,k] - z0[i,g])
 * The scale gradient is evaluated twice, by two routes:
 *   dds_P: through P_g[t,i] = sum_{k in g} X[t,k] * Wbar[i,k]   (as written above)
 *   dds_W: through dWhat = dY^T X:  sum_{k in g} (sum_t dY[t,i] X[t,k]) * Wbar[i,k]
 * Any of dX, dds_P, dds_W may be NULL to skip it. */
int oracle_bwd(const uint8_t *codes, const float *s0, const float *ds,
               const uint8_t *z0, const uint16_t *X, const uint16_t *dY,
               int T, int N, int K, int group,
               double *dX, double *dds_P, double *dds_W)
{
    const int G = groups_of(K, group), gs = gsize_of(K, group);
    if (dX) {
#pragma omp parallel for schedule(static)
        for (int t = 0; t < T; ++t) {
            for (int k = 0; k < K; ++k) {
                double acc = 0.0;
                for (int i = 0; i < N; ++i) {
                    const size_t sg = (size_t)i * G + k / gs;
                    volatile float sf = ds ? s0[sg] + ds[sg] : s0[sg];
                    const double w = (double)sf *
                        ((double)codes[(size_t)i * K + k] - (double)z0[sg]);
                    acc += bf16_to_double(dY[(size_t)t * N + i]) * w;
                }
                dX[(size_t)t * K + k] = acc;
            }
        }
    }
    if (dds_P) {
#pragma omp parallel for schedule(static)
        for (int i = 0; i < N; ++i) {
            for (int g = 0; g < G; ++g) {
                double acc = 0.0;
                for (int t = 0; t < T; ++t) {
                    double P = 0.0;
                    for (int k = g * gs; k < (g + 1) * gs; ++k)
                        P += bf16_to_double(X[(size_t)t * K + k]) *
                             ((double)codes[(size_t)i * K + k] -
                              (double)z0[(size_t)i * G + g]);
                    acc += bf16_to_double(dY[(size_t)t * N + i]) * P;
                }
                dds_P[(size_t)i * G + g] = acc;
            }
        }
    }
    if (dds_W) {
#pragma omp parallel for schedule(static)
        for (int i = 0; i < N; ++i) {
            for (int g = 0; g < G; ++g) {
                double acc = 0.0;
                for (int k = g * gs; k < (g + 1) * gs; ++k) {
                    double dW = 0.0;
                    for (int t = 0; t < T; ++t)
                        dW += bf16_to_double(dY[(size_t)t * N + i]) *
                              bf16_to_double(X[(size_t)t * K + k]);
                    acc += dW * ((double)codes[(size_t)i * K + k] -
                                 (double)z0[(size_t)i * G + g]);
                }
                dds_W[(size_t)i * G + g] = acc;
            }
        }
    }
    return 0;
}

/* Appendix K ("Choice of Updating Quantization Scales or Zero-Points") also trains the
 * zero-points, alone or together with the scales.  The zero-point then is the real number
 * z = z0 + dz (dz fp32, same shape as the scales; the sum is formed in fp32 as for s), the
 * codes stay frozen, and Eq. 2 reads  What[i,k] = s[i,g(k)] * (Q[i,k] - z[i,g(k)]).
 * Forward with such zero-points; dz may be NULL (= 0). */
int oracle_fwd_z(const uint8_t *codes, const float *s0, const float *ds,
                 const uint8_t *z0, const float *dz, const uint16_t *X,
                 int T, int N, int K, int group, double *Y)
{
    const int G = groups_of(K, group), gs = gsize_of(K, group);
#pragma omp parallel for schedule(static)
    for (int i = 0; i < N; ++i) {
        for (int t = 0; t < T; ++t) {
            double acc = 0.0;
            for (int k = 0; k < K; ++k) {
                const size_t sg = (size_t)i * G + k / gs;
                volatile float sf = ds ? s0[sg] + ds[sg] : s0[sg];
                volatile float zf = dz ? (float)z0[sg] + dz[sg] : (float)z0[sg];
                const double w = (double)sf *
                    ((double)codes[(size_t)i * K + k] - (double)zf);
                acc += bf16_to_double(X[(size_t)t * K + k]) * w;
            }
            Y[(size_t)t * N + i] = acc;
        }
    }
    return 0;
}

/* Chain rule through that forward:
 *   dX[t,k]  = sum_i dY[t,i] * s[i,g(k)] * (Q[i,k] - z[i,g(k)])
 *   dds[i,g] = sum_t dY[t,i] * sum_{k in g} X[t,k] * (Q[i,k] - z[i,g])
 *   ddz[i,g] = sum_t dY[t,i] * sum_{k in g} X[t,k] * (-s[i,g])
 * (What depends on z only through the term -s*z).  Any output may be NULL. */
int oracle_bwd_z(const uint8_t *codes, const float *s0, const float *ds,
                 const uint8_t *z0, const float *dz, const uint16_t *X,
                 const uint16_t *dY, int T, int N, int K, int group,
                 double *dX, double *dds, double *ddz)
{
    const int G = groups_of(K, group), gs = gsize_of(K, group);
    if (dX) {
#pragma omp parallel for schedule(static)
        for (int t = 0; t < T; ++t) {
            for (int k = 0; k < K; ++k) {
                double acc = 0.0;
                for (int i = 0; i < N; ++i) {
                    const size_t sg = (size_t)i * G + k / gs;
                    volatile float sf = ds ? s0[sg] + ds[sg] : s0[sg];
                    volatile float zf = dz ? (float)z0[sg] + dz[sg] : (float)z0[sg];
                    const double w = (double)sf *
                        ((double)codes[(size_t)i * K + k] - (double)zf);
                    acc += bf16_to_double(dY[(size_t)t * N + i]) * w;
                }
                dX[(size_t)t * K + k] = acc;
            }
        }
    }
    if (dds || ddz) {
#pragma omp parallel for schedule(static)
        for (int i = 0; i < N; ++i) {
            for (int g = 0; g < G; ++g) {
                const size_t sg = (size_t)i * G + g;
                volatile float sf = ds ? s0[sg] + ds[sg] : s0[sg];
                volatile float zf = dz ? (float)z0[sg] + dz[sg] : (float)z0[sg];
                double acc_s = 0.0, acc_z = 0.0;
                for (int t = 0; t < T; ++t) {
                    double P = 0.0, R = 0.0;
                    for (int k = g * gs; k < (g + 1) * gs; ++k) {
                        const double x = bf16_to_double(X[(size_t)t * K + k]);
                        P += x * ((double)codes[(size_t)i * K + k] - (double)zf);
                        R += x;
                    }
                    const double d = bf16_to_double(dY[(size_t)t * N + i]);
                    acc_s += d * P;
                    acc_z += d * R * (-(double)sf);
                }
                if (dds) dds[sg] = acc_s;
                if (ddz) ddz[sg] = acc_z;
            }
        }
    }
    return 0;
}

/* One AdamW step on ds (Appendix A names AdamW; constants are call
 * parameters).  The decayed parameter is the actual scale s0 + ds, since the
 * paper trains the scale itself:
 *   m <- b1 m + (1-b1) g ;  v <- b2 v + (1-b2) g^2
 *   mhat = m / (1 - b1^step) ; vhat = v / (1 - b2^step)
 *   ds <- ds - lr * ( mhat / (sqrt(vhat) + eps) + wd * (s0 + ds) )
 * All in fp64; step is 1-based. */
int oracle_adamw(size_t n, double *ds, const double *g, double *m, double *v,
                 const double *s0, double lr, double b1, double b2, double eps,
                 double wd, int step)
{
    if (step < 1) return 2;
    const double c1 = 1.0 - pow(b1, (double)step);
    const double c2 = 1.0 - pow(b2, (double)step);
    for (size_t j = 0; j < n; ++j) {
        m[j] = b1 * m[j] + (1.0 - b1) * g[j];
        v[j] = b2 * v[j] + (1.0 - b2) * g[j] * g[j];
        const double mhat = m[j] / c1, vhat = v[j] / c2;
        ds[j] = ds[j] - lr * (mhat / (sqrt(vhat) + eps) + wd * (s0[j] + ds[j]));
    }
    return 0;
}
