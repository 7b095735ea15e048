/*
 * KVComm cache-reuse step: float64 CPU oracle.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, plain statement of what the
 * reuse step computes, written from the paper (arxiv 2510.12872).  It is used by
 * the tests, by the smoke check and by the benchmark's CPU-baseline leg; the
 * product (the HIP library) never calls it and shares no code, header, table or
 * helper with it.
 *
 * Everything is computed in double precision with plain nested loops in the
 * order the paper states the steps.  OpenMP only distributes independent outer
 * iterations (one token, or one (layer, head) pair, per thread); no reduction is
 * split across threads, so results do not depend on the thread count.
 *
 * Tensor convention: dense row-major arrays of double.
 *   key/value caches        [L, H, S, D]    (layer, kv head, token, channel)
 *   anchor a's tensors      [L, H, S_a, D]  (its own length S_a = anc_len[a])
 *   queries / outputs       [L, Hq, Tq, D]
 * Weight granularity `gran` (what the norm ||h_phi - h_psi|| is reduced over):
 *   0  per token            n = S         index t            (Appendix
 *        "Overhead in Long-context Anchor Matching": the reduction leaves the
 *        shape [m,1,1,seq_len,1])
 *   1  per layer/head/token n = L*H*S     index (l*H+h)*S+t
 *   2  per segment          n = 1         index 0            (scalar weights as
 *        used by the entropy in Eq. "pred")
 * Distances and weights are stored [A, n] (anchor-major, as in the paper's
 * [m, ..., seq_len, ...] shape).
 *
 * Parity pins: every function below is pinned by tests/test_oracle_*.py against
 * closed forms, numpy/scipy library routines and invariants.  Agreement with a
 * real model's dense prefill is "parity unpinned": the paper prints no worked
 * numeric example and no weights are available.
 */
#include <math.h>
#include <stddef.h>
#include <stdlib.h>

/* ------------------------------------------------------------------------- */
/* O1.  RoPE rotation by a position delta (Sec. 3.1 "Preliminaries": k_n = R_n W_K h_n;
 * Sec. 3.1 "Positional Alignment is Indispensable": keys at positions n and
 * n+Delta differ by the orthogonal rotation R_Delta).
 * Half-split pairing: channel i is paired with channel i + D/2, and the pair
 * turns by the angle Delta * theta^(-2i/D).                                  */
void kvo_rope_rotate(const double *x, double *y, int D, double delta, double theta)
{
    int half = D / 2;
    for (int i = 0; i < half; ++i) {
        double freq = pow(theta, -2.0 * (double)i / (double)D);
        double phi = delta * freq;
        double c = cos(phi), s = sin(phi);
        double a = x[i], b = x[i + half];
        y[i] = a * c - b * s;
        y[i + half] = b * c + a * s;
    }
}

/* Which slot of a [A, n] distance/weight array belongs to (l, h, t). */
static size_t gran_index(int gran, int H, int S, int l, int h, int t)
{
    if (gran == 0) return (size_t)t;
    if (gran == 1) return ((size_t)l * H + h) * S + t;
    return 0;
}

static size_t gran_count(int gran, int L, int H, int S)
{
    if (gran == 0) return (size_t)S;
    if (gran == 1) return (size_t)L * H * S;
    return 1;
}

/* ------------------------------------------------------------------------- */
/* O2.  Anchor selection and distances (Eq. "pred": A_phi holds the anchors at
 * least as long as the sample; Eq. "ph_update": ||h_phi - h_psi||, with h the
 * base key cache).  Only the first S tokens of a longer anchor are compared.
 *   selected[a] = (anc_len[a] >= S)
 *   dist[a, j]  = sqrt( sum over the (l,h,t,i) that map to slot j of
 *                        (seg_k - anc_k[a])^2 )      for selected anchors,
 *                 0 for the others (never read afterwards).                  */
void kvo_distances(const double *seg_k, const double *const *anc_k, const int *anc_len,
                   int A, int L, int H, int S, int D, int gran,
                   double *dist, int *selected)
{
    size_t n = gran_count(gran, L, H, S);
    for (int a = 0; a < A; ++a) {
        selected[a] = (anc_len[a] >= S) ? 1 : 0;
        for (size_t j = 0; j < n; ++j) dist[(size_t)a * n + j] = 0.0;
    }
    for (int a = 0; a < A; ++a) {
        if (!selected[a]) continue;
        int Sa = anc_len[a];
        const double *ak = anc_k[a];
        double *da = dist + (size_t)a * n;
        if (gran == 2) {
            double acc = 0.0;
            for (int l = 0; l < L; ++l)
                for (int h = 0; h < H; ++h)
                    for (int t = 0; t < S; ++t)
                        for (int i = 0; i < D; ++i) {
                            double u = seg_k[(((size_t)l * H + h) * S + t) * D + i];
                            double w = ak[(((size_t)l * H + h) * Sa + t) * D + i];
                            acc += (u - w) * (u - w);
                        }
            da[0] = sqrt(acc);
        } else if (gran == 1) {
#pragma omp parallel for collapse(2) schedule(static)
            for (int l = 0; l < L; ++l)
                for (int h = 0; h < H; ++h)
                    for (int t = 0; t < S; ++t) {
                        double acc = 0.0;
                        for (int i = 0; i < D; ++i) {
                            double u = seg_k[(((size_t)l * H + h) * S + t) * D + i];
                            double w = ak[(((size_t)l * H + h) * Sa + t) * D + i];
                            acc += (u - w) * (u - w);
                        }
                        da[gran_index(1, H, S, l, h, t)] = sqrt(acc);
                    }
        } else {
#pragma omp parallel for schedule(static)
            for (int t = 0; t < S; ++t) {
                double acc = 0.0;
                for (int l = 0; l < L; ++l)
                    for (int h = 0; h < H; ++h)
                        for (int i = 0; i < D; ++i) {
                            double u = seg_k[(((size_t)l * H + h) * S + t) * D + i];
                            double w = ak[(((size_t)l * H + h) * Sa + t) * D + i];
                            acc += (u - w) * (u - w);
                        }
                da[t] = sqrt(acc);
            }
        }
    }
}

/* ------------------------------------------------------------------------- */
/* O3.  Weights: softmax of the negative distance across the anchor dimension
 * (Eq. "pred", Eq. "ph_update", the weight step of Algorithm 1), with a
 * temperature tau (the paper's rule is tau = 1).
 *   w[a, j] = exp(-(d[a,j] - dmin[j]) / tau) / sum_{a' selected} exp(-(d[a',j] - dmin[j]) / tau)
 * Unselected anchors get exactly 0.  nearest[j] is the selected anchor of
 * smallest distance, the lowest index among equals; -1 when none is selected
 * (then all weights of that slot are 0).                                      */
void kvo_weights(const double *dist, const int *selected, int A, size_t n, double tau,
                 double *w, int *nearest)
{
    for (size_t j = 0; j < n; ++j) {
        int best = -1;
        double dmin = 0.0;
        for (int a = 0; a < A; ++a) {
            if (!selected[a]) continue;
            double d = dist[(size_t)a * n + j];
            if (best < 0 || d < dmin) { best = a; dmin = d; }
        }
        nearest[j] = best;
        double denom = 0.0;
        for (int a = 0; a < A; ++a) {
            if (!selected[a]) continue;
            denom += exp(-(dist[(size_t)a * n + j] - dmin) / tau);
        }
        for (int a = 0; a < A; ++a) {
            if (!selected[a]) { w[(size_t)a * n + j] = 0.0; continue; }
            w[(size_t)a * n + j] = exp(-(dist[(size_t)a * n + j] - dmin) / tau) / denom;
        }
    }
}

/* ------------------------------------------------------------------------- */
/* O4.  Offset approximation (Eq. "ph_update"; Eq. "pf_update" is the same rule
 * applied to the neighbouring prefix segment's tensors with the placeholder's
 * weights).  The key is first rotated to its new position and only then receives
 * the estimated offset (Introduction, the paragraph on offset variance; Glossary
 * entry on key alignment).
 *   K^[l,h,t,:] = R_delta K[l,h,t,:] + sum_a w[a,j] * R_(delta - anc_delta[a]) dK_a[l,h,t,:]
 *   V^[l,h,t,:] =         V[l,h,t,:] + sum_a w[a,j] *                           dV_a[l,h,t,:]
 * An anchor's stored key deviation lives in the frame of the position delta it
 * was recorded at (anc_delta[a]); anc_delta == NULL means every anchor was
 * recorded at `delta`, which is exactly "rotate the base key, then add".
 * The sum runs over selected anchors only (anc_len[a] >= S).                  */
void kvo_align(const double *base_k, const double *base_v,
               const double *const *anc_dk, const double *const *anc_dv, const int *anc_len,
               const double *w, int gran, int A, int L, int H, int S, int D,
               double delta, const double *anc_delta, double theta,
               double *out_k, double *out_v)
{
    size_t n = gran_count(gran, L, H, S);
#pragma omp parallel for collapse(2) schedule(static)
    for (int l = 0; l < L; ++l)
        for (int h = 0; h < H; ++h) {
            double *rot = (double *)malloc(sizeof(double) * (size_t)D);
            for (int t = 0; t < S; ++t) {
                size_t row = (((size_t)l * H + h) * S + t) * D;
                size_t j = gran_index(gran, H, S, l, h, t);
                kvo_rope_rotate(base_k + row, rot, D, delta, theta);
                for (int i = 0; i < D; ++i) {
                    out_k[row + i] = rot[i];
                    out_v[row + i] = base_v[row + i];
                }
                for (int a = 0; a < A; ++a) {
                    if (anc_len[a] < S) continue;
                    size_t arow = (((size_t)l * H + h) * anc_len[a] + t) * D;
                    double wa = w[(size_t)a * n + j];
                    double rel = anc_delta ? (delta - anc_delta[a]) : 0.0;
                    kvo_rope_rotate(anc_dk[a] + arow, rot, D, rel, theta);
                    for (int i = 0; i < D; ++i) {
                        out_k[row + i] += wa * rot[i];
                        out_v[row + i] += wa * anc_dv[a][arow + i];
                    }
                }
            }
            free(rot);
        }
}

/* ------------------------------------------------------------------------- */
/* O5.  Causal attention of the Tq suffix queries over the assembled cache
 * (workflow step 4: the concatenated caches feed decoding; Sec. 3.1
 * defines q, k, v).  Query i of the suffix sits at cache position n_ctx + i and
 * sees keys 0 .. n_ctx + i.  Query head hq reads kv head hq / (Hq / Hkv).
 *   s_j = scale * <q_i, k_j>,  p = softmax_j(s),  o_i = sum_j p_j v_j
 *   lse_i = log sum_j exp(s_j)        (may be NULL)                           */
void kvo_suffix_attn(const double *q, const double *k, const double *v,
                     int L, int Hq, int Hkv, int D, int n_ctx, int tq, double scale,
                     double *out, double *lse)
{
    int N = n_ctx + tq;
    int G = Hq / Hkv;
#pragma omp parallel for collapse(2) schedule(static)
    for (int l = 0; l < L; ++l)
        for (int hq = 0; hq < Hq; ++hq) {
            int hk = hq / G;
            const double *kk = k + ((size_t)l * Hkv + hk) * N * D;
            const double *vv = v + ((size_t)l * Hkv + hk) * N * D;
            double *s = (double *)malloc(sizeof(double) * (size_t)N);
            for (int i = 0; i < tq; ++i) {
                const double *qi = q + (((size_t)l * Hq + hq) * tq + i) * D;
                double *oi = out + (((size_t)l * Hq + hq) * tq + i) * D;
                int last = n_ctx + i;
                double smax = 0.0;
                for (int j = 0; j <= last; ++j) {
                    double dot = 0.0;
                    for (int c = 0; c < D; ++c) dot += qi[c] * kk[(size_t)j * D + c];
                    s[j] = scale * dot;
                    if (j == 0 || s[j] > smax) smax = s[j];
                }
                double denom = 0.0;
                for (int j = 0; j <= last; ++j) denom += exp(s[j] - smax);
                for (int c = 0; c < D; ++c) oi[c] = 0.0;
                for (int j = 0; j <= last; ++j) {
                    double p = exp(s[j] - smax) / denom;
                    for (int c = 0; c < D; ++c) oi[c] += p * vv[(size_t)j * D + c];
                }
                if (lse) lse[((size_t)l * Hq + hq) * tq + i] = smax + log(denom);
            }
            free(s);
        }
}

/* Number of OpenMP threads the loops above will use (for the benchmark report). */
#ifdef _OPENMP
#include <omp.h>
int kvo_num_threads(void) { return omp_get_max_threads(); }
#else
int kvo_num_threads(void) { return 1; }
#endif

/* ------------------------------------------------------------------------- */
/* O6.  Offset capture (fallback branch of Algorithm 1: after a dense generation the
 * offset between the real and the base KV-cache of a placeholder, and of its
 * neighbouring prefix segment, fills a new anchor).  The deviation is stored in
 * the frame of the position delta it was recorded at, i.e. the inverse of O4
 * with a single anchor of weight 1:
 *   dK[l,h,t,:] = K_real[l,h,t,:] - R_delta K_base[l,h,t,:]
 *   dV[l,h,t,:] = V_real[l,h,t,:] -         V_base[l,h,t,:]                   */
void kvo_capture(const double *base_k, const double *base_v, const double *real_k, const double *real_v,
                 int L, int H, int S, int D, double delta, double theta, double *dk, double *dv)
{
#pragma omp parallel for collapse(2) schedule(static)
    for (int l = 0; l < L; ++l)
        for (int h = 0; h < H; ++h) {
            double *rot = (double *)malloc(sizeof(double) * (size_t)D);
            for (int t = 0; t < S; ++t) {
                size_t row = (((size_t)l * H + h) * S + t) * D;
                kvo_rope_rotate(base_k + row, rot, D, delta, theta);
                for (int i = 0; i < D; ++i) {
                    dk[row + i] = real_k[row + i] - rot[i];
                    dv[row + i] = real_v[row + i] - base_v[row + i];
                }
            }
            free(rot);
        }
}

/* ------------------------------------------------------------------------- */
/* O7.  Anchor prediction (Eq. "pred"): a sample becomes a new anchor when it is
 * longer than every anchor of the pool, or when the entropy of its weights over
 * the candidate anchors exceeds gamma * log |A_phi|.  The printed entropy lacks
 * its minus sign (it would be <= 0 and never exceed a non-negative threshold);
 * the sensitivity table (reuse rising with gamma) fixes H = - sum w log w.
 *   entropy[j] = - sum_{a selected, w > 0} w[a,j] log w[a,j]      per weight slot
 * The decision compares the mean entropy over the n slots (n = 1 for per-segment
 * weights, which is the paper's scalar case).  Returns 1 = new anchor, 0 = shareable.
 * An empty candidate set (no anchor as long as the sample) is case one.       */
int kvo_predict(const double *w, const int *selected, const int *anc_len, int A, size_t n,
                int seg_len, double gamma, double *entropy, double *mean_entropy)
{
    int n_sel = 0, max_len = 0;
    for (int a = 0; a < A; ++a) {
        if (selected[a]) ++n_sel;
        if (anc_len[a] > max_len) max_len = anc_len[a];
    }
    double sum = 0.0;
    for (size_t j = 0; j < n; ++j) {
        double hj = 0.0;
        for (int a = 0; a < A; ++a) {
            double x = w[(size_t)a * n + j];
            if (selected[a] && x > 0.0) hj -= x * log(x);
        }
        entropy[j] = hj;
        sum += hj;
    }
    *mean_entropy = n ? sum / (double)n : 0.0;
    if (seg_len > max_len) return 1;
    if (n_sel == 0) return 1;
    return (*mean_entropy > gamma * log((double)n_sel)) ? 1 : 0;
}

/* ------------------------------------------------------------------------- */
/* O8.  Weighting variants of the approximation-method ablation (appendix "Analysis
 * on the Approximation Method"):
 *   nearest: the whole weight goes to the selected anchor of smallest l2 distance
 *            (lowest index among equals);
 *   cosine : softmax across anchors of the cosine similarity between the segment's
 *            and the anchor's base keys, reduced over the same axes as the distance.
 * kvo_cosine writes sim[a, j] = <x, y> / (|x| |y|) for selected anchors (0 when a
 * norm is 0) and 0 for the others; kvo_weights_from_sim turns similarities into
 * softmax(sim / tau) over selected anchors; kvo_weights_nearest builds the one-hot. */
void kvo_cosine(const double *seg_k, const double *const *anc_k, const int *anc_len,
                int A, int L, int H, int S, int D, int gran, double *sim, int *selected)
{
    size_t n = gran_count(gran, L, H, S);
    double *dot = (double *)malloc(sizeof(double) * n);
    double *nx = (double *)malloc(sizeof(double) * n);
    double *ny = (double *)malloc(sizeof(double) * n);
    for (int a = 0; a < A; ++a) {
        selected[a] = (anc_len[a] >= S) ? 1 : 0;
        for (size_t j = 0; j < n; ++j) sim[(size_t)a * n + j] = 0.0;
        if (!selected[a]) continue;
        for (size_t j = 0; j < n; ++j) dot[j] = nx[j] = ny[j] = 0.0;
        int Sa = anc_len[a];
        for (int l = 0; l < L; ++l)
            for (int h = 0; h < H; ++h)
                for (int t = 0; t < S; ++t) {
                    size_t j = gran_index(gran, H, S, l, h, t);
                    for (int i = 0; i < D; ++i) {
                        double u = seg_k[(((size_t)l * H + h) * S + t) * D + i];
                        double v = anc_k[a][(((size_t)l * H + h) * Sa + t) * D + i];
                        dot[j] += u * v;
                        nx[j] += u * u;
                        ny[j] += v * v;
                    }
                }
        for (size_t j = 0; j < n; ++j) {
            double den = sqrt(nx[j]) * sqrt(ny[j]);
            sim[(size_t)a * n + j] = den > 0.0 ? dot[j] / den : 0.0;
        }
    }
    free(dot);
    free(nx);
    free(ny);
}

void kvo_weights_from_sim(const double *sim, const int *selected, int A, size_t n, double tau,
                          double *w, int *best_out)
{
    for (size_t j = 0; j < n; ++j) {
        int best = -1;
        double smax = 0.0;
        for (int a = 0; a < A; ++a) {
            if (!selected[a]) continue;
            double x = sim[(size_t)a * n + j];
            if (best < 0 || x > smax) { best = a; smax = x; }
        }
        best_out[j] = best;
        double denom = 0.0;
        for (int a = 0; a < A; ++a)
            if (selected[a]) denom += exp((sim[(size_t)a * n + j] - smax) / tau);
        for (int a = 0; a < A; ++a)
            w[(size_t)a * n + j] = selected[a] ? exp((sim[(size_t)a * n + j] - smax) / tau) / denom : 0.0;
    }
}

void kvo_weights_nearest(const double *dist, const int *selected, int A, size_t n, double *w, int *nearest)
{
    for (size_t j = 0; j < n; ++j) {
        int best = -1;
        double dmin = 0.0;
        for (int a = 0; a < A; ++a) {
            if (!selected[a]) continue;
            double d = dist[(size_t)a * n + j];
            if (best < 0 || d < dmin) { best = a; dmin = d; }
        }
        nearest[j] = best;
        for (int a = 0; a < A; ++a) w[(size_t)a * n + j] = (a == best) ? 1.0 : 0.0;
    }
}

/* ------------------------------------------------------------------------- */
/* O9.  Compressed anchor deviations (the appendix on memory cost notes that the deviation
 * tensors are small in magnitude, about half of the elements below 0.1, and names their
 * compression as future work).  Storage format used here: one byte per element in the OCP
 * 8-bit floating-point format E4M3 (1 sign, 4 exponent bits with bias 7, 3 mantissa bits; no
 * infinities; S.1111.111 is NaN; largest finite value 448; subnormals m/8 * 2^-6), times a
 * power-of-two scale per tensor:  value = scale * e4m3(byte).
 * Encoding rounds x / scale to the nearest representable value, ties to the even mantissa,
 * and saturates at +-448.  This is lossy: relative error at most 2^-4 for |x| >= scale * 2^-6,
 * absolute error at most scale * 2^-10 below that.                                          */
double kvo_e4m3_decode(unsigned char b)
{
    int sign = b >> 7, e = (b >> 3) & 15, m = b & 7;
    double v;
    if (e == 15 && m == 7) return NAN;
    if (e == 0) v = ldexp((double)m / 8.0, -6);
    else v = ldexp(1.0 + (double)m / 8.0, e - 7);
    return sign ? -v : v;
}

unsigned char kvo_e4m3_encode(double x)
{
    if (isnan(x)) return 0x7f;
    unsigned char sign = (unsigned char)(signbit(x) ? 0x80 : 0x00);
    double a = fabs(x);
    if (a >= 448.0) return (unsigned char)(sign | 0x7e);
    /* spacing of the grid around a: 2^-9 in the subnormal range and the first binade, else 2^(floor(log2 a) - 3) */
    int ex;
    (void)frexp(a, &ex);          /* a = f * 2^ex, f in [0.5, 1)  ->  floor(log2 a) = ex - 1 */
    int e_unb = ex - 1;
    if (a == 0.0 || e_unb < -6) e_unb = -6;
    double step = ldexp(1.0, e_unb - 3);
    double q = a / step;          /* exact: division by a power of two */
    double r = floor(q);
    double frac = q - r;
    if (frac > 0.5 || (frac == 0.5 && fmod(r, 2.0) == 1.0)) r += 1.0;
    double v = r * step;          /* a grid point, possibly the first of the next binade */
    /* turn the value back into bits by searching the (monotone) code table: plain and obviously right */
    for (int code = 0; code < 0x7f; ++code)
        if (kvo_e4m3_decode((unsigned char)code) == v) return (unsigned char)(sign | code);
    return (unsigned char)(sign | 0x7e);
}

void kvo_quantize(const double *x, size_t n, double scale, unsigned char *out)
{
    for (size_t i = 0; i < n; ++i) out[i] = kvo_e4m3_encode(x[i] / scale);
}

void kvo_dequantize(const unsigned char *b, size_t n, double scale, double *out)
{
    for (size_t i = 0; i < n; ++i) out[i] = scale * kvo_e4m3_decode(b[i]);
}
