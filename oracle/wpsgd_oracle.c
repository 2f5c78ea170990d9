/*
 * WP-SGD reference oracle -- TEST INFRASTRUCTURE, NOT PART OF THE PRODUCT PATH.
 *
 * A plain, slow, double-precision CPU implementation of what the GPU library
 * computes.  Nothing here is shared with the HIP sources: no headers, no
 * helpers, no tables.  It is written to be checked against the paper by eye:
 * no blocking, no fusion, no reordering beyond what the definitions state.
 *
 * What it follows (weighted parallel SGD, arXiv 1708.04801):
 *   - per-example objective  c^i(w) = lambda/2 |w|^2 + L(x^i, y^i, w.x^i)   (Eq. 4)
 *   - sequential SGD step    w_n = w_{n-1} - eta * d/dw c^i(w_{n-1})        (Eq. 5)
 *   - k chains of unequal length followed by one weighted sum           (Algorithm 1)
 *   - weight_i = (1-eta*lambda)^{T_i} / sum_j (1-eta*lambda)^{T_j}          (Eq. 6)
 *     with T_i the delay of chain i behind the fastest chain (Table I)
 *   - weight_i = r^{T_i} / sum_j r^{T_j} for a chosen contraction rate r    (Eq. 8)
 *   - benefit condition  2 sum_i rate^{T_i} > sqrt(k) + k      (Eq. 7 / Eq. 9, Cor. 3/4)
 *   - delayed-gradient server with its acceptance test    (Algorithms 3 and 4, Lemma 4)
 *
 * The paper does not define how a chain picks its n-th example beyond
 * "partition, shuffle, take the n-th"; this implementation replaces that by a
 * counter-based stream: Philox4x32-10 (Salmon, Moraes, Dror, Shaw, SC'11)
 * keyed by the seed, counter = (step, chain), first output word mapped to
 * [0, m) by multiply-shift.  Both sides implement it from the published
 * definition.
 *
 * Parity pins live in tests/test_oracle_pins.py (known-answer Philox vectors,
 * hand-computed weights, closed forms of the SGD recursion, finite-difference
 * gradient checks, brute force; for Algorithms 3/4 the scalar recurrence printed in the proof of
 * Lemma 4, the reduction to Eq. 5 at delay 0, and hand cases of the acceptance test).  Parity
 * unpinned: nothing in this file.
 *
 * Build: gcc -O2 -std=c11 -shared -fPIC -pthread wpsgd_oracle.c -o libwpsgd_oracle.so -lm
 */
#include <math.h>
#include <pthread.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#define ORACLE_OK 0
#define ORACLE_BAD_ARG (-1)
#define ORACLE_NO_MEM (-2)

enum { ORACLE_HINGE = 0, ORACLE_LOGISTIC = 1 };
enum { ORACLE_F32 = 0, ORACLE_BF16 = 1, ORACLE_F64 = 2 };

/* ------------------------------------------------------------------ */
/* Philox4x32-10, from the published definition (SC'11, section 3.3):  */
/* one round maps (c0,c1,c2,c3) with round key (k0,k1) to              */
/*   (hi(M1*c2)^c1^k0, lo(M1*c2), hi(M0*c0)^c3^k1, lo(M0*c0));         */
/* the key is bumped by the Weyl constants between rounds.             */
/* ------------------------------------------------------------------ */
void oracle_philox4x32_10(const uint32_t ctr[4], const uint32_t key[2], uint32_t out[4])
{
    const uint64_t M0 = 0xD2511F53u, M1 = 0xCD9E8D57u;
    const uint32_t W0 = 0x9E3779B9u, W1 = 0xBB67AE85u;
    uint32_t c0 = ctr[0], c1 = ctr[1], c2 = ctr[2], c3 = ctr[3];
    uint32_t k0 = key[0], k1 = key[1];
    for (int round = 0; round < 10; ++round) {
        uint64_t p0 = M0 * (uint64_t)c0;
        uint64_t p1 = M1 * (uint64_t)c2;
        uint32_t n0 = (uint32_t)(p1 >> 32) ^ c1 ^ k0;
        uint32_t n1 = (uint32_t)p1;
        uint32_t n2 = (uint32_t)(p0 >> 32) ^ c3 ^ k1;
        uint32_t n3 = (uint32_t)p0;
        c0 = n0; c1 = n1; c2 = n2; c3 = n3;
        k0 += W0; k1 += W1;
    }
    out[0] = c0; out[1] = c1; out[2] = c2; out[3] = c3;
}

/* Row visited by chain `chain` at step `n` (0-based):
 * counter = (n mod 2^32, n div 2^32, chain, 0), key = (seed mod 2^32, seed div 2^32),
 * j = floor(word0 * m / 2^32).  Needs 1 <= m < 2^32. */
int64_t oracle_sample_index(uint64_t seed, uint32_t chain, uint64_t n, int64_t m)
{
    uint32_t ctr[4] = { (uint32_t)(n & 0xffffffffu), (uint32_t)(n >> 32), chain, 0u };
    uint32_t key[2] = { (uint32_t)(seed & 0xffffffffu), (uint32_t)(seed >> 32) };
    uint32_t out[4];
    oracle_philox4x32_10(ctr, key, out);
    return (int64_t)(((uint64_t)out[0] * (uint64_t)m) >> 32);
}

int oracle_sample_indices(uint64_t seed, int64_t chain, int64_t n0, int64_t count,
                          int64_t m, int64_t *out)
{
    if (!out || count < 0 || n0 < 0 || chain < 0 || chain > 0xffffffffLL) return ORACLE_BAD_ARG;
    if (m < 1 || m > 0xffffffffLL) return ORACLE_BAD_ARG;
    for (int64_t t = 0; t < count; ++t)
        out[t] = oracle_sample_index(seed, (uint32_t)chain, (uint64_t)(n0 + t), m);
    return ORACLE_OK;
}

/* ------------------------------------------------------------------ */
/* Sampling as Algorithm 1 states it: "randomly partition the          */
/* examples, giving each node its share; randomly shuffle the data on  */
/* each node; get the n-th example".  Counter-based version: a keyed   */
/* permutation P of {0..m-1} shuffles all rows once; node i of k owns   */
/* the positions lo_i = floor(i*m/k) .. floor((i+1)*m/k) - 1 of the     */
/* shuffled order and reads them one after the other (wrapping round   */
/* if it is asked for more steps than it has rows):                    */
/*     row(i, n) = P(lo_i + n mod m_i).                                */
/* P is a 4-round Feistel network on 2h-bit numbers, h = ceil(b/2) with */
/* b the bit length of m-1 (h >= 1); round r sends (L, R) to            */
/* (R, L xor low_h(F_r(R))) with F_r(R) the first output word of        */
/* Philox4x32-10 on counter (R, r, 0x5348524D, 0xFFFFFFFF) and the      */
/* seed as key.  A result >= m is fed through the network again        */
/* (cycle walking), which keeps P a permutation of {0..m-1}.           */
/* ------------------------------------------------------------------ */
static uint32_t shuffle_position(uint64_t seed, uint32_t pos, uint32_t m)
{
    int bits = 0;
    for (uint32_t t = m - 1; t; t >>= 1) ++bits;
    int h = (bits + 1) / 2;
    if (h < 1) h = 1;
    const uint32_t low = ((uint32_t)1 << h) - 1u;
    uint32_t key[2] = { (uint32_t)(seed & 0xffffffffu), (uint32_t)(seed >> 32) };
    uint32_t x = pos;
    for (;;) {
        uint32_t left = x >> h, right = x & low;
        for (uint32_t round = 0; round < 4; ++round) {
            uint32_t ctr[4] = { right, round, 0x5348524Du, 0xFFFFFFFFu };
            uint32_t out[4];
            oracle_philox4x32_10(ctr, key, out);
            uint32_t next_right = left ^ (out[0] & low);
            left = right;
            right = next_right;
        }
        x = (left << h) | right;
        if (x < m) return x;
    }
}

int64_t oracle_shard_index(uint64_t seed, int64_t chain, int64_t k, uint64_t n, int64_t m)
{
    uint64_t lo = ((uint64_t)chain * (uint64_t)m) / (uint64_t)k;
    uint64_t hi = ((uint64_t)(chain + 1) * (uint64_t)m) / (uint64_t)k;
    uint64_t own = hi - lo;
    return (int64_t)shuffle_position(seed, (uint32_t)(lo + n % own), (uint32_t)m);
}

int oracle_shard_indices(uint64_t seed, int64_t chain, int64_t k, int64_t n0, int64_t count,
                         int64_t m, int64_t *out)
{
    if (!out || count < 0 || n0 < 0 || k < 1 || chain < 0 || chain >= k) return ORACLE_BAD_ARG;
    if (m < 1 || m > 0xffffffffLL || k > m) return ORACLE_BAD_ARG;
    for (int64_t t = 0; t < count; ++t)
        out[t] = oracle_shard_index(seed, chain, k, (uint64_t)(n0 + t), m);
    return ORACLE_OK;
}

/* ------------------------------------------------------------------ */
/* Stored value -> double, exactly.                                    */
/* ------------------------------------------------------------------ */
static double bf16_to_double(uint16_t h)
{
    uint32_t bits = (uint32_t)h << 16; /* bfloat16 is the top half of a binary32 */
    float f;
    memcpy(&f, &bits, sizeof f);
    return (double)f;
}

static double dense_at(const void *X, int xtype, int64_t ld, int64_t row, int64_t col)
{
    switch (xtype) {
    case ORACLE_F32:  return (double)((const float *)X)[row * ld + col];
    case ORACLE_BF16: return bf16_to_double(((const uint16_t *)X)[row * ld + col]);
    default:          return ((const double *)X)[row * ld + col];
    }
}

/* dL/dyhat for the two losses (L is a convex function of yhat = w.x, Eq. 4):
 *   hinge    L = max(0, 1 - y*yhat)      -> -y where y*yhat < 1, else 0
 *                                           (0 is taken at the kink y*yhat == 1)
 *   logistic L = log(1 + exp(-y*yhat))   -> -y / (1 + exp(y*yhat))               */
static double loss_slope(int loss, double y, double yhat)
{
    if (loss == ORACLE_HINGE)
        return (y * yhat < 1.0) ? -y : 0.0;
    return -y / (1.0 + exp(y * yhat));
}

/* ------------------------------------------------------------------ */
/* One chain, dense rows, explicit visit order idx[0..n).              */
/* w (length d) is read as w_0 and overwritten with w_n.               */
/* Eq. 5 with Eq. 4:  w_n = (1 - eta*lambda) w_{n-1} - eta * g * x,    */
/* g = dL/dyhat at yhat = w_{n-1}.x (the whole gradient, including the */
/* regulariser's lambda*w, is taken at w_{n-1}).                       */
/* min_margin (optional) receives min over steps of |1 - y*yhat|: how  */
/* close the hinge decision ever came to its kink.                     */
/* ------------------------------------------------------------------ */
int oracle_sgd_dense(const void *X, int xtype, int64_t m, int64_t d,
                     const float *y, const int64_t *idx, int64_t n,
                     double eta, double lambda, int loss,
                     double *w, double *min_margin)
{
    if (!X || !y || !w || (n > 0 && !idx) || m < 1 || d < 1 || n < 0) return ORACLE_BAD_ARG;
    if (xtype < ORACLE_F32 || xtype > ORACLE_F64) return ORACLE_BAD_ARG;
    if (loss != ORACLE_HINGE && loss != ORACLE_LOGISTIC) return ORACLE_BAD_ARG;
    double closest = INFINITY;
    for (int64_t step = 0; step < n; ++step) {
        int64_t j = idx[step];
        if (j < 0 || j >= m) return ORACLE_BAD_ARG;
        double yj = (double)y[j];
        double yhat = 0.0;
        for (int64_t c = 0; c < d; ++c)
            yhat += w[c] * dense_at(X, xtype, d, j, c);
        double g = loss_slope(loss, yj, yhat);
        double gap = fabs(1.0 - yj * yhat);
        if (gap < closest) closest = gap;
        for (int64_t c = 0; c < d; ++c)
            w[c] = (1.0 - eta * lambda) * w[c] - eta * g * dense_at(X, xtype, d, j, c);
    }
    if (min_margin) *min_margin = closest;
    return ORACLE_OK;
}

/* ------------------------------------------------------------------ */
/* One chain, CSR rows.                                                */
/* mode 0 ("plain"): the literal update, every coordinate shrunk every */
/*                   step -- this is the parity authority;             */
/* mode 1 ("lazy"):  the same recursion written as w = s*v with the    */
/*                   shrink carried by the scalar s; only used as the  */
/*                   timed CPU baseline on very wide data and checked  */
/*                   against mode 0 in the tests.                      */
/* ------------------------------------------------------------------ */
int oracle_sgd_csr(const int64_t *row_ptr, const int32_t *col_idx, const float *vals,
                   int64_t m, int64_t d, const float *y,
                   const int64_t *idx, int64_t n,
                   double eta, double lambda, int loss, int mode,
                   double *w, double *min_margin)
{
    if (!row_ptr || !col_idx || !vals || !y || !w || (n > 0 && !idx)) return ORACLE_BAD_ARG;
    if (m < 1 || d < 1 || n < 0 || (mode != 0 && mode != 1)) return ORACLE_BAD_ARG;
    if (loss != ORACLE_HINGE && loss != ORACLE_LOGISTIC) return ORACLE_BAD_ARG;
    double closest = INFINITY;
    double s = 1.0; /* lazy mode: w = s * (stored vector) */
    for (int64_t step = 0; step < n; ++step) {
        int64_t j = idx[step];
        if (j < 0 || j >= m) return ORACLE_BAD_ARG;
        int64_t lo = row_ptr[j], hi = row_ptr[j + 1];
        double yj = (double)y[j];
        double yhat = 0.0;
        for (int64_t p = lo; p < hi; ++p) {
            if (col_idx[p] < 0 || col_idx[p] >= d) return ORACLE_BAD_ARG;
            yhat += w[col_idx[p]] * (double)vals[p];
        }
        if (mode == 1) yhat *= s;
        double g = loss_slope(loss, yj, yhat);
        double gap = fabs(1.0 - yj * yhat);
        if (gap < closest) closest = gap;
        if (mode == 0) {
            for (int64_t c = 0; c < d; ++c)
                w[c] = (1.0 - eta * lambda) * w[c];
            for (int64_t p = lo; p < hi; ++p)
                w[col_idx[p]] -= eta * g * (double)vals[p];
        } else {
            s *= (1.0 - eta * lambda);
            if (s < 1e-200) { /* fold the scale back before it underflows */
                for (int64_t c = 0; c < d; ++c) w[c] *= s;
                s = 1.0;
            }
            for (int64_t p = lo; p < hi; ++p)
                w[col_idx[p]] -= (eta * g / s) * (double)vals[p];
        }
    }
    if (mode == 1)
        for (int64_t c = 0; c < d; ++c) w[c] *= s;
    if (min_margin) *min_margin = closest;
    return ORACLE_OK;
}

/* ------------------------------------------------------------------ */
/* Weights.  n_steps[i] is the number of steps chain i ran, so the     */
/* fastest chain consumed t = max_i n_steps[i] samples and chain i is  */
/* T_i = t - n_steps[i] behind it (Algorithm 1; Table I).              */
/* weight_i = rate^{T_i} / sum_j rate^{T_j}  (Eq. 6 with rate =        */
/* 1 - eta*lambda; Eq. 8 with rate = r).                               */
/* ------------------------------------------------------------------ */
int oracle_weights_rate(int64_t k, const int64_t *n_steps, double rate, double *a)
{
    if (k < 1 || !n_steps || !a || !(rate > 0.0) || rate > 1.0) return ORACLE_BAD_ARG;
    int64_t t = 0;
    for (int64_t i = 0; i < k; ++i) {
        if (n_steps[i] < 0) return ORACLE_BAD_ARG;
        if (n_steps[i] > t) t = n_steps[i];
    }
    double total = 0.0;
    for (int64_t j = 0; j < k; ++j)
        total += pow(rate, (double)(t - n_steps[j]));
    for (int64_t i = 0; i < k; ++i)
        a[i] = pow(rate, (double)(t - n_steps[i])) / total;
    return ORACLE_OK;
}

int oracle_weights(int64_t k, const int64_t *n_steps, double eta, double lambda, double *a)
{
    if (!(eta > 0.0) || lambda < 0.0 || !(eta * lambda < 1.0)) return ORACLE_BAD_ARG;
    return oracle_weights_rate(k, n_steps, 1.0 - eta * lambda, a);
}

/* Left side minus right side of  2 sum_i rate^{T_i} > sqrt(k) + k  (Eq. 7 / Eq. 9):
 * positive means the bound of the weighted output beats the fastest chain's. */
int oracle_benefit_margin(int64_t k, const int64_t *n_steps, double rate, double *margin)
{
    if (k < 1 || !n_steps || !margin || !(rate > 0.0) || rate > 1.0) return ORACLE_BAD_ARG;
    int64_t t = 0;
    for (int64_t i = 0; i < k; ++i) {
        if (n_steps[i] < 0) return ORACLE_BAD_ARG;
        if (n_steps[i] > t) t = n_steps[i];
    }
    double total = 0.0;
    for (int64_t i = 0; i < k; ++i)
        total += pow(rate, (double)(t - n_steps[i]));
    *margin = 2.0 * total - (sqrt((double)k) + (double)k);
    return ORACLE_OK;
}

/* Periodic averaging (Section III, Deduction 2): with chain j taking D_j steps between two
 * averages and the fastest taking span = max_j D_j, so that T_j = span - D_j, the text below the
 * deduction asks for  k / (sum_j rate^{T_j}) * rate^{span} < 1.  *value receives the left side. */
int oracle_span_condition(int64_t k, const int64_t *steps_per_span, double rate, double *value)
{
    if (k < 1 || !steps_per_span || !value || !(rate > 0.0) || rate > 1.0) return ORACLE_BAD_ARG;
    int64_t span = 0;
    for (int64_t j = 0; j < k; ++j) {
        if (steps_per_span[j] < 0) return ORACLE_BAD_ARG;
        if (steps_per_span[j] > span) span = steps_per_span[j];
    }
    double total = 0.0;
    for (int64_t j = 0; j < k; ++j)
        total += pow(rate, (double)(span - steps_per_span[j]));
    *value = (double)k / total * pow(rate, (double)span);
    return ORACLE_OK;
}

/* v = sum_i a_i * W[i,:]  (last line of Algorithm 1), i ascending. */
int oracle_combine(const double *W, const double *a, int64_t k, int64_t d, double *v)
{
    if (!W || !a || !v || k < 1 || d < 1) return ORACLE_BAD_ARG;
    for (int64_t c = 0; c < d; ++c) {
        double acc = 0.0;
        for (int64_t i = 0; i < k; ++i)
            acc += a[i] * W[i * d + c];
        v[c] = acc;
    }
    return ORACLE_OK;
}

/* ------------------------------------------------------------------ */
/* Regularised objective of a model on a data set (Eq. 3 with Eq. 4):  */
/*   c(w) = lambda/2 |w|^2 + (1/m) sum_j L(x^j, y^j, w.x^j)            */
/* and the fraction of rows with y * (w.x) <= 0 (prediction error).    */
/* Dense or CSR (pass X == NULL for CSR).                              */
/* ------------------------------------------------------------------ */
int oracle_objective(const void *X, int xtype,
                     const int64_t *row_ptr, const int32_t *col_idx, const float *vals,
                     int64_t m, int64_t d, const float *y, const double *w,
                     double lambda, int loss, double *objective, double *error_rate)
{
    if (!y || !w || m < 1 || d < 1) return ORACLE_BAD_ARG;
    if (!X && (!row_ptr || !col_idx || !vals)) return ORACLE_BAD_ARG;
    double sq = 0.0;
    for (int64_t c = 0; c < d; ++c) sq += w[c] * w[c];
    double total = 0.0;
    int64_t wrong = 0;
    for (int64_t j = 0; j < m; ++j) {
        double yhat = 0.0;
        if (X) {
            for (int64_t c = 0; c < d; ++c) yhat += w[c] * dense_at(X, xtype, d, j, c);
        } else {
            for (int64_t p = row_ptr[j]; p < row_ptr[j + 1]; ++p)
                yhat += w[col_idx[p]] * (double)vals[p];
        }
        double z = (double)y[j] * yhat;
        if (loss == ORACLE_HINGE) total += (z < 1.0) ? 1.0 - z : 0.0;
        else total += (z > 0.0) ? log1p(exp(-z)) : -z + log1p(exp(z));
        if (z <= 0.0) ++wrong;
    }
    if (objective) *objective = 0.5 * lambda * sq + total / (double)m;
    if (error_rate) *error_rate = (double)wrong / (double)m;
    return ORACLE_OK;
}

/* ------------------------------------------------------------------ */
/* WP-SGD with delay SGD (Section IV, Algorithms 3 and 4, Lemma 4).    */
/*                                                                    */
/* One server (chain) keeps the accepted iterates w_0, w_1, ..., w_J.  */
/* For every sample x (label y) it receives, the gradient has been     */
/* evaluated tau iterates ago (proof of Lemma 4):                      */
/*     cand = w_J - eta*lambda*w_{J-tau} - eta*u(w_{J-tau}.x)*x,       */
/* u = dL/dyhat; an iterate before the start is the start vector.      */
/* The candidate becomes w_{J+1} only if the Check function accepts;   */
/* otherwise it is abandoned and the next sample is tried.             */
/*                                                                    */
/* Check, for a triple (a, b, c) of consecutive iterates and the       */
/* sample x, with beta^2 = x.x and the projections L_w = x.w:          */
/*     rate  = (eta*lambda + c_star*eta*beta^2)^(1/tau)                */
/*     L_min = (L_b - rate*L_a) / (1 - rate)                           */
/*     accept iff L_c lies between L_min and L_b (ends included) and   */
/*     the part of b perpendicular to x is not longer than that of a.  */
/* The algorithm calls it on the iterates the delayed gradient spans   */
/* (before the update) and on (w_{J-1}, w_J, cand) (after it).         */
/* Readings taken where the listing is garbled or silent:              */
/* c_star = 1 (both losses have |dL/dyhat| <= 1); the                  */
/* tau-th root is taken with max(tau, 1); rate >= 1 rejects; the       */
/* perpendicular test follows the proof (the older iterate's           */
/* perpendicular part must be at least the newer's; the listing prints */
/* the opposite inequality), on squared lengths |w|^2 - L_w^2/beta^2;  */
/* a triple is tested only if all three iterates exist (no test        */
/* reaches before w_0), so the first update is always accepted;        */
/* the first call tests the triples inside w_{J-tau} .. w_J.           */
/* ------------------------------------------------------------------ */

/* One triple of Algorithm 4.  pa, pb: squared lengths of the parts of a and b perpendicular to
 * the sample.  *gap (if not NULL) receives how far the closest comparison was from a tie,
 * relative to the numbers compared. */
int oracle_check_triple(double La, double Lb, double Lc, double pa, double pb, double rate, double *gap)
{
    if (!(rate < 1.0)) {
        if (gap) *gap = INFINITY;
        return 0;
    }
    const double Lmin = (Lb - rate * La) / (1.0 - rate);
    const double lo = Lmin < Lb ? Lmin : Lb, hi = Lmin < Lb ? Lb : Lmin;
    const int inside = (lo <= Lc) && (Lc <= hi);
    const int shrinks = !(pb > pa);
    if (gap) {
        double scale = fabs(lo) > fabs(hi) ? fabs(lo) : fabs(hi);
        if (fabs(Lc) > scale) scale = fabs(Lc);
        if (scale < 1e-300) scale = 1e-300;
        double g1 = fabs(Lc - lo) / scale, g2 = fabs(Lc - hi) / scale;
        double ps = pa > pb ? pa : pb;
        if (ps < 1e-300) ps = 1e-300;
        double g3 = fabs(pa - pb) / ps;
        double g = g1 < g2 ? g1 : g2;
        *gap = g < g3 ? g : g3;
    }
    return inside && shrinks;
}

/* One server of Algorithm 3 over the explicit visit order idx[0..n).  w: start vector in, last
 * accepted iterate out.  check = 0 switches the Check function off (every candidate is accepted:
 * plain delay SGD).  *accepted receives J; *min_gap the closest any Check comparison came to a tie. */
int oracle_delay_sgd_dense(const void *X, int xtype, int64_t m, int64_t d, const float *y,
                           const int64_t *idx, int64_t n, double eta, double lambda, int loss,
                           int tau, int check, double *w, int64_t *accepted, double *min_gap)
{
    if (!X || !y || !w || (n > 0 && !idx) || m < 1 || d < 1 || n < 0 || tau < 0 || tau > 1024) return ORACLE_BAD_ARG;
    if (!(eta > 0.0) || lambda < 0.0 || !(eta * lambda < 1.0)) return ORACLE_BAD_ARG;
    const int reach = tau > 1 ? tau : 1;             /* the second call needs w_{J-1} even at tau = 0 */
    const int slots = reach + 2;                     /* w_{J-reach} .. w_J and the candidate */
    double *hist = (double *)malloc(sizeof(double) * (size_t)slots * (size_t)d);
    double *norm2 = (double *)malloc(sizeof(double) * (size_t)slots);
    double *x = (double *)malloc(sizeof(double) * (size_t)d);
    double *proj = (double *)malloc(sizeof(double) * (size_t)slots);
    if (!hist || !norm2 || !x || !proj) { free(hist); free(norm2); free(x); free(proj); return ORACLE_NO_MEM; }
#define ITER(t) (hist + (size_t)((t) % slots) * (size_t)d)
    int64_t J = 0;
    double n0 = 0.0;
    for (int64_t c = 0; c < d; ++c) { ITER(0)[c] = w[c]; n0 += w[c] * w[c]; }
    norm2[0] = n0;
    double closest = INFINITY;
    for (int64_t s = 0; s < n; ++s) {
        const int64_t j = idx[s];
        if (j < 0 || j >= m) { free(hist); free(norm2); free(x); free(proj); return ORACLE_BAD_ARG; }
        double beta2 = 0.0;
        for (int64_t c = 0; c < d; ++c) { x[c] = dense_at(X, xtype, d, j, c); beta2 += x[c] * x[c]; }
        const int64_t at = J - tau > 0 ? J - tau : 0;            /* where the gradient was evaluated */
        const double *wd = ITER(at), *wj = ITER(J);
        double yhat = 0.0;
        for (int64_t c = 0; c < d; ++c) yhat += wd[c] * x[c];
        const double g = loss_slope(loss, (double)y[j], yhat);
        double *cand = ITER(J + 1);
        double Lc = 0.0, nc = 0.0;
        for (int64_t c = 0; c < d; ++c) {
            cand[c] = wj[c] - eta * lambda * wd[c] - eta * g * x[c];
            Lc += cand[c] * x[c];
            nc += cand[c] * cand[c];
        }
        int flag = 1;
        if (check) {
            const double rate = pow(eta * lambda + eta * beta2, 1.0 / (double)(tau > 1 ? tau : 1));
            /* projections of the iterates the delayed gradient spans, w_{J-tau} .. w_J */
            const int64_t first = J - reach > 0 ? J - reach : 0;
            for (int64_t t = first; t <= J; ++t) {
                double L = 0.0;
                const double *wt = ITER(t);
                for (int64_t c = 0; c < d; ++c) L += wt[c] * x[c];
                proj[t % slots] = L;
            }
#define PERP2(t, L) (beta2 > 0.0 ? norm2[(t) % slots] - (L) * (L) / beta2 : norm2[(t) % slots])
            for (int64_t t = first + 2; t <= J && flag; ++t) {
                double gap;
                const double La = proj[(t - 2) % slots], Lb = proj[(t - 1) % slots], Lt = proj[t % slots];
                flag = oracle_check_triple(La, Lb, Lt, PERP2(t - 2, La), PERP2(t - 1, Lb), rate, &gap);
                if (gap < closest) closest = gap;
            }
            if (flag && J >= 1) {
                double gap;
                const double La = proj[(J - 1) % slots], Lb = proj[J % slots];
                flag = oracle_check_triple(La, Lb, Lc, PERP2(J - 1, La), PERP2(J, Lb), rate, &gap);
                if (gap < closest) closest = gap;
            }
#undef PERP2
        }
        if (flag) {
            ++J;
            norm2[J % slots] = nc;
        }
    }
    for (int64_t c = 0; c < d; ++c) w[c] = ITER(J)[c];
#undef ITER
    if (accepted) *accepted = J;
    if (min_gap) *min_gap = closest;
    free(hist); free(norm2); free(x); free(proj);
    return ORACLE_OK;
}

/* ------------------------------------------------------------------ */
/* All chains of Algorithm 1 ("for all i in 1..k parallel"): chain     */
/* chain_ids[q] starts from w_0 = w0_fill * ones, runs n_steps[q]      */
/* steps over the rows its Philox stream names, and leaves w in        */
/* W[q,:].  Chains are independent, so they are handed to threads one  */
/* at a time; within a chain nothing is parallel.                      */
/* ------------------------------------------------------------------ */
typedef struct {
    const void *X; int xtype;
    const int64_t *row_ptr; const int32_t *col_idx; const float *vals;
    int64_t m, d; const float *y;
    int64_t nq; const int64_t *chain_ids; const int64_t *n_steps;
    double eta, lambda; int loss; int csr_mode; uint64_t seed; double w0_fill;
    double *W; double *min_margin;
    int64_t next; int status; pthread_mutex_t lock;
} chains_job;

static void *chains_worker(void *arg)
{
    chains_job *job = (chains_job *)arg;
    for (;;) {
        pthread_mutex_lock(&job->lock);
        int64_t q = job->next++;
        pthread_mutex_unlock(&job->lock);
        if (q >= job->nq) break;
        int64_t n = job->n_steps[q];
        int64_t *idx = (int64_t *)malloc(sizeof(int64_t) * (size_t)(n > 0 ? n : 1));
        int rc = idx ? ORACLE_OK : ORACLE_NO_MEM;
        if (rc == ORACLE_OK)
            rc = oracle_sample_indices(job->seed, job->chain_ids[q], 0, n, job->m, idx);
        double *w = job->W + q * job->d;
        for (int64_t c = 0; c < job->d; ++c) w[c] = job->w0_fill;
        double *mm = job->min_margin ? job->min_margin + q : NULL;
        if (rc == ORACLE_OK) {
            if (job->X)
                rc = oracle_sgd_dense(job->X, job->xtype, job->m, job->d, job->y, idx, n,
                                      job->eta, job->lambda, job->loss, w, mm);
            else
                rc = oracle_sgd_csr(job->row_ptr, job->col_idx, job->vals, job->m, job->d,
                                    job->y, idx, n, job->eta, job->lambda, job->loss,
                                    job->csr_mode, w, mm);
        }
        free(idx);
        if (rc != ORACLE_OK) {
            pthread_mutex_lock(&job->lock);
            job->status = rc;
            pthread_mutex_unlock(&job->lock);
        }
    }
    return NULL;
}

int oracle_run_chains(const void *X, int xtype,
                      const int64_t *row_ptr, const int32_t *col_idx, const float *vals,
                      int64_t m, int64_t d, const float *y,
                      int64_t nq, const int64_t *chain_ids, const int64_t *n_steps,
                      double eta, double lambda, int loss, int csr_mode, uint64_t seed,
                      double w0_fill, int threads, double *W, double *min_margin)
{
    if (!y || !chain_ids || !n_steps || !W || nq < 1 || m < 1 || d < 1) return ORACLE_BAD_ARG;
    if (!X && (!row_ptr || !col_idx || !vals)) return ORACLE_BAD_ARG;
    if (!(eta > 0.0) || lambda < 0.0 || !(eta * lambda < 1.0)) return ORACLE_BAD_ARG;
    for (int64_t q = 0; q < nq; ++q)
        if (n_steps[q] < 0) return ORACLE_BAD_ARG;
    if (threads < 1) threads = 1;
    if (threads > 256) threads = 256;
    if ((int64_t)threads > nq) threads = (int)nq;
    chains_job job;
    memset(&job, 0, sizeof job);
    job.X = X; job.xtype = xtype; job.row_ptr = row_ptr; job.col_idx = col_idx; job.vals = vals;
    job.m = m; job.d = d; job.y = y; job.nq = nq; job.chain_ids = chain_ids; job.n_steps = n_steps;
    job.eta = eta; job.lambda = lambda; job.loss = loss; job.csr_mode = csr_mode; job.seed = seed;
    job.w0_fill = w0_fill; job.W = W; job.min_margin = min_margin; job.next = 0; job.status = ORACLE_OK;
    pthread_mutex_init(&job.lock, NULL);
    pthread_t tid[256];
    int started = 0;
    for (int t = 0; t < threads - 1; ++t)
        if (pthread_create(&tid[started], NULL, chains_worker, &job) == 0) ++started;
    chains_worker(&job);
    for (int t = 0; t < started; ++t) pthread_join(tid[t], NULL);
    pthread_mutex_destroy(&job.lock);
    return job.status;
}
