/*
 * ddl_oracle.c -- TEST INFRASTRUCTURE ONLY.
 *
 * Plain, slow, fp64 CPU statement of what the Decoupled DiLoCo synchronizer
 * computes for one fragment: Weight -> Merge -> OuterOpt (Algorithm 2, steps
 * "Weight", "mergeFn" and "OuterOpt").  It exists so that the HIP path can be
 * checked against something that a reader can compare with the paper by eye.
 * It shares no code, header, table or helper with the HIP library, and nothing
 * in the product path may call it: only the tests, the smoke check and the
 * CPU-baseline leg of the benchmark do.
 *
 * All pointers are HOST pointers.  Inputs keep their storage type (fp32 or
 * bf16); every input is widened exactly to double before any arithmetic and
 * every result is returned in double.
 *
 * Nothing here is blocked, fused, vectorised or reordered: one loop over the
 * elements, one inner loop over the learners, in the order the paper writes the
 * sums.
 *
 * PARITY UNPINNED (against the paper) for the 4-bit outer-gradient functions
 * ddl_oracle_q4_encode / ddl_oracle_q4_merge_fragment /
 * ddl_oracle_q4_rda_merge_fragment: the paper states only the width; the
 * block-wise format is this build's choice.  See their comment.
 */
#include <math.h>
#include <pthread.h>
#include <stddef.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

enum { ORACLE_OK = 0, ORACLE_BAD_ARG = 1, ORACLE_EMPTY_QUORUM = 2 };
enum { ORACLE_F32 = 0, ORACLE_BF16 = 1 };
#define ORACLE_MAX_LEARNERS 64

/* bf16 is the upper half of an IEEE fp32 word: widening is exact. */
static double widen_bf16(uint16_t h)
{
    uint32_t bits = (uint32_t)h << 16;
    float f;
    memcpy(&f, &bits, sizeof f);
    return (double)f;
}

static double learner_value(const void* base, int dtype, size_t i)
{
    if (dtype == ORACLE_BF16)
        return widen_bf16(((const uint16_t*)base)[i]);
    return (double)((const float*)base)[i];
}

/*
 * Weight, tokens-only form, normalised over the quorum.
 *
 * Raw weight of learner m is q_m * n_m: its token counter c^tokens since the
 * last sync of this fragment (Algorithm 1, counter update) if it is a member of
 * the reporting set M_t (Section 3.2), zero if it is absent (Section 4, "Syncer
 * worker": an absent learner takes part in the same Merge with weight 0).  The
 * weighted Merge divides by the sum of the weights over M_t (Appendix D.2,
 * weighted direct averaging), so the normalised weight is
 *     w_m = q_m n_m / sum_k q_k n_k.
 * A quorum whose weights sum to zero has no defined merge: ORACLE_EMPTY_QUORUM.
 */
int ddl_oracle_weights(const uint64_t* token_counts, const uint8_t* quorum_mask,
                       int M, double* w_out)
{
    if (!token_counts || !quorum_mask || !w_out || M < 1 || M > ORACLE_MAX_LEARNERS)
        return ORACLE_BAD_ARG;
    double S = 0.0;
    for (int m = 0; m < M; ++m) {
        if (quorum_mask[m] > 1)
            return ORACLE_BAD_ARG;
        if (quorum_mask[m])
            S += (double)token_counts[m];
    }
    if (S == 0.0)
        return ORACLE_EMPTY_QUORUM;
    for (int m = 0; m < M; ++m)
        w_out[m] = quorum_mask[m] ? (double)token_counts[m] / S : 0.0;
    return ORACLE_OK;
}

/*
 * The paper's own Weight function (Section 3.2): quantity x quality,
 *     Weight(c_tokens, c_steps) = c_tokens * (c_tokens / c_steps),
 * again zero for absent learners and normalised over the quorum.  A member of
 * the quorum with c_steps = 0 has taken no step since the last sync and so has
 * c_tokens = 0 too (both counters move together in Algorithm 1); its raw
 * weight is taken as 0.  c_steps = 0 with c_tokens > 0 cannot happen in the
 * protocol and is rejected.
 */
int ddl_oracle_weights_quality(const uint64_t* token_counts, const uint64_t* step_counts,
                               const uint8_t* quorum_mask, int M, double* w_out)
{
    if (!token_counts || !step_counts || !quorum_mask || !w_out || M < 1 ||
        M > ORACLE_MAX_LEARNERS)
        return ORACLE_BAD_ARG;
    double raw[ORACLE_MAX_LEARNERS];
    double S = 0.0;
    for (int m = 0; m < M; ++m) {
        raw[m] = 0.0;
        if (quorum_mask[m] > 1)
            return ORACLE_BAD_ARG;
        if (!quorum_mask[m])
            continue;
        if (step_counts[m] == 0) {
            if (token_counts[m] != 0)
                return ORACLE_BAD_ARG;
            continue;
        }
        double c_tok = (double)token_counts[m];
        raw[m] = c_tok * (c_tok / (double)step_counts[m]);
        S += raw[m];
    }
    if (S == 0.0)
        return ORACLE_EMPTY_QUORUM;
    for (int m = 0; m < M; ++m)
        w_out[m] = raw[m] / S;
    return ORACLE_OK;
}

/*
 * Merge (weighted direct averaging, Appendix D.2) followed by OuterOpt (SGD
 * with Nesterov momentum, Sections 2 and 3.2) on elements [lo, hi) of one flat
 * fragment, given already-normalised weights.
 *
 *   Delta_i = sum_{m in quorum} w_m * (Theta_i - theta_{m,i})
 *
 * The outer gradient is "old global minus learner" (Eq. 1, Eq. 2, Appendix
 * D.2).  Learners with w_m = 0 are skipped, not multiplied by zero, so whatever
 * an absent learner's buffer holds (garbage, NaN, nothing at all) cannot reach
 * the result.
 *
 * The paper names the outer optimiser but does not print its update.  The
 * reading taken is the momentum-buffer form with no dampening and no weight
 * decay,
 *   v'     = mu * v + Delta
 *   Theta' = Theta - lr * (Delta + mu * v')
 * which at mu = 0 is plain SGD, and at mu = 0, lr = 1 is weight averaging, as
 * Section 2 says it must be.
 */
static void merge_range(double* theta_out, double* v_out, const float* theta, const float* v,
                        const void* const* learner_params, int learner_dtype, const double* w,
                        int M, size_t lo, size_t hi, double lr, double mu)
{
    for (size_t i = lo; i < hi; ++i) {
        double Theta = (double)theta[i];
        double Delta = 0.0;
        for (int m = 0; m < M; ++m) {
            if (w[m] == 0.0)
                continue;
            Delta += w[m] * (Theta - learner_value(learner_params[m], learner_dtype, i));
        }
        double v_new = mu * (double)v[i] + Delta;
        double Theta_new = Theta - lr * (Delta + mu * v_new);
        theta_out[i] = Theta_new;
        v_out[i] = v_new;
    }
}

static int check_merge_args(const void* theta_out, const void* v_out, const void* theta,
                            const void* v, const void* const* learner_params, int learner_dtype,
                            const double* w, int M, size_t n, float lr, float mu)
{
    if (M < 1 || M > ORACLE_MAX_LEARNERS || !learner_params)
        return ORACLE_BAD_ARG;
    if (learner_dtype != ORACLE_F32 && learner_dtype != ORACLE_BF16)
        return ORACLE_BAD_ARG;
    if (!(lr >= 0.0f) || !(mu >= 0.0f) || isinf(lr) || isinf(mu))
        return ORACLE_BAD_ARG;
    if (n > 0 && (!theta_out || !v_out || !theta || !v))
        return ORACLE_BAD_ARG;
    for (int m = 0; m < M; ++m)
        if (w[m] != 0.0 && n > 0 && !learner_params[m])
            return ORACLE_BAD_ARG;
    return ORACLE_OK;
}

/*
 * One fragment sync on one flat array: Weight, Merge, OuterOpt.
 * theta_out / v_out receive the new global fragment and momentum in double;
 * theta / v are not modified.  On any error nothing is written.
 */
int ddl_oracle_merge_fragment(double* theta_out, double* v_out, const float* theta,
                              const float* v, const void* const* learner_params,
                              int learner_dtype, const uint64_t* token_counts,
                              const uint8_t* quorum_mask, int M, size_t n, float lr, float mu)
{
    double w[ORACLE_MAX_LEARNERS];
    int rc = ddl_oracle_weights(token_counts, quorum_mask, M, w);
    if (rc != ORACLE_OK)
        return rc;
    rc = check_merge_args(theta_out, v_out, theta, v, learner_params, learner_dtype, w, M, n, lr,
                          mu);
    if (rc != ORACLE_OK)
        return rc;
    merge_range(theta_out, v_out, theta, v, learner_params, learner_dtype, w, M, 0, n,
                (double)lr, (double)mu);
    return ORACLE_OK;
}

/*
 * Same, but with the normalised weights handed in (any non-negative weights
 * that the caller has already divided by their sum): lets a caller use the
 * quality-weighted form or any other Weight function.
 */
int ddl_oracle_merge_fragment_weighted(double* theta_out, double* v_out, const float* theta,
                                       const float* v, const void* const* learner_params,
                                       int learner_dtype, const double* w, int M, size_t n,
                                       float lr, float mu)
{
    if (!w)
        return ORACLE_BAD_ARG;
    int rc = check_merge_args(theta_out, v_out, theta, v, learner_params, learner_dtype, w, M, n,
                              lr, mu);
    if (rc != ORACLE_OK)
        return rc;
    merge_range(theta_out, v_out, theta, v, learner_params, learner_dtype, w, M, 0, n,
                (double)lr, (double)mu);
    return ORACLE_OK;
}

/*
 * Radial-directional averaging (Appendix D.2, "Radial-directional averaging"), weighted
 * form, followed by the same OuterOpt.  For a set of outer gradients d_m = Theta - theta_m
 * (m in the quorum, normalised weights w_m):
 *
 *     RDA = ( sum_m w_m ||d_m|| ) * phi( sum_m w_m phi(d_m) ),      phi(x) = x / ||x||_2
 *
 * i.e. norms and directions are averaged separately and the mean direction is projected
 * back to unit length.  The printed weighted formula has sum_m w_m d_m (a vector) where the
 * unweighted one has the mean of the norms; it is read as the weighted mean of the norms,
 * "completely analogously" as the text says.
 *
 * The paper does not say over which elements a norm is taken (it only says the magnitude
 * tensors are tiny next to the direction tensors).  Here a tensor is cut into consecutive
 * groups of `group_len` elements (the last one may be shorter) and RDA is applied to each
 * group on its own: group_len = row length gives one magnitude per row, group_len >= n one
 * per tensor.  phi is undefined at 0: a learner whose outer gradient is zero on a group adds
 * nothing to that group's mean direction (its zero norm still enters the mean norm), and a
 * group whose mean direction is zero gets Delta = 0.
 */
int ddl_oracle_rda_merge_fragment(double* theta_out, double* v_out, const float* theta,
                                  const float* v, const void* const* learner_params,
                                  int learner_dtype, const uint64_t* token_counts,
                                  const uint8_t* quorum_mask, int M, size_t n, size_t group_len,
                                  float lr, float mu)
{
    double w[ORACLE_MAX_LEARNERS];
    int rc = ddl_oracle_weights(token_counts, quorum_mask, M, w);
    if (rc != ORACLE_OK)
        return rc;
    rc = check_merge_args(theta_out, v_out, theta, v, learner_params, learner_dtype, w, M, n, lr,
                          mu);
    if (rc != ORACLE_OK)
        return rc;
    if (group_len == 0)
        return ORACLE_BAD_ARG;
    for (size_t lo = 0; lo < n; lo += group_len) {
        size_t hi = n - lo < group_len ? n : lo + group_len;
        /* norms of the outer gradients on this group, and their weighted mean */
        double norm[ORACLE_MAX_LEARNERS];
        double mean_norm = 0.0;
        for (int m = 0; m < M; ++m) {
            norm[m] = 0.0;
            if (w[m] == 0.0)
                continue;
            double ss = 0.0;
            for (size_t i = lo; i < hi; ++i) {
                double d = (double)theta[i] - learner_value(learner_params[m], learner_dtype, i);
                ss += d * d;
            }
            norm[m] = sqrt(ss);
            mean_norm += w[m] * norm[m];
        }
        /* weighted mean of the unit directions, kept in v_out as scratch, and its norm */
        double dir_ss = 0.0;
        for (size_t i = lo; i < hi; ++i) {
            double u = 0.0;
            for (int m = 0; m < M; ++m) {
                if (w[m] == 0.0 || norm[m] == 0.0)
                    continue;
                double d = (double)theta[i] - learner_value(learner_params[m], learner_dtype, i);
                u += w[m] * (d / norm[m]);
            }
            v_out[i] = u;
            dir_ss += u * u;
        }
        double dir_norm = sqrt(dir_ss);
        for (size_t i = lo; i < hi; ++i) {
            double Delta = dir_norm > 0.0 ? mean_norm * (v_out[i] / dir_norm) : 0.0;
            double Theta = (double)theta[i];
            double v_new = (double)mu * (double)v[i] + Delta;
            theta_out[i] = Theta - (double)lr * (Delta + (double)mu * v_new);
            v_out[i] = v_new;
        }
    }
    return ORACLE_OK;
}

/*
 * fp32 -> bf16 for the broadcast copy of the new global fragment (Algorithm 2, the Send back
 * to the learners; bf16 being the paper's wire format, Appendix D.3): round to nearest, ties
 * to even, written from the definition -- the two bf16 neighbours of x are found by clearing
 * the low 16 bits and by stepping one bf16 unit away from zero, the nearer one in exact
 * (double) arithmetic wins, a tie goes to the one whose last kept bit is 0.  NaN stays NaN
 * (sign and top payload bits kept, quiet bit set); overflow rounds to infinity.
 */
static uint16_t round_bf16(float x)
{
    uint32_t bits;
    memcpy(&bits, &x, sizeof bits);
    if ((bits & 0x7fffffffu) > 0x7f800000u)
        return (uint16_t)((bits >> 16) | 0x40u);
    uint32_t lo_bits = bits & 0xffff0000u;      /* neighbour towards zero */
    uint32_t hi_bits = lo_bits + 0x10000u;      /* neighbour away from zero (may be inf) */
    float lo, hi;
    memcpy(&lo, &lo_bits, sizeof lo);
    memcpy(&hi, &hi_bits, sizeof hi);
    if ((hi_bits & 0x7f800000u) == 0x7f800000u) {
        /* away-from-zero neighbour is infinity: its place on the real line, for the distance
         * test, is one bf16 step beyond the largest finite value */
        double step = ldexp(1.0, 127 - 7);
        double dlo = fabs((double)x - (double)lo);
        double dhi = step - dlo;
        if (dlo < dhi) return (uint16_t)(lo_bits >> 16);
        if (dhi < dlo) return (uint16_t)(hi_bits >> 16);
        return (uint16_t)((((lo_bits >> 16) & 1u) == 0 ? lo_bits : hi_bits) >> 16);
    }
    double dlo = fabs((double)x - (double)lo);
    double dhi = fabs((double)hi - (double)x);
    if (dlo < dhi) return (uint16_t)(lo_bits >> 16);
    if (dhi < dlo) return (uint16_t)(hi_bits >> 16);
    return (uint16_t)((((lo_bits >> 16) & 1u) == 0 ? lo_bits : hi_bits) >> 16);
}

void ddl_oracle_round_bf16(const float* x, uint16_t* out, size_t n)
{
    for (size_t i = 0; i < n; ++i)
        out[i] = round_bf16(x[i]);
}

/*
 * 4-bit outer gradients (Appendix D.3, "Outer gradients compression": outer gradients are
 * compressed to int4 before the merge).  PARITY UNPINNED against the paper: it fixes only the
 * width, 4 bits per value; block size, scale and rounding below are this build's choice of a
 * plain symmetric block-wise integer quantiser.  Given that format, the arithmetic is the
 * definition written out and is pinned by the tests (hand-packed bytes, round-trip error
 * bound, agreement with the direct-averaging oracle on exactly representable values).
 *
 * Format, per learner: the flat fragment is cut into blocks of `block_len` consecutive
 * elements (the last may be shorter); block b has one fp32 scale s_b; element i has a signed
 * 4-bit code q_i in two's complement, two codes per byte, element 2k in the low nibble of
 * byte k and element 2k+1 in its high nibble.  The value an (s, q) pair stands for is s * q.
 */
static int q4_code(const uint8_t* codes, size_t i)
{
    unsigned nib = (i & 1) ? (codes[i >> 1] >> 4) : (codes[i >> 1] & 0x0fu);
    return nib >= 8 ? (int)nib - 16 : (int)nib;
}

/*
 * Encoder: the outer gradient d_i = Theta_i - theta_{m,i} is formed in fp32; per block
 * a = max |d_i|, s = a / 7, q_i = round-half-even(d_i / s) clamped to [-7, 7]; an all-zero
 * block gets s = 0 and q = 0.  A floating-point value decides an integer here, so every step
 * is taken in fp32, the precision the GPU encoder works in (fp32 subtraction, IEEE division,
 * round to nearest even), not in double.  `codes_out` has (n + 1) / 2 bytes (an unused high
 * nibble is 0), `scales_out` has ceil(n / block_len) entries.
 */
int ddl_oracle_q4_encode(const float* theta, const void* learner, int learner_dtype, size_t n,
                         size_t block_len, uint8_t* codes_out, float* scales_out)
{
    if (block_len == 0 || (learner_dtype != ORACLE_F32 && learner_dtype != ORACLE_BF16))
        return ORACLE_BAD_ARG;
    if (n > 0 && (!theta || !learner || !codes_out || !scales_out))
        return ORACLE_BAD_ARG;
    memset(codes_out, 0, (n + 1) / 2);
    for (size_t b0 = 0, b = 0; b0 < n; b0 += block_len, ++b) {
        size_t b1 = b0 + block_len < n ? b0 + block_len : n;
        float a = 0.0f;
        for (size_t i = b0; i < b1; ++i) {
            float d = theta[i] - (float)learner_value(learner, learner_dtype, i);
            if (fabsf(d) > a)
                a = fabsf(d);
        }
        float s = a / 7.0f;
        scales_out[b] = s;
        if (!(s > 0.0f))
            continue;
        for (size_t i = b0; i < b1; ++i) {
            float d = theta[i] - (float)learner_value(learner, learner_dtype, i);
            float r = nearbyintf(d / s); /* default rounding mode: to nearest, ties to even */
            if (r > 7.0f) r = 7.0f;
            if (r < -7.0f) r = -7.0f;
            unsigned nib = (unsigned)((int)r & 0x0f);
            codes_out[i >> 1] |= (uint8_t)((i & 1) ? nib << 4 : nib);
        }
    }
    return ORACLE_OK;
}

/*
 * Merge of 4-bit outer gradients + OuterOpt: the outer gradient of learner m at element i is
 * s_{m, i / block_len} * q_{m,i}; the rest is weighted direct averaging and the outer step
 * exactly as in merge_range, in double.  Learners of weight zero are skipped.
 */
int ddl_oracle_q4_merge_fragment(double* theta_out, double* v_out, const float* theta,
                                 const float* v, const uint8_t* const* codes,
                                 const float* const* scales, const uint64_t* token_counts,
                                 const uint8_t* quorum_mask, int M, size_t n, size_t block_len,
                                 float lr, float mu)
{
    double w[ORACLE_MAX_LEARNERS];
    int rc = ddl_oracle_weights(token_counts, quorum_mask, M, w);
    if (rc != ORACLE_OK)
        return rc;
    if (block_len == 0 || !codes || !scales)
        return ORACLE_BAD_ARG;
    if (!(lr >= 0.0f) || !(mu >= 0.0f) || isinf(lr) || isinf(mu))
        return ORACLE_BAD_ARG;
    if (n > 0 && (!theta_out || !v_out || !theta || !v))
        return ORACLE_BAD_ARG;
    for (int m = 0; m < M; ++m)
        if (w[m] != 0.0 && n > 0 && (!codes[m] || !scales[m]))
            return ORACLE_BAD_ARG;
    for (size_t i = 0; i < n; ++i) {
        double Delta = 0.0;
        for (int m = 0; m < M; ++m) {
            if (w[m] == 0.0)
                continue;
            double d = (double)scales[m][i / block_len] * (double)q4_code(codes[m], i);
            Delta += w[m] * d;
        }
        double v_new = (double)mu * (double)v[i] + Delta;
        theta_out[i] = (double)theta[i] - (double)lr * (Delta + (double)mu * v_new);
        v_out[i] = v_new;
    }
    return ORACLE_OK;
}

/* The value learner data (cd, sc) stands for at element i: block scale times code. */
static double q4_value(const uint8_t* cd, const float* sc, size_t i, size_t block_len)
{
    return (double)sc[i / block_len] * (double)q4_code(cd, i);
}

/*
 * Radial-directional averaging of 4-bit outer gradients + OuterOpt: what the syncer computes
 * when the outer gradients arrive compressed (Appendix D.3: they are compressed before the
 * mergeFn of Algorithm 2) and the mergeFn is RDA (Appendix D.2, "Radial-directional
 * averaging"; Section 5.1).  The outer gradient of learner m at element i is the value its
 * (scale, code) pair stands for; norms are taken over groups of `group_len` consecutive
 * elements of the tensor (groups and scale blocks need not line up), and
 *
 *     Delta = ( sum_m w_m ||d_m|| ) * phi( sum_m w_m phi(d_m) )
 *
 * with the same readings as ddl_oracle_rda_merge_fragment (weighted mean of the norms; a
 * learner whose gradient is zero on a group adds no direction; a zero mean direction gives
 * Delta = 0).  PARITY UNPINNED against the paper as far as the 4-bit format and the group
 * length go, like the two functions it combines.
 */
int ddl_oracle_q4_rda_merge_fragment(double* theta_out, double* v_out, const float* theta,
                                     const float* v, const uint8_t* const* codes,
                                     const float* const* scales, const uint64_t* token_counts,
                                     const uint8_t* quorum_mask, int M, size_t n,
                                     size_t block_len, size_t group_len, float lr, float mu)
{
    double w[ORACLE_MAX_LEARNERS];
    int rc = ddl_oracle_weights(token_counts, quorum_mask, M, w);
    if (rc != ORACLE_OK)
        return rc;
    if (block_len == 0 || group_len == 0 || !codes || !scales)
        return ORACLE_BAD_ARG;
    if (!(lr >= 0.0f) || !(mu >= 0.0f) || isinf(lr) || isinf(mu))
        return ORACLE_BAD_ARG;
    if (n > 0 && (!theta_out || !v_out || !theta || !v))
        return ORACLE_BAD_ARG;
    for (int m = 0; m < M; ++m)
        if (w[m] != 0.0 && n > 0 && (!codes[m] || !scales[m]))
            return ORACLE_BAD_ARG;
    for (size_t g0 = 0; g0 < n; g0 += group_len) {
        size_t g1 = n - g0 < group_len ? n : g0 + group_len;
        /* radial part: the weighted mean R of the norms over the group */
        double len[ORACLE_MAX_LEARNERS];
        double R = 0.0;
        for (int m = 0; m < M; ++m) {
            len[m] = 0.0;
            if (w[m] == 0.0)
                continue;
            double acc = 0.0;
            for (size_t i = g0; i < g1; ++i) {
                double d = q4_value(codes[m], scales[m], i, block_len);
                acc += d * d;
            }
            len[m] = sqrt(acc);
            R += w[m] * len[m];
        }
        /* directional part: the weighted mean of the unit vectors (in v_out) and its norm */
        double uu = 0.0;
        for (size_t i = g0; i < g1; ++i) {
            double u = 0.0;
            for (int m = 0; m < M; ++m) {
                if (w[m] == 0.0 || len[m] == 0.0)
                    continue;
                u += w[m] * (q4_value(codes[m], scales[m], i, block_len) / len[m]);
            }
            v_out[i] = u;
            uu += u * u;
        }
        double U = sqrt(uu);
        for (size_t i = g0; i < g1; ++i) {
            double Delta = U > 0.0 ? R * (v_out[i] / U) : 0.0;
            double vn = (double)mu * (double)v[i] + Delta;
            theta_out[i] = (double)theta[i] - (double)lr * (Delta + (double)mu * vn);
            v_out[i] = vn;
        }
    }
    return ORACLE_OK;
}

/*
 * The identical scalar loop, with the element range cut into `nthreads`
 * contiguous chunks that run on their own threads.  Elements are independent,
 * so the result is bit-identical to ddl_oracle_merge_fragment.  Used only to
 * time the oracle on all host cores.
 */
struct chunk_job {
    double* theta_out;
    double* v_out;
    const float* theta;
    const float* v;
    const void* const* learner_params;
    int learner_dtype;
    const double* w;
    int M;
    size_t lo, hi;
    double lr, mu;
};

static void* chunk_main(void* arg)
{
    struct chunk_job* j = (struct chunk_job*)arg;
    merge_range(j->theta_out, j->v_out, j->theta, j->v, j->learner_params, j->learner_dtype, j->w,
                j->M, j->lo, j->hi, j->lr, j->mu);
    return NULL;
}

int ddl_oracle_merge_fragment_mt(double* theta_out, double* v_out, const float* theta,
                                 const float* v, const void* const* learner_params,
                                 int learner_dtype, const uint64_t* token_counts,
                                 const uint8_t* quorum_mask, int M, size_t n, float lr, float mu,
                                 int nthreads)
{
    double w[ORACLE_MAX_LEARNERS];
    int rc = ddl_oracle_weights(token_counts, quorum_mask, M, w);
    if (rc != ORACLE_OK)
        return rc;
    rc = check_merge_args(theta_out, v_out, theta, v, learner_params, learner_dtype, w, M, n, lr,
                          mu);
    if (rc != ORACLE_OK)
        return rc;
    if (nthreads < 1 || nthreads > 1024)
        return ORACLE_BAD_ARG;
    pthread_t* tid = (pthread_t*)malloc(sizeof(pthread_t) * (size_t)nthreads);
    struct chunk_job* job = (struct chunk_job*)malloc(sizeof(struct chunk_job) * (size_t)nthreads);
    if (!tid || !job) {
        free(tid);
        free(job);
        return ORACLE_BAD_ARG;
    }
    size_t per = (n + (size_t)nthreads - 1) / (size_t)nthreads;
    int started = 0;
    for (int t = 0; t < nthreads; ++t) {
        size_t lo = per * (size_t)t;
        size_t hi = lo + per < n ? lo + per : n;
        if (lo >= hi)
            break;
        struct chunk_job j = {theta_out, v_out, theta, v, learner_params, learner_dtype, w,
                              M, lo, hi, (double)lr, (double)mu};
        job[t] = j;
        if (pthread_create(&tid[t], NULL, chunk_main, &job[t]) != 0) {
            chunk_main(&job[t]); /* could not start a thread: do the chunk here */
            tid[t] = pthread_self();
            job[t].M = -1;
        }
        started = t + 1;
    }
    for (int t = 0; t < started; ++t)
        if (job[t].M != -1)
            pthread_join(tid[t], NULL);
    free(tid);
    free(job);
    return ORACLE_OK;
}
