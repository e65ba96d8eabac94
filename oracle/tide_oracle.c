/*
 * tide_oracle.c -- plain fp64 CPU oracle for the TIDE router hot path.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, obviously-correct
 * statement of what the path computes.  It is linked by the tests, by the
 * smoke check and by the benchmark's cpu_baseline leg, and by nothing else:
 * the product library never calls it and shares no code with it.
 *
 * What it follows (paper: "TIDE: Token-Informed Depth Execution"):
 *   - Eq. (2), Sec. 3.1 step 3: router  phi(h) = sigma(W_up SiLU(W_down RMSNorm(h)))
 *     with W_down in R^{b x d}, W_up in R^{1 x b}.
 *   - Sec. 3.4 kernel 1: the same chain (RMSNorm, down-projection, SiLU,
 *     up-projection, sigmoid), accumulation wider than the storage type,
 *     router weights kept in fp32.
 *   - Fig. 1 (inference step 3), Sec. 3.3, Alg. 1: strict "score > theta",
 *     checkpoints visited in ascending layer order, checkpoints below k_min
 *     skipped, the earliest firing checkpoint wins, no firing => no early exit.
 *
 * Readings where the paper is silent (each is also listed in the design notes):
 *   - RMSNorm(h)_i = h_i / sqrt(mean_i(h_i^2) + eps) * gamma_i  (eps inside the
 *     root, added to the mean square); the paper's router has gamma == 1.
 *   - optional biases b1 (after the down-projection) and b2 (after the
 *     up-projection); the paper's router has none (b1 == 0, b2 == 0).
 *   - W1 is stored [d, b] row-major, i.e. W1[i*b + j] = W_down[j][i].
 *   - SiLU(x) = x * sigma(x).
 *   - the threshold test is taken in the logit domain: sigma is strictly
 *     increasing, so  sigma(z) > theta  <=>  z > ln(theta / (1 - theta))  for
 *     0 < theta < 1; theta >= 1 never fires (the paper's "1.0 (off)" row of
 *     Table 4), theta <= 0 always fires.
 *   - exit is per token (Abstract, Fig. 1, Table 1), not per batch.
 *   - batch compaction (Sec. 3.4 kernel 2): at a checkpoint layer k the tokens split into those
 *     whose exit layer is <= k and those that continue; both lists keep the token order.
 *   - calibration labels (Sec. 3.1 step 2, Eq. (1)): cosine similarity of a checkpoint's hidden
 *     state with the last layer's, per token; label 1 iff it exceeds tau, strictly.
 *   - exit projection (Fig. 1 "LMHead(Norm(h_k))", Alg. 1 "LMHead(RMSNorm(H[k+1]))", Sec. 3.4
 *     kernels 3 and 4): the row handed to the LM head for token t is the model's final
 *     RMSNorm applied to the hidden state of the checkpoint the token exits at, written at
 *     the token's own position; a token that does not exit takes the last layer's hidden
 *     state (Alg. 1's "no early exit" branch).  The result is stored in the model's own
 *     type, i.e. the fp64 value is rounded ONCE, to nearest even, to the storage type.
 *
 * All arithmetic is double precision, summed left to right in index order.
 * Inputs are the very bytes the GPU path receives: hidden states in their
 * storage type (fp32 / IEEE fp16 / bfloat16 bit patterns, widened exactly),
 * router parameters in fp32 (widened exactly).
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

enum { ORACLE_F32 = 0, ORACLE_F16 = 1, ORACLE_BF16 = 2 };

/* ---- exact widening of the three storage types to double ---- */

static double widen_f32(const void* p, int64_t i) {
    float f;
    memcpy(&f, (const char*)p + 4 * i, 4);
    return (double)f;
}

static double widen_bf16(const void* p, int64_t i) {
    /* bfloat16 = the upper 16 bits of an IEEE binary32 */
    uint16_t h;
    memcpy(&h, (const char*)p + 2 * i, 2);
    uint32_t u = (uint32_t)h << 16;
    float f;
    memcpy(&f, &u, 4);
    return (double)f;
}

static double widen_f16(const void* p, int64_t i) {
    /* IEEE binary16: 1 sign, 5 exponent (bias 15), 10 fraction bits */
    uint16_t h;
    memcpy(&h, (const char*)p + 2 * i, 2);
    int sign = (h >> 15) & 1;
    int ex = (h >> 10) & 0x1f;
    int fr = h & 0x3ff;
    double v;
    if (ex == 0)
        v = ldexp((double)fr, -24);              /* zero and subnormals */
    else if (ex == 31)
        v = fr ? NAN : INFINITY;
    else
        v = ldexp(1.0 + (double)fr / 1024.0, ex - 15);
    return sign ? -v : v;
}

static double widen(const void* p, int dtype, int64_t i) {
    switch (dtype) {
    case ORACLE_F32: return widen_f32(p, i);
    case ORACLE_F16: return widen_f16(p, i);
    default:         return widen_bf16(p, i);
    }
}

/* ---- exact rounding of a double to a storage type (nearest, ties to even) ---- */

/* p significant bits; emin = frexp exponent of the smallest normal (value = m * 2^e, 0.5 <= |m| < 1);
 * emax = frexp exponent of the largest finite.  Below the normal range precision shrinks
 * (gradual underflow).  rint() rounds to nearest even in the default rounding mode.          */
static double round_to_format(double v, int p, int emin, int emax) {
    if (v == 0.0 || isnan(v) || isinf(v)) return v;
    int e;
    double m = frexp(v, &e);
    int bits = p;
    if (e < emin) bits = p - (emin - e);
    if (bits < 0) return copysign(0.0, v);         /* below half the smallest subnormal */
    double r = ldexp(rint(ldexp(m, bits)), e - bits);
    double top = ldexp(1.0 - ldexp(1.0, -p), emax); /* largest finite */
    if (fabs(r) > top) return copysign(INFINITY, v);
    return r;
}

static double round_to_storage(double v, int dtype) {
    switch (dtype) {
    case ORACLE_F32: return round_to_format(v, 24, -125, 128);
    case ORACLE_F16: return round_to_format(v, 11, -13, 16);
    default:         return round_to_format(v, 8, -125, 128);
    }
}

/* bit pattern of a value that is exactly representable in the storage type */
static void store_exact(void* p, int dtype, int64_t i, double r) {
    if (dtype == ORACLE_F32) {
        float f = (float)r;
        memcpy((char*)p + 4 * i, &f, 4);
    } else if (dtype == ORACLE_BF16) {
        float f = (float)r;
        uint32_t u;
        memcpy(&u, &f, 4);
        uint16_t h = (uint16_t)(u >> 16);
        memcpy((char*)p + 2 * i, &h, 2);
    } else {
        uint16_t h;
        uint16_t sign = signbit(r) ? 0x8000 : 0;
        double a = fabs(r);
        if (isnan(r)) h = 0x7e00;
        else if (isinf(r)) h = sign | 0x7c00;
        else if (a == 0.0) h = sign;
        else {
            int e;
            double m = frexp(a, &e);               /* a = m * 2^e */
            if (e < -13) h = sign | (uint16_t)ldexp(a, 24);              /* subnormal: a / 2^-24 */
            else h = sign | (uint16_t)(((e + 14) << 10) | ((int)ldexp(m, 11) & 0x3ff));
        }
        memcpy((char*)p + 2 * i, &h, 2);
    }
}

/* ---- scalar functions of Eq. (2) ---- */

/* logistic function, written in the branch that never overflows */
static double sigmoid(double x) {
    if (x >= 0.0) return 1.0 / (1.0 + exp(-x));
    double e = exp(x);
    return e / (1.0 + e);
}

static double silu(double x) { return x * sigmoid(x); }

/* sigma(z) > theta, decided on z (see header) */
static int fires(double z, double theta) {
    if (theta >= 1.0) return 0;
    if (theta <= 0.0) return 1;
    return z > log(theta / (1.0 - theta));
}

/* ---- one row: Eq. (2) ---- */

/* h: d storage-typed values starting at element index `off` of `hidden`.
 * norm (scratch, d doubles) receives RMSNorm(h); act (scratch, b doubles)
 * receives the pre-activation a_j.  Returns the logit z.                     */
static double router_logit_row(const void* hidden, int dtype, int64_t off, int64_t d, int64_t b,
                               const float* gamma, double eps, const float* W1, const float* b1,
                               const float* w2, double b2, double* norm, double* act) {
    double ss = 0.0;
    for (int64_t i = 0; i < d; ++i) {
        double x = widen(hidden, dtype, off + i);
        ss += x * x;
    }
    double r = 1.0 / sqrt(ss / (double)d + eps);
    for (int64_t i = 0; i < d; ++i) {
        double g = gamma ? (double)gamma[i] : 1.0;
        norm[i] = widen(hidden, dtype, off + i) * r * g;
    }
    /* down-projection a = W_down n + b1, with W1[i][j] = W_down[j][i] */
    for (int64_t j = 0; j < b; ++j) act[j] = b1 ? (double)b1[j] : 0.0;
    for (int64_t i = 0; i < d; ++i)
        for (int64_t j = 0; j < b; ++j) act[j] += norm[i] * (double)W1[i * b + j];
    /* up-projection of SiLU(a) */
    double z = b2;
    for (int64_t j = 0; j < b; ++j) z += (double)w2[j] * silu(act[j]);
    return z;
}

/* ---- exported: RMSNorm alone (for the pins on its invariants) ---- */

int tide_oracle_rmsnorm(const void* hidden, int dtype, int64_t T, int64_t d, int64_t row_stride,
                        const float* gamma, double eps, double* out /* [T,d] */) {
    if (T < 0 || d <= 0 || row_stride < d) return -1;
    for (int64_t t = 0; t < T; ++t) {
        double ss = 0.0;
        for (int64_t i = 0; i < d; ++i) {
            double x = widen(hidden, dtype, t * row_stride + i);
            ss += x * x;
        }
        double r = 1.0 / sqrt(ss / (double)d + eps);
        for (int64_t i = 0; i < d; ++i) {
            double g = gamma ? (double)gamma[i] : 1.0;
            out[t * d + i] = widen(hidden, dtype, t * row_stride + i) * r * g;
        }
    }
    return 0;
}

/* ---- exported: one router over T rows ---- */

int tide_oracle_router_eval(const void* hidden, int dtype, int64_t T, int64_t d, int64_t b,
                            int64_t row_stride, const float* gamma, double eps, const float* W1,
                            const float* b1, const float* w2, double b2, double theta,
                            double* logit /* [T] */, double* prob /* [T] */,
                            uint8_t* fire /* [T] */) {
    if (T < 0 || d <= 0 || b <= 0 || row_stride < d) return -1;
    int fail = 0;
#pragma omp parallel
    {
        double* norm = (double*)malloc(sizeof(double) * (size_t)d);
        double* act = (double*)malloc(sizeof(double) * (size_t)b);
        if (!norm || !act) {
#pragma omp atomic write
            fail = 1;
        } else {
#pragma omp for schedule(static)
            for (int64_t t = 0; t < T; ++t) {
                double z = router_logit_row(hidden, dtype, t * row_stride, d, b, gamma, eps, W1,
                                            b1, w2, b2, norm, act);
                if (logit) logit[t] = z;
                if (prob) prob[t] = sigmoid(z);
                if (fire) fire[t] = (uint8_t)fires(z, theta);
            }
        }
        free(norm);
        free(act);
    }
    return fail ? -2 : 0;
}

/* ---- exported: earliest exit over C checkpoints (Fig. 1 step 3, Alg. 1) ---- */

/* hidden [C,T,d] with strides in elements; gamma [C,d] (or NULL), W1 [C,d,b],
 * b1 [C,b] (or NULL), w2 [C,b], b2 [C], theta [C]; layer_ids [C] ascending.   */
int tide_oracle_select_exit(const void* hidden, int dtype, int64_t C, int64_t T, int64_t d,
                            int64_t b, int64_t ckpt_stride, int64_t row_stride, const float* gamma,
                            double eps, const float* W1, const float* b1, const float* w2,
                            const float* b2, const float* theta, const int32_t* layer_ids,
                            int32_t min_layer, int32_t no_exit_layer,
                            int32_t* exit_layer /* [T] */, double* logits /* [C,T] or NULL */,
                            uint32_t* fire_mask /* [T] or NULL, bit c = fired at checkpoint c */) {
    if (C < 1 || C > 32 || T < 0 || d <= 0 || b <= 0 || row_stride < d) return -1;
    for (int64_t c = 1; c < C; ++c)
        if (layer_ids[c] <= layer_ids[c - 1]) return -1;
    int fail = 0;
#pragma omp parallel
    {
        double* norm = (double*)malloc(sizeof(double) * (size_t)d);
        double* act = (double*)malloc(sizeof(double) * (size_t)b);
        if (!norm || !act) {
#pragma omp atomic write
            fail = 1;
        } else {
#pragma omp for schedule(static)
            for (int64_t t = 0; t < T; ++t) {
                int32_t chosen = no_exit_layer;
                int found = 0;
                uint32_t mask = 0;
                /* every checkpoint is evaluated so that logits/fire_mask are complete;
                 * the exit is the first one, in ascending order, that is eligible and fires */
                for (int64_t c = 0; c < C; ++c) {
                    double z = router_logit_row(
                        hidden, dtype, c * ckpt_stride + t * row_stride, d, b,
                        gamma ? gamma + c * d : NULL, eps, W1 + c * d * b,
                        b1 ? b1 + c * b : NULL, w2 + c * b, (double)b2[c], norm, act);
                    int f = fires(z, (double)theta[c]);
                    if (logits) logits[c * T + t] = z;
                    if (f) mask |= (uint32_t)1 << c;
                    if (f && !found && layer_ids[c] >= min_layer) {
                        chosen = layer_ids[c];
                        found = 1;
                    }
                }
                exit_layer[t] = chosen;
                if (fire_mask) fire_mask[t] = mask;
            }
        }
        free(norm);
        free(act);
    }
    return fail ? -2 : 0;
}

/* ---- exported: selection alone, from given fire bits (Alg. 1 lines 3-9 per token) ---- */

int tide_oracle_exit_from_fire(const uint8_t* fire /* [C,T] */, int64_t C, int64_t T,
                               const int32_t* layer_ids, int32_t min_layer, int32_t no_exit_layer,
                               int32_t* exit_layer /* [T] */) {
    if (C < 1 || T < 0) return -1;
    for (int64_t t = 0; t < T; ++t) {
        exit_layer[t] = no_exit_layer;
        for (int64_t c = 0; c < C; ++c) {
            if (layer_ids[c] < min_layer) continue;
            if (fire[c * T + t]) {
                exit_layer[t] = layer_ids[c];
                break;
            }
        }
    }
    return 0;
}

/* ---- exported: batch compaction (Sec. 3.4 kernel 2) ---- */

/* Separates the tokens that have exited at or before `layer` (exit_layer[t] <= layer) from those
 * that continue, as two index lists in ascending token order.  counts[0] = exited, counts[1] =
 * continuing.  exit_idx and cont_idx have room for T entries each; entries past the counts are
 * left untouched.                                                                             */
int tide_oracle_batch_compact(const int32_t* exit_layer, int64_t T, int32_t layer, int32_t* exit_idx,
                              int32_t* cont_idx, int32_t* counts) {
    if (T < 0) return -1;
    int32_t ne = 0, nc = 0;
    for (int64_t t = 0; t < T; ++t) {
        if (exit_layer[t] <= layer) exit_idx[ne++] = (int32_t)t;
        else cont_idx[nc++] = (int32_t)t;
    }
    counts[0] = ne;
    counts[1] = nc;
    return 0;
}

/* ---- exported: convergence labels of the calibration stage, Eq. (1) ---- */

/* s_k = (h_k . h_L) / (|h_k| |h_L|) per token and checkpoint; label = 1[s_k > tau] (strict;
 * tau = 0.98 in the paper).  hidden [C,T,d], final_hidden [T,d] (the last layer's states).
 * A zero vector gives 0/0 = NaN and the label 0.                                             */
int tide_oracle_cosine_labels(const void* hidden, int dtype, int64_t C, int64_t T, int64_t d,
                              int64_t ckpt_stride, int64_t row_stride, const void* final_hidden,
                              int64_t final_row_stride, double tau, double* sim /* [C,T] */,
                              uint8_t* label /* [C,T] */) {
    if (C < 1 || T < 0 || d <= 0 || row_stride < d || final_row_stride < d) return -1;
#pragma omp parallel for schedule(static)
    for (int64_t t = 0; t < T; ++t) {
        double nl = 0.0;
        for (int64_t i = 0; i < d; ++i) {
            double y = widen(final_hidden, dtype, t * final_row_stride + i);
            nl += y * y;
        }
        for (int64_t c = 0; c < C; ++c) {
            double dot = 0.0, nk = 0.0;
            for (int64_t i = 0; i < d; ++i) {
                double x = widen(hidden, dtype, c * ckpt_stride + t * row_stride + i);
                double y = widen(final_hidden, dtype, t * final_row_stride + i);
                dot += x * y;
                nk += x * x;
            }
            double s = dot / (sqrt(nk) * sqrt(nl));
            if (sim) sim[c * T + t] = s;
            if (label) label[c * T + t] = (uint8_t)(s > tau);
        }
    }
    return 0;
}

/* ---- exported: whole-batch exit, Alg. 1 read literally ---- */

/* Alg. 1 walks the checkpoints in ascending order, skips those below k_min and returns at the
 * first one whose score exceeds theta "for all tokens in batch"; otherwise there is no early
 * exit.  fire [C,T] are the per-token threshold tests.  Also returns, per checkpoint, how many
 * tokens fired (the numbers behind Table 1's distribution column).                           */
int tide_oracle_batch_exit(const uint8_t* fire /* [C,T] */, int64_t C, int64_t T,
                           const int32_t* layer_ids, int32_t min_layer, int32_t no_exit_layer,
                           int32_t* batch_exit_layer, int64_t* fire_counts /* [C] or NULL */) {
    if (C < 1 || T < 0) return -1;
    *batch_exit_layer = no_exit_layer;
    int decided = 0;
    for (int64_t c = 0; c < C; ++c) {
        int64_t n = 0;
        for (int64_t t = 0; t < T; ++t) n += fire[c * T + t] ? 1 : 0;
        if (fire_counts) fire_counts[c] = n;
        if (!decided && layer_ids[c] >= min_layer && n == T && T > 0) {
            *batch_exit_layer = layer_ids[c];
            decided = 1;
        }
    }
    return 0;
}

/* ---- exported: exit projection (Fig. 1 output box, Alg. 1 line 5, Sec. 3.4 kernels 3-4) ---- */

/* hidden [C,T,d] (strides in elements), final_hidden [T,d] or NULL, exit_layer [T],
 * layer_ids [C], gain [d] or NULL (ones).  out [T,d] in the storage type.  A token whose
 * exit_layer is not a checkpoint layer takes final_hidden's row, or is left untouched when
 * final_hidden is NULL.  written[t] (optional) = 1 iff row t of out was written.            */
int tide_oracle_exit_project(const void* hidden, int dtype, int64_t C, int64_t T, int64_t d,
                             int64_t ckpt_stride, int64_t row_stride, const void* final_hidden,
                             int64_t final_row_stride, const int32_t* exit_layer,
                             const int32_t* layer_ids, const float* gain, double eps, void* out,
                             int64_t out_row_stride, uint8_t* written) {
    if (C < 1 || T < 0 || d <= 0 || row_stride < d || out_row_stride < d) return -1;
    for (int64_t t = 0; t < T; ++t) {
        const void* src = NULL;
        int64_t off = 0;
        for (int64_t c = 0; c < C; ++c)
            if (layer_ids[c] == exit_layer[t]) {
                src = hidden;
                off = c * ckpt_stride + t * row_stride;
                break;
            }
        if (!src && final_hidden) {
            src = final_hidden;
            off = t * final_row_stride;
        }
        if (written) written[t] = src ? 1 : 0;
        if (!src) continue;
        double ss = 0.0;
        for (int64_t i = 0; i < d; ++i) {
            double x = widen(src, dtype, off + i);
            ss += x * x;
        }
        double r = 1.0 / sqrt(ss / (double)d + eps);
        for (int64_t i = 0; i < d; ++i) {
            double g = gain ? (double)gain[i] : 1.0;
            double y = widen(src, dtype, off + i) * r * g;
            store_exact(out, dtype, t * out_row_stride + i, round_to_storage(y, dtype));
        }
    }
    return 0;
}

double tide_oracle_round_to_storage(double v, int dtype) { return round_to_storage(v, dtype); }

/* ---- exported: scalar helpers, so that the pins can probe them directly ---- */

double tide_oracle_sigmoid(double x) { return sigmoid(x); }
double tide_oracle_silu(double x) { return silu(x); }
int tide_oracle_fires(double z, double theta) { return fires(z, theta); }
double tide_oracle_widen(const void* p, int dtype, int64_t i) { return widen(p, dtype, i); }

/* ---- threads ---- */

int tide_oracle_max_threads(void) {
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

void tide_oracle_set_threads(int n) {
#ifdef _OPENMP
    if (n > 0) omp_set_num_threads(n);
#else
    (void)n;
#endif
}
