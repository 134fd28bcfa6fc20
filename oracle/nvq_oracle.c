/*
 * nvq_oracle.c -- plain CPU oracle for the int4-weight decode linears.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, obviously-correct
 * definition that the GPU library is checked against.  It shares no code,
 * header, table or helper with the HIP path; only tests, the smoke check and
 * the benchmark's cpu_baseline leg may build or call it.
 *
 * What it follows (paper: "Per-Layer Precision Dispatch and the W4A8 Path",
 * and appendix "CUDA Kernel Implementation Details"):
 *   - weights: blocks of 32 along K, one fp16 scale per block, 4-bit codes
 *     stored as unsigned nibbles centred at 8 (signed code = nibble - 8);
 *   - activation quantisation: s = amax / 127, q = round(x / s), clamped to
 *     [-127, 127], reused by every matmul that reads the same input;
 *   - W4A8: int32 sum of code * q per block, then multiplied by s_w * s_x;
 *     the identity  sum (nib-8) q = sum nib q - 8 sum q  is the paper's
 *     "deferred bias correction" (checked in tests, not used here: the oracle
 *     evaluates the left-hand side, which is the plain definition);
 *   - W4A16: same weights against 16-bit float activations, wide accumulate;
 *   - routing: W4A16 if normalised score >= tau else W4A8 (Algorithm 1).
 *
 * Readings where the paper is silent (all listed in the design notes):
 *   weight scale = absmax / 7 rounded to fp16 (round-to-nearest-even);
 *   "round" = round-half-to-even; "/" = IEEE binary32 division;
 *   a zero scale gives all-zero codes; activations are bfloat16;
 *   activation scale is per token (act_group = 0) or per 32 (act_group = 32).
 *
 * Packed layout (byte-for-byte contract with the GPU library):
 *   qweight[n][g*16 + j], j < 16: low nibble = element 32g + j,
 *                                 high nibble = element 32g + 16 + j,
 *   stored nibble = code + 8;  scales[n][g] = IEEE binary16 bits.
 *
 * All floating-point outputs are accumulated in double and returned as
 * double; the caller rounds to the output type.  Loops are written in the
 * order of the definitions; OpenMP only distributes independent output rows.
 *
 * Pins (tests/test_oracle_*.py): fp16/bf16 conversions against numpy's
 * float16 over all 65536 halves and against struct-packed floats; hand cases
 * with power-of-two scales that separate half-to-even from half-away; the
 * |w - c s| <= s/2 bound; brute-force integer sums at the +-32512 extreme;
 * float64 numpy mat-vec on dequantised operands; the paper's score table with
 * its threshold counts.  No function here is "parity unpinned".
 */
#include <math.h>
#include <stdint.h>
#include <string.h>
#include <stddef.h>

#define ORC_OK 0
#define ORC_ERR_ARG 1
#define ORC_ERR_SHAPE 2
#define ORC_ERR_RANGE 3

/* ---------- number formats ------------------------------------------------ */

static float bits_to_float(uint32_t u) { float f; memcpy(&f, &u, 4); return f; }
static uint32_t float_to_bits(float f) { uint32_t u; memcpy(&u, &f, 4); return u; }

/* bfloat16 is the top half of a binary32: widening is exact. */
float orc_bf16_to_float(uint16_t h) { return bits_to_float((uint32_t)h << 16); }

/* binary32 -> bfloat16, round to nearest even (input generators use it). */
uint16_t orc_float_to_bf16(float f) {
    uint32_t u = float_to_bits(f);
    if ((u & 0x7fffffffu) > 0x7f800000u) return (uint16_t)((u >> 16) | 0x40u); /* NaN */
    uint32_t lsb = (u >> 16) & 1u;
    u += 0x7fffu + lsb;
    return (uint16_t)(u >> 16);
}

/* binary16 -> binary32, exact (normals, subnormals, inf, nan). */
float orc_half_to_float(uint16_t h) {
    uint32_t sign = (uint32_t)(h & 0x8000u) << 16;
    int exp = (h >> 10) & 0x1f;
    uint32_t man = h & 0x3ffu;
    if (exp == 0x1f) return bits_to_float(sign | 0x7f800000u | (man << 13));
    if (exp == 0) {
        /* subnormal: man * 2^-24, exact in binary32 */
        float v = (float)man * bits_to_float(0x33800000u); /* 2^-24 */
        return sign ? -v : v;
    }
    return bits_to_float(sign | ((uint32_t)(exp + 112) << 23) | (man << 13));
}

/* binary32 -> binary16, round to nearest even, overflow to inf. */
uint16_t orc_float_to_half(float f) {
    uint32_t u = float_to_bits(f);
    uint16_t sign = (uint16_t)((u >> 16) & 0x8000u);
    uint32_t a = u & 0x7fffffffu;
    if (a > 0x7f800000u) return (uint16_t)(sign | 0x7e00u);          /* NaN */
    if (a >= 0x47800000u) return (uint16_t)(sign | 0x7c00u);         /* >= 65536 (incl. inf) */
    if (a >= 0x38800000u) {                                          /* normal half range */
        uint32_t man = a & 0x7fffffu;
        uint32_t exp = (a >> 23) - 112u;                             /* 1..30 */
        uint32_t half = (exp << 10) | (man >> 13);
        uint32_t rem = man & 0x1fffu;
        if (rem > 0x1000u || (rem == 0x1000u && (half & 1u))) half++; /* may carry to inf: correct */
        return (uint16_t)(sign | half);
    }
    if (a < 0x33000000u) return sign;                                /* < 2^-25: rounds to zero */
    /* subnormal half: value = m * 2^-24 with m = round(a_value * 2^24) */
    {
        int e = (int)(a >> 23);                  /* biased exponent, 102..112 */
        uint32_t man = (a & 0x7fffffu) | 0x800000u; /* 24-bit significand */
        int shift = 126 - e;                     /* 14..24: bits to drop */
        uint32_t half = man >> shift;
        uint32_t rem = man & ((1u << shift) - 1u);
        uint32_t mid = 1u << (shift - 1);
        if (rem > mid || (rem == mid && (half & 1u))) half++;
        return (uint16_t)(sign | half);
    }
}

/* ---------- a1: weight quantise + pack ------------------------------------ */
/* W [N][K] fp32 -> qweight [N][K/2], scales [N][K/32] (fp16 bits).
 * Returns ORC_ERR_RANGE if some block's absmax/7 does not fit fp16. */
int orc_pack_int4(const float *W, int64_t N, int64_t K,
                  uint8_t *qweight, uint16_t *scales) {
    if (!W || !qweight || !scales) return ORC_ERR_ARG;
    if (N <= 0 || K <= 0 || (K % 32) != 0) return ORC_ERR_SHAPE;
    const int64_t G = K / 32;
    int bad = 0;
#pragma omp parallel for schedule(static) reduction(| : bad)
    for (int64_t n = 0; n < N; ++n) {
        for (int64_t g = 0; g < G; ++g) {
            const float *w = W + n * K + g * 32;
            float amax = 0.0f;
            for (int j = 0; j < 32; ++j) {
                float a = fabsf(w[j]);
                if (a > amax) amax = a;
            }
            float s32 = amax / 7.0f;
            uint16_t s16 = orc_float_to_half(s32);
            if ((s16 & 0x7c00u) == 0x7c00u) bad |= 1;
            float s = orc_half_to_float(s16);
            int code[32];
            for (int j = 0; j < 32; ++j) {
                int c = 0;
                if (s != 0.0f && (s16 & 0x7c00u) != 0x7c00u) {
                    float r = rintf(w[j] / s);
                    if (r < -8.0f) r = -8.0f;
                    if (r > 7.0f) r = 7.0f;
                    c = (int)r;
                }
                code[j] = c;
            }
            uint8_t *q = qweight + n * (K / 2) + g * 16;
            for (int j = 0; j < 16; ++j)
                q[j] = (uint8_t)((code[j] + 8) | ((code[j + 16] + 8) << 4));
            scales[n * G + g] = s16;
        }
    }
    return bad ? ORC_ERR_RANGE : ORC_OK;
}

/* signed code of element k of row n */
static inline int code_at(const uint8_t *qrow, int64_t k) {
    int64_t g = k / 32, j = k % 32;
    uint8_t b = qrow[g * 16 + (j % 16)];
    int nib = (j < 16) ? (b & 0x0f) : (b >> 4);
    return nib - 8;
}

/* Dequantise to double: Wd[n][k] = code * float(scale).  Test helper. */
int orc_dequant_int4(const uint8_t *qweight, const uint16_t *scales,
                     int64_t N, int64_t K, double *Wd) {
    if (!qweight || !scales || !Wd) return ORC_ERR_ARG;
    if (N <= 0 || K <= 0 || (K % 32) != 0) return ORC_ERR_SHAPE;
    const int64_t G = K / 32;
    for (int64_t n = 0; n < N; ++n)
        for (int64_t k = 0; k < K; ++k)
            Wd[n * K + k] = (double)code_at(qweight + n * (K / 2), k) *
                            (double)orc_half_to_float(scales[n * G + k / 32]);
    return ORC_OK;
}

/* Dense bf16 weights for the prefill path (paper: kernel table, the
 * dequantisation kernel that materialises 16-bit weights for a library GEMM;
 * here the 16-bit type is bf16).  out[n][k] = bf16_rne(code * scale); the
 * product of a 4-bit code and an fp16 scale is exact in binary32, so the only
 * rounding is the one to bf16. */
int orc_dequant_bf16(const uint8_t *qweight, const uint16_t *scales,
                     int64_t N, int64_t K, uint16_t *out) {
    if (!qweight || !scales || !out) return ORC_ERR_ARG;
    if (N <= 0 || K <= 0 || (K % 32) != 0) return ORC_ERR_SHAPE;
    const int64_t G = K / 32;
    for (int64_t n = 0; n < N; ++n)
        for (int64_t k = 0; k < K; ++k) {
            const double v = (double)code_at(qweight + n * (K / 2), k) *
                             (double)orc_half_to_float(scales[n * G + k / 32]);
            out[n * K + k] = orc_float_to_bf16((float)v);   /* (float)v is exact */
        }
    return ORC_OK;
}

/* ---------- a2: activation quantisation ----------------------------------- */
/* x bf16 [M][K] -> xq int8 [M][K]; xscale fp32 [M] (act_group 0) or
 * [M][K/32] (act_group 32); xgsum int32 [M][K/32] = sum of codes per block
 * of 32 (may be NULL). */
int orc_quant_act_i8(const uint16_t *x, int64_t M, int64_t K, int act_group,
                     int8_t *xq, float *xscale, int32_t *xgsum) {
    if (!x || !xq || !xscale) return ORC_ERR_ARG;
    if (M <= 0 || K <= 0 || (K % 32) != 0) return ORC_ERR_SHAPE;
    if (act_group != 0 && act_group != 32) return ORC_ERR_ARG;
    const int64_t G = K / 32;
    const int64_t span = act_group == 0 ? K : 32;   /* elements sharing a scale */
    const int64_t nspan = K / span;
    for (int64_t m = 0; m < M; ++m) {
        for (int64_t b = 0; b < nspan; ++b) {
            const uint16_t *xb = x + m * K + b * span;
            float amax = 0.0f;
            for (int64_t j = 0; j < span; ++j) {
                float a = fabsf(orc_bf16_to_float(xb[j]));
                if (a > amax) amax = a;
            }
            float s = amax / 127.0f;
            xscale[m * nspan + b] = s;
            for (int64_t j = 0; j < span; ++j) {
                int q = 0;
                if (s != 0.0f) {
                    float r = rintf(orc_bf16_to_float(xb[j]) / s);
                    if (r < -127.0f) r = -127.0f;
                    if (r > 127.0f) r = 127.0f;
                    q = (int)r;
                }
                xq[m * K + b * span + j] = (int8_t)q;
            }
        }
        if (xgsum) {
            for (int64_t g = 0; g < G; ++g) {
                int32_t t = 0;
                for (int j = 0; j < 32; ++j) t += xq[m * K + g * 32 + j];
                xgsum[m * G + g] = t;
            }
        }
    }
    return ORC_OK;
}

/* ---------- a3: W4A8 ------------------------------------------------------ */
/* acc[m][n][g] = sum_{j<32} code[n][32g+j] * xq[m][32g+j]        (int32)
 * y[m][n] = s_x[m] * sum_g s_w[n][g] * acc            (act_group 0)
 *         = sum_g s_w[n][g] * s_x[m][g] * acc         (act_group 32)
 * y is double [M][N]; acc may be NULL. */
int orc_gemv_w4a8(const uint8_t *qweight, const uint16_t *scales, int64_t N, int64_t K,
                  const int8_t *xq, const float *xscale, int act_group, int64_t M,
                  double *y, int32_t *acc) {
    if (!qweight || !scales || !xq || !xscale || !y) return ORC_ERR_ARG;
    if (N <= 0 || M <= 0 || K <= 0 || (K % 32) != 0) return ORC_ERR_SHAPE;
    if (act_group != 0 && act_group != 32) return ORC_ERR_ARG;
    const int64_t G = K / 32;
#pragma omp parallel for schedule(static)
    for (int64_t n = 0; n < N; ++n) {
        const uint8_t *qrow = qweight + n * (K / 2);
        for (int64_t m = 0; m < M; ++m) {
            double total = 0.0;
            for (int64_t g = 0; g < G; ++g) {
                int32_t a = 0;
                for (int j = 0; j < 32; ++j)
                    a += code_at(qrow, g * 32 + j) * (int32_t)xq[m * K + g * 32 + j];
                if (acc) acc[(m * N + n) * G + g] = a;
                double sw = (double)orc_half_to_float(scales[n * G + g]);
                if (act_group == 0) total += sw * (double)a;
                else total += sw * (double)xscale[m * G + g] * (double)a;
            }
            if (act_group == 0) total *= (double)xscale[m];
            y[m * N + n] = total;
        }
    }
    return ORC_OK;
}

/* The same integer block sums written the paper's way: unsigned nibble dot
 * product minus 8 * (sum of activation codes).  Exists so that a test can
 * check the deferred-correction identity as an integer equality. */
int orc_w4a8_acc_deferred(const uint8_t *qweight, int64_t N, int64_t K,
                          const int8_t *xq, const int32_t *xgsum, int64_t M,
                          int32_t *acc) {
    if (!qweight || !xq || !xgsum || !acc) return ORC_ERR_ARG;
    if (N <= 0 || M <= 0 || K <= 0 || (K % 32) != 0) return ORC_ERR_SHAPE;
    const int64_t G = K / 32;
    for (int64_t n = 0; n < N; ++n)
        for (int64_t m = 0; m < M; ++m)
            for (int64_t g = 0; g < G; ++g) {
                int32_t sumi = 0;
                for (int j = 0; j < 32; ++j) {
                    int nib = code_at(qweight + n * (K / 2), g * 32 + j) + 8;
                    sumi += nib * (int32_t)xq[m * K + g * 32 + j];
                }
                acc[(m * N + n) * G + g] = sumi - 8 * xgsum[m * G + g];
            }
    return ORC_OK;
}

/* ---------- a4: W4A16 ----------------------------------------------------- */
/* y[m][n] = sum_g s_w[n][g] * sum_{j<32} code * x[m][32g+j], double. */
int orc_gemv_w4a16(const uint8_t *qweight, const uint16_t *scales, int64_t N, int64_t K,
                   const uint16_t *x, int64_t M, double *y) {
    if (!qweight || !scales || !x || !y) return ORC_ERR_ARG;
    if (N <= 0 || M <= 0 || K <= 0 || (K % 32) != 0) return ORC_ERR_SHAPE;
    const int64_t G = K / 32;
#pragma omp parallel for schedule(static)
    for (int64_t n = 0; n < N; ++n) {
        const uint8_t *qrow = qweight + n * (K / 2);
        for (int64_t m = 0; m < M; ++m) {
            double total = 0.0;
            for (int64_t g = 0; g < G; ++g) {
                double inner = 0.0;
                for (int j = 0; j < 32; ++j)
                    inner += (double)code_at(qrow, g * 32 + j) *
                             (double)orc_bf16_to_float(x[m * K + g * 32 + j]);
                total += (double)orc_half_to_float(scales[n * G + g]) * inner;
            }
            y[m * N + n] = total;
        }
    }
    return ORC_OK;
}

/* ---------- input transforms of a linear layer (neighbouring decode kernels) -- */
/* Round a double to bf16, to nearest, ties to even, in ONE step (going through
 * float first could round twice).  Finite inputs in the normal bf16 range. */
uint16_t orc_double_to_bf16(double v) {
    uint16_t b = orc_float_to_bf16((float)v);
    /* the right answer is b or one of its neighbours: take the nearest of the
     * three, an exact tie goes to the even pattern */
    uint16_t best = b;
    double bd = fabs((double)orc_bf16_to_float(b) - v);
    for (int d = -1; d <= 1; d += 2) {
        uint16_t c = (uint16_t)(b + d);
        if ((c & 0x7f80u) == 0x7f80u || ((b ^ c) & 0x8000u)) continue; /* inf/nan, sign change */
        double cd = fabs((double)orc_bf16_to_float(c) - v);
        if (cd < bd || (cd == bd && (c & 1u) == 0 && (best & 1u) == 1)) {
            best = c;
            bd = cd;
        }
    }
    return best;
}

/* RMSNorm in front of a linear layer (paper: kernel table, the single-pass
 * RMS-norm kernel; the formula is the usual one, the paper does not restate
 * it).  Per token: h = x (+ res, rounded to bf16: the updated residual stream,
 * stored to h_out if given); out_k = bf16(h_k * gamma_k / sqrt(mean(h^2) + eps)).
 * x, res, out, h_out: bf16 [M][K]; gamma: bf16 [K]; res and h_out may be NULL. */
int orc_rms_norm(const uint16_t *x, const uint16_t *res, const uint16_t *gamma, double eps,
                 int64_t M, int64_t K, uint16_t *out, uint16_t *h_out) {
    if (!x || !gamma || !out) return ORC_ERR_ARG;
    if (M <= 0 || K <= 0) return ORC_ERR_SHAPE;
    for (int64_t m = 0; m < M; ++m) {
        double ss = 0.0;
        for (int64_t k = 0; k < K; ++k) {
            uint16_t hb = x[m * K + k];
            if (res)
                hb = orc_double_to_bf16((double)orc_bf16_to_float(hb) +
                                        (double)orc_bf16_to_float(res[m * K + k]));
            if (h_out) h_out[m * K + k] = hb;
            out[m * K + k] = hb; /* parked, normalised below */
            const double h = (double)orc_bf16_to_float(hb);
            ss += h * h;
        }
        const double r = 1.0 / sqrt(ss / (double)K + eps);
        for (int64_t k = 0; k < K; ++k) {
            const double h = (double)orc_bf16_to_float(out[m * K + k]);
            out[m * K + k] = orc_double_to_bf16(h * r * (double)orc_bf16_to_float(gamma[k]));
        }
    }
    return ORC_OK;
}

/* SiLU(gate) * up in front of the down projection (paper: kernel table, the
 * SiLU-multiply kernel).  out_k = bf16(g_k / (1 + exp(-g_k)) * u_k). */
int orc_silu_mul(const uint16_t *g, const uint16_t *u, int64_t M, int64_t K, uint16_t *out) {
    if (!g || !u || !out) return ORC_ERR_ARG;
    if (M <= 0 || K <= 0) return ORC_ERR_SHAPE;
    for (int64_t i = 0; i < M * K; ++i) {
        const double gv = (double)orc_bf16_to_float(g[i]);
        const double uv = (double)orc_bf16_to_float(u[i]);
        out[i] = orc_double_to_bf16(gv / (1.0 + exp(-gv)) * uv);
    }
    return ORC_OK;
}

/* ---------- a5: walk a layer list under a precision map ------------------- */
typedef struct {
    const uint8_t *qweight;   /* [N][K/2] */
    const uint16_t *scales;   /* [N][K/32] */
    int64_t N, K;
    const uint16_t *x;        /* bf16 [M][K] */
    double *y;                /* [M][N] */
    int precision;            /* 0 = W4A8, 1 = W4A16 */
    int in_op;                /* 0 = x as it is, 1 = RMSNorm(x (+ x2)) * gamma, 2 = SiLU(x) * x2 */
    const uint16_t *x2;       /* bf16 [M][K] or NULL */
    const uint16_t *gamma;    /* bf16 [K] (in_op 1) */
    double eps;               /* (in_op 1) */
    uint16_t *h_out;          /* bf16 [M][K] or NULL: x + x2 (in_op 1 with x2) */
    uint16_t *xt;             /* bf16 [M][K] scratch for the transformed input (in_op != 0) */
} orc_linear;

/* Entries run in order.  A W4A8 entry quantises its input first (an entry
 * that reads the same x as its predecessor would reuse the codes; the result
 * is identical, so the oracle simply recomputes).  scratch_q: >= M*maxK
 * bytes, scratch_s: >= M*maxK/32 floats. */
int orc_decode_linears(const orc_linear *L, int64_t n, int64_t M, int act_group,
                       int8_t *scratch_q, float *scratch_s) {
    if (!L || n < 0 || !scratch_q || !scratch_s) return ORC_ERR_ARG;
    for (int64_t i = 0; i < n; ++i) {
        int rc;
        const uint16_t *x = L[i].x;
        if (L[i].in_op == 1) {
            rc = orc_rms_norm(L[i].x, L[i].x2, L[i].gamma, L[i].eps, M, L[i].K, L[i].xt,
                              L[i].h_out);
            if (rc) return rc;
            x = L[i].xt;
        } else if (L[i].in_op == 2) {
            rc = orc_silu_mul(L[i].x, L[i].x2, M, L[i].K, L[i].xt);
            if (rc) return rc;
            x = L[i].xt;
        } else if (L[i].in_op != 0) {
            return ORC_ERR_ARG;
        }
        if (L[i].precision == 1) {
            rc = orc_gemv_w4a16(L[i].qweight, L[i].scales, L[i].N, L[i].K, x, M, L[i].y);
        } else if (L[i].precision == 0) {
            rc = orc_quant_act_i8(x, M, L[i].K, act_group, scratch_q, scratch_s, NULL);
            if (rc) return rc;
            rc = orc_gemv_w4a8(L[i].qweight, L[i].scales, L[i].N, L[i].K, scratch_q,
                               scratch_s, act_group, M, L[i].y, NULL);
        } else {
            rc = ORC_ERR_ARG;
        }
        if (rc) return rc;
    }
    return ORC_OK;
}

/* ---------- activation magnitudes and scores (Algorithm 1) ----------------- */
/* The two magnitudes Algorithm 1 takes per layer and token are Euclidean norms
 * of output vectors: of the query and value projections side by side (the
 * attention proxy) and of the feed-forward block's output.  out[m] =
 * sqrt(sum_n a[m][n]^2 + sum_n b[m][n]^2); b may be NULL (Nb = 0).
 * dtype 0: float32, 1: bf16 bits. */
static double elem_at(const void *p, int dtype, int64_t i) {
    return dtype == 0 ? (double)((const float *)p)[i]
                      : (double)orc_bf16_to_float(((const uint16_t *)p)[i]);
}
int orc_token_norms(const void *a, int64_t Na, const void *b, int64_t Nb, int64_t M, int dtype,
                    double *out) {
    if (!a || !out || (Nb > 0 && !b)) return ORC_ERR_ARG;
    if (Na <= 0 || Nb < 0 || M <= 0 || (dtype != 0 && dtype != 1)) return ORC_ERR_SHAPE;
    for (int64_t m = 0; m < M; ++m) {
        double sum = 0.0;
        for (int64_t n = 0; n < Na; ++n) {
            const double v = elem_at(a, dtype, m * Na + n);
            sum += v * v;
        }
        for (int64_t n = 0; n < Nb; ++n) {
            const double v = elem_at(b, dtype, m * Nb + n);
            sum += v * v;
        }
        out[m] = sqrt(sum);
    }
    return ORC_OK;
}

/* The score line of Algorithm 1: per layer the mean over the prompts of the
 * mean over a prompt's tokens of (attention proxy + feed-forward magnitude).
 * a_attn, a_ffn: [L][T] with the tokens of the k prompts one after the other,
 * T = sum of prompt_len. */
int orc_mcap_scores(const double *a_attn, const double *a_ffn, const int64_t *prompt_len,
                    int64_t k, int64_t L, double *s) {
    if (!a_attn || !a_ffn || !prompt_len || !s) return ORC_ERR_ARG;
    if (k <= 0 || L <= 0) return ORC_ERR_SHAPE;
    int64_t T = 0;
    for (int64_t j = 0; j < k; ++j) {
        if (prompt_len[j] <= 0) return ORC_ERR_SHAPE;
        T += prompt_len[j];
    }
    for (int64_t i = 0; i < L; ++i) {
        double over_prompts = 0.0;
        int64_t t0 = 0;
        for (int64_t j = 0; j < k; ++j) {
            double over_tokens = 0.0;
            for (int64_t t = t0; t < t0 + prompt_len[j]; ++t)
                over_tokens += a_attn[i * T + t] + a_ffn[i * T + t];
            over_prompts += over_tokens / (double)prompt_len[j];
            t0 += prompt_len[j];
        }
        s[i] = over_prompts / (double)k;
    }
    return ORC_OK;
}

/* ---------- routing rule (Algorithm 1, normalise + assign) ---------------- */
/* scores s[L] -> out[L]: 1 = W4A16 (normalised score >= tau), 0 = W4A8.
 * If max - min < eps every normalised score is 0. */
int orc_precision_from_scores(const double *s, int64_t L, double tau, double eps,
                              uint8_t *out, double *shat /* may be NULL */) {
    if (!s || !out || L <= 0) return ORC_ERR_ARG;
    double lo = s[0], hi = s[0];
    for (int64_t i = 1; i < L; ++i) {
        if (s[i] < lo) lo = s[i];
        if (s[i] > hi) hi = s[i];
    }
    for (int64_t i = 0; i < L; ++i) {
        double h = (hi - lo < eps) ? 0.0 : (s[i] - lo) / (hi - lo);
        if (shat) shat[i] = h;
        out[i] = (h >= tau) ? 1 : 0;
    }
    return ORC_OK;
}
