/*
 * CPU oracle for the Quant VideoGen KV-cache codec.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, plain reference that the
 * GPU library is checked against.  It shares no code, header, table or helper
 * with the HIP path, and nothing in the product path may call it.
 *
 * Every function follows one passage of the paper (section / equation given in
 * its comment) and is written as the definition reads: plain loops, fp64 where
 * the paper leaves the precision open, single IEEE fp32 operations where a
 * stored integer (a 2-bit code, a cluster id) depends on the rounding.
 * Compile with -ffp-contract=off so that no multiply-add is fused unless
 * fmaf() is written.
 *
 * Notation (paper Sec. 4 and Sec. 5 "Implementation"):
 *   N  tokens of one chunk of one head            d  head dimension
 *   K  number of centroids ("C groups" in Sec. 4) B  quantization group size
 *   S  smoothing stages (the paper's PRQ stages)  T  quantization rounds
 *   b  bit width, qmax = 2^(b-1) - 1 (Eq. 2)
 *
 * Pins (tests/test_oracle_*.py): brute-force numpy argmin, member-mean and
 * scipy/sklearn Lloyd, Eq. 3 error bound, exact-on-grid round trip, monotone
 * error in T, torch SDPA, numpy float16/bfloat16 conversions, and the paper's
 * printed compression ratios (Tables 1, 4, 5).
 * Cluster ids are 16-bit words here whatever K is (the codebook-size study of Sec. 5 goes to
 * K = 512); the Python wrapper hands them out as bytes when K <= 256, as a stored cache has them.
 * Parity unpinned: reconstruction quality on real model KV (Sec. 5 MSE gains)
 * cannot be checked here; no model weights exist in this build.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

/* cluster index of a token: 16 bits in memory here, whatever width a stored format gives it */
typedef uint16_t qid_t;

/* ------------------------------------------------------------------ */
/* number formats                                                     */
/* ------------------------------------------------------------------ */

static float bits_to_f32(uint32_t u) { float f; memcpy(&f, &u, 4); return f; }
static uint32_t f32_to_bits(float f) { uint32_t u; memcpy(&u, &f, 4); return u; }

/* bfloat16 is the upper half of an IEEE binary32. */
float qvgo_bf16_to_f32(uint16_t h) { return bits_to_f32((uint32_t)h << 16); }

/* binary32 -> bfloat16, round to nearest, ties to even. */
uint16_t qvgo_f32_to_bf16(float f) {
    uint32_t u = f32_to_bits(f);
    if ((u & 0x7fffffffu) > 0x7f800000u) return (uint16_t)((u >> 16) | 0x0040u); /* NaN */
    uint32_t lower = u & 0xffffu;
    uint32_t upper = u >> 16;
    if (lower > 0x8000u || (lower == 0x8000u && (upper & 1u))) upper += 1u;
    return (uint16_t)upper;
}

/* IEEE binary16 -> binary32 (exact). */
float qvgo_f16_to_f32(uint16_t h) {
    int sign = (h >> 15) & 1;
    int e = (h >> 10) & 0x1f;
    int m = h & 0x3ff;
    double v;
    if (e == 0)        v = ldexp((double)m, -24);               /* subnormal / zero */
    else if (e == 31)  v = m ? NAN : INFINITY;
    else               v = ldexp((double)(m + 1024), e - 25);
    return (float)(sign ? -v : v);
}

/* binary32 -> IEEE binary16, round to nearest, ties to even, with subnormals. */
uint16_t qvgo_f32_to_f16(float f) {
    uint32_t u = f32_to_bits(f);
    uint16_t sign = (uint16_t)((u >> 16) & 0x8000u);
    double a = fabs((double)f);
    if (isnan(f)) return (uint16_t)(sign | 0x7e00u);
    if (a >= 65520.0) return (uint16_t)(sign | 0x7c00u);       /* rounds to inf */
    if (a == 0.0) return sign;
    int e;
    (void)frexp(a, &e);                 /* a = m * 2^e, m in [0.5,1) */
    int ulp_exp = e - 11;               /* 11 significant bits for a normal */
    if (ulp_exp < -24) ulp_exp = -24;   /* subnormal spacing */
    double q = nearbyint(ldexp(a, -ulp_exp));   /* default mode: ties to even */
    double r = ldexp(q, ulp_exp);       /* exactly representable in binary16 */
    /* re-derive the fields from r */
    if (r == 0.0) return sign;
    if (r < ldexp(1.0, -14)) return (uint16_t)(sign | (uint16_t)ldexp(r, 24));
    (void)frexp(r, &e);                 /* r = m * 2^e, m in [0.5,1) */
    int be = e - 1 + 15;
    int mant = (int)(ldexp(r, 11 - e)) - 1024;
    return (uint16_t)(sign | (be << 10) | mant);
}

/* FP8 E4M3 (Sec. 5 "Implementation": the format of the per-group scales in the paper's
 * own kernels; the OCP 8-bit layout: 1 sign, 4 exponent bits with bias 7, 3 mantissa
 * bits, no infinity, S.1111.111 = NaN, largest finite 448, subnormals m/8 * 2^-6). */
float qvgo_e4m3_to_f32(uint8_t b) {
    int sign = (b >> 7) & 1, e = (b >> 3) & 0xf, m = b & 7;
    double v;
    if (e == 15 && m == 7) return NAN;
    if (e == 0) v = ldexp((double)m / 8.0, -6);
    else        v = ldexp(1.0 + (double)m / 8.0, e - 7);
    return (float)(sign ? -v : v);
}

/* binary32 -> E4M3: the nearest finite value, ties to the even code, found by
 * looking at every non-negative finite code.  Magnitudes beyond 448 saturate to
 * 448 (a scale must stay finite).  NaN -> the NaN code. */
uint8_t qvgo_f32_to_e4m3(float f) {
    uint8_t sign = (uint8_t)(signbit(f) ? 0x80 : 0);
    if (isnan(f)) return (uint8_t)(sign | 0x7f);
    double a = fabs((double)f);
    int best = 0;
    double bd = a;                                   /* distance to code 0 */
    for (int c = 1; c <= 0x7e; ++c) {
        double dist = fabs((double)qvgo_e4m3_to_f32((uint8_t)c) - a);
        if (dist < bd || (dist == bd && (c & 1) == 0)) { bd = dist; best = c; }
    }
    return (uint8_t)(sign | best);
}

/* ------------------------------------------------------------------ */
/* Sec. 4.1: semantic-based grouping (k-means)                        */
/* ------------------------------------------------------------------ */

/* Squared Euclidean distance between one token and one centroid, fp64,
 * channels in order.  The centroid is stored in bf16. */
static double sqdist(int d, const float *r, const uint16_t *c) {
    double acc = 0.0;
    for (int ch = 0; ch < d; ++ch) {
        double diff = (double)r[ch] - (double)qvgo_bf16_to_f32(c[ch]);
        acc += diff * diff;
    }
    return acc;
}

/* Assignment step of k-means (Sec. 4.1): every token joins the group whose
 * centroid is nearest; equal distances go to the lowest index.
 * best_dist (nullable) receives the winning squared distance. */
void qvgo_assign(int64_t N, int d, int K, const float *r, const uint16_t *cent,
                 qid_t *ids, double *best_dist) {
    for (int64_t n = 0; n < N; ++n) {
        int best = 0;
        double bd = sqdist(d, r + n * d, cent);
        for (int j = 1; j < K; ++j) {
            double dj = sqdist(d, r + n * d, cent + (int64_t)j * d);
            if (dj < bd) { bd = dj; best = j; }
        }
        ids[n] = (qid_t)best;
        if (best_dist) best_dist[n] = bd;
    }
}

/* Squared distance of each token to a GIVEN centroid index (for the tie
 * classification in the parity tests). */
void qvgo_dist_to(int64_t N, int d, const float *r, const uint16_t *cent,
                  const qid_t *ids, double *out) {
    for (int64_t n = 0; n < N; ++n)
        out[n] = sqdist(d, r + n * d, cent + (int64_t)ids[n] * d);
}

/* Update step (Sec. 4.1: the centroid is the mean value of its group).
 * Sum of the members in token order in fp64, divided by the member count,
 * rounded to binary32 and then to bf16 (the stored precision).  A group
 * without members keeps its previous centroid. */
void qvgo_update(int64_t N, int d, int K, const float *r, const qid_t *ids,
                 const uint16_t *cent_prev, uint16_t *cent_out, int32_t *counts) {
    double *sum = (double *)calloc((size_t)K * d, sizeof(double));
    int32_t *cnt = (int32_t *)calloc((size_t)K, sizeof(int32_t));
    for (int64_t n = 0; n < N; ++n) {
        int j = ids[n];
        cnt[j] += 1;
        for (int ch = 0; ch < d; ++ch) sum[(int64_t)j * d + ch] += (double)r[n * d + ch];
    }
    for (int j = 0; j < K; ++j) {
        for (int ch = 0; ch < d; ++ch) {
            int64_t o = (int64_t)j * d + ch;
            if (cnt[j] > 0) cent_out[o] = qvgo_f32_to_bf16((float)(sum[o] / (double)cnt[j]));
            else            cent_out[o] = cent_prev[o];
        }
        if (counts) counts[j] = cnt[j];
    }
    free(sum); free(cnt);
}

/* Lloyd iteration with a fixed count and a given start (Sec. 4.3: a chunk's
 * k-means starts from cached centroids): I times (assign, update), then one
 * more assign so that the ids belong to the stored centroids.
 * inertia (nullable, I+1 entries) receives the summed winning distance of
 * each assign pass. */
void qvgo_lloyd(int64_t N, int d, int K, int I, const float *r, const uint16_t *init,
                uint16_t *cent_out, qid_t *ids_out, double *inertia) {
    size_t tb = (size_t)K * d * sizeof(uint16_t);
    uint16_t *cur = (uint16_t *)malloc(tb), *nxt = (uint16_t *)malloc(tb);
    double *bd = (double *)malloc((size_t)(N > 0 ? N : 1) * sizeof(double));
    memcpy(cur, init, tb);
    for (int it = 0; it <= I; ++it) {
        qvgo_assign(N, d, K, r, cur, ids_out, bd);
        if (inertia) { double s = 0.0; for (int64_t n = 0; n < N; ++n) s += bd[n]; inertia[it] = s; }
        if (it == I) break;
        qvgo_update(N, d, K, r, ids_out, cur, nxt, NULL);
        uint16_t *t = cur; cur = nxt; nxt = t;
    }
    memcpy(cent_out, cur, tb);
    free(cur); free(nxt); free(bd);
}

/* Eq. 5: residual = token minus the centroid of its group (one fp32 subtract). */
void qvgo_residual(int64_t N, int d, const float *r_in, const uint16_t *cent,
                   const qid_t *ids, float *r_out) {
    for (int64_t n = 0; n < N; ++n)
        for (int ch = 0; ch < d; ++ch)
            r_out[n * d + ch] = r_in[n * d + ch] - qvgo_bf16_to_f32(cent[(int64_t)ids[n] * d + ch]);
}

/* ------------------------------------------------------------------ */
/* Sec. 3.2, Eq. 1-2: symmetric per-group integer quantization        */
/* ------------------------------------------------------------------ */

/* One round of b-bit group quantization of r, groups of B consecutive
 * channels of one token.  Scale = max|r| / qmax, stored in the scale format:
 * scale_fmt 0 = binary16, 1 = FP8 E4M3 (Sec. 5 "Implementation"), each rounded to
 * nearest even and saturated at the format's largest finite value; the
 * STORED scale is the one divided by, so that encode and decode agree.
 * q = round-half-even(r / scale) clamped to [-qmax, qmax].
 * The quantized part is removed from r in place: r <- r - scale*q (one fma),
 * which is what the next round sees.
 * q_out [N][d] signed levels; scales_out [N][d/B]: binary16 bits, or the E4M3
 * code in the low byte. */
static float scale_store(float s32, int scale_fmt, uint16_t *stored) {
    if (scale_fmt == 1) {
        if (s32 > 448.0f) s32 = 448.0f;                /* largest finite E4M3 */
        uint8_t c = qvgo_f32_to_e4m3(s32);
        *stored = c;
        return qvgo_e4m3_to_f32(c);
    }
    if (s32 > 65504.0f) s32 = 65504.0f;                /* largest finite binary16 */
    *stored = qvgo_f32_to_f16(s32);
    return qvgo_f16_to_f32(*stored);
}
static float scale_load(uint16_t stored, int scale_fmt) {
    return scale_fmt == 1 ? qvgo_e4m3_to_f32((uint8_t)stored) : qvgo_f16_to_f32(stored);
}

void qvgo_quant_round(int64_t N, int d, int B, int bits, int scale_fmt, float *r,
                      int8_t *q_out, uint16_t *scales_out) {
    const float qmax = (float)((1 << (bits - 1)) - 1);
    const int G = d / B;
    for (int64_t n = 0; n < N; ++n) {
        for (int g = 0; g < G; ++g) {
            float *rg = r + n * d + (int64_t)g * B;
            int8_t *qg = q_out + n * d + (int64_t)g * B;
            float m = 0.0f;
            for (int i = 0; i < B; ++i) { float a = fabsf(rg[i]); if (a > m) m = a; }
            float s = scale_store(m / qmax, scale_fmt, &scales_out[n * G + g]);
            if (s == 0.0f) { for (int i = 0; i < B; ++i) qg[i] = 0; continue; }
            float inv = 1.0f / s;
            for (int i = 0; i < B; ++i) {
                float u = rg[i] * inv;
                float q = rintf(u);                        /* ties to even */
                if (q > qmax) q = qmax;
                if (q < -qmax) q = -qmax;
                qg[i] = (int8_t)q;
                rg[i] = fmaf(-s, q, rg[i]);
            }
        }
    }
}

/* Bit packing of the stored codes (the paper leaves the packing open).  A level q in
 * [-qmax, qmax] is stored as its b-bit two's complement (q = -1 -> all ones), so a
 * signed bit-field extract returns q.  Element i of a token sits in byte i/(8/b), at
 * bit offset b*(i mod 8/b), lowest bits first.  n_elems must be a multiple of 8/b. */
void qvgo_pack(int64_t n_elems, int bits, const int8_t *q, uint8_t *packed) {
    const int per = 8 / bits, mask = (1 << bits) - 1;
    for (int64_t i = 0; i < n_elems / per; ++i) {
        unsigned byte = 0;
        for (int j = 0; j < per; ++j)
            byte |= ((unsigned)q[i * per + j] & (unsigned)mask) << (bits * j);
        packed[i] = (uint8_t)byte;
    }
}

void qvgo_unpack(int64_t n_elems, int bits, const uint8_t *packed, int8_t *q) {
    const int per = 8 / bits, mask = (1 << bits) - 1, sign = 1 << (bits - 1);
    for (int64_t i = 0; i < n_elems; ++i) {
        int code = (packed[i / per] >> (bits * (int)(i % per))) & mask;
        q[i] = (int8_t)((code & sign) ? code - (1 << bits) : code);
    }
}

/* ------------------------------------------------------------------ */
/* Sec. 4.2: encode one chunk of one head                             */
/* ------------------------------------------------------------------ */

/* S smoothing stages (each: k-means on the current residual, subtract the
 * assigned centroid, Eq. 5/6), then T rounds of b-bit group quantization of
 * what is left.  The paper's method is T = 1 (QVG: S = 1, QVG-Pro: S = 4);
 * S = 1 with T > 1 is the staged 2-bit quantization this build is graded on.
 * Sec. 4.2 does not say in which precision the residual travels from one
 * smoothing stage to the next; reading: as a bf16 tensor, the type of X itself
 * (one fp32 subtraction, rounded to nearest even), so every stage sees the same
 * kind of input.  The residual of the last stage is not stored and is quantized
 * from its fp32 value.
 *
 * x        [N][d] bf16
 * init     [S][K][d] bf16 start centroids per smoothing stage, or NULL
 * init_idx [K] token indices: when init is NULL, stage s starts from these
 *          tokens of its own input residual, rounded to bf16
 * I        Lloyd iterations (I = 0: one assign pass against the start centroids)
 * cent_out [S][K][d] bf16, ids_out [S][N]
 * codes_out [N][T][d*b/8], scales_out [N][T][d/B] (see qvgo_quant_round)
 * resid_out (nullable) [N][d] fp32: what remains after all rounds */
void qvgo_encode_unit(int64_t N, int d, int K, int B, int S, int T, int bits, int scale_fmt, int I,
                      const uint16_t *x, const uint16_t *init, const int32_t *init_idx,
                      uint16_t *cent_out, qid_t *ids_out,
                      uint8_t *codes_out, uint16_t *scales_out, float *resid_out) {
    const int G = d / B, cb = d * bits / 8;
    size_t nd = (size_t)(N > 0 ? N : 1) * d;
    float *r = (float *)malloc(nd * sizeof(float));
    float *r2 = (float *)malloc(nd * sizeof(float));
    int8_t *q = (int8_t *)malloc(nd);
    uint16_t *sc = (uint16_t *)malloc((size_t)(N > 0 ? N : 1) * G * sizeof(uint16_t));
    uint16_t *start = (uint16_t *)malloc((size_t)K * d * sizeof(uint16_t));
    for (int64_t i = 0; i < N * d; ++i) r[i] = qvgo_bf16_to_f32(x[i]);      /* R^(0) = X */

    for (int s = 0; s < S; ++s) {
        if (init) memcpy(start, init + (int64_t)s * K * d, (size_t)K * d * 2);
        else for (int j = 0; j < K; ++j)
            for (int ch = 0; ch < d; ++ch)
                start[j * d + ch] = qvgo_f32_to_bf16(r[(int64_t)init_idx[j] * d + ch]);
        uint16_t *cs = cent_out + (int64_t)s * K * d;
        qid_t *is = ids_out + (int64_t)s * N;
        qvgo_lloyd(N, d, K, I, r, start, cs, is, NULL);
        qvgo_residual(N, d, r, cs, is, r2);
        /* A residual that feeds another smoothing stage is a tensor of the input's type
         * (bf16, like X); the last one goes straight to the quantizer in fp32. */
        if (s + 1 < S)
            for (int64_t i = 0; i < N * d; ++i) r2[i] = qvgo_bf16_to_f32(qvgo_f32_to_bf16(r2[i]));
        float *t = r; r = r2; r2 = t;
    }
    for (int t = 0; t < T; ++t) {
        qvgo_quant_round(N, d, B, bits, scale_fmt, r, q, sc);
        for (int64_t n = 0; n < N; ++n) {
            qvgo_pack(d, bits, q + n * d, codes_out + (n * T + t) * cb);
            memcpy(scales_out + (n * T + t) * G, sc + n * G, (size_t)G * 2);
        }
    }
    if (resid_out) memcpy(resid_out, r, (size_t)N * d * sizeof(float));
    free(r); free(r2); free(q); free(sc); free(start);
}

/* Same as above but the centroids are given and kept (no Lloyd update):
 * assignment, residual, quantization rounds.  S = 1 only. */
void qvgo_encode_given_centroids(int64_t N, int d, int K, int B, int T, int bits, int scale_fmt,
                                 const uint16_t *x, const uint16_t *cent,
                                 qid_t *ids_out, uint8_t *codes_out, uint16_t *scales_out) {
    uint16_t *cdump = (uint16_t *)malloc((size_t)K * d * 2);
    qvgo_encode_unit(N, d, K, B, 1, T, bits, scale_fmt, 0, x, cent, NULL, cdump, ids_out,
                     codes_out, scales_out, NULL);
    free(cdump);
}

/* Same, with the assignment given too: residual and quantization rounds. */
void qvgo_encode_given_ids(int64_t N, int d, int B, int T, int bits, int scale_fmt,
                           const uint16_t *x, const uint16_t *cent, const qid_t *ids,
                           uint8_t *codes_out, uint16_t *scales_out) {
    const int G = d / B, cb = d * bits / 8;
    size_t nd = (size_t)(N > 0 ? N : 1) * d;
    float *r = (float *)malloc(nd * sizeof(float)), *r2 = (float *)malloc(nd * sizeof(float));
    int8_t *q = (int8_t *)malloc(nd);
    uint16_t *sc = (uint16_t *)malloc((size_t)(N > 0 ? N : 1) * G * 2);
    for (int64_t i = 0; i < N * d; ++i) r[i] = qvgo_bf16_to_f32(x[i]);
    qvgo_residual(N, d, r, cent, ids, r2);
    for (int t = 0; t < T; ++t) {
        qvgo_quant_round(N, d, B, bits, scale_fmt, r2, q, sc);
        for (int64_t n = 0; n < N; ++n) {
            qvgo_pack(d, bits, q + n * d, codes_out + (n * T + t) * cb);
            memcpy(scales_out + (n * T + t) * G, sc + n * G, (size_t)G * 2);
        }
    }
    free(r); free(r2); free(q); free(sc);
}

/* ------------------------------------------------------------------ */
/* Sec. 4.2 "dequantization process", Eq. 7                           */
/* ------------------------------------------------------------------ */

/* Replay: start from the assigned centroids (stage order 1..S, fp32 adds),
 * add scale*q of every quantization round (one fma each, round order 1..T),
 * round once to bf16.
 * cent [S][K][d], ids [S][N], codes [N][T][d*b/8], scales [N][T][d/B].
 * out_bf16 [N][d]; out_f32 (nullable) the value before the final rounding. */
void qvgo_decode_unit(int64_t N, int d, int K, int B, int S, int T, int bits, int scale_fmt,
                      const uint16_t *cent, const qid_t *ids, const uint8_t *codes,
                      const uint16_t *scales, uint16_t *out_bf16, float *out_f32) {
    const int G = d / B, cb = d * bits / 8;
    int8_t *q = (int8_t *)malloc((size_t)d);
    float *acc = (float *)malloc((size_t)d * sizeof(float));
    for (int64_t n = 0; n < N; ++n) {
        for (int ch = 0; ch < d; ++ch) {
            float a = 0.0f;
            for (int s = 0; s < S; ++s) {
                float c = qvgo_bf16_to_f32(cent[((int64_t)s * K + ids[(int64_t)s * N + n]) * d + ch]);
                a = (s == 0) ? c : a + c;
            }
            acc[ch] = a;
        }
        for (int t = 0; t < T; ++t) {
            qvgo_unpack(d, bits, codes + (n * T + t) * cb, q);
            for (int ch = 0; ch < d; ++ch) {
                float s = scale_load(scales[(n * T + t) * G + ch / B], scale_fmt);
                acc[ch] = fmaf(s, (float)q[ch], acc[ch]);
            }
        }
        for (int ch = 0; ch < d; ++ch) {
            out_bf16[n * d + ch] = qvgo_f32_to_bf16(acc[ch]);
            if (out_f32) out_f32[n * d + ch] = acc[ch];
        }
    }
    free(q); free(acc);
}

/* ------------------------------------------------------------------ */
/* attention over the decoded cache (the read path the codec serves)  */
/* ------------------------------------------------------------------ */

/* O = softmax(scale * Q K^T) V, no mask, one head, everything in fp64.
 * q [Nq][d], k [Nk][d], v [Nk][d] bf16.  out [Nq][d] fp64,
 * lse (nullable) [Nq] = log sum exp of the scaled scores. */
void qvgo_attention(int64_t Nq, int64_t Nk, int d, const uint16_t *q, const uint16_t *k,
                    const uint16_t *v, double scale, double *out, double *lse) {
    double *p = (double *)malloc((size_t)(Nk > 0 ? Nk : 1) * sizeof(double));
    for (int64_t i = 0; i < Nq; ++i) {
        double mx = -INFINITY;
        for (int64_t j = 0; j < Nk; ++j) {
            double s = 0.0;
            for (int ch = 0; ch < d; ++ch)
                s += (double)qvgo_bf16_to_f32(q[i * d + ch]) * (double)qvgo_bf16_to_f32(k[j * d + ch]);
            p[j] = s * scale;
            if (p[j] > mx) mx = p[j];
        }
        double z = 0.0;
        for (int64_t j = 0; j < Nk; ++j) { p[j] = exp(p[j] - mx); z += p[j]; }
        for (int ch = 0; ch < d; ++ch) {
            double o = 0.0;
            for (int64_t j = 0; j < Nk; ++j) o += p[j] * (double)qvgo_bf16_to_f32(v[j * d + ch]);
            out[i * d + ch] = o / z;
        }
        if (lse) lse[i] = mx + log(z);
    }
    free(p);
}

/* Rotary position embedding applied to decoded keys.  Sec. 5 "Implementation" caches keys
 * BEFORE the rotary embedding (they quantize better), so the attention read has to rotate each
 * decoded key by its position.  The paper does not print the rotation; reading: the usual
 * complex form on interleaved channel pairs (2i, 2i+1), angle given per token and pair by the
 * caller as a (cos, sin) table in binary16:
 *     y[2i]   = x[2i] cos - x[2i+1] sin        y[2i+1] = x[2i] sin + x[2i+1] cos
 * on the bf16 decoded key, each output one fp32 product and one fma, rounded to bf16 (the
 * type the attention contraction reads).
 * k [N][d] bf16, rope [N][d/2][2] binary16 (cos, sin), out [N][d] bf16. */
void qvgo_rope_keys(int64_t N, int d, const uint16_t *k, const uint16_t *rope, uint16_t *out) {
    for (int64_t n = 0; n < N; ++n)
        for (int i = 0; i < d / 2; ++i) {
            float x0 = qvgo_bf16_to_f32(k[n * d + 2 * i]), x1 = qvgo_bf16_to_f32(k[n * d + 2 * i + 1]);
            float c = qvgo_f16_to_f32(rope[(n * (d / 2) + i) * 2]);
            float sn = qvgo_f16_to_f32(rope[(n * (d / 2) + i) * 2 + 1]);
            float t0 = x1 * sn, t1 = x1 * c;
            out[n * d + 2 * i] = qvgo_f32_to_bf16(fmaf(x0, c, -t0));
            out[n * d + 2 * i + 1] = qvgo_f32_to_bf16(fmaf(x0, sn, t1));
        }
}

/* Two attention results over DISJOINT key sets A and B (the compressed cache and the current
 * chunk's own bf16 keys, Sec. 3.1: a chunk attends to the cached chunks and to itself) merged
 * into the attention over their union, from the outputs and the log-sum-exp of the scores:
 *     w_a = exp(lse_a - lse), w_b = exp(lse_b - lse), lse = log(exp(lse_a) + exp(lse_b)),
 *     o = w_a o_a + w_b o_b.
 * rows x d outputs in fp64, lse per row. */
void qvgo_attn_merge(int64_t rows, int d, const double *oa, const double *lsea,
                     const double *ob, const double *lseb, double *out, double *lse) {
    for (int64_t r = 0; r < rows; ++r) {
        double m = lsea[r] > lseb[r] ? lsea[r] : lseb[r];
        double wa = exp(lsea[r] - m), wb = exp(lseb[r] - m), z = wa + wb;
        for (int ch = 0; ch < d; ++ch) out[r * d + ch] = (wa * oa[r * d + ch] + wb * ob[r * d + ch]) / z;
        if (lse) lse[r] = m + log(z);
    }
}

/* ------------------------------------------------------------------ */
/* storage size (Sec. 5: compression ratio, memory breakdown)         */
/* ------------------------------------------------------------------ */

/* Bytes that one chunk of N tokens of one head occupies:
 * codes  T * N * d*b/8
 * scales T * N * (d/B) * scale_bytes
 * ids    S * N * id_bits/8
 * centroid tables S * K * d * 2 (bf16). */
double qvgo_chunk_bytes(int64_t N, int d, int K, int B, int S, int T, int bits,
                        double scale_bytes, double id_bits) {
    double codes = (double)T * (double)N * d * bits / 8.0;
    double scales = (double)T * (double)N * ((double)d / B) * scale_bytes;
    double ids = (double)S * (double)N * id_bits / 8.0;
    double cent = (double)S * K * d * 2.0;
    return codes + scales + ids + cent;
}

/* ------------------------------------------------------------------ */
/* batched drivers: independent (head, K-or-V) units in parallel      */
/* ------------------------------------------------------------------ */

void qvgo_encode_batch(int H, int64_t N, int d, int K, int B, int S, int T, int bits, int scale_fmt, int I,
                       const uint16_t *x, const uint16_t *init,
                       uint16_t *cent_out, qid_t *ids_out,
                       uint8_t *codes_out, uint16_t *scales_out) {
    const int G = d / B, cb = d * bits / 8;
#pragma omp parallel for schedule(dynamic, 1)
    for (int h = 0; h < H; ++h)
        qvgo_encode_unit(N, d, K, B, S, T, bits, scale_fmt, I,
                         x + (int64_t)h * N * d, init + (int64_t)h * S * K * d, NULL,
                         cent_out + (int64_t)h * S * K * d, ids_out + (int64_t)h * S * N,
                         codes_out + (int64_t)h * N * T * cb, scales_out + (int64_t)h * N * T * G, NULL);
}

void qvgo_decode_batch(int H, int64_t N, int d, int K, int B, int S, int T, int bits, int scale_fmt,
                       const uint16_t *cent, const qid_t *ids, const uint8_t *codes,
                       const uint16_t *scales, uint16_t *out_bf16) {
    const int G = d / B, cb = d * bits / 8;
#pragma omp parallel for schedule(dynamic, 1)
    for (int h = 0; h < H; ++h)
        qvgo_decode_unit(N, d, K, B, S, T, bits, scale_fmt,
                         cent + (int64_t)h * S * K * d, ids + (int64_t)h * S * N,
                         codes + (int64_t)h * N * T * cb, scales + (int64_t)h * N * T * G,
                         out_bf16 + (int64_t)h * N * d, NULL);
}

/* heads are independent; queries of one head are split over the threads */
void qvgo_attention_batch(int H, int64_t Nq, int64_t Nk, int d, const uint16_t *q,
                          const uint16_t *k, const uint16_t *v, double scale,
                          double *out, double *lse) {
    int64_t total = (int64_t)H * Nq;
#pragma omp parallel for schedule(dynamic, 4)
    for (int64_t w = 0; w < total; ++w) {
        int64_t h = w / Nq, i = w % Nq;
        qvgo_attention(1, Nk, d, q + (h * Nq + i) * d, k + h * Nk * d, v + h * Nk * d, scale,
                       out + (h * Nq + i) * d, lse ? lse + h * Nq + i : NULL);
    }
}

int qvgo_max_threads(void) {
#ifdef _OPENMP
    extern int omp_get_max_threads(void);
    return omp_get_max_threads();
#else
    return 1;
#endif
}
