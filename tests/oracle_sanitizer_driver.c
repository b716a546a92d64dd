/* Runs every exported function of the CPU oracle on small ragged shapes with heap buffers of
 * exactly the documented sizes, so that a build with -fsanitize=address,undefined reports any
 * access outside them.  TEST INFRASTRUCTURE: compiled and run by tests/test_oracle_sanitized.py.
 * Also checks a few identities on the way (decode of an encode is finite; pack/unpack round trip),
 * and prints "ok" when every case ran. */
#include "../oracle/qvg_oracle.c"

#include <stdio.h>

static uint32_t rng_state = 12345u;
static uint32_t rng(void) { rng_state = rng_state * 1664525u + 1013904223u; return rng_state >> 8; }
/* a bf16 value in about [-4, 4) */
static uint16_t rand_bf16(void) { return qvgo_f32_to_bf16(((float)(rng() & 0xffff) / 8192.0f) - 4.0f); }

#define NEW(type, n) ((type *)malloc((size_t)((n) > 0 ? (n) : 1) * sizeof(type)))

static int run_case(int64_t N, int d, int K, int B, int S, int T, int bits, int fmt, int I) {
    const int G = d / B, cb = d * bits / 8;
    uint16_t *x = NEW(uint16_t, N * d);
    for (int64_t i = 0; i < N * d; ++i) x[i] = rand_bf16();
    int32_t *idx = NEW(int32_t, K);
    for (int j = 0; j < K; ++j) idx[j] = (int32_t)(N > 0 ? (j * 7) % N : 0);
    uint16_t *cent = NEW(uint16_t, (int64_t)S * K * d);
    qid_t *ids = NEW(qid_t, (int64_t)S * N);
    uint8_t *codes = NEW(uint8_t, N * T * cb);
    uint16_t *scales = NEW(uint16_t, N * T * G);
    float *resid = NEW(float, N * d);
    /* start centroids drawn from tokens, then from a given table */
    qvgo_encode_unit(N, d, K, B, S, T, bits, fmt, I, x, NULL, idx, cent, ids, codes, scales, resid);
    uint16_t *init = NEW(uint16_t, (int64_t)S * K * d);
    memcpy(init, cent, (size_t)S * K * d * 2);
    qvgo_encode_unit(N, d, K, B, S, T, bits, fmt, I, x, init, NULL, cent, ids, codes, scales, NULL);
    uint16_t *out = NEW(uint16_t, N * d);
    float *outf = NEW(float, N * d);
    qvgo_decode_unit(N, d, K, B, S, T, bits, fmt, cent, ids, codes, scales, out, outf);
    qvgo_decode_unit(N, d, K, B, S, T, bits, fmt, cent, ids, codes, scales, out, NULL);
    int bad = 0;
    for (int64_t i = 0; i < N * d; ++i) if (!isfinite(outf[i])) bad = 1;
    if (S == 1) {
        qid_t *ids2 = NEW(qid_t, N);
        qvgo_encode_given_centroids(N, d, K, B, T, bits, fmt, x, cent, ids2, codes, scales);
        qvgo_encode_given_ids(N, d, B, T, bits, fmt, x, cent, ids2, codes, scales);
        float *r = NEW(float, N * d);
        for (int64_t i = 0; i < N * d; ++i) r[i] = qvgo_bf16_to_f32(x[i]);
        double *dist = NEW(double, N), *best = NEW(double, N);
        qvgo_assign(N, d, K, r, cent, ids2, best);
        qvgo_assign(N, d, K, r, cent, ids2, NULL);
        qvgo_dist_to(N, d, r, cent, ids2, dist);
        for (int64_t n = 0; n < N; ++n) if (dist[n] != best[n]) bad = 1;
        uint16_t *cn = NEW(uint16_t, (int64_t)K * d);
        int32_t *cnt = NEW(int32_t, K);
        qvgo_update(N, d, K, r, ids2, cent, cn, cnt);
        int64_t tot = 0;
        for (int j = 0; j < K; ++j) tot += cnt[j];
        if (tot != N) bad = 1;
        double *inertia = NEW(double, I + 1);                   /* one entry per assign pass */
        qvgo_lloyd(N, d, K, I, r, cent, cn, ids2, inertia);
        for (int it = 1; it <= I; ++it) if (inertia[it] > inertia[it - 1] * (1.0 + 1e-6) + 1e-9) bad = 1;
        free(inertia);
        float *r2 = NEW(float, N * d);
        qvgo_residual(N, d, r, cn, ids2, r2);
        int8_t *q = NEW(int8_t, N * d), *q2 = NEW(int8_t, N * d);
        uint16_t *sc = NEW(uint16_t, N * G);
        qvgo_quant_round(N, d, B, bits, fmt, r2, q, sc);
        uint8_t *pk = NEW(uint8_t, N * cb);
        qvgo_pack(N * d, bits, q, pk);
        qvgo_unpack(N * d, bits, pk, q2);
        if (memcmp(q, q2, (size_t)(N * d)) != 0) bad = 1;
        free(ids2); free(r); free(dist); free(best); free(cn); free(cnt); free(r2); free(q); free(q2); free(sc); free(pk);
    }
    free(x); free(idx); free(cent); free(ids); free(codes); free(scales); free(resid); free(init); free(out); free(outf);
    return bad;
}

static int run_batch(int H, int64_t N, int d, int K, int B, int S, int T, int bits, int fmt, int I) {
    const int G = d / B, cb = d * bits / 8;
    uint16_t *x = NEW(uint16_t, (int64_t)H * N * d), *init = NEW(uint16_t, (int64_t)H * S * K * d);
    for (int64_t i = 0; i < (int64_t)H * N * d; ++i) x[i] = rand_bf16();
    for (int64_t i = 0; i < (int64_t)H * S * K * d; ++i) init[i] = rand_bf16();
    uint16_t *cent = NEW(uint16_t, (int64_t)H * S * K * d);
    qid_t *ids = NEW(qid_t, (int64_t)H * S * N);
    uint8_t *codes = NEW(uint8_t, (int64_t)H * N * T * cb);
    uint16_t *scales = NEW(uint16_t, (int64_t)H * N * T * G);
    uint16_t *out = NEW(uint16_t, (int64_t)H * N * d);
    qvgo_encode_batch(H, N, d, K, B, S, T, bits, fmt, I, x, init, cent, ids, codes, scales);
    qvgo_decode_batch(H, N, d, K, B, S, T, bits, fmt, cent, ids, codes, scales, out);
    /* attention of 3 queries per head over the decoded cache, rotary keys, merge of two halves */
    const int64_t Nq = 3;
    uint16_t *q = NEW(uint16_t, (int64_t)H * Nq * d);
    for (int64_t i = 0; i < (int64_t)H * Nq * d; ++i) q[i] = rand_bf16();
    double *o = NEW(double, (int64_t)H * Nq * d), *lse = NEW(double, (int64_t)H * Nq);
    qvgo_attention_batch(H, Nq, N, d, q, out, out, 0.0883883, o, lse);
    int bad = 0;
    if (N >= 2) {
        const int64_t Na = N / 2, Nb = N - Na;
        double *oa = NEW(double, Nq * d), *la = NEW(double, Nq), *ob = NEW(double, Nq * d), *lb = NEW(double, Nq);
        double *om = NEW(double, Nq * d), *lm = NEW(double, Nq);
        qvgo_attention(Nq, Na, d, q, out, out, 0.0883883, oa, la);
        qvgo_attention(Nq, Nb, d, q, out + Na * d, out + Na * d, 0.0883883, ob, lb);
        qvgo_attn_merge(Nq, d, oa, la, ob, lb, om, lm);
        qvgo_attn_merge(Nq, d, oa, la, ob, lb, om, NULL);
        for (int64_t i = 0; i < Nq * d; ++i) if (fabs(om[i] - o[i]) > 1e-9 * (1.0 + fabs(o[i]))) bad = 1;
        for (int64_t i = 0; i < Nq; ++i) if (fabs(lm[i] - lse[i]) > 1e-9 * (1.0 + fabs(lse[i]))) bad = 1;
        free(oa); free(la); free(ob); free(lb); free(om); free(lm);
    }
    uint16_t *rope = NEW(uint16_t, N * (d / 2) * 2), *rk = NEW(uint16_t, N * d);
    for (int64_t i = 0; i < N * (d / 2); ++i) {
        double a = 0.01 * (double)(rng() & 1023);
        rope[2 * i] = qvgo_f32_to_f16((float)cos(a));
        rope[2 * i + 1] = qvgo_f32_to_f16((float)sin(a));
    }
    qvgo_rope_keys(N, d, out, rope, rk);
    free(x); free(init); free(cent); free(ids); free(codes); free(scales); free(out); free(q); free(o); free(lse); free(rope); free(rk);
    return bad;
}

int main(void) {
    int bad = 0;
    /* the formats of the conversions, every code once */
    for (int c = 0; c < 256; ++c) (void)qvgo_f32_to_e4m3(qvgo_e4m3_to_f32((uint8_t)c));
    for (int h = 0; h < 65536; h += 7) (void)qvgo_f32_to_f16(qvgo_f16_to_f32((uint16_t)h));
    /*               N    d   K   B  S  T bits fmt I */
    bad |= run_case(37, 128,   5, 64, 1, 2, 2, 0, 2);
    bad |= run_case(37, 128,   7, 16, 2, 1, 4, 1, 1);
    bad |= run_case(41, 128, 300, 32, 1, 3, 2, 0, 0);       /* more centroids than tokens, 16-bit ids */
    bad |= run_case(1,  128,   1, 128, 1, 1, 2, 1, 3);
    bad |= run_case(0,  128,   4, 64, 1, 2, 2, 0, 0);       /* empty chunk */
    bad |= run_case(19, 64,    6, 32, 4, 1, 2, 1, 1);
    bad |= run_batch(3, 23, 128, 5, 64, 1, 2, 2, 0, 1);
    bad |= run_batch(2, 17, 128, 9, 16, 2, 1, 4, 1, 0);
    (void)qvgo_chunk_bytes(4680, 128, 256, 64, 1, 1, 2, 1.0, 8.0);
    (void)qvgo_max_threads();
    if (bad) { printf("identity check failed\n"); return 1; }
    printf("ok\n");
    return 0;
}
