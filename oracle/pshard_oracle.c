/*
 * CPU oracle for the pipelined-sharding hot path: TEST INFRASTRUCTURE ONLY.
 *
 * The method is lossless (paper, Introduction and Section 3: sharding and
 * placement change where weights live and when they are copied, never the
 * operations executed), so the oracle is the plain un-sharded definition of
 * the decoder sub-layers in fp64.  It has no notion of shards, budgets,
 * streams, tiles or physical weight layouts, and shares no code with the HIP
 * library.  Only tests, the smoke check and the benchmark's cpu_baseline leg
 * may call it.
 *
 * Weight format (benchmark definition, config 1): blocks of 32 weights along
 * K, one fp16 scale d per block, 4-bit codes q in 0..15, w = d * (q - 8).
 * Logical arrays: scales fp16 bits [N][K/32], codes one per byte [N][K].
 *
 * "mirror" mode rounds to fp16 at the points where the GPU path stores fp16
 * tensors (projection outputs, SwiGLU output, residual sums).  Pure mode
 * (mirror = 0) never rounds.
 *
 * Parity pins: every function below is pinned by tests/test_oracle_pins.py
 * (brute force in pure Python, closed forms, textbook special cases).
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

/* ---- fp16 <-> fp64, written from the IEEE 754 binary16 definition -------- */

double orc_half_to_double(uint16_t h) {
    int sign = (h >> 15) & 1;
    int e = (h >> 10) & 0x1F;
    int m = h & 0x3FF;
    double v;
    if (e == 0)
        v = ldexp((double)m, -24);            /* subnormal: m * 2^-24 */
    else if (e == 31)
        v = m ? NAN : INFINITY;
    else
        v = ldexp((double)(m + 1024), e - 25); /* (1 + m/1024) * 2^(e-15) */
    return sign ? -v : v;
}

/* round-to-nearest-even of a double to the binary16 grid, returned as a double */
double orc_round_f16(double x) {
    if (x == 0.0 || isnan(x) || isinf(x)) return x;
    double a = fabs(x);
    int ex;
    frexp(a, &ex);                 /* a = f * 2^ex, f in [0.5, 1) */
    int e = ex - 1;                /* a in [2^e, 2^(e+1)) */
    if (e < -14) e = -14;          /* subnormal range shares the 2^-24 grid */
    double ulp = ldexp(1.0, e - 10);
    double r = nearbyint(a / ulp) * ulp; /* default rounding mode: ties to even */
    if (r >= 65520.0) r = INFINITY;      /* beyond the largest finite half after rounding */
    return x < 0 ? -r : r;
}

/* ---- dequantise: W[n][k] = d[n][k/32] * (q[n][k] - 8) --------------------- */

void orc_dequant(const uint16_t *scales, const uint8_t *codes, int64_t N, int64_t K, double *W) {
    int64_t nb = K / 32;
    for (int64_t n = 0; n < N; ++n)
        for (int64_t k = 0; k < K; ++k)
            W[n * K + k] = orc_half_to_double(scales[n * nb + k / 32]) * ((double)codes[n * K + k] - 8.0);
}

/* ---- linear: Y[m][n] = sum_k X[m][k] * W[n][k], k ascending, fp64 --------- */

void orc_linear(const double *X, int64_t M, const uint16_t *scales, const uint8_t *codes,
                int64_t N, int64_t K, double *Y) {
    int64_t nb = K / 32;
#pragma omp parallel for schedule(static)
    for (int64_t n = 0; n < N; ++n) {
        double *w = (double *)malloc(sizeof(double) * (size_t)K);
        for (int64_t k = 0; k < K; ++k)
            w[k] = orc_half_to_double(scales[n * nb + k / 32]) * ((double)codes[n * K + k] - 8.0);
        for (int64_t m = 0; m < M; ++m) {
            double acc = 0.0;
            for (int64_t k = 0; k < K; ++k) acc += X[m * K + k] * w[k];
            Y[m * N + n] = acc;
        }
        free(w);
    }
}

/* ---- RMSNorm with unit gain: y = x / sqrt(mean(x^2) + eps) ---------------- */

void orc_rmsnorm(const double *x, int64_t M, int64_t H, double eps, double *y) {
    for (int64_t m = 0; m < M; ++m) {
        double ss = 0.0;
        for (int64_t i = 0; i < H; ++i) ss += x[m * H + i] * x[m * H + i];
        double r = 1.0 / sqrt(ss / (double)H + eps);
        for (int64_t i = 0; i < H; ++i) y[m * H + i] = x[m * H + i] * r;
    }
}

/* ---- SwiGLU: s = silu(g) * u, silu(g) = g / (1 + exp(-g)) ----------------- */

void orc_swiglu(const double *g, const double *u, int64_t n, double *s) {
    for (int64_t i = 0; i < n; ++i) s[i] = g[i] / (1.0 + exp(-g[i])) * u[i];
}

/* ---- attention stand-in: identity on V with grouped-query broadcast --------
 * qkv row = [Q: n_q*hd | K: n_kv*hd | V: n_kv*hd]; output head h copies V head
 * floor(h / (n_q / n_kv)).  Equals softmax attention with a single key. */

void orc_attn_identity_v(const double *qkv, int64_t M, int n_q, int n_kv, int hd, double *A) {
    int64_t qkv_w = (int64_t)(n_q + 2 * n_kv) * hd;
    int64_t v0 = (int64_t)(n_q + n_kv) * hd;
    int group = n_q / n_kv;
    for (int64_t m = 0; m < M; ++m)
        for (int h = 0; h < n_q; ++h)
            for (int j = 0; j < hd; ++j)
                A[m * (int64_t)n_q * hd + (int64_t)h * hd + j] = qkv[m * qkv_w + v0 + (int64_t)(h / group) * hd + j];
}

/* ---- MoE routing: the top_k largest fp32 logits per token, ties to the lower
 * index, listed in descending-logit order; weights are the softmax over the
 * selected logits (equal to the full softmax renormalised over the selection). */

void orc_route_topk(const float *logits, int64_t M, int E, int top_k, int32_t *idx, double *w) {
    for (int64_t m = 0; m < M; ++m) {
        const float *l = logits + m * E;
        char *taken = (char *)calloc((size_t)E, 1);
        for (int j = 0; j < top_k; ++j) {
            int best = -1;
            for (int e = 0; e < E; ++e)
                if (!taken[e] && (best < 0 || l[e] > l[best])) best = e;
            taken[best] = 1;
            idx[m * top_k + j] = best;
        }
        free(taken);
        double lmax = (double)l[idx[m * top_k]];
        double den = 0.0;
        for (int j = 0; j < top_k; ++j) den += exp((double)l[idx[m * top_k + j]] - lmax);
        for (int j = 0; j < top_k; ++j) w[m * top_k + j] = exp((double)l[idx[m * top_k + j]] - lmax) / den;
    }
}

static void round_all(double *v, int64_t n, int mirror) {
    if (!mirror) return;
    for (int64_t i = 0; i < n; ++i) v[i] = orc_round_f16(v[i]);
}

/* ---- attention half of a decoder layer (pre-norm, residual) ----------------
 * h = x + Linear_O(IdentityV(Linear_QKV(RMSNorm(x)))) */

void orc_attn_half(const double *x, int64_t M, int H, int n_q, int n_kv, int hd, double eps,
                   const uint16_t *qkv_s, const uint8_t *qkv_c,
                   const uint16_t *o_s, const uint8_t *o_c, int mirror, double *h) {
    int64_t qkv_w = (int64_t)(n_q + 2 * n_kv) * hd, a_w = (int64_t)n_q * hd;
    double *n = (double *)malloc(sizeof(double) * (size_t)(M * H));
    double *qkv = (double *)malloc(sizeof(double) * (size_t)(M * qkv_w));
    double *A = (double *)malloc(sizeof(double) * (size_t)(M * a_w));
    orc_rmsnorm(x, M, H, eps, n);
    orc_linear(n, M, qkv_s, qkv_c, qkv_w, H, qkv);
    round_all(qkv, M * qkv_w, mirror);
    orc_attn_identity_v(qkv, M, n_q, n_kv, hd, A);
    orc_linear(A, M, o_s, o_c, H, a_w, h);
    for (int64_t i = 0; i < M * H; ++i) h[i] += x[i];
    round_all(h, M * H, mirror);
    free(n); free(qkv); free(A);
}

/* ---- decode attention over a KV cache (one new token) -----------------------
 * q [n_q][hd]; K, V [n_kv][T][hd] hold T positions (the cache plus the new token's own row, last).
 * Head h attends with kv head floor(h / (n_q / n_kv)): scores s_j = (q_h . K_j) / sqrt(hd),
 * p = softmax(s) over the T positions, A_h = sum_j p_j V_j.  Plain definition, fp64, the usual
 * max subtraction so exp cannot overflow.  No positional encoding is applied. */

void orc_attn_decode(const double *q, const double *K, const double *V, int64_t T,
                     int n_q, int n_kv, int hd, double *A) {
    int group = n_q / n_kv;
    double *s = (double *)malloc(sizeof(double) * (size_t)T);
    for (int h = 0; h < n_q; ++h) {
        const double *Kg = K + (int64_t)(h / group) * T * hd, *Vg = V + (int64_t)(h / group) * T * hd;
        double mx = -INFINITY, den = 0.0;
        for (int64_t j = 0; j < T; ++j) {
            double d = 0.0;
            for (int e = 0; e < hd; ++e) d += q[(int64_t)h * hd + e] * Kg[j * hd + e];
            s[j] = d / sqrt((double)hd);
            if (s[j] > mx) mx = s[j];
        }
        for (int64_t j = 0; j < T; ++j) { s[j] = exp(s[j] - mx); den += s[j]; }
        for (int e = 0; e < hd; ++e) {
            double o = 0.0;
            for (int64_t j = 0; j < T; ++j) o += s[j] / den * Vg[j * hd + e];
            A[(int64_t)h * hd + e] = o;
        }
    }
    free(s);
}

/* attention half of a decoder layer at one new token with a KV cache of C earlier positions:
 * qkv = Linear_QKV(RMSNorm(x)); the token's own K and V rows (as stored: fp16 when mirror) join the
 * cache as position C; h = x + Linear_O(Attention(q, K[0..C], V[0..C])).
 * Kc, Vc: fp16 bit patterns [n_kv][cap][hd], cap > C; row C of every head is written. */

void orc_attn_kv_half(const double *x, int H, int n_q, int n_kv, int hd, double eps,
                      const uint16_t *qkv_s, const uint8_t *qkv_c,
                      const uint16_t *o_s, const uint8_t *o_c,
                      uint16_t *Kc, uint16_t *Vc, int64_t cap, int64_t C, int mirror,
                      double *k_new, double *v_new, double *h) {
    int64_t qkv_w = (int64_t)(n_q + 2 * n_kv) * hd, a_w = (int64_t)n_q * hd, T = C + 1;
    double *n = (double *)malloc(sizeof(double) * (size_t)H);
    double *qkv = (double *)malloc(sizeof(double) * (size_t)qkv_w);
    double *A = (double *)malloc(sizeof(double) * (size_t)a_w);
    double *K = (double *)malloc(sizeof(double) * (size_t)(n_kv * T * hd));
    double *V = (double *)malloc(sizeof(double) * (size_t)(n_kv * T * hd));
    orc_rmsnorm(x, 1, H, eps, n);
    orc_linear(n, 1, qkv_s, qkv_c, qkv_w, H, qkv);
    round_all(qkv, qkv_w, mirror);
    for (int g = 0; g < n_kv; ++g) {
        for (int64_t j = 0; j < C; ++j)
            for (int e = 0; e < hd; ++e) {
                K[((int64_t)g * T + j) * hd + e] = orc_half_to_double(Kc[((int64_t)g * cap + j) * hd + e]);
                V[((int64_t)g * T + j) * hd + e] = orc_half_to_double(Vc[((int64_t)g * cap + j) * hd + e]);
            }
        for (int e = 0; e < hd; ++e) {
            double kn = qkv[(int64_t)(n_q + g) * hd + e], vn = qkv[(int64_t)(n_q + n_kv + g) * hd + e];
            K[((int64_t)g * T + C) * hd + e] = kn;
            V[((int64_t)g * T + C) * hd + e] = vn;
            k_new[(int64_t)g * hd + e] = kn;
            v_new[(int64_t)g * hd + e] = vn;
        }
    }
    orc_attn_decode(qkv, K, V, T, n_q, n_kv, hd, A);
    round_all(A, a_w, mirror);
    orc_linear(A, 1, o_s, o_c, H, a_w, h);
    for (int64_t i = 0; i < H; ++i) h[i] += x[i];
    round_all(h, H, mirror);
    free(n); free(qkv); free(A); free(K); free(V);
}

/* attention half for a CHUNK of M new tokens with a KV cache of C earlier positions (chunked
 * prefill over the cache; Section 3 lists the KV cache as a shard class and the tier size as the
 * chunk size).  Causal softmax attention, written out from its definition: token m of the chunk
 * sits at position C + m and attends over positions 0 .. C + m, i.e. the C cached rows and the
 * chunk's own tokens 0 .. m; the chunk tokens' K and V rows are their QKV projections (as stored:
 * fp16 when mirror) and join the cache as positions C .. C + M - 1.
 * x [M][H]; Kc, Vc fp16 bits [n_kv][cap][hd], cap >= C + M (rows from C on are not read);
 * k_new, v_new [M][n_kv][hd] receive the chunk's rows; h [M][H] = x + Linear_O(Attention). */

void orc_attn_kv_chunk_half(const double *x, int64_t M, int H, int n_q, int n_kv, int hd, double eps,
                            const uint16_t *qkv_s, const uint8_t *qkv_c,
                            const uint16_t *o_s, const uint8_t *o_c,
                            const uint16_t *Kc, const uint16_t *Vc, int64_t cap, int64_t C, int mirror,
                            double *k_new, double *v_new, double *h) {
    int64_t qkv_w = (int64_t)(n_q + 2 * n_kv) * hd, a_w = (int64_t)n_q * hd;
    double *n = (double *)malloc(sizeof(double) * (size_t)(M * H));
    double *qkv = (double *)malloc(sizeof(double) * (size_t)(M * qkv_w));
    double *A = (double *)malloc(sizeof(double) * (size_t)(M * a_w));
    orc_rmsnorm(x, M, H, eps, n);
    orc_linear(n, M, qkv_s, qkv_c, qkv_w, H, qkv);
    round_all(qkv, M * qkv_w, mirror);
    for (int64_t m = 0; m < M; ++m)
        for (int g = 0; g < n_kv; ++g)
            for (int e = 0; e < hd; ++e) {
                k_new[(m * n_kv + g) * hd + e] = qkv[m * qkv_w + (int64_t)(n_q + g) * hd + e];
                v_new[(m * n_kv + g) * hd + e] = qkv[m * qkv_w + (int64_t)(n_q + n_kv + g) * hd + e];
            }
    for (int64_t m = 0; m < M; ++m) {
        int64_t T = C + m + 1;          /* positions token m sees */
        double *K = (double *)malloc(sizeof(double) * (size_t)(n_kv * T * hd));
        double *V = (double *)malloc(sizeof(double) * (size_t)(n_kv * T * hd));
        for (int g = 0; g < n_kv; ++g)
            for (int64_t j = 0; j < T; ++j)
                for (int e = 0; e < hd; ++e) {
                    double kv, vv;
                    if (j < C) {
                        kv = orc_half_to_double(Kc[((int64_t)g * cap + j) * hd + e]);
                        vv = orc_half_to_double(Vc[((int64_t)g * cap + j) * hd + e]);
                    } else {
                        kv = k_new[((j - C) * n_kv + g) * hd + e];
                        vv = v_new[((j - C) * n_kv + g) * hd + e];
                    }
                    K[((int64_t)g * T + j) * hd + e] = kv;
                    V[((int64_t)g * T + j) * hd + e] = vv;
                }
        orc_attn_decode(qkv + m * qkv_w, K, V, T, n_q, n_kv, hd, A + m * a_w);
        free(K); free(V);
    }
    round_all(A, M * a_w, mirror);
    orc_linear(A, M, o_s, o_c, H, a_w, h);
    for (int64_t i = 0; i < M * H; ++i) h[i] += x[i];
    round_all(h, M * H, mirror);
    free(n); free(qkv); free(A);
}

/* ---- one gated FFN on already-normalised input n [M][H] --------------------
 * y = Linear_down(SwiGLU(Linear_gate(n), Linear_up(n))), y [M][H] not rounded */

void orc_ffn(const double *n, int64_t M, int H, int I,
             const uint16_t *g_s, const uint8_t *g_c, const uint16_t *u_s, const uint8_t *u_c,
             const uint16_t *d_s, const uint8_t *d_c, int mirror, double *y) {
    double *g = (double *)malloc(sizeof(double) * (size_t)(M * I));
    double *u = (double *)malloc(sizeof(double) * (size_t)(M * I));
    orc_linear(n, M, g_s, g_c, I, H, g);
    orc_linear(n, M, u_s, u_c, I, H, u);
    orc_swiglu(g, u, M * I, g);
    round_all(g, M * I, mirror);
    orc_linear(g, M, d_s, d_c, H, I, y);
    free(g); free(u);
}

/* ---- dense FFN half: out = h + FFN(RMSNorm(h)); residual optional ---------- */

void orc_dense_ffn_half(const double *h, int64_t M, int H, int I, double eps,
                        const uint16_t *g_s, const uint8_t *g_c, const uint16_t *u_s, const uint8_t *u_c,
                        const uint16_t *d_s, const uint8_t *d_c, int residual, int mirror, double *out) {
    double *n = (double *)malloc(sizeof(double) * (size_t)(M * H));
    orc_rmsnorm(h, M, H, eps, n);
    orc_ffn(n, M, H, I, g_s, g_c, u_s, u_c, d_s, d_c, mirror, out);
    if (residual)
        for (int64_t i = 0; i < M * H; ++i) out[i] += h[i];
    round_all(out, M * H, mirror);
    free(n);
}

/* ---- MoE FFN half: out = h + sum_j w_j * FFN_{e_j}(RMSNorm(h)), experts
 * combined in descending-logit order.  Expert weights arrive as arrays of
 * pointers indexed by expert id; only selected experts are dereferenced. */

void orc_moe_ffn_half(const double *h, int64_t M, int H, int I, int E, int top_k, double eps,
                      const float *logits,
                      const uint16_t *const *g_s, const uint8_t *const *g_c,
                      const uint16_t *const *u_s, const uint8_t *const *u_c,
                      const uint16_t *const *d_s, const uint8_t *const *d_c,
                      int mirror, double *out) {
    double *n = (double *)malloc(sizeof(double) * (size_t)(M * H));
    double *y = (double *)malloc(sizeof(double) * (size_t)H);
    int32_t *idx = (int32_t *)malloc(sizeof(int32_t) * (size_t)(M * top_k));
    double *w = (double *)malloc(sizeof(double) * (size_t)(M * top_k));
    orc_rmsnorm(h, M, H, eps, n);
    orc_route_topk(logits, M, E, top_k, idx, w);
    for (int64_t m = 0; m < M; ++m) {
        double *o = out + m * H;
        for (int i = 0; i < H; ++i) o[i] = 0.0;
        for (int j = 0; j < top_k; ++j) {
            int e = idx[m * top_k + j];
            orc_ffn(n + m * H, 1, H, I, g_s[e], g_c[e], u_s[e], u_c[e], d_s[e], d_c[e], mirror, y);
            for (int i = 0; i < H; ++i) o[i] += w[m * top_k + j] * y[i];
        }
        for (int i = 0; i < H; ++i) o[i] += h[m * H + i];
    }
    round_all(out, M * H, mirror);
    free(n); free(y); free(idx); free(w);
}
