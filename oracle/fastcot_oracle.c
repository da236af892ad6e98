/* CPU oracle for the FastCoT Jacobi decoding step.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, plain definition the GPU library is
 * checked against.  It shares no code with the GPU path; only tests, the smoke check and
 * the benchmark's cpu_baseline leg may call it.
 *
 * What it computes, and from where in the paper:
 *   - greedy autoregressive decoding, Eq. (1) of Sec. 3.1: oracle_greedy_ar
 *   - one Jacobi/FastCoT forward, Eq. (2) and Eq. (4): oracle_forward over a window of rows,
 *     each row attending the committed prefix plus the window slots before it
 *   - verification, Eq. (5) of Sec. 4.3: oracle_verify (match one by one, stop at first miss)
 *   - cache update and advance of the index I (Sec. 4.3, "Cache Update"), stop conditions
 *     (Sec. 4.4): oracle_jacobi_generate
 * The model is the Llama-style causal decoder the benchmark configurations fix (RMSNorm,
 * rotary embedding pairing element i with i + Dh/2, grouped-query attention, SwiGLU MLP,
 * untied LM head, no biases); the paper itself only names the model family (Sec. 5.1).
 *
 * Arithmetic: every floating-point value is `real` (double unless ORACLE_REAL is defined
 * otherwise at compile time).  Every row's arithmetic is independent of how many rows are
 * evaluated together and of the thread count: a dot product is always accumulated in
 * ascending index order by one thread.  Threads only split output columns / heads.
 *
 * Readings where the paper is silent or ambiguous are listed in the repository's design
 * notes; the ones that matter here: the window has W rows, row 0 carries the newest exact
 * token (the paper's window size c counts only the W-1 extra rows); a step accepts K+1
 * tokens where K is the length of the matching prefix; ties in argmax go to the lowest id.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#ifndef ORACLE_REAL
#define ORACLE_REAL double
#endif
typedef ORACLE_REAL real;

typedef struct {
    int32_t n_layers, d_model, n_heads, n_kv_heads, head_dim, d_ffn, vocab;
    float rms_eps, rope_base;
    int32_t wdtype; /* 0: weights are float arrays, 1: bf16 bit patterns in uint16 arrays */
} oracle_shape;

enum { T_EMB = 0, T_WLM, T_GF, T_WQ, T_WK, T_WV, T_WO, T_WG, T_WU, T_WD, T_G1, T_G2, T_COUNT };

typedef struct {
    oracle_shape s;
    const void* emb;   /* [vocab][d] */
    const void* wlm;   /* [d][vocab] */
    const float* gf;   /* [d] final norm gain, NULL = ones */
    const void** w[T_COUNT]; /* per-layer pointers for T_WQ..T_G2 (gains are float, NULL = ones) */
} oracle_model;

typedef struct {
    const oracle_model* m;
    int32_t max_seq;
    int32_t n;  /* committed length: positions [0,n) hold final K/V */
    real* kc;   /* [L][max_seq][Hkv*Dh], K stored after rotation */
    real* vc;   /* [L][max_seq][Hkv*Dh] */
} oracle_session;

int oracle_real_bytes(void) { return (int)sizeof(real); }

/* ---------------------------------------------------------------- model / session handles */
oracle_model* oracle_model_new(const oracle_shape* s) {
    oracle_model* m = (oracle_model*)calloc(1, sizeof(oracle_model));
    m->s = *s;
    for (int t = T_WQ; t < T_COUNT; ++t) m->w[t] = (const void**)calloc((size_t)s->n_layers, sizeof(void*));
    return m;
}
void oracle_model_free(oracle_model* m) {
    if (!m) return;
    for (int t = T_WQ; t < T_COUNT; ++t) free((void*)m->w[t]);
    free(m);
}
/* the caller keeps the arrays alive; layouts: linear weights row-major [in][out] */
int oracle_model_set(oracle_model* m, int tensor, int layer, const void* ptr) {
    if (tensor == T_EMB) m->emb = ptr;
    else if (tensor == T_WLM) m->wlm = ptr;
    else if (tensor == T_GF) m->gf = (const float*)ptr;
    else if (tensor >= T_WQ && tensor < T_COUNT && layer >= 0 && layer < m->s.n_layers) m->w[tensor][layer] = ptr;
    else return -1;
    return 0;
}

oracle_session* oracle_session_new(const oracle_model* m, int32_t max_seq) {
    oracle_session* ss = (oracle_session*)calloc(1, sizeof(oracle_session));
    size_t per = (size_t)m->s.n_layers * (size_t)max_seq * (size_t)(m->s.n_kv_heads * m->s.head_dim);
    ss->m = m; ss->max_seq = max_seq; ss->n = 0;
    ss->kc = (real*)calloc(per, sizeof(real));
    ss->vc = (real*)calloc(per, sizeof(real));
    if (!ss->kc || !ss->vc) { free(ss->kc); free(ss->vc); free(ss); return NULL; }
    return ss;
}
void oracle_session_free(oracle_session* ss) { if (ss) { free(ss->kc); free(ss->vc); free(ss); } }
int32_t oracle_session_len(const oracle_session* ss) { return ss->n; }
int oracle_session_set_len(oracle_session* ss, int32_t n) {
    if (n < 0 || n > ss->max_seq) return -1;
    ss->n = n; return 0;
}

/* ---------------------------------------------------------------- scalar building blocks */
static inline real wval(const void* w, int wdtype, size_t i) {
    if (wdtype == 0) return (real)((const float*)w)[i];
    uint32_t u = (uint32_t)((const uint16_t*)w)[i] << 16; /* bf16 -> fp32 is exact */
    float f; memcpy(&f, &u, 4);
    return (real)f;
}

/* out[i] = x[i] / sqrt(mean(x^2) + eps) * g[i]        (g == NULL means gain 1) */
void oracle_rmsnorm(const real* x, const float* g, int d, double eps, real* out) {
    real ss = 0;
    for (int i = 0; i < d; ++i) ss += x[i] * x[i];
    real r = (real)1 / (real)sqrt((double)(ss / (real)d) + eps);
    for (int i = 0; i < d; ++i) out[i] = x[i] * r * (g ? (real)g[i] : (real)1);
}

/* rotary embedding of one head vector at absolute position pos: element i (i < Dh/2) is
 * paired with element i + Dh/2 and the pair is rotated by pos * base^(-2i/Dh). */
void oracle_rope(real* v, int Dh, int pos, double base) {
    int half = Dh / 2;
    for (int i = 0; i < half; ++i) {
        double ang = (double)pos * pow(base, -2.0 * (double)i / (double)Dh);
        real c = (real)cos(ang), s = (real)sin(ang);
        real a = v[i], b = v[i + half];
        v[i] = a * c - b * s;
        v[i + half] = b * c + a * s;
    }
}

real oracle_silu(real z) { return z / ((real)1 + (real)exp(-(double)z)); }

/* Y[r][n] = sum_k X[r][k] * W[k][n], k ascending, for R rows.  Threads split columns. */
static void matmul_rows(const void* W, int wdtype, int K, int N, const real* X, int R, real* Y) {
    const int NB = 256;
    int nblocks = (N + NB - 1) / NB;
#pragma omp parallel for schedule(dynamic, 1)
    for (int b = 0; b < nblocks; ++b) {
        int n0 = b * NB, n1 = n0 + NB < N ? n0 + NB : N;
        for (int r = 0; r < R; ++r)
            for (int n = n0; n < n1; ++n) Y[(size_t)r * N + n] = 0;
        for (int k = 0; k < K; ++k) {
            if (wdtype == 0) {
                const float* wr = (const float*)W + (size_t)k * N;
                for (int r = 0; r < R; ++r) {
                    real xv = X[(size_t)r * K + k];
                    real* y = Y + (size_t)r * N;
                    for (int n = n0; n < n1; ++n) y[n] += xv * (real)wr[n];
                }
            } else {
                const uint16_t* wr = (const uint16_t*)W + (size_t)k * N;
                real wrow[256];
                for (int n = n0; n < n1; ++n) {
                    uint32_t u = (uint32_t)wr[n] << 16; float f; memcpy(&f, &u, 4);
                    wrow[n - n0] = (real)f;
                }
                for (int r = 0; r < R; ++r) {
                    real xv = X[(size_t)r * K + k];
                    real* y = Y + (size_t)r * N;
                    for (int n = n0; n < n1; ++n) y[n] += xv * wrow[n - n0];
                }
            }
        }
    }
}

/* attention of one query head vector q[Dh] over keys/values at positions 0..last (inclusive),
 * rows of kc/vc are `stride` reals apart: softmax(q.k/sqrt(Dh)) weighted sum of v. */
static void attend_one(const real* q, const real* kc, const real* vc, size_t stride, int last, int Dh,
                       real* out, real* scratch) {
    real inv = (real)1 / (real)sqrt((double)Dh);
    real mx = 0;
    for (int t = 0; t <= last; ++t) {
        const real* k = kc + (size_t)t * stride;
        real s = 0;
        for (int i = 0; i < Dh; ++i) s += q[i] * k[i];
        s *= inv;
        scratch[t] = s;
        if (t == 0 || s > mx) mx = s;
    }
    real den = 0;
    for (int t = 0; t <= last; ++t) { scratch[t] = (real)exp((double)(scratch[t] - mx)); den += scratch[t]; }
    for (int i = 0; i < Dh; ++i) out[i] = 0;
    for (int t = 0; t <= last; ++t) {
        const real* v = vc + (size_t)t * stride;
        real p = scratch[t] / den;
        for (int i = 0; i < Dh; ++i) out[i] += p * v[i];
    }
}

/* Window-causal attention on caller arrays (double in, double out), used to pin and to check
 * the isolated attention kernel.  q [R][H][Dh]; k, v [n+R][Hkv][Dh] (already rotated); row r
 * sees keys 0 .. n+r.  out [R][H*Dh].  Query head h reads kv head h / (H/Hkv). */
void oracle_attention_window(const double* q, const double* k, const double* v, int n, int R, int H,
                             int Hkv, int Dh, double* out) {
    size_t kvd = (size_t)Hkv * Dh, tot = (size_t)(n + R) * kvd;
    real* kr = (real*)malloc(tot * sizeof(real));
    real* vr = (real*)malloc(tot * sizeof(real));
    for (size_t i = 0; i < tot; ++i) { kr[i] = (real)k[i]; vr[i] = (real)v[i]; }
    int group = H / Hkv;
#pragma omp parallel for collapse(2) schedule(static)
    for (int r = 0; r < R; ++r)
        for (int h = 0; h < H; ++h) {
            real qv[512], ov[512];
            real* sc = (real*)malloc((size_t)(n + R) * sizeof(real));
            for (int i = 0; i < Dh; ++i) qv[i] = (real)q[((size_t)r * H + h) * Dh + i];
            int kvh = h / group;
            attend_one(qv, kr + (size_t)kvh * Dh, vr + (size_t)kvh * Dh, kvd, n + r, Dh, ov, sc);
            for (int i = 0; i < Dh; ++i) out[(size_t)r * H * Dh + (size_t)h * Dh + i] = (double)ov[i];
            free(sc);
        }
    free(kr); free(vr);
}

/* index of the largest value, lowest index on ties */
int32_t oracle_argmax(const real* v, int n) {
    int32_t best = 0;
    for (int i = 1; i < n; ++i) if (v[i] > v[best]) best = i;
    return best;
}

/* logits = act . W_lm on caller arrays; act [M][d] double, W [d][V]; logits [M][V] double
 * (nullable), amax [M] */
void oracle_lmhead_argmax(const double* act, const void* W, int wdtype, int M, int d, int V,
                          double* logits, int32_t* amax) {
    real* X = (real*)malloc((size_t)M * d * sizeof(real));
    real* Y = (real*)malloc((size_t)M * V * sizeof(real));
    for (size_t i = 0; i < (size_t)M * d; ++i) X[i] = (real)act[i];
    matmul_rows(W, wdtype, d, V, X, M, Y);
    for (int r = 0; r < M; ++r) {
        if (amax) amax[r] = oracle_argmax(Y + (size_t)r * V, V);
        if (logits) for (int n = 0; n < V; ++n) logits[(size_t)r * V + n] = (double)Y[(size_t)r * V + n];
    }
    free(X); free(Y);
}

/* ---------------------------------------------------------------- the decoder forward
 * Rows r = 0..R-1 carry token tok[r] at absolute position pos0 + r.  Row r attends cache
 * positions 0 .. pos0 + r (its own K/V included), i.e. the committed prefix plus the window
 * slots before it -- the causal-mask formulation of Eq. (2)/(4).  K/V of all R rows are
 * written at their positions; whether they become final is the caller's decision (n).
 * oracle_forward is made of three bodies -- embedding rows, decoder layers, final norm + LM head --
 * which oracle_embed / oracle_layers / oracle_head below expose one by one.
 */
static void embed_rows(const oracle_model* m, const int32_t* tok, int R, real* x) {
    const int d = m->s.d_model;
    for (int r = 0; r < R; ++r)
        for (int i = 0; i < d; ++i) x[(size_t)r * d + i] = wval(m->emb, m->s.wdtype, (size_t)tok[r] * d + i);
}

/* decoder layers l0 .. l1-1 applied in place to the residual stream x [R][d] of rows at positions pos0.. */
static void apply_layers(oracle_session* ss, int l0, int l1, int R, int pos0, real* x) {
    const oracle_model* m = ss->m;
    const oracle_shape* s = &m->s;
    const int d = s->d_model, H = s->n_heads, Hkv = s->n_kv_heads, Dh = s->head_dim, F = s->d_ffn;
    const int qd = H * Dh, kvd = Hkv * Dh, group = H / Hkv;
    real* nx = (real*)malloc((size_t)R * d * sizeof(real));
    real* q = (real*)malloc((size_t)R * qd * sizeof(real));
    real* kx = (real*)malloc((size_t)R * kvd * sizeof(real));
    real* vx = (real*)malloc((size_t)R * kvd * sizeof(real));
    real* att = (real*)malloc((size_t)R * qd * sizeof(real));
    real* proj = (real*)malloc((size_t)R * d * sizeof(real));
    real* gate = (real*)malloc((size_t)R * F * sizeof(real));
    real* up = (real*)malloc((size_t)R * F * sizeof(real));

    for (int l = l0; l < l1; ++l) {
        real* kcl = ss->kc + (size_t)l * ss->max_seq * kvd;
        real* vcl = ss->vc + (size_t)l * ss->max_seq * kvd;
        /* attention block */
        for (int r = 0; r < R; ++r)
            oracle_rmsnorm(x + (size_t)r * d, (const float*)m->w[T_G1][l], d, s->rms_eps, nx + (size_t)r * d);
        matmul_rows(m->w[T_WQ][l], s->wdtype, d, qd, nx, R, q);
        matmul_rows(m->w[T_WK][l], s->wdtype, d, kvd, nx, R, kx);
        matmul_rows(m->w[T_WV][l], s->wdtype, d, kvd, nx, R, vx);
        for (int r = 0; r < R; ++r) {
            int p = pos0 + r;
            for (int h = 0; h < H; ++h) oracle_rope(q + (size_t)r * qd + (size_t)h * Dh, Dh, p, s->rope_base);
            for (int h = 0; h < Hkv; ++h) oracle_rope(kx + (size_t)r * kvd + (size_t)h * Dh, Dh, p, s->rope_base);
            memcpy(kcl + (size_t)p * kvd, kx + (size_t)r * kvd, (size_t)kvd * sizeof(real));
            memcpy(vcl + (size_t)p * kvd, vx + (size_t)r * kvd, (size_t)kvd * sizeof(real));
        }
#pragma omp parallel for collapse(2) schedule(static)
        for (int r = 0; r < R; ++r)
            for (int h = 0; h < H; ++h) {
                real* sc = (real*)malloc((size_t)(pos0 + R) * sizeof(real));
                int kvh = h / group;
                attend_one(q + (size_t)r * qd + (size_t)h * Dh, kcl + (size_t)kvh * Dh, vcl + (size_t)kvh * Dh,
                           (size_t)kvd, pos0 + r, Dh, att + (size_t)r * qd + (size_t)h * Dh, sc);
                free(sc);
            }
        matmul_rows(m->w[T_WO][l], s->wdtype, qd, d, att, R, proj);
        for (size_t i = 0; i < (size_t)R * d; ++i) x[i] += proj[i];
        /* SwiGLU MLP block */
        for (int r = 0; r < R; ++r)
            oracle_rmsnorm(x + (size_t)r * d, (const float*)m->w[T_G2][l], d, s->rms_eps, nx + (size_t)r * d);
        matmul_rows(m->w[T_WG][l], s->wdtype, d, F, nx, R, gate);
        matmul_rows(m->w[T_WU][l], s->wdtype, d, F, nx, R, up);
        for (size_t i = 0; i < (size_t)R * F; ++i) gate[i] = oracle_silu(gate[i]) * up[i];
        matmul_rows(m->w[T_WD][l], s->wdtype, F, d, gate, R, proj);
        for (size_t i = 0; i < (size_t)R * d; ++i) x[i] += proj[i];
    }
    free(nx); free(q); free(kx); free(vx); free(att); free(proj); free(gate); free(up);
}

/* final norm, LM head, argmax of the residual stream x [R][d]; logits [R][vocab] as double and amax [R] nullable */
static void head_rows(const oracle_model* m, const real* x, int R, double* logits, int32_t* amax) {
    const int d = m->s.d_model, V = m->s.vocab;
    real* nx = (real*)malloc((size_t)R * d * sizeof(real));
    real* lg = (real*)malloc((size_t)R * V * sizeof(real));
    for (int r = 0; r < R; ++r) oracle_rmsnorm(x + (size_t)r * d, m->gf, d, m->s.rms_eps, nx + (size_t)r * d);
    matmul_rows(m->wlm, m->s.wdtype, d, V, nx, R, lg);
    for (int r = 0; r < R; ++r) {
        if (amax) amax[r] = oracle_argmax(lg + (size_t)r * V, V);
        if (logits) for (int n = 0; n < V; ++n) logits[(size_t)r * V + n] = (double)lg[(size_t)r * V + n];
    }
    free(nx); free(lg);
}

static int rows_ok(const oracle_session* ss, const int32_t* tok, int R, int pos0) {
    if (R <= 0 || pos0 < 0 || pos0 + R > ss->max_seq || ss->m->s.head_dim > 512) return 0;
    if (tok) for (int r = 0; r < R; ++r) if (tok[r] < 0 || tok[r] >= ss->m->s.vocab) return 0;
    return 1;
}

/* Outputs (nullable): logits [R][vocab] as double, amax [R], hidden [R][d] (residual stream
 * after the last layer, before the final norm) as double.  Returns 0, or -1 on bad arguments. */
int oracle_forward(oracle_session* ss, const int32_t* tok, int R, int pos0, double* logits,
                   int32_t* amax, double* hidden) {
    const oracle_model* m = ss->m;
    const int d = m->s.d_model;
    if (!rows_ok(ss, tok, R, pos0)) return -1;
    real* x = (real*)malloc((size_t)R * d * sizeof(real));
    embed_rows(m, tok, R, x);
    apply_layers(ss, 0, m->s.n_layers, R, pos0, x);
    if (hidden) for (size_t i = 0; i < (size_t)R * d; ++i) hidden[i] = (double)x[i];
    if (logits || amax) head_rows(m, x, R, logits, amax);
    free(x);
    return 0;
}

/* The same forward in three calls, so that a caller can hold the weights of one layer at a time (models whose
 * weights do not fit the host): oracle_embed gives the residual stream x [R][d] of the rows (as double: exact
 * for either build of `real`), oracle_layers applies layers l0 .. l1-1 to it in place (writing their K/V at
 * positions pos0.. of the session, as oracle_forward does), oracle_head gives logits and argmax.  The three are
 * the bodies oracle_forward itself is made of.  Return 0, or -1 on bad arguments. */
int oracle_embed(const oracle_model* m, const int32_t* tok, int R, double* x) {
    const int d = m->s.d_model;
    if (R <= 0) return -1;
    for (int r = 0; r < R; ++r) if (tok[r] < 0 || tok[r] >= m->s.vocab) return -1;
    real* xr = (real*)malloc((size_t)R * d * sizeof(real));
    embed_rows(m, tok, R, xr);
    for (size_t i = 0; i < (size_t)R * d; ++i) x[i] = (double)xr[i];
    free(xr);
    return 0;
}
int oracle_layers(oracle_session* ss, int l0, int l1, int R, int pos0, double* x) {
    const int d = ss->m->s.d_model;
    if (!rows_ok(ss, NULL, R, pos0) || l0 < 0 || l1 > ss->m->s.n_layers || l0 > l1) return -1;
    real* xr = (real*)malloc((size_t)R * d * sizeof(real));
    for (size_t i = 0; i < (size_t)R * d; ++i) xr[i] = (real)x[i];
    apply_layers(ss, l0, l1, R, pos0, xr);
    for (size_t i = 0; i < (size_t)R * d; ++i) x[i] = (double)xr[i];
    free(xr);
    return 0;
}
int oracle_head(const oracle_model* m, const double* x, int R, double* logits, int32_t* amax) {
    const int d = m->s.d_model;
    if (R <= 0) return -1;
    real* xr = (real*)malloc((size_t)R * d * sizeof(real));
    for (size_t i = 0; i < (size_t)R * d; ++i) xr[i] = (real)x[i];
    head_rows(m, xr, R, logits, amax);
    free(xr);
    return 0;
}

/* ---------------------------------------------------------------- Eq. (5): verification
 * w[0..W-1] is the window fed to the forward (w[0] exact, w[1..] approximate), o[0..W-1] the
 * per-row argmax (o[j] predicts the token after w[j]).  Approximate slot i is verified when
 * the fresh prediction for its position equals it: o[i-1] == w[i].  Slots are checked one by
 * one and the first miss stops the scan; the result K is the number of verified slots. */
int32_t oracle_verify(const int32_t* w, const int32_t* o, int32_t W) {
    int32_t K = 0;
    while (K < W - 1 && o[K] == w[K + 1]) ++K;
    return K;
}

/* ---------------------------------------------------------------- Eq. (1): greedy decoding
 * Feeds the prompt, then repeatedly appends the argmax token.  One token per forward.  Stops
 * after N tokens or after emitting eos (eos < 0: never).  Returns the number of tokens. */
int32_t oracle_greedy_ar(const oracle_model* m, const int32_t* prompt, int32_t P, int32_t N, int32_t eos,
                         int32_t* out) {
    oracle_session* ss = oracle_session_new(m, P + N + 1);
    int32_t got = 0, next = 0;
    if (!ss) return -5;
    if (P > 1 && oracle_forward(ss, prompt, P - 1, 0, NULL, NULL, NULL) != 0) { oracle_session_free(ss); return -1; }
    int32_t cur = prompt[P - 1];
    for (int32_t i = 0; i < N; ++i) {
        if (oracle_forward(ss, &cur, 1, P - 1 + i, NULL, &next, NULL) != 0) { got = -1; break; }
        out[got++] = next;
        if (eos >= 0 && next == eos) break;
        cur = next;
    }
    oracle_session_free(ss);
    return got;
}

/* ---------------------------------------------------------------- FastCoT decoding loop
 * One sequence.  buf[0..buf_len) is the Approximate Tokens Buffer (Sec. 4.2), buf[i] being the
 * current guess for generated token i; it is updated in place.  Per iteration (Sec. 4.1, 4.3):
 * fill the window from the buffer, one forward, verify (Eq. 5), write every fresh output back
 * to the buffer, accept K+1 tokens and advance.  Stops when N tokens are exact, when eos is
 * among the accepted tokens (output truncated after it), or after max_steps iterations
 * (max_steps <= 0: no cap).  Requires buf_len >= N + 2*W.
 * Outputs: out_ids[N]; *out_len; *out_steps; K_list[cap] (K of each iteration, nullable);
 * approx_tail[W-1] = the approximate tokens still in the window at stop (nullable).
 * Returns 0, -1 bad arguments, -5 out of memory. */
int oracle_jacobi_generate(const oracle_model* m, const int32_t* prompt, int32_t P, int32_t* buf,
                           int32_t buf_len, int32_t W, int32_t N, int32_t max_steps, int32_t eos,
                           int32_t* out_ids, int32_t* out_len, int32_t* out_steps, int32_t* K_list,
                           int32_t K_cap, int32_t* approx_tail) {
    if (P < 1 || W < 1 || N < 0 || buf_len < N + 2 * W) return -1;
    oracle_session* ss = oracle_session_new(m, P + N + 2 * W);
    if (!ss) return -5;
    int32_t* w = (int32_t*)malloc((size_t)W * sizeof(int32_t));
    int32_t* o = (int32_t*)malloc((size_t)W * sizeof(int32_t));
    int32_t n = P - 1, g = 0, steps = 0, len = 0, stop = 0, rc = 0;
    if (P > 1 && oracle_forward(ss, prompt, P - 1, 0, NULL, NULL, NULL) != 0) rc = -1;
    int32_t newest = prompt[P - 1];
    while (rc == 0 && g < N && !stop && (max_steps <= 0 || steps < max_steps)) {
        w[0] = newest;
        for (int32_t j = 1; j < W; ++j) w[j] = buf[g + j - 1];
        if (oracle_forward(ss, w, W, n, NULL, o, NULL) != 0) { rc = -1; break; }
        int32_t K = oracle_verify(w, o, W);
        for (int32_t j = 0; j < W; ++j) buf[g + j] = o[j];
        for (int32_t j = 0; j <= K && !stop; ++j) {
            if (len < N) out_ids[len++] = o[j];
            if (eos >= 0 && o[j] == eos) stop = 1;
        }
        if (K_list && steps < K_cap) K_list[steps] = K;
        newest = o[K];
        n += K + 1; g += K + 1; ++steps;
    }
    if (approx_tail) for (int32_t j = 0; j < W - 1; ++j) approx_tail[j] = buf[g + j];
    *out_len = len; *out_steps = steps;
    free(w); free(o); oracle_session_free(ss);
    return rc;
}
