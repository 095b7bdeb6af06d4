/*
 * CLaSp CPU oracle  --  TEST INFRASTRUCTURE, NOT THE PRODUCT.
 *
 * A plain, slow, fp64 implementation of what the CLaSp hot path computes:
 *   - one LLaMA-style pre-norm decoder layer f_l on a single row (Sec. 3.4, h_{l+1} = f_l(h_l);
 *     "DecoderLayer f_i" in the inputs of Algorithm 1),
 *   - a whole-model forward of one token with per-layer hidden-state capture, optionally with a
 *     skip mask (the draft model M_d of Sec. 3.3 is the verify model M_v minus the layers in S),
 *   - the layer-skip dynamic program of Eq. 2 / Algorithm 1 and its backtracking.
 *
 * Only tests, the smoke check and the benchmark's cpu_baseline leg may call this file. It shares no code
 * with the HIP library and includes none of its headers. Every dot product, norm and softmax accumulates in
 * double; activations are never rounded. Weights are taken as they are given (fp32, or bf16 bit patterns
 * widened exactly to double), so oracle and device read identical weight values.
 *
 * Readings of the paper where it is silent or inconsistent (listed in full in the design notes):
 *   - Eq. 1 prints "arg min" of the cosine; Eq. 2 takes a max and Algorithm 1 keeps the larger score, so the
 *     objective is read as maximisation.
 *   - Algorithm 1 lists states x_0..x_{L-1} but reads x_i up to i = L: L+1 states are taken, x_L being the
 *     output of the last layer before the final norm. Its loop is read as i = 1..L.
 *   - The slices 1:l+1 and :l are half-open; the comparison of the two score halves is element-wise.
 *   - Strict '>' keeps the computed candidate; ties (and NaN) keep the skip candidate.
 *   - "norm" in Algorithm 1 is L2 normalisation, x / max(||x||, 1e-12), so that the product is a cosine.
 *   - The backtracking starts at (L, M) and tests a stored choice bit instead of comparing vectors; the two
 *     agree because identical vectors give identical scores, hence a tie, hence "skip".
 *   - Every candidate row in the DP is the last accepted token re-imagined: position p, attending the
 *     full model's keys and values of positions 0..p-1 of that layer plus its own key/value (Sec. 3.6: the
 *     candidate states share one KV cache and do not see each other). The DP writes no KV.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

typedef struct {
    int32_t n_layers, d_model, n_heads, n_kv_heads, head_dim, d_ffn, vocab;
    int32_t wdtype; /* 0: float32 matrices, 1: bf16 bit patterns (uint16) */
    double rms_eps, rope_base;
    const void *embed;        /* [vocab][d_model]            */
    const void *lm_head;      /* [vocab][d_model]            */
    const float *final_norm;  /* [d_model] gains, float32    */
    const float *const *attn_norm; /* per layer [d_model]    */
    const float *const *mlp_norm;  /* per layer [d_model]    */
    const void *const *wq;    /* [n_heads*head_dim][d_model]     */
    const void *const *wk;    /* [n_kv_heads*head_dim][d_model]  */
    const void *const *wv;    /* [n_kv_heads*head_dim][d_model]  */
    const void *const *wo;    /* [d_model][n_heads*head_dim]     */
    const void *const *w_gate;/* [d_ffn][d_model]                */
    const void *const *w_up;  /* [d_ffn][d_model]                */
    const void *const *w_down;/* [d_model][d_ffn]                */
} oracle_model;

static inline double bf16_to_double(uint16_t b) {
    uint32_t u = ((uint32_t)b) << 16;
    float f;
    memcpy(&f, &u, 4);
    return (double)f;
}

static inline double w_at(const void *w, int wdtype, size_t idx) {
    return wdtype ? bf16_to_double(((const uint16_t *)w)[idx]) : (double)((const float *)w)[idx];
}

/* y[n] = sum_k W[n][k] x[k], W row-major [N][K]. */
static void matvec(const void *W, int wdtype, int N, int K, const double *x, double *y) {
#pragma omp parallel for schedule(static)
    for (int n = 0; n < N; ++n) {
        double acc = 0.0;
        size_t base = (size_t)n * (size_t)K;
        if (wdtype) {
            const uint16_t *w = (const uint16_t *)W + base;
#pragma omp simd reduction(+ : acc)
            for (int k = 0; k < K; ++k) acc += bf16_to_double(w[k]) * x[k];
        } else {
            const float *w = (const float *)W + base;
#pragma omp simd reduction(+ : acc)
            for (int k = 0; k < K; ++k) acc += (double)w[k] * x[k];
        }
        y[n] = acc;
    }
}

/* RMSNorm(x; g) = x / sqrt(mean(x^2) + eps) * g */
static void rmsnorm(const double *x, const float *g, int d, double eps, double *y) {
    double ss = 0.0;
    for (int k = 0; k < d; ++k) ss += x[k] * x[k];
    double r = 1.0 / sqrt(ss / (double)d + eps);
    for (int k = 0; k < d; ++k) y[k] = x[k] * r * (double)g[k];
}

/* Rotary embedding, half-split pairing: (v[k], v[k+hd/2]) rotated by pos * base^(-2k/hd). */
static void rope(double *v, int hd, int pos, double base) {
    int half = hd / 2;
    for (int k = 0; k < half; ++k) {
        double theta = (double)pos * pow(base, -2.0 * (double)k / (double)hd);
        double c = cos(theta), s = sin(theta);
        double a = v[k], b = v[k + half];
        v[k] = a * c - b * s;
        v[k + half] = b * c + a * s;
    }
}

/*
 * One decoder layer on one row:   a = h + Wo . Attn(RoPE(Wq n1), RoPE(Wk n1), Wv n1),  n1 = RMSNorm(h)
 *                                 out = a + Wd . (silu(Wg n2) * (Wu n2)),               n2 = RMSNorm(a)
 * The row sits at position `pos`; it attends cache rows 0..n_prefix-1 of this layer (keys already rotated)
 * and its own key/value. Kc/Vc: this layer's cache, double [.][n_kv_heads][head_dim].
 * k_new/v_new (may be NULL) receive the row's own rotated key and value.
 */
int clasp_oracle_layer(const oracle_model *m, int l, const double *h, int pos, int n_prefix,
                       const double *Kc, const double *Vc, double *out, double *k_new, double *v_new) {
    const int d = m->d_model, nq = m->n_heads, nkv = m->n_kv_heads, hd = m->head_dim, F = m->d_ffn;
    const int qd = nq * hd, kvd = nkv * hd, group = nq / nkv;
    if (l < 0 || l >= m->n_layers || n_prefix < 0 || pos < 0) return -1;
    double *n1 = malloc(sizeof(double) * d), *q = malloc(sizeof(double) * qd);
    double *k = malloc(sizeof(double) * kvd), *v = malloc(sizeof(double) * kvd);
    double *att = malloc(sizeof(double) * qd), *a = malloc(sizeof(double) * d);
    double *n2 = malloc(sizeof(double) * d), *gate = malloc(sizeof(double) * F);
    double *up = malloc(sizeof(double) * F), *proj = malloc(sizeof(double) * d);
    double *sc = malloc(sizeof(double) * (size_t)(n_prefix + 1));

    rmsnorm(h, m->attn_norm[l], d, m->rms_eps, n1);
    matvec(m->wq[l], m->wdtype, qd, d, n1, q);
    matvec(m->wk[l], m->wdtype, kvd, d, n1, k);
    matvec(m->wv[l], m->wdtype, kvd, d, n1, v);
    for (int hq = 0; hq < nq; ++hq) rope(q + hq * hd, hd, pos, m->rope_base);
    for (int hk = 0; hk < nkv; ++hk) rope(k + hk * hd, hd, pos, m->rope_base);

    const double scale = 1.0 / sqrt((double)hd);
    for (int hq = 0; hq < nq; ++hq) {
        const int hk = hq / group;
        const double *qv = q + hq * hd;
        double mx = -INFINITY;
        for (int t = 0; t <= n_prefix; ++t) {
            const double *kv = (t < n_prefix) ? Kc + ((size_t)t * nkv + hk) * hd : k + hk * hd;
            double s = 0.0;
            for (int e = 0; e < hd; ++e) s += qv[e] * kv[e];
            sc[t] = s * scale;
            if (sc[t] > mx) mx = sc[t];
        }
        double den = 0.0;
        for (int t = 0; t <= n_prefix; ++t) { sc[t] = exp(sc[t] - mx); den += sc[t]; }
        for (int e = 0; e < hd; ++e) {
            double acc = 0.0;
            for (int t = 0; t <= n_prefix; ++t) {
                const double *vv = (t < n_prefix) ? Vc + ((size_t)t * nkv + hk) * hd : v + hk * hd;
                acc += sc[t] * vv[e];
            }
            att[hq * hd + e] = acc / den;
        }
    }
    matvec(m->wo[l], m->wdtype, d, qd, att, proj);
    for (int e = 0; e < d; ++e) a[e] = h[e] + proj[e];

    rmsnorm(a, m->mlp_norm[l], d, m->rms_eps, n2);
    matvec(m->w_gate[l], m->wdtype, F, d, n2, gate);
    matvec(m->w_up[l], m->wdtype, F, d, n2, up);
    for (int e = 0; e < F; ++e) gate[e] = gate[e] / (1.0 + exp(-gate[e])) * up[e];
    matvec(m->w_down[l], m->wdtype, d, F, gate, proj);
    for (int e = 0; e < d; ++e) out[e] = a[e] + proj[e];

    if (k_new) memcpy(k_new, k, sizeof(double) * kvd);
    if (v_new) memcpy(v_new, v, sizeof(double) * kvd);
    free(n1); free(q); free(k); free(v); free(att); free(a); free(n2); free(gate); free(up); free(proj); free(sc);
    return 0;
}

/*
 * One token through the model at position `pos`, attending positions 0..pos-1 of each layer's cache.
 * skip (may be NULL): skip[l] != 0 leaves layer l out (the draft model of Sec. 3.3); such a layer's cache
 * row at `pos` is not written. K/V: double [n_layers][t_max][n_kv_heads][head_dim].
 * states_out (may be NULL): [(n_layers+1)][d_model], state l = input of layer l, state L = output of the last
 * layer before the final norm (only meaningful without a skip mask). logits_out (may be NULL): [vocab].
 */
int clasp_oracle_token(const oracle_model *m, int token, int pos, const uint8_t *skip, double *K, double *V,
                       int t_max, double *states_out, double *logits_out) {
    const int d = m->d_model, L = m->n_layers, kvd = m->n_kv_heads * m->head_dim;
    if (token < 0 || token >= m->vocab || pos < 0 || pos >= t_max) return -1;
    double *h = malloc(sizeof(double) * d), *o = malloc(sizeof(double) * d);
    double *kn = malloc(sizeof(double) * kvd), *vn = malloc(sizeof(double) * kvd);
    for (int e = 0; e < d; ++e) h[e] = w_at(m->embed, m->wdtype, (size_t)token * d + e);
    for (int l = 0; l < L; ++l) {
        if (states_out) memcpy(states_out + (size_t)l * d, h, sizeof(double) * d);
        if (skip && skip[l]) continue;
        double *Kl = K + (size_t)l * t_max * kvd, *Vl = V + (size_t)l * t_max * kvd;
        int rc = clasp_oracle_layer(m, l, h, pos, pos, Kl, Vl, o, kn, vn);
        if (rc) { free(h); free(o); free(kn); free(vn); return rc; }
        memcpy(Kl + (size_t)pos * kvd, kn, sizeof(double) * kvd);
        memcpy(Vl + (size_t)pos * kvd, vn, sizeof(double) * kvd);
        memcpy(h, o, sizeof(double) * d);
    }
    if (states_out) memcpy(states_out + (size_t)L * d, h, sizeof(double) * d);
    if (logits_out) {
        rmsnorm(h, m->final_norm, d, m->rms_eps, o);
        matvec(m->lm_head, m->wdtype, m->vocab, d, o, logits_out);
    }
    free(h); free(o); free(kn); free(vn);
    return 0;
}

/* cosine(a, b) with each vector L2-normalised as x / max(||x||, 1e-12). */
double clasp_oracle_cosine(const double *a, const double *b, int d) {
    double na = 0.0, nb = 0.0, ab = 0.0;
    for (int e = 0; e < d; ++e) { na += a[e] * a[e]; nb += b[e] * b[e]; ab += a[e] * b[e]; }
    na = fmax(sqrt(na), 1e-12);
    nb = fmax(sqrt(nb), 1e-12);
    return ab / (na * nb);
}

/*
 * The layer-skip dynamic program (Eq. 2, Algorithm 1) for one token.
 *   X        [(L+1)][d]   stored verify-pass states x_0..x_L of the token at position `pos`
 *   K, V     the full model's cache; rows 0..pos-1 of every layer are read, nothing is written
 *   M        skip budget, 0 <= M <= L
 *   override (may be NULL) [(L+1)*(M+1)] int8: -1 keep the oracle's own decision, 0 force "computed",
 *            1 force "skip" for that cell (used by tests to follow a device decision on a near-tie)
 * Outputs (each may be NULL), tables indexed [i*(M+1)+j]:
 *   sigma_c  cosine(x_i, f_{i-1}(g(i-1,j)))   for 1 <= j <= min(i-1,M), NaN elsewhere
 *   sigma_s  cosine(x_i, g(i-1,j-1))          for 1 <= j <= min(i,M),   NaN elsewhere
 *   choice   0 = computed candidate kept, 1 = skip candidate kept, 255 = cell not defined (j=0 or j>i)
 *   g_final  [d] = g(L, M);   skip_out [L] = backtracked skip set, 1 = skipped
 */
int clasp_oracle_dp(const oracle_model *m, const double *X, int pos, const double *K, const double *V, int t_max,
                    int M, const int8_t *override, double *sigma_c, double *sigma_s, uint8_t *choice,
                    double *g_final, uint8_t *skip_out) {
    const int d = m->d_model, L = m->n_layers, kvd = m->n_kv_heads * m->head_dim;
    if (M < 0 || M > L || pos < 0 || pos > t_max) return -1;
    const int W = M + 1;
    double *g_prev = calloc((size_t)W * d, sizeof(double)), *g_cur = calloc((size_t)W * d, sizeof(double));
    double *cand = malloc(sizeof(double) * d);
    uint8_t *C = malloc((size_t)(L + 1) * W);
    memset(C, 255, (size_t)(L + 1) * W);
    for (size_t c = 0; c < (size_t)(L + 1) * W; ++c) {
        if (sigma_c) sigma_c[c] = NAN;
        if (sigma_s) sigma_s[c] = NAN;
    }
    memcpy(g_prev, X, sizeof(double) * d); /* g(0,0) = x_0 */
    for (int i = 1; i <= L; ++i) {
        const double *xi = X + (size_t)i * d;
        memcpy(g_cur, xi, sizeof(double) * d); /* g(i,0) = x_i */
        const int ell = (i - 1 < M) ? i - 1 : M;
        const double *Kl = K + (size_t)(i - 1) * t_max * kvd, *Vl = V + (size_t)(i - 1) * t_max * kvd;
        for (int j = 1; j <= ell; ++j) {
            clasp_oracle_layer(m, i - 1, g_prev + (size_t)j * d, pos, pos, Kl, Vl, cand, NULL, NULL);
            const double *skipc = g_prev + (size_t)(j - 1) * d;
            double sc = clasp_oracle_cosine(cand, xi, d), ss = clasp_oracle_cosine(skipc, xi, d);
            int keep_computed = sc > ss;
            if (override && override[i * W + j] >= 0) keep_computed = (override[i * W + j] == 0);
            memcpy(g_cur + (size_t)j * d, keep_computed ? cand : skipc, sizeof(double) * d);
            C[i * W + j] = keep_computed ? 0 : 1;
            if (sigma_c) sigma_c[i * W + j] = sc;
            if (sigma_s) sigma_s[i * W + j] = ss;
        }
        if (i <= M) { /* all of the first i layers skipped: g(i,i) = g(i-1,i-1) */
            memcpy(g_cur + (size_t)i * d, g_prev + (size_t)(i - 1) * d, sizeof(double) * d);
            C[i * W + i] = 1;
            if (sigma_s) sigma_s[i * W + i] = clasp_oracle_cosine(g_prev + (size_t)(i - 1) * d, xi, d);
        }
        double *t = g_prev; g_prev = g_cur; g_cur = t;
    }
    if (g_final) memcpy(g_final, g_prev + (size_t)M * d, sizeof(double) * d);
    if (choice) memcpy(choice, C, (size_t)(L + 1) * W);
    if (skip_out) {
        memset(skip_out, 0, L);
        int i = L, j = M;
        while (i > 0 && j > 0) {
            if (C[i * W + j] == 1) { skip_out[i - 1] = 1; --j; }
            --i;
        }
    }
    free(g_prev); free(g_cur); free(cand); free(C);
    return 0;
}

int clasp_oracle_num_threads(void) {
    int n = 1;
#ifdef _OPENMP
#pragma omp parallel
    {
#pragma omp single
        n = omp_get_num_threads();
    }
#endif
    return n;
}
