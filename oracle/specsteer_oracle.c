/*
 * SpecSteer verify-and-recover: float64 CPU oracle.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, plain, obviously-correct
 * statement of what one Draft-Verify-Recover block computes (Algorithm 1,
 * Phases 2 and 3; Eq. 7 ratio-based verification rule; Eq. 8 steering
 * recovery logits; the sampling step of phase 3).  It shares no code, header,
 * table or helper with the HIP library and must never be called from the
 * product path: only the tests, the smoke check and the benchmark's
 * cpu_baseline leg may load it.
 *
 * Everything is computed in IEEE double precision.  Logits arrive as fp32 or
 * bf16 and are widened exactly; the three hyper-parameters arrive as fp32 and
 * are widened exactly.  There is no blocking, fusion or reordering: each step
 * below is the definition written out (two-pass log-sum-exp, sequential
 * cumulative sum).
 *
 * Readings taken where the paper is silent (all listed in the design notes):
 *   - a temperature T > 0 divides all three logit tensors wherever a softmax
 *     is taken (the paper has no temperature; T = 1 is the paper);
 *   - acceptance is "u <= alpha" exactly as Algorithm 1 writes it;
 *   - when every draft token is accepted a bonus token is drawn from the
 *     recovery distribution of the row after the last draft token;
 *   - uniforms[b][t], t < K_b, drives acceptance test t; uniforms[b][k_max]
 *     drives the single sampled token;
 *   - the sampled token is the inverse CDF in vocabulary-index order:
 *     the first j whose inclusive cumulative probability exceeds the uniform.
 *
 * Build: gcc -O2 -ffp-contract=off -fopenmp -shared -fPIC -o libspecsteer_oracle.so specsteer_oracle.c -lm
 * (no fused multiply-add: Eq. 8 is one multiply and one add, each rounded, so that an argmax over
 * it is reproducible bit for bit)
 * The OpenMP loop runs over the independent sequences only and changes no
 * arithmetic; it exists so the benchmark can time the oracle on all host cores.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

enum { SSO_F32 = 0, SSO_BF16 = 1 };

typedef struct {
    int32_t batch;       /* B */
    int32_t k_max;       /* padded draft length; logits hold k_max+1 rows per sequence */
    int32_t vocab;       /* V */
    int32_t dtype;       /* SSO_F32 or SSO_BF16, for all three logit tensors */
    int64_t stride_b;    /* element stride between sequences; 0 => (k_max+1)*V */
    int64_t stride_t;    /* element stride between positions; 0 => V */
    float lambda;        /* verification threshold (Eq. 7) */
    float beta;          /* steering-recovery strength (Eq. 8) */
    float temperature;   /* T > 0 */
    int32_t num_threads; /* OpenMP threads over sequences; <=1 => serial */
    int32_t greedy;      /* 0: draw the token by inverse CDF; 1: take argmax h_rec (lowest index on ties),
                            the deterministic decoding the paper's experiments use in place of the sampling step */
} sso_params;

/* Exact widening of one stored logit to double. */
static double widen(const void *base, int dtype, int64_t idx) {
    if (dtype == SSO_F32) {
        return (double)((const float *)base)[idx];
    } else {
        uint32_t bits = (uint32_t)((const uint16_t *)base)[idx] << 16;
        float f;
        memcpy(&f, &bits, sizeof f);
        return (double)f;
    }
}

/* row[v] = logit[v] / T, v = 0..V-1 */
static void scaled_row(const void *base, int dtype, int64_t off, int V, double T, double *row) {
    for (int v = 0; v < V; ++v) row[v] = widen(base, dtype, off + v) / T;
}

/* log sum_v exp(x[v]) with the maximum taken out first (two passes). */
static double log_sum_exp(const double *x, int V) {
    double m = x[0];
    for (int v = 1; v < V; ++v)
        if (x[v] > m) m = x[v];
    double s = 0.0;
    for (int v = 0; v < V; ++v) s += exp(x[v] - m);
    return m + log(s);
}

/*
 * One sequence.  Scratch rows g and sm hold V doubles each.
 * Returns through the out pointers for this sequence only (already offset).
 */
static void verify_one(const void *G, const void *Sp, const void *Sm, const int32_t *draft, int K,
                       const float *u, const sso_params *p, int64_t seq_off, int64_t st, double *g,
                       double *sm, int32_t *accepted_len, int32_t *next_token,
                       double *next_token_logprob, double *recovery_logprobs, double *draft_logprobs,
                       double *alpha_out, double *sample_margin) {
    const int V = p->vocab, kmax = p->k_max, dt = p->dtype;
    const double T = (double)p->temperature;
    const double lam = (double)p->lambda;
    const double beta = (double)p->beta;

    /* Phase 2: ratio-based verification, position by position, stop at the first rejection. */
    int n = K;
    for (int t = 0; t < K; ++t) {
        const int y = draft[t];
        scaled_row(G, dt, seq_off + (int64_t)t * st, V, T, g);
        scaled_row(Sm, dt, seq_off + (int64_t)t * st, V, T, sm);
        const double lpG = g[y] - log_sum_exp(g, V);   /* log P_LLM(y_t)  */
        const double lpS = sm[y] - log_sum_exp(sm, V); /* log P_SLM^-(y_t) */
        if (draft_logprobs) {
            draft_logprobs[2 * t + 0] = lpG;
            draft_logprobs[2 * t + 1] = lpS;
        }
        /* Eq. 7: alpha = min(1, P_LLM / (lambda * P_SLM^-)) */
        double alpha = exp(lpG - lpS - log(lam));
        if (alpha > 1.0) alpha = 1.0;
        if (alpha_out) alpha_out[t] = alpha;
        if (!((double)u[t] <= alpha)) {
            n = t;
            break;
        }
    }
    /* Diagnostics only: log-probs of the draft tokens the loop above never reached. */
    if (draft_logprobs) {
        for (int t = n + 1; t < K; ++t) {
            const int y = draft[t];
            scaled_row(G, dt, seq_off + (int64_t)t * st, V, T, g);
            scaled_row(Sm, dt, seq_off + (int64_t)t * st, V, T, sm);
            draft_logprobs[2 * t + 0] = g[y] - log_sum_exp(g, V);
            draft_logprobs[2 * t + 1] = sm[y] - log_sum_exp(sm, V);
        }
    }

    /* Phase 3 (or bonus): Eq. 8 at row n, then Softmax and one inverse-CDF draw. */
    const int64_t off = seq_off + (int64_t)n * st;
    int amax = 0;
    double hmax = -INFINITY;
    for (int v = 0; v < V; ++v) {
        const double hl = widen(G, dt, off + v);
        const double hp = widen(Sp, dt, off + v);
        const double hm = widen(Sm, dt, off + v);
        /* Eq. 8.  A token masked (-inf) in both specialist rows carries no steering: 0, not inf - inf. */
        const double hrec = hl + beta * ((hp == hm) ? 0.0 : hp - hm);
        if (hrec > hmax) { /* strict: the lowest index wins a tie */
            hmax = hrec;
            amax = v;
        }
        g[v] = hrec / T;
    }
    const double lse = log_sum_exp(g, V);
    for (int v = 0; v < V; ++v) g[v] -= lse; /* g is now log Softmax(h_rec / T) */
    if (recovery_logprobs) memcpy(recovery_logprobs, g, (size_t)V * sizeof(double));

    const double us = (double)u[kmax];
    double c = 0.0, margin = INFINITY;
    int tok = -1, last_pos = -1;
    for (int v = 0; v < V; ++v) {
        const double pv = exp(g[v]);
        c += pv;
        if (pv > 0.0) last_pos = v;
        if (tok < 0 && c > us) tok = v;
        const double d = fabs(c - us);
        if (d < margin) margin = d;
    }
    if (tok < 0) tok = last_pos; /* only reachable through rounding when us is within an ulp of 1 */
    if (p->greedy) {
        tok = amax;
        margin = INFINITY; /* no uniform is involved: nothing excuses a mismatch */
    }

    *accepted_len = n;
    *next_token = tok;
    if (next_token_logprob) *next_token_logprob = g[tok];
    if (sample_margin) *sample_margin = margin;
}

/*
 * All pointers are HOST pointers.
 *   G, S_ctx, S_noctx : [B, k_max+1, V] logits (dtype per params, strides per params)
 *   draft             : [B, k_max] int32, entries t >= K_b ignored
 *   draft_len         : [B] int32 or NULL (=> K_b = k_max)
 *   uniforms          : [B, k_max+1] fp32 in [0,1)
 * Outputs (any of the double* may be NULL):
 *   accepted_len [B], next_token [B]           : -1 marks a bad sequence
 *   next_token_logprob [B]                     : NaN for a bad sequence
 *   recovery_logprobs [B, V]                   : log Softmax(h_rec/T) at row n_b
 *   draft_logprobs [B, k_max, 2]               : (log P_LLM(y_t), log P_SLM^-(y_t)), t < K_b; NaN elsewhere
 *   alpha [B, k_max]                           : Eq. 7 at every position the loop tested; NaN elsewhere
 *   sample_margin [B]                          : min_j |CDF[j] - u_s|
 * Returns 0, or 1 for an argument error (nothing written).
 */
int specsteer_oracle_verify_block(const void *G, const void *S_ctx, const void *S_noctx,
                                  const int32_t *draft, const int32_t *draft_len,
                                  const float *uniforms, const sso_params *p, int32_t *accepted_len,
                                  int32_t *next_token, double *next_token_logprob,
                                  double *recovery_logprobs, double *draft_logprobs, double *alpha,
                                  double *sample_margin) {
    if (!G || !S_ctx || !S_noctx || !draft || !uniforms || !p || !accepted_len || !next_token) return 1;
    if (p->batch < 0 || p->k_max < 0 || p->vocab < 1) return 1;
    if (p->dtype != SSO_F32 && p->dtype != SSO_BF16) return 1;
    if (!(p->lambda > 0.0f) || !isfinite(p->lambda)) return 1;
    if (!(p->temperature > 0.0f) || !isfinite(p->temperature)) return 1;
    if (!isfinite(p->beta)) return 1;
    const int B = p->batch, kmax = p->k_max, V = p->vocab;
    const int64_t st = p->stride_t ? p->stride_t : (int64_t)V;
    const int64_t sb = p->stride_b ? p->stride_b : (int64_t)(kmax + 1) * st;
    int nthreads = p->num_threads > 1 ? p->num_threads : 1;
#ifndef _OPENMP
    nthreads = 1;
#endif

#pragma omp parallel num_threads(nthreads)
    {
        double *g = (double *)malloc((size_t)V * sizeof(double));
        double *sm = (double *)malloc((size_t)V * sizeof(double));
#pragma omp for schedule(dynamic, 1)
        for (int b = 0; b < B; ++b) {
            const int K = draft_len ? draft_len[b] : kmax;
            double *dl = draft_logprobs ? draft_logprobs + (size_t)b * kmax * 2 : NULL;
            double *al = alpha ? alpha + (size_t)b * kmax : NULL;
            if (dl)
                for (int i = 0; i < 2 * kmax; ++i) dl[i] = NAN;
            if (al)
                for (int i = 0; i < kmax; ++i) al[i] = NAN;
            int bad = (K < 0 || K > kmax);
            for (int t = 0; !bad && t < K; ++t) {
                const int y = draft[(size_t)b * kmax + t];
                if (y < 0 || y >= V) bad = 1;
            }
            if (bad) {
                accepted_len[b] = -1;
                next_token[b] = -1;
                if (next_token_logprob) next_token_logprob[b] = NAN;
                if (sample_margin) sample_margin[b] = NAN;
                continue;
            }
            verify_one(G, S_ctx, S_noctx, draft + (size_t)b * kmax, K,
                       uniforms + (size_t)b * (kmax + 1), p, (int64_t)b * sb, st, g, sm,
                       accepted_len + b, next_token + b,
                       next_token_logprob ? next_token_logprob + b : NULL,
                       recovery_logprobs ? recovery_logprobs + (size_t)b * V : NULL, dl, al,
                       sample_margin ? sample_margin + b : NULL);
        }
        free(g);
        free(sm);
    }
    return 0;
}

int specsteer_oracle_max_threads(void) {
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/* ------------------------------------------------------------------------------------------
 * Deployment split of the recovery step (deployment appendix, the downlink step).
 *
 * Cloud side: at the rejected row the non-private part of Eq. 8,
 *     h_cloud = h_LLM - beta * h_SLM^-,
 * is truncated to its top-k entries (k = 32 in the paper).  Edge side: the private term is added
 * back on those entries, h_rec = h_cloud + beta * h_SLM^+, and the token is resampled locally.
 *
 * Readings where the paper is silent: entries are ordered by decreasing h_cloud, ties by
 * increasing token id; the payload carries fp32 values; a token outside the top-k has
 * probability zero; the edge draws by inverse CDF in payload order (or takes the first maximum
 * when greedy); if V < k the unused slots hold id -1 and value -inf.
 * ------------------------------------------------------------------------------------------ */

typedef struct {
    double v;
    int32_t idx;
} sso_entry;

static int entry_before(const void *pa, const void *pb) {
    const sso_entry *a = (const sso_entry *)pa, *b = (const sso_entry *)pb;
    if (a->v > b->v) return -1;
    if (a->v < b->v) return 1;
    return (a->idx > b->idx) - (a->idx < b->idx);
}

/*
 * Host pointers.  row[b] in [0, k_max] selects the row of sequence b; a negative row marks a
 * flagged sequence (all ids -1, values -inf).  out_index [B, topk] int32, out_value [B, topk] fp32.
 * Only batch, k_max, vocab, dtype, strides and beta of the params are used.
 */
int specsteer_oracle_cloud_topk(const void *G, const void *S_noctx, const int32_t *row, const sso_params *p,
                                int32_t topk, int32_t *out_index, float *out_value) {
    if (!G || !S_noctx || !row || !p || !out_index || !out_value || topk < 1) return 1;
    const int B = p->batch, V = p->vocab, kmax = p->k_max, dt = p->dtype;
    const int64_t st = p->stride_t ? p->stride_t : (int64_t)V;
    const int64_t sb = p->stride_b ? p->stride_b : (int64_t)(kmax + 1) * st;
    const double beta = (double)p->beta;
    sso_entry *e = (sso_entry *)malloc((size_t)V * sizeof(sso_entry));
    for (int b = 0; b < B; ++b) {
        int32_t *oi = out_index + (size_t)b * topk;
        float *ov = out_value + (size_t)b * topk;
        for (int j = 0; j < topk; ++j) {
            oi[j] = -1;
            ov[j] = -INFINITY;
        }
        if (row[b] < 0 || row[b] > kmax) continue;
        const int64_t off = (int64_t)b * sb + (int64_t)row[b] * st;
        for (int v = 0; v < V; ++v) {
            const double hl = widen(G, dt, off + v);
            /* a token the generalist masks (-inf) stays masked whatever the specialist says */
            e[v].v = (hl == -INFINITY) ? -INFINITY : hl - beta * widen(S_noctx, dt, off + v);
            e[v].idx = v;
        }
        qsort(e, (size_t)V, sizeof(sso_entry), entry_before);
        for (int j = 0; j < topk && j < V; ++j) {
            oi[j] = e[j].idx;
            ov[j] = (float)e[j].v;
        }
    }
    free(e);
    return 0;
}

/*
 * Host pointers.  index/value [B, topk] as produced above, S_ctx [B, k_max+1, V], row [B],
 * uniform [B] fp32.  Outputs next_token [B] (-1 for a flagged sequence), next_token_logprob [B]
 * (log-softmax over the top-k candidates), cand_logprobs [B, topk] or NULL, sample_margin [B] or NULL.
 * Uses batch, k_max, vocab, dtype, strides, beta, temperature and greedy of the params.
 */
int specsteer_oracle_edge_resample(const int32_t *index, const float *value, const void *S_ctx, const int32_t *row,
                                   const float *uniform, const sso_params *p, int32_t topk, int32_t *next_token,
                                   double *next_token_logprob, double *cand_logprobs, double *sample_margin) {
    if (!index || !value || !S_ctx || !row || !uniform || !p || !next_token || topk < 1) return 1;
    const int B = p->batch, V = p->vocab, kmax = p->k_max, dt = p->dtype;
    const int64_t st = p->stride_t ? p->stride_t : (int64_t)V;
    const int64_t sb = p->stride_b ? p->stride_b : (int64_t)(kmax + 1) * st;
    const double beta = (double)p->beta, T = (double)p->temperature;
    double *h = (double *)malloc((size_t)topk * sizeof(double));
    for (int b = 0; b < B; ++b) {
        const int32_t *ix = index + (size_t)b * topk;
        const float *vl = value + (size_t)b * topk;
        int n = 0;
        while (n < topk && ix[n] >= 0) ++n; /* valid candidates are a prefix */
        if (cand_logprobs)
            for (int j = 0; j < topk; ++j) cand_logprobs[(size_t)b * topk + j] = -INFINITY;
        if (row[b] < 0 || row[b] > kmax || n == 0) {
            next_token[b] = -1;
            if (next_token_logprob) next_token_logprob[b] = NAN;
            if (sample_margin) sample_margin[b] = NAN;
            continue;
        }
        const int64_t off = (int64_t)b * sb + (int64_t)row[b] * st;
        int amax = 0;
        for (int j = 0; j < n; ++j) {
            h[j] = (double)vl[j] + beta * widen(S_ctx, dt, off + ix[j]); /* edge adds its private term */
            if (h[j] > h[amax]) amax = j;
        }
        double hs[64];
        double *x = topk <= 64 ? hs : (double *)malloc((size_t)topk * sizeof(double));
        for (int j = 0; j < n; ++j) x[j] = h[j] / T;
        const double lse = log_sum_exp(x, n);
        double c = 0.0, margin = INFINITY;
        int pick = -1, last_pos = -1;
        for (int j = 0; j < n; ++j) {
            const double lp = x[j] - lse;
            if (cand_logprobs) cand_logprobs[(size_t)b * topk + j] = lp;
            const double pj = exp(lp);
            c += pj;
            if (pj > 0.0) last_pos = j;
            if (pick < 0 && c > (double)uniform[b]) pick = j;
            const double d = fabs(c - (double)uniform[b]);
            if (d < margin) margin = d;
        }
        if (pick < 0) pick = last_pos;
        if (p->greedy) {
            pick = amax;
            margin = INFINITY;
        }
        next_token[b] = ix[pick];
        if (next_token_logprob) next_token_logprob[b] = x[pick] - lse;
        if (sample_margin) sample_margin[b] = margin;
        if (x != hs) free(x);
    }
    free(h);
    return 0;
}
