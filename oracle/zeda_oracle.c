/*
 * CPU oracle for one ZEDA MoE layer.  TEST INFRASTRUCTURE ONLY: the tests, the
 * smoke check and the benchmark's CPU-baseline leg call it; the product path
 * never does, and it shares no code with the HIP library.
 *
 * It is the definition written out, token by token, in double precision:
 *   - Section 2.1 ("Zero-Expert Injection"): a router scores N normal experts
 *     and N_Z zero experts; the top-K set S~(h) is taken over all N+N_Z; the
 *     layer output is Eq. 1,  y~(h) = sum_{i in S~(h), i normal} g~_i(h) E_i(h).
 *   - Section 4.3.4: the weights of the surviving normal experts are NOT
 *     renormalised after the zero experts are dropped (default); Eq. 7 is the
 *     renormalised ablation.
 *   - Appendix B: a copy expert returns its input, adding sum_{j zero} g~_j(h) h.
 *   - Appendix D, Eq. 9-10: an expert is a gate, an up and a down projection
 *     (6 H H_e FLOPs per token and expert); Eq. 14 and Eq. 18 are the
 *     whole-model FLOP ratios.
 *
 * Readings where the paper is silent (each listed in the design notes):
 *   - scores are a softmax over all N+N_Z logits; selection is on the logit
 *     rounded to fp32 (the precision the GPU kernel decides in), ties go to
 *     the lower index; slots are ordered by descending logit;
 *   - experts 0..N-1 are normal, N..N+N_Z-1 are zero experts (router rows of
 *     the zero experts are appended to the unchanged original rows);
 *   - gate_norm 0: g = softmax probability; 1 (default): g = p_i / sum of p
 *     over all K selected slots, zero experts included; 2: Eq. 7, p_i / sum of
 *     p over the selected normal experts;
 *   - the expert non-linearity is SwiGLU: W_down( silu(W_gate h) * (W_up h) );
 *   - an optional per-expert router bias is added to the logits (a device of
 *     the synthetic workloads; NULL gives the paper's router).
 *
 * No blocking, grouping or permutation: every token walks its own slots and
 * does three plain mat-vecs per normal expert.  OpenMP only spreads tokens over
 * cores; one token is always handled by one thread.
 *
 * Parity pins: see tests/test_oracle_pins.py (static top-K special case,
 * all-zero tokens, gate identities, FLOP count, the printed Table 13 values,
 * subset brute force, dense special case against numpy, copy-expert identity,
 * token-permutation and scaling invariants, stable-sort dispatch).
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

enum { GATE_SOFTMAX = 0, GATE_TOPK_NORM = 1, GATE_REAL_RENORM = 2 };

int oracle_num_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/* logits[e] = <x_t, W_r[e]> (+ bias[e]) for one token; Section 2.1 router over N+N_Z candidates. */
static void token_logits(const float *xt, const float *wr, const float *bias, int H, int NE, double *logit)
{
    for (int e = 0; e < NE; ++e) {
        double s = 0.0;
        const float *w = wr + (size_t)e * H;
        for (int h = 0; h < H; ++h) s += (double)xt[h] * (double)w[h];
        if (bias) s += (double)bias[e];
        logit[e] = s;
    }
}

/* Top-K set of Section 2.1 over all NE candidates, on fp32-rounded logits, lower index wins ties,
 * listed by descending logit; then the gates under the chosen normalisation. */
static void token_select(const double *logit, int N, int NE, int K, int gate_norm, int32_t *ids, double *gates,
                         char *taken)
{
    memset(taken, 0, (size_t)NE);
    for (int j = 0; j < K; ++j) {
        int best = -1;
        float bv = 0.f;
        for (int e = 0; e < NE; ++e) {
            if (taken[e]) continue;
            float v = (float)logit[e];
            if (best < 0 || v > bv) { best = e; bv = v; }
        }
        taken[best] = 1;
        ids[j] = best;
    }
    double mx = logit[0];
    for (int e = 1; e < NE; ++e) if (logit[e] > mx) mx = logit[e];
    double all = 0.0;
    for (int e = 0; e < NE; ++e) all += exp(logit[e] - mx);
    double denom = 1.0;
    if (gate_norm == GATE_TOPK_NORM) {
        denom = 0.0;
        for (int j = 0; j < K; ++j) denom += exp(logit[ids[j]] - mx) / all;
    } else if (gate_norm == GATE_REAL_RENORM) {
        denom = 0.0;
        for (int j = 0; j < K; ++j) if (ids[j] < N) denom += exp(logit[ids[j]] - mx) / all;
    }
    for (int j = 0; j < K; ++j) {
        double p = exp(logit[ids[j]] - mx) / all;
        gates[j] = (denom > 0.0) ? p / denom : 0.0;
    }
}

/* Router + selection for every token.  logits_out may be NULL. Returns 0, or -1 on bad arguments. */
int oracle_route(const float *x, const float *wr, const float *bias, int T, int H, int N, int Z, int K,
                 int gate_norm, int32_t *ids, double *gates, double *logits_out)
{
    const int NE = N + Z;
    if (T < 0 || H < 1 || N < 1 || Z < 0 || K < 1 || K > NE || gate_norm < 0 || gate_norm > 2) return -1;
#pragma omp parallel
    {
        double *logit = (double *)malloc(sizeof(double) * NE);
        char *taken = (char *)malloc((size_t)NE);
#pragma omp for schedule(static)
        for (int t = 0; t < T; ++t) {
            token_logits(x + (size_t)t * H, wr, bias, H, NE, logit);
            token_select(logit, N, NE, K, gate_norm, ids + (size_t)t * K, gates + (size_t)t * K, taken);
            if (logits_out) memcpy(logits_out + (size_t)t * NE, logit, sizeof(double) * NE);
        }
        free(logit);
        free(taken);
    }
    return 0;
}

/* Batch routing statistics of Section 2.2 (Eq. 4-6) for one layer, all tokens forming the batch B:
 *   f[i] = fraction of tokens whose top-K set holds expert i            (sums to K over i)
 *   P[i] = mean over tokens of the routing probability of expert i     (softmax over all N+Z logits; sums to 1)
 *   group sums f_E, P_E over the N normal experts and f_Z, P_Z over the Z zero experts,
 *   L_A  = alpha (N+Z)/K  sum_i f[i] P[i]                               (Eq. 4)
 *   L_GA = alpha (N+Z w)/K ( f_E P_E / N + f_Z P_Z / (Z w) )            (Eq. 5-6; the second term is dropped at Z = 0)
 *   r_ZE = f_Z / K.
 * summary[7] = {f_E, P_E, f_Z, P_Z, r_ZE, L_A, L_GA}.  Plain serial loops (the sums are over tokens). */
int oracle_routing_stats(const float *x, const float *wr, const float *bias, int T, int H, int N, int Z, int K,
                         double alpha, double w, double *f, double *P, double *summary)
{
    const int NE = N + Z;
    if (T < 1 || H < 1 || N < 1 || Z < 0 || K < 1 || K > NE || !(w > 0.0)) return -1;
    double *logit = (double *)malloc(sizeof(double) * NE);
    char *taken = (char *)malloc((size_t)NE);
    int32_t *ids = (int32_t *)malloc(sizeof(int32_t) * K);
    double *gates = (double *)malloc(sizeof(double) * K);
    for (int e = 0; e < NE; ++e) f[e] = P[e] = 0.0;
    for (int t = 0; t < T; ++t) {
        token_logits(x + (size_t)t * H, wr, bias, H, NE, logit);
        token_select(logit, N, NE, K, GATE_SOFTMAX, ids, gates, taken);
        for (int j = 0; j < K; ++j) f[ids[j]] += 1.0;
        double mx = logit[0];
        for (int e = 1; e < NE; ++e) if (logit[e] > mx) mx = logit[e];
        double all = 0.0;
        for (int e = 0; e < NE; ++e) all += exp(logit[e] - mx);
        for (int e = 0; e < NE; ++e) P[e] += exp(logit[e] - mx) / all;
    }
    double fE = 0.0, PE = 0.0, fZ = 0.0, PZ = 0.0, dot = 0.0;
    for (int e = 0; e < NE; ++e) {
        f[e] /= (double)T;
        P[e] /= (double)T;
        dot += f[e] * P[e];
        if (e < N) { fE += f[e]; PE += P[e]; } else { fZ += f[e]; PZ += P[e]; }
    }
    summary[0] = fE; summary[1] = PE; summary[2] = fZ; summary[3] = PZ;
    summary[4] = fZ / (double)K;
    summary[5] = alpha * (double)NE / (double)K * dot;
    summary[6] = alpha * ((double)N + (double)Z * w) / (double)K *
                 (fE * PE / (double)N + (Z > 0 ? fZ * PZ / ((double)Z * w) : 0.0));
    free(logit); free(taken); free(ids); free(gates);
    return 0;
}

/* Router rows of the Z zero experts (Section 2.1, "router initialization"): the N original rows stay as they
 * are; the new parameters are Gaussian with the mean and the (population) variance of the N*H original router
 * parameters.  The standard-normal draws are an input (normals[Z,H]), so that both sides of a parity test use
 * the same ones: rows[z,h] = mean + std * normals[z,h].  stats (may be NULL) receives {mean, variance}. */
int oracle_init_zero_rows(const float *wr, const float *normals, int N, int Z, int H, double *rows, double *stats)
{
    if (N < 1 || Z < 0 || H < 1) return -1;
    const size_t n = (size_t)N * H;
    double mean = 0.0, var = 0.0;
    for (size_t i = 0; i < n; ++i) mean += (double)wr[i];
    mean /= (double)n;
    for (size_t i = 0; i < n; ++i) var += ((double)wr[i] - mean) * ((double)wr[i] - mean);
    var /= (double)n;
    const double sd = sqrt(var);
    for (size_t i = 0; i < (size_t)Z * H; ++i) rows[i] = mean + sd * (double)normals[i];
    if (stats) { stats[0] = mean; stats[1] = var; }
    return 0;
}

/* One normal expert on one token (Appendix D: gate, up and down projections; SwiGLU reading):
 * y = W_down ( silu(W_gate h) * (W_up h) ).  act is scratch of I doubles. */
static void expert_apply(const float *xt, const float *wg, const float *wu, const float *wd, int H, int I,
                         double *act, double *y)
{
    for (int i = 0; i < I; ++i) {
        double g = 0.0, u = 0.0;
        const float *rg = wg + (size_t)i * H, *ru = wu + (size_t)i * H;
        for (int h = 0; h < H; ++h) {
            g += (double)rg[h] * (double)xt[h];
            u += (double)ru[h] * (double)xt[h];
        }
        act[i] = g / (1.0 + exp(-g)) * u;
    }
    for (int h = 0; h < H; ++h) {
        double s = 0.0;
        const float *rd = wd + (size_t)h * I;
        for (int i = 0; i < I; ++i) s += (double)rd[i] * act[i];
        y[h] = s;
    }
}

/* y = E_e(x_t) for a single (token row, expert) pair; exported for brute-force and stage tests. */
void oracle_expert(const float *xt, const float *wg_e, const float *wu_e, const float *wd_e, int H, int I, double *y)
{
    double *act = (double *)malloc(sizeof(double) * I);
    expert_apply(xt, wg_e, wu_e, wd_e, H, I, act, y);
    free(act);
}

/* Eq. 1 for every token.  ids[T,K], gates[T,K] are outputs as in oracle_route; out[T,H] double.
 * copy_expert != 0 adds Appendix B's copy term.  y_slot (may be NULL) receives the un-gated expert
 * output of every slot in token order, [T*K,H], zeros for zero-expert slots.
 * real_slots receives the number of (token, normal expert) pairs evaluated. */
int oracle_moe_forward(const float *x, const float *wr, const float *bias, const float *wg, const float *wu,
                       const float *wd, int T, int H, int I, int N, int Z, int K, int gate_norm, int copy_expert,
                       double *out, int32_t *ids, double *gates, double *y_slot, int64_t *real_slots)
{
    const int NE = N + Z;
    if (T < 0 || H < 1 || I < 1 || N < 1 || Z < 0 || K < 1 || K > NE || gate_norm < 0 || gate_norm > 2) return -1;
    int64_t total_real = 0;
#pragma omp parallel reduction(+ : total_real)
    {
        double *logit = (double *)malloc(sizeof(double) * NE);
        char *taken = (char *)malloc((size_t)NE);
        double *act = (double *)malloc(sizeof(double) * I);
        double *y = (double *)malloc(sizeof(double) * H);
#pragma omp for schedule(dynamic, 4)
        for (int t = 0; t < T; ++t) {
            const float *xt = x + (size_t)t * H;
            int32_t *tid = ids + (size_t)t * K;
            double *tg = gates + (size_t)t * K;
            double *o = out + (size_t)t * H;
            token_logits(xt, wr, bias, H, NE, logit);
            token_select(logit, N, NE, K, gate_norm, tid, tg, taken);
            for (int h = 0; h < H; ++h) o[h] = 0.0;
            for (int j = 0; j < K; ++j) {
                double *ys = y_slot ? y_slot + ((size_t)t * K + j) * H : NULL;
                int e = tid[j];
                if (e < N) { /* normal expert: the only terms Eq. 1 keeps */
                    expert_apply(xt, wg + (size_t)e * I * H, wu + (size_t)e * I * H, wd + (size_t)e * H * I, H, I,
                                 act, y);
                    for (int h = 0; h < H; ++h) o[h] += tg[j] * y[h];
                    if (ys) memcpy(ys, y, sizeof(double) * H);
                    total_real += 1;
                } else {     /* zero expert: Z_j(h) = 0, no computation */
                    if (ys) memset(ys, 0, sizeof(double) * H);
                    if (copy_expert) for (int h = 0; h < H; ++h) o[h] += tg[j] * (double)xt[h];
                }
            }
        }
        free(logit); free(taken); free(act); free(y);
    }
    if (real_slots) *real_slots = total_real;
    return 0;
}

/* Expert-sorted order of the normal-expert slots: the (expert, token, slot-rank) triples in
 * lexicographic order.  offsets[N+1], sorted_slot[T*K] (first offsets[N] entries valid, value t*K+j),
 * slot_to_row[T*K] (-1 for zero-expert slots). */
void oracle_dispatch(const int32_t *ids, int T, int K, int N, int32_t *offsets, int32_t *sorted_slot,
                     int32_t *slot_to_row)
{
    const int64_t S = (int64_t)T * K;
    int32_t row = 0;
    for (int64_t s = 0; s < S; ++s) { sorted_slot[s] = -1; slot_to_row[s] = -1; }
    for (int e = 0; e < N; ++e) {
        offsets[e] = row;
        for (int64_t s = 0; s < S; ++s) {
            if (ids[s] == e) { sorted_slot[row] = (int32_t)s; slot_to_row[s] = row; ++row; }
        }
    }
    offsets[N] = row;
}

/* Eq. 1's sum given per-slot expert outputs in expert-sorted rows (a stage check for the combine):
 * out[t] = sum_j [ids[t,j] < N] gates[t,j] * y_rows[slot_to_row[t*K+j]]. */
void oracle_combine(const double *y_rows, const int32_t *ids, const double *gates, const int32_t *slot_to_row, int T,
                    int H, int N, int K, double *out)
{
    for (int t = 0; t < T; ++t) {
        double *o = out + (size_t)t * H;
        for (int h = 0; h < H; ++h) o[h] = 0.0;
        for (int j = 0; j < K; ++j) {
            if (ids[(size_t)t * K + j] >= N) continue;
            const double *y = y_rows + (size_t)slot_to_row[(size_t)t * K + j] * H;
            for (int h = 0; h < H; ++h) o[h] += gates[(size_t)t * K + j] * y[h];
        }
    }
}

/* Pre-norm of the layer-stack workload (not part of the paper's layer, whose model leaves norms out, Appendix D):
 * out[t,:] = x[t,:] / sqrt(mean_h x[t,h]^2 + eps) * gamma[h]   (gamma may be NULL = 1). */
void oracle_rmsnorm(const double *x, const double *gamma, int T, int H, double eps, double *out)
{
    for (int t = 0; t < T; ++t) {
        double ss = 0.0;
        for (int h = 0; h < H; ++h) ss += x[(size_t)t * H + h] * x[(size_t)t * H + h];
        const double scale = 1.0 / sqrt(ss / H + eps);
        for (int h = 0; h < H; ++h) out[(size_t)t * H + h] = x[(size_t)t * H + h] * scale * (gamma ? gamma[h] : 1.0);
    }
}

/* Appendix D, Eq. 9 / Eq. 10: MoE-branch FLOPs for n tokens (r_ze = 0 and nz = 0 give the original model). */
double oracle_moe_flops(double n, double H, double He, double N, double NZ, double K, double r_ze)
{
    return 6.0 * (1.0 - r_ze) * K * n * H * He + 2.0 * (N + NZ) * n * H;
}

/* Appendix D, Eq. 14 (prefill != 0) and Eq. 18 (decode): F_ZEDA / F_orig at sequence length l. */
double oracle_flop_ratio(int prefill, double l, double H, double Hattn, double gkv, double He, double N, double NZ,
                         double K, double r_ze)
{
    double attn = (prefill ? 2.0 * l : (l - 1.0)) * Hattn + 2.0 * (1.0 + gkv) * H * Hattn;
    double zeda = attn + 3.0 * (1.0 - r_ze) * K * H * He + (N + NZ) * H;
    double orig = attn + 3.0 * K * H * He + N * H;
    return zeda / orig;
}
