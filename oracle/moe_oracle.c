/*
 * CPU oracle for the replicated top-1 MoE layer forward.  TEST INFRASTRUCTURE ONLY.
 *
 * A plain, slow, obviously-correct evaluation of what the hot path computes, written from the
 * paper: the Switch-style top-1 layer the paper's Methodology section runs, the replication pass of Algorithm 1, the capping heuristic
 * of the "Capacity capping" subsection, and the SRU equations of the "Simple Recurrent Unit
 * for expert prediction" subsection.  It shares no code with the GPU library and must never
 * be called from the product path: only the tests, the smoke check and the bench's CPU
 * baseline leg may load it.
 *
 * Arithmetic: every sum, exponential, sigmoid and tanh is evaluated in double.  Values are
 * rounded only where the interface stores them: a tensor of storage type 0 is binary32, of
 * storage type 1 is bf16 (upper half of binary32, round to nearest even), kept as uint16.
 * There is no blocking, fusion or reordering: each function is the definition written out,
 * reductions run in ascending index order.  OpenMP, when enabled, splits independent
 * tokens / rows / sequences across threads and nothing else.
 *
 * Pins (tests/test_oracle_*.py): the paper's printed replication scenario (64 tokens, 64
 * experts, two active experts -> 32 replicas each), Algorithm 1's closed form r_e = n_e at
 * slot capacity 1, plan invariants, a per-token brute force written separately in Python,
 * dense-library special cases (E = 1 reduces to relu(X W1) W2), SRU limiting cases and the
 * unrolled closed form of the c_t recurrence.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#define ORC_OK 0
#define ORC_BAD -1

/* ------------------------------------------------------------------ storage <-> double */
static double ld(const void *p, size_t i, int st)
{
    if (st == 0)
        return (double)((const float *)p)[i];
    uint32_t u = (uint32_t)((const uint16_t *)p)[i] << 16;
    float f;
    memcpy(&f, &u, 4);
    return (double)f;
}

/* nearest bf16 (8 significant bits, binary32 exponent range), ties to even, from a double */
static double round_bf16(double v)
{
    if (v == 0.0 || !isfinite(v))
        return v;
    int e;
    (void)frexp(v, &e);          /* |v| = m * 2^e, m in [0.5, 1) */
    int qe = e - 8;              /* quantum 2^qe keeps 8 significant bits */
    if (qe < -133)
        qe = -133;               /* subnormal range of the format */
    return ldexp(rint(ldexp(v, -qe)), qe); /* rint: current mode = nearest even */
}

static void st_(void *p, size_t i, int st, double v)
{
    if (st == 0) {
        ((float *)p)[i] = (float)v;
    } else {
        float f = (float)round_bf16(v); /* exact: the rounded value is a binary32 */
        uint32_t u;
        memcpy(&u, &f, 4);
        ((uint16_t *)p)[i] = (uint16_t)(u >> 16);
    }
}

/* ------------------------------------------------------------------ router
 * Top-1 softmax router of the Switch-style layer (Methodology; Preliminaries on softmax
 * routing).  logit[s][e] = sum_k x[s][k]*Wr[k][e] + b[e]; idx = argmax (lowest index on a
 * tie); prob = softmax(logit[s])[idx] = 1 / sum_j exp(logit_j - logit_idx).
 * Also returns the runner-up id and the top-2 gap, which the parity tests use to recognise
 * tokens whose argmax is decided inside float rounding noise.
 */
int orc_route(const void *x, const void *wr, const float *b, int T, int d, int E, int st,
              int32_t *idx, float *prob, double *logits_opt, int32_t *idx2_opt,
              double *margin_opt)
{
    if (!x || !wr || !idx || !prob || T < 0 || d <= 0 || E <= 0)
        return ORC_BAD;
#pragma omp parallel for schedule(static)
    for (int s = 0; s < T; ++s) {
        double *l = (double *)malloc(sizeof(double) * (size_t)E);
        for (int e = 0; e < E; ++e) {
            double acc = 0.0;
            for (int k = 0; k < d; ++k)
                acc += ld(x, (size_t)s * d + k, st) * ld(wr, (size_t)k * E + e, st);
            l[e] = acc + (b ? (double)b[e] : 0.0);
        }
        int best = 0;
        for (int e = 1; e < E; ++e)
            if (l[e] > l[best])
                best = e;
        int second = -1;
        for (int e = 0; e < E; ++e)
            if (e != best && (second < 0 || l[e] > l[second]))
                second = e;
        double z = 0.0;
        for (int e = 0; e < E; ++e)
            z += exp(l[e] - l[best]);
        idx[s] = best;
        prob[s] = (float)(1.0 / z);
        if (idx2_opt)
            idx2_opt[s] = second;
        if (margin_opt)
            margin_opt[s] = second >= 0 ? l[best] - l[second] : INFINITY;
        if (logits_opt)
            memcpy(logits_opt + (size_t)s * E, l, sizeof(double) * (size_t)E);
        free(l);
    }
    return ORC_OK;
}

/* ------------------------------------------------------------------ SRU predictor
 * Equations of the SRU subsection, per layer and time step t of each sequence:
 *   x'_t = W x_t;  f_t = sigma(W_f x_t + b_f);  r_t = sigma(W_r x_t + b_r);
 *   c_t = f_t * c_{t-1} + (1 - f_t) * x'_t,  c_{-1} = 0 at the start of every sequence;
 *   h_t = r_t * tanh(c_t) + (1 - r_t) * x_t.
 * When the layer's input width differs from its hidden width the highway term uses a fourth
 * projection W_h x_t in place of x_t.  w_cat[l] is [n_in_l, k*n_h] with column blocks
 * W | W_f | W_r | (W_h).  Each layer's output is stored in the activation storage type.
 * A linear head gives logits = h W_head + b_head; the prediction is the argmax (the step
 * "Expert k <- h_l(X_i[s])" of Algorithm 2).
 */
static double sigmoid(double v) { return 1.0 / (1.0 + exp(-v)); }

int orc_sru(const void *emb, int B, int L, int n_layers, int n_in, int n_h, int n_out,
            const void *const *w_cat, const float *const *b_f, const float *const *b_r,
            const void *w_head, const float *b_head, int st, int32_t *pred,
            double *logits_opt, int32_t *idx2_opt, double *margin_opt, void *h_out_opt)
{
    if (!emb || !w_cat || !w_head || !pred || B < 0 || L <= 0 || n_layers <= 0)
        return ORC_BAD;
    size_t Tt = (size_t)B * L;
    size_t esz = st == 0 ? 4 : 2;
    int wmax = n_in > n_h ? n_in : n_h;
    void *cur = malloc(Tt * (size_t)wmax * esz + 16);
    void *nxt = malloc(Tt * (size_t)wmax * esz + 16);
    memcpy(cur, emb, Tt * (size_t)n_in * esz);
    int nin = n_in;
    for (int l = 0; l < n_layers; ++l) {
        int k = nin == n_h ? 3 : 4;
        int ncol = k * n_h;
        const void *w = w_cat[l];
        const float *bf = b_f ? b_f[l] : NULL, *br = b_r ? b_r[l] : NULL;
#pragma omp parallel for schedule(static)
        for (int b = 0; b < B; ++b) {
            double *c = (double *)calloc((size_t)n_h, sizeof(double));
            double *u = (double *)malloc(sizeof(double) * (size_t)ncol);
            for (int t = 0; t < L; ++t) {
                size_t row = (size_t)b * L + t;
                for (int j = 0; j < ncol; ++j) {
                    double acc = 0.0;
                    for (int q = 0; q < nin; ++q)
                        acc += ld(cur, row * nin + q, st) * ld(w, (size_t)q * ncol + j, st);
                    u[j] = acc;
                }
                for (int j = 0; j < n_h; ++j) {
                    double f = sigmoid(u[n_h + j] + (bf ? (double)bf[j] : 0.0));
                    double r = sigmoid(u[2 * n_h + j] + (br ? (double)br[j] : 0.0));
                    c[j] = f * c[j] + (1.0 - f) * u[j];
                    double hw = k == 4 ? u[3 * n_h + j] : ld(cur, row * nin + j, st);
                    st_(nxt, row * n_h + j, st, r * tanh(c[j]) + (1.0 - r) * hw);
                }
            }
            free(c);
            free(u);
        }
        void *tmp = cur;
        cur = nxt;
        nxt = tmp;
        nin = n_h;
    }
    if (h_out_opt)
        memcpy(h_out_opt, cur, Tt * (size_t)n_h * esz);
#pragma omp parallel for schedule(static)
    for (long s = 0; s < (long)Tt; ++s) {
        double *lg = (double *)malloc(sizeof(double) * (size_t)n_out);
        for (int o = 0; o < n_out; ++o) {
            double acc = 0.0;
            for (int q = 0; q < n_h; ++q)
                acc += ld(cur, (size_t)s * n_h + q, st) * ld(w_head, (size_t)q * n_out + o, st);
            lg[o] = acc + (b_head ? (double)b_head[o] : 0.0);
        }
        int best = 0;
        for (int o = 1; o < n_out; ++o)
            if (lg[o] > lg[best])
                best = o;
        int second = -1;
        for (int o = 0; o < n_out; ++o)
            if (o != best && (second < 0 || lg[o] > lg[second]))
                second = o;
        pred[s] = best;
        if (idx2_opt)
            idx2_opt[s] = second;
        if (margin_opt)
            margin_opt[s] = second >= 0 ? lg[best] - lg[second] : INFINITY;
        if (logits_opt)
            memcpy(logits_opt + (size_t)s * n_out, lg, sizeof(double) * (size_t)n_out);
        free(lg);
    }
    free(cur);
    free(nxt);
    return ORC_OK;
}

/* ------------------------------------------------------------------ replica plan
 * Algorithm 1's replication pass with the cap of the "Capacity capping" subsection.
 *   n_e    = tokens whose (predicted or exact) id is e.
 *   want_e = extra physical slots expert e would get from Algorithm 1 if every slot holds at
 *            most C tokens: ceil(n_e / C) - 1 (C = 1 is the algorithm as printed: one
 *            replica per further token).
 *   Every expert owns one slot (Capacity capping subsection: no distinct expert's count falls
 *   below one; all experts stay resident here).  If the wanted extras D = sum want_e fit in the budget R
 *   they are all granted.  Otherwise the remaining space is divided by the count of replicas
 *   still to be added and the limits raised accordingly:
 *     policy 0: extra_e = floor(R * want_e / D); the < |wanting| slots that the floors leave
 *               go one at a time to the expert with the largest load per slot n_e / r_e
 *               among those still short of their want (ties: lowest id);
 *     policy 1: equal shares: repeatedly give every still-wanting expert
 *               min(floor(R_left / |wanting|), unmet); the final remainder as in policy 0.
 *   slot_base = exclusive scan of r_e; slots are numbered expert-major.
 */
static int most_loaded(const int32_t *n, const int32_t *r, const int64_t *want, int E)
{
    int best = -1;
    for (int e = 0; e < E; ++e) {
        if ((int64_t)r[e] - 1 >= want[e])
            continue;
        if (best < 0 || (int64_t)n[e] * r[best] > (int64_t)n[best] * r[e])
            best = e;
    }
    return best;
}

int orc_plan(const int32_t *idx, int T, int E, int R, int C, int policy, int32_t *counts,
             int32_t *replicas, int32_t *slot_base, int32_t *slot_expert, int32_t *n_slots)
{
    if (!idx || !counts || !replicas || T < 0 || E <= 0 || R < 0 || C < 1 ||
        (policy != 0 && policy != 1))
        return ORC_BAD;
    for (int e = 0; e < E; ++e)
        counts[e] = 0;
    for (int s = 0; s < T; ++s) {
        if (idx[s] < 0 || idx[s] >= E)
            return ORC_BAD;
        counts[idx[s]]++;
    }
    int64_t *want = (int64_t *)malloc(sizeof(int64_t) * (size_t)E);
    int64_t D = 0;
    for (int e = 0; e < E; ++e) {
        replicas[e] = 1;
        int64_t w = ((int64_t)counts[e] + C - 1) / C - 1;
        want[e] = w > 0 ? w : 0;
        D += want[e];
    }
    if (D <= R) {
        for (int e = 0; e < E; ++e)
            replicas[e] += (int32_t)want[e];
    } else {
        int64_t left = R;
        if (policy == 0) {
            for (int e = 0; e < E; ++e) {
                int64_t extra = (int64_t)R * want[e] / D;
                replicas[e] += (int32_t)extra;
                left -= extra;
            }
        } else {
            for (;;) {
                int64_t nw = 0;
                for (int e = 0; e < E; ++e)
                    nw += (int64_t)replicas[e] - 1 < want[e];
                if (nw == 0)
                    break;
                int64_t q = left / nw;
                if (q == 0)
                    break;
                for (int e = 0; e < E; ++e) {
                    int64_t unmet = want[e] - ((int64_t)replicas[e] - 1);
                    if (unmet <= 0)
                        continue;
                    int64_t g = q < unmet ? q : unmet;
                    replicas[e] += (int32_t)g;
                    left -= g;
                }
            }
        }
        while (left > 0) {
            int e = most_loaded(counts, replicas, want, E);
            if (e < 0)
                break;
            replicas[e] += 1;
            left -= 1;
        }
    }
    free(want);
    int32_t base = 0;
    for (int e = 0; e < E; ++e) {
        if (slot_base)
            slot_base[e] = base;
        if (slot_expert)
            for (int k = 0; k < replicas[e]; ++k)
                slot_expert[base + k] = e;
        base += replicas[e];
    }
    if (slot_base)
        slot_base[E] = base;
    if (n_slots)
        *n_slots = base;
    return ORC_OK;
}

/* ------------------------------------------------------------------ dispatch
 * Capacity-limited token dispatch of the specialised model (Algorithm 1: tokens are
 * re-pointed to physical replicas, each of which is an ordinary Switch expert holding at
 * most C tokens; "parallel processing of tokens is maintained as long as the batch size
 * remains within the capacity of the experts loaded onto the GPU").
 *   j(s)     = number of earlier tokens with the same expert (stable rank);
 *   kept     iff j(s) < r_e * C;   kept_e = min(n_e, r_e*C);
 *   expert_offset = exclusive scan of kept_e;   position(s) = expert_offset[e] + j(s);
 *   perm[position] = s,  inv[s] = position or -1;  x_perm[position] = x[s];
 *   the kept rows of e are cut into r_e contiguous slots whose sizes differ by at most one,
 *   larger first: slot k holds q + (k < rem) rows, q = kept_e div r_e, rem = kept_e mod r_e.
 * replicas == NULL means r_e = 1 for every expert.  slot_offset has max_slots+1 entries;
 * entries past the last slot hold K (the number of kept tokens).
 */
int orc_dispatch(const void *x, const int32_t *idx, const int32_t *replicas, int T, int d,
                 int E, int C, int max_slots, int st, int32_t *counts, int32_t *kept,
                 int32_t *expert_offset, int32_t *slot_offset, int32_t *perm, int32_t *inv,
                 void *x_perm)
{
    if (!idx || !counts || !kept || !expert_offset || !perm || !inv || T < 0 || E <= 0 ||
        C < 1 || d < 0)
        return ORC_BAD;
    int64_t P = 0;
    for (int e = 0; e < E; ++e) {
        int r = replicas ? replicas[e] : 1;
        if (r < 1)
            return ORC_BAD;
        P += r;
        counts[e] = 0;
    }
    if (slot_offset && P > max_slots)
        return ORC_BAD;
    for (int s = 0; s < T; ++s) {
        if (idx[s] < 0 || idx[s] >= E)
            return ORC_BAD;
        counts[idx[s]]++;
    }
    int32_t off = 0;
    for (int e = 0; e < E; ++e) {
        int64_t cap = (int64_t)(replicas ? replicas[e] : 1) * C;
        kept[e] = counts[e] < cap ? counts[e] : (int32_t)cap;
        expert_offset[e] = off;
        off += kept[e];
    }
    expert_offset[E] = off;
    if (slot_offset) {
        int p = 0;
        for (int e = 0; e < E; ++e) {
            int r = replicas ? replicas[e] : 1;
            int q = kept[e] / r, rem = kept[e] % r;
            int32_t o = expert_offset[e];
            for (int k = 0; k < r; ++k) {
                slot_offset[p++] = o;
                o += q + (k < rem);
            }
        }
        for (; p <= max_slots; ++p)
            slot_offset[p] = off;
    }
    int32_t *seen = (int32_t *)calloc((size_t)E, sizeof(int32_t));
    size_t esz = st == 0 ? 4 : 2;
    for (int s = 0; s < T; ++s) {
        int e = idx[s];
        int32_t j = seen[e]++;
        if (j < kept[e]) {
            int32_t pos = expert_offset[e] + j;
            perm[pos] = s;
            inv[s] = pos;
            if (x && x_perm)
                memcpy((char *)x_perm + (size_t)pos * d * esz, (const char *)x + (size_t)s * d * esz,
                       (size_t)d * esz);
        } else {
            inv[s] = -1;
        }
    }
    for (int i = off; i < T; ++i)
        perm[i] = -1;
    free(seen);
    return ORC_OK;
}

/* ------------------------------------------------------------------ expert FFN
 * The Switch-base expert applied to the rows of each slot: for a row in slot p, with
 * e = slot_expert[p]:  h = relu(x_perm[row] W1[e]) stored in the activation type, then
 * y_perm[row] = h W2[e] stored in the activation type.  W1 is [E, d, F], W2 is [E, F, d],
 * row-major.  rows_sel (optional) restricts the evaluation to the listed rows; other rows
 * of y_perm are left untouched.  h_opt (optional) receives h for the evaluated rows.
 */
int orc_ffn(const void *x_perm, const void *w1, const void *w2, const int32_t *slot_offset,
            const int32_t *slot_expert, int n_slots, int d, int F, int st,
            const int32_t *rows_sel, int n_sel, void *y_perm, void *h_opt)
{
    if (!x_perm || !w1 || !w2 || !slot_offset || !slot_expert || !y_perm || n_slots < 0)
        return ORC_BAD;
    int K = n_slots > 0 ? slot_offset[n_slots] : 0;
    int n = rows_sel ? n_sel : K;
    int bad = 0;
#pragma omp parallel for schedule(dynamic, 1)
    for (int i = 0; i < n; ++i) {
        int row = rows_sel ? rows_sel[i] : i;
        int p = -1;
        for (int q = 0; q < n_slots; ++q)
            if (row >= slot_offset[q] && row < slot_offset[q + 1])
                p = q;
        if (row < 0 || p < 0) {
            bad = 1;
            continue;
        }
        size_t e = (size_t)slot_expert[p];
        double *h = (double *)calloc((size_t)F, sizeof(double));
        double *y = (double *)calloc((size_t)d, sizeof(double));
        for (int k = 0; k < d; ++k) {
            double xk = ld(x_perm, (size_t)row * d + k, st);
            for (int f = 0; f < F; ++f)
                h[f] += xk * ld(w1, (e * d + k) * F + f, st);
        }
        for (int f = 0; f < F; ++f) {
            double v = h[f] > 0.0 ? h[f] : 0.0;
            v = st == 0 ? (double)(float)v : round_bf16(v);
            h[f] = v;
            if (h_opt)
                st_(h_opt, (size_t)row * F + f, st, v);
        }
        for (int f = 0; f < F; ++f)
            for (int j = 0; j < d; ++j)
                y[j] += h[f] * ld(w2, (e * F + f) * d + j, st);
        for (int j = 0; j < d; ++j)
            st_(y_perm, (size_t)row * d + j, st, y[j]);
        free(h);
        free(y);
    }
    return bad ? ORC_BAD : ORC_OK;
}

/* ------------------------------------------------------------------ combine
 * Kept token s (inv[s] >= 0): out[s] = (residual ? x[s] : 0) + prob[s] * y_perm[inv[s]],
 * rounded once to the activation type.  Dropped token: out[s] = x[s], bit for bit (tokens
 * over capacity pass through unchanged).
 */
int orc_combine(const void *y_perm, const void *x, const int32_t *inv, const float *prob,
                int T, int d, int st, int residual, void *out)
{
    if (!y_perm || !x || !inv || !prob || !out || T < 0 || d <= 0)
        return ORC_BAD;
    size_t esz = st == 0 ? 4 : 2;
#pragma omp parallel for schedule(static)
    for (int s = 0; s < T; ++s) {
        if (inv[s] < 0) {
            memcpy((char *)out + (size_t)s * d * esz, (const char *)x + (size_t)s * d * esz,
                   (size_t)d * esz);
            continue;
        }
        for (int j = 0; j < d; ++j) {
            double v = (double)prob[s] * ld(y_perm, (size_t)inv[s] * d + j, st);
            if (residual)
                v += ld(x, (size_t)s * d + j, st);
            st_(out, (size_t)s * d + j, st, v);
        }
    }
    return ORC_OK;
}

int orc_num_threads(void)
{
#ifdef _OPENMP
    extern int omp_get_max_threads(void);
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/* Timing only (the serial leg of the CPU baseline): the number of threads the parallel loops use. */
int orc_set_num_threads(int n)
{
#ifdef _OPENMP
    extern void omp_set_num_threads(int);
    if (n >= 1) omp_set_num_threads(n);
#endif
    return orc_num_threads();
}
