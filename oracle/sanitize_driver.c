/*
 * Stand-alone driver of the CPU oracle for sanitizer runs.  TEST INFRASTRUCTURE ONLY.
 *
 * Compiled together with moe_oracle.c under -fsanitize=address,undefined (an executable of its
 * own, so nothing has to be preloaded into another process).  It reads one case from a file,
 * runs every oracle function on it in the order of the layer (route -> plan -> dispatch -> expert
 * FFN -> combine, then the SRU predictor), and writes every output to a second file, which the
 * test compares bit for bit with what the ordinary build of the oracle returns for the same case.
 * It holds no arithmetic of the method.
 *
 * Input file: 16 int32 {T, d, F, E, C, R, st, policy, residual, B, L, n_layers, n_in, n_h, n_out, 0}
 * followed by x[T*d], wr[d*E] (storage type st), b[E] (float), w1[E*d*F], w2[E*F*d], emb[B*L*n_in],
 * per layer w_cat[n_in_l * k_l * n_h], b_f[n_h], b_r[n_h] (float), then w_head[n_h*n_out], b_head[n_out].
 * Output file, in this order: idx, prob, counts, replicas, slot_base, slot_expert, n_slots, kept,
 * expert_offset, slot_offset, perm, inv, h, y_perm, out, pred, sru_h.
 */
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>

int orc_route(const void *, const void *, const float *, int, int, int, int, int32_t *, float *, double *,
              int32_t *, double *);
int orc_sru(const void *, int, int, int, int, int, int, const void *const *, const float *const *,
            const float *const *, const void *, const float *, int, int32_t *, double *, int32_t *, double *,
            void *);
int orc_plan(const int32_t *, int, int, int, int, int, int32_t *, int32_t *, int32_t *, int32_t *, int32_t *);
int orc_dispatch(const void *, const int32_t *, const int32_t *, int, int, int, int, int, int, int32_t *,
                 int32_t *, int32_t *, int32_t *, int32_t *, int32_t *, void *);
int orc_ffn(const void *, const void *, const void *, const int32_t *, const int32_t *, int, int, int, int,
            const int32_t *, int, void *, void *);
int orc_combine(const void *, const void *, const int32_t *, const float *, int, int, int, int, void *);

static void *rd(FILE *f, size_t n, size_t esz)
{
    /* exact-size heap blocks: an access one element past any tensor is an error the sanitizer reports */
    void *p = malloc(n * esz ? n * esz : 1);
    if (!p || fread(p, esz, n, f) != n) {
        fprintf(stderr, "sanitize_driver: short input\n");
        exit(3);
    }
    return p;
}

static void *out_buf(size_t n, size_t esz) { return calloc(n * esz ? n * esz : 1, 1); }

static void wr(FILE *f, const void *p, size_t n, size_t esz)
{
    if (fwrite(p, esz, n, f) != n) {
        fprintf(stderr, "sanitize_driver: short output\n");
        exit(4);
    }
}

#define MUST(call)                                                 \
    do {                                                           \
        if ((call) != 0) {                                         \
            fprintf(stderr, "sanitize_driver: %s failed\n", #call); \
            exit(5);                                               \
        }                                                          \
    } while (0)

int main(int argc, char **argv)
{
    if (argc != 3) {
        fprintf(stderr, "usage: %s case.bin result.bin\n", argv[0]);
        return 2;
    }
    FILE *in = fopen(argv[1], "rb"), *out = fopen(argv[2], "wb");
    if (!in || !out)
        return 2;
    int32_t *hd = rd(in, 16, 4);
    const int T = hd[0], d = hd[1], F = hd[2], E = hd[3], C = hd[4], R = hd[5], st = hd[6], policy = hd[7],
              residual = hd[8], B = hd[9], L = hd[10], n_layers = hd[11], n_in = hd[12], n_h = hd[13],
              n_out = hd[14];
    const size_t esz = st == 0 ? 4 : 2;
    void *x = rd(in, (size_t)T * d, esz), *wrt = rd(in, (size_t)d * E, esz);
    float *b = rd(in, E, 4);
    void *w1 = rd(in, (size_t)E * d * F, esz), *w2 = rd(in, (size_t)E * F * d, esz);
    void *emb = rd(in, (size_t)B * L * n_in, esz);
    const void **w_cat = malloc(sizeof(void *) * (n_layers ? n_layers : 1));
    const float **b_f = malloc(sizeof(float *) * (n_layers ? n_layers : 1));
    const float **b_r = malloc(sizeof(float *) * (n_layers ? n_layers : 1));
    for (int l = 0; l < n_layers; ++l) {
        const int nin = l == 0 ? n_in : n_h, k = nin == n_h ? 3 : 4;
        w_cat[l] = rd(in, (size_t)nin * k * n_h, esz);
        b_f[l] = rd(in, n_h, 4);
        b_r[l] = rd(in, n_h, 4);
    }
    void *w_head = rd(in, (size_t)n_h * n_out, esz);
    float *b_head = rd(in, n_out, 4);

    /* the layer */
    int32_t *idx = out_buf(T, 4);
    float *prob = out_buf(T, 4);
    MUST(orc_route(x, wrt, b, T, d, E, st, idx, prob, NULL, NULL, NULL));
    int32_t *counts = out_buf(E, 4), *replicas = out_buf(E, 4), *slot_base = out_buf(E + 1, 4),
            *slot_expert = out_buf(E + R, 4), n_slots[1] = {0};
    for (int p = 0; p < E + R; ++p)
        slot_expert[p] = -1;
    MUST(orc_plan(idx, T, E, R, C, policy, counts, replicas, slot_base, slot_expert, n_slots));
    int32_t *dcounts = out_buf(E, 4), *kept = out_buf(E, 4), *expert_offset = out_buf(E + 1, 4),
            *slot_offset = out_buf(E + R + 1, 4), *perm = out_buf(T, 4), *inv = out_buf(T, 4);
    void *x_perm = out_buf((size_t)T * d, esz);
    MUST(orc_dispatch(x, idx, replicas, T, d, E, C, E + R, st, dcounts, kept, expert_offset, slot_offset, perm,
                      inv, x_perm));
    void *h = out_buf((size_t)T * F, esz), *y = out_buf((size_t)T * d, esz), *res = out_buf((size_t)T * d, esz);
    MUST(orc_ffn(x_perm, w1, w2, slot_offset, slot_expert, n_slots[0], d, F, st, NULL, 0, y, h));
    MUST(orc_combine(y, x, inv, prob, T, d, st, residual, res));
    wr(out, idx, T, 4);
    wr(out, prob, T, 4);
    wr(out, counts, E, 4);
    wr(out, replicas, E, 4);
    wr(out, slot_base, E + 1, 4);
    wr(out, slot_expert, E + R, 4);
    wr(out, n_slots, 1, 4);
    wr(out, kept, E, 4);
    wr(out, expert_offset, E + 1, 4);
    wr(out, slot_offset, E + R + 1, 4);
    wr(out, perm, T, 4);
    wr(out, inv, T, 4);
    wr(out, h, (size_t)T * F, esz);
    wr(out, y, (size_t)T * d, esz);
    wr(out, res, (size_t)T * d, esz);

    /* the predictor */
    int32_t *pred = out_buf((size_t)B * L, 4);
    void *sru_h = out_buf((size_t)B * L * n_h, esz);
    if (n_layers > 0)
        MUST(orc_sru(emb, B, L, n_layers, n_in, n_h, n_out, w_cat, b_f, b_r, w_head, b_head, st, pred, NULL, NULL,
                     NULL, sru_h));
    wr(out, pred, (size_t)B * L, 4);
    wr(out, sru_h, (size_t)B * L * n_h, esz);
    fclose(in);
    fclose(out);
    /* everything is freed so that the leak check of the sanitizer speaks about the oracle only */
    for (int l = 0; l < n_layers; ++l) {
        free((void *)w_cat[l]);
        free((void *)b_f[l]);
        free((void *)b_r[l]);
    }
    void *all[] = {hd, x, wrt, b, w1, w2, emb, w_cat, b_f, b_r, w_head, b_head, idx, prob, counts, replicas,
                   slot_base, slot_expert, dcounts, kept, expert_offset, slot_offset, perm, inv, x_perm, h, y, res,
                   pred, sru_h};
    for (size_t i = 0; i < sizeof(all) / sizeof(all[0]); ++i)
        free(all[i]);
    return 0;
}
