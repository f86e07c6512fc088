/* Test driver: runs the C oracle's entry points on a batch read from a binary file and writes
 * what they return to another, so that a build with -fsanitize=address,undefined can be compared
 * bit for bit with the ordinary build.  Test infrastructure only.
 *
 * Input (little endian): int32 D, H, L, k, group, single, B, n_tot, e_tot; int64 n_weights;
 * int32 n_nodes[B], n_edges[B], src[e_tot], dst[e_tot], placement[n_tot], cur[B];
 * double feats[n_tot * 3], weights[n_weights] (n_weights = 0: only levels and sets are computed).
 * Output: int32 status of every call, then int32 td[n_tot], bu[n_tot]; uint8 cls[n_tot];
 * double logits[B * D], probs[B * D], emb[n_tot * 2H], pooled[B * 3 * G * H]. */
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>

typedef struct { int32_t D, H, n_layers, k_sweeps, group_by_device, single_set; } orc_cfg;
size_t orc_weight_count(const orc_cfg *c);
int orc_levels(int32_t n, int32_t n_edges, const int32_t *src, const int32_t *dst, int32_t *td, int32_t *bu);
int orc_classes(int32_t n, int32_t n_edges, const int32_t *src, const int32_t *dst, int32_t cur, uint8_t *cls);
int orc_forward_batch(const orc_cfg *c, int32_t B, const int32_t *n_nodes, const int32_t *n_edges,
                      const int32_t *src, const int32_t *dst, const double *feats, const int32_t *placement,
                      const int32_t *cur, const double *weights, double *logits, double *probs, double *emb,
                      double *pooled, int32_t n_threads);

static void *take(FILE *f, size_t bytes)
{
    void *p = malloc(bytes ? bytes : 1);
    if (!p || fread(p, 1, bytes, f) != bytes) { fprintf(stderr, "short read\n"); exit(2); }
    return p;
}

int main(int argc, char **argv)
{
    if (argc != 3) { fprintf(stderr, "usage: %s in out\n", argv[0]); return 2; }
    FILE *f = fopen(argv[1], "rb");
    if (!f) return 2;
    int32_t *hd = take(f, 9 * sizeof(int32_t));
    int64_t *nw = take(f, sizeof(int64_t));
    const orc_cfg cfg = {hd[0], hd[1], hd[2], hd[3], hd[4], hd[5]};
    const int32_t B = hd[6], n_tot = hd[7], e_tot = hd[8];
    const int32_t G = cfg.group_by_device ? cfg.D : 1;
    int32_t *n_nodes = take(f, sizeof(int32_t) * (size_t)B), *n_edges = take(f, sizeof(int32_t) * (size_t)B);
    int32_t *src = take(f, sizeof(int32_t) * (size_t)e_tot), *dst = take(f, sizeof(int32_t) * (size_t)e_tot);
    int32_t *placement = take(f, sizeof(int32_t) * (size_t)n_tot), *cur = take(f, sizeof(int32_t) * (size_t)B);
    double *feats = take(f, sizeof(double) * 3 * (size_t)n_tot), *weights = take(f, sizeof(double) * (size_t)*nw);
    fclose(f);
    /* n_weights = 0: levels and sets only */
    if (*nw != 0 && (int64_t)orc_weight_count(&cfg) != *nw) { fprintf(stderr, "weight count\n"); return 2; }

    int32_t *td = calloc((size_t)n_tot + 1, sizeof(int32_t)), *bu = calloc((size_t)n_tot + 1, sizeof(int32_t));
    uint8_t *cls = calloc((size_t)n_tot + 1, 1);
    double *logits = calloc((size_t)B * cfg.D + 1, sizeof(double)), *probs = calloc((size_t)B * cfg.D + 1, sizeof(double));
    double *emb = calloc((size_t)n_tot * 2 * cfg.H + 1, sizeof(double));
    double *pooled = calloc((size_t)B * 3 * G * cfg.H + 1, sizeof(double));
    int32_t *status = calloc(2 * (size_t)B + 1, sizeof(int32_t));
    size_t n0 = 0, e0 = 0;
    for (int32_t b = 0; b < B; ++b) {
        status[2 * b] = orc_levels(n_nodes[b], n_edges[b], src + e0, dst + e0, td + n0, bu + n0);
        status[2 * b + 1] = orc_classes(n_nodes[b], n_edges[b], src + e0, dst + e0, cur[b], cls + n0);
        n0 += (size_t)n_nodes[b];
        e0 += (size_t)n_edges[b];
    }
    if (*nw != 0)
        status[2 * B] = orc_forward_batch(&cfg, B, n_nodes, n_edges, src, dst, feats, placement, cur, weights, logits,
                                          probs, emb, pooled, 2);
    FILE *o = fopen(argv[2], "wb");
    if (!o) return 2;
    fwrite(status, sizeof(int32_t), 2 * (size_t)B + 1, o);
    fwrite(td, sizeof(int32_t), (size_t)n_tot, o);
    fwrite(bu, sizeof(int32_t), (size_t)n_tot, o);
    fwrite(cls, 1, (size_t)n_tot, o);
    fwrite(logits, sizeof(double), (size_t)B * cfg.D, o);
    fwrite(probs, sizeof(double), (size_t)B * cfg.D, o);
    fwrite(emb, sizeof(double), (size_t)n_tot * 2 * cfg.H, o);
    fwrite(pooled, sizeof(double), (size_t)B * 3 * G * cfg.H, o);
    fclose(o);
    free(hd); free(nw); free(n_nodes); free(n_edges); free(src); free(dst); free(placement); free(cur);
    free(feats); free(weights); free(td); free(bu); free(cls); free(logits); free(probs); free(emb);
    free(pooled); free(status);
    return 0;
}
