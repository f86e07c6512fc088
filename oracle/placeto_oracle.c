/*
 * Float64 CPU oracle for the Placeto policy forward pass.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, plain definition that the HIP library
 * is checked against.  It shares no code with that library, and nothing outside tests/,
 * the smoke check and the benchmark's cpu_baseline leg may call it.
 *
 * What it computes follows Section 2.2 of the paper ("Policy Network Architecture",
 * steps 1-3 of the graph embedding) and the network shapes in Appendix A.7, with the
 * places where the text is silent resolved as stated next to each function.  There is no
 * blocking, fusion or reordering: one node at a time, one layer at a time, plain loops.
 *
 * Parity pins (tests/test_oracle_*.py): hand-derived values on a 3-node chain, a diamond
 * and a 2-node graph with asymmetric integer weights; the path-count closed form
 * (I - A^T)^-1 x under identity networks; a one-node graph against a library
 * feed-forward chain; boolean transitive closure for the three node sets; brute-force
 * longest paths for the levels; relabelling and aggregation-order invariance; locality of
 * the two sweeps.  Trained behaviour (Table 1, the generalisation CDFs) needs the
 * paper's models and weights: parity unpinned.
 *
 * Conventions
 *   edge (src, dst): dst receives a tensor from src, so src is a PARENT of dst
 *                    (Section 2: an op receives input tensors "from its parent ops").
 *   raw features of node v (Section 2.1, Section 2.2 step 1), F = D + 4 values:
 *       [ run time, output size, one-hot(device of v) (D values), is-current, is-visited ]
 *   weight blob: for every layer a row-major [in, out] matrix followed by `out` biases,
 *       in the order proj; f_td; g_td; f_bu; g_bu; l_par; l_chi; l_pll; h_par; h_chi;
 *       h_pll; policy layer 1; policy layer 2.
 */
#include <math.h>
#include <stddef.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

typedef struct {
    int32_t D;               /* devices */
    int32_t H;               /* embedding width */
    int32_t n_layers;        /* layers in each of f, g, l, h (Appendix A.7 uses 1) */
    int32_t k_sweeps;        /* repetitions of the message passing (Section 2.2 step 2) */
    int32_t group_by_device; /* 1: pool per (set, device); 0: per set, as printed */
    int32_t single_set;      /* 1: the "simple aggregator" of the paper's comparison of policy
                                architectures (Section 3.3): no partition into parents / children /
                                parallel nodes, every node other than v* is pooled in the first set */
} orc_cfg;

enum { ORC_OK = 0, ORC_ERR_ARG = -1, ORC_ERR_CYCLE = -2, ORC_ERR_MEM = -3 };

/* ------------------------------------------------------------------ adjacency lists */
typedef struct {
    int32_t n;
    int32_t *par_cnt, *chi_cnt;   /* number of parents / children of each node */
    int32_t **par, **chi;         /* the lists themselves, in edge-list order */
} adj_t;

static void adj_free(adj_t *a)
{
    if (a->par) for (int32_t v = 0; v < a->n; ++v) free(a->par[v]);
    if (a->chi) for (int32_t v = 0; v < a->n; ++v) free(a->chi[v]);
    free(a->par); free(a->chi); free(a->par_cnt); free(a->chi_cnt);
    memset(a, 0, sizeof *a);
}

static int adj_build(adj_t *a, int32_t n, int32_t n_edges, const int32_t *src, const int32_t *dst)
{
    memset(a, 0, sizeof *a);
    a->n = n;
    a->par_cnt = calloc((size_t)n, sizeof(int32_t));
    a->chi_cnt = calloc((size_t)n, sizeof(int32_t));
    a->par = calloc((size_t)n, sizeof(int32_t *));
    a->chi = calloc((size_t)n, sizeof(int32_t *));
    if (!a->par_cnt || !a->chi_cnt || !a->par || !a->chi) { adj_free(a); return ORC_ERR_MEM; }
    for (int32_t e = 0; e < n_edges; ++e) {
        if (src[e] < 0 || src[e] >= n || dst[e] < 0 || dst[e] >= n) { adj_free(a); return ORC_ERR_ARG; }
        a->chi_cnt[src[e]]++;
        a->par_cnt[dst[e]]++;
    }
    for (int32_t v = 0; v < n; ++v) {
        a->par[v] = malloc(sizeof(int32_t) * (size_t)(a->par_cnt[v] + 1));
        a->chi[v] = malloc(sizeof(int32_t) * (size_t)(a->chi_cnt[v] + 1));
        if (!a->par[v] || !a->chi[v]) { adj_free(a); return ORC_ERR_MEM; }
        a->par_cnt[v] = a->chi_cnt[v] = 0;
    }
    for (int32_t e = 0; e < n_edges; ++e) {
        a->chi[src[e]][a->chi_cnt[src[e]]++] = dst[e];
        a->par[dst[e]][a->par_cnt[dst[e]]++] = src[e];
    }
    return ORC_OK;
}

/* Any topological order (parents before children), by repeatedly removing nodes whose
 * parents have all been removed.  Returns ORC_ERR_CYCLE if the graph is not a DAG. */
static int topo_order(const adj_t *a, int32_t *order)
{
    int32_t n = a->n, head = 0, tail = 0;
    int32_t *left = malloc(sizeof(int32_t) * (size_t)(n + 1));
    if (!left) return ORC_ERR_MEM;
    for (int32_t v = 0; v < n; ++v) {
        left[v] = a->par_cnt[v];
        if (left[v] == 0) order[tail++] = v;
    }
    while (head < tail) {
        int32_t u = order[head++];
        for (int32_t i = 0; i < a->chi_cnt[u]; ++i) {
            int32_t c = a->chi[u][i];
            if (--left[c] == 0) order[tail++] = c;
        }
    }
    free(left);
    return tail == n ? ORC_OK : ORC_ERR_CYCLE;
}

/* ------------------------------------------------------------------ levels
 * Longest-path layering (the build's own notion, used by the level-synchronous sweeps):
 * td_level(v) = 0 for a root (no parents), else 1 + max over parents;
 * bu_level(v) = 0 for a leaf (no children), else 1 + max over children.
 * "Root" and "leaf" as in Section 2.2 step 2 (top-down from roots, bottom-up from leaves). */
int orc_levels(int32_t n, int32_t n_edges, const int32_t *src, const int32_t *dst,
               int32_t *td_level, int32_t *bu_level)
{
    adj_t a;
    int rc = adj_build(&a, n, n_edges, src, dst);
    if (rc) return rc;
    int32_t *order = malloc(sizeof(int32_t) * (size_t)(n + 1));
    if (!order) { adj_free(&a); return ORC_ERR_MEM; }
    rc = topo_order(&a, order);
    if (rc == ORC_OK) {
        for (int32_t i = 0; i < n; ++i) {
            int32_t v = order[i], lv = 0;
            for (int32_t j = 0; j < a.par_cnt[v]; ++j) {
                int32_t cand = td_level[a.par[v][j]] + 1;
                if (cand > lv) lv = cand;
            }
            td_level[v] = lv;
        }
        for (int32_t i = n - 1; i >= 0; --i) {
            int32_t v = order[i], lv = 0;
            for (int32_t j = 0; j < a.chi_cnt[v]; ++j) {
                int32_t cand = bu_level[a.chi[v][j]] + 1;
                if (cand > lv) lv = cand;
            }
            bu_level[v] = lv;
        }
    }
    free(order);
    adj_free(&a);
    return rc;
}

/* ------------------------------------------------------------------ node sets
 * Section 2.2 step 3: for the current node v*, S_parents = nodes that can reach v*,
 * S_children = nodes reachable from v*, S_parallel = nodes that can do neither.
 * v* itself belongs to none of them (its embedding enters the policy input separately).
 * Codes: 0 = v*, 1 = S_parents, 2 = S_children, 3 = S_parallel. */
static void mark_reachable(int32_t start, const int32_t *cnt, int32_t *const *nbr,
                           uint8_t *seen, int32_t *stack)
{
    int32_t top = 0;
    stack[top++] = start;
    seen[start] = 1;
    while (top) {
        int32_t u = stack[--top];
        for (int32_t i = 0; i < cnt[u]; ++i) {
            int32_t w = nbr[u][i];
            if (!seen[w]) { seen[w] = 1; stack[top++] = w; }
        }
    }
}

static int classes_from_adj(const adj_t *a, int32_t cur, uint8_t *cls)
{
    int32_t n = a->n;
    uint8_t *up = calloc((size_t)n + 1, 1), *down = calloc((size_t)n + 1, 1);
    int32_t *stack = malloc(sizeof(int32_t) * (size_t)(n + 1));
    if (!up || !down || !stack) { free(up); free(down); free(stack); return ORC_ERR_MEM; }
    mark_reachable(cur, a->par_cnt, a->par, up, stack);     /* walks parent links   */
    mark_reachable(cur, a->chi_cnt, a->chi, down, stack);   /* walks children links */
    for (int32_t u = 0; u < n; ++u) {
        if (u == cur) cls[u] = 0;
        else if (up[u]) cls[u] = 1;
        else if (down[u]) cls[u] = 2;
        else cls[u] = 3;
    }
    free(up); free(down); free(stack);
    return ORC_OK;
}

int orc_classes(int32_t n, int32_t n_edges, const int32_t *src, const int32_t *dst,
                int32_t cur, uint8_t *cls)
{
    if (cur < 0 || cur >= n) return ORC_ERR_ARG;
    adj_t a;
    int rc = adj_build(&a, n, n_edges, src, dst);
    if (rc) return rc;
    rc = classes_from_adj(&a, cur, cls);
    adj_free(&a);
    return rc;
}

/* ------------------------------------------------------------------ networks */
/* One feed-forward layer: y = W^T x + b with W row-major [n_in, n_out]; ReLU if asked.
 * Returns the position just past this layer's parameters. */
static const double *layer(const double *p, int32_t n_in, int32_t n_out, int relu,
                           const double *x, double *y)
{
    const double *W = p, *b = p + (size_t)n_in * n_out;
    for (int32_t j = 0; j < n_out; ++j) {
        double s = b[j];
        for (int32_t i = 0; i < n_in; ++i) s += x[i] * W[(size_t)i * n_out + j];
        y[j] = (relu && s < 0.0) ? 0.0 : s;
    }
    return b + n_out;
}

static size_t layer_size(int32_t n_in, int32_t n_out) { return (size_t)n_in * n_out + n_out; }

/* An embedding network (f, g, l_i or h_i): n_layers layers, ReLU after every one
 * (Appendix A.7: ReLU is the default activation; a final linear layer would make a
 * one-layer g(sum f(.)) linear).  First layer n_in -> H, the rest H -> H. */
static void mlp(const double *p, int32_t n_layers, int32_t n_in, int32_t H,
                const double *x, double *y, double *tmp_a, double *tmp_b)
{
    const double *in = x;
    int32_t width = n_in;
    for (int32_t l = 0; l < n_layers; ++l) {
        double *out = (l == n_layers - 1) ? y : ((l & 1) ? tmp_b : tmp_a);
        p = layer(p, width, H, 1, in, out);
        in = out;
        width = H;
    }
}

static size_t mlp_size(int32_t n_layers, int32_t n_in, int32_t H)
{
    size_t s = 0;
    for (int32_t l = 0; l < n_layers; ++l) s += layer_size(l == 0 ? n_in : H, H);
    return s;
}

size_t orc_weight_count(const orc_cfg *c)
{
    int32_t D = c->D, H = c->H, L = c->n_layers;
    int32_t groups = c->group_by_device ? D : 1;
    size_t s = layer_size(D + 4, H);
    s += 4 * mlp_size(L, H, H);          /* f_td g_td f_bu g_bu */
    s += 3 * mlp_size(L, 2 * H, H);      /* l_par l_chi l_pll   */
    s += 3 * mlp_size(L, H, H);          /* h_par h_chi h_pll   */
    s += layer_size((2 + 3 * groups) * H, H) + layer_size(H, D);
    return s;
}

/* One message-passing sweep in one direction (Section 2.2 step 2).
 * The printed update x_v <- g(sum_{u in xi(v)} f(x_u)) has no term for v itself; read
 * literally, roots would become g(0) and lose their features, yet the text says the
 * result summarises the whole sub-graph that can reach v.  The reading taken here keeps
 * v's own value as a residual:  s_v <- s_v + g( sum_{u in xi(v)} f(s_u) ),
 * visiting nodes so that every neighbour in xi(v) is final before v (one full pass from
 * the roots for top-down, from the leaves for bottom-up).  An empty sum is the zero
 * vector and still goes through g.  `order` lists nodes with xi-neighbours first. */
static void sweep(const double *f_par, const double *g_par, int32_t n_layers, int32_t H,
                  int32_t n, const int32_t *order, const int32_t *cnt, int32_t *const *nbr,
                  double *s /* [n,H] in/out */, double *msg /* [n,H] scratch */,
                  double *agg, double *upd, double *ta, double *tb)
{
    for (int32_t i = 0; i < n; ++i) {
        int32_t v = order[i];
        for (int32_t h = 0; h < H; ++h) agg[h] = 0.0;
        for (int32_t j = 0; j < cnt[v]; ++j) {
            const double *m = msg + (size_t)nbr[v][j] * H;   /* f(s_u), u already final */
            for (int32_t h = 0; h < H; ++h) agg[h] += m[h];
        }
        mlp(g_par, n_layers, H, H, agg, upd, ta, tb);
        for (int32_t h = 0; h < H; ++h) s[(size_t)v * H + h] += upd[h];
        mlp(f_par, n_layers, H, H, s + (size_t)v * H, msg + (size_t)v * H, ta, tb);
    }
}

/* Full forward pass for one graph.
 *   feats      [n,3]  run time, output size, is-visited
 *   placement  [n]    current device of each node, in [0, D)
 *   cur               the node whose placement is being decided
 *   weights           blob as described at the top (already at the precision under test)
 *   logits     [D]    pre-softmax outputs;  probs [D] softmax of them (may be NULL)
 *   emb        [n,2H] optional: [top-down ; bottom-up] embedding of every node
 *   pooled     [3,G,H] optional: the summed l_i outputs per (set, device group), G = D or 1
 */
int orc_forward_graph(const orc_cfg *c, int32_t n, int32_t n_edges,
                      const int32_t *src, const int32_t *dst, const double *feats,
                      const int32_t *placement, int32_t cur, const double *weights,
                      double *logits, double *probs, double *emb, double *pooled)
{
    const int32_t D = c->D, H = c->H, L = c->n_layers, F = D + 4;
    const int32_t G = c->group_by_device ? D : 1;
    const int32_t Z = (2 + 3 * G) * H;
    if (n < 1 || cur < 0 || cur >= n || D < 1 || H < 1 || L < 1 || c->k_sweeps < 0) return ORC_ERR_ARG;
    for (int32_t v = 0; v < n; ++v)
        if (placement[v] < 0 || placement[v] >= D) return ORC_ERR_ARG;

    adj_t a;
    int rc = adj_build(&a, n, n_edges, src, dst);
    if (rc) return rc;

    int32_t widest = Z > F ? Z : F;
    if (2 * H > widest) widest = 2 * H;
    int32_t *order = malloc(sizeof(int32_t) * (size_t)(n + 1));
    int32_t *rev = malloc(sizeof(int32_t) * (size_t)(n + 1));
    uint8_t *cls = malloc((size_t)n + 1);
    double *td = malloc(sizeof(double) * (size_t)n * H);
    double *bu = malloc(sizeof(double) * (size_t)n * H);
    double *msg = malloc(sizeof(double) * (size_t)n * H);
    double *P = calloc((size_t)3 * G * H, sizeof(double));
    double *buf = malloc(sizeof(double) * (size_t)(6 * widest + 8));
    if (!order || !rev || !cls || !td || !bu || !msg || !P || !buf) { rc = ORC_ERR_MEM; goto done; }
    double *phi = buf, *agg = buf + widest, *upd = buf + 2 * widest;
    double *ta = buf + 3 * widest, *tb = buf + 4 * widest, *z = buf + 5 * widest;

    rc = topo_order(&a, order);
    if (rc) goto done;
    for (int32_t i = 0; i < n; ++i) rev[i] = order[n - 1 - i];

    /* parameter positions in blob order */
    const double *p_proj = weights;
    const double *p_f_td = p_proj + layer_size(F, H);
    const double *p_g_td = p_f_td + mlp_size(L, H, H);
    const double *p_f_bu = p_g_td + mlp_size(L, H, H);
    const double *p_g_bu = p_f_bu + mlp_size(L, H, H);
    const double *p_l[3], *p_h[3];
    p_l[0] = p_g_bu + mlp_size(L, H, H);
    p_l[1] = p_l[0] + mlp_size(L, 2 * H, H);
    p_l[2] = p_l[1] + mlp_size(L, 2 * H, H);
    p_h[0] = p_l[2] + mlp_size(L, 2 * H, H);
    p_h[1] = p_h[0] + mlp_size(L, H, H);
    p_h[2] = p_h[1] + mlp_size(L, H, H);
    const double *p_pol = p_h[2] + mlp_size(L, H, H);

    /* Step 1: raw features, projected to the embedding width H (the message-passing
     * networks are reused at every step, so the state must have one fixed width). */
    for (int32_t v = 0; v < n; ++v) {
        phi[0] = feats[(size_t)v * 3 + 0];
        phi[1] = feats[(size_t)v * 3 + 1];
        for (int32_t d = 0; d < D; ++d) phi[2 + d] = (placement[v] == d) ? 1.0 : 0.0;
        phi[2 + D] = (v == cur) ? 1.0 : 0.0;
        phi[3 + D] = feats[(size_t)v * 3 + 2];
        layer(p_proj, F, H, 1, phi, td + (size_t)v * H);
        memcpy(bu + (size_t)v * H, td + (size_t)v * H, sizeof(double) * (size_t)H);
    }

    /* Step 2: k sweeps per direction; the directions have separate parameters and do not
     * mix until they are concatenated. */
    for (int32_t s = 0; s < c->k_sweeps; ++s) {
        sweep(p_f_td, p_g_td, L, H, n, order, a.par_cnt, a.par, td, msg, agg, upd, ta, tb);
        sweep(p_f_bu, p_g_bu, L, H, n, rev, a.chi_cnt, a.chi, bu, msg, agg, upd, ta, tb);
    }
    if (emb)
        for (int32_t v = 0; v < n; ++v) {
            memcpy(emb + (size_t)v * 2 * H, td + (size_t)v * H, sizeof(double) * (size_t)H);
            memcpy(emb + (size_t)v * 2 * H + H, bu + (size_t)v * H, sizeof(double) * (size_t)H);
        }

    /* Step 3: pooling.  P[i][d] = sum over u in S_i(v*) placed on device d of l_i(e_u),
     * e_u = [td_u ; bu_u]; then q[i][d] = h_i(P[i][d]), also for empty groups. */
    rc = classes_from_adj(&a, cur, cls);
    if (rc) goto done;
    if (c->single_set)
        for (int32_t u = 0; u < n; ++u) cls[u] = (u == cur) ? 0 : 1;
    for (int32_t u = 0; u < n; ++u) {
        if (cls[u] == 0) continue;
        int32_t i = cls[u] - 1;
        int32_t d = c->group_by_device ? placement[u] : 0;
        memcpy(agg, td + (size_t)u * H, sizeof(double) * (size_t)H);
        memcpy(agg + H, bu + (size_t)u * H, sizeof(double) * (size_t)H);
        mlp(p_l[i], L, 2 * H, H, agg, upd, ta, tb);
        double *acc = P + ((size_t)i * G + d) * H;
        for (int32_t h = 0; h < H; ++h) acc[h] += upd[h];
    }
    if (pooled) memcpy(pooled, P, sizeof(double) * (size_t)3 * G * H);

    /* Policy input: v*'s own embedding, then the 3*G pooled summaries. */
    memcpy(z, td + (size_t)cur * H, sizeof(double) * (size_t)H);
    memcpy(z + H, bu + (size_t)cur * H, sizeof(double) * (size_t)H);
    for (int32_t i = 0; i < 3; ++i)
        for (int32_t d = 0; d < G; ++d)
            mlp(p_h[i], L, H, H, P + ((size_t)i * G + d) * H,
                z + (size_t)(2 + i * G + d) * H, ta, tb);

    /* Policy network: two layers, ReLU on the hidden one, softmax on the output
     * (Appendix A.7). */
    const double *p2 = layer(p_pol, Z, H, 1, z, upd);
    layer(p2, H, D, 0, upd, logits);
    if (probs) {
        double mx = logits[0], tot = 0.0;
        for (int32_t d = 1; d < D; ++d) if (logits[d] > mx) mx = logits[d];
        for (int32_t d = 0; d < D; ++d) { probs[d] = exp(logits[d] - mx); tot += probs[d]; }
        for (int32_t d = 0; d < D; ++d) probs[d] /= tot;
    }

done:
    free(order); free(rev); free(cls); free(td); free(bu); free(msg); free(P); free(buf);
    adj_free(&a);
    return rc;
}

/* A batch of independent graphs, concatenated: graph b owns nodes
 * [sum n_nodes[:b], ...) and edges [sum n_edges[:b], ...), ids graph-local.
 * Graphs are spread over `n_threads` OpenMP threads; each graph is computed by the
 * single-threaded function above.  Returns the first non-zero status. */
int orc_forward_batch(const orc_cfg *c, int32_t B, const int32_t *n_nodes,
                      const int32_t *n_edges, const int32_t *src, const int32_t *dst,
                      const double *feats, const int32_t *placement, const int32_t *cur,
                      const double *weights, double *logits, double *probs, double *emb,
                      double *pooled, int32_t n_threads)
{
    int status = ORC_OK;
    const int32_t G = c->group_by_device ? c->D : 1;
    size_t *noff = malloc(sizeof(size_t) * (size_t)(B + 1));
    size_t *eoff = malloc(sizeof(size_t) * (size_t)(B + 1));
    if (!noff || !eoff) { free(noff); free(eoff); return ORC_ERR_MEM; }
    noff[0] = eoff[0] = 0;
    for (int32_t b = 0; b < B; ++b) {
        noff[b + 1] = noff[b] + (size_t)n_nodes[b];
        eoff[b + 1] = eoff[b] + (size_t)n_edges[b];
    }
    if (n_threads < 1) n_threads = 1;
#pragma omp parallel for schedule(dynamic, 1) num_threads(n_threads)
    for (int32_t b = 0; b < B; ++b) {
        int rc = orc_forward_graph(c, n_nodes[b], n_edges[b], src + eoff[b], dst + eoff[b],
                                   feats + noff[b] * 3, placement + noff[b], cur[b], weights,
                                   logits + (size_t)b * c->D,
                                   probs ? probs + (size_t)b * c->D : NULL,
                                   emb ? emb + noff[b] * 2 * c->H : NULL,
                                   pooled ? pooled + (size_t)b * 3 * G * c->H : NULL);
        if (rc) {
#pragma omp critical
            status = rc;
        }
    }
    free(noff); free(eoff);
    return status;
}
