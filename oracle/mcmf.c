/*
 * CPU checker for the MaxScore routing assignment (TEST INFRASTRUCTURE, not product code).
 *
 * Problem (Section 3.2, Eq. 7-8 and Table 1): tokens i = 0..T-1, experts j = 0..E-1, integer
 * rewards q[i][j].  Choose P in {0,1}^{T x E} with row sums <= k and column sums <= C that first
 * maximises the number of ones (maximum flow) and then the total reward sum P_ij q_ij (minimum
 * cost with cost = -reward).  The paper solves it by repeatedly augmenting along a cheapest
 * path ("SPFA", Section 3.2, paragraph on algorithm complexity).
 *
 * Two solvers, both successive cheapest augmenting paths:
 *   mcmf_literal     builds the graph of Table 1 arc by arc (source, T token nodes, E expert
 *                    nodes, sink; T + E + T*E arcs plus residual twins) and finds each path
 *                    with a queue-based Bellman-Ford.  Any T, E, k, C.  Slow.
 *   mcmf_contracted  same mathematics with the token layer contracted away: the nodes are the
 *                    E experts and the sink, an arc j -> j' stands for "move the cheapest
 *                    token that sits on j and not on j' from j to j'", expert potentials keep
 *                    reduced costs non-negative so a dense Dijkstra finds each path.  Needs
 *                    T*k <= E*min(C,T) (every token is then forced to ship k units, so paths
 *                    may start from the tokens in any order).
 * Both also exist with one k per token and one capacity per expert (the vectors k and c of
 * Eq. 7): in Table 1 the arc Source -> Token_i then gets capacity k[i] and Expert_j -> Sink
 * capacity c[j].
 *
 * Shares no code with the GPU library.
 */
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#define INF64 ((int64_t)1 << 60)

/* ------------------------------------------------------------------------------------------ */
/* Literal graph of Table 1.                                                                   */

typedef struct {
    int n, m;             /* nodes, arcs (incl. twins) */
    int *head, *nxt, *to; /* adjacency lists */
    int *cap;
    int64_t *cost;
} graph_t;

static void g_add(graph_t *g, int a, int b, int cap, int64_t cost)
{
    int e = g->m;
    g->to[e] = b; g->cap[e] = cap; g->cost[e] = cost; g->nxt[e] = g->head[a]; g->head[a] = e;
    e++;
    g->to[e] = a; g->cap[e] = 0; g->cost[e] = -cost; g->nxt[e] = g->head[b]; g->head[b] = e;
    g->m += 2;
}

/* Returns 0 on success.  P[T*E] receives the assignment, *flow the flow value, *total the
 * reward sum, *n_arcs the number of arcs of Table 1 that were built (without twins). */
/* kvec[i] is the capacity of the arc Source -> Token_i and caps[j] that of Expert_j -> Sink (the
 * vectors k and c of Eq. 7). */
int mcmf_literal_kc(const int64_t *q, int T, int E, const int *kvec, const int *caps, uint8_t *P, int64_t *flow,
                    int64_t *total, int64_t *n_arcs)
{
    if (T <= 0 || E <= 0 || !kvec || !caps) return 1;
    for (int i = 0; i < T; i++) if (kvec[i] < 0) return 1;
    for (int j = 0; j < E; j++) if (caps[j] < 0) return 1;
    int S = 0, Z = T + E + 1, n = T + E + 2;
    int64_t arcs = (int64_t)T + E + (int64_t)T * E;
    graph_t g;
    g.n = n; g.m = 0;
    g.head = malloc(sizeof(int) * n);
    g.nxt = malloc(sizeof(int) * 2 * arcs);
    g.to = malloc(sizeof(int) * 2 * arcs);
    g.cap = malloc(sizeof(int) * 2 * arcs);
    g.cost = malloc(sizeof(int64_t) * 2 * arcs);
    int64_t *dist = malloc(sizeof(int64_t) * n);
    int *par = malloc(sizeof(int) * n), *queue = malloc(sizeof(int) * n);
    uint8_t *inq = malloc(n);
    for (int v = 0; v < n; v++) g.head[v] = -1;
    for (int i = 0; i < T; i++) g_add(&g, S, 1 + i, kvec[i], 0);            /* Source -> Token_i  */
    for (int j = 0; j < E; j++) g_add(&g, 1 + T + j, Z, caps[j], 0);        /* Expert_j -> Sink   */
    int first_te = g.m;
    for (int i = 0; i < T; i++)                                             /* Token_i -> Expert_j */
        for (int j = 0; j < E; j++) g_add(&g, 1 + i, 1 + T + j, 1, -q[(int64_t)i * E + j]);
    *n_arcs = g.m / 2;

    int64_t f = 0;
    for (;;) {
        for (int v = 0; v < n; v++) { dist[v] = INF64; par[v] = -1; inq[v] = 0; }
        int qh = 0, qt = 0, qn = 0;
        dist[S] = 0; queue[qt] = S; qt = (qt + 1) % n; qn = 1; inq[S] = 1;
        while (qn) {
            int v = queue[qh]; qh = (qh + 1) % n; qn--; inq[v] = 0;
            for (int e = g.head[v]; e >= 0; e = g.nxt[e]) {
                if (g.cap[e] <= 0) continue;
                int w = g.to[e];
                if (dist[v] + g.cost[e] < dist[w]) {
                    dist[w] = dist[v] + g.cost[e]; par[w] = e;
                    if (!inq[w]) { queue[qt] = w; qt = (qt + 1) % n; qn++; inq[w] = 1; }
                }
            }
        }
        if (dist[Z] >= INF64) break;     /* no augmenting path left: the flow is maximum */
        int b = 1 << 30;
        for (int v = Z; v != S; v = g.to[par[v] ^ 1]) if (g.cap[par[v]] < b) b = g.cap[par[v]];
        for (int v = Z; v != S; v = g.to[par[v] ^ 1]) { g.cap[par[v]] -= b; g.cap[par[v] ^ 1] += b; }
        f += b;
    }
    int64_t tot = 0;
    for (int i = 0; i < T; i++)
        for (int j = 0; j < E; j++) {
            int e = first_te + 2 * (i * E + j);
            uint8_t on = g.cap[e] == 0;
            P[(int64_t)i * E + j] = on;
            if (on) tot += q[(int64_t)i * E + j];
        }
    *flow = f; *total = tot;
    free(g.head); free(g.nxt); free(g.to); free(g.cap); free(g.cost);
    free(dist); free(par); free(queue); free(inq);
    return 0;
}

/* The same k for every token, caps[j] on the arc Expert_j -> Sink. */
int mcmf_literal_caps(const int64_t *q, int T, int E, int k, const int *caps, uint8_t *P, int64_t *flow,
                      int64_t *total, int64_t *n_arcs)
{
    if (T <= 0 || k < 0) return 1;
    int *kvec = malloc(sizeof(int) * T);
    for (int i = 0; i < T; i++) kvec[i] = k;
    int rc = mcmf_literal_kc(q, T, E, kvec, caps, P, flow, total, n_arcs);
    free(kvec);
    return rc;
}

/* Uniform capacity C on every expert (Table 1 as printed). */
int mcmf_literal(const int64_t *q, int T, int E, int k, int C, uint8_t *P, int64_t *flow,
                 int64_t *total, int64_t *n_arcs)
{
    if (E <= 0 || C < 0) return 1;
    int *caps = malloc(sizeof(int) * E);
    for (int j = 0; j < E; j++) caps[j] = C;
    int rc = mcmf_literal_caps(q, T, E, k, caps, P, flow, total, n_arcs);
    free(caps);
    return rc;
}

/* ------------------------------------------------------------------------------------------ */
/* Contracted form.                                                                            */

typedef struct {
    int T, E;
    const int64_t *q;
    uint8_t *held;   /* [T*E] */
    int *pos;        /* [T*E] index of token in mem[j] while held */
    int **mem;       /* mem[j][0..load[j]) */
    int *load;
    int64_t *L;      /* [E*E] cheapest move j -> j' */
    int *arg;        /* [E*E] token realising it, -1 if none */
    uint8_t *dirty;  /* [E*E] entry must be recomputed before use */
} cstate_t;

static void c_recompute(cstate_t *s, int j, int j2)
{
    int E = s->E;
    int64_t best = INF64; int who = -1;
    for (int a = 0; a < s->load[j]; a++) {
        int u = s->mem[j][a];
        if (s->held[(int64_t)u * E + j2]) continue;
        int64_t v = s->q[(int64_t)u * E + j] - s->q[(int64_t)u * E + j2];
        if (v < best) { best = v; who = u; }
    }
    s->L[j * E + j2] = best; s->arg[j * E + j2] = who; s->dirty[j * E + j2] = 0;
}

static void c_add(cstate_t *s, int u, int j)
{
    int E = s->E;
    const int64_t *qu = s->q + (int64_t)u * E;
    uint8_t *hu = s->held + (int64_t)u * E;
    hu[j] = 1;
    s->pos[(int64_t)u * E + j] = s->load[j];
    s->mem[j][s->load[j]++] = u;
    for (int j2 = 0; j2 < E; j2++) {
        if (j2 == j) continue;
        if (!hu[j2]) {                       /* u can now be moved j -> j2 */
            int64_t v = qu[j] - qu[j2];
            if (!s->dirty[j * E + j2] && v < s->L[j * E + j2]) { s->L[j * E + j2] = v; s->arg[j * E + j2] = u; }
        } else if (s->arg[j2 * E + j] == u) { /* u can no longer be moved j2 -> j */
            s->dirty[j2 * E + j] = 1;
        }
    }
}

static void c_remove(cstate_t *s, int u, int j)
{
    int E = s->E;
    const int64_t *qu = s->q + (int64_t)u * E;
    uint8_t *hu = s->held + (int64_t)u * E;
    hu[j] = 0;
    int p = s->pos[(int64_t)u * E + j], last = s->mem[j][--s->load[j]];
    s->mem[j][p] = last; s->pos[(int64_t)last * E + j] = p;
    for (int j2 = 0; j2 < E; j2++) {
        if (j2 == j) continue;
        if (s->arg[j * E + j2] == u) s->dirty[j * E + j2] = 1;   /* lost the move j -> j2 */
        if (hu[j2]) {                                            /* gained the move j2 -> j */
            int64_t v = qu[j2] - qu[j];
            if (!s->dirty[j2 * E + j] && v < s->L[j2 * E + j]) { s->L[j2 * E + j] = v; s->arg[j2 * E + j] = u; }
        }
    }
}

/* Per-token kvec[i] <= E and per-expert capacities caps[j] (clamped to T); the precondition is
 * sum_i kvec[i] <= sum_j min(caps[j], T).
 * Returns 0 on success, 1 bad arguments, 2 precondition violated, 3 internal
 * invariant (negative reduced cost) violated, 4 a token cannot ship all its units although the
 * precondition holds (unequal capacities can leave fewer experts with room than a token needs:
 * the literal graph then gives the answer).  prices[E] receives expert prices p_j >= 0 with
 * p_j = 0 on every expert left with spare capacity, such that every token i holds kvec[i] experts of
 * largest q_ij - p_j (a dual optimum).  *n_paths = augmentations, *n_hops = expert hops. */
int mcmf_contracted_kc(const int64_t *q, int T, int E, const int *kvec, const int *caps, uint8_t *P,
                       int64_t *prices, int64_t *flow, int64_t *total, int64_t *n_paths, int64_t *n_hops)
{
    if (T <= 0 || E <= 0 || !kvec || !caps) return 1;
    int64_t demand = 0;
    for (int i = 0; i < T; i++) {
        if (kvec[i] < 0 || kvec[i] > E) return 1;
        demand += kvec[i];
    }
    int *cap = malloc(sizeof(int) * E);
    int64_t room = 0;
    for (int j = 0; j < E; j++) {
        if (caps[j] < 0) { free(cap); return 1; }
        cap[j] = caps[j] < T ? caps[j] : T;
        room += cap[j];
    }
    if (demand > room) { free(cap); return 2; }
    cstate_t s;
    s.T = T; s.E = E; s.q = q;
    s.held = calloc((size_t)T * E, 1);
    s.pos = malloc(sizeof(int) * (size_t)T * E);
    s.mem = malloc(sizeof(int *) * E);
    s.load = calloc(E, sizeof(int));
    for (int j = 0; j < E; j++) s.mem[j] = malloc(sizeof(int) * (cap[j] > 0 ? cap[j] : 1));
    s.L = malloc(sizeof(int64_t) * E * E);
    s.arg = malloc(sizeof(int) * E * E);
    s.dirty = calloc((size_t)E * E, 1);
    for (int a = 0; a < E * E; a++) { s.L[a] = INF64; s.arg[a] = -1; }
    int64_t *phi = calloc(E, sizeof(int64_t)), *d = malloc(sizeof(int64_t) * E);
    int *par = malloc(sizeof(int) * E), *partok = malloc(sizeof(int) * E), *path = malloc(sizeof(int) * E);
    uint8_t *done = malloc(E);
    int rc = 0;
    int64_t paths = 0, hops = 0;

    for (int i = 0; i < T && !rc; i++) {
        for (int rep = 0; rep < kvec[i] && !rc; rep++) {
            /* dense Dijkstra over experts + sink on reduced costs c + phi[a] - phi[b], phi[sink] = 0 */
            const int64_t *qi = q + (int64_t)i * E;
            for (int j = 0; j < E; j++) {
                done[j] = 0; par[j] = -1; partok[j] = -1;
                d[j] = s.held[(int64_t)i * E + j] ? INF64 : -qi[j] - phi[j];
            }
            int64_t dZ = INF64; int parZ = -1;
            for (;;) {
                int j = -1; int64_t best = INF64;
                for (int a = 0; a < E; a++) if (!done[a] && d[a] < best) { best = d[a]; j = a; }
                if (dZ <= best) break;            /* sink is the next node to settle (or nothing left) */
                done[j] = 1;
                if (s.load[j] < cap[j]) {         /* Expert_j -> Sink has residual capacity, cost 0 */
                    int64_t c = d[j] + phi[j];
                    if (c < dZ) { dZ = c; parZ = j; }
                }
                for (int j2 = 0; j2 < E; j2++) {
                    if (done[j2] || j2 == j) continue;
                    if (s.dirty[j * E + j2]) c_recompute(&s, j, j2);
                    int64_t l = s.L[j * E + j2];
                    if (l >= INF64) continue;
                    int64_t red = l + phi[j] - phi[j2];
                    if (red < 0) { rc = 3; break; }
                    if (d[j] + red < d[j2]) { d[j2] = d[j] + red; par[j2] = j; partok[j2] = s.arg[j * E + j2]; }
                }
                if (rc) break;
            }
            if (rc) break;
            if (parZ < 0) { rc = 4; break; }      /* this unit cannot be shipped (possible only with unequal capacities) */
            for (int j = 0; j < E; j++) phi[j] += (d[j] < dZ ? d[j] : dZ) - dZ;
            int len = 0;
            for (int j = parZ; j >= 0; j = par[j]) path[len++] = j;   /* sink side first */
            for (int a = 0; a + 1 < len; a++) {   /* move partok[path[a]] from path[a+1] to path[a] */
                int u = partok[path[a]];
                c_remove(&s, u, path[a + 1]);
                c_add(&s, u, path[a]);
            }
            c_add(&s, i, path[len - 1]);
            paths++; hops += len;
        }
    }
    int64_t tot = 0, f = 0;
    for (int64_t a = 0; a < (int64_t)T * E; a++) { P[a] = s.held[a]; if (s.held[a]) { tot += q[a]; f++; } }
    for (int j = 0; j < E; j++) prices[j] = -phi[j];
    *flow = f; *total = tot; *n_paths = paths; *n_hops = hops;
    for (int j = 0; j < E; j++) free(s.mem[j]);
    free(s.held); free(s.pos); free(s.mem); free(s.load); free(s.L); free(s.arg); free(s.dirty);
    free(phi); free(d); free(par); free(partok); free(path); free(done); free(cap);
    return rc;
}

/* The same k for every token. */
int mcmf_contracted_caps(const int64_t *q, int T, int E, int k, const int *caps, uint8_t *P, int64_t *prices,
                         int64_t *flow, int64_t *total, int64_t *n_paths, int64_t *n_hops)
{
    if (T <= 0 || k < 0) return 1;
    int *kvec = malloc(sizeof(int) * T);
    for (int i = 0; i < T; i++) kvec[i] = k;
    int rc = mcmf_contracted_kc(q, T, E, kvec, caps, P, prices, flow, total, n_paths, n_hops);
    free(kvec);
    return rc;
}

/* Uniform capacity C on every expert. */
int mcmf_contracted(const int64_t *q, int T, int E, int k, int C, uint8_t *P, int64_t *prices,
                    int64_t *flow, int64_t *total, int64_t *n_paths, int64_t *n_hops)
{
    if (E <= 0 || C < 0) return 1;
    int *caps = malloc(sizeof(int) * E);
    for (int j = 0; j < E; j++) caps[j] = C;
    int rc = mcmf_contracted_caps(q, T, E, k, caps, P, prices, flow, total, n_paths, n_hops);
    free(caps);
    return rc;
}
