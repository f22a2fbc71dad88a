/*
 * CPU ORACLE -- TEST INFRASTRUCTURE ONLY.  Not part of the product path.
 *
 * Plain, slow, textbook integer max-flow used to check the HIP library:
 *   - the value F(x, y; D) of a maximum flow in a capacitated digraph D, the only
 *     property of max-flow the paper relies on (Appendix E preamble, min-cut theorem);
 *   - the auxiliary network of Section 5.2 / Appendix E.1: a super-source s joined to
 *     every compute node, built explicitly per problem.
 * Two independent algorithms (Dinic, Edmonds-Karp) so that each checks the other.
 * The paper's own tool used push-relabel (Appendix C); these two are deliberately
 * a different algorithm family from the GPU path.  Shares no code with the HIP path.
 *
 * All capacities and flows are int64.  The caller guarantees that the sum of the
 * capacities leaving the source is below 2^62 (the Python wrapper checks it).
 */
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#include <pthread.h>

typedef struct {
    int32_t n;          /* vertices */
    int64_t m2;         /* residual arcs = 2 * input arcs; arc i and i^1 are a pair */
    int32_t *to;        /* [m2] head of residual arc                                */
    int64_t *res;       /* [m2] residual capacity                                   */
    int64_t *start;     /* [n+1] CSR offsets into `adj`                             */
    int64_t *adj;       /* [m2] residual arc ids grouped by tail                    */
} net_t;

static int net_build(net_t *g, int32_t n, int64_t m, const int32_t *tail,
                     const int32_t *head, const int64_t *cap)
{
    g->n = n; g->m2 = 2 * m;
    g->to = (int32_t *)malloc(sizeof(int32_t) * (size_t)(2 * m + 1));
    g->res = (int64_t *)malloc(sizeof(int64_t) * (size_t)(2 * m + 1));
    g->start = (int64_t *)calloc((size_t)n + 2, sizeof(int64_t));
    g->adj = (int64_t *)malloc(sizeof(int64_t) * (size_t)(2 * m + 1));
    if (!g->to || !g->res || !g->start || !g->adj) return -1;
    for (int64_t i = 0; i < m; ++i) {
        g->to[2 * i] = head[i];     g->res[2 * i] = cap[i];      /* forward  */
        g->to[2 * i + 1] = tail[i]; g->res[2 * i + 1] = 0;       /* backward */
        g->start[tail[i] + 1]++; g->start[head[i] + 1]++;
    }
    for (int32_t v = 0; v < n; ++v) g->start[v + 1] += g->start[v];
    int64_t *fill = (int64_t *)malloc(sizeof(int64_t) * ((size_t)n + 1));
    if (!fill) return -1;
    memcpy(fill, g->start, sizeof(int64_t) * (size_t)n);
    for (int64_t i = 0; i < m; ++i) {
        g->adj[fill[tail[i]]++] = 2 * i;
        g->adj[fill[head[i]]++] = 2 * i + 1;
    }
    free(fill);
    return 0;
}

static void net_free(net_t *g)
{
    free(g->to); free(g->res); free(g->start); free(g->adj);
}

/* ---------------------------------------------------------------- Dinic */

static int dinic_bfs(const net_t *g, int32_t src, int32_t dst, int32_t *level, int32_t *queue)
{
    for (int32_t v = 0; v < g->n; ++v) level[v] = -1;
    int32_t qh = 0, qt = 0;
    level[src] = 0; queue[qt++] = src;
    while (qh < qt) {
        int32_t u = queue[qh++];
        for (int64_t p = g->start[u]; p < g->start[u + 1]; ++p) {
            int64_t a = g->adj[p];
            int32_t w = g->to[a];
            if (g->res[a] > 0 && level[w] < 0) { level[w] = level[u] + 1; queue[qt++] = w; }
        }
    }
    return level[dst] >= 0;
}

/* iterative DFS: one augmenting path in the level graph per call; returns its bottleneck */
static int64_t dinic_augment(net_t *g, int32_t src, int32_t dst, const int32_t *level,
                             int64_t *cur, int64_t *path /* arc stack */, int32_t *pv /* vertex stack */)
{
    int32_t depth = 0;
    pv[0] = src;
    for (;;) {
        int32_t u = pv[depth];
        if (u == dst) {
            int64_t bott = INT64_MAX;
            for (int32_t i = 0; i < depth; ++i) if (g->res[path[i]] < bott) bott = g->res[path[i]];
            for (int32_t i = 0; i < depth; ++i) { g->res[path[i]] -= bott; g->res[path[i] ^ 1] += bott; }
            return bott;
        }
        int advanced = 0;
        while (cur[u] < g->start[u + 1]) {
            int64_t a = g->adj[cur[u]];
            int32_t w = g->to[a];
            if (g->res[a] > 0 && level[w] == level[u] + 1) {
                path[depth] = a; pv[++depth] = w; advanced = 1; break;
            }
            cur[u]++;
        }
        if (!advanced) {
            if (depth == 0) return 0;
            depth--;                 /* dead end: retreat and skip the arc that led here */
            cur[pv[depth]]++;
        }
    }
}

static int64_t dinic(net_t *g, int32_t src, int32_t dst)
{
    if (src == dst) return -1;
    int32_t n = g->n;
    int32_t *level = (int32_t *)malloc(sizeof(int32_t) * (size_t)n);
    int32_t *queue = (int32_t *)malloc(sizeof(int32_t) * (size_t)n);
    int32_t *pv = (int32_t *)malloc(sizeof(int32_t) * ((size_t)n + 1));
    int64_t *cur = (int64_t *)malloc(sizeof(int64_t) * (size_t)n);
    int64_t *path = (int64_t *)malloc(sizeof(int64_t) * ((size_t)n + 1));
    int64_t total = 0;
    while (dinic_bfs(g, src, dst, level, queue)) {
        memcpy(cur, g->start, sizeof(int64_t) * (size_t)n);
        int64_t f;
        while ((f = dinic_augment(g, src, dst, level, cur, path, pv)) > 0) total += f;
    }
    free(level); free(queue); free(pv); free(cur); free(path);
    return total;
}

/* ---------------------------------------------------------------- Edmonds-Karp */

static int64_t edmonds_karp(net_t *g, int32_t src, int32_t dst)
{
    if (src == dst) return -1;
    int32_t n = g->n;
    int64_t *pred = (int64_t *)malloc(sizeof(int64_t) * (size_t)n);   /* arc used to reach v */
    int32_t *queue = (int32_t *)malloc(sizeof(int32_t) * (size_t)n);
    int64_t total = 0;
    for (;;) {
        for (int32_t v = 0; v < n; ++v) pred[v] = -1;
        int32_t qh = 0, qt = 0;
        queue[qt++] = src; pred[src] = -2;
        while (qh < qt && pred[dst] == -1) {
            int32_t u = queue[qh++];
            for (int64_t p = g->start[u]; p < g->start[u + 1]; ++p) {
                int64_t a = g->adj[p];
                int32_t w = g->to[a];
                if (g->res[a] > 0 && pred[w] == -1) { pred[w] = a; queue[qt++] = w; }
            }
        }
        if (pred[dst] == -1) break;
        int64_t bott = INT64_MAX;
        for (int32_t v = dst; v != src; v = g->to[pred[v] ^ 1])
            if (g->res[pred[v]] < bott) bott = g->res[pred[v]];
        for (int32_t v = dst; v != src; v = g->to[pred[v] ^ 1]) {
            g->res[pred[v]] -= bott; g->res[pred[v] ^ 1] += bott;
        }
        total += bott;
    }
    free(pred); free(queue);
    return total;
}

/* ---------------------------------------------------------------- exported: generic s-t max-flow
 *
 * F(src, dst; D) for the digraph D given as an arc list (Appendix E preamble).
 * algo: 0 = Dinic, 1 = Edmonds-Karp.  If arc_flow is non-null it receives the flow
 * on each input arc (for capacity / conservation / min-cut certificate checks).
 * Returns the flow value, or -1 on bad arguments / out of memory.
 */
int64_t fco_maxflow(int32_t n_vertices, int64_t n_arcs, const int32_t *tail, const int32_t *head,
                    const int64_t *cap, int32_t src, int32_t dst, int32_t algo, int64_t *arc_flow)
{
    if (n_vertices <= 0 || n_arcs < 0 || src < 0 || dst < 0 || src >= n_vertices || dst >= n_vertices)
        return -1;
    for (int64_t i = 0; i < n_arcs; ++i)
        if (tail[i] < 0 || tail[i] >= n_vertices || head[i] < 0 || head[i] >= n_vertices || cap[i] < 0)
            return -1;
    net_t g;
    if (net_build(&g, n_vertices, n_arcs, tail, head, cap) != 0) return -1;
    int64_t f = algo == 0 ? dinic(&g, src, dst) : edmonds_karp(&g, src, dst);
    if (arc_flow)
        for (int64_t i = 0; i < n_arcs; ++i) arc_flow[i] = g.res[2 * i + 1];  /* flow = residual of the back arc */
    net_free(&g);
    return f;
}

/* ---------------------------------------------------------------- exported: batch over the auxiliary network
 *
 * For problem j: build the auxiliary network of Section 5.2 explicitly -- vertices
 * V + {s} with s = n_vertices, every topology arc e with capacity U_j * b_e, and an
 * arc (s, c) of capacity k_j for every compute node c (the sink included) -- and
 * return F(s, sink_j).  Problems are split statically over n_threads POSIX threads,
 * the paper's own parallelisation over sinks (Appendix C).
 */
typedef struct {
    int32_t n_vertices; int64_t n_arcs;
    const int32_t *tail, *head, *bandwidth; const uint8_t *is_compute;
    const int32_t *sink; const int64_t *U, *k; int64_t *flow_out;
    const int64_t *U_den;              /* null: U_j is an integer; else the multiplier is U_j / U_den_j, floored per arc */
    int64_t first, last; int32_t algo; int32_t n_compute;
} batch_job_t;

static void *batch_worker(void *arg)
{
    batch_job_t *job = (batch_job_t *)arg;
    int64_t m = job->n_arcs + job->n_compute;
    int32_t n = job->n_vertices + 1, s = job->n_vertices;
    int32_t *t2 = (int32_t *)malloc(sizeof(int32_t) * (size_t)(m + 1));
    int32_t *h2 = (int32_t *)malloc(sizeof(int32_t) * (size_t)(m + 1));
    int64_t *c2 = (int64_t *)malloc(sizeof(int64_t) * (size_t)(m + 1));
    for (int64_t j = job->first; j < job->last; ++j) {
        int64_t p = 0;
        for (int64_t i = 0; i < job->n_arcs; ++i, ++p) {
            t2[p] = job->tail[i]; h2[p] = job->head[i]; c2[p] = job->U[j] * (int64_t)job->bandwidth[i];
            if (job->U_den) c2[p] /= job->U_den[j];       /* nonnegative operands: C division is the floor */
        }
        for (int32_t v = 0; v < job->n_vertices; ++v)
            if (job->is_compute[v]) { t2[p] = s; h2[p] = v; c2[p] = job->k[j]; ++p; }
        job->flow_out[j] = fco_maxflow(n, m, t2, h2, c2, s, job->sink[j], job->algo, NULL);
    }
    free(t2); free(h2); free(c2);
    return NULL;
}

static int32_t batch_run(int32_t n_vertices, int64_t n_arcs, const int32_t *tail,
                         const int32_t *head, const int32_t *bandwidth,
                         const uint8_t *is_compute, int64_t n_problems, const int32_t *sink,
                         const int64_t *U, const int64_t *U_den, const int64_t *k, int64_t *flow_out,
                         int32_t algo, int32_t n_threads)
{
    if (n_threads < 1) n_threads = 1;
    if (n_threads > 256) n_threads = 256;
    int32_t n_compute = 0;
    for (int32_t v = 0; v < n_vertices; ++v) n_compute += is_compute[v] ? 1 : 0;
    batch_job_t jobs[256]; pthread_t th[256];
    int64_t per = (n_problems + n_threads - 1) / n_threads;
    for (int32_t t = 0; t < n_threads; ++t) {
        batch_job_t *jb = &jobs[t];
        jb->n_vertices = n_vertices; jb->n_arcs = n_arcs; jb->tail = tail; jb->head = head;
        jb->bandwidth = bandwidth; jb->is_compute = is_compute; jb->sink = sink; jb->U = U; jb->k = k;
        jb->U_den = U_den;
        jb->flow_out = flow_out; jb->algo = algo; jb->n_compute = n_compute;
        jb->first = t * per < n_problems ? t * per : n_problems;
        jb->last = (t + 1) * per < n_problems ? (t + 1) * per : n_problems;
    }
    if (n_threads == 1) { batch_worker(&jobs[0]); return 0; }
    for (int32_t t = 0; t < n_threads; ++t)
        if (pthread_create(&th[t], NULL, batch_worker, &jobs[t]) != 0) return -1;
    for (int32_t t = 0; t < n_threads; ++t) pthread_join(th[t], NULL);
    return 0;
}

int32_t fco_aux_maxflow_batch(int32_t n_vertices, int64_t n_arcs, const int32_t *tail,
                              const int32_t *head, const int32_t *bandwidth,
                              const uint8_t *is_compute, int64_t n_problems, const int32_t *sink,
                              const int64_t *U, const int64_t *k, int64_t *flow_out,
                              int32_t algo, int32_t n_threads)
{
    return batch_run(n_vertices, n_arcs, tail, head, bandwidth, is_compute, n_problems, sink, U, NULL, k,
                     flow_out, algo, n_threads);
}

/* The same batch on the network of the fixed-k test (Algorithm 3, Appendix E.4): a rational
 * multiplier U_j = U_num_j / U_den_j and every topology arc e with capacity floor(U_j * b_e);
 * source arcs k_j as before.  U_num_j * b_e must fit int64 (the caller checks). */
int32_t fco_aux_maxflow_batch_floor(int32_t n_vertices, int64_t n_arcs, const int32_t *tail,
                                    const int32_t *head, const int32_t *bandwidth,
                                    const uint8_t *is_compute, int64_t n_problems, const int32_t *sink,
                                    const int64_t *U_num, const int64_t *U_den, const int64_t *k,
                                    int64_t *flow_out, int32_t algo, int32_t n_threads)
{
    for (int64_t j = 0; j < n_problems; ++j) if (U_den[j] < 1) return -1;
    return batch_run(n_vertices, n_arcs, tail, head, bandwidth, is_compute, n_problems, sink, U_num, U_den, k,
                     flow_out, algo, n_threads);
}
