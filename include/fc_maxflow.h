/*
 * fc_maxflow.h -- C ABI of the batched integer max-flow feasibility library for
 * AMD MI355X (gfx950).
 *
 * The library implements the data-parallel hot path of ForestColl's schedule
 * generator (arXiv 2402.06787): the max-flow tests of the optimality search.
 * Notation follows the paper's Appendix A: G = (V = V_s u V_c, E) is the topology
 * digraph with integer link bandwidths b_e, N = |V_c| compute nodes, s the auxiliary
 * super-source, x the per-node broadcast bandwidth, k the source-arc capacity of the
 * integer network, U the edge-capacity multiplier (candidate 1/x = U/k), F(a,b;D) a
 * max-flow value.
 *
 * Conventions
 *  - Every function returns FC_OK (0) or a negative FC_E* code; outputs are not
 *    written on error unless stated.  Nothing throws or aborts across this boundary.
 *  - "host" pointers are ordinary CPU memory, borrowed for the duration of the call.
 *    "device" pointers are HIP device memory on the GPU that was current when the
 *    graph was uploaded; the caller owns them and keeps them alive until the work
 *    queued on `hip_stream` has finished.
 *  - `hip_stream` is a hipStream_t passed as void* (NULL = the default stream).
 *  - An fc_graph's topology is immutable after creation and it may be shared by concurrent
 *    calls on different streams as long as each call has its own workspace.  An uploaded graph
 *    also carries one scheduling hint per vertex (what the last max-flow into that sink cost),
 *    which the solver updates and the next call uses to start the expensive problems first; it
 *    affects the order problems run in, never a result, and concurrent calls may overwrite each
 *    other's hints freely.
 */
#ifndef FC_MAXFLOW_H
#define FC_MAXFLOW_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define FC_OK             0
#define FC_EINVAL        -1   /* null pointer, id out of range, negative bandwidth, N < 2, bad option  */
#define FC_EOVERFLOW     -2   /* a quantity does not fit the integer type the device path uses         */
#define FC_EDISCONNECTED -3   /* some compute node cannot reach another: the bound (star) is infinite  */
#define FC_ENOMEM        -4   /* host allocation failed                                                */
#define FC_EWORKSPACE    -5   /* workspace pointer null or smaller than *_workspace_bytes reports      */
#define FC_EDEVICE       -6   /* a HIP call failed, or no usable GPU / the graph is not on the device  */
#define FC_ENOCONVERGE   -7   /* a safety cap on device iterations was hit (indicates a bug)           */
#define FC_EUNSUPPORTED  -8   /* graph too large for the on-chip state layout of this build            */

/* value written to flow_out[j] when problem j itself is invalid (sink out of range, U < 1,
 * k < 1, or N*k >= 2^31); valid flows are always >= 1 */
#define FC_FLOW_INVALID     ((int32_t)-1)
/* the safety cap on device iterations was hit for problem j (a bug; never expected) */
#define FC_FLOW_NOCONVERGE  ((int32_t)-2)
/* N*k_j > 65535 needs the 32-bit on-chip layout, which does not fit this graph */
#define FC_FLOW_UNSUPPORTED ((int32_t)-3)

typedef struct fc_graph fc_graph;                  /* opaque; owned by the library            */
typedef struct { int64_t num, den; } fc_rational;  /* always reduced, den > 0                  */

/* Work counters summed over the problems of one call (all optional). */
typedef struct {
    uint64_t pushes;           /* residual-edge updates: one per (arc, push)                          */
    uint64_t relabels;         /* single-vertex height increases by the discharge step                */
    uint64_t arc_scans;        /* residual arcs examined by discharge steps                           */
    uint64_t global_relabels;  /* backward breadth-first relabelings from the sink                    */
    uint64_t gr_arc_scans;     /* residual arcs examined by those                                     */
    uint64_t level_steps;      /* discharge steps (one height level of one problem each)              */
    uint64_t discharges;       /* vertex discharges                                                   */
    uint64_t not_converged;    /* problems that hit the iteration cap (must be 0)                     */
    float    device_ms;        /* duration of the call's kernels, HIP events on `hip_stream`          */
} fc_stats;

/* Tuning knobs; zero-initialise and override what you need (0 = library default). */
typedef struct {
    int32_t threads_per_problem;   /* workgroup size, multiple of 64 in [64, 1024] (default: 256 when fewer
                                      than 8 problems fit a CU's LDS, else 128, 64 below 256 vertices)   */
    int32_t lanes_per_vertex;      /* power of two in [2, 64]: lanes that scan one vertex's arc list (default:
                                      the power of two next to a residual row's length -- the row a random
                                      arc lies in for the (sink, candidate) launches, the average row elsewhere) */
    int32_t global_relabel_steps;  /* relabel from the sink when this many level steps passed since
                                      the last one and some vertex was relabeled (default 32; launches of
                                      fc_construct_trees from kept flows: 4)                             */
    int32_t global_relabel_permille; /* ... or when relabels since then reach this fraction of |V|     */
    int32_t global_relabel_rises;  /* ... or when the working height level moved up this many times since
                                      then (-1: off; default: off, except fc_split_gamma_batch and
                                      fc_remove_switches on graphs of 256 vertices or more: 2, and tree
                                      launches from kept flows: 1)                                     */
    int32_t tight_sink_percent;    /* a problem whose sink cut U*B^-(t) (+k) is below this percentage of the
                                      demand N*k relabels from the sink the first time the working level
                                      moves up (default 200, -1: off)                                  */
    int32_t use_gap;               /* 1 = on (default), 2 = off: empty-height-level cut detection      */
    int32_t use_label_table;       /* 1 = on (default), 2 = off: initial exact labels from the
                                      per-sink distance table built at upload                          */
    int32_t force_wide;            /* 1 = always use 32-bit on-chip state (default: 16-bit when it fits) */
    int32_t max_level_steps;       /* safety cap per problem (default max(100000, 200*|V|))            */
    int32_t src_cap_bound;         /* > 0: the caller promises k_j <= this for every problem of the call.
                                      If N * bound <= 65535 only the 16-bit-state kernel is launched;
                                      a problem that breaks the promise gets FC_FLOW_UNSUPPORTED        */
    int32_t tree_certificate;      /* 1 = on, 2 = off (default off; fc_opt_throughput_search: default on).  At
                                      upload every sink gets a spanning in-tree of first arcs; a problem in
                                      which that tree alone can carry k units from every compute node within
                                      the capacities U * b_e has F = N * k, the most s can emit, and is
                                      answered from a per-sink ratio without running the solver (its
                                      counters stay 0).  Exact; it only skips work.                      */
    int32_t schedule;              /* 1 = on (default), 2 = off: start the problems that look hardest (least
                                      slack in the sink's own cut) first, so the launch has no long tail (a
                                      launch whose workgroups all fit the device at once is not ordered)  */
    int32_t tree_warm_start;       /* fc_construct_trees: 1 = on (default), 2 = off.  On: while a root-set grows, the
                                      flow that delivers the other root-sets' demands to a vertex y is kept on the
                                      device from launch to launch, repaired for the capacities that were used up
                                      since, and only the few units that decide mu are routed anew.  Off: every
                                      max-flow starts from nothing.  Same trees either way.                  */
    int32_t split_two_launches;    /* edge splitting: 1 = on, 2 = off.  On: the 2N max-flows of a pair are solved in two
                                      launches -- first the two problems without the compute node v, whose final
                                      preflows are kept; then the 2N with v, each of which is answered at once where
                                      the problem without v reached the value that settles gamma (one more sink never
                                      lowers a flow) and otherwise goes on from the kept preflow.  Same values.
                                      Default: on for a batch with at least twice as many max-flows as the device
                                      holds workgroups at a time (a smaller batch lasts as long as its slowest
                                      problem either way, and a second launch only adds to that)               */
    int32_t stats_time_only;       /* fc_maxflow_batch(_floor), fc_feasible(_floor) with stats: 1 = fill device_ms only.  The
                                      kernels then run exactly as without stats (counting costs a few per cent: every
                                      problem adds its counters up on chip and writes 32 bytes); the counters read 0  */
    int32_t split_carry;           /* fc_remove_switches: 1 = on (default), 2 = off.  On: while one switch is split, the preflow
                                      each (ingress link, type) problem without v ended with is kept on the device and the
                                      next batch's problem goes on from it, cut down to the new capacities and repaired,
                                      instead of starting from nothing.  Same D* and table either way.                  */
    int32_t split_reverse;         /* edge splitting in two launches: 1 = on, 2 = off (default: on unless the flow values are
                                      asked for).  On: a problem of the second launch gives the new sink v the units that
                                      still matter and pushes them backwards along the residual arcs to the excess the
                                      first launch left stranded, instead of moving all that excess towards v.  Same values. */
    int32_t tree_chain_states;     /* fc_construct_trees: states one launch looks ahead, 1 to 64 (default 32; 64 on
                                      digraphs of 1024 vertices or more; see there)                                       */
} fc_options;

/* ------------------------------------------------------------------------------------------
 * Graph ingest (the paper's problem definition, Section 5: a directed graph with integer link
 * bandwidths whose vertices are compute nodes V_c and switch nodes V_s).
 *
 * tail/head/bandwidth: host arrays of n_arcs directed arcs (tail -> head).  Vertex ids are
 * 0..n_vertices-1; the super-source s is implicit and never listed.  Parallel arcs are allowed
 * and their bandwidths add (integer capacity = number of multi-edges, Appendix E.1);
 * self-loops and zero-bandwidth arcs are ignored; antiparallel arcs are independent.  The
 * graph need not be Eulerian for the calls below.  is_compute: host array [n_vertices],
 * non-zero = compute node.
 *
 * fc_graph_build   : host-side part only (validation, merging, residual CSR); needs no GPU.
 * fc_graph_upload  : fc_graph_build + copy to the current HIP device + the per-sink tables (initial heights and
 *                    first-arc trees per sink, built by a kernel on the device; see fc_graph_sink_table).
 * Errors: FC_EINVAL (null pointers, ids out of range, negative bandwidth, fewer than two
 * compute nodes, n_vertices < 2), FC_EOVERFLOW (a merged bandwidth or an in-bandwidth sum
 * reaches 2^31), FC_ENOMEM, FC_EDEVICE, FC_EUNSUPPORTED (per-problem state exceeds on-chip memory).
 * On success *out owns host and device memory until fc_graph_free.
 */
int fc_graph_build(int32_t n_vertices, int64_t n_arcs, const int32_t *tail, const int32_t *head,
                   const int32_t *bandwidth, const uint8_t *is_compute, fc_graph **out);
int fc_graph_upload(int32_t n_vertices, int64_t n_arcs, const int32_t *tail, const int32_t *head,
                    const int32_t *bandwidth, const uint8_t *is_compute, fc_graph **out);
int fc_graph_free(fc_graph *g);

/* In-place bandwidth update of a graph that is already built or uploaded.  The edge-splitting loop (Appendix E.2,
 * the algorithm that removes the switch nodes) changes three capacities per split -- c(u, w) and c(w, t) go down by
 * gamma, c(u, t) goes up by gamma -- and asks for max-flows on the changed graph right away; what-if questions about a
 * degraded or upgraded link are of the same kind.  This call rewrites the bandwidth of existing links where they
 * lie: the residual CSR keeps its shape, its record numbering (fc_graph_csr) and its device addresses, and nothing
 * is allocated beyond a staging list of 8 bytes per changed record that the graph keeps for later calls.
 *
 * tail, head, bandwidth: host int32 [n_updates].  Link (tail[i], head[i]) -- one ordered vertex pair, as after the
 * merging of parallel arcs -- gets the bandwidth bandwidth[i] >= 0 (the new value, not a difference; when a link is
 * listed twice the later entry wins).  A link lowered to 0 stays in the CSR as a pair of records that carry nothing
 * and can be raised again.  A link that the graph does not have cannot be given bandwidth, because that would move
 * records: build the graph with fc_graph_upload_with_spares, which is fc_graph_upload except that an arc of
 * bandwidth 0 becomes such a link instead of being ignored (parallel arcs still add; self-loops are still ignored).
 * For the edge-splitting loop the spares are the links (u, t) over the ingress tails u and egress heads t of a switch.
 *
 * The facts fc_graph_info reports (min B^-, max b_e, gcd, Eulerian flag) follow the update.  The per-sink tables of
 * the uploaded graph (initial heights, first-arc trees: functions of the bandwidths) are
 *   refresh_tables = 1: rebuilt by the same kernel as in fc_graph_upload; every later call then behaves exactly as
 *                       on a fresh upload of the updated arc list;
 *   refresh_tables = 0: marked unusable until a later call with refresh_tables = 1: the solver kernels then start
 *                       each problem with a search for exact heights on the device instead.  Same values, slower
 *                       batches, a much cheaper update: the choice for loops that change the graph between launches.
 * Synchronous: waits for `hip_stream` first (launches that still read the records), returns when the device copy
 * is up to date.  Must not run concurrently with other calls on the same graph.  A graph from fc_graph_build gets
 * the host part only.
 * Errors: FC_EINVAL (null pointers, ids out of range, negative bandwidth, a link the graph does not have,
 * refresh_tables not 0 or 1), FC_EOVERFLOW (an in-bandwidth sum reaches 2^31) -- in both cases nothing was changed;
 * FC_ENOMEM; FC_EDEVICE (also: the graph lives on another GPU than the current one) -- after a device error during
 * the update the graph must only be freed. */
int fc_graph_upload_with_spares(int32_t n_vertices, int64_t n_arcs, const int32_t *tail, const int32_t *head,
                                const int32_t *bandwidth, const uint8_t *is_compute, fc_graph **out);
int fc_graph_update_arcs(fc_graph *g, int64_t n_updates, const int32_t *tail, const int32_t *head,
                         const int32_t *bandwidth, int32_t refresh_tables, void *hip_stream);

/* Facts Algorithm 1 and Proposition 3 need: N = |V_c|; number of arcs after merging;
 * min over compute nodes of the in-bandwidth B^-_G(v); max_e b_e; gcd of all b_e; whether
 * every vertex has equal in- and out-bandwidth (the paper's Eulerian assumption, needed only
 * by later stages).  Any output pointer may be null. */
int fc_graph_info(const fc_graph *g, int32_t *n_compute, int64_t *n_arcs_merged,
                  int64_t *min_in_bw_compute, int32_t *max_bw, int32_t *gcd_bw, int32_t *is_eulerian);

/* Non-uniform allgather / reduce-scatter (Section 5.7, "Other Collective Operations"): when compute
 * nodes send different amounts of data the capacities of s's arcs are adjusted.  Reading taken here:
 * compute node c has an integer weight m_c >= 0, its arc (s, c) has capacity m_c * k_j instead of k_j,
 * and N * k_j becomes k_j * (sum of the weights) wherever it appears -- the verdict's threshold, the
 * clamp of the capacities, the validity bound (< 2^31) and the 16-bit limit (<= 65535).
 *
 * weight_per_vertex: host int32 [n_vertices] (entries of switch nodes are ignored), or null to return
 * to unit weights.  The weights stay with the graph and apply to every later fc_maxflow_batch,
 * fc_maxflow_batch_floor, fc_feasible and fc_feasible_floor call; the tree certificate is not used
 * while they are set.  The searches and the edge-splitting calls, which the paper defines for unit
 * weights only, return FC_EUNSUPPORTED while they are set.  Synchronous (one small copy); must not
 * run concurrently with other calls on the same graph.
 * Errors: FC_EINVAL (negative weight, all weights zero), FC_EOVERFLOW (sum >= 2^31), FC_EDEVICE
 * (graph not uploaded, copy failed), FC_ENOMEM. */
int fc_graph_set_source_weights(fc_graph *g, const int32_t *weight_per_vertex);

/* Residual CSR as built on the host (for inspection and tests).  Vertex u owns records
 * row_ptr[u] .. row_ptr[u+1]-1; record r describes a residual arc u -> other[r] that belongs to
 * merged topology arc pair[r] of bandwidth bw[r]; forward[r] = 1 if the topology arc leaves u,
 * 0 if it enters u.  Pass null to skip an array; sizes: row_ptr [n_vertices+1], others
 * [2 * n_arcs_merged]. */
int fc_graph_csr(const fc_graph *g, int32_t *row_ptr, int32_t *other, int32_t *pair,
                 int32_t *bw, uint8_t *forward);

/* The per-sink tables of an uploaded graph as the device holds them, for inspection and tests (synchronous copies
 * from the current device).  For the vertex `sink` taken as the sink of a max-flow (Section 5.2: every compute node
 * is one in turn), before any flow has been pushed:
 *   label[v]        [n_vertices]  breadth-first distance from v to sink over links of positive bandwidth (n_vertices:
 *                                 cannot reach it) -- the exact initial heights of push-relabel;
 *   *label_hmax                   the largest finite label of a compute node;
 *   level_table     [64]          [0] = deepest level L, [1 + j] = where level L - j starts in the order below,
 *                                 [1 + L] = where the order ends;
 *   order_vertex[i], first_head[i], first_pair[i], first_bw[i]   [n_vertices]  the i-th vertex by decreasing label (ties
 *                                 by id) and the link along which its excess is sent first: head, merged-arc number
 *                                 (as in fc_graph_csr) and bandwidth; entries past the order's end are 0.  The first
 *                                 links form a spanning in-tree of the vertices that reach the sink, every link
 *                                 going exactly one level down;
 *   ratio           [2]           {num, den}: the largest (compute nodes in the subtree of v) / (bandwidth of v's first
 *                                 link) over that tree, den = 0 if some compute node cannot reach the sink -- the
 *                                 first-arc tree certificate: if k * num <= U * den, the tree alone carries N * k.
 * *have: bit 0 = labels exist (label, label_hmax are filled), bit 1 = the level order exists (the rest is filled):
 * large graphs (more than 8192 / 4096 vertices), sinks deeper than 62 levels, and graphs whose tables were switched
 * off by fc_graph_update_arcs have fewer.  Any output pointer but `have` may be null.
 * Errors: FC_EINVAL, FC_EDEVICE (graph not uploaded, copy failed), FC_ENOMEM. */
int fc_graph_sink_table(const fc_graph *g, int32_t sink, int32_t *have, int32_t *label, int32_t *label_hmax,
                        int32_t *level_table, int32_t *order_vertex, int32_t *first_head, int32_t *first_pair,
                        int32_t *first_bw, int32_t *ratio);

/* ------------------------------------------------------------------------------------------
 * fc_maxflow_batch -- many independent max-flows on the auxiliary network (Section 5.2,
 * Appendix E.1): problem j adds s with an arc (s, c) of capacity src_cap[j] = k_j for every
 * compute node c (the sink included), gives every topology arc e capacity edge_mult[j] * b_e
 * = U_j * b_e, and asks for F(s, sink[j]).  By the min-cut theorem that value is unique.
 *
 * d_sink, d_edge_mult, d_src_cap: device int32 [n_problems].  d_flow_out: device int32
 * [n_problems]; entry j receives F(s, sink_j) (>= k_j when sink_j is a compute node), or
 * FC_FLOW_INVALID if problem j is malformed (sink not a vertex, U_j < 1, k_j < 1,
 * N * k_j >= 2^31).  U_j * b_e may exceed 32 bits: capacities are clamped at N * k_j, which
 * cannot change the value.  The call is asynchronous on `hip_stream` unless `stats` is
 * non-null, in which case it synchronises the stream and fills *stats.
 * d_workspace: device scratch of at least fc_maxflow_batch_workspace_bytes(g, n_problems)
 * bytes, 256-byte aligned; contents are undefined afterwards; it may be reused by later
 * calls on the same stream.  n_problems == 0 is valid and does nothing.
 * Errors: FC_EINVAL, FC_EWORKSPACE, FC_EDEVICE; with stats: FC_ENOCONVERGE.
 */
size_t fc_maxflow_batch_workspace_bytes(const fc_graph *g, int64_t n_problems);
int fc_maxflow_batch(const fc_graph *g, int64_t n_problems, const int32_t *d_sink,
                     const int32_t *d_edge_mult, const int32_t *d_src_cap, int32_t *d_flow_out,
                     void *d_workspace, size_t workspace_bytes, void *hip_stream,
                     const fc_options *options_or_null, fc_stats *stats_or_null);

/* fc_maxflow_batch_static -- fc_maxflow_batch for callers that cannot allocate device memory: code that runs
 * under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same problems, same values;
 * the scratch the batch needs (the launch order that starts the expensive problems first, and its sort keys)
 * lives in a static array in the library's device image, 5 bytes per problem for at most
 * FC_MAXFLOW_BATCH_STATIC_MAX_PROBLEMS problems (1.25 MiB, held on every GPU the library runs on until the
 * process ends).  The call allocates and frees nothing, on the host side of the device or on the device, and
 * takes no workspace and no stats (counters need per-problem scratch and a synchronisation).
 * Arguments as for fc_maxflow_batch; asynchronous on `hip_stream`.  The graph must live on the current device.
 * All calls on one GPU share that GPU's array: two calls that overlap in time on one GPU (different streams,
 * different host threads) race on it and may run their problems in a poor order or skip some -- serialise them,
 * or use fc_maxflow_batch with a workspace per call.  Nothing in the array has to be cleared between calls.
 * Errors: FC_EWORKSPACE (n_problems above the maximum), FC_EINVAL, FC_EDEVICE (also: the graph is on another
 * GPU than the current one), FC_EUNSUPPORTED. */
#define FC_MAXFLOW_BATCH_STATIC_MAX_PROBLEMS 262144
int fc_maxflow_batch_static(const fc_graph *g, int64_t n_problems, const int32_t *d_sink,
                            const int32_t *d_edge_mult, const int32_t *d_src_cap, int32_t *d_flow_out,
                            void *hip_stream, const fc_options *options_or_null);

/* ------------------------------------------------------------------------------------------
 * fc_feasible -- the verdict of Theorem 1 in its integer form (Theorem 3 / Appendix E.1) for
 * each candidate j = (U_j, k_j):   feasible_j  <=>  min over v in V_c of F(s, v) >= N * k_j.
 * Runs N max-flows per candidate (every compute node as sink) in one batch.
 *
 * d_edge_mult, d_src_cap: device int32 [n_candidates].  d_feasible_out: device uint8
 * [n_candidates], 1 / 0 (0 also for malformed candidates).  d_witness_sink_or_null: device
 * int32 [n_candidates]: the smallest compute-node id v with F(s, v) < N * k_j, or -1.
 * d_flows_or_null: device int32 [n_candidates * N], candidate-major, compute nodes in
 * increasing id order: all per-sink flow values.  Workspace as above with
 * fc_feasible_workspace_bytes.  Asynchronous unless stats is non-null.
 */
size_t fc_feasible_workspace_bytes(const fc_graph *g, int32_t n_candidates);
int fc_feasible(const fc_graph *g, int32_t n_candidates, const int32_t *d_edge_mult,
                const int32_t *d_src_cap, uint8_t *d_feasible_out, int32_t *d_witness_sink_or_null,
                int32_t *d_flows_or_null, void *d_workspace, size_t workspace_bytes,
                void *hip_stream, const fc_options *options_or_null, fc_stats *stats_or_null);

/* ------------------------------------------------------------------------------------------
 * fc_opt_throughput_search -- the result of Algorithm 1 (Optimality Binary Search) and of
 * Proposition 3:  1/x* = max over cuts S of |S n V_c| / B^+(S) as the reduced fraction p/q,
 * then U = p / gcd(q, {b_e}) and k = q / gcd(q, {b_e}).
 *
 * The answer is unique, so any exact monotone search over Theorem 1's verdict returns it.
 * Instead of the paper's bisection (whose dyadic midpoints need ever larger integers) this
 * driver walks the Stern-Brocot tree between the paper's bounds (N-1)/B and N-1,
 * B = min over compute nodes of B^-(v), testing up to `candidates_per_round` fractions of
 * denominator <= B per fc_feasible round, so all device integers stay below 2^31.
 * Synchronous; allocates its own device scratch; results go to host memory.
 *
 * trace_* (optional, host, capacity trace_capacity): every candidate (U, k) evaluated and its
 * verdict, in evaluation order; *trace_len_or_null receives the total number evaluated (which
 * may exceed trace_capacity).  Errors: FC_EDISCONNECTED (candidate N-1 is infeasible),
 * FC_EOVERFLOW, FC_EINVAL, FC_EDEVICE, FC_ENOMEM.
 */
int fc_opt_throughput_search(const fc_graph *g, int32_t candidates_per_round,
                             fc_rational *inv_xstar, fc_rational *U, int64_t *k,
                             int32_t *rounds_or_null, void *hip_stream,
                             const fc_options *options_or_null,
                             int32_t *trace_U, int32_t *trace_k, uint8_t *trace_verdict,
                             int32_t trace_capacity, int32_t *trace_len_or_null);

/* The search logic alone, with the verdict supplied by the caller (host only, no GPU):
 * `verdicts(ctx, n, U, k, out)` must set out[i] = 1 iff candidate U[i]/k[i] >= 1/x*, and return
 * FC_OK or an error code, which is passed through.  n_compute = N, min_in_bw = B, gcd_bw =
 * gcd{b_e}.  fc_opt_throughput_search is this function with fc_feasible as the callback. */
typedef int (*fc_verdict_fn)(void *ctx, int32_t n, const int32_t *U, const int32_t *k, uint8_t *out);
int fc_search_with_verdicts(int32_t n_compute, int64_t min_in_bw, int32_t gcd_bw,
                            int32_t candidates_per_round, fc_verdict_fn verdicts, void *ctx,
                            fc_rational *inv_xstar, fc_rational *U, int64_t *k,
                            int32_t *rounds_or_null);

/* ------------------------------------------------------------------------------------------
 * Fixed k (Section 5.5, Appendix E.4, Algorithm 3).  With k trees per compute node fixed, a real
 * multiplier U is achievable iff  min over v in V_c of F(s, v) >= N * k  in the network whose
 * topology arcs have capacity floor(U * b_e) and whose arcs (s, c) have capacity k (Theorems 11
 * and 12); the communication time is M / (N k) * U.  A "link" e is one ordered vertex pair with the
 * summed bandwidth of its parallel input arcs, as everywhere in this library; the floor is per link.
 *
 * fc_maxflow_batch_floor / fc_feasible_floor are fc_maxflow_batch / fc_feasible with the rational
 * multiplier U_j = mult_num[j] / mult_den[j] (device int32 arrays; a problem or candidate with
 * mult_den < 1 is malformed like one with mult_num < 1).  Everything else -- outputs, workspace
 * sizes (the same *_workspace_bytes functions), stream and error behaviour -- is as above; the
 * tree_certificate option has no effect here.
 *
 * fc_fixed_k_search: U* = 1 / y*, the smallest achievable U for this k, as a reduced fraction;
 * its denominator is at most max_e b_e because some U* b_e is an integer.  Same search driver,
 * trace arguments and errors as fc_opt_throughput_search (trace_num / trace_den hold the tested
 * multipliers); FC_EOVERFLOW when (N - 1) * k * max_e b_e or N * k does not fit 31 bits.
 * fc_fixed_k_search_with_verdicts is the host-only search logic: `verdicts(ctx, n, num, den, out)`
 * must set out[i] = 1 iff num[i] / den[i] >= U*. */
int fc_maxflow_batch_floor(const fc_graph *g, int64_t n_problems, const int32_t *d_sink,
                           const int32_t *d_mult_num, const int32_t *d_mult_den, const int32_t *d_src_cap,
                           int32_t *d_flow_out, void *d_workspace, size_t workspace_bytes, void *hip_stream,
                           const fc_options *options_or_null, fc_stats *stats_or_null);
int fc_feasible_floor(const fc_graph *g, int32_t n_candidates, const int32_t *d_mult_num,
                      const int32_t *d_mult_den, const int32_t *d_src_cap, uint8_t *d_feasible_out,
                      int32_t *d_witness_sink_or_null, int32_t *d_flows_or_null, void *d_workspace,
                      size_t workspace_bytes, void *hip_stream, const fc_options *options_or_null,
                      fc_stats *stats_or_null);
int fc_fixed_k_search(const fc_graph *g, int32_t k, int32_t candidates_per_round, fc_rational *U_star,
                      int32_t *rounds_or_null, void *hip_stream, const fc_options *options_or_null,
                      int32_t *trace_num, int32_t *trace_den, uint8_t *trace_verdict, int32_t trace_capacity,
                      int32_t *trace_len_or_null);
int fc_fixed_k_search_with_verdicts(int32_t n_compute, int64_t min_in_bw, int32_t max_bw, int32_t k,
                                    int32_t candidates_per_round, fc_verdict_fn verdicts, void *ctx,
                                    fc_rational *U_star, int32_t *rounds_or_null);

/* ------------------------------------------------------------------------------------------
 * Edge splitting (Appendix E.2, the theorem that gives the maximum capacity gamma that can be split off).  D is the uploaded graph with every link capacity
 * multiplied by the integer U (the stage works on G({U b_e}); rescale the bandwidths first when
 * Proposition 3's U is a fraction), k the number of trees per compute node.  For pair i,
 * e = (u_i, w_i), f = (w_i, t_i) with w_i a switch node, gamma_i is the most capacity of e and f that can
 * be replaced by a direct arc (u_i, t_i) while  min over v in V_c of F(s, v) >= N k  keeps holding:
 *   gamma = min{ c(e), c(f),  min_v F(u, w; D_k + unbounded arcs (u,s), (u,t), (v,w)) - N k,
 *                             min_v F(w, t; D_k + unbounded arcs (w,s), (u,t), (v,t)) - N k },
 * 2N max-flows per pair, all pairs in one launch.  The theorem assumes D Eulerian (fc_graph_info
 * reports it) and the condition holding in D; neither is checked -- gamma is then just the formula.
 *
 * d_u, d_w, d_t: device int32 [n_pairs].  d_gamma_out: device int32 [n_pairs]; FC_GAMMA_INVALID for a pair
 * that is not two links through a switch node.  d_flows_or_null: device int32 [n_pairs][2][N], the two
 * families of flows in compute-node order; "unbounded" (a path of unbounded arcs exists) is reported as
 * the one value U * (sum of all b_e) + N k + 1, which exceeds every finite cut.  That value must stay
 * below 2^30 (FC_EOVERFLOW), and the 32-bit on-chip state must fit (FC_EUNSUPPORTED).  When the flows are
 * not asked for, a max-flow ends as soon as N k + min{c(e), c(f)} units have arrived -- from there on it
 * cannot be the term that decides gamma -- so gamma is the same and the work is much less; with
 * d_flows every value is the exact maximum.  Workspace, stream, options and stats as for
 * fc_maxflow_batch (no first-pass tables, launch order or certificate apply to these problems).  A large
 * batch is solved in two launches (options->split_two_launches): then the counters and the device time in
 * stats are those of the second launch, and a problem that the first launch settled counts no work at all. */
#define FC_GAMMA_INVALID (-2147483647 - 1)
size_t fc_split_gamma_workspace_bytes(const fc_graph *g, int64_t n_pairs);
int fc_split_gamma_batch(const fc_graph *g, int32_t U, int32_t k, int64_t n_pairs, const int32_t *d_u,
                         const int32_t *d_w, const int32_t *d_t, int32_t *d_gamma_out, int32_t *d_flows_or_null,
                         void *d_workspace, size_t workspace_bytes, void *hip_stream,
                         const fc_options *options_or_null, fc_stats *stats_or_null);

/* Algorithm 2 (Remove Switch Nodes, Appendix E.2) on the integer-capacity Eulerian digraph D given as host
 * arrays (capacity = number of multi-edges; parallel arcs add, self-loops and zero capacities are ignored): for
 * every switch w, every egress link f = (w, t) and every ingress link e = (u, w), in increasing id order, split
 * off gamma (fc_split_gamma_batch, U = 1) when it is positive.  Outputs (host, caller-allocated): the links of the
 * compute-only digraph D* and the path recovery table as rows (u, t, w, amount): `amount` of the capacity of
 * (u, t) was routed through switch w.  *n_out / *n_routes receive the row counts; if a capacity argument is too
 * small the call returns FC_EWORKSPACE with the counts set and nothing else written.  n_batches_or_null counts the
 * gamma launches.  Every batch re-uploads the current graph, so this is a driver for graphs that fit the 32-bit
 * on-chip state, not a tuned stage.  Errors: FC_EINVAL (also: D not Eulerian), FC_ENOCONVERGE (an egress link
 * could not be used up: min_v F(s, v) >= N k did not hold in D), FC_EOVERFLOW, FC_EUNSUPPORTED, FC_EDEVICE, FC_ENOMEM. */
int fc_remove_switches(int32_t n_vertices, int64_t n_arcs, const int32_t *tail, const int32_t *head,
                       const int32_t *capacity, const uint8_t *is_compute, int32_t k,
                       int64_t out_capacity, int64_t *n_out, int32_t *out_tail, int32_t *out_head, int32_t *out_cap,
                       int64_t route_capacity, int64_t *n_routes, int32_t *route_u, int32_t *route_t,
                       int32_t *route_w, int32_t *route_amount, int64_t *n_batches_or_null,
                       void *hip_stream, const fc_options *options_or_null);

const char *fc_strerror(int code);

/* ------------------------------------------------------------------------------------------
 * Spanning tree construction (Appendix E.3) on the compute-only digraph D* that switch removal leaves.
 * The state of the construction is: the remaining capacity g(e) of every link, and root-sets R_i with
 * demands m(R_i) (R_i = the vertices the m(R_i) identical out-trees of some root span so far).  An edge
 * (x, y) with x in R_grow and y outside it can be added to
 *   mu = min{ g(x, y), m(R_grow), F(x, y; D-bar) - sum of m(R_i) over i != grow }
 * of those trees, where D-bar adds a vertex s_i per other root-set with an arc (x, s_i) of capacity m(R_i)
 * and unbounded arcs (s_i, r), r in R_i (the theorem of Appendix E.3 that computes mu by one max-flow).
 *
 * fc_tree_mu_batch evaluates mu for many candidate edges of one state in one launch.  All arrays are host
 * arrays; the call is synchronous.  tail/head/capacity: the n_links links of D* over vertices
 * 0..n_vertices-1 with their remaining capacities (parallel entries add up).  set_ptr [n_sets+1],
 * set_members: the root-sets as lists; set_demand [n_sets] >= 1; grow_set: the one being grown.
 * mu_out [n_edges]: mu, or FC_MU_INVALID for an entry that is no link from inside R_grow to outside it.
 * flows_or_null [n_edges]: F(x, y; D-bar); without it a max-flow may stop as soon as it cannot decide mu.
 * The digraph, plus one vertex and its member arcs per root-set that has more than one member but does not
 * span yet (other than grow_set), must fit the 32-bit on-chip state (FC_EUNSUPPORTED otherwise), and the sum
 * of all capacities and demands must stay below 2^30 (FC_EOVERFLOW).  Other errors: FC_EINVAL, FC_EDEVICE, FC_ENOMEM, FC_ENOCONVERGE.
 *
 * fc_construct_trees runs the whole construction around such launches: every vertex u starts as the
 * root-set {u} with demand k; the first root-set (in creation order) that does not span yet is grown by the
 * first link leaving it, in (x, y) order, whose mu is positive; when mu is below its demand a copy keeps
 * the rest.  All candidate links of a state are evaluated in one launch (the ones before the first positive
 * mu are zero on this very state, so the result is that of trying them one by one), and the launch looks
 * ahead: it also evaluates the states that follow (options->tree_chain_states of them in all) if, each time,
 * the first link that was neither rejected before nor zero the last time any root-set tried it is accepted in
 * full; those results are used as far as the guesses turn out right.  A link whose mu was 0 is
 * not tried again while the same root-set grows (its mu cannot rise).  Unless options->tree_warm_start is 2
 * the launches do not start from nothing: the flow that brings the other root-sets' demands to a vertex y
 * is kept in device memory (n_vertices rows of one value per link, and as many again per state a launch looks
 * ahead: fewer states are looked ahead when that would exceed 2 GiB), a max-flow into y repairs it for the capacities used
 * up since and then only routes the units that decide mu.  The trees are the same either way.  Output: n_trees
 * root-sets; tree i has root tree_root[i], multiplicity tree_multiplicity[i] (they add up to k per root)
 * and the n_vertices - 1 edges tree_edge_x/y[i * (n_vertices - 1) ..] in the order they were added.
 * Needs min over v of F(s, v) >= N k to hold in D* (what switch removal preserves); FC_ENOCONVERGE if no
 * edge can be added.  FC_EWORKSPACE with *n_trees set when tree_capacity is too small. */
#define FC_MU_INVALID FC_GAMMA_INVALID
int fc_tree_mu_batch(int32_t n_vertices, int64_t n_links, const int32_t *tail, const int32_t *head,
                     const int32_t *capacity, int32_t n_sets, const int64_t *set_ptr, const int32_t *set_members,
                     const int32_t *set_demand, int32_t grow_set, int64_t n_edges, const int32_t *edge_x,
                     const int32_t *edge_y, int32_t *mu_out, int32_t *flows_or_null, void *hip_stream,
                     const fc_options *options_or_null);
int fc_construct_trees(int32_t n_vertices, int64_t n_links, const int32_t *tail, const int32_t *head,
                       const int32_t *capacity, int32_t k, int64_t tree_capacity, int64_t *n_trees,
                       int32_t *tree_root, int32_t *tree_multiplicity, int32_t *tree_edge_x, int32_t *tree_edge_y,
                       int64_t *n_batches_or_null, void *hip_stream, const fc_options *options_or_null);

#ifdef __cplusplus
}
#endif
#endif /* FC_MAXFLOW_H */
