// Host-side logic of the library: graph ingest (validation, merging of parallel arcs,
// residual CSR, the graph facts Algorithm 1 needs) and the exact search driver.
// Pure C++; no HIP calls in this file.
#include <algorithm>
#include <cstdlib>
#include <cstring>
#include <new>
#include <numeric>

#include "fc_internal.h"

namespace {

int64_t gcd64(int64_t a, int64_t b) {
    while (b) { int64_t t = a % b; a = b; b = t; }
    return a < 0 ? -a : a;
}

struct Arc { int32_t t, h; int64_t b; };

}  // namespace

// ---------------------------------------------------------------------------------------------
// Graph ingest.  The topology is the digraph G of the paper's problem definition (Section 5);
// parallel arcs add (Appendix E.1: integer capacity = number of multi-edges).
int fc_host_build(int32_t n_vertices, int64_t n_arcs, const int32_t *tail, const int32_t *head,
                  const int32_t *bandwidth, const uint8_t *is_compute, fc_graph **out, bool keep_zero_links) {
    if (!out || n_vertices < 2 || n_arcs < 0 || !is_compute) return FC_EINVAL;
    if (n_arcs > 0 && (!tail || !head || !bandwidth)) return FC_EINVAL;
    if (n_vertices > (1 << 24) || n_arcs > (int64_t(1) << 28)) return FC_EUNSUPPORTED;
    try {
        std::vector<Arc> arcs;
        arcs.reserve(size_t(n_arcs));
        for (int64_t i = 0; i < n_arcs; ++i) {
            if (tail[i] < 0 || tail[i] >= n_vertices || head[i] < 0 || head[i] >= n_vertices) return FC_EINVAL;
            if (bandwidth[i] < 0) return FC_EINVAL;
            if (tail[i] == head[i] || (bandwidth[i] == 0 && !keep_zero_links)) continue;   // carry nothing
            arcs.push_back({tail[i], head[i], bandwidth[i]});
        }
        std::sort(arcs.begin(), arcs.end(), [](const Arc &x, const Arc &y) {
            return x.t != y.t ? x.t < y.t : x.h < y.h;
        });
        size_t w = 0;
        for (size_t i = 0; i < arcs.size(); ++i) {
            if (w > 0 && arcs[w - 1].t == arcs[i].t && arcs[w - 1].h == arcs[i].h) arcs[w - 1].b += arcs[i].b;
            else arcs[w++] = arcs[i];
        }
        arcs.resize(w);

        fc_graph *g = new fc_graph();
        g->n = n_vertices;
        g->m0 = int64_t(arcs.size());
        g->is_compute.resize(size_t(n_vertices));
        for (int32_t v = 0; v < n_vertices; ++v) {
            g->is_compute[v] = is_compute[v] ? 1 : 0;
            if (is_compute[v]) g->compute_ids.push_back(v);
        }
        g->N = int32_t(g->compute_ids.size());
        g->sum_w = g->N;
        if (g->N < 2) { delete g; return FC_EINVAL; }

        std::vector<int64_t> in_bw(size_t(n_vertices), 0), out_bw(size_t(n_vertices), 0);
        std::vector<int32_t> deg(size_t(n_vertices) + 1, 0);
        int64_t gc = 0, mx = 0;
        for (const Arc &a : arcs) {
            if (a.b >= (int64_t(1) << 31)) { delete g; return FC_EOVERFLOW; }
            in_bw[a.h] += a.b; out_bw[a.t] += a.b;
            deg[a.t]++; deg[a.h]++;
            gc = gcd64(gc, a.b); mx = std::max(mx, a.b);
        }
        int64_t min_in = -1; int32_t eul = 1;
        for (int32_t v = 0; v < n_vertices; ++v) {
            if (in_bw[v] >= (int64_t(1) << 31)) { delete g; return FC_EOVERFLOW; }
            if (in_bw[v] != out_bw[v]) eul = 0;
            if (g->is_compute[v] && (min_in < 0 || in_bw[v] < min_in)) min_in = in_bw[v];
        }
        g->min_in_bw = min_in; g->max_bw = int32_t(mx); g->gcd_bw = int32_t(gc); g->eulerian = eul;
        for (const Arc &a : arcs) g->sum_bw += a.b;
        g->in_bw.resize(size_t(n_vertices));
        for (int32_t v = 0; v < n_vertices; ++v) g->in_bw[v] = int32_t(in_bw[v]);

        // residual CSR: row u lists first the arcs leaving u, then the reverses of arcs entering u
        g->row_ptr.assign(size_t(n_vertices) + 1, 0);
        for (int32_t v = 0; v < n_vertices; ++v) {
            g->row_ptr[v + 1] = g->row_ptr[v] + deg[v];
            g->max_row = std::max(g->max_row, deg[v]);
            g->row_seen += double(deg[v]) * double(deg[v]);
        }
        g->row_seen = g->row_ptr[size_t(n_vertices)] > 0 ? g->row_seen / double(g->row_ptr[size_t(n_vertices)]) : 0.0;
        size_t M = size_t(2 * g->m0);
        g->other.resize(M); g->pair.resize(M); g->bw.resize(M); g->fwd.resize(M);
        std::vector<int32_t> fill(g->row_ptr.begin(), g->row_ptr.end() - 1);
        for (size_t i = 0; i < arcs.size(); ++i) {            // forward records (arcs sorted by tail)
            int32_t r = fill[arcs[i].t]++;
            g->other[r] = arcs[i].h; g->pair[r] = int32_t(i); g->bw[r] = int32_t(arcs[i].b); g->fwd[r] = 1;
        }
        for (size_t i = 0; i < arcs.size(); ++i) {            // reverse records
            int32_t r = fill[arcs[i].h]++;
            g->other[r] = arcs[i].t; g->pair[r] = int32_t(i); g->bw[r] = int32_t(arcs[i].b); g->fwd[r] = 0;
        }
        *out = g;
        return FC_OK;
    } catch (const std::bad_alloc &) {
        return FC_ENOMEM;
    }
}

// ---------------------------------------------------------------------------------------------
// In-place bandwidth updates (the edge-splitting loop of Appendix E.2 lowers c(u, w) and c(w, t) and raises c(u, t)
// with every split).  The CSR keeps its shape: a link lowered to zero stays as a pair of records that carry nothing.
int fc_host_update_arcs(fc_graph *g, int64_t n_updates, const int32_t *tail, const int32_t *head,
                        const int32_t *bandwidth, std::vector<int32_t> &edits) {
    if (!g || n_updates < 0 || (n_updates > 0 && (!tail || !head || !bandwidth))) return FC_EINVAL;
    try {
        edits.clear();
        const int32_t n = g->n;
        // where every update lands: the forward record in the tail's row, the reverse record in the head's row
        std::vector<int32_t> rf(size_t(n_updates), -1), rr(size_t(n_updates), -1);
        for (int64_t i = 0; i < n_updates; ++i) {
            if (tail[i] < 0 || tail[i] >= n || head[i] < 0 || head[i] >= n || bandwidth[i] < 0) return FC_EINVAL;
            for (int32_t r = g->row_ptr[size_t(tail[i])]; r < g->row_ptr[size_t(tail[i]) + 1]; ++r)
                if (g->fwd[size_t(r)] && g->other[size_t(r)] == head[i]) { rf[size_t(i)] = r; break; }
            if (rf[size_t(i)] < 0) return FC_EINVAL;              // no such link: the CSR has no room for it
            const int32_t pr = g->pair[size_t(rf[size_t(i)])];
            for (int32_t r = g->row_ptr[size_t(head[i])]; r < g->row_ptr[size_t(head[i]) + 1]; ++r)
                if (!g->fwd[size_t(r)] && g->pair[size_t(r)] == pr) { rr[size_t(i)] = r; break; }
            if (rr[size_t(i)] < 0) return FC_EINVAL;              // (cannot happen: every link has both records)
        }
        // the graph facts after the updates, checked before anything is changed (a later update of a link wins)
        std::vector<int32_t> bw_new(g->bw);
        for (int64_t i = 0; i < n_updates; ++i) { bw_new[size_t(rf[size_t(i)])] = bandwidth[i]; bw_new[size_t(rr[size_t(i)])] = bandwidth[i]; }
        std::vector<int64_t> in_bw(size_t(n), 0), out_bw(size_t(n), 0);
        int64_t gc = 0, mx = 0, sum = 0;
        for (int32_t v = 0; v < n; ++v)
            for (int32_t r = g->row_ptr[size_t(v)]; r < g->row_ptr[size_t(v) + 1]; ++r) {
                if (!g->fwd[size_t(r)]) continue;
                const int64_t b = bw_new[size_t(r)];
                out_bw[size_t(v)] += b; in_bw[size_t(g->other[size_t(r)])] += b; sum += b;
                gc = gcd64(gc, b); mx = std::max(mx, b);
            }
        int64_t min_in = -1; int32_t eul = 1;
        for (int32_t v = 0; v < n; ++v) {
            if (in_bw[size_t(v)] >= (int64_t(1) << 31)) return FC_EOVERFLOW;
            if (in_bw[size_t(v)] != out_bw[size_t(v)]) eul = 0;
            if (g->is_compute[size_t(v)] && (min_in < 0 || in_bw[size_t(v)] < min_in)) min_in = in_bw[size_t(v)];
        }
        for (size_t r = 0; r < bw_new.size(); ++r)
            if (bw_new[r] != g->bw[r]) { edits.push_back(int32_t(r)); edits.push_back(bw_new[r]); }
        g->bw.swap(bw_new);
        for (int32_t v = 0; v < n; ++v) g->in_bw[size_t(v)] = int32_t(in_bw[size_t(v)]);
        g->sum_bw = sum; g->min_in_bw = min_in; g->max_bw = int32_t(mx); g->gcd_bw = int32_t(gc); g->eulerian = eul;
        return FC_OK;
    } catch (const std::bad_alloc &) {
        return FC_ENOMEM;
    }
}

extern "C" int fc_graph_build(int32_t n_vertices, int64_t n_arcs, const int32_t *tail, const int32_t *head,
                              const int32_t *bandwidth, const uint8_t *is_compute, fc_graph **out) {
    return fc_host_build(n_vertices, n_arcs, tail, head, bandwidth, is_compute, out);
}

extern "C" int fc_graph_info(const fc_graph *g, int32_t *n_compute, int64_t *n_arcs_merged,
                             int64_t *min_in_bw_compute, int32_t *max_bw, int32_t *gcd_bw, int32_t *is_eulerian) {
    if (!g) return FC_EINVAL;
    if (n_compute) *n_compute = g->N;
    if (n_arcs_merged) *n_arcs_merged = g->m0;
    if (min_in_bw_compute) *min_in_bw_compute = g->min_in_bw;
    if (max_bw) *max_bw = g->max_bw;
    if (gcd_bw) *gcd_bw = g->gcd_bw;
    if (is_eulerian) *is_eulerian = g->eulerian;
    return FC_OK;
}

extern "C" int fc_graph_csr(const fc_graph *g, int32_t *row_ptr, int32_t *other, int32_t *pair,
                            int32_t *bw, uint8_t *forward) {
    if (!g) return FC_EINVAL;
    size_t M = size_t(2 * g->m0);
    if (row_ptr) std::memcpy(row_ptr, g->row_ptr.data(), sizeof(int32_t) * (size_t(g->n) + 1));
    if (other && M) std::memcpy(other, g->other.data(), sizeof(int32_t) * M);
    if (pair && M) std::memcpy(pair, g->pair.data(), sizeof(int32_t) * M);
    if (bw && M) std::memcpy(bw, g->bw.data(), sizeof(int32_t) * M);
    if (forward && M) std::memcpy(forward, g->fwd.data(), M);
    return FC_OK;
}

// ---------------------------------------------------------------------------------------------
// Exact search for 1/x* (the output of Algorithm 1) and (U, k) (Proposition 3).
//
// Theorem 1 makes the verdict monotone in the candidate 1/x, and Appendix E.1 shows that 1/x*
// is a fraction whose denominator is at most B = min over compute nodes of B^-(v), inside
// [(N-1)/B, N-1].  The driver keeps Stern-Brocot neighbours lo = a/b (known infeasible, i.e.
// below 1/x*) and hi = c/d (known feasible): every fraction strictly between them has
// denominator >= b + d, so once b + d > B the answer is hi.  Each round tests a batch of
// fractions on the two "runs" that leave the current pair -- (a + i c)/(b + i d) towards hi
// and (i a + c)/(i b + d) towards lo -- and narrows the run index by a multi-way split.
namespace {

struct Frac { int64_t p, q; };

// up to `c` distinct probe indices strictly inside (lo, hi); geometric from lo when the gap is wide
void pick_probes(int64_t lo, int64_t hi, int32_t c, std::vector<int64_t> &out) {
    int64_t cnt = hi - lo - 1;
    if (cnt <= 0 || c <= 0) return;
    if (cnt <= c) { for (int64_t i = lo + 1; i < hi; ++i) out.push_back(i); return; }
    if (cnt <= int64_t(c) * c) {                       // even split: done in two rounds
        for (int32_t j = 0; j < c; ++j) out.push_back(lo + ((int64_t(j) + 1) * (cnt + 1)) / (c + 1));
        return;
    }
    int64_t ratio = 2;                                  // smallest integer with ratio^c >= cnt
    for (;; ++ratio) {
        int64_t pw = 1; bool enough = false;
        for (int32_t j = 0; j < c; ++j) { pw *= ratio; if (pw >= cnt) { enough = true; break; } }
        if (enough) break;
    }
    int64_t off = 1;
    for (int32_t j = 0; j < c && off <= cnt; ++j) { out.push_back(lo + off); off *= ratio; }
}

}  // namespace

namespace {

// The smallest fraction p/q with q <= den_bound for which the (monotone) verdict is "feasible",
// known to lie in (floor_below, top]: `top` itself is feasible (the caller has tested it) and the
// integer `floor_below` is infeasible without a test.  Stern-Brocot walk: keep neighbours lo
// (infeasible) < answer <= hi (feasible); every fraction strictly between them has denominator
// >= q_lo + q_hi, so once that exceeds den_bound the answer is hi.  Each round tests up to C
// fractions on the two runs (lo + i hi) and (i lo + hi), splitting the run index multi-way.
int smallest_feasible_fraction(int64_t top, int64_t floor_below, int64_t den_bound, int32_t C, fc_verdict_fn verdicts,
                               void *ctx, Frac *answer, int32_t *rounds_io) {
    const int64_t B = den_bound;
    int32_t rounds = *rounds_io;
    std::vector<int32_t> cu, ck; std::vector<uint8_t> cv;
    Frac lo{floor_below, 1}, hi{1, 0};               // hi = +infinity
    int dir = 0;                                     // 0: no run open; +1: towards hi; -1: towards lo
    int64_t run_lo = 0, run_hi = 0;                  // open run: index run_lo continues, run_hi stops
    int64_t imax_r = 0, imax_l = 0;
    for (;;) {
        if (dir == 0) {
            if (hi.q != 0 && lo.q + hi.q > B) break;                 // no fraction left between them
            imax_r = hi.q == 0 ? top - lo.p - 1 : (B - lo.q) / hi.q;   // (lo.p + i)/1 with i > imax_r is >= top
            imax_l = (B - hi.q) / lo.q;
            if (hi.q == 0 && imax_r < 1) { hi = Frac{top, 1}; continue; }  // lo.p + 1 == top, already tested
        }
        std::vector<int64_t> pr, pl;                 // probe indices on the two runs
        if (dir == 0) {
            pr.push_back(1);                          // the mediant, shared by both runs
            int32_t cl = (C - 1) / 2, cr = C - 1 - cl;
            pick_probes(1, imax_r + 1, cr, pr);
            pick_probes(1, imax_l + 1, cl, pl);
        } else if (dir > 0) pick_probes(run_lo, run_hi, C, pr);
        else pick_probes(run_lo, run_hi, C, pl);

        cu.clear(); ck.clear();
        for (int64_t i : pr) { cu.push_back(int32_t(lo.p + i * hi.p)); ck.push_back(int32_t(lo.q + i * hi.q)); }
        for (int64_t i : pl) { cu.push_back(int32_t(i * lo.p + hi.p)); ck.push_back(int32_t(i * lo.q + hi.q)); }
        cv.assign(cu.size(), 0);
        int rc = verdicts(ctx, int32_t(cu.size()), cu.data(), ck.data(), cv.data());
        ++rounds;
        if (rc != FC_OK) return rc;
        const uint8_t *vr = cv.data(), *vl = cv.data() + pr.size();

        if (dir == 0) {
            dir = vr[0] ? -1 : +1;
            if (dir > 0) { run_lo = 0; run_hi = imax_r + 1; }
            else { run_lo = 1; run_hi = imax_l + 1; }   // index 1 (the mediant) is feasible
        }
        if (dir > 0) {               // towards hi: infeasible ... infeasible feasible ... feasible
            for (size_t j = 0; j < pr.size(); ++j) {
                if (!vr[j]) run_lo = std::max(run_lo, pr[j]);
                else run_hi = std::min(run_hi, pr[j]);
            }
        } else {                     // towards lo: feasible ... feasible infeasible ... infeasible
            for (size_t j = 0; j < pl.size(); ++j) {
                if (vl[j]) run_lo = std::max(run_lo, pl[j]);
                else run_hi = std::min(run_hi, pl[j]);
            }
        }
        if (run_lo >= run_hi) return FC_ENOCONVERGE;    // verdicts were not monotone
        if (run_hi == run_lo + 1) {                     // run resolved: move the pair
            if (dir > 0) {
                Frac nlo{lo.p + run_lo * hi.p, lo.q + run_lo * hi.q};
                if (run_hi <= imax_r) hi = Frac{lo.p + run_hi * hi.p, lo.q + run_hi * hi.q};
                else if (hi.q == 0) hi = Frac{top, 1};
                lo = nlo;
            } else {
                Frac nhi{run_lo * lo.p + hi.p, run_lo * lo.q + hi.q};
                if (run_hi <= imax_l) lo = Frac{run_hi * lo.p + hi.p, run_hi * lo.q + hi.q};
                hi = nhi;
            }
            dir = 0;
        }
    }
    *answer = hi;
    *rounds_io = rounds;
    return FC_OK;
}

}  // namespace

extern "C" int fc_search_with_verdicts(int32_t n_compute, int64_t min_in_bw, int32_t gcd_bw,
                                       int32_t candidates_per_round, fc_verdict_fn verdicts, void *ctx,
                                       fc_rational *inv_xstar, fc_rational *U, int64_t *k,
                                       int32_t *rounds_or_null) {
    if (!verdicts || !inv_xstar || !U || !k || n_compute < 2 || candidates_per_round < 1 || gcd_bw < 0)
        return FC_EINVAL;
    const int64_t N = n_compute, B = min_in_bw;
    if (B < 1) return FC_EDISCONNECTED;                 // a compute node nothing can reach
    if ((N - 1) * B >= (int64_t(1) << 31) || N * B >= (int64_t(1) << 31)) return FC_EOVERFLOW;
    const int32_t C = std::max<int32_t>(candidates_per_round, 2);
    int32_t rounds = 0;
    try {
        // upper end of the paper's initial range: 1/x = N-1 must be feasible (B^+(S) >= 1 for all S)
        int32_t cu = int32_t(N - 1), ck = 1; uint8_t cv = 0;
        int rc = verdicts(ctx, 1, &cu, &ck, &cv);
        ++rounds;
        if (rc != FC_OK) return rc;
        if (!cv) return FC_EDISCONNECTED;
        // lower end: (N-1)/B <= 1/x*, so the integer just below it is infeasible without a test;
        // the denominator of 1/x* is at most B (Appendix E.1)
        Frac hi{0, 1};
        rc = smallest_feasible_fraction(N - 1, (N - 1 + B - 1) / B - 1, B, C, verdicts, ctx, &hi, &rounds);
        if (rc != FC_OK) return rc;
        int64_t g = gcd64(hi.q, gcd_bw);                 // Proposition 3
        if (g < 1) g = 1;
        inv_xstar->num = hi.p; inv_xstar->den = hi.q;
        U->num = hi.p; U->den = g;
        *k = hi.q / g;
        if (rounds_or_null) *rounds_or_null = rounds;
        return FC_OK;
    } catch (const std::bad_alloc &) {
        return FC_ENOMEM;
    }
}

extern "C" int fc_fixed_k_search_with_verdicts(int32_t n_compute, int64_t min_in_bw, int32_t max_bw, int32_t k,
                                               int32_t candidates_per_round, fc_verdict_fn verdicts, void *ctx,
                                               fc_rational *U_star, int32_t *rounds_or_null) {
    if (!verdicts || !U_star || n_compute < 2 || candidates_per_round < 1 || k < 1 || max_bw < 0) return FC_EINVAL;
    const int64_t N = n_compute, B = min_in_bw, top = (N - 1) * int64_t(k);
    if (B < 1 || max_bw < 1) return FC_EDISCONNECTED;
    // every candidate p/q has q <= max_bw and p/q <= top: p must fit 32 bits, and so must N * k
    if (top * int64_t(max_bw) >= (int64_t(1) << 31) || N * int64_t(k) >= (int64_t(1) << 31)) return FC_EOVERFLOW;
    const int32_t C = std::max<int32_t>(candidates_per_round, 2);
    int32_t rounds = 0;
    try {
        // upper end of the range of Algorithm 3: U = (N-1) k must be feasible
        int32_t cu = int32_t(top), cd = 1; uint8_t cv = 0;
        int rc = verdicts(ctx, 1, &cu, &cd, &cv);
        ++rounds;
        if (rc != FC_OK) return rc;
        if (!cv) return FC_EDISCONNECTED;
        // lower end: U* >= (N-1) k / B; at U* some U* b_e is an integer, so its denominator is at most max_bw
        Frac hi{0, 1};
        rc = smallest_feasible_fraction(top, (top + B - 1) / B - 1, max_bw, C, verdicts, ctx, &hi, &rounds);
        if (rc != FC_OK) return rc;
        U_star->num = hi.p; U_star->den = hi.q;
        if (rounds_or_null) *rounds_or_null = rounds;
        return FC_OK;
    } catch (const std::bad_alloc &) {
        return FC_ENOMEM;
    }
}

extern "C" const char *fc_strerror(int code) {
    switch (code) {
        case FC_OK: return "ok";
        case FC_EINVAL: return "invalid argument";
        case FC_EOVERFLOW: return "integer overflow";
        case FC_EDISCONNECTED: return "some compute node cannot reach another one";
        case FC_ENOMEM: return "out of host memory";
        case FC_EWORKSPACE: return "workspace missing or too small";
        case FC_EDEVICE: return "HIP device error";
        case FC_ENOCONVERGE: return "iteration cap hit";
        case FC_EUNSUPPORTED: return "graph too large for this build";
        default: return "unknown error";
    }
}
