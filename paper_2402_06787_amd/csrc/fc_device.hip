// Device side of the library: HIP kernels for gfx950 (MI355X) and the C-ABI entry points that
// launch them.
//
// One workgroup solves one max-flow problem (sink v_j, edge multiplier U_j, source-arc capacity
// k_j) of the auxiliary network of the paper's Section 5.2 with a level-synchronous
// push-relabel (push-relabel is the algorithm family the paper names in Appendix C; the
// schedule below is this library's own).  All per-problem state -- the flow on every topology
// arc, the height and excess of every vertex -- lives in LDS; only the shared, read-only
// topology (residual CSR records) is read from global memory, where it stays cache resident.
//
// The super-source is never materialised: its arcs (s, c) are saturated by the initial preflow
// (excess k_j at every compute node, the sink included) and, because s keeps the largest height,
// nothing is ever pushed back to it.  F(s, v_j) is the excess collected at the sink when no
// vertex that can still reach the sink holds excess (min-cut theorem, Appendix E preamble).
//
// The same kernel is instantiated three ways: integer multipliers U (Section 5.2, Appendix E.1),
// rational multipliers with capacities floor(U b_e) (fixed k, Section 5.5 / Algorithm 3), and the
// max-flows with an explicit source and unbounded arcs that edge splitting needs (Appendix E.2,
// Theorem 10).  Host code at the end: option handling, launches, and the entry points.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <mutex>
#include <new>
#include <map>
#include <set>
#include <vector>

#include "fc_internal.h"

#define FC_LVLS 128  // heights below this have a population count (gap detection)
#define FC_NSTAT 8   // per-problem counters: pushes, relabels, arc_scans, grs, gr_arc_scans, level_steps, discharges, not_converged

// Optional per-phase cycle accounting for tuning builds (-DFC_PHASE_TIMING): the per-problem
// counters relabels/global_relabels/gr_arc_scans/discharges are then replaced by the cycles
// thread 0 spent in level compaction / discharge / initialisation / everything else.
#ifdef FC_PHASE_TIMING
#define FC_TICK(var) do { long long now_ = clock64(); var += uint32_t(now_ - tick_); tick_ = now_; } while (0)
#else
#define FC_TICK(var) do { } while (0)
#endif

namespace {

constexpr int FC_ORDER_CHUNK = 16;     // consecutive entries of a launch order that share an XCD

// One of several graphs of a launch (explicit (source, sink) problems only): where its row offsets and arc
// records start relative to the launch's arrays, how many records it has, and the sum of its finite capacities.
struct GraphDesc { int32_t row_off, arc_off, n_rec, pad; long long sum_bw; };

struct KParams {
    int32_t n, N, m0;
    int32_t n_rec;               // residual arc records (at least 1: a zeroed dummy when the graph has no arcs)
    int32_t gr_lanes, gr_shift, gr_sub;   // global relabel: lanes per work-list entry (2^gr_shift), sub-chunks per entry
    const int32_t *row_ptr;
    const int4 *arc_wide;
    const uint2 *arc_compact;
    const uint8_t *is_compute;
    const uint16_t *labels;      // [n*n] exact initial heights per sink (row = sink), bit 15 = compute node; or null
    const uint16_t *label_hmax;  // [n] highest finite label of a compute node per sink
    const uint4 *p1;             // [n*n] first-pass entries per sink in level order, or null
    const uint16_t *level_off;   // [n*64] level boundaries in `order` per sink
    const int32_t *tree_ratio;   // [n*2] per sink {num, den}: first-arc tree certificate, or null (off)
    const int32_t *sink, *U, *k;
    const int32_t *Uden;         // rational multipliers U_j / Uden_j (kernels built for floor capacities), else null
    int32_t *flow_out;
    uint32_t *stats;             // [P * FC_NSTAT] or null
    int32_t gr_steps, gr_relabels, gr_rises, tight_pct, use_gap, max_steps;
    const int32_t *in_bw;        // [n] in-bandwidth of every vertex
    int32_t wide_available;      // the 32-bit-state kernel is launched too
    const int32_t *order;        // workgroup -> problem (hardest first), or null for the identity
    int32_t n_order;             // entries of `order`: an entry outside [0, n_order) is never followed
    int32_t order_chunked;       // problem-list launches: runs of FC_ORDER_CHUNK consecutive entries of `order` go to one XCD
    // candidate x sink launches (fc_feasible): workgroup b solves candidate b % cand_C for the sink that
    // has place b / cand_C in the order; the problem list is never written out
    int32_t cand_C;              // 0: plain problem list
    const int32_t *cand_U, *cand_k, *cand_D, *compute_ids;
    // edge-splitting launches (Theorem 10): workgroup (i * 2 + type) * N + a solves, for pair i = (u, w, t)
    // and the a-th compute node v, F(u, w) with unbounded arcs (u, s), (u, t), (v, w) (type 0) or F(w, t) with
    // unbounded arcs (w, s), (u, t), (v, t) (type 1); multiplier split_U and source arcs split_k for all
    const int32_t *split_u, *split_w, *split_t;
    int32_t split_U, split_k;
    int32_t split_early;         // 1: a problem may stop once N k + min{c(e), c(f)} units have arrived (only gamma is wanted);
                                 // 2: once N k + min{c(e), c(f)} + c(f) have (the caller also wants that much of the slack)
    // explicit (source, sink) launches (the max-flows of spanning tree construction, Appendix E.3): workgroup b
    // solves F(pair_src[b], pair_dst[b]) with the source's arcs saturated, the excess src_w[v] * split_k at every
    // flagged vertex, multiplier split_U, and may stop once pair_stop[b] units have arrived
    const int32_t *pair_src, *pair_dst, *pair_stop;
    const int32_t *pair_graph;   // null, or per problem the index of its graph in `graphs` (same vertex set, different arcs)
    const GraphDesc *graphs;
    long long sum_bw;            // sum of all link bandwidths (bounds every finite cut)
    const int32_t *src_w;        // [n] weight m_c of compute node c: arc (s, c) has capacity m_c * k (Section 5.7); null: all 1
    long long sum_w;             // sum of the weights (N while they are all 1): s emits at most sum_w * k
    uint32_t *sink_cost;         // [n] what the last problem of each sink cost (feeds the next launch's order)
};

struct ArcRec { int32_t w, pair, bw, fwd, last; };   // last: final record of its vertex's row

// Raw residual-arc record as stored in global memory, and its decoded form.  Loading and decoding
// are separate so that several loads can be in flight before the first one is consumed.
template <bool COMPACT> struct ArcRaw;
template <> struct ArcRaw<true> { uint2 q; };
template <> struct ArcRaw<false> { int4 q; };

template <bool COMPACT>
__device__ __forceinline__ ArcRaw<COMPACT> load_arc_raw(const KParams &p, int32_t a) {
    ArcRaw<COMPACT> r;
    if constexpr (COMPACT) r.q = p.arc_compact[a]; else r.q = p.arc_wide[a];
    return r;
}

template <bool COMPACT>
__device__ __forceinline__ ArcRec decode_arc(const ArcRaw<COMPACT> &raw) {
    ArcRec r;
    if constexpr (COMPACT) {
        r.w = int32_t(raw.q.x & 0x7fffu); r.fwd = int32_t((raw.q.x >> 15) & 1u); r.pair = int32_t(raw.q.x >> 16);
        r.bw = int32_t(raw.q.y & 0x7fffffffu); r.last = int32_t(raw.q.y >> 31);
    } else {
        r.w = raw.q.x; r.pair = raw.q.y; r.bw = raw.q.z; r.fwd = raw.q.w & 1; r.last = (raw.q.w >> 1) & 1;
    }
    return r;
}

template <bool COMPACT>
__device__ __forceinline__ ArcRec load_arc(const KParams &p, int32_t a) {
    return decode_arc<COMPACT>(load_arc_raw<COMPACT>(p, a));
}

// Capacity of a topology arc in one problem, clamped at N * k (no flow needs more than s can emit).
// Integer multiplier (Section 5.2, Appendix E.1): U * b_e; b_e > floor(N*k / U) is exactly the case
// U * b_e > N*k, so 32-bit arithmetic suffices.  Rational multiplier U / D (fixed k, Section 5.5 /
// Algorithm 3): floor(U * b_e / D); the quotient comes from a double-precision estimate corrected by
// the exact remainder (the product is below N*k*D < 2^62 and the quotient below 2^31, so the
// estimate is off by at most one).
template <bool RAT>
struct ArcCap {
    int32_t U, NK, sat, D; double invD;
    __device__ __forceinline__ ArcCap(int32_t U_, int32_t D_, int32_t NK_) : U(U_), NK(NK_), sat(0), D(D_), invD(1.0) {
        if (!RAT) sat = NK_ / U_;
        else {                               // floor(U b / D) >= N k  <=>  b >= ceil(N k D / U)
            const long long lim = ((long long)NK_ * D_ + U_ - 1) / U_;
            sat = lim - 1 > 0x7fffffffll ? 0x7fffffff : int32_t(lim - 1);
            invD = 1.0 / double(D_);
        }
    }
    __device__ __forceinline__ int32_t operator()(int32_t bw) const {
        if (!RAT) return bw > sat ? NK : U * bw;
        if (bw > sat) return NK;
        const long long prod = (long long)U * (long long)bw;
        long long q = (long long)(double(prod) * invD);
        const long long r = prod - q * D;
        if (r < 0) --q; else if (r >= D) ++q;
        return int32_t(q);
    }
};

// Workgroup barrier for code whose lanes communicate through LDS only: it waits for this wave's LDS
// operations and leaves global loads in flight, so table reads issued before it overlap the wait.
__device__ __forceinline__ void lds_barrier() {
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup", "local");
    __builtin_amdgcn_s_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup", "local");
}

// Cross-lane helpers.  Within a row of 16 lanes data moves through the VALU's data-parallel
// primitives (a few cycles) instead of the LDS crossbar that a general shuffle uses (an LDS round
// trip each); only groups wider than a row fall back to shuffles.
template <int CTRL>
__device__ __forceinline__ int32_t dpp_mov(int32_t fill, int32_t v) {
    // lanes whose source lane does not exist or is inactive get `fill`
    return __builtin_amdgcn_update_dpp(fill, v, CTRL, 0xf, 0xf, false);
}
constexpr int DPP_XOR1 = 0xB1, DPP_XOR2 = 0x4E;            // quad_perm [1,0,3,2] and [2,3,0,1]
constexpr int DPP_HALF_MIRROR = 0x141, DPP_MIRROR = 0x140; // lane i <-> 7-i within 8, i <-> 15-i within 16
constexpr int DPP_ROW_SHR = 0x110;                         // + s: lane i reads lane i-s of its row

// op-reduction over every aligned group of G lanes; every lane gets its group's result
template <int G, class Op>
__device__ __forceinline__ int32_t group_allreduce(int32_t v, Op op) {
    if (G >= 2) v = op(v, dpp_mov<DPP_XOR1>(v, v));
    if (G >= 4) v = op(v, dpp_mov<DPP_XOR2>(v, v));
    if (G >= 8) v = op(v, dpp_mov<DPP_HALF_MIRROR>(v, v));
    if (G >= 16) v = op(v, dpp_mov<DPP_MIRROR>(v, v));
    if (G >= 32) v = op(v, __shfl_xor(v, 16));
    if (G >= 64) v = op(v, __shfl_xor(v, 32));
    return v;
}

// inclusive prefix sum over every aligned group of G lanes (lg = lane index within the group)
template <int G>
__device__ __forceinline__ int32_t group_prefix_sum(int32_t x, int32_t lg) {
    int32_t incl = x;
    if (G <= 16) {
        if (G > 1) { const int32_t y = dpp_mov<DPP_ROW_SHR + 1>(0, incl); if (lg >= 1) incl += y; }
        if (G > 2) { const int32_t y = dpp_mov<DPP_ROW_SHR + 2>(0, incl); if (lg >= 2) incl += y; }
        if (G > 4) { const int32_t y = dpp_mov<DPP_ROW_SHR + 4>(0, incl); if (lg >= 4) incl += y; }
        if (G > 8) { const int32_t y = dpp_mov<DPP_ROW_SHR + 8>(0, incl); if (lg >= 8) incl += y; }
    } else {
#pragma unroll
        for (int s = 1; s < G; s <<= 1) {
            const int32_t y = __shfl_up(incl, s, G);
            if (lg >= s) incl += y;
        }
    }
    return incl;
}

// inclusive prefix sum over the wavefront (all 64 lanes must be active)
__device__ __forceinline__ int32_t wave_prefix_sum(int32_t x) {
    x += dpp_mov<DPP_ROW_SHR + 1>(0, x);
    x += dpp_mov<DPP_ROW_SHR + 2>(0, x);
    x += dpp_mov<DPP_ROW_SHR + 4>(0, x);
    x += dpp_mov<DPP_ROW_SHR + 8>(0, x);                            // inclusive within each row of 16
    x += __builtin_amdgcn_update_dpp(0, x, 0x142, 0xa, 0xf, false); // rows 1 and 3 add lane 15 of the row before
    x += __builtin_amdgcn_update_dpp(0, x, 0x143, 0xc, 0xf, false); // rows 2 and 3 add lane 31
    return x;
}

// maximum over the wavefront as a uniform value (all 64 lanes must be active)
__device__ __forceinline__ int32_t wave_max(int32_t v) {
    v = group_allreduce<16>(v, [](int32_t a, int32_t b) { return a > b ? a : b; });
    const int32_t a = __builtin_amdgcn_readlane(v, 0), b = __builtin_amdgcn_readlane(v, 16);
    const int32_t c = __builtin_amdgcn_readlane(v, 32), d = __builtin_amdgcn_readlane(v, 48);
    const int32_t ab = a > b ? a : b, cd = c > d ? c : d;
    return ab > cd ? ab : cd;
}

// LDS scalars shared by a workgroup.  Per-step scalars come in two sets indexed by step parity:
// thread 0 clears the other set after the first barrier of a step, when nobody can still read it.
struct Shared {
    int32_t cnt[2];        // length of the list being discharged
    int32_t down[2];       // some push of this step went to a non-sink vertex
    int32_t nrel[2];       // vertices relabeled in this step
    int32_t dnext[2];      // largest new height given in this step
    int32_t dcarry[2];     // largest height among the pending vertices carried over in this step
    int32_t back[2];       // per list array: pending entries occupy [back, n)
    int32_t tmp;           // scratch for rare scans
    int32_t pad;
    uint32_t st[FC_NSTAT];
    uint16_t off[64];      // level table of this sink: off[0] = deepest level L, off[1 + j] = start of level L - j
    int32_t lvl[FC_LVLS];  // number of vertices at height d, for 1 <= d < FC_LVLS
};

// Byte offsets of the per-problem LDS arrays.  COMPACT: every array 16-bit; else 32-bit.
struct Carve { uint32_t f, h, e, list0, list1, rp, sh, total; };

__host__ __device__ inline Carve carve_lds(int32_t n, int32_t m0, bool compact) {
    const uint32_t w = compact ? 2u : 4u;
    auto up = [](uint32_t x) { return (x + 15u) & ~15u; };
    Carve c; uint32_t off = 0;
    c.f = off; off += up(uint32_t(m0) * w);          // flow on every merged topology arc
    c.h = off; off += up(uint32_t(n) * w);           // height; n = cannot reach the sink
    c.e = off; off += up(uint32_t(n) * w);           // excess
    c.list0 = off; off += up(uint32_t(n) * w);       // two list arrays: the front holds the vertices being
    c.list1 = off; off += up(uint32_t(n) * w);       //   discharged, the back collects pending ones
    c.rp = off; off += up(uint32_t(n + 1) * w);      // residual CSR row offsets (copy of the shared ones)
    c.sh = off; off += up(uint32_t(sizeof(Shared)));
    c.total = off;
    return c;
}

// Per-problem state in LDS.  In the 16-bit layout two excess values share a dword and are
// updated with 32-bit atomics on that dword: a half never exceeds N*k <= 65535, so no carry
// crosses into its neighbour.
template <bool COMPACT>
struct State {
    using W = typename std::conditional<COMPACT, uint16_t, int32_t>::type;
    // a stuck vertex keeps its new height in h[] behind this flag until the step is over; during the
    // step every flagged vertex still counts as being at the step's level
    static constexpr int32_t NEWH = COMPACT ? 0x8000 : 0x40000000;
    W *f, *h, *e, *list0, *list1, *rp;
    Shared *sh;
    __device__ __forceinline__ int32_t excess(int32_t v) const { return int32_t(e[v]); }
    // returns the excess v had before
    __device__ __forceinline__ int32_t excess_add(int32_t v, int32_t d) const {
        if (COMPACT) {
            const uint32_t old = atomicAdd(reinterpret_cast<uint32_t *>(e) + (v >> 1), uint32_t(d) << ((v & 1) * 16));
            return int32_t((old >> ((v & 1) * 16)) & 0xffffu);
        }
        return atomicAdd(reinterpret_cast<int32_t *>(e) + v, d);
    }
    __device__ __forceinline__ void excess_add_noret(int32_t v, int32_t d) const {
        if (COMPACT) atomicAdd(reinterpret_cast<uint32_t *>(e) + (v >> 1), uint32_t(d) << ((v & 1) * 16));
        else atomicAdd(reinterpret_cast<int32_t *>(e) + v, d);
    }
    __device__ __forceinline__ void excess_sub(int32_t v, int32_t d) const {
        if (COMPACT) atomicSub(reinterpret_cast<uint32_t *>(e) + (v >> 1), uint32_t(d) << ((v & 1) * 16));
        else atomicSub(reinterpret_cast<int32_t *>(e) + v, d);
    }
    __device__ __forceinline__ int32_t height_during_step(int32_t v, int32_t d) const {
        const int32_t raw = int32_t(h[v]);
        return (raw & NEWH) ? d : raw;
    }
    // the two list arrays (selected by value: no indexed pointer table, which would live in scratch memory)
    __device__ __forceinline__ W *list(int32_t a) const { return a ? list1 : list0; }
    // put v on the pending part of list array `a`
    __device__ __forceinline__ void pend(int32_t a, int32_t v) const { list(a)[atomicSub(&sh->back[a], 1) - 1] = W(v); }
};

// Collect every vertex that holds excess, is not the sink and can still reach it on the pending
// part of list array `a` (emptied first).  Used at the start when there is no per-sink order and
// after a global relabel.  Returns after a barrier with the largest height among them (0 if none).
template <bool COMPACT>
__device__ __forceinline__ int32_t rebuild_pending(const State<COMPACT> &st, int32_t n, int32_t t, int32_t a) {
    using W = typename State<COMPACT>::W;
    constexpr int Q = 8;
    const int32_t tid = threadIdx.x, T = blockDim.x, lane = tid & 63;
    const unsigned long long below = (1ull << lane) - 1ull;
    if (tid == 0) { st.sh->back[a] = n; st.sh->tmp = 0; }
    lds_barrier();
    int32_t best = 0;
    for (int32_t base = 0; base < n; base += Q * T) {
        bool act[Q]; unsigned long long ba[Q]; int32_t tot = 0;
#pragma unroll
        for (int q = 0; q < Q; ++q) {
            act[q] = false; ba[q] = 0ull;
            if (base + q * T < n) {                               // uniform over the workgroup
                const int32_t v = base + q * T + tid;
                const int32_t vc = v < n ? v : n - 1;             // clamped: reads stay unconditional
                const int32_t hv = int32_t(st.h[vc]);
                act[q] = v < n && v != t && hv >= 1 && hv < n && st.excess(vc) > 0;
                if (act[q] && hv > best) best = hv;
                ba[q] = __ballot(act[q]);
                tot += __popcll(ba[q]);
            }
        }
        if (tot) {
            int32_t pos = 0;
            if (lane == 0) pos = atomicSub(&st.sh->back[a], tot) - tot;
            pos = __builtin_amdgcn_readfirstlane(pos);
#pragma unroll
            for (int q = 0; q < Q; ++q) {
                if (act[q]) st.list(a)[pos + __popcll(ba[q] & below)] = W(base + q * T + tid);
                pos += __popcll(ba[q]);
            }
        }
    }
    if (best > 0) atomicMax(&st.sh->tmp, best);
    lds_barrier();
    const int32_t r = st.sh->tmp;
    lds_barrier();
    return r;
}

#ifdef FC_GRDETAIL   // tuning builds: cycles in the frontier scans / expansions and the level count
#define FC_GRDBG_PARAM , uint32_t *g_grdbg
#define FC_GRDBG_ARG , grdbg
#else
#define FC_GRDBG_PARAM
#define FC_GRDBG_ARG
#endif
// Exact heights by backward breadth-first search from the sink over arcs with positive residual
// capacity; vertices that cannot reach the sink get height n.  Also recounts the level populations.
// Uses both list arrays (as one array of 2n entries) and the cnt and down scalars as scratch.  Ends
// with a barrier.
//
// The search reads every residual arc record once, so it is organised by records, not vertices: a
// frontier vertex puts one entry per span of its row on the work list (span = p.gr_lanes *
// p.gr_sub records, sized on the host so that at most 2n entries exist at a time), a group of
// p.gr_lanes lanes takes K entries at a time and has the K record loads in flight before it looks
// at the first.  A record carries a flag when it is the last of its row, so no row bounds are needed.
// `src`, `src2`, `sa`, `sb` (each -1 when absent): vertices that never get a height (explicit sources)
// and two more vertices that count as the sink (distance 0).
template <bool COMPACT, bool RAT>
__device__ void global_relabel(const KParams &p, const State<COMPACT> &st, int32_t t, const ArcCap<RAT> &arc_cap,
                               uint32_t &gr_scans FC_GRDBG_PARAM, int32_t src = -1, int32_t src2 = -1, int32_t sa = -1, int32_t sb = -1) {
    using W = typename State<COMPACT>::W;
#ifdef FC_GRDETAIL
    long long gtick_ = clock64();
#define FC_GTICK(i) do { long long now_ = clock64(); g_grdbg[i] += uint32_t(now_ - gtick_); gtick_ = now_; } while (0)
#else
#define FC_GTICK(i) do { } while (0)
#endif
    constexpr int K = 4, Q = 5;
    const int32_t tid = threadIdx.x, T = blockDim.x, n = p.n, lane = tid & 63;
    const int32_t gg = p.gr_lanes, S = p.gr_sub, span = gg * S;
    const int32_t lg = tid & (gg - 1), grp = tid >> p.gr_shift, ngrp = T >> p.gr_shift;
    const unsigned long long gmask = (gg == 64 ? ~0ull : ((1ull << gg) - 1ull)) << (lane & ~(gg - 1));
    const unsigned long long before_me = gmask & ((1ull << lane) - 1ull);      // lower lanes of my group
    const int32_t last_rec = p.n_rec - 1;
    W *const work = st.list0;              // list0 and list1 are adjacent
    lds_barrier();                         // slower wavefronts may still be reading what is overwritten here
    for (int32_t v = tid; v < n; v += T) st.h[v] = W(v == t || v == sa || v == sb ? 0 : n);
    for (int32_t i = tid; i < FC_LVLS; i += T) st.sh->lvl[i] = 0;
    if (tid == 0) { st.sh->cnt[0] = 0; st.sh->down[0] = 0; }
    lds_barrier();
    for (int32_t d = 0;; ++d) {
        const int32_t par = d & 1;
        // frontier scan: every vertex at distance d appends the starts of the spans of its row
        for (int32_t base = 0; base < n; base += Q * T) {
            int32_t row[Q], c[Q], mine = 0, verts = 0;
#pragma unroll
            for (int q = 0; q < Q; ++q) {
                const int32_t v = base + q * T + tid;
                const int32_t vc = v < n ? v : n - 1;             // clamped: reads stay unconditional
                const bool isd = int32_t(st.h[vc]) == d && v < n;
                row[q] = int32_t(st.rp[vc]);
                const int32_t len = int32_t(st.rp[vc + 1]) - row[q];
                c[q] = !isd ? 0 : (S == 1 ? (len + gg - 1) >> p.gr_shift : (len + span - 1) / span);
                mine += c[q];
                verts += isd ? 1 : 0;
            }
            const int32_t incl = wave_prefix_sum(mine | (verts << 20));   // two sums at once: entries <= 2n < 2^20, vertices <= 64 Q
            const int32_t tot = __builtin_amdgcn_readlane(incl, 63);
            if (tot) {
                int32_t pos = 0;
                if (lane == 0) { pos = atomicAdd(&st.sh->cnt[par], tot & 0xfffff); atomicAdd(&st.sh->down[par], tot >> 20); }
                pos = __builtin_amdgcn_readfirstlane(pos) + (incl & 0xfffff) - mine;
#pragma unroll
                for (int q = 0; q < Q; ++q)
                    for (int32_t j = 0; j < c[q]; ++j) work[pos++] = W(row[q] + j * span);
            }
        }
        lds_barrier();
        FC_GTICK(0);
        const int32_t cnt = st.sh->cnt[par];
        if (tid == 0) {
            st.sh->cnt[par ^ 1] = 0;
            if (d >= 1 && d < FC_LVLS) st.sh->lvl[d] = st.sh->down[par];
            st.sh->down[par ^ 1] = 0;
        }
#ifdef FC_GRDETAIL
        g_grdbg[2] += 1;
#endif
        if (st.sh->down[par] == 0) break;                        // empty frontier (a vertex without arcs adds no entry)
        for (int32_t i0 = grp; i0 < cnt; i0 += ngrp * K) {
            int32_t a0[K]; bool live[K];
#pragma unroll
            for (int q = 0; q < K; ++q) {
                const int32_t i = i0 + q * ngrp;
                live[q] = i < cnt;
                a0[q] = int32_t(work[live[q] ? i : cnt - 1]) + lg;
            }
            for (int32_t sub = 0; sub < S; ++sub) {               // S = 1 unless the graph is dense
                ArcRaw<COMPACT> raw[K];
#pragma unroll
                for (int q = 0; q < K; ++q) {
                    const int32_t a = a0[q] + sub * gg;
                    raw[q] = load_arc_raw<COMPACT>(p, a < last_rec ? a : last_rec);      // unconditional, in bounds
                }
                // all flow reads, then all height reads, then the writes: three LDS round trips
                int32_t x[K];                                     // tail of a residual arc into the frontier, else the sink
#pragma unroll
                for (int q = 0; q < K; ++q) {
                    const ArcRec r = decode_arc<COMPACT>(raw[q]);
                    const unsigned long long ends = __ballot(live[q] && r.last) & gmask;
                    const bool valid = live[q] && (ends & before_me) == 0ull;            // up to the row's last record
                    live[q] = live[q] && ends == 0ull;
                    const int32_t fv = int32_t(st.f[r.pair]);
                    const int32_t res = r.fwd ? fv : arc_cap(r.bw) - fv;                 // residual of r.w -> frontier vertex
                    x[q] = valid && res > 0 && r.w != src && r.w != src2 ? r.w : t;
                    if (valid) ++gr_scans;
                }
                int32_t hx[K];
#pragma unroll
                for (int q = 0; q < K; ++q) hx[q] = int32_t(st.h[x[q]]);
#pragma unroll
                for (int q = 0; q < K; ++q)
                    if (hx[q] == n) st.h[x[q]] = W(d + 1);        // same value from every writer; h[t] = 0
            }
        }
        lds_barrier();
        FC_GTICK(1);
    }
    lds_barrier();
    if (tid == 0) { st.sh->cnt[0] = st.sh->cnt[1] = 0; st.sh->down[0] = st.sh->down[1] = 0; }
    lds_barrier();
}

// One workgroup = one max-flow problem: a level-synchronous push-relabel.  In a step every listed
// vertex of ONE height level d is discharged with all heights frozen, so pushes only go to level
// d-1, no arc is touched from both ends and no listed vertex receives excess.  A vertex left with
// excess (all its admissible arcs saturated) gets its new height when the step is over.  The only
// concurrent updates are commutative integer atomics: the run is deterministic.
//
// First pass (when the per-sink tables exist).  Heights still equal the breadth-first labels, so
// level d is a slice of the sink's precomputed order and no list is needed: one lane per vertex
// pushes along the vertex's precomputed first arc, read with coalesced loads (fast part); a
// vertex whose excess that arc cannot take goes to the list and is finished by the group part.
// Levels are walked from the highest one holding a compute node down to 1.
//
// Afterwards (and from the start without tables) the kernel keeps a pending list: vertices that
// hold excess and are not being discharged.  Each step takes the highest pending level (highest-
// label-first), moves its vertices to the front of the other list array, carries the rest over,
// and discharges them with the group part; vertices that receive excess for the first time and
// vertices that were relabeled join the pending list.  No step scans all vertices.
//
// Group part: G lanes scan the residual row of one listed vertex in chunks, give all excess to the
// first admissible arc when it suffices, else split it by a segmented prefix sum in row order, and
// collect the smallest residual-neighbour height for the relabel in the same scan.
//
// Template flags: COMPACT = 16-bit on-chip state, RAT = rational multipliers (floor capacities),
// GEN = an edge-splitting problem (explicit source, "unbounded" arcs, no tables), G = lanes per vertex,
// OCC = wavefronts per SIMD the register allocation leaves room for.  A problem's LDS footprint decides how
// many wavefronts a CU can hold: large graphs stop at 5 per SIMD and get the build with the most
// registers; small graphs fit 8 per SIMD and run faster with fewer registers (a few spilled) and
// more wavefronts in flight.
template <bool COMPACT, bool RAT, bool GEN, int G, int OCC>
__global__ void __launch_bounds__(1024) __attribute__((amdgpu_waves_per_eu(OCC))) fc_push_relabel_kernel(KParams p) {
    static_assert(!GEN || (!COMPACT && !RAT), "the edge-splitting problems use the 32-bit state and integer multipliers");
    using W = typename State<COMPACT>::W;
    constexpr int32_t NEWH = State<COMPACT>::NEWH;
    extern __shared__ __align__(16) unsigned char smem[];
    const int32_t tid = threadIdx.x, T = blockDim.x, n = p.n, m0 = p.m0;
    int32_t j, t, U, k, D = 1;
    int32_t src = -1, src2 = -1, sa = -1, sb = -1;       // edge-splitting problems only (see below)
    int32_t gu = -1, gw = -1, gt = -1;                   // their pair e = (gu, gw), f = (gw, gt)
    if (GEN && p.pair_src) {
        j = int32_t(blockIdx.x); U = p.split_U; k = p.split_k;
        src = p.pair_src[j]; t = p.pair_dst[j];
        if (p.pair_graph) {                              // this problem's graph among the launch's
            const GraphDesc gd = p.graphs[p.pair_graph[j]];
            p.row_ptr += gd.row_off; p.arc_wide += gd.arc_off; p.n_rec = gd.n_rec; p.sum_bw = gd.sum_bw;
        }
        if (src < 0 || src >= n || t < 0 || t >= n || src == t) {
            if (tid == 0) p.flow_out[j] = FC_FLOW_INVALID;
            if (p.stats && tid < FC_NSTAT) p.stats[size_t(j) * FC_NSTAT + tid] = 0u;
            return;
        }
    } else if (GEN) {
        const int32_t a = int32_t(blockIdx.x) % p.N, it = int32_t(blockIdx.x) / p.N;
        const int32_t i = it >> 1, v = p.compute_ids[a];
        const int32_t pu = p.split_u[i], pw = p.split_w[i], pt = p.split_t[i];
        j = int32_t(blockIdx.x); U = p.split_U; k = p.split_k;
        gu = pu; gw = pw; gt = pt;
        if (pu < 0 || pu >= n || pw < 0 || pw >= n || pt < 0 || pt >= n || pu == pw || pw == pt) {
            if (tid == 0) p.flow_out[j] = FC_FLOW_INVALID;
            if (p.stats && tid < FC_NSTAT) p.stats[size_t(j) * FC_NSTAT + tid] = 0u;
            return;
        }
        // An unbounded arc (x, y) makes y as good a source as x, and x as good a sink as y, so its two ends
        // are merged: F(u, w) with the arcs (u, t) and (v, w) has the sources {u, t} and the sinks {w, v};
        // F(w, t) with the arcs (u, t) and (v, t) has the source w and the sinks {t, u, v}.  The source's
        // unbounded arc into s is what gives every compute node its k units.
        if ((it & 1) == 0) { src = pu; t = pw; src2 = pt != pu ? pt : -1; sa = v != pw ? v : -1; }
        else { src = pw; t = pt; sa = pu != pt ? pu : -1; sb = v != pt && v != pu ? v : -1; }
    } else if (p.cand_C) {
        // Workgroups go to the 8 XCDs (each with an L2 of its own) round-robin by index.  All candidates
        // of one sink read that sink's tables, so they are given indices that are equal modulo 8:
        // eight sinks are in flight side by side, one per XCD, each with its candidates one after another.
        const int32_t xcd = int32_t(blockIdx.x) & 7, q = int32_t(blockIdx.x) >> 3;
        const int32_t oct = q / p.cand_C, c = q - oct * p.cand_C;
        const int32_t place = oct * 8 + xcd;
        if (place >= p.N) return;                         // the last group of eight may be short
        const int32_t i = p.order ? p.order[place] : place;
        if (p.order && (i < 0 || i >= p.n_order)) return;
        j = c * p.N + i; t = p.compute_ids[i]; U = p.cand_U[c]; k = p.cand_k[c];
        if (RAT) D = p.cand_D[c];
    } else {
        if (p.order_chunked) {
            // the order lists the problems of one sink next to each other; workgroups go to the XCDs round-robin
            // by index, so a run of consecutive entries is given indices that are equal modulo 8 (see above)
            const int32_t xcd = int32_t(blockIdx.x) & 7, q = int32_t(blockIdx.x) >> 3;
            const int32_t idx = ((q / FC_ORDER_CHUNK) * 8 + xcd) * FC_ORDER_CHUNK + q % FC_ORDER_CHUNK;
            if (idx >= p.n_order) return;                 // the grid is padded to whole groups of eight runs
            j = p.order[idx];
        } else j = p.order ? p.order[blockIdx.x] : int32_t(blockIdx.x);
        if (p.order && (j < 0 || j >= p.n_order)) return;
        t = p.sink[j]; U = p.U[j]; k = p.k[j];
        if (RAT) D = p.Uden[j];
    }

    // ---- problem and its validity (uniform over the workgroup)
    const long long NKll = p.sum_w * (long long)k;       // all of s's arcs together: N * k, or k * (sum of the weights)
    const bool valid = t >= 0 && t < n && U >= 1 && k >= 1 && D >= 1 && NKll < (1ll << 31);
    if (!valid) {                       // both layouts write the same marker
        if (tid == 0) p.flow_out[j] = FC_FLOW_INVALID;
        if (p.stats && tid < FC_NSTAT) p.stats[size_t(j) * FC_NSTAT + tid] = 0u;
        return;
    }
    // the 16-bit layout holds flows up to 65535 = largest N*k it accepts; larger problems are left
    // to the 32-bit kernel, which in turn skips the ones the 16-bit kernel took
    const bool small = NKll <= 65535ll;
    if (GEN) {
        // "unbounded" = more than every finite cut carries: all link capacities plus all source arcs, plus one
        const long long big = (long long)U * p.sum_bw + NKll + 1;
        if (big >= (1ll << 30)) {
            if (tid == 0) p.flow_out[j] = FC_FLOW_UNSUPPORTED;
            if (p.stats && tid < FC_NSTAT) p.stats[size_t(j) * FC_NSTAT + tid] = 0u;
            return;
        }
    } else if (COMPACT) {
        if (!small) {
            if (!p.wide_available) {
                if (tid == 0) p.flow_out[j] = FC_FLOW_UNSUPPORTED;
                if (p.stats && tid < FC_NSTAT) p.stats[size_t(j) * FC_NSTAT + tid] = 0u;
            }
            return;
        }
    } else if (small && p.arc_compact != nullptr) return;
    // NK: what the sink can hold at most -- N * k, or the "unbounded" value of an edge-splitting problem;
    // capacities are clamped at it and the run ends when the sink holds it
    const int32_t NK = GEN ? int32_t((long long)U * p.sum_bw + NKll + 1) : int32_t(NKll);
    const ArcCap<RAT> arc_cap(U, D, NK);
    if (GEN && (sa == src || sb == src || (src2 >= 0 && sa == src2))) {   // a vertex is source and sink at once
        if (tid == 0) p.flow_out[j] = NK;
        if (p.stats && tid < FC_NSTAT) p.stats[size_t(j) * FC_NSTAT + tid] = 0u;
        return;
    }

    // The first pass sends every compute node's k units down the sink's first-arc tree; the arc below
    // vertex v then carries k * (compute nodes above it).  If even the most loaded arc, relative to
    // its bandwidth, has room (k * num <= U * den), no arc saturates, all N * k units arrive, and
    // that is the maximum the source can emit: the value is known without running the pass.
    if (p.tree_ratio) {
        const long long num = p.tree_ratio[2 * t], den = p.tree_ratio[2 * t + 1];
        if ((long long)k * num <= (long long)U * den) {
            if (tid == 0) { p.flow_out[j] = NK; p.sink_cost[t] = 1u; }
            if (p.stats && tid < FC_NSTAT) p.stats[size_t(j) * FC_NSTAT + tid] = 0u;
            return;
        }
    }

    const Carve cv = carve_lds(n, m0, COMPACT);
    State<COMPACT> st;
    st.f = reinterpret_cast<W *>(smem + cv.f); st.h = reinterpret_cast<W *>(smem + cv.h);
    st.e = reinterpret_cast<W *>(smem + cv.e);
    st.list0 = reinterpret_cast<W *>(smem + cv.list0); st.list1 = reinterpret_cast<W *>(smem + cv.list1);
    st.rp = reinterpret_cast<W *>(smem + cv.rp);
    st.sh = reinterpret_cast<Shared *>(smem + cv.sh);
    const int32_t lane = tid & 63;
    const int32_t lg = tid & (G - 1), grp = tid / G, ngrp = T / G;
    const unsigned long long gmask = (G == 64 ? ~0ull : ((1ull << G) - 1ull)) << (lane & ~(G - 1));

#ifdef FC_PHASE_TIMING
    long long tick_ = clock64();
#ifdef FC_WALLCLOCK
    const uint32_t wc_start_ = uint32_t(wall_clock64());
#endif
    uint32_t t_init = 0, t_compact = 0, t_discharge = 0, t_other = 0, t_post = 0, t_next = 0;
#endif
#ifdef FC_GRDETAIL
    uint32_t grdbg[3] = {0u, 0u, 0u};
#endif
    uint32_t c_push = 0, c_scan = 0, c_grscan = 0, c_rel = 0, c_dis = 0;   // per-thread counters
    uint32_t c_gr = 0, c_step = 0;                                         // thread 0 only

    // ---- preflow: every arc (s, c) saturated (excess k at every compute node), topology arcs empty
    const bool have_labels = p.labels != nullptr;
    int32_t stop_at = NK;                  // the run ends when this much has arrived
    const bool have_p1 = have_labels && p.p1 != nullptr;
    const uint4 *p1_row = have_p1 ? p.p1 + size_t(t) * size_t(n) : nullptr;
    int32_t d = have_labels ? int32_t(p.label_hmax[t]) : 0;   // first level: the highest one holding a compute node
    {
        uint4 *fz = reinterpret_cast<uint4 *>(smem + cv.f);
        const int32_t quads = int32_t((cv.h - cv.f) / 16);
        for (int32_t i = tid; i < quads; i += T) fz[i] = make_uint4(0u, 0u, 0u, 0u);
        // four vertices per lane when the 16-bit rows are 8-byte aligned (n a multiple of 4): the label row and the
        // row offsets come as 8- and 16-byte loads, heights, excess and offsets go out as 8-byte LDS stores
        const bool by_four = COMPACT && !GEN && have_labels && (n & 3) == 0 && p.src_w == nullptr;
        if (by_four) {
            const uint2 *lab4 = reinterpret_cast<const uint2 *>(p.labels + size_t(t) * size_t(n));
            const int4 *rp4 = reinterpret_cast<const int4 *>(p.row_ptr);
            uint2 *h2 = reinterpret_cast<uint2 *>(smem + cv.h), *e2 = reinterpret_cast<uint2 *>(smem + cv.e), *r2 = reinterpret_cast<uint2 *>(smem + cv.rp);
            for (int32_t i = tid; i < (n >> 2); i += T) {
                const uint2 l = lab4[i];
                const int4 r = rp4[i];
                h2[i] = make_uint2(l.x & 0x7fff7fffu, l.y & 0x7fff7fffu);
                e2[i] = make_uint2(((l.x >> 15) & 0x00010001u) * uint32_t(k), ((l.y >> 15) & 0x00010001u) * uint32_t(k));   // k < 2^16 here
                r2[i] = make_uint2(uint32_t(r.x) | (uint32_t(r.y) << 16), uint32_t(r.z) | (uint32_t(r.w) << 16));
            }
        }
        for (int32_t v = tid; v < n && !by_four; v += T) {
            st.rp[v] = W(p.row_ptr[v]);
            if (have_labels) {
                const uint32_t lc = p.labels[size_t(t) * size_t(n) + size_t(v)];
                uint32_t hv = lc & 0x7fffu;
                if (GEN) {
                    // distance to the nearest of the sinks; a source keeps the height n.  The tables measure
                    // distances in the whole graph, also along paths through a source: never too large, so valid.
                    if (sa >= 0) hv = min(hv, uint32_t(p.labels[size_t(sa) * size_t(n) + size_t(v)]) & 0x7fffu);
                    if (sb >= 0) hv = min(hv, uint32_t(p.labels[size_t(sb) * size_t(n) + size_t(v)]) & 0x7fffu);
                    if (v == src || v == src2) hv = uint32_t(n);
                }
                st.h[v] = W(hv);
                st.e[v] = W((lc & 0x8000u) ? (p.src_w ? k * p.src_w[v] : k) : 0);
            } else st.e[v] = W(p.is_compute[v] ? (p.src_w ? k * p.src_w[v] : k) : 0);
        }
        if (tid == 0) {
            st.rp[n] = W(p.row_ptr[n]);
            for (int i = 0; i < 2; ++i) { st.sh->cnt[i] = 0; st.sh->down[i] = 0; st.sh->nrel[i] = 0; st.sh->dnext[i] = 0; st.sh->dcarry[i] = 0; st.sh->back[i] = n; }
            st.sh->tmp = 0;
            for (int i = 0; i < FC_NSTAT; ++i) st.sh->st[i] = 0;
        }
        if (have_p1 && tid < 64) st.sh->off[tid] = p.level_off[size_t(t) * 64 + tid];
        for (int32_t i = tid; i < FC_LVLS; i += T) st.sh->lvl[i] = 0;
        lds_barrier();
        if (have_p1) {                     // level populations from the sink's level table
            const int32_t L = int32_t(st.sh->off[0]);
            if (tid >= 1 && tid <= L && tid < FC_LVLS) st.sh->lvl[tid] = int32_t(st.sh->off[2 + L - tid]) - int32_t(st.sh->off[1 + L - tid]);
        } else if (have_labels) {          // deep or large graphs: count (one atomic per wavefront and level run would be
            for (int32_t v = tid; v < n; v += T) {   // nicer; this path runs once per problem)
                const int32_t hv = int32_t(st.h[v]);
                if (hv >= 1 && hv < FC_LVLS) atomicAdd(&st.sh->lvl[hv], 1);
            }
        }
        if (GEN) {
            // preflow of the explicit sources: all their arcs are saturated.  Nothing ever returns to them
            // (they keep the height n), and what they hold themselves does not count.
            for (int which = 0; which < 2; ++which) {
                const int32_t x = which ? src2 : src;
                if (x < 0) continue;
                for (int32_t a = int32_t(st.rp[x]) + tid; a < int32_t(st.rp[x + 1]); a += T) {
                    const ArcRec r = load_arc<COMPACT>(p, a);
                    const int32_t cap = r.fwd ? arc_cap(r.bw) : 0;
                    if (cap > 0) { st.f[r.pair] = W(cap); st.excess_add_noret(r.w, cap); }
                }
            }
            lds_barrier();
            if (tid == 0) { st.e[src] = W(0); if (src2 >= 0) st.e[src2] = W(0); }
            lds_barrier();
        }
        if (GEN && p.pair_stop) {
            const int32_t lim = p.pair_stop[j];
            if (lim >= 0 && lim < NK) stop_at = lim;
        }
        if (GEN && p.split_early && !p.pair_src) {
            // gamma = min{c(e), c(f), min_v F - N k}: a flow of N k + min{c(e), c(f)} cannot be the binding term, so the
            // problem may stop when that much has arrived.  Both capacities are records of w's row.
            for (int32_t a = int32_t(st.rp[gw]) + tid; a < int32_t(st.rp[gw + 1]); a += T) {
                const ArcRec r = load_arc<COMPACT>(p, a);
                if (r.fwd && r.w == gt) atomicMax(&st.sh->st[0], uint32_t(arc_cap(r.bw)));
                if (!r.fwd && r.w == gu) atomicMax(&st.sh->st[1], uint32_t(arc_cap(r.bw)));
            }
            lds_barrier();
            const uint32_t cf = st.sh->st[0], ce = st.sh->st[1];
            stop_at = int32_t(NKll) + int32_t(ce < cf ? ce : cf) + (p.split_early == 2 ? int32_t(cf) : 0);
            if (stop_at > NK) stop_at = NK;                            // never above the "unbounded" value
            lds_barrier();
            if (tid == 0) { st.sh->st[0] = 0u; st.sh->st[1] = 0u; }
        }
        if (!have_labels) {
            global_relabel<COMPACT, RAT>(p, st, t, arc_cap, c_grscan FC_GRDBG_ARG, src, src2, sa, sb);
            if (tid == 0) ++c_gr;
        }
    }
    // what has arrived: at the sink, or at any of the sinks of an edge-splitting problem
    auto arrived = [&]() -> int32_t {
        int32_t a = st.excess(t);
        if (GEN) { if (sa >= 0) a += st.excess(sa); if (sb >= 0) a += st.excess(sb); }
        return a;
    };
    // first-pass entries are read one round ahead: the sink's levels lie back to back in p1_row, so
    // the entry a lane needs next is known before the current round (and its barrier) is done
    uint4 en_next = make_uint4(0u, 0u, 0u, 0u);
    bool fast = have_p1;                   // still in the table-driven first pass
    int32_t cur = 0;                       // list array whose front is discharged in this step
    int32_t pend_hmax = 0;                 // first pass: largest height put on the pending list so far
    int32_t prev_cnt = 0;                  // vertices discharged in the previous step (front of the other array)
    if (fast) {
        if (d >= 1) {
            const int32_t L = int32_t(st.sh->off[0]);
            const int32_t i0 = int32_t(st.sh->off[1 + L - d]) + tid;
            en_next = p1_row[i0 < n ? i0 : n - 1];
        }
    } else {
        d = rebuild_pending(st, n, t, 1);  // everything that holds excess, on array 1
        cur = 0;
    }
    FC_TICK(t_init);
    int32_t steps_since = 0, total_steps = 0, rel_since = 0, rises = 0;
    // a sink whose own cut has little slack tends to leave much excess stranded next to it after the
    // first pass: such problems get exact heights as soon as the working level first moves up
    int32_t rise_limit = p.gr_rises;
    if (p.tight_pct > 0 && !GEN) {
        const long long have = (long long)U * (long long)p.in_bw[t] / D + (p.is_compute[t] ? (p.src_w ? k * p.src_w[t] : k) : 0);
        if (have * 100ll < NKll * (long long)p.tight_pct) rise_limit = 1;
    }
    bool failed = false;

    // ---- steps: one height level each
    if (arrived() >= stop_at) d = 0;       // nothing to do (inside the loop the same test follows every step)
    while (d >= 1) {
        const int32_t sp = total_steps & 1;
        FC_TICK(t_other);
        int32_t cnt, lvltot = 0;
        if (fast) {
            // ---- fast part: one lane per vertex of the level, along its precomputed first arc.  That
            // arc carries no flow yet and its head still has its initial height d-1, because in the
            // first pass a vertex is touched for the first time in the step of its own level.
            const int32_t L = int32_t(st.sh->off[0]);
            const int32_t lo = int32_t(st.sh->off[1 + L - d]), hi = int32_t(st.sh->off[2 + L - d]);
            lvltot = hi - lo;
            for (int32_t base = 0; base < lvltot; base += T) {
                const int32_t pos = base + tid;
                const bool ok = pos < lvltot;
                const uint4 en = en_next;
                {   // next round of this level, else first round of the level below
                    const int32_t inext = (base + T < lvltot ? lo + base + T : hi) + tid;
                    en_next = p1_row[inext < n ? inext : n - 1];
                }
                const int32_t u = int32_t(en.z & 0xffffu);
                const int32_t ex = ok ? st.excess(u) : 0;
                if (ex > 0) {
                    const int32_t w = int32_t(en.x & 0x7fffu), pair = int32_t(en.x >> 16);
                    const int32_t cap = arc_cap(int32_t(en.y));
                    const int32_t delta = ex < cap ? ex : cap;
                    ++c_dis; ++c_scan; ++c_push;
                    st.f[pair] = W(delta);
                    st.excess_add_noret(w, delta);
                    st.excess_sub(u, delta);
                    if (w != t) st.sh->down[sp] = 1;
                    if (delta < ex) st.list(cur)[atomicAdd(&st.sh->cnt[sp], 1)] = W(u);   // the arc is full
                }
            }
        } else {
            // ---- take level d off the pending list (on the other array): its vertices go to the front
            // of this array, the rest is carried over to this array's pending part
            // The source has two parts: its pending part [b0, n), and its old front [0, prev_cnt) -- the
            // vertices discharged in the last step, of which the ones still holding excess were stuck
            // (they have their new heights by now).  One counter update per wavefront and destination.
            const int32_t src = cur ^ 1;
            const int32_t b0 = st.sh->back[src];
            const int32_t total = prev_cnt + (n - b0);
            const unsigned long long below = (1ull << lane) - 1ull;
            for (int32_t base = 0; base < total; base += T) {
                const int32_t i = base + tid;
                bool isd = false, carry = false;
                int32_t v = 0, hv = 0;
                if (i < total) {
                    v = int32_t(st.list(src)[i < prev_cnt ? i : b0 + (i - prev_cnt)]);
                    hv = int32_t(st.h[v]);
                    if (hv & NEWH) { hv &= ~NEWH; st.h[v] = W(hv); }      // relabeled in the last step: the new height takes effect
                    const bool alive = hv < n && (i >= prev_cnt || st.excess(v) > 0);
                    isd = alive && hv == d; carry = alive && hv != d;
                }
                const unsigned long long bd = __ballot(isd), bc = __ballot(carry);
                if (bd) {
                    int32_t pos = 0;
                    if (lane == 0) pos = atomicAdd(&st.sh->cnt[sp], __popcll(bd));
                    pos = __builtin_amdgcn_readfirstlane(pos);
                    if (isd) st.list(cur)[pos + __popcll(bd & below)] = W(v);
                }
                if (bc) {
                    int32_t pos = 0;
                    const int32_t m = wave_max(carry ? hv : 0);
                    if (lane == 0) { pos = atomicSub(&st.sh->back[cur], __popcll(bc)) - __popcll(bc); atomicMax(&st.sh->dcarry[sp], m); }
                    pos = __builtin_amdgcn_readfirstlane(pos);
                    if (carry) st.list(cur)[pos + __popcll(bc & below)] = W(v);
                }
            }
        }
        lds_barrier();
        cnt = st.sh->cnt[sp];
        if (tid == 0) {                    // nobody reads these any more; they are written again after the next barrier at the earliest
            st.sh->cnt[sp ^ 1] = 0; st.sh->down[sp ^ 1] = 0; st.sh->nrel[sp ^ 1] = 0; st.sh->dnext[sp ^ 1] = 0; st.sh->dcarry[sp ^ 1] = 0;
            if (!fast) st.sh->back[cur ^ 1] = n;
        }
        FC_TICK(t_compact);

        // ---- group part: G lanes scan one listed vertex's residual row, a chunk at a time
        for (int32_t i = grp; i < cnt; i += ngrp) {
            const int32_t u = int32_t(st.list(cur)[i]);
            const int32_t beg = int32_t(st.rp[u]), end = int32_t(st.rp[u + 1]);
            const int32_t ex = st.excess(u);
            int32_t rem = ex;
            int32_t minh = 0x7fffffff;
            if (lg == 0) ++c_dis;
            for (int32_t base = beg; base < end && rem > 0; base += G) {
                const int32_t a = base + lg;
                int32_t ra = 0, hw = 0, fv = 0;
                ArcRec r; r.w = 0; r.pair = 0; r.bw = 0; r.fwd = 0; r.last = 0;
                if (a < end) {
                    r = load_arc<COMPACT>(p, a);
                    ++c_scan;
                    fv = int32_t(st.f[r.pair]);
                    ra = r.fwd ? arc_cap(r.bw) - fv : fv;
                    hw = st.height_during_step(r.w, d);
                }
                const bool adm = ra > 0 && hw + 1 == d;
                if (ra > 0 && !adm && hw < minh) minh = hw;
                const unsigned long long bal = __ballot(adm) & gmask;
                if (bal) {
                    int32_t delta = 0, rem_new;
                    const bool first = adm && ((bal & ((1ull << lane) - 1ull)) == 0ull);
                    const unsigned long long absorbed = __ballot(first && ra >= rem) & gmask;
                    if (absorbed) {                       // first admissible arc takes everything
                        if (first) delta = rem;
                        rem_new = 0;
                    } else {                              // split the excess in arc order
                        const int32_t x = adm ? ra : 0;
                        const int32_t incl = group_prefix_sum<G>(x, lg);
                        const int32_t total = group_allreduce<G>(x, [](int32_t a, int32_t b) { return a + b; });
                        const int32_t excl = incl - x;
                        delta = rem - excl; if (delta > x) delta = x; if (delta < 0) delta = 0;
                        rem_new = total >= rem ? 0 : rem - total;
                    }
                    if (delta > 0) {
                        st.f[r.pair] = W(r.fwd ? fv + delta : fv - delta);
                        ++c_push;
                        if (fast) {                       // the level below is walked in table order anyway
                            st.excess_add_noret(r.w, delta);
                            if (r.w != t) st.sh->down[sp] = 1;
                        } else if (GEN ? d == 1 : r.w == t) {   // into the sink (an edge-splitting problem can have three)
                            st.excess_add_noret(r.w, delta);
                        } else if (st.excess_add(r.w, delta) == 0) {
                            st.pend(cur, r.w);            // first excess this vertex gets: it becomes pending
                            st.sh->down[sp] = 1;
                        }
                    }
                    rem = rem_new;
                }
            }
            if (rem > 0) {                                // every admissible arc is saturated: relabel
                minh = group_allreduce<G>(minh, [](int32_t a, int32_t b) { return a < b ? a : b; });
                if (lg == 0) {
                    const int32_t nh = minh >= n - 1 ? n : minh + 1;
                    st.h[u] = W(NEWH | nh);
                    atomicAdd(&st.sh->nrel[sp], 1);
                    if (d < FC_LVLS) atomicSub(&st.sh->lvl[d], 1);
                    if (nh < FC_LVLS) atomicAdd(&st.sh->lvl[nh], 1);
                    if (nh < n) atomicMax(&st.sh->dnext[sp], nh);
                    ++c_rel;
                }
            }
            if (lg == 0 && rem != ex) st.excess_sub(u, ex - rem);
        }
        lds_barrier();
        FC_TICK(t_discharge);
        const int32_t nrel = st.sh->nrel[sp], down = st.sh->down[sp];
        const int32_t arr = arrived();     // read with the step's other results; nothing below moves excess
        int32_t dn = st.sh->dnext[sp];
        const int32_t dcarry = st.sh->dcarry[sp];
        // level d lost its last vertex: nothing above it can reach the sink any more
        const bool gap = p.use_gap && nrel > 0 && d < FC_LVLS && st.sh->lvl[d] == 0;
        ++steps_since; ++total_steps;
        if (tid == 0) ++c_step;

        if (nrel) {
            rel_since += nrel;
            if (gap) {
                // (pending entries that die here are dropped when their turn comes)
                for (int32_t v = tid; v < n; v += T) {
                    const int32_t raw = int32_t(st.h[v]), hv = raw & ~NEWH;
                    if ((raw & NEWH) || (hv > d && hv < n)) st.h[v] = W(n);   // flagged = relabeled in this step = above d
                }
                lds_barrier();                 // everybody has read lvl[d]
                for (int32_t i = d + 1 + tid; i < FC_LVLS; i += T) st.sh->lvl[i] = 0;
                pend_hmax = 0; dn = 0;
                lds_barrier();
            } else if (fast) {
                // the new heights take effect (deferred so that the level's scans all saw the same
                // heights).  In the first pass the list is rebuilt for every level, so the relabeled
                // vertices move to the pending list, kept on array 1; afterwards they are found again
                // in this array's front, and their flags are cleared then.
                for (int32_t i = tid; i < cnt; i += T) {
                    const int32_t u = int32_t(st.list(cur)[i]);
                    const int32_t raw = int32_t(st.h[u]);
                    if (raw & NEWH) {
                        st.h[u] = W(raw & ~NEWH);
                        if ((raw & ~NEWH) < n) st.pend(1, u);
                    }
                }
                lds_barrier();
            }
        }
        FC_TICK(t_post);
        if (arr >= stop_at) break;
        if (total_steps >= p.max_steps) { failed = true; break; }

        // ---- next level
        if (fast) {
            if (dn > pend_hmax) pend_hmax = dn;
            if (d > 1) {
                d = d - 1;                                // lower levels still hold their compute nodes
                // level 1's lanes push into the sink before the step's first barrier: wait until every
                // wavefront has taken this step's "sink is full" decision
                if (d == 1) lds_barrier();
            }
            else {                                        // first pass over: continue with the pending list (on array 0)
                fast = false; cur = 0; prev_cnt = 0; d = pend_hmax; rises = 1;
            }
        } else {
            if (dcarry > dn) dn = dcarry;
            if (down && d - 1 > dn) dn = d - 1;
            if (dn > d) ++rises;
            d = dn;
            prev_cnt = cnt;
            cur ^= 1;
        }
        if (!fast && rel_since > 0 && (rel_since >= p.gr_relabels || steps_since >= p.gr_steps || rises >= rise_limit) && d >= 1) {
            global_relabel<COMPACT, RAT>(p, st, t, arc_cap, c_grscan FC_GRDBG_ARG, src, src2, sa, sb);
            if (tid == 0) ++c_gr;
            rel_since = 0; steps_since = 0; rises = 0;
            d = rebuild_pending(st, n, t, cur ^ 1);
            prev_cnt = 0;
            if (tid == 0) { st.sh->back[cur] = n; st.sh->dnext[0] = st.sh->dnext[1] = 0; }
            lds_barrier();
        }
        FC_TICK(t_next);
    }

    lds_barrier();
    if (tid == 0) {
        int32_t et = arrived();
        if (GEN && et > NK) et = NK;       // "unbounded" is reported as one value
        p.flow_out[j] = failed ? FC_FLOW_NOCONVERGE : et;
        if (!GEN) p.sink_cost[t] = uint32_t(total_steps) + 6u * c_gr + 1u;
    }
    if (p.stats) {
#ifndef FC_PHASE_TIMING
        // one LDS update per wavefront and counter: sum over the lanes first
#pragma unroll
        for (int s = 32; s > 0; s >>= 1) {
            c_push += __shfl_xor(c_push, s); c_scan += __shfl_xor(c_scan, s); c_grscan += __shfl_xor(c_grscan, s);
            c_rel += __shfl_xor(c_rel, s); c_dis += __shfl_xor(c_dis, s);
        }
        if (lane == 0) {
            atomicAdd(&st.sh->st[0], c_push); atomicAdd(&st.sh->st[2], c_scan); atomicAdd(&st.sh->st[4], c_grscan);
            atomicAdd(&st.sh->st[1], c_rel); atomicAdd(&st.sh->st[6], c_dis);
        }
#endif
        if (tid == 0) { st.sh->st[3] = c_gr; st.sh->st[5] = c_step; st.sh->st[7] = failed ? 1u : 0u; }
#ifdef FC_PHASE_TIMING
        lds_barrier();
        FC_TICK(t_other);
        if (tid == 0) { st.sh->st[0] = t_init; st.sh->st[1] = t_compact; st.sh->st[2] = t_discharge; st.sh->st[3] = t_post; st.sh->st[4] = t_next; st.sh->st[6] = t_other; }
#ifdef FC_WALLCLOCK
        if (tid == 0) { st.sh->st[4] = uint32_t(wall_clock64()); st.sh->st[6] = wc_start_; }
#endif
#ifdef FC_GRDETAIL
        if (tid == 0) { st.sh->st[3] = grdbg[0]; st.sh->st[6] = grdbg[1]; st.sh->st[5] = grdbg[2]; }
#endif
#endif
        lds_barrier();
        if (tid < FC_NSTAT) p.stats[size_t(j) * FC_NSTAT + tid] = st.sh->st[tid];
    }
}

// Launch order: workgroups are dispatched in index order and a hard problem can run twenty times
// longer than a typical one, so the hard ones must start first or the launch ends with a long
// tail of idle CUs.  Every solved problem leaves its cost (level steps, plus a charge per global
// relabel) in a per-sink array that lives with the graph; problems of one sink with nearby
// candidates cost about the same, so the next launch sorts by it.  A sink not seen yet is guessed
// from the slack of its own cut, the cut the paper's initial range uses (Appendix E.1): in-capacity
// U * B^-(sink) (+ k) over the demand N * k.  One workgroup counting-sorts all problems.
constexpr int FC_ORDER_BUCKETS = 256;

// sort key of a problem: bucket 0 holds the most expensive ones
__device__ __forceinline__ int32_t order_bucket(int32_t t, int32_t u, int32_t kk, int32_t n, long long sum_w, const int32_t *in_bw,
                                                const uint8_t *is_compute, const uint32_t *sink_cost) {
    constexpr int NB = FC_ORDER_BUCKETS;
    if (t < 0 || t >= n || u < 1 || kk < 1) return NB - 1;                  // nothing to solve
    int32_t cost = int32_t(sink_cost[t]);
    if (cost == 0) {
        const long long need = sum_w * kk;
        const long long have = (long long)u * in_bw[t] + (is_compute[t] ? kk : 0);
        // ratio have / need against 1, 1.25, 1.5, 2, 3, 4, 6
        cost = have < need ? 80 : have * 4 < need * 5 ? 60 : have * 2 < need * 3 ? 45 : have < need * 2 ? 35
             : have < need * 3 ? 28 : have < need * 4 ? 22 : have < need * 6 ? 16 : 10;
    }
    return NB - 1 - (cost < NB - 1 ? cost : NB - 1);
}

// counter[b] += 1 for every active lane, one LDS atomic per distinct b in the wavefront; returns the
// value each lane's own increment would have returned (all 64 lanes must call)
__device__ __forceinline__ int32_t wave_bucket_add(int32_t *counter, int32_t b, bool active) {
    const int32_t lane = threadIdx.x & 63;
    const unsigned long long below = (1ull << lane) - 1ull;
    unsigned long long todo = __ballot(active);
    int32_t pos = 0;
    while (todo) {
        const int32_t leader = __ffsll((long long)todo) - 1;
        const int32_t bb = __builtin_amdgcn_readlane(b, leader);
        const unsigned long long same = __ballot(active && b == bb);
        int32_t start = 0;
        if (lane == leader) start = atomicAdd(&counter[bb], __popcll(same));
        start = __builtin_amdgcn_readlane(start, leader);
        if (active && b == bb) pos = start + __popcll(same & below);
        todo &= ~same;
    }
    return pos;
}

// exclusive prefix sum of hist[] into base[] by one wavefront (threads 0..63 of the workgroup)
__device__ __forceinline__ void order_bucket_bases(const int32_t *hist, int32_t *base, int32_t tid) {
    int32_t acc = 0;
    for (int c0 = 0; c0 < FC_ORDER_BUCKETS; c0 += 64) {
        const int32_t x = hist[c0 + tid];
        const int32_t incl = wave_prefix_sum(x);
        base[c0 + tid] = acc + incl - x;
        acc += __builtin_amdgcn_readlane(incl, 63);
    }
}

__global__ void __launch_bounds__(1024) fc_order_kernel(long long P, int32_t n, long long sum_w, const int32_t *sink,
                                                        const int32_t *U, const int32_t *k, const int32_t *in_bw,
                                                        const uint8_t *is_compute, const uint32_t *sink_cost,
                                                        int32_t *order, const int32_t *Uden, uint8_t *keys) {
    constexpr int NB = FC_ORDER_BUCKETS, R = 8;
    // a rational multiplier U / Uden only enters the guess for sinks without history: its integer part will do
    auto mult = [&](long long jj) { const int32_t u = U[jj]; if (!Uden) return u; const int32_t dd = Uden[jj]; return dd >= 1 && u >= dd ? u / dd : (u >= 1 && dd >= 1 ? 1 : 0); };
    __shared__ int32_t hist[NB], base[NB];
    const int32_t tid = threadIdx.x, T = blockDim.x;
    for (int32_t b = tid; b < NB; b += T) hist[b] = 0;
    __syncthreads();
    // both passes take R problems per thread at a time so that the R load chains (sink -> cost) overlap
    for (long long j0 = 0; j0 < P; j0 += (long long)R * T) {
        int32_t b[R];
#pragma unroll
        for (int r = 0; r < R; ++r) {
            const long long jj = j0 + (long long)r * T + tid;
            b[r] = jj < P ? order_bucket(sink[jj], mult(jj), k[jj], n, sum_w, in_bw, is_compute, sink_cost) : -1;
        }
#pragma unroll
        for (int r = 0; r < R; ++r) {
            (void)wave_bucket_add(hist, b[r], b[r] >= 0);
            // the key is kept: the cost hints may change under a concurrent call on another stream, and the
            // second pass must see the very buckets the first one counted
            if (b[r] >= 0) keys[j0 + (long long)r * T + tid] = uint8_t(b[r]);
        }
    }
    __syncthreads();
    if (tid < 64) order_bucket_bases(hist, base, tid);
    __syncthreads();
    for (long long j0 = 0; j0 < P; j0 += (long long)R * T) {
        int32_t b[R];
#pragma unroll
        for (int r = 0; r < R; ++r) {
            const long long jj = j0 + (long long)r * T + tid;
            b[r] = jj < P ? int32_t(keys[jj]) : -1;
        }
#pragma unroll
        for (int r = 0; r < R; ++r) {
            const int32_t pos = wave_bucket_add(base, b[r], b[r] >= 0);
            if (b[r] >= 0) order[pos] = int32_t(j0 + (long long)r * T + tid);
        }
    }
}

// The same for graphs of at most FC_ORDER_BY_SINK_MAX vertices, where the per-vertex counters fit
// on chip: the SINKS are sorted by cost and every sink's problems follow each other in the order, so
// that they run at the same time on the same XCD and share the sink's tables in its L2 (the solver
// maps runs of FC_ORDER_CHUNK entries to one XCD).  A sink's key comes from its history, else from
// the guess for its first-listed problem.  Two passes over the problem list, one over the vertices.
constexpr int FC_ORDER_BY_SINK_MAX = 4096;

__global__ void __launch_bounds__(1024) fc_order_by_sink_kernel(long long P, int32_t n, long long sum_w,
                                                                const int32_t *__restrict__ sink, const int32_t *__restrict__ U,
                                                                const int32_t *__restrict__ k, const int32_t *__restrict__ in_bw,
                                                                const uint8_t *__restrict__ is_compute,
                                                                const uint32_t *__restrict__ sink_cost,
                                                                int32_t *__restrict__ order, const int32_t *__restrict__ Uden) {
    constexpr int NB = FC_ORDER_BUCKETS, NV = FC_ORDER_BY_SINK_MAX + 1, R = 8;
    __shared__ int32_t cnt[NV], rep[NV], hist[NB], base[NB];   // slot n: problems whose sink is not a vertex (last)
    const int32_t tid = threadIdx.x, T = blockDim.x;
    for (int32_t v = tid; v <= n; v += T) { cnt[v] = 0; rep[v] = 0x7fffffff; }
    for (int32_t b = tid; b < NB; b += T) hist[b] = 0;
    __syncthreads();
    for (long long j0 = 0; j0 < P; j0 += (long long)R * T) {
        int32_t t[R];
#pragma unroll
        for (int r = 0; r < R; ++r) {
            const long long jj = j0 + (long long)r * T + tid;
            t[r] = jj < P ? sink[jj] : -2;
        }
#pragma unroll
        for (int r = 0; r < R; ++r) {
            if (t[r] == -2) continue;
            const int32_t v = t[r] >= 0 && t[r] < n ? t[r] : n;
            atomicAdd(&cnt[v], 1);
            atomicMin(&rep[v], int32_t(j0 + (long long)r * T + tid));
        }
    }
    __syncthreads();
    // every listed sink's bucket, weighted by the number of its problems; the bucket is kept in rep[]
    for (int32_t v = tid; v <= n; v += T) {
        const int32_t c = cnt[v];
        int32_t b = NB - 1;
        if (c > 0 && v < n) {
            const int32_t jj = rep[v];
            int32_t u = U[jj];
            if (Uden) { const int32_t dd = Uden[jj]; u = dd >= 1 && u >= dd ? u / dd : (u >= 1 && dd >= 1 ? 1 : 0); }
            b = order_bucket(v, u, k[jj], n, sum_w, in_bw, is_compute, sink_cost);
        }
        rep[v] = b;
        if (c > 0) atomicAdd(&hist[b], c);
    }
    __syncthreads();
    if (tid < 64) order_bucket_bases(hist, base, tid);
    __syncthreads();
    // a contiguous range per sink inside its bucket (the invalid ones after every real sink of the last bucket)
    for (int32_t v = tid; v < n; v += T) {
        const int32_t c = cnt[v];
        if (c > 0) cnt[v] = atomicAdd(&base[rep[v]], c);
    }
    __syncthreads();
    if (tid == 0 && cnt[n] > 0) cnt[n] = atomicAdd(&base[NB - 1], cnt[n]);
    __syncthreads();
    for (long long j0 = 0; j0 < P; j0 += (long long)R * T) {
        int32_t t[R];
#pragma unroll
        for (int r = 0; r < R; ++r) {
            const long long jj = j0 + (long long)r * T + tid;
            t[r] = jj < P ? sink[jj] : -2;
        }
#pragma unroll
        for (int r = 0; r < R; ++r) {
            if (t[r] == -2) continue;
            const int32_t v = t[r] >= 0 && t[r] < n ? t[r] : n;
            order[atomicAdd(&cnt[v], 1)] = int32_t(j0 + (long long)r * T + tid);
        }
    }
}

// fc_feasible's problems are C candidates x N sinks (problem c * N + i).  Only the N sinks are
// sorted (by the cost of candidate 0): order[place] = i.  The solver derives each workgroup's
// (candidate, sink) from its index, so the C problems of a sink sit next to each other in the
// launch, which also keeps that sink's tables in cache while they run.
__global__ void __launch_bounds__(1024) fc_order_sinks_kernel(int32_t N, int32_t n, const int32_t *__restrict__ compute_ids,
                                                              const int32_t *__restrict__ cU, const int32_t *__restrict__ ck,
                                                              const int32_t *__restrict__ in_bw,
                                                              const uint8_t *__restrict__ is_compute,
                                                              const uint32_t *__restrict__ sink_cost,
                                                              int32_t *__restrict__ order, const int32_t *__restrict__ cD,
                                                              uint8_t *__restrict__ keys, long long sum_w) {
    constexpr int NB = FC_ORDER_BUCKETS, R = 4;
    __shared__ int32_t hist[NB], base[NB];
    const int32_t tid = threadIdx.x, T = blockDim.x;
    for (int32_t b = tid; b < NB; b += T) hist[b] = 0;
    __syncthreads();
    const int32_t d0 = cD ? cD[0] : 1, k0 = ck[0];
    const int32_t u0 = d0 >= 1 && cU[0] >= d0 ? cU[0] / d0 : (cU[0] >= 1 && d0 >= 1 ? 1 : 0);
    for (int32_t i0 = 0; i0 < N; i0 += R * T) {
        int32_t b[R];
#pragma unroll
        for (int r = 0; r < R; ++r) {
            const int32_t i = i0 + r * T + tid;
            b[r] = i < N ? order_bucket(compute_ids[i], u0, k0, n, sum_w, in_bw, is_compute, sink_cost) : -1;
        }
#pragma unroll
        for (int r = 0; r < R; ++r) {
            (void)wave_bucket_add(hist, b[r], b[r] >= 0);
            if (b[r] >= 0) keys[i0 + r * T + tid] = uint8_t(b[r]);       // kept for the second pass (see fc_order_kernel)
        }
    }
    __syncthreads();
    if (tid < 64) order_bucket_bases(hist, base, tid);
    __syncthreads();
    for (int32_t i0 = 0; i0 < N; i0 += R * T) {
        int32_t b[R];
#pragma unroll
        for (int r = 0; r < R; ++r) {
            const int32_t i = i0 + r * T + tid;
            b[r] = i < N ? int32_t(keys[i]) : -1;
        }
#pragma unroll
        for (int r = 0; r < R; ++r) {
            const int32_t pos = wave_bucket_add(base, b[r], b[r] >= 0);
            if (b[r] >= 0) order[pos] = i0 + r * T + tid;
        }
    }
}

// feasible_c = AND over sinks of [F(s, v) >= N * k_c] (Theorem 1 / Theorem 3); one workgroup per candidate.
// sum_w = N, or the sum of the compute nodes' weights when s's arcs have capacities m_c * k (Section 5.7).
__global__ void __launch_bounds__(256) fc_verdict_kernel(int32_t N, long long sum_w, const int32_t *compute_ids, const int32_t *ck,
                                                         const int32_t *cU, const int32_t *cD, const int32_t *flows,
                                                         uint8_t *feasible, int32_t *witness) {
    __shared__ int32_t s_wit;
    const int32_t c = blockIdx.x, tid = threadIdx.x;
    if (tid == 0) s_wit = 0x7fffffff;
    __syncthreads();
    const int32_t k = ck[c], U = cU[c];
    const long long need = sum_w * (long long)k;
    const bool ok_cand = U >= 1 && k >= 1 && (!cD || cD[c] >= 1) && need < (1ll << 31);
    int32_t best = 0x7fffffff;
    for (int32_t s = tid; s < N; s += blockDim.x) {
        int32_t fl = flows[size_t(c) * size_t(N) + size_t(s)];
        if (fl < 0 || (long long)fl < need) { int32_t v = compute_ids[s]; if (v < best) best = v; }
    }
    if (best != 0x7fffffff) atomicMin(&s_wit, best);
    __syncthreads();
    if (tid == 0) {
        bool feas = ok_cand && s_wit == 0x7fffffff;
        feasible[c] = feas ? 1 : 0;
        if (witness) witness[c] = (feas || !ok_cand) ? -1 : s_wit;
    }
}

__global__ void __launch_bounds__(256) fc_stats_reduce_kernel(long long P, const uint32_t *per_problem,
                                                              unsigned long long *totals) {
    __shared__ unsigned long long acc[FC_NSTAT];
    if (threadIdx.x < FC_NSTAT) acc[threadIdx.x] = 0ull;
    __syncthreads();
    unsigned long long mine[FC_NSTAT];
    for (int i = 0; i < FC_NSTAT; ++i) mine[i] = 0ull;
    for (long long j = (long long)blockIdx.x * blockDim.x + threadIdx.x; j < P; j += (long long)gridDim.x * blockDim.x)
        for (int i = 0; i < FC_NSTAT; ++i) mine[i] += per_problem[size_t(j) * FC_NSTAT + i];
    for (int i = 0; i < FC_NSTAT; ++i) if (mine[i]) atomicAdd(&acc[i], mine[i]);
    __syncthreads();
    if (threadIdx.x < FC_NSTAT && acc[threadIdx.x]) atomicAdd(&totals[threadIdx.x], acc[threadIdx.x]);
}

// ------------------------------------------------------------------------------------------ host helpers

#define HIP_TRY(expr) do { hipError_t e_ = (expr); if (e_ != hipSuccess) { return FC_EDEVICE; } } while (0)

size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

size_t lds_bytes(const fc_graph *g, bool compact) { return carve_lds(g->n, int32_t(g->m0), compact).total; }

// 15-bit vertex ids and arc ids, 16-bit row offsets
bool compact_ids_fit(const fc_graph *g) { return g->n <= 32767 && 2 * g->m0 <= 65535; }

struct Resolved {
    int32_t tree_certificate, T, G, gr_steps, gr_relabels, gr_rises, tight_pct, use_gap, use_labels, force_wide, max_steps, src_cap_bound, schedule;
};

int resolve_options(const fc_graph *g, const fc_options *o, Resolved *r) {
    fc_options z; std::memset(&z, 0, sizeof z);
    if (!o) o = &z;
    int32_t T = o->threads_per_problem;
    if (T == 0) {
        // A problem that fills much of a CU's LDS leaves room for few workgroups: give it four wavefronts.  When many
        // problems fit, one or two wavefronts each and more problems in flight are faster (measured on configs 3 to 5).
        const size_t wgs_by_lds = (160u * 1024u) / std::max<size_t>(lds_bytes(g, compact_ids_fit(g)), 1);
        T = wgs_by_lds < 8 ? 256 : (g->n >= 256 ? 128 : 64);
    }
    if (T < 64 || T > 1024 || (T % 64) != 0) return FC_EINVAL;
    int32_t G = o->lanes_per_vertex;
    if (G == 0) {
        double avg = g->n > 0 ? double(2 * g->m0) / double(g->n) : 1.0;
        G = 4; while (G < 64 && double(G) < 0.75 * avg) G *= 2;
    }
    if (G < 2 || G > 64 || (G & (G - 1)) != 0) return FC_EINVAL;
    if (G == 2) G = 4;
    r->T = T; r->G = G;
    r->gr_steps = o->global_relabel_steps > 0 ? o->global_relabel_steps : 32;
    int32_t permille = o->global_relabel_permille > 0 ? o->global_relabel_permille : 100;
    r->gr_relabels = std::max<int32_t>(1, int32_t((long long)g->n * permille / 1000));
    if (o->global_relabel_rises < -1 || o->tight_sink_percent < -1) return FC_EINVAL;
    r->gr_rises = o->global_relabel_rises > 0 ? o->global_relabel_rises : 0x7fffffff;   // default: off
    r->tight_pct = o->tight_sink_percent > 0 ? o->tight_sink_percent : (o->tight_sink_percent < 0 ? 0 : 200);
    if (o->use_gap < 0 || o->use_gap > 2 || o->use_label_table < 0 || o->use_label_table > 2) return FC_EINVAL;
    r->use_gap = o->use_gap != 2;
    r->use_labels = o->use_label_table != 2;
    r->force_wide = o->force_wide != 0;
    r->max_steps = o->max_level_steps > 0 ? o->max_level_steps : std::max<int32_t>(100000, 200 * g->n);
    if (o->src_cap_bound < 0) return FC_EINVAL;
    r->src_cap_bound = o->src_cap_bound;
    if (o->tree_certificate < 0 || o->tree_certificate > 2) return FC_EINVAL;
    r->tree_certificate = o->tree_certificate == 1;
    if (o->schedule < 0 || o->schedule > 2) return FC_EINVAL;
    r->schedule = o->schedule != 2;
    return FC_OK;
}

template <bool COMPACT, bool RAT, bool GEN, int G, int OCC>
int launch_occ(const KParams &kp, long long P, int32_t T, size_t lds, hipStream_t stream) {
    auto kern = fc_push_relabel_kernel<COMPACT, RAT, GEN, G, OCC>;
#ifdef FC_TUNING_BUILD
    if (const char *pad = getenv("FC_LDS_PAD")) lds += size_t(atol(pad));     // occupancy experiments: request more LDS than needed
#endif
    {   // the LDS a kernel may request is raised on demand, once per instantiation and size; host threads may race here
        static std::mutex guard;
        static size_t lds_allowed = 0;
        std::lock_guard<std::mutex> lock(guard);
        if (lds > lds_allowed) {
            HIP_TRY(hipFuncSetAttribute(reinterpret_cast<const void *>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, int(lds)));
            lds_allowed = lds;
        }
    }
    hipLaunchKernelGGL(kern, dim3(unsigned(P)), dim3(unsigned(T)), lds, stream, kp);
    HIP_TRY(hipGetLastError());
    return FC_OK;
}

// Which register budget: measured on MI355X, the edge-splitting kernels are fastest built for 6 wavefronts
// per SIMD; the others for as many as the LDS of a CU (160 KB) holds, between 5 and 8.
template <bool COMPACT, bool RAT, bool GEN, int G>
int launch_one(const KParams &kp, long long P, int32_t T, size_t lds, hipStream_t stream) {
    if constexpr (GEN) {
        return launch_occ<COMPACT, RAT, true, G, 6>(kp, P, T, lds, stream);
    } else {
        const size_t wgs_by_lds = std::min<size_t>(32, (160u * 1024u) / std::max<size_t>(lds, 1));
        const size_t waves_per_simd = wgs_by_lds * size_t(T / 64) / 4;      // what the LDS leaves room for
        if (waves_per_simd >= 8) return launch_occ<COMPACT, RAT, false, G, 8>(kp, P, T, lds, stream);
        if (waves_per_simd == 7) return launch_occ<COMPACT, RAT, false, G, 7>(kp, P, T, lds, stream);
        if (waves_per_simd == 6) return launch_occ<COMPACT, RAT, false, G, 6>(kp, P, T, lds, stream);
        return launch_occ<COMPACT, RAT, false, G, 5>(kp, P, T, lds, stream);
    }
}

template <bool COMPACT, bool RAT, bool GEN = false>
int launch_g(const KParams &kp, long long P, int32_t T, int32_t G, size_t lds, hipStream_t stream) {
    switch (G) {
        case 4: return launch_one<COMPACT, RAT, GEN, 4>(kp, P, T, lds, stream);
        case 8: return launch_one<COMPACT, RAT, GEN, 8>(kp, P, T, lds, stream);
        case 16: return launch_one<COMPACT, RAT, GEN, 16>(kp, P, T, lds, stream);
        case 32: return launch_one<COMPACT, RAT, GEN, 32>(kp, P, T, lds, stream);
        case 64: return launch_one<COMPACT, RAT, GEN, 64>(kp, P, T, lds, stream);
    }
    return FC_EINVAL;
}

// caller-provided scratch of a batch call: [per-problem counters][totals, 256 B][launch order][sort keys]
size_t ws_totals_off(long long P) { return align_up(size_t(P) * FC_NSTAT * 4, 256); }
size_t ws_order_off(long long P) { return ws_totals_off(P) + 256; }
size_t ws_keys_index(long long P) { return align_up(size_t(P) * 4, 256) / 4; }     // sort keys, one byte per problem, after the order (int32 units)
size_t stats_bytes(long long P) { return ws_order_off(P) + align_up(size_t(P) * 4, 256) + align_up(size_t(P), 256); }

struct StatsScratch { uint32_t *per_problem; unsigned long long *totals; };

// small launches fit the machine at once: order is moot
// problems given as candidates x compute nodes (problem c * N + i) instead of a list
struct CandidateGrid { int32_t C; const int32_t *d_U, *d_k, *d_D; };    // d_D: denominators of rational multipliers, or null

bool wants_order(const fc_graph *g, const Resolved &opt, long long P) { return opt.schedule && P > 2ll * g->n_cu; }

// the fields every launch shares: topology, heuristics, nothing problem-specific
void common_params(const fc_graph *g, const Resolved &opt, KParams *kp) {
    std::memset(kp, 0, sizeof *kp);
    kp->n = g->n; kp->N = g->N; kp->m0 = int32_t(g->m0);
    kp->n_rec = std::max<int32_t>(1, int32_t(2 * g->m0));
    {   // work-list entries of a global relabel: at most n (one per frontier vertex) + records / span <= 2n
        const long long rec = 2 * g->m0, nn = std::max<int32_t>(1, g->n);
        int32_t lanes = 4, shift = 2;
        while (lanes < 64 && (long long)lanes * nn < rec) { lanes *= 2; ++shift; }
        kp->gr_lanes = lanes; kp->gr_shift = shift;
        kp->gr_sub = int32_t(std::max<long long>(1, (rec + (long long)lanes * nn - 1) / ((long long)lanes * nn)));
    }
    kp->row_ptr = g->d_row_ptr;
    kp->arc_wide = reinterpret_cast<const int4 *>(g->d_arc_wide);
    kp->is_compute = g->d_is_compute;
    kp->compute_ids = g->d_compute_ids;
    kp->in_bw = g->d_in_bw; kp->sink_cost = g->d_sink_cost; kp->sum_bw = g->sum_bw;
    kp->src_w = g->d_src_weight; kp->sum_w = g->sum_w;
    kp->gr_steps = opt.gr_steps; kp->gr_relabels = opt.gr_relabels; kp->gr_rises = opt.gr_rises;
    kp->tight_pct = opt.tight_pct; kp->use_gap = opt.use_gap; kp->max_steps = opt.max_steps;
}

// Launch the solver kernels for P problems.  stats_ws: null, or room for P*FC_NSTAT u32 + FC_NSTAT u64.
int run_batch(const fc_graph *g, long long P, const int32_t *d_sink, const int32_t *d_U, const int32_t *d_k,
              int32_t *d_flow, const Resolved &opt, hipStream_t stream, uint32_t *d_stats_pp, int32_t *d_order,
              const CandidateGrid *grid = nullptr, hipEvent_t ev_solver_start = nullptr, const int32_t *d_Uden = nullptr) {
    const bool rational = grid ? grid->d_D != nullptr : d_Uden != nullptr;
    if (P > (1ll << 30)) return FC_EINVAL;
    KParams kp;
    common_params(g, opt, &kp);
    const bool compact_possible = !opt.force_wide && g->d_arc_compact != nullptr &&
                                  lds_bytes(g, true) <= size_t(g->lds_limit);
    bool wide_possible = lds_bytes(g, false) <= size_t(g->lds_limit);
    if (!compact_possible && !wide_possible) return FC_EUNSUPPORTED;
    // the caller vouches that every N * k_j fits the 16-bit layout: skip the 32-bit launch
    if (compact_possible && opt.src_cap_bound > 0 && (long long)g->sum_w * opt.src_cap_bound <= 65535ll) wide_possible = false;
    kp.arc_compact = compact_possible ? reinterpret_cast<const uint2 *>(g->d_arc_compact) : nullptr;
    kp.labels = opt.use_labels ? g->d_labels : nullptr;
    kp.label_hmax = g->d_label_hmax;
    kp.p1 = opt.use_labels ? reinterpret_cast<const uint4 *>(g->d_p1) : nullptr;
    kp.level_off = g->d_level_off;
    kp.tree_ratio = opt.tree_certificate && opt.use_labels && !rational && !g->d_src_weight ? g->d_tree_ratio : nullptr;   // the certificate's ratio test needs exact capacities U * b
    kp.sink = d_sink; kp.U = d_U; kp.k = d_k; kp.Uden = d_Uden; kp.flow_out = d_flow; kp.stats = d_stats_pp;
    kp.wide_available = wide_possible ? 1 : 0;
    if (grid) {
        kp.cand_C = grid->C; kp.cand_U = grid->d_U; kp.cand_k = grid->d_k; kp.cand_D = grid->d_D;
        if (wants_order(g, opt, P)) {
            hipLaunchKernelGGL(fc_order_sinks_kernel, dim3(1), dim3(1024), 0, stream, g->N, g->n, g->d_compute_ids,
                               grid->d_U, grid->d_k, g->d_in_bw, g->d_is_compute, g->d_sink_cost, d_order, grid->d_D,
                               reinterpret_cast<uint8_t *>(d_order + ws_keys_index(P)), (long long)g->sum_w);
            HIP_TRY(hipGetLastError());
            kp.order = d_order; kp.n_order = g->N;
        }
    } else if (wants_order(g, opt, P)) {
        if (g->n <= FC_ORDER_BY_SINK_MAX) {
            hipLaunchKernelGGL(fc_order_by_sink_kernel, dim3(1), dim3(1024), 0, stream, P, g->n, (long long)g->sum_w, d_sink, d_U, d_k,
                               g->d_in_bw, g->d_is_compute, g->d_sink_cost, d_order, d_Uden);
            kp.order_chunked = 1;
        } else {
            hipLaunchKernelGGL(fc_order_kernel, dim3(1), dim3(1024), 0, stream, P, g->n, (long long)g->sum_w, d_sink, d_U, d_k,
                               g->d_in_bw, g->d_is_compute, g->d_sink_cost, d_order, d_Uden,
                               reinterpret_cast<uint8_t *>(d_order + ws_keys_index(P)));
        }
        HIP_TRY(hipGetLastError());
        kp.order = d_order; kp.n_order = int32_t(P);
    }
    if (ev_solver_start) HIP_TRY(hipEventRecord(ev_solver_start, stream));    // after the ordering kernel
    // grid: one workgroup per problem; the candidate grid is padded to whole groups of eight sinks
    const long long grid_wgs = grid ? (long long)((g->N + 7) / 8) * 8 * grid->C
                             : kp.order_chunked ? (P + 8 * FC_ORDER_CHUNK - 1) / (8 * FC_ORDER_CHUNK) * (8 * FC_ORDER_CHUNK) : P;
    if (compact_possible) {
        int rc = rational ? launch_g<true, true>(kp, grid_wgs, opt.T, opt.G, lds_bytes(g, true), stream)
                          : launch_g<true, false>(kp, grid_wgs, opt.T, opt.G, lds_bytes(g, true), stream);
        if (rc != FC_OK) return rc;
    }
    if (wide_possible) {
        int rc = rational ? launch_g<false, true>(kp, grid_wgs, opt.T, opt.G, lds_bytes(g, false), stream)
                          : launch_g<false, false>(kp, grid_wgs, opt.T, opt.G, lds_bytes(g, false), stream);
        if (rc != FC_OK) return rc;
    }
    return FC_OK;
}

int fill_stats(long long P, uint32_t *d_pp, unsigned long long *d_tot, hipStream_t stream, hipEvent_t ev0,
               hipEvent_t ev1, fc_stats *out) {
    HIP_TRY(hipMemsetAsync(d_tot, 0, sizeof(unsigned long long) * FC_NSTAT, stream));
    if (P > 0) {
        unsigned blocks = unsigned(std::min<long long>((P + 255) / 256, 1024));
        hipLaunchKernelGGL(fc_stats_reduce_kernel, dim3(blocks), dim3(256), 0, stream, P, d_pp, d_tot);
        HIP_TRY(hipGetLastError());
    }
    unsigned long long h[FC_NSTAT];
    HIP_TRY(hipMemcpyAsync(h, d_tot, sizeof h, hipMemcpyDeviceToHost, stream));
    HIP_TRY(hipStreamSynchronize(stream));
    float ms = 0.f;
    HIP_TRY(hipEventElapsedTime(&ms, ev0, ev1));
    out->pushes = h[0]; out->relabels = h[1]; out->arc_scans = h[2]; out->global_relabels = h[3];
    out->gr_arc_scans = h[4]; out->level_steps = h[5]; out->discharges = h[6]; out->not_converged = h[7];
    out->device_ms = ms;
    return FC_OK;
}


}  // namespace

// ------------------------------------------------------------------------------------------ C ABI

namespace {
// with_tables = false skips the per-sink tables (for graphs that are only used by calls that cannot use them)
// 32-bit arc records {other end, topology arc, bandwidth, forward | last-of-row << 1} in row order
void fill_wide_records(const fc_graph *g, int4 *dst) {
    const size_t M = size_t(2 * g->m0);
    for (size_t i = 0; i < M; ++i) dst[i] = make_int4(g->other[i], g->pair[i], g->bw[i], g->fwd[i]);
    for (size_t v = 0; v < size_t(g->n); ++v) if (g->row_ptr[v + 1] > g->row_ptr[v]) dst[size_t(g->row_ptr[v + 1]) - 1].w |= 2;
}

int upload_impl(int32_t n_vertices, int64_t n_arcs, const int32_t *tail, const int32_t *head,
                const int32_t *bandwidth, const uint8_t *is_compute, bool with_tables, fc_graph **out) {
    if (!out) return FC_EINVAL;
    fc_graph *g = nullptr;
    int rc = fc_host_build(n_vertices, n_arcs, tail, head, bandwidth, is_compute, &g);
    if (rc != FC_OK) return rc;
    auto fail = [&](int code) { fc_graph_free(g); return code; };
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess) return fail(FC_EDEVICE);
    g->device = dev;
    int lds = 0, cus = 0;
    if (hipDeviceGetAttribute(&lds, hipDeviceAttributeMaxSharedMemoryPerBlock, dev) != hipSuccess) return fail(FC_EDEVICE);
    if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess) return fail(FC_EDEVICE);
    g->lds_limit = lds; g->n_cu = cus;
    if (lds_bytes(g, false) > size_t(lds) && !(compact_ids_fit(g) && lds_bytes(g, true) <= size_t(lds)))
        return fail(FC_EUNSUPPORTED);

    const size_t M = size_t(2 * g->m0), n = size_t(g->n);
    try {
        std::vector<int4> wide(M ? M : 1, make_int4(0, 0, 0, 0));
        std::vector<uint8_t> last(M ? M : 1, 0);                     // final record of a vertex's row
        for (size_t v = 0; v < n; ++v) if (g->row_ptr[v + 1] > g->row_ptr[v]) last[size_t(g->row_ptr[v + 1]) - 1] = 1;
        fill_wide_records(g, wide.data());
        g->on_device = true;
        if (hipMalloc(&g->d_row_ptr, sizeof(int32_t) * (n + 1)) != hipSuccess) return fail(FC_EDEVICE);
        if (hipMalloc(&g->d_arc_wide, sizeof(int4) * (M ? M : 1)) != hipSuccess) return fail(FC_EDEVICE);
        if (hipMalloc(&g->d_is_compute, n) != hipSuccess) return fail(FC_EDEVICE);
        if (hipMalloc(&g->d_compute_ids, sizeof(int32_t) * size_t(g->N)) != hipSuccess) return fail(FC_EDEVICE);
        if (hipMalloc(&g->d_in_bw, sizeof(int32_t) * n) != hipSuccess) return fail(FC_EDEVICE);
        if (hipMalloc(&g->d_sink_cost, sizeof(uint32_t) * n) != hipSuccess) return fail(FC_EDEVICE);
        if (hipMemset(g->d_sink_cost, 0, sizeof(uint32_t) * n) != hipSuccess) return fail(FC_EDEVICE);
        if (hipMemcpy(g->d_in_bw, g->in_bw.data(), sizeof(int32_t) * n, hipMemcpyHostToDevice) != hipSuccess) return fail(FC_EDEVICE);
        if (hipMemcpy(g->d_row_ptr, g->row_ptr.data(), sizeof(int32_t) * (n + 1), hipMemcpyHostToDevice) != hipSuccess) return fail(FC_EDEVICE);
        if (hipMemcpy(g->d_arc_wide, wide.data(), sizeof(int4) * (M ? M : 1), hipMemcpyHostToDevice) != hipSuccess) return fail(FC_EDEVICE);
        if (hipMemcpy(g->d_is_compute, g->is_compute.data(), n, hipMemcpyHostToDevice) != hipSuccess) return fail(FC_EDEVICE);
        if (hipMemcpy(g->d_compute_ids, g->compute_ids.data(), sizeof(int32_t) * size_t(g->N), hipMemcpyHostToDevice) != hipSuccess) return fail(FC_EDEVICE);
        if (compact_ids_fit(g)) {
            std::vector<uint2> cmp(M ? M : 1, make_uint2(0u, 0u));
            for (size_t i = 0; i < M; ++i)
                cmp[i] = make_uint2(uint32_t(g->other[i]) | (uint32_t(g->fwd[i]) << 15) | (uint32_t(g->pair[i]) << 16), uint32_t(g->bw[i]) | (uint32_t(last[i]) << 31));
            if (hipMalloc(&g->d_arc_compact, sizeof(uint2) * (M ? M : 1)) != hipSuccess) return fail(FC_EDEVICE);
            if (hipMemcpy(g->d_arc_compact, cmp.data(), sizeof(uint2) * (M ? M : 1), hipMemcpyHostToDevice) != hipSuccess) return fail(FC_EDEVICE);
        }
        // per-sink tables (built on the host from the topology alone), while they stay small: exact
        // initial labels (n^2 x 2 bytes) and, for graphs that fit the 16-bit record layout, first-pass
        // entries in level order (n^2 x 16 bytes)
        if (with_tables && n <= 8192) {
            const bool with_p1 = compact_ids_fit(g) && n <= 4096;
            std::vector<uint16_t> labels, hmax, level_off; std::vector<uint32_t> p1; std::vector<int32_t> tree_ratio;
            bool too_deep = false;
            int rc2 = fc_host_sink_tables(g, with_p1, labels, hmax, p1, level_off, tree_ratio, &too_deep);
            if (rc2 != FC_OK) return fail(rc2);
            if (hipMalloc(&g->d_labels, n * n * sizeof(uint16_t)) != hipSuccess) return fail(FC_EDEVICE);
            if (hipMalloc(&g->d_label_hmax, n * sizeof(uint16_t)) != hipSuccess) return fail(FC_EDEVICE);
            if (hipMemcpy(g->d_labels, labels.data(), n * n * sizeof(uint16_t), hipMemcpyHostToDevice) != hipSuccess) return fail(FC_EDEVICE);
            if (hipMemcpy(g->d_label_hmax, hmax.data(), n * sizeof(uint16_t), hipMemcpyHostToDevice) != hipSuccess) return fail(FC_EDEVICE);
            if (with_p1 && !too_deep) {                   // a sink deeper than the level table: no level order
                if (hipMalloc(&g->d_p1, n * n * 16) != hipSuccess) return fail(FC_EDEVICE);
                if (hipMalloc(&g->d_level_off, n * 64 * sizeof(uint16_t)) != hipSuccess) return fail(FC_EDEVICE);
                if (hipMemcpy(g->d_p1, p1.data(), n * n * 16, hipMemcpyHostToDevice) != hipSuccess) return fail(FC_EDEVICE);
                if (hipMemcpy(g->d_level_off, level_off.data(), n * 64 * sizeof(uint16_t), hipMemcpyHostToDevice) != hipSuccess) return fail(FC_EDEVICE);
                if (hipMalloc(&g->d_tree_ratio, n * 2 * sizeof(int32_t)) != hipSuccess) return fail(FC_EDEVICE);
                if (hipMemcpy(g->d_tree_ratio, tree_ratio.data(), n * 2 * sizeof(int32_t), hipMemcpyHostToDevice) != hipSuccess) return fail(FC_EDEVICE);
            }
        }
    } catch (const std::bad_alloc &) {
        return fail(FC_ENOMEM);
    }
    *out = g;
    return FC_OK;
}
}  // namespace

extern "C" int fc_graph_upload(int32_t n_vertices, int64_t n_arcs, const int32_t *tail, const int32_t *head,
                               const int32_t *bandwidth, const uint8_t *is_compute, fc_graph **out) {
    return upload_impl(n_vertices, n_arcs, tail, head, bandwidth, is_compute, true, out);
}

extern "C" int fc_graph_free(fc_graph *g) {
    if (!g) return FC_OK;
    if (g->on_device) {
        if (g->d_row_ptr) (void)hipFree(g->d_row_ptr);
        if (g->d_arc_wide) (void)hipFree(g->d_arc_wide);
        if (g->d_arc_compact) (void)hipFree(g->d_arc_compact);
        if (g->d_is_compute) (void)hipFree(g->d_is_compute);
        if (g->d_compute_ids) (void)hipFree(g->d_compute_ids);
        if (g->d_in_bw) (void)hipFree(g->d_in_bw);
        if (g->d_src_weight) (void)hipFree(g->d_src_weight);
        if (g->d_sink_cost) (void)hipFree(g->d_sink_cost);
        if (g->d_tree_ratio) (void)hipFree(g->d_tree_ratio);
        if (g->d_labels) (void)hipFree(g->d_labels);
        if (g->d_label_hmax) (void)hipFree(g->d_label_hmax);
        if (g->d_p1) (void)hipFree(g->d_p1);
        if (g->d_level_off) (void)hipFree(g->d_level_off);
    }
    delete g;
    return FC_OK;
}

extern "C" int fc_graph_set_source_weights(fc_graph *g, const int32_t *weight_per_vertex) {
    if (!g) return FC_EINVAL;
    if (!g->on_device) return FC_EDEVICE;
    if (!weight_per_vertex) {                            // back to the uniform case
        if (g->d_src_weight) { (void)hipFree(g->d_src_weight); g->d_src_weight = nullptr; }
        g->src_weight.clear(); g->sum_w = g->N;
        return FC_OK;
    }
    try {
        std::vector<int32_t> wts(size_t(g->n), 0);
        long long sum = 0;
        for (int32_t v = 0; v < g->n; ++v) {
            if (!g->is_compute[size_t(v)]) continue;     // entries of switches are ignored
            if (weight_per_vertex[v] < 0) return FC_EINVAL;
            wts[size_t(v)] = weight_per_vertex[v]; sum += weight_per_vertex[v];
        }
        if (sum < 1) return FC_EINVAL;
        if (sum >= (1ll << 31)) return FC_EOVERFLOW;
        if (!g->d_src_weight && hipMalloc(&g->d_src_weight, sizeof(int32_t) * size_t(g->n)) != hipSuccess) { g->d_src_weight = nullptr; return FC_EDEVICE; }
        if (hipMemcpy(g->d_src_weight, wts.data(), sizeof(int32_t) * size_t(g->n), hipMemcpyHostToDevice) != hipSuccess) return FC_EDEVICE;
        g->src_weight.swap(wts); g->sum_w = sum;
    } catch (const std::bad_alloc &) {
        return FC_ENOMEM;
    }
    return FC_OK;
}

extern "C" size_t fc_maxflow_batch_workspace_bytes(const fc_graph *g, int64_t n_problems) {
    if (!g || n_problems < 0) return 0;
    return stats_bytes(n_problems);
}

namespace {
int maxflow_batch_impl(const fc_graph *g, int64_t n_problems, const int32_t *d_sink,
                       const int32_t *d_edge_mult, const int32_t *d_mult_den, const int32_t *d_src_cap, int32_t *d_flow_out,
                       void *d_workspace, size_t workspace_bytes, void *hip_stream,
                       const fc_options *options_or_null, fc_stats *stats_or_null) {
    if (!g || n_problems < 0) return FC_EINVAL;
    if (!g->on_device) return FC_EDEVICE;
    Resolved opt;
    int rc = resolve_options(g, options_or_null, &opt);
    if (rc != FC_OK) return rc;
    if (n_problems == 0) { if (stats_or_null) std::memset(stats_or_null, 0, sizeof *stats_or_null); return FC_OK; }
    if (!d_sink || !d_edge_mult || !d_src_cap || !d_flow_out) return FC_EINVAL;
    if (!d_workspace || workspace_bytes < stats_bytes(n_problems) || (reinterpret_cast<uintptr_t>(d_workspace) & 255u)) return FC_EWORKSPACE;
    hipStream_t stream = reinterpret_cast<hipStream_t>(hip_stream);
    uint32_t *d_pp = reinterpret_cast<uint32_t *>(d_workspace);
    unsigned long long *d_tot = reinterpret_cast<unsigned long long *>(reinterpret_cast<unsigned char *>(d_workspace) + align_up(size_t(n_problems) * FC_NSTAT * 4, 256));
    int32_t *d_order = reinterpret_cast<int32_t *>(reinterpret_cast<unsigned char *>(d_workspace) + ws_order_off(n_problems));
    if (!stats_or_null) return run_batch(g, n_problems, d_sink, d_edge_mult, d_src_cap, d_flow_out, opt, stream, nullptr, d_order, nullptr, nullptr, d_mult_den);

    hipEvent_t ev0, ev1;
    HIP_TRY(hipEventCreate(&ev0));
    if (hipEventCreate(&ev1) != hipSuccess) { (void)hipEventDestroy(ev0); return FC_EDEVICE; }
    auto done = [&](int code) { (void)hipEventDestroy(ev0); (void)hipEventDestroy(ev1); return code; };
    rc = run_batch(g, n_problems, d_sink, d_edge_mult, d_src_cap, d_flow_out, opt, stream, d_pp, d_order, nullptr, ev0, d_mult_den);
    if (rc != FC_OK) return done(rc);
    if (hipEventRecord(ev1, stream) != hipSuccess) return done(FC_EDEVICE);
    rc = fill_stats(n_problems, d_pp, d_tot, stream, ev0, ev1, stats_or_null);
    if (rc != FC_OK) return done(rc);
    return done(stats_or_null->not_converged ? FC_ENOCONVERGE : FC_OK);
}
}  // namespace

extern "C" int fc_maxflow_batch(const fc_graph *g, int64_t n_problems, const int32_t *d_sink,
                                const int32_t *d_edge_mult, const int32_t *d_src_cap, int32_t *d_flow_out,
                                void *d_workspace, size_t workspace_bytes, void *hip_stream,
                                const fc_options *options_or_null, fc_stats *stats_or_null) {
    return maxflow_batch_impl(g, n_problems, d_sink, d_edge_mult, nullptr, d_src_cap, d_flow_out, d_workspace,
                              workspace_bytes, hip_stream, options_or_null, stats_or_null);
}

extern "C" int fc_maxflow_batch_floor(const fc_graph *g, int64_t n_problems, const int32_t *d_sink,
                                      const int32_t *d_mult_num, const int32_t *d_mult_den, const int32_t *d_src_cap,
                                      int32_t *d_flow_out, void *d_workspace, size_t workspace_bytes, void *hip_stream,
                                      const fc_options *options_or_null, fc_stats *stats_or_null) {
    if (n_problems > 0 && !d_mult_den) return FC_EINVAL;
    return maxflow_batch_impl(g, n_problems, d_sink, d_mult_num, d_mult_den, d_src_cap, d_flow_out, d_workspace,
                              workspace_bytes, hip_stream, options_or_null, stats_or_null);
}

extern "C" size_t fc_feasible_workspace_bytes(const fc_graph *g, int32_t n_candidates) {
    if (!g || n_candidates < 0) return 0;
    size_t P = size_t(n_candidates) * size_t(g->N);
    return align_up(P * 4, 256) + stats_bytes((long long)P);
}

namespace {
int feasible_impl(const fc_graph *g, int32_t n_candidates, const int32_t *d_edge_mult, const int32_t *d_mult_den,
                           const int32_t *d_src_cap, uint8_t *d_feasible_out, int32_t *d_witness_sink_or_null,
                           int32_t *d_flows_or_null, void *d_workspace, size_t workspace_bytes,
                           void *hip_stream, const fc_options *options_or_null, fc_stats *stats_or_null) {
    if (!g || n_candidates < 0) return FC_EINVAL;
    if (!g->on_device) return FC_EDEVICE;
    Resolved opt;
    int rc = resolve_options(g, options_or_null, &opt);
    if (rc != FC_OK) return rc;
    if (n_candidates == 0) { if (stats_or_null) std::memset(stats_or_null, 0, sizeof *stats_or_null); return FC_OK; }
    if (!d_edge_mult || !d_src_cap || !d_feasible_out) return FC_EINVAL;
    if (!d_workspace || workspace_bytes < fc_feasible_workspace_bytes(g, n_candidates) || (reinterpret_cast<uintptr_t>(d_workspace) & 255u)) return FC_EWORKSPACE;
    hipStream_t stream = reinterpret_cast<hipStream_t>(hip_stream);
    const long long P = (long long)n_candidates * g->N;
    unsigned char *ws = reinterpret_cast<unsigned char *>(d_workspace);
    size_t slab = align_up(size_t(P) * 4, 256);
    // workspace: [flows, one int per problem][the batch scratch]
    int32_t *d_flow = d_flows_or_null ? d_flows_or_null : reinterpret_cast<int32_t *>(ws);
    uint32_t *d_pp = reinterpret_cast<uint32_t *>(ws + slab);
    unsigned long long *d_tot = reinterpret_cast<unsigned long long *>(ws + slab + ws_totals_off(P));

    hipEvent_t ev0 = nullptr, ev1 = nullptr;
    if (stats_or_null) {
        HIP_TRY(hipEventCreate(&ev0));
        if (hipEventCreate(&ev1) != hipSuccess) { (void)hipEventDestroy(ev0); return FC_EDEVICE; }
    }
    auto done = [&](int code) { if (ev0) (void)hipEventDestroy(ev0); if (ev1) (void)hipEventDestroy(ev1); return code; };
    int32_t *d_order = reinterpret_cast<int32_t *>(ws + slab + ws_order_off(P));
    // the problem list (candidate c, compute node i) -> c * N + i is never written out: the solver
    // derives each workgroup's problem from its index.  device_ms brackets the solver kernel(s) only.
    const CandidateGrid grid{n_candidates, d_edge_mult, d_src_cap, d_mult_den};
    rc = run_batch(g, P, nullptr, nullptr, nullptr, d_flow, opt, stream, stats_or_null ? d_pp : nullptr, d_order, &grid, ev0);
    if (rc != FC_OK) return done(rc);
    if (stats_or_null && hipEventRecord(ev1, stream) != hipSuccess) return done(FC_EDEVICE);
    hipLaunchKernelGGL(fc_verdict_kernel, dim3(unsigned(n_candidates)), dim3(256), 0, stream, g->N, (long long)g->sum_w, g->d_compute_ids,
                       d_src_cap, d_edge_mult, d_mult_den, d_flow, d_feasible_out, d_witness_sink_or_null);
    if (hipGetLastError() != hipSuccess) return done(FC_EDEVICE);
    if (!stats_or_null) return done(FC_OK);
    rc = fill_stats(P, d_pp, d_tot, stream, ev0, ev1, stats_or_null);
    if (rc != FC_OK) return done(rc);
    return done(stats_or_null->not_converged ? FC_ENOCONVERGE : FC_OK);
}
}  // namespace

extern "C" int fc_feasible(const fc_graph *g, int32_t n_candidates, const int32_t *d_edge_mult,
                           const int32_t *d_src_cap, uint8_t *d_feasible_out, int32_t *d_witness_sink_or_null,
                           int32_t *d_flows_or_null, void *d_workspace, size_t workspace_bytes,
                           void *hip_stream, const fc_options *options_or_null, fc_stats *stats_or_null) {
    return feasible_impl(g, n_candidates, d_edge_mult, nullptr, d_src_cap, d_feasible_out, d_witness_sink_or_null,
                         d_flows_or_null, d_workspace, workspace_bytes, hip_stream, options_or_null, stats_or_null);
}

extern "C" int fc_feasible_floor(const fc_graph *g, int32_t n_candidates, const int32_t *d_mult_num,
                                 const int32_t *d_mult_den, const int32_t *d_src_cap, uint8_t *d_feasible_out,
                                 int32_t *d_witness_sink_or_null, int32_t *d_flows_or_null, void *d_workspace,
                                 size_t workspace_bytes, void *hip_stream, const fc_options *options_or_null,
                                 fc_stats *stats_or_null) {
    if (n_candidates > 0 && !d_mult_den) return FC_EINVAL;
    return feasible_impl(g, n_candidates, d_mult_num, d_mult_den, d_src_cap, d_feasible_out, d_witness_sink_or_null,
                         d_flows_or_null, d_workspace, workspace_bytes, hip_stream, options_or_null, stats_or_null);
}

namespace {
struct SearchCtx {
    const fc_graph *g; hipStream_t stream; const fc_options *opt;
    int32_t *d_U, *d_k; uint8_t *d_v; void *d_ws; size_t ws_bytes; int32_t cap;
    int32_t *tU, *tk; uint8_t *tv; int32_t tcap; int32_t tlen;
    int32_t fixed_k;                   // > 0: candidates are rational multipliers num / den tested with this k
};
int search_verdicts(void *vctx, int32_t n, const int32_t *U, const int32_t *k, uint8_t *out) {
    SearchCtx *c = static_cast<SearchCtx *>(vctx);
    if (n > c->cap) return FC_EINVAL;
    fc_options o; std::memset(&o, 0, sizeof o);
    if (c->opt) o = *c->opt;
    o.src_cap_bound = 0;
    if (o.tree_certificate == 0) o.tree_certificate = 1;       // the search needs verdicts, not counters
    int rc;
    HIP_TRY(hipMemcpyAsync(c->d_U, U, sizeof(int32_t) * size_t(n), hipMemcpyHostToDevice, c->stream));
    HIP_TRY(hipMemcpyAsync(c->d_k, k, sizeof(int32_t) * size_t(n), hipMemcpyHostToDevice, c->stream));
    if (c->fixed_k > 0) {              // k[] holds the denominators; the source arcs are the fixed k
        o.src_cap_bound = c->fixed_k;
        std::vector<int32_t> kk(size_t(n), c->fixed_k);
        int32_t *d_fixed = c->d_U + c->cap;
        HIP_TRY(hipMemcpyAsync(d_fixed, kk.data(), sizeof(int32_t) * size_t(n), hipMemcpyHostToDevice, c->stream));
        HIP_TRY(hipStreamSynchronize(c->stream));               // kk goes out of scope
        rc = fc_feasible_floor(c->g, n, c->d_U, c->d_k, d_fixed, c->d_v, nullptr, nullptr, c->d_ws, c->ws_bytes, c->stream, &o, nullptr);
    } else {
        for (int32_t i = 0; i < n; ++i) o.src_cap_bound = std::max(o.src_cap_bound, k[i]);
        rc = fc_feasible(c->g, n, c->d_U, c->d_k, c->d_v, nullptr, nullptr, c->d_ws, c->ws_bytes, c->stream, &o, nullptr);
    }
    if (rc != FC_OK) return rc;
    HIP_TRY(hipMemcpyAsync(out, c->d_v, size_t(n), hipMemcpyDeviceToHost, c->stream));
    HIP_TRY(hipStreamSynchronize(c->stream));
    for (int32_t i = 0; i < n; ++i) {
        if (c->tlen < c->tcap) {
            if (c->tU) c->tU[c->tlen] = U[i];
            if (c->tk) c->tk[c->tlen] = k[i];
            if (c->tv) c->tv[c->tlen] = out[i];
        }
        c->tlen++;
    }
    return FC_OK;
}
}  // namespace

extern "C" int fc_opt_throughput_search(const fc_graph *g, int32_t candidates_per_round, fc_rational *inv_xstar,
                                        fc_rational *U, int64_t *k, int32_t *rounds_or_null, void *hip_stream,
                                        const fc_options *options_or_null, int32_t *trace_U, int32_t *trace_k,
                                        uint8_t *trace_verdict, int32_t trace_capacity, int32_t *trace_len_or_null) {
    if (!g || !inv_xstar || !U || !k || candidates_per_round < 1 || candidates_per_round > 4096 || trace_capacity < 0) return FC_EINVAL;
    if (!g->on_device) return FC_EDEVICE;
    if (g->d_src_weight) return FC_EUNSUPPORTED;         // the paper defines this only for unit weights
    Resolved opt;
    int rc = resolve_options(g, options_or_null, &opt);
    if (rc != FC_OK) return rc;
    SearchCtx c; std::memset(&c, 0, sizeof c);
    c.g = g; c.stream = reinterpret_cast<hipStream_t>(hip_stream); c.opt = options_or_null;
    c.cap = std::max<int32_t>(candidates_per_round, 2);
    c.tU = trace_U; c.tk = trace_k; c.tv = trace_verdict; c.tcap = trace_capacity; c.tlen = 0;
    c.ws_bytes = fc_feasible_workspace_bytes(g, c.cap);
    auto cleanup = [&]() {
        if (c.d_U) (void)hipFree(c.d_U); if (c.d_k) (void)hipFree(c.d_k);
        if (c.d_v) (void)hipFree(c.d_v); if (c.d_ws) (void)hipFree(c.d_ws);
    };
    if (hipMalloc(&c.d_U, sizeof(int32_t) * 2 * size_t(c.cap)) != hipSuccess || hipMalloc(&c.d_k, sizeof(int32_t) * size_t(c.cap)) != hipSuccess ||
        hipMalloc(&c.d_v, size_t(c.cap)) != hipSuccess || hipMalloc(&c.d_ws, c.ws_bytes) != hipSuccess) { cleanup(); return FC_EDEVICE; }
    fc_rational r1, r2; int64_t kk = 0; int32_t rounds = 0;
    rc = fc_search_with_verdicts(g->N, g->min_in_bw, g->gcd_bw, candidates_per_round, search_verdicts, &c, &r1, &r2, &kk, &rounds);
    cleanup();
    if (rc != FC_OK) return rc;
    *inv_xstar = r1; *U = r2; *k = kk;
    if (rounds_or_null) *rounds_or_null = rounds;
    if (trace_len_or_null) *trace_len_or_null = c.tlen;
    return FC_OK;
}

namespace {
// gamma of Theorem 10 for one pair per workgroup: the smaller of the two capacities and of the two
// slacks  min_v F - N k  over the pair's 2N flows.
__global__ void __launch_bounds__(256) fc_split_gamma_kernel(int32_t N, int32_t n, int32_t U, int32_t k,
                                                             const int32_t *pu, const int32_t *pw, const int32_t *pt,
                                                             const int32_t *flows, const int32_t *row_ptr, const int4 *arcs,
                                                             const uint8_t *is_compute, int32_t *gamma, int32_t *slack_or_null) {
    __shared__ int32_t s_min, s_bad;
    const int32_t i = blockIdx.x, tid = threadIdx.x;
    if (tid == 0) { s_min = 0x7fffffff; s_bad = 0; }
    __syncthreads();
    int32_t best = 0x7fffffff, bad = 0;
    for (int32_t r = tid; r < 2 * N; r += blockDim.x) {
        const int32_t fl = flows[size_t(i) * size_t(2 * N) + size_t(r)];
        if (fl < 0) bad = 1; else if (fl < best) best = fl;
    }
    if (bad) atomicOr(&s_bad, 1);
    if (best != 0x7fffffff) atomicMin(&s_min, best);
    __syncthreads();
    if (tid == 0) {
        const int32_t u = pu[i], w = pw[i], t = pt[i];
        long long ce = -1, cf = -1;
        if (!s_bad && u >= 0 && u < n && w >= 0 && w < n && t >= 0 && t < n && !is_compute[w]) {
            for (int32_t a = row_ptr[u]; a < row_ptr[u + 1]; ++a) if ((arcs[a].w & 1) && arcs[a].x == w) ce = (long long)U * arcs[a].z;
            for (int32_t a = row_ptr[w]; a < row_ptr[w + 1]; ++a) if ((arcs[a].w & 1) && arcs[a].x == t) cf = (long long)U * arcs[a].z;
        }
        if (ce < 1 || cf < 1) { gamma[i] = FC_GAMMA_INVALID; if (slack_or_null) slack_or_null[i] = 0; }   // not two links through a switch, or a failed flow
        else {
            long long gm = (long long)s_min - (long long)N * k;
            if (slack_or_null) slack_or_null[i] = int32_t(gm);       // min_v F - N k, or a lower bound of it where a flow stopped early
            if (ce < gm) gm = ce;
            if (cf < gm) gm = cf;
            gamma[i] = int32_t(gm);
        }
    }
}
}  // namespace

extern "C" size_t fc_split_gamma_workspace_bytes(const fc_graph *g, int64_t n_pairs) {
    if (!g || n_pairs < 0) return 0;
    const long long P = (long long)n_pairs * 2 * g->N;
    return align_up(size_t(P) * 4, 256) + stats_bytes(P);
}

namespace {
// fc_split_gamma_batch, and for the switch-removal loop a variant that also returns every pair's slack
// min_v F - N k (exact, or the lower bound N k + min{c(e), c(f)} + c(f) - N k at which its flows stopped)
int split_gamma_impl(const fc_graph *g, int32_t U, int32_t k, int64_t n_pairs, const int32_t *d_u,
                     const int32_t *d_w, const int32_t *d_t, int32_t *d_gamma_out,
                     int32_t *d_flows_or_null, void *d_workspace, size_t workspace_bytes,
                     void *hip_stream, const fc_options *options_or_null, fc_stats *stats_or_null, int32_t *d_slack_or_null) {
    if (!g || n_pairs < 0 || U < 1 || k < 1) return FC_EINVAL;
    if (!g->on_device) return FC_EDEVICE;
    if (g->d_src_weight) return FC_EUNSUPPORTED;         // the paper defines this only for unit weights
    Resolved opt;
    int rc = resolve_options(g, options_or_null, &opt);
    if (rc != FC_OK) return rc;
    if (n_pairs == 0) { if (stats_or_null) std::memset(stats_or_null, 0, sizeof *stats_or_null); return FC_OK; }
    if (!d_u || !d_w || !d_t || !d_gamma_out) return FC_EINVAL;
    const long long P = (long long)n_pairs * 2 * g->N;
    if (P > (1ll << 30)) return FC_EINVAL;
    if ((long long)U * g->sum_bw + (long long)g->N * k + 1 >= (1ll << 30)) return FC_EOVERFLOW;
    if (lds_bytes(g, false) > size_t(g->lds_limit)) return FC_EUNSUPPORTED;      // these problems use the 32-bit state
    if (!d_workspace || workspace_bytes < fc_split_gamma_workspace_bytes(g, n_pairs) || (reinterpret_cast<uintptr_t>(d_workspace) & 255u)) return FC_EWORKSPACE;
    hipStream_t stream = reinterpret_cast<hipStream_t>(hip_stream);
    unsigned char *ws = reinterpret_cast<unsigned char *>(d_workspace);
    const size_t slab = align_up(size_t(P) * 4, 256);
    int32_t *d_flow = d_flows_or_null ? d_flows_or_null : reinterpret_cast<int32_t *>(ws);
    uint32_t *d_pp = reinterpret_cast<uint32_t *>(ws + slab);
    unsigned long long *d_tot = reinterpret_cast<unsigned long long *>(ws + slab + ws_totals_off(P));

    // these problems strand much excess (a source's saturated arcs carry more than the sinks take): on the
    // larger graphs exact heights after the second upward move of the working level save many steps
    if (!(options_or_null && options_or_null->global_relabel_rises) && g->n >= 256) opt.gr_rises = 2;
    KParams kp;
    common_params(g, opt, &kp);                          // no first-pass tables, no launch order: those fields stay null
    // initial heights from the per-sink distance tables (the distance to the nearest sink) instead of a first
    // search in the kernel: pays on the larger graphs (config 4: +10 % with exact flows, +38 % with early stops),
    // not on small ones (config 3: -5 % and -11 %)
    kp.labels = opt.use_labels && g->n >= 256 ? g->d_labels : nullptr;
    kp.label_hmax = g->d_label_hmax;
    kp.split_u = d_u; kp.split_w = d_w; kp.split_t = d_t; kp.split_U = U; kp.split_k = k;
    kp.split_early = d_flows_or_null ? 0 : (d_slack_or_null ? 2 : 1);   // exact flow values only when the caller wants to see them
    kp.flow_out = d_flow; kp.stats = stats_or_null ? d_pp : nullptr;
    kp.wide_available = 1;

    hipEvent_t ev0 = nullptr, ev1 = nullptr;
    if (stats_or_null) {
        HIP_TRY(hipEventCreate(&ev0));
        if (hipEventCreate(&ev1) != hipSuccess) { (void)hipEventDestroy(ev0); return FC_EDEVICE; }
    }
    auto done = [&](int code) { if (ev0) (void)hipEventDestroy(ev0); if (ev1) (void)hipEventDestroy(ev1); return code; };
    if (stats_or_null && hipEventRecord(ev0, stream) != hipSuccess) return done(FC_EDEVICE);
    // these problems start without tables, in worklist mode: fewer wavefronts per problem pay off
    // (four when few problems fit a CU's LDS and the runs are short because they may stop early: config 4 +12 %)
    const bool roomy = (160u * 1024u) / std::max<size_t>(lds_bytes(g, false), 1) >= 8;
    const int32_t T_gen = (options_or_null && options_or_null->threads_per_problem) ? opt.T
                        : (!roomy && kp.split_early) ? 256 : (g->n >= 256 ? 128 : 64);
    rc = launch_g<false, false, true>(kp, P, T_gen, opt.G, lds_bytes(g, false), stream);
    if (rc != FC_OK) return done(rc);
    if (stats_or_null && hipEventRecord(ev1, stream) != hipSuccess) return done(FC_EDEVICE);
    hipLaunchKernelGGL(fc_split_gamma_kernel, dim3(unsigned(n_pairs)), dim3(256), 0, stream, g->N, g->n, U, k, d_u, d_w, d_t,
                       d_flow, g->d_row_ptr, reinterpret_cast<const int4 *>(g->d_arc_wide), g->d_is_compute, d_gamma_out, d_slack_or_null);
    if (hipGetLastError() != hipSuccess) return done(FC_EDEVICE);
    if (!stats_or_null) return done(FC_OK);
    rc = fill_stats(P, d_pp, d_tot, stream, ev0, ev1, stats_or_null);
    if (rc != FC_OK) return done(rc);
    return done(stats_or_null->not_converged ? FC_ENOCONVERGE : FC_OK);
}
}  // namespace

extern "C" int fc_split_gamma_batch(const fc_graph *g, int32_t U, int32_t k, int64_t n_pairs, const int32_t *d_u,
                                    const int32_t *d_w, const int32_t *d_t, int32_t *d_gamma_out,
                                    int32_t *d_flows_or_null, void *d_workspace, size_t workspace_bytes,
                                    void *hip_stream, const fc_options *options_or_null, fc_stats *stats_or_null) {
    return split_gamma_impl(g, U, k, n_pairs, d_u, d_w, d_t, d_gamma_out, d_flows_or_null, d_workspace, workspace_bytes,
                            hip_stream, options_or_null, stats_or_null, nullptr);
}

extern "C" int fc_fixed_k_search(const fc_graph *g, int32_t k, int32_t candidates_per_round, fc_rational *U_star,
                                 int32_t *rounds_or_null, void *hip_stream, const fc_options *options_or_null,
                                 int32_t *trace_num, int32_t *trace_den, uint8_t *trace_verdict, int32_t trace_capacity,
                                 int32_t *trace_len_or_null) {
    if (!g || !U_star || k < 1 || candidates_per_round < 1 || candidates_per_round > 4096 || trace_capacity < 0) return FC_EINVAL;
    if (!g->on_device) return FC_EDEVICE;
    if (g->d_src_weight) return FC_EUNSUPPORTED;         // the paper defines this only for unit weights
    Resolved opt;
    int rc = resolve_options(g, options_or_null, &opt);
    if (rc != FC_OK) return rc;
    SearchCtx c; std::memset(&c, 0, sizeof c);
    c.g = g; c.stream = reinterpret_cast<hipStream_t>(hip_stream); c.opt = options_or_null; c.fixed_k = k;
    c.cap = std::max<int32_t>(candidates_per_round, 2);
    c.tU = trace_num; c.tk = trace_den; c.tv = trace_verdict; c.tcap = trace_capacity; c.tlen = 0;
    c.ws_bytes = fc_feasible_workspace_bytes(g, c.cap);
    auto cleanup = [&]() {
        if (c.d_U) (void)hipFree(c.d_U); if (c.d_k) (void)hipFree(c.d_k);
        if (c.d_v) (void)hipFree(c.d_v); if (c.d_ws) (void)hipFree(c.d_ws);
    };
    if (hipMalloc(&c.d_U, sizeof(int32_t) * 2 * size_t(c.cap)) != hipSuccess || hipMalloc(&c.d_k, sizeof(int32_t) * size_t(c.cap)) != hipSuccess ||
        hipMalloc(&c.d_v, size_t(c.cap)) != hipSuccess || hipMalloc(&c.d_ws, c.ws_bytes) != hipSuccess) { cleanup(); return FC_EDEVICE; }
    fc_rational r; int32_t rounds = 0;
    rc = fc_fixed_k_search_with_verdicts(g->N, g->min_in_bw, g->max_bw, k, candidates_per_round, search_verdicts, &c, &r, &rounds);
    cleanup();
    if (rc != FC_OK) return rc;
    *U_star = r;
    if (rounds_or_null) *rounds_or_null = rounds;
    if (trace_len_or_null) *trace_len_or_null = c.tlen;
    return FC_OK;
}

// Algorithm 2 (Remove Switch Nodes, Appendix E.2) around the gamma batches: host loop, one batch per accepted
// split.  For a fixed egress link f = (w, t) the gammas of all remaining ingress links are evaluated on the
// current graph in one launch; the first positive one (in ingress order) is applied -- the ones before it are
// zero on this very graph, exactly what the one-at-a-time loop of the pseudocode would have found -- and the
// rest is evaluated again on the new graph.
namespace {
// Memory that fc_remove_switches keeps over its batches.  Every accepted split changes the graph, so
// every batch needs the residual CSR anew -- but no fresh allocation and only one copy: the host
// fills a pinned image [row offsets | in-bandwidths | pair lists | arc records] and one transfer puts
// it into a device block of the same layout, which also holds what does not change (compute flags
// and ids), the gamma values and the batch call's workspace.
struct SplitPool {
    int32_t n = 0, N = 0;
    size_t rec_cap = 0, pair_cap = 0;                     // arc records and pairs there is room for
    size_t off_row = 0, off_inbw = 0, off_wts = 0, off_pairs = 0, off_wide = 0, off_is = 0, off_ids = 0, off_cost = 0, off_gamma = 0, off_ws = 0, ws_bytes = 0;
    unsigned char *d_blob = nullptr, *h_blob = nullptr;   // h_blob: pinned, covers [0, off_ws)
    SplitPool() = default;
    SplitPool(const SplitPool &) = delete;
    SplitPool &operator=(const SplitPool &) = delete;
    ~SplitPool() { release(); }
    void release() {
        if (d_blob) (void)hipFree(d_blob);
        if (h_blob) (void)hipHostFree(h_blob);
        d_blob = nullptr; h_blob = nullptr; rec_cap = 0; pair_cap = 0;
    }
    // room for `recs` arc records and `pairs` pairs; growing re-creates both blocks (contents are rewritten by every batch)
    // (with_workspace: room for the counters and flows of pairs * 2N edge-splitting max-flows behind the block)
    int ensure(const fc_graph *h, size_t recs, size_t pairs, hipStream_t stream, bool with_workspace = true) {
        if (d_blob && n == h->n && N == h->N && recs <= rec_cap && pairs <= pair_cap) return FC_OK;
        // more room only where it ran out (the block is also rebuilt when the vertex set changes)
        const size_t want_rec = recs > rec_cap ? std::max<size_t>(recs + recs / 2 + 64, 2 * rec_cap) : rec_cap;    // splits add links: leave headroom
        const size_t want_pairs = pairs > pair_cap ? std::max<size_t>(std::max<size_t>(pairs, 1), d_blob ? 2 * pair_cap : size_t(h->n)) : pair_cap;
        if (d_blob && hipStreamSynchronize(stream) != hipSuccess) return FC_EDEVICE;
        release();
        n = h->n; N = h->N;
        size_t o = 0;
        off_row = o; o = align_up(o + sizeof(int32_t) * (size_t(n) + 1), 256);
        off_inbw = o; o = align_up(o + sizeof(int32_t) * size_t(n), 256);
        off_wts = o; o = align_up(o + sizeof(int32_t) * size_t(n), 256);     // source weights (tree construction)
        off_pairs = o; o = align_up(o + sizeof(int32_t) * 3 * want_pairs, 256);
        off_wide = o; o = align_up(o + sizeof(int4) * want_rec, 256);
        off_is = o; o = align_up(o + size_t(n), 256);
        off_ids = o; o = align_up(o + sizeof(int32_t) * size_t(N), 256);
        off_cost = o; o = align_up(o + sizeof(uint32_t) * size_t(n), 256);
        off_gamma = o; o = align_up(o + sizeof(int32_t) * 2 * want_pairs, 256);   // gamma values, then slacks
        off_ws = o;
        const long long P = (long long)want_pairs * 2 * N;
        ws_bytes = with_workspace ? align_up(size_t(P) * 4, 256) + stats_bytes(P) : 0;
        if (hipMalloc(reinterpret_cast<void **>(&d_blob), off_ws + ws_bytes) != hipSuccess) { d_blob = nullptr; return FC_EDEVICE; }
        if (hipHostMalloc(reinterpret_cast<void **>(&h_blob), off_ws, hipHostMallocDefault) != hipSuccess) { h_blob = nullptr; release(); return FC_EDEVICE; }
        rec_cap = want_rec; pair_cap = want_pairs;
        std::memset(h_blob, 0, off_ws);
        std::memcpy(h_blob + off_is, h->is_compute.data(), size_t(n));
        std::memcpy(h_blob + off_ids, h->compute_ids.data(), sizeof(int32_t) * size_t(N));
        if (hipMemcpyAsync(d_blob + off_is, h_blob + off_is, off_gamma - off_is, hipMemcpyHostToDevice, stream) != hipSuccess) return FC_EDEVICE;
        return FC_OK;
    }
};
}  // namespace

// ---------------------------------------------------------------------------------------------
// Spanning tree construction (Appendix E.3).  mu for an edge (x, y) that leaves the root-set being
// grown is  min{ g(x, y), m(R_grow), F(x, y; D-bar) - sum of the other demands },  where D-bar adds to
// the digraph one vertex s_i per other root-set with an arc (x, s_i) of capacity m(R_i) and unbounded
// arcs from s_i to the members of R_i.  The arcs (x, s_i) never exist as arcs here: they are saturated
// by definition of the preflow, so s_i simply starts with the excess m(R_i) -- the same device that
// gives the compute nodes their k units in the auxiliary network.  Most s_i are not needed either (see
// TreeCsr::build).  All candidate edges of a state are explicit (source, sink) problems of one launch.
namespace {
struct TreeState {
    int32_t n = 0;                                       // vertices of D*
    std::map<std::pair<int32_t, int32_t>, long long> g;  // remaining capacities
    std::vector<std::vector<int32_t>> members;           // root-sets, members in increasing order
    std::vector<uint8_t> inside;                         // [set][vertex] membership
    std::vector<long long> demand;
};

int tree_state_from_arrays(int32_t n_vertices, int64_t n_links, const int32_t *tail, const int32_t *head, const int32_t *capacity,
                           int32_t n_sets, const int64_t *set_ptr, const int32_t *set_members, const int32_t *set_demand, TreeState *st) {
    if (n_vertices < 2 || n_links < 0 || n_sets < 2 || !set_ptr || !set_demand || (n_links > 0 && (!tail || !head || !capacity))) return FC_EINVAL;
    st->n = n_vertices;
    for (int64_t i = 0; i < n_links; ++i) {
        if (tail[i] < 0 || tail[i] >= n_vertices || head[i] < 0 || head[i] >= n_vertices || capacity[i] < 0) return FC_EINVAL;
        if (tail[i] != head[i] && capacity[i] > 0) st->g[std::make_pair(tail[i], head[i])] += capacity[i];
    }
    st->members.assign(size_t(n_sets), std::vector<int32_t>());
    st->inside.assign(size_t(n_sets) * size_t(n_vertices), 0);
    st->demand.assign(size_t(n_sets), 0);
    for (int32_t i = 0; i < n_sets; ++i) {
        if (set_ptr[i] > set_ptr[i + 1] || set_ptr[i] < 0 || set_demand[i] < 1) return FC_EINVAL;
        st->demand[size_t(i)] = set_demand[i];
        for (int64_t q = set_ptr[i]; q < set_ptr[i + 1]; ++q) {
            const int32_t r = set_members[q];
            if (r < 0 || r >= n_vertices) return FC_EINVAL;
            if (!st->inside[size_t(i) * size_t(n_vertices) + size_t(r)]) { st->inside[size_t(i) * size_t(n_vertices) + size_t(r)] = 1; st->members[size_t(i)].push_back(r); }
        }
        std::sort(st->members[size_t(i)].begin(), st->members[size_t(i)].end());
        if (st->members[size_t(i)].empty()) return FC_EINVAL;
    }
    return FC_OK;
}
}  // namespace

namespace {
// The residual CSR of D-bar for the construction's current state, kept on the host and edited in place: an
// accepted edge (x, y) of amount m lowers g(x, y) by m (an arc that reaches 0 stays as a record of capacity 0,
// which carries nothing); the grown root-set itself has no vertex in the network.  Copies with further edits
// are the graphs of the states a launch speculates on.
struct TreeCsr {
    int32_t nv = 0, m0 = 0;
    long long sum_g = 0;                                 // finite capacities only
    long long others = 0;                                // demands of the root-sets that are in the graph: F is measured against them
    long long spanning = 0;                              // demands of the root-sets left out because they span already
    std::vector<int32_t> row_ptr;                        // [nv + 1]
    std::vector<int4> rec;                               // {other, pair, capacity, forward | last-of-row << 1}
    std::vector<int32_t> weight;                         // [nv] excess a vertex starts with

    // D-bar for growing root-set `grow`, without the vertices it does not need.  A root-set that spans already has
    // an unbounded arc into y: its demand always arrives, so it is left out and its demand is not counted.  The
    // vertex s_l of a one-member root-set {u} only hands its m to u: u starts with that excess instead.  What
    // remains are the partly grown copies, each with its vertex and unbounded arcs to its members.
    int build(const TreeState &st, int32_t grow, int32_t unbounded) {
        const int32_t n = st.n, H = int32_t(st.members.size());
        std::vector<int32_t> at, ah, ab;
        sum_g = 0; others = 0; spanning = 0;
        for (const auto &kv : st.g) { at.push_back(kv.first.first); ah.push_back(kv.first.second); ab.push_back(int32_t(kv.second)); sum_g += kv.second; }
        std::vector<int32_t> wts(size_t(n), 0);
        int32_t extra = 0;
        for (int32_t l = 0; l < H; ++l) {
            if (l == grow) continue;
            const auto &R = st.members[size_t(l)];
            if (int32_t(R.size()) == n) { spanning += st.demand[size_t(l)]; continue; }
            others += st.demand[size_t(l)];
            if (R.size() == 1) { wts[size_t(R[0])] += int32_t(st.demand[size_t(l)]); continue; }
            for (int32_t r : R) { at.push_back(n + extra); ah.push_back(r); ab.push_back(unbounded); }
            wts.push_back(int32_t(st.demand[size_t(l)]));
            ++extra;
        }
        weight = wts;
        std::vector<uint8_t> flagged(size_t(n + extra), 1);    // every vertex may start with excess (most weights are 0)
        fc_graph *h = nullptr;
        const int rc = fc_host_build(n + extra, int64_t(at.size()), at.data(), ah.data(), ab.data(), flagged.data(), &h);
        if (rc != FC_OK) return rc;
        nv = h->n; m0 = int32_t(h->m0);
        row_ptr = h->row_ptr;
        rec.assign(size_t(2 * h->m0), make_int4(0, 0, 0, 0));
        fill_wide_records(h, rec.data());
        fc_graph_free(h);
        return FC_OK;
    }
    void lower(int32_t a, int32_t b, long long by) {       // the arc exists
        for (int32_t q = row_ptr[size_t(a)]; q < row_ptr[size_t(a) + 1]; ++q)
            if ((rec[size_t(q)].w & 1) && rec[size_t(q)].x == b) rec[size_t(q)].z -= int32_t(by);
        for (int32_t q = row_ptr[size_t(b)]; q < row_ptr[size_t(b) + 1]; ++q)
            if (!(rec[size_t(q)].w & 1) && rec[size_t(q)].x == a) rec[size_t(q)].z -= int32_t(by);
        sum_g -= by;
    }
};

// device block + pinned image for launches on several graphs of one vertex set
struct TreePool {
    unsigned char *d = nullptr, *h = nullptr;
    size_t cap = 0;
    ~TreePool() { release(); }
    TreePool() = default;
    TreePool(const TreePool &) = delete;
    TreePool &operator=(const TreePool &) = delete;
    void release() { if (d) (void)hipFree(d); if (h) (void)hipHostFree(h); d = nullptr; h = nullptr; cap = 0; }
    int ensure(size_t bytes, hipStream_t stream) {
        if (bytes <= cap) return FC_OK;
        if (d && hipStreamSynchronize(stream) != hipSuccess) return FC_EDEVICE;
        release();
        const size_t want = bytes + bytes / 2;
        if (hipMalloc(reinterpret_cast<void **>(&d), want) != hipSuccess) { d = nullptr; return FC_EDEVICE; }
        if (hipHostMalloc(reinterpret_cast<void **>(&h), want, hipHostMallocDefault) != hipSuccess) { h = nullptr; release(); return FC_EDEVICE; }
        cap = want;
        return FC_OK;
    }
};

struct ChainState {                                       // one speculated state: its graph and candidate edges
    TreeCsr csr;
    std::vector<int32_t> xs, ys;
    std::vector<long long> cap_xy;                        // g(x, y) in this state
    int32_t guess = -1;                                   // index of the candidate expected to be accepted in full, or -1
};

// One launch for a chain of states of root-set `grow`: chain[0] is the current state, chain[j + 1] is chain[j]
// after its guessed edge.  flows[j][q] receives F for candidate q of state j.
int tree_chain_launch(const TreeState &st, int32_t grow, const std::vector<ChainState> &chain, bool exact_flows,
                      std::vector<std::vector<int32_t>> &flows, hipStream_t stream, const fc_options *options_or_null, TreePool &pool) {
    const int32_t nv = chain[0].csr.nv, H = nv;          // every vertex is flagged as one that may start with excess
    const long long others = chain[0].csr.others;
    const size_t J = chain.size();
    size_t E = 0, recs = 0; int32_t m0max = 0;
    for (const ChainState &c : chain) { E += c.xs.size(); recs += c.csr.rec.size(); m0max = std::max(m0max, c.csr.m0); }
    // layout (256-byte aligned sections)
    size_t o = 0;
    const size_t off_desc = o; o = align_up(o + sizeof(GraphDesc) * J, 256);
    const size_t off_rows = o; o = align_up(o + sizeof(int32_t) * J * (size_t(nv) + 1), 256);
    const size_t off_pairs = o; o = align_up(o + sizeof(int32_t) * 4 * E, 256);
    const size_t off_wts = o; o = align_up(o + sizeof(int32_t) * size_t(nv), 256);
    const size_t off_is = o; o = align_up(o + size_t(nv), 256);
    const size_t off_ids = o; o = align_up(o + sizeof(int32_t) * size_t(H), 256);
    const size_t off_cost = o; o = align_up(o + sizeof(uint32_t) * size_t(nv), 256);
    const size_t off_rec = o; o = align_up(o + sizeof(int4) * std::max<size_t>(recs, 1), 256);
    const size_t upload = o;
    const size_t off_flow = o; o = align_up(o + sizeof(int32_t) * E, 256);
    int rc = pool.ensure(o, stream);
    if (rc != FC_OK) return rc;
    GraphDesc *desc = reinterpret_cast<GraphDesc *>(pool.h + off_desc);
    int32_t *rows = reinterpret_cast<int32_t *>(pool.h + off_rows), *pairs = reinterpret_cast<int32_t *>(pool.h + off_pairs);
    int32_t *wts = reinterpret_cast<int32_t *>(pool.h + off_wts), *ids = reinterpret_cast<int32_t *>(pool.h + off_ids);
    int4 *rec = reinterpret_cast<int4 *>(pool.h + off_rec);
    std::memset(pool.h + off_wts, 0, off_rec - off_wts);
    for (int32_t v = 0; v < nv; ++v) { wts[v] = chain[0].csr.weight[size_t(v)]; pool.h[off_is + size_t(v)] = 1; ids[v] = v; }
    size_t e = 0, r = 0;
    for (size_t j = 0; j < J; ++j) {
        const ChainState &c = chain[j];
        desc[j].row_off = int32_t(j * (size_t(nv) + 1)); desc[j].arc_off = int32_t(r); desc[j].n_rec = std::max<int32_t>(1, int32_t(c.csr.rec.size()));
        desc[j].pad = 0; desc[j].sum_bw = c.csr.sum_g;
        std::memcpy(rows + j * (size_t(nv) + 1), c.csr.row_ptr.data(), sizeof(int32_t) * (size_t(nv) + 1));
        if (!c.csr.rec.empty()) std::memcpy(rec + r, c.csr.rec.data(), sizeof(int4) * c.csr.rec.size());
        r += c.csr.rec.size();
        for (size_t q = 0; q < c.xs.size(); ++q, ++e) {
            pairs[e] = c.xs[q]; pairs[E + e] = c.ys[q];
            // a max-flow may stop once it cannot decide mu any more: at the other demands + min{g(x, y), m(R_grow)}
            pairs[2 * E + e] = exact_flows ? -1 : int32_t(others + std::min<long long>(c.cap_xy[q], st.demand[size_t(grow)]));
            pairs[3 * E + e] = int32_t(j);
        }
    }
    // a host-side stand-in for the graph object: the launch helpers read sizes and device pointers from it
    fc_graph hg;
    hg.n = nv; hg.N = H; hg.m0 = m0max; hg.sum_w = others; hg.sum_bw = chain[0].csr.sum_g;
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || hipDeviceGetAttribute(&hg.lds_limit, hipDeviceAttributeMaxSharedMemoryPerBlock, dev) != hipSuccess ||
        hipDeviceGetAttribute(&hg.n_cu, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess) return FC_EDEVICE;
    hg.device = dev; hg.on_device = true;
    hg.d_row_ptr = reinterpret_cast<int32_t *>(pool.d + off_rows);
    hg.d_arc_wide = pool.d + off_rec;
    hg.d_is_compute = pool.d + off_is;
    hg.d_compute_ids = reinterpret_cast<int32_t *>(pool.d + off_ids);
    hg.d_in_bw = reinterpret_cast<int32_t *>(pool.d + off_cost);       // unused by these launches; any [nv] array will do
    hg.d_sink_cost = reinterpret_cast<uint32_t *>(pool.d + off_cost);
    hg.d_src_weight = reinterpret_cast<int32_t *>(pool.d + off_wts);
    auto done = [&](int code) {                          // the pool owns the device memory
        hg.on_device = false;
        hg.d_row_ptr = nullptr; hg.d_arc_wide = nullptr; hg.d_is_compute = nullptr; hg.d_compute_ids = nullptr; hg.d_in_bw = nullptr;
        hg.d_sink_cost = nullptr; hg.d_src_weight = nullptr;
        return code;
    };
    if (lds_bytes(&hg, false) > size_t(hg.lds_limit)) return done(FC_EUNSUPPORTED);
    if (hipMemcpyAsync(pool.d, pool.h, upload, hipMemcpyHostToDevice, stream) != hipSuccess) return done(FC_EDEVICE);
    Resolved opt;
    rc = resolve_options(&hg, options_or_null, &opt);
    if (rc != FC_OK) return done(rc);
    KParams kp;
    common_params(&hg, opt, &kp);
    int32_t *d_pairs = reinterpret_cast<int32_t *>(pool.d + off_pairs);
    kp.pair_src = d_pairs; kp.pair_dst = d_pairs + E; kp.pair_stop = d_pairs + 2 * E; kp.pair_graph = d_pairs + 3 * E;
    kp.graphs = reinterpret_cast<const GraphDesc *>(pool.d + off_desc);
    kp.split_U = 1; kp.split_k = 1;
    kp.flow_out = reinterpret_cast<int32_t *>(pool.d + off_flow); kp.wide_available = 1;
    const int32_t T = (options_or_null && options_or_null->threads_per_problem) ? opt.T : (nv >= 256 ? 128 : 64);
    rc = launch_g<false, false, true>(kp, (long long)E, T, opt.G, lds_bytes(&hg, false), stream);
    if (rc != FC_OK) return done(rc);
    const int32_t *h_flow = reinterpret_cast<const int32_t *>(pool.h + off_flow);
    if (hipMemcpyAsync(pool.h + off_flow, pool.d + off_flow, sizeof(int32_t) * E, hipMemcpyDeviceToHost, stream) != hipSuccess ||
        hipStreamSynchronize(stream) != hipSuccess) return done(FC_EDEVICE);
    flows.assign(J, std::vector<int32_t>());
    e = 0;
    for (size_t j = 0; j < J; ++j) { flows[j].assign(h_flow + e, h_flow + e + chain[j].xs.size()); e += chain[j].xs.size(); }
    return done(FC_OK);
}
}  // namespace

extern "C" int fc_tree_mu_batch(int32_t n_vertices, int64_t n_links, const int32_t *tail, const int32_t *head, const int32_t *capacity,
                                int32_t n_sets, const int64_t *set_ptr, const int32_t *set_members, const int32_t *set_demand,
                                int32_t grow_set, int64_t n_edges, const int32_t *edge_x, const int32_t *edge_y,
                                int32_t *mu_out, int32_t *flows_or_null, void *hip_stream, const fc_options *options_or_null) {
    if (n_edges < 0 || grow_set < 0 || grow_set >= n_sets || (n_edges > 0 && (!edge_x || !edge_y || !mu_out))) return FC_EINVAL;
    try {
        TreeState st;
        int rc = tree_state_from_arrays(n_vertices, n_links, tail, head, capacity, n_sets, set_ptr, set_members, set_demand, &st);
        if (rc != FC_OK) return rc;
        if (n_edges == 0) return FC_OK;
        const int32_t n = st.n;
        long long sum_g = 0, all = 0;
        for (const auto &kv : st.g) sum_g += kv.second;
        for (long long m : st.demand) all += m;
        const long long unbounded = sum_g + all + 1;
        if (unbounded >= (1ll << 30)) return FC_EOVERFLOW;
        std::vector<ChainState> chain(1);
        ChainState &c = chain[0];
        rc = c.csr.build(st, grow_set, int32_t(unbounded));
        if (rc != FC_OK) return rc;
        // entries that are no link from inside the root-set to outside it are not sent at all
        std::vector<int64_t> slot(size_t(n_edges), -1);
        for (int64_t j = 0; j < n_edges; ++j) {
            const int32_t x = edge_x[j], y = edge_y[j];
            mu_out[j] = FC_GAMMA_INVALID;
            if (flows_or_null) flows_or_null[j] = FC_FLOW_INVALID;
            if (x < 0 || x >= n || y < 0 || y >= n) continue;
            const auto it = st.g.find(std::make_pair(x, y));
            if (it == st.g.end() || !st.inside[size_t(grow_set) * size_t(n) + size_t(x)] || st.inside[size_t(grow_set) * size_t(n) + size_t(y)]) continue;
            slot[size_t(j)] = int64_t(c.xs.size());
            c.xs.push_back(x); c.ys.push_back(y); c.cap_xy.push_back(it->second);
        }
        if (c.xs.empty()) return FC_OK;
        TreePool pool;
        std::vector<std::vector<int32_t>> flows;
        rc = tree_chain_launch(st, grow_set, chain, flows_or_null != nullptr, flows, reinterpret_cast<hipStream_t>(hip_stream), options_or_null, pool);
        if (rc != FC_OK) return rc;
        for (int64_t j = 0; j < n_edges; ++j) {
            if (slot[size_t(j)] < 0) continue;
            const size_t q = size_t(slot[size_t(j)]);
            const int32_t fl = flows[0][q];
            if (fl == FC_FLOW_NOCONVERGE) return FC_ENOCONVERGE;
            if (fl < 0) continue;
            // the root-sets that span already were left out of the network: their demands always arrive
            if (flows_or_null) flows_or_null[j] = int32_t(std::min<long long>((long long)fl + c.csr.spanning, (1ll << 31) - 1));
            mu_out[j] = int32_t(std::min<long long>(std::min<long long>(c.cap_xy[q], st.demand[size_t(grow_set)]), (long long)fl - c.csr.others));
        }
        return FC_OK;
    } catch (const std::bad_alloc &) {
        return FC_ENOMEM;
    }
}

extern "C" int fc_construct_trees(int32_t n_vertices, int64_t n_links, const int32_t *tail, const int32_t *head, const int32_t *capacity,
                                  int32_t k, int64_t tree_capacity, int64_t *n_trees, int32_t *tree_root, int32_t *tree_multiplicity,
                                  int32_t *tree_edge_x, int32_t *tree_edge_y, int64_t *n_batches_or_null,
                                  void *hip_stream, const fc_options *options_or_null) {
    if (n_vertices < 2 || k < 1 || !n_trees || tree_capacity < 0) return FC_EINVAL;
    hipStream_t stream = reinterpret_cast<hipStream_t>(hip_stream);
    constexpr size_t FC_TREE_CHAIN = 8;                  // states a launch looks ahead
    try {
        TreeState st;
        std::vector<int64_t> ptr(size_t(n_vertices) + 1, 0);
        std::vector<int32_t> mem(size_t(n_vertices), 0), dem(size_t(n_vertices), k);
        for (int32_t u = 0; u < n_vertices; ++u) { ptr[size_t(u) + 1] = u + 1; mem[size_t(u)] = u; }
        int rc = tree_state_from_arrays(n_vertices, n_links, tail, head, capacity, n_vertices, ptr.data(), mem.data(), dem.data(), &st);
        if (rc != FC_OK) return rc;
        const int32_t n = n_vertices;
        long long sum_g0 = 0;
        for (const auto &kv : st.g) sum_g0 += kv.second;
        const long long unbounded = sum_g0 + (long long)n * k + 1;      // above every finite cut of every state (capacities only shrink)
        if (unbounded >= (1ll << 30)) return FC_EOVERFLOW;
        std::vector<int32_t> root(size_t(n), 0);
        for (int32_t u = 0; u < n; ++u) root[size_t(u)] = u;
        std::vector<std::vector<std::pair<int32_t, int32_t>>> edges((size_t(n)));
        int64_t batches = 0;
        TreePool pool;
        TreeCsr cur;
        bool cur_valid = false;
        std::vector<ChainState> chain;
        std::vector<std::vector<int32_t>> flows;
        for (size_t i = 0; i < st.members.size(); ++i) {               // copies are appended while this runs
            std::set<std::pair<int32_t, int32_t>> rejected;            // edges that had mu = 0 for this root-set: guessed to stay so
            cur_valid = false;                                          // another root-set grows: another network
            while (int32_t(st.members[i].size()) < n) {
                if (!cur_valid) { rc = cur.build(st, int32_t(i), int32_t(unbounded)); if (rc != FC_OK) return rc; cur_valid = true; }
                const long long others = cur.others;
                // the chain: every state's candidates in (x, y) order; its guess is the first one not rejected before,
                // taken in full; the next state is this one after that edge
                chain.clear();
                std::vector<uint8_t> in_set(st.inside.begin() + long(i * size_t(n)), st.inside.begin() + long((i + 1) * size_t(n)));
                std::map<std::pair<int32_t, int32_t>, long long> used;  // capacity the chain's guesses have taken
                int32_t inside_count = int32_t(st.members[i].size());
                for (size_t j = 0; j < FC_TREE_CHAIN && inside_count < n; ++j) {
                    chain.emplace_back();
                    ChainState &c = chain.back();
                    c.csr = j == 0 ? cur : chain[j - 1].csr;
                    if (j > 0) {                                        // the grown set has no vertex in the network: only g changes
                        const ChainState &pc = chain[j - 1];
                        c.csr.lower(pc.xs[size_t(pc.guess)], pc.ys[size_t(pc.guess)], st.demand[i]);
                    }
                    for (const auto &kv : st.g) {
                        const auto u_it = used.find(kv.first);
                        const long long left = kv.second - (u_it == used.end() ? 0 : u_it->second);
                        if (left > 0 && in_set[size_t(kv.first.first)] && !in_set[size_t(kv.first.second)]) { c.xs.push_back(kv.first.first); c.ys.push_back(kv.first.second); c.cap_xy.push_back(left); }
                    }
                    if (c.xs.empty()) { if (j == 0) return FC_ENOCONVERGE; chain.pop_back(); break; }
                    for (size_t q = 0; q < c.xs.size(); ++q)
                        if (!rejected.count(std::make_pair(c.xs[q], c.ys[q]))) { c.guess = int32_t(q); break; }
                    if (c.guess < 0 || c.cap_xy[size_t(c.guess)] < st.demand[i]) { c.guess = -1; break; }   // no guess, or it would need a copy
                    used[std::make_pair(c.xs[size_t(c.guess)], c.ys[size_t(c.guess)])] += st.demand[i];
                    in_set[size_t(c.ys[size_t(c.guess)])] = 1; ++inside_count;
                }
                rc = tree_chain_launch(st, int32_t(i), chain, false, flows, stream, options_or_null, pool);
                ++batches;
                if (rc != FC_OK) return rc;
                // walk the chain: a state's result counts only while every guess before it was right
                for (size_t j = 0; j < chain.size() && int32_t(st.members[i].size()) < n; ++j) {
                    const ChainState &c = chain[j];
                    size_t hit = c.xs.size(); long long m = 0;
                    for (size_t q = 0; q < c.xs.size(); ++q) {
                        const int32_t fl = flows[j][q];
                        if (fl == FC_FLOW_NOCONVERGE || fl < 0) return FC_ENOCONVERGE;
                        const long long mu = std::min<long long>(std::min<long long>(c.cap_xy[q], st.demand[i]), (long long)fl - others);
                        if (mu < 0) return FC_ENOCONVERGE;              // the packing condition does not hold for this input
                        if (mu > 0) { hit = q; m = mu; break; }
                        rejected.insert(std::make_pair(c.xs[q], c.ys[q]));
                    }
                    if (hit == c.xs.size()) return FC_ENOCONVERGE;
                    const int32_t x = c.xs[hit], y = c.ys[hit];
                    const bool as_guessed = int32_t(hit) == c.guess && m == st.demand[i] && j + 1 < chain.size();
                    if (m < st.demand[i]) {                             // a copy keeps the rest of the multiplicity
                        st.members.push_back(st.members[i]); st.demand.push_back(st.demand[i] - m); root.push_back(root[i]);
                        edges.push_back(edges[i]);
                        st.inside.insert(st.inside.end(), st.inside.begin() + long(i * size_t(n)), st.inside.begin() + long((i + 1) * size_t(n)));
                        st.demand[i] = m;
                        cur_valid = false;                              // one more root-set vertex: the graph is built anew
                    }
                    edges[i].push_back(std::make_pair(x, y));
                    st.inside[i * size_t(n) + size_t(y)] = 1;
                    st.members[i].insert(std::upper_bound(st.members[i].begin(), st.members[i].end(), y), y);
                    auto it = st.g.find(std::make_pair(x, y));
                    it->second -= m;
                    if (it->second == 0) st.g.erase(it);
                    if (as_guessed) continue;                           // the next state of the chain is the true one
                    // the chain ends here: the current graph is this state's plus the edge that was really taken
                    if (cur_valid) { cur = c.csr; cur.lower(x, y, m); }
                    break;
                }
            }
        }
        *n_trees = int64_t(st.members.size());
        if (n_batches_or_null) *n_batches_or_null = batches;
        if (*n_trees > tree_capacity) return FC_EWORKSPACE;
        if (!tree_root || !tree_multiplicity || !tree_edge_x || !tree_edge_y) return FC_EINVAL;
        for (size_t i = 0; i < st.members.size(); ++i) {
            tree_root[i] = root[i]; tree_multiplicity[i] = int32_t(st.demand[i]);
            for (size_t q = 0; q < edges[i].size(); ++q) { tree_edge_x[i * size_t(n - 1) + q] = edges[i][q].first; tree_edge_y[i * size_t(n - 1) + q] = edges[i][q].second; }
        }
        return FC_OK;
    } catch (const std::bad_alloc &) {
        return FC_ENOMEM;
    }
}

extern "C" int fc_remove_switches(int32_t n_vertices, int64_t n_arcs, const int32_t *tail, const int32_t *head,
                                  const int32_t *capacity, const uint8_t *is_compute, int32_t k,
                                  int64_t out_capacity, int64_t *n_out, int32_t *out_tail, int32_t *out_head, int32_t *out_cap,
                                  int64_t route_capacity, int64_t *n_routes, int32_t *route_u, int32_t *route_t,
                                  int32_t *route_w, int32_t *route_amount, int64_t *n_batches_or_null,
                                  void *hip_stream, const fc_options *options_or_null) {
    if (n_vertices < 1 || n_arcs < 0 || k < 1 || !is_compute || !n_out || !n_routes || out_capacity < 0 || route_capacity < 0 ||
        (n_arcs > 0 && (!tail || !head || !capacity))) return FC_EINVAL;
    hipStream_t stream = reinterpret_cast<hipStream_t>(hip_stream);
    typedef std::pair<int32_t, int32_t> Key;
    try {
        std::map<Key, long long> cap;
        for (int64_t i = 0; i < n_arcs; ++i) {
            if (tail[i] < 0 || tail[i] >= n_vertices || head[i] < 0 || head[i] >= n_vertices || capacity[i] < 0) return FC_EINVAL;
            if (tail[i] != head[i] && capacity[i] > 0) cap[Key(tail[i], head[i])] += capacity[i];
        }
        {   // Theorems 9 and 10 are about Eulerian digraphs
            std::vector<long long> bal(size_t(n_vertices), 0);
            for (const auto &kv : cap) { bal[size_t(kv.first.first)] -= kv.second; bal[size_t(kv.first.second)] += kv.second; }
            for (long long b : bal) if (b != 0) return FC_EINVAL;
        }
        std::map<Key, std::map<int32_t, long long>> table;
        int64_t batches = 0;
        std::vector<int32_t> at, ah, ab, pu, pw, pt, gam;
        SplitPool pool;
        int dev = -1, lds_limit = 0, n_cu = 0;
        if (hipGetDevice(&dev) != hipSuccess || hipDeviceGetAttribute(&lds_limit, hipDeviceAttributeMaxSharedMemoryPerBlock, dev) != hipSuccess ||
            hipDeviceGetAttribute(&n_cu, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess) return FC_EDEVICE;
        auto cleanup = [&]() { (void)hipStreamSynchronize(stream); pool.release(); };
        for (int32_t w = 0; w < n_vertices; ++w) {
            if (is_compute[w]) continue;
            std::vector<int32_t> egress;
            for (auto it = cap.lower_bound(Key(w, 0)); it != cap.end() && it->first.first == w; ++it) egress.push_back(it->first.second);
            for (int32_t t : egress) {
                std::vector<int32_t> ingress;
                for (const auto &kv : cap) if (kv.first.second == w) ingress.push_back(kv.first.first);
                size_t pos = 0;
                while (pos < ingress.size() && cap.count(Key(w, t))) {
                    pu.clear(); pw.clear(); pt.clear();
                    std::vector<size_t> which;
                    for (size_t j = pos; j < ingress.size(); ++j)
                        if (cap.count(Key(ingress[j], w))) { pu.push_back(ingress[j]); pw.push_back(w); pt.push_back(t); which.push_back(j); }
                    if (pu.empty()) break;
                    at.clear(); ah.clear(); ab.clear();
                    for (const auto &kv : cap) {
                        if (kv.second >= (1ll << 31)) { cleanup(); return FC_EOVERFLOW; }
                        at.push_back(kv.first.first); ah.push_back(kv.first.second); ab.push_back(int32_t(kv.second));
                    }
                    // the split graph of this batch: residual CSR on the host, then one transfer into the pool
                    fc_graph *h = nullptr;
                    int rc = fc_host_build(n_vertices, int64_t(at.size()), at.data(), ah.data(), ab.data(), is_compute, &h);
                    if (rc != FC_OK) { cleanup(); return rc; }
                    const size_t np = pu.size(), M = size_t(2 * h->m0);
                    rc = pool.ensure(h, M, np, stream);
                    if (rc != FC_OK) { fc_graph_free(h); cleanup(); return rc; }
                    std::memcpy(pool.h_blob + pool.off_row, h->row_ptr.data(), sizeof(int32_t) * (size_t(h->n) + 1));
                    std::memcpy(pool.h_blob + pool.off_inbw, h->in_bw.data(), sizeof(int32_t) * size_t(h->n));
                    int32_t *hp = reinterpret_cast<int32_t *>(pool.h_blob + pool.off_pairs);
                    std::memcpy(hp, pu.data(), sizeof(int32_t) * np);
                    std::memcpy(hp + pool.pair_cap, pw.data(), sizeof(int32_t) * np);
                    std::memcpy(hp + 2 * pool.pair_cap, pt.data(), sizeof(int32_t) * np);
                    fill_wide_records(h, reinterpret_cast<int4 *>(pool.h_blob + pool.off_wide));
                    h->on_device = true; h->device = dev; h->lds_limit = lds_limit; h->n_cu = n_cu;
                    h->d_row_ptr = reinterpret_cast<int32_t *>(pool.d_blob + pool.off_row);
                    h->d_in_bw = reinterpret_cast<int32_t *>(pool.d_blob + pool.off_inbw);
                    h->d_arc_wide = pool.d_blob + pool.off_wide;
                    h->d_is_compute = pool.d_blob + pool.off_is;
                    h->d_compute_ids = reinterpret_cast<int32_t *>(pool.d_blob + pool.off_ids);
                    h->d_sink_cost = reinterpret_cast<uint32_t *>(pool.d_blob + pool.off_cost);
                    int32_t *d_pairs = reinterpret_cast<int32_t *>(pool.d_blob + pool.off_pairs);
                    int32_t *d_gamma = reinterpret_cast<int32_t *>(pool.d_blob + pool.off_gamma);
                    int32_t *h_gamma = reinterpret_cast<int32_t *>(pool.h_blob + pool.off_gamma);
                    bool ok = hipMemcpyAsync(pool.d_blob, pool.h_blob, pool.off_wide + sizeof(int4) * M, hipMemcpyHostToDevice, stream) == hipSuccess;
                    if (ok) {
                        rc = split_gamma_impl(h, 1, k, int64_t(np), d_pairs, d_pairs + pool.pair_cap, d_pairs + 2 * pool.pair_cap, d_gamma, nullptr,
                                              pool.d_blob + pool.off_ws, pool.ws_bytes, stream, options_or_null, nullptr, d_gamma + pool.pair_cap);
                        ok = rc == FC_OK && hipMemcpyAsync(h_gamma, d_gamma, sizeof(int32_t) * (pool.pair_cap + np), hipMemcpyDeviceToHost, stream) == hipSuccess &&
                             hipStreamSynchronize(stream) == hipSuccess;
                    }
                    // the pool owns the device memory: detach it before the host graph goes
                    h->on_device = false;
                    h->d_row_ptr = nullptr; h->d_in_bw = nullptr; h->d_arc_wide = nullptr; h->d_is_compute = nullptr; h->d_compute_ids = nullptr; h->d_sink_cost = nullptr;
                    fc_graph_free(h);
                    ++batches;
                    if (!ok) { cleanup(); return rc != FC_OK ? rc : FC_EDEVICE; }
                    gam.assign(h_gamma, h_gamma + np);
                    const int32_t *slk = h_gamma + pool.pair_cap;
                    // Walk the ingress links in order.  Until a split is applied every gamma is exact for the current graph
                    // (zeros are skipped).  After splits of total amount `applied`, a later pair need not be evaluated again
                    // when its flows cannot have become binding: no cut holds both e and f, so a split of gamma lowers any
                    // max-flow by at most gamma, and if slack - applied >= min{c(e), c(f) now} that minimum is its gamma.
                    long long applied = 0;
                    size_t q = 0;
                    for (; q < which.size(); ++q) {
                        const auto f_it = cap.find(Key(w, t));
                        if (f_it == cap.end()) break;                        // f is used up
                        const int32_t u = pu[q];
                        long long gmm;
                        if (applied == 0) {
                            if (gam[q] < 0) { cleanup(); return FC_ENOCONVERGE; }     // invalid, or min_v F(s, v) >= N k does not hold in D
                            if (gam[q] == 0) continue;
                            gmm = gam[q];
                        } else {
                            const long long m = std::min<long long>(cap.at(Key(u, w)), f_it->second);
                            if (gam[q] > 0 && (long long)slk[q] - applied >= m) gmm = m;
                            else break;                                      // this one has to be evaluated on the current graph
                        }
                        auto take = [&](Key key) { auto it = cap.find(key); it->second -= gmm; if (it->second == 0) cap.erase(it); };
                        take(Key(u, w)); take(Key(w, t));
                        if (u != t) { cap[Key(u, t)] += gmm; table[Key(u, t)][w] += gmm; }   // a detour u -> w -> u just disappears
                        applied += gmm;
                    }
                    if (applied == 0) break;                                 // no ingress link can give anything to f
                    pos = q < which.size() ? which[q] : ingress.size();
                }
                if (cap.count(Key(w, t))) { cleanup(); return FC_ENOCONVERGE; }   // Theorem 9 promises f can be used up: the input broke its conditions
            }
        }
        cleanup();
        int64_t nr = 0;
        for (const auto &kv : table) nr += int64_t(kv.second.size());
        *n_out = int64_t(cap.size()); *n_routes = nr;
        if (n_batches_or_null) *n_batches_or_null = batches;
        if (int64_t(cap.size()) > out_capacity || nr > route_capacity) return FC_EWORKSPACE;    // sizes are set: call again with room
        int64_t i = 0;
        for (const auto &kv : cap) {
            if (kv.second >= (1ll << 31)) return FC_EOVERFLOW;
            out_tail[i] = kv.first.first; out_head[i] = kv.first.second; out_cap[i] = int32_t(kv.second); ++i;
        }
        i = 0;
        for (const auto &kv : table)
            for (const auto &rw : kv.second) { route_u[i] = kv.first.first; route_t[i] = kv.first.second; route_w[i] = rw.first; route_amount[i] = int32_t(rw.second); ++i; }
        return FC_OK;
    } catch (const std::bad_alloc &) {
        return FC_ENOMEM;
    }
}
