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
// max-flows with an explicit source and unbounded arcs that edge splitting needs (Appendix E.2, the
// theorem that gives the maximum capacity that can be split off).  The source is split over the included files below; they form one translation unit.
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

#include "fc_solver_kernels.inc"   // device code
#include "fc_launch.inc"           // option defaults, kernel build selection, launches
#include "fc_api.inc"              // C ABI: graphs, batches, verdicts, searches, edge-splitting batches
#include "fc_surgery.inc"          // C ABI: spanning tree construction, switch removal
