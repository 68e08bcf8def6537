// Sharding planner (Section V-B): picks the device meshes over which P, G and OS are sharded by
// minimising the per-step communication time under the GPU memory limit.  Host only.
//
// Search: instead of every tuple in [1..R] x [1..N] per component, only what the two pre-filters
// of Section V-B leave: intra-node factors that divide s_dp^0 = R, inter-node factors that divide
// s_dp^1 = N (Eq. 5, 6), and inter-node factors above 1 only together with the full node (Eq. 7):
// each component's mesh is one of (d, 1) with d | R, or (R, e) with e | N, e > 1.  The chains
// s_p <= s_g <= s_os per dimension (Eq. 3, 4) and s_g in {s_p, s_os} (Section IV-C.3) then leave
// a few dozen candidates, each priced with the formulas of Section IV-C / IV-D.
#include <math.h>
#include <stdint.h>
#include <stdlib.h>

#include <algorithm>
#include <vector>

#include "amsp.h"

namespace {

struct Mesh {
    uint32_t a, b;   // GPUs per node x nodes
};

// Effective bandwidth of `op` at message size v on mesh (p0, p1): linear in v between the profiled
// sizes, the end values outside them; < 0 if that mesh was not profiled for that operation.
double bandwidth(const amsp_bw_sample *table, uint32_t rows, uint32_t op, double v, uint32_t p0, uint32_t p1) {
    std::vector<std::pair<double, double>> pts;
    for (uint32_t i = 0; i < rows; ++i)
        if (table[i].op == op && table[i].p0 == p0 && table[i].p1 == p1) pts.emplace_back(table[i].bytes, table[i].bytes_per_s);
    if (pts.empty()) return -1.0;
    std::sort(pts.begin(), pts.end());
    if (v <= pts.front().first) return pts.front().second;
    if (v >= pts.back().first) return pts.back().second;
    for (size_t i = 0; i + 1 < pts.size(); ++i) {
        if (v >= pts[i].first && v <= pts[i + 1].first) {
            const double span = pts[i + 1].first - pts[i].first;
            if (span == 0.0) return pts[i].second;
            return pts[i].second + (pts[i + 1].second - pts[i].second) * (v - pts[i].first) / span;
        }
    }
    return pts.back().second;
}

// t(o, v, mesh) = v / w; a one-GPU mesh costs nothing; < 0 if it cannot be priced.
double coll_time(const amsp_bw_sample *table, uint32_t rows, uint32_t op, double v, uint32_t p0, uint32_t p1) {
    if ((uint64_t)p0 * p1 == 1) return 0.0;
    const double w = bandwidth(table, rows, op, v, p0, p1);
    return w > 0.0 ? v / w : -1.0;
}

std::vector<Mesh> meshes(uint32_t R, uint32_t N) {
    std::vector<Mesh> out;
    for (uint32_t d = 1; d <= R; ++d)
        if (R % d == 0) out.push_back(Mesh{d, 1});
    for (uint32_t e = 2; e <= N; ++e)
        if (N % e == 0) out.push_back(Mesh{R, e});
    return out;   // ordered by (a, b) lexicographically, as the plain search would meet them
}

bool lex_less(const amsp_plan &x, const amsp_plan &y) {
    const uint32_t a[6] = {x.sp0, x.sp1, x.sg0, x.sg1, x.sos0, x.sos1};
    const uint32_t b[6] = {y.sp0, y.sp1, y.sg0, y.sg1, y.sos0, y.sos1};
    return std::lexicographical_compare(a, a + 6, b, b + 6);
}

}  // namespace

static int plan_sharding(const amsp_plan_problem *pb, const amsp_bw_sample *table, uint32_t rows, amsp_plan *best,
                         uint32_t *feasible_count) {
    if (pb == nullptr || best == nullptr) return AMSP_ENULL;
    if (rows > 0 && table == nullptr) return AMSP_ENULL;
    if (pb->modules_per_layer > 0 && pb->module_params == nullptr) return AMSP_ENULL;
    if (pb->gpus_per_node == 0 || pb->nodes == 0 || pb->micro_batches == 0 || !(pb->phi > 0.0) ||
        !(pb->bucket_bytes > 0.0))
        return AMSP_EINVAL;
    const uint32_t R = pb->gpus_per_node, N = pb->nodes, M = pb->micro_batches;
    const double phi = pb->phi, U = pb->bucket_bytes;
    const std::vector<Mesh> ms = meshes(R, N);
    bool found = false;
    uint32_t count = 0;
    amsp_plan cur;
    for (const Mesh &p : ms)
        for (const Mesh &g : ms)
            for (const Mesh &o : ms) {
                if (!(p.a <= g.a && g.a <= o.a && p.b <= g.b && g.b <= o.b)) continue;            // Eq. 3, 4
                const bool g_is_p = g.a == p.a && g.b == p.b, g_is_o = g.a == o.a && g.b == o.b;
                if (!g_is_p && !g_is_o) continue;                                                  // s_g in {s_p, s_os}
                const double sp = (double)p.a * p.b, sg = (double)g.a * g.b, so = (double)o.a * o.b;
                const double d_ms = 2.0 * phi / sp + 2.0 * phi / sg + 12.0 * phi / so;
                if (d_ms + pb->activation_bytes + pb->tmp_bytes > pb->gpu_memory_bytes) continue;  // Eq. 2
                bool priced = true;
                double t_p = 0.0;
                for (uint32_t i = 0; i < pb->modules_per_layer && priced; ++i) {
                    const double v = 2.0 * pb->module_params[i];
                    const double ag = coll_time(table, rows, AMSP_OP_ALLGATHER, v, p.a, p.b);
                    const double rs = coll_time(table, rows, AMSP_OP_REDUCESCATTER, v, p.a, p.b);
                    if (ag < 0.0 || rs < 0.0) priced = false;
                    else t_p += 2.0 * ag + rs;
                }
                t_p *= (double)M * pb->layers;
                const double ar_os = coll_time(table, rows, AMSP_OP_ALLREDUCE, U, R / p.a, N / p.b);
                const double bc = coll_time(table, rows, AMSP_OP_BROADCAST, 2.0 * phi / so, o.a / p.a, o.b / p.b);
                const double ar_g = coll_time(table, rows, AMSP_OP_ALLREDUCE, U, g.a / p.a, g.b / p.b);
                if (!priced || ar_os < 0.0 || bc < 0.0 || ar_g < 0.0) continue;
                cur.sp0 = p.a; cur.sp1 = p.b; cur.sg0 = g.a; cur.sg1 = g.b; cur.sos0 = o.a; cur.sos1 = o.b;
                cur.t_p = t_p;
                cur.t_os0 = 2.0 * phi / (U * sp) * ar_os;
                cur.t_os1 = so / sp * bc;
                cur.t_g = (double)(M - 1) * 2.0 * phi / (U * sp) * ar_g;
                cur.t_comm = cur.t_p + cur.t_g + cur.t_os0 + cur.t_os1;
                cur.d_modelstate = d_ms;
                ++count;
                // smallest time; on a tie the tuple that comes first lexicographically
                if (!found || cur.t_comm < best->t_comm || (cur.t_comm == best->t_comm && lex_less(cur, *best))) {
                    *best = cur;
                    found = true;
                }
            }
    if (feasible_count != nullptr) *feasible_count = count;
    return found ? AMSP_OK : AMSP_ENOPLAN;
}

// Nothing may leave through the C boundary: running out of host memory for the (small) working lists is
// reported as "no plan".
extern "C" int amsp_plan_sharding(const amsp_plan_problem *pb, const amsp_bw_sample *table, uint32_t rows,
                                  amsp_plan *best, uint32_t *feasible_count) {
    try {
        return plan_sharding(pb, table, rows, best, feasible_count);
    } catch (...) {
        return AMSP_ENOPLAN;
    }
}
