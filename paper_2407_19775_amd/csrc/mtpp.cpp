// Max-throughput slicing of a topological order (include/mtpp.h): host code, no GPU.
//
// All segment costs f(order[l..r]) are set up row by row (fixed l, growing r) with running sums: the work and
// the parameters are prefix sums, peak is a running maximum of per-operation working sets, the incoming
// tensors are added when their first consumer enters the segment (a stamp per producer), and the outgoing
// tensors are those whose last consumer lies beyond r (an operation enters the sum with the segment's end and
// leaves it at the position of its last consumer).  The dynamic programme then minimises the largest cost.
#include "../../include/mtpp.h"

#include <algorithm>
#include <limits>
#include <queue>
#include <vector>

namespace {

struct Graph {
  int n;
  std::vector<std::vector<int>> pred, succ;
};

bool build(int n, int m, const int32_t* from, const int32_t* to, Graph& g) {
  if (n < 1 || m < 0 || (m > 0 && (!from || !to))) return false;
  g.n = n;
  g.pred.assign(n, {});
  g.succ.assign(n, {});
  for (int e = 0; e < m; ++e) {
    if (from[e] < 0 || from[e] >= n || to[e] < 0 || to[e] >= n) return false;
    g.succ[from[e]].push_back(to[e]);
    g.pred[to[e]].push_back(from[e]);
  }
  for (auto& p : g.pred) {   // a producer counts once per consumer
    std::sort(p.begin(), p.end());
    p.erase(std::unique(p.begin(), p.end()), p.end());
  }
  return true;
}

bool kahn(const Graph& g, std::vector<int>& order) {
  std::vector<int> indeg(g.n, 0);
  for (int u = 0; u < g.n; ++u)
    for (int v : g.succ[u]) ++indeg[v];
  std::priority_queue<int, std::vector<int>, std::greater<int>> ready;
  for (int v = 0; v < g.n; ++v)
    if (indeg[v] == 0) ready.push(v);
  order.clear();
  while (!ready.empty()) {
    const int v = ready.top();
    ready.pop();
    order.push_back(v);
    for (int w : g.succ[v])
      if (--indeg[w] == 0) ready.push(w);
  }
  return (int)order.size() == g.n;
}

// positions of the operations in the order; false if it is not a permutation that respects every edge
bool positions(const Graph& g, const int32_t* order, std::vector<int>& pos) {
  pos.assign(g.n, -1);
  for (int i = 0; i < g.n; ++i) {
    if (order[i] < 0 || order[i] >= g.n || pos[order[i]] != -1) return false;
    pos[order[i]] = i;
  }
  for (int u = 0; u < g.n; ++u)
    for (int v : g.succ[u])
      if (pos[u] >= pos[v]) return false;
  return true;
}

// cost[l][r - l] = f(order[l..r]) for every 0 <= l <= r < n
void segment_costs(const Graph& g, const int32_t* order, const std::vector<int>& pos, const double* work,
                   const double* sizeparam, const double* sizeout, double B, double M,
                   std::vector<std::vector<double>>& cost) {
  const int n = g.n;
  std::vector<double> ws(n);            // working set of the operation at a position
  std::vector<int> last_use(n, -1);     // position of the last consumer of the operation at a position
  std::vector<std::vector<int>> ends_at(n);   // positions whose last consumer sits at this position
  for (int i = 0; i < n; ++i) {
    const int v = order[i];
    double s = sizeout[v];
    for (int u : g.pred[v]) s += sizeout[u];
    ws[i] = s;
    for (int w : g.succ[v]) last_use[i] = std::max(last_use[i], pos[w]);
    if (last_use[i] >= 0) ends_at[last_use[i]].push_back(i);
  }
  std::vector<int> stamp(n, -1);
  cost.assign(n, {});
  for (int l = 0; l < n; ++l) {
    cost[l].resize(n - l);
    double w_sum = 0, p_sum = 0, peak = 0, in_sum = 0, out_sum = 0;
    for (int r = l; r < n; ++r) {
      const int v = order[r];
      w_sum += work[v];
      p_sum += sizeparam[v];
      peak = std::max(peak, ws[r]);
      for (int u : g.pred[v])
        if (pos[u] < l && stamp[u] != l) {
          stamp[u] = l;
          in_sum += sizeout[u];
        }
      for (int i : ends_at[r])           // their last consumer is now inside
        if (i >= l) out_sum -= sizeout[order[i]];
      if (last_use[r] > r) out_sum += sizeout[v];
      const double overflow = std::max(0.0, p_sum + peak - M) / B + peak / B;
      cost[l][r - l] = in_sum / B + w_sum + overflow + out_sum / B;
    }
  }
}

}  // namespace

extern "C" {

int mtpp_kahn_order(int n, int m, const int32_t* edge_from, const int32_t* edge_to, int32_t* order_out) {
  Graph g;
  if (!order_out || !build(n, m, edge_from, edge_to, g)) return MTPP_E_ARG;
  std::vector<int> order;
  if (!kahn(g, order)) return MTPP_E_CYCLE;
  std::copy(order.begin(), order.end(), order_out);
  return MTPP_OK;
}

int mtpp_block_cost(int n, int m, const int32_t* edge_from, const int32_t* edge_to, const double* work,
                    const double* sizeparam, const double* sizeout, const int32_t* order, int first, int last,
                    double B, double M, double* cost_out) {
  Graph g;
  if (!work || !sizeparam || !sizeout || !order || !cost_out || !(B > 0) || !build(n, m, edge_from, edge_to, g))
    return MTPP_E_ARG;
  if (first < 0 || last < first || last >= n) return MTPP_E_ARG;
  std::vector<int> pos;
  if (!positions(g, order, pos)) return MTPP_E_CYCLE;
  // written out for the one block, not taken from the table of all segments
  std::vector<char> in_block(n, 0), counted(n, 0);
  for (int i = first; i <= last; ++i) in_block[order[i]] = 1;
  double w_sum = 0, p_sum = 0, peak = 0, in_sum = 0, out_sum = 0;
  for (int i = first; i <= last; ++i) {
    const int v = order[i];
    w_sum += work[v];
    p_sum += sizeparam[v];
    double s = sizeout[v];
    for (int u : g.pred[v]) {
      s += sizeout[u];
      if (!in_block[u] && !counted[u]) {
        counted[u] = 1;
        in_sum += sizeout[u];
      }
    }
    peak = std::max(peak, s);
    bool leaves = false;
    for (int w : g.succ[v]) leaves = leaves || !in_block[w];
    if (leaves) out_sum += sizeout[v];
  }
  *cost_out = in_sum / B + w_sum + (std::max(0.0, p_sum + peak - M) / B + peak / B) + out_sum / B;
  return MTPP_OK;
}

int mtpp_slice_order(int n, int m, const int32_t* edge_from, const int32_t* edge_to, const double* work,
                     const double* sizeparam, const double* sizeout, const int32_t* order, int k, double B, double M,
                     double* bottleneck_out, int32_t* n_blocks_out, int32_t* block_end_out) {
  Graph g;
  if (!work || !sizeparam || !sizeout || !bottleneck_out || !n_blocks_out || !block_end_out || !(B > 0) || k < 1 ||
      n > MTPP_MAX_N || !build(n, m, edge_from, edge_to, g))
    return MTPP_E_ARG;
  std::vector<int> own;
  if (!order) {
    if (!kahn(g, own)) return MTPP_E_CYCLE;
    order = own.data();
  }
  std::vector<int> pos;
  if (!positions(g, order, pos)) return MTPP_E_CYCLE;
  std::vector<std::vector<double>> cost;
  segment_costs(g, order, pos, work, sizeparam, sizeout, B, M, cost);

  // best[j][r]: smallest bottleneck of the first r operations in exactly j blocks; cut[j][r]: start of the last one
  const int kk = std::min(k, n);
  const double inf = std::numeric_limits<double>::infinity();
  std::vector<std::vector<double>> best(kk + 1, std::vector<double>(n + 1, inf));
  std::vector<std::vector<int>> cut(kk + 1, std::vector<int>(n + 1, 0));
  for (int r = 1; r <= n; ++r) best[1][r] = cost[0][r - 1];
  for (int j = 2; j <= kk; ++j)
    for (int r = j; r <= n; ++r)
      for (int l = j - 1; l < r; ++l) {        // the last block is order[l .. r-1]; smallest l wins ties
        const double c = std::max(best[j - 1][l], cost[l][r - 1 - l]);
        if (c < best[j][r]) {
          best[j][r] = c;
          cut[j][r] = l;
        }
      }
  int blocks = 1;
  for (int j = 2; j <= kk; ++j)
    if (best[j][n] < best[blocks][n]) blocks = j;   // ties go to fewer blocks
  *bottleneck_out = best[blocks][n];
  *n_blocks_out = blocks;
  int r = n;
  for (int j = blocks; j >= 1; --j) {
    block_end_out[j - 1] = r;
    r = (j > 1) ? cut[j][r] : 0;
  }
  return MTPP_OK;
}

}  // extern "C"
