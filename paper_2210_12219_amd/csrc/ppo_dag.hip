// From a model's layer graph to the chain the search works on (paper Sec. III-A): host code, no GPU work.
//
// Topological depth LP(v) = length of the longest path from the source to v (relaxation in topological
// order).  A vertex u is the next candidate partition point after p iff no other vertex has its depth and
// every path leaving p reaches u before it reaches a vertex deeper than u.  The chain's layer i is what lies
// after partition point i-1 up to and including partition point i; what lies after the last point is a last
// layer of its own.
#include <cstdint>
#include <vector>

#include "ppo.h"

namespace {

struct Graph {
    int V = 0;
    std::vector<int> first, adj;   // successors of v: adj[first[v] .. first[v+1])
};

}  // namespace

extern "C" int ppo_chain_from_dag(int n_vertices, int n_edges, const int32_t* edge_src, const int32_t* edge_dst,
                                  const float* weight, const float* out_size, int max_layers, float* t, float* m,
                                  int32_t* point, int32_t* n_layers) {
    if (n_vertices < 1 || n_edges < 0 || max_layers < 1) return PPO_EINVAL;
    if (!weight || !out_size || !t || !m || !point || !n_layers || (n_edges > 0 && (!edge_src || !edge_dst))) return PPO_EINVAL;
    const int V = n_vertices;
    Graph g;
    g.V = V;
    g.first.assign(V + 1, 0);
    std::vector<int> indeg(V, 0);
    for (int e = 0; e < n_edges; ++e) {
        const int a = edge_src[e], b = edge_dst[e];
        if (a < 0 || a >= V || b < 0 || b >= V || a == b) return PPO_EINVAL;
        ++g.first[a + 1];
        ++indeg[b];
    }
    for (int v = 0; v < V; ++v) g.first[v + 1] += g.first[v];
    g.adj.resize(n_edges);
    {
        std::vector<int> fill(g.first.begin(), g.first.end() - 1);
        for (int e = 0; e < n_edges; ++e) g.adj[fill[edge_src[e]]++] = edge_dst[e];
    }
    // one source; topological order (Kahn); depth by relaxing the successors of each vertex in that order
    int source = -1;
    for (int v = 0; v < V; ++v)
        if (indeg[v] == 0) {
            if (source >= 0) return PPO_EINVAL;
            source = v;
        }
    if (source < 0) return PPO_EINVAL;
    std::vector<int> order, depth(V, 0), left(indeg);
    order.reserve(V);
    order.push_back(source);
    for (size_t head = 0; head < order.size(); ++head) {
        const int v = order[head];
        for (int e = g.first[v]; e < g.first[v + 1]; ++e) {
            const int u = g.adj[e];
            if (depth[v] + 1 > depth[u]) depth[u] = depth[v] + 1;
            if (--left[u] == 0) order.push_back(u);
        }
    }
    if ((int)order.size() != V) return PPO_EINVAL;   // a cycle
    int deepest = 0;
    for (int v = 0; v < V; ++v) deepest = depth[v] > deepest ? depth[v] : deepest;
    std::vector<int> at_depth(deepest + 1, 0), vertex_at(deepest + 1, -1);
    for (int v = 0; v < V; ++v) {
        ++at_depth[depth[v]];
        vertex_at[depth[v]] = v;
    }
    // partition points in order of depth
    // Every path that leaves the last point p must reach the candidate u (alone at depth d) before a deeper
    // vertex, and a path that ends does not reach it.  An edge leads to a strictly deeper vertex, and every
    // vertex deeper than p is reached from p (all paths from the source pass p first).  So u qualifies iff no
    // vertex of depth in [depth(p), d) is a dead end or has a successor deeper than d: one running maximum of
    // "deepest successor" over the depth levels since p, no recursion, linear in the size of the graph.
    constexpr int kDeadEnd = 0x7FFFFFFF;
    std::vector<int> reach_of_level(deepest + 1, 0);
    for (int v = 0; v < V; ++v) {
        int far = g.first[v + 1] > g.first[v] ? 0 : kDeadEnd;
        for (int e = g.first[v]; e < g.first[v + 1]; ++e) far = depth[g.adj[e]] > far ? depth[g.adj[e]] : far;
        if (far > reach_of_level[depth[v]]) reach_of_level[depth[v]] = far;
    }
    std::vector<int> points{source};
    int reach = reach_of_level[0];   // deepest successor of the levels from the last point's to d - 1
    for (int d = 1; d <= deepest; ++d) {
        if (at_depth[d] == 1 && reach <= d) {
            points.push_back(vertex_at[d]);
            reach = 0;
        }
        if (reach_of_level[d] > reach) reach = reach_of_level[d];
    }
    const bool tail = depth[points.back()] < deepest;
    const int L = (int)points.size() + (tail ? 1 : 0);
    *n_layers = L;
    if (L > max_layers) return PPO_ENOSPC;
    // layer of a vertex: the first partition point at its depth or deeper (the tail after the last one)
    std::vector<int> layer_of_depth(deepest + 1);
    for (int d = 0, i = 0; d <= deepest; ++d) {
        while (i < (int)points.size() && depth[points[i]] < d) ++i;
        layer_of_depth[d] = i;
    }
    std::vector<double> sum(L, 0.0);
    for (int v = 0; v < V; ++v) sum[layer_of_depth[depth[v]]] += (double)weight[v];
    for (int i = 0; i < L; ++i) {
        m[i] = (float)sum[i];
        const bool is_point = i < (int)points.size();
        t[i] = is_point ? out_size[points[i]] : 0.0f;
        point[i] = is_point ? points[i] : -1;
    }
    return PPO_OK;
}
