// Maximum-weight matching in general graphs: exact subset recursion and the
// blossom algorithm (Edmonds' method for weighted general matching in its
// O(V^3) primal-dual formulation).
#include "matching.hpp"

#include <algorithm>
#include <deque>

namespace sar {

// ---- exact recursion over subsets ---------------------------------------------
// best[mask]: weight of the heaviest matching inside `mask`.  The lowest vertex i
// of the mask stays unmatched (first option) or pairs with a higher vertex j of
// the mask (ascending j); a later option replaces an earlier one only if strictly
// heavier.  Masks are visited in increasing order, so sub-results are ready.
int64_t max_weight_matching_subsets(int k, const std::vector<int64_t>& weight, std::vector<int>& mate) {
    const uint32_t nmasks = 1u << k;
    std::vector<int64_t> best(nmasks, 0);
    std::vector<int8_t> choice(nmasks, -1);
    for (uint32_t mask = 1; mask < nmasks; ++mask) {
        const int i = __builtin_ctz(mask);
        const uint32_t rest = mask & (mask - 1);
        int64_t b = best[rest];
        int8_t pick = -1;
        for (uint32_t m = rest; m; m &= m - 1) {
            const int j = __builtin_ctz(m);
            const int64_t w = weight[size_t(i) * k + j];
            if (w == 0) continue;
            const int64_t cand = w + best[rest & ~(1u << j)];
            if (cand > b) {
                b = cand;
                pick = int8_t(j);
            }
        }
        best[mask] = b;
        choice[mask] = pick;
    }
    mate.assign(k, -1);
    for (uint32_t mask = nmasks - 1; mask;) {
        const int i = __builtin_ctz(mask);
        const int j = choice[mask];
        mask &= mask - 1;
        if (j < 0) continue;
        mask &= ~(1u << j);
        mate[i] = j;
        mate[j] = i;
    }
    return k ? best[nmasks - 1] : 0;
}

// ---- blossom algorithm ------------------------------------------------------------
// Vertices 1..n; blossoms take ids n+1..2n.  Dual variables `dual` are kept at
// twice their value so that every adjustment stays integral.  An edge is tight
// when slack(e) = dual[u] + dual[v] - 2 w(e) is zero.  A phase grows alternating
// trees from every free vertex (label 0 = even / outer, 1 = odd / inner), shrinks
// odd cycles into blossoms, adjusts duals when no tight edge is left, expands
// inner blossoms whose dual reaches zero, and ends with an augmentation or when a
// free vertex's dual reaches zero (then no augmenting path can gain weight).
namespace {

class Blossom {
public:
    Blossom(int n, const std::vector<int64_t>& weight) : n_(n), top_(n) {
        const int cap = 2 * n + 1;
        edge_.assign(cap, std::vector<Edge>(cap));
        for (int u = 0; u < cap; ++u)
            for (int v = 0; v < cap; ++v) edge_[u][v] = Edge{u, v, 0};
        for (int a = 0; a < n; ++a)
            for (int b = 0; b < n; ++b)
                if (a != b) edge_[a + 1][b + 1].w = weight[size_t(a) * n + b];
        dual_.assign(cap, 0);
        mate_.assign(cap, 0);
        slack_from_.assign(cap, 0);
        surface_.assign(cap, 0);
        parent_.assign(cap, 0);
        label_.assign(cap, -1);
        stamp_.assign(cap, 0);
        member_of_.assign(cap, std::vector<int>(n + 1, 0));
        cycle_.assign(cap, {});
    }

    void solve(std::vector<int>& mate) {
        int64_t heaviest = 0;
        for (int u = 1; u <= n_; ++u) {
            surface_[u] = u;
            for (int v = 1; v <= n_; ++v) {
                member_of_[u][v] = u == v ? u : 0;
                heaviest = std::max(heaviest, edge_[u][v].w);
            }
        }
        for (int u = 1; u <= n_; ++u) dual_[u] = heaviest;
        while (phase()) {
        }
        mate.assign(n_, -1);
        for (int u = 1; u <= n_; ++u)
            if (mate_[u]) mate[u - 1] = mate_[u] - 1;
    }

private:
    struct Edge {
        int u, v;
        int64_t w;
    };

    int64_t slack(const Edge& e) const { return dual_[e.u] + dual_[e.v] - 2 * edge_[e.u][e.v].w; }

    // remember, per surface node x, the outer vertex with the tightest edge into it
    void offer_slack(int u, int x) {
        if (!slack_from_[x] || slack(edge_[u][x]) < slack(edge_[slack_from_[x]][x])) slack_from_[x] = u;
    }

    void recompute_slack(int x) {
        slack_from_[x] = 0;
        for (int u = 1; u <= n_; ++u)
            if (edge_[u][x].w > 0 && surface_[u] != x && label_[surface_[u]] == 0) offer_slack(u, x);
    }

    void enqueue(int x) {
        if (x <= n_) {
            queue_.push_back(x);
            return;
        }
        for (int sub : cycle_[x]) enqueue(sub);
    }

    void set_surface(int x, int b) {
        surface_[x] = b;
        if (x > n_)
            for (int sub : cycle_[x]) set_surface(sub, b);
    }

    // position of sub-blossom `sub` in b's cycle, with the cycle oriented so that
    // the position is even (an even-length alternating path leads back to the base)
    int even_position(int b, int sub) {
        std::vector<int>& c = cycle_[b];
        const int pos = int(std::find(c.begin(), c.end(), sub) - c.begin());
        if (pos % 2 == 1) {
            std::reverse(c.begin() + 1, c.end());
            return int(c.size()) - pos;
        }
        return pos;
    }

    void set_mate(int u, int v) {
        mate_[u] = edge_[u][v].v;
        if (u <= n_) return;
        const Edge e = edge_[u][v];
        const int sub = member_of_[u][e.u];
        const int pos = even_position(u, sub);
        std::vector<int>& c = cycle_[u];
        for (int i = 0; i < pos; ++i) set_mate(c[i], c[i ^ 1]);
        set_mate(sub, v);
        std::rotate(c.begin(), c.begin() + pos, c.end());
    }

    void augment(int u, int v) {
        for (;;) {
            const int next = surface_[mate_[u]];
            set_mate(u, v);
            if (!next) return;
            set_mate(next, surface_[parent_[next]]);
            u = surface_[parent_[next]];
            v = next;
        }
    }

    int common_ancestor(int u, int v) {
        for (++clock_; u || v; std::swap(u, v)) {
            if (!u) continue;
            if (stamp_[u] == clock_) return u;
            stamp_[u] = clock_;
            u = surface_[mate_[u]];
            if (u) u = surface_[parent_[u]];
        }
        return 0;
    }

    void shrink(int u, int base, int v) {
        int b = n_ + 1;
        while (b <= top_ && surface_[b]) ++b;
        if (b > top_) ++top_;
        dual_[b] = 0;
        label_[b] = 0;
        mate_[b] = mate_[base];
        std::vector<int>& c = cycle_[b];
        c.clear();
        c.push_back(base);
        for (int x = u, y; x != base; x = surface_[parent_[y]]) {
            c.push_back(x);
            c.push_back(y = surface_[mate_[x]]);
            enqueue(y);
        }
        std::reverse(c.begin() + 1, c.end());
        for (int x = v, y; x != base; x = surface_[parent_[y]]) {
            c.push_back(x);
            c.push_back(y = surface_[mate_[x]]);
            enqueue(y);
        }
        set_surface(b, b);
        for (int x = 1; x <= top_; ++x) edge_[b][x].w = edge_[x][b].w = 0;
        for (int x = 1; x <= n_; ++x) member_of_[b][x] = 0;
        for (int sub : c) {
            // the blossom's edge to x: the tightest real edge of any member
            for (int x = 1; x <= top_; ++x)
                if (edge_[sub][x].w > 0 &&
                    (edge_[b][x].w == 0 || slack(edge_[sub][x]) < slack(edge_[b][x]))) {
                    edge_[b][x] = edge_[sub][x];
                    edge_[x][b] = edge_[x][sub];
                }
            for (int x = 1; x <= n_; ++x)
                if (member_of_[sub][x]) member_of_[b][x] = sub;
        }
        recompute_slack(b);
    }

    void expand(int b) {
        std::vector<int>& c = cycle_[b];
        for (int sub : c) set_surface(sub, sub);
        const int entry = member_of_[b][edge_[b][parent_[b]].u];
        const int pos = even_position(b, entry);
        for (int i = 0; i < pos; i += 2) {
            const int inner = c[i], outer = c[i + 1];
            parent_[inner] = edge_[outer][inner].u;
            label_[inner] = 1;
            label_[outer] = 0;
            slack_from_[inner] = 0;
            recompute_slack(outer);
            enqueue(outer);
        }
        label_[entry] = 1;
        parent_[entry] = parent_[b];
        for (size_t i = size_t(pos) + 1; i < c.size(); ++i) {
            label_[c[i]] = -1;
            recompute_slack(c[i]);
        }
        surface_[b] = 0;
    }

    // a tight edge from an outer vertex: grow the tree, or shrink, or augment
    bool scan_tight(const Edge& e) {
        const int u = surface_[e.u], v = surface_[e.v];
        if (label_[v] == -1) {
            parent_[v] = e.u;
            label_[v] = 1;
            const int nu = surface_[mate_[v]];
            slack_from_[v] = slack_from_[nu] = 0;
            label_[nu] = 0;
            enqueue(nu);
        } else if (label_[v] == 0) {
            const int base = common_ancestor(u, v);
            if (!base) {
                augment(u, v);
                augment(v, u);
                return true;
            }
            shrink(u, base, v);
        }
        return false;
    }

    bool phase() {
        std::fill(label_.begin() + 1, label_.begin() + top_ + 1, -1);
        std::fill(slack_from_.begin() + 1, slack_from_.begin() + top_ + 1, 0);
        queue_.clear();
        for (int x = 1; x <= top_; ++x)
            if (surface_[x] == x && !mate_[x]) {
                parent_[x] = 0;
                label_[x] = 0;
                enqueue(x);
            }
        if (queue_.empty()) return false;
        for (;;) {
            while (!queue_.empty()) {
                const int u = queue_.front();
                queue_.pop_front();
                if (label_[surface_[u]] == 1) continue;
                for (int v = 1; v <= n_; ++v)
                    if (edge_[u][v].w > 0 && surface_[u] != surface_[v]) {
                        if (slack(edge_[u][v]) == 0) {
                            if (scan_tight(edge_[u][v])) return true;
                        } else {
                            offer_slack(u, surface_[v]);
                        }
                    }
            }
            // dual adjustment: the largest step that keeps every constraint
            int64_t step = INT64_MAX;
            for (int b = n_ + 1; b <= top_; ++b)
                if (surface_[b] == b && label_[b] == 1) step = std::min(step, dual_[b] / 2);
            for (int x = 1; x <= top_; ++x)
                if (surface_[x] == x && slack_from_[x]) {
                    if (label_[x] == -1)
                        step = std::min(step, slack(edge_[slack_from_[x]][x]));
                    else if (label_[x] == 0)
                        step = std::min(step, slack(edge_[slack_from_[x]][x]) / 2);
                }
            for (int u = 1; u <= n_; ++u)
                if (label_[surface_[u]] == 0 && dual_[u] <= step) return false;   // a free vertex's dual hits zero: optimal
            for (int u = 1; u <= n_; ++u) {               // (checked first: an unbounded step must not be added to anything)
                if (label_[surface_[u]] == 0)
                    dual_[u] -= step;
                else if (label_[surface_[u]] == 1)
                    dual_[u] += step;
            }
            for (int b = n_ + 1; b <= top_; ++b)
                if (surface_[b] == b) {
                    if (label_[b] == 0)
                        dual_[b] += step * 2;
                    else if (label_[b] == 1)
                        dual_[b] -= step * 2;
                }
            queue_.clear();
            for (int x = 1; x <= top_; ++x)
                if (surface_[x] == x && slack_from_[x] && surface_[slack_from_[x]] != x &&
                    slack(edge_[slack_from_[x]][x]) == 0)
                    if (scan_tight(edge_[slack_from_[x]][x])) return true;
            for (int b = n_ + 1; b <= top_; ++b)
                if (surface_[b] == b && label_[b] == 1 && dual_[b] == 0) expand(b);
        }
    }

    int n_, top_;
    int clock_ = 0;
    std::vector<std::vector<Edge>> edge_;
    std::vector<int64_t> dual_;
    std::vector<int> mate_, slack_from_, surface_, parent_, label_, stamp_;
    std::vector<std::vector<int>> member_of_, cycle_;
    std::deque<int> queue_;
};

}  // namespace

int64_t max_weight_matching_blossom(int k, const std::vector<int64_t>& weight, std::vector<int>& mate) {
    mate.assign(k, -1);
    if (k < 2) return 0;
    Blossom solver(k, weight);
    solver.solve(mate);
    int64_t total = 0;
    for (int a = 0; a < k; ++a)
        if (mate[a] > a) total += weight[size_t(a) * k + mate[a]];
    return total;
}

}  // namespace sar
