// Host-side analytical performance model and hierarchical scheduler of HexiSeq (Sec. 4.2-4.3, App. A-B):
// scores a schedule (A2A groups, group sequence lengths L_k, per-rank shards s_d and head counts n_d) and
// searches the schedule space in three stages.  No device code; double precision, every formula evaluated in
// the order the paper writes it.  Readings of what the paper leaves open are stated at each function.
#include <algorithm>
#include <atomic>
#include <thread>
#include <cmath>
#include <cstdarg>
#include <cstdio>
#include <cstdint>
#include <limits>
#include <numeric>
#include <vector>
#include "hexi_attn.h"

#define HEXI_EXPORT extern "C" __attribute__((visibility("default")))

int hexi_set_error(int code, const char* fmt, ...);   // defined with the other entry points

namespace {

constexpr double INF = std::numeric_limits<double>::infinity();

struct Cluster {
    int n;
    const double *c, *b, *m, *m_static, *alpha, *bw;
    double al(int i, int j) const { return alpha[(size_t)i * n + j]; }
    double w(int i, int j) const { return bw[(size_t)i * n + j]; }
};

struct Model {
    long long l_tot;
    long long B, H, d_h, N, P;
    double gamma;
};

struct Sched {
    std::vector<std::vector<int>> groups;   // ring order, devices ascending
    std::vector<long long> l_group, s_pre;
    std::vector<int> n_heads;
};

// ---------------------------------------------------------------- performance model (App. A)

// T_nonattn(d) = max(72 B s_d H^2 / c_d, 40 B s_d H P / b_d)
double t_nonattn(const Cluster& cl, const Model& mo, const Sched& T, int d)
{
    const double flops = 72.0 * (double)mo.B * (double)T.s_pre[d] * (double)mo.H * (double)mo.H;
    const double vol = 40.0 * (double)mo.B * (double)T.s_pre[d] * (double)mo.H * (double)mo.P;
    return std::max(flops / cl.c[d], vol / cl.b[d]);
}

// T_A2A(G_k) = 4 max_{d != j in G_k} (alpha_dj + beta_dj V(d->j)),  V(d->j) = 3 B s_d (n_j d_h) P
double t_a2a(const Cluster& cl, const Model& mo, const Sched& T, int k)
{
    double worst = 0.0;
    for (int d : T.groups[k])
        for (int j : T.groups[k]) {
            if (j == d) continue;
            const double vol = 3.0 * (double)mo.B * (double)T.s_pre[d] * (double)((long long)T.n_heads[j] * mo.d_h) * (double)mo.P;
            worst = std::max(worst, cl.al(d, j) + vol / cl.w(d, j));
        }
    return 4.0 * worst;
}

// Ring step t: group k computes against the KV block that originated in group (k - t) mod K and, for t > 0,
// receives it from its ring predecessor (k - 1) mod K.  Heads lie over a group's devices in device order; the
// senders of device d are the predecessor's devices whose head ranges overlap d's, each sending its overlap, in
// parallel.  With identical layouts this is the paper's single-peer formula.
double t_step(const Cluster& cl, const Model& mo, const Sched& T, int t)
{
    const int K = (int)T.groups.size();
    double worst = 0.0;
    for (int k = 0; k < K; ++k) {
        const int src = ((k - t) % K + K) % K, pred = ((k - 1) % K + K) % K;
        int lo = 0;
        for (int d : T.groups[k]) {
            const int hi = lo + T.n_heads[d];
            const double flops = 16.0 * (double)mo.B * (double)T.l_group[k] * (double)T.l_group[src] * (double)((long long)T.n_heads[d] * mo.d_h);
            double cost = flops / cl.c[d];
            if (t > 0 && T.n_heads[d] > 0) {
                const double msg = 4.0 * (double)mo.B * (double)T.l_group[src] * (double)((long long)T.n_heads[d] * mo.d_h) * (double)mo.P;
                double comm = 0.0;
                int ulo = 0;
                for (int u : T.groups[pred]) {
                    const int uhi = ulo + T.n_heads[u];
                    const int ov = std::min(hi, uhi) - std::max(lo, ulo);
                    if (ov > 0) comm = std::max(comm, cl.al(u, d) + (msg * (double)ov / (double)T.n_heads[d]) / cl.w(u, d));
                    ulo = uhi;
                }
                cost = std::max(cost, comm);
            }
            worst = std::max(worst, cost);
            lo = hi;
        }
    }
    return worst;
}

// T_blk = max_d T_nonattn(d) + max_k T_A2A(G_k) + sum_t T_step(t)
double t_blk(const Cluster& cl, const Model& mo, const Sched& T, double* terms = nullptr)
{
    double a = 0.0, b = 0.0, c = 0.0;
    for (int d = 0; d < cl.n; ++d) a = d == 0 ? t_nonattn(cl, mo, T, d) : std::max(a, t_nonattn(cl, mo, T, d));
    for (int k = 0; k < (int)T.groups.size(); ++k) b = k == 0 ? t_a2a(cl, mo, T, k) : std::max(b, t_a2a(cl, mo, T, k));
    for (int t = 0; t < (int)T.groups.size(); ++t) c += t_step(cl, mo, T, t);
    if (terms) { terms[1] = a; terms[2] = b; terms[3] = c; }
    return a + b + c;
}

// Mem_act(d) = B P (gamma s_d H + 2 L_G(d) n_d d_h)
double mem_act(const Model& mo, const Sched& T, int d, int k)
{
    return (double)(mo.B * mo.P) * (mo.gamma * (double)T.s_pre[d] * (double)mo.H + 2.0 * (double)T.l_group[k] * (double)((long long)T.n_heads[d] * mo.d_h));
}

bool feasible(const Cluster& cl, const Model& mo, const Sched& T)
{
    for (int k = 0; k < (int)T.groups.size(); ++k)
        for (int d : T.groups[k])
            if (cl.m_static[d] + mem_act(mo, T, d, k) > cl.m[d]) return false;
    return true;
}

// ---------------------------------------------------------------- scheduler (Sec. 4.3, App. B)

// Multiples of `quantum` that sum to `total`, proportional to `weights`; leftover units go to the largest
// fractional parts, ties to the lower index.
std::vector<long long> largest_remainder(long long total, const std::vector<double>& weights, long long quantum)
{
    const long long units = total / quantum;
    double wsum = 0.0;
    for (double w : weights) wsum += w;
    const int n = (int)weights.size();
    std::vector<double> exact(n);
    std::vector<long long> base(n);
    long long used = 0;
    for (int i = 0; i < n; ++i) {
        exact[i] = (double)units * (weights[i] / wsum);
        base[i] = (long long)std::floor(exact[i]);
        used += base[i];
    }
    std::vector<int> order(n);
    std::iota(order.begin(), order.end(), 0);
    std::stable_sort(order.begin(), order.end(), [&](int x, int y) { return (exact[x] - (double)base[x]) > (exact[y] - (double)base[y]); });
    for (long long i = 0; i < units - used && i < n; ++i) base[order[i]] += 1;
    for (auto& v : base) v *= quantum;
    return base;
}

using Partition = std::vector<std::vector<int>>;

// Connected components of the edges whose bandwidth (slower direction) is at least `threshold`, ordered by
// their smallest device.
Partition components(const Cluster& cl, double threshold)
{
    const int n = cl.n;
    std::vector<int> parent(n);
    std::iota(parent.begin(), parent.end(), 0);
    auto find = [&](int x) {
        while (parent[x] != x) { parent[x] = parent[parent[x]]; x = parent[x]; }
        return x;
    };
    for (int i = 0; i < n; ++i)
        for (int j = i + 1; j < n; ++j)
            if (std::min(cl.w(i, j), cl.w(j, i)) >= threshold) {
                const int ri = find(i), rj = find(j);
                if (ri != rj) parent[std::max(ri, rj)] = std::min(ri, rj);
            }
    Partition out;
    std::vector<int> slot(n, -1);
    for (int d = 0; d < n; ++d) {
        const int r = find(d);
        if (slot[r] < 0) { slot[r] = (int)out.size(); out.emplace_back(); }
        out[slot[r]].push_back(d);
    }
    return out;
}

double intra_bandwidth(const Cluster& cl, const Partition& p)
{
    double worst = INF;
    for (const auto& g : p)
        for (int i : g)
            for (int j : g)
                if (i != j) worst = std::min(worst, std::min(cl.w(i, j), cl.w(j, i)));
    return worst;
}

// Stage I.  Candidates: the three baseline layouts (singletons, one group, equal consecutive groups of every
// divisor size), then the agglomeration levels from the fastest bandwidth down, stopped before the first level
// more than gap_ratio times slower than the previous one.  Ranked by the smallest intra-group bandwidth, then
// fewer groups, then first appearance; the baselines always stay, the rest fill up to m1.
std::vector<Partition> partition_topology(const Cluster& cl, int m1, double gap_ratio)
{
    const int n = cl.n;
    std::vector<Partition> cands;
    auto add = [&](const Partition& p) {
        for (const auto& q : cands) if (q == p) return;
        cands.push_back(p);
    };
    { Partition p; for (int d = 0; d < n; ++d) p.push_back({d}); add(p); }
    { Partition p(1); for (int d = 0; d < n; ++d) p[0].push_back(d); add(p); }
    for (int size = 2; size < n; ++size)
        if (n % size == 0) {
            Partition p;
            for (int a = 0; a < n; a += size) { std::vector<int> g; for (int d = a; d < a + size; ++d) g.push_back(d); p.push_back(g); }
            add(p);
        }
    const int n_base = (int)cands.size();
    std::vector<double> levels;
    for (int i = 0; i < n; ++i) for (int j = i + 1; j < n; ++j) levels.push_back(std::min(cl.w(i, j), cl.w(j, i)));
    std::sort(levels.begin(), levels.end(), std::greater<double>());
    levels.erase(std::unique(levels.begin(), levels.end()), levels.end());
    bool have_prev = false;
    double prev = 0.0;
    for (double lv : levels) {
        if (have_prev && prev > gap_ratio * lv) break;
        add(components(cl, lv));
        prev = lv; have_prev = true;
    }
    struct Ranked { double bw; int n_groups, idx; };
    std::vector<Ranked> ranked;
    for (int i = 0; i < (int)cands.size(); ++i) ranked.push_back({intra_bandwidth(cl, cands[i]), (int)cands[i].size(), i});
    auto better = [](const Ranked& x, const Ranked& y) {
        if (x.bw != y.bw) return x.bw > y.bw;
        if (x.n_groups != y.n_groups) return x.n_groups < y.n_groups;
        return x.idx < y.idx;
    };
    std::sort(ranked.begin(), ranked.end(), better);
    std::vector<Ranked> keep;
    for (const auto& r : ranked) if (r.idx < n_base) keep.push_back(r);
    for (const auto& r : ranked) {
        if ((int)keep.size() >= std::max(m1, n_base)) break;
        if (r.idx >= n_base) keep.push_back(r);
    }
    std::sort(keep.begin(), keep.end(), better);
    std::vector<Partition> out;
    for (const auto& r : keep) out.push_back(cands[r.idx]);
    return out;
}

// Stage I, second half (Alg. 1 line 2): a group of a retained partition summarised as one super-node -- aggregate
// compute and memory bandwidth, the activation budget of its tightest device, and mean link costs (startup latency,
// inverse bandwidth) over its ordered intra-group pairs and over the edges from its ring predecessor's devices to its
// own.  Stage II prices group-level plans on these summaries alone.
struct SuperNode {
    double size, compute, mem_bw, mem;
    double alpha_in, beta_in, alpha_ring, beta_ring;
};

std::vector<SuperNode> abstract_super_nodes(const Cluster& cl, const Partition& groups)
{
    const int K = (int)groups.size();
    std::vector<SuperNode> nodes(K);
    for (int k = 0; k < K; ++k) {
        const auto& g = groups[k];
        SuperNode sn{(double)g.size(), 0.0, 0.0, INF, 0.0, 0.0, 0.0, 0.0};
        int pairs = 0;
        for (int d : g) {
            sn.compute += cl.c[d];
            sn.mem_bw += cl.b[d];
            sn.mem = std::min(sn.mem, cl.m[d] - cl.m_static[d]);
            for (int j : g)
                if (d != j) { sn.alpha_in += cl.al(d, j); sn.beta_in += 1.0 / cl.w(d, j); ++pairs; }
        }
        if (pairs) { sn.alpha_in = sn.alpha_in / pairs; sn.beta_in = sn.beta_in / pairs; }
        if (K > 1) {
            const auto& pred = groups[(k - 1 + K) % K];
            for (int u : pred)
                for (int d : g) { sn.alpha_ring += cl.al(u, d); sn.beta_ring += 1.0 / cl.w(u, d); }
            const double edges = (double)(pred.size() * g.size());
            sn.alpha_ring = sn.alpha_ring / edges; sn.beta_ring = sn.beta_ring / edges;
        }
        nodes[k] = sn;
    }
    return nodes;
}

// Coarse T_blk of a group-level plan: every group one device that splits its tokens and heads evenly.
double supernode_cost(const std::vector<SuperNode>& nodes, const Model& mo, const std::vector<long long>& lens)
{
    const int K = (int)nodes.size();
    const double B = (double)mo.B, H = (double)mo.H, P = (double)mo.P, N = (double)mo.N, d_h = (double)mo.d_h;
    double nonattn = 0.0, a2a = 0.0, ring = 0.0;
    for (int k = 0; k < K; ++k) {
        const double L = (double)lens[k];
        const double t = std::max(72.0 * B * L * H * H / nodes[k].compute, 40.0 * B * L * H * P / nodes[k].mem_bw);
        nonattn = k == 0 ? t : std::max(nonattn, t);
        if (nodes[k].size > 1.0) {
            const double vol = 3.0 * B * (L / nodes[k].size) * ((N / nodes[k].size) * d_h) * P;
            a2a = std::max(a2a, 4.0 * (nodes[k].alpha_in + nodes[k].beta_in * vol));
        }
    }
    for (int t = 0; t < K; ++t) {
        double worst = 0.0;
        for (int k = 0; k < K; ++k) {
            const int src = ((k - t) % K + K) % K;
            double cost = 16.0 * B * (double)lens[k] * (double)lens[src] * (N * d_h) / nodes[k].compute;
            if (t > 0) {
                const double msg = 4.0 * B * (double)lens[src] * ((N / nodes[k].size) * d_h) * P;
                cost = std::max(cost, nodes[k].alpha_ring + nodes[k].beta_ring * msg);
            }
            worst = std::max(worst, cost);
        }
        ring += worst;
    }
    return nonattn + a2a + ring;
}

bool supernode_feasible(const std::vector<SuperNode>& nodes, const Model& mo, const std::vector<long long>& lens)
{
    for (size_t k = 0; k < nodes.size(); ++k) {
        const double L = (double)lens[k];
        if ((double)(mo.B * mo.P) * (mo.gamma * (L / nodes[k].size) * (double)mo.H + 2.0 * L * (((double)mo.N / nodes[k].size) * (double)mo.d_h)) > nodes[k].mem)
            return false;
    }
    return true;
}

// Stage III initial assignment: s_d and n_d proportional to c_d within the group (uniform for the uniform seed).
Sched initialize_assignment(const Cluster& cl, const Model& mo, const Partition& groups, const std::vector<long long>& l_group, bool uniform, long long q)
{
    Sched T;
    T.groups = groups; T.l_group = l_group;
    T.s_pre.assign(cl.n, 0); T.n_heads.assign(cl.n, 0);
    for (int k = 0; k < (int)groups.size(); ++k) {
        std::vector<double> w;
        for (int d : groups[k]) w.push_back(uniform ? 1.0 : cl.c[d]);
        const auto s = largest_remainder(l_group[k], w, q), h = largest_remainder(mo.N, w, 1);
        for (size_t i = 0; i < groups[k].size(); ++i) { T.s_pre[groups[k][i]] = s[i]; T.n_heads[groups[k][i]] = (int)h[i]; }
    }
    return T;
}

struct GroupPlan { std::vector<long long> lens; bool uniform; };

// Stage II.  Seeds: uniform (L_k by device count), compute-proportional, square-root-compute, memory-capped;
// perturbations: `perturb` of L_tot moved between ring-adjacent groups, both directions.
std::vector<GroupPlan> generate_candidates(const Cluster& cl, const Model& mo, const Partition& groups, long long q, double perturb)
{
    const int K = (int)groups.size();
    std::vector<double> comp(K), cnt(K), root(K);
    for (int k = 0; k < K; ++k) {
        double s = 0.0;
        for (int d : groups[k]) s += cl.c[d];
        comp[k] = s; cnt[k] = (double)groups[k].size(); root[k] = std::sqrt(s);
    }
    std::vector<GroupPlan> seeds;
    seeds.push_back({largest_remainder(mo.l_tot, cnt, q), true});
    seeds.push_back({largest_remainder(mo.l_tot, comp, q), false});
    seeds.push_back({largest_remainder(mo.l_tot, root, q), false});
    std::vector<long long> cap(K);
    for (int k = 0; k < K; ++k) {
        double budget = INF;
        for (int d : groups[k]) budget = std::min(budget, cl.m[d] - cl.m_static[d]);
        const double len = (double)groups[k].size();
        const double per_token = (double)(mo.B * mo.P) * (mo.gamma * (double)mo.H / len + 2.0 * ((double)mo.N / len) * (double)mo.d_h);
        cap[k] = (long long)std::floor(std::max(0.0, budget / per_token) / (double)q) * q;
    }
    std::vector<long long> lens = largest_remainder(mo.l_tot, comp, q);
    for (int round = 0; round < K; ++round) {
        std::vector<int> over;
        for (int k = 0; k < K; ++k) if (lens[k] > cap[k]) over.push_back(k);
        if (over.empty()) break;
        long long excess = 0;
        for (int k : over) { excess += lens[k] - cap[k]; lens[k] = cap[k]; }
        std::vector<int> free_k;
        for (int k = 0; k < K; ++k) if (lens[k] < cap[k]) free_k.push_back(k);
        if (free_k.empty()) break;
        std::vector<double> w;
        for (int k : free_k) w.push_back(comp[k]);
        const auto extra = largest_remainder(excess, w, q);
        for (size_t i = 0; i < free_k.size(); ++i) lens[free_k[i]] += extra[i];
    }
    if (std::accumulate(lens.begin(), lens.end(), 0LL) == mo.l_tot) seeds.push_back({lens, false});
    std::vector<GroupPlan> out;
    auto add = [&](const std::vector<long long>& l, bool uniform) {
        for (long long x : l) if (x <= 0) return;
        for (const auto& o : out) if (o.lens == l && o.uniform == uniform) return;
        out.push_back({l, uniform});
    };
    const long long delta = ((long long)((double)mo.l_tot * perturb) / q) * q;
    for (const auto& s : seeds) add(s.lens, s.uniform);
    for (const auto& s : seeds)
        if (K > 1 && delta > 0)
            for (int k = 0; k < K; ++k) {
                const int nbs[2] = {(k + 1) % K, (k - 1 + K) % K};
                for (int nb : nbs)
                    if (nb != k && s.lens[k] > delta) {
                        std::vector<long long> moved = s.lens;
                        moved[k] -= delta; moved[nb] += delta;
                        add(moved, false);
                    }
            }
    return out;
}

// Ring cost of group k at step t: the slowest of its devices (the inner part of T_step, per group).
double group_step(const Cluster& cl, const Model& mo, const Sched& T, int t, int k)
{
    const int K = (int)T.groups.size();
    const int src = ((k - t) % K + K) % K, pred = ((k - 1) % K + K) % K;
    double worst = 0.0;
    int lo = 0;
    for (int d : T.groups[k]) {
        const int hi = lo + T.n_heads[d];
        const double flops = 16.0 * (double)mo.B * (double)T.l_group[k] * (double)T.l_group[src] * (double)((long long)T.n_heads[d] * mo.d_h);
        double cost = flops / cl.c[d];
        if (t > 0 && T.n_heads[d] > 0) {
            const double msg = 4.0 * (double)mo.B * (double)T.l_group[src] * (double)((long long)T.n_heads[d] * mo.d_h) * (double)mo.P;
            double comm = 0.0;
            int ulo = 0;
            for (int u : T.groups[pred]) {
                const int uhi = ulo + T.n_heads[u];
                const int ov = std::min(hi, uhi) - std::max(lo, ulo);
                if (ov > 0) comm = std::max(comm, cl.al(u, d) + (msg * (double)ov / (double)T.n_heads[d]) / cl.w(u, d));
                ulo = uhi;
            }
            cost = std::max(cost, comm);
        }
        worst = std::max(worst, cost);
        lo = hi;
    }
    return worst;
}

// Coordinate descent of Stage III: ordered pairs of distinct devices in the same or ring-adjacent groups,
// lexicographic; per pair first `move_tokens` tokens from a to b (the group lengths follow when the groups
// differ), then one head from a to b (same group only); the first strictly improving feasible move is taken.
// The model's terms are kept per device (T_nonattn), per group (T_A2A) and per (step, group) (ring cost), and a
// proposal recomputes only the entries its move touches: a token move inside a group changes two devices'
// T_nonattn and the group's T_A2A; one between groups also the ring cost of every (step, group) whose query or
// source block is one of the two; a head move the group's T_A2A, its own ring costs and its ring successor's
// (whose senders' head ranges moved).  The terms are combined exactly as in t_blk, so the values are the same.
double refine(const Cluster& cl, const Model& mo, Sched& T, int i_max, long long move_tokens)
{
    const int K = (int)T.groups.size(), n = cl.n;
    std::vector<int> group_of(n);
    for (int k = 0; k < K; ++k) for (int d : T.groups[k]) group_of[d] = k;
    std::vector<double> na(n), a2a(K), ring((size_t)K * K), na2, a2a2, ring2;
    for (int d = 0; d < n; ++d) na[d] = t_nonattn(cl, mo, T, d);
    for (int k = 0; k < K; ++k) a2a[k] = t_a2a(cl, mo, T, k);
    for (int t = 0; t < K; ++t) for (int k = 0; k < K; ++k) ring[(size_t)t * K + k] = group_step(cl, mo, T, t, k);
    auto total = [&](const std::vector<double>& v_na, const std::vector<double>& v_a2a, const std::vector<double>& v_ring) {
        double a = v_na[0], b = v_a2a[0], c = 0.0;
        for (int d = 1; d < n; ++d) a = std::max(a, v_na[d]);
        for (int k = 1; k < K; ++k) b = std::max(b, v_a2a[k]);
        for (int t = 0; t < K; ++t) {
            double w = 0.0;
            for (int k = 0; k < K; ++k) w = std::max(w, v_ring[(size_t)t * K + k]);
            c += w;
        }
        return a + b + c;
    };
    auto fits = [&](int d) { return !(cl.m_static[d] + mem_act(mo, T, d, group_of[d]) > cl.m[d]); };
    double C = total(na, a2a, ring);
    bool improved = true;
    for (int it = 0; improved && it < i_max; ++it) {
        improved = false;
        for (int a = 0; a < n && !improved; ++a)
            for (int b = 0; b < n && !improved; ++b) {
                if (a == b) continue;
                const int ka = group_of[a], kb = group_of[b];
                if (!(ka == kb || ((kb - ka) % K + K) % K == 1 || ((ka - kb) % K + K) % K == 1)) continue;
                if (T.s_pre[a] >= move_tokens && (ka == kb || T.l_group[ka] > move_tokens)) {
                    T.s_pre[a] -= move_tokens; T.s_pre[b] += move_tokens;
                    if (ka != kb) { T.l_group[ka] -= move_tokens; T.l_group[kb] += move_tokens; }
                    bool ok = fits(a) && fits(b);
                    if (ok && ka != kb) {
                        for (int d : T.groups[ka]) ok = ok && fits(d);
                        for (int d : T.groups[kb]) ok = ok && fits(d);
                    }
                    if (ok) {
                        na2 = na; a2a2 = a2a; ring2 = ring;
                        na2[a] = t_nonattn(cl, mo, T, a); na2[b] = t_nonattn(cl, mo, T, b);
                        a2a2[ka] = t_a2a(cl, mo, T, ka);
                        if (kb != ka) {
                            a2a2[kb] = t_a2a(cl, mo, T, kb);
                            for (int t = 0; t < K; ++t) {
                                ring2[(size_t)t * K + ka] = group_step(cl, mo, T, t, ka);
                                ring2[(size_t)t * K + kb] = group_step(cl, mo, T, t, kb);
                            }
                            for (int k = 0; k < K; ++k) {     // groups that receive one of the two blocks at some step
                                const int ta = ((k - ka) % K + K) % K, tb = ((k - kb) % K + K) % K;
                                ring2[(size_t)ta * K + k] = group_step(cl, mo, T, ta, k);
                                ring2[(size_t)tb * K + k] = group_step(cl, mo, T, tb, k);
                            }
                        }
                        const double c2 = total(na2, a2a2, ring2);
                        if (c2 < C) { na.swap(na2); a2a.swap(a2a2); ring.swap(ring2); C = c2; improved = true; break; }
                    }
                    T.s_pre[a] += move_tokens; T.s_pre[b] -= move_tokens;
                    if (ka != kb) { T.l_group[ka] += move_tokens; T.l_group[kb] -= move_tokens; }
                }
                if (ka == kb && T.n_heads[a] >= 1) {
                    T.n_heads[a] -= 1; T.n_heads[b] += 1;
                    if (fits(a) && fits(b)) {
                        a2a2 = a2a; ring2 = ring;
                        a2a2[ka] = t_a2a(cl, mo, T, ka);
                        const int succ = (ka + 1) % K;
                        for (int t = 0; t < K; ++t) {
                            ring2[(size_t)t * K + ka] = group_step(cl, mo, T, t, ka);
                            ring2[(size_t)t * K + succ] = group_step(cl, mo, T, t, succ);
                        }
                        const double c2 = total(na, a2a2, ring2);
                        if (c2 < C) { a2a.swap(a2a2); ring.swap(ring2); C = c2; improved = true; break; }
                    }
                    T.n_heads[a] += 1; T.n_heads[b] -= 1;
                }
            }
    }
    return C;
}

int check_inputs(const hexi_cluster* cl, const hexi_model* mo)
{
    if (!cl || !mo) return hexi_set_error(HEXI_EINVAL, "null cluster or model");
    if (cl->n_devices < 1 || cl->n_devices > HEXI_SCHED_MAX_DEVICES) return hexi_set_error(HEXI_EINVAL, "n_devices %d out of range", cl->n_devices);
    if (!cl->c || !cl->b || !cl->m || !cl->m_static || !cl->alpha || !cl->bw) return hexi_set_error(HEXI_EINVAL, "null cluster array");
    const int n = cl->n_devices;
    for (int d = 0; d < n; ++d)
        if (!(cl->c[d] > 0.0) || !(cl->b[d] > 0.0) || !(cl->m[d] >= 0.0) || !(cl->m_static[d] >= 0.0)) return hexi_set_error(HEXI_EINVAL, "device %d: non-positive rate or negative memory", d);
    for (int i = 0; i < n; ++i)
        for (int j = 0; j < n; ++j)
            if (i != j && (!(cl->bw[(size_t)i * n + j] > 0.0) || !(cl->alpha[(size_t)i * n + j] >= 0.0))) return hexi_set_error(HEXI_EINVAL, "link %d->%d: non-positive bandwidth or negative latency", i, j);
    if (mo->l_tot < 1 || mo->batch < 1 || mo->hidden < 1 || mo->head_dim < 1 || mo->n_heads < 1 || mo->dtype_bytes < 1 || !(mo->gamma_act >= 0.0))
        return hexi_set_error(HEXI_EINVAL, "bad model sizes");
    return HEXI_OK;
}

Cluster wrap(const hexi_cluster* c) { return Cluster{c->n_devices, c->c, c->b, c->m, c->m_static, c->alpha, c->bw}; }
Model wrap(const hexi_model* m) { return Model{m->l_tot, m->batch, m->hidden, m->head_dim, m->n_heads, m->dtype_bytes, m->gamma_act}; }

}  // namespace

HEXI_EXPORT int hexi_sched_cost(const hexi_cluster* cluster, const hexi_model* model, const hexi_schedule* schedule, double* terms, int32_t* is_feasible)
{
    int rc = check_inputs(cluster, model);
    if (rc != HEXI_OK) return rc;
    if (!schedule || !schedule->group_of || !schedule->l_group || !schedule->s_pre || !schedule->n_heads) return hexi_set_error(HEXI_EINVAL, "null schedule array");
    const Cluster cl = wrap(cluster);
    const Model mo = wrap(model);
    const int K = schedule->n_groups;
    if (K < 1 || K > cl.n) return hexi_set_error(HEXI_EINVAL, "n_groups %d out of range", K);
    Sched T;
    T.groups.assign(K, {});
    T.l_group.assign(schedule->l_group, schedule->l_group + K);
    T.s_pre.assign(schedule->s_pre, schedule->s_pre + cl.n);
    T.n_heads.assign(schedule->n_heads, schedule->n_heads + cl.n);
    for (int d = 0; d < cl.n; ++d) {
        if (schedule->group_of[d] < 0 || schedule->group_of[d] >= K) return hexi_set_error(HEXI_EINVAL, "group_of[%d] = %d out of range", d, schedule->group_of[d]);
        T.groups[schedule->group_of[d]].push_back(d);
        if (T.s_pre[d] < 0 || T.n_heads[d] < 0) return hexi_set_error(HEXI_EINVAL, "negative shard or head count on device %d", d);
    }
    long long l_sum = 0;
    for (int k = 0; k < K; ++k) {
        if (T.groups[k].empty() || T.l_group[k] <= 0) return hexi_set_error(HEXI_EINVAL, "group %d is empty or has no tokens", k);
        long long s = 0, h = 0;
        for (int d : T.groups[k]) { s += T.s_pre[d]; h += T.n_heads[d]; }
        if (s != T.l_group[k]) return hexi_set_error(HEXI_EINVAL, "shards of group %d sum to %lld, not L_k = %lld", k, s, T.l_group[k]);
        if (h != mo.N) return hexi_set_error(HEXI_EINVAL, "heads of group %d sum to %lld, not %lld", k, h, mo.N);
        l_sum += T.l_group[k];
    }
    if (l_sum != mo.l_tot) return hexi_set_error(HEXI_EINVAL, "group lengths sum to %lld, not L_tot = %lld", l_sum, mo.l_tot);
    double t[4] = {0, 0, 0, 0};
    t[0] = t_blk(cl, mo, T, t);
    if (terms) for (int i = 0; i < 4; ++i) terms[i] = t[i];
    if (is_feasible) *is_feasible = feasible(cl, mo, T) ? 1 : 0;
    return HEXI_OK;
}

HEXI_EXPORT int hexi_sched_solve(const hexi_cluster* cluster, const hexi_model* model, const hexi_sched_opts* opts, hexi_schedule* out, double* cost)
{
    int rc = check_inputs(cluster, model);
    if (rc != HEXI_OK) return rc;
    if (!out || !out->group_of || !out->l_group || !out->s_pre || !out->n_heads) return hexi_set_error(HEXI_EINVAL, "null schedule array");
    const Cluster cl = wrap(cluster);
    const Model mo = wrap(model);
    const int m1 = opts && opts->m1 > 0 ? opts->m1 : 64, m2 = opts && opts->m2 > 0 ? opts->m2 : 16, i_max = opts && opts->i_max > 0 ? opts->i_max : 100;
    const double gap_ratio = opts && opts->gap_ratio > 0.0 ? opts->gap_ratio : 4.0, perturb = opts && opts->perturb > 0.0 ? opts->perturb : 1.0 / 32;
    const long long q = opts && opts->token_quantum > 0 ? opts->token_quantum : 64;
    if (mo.l_tot % q) return hexi_set_error(HEXI_EINVAL, "L_tot = %lld is not a multiple of the token quantum %lld", mo.l_tot, q);
    const long long move_tokens = opts && opts->move_tokens > 0 ? opts->move_tokens : std::max(1LL, mo.l_tot / (q * cl.n * 16)) * q;
    // Stages I and II: the shortlist of (partition, group plan) starting points, in a fixed order
    std::vector<Sched> starts;
    for (const Partition& groups : partition_topology(cl, m1, gap_ratio)) {
        // Stage II on the partition's super-node summaries: the m2 cheapest group-level plans that fit the groups'
        // memory proxies go on; a plan whose initial rank-level assignment fails the per-device filter is dropped
        const auto nodes = abstract_super_nodes(cl, groups);
        struct Scored { double cost; int idx; };
        std::vector<Scored> scored;
        const auto plans = generate_candidates(cl, mo, groups, q, perturb);
        for (int i = 0; i < (int)plans.size(); ++i)
            if (supernode_feasible(nodes, mo, plans[i].lens)) scored.push_back({supernode_cost(nodes, mo, plans[i].lens), i});
        std::sort(scored.begin(), scored.end(), [](const Scored& x, const Scored& y) { return x.cost != y.cost ? x.cost < y.cost : x.idx < y.idx; });
        for (int i = 0; i < (int)scored.size() && i < m2; ++i) {
            Sched T = initialize_assignment(cl, mo, groups, plans[scored[i].idx].lens, plans[scored[i].idx].uniform, q);
            if (feasible(cl, mo, T)) starts.push_back(T);
        }
    }
    // Stage III: the descents are independent of each other, so they run on the host's cores; the winner is
    // picked afterwards in shortlist order (first strictly smaller cost), so the result does not depend on timing
    std::vector<double> costs(starts.size(), INF);
    {
        std::atomic<size_t> next{0};
        auto worker = [&]() {
            for (size_t i = next.fetch_add(1); i < starts.size(); i = next.fetch_add(1)) costs[i] = refine(cl, mo, starts[i], i_max, move_tokens);
        };
        unsigned n_threads = std::thread::hardware_concurrency();
        n_threads = n_threads == 0 ? 1 : (n_threads > 16 ? 16 : n_threads);
        if (n_threads > starts.size()) n_threads = (unsigned)starts.size();
        std::vector<std::thread> pool;
        for (unsigned t = 1; t < n_threads; ++t) pool.emplace_back(worker);
        worker();
        for (auto& th : pool) th.join();
    }
    Sched best;
    double best_c = INF;
    for (size_t i = 0; i < starts.size(); ++i)
        if (costs[i] < best_c) { best = starts[i]; best_c = costs[i]; }
    if (best_c == INF) return hexi_set_error(HEXI_EINFEASIBLE, "no candidate schedule passes the memory filter");
    out->n_groups = (int)best.groups.size();
    for (int k = 0; k < out->n_groups; ++k) {
        out->l_group[k] = best.l_group[k];
        for (int d : best.groups[k]) out->group_of[d] = k;
    }
    for (int d = 0; d < cl.n; ++d) { out->s_pre[d] = best.s_pre[d]; out->n_heads[d] = best.n_heads[d]; }
    if (cost) *cost = best_c;
    return HEXI_OK;
}
