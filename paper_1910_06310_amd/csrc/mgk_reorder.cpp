// Vertex orderings for tile packing (Section IV-A).  Host only, no GPU code.
//
// The partition-based reordering follows the goal stated with Eq. 3: a
// perfectly balanced K = ceil(n/t)-way partition with as few connected part
// pairs as possible.  The paper obtains it from an external recursive
// hypergraph bipartitioner; this is an independent heuristic with the same
// objective: recursive bisection (greedy growing + exact-balance swap
// refinement on the edge cut) followed by a K-way swap refinement that
// evaluates Eq. 3 directly, with the edge cut as tie-break.  Any permutation
// gives the same kernel values; only the tile count depends on it.
#include "mgk_reorder.h"

#include <algorithm>
#include <numeric>
#include <queue>
#include <unordered_map>

std::vector<int32_t> mgk_order_identity(int n) {
    std::vector<int32_t> p(n);
    std::iota(p.begin(), p.end(), 0);
    return p;
}

// ---------------------------------------------------------------- Morton curve
std::vector<int32_t> mgk_order_morton(int n, int dim, const float* coords) {
    const int bits = 21 / dim;   // 21, 10 or 7 bits per coordinate
    std::vector<float> lo(dim, 0.f), hi(dim, 0.f);
    for (int a = 0; a < dim; ++a) {
        lo[a] = hi[a] = n ? coords[a] : 0.f;
        for (int v = 1; v < n; ++v) {
            lo[a] = std::min(lo[a], coords[(size_t)v * dim + a]);
            hi[a] = std::max(hi[a], coords[(size_t)v * dim + a]);
        }
    }
    std::vector<std::pair<uint64_t, int32_t>> key(n);
    const double cells = (double)(1u << bits);
    for (int v = 0; v < n; ++v) {
        uint64_t k = 0;
        for (int a = 0; a < dim; ++a) {
            const double span = (double)hi[a] - (double)lo[a];
            const double u = span > 0.0 ? ((double)coords[(size_t)v * dim + a] - lo[a]) / span : 0.0;
            const uint64_t q = (uint64_t)std::min(cells - 1.0, std::max(0.0, u * cells));
            for (int b = 0; b < bits; ++b) k |= ((q >> b) & 1ull) << (dim * b + a);
        }
        key[v] = {k, v};
    }
    std::stable_sort(key.begin(), key.end(),
                     [](const std::pair<uint64_t, int32_t>& x, const std::pair<uint64_t, int32_t>& y) { return x.first < y.first; });
    std::vector<int32_t> perm(n);
    for (int r = 0; r < n; ++r) perm[key[r].second] = r;
    return perm;
}

// ---------------------------------------------------------------- RCM
namespace {

// BFS levels inside the vertex subset marked by in_set == tag; returns the
// last vertex reached (an end of a long shortest path) and fills `order`.
int bfs_far(const MgkAdj& g, int start, const std::vector<int>& in_set, int tag,
            std::vector<int>& dist, std::vector<int32_t>& order) {
    order.clear();
    order.push_back(start);
    dist[start] = 0;
    for (size_t h = 0; h < order.size(); ++h) {
        int v = order[h];
        for (int k = g.ptr[v]; k < g.ptr[v + 1]; ++k) {
            int w = g.idx[k];
            if (in_set[w] == tag && dist[w] < 0) {
                dist[w] = dist[v] + 1;
                order.push_back(w);
            }
        }
    }
    int far = order.back();
    for (int v : order) dist[v] = -1;
    return far;
}

}  // namespace

std::vector<int32_t> mgk_order_rcm(const MgkAdj& g) {
    const int n = g.n;
    std::vector<int32_t> seq;
    seq.reserve(n);
    std::vector<int> in_set(n, 0), dist(n, -1);
    std::vector<char> done(n, 0);
    std::vector<int32_t> tmp, nb;
    auto deg = [&](int v) { return g.ptr[v + 1] - g.ptr[v]; };
    for (int s0 = 0; s0 < n; ++s0) {
        if (done[s0]) continue;
        // pseudo-peripheral start: two sweeps
        int s = bfs_far(g, s0, in_set, 0, dist, tmp);
        s = bfs_far(g, s, in_set, 0, dist, tmp);
        size_t head = seq.size();
        seq.push_back(s);
        done[s] = 1;
        in_set[s] = 1;
        for (; head < seq.size(); ++head) {
            int v = seq[head];
            nb.clear();
            for (int k = g.ptr[v]; k < g.ptr[v + 1]; ++k)
                if (!done[g.idx[k]]) { nb.push_back(g.idx[k]); done[g.idx[k]] = 1; in_set[g.idx[k]] = 1; }
            std::sort(nb.begin(), nb.end(), [&](int a, int b) {
                return deg(a) != deg(b) ? deg(a) < deg(b) : a < b;
            });
            for (int w : nb) seq.push_back(w);
        }
    }
    std::vector<int32_t> perm(n);
    for (int k = 0; k < n; ++k) perm[seq[k]] = n - 1 - k;
    return perm;
}

// ---------------------------------------------------------------- PBR
namespace {

struct Bisector {
    const MgkAdj& g;
    int t;
    std::vector<int32_t> part;   // result: part id per vertex
    std::vector<int> mark;       // scratch: subset tag per vertex
    std::vector<int> side;       // 0 / 1 inside the current subset
    std::vector<int> gain;
    std::vector<char> locked;
    std::vector<int> dist;
    std::vector<int32_t> tmp;
    int tag_counter = 0;

    Bisector(const MgkAdj& g_, int t_)
        : g(g_), t(t_), part(g_.n, 0), mark(g_.n, 0), side(g_.n, 0), gain(g_.n, 0),
          locked(g_.n, 0), dist(g_.n, -1) {}

    void run() {
        std::vector<int32_t> all(g.n);
        std::iota(all.begin(), all.end(), 0);
        split(all, 0, (g.n + t - 1) / t);
    }

    void split(std::vector<int32_t>& V, int first_part, int nparts) {
        if (nparts <= 1) {
            for (int v : V) part[v] = first_part;
            return;
        }
        const int kl = (nparts + 1) / 2;
        const int size_l = kl * t;
        const int tag = ++tag_counter;
        for (int v : V) { mark[v] = tag; side[v] = 1; }

        // ---- greedy growing of side 0 from a far-apart vertex
        int start = V[0];
        for (int v : V)
            if (g.ptr[v + 1] - g.ptr[v] < g.ptr[start + 1] - g.ptr[start]) start = v;
        start = bfs_far(g, start, mark, tag, dist, tmp);
        // conn[v] = edges from v into side 0 (only for side-1 vertices of the subset)
        for (int v : V) gain[v] = 0;
        int grown = 0;
        auto add_to_left = [&](int v) {
            side[v] = 0;
            ++grown;
            for (int k = g.ptr[v]; k < g.ptr[v + 1]; ++k) {
                int w = g.idx[k];
                if (mark[w] == tag) ++gain[w];
            }
        };
        add_to_left(start);
        while (grown < size_l) {
            int best = -1, best_key = 0;
            for (int v : V) {
                if (side[v] == 0) continue;
                // prefer vertices mostly attached to the grown side; among
                // unattached ones (new component) prefer low degree
                int in_sub = 0;
                for (int k = g.ptr[v]; k < g.ptr[v + 1]; ++k) in_sub += mark[g.idx[k]] == tag;
                int key = gain[v] > 0 ? 1000000 + 2 * gain[v] - in_sub : -in_sub;
                if (best < 0 || key > best_key) { best = v; best_key = key; }
            }
            add_to_left(best);
        }

        refine_bisection(V, tag);

        std::vector<int32_t> L, R;
        L.reserve(size_l);
        R.reserve(V.size() - size_l);
        for (int v : V) (side[v] == 0 ? L : R).push_back(v);
        V.clear();
        V.shrink_to_fit();
        split(L, first_part, kl);
        split(R, first_part + kl, nparts - kl);
    }

    // Kernighan-Lin style passes of pairwise swaps (sizes stay exact),
    // minimising the number of cut edges inside the subset.
    void refine_bisection(const std::vector<int32_t>& V, int tag) {
        const int max_pass = 6;
        for (int pass = 0; pass < max_pass; ++pass) {
            for (int v : V) {
                int ext = 0, in = 0;
                for (int k = g.ptr[v]; k < g.ptr[v + 1]; ++k) {
                    int w = g.idx[k];
                    if (mark[w] != tag) continue;
                    (side[w] == side[v] ? in : ext)++;
                }
                gain[v] = ext - in;
                locked[v] = 0;
            }
            std::vector<std::pair<int, int>> swaps;
            int cum = 0, best_cum = 0;
            size_t best_len = 0;
            const size_t max_swaps = std::min<size_t>(V.size() / 2, 64 + V.size() / 8);
            for (size_t s = 0; s < max_swaps; ++s) {
                // best unlocked vertex on each side, then correct for a shared edge
                int a = -1, b = -1;
                for (int v : V) {
                    if (locked[v]) continue;
                    if (side[v] == 0) { if (a < 0 || gain[v] > gain[a]) a = v; }
                    else { if (b < 0 || gain[v] > gain[b]) b = v; }
                }
                if (a < 0 || b < 0) break;
                // look for a better partner among the top candidates of side 1
                int best_b = b, best_g = -1000000;
                for (int v : V) {
                    if (locked[v] || side[v] != 1 || gain[v] < gain[b] - 2) continue;
                    int adj = 0;
                    for (int k = g.ptr[a]; k < g.ptr[a + 1]; ++k) adj += g.idx[k] == v;
                    int gsum = gain[a] + gain[v] - 2 * adj;
                    if (gsum > best_g) { best_g = gsum; best_b = v; }
                }
                b = best_b;
                if (best_g < -4 && cum <= best_cum) break;  // hopeless tail
                // apply swap
                for (int pass_v = 0; pass_v < 2; ++pass_v) {
                    int v = pass_v ? b : a;
                    for (int k = g.ptr[v]; k < g.ptr[v + 1]; ++k) {
                        int w = g.idx[k];
                        if (mark[w] != tag || w == a || w == b) continue;
                        gain[w] += (side[w] == side[v]) ? 2 : -2;
                    }
                }
                side[a] = 1; side[b] = 0;
                locked[a] = locked[b] = 1;
                cum += best_g;
                swaps.emplace_back(a, b);
                if (cum > best_cum) { best_cum = cum; best_len = swaps.size(); }
            }
            for (size_t s = swaps.size(); s > best_len; --s) {
                side[swaps[s - 1].first] = 0;
                side[swaps[s - 1].second] = 1;
            }
            if (best_cum <= 0) break;
        }
    }
};

// Edge counts between parts: dense for moderate K, hashed otherwise.
struct PairCounts {
    int K;
    bool dense;
    std::vector<int32_t> d;
    std::unordered_map<uint64_t, int32_t> h;
    explicit PairCounts(int K_) : K(K_), dense(K_ <= 1024) {
        if (dense) d.assign((size_t)K * K, 0);
    }
    static uint64_t key(int a, int b) {
        if (a > b) std::swap(a, b);
        return ((uint64_t)(uint32_t)a << 32) | (uint32_t)b;
    }
    int get(int a, int b) const {
        if (dense) return d[(size_t)std::min(a, b) * K + std::max(a, b)];
        auto it = h.find(key(a, b));
        return it == h.end() ? 0 : it->second;
    }
    void add(int a, int b, int delta) {
        if (dense) d[(size_t)std::min(a, b) * K + std::max(a, b)] += delta;
        else h[key(a, b)] += delta;
    }
};

// K-way refinement on the objective of Eq. 3: swap two vertices of different
// parts when that lowers the number of connected part pairs (ties: fewer cut
// edges).  Part sizes never change.
void kway_refine(const MgkAdj& g, std::vector<int32_t>& part, int K, int max_pass) {
    if (K < 2) return;
    PairCounts C(K);
    for (int v = 0; v < g.n; ++v)
        for (int k = g.ptr[v]; k < g.ptr[v + 1]; ++k) {
            int w = g.idx[k];
            if (v < w) C.add(part[v], part[w], 1);
        }
    std::vector<std::vector<int32_t>> members(K);
    for (int v = 0; v < g.n; ++v) members[part[v]].push_back(v);

    // Trading places of v (part A) and u (part B) only changes the edge counts
    // of pairs (A, P) and (B, P): dA[P] / dB[P] hold those changes.
    std::vector<int> dA(K, 0), dB(K, 0), touched;
    std::vector<char> seen(K, 0);
    auto touch = [&](int P) {
        if (!seen[P]) { seen[P] = 1; touched.push_back(P); }
    };
    auto collect = [&](int v, int u) {
        const int A = part[v], B = part[u];
        for (int P : touched) { dA[P] = dB[P] = 0; seen[P] = 0; }
        touched.clear();
        for (int k = g.ptr[v]; k < g.ptr[v + 1]; ++k) {
            int w = g.idx[k];
            if (w == u) continue;
            const int P = part[w];
            touch(P); dA[P] -= 1; dB[P] += 1;
        }
        for (int k = g.ptr[u]; k < g.ptr[u + 1]; ++k) {
            int w = g.idx[k];
            if (w == v) continue;
            const int P = part[w];
            touch(P); dB[P] -= 1; dA[P] += 1;
        }
        (void)A; (void)B;
    };
    auto change = [&](int a, int b, int d) { const int c = C.get(a, b); return ((c + d) > 0) - (c > 0); };
    // change of (connected pairs, cut edges) if v (part A) and u (part B) trade places
    auto eval_swap = [&](int v, int u, int& dpairs, int& dcut) {
        const int A = part[v], B = part[u];
        collect(v, u);
        dpairs = 0; dcut = 0;
        for (int P : touched) {
            if (P == A || P == B) continue;
            if (dA[P]) { dpairs += change(A, P, dA[P]); dcut += dA[P]; }
            if (dB[P]) { dpairs += change(B, P, dB[P]); dcut += dB[P]; }
        }
        const int dab = dA[B] + dB[A];
        if (dab) { dpairs += change(A, B, dab); dcut += dab; }
    };
    auto apply_swap = [&](int v, int u) {
        const int A = part[v], B = part[u];
        collect(v, u);
        for (int P : touched) {
            if (P != A && P != B) {
                if (dA[P]) C.add(A, P, dA[P]);
                if (dB[P]) C.add(B, P, dB[P]);
            }
        }
        const int dab = dA[B] + dB[A];
        if (dab) C.add(A, B, dab);
        // diagonal counts are never read
        part[v] = B; part[u] = A;
        std::replace(members[A].begin(), members[A].end(), v, u);
        std::replace(members[B].begin(), members[B].end(), u, v);
    };

    int64_t connected = 0;  // current value of Eq. 3
    for (int a = 0; a < K && C.dense; ++a)
        for (int b = a + 1; b < K; ++b) connected += C.get(a, b) > 0;
    if (!C.dense)
        for (auto& kv : C.h) connected += (kv.first >> 32) != (kv.first & 0xffffffffu) && kv.second > 0;
    std::vector<int> cand_parts;
    for (int pass = 0; pass < max_pass; ++pass) {
        bool improved = false;
        int64_t gained = 0;
        for (int v = 0; v < g.n; ++v) {
            const int A = part[v];
            cand_parts.clear();
            for (int k = g.ptr[v]; k < g.ptr[v + 1]; ++k) {
                int P = part[g.idx[k]];
                if (P != A && std::find(cand_parts.begin(), cand_parts.end(), P) == cand_parts.end())
                    cand_parts.push_back(P);
            }
            if (cand_parts.empty()) continue;
            int best_u = -1, best_dp = 0, best_dc = 0;
            for (int B : cand_parts)
                for (int u : members[B]) {
                    int dp, dc;
                    eval_swap(v, u, dp, dc);
                    if (dp < best_dp || (dp == best_dp && dc < best_dc)) {
                        best_dp = dp; best_dc = dc; best_u = u;
                    }
                }
            if (best_u >= 0) {
                apply_swap(v, best_u);
                improved = true;
                gained -= best_dp;
            }
        }
        connected -= gained;
        // stop when a whole pass removes less than 0.5 % of the connected pairs
        if (!improved || gained * 200 < connected) break;
    }
}

}  // namespace

std::vector<int32_t> mgk_order_pbr(const MgkAdj& g, int t) {
    const int n = g.n;
    const int K = (n + t - 1) / t;
    if (K <= 1) return mgk_order_identity(n);
    // With an average degree of several tiles' width every pair of parts is
    // connected whatever the order: nothing to gain, and the swap search would
    // cost O(n K t deg^2).
    if ((int64_t)g.idx.size() > (int64_t)4 * t * n) return mgk_order_identity(n);
    // Three starting partitions, each refined on Eq. 3; the best one wins:
    // recursive bisection, blocks of t consecutive vertices in reverse
    // Cuthill-McKee order (strong on banded / lattice-like graphs), and blocks
    // of the given order (strong when the input already has locality).
    auto blocks_of = [&](const std::vector<int32_t>& order) {
        std::vector<int32_t> part(n);
        for (int v = 0; v < n; ++v) part[v] = order[v] / t;
        return part;
    };
    auto to_perm = [&](const std::vector<int32_t>& part) {
        std::vector<int32_t> perm(n), fill(K, 0);
        for (int v = 0; v < n; ++v) perm[v] = part[v] * t + fill[part[v]]++;
        return perm;
    };
    Bisector bis(g, t);
    bis.run();
    std::vector<std::vector<int32_t>> starts;
    starts.push_back(bis.part);
    starts.push_back(blocks_of(mgk_order_rcm(g)));
    starts.push_back(blocks_of(mgk_order_identity(n)));
    std::vector<int32_t> best_perm;
    int64_t best_count = -1;
    for (auto& part : starts) {
        kway_refine(g, part, K, 8);
        std::vector<int32_t> perm = to_perm(part);
        const int64_t count = mgk_count_offdiag_tiles(g, perm, t);
        if (best_count < 0 || count < best_count) { best_count = count; best_perm.swap(perm); }
    }
    return best_perm;
}

int64_t mgk_count_offdiag_tiles(const MgkAdj& g, const std::vector<int32_t>& perm, int t) {
    std::vector<uint64_t> keys;
    for (int v = 0; v < g.n; ++v)
        for (int k = g.ptr[v]; k < g.ptr[v + 1]; ++k) {
            int a = perm[v] / t, b = perm[g.idx[k]] / t;
            if (a != b) keys.push_back(((uint64_t)(uint32_t)a << 32) | (uint32_t)b);
        }
    std::sort(keys.begin(), keys.end());
    return (int64_t)(std::unique(keys.begin(), keys.end()) - keys.begin());
}
