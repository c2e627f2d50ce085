// Topology front-end, host only (paper Section 3.2: homogeneous, ring, symmetric and asymmetric
// tree topologies in nested-list notation; Section 4.2: the min-max exchange problem, its
// closed-form solution without latency, and the merge of asymmetric trees).  These functions
// produce the tables that tamoe_topo_pattern consumes; nothing here touches the GPU.
#include <algorithm>
#include <cmath>
#include <cstdint>
#include <cstring>
#include <numeric>
#include <string>
#include <vector>

#include "internal.h"

namespace tamoe {
namespace {

// ---- trees -------------------------------------------------------------------------------------
struct Node {
    int devices = 0;          // > 0: a switch with that many devices and no sub-switches
    int first_device = 0;     // device switch: number of its first device in the tree as given
    std::vector<Node> kids;   // otherwise: the elements of the list
};

struct Parser {
    const char* p;
    bool ok = true;
    int devices_seen = 0;
    void blanks() {
        while (*p == ' ' || *p == '\t') ++p;
    }
    Node element() {
        Node n;
        blanks();
        if (*p >= '0' && *p <= '9') {
            long v = 0;
            while (*p >= '0' && *p <= '9') {
                v = v * 10 + (*p - '0');
                if (v > 65536) ok = false, v = 65536;
                ++p;
            }
            if (v <= 0) ok = false;
            n.devices = (int)v;
            n.first_device = devices_seen;
            devices_seen += (int)v;
            return n;
        }
        if (*p != '[') {
            ok = false;
            return n;
        }
        ++p;
        while (ok) {
            n.kids.push_back(element());
            blanks();
            if (*p == ',') {
                ++p;
            } else if (*p == ']') {
                ++p;
                break;
            } else {
                ok = false;
            }
        }
        return n;
    }
};

int height(const Node& n) {
    if (n.devices > 0) return 1;
    int h = 0;
    for (const Node& c : n.kids) h = std::max(h, height(c));
    return h + 1;
}

int device_count(const Node& n) {
    if (n.devices > 0) return n.devices;
    int total = 0;
    for (const Node& c : n.kids) total += device_count(c);
    return total;
}

// Merge at one list (Section 4.2, last paragraph; the paper shows [[2,2],[2]] -> [[2,2,2]] and names
// the aim, a symmetric tree).  The elements with the most members are the full sub-trees, the smaller
// ones the separate nodes.  Every separate node, left to right, empties itself into a full sub-tree
// of its own height: the least loaded one (members received so far), the nearest of those, the left
// one at equal distance.  The sizes are taken once, before anything moves.
void absorb_separate_nodes(Node& n) {
    const size_t cnt = n.kids.size();
    size_t largest = 0;
    for (const Node& c : n.kids) {
        if (c.devices > 0) return;        // device switches are never merged
        largest = std::max(largest, c.kids.size());
    }
    std::vector<size_t> size(cnt), received(cnt, 0);
    std::vector<int> h(cnt), into(cnt, -1);
    for (size_t i = 0; i < cnt; ++i) {
        size[i] = n.kids[i].kids.size();
        h[i] = height(n.kids[i]);
    }
    bool moved = false;
    for (size_t i = 0; i < cnt; ++i) {
        if (size[i] == largest) continue;
        // lightest load among the full sub-trees this node may join
        size_t lightest = SIZE_MAX;
        for (size_t j = 0; j < cnt; ++j)
            if (size[j] == largest && h[j] == h[i]) lightest = std::min(lightest, received[j]);
        if (lightest == SIZE_MAX) continue;  // no full sub-tree of this height: the node stays
        // walk outwards from the node, left before right, to the first one that carries that load
        for (size_t dist = 1; dist < cnt && into[i] < 0; ++dist) {
            const size_t l = i - dist, r = i + dist;   // l wraps around below zero and then fails l < cnt
            if (l < cnt && size[l] == largest && h[l] == h[i] && received[l] == lightest)
                into[i] = (int)l;
            else if (r < cnt && size[r] == largest && h[r] == h[i] && received[r] == lightest)
                into[i] = (int)r;
        }
        received[(size_t)into[i]] += size[i];
        moved = true;
    }
    if (!moved) return;
    // members move in the order the separate nodes were visited; the emptied nodes disappear
    for (size_t i = 0; i < cnt; ++i) {
        if (into[i] < 0) continue;
        Node& dst = n.kids[(size_t)into[i]];
        for (Node& m : n.kids[i].kids) dst.kids.push_back(std::move(m));
        n.kids[i].kids.clear();
    }
    std::vector<Node> rest;
    for (size_t i = 0; i < cnt; ++i)
        if (into[i] < 0) rest.push_back(std::move(n.kids[i]));
    n.kids = std::move(rest);
}

// One pass from the leaves up; a list that has taken members in is not looked at again.
void merge(Node& n) {
    if (n.devices > 0) return;
    for (Node& c : n.kids) merge(c);
    absorb_separate_nodes(n);
}

// chain[dev] = (number, height) of the switches above device `dev` (numbered as in the tree as
// given), lowest first; order: the device numbers from left to right in the tree as it stands
void collect_chains(const Node& n, int& next_id, std::vector<std::pair<int, int>>& above,
                    std::vector<std::vector<std::pair<int, int>>>& chain, std::vector<int>& order) {
    above.push_back({next_id++, height(n)});
    if (n.devices > 0) {
        for (int q = 0; q < n.devices; ++q) {
            chain[(size_t)(n.first_device + q)].assign(above.rbegin(), above.rend());
            order.push_back(n.first_device + q);
        }
    } else {
        for (const Node& c : n.kids) collect_chains(c, next_id, above, chain, order);
    }
    above.pop_back();
}

void print(const Node& n, std::string& out) {
    if (n.devices > 0) {
        out += std::to_string(n.devices);
        return;
    }
    out += '[';
    for (size_t i = 0; i < n.kids.size(); ++i) {
        if (i) out += ',';
        print(n.kids[i], out);
    }
    out += ']';
}

}  // namespace
}  // namespace tamoe

using namespace tamoe;

extern "C" int tamoe_tree_levels(const char* tree, int merge_asymmetric, int max_P, int32_t* level, int* P_out,
                                 char* tree_out, size_t tree_out_len, int32_t* device_order) {
    const char* fn = "tamoe_tree_levels";
    clear_error();
    if (tree == nullptr || level == nullptr || P_out == nullptr) return fail(TAMOE_INVALID_ARG, "%s: NULL pointer", fn);
    if (max_P <= 0) return fail(TAMOE_INVALID_ARG, "%s: max_P = %d must be positive", fn, max_P);
    Parser ps{tree};
    Node root = ps.element();
    ps.blanks();
    if (!ps.ok || *ps.p != '\0')
        return fail(TAMOE_INVALID_ARG, "%s: cannot read \"%s\" as a nested list of positive device counts (at offset %d)",
                    fn, tree, (int)(ps.p - tree));
    if (merge_asymmetric) merge(root);
    const int P = device_count(root);
    if (P > max_P) return fail(TAMOE_INVALID_ARG, "%s: the tree has %d devices, the table has room for %d", fn, P, max_P);
    std::vector<std::vector<std::pair<int, int>>> chain((size_t)P);
    std::vector<std::pair<int, int>> above;
    std::vector<int> order;
    int next_id = 0;
    collect_chains(root, next_id, above, chain, order);
    if (device_order != nullptr)
        for (int i = 0; i < P; ++i) device_order[i] = order[(size_t)i];
    for (int i = 0; i < P; ++i) {
        for (int j = 0; j < P; ++j) {
            int lv = 0;
            if (i != j) {
                // lowest switch of i's chain that is also above j
                for (const auto& a : chain[i]) {
                    bool shared = false;
                    for (const auto& b : chain[j]) shared |= a.first == b.first;
                    if (shared) {
                        lv = a.second;
                        break;
                    }
                }
            }
            level[(size_t)i * P + j] = lv;
        }
    }
    *P_out = P;
    if (tree_out != nullptr && tree_out_len > 0) {
        std::string text;
        print(root, text);
        if (text.size() + 1 > tree_out_len)
            return fail(TAMOE_INVALID_ARG, "%s: tree_out has room for %zu characters, %zu needed", fn, tree_out_len,
                        text.size() + 1);
        std::memcpy(tree_out, text.c_str(), text.size() + 1);
    }
    return TAMOE_OK;
}

extern "C" int tamoe_ring_table(const double* beta_link, const double* alpha_link, int P, double self_beta,
                                double self_alpha, double* beta, double* alpha, int32_t* level) {
    const char* fn = "tamoe_ring_table";
    clear_error();
    if (beta_link == nullptr || beta == nullptr || level == nullptr) return fail(TAMOE_INVALID_ARG, "%s: NULL pointer", fn);
    if (P < 2) return fail(TAMOE_INVALID_ARG, "%s: a ring needs at least 2 devices, P = %d", fn, P);
    for (int q = 0; q < P; ++q) {
        if (!(beta_link[q] > 0.0) || !std::isfinite(beta_link[q]))
            return fail(TAMOE_INVALID_ARG, "%s: beta_link[%d] = %g is not a positive finite number", fn, q, beta_link[q]);
        if (alpha_link != nullptr && (!(alpha_link[q] >= 0.0) || !std::isfinite(alpha_link[q])))
            return fail(TAMOE_INVALID_ARG, "%s: alpha_link[%d] = %g is not a finite number >= 0", fn, q, alpha_link[q]);
    }
    if (!(self_beta > 0.0) || !std::isfinite(self_beta) || !(self_alpha >= 0.0) || !std::isfinite(self_alpha))
        return fail(TAMOE_INVALID_ARG, "%s: self_beta must be positive, self_alpha non-negative, both finite", fn);
    // walking upwards from i: after h hops the bottleneck and latency of the ascending arc i -> i+h;
    // the descending arc to the same device is the ascending arc from it back to i
    std::vector<double> up_b((size_t)P * P), up_a((size_t)P * P, 0.0);
    for (int i = 0; i < P; ++i) {
        double worst = 0.0, lat = 0.0;
        for (int h = 1; h < P; ++h) {
            const int link = (i + h - 1) % P;
            worst = std::max(worst, beta_link[link]);
            lat += alpha_link != nullptr ? alpha_link[link] : 0.0;
            up_b[(size_t)i * P + (i + h) % P] = worst;
            up_a[(size_t)i * P + (i + h) % P] = lat;
        }
    }
    for (int i = 0; i < P; ++i) {
        for (int j = 0; j < P; ++j) {
            const size_t o = (size_t)i * P + j;
            if (i == j) {
                beta[o] = self_beta;
                if (alpha) alpha[o] = self_alpha;
                level[o] = 0;
                continue;
            }
            const int h_up = (j - i + P) % P, h_down = P - h_up;
            const double b_up = up_b[o], b_down = up_b[(size_t)j * P + i];
            const bool ascending = b_up < b_down || (b_up == b_down && h_up <= h_down);
            beta[o] = ascending ? b_up : b_down;
            if (alpha) alpha[o] = ascending ? up_a[o] : up_a[(size_t)j * P + i];
            level[o] = ascending ? h_up : h_down;
        }
    }
    return TAMOE_OK;
}

// The optimum loads a set of links up to a common finishing time T and leaves the others (latency
// >= T) idle.  Links sorted by latency: the loaded set is a prefix; with m links loaded,
// T_m = (k*S + sum a_j / g_j) / (sum 1 / g_j), g_j = beta_j * bytes, and the right m is the one
// whose T_m lies above its own latencies and not above the next one.
extern "C" int tamoe_minmax_pattern(const double* alpha_row, const double* beta_row, int P, int N, int k, int64_t S,
                                    double bytes_per_row, double* c_hat, double* t_comm) {
    const char* fn = "tamoe_minmax_pattern";
    clear_error();
    if (beta_row == nullptr || c_hat == nullptr) return fail(TAMOE_INVALID_ARG, "%s: NULL pointer", fn);
    if (N <= 0 || P <= 0 || k <= 0 || S <= 0)
        return fail(TAMOE_INVALID_ARG, "%s: N = %d, P = %d, k = %d, S = %lld must all be positive", fn, N, P, k,
                    (long long)S);
    if (N % P != 0) return fail(TAMOE_INVALID_ARG, "%s: N = %d is not a multiple of P = %d", fn, N, P);
    if (!(bytes_per_row > 0.0) || !std::isfinite(bytes_per_row))
        return fail(TAMOE_INVALID_ARG, "%s: bytes_per_row must be positive and finite", fn);
    for (int j = 0; j < P; ++j) {
        if (!(beta_row[j] > 0.0) || !std::isfinite(beta_row[j]))
            return fail(TAMOE_INVALID_ARG, "%s: beta_row[%d] = %g is not a positive finite number", fn, j, beta_row[j]);
        if (alpha_row != nullptr && (!(alpha_row[j] >= 0.0) || !std::isfinite(alpha_row[j])))
            return fail(TAMOE_INVALID_ARG, "%s: alpha_row[%d] = %g is not a finite number >= 0", fn, j, alpha_row[j]);
    }
    std::vector<int> order(P);
    std::iota(order.begin(), order.end(), 0);
    auto lat = [&](int j) { return alpha_row != nullptr ? alpha_row[j] : 0.0; };
    std::stable_sort(order.begin(), order.end(), [&](int a, int b) { return lat(a) < lat(b); });
    const double rows = (double)k * (double)S;
    double num = rows, den = 0.0, T = 0.0;
    for (int m = 0; m < P; ++m) {
        const int j = order[m];
        const double g = beta_row[j] * bytes_per_row;
        num += lat(j) / g;
        den += 1.0 / g;
        T = num / den;
        if (m + 1 == P || T <= lat(order[m + 1])) break;
    }
    const int E = N / P;
    for (int e = 0; e < N; ++e) {
        const int j = e / E;
        const double v = T > lat(j) ? (T - lat(j)) / (beta_row[j] * bytes_per_row) : 0.0;
        c_hat[e] = v / (double)E;
    }
    if (t_comm != nullptr) *t_comm = T;
    return TAMOE_OK;
}
