// Scale-plan generation: host code only (see blitz_plan.h for the model and the steps).
#include <algorithm>
#include <new>
#include <set>
#include <vector>

#include "blitz_layer.h"
#include "blitz_plan.h"

namespace {

struct PNode {
    const bz_plan_node* n;
    double agg;
};

double pair_bw(const PNode& a, const PNode& b, double oversub) {
    const double w = a.agg < b.agg ? a.agg : b.agg;
    return a.n->leaf == b.n->leaf ? w : w / oversub;
}

// stronger node first, then lower id
bool stronger(const PNode* a, const PNode* b) {
    if (a->agg != b->agg) return a->agg > b->agg;
    return a->n->id < b->n->id;
}

struct Chain {
    const PNode* root;
    std::vector<const PNode*> targets;
};

}  // namespace

extern "C" int bz_plan_generate(const bz_plan_node* nodes, int n_nodes, int n_targets, double oversub, int n_layers,
                                double layer_bytes, bz_plan_hop* hops, int max_hops, int* n_hops, int* n_chains,
                                int* interferes) try {
    if (!nodes || !hops || !n_hops || n_nodes < 1 || n_targets < 1 || n_layers < 1) return BZ_EINVAL;
    if (!(oversub >= 1.0) || !(layer_bytes > 0.0)) return BZ_EINVAL;
    std::vector<PNode> all((size_t)n_nodes);
    std::set<int> ids;
    for (int i = 0; i < n_nodes; ++i) {
        const bz_plan_node& v = nodes[i];
        if (v.id < 0 || v.n_gpus < 1 || !(v.gpu_bw > 0.0)) return BZ_EINVAL;
        if (v.role != BZ_PLAN_SOURCE && v.role != BZ_PLAN_SPARE && v.role != BZ_PLAN_OTHER) return BZ_EINVAL;
        if (!ids.insert(v.id).second) return BZ_EINVAL;
        all[i] = PNode{&v, v.n_gpus * v.gpu_bw};
    }
    // step 1: usable sources
    std::vector<const PNode*> src;
    bool any_source = false;
    for (const PNode& p : all)
        if (p.n->role == BZ_PLAN_SOURCE) {
            any_source = true;
            if (!p.n->out_busy) src.push_back(&p);
        }
    if (!any_source) return BZ_ECAPACITY;
    bool forced = false;
    if (src.empty()) {
        forced = true;
        for (const PNode& p : all)
            if (p.n->role == BZ_PLAN_SOURCE) src.push_back(&p);
    }
    std::sort(src.begin(), src.end(), stronger);
    std::set<int> src_leaf;
    for (const PNode* s : src) src_leaf.insert(s->n->leaf);
    // step 2: targets
    std::vector<const PNode*> spare;
    for (const PNode& p : all)
        if (p.n->role == BZ_PLAN_SPARE) spare.push_back(&p);
    if ((int)spare.size() < n_targets || max_hops < n_targets) return BZ_ECAPACITY;
    std::sort(spare.begin(), spare.end(), [&](const PNode* a, const PNode* b) {
        const bool la = src_leaf.count(a->n->leaf) != 0, lb = src_leaf.count(b->n->leaf) != 0;
        if (la != lb) return la;
        return stronger(a, b);
    });
    spare.resize((size_t)n_targets);                     // already strongest-first within each class
    // step 3: one chain per usable source (possibly empty)
    std::vector<Chain> chains;
    for (const PNode* s : src) chains.push_back(Chain{s, {}});
    std::vector<size_t> next_in_leaf;                    // per leaf: which of its roots gets the next target
    std::vector<int> leaf_ids(src_leaf.begin(), src_leaf.end());
    next_in_leaf.assign(leaf_ids.size(), 0);
    for (const PNode* t : spare) {
        const auto it = std::lower_bound(leaf_ids.begin(), leaf_ids.end(), t->n->leaf);
        if (it != leaf_ids.end() && *it == t->n->leaf) {
            // the leaf's roots in strength order are a subsequence of `chains` (sorted the same way)
            std::vector<size_t> roots;
            for (size_t c = 0; c < chains.size(); ++c)
                if (chains[c].root->n->leaf == t->n->leaf) roots.push_back(c);
            size_t& turn = next_in_leaf[(size_t)(it - leaf_ids.begin())];
            chains[roots[turn % roots.size()]].targets.push_back(t);
            ++turn;
        }
    }
    for (const PNode* t : spare) {
        if (src_leaf.count(t->n->leaf)) continue;
        size_t best = 0;
        for (size_t c = 1; c < chains.size(); ++c) {
            const double bc = pair_bw(*chains[c].root, *t, oversub), bb = pair_bw(*chains[best].root, *t, oversub);
            if (bc != bb) {
                if (bc > bb) best = c;
            } else if (chains[c].targets.size() != chains[best].targets.size()) {
                if (chains[c].targets.size() < chains[best].targets.size()) best = c;
            } else if (chains[c].root->n->id < chains[best].root->n->id) {
                best = c;
            }
        }
        chains[best].targets.push_back(t);
    }
    // step 4 + output, chains by root id
    std::sort(chains.begin(), chains.end(), [](const Chain& a, const Chain& b) { return a.root->n->id < b.root->n->id; });
    int h = 0, nc = 0;
    std::vector<double> prev((size_t)n_layers), cur((size_t)n_layers);
    for (Chain& ch : chains) {
        if (ch.targets.empty()) continue;
        std::sort(ch.targets.begin(), ch.targets.end(), [&](const PNode* a, const PNode* b) {
            const double wa = pair_bw(*ch.root, *a, oversub), wb = pair_bw(*ch.root, *b, oversub);
            if (wa != wb) return wa > wb;
            return a->n->id < b->n->id;
        });
        std::fill(prev.begin(), prev.end(), 0.0);
        const PNode* from = ch.root;
        for (size_t k = 0; k < ch.targets.size(); ++k) {
            const PNode* to = ch.targets[k];
            const double bw = pair_bw(*from, *to, oversub);
            double t = 0.0;
            for (int l = 0; l < n_layers; ++l) {
                t = (prev[(size_t)l] > t ? prev[(size_t)l] : t) + layer_bytes / bw;
                cur[(size_t)l] = t;
            }
            hops[h++] = bz_plan_hop{nc, from->n->id, to->n->id, k + 1 == ch.targets.size() ? 1 : 0, bw, t};
            prev.swap(cur);
            from = to;
        }
        ++nc;
    }
    *n_hops = h;
    if (n_chains) *n_chains = nc;
    if (interferes) *interferes = forced ? 1 : 0;
    return BZ_OK;
} catch (const std::bad_alloc&) {
    return BZ_ENOMEM;
} catch (...) {
    return BZ_EINVAL;
}
