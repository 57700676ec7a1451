// pc_collapse: rewrite a block DAG with consecutive sum / sum or product / product blocks into an alternating one
// (footnote to Def. 2).  Host only.  A product block takes over the children of its product children; a sum block takes
// over the children of its sum children with the K x K weight blocks multiplied,
//   sum_j A[i][j] sum_k B[j][k] c_k = sum_k (A B)[i][k] c_k,
// and several paths to one child add up.  The result follows the canonical form stated in pc.h.
#include <algorithm>
#include <cstring>
#include <map>
#include <memory>
#include <new>
#include <string>
#include <vector>

#include "pc_internal.h"

struct pc_collapsed {
    pc_dag dag{};
    std::vector<uint8_t> type;
    std::vector<int32_t> n_real, child, param_blk, in_var, in_table, block_map;
    std::vector<int64_t> child_ptr;
    std::vector<float> theta;
};

namespace {

using Matrix = std::shared_ptr<std::vector<double>>;                    // K x K, row-major

struct SumEdge {
    int32_t child;
    int32_t pb;                                                         // original parameter block, or -1: `m` holds the weights
    Matrix m;
};
struct FlatSum { std::vector<SumEdge> edges; bool changed = false, done = false; };

struct Collapser {
    const pc_dag *d;
    const float *theta;
    int32_t K;
    std::vector<std::vector<int32_t>> prod;                             // flattened children of product blocks
    std::vector<char> prod_done;
    std::vector<FlatSum> sums;
    std::string error;

    Matrix weights(const SumEdge &e) const
    {
        if (e.m) return e.m;
        auto out = std::make_shared<std::vector<double>>((size_t)K * K);
        const float *src = theta + ((int64_t)e.pb + 1) * K * K;
        for (int64_t i = 0; i < (int64_t)K * K; ++i) (*out)[i] = (double)src[i];
        return out;
    }
    Matrix multiply(const Matrix &A, const Matrix &B) const
    {
        auto out = std::make_shared<std::vector<double>>((size_t)K * K, 0.0);
        for (int i = 0; i < K; ++i)
            for (int j = 0; j < K; ++j) {
                const double a = (*A)[(size_t)i * K + j];
                if (a == 0.0) continue;
                for (int k = 0; k < K; ++k) (*out)[(size_t)i * K + k] += a * (*B)[(size_t)j * K + k];
            }
        return out;
    }
};

}  // namespace

using namespace pc;

extern "C" {

pc_status pc_collapse(const pc_dag *dag, const float *theta, pc_collapsed **out)
{
    if (!dag || !theta || !out) return fail(PC_ERR_ARG, "NULL argument");
    const int32_t K = dag->K, n = dag->n_blocks;
    if (K < 1 || K > 128 || n < 1 || !dag->type || !dag->n_real || !dag->child_ptr || !dag->child || !dag->param_blk ||
        !dag->in_var || !dag->in_table || dag->root_block < 0 || dag->root_block >= n)
        return fail(PC_ERR_ARG, "invalid DAG description");
    for (int32_t u = 0; u < n; ++u) {
        if (dag->type[u] > KIND_SUM || dag->child_ptr[u] > dag->child_ptr[u + 1]) return fail(PC_ERR_ARG, "invalid block type or child list");
        for (int64_t e = dag->child_ptr[u]; e < dag->child_ptr[u + 1]; ++e) {
            if (dag->child[e] < 0 || dag->child[e] >= n) return fail(PC_ERR_ARG, "child id out of range");
            if (dag->type[u] == KIND_SUM && (dag->param_blk[e] < 0 || dag->param_blk[e] >= dag->n_param_blocks))
                return fail(PC_ERR_ARG, "parameter block id out of range");
        }
    }
    // children before parents (iterative depth-first post-order); a back edge is a cycle
    std::vector<int32_t> order;
    {
        std::vector<char> state((size_t)n, 0);
        std::vector<int64_t> next((size_t)n, 0);
        std::vector<int32_t> stack;
        for (int32_t s = 0; s < n; ++s) {
            if (state[s]) continue;
            stack.push_back(s); state[s] = 1; next[s] = dag->child_ptr[s];
            while (!stack.empty()) {
                const int32_t u = stack.back();
                if (next[u] < dag->child_ptr[u + 1]) {
                    const int32_t c = dag->child[next[u]++];
                    if (state[c] == 1) return fail(PC_ERR_CYCLE, "the block graph has a cycle");
                    if (state[c] == 0) { state[c] = 1; next[c] = dag->child_ptr[c]; stack.push_back(c); }
                } else {
                    state[u] = 2; order.push_back(u); stack.pop_back();
                }
            }
        }
    }
    Collapser cl{dag, theta, K, std::vector<std::vector<int32_t>>((size_t)n), std::vector<char>((size_t)n, 0),
                 std::vector<FlatSum>((size_t)n), std::string()};
    for (int32_t u : order) {
        if (dag->type[u] == KIND_PRODUCT) {
            std::vector<int32_t> &dst = cl.prod[u];
            for (int64_t e = dag->child_ptr[u]; e < dag->child_ptr[u + 1]; ++e) {
                const int32_t c = dag->child[e];
                if (dag->type[c] == KIND_PRODUCT) dst.insert(dst.end(), cl.prod[c].begin(), cl.prod[c].end());
                else dst.push_back(c);
            }
            std::vector<int32_t> sorted(dst);
            std::sort(sorted.begin(), sorted.end());
            if (std::adjacent_find(sorted.begin(), sorted.end()) != sorted.end())
                return fail(PC_ERR_NOT_BLOCK_SPARSE, "product block " + std::to_string(u) + " reaches a child twice");
        } else if (dag->type[u] == KIND_SUM) {
            FlatSum &fs = cl.sums[u];
            std::map<int32_t, size_t> at;                               // child -> position in fs.edges
            auto add = [&](int32_t child, int32_t pb, const Matrix &m) {
                auto it = at.find(child);
                if (it == at.end()) {
                    at[child] = fs.edges.size();
                    fs.edges.push_back(SumEdge{child, pb, m});
                    return;
                }
                fs.changed = true;                                      // a second path to the same child: the weights add
                SumEdge &old = fs.edges[it->second];
                Matrix a = cl.weights(old), b = cl.weights(SumEdge{child, pb, m});
                auto s2 = std::make_shared<std::vector<double>>(*a);
                for (size_t i = 0; i < s2->size(); ++i) (*s2)[i] += (*b)[i];
                old.pb = -1;
                old.m = s2;
            };
            for (int64_t e = dag->child_ptr[u]; e < dag->child_ptr[u + 1]; ++e) {
                const int32_t c = dag->child[e], pb = dag->param_blk[e];
                if (dag->type[c] == KIND_SUM) {
                    fs.changed = true;
                    const Matrix A = cl.weights(SumEdge{c, pb, nullptr});
                    for (const SumEdge &ce : cl.sums[c].edges) add(ce.child, -1, cl.multiply(A, cl.weights(ce)));
                } else {
                    add(c, pb, nullptr);
                }
            }
        }
    }
    // blocks reachable from the root through the new edges, renumbered in ascending order of their old ids
    std::vector<char> reach((size_t)n, 0);
    {
        std::vector<int32_t> stack{dag->root_block};
        while (!stack.empty()) {
            const int32_t u = stack.back(); stack.pop_back();
            if (reach[u]) continue;
            reach[u] = 1;
            if (dag->type[u] == KIND_PRODUCT) for (int32_t c : cl.prod[u]) stack.push_back(c);
            else if (dag->type[u] == KIND_SUM) for (const SumEdge &e : cl.sums[u].edges) stack.push_back(e.child);
        }
    }
    pc_collapsed *r = new (std::nothrow) pc_collapsed();
    if (!r) return fail(PC_ERR_ARG, "out of host memory");
    r->block_map.assign((size_t)n, -1);
    int32_t n_new = 0;
    for (int32_t u = 0; u < n; ++u) if (reach[u]) r->block_map[u] = n_new++;
    std::map<int32_t, int32_t> pb_new;                                  // original parameter block -> new id (first use)
    std::vector<Matrix> mats;
    std::vector<int32_t> mats_src;                                      // original block to copy, or -1: mats[i]
    r->child_ptr.push_back(0);
    for (int32_t u = 0; u < n; ++u) {
        if (!reach[u]) continue;
        r->type.push_back(dag->type[u]);
        r->n_real.push_back(dag->n_real[u]);
        r->in_var.push_back(dag->in_var[u]);
        r->in_table.push_back(dag->in_table[u]);
        if (dag->type[u] == KIND_PRODUCT) {
            for (int32_t c : cl.prod[u]) { r->child.push_back(r->block_map[c]); r->param_blk.push_back(-1); }
        } else if (dag->type[u] == KIND_SUM) {
            const FlatSum &fs = cl.sums[u];
            for (const SumEdge &e : fs.edges) {
                r->child.push_back(r->block_map[e.child]);
                if (!fs.changed && e.pb >= 0) {                         // untouched block: keeps its parameter blocks and ties
                    auto it = pb_new.find(e.pb);
                    if (it == pb_new.end()) {
                        it = pb_new.emplace(e.pb, (int32_t)mats.size()).first;
                        mats.push_back(nullptr); mats_src.push_back(e.pb);
                    }
                    r->param_blk.push_back(it->second);
                } else {
                    r->param_blk.push_back((int32_t)mats.size());
                    mats.push_back(e.m); mats_src.push_back(e.m ? -1 : e.pb);
                }
            }
        }
        r->child_ptr.push_back((int64_t)r->child.size());
    }
    r->theta.assign(((size_t)mats.size() + 1) * K * K, 0.0f);
    for (size_t p = 0; p < mats.size(); ++p) {
        float *dst = r->theta.data() + (p + 1) * K * K;
        if (mats_src[p] >= 0) std::memcpy(dst, theta + ((int64_t)mats_src[p] + 1) * K * K, sizeof(float) * K * K);
        else for (int64_t i = 0; i < (int64_t)K * K; ++i) dst[i] = (float)(*mats[p])[i];
    }
    r->dag = *dag;
    r->dag.n_blocks = n_new;
    r->dag.root_block = r->block_map[dag->root_block];
    r->dag.type = r->type.data(); r->dag.n_real = r->n_real.data();
    r->dag.child_ptr = r->child_ptr.data(); r->dag.child = r->child.data(); r->dag.param_blk = r->param_blk.data();
    r->dag.n_param_blocks = (int32_t)mats.size();
    r->dag.in_var = r->in_var.data(); r->dag.in_table = r->in_table.data();
    *out = r;
    return PC_OK;
}

// Block order for the product-scratch mode of pc_compile: input and sum blocks first (their relative order kept), then
// the product blocks grouped by the depth of the sum blocks that read them (groups ascending, order kept inside).
pc_status pc_order_for_scratch(const pc_dag *dag, pc_collapsed **out)
{
    if (!dag || !out) return fail(PC_ERR_ARG, "NULL argument");
    const int32_t n = dag->n_blocks;
    if (dag->K < 1 || n < 1 || !dag->type || !dag->n_real || !dag->child_ptr || !dag->in_var || !dag->in_table ||
        (dag->child_ptr[n] > 0 && (!dag->child || !dag->param_blk)))
        return fail(PC_ERR_ARG, "invalid DAG description");
    for (int64_t e = 0; e < dag->child_ptr[n]; ++e)
        if (dag->child[e] < 0 || dag->child[e] >= n) return fail(PC_ERR_ARG, "child id out of range");
    // longest-path depth, children before parents
    std::vector<int32_t> depth((size_t)n, 0), pending((size_t)n, 0), order;
    std::vector<std::vector<int32_t>> parents((size_t)n);
    for (int32_t u = 0; u < n; ++u) {
        pending[u] = (int32_t)(dag->child_ptr[u + 1] - dag->child_ptr[u]);
        for (int64_t e = dag->child_ptr[u]; e < dag->child_ptr[u + 1]; ++e) parents[dag->child[e]].push_back(u);
        if (pending[u] == 0) order.push_back(u);
    }
    for (size_t i = 0; i < order.size(); ++i) {
        const int32_t u = order[i];
        for (int32_t p : parents[u]) {
            depth[p] = std::max(depth[p], depth[u] + 1);
            if (--pending[p] == 0) order.push_back(p);
        }
    }
    if ((int32_t)order.size() != n) return fail(PC_ERR_CYCLE, "the block graph has a cycle");
    // product blocks: one copy per depth of the sum blocks that read them (a copy is read by sum blocks of one depth only
    // and can be evaluated right before them); key = that depth, unread blocks last
    const int64_t kUnread = (int64_t)1 << 40;
    std::vector<std::pair<int64_t, int32_t>> keyed;                     // (group key, old id)
    for (int32_t u = 0; u < n; ++u) {
        if (dag->type[u] != KIND_PRODUCT) { keyed.emplace_back(-1, u); continue; }
        std::vector<int32_t> ds;
        for (int32_t p : parents[u]) ds.push_back(depth[p]);
        std::sort(ds.begin(), ds.end());
        ds.erase(std::unique(ds.begin(), ds.end()), ds.end());
        if (ds.empty()) keyed.emplace_back(kUnread, u);
        for (int32_t dd : ds) keyed.emplace_back(dd, u);
    }
    std::stable_sort(keyed.begin(), keyed.end(), [](const std::pair<int64_t, int32_t> &a, const std::pair<int64_t, int32_t> &b) { return a.first < b.first; });
    const int32_t n_new = (int32_t)keyed.size();
    pc_collapsed *r = new (std::nothrow) pc_collapsed();
    if (!r) return fail(PC_ERR_ARG, "out of host memory");
    r->block_map.assign((size_t)n, -1);
    std::map<std::pair<int32_t, int64_t>, int32_t> copy_of;             // (old product id, reader depth) -> new id
    for (int32_t i = 0; i < n_new; ++i) {
        if (r->block_map[keyed[i].second] < 0) r->block_map[keyed[i].second] = i;     // a product block: its first copy
        copy_of[{keyed[i].second, keyed[i].first}] = i;
    }
    r->child_ptr.push_back(0);
    for (int32_t i = 0; i < n_new; ++i) {
        const int32_t u = keyed[i].second;
        r->type.push_back(dag->type[u]); r->n_real.push_back(dag->n_real[u]);
        r->in_var.push_back(dag->in_var[u]); r->in_table.push_back(dag->in_table[u]);
        for (int64_t e = dag->child_ptr[u]; e < dag->child_ptr[u + 1]; ++e) {
            const int32_t ch = dag->child[e];
            // a sum block reads the copy made for its depth; everything else keeps its one image
            r->child.push_back(dag->type[u] == KIND_SUM && dag->type[ch] == KIND_PRODUCT ? copy_of[{ch, (int64_t)depth[u]}] : r->block_map[ch]);
            r->param_blk.push_back(dag->param_blk[e]);
        }
        r->child_ptr.push_back((int64_t)r->child.size());
    }
    r->dag = *dag;
    r->dag.n_blocks = n_new;
    r->dag.root_block = r->block_map[dag->root_block];
    r->dag.type = r->type.data(); r->dag.n_real = r->n_real.data();
    r->dag.child_ptr = r->child_ptr.data(); r->dag.child = r->child.data(); r->dag.param_blk = r->param_blk.data();
    r->dag.in_var = r->in_var.data(); r->dag.in_table = r->in_table.data();
    r->dag.product_scratch = 1;
    *out = r;
    return PC_OK;
}

const pc_dag *pc_collapsed_dag(const pc_collapsed *r) { return r ? &r->dag : nullptr; }

const float *pc_collapsed_theta(const pc_collapsed *r, int64_t *len)
{
    if (!r) return nullptr;
    if (len) *len = (int64_t)r->theta.size();
    return r->theta.data();
}

const int32_t *pc_collapsed_block_map(const pc_collapsed *r) { return r ? r->block_map.data() : nullptr; }

void pc_collapsed_destroy(pc_collapsed *r) { delete r; }

}  // extern "C"
