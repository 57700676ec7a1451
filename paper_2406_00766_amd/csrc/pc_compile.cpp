// Host side of pc_compile: validation, layering by depth (Sec. 3), grouping of node blocks by
// neighbour count (Sec. 4.3, App. A.1 / Alg. 2) and construction of the forward and backward
// index tensors (Sec. 4.3, App. A.2).  Integer work only.
//
// Canonical form (the paper leaves ordering open; these rules make the tables unique):
//   * node offset of block u is (u+1)*K, offset 0 is the null block; parameter offset of block p
//     is (p+1)*K*K, offset 0 is the all-zero block; padding entries are 0 / 0;
//   * depth(input) = 0, depth(n) = 1 + max depth(children); layers: inputs, then for each depth the
//     product blocks, then the sum blocks;
//   * blocks ascend by id inside a layer and inside a group; a block joins the smallest capacity
//     that holds its count; a row lists its neighbours by ascending node offset;
//   * product layers get the same forward / backward table pair as sum layers.
#include <algorithm>
#include <cstring>
#include <limits>
#include <map>
#include <numeric>

#include "pc_internal.h"

namespace pc {

static thread_local std::string g_last_error;
void set_error(const std::string &msg) { g_last_error = msg; }
pc_status fail(pc_status st, const std::string &msg) { g_last_error = msg; return st; }
const char *last_error_cstr() { return g_last_error.c_str(); }

// Alg. 2 with the following reading of the printed listing: group counts are tried from 1 upwards
// and the first one whose optimal padded size is within sum*(1+tol) wins (the text asks for the
// fewest groups), else max_groups; the back-pointers are followed through decreasing group count;
// the result is the set of distinct capacities; integer arithmetic throughout; on equal cost the
// smallest split index wins.
std::vector<int32_t> partition_groups(const std::vector<int32_t> &counts, int32_t max_groups, int32_t tol_permille)
{
    std::vector<int32_t> caps;
    if (counts.empty()) return caps;
    std::map<int32_t, int64_t> hist;
    for (int32_t v : counts) ++hist[v];
    std::vector<int64_t> val, cum;
    int64_t running = 0, total = 0;
    for (auto &kv : hist) {
        val.push_back(kv.first);
        running += kv.second;
        cum.push_back(running);
        total += (int64_t)kv.first * kv.second;
    }
    const int L = (int)val.size();
    const int G = std::max<int32_t>(1, max_groups);
    const int64_t target = total + (total * (int64_t)tol_permille + 999) / 1000;

    // cost[n][i]: least padded size of the i+1 smallest distinct counts using at most n capacities,
    // the largest of which is val[i]
    std::vector<std::vector<int64_t>> cost(G + 1, std::vector<int64_t>(L, 0));
    std::vector<std::vector<int32_t>> prev(G + 1, std::vector<int32_t>(L, 0));
    for (int i = 0; i < L; ++i) cost[1][i] = val[i] * cum[i];
    int n_sel = 1;
    if (cost[1][L - 1] > target) {
        n_sel = G;
        for (int n = 2; n <= G; ++n) {
            cost[n][0] = val[0] * cum[0];
            prev[n][0] = 0;
            for (int i = 1; i < L; ++i) {
                int64_t best = std::numeric_limits<int64_t>::max();
                int32_t arg = -1;
                for (int j = 0; j < i; ++j) {
                    const int64_t cand = cost[n - 1][j] + val[i] * (cum[i] - cum[j]);
                    if (cand < best) { best = cand; arg = j; }
                }
                cost[n][i] = best;
                prev[n][i] = arg;
            }
            if (cost[n][L - 1] <= target) { n_sel = n; break; }
        }
    }
    int i = L - 1;
    for (int n = n_sel; n >= 1; --n) {
        caps.push_back((int32_t)val[i]);
        if (n > 1) i = prev[n][i];
    }
    std::sort(caps.begin(), caps.end());
    caps.erase(std::unique(caps.begin(), caps.end()), caps.end());
    return caps;
}

namespace {

struct Row {
    int64_t id;                                        // node offset of the row's own block
    std::vector<std::pair<int64_t, int64_t>> nbrs;     // (neighbour node offset, parameter offset)
};

bool fits_i32(int64_t v) { return v >= 0 && v <= std::numeric_limits<int32_t>::max(); }

// rows arrive in ascending id; neighbours get sorted here
pc_status build_groups(std::vector<Row> &rows, int32_t max_groups, int32_t tol_permille,
                       std::vector<GroupTab> &out)
{
    std::vector<int32_t> counts(rows.size());
    for (size_t r = 0; r < rows.size(); ++r) counts[r] = (int32_t)rows[r].nbrs.size();
    const std::vector<int32_t> caps = partition_groups(counts, max_groups, tol_permille);
    out.assign(caps.size(), GroupTab());
    for (size_t g = 0; g < caps.size(); ++g) out[g].width = caps[g];
    for (Row &row : rows) {
        const int32_t cnt = (int32_t)row.nbrs.size();
        const size_t g = std::lower_bound(caps.begin(), caps.end(), cnt) - caps.begin();
        GroupTab &gt = out[g];
        std::sort(row.nbrs.begin(), row.nbrs.end());
        if (!fits_i32(row.id)) return fail(PC_ERR_TOO_LARGE, "node offset exceeds int32");
        gt.ids.push_back((int32_t)row.id);
        gt.aux.push_back(cnt << AUX_COUNT_SHIFT);
        for (int32_t j = 0; j < gt.width; ++j) {
            int64_t a = 0, p = 0;
            if (j < cnt) { a = row.nbrs[j].first; p = row.nbrs[j].second; }
            if (!fits_i32(a) || !fits_i32(p)) return fail(PC_ERR_TOO_LARGE, "table entry exceeds int32");
            gt.nbr.push_back((int32_t)a);
            gt.par.push_back((int32_t)p);
        }
        ++gt.n_rows;
    }
    for (GroupTab &gt : out) {
        std::vector<int32_t> ps;
        for (int32_t p : gt.par) if (p != 0) ps.push_back(p);
        std::sort(ps.begin(), ps.end());
        gt.tied_in_group = std::adjacent_find(ps.begin(), ps.end()) != ps.end();
    }
    return PC_OK;
}

}  // namespace

pc_status compile_host(const pc_dag *d, pc_circuit *c, bool tables_on_host)
{
    if (!d) return fail(PC_ERR_ARG, "dag is NULL");
    if (d->K < 1 || d->n_blocks < 1) return fail(PC_ERR_ARG, "K and n_blocks must be positive");
    if (!d->type || !d->n_real || !d->child_ptr || !d->in_var || !d->in_table)
        return fail(PC_ERR_ARG, "a dag array is NULL");
    const int32_t n = d->n_blocks, K = d->K;
    const int64_t n_edges = d->child_ptr[n];
    if (d->child_ptr[0] != 0 || n_edges < 0) return fail(PC_ERR_ARG, "child_ptr must start at 0");
    if (n_edges > 0 && (!d->child || !d->param_blk)) return fail(PC_ERR_ARG, "child / param_blk is NULL");
    if (d->root_block < 0 || d->root_block >= n || d->type[d->root_block] != KIND_SUM)
        return fail(PC_ERR_ARG, "root_block must name a sum block");
    if (d->n_param_blocks < 0 || d->n_vars < 1 || d->n_cats < 1 || d->n_tables < 1)
        return fail(PC_ERR_ARG, "n_param_blocks / n_vars / n_cats / n_tables out of range");
    if ((int64_t)(n + 1) * K > std::numeric_limits<int32_t>::max())
        return fail(PC_ERR_TOO_LARGE, "node offsets exceed int32");
    if (((int64_t)d->n_param_blocks + 1) * K * K > std::numeric_limits<int32_t>::max())
        return fail(PC_ERR_TOO_LARGE, "parameter offsets exceed int32");
    if ((int64_t)d->n_tables * d->n_cats > std::numeric_limits<int32_t>::max())
        return fail(PC_ERR_TOO_LARGE, "categorical table rows exceed int32");
    if (K > 128) return fail(PC_ERR_ARG, "block sizes above 128 are not supported");

    for (int32_t u = 0; u < n; ++u) {
        if (d->type[u] > KIND_SUM) return fail(PC_ERR_ARG, "unknown block type");
        if (d->n_real[u] < 1 || d->n_real[u] > K) return fail(PC_ERR_ARG, "n_real out of range");
        const int64_t e0 = d->child_ptr[u], e1 = d->child_ptr[u + 1];
        if (e1 < e0) return fail(PC_ERR_ARG, "child_ptr not monotone");
        if (d->type[u] == KIND_INPUT) {
            if (e1 != e0) return fail(PC_ERR_NOT_ALTERNATING, "input block with children");
            if (d->in_var[u] < 0 || d->in_var[u] >= d->n_vars) return fail(PC_ERR_ARG, "in_var out of range");
            if (d->in_table[u] < 0 || d->in_table[u] >= d->n_tables) return fail(PC_ERR_ARG, "in_table out of range");
            continue;
        }
        if (e1 == e0) return fail(PC_ERR_NOT_BLOCK_SPARSE, "inner block without children");
        std::vector<int32_t> seen;
        for (int64_t e = e0; e < e1; ++e) {
            const int32_t ch = d->child[e];
            if (ch < 0 || ch >= n) return fail(PC_ERR_ARG, "child id out of range");
            if (d->type[u] == KIND_SUM) {
                if (d->type[ch] != KIND_PRODUCT) return fail(PC_ERR_NOT_ALTERNATING, "sum block with a non-product child");
                if (d->param_blk[e] < 0 || d->param_blk[e] >= d->n_param_blocks)
                    return fail(PC_ERR_ARG, "param_blk out of range");
            } else if (d->type[ch] == KIND_PRODUCT) {
                return fail(PC_ERR_NOT_ALTERNATING, "product block with a product child");
            }
            seen.push_back(ch);
        }
        std::sort(seen.begin(), seen.end());
        if (std::adjacent_find(seen.begin(), seen.end()) != seen.end())
            return fail(PC_ERR_NOT_BLOCK_SPARSE, "duplicate (parent, child) block pair");
    }

    // Longest-path depth by peeling blocks whose children are all done (also detects cycles).
    std::vector<int32_t> depth(n, 0), pending(n, 0), par_ptr(n + 1, 0);
    for (int64_t e = 0; e < n_edges; ++e) ++par_ptr[d->child[e] + 1];
    for (int32_t u = 0; u < n; ++u) par_ptr[u + 1] += par_ptr[u];
    std::vector<int32_t> par_of(n_edges), fill(par_ptr.begin(), par_ptr.end() - 1);
    for (int32_t u = 0; u < n; ++u)
        for (int64_t e = d->child_ptr[u]; e < d->child_ptr[u + 1]; ++e) par_of[fill[d->child[e]]++] = u;
    std::vector<int32_t> ready;
    for (int32_t u = 0; u < n; ++u) {
        pending[u] = (int32_t)(d->child_ptr[u + 1] - d->child_ptr[u]);
        if (pending[u] == 0) ready.push_back(u);
    }
    int32_t done = 0, max_depth = 0;
    while (!ready.empty()) {
        const int32_t u = ready.back();
        ready.pop_back();
        ++done;
        max_depth = std::max(max_depth, depth[u]);
        for (int32_t k = par_ptr[u]; k < par_ptr[u + 1]; ++k) {
            const int32_t p = par_of[k];
            depth[p] = std::max(depth[p], depth[u] + 1);
            if (--pending[p] == 0) ready.push_back(p);
        }
    }
    if (done != n) return fail(PC_ERR_CYCLE, "the block graph has a cycle");

    if (par_ptr[d->root_block + 1] != par_ptr[d->root_block]) return fail(PC_ERR_ARG, "the root block must not have parents");
    // Product-scratch mode (Sec. 5): a product block is evaluated as late as possible -- in the layer right before the
    // sum blocks that read it (all of one depth) -- so that a product layer is read by the next sum layer only and its
    // values can share one scratch.  Product blocks nobody reads form a last layer of their own.
    c->product_scratch = d->product_scratch != 0;
    if (c->product_scratch) {
        bool orphan = false;
        for (int32_t u = 0; u < n; ++u) {
            if (d->type[u] != KIND_PRODUCT) continue;
            if (par_ptr[u] == par_ptr[u + 1]) { orphan = true; continue; }
            const int32_t ds = depth[par_of[par_ptr[u]]];
            for (int32_t k = par_ptr[u]; k < par_ptr[u + 1]; ++k)
                if (depth[par_of[k]] != ds) return fail(PC_ERR_ARG, "product_scratch: a product block is read by sum blocks of different depths");
            depth[u] = ds;
        }
        if (orphan) {
            for (int32_t u = 0; u < n; ++u)
                if (d->type[u] == KIND_PRODUCT && par_ptr[u] == par_ptr[u + 1]) depth[u] = max_depth + 1;
            max_depth += 1;
        }
    }
    // per block: the smallest and the largest depth among its parents (the last and the first layer of the
    // backward sweep that feed it; all parents of a block are of one kind, so a depth names one layer)
    std::vector<int32_t> last_parent_depth(n, -1), first_parent_depth(n, -1);
    for (int32_t u = 0; u < n; ++u)
        for (int32_t k = par_ptr[u]; k < par_ptr[u + 1]; ++k) {
            const int32_t dp = depth[par_of[k]];
            if (last_parent_depth[u] < 0 || dp < last_parent_depth[u]) last_parent_depth[u] = dp;
            if (dp > first_parent_depth[u]) first_parent_depth[u] = dp;
        }
    // blocks no layer of the backward sweep writes: sum blocks as node offsets (flow and log_nf initialised),
    // other blocks and the null block as ~offset (flow zeroed only)
    c->init_ids.clear();
    c->init_ids.push_back(~0);
    // (product-scratch mode: product blocks nobody reads are the last layer; their window is cleared when the backward
    // sweep reaches it, and their rows do not exist in the flow buffer)
    for (int32_t u = 0; u < n; ++u)
        if (last_parent_depth[u] < 0 && !(c->product_scratch && d->type[u] == KIND_PRODUCT))
            c->init_ids.push_back(d->type[u] == KIND_SUM ? (u + 1) * K : ~((u + 1) * K));

    c->K = K; c->n_blocks = n; c->root_block = d->root_block; c->n_param_blocks = d->n_param_blocks;
    c->n_vars = d->n_vars; c->n_cats = d->n_cats; c->n_tables = d->n_tables;
    c->layers.clear();
    c->an_depth = depth;                                  // kept for the device table builder
    c->an_last_parent_depth = last_parent_depth;
    c->an_first_parent_depth = first_parent_depth;

    // bucket blocks: layer key = 2*depth + (sum ? 1 : 0); inputs are layer 0
    std::vector<std::vector<int32_t>> bucket(2 * (size_t)max_depth + 2);      // max_depth includes the layer of unread products
    for (int32_t u = 0; u < n; ++u) {
        const size_t key = d->type[u] == KIND_INPUT ? 0 : 2 * (size_t)depth[u] + (d->type[u] == KIND_SUM ? 1 : 0);
        bucket[key].push_back(u);
    }
    for (size_t key = 0; key < bucket.size(); ++key) {
        const std::vector<int32_t> &blocks = bucket[key];
        if (blocks.empty()) continue;
        LayerTab layer;
        layer.kind = key == 0 ? KIND_INPUT : d->type[blocks[0]];
        layer.depth = key == 0 ? 0 : depth[blocks[0]];
        for (int32_t u : blocks) layer.blk_ids.push_back((u + 1) * K);
        if (layer.kind == KIND_INPUT) {
            GroupTab g;
            g.n_rows = (int32_t)blocks.size();
            g.width = 1;
            for (int32_t u : blocks) {
                g.ids.push_back((u + 1) * K);
                g.nbr.push_back(d->in_var[u]);
                g.par.push_back(d->in_table[u]);
            }
            std::vector<int32_t> tabs = g.par;                          // a table shared by several blocks: flows collide
            std::sort(tabs.begin(), tabs.end());
            g.tied_in_group = std::adjacent_find(tabs.begin(), tabs.end()) != tabs.end();
            layer.fwd.push_back(std::move(g));
        } else if (tables_on_host) {
            std::vector<Row> fwd_rows;
            std::map<int32_t, Row> by_child;                       // ordered: ascending child block id
            for (int32_t u : blocks) {
                Row r;
                r.id = (int64_t)(u + 1) * K;
                for (int64_t e = d->child_ptr[u]; e < d->child_ptr[u + 1]; ++e) {
                    const int32_t ch = d->child[e];
                    const int64_t p = layer.kind == KIND_SUM ? ((int64_t)d->param_blk[e] + 1) * K * K : 0;
                    r.nbrs.emplace_back((int64_t)(ch + 1) * K, p);
                    Row &br = by_child[ch];
                    br.id = (int64_t)(ch + 1) * K;
                    br.nbrs.emplace_back(r.id, p);
                }
                fwd_rows.push_back(std::move(r));
            }
            std::vector<Row> bwd_rows;
            for (auto &kv : by_child) bwd_rows.push_back(std::move(kv.second));
            pc_status st = build_groups(fwd_rows, d->max_groups, d->tol_permille, layer.fwd);
            if (st != PC_OK) return st;
            st = build_groups(bwd_rows, d->max_groups, d->tol_permille, layer.bwd);
            if (st != PC_OK) return st;
            for (GroupTab &gt : layer.bwd)
                for (size_t i = 0; i < gt.ids.size(); ++i) {
                    const int32_t ch = gt.ids[i] / K - 1;
                    gt.aux[i] |= bwd_row_flags(layer.kind, d->type[ch], layer.depth, last_parent_depth[ch],
                                               first_parent_depth[ch]);
                }
        }
        if (c->product_scratch && layer.kind == KIND_PRODUCT) {
            layer.scr_first_block = blocks.front();
            if (blocks.back() - blocks.front() + 1 != (int32_t)blocks.size())
                return fail(PC_ERR_ARG, "product_scratch: the product blocks of a layer must have consecutive ids (pc_order_for_scratch)");
            c->max_window_blocks = std::max(c->max_window_blocks, (int32_t)blocks.size());
        }
        c->layers.push_back(std::move(layer));
    }
    if (c->product_scratch) {
        // input and sum blocks first, product blocks behind them; every sum layer reads the product layer before it
        c->n_persistent_blocks = 0;
        for (int32_t u = 0; u < n; ++u) if (d->type[u] != KIND_PRODUCT) ++c->n_persistent_blocks;
        for (int32_t u = 0; u < n; ++u)
            if ((d->type[u] == KIND_PRODUCT) != (u >= c->n_persistent_blocks))
                return fail(PC_ERR_ARG, "product_scratch: input and sum blocks must come before the product blocks (pc_order_for_scratch)");
        std::vector<int32_t> layer_of(n, 0);
        for (size_t li = 0; li < c->layers.size(); ++li)
            for (int32_t id : c->layers[li].blk_ids) layer_of[id / K - 1] = (int32_t)li;
        for (size_t li = 0; li < c->layers.size(); ++li) {
            LayerTab &L = c->layers[li];
            if (L.kind != KIND_SUM) continue;
            std::map<int32_t, std::vector<std::pair<int32_t, int32_t>>> users;        // parameter block -> pairs of this layer
            for (int32_t id : L.blk_ids) {
                const int32_t u = id / K - 1;
                for (int64_t e = d->child_ptr[u]; e < d->child_ptr[u + 1]; ++e) {
                    if (layer_of[d->child[e]] != (int32_t)li - 1) return fail(PC_ERR_ARG, "product_scratch: a sum layer must read the product layer before it");
                    users[d->param_blk[e]].emplace_back(id, (d->child[e] + 1) * K);
                }
            }
            L.pf_ptr.assign(1, 0);
            for (auto &kv : users) {
                L.pf_pb.push_back((kv.first + 1) * K * K);
                for (auto &sc : kv.second) { L.pf_sum.push_back(sc.first); L.pf_child.push_back(sc.second); }
                L.pf_ptr.push_back((int32_t)L.pf_sum.size());
            }
        }
    }

    // EM normalisation map.  A sum node's weights span all parameter blocks of its block's edges;
    // tied sum blocks must share that whole list (else the normalisation is ill defined).
    const int32_t P = d->n_param_blocks;
    c->pb_group.assign(P + 1, -1);
    c->pb_rows.assign(P + 1, 0);
    c->pb_cols.assign(P + 1, 0);
    c->group_nch.clear();
    std::vector<std::vector<int32_t>> group_list;
    for (int32_t u = 0; u < n; ++u) {
        if (d->type[u] != KIND_SUM) continue;
        std::vector<int32_t> list;
        int32_t nch = 0;
        for (int64_t e = d->child_ptr[u]; e < d->child_ptr[u + 1]; ++e) {
            list.push_back(d->param_blk[e]);
            nch += d->n_real[d->child[e]];
        }
        std::vector<int32_t> sorted = list;
        std::sort(sorted.begin(), sorted.end());
        if (std::adjacent_find(sorted.begin(), sorted.end()) != sorted.end())
            return fail(PC_ERR_TIE, "a sum block uses one parameter block for two children");
        const int32_t g0 = c->pb_group[list[0] + 1];
        if (g0 < 0) {
            for (int32_t p : list)
                if (c->pb_group[p + 1] >= 0) return fail(PC_ERR_TIE, "sum blocks share only part of their parameter blocks");
            const int32_t g = (int32_t)group_list.size();
            size_t k = 0;
            for (int64_t e = d->child_ptr[u]; e < d->child_ptr[u + 1]; ++e, ++k) {
                c->pb_group[list[k] + 1] = g;
                c->pb_rows[list[k] + 1] = d->n_real[u];
                c->pb_cols[list[k] + 1] = d->n_real[d->child[e]];
            }
            group_list.push_back(list);
            c->group_nch.push_back(nch);
        } else {
            if (group_list[g0] != list) return fail(PC_ERR_TIE, "sum blocks share only part of their parameter blocks");
            size_t k = 0;
            for (int64_t e = d->child_ptr[u]; e < d->child_ptr[u + 1]; ++e, ++k)
                if (c->pb_rows[list[k] + 1] != d->n_real[u] || c->pb_cols[list[k] + 1] != d->n_real[d->child[e]])
                    return fail(PC_ERR_TIE, "tied parameter blocks with different numbers of real nodes");
        }
    }
    c->n_em_groups = (int32_t)group_list.size();

    // Parameter-centric flow tables (App. A.3): every (sum block, child block) pair that uses a parameter
    // block, so that the flows of tied edges are reduced together; pairs in ascending sum-block order.
    std::vector<std::vector<std::pair<int32_t, int32_t>>> users(P);
    for (int32_t u = 0; u < n; ++u) {
        if (d->type[u] != KIND_SUM) continue;
        for (int64_t e = d->child_ptr[u]; e < d->child_ptr[u + 1]; ++e)
            users[d->param_blk[e]].emplace_back((u + 1) * K, (d->child[e] + 1) * K);
    }
    c->pf_pb.clear(); c->pf_ptr.assign(1, 0); c->pf_sum.clear(); c->pf_child.clear();
    for (int32_t p = 0; p < P; ++p) {
        if (users[p].empty()) continue;
        c->pf_pb.push_back((p + 1) * K * K);
        for (auto &sc : users[p]) { c->pf_sum.push_back(sc.first); c->pf_child.push_back(sc.second); }
        c->pf_ptr.push_back((int32_t)c->pf_sum.size());
    }
    return PC_OK;
}

}  // namespace pc
