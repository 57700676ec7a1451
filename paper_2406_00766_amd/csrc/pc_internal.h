// Internal structures of libpc (not part of the C ABI).
#pragma once
#include <cstdint>
#include <string>
#include <vector>

#include "pc.h"

namespace pc {

enum : int { KIND_INPUT = 0, KIND_PRODUCT = 1, KIND_SUM = 2 };

// Flags of one row (= one child block) of a layer's backward tables.
//   BWD_FINAL  product layer, sum child: this is the last layer that adds to the child's flow, which is complete
//              afterwards (log_nf of Alg. 3 / 4 is produced here)
//   BWD_FIRST  this is the first layer of the backward sweep that adds to the child's flow: the kernel stores
//              instead of accumulating, so the flow buffer needs no clearing (the '=' of Alg. 4's last line)
// The per-row word of a group (GroupTab::aux) holds these flags in its low byte and the row's number of real
// neighbours (the rest of the row is padding) from bit AUX_COUNT_SHIFT up.
enum : int32_t { BWD_FINAL = 1, BWD_FIRST = 2, AUX_COUNT_SHIFT = 8 };
inline int32_t bwd_row_flags(int layer_kind, int child_kind, int32_t layer_depth, int32_t last_parent_depth,
                             int32_t first_parent_depth)
{
    int32_t f = 0;
    if (layer_kind == KIND_PRODUCT && child_kind == KIND_SUM && last_parent_depth == layer_depth) f |= BWD_FINAL;
    if (first_parent_depth == layer_depth) f |= BWD_FIRST;
    return f;
}

// One group of a layer: rows padded to a common width (Sec. 4.3).
struct GroupTab {
    int32_t n_rows = 0, width = 0;
    std::vector<int32_t> ids, nbr, par;              // host copies
    std::vector<int32_t> aux;                        // per row: neighbour count << AUX_COUNT_SHIFT | BWD_* flags
    int32_t *d_ids = nullptr, *d_nbr = nullptr, *d_par = nullptr, *d_aux = nullptr;
    bool tied_in_group = false;                       // a parameter block occurs twice: flows need atomics
};

struct LayerTab {
    int32_t kind = 0, depth = 0;
    std::vector<GroupTab> fwd, bwd;
    std::vector<int32_t> blk_ids;                     // node offsets of all blocks of the layer, ascending
    int32_t *d_blk_ids = nullptr;
    // product-scratch mode (Sec. 5): a product layer's blocks are one contiguous id range that lives in the scratch
    // window; a sum layer has its own parameter-flow table (its products are gone when the sweep moves on)
    int32_t scr_first_block = -1;                     // product layers: id of the first block of the layer
    std::vector<int32_t> pf_pb, pf_ptr, pf_sum, pf_child;
    int32_t *d_pf_pb = nullptr, *d_pf_ptr = nullptr, *d_pf_sum = nullptr, *d_pf_child = nullptr;
};

}  // namespace pc

struct pc_circuit {
    int32_t K = 0, n_blocks = 0, root_block = 0, n_param_blocks = 0;
    int32_t n_vars = 0, n_cats = 0, n_tables = 0;
    std::vector<pc::LayerTab> layers;

    // EM normalisation: parameter block -> (row group, real rows, real cols); row group -> child count
    int32_t n_em_groups = 0;
    std::vector<int32_t> pb_group, pb_rows, pb_cols, group_nch;
    int32_t *d_pb_group = nullptr, *d_pb_rows = nullptr, *d_pb_cols = nullptr, *d_group_nch = nullptr;
    float *d_zrow = nullptr;                          // [n_em_groups * K] row sums of flows
    float *d_ztab = nullptr;                          // [n_tables * K] column sums of table flows

    // parameter-centric flow tables: parameter block offset -> CSR list of (sum block, child block) node offsets
    std::vector<int32_t> pf_pb, pf_ptr, pf_sum, pf_child;
    int32_t *d_pf_pb = nullptr, *d_pf_ptr = nullptr, *d_pf_sum = nullptr, *d_pf_child = nullptr;

    // blocks without parents, which no layer of the backward sweep writes.  Sum blocks (the root among them) as
    // node offsets; other blocks and the null block as ~offset
    std::vector<int32_t> init_ids;
    int32_t *d_init_ids = nullptr;

    // product-scratch mode: product log-probabilities live in a window of max_window_blocks blocks behind the
    // n_persistent_blocks input and sum blocks
    bool product_scratch = false;
    int32_t n_persistent_blocks = 0, max_window_blocks = 0;

    void *d_arena = nullptr;                          // one device allocation behind every d_* above
    size_t arena_bytes = 0;
    bool on_device = false;

    // analysis results handed from compile_host to build_tables_device (cleared afterwards)
    std::vector<int32_t> an_depth, an_last_parent_depth, an_first_parent_depth;

    // optional per-kernel-class timing (pc_profile_*)
    void *profiler = nullptr;                         // pc::Profiler*, owned
    void *plan = nullptr;                             // launch plan (group sets per layer), owned
    int64_t prof_launches[16] = {0};
    double prof_ms[16] = {0.0};

    // state linking pc_backward to the preceding pc_forward
    const void *fw_workspace = nullptr;
    const void *fw_theta = nullptr, *fw_tables = nullptr, *fw_x = nullptr, *fw_mask = nullptr;
    int32_t fw_B = -1;
};

namespace pc {

void set_error(const std::string &msg);
pc_status fail(pc_status st, const std::string &msg);

// Host part of compilation: validation, layering, grouping, table construction, EM maps.
// tables_on_host = false leaves the sum / product layer tables to build_tables_device.
pc_status compile_host(const pc_dag *dag, pc_circuit *c, bool tables_on_host);
// Device part of compilation: transposes the block graph, sorts neighbour lists and fills every forward and
// backward table with HIP kernels; allocates the handle's device arena and uploads the remaining metadata.
pc_status build_tables_device(const pc_dag *dag, pc_circuit *c, void *stream);
// Alg. 2 (App. A.1): ascending group capacities for the given neighbour counts.
std::vector<int32_t> partition_groups(const std::vector<int32_t> &counts, int32_t max_groups, int32_t tol_permille);

}  // namespace pc
