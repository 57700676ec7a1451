// Launchers of the HIP kernels (internal).
#pragma once
#include <hip/hip_runtime.h>

#include <cstdint>
#include <vector>

namespace pc {

struct GroupDev {            // device view of one table group
    int32_t n_rows, width;
    const int32_t *ids, *nbr, *par;
    bool tied;
    const int32_t *aux;      // per row: real neighbours << 8 | bit 0 flow final after this layer | bit 1 first layer to write it
};

// Table groups of one layer that one launch covers (a kernel argument, passed by value).  Rows of the launch are
// numbered through the groups; group g holds rows first[g] .. first[g + 1].
constexpr int PC_MAX_SET = 8;
struct GroupSet {
    int32_t n;
    int32_t first[PC_MAX_SET + 1];
    int32_t width[PC_MAX_SET];
    const int32_t *ids[PC_MAX_SET], *nbr[PC_MAX_SET], *par[PC_MAX_SET], *aux[PC_MAX_SET];
};

struct ParamFlowDev {        // parameter blocks with the (sum block, child block) pairs that use them
    int32_t n_pb;
    const int32_t *pb, *ptr, *sum, *child;
    int64_t n_pairs;         // entries of sum / child
};

struct EmDev {
    int32_t n_groups;
    const int32_t *pb_group, *pb_rows, *pb_cols, *group_nch;
    float *zrow, *ztab;
};

void set_force_generic(bool on);

// Optional per-launch timing: when a profiler is installed, every launcher brackets its kernel with two
// HIP events on the launch stream; totals per kernel class are summed when the profile is read.
enum KernelClass : int {
    KC_MISC = 0, KC_INPUT_FWD, KC_PROD_FWD, KC_SUM_FWD, KC_LOGNF, KC_SUM_BWD_CHILD, KC_SUM_BWD_PARAM, KC_PROD_BWD,
    KC_INPUT_BWD, KC_EM, KC_SPLIT, KC_COUNT
};
struct Profiler {
    struct Rec { int cls; hipEvent_t a, b; };
    std::vector<Rec> recs;
    int64_t bf16_launches[16] = {0};                    // per class: launches that ran on the bf16 matrix cores
    std::vector<hipEvent_t> pool;
    hipEvent_t get();
    void collect(int64_t *launches, double *ms);      // waits for the recorded events, adds to the totals
    ~Profiler();
};
void set_profiler(Profiler *p);                        // nullptr switches timing off

void launch_fill(float *p, int64_t n, float v, hipStream_t s);
void launch_prepare_x(const int32_t *x, const uint8_t *mask, int32_t B, int32_t D, int64_t Bs, int32_t n_cats,
                      int32_t *xT, hipStream_t s);
void launch_readout(const float *l, const float *R, int64_t root_row, int64_t root_blk, int64_t Bs, int32_t B, float *ll,
                    hipStream_t s);
void launch_init_flows(const float *l, float *F, float *N, float *nfmax, const int32_t *blk_ids, int32_t n_blk,
                       int32_t root_id, int32_t K, int64_t Bs, int32_t B, hipStream_t s);
void launch_input_fwd(const float *tables, const int32_t *xT, const GroupDev &g, int32_t K, int32_t n_cats, int64_t Bs,
                      float *l, hipStream_t s);
void launch_input_bwd(const float *F, const int32_t *xT, const GroupDev &g, int32_t K, int32_t n_cats, int64_t Bs,
                      float *table_flow, hipStream_t s);
// The four layer launchers take all table groups of the layer, packed into sets by make_group_sets: the groups of a
// layer are independent of one another, and one launch covers a whole set.
std::vector<GroupSet> make_group_sets(const std::vector<GroupDev> &groups);
// Ph / Pl non-null: the kernel also writes the bf16 value planes of its rows (see launch_split_p)
// l: base the children are read from, lout: base the products are written to (the same, except in the product-scratch mode)
void launch_prod_fwd(const float *l, float *lout, float *R, const std::vector<GroupSet> &sets, int32_t K, int64_t Bs, void *Ph, void *Pl,
                     hipStream_t s);
// Fpar: base the parents' flows are read from (= F, except in the product-scratch mode)
void launch_prod_bwd(const float *l, float *F, const float *Fpar, float *N, float *nfmax, const std::vector<GroupSet> &sets, int32_t K,
                     int64_t Bs, void *Ph, void *Pl, hipStream_t s);
// lch: base the product children are read from; l: base of the sum rows written
void launch_sum_fwd(const float *theta, const float *lch, float *l, float *R, const std::vector<GroupSet> &sets, int32_t K,
                    int64_t Bs, hipStream_t s);
void launch_sum_bwd_child(const float *theta, const float *l, const float *R, const float *N, const float *nfmax, float *F,
                          const std::vector<GroupSet> &sets, int32_t K, int64_t Bs, hipStream_t s);
void launch_sum_bwd_param_generic(const float *theta, const float *l, const float *R, const float *N, float *G,
                                  const GroupDev &g, int32_t K, int64_t Bs, int32_t B, hipStream_t s);
// bf16-split path (long dense reductions): operand planes and the kernels that read them
bool sum_layer_takes_bf16(int32_t K, int32_t n_groups, int32_t n_rows, int32_t width, int64_t Bs);
void launch_split_theta(const float *theta, int64_t n_blocks, int32_t K, bool transposed, void *Th, void *Tl, hipStream_t s);
void launch_split_p(const float *X, const float *ref, const int32_t *blk_ids, int32_t n_blk, int32_t K, int64_t Bs, void *Ph,
                    void *Pl, hipStream_t s);
void launch_sum_bf16(const void *Th, const void *Tl, const void *Ph, const void *Pl, float *l, float *R, const float *nfmax,
                     float *F, bool bwd, const GroupSet &gs, int32_t K, int64_t Bs, hipStream_t s);
bool param_flow_by_block(int32_t K);
void launch_param_flow(const float *theta, const float *l, const float *R, const float *N, const float *nfmax, float *G,
                       const ParamFlowDev &pf, int32_t K, int64_t Bs, hipStream_t s);
void launch_em(float *theta, float *tables, float *theta_flow, float *table_flow, const EmDev &em, int32_t K,
               int32_t n_param_blocks, int32_t n_tables, int32_t n_cats, float step, float pc, hipStream_t s);

}  // namespace pc
