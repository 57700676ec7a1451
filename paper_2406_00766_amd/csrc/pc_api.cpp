// C-ABI entry points of libpc: compile + upload, inspection, forward, backward, EM step.
#include <hip/hip_runtime.h>

#include <cstdlib>
#include <cstring>
#include <mutex>
#include <new>
#include <string>

#include "pc_internal.h"
#include "pc_kernels.h"

namespace pc {
const char *last_error_cstr();

static pc_status hip_fail(hipError_t e, const char *what)
{
    return fail(PC_ERR_HIP, std::string(what) + ": " + hipGetErrorString(e));
}

#define PC_HIP(call)                                      \
    do {                                                  \
        hipError_t e_ = (call);                           \
        if (e_ != hipSuccess) return hip_fail(e_, #call); \
    } while (0)

static inline size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

// Workspace of pc_forward_static: a fixed array in every GPU's memory, there from the moment the library is loaded
// until the process ends.  In host code the name `scratch` is only a handle for hipGetSymbolAddress -- each device
// holds its own copy at its own address, looked up once per device by static_scratch() and used from then on.
static __device__ __align__(256) __attribute__((used)) unsigned char scratch[PC_STATIC_SCRATCH_BYTES];
constexpr int kMaxDevices = 64;
static std::mutex g_scratch_mutex;
static void *g_scratch_ptr[kMaxDevices] = {nullptr};

static pc_status static_scratch(void **out)
{
    int device = -1;
    PC_HIP(hipGetDevice(&device));
    if (device < 0 || device >= kMaxDevices) return fail(PC_ERR_ARG, "device ordinal out of range");
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[device]) {
        void *ptr = nullptr;
        PC_HIP(hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)));     // the current device's copy
        if (!ptr) return fail(PC_ERR_HIP, "hipGetSymbolAddress returned a null address for the static scratch");
        g_scratch_ptr[device] = ptr;
    }
    *out = g_scratch_ptr[device];
    return PC_OK;
}

// One arena for every table: sizes first, then pointers.  Host copies are uploaded where they exist; tables built
// on the device only get their space.
pc_status upload(pc_circuit *c, hipStream_t stream)
{
    size_t bytes = 0;
    auto reserve = [&](size_t n_i32) { size_t off = bytes; bytes = align_up(bytes + n_i32 * 4, 256); return off; };
    struct Fix { void **dst; size_t off; const void *src; size_t n; };
    std::vector<Fix> fixes;
    auto add = [&](int32_t **dst, const std::vector<int32_t> &v) {
        fixes.push_back({(void **)dst, reserve(v.size()), v.data(), v.size() * 4});
    };
    auto add_sized = [&](int32_t **dst, const std::vector<int32_t> &v, size_t n) {   // n entries, copied only if present
        fixes.push_back({(void **)dst, reserve(n), v.data(), v.size() == n ? n * 4 : 0});
    };
    for (auto &layer : c->layers) {
        add(&layer.d_blk_ids, layer.blk_ids);
        for (auto *groups : {&layer.fwd, &layer.bwd})
            for (auto &g : *groups) {
                add_sized(&g.d_ids, g.ids, (size_t)g.n_rows);
                add_sized(&g.d_nbr, g.nbr, (size_t)g.n_rows * g.width);
                add_sized(&g.d_par, g.par, (size_t)g.n_rows * g.width);
                add(&g.d_aux, g.aux);
            }
        if (!layer.pf_pb.empty()) {
            add(&layer.d_pf_pb, layer.pf_pb); add(&layer.d_pf_ptr, layer.pf_ptr);
            add(&layer.d_pf_sum, layer.pf_sum); add(&layer.d_pf_child, layer.pf_child);
        }
    }
    add(&c->d_pb_group, c->pb_group); add(&c->d_pb_rows, c->pb_rows); add(&c->d_pb_cols, c->pb_cols);
    add(&c->d_group_nch, c->group_nch);
    add(&c->d_init_ids, c->init_ids);
    add(&c->d_pf_pb, c->pf_pb); add(&c->d_pf_ptr, c->pf_ptr); add(&c->d_pf_sum, c->pf_sum); add(&c->d_pf_child, c->pf_child);
    const size_t zrow_off = reserve((size_t)c->n_em_groups * c->K + 1);
    const size_t ztab_off = reserve((size_t)c->n_tables * c->K + 1);
    PC_HIP(hipMalloc(&c->d_arena, bytes));
    c->arena_bytes = bytes;
    char *base = (char *)c->d_arena;
    for (auto &f : fixes) {
        *f.dst = base + f.off;
        if (f.n) PC_HIP(hipMemcpyAsync(base + f.off, f.src, f.n, hipMemcpyHostToDevice, stream));
    }
    c->d_zrow = (float *)(base + zrow_off);
    c->d_ztab = (float *)(base + ztab_off);
    PC_HIP(hipStreamSynchronize(stream));
    c->on_device = true;
    return PC_OK;
}

struct ProfScope {                                   // installs the circuit's profiler for the calling thread
    explicit ProfScope(pc_circuit *c) { set_profiler(c ? (Profiler *)c->profiler : nullptr); }
    ~ProfScope() { set_profiler(nullptr); }
};

static const char *const kClassNames[KC_COUNT] = {"misc", "input_fwd", "prod_fwd", "sum_fwd", "lognf", "sum_bwd_child",
                                                  "sum_bwd_param", "prod_bwd", "input_bwd", "em", "split"};

static GroupDev dev(const GroupTab &g) { return GroupDev{g.n_rows, g.width, g.d_ids, g.d_nbr, g.d_par, g.tied_in_group, g.d_aux}; }

// Group sets of every layer, built once after the tables are on the device.
struct LaunchPlan {
    struct Layer { std::vector<GroupSet> fwd, bwd; bool orphan_sum = false; };   // orphan_sum: a sum block of the layer has no parent
    std::vector<Layer> layers;
};
static LaunchPlan *make_plan(const pc_circuit *c)
{
    LaunchPlan *p = new (std::nothrow) LaunchPlan();
    if (!p) return nullptr;
    p->layers.resize(c->layers.size());
    for (size_t li = 0; li < c->layers.size(); ++li) {
        std::vector<GroupDev> f, b;
        for (const GroupTab &g : c->layers[li].fwd) f.push_back(dev(g));
        for (const GroupTab &g : c->layers[li].bwd) b.push_back(dev(g));
        p->layers[li].fwd = make_group_sets(f);
        p->layers[li].bwd = make_group_sets(b);
        if (c->layers[li].kind == KIND_SUM)
            for (int32_t id : c->layers[li].blk_ids)
                for (int32_t e : c->init_ids) if (e == id) p->layers[li].orphan_sum = true;
    }
    return p;
}

struct Ws {
    int64_t Bs;
    size_t l_off, f_off, n_off, r_off, mx_off, xt_off, total;
    size_t th_off, tl_off, tth_off, ttl_off, ph_off, pl_off;   // bf16 operand planes (only where a layer takes the bf16 kernels)
    bool bf16;
    int64_t l_rows;                                   // rows of l: all of them, or the persistent ones and the product window
};
// Product-scratch mode: base pointer through which the rows of product layer L (a contiguous range of block ids) land
// in the window behind the persistent rows of l; node offsets stay what they are.
static inline float *window_base(const pc_circuit *c, const LayerTab &L, float *l, int64_t Bs)
{
    return l + ((int64_t)c->n_persistent_blocks - L.scr_first_block) * c->K * Bs;
}

static inline bool misaligned(const void *p) { return ((uintptr_t)p & 15) != 0; }   // kernels use 16-byte accesses

static Ws ws_layout(const pc_circuit *c, int32_t B)
{
    Ws w;
    w.Bs = ((int64_t)B + 31) / 32 * 32;
    const size_t rows = ((size_t)c->n_blocks + 1) * c->K;
    const size_t node = align_up(rows * w.Bs * 4, 256);
    // product-scratch mode: l holds the null block, the input and sum blocks and one window for the largest product layer
    w.l_rows = c->product_scratch ? ((int64_t)c->n_persistent_blocks + 1 + c->max_window_blocks) * c->K : (int64_t)rows;
    const size_t lnode = align_up((size_t)w.l_rows * w.Bs * 4, 256);
    // ... and so does F (a product layer's flows are written by the sum layer above it and read by the layer itself right
    // after); log_nf exists for sum rows only, which are among the persistent ones
    const size_t fnode = c->product_scratch ? lnode : node;
    const size_t nnode = c->product_scratch ? align_up(((size_t)c->n_persistent_blocks + 1) * c->K * w.Bs * 4, 256) : node;
    w.l_off = 0; w.f_off = lnode; w.n_off = lnode + fnode;
    const size_t per_block = align_up(((size_t)c->n_blocks + 1) * w.Bs * 4, 256);
    w.r_off = lnode + fnode + nnode;
    w.mx_off = w.r_off + per_block;
    w.xt_off = w.mx_off + per_block;
    w.total = w.xt_off + align_up((size_t)c->n_vars * w.Bs * 4, 256);
    // layers with long dense rows run on the bf16 matrix cores and need theta and the node values split into planes
    w.bf16 = false;
    for (const LayerTab &L : c->layers)
        if (!c->product_scratch && L.kind == KIND_SUM && L.fwd.size() == 1 && sum_layer_takes_bf16(c->K, 1, L.fwd[0].n_rows, L.fwd[0].width, w.Bs)) w.bf16 = true;
    w.th_off = w.tl_off = w.tth_off = w.ttl_off = w.ph_off = w.pl_off = 0;
    if (w.bf16) {
        const size_t tplane = align_up(((size_t)c->n_param_blocks + 1) * c->K * c->K * 2, 256), pplane = align_up(rows * w.Bs * 2, 256);
        w.th_off = w.total; w.tl_off = w.th_off + tplane;               // theta, hi and lo
        w.tth_off = w.tl_off + tplane; w.ttl_off = w.tth_off + tplane;  // theta transposed (backward)
        w.ph_off = w.ttl_off + tplane; w.pl_off = w.ph_off + pplane;    // node values: product rows forward, sum rows backward
        w.total = w.pl_off + pplane;
    }
    return w;
}

}  // namespace pc

using namespace pc;

extern "C" {

const char *pc_last_error(void) { return last_error_cstr(); }

// Host-only compilation (no GPU touched): used to check the compiled tables on machines without a GPU.
pc_status pc_compile_host(const pc_dag *dag, pc_circuit **out)
{
    if (!out) return fail(PC_ERR_ARG, "out is NULL");
    pc_circuit *c = new (std::nothrow) pc_circuit();
    if (!c) return fail(PC_ERR_ARG, "out of host memory");
    pc_status st = compile_host(dag, c, /*tables_on_host=*/true);
    if (st != PC_OK) { delete c; return st; }
    *out = c;
    return PC_OK;
}

pc_status pc_compile(const pc_dag *dag, void *stream, pc_circuit **out)
{
    if (!out) return fail(PC_ERR_ARG, "out is NULL");
    pc_circuit *c = new (std::nothrow) pc_circuit();
    if (!c) return fail(PC_ERR_ARG, "out of host memory");
    pc_status st = compile_host(dag, c, /*tables_on_host=*/false);      // validation, layering, EM and flow maps
    if (st == PC_OK) st = build_tables_device(dag, c, stream);          // groups (Alg. 2) + tables filled by HIP kernels
    if (st == PC_OK && !(c->plan = make_plan(c))) st = fail(PC_ERR_ARG, "out of host memory");
    if (st != PC_OK) { pc_destroy(c); return st; }
    const char *env = std::getenv("PC_FORCE_GENERIC");
    set_force_generic(env && env[0] == '1');
    *out = c;
    return PC_OK;
}

void pc_destroy(pc_circuit *c)
{
    if (!c) return;
    if (c->d_arena) (void)hipFree(c->d_arena);
    delete (Profiler *)c->profiler;
    delete (LaunchPlan *)c->plan;
    delete c;
}

pc_status pc_get_sizes(const pc_circuit *c, pc_sizes *out)
{
    if (!c || !out) return fail(PC_ERR_ARG, "NULL argument");
    out->K = c->K; out->n_blocks = c->n_blocks; out->n_layers = (int32_t)c->layers.size();
    out->n_rows = ((int64_t)c->n_blocks + 1) * c->K;
    out->theta_len = ((int64_t)c->n_param_blocks + 1) * c->K * c->K;
    out->tables_len = (int64_t)c->n_tables * c->n_cats * c->K;
    out->n_vars = c->n_vars; out->n_cats = c->n_cats; out->n_tables = c->n_tables;
    return PC_OK;
}

pc_status pc_get_layer(const pc_circuit *c, int32_t layer, pc_layer_desc *out)
{
    if (!c || !out) return fail(PC_ERR_ARG, "NULL argument");
    if (layer < 0 || layer >= (int32_t)c->layers.size()) return fail(PC_ERR_ARG, "layer out of range");
    const LayerTab &L = c->layers[layer];
    out->kind = L.kind; out->depth = L.depth;
    out->n_fwd_groups = (int32_t)L.fwd.size(); out->n_bwd_groups = (int32_t)L.bwd.size();
    return PC_OK;
}

static const GroupTab *find_group(const pc_circuit *c, int32_t layer, int32_t dir, int32_t group)
{
    if (!c || layer < 0 || layer >= (int32_t)c->layers.size() || (dir != 0 && dir != 1)) return nullptr;
    const auto &gs = dir == 0 ? c->layers[layer].fwd : c->layers[layer].bwd;
    if (group < 0 || group >= (int32_t)gs.size()) return nullptr;
    return &gs[group];
}

pc_status pc_get_group(const pc_circuit *c, int32_t layer, int32_t dir, int32_t group, pc_group_desc *out)
{
    const GroupTab *g = find_group(c, layer, dir, group);
    if (!g || !out) return fail(PC_ERR_ARG, "layer / dir / group out of range");
    out->n_rows = g->n_rows; out->width = g->width;
    out->ids = g->d_ids; out->nbr = g->d_nbr; out->par = g->d_par;
    return PC_OK;
}

pc_status pc_copy_group(const pc_circuit *c, int32_t layer, int32_t dir, int32_t group,
                        int32_t *ids_host, int32_t *nbr_host, int32_t *par_host)
{
    const GroupTab *g = find_group(c, layer, dir, group);
    if (!g) return fail(PC_ERR_ARG, "layer / dir / group out of range");
    const size_t n_ids = (size_t)g->n_rows * 4, n_tab = (size_t)g->n_rows * g->width * 4;
    if (c->on_device) {                                   // what the kernels really read
        if (ids_host && n_ids) PC_HIP(hipMemcpy(ids_host, g->d_ids, n_ids, hipMemcpyDeviceToHost));
        if (nbr_host && n_tab) PC_HIP(hipMemcpy(nbr_host, g->d_nbr, n_tab, hipMemcpyDeviceToHost));
        if (par_host && n_tab) PC_HIP(hipMemcpy(par_host, g->d_par, n_tab, hipMemcpyDeviceToHost));
    } else {
        if (g->ids.size() * 4 != n_ids || g->nbr.size() * 4 != n_tab) return fail(PC_ERR_STATE, "tables live on the device");
        if (ids_host) std::memcpy(ids_host, g->ids.data(), n_ids);
        if (nbr_host) std::memcpy(nbr_host, g->nbr.data(), n_tab);
        if (par_host) std::memcpy(par_host, g->par.data(), n_tab);
    }
    return PC_OK;
}

pc_status pc_workspace_layout(const pc_circuit *c, int32_t B, pc_ws_layout *out)
{
    if (!c || !out) return fail(PC_ERR_ARG, "NULL argument");
    if (B < 1) return fail(PC_ERR_ARG, "B must be positive");
    if (B > PC_MAX_BATCH) return fail(PC_ERR_TOO_LARGE, "more than PC_MAX_BATCH samples in one call");
    const Ws w = ws_layout(c, B);
    out->stride = w.Bs; out->l_offset = w.l_off; out->f_offset = w.f_off; out->n_offset = w.n_off;
    out->r_offset = w.r_off;
    out->total_bytes = w.total;
    out->l_rows = w.l_rows;
    return PC_OK;
}

pc_status pc_workspace_bytes(const pc_circuit *c, int32_t B, size_t *bytes)
{
    pc_ws_layout lay;
    if (!bytes) return fail(PC_ERR_ARG, "NULL argument");
    pc_status st = pc_workspace_layout(c, B, &lay);
    if (st == PC_OK) *bytes = lay.total_bytes;
    return st;
}

// The forward pass proper: argument checks, then kernels only.  `profiled` installs the circuit's per-launch timer.
static pc_status forward_on(pc_circuit *c, const float *theta, const float *tables, const int32_t *x, const uint8_t *mask,
                            int32_t B, void *workspace, size_t workspace_bytes, float *ll, hipStream_t s, bool profiled)
{
    if (!c || !theta || !tables || !x || !workspace || !ll) return fail(PC_ERR_ARG, "NULL argument");
    if (!c->on_device) return fail(PC_ERR_STATE, "circuit was compiled without a device");
    if (B < 1) return fail(PC_ERR_ARG, "B must be positive");
    if (B > PC_MAX_BATCH) return fail(PC_ERR_TOO_LARGE, "more than PC_MAX_BATCH samples in one call");
    if (misaligned(theta) || misaligned(tables) || misaligned(workspace))
        return fail(PC_ERR_ARG, "theta, tables and workspace must be 16-byte aligned");
    const Ws w = ws_layout(c, B);
    if (workspace_bytes < w.total) return fail(PC_ERR_WORKSPACE, "workspace smaller than pc_workspace_bytes");
    ProfScope prof(profiled ? c : nullptr);
    char *base = (char *)workspace;
    float *l = (float *)(base + w.l_off), *R = (float *)(base + w.r_off);
    int32_t *xT = (int32_t *)(base + w.xt_off);
    const int32_t K = c->K;
    c->fw_B = -1;

    launch_prepare_x(x, mask, B, c->n_vars, w.Bs, c->n_cats, xT, s);
    launch_fill(l, (int64_t)K * w.Bs, 0.0f, s);                                  // null block: probability 1
    launch_fill(R, ((int64_t)c->n_blocks + 1) * w.Bs, 0.0f, s);                  // input and null blocks: R = 0
    const LaunchPlan &plan = *(const LaunchPlan *)c->plan;
    if (w.bf16) launch_split_theta(theta, (int64_t)c->n_param_blocks + 1, K, false, base + w.th_off, base + w.tl_off, s);
    for (size_t li = 0; li < c->layers.size(); ++li) {
        const LayerTab &L = c->layers[li];
        if (L.kind == KIND_INPUT) {
            launch_input_fwd(tables, xT, dev(L.fwd[0]), K, c->n_cats, w.Bs, l, s);
        } else if (L.kind == KIND_PRODUCT) {
            launch_prod_fwd(l, c->product_scratch ? window_base(c, L, l, w.Bs) : l, R, plan.layers[li].fwd, K, w.Bs,
                            w.bf16 ? base + w.ph_off : nullptr, w.bf16 ? base + w.pl_off : nullptr, s);
        } else if (w.bf16 && L.fwd.size() == 1 && sum_layer_takes_bf16(K, 1, L.fwd[0].n_rows, L.fwd[0].width, w.Bs)) {
            launch_sum_bf16(base + w.th_off, base + w.tl_off, base + w.ph_off, base + w.pl_off, l, R, nullptr, nullptr, false,
                            plan.layers[li].fwd[0], K, w.Bs, s);
        } else {
            // product-scratch mode: the children are the product layer just before, in the window
            launch_sum_fwd(theta, c->product_scratch ? window_base(c, c->layers[li - 1], l, w.Bs) : l, l, R, plan.layers[li].fwd, K,
                           w.Bs, s);
        }
    }
    launch_readout(l, R, (int64_t)(c->root_block + 1) * K, (int64_t)c->root_block + 1, w.Bs, B, ll, s);
    PC_HIP(hipGetLastError());
    return PC_OK;
}

pc_status pc_forward(pc_circuit *c, const float *theta, const float *tables, const int32_t *x,
                     const uint8_t *mask, int32_t B, void *workspace, size_t workspace_bytes,
                     float *ll, void *stream)
{
    pc_status st = forward_on(c, theta, tables, x, mask, B, workspace, workspace_bytes, ll, (hipStream_t)stream, true);
    if (st != PC_OK) return st;
    c->fw_workspace = workspace; c->fw_theta = theta; c->fw_tables = tables; c->fw_x = x; c->fw_mask = mask;
    c->fw_B = B;
    return PC_OK;
}

pc_status pc_forward_static(pc_circuit *c, const float *theta, const float *tables, const int32_t *x,
                            const uint8_t *mask, int32_t B, float *ll, void *stream)
{
    if (!c) return fail(PC_ERR_ARG, "NULL argument");
    if (B < 1) return fail(PC_ERR_ARG, "B must be positive");
    if (B > PC_MAX_BATCH) return fail(PC_ERR_TOO_LARGE, "more than PC_MAX_BATCH samples in one call");
    const Ws w = ws_layout(c, B);
    if (w.total > (size_t)PC_STATIC_SCRATCH_BYTES)
        return fail(PC_ERR_WORKSPACE, "this circuit and batch need " + std::to_string(w.total) +
                                          " bytes of workspace, more than the PC_STATIC_SCRATCH_BYTES = " +
                                          std::to_string((size_t)PC_STATIC_SCRATCH_BYTES) + " of pc_forward_static");
    void *ws = nullptr;
    pc_status st = static_scratch(&ws);
    if (st != PC_OK) return st;
    // no per-launch timing here: the timer creates events
    return forward_on(c, theta, tables, x, mask, B, ws, (size_t)PC_STATIC_SCRATCH_BYTES, ll, (hipStream_t)stream, false);
}

pc_status pc_backward(pc_circuit *c, const float *theta, const float *tables, const int32_t *x,
                      const uint8_t *mask, int32_t B, void *workspace, size_t workspace_bytes,
                      float *theta_flow, float *table_flow, void *stream)
{
    if (!c || !theta || !tables || !x || !workspace) return fail(PC_ERR_ARG, "NULL argument");
    if (!c->on_device) return fail(PC_ERR_STATE, "circuit was compiled without a device");
    if (c->fw_B != B || c->fw_workspace != workspace || c->fw_theta != theta || c->fw_tables != tables ||
        c->fw_x != x || c->fw_mask != mask)
        return fail(PC_ERR_STATE, "pc_backward needs the pc_forward that just ran on the same arguments");
    if (misaligned(theta_flow) || misaligned(table_flow))
        return fail(PC_ERR_ARG, "theta_flow and table_flow must be 16-byte aligned");
    const Ws w = ws_layout(c, B);
    if (workspace_bytes < w.total) return fail(PC_ERR_WORKSPACE, "workspace smaller than pc_workspace_bytes");
    hipStream_t s = (hipStream_t)stream;
    ProfScope prof(c);
    char *base = (char *)workspace;
    float *l = (float *)(base + w.l_off), *F = (float *)(base + w.f_off), *N = (float *)(base + w.n_off);
    float *nfmax = (float *)(base + w.mx_off);
    const float *R = (const float *)(base + w.r_off);
    const int32_t *xT = (const int32_t *)(base + w.xt_off);
    const int32_t K = c->K;

    // block sizes with a by-parameter-block kernel (1-16, 32, 64, 128): parameter flows of the whole circuit in one
    // launch after the sweep (N and nfmax of every sum layer stay valid until then); other block sizes: layer by layer
    const bool batched_params = param_flow_by_block(K);
    // no clearing of F: every block's flow is stored by the first layer that feeds it, blocks nobody feeds are
    // initialised here
    const LaunchPlan &plan = *(const LaunchPlan *)c->plan;
    launch_init_flows(l, F, N, nfmax, c->d_init_ids, (int32_t)c->init_ids.size(), (c->root_block + 1) * K, K, w.Bs, B, s);
    bool theta_t_split = false;
    for (size_t li = c->layers.size(); li-- > 0;) {
        const LayerTab &L = c->layers[li];
        if (L.kind == KIND_SUM && w.bf16 && L.bwd.size() == 1 &&
            sum_layer_takes_bf16(K, 1, L.bwd[0].n_rows, L.bwd[0].width, w.Bs)) {
            // long dense rows: bf16 matrix cores on planes of theta^T (once per pass) and of this layer's exp(log_nf - max)
            if (!theta_t_split) launch_split_theta(theta, (int64_t)c->n_param_blocks + 1, K, true, base + w.tth_off, base + w.ttl_off, s);
            theta_t_split = true;
            // the planes of exp(log_nf - max) were written by the product layers that finished these blocks' flows; a
            // block without parents (initialised by k_init_flows) has none, so such a layer splits here
            if (plan.layers[li].orphan_sum) launch_split_p(N, nfmax, L.d_blk_ids, (int32_t)L.blk_ids.size(), K, w.Bs, base + w.ph_off, base + w.pl_off, s);
            launch_sum_bf16(base + w.tth_off, base + w.ttl_off, base + w.ph_off, base + w.pl_off, l, const_cast<float *>(R), nfmax, F,
                            true, plan.layers[li].bwd[0], K, w.Bs, s);
            if (theta_flow && !batched_params)
                for (const GroupTab &g : L.fwd) launch_sum_bwd_param_generic(theta, l, R, N, theta_flow, dev(g), K, w.Bs, B, s);
        } else if (L.kind == KIND_SUM && c->product_scratch) {
            // Sec. 5: the product layer this sum layer reads is evaluated again into the scratch window, then the flows
            // to the children and this layer's parameter flows are taken while its values are there
            const LayerTab &P = c->layers[li - 1];
            float *lp = window_base(c, P, l, w.Bs);
            launch_prod_fwd(l, lp, const_cast<float *>(R), plan.layers[li - 1].fwd, K, w.Bs, nullptr, nullptr, s);
            launch_sum_bwd_child(theta, lp, R, N, nfmax, window_base(c, P, F, w.Bs), plan.layers[li].bwd, K, w.Bs, s);
            if (theta_flow && batched_params) {
                ParamFlowDev pf{(int32_t)L.pf_pb.size(), L.d_pf_pb, L.d_pf_ptr, L.d_pf_sum, L.d_pf_child, (int64_t)L.pf_sum.size()};
                launch_param_flow(theta, lp, R, N, nfmax, theta_flow, pf, K, w.Bs, s);
            } else if (theta_flow) {
                for (const GroupTab &g : L.fwd) launch_sum_bwd_param_generic(theta, lp, R, N, theta_flow, dev(g), K, w.Bs, B, s);
            }
        } else if (L.kind == KIND_SUM) {
            launch_sum_bwd_child(theta, l, R, N, nfmax, F, plan.layers[li].bwd, K, w.Bs, s);
            if (theta_flow && !batched_params)
                for (const GroupTab &g : L.fwd) launch_sum_bwd_param_generic(theta, l, R, N, theta_flow, dev(g), K, w.Bs, B, s);
        } else if (L.kind == KIND_PRODUCT && c->product_scratch) {
            float *Fw = window_base(c, L, F, w.Bs);
            // the layer of product blocks nobody reads (the last one) has flow 0
            if (li + 1 == c->layers.size())
                launch_fill(Fw + (int64_t)(L.scr_first_block + 1) * K * w.Bs, (int64_t)L.blk_ids.size() * K * w.Bs, 0.0f, s);
            launch_prod_bwd(l, F, Fw, N, nfmax, plan.layers[li].bwd, K, w.Bs, nullptr, nullptr, s);
        } else if (L.kind == KIND_PRODUCT) {
            launch_prod_bwd(l, F, F, N, nfmax, plan.layers[li].bwd, K, w.Bs, w.bf16 ? base + w.ph_off : nullptr, w.bf16 ? base + w.pl_off : nullptr, s);
        } else if (table_flow) {
            launch_input_bwd(F, xT, dev(L.fwd[0]), K, c->n_cats, w.Bs, table_flow, s);
        }
    }
    if (theta_flow && batched_params && !c->product_scratch) {
        ParamFlowDev pf{(int32_t)c->pf_pb.size(), c->d_pf_pb, c->d_pf_ptr, c->d_pf_sum, c->d_pf_child, (int64_t)c->pf_sum.size()};
        launch_param_flow(theta, l, R, N, nfmax, theta_flow, pf, K, w.Bs, s);
    }
    PC_HIP(hipGetLastError());
    return PC_OK;
}

pc_status pc_em_step(pc_circuit *c, float *theta, float *tables, float *theta_flow, float *table_flow,
                     float step, float pseudocount, void *stream)
{
    if (!c || !theta || !tables || !theta_flow || !table_flow) return fail(PC_ERR_ARG, "NULL argument");
    if (!c->on_device) return fail(PC_ERR_STATE, "circuit was compiled without a device");
    if (!(step >= 0.0f && step <= 1.0f) || !(pseudocount >= 0.0f)) return fail(PC_ERR_ARG, "step in [0,1], pseudocount >= 0");
    if (misaligned(theta) || misaligned(tables) || misaligned(theta_flow) || misaligned(table_flow))
        return fail(PC_ERR_ARG, "theta, tables and their flow arrays must be 16-byte aligned");
    ProfScope prof(c);
    EmDev em{c->n_em_groups, c->d_pb_group, c->d_pb_rows, c->d_pb_cols, c->d_group_nch, c->d_zrow, c->d_ztab};
    launch_em(theta, tables, theta_flow, table_flow, em, c->K, c->n_param_blocks, c->n_tables, c->n_cats, step,
              pseudocount, (hipStream_t)stream);
    launch_fill(theta_flow, (int64_t)c->K * c->K, 0.0f, (hipStream_t)stream);     // the padding block of the flows
    PC_HIP(hipGetLastError());
    c->fw_B = -1;
    return PC_OK;
}

pc_status pc_profile_enable(pc_circuit *c, int32_t on)
{
    if (!c) return fail(PC_ERR_ARG, "NULL argument");
    delete (Profiler *)c->profiler;
    c->profiler = on ? new (std::nothrow) Profiler() : nullptr;
    for (int k = 0; k < KC_COUNT; ++k) { c->prof_launches[k] = 0; c->prof_ms[k] = 0.0; }
    return PC_OK;
}

pc_status pc_profile_read(pc_circuit *c, pc_profile *out)
{
    if (!c || !out) return fail(PC_ERR_ARG, "NULL argument");
    if (c->profiler) ((Profiler *)c->profiler)->collect(c->prof_launches, c->prof_ms);
    out->n_classes = KC_COUNT;
    for (int k = 0; k < PC_MAX_KERNEL_CLASSES; ++k) {
        out->launches[k] = k < KC_COUNT ? c->prof_launches[k] : 0;
        out->ms[k] = k < KC_COUNT ? c->prof_ms[k] : 0.0;
        out->bf16_launches[k] = (c->profiler && k < KC_COUNT) ? ((Profiler *)c->profiler)->bf16_launches[k] : 0;
    }
    PC_HIP(hipGetLastError());
    return PC_OK;
}

const char *pc_kernel_class_name(int32_t cls) { return cls >= 0 && cls < KC_COUNT ? kClassNames[cls] : ""; }

}  // extern "C"
