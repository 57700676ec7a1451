// Device side of pc_compile: the block compiler that turns the block-level DAG into per-group index
// tensors (Sec. 4.3: sum_ids / prod_ids / param_ids; App. A.2: ch_ids / par_ids / par_param_ids; the same
// pair for product layers).
//
// Host (pc_compile.cpp): validation, longest-path depths, layers, Alg. 2 on the neighbour counts.
// Device (here), all integer work over the edges:
//   1. parents per block: count (atomics), exclusive scan, scatter -- a transpose of the child CSR;
//   2. every parent list is sorted by (layer of the parent, parent id) and cut into runs of one layer:
//      each run is one row of that layer's backward tables; run descriptors go back to the host, which
//      only sees O(#rows) data, groups the rows (Alg. 2) and returns where each row is to be written;
//   3. fill kernels write forward rows (children sorted ascending) and backward rows (parents ascending)
//      as node / parameter offsets, padded with 0 / 0 to the group width.
// Atomics make the order inside a scattered list arbitrary; the per-list sort restores the canonical order,
// so the tables are bit-identical from run to run and equal to the host builder's.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cstdint>
#include <limits>
#include <vector>

#include "pc_internal.h"

namespace pc {

namespace {

#define PC_HIP(call)                                                                        \
    do {                                                                                    \
        hipError_t e_ = (call);                                                             \
        if (e_ != hipSuccess) return fail(PC_ERR_HIP, std::string(#call) + ": " + hipGetErrorString(e_)); \
    } while (0)

__global__ void k_edge_src(const int32_t *__restrict__ ptr, int32_t n, int32_t *__restrict__ src)
{
    const int u = blockIdx.x * blockDim.x + threadIdx.x;
    if (u >= n) return;
    for (int32_t e = ptr[u]; e < ptr[u + 1]; ++e) src[e] = u;
}

__global__ void k_count_parents(const int32_t *__restrict__ child, int32_t n_edges, int32_t *__restrict__ cnt)
{
    const int e = blockIdx.x * blockDim.x + threadIdx.x;
    if (e < n_edges) atomicAdd(cnt + child[e], 1);
}

// exclusive scan of in[0..n) into out[0..n], one workgroup of 1024 threads, each owning a contiguous chunk
__global__ __launch_bounds__(1024) void k_exclusive_scan(const int32_t *__restrict__ in, int32_t n, int32_t *__restrict__ out)
{
    __shared__ int32_t part[1024];
    const int t = threadIdx.x;
    const int32_t chunk = (n + 1023) / 1024;
    const int32_t lo = min(n, t * chunk), hi = min(n, lo + chunk);
    int32_t s = 0;
    for (int32_t i = lo; i < hi; ++i) s += in[i];
    part[t] = s;
    __syncthreads();
    for (int off = 1; off < 1024; off <<= 1) {                       // Hillis-Steele inclusive scan of the partials
        const int32_t v = t >= off ? part[t - off] : 0;
        __syncthreads();
        part[t] += v;
        __syncthreads();
    }
    int32_t run = t == 0 ? 0 : part[t - 1];
    for (int32_t i = lo; i < hi; ++i) { out[i] = run; run += in[i]; }
    if (t == 1023) out[n] = part[1023];
}

__global__ void k_scatter_parents(const int32_t *__restrict__ child, int32_t n_edges, const int32_t *__restrict__ pptr,
                                  int32_t *__restrict__ cursor, int32_t *__restrict__ tp)
{
    const int e = blockIdx.x * blockDim.x + threadIdx.x;
    if (e >= n_edges) return;
    const int32_t c = child[e];
    tp[pptr[c] + atomicAdd(cursor + c, 1)] = e;
}

// per block: sort its incoming edges by (layer of the source, source id); count the runs of equal layer.
// Keys are distinct (a block pair has one edge), so the result does not depend on the order the scatter left.
// Short lists: insertion sort; long ones (a child block of a wide small-K layer has some thousand parents): an
// in-place heap sort, n log n key look-ups instead of n^2 / 4.
__device__ __forceinline__ int64_t parent_key(const int32_t *__restrict__ src, const int32_t *__restrict__ layer_of, int32_t e)
{
    const int32_t s = src[e];
    return ((int64_t)layer_of[s] << 32) | (uint32_t)s;
}

__device__ void sift_down(int32_t *__restrict__ a, int32_t root, int32_t end, const int32_t *__restrict__ src,
                          const int32_t *__restrict__ layer_of)
{
    const int32_t moving = a[root];
    const int64_t key = parent_key(src, layer_of, moving);
    for (;;) {
        int32_t kid = 2 * root + 1;
        if (kid >= end) break;
        int64_t kk = parent_key(src, layer_of, a[kid]);
        if (kid + 1 < end) {
            const int64_t k2 = parent_key(src, layer_of, a[kid + 1]);
            if (k2 > kk) { kk = k2; ++kid; }
        }
        if (kk <= key) break;
        a[root] = a[kid];
        root = kid;
    }
    a[root] = moving;
}

__global__ void k_sort_parent_lists(const int32_t *__restrict__ pptr, int32_t n, const int32_t *__restrict__ src,
                                    const int32_t *__restrict__ layer_of, int32_t *__restrict__ tp,
                                    int32_t *__restrict__ n_runs)
{
    const int c = blockIdx.x * blockDim.x + threadIdx.x;
    if (c >= n) return;
    const int32_t lo = pptr[c], hi = pptr[c + 1], len = hi - lo;
    if (len <= 24) {
        for (int32_t i = lo + 1; i < hi; ++i) {
            const int32_t e = tp[i];
            const int64_t key = parent_key(src, layer_of, e);
            int32_t j = i - 1;
            while (j >= lo) {
                const int32_t f = tp[j];
                if (parent_key(src, layer_of, f) <= key) break;
                tp[j + 1] = f;
                --j;
            }
            tp[j + 1] = e;
        }
    } else {
        int32_t *a = tp + lo;
        for (int32_t r = len / 2 - 1; r >= 0; --r) sift_down(a, r, len, src, layer_of);
        for (int32_t end = len - 1; end > 0; --end) {
            const int32_t top = a[0];
            a[0] = a[end];
            a[end] = top;
            sift_down(a, 0, end, src, layer_of);
        }
    }
    int32_t runs = 0;
    for (int32_t i = lo; i < hi; ++i)
        if (i == lo || layer_of[src[tp[i]]] != layer_of[src[tp[i - 1]]]) ++runs;
    n_runs[c] = runs;
}

__global__ void k_emit_rows(const int32_t *__restrict__ pptr, int32_t n, const int32_t *__restrict__ src,
                            const int32_t *__restrict__ layer_of, const int32_t *__restrict__ tp,
                            const int32_t *__restrict__ row_ptr, int32_t *__restrict__ row_layer,
                            int32_t *__restrict__ row_child, int32_t *__restrict__ row_start, int32_t *__restrict__ row_cnt)
{
    const int c = blockIdx.x * blockDim.x + threadIdx.x;
    if (c >= n) return;
    const int32_t lo = pptr[c], hi = pptr[c + 1];
    int32_t row = row_ptr[c] - 1;
    for (int32_t i = lo; i < hi; ++i) {
        const int32_t L = layer_of[src[tp[i]]];
        if (i == lo || L != layer_of[src[tp[i - 1]]]) {
            ++row;
            row_layer[row] = L; row_child[row] = c; row_start[row] = i; row_cnt[row] = 0;
        }
        ++row_cnt[row];
    }
}

// forward rows: block u -> ids entry, children (node offsets) and parameter offsets, sorted by child ascending
// inside the output row, padded with 0 / 0 to the group width
__global__ void k_fill_forward(const int32_t *__restrict__ ptr, int32_t n, const int32_t *__restrict__ child,
                               const int32_t *__restrict__ param, const uint8_t *__restrict__ type, int32_t K,
                               int32_t *const *__restrict__ ids_at, int32_t *const *__restrict__ nbr_at,
                               int32_t *const *__restrict__ par_at, const int32_t *__restrict__ width)
{
    const int u = blockIdx.x * blockDim.x + threadIdx.x;
    if (u >= n || ids_at[u] == nullptr) return;
    const int32_t lo = ptr[u], cnt = ptr[u + 1] - lo, w = width[u];
    const bool is_sum = type[u] == KIND_SUM;
    int32_t *nbr = nbr_at[u], *par = par_at[u];
    *ids_at[u] = (u + 1) * K;
    for (int32_t j = 0; j < cnt; ++j) {                               // insertion sort into the output row
        const int32_t c = (child[lo + j] + 1) * K;
        const int32_t p = is_sum ? (param[lo + j] + 1) * K * K : 0;
        int32_t i = j - 1;
        while (i >= 0 && nbr[i] > c) { nbr[i + 1] = nbr[i]; par[i + 1] = par[i]; --i; }
        nbr[i + 1] = c; par[i + 1] = p;
    }
    for (int32_t j = cnt; j < w; ++j) { nbr[j] = 0; par[j] = 0; }
}

// backward rows: run r of a sorted parent list -> ids entry (child), parents and parameter offsets, padded
__global__ void k_fill_backward(int32_t n_rows, const int32_t *__restrict__ row_child, const int32_t *__restrict__ row_start,
                                const int32_t *__restrict__ row_cnt, const int32_t *__restrict__ tp,
                                const int32_t *__restrict__ src, const int32_t *__restrict__ param,
                                const uint8_t *__restrict__ type, int32_t K, int32_t *const *__restrict__ ids_at,
                                int32_t *const *__restrict__ nbr_at, int32_t *const *__restrict__ par_at,
                                const int32_t *__restrict__ width)
{
    const int r = blockIdx.x * blockDim.x + threadIdx.x;
    if (r >= n_rows) return;
    int32_t *nbr = nbr_at[r], *par = par_at[r];
    *ids_at[r] = (row_child[r] + 1) * K;
    const int32_t cnt = row_cnt[r], w = width[r];
    for (int32_t j = 0; j < cnt; ++j) {
        const int32_t e = tp[row_start[r] + j], u = src[e];
        nbr[j] = (u + 1) * K;
        par[j] = type[u] == KIND_SUM ? (param[e] + 1) * K * K : 0;
    }
    for (int32_t j = cnt; j < w; ++j) { nbr[j] = 0; par[j] = 0; }
}

template <typename T>
struct DevBuf {                                                        // temporary device array, freed on scope exit
    T *p = nullptr;
    ~DevBuf() { if (p) (void)hipFree(p); }
    hipError_t alloc(size_t n) { return hipMalloc(&p, (n ? n : 1) * sizeof(T)); }
};

inline unsigned blocks_for(int64_t n) { return (unsigned)((n + 255) / 256 > 0 ? (n + 255) / 256 : 1); }

// rows (each with a neighbour count) -> groups by Alg. 2; returns group index and rank inside the group per row
void assign_groups(const std::vector<int32_t> &counts, int32_t max_groups, int32_t tol_permille,
                   std::vector<GroupTab> &groups, std::vector<int32_t> &grp, std::vector<int32_t> &rank)
{
    const std::vector<int32_t> caps = partition_groups(counts, max_groups, tol_permille);
    groups.assign(caps.size(), GroupTab());
    for (size_t g = 0; g < caps.size(); ++g) groups[g].width = caps[g];
    grp.resize(counts.size()); rank.resize(counts.size());
    for (size_t r = 0; r < counts.size(); ++r) {
        const size_t g = std::lower_bound(caps.begin(), caps.end(), counts[r]) - caps.begin();
        grp[r] = (int32_t)g;
        rank[r] = groups[g].n_rows++;
    }
}

}  // namespace

pc_status upload(pc_circuit *c, hipStream_t stream);                   // pc_api.cpp: allocates the arena, copies host metadata

pc_status build_tables_device(const pc_dag *d, pc_circuit *c, void *stream_v)
{
    hipStream_t stream = (hipStream_t)stream_v;
    const int32_t n = d->n_blocks, K = d->K;
    const int64_t E64 = d->child_ptr[n];
    if (E64 > std::numeric_limits<int32_t>::max()) return fail(PC_ERR_TOO_LARGE, "edge count exceeds int32");
    const int32_t E = (int32_t)E64;

    // block -> layer index (layer 0 = inputs)
    std::vector<int32_t> layer_of(n, 0), ptr32(n + 1);
    for (size_t li = 1; li < c->layers.size(); ++li)
        for (int32_t id : c->layers[li].blk_ids) layer_of[id / K - 1] = (int32_t)li;
    for (int32_t u = 0; u <= n; ++u) ptr32[u] = (int32_t)d->child_ptr[u];

    DevBuf<int32_t> d_ptr, d_child, d_param, d_layer, d_src, d_pcnt, d_pptr, d_cursor, d_tp, d_runs, d_rowptr;
    DevBuf<uint8_t> d_type;
    PC_HIP(d_ptr.alloc(n + 1)); PC_HIP(d_child.alloc(E)); PC_HIP(d_param.alloc(E)); PC_HIP(d_layer.alloc(n));
    PC_HIP(d_src.alloc(E)); PC_HIP(d_pcnt.alloc(n)); PC_HIP(d_pptr.alloc(n + 1)); PC_HIP(d_cursor.alloc(n));
    PC_HIP(d_tp.alloc(E)); PC_HIP(d_runs.alloc(n)); PC_HIP(d_rowptr.alloc(n + 1)); PC_HIP(d_type.alloc(n));
    PC_HIP(hipMemcpyAsync(d_ptr.p, ptr32.data(), (size_t)(n + 1) * 4, hipMemcpyHostToDevice, stream));
    if (E) PC_HIP(hipMemcpyAsync(d_child.p, d->child, (size_t)E * 4, hipMemcpyHostToDevice, stream));
    if (E) PC_HIP(hipMemcpyAsync(d_param.p, d->param_blk, (size_t)E * 4, hipMemcpyHostToDevice, stream));
    PC_HIP(hipMemcpyAsync(d_layer.p, layer_of.data(), (size_t)n * 4, hipMemcpyHostToDevice, stream));
    PC_HIP(hipMemcpyAsync(d_type.p, d->type, (size_t)n, hipMemcpyHostToDevice, stream));
    PC_HIP(hipMemsetAsync(d_pcnt.p, 0, (size_t)n * 4, stream));
    PC_HIP(hipMemsetAsync(d_cursor.p, 0, (size_t)n * 4, stream));

    // 1. transpose the child lists; 2. sort every parent list and cut it into per-layer runs
    hipLaunchKernelGGL(k_edge_src, dim3(blocks_for(n)), dim3(256), 0, stream, d_ptr.p, n, d_src.p);
    hipLaunchKernelGGL(k_count_parents, dim3(blocks_for(E)), dim3(256), 0, stream, d_child.p, E, d_pcnt.p);
    hipLaunchKernelGGL(k_exclusive_scan, dim3(1), dim3(1024), 0, stream, d_pcnt.p, n, d_pptr.p);
    hipLaunchKernelGGL(k_scatter_parents, dim3(blocks_for(E)), dim3(256), 0, stream, d_child.p, E, d_pptr.p, d_cursor.p, d_tp.p);
    hipLaunchKernelGGL(k_sort_parent_lists, dim3(blocks_for(n)), dim3(256), 0, stream, d_pptr.p, n, d_src.p, d_layer.p,
                       d_tp.p, d_runs.p);
    hipLaunchKernelGGL(k_exclusive_scan, dim3(1), dim3(1024), 0, stream, d_runs.p, n, d_rowptr.p);
    int32_t n_brows = 0;
    PC_HIP(hipMemcpyAsync(&n_brows, d_rowptr.p + n, 4, hipMemcpyDeviceToHost, stream));
    PC_HIP(hipStreamSynchronize(stream));

    DevBuf<int32_t> d_rlayer, d_rchild, d_rstart, d_rcnt;
    PC_HIP(d_rlayer.alloc(n_brows)); PC_HIP(d_rchild.alloc(n_brows)); PC_HIP(d_rstart.alloc(n_brows)); PC_HIP(d_rcnt.alloc(n_brows));
    hipLaunchKernelGGL(k_emit_rows, dim3(blocks_for(n)), dim3(256), 0, stream, d_pptr.p, n, d_src.p, d_layer.p, d_tp.p,
                       d_rowptr.p, d_rlayer.p, d_rchild.p, d_rstart.p, d_rcnt.p);
    std::vector<int32_t> rlayer(n_brows), rchild(n_brows), rcnt(n_brows);
    if (n_brows) {
        PC_HIP(hipMemcpyAsync(rlayer.data(), d_rlayer.p, (size_t)n_brows * 4, hipMemcpyDeviceToHost, stream));
        PC_HIP(hipMemcpyAsync(rchild.data(), d_rchild.p, (size_t)n_brows * 4, hipMemcpyDeviceToHost, stream));
        PC_HIP(hipMemcpyAsync(rcnt.data(), d_rcnt.p, (size_t)n_brows * 4, hipMemcpyDeviceToHost, stream));
    }
    PC_HIP(hipStreamSynchronize(stream));

    // host: O(#rows) grouping (Alg. 2) of forward rows (blocks) and backward rows (runs), layer by layer
    std::vector<int32_t> f_grp(n, -1), f_rank(n, 0);
    std::vector<int32_t> b_grp(n_brows, -1), b_rank(n_brows, 0);
    std::vector<std::vector<int32_t>> rows_of_layer(c->layers.size());
    for (int32_t r = 0; r < n_brows; ++r) rows_of_layer[rlayer[r]].push_back(r);   // rows ascend by child inside a layer
    for (size_t li = 1; li < c->layers.size(); ++li) {
        LayerTab &L = c->layers[li];
        std::vector<int32_t> counts, grp, rank;
        for (int32_t id : L.blk_ids) { const int32_t u = id / K - 1; counts.push_back(ptr32[u + 1] - ptr32[u]); }
        assign_groups(counts, d->max_groups, d->tol_permille, L.fwd, grp, rank);
        for (size_t i = 0; i < L.blk_ids.size(); ++i) { const int32_t u = L.blk_ids[i] / K - 1; f_grp[u] = grp[i]; f_rank[u] = rank[i]; }
        for (GroupTab &g : L.fwd) g.aux.assign(g.n_rows, 0);
        for (size_t i = 0; i < L.blk_ids.size(); ++i) L.fwd[grp[i]].aux[rank[i]] = counts[i] << AUX_COUNT_SHIFT;
        for (GroupTab &g : L.fwd) g.tied_in_group = L.kind == KIND_SUM;       // conservative: only the generic kernels look at it
        std::vector<int32_t> &rows = rows_of_layer[li];
        std::sort(rows.begin(), rows.end(), [&](int32_t a, int32_t b) { return rchild[a] < rchild[b]; });
        counts.clear();
        for (int32_t r : rows) counts.push_back(rcnt[r]);
        assign_groups(counts, d->max_groups, d->tol_permille, L.bwd, grp, rank);
        for (size_t i = 0; i < rows.size(); ++i) { b_grp[rows[i]] = grp[i]; b_rank[rows[i]] = rank[i]; }
        for (GroupTab &g : L.bwd) g.aux.assign(g.n_rows, 0);
        for (size_t i = 0; i < rows.size(); ++i) {
            const int32_t ch = rchild[rows[i]];
            L.bwd[grp[i]].aux[rank[i]] = (counts[i] << AUX_COUNT_SHIFT) |
                                         bwd_row_flags(L.kind, d->type[ch], L.depth, c->an_last_parent_depth[ch],
                                                       c->an_first_parent_depth[ch]);
        }
    }

    pc_status st = upload(c, stream);                                  // arena: every group now has its size
    if (st != PC_OK) return st;

    // where each row goes
    std::vector<int32_t *> f_ids(n, nullptr), f_nbr(n, nullptr), f_par(n, nullptr);
    std::vector<int32_t> f_w(n, 0);
    std::vector<int32_t *> b_ids(n_brows, nullptr), b_nbr(n_brows, nullptr), b_par(n_brows, nullptr);
    std::vector<int32_t> b_w(n_brows, 0);
    for (size_t li = 1; li < c->layers.size(); ++li) {
        LayerTab &L = c->layers[li];
        for (int32_t id : L.blk_ids) {
            const int32_t u = id / K - 1;
            GroupTab &g = L.fwd[f_grp[u]];
            f_ids[u] = g.d_ids + f_rank[u]; f_nbr[u] = g.d_nbr + (int64_t)f_rank[u] * g.width;
            f_par[u] = g.d_par + (int64_t)f_rank[u] * g.width; f_w[u] = g.width;
        }
        for (int32_t r : rows_of_layer[li]) {
            GroupTab &g = L.bwd[b_grp[r]];
            b_ids[r] = g.d_ids + b_rank[r]; b_nbr[r] = g.d_nbr + (int64_t)b_rank[r] * g.width;
            b_par[r] = g.d_par + (int64_t)b_rank[r] * g.width; b_w[r] = g.width;
        }
    }
    DevBuf<int32_t *> d_fids, d_fnbr, d_fpar, d_bids, d_bnbr, d_bpar;
    DevBuf<int32_t> d_fw, d_bw;
    PC_HIP(d_fids.alloc(n)); PC_HIP(d_fnbr.alloc(n)); PC_HIP(d_fpar.alloc(n)); PC_HIP(d_fw.alloc(n));
    PC_HIP(d_bids.alloc(n_brows)); PC_HIP(d_bnbr.alloc(n_brows)); PC_HIP(d_bpar.alloc(n_brows)); PC_HIP(d_bw.alloc(n_brows));
    PC_HIP(hipMemcpyAsync(d_fids.p, f_ids.data(), (size_t)n * sizeof(int32_t *), hipMemcpyHostToDevice, stream));
    PC_HIP(hipMemcpyAsync(d_fnbr.p, f_nbr.data(), (size_t)n * sizeof(int32_t *), hipMemcpyHostToDevice, stream));
    PC_HIP(hipMemcpyAsync(d_fpar.p, f_par.data(), (size_t)n * sizeof(int32_t *), hipMemcpyHostToDevice, stream));
    PC_HIP(hipMemcpyAsync(d_fw.p, f_w.data(), (size_t)n * 4, hipMemcpyHostToDevice, stream));
    if (n_brows) {
        PC_HIP(hipMemcpyAsync(d_bids.p, b_ids.data(), (size_t)n_brows * sizeof(int32_t *), hipMemcpyHostToDevice, stream));
        PC_HIP(hipMemcpyAsync(d_bnbr.p, b_nbr.data(), (size_t)n_brows * sizeof(int32_t *), hipMemcpyHostToDevice, stream));
        PC_HIP(hipMemcpyAsync(d_bpar.p, b_par.data(), (size_t)n_brows * sizeof(int32_t *), hipMemcpyHostToDevice, stream));
        PC_HIP(hipMemcpyAsync(d_bw.p, b_w.data(), (size_t)n_brows * 4, hipMemcpyHostToDevice, stream));
    }
    // 3. fill
    hipLaunchKernelGGL(k_fill_forward, dim3(blocks_for(n)), dim3(256), 0, stream, d_ptr.p, n, d_child.p, d_param.p, d_type.p, K,
                       d_fids.p, d_fnbr.p, d_fpar.p, d_fw.p);
    if (n_brows)
        hipLaunchKernelGGL(k_fill_backward, dim3(blocks_for(n_brows)), dim3(256), 0, stream, n_brows, d_rchild.p, d_rstart.p,
                           d_rcnt.p, d_tp.p, d_src.p, d_param.p, d_type.p, K, d_bids.p, d_bnbr.p, d_bpar.p, d_bw.p);
    PC_HIP(hipGetLastError());
    PC_HIP(hipStreamSynchronize(stream));                               // temporaries are freed on return
    c->an_depth.clear(); c->an_last_parent_depth.clear(); c->an_first_parent_depth.clear();
    return PC_OK;
}

}  // namespace pc
