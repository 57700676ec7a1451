// HIP kernels (gfx950) and their launchers for the layered forward / backward passes.
//
// Node buffers are row-major [node offset][sample], samples contiguous (l_prod in R^{N x B},
// l_sum in R^{M x B} of Sec. 4.3), row stride Bs = B rounded up to 32.
//
// Log-probabilities are kept as  log p(node, b) = R[block, b] + l[node, b]:  R is an integer-valued
// float per (block, sample) and l a small fp32 residual.  Deep circuits reach log-probabilities of
// -10^4 and below, where one fp32 holds only ~1e-3 absolute -- too coarse for the ratios p_c / p_n of
// Def. 2.  Product blocks renormalise (R = sum of the children's R + round(column max), l = rest);
// a sum block takes R = max of its children's R; differences of R are exact, so every exp() below
// sees a small, accurately known argument.  The paper stores plain fp32 log-probabilities.
//
// Sum layers use v_mfma_f32_32x32x2_f32.  Operand layout of that instruction (wave64):
//   A (32 x 2): lane holds A[i = lane % 32][k = lane / 32]
//   B (2 x 32): lane holds B[k = lane / 32][j = lane % 32]
//   D (32 x 32): register r of a lane holds D[i = 8 * (r / 4) + 4 * (lane / 32) + r % 4][j = lane % 32]
// With sum nodes on i and samples on j, every lane owns one sample column, so the per-sample
// running maximum of the log-sum-exp is a per-lane scalar.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <atomic>
#include <cmath>
#include <cstdint>
#include <cstring>

#include "pc_kernels.h"

namespace pc {

typedef float floatx16 __attribute__((ext_vector_type(16)));
typedef float floatx4 __attribute__((ext_vector_type(4)));

#define PC_NEG_INF (-__builtin_inff())
// Sum-layer terms are theta * exp(value - running maximum + PC_UP).  The maximum is taken over the values alone (as in
// Alg. 1 / Alg. 4), so without the upward shift a term with a large weight whose value lies 87 nats below that of a
// child with a weight near FLT_MIN would be flushed to zero although it dominates the sum.  With it every term or
// factor that underflows is at least e^-20 smaller than the largest term kept, and nothing can overflow.  The shift
// is kept small because the result is  maximum - PC_UP + log(sum): the larger the two cancelling parts, the larger
// the absolute rounding error of a log-probability near zero.
#define PC_UP 20.0f
// Rescaling an accumulator when the running maximum grows by -delta: the factor exp(delta) itself may leave the
// fp32 range where accumulator * factor does not (the accumulator can be as large as e^28 times the term count),
// so the factor is applied as two multiplications by exp(delta / 2); below delta = -174 the result is nil anyway.
__device__ inline float pc_half_scale(float delta) { return __expf(0.5f * fmaxf(delta, -174.0f)); }
// The running maximum is only a reference: it is raised (and the accumulator rescaled) when a chunk exceeds it by
// more than PC_LAZY nats, not at every new maximum -- with 64 columns per wave some column has a new maximum in
// almost every chunk, and the rescale costs a multiplication per accumulator register.  Terms reach e^(PC_UP + PC_LAZY).
#define PC_LAZY 8.0f

// ------------------------------------------------------------------------------------------
// small utility kernels
// ------------------------------------------------------------------------------------------
__global__ void k_fill(float *p, int64_t n, float v)
{
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += stride) p[i] = v;
}

// xT[v][b] = category, -1 if marginalised (mask, or padding column b >= B), -2 if out of range.
__global__ void k_prepare_x(const int32_t *__restrict__ x, const uint8_t *__restrict__ mask, int32_t B, int32_t D,
                            int64_t Bs, int32_t n_cats, int32_t *__restrict__ xT)
{
    __shared__ int32_t tile[32][33];
    const int b0 = blockIdx.x * 32, v0 = blockIdx.y * 32;
    const int tx = threadIdx.x & 31, ty = threadIdx.x >> 5;           // 256 threads: ty in 0..7
    for (int r = ty; r < 32; r += 8) {
        const int b = b0 + r, v = v0 + tx;
        int32_t val = -1;
        if (b < B && v < D) {
            const int64_t idx = (int64_t)b * D + v;
            val = x[idx];
            if (val < 0 || val >= n_cats) val = -2;
            if (mask && mask[idx]) val = -1;
        }
        tile[r][tx] = val;
    }
    __syncthreads();
    for (int r = ty; r < 32; r += 8) {
        const int v = v0 + r, b = b0 + tx;
        if (v < D && b < Bs) xT[(int64_t)v * Bs + b] = tile[tx][r];
    }
}

__global__ void k_readout(const float *__restrict__ l, const float *__restrict__ R, int64_t root_row, int64_t root_blk,
                          int64_t Bs, int32_t B, float *__restrict__ ll)
{
    const int b = blockIdx.x * blockDim.x + threadIdx.x;
    if (b < B) ll[b] = R[root_blk * Bs + b] + l[root_row * Bs + b];
}

// ------------------------------------------------------------------------------------------
// input layer (categorical): l[n,b] = log table[t][x_b,v][k]
// ------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void k_input_fwd(const float *__restrict__ tables, const int32_t *__restrict__ xT,
                                                   const int32_t *__restrict__ ids, const int32_t *__restrict__ var,
                                                   const int32_t *__restrict__ tab, int32_t K, int32_t n_cats,
                                                   int64_t Bs, float *__restrict__ l)
{
    const int u = blockIdx.x;
    const int64_t b = (int64_t)blockIdx.y * 256 + threadIdx.x;
    if (b >= Bs) return;
    const int32_t xv = xT[(int64_t)var[u] * Bs + b];
    float *out = l + (int64_t)ids[u] * Bs + b;
    if (xv < 0) {
        const float v = xv == -1 ? 0.0f : PC_NEG_INF;
        for (int k = 0; k < K; ++k) out[(int64_t)k * Bs] = v;
        return;
    }
    const float *row = tables + ((int64_t)tab[u] * n_cats + xv) * K;
    if ((K & 3) == 0) {
        for (int k = 0; k < K; k += 4) {
            const float4 t = *reinterpret_cast<const float4 *>(row + k);
            out[(int64_t)(k + 0) * Bs] = __logf(t.x);
            out[(int64_t)(k + 1) * Bs] = __logf(t.y);
            out[(int64_t)(k + 2) * Bs] = __logf(t.z);
            out[(int64_t)(k + 3) * Bs] = __logf(t.w);
        }
    } else {
        for (int k = 0; k < K; ++k) out[(int64_t)k * Bs] = __logf(row[k]);
    }
}

// The same through an LDS tile, for K a multiple of 4: one workgroup per (block, 64 samples).  K / 4 lanes fetch one
// sample's table row with 16-byte loads (every global read is a whole contiguous row), the logs go into a
// [K x 64] tile, and the tile leaves as 16-byte stores along the batch -- no access is narrower than a row.
__global__ __launch_bounds__(256) void k_input_fwd_tile(const float *__restrict__ tables, const int32_t *__restrict__ xT,
                                                        const int32_t *__restrict__ ids, const int32_t *__restrict__ var,
                                                        const int32_t *__restrict__ tab, int32_t K, int32_t n_cats,
                                                        int64_t Bs, float *__restrict__ l)
{
    extern __shared__ float smem[];
    float *tile = smem;                                                 // [K][65]
    int *cats = reinterpret_cast<int *>(tile + K * 65);
    const int u = blockIdx.x;
    const int64_t b0 = (int64_t)blockIdx.y * 64;
    if (threadIdx.x < 64) cats[threadIdx.x] = (b0 + threadIdx.x < Bs) ? xT[(int64_t)var[u] * Bs + b0 + threadIdx.x] : -1;
    __syncthreads();
    const int lps = K / 4;                                              // lanes per sample
    const float *tbase = tables + (int64_t)tab[u] * n_cats * K;
    for (int idx = threadIdx.x; idx < 64 * lps; idx += 256) {
        const int sidx = idx / lps, kl = idx - sidx * lps;
        const int xv = cats[sidx];
        float4 t;
        if (xv >= 0) {
            const float4 r = *reinterpret_cast<const float4 *>(tbase + (int64_t)xv * K + kl * 4);
            t = make_float4(__logf(r.x), __logf(r.y), __logf(r.z), __logf(r.w));
        } else {
            const float v = xv == -1 ? 0.0f : PC_NEG_INF;               // marginalised / tail : out-of-range category
            t = make_float4(v, v, v, v);
        }
        float *dst = tile + (kl * 4) * 65 + sidx;
        dst[0] = t.x; dst[65] = t.y; dst[130] = t.z; dst[195] = t.w;
    }
    __syncthreads();
    const int32_t id = ids[u];
    for (int idx = threadIdx.x; idx < K * 16; idx += 256) {
        const int row = idx >> 4, c4 = (idx & 15) * 4;
        if (b0 + c4 < Bs) {
            const float *src = tile + row * 65 + c4;
            *reinterpret_cast<float4 *>(l + (int64_t)(id + row) * Bs + b0 + c4) = make_float4(src[0], src[1], src[2], src[3]);
        }
    }
}

// table_flow[t][x_b,v][k] += F[n,b] for observed variables.
// The first two variants bring a [K rows x 64 samples] tile of the flow buffer into LDS with coalesced 16-byte
// loads along the batch, then turn it: a group of lanes owns consecutive nodes k of ONE sample, so every add
// touches consecutive floats of one table row.
//   hist : one workgroup per input block; the adds go into an LDS copy of the block's [n_cats x K] table slice
//          (LDS float atomics), flushed once with coalesced read-modify-writes (atomics only if the table is
//          shared by several blocks).  Used when the slice fits in LDS.
//   direct: one workgroup per (block, 64 samples); global float atomics, 64 consecutive floats per wave op.
//   sorted: below; used for tables of up to 1024 categories when hist does not apply.
__device__ inline void input_bwd_load_tile(const float *__restrict__ F, const int32_t *__restrict__ xT, int32_t id,
                                           int32_t var, int32_t K, int64_t Bs, int64_t b0, float *tile, int *cats)
{
    for (int idx = threadIdx.x; idx < K * 16; idx += 256) {
        const int row = idx >> 4, c4 = (idx & 15) * 4;
        float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
        if (b0 + c4 < Bs) v = *reinterpret_cast<const float4 *>(F + (int64_t)(id + row) * Bs + b0 + c4);
        float *dst = tile + row * 65 + c4;
        dst[0] = v.x; dst[1] = v.y; dst[2] = v.z; dst[3] = v.w;
    }
    if (threadIdx.x < 64) cats[threadIdx.x] = (b0 + threadIdx.x < Bs) ? xT[(int64_t)var * Bs + b0 + threadIdx.x] : -1;
}

__global__ __launch_bounds__(256) void k_input_bwd_hist(const float *__restrict__ F, const int32_t *__restrict__ xT,
                                                        const int32_t *__restrict__ ids, const int32_t *__restrict__ var,
                                                        const int32_t *__restrict__ tab, int32_t K, int32_t n_cats,
                                                        int64_t Bs, float *__restrict__ table_flow, int lps, int atomic_flush)
{
    extern __shared__ float smem[];
    float *hist = smem, *tile = smem + (size_t)n_cats * K;
    int *cats = reinterpret_cast<int *>(tile + K * 65);
    const int u = blockIdx.x;
    const int32_t id = ids[u];
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int spi = 64 / lps;                                          // samples per wave instruction
    const int kl = lane % lps, sl = lane / lps;
    for (int i = threadIdx.x; i < n_cats * K; i += 256) hist[i] = 0.0f;
    for (int64_t b0 = 0; b0 < Bs; b0 += 64) {
        __syncthreads();
        input_bwd_load_tile(F, xT, id, var[u], K, Bs, b0, tile, cats);
        __syncthreads();
        for (int s = wave * spi + sl; s < 64; s += 4 * spi) {
            const int cat = cats[s];
            if (cat < 0) continue;
            for (int k = kl; k < K; k += lps) {
                const float f = tile[k * 65 + s];
                if (f != 0.0f) atomicAdd(hist + cat * K + k, f);
            }
        }
    }
    __syncthreads();
    float *dst = table_flow + (int64_t)tab[u] * n_cats * K;
    for (int i = threadIdx.x; i < n_cats * K; i += 256) {
        const float v = hist[i];
        if (v != 0.0f) { if (atomic_flush) atomicAdd(dst + i, v); else dst[i] += v; }
    }
}

__global__ __launch_bounds__(256) void k_input_bwd_direct(const float *__restrict__ F, const int32_t *__restrict__ xT,
                                                          const int32_t *__restrict__ ids, const int32_t *__restrict__ var,
                                                          const int32_t *__restrict__ tab, int32_t K, int32_t n_cats,
                                                          int64_t Bs, float *__restrict__ table_flow, int lps)
{
    extern __shared__ float smem[];
    float *tile = smem;
    int *cats = reinterpret_cast<int *>(tile + K * 65);
    const int u = blockIdx.x;
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int spi = 64 / lps;
    const int kl = lane % lps, sl = lane / lps;
    input_bwd_load_tile(F, xT, ids[u], var[u], K, Bs, (int64_t)blockIdx.y * 64, tile, cats);
    __syncthreads();
    float *base = table_flow + (int64_t)tab[u] * n_cats * K;
    for (int s = wave * spi + sl; s < 64; s += 4 * spi) {
        const int cat = cats[s];
        if (cat < 0) continue;
        for (int k = kl; k < K; k += lps) {
            const float f = tile[k * 65 + s];
            if (f != 0.0f) atomicAdd(base + (int64_t)cat * K + k, f);
        }
    }
}

// Third variant, for tables with at most 1024 categories: one workgroup per (input block, slab of SB samples).
// The slab's samples are ordered by category with a counting sort in LDS; the block's [K x SB] flows are brought
// into an LDS tile with the columns in that order, so the samples of a category sit side by side, and every category
// that occurs gets ONE add per node -- the sum over its samples -- instead of one per sample.  The adds that remain
// are atomic even where the workgroup is the only writer of its rows: an atomic is sent and forgotten, a plain
// read-modify-write waits for its read (measured: 0.87 against 0.55 ms on 12 K blocks).  The order of the samples of
// a category is whatever the sort's atomics gave, so sums may differ in the last bit between runs, as with the
// other variants.
__global__ __launch_bounds__(256) void k_input_bwd_sorted(const float *__restrict__ F, const int32_t *__restrict__ xT,
                                                          const int32_t *__restrict__ ids, const int32_t *__restrict__ var,
                                                          const int32_t *__restrict__ tab, int32_t K, int32_t n_cats,
                                                          int64_t Bs, float *__restrict__ table_flow, int SB, int lpc)
{
    extern __shared__ float smem[];
    const int LDT = SB + 1;                                             // odd row stride: column reads conflict-free
    float *tile = smem;                                                 // [K][SB + 1], columns ordered by category
    int *cats = reinterpret_cast<int *>(tile + (size_t)K * LDT);        // [SB] category of a sample, < 0: no flow
    int *pos = cats + SB;                                               // [SB] column of a sample in the tile, -1: none
    int *start = pos + SB;                                              // [n_cats + 1] counts, then segment starts
    int *wsum = start + n_cats + 1;                                     // [4] scan scratch
    const int u = blockIdx.x, tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
    const int64_t b0 = (int64_t)blockIdx.y * SB;
    const int nb = (int)((Bs - b0) < SB ? (Bs - b0) : SB);              // samples of this slab (a multiple of 32)
    const int32_t id = ids[u];

    for (int c = tid; c <= n_cats; c += 256) start[c] = 0;
    for (int i = tid; i < nb; i += 256) cats[i] = xT[(int64_t)var[u] * Bs + b0 + i];
    __syncthreads();
    // counting sort: rank inside the category, counts -> exclusive scan -> columns
    int rank[4];                                                        // SB <= 1024: at most 4 samples per thread
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        const int i = tid + 256 * j;
        rank[j] = (i < nb && cats[i] >= 0) ? atomicAdd(start + cats[i], 1) : 0;
    }
    __syncthreads();
    const int per = (n_cats + 255) / 256;                               // categories per thread (<= 4)
    int loc[4], tot = 0;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        const int c = tid * per + j;
        loc[j] = (j < per && c < n_cats) ? start[c] : 0;
        tot += loc[j];
    }
    int incl = tot;                                                     // inclusive scan over the wave, then over the 4 waves
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) {
        const int v = __shfl_up(incl, off);
        if (lane >= off) incl += v;
    }
    if (lane == 63) wsum[wave] = incl;
    __syncthreads();
    int run = incl - tot;
    for (int w2 = 0; w2 < wave; ++w2) run += wsum[w2];
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        const int c = tid * per + j;
        if (j < per && c < n_cats) { start[c] = run; run += loc[j]; }
    }
    if (tid == 255) start[n_cats] = run;
    __syncthreads();
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        const int i = tid + 256 * j;
        if (i < nb) pos[i] = cats[i] >= 0 ? start[cats[i]] + rank[j] : -1;
    }
    __syncthreads();
    // flows of the block: 16-byte loads along the batch, columns scattered into category order
    // (eight loads in flight per thread: a load waited for on its own costs a trip to HBM)
    const int n4 = nb / 4, total = K * n4;
    for (int base0 = tid; base0 < total; base0 += 256 * 8) {
        float4 v[8];
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            const int idx = base0 + 256 * j;
            const int row = idx / n4, c4 = (idx - row * n4) * 4;
            v[j] = idx < total ? *reinterpret_cast<const float4 *>(F + (int64_t)(id + row) * Bs + b0 + c4)
                               : make_float4(0.f, 0.f, 0.f, 0.f);
        }
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            const int idx = base0 + 256 * j;
            if (idx >= total) break;
            const int row = idx / n4, c4 = (idx - row * n4) * 4;
            float *dst = tile + row * LDT;
            const int p0 = pos[c4], p1 = pos[c4 + 1], p2 = pos[c4 + 2], p3 = pos[c4 + 3];
            if (p0 >= 0) dst[p0] = v[j].x;
            if (p1 >= 0) dst[p1] = v[j].y;
            if (p2 >= 0) dst[p2] = v[j].z;
            if (p3 >= 0) dst[p3] = v[j].w;
        }
    }
    __syncthreads();
    // one group of lpc lanes per category at a time; a lane owns nodes k, k + lpc, ...
    const int grp = tid / lpc, kl = tid % lpc, n_grp = 256 / lpc;
    float *base = table_flow + (int64_t)tab[u] * n_cats * K;
    for (int c = grp; c < n_cats; c += n_grp) {
        const int s0 = start[c], s1 = start[c + 1];
        if (s0 == s1) continue;
        for (int k = kl; k < K; k += lpc) {
            const float *src = tile + k * LDT;
            float a0 = 0.0f, a1 = 0.0f, a2 = 0.0f, a3 = 0.0f;
            int sidx = s0;
            for (; sidx + 4 <= s1; sidx += 4) { a0 += src[sidx]; a1 += src[sidx + 1]; a2 += src[sidx + 2]; a3 += src[sidx + 3]; }
            for (; sidx < s1; ++sidx) a0 += src[sidx];
            const float acc = (a0 + a1) + (a2 + a3);
            if (acc != 0.0f) atomicAdd(base + (int64_t)c * K + k, acc);
        }
    }
}

// Group of launch row `row` in a set (wave-uniform).  Kernels are instantiated for one group (MULTI = false: the deep
// narrow circuits, where anything extra shows in a launch of a few microseconds) and for several: there the group
// index is found with a few scalar compares and the group's fields are read from the argument at that index (one
// more dependent scalar load, which launches with several groups -- thousands of workgroups -- hide).
struct GroupRow { int32_t r, width; const int32_t *ids, *nbr, *par, *aux; };
template <bool MULTI>
__device__ inline GroupRow locate_row(const GroupSet &gs, int row)
{
    if (!MULTI) return GroupRow{row, gs.width[0], gs.ids[0], gs.nbr[0], gs.par[0], gs.aux[0]};   // a set of one group
    int g = 0;                                                          // groups are in row order: count the starts passed
#pragma unroll
    for (int i = 1; i < PC_MAX_SET; ++i) g += (i < gs.n && row >= gs.first[i]) ? 1 : 0;
    return GroupRow{row - gs.first[g], gs.width[g], gs.ids[g], gs.nbr[g], gs.par[g], gs.aux[g]};
}

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef float floatx2 __attribute__((ext_vector_type(2)));

__device__ inline void bf16_split2(float a, float b, uint32_t &hi, uint32_t &lo)
{
    const floatx2 v = {a, b};
    const bf16x2 h = __builtin_convertvector(v, bf16x2);               // round to nearest even
    const floatx2 hf = __builtin_convertvector(h, floatx2);
    const bf16x2 l = __builtin_convertvector(v - hf, bf16x2);
    hi = __builtin_bit_cast(uint32_t, h);
    lo = __builtin_bit_cast(uint32_t, l);
}

// One 1 KiB tile of the value planes read by the bf16 sum kernels (see there): exp(X + sh) of 16 node rows x 32 columns,
// split into hi and lo bf16 values; lane (j = lane % 32, h = lane / 32) owns rows 8 h .. 8 h + 7 of column j.  `sh` is
// the lane's shift (per column), -inf for a column without flow.  row0 = first node row of the slice.
// `src` points at the lane's column in the slice's first row (global rows, or a tile in LDS), `ld` is its row stride.
__device__ inline void split_value_rows(const float *src, int64_t ld, float sh, int64_t row0, int ct, int n_ct,
                                        uint4 *__restrict__ Ph, uint4 *__restrict__ Pl, int lane)
{
    const int h = lane >> 5;
    float v[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) v[e] = __expf(src[(8 * h + e) * ld] + sh);
    uint32_t hi[4], lo[4];
#pragma unroll
    for (int e = 0; e < 4; ++e) bf16_split2(v[2 * e], v[2 * e + 1], hi[e], lo[e]);
    const int64_t tile = (row0 / 16) * n_ct + ct;
    Ph[tile * 64 + lane] = make_uint4(hi[0], hi[1], hi[2], hi[3]);
    Pl[tile * 64 + lane] = make_uint4(lo[0], lo[1], lo[2], lo[3]);
}
__device__ inline void split_value_tile(const float *__restrict__ X, float sh, int64_t row0, int ct, int n_ct, int64_t Bs,
                                        uint4 *__restrict__ Ph, uint4 *__restrict__ Pl, int lane)
{
    split_value_rows(X + row0 * Bs + (int64_t)ct * 32 + (lane & 31), Bs, sh, row0, ct, n_ct, Ph, Pl, lane);
}

// ------------------------------------------------------------------------------------------
// product layers: forward adds child log-probs (Sec. 3); backward adds parent flows (Def. 2)
// ------------------------------------------------------------------------------------------
// Block-wise product kernels.  Workgroup = one node block x 64 sample columns; thread (rg, cl) owns rows
// rg, rg+16, ... of 4 adjacent columns (16-byte accesses along the batch), so a K-row block is K/16 rows
// deep per thread and all its loads are independent.  Column maxima over the K rows go through one
// shuffle stage (4 row groups per wave) and one LDS stage (4 waves).
template <int CL>
__device__ inline void block_col_max(float (&mx)[4], float (*red)[64], int wave, int cl)
{
#pragma unroll
    for (int v = 0; v < 4; ++v) {
        if (CL == 8) mx[v] = fmaxf(mx[v], __shfl_xor(mx[v], 8));
        mx[v] = fmaxf(mx[v], __shfl_xor(mx[v], 16));
        mx[v] = fmaxf(mx[v], __shfl_xor(mx[v], 32));
    }
    if ((threadIdx.x & 63) < CL) {
#pragma unroll
        for (int v = 0; v < 4; ++v) red[wave][cl * 4 + v] = mx[v];
    }
    __syncthreads();
#pragma unroll
    for (int v = 0; v < 4; ++v) {
        const int c = cl * 4 + v;
        mx[v] = fmaxf(fmaxf(red[0][c], red[1][c]), fmaxf(red[2][c], red[3][c]));
    }
}

// Both kernels walk the row's real neighbours (count in the row's flag word) U at a time: the U neighbour ids are
// fetched first, then all their loads are issued together, so a row costs one memory round trip per U neighbours
// instead of one per neighbour (small layers are latency-bound).  RPT = rows per thread = ceil(K / 16).

// forward (Sec. 3): s = sum of the children's residuals; the column maximum over the K rows is rounded to an
// integer and moved into R.  ACC = double for rows with many children (a leaf product over 98 pixels adds up to
// -540, where one fp32 step is 6e-5: summed in fp32 the residuals -- and with them every flow ratio p_c / p_n below --
// would be off by up to 1e-3); the rounded maximum is subtracted in that precision, the small residual is stored as fp32.
template <typename ACC> struct Acc4 { ACC x, y, z, w; };
// `l` is the base the children are read from, `lout` the base the block's own rows are written to: the same buffer,
// except in the product-scratch mode (Sec. 5), where product rows live in a window that every product layer reuses.
template <int RPT, int U, bool MULTI, int CL, typename ACC, bool PLANES>
__global__ __launch_bounds__(256) void k_prod_fwd(const float *__restrict__ l, float *__restrict__ lout, float *__restrict__ R,
                                                  const GroupSet gs, int32_t K, int64_t Bs, uint4 *__restrict__ Ph,
                                                  uint4 *__restrict__ Pl)
{
    __shared__ float red[4][64];
    const GroupRow gr = locate_row<MULTI>(gs, blockIdx.x);
    const int r = gr.r;
    constexpr int RG = 256 / CL;                                        // row groups: a thread owns rows rg, rg + RG, ...
    const int rg = threadIdx.x / CL, cl = threadIdx.x % CL, wave = threadIdx.x >> 6;
    const int64_t b = (int64_t)blockIdx.y * (4 * CL) + cl * 4;
    const bool in = b < Bs;                                            // Bs is a multiple of 32: b..b+3 all inside
    const int32_t *row_nbr = gr.nbr + (int64_t)r * gr.width;
    const int32_t cnt = gr.aux[r] >> 8;
    const int32_t id = gr.ids[r];
    Acc4<ACC> s[RPT];
    float mx[4] = {PC_NEG_INF, PC_NEG_INF, PC_NEG_INF, PC_NEG_INF};
    float4 rsum = make_float4(0.f, 0.f, 0.f, 0.f);
#pragma unroll
    for (int i = 0; i < RPT; ++i) s[i] = Acc4<ACC>{0, 0, 0, 0};
    if (in) {
        for (int j0 = 0; j0 < cnt; j0 += U) {
            int32_t ch[U];
#pragma unroll
            for (int u = 0; u < U; ++u) ch[u] = j0 + u < cnt ? row_nbr[j0 + u] : 0;
            float4 t[U][RPT], tr[U];
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const bool on = j0 + u < cnt;                          // uniform over the workgroup
#pragma unroll
                for (int i = 0; i < RPT; ++i) {
                    const int k = rg + RG * i;
                    t[u][i] = (on && k < K) ? *reinterpret_cast<const float4 *>(l + (int64_t)(ch[u] + k) * Bs + b)
                                            : make_float4(0.f, 0.f, 0.f, 0.f);
                }
                tr[u] = (on && rg == 0) ? *reinterpret_cast<const float4 *>(R + (int64_t)(ch[u] / K) * Bs + b)
                                        : make_float4(0.f, 0.f, 0.f, 0.f);
            }
            // the U values of a round are added in fp32, the rounds in ACC (double for rows of many children: a running
            // fp32 sum of a hundred residuals loses more than the flows' tolerance allows, a sum of U does not)
#pragma unroll
            for (int i = 0; i < RPT; ++i) {
                float4 part = t[0][i];
#pragma unroll
                for (int u = 1; u < U; ++u) { part.x += t[u][i].x; part.y += t[u][i].y; part.z += t[u][i].z; part.w += t[u][i].w; }
                s[i].x += (ACC)part.x; s[i].y += (ACC)part.y; s[i].z += (ACC)part.z; s[i].w += (ACC)part.w;
            }
#pragma unroll
            for (int u = 0; u < U; ++u) { rsum.x += tr[u].x; rsum.y += tr[u].y; rsum.z += tr[u].z; rsum.w += tr[u].w; }
        }
#pragma unroll
        for (int i = 0; i < RPT; ++i)
            if (rg + RG * i < K) {
                mx[0] = fmaxf(mx[0], (float)s[i].x); mx[1] = fmaxf(mx[1], (float)s[i].y);
                mx[2] = fmaxf(mx[2], (float)s[i].z); mx[3] = fmaxf(mx[3], (float)s[i].w);
            }
    }
    block_col_max<CL>(mx, red, wave, cl);
    if (!PLANES && !in) return;
    float sh4[4];
#pragma unroll
    for (int v = 0; v < 4; ++v) sh4[v] = mx[v] > PC_NEG_INF ? rintf(mx[v]) : 0.0f;
    if (in) {
        const float (&sh)[4] = sh4;
        if (rg == 0)
            *reinterpret_cast<float4 *>(R + (int64_t)(id / K) * Bs + b) = make_float4(rsum.x + sh[0], rsum.y + sh[1], rsum.z + sh[2], rsum.w + sh[3]);
#pragma unroll
        for (int i = 0; i < RPT; ++i) {
            const int k = rg + RG * i;
            if (k < K)
                *reinterpret_cast<float4 *>(lout + (int64_t)(id + k) * Bs + b) =
                    make_float4((float)(s[i].x - (ACC)sh[0]), (float)(s[i].y - (ACC)sh[1]), (float)(s[i].z - (ACC)sh[2]),
                                (float)(s[i].w - (ACC)sh[3]));
        }
    }
    if (PLANES) {
        // the block's tile again as bf16 operand planes for a sum layer that runs on the bf16 matrix cores (this saves
        // the launch of k_split_p), taken from a copy of the tile in LDS: a lane of the plane layout owns eight rows of one
        // column, a thread here four columns of RPT rows
        constexpr int LDT = 4 * CL + 1;
        __shared__ float ptile[PLANES ? 128 * LDT : 1];
        if (in) {
#pragma unroll
            for (int i = 0; i < RPT; ++i) {
                const int k = rg + RG * i;
                if (k < K) {
                    float *dst = ptile + k * LDT + cl * 4;
                    dst[0] = (float)(s[i].x - (ACC)sh4[0]); dst[1] = (float)(s[i].y - (ACC)sh4[1]);
                    dst[2] = (float)(s[i].z - (ACC)sh4[2]); dst[3] = (float)(s[i].w - (ACC)sh4[3]);
                }
            }
        }
        __syncthreads();
        const int n_ct = (int)(Bs / 32), lane = threadIdx.x & 63;
        constexpr int CTW = CL / 8;                                     // 32-column tiles of the workgroup
        for (int it = wave; it < (K / 16) * CTW; it += 4) {
            const int ks = it / CTW, cw = it % CTW, ct = (int)blockIdx.y * CTW + cw;
            if (ct < n_ct)
                split_value_rows(ptile + 16 * ks * LDT + cw * 32 + (lane & 31), LDT, PC_UP, (int64_t)id + 16 * ks, ct, n_ct, Ph, Pl, lane);
        }
    }
}

// backward (Def. 2): rows = child blocks (sum / input blocks), neighbours = their product parents in this layer;
// F_child += sum of the parents' flows ('=' where this is the first layer that feeds the block, flag bit 1, so
// the flow buffer is never cleared).  Where this layer is the last one that feeds a SUM block (flag bit 0) its
// flow is final, so log_nf = log F - l (Alg. 3 / 4) and its column maximum per block are produced here.
// `Fpar` is the base the parents' (product blocks') flows are read from, `F` the base of the rows' own flows: the same
// buffer, except in the product-scratch mode, where product rows live in a window.
template <int RPT, int U, bool MULTI, int CL, bool PLANES>
__global__ __launch_bounds__(256) void k_prod_bwd(const float *__restrict__ l, float *__restrict__ F, const float *__restrict__ Fpar,
                                                  float *__restrict__ N, float *__restrict__ nfmax, const GroupSet gs, int32_t K,
                                                  int64_t Bs, uint4 *__restrict__ Ph, uint4 *__restrict__ Pl)
{
    __shared__ float red[4][64];
    const GroupRow gr = locate_row<MULTI>(gs, blockIdx.x);
    const int r = gr.r;
    constexpr int RG = 256 / CL;                                        // row groups: a thread owns rows rg, rg + RG, ...
    const int rg = threadIdx.x / CL, cl = threadIdx.x % CL, wave = threadIdx.x >> 6;
    const int64_t b = (int64_t)blockIdx.y * (4 * CL) + cl * 4;
    const bool in = b < Bs;
    const int32_t *row_nbr = gr.nbr + (int64_t)r * gr.width;
    const int32_t id = gr.ids[r];
    const int32_t fl = gr.aux[r];                                       // uniform over the workgroup
    const bool final_flow = (fl & 1) != 0, first = (fl & 2) != 0;
    const int32_t cnt = fl >> 8;
    float4 f[RPT], lv[RPT];
    if (in) {
#pragma unroll
        for (int i = 0; i < RPT; ++i) {
            const int k = rg + RG * i;
            f[i] = (k < K && !first) ? *reinterpret_cast<const float4 *>(F + (int64_t)(id + k) * Bs + b)
                                     : make_float4(0.f, 0.f, 0.f, 0.f);
            // the block's own log-probabilities, needed only for log_nf: fetched with everything else
            lv[i] = (k < K && final_flow) ? *reinterpret_cast<const float4 *>(l + (int64_t)(id + k) * Bs + b)
                                          : make_float4(0.f, 0.f, 0.f, 0.f);
        }
        for (int j0 = 0; j0 < cnt; j0 += U) {
            int32_t pa[U];
#pragma unroll
            for (int u = 0; u < U; ++u) pa[u] = j0 + u < cnt ? row_nbr[j0 + u] : 0;
            float4 t[U][RPT];
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const bool on = j0 + u < cnt;                          // uniform over the workgroup
#pragma unroll
                for (int i = 0; i < RPT; ++i) {
                    const int k = rg + RG * i;
                    t[u][i] = (on && k < K) ? *reinterpret_cast<const float4 *>(Fpar + (int64_t)(pa[u] + k) * Bs + b)
                                            : make_float4(0.f, 0.f, 0.f, 0.f);
                }
            }
#pragma unroll
            for (int u = 0; u < U; ++u)
#pragma unroll
                for (int i = 0; i < RPT; ++i) {
                    f[i].x += t[u][i].x; f[i].y += t[u][i].y; f[i].z += t[u][i].z; f[i].w += t[u][i].w;
                }
        }
#pragma unroll
        for (int i = 0; i < RPT; ++i) {
            const int k = rg + RG * i;
            if (k < K) *reinterpret_cast<float4 *>(F + (int64_t)(id + k) * Bs + b) = f[i];
        }
    }
    if (!final_flow) return;
    float mx[4] = {PC_NEG_INF, PC_NEG_INF, PC_NEG_INF, PC_NEG_INF};
    float4 nfv[PLANES ? RPT : 1];
    if (in) {
#pragma unroll
        for (int i = 0; i < RPT; ++i) {
            const int k = rg + RG * i;
            if (k < K) {
                float4 nf;
                nf.x = (f[i].x > 0.0f && lv[i].x > PC_NEG_INF) ? __logf(f[i].x) - lv[i].x : PC_NEG_INF;
                nf.y = (f[i].y > 0.0f && lv[i].y > PC_NEG_INF) ? __logf(f[i].y) - lv[i].y : PC_NEG_INF;
                nf.z = (f[i].z > 0.0f && lv[i].z > PC_NEG_INF) ? __logf(f[i].z) - lv[i].z : PC_NEG_INF;
                nf.w = (f[i].w > 0.0f && lv[i].w > PC_NEG_INF) ? __logf(f[i].w) - lv[i].w : PC_NEG_INF;
                *reinterpret_cast<float4 *>(N + (int64_t)(id + k) * Bs + b) = nf;
                if (PLANES) nfv[i] = nf;
                mx[0] = fmaxf(mx[0], nf.x); mx[1] = fmaxf(mx[1], nf.y); mx[2] = fmaxf(mx[2], nf.z); mx[3] = fmaxf(mx[3], nf.w);
            }
        }
    }
    block_col_max<CL>(mx, red, wave, cl);
    if (in && rg == 0) *reinterpret_cast<float4 *>(nfmax + (int64_t)(id / K) * Bs + b) = make_float4(mx[0], mx[1], mx[2], mx[3]);
    if (PLANES) {
        // exp(log_nf - column maximum + PC_UP) of the block as bf16 operand planes for a sum layer whose backward pass
        // runs on the bf16 matrix cores (saves the launch of k_split_p), taken from a copy of the tile in LDS (row K: the
        // column maxima)
        constexpr int LDT = 4 * CL + 1;
        __shared__ float ptile[PLANES ? 129 * LDT : 1];
        if (in) {
#pragma unroll
            for (int i = 0; i < RPT; ++i) {
                const int k = rg + RG * i;
                if (k < K) {
                    float *dst = ptile + k * LDT + cl * 4;
                    dst[0] = nfv[i].x; dst[1] = nfv[i].y; dst[2] = nfv[i].z; dst[3] = nfv[i].w;
                }
            }
            if (rg == 0) {
                float *dst = ptile + 128 * LDT + cl * 4;
                dst[0] = mx[0]; dst[1] = mx[1]; dst[2] = mx[2]; dst[3] = mx[3];
            }
        }
        __syncthreads();
        const int n_ct = (int)(Bs / 32), lane = threadIdx.x & 63;
        constexpr int CTW = CL / 8;                                     // 32-column tiles of the workgroup
        for (int it = wave; it < (K / 16) * CTW; it += 4) {
            const int ks = it / CTW, cw = it % CTW, ct = (int)blockIdx.y * CTW + cw;
            if (ct >= n_ct) continue;
            const float top = ptile[128 * LDT + cw * 32 + (lane & 31)];
            split_value_rows(ptile + 16 * ks * LDT + cw * 32 + (lane & 31), LDT, top > PC_NEG_INF ? PC_UP - top : PC_NEG_INF,
                             (int64_t)id + 16 * ks, ct, n_ct, Ph, Pl, lane);
        }
    }
}

// Blocks without parents, which no layer of the backward sweep writes.  An entry >= 0 is a sum block: the root
// (flow 1 on node 0 of real samples with non-zero probability, Def. 2) or a sum block nobody uses (flow 0); its
// log_nf rows and block maximum are set as well.  An entry < 0 is ~offset of another block (the null block, a
// product or input block nobody uses): its flow rows are zeroed.  One workgroup per entry and 256 columns.
__global__ __launch_bounds__(256) void k_init_flows(const float *__restrict__ l, float *__restrict__ F, float *__restrict__ N,
                                                    float *__restrict__ nfmax, const int32_t *__restrict__ blk_ids,
                                                    int32_t root_id, int32_t K, int64_t Bs, int32_t B)
{
    const int32_t entry = blk_ids[blockIdx.x];
    const int64_t b = (int64_t)blockIdx.y * 256 + threadIdx.x;
    if (b >= Bs) return;
    if (entry < 0) {
        const int32_t id = ~entry;
        for (int k = 0; k < K; ++k) F[(int64_t)(id + k) * Bs + b] = 0.0f;
        return;
    }
    const int32_t id = entry;
    float top = PC_NEG_INF, f0 = 0.0f;
    if (id == root_id) {
        const float lv = l[(int64_t)id * Bs + b];
        const bool live = b < B && lv > PC_NEG_INF;
        f0 = live ? 1.0f : 0.0f;
        top = live ? -lv : PC_NEG_INF;
    }
    for (int k = 0; k < K; ++k) {
        F[(int64_t)(id + k) * Bs + b] = k == 0 ? f0 : 0.0f;
        N[(int64_t)(id + k) * Bs + b] = k == 0 ? top : PC_NEG_INF;
    }
    nfmax[(int64_t)(id / K) * Bs + b] = top;
}

// ------------------------------------------------------------------------------------------
// generic sum-layer kernels (any K, one thread per output, no matrix cores) -- the node x sample
// parallelisation of Sec. 3, kept for block sizes the MFMA kernels do not cover
// ------------------------------------------------------------------------------------------
__device__ inline void lse_push(float &m, float &s, float t)
{
    if (t > m) { s = s * __expf(m - t) + 1.0f; m = t; }
    else s += __expf(t - m);
}

__global__ __launch_bounds__(256) void k_sum_fwd_generic(const float *__restrict__ theta, const float *__restrict__ lch,
                                                         float *__restrict__ l, float *__restrict__ R, const int32_t *__restrict__ ids,
                                                         const int32_t *__restrict__ nbr, const int32_t *__restrict__ par,
                                                         int32_t n_rows, int32_t width, int32_t K, int64_t Bs)
{
    const int64_t total = (int64_t)n_rows * K * Bs;
    for (int64_t t = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; t < total; t += (int64_t)gridDim.x * blockDim.x) {
        const int64_t row = t / Bs, b = t - row * Bs;
        const int32_t r = (int32_t)(row / K), i = (int32_t)(row - (int64_t)r * K);
        float Rn = PC_NEG_INF;
        for (int j = 0; j < width; ++j)
            if (par[(int64_t)r * width + j] != 0) Rn = fmaxf(Rn, R[(int64_t)(nbr[(int64_t)r * width + j] / K) * Bs + b]);
        float m = PC_NEG_INF, s = 0.0f;
        for (int j = 0; j < width; ++j) {
            const int32_t ns = nbr[(int64_t)r * width + j], ps = par[(int64_t)r * width + j];
            if (ps == 0) continue;
            const float d = R[(int64_t)(ns / K) * Bs + b] - Rn;
            for (int jj = 0; jj < K; ++jj) {
                const float th = theta[(int64_t)ps + (int64_t)i * K + jj];
                const float v = lch[(int64_t)(ns + jj) * Bs + b] + d;
                if (th > 0.0f && v > PC_NEG_INF) lse_push(m, s, __logf(th) + v);
            }
        }
        l[(int64_t)(ids[r] + i) * Bs + b] = m > PC_NEG_INF ? m + __logf(s) : PC_NEG_INF;
        if (i == 0) R[(int64_t)(ids[r] / K) * Bs + b] = Rn;
    }
}

__global__ __launch_bounds__(256) void k_sum_bwd_child_generic(const float *__restrict__ theta, const float *__restrict__ l,
                                                               const float *__restrict__ R, const float *__restrict__ N,
                                                               float *__restrict__ F, const int32_t *__restrict__ ids,
                                                               const int32_t *__restrict__ nbr, const int32_t *__restrict__ par,
                                                               const int32_t *__restrict__ flags, int32_t n_rows,
                                                               int32_t width, int32_t K, int64_t Bs)
{
    const int64_t total = (int64_t)n_rows * K * Bs;
    for (int64_t t = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; t < total; t += (int64_t)gridDim.x * blockDim.x) {
        const int64_t row = t / Bs, b = t - row * Bs;
        const int32_t r = (int32_t)(row / K), jj = (int32_t)(row - (int64_t)r * K);
        const float Rc = R[(int64_t)(ids[r] / K) * Bs + b];
        float m = PC_NEG_INF, s = 0.0f;
        for (int j = 0; j < width; ++j) {
            const int32_t ms = nbr[(int64_t)r * width + j], ps = par[(int64_t)r * width + j];
            if (ps == 0) continue;
            const float d = Rc - R[(int64_t)(ms / K) * Bs + b];
            for (int i = 0; i < K; ++i) {
                const float th = theta[(int64_t)ps + (int64_t)i * K + jj];
                const float nf = N[(int64_t)(ms + i) * Bs + b] + d;
                if (th > 0.0f && nf > PC_NEG_INF) lse_push(m, s, __logf(th) + nf);
            }
        }
        const int64_t at = (int64_t)(ids[r] + jj) * Bs + b;
        const float lc = l[at];
        const float add = (m > PC_NEG_INF && lc > PC_NEG_INF) ? __expf(m + __logf(s) + lc) : 0.0f;
        F[at] = (flags[r] & 2) ? add : F[at] + add;                     // first layer that feeds the block stores
    }
}

__global__ __launch_bounds__(256) void k_sum_bwd_param_generic(const float *__restrict__ theta, const float *__restrict__ l,
                                                               const float *__restrict__ R, const float *__restrict__ N,
                                                               float *__restrict__ G, const int32_t *__restrict__ ids,
                                                               const int32_t *__restrict__ nbr, const int32_t *__restrict__ par,
                                                               int32_t n_rows, int32_t width, int32_t K, int64_t Bs, int32_t B,
                                                               int atomic)
{
    const int64_t per_row = (int64_t)width * K * K;
    const int64_t total = (int64_t)n_rows * per_row;
    for (int64_t t = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; t < total; t += (int64_t)gridDim.x * blockDim.x) {
        const int32_t r = (int32_t)(t / per_row);
        int64_t rem = t - (int64_t)r * per_row;
        const int32_t j = (int32_t)(rem / ((int64_t)K * K));
        rem -= (int64_t)j * K * K;
        const int32_t i = (int32_t)(rem / K), jj = (int32_t)(rem - (int64_t)i * K);
        const int32_t ns = nbr[(int64_t)r * width + j], ps = par[(int64_t)r * width + j];
        if (ps == 0) continue;
        const float th = theta[(int64_t)ps + (int64_t)i * K + jj];
        if (!(th > 0.0f)) continue;
        const float *nrow = N + (int64_t)(ids[r] + i) * Bs;
        const float *lrow = l + (int64_t)(ns + jj) * Bs;
        const float *Rs = R + (int64_t)(ids[r] / K) * Bs, *Rc = R + (int64_t)(ns / K) * Bs;
        const float lth = __logf(th);                                   // inside the exponent: every term is an edge flow <= 1
        float acc = 0.0f;
        for (int b = 0; b < B; ++b) {
            const float nf = nrow[b], lc = lrow[b];
            if (nf > PC_NEG_INF && lc > PC_NEG_INF) acc += __expf(nf + lc + (Rc[b] - Rs[b]) + lth);
        }
        float *dst = G + (int64_t)ps + (int64_t)i * K + jj;
        if (atomic) atomicAdd(dst, acc); else *dst += acc;
    }
}

// ------------------------------------------------------------------------------------------
// small-block sum-layer kernels (K in {1, 2, 4, 8, 16}): block-based parallelisation (Sec. 4.1) on the vector
// ALU.  A thread owns one sample column of one node block: it reads each of the K neighbour values once,
// exponentiates it once and uses it for all K outputs of the block -- the K-fold cut in reloads and in
// exponentials that Sec. 4.1 describes.  The K x K weights have workgroup-uniform addresses and ride in scalar
// registers.  Linear-space accumulators with a running maximum, as in the MFMA kernels.
// ------------------------------------------------------------------------------------------
// Two-factor split of a parameter-flow term exp(log_nf_s + l_c + dR) of one sample (dR = R_child - R_sum, an exact
// integer).  With a = max_s log_nf_s over the sum block and g = a + dR -- the children are product blocks, whose
// largest residual lies within +-0.5 of 0, so e^g is the size of the sample's largest term in this block pair, and
// theta p_c / p_s <= 1 with theta >= FLT_MIN bounds g by 87.3 --
//   first factor  exp(log_nf_s - a + s_b)            <= e^s_b
//   second factor exp(l_c + g - s_b - PC_SPLIT_SCALE) <= e^(s_b + 0.5)     with s_b = (g - PC_SPLIT_SCALE) / 2 <= 31.65
// Any per-sample shift is valid (it only moves scale between the factors); this one gives both factors the same
// head-room, so each keeps 87 + s_b nats below its largest value.  The products carry the fixed scale e^-PC_SPLIT_SCALE,
// taken out again when the flow is written: a sum over up to 2^21 samples times a thousand tied instances of terms
// as large as 1 / FLT_MIN then still fits fp32.  What is lost: a product below FLT_MIN, i.e. a term below
// FLT_MIN * e^PC_SPLIT_SCALE = 3.2e-28, and -- only in a sample with g > 23.4, which takes a weight below e^-23 on an
// edge that nevertheless carries the block's largest flow ratio -- a term below e^(g / 2 - 75) whose factor underflows
// (at most e^-31.4).  (A fixed first shift of 31 lost every term of a sample with g < -32, the common case of a block
// pair that carries little flow.)
#define PC_SPLIT_SCALE 24.0f
#define PC_SPLIT_CAP 32.5f
#define PC_SPLIT_OUT 2.6489122e10f   /* e^24 */
__device__ inline float pc_split_shift(float g) { return fminf(fmaxf(0.5f * (g - PC_SPLIT_SCALE), -40.0f), 31.5f); }
// flow += theta * sum * e^24 without leaving the fp32 range on the way: theta may be FLT_MIN (theta * sum would be
// subnormal) and the sum as large as e^85 (sum * e^24 would overflow); theta * 2^40 is a normal number below 2^41 and
// (theta * 2^40) * sum = flow * 2^5.4
__device__ inline float pc_flow_out(float th, float sum) { return ((th * 0x1p+40f) * sum) * (PC_SPLIT_OUT * 0x1p-40f); }
template <int K>
__global__ __launch_bounds__(256) void k_sum_fwd_small(const float *__restrict__ theta, const float *__restrict__ lch,
                                                       float *__restrict__ l, float *__restrict__ R, const int32_t *__restrict__ ids,
                                                       const int32_t *__restrict__ nbr, const int32_t *__restrict__ par,
                                                       const int32_t *__restrict__ flags, int32_t width, int64_t Bs)
{
    const int r = blockIdx.x;
    const int64_t b = (int64_t)blockIdx.y * 256 + threadIdx.x;
    if (b >= Bs) return;
    const int32_t *row_nbr = nbr + (int64_t)r * width, *row_par = par + (int64_t)r * width;
    const int32_t cnt = flags[r] >> 8, id = ids[r];
    float acc[K];
#pragma unroll
    for (int i = 0; i < K; ++i) acc[i] = 0.0f;
    float m = PC_NEG_INF, Rrow = PC_NEG_INF;                            // Rrow: largest child reference seen so far
    // U neighbours at a time: their ids first, then all their loads together -- one memory round trip per U
    // neighbours (with one thread per sample column nothing else hides that latency at the smallest block sizes)
    constexpr int U = K == 1 ? 8 : K == 2 ? 4 : K == 4 ? 2 : 1;
    for (int j0 = 0; j0 < cnt; j0 += U) {
        int32_t nsv[U], pov[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int jc = j0 + u < cnt ? j0 + u : cnt - 1;             // past the end: the last neighbour again, unused
            nsv[u] = row_nbr[jc];
            pov[u] = row_par[jc];
        }
        float vv[U][K], RBv[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
#pragma unroll
            for (int jj = 0; jj < K; ++jj) vv[u][jj] = lch[(int64_t)(nsv[u] + jj) * Bs + b];
            RBv[u] = R[(int64_t)(nsv[u] / K) * Bs + b];
        }
#pragma unroll
        for (int u = 0; u < U; ++u) {
            if (j0 + u >= cnt) break;                                   // uniform over the workgroup
            const float *th = theta + pov[u];
            const float(&v)[K] = vv[u];
            const float RB = RBv[u];
            const float Rn = fmaxf(Rrow, RB);
            m += Rrow - Rn;                                             // exact integer shift; -inf stays -inf
            Rrow = Rn;
            const float d = RB - Rrow;
            float bm = v[0];
#pragma unroll
            for (int jj = 1; jj < K; ++jj) bm = fmaxf(bm, v[jj]);
            bm += d;
            if (bm > m + PC_LAZY) {
                const float sc = pc_half_scale(m - bm);                 // m = -inf: the accumulators are 0
#pragma unroll
                for (int i = 0; i < K; ++i) acc[i] = acc[i] * sc * sc;
                m = bm;
            }
            const float sh = m > PC_NEG_INF ? d - m + PC_UP : 0.0f;     // dead column: v = -inf -> p = 0
            float pv[K];
#pragma unroll
            for (int jj = 0; jj < K; ++jj) pv[jj] = __expf(v[jj] + sh);
#pragma unroll
            for (int i = 0; i < K; ++i) {
#pragma unroll
                for (int jj = 0; jj < K; ++jj) acc[i] = fmaf(th[i * K + jj], pv[jj], acc[i]);
                if (K == 16 && i % 4 == 3) __builtin_amdgcn_sched_barrier(0);   // keeps the 256 weights from all being live in scalar registers
            }
        }
    }
#pragma unroll
    for (int i = 0; i < K; ++i) l[(int64_t)(id + i) * Bs + b] = acc[i] > 0.0f ? m - PC_UP + __logf(acc[i]) : PC_NEG_INF;
    R[(int64_t)(id / K) * Bs + b] = Rrow;
}

template <int K>
__global__ __launch_bounds__(256) void k_sum_bwd_small(const float *__restrict__ theta, const float *__restrict__ l,
                                                       const float *__restrict__ R, const float *__restrict__ N,
                                                       const float *__restrict__ nfmax, float *__restrict__ F,
                                                       const int32_t *__restrict__ ids, const int32_t *__restrict__ nbr,
                                                       const int32_t *__restrict__ par, const int32_t *__restrict__ flags,
                                                       int32_t width, int64_t Bs)
{
    const int r = blockIdx.x;
    const int64_t b = (int64_t)blockIdx.y * 256 + threadIdx.x;
    if (b >= Bs) return;
    const int32_t *row_nbr = nbr + (int64_t)r * width, *row_par = par + (int64_t)r * width;
    const int32_t fl = flags[r], id = ids[r];
    const int32_t cnt = fl >> 8;
    const bool first = (fl & 2) != 0;
    const float Rc = R[(int64_t)(id / K) * Bs + b];
    float lown[K];
#pragma unroll
    for (int jj = 0; jj < K; ++jj) lown[jj] = l[(int64_t)(id + jj) * Bs + b];
    float acc[K];
#pragma unroll
    for (int jj = 0; jj < K; ++jj) acc[jj] = 0.0f;
    float m = PC_NEG_INF;
    constexpr int U = K == 1 ? 8 : K == 2 ? 4 : K == 4 ? 2 : 1;         // neighbours in flight, as in the forward kernel
    for (int j0 = 0; j0 < cnt; j0 += U) {
        int32_t msv[U], pov[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int jc = j0 + u < cnt ? j0 + u : cnt - 1;
            msv[u] = row_nbr[jc];
            pov[u] = row_par[jc];
        }
        float nvv[U][K], Rp[U], bmv[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
#pragma unroll
            for (int i = 0; i < K; ++i) nvv[u][i] = N[(int64_t)(msv[u] + i) * Bs + b];
            Rp[u] = R[(int64_t)(msv[u] / K) * Bs + b];
            bmv[u] = nfmax[(int64_t)(msv[u] / K) * Bs + b];
        }
#pragma unroll
        for (int u = 0; u < U; ++u) {
            if (j0 + u >= cnt) break;                                   // uniform over the workgroup
            const float *th = theta + pov[u];
            const float(&nv)[K] = nvv[u];
            const float d = Rc - Rp[u];
            const float bm = bmv[u] + d;
            if (bm > m + PC_LAZY) {
                const float sc = pc_half_scale(m - bm);
#pragma unroll
                for (int jj = 0; jj < K; ++jj) acc[jj] = acc[jj] * sc * sc;
                m = bm;
            }
            const float sh = m > PC_NEG_INF ? d - m + PC_UP : 0.0f;
            float pv[K];
#pragma unroll
            for (int i = 0; i < K; ++i) pv[i] = __expf(nv[i] + sh);
#pragma unroll
            for (int i = 0; i < K; ++i)
#pragma unroll
                for (int jj = 0; jj < K; ++jj) acc[jj] = fmaf(th[i * K + jj], pv[i], acc[jj]);
        }
    }
#pragma unroll
    for (int jj = 0; jj < K; ++jj) {
        const int64_t at = (int64_t)(id + jj) * Bs + b;
        const float add = (acc[jj] > 0.0f && lown[jj] > PC_NEG_INF) ? __expf(__logf(acc[jj]) + (m - PC_UP) + lown[jj]) : 0.0f;
        if (first) F[at] = add;                                         // first layer that feeds the block stores
        else if (add > 0.0f) F[at] += add;
    }
}

// Backward to the parameters for small blocks, by parameter block like k_param_flow_mfma: one wave per parameter
// block, lanes = samples.  Per pass a lane holds IG x K partial sums of the two-factor products (the same
// balanced split as the MFMA kernel); at the end the 64 lanes are reduced with an exchange-and-halve butterfly
// (each step a lane hands half of its values to its partner and adds the partner's other half), which costs
// about 4 operations per value instead of 12.
template <int K, int IG>
__global__ __launch_bounds__(256) void k_param_flow_small(const float *__restrict__ theta, const float *__restrict__ l,
                                                          const float *__restrict__ R, const float *__restrict__ N,
                                                          const float *__restrict__ nfmax, float *__restrict__ G,
                                                          const int32_t *__restrict__ pf_pb, const int32_t *__restrict__ pf_ptr,
                                                          const int32_t *__restrict__ pf_sum, const int32_t *__restrict__ pf_child,
                                                          int32_t n_pb, int64_t Bs)
{
    constexpr int A = IG * K;                                           // values per lane and pass
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int lane = threadIdx.x & 63;
    const int64_t pidx = (int64_t)blockIdx.x * 4 + wave;
    if (pidx >= n_pb) return;                                           // wave-uniform; no workgroup barrier below
    const int32_t pb = pf_pb[pidx];
    const int i0 = pf_ptr[pidx], i1 = pf_ptr[pidx + 1];
    for (int ig = 0; ig < K; ig += IG) {
        float acc[A];
#pragma unroll
        for (int a = 0; a < A; ++a) acc[a] = 0.0f;
        for (int inst = i0; inst < i1; ++inst) {
            const int32_t ms = pf_sum[inst], ns = pf_child[inst];
            for (int64_t b = lane; b < Bs; b += 64) {
                const float mx = nfmax[(int64_t)(ms / K) * Bs + b];
                const float dR = R[(int64_t)(ns / K) * Bs + b] - R[(int64_t)(ms / K) * Bs + b];
                const bool live = mx > PC_NEG_INF;                      // dead sample: both factors 0
                const float sb = pc_split_shift(mx + dR);
                const float qa = live ? sb - mx : PC_NEG_INF;
                const float qb = live ? mx + dR - sb - PC_SPLIT_SCALE : PC_NEG_INF;
                float fa[IG], fb[K];
#pragma unroll
                for (int i = 0; i < IG; ++i) fa[i] = __expf(N[(int64_t)(ms + ig + i) * Bs + b] + qa);
#pragma unroll
                for (int jj = 0; jj < K; ++jj) fb[jj] = __expf(fminf(l[(int64_t)(ns + jj) * Bs + b] + qb, PC_SPLIT_CAP));
#pragma unroll
                for (int i = 0; i < IG; ++i)
#pragma unroll
                    for (int jj = 0; jj < K; ++jj) acc[i * K + jj] = fmaf(fa[i], fb[jj], acc[i * K + jj]);
            }
        }
        // reduce over the 64 lanes
        int cur = A, idx = 0;                                           // idx: first of the values this lane still holds
#pragma unroll
        for (int dist = 32; dist >= 1; dist >>= 1) {
            if (cur > 1) {
                const int h = cur / 2;
                const bool up = (lane & dist) != 0;
#pragma unroll
                for (int e = 0; e < A / 2; ++e) {
                    if (e < h) {
                        const float lo = acc[e], hi = acc[e + h];
                        const float give = up ? lo : hi, keep = up ? hi : lo;
                        acc[e] = keep + __shfl_xor(give, dist);
                    }
                }
                idx += up ? h : 0;
                cur = h;
            } else {
                acc[0] += __shfl_xor(acc[0], dist);
            }
        }
        // cur values per lane; lanes that differ only in the bits of the plain-sum steps hold copies
        constexpr int HALVINGS = A >= 64 ? 6 : (A == 32 ? 5 : A == 16 ? 4 : A == 8 ? 3 : A == 4 ? 2 : A == 2 ? 1 : 0);
        constexpr int COPIES = 64 >> HALVINGS;
        if ((lane & (COPIES - 1)) == 0) {
#pragma unroll
            for (int e = 0; e < (A >= 64 ? A / 64 : 1); ++e) {
                const int a = idx + e;                                  // = i * K + jj inside this pass
                const int64_t at = (int64_t)pb + (int64_t)ig * K + a;
                const float th = theta[at];
                if (th > 0.0f) G[at] += pc_flow_out(th, acc[e]);
            }
        }
    }
}

// ------------------------------------------------------------------------------------------
// MFMA sum-layer kernels (K % 32 == 0).  Workgroup = 4 waves; a wave owns 32 sample columns.
// ------------------------------------------------------------------------------------------

// Forward (role of Alg. 1) and backward-to-children (role of Alg. 4) share one kernel.
//
// A wave owns a tile of TM = 32*RT rows of one node block x 32 sample columns and a share of the row's
// neighbour chunks (KC = 32 nodes per chunk).  The rows are sum nodes (forward) or child product nodes
// (backward).  A workgroup holds 4 waves: SPLIT of them share one output tile and take the chunks
// round-robin (split of the reduction dimension, so that small batches still fill every SIMD with two
// waves -- a wave cannot overlap its own VALU work with its own MFMAs, a second wave can), the other
// factor 4/SPLIT spans adjacent column tiles.  Per chunk and wave:
//   * forward: the theta sub-block [TM x KC] (row = sum node, contiguous along the children) is fetched with
//     coalesced 16-byte loads and staged in a wave-private LDS tile only to reach the MFMA A-operand layout (LDS
//     operations of one wave complete in order, so no barrier and no double buffer are needed), then read back
//     whole into registers with 16-byte reads;
//   * backward: the operand is the transpose -- lane i needs theta[parent][child i] -- and that IS coalesced in
//     memory (32 consecutive children of one parent row), so it goes straight from L2 into the A-operand layout;
//   * the KC x 32 neighbour values go straight from L2 into the MFMA B-operand layout;
//   * the chunks follow one another without software pipelining: the loop needs 75-150 registers, so 3-6 waves
//     share a SIMD and hide each other's waits.  (A pipelined version -- two operand sets, theta of chunk c+1
//     staged during the arithmetic of chunk c, 190-230 registers, two waves per SIMD -- was slower in every
//     configuration measured, and so was prefetching only the next theta sub-block.)  The exception is a launch
//     too small to put more than one wave on a SIMD (the top layers of a deep narrow circuit, a root): there the
//     PF instantiation requests the next chunk before it works on the current one.
//   forward : value = l (log-prob residual) + (R_child - R_sum); the chunk maximum is taken in registers
//   backward: value = N (log F - l of the parent) + (R_child - R_parent); the block maximum is nfmax
// Values are shifted by the running per-sample maximum, exponentiated in registers and multiplied on
// the matrix cores (MFMA step q of a chunk pairs lanes 0-31 with node 8*(q/4) + q%4 and lanes 32-63 with
// node 8*(q/4) + 4 + q%4, so that one 16-byte LDS read yields the A operands of four steps); the
// accumulator stays in linear space and is rescaled when the maximum grows (the same sum as the
// per-block log-space update of the accumulator in Alg. 1 / Alg. 4, with one log per output instead of one
// per block).  Partial sums of the SPLIT waves are merged through LDS at the end.  No lane-dependent
// branch surrounds an MFMA.
#define PC_LOG2E 1.4426950408889634f
// buffer descriptor of the main-loop loads: raw (stride 0), 2 GiB window from the chunk's base, 32-bit data format
#define PC_BUF_RANGE 0x7fffffff
#define PC_BUF_FLAGS 0x00020000
template <int K, int RT, int SPLIT, bool BWD, bool MULTI, int MODE>
__global__ __launch_bounds__(256, 2) void k_sum_mfma(const float *__restrict__ theta, float *__restrict__ l,
                                                     float *__restrict__ R, const float *__restrict__ N,
                                                     const float *__restrict__ nfmax, float *__restrict__ F,
                                                     const GroupSet gs, int64_t Bs)
{
    constexpr int KC = 32;
    constexpr int TM = 32 * RT;
    constexpr int SUB = K / TM;
    constexpr int NQ = KC / 2;                                          // MFMA steps per chunk
    constexpr int CPB = K / KC;                                         // chunks per neighbour block
    constexpr int NCT = 4 / SPLIT;                                      // column tiles per workgroup
    constexpr int NF4 = TM * KC / 4 / 64;                               // forward: 16-byte loads per lane per chunk
    constexpr int LDA = KC + 4;                                         // LDS row stride (floats): b128 reads conflict-free
    constexpr int TILE = BWD ? 0 : TM * LDA;                            // the backward kernel stages nothing
    constexpr int XCH = RT * 16 * 64 + 128;                             // one partial accumulator, its maxima and references
    constexpr int WSZ = TILE > XCH ? TILE : XCH;
    static_assert(K % TM == 0 && (SPLIT == 1 || SPLIT == 2 || SPLIT == 4), "tile shape");
    __shared__ float lds[4 * WSZ];

    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int lane = threadIdx.x & 63, half = lane >> 5, l32 = lane & 31;
    const int ct = wave / SPLIT, sp = wave % SPLIT;
    const GroupRow gr = locate_row<MULTI>(gs, blockIdx.x / SUB);
    const int r = gr.r, sub = blockIdx.x % SUB;
    const int64_t col0 = ((int64_t)blockIdx.y * NCT + ct) * 32;
    const bool active = col0 < Bs;                                      // wave-uniform
    const int64_t col = (active ? col0 : 0) + l32;
    const int32_t *row_nbr = gr.nbr + (int64_t)r * gr.width, *row_par = gr.par + (int64_t)r * gr.width;
    const int32_t id = gr.ids[r];
    const int32_t fl = gr.aux[r];                                       // wave-uniform
    // backward: the first layer of the sweep that feeds this block stores its flow, later ones accumulate
    const bool first = (fl & 2) != 0;
    float *buf = lds + wave * WSZ;
    const int n_chunks = (fl >> 8) * CPB;                               // real neighbours; padding sits at the end of a row

    // block reference of this row.  Backward: the row's own.  Forward: the maximum of the children's, found
    // on the fly -- Rrow is the maximum over the chunks seen so far and the running maximum m is relative to it
    float Rrow = PC_NEG_INF;
    if (BWD) Rrow = R[(int64_t)(id / K) * Bs + col];

    floatx16 acc[RT];
#pragma unroll
    for (int rt = 0; rt < RT; ++rt)
#pragma unroll
        for (int e = 0; e < 16; ++e) acc[rt][e] = 0.0f;
    float m = PC_NEG_INF;
    // backward: the rows' own log-probabilities are needed only at the end; fetched now, their latency is hidden
    // behind the whole reduction (short reductions are latency-bound)
    // (the tile's rows through one buffer descriptor at its first row: per-lane offset = rows 4 * half + (0..3) of a
    // group of 8 rows and the column, scalar offset per row -- no per-element address arithmetic)
    floatx16 lown[BWD ? RT : 1];
    const int ooff = (int)(((int64_t)(4 * half) * Bs + col) * 4);
    if (BWD) {
        const __amdgpu_buffer_rsrc_t rl =
            __builtin_amdgcn_make_buffer_rsrc((void *)(l + (int64_t)(id + sub * TM) * Bs), 0, PC_BUF_RANGE, PC_BUF_FLAGS);
#pragma unroll
        for (int rt = 0; rt < RT; ++rt)
#pragma unroll
            for (int e = 0; e < 16; ++e) {
                const int so = __builtin_amdgcn_readfirstlane((int)((int64_t)(rt * 32 + 8 * (e / 4) + (e % 4)) * Bs * 4));
                lown[rt][e] = __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(rl, ooff, so, 0));
            }
    }

    // Operands of one chunk: `ar` the MFMA A operands (theta), `v` the neighbour values with their block scalars;
    // forward only: `th` carries the theta sub-block from global memory to the LDS tile.
    // All loads of the loop are buffer loads: a wave-uniform descriptor per chunk (base = first row of the chunk), a
    // loop-invariant per-lane byte offset and a compile-time scalar offset, so they need no vector address
    // arithmetic (the vector ALU issues instead of the matrix cores, not beside them).
    struct Operands {
        floatx4 th[BWD ? 1 : NF4];
        float ar[NQ][RT], v[NQ];
        float rb, bm;
    };
    const float *vsrc = N;                                              // forward: the children's log-probabilities (passed as N)
    int voff[4];                                                        // neighbour values: rows 0-3 of a group of 8 rows
#pragma unroll
    for (int rr = 0; rr < 4; ++rr) voff[rr] = (int)(((int64_t)(4 * half + rr) * Bs + col) * 4);
    int soff[NQ / 4];                                                   // groups of 8 rows
#pragma unroll
    for (int g = 0; g < NQ / 4; ++g) soff[g] = __builtin_amdgcn_readfirstlane((int)((int64_t)(8 * g) * Bs * 4));
    // theta: forward, 16-byte pieces of rows of the sub-block; backward, one child column of parent rows 0 / 4
    const int toff = BWD ? ((4 * half) * K + l32) * 4 : ((lane / (KC / 4)) * K + (lane % (KC / 4)) * 4) * 4;

    float sh2 = 0.0f;
    constexpr bool PF = MODE == 1, WAIT_ALL = MODE == 2;                // schedules chosen by the launcher, see below
    // loads of chunk c into an operand set (nothing is computed on the loaded values here: any arithmetic would wait)
    auto load_chunk = [&](int c, Operands &o) {
        const int j = c / CPB, kc = c % CPB;
        const int32_t ps = row_par[j];
        const float *tb = BWD ? theta + (int64_t)ps + (int64_t)(kc * KC) * K + sub * TM
                              : theta + (int64_t)ps + (int64_t)(sub * TM) * K + kc * KC;
        const __amdgpu_buffer_rsrc_t rth = __builtin_amdgcn_make_buffer_rsrc((void *)tb, 0, PC_BUF_RANGE, PC_BUF_FLAGS);
        if (BWD) {
#pragma unroll
            for (int q = 0; q < NQ; ++q)
#pragma unroll
                for (int rt = 0; rt < RT; ++rt)
                    o.ar[q][rt] = __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(
                                                                rth, toff, ((8 * (q / 4) + (q % 4)) * K + rt * 32) * 4, 0));
        } else {
#pragma unroll
            for (int i = 0; i < NF4; ++i)                               // 64 lanes cover 64 / (KC / 4) rows
                o.th[i] = __builtin_bit_cast(floatx4, __builtin_amdgcn_raw_buffer_load_b128(
                                                          rth, toff, i * (64 / (KC / 4)) * K * 4, 0));
        }
        const int32_t ns = row_nbr[j];
        const float *src = vsrc + (int64_t)(ns + kc * KC) * Bs;
        const __amdgpu_buffer_rsrc_t rv = __builtin_amdgcn_make_buffer_rsrc((void *)src, 0, PC_BUF_RANGE, PC_BUF_FLAGS);
#pragma unroll
        for (int q = 0; q < NQ; ++q)
            o.v[q] = __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(rv, voff[q % 4], soff[q / 4], 0));
        o.rb = (R + (int64_t)(ns / K) * Bs)[(uint32_t)col];
        if (BWD) o.bm = (nfmax + (int64_t)(ns / K) * Bs)[(uint32_t)col];
    };
    // arithmetic of a loaded chunk
    auto run_chunk = [&](Operands &o) {
        // ---- forward: theta registers -> LDS tile -> A operands of the whole chunk ----
        if (!BWD) {
#pragma unroll
            for (int i = 0; i < NF4; ++i) {
                const int t = lane + i * 64;
                *reinterpret_cast<floatx4 *>(buf + (t / (KC / 4)) * LDA + (t % (KC / 4)) * 4) = o.th[i];
            }
#pragma unroll
            for (int rt = 0; rt < RT; ++rt)
#pragma unroll
                for (int g = 0; g < NQ / 4; ++g) {
                    const floatx4 a4 = *reinterpret_cast<const floatx4 *>(buf + (rt * 32 + l32) * LDA + 8 * g + 4 * half);
                    o.ar[4 * g + 0][rt] = a4[0]; o.ar[4 * g + 1][rt] = a4[1];
                    o.ar[4 * g + 2][rt] = a4[2]; o.ar[4 * g + 3][rt] = a4[3];
                }
        }
        // ---- per-chunk scalars: reference, maximum, rescale of the accumulator; leaves sh2 for the exponentials ----
        {
            if (!BWD) {                                                 // a larger reference: m moves by an exact integer
                const float Rn = fmaxf(Rrow, o.rb);
                m += Rrow - Rn;                                         // -inf stays -inf (rb is finite)
                Rrow = Rn;
            }
            const float d = BWD ? Rrow - o.rb : o.rb - Rrow;            // exact integer <= 0
            float cmax;
            if (BWD) {
                cmax = o.bm + d;
            } else {
                cmax = PC_NEG_INF;
#pragma unroll
                for (int q = 0; q < NQ; ++q) cmax = fmaxf(cmax, o.v[q]);
                cmax = fmaxf(cmax, __shfl_xor(cmax, 32)) + d;
            }
            const float m_new = cmax > m + PC_LAZY ? cmax : m;          // -inf + 8 = -inf: the first finite chunk sets it
            const bool dead = !(m_new > PC_NEG_INF);                    // every term of this column so far is 0
            if (__any(m_new != m)) {
                const float scale = dead ? 1.0f : pc_half_scale(m - m_new);   // m = -inf: acc is 0 anyway
#pragma unroll
                for (int rt = 0; rt < RT; ++rt)
#pragma unroll
                    for (int e = 0; e < 16; ++e) acc[rt][e] = acc[rt][e] * scale * scale;
            }
            m = m_new;
            // exp(v + d - m) = exp2(v * log2e + sh2); dead column: v = -inf -> 0
            sh2 = dead ? 0.0f : (d - m_new + PC_UP) * PC_LOG2E;
        }
        // ---- the chunk's MFMA steps ----
        // WAIT_ALL (backward, long reductions, at most two waves per SIMD): all loads of the chunk are waited for
        // before the first MFMA.  Left alone, the compiler lets each MFMA wait for just its own operand, and the matrix
        // pipe then runs in stop-and-go behind the loads for the whole chunk (config 4: 82 -> 78 us per layer).  With
        // more waves per SIMD, or rows of a few chunks, it is faster the other way (dense 1024 x 1024 layers at K = 32:
        // 2.2 against 3.4 ms), and a run-time test here costs as much as the wait itself -- hence an instantiation of
        // its own.  (The forward kernel waits in any case: its
        // chunk maximum needs every value.)  0x0F70 = vmcnt(0), the other counters at their maxima.
        if (WAIT_ALL) __builtin_amdgcn_s_waitcnt(0x0F70);
#pragma unroll
        for (int q = 0; q < NQ; ++q) {
            const float p = __builtin_amdgcn_exp2f(fmaf(o.v[q], PC_LOG2E, sh2));
#pragma unroll
            for (int rt = 0; rt < RT; ++rt) acc[rt] = __builtin_amdgcn_mfma_f32_32x32x2f32(o.ar[q][rt], p, acc[rt], 0, 0, 0);
        }
    };
    if (!PF) {
        Operands o;
        for (int c = sp; c < n_chunks; c += SPLIT) {
            load_chunk(c, o);
            run_chunk(o);
        }
    } else {
        // small launches (one wave per SIMD or fewer): nobody else hides this wave's loads, so the next chunk is
        // requested before the current one is worked on -- two operand sets, chunks in pairs
        Operands oa, ob;
        if (sp < n_chunks) load_chunk(sp, oa);
        int c = sp;
        for (; c + SPLIT < n_chunks; c += 2 * SPLIT) {
            load_chunk(c + SPLIT, ob);
            run_chunk(oa);
            if (c + 2 * SPLIT < n_chunks) load_chunk(c + 2 * SPLIT, oa);
            run_chunk(ob);
        }
        if (c < n_chunks) run_chunk(oa);
    }

    if (SPLIT > 1) {                                                    // merge the partial sums of the SPLIT waves of a tile
        __syncthreads();
        if (sp != 0) {
#pragma unroll
            for (int rt = 0; rt < RT; ++rt)
#pragma unroll
                for (int e = 0; e < 16; ++e) buf[(rt * 16 + e) * 64 + lane] = acc[rt][e];
            buf[RT * 16 * 64 + lane] = m;
            if (!BWD) buf[RT * 16 * 64 + 64 + lane] = Rrow;
        }
        __syncthreads();
        if (sp != 0) return;
#pragma unroll 1                                                        // unrolled, the loads of all partners are hoisted: 45 registers
        for (int s = 1; s < SPLIT; ++s) {
            const float *ob = lds + (wave + s) * WSZ;
            float mo = ob[RT * 16 * 64 + lane];
            if (!BWD) {                                                 // bring both partial sums to the larger reference
                const float Ro = ob[RT * 16 * 64 + 64 + lane];          // -inf: that wave had no chunk (its sum is 0)
                const float Rn = fmaxf(Rrow, Ro);
                m += Rrow - Rn;
                mo = Ro > PC_NEG_INF ? mo + (Ro - Rn) : PC_NEG_INF;
                Rrow = Rn;
            }
            const float m_new = fmaxf(m, mo);
            const bool dead = !(m_new > PC_NEG_INF);
            const float s0 = dead ? 1.0f : pc_half_scale(m - m_new), s1 = dead ? 0.0f : pc_half_scale(mo - m_new);
#pragma unroll
            for (int rt = 0; rt < RT; ++rt)
#pragma unroll
                for (int e = 0; e < 16; ++e) acc[rt][e] = acc[rt][e] * s0 * s0 + ob[(rt * 16 + e) * 64 + lane] * s1 * s1;
            m = m_new;
        }
    }
    if (!active) return;
    if (!BWD && sub == 0 && half == 0) R[(int64_t)(id / K) * Bs + col] = Rrow;
    // Results out.  The rows are addressed through one buffer descriptor at the tile's first row with a scalar offset
    // per row.  Backward: log and exp are the hardware's base-2 instructions (the accumulator of a column with any
    // term is a normal number -- the largest term is at least FLT_MIN * e^PC_UP -- so no denormal care is needed).
    float *out = BWD ? F : l;
    const __amdgpu_buffer_rsrc_t ro =
        __builtin_amdgcn_make_buffer_rsrc((void *)(out + (int64_t)(id + sub * TM) * Bs), 0, PC_BUF_RANGE, PC_BUF_FLAGS);
    const float mb = (m - PC_UP) * PC_LOG2E;
#pragma unroll
    for (int rt = 0; rt < RT; ++rt)
#pragma unroll
        for (int e = 0; e < 16; ++e) {
            const int so = __builtin_amdgcn_readfirstlane((int)((int64_t)(rt * 32 + 8 * (e / 4) + (e % 4)) * Bs * 4));
            const float a = acc[rt][e];
            if (BWD) {
                const float lg = __builtin_amdgcn_logf(a);              // log2; a = 0 -> -inf
                const float lc = lown[rt][e];
                // exp(ln a + (m - PC_UP) + lc); a = 0 or lc = -inf gives exp2(-inf) = 0
                const float add = __builtin_amdgcn_exp2f(lg + fmaf(lc, PC_LOG2E, mb));
                if (first) {
                    __builtin_amdgcn_raw_buffer_store_b32(__builtin_bit_cast(int, add), ro, ooff, so, 0);
                } else if (add > 0.0f) {
                    const float old = __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(ro, ooff, so, 0));
                    __builtin_amdgcn_raw_buffer_store_b32(__builtin_bit_cast(int, old + add), ro, ooff, so, 0);
                }
            } else {
                // ln a + (m - PC_UP), with the logarithm taken of a / 2^24: the accumulator of a live column is around
                // e^PC_UP, and a base-2 logarithm near 0 is far more accurate in absolute terms than one near 29 --
                // these errors add up from layer to layer (a log-likelihood near 0 has an absolute tolerance of 1e-5).
                // a = 0: -inf.  (a >= FLT_MIN * e^PC_UP > 2^-98, so a / 2^24 is a normal number.)
                const float v = fmaf(__builtin_amdgcn_logf(a * 0x1p-24f), 0.6931471805599453f, m + (16.635532333f - PC_UP));
                __builtin_amdgcn_raw_buffer_store_b32(__builtin_bit_cast(int, v), ro, ooff, so, 0);
            }
        }
}

// ------------------------------------------------------------------------------------------
// Long dense reductions on the bf16 matrix cores (fp32 values split in two)
// ------------------------------------------------------------------------------------------
// The fp32 MFMA rate (157 TFLOP/s) is a sixteenth of the bf16 rate.  Every term of a sum node is non-negative, so a
// product theta * p can be taken as  th*ph + th*pl + tl*ph  with theta = th + tl and p = ph + pl split into two bf16
// values each (8 + 8 significant bits, round to nearest): three bf16 MFMAs with fp32 accumulation per fp32 MFMA's
// worth of work, relative error of a term about 2^-17, no cancellation.  Used for rows with long reductions (the
// dense layers of a large HMM), where the fp32 kernel is bound by the matrix cores.
//
// Operands are prepared once, in the order the MFMA wants them, so that the main loop is loads and MFMAs only:
//   * theta planes (k_split_theta, once per forward pass): per parameter block and (32-row tile rt, 16-column slice
//     ks) one 1 KiB tile -- lane (i = lane % 32, h = lane / 32) owns theta[32 rt + i][16 ks + 8 h .. + 7] as 8 bf16;
//   * value planes (k_split_p, per product layer): p = exp(l + PC_UP) of the residual log-probabilities -- at most
//     e^(PC_UP + 0.5), a product block's largest residual is within 0.5 of 0 -- per (16-node slice, 32-column tile)
//     one 1 KiB tile: lane (j = lane % 32, h) owns p[16 slice + 8 h .. + 7][32 tile + j].
// What the fp32 kernel does per value (running maximum, exponential) happens per child BLOCK here: a block's values
// are relative to its integer reference R_c, the block's partial sums are accumulated on their own and added to the
// row's accumulator with the factor exp(R_c - R_row) (R_row = largest reference so far; the accumulator is rescaled
// when it grows).  v_mfma_f32_32x32x16_bf16: A 32 x 16, B 16 x 32, D as for the fp32 instruction.

// theta [n_blocks][K][K] fp32 -> planes Th, Tl of 1 KiB tiles [block][rt][ks][lane][8]; TRANSPOSED: the tiles of
// theta^T (rows = children), for the backward kernel.  One wave per tile.
template <bool TRANSPOSED>
__global__ __launch_bounds__(256) void k_split_theta(const float *__restrict__ theta, int64_t n_tiles, int32_t K,
                                                     uint4 *__restrict__ Th, uint4 *__restrict__ Tl)
{
    const int64_t tile = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    if (tile >= n_tiles) return;
    const int lane = threadIdx.x & 63, i = lane & 31, h = lane >> 5;
    const int nks = K / 16, nrt = K / 32;
    const int ks = (int)(tile % nks), rt = (int)((tile / nks) % nrt);
    const int64_t pb = tile / ((int64_t)nks * nrt);
    const float *src = theta + pb * K * K;
    float v[8];
    if (!TRANSPOSED) {
        const float4 *q = reinterpret_cast<const float4 *>(src + (int64_t)(32 * rt + i) * K + 16 * ks + 8 * h);
        const float4 a = q[0], b = q[1];
        v[0] = a.x; v[1] = a.y; v[2] = a.z; v[3] = a.w; v[4] = b.x; v[5] = b.y; v[6] = b.z; v[7] = b.w;
    } else {
#pragma unroll
        for (int e = 0; e < 8; ++e) v[e] = src[(int64_t)(16 * ks + 8 * h + e) * K + 32 * rt + i];
    }
    uint32_t hi[4], lo[4];
#pragma unroll
    for (int e = 0; e < 4; ++e) bf16_split2(v[2 * e], v[2 * e + 1], hi[e], lo[e]);
    Th[tile * 64 + lane] = make_uint4(hi[0], hi[1], hi[2], hi[3]);
    Tl[tile * 64 + lane] = make_uint4(lo[0], lo[1], lo[2], lo[3]);
}

// value planes of the given node blocks: X = l (forward: residual log-probabilities of product blocks) gives
// exp(l + PC_UP); with a block reference `ref` (backward: X = log_nf of sum blocks, ref = their column maxima) gives
// exp(X - ref + PC_UP).  One wave per (block, 16-node slice, 32-column tile).
__global__ __launch_bounds__(256) void k_split_p(const float *__restrict__ X, const float *__restrict__ ref,
                                                 const int32_t *__restrict__ blk_ids, int32_t n_blk, int32_t K, int64_t Bs,
                                                 uint4 *__restrict__ Ph, uint4 *__restrict__ Pl)
{
    const int n_ct = (int)(Bs / 32), nks = K / 16;
    const int64_t item = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    if (item >= (int64_t)n_blk * nks * n_ct) return;
    const int lane = threadIdx.x & 63;
    const int ct = (int)(item % n_ct), ks = (int)((item / n_ct) % nks);
    const int32_t id = blk_ids[item / ((int64_t)n_ct * nks)];
    float sh = PC_UP;
    if (ref) {
        const float r = ref[(int64_t)(id / K) * Bs + (int64_t)ct * 32 + (lane & 31)];
        sh = r > PC_NEG_INF ? PC_UP - r : PC_NEG_INF;                   // a block without flow: every factor 0
    }
    split_value_tile(X, sh, (int64_t)id + 16 * ks, ct, n_ct, Bs, Ph, Pl, lane);
}

// Sum layer on the planes, forward (rows = sum blocks, neighbours = their product children) and backward to the
// children (rows = product blocks, neighbours = their sum parents, theta planes transposed).  Workgroup = 4 waves that
// share one output tile of 64 rows x 32 CT columns and take the row's neighbour blocks in turn (a split of the
// reduction); at the end the tile's 32 x 32 parts are dealt to the waves, which merge the four partial sums through
// LDS and write the results.  Per 16-node slice a wave fetches 2 + 2 theta tiles and CT + CT value tiles
// (hi and lo planes, 16 bytes per lane each, 1 KiB per wave load) and issues 6 CT MFMAs; the operands of D slices are
// in flight at any time (a ring of D register sets that runs across the neighbour blocks).
//   forward : block scale = R_c (integer reference of the child block); result l = ln(sum) - PC_UP relative to the
//             largest reference, which becomes the row's own
//   backward: block scale = nfmax_s + (R_row - R_s) (column maximum of the parent's log_nf, brought to the row's
//             reference); result F += exp(ln(sum) + scale - PC_UP + l_row)
// Measured on 4096 x 4096 layers at B = 256: 40 us per layer with CT = 1 and 32-34 us with CT = 2 (one workgroup per
// CU, one wave per SIMD) against 80 us on the fp32 matrix cores; the matrix work itself is 10 us.  The rest is the
// rate at which a CU's vector memory pipeline delivers the 1 KiB operand loads (a 128-byte line per 4.8 cycles,
// whatever the ring depth; CT = 2 needs two thirds of the bytes per MFMA) on top of some 20 us that do not depend on
// the traffic (launch, row headers, the per-block folds, the merge, the epilogue).
template <int K, int D, bool BWD, int CT>
__global__ __launch_bounds__(256, CT == 1 ? 2 : 1) void k_sum_bf16(const uint4 *__restrict__ Th, const uint4 *__restrict__ Tl,
                                                                   const uint4 *__restrict__ Ph, const uint4 *__restrict__ Pl,
                                                                   float *__restrict__ l, float *__restrict__ R,
                                                                   const float *__restrict__ nfmax, float *__restrict__ F,
                                                                   const GroupSet gs, int64_t Bs)
{
    constexpr int NKS = K / 16, NRT = K / 32, SUB = K / 64;
    static_assert(NKS % D == 0, "the ring must divide a block's slices");
    __shared__ float lds[2 * CT * 3 * 1024 + 4 * CT * 64];              // partial tiles of the merge and the waves' references
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int lane = threadIdx.x & 63, half = lane >> 5, l32 = lane & 31;
    const GroupRow gr = locate_row<false>(gs, blockIdx.x / SUB);
    const int r = gr.r, sub = blockIdx.x % SUB;
    const int n_ct = (int)(Bs / 32);
    const int ct0 = blockIdx.y * CT;
    const int64_t col0 = (int64_t)ct0 * 32 + l32;                       // column of tile c: col0 + 32 c
    const int32_t *row_nbr = gr.nbr + (int64_t)r * gr.width, *row_par = gr.par + (int64_t)r * gr.width;
    const int32_t id = gr.ids[r];
    const int32_t fl = gr.aux[r];
    const int cnt = fl >> 8;
    float Rown[CT];
#pragma unroll
    for (int c = 0; c < CT; ++c) Rown[c] = BWD ? R[(int64_t)(id / K) * Bs + col0 + 32 * c] : 0.0f;

    floatx16 acc[2][CT], blk[2][CT];
    float m[CT], cm[CT];                                                // reference of the accumulator, of the current block
#pragma unroll
    for (int c = 0; c < CT; ++c) {
        m[c] = PC_NEG_INF;
        cm[c] = PC_NEG_INF;
#pragma unroll
        for (int rt = 0; rt < 2; ++rt)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[rt][c][e] = 0.0f;
    }

    struct Ops { uint4 ah[2], al[2], bh[CT], bl[CT]; };
    const int n_my = cnt > wave ? (cnt - wave + 3) / 4 : 0;             // neighbour blocks wave, wave + 4, ...
    auto load_slice = [&](int32_t ns, int32_t ps, int ks, Ops &o) {
        const int64_t ta = (((int64_t)(ps / (K * K)) * NRT + 2 * sub) * NKS + ks) * 64 + lane;   // rt advances by NKS tiles
        const int64_t tb = ((int64_t)(ns / 16 + ks) * n_ct + ct0) * 64 + lane;
#pragma unroll
        for (int rt = 0; rt < 2; ++rt) { o.ah[rt] = Th[ta + (int64_t)rt * NKS * 64]; o.al[rt] = Tl[ta + (int64_t)rt * NKS * 64]; }
#pragma unroll
        for (int c = 0; c < CT; ++c) { o.bh[c] = Ph[tb + 64 * c]; o.bl[c] = Pl[tb + 64 * c]; }
    };
    // The loop over the wave's neighbour blocks is straight-line inside (every slot of the ring is refilled
    // unconditionally: past the last block the refill repeats that block and is never used), so that the compiler can
    // count the loads in flight and wait for just the oldest set; a branch around a load makes it wait for all of them.
    Ops o[D];
    int32_t ns_cur = 0, ps_cur = 0;
    if (n_my > 0) {
        ns_cur = row_nbr[wave];
        ps_cur = row_par[wave];
#pragma unroll
        for (int d = 0; d < D; ++d) load_slice(ns_cur, ps_cur, d, o[d]);
    }
    for (int bi = 0; bi < n_my; ++bi) {
        const int jn = wave + 4 * (bi + 1 < n_my ? bi + 1 : bi);
        const int32_t ns_nxt = row_nbr[jn], ps_nxt = row_par[jn];
#pragma unroll
        for (int c = 0; c < CT; ++c) {
            const float Rn = R[(int64_t)(ns_cur / K) * Bs + col0 + 32 * c];   // finite
            cm[c] = BWD ? nfmax[(int64_t)(ns_cur / K) * Bs + col0 + 32 * c] + (Rown[c] - Rn) : Rn;
        }
#pragma unroll
        for (int ks = 0; ks < NKS; ++ks) {
            Ops &cur = o[ks % D];
            if (ks == 0) {
#pragma unroll
                for (int c = 0; c < CT; ++c)
#pragma unroll
                    for (int rt = 0; rt < 2; ++rt)
#pragma unroll
                        for (int e = 0; e < 16; ++e) blk[rt][c][e] = 0.0f;
            }
            // three products per tile, small ones first; the tiles take turns so that no MFMA waits for the one before
#pragma unroll
            for (int step = 0; step < 3; ++step)
#pragma unroll
                for (int c = 0; c < CT; ++c)
#pragma unroll
                    for (int rt = 0; rt < 2; ++rt) {
                        const bf16x8 a = __builtin_bit_cast(bf16x8, step == 0 ? cur.al[rt] : cur.ah[rt]);
                        const bf16x8 b = __builtin_bit_cast(bf16x8, step == 1 ? cur.bl[c] : cur.bh[c]);
                        blk[rt][c] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, blk[rt][c], 0, 0, 0);
                    }
            if (ks + D < NKS) load_slice(ns_cur, ps_cur, ks + D, cur);
            else load_slice(ns_nxt, ps_nxt, ks + D - NKS, cur);
            __builtin_amdgcn_sched_barrier(0);                          // keeps the refill here, D - 1 slices ahead of its use
        }
        // the block's partial sums join the row's accumulator, both brought to the larger reference
#pragma unroll
        for (int c = 0; c < CT; ++c) {
            const float mn = fmaxf(m[c], cm[c]);
            const float sa = m[c] > PC_NEG_INF ? __expf(m[c] - mn) : 0.0f, sb = cm[c] > PC_NEG_INF ? __expf(cm[c] - mn) : 0.0f;
            m[c] = mn;
#pragma unroll
            for (int rt = 0; rt < 2; ++rt)
#pragma unroll
                for (int e = 0; e < 16; ++e) acc[rt][c][e] = acc[rt][c][e] * sa + blk[rt][c][e] * sb;
        }
        ns_cur = ns_nxt;
        ps_cur = ps_nxt;
    }

    // Merge and results: the 2 CT tiles of 32 x 32 outputs are dealt to the waves, tile u = 2 c + rt to wave u; every
    // wave leaves its partial sums of the tiles it does not own in LDS (three sets per tile) and its references.
    constexpr int NU = 2 * CT;
    float *mref = lds + NU * 3 * 1024;
#pragma unroll
    for (int c = 0; c < CT; ++c) {
#pragma unroll
        for (int rt = 0; rt < 2; ++rt) {
            const int u = c * 2 + rt;
            if (wave != u) {
                float *dst = lds + (u * 3 + (wave < u ? wave : wave - 1)) * 1024;
#pragma unroll
                for (int e = 0; e < 16; ++e) dst[e * 64 + lane] = acc[rt][c][e];
            }
        }
        mref[(wave * CT + c) * 64 + lane] = m[c];
    }
    __syncthreads();
    const bool first = (fl & 2) != 0;                                   // backward: the first layer that feeds the block stores
#pragma unroll
    for (int u = 0; u < NU; ++u) {
        if (wave != u) continue;                                        // uniform: a wave takes one of the branches
        const int c = u / 2, rt = u % 2;
        const int64_t col = col0 + 32 * c;
        // backward: the rows' own log-probabilities (and, where this layer accumulates, the flows so far) are all
        // requested before the first of them is used -- a load inside the per-element branch would be waited for on its
        // own, 16 times
        floatx16 lown, fold;
        if (BWD) {
#pragma unroll
            for (int e = 0; e < 16; ++e) {
                const int64_t at = (int64_t)(id + sub * 64 + rt * 32 + 8 * (e / 4) + 4 * half + (e % 4)) * Bs + col;
                lown[e] = l[at];
                fold[e] = first ? 0.0f : F[at];
            }
        }
        float mw[4], mt = PC_NEG_INF;                                   // the four waves' references of this column; -inf: no block
#pragma unroll
        for (int w = 0; w < 4; ++w) { mw[w] = mref[(w * CT + c) * 64 + lane]; mt = fmaxf(mt, mw[w]); }
        floatx16 tot;
#pragma unroll
        for (int e = 0; e < 16; ++e) tot[e] = 0.0f;
#pragma unroll
        for (int w = 0; w < 4; ++w) {
            const float sc = mw[w] > PC_NEG_INF ? __expf(mw[w] - mt) : 0.0f;
            if (w == u) {
#pragma unroll
                for (int e = 0; e < 16; ++e) tot[e] += acc[rt][c][e] * sc;
            } else {
                const float *src = lds + (u * 3 + (w < u ? w : w - 1)) * 1024;
#pragma unroll
                for (int e = 0; e < 16; ++e) tot[e] += src[e * 64 + lane] * sc;
            }
        }
        if (!BWD && sub == 0 && rt == 0 && half == 0) R[(int64_t)(id / K) * Bs + col] = mt;
#pragma unroll
        for (int e = 0; e < 16; ++e) {
            const int row = sub * 64 + rt * 32 + 8 * (e / 4) + 4 * half + (e % 4);
            const int64_t at = (int64_t)(id + row) * Bs + col;
            if (!BWD) {
                // ln(sum) - PC_UP, the logarithm taken of sum / 2^24 (see the fp32 kernel)
                l[at] = fmaf(__builtin_amdgcn_logf(tot[e] * 0x1p-24f), 0.6931471805599453f, 16.635532333f - PC_UP);
            } else {
                // exp(ln(sum) + (m - PC_UP) + l_row); sum = 0 or l_row = -inf gives exp2(-inf) = 0
                const float lg = __builtin_amdgcn_logf(tot[e]);
                const float add = __builtin_amdgcn_exp2f(lg + (lown[e] + (mt - PC_UP)) * PC_LOG2E);
                F[at] = fold[e] + (mt > PC_NEG_INF ? add : 0.0f);
            }
        }
    }
}

// Backward to the parameters (role of Alg. 3), organised by PARAMETER BLOCK instead of by layer: one launch
// covers every parameter block of the circuit after the backward sweep.  A wave owns a TMW x TNW tile
// (up to 64 x 64) of one K x K parameter block and reduces over the batch of every (sum block, child
// block) pair that uses the block -- all tied instances, e.g. the T-1 transition layers of an HMM
// (App. A.3) -- in registers, so each flow element is read-modified-written once per call, without
// atomics and without the per-layer accumulation that closes Alg. 3.
//
// Each term exp(log_nf_s + l_c) is split into two fp32 factors around a per-sample shift (any shift is
// valid: it only moves scale between the factors) -- the balanced split defined with PC_SPLIT_SCALE above.  Alg. 3
// shifts by the block maximum a alone, which can drop products of order one when a weight is as small as FLT_MIN.
//
// Per chunk of 32 samples a wave fetches its TMW rows of N and TNW rows of l with 16-byte loads along
// the batch, applies the exponentials, and stages both tiles in wave-private LDS (row stride 36 floats)
// to reach the MFMA operand layouts (batch index on k: step q pairs lanes 0-31 with sample 8*(q/4) + q%4
// and lanes 32-63 with sample 8*(q/4) + 4 + q%4); loads of the next chunk are issued before the
// arithmetic of the current one.
template <int K, int RT, int CT, bool ONE>
__global__ __launch_bounds__(256, 2) void k_param_flow_mfma(const float *__restrict__ theta, const float *__restrict__ l,
                                                            const float *__restrict__ R, const float *__restrict__ N,
                                                            const float *__restrict__ nfmax, float *__restrict__ G,
                                                            const int32_t *__restrict__ pf_pb, const int32_t *__restrict__ pf_ptr,
                                                            const int32_t *__restrict__ pf_sum, const int32_t *__restrict__ pf_child,
                                                            int32_t n_pb, int32_t n_split, int64_t Bs)
{
    constexpr int TMW = 32 * RT, TNW = 32 * CT;
    constexpr int TPB = (K / TMW) * (K / TNW);                          // wave tiles per parameter block
    constexpr int LD = 36;                                              // LDS row stride: 16-byte rows, b128 reads conflict-free
    constexpr int NA4 = TMW * 8 / 64, NB4 = TNW * 8 / 64;               // 16-byte loads per lane per chunk
    // ONE (short reductions): a single tile per wave, used for N's factors and then for l's (LDS operations of one wave
    // complete in order) -- half the LDS, twice the workgroups per CU; the second staging then waits for the first
    // operand read, which costs more than it gains once a block has 16 chunks or more.
    constexpr int TLD = ONE ? (TMW > TNW ? TMW : TNW) : TMW + TNW;
    __shared__ float lds[4 * TLD * LD];

    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int lane = threadIdx.x & 63, half = lane >> 5, l32 = lane & 31;
    // n_split > 1 (a handful of parameter blocks with many tied pairs each, e.g. a small HMM): the pairs of a block
    // are dealt to n_split waves, which add their partial flows atomically
    const int64_t wtile = (int64_t)blockIdx.x * 4 + wave;
    const int64_t tile = wtile / n_split;
    const int spl = (int)(wtile % n_split);
    const int pidx = (int)(tile / TPB), tin = (int)(tile % TPB);
    if (pidx >= n_pb) return;                                           // wave-uniform; no workgroup barrier below
    const int r0 = (tin / (K / TNW)) * TMW, c0 = (tin % (K / TNW)) * TNW;
    const int32_t pb = pf_pb[pidx];
    const int i0 = pf_ptr[pidx], i1 = pf_ptr[pidx + 1];
    float *Qs = lds + wave * TLD * LD, *Ps = ONE ? Qs : Qs + TMW * LD;
    const int srow = lane >> 3, sc4 = (lane & 7) * 4;                   // staging: 8 lanes x 16 bytes per row of 32 samples

    floatx16 acc[RT][CT];
#pragma unroll
    for (int rt = 0; rt < RT; ++rt)
#pragma unroll
        for (int ct = 0; ct < CT; ++ct)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[rt][ct][e] = 0.0f;

    const int chunks_per_inst = (int)(Bs / 32);
    const int n_mine = i1 - i0 > spl ? (i1 - i0 - spl + n_split - 1) / n_split : 0;   // pairs spl, spl + n_split, ...
    const int n_chunks = n_mine * chunks_per_inst;
    floatx4 nf_next[NA4], lc_next[NB4], mx_next, rs_next, rc_next;

#define PC_ISSUE(C)                                                                                                   \
    do {                                                                                                              \
        const int inst_ = i0 + spl + ((C) / chunks_per_inst) * n_split;                                               \
        const int64_t b0_ = (int64_t)((C) % chunks_per_inst) * 32 + sc4;                                              \
        const int32_t ms_ = pf_sum[inst_], ns_ = pf_child[inst_];                                                     \
        const float *np_ = N + (int64_t)(ms_ + r0 + srow) * Bs + b0_;                                                 \
        const float *lp_ = l + (int64_t)(ns_ + c0 + srow) * Bs + b0_;                                                 \
        _Pragma("unroll") for (int i = 0; i < NA4; ++i) nf_next[i] = *reinterpret_cast<const floatx4 *>(np_ + (int64_t)(8 * i) * Bs); \
        _Pragma("unroll") for (int i = 0; i < NB4; ++i) lc_next[i] = *reinterpret_cast<const floatx4 *>(lp_ + (int64_t)(8 * i) * Bs); \
        mx_next = *reinterpret_cast<const floatx4 *>(nfmax + (int64_t)(ms_ / K) * Bs + b0_);                          \
        rs_next = *reinterpret_cast<const floatx4 *>(R + (int64_t)(ms_ / K) * Bs + b0_);                              \
        rc_next = *reinterpret_cast<const floatx4 *>(R + (int64_t)(ns_ / K) * Bs + b0_);                              \
    } while (0)

    if (n_chunks > 0) PC_ISSUE(0);
    for (int c = 0; c < n_chunks; ++c) {
        // exponentials of the fetched chunk, staged in the wave's LDS tiles
        floatx4 qa, qb;                                                 // per-sample shifts in log2 units
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const bool live = mx_next[e] > PC_NEG_INF;
            const float g = mx_next[e] + (rc_next[e] - rs_next[e]);
            const float sb = pc_split_shift(g);
            qa[e] = live ? (sb - mx_next[e]) * PC_LOG2E : PC_NEG_INF;                      // dead sample: both factors 0
            qb[e] = live ? (g - sb - PC_SPLIT_SCALE) * PC_LOG2E : PC_NEG_INF;
        }
#pragma unroll
        for (int i = 0; i < NA4; ++i) {
            floatx4 q;
#pragma unroll
            for (int e = 0; e < 4; ++e) q[e] = __builtin_amdgcn_exp2f(fmaf(nf_next[i][e], PC_LOG2E, qa[e]));
            *reinterpret_cast<floatx4 *>(Qs + (8 * i + srow) * LD + sc4) = q;
        }
        // operands of the whole chunk into registers (LDS operations of one wave complete in order); with a single tile
        // the first operand has to be read before the second is staged
        float areg[16][RT], breg[16][CT];
#define PC_READ_AREG()                                                                                                \
    _Pragma("unroll") for (int rt = 0; rt < RT; ++rt)                                                                 \
        _Pragma("unroll") for (int g = 0; g < 4; ++g) {                                                               \
            const floatx4 a4 = *reinterpret_cast<const floatx4 *>(Qs + (rt * 32 + l32) * LD + 8 * g + 4 * half);      \
            areg[4 * g + 0][rt] = a4[0]; areg[4 * g + 1][rt] = a4[1]; areg[4 * g + 2][rt] = a4[2]; areg[4 * g + 3][rt] = a4[3]; \
        }
        if (ONE) PC_READ_AREG();
#pragma unroll
        for (int i = 0; i < NB4; ++i) {
            floatx4 p;
#pragma unroll
            for (int e = 0; e < 4; ++e)
                p[e] = __builtin_amdgcn_exp2f(fminf(fmaf(lc_next[i][e], PC_LOG2E, qb[e]), PC_SPLIT_CAP * PC_LOG2E));
            *reinterpret_cast<floatx4 *>(Ps + (8 * i + srow) * LD + sc4) = p;
        }
        if (c + 1 < n_chunks) PC_ISSUE(c + 1);
        if (!ONE) PC_READ_AREG();
#undef PC_READ_AREG
#pragma unroll
        for (int ct = 0; ct < CT; ++ct)
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                const floatx4 b4 = *reinterpret_cast<const floatx4 *>(Ps + (ct * 32 + l32) * LD + 8 * g + 4 * half);
                breg[4 * g + 0][ct] = b4[0]; breg[4 * g + 1][ct] = b4[1]; breg[4 * g + 2][ct] = b4[2]; breg[4 * g + 3][ct] = b4[3];
            }
#pragma unroll
        for (int q = 0; q < 16; ++q)
#pragma unroll
            for (int rt = 0; rt < RT; ++rt)
#pragma unroll
                for (int ct = 0; ct < CT; ++ct)
                    acc[rt][ct] = __builtin_amdgcn_mfma_f32_32x32x2f32(areg[q][rt], breg[q][ct], acc[rt][ct], 0, 0, 0);
    }
#undef PC_ISSUE

#pragma unroll
    for (int rt = 0; rt < RT; ++rt)
#pragma unroll
        for (int ct = 0; ct < CT; ++ct)
#pragma unroll
            for (int e = 0; e < 16; ++e) {
                const int i = r0 + rt * 32 + 8 * (e / 4) + 4 * half + (e % 4);
                const int64_t at = (int64_t)pb + (int64_t)i * K + c0 + ct * 32 + l32;
                const float th = theta[at];
                if (th > 0.0f) {                                        // theta = 0: no flow (and never 0 * inf)
                    if (n_split > 1) atomicAdd(G + at, pc_flow_out(th, acc[rt][ct][e]));
                    else G[at] += pc_flow_out(th, acc[rt][ct][e]);
                }
            }
}

// The same computation for K = 64 and 128 with the staging shared by the workgroup: the four waves own the four
// quarters of one K x K parameter block, and every fetched row is used by two of them.  Per chunk of 32 samples the
// 256 threads fetch and exponentiate the K rows of N and the K rows of l ONCE (K / 32 + K / 32 sixteen-byte loads per
// thread; the per-wave kernel needs four times as many at K = 128) into a workgroup tile in LDS; each wave then reads
// the K / 2 + K / 2 rows of its quarter.  Two forms (template parameter ONE, see inside): for long reductions the tile
// is double-buffered, so one barrier per chunk suffices, and the loads run two chunks ahead of the arithmetic -- a
// chunk's matrix work (1.7 us) is shorter than a trip to HBM, which some of a chunk's loads always take; for short
// reductions one tile and one register set, and many more waves per SIMD.
template <int K, bool ONE, bool BF>
__global__ __launch_bounds__(256, 2) void k_param_flow_mfma_wg(const float *__restrict__ theta, const float *__restrict__ l,
                                                               const float *__restrict__ R, const float *__restrict__ N,
                                                               const float *__restrict__ nfmax, float *__restrict__ G,
                                                               const int32_t *__restrict__ pf_pb, const int32_t *__restrict__ pf_ptr,
                                                               const int32_t *__restrict__ pf_sum, const int32_t *__restrict__ pf_child,
                                                               int32_t n_split, int64_t Bs)
{
    constexpr int LD = 36;                                              // LDS row stride: 16-byte rows, b128 reads conflict-free
    // BF (long reductions): the factors are split into hi / lo bf16 values when they are staged -- four planes (Q hi, Q
    // lo, P hi, P lo) of K rows x 32 samples, row stride 80 bytes (16-byte reads of 16 consecutive rows hit distinct
    // banks) -- and a product is qh*ph + qh*pl + ql*ph on v_mfma_f32_32x32x16_bf16: 24 MFMAs of 32 cycles per chunk and
    // wave instead of 64 of 64 cycles; all terms are non-negative, relative error about 2^-17.
    constexpr int LDB = 20;                                             // bf16 planes: row stride in dwords
    constexpr int TILE = BF ? 4 * K * LDB : 2 * K * LD;                 // K rows of factors from N, K rows from l
    constexpr int Q = K / 2, QT = Q / 32;                               // a wave's quarter: Q x Q, QT x QT MFMA tiles
    static_assert(!(BF && ONE), "the bf16 form exists for long reductions only");
    constexpr int NL = K / 32;                                          // 16-byte loads per thread, chunk and array
    static_assert(K == 64 || K == 128, "workgroup-shared parameter-flow kernel");
    // ONE (short reductions -- a parameter block used by one pair, B / 32 chunks -- and many small workgroups): one LDS
    // tile, one register set, operands in two halves: at K = 64 68 registers and 18 KB of LDS, seven waves per SIMD hide
    // the waits and the second barrier per chunk.  Otherwise (long reductions: tied blocks, e.g. the 31 layers of an
    // HMM): two tiles, loads two chunks ahead -- two workgroups of K = 128 fit a CU either way, and the loop has to hide
    // its own waits.
    __shared__ float lds[(ONE ? 1 : 2) * TILE];

    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int lane = threadIdx.x & 63, half = lane >> 5, l32 = lane & 31;
    const int r0 = (wave >> 1) * Q, c0 = (wave & 1) * Q;                // this wave's quarter of the block
    // n_split > 1: the pairs of a block are dealt to n_split workgroups, which add their partial flows atomically
    // (a handful of blocks with many tied pairs each would otherwise keep a handful of workgroups busy)
    const int pidx = blockIdx.x / n_split, spl = blockIdx.x % n_split;
    const int32_t pb = pf_pb[pidx];
    const int i0 = pf_ptr[pidx], i1 = pf_ptr[pidx + 1];
    const int srow = threadIdx.x >> 3, sc4 = (threadIdx.x & 7) * 4;     // staging: 8 threads x 16 bytes per row, 32 rows per pass

    floatx16 acc[QT][QT];
#pragma unroll
    for (int rt = 0; rt < QT; ++rt)
#pragma unroll
        for (int ct = 0; ct < QT; ++ct)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[rt][ct][e] = 0.0f;

    const int chunks_per_inst = (int)(Bs / 32);
    const int n_mine = i1 - i0 > spl ? (i1 - i0 - spl + n_split - 1) / n_split : 0;   // pairs spl, spl + n_split, ...
    const int n_chunks = n_mine * chunks_per_inst;
    // two register sets of fetched tiles (loads two chunks ahead)
    floatx4 nfA[NL], lcA[NL], mxA, rsA, rcA;
    floatx4 nfB[NL], lcB[NL], mxB, rsB, rcB;
    const int voff = (int)(((int64_t)srow * Bs + sc4) * 4), voff1 = sc4 * 4;
    int soff[NL];
#pragma unroll
    for (int i = 0; i < NL; ++i) soff[i] = __builtin_amdgcn_readfirstlane((int)((int64_t)(32 * i) * Bs * 4));

#define PC_ISSUE(C, NF, LC, MX, RS, RC)                                                                               \
    do {                                                                                                              \
        const int inst_ = i0 + spl + ((C) / chunks_per_inst) * n_split;                                               \
        const int64_t b0_ = (int64_t)((C) % chunks_per_inst) * 32;                                                    \
        const int32_t ms_ = pf_sum[inst_], ns_ = pf_child[inst_];                                                     \
        const __amdgpu_buffer_rsrc_t rn_ = __builtin_amdgcn_make_buffer_rsrc((void *)(N + (int64_t)ms_ * Bs + b0_), 0, PC_BUF_RANGE, PC_BUF_FLAGS); \
        const __amdgpu_buffer_rsrc_t rl_ = __builtin_amdgcn_make_buffer_rsrc((void *)(l + (int64_t)ns_ * Bs + b0_), 0, PC_BUF_RANGE, PC_BUF_FLAGS); \
        _Pragma("unroll") for (int i = 0; i < NL; ++i)                                                                \
            NF[i] = __builtin_bit_cast(floatx4, __builtin_amdgcn_raw_buffer_load_b128(rn_, voff, soff[i], 0));        \
        _Pragma("unroll") for (int i = 0; i < NL; ++i)                                                                \
            LC[i] = __builtin_bit_cast(floatx4, __builtin_amdgcn_raw_buffer_load_b128(rl_, voff, soff[i], 0));        \
        const __amdgpu_buffer_rsrc_t rm_ = __builtin_amdgcn_make_buffer_rsrc((void *)(nfmax + (int64_t)(ms_ / K) * Bs + b0_), 0, PC_BUF_RANGE, PC_BUF_FLAGS); \
        const __amdgpu_buffer_rsrc_t rs_ = __builtin_amdgcn_make_buffer_rsrc((void *)(R + (int64_t)(ms_ / K) * Bs + b0_), 0, PC_BUF_RANGE, PC_BUF_FLAGS); \
        const __amdgpu_buffer_rsrc_t rc_ = __builtin_amdgcn_make_buffer_rsrc((void *)(R + (int64_t)(ns_ / K) * Bs + b0_), 0, PC_BUF_RANGE, PC_BUF_FLAGS); \
        MX = __builtin_bit_cast(floatx4, __builtin_amdgcn_raw_buffer_load_b128(rm_, voff1, 0, 0));                    \
        RS = __builtin_bit_cast(floatx4, __builtin_amdgcn_raw_buffer_load_b128(rs_, voff1, 0, 0));                    \
        RC = __builtin_bit_cast(floatx4, __builtin_amdgcn_raw_buffer_load_b128(rc_, voff1, 0, 0));                    \
    } while (0)

    // exponentials of a fetched chunk into tile T of the workgroup (this thread's rows srow, srow + 32, ...)
#define PC_STAGE(T, NF, LC, MX, RS, RC)                                                                               \
    do {                                                                                                              \
        float *Qt_ = lds + (T) * TILE, *Pt_ = Qt_ + K * LD;                                                           \
        floatx4 qa, qb;                                                 /* per-sample shifts in log2 units */         \
        _Pragma("unroll") for (int e = 0; e < 4; ++e) {                                                               \
            const bool live = MX[e] > PC_NEG_INF;                                                                     \
            const float g_ = MX[e] + (RC[e] - RS[e]);                                                                 \
            const float sb_ = pc_split_shift(g_);                                                                     \
            qa[e] = live ? (sb_ - MX[e]) * PC_LOG2E : PC_NEG_INF;       /* dead sample: both factors 0 */             \
            qb[e] = live ? (g_ - sb_ - PC_SPLIT_SCALE) * PC_LOG2E : PC_NEG_INF;                                       \
        }                                                                                                             \
        _Pragma("unroll") for (int i = 0; i < NL; ++i) {                                                              \
            floatx4 q, p;                                                                                             \
            _Pragma("unroll") for (int e = 0; e < 4; ++e) {                                                           \
                q[e] = __builtin_amdgcn_exp2f(fmaf(NF[i][e], PC_LOG2E, qa[e]));                                       \
                p[e] = __builtin_amdgcn_exp2f(fminf(fmaf(LC[i][e], PC_LOG2E, qb[e]), PC_SPLIT_CAP * PC_LOG2E));      \
            }                                                                                                         \
            *reinterpret_cast<floatx4 *>(Qt_ + (32 * i + srow) * LD + sc4) = q;                                       \
            *reinterpret_cast<floatx4 *>(Pt_ + (32 * i + srow) * LD + sc4) = p;                                       \
        }                                                                                                             \
    } while (0)

    // this wave's operands from tile T, then the products -- in two halves of eight steps (half the operand registers)
#define PC_MATH(T)                                                                                             \
    do {                                                                                                              \
        const float *Qt_ = lds + (T) * TILE + r0 * LD, *Pt_ = lds + (T) * TILE + (K + c0) * LD;                       \
        _Pragma("unroll") for (int h2 = 0; h2 < 2; ++h2) {                                                            \
            float areg[8][QT], breg[8][QT];                                                                           \
            _Pragma("unroll") for (int rt = 0; rt < QT; ++rt)                                                         \
                _Pragma("unroll") for (int g = 0; g < 2; ++g) {                                                       \
                    const floatx4 a4 = *reinterpret_cast<const floatx4 *>(Qt_ + (rt * 32 + l32) * LD + 8 * (2 * h2 + g) + 4 * half); \
                    areg[4 * g + 0][rt] = a4[0]; areg[4 * g + 1][rt] = a4[1]; areg[4 * g + 2][rt] = a4[2]; areg[4 * g + 3][rt] = a4[3]; \
                    const floatx4 b4 = *reinterpret_cast<const floatx4 *>(Pt_ + (rt * 32 + l32) * LD + 8 * (2 * h2 + g) + 4 * half); \
                    breg[4 * g + 0][rt] = b4[0]; breg[4 * g + 1][rt] = b4[1]; breg[4 * g + 2][rt] = b4[2]; breg[4 * g + 3][rt] = b4[3]; \
                }                                                                                                     \
            _Pragma("unroll") for (int q = 0; q < 8; ++q)                                                             \
                _Pragma("unroll") for (int rt = 0; rt < QT; ++rt)                                                     \
                    _Pragma("unroll") for (int ct = 0; ct < QT; ++ct)                                                 \
                        acc[rt][ct] = __builtin_amdgcn_mfma_f32_32x32x2f32(areg[q][rt], breg[q][ct], acc[rt][ct], 0, 0, 0); \
        }                                                                                                             \
    } while (0)

    // the same with the factors split into bf16 planes (BF)
#define PC_STAGE_BF(T, NF, LC, MX, RS, RC)                                                                            \
    do {                                                                                                              \
        uint32_t *Qh_ = reinterpret_cast<uint32_t *>(lds) + (T) * TILE, *Ql_ = Qh_ + K * LDB, *Ph_ = Ql_ + K * LDB,   \
                 *Pl_ = Ph_ + K * LDB;                                                                                \
        floatx4 qa, qb;                                                                                               \
        _Pragma("unroll") for (int e = 0; e < 4; ++e) {                                                               \
            const bool live = MX[e] > PC_NEG_INF;                                                                     \
            const float g_ = MX[e] + (RC[e] - RS[e]);                                                                 \
            const float sb_ = pc_split_shift(g_);                                                                     \
            qa[e] = live ? (sb_ - MX[e]) * PC_LOG2E : PC_NEG_INF;                                                     \
            qb[e] = live ? (g_ - sb_ - PC_SPLIT_SCALE) * PC_LOG2E : PC_NEG_INF;                                       \
        }                                                                                                             \
        _Pragma("unroll") for (int i = 0; i < NL; ++i) {                                                              \
            floatx4 q, p;                                                                                             \
            _Pragma("unroll") for (int e = 0; e < 4; ++e) {                                                           \
                q[e] = __builtin_amdgcn_exp2f(fmaf(NF[i][e], PC_LOG2E, qa[e]));                                       \
                p[e] = __builtin_amdgcn_exp2f(fminf(fmaf(LC[i][e], PC_LOG2E, qb[e]), PC_SPLIT_CAP * PC_LOG2E));      \
            }                                                                                                         \
            uint32_t h0, l0, h1, l1;                                                                                  \
            const int at_ = (32 * i + srow) * LDB + (sc4 >> 1);                                                       \
            bf16_split2(q[0], q[1], h0, l0); bf16_split2(q[2], q[3], h1, l1);                                         \
            *reinterpret_cast<uint2 *>(Qh_ + at_) = make_uint2(h0, h1);                                               \
            *reinterpret_cast<uint2 *>(Ql_ + at_) = make_uint2(l0, l1);                                               \
            bf16_split2(p[0], p[1], h0, l0); bf16_split2(p[2], p[3], h1, l1);                                         \
            *reinterpret_cast<uint2 *>(Ph_ + at_) = make_uint2(h0, h1);                                               \
            *reinterpret_cast<uint2 *>(Pl_ + at_) = make_uint2(l0, l1);                                               \
        }                                                                                                             \
    } while (0)
#define PC_MATH_BF(T)                                                                                                 \
    do {                                                                                                              \
        const uint32_t *Qh_ = reinterpret_cast<const uint32_t *>(lds) + (T) * TILE, *Ql_ = Qh_ + K * LDB,             \
                       *Ph_ = Ql_ + K * LDB, *Pl_ = Ph_ + K * LDB;                                                    \
        _Pragma("unroll") for (int ks = 0; ks < 2; ++ks) {                                                            \
            bf16x8 ah[QT], al[QT], bh[QT], bl[QT];                                                                    \
            _Pragma("unroll") for (int rt = 0; rt < QT; ++rt) {                                                       \
                const int ra_ = (r0 + rt * 32 + l32) * LDB + 8 * ks + 4 * half, rb_ = (c0 + rt * 32 + l32) * LDB + 8 * ks + 4 * half; \
                ah[rt] = __builtin_bit_cast(bf16x8, *reinterpret_cast<const uint4 *>(Qh_ + ra_));                     \
                al[rt] = __builtin_bit_cast(bf16x8, *reinterpret_cast<const uint4 *>(Ql_ + ra_));                     \
                bh[rt] = __builtin_bit_cast(bf16x8, *reinterpret_cast<const uint4 *>(Ph_ + rb_));                     \
                bl[rt] = __builtin_bit_cast(bf16x8, *reinterpret_cast<const uint4 *>(Pl_ + rb_));                     \
            }                                                                                                         \
            _Pragma("unroll") for (int rt = 0; rt < QT; ++rt)                                                         \
                _Pragma("unroll") for (int ct = 0; ct < QT; ++ct) {                                                   \
                    acc[rt][ct] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(al[rt], bh[ct], acc[rt][ct], 0, 0, 0);      \
                    acc[rt][ct] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ah[rt], bl[ct], acc[rt][ct], 0, 0, 0);      \
                    acc[rt][ct] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ah[rt], bh[ct], acc[rt][ct], 0, 0, 0);      \
                }                                                                                                     \
        }                                                                                                             \
    } while (0)

    // n_chunks is the same for all four waves, so every wave reaches every barrier
    if (ONE) {
        if (n_chunks > 0) PC_ISSUE(0, nfA, lcA, mxA, rsA, rcA);
        for (int c = 0; c < n_chunks; ++c) {
            if (c > 0) __syncthreads();                                 // the tile has been read by everybody
            PC_STAGE(0, nfA, lcA, mxA, rsA, rcA);
            if (c + 1 < n_chunks) PC_ISSUE(c + 1, nfA, lcA, mxA, rsA, rcA);
            __syncthreads();
            PC_MATH(0);
        }
    } else {
    if (n_chunks > 0) PC_ISSUE(0, nfA, lcA, mxA, rsA, rcA);
    if (n_chunks > 1) PC_ISSUE(1, nfB, lcB, mxB, rsB, rcB);
    int c = 0;
    for (; c + 1 < n_chunks; c += 2) {                                  // pairs of chunks; a last single chunk follows
        if (BF) PC_STAGE_BF(0, nfA, lcA, mxA, rsA, rcA); else PC_STAGE(0, nfA, lcA, mxA, rsA, rcA);
        if (c + 2 < n_chunks) PC_ISSUE(c + 2, nfA, lcA, mxA, rsA, rcA);
        __syncthreads();
        if (BF) PC_MATH_BF(0); else PC_MATH(0);
        if (BF) PC_STAGE_BF(1, nfB, lcB, mxB, rsB, rcB); else PC_STAGE(1, nfB, lcB, mxB, rsB, rcB);
        if (c + 3 < n_chunks) PC_ISSUE(c + 3, nfB, lcB, mxB, rsB, rcB);
        __syncthreads();
        if (BF) PC_MATH_BF(1); else PC_MATH(1);
    }
    if (c < n_chunks) {
        if (BF) PC_STAGE_BF(0, nfA, lcA, mxA, rsA, rcA); else PC_STAGE(0, nfA, lcA, mxA, rsA, rcA);
        __syncthreads();
        if (BF) PC_MATH_BF(0); else PC_MATH(0);
    }
    }
#undef PC_ISSUE
#undef PC_STAGE
#undef PC_MATH
#undef PC_STAGE_BF
#undef PC_MATH_BF

    // flows out: all loads of a 32 x 32 tile first, then the arithmetic, then the stores (a load between two stores
    // would be waited for on its own); theta = 0: no flow (and never 0 * inf)
#pragma unroll
    for (int rt = 0; rt < QT; ++rt)
#pragma unroll
        for (int ct = 0; ct < QT; ++ct) {
            floatx16 thv, gv;
#pragma unroll
            for (int e = 0; e < 16; ++e) {
                const int i = r0 + rt * 32 + 8 * (e / 4) + 4 * half + (e % 4);
                const int64_t at = (int64_t)pb + (int64_t)i * K + c0 + ct * 32 + l32;
                thv[e] = theta[at];
                gv[e] = G[at];
            }
#pragma unroll
            for (int e = 0; e < 16; ++e) {
                const int i = r0 + rt * 32 + 8 * (e / 4) + 4 * half + (e % 4);
                const int64_t at = (int64_t)pb + (int64_t)i * K + c0 + ct * 32 + l32;
                const float inc = thv[e] > 0.0f ? pc_flow_out(thv[e], acc[rt][ct][e]) : 0.0f;
                if (n_split > 1) { if (inc != 0.0f) atomicAdd(G + at, inc); }
                else G[at] = gv[e] + inc;
            }
        }
}

// ------------------------------------------------------------------------------------------
// EM update
// ------------------------------------------------------------------------------------------
// zrow[g*K + i] += sum of real columns of row i of parameter block pb (g = its normalisation group)
__global__ __launch_bounds__(256) void k_em_rowsum(const float *__restrict__ G, const int32_t *__restrict__ pb_group,
                                                   const int32_t *__restrict__ pb_rows, const int32_t *__restrict__ pb_cols,
                                                   int32_t K, float *__restrict__ zrow)
{
    const int pb = blockIdx.x + 1;
    const int g = pb_group[pb];
    if (g < 0) return;
    const int rows = pb_rows[pb], cols = pb_cols[pb];
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    for (int i = wave; i < rows; i += 4) {
        float s = 0.0f;
        for (int jj = lane; jj < cols; jj += 64) s += G[(int64_t)pb * K * K + (int64_t)i * K + jj];
#pragma unroll
        for (int o = 32; o > 0; o >>= 1) s += __shfl_xor(s, o);
        if (lane == 0) atomicAdd(zrow + (int64_t)g * K + i, s);
    }
}

__global__ __launch_bounds__(256) void k_em_theta(float *__restrict__ theta, float *__restrict__ G,
                                                  const int32_t *__restrict__ pb_group, const int32_t *__restrict__ pb_rows,
                                                  const int32_t *__restrict__ pb_cols, const int32_t *__restrict__ group_nch,
                                                  const float *__restrict__ zrow, int32_t K, float step, float pc)
{
    const int pb = blockIdx.x + 1;
    const int g = pb_group[pb];
    const int64_t base = (int64_t)pb * K * K;
    if (g >= 0) {
        const int rows = pb_rows[pb], cols = pb_cols[pb];
        const float share = pc / (float)group_nch[g];
        for (int t = threadIdx.x; t < K * K; t += 256) {
            const int i = t / K, jj = t - i * K;
            if (i < rows && jj < cols) {
                const float z = zrow[(int64_t)g * K + i] + pc;
                if (z > 0.0f) {
                    const float nw = (G[base + t] + share) / z;
                    theta[base + t] = (1.0f - step) * theta[base + t] + step * nw;
                }
            }
        }
    }
    for (int t = threadIdx.x; t < K * K; t += 256) G[base + t] = 0.0f;
}

// Row sums and update for K a power of two >= 4: a thread owns four consecutive columns of one row (16-byte
// accesses); the K / 4 lanes of a row are neighbours in a wave, so a row sum is a few shuffles.
__global__ __launch_bounds__(256) void k_em_rowsum_v4(const float *__restrict__ G, const int32_t *__restrict__ pb_group,
                                                      const int32_t *__restrict__ pb_rows, const int32_t *__restrict__ pb_cols,
                                                      int32_t K, float *__restrict__ zrow)
{
    const int pb = blockIdx.x + 1;
    const int g = pb_group[pb];
    if (g < 0) return;
    const int rows = pb_rows[pb], cols = pb_cols[pb];
    const int k4n = K / 4;
    const float4 *src = reinterpret_cast<const float4 *>(G + (int64_t)pb * K * K);
    for (int q0 = 0; q0 < K * k4n; q0 += 256) {                         // uniform trip count: shuffles see whole waves
        const int q = q0 + threadIdx.x;
        const int i = q / k4n, kq = q - i * k4n;
        float sum = 0.0f;
        if (i < rows) {
            const float4 v = src[q];
            const int j0 = kq * 4;
            sum = (j0 < cols ? v.x : 0.0f) + (j0 + 1 < cols ? v.y : 0.0f) + (j0 + 2 < cols ? v.z : 0.0f) +
                  (j0 + 3 < cols ? v.w : 0.0f);
        }
        for (int o = k4n >> 1; o > 0; o >>= 1) sum += __shfl_xor(sum, o);
        if (kq == 0 && i < rows) atomicAdd(zrow + (int64_t)g * K + i, sum);
    }
}

__global__ __launch_bounds__(256) void k_em_theta_v4(float *__restrict__ theta, float *__restrict__ G,
                                                     const int32_t *__restrict__ pb_group, const int32_t *__restrict__ pb_rows,
                                                     const int32_t *__restrict__ pb_cols, const int32_t *__restrict__ group_nch,
                                                     const float *__restrict__ zrow, int32_t K, float step, float pc)
{
    const int pb = blockIdx.x + 1;
    const int g = pb_group[pb];
    const int k4n = K / 4;
    float4 *th4 = reinterpret_cast<float4 *>(theta + (int64_t)pb * K * K);
    float4 *g4 = reinterpret_cast<float4 *>(G + (int64_t)pb * K * K);
    const int rows = g >= 0 ? pb_rows[pb] : 0, cols = g >= 0 ? pb_cols[pb] : 0;
    const float share = g >= 0 ? pc / (float)group_nch[g] : 0.0f;
    for (int q = threadIdx.x; q < K * k4n; q += 256) {
        const int i = q / k4n, j0 = (q - i * k4n) * 4;
        if (i < rows && j0 < cols) {
            const float z = zrow[(int64_t)g * K + i] + pc;
            if (z > 0.0f) {
                const float4 fl = g4[q];
                float4 w = th4[q];
                w.x = (1.0f - step) * w.x + step * ((fl.x + share) / z);
                if (j0 + 1 < cols) w.y = (1.0f - step) * w.y + step * ((fl.y + share) / z);
                if (j0 + 2 < cols) w.z = (1.0f - step) * w.z + step * ((fl.z + share) / z);
                if (j0 + 3 < cols) w.w = (1.0f - step) * w.w + step * ((fl.w + share) / z);
                th4[q] = w;
            }
        }
        g4[q] = make_float4(0.f, 0.f, 0.f, 0.f);
    }
}

// ztab[t*K + k] += sum over a slab of categories of table_flow[t][c][k]
__global__ __launch_bounds__(256) void k_em_tabsum(const float *__restrict__ Gt, int32_t K, int32_t n_cats,
                                                   int32_t cats_per_block, float *__restrict__ ztab)
{
    const int t = blockIdx.x;
    const int c0 = blockIdx.y * cats_per_block;
    const int c1 = min(n_cats, c0 + cats_per_block);
    for (int k = threadIdx.x; k < K; k += 256) {
        float s = 0.0f;
        for (int c = c0; c < c1; ++c) s += Gt[((int64_t)t * n_cats + c) * K + k];
        atomicAdd(ztab + (int64_t)t * K + k, s);
    }
}

// The same for K a multiple of 4 (K <= 128): a thread owns four consecutive nodes, the 256 threads cover
// 1024 / K categories per pass with 16-byte loads (four in flight per thread), partial sums meet in LDS.
__global__ __launch_bounds__(256) void k_em_tabsum_v4(const float *__restrict__ Gt, int32_t K, int32_t n_cats,
                                                      int32_t cats_per_block, float *__restrict__ ztab)
{
    __shared__ float4 red[256];
    const int t = blockIdx.x;
    const int c0 = blockIdx.y * cats_per_block;
    const int c1 = min(n_cats, c0 + cats_per_block);
    const int k4n = K / 4, kq = threadIdx.x % k4n, rs = threadIdx.x / k4n, R = 256 / k4n;
    float4 acc = make_float4(0.f, 0.f, 0.f, 0.f);
    if (rs < R) {
        const float4 *src = reinterpret_cast<const float4 *>(Gt + (int64_t)t * n_cats * K) + kq;
        for (int c = c0 + rs; c < c1; c += 4 * R) {
            float4 v[4];
#pragma unroll
            for (int j = 0; j < 4; ++j)
                v[j] = c + j * R < c1 ? src[(int64_t)(c + j * R) * k4n] : make_float4(0.f, 0.f, 0.f, 0.f);
#pragma unroll
            for (int j = 0; j < 4; ++j) { acc.x += v[j].x; acc.y += v[j].y; acc.z += v[j].z; acc.w += v[j].w; }
        }
    }
    red[threadIdx.x] = acc;
    __syncthreads();
    if (threadIdx.x < k4n) {
        float4 sum = make_float4(0.f, 0.f, 0.f, 0.f);
        for (int r2 = 0; r2 < R; ++r2) {
            const float4 v = red[r2 * k4n + threadIdx.x];
            sum.x += v.x; sum.y += v.y; sum.z += v.z; sum.w += v.w;
        }
        float *dst = ztab + (int64_t)t * K + threadIdx.x * 4;
        atomicAdd(dst + 0, sum.x); atomicAdd(dst + 1, sum.y); atomicAdd(dst + 2, sum.z); atomicAdd(dst + 3, sum.w);
    }
}

__global__ __launch_bounds__(256) void k_em_tables(float *__restrict__ tables, float *__restrict__ Gt,
                                                   const float *__restrict__ ztab, int32_t K, int32_t n_cats,
                                                   int64_t total, float step, float pc)
{
    const float share = pc / (float)n_cats;
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < total; i += (int64_t)gridDim.x * blockDim.x) {
        const int64_t tc = i / K;
        const int k = (int)(i - tc * K);
        const int64_t t = tc / n_cats;
        const float z = ztab[t * K + k] + pc;
        if (z > 0.0f) {
            const float nw = (Gt[i] + share) / z;
            tables[i] = (1.0f - step) * tables[i] + step * nw;
        }
        Gt[i] = 0.0f;
    }
}

// The same for K a multiple of 4: one table per blockIdx.x, a thread owns four consecutive nodes of one category
// (16-byte accesses, 32-bit index arithmetic, the column sums of the table read once per thread).
__global__ __launch_bounds__(256) void k_em_tables_v4(float *__restrict__ tables, float *__restrict__ Gt,
                                                      const float *__restrict__ ztab, int32_t K, int32_t n_cats,
                                                      float step, float pc)
{
    const float share = pc / (float)n_cats;
    const int t = blockIdx.x;
    const int k4n = K / 4, kq = threadIdx.x % k4n, rs = threadIdx.x / k4n, R = 256 / k4n;
    if (rs >= R) return;
    const float4 zr = *reinterpret_cast<const float4 *>(ztab + (int64_t)t * K + kq * 4);
    const float4 z = make_float4(zr.x + pc, zr.y + pc, zr.z + pc, zr.w + pc);
    float4 *tb = reinterpret_cast<float4 *>(tables + (int64_t)t * n_cats * K) + kq;
    float4 *gb = reinterpret_cast<float4 *>(Gt + (int64_t)t * n_cats * K) + kq;
    for (int c = blockIdx.y * R + rs; c < n_cats; c += gridDim.y * R) {
        const int64_t at = (int64_t)c * k4n;
        const float4 g = gb[at];
        float4 w = tb[at];
        if (z.x > 0.0f) w.x = (1.0f - step) * w.x + step * ((g.x + share) / z.x);
        if (z.y > 0.0f) w.y = (1.0f - step) * w.y + step * ((g.y + share) / z.y);
        if (z.z > 0.0f) w.z = (1.0f - step) * w.z + step * ((g.z + share) / z.z);
        if (z.w > 0.0f) w.w = (1.0f - step) * w.w + step * ((g.w + share) / z.w);
        tb[at] = w;
        gb[at] = make_float4(0.f, 0.f, 0.f, 0.f);
    }
}

// ------------------------------------------------------------------------------------------
// launchers
// ------------------------------------------------------------------------------------------
static thread_local Profiler *g_prof = nullptr;
void set_profiler(Profiler *p) { g_prof = p; }

hipEvent_t Profiler::get()
{
    if (!pool.empty()) { hipEvent_t e = pool.back(); pool.pop_back(); return e; }
    hipEvent_t e = nullptr;
    (void)hipEventCreate(&e);
    return e;
}

void Profiler::collect(int64_t *launches, double *ms)
{
    for (Rec &r : recs) {
        float t = 0.0f;
        if (hipEventSynchronize(r.b) == hipSuccess && hipEventElapsedTime(&t, r.a, r.b) == hipSuccess) {
            launches[r.cls] += 1;
            ms[r.cls] += t;
        }
        pool.push_back(r.a);
        pool.push_back(r.b);
    }
    recs.clear();
}

Profiler::~Profiler()
{
    for (Rec &r : recs) { (void)hipEventDestroy(r.a); (void)hipEventDestroy(r.b); }
    for (hipEvent_t e : pool) (void)hipEventDestroy(e);
}

namespace {
struct Timed {                                                          // brackets one kernel launch
    hipStream_t s;
    hipEvent_t b = nullptr;
    Timed(int cls, hipStream_t stream) : s(stream)
    {
        if (!g_prof) return;
        hipEvent_t a = g_prof->get();
        b = g_prof->get();
        (void)hipEventRecord(a, s);
        g_prof->recs.push_back({cls, a, b});
    }
    ~Timed() { if (b) (void)hipEventRecord(b, s); }
};
}  // namespace

static inline int grid_for(int64_t items, int per_block = 256, int cap = 1 << 16)
{
    int64_t g = (items + per_block - 1) / per_block;
    if (g < 1) g = 1;
    if (g > cap) g = cap;
    return (int)g;
}

static bool g_force_generic = false;
void set_force_generic(bool on) { g_force_generic = on; }
static inline bool use_mfma(int32_t K) { return !g_force_generic && (K == 32 || K == 64 || K == 128); }
static inline bool use_small(int32_t K) { return !g_force_generic && (K == 1 || K == 2 || K == 4 || K == 8 || K == 16); }
#define PC_DISPATCH_SMALL(KERNEL, ...)                                                                     \
    do {                                                                                                   \
        if (K == 1) hipLaunchKernelGGL((KERNEL<1>), __VA_ARGS__);                                          \
        else if (K == 2) hipLaunchKernelGGL((KERNEL<2>), __VA_ARGS__);                                     \
        else if (K == 4) hipLaunchKernelGGL((KERNEL<4>), __VA_ARGS__);                                     \
        else if (K == 8) hipLaunchKernelGGL((KERNEL<8>), __VA_ARGS__);                                     \
        else hipLaunchKernelGGL((KERNEL<16>), __VA_ARGS__);                                                \
    } while (0)

void launch_fill(float *p, int64_t n, float v, hipStream_t s)
{
    Timed timed(KC_MISC, s);
    if (n <= 0) return;
    hipLaunchKernelGGL(k_fill, dim3(grid_for(n, 256, 4096)), dim3(256), 0, s, p, n, v);
}

void launch_prepare_x(const int32_t *x, const uint8_t *mask, int32_t B, int32_t D, int64_t Bs, int32_t n_cats,
                      int32_t *xT, hipStream_t s)
{
    Timed timed(KC_MISC, s);
    dim3 grid((unsigned)((Bs + 31) / 32), (unsigned)((D + 31) / 32));
    hipLaunchKernelGGL(k_prepare_x, grid, dim3(256), 0, s, x, mask, B, D, Bs, n_cats, xT);
}

void launch_readout(const float *l, const float *R, int64_t root_row, int64_t root_blk, int64_t Bs, int32_t B, float *ll,
                    hipStream_t s)
{
    Timed timed(KC_MISC, s);
    hipLaunchKernelGGL(k_readout, dim3((B + 255) / 256), dim3(256), 0, s, l, R, root_row, root_blk, Bs, B, ll);
}

void launch_init_flows(const float *l, float *F, float *N, float *nfmax, const int32_t *blk_ids, int32_t n_blk,
                       int32_t root_id, int32_t K, int64_t Bs, int32_t B, hipStream_t s)
{
    if (n_blk == 0) return;
    Timed timed(KC_MISC, s);
    dim3 grid((unsigned)n_blk, (unsigned)((Bs + 255) / 256));
    hipLaunchKernelGGL(k_init_flows, grid, dim3(256), 0, s, l, F, N, nfmax, blk_ids, root_id, K, Bs, B);
}

void launch_input_fwd(const float *tables, const int32_t *xT, const GroupDev &g, int32_t K, int32_t n_cats, int64_t Bs,
                      float *l, hipStream_t s)
{
    Timed timed(KC_INPUT_FWD, s);
    if (g.n_rows == 0) return;
    if ((K & 3) == 0 && K <= 64) {                                    // larger blocks: the tile costs occupancy, rows are long enough
        dim3 grid((unsigned)g.n_rows, (unsigned)((Bs + 63) / 64));
        const size_t lds = (size_t)K * 65 * 4 + 64 * 4;
        hipLaunchKernelGGL(k_input_fwd_tile, grid, dim3(256), lds, s, tables, xT, g.ids, g.nbr, g.par, K, n_cats, Bs, l);
    } else {
        dim3 grid((unsigned)g.n_rows, (unsigned)((Bs + 255) / 256));
        hipLaunchKernelGGL(k_input_fwd, grid, dim3(256), 0, s, tables, xT, g.ids, g.nbr, g.par, K, n_cats, Bs, l);
    }
}

void launch_input_bwd(const float *F, const int32_t *xT, const GroupDev &g, int32_t K, int32_t n_cats, int64_t Bs,
                      float *table_flow, hipStream_t s)
{
    if (g.n_rows == 0) return;
    Timed timed(KC_INPUT_BWD, s);
    int lps = 1;                                                       // lanes per sample: next power of two >= K, at most 64
    while (lps < K && lps < 64) lps <<= 1;
    const size_t tile_bytes = ((size_t)K * 65 + 64) * 4;
    const size_t hist_bytes = (size_t)n_cats * K * 4 + tile_bytes;
    // more than 64 KB of dynamic LDS has to be allowed per kernel, once on every device the library runs on
    static std::atomic<uint64_t> attr_set{0};
    int dev = 0;
    (void)hipGetDevice(&dev);
    const uint64_t bit = 1ull << (dev & 63);
    if (!(attr_set.load(std::memory_order_relaxed) & bit)) {
        (void)hipFuncSetAttribute(reinterpret_cast<const void *>(k_input_bwd_hist), hipFuncAttributeMaxDynamicSharedMemorySize,
                                  96 * 1024);
        (void)hipFuncSetAttribute(reinterpret_cast<const void *>(k_input_bwd_sorted), hipFuncAttributeMaxDynamicSharedMemorySize,
                                  96 * 1024);
        attr_set.fetch_or(bit, std::memory_order_relaxed);
    }
    // slab of samples for the sorted variant: a [K x SB] tile of at most 34 KB, four workgroups per CU (66 KB tiles
    // combine more samples per category and were 5 % slower; 18 KB tiles 10 % slower)
    int SB = 1024;
    while (SB > 32 && (size_t)K * (SB + 1) * 4 > 34 * 1024) SB >>= 1;
    if (SB > Bs) SB = (int)Bs;
    const size_t sorted_bytes = ((size_t)K * (SB + 1) + 2 * (size_t)SB + n_cats + 1 + 4) * 4;
    if (hist_bytes <= 96 * 1024 && (int64_t)n_cats * 4 <= Bs) {           // many samples per category: privatise in LDS
        hipLaunchKernelGGL(k_input_bwd_hist, dim3((unsigned)g.n_rows), dim3(256), hist_bytes, s, F, xT, g.ids, g.nbr, g.par, K,
                           n_cats, Bs, table_flow, lps, g.tied ? 1 : 0);
    } else if (n_cats <= 1024 && SB >= 64) {                             // few samples per category: combine them first
        const int n_slabs = (int)((Bs + SB - 1) / SB);
        dim3 grid((unsigned)g.n_rows, (unsigned)n_slabs);
        hipLaunchKernelGGL(k_input_bwd_sorted, grid, dim3(256), sorted_bytes, s, F, xT, g.ids, g.nbr, g.par, K, n_cats, Bs,
                           table_flow, SB, lps);
    } else {
        dim3 grid((unsigned)g.n_rows, (unsigned)((Bs + 63) / 64));
        hipLaunchKernelGGL(k_input_bwd_direct, grid, dim3(256), tile_bytes, s, F, xT, g.ids, g.nbr, g.par, K, n_cats, Bs,
                           table_flow, lps);
    }
}

// rows per thread and neighbours in flight by block size: 8-16 outstanding 16-byte loads per thread (at K = 32 eight
// neighbours in flight cost a fifth of the occupancy and 15 % of the PD's product-layer time)
#define PC_DISPATCH_PROD_M(KERNEL, MULTI, ...)                                                             \
    do {                                                                                                   \
        if (narrow) {                                /* 32 columns per workgroup: twice the workgroups, half the rows per thread */ \
            if (K <= 32) hipLaunchKernelGGL((KERNEL(1, 8, MULTI, 8)), __VA_ARGS__);                        \
            else if (K <= 64) hipLaunchKernelGGL((KERNEL(2, 4, MULTI, 8)), __VA_ARGS__);                   \
            else hipLaunchKernelGGL((KERNEL(4, 4, MULTI, 8)), __VA_ARGS__);                                \
        } else if (K <= 16) hipLaunchKernelGGL((KERNEL(1, 8, MULTI, 16)), __VA_ARGS__);                    \
        else if (K <= 32) hipLaunchKernelGGL((KERNEL(2, 4, MULTI, 16)), __VA_ARGS__);                      \
        else if (K <= 64) hipLaunchKernelGGL((KERNEL(4, 4, MULTI, 16)), __VA_ARGS__);                      \
        else hipLaunchKernelGGL((KERNEL(8, 2, MULTI, 16)), __VA_ARGS__);                                   \
    } while (0)
#define PC_DISPATCH_PROD(KERNEL, ...)                                                                      \
    do {                                                                                                   \
        if (gs.n > 1) PC_DISPATCH_PROD_M(KERNEL, true, __VA_ARGS__);                                       \
        else PC_DISPATCH_PROD_M(KERNEL, false, __VA_ARGS__);                                               \
    } while (0)
#define PC_PROD_FWD_F32(RPT, U, MULTI, CL) k_prod_fwd<RPT, U, MULTI, CL, float, false>
#define PC_PROD_FWD_F64(RPT, U, MULTI, CL) k_prod_fwd<RPT, U, MULTI, CL, double, false>
#define PC_PROD_FWD_F32_P(RPT, U, MULTI, CL) k_prod_fwd<RPT, U, MULTI, CL, float, true>
#define PC_PROD_FWD_F64_P(RPT, U, MULTI, CL) k_prod_fwd<RPT, U, MULTI, CL, double, true>
#define PC_PROD_BWD(RPT, U, MULTI, CL) k_prod_bwd<RPT, U, MULTI, CL, false>
#define PC_PROD_BWD_P(RPT, U, MULTI, CL) k_prod_bwd<RPT, U, MULTI, CL, true>
// small launches (the deep narrow circuits) use 32-column workgroups
static inline bool prod_narrow(const GroupSet &gs, int64_t Bs) { return (int64_t)gs.first[gs.n] * ((Bs + 63) / 64) < 1024; }

// Sets of at most PC_MAX_SET groups, widest rows first (the longest rows start first, so they do not trail the launch).
std::vector<GroupSet> make_group_sets(const std::vector<GroupDev> &groups)
{
    std::vector<const GroupDev *> order;
    for (const GroupDev &g : groups)
        if (g.n_rows > 0) order.push_back(&g);
    std::stable_sort(order.begin(), order.end(), [](const GroupDev *a, const GroupDev *b) { return a->width > b->width; });
    std::vector<GroupSet> sets;
    for (size_t i = 0; i < order.size(); ++i) {
        if (i % PC_MAX_SET == 0) { sets.emplace_back(); std::memset(&sets.back(), 0, sizeof(GroupSet)); }
        GroupSet &gs = sets.back();
        const GroupDev &g = *order[i];
        const int k = gs.n++;
        gs.first[k + 1] = gs.first[k] + g.n_rows;
        gs.width[k] = g.width;
        gs.ids[k] = g.ids; gs.nbr[k] = g.nbr; gs.par[k] = g.par; gs.aux[k] = g.aux;
    }
    return sets;
}
static inline int32_t set_rows(const GroupSet &gs) { return gs.first[gs.n]; }
static inline int32_t set_width(const GroupSet &gs)
{
    int32_t w = 0;
    for (int k = 0; k < gs.n; ++k) w = std::max(w, gs.width[k]);
    return w;
}

void launch_prod_fwd(const float *l, float *lout, float *R, const std::vector<GroupSet> &sets, int32_t K, int64_t Bs, void *Ph, void *Pl,
                     hipStream_t s)
{
    uint4 *ph = (uint4 *)Ph, *pl = (uint4 *)Pl;                          // non-null: also write the bf16 value planes
    for (const GroupSet &gs : sets) {
        Timed timed(KC_PROD_FWD, s);
        const bool narrow = prod_narrow(gs, Bs);
        dim3 grid((unsigned)set_rows(gs), (unsigned)(narrow ? (Bs + 31) / 32 : (Bs + 63) / 64));
        // rows with more than eight children (leaf products over many variables) are summed in double
        if (ph && (K % 16) == 0) {
            if (set_width(gs) > 8) PC_DISPATCH_PROD(PC_PROD_FWD_F64_P, grid, dim3(256), 0, s, l, lout, R, gs, K, Bs, ph, pl);
            else PC_DISPATCH_PROD(PC_PROD_FWD_F32_P, grid, dim3(256), 0, s, l, lout, R, gs, K, Bs, ph, pl);
        } else if (set_width(gs) > 8) PC_DISPATCH_PROD(PC_PROD_FWD_F64, grid, dim3(256), 0, s, l, lout, R, gs, K, Bs, ph, pl);
        else PC_DISPATCH_PROD(PC_PROD_FWD_F32, grid, dim3(256), 0, s, l, lout, R, gs, K, Bs, ph, pl);
    }
}

void launch_prod_bwd(const float *l, float *F, const float *Fpar, float *N, float *nfmax, const std::vector<GroupSet> &sets, int32_t K,
                     int64_t Bs, void *Ph, void *Pl, hipStream_t s)
{
    uint4 *ph = (uint4 *)Ph, *pl = (uint4 *)Pl;                          // non-null: also write the bf16 planes of finished sum blocks
    for (const GroupSet &gs : sets) {
        Timed timed(KC_PROD_BWD, s);
        const bool narrow = prod_narrow(gs, Bs);
        dim3 grid((unsigned)set_rows(gs), (unsigned)(narrow ? (Bs + 31) / 32 : (Bs + 63) / 64));
        if (ph && (K % 16) == 0) PC_DISPATCH_PROD(PC_PROD_BWD_P, grid, dim3(256), 0, s, l, F, Fpar, N, nfmax, gs, K, Bs, ph, pl);
        else PC_DISPATCH_PROD(PC_PROD_BWD, grid, dim3(256), 0, s, l, F, Fpar, N, nfmax, gs, K, Bs, ph, pl);
    }
}

// forward / backward-to-children: (K, rows per wave tile / 32, waves sharing one tile)
#define PC_SUM_CASE(KK, RR, SS, BWD, ...)                                                                  \
    if (K == KK && rt == RR && split == SS) {                                                              \
        if (gs.n > 1) hipLaunchKernelGGL((k_sum_mfma<KK, RR, SS, BWD, true, 0>), __VA_ARGS__);             \
        else if (RR == 1 && prefetch) hipLaunchKernelGGL((k_sum_mfma<KK, 1, SS, BWD, false, 1>), __VA_ARGS__); \
        else if (BWD && wait_all) hipLaunchKernelGGL((k_sum_mfma<KK, RR, SS, BWD, false, BWD ? 2 : 0>), __VA_ARGS__); \
        else hipLaunchKernelGGL((k_sum_mfma<KK, RR, SS, BWD, false, 0>), __VA_ARGS__);                     \
        break;                                                                                             \
    }
#define PC_DISPATCH_SUM(BWD, ...)                                                                         \
    do {                                                                                                  \
        PC_SUM_CASE(32, 1, 1, BWD, __VA_ARGS__) PC_SUM_CASE(32, 1, 2, BWD, __VA_ARGS__) PC_SUM_CASE(32, 1, 4, BWD, __VA_ARGS__)    \
        PC_SUM_CASE(64, 1, 1, BWD, __VA_ARGS__) PC_SUM_CASE(64, 1, 2, BWD, __VA_ARGS__) PC_SUM_CASE(64, 1, 4, BWD, __VA_ARGS__)    \
        PC_SUM_CASE(64, 2, 1, BWD, __VA_ARGS__) PC_SUM_CASE(64, 2, 2, BWD, __VA_ARGS__) PC_SUM_CASE(64, 2, 4, BWD, __VA_ARGS__)    \
        PC_SUM_CASE(128, 1, 1, BWD, __VA_ARGS__) PC_SUM_CASE(128, 1, 2, BWD, __VA_ARGS__) PC_SUM_CASE(128, 1, 4, BWD, __VA_ARGS__) \
        PC_SUM_CASE(128, 2, 1, BWD, __VA_ARGS__) PC_SUM_CASE(128, 2, 2, BWD, __VA_ARGS__) PC_SUM_CASE(128, 2, 4, BWD, __VA_ARGS__) \
    } while (0)

// Tile shape for the forward / backward-to-children kernel: the largest row tile (least exp work and
// neighbour traffic per flop) that still leaves two waves per SIMD (2048 waves on 256 CUs), splitting
// the reduction over up to four waves when rows x columns alone are too few.
static void pick_sum_shape(int32_t K, int32_t n_rows, int32_t width, int64_t Bs, int &rt, int &split)
{
    const int64_t col_tiles = (Bs + 31) / 32;
    const int64_t want = 2048;
    rt = K / 32 > 2 ? 2 : K / 32;                                      // 64-row wave tiles at most (register budget)
    while (rt > 1 && (int64_t)n_rows * (K / (32 * rt)) * col_tiles * 4 < want) rt >>= 1;
    const int64_t tiles = (int64_t)n_rows * (K / (32 * rt)) * col_tiles;
    split = 1;
    while (split < 4 && tiles * split < want && (int64_t)width * (K / 32) >= 2 * split) split <<= 1;
}

void launch_sum_fwd(const float *theta, const float *lch, float *l, float *R, const std::vector<GroupSet> &sets, int32_t K,
                    int64_t Bs, hipStream_t s)
{
    if (use_mfma(K)) {
        for (const GroupSet &gs : sets) {
            Timed timed(KC_SUM_FWD, s);
            int rt, split;
            pick_sum_shape(K, set_rows(gs), set_width(gs), Bs, rt, split);
            const int64_t cols_per_wg = 32 * (4 / split);
            dim3 grid((unsigned)(set_rows(gs) * (K / (32 * rt))), (unsigned)((Bs + cols_per_wg - 1) / cols_per_wg));
            const bool prefetch = (int64_t)grid.x * grid.y * 4 <= 1024;    // at most one wave per SIMD
            // long reductions at two waves per SIMD or fewer: see WAIT_ALL in the kernel
            const bool wait_all = (int64_t)set_width(gs) * (K / 32) >= 16 * split && (int64_t)grid.x * grid.y * 4 <= 2048;
            (void)wait_all;
            PC_DISPATCH_SUM(false, grid, dim3(256), 0, s, theta, l, R, lch, (const float *)nullptr,
                            (float *)nullptr, gs, Bs);
        }
        return;
    }
    // other block sizes: one launch per group
    for (const GroupSet &gs : sets) for (int k = 0; k < gs.n; ++k) {
        const GroupDev g{gs.first[k + 1] - gs.first[k], gs.width[k], gs.ids[k], gs.nbr[k], gs.par[k], false, gs.aux[k]};
        Timed timed(KC_SUM_FWD, s);
        if (use_small(K)) {
            dim3 grid((unsigned)g.n_rows, (unsigned)((Bs + 255) / 256));
            PC_DISPATCH_SMALL(k_sum_fwd_small, grid, dim3(256), 0, s, theta, lch, l, R, g.ids, g.nbr, g.par, g.aux, g.width, Bs);
        } else {
            const int64_t items = (int64_t)g.n_rows * K * Bs;
            hipLaunchKernelGGL(k_sum_fwd_generic, dim3(grid_for(items)), dim3(256), 0, s, theta, lch, l, R, g.ids, g.nbr, g.par,
                               g.n_rows, g.width, K, Bs);
        }
    }
}

void launch_sum_bwd_child(const float *theta, const float *l, const float *R, const float *N, const float *nfmax, float *F,
                          const std::vector<GroupSet> &sets, int32_t K, int64_t Bs, hipStream_t s)
{
    if (use_mfma(K)) {
        for (const GroupSet &gs : sets) {
            Timed timed(KC_SUM_BWD_CHILD, s);
            int rt, split;
            pick_sum_shape(K, set_rows(gs), set_width(gs), Bs, rt, split);
            const int64_t cols_per_wg = 32 * (4 / split);
            dim3 grid((unsigned)(set_rows(gs) * (K / (32 * rt))), (unsigned)((Bs + cols_per_wg - 1) / cols_per_wg));
            const bool prefetch = (int64_t)grid.x * grid.y * 4 <= 1024;    // at most one wave per SIMD
            // long reductions at two waves per SIMD or fewer: see WAIT_ALL in the kernel
            const bool wait_all = (int64_t)set_width(gs) * (K / 32) >= 16 * split && (int64_t)grid.x * grid.y * 4 <= 2048;
            (void)wait_all;
            PC_DISPATCH_SUM(true, grid, dim3(256), 0, s, theta, const_cast<float *>(l), const_cast<float *>(R), N, nfmax,
                            F, gs, Bs);
        }
        return;
    }
    // other block sizes: one launch per group
    for (const GroupSet &gs : sets) for (int k = 0; k < gs.n; ++k) {
        const GroupDev g{gs.first[k + 1] - gs.first[k], gs.width[k], gs.ids[k], gs.nbr[k], gs.par[k], false, gs.aux[k]};
        Timed timed(KC_SUM_BWD_CHILD, s);
        if (use_small(K)) {
            dim3 grid((unsigned)g.n_rows, (unsigned)((Bs + 255) / 256));
            PC_DISPATCH_SMALL(k_sum_bwd_small, grid, dim3(256), 0, s, theta, l, R, N, nfmax, F, g.ids, g.nbr, g.par, g.aux,
                              g.width, Bs);
        } else {
            const int64_t items = (int64_t)g.n_rows * K * Bs;
            hipLaunchKernelGGL(k_sum_bwd_child_generic, dim3(grid_for(items)), dim3(256), 0, s, theta, l, R, N, F, g.ids, g.nbr,
                               g.par, g.aux, g.n_rows, g.width, K, Bs);
        }
    }
}

void launch_sum_bwd_param_generic(const float *theta, const float *l, const float *R, const float *N, float *G,
                                  const GroupDev &g, int32_t K, int64_t Bs, int32_t B, hipStream_t s)
{
    if (g.n_rows == 0) return;
    Timed timed(KC_SUM_BWD_PARAM, s);
    const int64_t items = (int64_t)g.n_rows * g.width * K * K;
    hipLaunchKernelGGL(k_sum_bwd_param_generic, dim3(grid_for(items)), dim3(256), 0, s, theta, l, R, N, G, g.ids, g.nbr,
                       g.par, g.n_rows, g.width, K, Bs, B, g.tied ? 1 : 0);
}

static int bf16_enabled()                                              // PC_BF16=0 keeps every layer on the fp32 matrix cores
{
    static const int on = [] { const char *e = std::getenv("PC_BF16"); return (e && e[0] == '0') ? 0 : 1; }();
    return on;
}

bool param_flow_by_block(int32_t K) { return use_mfma(K) || use_small(K); }

void launch_param_flow(const float *theta, const float *l, const float *R, const float *N, const float *nfmax, float *G,
                       const ParamFlowDev &pf, int32_t K, int64_t Bs, hipStream_t s)
{
    if (pf.n_pb == 0) return;
    Timed timed(KC_SUM_BWD_PARAM, s);
    if (use_small(K)) {
        const dim3 grid((unsigned)((pf.n_pb + 3) / 4));
#define PC_PF_SMALL(KK, IG)                                                                                         \
    hipLaunchKernelGGL((k_param_flow_small<KK, IG>), grid, dim3(256), 0, s, theta, l, R, N, nfmax, G, pf.pb, pf.ptr, \
                       pf.sum, pf.child, pf.n_pb, Bs)
        if (K == 1) PC_PF_SMALL(1, 1);
        else if (K == 2) PC_PF_SMALL(2, 2);
        else if (K == 4) PC_PF_SMALL(4, 4);
        else if (K == 8) PC_PF_SMALL(8, 8);
        else PC_PF_SMALL(16, 8);
#undef PC_PF_SMALL
    } else if (K == 32) {
        // few blocks with many tied pairs each: split the pairs over waves until the launch has some 256 of them
        const int64_t avg_pairs = pf.n_pairs / pf.n_pb;
        const int n_split = (int)std::max<int64_t>(1, std::min<int64_t>(avg_pairs, 256 / pf.n_pb));
        const unsigned wgs = (unsigned)(((int64_t)pf.n_pb * n_split + 3) / 4);
        if ((int64_t)pf.n_pairs * (Bs / 32) < 12 * (int64_t)pf.n_pb * n_split)   // fewer than 12 chunks per wave on average
            hipLaunchKernelGGL((k_param_flow_mfma<32, 1, 1, true>), dim3(wgs), dim3(256), 0, s, theta, l,
                               R, N, nfmax, G, pf.pb, pf.ptr, pf.sum, pf.child, pf.n_pb, n_split, Bs);
        else
            hipLaunchKernelGGL((k_param_flow_mfma<32, 1, 1, false>), dim3(wgs), dim3(256), 0, s, theta, l,
                               R, N, nfmax, G, pf.pb, pf.ptr, pf.sum, pf.child, pf.n_pb, n_split, Bs);
    } else {
        // few blocks with many tied pairs each: split the pairs over workgroups until the launch has some 256 of them
        const int n_split = (int)std::max<int64_t>(1, std::min<int64_t>(pf.n_pairs / pf.n_pb, 256 / pf.n_pb));
        // short reductions (fewer than 64 chunks per workgroup on average): the single-tile form
        const bool one = (int64_t)pf.n_pairs * (Bs / 32) < 64 * (int64_t)pf.n_pb * n_split;
#define PC_PF_WG(KK, ONE, BF)                                                                                       \
    hipLaunchKernelGGL((k_param_flow_mfma_wg<KK, ONE, BF>), dim3((unsigned)pf.n_pb * n_split), dim3(256), 0, s, theta, l, R, N, \
                       nfmax, G, pf.pb, pf.ptr, pf.sum, pf.child, n_split, Bs)
        // long reductions (128 chunks per workgroup or more: tied blocks of a large model): bf16-split products
        const bool bf = bf16_enabled() && (int64_t)pf.n_pairs * (Bs / 32) >= 128 * (int64_t)pf.n_pb * n_split;
        if (bf && !one && g_prof) g_prof->bf16_launches[KC_SUM_BWD_PARAM] += 1;
        if (K == 64 && one) PC_PF_WG(64, true, false);
        else if (K == 64 && bf) PC_PF_WG(64, false, true);
        else if (K == 64) PC_PF_WG(64, false, false);
        else if (one) PC_PF_WG(128, true, false);
        else if (bf) PC_PF_WG(128, false, true);
        else PC_PF_WG(128, false, false);
#undef PC_PF_WG
    }
}

// ---- bf16-split path for long dense reductions ----
// A layer takes the bf16 kernel when its rows are long (at least 2048 children: the fp32 kernel is bound by the matrix
// cores there) and the launch has a workgroup for every fourth CU at least.
bool sum_layer_takes_bf16(int32_t K, int32_t n_groups, int32_t n_rows, int32_t width, int64_t Bs)
{
    if (!bf16_enabled() || g_force_generic || (K != 64 && K != 128) || n_groups != 1) return false;
    return (int64_t)width * K >= 2048 && (int64_t)n_rows * (K / 64) * (Bs / 32) >= 128;
}

void launch_split_theta(const float *theta, int64_t n_blocks, int32_t K, bool transposed, void *Th, void *Tl, hipStream_t s)
{
    Timed timed(KC_SPLIT, s);
    const int64_t n_tiles = n_blocks * (K / 32) * (K / 16);
    const dim3 grid((unsigned)((n_tiles + 3) / 4));
    if (transposed) hipLaunchKernelGGL(k_split_theta<true>, grid, dim3(256), 0, s, theta, n_tiles, K, (uint4 *)Th, (uint4 *)Tl);
    else hipLaunchKernelGGL(k_split_theta<false>, grid, dim3(256), 0, s, theta, n_tiles, K, (uint4 *)Th, (uint4 *)Tl);
}

void launch_split_p(const float *X, const float *ref, const int32_t *blk_ids, int32_t n_blk, int32_t K, int64_t Bs, void *Ph,
                    void *Pl, hipStream_t s)
{
    if (n_blk == 0) return;
    Timed timed(KC_SPLIT, s);
    const int64_t items = (int64_t)n_blk * (K / 16) * (Bs / 32);
    hipLaunchKernelGGL(k_split_p, dim3((unsigned)((items + 3) / 4)), dim3(256), 0, s, X, ref, blk_ids, n_blk, K, Bs, (uint4 *)Ph,
                       (uint4 *)Pl);
}

void launch_sum_bf16(const void *Th, const void *Tl, const void *Ph, const void *Pl, float *l, float *R, const float *nfmax,
                     float *F, bool bwd, const GroupSet &gs, int32_t K, int64_t Bs, hipStream_t s)
{
    Timed timed(bwd ? KC_SUM_BWD_CHILD : KC_SUM_FWD, s);
    if (g_prof) g_prof->bf16_launches[bwd ? KC_SUM_BWD_CHILD : KC_SUM_FWD] += 1;
    // 64 x 64 tiles per wave (two thirds of the operand bytes per MFMA) where they still give every CU a workgroup;
    // PC_BF16_CT=1 / 2 forces one form (measurements)
    static const int force_ct = getenv("PC_BF16_CT") ? atoi(getenv("PC_BF16_CT")) : 0;
    const int64_t tiles64 = (int64_t)set_rows(gs) * (K / 64) * (Bs / 64);
    const bool wide = Bs % 64 == 0 && (force_ct ? force_ct == 2 : tiles64 >= 200);
    const dim3 grid((unsigned)(set_rows(gs) * (K / 64)), (unsigned)(Bs / (wide ? 64 : 32)));
#define PC_BF16_SUM(KK, BB)                                                                                            \
    do {                                                                                                               \
        if (wide) hipLaunchKernelGGL((k_sum_bf16<KK, 2, BB, 2>), grid, dim3(256), 0, s, (const uint4 *)Th, (const uint4 *)Tl, \
                                     (const uint4 *)Ph, (const uint4 *)Pl, l, R, nfmax, F, gs, Bs);                     \
        else hipLaunchKernelGGL((k_sum_bf16<KK, 2, BB, 1>), grid, dim3(256), 0, s, (const uint4 *)Th, (const uint4 *)Tl, \
                                (const uint4 *)Ph, (const uint4 *)Pl, l, R, nfmax, F, gs, Bs);                          \
    } while (0)
    if (K == 64) { if (bwd) PC_BF16_SUM(64, true); else PC_BF16_SUM(64, false); }
    else { if (bwd) PC_BF16_SUM(128, true); else PC_BF16_SUM(128, false); }
#undef PC_BF16_SUM
}

void launch_em(float *theta, float *tables, float *theta_flow, float *table_flow, const EmDev &em, int32_t K,
               int32_t n_param_blocks, int32_t n_tables, int32_t n_cats, float step, float pc, hipStream_t s)
{
    launch_fill(em.zrow, (int64_t)em.n_groups * K, 0.0f, s);
    launch_fill(em.ztab, (int64_t)n_tables * K, 0.0f, s);
    Timed timed(KC_EM, s);
    if (n_param_blocks > 0 && K >= 4 && (K & (K - 1)) == 0) {          // 16-byte accesses
        hipLaunchKernelGGL(k_em_rowsum_v4, dim3(n_param_blocks), dim3(256), 0, s, theta_flow, em.pb_group, em.pb_rows,
                           em.pb_cols, K, em.zrow);
        hipLaunchKernelGGL(k_em_theta_v4, dim3(n_param_blocks), dim3(256), 0, s, theta, theta_flow, em.pb_group, em.pb_rows,
                           em.pb_cols, em.group_nch, em.zrow, K, step, pc);
    } else if (n_param_blocks > 0) {
        hipLaunchKernelGGL(k_em_rowsum, dim3(n_param_blocks), dim3(256), 0, s, theta_flow, em.pb_group, em.pb_rows,
                           em.pb_cols, K, em.zrow);
        hipLaunchKernelGGL(k_em_theta, dim3(n_param_blocks), dim3(256), 0, s, theta, theta_flow, em.pb_group, em.pb_rows,
                           em.pb_cols, em.group_nch, em.zrow, K, step, pc);
    }
    if ((K & 3) == 0) {                                                // 16-byte accesses
        const int rows_per_pass = 256 / (K / 4);
        // about 2048 workgroups when the tables are few, at least four loads per thread
        const int64_t max_slabs = std::max<int64_t>(1, n_cats / (4 * rows_per_pass));
        const int64_t slabs = std::min<int64_t>(max_slabs, std::max<int64_t>(1, 2048 / n_tables));
        const int cats_per_block = (int)((n_cats + slabs - 1) / slabs);
        dim3 grid((unsigned)n_tables, (unsigned)((n_cats + cats_per_block - 1) / cats_per_block));
        hipLaunchKernelGGL(k_em_tabsum_v4, grid, dim3(256), 0, s, table_flow, K, n_cats, cats_per_block, em.ztab);
        // enough workgroups per table to fill the chip when there are few tables, one pass otherwise
        const int per_table = (int)std::min<int64_t>((n_cats + rows_per_pass - 1) / rows_per_pass,
                                                     std::max<int64_t>(1, 4096 / n_tables));
        hipLaunchKernelGGL(k_em_tables_v4, dim3((unsigned)n_tables, (unsigned)per_table), dim3(256), 0, s, tables, table_flow,
                           em.ztab, K, n_cats, step, pc);
    } else {
        const int cats_per_block = 64;
        dim3 grid((unsigned)n_tables, (unsigned)((n_cats + cats_per_block - 1) / cats_per_block));
        hipLaunchKernelGGL(k_em_tabsum, grid, dim3(256), 0, s, table_flow, K, n_cats, cats_per_block, em.ztab);
        const int64_t total = (int64_t)n_tables * n_cats * K;
        hipLaunchKernelGGL(k_em_tables, dim3(grid_for(total)), dim3(256), 0, s, tables, table_flow, em.ztab, K, n_cats, total,
                           step, pc);
    }
}

}  // namespace pc
