// Database side of the inverted index on gfx950 (Section 2.2 of the paper): which cell a vector
// falls in, and the list order of a database.
//
//   assign   cell(x) = index of the closest coarse centroid (float64 distances from the
//            differences, ties to the lowest cell) -- the vector quantizer q_i of Section 2.2.
//   group    a stable grouping by cell: list_off[c] = number of vectors in cells < c, and
//            ids[list_off[c] + r] = the r-th vector (in input order) of cell c.
//
// The codes of the residuals are then written in list order by the encoder (qadc_encode.hip).
//
// assign: a workgroup of 256 threads takes 128 vectors and walks over all cells 128 at a time;
// 16 components of both go through LDS as float64 per step, every thread accumulates 8 x 8
// distances (one subtraction and one fused multiply-add per component) and keeps, per vector,
// the best of the cells it has seen; the 16 threads of a vector compare their candidates at the
// end under the order (distance, cell).  Vector-ALU bound: 2 float64 operations per (vector,
// cell, component).
//
// group: the database is cut into P contiguous parts, one wavefront per part.  Pass 1 counts
// cnt[part][cell]; a column pass turns each column into running sums over the parts and yields
// the list sizes; one workgroup scans those into list_off; in pass 2 every wavefront walks its
// part 64 vectors at a time: lanes of the same cell find each other with one ballot per bit of
// the cell id, the first of them advances cnt[part][cell] by their number with one atomic, and
// each lane's position is list_off[cell] + that value + its rank among them.  Positions depend
// only on the input, never on timing: a part's counters are touched by its wavefront alone.

#include "qadc_common.h"
#include <algorithm>

namespace qadc {

constexpr int ASG_TM = 128;  // vectors per workgroup
constexpr int ASG_TN = 128;  // cells per step
constexpr int ASG_TK = 16;   // components per step
constexpr int ASG_LD = ASG_TM + 2;  // row stride in doubles: keeps 16-byte alignment, shifts the banks

// Thread (tx, ty), tx = tid & 15, ty = tid >> 4, owns the vectors 8*ty .. 8*ty+7 of the tile and
// the cells 32*k + 2*tx + e (k < 4, e < 2): a wavefront's 16-byte reads of the cells are
// contiguous across its lanes, its reads of the vectors are the same for 16 lanes.
__global__ __launch_bounds__(256) void ivf_assign_kernel(const float *__restrict__ coarse, int K, int d,
                                                         const float *__restrict__ x, int64_t ldx, int64_t n,
                                                         int32_t *__restrict__ cells, int scale, int accumulate)
{
    __shared__ __attribute__((aligned(16))) double xs[ASG_TK][ASG_LD];
    __shared__ __attribute__((aligned(16))) double cs[ASG_TK][ASG_LD];
    __shared__ double cand_d[ASG_TM][16];
    __shared__ int cand_c[ASG_TM][16];
    const int tid = threadIdx.x;
    const int tx = tid & 15, ty = tid >> 4;
    const int64_t i0 = (int64_t)blockIdx.x * ASG_TM;
    double best_d[8];
    int best_c[8];
#pragma unroll
    for (int a = 0; a < 8; ++a) { best_d[a] = __builtin_inf(); best_c[a] = 0x7fffffff; }

    for (int c0 = 0; c0 < K; c0 += ASG_TN) {
        double acc[8][8];
#pragma unroll
        for (int a = 0; a < 8; ++a)
#pragma unroll
            for (int b = 0; b < 8; ++b) acc[a][b] = 0.0;
        for (int t0 = 0; t0 < d; t0 += ASG_TK) {
            // 128 x 16 elements of x and of the centroids, eight of each per thread, zero beyond the edges
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                const int idx = tid + e * 256;
                const int row = idx >> 4, col = idx & 15;
                const int t = t0 + col;
                const int64_t i = i0 + row;
                const int c = c0 + row;
                xs[col][row] = (i < n && t < d) ? (double)x[i * ldx + t] : 0.0;
                cs[col][row] = (c < K && t < d) ? (double)coarse[(size_t)c * d + t] : 0.0;
            }
            __syncthreads();
#pragma unroll 4
            for (int kk = 0; kk < ASG_TK; ++kk) {
                double xv[8], cv[8];
#pragma unroll
                for (int a = 0; a < 8; a += 2) {
                    const double2 v = *reinterpret_cast<const double2 *>(&xs[kk][8 * ty + a]);
                    xv[a] = v.x; xv[a + 1] = v.y;
                }
#pragma unroll
                for (int k = 0; k < 4; ++k) {
                    const double2 v = *reinterpret_cast<const double2 *>(&cs[kk][32 * k + 2 * tx]);
                    cv[2 * k] = v.x; cv[2 * k + 1] = v.y;
                }
#pragma unroll
                for (int a = 0; a < 8; ++a)
#pragma unroll
                    for (int b = 0; b < 8; ++b) {
                        const double df = xv[a] - cv[b];
                        acc[a][b] = fma(df, df, acc[a][b]);
                    }
            }
            __syncthreads();
        }
        // the smaller distance wins, the lower cell among equal distances
#pragma unroll
        for (int a = 0; a < 8; ++a)
#pragma unroll
            for (int b = 0; b < 8; ++b) {
                const int c = c0 + 32 * (b >> 1) + 2 * tx + (b & 1);
                if (c < K && (acc[a][b] < best_d[a] || (acc[a][b] == best_d[a] && c < best_c[a]))) {
                    best_d[a] = acc[a][b];
                    best_c[a] = c;
                }
            }
    }
#pragma unroll
    for (int a = 0; a < 8; ++a) {
        cand_d[8 * ty + a][tx] = best_d[a];
        cand_c[8 * ty + a][tx] = best_c[a];
    }
    __syncthreads();
    if (tid < ASG_TM) {
        const int64_t i = i0 + tid;
        if (i < n) {
            double bd = cand_d[tid][0];
            int bc = cand_c[tid][0];
            for (int k = 1; k < 16; ++k) {
                const double dd = cand_d[tid][k];
                const int cc = cand_c[tid][k];
                if (dd < bd || (dd == bd && cc < bc)) { bd = dd; bc = cc; }
            }
            cells[i] = (accumulate ? cells[i] : 0) + bc * scale;
        }
    }
}

int ivf_assign(const float *coarse, int K, int d, const float *x, int64_t n, int32_t *cells, hipStream_t st)
{
    if (K < 1 || d < 1 || n < 0)
        return fail(QADC_EINVAL, "qadc_ivf_assign: K=%d d=%d n=%lld", K, d, (long long)n);
    if (n == 0) return QADC_OK;
    if (!coarse || !x || !cells) return fail(QADC_EINVAL, "qadc_ivf_assign: null pointer");
    const int64_t grid = ceil_div(n, ASG_TM);
    if (grid > 0x7fffffffll) return fail(QADC_EINVAL, "qadc_ivf_assign: n too large for one call");
    hipLaunchKernelGGL(ivf_assign_kernel, dim3((unsigned)grid), dim3(256), 0, st, coarse, K, d, x, (int64_t)d, n,
                       cells, 1, 0);
    QADC_HIP_TRY(hipGetLastError());
    return QADC_OK;
}

// Cells of an inverted multi-index: the coarse quantizer is the product of two quantizers of K
// centroids over the two halves of the vector, cell = K * (closest of halves[0] to the first half)
// + (closest of halves[1] to the second half).  Two passes of the assignment kernel over the
// halves of the rows of x.
int multi_index_assign(const float *halves, int K, int d, const float *x, int64_t n, int32_t *cells,
                       hipStream_t st)
{
    if (K < 1 || K > 16384 || d < 2 || (d & 1) || n < 0)
        return fail(QADC_EINVAL, "qadc_multi_index_assign: K=%d d=%d n=%lld", K, d, (long long)n);
    if (n == 0) return QADC_OK;
    if (!halves || !x || !cells) return fail(QADC_EINVAL, "qadc_multi_index_assign: null pointer");
    const int64_t grid = ceil_div(n, ASG_TM);
    if (grid > 0x7fffffffll) return fail(QADC_EINVAL, "qadc_multi_index_assign: n too large for one call");
    const int dh = d / 2;
    hipLaunchKernelGGL(ivf_assign_kernel, dim3((unsigned)grid), dim3(256), 0, st, halves, K, dh, x, (int64_t)d, n,
                       cells, K, 0);
    hipLaunchKernelGGL(ivf_assign_kernel, dim3((unsigned)grid), dim3(256), 0, st, halves + (size_t)K * dh, K, dh,
                       x + dh, (int64_t)d, n, cells, 1, 1);
    QADC_HIP_TRY(hipGetLastError());
    return QADC_OK;
}

// ------------------------------------------------------------------ group

constexpr int GRP_MAX_PARTS = 1024;
constexpr int64_t GRP_MIN_PART = 4096;       // vectors per part, at least
constexpr int64_t GRP_MAX_COUNTERS = 1ll << 26;  // parts * K, at most (256 MiB of counters)
constexpr int GRP_MAX_K = 1 << 24;

struct GroupPlan {
    int P;
    int64_t part;  // vectors per part, a multiple of 64
    size_t cnt_off, size_off, total;
};

static bool make_group_plan(int64_t n, int K, GroupPlan *g)
{
    if (n < 0 || n > 0xffffffffll || K < 1 || K > GRP_MAX_K) return false;
    int64_t P = std::max<int64_t>(1, std::min<int64_t>(GRP_MAX_PARTS, n / GRP_MIN_PART));
    P = std::max<int64_t>(1, std::min<int64_t>(P, GRP_MAX_COUNTERS / K));
    g->P = (int)P;
    g->part = std::max<int64_t>(64, ceil_div(ceil_div(std::max<int64_t>(n, 1), P), 64) * 64);
    g->cnt_off = 0;
    g->size_off = align_up((size_t)P * K * sizeof(unsigned), 256);
    g->total = g->size_off + align_up((size_t)K * sizeof(unsigned), 256);
    return true;
}

size_t ivf_group_workspace(int64_t n, int K)
{
    GroupPlan g;
    return make_group_plan(n, K, &g) ? g.total : 0;
}

__global__ void grp_zero_kernel(uint4 *p, size_t n16)
{
    size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    for (; i < n16; i += stride) p[i] = make_uint4(0, 0, 0, 0);
}

// What a grouping pass sorts by.  The vector met at place i of the pass is perm[i] (i itself
// without perm); its cell is cells[that vector]; the key is the cell (mode 0), or, for the two
// passes over the product cells c = hi*Kh + lo of a multi-index, lo (mode 1) and hi (mode 2).  A
// cell outside [0, cell_end) has no key: the vector is left out.  n_dev, when set, holds the
// number of places of the pass (what the pass before placed).
struct GroupKeys {
    const int32_t *cells;
    const uint32_t *perm;
    const int64_t *n_dev;
    int mode, Kh, cell_end;
};

__device__ inline int group_key(const GroupKeys &g, int64_t i, uint32_t *vec)
{
    const uint32_t v = g.perm ? g.perm[i] : (uint32_t)i;
    *vec = v;
    const int c = g.cells[v];
    if (c < 0 || c >= g.cell_end) return -1;
    return g.mode == 0 ? c : g.mode == 1 ? c % g.Kh : c / g.Kh;
}

// one wavefront per part: cnt[part][key] += 1
__global__ __launch_bounds__(256) void grp_count_kernel(GroupKeys g, int64_t n, int K, int64_t part, int P,
                                                        unsigned *__restrict__ cnt)
{
    const int w = blockIdx.x * 4 + (threadIdx.x >> 6);
    if (w >= P) return;
    const int lane = threadIdx.x & 63;
    if (g.n_dev) n = min(n, *g.n_dev);
    const int64_t lo = (int64_t)w * part, hi = min(n, lo + part);
    unsigned *row = cnt + (size_t)w * K;
    for (int64_t i = lo + lane; i < hi; i += 64) {
        uint32_t v;
        const int c = group_key(g, i, &v);
        if (c >= 0) atomicAdd(&row[c], 1u);
    }
}

// one thread per cell: the column becomes its running sums over the parts; size[cell] = its total
__global__ __launch_bounds__(256) void grp_column_kernel(unsigned *__restrict__ cnt, int K, int P,
                                                         unsigned *__restrict__ size)
{
    const int c = blockIdx.x * 256 + threadIdx.x;
    if (c >= K) return;
    unsigned run = 0;
    for (int p = 0; p < P; ++p) {
        const unsigned v = cnt[(size_t)p * K + c];
        cnt[(size_t)p * K + c] = run;
        run += v;
    }
    size[c] = run;
}

// one workgroup: list_off = exclusive running sum of size, list_off[K] = total
__global__ __launch_bounds__(1024) void grp_offsets_kernel(const unsigned *__restrict__ size, int K,
                                                           int64_t *__restrict__ list_off)
{
    __shared__ unsigned long long wsum[16];
    __shared__ unsigned long long carry_s;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    if (tid == 0) carry_s = 0;
    __syncthreads();
    for (int c0 = 0; c0 < K; c0 += 1024) {
        const int c = c0 + tid;
        const unsigned long long v = c < K ? size[c] : 0;
        unsigned long long inc = v;  // inclusive sum inside the wavefront
#pragma unroll
        for (int s = 1; s < 64; s <<= 1) {
            const unsigned long long o = __shfl_up(inc, s);
            if (lane >= s) inc += o;
        }
        if (lane == 63) wsum[wave] = inc;
        __syncthreads();
        unsigned long long before = carry_s;
        for (int k = 0; k < wave; ++k) before += wsum[k];
        if (c < K) list_off[c] = (int64_t)(before + inc - v);
        __syncthreads();
        if (tid == 1023) carry_s = before + inc;
        __syncthreads();
    }
    if (tid == 0) list_off[K] = (int64_t)carry_s;
}

// one wavefront per part, 64 vectors per step, in the order of the pass
__global__ __launch_bounds__(256) void grp_place_kernel(GroupKeys g, int64_t n, int K, int nbits, int64_t part,
                                                        int P, unsigned *__restrict__ cnt,
                                                        const int64_t *__restrict__ list_off,
                                                        uint32_t *__restrict__ ids)
{
    const int w = blockIdx.x * 4 + (threadIdx.x >> 6);
    if (w >= P) return;
    const int lane = threadIdx.x & 63;
    if (g.n_dev) n = min(n, *g.n_dev);
    const int64_t lo = (int64_t)w * part, hi = min(n, lo + part);
    unsigned *row = cnt + (size_t)w * K;
    for (int64_t s = lo; s < hi; s += 64) {  // uniform over the wavefront
        const int64_t i = s + lane;
        uint32_t v = 0;
        const int c = i < hi ? group_key(g, i, &v) : -1;
        const bool valid = c >= 0;
        unsigned long long peers = __ballot(valid);
        for (int b = 0; b < nbits; ++b) {
            const bool bit = (c >> b) & 1;
            const unsigned long long m = __ballot(valid && bit);
            peers &= bit ? m : ~m;
        }
        if (valid) {  // peers holds this lane at least
            const int leader = __ffsll((long long)peers) - 1;
            unsigned base = 0;
            if (lane == leader) base = atomicAdd(&row[c], (unsigned)__popcll(peers));
            base = __shfl(base, leader);
            const int64_t pos = list_off[c] + base + rank_in_mask(peers);
            ids[pos] = v;
        }
    }
}

// One grouping pass: list_off [K+1] and ids from the keys of `g`; cnt and size are scratch of the
// plan's sizes and are cleared here.
static void group_pass(const GroupKeys &g, int64_t n, int K, const GroupPlan &pl, char *ws, int64_t *list_off,
                       uint32_t *ids, hipStream_t st)
{
    unsigned *cnt = (unsigned *)(ws + pl.cnt_off);
    unsigned *size = (unsigned *)(ws + pl.size_off);
    const size_t n16 = pl.total / 16;
    hipLaunchKernelGGL(grp_zero_kernel, dim3((unsigned)std::min<size_t>(4096, ceil_div(n16, 256))), dim3(256), 0,
                       st, (uint4 *)ws, n16);
    const unsigned wg = (unsigned)ceil_div(pl.P, 4);
    if (n > 0) hipLaunchKernelGGL(grp_count_kernel, dim3(wg), dim3(256), 0, st, g, n, K, pl.part, pl.P, cnt);
    hipLaunchKernelGGL(grp_column_kernel, dim3((unsigned)ceil_div(K, 256)), dim3(256), 0, st, cnt, K, pl.P, size);
    hipLaunchKernelGGL(grp_offsets_kernel, dim3(1), dim3(1024), 0, st, size, K, list_off);
    if (n > 0) {
        int nbits = 1;
        while ((1ll << nbits) < K) ++nbits;
        hipLaunchKernelGGL(grp_place_kernel, dim3(wg), dim3(256), 0, st, g, n, K, nbits, pl.part, pl.P, cnt,
                           list_off, ids);
    }
}

int ivf_group(const int32_t *cells, int64_t n, int K, int64_t *list_off, uint32_t *ids, void *workspace,
              size_t workspace_bytes, hipStream_t st)
{
    GroupPlan g;
    if (!make_group_plan(n, K, &g))
        return fail(QADC_EINVAL, "qadc_ivf_group: n=%lld (at most 2^32) K=%d (at most 2^24)", (long long)n, K);
    if (!list_off || !workspace || (n > 0 && (!cells || !ids)))
        return fail(QADC_EINVAL, "qadc_ivf_group: null pointer");
    if (workspace_bytes < g.total || ((uintptr_t)workspace & 15))
        return fail(QADC_ENOMEM, "qadc_ivf_group: workspace of %zu bytes, %zu needed (16-byte aligned)",
                    workspace_bytes, g.total);
    group_pass(GroupKeys{cells, nullptr, nullptr, 0, 1, K}, n, K, g, (char *)workspace, list_off, ids, st);
    QADC_HIP_TRY(hipGetLastError());
    return QADC_OK;
}

// ---------------------------------------------------- group, occupied cells of a multi-index
//
// K*K cells are too many for one counter each, and most are empty.  The vectors are sorted by cell
// with two stable grouping passes over K keys -- by the second half's centroid, then, in that order,
// by the first half's -- which leaves them ordered by (first, second) = by cell id, input order
// kept inside a cell.  The places where the cell changes are the list boundaries: workgroups count
// them per 1024 places, one workgroup turns the counts into running sums, and a second pass writes
// each boundary's cell and place at its number.

constexpr int MIG_BLOCK = 1024;  // places per workgroup of the boundary kernels, 4 per thread

struct MiGroupPlan {
    GroupPlan g;
    int64_t nblocks;
    size_t perm_off, offa_off, offb_off, bcnt_off, boff_off, total;
};

static bool make_mi_group_plan(int64_t n, int Kh, MiGroupPlan *p)
{
    if (Kh < 1 || Kh > 16384 || !make_group_plan(n, Kh, &p->g)) return false;
    p->nblocks = std::max<int64_t>(1, ceil_div(n, MIG_BLOCK));
    size_t o = align_up(p->g.total, 256);
    p->perm_off = o; o += align_up((size_t)std::max<int64_t>(n, 1) * sizeof(uint32_t), 256);
    p->offa_off = o; o += align_up((size_t)(Kh + 1) * sizeof(int64_t), 256);
    p->offb_off = o; o += align_up((size_t)(Kh + 1) * sizeof(int64_t), 256);
    p->bcnt_off = o; o += align_up((size_t)p->nblocks * sizeof(unsigned), 256);
    p->boff_off = o; o += align_up((size_t)(p->nblocks + 1) * sizeof(int64_t), 256);
    p->total = o;
    return true;
}

size_t multi_index_group_workspace(int64_t n, int Kh)
{
    MiGroupPlan p;
    return make_mi_group_plan(n, Kh, &p) ? p.total : 0;
}

// is place p the first of its cell?  (places at and beyond n_valid are no boundaries)
__device__ inline bool mig_boundary(const int32_t *cells, const uint32_t *ids, int64_t p, int64_t n_valid, int *cell)
{
    if (p >= n_valid) return false;
    const int c = cells[ids[p]];
    *cell = c;
    return p == 0 || cells[ids[p - 1]] != c;
}

__global__ __launch_bounds__(256) void mig_count_kernel(const int32_t *__restrict__ cells,
                                                        const uint32_t *__restrict__ ids,
                                                        const int64_t *__restrict__ n_valid_p,
                                                        unsigned *__restrict__ bcnt)
{
    __shared__ unsigned wsum[4];
    const int64_t n_valid = *n_valid_p;
    const int64_t p0 = (int64_t)blockIdx.x * MIG_BLOCK + threadIdx.x * 4;
    unsigned c = 0;
    int cell;
#pragma unroll
    for (int e = 0; e < 4; ++e) c += mig_boundary(cells, ids, p0 + e, n_valid, &cell) ? 1u : 0u;
#pragma unroll
    for (int s = 32; s >= 1; s >>= 1) c += __shfl_xor(c, s);
    if ((threadIdx.x & 63) == 0) wsum[threadIdx.x >> 6] = c;
    __syncthreads();
    if (threadIdx.x == 0) bcnt[blockIdx.x] = wsum[0] + wsum[1] + wsum[2] + wsum[3];
}

__global__ __launch_bounds__(256) void mig_write_kernel(const int32_t *__restrict__ cells,
                                                        const uint32_t *__restrict__ ids,
                                                        const int64_t *__restrict__ n_valid_p,
                                                        const int64_t *__restrict__ boff, int64_t nblocks,
                                                        int64_t max_lists, uint32_t *__restrict__ cell_ids,
                                                        int64_t *__restrict__ list_off,
                                                        int64_t *__restrict__ n_lists)
{
    __shared__ unsigned wsum[4];
    const int64_t n_valid = *n_valid_p;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int64_t p0 = (int64_t)blockIdx.x * MIG_BLOCK + tid * 4;
    bool flag[4];
    int cell[4];
    unsigned c = 0;
#pragma unroll
    for (int e = 0; e < 4; ++e) {
        cell[e] = 0;
        flag[e] = mig_boundary(cells, ids, p0 + e, n_valid, &cell[e]);
        c += flag[e] ? 1u : 0u;
    }
    unsigned inc = c;  // inclusive sum inside the wavefront
#pragma unroll
    for (int s = 1; s < 64; s <<= 1) {
        const unsigned o = __shfl_up(inc, s);
        if (lane >= s) inc += o;
    }
    if (lane == 63) wsum[wave] = inc;
    __syncthreads();
    unsigned before = inc - c;
    for (int k = 0; k < wave; ++k) before += wsum[k];
    int64_t slot = boff[blockIdx.x] + before;
#pragma unroll
    for (int e = 0; e < 4; ++e)
        if (flag[e]) {
            if (slot < max_lists) {
                cell_ids[slot] = (uint32_t)cell[e];
                list_off[slot] = p0 + e;
            }
            ++slot;
        }
    if (blockIdx.x == 0 && tid == 0) {
        const int64_t L = boff[nblocks];
        n_lists[0] = L;
        list_off[min(L, max_lists)] = n_valid;
    }
}

int multi_index_group(const int32_t *cells, int64_t n, int Kh, int64_t max_lists, uint32_t *cell_ids,
                      int64_t *list_off, uint32_t *ids, int64_t *n_lists, void *workspace, size_t workspace_bytes,
                      hipStream_t st)
{
    MiGroupPlan p;
    if (!make_mi_group_plan(n, Kh, &p))
        return fail(QADC_EINVAL, "qadc_multi_index_group: n=%lld (at most 2^32) K=%d (at most 16384)", (long long)n, Kh);
    if (max_lists < std::min<int64_t>(n, (int64_t)Kh * Kh))
        return fail(QADC_EINVAL, "qadc_multi_index_group: max_lists=%lld, min(n, K*K)=%lld needed", (long long)max_lists,
                    (long long)std::min<int64_t>(n, (int64_t)Kh * Kh));
    if (!list_off || !n_lists || !workspace || (n > 0 && (!cells || !ids || !cell_ids)))
        return fail(QADC_EINVAL, "qadc_multi_index_group: null pointer");
    if (workspace_bytes < p.total || ((uintptr_t)workspace & 15))
        return fail(QADC_ENOMEM, "qadc_multi_index_group: workspace of %zu bytes, %zu needed (16-byte aligned)",
                    workspace_bytes, p.total);
    char *ws = (char *)workspace;
    uint32_t *perm = (uint32_t *)(ws + p.perm_off);
    int64_t *offa = (int64_t *)(ws + p.offa_off);
    int64_t *offb = (int64_t *)(ws + p.offb_off);
    unsigned *bcnt = (unsigned *)(ws + p.bcnt_off);
    int64_t *boff = (int64_t *)(ws + p.boff_off);
    const int cell_end = Kh * Kh;
    group_pass(GroupKeys{cells, nullptr, nullptr, 1, Kh, cell_end}, n, Kh, p.g, ws, offa, perm, st);
    group_pass(GroupKeys{cells, perm, offa + Kh, 2, Kh, cell_end}, n, Kh, p.g, ws, offb, ids, st);
    hipLaunchKernelGGL(mig_count_kernel, dim3((unsigned)p.nblocks), dim3(256), 0, st, cells, ids, offb + Kh, bcnt);
    hipLaunchKernelGGL(grp_offsets_kernel, dim3(1), dim3(1024), 0, st, bcnt, (int)p.nblocks, boff);
    hipLaunchKernelGGL(mig_write_kernel, dim3((unsigned)p.nblocks), dim3(256), 0, st, cells, ids, offb + Kh, boff,
                       p.nblocks, max_lists, cell_ids, list_off, n_lists);
    QADC_HIP_TRY(hipGetLastError());
    return QADC_OK;
}

}  // namespace qadc
