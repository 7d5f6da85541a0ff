// CSR first layer (the real-sim-shaped workload: ~50 non-zeros in 20,958 columns per row).
// The paper processes its datasets densely and leaves sparse input to future work
// (Section 8); the forward pass (Section 3, Eq. (1)), the gradient (Eq. (2)) and the update
// (Eq. (3)) of layer 1 are the same sums, run over the stored non-zeros only.
//
// gfx950 design: layer-1 weights are kept TRANSPOSED on the device (W1t: d_0 x d_1), so
// that the weights of one input column are one contiguous row: the forward SpMM gathers
// whole rows with 16-byte coalesced loads, and the gradient/update touches only the rows
// of columns that occur in the batch.  The gradient is column-segmented: the batch's
// non-zeros are bucketed by column (a per-batch CSC built on the device) and every column
// sums its rows of delta_1 once, then updates its weight row with a plain read-modify-write;
// a long column is shared by the 16-lane groups of one workgroup, whose partial sums meet
// in LDS in a fixed order.  Everything is HBM/L2-bandwidth work; no MFMA.
#include "hb_internal.h"

#include <mutex>
#include <stdlib.h>

namespace hb {
namespace {

constexpr int SP_NT = 128;    // threads per row / per chunk: one float4 each for d_1 = 512
constexpr int CHUNK = 128;    // a column with more entries is shared by several groups / workgroups
// One descriptor per column that occurs in the batch, laid out by size class: first the
// columns of at most LIGHT_MAX entries (most columns of a skewed distribution) by their exact
// number of entries, then those of at most CHUNK entries by their number of 16-entry gather
// windows, then the long ones.  A gather is one instruction for the four 16-lane groups of a
// wavefront and costs the texture-address unit the same 16 cycles however many of its lanes
// are active (measured: a quarter of the groups active, same time), and that unit is what
// bounds these kernels (83 % busy): so the groups of a wavefront should want the same number of
// gathers.  (In column order, a 128-entry column beside three one-entry columns left three
// quarters of seven gather windows idle.)
constexpr int LIGHT_MAX = 16;
constexpr int N_LIGHT = LIGHT_MAX;             // classes 0 .. 15: 1 .. 16 entries
constexpr int N_MID = CHUNK / 16 - 1;          // classes 16 .. 22: 2 .. 8 windows
constexpr int N_CLASS = N_LIGHT + N_MID + 1;   // class 23: more than CHUNK entries
__host__ __device__ inline int chunk_class(int cnt)
{
    if (cnt <= LIGHT_MAX) return cnt > 0 ? cnt - 1 : 0;
    if (cnt <= CHUNK) return N_LIGHT + (cnt + 15) / 16 - 2;
    return N_CLASS - 1;
}
// A column of more than SPLIT entries gets several descriptors, one per part of about equal
// length (whole gather windows), so that its parts run on different compute units.
constexpr int SPLIT = 1024;
__host__ __device__ inline int chunks_of(int cnt) { return cnt <= 0 ? 0 : (cnt + SPLIT - 1) / SPLIT; }
__host__ __device__ inline int part_len(int cnt, int parts) { return (((cnt + parts - 1) / parts) + 15) & ~15; }

constexpr int SPMM_CAP = 512;  // entries of a row staged in LDS at a time (forward product)

__device__ __forceinline__ float act_apply(float z, int act)
{
    if (act == ACT_SIGMOID) return 1.0f / (1.0f + __expf(-z));
    if (act == ACT_RELU) return fmaxf(z, 0.f);
    return z;
}

// A_1[i,:] = f(b_1 + sum_p vals[p] * W1t[col[p], :]), one workgroup per row
__global__ __launch_bounds__(SP_NT) void spmm_fwd_kernel(SpmmArgs a)
{
    const long long i = blockIdx.x;
    const int beg = a.row_ptr[i], end = a.row_ptr[i + 1];
    float *__restrict__ out = a.out + i * a.ldo;
    const int n4v = a.d1 >> 2;
    if (a.vec && n4v <= SP_NT) {
        // Outputs of up to 4 x SP_NT floats (one float4 per thread): the row's column indices
        // and values are brought into LDS once, coalesced, SPMM_CAP entries at a time, so that
        // the gathers do not each wait for a scalar load of their index first, and sixteen
        // weight-row gathers are in flight per thread.
        __shared__ int s_col[SPMM_CAP];
        __shared__ float s_val[SPMM_CAP];
        const int q = threadIdx.x;
        const bool live = q < n4v;
        float4 acc = live ? reinterpret_cast<const float4 *>(a.bias)[q] : make_float4(0.f, 0.f, 0.f, 0.f);
        for (int base = beg; base < end; base += SPMM_CAP) {
            const int n = min(SPMM_CAP, end - base);
            if (base != beg) __syncthreads();  // the previous chunk has been consumed
            for (int t = threadIdx.x; t < n; t += SP_NT) {
                s_col[t] = a.col_idx[base + t];
                s_val[t] = a.vals[base + t];
            }
            __syncthreads();
            if (live) {
                int p = 0;
                for (; p + 16 <= n; p += 16) {
                    float4 w[16];
#pragma unroll
                    for (int u = 0; u < 16; ++u)
                        w[u] = reinterpret_cast<const float4 *>(a.W1t + (size_t)s_col[p + u] * a.ldw)[q];
#pragma unroll
                    for (int u = 0; u < 16; ++u) {  // added in index order
                        const float v = s_val[p + u];
                        acc.x += v * w[u].x; acc.y += v * w[u].y; acc.z += v * w[u].z; acc.w += v * w[u].w;
                    }
                }
                if (p < n) {  // the tail: indices past the end are clamped, their values zero
                    float4 w[16];
#pragma unroll
                    for (int u = 0; u < 16; ++u)
                        w[u] = reinterpret_cast<const float4 *>(a.W1t + (size_t)s_col[min(p + u, n - 1)] * a.ldw)[q];
#pragma unroll
                    for (int u = 0; u < 16; ++u) {
                        const float v = (p + u < n) ? s_val[p + u] : 0.f;
                        acc.x += v * w[u].x; acc.y += v * w[u].y; acc.z += v * w[u].z; acc.w += v * w[u].w;
                    }
                }
            }
        }
        if (live) {
            acc.x = act_apply(acc.x, a.act); acc.y = act_apply(acc.y, a.act);
            acc.z = act_apply(acc.z, a.act); acc.w = act_apply(acc.w, a.act);
            reinterpret_cast<float4 *>(out)[q] = acc;
        }
    } else if (a.vec) {
        const int n4 = a.d1 >> 2;
        for (int q = threadIdx.x; q < n4; q += SP_NT) {
            float4 acc = reinterpret_cast<const float4 *>(a.bias)[q];
            int p = beg;
            for (; p + 8 <= end; p += 8) {  // eight row gathers in flight; added in index order
                float4 w[8];
                float v[8];
#pragma unroll
                for (int u = 0; u < 8; ++u) {
                    v[u] = a.vals[p + u];
                    w[u] = reinterpret_cast<const float4 *>(a.W1t + (size_t)a.col_idx[p + u] * a.ldw)[q];
                }
#pragma unroll
                for (int u = 0; u < 8; ++u) {
                    acc.x += v[u] * w[u].x; acc.y += v[u] * w[u].y; acc.z += v[u] * w[u].z; acc.w += v[u] * w[u].w;
                }
            }
            if (p < end) {  // the tail, also fetched together
                float4 w[8];
                float v[8];
#pragma unroll
                for (int u = 0; u < 8; ++u) {
                    const bool ok = p + u < end;
                    v[u] = ok ? a.vals[p + u] : 0.f;
                    w[u] = ok ? reinterpret_cast<const float4 *>(a.W1t + (size_t)a.col_idx[p + u] * a.ldw)[q]
                              : make_float4(0.f, 0.f, 0.f, 0.f);
                }
#pragma unroll
                for (int u = 0; u < 8; ++u)
                    if (p + u < end) {
                        acc.x += v[u] * w[u].x; acc.y += v[u] * w[u].y; acc.z += v[u] * w[u].z; acc.w += v[u] * w[u].w;
                    }
            }
            acc.x = act_apply(acc.x, a.act); acc.y = act_apply(acc.y, a.act);
            acc.z = act_apply(acc.z, a.act); acc.w = act_apply(acc.w, a.act);
            reinterpret_cast<float4 *>(out)[q] = acc;
        }
    } else {
        for (int j = threadIdx.x; j < a.d1; j += SP_NT) {
            float acc = a.bias[j];
            for (int p = beg; p < end; ++p)
                acc += a.vals[p] * a.W1t[(size_t)a.col_idx[p] * a.ldw + j];
            out[j] = act_apply(acc, a.act);
        }
    }
}

// ---- per-batch CSC by a multi-block counting sort (no global atomics: under a Zipf column
// distribution thousands of non-zeros share the hottest columns, and atomics on one address
// serialise).  Block b owns a contiguous range of rows:
//   1. csc_hist_kernel   block-local column histogram in LDS -> hist[b][c]
//   2. csc_colsum_kernel per column: exclusive prefix over blocks (in place) and total cnt[c]
//   3. col_scan_kernel   exclusive scan of cnt over columns -> col_start, chunk_start, and
//                        the chunk descriptors of the gradient kernel
//   4. csc_place_kernel  block b re-reads its rows; its LDS cursor of column c starts at
//                        col_start[c] + hist[b][c]; LDS atomics hand out the positions.
constexpr int CSC_NT = 1024;

__global__ __launch_bounds__(CSC_NT) void csc_hist_kernel(const int32_t *__restrict__ row_ptr,
                                                          const int32_t *__restrict__ col_idx,
                                                          long long B, int rows_per_block, int d0,
                                                          int32_t *__restrict__ hist)
{
    extern __shared__ int32_t s_hist[];
    for (int c = threadIdx.x; c < d0; c += CSC_NT) s_hist[c] = 0;
    __syncthreads();
    const long long r0 = (long long)blockIdx.x * rows_per_block;
    const long long r1 = min(B, r0 + rows_per_block);
    if (r0 < r1) {
        const int beg = row_ptr[r0], end = row_ptr[r1];
        // eight column indices are requested before the first LDS atomic needs one
        for (int p0 = beg + threadIdx.x; p0 < end; p0 += 8 * CSC_NT) {
            int c[8];
#pragma unroll
            for (int u = 0; u < 8; ++u) {
                const int p = p0 + u * CSC_NT;
                c[u] = (p < end) ? col_idx[p] : -1;
            }
#pragma unroll
            for (int u = 0; u < 8; ++u)
                if (c[u] >= 0) atomicAdd(&s_hist[c[u]], 1);
        }
    }
    __syncthreads();
    int32_t *out = hist + (size_t)blockIdx.x * d0;
    for (int c = threadIdx.x; c < d0; c += CSC_NT) out[c] = s_hist[c];
}

// Columns are handled in groups of 256 (one workgroup each) by the next two kernels.
constexpr int COLG = 256;

__device__ __forceinline__ int wave_incl_scan(int v, int lane)
{
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) {
        const int t = __shfl_up(v, o, 64);
        if (lane >= o) v += t;
    }
    return v;
}

// Sums over the workgroup's four wavefronts of N values; every thread gets the results.
template <int N>
__device__ __forceinline__ void group_sum(int (&v)[N], int *red /* 4 N ints of LDS */)
{
#pragma unroll
    for (int i = 0; i < N; ++i)
#pragma unroll
        for (int o = 32; o > 0; o >>= 1) v[i] += __shfl_xor(v[i], o, 64);
    const int wave = threadIdx.x >> 6;
    if ((threadIdx.x & 63) == 0) {
#pragma unroll
        for (int i = 0; i < N; ++i) red[4 * i + wave] = v[i];
    }
    __syncthreads();
#pragma unroll
    for (int i = 0; i < N; ++i) v[i] = red[4 * i] + red[4 * i + 1] + red[4 * i + 2] + red[4 * i + 3];
}

// Per column: exclusive prefix of its counts over the row blocks (in place in hist) and the
// total cnt[c]; per group of 256 columns: the group's totals of entries and of chunks per size
// class (group_tot[g], group_tot[(1 + class) n_groups + g]).
__global__ __launch_bounds__(COLG) void csc_colsum_kernel(int32_t *__restrict__ hist, int n_blocks, int d0,
                                                          int32_t *__restrict__ cnt,
                                                          int32_t *__restrict__ group_tot)
{
    __shared__ int red[4 * (1 + N_CLASS)];
    const int c = blockIdx.x * COLG + threadIdx.x;
    int run = 0;
    if (c < d0) {
        for (int b0 = 0; b0 < n_blocks; b0 += 16) {  // sixteen loads in flight, then the prefix
            int h[16];
#pragma unroll
            for (int u = 0; u < 16; ++u) h[u] = (b0 + u < n_blocks) ? hist[(size_t)(b0 + u) * d0 + c] : 0;
#pragma unroll
            for (int u = 0; u < 16; ++u)
                if (b0 + u < n_blocks) {
                    hist[(size_t)(b0 + u) * d0 + c] = run;
                    run += h[u];
                }
        }
        cnt[c] = run;
    }
    int tot[1 + N_CLASS] = {run};
    const int cls = chunk_class(run), ch = chunks_of(run);
#pragma unroll
    for (int k = 0; k < N_CLASS; ++k) tot[1 + k] = (k == cls) ? ch : 0;
    group_sum(tot, red);
    if (threadIdx.x == 0) {
#pragma unroll
        for (int i = 0; i <= N_CLASS; ++i) group_tot[i * gridDim.x + blockIdx.x] = tot[i];
    }
}

// Exclusive scan of cnt[0..n) (-> col_start) and the position of every column's descriptor
// (-> chunk_start; [n] = number of descriptors, [n + 1] = those of at most LIGHT_MAX entries,
// [n + 2] = of at most CHUNK entries): the columns of size class 0 come first, in column
// order, then class 1, and so on.  One descriptor {column, first entry, end entry, parts of the
// column} per column that occurs in the batch (per part of a column of more than SPLIT entries)
// lets the gradient kernel find its work with one load.
// One workgroup per group of 256 columns: it adds up the totals of the groups before it (and the
// class totals of ALL groups), scans its own columns with shuffles, and writes its outputs
// coalesced.  A column with several parts goes on an LDS list and the whole workgroup writes
// its descriptors.
// (A single-workgroup scan of all 21k columns took 20-60 us in three different forms: one
// CU's shuffle latency and store issue rate bound it.)
__global__ __launch_bounds__(COLG) void col_scan_kernel(const int32_t *__restrict__ cnt,
                                                        const int32_t *__restrict__ group_tot, int n,
                                                        int32_t *__restrict__ col_start,
                                                        int32_t *__restrict__ chunk_start,
                                                        int4 *__restrict__ chunk_desc)
{
    __shared__ int red[4 * (1 + N_CLASS)], w_a[4], w_c[4][N_CLASS];
    __shared__ int n_heavy;
    __shared__ int4 heavy[COLG];
    const int t = threadIdx.x, lane = t & 63, wave = t >> 6;
    const int g = blockIdx.x, n_groups = gridDim.x;
    const int c = g * COLG + t;
    const int v = (c < n) ? cnt[c] : 0;
    int before[1 + N_CLASS] = {};  // entries / chunks per class in the groups before this one
    int all[N_CLASS] = {};         // chunks per class of all groups
    for (int j = t; j < n_groups; j += COLG) {
        if (j < g) before[0] += group_tot[j];
#pragma unroll
        for (int k = 0; k < N_CLASS; ++k) {
            const int x = group_tot[(1 + k) * n_groups + j];
            if (j < g) before[1 + k] += x;
            all[k] += x;
        }
    }
    if (t == 0) n_heavy = 0;
    group_sum(before, red);  // its barrier also publishes n_heavy
    __syncthreads();         // red is reused
    group_sum(all, red);
    const int cls = chunk_class(v), ch = chunks_of(v);
    const int ia = wave_incl_scan(v, lane);
    int ic[N_CLASS];
#pragma unroll
    for (int k = 0; k < N_CLASS; ++k) ic[k] = wave_incl_scan(k == cls ? ch : 0, lane);
    if (lane == 63) {
        w_a[wave] = ia;
#pragma unroll
        for (int k = 0; k < N_CLASS; ++k) w_c[wave][k] = ic[k];
    }
    __syncthreads();
    int first_e = before[0] + ia - v;
    int first_ch = 0;  // chunks of the classes before this column's, then the earlier chunks of its own class
#pragma unroll
    for (int k = 0; k < N_CLASS; ++k) {
        if (k < cls) first_ch += all[k];
        if (k == cls) {
            first_ch += before[1 + k] + ic[k] - ch;
            for (int w = 0; w < wave; ++w) first_ch += w_c[w][k];
        }
    }
    for (int w = 0; w < wave; ++w) first_e += w_a[w];
    if (c < n) {
        col_start[c] = first_e;
        chunk_start[c] = first_ch;
        if (c == n - 1) {
            int total = 0;
#pragma unroll
            for (int k = 0; k < N_CLASS; ++k) total += all[k];
            col_start[n] = first_e + v;
            chunk_start[n] = total;
            int light = 0, mid = 0;
#pragma unroll
            for (int k = 0; k < N_LIGHT; ++k) light += all[k];
#pragma unroll
            for (int k = N_LIGHT; k < N_CLASS - 1; ++k) mid += all[k];
            chunk_start[n + 1] = light;
            chunk_start[n + 2] = light + mid;
        }
        if (ch == 1) chunk_desc[first_ch] = make_int4(c, first_e, first_e + v, 1);
        else if (ch > 1) heavy[atomicAdd(&n_heavy, 1)] = make_int4(c, first_e, v, first_ch);
    }
    __syncthreads();
    const int nh = n_heavy;  // the whole workgroup writes the descriptors of a column's parts
    for (int k = 0; k < nh; ++k) {
        const int4 h = heavy[k];  // {column, first entry, entries, first descriptor}
        const int parts = chunks_of(h.z), len = part_len(h.z, parts);
        for (int q = t; q < parts; q += COLG)
            chunk_desc[h.w + q] = make_int4(h.x, min(h.y + h.z, h.y + q * len), min(h.y + h.z, h.y + (q + 1) * len), parts);
    }
}

__global__ __launch_bounds__(CSC_NT) void csc_place_kernel(const int32_t *__restrict__ row_ptr,
                                                           const int32_t *__restrict__ col_idx,
                                                           const float *__restrict__ vals, long long B,
                                                           int rows_per_block, int d0,
                                                           const int32_t *__restrict__ hist,
                                                           const int32_t *__restrict__ col_start,
                                                           int2 *__restrict__ csc_ent)
{
    extern __shared__ int32_t s_cur[];
    const int32_t *mine = hist + (size_t)blockIdx.x * d0;
    // LDS holds how many entries of each column this block has placed so far; the column's
    // base offset (col_start + this block's exclusive prefix) is fetched per non-zero, which
    // touches far fewer words than initialising d0 cursors from global memory would
    for (int c = threadIdx.x; c < d0; c += CSC_NT) s_cur[c] = 0;
    __syncthreads();
    const long long r0 = (long long)blockIdx.x * rows_per_block;
    const long long r1 = min(B, r0 + rows_per_block);
    if (r0 >= r1) return;
    // the block's slice of row_ptr sits behind the cursors in LDS: rows are found by bisection there
    int32_t *s_rp = s_cur + d0;
    const int nr = (int)(r1 - r0);
    for (int i = threadIdx.x; i <= nr; i += CSC_NT) s_rp[i] = row_ptr[r0 + i];
    __syncthreads();
    const int beg = s_rp[0], end = s_rp[nr];
    // one thread per non-zero of the block's contiguous range, four at a time so that the
    // dependent loads (column -> base offsets -> position) of the four overlap
    for (int p0 = beg + threadIdx.x; p0 < end; p0 += 4 * CSC_NT) {
        int c[4], base[4];
        float val[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const int p = p0 + u * CSC_NT;
            c[u] = (p < end) ? col_idx[p] : -1;
            val[u] = (p < end) ? vals[p] : 0.f;
        }
#pragma unroll
        for (int u = 0; u < 4; ++u) base[u] = (c[u] >= 0) ? col_start[c[u]] + mine[c[u]] : 0;
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            if (c[u] < 0) continue;
            const int p = p0 + u * CSC_NT;
            int lo = 0, hi = nr;  // s_rp[lo] <= p < s_rp[hi]
            while (hi - lo > 1) {
                const int mid = (lo + hi) >> 1;
                if (s_rp[mid] <= p) lo = mid; else hi = mid;
            }
            const int pos = base[u] + atomicAdd(&s_cur[c[u]], 1);
            csc_ent[pos] = make_int2((int)(r0 + lo), __float_as_int(val[u]));
        }
    }
}

// One workgroup per column that occurs in the batch:
//   g[:] = sum_e val[e] * delta_1[row[e], :]   over the column's entries {row, val} of csc_ent
// then W1t[c,:] -= lr * g, or in gradient mode dW_1[:, c] = g in the flat out x in layout.
// A descriptor of more than CHUNK entries (the last class) is cut into up to FB_PARTS parts: its
// workgroup takes the first, and the FB_EXTRA workgroups behind the descriptors walk over the
// other parts of all such descriptors; the sums of a column's parts meet through fp32 atomic adds.
constexpr int FB_PARTS = 32, FB_EXTRA = 2048;
__device__ __forceinline__ int fb_part_len(int cnt)
{
    const int per = (((cnt + FB_PARTS - 1) / FB_PARTS) + 15) & ~15;
    return per > CHUNK ? per : CHUNK;
}

// entries [e_beg, e_end) of column c: their sum, then the update (plain if `single`)
__device__ __forceinline__ void sparse_dw_part(const SparseDwArgs &a, int c, int e_beg, int e_end, bool single)
{
    if (a.vec) {
        const int n4 = a.d1 >> 2;
        for (int q = threadIdx.x; q < n4; q += SP_NT) {
            float4 g = {0.f, 0.f, 0.f, 0.f};
            int e = e_beg;
            for (; e + 16 <= e_end; e += 16) {  // sixteen row gathers in flight; added in index order
                float4 d[16];
                float v[16];
#pragma unroll
                for (int u = 0; u < 16; ++u) {
                    const int2 en = a.csc_ent[e + u];
                    v[u] = __int_as_float(en.y);
                    d[u] = reinterpret_cast<const float4 *>(a.delta + (size_t)en.x * a.ldd)[q];
                }
#pragma unroll
                for (int u = 0; u < 16; ++u) {
                    g.x += v[u] * d[u].x; g.y += v[u] * d[u].y; g.z += v[u] * d[u].z; g.w += v[u] * d[u].w;
                }
            }
            if (e < e_end) {  // the tail, also fetched together (entries past the end read as zero)
                float4 d[16];
                float v[16];
#pragma unroll
                for (int u = 0; u < 16; ++u) {
                    const bool ok = e + u < e_end;
                    const int2 en = a.csc_ent[ok ? e + u : e];
                    v[u] = ok ? __int_as_float(en.y) : 0.f;
                    d[u] = ok ? reinterpret_cast<const float4 *>(a.delta + (size_t)en.x * a.ldd)[q]
                              : make_float4(0.f, 0.f, 0.f, 0.f);
                }
#pragma unroll
                for (int u = 0; u < 16; ++u)
                    if (e + u < e_end) {
                        g.x += v[u] * d[u].x; g.y += v[u] * d[u].y; g.z += v[u] * d[u].z; g.w += v[u] * d[u].w;
                    }
            }
            if (a.grad_out) {
                float *o = a.grad_out + (size_t)(4 * q) * a.d0 + c;
                if (single) { o[0] = g.x; o[a.d0] = g.y; o[2 * (size_t)a.d0] = g.z; o[3 * (size_t)a.d0] = g.w; }
                else {
                    atomicAdd(o, g.x); atomicAdd(o + a.d0, g.y);
                    atomicAdd(o + 2 * (size_t)a.d0, g.z); atomicAdd(o + 3 * (size_t)a.d0, g.w);
                }
            } else {
                float *w = a.W1t + (size_t)c * a.ldw + 4 * q;
                if (single) {
                    float4 x = *reinterpret_cast<float4 *>(w);
                    x.x -= a.lr * g.x; x.y -= a.lr * g.y; x.z -= a.lr * g.z; x.w -= a.lr * g.w;
                    *reinterpret_cast<float4 *>(w) = x;
                } else {
                    atomicAdd(w, -a.lr * g.x); atomicAdd(w + 1, -a.lr * g.y);
                    atomicAdd(w + 2, -a.lr * g.z); atomicAdd(w + 3, -a.lr * g.w);
                }
            }
        }
    } else {
        for (int j = threadIdx.x; j < a.d1; j += SP_NT) {
            float g = 0.f;
            for (int e = e_beg; e < e_end; ++e)
            {
                const int2 en = a.csc_ent[e];
                g += __int_as_float(en.y) * a.delta[(size_t)en.x * a.ldd + j];
            }
            if (a.grad_out) {
                float *o = a.grad_out + (size_t)j * a.d0 + c;
                if (single) *o = g; else atomicAdd(o, g);
            } else {
                float *w = a.W1t + (size_t)c * a.ldw + j;
                if (single) *w -= a.lr * g; else atomicAdd(w, -a.lr * g);
            }
        }
    }
}

__global__ __launch_bounds__(SP_NT) void sparse_dw_kernel(SparseDwArgs a, int max_desc)
{
    const int n_desc = a.chunk_start[a.d0], n01 = a.chunk_start[a.d0 + 2];
    if ((int)blockIdx.x < max_desc) {
        if ((int)blockIdx.x >= n_desc) return;
        const int4 desc = a.chunk_desc[blockIdx.x];
        const int per = fb_part_len(desc.z - desc.y);
        sparse_dw_part(a, desc.x, desc.y, min(desc.z, desc.y + per), desc.w == 1 && desc.z - desc.y <= per);
        return;
    }
    const int n_work = (n_desc - n01) * (FB_PARTS - 1);
    for (int w = (int)blockIdx.x - max_desc; w < n_work; w += FB_EXTRA) {
        const int4 desc = a.chunk_desc[n01 + w / (FB_PARTS - 1)];
        const int per = fb_part_len(desc.z - desc.y);
        const int beg = desc.y + (1 + w % (FB_PARTS - 1)) * per;
        if (beg < desc.z) sparse_dw_part(a, desc.x, beg, min(desc.z, beg + per), false);
    }
}

// ---- XCD-sliced forms of the two gather kernels (d_1 a multiple of 64 with d_1 / 64 dividing,
// or a multiple of, 8).
//
// Both kernels above gather one whole 2 KB row (of W1t, of delta_1) per stored entry: 0.69 GB
// per batch of the real-sim shape, from tensors of 43 MB and 17 MB that no 4 MB L2 holds, so
// the gathers are served by the fabric behind the L2s (the backward kernel ran at 7.5 TB/s of
// gathers).  Here the feature dimension d_1 is cut
// into slices of 64 floats and slice s is given to XCD s % 8 (workgroup ids go round-robin over
// the XCDs): an XCD then only ever touches its 256-byte piece of every row -- 2 MB of delta_1
// at B = 8192, 5 MB of W1t of which the hot rows stay -- and the gathers hit its own L2.
// A group of 16 lanes owns one (row, slice) or (chunk, slice): one float4 per lane; the
// group's indices and values are loaded 16 at a time, one per lane, and handed round with
// lane shuffles, so 16 gathers are in flight per lane without any LDS staging.  Entries are
// added in index order.  Measured on the real-sim shape (B = 8192, CSC build on the same
// stream): forward 42.6 -> 39.5 us, weight gradient 91.4 -> 70.4 us; the gathers now run at
// about half of what the L2s can deliver (17.6 and 9.8 TB/s).
constexpr int SL = 64;       // floats per slice
constexpr int XS_NT = 256;   // 16 groups of 16 lanes

struct SliceMap {
    int n_sl;       // slices of d_1
    int reps;       // slices per XCD             (n_sl % 8 == 0), else 1
    int parts;      // XCDs that share one slice  (8 % n_sl == 0), else 1
};

// workgroup id -> (slice, unit); units are dealt to the `parts` XCDs of a slice in turn
__device__ __forceinline__ void slice_of_block(const SliceMap &m, int b, int &slice, int &unit)
{
    const int x = b & 7, q = b >> 3;
    if (m.parts == 1) {
        slice = x + 8 * (q % m.reps);
        unit = q / m.reps;
    } else {
        slice = x % m.n_sl;
        unit = q * m.parts + x / m.n_sl;
    }
}

// One group of 16 lanes: sum over entries [beg, end) of val[e] * src[idx[e] * ld + 0..3] (src
// already points at the lane's float4 of the slice).  idx / val are read 16 entries at a time,
// lane l taking entry p + l; a full window issues its 16 gathers together, the last, partial
// window four at a time (lanes past the end hold the last valid index and a zero value).
// (One form for both -- 16 gathers, each group's lanes switched off past its end, an
// instruction that no group of the wavefront needs skipped -- issues 15 % fewer gathers in the
// forward product and is slower, 41.0 -> 42.7 us: a branch per gather.)
// AHEAD: the next window's idx / val are requested in front of the current window's gathers.
// For a long run of windows on one group (the critical path of a long column) that takes one
// of two round trips out of every window; where many short runs keep the memory pipeline full
// it only adds to the traffic in flight (forward product: 39.5 -> 42.6 us).
// Where the entries {index, value} of a gather run come from: the caller's CSR arrays, or the
// per-batch CSC copy (one 8-byte word per entry).
struct CsrEntries {
    const int32_t *__restrict__ idx;
    const float *__restrict__ val;
    __device__ __forceinline__ void get(int at, bool live, int &i, float &v) const
    {
        i = idx[at];
        v = live ? val[at] : 0.f;
    }
};
struct CscEntries {
    const int2 *__restrict__ ent;
    __device__ __forceinline__ void get(int at, bool live, int &i, float &v) const
    {
        const int2 e = ent[at];
        i = e.x;
        v = live ? __int_as_float(e.y) : 0.f;
    }
};

template <bool AHEAD = false, class Entries>
__device__ __forceinline__ float4 group_gather_sum(float4 acc, const Entries en, int beg, int end,
                                                   const float *__restrict__ src, size_t ld, int l)
{
    int nx_i = 0;
    float nx_v = 0.f;
    if (AHEAD && beg < end) en.get(min(beg + l, end - 1), beg + l < end, nx_i, nx_v);
    for (int p = beg; p < end; p += 16) {
        int my_i;
        float my_v;
        if (AHEAD) {
            my_i = nx_i;
            my_v = nx_v;
            if (p + 16 < end) en.get(min(p + 16 + l, end - 1), p + 16 + l < end, nx_i, nx_v);
        } else {
            en.get(min(p + l, end - 1), p + l < end, my_i, my_v);
        }
        if (p + 16 <= end) {
            float4 w[16];
#pragma unroll
            for (int u = 0; u < 16; ++u)
                w[u] = *reinterpret_cast<const float4 *>(src + (size_t)__shfl(my_i, u, 16) * ld);
#pragma unroll
            for (int u = 0; u < 16; ++u) {
                const float v = __shfl(my_v, u, 16);
                acc.x += v * w[u].x; acc.y += v * w[u].y; acc.z += v * w[u].z; acc.w += v * w[u].w;
            }
        } else {
            for (int u0 = 0; p + u0 < end; u0 += 4) {
                float4 w[4];
#pragma unroll
                for (int u = 0; u < 4; ++u)
                    w[u] = *reinterpret_cast<const float4 *>(src + (size_t)__shfl(my_i, u0 + u, 16) * ld);
#pragma unroll
                for (int u = 0; u < 4; ++u) {
                    const float v = __shfl(my_v, u0 + u, 16);
                    acc.x += v * w[u].x; acc.y += v * w[u].y; acc.z += v * w[u].z; acc.w += v * w[u].w;
                }
            }
        }
    }
    return acc;
}

// A_1[i, slice] = f(b_1 + sum_p vals[p] * W1t[col[p], slice]); unit = 16 consecutive rows
__global__ __launch_bounds__(XS_NT) void spmm_fwd_sliced_kernel(SpmmArgs a, long long B, SliceMap m, int units)
{
    int slice, unit;
    slice_of_block(m, blockIdx.x, slice, unit);
    if (unit >= units) return;
    const int g = threadIdx.x >> 4, l = threadIdx.x & 15;
    const long long row = (long long)unit * 16 + g;
    if (row >= B) return;
    const int beg = a.row_ptr[row], end = a.row_ptr[row + 1];
    const int col0 = slice * SL + 4 * l;
    float4 acc = *reinterpret_cast<const float4 *>(a.bias + col0);
    acc = group_gather_sum(acc, CsrEntries{a.col_idx, a.vals}, beg, end, a.W1t + col0, (size_t)a.ldw, l);
    acc.x = act_apply(acc.x, a.act); acc.y = act_apply(acc.y, a.act);
    acc.z = act_apply(acc.z, a.act); acc.w = act_apply(acc.w, a.act);
    *reinterpret_cast<float4 *>(a.out + (size_t)row * a.ldo + col0) = acc;
}

// W1t[c, slice] -= lr * g (or the gradient output) for the sum g of column c
__device__ __forceinline__ void apply_column_sum(const SparseDwArgs &a, int c, int col0, float4 g)
{
    if (a.grad_out) {
        float *o = a.grad_out + (size_t)col0 * a.d0 + c;
        o[0] = g.x; o[a.d0] = g.y; o[2 * (size_t)a.d0] = g.z; o[3 * (size_t)a.d0] = g.w;
    } else {
        float *w = a.W1t + (size_t)c * a.ldw + col0;
        float4 x = *reinterpret_cast<float4 *>(w);
        x.x -= a.lr * g.x; x.y -= a.lr * g.y; x.z -= a.lr * g.z; x.w -= a.lr * g.w;
        *reinterpret_cast<float4 *>(w) = x;
    }
}

// the same for one of several parts of a column, whose sums meet through fp32 atomic adds
__device__ __forceinline__ void apply_part_sum(const SparseDwArgs &a, int c, int col0, float4 g)
{
    if (a.grad_out) {
        float *o = a.grad_out + (size_t)col0 * a.d0 + c;
        atomicAdd(o, g.x); atomicAdd(o + a.d0, g.y);
        atomicAdd(o + 2 * (size_t)a.d0, g.z); atomicAdd(o + 3 * (size_t)a.d0, g.w);
    } else {
        float *w = a.W1t + (size_t)c * a.ldw + col0;
        atomicAdd(w, -a.lr * g.x); atomicAdd(w + 1, -a.lr * g.y);
        atomicAdd(w + 2, -a.lr * g.z); atomicAdd(w + 3, -a.lr * g.w);
    }
}

// g[slice] = sum_e val[e] * delta_1[row[e], slice] over one column's entries, then the update of
// W1t[c, slice] (or the gradient output).  unit = one workgroup = 16 groups of 16 lanes.
// First come the descriptors of more than CHUNK entries, a unit each (the
// head of a skewed distribution holds half of all entries in a few hundred columns): the 16
// groups share one column's entries in contiguous runs of whole gather windows, their sums
// meet in LDS and are added in group order, and the first group updates the row (with one fp32
// atomic add per 128-entry chunk instead, the kernel took 65.8 us on the real-sim shape; a
// plain, racing read-modify-write in their place, to price them: 52.7).  Such a workgroup is
// bound by what ONE compute unit gathers -- the hottest column of that batch, 8,100 entries,
// took 43 us, as long as the rest of the kernel -- so a column of more than SPLIT entries
// comes as several descriptors whose workgroups add their sums with fp32 atomic adds (a few
// dozen columns, about a hundred parts).
// Last the columns of at most LIGHT_MAX entries (most of them one to three): a group takes
// LP of them at once and issues every step of their chains (descriptors, indices, gathers
// LR per column and round, weight rows) for all LP together -- one such column alone is five
// dependent round trips with nothing to overlap them but other groups.  Between the two, the
// columns of 2 .. 8 gather windows, one per group.  Within each class range the units run from
// the largest columns down, so that the launch ends on its shortest work.
// (Requesting the descriptor together with the descriptor count, and the weight row of a
// class-1 column before the gathers instead of after them, was slower: 70 -> 76 us.)
constexpr int LP = 4, LR = 2, DW_UNITS = 1024;
__global__ __launch_bounds__(XS_NT) void sparse_dw_sliced_kernel(SparseDwArgs a, SliceMap m, int units)
{
    int slice, unit;
    slice_of_block(m, blockIdx.x, slice, unit);
    if (unit >= units) return;
    const int g16 = threadIdx.x >> 4, l = threadIdx.x & 15;
    const int n_desc = a.chunk_start[a.d0], n_light = a.chunk_start[a.d0 + 1], n01 = a.chunk_start[a.d0 + 2];
    const int col0 = slice * SL + 4 * l;
    const int long_units = n_desc - n01, mid_units = (n01 - n_light + 15) / 16;
    const int light_units = (n_light + 16 * LP - 1) / (16 * LP);
    const int need = long_units + mid_units + light_units;
    __shared__ float4 part[16][16];
    // the launch has a fixed number of units (how many the batch needs is only known here):
    // a unit takes every `units`-th piece of work, long descriptors first
    for (int vu = unit; vu < need; vu += units) {
        if (vu < long_units) {
            const int4 desc = a.chunk_desc[n01 + vu];
            const int per = (((desc.z - desc.y + 15) >> 4) + 15) & ~15;  // entries per group: whole windows
            const int beg = min(desc.z, desc.y + g16 * per);
            float4 g = {0.f, 0.f, 0.f, 0.f};
            g = group_gather_sum<true>(g, CscEntries{a.csc_ent}, beg, min(desc.z, beg + per), a.delta + col0, (size_t)a.ldd, l);
            part[g16][l] = g;
            __syncthreads();
            if (g16 == 0) {
                float4 sum = part[0][l];
#pragma unroll
                for (int k = 1; k < 16; ++k) {
                    const float4 p = part[k][l];
                    sum.x += p.x; sum.y += p.y; sum.z += p.z; sum.w += p.w;
                }
                if (desc.w == 1) apply_column_sum(a, desc.x, col0, sum);
                else apply_part_sum(a, desc.x, col0, sum);
            }
            __syncthreads();  // part is reused
            continue;
        }
        // the columns of 2 .. 8 windows next, longest first, so that the kernel ends on short work
        if (vu < long_units + mid_units) {
            const int j = n_light + (mid_units - 1 - (vu - long_units)) * 16 + g16;
            if (j >= n01) continue;
            const int4 desc = a.chunk_desc[j];
            float4 g = {0.f, 0.f, 0.f, 0.f};
            g = group_gather_sum(g, CscEntries{a.csc_ent}, desc.y, desc.z, a.delta + col0, (size_t)a.ldd, l);
            apply_column_sum(a, desc.x, col0, g);
            continue;
        }
        const int first = ((need - 1 - vu) * 16 + g16) * LP;  // also from the largest down
        if (first >= n_light) continue;
        int c[LP], n[LP], my_i[LP];
        float my_v[LP];
        // lane k of the group fetches descriptor k; the others get it by shuffle
        const int4 mine = a.chunk_desc[min(first + min(l, LP - 1), n_light - 1)];
        int n_max = 0;
#pragma unroll
        for (int k = 0; k < LP; ++k) {
            c[k] = __shfl(mine.x, k, 16);
            const int e0 = __shfl(mine.y, k, 16), e1 = __shfl(mine.z, k, 16);
            n[k] = (first + k < n_light) ? e1 - e0 : 0;  // 1 .. LIGHT_MAX entries
            n_max = max(n_max, n[k]);
            // lanes past the end hold the last entry's row and a zero value
            const int2 en = a.csc_ent[e0 + min(l, max(n[k], 1) - 1)];
            my_i[k] = en.x;
            my_v[k] = (l < n[k]) ? __int_as_float(en.y) : 0.f;
        }
        float4 g[LP];
#pragma unroll
        for (int k = 0; k < LP; ++k) g[k] = make_float4(0.f, 0.f, 0.f, 0.f);
        const float *src = a.delta + col0;
        int u0 = 0;
        for (; u0 + LR <= n_max; u0 += LR) {
            float4 w[LP][LR];
#pragma unroll
            for (int k = 0; k < LP; ++k)
#pragma unroll
                for (int u = 0; u < LR; ++u)
                    w[k][u] = *reinterpret_cast<const float4 *>(src + (size_t)__shfl(my_i[k], u0 + u, 16) * a.ldd);
#pragma unroll
            for (int k = 0; k < LP; ++k)
#pragma unroll
                for (int u = 0; u < LR; ++u) {
                    const float v = __shfl(my_v[k], u0 + u, 16);
                    g[k].x += v * w[k][u].x; g[k].y += v * w[k][u].y; g[k].z += v * w[k][u].z; g[k].w += v * w[k][u].w;
                }
        }
        if (u0 < n_max) {  // an odd number of entries (the four columns mostly have the same): one gather each
            float4 w[LP];
#pragma unroll
            for (int k = 0; k < LP; ++k)
                w[k] = *reinterpret_cast<const float4 *>(src + (size_t)__shfl(my_i[k], u0, 16) * a.ldd);
#pragma unroll
            for (int k = 0; k < LP; ++k) {
                const float v = __shfl(my_v[k], u0, 16);
                g[k].x += v * w[k].x; g[k].y += v * w[k].y; g[k].z += v * w[k].z; g[k].w += v * w[k].w;
            }
        }
        if (a.grad_out) {
#pragma unroll
            for (int k = 0; k < LP; ++k)
                if (first + k < n_light) apply_column_sum(a, c[k], col0, g[k]);
        } else {  // the LP weight rows are requested together (distinct columns: no row twice)
            float4 x[LP];
#pragma unroll
            for (int k = 0; k < LP; ++k) x[k] = *reinterpret_cast<const float4 *>(a.W1t + (size_t)c[k] * a.ldw + col0);
#pragma unroll
            for (int k = 0; k < LP; ++k) {
                x[k].x -= a.lr * g[k].x; x[k].y -= a.lr * g[k].y; x[k].z -= a.lr * g[k].z; x[k].w -= a.lr * g[k].w;
                if (first + k < n_light) *reinterpret_cast<float4 *>(a.W1t + (size_t)c[k] * a.ldw + col0) = x[k];
            }
        }
    }
}

// partial[s][j] = sum over the s-th slice of rows of delta[i][j]   (bias gradient of layer 1)
__global__ __launch_bounds__(256) void colsum_kernel(const float *__restrict__ delta, int ldd,
                                                     long long B, int d, int rows_per_split,
                                                     float *__restrict__ partial)
{
    __shared__ float red[4][64];
    const int col = blockIdx.x * 64 + (threadIdx.x & 63);
    const int rg = threadIdx.x >> 6;
    const long long r0 = (long long)blockIdx.y * rows_per_split;
    const long long r1 = min(B, r0 + rows_per_split);
    float s = 0.f;
    if (col < d) {
        // eight rows requested before the first is added: the slice is a chain of loads otherwise
        long long i = r0 + rg;
        float s1 = 0.f;
        for (; i + 28 < r1; i += 32) {
            float v[8];
#pragma unroll
            for (int u = 0; u < 8; ++u) v[u] = delta[(i + 4 * u) * ldd + col];
            s += (v[0] + v[1]) + (v[2] + v[3]);
            s1 += (v[4] + v[5]) + (v[6] + v[7]);
        }
        for (; i < r1; i += 4) s += delta[i * ldd + col];
        s += s1;
    }
    red[rg][threadIdx.x & 63] = s;
    __syncthreads();
    if (rg == 0 && col < d)
        partial[(size_t)blockIdx.y * d + col] = red[0][threadIdx.x] + red[1][threadIdx.x] +
                                                 red[2][threadIdx.x] + red[3][threadIdx.x];
}

// out[c][r] = in[r][c]  (R x C -> C x R), 32 x 32 tiles through LDS
__global__ __launch_bounds__(256) void transpose_kernel(const float *__restrict__ in, float *__restrict__ out,
                                                        int R, int C)
{
    __shared__ float t[32][33];
    const int tx = threadIdx.x & 31, ty = threadIdx.x >> 5;  // 32 x 8
    const int c0 = blockIdx.x * 32, r0 = blockIdx.y * 32;
    for (int k = ty; k < 32; k += 8)
        if (r0 + k < R && c0 + tx < C) t[k][tx] = in[(size_t)(r0 + k) * C + c0 + tx];
    __syncthreads();
    for (int k = ty; k < 32; k += 8)
        if (c0 + k < C && r0 + tx < R) out[(size_t)(c0 + k) * R + r0 + tx] = t[tx][k];
}

}  // namespace

// The sliced kernels apply when d_1 is a whole number of 64-float slices that divides, or is a
// multiple of, the 8 XCDs.  HB_SPARSE_SLICED=0 (tuning aid) keeps the row-per-workgroup kernels.
static bool slice_map(int d1, int vec, SliceMap *m)
{
    static const bool off = getenv("HB_SPARSE_SLICED") && atoi(getenv("HB_SPARSE_SLICED")) == 0;
    if (off || !vec || d1 < SL || d1 % SL != 0) return false;
    const int n = d1 / SL;
    if (n % 8 == 0) { *m = SliceMap{n, n / 8, 1}; return true; }
    if (8 % n == 0) { *m = SliceMap{n, 1, 8 / n}; return true; }
    return false;
}

// workgroups of a sliced launch over `units` units
static long long sliced_blocks(const SliceMap &m, long long units)
{
    return m.parts == 1 ? 8LL * m.reps * units : 8LL * ((units + m.parts - 1) / m.parts);
}

hipError_t launch_spmm_fwd(const SpmmArgs &a, long long B, hipStream_t stream, const LaunchEvents &ev)
{
    SliceMap m;
    if (slice_map(a.d1, a.vec, &m)) {
        const long long units = (B + 15) / 16;
        const long long blocks = sliced_blocks(m, units);
        if (blocks <= 0x7fffffffLL)
            return launch_kernel(spmm_fwd_sliced_kernel, dim3((unsigned)blocks), dim3(XS_NT), stream, ev, a, B, m,
                                 (int)units);
    }
    return launch_kernel(spmm_fwd_kernel, dim3((unsigned)B), dim3(SP_NT), stream, ev, a);
}

size_t sparse_desc_capacity(int d0, long long nnz_cap) { return (size_t)d0 + 1 + (size_t)(nnz_cap / SPLIT); }

int csc_blocks(long long B)
{
    long long nb = (B + 127) / 128;  // at least 128 rows per block
    if (nb > 64) nb = 64;
    if (nb < 1) nb = 1;
    return (int)nb;
}

// The per-block column histogram plus the block's slice of row_ptr must fit LDS.
bool csc_supported(int d0, long long max_B)
{
    const int nb = csc_blocks(max_B);
    const long long rows_per_block = (max_B + nb - 1) / nb;
    return ((long long)d0 + rows_per_block + 1) * (long long)sizeof(int32_t) <= 150 * 1024;
}

// cnt[d0 + 1] followed by the per-group totals of the column scan
size_t csc_cnt_elems(int d0) { return (size_t)d0 + 1 + (1 + N_CLASS) * (size_t)((d0 + COLG - 1) / COLG); }

size_t csc_hist_elems(long long max_B, int d0) { return (size_t)csc_blocks(max_B) * (size_t)d0; }


hipError_t launch_csc_build(const int32_t *row_ptr, const int32_t *col_idx, const float *vals,
                            long long nnz, long long B, int d0, int32_t *hist, int32_t *cnt,
                            int32_t *col_start, int32_t *chunk_start, int4 *chunk_desc, int2 *csc_ent,
                            hipStream_t stream, const LaunchEvents &ev_hist,
                            const LaunchEvents &ev_colsum, const LaunchEvents &ev_scan,
                            const LaunchEvents &ev_place)
{
    (void)nnz;
    const int nb = csc_blocks(B);
    const int rows_per_block = (int)((B + nb - 1) / nb);
    const size_t lds = ((size_t)d0 + (size_t)rows_per_block + 1) * sizeof(int32_t);
    // more than 64 KB of dynamic LDS has to be requested per kernel
    static std::mutex lds_mu;  // handles on different host threads launch concurrently
    static size_t lds_granted = 0;
    if (lds > 32 * 1024) {
        std::lock_guard<std::mutex> lk(lds_mu);
        if (lds > lds_granted) {
            hipError_t ea = hipFuncSetAttribute(reinterpret_cast<const void *>(csc_hist_kernel),
                                                hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
            if (ea == hipSuccess)
                ea = hipFuncSetAttribute(reinterpret_cast<const void *>(csc_place_kernel),
                                         hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
            if (ea != hipSuccess) return ea;
            lds_granted = lds;
        }
    }
    if (ev_hist.start)
        hipExtLaunchKernelGGL(csc_hist_kernel, dim3(nb), dim3(CSC_NT), (unsigned)lds, stream, ev_hist.start,
                              ev_hist.stop, 0, row_ptr, col_idx, B, rows_per_block, d0, hist);
    else
        hipLaunchKernelGGL(csc_hist_kernel, dim3(nb), dim3(CSC_NT), lds, stream, row_ptr, col_idx, B,
                           rows_per_block, d0, hist);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    const int n_groups = (d0 + COLG - 1) / COLG;
    int32_t *group_tot = cnt + d0 + 1;  // cnt holds csc_cnt_elems(d0) words
    e = launch_kernel(csc_colsum_kernel, dim3((unsigned)n_groups), dim3(COLG), stream, ev_colsum, hist, nb, d0,
                      cnt, group_tot);
    if (e != hipSuccess) return e;
    e = launch_kernel(col_scan_kernel, dim3((unsigned)n_groups), dim3(COLG), stream, ev_scan,
                      static_cast<const int32_t *>(cnt), static_cast<const int32_t *>(group_tot), d0, col_start,
                      chunk_start, chunk_desc);
    if (e != hipSuccess) return e;
    if (ev_place.start)
        hipExtLaunchKernelGGL(csc_place_kernel, dim3(nb), dim3(CSC_NT), (unsigned)lds, stream, ev_place.start,
                              ev_place.stop, 0, row_ptr, col_idx, vals, B, rows_per_block, d0,
                              static_cast<const int32_t *>(hist), static_cast<const int32_t *>(col_start),
                              csc_ent);
    else
        hipLaunchKernelGGL(csc_place_kernel, dim3(nb), dim3(CSC_NT), lds, stream, row_ptr, col_idx, vals, B,
                           rows_per_block, d0, static_cast<const int32_t *>(hist),
                           static_cast<const int32_t *>(col_start), csc_ent);
    return hipGetLastError();
}

hipError_t launch_sparse_dw(const SparseDwArgs &a, long long nnz, hipStream_t stream, const LaunchEvents &ev)
{
    // descriptors: one per distinct column of the batch + the extra parts of the very long ones
    const long long max_cols = (nnz < a.d0 ? nnz : a.d0) + nnz / SPLIT;
    if (nnz <= 0) return hipSuccess;
    SliceMap m;
    if (slice_map(a.d1, a.vec, &m)) {
        // what the batch can need at most -- a unit per long descriptor, ceil(light / (16 LP)) +
        // ceil(others / 16) for the rest -- but no more than DW_UNITS: the kernel walks over
        // its work with that stride, and workgroups that find none cost a dispatch each (7,600
        // of them behind the real-sim batch's 7,100: 1.8 us)
        const long long max_long = nnz / (CHUNK + 1) + nnz / SPLIT;
        long long units = max_long + (max_cols + 15) / 16 + 2;
        const char *cap_env = getenv("HB_DW_UNITS");  // tuning and test aid; read per call
        const long long cap = cap_env && atoi(cap_env) > 0 ? atoi(cap_env) : DW_UNITS;
        if (units > cap) units = cap;
        const long long blocks = sliced_blocks(m, units);
        if (blocks <= 0x7fffffffLL)
            return launch_kernel(sparse_dw_sliced_kernel, dim3((unsigned)blocks), dim3(XS_NT), stream, ev, a, m,
                                 (int)units);
    }
    return launch_kernel(sparse_dw_kernel, dim3((unsigned)(max_cols + FB_EXTRA)), dim3(SP_NT), stream, ev, a,
                         (int)max_cols);
}

hipError_t launch_colsum(const float *delta, int ldd, long long B, int d, int splits, float *partial,
                         hipStream_t stream, const LaunchEvents &ev)
{
    const int rows_per_split = (int)((B + splits - 1) / splits);
    return launch_kernel(colsum_kernel, dim3((unsigned)((d + 63) / 64), (unsigned)splits), dim3(256), stream,
                         ev, delta, ldd, B, d, rows_per_split, partial);
}

hipError_t launch_transpose(const float *in, float *out, int R, int C, hipStream_t stream)
{
    transpose_kernel<<<dim3((unsigned)((C + 31) / 32), (unsigned)((R + 31) / 32)), 256, 0, stream>>>(in, out, R, C);
    return hipGetLastError();
}

}  // namespace hb
