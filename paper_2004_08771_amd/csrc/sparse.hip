// CSR first layer (the real-sim-shaped workload: ~50 non-zeros in 20,958 columns per row).
// The paper processes its datasets densely and leaves sparse input to future work
// (Section 8); the forward pass (Section 3, Eq. (1)), the gradient (Eq. (2)) and the update
// (Eq. (3)) of layer 1 are the same sums, run over the stored non-zeros only.
//
// gfx950 design: layer-1 weights are kept TRANSPOSED on the device (W1t: d_0 x d_1), so
// that the weights of one input column are one contiguous row: the forward SpMM gathers
// whole rows with 16-byte coalesced loads, and the gradient/update touches only the rows
// of columns that occur in the batch.  The gradient is column-segmented: the batch's
// non-zeros are bucketed by column (a per-batch CSC built on the device), long columns
// are cut into chunks, and every chunk sums its rows of delta_1 once; a column that fits
// one chunk is updated with a plain read-modify-write, longer ones with fp32 atomic adds
// of their chunk sums.  Everything is HBM/L2-bandwidth work; no MFMA.
#include "hb_internal.h"

namespace hb {
namespace {

constexpr int SP_NT = 128;    // threads per row / per chunk: one float4 each for d_1 = 512
constexpr int CHUNK = 128;    // non-zeros per gradient chunk

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
    if (a.vec) {
        const int n4 = a.d1 >> 2;
        for (int q = threadIdx.x; q < n4; q += SP_NT) {
            float4 acc = reinterpret_cast<const float4 *>(a.bias)[q];
            for (int p = beg; p < end; ++p) {
                const int c = a.col_idx[p];
                const float v = a.vals[p];
                const float4 w = reinterpret_cast<const float4 *>(a.W1t + (size_t)c * a.ldw)[q];
                acc.x += v * w.x; acc.y += v * w.y; acc.z += v * w.z; acc.w += v * w.w;
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
//   3. col_scan_kernel   exclusive scan of cnt over columns -> col_start, chunk_start
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
        for (int p = beg + threadIdx.x; p < end; p += CSC_NT) atomicAdd(&s_hist[col_idx[p]], 1);
    }
    __syncthreads();
    int32_t *out = hist + (size_t)blockIdx.x * d0;
    for (int c = threadIdx.x; c < d0; c += CSC_NT) out[c] = s_hist[c];
}

__global__ __launch_bounds__(256) void csc_colsum_kernel(int32_t *__restrict__ hist, int n_blocks, int d0,
                                                         int32_t *__restrict__ cnt)
{
    const int c = blockIdx.x * 256 + threadIdx.x;
    if (c >= d0) return;
    int run = 0;
    for (int b = 0; b < n_blocks; ++b) {
        const int h = hist[(size_t)b * d0 + c];
        hist[(size_t)b * d0 + c] = run;
        run += h;
    }
    cnt[c] = run;
}

// One workgroup: exclusive scans of cnt[0..n) (-> col_start) and of the chunk counts
// ceil(cnt / CHUNK) (-> chunk_start); both get their totals at index n.
__global__ __launch_bounds__(1024) void col_scan_kernel(const int32_t *__restrict__ cnt, int n,
                                                        int32_t *__restrict__ col_start,
                                                        int32_t *__restrict__ chunk_start)
{
    extern __shared__ int32_t s_cnt[];  // n entries
    __shared__ int s_a[1024], s_b[1024];
    const int tid = threadIdx.x;
    for (int c = tid; c < n; c += 1024) s_cnt[c] = cnt[c];
    __syncthreads();
    const int per = (n + 1023) / 1024;
    const int lo = min(n, tid * per), hi = min(n, lo + per);
    int sa = 0, sb = 0;
    for (int c = lo; c < hi; ++c) {
        sa += s_cnt[c];
        sb += (s_cnt[c] + CHUNK - 1) / CHUNK;
    }
    s_a[tid] = sa;
    s_b[tid] = sb;
    __syncthreads();
    for (int off = 1; off < 1024; off <<= 1) {  // Hillis-Steele inclusive scan
        int va = 0, vb = 0;
        if (tid >= off) { va = s_a[tid - off]; vb = s_b[tid - off]; }
        __syncthreads();
        s_a[tid] += va;
        s_b[tid] += vb;
        __syncthreads();
    }
    int ra = s_a[tid] - sa, rb = s_b[tid] - sb;  // exclusive prefix of this thread's range
    for (int c = lo; c < hi; ++c) {
        const int v = s_cnt[c];
        col_start[c] = ra;
        chunk_start[c] = rb;
        ra += v;
        rb += (v + CHUNK - 1) / CHUNK;
    }
    if (tid == 1023) {
        col_start[n] = s_a[1023];
        chunk_start[n] = s_b[1023];
    }
}

__global__ __launch_bounds__(CSC_NT) void csc_place_kernel(const int32_t *__restrict__ row_ptr,
                                                           const int32_t *__restrict__ col_idx,
                                                           const float *__restrict__ vals, long long B,
                                                           int rows_per_block, int d0,
                                                           const int32_t *__restrict__ hist,
                                                           const int32_t *__restrict__ col_start,
                                                           int32_t *__restrict__ csc_row,
                                                           float *__restrict__ csc_val)
{
    extern __shared__ int32_t s_cur[];
    const int32_t *mine = hist + (size_t)blockIdx.x * d0;
    for (int c = threadIdx.x; c < d0; c += CSC_NT) s_cur[c] = col_start[c] + mine[c];
    __syncthreads();
    const long long r0 = (long long)blockIdx.x * rows_per_block;
    const long long r1 = min(B, r0 + rows_per_block);
    // one wavefront per row, lanes over the row's non-zeros
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    for (long long row = r0 + wave; row < r1; row += CSC_NT / 64) {
        const int beg = row_ptr[row], end = row_ptr[row + 1];
        for (int p = beg + lane; p < end; p += 64) {
            const int pos = atomicAdd(&s_cur[col_idx[p]], 1);
            csc_row[pos] = (int32_t)row;
            csc_val[pos] = vals[p];
        }
    }
}

// One workgroup per chunk of one column's entries:
//   g[:] = sum_e csc_val[e] * delta_1[csc_row[e], :]
// then W1t[c,:] -= lr * g (plain for a single-chunk column, atomic otherwise), or in
// gradient mode dW_1[:, c] (+)= g in the flat out x in layout.
__global__ __launch_bounds__(SP_NT) void sparse_dw_kernel(SparseDwArgs a)
{
    const int total_chunks = a.chunk_start[a.d0];
    const int chunk = blockIdx.x;
    if (chunk >= total_chunks) return;
    // largest c with chunk_start[c] <= chunk (columns without entries have equal starts)
    int lo = 0, hi = a.d0;
    while (hi - lo > 1) {
        const int mid = (lo + hi) >> 1;
        if (a.chunk_start[mid] <= chunk) lo = mid; else hi = mid;
    }
    const int c = lo;
    const int n_chunks = a.chunk_start[c + 1] - a.chunk_start[c];
    const int seg_beg = a.col_start[c], seg_end = a.col_start[c + 1];
    const int e_beg = seg_beg + (chunk - a.chunk_start[c]) * CHUNK;
    const int e_end = min(seg_end, e_beg + CHUNK);
    const bool single = (n_chunks == 1);

    if (a.vec) {
        const int n4 = a.d1 >> 2;
        for (int q = threadIdx.x; q < n4; q += SP_NT) {
            float4 g = {0.f, 0.f, 0.f, 0.f};
            for (int e = e_beg; e < e_end; ++e) {
                const float v = a.csc_val[e];
                const float4 d = reinterpret_cast<const float4 *>(a.delta + (size_t)a.csc_row[e] * a.ldd)[q];
                g.x += v * d.x; g.y += v * d.y; g.z += v * d.z; g.w += v * d.w;
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
                g += a.csc_val[e] * a.delta[(size_t)a.csc_row[e] * a.ldd + j];
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
    if (col < d)
        for (long long i = r0 + rg; i < r1; i += 4) s += delta[i * ldd + col];
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

hipError_t launch_spmm_fwd(const SpmmArgs &a, long long B, hipStream_t stream, const LaunchEvents &ev)
{
    return launch_kernel(spmm_fwd_kernel, dim3((unsigned)B), dim3(SP_NT), stream, ev, a);
}

int sparse_chunk() { return CHUNK; }

int csc_blocks(long long B)
{
    long long nb = (B + 127) / 128;  // at least 128 rows per block
    if (nb > 64) nb = 64;
    if (nb < 1) nb = 1;
    return (int)nb;
}

size_t csc_hist_elems(long long max_B, int d0) { return (size_t)csc_blocks(max_B) * (size_t)d0; }

bool csc_supported(int d0) { return (size_t)d0 * sizeof(int32_t) <= 150 * 1024; }

hipError_t launch_csc_build(const int32_t *row_ptr, const int32_t *col_idx, const float *vals,
                            long long nnz, long long B, int d0, int32_t *hist, int32_t *cnt,
                            int32_t *col_start, int32_t *chunk_start, int32_t *csc_row, float *csc_val,
                            hipStream_t stream, const LaunchEvents &ev_hist,
                            const LaunchEvents &ev_scan, const LaunchEvents &ev_place)
{
    (void)nnz;
    const int nb = csc_blocks(B);
    const int rows_per_block = (int)((B + nb - 1) / nb);
    const size_t lds = (size_t)d0 * sizeof(int32_t);
    // more than 64 KB of dynamic LDS has to be requested per kernel
    static size_t lds_granted = 0;
    if (lds > 32 * 1024 && lds > lds_granted) {
        hipError_t ea = hipFuncSetAttribute(reinterpret_cast<const void *>(csc_hist_kernel),
                                            hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        if (ea == hipSuccess)
            ea = hipFuncSetAttribute(reinterpret_cast<const void *>(col_scan_kernel),
                                     hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        if (ea == hipSuccess)
            ea = hipFuncSetAttribute(reinterpret_cast<const void *>(csc_place_kernel),
                                     hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        if (ea != hipSuccess) return ea;
        lds_granted = lds;
    }
    if (ev_hist.start)
        hipExtLaunchKernelGGL(csc_hist_kernel, dim3(nb), dim3(CSC_NT), (unsigned)lds, stream, ev_hist.start,
                              ev_hist.stop, 0, row_ptr, col_idx, B, rows_per_block, d0, hist);
    else
        hipLaunchKernelGGL(csc_hist_kernel, dim3(nb), dim3(CSC_NT), lds, stream, row_ptr, col_idx, B,
                           rows_per_block, d0, hist);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    e = launch_kernel(csc_colsum_kernel, dim3((unsigned)((d0 + 255) / 256)), dim3(256), stream, LaunchEvents(),
                      hist, nb, d0, cnt);
    if (e != hipSuccess) return e;
    if (ev_scan.start)
        hipExtLaunchKernelGGL(col_scan_kernel, dim3(1), dim3(1024), (unsigned)lds, stream, ev_scan.start,
                              ev_scan.stop, 0, static_cast<const int32_t *>(cnt), d0, col_start, chunk_start);
    else
        hipLaunchKernelGGL(col_scan_kernel, dim3(1), dim3(1024), lds, stream,
                           static_cast<const int32_t *>(cnt), d0, col_start, chunk_start);
    e = hipGetLastError();
    if (e != hipSuccess) return e;
    if (ev_place.start)
        hipExtLaunchKernelGGL(csc_place_kernel, dim3(nb), dim3(CSC_NT), (unsigned)lds, stream, ev_place.start,
                              ev_place.stop, 0, row_ptr, col_idx, vals, B, rows_per_block, d0,
                              static_cast<const int32_t *>(hist), static_cast<const int32_t *>(col_start),
                              csc_row, csc_val);
    else
        hipLaunchKernelGGL(csc_place_kernel, dim3(nb), dim3(CSC_NT), lds, stream, row_ptr, col_idx, vals, B,
                           rows_per_block, d0, static_cast<const int32_t *>(hist),
                           static_cast<const int32_t *>(col_start), csc_row, csc_val);
    return hipGetLastError();
}

hipError_t launch_sparse_dw(const SparseDwArgs &a, long long max_chunks, hipStream_t stream,
                            const LaunchEvents &ev)
{
    if (max_chunks <= 0) return hipSuccess;
    return launch_kernel(sparse_dw_kernel, dim3((unsigned)max_chunks), dim3(SP_NT), stream, ev, a);
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
