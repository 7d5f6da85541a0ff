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

// ---- per-batch CSC: count, scan, fill
__global__ __launch_bounds__(256) void col_count_kernel(const int32_t *__restrict__ col_idx,
                                                        long long nnz, int32_t *__restrict__ cnt)
{
    const long long step = (long long)gridDim.x * 256;
    for (long long p = (long long)blockIdx.x * 256 + threadIdx.x; p < nnz; p += step)
        atomicAdd(&cnt[col_idx[p]], 1);
}

// One workgroup: exclusive scans of cnt[0..n) (-> col_start) and of the chunk counts
// ceil(cnt / CHUNK) (-> chunk_start); both get their totals at index n.  Also clears
// cursor[] for the fill pass.
__global__ __launch_bounds__(1024) void col_scan_kernel(const int32_t *__restrict__ cnt, int n,
                                                        int32_t *__restrict__ col_start,
                                                        int32_t *__restrict__ chunk_start,
                                                        int32_t *__restrict__ cursor)
{
    __shared__ int s_a[1024], s_b[1024];
    const int tid = threadIdx.x;
    const int per = (n + 1023) / 1024;
    const int lo = min(n, tid * per), hi = min(n, lo + per);
    int sa = 0, sb = 0;
    for (int c = lo; c < hi; ++c) {
        sa += cnt[c];
        sb += (cnt[c] + CHUNK - 1) / CHUNK;
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
        col_start[c] = ra;
        chunk_start[c] = rb;
        cursor[c] = 0;
        ra += cnt[c];
        rb += (cnt[c] + CHUNK - 1) / CHUNK;
    }
    if (tid == 1023) {
        col_start[n] = s_a[1023];
        chunk_start[n] = s_b[1023];
    }
}

__global__ __launch_bounds__(256) void csc_fill_kernel(const int32_t *__restrict__ row_ptr,
                                                       const int32_t *__restrict__ col_idx,
                                                       const float *__restrict__ vals, long long B,
                                                       const int32_t *__restrict__ col_start,
                                                       int32_t *__restrict__ cursor,
                                                       int32_t *__restrict__ csc_row,
                                                       float *__restrict__ csc_val)
{
    // one wavefront per row, lanes over the row's non-zeros
    const long long row = ((long long)blockIdx.x * 256 + threadIdx.x) >> 6;
    const int lane = threadIdx.x & 63;
    if (row >= B) return;
    const int beg = row_ptr[row], end = row_ptr[row + 1];
    for (int p = beg + lane; p < end; p += 64) {
        const int c = col_idx[p];
        const int pos = col_start[c] + atomicAdd(&cursor[c], 1);
        csc_row[pos] = (int32_t)row;
        csc_val[pos] = vals[p];
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

hipError_t launch_csc_build(const int32_t *row_ptr, const int32_t *col_idx, const float *vals,
                            long long nnz, long long B, int d0, int32_t *cnt, int32_t *col_start,
                            int32_t *chunk_start, int32_t *cursor, int32_t *csc_row, float *csc_val,
                            hipStream_t stream, const LaunchEvents &ev_count,
                            const LaunchEvents &ev_scan, const LaunchEvents &ev_fill)
{
    hipError_t e = launch_fill_u32(reinterpret_cast<unsigned int *>(cnt), d0 + 1, 0u, stream);
    if (e != hipSuccess) return e;
    if (nnz > 0) {
        long long b = (nnz + 255) / 256;
        if (b > 2048) b = 2048;
        e = launch_kernel(col_count_kernel, dim3((unsigned)b), dim3(256), stream, ev_count, col_idx, nnz, cnt);
        if (e != hipSuccess) return e;
    }
    e = launch_kernel(col_scan_kernel, dim3(1), dim3(1024), stream, ev_scan,
                      static_cast<const int32_t *>(cnt), d0, col_start, chunk_start, cursor);
    if (e != hipSuccess) return e;
    if (nnz > 0) {
        const long long blocks = (B * 64 + 255) / 256;
        e = launch_kernel(csc_fill_kernel, dim3((unsigned)blocks), dim3(256), stream, ev_fill, row_ptr,
                          col_idx, vals, B, static_cast<const int32_t *>(col_start), cursor, csc_row, csc_val);
    }
    return e;
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
