// Element-wise and reduction kernels of the mini-batch step: softmax / logistic loss with
// the output delta (Section 7.1 of the paper: softmax output, cross-entropy loss), the
// SGD update (Section 3, Eq. (3): W <- W - eta g) fused with the reduction of the
// split-K gradient partials, and the replica/global-model blend (Section 6.2).
// All of these are HBM-bound streaming kernels: coalesced 16-byte accesses, wavefront
// shuffles for the row reductions, no atomics.  The loss kernel leaves one partial sum per
// block; the kernel that runs next in the stream anyway (the update, or a one-block
// finalise kernel in loss-only / gradient-only calls) adds them up in index order.
#include "hb_internal.h"

namespace hb {
namespace {

constexpr int LOSS_NT = 256;

// round to nearest even through gfx950's v_cvt_pk_bf16_f32 (bit-identical to the integer
// formula for every non-NaN input; NaN stays NaN)
__device__ __forceinline__ unsigned short f32_to_bf16_rne(float f)
{
    return __builtin_bit_cast(unsigned short, (__bf16)f);
}

// G lanes cooperate on one row (G = power of two <= 64).  Softmax cross-entropy:
//   l_i = logsumexp(z_i) - z_i[c_i],  delta = (softmax(z_i) - onehot(c_i)) / B.
// Logistic with one output: l_i = log(1 + exp(-y z)), delta = -y sigma(-y z) / B.
// The mean loss is summed in a fixed order: per-thread, per-block tree, then the block
// partials in index order by loss_finalize() in a later kernel.
template <int G>
__global__ __launch_bounds__(LOSS_NT) void loss_kernel(LossArgs a)
{
    constexpr int ROWS_PER_BLOCK = LOSS_NT / G;
    const int tid = threadIdx.x;
    const int g = tid % G;
    const long long row = (long long)blockIdx.x * ROWS_PER_BLOCK + tid / G;
    const float invB = 1.0f / (float)a.B;
    float row_loss = 0.f;

    if (row < a.B) {
        const float *z = a.Z + row * a.ldz;
        const int yi = a.y[row];
        // bf16 delta with padded rows: the padding is part of the next product's contraction
        if (a.delta && a.delta_bf16 && a.zero_pad)
            for (int k = a.K + g; k < a.ldd; k += G) static_cast<unsigned short *>(a.delta)[row * a.ldd + k] = 0;
        if (a.loss == 1 && a.K == 1) {
            if (g == 0) {
                const float yf = (float)yi;
                const float m = yf * z[0];
                row_loss = fmaxf(-m, 0.f) + log1pf(__expf(-fabsf(m)));
                const float e = __expf(-fabsf(m));
                const float s = (m >= 0.f) ? e / (1.f + e) : 1.f / (1.f + e);  // sigma(-m)
                const float d = -yf * s * invB;
                if (a.delta) {
                    if (a.delta_bf16) static_cast<unsigned short *>(a.delta)[row * a.ldd] = f32_to_bf16_rne(d);
                    else static_cast<float *>(a.delta)[row * a.ldd] = d;
                }
            }
        } else if (G == 64 && a.vec4 && a.K <= 1024) {
            // wide rows (up to 1024 outputs) with 16-byte aligned rows: the row is read once,
            // four floats per lane and pass, and stays in registers for all three sweeps
            const int c = (a.loss == 1) ? (yi + 1) / 2 : yi;
            float4 v[4];
            float mx = -INFINITY, zc = 0.f;
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const int k0 = 4 * (g + 64 * i);
                v[i] = make_float4(-INFINITY, -INFINITY, -INFINITY, -INFINITY);
                if (k0 < a.K) {
                    const float4 t = *reinterpret_cast<const float4 *>(z + k0);  // k0 + 3 < ldz: rows are padded to 4
                    v[i].x = t.x;
                    if (k0 + 1 < a.K) v[i].y = t.y;
                    if (k0 + 2 < a.K) v[i].z = t.z;
                    if (k0 + 3 < a.K) v[i].w = t.w;
                }
            }
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const int k0 = 4 * (g + 64 * i);
                mx = fmaxf(mx, fmaxf(fmaxf(v[i].x, v[i].y), fmaxf(v[i].z, v[i].w)));
                if (c >= k0 && c < k0 + 4) zc = (c == k0) ? v[i].x : (c == k0 + 1) ? v[i].y : (c == k0 + 2) ? v[i].z : v[i].w;
            }
#pragma unroll
            for (int o = 32; o > 0; o >>= 1) {
                mx = fmaxf(mx, __shfl_xor(mx, o, 64));
                zc += __shfl_xor(zc, o, 64);
            }
            float se = 0.f;
#pragma unroll
            for (int i = 0; i < 4; ++i)  // exp(-inf) = 0 for the masked tail
                se += (__expf(v[i].x - mx) + __expf(v[i].y - mx)) + (__expf(v[i].z - mx) + __expf(v[i].w - mx));
#pragma unroll
            for (int o = 32; o > 0; o >>= 1) se += __shfl_xor(se, o, 64);
            const float lse = mx + __logf(se);
            if (g == 0) row_loss = lse - zc;
            if (a.delta) {
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    const int k0 = 4 * (g + 64 * i);
                    if (k0 >= a.K) continue;
                    float d[4] = {v[i].x, v[i].y, v[i].z, v[i].w};
#pragma unroll
                    for (int j = 0; j < 4; ++j) d[j] = (__expf(d[j] - lse) - (k0 + j == c ? 1.f : 0.f)) * invB;
                    if (k0 + 4 <= a.K) {
                        if (a.delta_bf16) {
                            uint2 pk;
                            pk.x = (unsigned)f32_to_bf16_rne(d[0]) | ((unsigned)f32_to_bf16_rne(d[1]) << 16);
                            pk.y = (unsigned)f32_to_bf16_rne(d[2]) | ((unsigned)f32_to_bf16_rne(d[3]) << 16);
                            *reinterpret_cast<uint2 *>(static_cast<unsigned short *>(a.delta) + row * a.ldd + k0) = pk;
                        } else {
                            *reinterpret_cast<float4 *>(static_cast<float *>(a.delta) + row * a.ldd + k0) =
                                make_float4(d[0], d[1], d[2], d[3]);
                        }
                    } else {
                        for (int j = 0; j < 4 && k0 + j < a.K; ++j) {
                            if (a.delta_bf16) static_cast<unsigned short *>(a.delta)[row * a.ldd + k0 + j] = f32_to_bf16_rne(d[j]);
                            else static_cast<float *>(a.delta)[row * a.ldd + k0 + j] = d[j];
                        }
                    }
                }
            }
        } else {
            const int c = (a.loss == 1) ? (yi + 1) / 2 : yi;
            float mx = -INFINITY, zc = 0.f;
            for (int k = g; k < a.K; k += G) {
                const float v = z[k];
                mx = fmaxf(mx, v);
                if (k == c) zc = v;
            }
#pragma unroll
            for (int o = G / 2; o > 0; o >>= 1) {
                mx = fmaxf(mx, __shfl_xor(mx, o, G));
                zc += __shfl_xor(zc, o, G);
            }
            float se = 0.f;
            for (int k = g; k < a.K; k += G) se += __expf(z[k] - mx);
#pragma unroll
            for (int o = G / 2; o > 0; o >>= 1) se += __shfl_xor(se, o, G);
            const float lse = mx + __logf(se);
            if (g == 0) row_loss = lse - zc;
            if (a.delta) {
                for (int k = g; k < a.K; k += G) {
                    const float d = (__expf(z[k] - lse) - (k == c ? 1.f : 0.f)) * invB;
                    if (a.delta_bf16) static_cast<unsigned short *>(a.delta)[row * a.ldd + k] = f32_to_bf16_rne(d);
                    else static_cast<float *>(a.delta)[row * a.ldd + k] = d;
                }
            }
        }
    }

    // block sum of row_loss in a fixed order; the block partials are added up by whoever
    // consumes the loss next on the stream (the update kernel or loss_finalize_kernel), so no
    // fence, ticket or atomic is needed here
    __shared__ float red[LOSS_NT];
    red[tid] = row_loss;
    __syncthreads();
#pragma unroll
    for (int s = LOSS_NT / 2; s > 0; s >>= 1) {
        if (tid < s) red[tid] += red[tid + s];
        __syncthreads();
    }
    if (tid == 0) a.block_partials[blockIdx.x] = red[0];
}

// mean loss = (sum of the block partials, in index order per thread then a fixed tree) / B
__device__ __forceinline__ void loss_finalize(const LossFinalize &f, double *dred /* 256 */)
{
    const int tid = threadIdx.x;
    double s = 0.0;
    for (int i = tid; i < f.n; i += 256) s += (double)f.partials[i];
    dred[tid] = s;
    __syncthreads();
#pragma unroll
    for (int st = 128; st > 0; st >>= 1) {
        if (tid < st) dred[tid] += dred[tid + st];
        __syncthreads();
    }
    if (tid == 0) {
        const float mean = (float)(dred[0] / (double)f.B);
        f.out[0] = mean;
        if (f.out2) f.out2[0] = mean;
    }
}

__global__ __launch_bounds__(256) void loss_finalize_kernel(LossFinalize f)
{
    __shared__ double dred[256];
    loss_finalize(f, dred);
}

int loss_group(int K)
{
    int g = 1;
    while (g < K && g < 64) g <<= 1;
    return g;
}

// ---------------------------------------------------------------- update
constexpr int UPD_NT = 256;

// Lanes per element that share the sum over the splits: enough that no lane adds more
// than 8 partials (a long serial chain of dependent-latency loads is what made this kernel
// slow), at most 64.
__host__ __device__ inline int split_lanes(int splits)
{
    int t = 1;
    while (t < 64 && t * 8 < splits) t <<= 1;
    return t;
}

__device__ __forceinline__ void vadd(float4 &g, const float4 &w) { g.x += w.x; g.y += w.y; g.z += w.z; g.w += w.w; }
__device__ __forceinline__ void vadd(float &g, const float &w) { g += w; }
__device__ __forceinline__ void vaxpy(float4 &p, float lr, const float4 &g)
{
    p.x -= lr * g.x; p.y -= lr * g.y; p.z -= lr * g.z; p.w -= lr * g.w;
}
__device__ __forceinline__ void vaxpy(float &p, float lr, const float &g) { p -= lr * g; }

// One segment, elements of type V (float4 when everything is 16-byte aligned, else float).
// T lanes per element: lane t adds splits t, t+T, ... (in that order), the T sums meet in
// LDS and are added in lane order.  Adjacent lanes hold adjacent elements of the same split.
template <typename V>
__device__ __forceinline__ void update_segment(const UpdateSeg &sg, long long nv, long long stride_v, float lr,
                                               int write_grad, V *sred)
{
    const V *__restrict__ part = reinterpret_cast<const V *>(sg.partial);
    const int T = split_lanes(sg.splits);
    const int EPB = UPD_NT / T;  // elements per block
    const int e_local = threadIdx.x % EPB, t = threadIdx.x / EPB;
    for (long long e0 = (long long)blockIdx.x * EPB; e0 < nv; e0 += (long long)gridDim.x * EPB) {
        const long long i = e0 + e_local;
        V g = V();
        if (i < nv) {
            V v[8];
#pragma unroll
            for (int u = 0; u < 8; ++u) {
                const int s = t + u * T;
                v[u] = V();
                if (s < sg.splits) v[u] = part[s * stride_v + i];
            }
#pragma unroll
            for (int u = 0; u < 8; ++u) vadd(g, v[u]);
            for (int s = t + 8 * T; s < sg.splits; s += T) vadd(g, part[s * stride_v + i]);  // splits > 512
        }
        if (T > 1) {
            sred[threadIdx.x] = g;
            __syncthreads();
            if (t == 0)
                for (int q = 1; q < T; ++q) vadd(g, sred[q * EPB + e_local]);
            __syncthreads();
        }
        if (t == 0 && i < nv) {
            if (write_grad) {
                reinterpret_cast<V *>(sg.grad_out)[i] = g;
            } else {
                V w = reinterpret_cast<V *>(sg.param)[i];
                vaxpy(w, lr, g);
                reinterpret_cast<V *>(sg.param)[i] = w;
            }
        }
    }
}

__global__ __launch_bounds__(UPD_NT) void update_kernel(UpdateArgs a)
{
    __shared__ double dred[256];
    __shared__ float4 sred[UPD_NT];
    if ((int)blockIdx.y == a.n_seg) {  // the extra row of the grid finishes the loss
        if (blockIdx.x == 0) loss_finalize(a.fin, dred);
        return;
    }
    const UpdateSeg &sg = a.seg[blockIdx.y];
    const long long n = sg.count;
    const bool vec_ok = ((n & 3) == 0) && ((sg.stride & 3) == 0) &&
                        ((reinterpret_cast<uintptr_t>(sg.partial) & 15) == 0) &&
                        ((reinterpret_cast<uintptr_t>(a.write_grad ? sg.grad_out : sg.param) & 15) == 0);
    if (vec_ok) update_segment<float4>(sg, n >> 2, sg.stride >> 2, a.lr, a.write_grad, sred);
    else update_segment<float>(sg, n, sg.stride, a.lr, a.write_grad, reinterpret_cast<float *>(sred));
}

__global__ __launch_bounds__(256) void merge_kernel(float *__restrict__ D, float *__restrict__ H,
                                                    long long n, float w)
{
    const long long step = (long long)gridDim.x * 256;
    for (long long i = (long long)blockIdx.x * 256 + threadIdx.x; i < n; i += step) {
        // the end points are exact copies, not (1-w) h + w d with rounding
        const float d = D[i], h = H[i];
        const float m = (w == 0.f) ? h : (w == 1.f) ? d : (1.f - w) * h + w * d;
        D[i] = m;
        H[i] = m;
    }
}

__global__ __launch_bounds__(256) void fill_u32_kernel(unsigned int *p, long long n, unsigned int v)
{
    const long long step = (long long)gridDim.x * 256;
    for (long long i = (long long)blockIdx.x * 256 + threadIdx.x; i < n; i += step) p[i] = v;
}

}  // namespace

int loss_grid_blocks(long long B, int K)
{
    const int rows_per_block = LOSS_NT / loss_group(K);
    return (int)((B + rows_per_block - 1) / rows_per_block);
}

hipError_t launch_loss(const LossArgs &args, hipStream_t stream, const LaunchEvents &ev)
{
    LossArgs a = args;
    a.vec4 = (a.ldz % 4 == 0) && ((reinterpret_cast<size_t>(a.Z) & 15) == 0) &&
             (a.delta == nullptr ||
              ((a.ldd % 4 == 0) && ((reinterpret_cast<size_t>(a.delta) & (a.delta_bf16 ? 7 : 15)) == 0)));
    const dim3 grid((unsigned)loss_grid_blocks(a.B, a.K)), block(LOSS_NT);
    switch (loss_group(a.K)) {
    case 1: return launch_kernel(loss_kernel<1>, grid, block, stream, ev, a);
    case 2: return launch_kernel(loss_kernel<2>, grid, block, stream, ev, a);
    case 4: return launch_kernel(loss_kernel<4>, grid, block, stream, ev, a);
    case 8: return launch_kernel(loss_kernel<8>, grid, block, stream, ev, a);
    case 16: return launch_kernel(loss_kernel<16>, grid, block, stream, ev, a);
    case 32: return launch_kernel(loss_kernel<32>, grid, block, stream, ev, a);
    default: return launch_kernel(loss_kernel<64>, grid, block, stream, ev, a);
    }
}

hipError_t launch_update(const UpdateArgs &a, hipStream_t stream, const LaunchEvents &ev)
{
    const int extra = a.fin.n > 0 ? 1 : 0;
    if (a.n_seg <= 0 && !extra) return hipSuccess;
    long long bx = 1;
    for (int i = 0; i < a.n_seg; ++i) {  // blocks the largest segment wants (float4 elements)
        const int epb = UPD_NT / split_lanes(a.seg[i].splits);
        const long long b = ((a.seg[i].count + 3) / 4 + epb - 1) / epb;
        if (b > bx) bx = b;
    }
    if (bx > 1024) bx = 1024;
    return launch_kernel(update_kernel, dim3((unsigned)bx, (unsigned)(a.n_seg + extra), 1), dim3(UPD_NT),
                         stream, ev, a);
}

hipError_t launch_loss_finalize(const LossFinalize &f, hipStream_t stream, const LaunchEvents &ev)
{
    return launch_kernel(loss_finalize_kernel, dim3(1), dim3(256), stream, ev, f);
}

hipError_t launch_merge(float *D, float *H, long long n, float w, hipStream_t stream)
{
    long long b = (n + 255) / 256;
    if (b > 4096) b = 4096;
    if (b < 1) b = 1;
    merge_kernel<<<(unsigned)b, 256, 0, stream>>>(D, H, n, w);
    return hipGetLastError();
}

// Debug aid: number of labels outside their domain (class index in [0, K) for softmax
// cross-entropy; +1 / -1 for the logistic loss), added to *bad.
__global__ __launch_bounds__(256) void label_check_kernel(const int32_t *__restrict__ y, long long B, int K,
                                                          int loss, unsigned int *bad)
{
    const long long step = (long long)gridDim.x * 256;
    unsigned int n = 0;
    for (long long i = (long long)blockIdx.x * 256 + threadIdx.x; i < B; i += step) {
        const int v = y[i];
        n += (loss == 1) ? (v != 1 && v != -1) : (v < 0 || v >= K);
    }
    if (n) atomicAdd(bad, n);
}

hipError_t launch_label_check(const int32_t *y, long long B, int K, int loss, unsigned int *bad, hipStream_t stream)
{
    long long b = (B + 255) / 256;
    if (b > 1024) b = 1024;
    if (b < 1) b = 1;
    label_check_kernel<<<(unsigned)b, 256, 0, stream>>>(y, B, K, loss, bad);
    return hipGetLastError();
}

// Counts what makes a CSR batch unusable: column indices outside [0, d0), a row pointer that
// does not start at 0, decreases, or does not end at nnz.
__global__ __launch_bounds__(256) void csr_check_kernel(const int32_t *__restrict__ row_ptr,
                                                        const int32_t *__restrict__ col_idx, long long nnz,
                                                        long long B, int d0, unsigned int *bad)
{
    const long long step = (long long)gridDim.x * 256;
    const long long t0 = (long long)blockIdx.x * 256 + threadIdx.x;
    unsigned int n = 0;
    for (long long i = t0; i < nnz; i += step) n += (unsigned int)col_idx[i] >= (unsigned int)d0;
    for (long long i = t0; i <= B; i += step) {
        const int v = row_ptr[i];
        n += (i == 0 && v != 0) || (i == B && v != nnz) || (i > 0 && v < row_ptr[i - 1]) || v < 0 || v > nnz;
    }
    if (n) atomicAdd(bad, n);
}

hipError_t launch_csr_check(const int32_t *row_ptr, const int32_t *col_idx, long long nnz, long long B, int d0,
                            unsigned int *bad, hipStream_t stream)
{
    long long b = ((nnz > B ? nnz : B + 1) + 255) / 256;
    if (b > 1024) b = 1024;
    if (b < 1) b = 1;
    csr_check_kernel<<<(unsigned)b, 256, 0, stream>>>(row_ptr, col_idx, nnz, B, d0, bad);
    return hipGetLastError();
}

hipError_t launch_fill_u32(unsigned int *p, long long n, unsigned int v, hipStream_t stream)
{
    long long b = (n + 255) / 256;
    if (b > 4096) b = 4096;
    if (b < 1) b = 1;
    fill_u32_kernel<<<(unsigned)b, 256, 0, stream>>>(p, n, v);
    return hipGetLastError();
}

}  // namespace hb
