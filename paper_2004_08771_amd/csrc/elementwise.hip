// Element-wise and reduction kernels of the mini-batch step: softmax / logistic loss with
// the output delta (Section 7.1 of the paper: softmax output, cross-entropy loss), the
// SGD update (Section 3, Eq. (3): W <- W - eta g) fused with the reduction of the
// split-K gradient partials, and the replica/global-model blend (Section 6.2).
// All of these are HBM-bound streaming kernels: coalesced 16-byte accesses, wavefront
// shuffles for the row reductions, no atomics on data (one atomic ticket per block for the
// deterministic final loss sum).
#include "hb_internal.h"

namespace hb {
namespace {

constexpr int LOSS_NT = 256;

__device__ __forceinline__ unsigned short f32_to_bf16_rne(float f)
{
    unsigned int u = __float_as_uint(f);
    if ((u & 0x7f800000u) == 0x7f800000u) return (unsigned short)(u >> 16);  // inf / nan
    const unsigned int lsb = (u >> 16) & 1u;
    u += 0x7fffu + lsb;
    return (unsigned short)(u >> 16);
}

// G lanes cooperate on one row (G = power of two <= 64).  Softmax cross-entropy:
//   l_i = logsumexp(z_i) - z_i[c_i],  delta = (softmax(z_i) - onehot(c_i)) / B.
// Logistic with one output: l_i = log(1 + exp(-y z)), delta = -y sigma(-y z) / B.
// The mean loss is summed in a fixed order: per-thread, per-block tree, then the last
// block to finish adds the block partials in index order.
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

    // block sum of row_loss (fixed order)
    __shared__ float red[LOSS_NT];
    __shared__ bool is_last;
    red[tid] = row_loss;
    __syncthreads();
#pragma unroll
    for (int s = LOSS_NT / 2; s > 0; s >>= 1) {
        if (tid < s) red[tid] += red[tid + s];
        __syncthreads();
    }
    if (tid == 0) {
        a.block_partials[blockIdx.x] = red[0];
        __threadfence();
        const unsigned int ticket = atomicAdd(a.counter, 1u);
        is_last = (ticket == gridDim.x - 1);
    }
    __syncthreads();
    if (is_last) {
        __threadfence();
        double s = 0.0;
        for (unsigned int i = tid; i < gridDim.x; i += LOSS_NT)
            s += (double)__hip_atomic_load(&a.block_partials[i], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        __shared__ double dred[LOSS_NT];
        dred[tid] = s;
        __syncthreads();
#pragma unroll
        for (int st = LOSS_NT / 2; st > 0; st >>= 1) {
            if (tid < st) dred[tid] += dred[tid + st];
            __syncthreads();
        }
        if (tid == 0) {
            const float mean = (float)(dred[0] / (double)a.B);
            a.loss_out[0] = mean;
            if (a.loss_out2) a.loss_out2[0] = mean;
            *a.counter = 0u;  // ready for the next launch on this stream
        }
    }
}

int loss_group(int K)
{
    int g = 1;
    while (g < K && g < 64) g <<= 1;
    return g;
}

// ---------------------------------------------------------------- update
constexpr int UPD_NT = 256;

__global__ __launch_bounds__(UPD_NT) void update_kernel(UpdateArgs a)
{
    const UpdateSeg &sg = a.seg[blockIdx.y];
    const long long n = sg.count;
    const long long stride = sg.stride;
    const float *__restrict__ part = sg.partial;
    const bool vec_ok = ((n & 3) == 0) && ((stride & 3) == 0) &&
                        ((reinterpret_cast<uintptr_t>(part) & 15) == 0) &&
                        ((reinterpret_cast<uintptr_t>(a.write_grad ? sg.grad_out : sg.param) & 15) == 0);
    const long long step = (long long)gridDim.x * UPD_NT;
    if (vec_ok) {
        const long long n4 = n >> 2;
        for (long long i = (long long)blockIdx.x * UPD_NT + threadIdx.x; i < n4; i += step) {
            float4 g = reinterpret_cast<const float4 *>(part)[i];
            for (int s = 1; s < sg.splits; ++s) {
                const float4 t = reinterpret_cast<const float4 *>(part + s * stride)[i];
                g.x += t.x; g.y += t.y; g.z += t.z; g.w += t.w;
            }
            if (a.write_grad) {
                reinterpret_cast<float4 *>(sg.grad_out)[i] = g;
            } else {
                float4 w = reinterpret_cast<float4 *>(sg.param)[i];
                w.x -= a.lr * g.x; w.y -= a.lr * g.y; w.z -= a.lr * g.z; w.w -= a.lr * g.w;
                reinterpret_cast<float4 *>(sg.param)[i] = w;
                if (sg.shadow) {
                    ushort4 b;
                    b.x = f32_to_bf16_rne(w.x); b.y = f32_to_bf16_rne(w.y);
                    b.z = f32_to_bf16_rne(w.z); b.w = f32_to_bf16_rne(w.w);
                    reinterpret_cast<ushort4 *>(sg.shadow)[i] = b;
                }
            }
        }
    } else {
        for (long long i = (long long)blockIdx.x * UPD_NT + threadIdx.x; i < n; i += step) {
            float g = part[i];
            for (int s = 1; s < sg.splits; ++s) g += part[s * stride + i];
            if (a.write_grad) {
                sg.grad_out[i] = g;
            } else {
                const float w = sg.param[i] - a.lr * g;
                sg.param[i] = w;
                if (sg.shadow) static_cast<unsigned short *>(sg.shadow)[i] = f32_to_bf16_rne(w);
            }
        }
    }
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

hipError_t launch_loss(const LossArgs &a, hipStream_t stream, const LaunchEvents &ev)
{
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
    if (a.n_seg <= 0) return hipSuccess;
    long long mx = 0;
    for (int i = 0; i < a.n_seg; ++i) mx = a.seg[i].count > mx ? a.seg[i].count : mx;
    long long bx = (mx / 4 + UPD_NT - 1) / UPD_NT;
    if (bx < 1) bx = 1;
    if (bx > 2048) bx = 2048;
    return launch_kernel(update_kernel, dim3((unsigned)bx, (unsigned)a.n_seg, 1), dim3(UPD_NT), stream,
                         ev, a);
}

hipError_t launch_merge(float *D, float *H, long long n, float w, hipStream_t stream)
{
    long long b = (n + 255) / 256;
    if (b > 4096) b = 4096;
    if (b < 1) b = 1;
    merge_kernel<<<(unsigned)b, 256, 0, stream>>>(D, H, n, w);
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
