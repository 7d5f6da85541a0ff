// Fused output layer for narrow outputs (d_L <= 16: the 7-class and 2-class workloads).
// One kernel does, for a block of R batch rows whose input activations A_{L-1} are read from
// HBM exactly once into LDS:
//   Z_L = A_{L-1} W_L^T + b_L                       (Section 3, Eq. (1), last layer)
//   loss and D_L = d(mean loss)/dZ_L                (Section 7.1: softmax + cross-entropy)
//   D_{L-1} = (D_L W_L) * f'(A_{L-1})               (Eq. (2), backward-data)
//   dW_L, db_L partial sums over the block's rows   (Eq. (2), weight gradient)
// With d_L = 7 these four products are HBM-bound (arithmetic intensity ~3.5 flop/B): as
// separate MFMA launches each of them re-read the same 8 MB of activations and paid a
// launch; fused, the traffic is one read of A_{L-1} and one write of D_{L-1}.
// LDS: R x (d + 4) floats of activations + W_L + D_L; R is chosen per batch so that the grid
// has about one block per CU (R = 16 at B = 4096).  512 threads per block.
#include "hb_internal.h"

#include <mutex>
#include <stdlib.h>

namespace hb {
namespace {

constexpr int OL_NT = 512;
constexpr int OL_KMAX = 16;  // widest output handled here

__device__ __forceinline__ float4 ld4(const float *p) { return *reinterpret_cast<const float4 *>(p); }

// K (the number of outputs) is a template parameter: every loop over the outputs unrolls
// without a branch, so the LDS reads and lane exchanges of all outputs are in flight together
// instead of one round trip per output.
template <int K>
__global__ __launch_bounds__(OL_NT) void out_layer_kernel(OutLayerArgs a)
{
    static_assert(K >= 1 && K <= OL_KMAX, "output width");
    extern __shared__ __attribute__((aligned(16))) float sm[];
    const int d = a.d, R = a.R;
    const int lda_s = d + 4;                    // LDS row stride of the activation tile
    float *sW = sm;                             // K x d
    float *sD = sW + (size_t)K * d;             // R x OL_KMAX : D_L
    float *sB = sD + (size_t)R * OL_KMAX;       // OL_KMAX     : b_L
    float *sRed = sB + OL_KMAX;                 // OL_NT / 64  : loss partials of the wavefronts
    float *sA = sRed + OL_NT / 64;              // R x lda_s
    const int tid = threadIdx.x;
    const long long r0 = (long long)blockIdx.x * R;
    const int d4 = d >> 2;

    // ---- P1: activations, weights, bias -> LDS (16-byte coalesced).  Everything the block
    // needs from memory is requested before the first wait: the label of the thread's row,
    // the first four activation vectors per thread, then weights and bias.
    const int TPR = OL_NT / R;                  // 8 .. 64, power of two
    const int row = tid / TPR, c = tid - row * TPR;
    const bool row_ok = (r0 + row < a.B);
    int yi = 0;
    if (c == 0 && row_ok) yi = a.y[r0 + row];
    float4 v[4];
    int off[4];
    auto load_a = [&](int base) {
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const int idx = base + u * OL_NT;
            v[u] = make_float4(0.f, 0.f, 0.f, 0.f);
            off[u] = -1;
            if (idx < R * d4) {
                const int ar = idx / d4, c4 = idx - ar * d4;
                off[u] = ar * lda_s + 4 * c4;
                if (r0 + ar < a.B) v[u] = ld4(a.A + (size_t)(r0 + ar) * a.lda + 4 * c4);
            }
        }
    };
    auto store_a = [&]() {
#pragma unroll
        for (int u = 0; u < 4; ++u)
            if (off[u] >= 0) *reinterpret_cast<float4 *>(&sA[off[u]]) = v[u];
    };
    load_a(tid);
    for (int idx = tid; idx < K * d4; idx += OL_NT)
        *reinterpret_cast<float4 *>(&sW[4 * idx]) = ld4(a.W + 4 * (size_t)idx);
    if (tid < K) sB[tid] = a.bias[tid];
    store_a();
    for (int base = tid + 4 * OL_NT; base < R * d4; base += 4 * OL_NT) {
        load_a(base);
        store_a();
    }
    __syncthreads();

    // ---- P2: logits.  TPR adjacent lanes share a row, each takes every TPR-th float4 of k
    float z[OL_KMAX];
#pragma unroll
    for (int j = 0; j < OL_KMAX; ++j) z[j] = 0.f;
    for (int c4 = c; c4 < d4; c4 += TPR) {
        const float4 x = *reinterpret_cast<const float4 *>(&sA[row * lda_s + 4 * c4]);
#pragma unroll
        for (int j = 0; j < OL_KMAX; ++j)
            if (j < K) {
                const float4 w = *reinterpret_cast<const float4 *>(&sW[j * d + 4 * c4]);
                z[j] += x.x * w.x + x.y * w.y + x.z * w.z + x.w * w.w;
            }
    }
    for (int o = TPR >> 1; o > 0; o >>= 1) {  // all K exchanges of a step are issued together
        float t[OL_KMAX];
#pragma unroll
        for (int j = 0; j < OL_KMAX; ++j)
            if (j < K) t[j] = __shfl_xor(z[j], o, 64);
#pragma unroll
        for (int j = 0; j < OL_KMAX; ++j)
            if (j < K) z[j] += t[j];
    }

    // ---- P3: loss and D_L for the row (one lane per row)
    float row_loss = 0.f;
    if (c == 0) {
        const float invB = 1.0f / (float)a.B;
        float dl[OL_KMAX];
#pragma unroll
        for (int j = 0; j < OL_KMAX; ++j) dl[j] = 0.f;
        if (row_ok) {
#pragma unroll
            for (int j = 0; j < OL_KMAX; ++j)
                if (j < K) z[j] += sB[j];
            if (a.loss == 1 && K == 1) {
                const float yf = (float)yi, mg = yf * z[0];
                const float e = __expf(-fabsf(mg));
                row_loss = fmaxf(-mg, 0.f) + log1pf(e);
                const float s = (mg >= 0.f) ? e / (1.f + e) : 1.f / (1.f + e);
                dl[0] = -yf * s * invB;
            } else {
                const int cls = (a.loss == 1) ? (yi + 1) / 2 : yi;
                float mx = -INFINITY, zc = 0.f;
#pragma unroll
                for (int j = 0; j < OL_KMAX; ++j)
                    if (j < K) {
                        mx = fmaxf(mx, z[j]);
                        if (j == cls) zc = z[j];
                    }
                float se = 0.f;
#pragma unroll
                for (int j = 0; j < OL_KMAX; ++j)
                    if (j < K) se += __expf(z[j] - mx);
                const float lse = mx + __logf(se);
                row_loss = lse - zc;
#pragma unroll
                for (int j = 0; j < OL_KMAX; ++j)
                    if (j < K) dl[j] = (__expf(z[j] - lse) - (j == cls ? 1.f : 0.f)) * invB;
            }
            if (a.Z) {
#pragma unroll
                for (int j = 0; j < K; ++j) a.Z[(size_t)(r0 + row) * a.ldz + j] = z[j];
            }
            if (a.DL) {
#pragma unroll
                for (int j = 0; j < K; ++j) a.DL[(size_t)(r0 + row) * a.ldz + j] = dl[j];
            }
        }
#pragma unroll
        for (int j = 0; j < OL_KMAX; ++j) sD[row * OL_KMAX + j] = dl[j];  // zero rows past B
    }

    // loss: wavefront sums -> block sum; the block partials are added up by the next consumer
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) row_loss += __shfl_xor(row_loss, o, 64);
    if ((tid & 63) == 0) sRed[tid >> 6] = row_loss;
    __syncthreads();  // also publishes sD
    if (tid == 0) {
        float s = 0.f;
        for (int w = 0; w < OL_NT / 64; ++w) s += sRed[w];
        a.block_partials[blockIdx.x] = s;
    }
    if (!a.backward) return;

    // P4 and P5 only read LDS and are independent.  When the weight-gradient partial needs no
    // more than a quarter of the block (d <= 512), its wavefronts run it while the others do
    // the backward-data part: side by side instead of one after the other.
    const int w_wave_threads = ((d4 + 63) / 64) * 64;            // whole wavefronts that cover d4
    const bool split = a.Dprev != nullptr && w_wave_threads * 4 <= OL_NT;
    const int p4_first = split ? w_wave_threads : 0;             // first thread of the P4 group
    const int p4_threads = OL_NT - p4_first;

    // ---- P4: D_{L-1}[i][k] = (sum_j D_L[i][j] W[j][k]) * f'(A[i][k]), 16-byte stores along k
    if (a.Dprev && tid >= p4_first) {
        for (int idx = tid - p4_first; idx < R * d4; idx += p4_threads) {
            const int i = idx / d4, c4 = idx - i * d4;
            if (r0 + i >= a.B) continue;
            float4 s = {0.f, 0.f, 0.f, 0.f};
            alignas(16) float dl[OL_KMAX];
#pragma unroll
            for (int q = 0; q < (K + 3) / 4; ++q)
                *reinterpret_cast<float4 *>(&dl[4 * q]) = *reinterpret_cast<const float4 *>(&sD[i * OL_KMAX + 4 * q]);
#pragma unroll
            for (int j = 0; j < OL_KMAX; ++j)
                if (j < K) {
                    const float dj = dl[j];
                    const float4 w = *reinterpret_cast<const float4 *>(&sW[j * d + 4 * c4]);
                    s.x += dj * w.x; s.y += dj * w.y; s.z += dj * w.z; s.w += dj * w.w;
                }
            const float4 o = *reinterpret_cast<const float4 *>(&sA[i * lda_s + 4 * c4]);
            if (a.act == ACT_SIGMOID) {
                s.x *= o.x * (1.f - o.x); s.y *= o.y * (1.f - o.y);
                s.z *= o.z * (1.f - o.z); s.w *= o.w * (1.f - o.w);
            } else if (a.act == ACT_RELU) {
                s.x = o.x > 0.f ? s.x : 0.f; s.y = o.y > 0.f ? s.y : 0.f;
                s.z = o.z > 0.f ? s.z : 0.f; s.w = o.w > 0.f ? s.w : 0.f;
            }
            *reinterpret_cast<float4 *>(a.Dprev + (size_t)(r0 + i) * a.ldp + 4 * c4) = s;
        }
    }

    // ---- P5: dW_L partial of this block, dW[j][k] = sum_i D_L[i][j] A[i][k]: one thread per
    // float4 of k, all R rows (R is small: the grid is sized to one block per CU)
    float *out = a.dW_partial + (size_t)blockIdx.x * K * d;
    if (split && tid >= p4_first) return;   // the backward-data wavefronts are done
    for (int c4 = tid; c4 < d4; c4 += OL_NT) {
        float4 g[OL_KMAX];
#pragma unroll
        for (int j = 0; j < OL_KMAX; ++j) g[j] = make_float4(0.f, 0.f, 0.f, 0.f);
#pragma unroll 4
        for (int i = 0; i < R; ++i) {  // R is a multiple of 8
            const float4 x = *reinterpret_cast<const float4 *>(&sA[i * lda_s + 4 * c4]);
            alignas(16) float dl[OL_KMAX];
#pragma unroll
            for (int q = 0; q < (K + 3) / 4; ++q)
                *reinterpret_cast<float4 *>(&dl[4 * q]) = *reinterpret_cast<const float4 *>(&sD[i * OL_KMAX + 4 * q]);
#pragma unroll
            for (int j = 0; j < OL_KMAX; ++j)
                if (j < K) {
                    const float dj = dl[j];
                    g[j].x += dj * x.x; g[j].y += dj * x.y; g[j].z += dj * x.z; g[j].w += dj * x.w;
                }
        }
#pragma unroll
        for (int j = 0; j < OL_KMAX; ++j)
            if (j < K) *reinterpret_cast<float4 *>(out + (size_t)j * d + 4 * c4) = g[j];
    }
    if (tid < K) {  // db_L partial
        float s = 0.f;
        for (int i = 0; i < R; ++i) s += sD[i * OL_KMAX + tid];
        a.db_partial[(size_t)blockIdx.x * K + tid] = s;
    }
}

size_t lds_bytes(int R, int d, int K)
{
    const size_t tile = (size_t)R * (d + 4);  // activation tile
    return sizeof(float) * (tile + (size_t)K * d + (size_t)R * OL_KMAX + OL_KMAX + OL_NT / 64);
}

}  // namespace

int out_layer_min_rows() { return 8; }

int out_layer_rows(int d, int K)
{
    if (K < 1 || K > OL_KMAX || d < 4 || (d & 3) != 0) return 0;
    for (int R = 64; R >= 8; R >>= 1)
        if (lds_bytes(R, d, K) <= 150 * 1024) return R;
    return 0;
}

// Rows per block for a batch of B rows: as many blocks as the device has CUs when B allows,
// at least out_layer_min_rows() rows, at most what fits LDS.
int out_layer_rows_for_batch(int d, int K, long long B)
{
    const int rmax = out_layer_rows(d, K);
    if (rmax == 0) return 0;
    int R = out_layer_min_rows();
    while (R < rmax && (long long)R * 2 * 256 <= B) R <<= 1;
    static const int forced = getenv("HB_OL_ROWS") ? atoi(getenv("HB_OL_ROWS")) : 0;  // tuning aid: 8, 16, 32, 64
    if (forced >= out_layer_min_rows() && forced <= rmax && (forced & (forced - 1)) == 0) R = forced;
    return R;
}

hipError_t launch_out_layer(OutLayerArgs a, hipStream_t stream, const LaunchEvents &ev)
{
    a.R = out_layer_rows_for_batch(a.d, a.K, a.B);
    if (a.R == 0) return hipErrorInvalidValue;
    const size_t lds = lds_bytes(a.R, a.d, a.K);
    const dim3 grid((unsigned)((a.B + a.R - 1) / a.R)), block(OL_NT);
    static std::mutex granted_mu;  // handles on different host threads launch concurrently
    static size_t granted[OL_KMAX + 1] = {};
    hipError_t e = hipErrorInvalidValue;
    switch (a.K) {
#define HB_OL_CASE(KK)                                                                                   \
    case KK:                                                                                             \
        e = hipSuccess;                                                                                  \
        {                                                                                                \
            std::lock_guard<std::mutex> lk(granted_mu);                                                  \
            if (lds > granted[KK]) {                                                                     \
                e = hipFuncSetAttribute(reinterpret_cast<const void *>(out_layer_kernel<KK>),            \
                                        hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);           \
                if (e == hipSuccess) granted[KK] = lds;                                                  \
            }                                                                                            \
        }                                                                                                \
        if (e != hipSuccess) return e;                                                                   \
        if (ev.start)                                                                                    \
            hipExtLaunchKernelGGL(out_layer_kernel<KK>, grid, block, (unsigned)lds, stream, ev.start,    \
                                  ev.stop, 0, a);                                                        \
        else                                                                                             \
            hipLaunchKernelGGL(out_layer_kernel<KK>, grid, block, lds, stream, a);                       \
        break;
        HB_OL_CASE(1) HB_OL_CASE(2) HB_OL_CASE(3) HB_OL_CASE(4) HB_OL_CASE(5) HB_OL_CASE(6) HB_OL_CASE(7)
        HB_OL_CASE(8) HB_OL_CASE(9) HB_OL_CASE(10) HB_OL_CASE(11) HB_OL_CASE(12) HB_OL_CASE(13)
        HB_OL_CASE(14) HB_OL_CASE(15) HB_OL_CASE(16)
#undef HB_OL_CASE
    default:
        return hipErrorInvalidValue;
    }
    return hipGetLastError();
}

}  // namespace hb
