// bf16 MFMA GEMM for the mixed-precision mode (bf16 weights / activations, fp32 master
// weights and accumulation) of the mini-batch step: the same three layer products as the
// fp32 path (Section 3 of the paper, Eq. (1) forward and Eq. (2) backward).
//
// gfx950 design: ONE kernel shape -- both operands K-major ("NT"), the layout
// v_mfma_f32_32x32x16_bf16 wants (8 consecutive k per lane) -- and no transposing loads in
// the hot loop.  The other two products are brought to that shape by keeping every bf16
// tensor that is later contracted over its row index in a second, transposed copy, written
// by the epilogue that produces it:
//   forward   Z_l     = A_{l-1} . W_l^T        A = A_{l-1} [B x d],   B = W_l   [d_l x d_{l-1}]
//   backward  D_{l-1} = (D_l . W_l) * f'       A = D_l     [B x d_l], B = W_l^T [d_{l-1} x d_l]
//   gradient  dW_l    = D_l^T . A_{l-1}        A = D_l^T   [d_l x B], B = A_{l-1}^T [d_{l-1} x B]
// 256-thread workgroups, 256 x 128 x 32 (or 128 x 128 x 32) tiles, four wavefronts of 4 x 2 (2 x 2)
// MFMA blocks, operands global -> registers -> LDS (double-buffered, 16-byte accesses throughout).
// The weight-gradient epilogue applies the SGD update (Eq. (3)) to the fp32 master weights
// and refreshes both bf16 copies of W_l in the same pass.
#include "hb_internal.h"

#include <stdlib.h>

namespace hb {
namespace {

typedef __bf16 v8bf __attribute__((ext_vector_type(8)));
typedef float v16f __attribute__((ext_vector_type(16)));
typedef unsigned short bf16_t;  // storage type

constexpr int NT = 256;

__device__ __forceinline__ bf16_t f2bf(float f)
{
    unsigned int u = __float_as_uint(f);
    if ((u & 0x7f800000u) == 0x7f800000u) return (bf16_t)(u >> 16);
    u += 0x7fffu + ((u >> 16) & 1u);
    return (bf16_t)(u >> 16);
}
__device__ __forceinline__ float bf2f(bf16_t b) { return __uint_as_float((unsigned int)b << 16); }

// One operand tile: ROWS x BK bf16, K-major, LDS rows padded by 8 elements (16 bytes) so that
// the 16-byte fragment reads of 8 consecutive lanes fall into disjoint bank groups.
template <int ROWS, int BK>
struct TileB {
    static constexpr int LD = BK + 8;
    static constexpr int ELEMS = ROWS * LD;
    static constexpr int VPT = ROWS * BK / 8 / NT;  // 16-byte vectors per thread
    static_assert(ROWS * BK / 8 % NT == 0, "tile must split evenly over the workgroup");

    // guarded: anything outside [0, nrows) x [.., kend) reads as zero
    static __device__ __forceinline__ void load(uint4 (&reg)[VPT], const bf16_t *__restrict__ P, long long ld,
                                                int row0, int nrows, int k0, int kend, bool vec, int tid)
    {
#pragma unroll
        for (int v = 0; v < VPT; ++v) {
            const int idx = tid + v * NT;
            const int kq = idx % (BK / 8), r = idx / (BK / 8);
            const int row = row0 + r, k = k0 + kq * 8;
            uint4 x = {0u, 0u, 0u, 0u};
            if (row < nrows && k < kend) {
                const bf16_t *p = P + (size_t)row * ld + k;
                if (vec && k + 8 <= kend) {
                    x = *reinterpret_cast<const uint4 *>(p);
                } else {
                    unsigned int w[4] = {0u, 0u, 0u, 0u};
#pragma unroll
                    for (int e = 0; e < 8; ++e)
                        if (k + e < kend) w[e >> 1] |= (unsigned int)p[e] << (16 * (e & 1));
                    x = make_uint4(w[0], w[1], w[2], w[3]);
                }
            }
            reg[v] = x;
        }
    }
    // no guards: the tile lies inside the matrix, rows are 16-byte aligned
    static __device__ __forceinline__ void load_fast(uint4 (&reg)[VPT], const bf16_t *__restrict__ P,
                                                     long long ld, int row0, int k0, int tid)
    {
#pragma unroll
        for (int v = 0; v < VPT; ++v) {
            const int idx = tid + v * NT;
            const int kq = idx % (BK / 8), r = idx / (BK / 8);
            reg[v] = *reinterpret_cast<const uint4 *>(P + (size_t)(row0 + r) * ld + k0 + kq * 8);
        }
    }
    static __device__ __forceinline__ void store(bf16_t *S, const uint4 (&reg)[VPT], int tid)
    {
#pragma unroll
        for (int v = 0; v < VPT; ++v) {
            const int idx = tid + v * NT;
            const int kq = idx % (BK / 8), r = idx / (BK / 8);
            *reinterpret_cast<uint4 *>(&S[r * LD + kq * 8]) = reg[v];
        }
    }
};

__device__ __forceinline__ float act_fwd(float z, int act)
{
    if (act == ACT_SIGMOID) return __builtin_amdgcn_rcpf(1.0f + __expf(-z));
    if (act == ACT_RELU) return fmaxf(z, 0.f);
    return z;
}

template <int BM, int BN, int BK>
constexpr size_t lds_bytes_bf16()
{
    return 2 * (size_t)(TileB<BM, BK>::ELEMS + TileB<BN, BK>::ELEMS) * sizeof(bf16_t);
}

// Workgroup tile BM x BN, four wavefronts as 2 x 2, each (BM/2) x (BN/2) = TM x TN blocks of
// 32 x 32.  Same three-level software pipeline as the fp32 kernel: global loads two k-tiles
// ahead, LDS double-buffered and written early, fragments of the next k-step read under the
// MFMAs of the current one, one barrier per k-tile.
template <int BM, int BN, int BK, int KIND>
__global__ __launch_bounds__(NT, 2) void gemm_bf16_nt_kernel(GemmBf16Args a)  // two workgroups per CU
{
    constexpr int WM = BM / 2, WN = BN / 2;
    constexpr int TM = WM / 32, TN = WN / 32;
    constexpr int G = BK / 16;  // MFMA k-steps per tile
    static_assert(G % 2 == 0, "fragment slots alternate with the k-step parity");
    using TA = TileB<BM, BK>;
    using TB = TileB<BN, BK>;
    constexpr int STAGE = TA::ELEMS + TB::ELEMS;
    extern __shared__ __attribute__((aligned(16))) unsigned char smem_raw[];
    bf16_t *smem = reinterpret_cast<bf16_t *>(smem_raw);

    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int r = lane & 31, h = lane >> 5;
    const int wm = wave & 1, wn = wave >> 1;

    int id = blockIdx.x;
    const int T = gridDim.x;
    if ((T & 7) == 0) id = (id & 7) * (T >> 3) + (id >> 3);  // XCD-aware tile order
    const int tile_m = id / a.tiles_n, tile_n = id - tile_m * a.tiles_n;
    const int m0 = tile_m * BM, n0 = tile_n * BN;
    const int nk = (a.K + BK - 1) / BK;

    const bf16_t *__restrict__ A = static_cast<const bf16_t *>(a.A);
    const bf16_t *__restrict__ Bm = static_cast<const bf16_t *>(a.B);
    const bool a_fast = a.a_vec && (m0 + BM <= a.M), b_fast = a.b_vec && (n0 + BN <= a.N);

    v16f acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;

    uint4 ra[TA::VPT], rb[TB::VPT];
    auto load_tile = [&](int t) {
        const int k0 = t * BK;
        const bool kfull = (k0 + BK <= a.K);
        if (a_fast && kfull) TA::load_fast(ra, A, a.lda, m0, k0, tid);
        else TA::load(ra, A, a.lda, m0, a.M, k0, a.K, a.a_vec != 0, tid);
        if (b_fast && kfull) TB::load_fast(rb, Bm, a.ldb, n0, k0, tid);
        else TB::load(rb, Bm, a.ldb, n0, a.N, k0, a.K, a.b_vec != 0, tid);
    };
    v8bf fa[2][TM], fb[2][TN];
    auto read_frags = [&](int slot, const bf16_t *As, const bf16_t *Bs, int kk) {
#pragma unroll
        for (int i = 0; i < TM; ++i)
            fa[slot][i] = *reinterpret_cast<const v8bf *>(&As[(wm * WM + i * 32 + r) * TA::LD + kk * 16 + h * 8]);
#pragma unroll
        for (int j = 0; j < TN; ++j)
            fb[slot][j] = *reinterpret_cast<const v8bf *>(&Bs[(wn * WN + j * 32 + r) * TB::LD + kk * 16 + h * 8]);
    };
    auto mfma_step = [&](int slot) {
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int j = 0; j < TN; ++j)
                acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[slot][i], fb[slot][j], acc[i][j], 0, 0, 0);
    };

    load_tile(0);
    TA::store(smem, ra, tid);
    TB::store(smem + TA::ELEMS, rb, tid);
    if (nk > 1) load_tile(1);
    __syncthreads();
    read_frags(0, smem, smem + TA::ELEMS, 0);

    for (int kt = 0; kt < nk; ++kt) {
        const bf16_t *As = smem + (kt & 1) * STAGE;
        const bf16_t *Bs = As + TA::ELEMS;
        bf16_t *An = smem + ((kt + 1) & 1) * STAGE;
        if (kt + 1 < nk) {  // tile kt+1 -> the stage nobody reads during this iteration
            TA::store(An, ra, tid);
            TB::store(An + TA::ELEMS, rb, tid);
        }
        if (kt + 2 < nk) load_tile(kt + 2);
#pragma unroll
        for (int kk = 0; kk + 1 < G; ++kk) {
            read_frags((kk + 1) & 1, As, Bs, kk + 1);
            mfma_step(kk & 1);
        }
        __syncthreads();  // tile kt fully read by everyone, tile kt+1 fully written
        if (kt + 1 < nk) read_frags(0, An, An + TA::ELEMS, 0);
        mfma_step((G - 1) & 1);
    }

    // ---- epilogue.  acc[i][j][v] = C(row, col): row = 8 (v / 4) + 4 h + (v % 4), col = r
#pragma unroll
    for (int j = 0; j < TN; ++j) {
        const int n = n0 + wn * WN + j * 32 + r;
        const bool n_ok = n < a.N;
        float bias = 0.f;
        if (KIND == GEMM_FWD && a.bias != nullptr && n_ok) bias = a.bias[n];
#pragma unroll
        for (int i = 0; i < TM; ++i) {
#pragma unroll
            for (int q = 0; q < 4; ++q) {  // groups of 4 consecutive rows
                const int mq = m0 + wm * WM + i * 32 + 8 * q + 4 * h;
                float x[4];
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    const int m = mq + e;
                    float val = acc[i][j][4 * q + e];
                    if (m < a.M && n_ok) {
                        if (KIND == GEMM_FWD) {
                            val = act_fwd(val + bias, a.act);
                            if (a.C_f32) static_cast<float *>(a.C_f32)[(size_t)m * a.ldc + n] = val;
                        } else if (KIND == GEMM_DA) {
                            const float o = bf2f(static_cast<const bf16_t *>(a.aux)[(size_t)m * a.ldaux + n]);
                            if (a.act == ACT_SIGMOID) val *= o * (1.f - o);
                            else if (a.act == ACT_RELU) val = (o > 0.f) ? val : 0.f;
                        } else {  // GEMM_DW
                            float *cf = static_cast<float *>(a.C_f32) + (size_t)m * a.ldc + n;
                            if (a.write_grad) {
                                *cf = val;
                            } else {
                                val = *cf - a.lr * val;  // Eq. (3) on the fp32 master weight
                                *cf = val;
                            }
                        }
                        if (a.C_bf16) static_cast<bf16_t *>(a.C_bf16)[(size_t)m * a.ldcb + n] = f2bf(val);
                    }
                    x[e] = val;
                }
                if (a.Ct_bf16 && n_ok && !(KIND == GEMM_DW && a.write_grad)) {
                    bf16_t *ct = static_cast<bf16_t *>(a.Ct_bf16) + (size_t)n * a.ldct + mq;
                    if (mq + 4 <= a.M && (a.ldct & 3) == 0) {
                        uint2 pk;
                        pk.x = (unsigned int)f2bf(x[0]) | ((unsigned int)f2bf(x[1]) << 16);
                        pk.y = (unsigned int)f2bf(x[2]) | ((unsigned int)f2bf(x[3]) << 16);
                        *reinterpret_cast<uint2 *>(ct) = pk;
                    } else {
#pragma unroll
                        for (int e = 0; e < 4; ++e)
                            if (mq + e < a.M) ct[e] = f2bf(x[e]);
                    }
                }
            }
        }
    }
}

// out[c][r] = in[r][c] for bf16 matrices (R x C, leading dimensions ldi / ldo), 64 x 64 tiles
__global__ __launch_bounds__(256) void transpose_bf16_kernel(const bf16_t *__restrict__ in, long long ldi,
                                                             bf16_t *__restrict__ out, long long ldo, int R, int C)
{
    __shared__ bf16_t t[64][66];
    const int tx = threadIdx.x & 63, ty = threadIdx.x >> 6;  // 64 x 4
    const int c0 = blockIdx.x * 64, r0 = blockIdx.y * 64;
    for (int k = ty; k < 64; k += 4)
        if (r0 + k < R && c0 + tx < C) t[k][tx] = in[(size_t)(r0 + k) * ldi + c0 + tx];
    __syncthreads();
    for (int k = ty; k < 64; k += 4)
        if (c0 + k < C && r0 + tx < R) out[(size_t)(c0 + k) * ldo + r0 + tx] = t[tx][k];
}

// bf16 copies of an fp32 weight matrix W [R x C]: shadow [R x lds_] and shadow_t [C x ldt]
__global__ __launch_bounds__(256) void shadow_kernel(const float *__restrict__ W, int R, int C,
                                                     bf16_t *__restrict__ shadow, long long lds_,
                                                     bf16_t *__restrict__ shadow_t, long long ldt)
{
    __shared__ bf16_t t[64][66];
    const int tx = threadIdx.x & 63, ty = threadIdx.x >> 6;
    const int c0 = blockIdx.x * 64, r0 = blockIdx.y * 64;
    for (int k = ty; k < 64; k += 4)
        if (r0 + k < R && c0 + tx < C) {
            const bf16_t b = f2bf(W[(size_t)(r0 + k) * C + c0 + tx]);
            t[k][tx] = b;
            shadow[(size_t)(r0 + k) * lds_ + c0 + tx] = b;
        }
    __syncthreads();
    for (int k = ty; k < 64; k += 4)
        if (c0 + k < C && r0 + tx < R) shadow_t[(size_t)(c0 + k) * ldt + r0 + tx] = t[tx][k];
}

// Bias gradient from the transposed delta (one wavefront per output unit j):
//   g = sum_b Dt[j][b];  b_l[j] -= lr g   or   grad[j] = g
__global__ __launch_bounds__(256) void rowsum_bias_kernel(const bf16_t *__restrict__ Dt, long long ld, int d,
                                                          long long B, float *__restrict__ bias,
                                                          float *__restrict__ grad, float lr)
{
    const int j = blockIdx.x * 4 + (threadIdx.x >> 6);
    const int lane = threadIdx.x & 63;
    if (j >= d) return;
    const bf16_t *row = Dt + (size_t)j * ld;
    float s = 0.f;
    for (long long b = lane; b < B; b += 64) s += bf2f(row[b]);
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) s += __shfl_xor(s, o, 64);
    if (lane == 0) {
        if (grad) grad[j] = s;
        else bias[j] -= lr * s;
    }
}

template <int BM, int BN, int BK>
hipError_t launch_shape_bf16(GemmKind kind, GemmBf16Args a, hipStream_t stream, const LaunchEvents &ev)
{
    constexpr size_t LDS = lds_bytes_bf16<BM, BN, BK>();
    void (*k)(GemmBf16Args) = kind == GEMM_FWD  ? gemm_bf16_nt_kernel<BM, BN, BK, GEMM_FWD>
                              : kind == GEMM_DA ? gemm_bf16_nt_kernel<BM, BN, BK, GEMM_DA>
                                                : gemm_bf16_nt_kernel<BM, BN, BK, GEMM_DW>;
    static bool attr_set[3] = {false, false, false};  // per instantiation (BM, BN, BK) and kind
    if (LDS > 48 * 1024 && !attr_set[kind]) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(k),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)LDS);
        if (e != hipSuccess) return e;
        attr_set[kind] = true;
    }
    a.tiles_m = (a.M + BM - 1) / BM;
    a.tiles_n = (a.N + BN - 1) / BN;
    const long long tiles = (long long)a.tiles_m * a.tiles_n;
    if (tiles > 0x7fffffffLL) return hipErrorInvalidValue;
    const dim3 grid((unsigned)tiles), block(NT);
    if (ev.start)
        hipExtLaunchKernelGGL(k, grid, block, (unsigned)LDS, stream, ev.start, ev.stop, 0, a);
    else
        hipLaunchKernelGGL(k, grid, block, LDS, stream, a);
    return hipGetLastError();
}

int env_int_bf16(const char *name, int dflt)
{
    const char *v = getenv(name);
    return (v && *v) ? atoi(v) : dflt;
}

}  // namespace

hipError_t launch_gemm_bf16(GemmKind kind, GemmBf16Args a, hipStream_t stream, const LaunchEvents &ev)
{
    if (a.M <= 0 || a.N <= 0 || a.K <= 0) return hipErrorInvalidValue;
    // 256 x 128 tiles (4 x 2 MFMA blocks per wavefront: 6 fragment reads per 8 MFMAs) when they
    // still give two workgroups per CU, else 128 x 128.  HB_BF16_TILE = 1 / 2 forces (tuning aid).
    static const int forced = env_int_bf16("HB_BF16_TILE", 0);
    const long long big_tiles = (long long)((a.M + 255) / 256) * ((a.N + 127) / 128);
    const bool big = forced == 1 ? true : forced == 2 ? false : forced == 3 ? false : big_tiles >= 512;
    if (big) return launch_shape_bf16<256, 128, 32>(kind, a, stream, ev);
    if (forced == 3) return launch_shape_bf16<128, 128, 32>(kind, a, stream, ev);
    return launch_shape_bf16<128, 128, 64>(kind, a, stream, ev);
}

hipError_t launch_transpose_bf16(const void *in, long long ldi, void *out, long long ldo, int R, int C,
                                 hipStream_t stream, const LaunchEvents &ev)
{
    return launch_kernel(transpose_bf16_kernel, dim3((unsigned)((C + 63) / 64), (unsigned)((R + 63) / 64)),
                         dim3(256), stream, ev, static_cast<const bf16_t *>(in), ldi, static_cast<bf16_t *>(out),
                         ldo, R, C);
}

hipError_t launch_shadow(const float *W, int R, int C, void *shadow, long long lds_, void *shadow_t,
                         long long ldt, hipStream_t stream)
{
    return launch_kernel(shadow_kernel, dim3((unsigned)((C + 63) / 64), (unsigned)((R + 63) / 64)), dim3(256),
                         stream, LaunchEvents(), W, R, C, static_cast<bf16_t *>(shadow), lds_,
                         static_cast<bf16_t *>(shadow_t), ldt);
}

hipError_t launch_rowsum_bias(const void *Dt, long long ld, int d, long long B, float *bias, float *grad,
                              float lr, hipStream_t stream, const LaunchEvents &ev)
{
    return launch_kernel(rowsum_bias_kernel, dim3((unsigned)((d + 3) / 4)), dim3(256), stream, ev,
                         static_cast<const bf16_t *>(Dt), ld, d, B, bias, grad, lr);
}

}  // namespace hb
