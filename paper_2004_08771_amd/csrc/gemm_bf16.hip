// bf16 MFMA GEMM for the mixed-precision mode (bf16 weights / activations, fp32 master
// weights and accumulation) of the mini-batch step: the same three layer products as the
// fp32 path (Section 3 of the paper, Eq. (1) forward and Eq. (2) backward).
//
// gfx950 design: v_mfma_f32_32x32x16_bf16 wants 8 consecutive k per lane.
//   forward   Z_l     = A_{l-1} . W_l^T        A = A_{l-1} [B x d],   B = W_l   [d_l x d_{l-1}]   both K-major
//   backward  D_{l-1} = (D_l . W_l) * f'       A = D_l     [B x d_l], B = W_l^T [d_{l-1} x d_l]   both K-major
//   gradient  dW_l    = D_l^T . A_{l-1}        contraction over the batch, the ROW index of both
// The weights exist as two bf16 copies (W_l and W_l^T), rewritten by the weight-gradient
// epilogue, which also applies the SGD update (Eq. (3)) to the fp32 master weights.  The
// weight gradient reads D_l and A_{l-1} as they are, batch-major, through the transposing LDS
// read of gfx950 (LDS-direct kernel, BMAJ form); only where it cannot (rows that are not
// 16-byte aligned, products too small for 256 x 256 tiles) do the epilogues that produce a
// tensor also write its transposed copy, and the product runs K-major like the other two.
// Two kernel families: gemm_bf16_nt_kernel (256-thread workgroups, 256 x 128 x 32 or
// 128 x 128 tiles, four wavefronts, operands global -> registers -> LDS, double-buffered,
// 16-byte accesses throughout) for small or unaligned products, gemm_bf16_dma_kernel
// (256 x 256 x 64, LDS-direct loads) for the large ones.
#include "hb_internal.h"

#include <mutex>
#include <stdlib.h>

namespace hb {
namespace {

typedef __bf16 v8bf __attribute__((ext_vector_type(8)));
typedef float v16f __attribute__((ext_vector_type(16)));
typedef unsigned short bf16_t;  // storage type

constexpr int NT = 256;

// fp32 -> bf16, round to nearest even: gfx950's v_cvt_pk_bf16_f32 (checked against the bit
// formula u + 0x7fff + ((u >> 16) & 1) on all 2^32 inputs: identical for every non-NaN value,
// NaN stays NaN).  One instruction per pair instead of about seven integer operations per
// value, which the epilogues of the GEMMs run 128 times per lane and tile.
typedef float f32x2_t __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
__device__ __forceinline__ bf16_t f2bf(float f) { return __builtin_bit_cast(bf16_t, (__bf16)f); }
__device__ __forceinline__ unsigned int pack2bf(float lo, float hi)
{
    const f32x2_t v = {lo, hi};
    return __builtin_bit_cast(unsigned int, __builtin_convertvector(v, bf16x2_t));
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

// The activation is a template argument of the epilogues: tested at run time per value, it
// became three scalar branches in front of each of a lane's 128 outputs (about 5 us per
// 256 x 256 tile, with the MFMA pipes idle).
template <int ACT>
__device__ __forceinline__ float act_fwd(float z)
{
    if (ACT == ACT_SIGMOID) return __builtin_amdgcn_rcpf(1.0f + __expf(-z));
    if (ACT == ACT_RELU) return fmaxf(z, 0.f);
    return z;
}
template <int V>
struct IntC {
    static constexpr int value = V;
};
// calls f(IntC<activation>, IntC<mask ? 1 : 0>) with the run-time activation as a constant
template <typename F>
__device__ __forceinline__ void with_activation(int act, bool mask, F &&f)
{
    if (act == ACT_RELU) {
        if (mask) f(IntC<ACT_RELU>(), IntC<1>());
        else f(IntC<ACT_RELU>(), IntC<0>());
    } else if (act == ACT_SIGMOID) {
        f(IntC<ACT_SIGMOID>(), IntC<0>());
    } else {
        f(IntC<ACT_NONE>(), IntC<0>());
    }
}

// ReLU decision bits of one 32 x 32 block (see GemmBf16Args::mask_out): position of the value
// (q, e) = row 8 q + 4 h + e in the lane's 16-bit word, the word from the lane's 16 packed
// bf16 values (pk[q] = rows e = 0..3 of group q), and the use of a bit on a backward value.
// "Positive" is: sign clear and magnitude not zero (true for a NaN as well, where `> 0` is not).
__device__ __forceinline__ constexpr int relu_bit_pos(int q, int e) { return 8 * (e & 1) + 2 * q + (e >> 1); }
__device__ __forceinline__ unsigned relu_bits(const uint2 (&pk)[4])
{
    unsigned acc = 0;
#pragma unroll
    for (int k = 0; k < 8; ++k) {  // dword k holds (q, e) = (k / 2, 2 (k % 2)) below (q, e + 1)
        const unsigned x = (k & 1) ? pk[k >> 1].y : pk[k >> 1].x;
        const unsigned t = ((x & 0x7fff7fffu) + 0x7fff7fffu) & ~x;  // bits 15 / 31: the half is positive
        acc = (t & 0x80008000u) | (acc >> 1);
    }
    // the low halves of dwords 0..7 now sit at bits 8..15, the high halves at bits 24..31
    return ((acc >> 8) & 0xffu) | ((acc >> 16) & 0xff00u);
}
__device__ __forceinline__ float relu_keep(float val, unsigned word, int q, int e)
{
    const int m = (int)(word << (31 - relu_bit_pos(q, e))) >> 31;  // 0 or -1 (one v_bfe_i32)
    return __uint_as_float(__float_as_uint(val) & (unsigned)m);
}

template <int BM, int BN, int BK>
constexpr size_t lds_bytes_bf16()
{
    return 2 * (size_t)(TileB<BM, BK>::ELEMS + TileB<BN, BK>::ELEMS) * sizeof(bf16_t);
}

// Epilogue shared by both kernels.  acc[i][j][v] = C(row, col) of the wavefront's block (i, j):
// row = 8 (v / 4) + 4 h + (v % 4), col = r.  (mw, nw) is the wavefront's first row / column and
// must be wavefront-uniform: every address below is a scalar base (row, column block) plus a
// per-lane byte offset that does not change during the epilogue, so the 128 outputs of a lane
// cost no address registers.
// FULL: the wavefront's tile lies inside the matrix and the 8-byte accesses are aligned; no
// guards, and what a column block needs from memory (bias, the activations of the
// backward-data derivative, the fp32 master weights of the fused update) is requested before
// its first use, so that those loads are in flight together instead of one round trip each.
// ACT: the activation (forward, backward-data).  MASK: the ReLU decision bits are written
// (forward: mask_out) / read instead of the activations (backward-data: mask_in).
template <int KIND, int TM, int TN, bool FULL, int ACT, bool MASK>
__device__ __forceinline__ void epilogue_bf16_impl(const GemmBf16Args &a, v16f (&acc)[TM][TN], int mw, int nw, int r,
                                                   int h)
{
    const bool has_cf = a.C_f32 != nullptr, has_cb = a.C_bf16 != nullptr;
    const bool has_ct = a.Ct_bf16 != nullptr && !(KIND == GEMM_DW && a.write_grad);
    const bool use_t = (KIND == GEMM_DA) && a.aux_t != nullptr && (a.ldauxt & 3) == 0;
    constexpr bool use_mask = (KIND == GEMM_DA) && MASK;
    const bool ct_vec = (a.ldct & 3) == 0;
    // per-lane byte offsets (row part 4 h, column part r)
    const unsigned lo_cf = (unsigned)(4 * h * (int)a.ldc + r) * 4u;
    const unsigned lo_cb = (unsigned)(4 * h * (int)a.ldcb + r) * 2u;
    const unsigned lo_ct = (unsigned)(r * (int)a.ldct + 4 * h) * 2u;
    const unsigned lo_at = (unsigned)(r * (int)a.ldauxt + 4 * h) * 2u;
    const unsigned lo_ax = (unsigned)(4 * h * (int)a.ldaux + r) * 2u;
    unsigned char *const cf0 = static_cast<unsigned char *>(a.C_f32);
    unsigned char *const cb0 = static_cast<unsigned char *>(a.C_bf16);
    unsigned char *const ct0 = static_cast<unsigned char *>(a.Ct_bf16);
    const unsigned char *const at0 = static_cast<const unsigned char *>(a.aux_t);
    const unsigned char *const ax0 = static_cast<const unsigned char *>(a.aux);
#pragma unroll
    for (int j = 0; j < TN; ++j) {
        const int nb = nw + j * 32;  // uniform
        const int n = nb + r;
        const bool n_ok = FULL || n < a.N;
        float bias = 0.f;
        if (KIND == GEMM_FWD && a.bias != nullptr && n_ok) bias = a.bias[n];
        uint2 ot[TM][4];
        if (KIND == GEMM_DA && FULL && !use_mask) {
#pragma unroll
            for (int i = 0; i < TM; ++i)
#pragma unroll
                for (int q = 0; q < 4; ++q)
                    ot[i][q] = *reinterpret_cast<const uint2 *>(
                        at0 + ((size_t)nb * a.ldauxt + (mw + i * 32 + 8 * q)) * 2 + lo_at);
            __builtin_amdgcn_sched_barrier(0);
        }
        // ReLU decision bits: a block is addressed only when it holds a valid element (the
        // array covers ceil(M / 32) x ceil(N / 32) blocks)
        unsigned mword[TM];
#pragma unroll
        for (int i = 0; i < TM; ++i) {
            mword[i] = 0u;
            if (KIND == GEMM_DA && use_mask && (FULL || (mw + i * 32 < a.M && nb < a.N)))
                mword[i] = a.mask_in[((size_t)((mw + i * 32) >> 5) * a.mask_nb + (nb >> 5)) * 64 + 32 * h + r];
        }
        float csum = 0.f;  // backward-data: sum of the lane's stored results of this column
#pragma unroll
        for (int i = 0; i < TM; ++i) {
            unsigned mbits = 0u;
            float w[16];
            if (KIND == GEMM_DW && FULL && !a.write_grad) {
#pragma unroll
                for (int v = 0; v < 16; ++v)
                    w[v] = *reinterpret_cast<const float *>(
                        cf0 + ((size_t)(mw + i * 32 + 8 * (v >> 2) + (v & 3)) * a.ldc + nb) * 4 + lo_cf);
                __builtin_amdgcn_sched_barrier(0);
            }
#pragma unroll
            for (int q = 0; q < 4; ++q) {  // groups of 4 consecutive rows
                const int mb = mw + i * 32 + 8 * q;  // uniform; this lane's rows are mb + 4 h + e
                const int mq = mb + 4 * h;
                uint2 o4 = {0u, 0u};
                if (KIND == GEMM_DA && !use_mask) {
                    if (FULL) o4 = ot[i][q];
                    else if (use_t && n_ok && mq < a.M)  // rows of the copy are padded to 4: in bounds
                        o4 = *reinterpret_cast<const uint2 *>(at0 + ((size_t)nb * a.ldauxt + mb) * 2 + lo_at);
                }
                float x[4];
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    float val = acc[i][j][4 * q + e];
                    if (FULL || (mq + e < a.M && n_ok)) {
                        if (KIND == GEMM_FWD) {
                            val = act_fwd<ACT>(val + bias);
                            if (has_cf)
                                *reinterpret_cast<float *>(cf0 + ((size_t)(mb + e) * a.ldc + nb) * 4 + lo_cf) = val;
                            if (MASK) {
                                const bf16_t b = f2bf(val);
                                if ((b & 0x7fffu) != 0 && (b & 0x8000u) == 0) mbits |= 1u << relu_bit_pos(q, e);
                            }
                        } else if (KIND == GEMM_DA && use_mask) {
                            val = relu_keep(val, mword[i], q, e);
                        } else if (KIND == GEMM_DA) {
                            float o;
                            if (FULL || use_t) {
                                const unsigned int pw = (e < 2) ? o4.x : o4.y;
                                o = __uint_as_float((e & 1) ? (pw & 0xffff0000u) : (pw << 16));
                            } else {
                                o = bf2f(*reinterpret_cast<const bf16_t *>(ax0 + ((size_t)(mb + e) * a.ldaux + nb) * 2 +
                                                                            lo_ax));
                            }
                            if (ACT == ACT_SIGMOID) val *= o * (1.f - o);
                            else if (ACT == ACT_RELU) val = (o > 0.f) ? val : 0.f;
                        } else {  // GEMM_DW
                            float *cf = reinterpret_cast<float *>(cf0 + ((size_t)(mb + e) * a.ldc + nb) * 4 + lo_cf);
                            if (!a.write_grad) val = (FULL ? w[4 * q + e] : *cf) - a.lr * val;  // Eq. (3), fp32 master
                            *cf = val;
                        }
                        if (has_cb)
                            *reinterpret_cast<bf16_t *>(cb0 + ((size_t)(mb + e) * a.ldcb + nb) * 2 + lo_cb) = f2bf(val);
                        if (KIND == GEMM_DA && a.colsum_partial != nullptr) csum += bf2f(f2bf(val));
                    }
                    x[e] = val;
                }
                if (has_ct && n_ok) {
                    unsigned char *ct = ct0 + ((size_t)nb * a.ldct + mb) * 2 + lo_ct;
                    if (FULL || (mq + 4 <= a.M && ct_vec)) {
                        uint2 pk;
                        pk.x = pack2bf(x[0], x[1]);
                        pk.y = pack2bf(x[2], x[3]);
                        *reinterpret_cast<uint2 *>(ct) = pk;
                    } else {
#pragma unroll
                        for (int e = 0; e < 4; ++e)
                            if (mq + e < a.M) reinterpret_cast<bf16_t *>(ct)[e] = f2bf(x[e]);
                    }
                }
                // keep the scheduler from pulling later groups' conversions up: with 128
                // accumulators live it runs out of registers
                __builtin_amdgcn_sched_barrier(0);
            }
            if (KIND == GEMM_FWD && MASK && (FULL || (mw + i * 32 < a.M && nb < a.N)))
                a.mask_out[((size_t)((mw + i * 32) >> 5) * a.mask_nb + (nb >> 5)) * 64 + 32 * h + r] =
                    (unsigned short)mbits;
        }
        // column sums over the wavefront's 128 rows (LDS-direct kernel only: mw is a multiple of
        // 128): the two half-wavefronts hold alternate groups of four rows
        if (KIND == GEMM_DA && a.colsum_partial != nullptr) {
            csum += __shfl_xor(csum, 32, 64);
            if (h == 0 && n_ok) a.colsum_partial[(size_t)(mw >> 7) * a.N + n] = csum;
        }
    }
}

template <int KIND, int TM, int TN>
__device__ __forceinline__ void epilogue_bf16(const GemmBf16Args &a, v16f (&acc)[TM][TN], int mw, int nw, int r,
                                              int h)
{
    const bool mask = KIND == GEMM_FWD  ? (a.mask_out != nullptr && a.act == ACT_RELU)
                      : KIND == GEMM_DA ? (a.mask_in != nullptr && a.act == ACT_RELU)
                                        : false;
    const bool full = (mw + 32 * TM <= a.M) && (nw + 32 * TN <= a.N) &&
                      (a.Ct_bf16 == nullptr || (a.ldct & 3) == 0) &&
                      (KIND != GEMM_DA || mask || (a.aux_t != nullptr && (a.ldauxt & 3) == 0));
    with_activation(KIND == GEMM_DW ? (int)ACT_NONE : a.act, mask, [&](auto act_c, auto mask_c) {
        constexpr int ACT = decltype(act_c)::value;
        constexpr bool MASK = decltype(mask_c)::value != 0;
        if (full) epilogue_bf16_impl<KIND, TM, TN, true, ACT, MASK>(a, acc, mw, nw, r, h);
        else epilogue_bf16_impl<KIND, TM, TN, false, ACT, MASK>(a, acc, mw, nw, r, h);
    });
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

    epilogue_bf16<KIND, TM, TN>(a, acc, __builtin_amdgcn_readfirstlane(m0 + wm * WM),
                                __builtin_amdgcn_readfirstlane(n0 + wn * WN), r, h);
}

// ---- 256 x 256 x 64 kernel with LDS-direct loads ------------------------------------------
// Used when both operands allow 16-byte loads and the product is large enough for 256 x 256
// tiles.  512 threads: eight wavefronts as 2 x 4, each 128 x 64 (4 x 2 MFMA blocks), two per
// SIMD.  Differences from the kernel above:
//   * operand tiles go global -> LDS directly (global_load_lds_dwordx4: lane i of a wavefront
//     writes its 16 bytes at LDS base + 16 i), no staging registers and no ds_write;
//   * a k-tile row is 128 bytes, one whole cache line: with 64-byte rows every line was
//     fetched twice from L2 (the 32 KB L1 does not keep it for an iteration), and the
//     L2 -> L1 path (64 B/clk/CU) became the limit; the square tile needs 32 B/clk/CU at
//     full MFMA rate;
//   * rows are not padded; the eight 16-byte chunks of tile row R are stored at slot
//     c ^ swz(R), which keeps both the direct loads (a wavefront fills 1 KB contiguously) and
//     the MFMA fragment reads free of bank conflicts;
//   * out-of-range rows of an edge tile are clamped to the last valid row when loading (their
//     results are never stored), so the main loop has no guards; a K tail shorter than a tile
//     is multiplied after the loop from a masked, register-staged copy.
// LDS holds two stages of the A tile and three of the B tile (32 KB each: all 160 KB).  Per
// iteration every wavefront issues eight loads, two under each of the four MFMA groups (all
// at once they fill the address queue of the vector memory unit and the MFMA pipes idle while
// it drains): A of tile kt+1 under the last group of kt-1 and the first of kt, B of tile kt+2
// under groups two and three of kt, so that every load has at least two MFMA groups (B: more
// than an iteration) to land; an L2 round trip measured here takes ~550 cycles on average.
// Waits and barriers inside the main loop are written out by hand: at a workgroup barrier the
// compiler would also wait for the direct loads that were only just issued.
typedef __attribute__((address_space(1))) const void *gptr_t;
typedef __attribute__((address_space(3))) void *lptr_t;
typedef int v2i __attribute__((ext_vector_type(2)));
template <int K>
struct KStep {
    static constexpr int value = K;
};

// gfx950's transposing LDS read of 8 bytes per lane at LDS byte address addr + OFF.  Written as
// an instruction, not through the compiler's builtin: for the builtin the compiler cannot
// tell that the read does not touch what the LDS-direct loads in flight are writing, and puts
// a wait for ALL of them (vmcnt(0)) in front of every read (the weight gradient
// 4096 x 4096 x 16384 took 530 us that way).  The compiler does not wait for the result
// either: every use below sits behind an explicit lgkmcnt(0) and a scheduling barrier.
template <int OFF>
__device__ __forceinline__ v2i lds_read_tr16_b64(unsigned addr)
{
    static_assert(OFF >= 0 && OFF < 65536, "16-bit offset field");
    v2i v;
    asm volatile("ds_read_b64_tr_b16 %0, %1 offset:%2" : "=v"(v) : "v"(addr), "n"(OFF));
    return v;
}

// slot permutation of tile row R: bit 0 of the chunk index (the half-wavefront h of a fragment
// read) is never mixed with the row bits that vary inside one 16-lane group
__device__ __forceinline__ int swz(int R)
{
    const int q = (R >> 1) & 7;
    return ((q & 3) << 1) | (q >> 2);
}

constexpr int DMA_NT = 512;
constexpr int DMA_BM = 256, DMA_BN = 256, DMA_BK = 64;
constexpr int DMA_ROW_BYTES = DMA_BK * 2;  // 128
constexpr int DMA_A_BYTES = DMA_BM * DMA_ROW_BYTES, DMA_B_BYTES = DMA_BN * DMA_ROW_BYTES;
constexpr int DMA_A_STAGES = 2, DMA_B_STAGES = 3;
constexpr int DMA_B_BASE = DMA_A_STAGES * DMA_A_BYTES;
constexpr size_t DMA_LDS_BYTES = (size_t)DMA_B_BASE + (size_t)DMA_B_STAGES * DMA_B_BYTES;  // 163,840: all of a CU's LDS

// Epilogue of the LDS-direct kernel when the whole workgroup tile lies inside the matrix (for
// the weight gradient: the form with the fused update, whose fp32 master weights are read
// and written directly): both bf16 outputs (row-major and transposed) leave
// through LDS, so that every global store is 16 bytes per lane and covers whole cache lines
// (128 bytes per row-major row, 256 per transposed row).  Straight from the MFMA layout a
// lane owns four consecutive rows of one column: 128 two-byte stores plus 32 eight-byte
// ones per lane, and the forward product took 86 us longer with them than with plain fp32
// output of the same size.  Each wavefront has 20 KB of LDS to itself (the operand stages
// are dead by now), used twice: 128 rows x 144 bytes for the row-major tile, then 64 rows x
// 272 bytes for the transposed one.
constexpr int EPI_REGION = 20480;
constexpr int EPI_SC = 144;  // row stride of the 128 x 64 row-major tile (128 bytes + 16)
constexpr int EPI_ST = 272;  // row stride of the 64 x 128 transposed tile (256 bytes + 16)
static_assert(128 * EPI_SC <= EPI_REGION && 64 * EPI_ST <= EPI_REGION && 8 * EPI_REGION <= (int)DMA_LDS_BYTES, "LDS");

// mword: backward-data product with ReLU decision bits (use_mask): the lane's words of its eight
// blocks, requested by the caller before the main loop.
template <int KIND, int ACT, bool MASK>
__device__ __forceinline__ void epilogue_bf16_lds(const GemmBf16Args &a, v16f (&acc)[4][2], unsigned char *region,
                                                  int mw, int nw, int lane, const unsigned (&mword)[4][2])
{
    constexpr bool use_mask = (KIND == GEMM_DA) && MASK;
    constexpr int TM = 4, TN = 2;
    const int r = lane & 31, h = lane >> 5;
    // ---- values -> bf16, four consecutive rows packed per (i, j, q)
    uint2 pk[TM][TN][4];
    const unsigned lo_at = (unsigned)(r * (int)a.ldauxt + 4 * h) * 2u;
    const unsigned char *const at0 = static_cast<const unsigned char *>(a.aux_t);
    const unsigned lo_cf = (unsigned)(4 * h * (int)a.ldc + r) * 4u;
    unsigned char *const cf0 = static_cast<unsigned char *>(a.C_f32);
#pragma unroll
    for (int j = 0; j < TN; ++j) {
        const int nb = nw + j * 32;
        float bias = 0.f;
        if (KIND == GEMM_FWD && a.bias != nullptr) bias = a.bias[nb + r];
        uint2 ot[TM][4];
        if (KIND == GEMM_DA && !use_mask) {
#pragma unroll
            for (int i = 0; i < TM; ++i)
#pragma unroll
                for (int q = 0; q < 4; ++q)
                    ot[i][q] = *reinterpret_cast<const uint2 *>(
                        at0 + ((size_t)nb * a.ldauxt + (mw + i * 32 + 8 * q)) * 2 + lo_at);
            __builtin_amdgcn_sched_barrier(0);
        }
#pragma unroll
        for (int i = 0; i < TM; ++i) {
            // weight gradient: the 16 fp32 master weights of this 32 x 32 block that the lane
            // updates are requested together.  Fetched four at a time between the stores of
            // the previous four (which the compiler must assume to alias), every group of four
            // was a round trip to memory of its own: 64 per lane and tile.
            float wm[4][4];
            if (KIND == GEMM_DW) {
#pragma unroll
                for (int q = 0; q < 4; ++q)
#pragma unroll
                    for (int e = 0; e < 4; ++e)
                        wm[q][e] = *reinterpret_cast<const float *>(
                            cf0 + ((size_t)(mw + i * 32 + 8 * q + e) * a.ldc + nb) * 4 + lo_cf);
                __builtin_amdgcn_sched_barrier(0);
            }
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                float (&w)[4] = wm[q];
                float x[4];
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    float val = acc[i][j][4 * q + e];
                    if (KIND == GEMM_FWD) {
                        val = act_fwd<ACT>(val + bias);
                    } else if (KIND == GEMM_DA) {
                        if (use_mask) {
                            val = relu_keep(val, mword[i][j], q, e);
                        } else {
                            const unsigned int pw = (e < 2) ? ot[i][q].x : ot[i][q].y;
                            const float o = __uint_as_float((e & 1) ? (pw & 0xffff0000u) : (pw << 16));
                            if (ACT == ACT_SIGMOID) val *= o * (1.f - o);
                            else if (ACT == ACT_RELU) val = (o > 0.f) ? val : 0.f;
                        }
                    } else {  // Eq. (3) on the fp32 master weight, stored back directly
                        val = w[e] - a.lr * val;
                        *reinterpret_cast<float *>(cf0 + ((size_t)(mw + i * 32 + 8 * q + e) * a.ldc + nb) * 4 + lo_cf) = val;
                    }
                    x[e] = val;
                }
                pk[i][j][q].x = pack2bf(x[0], x[1]);
                pk[i][j][q].y = pack2bf(x[2], x[3]);
                __builtin_amdgcn_sched_barrier(0);
            }
        }
    }
    // ---- backward-data: column sums of the stored values over the wavefront's 128 rows (the
    // bias gradient of the layer below), in a fixed order; the two half-wavefronts hold
    // alternate groups of four rows
    if (KIND == GEMM_DA && a.colsum_partial != nullptr) {
#pragma unroll
        for (int j = 0; j < TN; ++j) {
            float s = 0.f;
#pragma unroll
            for (int i = 0; i < TM; ++i)
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    const uint2 v = pk[i][j][q];
                    s += (__uint_as_float(v.x << 16) + __uint_as_float(v.x & 0xffff0000u)) +
                         (__uint_as_float(v.y << 16) + __uint_as_float(v.y & 0xffff0000u));
                }
            s += __shfl_xor(s, 32, 64);
            if (h == 0) a.colsum_partial[(size_t)(mw >> 7) * a.N + nw + j * 32 + r] = s;
        }
    }
    // ---- row-major copy: T[m][n], lane writes its four rows of column j*32 + r
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                unsigned char *p = region + (i * 32 + 8 * q + 4 * h) * EPI_SC + (j * 32 + r) * 2;
                *reinterpret_cast<bf16_t *>(p) = (bf16_t)(pk[i][j][q].x & 0xffffu);
                *reinterpret_cast<bf16_t *>(p + EPI_SC) = (bf16_t)(pk[i][j][q].x >> 16);
                *reinterpret_cast<bf16_t *>(p + 2 * EPI_SC) = (bf16_t)(pk[i][j][q].y & 0xffffu);
                *reinterpret_cast<bf16_t *>(p + 3 * EPI_SC) = (bf16_t)(pk[i][j][q].y >> 16);
            }
    {
        unsigned char *const cb = static_cast<unsigned char *>(a.C_bf16) + ((size_t)mw * a.ldcb + nw) * 2;
#pragma unroll
        for (int it = 0; it < 16; ++it) {  // 128 rows x 8 chunks of 16 bytes
            const int c = it * 64 + lane, row = c >> 3, ch = c & 7;
            const uint4 v = *reinterpret_cast<const uint4 *>(region + row * EPI_SC + ch * 16);
            *reinterpret_cast<uint4 *>(cb + (size_t)row * a.ldcb * 2 + ch * 16) = v;
        }
    }
    // ---- forward product of a ReLU layer: the decision bits of the lane's eight blocks, worked
    // out while the stores above drain
    if (KIND == GEMM_FWD && MASK) {
        unsigned short *const mo = a.mask_out + ((size_t)(mw >> 5) * a.mask_nb + (nw >> 5)) * 64 + lane;
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int j = 0; j < TN; ++j) mo[((size_t)i * a.mask_nb + j) * 64] = (unsigned short)relu_bits(pk[i][j]);
    }
    if (a.Ct_bf16 == nullptr) return;  // uniform
    // ---- transposed copy: T[n][m], lane writes 8 bytes (its four rows) into row j*32 + r.  The
    // region is reused: LDS operations of a wavefront execute in order
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int q = 0; q < 4; ++q)
                *reinterpret_cast<uint2 *>(region + (j * 32 + r) * EPI_ST + (i * 32 + 8 * q + 4 * h) * 2) = pk[i][j][q];
    {
        unsigned char *const ct = static_cast<unsigned char *>(a.Ct_bf16) + ((size_t)nw * a.ldct + mw) * 2;
#pragma unroll
        for (int it = 0; it < 16; ++it) {  // 64 rows x 16 chunks of 16 bytes
            const int c = it * 64 + lane, row = c >> 4, ch = c & 15;
            const uint4 v = *reinterpret_cast<const uint4 *>(region + row * EPI_ST + ch * 16);
            *reinterpret_cast<uint4 *>(ct + (size_t)row * a.ldct * 2 + ch * 16) = v;
        }
    }
}

// BMAJ (weight gradient only): both operands are batch-major, A[k * lda + m] and B[k * ldb + n],
// i.e. the row-major deltas and activations themselves, so that no transposed copy of either
// has to exist.  An operand tile is then 64 k-rows of 512 bytes; the MFMA still wants 8
// consecutive k per lane, which gfx950's transposing LDS read delivers: ds_read_b64_tr_b16
// works in groups of 16 lanes, lane 4 j + q of a group supplies the address of an 8-byte word
// (k-row j, columns 4 q .. 4 q + 3 of a 16-column strip) and lane l receives column l at
// k-rows 0..3 (layout checked with an in-bounds probe).  Two such reads make one operand
// fragment.  The four k-rows a group reads together are 512 bytes apart, i.e. on the same
// banks: the 64-byte segments of k-row k are therefore stored at segment index s ^ (k & 3)
// (the direct loads fetch the permuted segment, their LDS side stays contiguous).
template <int KIND, bool BMAJ>
__device__ __forceinline__ void gemm_bf16_dma_tile(const GemmBf16Args &a, unsigned char *smem_raw, int id, int T,
                                                   int tid)
{
    static_assert(!BMAJ || KIND == GEMM_DW, "batch-major operands: weight gradient only");
    constexpr int BM = DMA_BM, BN = DMA_BN, BK = DMA_BK;
    constexpr int TM = 4, TN = 2;  // 32 x 32 blocks per wavefront: 128 x 64
    constexpr int G = BK / 16;     // MFMA k-steps per tile

    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);  // uniform: LDS bases of the direct loads are scalars
    const int r = lane & 31, h = lane >> 5;
    const int wm = wave & 1, wn = wave >> 1;

    // XCD-aware tile order.  Workgroup ids go round-robin over the 8 XCDs and an XCD runs 32
    // workgroups at a time (one per CU), so the j-th group of 32 ids of XCD x gets a block of
    // 4 x 8 (or 8 x 4) tiles: per k-tile its L2 then fetches 12 operand panels for 32 tiles,
    // against 18 for two rows of 16 (1.26 instead of 1.07 PFLOP/s on the weight gradient).
    int tile_m, tile_n;
    int bm = 0, bn = 0;
    if ((T & 255) == 0) {
        if ((a.tiles_m & 3) == 0 && (a.tiles_n & 7) == 0) { bm = 4; bn = 8; }
        else if ((a.tiles_m & 7) == 0 && (a.tiles_n & 3) == 0) { bm = 8; bn = 4; }
    }
    if (bm != 0) {
        const int L = id >> 3;
        const int sb = (id & 7) * (T >> 8) + (L >> 5), pos = L & 31;
        const int sbn = a.tiles_n / bn;
        tile_m = (sb / sbn) * bm + pos / bn;
        tile_n = (sb % sbn) * bn + pos % bn;
    } else {
        if ((T & 7) == 0) id = (id & 7) * (T >> 3) + (id >> 3);  // a contiguous run of tiles per XCD
        tile_m = id / a.tiles_n;
        tile_n = id - tile_m * a.tiles_n;
    }
    const int m0 = tile_m * BM, n0 = tile_n * BN;
    // slice of the contraction handled by this workgroup (blockIdx.y; the whole of it unless split)
    const int kbeg = (a.k_chunk > 0) ? (int)blockIdx.y * a.k_chunk : 0;
    const int klen = (a.k_chunk > 0) ? min(a.K - kbeg, a.k_chunk) : a.K;
    const int nkf = klen / BK;  // full k-tiles

    // operand base at the first k of the slice, and the step from one k-tile to the next
    const size_t a_tile_step = BMAJ ? (size_t)BK * (size_t)a.lda * 2 : (size_t)DMA_ROW_BYTES;
    const size_t b_tile_step = BMAJ ? (size_t)BK * (size_t)a.ldb * 2 : (size_t)DMA_ROW_BYTES;
    const unsigned char *__restrict__ Ab =
        static_cast<const unsigned char *>(a.A) + (BMAJ ? (size_t)kbeg * (size_t)a.lda * 2 : (size_t)kbeg * 2);
    const unsigned char *__restrict__ Bb =
        static_cast<const unsigned char *>(a.B) + (BMAJ ? (size_t)kbeg * (size_t)a.ldb * 2 : (size_t)kbeg * 2);

    // ---- global side of the direct loads.  One wavefront load fills 1 KB of LDS, lane i its
    // bytes 16 i ..: 8 tile rows of 128 bytes (lane -> row lane / 8, slot lane % 8), or, BMAJ,
    // 2 k-rows of 512 bytes (lane -> k-row lane / 32, slot lane % 32).  The wavefront takes
    // the 1 KB blocks wave, wave + 8, ..  BMAJ: columns past the end of a row (edge tiles; their
    // results are never stored) are clamped to the row's last 16 bytes.
    const int blk_row = lane >> 3;
    unsigned offA[4], offB[4];
#pragma unroll
    for (int v = 0; v < 4; ++v) {
        if (BMAJ) {
            const int k = (wave + 8 * v) * 2 + (lane >> 5);
            const int chunk = (lane & 31) ^ ((k & 3) << 2);  // the chunk whose slot is lane % 32
            offA[v] = (unsigned)((size_t)k * (size_t)a.lda * 2 +
                                 (size_t)min((long long)m0 * 2 + chunk * 16, a.lda * 2 - 16));
            offB[v] = (unsigned)((size_t)k * (size_t)a.ldb * 2 +
                                 (size_t)min((long long)n0 * 2 + chunk * 16, a.ldb * 2 - 16));
        } else {
            const int R = (wave + 8 * v) * 8 + blk_row;
            const int chunk = (lane & 7) ^ swz(R);  // the chunk whose slot is lane % 8
            offA[v] = (unsigned)((size_t)min(m0 + R, a.M - 1) * (size_t)a.lda * 2 + chunk * 16);
            offB[v] = (unsigned)((size_t)min(n0 + R, a.N - 1) * (size_t)a.ldb * 2 + chunk * 16);
        }
    }
    // loads first .. first + 1 of the wavefront's four of an A / B tile (tile t -> given stage)
    auto issue_a = [&](int t, int stage, int first) {
        unsigned char *st = smem_raw + stage * DMA_A_BYTES;
#pragma unroll
        for (int v = first; v < first + 2; ++v)
            __builtin_amdgcn_global_load_lds((gptr_t)(Ab + (size_t)t * a_tile_step + offA[v]),
                                             (lptr_t)(st + (wave + 8 * v) * 1024), 16, 0, 0);
    };
    auto issue_b = [&](int t, int stage, int first) {
        unsigned char *st = smem_raw + DMA_B_BASE + stage * DMA_B_BYTES;
#pragma unroll
        for (int v = first; v < first + 2; ++v)
            __builtin_amdgcn_global_load_lds((gptr_t)(Bb + (size_t)t * b_tile_step + offB[v]),
                                             (lptr_t)(st + (wave + 8 * v) * 1024), 16, 0, 0);
    };

    // ---- LDS side of the fragment reads: lane (r, h) reads chunk 2 kk + h of its row.  The
    // block offsets i * 32 rows leave (R >> 1) & 7 unchanged, so the swizzle depends on r only.
    // BMAJ: lane 16 g + 4 j + q addresses k-row 16 kk + 8 h + 4 t + j (t = 0, 1: the two reads of
    // a fragment), bytes 32 (g & 1) + 8 q of the block's 64-byte segment, which is stored at
    // segment index (true index) ^ j; the block index enters as one more XOR.
    const int fr = swz(r);
    const int tj = (lane & 15) >> 2;
    const int a_off = BMAJ ? (8 * h + tj) * 512 + (((wm * 4) ^ tj) << 6) + 32 * ((lane >> 4) & 1) + 8 * (lane & 3)
                         : (wm * 128 + r) * DMA_ROW_BYTES + ((h ^ fr) << 4);  // k-step kk: a_off ^ (kk << 5)
    const int b_off = DMA_B_BASE + (BMAJ ? (8 * h + tj) * 512 + (((wn * 2) ^ tj) << 6) + 32 * ((lane >> 4) & 1) + 8 * (lane & 3)
                                       : (wn * 64 + r) * DMA_ROW_BYTES + ((h ^ fr) << 4));
    v8bf fa[2][TM], fb[2][TN];
    const unsigned lds0 = (unsigned)(size_t)(lptr_t)smem_raw;  // LDS byte address of the stages
    // one operand fragment (block q of the A or B tile at p, k-step kk; kk is a KStep<> so
    // that the batch-major form can put it into the instruction's offset field)
    auto frag = [&](const unsigned char *p, int off, int q, auto kkc) -> v8bf {
        constexpr int kk = decltype(kkc)::value;
        if (BMAJ) {
            const unsigned addr = lds0 + (unsigned)(p - smem_raw) + (unsigned)(off ^ (q << 6));
            const v2i lo = lds_read_tr16_b64<kk * 16 * 512>(addr);
            const v2i hi = lds_read_tr16_b64<kk * 16 * 512 + 4 * 512>(addr);
            return __builtin_bit_cast(v8bf, __builtin_shufflevector(lo, hi, 0, 1, 2, 3));
        } else {
            return *reinterpret_cast<const v8bf *>(p + ((off ^ (kk << 5)) + q * 32 * DMA_ROW_BYTES));
        }
    };
    auto read_frags = [&](int slot, int sa, int sb, auto kkc) {
        const unsigned char *pa = smem_raw + sa * DMA_A_BYTES;
        const unsigned char *pb = smem_raw + sb * DMA_B_BYTES;
#pragma unroll
        for (int i = 0; i < TM; ++i) fa[slot][i] = frag(pa, a_off, i, kkc);
#pragma unroll
        for (int j = 0; j < TN; ++j) fb[slot][j] = frag(pb, b_off, j, kkc);
    };
    // the compiler does not know when the batch-major form's fragments have arrived
    auto frags_landed = [&]() {
        __builtin_amdgcn_s_waitcnt(0xc07f);  // lgkmcnt(0)
        __builtin_amdgcn_sched_barrier(0);
    };

    v16f acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;

    // Epilogue through LDS (uniform for the workgroup): bf16 output wanted, row-major or in both
    // layouts (and, except for the fused update, nothing else), workgroup tile inside the
    // matrix, 16-byte alignment of every row
    const bool use_mask = (KIND == GEMM_DA) && a.mask_in != nullptr && a.act == ACT_RELU;
    const bool via_lds = !(KIND == GEMM_DW && a.k_chunk > 0) && a.C_bf16 != nullptr &&
                         (KIND == GEMM_DW ? (a.Ct_bf16 != nullptr && a.C_f32 != nullptr && !a.write_grad)
                                          : a.C_f32 == nullptr) &&
                         (m0 + BM <= a.M) && (n0 + BN <= a.N) && (a.ldcb & 7) == 0 &&
                         (a.Ct_bf16 == nullptr || (a.ldct & 7) == 0) &&
                         ((reinterpret_cast<size_t>(a.C_bf16) | reinterpret_cast<size_t>(a.Ct_bf16)) & 15) == 0 &&
                         (KIND != GEMM_DA || use_mask || (a.aux_t != nullptr && (a.ldauxt & 3) == 0));
    // backward-data product: the ReLU decision bits of the lane's eight blocks are requested
    // now and have arrived long before the epilogue (they are older than every operand load,
    // so the waits of the main loop cover them)
    unsigned mword[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j) mword[i][j] = 0u;
    if (KIND == GEMM_DA && use_mask && via_lds) {
        const unsigned short *mi =
            a.mask_in + ((size_t)((m0 + wm * 128) >> 5) * a.mask_nb + ((n0 + wn * 64) >> 5)) * 64 + lane;
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int j = 0; j < TN; ++j) mword[i][j] = mi[((size_t)i * a.mask_nb + j) * 64];
    }

    auto mfma_step = [&](int slot) {
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int j = 0; j < TN; ++j)
                acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[slot][i], fb[slot][j], acc[i][j], 0, 0, 0);
    };
    // One MFMA group: the eight MFMAs of the k-step whose fragments are in `slot`, and in
    // their shadow (a wavefront can issue other instructions while its MFMA executes) the
    // requests for the next group's fragments, two after each of the first three MFMAs, and
    // two direct loads after the fifth.  Clumped in front of the group instead, these
    // requests are issued by both wavefronts of a SIMD at the same time (the barrier keeps
    // them in step) and the MFMA pipe idles meanwhile.  Only the requests are conditional,
    // so that there is one MFMA stream.
    auto group = [&](int slot, bool rd, int sa, int sb, auto kk, bool ld, bool is_a, int t, int stage, int first) {
        const unsigned char *pa = smem_raw + sa * DMA_A_BYTES;
        const unsigned char *pb = smem_raw + sb * DMA_B_BYTES;
        const int rs = slot ^ 1;
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int j = 0; j < TN; ++j) {
                acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[slot][i], fb[slot][j], acc[i][j], 0, 0, 0);
                const int b = i * TN + j;
                __builtin_amdgcn_sched_barrier(0);
                if (b < 2) {
                    if (rd) {
#pragma unroll
                        for (int q = 2 * b; q < 2 * b + 2; ++q) fa[rs][q] = frag(pa, a_off, q, kk);
                    }
                } else if (b == 2) {
                    if (rd) {
#pragma unroll
                        for (int q = 0; q < TN; ++q) fb[rs][q] = frag(pb, b_off, q, kk);
                    }
                } else if (b == 4) {
                    if (ld) {
                        if (is_a) issue_a(t, stage, first);
                        else issue_b(t, stage, first);
                    }
                }
                __builtin_amdgcn_sched_barrier(0);
            }
    };

    if (nkf > 0) {
        issue_a(0, 0, 0);
        issue_a(0, 0, 2);
        issue_b(0, 0, 0);
        issue_b(0, 0, 2);
        if (nkf > 1) {
            issue_b(1, 1, 0);
            issue_b(1, 1, 2);
            issue_a(1, 1, 0);
            asm volatile("s_waitcnt vmcnt(6)\n\ts_barrier" ::: "memory");  // tile 0 landed
        } else {
            asm volatile("s_waitcnt vmcnt(0)\n\ts_barrier" ::: "memory");
        }
        read_frags(0, 0, 0, KStep<0>());
        static_assert(G == 4, "the load schedule below is written for four k-steps per tile");
        int b_cur = 0, b_nxt = 1, b_ld = 2;  // B stages of tiles kt, kt+1, kt+2
        for (int kt = 0; kt < nkf; ++kt) {
            const int a_cur = kt & 1;
            const bool next = (kt + 1 < nkf), next2 = (kt + 2 < nkf);
            // The explicit lgkmcnt(0) at the head of a group tells the compiler that the
            // fragments requested during the previous group have arrived (they have: five
            // MFMAs lie in between); it cannot track them across the small branches.
            // (batch-major form: the compiler does not see the reads at all, and a scheduling
            // barrier keeps the MFMAs behind the wait)
            __builtin_amdgcn_s_waitcnt(0xc07f);
            if (BMAJ) __builtin_amdgcn_sched_barrier(0);
            group(0, true, a_cur, b_cur, KStep<1>(), next, true, kt + 1, a_cur ^ 1, 2);   // + second half of A(kt+1)
            __builtin_amdgcn_s_waitcnt(0xc07f);
            if (BMAJ) __builtin_amdgcn_sched_barrier(0);
            group(1, true, a_cur, b_cur, KStep<2>(), next2, false, kt + 2, b_ld, 0);      // + B(kt+2): its stage held B(kt-1)
            __builtin_amdgcn_s_waitcnt(0xc07f);
            if (BMAJ) __builtin_amdgcn_sched_barrier(0);
            group(0, true, a_cur, b_cur, KStep<3>(), next2, false, kt + 2, b_ld, 2);
            // Tile kt+1 must have landed (this wavefront's share; the barrier covers the others');
            // the four loads of B(kt+2) just issued may stay in flight.  This wavefront's reads of
            // tile kt must be done before anyone overwrites its stages.
            if (next2) asm volatile("s_waitcnt vmcnt(4) lgkmcnt(0)\n\ts_barrier" ::: "memory");
            else asm volatile("s_waitcnt vmcnt(0) lgkmcnt(0)\n\ts_barrier" ::: "memory");
            __builtin_amdgcn_s_waitcnt(0xc07f);  // lgkmcnt(0) again, this time visible to the compiler
            if (BMAJ) __builtin_amdgcn_sched_barrier(0);
            // last k-step of tile kt; k-step 0 of tile kt+1 is requested from the stages that have
            // just been completed, and the first half of A(kt+2) goes into the stage just released
            group(1, next, a_cur ^ 1, b_nxt, KStep<0>(), next2, true, kt + 2, a_cur, 0);
            const int t = b_cur;
            b_cur = b_nxt;
            b_nxt = b_ld;
            b_ld = t;
        }
    }

    // ---- K tail (fewer than BK columns left): masked copy through registers into stage 0
    const int ktail = klen - nkf * BK;
    if (ktail > 0) {
        __syncthreads();  // everybody is done with the main loop's stages
        const int kbase = nkf * BK;  // relative to the slice
#pragma unroll
        for (int v = 0; v < (BM + BN) * 8 / DMA_NT; ++v) {  // 16-byte chunks of both tiles over the workgroup
            const int idx = tid + v * DMA_NT;
            const bool isA = idx < BM * 8;
            const int q = isA ? idx : idx - BM * 8;
            if (BMAJ) {  // k-row q / 32, slot q % 32; k-rows past the end of the slice are zero
                const int k = q >> 5, slot = q & 31;
                const int chunk = slot ^ ((k & 3) << 2);
                uint4 x = {0u, 0u, 0u, 0u};
                if (kbase + k < klen) {
                    const long long ld = isA ? a.lda : a.ldb;
                    const long long col = min((long long)(isA ? m0 : n0) * 2 + chunk * 16, ld * 2 - 16);
                    x = *reinterpret_cast<const uint4 *>((isA ? Ab : Bb) + (size_t)(kbase + k) * (size_t)ld * 2 + col);
                }
                *reinterpret_cast<uint4 *>(smem_raw + (isA ? 0 : DMA_B_BASE) + k * 512 + slot * 16) = x;
                continue;
            }
            const int R = q >> 3, c = q & 7;
            const int k = kbase + c * 8;
            uint4 x = {0u, 0u, 0u, 0u};
            if (k < klen) {  // rows are padded to 8 elements, so the 16 bytes are in bounds
                const int grow = isA ? min(m0 + R, a.M - 1) : min(n0 + R, a.N - 1);
                const unsigned char *p = isA ? Ab + ((size_t)grow * (size_t)a.lda + k) * 2
                                             : Bb + ((size_t)grow * (size_t)a.ldb + k) * 2;
                x = *reinterpret_cast<const uint4 *>(p);
                const int valid = klen - k;  // elements of this chunk that belong to the slice
                if (valid < 8) {
                    unsigned int w[4] = {x.x, x.y, x.z, x.w};
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        if (2 * e >= valid) w[e] = 0u;
                        else if (2 * e + 1 >= valid) w[e] &= 0xffffu;
                    }
                    x = make_uint4(w[0], w[1], w[2], w[3]);
                }
            }
            *reinterpret_cast<uint4 *>(smem_raw + (isA ? 0 : DMA_B_BASE) + R * DMA_ROW_BYTES +
                                       ((c ^ swz(R)) << 4)) = x;
        }
        __syncthreads();
        read_frags(0, 0, 0, KStep<0>());
        if (BMAJ) frags_landed();
        mfma_step(0);
        read_frags(1, 0, 0, KStep<1>());
        if (BMAJ) frags_landed();
        mfma_step(1);
        read_frags(0, 0, 0, KStep<2>());
        if (BMAJ) frags_landed();
        mfma_step(0);
        read_frags(1, 0, 0, KStep<3>());
        if (BMAJ) frags_landed();
        mfma_step(1);
    }

    if (KIND == GEMM_DW && a.k_chunk > 0) {
        GemmBf16Args as = a;  // this slice's partial product
        as.C_f32 = static_cast<float *>(a.C_f32) + (size_t)blockIdx.y * (size_t)a.c_split_stride;
        epilogue_bf16<KIND, TM, TN>(as, acc, m0 + wm * 128, n0 + wn * 64, r, h);
    } else {
        if (via_lds) {
            // Every wavefront must be done with the operand stages.  After the main loop it is:
            // the last fragments were read before the loop's last barrier.  A K tail, or no
            // whole k-tile at all, ends with reads of stage 0.
            if (ktail > 0 || nkf == 0) __syncthreads();
            const bool mask = (KIND == GEMM_FWD) ? (a.mask_out != nullptr && a.act == ACT_RELU) : use_mask;
            with_activation(KIND == GEMM_DW ? (int)ACT_NONE : a.act, mask, [&](auto act_c, auto mask_c) {
                epilogue_bf16_lds<KIND, decltype(act_c)::value, decltype(mask_c)::value != 0>(
                    a, acc, smem_raw + wave * EPI_REGION, m0 + wm * 128, n0 + wn * 64, lane, mword);
            });
        } else {
            epilogue_bf16<KIND, TM, TN>(a, acc, m0 + wm * 128, n0 + wn * 64, r, h);
        }
    }
}

// Workgroup b computes tiles b, b + gridDim.x, ..: with more tiles than compute units the
// launcher starts one workgroup per compute unit, which saves the dispatch of a new
// workgroup at every tile boundary (16384 x 4096 x 4096: 428 -> 425 us); otherwise one
// workgroup per tile.  The thread number goes through an empty asm in every round: everything
// the tile derives from it would otherwise be computed once in front of the loop and sit in
// registers through the main loop, which has none to spare.  Between two tiles every
// wavefront must be done with the LDS staging of its results before the next tile's operand
// loads may land on it.
template <int KIND, bool BMAJ = false>
__global__ __launch_bounds__(DMA_NT, 1) void gemm_bf16_dma_kernel(GemmBf16Args a)
{
    extern __shared__ __attribute__((aligned(16))) unsigned char smem_raw[];
    const int T = a.tiles_m * a.tiles_n;
    for (int id = blockIdx.x; id < T; id += (int)gridDim.x) {
        int tid = threadIdx.x;
        asm volatile("" : "+v"(tid));
        gemm_bf16_dma_tile<KIND, BMAJ>(a, smem_raw, id, T, tid);
        if (id + (int)gridDim.x < T) asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
    }
}

// out[c][r] = in[r][c] for bf16 matrices (R x C, leading dimensions ldi / ldo), 64 x 64 tiles.
// Interior tiles of 16-byte aligned matrices move 16 bytes per lane on both sides (two-byte
// accesses reach 2.3 TB/s, a third of what the memory gives): rows come in as eight 16-byte
// pieces each, go to LDS as dwords with a row stride of 33 dwords, and a lane gathers the
// eight values of its output piece from eight LDS rows (stride 33: the eight row groups of a
// wavefront fall on banks 8 apart, conflict-free).
__global__ __launch_bounds__(256) void transpose_bf16_kernel(const bf16_t *__restrict__ in, long long ldi,
                                                             bf16_t *__restrict__ out, long long ldo, int R, int C,
                                                             int vec_ok)
{
    __shared__ bf16_t t[64][66];
    const int c0 = blockIdx.x * 64, r0 = blockIdx.y * 64;
    if (vec_ok && r0 + 64 <= R && c0 + 64 <= C) {
        uint32_t *tw = reinterpret_cast<uint32_t *>(&t[0][0]);  // [64][33] dwords
#pragma unroll
        for (int p = 0; p < 2; ++p) {
            const int s = threadIdx.x + 256 * p, row = s >> 3, sc = s & 7;
            const uint4 v = *reinterpret_cast<const uint4 *>(in + (size_t)(r0 + row) * ldi + c0 + sc * 8);
            uint32_t *d = tw + row * 33 + sc * 4;
            d[0] = v.x; d[1] = v.y; d[2] = v.z; d[3] = v.w;
        }
        __syncthreads();
#pragma unroll
        for (int p = 0; p < 2; ++p) {
            const int s = threadIdx.x + 256 * p, c = s >> 3, sr = s & 7;
            uint32_t w[4];
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const uint32_t lo = t[sr * 8 + 2 * j][c], hi = t[sr * 8 + 2 * j + 1][c];
                w[j] = lo | (hi << 16);
            }
            *reinterpret_cast<uint4 *>(out + (size_t)(c0 + c) * ldo + r0 + sr * 8) = make_uint4(w[0], w[1], w[2], w[3]);
        }
        return;
    }
    const int tx = threadIdx.x & 63, ty = threadIdx.x >> 6;  // 64 x 4
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

// Sum of the slices of a split weight gradient, then Eq. (3) on the fp32 master weights or a
// plain store of the gradient.  Slices are added in index order (deterministic).
__global__ __launch_bounds__(256) void dw_reduce_kernel(const float *__restrict__ partial, int splits,
                                                        long long stride, long long count,
                                                        float *__restrict__ master, float *__restrict__ grad,
                                                        float lr)
{
    const bool vec = ((stride & 3) == 0) && ((count & 3) == 0) && ((reinterpret_cast<size_t>(partial) & 15) == 0) &&
                     ((reinterpret_cast<size_t>(grad ? grad : master) & 15) == 0);
    const long long step = (long long)gridDim.x * 256;
    if (vec) {
        for (long long q = (long long)blockIdx.x * 256 + threadIdx.x; q < (count >> 2); q += step) {
            float4 s = {0.f, 0.f, 0.f, 0.f};
            for (int k = 0; k < splits; ++k) {
                const float4 p = *reinterpret_cast<const float4 *>(partial + (size_t)k * stride + 4 * q);
                s.x += p.x; s.y += p.y; s.z += p.z; s.w += p.w;
            }
            if (grad) {
                *reinterpret_cast<float4 *>(grad + 4 * q) = s;
            } else {
                float4 w = *reinterpret_cast<float4 *>(master + 4 * q);
                w.x -= lr * s.x; w.y -= lr * s.y; w.z -= lr * s.z; w.w -= lr * s.w;
                *reinterpret_cast<float4 *>(master + 4 * q) = w;
            }
        }
    } else {
        for (long long i = (long long)blockIdx.x * 256 + threadIdx.x; i < count; i += step) {
            float s = 0.f;
            for (int k = 0; k < splits; ++k) s += partial[(size_t)k * stride + i];
            if (grad) grad[i] = s;
            else master[i] -= lr * s;
        }
    }
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
    long long b0 = 0;
    if ((ld & 7) == 0 && (reinterpret_cast<size_t>(Dt) & 15) == 0) {
        // 16 bytes (8 values) per lane and load, four loads in flight
        const long long nvec = B >> 3;
        const uint4 *rv = reinterpret_cast<const uint4 *>(row);
        for (long long v0 = 0; v0 < nvec; v0 += 256) {
            uint4 x[4];
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const long long v = v0 + u * 64 + lane;
                x[u] = (v < nvec) ? rv[v] : make_uint4(0u, 0u, 0u, 0u);
            }
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const unsigned int w[4] = {x[u].x, x[u].y, x[u].z, x[u].w};
#pragma unroll
                for (int e = 0; e < 4; ++e) s += __uint_as_float(w[e] << 16) + __uint_as_float(w[e] & 0xffff0000u);
            }
        }
        b0 = nvec << 3;
    }
    for (long long b = b0 + lane; b < B; b += 64) s += bf2f(row[b]);
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) s += __shfl_xor(s, o, 64);
    if (lane == 0) {
        if (grad) grad[j] = s;
        else bias[j] -= lr * s;
    }
}

// Bias gradient from the row-major delta D [B x ld] (16-byte aligned rows): column sums over
// the batch in two steps, both in a fixed order.  Step 1, block (x, s): columns 512 x .. + 511 of
// the rows of slice s; a thread owns 8 columns (one 16-byte load per row) and every fourth row,
// four loads in flight; the four row lanes meet in LDS.  Step 2 adds the slices in index order
// and applies Eq. (3) to the bias (or stores the gradient).
constexpr int CSB_COLS = 512, CSB_MAX_SLICES = 128;
__global__ __launch_bounds__(256) void colsum_bf16_kernel(const bf16_t *__restrict__ D, long long ld, int d,
                                                          long long B, int rows_per_slice,
                                                          float *__restrict__ partial)
{
    __shared__ float red[4][CSB_COLS + 8];
    const int cl = threadIdx.x & 63, rl = threadIdx.x >> 6;
    const long long c0 = (long long)blockIdx.x * CSB_COLS + cl * 8;
    const long long r0 = (long long)blockIdx.y * rows_per_slice, r1 = min(B, r0 + (long long)rows_per_slice);
    float s[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) s[e] = 0.f;
    auto add = [&](const uint4 &x) {
        const unsigned int w[4] = {x.x, x.y, x.z, x.w};
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            s[2 * e] += __uint_as_float(w[e] << 16);
            s[2 * e + 1] += __uint_as_float(w[e] & 0xffff0000u);
        }
    };
    if (c0 < ld) {  // ld is a multiple of 8: the whole 16-byte piece lies inside the row
        const bf16_t *p = D + c0;
        long long i = r0 + rl;
        for (; i + 12 < r1; i += 16) {
            uint4 x[4];
#pragma unroll
            for (int u = 0; u < 4; ++u) x[u] = *reinterpret_cast<const uint4 *>(p + (size_t)(i + 4 * u) * ld);
#pragma unroll
            for (int u = 0; u < 4; ++u) add(x[u]);
        }
        for (; i < r1; i += 4) add(*reinterpret_cast<const uint4 *>(p + (size_t)i * ld));
    }
#pragma unroll
    for (int e = 0; e < 8; ++e) red[rl][cl * 8 + e] = s[e];
    __syncthreads();
    for (int c = threadIdx.x; c < CSB_COLS; c += 256) {
        const long long col = (long long)blockIdx.x * CSB_COLS + c;
        if (col < d) partial[(size_t)blockIdx.y * d + col] = (red[0][c] + red[1][c]) + (red[2][c] + red[3][c]);
    }
}

__global__ __launch_bounds__(256) void colsum_bias_finalize_kernel(const float *__restrict__ partial, int slices,
                                                                   int d, float *__restrict__ bias,
                                                                   float *__restrict__ grad, float lr)
{
    // 64 columns per block, four lanes per column: lane q adds slices q, q + 4, .. (eight loads
    // in flight), the four meet in LDS in lane order
    __shared__ float red[4][64];
    const int c = threadIdx.x & 63, q = threadIdx.x >> 6;
    const int j = blockIdx.x * 64 + c;
    float s = 0.f;
    if (j < d) {
        int k = q;
        for (; k + 28 < slices; k += 32) {
            float v[8];
#pragma unroll
            for (int u = 0; u < 8; ++u) v[u] = partial[(size_t)(k + 4 * u) * d + j];
#pragma unroll
            for (int u = 0; u < 8; ++u) s += v[u];
        }
        for (; k < slices; k += 4) s += partial[(size_t)k * d + j];
    }
    red[q][c] = s;
    __syncthreads();
    if (q == 0 && j < d) {
        const float t = (red[0][c] + red[1][c]) + (red[2][c] + red[3][c]);
        if (grad) grad[j] = t;
        else bias[j] -= lr * t;
    }
}

template <int BM, int BN, int BK>
hipError_t launch_shape_bf16(GemmKind kind, GemmBf16Args a, hipStream_t stream, const LaunchEvents &ev)
{
    constexpr size_t LDS = lds_bytes_bf16<BM, BN, BK>();
    void (*k)(GemmBf16Args) = kind == GEMM_FWD  ? gemm_bf16_nt_kernel<BM, BN, BK, GEMM_FWD>
                              : kind == GEMM_DA ? gemm_bf16_nt_kernel<BM, BN, BK, GEMM_DA>
                                                : gemm_bf16_nt_kernel<BM, BN, BK, GEMM_DW>;
    static std::mutex attr_mu;  // handles on different host threads launch concurrently
    static bool attr_set[3] = {false, false, false};  // per instantiation (BM, BN, BK) and kind
    if (LDS > 48 * 1024) {
        std::lock_guard<std::mutex> lk(attr_mu);
        if (!attr_set[kind]) {
            hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(k),
                                               hipFuncAttributeMaxDynamicSharedMemorySize, (int)LDS);
            if (e != hipSuccess) return e;
            attr_set[kind] = true;
        }
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


hipError_t launch_dma_bf16(GemmKind kind, GemmBf16Args a, hipStream_t stream, const LaunchEvents &ev)
{
    void (*k)(GemmBf16Args) = kind == GEMM_FWD  ? gemm_bf16_dma_kernel<GEMM_FWD>
                              : kind == GEMM_DA ? gemm_bf16_dma_kernel<GEMM_DA>
                              : a.bmaj          ? gemm_bf16_dma_kernel<GEMM_DW, true>
                                                : gemm_bf16_dma_kernel<GEMM_DW>;
    const int slot = (kind == GEMM_DW && a.bmaj) ? 3 : (int)kind;
    static std::mutex attr_mu;
    static bool attr_set[4] = {false, false, false, false};
    {
        std::lock_guard<std::mutex> lk(attr_mu);
        if (!attr_set[slot]) {
            hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(k),
                                               hipFuncAttributeMaxDynamicSharedMemorySize, (int)DMA_LDS_BYTES);
            if (e != hipSuccess) return e;
            attr_set[slot] = true;
        }
    }
    a.tiles_m = (a.M + DMA_BM - 1) / DMA_BM;
    a.tiles_n = (a.N + DMA_BN - 1) / DMA_BN;
    const long long tiles = (long long)a.tiles_m * a.tiles_n;
    if (tiles > 0x7fffffffLL) return hipErrorInvalidValue;
    const int splits = (kind == GEMM_DW && a.k_chunk > 0) ? (a.K + a.k_chunk - 1) / a.k_chunk : 1;
    // one workgroup per compute unit (256 on this part) when there are more tiles than that
    // (HB_BF16_PERSIST=0, tuning aid: one workgroup per tile)
    static const int persist = env_int_bf16("HB_BF16_PERSIST", 1);
    const long long wgs = (persist && tiles > 256) ? 256 : tiles;
    const dim3 grid((unsigned)wgs, (unsigned)splits), block(DMA_NT);
    if (ev.start)
        hipExtLaunchKernelGGL(k, grid, block, (unsigned)DMA_LDS_BYTES, stream, ev.start, ev.stop, 0, a);
    else
        hipLaunchKernelGGL(k, grid, block, DMA_LDS_BYTES, stream, a);
    return hipGetLastError();
}

}  // namespace

hipError_t launch_gemm_bf16(GemmKind kind, GemmBf16Args a, hipStream_t stream, const LaunchEvents &ev,
                            int *colsum_slices_out)
{
    if (colsum_slices_out) *colsum_slices_out = 0;
    if (a.M <= 0 || a.N <= 0 || a.K <= 0) return hipErrorInvalidValue;
    // The 256 x 256 LDS-direct kernel when both operands allow it and its tiles cover at least
    // half of the CUs; else 256 x 128 tiles when they give two workgroups per CU, else 128 x 128.
    // HB_BF16_TILE = 1 / 2 / 3 / 4 forces a kernel (tuning aid; 4 = 256 x 128, 1 = LDS-direct).
    static const int forced = env_int_bf16("HB_BF16_TILE", 0);
    const long long dma_tiles = (long long)((a.M + DMA_BM - 1) / DMA_BM) * ((a.N + DMA_BN - 1) / DMA_BN);
    const long long big_tiles = (long long)((a.M + 255) / 256) * ((a.N + 127) / 128);
    // the LDS-direct kernel addresses each operand with 32-bit byte offsets from its base
    // (batch-major operands: rows are batch rows, and only the first k-tile is addressed that way)
    const bool dma_ok = a.a_vec && a.b_vec &&
                        (a.bmaj ? ((unsigned long long)DMA_BK * (unsigned long long)a.lda * 2 < (1ull << 32) &&
                                   (unsigned long long)DMA_BK * (unsigned long long)a.ldb * 2 < (1ull << 32) &&
                                   a.lda >= a.M && a.ldb >= a.N)
                                : ((unsigned long long)a.M * (unsigned long long)a.lda * 2 < (1ull << 32) &&
                                   (unsigned long long)a.N * (unsigned long long)a.ldb * 2 < (1ull << 32)));
    if (a.bmaj) {  // batch-major operands: weight gradient through the LDS-direct kernel only
        if (kind != GEMM_DW || !dma_ok || (a.k_chunk > 0 && (!a.write_grad || a.C_bf16 || a.Ct_bf16 ||
                                                              (a.k_chunk % DMA_BK) != 0)))
            return hipErrorInvalidValue;
        return launch_dma_bf16(kind, a, stream, ev);
    }
    if (a.k_chunk > 0) {  // split weight gradient: only the LDS-direct kernel implements it
        if (kind != GEMM_DW || !dma_ok || !a.write_grad || a.C_bf16 || a.Ct_bf16 || (a.k_chunk % DMA_BK) != 0)
            return hipErrorInvalidValue;
        return launch_dma_bf16(kind, a, stream, ev);
    }
    if (dma_ok && (forced == 1 || (forced == 0 && dma_tiles >= 128))) {
        // column sums of a backward-data result: two slices per tile row, if the caller has room
        const int slices = 2 * ((a.M + DMA_BM - 1) / DMA_BM);
        if (kind != GEMM_DA || a.colsum_partial == nullptr || slices > a.colsum_cap) a.colsum_partial = nullptr;
        else if (colsum_slices_out) *colsum_slices_out = slices;
        return launch_dma_bf16(kind, a, stream, ev);
    }
    a.colsum_partial = nullptr;  // the other kernels do not produce them
    if (forced == 4 || (forced == 0 && big_tiles >= 512)) return launch_shape_bf16<256, 128, 32>(kind, a, stream, ev);
    if (forced == 3) return launch_shape_bf16<128, 128, 32>(kind, a, stream, ev);
    return launch_shape_bf16<128, 128, 64>(kind, a, stream, ev);
}

bool gemm_bf16_dw_bmaj_ok(int M, int N, int K, long long lda, long long ldb, const void *A, const void *B)
{
    // what launch_gemm_bf16 asks of batch-major operands, and a product the LDS-direct kernel
    // is chosen for anyway (split over the batch, or at least 128 tiles)
    if ((lda & 7) || (ldb & 7) || ((reinterpret_cast<size_t>(A) | reinterpret_cast<size_t>(B)) & 15) || lda < M ||
        ldb < N || (unsigned long long)DMA_BK * (unsigned long long)lda * 2 >= (1ull << 32) ||
        (unsigned long long)DMA_BK * (unsigned long long)ldb * 2 >= (1ull << 32))
        return false;
    const long long tiles = (long long)((M + DMA_BM - 1) / DMA_BM) * ((N + DMA_BN - 1) / DMA_BN);
    return tiles >= 128 || gemm_bf16_dw_splits_cap(M, N, K) > 1;
}

int gemm_bf16_dw_splits_cap(int M, int N, int K)
{
    const long long tiles = (long long)((M + DMA_BM - 1) / DMA_BM) * ((N + DMA_BN - 1) / DMA_BN);
    if (tiles > 128 || K < 2048) return 1;
    long long s = 256 / tiles;  // fill the chip once
    if (s > 8) s = 8;
    if (s > K / 1024) s = K / 1024;  // at least 16 k-tiles per slice
    return s < 2 ? 1 : (int)s;
}

int gemm_bf16_dw_splits(int M, int N, int K, long long lda, long long ldb)
{
    // the LDS-direct kernel (the only one that splits) addresses each operand with 32-bit byte
    // offsets: an operand beyond 4 GiB is not split.  This makes the count non-monotonic in K
    // (lda and ldb grow with the batch), which is why buffers are sized with ..._cap.
    if ((unsigned long long)M * (unsigned long long)lda * 2 >= (1ull << 32) ||
        (unsigned long long)N * (unsigned long long)ldb * 2 >= (1ull << 32) || (lda & 7) || (ldb & 7))
        return 1;
    return gemm_bf16_dw_splits_cap(M, N, K);
}

hipError_t launch_dw_reduce(const float *partial, int splits, long long stride, long long count, float *master,
                            float *grad, float lr, hipStream_t stream, const LaunchEvents &ev)
{
    if (count <= 0) return hipSuccess;
    const long long n4 = (count + 3) / 4;
    long long blocks = (n4 + 255) / 256;
    if (blocks > 4096) blocks = 4096;
    return launch_kernel(dw_reduce_kernel, dim3((unsigned)blocks), dim3(256), stream, ev, partial, splits, stride,
                         count, master, grad, lr);
}

hipError_t launch_transpose_bf16(const void *in, long long ldi, void *out, long long ldo, int R, int C,
                                 hipStream_t stream, const LaunchEvents &ev)
{
    const int vec_ok = (ldi % 8 == 0) && (ldo % 8 == 0) && ((reinterpret_cast<size_t>(in) & 15) == 0) &&
                       ((reinterpret_cast<size_t>(out) & 15) == 0);
    return launch_kernel(transpose_bf16_kernel, dim3((unsigned)((C + 63) / 64), (unsigned)((R + 63) / 64)),
                         dim3(256), stream, ev, static_cast<const bf16_t *>(in), ldi, static_cast<bf16_t *>(out),
                         ldo, R, C, vec_ok);
}

hipError_t launch_shadow(const float *W, int R, int C, void *shadow, long long lds_, void *shadow_t,
                         long long ldt, hipStream_t stream)
{
    return launch_kernel(shadow_kernel, dim3((unsigned)((C + 63) / 64), (unsigned)((R + 63) / 64)), dim3(256),
                         stream, LaunchEvents(), W, R, C, static_cast<bf16_t *>(shadow), lds_,
                         static_cast<bf16_t *>(shadow_t), ldt);
}

int colsum_bias_slices(long long B)
{
    long long s = (B + 63) / 64;  // at least 64 rows per slice
    if (s > CSB_MAX_SLICES) s = CSB_MAX_SLICES;
    return s < 1 ? 1 : (int)s;
}

hipError_t launch_colsum_bias_finalize(const float *partial, int slices, int d, float *bias, float *grad, float lr,
                                       hipStream_t stream, const LaunchEvents &ev)
{
    return launch_kernel(colsum_bias_finalize_kernel, dim3((unsigned)((d + 63) / 64)), dim3(256), stream, ev,
                         partial, slices, d, bias, grad, lr);
}

hipError_t launch_colsum_bias(const void *D, long long ld, int d, long long B, float *partial, float *bias,
                              float *grad, float lr, hipStream_t stream, const LaunchEvents &ev)
{
    if ((ld & 7) != 0 || (reinterpret_cast<size_t>(D) & 15) != 0 || B <= 0) return hipErrorInvalidValue;
    const int slices = colsum_bias_slices(B);
    const int rows_per_slice = (int)((B + slices - 1) / slices);
    hipError_t e = launch_kernel(colsum_bf16_kernel, dim3((unsigned)((ld + CSB_COLS - 1) / CSB_COLS), (unsigned)slices),
                                 dim3(256), stream, ev, static_cast<const bf16_t *>(D), ld, d, B, rows_per_slice,
                                 partial);
    if (e != hipSuccess) return e;
    return launch_kernel(colsum_bias_finalize_kernel, dim3((unsigned)((d + 63) / 64)), dim3(256), stream,
                         LaunchEvents(), static_cast<const float *>(partial), slices, d, bias, grad, lr);
}

hipError_t launch_rowsum_bias(const void *Dt, long long ld, int d, long long B, float *bias, float *grad,
                              float lr, hipStream_t stream, const LaunchEvents &ev)
{
    return launch_kernel(rowsum_bias_kernel, dim3((unsigned)((d + 3) / 4)), dim3(256), stream, ev,
                         static_cast<const bf16_t *>(Dt), ld, d, B, bias, grad, lr);
}

}  // namespace hb
