// fp32 MFMA GEMM for the three dense layer products of the mini-batch step
// (Section 3 of the paper: forward Eq. (1), backward Eq. (2); on a batch the
// matrix-vector products become matrix-matrix products, the dominant cost).
//
// gfx950 design: 256-thread workgroups (4 wavefronts of 64), v_mfma_f32_32x32x2_f32
// blocks, operands staged global -> registers -> LDS with a double-buffered LDS tile:
// global loads run two k-tiles ahead, the next tile is written to the idle LDS stage
// early in the current tile, fragments are read one MFMA step ahead, one barrier per tile.
// K-major operands are read from LDS as 16-byte vectors along k (the k index is permuted
// identically for both operands, which leaves the contraction unchanged); M-major
// operands are read one float per lane with the 32 rows of a block on consecutive
// addresses.  Epilogues fuse bias + activation (forward), the activation derivative
// (backward-data) and the bias-gradient column sums (weight gradient); interior tiles take
// a form without guards that requests everything it reads in one batch.  Products with few
// output tiles (small batches) run a second kernel family further down: 32 x 32 tiles with
// the contraction split over the four wavefronts of a workgroup.
#include "hb_internal.h"

#include <stdlib.h>

#include <type_traits>

namespace hb {
namespace {

typedef float v16f __attribute__((ext_vector_type(16)));
typedef float v4f __attribute__((ext_vector_type(4)));

constexpr int NT = 256;  // threads per workgroup

template <int ROWS, int BK, bool KMAJ>
struct Tile {
    static_assert(ROWS % 32 == 0 && BK % 8 == 0, "tile shape");
    static constexpr int LD = KMAJ ? (BK + 4) : (ROWS + 8);
    static constexpr int FLOATS = KMAJ ? ROWS * LD : BK * LD;
    static constexpr int VECS = ROWS * BK / 4;
    static constexpr int VPT = (VECS + NT - 1) / NT;

    // global -> registers; everything outside [0,nrows) x [.., kend) reads as zero
    static __device__ __forceinline__ void load(v4f (&reg)[VPT], const float *__restrict__ P,
                                                int ld, int row0, int nrows, int k0, int kend,
                                                bool vec, int tid)
    {
#pragma unroll
        for (int v = 0; v < VPT; ++v) {
            const int idx = tid + v * NT;
            v4f x = {0.f, 0.f, 0.f, 0.f};
            if (VECS % NT == 0 || idx < VECS) {
                if (KMAJ) {
                    const int kq = idx % (BK / 4), r = idx / (BK / 4);
                    const int row = row0 + r, k = k0 + kq * 4;
                    if (row < nrows && k < kend) {
                        const float *p = P + (size_t)row * ld + k;
                        if (vec && k + 4 <= kend) {
                            x = *reinterpret_cast<const v4f *>(p);
                        } else {
                            x.x = p[0];
                            if (k + 1 < kend) x.y = p[1];
                            if (k + 2 < kend) x.z = p[2];
                            if (k + 3 < kend) x.w = p[3];
                        }
                    }
                } else {
                    const int mq = idx % (ROWS / 4), kk = idx / (ROWS / 4);
                    const int row = row0 + mq * 4, k = k0 + kk;
                    if (k < kend && row < nrows) {
                        const float *p = P + (size_t)k * ld + row;
                        if (vec && row + 4 <= nrows) {
                            x = *reinterpret_cast<const v4f *>(p);
                        } else {
                            x.x = p[0];
                            if (row + 1 < nrows) x.y = p[1];
                            if (row + 2 < nrows) x.z = p[2];
                            if (row + 3 < nrows) x.w = p[3];
                        }
                    }
                }
            }
            reg[v] = x;
        }
    }

    // The same tile without any guard: legal when the tile lies inside the matrix in both
    // directions.  vec: 16-byte loads, else four 4-byte loads (rows that are not 16-byte
    // aligned, e.g. the caller's X with d_0 = 54).
    static __device__ __forceinline__ void load_fast(v4f (&reg)[VPT], const float *__restrict__ P,
                                                     int ld, int row0, int k0, bool vec, int tid)
    {
#pragma unroll
        for (int v = 0; v < VPT; ++v) {
            const int idx = tid + v * NT;
            if (VECS % NT == 0 || idx < VECS) {
                const float *p;
                if (KMAJ) {
                    const int kq = idx % (BK / 4), r = idx / (BK / 4);
                    p = P + (size_t)(row0 + r) * ld + k0 + kq * 4;
                } else {
                    const int mq = idx % (ROWS / 4), kk = idx / (ROWS / 4);
                    p = P + (size_t)(k0 + kk) * ld + row0 + mq * 4;
                }
                if (vec) {
                    reg[v] = *reinterpret_cast<const v4f *>(p);
                } else {
                    v4f x;
                    x.x = p[0];
                    x.y = p[1];
                    x.z = p[2];
                    x.w = p[3];
                    reg[v] = x;
                }
            }
        }
    }

    // registers -> LDS (same element <-> thread mapping as load)
    static __device__ __forceinline__ void store(float *S, const v4f (&reg)[VPT], int tid)
    {
#pragma unroll
        for (int v = 0; v < VPT; ++v) {
            const int idx = tid + v * NT;
            if (VECS % NT == 0 || idx < VECS) {
                if (KMAJ) {
                    const int kq = idx % (BK / 4), r = idx / (BK / 4);
                    *reinterpret_cast<v4f *>(&S[r * LD + kq * 4]) = reg[v];
                } else {
                    const int mq = idx % (ROWS / 4), kk = idx / (ROWS / 4);
                    *reinterpret_cast<v4f *>(&S[kk * LD + mq * 4]) = reg[v];
                }
            }
        }
    }

    // The four operand values of tile row `row` for the MFMA steps of k-group g:
    // f[j] = element(row, k = 8 g + 4 h + j), h = lane / 32.
    static __device__ __forceinline__ v4f frag(const float *S, int row, int g, int h)
    {
        if (KMAJ) {
            return *reinterpret_cast<const v4f *>(&S[row * LD + g * 8 + h * 4]);
        } else {
            const float *p = &S[(g * 8 + h * 4) * LD + row];
            v4f f;
            f.x = p[0];
            f.y = p[LD];
            f.z = p[2 * LD];
            f.w = p[3 * LD];
            return f;
        }
    }
};

__device__ __forceinline__ float sigmoidf_fast(float z)
{
    return __builtin_amdgcn_rcpf(1.0f + __expf(-z));  // v_rcp_f32: 1 ulp, no division sequence
}

template <int V>
struct IntC {
    static constexpr int value = V;
};
// calls f(IntC<activation>) with the run-time activation as a constant
template <typename F>
__device__ __forceinline__ void with_activation(int act, F &&f)
{
    if (act == ACT_SIGMOID) f(IntC<ACT_SIGMOID>());
    else if (act == ACT_RELU) f(IntC<ACT_RELU>());
    else f(IntC<ACT_NONE>());
}

// LDS floats one workgroup of this shape needs (two stages of an A and a B tile)
template <int BM, int BN, int BK, bool A_KMAJ, bool B_KMAJ>
constexpr int lds_floats()
{
    return 2 * (Tile<BM, BK, A_KMAJ>::FLOATS + Tile<BN, BK, B_KMAJ>::FLOATS);
}

// XCD-aware tile order: consecutive hardware workgroup ids go round-robin over the 8 XCDs,
// so give each XCD a contiguous run of the T tiles (they share an A row panel in its L2).
__device__ __forceinline__ int xcd_tile_order(int b, int T)
{
    return ((T & 7) == 0) ? (b & 7) * (T >> 3) + (b >> 3) : b;
}

// One output tile (index id in n-fastest order) of one K-slice (split) of C = A . B^T.
template <int BM, int BN, int BK, int WAVES_M, bool A_KMAJ, bool B_KMAJ, int KIND>
__device__ __forceinline__ void gemm_f32_tile(const GemmArgs &a, float *smem, int id, int split)
{
    constexpr int WAVES_N = 4 / WAVES_M;
    constexpr int WM = BM / WAVES_M, WN = BN / WAVES_N;
    constexpr int TM = WM / 32, TN = WN / 32;
    static_assert(TM >= 1 && TN >= 1 && WM % 32 == 0 && WN % 32 == 0, "wave tile");
    using TA = Tile<BM, BK, A_KMAJ>;
    using TB = Tile<BN, BK, B_KMAJ>;
    constexpr int STAGE = TA::FLOATS + TB::FLOATS;

    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int r = lane & 31, h = lane >> 5;
    const int wm = wave % WAVES_M, wn = wave / WAVES_M;

    const int tile_m = id / a.tiles_n, tile_n = id - tile_m * a.tiles_n;
    const int m0 = tile_m * BM, n0 = tile_n * BN;
    const int kbeg = split * a.k_chunk;
    const int kend = min(a.K, kbeg + a.k_chunk);
    const int nk = (kend - kbeg + BK - 1) / BK;

    const float *__restrict__ A = static_cast<const float *>(a.A);
    const float *__restrict__ Bm = static_cast<const float *>(a.B);

    // With a single 32 x 32 block per wavefront every MFMA would depend on the one before
    // it; two accumulators per block, fed by alternating k-groups, give two independent chains.
    constexpr int CHAINS = (TM * TN == 1) ? 2 : 1;
    v16f acc[TM][TN][CHAINS];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int c = 0; c < CHAINS; ++c)
#pragma unroll
                for (int v = 0; v < 16; ++v) acc[i][j][c][v] = 0.f;

    // tiles that lie inside the matrix are loaded without guards (uniform per workgroup)
    const bool a_in = (m0 + BM <= a.M), b_in = (n0 + BN <= a.N);

    // DW only: column sums of the A tile (the bias gradient), by the blocks of the first tile
    // column.  All threads share the work: thread (crow, cpart) adds every CP-th k of row crow,
    // the CP partial sums meet in LDS after the loop (one wavefront alone did 32 LDS reads per
    // k-tile in front of its MFMAs, and its workgroup waited for it at every barrier: the paired
    // launch at B = 4096 42.4 -> 42.0 us).
    constexpr int CP = NT / BM;
    const int crow = tid % BM, cpart = tid / BM;
    float colsum = 0.f;
    const bool do_colsum = (KIND == GEMM_DW) && a.colsum != nullptr && tile_n == 0;

    // forward: the lane's bias values are requested now, not after the main loop
    float bias_pre[TN];
#pragma unroll
    for (int j = 0; j < TN; ++j) {
        const int n = n0 + wn * WN + j * 32 + r;
        bias_pre[j] = (KIND == GEMM_FWD && a.bias != nullptr && n < a.N) ? a.bias[n] : 0.f;
    }

    // Software pipeline, three levels deep:
    //   global -> registers : the loads of tile kt+2 are issued at the top of iteration kt
    //   registers -> LDS    : just before that, tile kt+1 (loaded during iteration kt-1) is
    //                         written to the idle LDS stage, long before anyone needs it
    //   LDS -> fragments    : the fragments of k-group g+1 are read while the MFMAs of group g
    //                         run; the first group of tile kt+1 is read right after the
    //                         barrier, under the last MFMAs of tile kt.
    // One barrier per k-tile; nothing but the barrier itself sits between two MFMA groups.
    constexpr int G = BK / 8;
    static_assert(G % 2 == 0, "fragment slots alternate with the k-group parity");
    v4f ra[TA::VPT], rb[TB::VPT];
    auto load_tile = [&](int t) {
        const int k0 = kbeg + t * BK;
        const bool kfull = (k0 + BK <= kend);
        if (a_in && kfull) TA::load_fast(ra, A, a.lda, m0, k0, a.a_vec != 0, tid);
        else TA::load(ra, A, a.lda, m0, a.M, k0, kend, a.a_vec != 0, tid);
        if (b_in && kfull) TB::load_fast(rb, Bm, a.ldb, n0, k0, a.b_vec != 0, tid);
        else TB::load(rb, Bm, a.ldb, n0, a.N, k0, kend, a.b_vec != 0, tid);
    };
    v4f fa[2][TM], fb[2][TN];
    auto read_frags = [&](int slot, const float *As, const float *Bs, int g) {
#pragma unroll
        for (int i = 0; i < TM; ++i) fa[slot][i] = TA::frag(As, wm * WM + i * 32 + r, g, h);
#pragma unroll
        for (int j = 0; j < TN; ++j) fb[slot][j] = TB::frag(Bs, wn * WN + j * 32 + r, g, h);
    };
    auto mfma_group = [&](int slot, int chain) {
#pragma unroll
        for (int s = 0; s < 4; ++s)
#pragma unroll
            for (int i = 0; i < TM; ++i)
#pragma unroll
                for (int j = 0; j < TN; ++j)
                    acc[i][j][chain % CHAINS] = __builtin_amdgcn_mfma_f32_32x32x2f32(
                        fa[slot][i][s], fb[slot][j][s], acc[i][j][chain % CHAINS], 0, 0, 0);
    };

    // Interior tiles with 16-byte aligned rows and a whole number of k-tiles take a loop without
    // any guard, in which every memory operation has a fixed place between the MFMAs of a
    // group (a wavefront can issue other instructions while its MFMA executes): the fragment
    // reads of the next group after the group's first MFMA, the LDS write of tile kt+1 in
    // group 0, the global loads of tile kt+2 in group 1.  The explicit lgkmcnt(0) at the head
    // of a group tells the compiler that the reads of the previous group have arrived; left
    // to itself it places the reads next to their first use and waits for them there.
    // (a last, partial k-tile is loaded through the guarded path, which pads it with zeros)
    const bool fast = (G == 4) && a_in && b_in && a.a_vec != 0 && a.b_vec != 0 && nk > 0 && !a.no_fast_loop;
    const int nk_full = (kend - kbeg) / BK;  // tiles [0, nk_full) are whole
    if (fast) {
        auto group = [&](int slot, int chain, auto &&extra) {
            bool first = true;
#pragma unroll
            for (int s = 0; s < 4; ++s)
#pragma unroll
                for (int i = 0; i < TM; ++i)
#pragma unroll
                    for (int j = 0; j < TN; ++j) {
                        acc[i][j][chain % CHAINS] = __builtin_amdgcn_mfma_f32_32x32x2f32(
                            fa[slot][i][s], fb[slot][j][s], acc[i][j][chain % CHAINS], 0, 0, 0);
                        if (first) {
                            first = false;
                            __builtin_amdgcn_sched_barrier(0);
                            extra();
                            __builtin_amdgcn_sched_barrier(0);
                        }
                    }
        };
        auto load_any = [&](int t) {
            if (t < nk_full) {
                TA::load_fast(ra, A, a.lda, m0, kbeg + t * BK, true, tid);
                TB::load_fast(rb, Bm, a.ldb, n0, kbeg + t * BK, true, tid);
            } else {
                TA::load(ra, A, a.lda, m0, a.M, kbeg + t * BK, kend, true, tid);
                TB::load(rb, Bm, a.ldb, n0, a.N, kbeg + t * BK, kend, true, tid);
            }
        };
        load_any(0);
        TA::store(smem, ra, tid);
        TB::store(smem + TA::FLOATS, rb, tid);
        if (nk > 1) load_any(1);
        __syncthreads();
        read_frags(0, smem, smem + TA::FLOATS, 0);
        for (int kt = 0; kt < nk; ++kt) {
            const float *As = smem + (kt & 1) * STAGE;
            const float *Bs = As + TA::FLOATS;
            float *An = smem + ((kt + 1) & 1) * STAGE;
            const bool next = (kt + 1 < nk), next2 = (kt + 2 < nk);
            if (KIND == GEMM_DW && !A_KMAJ) {
                if (do_colsum) {
#pragma unroll
                    for (int k = 0; k < BK / CP; ++k) colsum += As[(cpart + k * CP) * TA::LD + crow];
                }
            }
            __builtin_amdgcn_s_waitcnt(0xc07f);  // lgkmcnt(0)
            group(0, 0, [&]() {
                read_frags(1, As, Bs, 1);
                if (next) {  // tile kt+1 -> the stage nobody reads during this iteration
                    TA::store(An, ra, tid);
                    TB::store(An + TA::FLOATS, rb, tid);
                }
            });
            __builtin_amdgcn_s_waitcnt(0xc07f);
            group(1, 1, [&]() {
                read_frags(0, As, Bs, 2);
                if (next2) load_any(kt + 2);
            });
            __builtin_amdgcn_s_waitcnt(0xc07f);
            group(0, 2, [&]() { read_frags(1, As, Bs, 3); });
            __syncthreads();  // tile kt fully read by everyone, tile kt+1 fully written
            __builtin_amdgcn_s_waitcnt(0xc07f);
            group(1, 3, [&]() {
                if (next) read_frags(0, An, An + TA::FLOATS, 0);
            });
        }
    } else {
    if (nk > 0) {
        load_tile(0);
        TA::store(smem, ra, tid);
        TB::store(smem + TA::FLOATS, rb, tid);
        if (nk > 1) load_tile(1);
    }
    __syncthreads();
    if (nk > 0) read_frags(0, smem, smem + TA::FLOATS, 0);

    for (int kt = 0; kt < nk; ++kt) {
        const float *As = smem + (kt & 1) * STAGE;
        const float *Bs = As + TA::FLOATS;
        float *An = smem + ((kt + 1) & 1) * STAGE;
        if (kt + 1 < nk) {  // tile kt+1 -> the stage nobody reads during this iteration
            TA::store(An, ra, tid);
            TB::store(An + TA::FLOATS, rb, tid);
        }
        if (kt + 2 < nk) load_tile(kt + 2);
        if (KIND == GEMM_DW && !A_KMAJ) {
            if (do_colsum) {
#pragma unroll
                for (int k = 0; k < BK / CP; ++k) colsum += As[(cpart + k * CP) * TA::LD + crow];
            }
        }
#pragma unroll
        for (int g = 0; g + 1 < G; ++g) {
            read_frags((g + 1) & 1, As, Bs, g + 1);
            mfma_group(g & 1, g);
        }
        __syncthreads();  // tile kt fully read by everyone, tile kt+1 fully written
        if (kt + 1 < nk) read_frags(0, An, An + TA::FLOATS, 0);
        mfma_group((G - 1) & 1, G - 1);
    }
    }

    if (KIND == GEMM_DW) {
        if (do_colsum) {  // uniform per workgroup; after the loop's last barrier nobody reads a stage
            smem[cpart * BM + crow] = colsum;
            __syncthreads();
            if (tid < BM && m0 + tid < a.M) {
                float s = smem[tid];
#pragma unroll
                for (int q = 1; q < CP; ++q) s += smem[q * BM + tid];
                a.colsum[(size_t)split * a.M + m0 + tid] = s;
            }
        }
    }

    // ---- epilogue.  acc[i][j][v] is C(row, col) with
    //      row = 8 (v / 4) + 4 h + (v % 4), col = r   inside its 32 x 32 block.
    // The activation enters as a constant: tested per value at run time it was three scalar
    // branches in front of every one of the lane's outputs.
    float *__restrict__ C = static_cast<float *>(a.C) + (size_t)split * a.c_split_stride;
    auto epilogue = [&](auto act_c) {
    constexpr int ACT = decltype(act_c)::value;
    if (a_in && b_in) {
        // Interior tile: no guards.  The backward-data product requests the 16 activation
        // values a lane needs for the derivative together; behind a bounds check per element
        // each load waited for the one before it (16 round trips to memory per block).
        // Every address is a wavefront-uniform base (block row, block column, row inside the
        // block: scalar arithmetic) plus one per-lane offset that is the same for all 16 values,
        // instead of a 64-bit multiply-add per value and lane.
        const float *__restrict__ aux = static_cast<const float *>(a.aux);
        const int wave_u = __builtin_amdgcn_readfirstlane(wave);
        const int wm_u = wave_u % WAVES_M, wn_u = wave_u / WAVES_M;
        const unsigned lo_c = (unsigned)(4 * h * a.ldc + r), lo_x = (unsigned)(4 * h * a.ldaux + r);
#pragma unroll
        for (int j = 0; j < TN; ++j) {
            const int nb = n0 + wn_u * WN + j * 32;  // uniform
            const float bias = bias_pre[j];
#pragma unroll
            for (int i = 0; i < TM; ++i) {
                const int mbu = m0 + wm_u * WM + i * 32;  // uniform; the lane's rows are mbu + 8 (v / 4) + 4 h + v % 4
                float o[16];
                if (KIND == GEMM_DA) {
#pragma unroll
                    for (int v = 0; v < 16; ++v)
                        o[v] = (aux + ((size_t)(mbu + 8 * (v >> 2) + (v & 3)) * a.ldaux + nb))[lo_x];
                }
#pragma unroll
                for (int v = 0; v < 16; ++v) {
                    float x = acc[i][j][0][v];
                    if (CHAINS == 2) x += acc[i][j][CHAINS - 1][v];
                    if (KIND == GEMM_FWD) {
                        x += bias;
                        if (ACT == ACT_SIGMOID) x = sigmoidf_fast(x);
                        else if (ACT == ACT_RELU) x = fmaxf(x, 0.f);
                    } else if (KIND == GEMM_DA) {
                        if (ACT == ACT_SIGMOID) x *= o[v] * (1.f - o[v]);
                        else if (ACT == ACT_RELU) x = (o[v] > 0.f) ? x : 0.f;
                    }
                    (C + ((size_t)(mbu + 8 * (v >> 2) + (v & 3)) * a.ldc + nb))[lo_c] = x;
                }
            }
        }
        return;
    }
#pragma unroll
    for (int j = 0; j < TN; ++j) {
        const int n = n0 + wn * WN + j * 32 + r;
        const bool n_ok = n < a.N;
        const float bias = bias_pre[j];
#pragma unroll
        for (int i = 0; i < TM; ++i) {
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int m = m0 + wm * WM + i * 32 + 8 * (v >> 2) + 4 * h + (v & 3);
                if (m < a.M && n_ok) {
                    float x = acc[i][j][0][v];
                    if (CHAINS == 2) x += acc[i][j][CHAINS - 1][v];
                    if (KIND == GEMM_FWD) {
                        x += bias;
                        if (ACT == ACT_SIGMOID) x = sigmoidf_fast(x);
                        else if (ACT == ACT_RELU) x = fmaxf(x, 0.f);
                    } else if (KIND == GEMM_DA) {
                        const float o = static_cast<const float *>(a.aux)[(size_t)m * a.ldaux + n];
                        if (ACT == ACT_SIGMOID) x *= o * (1.f - o);
                        else if (ACT == ACT_RELU) x = (o > 0.f) ? x : 0.f;
                    }
                    C[(size_t)m * a.ldc + n] = x;
                }
            }
        }
    }
    };
    with_activation(KIND == GEMM_DW ? (int)ACT_NONE : a.act, epilogue);
}

template <int BM, int BN, int BK, int WAVES_M, bool A_KMAJ, bool B_KMAJ, int KIND>
__global__ __launch_bounds__(NT) void gemm_f32_kernel(GemmArgs a)
{
    __shared__ __attribute__((aligned(16))) float smem[lds_floats<BM, BN, BK, A_KMAJ, B_KMAJ>()];
    gemm_f32_tile<BM, BN, BK, WAVES_M, A_KMAJ, B_KMAJ, KIND>(a, smem, xcd_tile_order(blockIdx.x, gridDim.x),
                                                             blockIdx.y);
}

// Backward of one hidden layer in ONE launch: the backward-data product D_{l-1} = (D_l W_l) f'
// (64 x 64 x 32 tiles) and the weight-gradient product dW_l = D_l^T A_{l-1} (DW_BM x 64 x 32
// tiles x K-slices, DW_BM = 128 or 64).  Both only read D_l, so they are independent; sharing
// a launch lets the prologue / epilogue of one hide under the main loop of the other and pays
// the per-launch latencies once.
template <int DW_BM>
__global__ __launch_bounds__(NT) void gemm_f32_bwd_pair_kernel(GemmArgs da, GemmArgs dw, int n_dw)
{
    constexpr int LDS_DA = lds_floats<64, 64, 32, true, false>();
    constexpr int LDS_DW = lds_floats<DW_BM, 64, 32, false, false>();
    __shared__ __attribute__((aligned(16))) float smem[LDS_DA > LDS_DW ? LDS_DA : LDS_DW];
    const int b = blockIdx.x;
    if (b < n_dw) {  // the weight-gradient blocks are the longer ones: they are dispatched first
        const int tiles = dw.tiles_m * dw.tiles_n;
        if ((dw.splits & 7) == 0) {
            // Workgroup ids go round-robin over the 8 XCDs, each with an L2 of its own.  Slice s of
            // the batch is given to XCD s % 8, all of its output tiles: the XCD then reads only its
            // slices' rows of D_l and A_{l-1}, once.  (Dealt out tile by tile, every XCD read every
            // row of A_{l-1}: 8 x 8.4 MB at B = 4096 for 8.4 MB of activations.)  The backward-data
            // blocks below give XCD x a contiguous run of row tiles -- at the usual sizes the very
            // rows of slice x -- so both products find D_l and A_{l-1} in the same L2.
            const int q = b >> 3;
            gemm_f32_tile<DW_BM, 64, 32, 2, false, false, GEMM_DW>(dw, smem, q % tiles, (b & 7) + 8 * (q / tiles));
        } else {
            gemm_f32_tile<DW_BM, 64, 32, 2, false, false, GEMM_DW>(dw, smem, xcd_tile_order(b % tiles, tiles), b / tiles);
        }
    } else {
        const int n_da = gridDim.x - n_dw;
        gemm_f32_tile<64, 64, 32, 2, true, false, GEMM_DA>(da, smem, xcd_tile_order(b - n_dw, n_da), 0);
    }
}

// ---- small products: one 32 x 32 output block per workgroup, the contraction split over
// the four wavefronts.
//
// With few output tiles (a small batch) the 64 x 64 kernel leaves most compute units idle
// while each wavefront walks the whole contraction alone: K / 2 dependent-issue MFMAs of 64
// cycles each are the run time, whatever the batch.  Here every workgroup owns one 32 x 32
// block and its wavefront w takes the k-groups {w, w + 4, ...} of every k-tile, so the MFMA
// chain per wavefront is a quarter as long and four times as many workgroups exist.  The four
// partial blocks meet in LDS (the tile stages are free by then) and every wavefront finishes
// eight rows of the block with the fused epilogue.
template <int BK, bool A_KMAJ, bool B_KMAJ, int KIND>
__device__ __forceinline__ void gemm_f32_small_tile(const GemmArgs &a, float *smem, int id, int split)
{
    using TA = Tile<32, BK, A_KMAJ>;
    using TB = Tile<32, BK, B_KMAJ>;
    constexpr int STAGE = TA::FLOATS + TB::FLOATS;
    constexpr int G = BK / 8;  // k-groups of 8 per tile
    static_assert(G % 4 == 0, "k-groups are dealt to four wavefronts");
    constexpr int Q = G / 4;   // k-groups per wavefront and tile
    constexpr int RED_LD = 40, RED = 32 * RED_LD;  // 4 rows apart = 32 banks apart
    static_assert(2 * STAGE >= 4 * RED, "partial blocks reuse the tile stages");

    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int r = lane & 31, h = lane >> 5;

    const int tile_m = id / a.tiles_n, tile_n = id - tile_m * a.tiles_n;
    const int m0 = tile_m * 32, n0 = tile_n * 32;
    const int kbeg = split * a.k_chunk;
    const int kend = min(a.K, kbeg + a.k_chunk);
    const int nk = (kend - kbeg + BK - 1) / BK;

    const float *__restrict__ A = static_cast<const float *>(a.A);
    const float *__restrict__ Bm = static_cast<const float *>(a.B);

    v16f acc[2];  // two independent MFMA chains
#pragma unroll
    for (int c = 0; c < 2; ++c)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[c][v] = 0.f;

    const bool a_in = (m0 + 32 <= a.M), b_in = (n0 + 32 <= a.N);
    float colsum = 0.f;
    const bool do_colsum = (KIND == GEMM_DW) && a.colsum != nullptr && tile_n == 0;
    // forward: the lane's bias is requested now, not after the reduction
    const float bias_pre = (KIND == GEMM_FWD && a.bias != nullptr && n0 + r < a.N) ? a.bias[n0 + r] : 0.f;

    v4f ra[TA::VPT], rb[TB::VPT];
    auto load_tile = [&](int t) {
        const int k0 = kbeg + t * BK;
        const bool kfull = (k0 + BK <= kend);
        if (a_in && kfull) TA::load_fast(ra, A, a.lda, m0, k0, a.a_vec != 0, tid);
        else TA::load(ra, A, a.lda, m0, a.M, k0, kend, a.a_vec != 0, tid);
        if (b_in && kfull) TB::load_fast(rb, Bm, a.ldb, n0, k0, a.b_vec != 0, tid);
        else TB::load(rb, Bm, a.ldb, n0, a.N, k0, kend, a.b_vec != 0, tid);
    };
    v4f fa[Q], fb[Q];
    auto read_frags = [&](const float *As, const float *Bs) {
#pragma unroll
        for (int q = 0; q < Q; ++q) {
            fa[q] = TA::frag(As, r, wave + 4 * q, h);
            fb[q] = TB::frag(Bs, r, wave + 4 * q, h);
        }
    };

    // global loads run two k-tiles ahead, the LDS write one tile ahead, the fragments of tile
    // kt+1 are read right after the barrier of tile kt, under its last MFMAs
    load_tile(0);
    TA::store(smem, ra, tid);
    TB::store(smem + TA::FLOATS, rb, tid);
    if (nk > 1) load_tile(1);
    __syncthreads();
    read_frags(smem, smem + TA::FLOATS);
    for (int kt = 0; kt < nk; ++kt) {
        const float *As = smem + (kt & 1) * STAGE;
        float *An = smem + ((kt + 1) & 1) * STAGE;
        const bool next = (kt + 1 < nk);
        if (next) {
            TA::store(An, ra, tid);
            TB::store(An + TA::FLOATS, rb, tid);
        }
        if (kt + 2 < nk) load_tile(kt + 2);
        if (KIND == GEMM_DW && !A_KMAJ) {
            if (do_colsum && tid < 32) {
#pragma unroll
                for (int k = 0; k < BK; ++k) colsum += As[k * TA::LD + tid];
            }
        }
        v4f ca[Q], cb[Q];
#pragma unroll
        for (int q = 0; q < Q; ++q) {
            ca[q] = fa[q];
            cb[q] = fb[q];
        }
#pragma unroll
        for (int s = 0; s < 2; ++s)
#pragma unroll
            for (int q = 0; q < Q; ++q)
                acc[q & 1] = __builtin_amdgcn_mfma_f32_32x32x2f32(ca[q][s], cb[q][s], acc[q & 1], 0, 0, 0);
        __syncthreads();  // tile kt read by everyone (fragments are in registers), tile kt+1 written
        if (next) read_frags(An, An + TA::FLOATS);
#pragma unroll
        for (int s = 2; s < 4; ++s)
#pragma unroll
            for (int q = 0; q < Q; ++q)
                acc[q & 1] = __builtin_amdgcn_mfma_f32_32x32x2f32(ca[q][s], cb[q][s], acc[q & 1], 0, 0, 0);
    }

    // ---- the four partial blocks meet in LDS.  acc[.][v] is C(row, col) with
    //      row = 8 (v / 4) + 4 h + (v % 4), col = r.  After the loop's last barrier nobody
    //      reads a tile stage any more (the DW column sums read theirs before it).
    float *mine = smem + wave * RED;
#pragma unroll
    for (int v = 0; v < 16; ++v)
        mine[(8 * (v >> 2) + 4 * h + (v & 3)) * RED_LD + r] = acc[0][v] + acc[1][v];
    __syncthreads();

    float *__restrict__ C = static_cast<float *>(a.C) + (size_t)split * a.c_split_stride;
    const int n = n0 + r;
    const bool n_ok = n < a.N;
    const float bias = bias_pre;
    float o4[4] = {0.f, 0.f, 0.f, 0.f};
    if (KIND == GEMM_DA && a_in && b_in) {  // the four activation values of the lane, requested together
#pragma unroll
        for (int p = 0; p < 4; ++p)
            o4[p] = static_cast<const float *>(a.aux)[(size_t)(m0 + 8 * wave + 2 * p + h) * a.ldaux + n];
    }
    with_activation(KIND == GEMM_DW ? (int)ACT_NONE : a.act, [&](auto act_c) {
        constexpr int ACT = decltype(act_c)::value;
#pragma unroll
        for (int p = 0; p < 4; ++p) {
            const int row = 8 * wave + 2 * p + h;
            const int m = m0 + row;
            float x = smem[row * RED_LD + r] + smem[RED + row * RED_LD + r] +
                      (smem[2 * RED + row * RED_LD + r] + smem[3 * RED + row * RED_LD + r]);
            if (m < a.M && n_ok) {
                if (KIND == GEMM_FWD) {
                    x += bias;
                    if (ACT == ACT_SIGMOID) x = sigmoidf_fast(x);
                    else if (ACT == ACT_RELU) x = fmaxf(x, 0.f);
                } else if (KIND == GEMM_DA) {
                    const float o = (a_in && b_in) ? o4[p] : static_cast<const float *>(a.aux)[(size_t)m * a.ldaux + n];
                    if (ACT == ACT_SIGMOID) x *= o * (1.f - o);
                    else if (ACT == ACT_RELU) x = (o > 0.f) ? x : 0.f;
                }
                C[(size_t)m * a.ldc + n] = x;
            }
        }
    });
    if (KIND == GEMM_DW) {
        if (do_colsum && tid < 32 && m0 + tid < a.M)
            a.colsum[(size_t)split * a.M + m0 + tid] = colsum;
    }
}

constexpr int SMALL_BK = 64;

template <bool A_KMAJ, bool B_KMAJ, int KIND>
__global__ __launch_bounds__(NT) void gemm_f32_small_kernel(GemmArgs a)
{
    __shared__ __attribute__((aligned(16))) float smem[lds_floats<32, 32, SMALL_BK, A_KMAJ, B_KMAJ>()];
    gemm_f32_small_tile<SMALL_BK, A_KMAJ, B_KMAJ, KIND>(a, smem, xcd_tile_order(blockIdx.x, gridDim.x),
                                                       blockIdx.y);
}

// The backward pair of one hidden layer (see gemm_f32_bwd_pair_kernel) for small batches.
__global__ __launch_bounds__(NT) void gemm_f32_small_pair_kernel(GemmArgs da, GemmArgs dw, int n_dw)
{
    constexpr int LDS_DA = lds_floats<32, 32, SMALL_BK, true, false>();
    constexpr int LDS_DW = lds_floats<32, 32, SMALL_BK, false, false>();
    __shared__ __attribute__((aligned(16))) float smem[LDS_DA > LDS_DW ? LDS_DA : LDS_DW];
    const int b = blockIdx.x;
    if (b < n_dw) {
        const int tiles = dw.tiles_m * dw.tiles_n;
        gemm_f32_small_tile<SMALL_BK, false, false, GEMM_DW>(dw, smem, xcd_tile_order(b % tiles, tiles), b / tiles);
    } else {
        const int n_da = gridDim.x - n_dw;
        gemm_f32_small_tile<SMALL_BK, true, false, GEMM_DA>(da, smem, xcd_tile_order(b - n_dw, n_da), 0);
    }
}

int env_int(const char *name, int dflt)
{
    const char *s = getenv(name);
    return (s && *s) ? atoi(s) : dflt;
}

// Workgroups wanted per launch: two per compute unit on a 256-CU device.
int target_wgs()
{
    static const int v = env_int("HB_GEMM_WGS", 512);  // tuning aid
    return v;
}

struct Shape {
    int bm, bn, bk;
};

// Tile shapes that are instantiated.  HB_GEMM_TILE = 1..5 forces one (tuning aid).
constexpr Shape SHAPES[] = {{64, 64, 16}, {64, 64, 32}, {128, 64, 16}, {128, 64, 32}, {128, 128, 16}};
constexpr int K_CHUNK_ALIGN = 32;  // split-K slices are multiples of every BK above

Shape pick_shape(GemmKind kind, int M, int N)
{
    static const int forced = env_int("HB_GEMM_TILE", 0);
    if (forced >= 1 && forced <= 5) return SHAPES[forced - 1];
    // measured on 4096 x 512 x 512 (MI355X): forward / backward-data are fastest with
    // 64 x 64 x 32 tiles (two workgroups per CU), the split-K weight gradient with 128 x 64 x 32
    (void)N;
    if (kind == GEMM_DW && M >= 128) return SHAPES[3];
    return SHAPES[1];
}

template <int BM, int BN, int BK, int WAVES_M>
hipError_t launch_shape(GemmKind kind, const GemmArgs &a, dim3 grid, hipStream_t stream,
                        const LaunchEvents &ev)
{
    switch (kind) {
    case GEMM_FWD:
        return launch_kernel(gemm_f32_kernel<BM, BN, BK, WAVES_M, true, true, GEMM_FWD>, grid,
                             dim3(NT), stream, ev, a);
    case GEMM_DA:
        return launch_kernel(gemm_f32_kernel<BM, BN, BK, WAVES_M, true, false, GEMM_DA>, grid,
                             dim3(NT), stream, ev, a);
    case GEMM_DW:
        return launch_kernel(gemm_f32_kernel<BM, BN, BK, WAVES_M, false, false, GEMM_DW>, grid,
                             dim3(NT), stream, ev, a);
    }
    return hipErrorInvalidValue;
}

struct SplitPlan {
    int splits, chunk;
};

// Split-K plan for the weight-gradient product (its contraction runs over the batch):
// enough slices to fill the device, each a multiple of BK long, none empty.
SplitPlan plan_splits(int tiles, int K, int max_splits, int wgs = 0)
{
    if (wgs <= 0) wgs = target_wgs();
    int s = (wgs + tiles - 1) / tiles;
    const int by_k = (K + 4 * K_CHUNK_ALIGN - 1) / (4 * K_CHUNK_ALIGN);  // slices of >= 128
    if (s > by_k) s = by_k;
    if (s > max_splits) s = max_splits;
    if (s < 1) s = 1;
    const int chunk = ((K + s - 1) / s + K_CHUNK_ALIGN - 1) / K_CHUNK_ALIGN * K_CHUNK_ALIGN;
    return {(K + chunk - 1) / chunk, chunk};
}

// Products with fewer 64 x 64 output tiles than this (forward / backward-data), or a
// contraction shorter than small_k_max() (weight gradient, whose contraction is the batch),
// go to the 32 x 32 split-wavefront kernel.  HB_GEMM_SMALL_TILES / HB_GEMM_SMALL_K: tuning aids
// (0 switches the small kernels off).
int small_tiles_max()
{
    static const int v = env_int("HB_GEMM_SMALL_TILES", 160);  // measured crossover: B = 1280 for 512-wide layers
    return v;
}
int small_k_max()
{
    static const int v = env_int("HB_GEMM_SMALL_K", 2048);
    return v;
}
bool small_out(int M, int N, int K)
{
    static const int forced = env_int("HB_GEMM_TILE", 0);
    return forced == 0 && K >= 64 && (long long)((M + 63) / 64) * ((N + 63) / 64) < small_tiles_max();
}
bool small_dw(int K)
{
    static const int forced = env_int("HB_GEMM_TILE", 0);
    return forced == 0 && K >= 64 && K < small_k_max();
}
// A weight gradient launched on its own (not paired with a backward-data product) whose output
// is only a few tiles -- the first layer of a narrow input, 512 x 54 -- stays with the small
// kernel up to four times that contraction length: with so few tiles the 64-wide kernel needs
// tens of K-slices to fill the chip, and every slice is a partial the update has to read
// (B = 4096, 512 x 54: 12.4 -> 11.0 us, and the update 7.7 -> 7.2 us).
long long small_dw_alone_kmax(int M, int N)  // contractions below this go to the small kernel
{
    const bool few_tiles = (long long)((M + 63) / 64) * ((N + 63) / 64) <= 16;
    return few_tiles ? 4 * (long long)small_k_max() : (long long)small_k_max();
}
bool small_dw_alone(int M, int N, int K)
{
    static const int forced = env_int("HB_GEMM_TILE", 0);
    return forced == 0 && K >= 64 && K < small_dw_alone_kmax(M, N);
}
// K-slices of the small weight-gradient kernel: at most 512 long (multiples of its k-tile)
SplitPlan plan_small_splits(int K, int max_splits)
{
    int s = (K + 511) / 512;
    if (s > max_splits) s = max_splits;
    if (s < 1) s = 1;
    const int chunk = ((K + s - 1) / s + SMALL_BK - 1) / SMALL_BK * SMALL_BK;
    return {(K + chunk - 1) / chunk, chunk};
}

}  // namespace

int gemm_f32_dw_splits(int M, int N, int K, int max_splits)
{
    const Shape sh = pick_shape(GEMM_DW, M, N);
    const int tiles = ((M + sh.bm - 1) / sh.bm) * ((N + sh.bn - 1) / sh.bn);
    const int big = plan_splits(tiles, K, max_splits).splits;
    // longest contraction the small kernel can be given for any batch up to K
    const long long kmax = small_dw_alone_kmax(M, N);
    const int ks = K < kmax ? K : (int)(kmax - 1);
    const int small = (ks >= 64) ? plan_small_splits(ks, max_splits).splits : 1;
    return big > small ? big : small;
}

hipError_t launch_gemm_f32(GemmKind kind, GemmArgs a, int max_splits, int *splits_out,
                           hipStream_t stream, const LaunchEvents &ev)
{
    if (a.M <= 0 || a.N <= 0 || a.K <= 0) return hipErrorInvalidValue;
    if (kind == GEMM_DW ? small_dw_alone(a.M, a.N, a.K) : small_out(a.M, a.N, a.K)) {
        a.tiles_m = (a.M + 31) / 32;
        a.tiles_n = (a.N + 31) / 32;
        const long long tiles = (long long)a.tiles_m * a.tiles_n;
        if (tiles > 0x7fffffffLL) return hipErrorInvalidValue;
        SplitPlan sp = {1, (a.K + SMALL_BK - 1) / SMALL_BK * SMALL_BK};
        if (kind == GEMM_DW) sp = plan_small_splits(a.K, max_splits);
        a.splits = sp.splits;
        a.k_chunk = sp.chunk;
        if (splits_out) *splits_out = sp.splits;
        const dim3 grid((unsigned)tiles, (unsigned)sp.splits, 1);
        switch (kind) {
        case GEMM_FWD:
            return launch_kernel(gemm_f32_small_kernel<true, true, GEMM_FWD>, grid, dim3(NT), stream, ev, a);
        case GEMM_DA:
            return launch_kernel(gemm_f32_small_kernel<true, false, GEMM_DA>, grid, dim3(NT), stream, ev, a);
        case GEMM_DW:
            return launch_kernel(gemm_f32_small_kernel<false, false, GEMM_DW>, grid, dim3(NT), stream, ev, a);
        }
        return hipErrorInvalidValue;
    }
    const Shape sh = pick_shape(kind, a.M, a.N);
    static const int no_fast = env_int("HB_GEMM_NOFAST", 0);
    a.no_fast_loop = no_fast;
    a.tiles_m = (a.M + sh.bm - 1) / sh.bm;
    a.tiles_n = (a.N + sh.bn - 1) / sh.bn;
    const long long tiles = (long long)a.tiles_m * a.tiles_n;
    if (tiles > 0x7fffffffLL) return hipErrorInvalidValue;
    SplitPlan sp = {1, (a.K + K_CHUNK_ALIGN - 1) / K_CHUNK_ALIGN * K_CHUNK_ALIGN};
    if (kind == GEMM_DW) sp = plan_splits((int)tiles, a.K, max_splits);
    a.splits = sp.splits;
    a.k_chunk = sp.chunk;
    if (splits_out) *splits_out = sp.splits;
    const dim3 grid((unsigned)tiles, (unsigned)sp.splits, 1);
    if (sh.bm == 64 && sh.bk == 16) return launch_shape<64, 64, 16, 2>(kind, a, grid, stream, ev);
    if (sh.bm == 64 && sh.bk == 32) return launch_shape<64, 64, 32, 2>(kind, a, grid, stream, ev);
    if (sh.bn == 64 && sh.bk == 16) return launch_shape<128, 64, 16, 2>(kind, a, grid, stream, ev);
    if (sh.bn == 64 && sh.bk == 32) return launch_shape<128, 64, 32, 2>(kind, a, grid, stream, ev);
    return launch_shape<128, 128, 16, 2>(kind, a, grid, stream, ev);
}


// dA_l and dW_l of one hidden layer in one launch (see gemm_f32_bwd_pair_kernel).  Only for
// shapes the fixed tile shapes of that kernel suit; the caller falls back to two launches
// when this returns false from gemm_f32_pair_ok.
bool gemm_f32_pair_ok(const GemmArgs &da, const GemmArgs &dw)
{
    static const int off = env_int("HB_NO_PAIR", 0);
    return !off && da.M >= 64 && da.N >= 64 && da.K >= 32 && dw.M >= 128 && dw.N >= 64 && dw.K >= 32;
}

hipError_t launch_gemm_f32_bwd_pair(GemmArgs da, GemmArgs dw, int max_splits, int *splits_out,
                                    hipStream_t stream, const LaunchEvents &ev)
{
    static const int pair_wgs = env_int("HB_PAIR_WGS", 256);  // weight-gradient blocks wanted (tuning aid)
    static const int no_fast = env_int("HB_GEMM_NOFAST", 0);
    da.no_fast_loop = dw.no_fast_loop = no_fast;
    if (small_out(da.M, da.N, da.K) && small_dw(dw.K)) {
        da.tiles_m = (da.M + 31) / 32;
        da.tiles_n = (da.N + 31) / 32;
        da.splits = 1;
        da.k_chunk = (da.K + SMALL_BK - 1) / SMALL_BK * SMALL_BK;
        dw.tiles_m = (dw.M + 31) / 32;
        dw.tiles_n = (dw.N + 31) / 32;
        const long long n_da = (long long)da.tiles_m * da.tiles_n;
        const long long t_dw = (long long)dw.tiles_m * dw.tiles_n;
        const SplitPlan sp = plan_small_splits(dw.K, max_splits);
        dw.splits = sp.splits;
        dw.k_chunk = sp.chunk;
        if (splits_out) *splits_out = sp.splits;
        const long long blocks = n_da + t_dw * sp.splits;
        if (blocks > 0x7fffffffLL) return hipErrorInvalidValue;
        return launch_kernel(gemm_f32_small_pair_kernel, dim3((unsigned)blocks), dim3(NT), stream, ev, da, dw,
                             (int)(t_dw * sp.splits));
    }
    da.tiles_m = (da.M + 63) / 64;
    da.tiles_n = (da.N + 63) / 64;
    da.splits = 1;
    da.k_chunk = (da.K + K_CHUNK_ALIGN - 1) / K_CHUNK_ALIGN * K_CHUNK_ALIGN;
    const long long n_da = (long long)da.tiles_m * da.tiles_n;
    // While everything fits the device at once (four 64 x 64 workgroups per CU by LDS), the
    // weight gradient takes 64 x 64 tiles too: 2 x pair_wgs blocks as long as the backward-data
    // ones, so no compute unit ends on a lone long block (measured at B = 2048 and 4096:
    // 45 instead of 47 us; with more backward-data blocks than that the 128-row tile wins).
    static const int dw64_env = env_int("HB_PAIR_DW64", -1);  // tuning aid: 0 / 1 force
    const bool dw64 = dw64_env >= 0 ? dw64_env != 0 : (n_da + 2 * pair_wgs <= 4 * 256);
    dw.tiles_m = dw64 ? (dw.M + 63) / 64 : (dw.M + 127) / 128;
    dw.tiles_n = (dw.N + 63) / 64;
    const long long t_dw = (long long)dw.tiles_m * dw.tiles_n;
    if (n_da > 0x3fffffffLL || t_dw > 0x3fffffffLL) return hipErrorInvalidValue;
    const SplitPlan sp = plan_splits((int)t_dw, dw.K, max_splits, dw64 ? 2 * pair_wgs : pair_wgs);
    dw.splits = sp.splits;
    dw.k_chunk = sp.chunk;
    if (splits_out) *splits_out = sp.splits;
    const long long blocks = n_da + t_dw * sp.splits;
    if (blocks > 0x7fffffffLL) return hipErrorInvalidValue;
    if (dw64)
        return launch_kernel(gemm_f32_bwd_pair_kernel<64>, dim3((unsigned)blocks), dim3(NT), stream, ev, da, dw,
                             (int)(t_dw * sp.splits));
    return launch_kernel(gemm_f32_bwd_pair_kernel<128>, dim3((unsigned)blocks), dim3(NT), stream, ev, da, dw,
                         (int)(t_dw * sp.splits));
}

}  // namespace hb
