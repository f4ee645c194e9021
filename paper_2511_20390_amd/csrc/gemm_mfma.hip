// bf16 MFMA GEMM for the dense projections of the DiT blocks (QKV, attention
// out-projection, MLP FC1/FC2 of the packed target forward, Alg. 1):
//   C[M,N] = X[M,K] . W[N,K]^T  (+bias, fused epilogue), fp32 accumulation.
// Both operands are K-contiguous, which is exactly the per-lane operand layout of
// v_mfma_f32_32x32x16_bf16 (lane l: row/col l%32, 8 consecutive k at 8*(l/32)).
//
// Design for gfx950 (64-wide wavefronts, 160 KB LDS per CU, 512 registers per lane):
//  * workgroup = 4 or 8 wavefronts in a WGM x WGN grid, macro tile BM x BN (256x256 and
//    384x192 with 8 wavefronts - two per SIMD, so one wavefront's memory instructions issue
//    under the other's MFMAs - 256x128 / 128x128 / 96x128 / 160x128 with 4 for small problems), K slices of
//    64; each wavefront owns (BM/WGM) x (BN/WGN) as TM x TN MFMA tiles of 32x32 and keeps
//    the accumulators in registers for the whole K loop.
//  * the MFMA takes the WEIGHT rows as its A operand and the activation rows as its
//    B operand, i.e. it accumulates C^T tiles: a lane then owns one output ROW m
//    (lane % 32) and runs of 4 consecutive output columns n per register group.  Each
//    32-row block of output is transposed through a wave-private piece of the (by then idle)
//    LDS tiles so that global accesses cover whole rows of the wave's tile with consecutive
//    lanes - a row otherwise lives in two lanes, 32 bytes per row and instruction, and such
//    partial-line writes cost up to 1.8x the algorithmic write traffic at the memory
//    controller.  For bf16 output one v_permlane32_swap first pairs the two half-waves' runs
//    into 8 consecutive bf16; the fp32 residual update is a float4 read-modify-write on the
//    transposed block with all loads of a group issued before its first store.
//  * LDS: two stages of [BM + BN rows][64 bf16]; the 16-byte chunk index of a row is
//    XOR-swizzled with (row / 2) % 8: a ds_read_b128 is served 16 lanes at a time over 64
//    banks (256 bytes), and with this pattern the 16 rows of a pass hit 16 distinct 16-byte
//    bank groups (the conflict counter reads zero; swizzling with row % 8 leaves rows r and
//    r + 8 on the same banks, a 2-way conflict on every fragment read).  Global loads stay
//    128-byte coalesced.
//  * global loads are buffer loads (descriptor + one per-lane offset + scalar offsets):
//    no address registers, and rows past the end of a ragged edge tile read as zero.
//  * software pipeline: global loads run two slices ahead (slice kt+2 is in flight in
//    registers while slice kt+1 is written to the other LDS stage and slice kt is
//    multiplied); the LDS writes and the refills are spread over three of the four
//    k-steps; MFMA operand fragments are double-buffered in registers so every LDS read
//    is issued one k-step before its use; issue order is pinned with
//    sched_group_barrier.  One barrier per slice, placed before the last k-step so the
//    first fragments of the next slice are read under that step's MFMAs.
//  * workgroup ids are remapped so that each of the 8 XCDs (round-robin dispatch)
//    works on a compact, L2-friendly group of tiles.
//  * the tile configuration is chosen per problem from a measured time model (whole
//    rounds of workgroups x (K slices x time per slice + per-tile fixed cost)).
//  * FREE_FP32 mode runs the same kernel on fp32 operands: a K slice is still 128 bytes per row
//    (32 values), a fragment still one 16-byte chunk per lane, and each chunk pair feeds four
//    v_mfma_f32_32x32x2_f32 (one per element of the chunk: lane group 0 supplies k = 4 c + e,
//    group 1 supplies k = 4 (c + 1) + e, the same pairing for both operands); full fp32
//    products and accumulation, fp32 output through the LDS-staged row-major stores.
#include <algorithm>
#include <cmath>
#include <cstdlib>
#include <type_traits>

#include "free_internal.h"

namespace freemi {

namespace {

typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
typedef float f32x2_t __attribute__((ext_vector_type(2)));
typedef float f32x4_t __attribute__((ext_vector_type(4)));
typedef float f32x16_t __attribute__((ext_vector_type(16)));
typedef uint32_t u32x4_t __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2_t __attribute__((ext_vector_type(2)));

constexpr int BK = 64;                    // bf16 elements per K slice (128 bytes per row)
constexpr int kRowBytes = BK * 2;
constexpr int kNumXcd = 8;

__device__ inline float gelu_fast(float v) {
    // tanh-form GELU: 0.5 v (1 + tanh(u)) = v / (1 + exp(-2u)), u = sqrt(2/pi)(v + 0.044715 v^3)
    // exp(-2u) = 2^(v (a + b v^2)) with the constants folded; v_exp_f32 and v_rcp_f32 directly (1 ulp each,
    // far below the bf16 rounding of the result).  The correctly rounded reciprocal is a ten-instruction
    // division sequence per element, and this runs on every element of the MLP's hidden layer while the
    // matrix cores wait.  2^t overflows to +inf for very negative v: 1 / inf = 0, the right limit.
    constexpr float a = -2.0f * 0.7978845608028654f * 1.4426950408889634f;
    constexpr float b = a * 0.044715f;
    const float t = v * fmaf(v * v, b, a);
    return v * __builtin_amdgcn_rcpf(1.0f + __builtin_amdgcn_exp2f(t));
}

__device__ inline uint32_t pack2(float lo, float hi) {
    const f32x2_t f = {lo, hi};
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(f, bf16x2_t));   // v_cvt_pk_bf16_f32 (RNE)
}

// Issue-order hints for one k-step of MF MFMAs: every MFMA is followed by at most one
// fragment read (NR of them), one LDS write (NW) and one global load (NL), so the matrix
// pipe never waits behind a burst of memory instructions.
constexpr int kMfma = 0x008, kVmemRd = 0x020, kDsRd = 0x100, kDsWr = 0x200;
template <int Q, int MF, int NR, int NW, int NL>
__device__ __forceinline__ void sched_hints() {
    if constexpr (Q < MF) {
        __builtin_amdgcn_sched_group_barrier(kMfma, 1, 0);
        if constexpr (Q < NR) __builtin_amdgcn_sched_group_barrier(kDsRd, 1, 0);
        if constexpr (Q < NW) __builtin_amdgcn_sched_group_barrier(kDsWr, 1, 0);
        if constexpr (Q < NL) __builtin_amdgcn_sched_group_barrier(kVmemRd, 1, 0);
        sched_hints<Q + 1, MF, NR, NW, NL>();
    } else {
        __builtin_amdgcn_sched_barrier(0);
    }
}

// XCD-aware tile order: workgroup ids are dealt round-robin to the 8 XCDs, so the
// ids of one XCD are made contiguous first, then walked in groups of kGroupM row
// tiles (column-major inside a group) so concurrent workgroups share X and W panels.
__device__ inline void tile_coords(int kGroupM, int pid, int tiles_m, int tiles_n, int* tm, int* tn) {
    const int total = tiles_m * tiles_n;
    const int q = total / kNumXcd, r = total % kNumXcd;
    const int x = pid % kNumXcd, j = pid / kNumXcd;
    const int npid = x * q + (x < r ? x : r) + j;
    const int per_group = kGroupM * tiles_n;
    const int group = npid / per_group;
    const int first_m = group * kGroupM;
    const int gsize = (tiles_m - first_m < kGroupM) ? tiles_m - first_m : kGroupM;
    const int in_group = npid % per_group;
    *tm = first_m + in_group % gsize;
    *tn = in_group / gsize;
}

// Epilogue shared by the GEMM kernels.  Register e of acc[i][j] in lane l is output row
// m = gm_lane + 32 i (gm_lane already includes l % 32), column n = gn_wave + 32 j + 8 (e/4) + 4 lhi + e%4.
// QB: for the residual update, chunks per lane whose loads are in flight together in the LDS-staged form; 0
// selects the direct form.
// Folded LayerNorm (see LnFold): kPrep - the residual update also writes z and the partial row sums;
// kLn - the accumulators hold z W^T - mu c1 + c0 / r (the kernel adds the rank-2 term as an extra k-step before
// its K loop), so the output is r acc with the per-row factor ln_a = r of this lane's rows: no bias, one
// multiplication per element.
template <typename OT, int TM, int TN, int EPI, int QB>
__device__ __forceinline__ void write_tile(const f32x16_t (&acc)[TM][TN], int gm_lane, int gn_wave, int lane, int32_t M,
                                           int32_t N, int32_t vec_ok, const float* __restrict__ bias,
                                           OT* __restrict__ out, float* __restrict__ resid, const RowVec& gate,
                                           char* wave_lds, const LnFold& ln, const float (&ln_a)[TM]) {
    constexpr bool kF32Out = std::is_same<OT, float>::value;   // fp32 mode: the output of the bias / GELU epilogues is fp32
    constexpr bool kPrep = EPI == FREE_EPI_GATE_RESID_PREP;
    constexpr bool kResid = EPI == FREE_EPI_GATE_RESID || kPrep;
    constexpr bool kLn = EPI == FREE_EPI_LN_BIAS || EPI == FREE_EPI_LN_BIAS_GELU;
    constexpr bool kGelu = EPI == FREE_EPI_BIAS_GELU || EPI == FREE_EPI_LN_BIAS_GELU;
    static_assert(!kPrep || (QB > 0 && TN == 4), "z and the row sums come out of the staged residual update of a 128-column wavefront");
    static_assert(!kLn || !kF32Out, "folded LayerNorm: bf16 path only");
    const int lhi = lane >> 5;
    if (vec_ok) {
        // N % 8 == 0 and 16-byte aligned rows: runs of 4 / 8 columns are all inside or all outside.
        // Rows past M and runs past N (ragged edge tiles) are masked per lane.
        if constexpr (kF32Out && !kResid && QB == 0) {
            // fp32 output straight from the accumulator layout (four-wavefront configurations)
#pragma unroll
            for (int j = 0; j < TN; ++j) {
                const int gn0 = gn_wave + j * 32 + 4 * lhi;
#pragma unroll
                for (int e4 = 0; e4 < 4; ++e4) {
                    if (gn0 + 8 * e4 >= N) continue;
                    const f32x4_t bv = *reinterpret_cast<const f32x4_t*>(bias + gn0 + 8 * e4);
#pragma unroll
                    for (int i = 0; i < TM; ++i) {
                        const int gm = gm_lane + i * 32;
                        if (gm >= M) continue;
                        f32x4_t o;
#pragma unroll
                        for (int c = 0; c < 4; ++c) {
                            o[c] = acc[i][j][4 * e4 + c] + bv[c];
                            if (kGelu) o[c] = gelu_fast(o[c]);
                        }
                        *reinterpret_cast<f32x4_t*>(reinterpret_cast<float*>(out) + static_cast<int64_t>(gm) * N + gn0 + 8 * e4) = o;
                    }
                }
            }
        } else if constexpr (EPI == FREE_EPI_GATE_RESID && QB == 0) {
            // read-modify-write of the fp32 residual stream straight from the accumulator layout (32 rows x
            // 32 bytes per instruction).  All loads of a column tile j are issued before its first store (a
            // store would otherwise fence the following loads).  Faster than the staged form below for the
            // four-wavefront configurations: with one wavefront per SIMD the LDS round trip is not hidden.
            const float* __restrict__ gbase = gate.base;
            int64_t g_off[TM], r_off[TM];
            bool row_ok[TM];
#pragma unroll
            for (int i = 0; i < TM; ++i) {
                const int gm = gm_lane + i * 32;
                row_ok[i] = gm < M;
                g_off[i] = static_cast<int64_t>(gm / gate.rows_per_sample) * gate.stride;
                r_off[i] = static_cast<int64_t>(gm) * N;
            }
#pragma unroll
            for (int j = 0; j < TN; ++j) {
                const int gn0 = gn_wave + j * 32 + 4 * lhi;
                f32x4_t bv[4], g[TM][4], r[TM][4];
#pragma unroll
                for (int e4 = 0; e4 < 4; ++e4)
                    if (gn0 + 8 * e4 < N) bv[e4] = *reinterpret_cast<const f32x4_t*>(bias + gn0 + 8 * e4);
#pragma unroll
                for (int i = 0; i < TM; ++i)
#pragma unroll
                    for (int e4 = 0; e4 < 4; ++e4)
                        if (row_ok[i] && gn0 + 8 * e4 < N) {
                            g[i][e4] = *reinterpret_cast<const f32x4_t*>(gbase + g_off[i] + gn0 + 8 * e4);
                            r[i][e4] = *reinterpret_cast<const f32x4_t*>(resid + r_off[i] + gn0 + 8 * e4);
                        }
#pragma unroll
                for (int i = 0; i < TM; ++i)
#pragma unroll
                    for (int e4 = 0; e4 < 4; ++e4)
                        if (row_ok[i] && gn0 + 8 * e4 < N) {
#pragma unroll
                            for (int c = 0; c < 4; ++c)
                                r[i][e4][c] = fmaf(g[i][e4][c], acc[i][j][4 * e4 + c] + bv[e4][c], r[i][e4][c]);
                            *reinterpret_cast<f32x4_t*>(resid + r_off[i] + gn0 + 8 * e4) = r[i][e4];
                        }
            }
        } else if constexpr (kResid || kF32Out) {
            // read-modify-write of the fp32 residual stream (or, in fp32 mode, the plain fp32 output of the
            // bias / GELU epilogues: same staging, no read).  As for the bf16 output below, the accumulator
            // layout would touch 32 rows x 32 bytes per instruction; each 32-row block is staged in the
            // wave-private LDS region CG column tiles at a time (rows padded by 16 bytes) and read back
            // row-major, so that the loads and stores of the residual cover whole 128-byte lines.
            constexpr int CG = (TN % 2 == 0) ? 2 : 1;          // column tiles per staged group (rows of 256 / 128 bytes)
            constexpr int CH = CG * 8;                         // 16-byte chunks (4 floats) per staged row
            constexpr int kStageRow = (CH + 1) * 16;
            constexpr int NQ = 32 * CH / 64;                   // chunks per lane per group
            const int l32 = lane & 31;
            const float* __restrict__ gbase = gate.base;
#pragma unroll
            for (int i = 0; i < TM; ++i) {
                const int gm_blk = gm_lane - l32 + i * 32;     // first row of the block (wave-uniform)
                // one sample for the whole block (the usual case: rows per sample a multiple of 32)?
                const int s_first = gm_blk / gate.rows_per_sample;
                const bool one_sample = (gm_blk + 31) / gate.rows_per_sample == s_first;
                // kPrep: sums of x and x^2 over this wavefront's 128 columns, for the rows 4 q + lane / 16 of the block
                // (ps[2 q], ps[2 q + 1]); this lane adds the four columns of its chunk in each staged group
                [[maybe_unused]] float ps[2 * NQ];
                if constexpr (kPrep) {
#pragma unroll
                    for (int k = 0; k < 2 * NQ; ++k) ps[k] = 0.f;
                }
#pragma unroll
                for (int jg = 0; jg < TN; jg += CG) {
#pragma unroll
                    for (int jj = 0; jj < CG; ++jj)
#pragma unroll
                        for (int e4 = 0; e4 < 4; ++e4) {
                            const f32x4_t v = {acc[i][jg + jj][4 * e4], acc[i][jg + jj][4 * e4 + 1],
                                               acc[i][jg + jj][4 * e4 + 2], acc[i][jg + jj][4 * e4 + 3]};
                            // columns jj*32 + 8 e4 + 4 lhi .. +3 -> chunk 8 jj + 2 e4 + lhi
                            *reinterpret_cast<f32x4_t*>(wave_lds + l32 * kStageRow + ((8 * jj + 2 * e4 + lhi) << 4)) = v;
                        }
                    // batches of 4 chunks per lane: all loads of a batch before its first store, and few
                    // enough registers beside the accumulators.  A lane's chunks of a group are the same four
                    // columns of different rows (64 % CH == 0), so the bias and - when the block lies in one sample -
                    // the gate and the next scale are loaded once per group, not once per chunk: per chunk they
                    // would quadruple what the epilogue pulls through the L1.
                    constexpr int QN = (QB > 0 && QB < NQ) ? QB : NQ;
                    static_assert(NQ % QN == 0 && 64 % CH == 0, "whole batches; one chunk column per lane");
                    const int gn = gn_wave + jg * 32 + (lane % CH) * 4;
                    f32x4_t bvc = {0.f, 0.f, 0.f, 0.f}, gc = {0.f, 0.f, 0.f, 0.f};
                    [[maybe_unused]] f32x4_t snc = {0.f, 0.f, 0.f, 0.f};
                    if (gn < N) {
                        bvc = *reinterpret_cast<const f32x4_t*>(bias + gn);
                        if constexpr (kResid) {
                            if (one_sample) {
                                gc = *reinterpret_cast<const f32x4_t*>(gbase + static_cast<int64_t>(s_first) * gate.stride + gn);
                                if constexpr (kPrep)
                                    snc = *reinterpret_cast<const f32x4_t*>(ln.scale_next + static_cast<int64_t>(s_first) * gate.stride + gn);
                            }
                        }
                    }
#pragma unroll
                    for (int q0 = 0; q0 < NQ; q0 += QN) {
                        f32x4_t r[QN], g[QN];
                        [[maybe_unused]] f32x4_t sn[QN];
                        int64_t off[QN];
                        bool ok[QN];
#pragma unroll
                        for (int q = 0; q < QN; ++q) {
                            const int f = (q0 + q) * 64 + lane;
                            const int gm = gm_blk + f / CH;
                            ok[q] = gm < M && gn < N;
                            off[q] = static_cast<int64_t>(gm) * N + gn;
                            g[q] = gc;
                            if constexpr (kPrep) sn[q] = snc;
                            if (ok[q]) {
                                if constexpr (kResid) {
                                    r[q] = *reinterpret_cast<const f32x4_t*>(resid + off[q]);
                                    if (!one_sample) {
                                        const int64_t so = static_cast<int64_t>(gm / gate.rows_per_sample) * gate.stride + gn;
                                        g[q] = *reinterpret_cast<const f32x4_t*>(gbase + so);
                                        if constexpr (kPrep) sn[q] = *reinterpret_cast<const f32x4_t*>(ln.scale_next + so);
                                    }
                                }
                            }
                        }
#pragma unroll
                        for (int q = 0; q < QN; ++q)
                            if (ok[q]) {
                                const int f = (q0 + q) * 64 + lane;
                                const f32x4_t v = *reinterpret_cast<const f32x4_t*>(wave_lds + (f / CH) * kStageRow + ((f % CH) << 4));
                                if constexpr (kResid) {
#pragma unroll
                                    for (int c = 0; c < 4; ++c) r[q][c] = fmaf(g[q][c], v[c] + bvc[c], r[q][c]);
                                    *reinterpret_cast<f32x4_t*>(resid + off[q]) = r[q];
                                    if constexpr (kPrep) {
                                        const u32x2_t zz = {pack2(r[q][0] * (1.0f + sn[q][0]), r[q][1] * (1.0f + sn[q][1])),
                                                            pack2(r[q][2] * (1.0f + sn[q][2]), r[q][3] * (1.0f + sn[q][3]))};
                                        *reinterpret_cast<u32x2_t*>(static_cast<bf16_t*>(ln.z) + off[q]) = zz;
                                        ps[2 * (q0 + q)] += (r[q][0] + r[q][1]) + (r[q][2] + r[q][3]);
                                        ps[2 * (q0 + q) + 1] += (r[q][0] * r[q][0] + r[q][1] * r[q][1]) +
                                                                (r[q][2] * r[q][2] + r[q][3] * r[q][3]);
                                    }
                                } else {
#pragma unroll
                                    for (int c = 0; c < 4; ++c) {
                                        r[q][c] = v[c] + bvc[c];
                                        if (kGelu) r[q][c] = gelu_fast(r[q][c]);
                                    }
                                    *reinterpret_cast<f32x4_t*>(reinterpret_cast<float*>(out) + off[q]) = r[q];
                                }
                            }
                    }
                }
                if constexpr (kPrep) {
                    // The 16 lanes that share lane / 16 hold partial sums ps[k] of the same rows 4 q + lane / 16
                    // (k = 2 q + 0 / 1): a halving exchange (each step a lane keeps the half of its
                    // values whose index bit matches its lane bit and adds the partner's) leaves sum k in the
                    // lane with lane % 16 == k.  Fixed order: the result does not depend on timing.
                    float w8[8], w4[4], w2[2];
                    const bool b3 = lane & 8, b2 = lane & 4, b1 = lane & 2, b0 = lane & 1;
#pragma unroll
                    for (int k = 0; k < 8; ++k) {
                        const float keep = b3 ? ps[8 + k] : ps[k], give = b3 ? ps[k] : ps[8 + k];
                        w8[k] = keep + __shfl_xor(give, 8, 64);
                    }
#pragma unroll
                    for (int k = 0; k < 4; ++k) {
                        const float keep = b2 ? w8[4 + k] : w8[k], give = b2 ? w8[k] : w8[4 + k];
                        w4[k] = keep + __shfl_xor(give, 4, 64);
                    }
#pragma unroll
                    for (int k = 0; k < 2; ++k) {
                        const float keep = b1 ? w4[2 + k] : w4[k], give = b1 ? w4[k] : w4[2 + k];
                        w2[k] = keep + __shfl_xor(give, 2, 64);
                    }
                    const float keep = b0 ? w2[1] : w2[0], give = b0 ? w2[0] : w2[1];
                    const float total = keep + __shfl_xor(give, 1, 64);
                    const int k = lane & 15;                       // = 2 q + (0: sum, 1: sum of squares)
                    const int gm = gm_blk + 4 * (k >> 1) + (lane >> 4);
                    if (gm < M && gn_wave < N)
                        ln.stats[(static_cast<int64_t>(gm) * ln.slots + gn_wave / kLnSlotCols) * 2 + (k & 1)] = total;
                }
            }
        } else {
            // bf16 output.  In the accumulator layout a row lives in two lanes only, so a direct store
            // touches 32 rows x 32 bytes per instruction (partial cache lines).  Each 32-row block is
            // instead packed to bf16, staged in a wave-private LDS region (rows padded by 16 bytes: the
            // 16 lanes of a ds_write_b128 pass hit 16 distinct bank groups) and read back row-major, so
            // that consecutive lanes store consecutive 16-byte chunks of whole output rows.
            constexpr int CH = TN * 4;                         // 16-byte chunks per staged row
            constexpr int kStageRow = (CH + 1) * 16;           // bytes per staged row
            const int l32 = lane & 31;
            [[maybe_unused]] f32x4_t blo[kLn ? 1 : TN][2], bhi[kLn ? 1 : TN][2];
            if constexpr (!kLn) {
#pragma unroll
                for (int j = 0; j < TN; ++j)
#pragma unroll
                    for (int e8 = 0; e8 < 2; ++e8) {
                        // this lane's two runs: n = nb + 4 lhi + {0..3} (lo) and nb + 8 + 4 lhi + {0..3} (hi);
                        // nb is a multiple of 16 and N of 8, so nb < N covers the lo run and nb + 8 < N the hi run
                        const int nb = gn_wave + j * 32 + 16 * e8;
                        blo[j][e8] = f32x4_t{0.f, 0.f, 0.f, 0.f};
                        bhi[j][e8] = f32x4_t{0.f, 0.f, 0.f, 0.f};
                        if (nb < N) blo[j][e8] = *reinterpret_cast<const f32x4_t*>(bias + nb + 4 * lhi);
                        if (nb + 8 < N) bhi[j][e8] = *reinterpret_cast<const f32x4_t*>(bias + nb + 8 + 4 * lhi);
                    }
            }
#pragma unroll
            for (int i = 0; i < TM; ++i) {
#pragma unroll
                for (int j = 0; j < TN; ++j)
#pragma unroll
                    for (int e8 = 0; e8 < 2; ++e8) {
                        float v[8];
                        if constexpr (kLn) {
#pragma unroll
                            for (int c = 0; c < 8; ++c) v[c] = ln_a[i] * acc[i][j][8 * e8 + c];
                        } else {
#pragma unroll
                            for (int c = 0; c < 4; ++c) {
                                v[c] = acc[i][j][8 * e8 + c] + blo[j][e8][c];
                                v[4 + c] = acc[i][j][8 * e8 + 4 + c] + bhi[j][e8][c];
                            }
                        }
                        if (kGelu) {
#pragma unroll
                            for (int c = 0; c < 8; ++c) v[c] = gelu_fast(v[c]);
                        }
                        uint32_t lo0 = pack2(v[0], v[1]), lo1 = pack2(v[2], v[3]);
                        uint32_t hi0 = pack2(v[4], v[5]), hi1 = pack2(v[6], v[7]);
                        // lower half-wave keeps its lo run and receives the partner's lo run (n+4..7);
                        // upper half-wave receives the partner's hi run (n+8..11) and keeps its own hi run
                        const u32x2_t s0 = __builtin_amdgcn_permlane32_swap(lo0, hi0, false, false);
                        const u32x2_t s1 = __builtin_amdgcn_permlane32_swap(lo1, hi1, false, false);
                        const u32x4_t o = {s0[0], s1[0], s0[1], s1[1]};
                        // row l32 of the block, columns j*32 + 16*e8 + 8*lhi .. +7 -> chunk 4j + 2 e8 + lhi
                        *reinterpret_cast<u32x4_t*>(wave_lds + l32 * kStageRow + ((4 * j + 2 * e8 + lhi) << 4)) = o;
                    }
                // read back: flat chunk f = q*64 + lane over 32 rows x CH chunks
#pragma unroll
                for (int q = 0; q < (32 * CH + 63) / 64; ++q) {
                    const int f = q * 64 + lane;
                    const int row = f / CH, ch = f % CH;
                    if ((32 * CH) % 64 != 0 && f >= 32 * CH) continue;
                    const u32x4_t o = *reinterpret_cast<const u32x4_t*>(wave_lds + row * kStageRow + (ch << 4));
                    const int gm = gm_lane - l32 + i * 32 + row, gn = gn_wave + ch * 8;
                    if (gm < M && gn < N)
                        *reinterpret_cast<u32x4_t*>(reinterpret_cast<bf16_t*>(out) + static_cast<int64_t>(gm) * N + gn) = o;
                }
            }
        }
        return;
    }
    // unaligned output: element-wise with bounds checks (the folded-LayerNorm epilogues are launched on
    // aligned shapes only)
    if constexpr (kLn || kPrep) return;
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
        for (int i = 0; i < TM; ++i) {
            const int gm = gm_lane + i * 32;
            if (gm >= M) continue;
#pragma unroll
            for (int e = 0; e < 16; ++e) {
                const int gn = gn_wave + j * 32 + 8 * (e >> 2) + 4 * lhi + (e & 3);
                if (gn >= N) continue;
                const float v = acc[i][j][e] + bias[gn];
                const int64_t o = static_cast<int64_t>(gm) * N + gn;
                if (EPI == FREE_EPI_BIAS) {
                    store_f(out + o, v);
                } else if (EPI == FREE_EPI_BIAS_GELU) {
                    store_f(out + o, gelu_fast(v));
                } else {
                    const float g = gate.base[static_cast<int64_t>(gm / gate.rows_per_sample) * gate.stride + gn];
                    resid[o] = fmaf(g, v, resid[o]);
                }
            }
        }
}

// T: bf16_t or float (operands and the output of the bias / GELU epilogues).  EVEN_K: K a multiple of the
// slice (64 bf16 or 32 fp32: no predicates in the K loop).  Rows past the end of a ragged M / N tile read
// as zero (extra rows are computed, never stored).
template <typename T, int BM, int BN, int WGM, int WGN, int EPI, bool EVEN_K>
__global__ __launch_bounds__(WGM * WGN * 64) void gemm_bf16_kernel(
    const T* __restrict__ X, const T* __restrict__ W, const float* __restrict__ bias, int32_t M,
    int32_t N, int32_t K, int32_t tiles_m, int32_t tiles_n, int32_t group_m, int32_t vec_ok,
    T* __restrict__ out, float* __restrict__ resid, RowVec gate, LnFold ln) {
    static_assert(WGM * WGN == 4 || WGM * WGN == 8, "four or eight wavefronts per workgroup");
    constexpr bool kF32 = std::is_same<T, float>::value;
    constexpr int ES = static_cast<int>(sizeof(T));    // bytes per element
    constexpr int BKE = kRowBytes / ES;                // elements per K slice
    constexpr int CE = 16 / ES;                        // elements per 16-byte chunk
    constexpr int NT = WGM * WGN * 64;                 // threads per workgroup
    constexpr int RP = NT / 8;                         // tile rows covered by one pass of 16-byte loads
    constexpr int TM = BM / WGM / 32, TN = BN / WGN / 32;
    constexpr int LA = BM / RP, LB = BN / RP;          // 16-byte loads per thread per slice
    constexpr int kStageBytes = (BM + BN) * kRowBytes;
    extern __shared__ __attribute__((aligned(16))) char lds[];

    int tile_m, tile_n;
    tile_coords(group_m, blockIdx.x, tiles_m, tiles_n, &tile_m, &tile_n);
    const int m0 = tile_m * BM, n0 = tile_n * BN;
    // (the wavefront index as a scalar: the position of the wavefront's part of the tile, the test for an all-padding
    // wavefront and the LDS offsets that follow from it stay in scalar registers)
    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm = wave / WGN, wn = wave % WGN;

    // ---- global -> register staging: chunk idx = i*NT + tid, row = idx/8, chunk = idx%8
    const int ld_chunk = tid & 7;
    const int ld_row = tid >> 3;
    // Buffer descriptors over the rows of this tile: a load past the end of the matrix (rows
    // of a ragged edge tile) returns zeros, so no row clamping and no address registers -
    // one per-lane byte offset plus wave-uniform (scalar) offsets per load and per slice.
    const int64_t x_left = static_cast<int64_t>(M - m0) * K * ES, w_left = static_cast<int64_t>(N - n0) * K * ES;
    const __amdgpu_buffer_rsrc_t xsrd = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<T*>(X + static_cast<int64_t>(m0) * K), 0,
        static_cast<int>(x_left < 0x7fffffff ? x_left : 0x7fffffff), 0x00020000);
    const __amdgpu_buffer_rsrc_t wsrd = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<T*>(W + static_cast<int64_t>(n0) * K), 0,
        static_cast<int>(w_left < 0x7fffffff ? w_left : 0x7fffffff), 0x00020000);
    const int ld_voff = ld_row * K * ES + ld_chunk * 16;      // per-lane byte offset inside the tile
    const int pass_bytes = RP * K * ES;                       // RP rows further down per load index
    const int st_off = ld_row * kRowBytes + ((ld_chunk ^ ((ld_row >> 1) & 7)) << 4);   // + i*RP rows per load
    u32x4_t sreg[LA + LB];                              // staging registers: one K slice in flight
    const int nk = (K + BKE - 1) / BKE;

    // staging register idx in [0, LA + LB): the first LA hold X rows, the rest W rows
    constexpr int NS = LA + LB;
    auto fetch_range = [&](int kt, int lo, int hi) {
        const int kbyte = kt * kRowBytes;
        const bool in_k = EVEN_K || (kt * BKE + ld_chunk * CE) < K;   // K a multiple of the chunk: all in or all out
#pragma unroll
        for (int idx = 0; idx < NS; ++idx) {
            if (idx < lo || idx >= hi) continue;
            const u32x4_t v = (idx < LA)
                                  ? __builtin_amdgcn_raw_buffer_load_b128(xsrd, ld_voff, idx * pass_bytes + kbyte, 0)
                                  : __builtin_amdgcn_raw_buffer_load_b128(wsrd, ld_voff, (idx - LA) * pass_bytes + kbyte, 0);
            sreg[idx] = in_k ? v : u32x4_t{0, 0, 0, 0};
        }
    };
    auto stash_range = [&](int stage, int lo, int hi) {
        char* base = lds + stage * kStageBytes + st_off;
#pragma unroll
        for (int idx = 0; idx < NS; ++idx) {
            if (idx < lo || idx >= hi) continue;
            const int row = (idx < LA) ? idx * RP : BM + (idx - LA) * RP;
            *reinterpret_cast<u32x4_t*>(base + row * kRowBytes) = sreg[idx];
        }
    };

    // ---- MFMA operand fragments: row fixed per lane, chunk varies with the k step
    const int l32 = lane & 31, lhi = lane >> 5;
    const int sw = (l32 >> 1) & 7;                         // (row / 2) % 8 (tile row offsets are multiples of 32)
    const int x_row0 = (wm * TM * 32 + l32) * kRowBytes;           // + i*32 rows
    const int w_row0 = (BM + wn * TN * 32 + l32) * kRowBytes;      // + j*32 rows
    u32x4_t fx[2][TM], fw[2][TN];                      // one 16-byte chunk each: 8 bf16 or 4 fp32
    // A wavefront whose part of the tile lies wholly past N or M (N = 1152 is 4.5 tiles of 256 columns: the right
    // half of every fifth tile) takes part in the staging and the barriers only: its products would be thrown
    // away, and on a chip that runs at its power limit they are not free for the others.
    // (bf16 only: in the fp32 instantiation, whose K loop is matrix-bound, the branch costs 4 % on every launch)
    // How the test enters the K loop depends on the wavefronts a SIMD holds.  Eight-wavefront workgroups (two per
    // SIMD) keep it inside the loop: it splits the body into basic blocks, each k-step becomes "LDS traffic, wait
    // for all of it, eight products", and the two wavefronts of a SIMD alternate - measured faster than the
    // interleaved form.  Four-wavefront workgroups (one per SIMD: the tiles of problems with few rows) have nobody
    // to alternate with: there the wait for the NEXT step's fragments in front of every burst is pure latency
    // (measured 0.66 us per slice for 0.22 us of products), so they take one of two straight-line copies of the
    // loop (with / without products, chosen once), in which the compiler counts the LDS reads in flight and the
    // products of a step overlap the reads of the next.
    const bool wave_on = kF32 || ((n0 + wn * TN * 32 < N) && (m0 + wm * TM * 32 < M));
    constexpr bool kStraight = !kF32 && WGM * WGN <= 4;
    struct InLoop {};                                  // tag: test the flag inside the loop
    auto is_on = [&](auto tag) {
        if constexpr (std::is_same<decltype(tag), InLoop>::value) return wave_on;
        else return decltype(tag)::value;
    };
    auto load_frags = [&](const char* base, int ks, int buf, auto tag) {
        if (!is_on(tag)) return;
        const int choff = (((ks << 1) | lhi) ^ sw) << 4;
#pragma unroll
        for (int i = 0; i < TM; ++i)
            fx[buf][i] = *reinterpret_cast<const u32x4_t*>(base + x_row0 + i * 32 * kRowBytes + choff);
#pragma unroll
        for (int j = 0; j < TN; ++j)
            fw[buf][j] = *reinterpret_cast<const u32x4_t*>(base + w_row0 + j * 32 * kRowBytes + choff);
    };

    f32x16_t acc[TM][TN];                                  // acc[i][j]: rows n (tile j), columns m (tile i)
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;
    constexpr bool kLnEpi = EPI == FREE_EPI_LN_BIAS || EPI == FREE_EPI_LN_BIAS_GELU;
    [[maybe_unused]] float ln_a[TM];                       // folded LayerNorm: r of this lane's rows

    auto mma = [&](int buf, auto tag) {
        if (!is_on(tag)) return;
        if constexpr (kF32) {
            // element e of the chunk: the lanes of group 0 / 1 hold the two k of one 32x32x2 product
#pragma unroll
            for (int e = 0; e < 4; ++e)
#pragma unroll
                for (int i = 0; i < TM; ++i)
#pragma unroll
                    for (int j = 0; j < TN; ++j) {
                        // (copied out first: a bit cast applied directly to a vector element read element 0)
                        const uint32_t wbits = fw[buf][j][e], xbits = fx[buf][i][e];
                        acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(__builtin_bit_cast(float, wbits),
                                                                        __builtin_bit_cast(float, xbits),
                                                                        acc[i][j], 0, 0, 0);
                    }
        } else {
#pragma unroll
            for (int i = 0; i < TM; ++i)
#pragma unroll
                for (int j = 0; j < TN; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8_t, fw[buf][j]),
                                                                        __builtin_bit_cast(bf16x8_t, fx[buf][i]),
                                                                        acc[i][j], 0, 0, 0);
        }
    };
    // One K slice.  Precondition: fragments of k-step 0 are in buffer 0.  The staging
    // registers hold slice kt+1; they are written to the other LDS stage in three
    // portions (k-steps 0..2), and each freed portion is immediately refilled with the
    // global loads of slice kt+2.  Spreading the LDS writes matters: the LDS write path
    // is much narrower than the read path, a burst of 16 writes per lane stalls issue.
    //   k-step 0..2: multiply | read fragments of the next step | write + refill a third
    //   barrier: the other stage is complete, this stage will not be read again
    //   k-step 3: multiply | read fragments of step 0 of slice kt+1 from the other stage
    constexpr int MF = TM * TN * (kF32 ? 4 : 1), NR = TM + TN;
    constexpr int C1 = (NS + 2) / 3, C2 = (2 * NS + 2) / 3;      // portion boundaries
    auto slice = [&](int kt, auto stash_next, auto fetch_ahead, auto tag) {
        constexpr bool kStash = decltype(stash_next)::value, kFetch = decltype(fetch_ahead)::value;
        const char* base = lds + (kt & 1) * kStageBytes;
        const int nst = (kt + 1) & 1;
        load_frags(base, 1, 1, tag);
        if (kStash) stash_range(nst, 0, C1);
        if (kFetch) fetch_range(kt + 2, 0, C1);
        mma(0, tag);
        sched_hints<0, MF, NR, kStash ? C1 : 0, kFetch ? C1 : 0>();
        load_frags(base, 2, 0, tag);
        if (kStash) stash_range(nst, C1, C2);
        if (kFetch) fetch_range(kt + 2, C1, C2);
        mma(1, tag);
        sched_hints<0, MF, NR, kStash ? C2 - C1 : 0, kFetch ? C2 - C1 : 0>();
        load_frags(base, 3, 1, tag);
        if (kStash) stash_range(nst, C2, NS);
        if (kFetch) fetch_range(kt + 2, C2, NS);
        mma(0, tag);
        sched_hints<0, MF, NR, kStash ? NS - C2 : 0, kFetch ? NS - C2 : 0>();
        __syncthreads();
        if (kStash) load_frags(lds + nst * kStageBytes, 0, 0, tag);
        mma(1, tag);
        sched_hints<0, MF, kStash ? NR : 0, 0, 0>();
    };
    const std::true_type yes{};
    const std::false_type no{};

    // ---- prologue: slice 0 through the registers into LDS stage 0, slice 1 into the registers
    fetch_range(0, 0, NS);
    // Folded LayerNorm: with mu and rho = sqrt(var + eps) of a row, the output is (z W^T - mu c1 + rho c0) / rho.
    // The rank-2 term -mu c1 + rho c0 is one extra k-step of the matrix product, issued in this prologue: row m
    // contributes the k-vector (-mu_h, -mu_l, -mu_h, rho_h, rho_l, rho_h, 0 ...), column n the k-vector
    // (c1_h, c1_h, c1_l, c0_h, c0_h, c0_l, 0 ...), with _h the bf16 value and _l the bf16 value of the remainder
    // (the product of two remainders, 2^-18 relative, is dropped).  Its loads - the partial sums of this lane's
    // rows, c1 / c0 of its columns - are requested right behind slice 0 and consumed while slice 1 is in flight;
    // nothing of it stays in registers through the K loop except 1 / rho per row, which the epilogue multiplies by.
    // Every 32-row block lies in one sample (rows per sample a multiple of 32).  The lower half-wave adds the first
    // half of a row's slots in index order, the upper one the rest, then the two sums are added - a fixed order.
    constexpr int kHalfSlots = 8;                          // up to 16 slots: rows of up to 2048 values
    [[maybe_unused]] float2 ln_p[kLnEpi ? TM : 1][kHalfSlots];
    [[maybe_unused]] float ln_c1[kLnEpi ? TM : 1][TN], ln_c0[kLnEpi ? TM : 1][TN];
    [[maybe_unused]] int ln_kn = 0;
    if constexpr (kLnEpi) {
        const int rps = ln.rows_per_sample;
        const int half = (ln.slots + 1) / 2;
        const int k0 = lhi ? half : 0;
        ln_kn = lhi ? ln.slots - half : half;              // this half-wave's slots
#pragma unroll
        for (int i = 0; i < TM; ++i) {
            const int gm_blk = m0 + wm * TM * 32 + i * 32;
            const int gm = gm_blk + l32;
            // (rows past M and slots past the end re-read a valid entry with weight zero: no branches)
            const float2* st = reinterpret_cast<const float2*>(ln.stats) + static_cast<int64_t>(gm < M ? gm : M - 1) * ln.slots;
#pragma unroll
            for (int k = 0; k < kHalfSlots; ++k) ln_p[i][k] = st[k0 + (k < ln_kn ? k : 0)];
            // c1 / c0 of this block's sample: loaded again only where the sample changes (wave-uniform)
            const int smp = (gm_blk < M ? gm_blk : M - 1) / rps;
            const int smp_prev = i == 0 ? -1 : ((gm_blk - 32 < M ? gm_blk - 32 : M - 1) / rps);
#pragma unroll
            for (int j = 0; j < TN; ++j) {
                if (smp != smp_prev) {
                    const int n = n0 + wn * TN * 32 + j * 32 + l32;
                    const int64_t o = static_cast<int64_t>(smp) * ln.fold_stride + (n < N ? n : 0);
                    ln_c1[i][j] = ln.c1[o];
                    ln_c0[i][j] = ln.c0[o];
                } else {
                    ln_c1[i][j] = ln_c1[i > 0 ? i - 1 : 0][j];
                    ln_c0[i][j] = ln_c0[i > 0 ? i - 1 : 0][j];
                }
            }
        }
    }
    stash_range(0, 0, NS);
    if (nk > 1) fetch_range(1, 0, NS);
    if constexpr (kLnEpi) {
        const auto split = [](float v, float* hi, float* lo) {
            *hi = __uint_as_float(pack2(v, 0.f) << 16);
            *lo = v - *hi;
        };
#pragma unroll
        for (int i = 0; i < TM; ++i) {
            float s1 = 0.f, s2 = 0.f;
#pragma unroll
            for (int k = 0; k < kHalfSlots; ++k) {
                s1 += k < ln_kn ? ln_p[i][k].x : 0.f;
                s2 += k < ln_kn ? ln_p[i][k].y : 0.f;
            }
            const float o1 = __shfl_xor(s1, 32, 64), o2 = __shfl_xor(s2, 32, 64);
            s1 = lhi ? o1 + s1 : s1 + o1;                  // first half + second half in both lanes
            s2 = lhi ? o2 + s2 : s2 + o2;
            const float mean = s1 * ln.inv_width;
            const float var = fmaxf(s2 * ln.inv_width - mean * mean, 0.f);
            ln_a[i] = rsqrtf(var + kLnEps);
            float mh, ml, rh, rl;
            split(-mean, &mh, &ml);
            split(1.0f / ln_a[i], &rh, &rl);
            const u32x4_t xk = lhi ? u32x4_t{0, 0, 0, 0} : u32x4_t{pack2(mh, ml), pack2(mh, rh), pack2(rl, rh), 0};
#pragma unroll
            for (int j = 0; j < TN; ++j) {
                const int n = n0 + wn * TN * 32 + j * 32 + l32;
                float c1h, c1l, c0h, c0l;
                split(n < N ? ln_c1[i][j] : 0.f, &c1h, &c1l);
                split(n < N ? ln_c0[i][j] : 0.f, &c0h, &c0l);
                const u32x4_t wk = lhi ? u32x4_t{0, 0, 0, 0} : u32x4_t{pack2(c1h, c1h), pack2(c1l, c0h), pack2(c0h, c0l), 0};
                acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8_t, wk),
                                                                    __builtin_bit_cast(bf16x8_t, xk), acc[i][j], 0, 0, 0);
            }
        }
    }
    __syncthreads();
    // ---- steady state: slice kt multiplies while slice kt+1 moves registers -> LDS and
    //      slice kt+2 is requested from global memory
    auto k_loop = [&](auto tag) {
        load_frags(lds, 0, 0, tag);
        int kt = 0;
        for (; kt + 2 < nk; ++kt) slice(kt, yes, yes, tag);
        if (kt + 1 < nk) {
            slice(kt, yes, no, tag);
            ++kt;
        }
        slice(kt, no, no, tag);
    };
    if constexpr (kF32) {
        k_loop(yes);
    } else if constexpr (kStraight) {
        if (wave_on) k_loop(yes);
        else k_loop(no);
    } else {
        k_loop(InLoop{});
    }

    // ---- epilogue
    // after the barrier of the last slice no wavefront reads the LDS tiles any more: each wavefront
    // may use a private region of them to transpose its output
    constexpr bool kResidEpi = EPI == FREE_EPI_GATE_RESID || EPI == FREE_EPI_GATE_RESID_PREP;
    constexpr int kWaveStage = (kResidEpi || kF32) ? 32 * (((TN % 2 == 0 ? 2 : 1) * 8 + 1) * 16)   // fp32 groups
                                                   : 32 * (TN * 64 + 16);                            // bf16 rows
    static_assert(WGM * WGN * kWaveStage <= 2 * kStageBytes, "output staging must fit in the K-loop tiles");
    constexpr int kResidBatch = (WGM * WGN == 8) ? 4 : 0;
    float ln_scale[TM];
#pragma unroll
    for (int i = 0; i < TM; ++i) ln_scale[i] = 1.0f;
    if constexpr (kLnEpi) {
#pragma unroll
        for (int i = 0; i < TM; ++i) ln_scale[i] = ln_a[i];
    }
    write_tile<T, TM, TN, EPI, kResidBatch>(acc, m0 + wm * TM * 32 + l32, n0 + wn * TN * 32, lane, M, N, vec_ok, bias, out, resid, gate,
                            lds + wave * kWaveStage, ln, ln_scale);
}

int device_cus() {
    static int cus = [] {
        int dev = 0, n = 0;
        if (hipGetDevice(&dev) != hipSuccess ||
            hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n < 1)
            n = 256;
        return n;
    }();
    return cus;
}

template <typename T, int BM, int BN, int WGM, int WGN, int EPI, bool EVEN_K>
int32_t launch_one(const T* X, const T* W, const float* bias, int32_t M, int32_t N, int32_t K, T* out,
                   float* resid, RowVec gate, hipStream_t s, const LnFold& ln = LnFold{}) {
    const int tiles_m = (M + BM - 1) / BM, tiles_n = (N + BN - 1) / BN;
    const size_t lds = 2 * static_cast<size_t>(BM + BN) * kRowBytes;
    auto kern = gemm_bf16_kernel<T, BM, BN, WGM, WGN, EPI, EVEN_K>;
    static bool attr_set = false;
    if (!attr_set) {
        if (!hip_ok(hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                                        hipFuncAttributeMaxDynamicSharedMemorySize, static_cast<int>(lds))))
            return FREE_ERR_HIP;
        attr_set = true;
    }
    // the vector epilogue needs 16-byte aligned rows of out / resid / bias / gate
    auto al16 = [](const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; };
    const bool vec = ((N & 7) == 0) && al16(bias) && al16(out) && al16(resid) && al16(gate.base) &&
                     ((gate.stride & 3) == 0);
    const int32_t vec_ok = vec ? 1 : 0;
    // Row tiles per group of the tile order.  Several rounds of workgroups: the 32 that run together on an
    // XCD should cover a x b tiles with a BM ~ b BN, the shape that needs the fewest distinct X and W panels
    // (first-touch misses of that XCD's L2).  A single round: every XCD holds total / 8 tiles for the whole
    // kernel, and a group of exactly that many tiles - whole tile rows - keeps each X panel in one L2
    // (FC2 at 12288 rows: 361 MB fetched with groups of 8 row tiles, X read by two or three XCDs each).
    // This is about traffic, not time: the Infinity Cache served the repeats at no measurable cost.
    const int total = tiles_m * tiles_n;
    int group_m = BM > BN ? 4 : 8;
    if (total <= device_cus()) {
        const int per_xcd = (total + kNumXcd - 1) / kNumXcd;
        group_m = std::max(1, (per_xcd + tiles_n / 2) / tiles_n);
    }
    if ((EPI == FREE_EPI_LN_BIAS || EPI == FREE_EPI_LN_BIAS_GELU || EPI == FREE_EPI_GATE_RESID_PREP) && !vec)
        return FREE_ERR_SHAPE;                                   // the folded-LayerNorm epilogues have no element-wise form
    hipLaunchKernelGGL(kern, dim3(total), dim3(WGM * WGN * 64), lds, s, X, W, bias, M, N, K, tiles_m, tiles_n, group_m,
                       vec_ok, out, resid, gate, ln);
    return launch_ok() ? FREE_OK : FREE_ERR_HIP;
}

template <typename T, int BM, int BN, int WGM, int WGN>
int32_t launch_cfg(const T* X, const T* W, const float* bias, int32_t M, int32_t N, int32_t K,
                   int32_t epi, T* out, float* resid, RowVec gate, hipStream_t s) {
    const bool even = (K % (kRowBytes / static_cast<int>(sizeof(T)))) == 0;
#define FREE_GEMM_CASE(E)                                                                                    \
    case E:                                                                                                  \
        return even ? launch_one<T, BM, BN, WGM, WGN, E, true>(X, W, bias, M, N, K, out, resid, gate, s)     \
                    : launch_one<T, BM, BN, WGM, WGN, E, false>(X, W, bias, M, N, K, out, resid, gate, s)
    switch (epi) {
        FREE_GEMM_CASE(FREE_EPI_BIAS);
        FREE_GEMM_CASE(FREE_EPI_BIAS_GELU);
        FREE_GEMM_CASE(FREE_EPI_GATE_RESID);
        default: return FREE_ERR_RANGE;
    }
#undef FREE_GEMM_CASE
}

// Estimated time (us) of a tile configuration on `cus` compute units: workgroup rounds times
// (K slices x measured time per slice + per-tile prologue/epilogue), measured on MI355X in bf16 (one machine's
// microseconds: machines of the type differ by a few per cent, and half-share launches reuse them).  nk: 128-byte
// K slices; slice_scale: time of a slice relative to bf16 (fp32: 4.4 - four 16-pass MFMAs per chunk pair instead of
// one 8-pass MFMA, at the slightly higher clock the fp32 products leave).
double cfg_time(int M, int N, int nk, int bm, int bn, double us_per_slice, double us_fixed, int cus) {
    const double tiles = static_cast<double>((M + bm - 1) / bm) * ((N + bn - 1) / bn);
    const double rounds = std::ceil(tiles / cus);
    return rounds * (nk * us_per_slice + us_fixed);
}

// The 128x128 configuration is small enough for two workgroups per CU: measured 0.6 us per slice for a
// workgroup that has its CU to itself and 1.05 us each for two that share one.  Used for problems of
// few rows (the drafter, single-state steps), where it decides between half-empty rounds of large
// tiles and fuller rounds of small ones.
double small_tile_time(int M, int N, int nk, double sc, int cus) {
    const double tiles = static_cast<double>((M + 127) / 128) * ((N + 127) / 128);
    const double shared = nk * 1.05 * sc + 4.0, alone = nk * 0.6 * sc + 4.0;
    const double full = std::floor(tiles / (2.0 * cus));
    const double rest = tiles - full * 2.0 * cus;
    return full * shared + (rest == 0.0 ? 0.0 : (rest <= cus ? alone : shared));
}

// cu_share: how many launches of this size are expected to run side by side (the halves of a packed batch on two
// streams); the tile configuration is chosen for that share of the compute units.  Tiles change how the output
// is cut, never the order in which a dot product is summed, so the result does not depend on it.
template <typename T>
int32_t choose_and_launch(const T* X, const T* W, const float* bias, int32_t M, int32_t N, int32_t K, int32_t epi,
                          T* out, float* resid, RowVec gate, hipStream_t s, int cu_share, const LnFold* ln) {
    if ((reinterpret_cast<uintptr_t>(X) | reinterpret_cast<uintptr_t>(W)) & 15u) return FREE_ERR_SHAPE;
    constexpr int kSliceElems = kRowBytes / static_cast<int>(sizeof(T));
    const double sc = sizeof(T) == 4 ? 4.4 : 1.0;
    const int nk = (K + kSliceElems - 1) / kSliceElems;
    const int cus = std::max(1, device_cus() / std::max(1, cu_share));
    const double t256 = cfg_time(M, N, nk, 256, 256, 1.83 * sc, 9.0, cus);
    const double t384 = cfg_time(M, N, nk, 384, 192, 2.06 * sc, 10.0, cus);
    if (epi == FREE_EPI_LN_BIAS || epi == FREE_EPI_LN_BIAS_GELU || epi == FREE_EPI_GATE_RESID_PREP) {
        // folded LayerNorm: the two large eight-wavefront tiles only, K a whole number of slices
        if constexpr (std::is_same<T, bf16_t>::value) {
            if (ln == nullptr || K % kSliceElems != 0) return FREE_ERR_SHAPE;
            if (epi == FREE_EPI_GATE_RESID_PREP)
                return launch_one<T, 256, 256, 4, 2, FREE_EPI_GATE_RESID_PREP, true>(X, W, bias, M, N, K, out, resid, gate, s, *ln);
            if (epi == FREE_EPI_LN_BIAS)
                return t384 < t256 ? launch_one<T, 384, 192, 4, 2, FREE_EPI_LN_BIAS, true>(X, W, bias, M, N, K, out, resid, gate, s, *ln)
                                   : launch_one<T, 256, 256, 4, 2, FREE_EPI_LN_BIAS, true>(X, W, bias, M, N, K, out, resid, gate, s, *ln);
            return t384 < t256 ? launch_one<T, 384, 192, 4, 2, FREE_EPI_LN_BIAS_GELU, true>(X, W, bias, M, N, K, out, resid, gate, s, *ln)
                               : launch_one<T, 256, 256, 4, 2, FREE_EPI_LN_BIAS_GELU, true>(X, W, bias, M, N, K, out, resid, gate, s, *ln);
        } else {
            return FREE_ERR_SHAPE;
        }
    }
    const double t2x1 = cfg_time(M, N, nk, 256, 128, 1.31 * sc, 6.0, cus);
    const double t128 = M <= 4096 ? small_tile_time(M, N, nk, sc, cus) : cfg_time(M, N, nk, 128, 128, 0.80 * sc, 4.0, cus);
    // 96 x 128 (one row of four wavefronts, each 96 x 32): for problems of few rows and few columns, where
    // 128 x 128 tiles leave compute units empty (2048 x 1152: 144 tiles on 256 CUs; 198 of three quarters the work)
    double t96 = 1e30;
    {
        const double tiles = static_cast<double>((M + 95) / 96) * ((N + 127) / 128);
        if (tiles <= cus && M <= 4096) t96 = nk * 0.47 * sc + 4.0;      // measured 0.47 us per slice
    }
    // 160 x 128 (same shape of workgroup, 160 x 32 per wavefront): for few rows and many columns, where 128 x 128
    // tiles spill into a second round (2048 x 4608: 576 tiles on 512 slots; 468 of 160 x 128).  Measured about
    // 1.25 x the slice time of 128 x 128, alone and shared.
    double t160 = 1e30;
    if (M <= 4096) {
        const double tiles = static_cast<double>((M + 159) / 160) * ((N + 127) / 128);
        if (tiles <= cus) t160 = nk * 0.80 * sc + 4.0;
        else if (tiles <= 2.0 * cus) t160 = nk * 1.40 * sc + 4.0;
    }
    const double best = std::fmin(std::fmin(std::fmin(t256, t384), std::fmin(t2x1, t128)), std::fmin(t96, t160));
    if (best == t160) return launch_cfg<T, 160, 128, 1, 4>(X, W, bias, M, N, K, epi, out, resid, gate, s);
    if (best == t96) return launch_cfg<T, 96, 128, 1, 4>(X, W, bias, M, N, K, epi, out, resid, gate, s);
    if (best == t384) return launch_cfg<T, 384, 192, 4, 2>(X, W, bias, M, N, K, epi, out, resid, gate, s);
    if (best == t256) return launch_cfg<T, 256, 256, 4, 2>(X, W, bias, M, N, K, epi, out, resid, gate, s);
    if (best == t2x1) return launch_cfg<T, 256, 128, 2, 2>(X, W, bias, M, N, K, epi, out, resid, gate, s);
    return launch_cfg<T, 128, 128, 2, 2>(X, W, bias, M, N, K, epi, out, resid, gate, s);
}

}  // namespace

bool mfma_linear_supported(int32_t M, int32_t N, int32_t K) {
    // 32-bit byte offsets inside a tile: up to 384 rows of K bf16
    return M >= 1 && N >= 1 && K >= 8 && (K % 8) == 0 && static_cast<int64_t>(K) * 2 * 384 < (1ll << 31);
}

bool mfma_linear_f32_supported(int32_t M, int32_t N, int32_t K) {
    // whole 16-byte chunks of fp32; 32-bit byte offsets inside a tile: up to 384 rows of K fp32
    return M >= 1 && N >= 1 && K >= 4 && (K % 4) == 0 && static_cast<int64_t>(K) * 4 * 384 < (1ll << 31);
}

int32_t launch_linear_mfma(const bf16_t* X, const bf16_t* W, const float* bias, int32_t M, int32_t N, int32_t K,
                           int32_t epi, bf16_t* out, float* resid, RowVec gate, hipStream_t s, int cu_share,
                           const LnFold* ln) {
    if (!mfma_linear_supported(M, N, K)) return FREE_ERR_SHAPE;
    if (ln != nullptr) {
        // producer: the rows being normalised are this GEMM's output rows (width N); consumer: its input rows (width K)
        const int32_t width = epi == FREE_EPI_GATE_RESID_PREP ? N : K;
        const auto al16 = [](const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; };
        if (width % kLnSlotCols != 0 || ln->slots != width / kLnSlotCols || ln->stats == nullptr ||
            (reinterpret_cast<uintptr_t>(ln->stats) & 7u))
            return FREE_ERR_SHAPE;
        if (epi == FREE_EPI_GATE_RESID_PREP) {
            if (ln->z == nullptr || ln->scale_next == nullptr || !al16(ln->z) || !al16(ln->scale_next)) return FREE_ERR_SHAPE;
        } else {
            if (ln->c1 == nullptr || ln->c0 == nullptr || !al16(ln->c1) || !al16(ln->c0) || (ln->fold_stride & 3) ||
                ln->rows_per_sample < 32 || ln->rows_per_sample % 32 != 0)
                return FREE_ERR_SHAPE;
        }
    }
    return choose_and_launch<bf16_t>(X, W, bias, M, N, K, epi, out, resid, gate, s, cu_share, ln);
}

bool mfma_ln_fold_supported(int32_t M, int32_t D, int32_t rows_per_sample) {
    // (a 32-row block of a tile then lies in one sample; up to 16 slots of partial sums per row)
    return M >= 1 && D % kLnSlotCols == 0 && D <= 16 * kLnSlotCols && rows_per_sample >= 32 && rows_per_sample % 32 == 0;
}

int32_t launch_linear_mfma_f32(const float* X, const float* W, const float* bias, int32_t M, int32_t N, int32_t K,
                               int32_t epi, float* out, float* resid, RowVec gate, hipStream_t s, int cu_share) {
    if (!mfma_linear_f32_supported(M, N, K)) return FREE_ERR_SHAPE;
    return choose_and_launch<float>(X, W, bias, M, N, K, epi, out, resid, gate, s, cu_share, nullptr);
}

}  // namespace freemi
