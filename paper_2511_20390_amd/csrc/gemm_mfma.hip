// bf16 MFMA GEMM for the dense projections of the DiT blocks (QKV, attention
// out-projection, MLP FC1/FC2 of the packed target forward, Alg. 1):
//   C[M,N] = A[M,K] . W[N,K]^T  (+bias, fused epilogue), fp32 accumulation.
// Both operands are K-contiguous, which is exactly the per-lane operand layout of
// v_mfma_f32_32x32x16_bf16 (lane l: row/col l%32, 8 consecutive k at 8*(l/32)).
//
// Tiling (gfx950: 64-wide wavefronts, 160 KB LDS per CU, 512 VGPR+AGPR per lane):
//   workgroup = 256 threads = 4 wavefronts in a WGM x WGN grid, macro tile BM x BN,
//   K slices of 64; each wavefront owns (BM/WGM) x (BN/WGN) as TM x TN MFMA tiles
//   of 32x32, accumulators stay in registers for the whole K loop.
//   LDS: two stages of [BM + BN rows][64 bf16]; the 16-byte chunk index of every
//   row is XOR-swizzled with (row % 8) so that the 8 lanes served per LDS cycle by
//   ds_read_b128 hit 8 distinct chunk columns (no bank conflicts) while global
//   loads stay 128-byte coalesced.  The next K slice is fetched into registers
//   while the current one is multiplied (one barrier per slice).
//   Workgroup ids are remapped so that the 8 XCDs (round-robin dispatch) each work
//   on a compact, L2-friendly group of tiles.
#include <cmath>

#include "free_internal.h"

namespace freemi {

namespace {

typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef float f32x16_t __attribute__((ext_vector_type(16)));
typedef uint32_t u32x4_t __attribute__((ext_vector_type(4)));

constexpr int kThreads = 256;
constexpr int BK = 64;                    // bf16 elements per K slice (128 bytes per row)
constexpr int kRowBytes = BK * 2;
constexpr int kNumXcd = 8;
constexpr int kGroupM = 8;

__device__ inline float gelu_fast(float v) {
    // tanh-form GELU: 0.5 v (1 + tanh(u)) = v / (1 + exp(-2u)), u = sqrt(2/pi)(v + 0.044715 v^3)
    const float u = 0.7978845608028654f * (v + 0.044715f * v * v * v);
    return v * __frcp_rn(1.0f + __expf(-2.0f * u));
}

// XCD-aware tile order: workgroup ids are dealt round-robin to the 8 XCDs, so the
// ids of one XCD are made contiguous first, then walked in groups of kGroupM row
// tiles (column-major inside a group) so concurrent workgroups share A and W panels.
__device__ inline void tile_coords(int pid, int tiles_m, int tiles_n, int* tm, int* tn) {
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

template <int BM, int BN, int WGM, int WGN, int EPI>
__global__ __launch_bounds__(kThreads) void gemm_bf16_kernel(
    const bf16_t* __restrict__ A, const bf16_t* __restrict__ W, const float* __restrict__ bias, int32_t M,
    int32_t N, int32_t K, int32_t tiles_m, int32_t tiles_n, bf16_t* __restrict__ out, float* __restrict__ resid,
    RowVec gate) {
    static_assert(WGM * WGN == 4, "four wavefronts per workgroup");
    constexpr int TM = BM / WGM / 32, TN = BN / WGN / 32;
    constexpr int LA = BM / 32, LB = BN / 32;          // 16-byte loads per thread per slice
    constexpr int kStageBytes = (BM + BN) * kRowBytes;
    extern __shared__ __attribute__((aligned(16))) char lds[];

    int tile_m, tile_n;
    tile_coords(blockIdx.x, tiles_m, tiles_n, &tile_m, &tile_n);
    const int m0 = tile_m * BM, n0 = tile_n * BN;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave / WGN, wn = wave % WGN;

    // ---- global -> register staging: chunk idx = i*256 + tid, row = idx/8, chunk = idx%8
    const int ld_row = tid >> 3, ld_chunk = tid & 7;
    const char* a_src[LA];
    const char* b_src[LB];
    int a_dst[LA], b_dst[LB];
#pragma unroll
    for (int i = 0; i < LA; ++i) {
        const int row = ld_row + 32 * i;
        int gm = m0 + row;
        if (gm >= M) gm = M - 1;                        // clamped rows are computed but never stored
        a_src[i] = reinterpret_cast<const char*>(A + static_cast<int64_t>(gm) * K) + ld_chunk * 16;
        a_dst[i] = row * kRowBytes + ((ld_chunk ^ (row & 7)) << 4);
    }
#pragma unroll
    for (int i = 0; i < LB; ++i) {
        const int row = ld_row + 32 * i;
        int gn = n0 + row;
        if (gn >= N) gn = N - 1;
        b_src[i] = reinterpret_cast<const char*>(W + static_cast<int64_t>(gn) * K) + ld_chunk * 16;
        b_dst[i] = BM * kRowBytes + row * kRowBytes + ((ld_chunk ^ (row & 7)) << 4);
    }
    u32x4_t sa[LA], sb[LB];
    const int nk = (K + BK - 1) / BK;

    auto fetch = [&](int kt) {
        const int kbyte = kt * kRowBytes;
        const bool in_k = (kt * BK + ld_chunk * 8) < K;    // K % 8 == 0: a chunk is all in or all out
#pragma unroll
        for (int i = 0; i < LA; ++i)
            sa[i] = in_k ? *reinterpret_cast<const u32x4_t*>(a_src[i] + kbyte) : u32x4_t{0, 0, 0, 0};
#pragma unroll
        for (int i = 0; i < LB; ++i)
            sb[i] = in_k ? *reinterpret_cast<const u32x4_t*>(b_src[i] + kbyte) : u32x4_t{0, 0, 0, 0};
    };
    auto stash = [&](int stage) {
        char* base = lds + stage * kStageBytes;
#pragma unroll
        for (int i = 0; i < LA; ++i) *reinterpret_cast<u32x4_t*>(base + a_dst[i]) = sa[i];
#pragma unroll
        for (int i = 0; i < LB; ++i) *reinterpret_cast<u32x4_t*>(base + b_dst[i]) = sb[i];
    };

    // ---- MFMA operand addresses in LDS (row fixed per lane, chunk varies with the k step)
    const int l32 = lane & 31, lhi = lane >> 5;
    int a_row_off[TM], b_row_off[TN];
#pragma unroll
    for (int i = 0; i < TM; ++i) a_row_off[i] = (wm * TM * 32 + i * 32 + l32) * kRowBytes;
#pragma unroll
    for (int j = 0; j < TN; ++j) b_row_off[j] = BM * kRowBytes + (wn * TN * 32 + j * 32 + l32) * kRowBytes;
    const int sw = l32 & 7;                                // (row % 8): tile row offsets are multiples of 32

    f32x16_t acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;

    fetch(0);
    stash(0);
    __syncthreads();
    for (int kt = 0; kt < nk; ++kt) {
        const bool more = kt + 1 < nk;
        if (more) fetch(kt + 1);
        const char* base = lds + (kt & 1) * kStageBytes;
#pragma unroll
        for (int ks = 0; ks < BK / 16; ++ks) {
            const int choff = (((ks << 1) | lhi) ^ sw) << 4;
            bf16x8_t af[TM], bfr[TN];
#pragma unroll
            for (int i = 0; i < TM; ++i)
                af[i] = *reinterpret_cast<const bf16x8_t*>(base + a_row_off[i] + choff);
#pragma unroll
            for (int j = 0; j < TN; ++j)
                bfr[j] = *reinterpret_cast<const bf16x8_t*>(base + b_row_off[j] + choff);
#pragma unroll
            for (int i = 0; i < TM; ++i)
#pragma unroll
                for (int j = 0; j < TN; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[i], bfr[j], acc[i][j], 0, 0, 0);
        }
        if (more) stash((kt + 1) & 1);
        __syncthreads();
    }

    // ---- epilogue.  Accumulator register e of lane l holds
    //      row 8*(e/4) + 4*(l/32) + e%4, column l%32 of its 32x32 tile.
#pragma unroll
    for (int j = 0; j < TN; ++j) {
        const int gn = n0 + wn * TN * 32 + j * 32 + l32;
        if (gn >= N) continue;
        const float bv = bias[gn];
#pragma unroll
        for (int i = 0; i < TM; ++i) {
            const int row_base = m0 + wm * TM * 32 + i * 32 + 4 * lhi;
#pragma unroll
            for (int e = 0; e < 16; ++e) {
                const int gm = row_base + 8 * (e >> 2) + (e & 3);
                if (gm >= M) continue;
                const float v = acc[i][j][e] + bv;
                const int64_t o = static_cast<int64_t>(gm) * N + gn;
                if (EPI == FREE_EPI_BIAS) {
                    out[o] = float_to_bf16(v);
                } else if (EPI == FREE_EPI_BIAS_GELU) {
                    out[o] = float_to_bf16(gelu_fast(v));
                } else {
                    const float g = gate.base[static_cast<int64_t>(gm / gate.rows_per_sample) * gate.stride + gn];
                    resid[o] = fmaf(g, v, resid[o]);
                }
            }
        }
    }
}

template <int BM, int BN, int WGM, int WGN>
int32_t launch_cfg(const bf16_t* A, const bf16_t* W, const float* bias, int32_t M, int32_t N, int32_t K,
                   int32_t epi, bf16_t* out, float* resid, RowVec gate, hipStream_t s) {
    const int tiles_m = (M + BM - 1) / BM, tiles_n = (N + BN - 1) / BN;
    const size_t lds = 2 * static_cast<size_t>(BM + BN) * kRowBytes;
    const dim3 grid(tiles_m * tiles_n), block(kThreads);
#define FREE_GEMM_LAUNCH(E)                                                                                     \
    do {                                                                                                        \
        auto kern = gemm_bf16_kernel<BM, BN, WGM, WGN, E>;                                                      \
        static bool attr_set = false;                                                                           \
        if (!attr_set) {                                                                                        \
            if (!hip_ok(hipFuncSetAttribute(reinterpret_cast<const void*>(kern),                                \
                                            hipFuncAttributeMaxDynamicSharedMemorySize, static_cast<int>(lds)))) \
                return FREE_ERR_HIP;                                                                            \
            attr_set = true;                                                                                    \
        }                                                                                                       \
        hipLaunchKernelGGL(kern, grid, block, lds, s, A, W, bias, M, N, K, tiles_m, tiles_n, out, resid, gate); \
    } while (0)
    switch (epi) {
        case FREE_EPI_BIAS: FREE_GEMM_LAUNCH(FREE_EPI_BIAS); break;
        case FREE_EPI_BIAS_GELU: FREE_GEMM_LAUNCH(FREE_EPI_BIAS_GELU); break;
        case FREE_EPI_GATE_RESID: FREE_GEMM_LAUNCH(FREE_EPI_GATE_RESID); break;
        default: return FREE_ERR_RANGE;
    }
#undef FREE_GEMM_LAUNCH
    return launch_ok() ? FREE_OK : FREE_ERR_HIP;
}

// Fraction of the last wave of workgroups that is busy, times a per-shape efficiency guess.
double cfg_score(int M, int N, int bm, int bn, double shape_eff) {
    const double tiles = static_cast<double>((M + bm - 1) / bm) * ((N + bn - 1) / bn);
    const double waves = std::ceil(tiles / 256.0);
    const double useful = (static_cast<double>(M) * N) / (tiles * bm * bn);
    return tiles / (waves * 256.0) * useful * shape_eff;
}

}  // namespace

bool mfma_linear_supported(int32_t M, int32_t N, int32_t K) {
    return M >= 1 && N >= 1 && K >= 8 && (K % 8) == 0;
}

int32_t launch_linear_mfma(const bf16_t* A, const bf16_t* W, const float* bias, int32_t M, int32_t N, int32_t K,
                           int32_t epi, bf16_t* out, float* resid, RowVec gate, hipStream_t s) {
    if (!mfma_linear_supported(M, N, K)) return FREE_ERR_SHAPE;
    if ((reinterpret_cast<uintptr_t>(A) | reinterpret_cast<uintptr_t>(W)) & 15u) return FREE_ERR_SHAPE;
    const double s256 = cfg_score(M, N, 256, 256, 1.00);
    const double s2x1 = cfg_score(M, N, 256, 128, 0.90);
    const double s128 = cfg_score(M, N, 128, 128, 0.75);
    if (s256 >= s2x1 && s256 >= s128)
        return launch_cfg<256, 256, 2, 2>(A, W, bias, M, N, K, epi, out, resid, gate, s);
    if (s2x1 >= s128) return launch_cfg<256, 128, 2, 2>(A, W, bias, M, N, K, epi, out, resid, gate, s);
    return launch_cfg<128, 128, 2, 2>(A, W, bias, M, N, K, epi, out, resid, gate, s);
}

}  // namespace freemi
