// Flash-style softmax attention on bf16 MFMA for the DiT blocks of the packed
// target forward (Alg. 1): per (sample, head), out = softmax(q k^T / sqrt(dh)) v,
// non-causal, fp32 online softmax, Q/K/V tiles staged in LDS.
//
// Formulation chosen for the CDNA accumulator layout: the score tile is computed
// TRANSPOSED, S^T = K Q^T (rows = keys, columns = queries), with
// v_mfma_f32_32x32x16_bf16.  In the accumulator layout a lane then owns one query
// column (lane % 32) and half of the key rows, so
//   * the softmax statistics of a query are lane-local (one exchange with lane^32),
//   * the probabilities are already in the B-operand layout of the second product
//     O^T = V^T P^T (rows = head dim, columns = queries): no shuffle, no LDS trip,
//   * rescaling O^T by the per-query factor is a per-lane scalar multiply.
// The key order inside each 32-key block is permuted when K is written to LDS
// (bits 2 and 3 of the row index swapped) so that the 8 probabilities a lane feeds
// to one MFMA belong to 8 CONSECUTIVE keys: the matching V^T operand is then a
// pair of transposing LDS reads (ds_read_b64_tr_b16) of the row-major V tile.
// Head dim 72 (DiT-XL): the contraction over d is padded 72 -> 80 with zero chunks
// in LDS; the O^T rows are padded 72 -> 96 and the pad rows are never stored (row 72 carries the
// softmax denominator: column 72 of the V tile is set to one).
#include <cmath>
#include <type_traits>

#include "free_internal.h"

namespace freemi {

namespace {

typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef float f32x16_t __attribute__((ext_vector_type(16)));
typedef uint32_t u32x4_t __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2_t __attribute__((ext_vector_type(2)));
typedef short v4s_t __attribute__((ext_vector_type(4)));
typedef short v8s_t __attribute__((ext_vector_type(8)));

constexpr int kThreads = 256;
constexpr int BKV = 64;                   // keys per LDS tile

__device__ inline int swap_bits_2_3(int r) { return (r & ~12) | ((r & 4) << 1) | ((r & 8) >> 1); }

__device__ inline uint32_t pack_bf16x2(float lo, float hi) { return pack_bf16_pair(lo, hi); }   // v_cvt_pk_bf16_f32

// amdgpu_waves_per_eu: with at most 256 registers per lane the compiler uses the VGPR form of the MFMAs -
// with the default budget of 512 it parks accumulators in AGPRs and moves them back and forth for the
// softmax (several hundred v_accvgpr moves per key tile).  Head dims up to 72 run three workgroups per CU
// (168 registers, 47 KB of LDS each): the phases of a tile - S^T on the matrix pipe, softmax on the VALU,
// O^T on the matrix pipe - are serial inside a wavefront, so what overlaps them is the number of
// wavefronts per SIMD; the third one is worth more (measured 4.5 %) than the second set of K/V staging
// registers it costs.
template <int DH, int QT>
__global__ __launch_bounds__(kThreads) __attribute__((amdgpu_waves_per_eu(DH <= 72 ? 3 : 2, DH <= 72 ? 3 : 2))) void attn_mfma_kernel(const bf16_t* __restrict__ qkv, int32_t N,
                                                             int32_t heads, float scale_log2,
                                                             bf16_t* __restrict__ out) {
    constexpr int KSTEPS = (DH + 15) / 16;            // MFMA k-steps over the head dim (S^T)
    constexpr int DCH = DH / 8;                       // 16-byte chunks per Q/K/V row
    constexpr int DT = (DH + 31) / 32;                // 32-row tiles of O^T
    constexpr int kSets = DH <= 72 ? 1 : 2;           // K/V register sets: tiles in flight from global memory
    constexpr bool kSumByMfma = (DH % 32) != 0;       // a spare row of O^T can carry the softmax denominator
    constexpr int KROW = ((2 * KSTEPS) | 1) * 16;     // bytes per K row in LDS (odd # of chunks)
    constexpr int BQ = 4 * 32 * QT;                   // queries per workgroup
    constexpr int NLD = (BKV * DCH + kThreads - 1) / kThreads;   // 16-byte loads per thread per tile
    // V stays row-major in LDS ([key][d]) and is read with the transposing LDS load; a row stride of
    // 64 or 192 (mod 256) bytes puts the 4 keys x 64 bytes that 32 lanes of such a load touch on
    // disjoint banks
    constexpr int VROW = DT == 1 ? 64 : (DT <= 3 ? 192 : 320);
    constexpr int kKBytes = BKV * KROW, kVBytes = BKV * VROW;
    __shared__ __attribute__((aligned(16))) char sKbuf[2 * kKBytes];      // two stages: tile t is multiplied
    __shared__ __attribute__((aligned(16))) char sVbuf[2 * kVBytes];      // while tile t+1 is written

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int l32 = lane & 31, g = lane >> 5;
    // Workgroup ids are dealt round-robin to the 8 XCDs (each with its own L2).  All query
    // tiles of one (sample, head) re-read the same K and V, so they are placed on ONE XCD,
    // back to back: id L -> XCD L % 8; pair index = L % 8 + 8 * (L / (8 nq)), tile = (L / 8) % nq.
    const int nq = (N + BQ - 1) / BQ;
    const int n_pairs = static_cast<int>(gridDim.x) / nq;       // (sample, head) pairs
    int pair_idx, q_tile;
    if (n_pairs % 8 == 0) {
        const int L = blockIdx.x;
        pair_idx = (L & 7) + 8 * (L / (8 * nq));
        q_tile = (L >> 3) % nq;
    } else {
        pair_idx = blockIdx.x / nq;
        q_tile = blockIdx.x % nq;
    }
    const int h = pair_idx % heads, b = pair_idx / heads;
    const int D = heads * DH;
    const int64_t row0 = static_cast<int64_t>(b) * N;
    const int q_base = q_tile * BQ + wave * 32 * QT;
    const size_t row_bytes = static_cast<size_t>(3) * D * 2;
    const char* qkv_b = reinterpret_cast<const char*>(qkv);

    // zero the pad chunks of K (d in [DH, 16*KSTEPS)) and the pad rows of V^T once
    for (int i = tid; i < 2 * BKV * (KROW / 16); i += kThreads) {
        const int c = i % (KROW / 16);
        if (c >= DCH) *reinterpret_cast<u32x4_t*>(sKbuf + (i / (KROW / 16)) * KROW + c * 16) = u32x4_t{0, 0, 0, 0};
    }
    // ... except, when the head dimension leaves pad columns (kSumByMfma), column DH of V, which is one
    // (bf16 0x3F80) for every key: row DH of O^T then accumulates the sum of the probabilities in the matrix
    // pipe, rescaled together with O^T, instead of one VALU addition per score
    for (int i = tid; i < 2 * BKV * (VROW / 16); i += kThreads) {
        const int c = i % (VROW / 16);
        if (c >= DCH)
            *reinterpret_cast<u32x4_t*>(sVbuf + (i / (VROW / 16)) * VROW + c * 16) =
                u32x4_t{(kSumByMfma && c == DCH) ? 0x3F80u : 0u, 0, 0, 0};
    }

    // Q^T fragments (B operand of S^T): lane holds query column l32, k-slots d = 16 ks + 8 g + j
    bf16x8_t qf[QT][KSTEPS];
#pragma unroll
    for (int qt = 0; qt < QT; ++qt) {
        int q = q_base + qt * 32 + l32;
        if (q >= N) q = N - 1;
        const char* src = qkv_b + (row0 + q) * row_bytes + static_cast<size_t>(h) * DH * 2;
#pragma unroll
        for (int ks = 0; ks < KSTEPS; ++ks) {
            const int c = 2 * ks + g;
            u32x4_t v = {0, 0, 0, 0};
            if (c < DCH) v = *reinterpret_cast<const u32x4_t*>(src + c * 16);
            qf[qt][ks] = __builtin_bit_cast(bf16x8_t, v);
        }
    }

    // global -> register staging of one K/V tile: thread chunk idx = tid + 256 i -> key row idx / DCH,
    // 16-byte chunk idx % DCH of that row, for K and for V alike (lanes walk the chunks of a row).
    // Buffer loads over the rows of this sample: keys past N read as zero (on gfx950 the scalar offset
    // takes part in the range check, measured), the tile and the K / V column offsets are wave-uniform
    // scalar offsets, one per-lane byte offset per load.
    const __amdgpu_buffer_rsrc_t srd = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<char*>(qkv_b) + row0 * row_bytes, 0, static_cast<int>(N * row_bytes), 0x00020000);
    const int k_col = (D + h * DH) * 2, v_col = (2 * D + h * DH) * 2;
    int ld_off[NLD];
#pragma unroll
    for (int i = 0; i < NLD; ++i) {
        const int idx = tid + kThreads * i;
        ld_off[i] = (idx / DCH) * static_cast<int>(row_bytes) + (idx % DCH) * 16;
    }
    // kSets register sets: the loads of tiles t+2 .. t+1+kSets are in flight while tile t is processed
    u32x4_t kreg[kSets][NLD], vreg[kSets][NLD];
    auto fetch = [&](int t, auto set) {
        constexpr int S = decltype(set)::value;
        const int tile_off = t * BKV * static_cast<int>(row_bytes);
#pragma unroll
        for (int i = 0; i < NLD; ++i) {
            if (tid + kThreads * i < BKV * DCH) {
                kreg[S][i] = __builtin_amdgcn_raw_buffer_load_b128(srd, ld_off[i], tile_off + k_col, 0);
                vreg[S][i] = __builtin_amdgcn_raw_buffer_load_b128(srd, ld_off[i], tile_off + v_col, 0);
            }
        }
    };
    auto stash = [&](int stage, auto set) {
        constexpr int S = decltype(set)::value;
        char* sK = sKbuf + stage * kKBytes;
        char* sV = sVbuf + stage * kVBytes;
#pragma unroll
        for (int i = 0; i < NLD; ++i) {
            const int idx = tid + kThreads * i;
            if (idx < BKV * DCH) {
                const int r = idx / DCH;
                const int lr = (r & ~31) | swap_bits_2_3(r & 31);
                *reinterpret_cast<u32x4_t*>(sK + lr * KROW + (idx % DCH) * 16) = kreg[S][i];
                *reinterpret_cast<u32x4_t*>(sV + r * VROW + (idx % DCH) * 16) = vreg[S][i];
            }
        }
    };
    // Transposing read of V (ds_read_b64_tr_b16).  Within 16 lanes, lane i receives element i % 4 of
    // the 8 bytes addressed by lanes i/4, i/4 + 4, i/4 + 8, i/4 + 12.  With source lane r of 16-lane
    // group G pointing at V[8 (G/2) + r/4][16 (G%2) + 4 (r%4) ..+3], lane l gets 4 consecutive keys
    // 8 (l/32) + 0..3 of head-dim column l % 32: half of the A operand of O^T += V^T P^T; the same
    // read 4 rows further down gives the other half.
    const int vtr_off = (8 * (lane >> 5) + ((lane & 15) >> 2)) * VROW + (16 * ((lane >> 4) & 1) + 4 * (lane & 3)) * 2;

    f32x16_t o[DT][QT];
#pragma unroll
    for (int dt = 0; dt < DT; ++dt)
#pragma unroll
        for (int qt = 0; qt < QT; ++qt)
#pragma unroll
            for (int e = 0; e < 16; ++e) o[dt][qt][e] = 0.f;
    // m_ref: the reference maximum the exponentials of a query column are taken against.
    // It follows the running maximum lazily: O^T and the running sum are rescaled only when the
    // maximum has grown by more than kLazy (in log2 units) since the last rescale, so that
    // probabilities stay below 2^kLazy (harmless in bf16/fp32) and the 3 x 16 accumulator
    // registers are rarely touched by the VALU.
    constexpr float kLazy = 8.0f;
    constexpr int kPrioMfma = 2;       // wave priority while issuing the MFMA blocks (0 in the softmax): measured 2.5 %
    float m_ref[QT], l_run[QT];
#pragma unroll
    for (int qt = 0; qt < QT; ++qt) { m_ref[qt] = -INFINITY; l_run[qt] = 0.f; }

    const int ntiles = (N + BKV - 1) / BKV;
    const std::integral_constant<int, 0> set0{};
    const std::integral_constant<int, kSets - 1> set1{};
    fetch(0, set0);
    stash(0, set0);
    if (ntiles > 1) fetch(1, set1);
    if (kSets == 2 && ntiles > 2) fetch(2, set0);
    __syncthreads();
    // tile t: its K/V are in LDS stage t % 2; tile t+1 sits in register set (t+1) % 2
    auto tile = [&](int t, auto ragged, auto next_set) {
        constexpr bool kRagged = decltype(ragged)::value;
        const int kv0 = t * BKV;
        const char* sK = sKbuf + (t & 1) * kKBytes;
        const char* sV = sVbuf + (t & 1) * kVBytes;

        // ---- S^T = K Q^T for the two 32-key blocks of the tile
        __builtin_amdgcn_s_setprio(kPrioMfma);
        f32x16_t st[2][QT];
#pragma unroll
        for (int kb = 0; kb < 2; ++kb)
#pragma unroll
            for (int qt = 0; qt < QT; ++qt)
#pragma unroll
                for (int e = 0; e < 16; ++e) st[kb][qt][e] = 0.f;
#pragma unroll
        for (int ks = 0; ks < KSTEPS; ++ks) {
            bf16x8_t kf[2];
#pragma unroll
            for (int kb = 0; kb < 2; ++kb)
                kf[kb] = *reinterpret_cast<const bf16x8_t*>(sK + (kb * 32 + l32) * KROW + (2 * ks + g) * 16);
#pragma unroll
            for (int kb = 0; kb < 2; ++kb)
#pragma unroll
                for (int qt = 0; qt < QT; ++qt)
                    st[kb][qt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[kb], qf[qt][ks], st[kb][qt], 0, 0, 0);
        }
        __builtin_amdgcn_s_setprio(0);
        // the next tile moves from registers to the other LDS stage while this one is processed;
        // the tile after it is requested from global memory
        if (t + 1 < ntiles) stash((t + 1) & 1, next_set);
        if (t + 1 + kSets < ntiles) fetch(t + 1 + kSets, next_set);

        // keys past N (last tile only): accumulator register e of block kb holds the key
        // kv0 + 32 kb + 16 (e/8) + 8 g + 4 ((e/4)%2) + e%4   (LDS rows were permuted on the way in)
        if (kRagged) {
#pragma unroll
            for (int kb = 0; kb < 2; ++kb)
#pragma unroll
                for (int e = 0; e < 16; ++e) {
                    const int kv = kv0 + 32 * kb + 16 * (e >> 3) + 8 * g + 4 * ((e >> 2) & 1) + (e & 3);
                    if (kv >= N) {
#pragma unroll
                        for (int qt = 0; qt < QT; ++qt) st[kb][qt][e] = -INFINITY;
                    }
                }
        }

        // ---- online softmax per query column, probabilities packed straight into MFMA operands
        bf16x8_t pf[QT][2][2];
#pragma unroll
        for (int qt = 0; qt < QT; ++qt) {
            float mx = st[0][qt][0];
#pragma unroll
            for (int kb = 0; kb < 2; ++kb)
#pragma unroll
                for (int e = 0; e < 16; ++e) mx = fmaxf(mx, st[kb][qt][e]);
            {   // both half-waves of a column agree: v_permlane32_swap leaves {own, partner} in the two
                // results (in either order), without the LDS round trip of a bpermute
                const uint32_t mb32 = __builtin_bit_cast(uint32_t, mx);
                const u32x2_t sw = __builtin_amdgcn_permlane32_swap(mb32, mb32, false, false);
                const uint32_t s0 = sw[0], s1 = sw[1];
                mx = fmaxf(__builtin_bit_cast(float, s0), __builtin_bit_cast(float, s1));
            }
            if (__builtin_expect(__any((mx - m_ref[qt]) * scale_log2 > kLazy), 0)) {     // also true for the first tile (m_ref = -inf)
                const float m_new = fmaxf(m_ref[qt], mx);
                const float alpha = __builtin_amdgcn_exp2f((m_ref[qt] - m_new) * scale_log2);
                if constexpr (!kSumByMfma) l_run[qt] *= alpha;
#pragma unroll
                for (int dt = 0; dt < DT; ++dt)
#pragma unroll
                    for (int e = 0; e < 16; ++e) o[dt][qt][e] *= alpha;
                m_ref[qt] = m_new;
            }
            const float mb = m_ref[qt] * scale_log2;
            [[maybe_unused]] float sum = 0.f;
#pragma unroll
            for (int kb = 0; kb < 2; ++kb)
#pragma unroll
                for (int hh = 0; hh < 2; ++hh) {
                    float p[8];
#pragma unroll
                    for (int j = 0; j < 8; ++j) {
                        p[j] = __builtin_amdgcn_exp2f(fmaf(st[kb][qt][8 * hh + j], scale_log2, -mb));
                        if constexpr (!kSumByMfma) sum += p[j];
                    }
                    u32x4_t pk = {pack_bf16x2(p[0], p[1]), pack_bf16x2(p[2], p[3]), pack_bf16x2(p[4], p[5]),
                                  pack_bf16x2(p[6], p[7])};
                    pf[qt][kb][hh] = __builtin_bit_cast(bf16x8_t, pk);
                }
            if constexpr (!kSumByMfma) l_run[qt] += sum;
        }

        // ---- O^T += V^T P^T
        __builtin_amdgcn_s_setprio(kPrioMfma);
#pragma unroll
        for (int kb = 0; kb < 2; ++kb)
#pragma unroll
            for (int hh = 0; hh < 2; ++hh) {
#pragma unroll
                for (int dt = 0; dt < DT; ++dt) {
                    using lds_v4 = __attribute__((address_space(3))) v4s_t*;
                    const char* vp = sV + (kb * 32 + hh * 16) * VROW + dt * 64 + vtr_off;
                    const v4s_t vlo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_v4)(vp));
                    const v4s_t vhi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_v4)(vp + 4 * VROW));
                    const v8s_t v8 = __builtin_shufflevector(vlo, vhi, 0, 1, 2, 3, 4, 5, 6, 7);
                    const bf16x8_t vf = __builtin_bit_cast(bf16x8_t, v8);
#pragma unroll
                    for (int qt = 0; qt < QT; ++qt)
                        o[dt][qt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf, pf[qt][kb][hh], o[dt][qt], 0, 0, 0);
                }
            }
        __builtin_amdgcn_s_setprio(0);
        __syncthreads();          // stage (t+1)&1 is complete; stage t&1 may be overwritten next iteration
    };
    // full tiles need no key masking; only a ragged last tile does
    const int nfull = N / BKV;
    int t = 0;
    for (; t + 1 < nfull; t += 2) {
        tile(t, std::false_type{}, set1);
        tile(t + 1, std::false_type{}, set0);
    }
    if (t < nfull) {
        tile(t, std::false_type{}, set1);
        ++t;
    }
    if (t < ntiles) {
        if (t & 1) tile(t, std::true_type{}, set0);
        else tile(t, std::true_type{}, set1);
    }

    // ---- normalise and store: register e of O^T tile dt is row d = 32 dt + 8 (e/4) + 4 g + e%4, column l32
#pragma unroll
    for (int qt = 0; qt < QT; ++qt) {
        const int q = q_base + qt * 32 + l32;
        float l_tot;
        if constexpr (kSumByMfma) {
            // row DH of O^T: tile DH / 32, register 4 (r / 8) + r % 4 of the half-wave (r % 8) / 4, r = DH % 32
            constexpr int r = DH % 32;
            const float mine = o[DH / 32][qt][4 * (r / 8) + r % 4];
            const float other = __shfl_xor(mine, 32, 64);
            l_tot = (g == (r % 8) / 4) ? mine : other;
        } else {
            l_tot = l_run[qt] + __shfl_xor(l_run[qt], 32, 64);
        }
        if (q >= N) continue;
        const float inv = 1.0f / l_tot;
        char* dst = reinterpret_cast<char*>(out) + ((row0 + q) * D + static_cast<size_t>(h) * DH) * 2;
#pragma unroll
        for (int dt = 0; dt < DT; ++dt)
#pragma unroll
            for (int e4 = 0; e4 < 4; ++e4) {
                const int d = 32 * dt + 8 * e4 + 4 * g;
                if (d < DH) {
                    u32x2_t v = {pack_bf16x2(o[dt][qt][4 * e4] * inv, o[dt][qt][4 * e4 + 1] * inv),
                                 pack_bf16x2(o[dt][qt][4 * e4 + 2] * inv, o[dt][qt][4 * e4 + 3] * inv)};
                    *reinterpret_cast<u32x2_t*>(dst + d * 2) = v;
                }
            }
    }
}

template <int DH>
int32_t launch_dh(const bf16_t* qkv, int32_t B, int32_t N, int32_t heads, bf16_t* out, hipStream_t s) {
    const float scale_log2 = 1.4426950408889634f / std::sqrt(static_cast<float>(DH));
    // one 32-query tile per wavefront: 128 queries per workgroup, two or three workgroups per CU
    // (measured faster than two query tiles per wavefront at one workgroup per CU)
    const int64_t total = static_cast<int64_t>((N + 127) / 128) * heads * B;
    if (total > 0x7fffffff) return FREE_ERR_SHAPE;
    dim3 grid(static_cast<unsigned>(total));
    hipLaunchKernelGGL((attn_mfma_kernel<DH, 1>), grid, dim3(kThreads), 0, s, qkv, N, heads, scale_log2, out);
    return launch_ok() ? FREE_OK : FREE_ERR_HIP;
}

}  // namespace

bool mfma_attention_supported(int32_t N, int32_t dh) {
    return N >= 1 && (dh == 16 || dh == 64 || dh == 72 || dh == 128);
}

int32_t launch_attention_mfma(const bf16_t* qkv, int32_t B, int32_t N, int32_t heads, int32_t dh, bf16_t* out,
                              hipStream_t s) {
    if (reinterpret_cast<uintptr_t>(qkv) & 15u) return FREE_ERR_SHAPE;
    if (B > 65535 || heads > 65535) return FREE_ERR_SHAPE;
    // one sample's rows are addressed through a buffer descriptor with 32-bit byte offsets
    if (static_cast<int64_t>(N) * 3 * heads * dh * 2 >= (1ll << 31)) return FREE_ERR_SHAPE;
    switch (dh) {
        case 16: return launch_dh<16>(qkv, B, N, heads, out, s);
        case 64: return launch_dh<64>(qkv, B, N, heads, out, s);
        case 72: return launch_dh<72>(qkv, B, N, heads, out, s);
        case 128: return launch_dh<128>(qkv, B, N, heads, out, s);
        default: return FREE_ERR_SHAPE;
    }
}

}  // namespace freemi
