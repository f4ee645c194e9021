// Flash-style softmax attention in full fp32 on the matrix cores, for the FREE_FP32 mode of the
// packed target forward (Alg. 1): per (sample, head), out = softmax(q k^T / sqrt(dh)) v,
// non-causal, fp32 operands, products and online softmax (v_mfma_f32_32x32x2_f32).
//
// Same formulation as the bf16 kernel of attn_mfma.hip: the score tile is computed TRANSPOSED,
// S^T = K Q^T (rows = keys, columns = queries), so that in the accumulator layout a lane owns one
// query column (lane % 32) and half of the key rows: the softmax statistics are lane-local (one
// exchange with lane ^ 32), and the probabilities are already the B operand of the second
// product O^T = V^T P^T - register e of the score tile holds key 8 (e / 4) + 4 (lane / 32) + e % 4,
// and one 32x32x2 product contracts over exactly the two keys that the two half-waves hold in
// register e.  The matching A operand is one float per lane, V[key][d = lane % 32 (+ 32 per row
// tile of O^T)], read from a row-major V tile in LDS (32 consecutive floats per half-wave).
// The contraction over the head dim uses 16-byte fragments like the fp32 GEMM: lane group g reads
// chunk 2 j + g of its K row (and holds the same chunks of its Q row in registers); element e of
// the chunk pair (2 j, 2 j + 1) is one 32x32x2 product.
// One workgroup = 4 wavefronts x 32 queries; key tiles of 32; the K/V tile t+1 is in flight from
// global memory in registers while tile t is multiplied.
#include <cmath>

#include "free_internal.h"

namespace freemi {

namespace {

typedef float f32x4_t __attribute__((ext_vector_type(4)));
typedef float f32x16_t __attribute__((ext_vector_type(16)));

constexpr int kThreads = 256;
constexpr int BKV = 32;                   // keys per tile

template <int DH>
__global__ __launch_bounds__(kThreads) void attn_f32_mfma_kernel(const float* __restrict__ qkv, int32_t N,
                                                                 int32_t heads, float scale_log2,
                                                                 float* __restrict__ out) {
    static_assert(DH % 8 == 0 && DH <= 128, "whole chunk pairs");
    constexpr int NC = DH / 4;            // 16-byte chunks per row
    constexpr int NP = DH / 8;            // chunk pairs: groups of four 32x32x2 products
    constexpr int DT = (DH + 31) / 32;    // 32-row tiles of O^T
    constexpr int KP = DH + 4;            // K row pitch in floats: an odd number of chunks (conflict-free b128 reads)
    constexpr int VP = (DH % 16 == 8) ? DH : DH + 8;   // V row pitch = 8 mod 16: rows 4 apart land on the other 32 banks
    constexpr int NLD = (BKV * NC + kThreads - 1) / kThreads;
    __shared__ __attribute__((aligned(16))) float sK[BKV * KP];
    __shared__ __attribute__((aligned(16))) float sV[BKV * VP + 32 * DT];   // the pad rows of O^T read past a row's end

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int l32 = lane & 31, g = lane >> 5;
    const int nq = (N + 127) / 128;
    const int pair_idx = blockIdx.x / nq, q_tile = blockIdx.x % nq;
    const int h = pair_idx % heads, b = pair_idx / heads;
    const int D = heads * DH;
    const int64_t row0 = static_cast<int64_t>(b) * N;
    const int64_t row_stride = static_cast<int64_t>(3) * D;       // floats
    const int q_base = q_tile * 128 + wave * 32;

    // Q fragments: lane holds query column l32, chunks 2 j + g
    f32x4_t qf[NP];
    {
        int q = q_base + l32;
        if (q >= N) q = N - 1;
        const float* src = qkv + (row0 + q) * row_stride + h * DH;
#pragma unroll
        for (int j = 0; j < NP; ++j) qf[j] = *reinterpret_cast<const f32x4_t*>(src + 4 * (2 * j + g));
    }

    // staging of one K/V tile: chunk idx = tid + 256 i -> key row idx / NC, chunk idx % NC (rows past N are clamped:
    // their scores are masked, and their probabilities are zero)
    f32x4_t kreg[NLD], vreg[NLD];
    auto fetch = [&](int t) {
#pragma unroll
        for (int i = 0; i < NLD; ++i) {
            const int idx = tid + kThreads * i;
            if (idx < BKV * NC) {
                int kv = t * BKV + idx / NC;
                if (kv >= N) kv = N - 1;
                const float* src = qkv + (row0 + kv) * row_stride + h * DH + (idx % NC) * 4;
                kreg[i] = *reinterpret_cast<const f32x4_t*>(src + D);
                vreg[i] = *reinterpret_cast<const f32x4_t*>(src + 2 * D);
            }
        }
    };
    auto stash = [&]() {
#pragma unroll
        for (int i = 0; i < NLD; ++i) {
            const int idx = tid + kThreads * i;
            if (idx < BKV * NC) {
                const int r = idx / NC, c = idx % NC;
                *reinterpret_cast<f32x4_t*>(sK + r * KP + c * 4) = kreg[i];
                *reinterpret_cast<f32x4_t*>(sV + r * VP + c * 4) = vreg[i];
            }
        }
    };

    f32x16_t o[DT];
#pragma unroll
    for (int dt = 0; dt < DT; ++dt)
#pragma unroll
        for (int e = 0; e < 16; ++e) o[dt][e] = 0.f;
    float m_run = -INFINITY, l_run = 0.f;

    const int ntiles = (N + BKV - 1) / BKV;
    fetch(0);
    for (int t = 0; t < ntiles; ++t) {
        __syncthreads();                      // every wavefront is done with the previous tile
        stash();
        __syncthreads();
        if (t + 1 < ntiles) fetch(t + 1);

        // ---- S^T = K Q^T for the 32 keys of the tile
        f32x16_t st;
#pragma unroll
        for (int e = 0; e < 16; ++e) st[e] = 0.f;
#pragma unroll
        for (int j = 0; j < NP; ++j) {
            const f32x4_t kf = *reinterpret_cast<const f32x4_t*>(sK + l32 * KP + 4 * (2 * j + g));
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const float kv = kf[e], qv = qf[j][e];
                st = __builtin_amdgcn_mfma_f32_32x32x2f32(kv, qv, st, 0, 0, 0);
            }
        }
        if ((t + 1) * BKV > N) {              // ragged last tile: keys past N
#pragma unroll
            for (int e = 0; e < 16; ++e)
                if (t * BKV + 8 * (e >> 2) + 4 * g + (e & 3) >= N) st[e] = -INFINITY;
        }

        // ---- online softmax of the query column
        float mx = st[0];
#pragma unroll
        for (int e = 1; e < 16; ++e) mx = fmaxf(mx, st[e]);
        mx = fmaxf(mx, __shfl_xor(mx, 32, 64));
        const float m_new = fmaxf(m_run, mx);           // finite: the first key of every tile exists
        const float alpha = __builtin_amdgcn_exp2f((m_run - m_new) * scale_log2);
        const float mb = m_new * scale_log2;
        float p[16], sum = 0.f;
#pragma unroll
        for (int e = 0; e < 16; ++e) {
            p[e] = __builtin_amdgcn_exp2f(fmaf(st[e], scale_log2, -mb));
            sum += p[e];
        }
        l_run = fmaf(l_run, alpha, sum);
        m_run = m_new;
#pragma unroll
        for (int dt = 0; dt < DT; ++dt)
#pragma unroll
            for (int e = 0; e < 16; ++e) o[dt][e] *= alpha;

        // ---- O^T += V^T P^T: register e pairs the keys 8 (e / 4) + e % 4 (+ 4 for the upper half-wave)
#pragma unroll
        for (int e = 0; e < 16; ++e) {
            const float* vrow = sV + (8 * (e >> 2) + 4 * g + (e & 3)) * VP + l32;
#pragma unroll
            for (int dt = 0; dt < DT; ++dt) {
                const float vv = vrow[32 * dt];
                o[dt] = __builtin_amdgcn_mfma_f32_32x32x2f32(vv, p[e], o[dt], 0, 0, 0);
            }
        }
    }

    // ---- normalise and store: register e of O^T tile dt is row d = 32 dt + 8 (e / 4) + 4 g + e % 4, column l32
    const float l_tot = l_run + __shfl_xor(l_run, 32, 64);
    const int q = q_base + l32;
    if (q >= N) return;
    const float inv = 1.0f / l_tot;
    float* dst = out + (row0 + q) * D + h * DH;
#pragma unroll
    for (int dt = 0; dt < DT; ++dt)
#pragma unroll
        for (int e4 = 0; e4 < 4; ++e4) {
            const int d = 32 * dt + 8 * e4 + 4 * g;
            if (d < DH) {
                const f32x4_t v = {o[dt][4 * e4] * inv, o[dt][4 * e4 + 1] * inv, o[dt][4 * e4 + 2] * inv,
                                   o[dt][4 * e4 + 3] * inv};
                *reinterpret_cast<f32x4_t*>(dst + d) = v;
            }
        }
}

template <int DH>
int32_t launch_dh(const float* qkv, int32_t B, int32_t N, int32_t heads, float* out, hipStream_t s) {
    const float scale_log2 = 1.4426950408889634f / std::sqrt(static_cast<float>(DH));
    const int64_t total = static_cast<int64_t>((N + 127) / 128) * heads * B;
    if (total > 0x7fffffff) return FREE_ERR_SHAPE;
    hipLaunchKernelGGL((attn_f32_mfma_kernel<DH>), dim3(static_cast<unsigned>(total)), dim3(kThreads), 0, s, qkv, N,
                       heads, scale_log2, out);
    return launch_ok() ? FREE_OK : FREE_ERR_HIP;
}

}  // namespace

bool mfma_attention_f32_supported(int32_t N, int32_t dh) {
    return N >= 1 && (dh == 16 || dh == 64 || dh == 72 || dh == 128);
}

int32_t launch_attention_mfma_f32(const float* qkv, int32_t B, int32_t N, int32_t heads, int32_t dh, float* out,
                                  hipStream_t s) {
    if ((reinterpret_cast<uintptr_t>(qkv) | reinterpret_cast<uintptr_t>(out)) & 15u) return FREE_ERR_SHAPE;
    switch (dh) {
        case 16: return launch_dh<16>(qkv, B, N, heads, out, s);
        case 64: return launch_dh<64>(qkv, B, N, heads, out, s);
        case 72: return launch_dh<72>(qkv, B, N, heads, out, s);
        case 128: return launch_dh<128>(qkv, B, N, heads, out, s);
        default: return FREE_ERR_SHAPE;
    }
}

}  // namespace freemi
