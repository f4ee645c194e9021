// Final layer of the DiT (LayerNorm without affine, per-sample modulate, linear D -> p*p*C_out,
// unpatchify to [B, C_out, H, W]) for bf16 weights, on the matrix cores.
//
// One workgroup per 16 token rows, four wavefronts that split the hidden dimension in four
// contiguous quarters: a lane holds its 8-float pieces of the quarter in registers (72 floats at
// D = 1152), so the rows are read from memory exactly once, all workgroups' loads are in flight
// together, and the two-pass statistics (mean, then centred variance) run on registers with one
// small LDS exchange between the wavefronts each.  The normalised, modulated values are split into
// a bf16 high part and a bf16 remainder (two v_mfma_f32_16x16x32_bf16 per k-step), so the fp32
// activations lose nothing that matters against the fp32 accumulation; weight rows are the A
// operand, read from global memory (L2) in operand layout.  The four partial 32 x 16 products are
// added through LDS and scattered to the image layout.
//
// The per-row kernel this replaces re-read the whole weight matrix (74 KB) from cache for every
// token row and reduced each of the 32 outputs across the wavefront separately: 120 us at 12288
// rows against 10 us for reading the rows once.
#include "free_internal.h"

namespace freemi {

namespace {

typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef float f32x4_t __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4_t __attribute__((ext_vector_type(4)));

constexpr int kThreads = 256;
constexpr int kRows = 16;                 // token rows per workgroup (the N dimension of the MFMA)

template <int NS>                         // k-steps of 32 per wavefront: D = 128 NS
__global__ __launch_bounds__(kThreads) void final_layer_mfma_kernel(
    const float* __restrict__ x, RowVec shift, RowVec scale, int32_t M, int32_t gh, int32_t gw, int32_t p,
    int32_t c_out, const bf16_t* __restrict__ w, const float* __restrict__ bias, float* __restrict__ out) {
    constexpr int D = 128 * NS;
    __shared__ float red[2][4][kRows];
    __shared__ __attribute__((aligned(16))) float part[4][2][64][4];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int l16 = lane & 15, lq = lane >> 4;
    const int row0 = blockIdx.x * kRows;
    const int row = row0 + l16 < M ? row0 + l16 : M - 1;          // rows past M repeat the last one, never stored
    const int k0 = wave * NS * 32 + lq * 8;                        // + 32 s: this lane's 8 columns of k-step s
    const float* xr = x + static_cast<int64_t>(row) * D + k0;
    f32x4_t xa[NS][2];
#pragma unroll
    for (int s = 0; s < NS; ++s) {
        xa[s][0] = *reinterpret_cast<const f32x4_t*>(xr + 32 * s);
        xa[s][1] = *reinterpret_cast<const f32x4_t*>(xr + 32 * s + 4);
    }
    // a row lives in the four lanes l16 + 16 lq of each of the four wavefronts
    auto row_total = [&](float v, int slot) {
        v += __shfl_xor(v, 16, 64);
        v += __shfl_xor(v, 32, 64);
        if (lq == 0) red[slot][wave][l16] = v;
        __syncthreads();
        return (red[slot][0][l16] + red[slot][1][l16]) + (red[slot][2][l16] + red[slot][3][l16]);
    };
    float sum = 0.f;
#pragma unroll
    for (int s = 0; s < NS; ++s)
#pragma unroll
        for (int h = 0; h < 2; ++h) sum += (xa[s][h][0] + xa[s][h][1]) + (xa[s][h][2] + xa[s][h][3]);
    const float mean = row_total(sum, 0) / static_cast<float>(D);
    float q = 0.f;
#pragma unroll
    for (int s = 0; s < NS; ++s)
#pragma unroll
        for (int h = 0; h < 2; ++h) {
            const float a = xa[s][h][0] - mean, b = xa[s][h][1] - mean, c = xa[s][h][2] - mean, d = xa[s][h][3] - mean;
            q += (a * a + b * b) + (c * c + d * d);
        }
    const float rstd = rsqrtf(row_total(q, 1) / static_cast<float>(D) + kLnEps);

    const float* shr = shift.base + static_cast<int64_t>(row / shift.rows_per_sample) * shift.stride + k0;
    const float* scr = scale.base + static_cast<int64_t>(row / scale.rows_per_sample) * scale.stride + k0;
    const int P = p * p * c_out;
    f32x4_t acc[2] = {{0.f, 0.f, 0.f, 0.f}, {0.f, 0.f, 0.f, 0.f}};
    // k-steps in groups of kG: the shift, scale and weight pieces of a whole group are requested together and
    // only then used - one memory round trip per group on the critical path of the workgroup instead of two per
    // k-step (left to itself the compiler keeps 72 registers and waits for every piece where it is used)
    // (groups of two: 152 registers at NS = 9, three wavefronts per SIMD - every workgroup of a 12288-row launch
    // resident at once; groups of three need 176 and were slower there)
    constexpr int kG = 2;
#pragma unroll
    for (int g0 = 0; g0 < NS; g0 += kG) {
        f32x4_t shv[kG][2], scv[kG][2];
        u32x4_t wv[kG][2];
#pragma unroll
        for (int u = 0; u < kG; ++u) {
            const int s = g0 + u;
            if (s >= NS) continue;
#pragma unroll
            for (int h = 0; h < 2; ++h) {
                shv[u][h] = *reinterpret_cast<const f32x4_t*>(shr + 32 * s + 4 * h);
                scv[u][h] = *reinterpret_cast<const f32x4_t*>(scr + 32 * s + 4 * h);
            }
#pragma unroll
            for (int t = 0; t < 2; ++t) {
                const int o = 16 * t + l16;
                // (outputs past P re-read row 0 and are multiplied into columns that are never stored)
                wv[u][t] = *reinterpret_cast<const u32x4_t*>(w + static_cast<int64_t>(o < P ? o : 0) * D + k0 + 32 * s);
            }
        }
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int u = 0; u < kG; ++u) {
            const int s = g0 + u;
            if (s >= NS) continue;
            uint32_t hi[4], lo[4];
#pragma unroll
            for (int h = 0; h < 2; ++h) {
                float v[4];
#pragma unroll
                for (int c = 0; c < 4; ++c) v[c] = fmaf((xa[s][h][c] - mean) * rstd, 1.0f + scv[u][h][c], shv[u][h][c]);
#pragma unroll
                for (int c2 = 0; c2 < 2; ++c2) {
                    const uint32_t hp = pack_bf16_pair(v[2 * c2], v[2 * c2 + 1]);
                    hi[2 * h + c2] = hp;
                    lo[2 * h + c2] = pack_bf16_pair(v[2 * c2] - __uint_as_float(hp << 16),
                                                    v[2 * c2 + 1] - __uint_as_float(hp & 0xffff0000u));
                }
            }
            const bf16x8_t bh = __builtin_bit_cast(bf16x8_t, u32x4_t{hi[0], hi[1], hi[2], hi[3]});
            const bf16x8_t bl = __builtin_bit_cast(bf16x8_t, u32x4_t{lo[0], lo[1], lo[2], lo[3]});
#pragma unroll
            for (int t = 0; t < 2; ++t) {
                const int o = 16 * t + l16;
                const bf16x8_t a = __builtin_bit_cast(bf16x8_t, o < P ? wv[u][t] : u32x4_t{0, 0, 0, 0});
                acc[t] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, bh, acc[t], 0, 0, 0);
                acc[t] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, bl, acc[t], 0, 0, 0);
            }
        }
    }
    // accumulator register i of lane l: output 16 t + 4 (l / 16) + i, token row l % 16
#pragma unroll
    for (int t = 0; t < 2; ++t) *reinterpret_cast<f32x4_t*>(part[wave][t][lane]) = acc[t];
    __syncthreads();
    if (tid < 128) {
        const int t = tid >> 6, ln = tid & 63;
        f32x4_t v = *reinterpret_cast<const f32x4_t*>(part[0][t][ln]);
#pragma unroll
        for (int wv = 1; wv < 4; ++wv) {
            const f32x4_t u = *reinterpret_cast<const f32x4_t*>(part[wv][t][ln]);
#pragma unroll
            for (int i = 0; i < 4; ++i) v[i] += u[i];
        }
        const int r = row0 + (ln & 15);
        if (r < M) {
            const int ntok = gh * gw;
            const int b = r / ntok, n = r % ntok;
            const int gi = n / gw, gj = n % gw;
            const int H = gh * p, Wd = gw * p;
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const int o = 16 * t + 4 * (ln >> 4) + i;
                if (o < P) {
                    const int c = o % c_out, pq = (o / c_out) % p, ph = o / (c_out * p);
                    out[((static_cast<int64_t>(b) * c_out + c) * H + gi * p + ph) * Wd + gj * p + pq] = v[i] + bias[o];
                }
            }
        }
    }
}

}  // namespace

// bf16 weights, D one of 384 / 768 / 1024 / 1152 (the DiT-S/B/L/XL widths), at most 32 outputs per
// token, 16-byte aligned rows of x, the weights and the modulation vectors.
bool final_mfma_supported(int32_t D, int32_t P) {
    return (D == 384 || D == 768 || D == 1024 || D == 1152) && P >= 1 && P <= 32;
}

int32_t launch_final_layer_mfma(const float* x, RowVec shift, RowVec scale, int32_t M, int32_t gh, int32_t gw,
                                int32_t p, int32_t c_out, int32_t D, const bf16_t* w, const float* bias, float* out,
                                hipStream_t s) {
    const dim3 grid((M + kRows - 1) / kRows), block(kThreads);
#define FREE_FIN_MFMA(NS)                                                                                        \
    hipLaunchKernelGGL(final_layer_mfma_kernel<NS>, grid, block, 0, s, x, shift, scale, M, gh, gw, p, c_out, w, bias, out)
    switch (D) {
        case 384: FREE_FIN_MFMA(3); break;
        case 768: FREE_FIN_MFMA(6); break;
        case 1024: FREE_FIN_MFMA(8); break;
        case 1152: FREE_FIN_MFMA(9); break;
        default: return FREE_ERR_SHAPE;
    }
#undef FREE_FIN_MFMA
    return launch_ok() ? FREE_OK : FREE_ERR_HIP;
}

}  // namespace freemi
