// Straightforward kernels of the class-conditional DiT forward (the network the
// packed target pass of Alg. 1 evaluates; the paper cites DiT and fixes none of
// its internals).  Everything that is not a large dense contraction lives here:
// conditioning MLP, adaLN modulation GEMV, patch embedding, LayerNorm+modulate,
// final layer + unpatchify, guidance + eps->mean (Eq. ddpm_update).  It also
// holds the plain (non-MFMA) linear and attention kernels used by the fp32 mode
// and as the shape fallback of the bf16 mode.
#include "free_internal.h"

namespace freemi {

namespace {

constexpr int kThreads = 256;
constexpr int kWaves = kThreads / 64;
constexpr int kMaxFinalLds = 160 * 1024;          // LDS of one CU: the final projection matrix must fit

__device__ inline float wave_sum_f(float v) {
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off, 64);
    return v;
}

// ---------------------------------------------------------------------------
// Conditioning: c = W2 silu(W1 temb(t) + b1) + b2 + table[y];  sc = silu(c)
// ---------------------------------------------------------------------------
// temb[b, :] = [cos(t w_j) | sin(t w_j)], w_j = 10000^(-j/half).  The angle is
// formed in fp64 (t up to 999 times w_0 = 1 would lose 4 digits in fp32).
__global__ void timestep_embed_kernel(const int32_t* __restrict__ t, int32_t B, int32_t tfreq,
                                      float* __restrict__ temb) {
    const int half = tfreq / 2;
    const int idx = blockIdx.x * blockDim.x + threadIdx.x;
    if (idx >= B * half) return;
    const int b = idx / half, j = idx % half;
    const double w = exp(-9.210340371976184 * static_cast<double>(j) / static_cast<double>(half));
    const double ang = static_cast<double>(t[b]) * w;
    temb[b * tfreq + j] = static_cast<float>(cos(ang));
    temb[b * tfreq + half + j] = static_cast<float>(sin(ang));
}

// out[b, j] = act(sum_i in[b, i] W[j, i] + bias[j] + table[row[b], j]); one wavefront per (b, j).
template <bool SILU>
__global__ __launch_bounds__(kThreads) void small_linear_kernel(
    const float* __restrict__ in, int32_t B, int32_t K, int32_t N, const float* __restrict__ W,
    const float* __restrict__ bias, const float* __restrict__ table, const int32_t* __restrict__ row,
    float* __restrict__ out) {
    const int j = blockIdx.x * kWaves + (threadIdx.x >> 6);
    const int b = blockIdx.y;
    const int lane = threadIdx.x & 63;
    if (j >= N) return;
    const float* x = in + static_cast<int64_t>(b) * K;
    const float* w = W + static_cast<int64_t>(j) * K;
    float acc = 0.f;
    for (int i = lane; i < K; i += 64) acc = fmaf(x[i], w[i], acc);
    acc = wave_sum_f(acc);
    if (lane == 0) {
        float v = acc + bias[j];
        if (table) v += table[static_cast<int64_t>(row[b]) * N + j];
        out[static_cast<int64_t>(b) * N + j] = SILU ? silu_f(v) : v;
    }
}

// The same with one wavefront per output column j for ALL samples: the weight row is read once per eight samples
// instead of once per sample, in 16-byte pieces, and a launch has N / 4 workgroups instead of B N / 4
// (K % 4 == 0, 16-byte aligned rows).  Sample b0 + q is reduced in lane order and written by lane q.
template <bool SILU>
__global__ __launch_bounds__(kThreads) void small_linear_rows_kernel(
    const float* __restrict__ in, int32_t B, int32_t K, int32_t N, const float* __restrict__ W,
    const float* __restrict__ bias, const float* __restrict__ table, const int32_t* __restrict__ row,
    float* __restrict__ out) {
    constexpr int kSamples = 8;
    const int j = blockIdx.x * kWaves + __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int lane = threadIdx.x & 63;
    if (j >= N) return;
    const float4* w4 = reinterpret_cast<const float4*>(W + static_cast<int64_t>(j) * K);
    const int k4 = K / 4;
    for (int b0 = 0; b0 < B; b0 += kSamples) {
        float acc[kSamples];
#pragma unroll
        for (int q = 0; q < kSamples; ++q) acc[q] = 0.f;
#pragma unroll 2
        for (int i = lane; i < k4; i += 64) {
            const float4 wv = w4[i];
#pragma unroll
            for (int q = 0; q < kSamples; ++q) {
                const int b = b0 + q < B ? b0 + q : B - 1;         // past the end: the last sample again, not stored
                const float4 xv = reinterpret_cast<const float4*>(in + static_cast<int64_t>(b) * K)[i];
                acc[q] = fmaf(xv.w, wv.w, fmaf(xv.z, wv.z, fmaf(xv.y, wv.y, fmaf(xv.x, wv.x, acc[q]))));
            }
        }
        float mine = 0.f;
#pragma unroll
        for (int q = 0; q < kSamples; ++q) {
            const float t = wave_sum_f(acc[q]);
            if (lane == q) mine = t;
        }
        const int b = b0 + lane;
        if (lane < kSamples && b < B) {
            float v = mine + bias[j];
            if (table) v += table[static_cast<int64_t>(row[b]) * N + j];
            out[static_cast<int64_t>(b) * N + j] = SILU ? silu_f(v) : v;
        }
    }
}

// ---------------------------------------------------------------------------
// adaLN modulation for all blocks and the final layer in one launch:
//   mod[b, r] = sum_i sc[b, i] W_r[i] + bias_r
// Rows come from n_mats matrices (device pointer table); HBM-bound on the
// weights (a third of all DiT parameters), every weight byte is read once.
// ---------------------------------------------------------------------------
constexpr int kAdaBatch = 16;   // batch rows kept in LDS / accumulators per pass

template <typename WT>
struct WVec;
template <>
struct WVec<float> {
    static constexpr int N = 4;
    typedef float4 raw;
    __device__ static void unpack(const raw& r, float* f) { f[0] = r.x; f[1] = r.y; f[2] = r.z; f[3] = r.w; }
};
template <>
struct WVec<bf16_t> {
    static constexpr int N = 8;
    typedef uint4 raw;
    __device__ static void unpack(const raw& r, float* f) {
        const uint32_t w[4] = {r.x, r.y, r.z, r.w};
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            f[2 * i] = __uint_as_float(w[i] << 16);
            f[2 * i + 1] = __uint_as_float(w[i] & 0xffff0000u);
        }
    }
};

template <typename WT>
__global__ __launch_bounds__(kThreads) void adaln_kernel(
    const float* __restrict__ sc, int32_t B, int32_t D, const void* const* __restrict__ w_tab,
    const float* const* __restrict__ b_tab, const int32_t* __restrict__ row_start, int32_t n_mats,
    int32_t total_rows, int32_t rows_per_wave, float* __restrict__ mod) {
    extern __shared__ float sh_sc[];                 // [min(B, kAdaBatch), D]
    constexpr int V = WVec<WT>::N;
    const int lane = threadIdx.x & 63;
    const int wave_global = blockIdx.x * kWaves + (threadIdx.x >> 6);
    const int r_lo = wave_global * rows_per_wave;
    const int nvec = D / V;

    for (int b0 = 0; b0 < B; b0 += kAdaBatch) {
        const int nb = (B - b0 < kAdaBatch) ? B - b0 : kAdaBatch;
        __syncthreads();
        for (int i = threadIdx.x; i < nb * D; i += kThreads) sh_sc[i] = sc[static_cast<int64_t>(b0) * D + i];
        __syncthreads();
        int mat = 0;
        for (int rr = 0; rr < rows_per_wave; ++rr) {
            const int r = r_lo + rr;
            if (r >= total_rows) break;
            while (mat + 1 < n_mats && r >= row_start[mat + 1]) ++mat;
            const int lr = r - row_start[mat];
            const WT* w = static_cast<const WT*>(w_tab[mat]) + static_cast<int64_t>(lr) * D;
            float acc[kAdaBatch];
#pragma unroll
            for (int b = 0; b < kAdaBatch; ++b) acc[b] = 0.f;
            for (int c = lane; c < nvec; c += 64) {
                const typename WVec<WT>::raw raw = reinterpret_cast<const typename WVec<WT>::raw*>(w)[c];
                float wf[V];
                WVec<WT>::unpack(raw, wf);
#pragma unroll
                for (int b = 0; b < kAdaBatch; ++b) {
                    if (b < nb) {
                        const float* s = sh_sc + b * D + c * V;
#pragma unroll
                        for (int v = 0; v < V; ++v) acc[b] = fmaf(wf[v], s[v], acc[b]);
                    }
                }
            }
            const float bias = b_tab[mat][lr];
#pragma unroll
            for (int b = 0; b < kAdaBatch; ++b) {
                if (b < nb) {
                    const float v = wave_sum_f(acc[b]);
                    if (lane == 0) mod[static_cast<int64_t>(b0 + b) * total_rows + r] = v + bias;
                }
            }
        }
    }
}

// ---------------------------------------------------------------------------
// Patch embedding: token (gi, gj) of sample b = W_p . flatten_{c,ph,pw}(patch) + b_p + pos
// x_mod: sample b reads latent b % x_mod (guidance duplicates the K states).
// ---------------------------------------------------------------------------
__global__ __launch_bounds__(kThreads) void patch_embed_kernel(
    const float* __restrict__ x, int32_t x_mod, int32_t C, int32_t H, int32_t W, int32_t p, int32_t D,
    const float* __restrict__ pw, const float* __restrict__ pb, const float* __restrict__ pos,
    float* __restrict__ out) {
    extern __shared__ float patch[];                 // [C p p]
    const int gw = W / p;
    const int n = blockIdx.x, b = blockIdx.y;
    const int gi = n / gw, gj = n % gw;
    const int plen = C * p * p;
    const float* xb = x + static_cast<int64_t>(b % x_mod) * C * H * W;
    for (int q = threadIdx.x; q < plen; q += kThreads) {
        const int c = q / (p * p), ph = (q / p) % p, pq = q % p;
        patch[q] = xb[(static_cast<int64_t>(c) * H + gi * p + ph) * W + gj * p + pq];
    }
    __syncthreads();
    const int64_t row = static_cast<int64_t>(b) * gridDim.x + n;
    for (int j = threadIdx.x; j < D; j += kThreads) {
        float acc = pb[j];
        const float* w = pw + static_cast<int64_t>(j) * plen;
        for (int q = 0; q < plen; ++q) acc = fmaf(patch[q], w[q], acc);
        out[row * D + j] = acc + pos[static_cast<int64_t>(n) * D + j];
    }
}

// Same operation for patches of 16 values (4 channels, 2 x 2) with each thread's weight rows held in
// registers over a run of kPatchTok tokens: read per token from cache the D x 16 matrix costs 74 KB per
// token at D = 1152, two orders of magnitude more than the token's 4.6 KB of output.
constexpr int kPatchTok = 16;
constexpr int kPatchUnroll = 4;
template <int NR>
__global__ __launch_bounds__(kThreads) void patch_embed16_kernel(
    const float* __restrict__ x, int32_t x_mod, int32_t C, int32_t H, int32_t W, int32_t p, int32_t D,
    const float* __restrict__ pw, const float* __restrict__ pb, const float* __restrict__ pos,
    float* __restrict__ out, int32_t ntok) {
    __shared__ __attribute__((aligned(16))) float patch[kPatchTok][16];
    const int gw = W / p;
    const int n0 = blockIdx.x * kPatchTok, b = blockIdx.y;
    const float* xb = x + static_cast<int64_t>(b % x_mod) * C * H * W;
    for (int e = threadIdx.x; e < kPatchTok * 16; e += kThreads) {
        const int tk = e >> 4, q = e & 15;
        const int n = n0 + tk;
        float v = 0.f;
        if (n < ntok) {
            const int gi = n / gw, gj = n % gw;
            const int c = q / (p * p), ph = (q / p) % p, pq = q % p;
            v = xb[(static_cast<int64_t>(c) * H + gi * p + ph) * W + gj * p + pq];
        }
        patch[tk][q] = v;
    }
    float4 w[NR][4];
    float bias[NR];
#pragma unroll
    for (int r = 0; r < NR; ++r) {
        const int j = threadIdx.x + kThreads * r;
        bias[r] = 0.f;
#pragma unroll
        for (int q4 = 0; q4 < 4; ++q4) w[r][q4] = make_float4(0.f, 0.f, 0.f, 0.f);
        if (j < D) {
            bias[r] = pb[j];
#pragma unroll
            for (int q4 = 0; q4 < 4; ++q4) w[r][q4] = reinterpret_cast<const float4*>(pw + static_cast<int64_t>(j) * 16)[q4];
        }
    }
    __syncthreads();
    // groups of kPatchUnroll tokens: the position-table loads of a whole group are issued together, so their
    // latency is paid once per group and not once per token (a block has nothing else to hide it behind)
    for (int tk0 = 0; tk0 < kPatchTok; tk0 += kPatchUnroll) {
        if (n0 + tk0 >= ntok) break;
        float pe[kPatchUnroll][NR];
#pragma unroll
        for (int u = 0; u < kPatchUnroll; ++u)
#pragma unroll
            for (int r = 0; r < NR; ++r) {
                const int n = n0 + tk0 + u, j = threadIdx.x + kThreads * r;
                pe[u][r] = (n < ntok && j < D) ? pos[static_cast<int64_t>(n) * D + j] : 0.f;
            }
#pragma unroll
        for (int u = 0; u < kPatchUnroll; ++u) {
            const int n = n0 + tk0 + u;
            if (n >= ntok) break;
            float4 pv[4];
#pragma unroll
            for (int q4 = 0; q4 < 4; ++q4) pv[q4] = reinterpret_cast<const float4*>(patch[tk0 + u])[q4];
            const int64_t row = static_cast<int64_t>(b) * ntok + n;
#pragma unroll
            for (int r = 0; r < NR; ++r) {
                const int j = threadIdx.x + kThreads * r;
                if (j < D) {
                    float acc = bias[r];
#pragma unroll
                    for (int q4 = 0; q4 < 4; ++q4) {           // same summation order as the generic kernel
                        acc = fmaf(pv[q4].x, w[r][q4].x, acc);
                        acc = fmaf(pv[q4].y, w[r][q4].y, acc);
                        acc = fmaf(pv[q4].z, w[r][q4].z, acc);
                        acc = fmaf(pv[q4].w, w[r][q4].w, acc);
                    }
                    out[row * D + j] = acc + pe[u][r];
                }
            }
        }
    }
}

// The same for widths up to 4 * kPeThreads (every DiT size) with four consecutive output columns per thread: the
// position table is read and the tokens are written 16 bytes per lane, and the four weight rows of a thread stay in
// registers.  A workgroup takes kPeTok consecutive tokens of up to kPeSamples samples: the position vectors are
// loaded once and reused for every sample, all latent values it needs are gathered into LDS up front, and a
// two-sample launch (the drafter's) still covers every CU.
constexpr int kPeThreads = 320;            // 288 of them carry columns at D = 1152
constexpr int kPeTok = 4;
constexpr int kPeSamples = 16;
__global__ __launch_bounds__(kPeThreads) void patch_embed16v_kernel(
    const float* __restrict__ x, int32_t x_mod, int32_t B, int32_t C, int32_t H, int32_t W, int32_t p, int32_t D,
    const float* __restrict__ pw, const float* __restrict__ pb, const float* __restrict__ pos,
    float* __restrict__ out, int32_t ntok) {
    __shared__ __attribute__((aligned(16))) float patch[kPeSamples][kPeTok][16];
    const int gw = W / p;
    const int n0 = blockIdx.x * kPeTok, b0 = blockIdx.y * kPeSamples;
    const int nb = B - b0 < kPeSamples ? B - b0 : kPeSamples;
    for (int e = threadIdx.x; e < nb * kPeTok * 16; e += kPeThreads) {
        const int sb = e / (kPeTok * 16), tk = (e >> 4) % kPeTok, q = e & 15;
        const int n = n0 + tk;
        float v = 0.f;
        if (n < ntok) {
            const float* xb = x + static_cast<int64_t>((b0 + sb) % x_mod) * C * H * W;
            const int gi = n / gw, gj = n % gw;
            const int c = q / (p * p), ph = (q / p) % p, pq = q % p;
            v = xb[(static_cast<int64_t>(c) * H + gi * p + ph) * W + gj * p + pq];
        }
        patch[sb][tk][q] = v;
    }
    const int j0 = 4 * static_cast<int>(threadIdx.x);
    const bool col_on = j0 < D;
    const int jc = col_on ? j0 : 0;                     // idle lanes re-read column 0 and store nothing
    float4 w[4][4];
#pragma unroll
    for (int c = 0; c < 4; ++c)
#pragma unroll
        for (int q4 = 0; q4 < 4; ++q4) w[c][q4] = reinterpret_cast<const float4*>(pw + static_cast<int64_t>(jc + c) * 16)[q4];
    const float4 bias = *reinterpret_cast<const float4*>(pb + jc);
    float4 pe[kPeTok];
#pragma unroll
    for (int u = 0; u < kPeTok; ++u) {
        const int n = n0 + u < ntok ? n0 + u : ntok - 1;
        pe[u] = *reinterpret_cast<const float4*>(pos + static_cast<int64_t>(n) * D + jc);
    }
    __syncthreads();
    for (int sb = 0; sb < nb; ++sb) {
#pragma unroll
        for (int u = 0; u < kPeTok; ++u) {
            const int n = n0 + u;
            float4 pv[4];
#pragma unroll
            for (int q4 = 0; q4 < 4; ++q4) pv[q4] = reinterpret_cast<const float4*>(patch[sb][u])[q4];
            float o[4];
#pragma unroll
            for (int c = 0; c < 4; ++c) {
                float acc = c == 0 ? bias.x : (c == 1 ? bias.y : (c == 2 ? bias.z : bias.w));
#pragma unroll
                for (int q4 = 0; q4 < 4; ++q4) {               // same summation order as the generic kernel
                    acc = fmaf(pv[q4].x, w[c][q4].x, acc);
                    acc = fmaf(pv[q4].y, w[c][q4].y, acc);
                    acc = fmaf(pv[q4].z, w[c][q4].z, acc);
                    acc = fmaf(pv[q4].w, w[c][q4].w, acc);
                }
                o[c] = acc;
            }
            if (col_on && n < ntok)
                *reinterpret_cast<float4*>(out + (static_cast<int64_t>(b0 + sb) * ntok + n) * D + j0) =
                    make_float4(o[0] + pe[u].x, o[1] + pe[u].y, o[2] + pe[u].z, o[3] + pe[u].w);
        }
    }
}

// ---------------------------------------------------------------------------
// LayerNorm (no affine, biased variance, eps 1e-6) + per-sample modulate.
// One wavefront per row; statistics in fp32, two-pass (mean, then centred
// second moment), wavefront-shuffle reductions.
// ---------------------------------------------------------------------------
template <typename OT>
__global__ __launch_bounds__(kThreads) void ln_modulate_kernel(
    const float* __restrict__ x, RowVec shift, RowVec scale, int32_t M, int32_t D, OT* __restrict__ out) {
    const int64_t row = static_cast<int64_t>(blockIdx.x) * kWaves + (threadIdx.x >> 6);
    const int lane = threadIdx.x & 63;
    if (row >= M) return;
    const float* xr = x + row * D;
    float s = 0.f;
    for (int i = lane; i < D; i += 64) s += xr[i];
    const float mean = wave_sum_f(s) / static_cast<float>(D);
    float q = 0.f;
    for (int i = lane; i < D; i += 64) {
        const float c = xr[i] - mean;
        q = fmaf(c, c, q);
    }
    const float rstd = rsqrtf(wave_sum_f(q) / static_cast<float>(D) + kLnEps);
    const float* sh = shift.base + (row / shift.rows_per_sample) * shift.stride;
    const float* sc = scale.base + (row / scale.rows_per_sample) * scale.stride;
    OT* o = out + row * D;
    for (int i = lane; i < D; i += 64) {
        const float v = (xr[i] - mean) * rstd;
        store_f(o + i, fmaf(v, 1.0f + sc[i], sh[i]));
    }
}

// Same operation with the row held in registers: one 16-byte load per element group,
// statistics from registers, one packed store.  HBM-bound (reads 4 B, writes 2 or 4 B per
// element); needs D % 4 == 0, D <= 256 NV and 16-byte aligned rows.
// A wavefront walks kLnRows consecutive rows (4 when there are enough rows to fill the chip that way, else 1): the shift / scale vectors of a sample (as many bytes as the row
// itself, each) stay in registers while the sample does not change - read per row they triple the traffic
// through the L1 - and the next row is requested before the current one is reduced.
template <typename OT, int NV, int kLnRows>
__global__ __launch_bounds__(kThreads) void ln_modulate_vec_kernel(
    const float* __restrict__ x, RowVec shift, RowVec scale, int32_t M, int32_t D, OT* __restrict__ out) {
    const int64_t row0 = (static_cast<int64_t>(blockIdx.x) * kWaves + (threadIdx.x >> 6)) * kLnRows;
    const int lane = threadIdx.x & 63;
    if (row0 >= M) return;
    const int nrows = M - row0 < kLnRows ? static_cast<int>(M - row0) : kLnRows;
    const int nvec = D >> 2;
    auto load_row = [&](float4 (&dst)[NV], int64_t row) {
        const float4* xr = reinterpret_cast<const float4*>(x + row * D);
#pragma unroll
        for (int k = 0; k < NV; ++k) {
            const int v = lane + 64 * k;
            dst[k] = (v < nvec) ? xr[v] : make_float4(0.f, 0.f, 0.f, 0.f);
        }
    };
    float4 xv[NV], xn[NV], shv[NV], scv[NV];
    int64_t sh_smp = -1, sc_smp = -1;
    load_row(xv, row0);
    for (int r = 0; r < nrows; ++r) {
        const int64_t row = row0 + r;
        if (r + 1 < nrows) load_row(xn, row + 1);
        const int64_t s_sh = row / shift.rows_per_sample, s_sc = row / scale.rows_per_sample;
        if (s_sh != sh_smp) {                                  // wave-uniform
            const float4* sh = reinterpret_cast<const float4*>(shift.base + s_sh * shift.stride);
#pragma unroll
            for (int k = 0; k < NV; ++k)
                if (lane + 64 * k < nvec) shv[k] = sh[lane + 64 * k];
            sh_smp = s_sh;
        }
        if (s_sc != sc_smp) {
            const float4* sc = reinterpret_cast<const float4*>(scale.base + s_sc * scale.stride);
#pragma unroll
            for (int k = 0; k < NV; ++k)
                if (lane + 64 * k < nvec) scv[k] = sc[lane + 64 * k];
            sc_smp = s_sc;
        }
        float s = 0.f;
#pragma unroll
        for (int k = 0; k < NV; ++k) s += (xv[k].x + xv[k].y) + (xv[k].z + xv[k].w);
        const float mean = wave_sum_f(s) / static_cast<float>(D);
        float q = 0.f;
#pragma unroll
        for (int k = 0; k < NV; ++k) {
            if (lane + 64 * k < nvec) {
                const float a = xv[k].x - mean, b = xv[k].y - mean, c = xv[k].z - mean, d = xv[k].w - mean;
                q += (a * a + b * b) + (c * c + d * d);
            }
        }
        const float rstd = rsqrtf(wave_sum_f(q) / static_cast<float>(D) + kLnEps);
#pragma unroll
        for (int k = 0; k < NV; ++k) {
            const int v = lane + 64 * k;
            if (v < nvec) {
                const float4 h = shv[k], c = scv[k];
                const float o0 = fmaf((xv[k].x - mean) * rstd, 1.0f + c.x, h.x);
                const float o1 = fmaf((xv[k].y - mean) * rstd, 1.0f + c.y, h.y);
                const float o2 = fmaf((xv[k].z - mean) * rstd, 1.0f + c.z, h.z);
                const float o3 = fmaf((xv[k].w - mean) * rstd, 1.0f + c.w, h.w);
                if constexpr (sizeof(OT) == 2) {
                    uint2 pk;
                    pk.x = pack_bf16_pair(o0, o1);
                    pk.y = pack_bf16_pair(o2, o3);
                    reinterpret_cast<uint2*>(out + row * D)[v] = pk;
                } else {
                    reinterpret_cast<float4*>(out + row * D)[v] = make_float4(o0, o1, o2, o3);
                }
            }
        }
#pragma unroll
        for (int k = 0; k < NV; ++k) xv[k] = xn[k];
    }
}

// ---------------------------------------------------------------------------
// Plain tiled linear layer: out = epilogue(A[M,K] W[N,K]^T + bias), fp32 accumulate.
// 64x64 tile, 16-deep K slices in LDS, 4x4 outputs per thread.
// ---------------------------------------------------------------------------
template <typename T, int EPI>
__global__ __launch_bounds__(kThreads) void linear_simple_kernel(
    const T* __restrict__ A, const T* __restrict__ W, const float* __restrict__ bias, int32_t M, int32_t N,
    int32_t K, T* __restrict__ out, float* __restrict__ resid, RowVec gate) {
    constexpr int BM = 64, BN = 64, BK = 16;
    __shared__ float sA[BK][BM + 4];
    __shared__ float sW[BK][BN + 4];
    const int tx = threadIdx.x % 16, ty = threadIdx.x / 16;
    const int m0 = blockIdx.y * BM, n0 = blockIdx.x * BN;
    float acc[4][4];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) acc[i][j] = 0.f;

    for (int k0 = 0; k0 < K; k0 += BK) {
        // each thread loads 4 elements of each tile: tile element e = threadIdx.x + 256 i
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int e = threadIdx.x + kThreads * i;
            const int r = e / BK, kk = e % BK;
            const int gm = m0 + r, gn = n0 + r, gk = k0 + kk;
            sA[kk][r] = (gm < M && gk < K) ? load_f(A + static_cast<int64_t>(gm) * K + gk) : 0.f;
            sW[kk][r] = (gn < N && gk < K) ? load_f(W + static_cast<int64_t>(gn) * K + gk) : 0.f;
        }
        __syncthreads();
#pragma unroll
        for (int kk = 0; kk < BK; ++kk) {
            float a[4], w[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) a[i] = sA[kk][ty * 4 + i];
#pragma unroll
            for (int j = 0; j < 4; ++j) w[j] = sW[kk][tx * 4 + j];
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
                for (int j = 0; j < 4; ++j) acc[i][j] = fmaf(a[i], w[j], acc[i][j]);
        }
        __syncthreads();
    }
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int gm = m0 + ty * 4 + i;
        if (gm >= M) continue;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int gn = n0 + tx * 4 + j;
            if (gn >= N) continue;
            float v = acc[i][j] + bias[gn];
            const int64_t o = static_cast<int64_t>(gm) * N + gn;
            if (EPI == FREE_EPI_BIAS) {
                store_f(out + o, v);
            } else if (EPI == FREE_EPI_BIAS_GELU) {
                store_f(out + o, gelu_tanh_f(v));
            } else {
                const float g = gate.base[static_cast<int64_t>(gm / gate.rows_per_sample) * gate.stride + gn];
                resid[o] = fmaf(g, v, resid[o]);
            }
        }
    }
}

// ---------------------------------------------------------------------------
// Plain attention: one thread per query row, K/V tiles broadcast from LDS,
// online softmax in fp32.
// ---------------------------------------------------------------------------
template <typename T, int DH>
__global__ __launch_bounds__(128) void attention_simple_kernel(const T* __restrict__ qkv, int32_t N,
                                                               int32_t heads, int32_t dh,
                                                               T* __restrict__ out) {
    constexpr int BQ = 128, BKV = 32;
    __shared__ float sK[BKV][DH];
    __shared__ float sV[BKV][DH];
    const int h = blockIdx.y, b = blockIdx.z;
    const int D = heads * dh;
    const int64_t row0 = static_cast<int64_t>(b) * N;
    const int qi = blockIdx.x * BQ + threadIdx.x;
    const bool active = qi < N;
    const float scale = 1.0f / sqrtf(static_cast<float>(dh));

    float q[DH], o[DH];
#pragma unroll
    for (int i = 0; i < DH; ++i) {
        q[i] = (active && i < dh) ? load_f(qkv + (row0 + qi) * 3 * D + h * dh + i) * scale : 0.f;
        o[i] = 0.f;
    }
    float mx = -INFINITY, l = 0.f;

    for (int kv0 = 0; kv0 < N; kv0 += BKV) {
        __syncthreads();
        for (int e = threadIdx.x; e < BKV * DH; e += BQ) {
            const int r = e / DH, c = e % DH;
            const int kv = kv0 + r;
            float kk = 0.f, vv = 0.f;
            if (kv < N && c < dh) {
                const T* base = qkv + (row0 + kv) * 3 * D + h * dh + c;
                kk = load_f(base + D);
                vv = load_f(base + 2 * D);
            }
            sK[r][c] = kk;
            sV[r][c] = vv;
        }
        __syncthreads();
        const int nkv = (N - kv0 < BKV) ? N - kv0 : BKV;
        float s[BKV];
        float tmax = -INFINITY;
#pragma unroll
        for (int r = 0; r < BKV; ++r) {
            float a = 0.f;
#pragma unroll
            for (int i = 0; i < DH; ++i) a = fmaf(q[i], sK[r][i], a);
            s[r] = (r < nkv) ? a : -INFINITY;
            tmax = fmaxf(tmax, s[r]);
        }
        const float nm = fmaxf(mx, tmax);
        const float corr = expf(mx - nm);
        l *= corr;
#pragma unroll
        for (int i = 0; i < DH; ++i) o[i] *= corr;
#pragma unroll
        for (int r = 0; r < BKV; ++r) {
            const float pr = expf(s[r] - nm);          // exp(-inf) = 0 for padded keys
            l += pr;
#pragma unroll
            for (int i = 0; i < DH; ++i) o[i] = fmaf(pr, sV[r][i], o[i]);
        }
        mx = nm;
    }
    if (active) {
        const float inv = 1.0f / l;
#pragma unroll
        for (int i = 0; i < DH; ++i)
            if (i < dh) store_f(out + (row0 + qi) * D + h * dh + i, o[i] * inv);
    }
}

// ---------------------------------------------------------------------------
// Final layer: LN + modulate, Linear(D -> p^2 c_out), unpatchify to [B, c_out, H, W].
// One wavefront per token.
// ---------------------------------------------------------------------------
template <typename WT>
__global__ __launch_bounds__(kThreads) void final_layer_kernel(
    const float* __restrict__ x, RowVec shift, RowVec scale, int32_t M, int32_t gh, int32_t gw, int32_t p,
    int32_t c_out, int32_t D, const WT* __restrict__ w, const float* __restrict__ bias,
    float* __restrict__ out) {
    constexpr int OC = 8;                                // outputs per pass
    const int64_t row = static_cast<int64_t>(blockIdx.x) * kWaves + (threadIdx.x >> 6);
    const int lane = threadIdx.x & 63;
    if (row >= M) return;
    const float* xr = x + row * D;
    float s = 0.f;
    for (int i = lane; i < D; i += 64) s += xr[i];
    const float mean = wave_sum_f(s) / static_cast<float>(D);
    float q = 0.f;
    for (int i = lane; i < D; i += 64) {
        const float c = xr[i] - mean;
        q = fmaf(c, c, q);
    }
    const float rstd = rsqrtf(wave_sum_f(q) / static_cast<float>(D) + kLnEps);
    const float* sh = shift.base + (row / shift.rows_per_sample) * shift.stride;
    const float* sc = scale.base + (row / scale.rows_per_sample) * scale.stride;
    const int ntok = gh * gw;
    const int b = static_cast<int>(row / ntok), n = static_cast<int>(row % ntok);
    const int gi = n / gw, gj = n % gw;
    const int P = p * p * c_out;
    const int H = gh * p, Wd = gw * p;
    for (int o0 = 0; o0 < P; o0 += OC) {
        float acc[OC];
#pragma unroll
        for (int k = 0; k < OC; ++k) acc[k] = 0.f;
        for (int i = lane; i < D; i += 64) {
            const float v = fmaf((xr[i] - mean) * rstd, 1.0f + sc[i], sh[i]);
#pragma unroll
            for (int k = 0; k < OC; ++k)
                if (o0 + k < P) acc[k] = fmaf(v, load_f(w + static_cast<int64_t>(o0 + k) * D + i), acc[k]);
        }
#pragma unroll
        for (int k = 0; k < OC; ++k) {
            const float v = wave_sum_f(acc[k]);
            const int o = o0 + k;
            if (lane == 0 && o < P) {
                const int c = o % c_out, pq = (o / c_out) % p, ph = o / (c_out * p);
                out[((static_cast<int64_t>(b) * c_out + c) * H + gi * p + ph) * Wd + gj * p + pq] = v + bias[o];
            }
        }
    }
}

// One wavefront per token row, read once: the normalised, modulated row stays in
// registers (NV float4 per lane) and every output column is a dot product of registers
// with a weight row streamed from cache.  Needs D % 4 == 0, D <= 256 NV, 16-byte rows.
template <typename WT, int NV>
__global__ __launch_bounds__(kThreads) void final_layer_row_kernel(
    const float* __restrict__ x, RowVec shift, RowVec scale, int32_t M, int32_t gh, int32_t gw, int32_t p,
    int32_t c_out, int32_t D, const WT* __restrict__ w, const float* __restrict__ bias,
    float* __restrict__ out) {
    const int64_t row = static_cast<int64_t>(blockIdx.x) * kWaves + (threadIdx.x >> 6);
    const int lane = threadIdx.x & 63;
    if (row >= M) return;
    const int nvec = D >> 2;
    const float4* xr = reinterpret_cast<const float4*>(x + row * D);
    float4 xv[NV];
    float s = 0.f;
#pragma unroll
    for (int k = 0; k < NV; ++k) {
        const int v = lane + 64 * k;
        xv[k] = (v < nvec) ? xr[v] : make_float4(0.f, 0.f, 0.f, 0.f);
        s += (xv[k].x + xv[k].y) + (xv[k].z + xv[k].w);
    }
    const float mean = wave_sum_f(s) / static_cast<float>(D);
    float q = 0.f;
#pragma unroll
    for (int k = 0; k < NV; ++k) {
        if (lane + 64 * k < nvec) {
            const float a = xv[k].x - mean, b = xv[k].y - mean, c = xv[k].z - mean, d = xv[k].w - mean;
            q += (a * a + b * b) + (c * c + d * d);
        }
    }
    const float rstd = rsqrtf(wave_sum_f(q) / static_cast<float>(D) + kLnEps);
    const float4* sh = reinterpret_cast<const float4*>(shift.base + (row / shift.rows_per_sample) * shift.stride);
    const float4* sc = reinterpret_cast<const float4*>(scale.base + (row / scale.rows_per_sample) * scale.stride);
#pragma unroll
    for (int k = 0; k < NV; ++k) {
        const int v = lane + 64 * k;
        if (v < nvec) {
            const float4 h = sh[v], c = sc[v];
            xv[k].x = fmaf((xv[k].x - mean) * rstd, 1.0f + c.x, h.x);
            xv[k].y = fmaf((xv[k].y - mean) * rstd, 1.0f + c.y, h.y);
            xv[k].z = fmaf((xv[k].z - mean) * rstd, 1.0f + c.z, h.z);
            xv[k].w = fmaf((xv[k].w - mean) * rstd, 1.0f + c.w, h.w);
        } else {
            xv[k] = make_float4(0.f, 0.f, 0.f, 0.f);
        }
    }
    const int ntok = gh * gw;
    const int b = static_cast<int>(row / ntok), n = static_cast<int>(row % ntok);
    const int gi = n / gw, gj = n % gw;
    const int P = p * p * c_out;
    const int H = gh * p, Wd = gw * p;
    for (int o = 0; o < P; ++o) {
        const WT* wr = w + static_cast<int64_t>(o) * D;
        float acc = 0.f;
#pragma unroll
        for (int k = 0; k < NV; ++k) {
            const int v = lane + 64 * k;
            if (v < nvec) {
                float w0, w1, w2, w3;
                if constexpr (sizeof(WT) == 2) {
                    const uint2 pk = reinterpret_cast<const uint2*>(wr)[v];
                    w0 = __uint_as_float(pk.x << 16);
                    w1 = __uint_as_float(pk.x & 0xffff0000u);
                    w2 = __uint_as_float(pk.y << 16);
                    w3 = __uint_as_float(pk.y & 0xffff0000u);
                } else {
                    const float4 f = reinterpret_cast<const float4*>(wr)[v];
                    w0 = f.x; w1 = f.y; w2 = f.z; w3 = f.w;
                }
                acc = fmaf(xv[k].x, w0, acc);
                acc = fmaf(xv[k].y, w1, acc);
                acc = fmaf(xv[k].z, w2, acc);
                acc = fmaf(xv[k].w, w3, acc);
            }
        }
        acc = wave_sum_f(acc);
        if (lane == 0) {
            const int c = o % c_out, pq = (o / c_out) % p, ph = o / (c_out * p);
            out[((static_cast<int64_t>(b) * c_out + c) * H + gi * p + ph) * Wd + gj * p + pq] = acc + bias[o];
        }
    }
}

// Few rows (e.g. the drafter's two samples): weights staged in LDS, all P dot products kept per lane.
// Same operation with the token row read once: the normalised, modulated row stays in
// registers (NV float4 per lane) and every output column is a dot product of registers
// with a weight row streamed from cache.  Needs D % 4 == 0, D <= 256 NV, 16-byte rows.
// The P <= 32 partial dot products of a lane are reduced over the wavefront together: five
// halving exchanges (lane ^ 32, 16, 8, 4, 2: each lane keeps half of its values and adds the
// partner's other half) leave one output per lane pair, one more exchange completes it - 32
// cross-lane operations in independent groups instead of six dependent ones per output.
template <typename WT, int NV, bool kStage>
__global__ __launch_bounds__(kThreads) void final_layer_vec_kernel(
    const float* __restrict__ x, RowVec shift, RowVec scale, int32_t M, int32_t gh, int32_t gw, int32_t p,
    int32_t c_out, int32_t D, const WT* __restrict__ w, const float* __restrict__ bias,
    float* __restrict__ out) {
    // kStage (few rows, e.g. the drafter's two samples): the projection matrix (P x D, 74 KB in bf16 at
    // DiT-XL/2) is staged in LDS once per workgroup and every wavefront walks token rows with a grid
    // stride; read per row from L2 it costs P D bytes of cache traffic per token and that dominates when
    // there are too few wavefronts to hide it.  With many rows one wavefront per row and weights
    // from cache is faster (more wavefronts in flight).
    extern __shared__ __attribute__((aligned(16))) char lds_w_raw[];
    const WT* lw = kStage ? reinterpret_cast<const WT*>(lds_w_raw) : w;
    if (kStage) {
        const int n16 = (p * p * c_out * D * static_cast<int>(sizeof(WT))) / 16;
        const uint4* src = reinterpret_cast<const uint4*>(w);
        uint4* dst = reinterpret_cast<uint4*>(lds_w_raw);
        for (int i = threadIdx.x; i < n16; i += kThreads) dst[i] = src[i];
    }
    if (kStage) __syncthreads();
    const int lane = threadIdx.x & 63;
    for (int64_t row = static_cast<int64_t>(blockIdx.x) * kWaves + (threadIdx.x >> 6); row < M;
         row += static_cast<int64_t>(gridDim.x) * kWaves) {
    const int nvec = D >> 2;
    const float4* xr = reinterpret_cast<const float4*>(x + row * D);
    float4 xv[NV];
    float s = 0.f;
#pragma unroll
    for (int k = 0; k < NV; ++k) {
        const int v = lane + 64 * k;
        xv[k] = (v < nvec) ? xr[v] : make_float4(0.f, 0.f, 0.f, 0.f);
        s += (xv[k].x + xv[k].y) + (xv[k].z + xv[k].w);
    }
    const float mean = wave_sum_f(s) / static_cast<float>(D);
    float q = 0.f;
#pragma unroll
    for (int k = 0; k < NV; ++k) {
        if (lane + 64 * k < nvec) {
            const float a = xv[k].x - mean, b = xv[k].y - mean, c = xv[k].z - mean, d = xv[k].w - mean;
            q += (a * a + b * b) + (c * c + d * d);
        }
    }
    const float rstd = rsqrtf(wave_sum_f(q) / static_cast<float>(D) + kLnEps);
    const float4* sh = reinterpret_cast<const float4*>(shift.base + (row / shift.rows_per_sample) * shift.stride);
    const float4* sc = reinterpret_cast<const float4*>(scale.base + (row / scale.rows_per_sample) * scale.stride);
#pragma unroll
    for (int k = 0; k < NV; ++k) {
        const int v = lane + 64 * k;
        if (v < nvec) {
            const float4 h = sh[v], c = sc[v];
            xv[k].x = fmaf((xv[k].x - mean) * rstd, 1.0f + c.x, h.x);
            xv[k].y = fmaf((xv[k].y - mean) * rstd, 1.0f + c.y, h.y);
            xv[k].z = fmaf((xv[k].z - mean) * rstd, 1.0f + c.z, h.z);
            xv[k].w = fmaf((xv[k].w - mean) * rstd, 1.0f + c.w, h.w);
        } else {
            xv[k] = make_float4(0.f, 0.f, 0.f, 0.f);
        }
    }
    const int ntok = gh * gw;
    const int b = static_cast<int>(row / ntok), n = static_cast<int>(row % ntok);
    const int gi = n / gw, gj = n % gw;
    const int P = p * p * c_out;
    const int H = gh * p, Wd = gw * p;
    for (int o0 = 0; o0 < P; o0 += 32) {
        float acc[32];
#pragma unroll
        for (int j = 0; j < 32; ++j) {
            acc[j] = 0.f;
            if (o0 + j < P) {
                const WT* wr = lw + static_cast<int64_t>(o0 + j) * D;
#pragma unroll
                for (int k = 0; k < NV; ++k) {
                    const int v = lane + 64 * k;
                    if (v < nvec) {
                        float w0, w1, w2, w3;
                        if constexpr (sizeof(WT) == 2) {
                            const uint2 pk = reinterpret_cast<const uint2*>(wr)[v];
                            w0 = __uint_as_float(pk.x << 16);
                            w1 = __uint_as_float(pk.x & 0xffff0000u);
                            w2 = __uint_as_float(pk.y << 16);
                            w3 = __uint_as_float(pk.y & 0xffff0000u);
                        } else {
                            const float4 f = reinterpret_cast<const float4*>(wr)[v];
                            w0 = f.x; w1 = f.y; w2 = f.z; w3 = f.w;
                        }
                        acc[j] = fmaf(xv[k].x, w0, acc[j]);
                        acc[j] = fmaf(xv[k].y, w1, acc[j]);
                        acc[j] = fmaf(xv[k].z, w2, acc[j]);
                        acc[j] = fmaf(xv[k].w, w3, acc[j]);
                    }
                }
            }
        }
        // halving exchanges: after the step with offset 32 >> t a lane holds 16 >> t values
#pragma unroll
        for (int t = 0; t < 5; ++t) {
            const int off = 32 >> t, half = 16 >> t;
            const bool upper = (lane & off) != 0;
#pragma unroll
            for (int j = 0; j < 16; ++j) {
                if (j < half) {
                    const float send = upper ? acc[j] : acc[j + half];
                    const float keep = upper ? acc[j + half] : acc[j];
                    acc[j] = keep + __shfl_xor(send, off, 64);
                }
            }
        }
        const float total = acc[0] + __shfl_xor(acc[0], 1, 64);
        // the value a lane ends with: bit 5 of the lane chose the upper 16 outputs, bit 4 the upper 8 of those, ...
        const int o = o0 + ((lane >> 5) & 1) * 16 + ((lane >> 4) & 1) * 8 + ((lane >> 3) & 1) * 4 + ((lane >> 2) & 1) * 2 +
                      ((lane >> 1) & 1);
        if ((lane & 1) == 0 && o < P) {
            const int c = o % c_out, pq = (o / c_out) % p, ph = o / (c_out * p);
            out[((static_cast<int64_t>(b) * c_out + c) * H + gi * p + ph) * Wd + gj * p + pq] = total + bias[o];
        }
    }
    }
}

// ---------------------------------------------------------------------------
// Guidance + eps -> mean (Eq. ddpm_update): m_k = coef_x[k] x_k + coef_eps[k] eps_k,
// eps = eps_null + s (eps_cond - eps_null) when the batch carries both halves.
// ---------------------------------------------------------------------------
// Optionally also the draw of the next state, x_next = m + sigma_step[k] * xi (Alg. 1: next draft, or the
// plain target step); x_next may be x_states itself (each thread reads its element before it writes it).
__global__ void eps_to_mean_kernel(const float* __restrict__ eps_out, const float* x_states,
                                   const float* __restrict__ coef_x, const float* __restrict__ coef_eps,
                                   float cfg_scale, int32_t use_cfg, int32_t K, int32_t C, int32_t c_out,
                                   int64_t hw, float* __restrict__ m_out, float* __restrict__ eps_guided,
                                   const float* __restrict__ sigma_step, const float* __restrict__ xi,
                                   float* x_next) {
    const int64_t idx = static_cast<int64_t>(blockIdx.x) * blockDim.x + threadIdx.x;
    const int64_t per = static_cast<int64_t>(C) * hw;
    if (idx >= per * K) return;
    const int k = static_cast<int>(idx / per);
    const int64_t rem = idx % per;                        // c * hw + s
    float eps = eps_out[static_cast<int64_t>(k) * c_out * hw + rem];
    if (use_cfg) {
        const float en = eps_out[static_cast<int64_t>(K + k) * c_out * hw + rem];
        eps = fmaf(cfg_scale, eps - en, en);
    }
    const float m = fmaf(coef_x[k], x_states[idx], coef_eps[k] * eps);
    m_out[idx] = m;
    if (eps_guided) eps_guided[idx] = eps;
    if (x_next) x_next[idx] = fmaf(sigma_step[k], xi[idx], m);
}

__global__ void pack_cond_kernel(const int32_t* __restrict__ t, int32_t y, int32_t null_label, int32_t K,
                                 int32_t dup, int32_t* __restrict__ t_out, int32_t* __restrict__ y_out) {
    const int b = blockIdx.x * blockDim.x + threadIdx.x;
    if (b >= K * dup) return;
    t_out[b] = t[b % K];
    y_out[b] = (b < K) ? y : null_label;
}

}  // namespace

// ============================ host launch wrappers ============================

int32_t launch_conditioning(const int32_t* t, const int32_t* y, int32_t B, int32_t D, int32_t tfreq,
                            const float* w1, const float* b1, const float* w2, const float* b2,
                            const float* ytab, float* h1, float* sc, hipStream_t s) {
    // h1 doubles as [B, tfreq] timestep embedding followed by [B, D] hidden
    float* temb = h1;
    float* hid = h1 + static_cast<int64_t>(B) * tfreq;
    const int n = B * (tfreq / 2);
    hipLaunchKernelGGL(timestep_embed_kernel, dim3((n + 255) / 256), dim3(256), 0, s, t, B, tfreq, temb);
    if (!launch_ok()) return FREE_ERR_HIP;
    auto al16 = [](const void* q) { return (reinterpret_cast<uintptr_t>(q) & 15u) == 0; };
    if (tfreq % 4 == 0 && D % 4 == 0 && al16(h1) && al16(w1) && al16(w2)) {
        const dim3 g((D + kWaves - 1) / kWaves);
        hipLaunchKernelGGL(small_linear_rows_kernel<true>, g, dim3(kThreads), 0, s, temb, B, tfreq, D, w1, b1,
                           static_cast<const float*>(nullptr), static_cast<const int32_t*>(nullptr), hid);
        if (!launch_ok()) return FREE_ERR_HIP;
        hipLaunchKernelGGL(small_linear_rows_kernel<true>, g, dim3(kThreads), 0, s, hid, B, D, D, w2, b2, ytab, y, sc);
        return launch_ok() ? FREE_OK : FREE_ERR_HIP;
    }
    dim3 g((D + kWaves - 1) / kWaves, B);
    hipLaunchKernelGGL(small_linear_kernel<true>, g, dim3(kThreads), 0, s, temb, B, tfreq, D, w1, b1,
                       static_cast<const float*>(nullptr), static_cast<const int32_t*>(nullptr), hid);
    if (!launch_ok()) return FREE_ERR_HIP;
    hipLaunchKernelGGL(small_linear_kernel<true>, g, dim3(kThreads), 0, s, hid, B, D, D, w2, b2, ytab, y, sc);
    if (!launch_ok()) return FREE_ERR_HIP;
    return FREE_OK;
}

int32_t launch_adaln(const float* sc, int32_t B, int32_t D, const void* const* w_tab,
                     const float* const* b_tab, const int32_t* row_start, int32_t n_mats,
                     int32_t total_rows, int32_t dtype, float* mod, hipStream_t s) {
    const int rows_per_wave = 8;
    const int waves = (total_rows + rows_per_wave - 1) / rows_per_wave;
    const int blocks = (waves + kWaves - 1) / kWaves;
    const int nb = B < kAdaBatch ? B : kAdaBatch;
    const size_t lds = static_cast<size_t>(nb) * D * sizeof(float);
    if (lds > 150 * 1024) return FREE_ERR_SHAPE;
    if (dtype == FREE_BF16) {
        if (!hip_ok(hipFuncSetAttribute(reinterpret_cast<const void*>(adaln_kernel<bf16_t>),
                                        hipFuncAttributeMaxDynamicSharedMemorySize, static_cast<int>(lds))))
            return FREE_ERR_HIP;
        hipLaunchKernelGGL(adaln_kernel<bf16_t>, dim3(blocks), dim3(kThreads), lds, s, sc, B, D, w_tab, b_tab,
                           row_start, n_mats, total_rows, rows_per_wave, mod);
    } else {
        if (!hip_ok(hipFuncSetAttribute(reinterpret_cast<const void*>(adaln_kernel<float>),
                                        hipFuncAttributeMaxDynamicSharedMemorySize, static_cast<int>(lds))))
            return FREE_ERR_HIP;
        hipLaunchKernelGGL(adaln_kernel<float>, dim3(blocks), dim3(kThreads), lds, s, sc, B, D, w_tab, b_tab,
                           row_start, n_mats, total_rows, rows_per_wave, mod);
    }
    return launch_ok() ? FREE_OK : FREE_ERR_HIP;
}

int32_t launch_patch_embed(const float* x, int32_t x_mod, int32_t B, int32_t C, int32_t H, int32_t W,
                           int32_t p, int32_t D, const float* pw, const float* pb, const float* pos,
                           float* out, hipStream_t s) {
    const int ntok = (H / p) * (W / p);
    auto al16 = [](const void* q) { return (reinterpret_cast<uintptr_t>(q) & 15u) == 0; };
    if (C * p * p == 16 && D % 4 == 0 && D <= 4 * kPeThreads && al16(pw) && al16(pb) && al16(pos) && al16(out)) {
        hipLaunchKernelGGL(patch_embed16v_kernel, dim3((ntok + kPeTok - 1) / kPeTok, (B + kPeSamples - 1) / kPeSamples),
                           dim3(kPeThreads), 0, s, x, x_mod, B, C, H, W, p, D, pw, pb, pos, out, ntok);
        return launch_ok() ? FREE_OK : FREE_ERR_HIP;
    }
    if (C * p * p == 16 && D <= 8 * kThreads && (reinterpret_cast<uintptr_t>(pw) & 15u) == 0) {
        const dim3 grid((ntok + kPatchTok - 1) / kPatchTok, B);
        const int nr = (D + kThreads - 1) / kThreads;
#define FREE_PE_CASE(NR)                                                                                        \
    hipLaunchKernelGGL(patch_embed16_kernel<NR>, grid, dim3(kThreads), 0, s, x, x_mod, C, H, W, p, D, pw, pb, pos, \
                       out, ntok)
        if (nr <= 1) FREE_PE_CASE(1);
        else if (nr <= 2) FREE_PE_CASE(2);
        else if (nr <= 5) FREE_PE_CASE(5);
        else FREE_PE_CASE(8);
#undef FREE_PE_CASE
        return launch_ok() ? FREE_OK : FREE_ERR_HIP;
    }
    const size_t lds = static_cast<size_t>(C) * p * p * sizeof(float);
    hipLaunchKernelGGL(patch_embed_kernel, dim3(ntok, B), dim3(kThreads), lds, s, x, x_mod, C, H, W, p, D, pw,
                       pb, pos, out);
    return launch_ok() ? FREE_OK : FREE_ERR_HIP;
}

int32_t launch_ln_modulate(const float* x, RowVec shift, RowVec scale, int32_t M, int32_t D, int32_t dtype,
                           void* out, hipStream_t s) {
    const int blocks = (M + kWaves - 1) / kWaves;
    auto al16 = [](const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; };
    const bool vec = (D % 4 == 0) && D <= 2048 && al16(x) && al16(out) && al16(shift.base) && al16(scale.base) &&
                     (shift.stride % 4 == 0) && (scale.stride % 4 == 0);
    if (vec) {
        const int nv = (D / 4 + 63) / 64;
#define FREE_LN_CASE(OT, NV)                                                                                   \
    do {                                                                                                       \
        if (rows_per_wave == 4)                                                                                \
            hipLaunchKernelGGL((ln_modulate_vec_kernel<OT, NV, 4>), dim3((blocks + 3) / 4), dim3(kThreads), 0, s, x, \
                               shift, scale, M, D, static_cast<OT*>(out));                                     \
        else if (rows_per_wave == 2)                                                                           \
            hipLaunchKernelGGL((ln_modulate_vec_kernel<OT, NV, 2>), dim3((blocks + 1) / 2), dim3(kThreads), 0, s, x, \
                               shift, scale, M, D, static_cast<OT*>(out));                                     \
        else                                                                                                   \
            hipLaunchKernelGGL((ln_modulate_vec_kernel<OT, NV, 1>), dim3(blocks), dim3(kThreads), 0, s, x, shift, \
                               scale, M, D, static_cast<OT*>(out));                                            \
    } while (0)
        // measured at D = 1152: 12288 rows 19.3 / 16.2 / 15.8 us with 1 / 2 / 4 rows per wavefront, 6144 rows
        // 10.4 / 9.1 / 10.0 us; with few rows the chain of one row's latencies is what counts
        const int rows_per_wave = M >= 8192 ? 4 : (M >= 4096 ? 2 : 1);
        if (dtype == FREE_BF16) {
            if (nv <= 1) FREE_LN_CASE(bf16_t, 1);
            else if (nv <= 2) FREE_LN_CASE(bf16_t, 2);
            else if (nv <= 5) FREE_LN_CASE(bf16_t, 5);
            else FREE_LN_CASE(bf16_t, 8);
        } else {
            if (nv <= 1) FREE_LN_CASE(float, 1);
            else if (nv <= 2) FREE_LN_CASE(float, 2);
            else if (nv <= 5) FREE_LN_CASE(float, 5);
            else FREE_LN_CASE(float, 8);
        }
#undef FREE_LN_CASE
        return launch_ok() ? FREE_OK : FREE_ERR_HIP;
    }
    if (dtype == FREE_BF16)
        hipLaunchKernelGGL(ln_modulate_kernel<bf16_t>, dim3(blocks), dim3(kThreads), 0, s, x, shift, scale, M, D,
                           static_cast<bf16_t*>(out));
    else
        hipLaunchKernelGGL(ln_modulate_kernel<float>, dim3(blocks), dim3(kThreads), 0, s, x, shift, scale, M, D,
                           static_cast<float*>(out));
    return launch_ok() ? FREE_OK : FREE_ERR_HIP;
}

template <typename T>
static int32_t linear_simple_t(const T* A, const T* W, const float* bias, int32_t M, int32_t N, int32_t K,
                               int32_t epi, T* out, float* resid, RowVec gate, hipStream_t s) {
    dim3 g((N + 63) / 64, (M + 63) / 64);
    switch (epi) {
        case FREE_EPI_BIAS:
            hipLaunchKernelGGL((linear_simple_kernel<T, FREE_EPI_BIAS>), g, dim3(kThreads), 0, s, A, W, bias, M, N,
                               K, out, resid, gate);
            break;
        case FREE_EPI_BIAS_GELU:
            hipLaunchKernelGGL((linear_simple_kernel<T, FREE_EPI_BIAS_GELU>), g, dim3(kThreads), 0, s, A, W, bias,
                               M, N, K, out, resid, gate);
            break;
        case FREE_EPI_GATE_RESID:
            hipLaunchKernelGGL((linear_simple_kernel<T, FREE_EPI_GATE_RESID>), g, dim3(kThreads), 0, s, A, W, bias,
                               M, N, K, out, resid, gate);
            break;
        default:
            return FREE_ERR_RANGE;
    }
    return launch_ok() ? FREE_OK : FREE_ERR_HIP;
}

int32_t launch_linear_simple(const void* A, const void* W, const float* bias, int32_t M, int32_t N, int32_t K,
                             int32_t dtype, int32_t epi, void* out, float* resid, RowVec gate, hipStream_t s) {
    if (dtype == FREE_BF16)
        return linear_simple_t(static_cast<const bf16_t*>(A), static_cast<const bf16_t*>(W), bias, M, N, K, epi,
                               static_cast<bf16_t*>(out), resid, gate, s);
    return linear_simple_t(static_cast<const float*>(A), static_cast<const float*>(W), bias, M, N, K, epi,
                           static_cast<float*>(out), resid, gate, s);
}

template <typename T>
static int32_t attention_simple_t(const T* qkv, int32_t B, int32_t N, int32_t heads, int32_t dh, T* out,
                                  hipStream_t s) {
    dim3 g((N + 127) / 128, heads, B);
#define FREE_ATTN_CASE(DHMAX)                                                                          \
    hipLaunchKernelGGL((attention_simple_kernel<T, DHMAX>), g, dim3(128), 0, s, qkv, N, heads, dh, out)
    if (dh <= 16) FREE_ATTN_CASE(16);
    else if (dh <= 32) FREE_ATTN_CASE(32);
    else if (dh <= 64) FREE_ATTN_CASE(64);
    else if (dh <= 72) FREE_ATTN_CASE(72);
    else if (dh <= 128) FREE_ATTN_CASE(128);
    else return FREE_ERR_SHAPE;
#undef FREE_ATTN_CASE
    return launch_ok() ? FREE_OK : FREE_ERR_HIP;
}

int32_t launch_attention_simple(const void* qkv, int32_t B, int32_t N, int32_t heads, int32_t dh, int32_t dtype,
                                void* out, hipStream_t s) {
    if (dtype == FREE_BF16)
        return attention_simple_t(static_cast<const bf16_t*>(qkv), B, N, heads, dh, static_cast<bf16_t*>(out), s);
    return attention_simple_t(static_cast<const float*>(qkv), B, N, heads, dh, static_cast<float*>(out), s);
}

int32_t launch_final_layer(const float* x, RowVec shift, RowVec scale, int32_t B, int32_t gh, int32_t gw,
                           int32_t p, int32_t c_out, int32_t D, const void* w, const float* bias, int32_t dtype,
                           float* out, hipStream_t s) {
    const int M = B * gh * gw;
    const int blocks = (M + kWaves - 1) / kWaves;
    auto al16 = [](const void* q) { return (reinterpret_cast<uintptr_t>(q) & 15u) == 0; };
    bool vec = (D % 4 == 0) && D <= 2048 && al16(x) && al16(w) && al16(shift.base) && al16(scale.base) &&
                     (shift.stride % 4 == 0) && (scale.stride % 4 == 0);
    const size_t lds_bytes = static_cast<size_t>(p) * p * c_out * D * (dtype == FREE_BF16 ? 2 : 4);
    if (vec && dtype == FREE_BF16 && final_mfma_supported(D, p * p * c_out))
        return launch_final_layer_mfma(x, shift, scale, M, gh, gw, p, c_out, D, static_cast<const bf16_t*>(w), bias,
                                       out, s);
    if (vec) {
        const int nv = (D / 4 + 63) / 64;
        // few rows: stage the weights in LDS, as many workgroups as fit on the chip at once (LDS-limited),
        // each walking rows with a grid stride; many rows: one wavefront per row
        const bool stage = M <= 4096 && lds_bytes <= static_cast<size_t>(kMaxFinalLds) && lds_bytes % 16 == 0;
        const int per_cu = lds_bytes * 2 <= static_cast<size_t>(kMaxFinalLds) ? 2 : 1;
        const int vblocks = blocks < 256 * per_cu ? blocks : 256 * per_cu;
#define FREE_ROW_CASE(WT, NV)                                                                                  \
    hipLaunchKernelGGL((final_layer_row_kernel<WT, NV>), dim3(blocks), dim3(kThreads), 0, s, x, shift, scale, M, gh, \
                       gw, p, c_out, D, static_cast<const WT*>(w), bias, out)
        if (!stage) {
            if (dtype == FREE_BF16) {
                if (nv <= 1) FREE_ROW_CASE(bf16_t, 1);
                else if (nv <= 2) FREE_ROW_CASE(bf16_t, 2);
                else if (nv <= 5) FREE_ROW_CASE(bf16_t, 5);
                else FREE_ROW_CASE(bf16_t, 8);
            } else {
                if (nv <= 1) FREE_ROW_CASE(float, 1);
                else if (nv <= 2) FREE_ROW_CASE(float, 2);
                else if (nv <= 5) FREE_ROW_CASE(float, 5);
                else FREE_ROW_CASE(float, 8);
            }
            return launch_ok() ? FREE_OK : FREE_ERR_HIP;
        }
#undef FREE_ROW_CASE
#define FREE_FIN_CASE(WT, NV)                                                                                  \
    do {                                                                                                       \
        auto kern = final_layer_vec_kernel<WT, NV, true>;                                                      \
        static bool attr_set = false;                                                                          \
        if (stage && !attr_set) {                                                                              \
            if (!hip_ok(hipFuncSetAttribute(reinterpret_cast<const void*>(kern),                               \
                                            hipFuncAttributeMaxDynamicSharedMemorySize, kMaxFinalLds)))        \
                return FREE_ERR_HIP;                                                                           \
            attr_set = true;                                                                                   \
        }                                                                                                      \
        hipLaunchKernelGGL(kern, dim3(vblocks), dim3(kThreads), stage ? lds_bytes : 0, s, x, shift, scale, M,  \
                           gh, gw, p,                                                                          \
                           c_out, D, static_cast<const WT*>(w), bias, out);                                    \
    } while (0)
        if (dtype == FREE_BF16) {
            if (nv <= 1) FREE_FIN_CASE(bf16_t, 1);
            else if (nv <= 2) FREE_FIN_CASE(bf16_t, 2);
            else if (nv <= 5) FREE_FIN_CASE(bf16_t, 5);
            else FREE_FIN_CASE(bf16_t, 8);
        } else {
            if (nv <= 1) FREE_FIN_CASE(float, 1);
            else if (nv <= 2) FREE_FIN_CASE(float, 2);
            else if (nv <= 5) FREE_FIN_CASE(float, 5);
            else FREE_FIN_CASE(float, 8);
        }
#undef FREE_FIN_CASE
        return launch_ok() ? FREE_OK : FREE_ERR_HIP;
    }
    if (dtype == FREE_BF16)
        hipLaunchKernelGGL(final_layer_kernel<bf16_t>, dim3(blocks), dim3(kThreads), 0, s, x, shift, scale, M, gh,
                           gw, p, c_out, D, static_cast<const bf16_t*>(w), bias, out);
    else
        hipLaunchKernelGGL(final_layer_kernel<float>, dim3(blocks), dim3(kThreads), 0, s, x, shift, scale, M, gh,
                           gw, p, c_out, D, static_cast<const float*>(w), bias, out);
    return launch_ok() ? FREE_OK : FREE_ERR_HIP;
}

// ---- drafter helpers (Sec. 3.2: FC layer on [embedding | propagated feature]; Alg. 1 drafting loop) ----
// fin[m, 0:D] = emb[m, :], fin[m, D:2D] = feat[m, :] in the compute type; 4 elements per thread (D % 4 == 0).
// zero_out (nullable, [M, D], may be feat itself): cleared on the way - the stream the fusion GEMM then
// accumulates into; the thread that clears an element of feat is the one that has just read it.
template <typename OT>
__global__ __launch_bounds__(256) void fuse_pack_kernel(const float* __restrict__ emb, const float* feat, int64_t M,
                                                        int32_t D, OT* __restrict__ fin, float* zero_out) {
    const int64_t q = static_cast<int64_t>(blockIdx.x) * 256 + threadIdx.x;       // group of 4 output elements
    const int32_t per_row = 2 * D / 4;
    if (q >= M * per_row) return;
    const int64_t m = q / per_row;
    const int32_t c = static_cast<int32_t>(q % per_row) * 4;
    const float4 v = c < D ? *reinterpret_cast<const float4*>(emb + m * D + c)
                           : *reinterpret_cast<const float4*>(feat + m * D + (c - D));
    if (zero_out && c >= D) *reinterpret_cast<float4*>(zero_out + m * D + (c - D)) = float4{0.f, 0.f, 0.f, 0.f};
    OT* o = fin + m * 2 * D + c;
    if constexpr (sizeof(OT) == 2) {
        uint2 pk = {pack_bf16_pair(v.x, v.y), pack_bf16_pair(v.z, v.w)};
        *reinterpret_cast<uint2*>(o) = pk;
    } else {
        *reinterpret_cast<float4*>(o) = v;
    }
}

// Range checks of device-resident inputs (opt-in, never on the hot path): bit 0 a timestep outside [0, T),
// bit 1 a sigma that is not positive and finite, bit 2 a uniform outside [0, 1], bit 3 a lambda outside
// [0, 1] (NaN fails every check).  Violations are OR-ed into *flags.
__global__ __launch_bounds__(256) void validate_kernel(const int32_t* __restrict__ t, int64_t n_t, int32_t T,
                                                       const float* __restrict__ sigma, const float* __restrict__ u,
                                                       const float* __restrict__ lambda, int64_t n,
                                                       unsigned int* __restrict__ flags) {
    const int64_t i = static_cast<int64_t>(blockIdx.x) * 256 + threadIdx.x;
    unsigned int bad = 0;
    if (t && i < n_t && (t[i] < 0 || t[i] >= T)) bad |= 1u;
    if (i < n) {
        if (sigma && !(sigma[i] > 0.f && sigma[i] < INFINITY)) bad |= 2u;
        if (u && !(u[i] >= 0.f && u[i] <= 1.f)) bad |= 4u;
        if (lambda && !(lambda[i] >= 0.f && lambda[i] <= 1.f)) bad |= 8u;
    }
    if (bad) atomicOr(flags, bad);
}


// Frozen-target drafting (Sec. 2; used by the self-speculative run of Sec. 3.4): one noise estimate e is
// reused for K steps, m^_k = coef_x[k] x^_k + coef_eps[k] e, x^_{k+1} = m^_k + sigma[k] xi[k]; every latent
// element is an independent recurrence, so one thread walks all K steps of its element.
__global__ __launch_bounds__(256) void frozen_draft_kernel(const float* __restrict__ x_a, const float* __restrict__ e,
                                                           const float* __restrict__ coef_x,
                                                           const float* __restrict__ coef_eps,
                                                           const float* __restrict__ sigma, const float* __restrict__ xi,
                                                           int32_t K, int64_t d, float* __restrict__ x_states,
                                                           float* __restrict__ x_last, float* __restrict__ m_draft) {
    const int64_t i = static_cast<int64_t>(blockIdx.x) * 256 + threadIdx.x;
    if (i >= d) return;
    float x = x_a[i];
    const float ev = e[i];
    for (int k = 0; k < K; ++k) {
        x_states[k * d + i] = x;
        const float m = fmaf(coef_x[k], x, coef_eps[k] * ev);
        m_draft[k * d + i] = m;
        x = fmaf(sigma[k], xi[k * d + i], m);
    }
    x_last[i] = x;
}

// out[k] = || a_k - b_k ||_2^2 over d elements, fp64 accumulation, one workgroup per k (small K, d ~ 1e4..1e5)
__global__ __launch_bounds__(256) void sqdist_kernel(const float* __restrict__ a, const float* __restrict__ b, int64_t d,
                                                     double* __restrict__ out) {
    __shared__ double part[256];
    const int k = blockIdx.x;
    double acc = 0.0;
    for (int64_t i = threadIdx.x; i < d; i += 256) {
        const double v = static_cast<double>(a[k * d + i]) - static_cast<double>(b[k * d + i]);
        acc += v * v;
    }
    part[threadIdx.x] = acc;
    __syncthreads();
    for (int s = 128; s > 0; s >>= 1) {
        if (threadIdx.x < s) part[threadIdx.x] += part[threadIdx.x + s];
        __syncthreads();
    }
    if (threadIdx.x == 0) out[k] = part[0];
}

int32_t launch_eps_to_mean(const float* eps_out, const float* x_states, const float* coef_x,
                           const float* coef_eps, float cfg_scale, int32_t K, int32_t C, int32_t c_out,
                           int64_t hw, float* m_out, hipStream_t s, float* eps_guided, const float* sigma_step,
                           const float* xi, float* x_next) {
    const int64_t n = static_cast<int64_t>(K) * C * hw;
    const int use_cfg = cfg_scale > 1.0f ? 1 : 0;
    if (x_next && (!sigma_step || !xi)) return FREE_ERR_NULL;
    hipLaunchKernelGGL(eps_to_mean_kernel, dim3(static_cast<unsigned>((n + 255) / 256)), dim3(256), 0, s, eps_out,
                       x_states, coef_x, coef_eps, cfg_scale, use_cfg, K, C, c_out, hw, m_out, eps_guided, sigma_step,
                       xi, x_next);
    return launch_ok() ? FREE_OK : FREE_ERR_HIP;
}

int32_t launch_pack_cond(const int32_t* t, int32_t y, int32_t null_label, int32_t K, int32_t dup,
                         int32_t* t_out, int32_t* y_out, hipStream_t s) {
    const int n = K * dup;
    hipLaunchKernelGGL(pack_cond_kernel, dim3((n + 63) / 64), dim3(64), 0, s, t, y, null_label, K, dup, t_out,
                       y_out);
    return launch_ok() ? FREE_OK : FREE_ERR_HIP;
}

int32_t launch_fuse_pack(const float* emb, const float* feat, int64_t M, int32_t D, int32_t dtype, void* fin,
                         float* zero_out, hipStream_t s) {
    if (D % 4) return FREE_ERR_SHAPE;
    const int64_t groups = M * (2 * D / 4);
    const unsigned blocks = static_cast<unsigned>((groups + 255) / 256);
    if (dtype == FREE_BF16)
        hipLaunchKernelGGL(fuse_pack_kernel<bf16_t>, dim3(blocks), dim3(256), 0, s, emb, feat, M, D,
                           static_cast<bf16_t*>(fin), zero_out);
    else
        hipLaunchKernelGGL(fuse_pack_kernel<float>, dim3(blocks), dim3(256), 0, s, emb, feat, M, D,
                           static_cast<float*>(fin), zero_out);
    return launch_ok() ? FREE_OK : FREE_ERR_HIP;
}

int32_t run_validate(const int32_t* t, int64_t n_t, int32_t T, const float* sigma, const float* u,
                     const float* lambda, int64_t n, uint32_t* violations, hipStream_t s) {
    unsigned int* flags = nullptr;
    if (!hip_ok(hipMalloc(&flags, sizeof(unsigned int)))) return FREE_ERR_HIP;
    unsigned int host = 0;
    int32_t rc = FREE_ERR_HIP;
    do {
        if (!hip_ok(hipMemcpyAsync(flags, &host, sizeof(host), hipMemcpyHostToDevice, s))) break;
        const int64_t most = n_t > n ? n_t : n;
        if (most > 0) {
            hipLaunchKernelGGL(validate_kernel, dim3(static_cast<unsigned>((most + 255) / 256)), dim3(256), 0, s, t, n_t,
                               T, sigma, u, lambda, n, flags);
            if (!launch_ok()) break;
        }
        if (!hip_ok(hipMemcpyAsync(&host, flags, sizeof(host), hipMemcpyDeviceToHost, s))) break;
        if (!hip_ok(hipStreamSynchronize(s))) break;
        rc = FREE_OK;
    } while (false);
    (void)hipFree(flags);
    if (rc != FREE_OK) return rc;
    if (violations) *violations = host;
    return host ? FREE_ERR_RANGE : FREE_OK;
}

int32_t launch_frozen_draft(const float* x_a, const float* e, const float* coef_x, const float* coef_eps,
                            const float* sigma, const float* xi, int32_t K, int64_t d, float* x_states, float* x_last,
                            float* m_draft, hipStream_t s) {
    hipLaunchKernelGGL(frozen_draft_kernel, dim3(static_cast<unsigned>((d + 255) / 256)), dim3(256), 0, s, x_a, e, coef_x,
                       coef_eps, sigma, xi, K, d, x_states, x_last, m_draft);
    return launch_ok() ? FREE_OK : FREE_ERR_HIP;
}

int32_t launch_sqdist(const float* a, const float* b, int32_t K, int64_t d, double* out, hipStream_t s) {
    hipLaunchKernelGGL(sqdist_kernel, dim3(K), dim3(256), 0, s, a, b, d, out);
    return launch_ok() ? FREE_OK : FREE_ERR_HIP;
}

}  // namespace freemi
