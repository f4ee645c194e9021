// Verification of the K drafts of each trajectory (Alg. 2, Eq. qp, Eq. acc_relax,
// verification loop of Alg. 1).  HBM-bound: one streaming pass over
// (m, m^, x^) per (trajectory, draft) pair, 12 bytes and ~8 flops per element.
//
// Two launches:
//   1. verify_partial_kernel: grid (splits, pairs).  Each workgroup streams one
//      chunk of one pair with 16-byte loads and reduces the two sums
//        s2 = sum (m^ - m)^2,   s3 = sum (m^ - m)(x^ - m^)
//      in fp64 (fixed tree: lane -> wavefront shuffle -> LDS), then writes one
//      (s2, s3) partial.  The log-ratio of Eq. (qp) is l = -(s3 + s2/2)/sigma^2.
//   2. verify_finish_kernel: grid (rchunks, n_traj).  Every workgroup of a
//      trajectory re-adds that trajectory's partials in the same fixed order,
//      takes the K decisions, finds the first rejection, and (if there is one)
//      writes its chunk of the reflected sample
//        x = m + (x^ - m^) - 2 (s3/s2)(m^ - m)        (Alg. 2, rejection branch).
#include "free_internal.h"

namespace freemi {

namespace {

typedef float f32x4 __attribute__((ext_vector_type(4)));

constexpr int kThreads = 256;
constexpr int kChunkQuantum = 1024;       // elements; chunk sizes are multiples of this
constexpr int kTargetBlocks = 1536;       // ~6 workgroups per CU on 256 CUs, 12 loads of 16 bytes in flight per lane
constexpr int kReflectChunk = 1024;       // elements of x_out per workgroup in launch 2 (one float4 per lane)

struct Plan {
    int64_t chunk;      // elements per workgroup in launch 1
    int32_t splits;     // workgroups per pair
};

Plan make_plan(int32_t n_traj, int32_t K, int64_t d) {
    int64_t pairs = static_cast<int64_t>(n_traj) * K;
    int64_t max_splits = (d + kChunkQuantum - 1) / kChunkQuantum;
    int64_t want = (kTargetBlocks + pairs - 1) / pairs;
    if (want < 1) want = 1;
    if (want > max_splits) want = max_splits;
    int64_t chunk = (d + want - 1) / want;
    chunk = (chunk + kChunkQuantum - 1) / kChunkQuantum * kChunkQuantum;
    Plan p;
    p.chunk = chunk;
    p.splits = static_cast<int32_t>((d + chunk - 1) / chunk);
    if (p.splits < 1) p.splits = 1;
    return p;
}

__device__ inline const float* draft_ptr(const float* x_draft, const float* x_last, int64_t pair,
                                         int32_t K, int64_t d) {
    if (x_last != nullptr) {                     // single trajectory, drafts = shifted states
        int32_t k = static_cast<int32_t>(pair);
        return (k < K - 1) ? x_draft + static_cast<int64_t>(k + 1) * d : x_last;
    }
    return x_draft + pair * d;
}

__device__ inline double wave_sum(double v) {
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off, 64);
    return v;
}

__device__ inline void accum(double& s2, double& s3, float m, float mh, float xh) {
    double dm = static_cast<double>(mh) - static_cast<double>(m);
    double r = static_cast<double>(xh) - static_cast<double>(mh);
    s2 = fma(dm, dm, s2);
    s3 = fma(dm, r, s3);
}

template <bool VEC>
__global__ __launch_bounds__(kThreads) void verify_partial_kernel(
    const float* __restrict__ m_target, const float* __restrict__ m_draft,
    const float* __restrict__ x_draft, const float* __restrict__ x_last, int32_t K, int64_t d,
    int64_t chunk, double* __restrict__ partial) {
    const int64_t pair = blockIdx.y;
    const int32_t split = blockIdx.x;
    const float* m = m_target + pair * d;
    const float* mh = m_draft + pair * d;
    const float* xh = draft_ptr(x_draft, x_last, pair, K, d);
    const int64_t lo = static_cast<int64_t>(split) * chunk;
    int64_t hi = lo + chunk;
    if (hi > d) hi = d;

    double s2 = 0.0, s3 = 0.0;
    if (VEC) {
        // d % 4 == 0 and 16-byte aligned bases: whole float4 groups only
        const f32x4* m4 = reinterpret_cast<const f32x4*>(m);
        const f32x4* mh4 = reinterpret_cast<const f32x4*>(mh);
        const f32x4* xh4 = reinterpret_cast<const f32x4*>(xh);
        const int64_t lo4 = lo >> 2, hi4 = hi >> 2;
        int64_t i = lo4 + threadIdx.x;
        // 4 independent 16-byte loads per array in flight per lane
        for (; i + 3 * kThreads < hi4; i += 4 * kThreads) {
            f32x4 a[4], b[4], c[4];
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                a[j] = m4[i + j * kThreads];
                b[j] = mh4[i + j * kThreads];
                c[j] = xh4[i + j * kThreads];
            }
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                accum(s2, s3, a[j].x, b[j].x, c[j].x);
                accum(s2, s3, a[j].y, b[j].y, c[j].y);
                accum(s2, s3, a[j].z, b[j].z, c[j].z);
                accum(s2, s3, a[j].w, b[j].w, c[j].w);
            }
        }
        for (; i < hi4; i += kThreads) {
            f32x4 a = m4[i], b = mh4[i], c = xh4[i];
            accum(s2, s3, a.x, b.x, c.x);
            accum(s2, s3, a.y, b.y, c.y);
            accum(s2, s3, a.z, b.z, c.z);
            accum(s2, s3, a.w, b.w, c.w);
        }
    } else {
        for (int64_t i = lo + threadIdx.x; i < hi; i += kThreads) accum(s2, s3, m[i], mh[i], xh[i]);
    }

    s2 = wave_sum(s2);
    s3 = wave_sum(s3);
    __shared__ double red[2][kThreads / 64];
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    if (lane == 0) { red[0][wave] = s2; red[1][wave] = s3; }
    __syncthreads();
    if (threadIdx.x == 0) {
        double t2 = 0.0, t3 = 0.0;
#pragma unroll
        for (int w = 0; w < kThreads / 64; ++w) { t2 += red[0][w]; t3 += red[1][w]; }
        double* out = partial + (pair * gridDim.x + split) * 2;
        out[0] = t2;
        out[1] = t3;
    }
}

__global__ __launch_bounds__(kThreads) void verify_finish_kernel(
    const float* __restrict__ m_target, const float* __restrict__ m_draft,
    const float* __restrict__ x_draft, const float* __restrict__ x_last,
    const float* __restrict__ sigma, const float* __restrict__ u, const float* __restrict__ lambda,
    int32_t K, int64_t d, int32_t splits, const double* __restrict__ partial,
    float* __restrict__ log_ratio, uint8_t* __restrict__ accept, int32_t* __restrict__ n_accept,
    float* __restrict__ x_out) {
    const int64_t traj = blockIdx.y;
    __shared__ double sh_s2[FREE_MAX_DRAFTS];
    __shared__ double sh_s3[FREE_MAX_DRAFTS];
    __shared__ uint8_t sh_acc[FREE_MAX_DRAFTS];
    __shared__ int32_t sh_first;

    for (int k = threadIdx.x; k < K; k += kThreads) {
        const int64_t pair = traj * K + k;
        const double* p = partial + pair * splits * 2;
        double s2 = 0.0, s3 = 0.0;
        for (int s = 0; s < splits; ++s) { s2 += p[2 * s]; s3 += p[2 * s + 1]; }
        const double sg = static_cast<double>(sigma[pair]);
        const double l = -(s3 + 0.5 * s2) / (sg * sg);          // Eq. (qp)
        const double lam = lambda ? static_cast<double>(lambda[pair]) : 1.0;
        const double thr = fmin(0.0, lam * l);                  // Eq. (acc_relax) in the log domain
        const float uu = u[pair];
        bool ok = (s2 == 0.0) || (uu <= 0.0f) || (log(static_cast<double>(uu)) <= thr);
        sh_s2[k] = s2;
        sh_s3[k] = s3;
        sh_acc[k] = ok ? 1 : 0;
        if (blockIdx.x == 0) {
            log_ratio[pair] = static_cast<float>(l);
            accept[pair] = ok ? 1 : 0;
        }
    }
    __syncthreads();
    if (threadIdx.x == 0) {
        int32_t first = K;
        for (int k = 0; k < K; ++k) {
            if (!sh_acc[k]) { first = k; break; }
        }
        sh_first = first;
        if (blockIdx.x == 0) n_accept[traj] = first;
    }
    __syncthreads();
    const int32_t k = sh_first;
    if (k >= K) return;                                          // nothing rejected: x_out untouched

    const double c = 2.0 * sh_s3[k] / sh_s2[k];                  // 2 e^T(x^ - m^) / ||m^ - m||
    const int64_t pair = traj * K + k;
    const float* m = m_target + pair * d;
    const float* mh = m_draft + pair * d;
    const float* xh = draft_ptr(x_draft, x_last, pair, K, d);
    float* xo = x_out + traj * d;
    const int64_t lo = static_cast<int64_t>(blockIdx.x) * kReflectChunk;
    int64_t hi = lo + kReflectChunk;
    if (hi > d) hi = d;
    const bool vec = ((d & 3) == 0) && ((reinterpret_cast<uintptr_t>(m) | reinterpret_cast<uintptr_t>(mh) |
                                         reinterpret_cast<uintptr_t>(xh) | reinterpret_cast<uintptr_t>(xo)) & 15u) == 0;
    if (vec) {
        for (int64_t i = lo + 4 * threadIdx.x; i < hi; i += 4 * kThreads) {
            const f32x4 a = *reinterpret_cast<const f32x4*>(m + i), b = *reinterpret_cast<const f32x4*>(mh + i),
                        x = *reinterpret_cast<const f32x4*>(xh + i);
            f32x4 o;
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const double mm = a[j], mmh = b[j], xx = x[j];
                o[j] = static_cast<float>(mm + (xx - mmh) - c * (mmh - mm));
            }
            *reinterpret_cast<f32x4*>(xo + i) = o;
        }
        return;
    }
    for (int64_t i = lo + threadIdx.x; i < hi; i += kThreads) {
        const double mm = m[i], mmh = mh[i], xx = xh[i];
        xo[i] = static_cast<float>(mm + (xx - mmh) - c * (mmh - mm));
    }
}

inline bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

}  // namespace

size_t verify_workspace_bytes(int32_t n_traj, int32_t K, int64_t d) {
    if (n_traj < 1 || K < 1 || d < 1) return 0;
    Plan p = make_plan(n_traj, K, d);
    size_t bytes = static_cast<size_t>(n_traj) * K * p.splits * 2 * sizeof(double);
    return (bytes + 255) / 256 * 256;
}

int32_t launch_verify(const VerifyArgs& a, void* ws, size_t ws_bytes, hipStream_t s) {
    const size_t need = verify_workspace_bytes(a.n_traj, a.K, a.d);
    if (ws == nullptr || ws_bytes < need || (reinterpret_cast<uintptr_t>(ws) & 7u)) return FREE_ERR_WORKSPACE;
    const Plan p = make_plan(a.n_traj, a.K, a.d);
    const int64_t pairs = static_cast<int64_t>(a.n_traj) * a.K;
    if (pairs > 65535 || a.n_traj > 65535) return FREE_ERR_SHAPE;    // grid.y limit
    double* partial = static_cast<double*>(ws);
    const bool vec = (a.d % 4 == 0) && aligned16(a.m_target) && aligned16(a.m_draft) &&
                     aligned16(a.x_draft) && (a.x_last == nullptr || aligned16(a.x_last));
    dim3 g1(p.splits, static_cast<unsigned>(pairs));
    {
    ProfScope prof(PROF_VERIFY_PARTIAL, s);
    if (vec) {
        hipLaunchKernelGGL(verify_partial_kernel<true>, g1, dim3(kThreads), 0, s, a.m_target, a.m_draft,
                           a.x_draft, a.x_last, a.K, a.d, p.chunk, partial);
    } else {
        hipLaunchKernelGGL(verify_partial_kernel<false>, g1, dim3(kThreads), 0, s, a.m_target, a.m_draft,
                           a.x_draft, a.x_last, a.K, a.d, p.chunk, partial);
    }
    }
    if (!launch_ok()) return FREE_ERR_HIP;
    ProfScope prof(PROF_VERIFY_FINISH, s);
    const unsigned rchunks = static_cast<unsigned>((a.d + kReflectChunk - 1) / kReflectChunk);
    hipLaunchKernelGGL(verify_finish_kernel, dim3(rchunks, a.n_traj), dim3(kThreads), 0, s, a.m_target,
                       a.m_draft, a.x_draft, a.x_last, a.sigma, a.u, a.lambda, a.K, a.d, p.splits, partial,
                       a.log_ratio, a.accept, a.n_accept, a.x_out);
    if (!launch_ok()) return FREE_ERR_HIP;
    return FREE_OK;
}

}  // namespace freemi
