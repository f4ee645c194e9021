// Verification of the K drafts of each trajectory (Alg. 2, Eq. qp, Eq. acc_relax,
// verification loop of Alg. 1).  HBM-bound: one streaming pass over
// (m, m^, x^) per (trajectory, draft) pair, 12 bytes and ~8 flops per element.
//
// ONE launch, verify_fused_kernel, a one-dimensional grid of pairs x splits workgroups
// ordered trajectory-major (all chunks of trajectory 0 first):
//   1. every workgroup streams one chunk of one pair with 16-byte loads and reduces
//        s2 = sum (m^ - m)^2,   s3 = sum (m^ - m)(x^ - m^)
//      in fp64 (fixed tree: lane -> wavefront shuffle -> LDS) and writes one (s2, s3)
//      partial to the workspace.  The log-ratio of Eq. (qp) is l = -(s3 + s2/2)/sigma^2.
//   2. it then takes a ticket from the trajectory's arrival counter (a device-scope
//      vector atomic in the workspace, bracketed by device-scope fences).  The workgroup
//      that draws the last ticket of a trajectory - all partials of the trajectory are
//      then visible to it - re-adds them in a fixed order, takes the K decisions, finds
//      the first rejection, writes log_ratio / accept / n_accept and, if a draft was
//      rejected, the reflected sample
//        x = m + (x^ - m^) - 2 (s3/s2)(m^ - m)        (Alg. 2, rejection branch),
//      whose inputs were streamed moments ago and are still in the memory-side cache.
//      It finally puts the counter back to zero.  No workgroup ever waits for another.
// Because trajectories finish one after the other, only the last one's finishing step
// is not overlapped with the streaming of the others.
// The counters must be zero when the kernel starts: launch_verify clears them with a
// small fill kernel unless the caller says a kernel before it on the stream has done so.
#include "free_internal.h"

namespace freemi {

namespace {

typedef float f32x4 __attribute__((ext_vector_type(4)));

constexpr int kThreads = 256;
constexpr int kChunkQuantum = 1024;       // elements; chunk sizes are multiples of this
constexpr int kTargetBlocks = 1536;       // ~6 workgroups per CU on 256 CUs, 12 loads of 16 bytes in flight per lane
constexpr int kCounterAlign = 256;        // bytes; the partial sums follow the counters
constexpr int64_t kFusedReflectMax = 1 << 18;   // elements per state up to which the finishing workgroup reflects by itself
constexpr int kReflectChunk = 4096;       // elements of x_out per workgroup of the separate reflection launch

struct Plan {
    int64_t chunk;      // elements per workgroup
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

size_t counter_bytes(int32_t n_traj) {
    return (static_cast<size_t>(n_traj) * sizeof(uint32_t) + kCounterAlign - 1) / kCounterAlign * kCounterAlign;
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

__global__ void clear_u32_kernel(uint32_t* __restrict__ p, int32_t n) {
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) p[i] = 0u;
}

template <bool VEC>
__global__ __launch_bounds__(kThreads) void verify_fused_kernel(
    const float* __restrict__ m_target, const float* __restrict__ m_draft,
    const float* __restrict__ x_draft, const float* __restrict__ x_last,
    const float* __restrict__ sigma, const float* __restrict__ u, const float* __restrict__ lambda,
    int32_t K, int64_t d, int64_t chunk, int32_t splits, int32_t reflect_here, uint32_t* counters, double* partial,
    float* __restrict__ log_ratio, uint8_t* __restrict__ accept, int32_t* __restrict__ n_accept,
    float* __restrict__ x_out) {
    const int64_t pair = blockIdx.x / splits;
    const int32_t split = blockIdx.x % splits;
    const int64_t traj = pair / K;
    {
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
        __shared__ int32_t sh_last;
        const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
        if (lane == 0) { red[0][wave] = s2; red[1][wave] = s3; }
        __syncthreads();
        if (threadIdx.x == 0) {
            double t2 = 0.0, t3 = 0.0;
#pragma unroll
            for (int w = 0; w < kThreads / 64; ++w) { t2 += red[0][w]; t3 += red[1][w]; }
            double* out = partial + (pair * splits + split) * 2;
            __hip_atomic_store(out, t2, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            __hip_atomic_store(out + 1, t3, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            __threadfence();                                     // the partial is visible device-wide before the ticket
            const uint32_t ticket = atomicAdd(counters + traj, 1u);
            sh_last = ticket == static_cast<uint32_t>(K) * static_cast<uint32_t>(splits) - 1u;
        }
        __syncthreads();
        if (!sh_last) return;
        __threadfence();                                         // every partial of the trajectory is visible from here on
    }

    // ---- the workgroup that completed the trajectory: decisions, first rejection, reflection
    __shared__ double sh_s2[FREE_MAX_DRAFTS];
    __shared__ double sh_s3[FREE_MAX_DRAFTS];
    __shared__ uint8_t sh_acc[FREE_MAX_DRAFTS];
    __shared__ int32_t sh_first;
    for (int k = threadIdx.x; k < K; k += kThreads) {
        const int64_t pr = traj * K + k;
        double* p = partial + pr * splits * 2;
        double s2 = 0.0, s3 = 0.0;
        for (int s = 0; s < splits; ++s) {
            s2 += __hip_atomic_load(p + 2 * s, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            s3 += __hip_atomic_load(p + 2 * s + 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
        const double sg = static_cast<double>(sigma[pr]);
        const double l = -(s3 + 0.5 * s2) / (sg * sg);          // Eq. (qp)
        const double lam = lambda ? static_cast<double>(lambda[pr]) : 1.0;
        const double thr = fmin(0.0, lam * l);                  // Eq. (acc_relax) in the log domain
        const float uu = u[pr];
        const bool ok = (s2 == 0.0) || (uu <= 0.0f) || (log(static_cast<double>(uu)) <= thr);
        sh_s2[k] = s2;
        sh_s3[k] = s3;
        sh_acc[k] = ok ? 1 : 0;
        log_ratio[pr] = static_cast<float>(l);
        accept[pr] = ok ? 1 : 0;
    }
    __syncthreads();
    if (threadIdx.x == 0) {
        int32_t first = K;
        for (int k = 0; k < K; ++k) {
            if (!sh_acc[k]) { first = k; break; }
        }
        sh_first = first;
        n_accept[traj] = first;
        counters[traj] = 0u;                                     // ready for the next call on this workspace
    }
    __syncthreads();
    const int32_t k = sh_first;
    if (k >= K || !reflect_here) return;                         // nothing rejected: x_out untouched

    const double c = 2.0 * sh_s3[k] / sh_s2[k];                  // 2 e^T(x^ - m^) / ||m^ - m||
    const int64_t pr = traj * K + k;
    const float* m = m_target + pr * d;
    const float* mh = m_draft + pr * d;
    const float* xh = draft_ptr(x_draft, x_last, pr, K, d);
    float* xo = x_out + traj * d;
    const bool vec = ((d & 3) == 0) && ((reinterpret_cast<uintptr_t>(m) | reinterpret_cast<uintptr_t>(mh) |
                                         reinterpret_cast<uintptr_t>(xh) | reinterpret_cast<uintptr_t>(xo)) & 15u) == 0;
    if (vec) {
        const f32x4* m4 = reinterpret_cast<const f32x4*>(m);
        const f32x4* mh4 = reinterpret_cast<const f32x4*>(mh);
        const f32x4* xh4 = reinterpret_cast<const f32x4*>(xh);
        f32x4* xo4 = reinterpret_cast<f32x4*>(xo);
        const int64_t n4 = d >> 2;
        auto reflect4 = [&](const f32x4& a, const f32x4& b, const f32x4& x) {
            f32x4 o;
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const double mm = a[j], mmh = b[j], xx = x[j];
                o[j] = static_cast<float>(mm + (xx - mmh) - c * (mmh - mm));
            }
            return o;
        };
        int64_t i = threadIdx.x;
        for (; i + 3 * kThreads < n4; i += 4 * kThreads) {
            f32x4 a[4], b[4], x[4];
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                a[j] = m4[i + j * kThreads];
                b[j] = mh4[i + j * kThreads];
                x[j] = xh4[i + j * kThreads];
            }
#pragma unroll
            for (int j = 0; j < 4; ++j) xo4[i + j * kThreads] = reflect4(a[j], b[j], x[j]);
        }
        for (; i < n4; i += kThreads) xo4[i] = reflect4(m4[i], mh4[i], xh4[i]);
        return;
    }
    for (int64_t i = threadIdx.x; i < d; i += kThreads) {
        const double mm = m[i], mmh = mh[i], xx = xh[i];
        xo[i] = static_cast<float>(mm + (xx - mmh) - c * (mmh - mm));
    }
}

// States too long for one workgroup to reflect: a second launch, grid (chunks, n_traj).  Every workgroup re-adds
// the partial sums of its trajectory's first rejected draft in the same fixed order as the fused kernel.
__global__ __launch_bounds__(kThreads) void verify_reflect_kernel(
    const float* __restrict__ m_target, const float* __restrict__ m_draft, const float* __restrict__ x_draft,
    const float* __restrict__ x_last, int32_t K, int64_t d, int32_t splits, const double* __restrict__ partial,
    const int32_t* __restrict__ n_accept, float* __restrict__ x_out) {
    const int64_t traj = blockIdx.y;
    const int32_t k = n_accept[traj];
    if (k >= K) return;
    const int64_t pr = traj * K + k;
    const double* p = partial + pr * splits * 2;
    double s2 = 0.0, s3 = 0.0;
    for (int s = 0; s < splits; ++s) { s2 += p[2 * s]; s3 += p[2 * s + 1]; }
    const double c = 2.0 * s3 / s2;
    const float* m = m_target + pr * d;
    const float* mh = m_draft + pr * d;
    const float* xh = draft_ptr(x_draft, x_last, pr, K, d);
    float* xo = x_out + traj * d;
    const int64_t lo = static_cast<int64_t>(blockIdx.x) * kReflectChunk;
    int64_t hi = lo + kReflectChunk;
    if (hi > d) hi = d;
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
    size_t bytes = counter_bytes(n_traj) + static_cast<size_t>(n_traj) * K * p.splits * 2 * sizeof(double);
    return (bytes + 255) / 256 * 256;
}

uint32_t* verify_counters(void* ws) { return static_cast<uint32_t*>(ws); }

int32_t launch_verify(const VerifyArgs& a, void* ws, size_t ws_bytes, bool counters_are_zero, hipStream_t s) {
    const size_t need = verify_workspace_bytes(a.n_traj, a.K, a.d);
    if (ws == nullptr || ws_bytes < need || (reinterpret_cast<uintptr_t>(ws) & 7u)) return FREE_ERR_WORKSPACE;
    const Plan p = make_plan(a.n_traj, a.K, a.d);
    const int64_t blocks = static_cast<int64_t>(a.n_traj) * a.K * p.splits;
    if (blocks > 0x7fffffffll) return FREE_ERR_SHAPE;             // one-dimensional grid
    uint32_t* counters = verify_counters(ws);
    double* partial = reinterpret_cast<double*>(static_cast<char*>(ws) + counter_bytes(a.n_traj));
    if (!counters_are_zero) {
        hipLaunchKernelGGL(clear_u32_kernel, dim3((a.n_traj + 255) / 256), dim3(256), 0, s, counters, a.n_traj);
        if (!launch_ok()) return FREE_ERR_HIP;
    }
    const bool vec = (a.d % 4 == 0) && aligned16(a.m_target) && aligned16(a.m_draft) &&
                     aligned16(a.x_draft) && (a.x_last == nullptr || aligned16(a.x_last));
    const int32_t reflect_here = a.d <= kFusedReflectMax ? 1 : 0;
    if (!reflect_here && a.n_traj > 65535) return FREE_ERR_SHAPE;  // second grid dimension of the reflection launch
    ProfScope prof(a.prof, PROF_VERIFY, s);
    const dim3 grid(static_cast<unsigned>(blocks));
    if (vec) {
        hipLaunchKernelGGL(verify_fused_kernel<true>, grid, dim3(kThreads), 0, s, a.m_target, a.m_draft, a.x_draft,
                           a.x_last, a.sigma, a.u, a.lambda, a.K, a.d, p.chunk, p.splits, reflect_here, counters, partial,
                           a.log_ratio, a.accept, a.n_accept, a.x_out);
    } else {
        hipLaunchKernelGGL(verify_fused_kernel<false>, grid, dim3(kThreads), 0, s, a.m_target, a.m_draft, a.x_draft,
                           a.x_last, a.sigma, a.u, a.lambda, a.K, a.d, p.chunk, p.splits, reflect_here, counters, partial,
                           a.log_ratio, a.accept, a.n_accept, a.x_out);
    }
    if (!launch_ok()) return FREE_ERR_HIP;
    if (!reflect_here) {
        const unsigned rchunks = static_cast<unsigned>((a.d + kReflectChunk - 1) / kReflectChunk);
        hipLaunchKernelGGL(verify_reflect_kernel, dim3(rchunks, a.n_traj), dim3(kThreads), 0, s, a.m_target, a.m_draft,
                           a.x_draft, a.x_last, a.K, a.d, p.splits, partial, a.n_accept, a.x_out);
        if (!launch_ok()) return FREE_ERR_HIP;
    }
    return FREE_OK;
}

}  // namespace freemi
