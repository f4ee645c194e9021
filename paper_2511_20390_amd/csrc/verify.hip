// Verification of the K drafts of each trajectory (Alg. 2, Eq. qp, Eq. acc_relax,
// verification loop of Alg. 1).  HBM-bound: one streaming pass over
// (m, m^, x^) per (trajectory, draft) pair, 12 bytes and ~8 flops per element.
//
// Two launches:
//   1. verify_partial_kernel: a one-dimensional grid of pairs x splits workgroups.  Each
//      workgroup streams one chunk of one pair with 16-byte loads, all of a lane's loads
//      in flight at once, and reduces the two sums
//        s2 = sum (m^ - m)^2,   s3 = sum (m^ - m)(x^ - m^)
//      in fp64 (fixed tree: lane -> wavefront shuffle -> LDS), then writes one (s2, s3)
//      partial.  The log-ratio of Eq. (qp) is l = -(s3 + s2/2)/sigma^2.
//   2. verify_finish_kernel: grid (rchunks, n_traj), 4096 elements of a state per
//      workgroup.  Every wavefront re-adds its trajectory's partials in the same fixed
//      order (lane k takes draft k: no barrier, no LDS), takes the K decisions, finds the
//      first rejection by a wavefront ballot and, if there is one, writes its part of the
//      reflected sample
//        x = m + (x^ - m^) - 2 (s3/s2)(m^ - m)        (Alg. 2, rejection branch)
//      with the twelve 16-byte loads of a lane in flight together; the inputs were
//      streamed by launch 1 moments ago and are still in the memory-side cache.
// A single launch in which the workgroup that completes a trajectory (arrival counter,
// device-scope atomics) finishes it was built and measured: the store -> atomic ->
// load chain every workgroup then ends with, and the reflection of a whole state by one
// workgroup, cost 11-20 us against the 2 us of a kernel boundary (31-40 us per call
// instead of 20), and device-scope fences (one cache write-back and invalidation per
// workgroup) made it 139 us.  Not kept.
#include <hip/hip_ext.h>

#include <mutex>

#include "free_internal.h"

// Scratch memory of spec_verify_static, the entry point for callers that cannot allocate: the partial sums of
// the streaming launch.  One copy per GPU the library runs on, held until the process ends.  In host code
// the name below is only a handle for hipGetSymbolAddress, never a device address.
static __device__ __align__(256) unsigned char scratch[FREE_STATIC_SCRATCH_BYTES];

namespace freemi {

namespace {

typedef float f32x4 __attribute__((ext_vector_type(4)));

constexpr int kTargetThreads = 1536 * 256;   // threads of launch 1: 24 wavefronts per CU on 256 CUs
constexpr int kFinishThreads = 256;
constexpr int kReflectChunk = 16 * kFinishThreads;   // elements of x_out per workgroup in launch 2 (4 float4 per lane)

struct Plan {
    int64_t chunk;      // elements per workgroup in launch 1
    int32_t splits;     // workgroups per pair
};

// threads: workgroup size; depth: float4 per lane and array.  Chunk sizes are multiples of one float4 per lane.
Plan make_plan(int32_t n_traj, int32_t K, int64_t d, int threads, int depth) {
    const int64_t quantum = 4 * threads;
    const int64_t target_blocks = static_cast<int64_t>(kTargetThreads) * 4 / (static_cast<int64_t>(threads) * depth);
    int64_t pairs = static_cast<int64_t>(n_traj) * K;
    int64_t max_splits = (d + quantum - 1) / quantum;
    int64_t want = (target_blocks + pairs - 1) / pairs;
    if (want < 1) want = 1;
    if (want > max_splits) want = max_splits;
    int64_t chunk = (d + want - 1) / want;
    chunk = (chunk + quantum - 1) / quantum * quantum;
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

// per-element variance: both factors divided by the element's standard deviation (whitened coordinates)
__device__ inline void accum_w(double& s2, double& s3, float m, float mh, float xh, float sg) {
    const double inv = 1.0 / static_cast<double>(sg);
    const double dm = (static_cast<double>(mh) - static_cast<double>(m)) * inv;
    const double r = (static_cast<double>(xh) - static_cast<double>(mh)) * inv;
    s2 = fma(dm, dm, s2);
    s3 = fma(dm, r, s3);
}

template <bool NT>
__device__ inline f32x4 stream_load(const f32x4* p) {
    if (NT) return __builtin_nontemporal_load(p);
    return *p;
}

// kThreads lanes; DEPTH float4 per lane and array in flight; VEC: d % 4 == 0 and 16-byte aligned bases;
// NT: loads marked non-temporal (the inputs are read once by this launch); DIAG: sigma_elem [pairs, d] holds
// one standard deviation per element and the sums are taken in whitened coordinates
template <int kThreads, int DEPTH, bool VEC, bool NT, bool DIAG>
__global__ __launch_bounds__(kThreads) void verify_partial_kernel(
    const float* __restrict__ m_target, const float* __restrict__ m_draft,
    const float* __restrict__ x_draft, const float* __restrict__ x_last, const float* __restrict__ sigma_elem,
    int32_t K, int64_t d, int64_t chunk, int32_t splits, double* __restrict__ partial) {
    const int64_t pair = blockIdx.x / splits;
    const int32_t split = blockIdx.x % splits;
    const float* m = m_target + pair * d;
    const float* mh = m_draft + pair * d;
    const float* xh = draft_ptr(x_draft, x_last, pair, K, d);
    const float* sg = DIAG ? sigma_elem + pair * d : nullptr;
    const int64_t lo = static_cast<int64_t>(split) * chunk;
    int64_t hi = lo + chunk;
    if (hi > d) hi = d;

    double s2 = 0.0, s3 = 0.0;
    auto add4 = [&](const f32x4& a, const f32x4& b, const f32x4& c, const f32x4& w) {
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            if (DIAG) accum_w(s2, s3, a[e], b[e], c[e], w[e]);
            else accum(s2, s3, a[e], b[e], c[e]);
        }
    };
    if (VEC) {
        const f32x4* m4 = reinterpret_cast<const f32x4*>(m);
        const f32x4* mh4 = reinterpret_cast<const f32x4*>(mh);
        const f32x4* xh4 = reinterpret_cast<const f32x4*>(xh);
        const f32x4* sg4 = reinterpret_cast<const f32x4*>(sg);
        const int64_t lo4 = lo >> 2, hi4 = hi >> 2;
        int64_t i = lo4 + threadIdx.x;
        for (; i + (DEPTH - 1) * kThreads < hi4; i += DEPTH * kThreads) {
            f32x4 a[DEPTH], b[DEPTH], c[DEPTH], w[DEPTH];
#pragma unroll
            for (int j = 0; j < DEPTH; ++j) {
                a[j] = stream_load<NT>(m4 + i + j * kThreads);
                b[j] = stream_load<NT>(mh4 + i + j * kThreads);
                c[j] = stream_load<NT>(xh4 + i + j * kThreads);
                if (DIAG) w[j] = stream_load<NT>(sg4 + i + j * kThreads);
            }
#pragma unroll
            for (int j = 0; j < DEPTH; ++j) add4(a[j], b[j], c[j], w[j]);
        }
        for (; i < hi4; i += kThreads) {
            const f32x4 w = DIAG ? sg4[i] : f32x4{1.f, 1.f, 1.f, 1.f};
            add4(m4[i], mh4[i], xh4[i], w);
        }
    } else {
        for (int64_t i = lo + threadIdx.x; i < hi; i += kThreads) {
            if (DIAG) accum_w(s2, s3, m[i], mh[i], xh[i], sg[i]);
            else accum(s2, s3, m[i], mh[i], xh[i]);
        }
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
        double* out = partial + (pair * splits + split) * 2;
        out[0] = t2;
        out[1] = t3;
    }
}

__global__ __launch_bounds__(kFinishThreads) void verify_finish_kernel(
    const float* __restrict__ m_target, const float* __restrict__ m_draft,
    const float* __restrict__ x_draft, const float* __restrict__ x_last,
    const float* __restrict__ sigma, const float* __restrict__ u, const float* __restrict__ lambda,
    int32_t K, int64_t d, int32_t splits, const double* __restrict__ partial,
    float* __restrict__ log_ratio, uint8_t* __restrict__ accept, int32_t* __restrict__ n_accept,
    float* __restrict__ x_out) {
    const int64_t traj = blockIdx.y;
    const int lane = threadIdx.x & 63;
    const bool writer = blockIdx.x == 0 && threadIdx.x < 64;      // one wavefront per trajectory writes the scalars
    // every wavefront by itself: lane j takes drafts j, j + 64, ... in order; the first rejection so far and
    // the two sums of that draft are wave-uniform
    int32_t first = K;
    double f2 = 0.0, f3 = 0.0;
    for (int k0 = 0; k0 < K && first == K; k0 += 64) {
        const int k = k0 + lane;
        double s2 = 0.0, s3 = 0.0;
        bool ok = true;
        if (k < K) {
            const int64_t pr = traj * K + k;
            // Everything this lane needs is requested before anything is used: the three scalars (a null pointer
            // reads u in its place and is replaced by one below) and the partial sums eight at a time - one memory
            // round trip per batch instead of one per value, on the critical path of every workgroup of the launch.
            // The sums are added in index order whatever the batching (entries past the end add an exact zero).
            const float uu = u[pr];
            const float sg_raw = (sigma ? sigma : u)[pr];
            const float lam_raw = (lambda ? lambda : u)[pr];
            const double2* p = reinterpret_cast<const double2*>(partial + pr * splits * 2);
            for (int s0 = 0; s0 < splits; s0 += 8) {
                double2 v[8];
#pragma unroll
                for (int j = 0; j < 8; ++j) v[j] = p[s0 + j < splits ? s0 + j : splits - 1];
#pragma unroll
                for (int j = 0; j < 8; ++j) {
                    s2 += s0 + j < splits ? v[j].x : 0.0;
                    s3 += s0 + j < splits ? v[j].y : 0.0;
                }
            }
            const double sg = sigma ? static_cast<double>(sg_raw) : 1.0;      // null: the sums are whitened already
            const double l = -(s3 + 0.5 * s2) / (sg * sg);          // Eq. (qp)
            const double lam = lambda ? static_cast<double>(lam_raw) : 1.0;
            const double thr = fmin(0.0, lam * l);                  // Eq. (acc_relax) in the log domain
            ok = (s2 == 0.0) || (uu <= 0.0f) || (log(static_cast<double>(uu)) <= thr);
            if (writer) {
                log_ratio[pr] = static_cast<float>(l);
                accept[pr] = ok ? 1 : 0;
            }
        }
        const unsigned long long rej = __ballot(!ok);
        if (rej != 0ull) {
            const int src = __ffsll(static_cast<long long>(rej)) - 1;
            first = k0 + src;
            f2 = __shfl(s2, src, 64);
            f3 = __shfl(s3, src, 64);
        }
    }
    if (writer) {
        // the stand-alone decisions of the drafts behind the first rejection are still owed
        for (int k = (first / 64 + 1) * 64 + lane; first < K && k < K; k += 64) {
            const int64_t pr = traj * K + k;
            const double* p = partial + pr * splits * 2;
            double s2 = 0.0, s3 = 0.0;
            for (int s = 0; s < splits; ++s) { s2 += p[2 * s]; s3 += p[2 * s + 1]; }
            const double sg = sigma ? static_cast<double>(sigma[pr]) : 1.0;
            const double l = -(s3 + 0.5 * s2) / (sg * sg);
            const double lam = lambda ? static_cast<double>(lambda[pr]) : 1.0;
            const float uu = u[pr];
            const bool ok = (s2 == 0.0) || (uu <= 0.0f) || (log(static_cast<double>(uu)) <= fmin(0.0, lam * l));
            log_ratio[pr] = static_cast<float>(l);
            accept[pr] = ok ? 1 : 0;
        }
        if (lane == 0) n_accept[traj] = first;
    }
    const int32_t k = first;
    if (k >= K) return;                                          // nothing rejected: x_out untouched

    const double c = 2.0 * f3 / f2;                              // 2 e^T(x^ - m^) / ||m^ - m||
    const int64_t pr = traj * K + k;
    const float* m = m_target + pr * d;
    const float* mh = m_draft + pr * d;
    const float* xh = draft_ptr(x_draft, x_last, pr, K, d);
    float* xo = x_out + traj * d;
    const int64_t lo = static_cast<int64_t>(blockIdx.x) * kReflectChunk;
    int64_t hi = lo + kReflectChunk;
    if (hi > d) hi = d;
    const bool vec = ((d & 3) == 0) && ((reinterpret_cast<uintptr_t>(m) | reinterpret_cast<uintptr_t>(mh) |
                                         reinterpret_cast<uintptr_t>(xh) | reinterpret_cast<uintptr_t>(xo)) & 15u) == 0;
    if (vec) {
        f32x4 a[4], b[4], x[4];
        const int64_t i0 = (lo >> 2) + threadIdx.x, n4 = hi >> 2;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int64_t i = i0 + j * kFinishThreads;
            if (i < n4) {
                a[j] = reinterpret_cast<const f32x4*>(m)[i];
                b[j] = reinterpret_cast<const f32x4*>(mh)[i];
                x[j] = reinterpret_cast<const f32x4*>(xh)[i];
            }
        }
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int64_t i = i0 + j * kFinishThreads;
            if (i < n4) {
                f32x4 o;
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    const double mm = a[j][e], mmh = b[j][e], xx = x[j][e];
                    o[e] = static_cast<float>(mm + (xx - mmh) - c * (mmh - mm));
                }
                reinterpret_cast<f32x4*>(xo)[i] = o;
            }
        }
        return;
    }
    for (int64_t i = lo + threadIdx.x; i < hi; i += kFinishThreads) {
        const double mm = m[i], mmh = mh[i], xx = xh[i];
        xo[i] = static_cast<float>(mm + (xx - mmh) - c * (mmh - mm));
    }
}

inline bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

// launch 1: 256 lanes, four float4 per lane and array, non-temporal loads (measured against 512 / 1024 lanes and
// two / eight float4: equal within noise at 75 MB; the non-temporal marking is worth 13 % at 453 MB)
constexpr int kPartialThreads = 256, kPartialDepth = 4;

// ev (nullable): start and stop events attached to the dispatch itself (the kernel's own begin and end)
template <typename... Args>
void launch_timed(void (*kernel)(Args...), dim3 grid, dim3 block, hipStream_t s, hipEvent_t* ev, Args... args) {
    if (ev) hipExtLaunchKernelGGL(kernel, grid, block, 0, s, ev[0], ev[1], 0, args...);
    else hipLaunchKernelGGL(kernel, grid, block, 0, s, args...);
}

}  // namespace

size_t verify_workspace_bytes(int32_t n_traj, int32_t K, int64_t d) {
    if (n_traj < 1 || K < 1 || d < 1) return 0;
    Plan p = make_plan(n_traj, K, d, kPartialThreads, kPartialDepth);
    size_t bytes = static_cast<size_t>(n_traj) * K * p.splits * 2 * sizeof(double);
    return (bytes + 255) / 256 * 256;
}

int32_t static_verify_scratch(void** ptr) {
    constexpr int kMaxDevices = 64;
    static void* dev_ptr[kMaxDevices] = {};          // address of this library's array on each device
    static std::mutex mu;
    int dev = 0;
    if (!hip_ok(hipGetDevice(&dev))) return FREE_ERR_HIP;
    if (dev < 0 || dev >= kMaxDevices) return FREE_ERR_LIMIT;
    std::lock_guard<std::mutex> lock(mu);
    if (!dev_ptr[dev]) {
        void* p = nullptr;
        if (!hip_ok(hipGetSymbolAddress(&p, HIP_SYMBOL(scratch))) || !p) return FREE_ERR_HIP;
        dev_ptr[dev] = p;
    }
    *ptr = dev_ptr[dev];
    return FREE_OK;
}

int32_t launch_verify(const VerifyArgs& a, void* ws, size_t ws_bytes, hipStream_t s, hipEvent_t* ev4) {
    const size_t need = verify_workspace_bytes(a.n_traj, a.K, a.d);
    if (ws == nullptr || ws_bytes < need || (reinterpret_cast<uintptr_t>(ws) & 7u)) return FREE_ERR_WORKSPACE;
    const Plan p = make_plan(a.n_traj, a.K, a.d, kPartialThreads, kPartialDepth);
    const int64_t blocks = static_cast<int64_t>(a.n_traj) * a.K * p.splits;
    if (blocks > 0x7fffffffll || a.n_traj > 65535) return FREE_ERR_SHAPE;   // grid.x of launch 1, grid.y of launch 2
    double* partial = static_cast<double*>(ws);
    const bool vec = (a.d % 4 == 0) && aligned16(a.m_target) && aligned16(a.m_draft) &&
                     aligned16(a.x_draft) && (a.x_last == nullptr || aligned16(a.x_last)) &&
                     (a.sigma_elem == nullptr || aligned16(a.sigma_elem));
    ProfScope prof(a.prof, PROF_VERIFY, s);
    const dim3 g1(static_cast<unsigned>(blocks)), b1(kPartialThreads);
#define FREE_VERIFY_PARTIAL(VEC, DIAG)                                                                              \
    launch_timed(verify_partial_kernel<kPartialThreads, kPartialDepth, VEC, true, DIAG>, g1, b1, s, ev4, a.m_target, \
                 a.m_draft, a.x_draft, a.x_last, a.sigma_elem, a.K, a.d, p.chunk, p.splits, partial)
    if (a.sigma_elem) {
        if (vec) FREE_VERIFY_PARTIAL(true, true);
        else FREE_VERIFY_PARTIAL(false, true);
    } else {
        if (vec) FREE_VERIFY_PARTIAL(true, false);
        else FREE_VERIFY_PARTIAL(false, false);
    }
#undef FREE_VERIFY_PARTIAL
    if (!launch_ok()) return FREE_ERR_HIP;
    const unsigned rchunks = static_cast<unsigned>((a.d + kReflectChunk - 1) / kReflectChunk);
    launch_timed(verify_finish_kernel, dim3(rchunks, a.n_traj), dim3(kFinishThreads), s, ev4 ? ev4 + 2 : nullptr,
                 a.m_target, a.m_draft, a.x_draft, a.x_last, a.sigma, a.u, a.lambda, a.K, a.d, p.splits,
                 static_cast<const double*>(partial), a.log_ratio, a.accept, a.n_accept, a.x_out);
    if (!launch_ok()) return FREE_ERR_HIP;
    return FREE_OK;
}

}  // namespace freemi
