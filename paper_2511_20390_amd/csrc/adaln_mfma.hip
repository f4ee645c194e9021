// adaLN modulation of every block and of the final layer in one launch (bf16 weights; fp32 weights below):
//   mod[b, r] = sum_i SiLU(c)[b, i] W_r[i] + bias_r       (packed batch b, row r of the
//   stacked modulation matrices; the conditioning vector c is constant across blocks,
//   so the whole stack is one skinny GEMM that reads a third of all DiT parameters).
// HBM-bound: every weight byte is needed exactly once per forward.  The packed batch
// (<= 16 states per pass) is the N dimension of v_mfma_f32_16x16x32_bf16; weight rows are
// the A operand and are loaded straight from global memory in the MFMA operand layout
// (lane l: row l%16, 16 bytes at k = 8*(l/16)), so they never touch LDS.  The activation
// operand lives in LDS, split into a bf16 high part and a bf16 remainder (two MFMAs per
// k-step) so that the fp32 conditioning vector loses no precision.
// fp32 weights (FREE_FP32 mode) take the same route with v_mfma_f32_16x16x4_f32: a lane's 16 bytes are four
// consecutive k of its row and feed four products, the activation operand is 16 bytes of the fp32 vector in LDS
// at the same offset (lane group q of product j contracts k = 16 s + 4 q + j on both sides).
#include "free_internal.h"

namespace freemi {

namespace {

typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef float f32x4_t __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4_t __attribute__((ext_vector_type(4)));

constexpr int kWaves = 8;                  // per workgroup: they share one staged copy of the activations
constexpr int kThreads = 64 * kWaves;
constexpr int kChunk = 6;                  // k-steps (1 KB of weights per wavefront each) per register set
constexpr int kBatch = 16;

// kExact: the k-steps of a row (64 bytes each: D / 32 in bf16, D / 16 in fp32; DiT-XL: 36 / 72) are a multiple of
// 2 * kChunk, so every load and product below is issued
// unconditionally.  With the guards of the general form the compiler cannot count the loads in flight and waits
// for all of them (vmcnt(0)) before the first product of a register set - the other set's loads included.
template <bool kExact, bool kF32>
__global__ __launch_bounds__(kThreads) void adaln_mfma_kernel(
    const float* __restrict__ sc, int32_t B, int32_t D, const void* const* __restrict__ w_tab,
    const float* const* __restrict__ b_tab, const int32_t* __restrict__ row_start, int32_t n_mats,
    int32_t total_rows, int32_t blocks_per_wave, float* __restrict__ mod) {
    extern __shared__ __attribute__((aligned(16))) char lds[];
    constexpr int kEl = kF32 ? 4 : 2;                       // bytes per weight
    const int row_bytes = D * kEl + 16;                     // odd number of 16-byte chunks per row
    char* s_hi = lds;                                       // (fp32 weights: the fp32 vector itself, one set)
    char* s_lo = lds + kBatch * row_bytes;
    // (the wavefront index is made a scalar: row blocks, matrix index and table lookups then stay in scalar
    // registers - as per-lane values every table lookup is a vector load whose wait drains the weight loads)
    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);

    // stage SiLU(c) as hi + lo bf16 parts; rows past B are zero.  Every thread requests its (up to kStage) 16-byte
    // pieces before it converts the first one: one memory round trip per batch instead of one per piece, and this
    // prologue is exposed - all workgroups of the launch are resident at once and start with it.
    {
        constexpr int kStage = 9;
        const int per_row = D / 4, nvec = kBatch * per_row;
        for (int base = tid; base < nvec; base += kThreads * kStage) {
            float4 v[kStage];
#pragma unroll
            for (int u = 0; u < kStage; ++u) {
                const int i = base + u * kThreads;
                const int b = i / per_row, p = i - b * per_row;
                const bool live = i < nvec && b < B;
                v[u] = reinterpret_cast<const float4*>(sc + static_cast<int64_t>(live ? b : 0) * D)[live ? p : 0];
            }
#pragma unroll
            for (int u = 0; u < kStage; ++u) {
                const int i = base + u * kThreads;
                if (i < nvec) {
                    const int b = i / per_row, p = i - b * per_row;
                    const bool live = b < B;
                    const float x0 = live ? v[u].x : 0.f, x1 = live ? v[u].y : 0.f, x2 = live ? v[u].z : 0.f, x3 = live ? v[u].w : 0.f;
                    if constexpr (kF32) {
                        *reinterpret_cast<float4*>(s_hi + b * row_bytes + p * 16) = float4{x0, x1, x2, x3};
                        continue;
                    }
                    const uint32_t h0 = pack_bf16_pair(x0, x1), h1 = pack_bf16_pair(x2, x3);
                    const uint32_t l0 = pack_bf16_pair(x0 - __uint_as_float(h0 << 16), x1 - __uint_as_float(h0 & 0xffff0000u));
                    const uint32_t l1 = pack_bf16_pair(x2 - __uint_as_float(h1 << 16), x3 - __uint_as_float(h1 & 0xffff0000u));
                    *reinterpret_cast<uint2*>(s_hi + b * row_bytes + p * 8) = uint2{h0, h1};
                    *reinterpret_cast<uint2*>(s_lo + b * row_bytes + p * 8) = uint2{l0, l1};
                }
            }
        }
    }
    __syncthreads();

    const int l16 = lane & 15, lq = lane >> 4;
    const int nblocks = total_rows / 16;
    const int first = (blockIdx.x * kWaves + wave) * blocks_per_wave;
    const char* bh = s_hi + l16 * row_bytes + lq * 16;
    const char* bl = s_lo + l16 * row_bytes + lq * 16;
    const int steps = D * kEl / 64;
    // Weight rows stream through two register sets of kChunk k-steps each: the loads of one set are in
    // flight while the other is multiplied, across row blocks too (the first chunk of the next block is
    // requested before the last chunk of this one is multiplied).  The pointers come from a table in
    // memory, so they are cast to the global address space explicitly - as generic pointers every load
    // would be a flat load that the compiler must order against the LDS reads, one load in flight per
    // wavefront.
    using gvec = const __attribute__((address_space(1))) u32x4_t*;
    u32x4_t wa[kChunk], wb[kChunk];
    auto load = [&](u32x4_t (&dst)[kChunk], const char* wrow, int st0) {
#pragma unroll
        for (int u = 0; u < kChunk; ++u)
            if (kExact || st0 + u < steps) dst[u] = *(gvec)(wrow + (st0 + u) * 64);
    };
    int mat = 0;
    auto row_ptr = [&](int blk) {          // advances `mat` to the matrix that holds row block blk
        const int r0 = blk * 16;
        while (mat + 1 < n_mats && r0 >= row_start[mat + 1]) ++mat;
        return static_cast<const char*>(w_tab[mat]) + (static_cast<int64_t>(r0 - row_start[mat] + l16) * D) * kEl + lq * 16;
    };
    const int last = (first + blocks_per_wave < nblocks) ? first + blocks_per_wave : nblocks;
    const char* wrow = nullptr;
    if (first < last) {
        wrow = row_ptr(first);
        load(wa, wrow, 0);
    }
    f32x4_t kept[3] = {};
    for (int blk = first; blk < last; ++blk) {
        const int r0 = blk * 16;
        const int cur_mat = mat;
        const int lr0 = r0 - row_start[cur_mat];
        // (after the last block of an exact launch the prefetch re-reads this block's first chunk: in bounds, unused)
        const char* wnext = (blk + 1 < last) ? row_ptr(blk + 1) : (kExact ? wrow : nullptr);
        // (requested before the weights of this block: loads complete in order, so a bias load placed after the
        // k loop would wait for the next block's prefetch)
        const f32x4_t bias = *(const __attribute__((address_space(1))) f32x4_t*)(b_tab[cur_mat] + lr0 + 4 * lq);
        f32x4_t acc = {0.f, 0.f, 0.f, 0.f};
        auto multiply = [&](const u32x4_t (&src)[kChunk], int st0) {
#pragma unroll
            for (int u = 0; u < kChunk; ++u)
                if (kExact || st0 + u < steps) {
                    if constexpr (kF32) {
                        const f32x4_t a = __builtin_bit_cast(f32x4_t, src[u]);
                        const f32x4_t x = *reinterpret_cast<const f32x4_t*>(bh + (st0 + u) * 64);
#pragma unroll
                        for (int j = 0; j < 4; ++j) acc = __builtin_amdgcn_mfma_f32_16x16x4f32(a[j], x[j], acc, 0, 0, 0);
                        continue;
                    }
                    const bf16x8_t a = __builtin_bit_cast(bf16x8_t, src[u]);
                    const bf16x8_t h = *reinterpret_cast<const bf16x8_t*>(bh + (st0 + u) * 64);
                    const bf16x8_t l = *reinterpret_cast<const bf16x8_t*>(bl + (st0 + u) * 64);
                    acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, h, acc, 0, 0, 0);
                    acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, l, acc, 0, 0, 0);
                }
        };
        if constexpr (kExact) {
            // at least one pass (the launch checks steps >= 2 kChunk): a loop that may be skipped would make the
            // bias load the youngest one on that path and the wait before the store a wait for everything
            int st0 = 0;
            do {
                load(wb, wrow, st0 + kChunk);
                __builtin_amdgcn_sched_barrier(0);      // the loads stay ahead of the products they overlap
                multiply(wa, st0);
                __builtin_amdgcn_sched_barrier(0);
                load(wa, (st0 + 2 * kChunk < steps) ? wrow + (st0 + 2 * kChunk) * 64 : wnext, 0);
                __builtin_amdgcn_sched_barrier(0);
                multiply(wb, st0 + kChunk);
                st0 += 2 * kChunk;
            } while (st0 < steps);
        } else {
            for (int st0 = 0; st0 < steps; st0 += 2 * kChunk) {
                load(wb, wrow, st0 + kChunk);
                multiply(wa, st0);
                if (st0 + 2 * kChunk < steps) load(wa, wrow, st0 + 2 * kChunk);
                else if (wnext) load(wa, wnext, 0);
                multiply(wb, st0 + kChunk);
            }
        }
        wrow = wnext;
        // accumulator register i of lane l: weight row 4*(l/16) + i, batch column l%16
        f32x4_t o;
#pragma unroll
        for (int i = 0; i < 4; ++i) o[i] = acc[i] + bias[i];
        // the results of a wavefront's first three blocks (all of them at the usual launch shape) are kept and
        // stored together at the end: 192 contiguous bytes per sample in three stores back to back, instead of 64
        // bytes per block scattered through the weight stream (measured 3.5 us of 99 at DiT-XL/2, 12 samples)
        const int jb = blk - first;
        if (jb == 0) kept[0] = o;
        else if (jb == 1) kept[1] = o;
        else if (jb == 2) kept[2] = o;
        else if (l16 < B) *reinterpret_cast<f32x4_t*>(mod + static_cast<int64_t>(l16) * total_rows + r0 + 4 * lq) = o;
    }
    if (l16 < B) {
        float* dst = mod + static_cast<int64_t>(l16) * total_rows + first * 16 + 4 * lq;
        if (first < last) *reinterpret_cast<f32x4_t*>(dst) = kept[0];
        if (first + 1 < last) *reinterpret_cast<f32x4_t*>(dst + 16) = kept[1];
        if (first + 2 < last) *reinterpret_cast<f32x4_t*>(dst + 32) = kept[2];
    }
}

}  // namespace

// Supported: bf16 or fp32 weights, D % 32 == 0; every matrix has a multiple of 16 rows (true for
// the 6D / 2D row stacks when D % 8 == 0).  16-byte aligned weight rows, biases and mod.
bool adaln_mfma_supported(int32_t D, int32_t total_rows) { return D % 32 == 0 && total_rows % 16 == 0 && D <= 2048; }

int32_t launch_adaln_mfma(const float* sc, int32_t B, int32_t D, const void* const* w_tab,
                          const float* const* b_tab, const int32_t* row_start, int32_t n_mats,
                          int32_t total_rows, int32_t mode, float* mod, hipStream_t s) {
    if ((reinterpret_cast<uintptr_t>(sc) | reinterpret_cast<uintptr_t>(mod)) & 15u) return FREE_ERR_SHAPE;
    if (!adaln_mfma_supported(D, total_rows)) return FREE_ERR_SHAPE;
    const bool f32 = mode == FREE_FP32;
    const int nblocks = total_rows / 16;
    // about 16 wavefronts per CU at the DiT-XL size (12096 row blocks): measured best among 2, 3, 6, 12
    const int blocks_per_wave = nblocks >= 8192 ? 3 : 1;
    const int waves = (nblocks + blocks_per_wave - 1) / blocks_per_wave;
    const int grid = (waves + kWaves - 1) / kWaves;
    const int el = f32 ? 4 : 2;
    const size_t lds = (f32 ? 1 : 2) * static_cast<size_t>(kBatch) * (D * el + 16);
    const int steps = D * el / 64;
    const bool exact = steps >= 2 * kChunk && steps % (2 * kChunk) == 0;
    using kernel_t = void (*)(const float*, int32_t, int32_t, const void* const*, const float* const*, const int32_t*,
                              int32_t, int32_t, int32_t, float*);
    static const kernel_t kernels[4] = {adaln_mfma_kernel<false, false>, adaln_mfma_kernel<true, false>,
                                        adaln_mfma_kernel<false, true>, adaln_mfma_kernel<true, true>};
    const int which = 2 * f32 + exact;
    const kernel_t kernel = kernels[which];
    static bool attr_set[4] = {false, false, false, false};
    if (!attr_set[which]) {
        if (!hip_ok(hipFuncSetAttribute(reinterpret_cast<const void*>(kernel),
                                        hipFuncAttributeMaxDynamicSharedMemorySize, 150 * 1024)))
            return FREE_ERR_HIP;
        attr_set[which] = true;
    }
    for (int b0 = 0; b0 < B; b0 += kBatch) {
        const int nb = (B - b0 < kBatch) ? B - b0 : kBatch;
        hipLaunchKernelGGL(kernel, dim3(grid), dim3(kThreads), lds, s, sc + static_cast<int64_t>(b0) * D,
                           nb, D, w_tab, b_tab, row_start, n_mats, total_rows, blocks_per_wave,
                           mod + static_cast<int64_t>(b0) * total_rows);
        if (!launch_ok()) return FREE_ERR_HIP;
    }
    return FREE_OK;
}

}  // namespace freemi
