// Fold vectors of the LayerNorms that are folded into the GEMMs around them (bf16 weights), for every
// block of the packed target forward (Alg. 1) in one launch.  With the modulation of a block's LayerNorm,
// LN(x) (1 + scale) + shift, followed by the linear layer y = (.) W^T + b:
//   y = r (z W^T) - r mu c1 + c0,   z = x (1 + scale),
//   c1[s, n] = sum_k (1 + scale[s, k]) W[n, k],   c0[s, n] = sum_k shift[s, k] W[n, k] + b[n]
// per packed sample s.  Two such layers per block: QKV (first LayerNorm) and the MLP's first layer (second).
// HBM-bound like the adaLN modulation: every weight row is read once.  Weight rows are the A operand of
// v_mfma_f32_16x16x32_bf16, straight from global memory in the operand layout; the packed batch (<= 16 samples
// per pass) is the N dimension; the two activation vectors of each sample are staged in LDS rounded to bf16 (the
// error this leaves in c1 / c0, 2^-9 relative per term, is that of the bf16 operands of the GEMM they are
// folded into; a second product with the remainders measured 40 % slower - twice the LDS, one workgroup per CU).
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
constexpr int kBlocksPerWave = 3;          // 16-row blocks per wavefront
constexpr int kSegRows = 16 * kWaves * kBlocksPerWave;      // weight rows per workgroup: 384

// Workgroup -> (block l, layer which, row segment).  mod: [B, mod_stride] adaLN output, block l's vectors at
// l * 6 D + {0: shift1, 1: scale1, 2: gate1, 3: shift2, 4: scale2, 5: gate2} * D.  w_tab / b_tab: 2 * depth
// pointers (block l: QKV at 2 l, MLP-1 at 2 l + 1).  fold: [B, fold_stride]: c1 of all layers (block l: QKV rows,
// then MLP-1 rows), then, total_rows further, c0 in the same order.
// kExact: D / 32 is a multiple of 2 * kChunk and at least that (DiT-XL: 36 steps): every load and product is issued
// unconditionally and the k loop runs at least once, so the compiler can count the loads in flight; with the guards
// of the general form it waits for all of them before the first product of a register set.
template <bool kExact>
__global__ __launch_bounds__(kThreads) void ln_fold_kernel(
    const float* __restrict__ mod, int32_t B, int32_t D, int32_t mod_stride, int32_t rows_qkv, int32_t rows_fc1,
    const void* const* __restrict__ w_tab, const float* const* __restrict__ b_tab, float* __restrict__ fold,
    int64_t fold_stride, int32_t total_rows) {
    extern __shared__ __attribute__((aligned(16))) char lds[];
    const int row_bytes = D * 2 + 16;                       // odd number of 16-byte chunks per row
    const int set_bytes = kBatch * row_bytes;
    char* s1_hi = lds;                                      // 1 + scale
    char* s0_hi = lds + set_bytes;                          // shift
    // (the wavefront index as a scalar: row-block bookkeeping stays in scalar registers)
    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);

    const int segs_qkv = (rows_qkv + kSegRows - 1) / kSegRows, segs_fc1 = (rows_fc1 + kSegRows - 1) / kSegRows;
    const int per_block = segs_qkv + segs_fc1;
    const int l = blockIdx.x / per_block, sidx = blockIdx.x % per_block;
    const int which = sidx < segs_qkv ? 0 : 1;
    const int seg = which ? sidx - segs_qkv : sidx;
    const int rows = which ? rows_fc1 : rows_qkv;
    const int out_row0 = l * (rows_qkv + rows_fc1) + (which ? rows_qkv : 0);     // first output row of this layer
    const float* shift = mod + static_cast<int64_t>(l) * 6 * D + (which ? 3 : 0) * D;
    const float* scale = shift + D;

    // stage (1 + scale) and shift of every sample rounded to bf16; rows past B are zero.  Every thread requests its
    // (up to kStage) pairs of 16-byte pieces before it converts the first one: one memory round trip per batch.
    {
        constexpr int kStage = 9;
        const int per_row = D / 4, nvec = kBatch * per_row;
        for (int base = tid; base < nvec; base += kThreads * kStage) {
            float4 vs[kStage], vt[kStage];
#pragma unroll
            for (int u = 0; u < kStage; ++u) {
                const int i = base + u * kThreads;
                const int b = i / per_row, p = i - b * per_row;
                const bool live = i < nvec && b < B;
                const int64_t off = static_cast<int64_t>(live ? b : 0) * mod_stride;
                vs[u] = reinterpret_cast<const float4*>(scale + off)[live ? p : 0];
                vt[u] = reinterpret_cast<const float4*>(shift + off)[live ? p : 0];
            }
#pragma unroll
            for (int u = 0; u < kStage; ++u) {
                const int i = base + u * kThreads;
                if (i < nvec) {
                    const int b = i / per_row, p = i - b * per_row;
                    const bool live = b < B;
                    const float a0 = live ? 1.0f + vs[u].x : 0.f, a1 = live ? 1.0f + vs[u].y : 0.f;
                    const float a2 = live ? 1.0f + vs[u].z : 0.f, a3 = live ? 1.0f + vs[u].w : 0.f;
                    const float t0 = live ? vt[u].x : 0.f, t1 = live ? vt[u].y : 0.f, t2 = live ? vt[u].z : 0.f, t3 = live ? vt[u].w : 0.f;
                    *reinterpret_cast<uint2*>(s1_hi + b * row_bytes + p * 8) = uint2{pack_bf16_pair(a0, a1), pack_bf16_pair(a2, a3)};
                    *reinterpret_cast<uint2*>(s0_hi + b * row_bytes + p * 8) = uint2{pack_bf16_pair(t0, t1), pack_bf16_pair(t2, t3)};
                }
            }
        }
    }
    __syncthreads();

    const int l16 = lane & 15, lq = lane >> 4;
    const int act_off = l16 * row_bytes + lq * 16;
    const int steps = D / 32;
    const int nblocks = rows / 16;
    const int first = seg * (kSegRows / 16) + wave * kBlocksPerWave;
    const int last = first + kBlocksPerWave < nblocks ? first + kBlocksPerWave : nblocks;
    // (global address space stated explicitly: the pointer comes from a table in memory, and as a generic
    // pointer every load would be a flat load ordered against the LDS reads)
    using gvec = const __attribute__((address_space(1))) u32x4_t*;
    const char* wmat = static_cast<const char*>(w_tab[2 * l + which]);
    const float* bias = b_tab[2 * l + which];
    u32x4_t wa[kChunk], wb[kChunk];
    auto load = [&](u32x4_t (&dst)[kChunk], const char* wrow, int st0) {
#pragma unroll
        for (int u = 0; u < kChunk; ++u)
            if (kExact || st0 + u < steps) dst[u] = *(gvec)(wrow + (st0 + u) * 64);
    };
    auto row_ptr = [&](int blk) { return wmat + (static_cast<int64_t>(blk * 16 + l16) * D) * 2 + lq * 16; };
    const char* wrow = nullptr;
    if (first < last) {
        wrow = row_ptr(first);
        load(wa, wrow, 0);
    }
    for (int blk = first; blk < last; ++blk) {
        const int r0 = blk * 16;
        // (after the last block of an exact launch the prefetch re-reads this block's first chunk: in bounds, unused)
        const char* wnext = (blk + 1 < last) ? row_ptr(blk + 1) : (kExact ? wrow : nullptr);
        // (requested before this block's weights: loads complete in order, and as a global - not generic - load)
        const f32x4_t bv = *(const __attribute__((address_space(1))) f32x4_t*)(bias + r0 + 4 * lq);
        f32x4_t acc1 = {0.f, 0.f, 0.f, 0.f}, acc0 = {0.f, 0.f, 0.f, 0.f};
        auto multiply = [&](const u32x4_t (&src)[kChunk], int st0) {
#pragma unroll
            for (int u = 0; u < kChunk; ++u)
                if (kExact || st0 + u < steps) {
                    const bf16x8_t a = __builtin_bit_cast(bf16x8_t, src[u]);
                    const int o = act_off + (st0 + u) * 64;
                    acc1 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, *reinterpret_cast<const bf16x8_t*>(s1_hi + o), acc1, 0, 0, 0);
                    acc0 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, *reinterpret_cast<const bf16x8_t*>(s0_hi + o), acc0, 0, 0, 0);
                }
        };
        if constexpr (kExact) {
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
        // accumulator register i of lane l: weight row 4 (l / 16) + i, sample l % 16
        f32x4_t o0;
#pragma unroll
        for (int i = 0; i < 4; ++i) o0[i] = acc0[i] + bv[i];
        if (l16 < B) {
            float* dst = fold + static_cast<int64_t>(l16) * fold_stride + out_row0 + r0 + 4 * lq;
            *reinterpret_cast<f32x4_t*>(dst) = acc1;
            *reinterpret_cast<f32x4_t*>(dst + total_rows) = o0;
        }
    }
}

}  // namespace

// Supported: bf16 weights, D % 32 == 0, D <= 2048 (two staged vector sets of 16 rows in LDS), both row counts
// multiples of 16; 16-byte aligned weight rows, biases, mod and fold rows.
bool ln_fold_supported(int32_t D, int32_t rows_qkv, int32_t rows_fc1) {
    return D % 32 == 0 && D <= 2048 && rows_qkv % 16 == 0 && rows_fc1 % 16 == 0;
}

int32_t launch_ln_fold(const float* mod, int32_t B, int32_t D, int32_t mod_stride, int32_t depth, int32_t rows_qkv,
                       int32_t rows_fc1, const void* const* w_tab, const float* const* b_tab, float* fold,
                       int64_t fold_stride, hipStream_t s) {
    if (!ln_fold_supported(D, rows_qkv, rows_fc1)) return FREE_ERR_SHAPE;
    const int32_t total_rows = depth * (rows_qkv + rows_fc1);
    if ((reinterpret_cast<uintptr_t>(mod) | reinterpret_cast<uintptr_t>(fold)) & 15u) return FREE_ERR_SHAPE;
    if (fold_stride < 2 * static_cast<int64_t>(total_rows) || (fold_stride & 3) || (mod_stride & 3)) return FREE_ERR_SHAPE;
    const size_t lds = 2 * static_cast<size_t>(kBatch) * (static_cast<size_t>(D) * 2 + 16);
    const bool exact = D >= 64 * kChunk && (D / 32) % (2 * kChunk) == 0;
    auto kernel = exact ? ln_fold_kernel<true> : ln_fold_kernel<false>;
    static bool attr_set[2] = {false, false};
    if (!attr_set[exact]) {
        if (!hip_ok(hipFuncSetAttribute(reinterpret_cast<const void*>(kernel),
                                        hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024)))
            return FREE_ERR_HIP;
        attr_set[exact] = true;
    }
    const int per_block = (rows_qkv + kSegRows - 1) / kSegRows + (rows_fc1 + kSegRows - 1) / kSegRows;
    for (int b0 = 0; b0 < B; b0 += kBatch) {
        const int nb = (B - b0 < kBatch) ? B - b0 : kBatch;
        hipLaunchKernelGGL(kernel, dim3(depth * per_block), dim3(kThreads), lds, s,
                           mod + static_cast<int64_t>(b0) * mod_stride, nb, D, mod_stride, rows_qkv, rows_fc1, w_tab, b_tab,
                           fold + static_cast<int64_t>(b0) * fold_stride, fold_stride, total_rows);
        if (!launch_ok()) return FREE_ERR_HIP;
    }
    return FREE_OK;
}

}  // namespace freemi
