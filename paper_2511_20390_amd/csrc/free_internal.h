// Internal declarations shared by the translation units of libfree_mi355x.
// Host-side launch wrappers only; every kernel lives in exactly one .hip file.
#pragma once

#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include "../../include/free_mi355x.h"

namespace freemi {

// ---- bf16 storage type: raw bits, round-to-nearest-even conversion ----------
struct bf16_t {
    uint16_t v;
};

__host__ __device__ inline float bf16_to_float(bf16_t h) {
    union { uint32_t u; float f; } c;
    c.u = static_cast<uint32_t>(h.v) << 16;
    return c.f;
}

__host__ __device__ inline bf16_t float_to_bf16(float f) {
    union { uint32_t u; float f; } c;
    c.f = f;
    uint32_t u = c.u;
    bf16_t r;
    if ((u & 0x7fffffffu) > 0x7f800000u) {          // NaN stays NaN
        r.v = static_cast<uint16_t>((u >> 16) | 0x40u);
        return r;
    }
    u += 0x7fffu + ((u >> 16) & 1u);
    r.v = static_cast<uint16_t>(u >> 16);
    return r;
}

#if defined(__HIPCC__)
// two floats -> packed bf16 pair (low half = first), hardware round-to-nearest-even
__device__ inline uint32_t pack_bf16_pair(float lo, float hi) {
    typedef float f2_t __attribute__((ext_vector_type(2)));
    typedef __bf16 b2_t __attribute__((ext_vector_type(2)));
    const f2_t f = {lo, hi};
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(f, b2_t));
}
#endif

__device__ inline float load_f(const float* p) { return *p; }
__device__ inline float load_f(const bf16_t* p) { return bf16_to_float(*p); }
__device__ inline void store_f(float* p, float v) { *p = v; }
__device__ inline void store_f(bf16_t* p, float v) { *p = float_to_bf16(v); }

__host__ __device__ inline float gelu_tanh_f(float v) {
    const float k = 0.7978845608028654f;            // sqrt(2/pi)
    float inner = k * (v + 0.044715f * v * v * v);
    return 0.5f * v * (1.0f + tanhf(inner));
}

__host__ __device__ inline float silu_f(float v) { return v / (1.0f + expf(-v)); }

constexpr float kLnEps = 1e-6f;

// Per-sample modulation / gate vector of an epilogue or a LayerNorm:
// value for (row m, column n) = base[(m / rows_per_sample) * stride + n].
struct RowVec {
    const float* base;
    int32_t stride;
    int32_t rows_per_sample;
};

// LayerNorm + modulate folded into the GEMMs on both sides of it (bf16 matrix-core path only).
// With z = x (1 + scale) rounded to bf16, row mean mu and r = 1 / sqrt(var + eps):
//   (LN(x) (1 + scale) + shift) W^T + b = r (z W^T) - r mu c1 + c0,
//   c1[n] = sum_k (1 + scale[k]) W[n, k],  c0[n] = sum_k shift[k] W[n, k] + b[n]   (per sample).
// The GEMM that updates the residual stream (producer, FREE_EPI_GATE_RESID_PREP) also writes z for the
// next LayerNorm and, per row and per 128-column slot, the sums of x and x^2; the GEMM that consumes the
// normalised rows (FREE_EPI_LN_BIAS / FREE_EPI_LN_BIAS_GELU) multiplies z and applies r, mu, c1, c0 in
// its epilogue.  No separate pass over the residual stream, no atomics: every partial sum has one writer
// and the consumer adds the slots of a row in a fixed order.
constexpr int FREE_EPI_LN_BIAS = 3, FREE_EPI_LN_BIAS_GELU = 4, FREE_EPI_GATE_RESID_PREP = 5;
constexpr int kLnSlotCols = 128;           // columns of the residual stream per partial-sum slot
struct LnFold {
    // producer: scale vector of the NEXT LayerNorm (indexed like the gate: same stride and rows per sample),
    // z [M, N] bf16 and stats [M, slots, 2] fp32 are outputs.  consumer: stats is an input.
    const float* scale_next = nullptr;
    void* z = nullptr;
    float* stats = nullptr;
    int32_t slots = 0;                     // width of the normalised rows / kLnSlotCols
    // consumer: c1 / c0 of sample s start at c1[s * fold_stride] (N entries each, 16-byte aligned)
    const float* c1 = nullptr;
    const float* c0 = nullptr;
    int64_t fold_stride = 0;
    int32_t rows_per_sample = 1;
    float inv_width = 0.f;                 // 1 / width of the normalised rows
};

// Thread-local HIP error memo (free_last_hip_error).
void note_hip_error(hipError_t e);
inline bool hip_ok(hipError_t e) {
    if (e != hipSuccess) { note_hip_error(e); return false; }
    return true;
}
inline bool launch_ok() { return hip_ok(hipGetLastError()); }

// ---- optional per-kernel timing (free_profile_begin / free_profile_end) --------
// A Profiler belongs to a model handle.  While it is on, a ProfScope records a HIP event on the
// launch stream before and after the launches it brackets; with a null or idle profiler it does nothing.
enum ProfCat {
    PROF_COND = 0, PROF_ADALN, PROF_PATCH, PROF_LN_MOD, PROF_GEMM_QKV, PROF_ATTN, PROF_GEMM_PROJ,
    PROF_GEMM_FC1, PROF_GEMM_FC2, PROF_FINAL, PROF_EPS2MEAN, PROF_VERIFY,
    PROF_NCAT
};
static_assert(PROF_NCAT == FREE_PROF_NCAT, "category count is part of the ABI");
struct Profiler;
struct ProfScope {
    ProfScope(Profiler* p, int cat, hipStream_t s);
    ~ProfScope();
    Profiler* prof;
    int slot;
    hipStream_t stream;
};

// ---- verification (verify.hip) -------------------------------------------------
struct VerifyArgs {
    const float* m_target;   // [n_traj, K, d]
    const float* m_draft;    // [n_traj, K, d]
    const float* x_draft;    // [n_traj, K, d]; or, when x_last != nullptr, the K packed
                             // states of ONE trajectory: draft k is x_draft + (k+1) d
    const float* x_last;     // nullptr, or the K-th draft of the single trajectory
    const float* sigma; const float* u; const float* lambda;   // sigma [n_traj, K]; nullptr with sigma_elem
    int32_t n_traj, K; int64_t d;
    float* log_ratio; uint8_t* accept; int32_t* n_accept; float* x_out;
    Profiler* prof;          // nullptr, or the profiler of the handle the call belongs to
    const float* sigma_elem = nullptr;   // nullptr, or one standard deviation per element [n_traj, K, d]
};
size_t verify_workspace_bytes(int32_t n_traj, int32_t K, int64_t d);
// device address, on the current device, of the library's static scratch array (FREE_STATIC_SCRATCH_BYTES);
// looked up once per device with hipGetSymbolAddress, no allocation
int32_t static_verify_scratch(void** ptr);
// ev4 (nullable): four events, attached as start / stop to the dispatches of the two launches (benchmark timing)
int32_t launch_verify(const VerifyArgs& a, void* ws, size_t ws_bytes, hipStream_t s, hipEvent_t* ev4 = nullptr);

// ---- simple DiT kernels, both dtypes (dit_kernels.hip) ---------------------------
int32_t launch_conditioning(const int32_t* t, const int32_t* y, int32_t B, int32_t D, int32_t tfreq,
                            const float* w1, const float* b1, const float* w2, const float* b2,
                            const float* ytab, float* h1, float* sc, hipStream_t s);
// mod[b, r] = sum_i sc[b, i] W_r[i] + bias_r; rows r come from n_mats matrices of
// rows_per_mat rows each (device pointer tables), plus they are laid out back to
// back in mod with the given offsets.
int32_t launch_adaln(const float* sc, int32_t B, int32_t D, const void* const* w_tab,
                     const float* const* b_tab, const int32_t* row_start, int32_t n_mats,
                     int32_t total_rows, int32_t dtype, float* mod, hipStream_t s);
int32_t launch_patch_embed(const float* x, int32_t x_mod, int32_t B, int32_t C, int32_t H, int32_t W,
                           int32_t p, int32_t D, const float* pw, const float* pb, const float* pos,
                           float* out, hipStream_t s);
int32_t launch_ln_modulate(const float* x, RowVec shift, RowVec scale, int32_t M, int32_t D,
                           int32_t dtype, void* out, hipStream_t s);
int32_t launch_linear_simple(const void* A, const void* W, const float* bias, int32_t M, int32_t N,
                             int32_t K, int32_t dtype, int32_t epi, void* out, float* resid,
                             RowVec gate, hipStream_t s);
int32_t launch_attention_simple(const void* qkv, int32_t B, int32_t N, int32_t heads, int32_t dh,
                                int32_t dtype, void* out, hipStream_t s);
int32_t launch_final_layer(const float* x, RowVec shift, RowVec scale, int32_t B, int32_t gh, int32_t gw,
                           int32_t p, int32_t c_out, int32_t D, const void* w, const float* bias,
                           int32_t dtype, float* out, hipStream_t s);
int32_t launch_eps_to_mean(const float* eps_out, const float* x_states, const float* coef_x,
                           const float* coef_eps, float cfg_scale, int32_t K, int32_t C, int32_t c_out,
                           int64_t hw, float* m_out, hipStream_t s, float* eps_guided = nullptr,
                           const float* sigma_step = nullptr, const float* xi = nullptr, float* x_next = nullptr);
int32_t launch_pack_cond(const int32_t* t, int32_t y, int32_t null_label, int32_t K, int32_t dup,
                         int32_t* t_out, int32_t* y_out, hipStream_t s);

// drafter helper: fin = [emb | feat] in the compute type, zero_out (nullable) cleared
int32_t launch_fuse_pack(const float* emb, const float* feat, int64_t M, int32_t D, int32_t dtype, void* fin,
                         float* zero_out, hipStream_t s);
// blocking range check of device-resident inputs (any pointer may be null); bit mask of violations
int32_t run_validate(const int32_t* t, int64_t n_t, int32_t T, const float* sigma, const float* u,
                     const float* lambda, int64_t n, uint32_t* violations, hipStream_t s);
// calib.hip: register-only MFMA loop on every CU; sustained TFLOP/s and shader clock (MHz) while it runs
int32_t run_mfma_ceiling(int32_t iters, double* tflops, double* mhz, hipStream_t s);

// frozen-target drafting of K steps from one noise estimate e [d]; out[k] = ||a_k - b_k||^2 (fp64)
int32_t launch_frozen_draft(const float* x_a, const float* e, const float* coef_x, const float* coef_eps,
                            const float* sigma, const float* xi, int32_t K, int64_t d, float* x_states, float* x_last,
                            float* m_draft, hipStream_t s);
int32_t launch_sqdist(const float* a, const float* b, int32_t K, int64_t d, double* out, hipStream_t s);

// ---- MFMA adaLN modulation GEMV, bf16 or fp32 weights as `mode` says (adaln_mfma.hip)
bool adaln_mfma_supported(int32_t D, int32_t total_rows);
// final_mfma.hip: final layer on the matrix cores (bf16 weights, DiT-S/B/L/XL widths)
bool final_mfma_supported(int32_t D, int32_t P);
int32_t launch_final_layer_mfma(const float* x, RowVec shift, RowVec scale, int32_t M, int32_t gh, int32_t gw,
                                int32_t p, int32_t c_out, int32_t D, const bf16_t* w, const float* bias, float* out,
                                hipStream_t s);
int32_t launch_adaln_mfma(const float* sc, int32_t B, int32_t D, const void* const* w_tab,
                          const float* const* b_tab, const int32_t* row_start, int32_t n_mats,
                          int32_t total_rows, int32_t mode, float* mod, hipStream_t s);

// ---- MFMA kernels, bf16 only (gemm_mfma.hip, attn_mfma.hip) ------------------------
bool mfma_linear_supported(int32_t M, int32_t N, int32_t K);
int32_t launch_linear_mfma(const bf16_t* A, const bf16_t* W, const float* bias, int32_t M, int32_t N,
                           int32_t K, int32_t epi, bf16_t* out, float* resid, RowVec gate, hipStream_t s, int cu_share = 1,
                           const LnFold* ln = nullptr);
// shapes the folded-LayerNorm epilogues cover: M rows of width D normalised, rows_per_sample tokens per sample
bool mfma_ln_fold_supported(int32_t M, int32_t D, int32_t rows_per_sample);
// the same kernel on fp32 operands (v_mfma_f32_32x32x2_f32), fp32 output
bool mfma_linear_f32_supported(int32_t M, int32_t N, int32_t K);
int32_t launch_linear_mfma_f32(const float* A, const float* W, const float* bias, int32_t M, int32_t N,
                               int32_t K, int32_t epi, float* out, float* resid, RowVec gate, hipStream_t s,
                               int cu_share = 1);
// fold vectors of all blocks in one launch (lnfold_mfma.hip); see LnFold
bool ln_fold_supported(int32_t D, int32_t rows_qkv, int32_t rows_fc1);
int32_t launch_ln_fold(const float* mod, int32_t B, int32_t D, int32_t mod_stride, int32_t depth, int32_t rows_qkv,
                       int32_t rows_fc1, const void* const* w_tab, const float* const* b_tab, float* fold,
                       int64_t fold_stride, hipStream_t s);
bool mfma_attention_supported(int32_t N, int32_t dh);
int32_t launch_attention_mfma(const bf16_t* qkv, int32_t B, int32_t N, int32_t heads, int32_t dh,
                              bf16_t* out, hipStream_t s);
// fp32 operands and softmax on the matrix cores (attn_f32_mfma.hip); qkv and out 16-byte aligned
bool mfma_attention_f32_supported(int32_t N, int32_t dh);
int32_t launch_attention_mfma_f32(const float* qkv, int32_t B, int32_t N, int32_t heads, int32_t dh,
                                  float* out, hipStream_t s);

}  // namespace freemi
