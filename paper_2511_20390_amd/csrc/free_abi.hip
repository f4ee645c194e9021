// C-ABI entry points of libfree_mi355x: argument checks, the model handle, the
// workspace carve-up and the chaining of kernels for the packed target forward
// (Alg. 1, "compute means ... in parallel"), the verification loop (Alg. 2 inside
// Alg. 1) and a whole round.  All arithmetic runs in the HIP kernels; the only
// host-side mathematics is the diffusion schedule helper (Eq. ddpm_update) and the
// fixed positional table computed once at handle creation.
#include <algorithm>
#include <cmath>
#include <cstring>
#include <new>
#include <vector>

#include "free_internal.h"

namespace freemi {

static thread_local int32_t g_last_hip_error = 0;
void note_hip_error(hipError_t e) { g_last_hip_error = static_cast<int32_t>(e); }

// ---- per-kernel timing ------------------------------------------------------------
struct Profiler {
    bool on = false;
    std::vector<hipEvent_t> ev;      // pairs: 2*slot = start, 2*slot+1 = stop
    std::vector<int> cat;            // category of each used slot
    size_t used = 0;
};

namespace {
// free_dit_tune: kTuneRounds runs of kTuneRun forwards per schedule, the eligible schedules in turn (1, 2, 3, 1, 2,
// 3, ...); the first forward of a run is not timed (the schedules leave clocks and caches in different states), the
// others are timed together, and the first run of each schedule is not counted
constexpr int kMaxParts = 3;                  // streams the block stack of one forward may be cut over
constexpr int kTuneRounds = 3, kTuneRun = 4;
constexpr int kTuneTrials = kTuneRounds * kMaxParts;      // event pairs the handle keeps for it
constexpr int kTuneSlots = 8;                 // batch sizes a handle remembers a tuned schedule for
constexpr int64_t kMinSplitRows = 2048;       // token rows per part below which the split does not pay
// token rows from which the folded-LayerNorm path is taken by default: its GEMMs use the two large tiles only
constexpr int64_t kMinFoldRows = 4096;
constexpr size_t kMaxProfSlots = 8192;
}  // namespace

ProfScope::ProfScope(Profiler* p, int c, hipStream_t s) : prof(p), slot(-1), stream(s) {
    if (!p || !p->on || p->used >= kMaxProfSlots) return;
    const size_t k = p->used;
    while (p->ev.size() < 2 * (k + 1)) {
        hipEvent_t e;
        if (!hip_ok(hipEventCreate(&e))) return;
        p->ev.push_back(e);
    }
    if (!hip_ok(hipEventRecord(p->ev[2 * k], s))) return;
    if (p->cat.size() <= k) p->cat.resize(k + 1);
    p->cat[k] = c;
    p->used = k + 1;
    slot = static_cast<int>(k);
}

ProfScope::~ProfScope() {
    if (slot >= 0) (void)hip_ok(hipEventRecord(prof->ev[2 * slot + 1], stream));
}

namespace {

constexpr size_t kAlign = 256;
inline size_t align_up(size_t v) { return (v + kAlign - 1) / kAlign * kAlign; }

struct Dims {
    int32_t C, H, W, p, D, depth, heads, dh, F, classes, c_out, tfreq, mode;
    int32_t gh, gw, ntok, P;
    int64_t d;            // latent size C*H*W
    int32_t mod_rows;     // depth*6D + 2D
};

bool make_dims(const free_dit_config* c, Dims* o) {
    if (!c) return false;
    if (c->in_ch < 1 || c->lat_h < 1 || c->lat_w < 1 || c->patch < 1 || c->hidden < 8 || c->depth < 0 ||
        c->heads < 1 || c->mlp_hidden < 8 || c->num_classes < 1 || c->t_freq_dim < 2)
        return false;
    if (c->lat_h % c->patch || c->lat_w % c->patch) return false;
    if (c->hidden % c->heads || c->hidden % 8 || c->mlp_hidden % 8 || c->t_freq_dim % 2) return false;
    if (c->mode != FREE_FP32 && c->mode != FREE_BF16) return false;
    const int dh = c->hidden / c->heads;
    if (dh > 128) return false;
    if (c->mode == FREE_BF16 && dh % 8) return false;
    o->C = c->in_ch; o->H = c->lat_h; o->W = c->lat_w; o->p = c->patch; o->D = c->hidden;
    o->depth = c->depth; o->heads = c->heads; o->dh = dh; o->F = c->mlp_hidden;
    o->classes = c->num_classes; o->c_out = c->in_ch * (c->learn_sigma ? 2 : 1);
    o->tfreq = c->t_freq_dim; o->mode = c->mode;
    o->gh = c->lat_h / c->patch; o->gw = c->lat_w / c->patch; o->ntok = o->gh * o->gw;
    o->P = c->patch * c->patch * o->c_out;
    o->d = static_cast<int64_t>(c->in_ch) * c->lat_h * c->lat_w;
    o->mod_rows = c->depth * 6 * c->hidden + 2 * c->hidden;
    return true;
}

// Workspace carve-up for a forward on B packed states (offsets in bytes).
struct WsLayout {
    size_t cond_h, sc, mod, tpack, ypack, xres, xn, qkv, att, hmid, eps, mtarget, vpart, vpart_bytes, fold, stats, total;
};

// floats per sample of the fold vectors: c1 of every block's QKV and MLP-1 rows, then c0 of the same
int64_t fold_stride(const Dims& d) { return 2 * static_cast<int64_t>(d.depth) * (3 * d.D + d.F); }

WsLayout make_layout(const Dims& d, int32_t B) {
    WsLayout L;
    const size_t es = d.mode == FREE_BF16 ? 2 : 4;
    const size_t M = static_cast<size_t>(B) * d.ntok;
    size_t off = 0;
    auto take = [&](size_t bytes) { size_t o = off; off += align_up(bytes); return o; };
    L.cond_h = take(static_cast<size_t>(B) * (d.tfreq + d.D) * 4);
    L.sc = take(static_cast<size_t>(B) * d.D * 4);
    L.mod = take(static_cast<size_t>(B) * d.mod_rows * 4);
    L.tpack = take(static_cast<size_t>(B) * 4);
    L.ypack = take(static_cast<size_t>(B) * 4);
    L.xres = take(M * d.D * 4);
    L.xn = take(M * d.D * es);
    L.qkv = take(M * 3 * d.D * es);
    L.att = take(M * d.D * es);
    L.hmid = take(M * d.F * es);
    L.eps = take(static_cast<size_t>(B) * d.c_out * d.H * d.W * 4);
    L.mtarget = take(static_cast<size_t>(B) * d.d * 4);
    // verification of the round's drafts: K = B without guidance, K = B / 2 with it
    L.vpart_bytes = std::max(verify_workspace_bytes(1, B, d.d), verify_workspace_bytes(1, (B + 1) / 2, d.d));
    L.vpart = take(L.vpart_bytes);
    // folded LayerNorm (bf16): c1 | c0 of both folded layers of every block per sample, partial row sums per token row
    L.fold = take(d.mode == FREE_BF16 ? static_cast<size_t>(B) * fold_stride(d) * 4 : 0);
    L.stats = take(d.mode == FREE_BF16 ? M * ((d.D + kLnSlotCols - 1) / kLnSlotCols) * 2 * 4 : 0);
    L.total = off;
    return L;
}

}  // namespace
}  // namespace freemi

using namespace freemi;

struct free_dit_s {
    free_dit_config cfg;
    Dims dims;
    std::vector<const void*> w;         // borrowed device pointers, in ABI order
    // device-side tables owned by the handle
    void* dev_block = nullptr;
    const void* const* ada_w_tab = nullptr;
    const float* const* ada_b_tab = nullptr;
    const int32_t* ada_row_start = nullptr;
    const float* pos = nullptr;
    // folded LayerNorm: device tables of the 2 * depth weight / bias pointers (block l: QKV, MLP-1)
    const void* const* fold_w_tab = nullptr;
    const float* const* fold_b_tab = nullptr;
    int32_t ln_fold = FREE_LN_FOLD_AUTO;
    int device = 0;
    // side streams (default priority): the parts of a packed batch after the first run on them, concurrently with
    // the first part on the caller's stream
    hipStream_t side[kMaxParts - 1] = {};
    hipEvent_t ev_fork = nullptr;
    hipEvent_t ev_join[kMaxParts - 1] = {};
    // one more side stream (default priority): the fold vectors of the folded LayerNorms are computed on it while
    // the first block runs up to its out-projection; ev_fold_go orders it after the modulation, the block
    // stack waits for ev_fold_done before the first GEMM that reads the vectors
    hipStream_t fold_stream = nullptr;
    hipEvent_t ev_fold_go = nullptr, ev_fold_done = nullptr;
    // Schedule of the block stack: forced (1, 2 or 3 streams) for every batch size, or 0 = per batch size what
    // free_dit_tune measured, one stream where nothing was measured.
    int32_t forced_streams = 0;
    struct Tuned { int32_t batch = 0, choice = 0; } tuned[kTuneSlots];
    int32_t tuned_next = 0;                   // slot the next new batch size overwrites
    hipEvent_t tune_ev[kTuneTrials][2] = {};  // [trial][start, stop], created on first use by free_dit_tune
    Profiler prof;

    int32_t streams_for(int32_t B) const {
        if (forced_streams) return forced_streams;
        for (const Tuned& t : tuned)
            if (t.batch == B && t.choice) return t.choice;
        return 1;
    }
    // a batch may be cut into `parts` when every part keeps enough token rows to fill the chip
    bool parts_eligible(int32_t B, int32_t parts) const {
        return parts == 1 || (B >= parts && static_cast<int64_t>(B / parts) * dims.ntok >= kMinSplitRows);
    }
    // what a forward on B samples does: the wanted schedule, or the next smaller one that B allows
    int32_t parts_for(int32_t B) const {
        int32_t n = streams_for(B);
        while (n > 1 && !parts_eligible(B, n)) --n;
        return n;
    }

    const void* blk(int l, int which) const { return w[7 + 10 * l + which]; }
    const void* fin(int which) const { return w[7 + 10 * dims.depth + which]; }
    // shapes the folded-LayerNorm path covers, and whether a forward on B samples takes it
    bool ln_fold_covers() const {
        const Dims& d = dims;
        return d.mode == FREE_BF16 && mfma_ln_fold_supported(d.ntok, d.D, d.ntok) && ln_fold_supported(d.D, 3 * d.D, d.F) &&
               d.D % 64 == 0 && d.F % 64 == 0 && d.depth >= 1;
    }
    bool ln_fold_for(int32_t B) const {
        if (ln_fold == FREE_LN_FOLD_OFF || !ln_fold_covers()) return false;
        return ln_fold == FREE_LN_FOLD_REQUIRE || static_cast<int64_t>(B) * dims.ntok >= kMinFoldRows;
    }
};

struct free_drafter_s {
    free_dit_t target = nullptr;
    int depth = 1;
    int32_t mod_rows = 0;                // depth*6D + 2D
    std::vector<const void*> w;          // borrowed device pointers, in ABI order
    void* dev_block = nullptr;           // adaLN pointer tables, row starts, a vector of ones
    const void* const* ada_w_tab = nullptr;
    const float* const* ada_b_tab = nullptr;
    const int32_t* ada_row_start = nullptr;
    const float* ones = nullptr;         // [D]

    const void* const* blkw() const { return w.data() + 2; }
    const void* fin(int which) const { return w[2 + 10 * depth + which]; }
};

namespace {

enum { W_PATCH_W = 0, W_PATCH_B, W_T_W1, W_T_B1, W_T_W2, W_T_B2, W_Y_TABLE };
enum { B_ADA_W = 0, B_ADA_B, B_QKV_W, B_QKV_B, B_PROJ_W, B_PROJ_B, B_FC1_W, B_FC1_B, B_FC2_W, B_FC2_B };
enum { F_ADA_W = 0, F_ADA_B, F_W, F_B };

int32_t linear_dispatch(const Dims& d, const void* A, const void* W, const float* bias, int32_t M, int32_t N,
                        int32_t K, int32_t epi, void* out, float* resid, RowVec gate, hipStream_t s, int cu_share = 1,
                        const LnFold* ln = nullptr) {
    if (d.mode == FREE_BF16 && mfma_linear_supported(M, N, K))
        return launch_linear_mfma(static_cast<const bf16_t*>(A), static_cast<const bf16_t*>(W), bias, M, N, K, epi,
                                  static_cast<bf16_t*>(out), resid, gate, s, cu_share, ln);
    if (ln != nullptr) return FREE_ERR_SHAPE;                 // the folded-LayerNorm epilogues exist on that path only
    if (d.mode == FREE_FP32 && mfma_linear_f32_supported(M, N, K))
        return launch_linear_mfma_f32(static_cast<const float*>(A), static_cast<const float*>(W), bias, M, N, K, epi,
                                      static_cast<float*>(out), resid, gate, s, cu_share);
    return launch_linear_simple(A, W, bias, M, N, K, d.mode, epi, out, resid, gate, s);
}

int32_t attention_dispatch(const Dims& d, const void* qkv, int32_t B, void* out, hipStream_t s) {
    if (d.mode == FREE_BF16 && mfma_attention_supported(d.ntok, d.dh))
        return launch_attention_mfma(static_cast<const bf16_t*>(qkv), B, d.ntok, d.heads, d.dh,
                                     static_cast<bf16_t*>(out), s);
    if (d.mode == FREE_FP32 && mfma_attention_f32_supported(d.ntok, d.dh))
        return launch_attention_mfma_f32(static_cast<const float*>(qkv), B, d.ntok, d.heads, d.dh,
                                         static_cast<float*>(out), s);
    return launch_attention_simple(qkv, B, d.ntok, d.heads, d.dh, d.mode, out, s);
}

#define FREE_TRY(expr)                      \
    do {                                    \
        int32_t st__ = (expr);              \
        if (st__ != FREE_OK) return st__;   \
    } while (0)

// The packed forward.  x_mod: packed state b reads latent b % x_mod.
// Activation buffers of a forward on B samples (token rows are sample-major).
struct ActBufs {
    float* xres;   // residual stream [B*ntok, D] fp32
    void* xn;      // LN output       [B*ntok, D]   compute type
    void* qkv;     //                 [B*ntok, 3D]
    void* att;     //                 [B*ntok, D]
    void* hmid;    //                 [B*ntok, F]
};

// `nblk` adaLN-Zero blocks on samples [b0, b0 + nb) of a batch.  blkw holds 10 pointers per block
// (B_* order); block l's six modulation vectors of sample b are mod[b * mod_rows + l * 6D ..].
// cu_share: number of such stacks running side by side on different streams (tile choice of the GEMMs).
// fold_ready (nullable): event after which fold->vec is complete; waited for on `s` before the first use.
// fold (nullable): the LayerNorms are folded into the GEMMs around them (all but the first one of block 0, whose
// input no GEMM of this stack produced): fold->vec holds the fold vectors of all samples of the batch, fold->stats the
// partial row sums of all token rows.
struct FoldBufs {
    const float* vec;     // [B, stride]
    int64_t stride;
    float* stats;         // [B*ntok, slots, 2]
    int32_t slots;
};
int32_t run_block_stack(const Dims& d, const void* const* blkw, int nblk, const float* mod, int32_t mod_rows,
                        const ActBufs& a, int b0, int nb, hipStream_t s, Profiler* pf, int cu_share = 1,
                        const FoldBufs* fold = nullptr, hipEvent_t fold_ready = nullptr) {
    const size_t esz = d.mode == FREE_BF16 ? 2 : 4;
    const int32_t M = nb * d.ntok;
    const int64_t r0 = static_cast<int64_t>(b0) * d.ntok;
    float* xres_h = a.xres + r0 * d.D;
    void* xn_h = static_cast<char*>(a.xn) + r0 * d.D * esz;
    void* qkv_h = static_cast<char*>(a.qkv) + r0 * 3 * d.D * esz;
    void* att_h = static_cast<char*>(a.att) + r0 * d.D * esz;
    void* hmid_h = static_cast<char*>(a.hmid) + r0 * d.F * esz;
    auto vec = [&](int l, int which) {
        RowVec r;
        r.base = mod + static_cast<int64_t>(b0) * mod_rows + static_cast<int64_t>(l) * 6 * d.D +
                 static_cast<int64_t>(which) * d.D;
        r.stride = mod_rows;
        r.rows_per_sample = d.ntok;
        return r;
    };
    auto W = [&](int l, int which) { return blkw[10 * l + which]; };
    auto Bv = [&](int l, int which) { return static_cast<const float*>(blkw[10 * l + which]); };
    // folded LayerNorm: consumer side (which = 0: QKV, 1: MLP-1) and producer side (scale of the next LayerNorm)
    const int64_t fold_rows = static_cast<int64_t>(nblk) * (3 * d.D + d.F);
    auto consumer = [&](int l, int which) {
        LnFold f;
        f.stats = fold->stats + r0 * fold->slots * 2;
        f.slots = fold->slots;
        f.c1 = fold->vec + static_cast<int64_t>(b0) * fold->stride + static_cast<int64_t>(l) * (3 * d.D + d.F) + (which ? 3 * d.D : 0);
        f.c0 = f.c1 + fold_rows;
        f.fold_stride = fold->stride;
        f.rows_per_sample = d.ntok;
        f.inv_width = 1.0f / static_cast<float>(d.D);
        return f;
    };
    auto producer = [&](const RowVec& scale_next) {
        LnFold f;
        f.scale_next = scale_next.base;
        f.z = xn_h;
        f.stats = fold->stats + r0 * fold->slots * 2;
        f.slots = fold->slots;
        return f;
    };
    for (int l = 0; l < nblk; ++l) {
        // x += gate1 * Proj(Attn(LN(x)(1+scale1)+shift1))
        if (fold && l > 0) {
            ProfScope prof(pf, PROF_GEMM_QKV, s);
            const LnFold f = consumer(l, 0);
            FREE_TRY(linear_dispatch(d, xn_h, W(l, B_QKV_W), Bv(l, B_QKV_B), M, 3 * d.D, d.D, FREE_EPI_LN_BIAS, qkv_h,
                                     nullptr, RowVec{nullptr, 0, 1}, s, cu_share, &f));
        } else {
            {
                ProfScope prof(pf, PROF_LN_MOD, s);
                FREE_TRY(launch_ln_modulate(xres_h, vec(l, 0), vec(l, 1), M, d.D, d.mode, xn_h, s));
            }
            ProfScope prof(pf, PROF_GEMM_QKV, s);
            FREE_TRY(linear_dispatch(d, xn_h, W(l, B_QKV_W), Bv(l, B_QKV_B), M, 3 * d.D, d.D, FREE_EPI_BIAS, qkv_h,
                                     nullptr, RowVec{nullptr, 0, 1}, s, cu_share));
        }
        {
            ProfScope prof(pf, PROF_ATTN, s);
            FREE_TRY(attention_dispatch(d, qkv_h, nb, att_h, s));
        }
        if (fold) {
            // the out-projection also prepares the second LayerNorm: z = x (1 + scale2), partial row sums
            ProfScope prof(pf, PROF_GEMM_PROJ, s);
            const LnFold f = producer(vec(l, 4));
            FREE_TRY(linear_dispatch(d, att_h, W(l, B_PROJ_W), Bv(l, B_PROJ_B), M, d.D, d.D, FREE_EPI_GATE_RESID_PREP,
                                     nullptr, xres_h, vec(l, 2), s, cu_share, &f));
        } else {
            ProfScope prof(pf, PROF_GEMM_PROJ, s);
            FREE_TRY(linear_dispatch(d, att_h, W(l, B_PROJ_W), Bv(l, B_PROJ_B), M, d.D, d.D, FREE_EPI_GATE_RESID,
                                     nullptr, xres_h, vec(l, 2), s, cu_share));
        }
        // x += gate2 * FC2(gelu(FC1(LN(x)(1+scale2)+shift2)))
        if (fold) {
            // (the first GEMM that reads the fold vectors: they may still be on their way on another stream)
            if (l == 0 && fold_ready && !hip_ok(hipStreamWaitEvent(s, fold_ready, 0))) return FREE_ERR_HIP;
            ProfScope prof(pf, PROF_GEMM_FC1, s);
            const LnFold f = consumer(l, 1);
            FREE_TRY(linear_dispatch(d, xn_h, W(l, B_FC1_W), Bv(l, B_FC1_B), M, d.F, d.D, FREE_EPI_LN_BIAS_GELU, hmid_h,
                                     nullptr, RowVec{nullptr, 0, 1}, s, cu_share, &f));
        } else {
            {
                ProfScope prof(pf, PROF_LN_MOD, s);
                FREE_TRY(launch_ln_modulate(xres_h, vec(l, 3), vec(l, 4), M, d.D, d.mode, xn_h, s));
            }
            ProfScope prof(pf, PROF_GEMM_FC1, s);
            FREE_TRY(linear_dispatch(d, xn_h, W(l, B_FC1_W), Bv(l, B_FC1_B), M, d.F, d.D, FREE_EPI_BIAS_GELU, hmid_h,
                                     nullptr, RowVec{nullptr, 0, 1}, s, cu_share));
        }
        if (fold && l + 1 < nblk) {
            // the MLP's second layer prepares the first LayerNorm of the next block
            ProfScope prof(pf, PROF_GEMM_FC2, s);
            const LnFold f = producer(vec(l + 1, 1));
            FREE_TRY(linear_dispatch(d, hmid_h, W(l, B_FC2_W), Bv(l, B_FC2_B), M, d.D, d.F, FREE_EPI_GATE_RESID_PREP,
                                     nullptr, xres_h, vec(l, 5), s, cu_share, &f));
        } else {
            ProfScope prof(pf, PROF_GEMM_FC2, s);
            FREE_TRY(linear_dispatch(d, hmid_h, W(l, B_FC2_W), Bv(l, B_FC2_B), M, d.D, d.F, FREE_EPI_GATE_RESID,
                                     nullptr, xres_h, vec(l, 5), s, cu_share));
        }
    }
    return FREE_OK;
}

int32_t forward_impl(free_dit_t h, const float* x, int32_t x_mod, const int32_t* t, const int32_t* y, int32_t B,
                     float* eps_out, float* top_feat, char* ws, hipStream_t s) {
    const Dims& d = h->dims;
    const WsLayout L = make_layout(d, B);
    const int32_t M = B * d.ntok;
    float* cond_h = reinterpret_cast<float*>(ws + L.cond_h);
    float* sc = reinterpret_cast<float*>(ws + L.sc);
    float* mod = reinterpret_cast<float*>(ws + L.mod);
    float* xres = reinterpret_cast<float*>(ws + L.xres);
    void* xn = ws + L.xn;
    void* qkv = ws + L.qkv;
    void* att = ws + L.att;
    void* hmid = ws + L.hmid;

    {
    ProfScope prof(&h->prof, PROF_COND, s);
    FREE_TRY(launch_conditioning(t, y, B, d.D, d.tfreq, static_cast<const float*>(h->w[W_T_W1]),
                                 static_cast<const float*>(h->w[W_T_B1]), static_cast<const float*>(h->w[W_T_W2]),
                                 static_cast<const float*>(h->w[W_T_B2]),
                                 static_cast<const float*>(h->w[W_Y_TABLE]), cond_h, sc, s));
    }
    {
    ProfScope prof(&h->prof, PROF_ADALN, s);
    if (adaln_mfma_supported(d.D, d.mod_rows))
        FREE_TRY(launch_adaln_mfma(sc, B, d.D, h->ada_w_tab, h->ada_b_tab, h->ada_row_start, d.depth + 1,
                                   d.mod_rows, d.mode, mod, s));
    else
        FREE_TRY(launch_adaln(sc, B, d.D, h->ada_w_tab, h->ada_b_tab, h->ada_row_start, d.depth + 1, d.mod_rows,
                              d.mode, mod, s));
    }
    const bool folded = h->ln_fold_for(B);
    if (h->ln_fold == FREE_LN_FOLD_REQUIRE && !folded) return FREE_ERR_SHAPE;
    FoldBufs fb{reinterpret_cast<const float*>(ws + L.fold), fold_stride(d), reinterpret_cast<float*>(ws + L.stats),
                d.D / kLnSlotCols};
    hipEvent_t fold_ready = nullptr;
    if (folded && h->prof.on) {
        ProfScope prof(&h->prof, PROF_ADALN, s);
        FREE_TRY(launch_ln_fold(mod, B, d.D, d.mod_rows, d.depth, 3 * d.D, d.F, h->fold_w_tab, h->fold_b_tab,
                                reinterpret_cast<float*>(ws + L.fold), fb.stride, s));
    } else if (folded) {
        // bandwidth-bound and needed only from the first block's MLP on: beside the main stream, so that it
        // fills the compute units the first block's kernels leave idle
        if (!hip_ok(hipEventRecord(h->ev_fold_go, s))) return FREE_ERR_HIP;
        if (!hip_ok(hipStreamWaitEvent(h->fold_stream, h->ev_fold_go, 0))) return FREE_ERR_HIP;
        FREE_TRY(launch_ln_fold(mod, B, d.D, d.mod_rows, d.depth, 3 * d.D, d.F, h->fold_w_tab, h->fold_b_tab,
                                reinterpret_cast<float*>(ws + L.fold), fb.stride, h->fold_stream));
        if (!hip_ok(hipEventRecord(h->ev_fold_done, h->fold_stream))) return FREE_ERR_HIP;
        fold_ready = h->ev_fold_done;
    }
    {
    ProfScope prof(&h->prof, PROF_PATCH, s);
    FREE_TRY(launch_patch_embed(x, x_mod, B, d.C, d.H, d.W, d.p, d.D, static_cast<const float*>(h->w[W_PATCH_W]),
                                static_cast<const float*>(h->w[W_PATCH_B]), h->pos, xres, s));
    }
    const ActBufs act{xres, xn, qkv, att, hmid};
    const void* const* blkw = h->w.data() + 7;
    auto run_blocks = [&](int b0, int nb, hipStream_t st, int cu_share) -> int32_t {
        return run_block_stack(d, blkw, d.depth, mod, d.mod_rows, act, b0, nb, st, &h->prof, cu_share,
                               folded ? &fb : nullptr, fold_ready);
    };
    // The samples of a packed batch are independent through all blocks, so the batch can be cut in two halves
    // or three thirds that run on as many streams forked from (and joined back into) the caller's stream: while
    // one part is in a bandwidth-bound phase (layer norm, the residual read-modify-write at the end
    // of a GEMM, the first and last wave of tiles) the other parts' matrix kernels fill the idle
    // compute units.  Which schedule is faster differs between machines of the same type by a few
    // per cent either way, so one stream is the default and free_dit_tune measures on request.
    // All give the same numbers.  Per-kernel profiling needs serial execution, and small batches are
    // launch bound, so both keep the single stream.  Nothing here waits on the host.
    const int parts = h->prof.on ? 1 : h->parts_for(B);
    if (parts > 1) {
        // the first part stays on the caller's stream, the others go to side streams (with the stream of the fold
        // vectors that makes at most four streams, the number of hardware queues a process has by default)
        if (!hip_ok(hipEventRecord(h->ev_fork, s))) return FREE_ERR_HIP;
        auto bounds = [&](int i, int* b0, int* b1) {
            *b0 = static_cast<int>(static_cast<int64_t>(i) * B / parts);
            *b1 = static_cast<int>(static_cast<int64_t>(i + 1) * B / parts);
        };
        int b0, b1;
        for (int i = 1; i < parts; ++i) {
            bounds(i, &b0, &b1);
            if (!hip_ok(hipStreamWaitEvent(h->side[i - 1], h->ev_fork, 0))) return FREE_ERR_HIP;
            FREE_TRY(run_blocks(b0, b1 - b0, h->side[i - 1], parts));
            if (!hip_ok(hipEventRecord(h->ev_join[i - 1], h->side[i - 1]))) return FREE_ERR_HIP;
        }
        bounds(0, &b0, &b1);
        FREE_TRY(run_blocks(b0, b1 - b0, s, parts));
        for (int i = 1; i < parts; ++i)
            if (!hip_ok(hipStreamWaitEvent(s, h->ev_join[i - 1], 0))) return FREE_ERR_HIP;
    } else {
        FREE_TRY(run_blocks(0, B, s, 1));
    }
    if (top_feat) {
        if (!hip_ok(hipMemcpyAsync(top_feat, xres, static_cast<size_t>(M) * d.D * 4, hipMemcpyDeviceToDevice, s)))
            return FREE_ERR_HIP;
    }
    RowVec fsh{mod + static_cast<int64_t>(d.depth) * 6 * d.D, d.mod_rows, d.ntok};
    RowVec fsc{mod + static_cast<int64_t>(d.depth) * 6 * d.D + d.D, d.mod_rows, d.ntok};
    ProfScope prof(&h->prof, PROF_FINAL, s);
    FREE_TRY(launch_final_layer(xres, fsh, fsc, B, d.gh, d.gw, d.p, d.c_out, d.D, h->fin(F_W),
                                static_cast<const float*>(h->fin(F_B)), d.mode, eps_out, s));
    return FREE_OK;
}

int32_t check_ws(const void* ws, size_t ws_bytes, size_t need) {
    if (!ws || (reinterpret_cast<uintptr_t>(ws) & (kAlign - 1)) || ws_bytes < need) return FREE_ERR_WORKSPACE;
    return FREE_OK;
}

}  // namespace

extern "C" {

const char* free_version(void) { return "free-mi355x 0.1 (gfx950)"; }

const char* free_status_string(int32_t st) {
    switch (st) {
        case FREE_OK: return "ok";
        case FREE_ERR_NULL: return "a required pointer is NULL";
        case FREE_ERR_SHAPE: return "inconsistent or unsupported sizes";
        case FREE_ERR_RANGE: return "scalar argument out of range";
        case FREE_ERR_DTYPE: return "unknown compute mode";
        case FREE_ERR_WORKSPACE: return "workspace missing, misaligned or too small";
        case FREE_ERR_HIP: return "HIP runtime error";
        case FREE_ERR_LIMIT: return "problem larger than a fixed built-in limit";
        default: return "unknown status";
    }
}

int32_t free_last_hip_error(void) { return g_last_hip_error; }

int32_t free_dit_set_streams(free_dit_t h, int32_t n) {
    if (!h) return FREE_ERR_NULL;
    if (n < 0 || n > kMaxParts) return FREE_ERR_RANGE;
    h->forced_streams = n;
    return FREE_OK;
}

int32_t free_dit_set_ln_fold(free_dit_t h, int32_t mode) {
    if (!h) return FREE_ERR_NULL;
    if (mode != FREE_LN_FOLD_OFF && mode != FREE_LN_FOLD_AUTO && mode != FREE_LN_FOLD_REQUIRE) return FREE_ERR_RANGE;
    if (mode == FREE_LN_FOLD_REQUIRE && !h->ln_fold_covers()) return FREE_ERR_SHAPE;
    h->ln_fold = mode;
    return FREE_OK;
}

int32_t free_dit_ln_fold_active(free_dit_t h, int32_t B) {
    if (!h) return FREE_ERR_NULL;
    if (B < 1) return FREE_ERR_SHAPE;
    return h->ln_fold_for(B) ? 1 : 0;
}

int32_t free_dit_stream_choice(free_dit_t h, int32_t B) {
    if (!h) return FREE_ERR_NULL;
    if (B < 1) return FREE_ERR_SHAPE;
    return h->parts_for(B);
}

int32_t free_profile_begin(free_dit_t h) {
    if (!h) return FREE_ERR_NULL;
    h->prof.used = 0;
    h->prof.on = true;
    return FREE_OK;
}

int32_t free_profile_end(free_dit_t h, float* ms, int32_t* launches) {
    if (!h) return FREE_ERR_NULL;
    Profiler& pf = h->prof;
    pf.on = false;
    if (!ms || !launches) return FREE_ERR_NULL;
    for (int c = 0; c < FREE_PROF_NCAT; ++c) { ms[c] = 0.f; launches[c] = 0; }
    for (size_t k = 0; k < pf.used; ++k) {
        if (!hip_ok(hipEventSynchronize(pf.ev[2 * k + 1]))) return FREE_ERR_HIP;
        float t = 0.f;
        if (!hip_ok(hipEventElapsedTime(&t, pf.ev[2 * k], pf.ev[2 * k + 1]))) return FREE_ERR_HIP;
        ms[pf.cat[k]] += t;
        launches[pf.cat[k]] += 1;
    }
    pf.used = 0;
    return FREE_OK;
}

int32_t free_validate_inputs(const int32_t* t, int64_t n_t, int32_t T, const float* sigma, const float* u,
                             const float* lambda, int64_t n, uint32_t* violations, void* stream) {
    if (n_t < 0 || n < 0 || (t && T < 1)) return FREE_ERR_SHAPE;
    if (n_t > (1ll << 38) || n > (1ll << 38)) return FREE_ERR_SHAPE;
    return run_validate(t, t ? n_t : 0, T, sigma, u, lambda, (sigma || u || lambda) ? n : 0, violations,
                        static_cast<hipStream_t>(stream));
}

int32_t free_mfma_ceiling(int32_t iters, double* tflops, double* mhz, void* stream) {
    if (!tflops || !mhz) return FREE_ERR_NULL;
    if (iters < 1 || iters > (1 << 24)) return FREE_ERR_RANGE;
    return run_mfma_ceiling(iters, tflops, mhz, static_cast<hipStream_t>(stream));
}

const char* free_profile_category_name(int32_t c) {
    static const char* names[FREE_PROF_NCAT] = {"conditioning", "adaln", "patch_embed", "ln_modulate", "gemm_qkv",
                                                "attention", "gemm_proj", "gemm_fc1", "gemm_fc2", "final_layer",
                                                "eps_to_mean", "verify"};
    return (c >= 0 && c < FREE_PROF_NCAT) ? names[c] : "unknown";
}

int32_t free_ddpm_schedule(int32_t T, double beta_start, double beta_end, double* coef_x, double* coef_eps,
                           double* sigma) {
    if (T < 2) return FREE_ERR_SHAPE;
    if (!(beta_start > 0.0) || !(beta_end >= beta_start) || !(beta_end < 1.0)) return FREE_ERR_RANGE;
    double abar = 1.0, abar_prev = 1.0, sigma1 = 0.0;
    for (int i = 0; i < T; ++i) {
        const double beta = beta_start + (beta_end - beta_start) * static_cast<double>(i) / (T - 1);
        const double alpha = 1.0 - beta;
        abar_prev = abar;
        abar *= alpha;
        if (coef_x) coef_x[i] = 1.0 / std::sqrt(alpha);
        if (coef_eps) coef_eps[i] = -beta / (std::sqrt(1.0 - abar) * std::sqrt(alpha));
        const double var = beta * (1.0 - abar_prev) / (1.0 - abar);      // posterior variance
        if (sigma) sigma[i] = std::sqrt(var);
        if (i == 1) sigma1 = std::sqrt(var);
    }
    if (sigma) sigma[0] = sigma1;          // index 0 has zero variance: clipped to index 1
    return FREE_OK;
}

int32_t free_sde_schedule(int32_t T, double beta_start, double beta_end, double stochasticity, double* coef_x,
                          double* coef_eps, double* sigma) {
    if (T < 2) return FREE_ERR_SHAPE;
    if (!(beta_start > 0.0) || !(beta_end >= beta_start) || !(beta_end < 1.0) || !(stochasticity >= 0.0))
        return FREE_ERR_RANGE;
    double abar = 1.0;
    for (int i = 0; i < T; ++i) {
        const double beta = beta_start + (beta_end - beta_start) * static_cast<double>(i) / (T - 1);
        abar *= 1.0 - beta;
        if (coef_x) coef_x[i] = 1.0 + 0.5 * beta;
        if (coef_eps) coef_eps[i] = -0.5 * (1.0 + stochasticity * stochasticity) * beta / std::sqrt(1.0 - abar);
        if (sigma) sigma[i] = stochasticity * std::sqrt(beta);
    }
    return FREE_OK;
}

int32_t free_weight_count(const free_dit_config* cfg) {
    Dims d;
    if (!make_dims(cfg, &d)) return FREE_ERR_SHAPE;
    return 7 + 10 * d.depth + 4;
}

int32_t free_dit_create(const free_dit_config* cfg, const void* const* weight_ptrs, int32_t n_ptrs,
                        free_dit_t* out) {
    if (!cfg || !weight_ptrs || !out) return FREE_ERR_NULL;
    if (cfg->mode != FREE_FP32 && cfg->mode != FREE_BF16) return FREE_ERR_DTYPE;
    Dims d;
    if (!make_dims(cfg, &d)) return FREE_ERR_SHAPE;
    if (n_ptrs != 7 + 10 * d.depth + 4) return FREE_ERR_SHAPE;
    for (int i = 0; i < n_ptrs; ++i) {
        if (!weight_ptrs[i]) return FREE_ERR_NULL;
        if (reinterpret_cast<uintptr_t>(weight_ptrs[i]) & 15u) return FREE_ERR_SHAPE;
    }
    free_dit_s* h = new (std::nothrow) free_dit_s();
    if (!h) return FREE_ERR_HIP;
    h->cfg = *cfg;
    h->dims = d;
    h->w.assign(weight_ptrs, weight_ptrs + n_ptrs);
    if (!hip_ok(hipGetDevice(&h->device))) { delete h; return FREE_ERR_HIP; }

    // device block: [w_tab (depth+1 ptrs) | b_tab (depth+1 ptrs) | row_start (depth+2 ints) | pos (ntok*D floats) |
    //                fold_w_tab (2 depth ptrs) | fold_b_tab (2 depth ptrs)]
    const int n_mats = d.depth + 1;
    const size_t off_w = 0;
    const size_t off_b = align_up(off_w + n_mats * sizeof(void*));
    const size_t off_r = align_up(off_b + n_mats * sizeof(void*));
    const size_t off_p = align_up(off_r + (n_mats + 1) * sizeof(int32_t));
    const size_t off_fw = align_up(off_p + static_cast<size_t>(d.ntok) * d.D * sizeof(float));
    const size_t off_fb = align_up(off_fw + 2 * d.depth * sizeof(void*));
    const size_t total = off_fb + 2 * d.depth * sizeof(void*);
    std::vector<char> host(total, 0);
    const void** wt = reinterpret_cast<const void**>(host.data() + off_w);
    const void** bt = reinterpret_cast<const void**>(host.data() + off_b);
    int32_t* rs = reinterpret_cast<int32_t*>(host.data() + off_r);
    for (int l = 0; l < d.depth; ++l) {
        wt[l] = h->blk(l, B_ADA_W);
        bt[l] = h->blk(l, B_ADA_B);
        rs[l] = l * 6 * d.D;
    }
    const void** fwt = reinterpret_cast<const void**>(host.data() + off_fw);
    const void** fbt = reinterpret_cast<const void**>(host.data() + off_fb);
    for (int l = 0; l < d.depth; ++l) {
        fwt[2 * l] = h->blk(l, B_QKV_W);
        fbt[2 * l] = h->blk(l, B_QKV_B);
        fwt[2 * l + 1] = h->blk(l, B_FC1_W);
        fbt[2 * l + 1] = h->blk(l, B_FC1_B);
    }
    wt[d.depth] = h->fin(F_ADA_W);
    bt[d.depth] = h->fin(F_ADA_B);
    rs[d.depth] = d.depth * 6 * d.D;
    rs[d.depth + 1] = d.mod_rows;
    // fixed 2-D sin-cos table: token (i, j) -> [sin(j w) | cos(j w) | sin(i w) | cos(i w)], w_k = 10000^(-k/(D/4))
    float* pos = reinterpret_cast<float*>(host.data() + off_p);
    const int q = d.D / 4;
    for (int i = 0; i < d.gh; ++i)
        for (int j = 0; j < d.gw; ++j) {
            float* row = pos + (static_cast<size_t>(i) * d.gw + j) * d.D;
            for (int k = 0; k < q; ++k) {
                const double w = std::pow(10000.0, -static_cast<double>(k) / q);
                row[k] = static_cast<float>(std::sin(j * w));
                row[q + k] = static_cast<float>(std::cos(j * w));
                row[2 * q + k] = static_cast<float>(std::sin(i * w));
                row[3 * q + k] = static_cast<float>(std::cos(i * w));
            }
        }
    if (!hip_ok(hipMalloc(&h->dev_block, total))) { delete h; return FREE_ERR_HIP; }
    if (!hip_ok(hipMemcpy(h->dev_block, host.data(), total, hipMemcpyHostToDevice))) {
        (void)hipFree(h->dev_block);
        delete h;
        return FREE_ERR_HIP;
    }
    char* db = static_cast<char*>(h->dev_block);
    h->ada_w_tab = reinterpret_cast<const void* const*>(db + off_w);
    h->ada_b_tab = reinterpret_cast<const float* const*>(db + off_b);
    h->ada_row_start = reinterpret_cast<const int32_t*>(db + off_r);
    h->pos = reinterpret_cast<const float*>(db + off_p);
    h->fold_w_tab = reinterpret_cast<const void* const*>(db + off_fw);
    h->fold_b_tab = reinterpret_cast<const float* const*>(db + off_fb);
    bool ok = hip_ok(hipEventCreateWithFlags(&h->ev_fork, hipEventDisableTiming));
    for (int i = 0; i < kMaxParts - 1 && ok; ++i)
        ok = hip_ok(hipStreamCreateWithFlags(&h->side[i], hipStreamNonBlocking)) &&
             hip_ok(hipEventCreateWithFlags(&h->ev_join[i], hipEventDisableTiming));
    ok = ok && hip_ok(hipStreamCreateWithFlags(&h->fold_stream, hipStreamNonBlocking)) &&
         hip_ok(hipEventCreateWithFlags(&h->ev_fold_go, hipEventDisableTiming)) &&
         hip_ok(hipEventCreateWithFlags(&h->ev_fold_done, hipEventDisableTiming));
    if (!ok) {
        (void)free_dit_destroy(h);
        return FREE_ERR_HIP;
    }
    *out = h;
    return FREE_OK;
}

int32_t free_dit_destroy(free_dit_t h) {
    if (!h) return FREE_ERR_NULL;
    int32_t st = FREE_OK;
    for (int i = 0; i < kMaxParts - 1; ++i) {
        if (h->side[i] && !hip_ok(hipStreamSynchronize(h->side[i]))) st = FREE_ERR_HIP;
        if (h->side[i] && !hip_ok(hipStreamDestroy(h->side[i]))) st = FREE_ERR_HIP;
        if (h->ev_join[i] && !hip_ok(hipEventDestroy(h->ev_join[i]))) st = FREE_ERR_HIP;
    }
    if (h->ev_fork && !hip_ok(hipEventDestroy(h->ev_fork))) st = FREE_ERR_HIP;
    if (h->fold_stream && !hip_ok(hipStreamSynchronize(h->fold_stream))) st = FREE_ERR_HIP;
    if (h->fold_stream && !hip_ok(hipStreamDestroy(h->fold_stream))) st = FREE_ERR_HIP;
    if (h->ev_fold_go && !hip_ok(hipEventDestroy(h->ev_fold_go))) st = FREE_ERR_HIP;
    if (h->ev_fold_done && !hip_ok(hipEventDestroy(h->ev_fold_done))) st = FREE_ERR_HIP;
    for (int i = 0; i < kTuneTrials; ++i)
        for (int j = 0; j < 2; ++j)
            if (h->tune_ev[i][j] && !hip_ok(hipEventDestroy(h->tune_ev[i][j]))) st = FREE_ERR_HIP;
    for (hipEvent_t e : h->prof.ev)
        if (!hip_ok(hipEventDestroy(e))) st = FREE_ERR_HIP;
    if (h->dev_block && !hip_ok(hipFree(h->dev_block))) st = FREE_ERR_HIP;
    delete h;
    return st;
}

size_t free_workspace_bytes(const free_dit_config* cfg, int32_t B) {
    Dims d;
    if (!make_dims(cfg, &d) || B < 1) return 0;
    return make_layout(d, B).total;
}

int32_t dit_forward_packed(free_dit_t h, const float* x, const int32_t* t, const int32_t* y, int32_t B,
                           float* eps_out, float* top_feat, void* workspace, size_t ws_bytes, void* stream) {
    if (!h || !x || !t || !y || !eps_out) return FREE_ERR_NULL;
    if (B < 1 || static_cast<int64_t>(B) * h->dims.ntok > INT32_MAX / 4) return FREE_ERR_SHAPE;
    FREE_TRY(check_ws(workspace, ws_bytes, make_layout(h->dims, B).total));
    return forward_impl(h, x, B, t, y, B, eps_out, top_feat, static_cast<char*>(workspace),
                        static_cast<hipStream_t>(stream));
}

int32_t free_dit_tune(free_dit_t h, const float* x, const int32_t* t, const int32_t* y, int32_t B, float* eps_out,
                      void* workspace, size_t ws_bytes, void* stream) {
    if (!h || !x || !t || !y || !eps_out) return FREE_ERR_NULL;
    if (B < 1 || static_cast<int64_t>(B) * h->dims.ntok > INT32_MAX / 4) return FREE_ERR_SHAPE;
    FREE_TRY(check_ws(workspace, ws_bytes, make_layout(h->dims, B).total));
    hipStream_t s = static_cast<hipStream_t>(stream);
    int32_t sched[kMaxParts];
    int ns = 0;
    for (int32_t n = 1; n <= kMaxParts; ++n)
        if (h->parts_eligible(B, n)) sched[ns++] = n;
    if (ns < 2) return FREE_OK;                         // such a batch never splits: nothing to measure
    const int groups = kTuneRounds * ns;
    for (int i = 0; i < groups; ++i)
        for (int j = 0; j < 2; ++j)
            if (!h->tune_ev[i][j] && !hip_ok(hipEventCreate(&h->tune_ev[i][j]))) return FREE_ERR_HIP;
    const int32_t forced_before = h->forced_streams;
    const bool prof_before = h->prof.on;
    h->prof.on = false;
    int32_t st = FREE_OK;
    for (int i = 0; i < groups && st == FREE_OK; ++i) {
        h->forced_streams = sched[i % ns];
        for (int r = 0; r < kTuneRun && st == FREE_OK; ++r) {
            if (r == 1 && !hip_ok(hipEventRecord(h->tune_ev[i][0], s))) st = FREE_ERR_HIP;
            if (st == FREE_OK) st = forward_impl(h, x, B, t, y, B, eps_out, nullptr, static_cast<char*>(workspace), s);
        }
        if (st == FREE_OK && !hip_ok(hipEventRecord(h->tune_ev[i][1], s))) st = FREE_ERR_HIP;
    }
    h->forced_streams = forced_before;
    h->prof.on = prof_before;
    if (st != FREE_OK) return st;
    // total time of the counted runs of each schedule; several streams must win by more than half a per cent
    float tot[kMaxParts] = {};
    for (int i = ns; i < groups; ++i) {
        float el = 0.f;
        if (!hip_ok(hipEventSynchronize(h->tune_ev[i][1])) ||
            !hip_ok(hipEventElapsedTime(&el, h->tune_ev[i][0], h->tune_ev[i][1])))
            return FREE_ERR_HIP;
        tot[i % ns] += el;
    }
    int best = 1;
    for (int k = 2; k < ns; ++k)
        if (tot[k] < tot[best]) best = k;
    const int32_t choice = tot[best] < 0.995f * tot[0] ? sched[best] : 1;
    int slot = -1;
    for (int i = 0; i < kTuneSlots; ++i)
        if (h->tuned[i].batch == B) slot = i;
    if (slot < 0) {
        slot = h->tuned_next;
        h->tuned_next = (h->tuned_next + 1) % kTuneSlots;
    }
    h->tuned[slot].batch = B;
    h->tuned[slot].choice = choice;
    return FREE_OK;
}

size_t spec_verify_workspace_bytes(int32_t n_traj, int32_t K, int64_t d) {
    if (K > FREE_MAX_DRAFTS) return 0;
    return verify_workspace_bytes(n_traj, K, d);
}

int32_t spec_verify(const float* m_target, const float* m_draft, const float* x_draft, const float* sigma,
                    const float* u, const float* lambda, int32_t n_traj, int32_t K, int64_t d, float* log_ratio,
                    uint8_t* accept, int32_t* n_accept, float* x_out, void* workspace, size_t ws_bytes,
                    void* stream) {
    if (!m_target || !m_draft || !x_draft || !sigma || !u || !log_ratio || !accept || !n_accept || !x_out)
        return FREE_ERR_NULL;
    if (n_traj < 0 || K < 1 || K > FREE_MAX_DRAFTS || d < 1) return FREE_ERR_SHAPE;
    if (n_traj == 0) return FREE_OK;
    VerifyArgs a{m_target, m_draft, x_draft, nullptr, sigma, u, lambda, n_traj, K, d,
                 log_ratio, accept, n_accept, x_out, nullptr};
    return launch_verify(a, workspace, ws_bytes, static_cast<hipStream_t>(stream));
}

int32_t spec_verify_diag(const float* m_target, const float* m_draft, const float* x_draft, const float* sigma_elem,
                         const float* u, const float* lambda, int32_t n_traj, int32_t K, int64_t d, float* log_ratio,
                         uint8_t* accept, int32_t* n_accept, float* x_out, void* workspace, size_t ws_bytes,
                         void* stream) {
    if (!m_target || !m_draft || !x_draft || !sigma_elem || !u || !log_ratio || !accept || !n_accept || !x_out)
        return FREE_ERR_NULL;
    if (n_traj < 0 || K < 1 || K > FREE_MAX_DRAFTS || d < 1) return FREE_ERR_SHAPE;
    if (n_traj == 0) return FREE_OK;
    VerifyArgs a{m_target, m_draft, x_draft, nullptr, nullptr, u, lambda, n_traj, K, d,
                 log_ratio, accept, n_accept, x_out, nullptr, sigma_elem};
    return launch_verify(a, workspace, ws_bytes, static_cast<hipStream_t>(stream));
}

int32_t spec_verify_static(const float* m_target, const float* m_draft, const float* x_draft, const float* sigma,
                           const float* u, const float* lambda, int32_t n_traj, int32_t K, int64_t d,
                           float* log_ratio, uint8_t* accept, int32_t* n_accept, float* x_out, void* stream) {
    if (!m_target || !m_draft || !x_draft || !sigma || !u || !log_ratio || !accept || !n_accept || !x_out)
        return FREE_ERR_NULL;
    if (n_traj < 0 || K < 1 || K > FREE_MAX_DRAFTS || d < 1) return FREE_ERR_SHAPE;
    if (n_traj == 0) return FREE_OK;
    if (verify_workspace_bytes(n_traj, K, d) > FREE_STATIC_SCRATCH_BYTES) return FREE_ERR_LIMIT;
    void* ws = nullptr;
    FREE_TRY(static_verify_scratch(&ws));
    VerifyArgs a{m_target, m_draft, x_draft, nullptr, sigma, u, lambda, n_traj, K, d,
                 log_ratio, accept, n_accept, x_out, nullptr};
    return launch_verify(a, ws, FREE_STATIC_SCRATCH_BYTES, static_cast<hipStream_t>(stream));
}

int32_t spec_verify_timed(const float* m_target, const float* m_draft, const float* x_draft, const float* sigma,
                          const float* u, const float* lambda, int32_t n_traj, int32_t K, int64_t d, float* log_ratio,
                          uint8_t* accept, int32_t* n_accept, float* x_out, void* workspace, size_t ws_bytes,
                          void* stream, float* stream_ms, float* finish_ms) {
    if (!m_target || !m_draft || !x_draft || !sigma || !u || !log_ratio || !accept || !n_accept || !x_out ||
        !stream_ms || !finish_ms)
        return FREE_ERR_NULL;
    if (n_traj < 1 || K < 1 || K > FREE_MAX_DRAFTS || d < 1) return FREE_ERR_SHAPE;
    hipStream_t s = static_cast<hipStream_t>(stream);
    hipEvent_t ev[4] = {nullptr, nullptr, nullptr, nullptr};
    int32_t st = FREE_OK;
    for (int i = 0; i < 4 && st == FREE_OK; ++i)
        if (!hip_ok(hipEventCreate(&ev[i]))) st = FREE_ERR_HIP;
    if (st == FREE_OK) {
        VerifyArgs a{m_target, m_draft, x_draft, nullptr, sigma, u, lambda, n_traj, K, d,
                     log_ratio, accept, n_accept, x_out, nullptr};
        st = launch_verify(a, workspace, ws_bytes, s, ev);
    }
    if (st == FREE_OK && (!hip_ok(hipEventSynchronize(ev[3])) || !hip_ok(hipEventElapsedTime(stream_ms, ev[0], ev[1])) ||
                          !hip_ok(hipEventElapsedTime(finish_ms, ev[2], ev[3]))))
        st = FREE_ERR_HIP;
    for (int i = 0; i < 4; ++i)
        if (ev[i]) (void)hipEventDestroy(ev[i]);
    return st;
}

int32_t spec_round(free_dit_t h, const float* x_states, const float* x_last, const float* m_draft,
                   const int32_t* t, int32_t y, float cfg_scale, const float* coef_x, const float* coef_eps,
                   const float* sigma, const float* u, const float* lambda, int32_t K, float* m_target_out,
                   float* log_ratio, uint8_t* accept, int32_t* n_accept, float* x_out, void* workspace,
                   size_t ws_bytes, void* stream) {
    if (!h || !x_states || !x_last || !m_draft || !t || !coef_x || !coef_eps || !sigma || !u || !log_ratio ||
        !accept || !n_accept || !x_out)
        return FREE_ERR_NULL;
    const Dims& d = h->dims;
    if (K < 1 || K > FREE_MAX_DRAFTS) return FREE_ERR_SHAPE;
    if (y < 0 || y > d.classes) return FREE_ERR_RANGE;
    if (!(cfg_scale == cfg_scale)) return FREE_ERR_RANGE;
    const int32_t dup = cfg_scale > 1.0f ? 2 : 1;
    const int32_t B = K * dup;
    const WsLayout L = make_layout(d, B);
    FREE_TRY(check_ws(workspace, ws_bytes, L.total));
    char* ws = static_cast<char*>(workspace);
    hipStream_t s = static_cast<hipStream_t>(stream);
    int32_t* tp = reinterpret_cast<int32_t*>(ws + L.tpack);
    int32_t* yp = reinterpret_cast<int32_t*>(ws + L.ypack);
    float* eps = reinterpret_cast<float*>(ws + L.eps);
    float* mt = m_target_out ? m_target_out : reinterpret_cast<float*>(ws + L.mtarget);
    FREE_TRY(launch_pack_cond(t, y, d.classes, K, dup, tp, yp, s));
    FREE_TRY(forward_impl(h, x_states, K, tp, yp, B, eps, nullptr, ws, s));
    {
        ProfScope prof(&h->prof, PROF_EPS2MEAN, s);
        FREE_TRY(launch_eps_to_mean(eps, x_states, coef_x, coef_eps, cfg_scale, K, d.C, d.c_out,
                                    static_cast<int64_t>(d.H) * d.W, mt, s));
    }
    VerifyArgs a{mt, m_draft, x_states, x_last, sigma, u, lambda, 1, K, d.d, log_ratio, accept, n_accept, x_out,
                 &h->prof};
    return launch_verify(a, ws + L.vpart, L.vpart_bytes, s);
}

int32_t free_op_linear(const void* A, const void* W, const float* bias, int32_t M, int32_t N, int32_t Kdim,
                       int32_t dtype, int32_t epilogue, void* out, float* resid, const float* gate,
                       int32_t gate_stride, int32_t rows_per_sample, void* stream) {
    if (!A || !W || !bias) return FREE_ERR_NULL;
    if (dtype != FREE_FP32 && dtype != FREE_BF16) return FREE_ERR_DTYPE;
    if (M < 1 || N < 1 || Kdim < 1) return FREE_ERR_SHAPE;
    if (epilogue == FREE_EPI_GATE_RESID) {
        if (!resid || !gate) return FREE_ERR_NULL;
        if (rows_per_sample < 1) return FREE_ERR_SHAPE;
    } else if (epilogue == FREE_EPI_BIAS || epilogue == FREE_EPI_BIAS_GELU) {
        if (!out) return FREE_ERR_NULL;
    } else {
        return FREE_ERR_RANGE;
    }
    Dims d{};
    d.mode = dtype;
    RowVec g{gate, gate_stride, rows_per_sample > 0 ? rows_per_sample : 1};
    return linear_dispatch(d, A, W, bias, M, N, Kdim, epilogue, out, resid, g, static_cast<hipStream_t>(stream));
}

int32_t free_op_ln_fold_vectors(const float* mod, int32_t B, int32_t hidden, int32_t ffn, int32_t mod_stride,
                                int32_t depth, const void* const* w_qkv, const float* const* b_qkv,
                                const void* const* w_fc1, const float* const* b_fc1, float* fold,
                                int64_t fold_stride, void* stream) {
    if (!mod || !w_qkv || !b_qkv || !w_fc1 || !b_fc1 || !fold) return FREE_ERR_NULL;
    if (B < 1 || hidden < 1 || ffn < 1 || depth < 1 || depth > 4096 || mod_stride < 6 * depth * hidden) return FREE_ERR_SHAPE;
    if (!ln_fold_supported(hidden, 3 * hidden, ffn)) return FREE_ERR_SHAPE;
    std::vector<const void*> tab(4 * static_cast<size_t>(depth));
    for (int l = 0; l < depth; ++l) {
        if (!w_qkv[l] || !b_qkv[l] || !w_fc1[l] || !b_fc1[l]) return FREE_ERR_NULL;
        tab[2 * l] = w_qkv[l];
        tab[2 * l + 1] = w_fc1[l];
        tab[2 * depth + 2 * l] = b_qkv[l];
        tab[2 * depth + 2 * l + 1] = b_fc1[l];
    }
    void* dev = nullptr;
    if (!hip_ok(hipMalloc(&dev, tab.size() * sizeof(void*)))) return FREE_ERR_HIP;
    int32_t st = FREE_OK;
    hipStream_t s = static_cast<hipStream_t>(stream);
    if (!hip_ok(hipMemcpy(dev, tab.data(), tab.size() * sizeof(void*), hipMemcpyHostToDevice))) st = FREE_ERR_HIP;
    if (st == FREE_OK)
        st = launch_ln_fold(mod, B, hidden, mod_stride, depth, 3 * hidden, ffn, static_cast<const void* const*>(dev),
                            reinterpret_cast<const float* const*>(static_cast<const void* const*>(dev) + 2 * depth), fold,
                            fold_stride, s);
    if (!hip_ok(hipStreamSynchronize(s)) && st == FREE_OK) st = FREE_ERR_HIP;
    if (!hip_ok(hipFree(dev)) && st == FREE_OK) st = FREE_ERR_HIP;
    return st;
}

int32_t free_op_linear_resid_prep(const void* A, const void* W, const float* bias, int32_t M, int32_t N,
                                  int32_t Kdim, float* resid, const float* gate, const float* scale_next,
                                  int32_t mod_stride, int32_t rows_per_sample, void* z, float* stats,
                                  void* stream) {
    if (!A || !W || !bias || !resid || !gate || !scale_next || !z || !stats) return FREE_ERR_NULL;
    if (M < 1 || N < 1 || Kdim < 1 || rows_per_sample < 1 || N % kLnSlotCols != 0) return FREE_ERR_SHAPE;
    Dims d{};
    d.mode = FREE_BF16;
    LnFold f;
    f.scale_next = scale_next;
    f.z = z;
    f.stats = stats;
    f.slots = N / kLnSlotCols;
    return linear_dispatch(d, A, W, bias, M, N, Kdim, FREE_EPI_GATE_RESID_PREP, nullptr, resid,
                           RowVec{gate, mod_stride, rows_per_sample}, static_cast<hipStream_t>(stream), 1, &f);
}

int32_t free_op_linear_ln(const void* z, const void* W, int32_t M, int32_t N, int32_t Kdim, const float* stats,
                          const float* c1, const float* c0, int64_t fold_stride, int32_t rows_per_sample,
                          int32_t gelu, void* out, void* stream) {
    if (!z || !W || !stats || !c1 || !c0 || !out) return FREE_ERR_NULL;
    if (M < 1 || N < 1 || Kdim < 1 || Kdim % kLnSlotCols != 0) return FREE_ERR_SHAPE;
    if (!mfma_ln_fold_supported(M, Kdim, rows_per_sample)) return FREE_ERR_SHAPE;
    Dims d{};
    d.mode = FREE_BF16;
    LnFold f;
    f.stats = const_cast<float*>(stats);
    f.slots = Kdim / kLnSlotCols;
    f.c1 = c1;
    f.c0 = c0;
    f.fold_stride = fold_stride;
    f.rows_per_sample = rows_per_sample;
    f.inv_width = 1.0f / static_cast<float>(Kdim);
    // (the bias is inside c0; the kernel still wants a valid, aligned pointer for the argument)
    return linear_dispatch(d, z, W, c0, M, N, Kdim, gelu ? FREE_EPI_LN_BIAS_GELU : FREE_EPI_LN_BIAS, out, nullptr,
                           RowVec{nullptr, 0, 1}, static_cast<hipStream_t>(stream), 1, &f);
}

int32_t free_op_attention(const void* qkv, int32_t B, int32_t N, int32_t heads, int32_t dh, int32_t dtype,
                          void* out, void* stream) {
    if (!qkv || !out) return FREE_ERR_NULL;
    if (dtype != FREE_FP32 && dtype != FREE_BF16) return FREE_ERR_DTYPE;
    if (B < 1 || N < 1 || heads < 1 || dh < 1 || dh > 128) return FREE_ERR_SHAPE;
    Dims d{};
    d.mode = dtype;
    d.ntok = N;
    d.heads = heads;
    d.dh = dh;
    return attention_dispatch(d, qkv, B, out, static_cast<hipStream_t>(stream));
}

int32_t free_op_ln_modulate(const float* x, const float* shift, const float* scale, int32_t mod_stride, int32_t M,
                            int32_t D, int32_t rows_per_sample, int32_t dtype, void* out, void* stream) {
    if (!x || !shift || !scale || !out) return FREE_ERR_NULL;
    if (dtype != FREE_FP32 && dtype != FREE_BF16) return FREE_ERR_DTYPE;
    if (M < 1 || D < 1 || rows_per_sample < 1) return FREE_ERR_SHAPE;
    return launch_ln_modulate(x, RowVec{shift, mod_stride, rows_per_sample},
                              RowVec{scale, mod_stride, rows_per_sample}, M, D, dtype, out,
                              static_cast<hipStream_t>(stream));
}

}  // extern "C"

namespace {

// Workspace of the drafter on B samples.
constexpr int kHoistRows = 16;          // samples of one adaLN pass

struct DraftLayout {
    size_t cond_h, sc, mod, tpack, ypack, emb, fin, xn, qkv, att, hmid, eps, feat, total;
};

DraftLayout make_draft_layout(const Dims& d, int32_t mod_rows, int32_t B) {
    DraftLayout L;
    const size_t es = d.mode == FREE_BF16 ? 2 : 4;
    const size_t M = static_cast<size_t>(B) * d.ntok;
    size_t off = 0;
    auto take = [&](size_t bytes) { size_t o = off; off += align_up(bytes); return o; };
    // conditioning buffers hold at least kHoistRows samples: draft_round computes the conditioning and the
    // modulation vectors of all its K steps (their timesteps are known up front) in one go
    const size_t CB = static_cast<size_t>(B > kHoistRows ? B : kHoistRows);
    L.cond_h = take(CB * (d.tfreq + d.D) * 4);
    L.sc = take(CB * d.D * 4);
    L.mod = take(CB * mod_rows * 4);
    L.tpack = take(CB * 4);
    L.ypack = take(CB * 4);
    L.emb = take(M * d.D * 4);
    L.fin = take(M * 2 * d.D * es);
    L.xn = take(M * d.D * es);
    L.qkv = take(M * 3 * d.D * es);
    L.att = take(M * d.D * es);
    L.hmid = take(M * d.F * es);
    L.eps = take(static_cast<size_t>(B) * d.c_out * d.H * d.W * 4);
    L.feat = take(M * d.D * 4);
    L.total = off;
    return L;
}

// One drafter evaluation (Sec. 3.2).  Sample b reads the latent x[b % x_mod]; f_out doubles as the
// residual stream of the drafter's blocks (it IS the predicted feature when they are done), and
// f_prev is consumed before f_out is first written, so the two may alias.
// Conditioning (shared embedding layers of the target) and the drafter's modulation vectors for B samples.
int32_t drafter_modulation(free_drafter_t dr, const int32_t* t, const int32_t* y, int32_t B, float* cond_h, float* sc,
                           float* mod, hipStream_t s) {
    free_dit_t h = dr->target;
    const Dims& d = h->dims;
    FREE_TRY(launch_conditioning(t, y, B, d.D, d.tfreq, static_cast<const float*>(h->w[W_T_W1]),
                                 static_cast<const float*>(h->w[W_T_B1]), static_cast<const float*>(h->w[W_T_W2]),
                                 static_cast<const float*>(h->w[W_T_B2]),
                                 static_cast<const float*>(h->w[W_Y_TABLE]), cond_h, sc, s));
    if (adaln_mfma_supported(d.D, dr->mod_rows))
        return launch_adaln_mfma(sc, B, d.D, dr->ada_w_tab, dr->ada_b_tab, dr->ada_row_start, dr->depth + 1,
                                 dr->mod_rows, d.mode, mod, s);
    return launch_adaln(sc, B, d.D, dr->ada_w_tab, dr->ada_b_tab, dr->ada_row_start, dr->depth + 1, dr->mod_rows,
                        d.mode, mod, s);
}

// mod_pre (nullable): modulation vectors computed by the caller, sample b at mod_pre + b * mod_stride; then t
// and y are not read.
int32_t drafter_forward_impl(free_drafter_t dr, const float* x, int32_t x_mod, const float* f_prev, const int32_t* t,
                             const int32_t* y, int32_t B, float* eps_out, float* f_out, char* ws, hipStream_t s,
                             const float* mod_pre = nullptr, int32_t mod_stride = 0) {
    free_dit_t h = dr->target;
    const Dims& d = h->dims;
    const DraftLayout L = make_draft_layout(d, dr->mod_rows, B);
    const int64_t M = static_cast<int64_t>(B) * d.ntok;
    float* cond_h = reinterpret_cast<float*>(ws + L.cond_h);
    float* sc = reinterpret_cast<float*>(ws + L.sc);
    const float* mod = mod_pre;
    if (!mod_pre) {
        FREE_TRY(drafter_modulation(dr, t, y, B, cond_h, sc, reinterpret_cast<float*>(ws + L.mod), s));
        mod = reinterpret_cast<float*>(ws + L.mod);
        mod_stride = dr->mod_rows;
    }
    float* emb = reinterpret_cast<float*>(ws + L.emb);
    void* fin = ws + L.fin;
    FREE_TRY(launch_patch_embed(x, x_mod, B, d.C, d.H, d.W, d.p, d.D, static_cast<const float*>(h->w[W_PATCH_W]),
                                static_cast<const float*>(h->w[W_PATCH_B]), h->pos, emb, s));
    // z = fuse_w [emb | f_prev] + fuse_b, accumulated in fp32 straight into the residual stream:
    // residual epilogue on a zeroed stream with a gate of ones
    FREE_TRY(launch_fuse_pack(emb, f_prev, M, d.D, d.mode, fin, f_out, s));
    FREE_TRY(linear_dispatch(d, fin, dr->w[0], static_cast<const float*>(dr->w[1]), static_cast<int32_t>(M), d.D,
                             2 * d.D, FREE_EPI_GATE_RESID, nullptr, f_out, RowVec{dr->ones, 0, 1}, s));
    const ActBufs act{f_out, ws + L.xn, ws + L.qkv, ws + L.att, ws + L.hmid};
    FREE_TRY(run_block_stack(d, dr->blkw(), dr->depth, mod, mod_stride, act, 0, B, s, &h->prof));
    RowVec fsh{mod + static_cast<int64_t>(dr->depth) * 6 * d.D, mod_stride, d.ntok};
    RowVec fsc{mod + static_cast<int64_t>(dr->depth) * 6 * d.D + d.D, mod_stride, d.ntok};
    return launch_final_layer(f_out, fsh, fsc, B, d.gh, d.gw, d.p, d.c_out, d.D, dr->fin(F_W),
                              static_cast<const float*>(dr->fin(F_B)), d.mode, eps_out, s);
}

}  // namespace

extern "C" {

int32_t free_drafter_weight_count(int32_t drafter_depth) {
    return drafter_depth < 1 ? -1 : 2 + 10 * drafter_depth + 4;
}

int32_t free_drafter_create(free_dit_t target, int32_t drafter_depth, const void* const* weight_ptrs,
                            int32_t n_ptrs, free_drafter_t* out) {
    if (!target || !weight_ptrs || !out) return FREE_ERR_NULL;
    if (drafter_depth < 1 || drafter_depth > 64 || n_ptrs != free_drafter_weight_count(drafter_depth))
        return FREE_ERR_SHAPE;
    for (int i = 0; i < n_ptrs; ++i) {
        if (!weight_ptrs[i]) return FREE_ERR_NULL;
        if (reinterpret_cast<uintptr_t>(weight_ptrs[i]) & 15u) return FREE_ERR_SHAPE;
    }
    const Dims& d = target->dims;
    free_drafter_s* dr = new (std::nothrow) free_drafter_s();
    if (!dr) return FREE_ERR_HIP;
    dr->target = target;
    dr->depth = drafter_depth;
    dr->mod_rows = drafter_depth * 6 * d.D + 2 * d.D;
    dr->w.assign(weight_ptrs, weight_ptrs + n_ptrs);
    // device block: [w_tab | b_tab | row_start | ones (D floats)]
    const int n_mats = drafter_depth + 1;
    const size_t off_w = 0;
    const size_t off_b = align_up(off_w + n_mats * sizeof(void*));
    const size_t off_r = align_up(off_b + n_mats * sizeof(void*));
    const size_t off_o = align_up(off_r + (n_mats + 1) * sizeof(int32_t));
    const size_t total = off_o + static_cast<size_t>(d.D) * sizeof(float);
    std::vector<char> host(total, 0);
    const void** wt = reinterpret_cast<const void**>(host.data() + off_w);
    const void** bt = reinterpret_cast<const void**>(host.data() + off_b);
    int32_t* rs = reinterpret_cast<int32_t*>(host.data() + off_r);
    for (int l = 0; l < drafter_depth; ++l) {
        wt[l] = dr->blkw()[10 * l + B_ADA_W];
        bt[l] = dr->blkw()[10 * l + B_ADA_B];
        rs[l] = l * 6 * d.D;
    }
    wt[drafter_depth] = dr->fin(F_ADA_W);
    bt[drafter_depth] = dr->fin(F_ADA_B);
    rs[drafter_depth] = drafter_depth * 6 * d.D;
    rs[drafter_depth + 1] = dr->mod_rows;
    float* ones = reinterpret_cast<float*>(host.data() + off_o);
    for (int i = 0; i < d.D; ++i) ones[i] = 1.0f;
    if (!hip_ok(hipMalloc(&dr->dev_block, total)) ||
        !hip_ok(hipMemcpy(dr->dev_block, host.data(), total, hipMemcpyHostToDevice))) {
        if (dr->dev_block) (void)hipFree(dr->dev_block);
        delete dr;
        return FREE_ERR_HIP;
    }
    char* db = static_cast<char*>(dr->dev_block);
    dr->ada_w_tab = reinterpret_cast<const void* const*>(db + off_w);
    dr->ada_b_tab = reinterpret_cast<const float* const*>(db + off_b);
    dr->ada_row_start = reinterpret_cast<const int32_t*>(db + off_r);
    dr->ones = reinterpret_cast<const float*>(db + off_o);
    *out = dr;
    return FREE_OK;
}

int32_t free_drafter_destroy(free_drafter_t dr) {
    if (!dr) return FREE_ERR_NULL;
    int32_t st = FREE_OK;
    if (dr->dev_block && !hip_ok(hipFree(dr->dev_block))) st = FREE_ERR_HIP;
    delete dr;
    return st;
}

size_t free_drafter_workspace_bytes(free_dit_t target, int32_t drafter_depth, int32_t B) {
    if (!target || drafter_depth < 1 || B < 1) return 0;
    const Dims& d = target->dims;
    return make_draft_layout(d, drafter_depth * 6 * d.D + 2 * d.D, B).total;
}

int32_t drafter_forward(free_drafter_t dr, const float* x, const float* f_prev, const int32_t* t,
                        const int32_t* y, int32_t B, float* eps_out, float* f_out, void* workspace,
                        size_t ws_bytes, void* stream) {
    if (!dr || !x || !f_prev || !t || !y || !eps_out || !f_out) return FREE_ERR_NULL;
    if (B < 1) return FREE_ERR_SHAPE;
    const Dims& d = dr->target->dims;
    FREE_TRY(check_ws(workspace, ws_bytes, make_draft_layout(d, dr->mod_rows, B).total));
    if ((reinterpret_cast<uintptr_t>(f_prev) | reinterpret_cast<uintptr_t>(f_out)) & 15u) return FREE_ERR_SHAPE;
    return drafter_forward_impl(dr, x, B, f_prev, t, y, B, eps_out, f_out, static_cast<char*>(workspace),
                                static_cast<hipStream_t>(stream));
}

int32_t draft_round(free_drafter_t dr, const float* x_a, const float* f_a, const int32_t* t, int32_t y,
                    float cfg_scale, const float* coef_x, const float* coef_eps, const float* sigma,
                    const float* xi, int32_t K, float* x_states, float* x_last, float* m_draft,
                    float* f_last, void* workspace, size_t ws_bytes, void* stream) {
    if (!dr || !x_a || !f_a || !t || !coef_x || !coef_eps || !sigma || !xi || !x_states || !x_last || !m_draft)
        return FREE_ERR_NULL;
    const Dims& d = dr->target->dims;
    if (K < 1 || K > FREE_MAX_DRAFTS) return FREE_ERR_SHAPE;
    if (y < 0 || y > d.classes) return FREE_ERR_RANGE;
    if (!(cfg_scale == cfg_scale)) return FREE_ERR_RANGE;
    const int32_t dup = cfg_scale > 1.0f ? 2 : 1;
    const DraftLayout L = make_draft_layout(d, dr->mod_rows, dup);
    FREE_TRY(check_ws(workspace, ws_bytes, L.total));
    if ((reinterpret_cast<uintptr_t>(f_a) | reinterpret_cast<uintptr_t>(f_last)) & 15u) return FREE_ERR_SHAPE;
    char* ws = static_cast<char*>(workspace);
    hipStream_t s = static_cast<hipStream_t>(stream);
    int32_t* tp = reinterpret_cast<int32_t*>(ws + L.tpack);
    int32_t* yp = reinterpret_cast<int32_t*>(ws + L.ypack);
    float* eps = reinterpret_cast<float*>(ws + L.eps);
    float* feat = f_last ? f_last : reinterpret_cast<float*>(ws + L.feat);
    const size_t feat_bytes = static_cast<size_t>(dup) * d.ntok * d.D * 4;
    const int64_t hw = static_cast<int64_t>(d.H) * d.W;
    if (!hip_ok(hipMemcpyAsync(x_states, x_a, static_cast<size_t>(d.d) * 4, hipMemcpyDeviceToDevice, s)))
        return FREE_ERR_HIP;
    if (feat != f_a && !hip_ok(hipMemcpyAsync(feat, f_a, feat_bytes, hipMemcpyDeviceToDevice, s)))
        return FREE_ERR_HIP;
    // The timesteps of all K steps are known: their conditioning and modulation vectors are computed in one
    // pass (packed as [cond x K | null x K], so step k reads samples k and K + k), not once per step.
    const bool hoist = K * dup <= kHoistRows;
    const float* mod_all = nullptr;
    if (hoist) {
        FREE_TRY(launch_pack_cond(t, y, d.classes, K, dup, tp, yp, s));
        FREE_TRY(drafter_modulation(dr, tp, yp, K * dup, reinterpret_cast<float*>(ws + L.cond_h),
                                    reinterpret_cast<float*>(ws + L.sc), reinterpret_cast<float*>(ws + L.mod), s));
        mod_all = reinterpret_cast<const float*>(ws + L.mod);
    }
    for (int k = 0; k < K; ++k) {
        const float* xk = x_states + static_cast<int64_t>(k) * d.d;
        float* mk = m_draft + static_cast<int64_t>(k) * d.d;
        float* xn = k + 1 < K ? x_states + static_cast<int64_t>(k + 1) * d.d : x_last;
        if (hoist) {
            FREE_TRY(drafter_forward_impl(dr, xk, 1, feat, nullptr, nullptr, dup, eps, feat, ws, s,
                                          mod_all + static_cast<int64_t>(k) * dr->mod_rows, K * dr->mod_rows));
        } else {
            FREE_TRY(launch_pack_cond(t + k, y, d.classes, 1, dup, tp, yp, s));
            FREE_TRY(drafter_forward_impl(dr, xk, 1, feat, tp, yp, dup, eps, feat, ws, s));
        }
        FREE_TRY(launch_eps_to_mean(eps, xk, coef_x + k, coef_eps + k, cfg_scale, 1, d.C, d.c_out, hw, mk, s, nullptr,
                                    sigma + k, xi + static_cast<int64_t>(k) * d.d, xn));
    }
    return FREE_OK;
}

}  // extern "C"

namespace {

// Workspace of the sampler: the target's and the drafter's own workspaces plus the round's buffers.
struct LoopLayout {
    size_t ws_target, ws_draft, x_cur, x_states, x_last, m_draft, m_target, log_ratio, accept, n_accept, x_refl,
        top_feat, feat, tp, yp, eps, eps_guided, dist, total;
};

LoopLayout make_loop_layout(const Dims& d, int32_t drafter_mod_rows, int32_t L, int32_t dup) {
    LoopLayout o;
    size_t off = 0;
    auto take = [&](size_t bytes) { size_t r = off; off += align_up(bytes); return r; };
    const size_t dd = static_cast<size_t>(d.d) * 4, fd = static_cast<size_t>(d.ntok) * d.D * 4;
    o.ws_target = take(make_layout(d, L * dup).total);
    o.ws_draft = take(drafter_mod_rows > 0 ? make_draft_layout(d, drafter_mod_rows, dup).total : 0);
    o.x_cur = take(dd);
    o.x_states = take(dd * L);
    o.x_last = take(dd);
    o.m_draft = take(dd * L);
    o.m_target = take(dd * L);
    o.log_ratio = take(static_cast<size_t>(L) * 4);
    o.accept = take(static_cast<size_t>(L));
    o.n_accept = take(4);
    o.x_refl = take(dd);
    o.top_feat = take(drafter_mod_rows > 0 ? fd * L * dup : 0);
    o.feat = take(drafter_mod_rows > 0 ? fd * dup : dd);      // top-block features, or one frozen noise estimate
    o.tp = take(static_cast<size_t>(L) * dup * 4);
    o.yp = take(static_cast<size_t>(L) * dup * 4);
    o.eps = take(static_cast<size_t>(L) * dup * d.c_out * d.H * d.W * 4);
    o.eps_guided = take(dd * L);
    o.dist = take(sizeof(double) * FREE_MAX_DRAFTS);
    o.total = off;
    return o;
}

inline float* F0(char* ws, size_t off) { return reinterpret_cast<float*>(ws + off); }

// The sampler of Alg. 1.  dr != nullptr: feature-level drafter; dr == nullptr: frozen-target drafting
// (self-speculative run of Sec. 3.4: the guided noise estimate of the latest target evaluation is the
// "feature"), with the deviation || eps_frozen - eps_target ||_2 and the outcome of every checked draft
// logged to eps_delta / accepted (host arrays of S entries, NaN / -1 where nothing was checked).
int32_t sample_loop(free_dit_t h, free_drafter_t dr, const float* x_init, int32_t y, float cfg_scale, int32_t S,
                    int32_t n_spec, int32_t L, const int32_t* tmap, const float* coef_x, const float* coef_eps,
                    const float* sigma, const float* xi, const float* u, const float* lambda, float* x_result,
                    int32_t* stats, int32_t* n_accept_log, float* eps_delta, int8_t* accepted, void* workspace,
                    size_t ws_bytes, hipStream_t s) {
    if (!x_init || !tmap || !coef_x || !coef_eps || !sigma || !xi || !u || !x_result) return FREE_ERR_NULL;

    const Dims& d = h->dims;
    if (S < 1 || n_spec < 0 || n_spec > S || L < 1 || L > FREE_MAX_DRAFTS) return FREE_ERR_SHAPE;
    if (y < 0 || y > d.classes) return FREE_ERR_RANGE;
    if (!(cfg_scale == cfg_scale)) return FREE_ERR_RANGE;
    const int32_t dup = cfg_scale > 1.0f ? 2 : 1;
    const bool frozen = dr == nullptr;
    const LoopLayout o = make_loop_layout(d, frozen ? 0 : dr->mod_rows, L, dup);
    FREE_TRY(check_ws(workspace, ws_bytes, o.total));
    char* ws = static_cast<char*>(workspace);
    if (eps_delta)
        for (int k = 0; k < S; ++k) eps_delta[k] = std::nanf("");
    if (accepted)
        for (int k = 0; k < S; ++k) accepted[k] = -1;
    float* eps_g = F0(ws, o.eps_guided);          // guided noise estimates of the latest target call [L, d]
    double* dist = reinterpret_cast<double*>(ws + o.dist);
    auto F = [&](size_t off) { return reinterpret_cast<float*>(ws + off); };
    float* x_cur = F(o.x_cur);
    float* feat = F(o.feat);
    float* top = F(o.top_feat);
    int32_t* tp = reinterpret_cast<int32_t*>(ws + o.tp);
    int32_t* yp = reinterpret_cast<int32_t*>(ws + o.yp);
    int32_t* n_acc_dev = reinterpret_cast<int32_t*>(ws + o.n_accept);
    const size_t dd = static_cast<size_t>(d.d) * 4, fd = static_cast<size_t>(d.ntok) * d.D * 4;
    const int64_t hw = static_cast<int64_t>(d.H) * d.W;
    auto copy = [&](void* dst, const void* src, size_t n) {
        return hip_ok(hipMemcpyAsync(dst, src, n, hipMemcpyDeviceToDevice, s)) ? FREE_OK : FREE_ERR_HIP;
    };
    int32_t st[4] = {0, 0, 0, 0};       // target calls, rounds, accepted drafts, drafter steps
    FREE_TRY(copy(x_cur, x_init, dd));
    bool have_feat = false;
    int i = 0, round = 0;
    while (i < S) {
        if (!have_feat || i >= n_spec) {
            // plain target step: x_{i+1} = m_i + sigma_i xi_i; its top-block feature starts the next round
            FREE_TRY(launch_pack_cond(tmap + i, y, d.classes, 1, dup, tp, yp, s));
            FREE_TRY(forward_impl(h, x_cur, 1, tp, yp, dup, F(o.eps), frozen ? nullptr : feat, ws + o.ws_target, s));
            FREE_TRY(launch_eps_to_mean(F(o.eps), x_cur, coef_x + i, coef_eps + i, cfg_scale, 1, d.C, d.c_out, hw,
                                        F(o.m_target), s, frozen ? feat : nullptr, sigma + i,
                                        xi + static_cast<int64_t>(i) * d.d, x_cur));
            have_feat = true;
            ++st[0];
            ++i;
            continue;
        }
        const int K = L < n_spec - i ? L : n_spec - i;
        const int B = K * dup;
        if (frozen)
            FREE_TRY(launch_frozen_draft(x_cur, feat, coef_x + i, coef_eps + i, sigma + i,
                                         xi + static_cast<int64_t>(i) * d.d, K, d.d, F(o.x_states), F(o.x_last),
                                         F(o.m_draft), s));
        else
            FREE_TRY(draft_round(dr, x_cur, feat, tmap + i, y, cfg_scale, coef_x + i, coef_eps + i, sigma + i,
                                 xi + static_cast<int64_t>(i) * d.d, K, F(o.x_states), F(o.x_last), F(o.m_draft), feat,
                                 ws + o.ws_draft, make_draft_layout(d, dr->mod_rows, dup).total, s));
        const WsLayout TL = make_layout(d, B);
        FREE_TRY(launch_pack_cond(tmap + i, y, d.classes, K, dup, tp, yp, s));
        FREE_TRY(forward_impl(h, F(o.x_states), K, tp, yp, B, F(o.eps), frozen ? nullptr : top, ws + o.ws_target, s));
        FREE_TRY(launch_eps_to_mean(F(o.eps), F(o.x_states), coef_x + i, coef_eps + i, cfg_scale, K, d.C, d.c_out, hw,
                                    F(o.m_target), s, frozen ? eps_g : nullptr));
        if (eps_delta) FREE_TRY(launch_sqdist(F(o.m_draft), F(o.m_target), K, d.d, dist, s));
        VerifyArgs a{F(o.m_target), F(o.m_draft), F(o.x_states), F(o.x_last), sigma + i, u + i,
                     lambda ? lambda + i : nullptr, 1, K, d.d, F(o.log_ratio),
                     reinterpret_cast<uint8_t*>(ws + o.accept), n_acc_dev, F(o.x_refl), &h->prof};
        FREE_TRY(launch_verify(a, ws + o.ws_target + TL.vpart, TL.vpart_bytes, s));
        int32_t n = 0;
        if (!hip_ok(hipMemcpyAsync(&n, n_acc_dev, 4, hipMemcpyDeviceToHost, s)) || !hip_ok(hipStreamSynchronize(s)))
            return FREE_ERR_HIP;
        if (n < 0 || n > K) return FREE_ERR_HIP;
        if (eps_delta || accepted) {
            // the drafts 0 .. min(n, K-1) were checked: ||m^ - m|| / |coef_eps| = ||eps^ - eps|| (same state)
            const int checked = n == K ? K : n + 1;
            double hd[FREE_MAX_DRAFTS];
            float hc[FREE_MAX_DRAFTS];
            if (!hip_ok(hipMemcpyAsync(hd, dist, sizeof(double) * K, hipMemcpyDeviceToHost, s)) ||
                !hip_ok(hipMemcpyAsync(hc, coef_eps + i, sizeof(float) * K, hipMemcpyDeviceToHost, s)) ||
                !hip_ok(hipStreamSynchronize(s)))
                return FREE_ERR_HIP;
            for (int k = 0; k < checked; ++k) {
                if (eps_delta) eps_delta[i + k] = static_cast<float>(std::sqrt(hd[k]) / std::fabs(hc[k]));
                if (accepted) accepted[i + k] = k < n ? 1 : 0;
            }
        }
        if (n_accept_log) n_accept_log[round] = n;
        ++round;
        ++st[0];
        ++st[1];
        st[2] += n;
        st[3] += K;
        // the feature of the packed state whose transition was taken: index K-1 (all accepted) or n,
        // of the label branch (row j) and of the null branch (row K + j)
        const int j = n == K ? K - 1 : n;
        if (frozen) {
            FREE_TRY(copy(feat, reinterpret_cast<char*>(eps_g) + static_cast<size_t>(j) * dd, dd));
        } else {
            for (int b = 0; b < dup; ++b)
                FREE_TRY(copy(reinterpret_cast<char*>(feat) + b * fd,
                              reinterpret_cast<char*>(top) + (static_cast<size_t>(b) * K + j) * fd, fd));
        }
        FREE_TRY(copy(x_cur, n == K ? F(o.x_last) : F(o.x_refl), dd));
        i += n == K ? K : n + 1;
    }
    FREE_TRY(copy(x_result, x_cur, dd));
    if (!hip_ok(hipStreamSynchronize(s))) return FREE_ERR_HIP;
    if (stats)
        for (int k = 0; k < 4; ++k) stats[k] = st[k];
    return FREE_OK;
}

}  // namespace

extern "C" {

size_t free_sample_workspace_bytes(free_drafter_t dr, int32_t L, float cfg_scale) {
    if (!dr || L < 1 || L > FREE_MAX_DRAFTS || !(cfg_scale == cfg_scale)) return 0;
    return make_loop_layout(dr->target->dims, dr->mod_rows, L, cfg_scale > 1.0f ? 2 : 1).total;
}

int32_t free_sample(free_drafter_t dr, const float* x_init, int32_t y, float cfg_scale, int32_t S, int32_t n_spec,
                    int32_t L, const int32_t* tmap, const float* coef_x, const float* coef_eps, const float* sigma,
                    const float* xi, const float* u, const float* lambda, float* x_result, int32_t* stats,
                    int32_t* n_accept_log, void* workspace, size_t ws_bytes, void* stream) {
    if (!dr) return FREE_ERR_NULL;
    return sample_loop(dr->target, dr, x_init, y, cfg_scale, S, n_spec, L, tmap, coef_x, coef_eps, sigma, xi, u, lambda,
                       x_result, stats, n_accept_log, nullptr, nullptr, workspace, ws_bytes,
                       static_cast<hipStream_t>(stream));
}

size_t free_self_speculative_workspace_bytes(free_dit_t target, int32_t L, float cfg_scale) {
    if (!target || L < 1 || L > FREE_MAX_DRAFTS || !(cfg_scale == cfg_scale)) return 0;
    return make_loop_layout(target->dims, 0, L, cfg_scale > 1.0f ? 2 : 1).total;
}

int32_t free_self_speculative(free_dit_t target, const float* x_init, int32_t y, float cfg_scale, int32_t S,
                              int32_t n_spec, int32_t L, const int32_t* tmap, const float* coef_x,
                              const float* coef_eps, const float* sigma, const float* xi, const float* u,
                              const float* lambda, float* x_result, int32_t* stats, int32_t* n_accept_log,
                              float* eps_delta, int8_t* accepted, void* workspace, size_t ws_bytes, void* stream) {
    if (!target) return FREE_ERR_NULL;
    return sample_loop(target, nullptr, x_init, y, cfg_scale, S, n_spec, L, tmap, coef_x, coef_eps, sigma, xi, u, lambda,
                       x_result, stats, n_accept_log, eps_delta, accepted, workspace, ws_bytes,
                       static_cast<hipStream_t>(stream));
}

int32_t free_lambda_profile(const float* eps_delta, int32_t S, int32_t window, float* lambda_out) {
    if (!eps_delta || !lambda_out) return FREE_ERR_NULL;
    if (S < 1 || window < 1 || window % 2 == 0) return FREE_ERR_SHAPE;
    // isotonic least squares (pool adjacent violators); NaN entries carry no weight
    struct Blk { double sum, w; int n; };
    std::vector<Blk> blk;
    blk.reserve(S);
    bool any = false;
    for (int i = 0; i < S; ++i) {
        const bool has = eps_delta[i] == eps_delta[i];
        any = any || has;
        blk.push_back(Blk{has ? static_cast<double>(eps_delta[i]) : 0.0, has ? 1.0 : 0.0, 1});
        while (blk.size() > 1) {
            Blk& a = blk[blk.size() - 2];
            const Blk& b = blk.back();
            if (a.w == 0.0 || b.w == 0.0 || a.sum / a.w > b.sum / b.w) {
                a.sum += b.sum; a.w += b.w; a.n += b.n;
                blk.pop_back();
            } else {
                break;
            }
        }
    }
    if (!any) return FREE_ERR_RANGE;
    std::vector<double> g;
    g.reserve(S);
    for (const Blk& b : blk) g.insert(g.end(), b.n, b.sum / b.w);
    if (window > 1) {                     // centred moving average, ends held: keeps the fit monotone
        const int hw = window / 2;
        std::vector<double> sm(S);
        for (int i = 0; i < S; ++i) {
            double acc = 0.0;
            for (int j = i - hw; j <= i + hw; ++j) acc += g[j < 0 ? 0 : (j >= S ? S - 1 : j)];
            sm[i] = acc / window;
        }
        g.swap(sm);
    }
    const double g0 = g[0] > 1e-300 ? g[0] : 1e-300;
    for (int i = 0; i < S; ++i) lambda_out[i] = static_cast<float>(g0 / (g[i] > 1e-300 ? g[i] : 1e-300));
    return FREE_OK;
}

}  // extern "C"
