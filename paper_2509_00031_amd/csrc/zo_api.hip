// C ABI of the library (see include/zoqat.h): argument checks, the context with its workspace
// layout, and the schedule of one quantized forward / one ZO step over the kernels.
#include "../../include/zoqat.h"
#include "zo_internal.h"

#include <cmath>
#include <cstdio>
#include <cstring>
#include <string>
#include <mutex>
#include <vector>

namespace {

inline size_t align_up(size_t v, size_t a = 256) { return (v + a - 1) / a * a; }
inline bool aligned16(const void* p) { return ((uintptr_t)p & 15) == 0; }

static_assert(ZO_MAX_DIRECTIONS == ZO_MAX_DIRECTIONS_INTERNAL, "public and internal direction limits differ");

enum { ZO_GROUP_MODEL = 0, ZO_GROUP_SMOOTH = 1, ZO_GROUP_CLIP = 2 };   // learning-rate groups

struct param_desc {
    int64_t rows, cols;
    bool quantized;
    int lr_group = ZO_GROUP_MODEL;
    int owner = -1;      // quantized linear: the linear that carries the smoothing pair of its input (q for q/k/v, gate for gate/up)
    int clip = -1;       // quantized linear: index of its step tensor (zero point, alpha, beta follow), or -1
    int smooth = -1;     // quantized linear: index of the s tensor of its input (delta follows), or -1
};

bool describe_base_params(const zo_config& c, std::vector<param_desc>& out);

// Parameter list of a configuration in the fixed order of the header: the model's tensors, then for
// every quantized linear in that order the tensors of Eq. 5 (learn_clip) and Eq. 4 (learn_smooth).
bool describe_params(const zo_config& c, std::vector<param_desc>& out)
{
    if (!describe_base_params(c, out)) return false;
    const int nbase = (int)out.size();
    for (int t = 0; t < nbase; ++t) {
        if (!out[t].quantized) continue;
        const int64_t g = c.w_group > 0 ? c.w_group : out[t].cols;
        if (c.learn_clip) {
            out[t].clip = (int)out.size();
            for (int j = 0; j < 4; ++j) {
                param_desc d{out[t].rows, out[t].cols / g, false};
                d.lr_group = ZO_GROUP_CLIP;
                out.push_back(d);
            }
        }
        if (c.learn_smooth && out[t].owner == t) {
            out[t].smooth = (int)out.size();
            for (int j = 0; j < 2; ++j) {
                param_desc d{1, out[t].cols, false};
                d.lr_group = ZO_GROUP_SMOOTH;
                out.push_back(d);
            }
        }
    }
    if (c.learn_smooth)
        for (int t = 0; t < nbase; ++t)
            if (out[t].quantized) out[t].smooth = out[out[t].owner].smooth;
    return true;
}

bool describe_base_params(const zo_config& c, std::vector<param_desc>& out)
{
    out.clear();
    const int64_t d = c.d_model, f = c.d_ffn, V = c.vocab;
    if (c.arch == ZO_ARCH_LINEAR) {
        if (d <= 0 || f <= 0) return false;
        out.push_back({f, d, true});
        out[0].owner = 0;
        return true;
    }
    if (c.arch != ZO_ARCH_LLAMA && c.arch != ZO_ARCH_OPT) return false;
    if (d <= 0 || f <= 0 || V <= 0 || c.n_layers < 0 || c.n_heads <= 0 || c.max_seq <= 0) return false;
    out.push_back({V, d, false});
    if (c.arch == ZO_ARCH_OPT) out.push_back({c.max_seq, d, false});
    for (int l = 0; l < c.n_layers; ++l) {
        // owner: q for q/k/v, gate for gate/up (they read the same activation), otherwise the linear itself
        auto linear = [&](int64_t rows, int64_t cols, int owner_back) {
            out.push_back({rows, cols, true});
            out.back().owner = (int)out.size() - 1 - owner_back;
        };
        if (c.arch == ZO_ARCH_LLAMA) {
            out.push_back({1, d, false});
            linear(d, d, 0); linear(d, d, 1); linear(d, d, 2); linear(d, d, 0);
            out.push_back({1, d, false});
            linear(f, d, 0);
            linear(f, d, 1);
            linear(d, f, 0);
        } else {
            out.push_back({1, d, false}); out.push_back({1, d, false});
            linear(d, d, 0); out.push_back({1, d, false});
            linear(d, d, 2); out.push_back({1, d, false});
            linear(d, d, 4); out.push_back({1, d, false});
            linear(d, d, 0); out.push_back({1, d, false});
            out.push_back({1, d, false}); out.push_back({1, d, false});
            linear(f, d, 0); out.push_back({1, f, false});
            linear(d, f, 0); out.push_back({1, d, false});
        }
    }
    out.push_back({1, d, false});
    if (c.arch == ZO_ARCH_OPT) out.push_back({1, d, false});
    out.push_back({V, d, false});
    return true;
}

zo_status check_config(const zo_config& c)
{
    std::vector<param_desc> p;
    if (!describe_params(c, p)) return ZO_EINVAL;
    if (c.act_dtype != ZO_ACT_FP32 && c.act_dtype != ZO_ACT_BF16) return ZO_EINVAL;
    if (c.w_bits < 0 || c.w_bits > 8) return ZO_EINVAL;
    if (!(c.a_bits == 16 || (c.a_bits >= 2 && c.a_bits <= 8))) return ZO_EINVAL;
    if (c.w_group < 0) return ZO_EINVAL;
    if ((c.d_model & 7) || (c.d_ffn & 7)) return ZO_ESHAPE;
    if (c.w_bits > 0 && c.w_group > 0 && ((c.w_group & 7) || c.d_model % c.w_group || c.d_ffn % c.w_group)) return ZO_ESHAPE;
    if (c.learn_clip < 0 || c.learn_clip > 1 || c.learn_smooth < 0 || c.learn_smooth > 1) return ZO_EINVAL;
    if ((c.learn_clip || c.learn_smooth) && c.w_bits == 0) return ZO_EINVAL;
    if (c.learn_smooth && (!c.learn_clip || c.a_bits >= 16)) return ZO_EUNSUPPORTED;
    if ((c.learn_clip || c.learn_smooth) && c.lightweight) return ZO_EUNSUPPORTED;
    if (c.no_fused < 0 || c.no_fused > 1) return ZO_EINVAL;
    if (c.master_dtype < 0 || c.master_dtype > 1 || c.master_round < 0 || c.master_round > 1) return ZO_EINVAL;
    if (c.master_dtype == ZO_MASTER_F16 && (c.learn_clip || c.learn_smooth)) return ZO_EUNSUPPORTED;
    if (c.arch != ZO_ARCH_LINEAR) {
        if (c.d_model % c.n_heads) return ZO_ESHAPE;
        const int dh = c.d_model / c.n_heads;
        if (dh != 16 && dh != 32 && dh != 64 && dh != 128) return ZO_EUNSUPPORTED;
    }
    if (c.mma != ZO_MMA_BF16 && c.mma != ZO_MMA_INT8) return ZO_EINVAL;
    if (c.mma == ZO_MMA_INT8) {
        // every quantized linear must be expressible on the integer route (K = d_model and K = d_ffn); fused operands
        // (q | k | v, gate | up) put each tensor at a 256-channel tile boundary of the rows of steps
        if (c.lightweight || c.learn_clip || c.learn_smooth) return ZO_EUNSUPPORTED;
        if (!zo_i8_supported(1, 256, c.d_model, c.w_bits, c.w_group, c.a_bits)) return ZO_EUNSUPPORTED;
        if (c.arch != ZO_ARCH_LINEAR) {
            if (!zo_i8_supported(1, 256, c.d_ffn, c.w_bits, c.w_group, c.a_bits)) return ZO_EUNSUPPORTED;
            if ((c.d_model & 255) || (c.d_ffn & 255)) return ZO_EUNSUPPORTED;
        }
    }
    return ZO_OK;
}

// Workspace layout for B x S tokens.  Offsets in bytes, everything 256-byte aligned.
struct layout {
    size_t scalars;            // fp32[16 + 8 q_max]: loss[2] at 0, {L+, L-, g, c_model, c_smooth, c_clip} at 2; direction i of a
                               // q-direction step: loss[2] at 16 + 8 i, its six values at 16 + 8 i + 2
    size_t rope_cos, rope_sin; // fp32 [max_seq][dh/2]
    size_t what[2];            // de-quantized weights of the current linear(s), per branch
    size_t what_bytes;         // size of each
    size_t vec[2];             // perturbed small vectors of the current sub-layer, per branch: slots 0 gain,
                               // 1 norm bias, 2 linear bias, 3 smoothing s, 4 1/s, 5 smoothing delta
    size_t vec_stride;         // floats per vector slot
    size_t qp[2][4];           // perturbed step / zero point / alpha / beta of the current linear(s), per branch
    size_t qp_elems;
    struct per_branch {
        size_t x, h, hq, qkv, att, gu, act, logits, rowloss;
    } br[2];
    size_t kpart, kpart_bytes; // fp32 partial sums of GEMMs whose K is split (a few hundred tokens, narrow N); 0 bytes: none
    size_t total;
};

layout make_layout(const zo_config& c, int B, int S)
{
    layout L{};
    const size_t ts = zo_tsize(c.act_dtype);
    const size_t d = c.d_model, f = c.d_ffn, V = c.vocab > 0 ? c.vocab : 0;
    size_t off = 0;
    auto take = [&](size_t bytes) { size_t o = off; off += align_up(bytes); return o; };
    L.scalars = take((16 + 8 * ZO_MAX_DIRECTIONS) * sizeof(float));
    const size_t gsz = c.w_group > 0 ? (size_t)c.w_group : 0;
    if (c.arch == ZO_ARCH_LINEAR) {
        const size_t M = B;
        L.what_bytes = f * d * ts;
        for (int b = 0; b < 2; ++b) L.what[b] = take(L.what_bytes);
        L.vec_stride = align_up((d > f ? d : f) * sizeof(float)) / sizeof(float);
        for (int b = 0; b < 2; ++b) L.vec[b] = take(6 * L.vec_stride * sizeof(float));
        L.qp_elems = c.learn_clip ? f * (gsz ? d / gsz : 1) : 0;
        for (int b = 0; b < 2; ++b)
            for (int j = 0; j < 4; ++j) L.qp[b][j] = take(L.qp_elems * sizeof(float));
        for (int b = 0; b < 2; ++b) {
            L.br[b].hq = take(M * d * ts + (c.mma == ZO_MMA_INT8 ? 512 + 8 * M : 0));   // integer route: codes, then per-row step / offset
            L.br[b].logits = take(M * f * ts);      // output Y
            L.br[b].rowloss = take(M * sizeof(float));
        }
        L.total = off;
        return L;
    }
    const size_t M = (size_t)B * S;
    const size_t dh = d / c.n_heads;
    L.rope_cos = take((size_t)c.max_seq * (dh / 2) * sizeof(float));
    L.rope_sin = take((size_t)c.max_seq * (dh / 2) * sizeof(float));
    size_t max_nk = V * d;
    const size_t ffn_rows = c.arch == ZO_ARCH_LLAMA ? 2 * f : f;
    if (3 * d * d > max_nk) max_nk = 3 * d * d;
    if (ffn_rows * d > max_nk) max_nk = ffn_rows * d;
    L.what_bytes = max_nk * ts;
    for (int b = 0; b < 2; ++b) L.what[b] = take(L.what_bytes);
    L.vec_stride = d > f ? d : f;
    if (3 * d > L.vec_stride) L.vec_stride = 3 * d;
    if (ffn_rows > L.vec_stride) L.vec_stride = ffn_rows;
    L.vec_stride = align_up(L.vec_stride * sizeof(float)) / sizeof(float);
    for (int b = 0; b < 2; ++b) L.vec[b] = take(6 * L.vec_stride * sizeof(float));
    if (c.learn_clip) {
        const size_t gd = gsz ? d / gsz : 1, gf = gsz ? f / gsz : 1;     // groups per row for K = d, K = f
        L.qp_elems = 3 * d * gd;
        if (ffn_rows * gd > L.qp_elems) L.qp_elems = ffn_rows * gd;
        if (d * gf > L.qp_elems) L.qp_elems = d * gf;
    }
    for (int b = 0; b < 2; ++b)
        for (int j = 0; j < 4; ++j) L.qp[b][j] = take(L.qp_elems * sizeof(float));
    for (int b = 0; b < 2; ++b) {
        auto& r = L.br[b];
        r.x = take(M * d * ts);
        r.h = take(M * d * ts);
        r.hq = take(M * (d > f ? d : f) * ts + (c.mma == ZO_MMA_INT8 ? 512 + 8 * M : 0));   // integer route: codes, then per-row step / offset
        r.qkv = take(M * 3 * d * ts);
        r.att = take(M * d * ts);
        r.gu = take(M * ffn_rows * ts);
        r.act = take(M * f * ts);
        // logits: fp32 [M][V] -- or, where the lm_head GEMM forms the cross entropy in its epilogue, its per-tile
        // partial results and target logits (and room for the logits of calls too small for that route)
        size_t lg = M * V * sizeof(float);
        if (zo_gemm_ce_supported((int)M, (int)V, (int)d, c.act_dtype == ZO_ACT_BF16 ? ZO_T_BF16 : ZO_T_F32)) {
            const size_t small = ((size_t)256 * 256 * 128 + (size_t)ZO_FUSED_MAX_M * V) * sizeof(float);
            const size_t ce = (zo_gemm_ce_part_floats((int)M, (int)V) + M) * sizeof(float);
            lg = lg < small ? lg : (ce > small ? ce : small);
        }
        r.logits = take(lg);
        r.rowloss = take(M * sizeof(float));
    }
    // K-split scratch: calls with fewer tokens than (B, S) may split where the full shape does not, so room for the most any
    // shape can ask for (at most 1024 workgroups, each a 128 x 128 fp32 tile)
    L.kpart_bytes = c.act_dtype == ZO_ACT_BF16 ? (size_t)1024 * 128 * 128 * sizeof(float) : 0;
    L.kpart = take(L.kpart_bytes);
    L.total = off;
    return L;
}

}  // namespace

struct zo_ctx {
    zo_config cfg;
    std::vector<zo_tensor> params;
    std::vector<param_desc> desc;
    // frozen, pre-quantized storage of a non-trainable linear (lightweight variant); codes == NULL: none
    struct frozen_int4 { const void* codes; const void* step; const int16_t* zp; int group; };
    std::vector<frozen_int4> frozen;
    int n_packed = 0;     // tensors with packed storage attached
    // the packed tensors can share a fused launch sequence with the trainable ones: their group gives the same
    // slab width as the configuration's (so one fragment-ordered copy of the activations serves all tensors of a GEMM)
    bool packed_fusable = true;
    char* ws;
    size_t ws_bytes;
    int max_B, max_S;
    hipStream_t st;
    layout L;           // for max_B x max_S
    int last_M;
    uint32_t routes = 0;  // ZO_ROUTE_* bits of the last forward
    std::string err;
    // optional per-launch timing (zo_profile_begin / zo_profile_end)
    bool prof = false;
    uint32_t prof_mask = 0xFFFFFFFFu;     // categories whose launches are bracketed
    std::vector<hipEvent_t> ev_pool;      // created on demand, reused across sessions
    size_t ev_used = 0;
    std::vector<int> ev_cat;              // category of event pair i = events 2i, 2i+1
    std::vector<float> rope_host[2];      // source of the asynchronous upload of the rotary table: lives as long as the context
};

namespace {

zo_status fail(zo_ctx* c, zo_status s, const char* what, hipError_t e = hipSuccess)
{
    if (c) {
        c->err = what;
        if (e != hipSuccess) { c->err += ": "; c->err += hipGetErrorString(e); }
    }
    return s;
}

// Brackets the launches issued during its lifetime with two events on the context's stream.
struct prof_scope {
    zo_ctx* c;
    bool on;
    prof_scope(zo_ctx* ctx, int cat) : c(ctx), on(ctx && ctx->prof && ((ctx->prof_mask >> cat) & 1u))
    {
        if (!on) return;
        while (c->ev_pool.size() < c->ev_used + 2) {
            hipEvent_t e;
            if (hipEventCreate(&e) != hipSuccess) { on = false; return; }
            c->ev_pool.push_back(e);
        }
        c->ev_cat.push_back(cat);
        (void)hipEventRecord(c->ev_pool[c->ev_used], c->st);
    }
    ~prof_scope()
    {
        if (!on) return;
        (void)hipEventRecord(c->ev_pool[c->ev_used + 1], c->st);
        c->ev_used += 2;
    }
};

#define ZO_HIP(ctx, call)                                                  \
    do {                                                                   \
        hipError_t e_ = (call);                                            \
        if (e_ != hipSuccess) return fail((ctx), ZO_EHIP, #call, e_);      \
    } while (0)

#define ZO_TRY_(x) do { zo_status s__ = (x); if (s__ != ZO_OK) return s__; } while (0)

inline bool trainable(const zo_ctx* c, int i) { return !c->cfg.lightweight || c->params[i].trainable; }

// One forward for nb branches: branch 0 at +eps (or eps_signed when nb == 1), branch 1 at -eps.
struct fwd {
    zo_ctx* c;
    int nb;
    float eps;          // magnitude for paired mode, signed value for single mode
    uint64_t seed;
    int M, S;
    bool sm_on = false;   // the activation being quantized next is smoothed (set by smooth_prepare)
    int pos0 = 0;         // generator: position of the first row (rotary angles / learned positions start there)
    float* alias[2] = {nullptr, nullptr};   // vector slots 0 / 1 served straight from an un-perturbed fp32 master (see vector())
    // small-M route: the tensors of the next GEMM whose tiles are built inside the fused kernel instead of
    // being written to the operand buffers (all of them or none: eligibility depends on the shared shape only)
    struct pend { int t; int64_t row0; bool quantize; bool packed; };
    pend pending[4];
    int npend = 0;
    int nweights = 0;     // operand tensors requested since the last GEMM (deferred or materialised)
    // integer route (zo_config.mma = ZO_MMA_INT8): the operand buffers hold signed-byte codes instead of de-quantized values.
    //   what[b]: [0, what_bytes / 2) codes [N][K]; then the rows of steps at what_bytes / 2, r[N] at + what_bytes / 8 and the
    //            per-group parts of r at + what_bytes / 4 (all far below those bounds: K / group >= ... floats per channel)
    //   hq of branch b: codes [M][K]; per-token step and offset (two fp32 rows of M) behind M * max(d, f) bytes
    int next_t = -1;      // the quantized linear whose input is being prepared (set by smooth_prepare)
    int gemm_N = 0;       // rows of the fused operand the next tensors are blocks of (set before their weights() calls)
    bool x_codes = false, w_codes = false;
    bool i8_route(int t) const
    {
        return c->cfg.mma == ZO_MMA_INT8 && t >= 0 && c->desc[t].quantized && !c->frozen[t].codes && !fused_ok(t, true);
    }
    size_t i8_ws_off() const { return c->L.what_bytes / 2; }
    size_t i8_wr_off() const { return c->L.what_bytes / 2 + c->L.what_bytes / 8; }
    size_t i8_rpart_off() const { return c->L.what_bytes / 2 + c->L.what_bytes / 4; }
    size_t i8_xs_off() const
    {
        const size_t w = c->cfg.arch == ZO_ARCH_LINEAR ? (size_t)c->cfg.d_model
                                                         : (size_t)(c->cfg.d_model > c->cfg.d_ffn ? c->cfg.d_model : c->cfg.d_ffn);
        return align_up((size_t)M * w);
    }
    int* i8_flag() const { return at<int>(c->L.scalars) + 15; }
    // per-token codes of the stored activation `in` (K columns) into hq, for the integer route
    zo_status act_codes(size_t layout::per_branch::*in, int K, size_t layout::per_branch::** used)
    {
        prof_scope ps(c, ZO_PROF_ACT_QUANT);
        for (int b = 0; b < nb; ++b) {
            char* hq = at(c->L.br[b].hq);
            ZO_HIP(c, zo_launch_act_codes_i8(at(c->L.br[b].*in), (int8_t*)hq, (float*)(hq + i8_xs_off()), (float*)(hq + i8_xs_off()) + M, M, K,
                                             c->cfg.a_bits, c->cfg.a_sym, dt(), c->st));
        }
        x_codes = true;
        *used = &layout::per_branch::hq;
        return ZO_OK;
    }
    bool fused_ok(int t, bool quantize) const
    {
        const zo_config& cfg = c->cfg;
        if (cfg.no_fused || cfg.act_dtype != ZO_ACT_BF16 || cfg.learn_clip) return false;
        const param_desc& p = c->desc[t];
        // with packed tensors attached the small-M kernels pay up to 64 tokens only: the packed-codes kernel's time grows with the
        // m-tiles it carries, expanding the codes once and running the plain GEMM does not (13B shapes, 128 tokens: 35.3 ms per
        // step through the small-M kernels, 31.4 ms without; 64 tokens: 25.7 against 29.4 ms)
        if (c->n_packed > 0 && M > 64) return false;
        if (c->frozen[t].codes)                          // stored codes: expanded inside the kernel
            return c->packed_fusable && zo_int4_fused_supported(M, (int)p.rows, (int)p.cols, c->frozen[t].group);
        if (c->n_packed > 0 && !c->packed_fusable) return false;
        const int64_t g = cfg.w_group > 0 ? cfg.w_group : p.cols;
        return zo_fused_supported(M, (int)p.rows, (int)p.cols, quantize ? cfg.w_bits : 0, (int)g);
    }
    template <typename T = char> T* at(size_t off) const { return (T*)(c->ws + off); }
    int dt() const { return c->cfg.act_dtype; }
    int wd() const { return c->cfg.master_dtype == ZO_MASTER_F16 ? ZO_W_F16 : ZO_W_F32; }
    float eps_of(int tensor) const { return trainable(c, tensor) ? eps : 0.0f; }

    bool frozen(int t) const { return c->frozen[t].codes != nullptr; }
    // Q(W +- eps u) of tensor `t` ([rows][cols]) into rows [row0, row0+rows) of the what buffers.
    // shared: every tensor of this GEMM is frozen, so one copy of the operand serves both branches.
    zo_status weights(int t, int64_t row0, bool quantize, bool shared = false, int ilv = 0)
    {
        const param_desc& p = c->desc[t];
        nweights += 1;
        if (ilv == 0 && npend < 4 && fused_ok(t, quantize)) {
            pending[npend++] = pend{t, row0, quantize, c->frozen[t].codes != nullptr};
            return ZO_OK;
        }
        const size_t ts = zo_tsize(dt());
        if (quantize && i8_route(t)) {
            // signed-byte operands of both branches, their steps in the slot layout of the fused operand, r[n]
            const int K = (int)p.cols, G = K / (c->cfg.w_group > 0 ? c->cfg.w_group : K);
            const int n_total = gemm_N > 0 ? gemm_N : (int)p.rows;
            // (SwiGLU: gate and up interleave into one block of 2 f rows starting at row0 = 0)
            if ((row0 & 255) || row0 + p.rows * (ilv == 1 || ilv == 2 ? 2 : 1) > n_total)
                return fail(c, ZO_EUNSUPPORTED, "integer route: operand block not at a tile boundary");
            char* w0 = at(c->L.what[0]);
            char* w1 = nb == 2 ? at(c->L.what[1]) : nullptr;
            auto f32at = [&](char* base, size_t off, size_t idx) { return base ? (float*)(base + off) + idx : nullptr; };
            prof_scope ps(c, ZO_PROF_WEIGHT_QUANT);
            ZO_HIP(c, zo_launch_weight_codes_i8(c->params[t].ptr, (int)p.rows, K, c->cfg.w_bits, c->cfg.w_group, seed, t, eps_of(t), wd(),
                                                (int8_t*)w0 + (size_t)row0 * K, w1 ? (int8_t*)w1 + (size_t)row0 * K : nullptr,
                                                f32at(w0, i8_ws_off(), (size_t)row0), f32at(w1, i8_ws_off(), (size_t)row0),
                                                f32at(w0, i8_wr_off(), (size_t)row0), f32at(w1, i8_wr_off(), (size_t)row0),
                                                f32at(w0, i8_rpart_off(), (size_t)row0 * G), f32at(w1, i8_rpart_off(), (size_t)row0 * G),
                                                i8_flag(), c->st, (n_total + 255) / 256, ilv));
            w_codes = true;
            return ZO_OK;
        }
        void* op = at(c->L.what[0]) + (size_t)row0 * p.cols * ts;
        void* om = nb == 2 ? at(c->L.what[1]) + (size_t)row0 * p.cols * ts : nullptr;
        const int bits = quantize ? c->cfg.w_bits : 0;
        prof_scope ps(c, ZO_PROF_WEIGHT_QUANT);
        const zo_ctx::frozen_int4& fz = c->frozen[t];
        if (fz.codes) {                                  // stored codes: the same operand for both branches
            ZO_HIP(c, zo_launch_dequant_int4(fz.codes, fz.step, fz.zp, (int)p.rows, (int)p.cols, fz.group, dt(), op,
                                             shared ? nullptr : om, c->st, ilv));
            return ZO_OK;
        }
        if (quantize && p.clip >= 0) {
            // Eq. 5: perturb the four parameter tensors of this linear, then quantize with them
            const int64_t G = p.cols / (c->cfg.w_group > 0 ? c->cfg.w_group : p.cols);
            const int64_t qoff = row0 * G, qn = p.rows * G;
            const float* q[2][4] = {};
            for (int j = 0; j < 4; ++j) {
                float* qp = at<float>(c->L.qp[0][j]) + qoff;
                float* qm = nb == 2 ? at<float>(c->L.qp[1][j]) + qoff : nullptr;
                ZO_HIP(c, zo_launch_fq_weight((const float*)c->params[p.clip + j].ptr, 1, (int)qn, 0, 0, seed, p.clip + j,
                                              eps_of(p.clip + j), ZO_T_F32, qp, qm, nullptr, nullptr, nullptr, c->st));
                q[0][j] = qp;
                q[1][j] = qm;
            }
            const zo_learned lp{q[0][0], q[0][1], q[0][2], q[0][3], p.smooth >= 0 ? vec(0, 3) : nullptr};
            const zo_learned lm{q[1][0], q[1][1], q[1][2], q[1][3], (p.smooth >= 0 && nb == 2) ? vec(1, 3) : nullptr};
            ZO_HIP(c, zo_launch_fq_weight_learned((const float*)c->params[t].ptr, (int)p.rows, (int)p.cols, bits, c->cfg.w_group, seed, t,
                                                  eps_of(t), dt(), lp, lm, op, om, nullptr, c->st, ilv));
            return ZO_OK;
        }
        ZO_HIP(c, zo_launch_fq_weight(c->params[t].ptr, (int)p.rows, (int)p.cols, bits, c->cfg.w_group,
                                      seed, t, eps_of(t), dt(), op, om, nullptr, nullptr, nullptr, c->st, wd(), ilv));
        return ZO_OK;
    }
    // The gate / up pair of a Llama-shaped block can leave the GEMM as silu(gate) * up: large bf16 shapes, plain
    // quantizer (no learned tensors, groups the streaming quantizer kernel handles), tensors not on the small-M route.
    // The rotary embedding of a Llama-shaped block can be applied by the epilogue of the fused q | k | v GEMM: head
    // dimension 128, large bf16 shapes, plain quantizer, tensors not on the small-M route.
    bool rope_in_gemm(int t_q) const
    {
        const zo_config& cfg = c->cfg;
        if (cfg.no_fused || cfg.arch != ZO_ARCH_LLAMA || cfg.learn_smooth) return false;      // smoothing gives these linears a bias
        if (cfg.d_model / cfg.n_heads != 128 || fused_ok(t_q, true)) return false;
        if (i8_route(t_q)) return false;                 // (measured slower in the integer GEMM's epilogue than stand-alone)
        return zo_gemm_rope_supported(M, 3 * cfg.d_model, cfg.d_model, dt());
    }
    bool swiglu_in_gemm(int t_gate) const
    {
        const zo_config& cfg = c->cfg;
        if (cfg.no_fused || cfg.arch != ZO_ARCH_LLAMA || cfg.learn_smooth) return false;      // smoothing gives these linears a bias
        if ((cfg.d_ffn & 31) || fused_ok(t_gate, true) || fused_ok(t_gate + 1, true)) return false;
        if (i8_route(t_gate)) return dt() == ZO_T_BF16;              // the integer GEMM has the same epilogue (bf16 output)
        return zo_gemm_swiglu_supported(M, 2 * cfg.d_ffn, cfg.d_model, dt());
    }
    // Eq. 4, activation side of the linears whose input is smoothed by the pair carried by linear `t`:
    // perturbed s into slot 3, its reciprocal into slot 4, perturbed delta into slot 5 (no-op without smoothing)
    zo_status smooth_prepare(int t)
    {
        const param_desc& p = c->desc[t];
        next_t = t;
        sm_on = p.smooth >= 0;
        if (!sm_on) return ZO_OK;
        ZO_TRY_(vector(p.smooth, 3));
        ZO_TRY_(vector(p.smooth + 1, 5));
        prof_scope ps(c, ZO_PROF_WEIGHT_QUANT);
        for (int b = 0; b < nb; ++b) ZO_HIP(c, zo_launch_reciprocal(vec(b, 3), vec(b, 4), p.cols, c->st));
        return ZO_OK;
    }
    const float* sm_delta(int b) const { return sm_on ? vec(b, 5) : nullptr; }
    const float* sm_inv(int b) const { return sm_on ? vec(b, 4) : nullptr; }
    // bias of the smoothed linear `t`: slot 2 [o ..) = (perturbed bias already there, if has_bias) + delta' W'^T
    zo_status bias_shift(int t, int64_t o, bool has_bias)
    {
        const param_desc& p = c->desc[t];
        if (p.smooth < 0) return ZO_OK;
        prof_scope ps(c, ZO_PROF_WEIGHT_QUANT);
        float* bp = vec(0, 2) + o;
        float* bm = nb == 2 ? vec(1, 2) + o : nullptr;
        ZO_HIP(c, zo_launch_bias_shift((const float*)c->params[t].ptr, (int)p.rows, (int)p.cols, seed, t, eps_of(t), vec(0, 5),
                                       nb == 2 ? vec(1, 5) : nullptr, has_bias ? bp : nullptr, has_bias ? bm : nullptr, bp, bm, c->st));
        return ZO_OK;
    }
    // perturbed fp32 vector of tensor `t` into vector slot `slot` at float offset `o`
    zo_status vector(int t, int slot, int64_t o = 0)
    {
        const param_desc& p = c->desc[t];
        // a norm gain / bias that is not perturbed (frozen tensor, or eps = 0) and lies in fp32 is read where it is
        if (slot < 2) {
            alias[slot] = (o == 0 && eps_of(t) == 0.0f && wd() == ZO_W_F32) ? (float*)c->params[t].ptr : nullptr;
            if (alias[slot]) return ZO_OK;
        }
        float* op = at<float>(c->L.vec[0]) + slot * c->L.vec_stride + o;
        float* om = nb == 2 ? at<float>(c->L.vec[1]) + slot * c->L.vec_stride + o : nullptr;
        prof_scope ps(c, ZO_PROF_WEIGHT_QUANT);
        ZO_HIP(c, zo_launch_fq_weight(c->params[t].ptr, 1, (int)p.cols, 0, 0, seed, t, eps_of(t), ZO_T_F32,
                                      op, om, nullptr, nullptr, nullptr, c->st, wd()));
        return ZO_OK;
    }
    float* vec(int b, int slot) const
    {
        if (slot < 2 && alias[slot]) return alias[slot];
        return at<float>(c->L.vec[b]) + slot * c->L.vec_stride;
    }

    zo_status norm(size_t layout::per_branch::*in, size_t layout::per_branch::*out, bool has_beta)
    {
        prof_scope ps(c, ZO_PROF_OTHER);
        for (int b = 0; b < nb; ++b)
            ZO_HIP(c, zo_launch_norm(at(c->L.br[b].*in), vec(b, 0), has_beta ? vec(b, 1) : nullptr, at(c->L.br[b].*out),
                                     M, c->cfg.d_model, 1e-5f, dt(), c->st));
        return ZO_OK;
    }
    // norm followed by the per-token quantizer, fused when the row fits in registers
    zo_status norm_quant(size_t layout::per_branch::*in, bool has_beta, size_t layout::per_branch::** used)
    {
        const int d = c->cfg.d_model;
        if (c->cfg.a_bits >= 16 || !zo_norm_quant_supported(d)) {
            zo_status s_ = norm(in, &layout::per_branch::h, has_beta);
            if (s_ != ZO_OK) return s_;
            return act_quant(&layout::per_branch::h, d, used);
        }
        const bool i8 = i8_route(next_t);                // integer route: the same kernel leaves signed-byte codes
        prof_scope ps(c, ZO_PROF_ACT_QUANT);
        for (int b = 0; b < nb; ++b) {
            char* hq = at(c->L.br[b].hq);
            ZO_HIP(c, zo_launch_norm_quant(at(c->L.br[b].*in), vec(b, 0), has_beta ? vec(b, 1) : nullptr, hq,
                                           M, d, 1e-5f, c->cfg.a_bits, c->cfg.a_sym, dt(), sm_delta(b), sm_inv(b), c->st,
                                           i8 ? (int8_t*)hq : nullptr, i8 ? (float*)(hq + i8_xs_off()) : nullptr,
                                           i8 ? (float*)(hq + i8_xs_off()) + M : nullptr));
        }
        x_codes = i8;
        *used = &layout::per_branch::hq;
        return ZO_OK;
    }
    // per-token quantizer of the input of a quantized linear; returns which buffer holds X^
    zo_status act_quant(size_t layout::per_branch::*in, int K, size_t layout::per_branch::** used)
    {
        if (c->cfg.a_bits >= 16) { *used = in; return ZO_OK; }
        const bool i8 = i8_route(next_t);
        if (i8 && !zo_swiglu_quant_supported(K)) return act_codes(in, K, used);
        prof_scope ps(c, ZO_PROF_ACT_QUANT);
        for (int b = 0; b < nb; ++b) {
            char* hq = at(c->L.br[b].hq);
            if (zo_swiglu_quant_supported(K))             // row kept in registers: one read and one write per element
                ZO_HIP(c, zo_launch_swiglu_quant(at(c->L.br[b].*in), nullptr, hq, M, K, K, c->cfg.a_bits, c->cfg.a_sym,
                                                 dt(), sm_delta(b), sm_inv(b), c->st, i8 ? (int8_t*)hq : nullptr,
                                                 i8 ? (float*)(hq + i8_xs_off()) : nullptr, i8 ? (float*)(hq + i8_xs_off()) + M : nullptr));
            else
                ZO_HIP(c, zo_launch_fq_act(at(c->L.br[b].*in), at(c->L.br[b].hq), M, K, c->cfg.a_bits, c->cfg.a_sym, dt(),
                                           nullptr, nullptr, nullptr, sm_delta(b), sm_inv(b), c->st));
        }
        x_codes = i8;
        *used = &layout::per_branch::hq;
        return ZO_OK;
    }
    zo_status gemm(size_t layout::per_branch::*in, size_t layout::per_branch::*out, int N, int K, bool bias, bool relu,
                   bool residual, bool out_f32 = false, bool w_shared = false, bool swiglu = false, bool rope = false,
                   const int32_t* ce_ids = nullptr)
    {
        const int requested = nweights;
        nweights = 0;
        if (swiglu) c->routes |= ZO_ROUTE_SWIGLU_IN_GEMM;
        if (rope) c->routes |= ZO_ROUTE_ROPE_IN_GEMM;
        if (ce_ids) c->routes |= ZO_ROUTE_CE_IN_GEMM;
        if (npend > 0 && npend != requested) {           // cannot happen: the tensors of one GEMM share shape and route
            npend = 0;
            return fail(c, ZO_EUNSUPPORTED, "tensors of one GEMM took different routes");
        }
        if (npend > 0) {
            const int64_t ts_ = (int64_t)zo_tsize(dt());
            // from a few m-tiles on the kernel is fed from a fragment-ordered copy of the activations, kept in the
            // (otherwise idle) operand buffers
            bool any_packed = false;
            for (int i = 0; i < npend; ++i) any_packed = any_packed || pending[i].packed;
            // both branches' copies sit side by side in the FIRST operand buffer; the second one stays free for the fp32
            // partial sums of the packed-codes kernel's K split
            // one token, one branch (a decoding step): packed tensors take the matrix-vector kernel, which reads X as it lies
            bool all_gemv = true;
            for (int i = 0; i < npend; ++i)
                all_gemv = all_gemv && pending[i].packed && c->frozen[pending[i].t].group == c->frozen[pending[0].t].group &&
                           zo_int4_gemv_supported(M, nb, (int)c->desc[pending[i].t].rows, K, c->frozen[pending[i].t].group);
            const size_t rl_bytes = align_up(zo_fused_relayout_bytes(M, K));
            const bool relayout = (M > 32 || (any_packed && !all_gemv)) && 2 * rl_bytes <= c->L.what_bytes;
            const int64_t sxf = (int64_t)(rl_bytes / 2);
            if (relayout) {
                prof_scope ps(c, ZO_PROF_OTHER);
                ZO_HIP(c, zo_launch_fused_relayout(at(c->L.br[0].*in), nb == 2 ? (int64_t)(c->L.br[1].*in - c->L.br[0].*in) / ts_ : 0, M, K,
                                                   nb, pending[0].quantize ? c->cfg.w_bits : 0, c->cfg.w_group, at(c->L.what[0]), sxf, c->st));
            }
            bool launched[4] = {false, false, false, false};
            if (all_gemv) {
                // a decoding step: every tensor of this GEMM is a packed matrix applied to the one token -- one launch for all
                zo_fused_args fa[4];
                for (int i = 0; i < npend; ++i) {
                    const pend& pe = pending[i];
                    const zo_ctx::frozen_int4& fz = c->frozen[pe.t];
                    zo_fused_args f{};
                    f.X = at(c->L.br[0].*in);
                    f.Y = at(c->L.br[0].*out) + (size_t)pe.row0 * (out_f32 ? 4 : ts_);
                    f.bias = bias ? vec(0, 2) + pe.row0 : nullptr;
                    f.residual = residual ? f.Y : nullptr;
                    f.M = M; f.N = (int)c->desc[pe.t].rows; f.K = K; f.nb = nb; f.ldY = N;
                    f.codes = fz.codes; f.step16 = fz.step; f.zp = fz.zp; f.group = fz.group;
                    f.relu = relu; f.out_f32 = out_f32;
                    fa[i] = f;
                }
                c->routes |= ZO_ROUTE_FUSED_INT4;
                prof_scope ps(c, ZO_PROF_FUSED_INT4);
                ZO_HIP(c, zo_launch_int4_gemv_multi(fa, npend, c->st));
                npend = 0;
                return ZO_OK;
            }
            for (int i = 0; i < npend; ++i) {
                if (launched[i]) continue;
                const pend& pe = pending[i];
                const param_desc& p = c->desc[pe.t];
                zo_fused_args f{};
                f.X = at(c->L.br[0].*in);
                if (relayout) { f.Xfrag = at(c->L.what[0]); f.strideXfrag = sxf; }
                f.W = c->params[pe.t].ptr;
                f.wdtype = wd();
                f.Y = at(c->L.br[0].*out) + (size_t)pe.row0 * (out_f32 ? 4 : ts_);
                f.bias = bias ? vec(0, 2) + pe.row0 : nullptr;
                f.residual = residual ? f.Y : nullptr;
                f.M = M; f.N = (int)p.rows; f.K = K; f.nb = nb;
                f.ldY = N;
                if (nb == 2) {
                    f.strideX = (int64_t)(c->L.br[1].*in - c->L.br[0].*in) / ts_;
                    f.strideY = (int64_t)(c->L.br[1].*out - c->L.br[0].*out) / (out_f32 ? 4 : ts_);
                    f.strideBias = (int64_t)(c->L.vec[1] - c->L.vec[0]) / 4;
                    f.strideRes = f.strideY;
                }
                f.bits = pe.quantize ? c->cfg.w_bits : 0;
                f.group = c->cfg.w_group;
                f.eps = eps_of(pe.t);
                f.relu = relu;
                f.out_f32 = out_f32;
                c->routes |= pe.packed ? ZO_ROUTE_FUSED_INT4 : ZO_ROUTE_FUSED_SMALL_M;
                prof_scope ps(c, pe.packed ? ZO_PROF_FUSED_INT4 : ZO_PROF_FUSED);   // one bracket per kernel launch
                if (pe.packed) {
                    const zo_ctx::frozen_int4& fz = c->frozen[pe.t];
                    f.codes = fz.codes; f.step16 = fz.step; f.zp = fz.zp; f.group = fz.group;
                    if (zo_int4_gemv_supported(M, nb, f.N, K, f.group)) {
                        ZO_HIP(c, zo_launch_int4_gemv(f, c->st));
                        continue;
                    }
                    // split-K form when its partial sums fit into the second (idle) operand buffer
                    if (relayout && zo_int4_splitk_scratch_bytes(M, f.N, K, f.group) <= c->L.what_bytes)
                        ZO_HIP(c, zo_launch_int4_gemm_splitk(f, at(c->L.what[1]), c->st));
                    else
                        ZO_HIP(c, zo_launch_int4_gemm_fused(f, c->st));
                    continue;
                }
                // a later tensor of the same shape and settings (query and value projections, gate and up) shares the launch:
                // together their workgroups leave fewer CUs idle in the last round
                int j = -1;
                for (int k2 = i + 1; k2 < npend && j < 0; ++k2) {
                    const pend& pk = pending[k2];
                    if (!launched[k2] && !pk.packed && pk.quantize == pe.quantize && c->desc[pk.t].rows == p.rows &&
                        eps_of(pk.t) == f.eps)
                        j = k2;
                }
                if (j >= 0) {
                    const pend& pk = pending[j];
                    zo_fused_second f2{};
                    f2.W = c->params[pk.t].ptr;
                    f2.Y = at(c->L.br[0].*out) + (size_t)pk.row0 * (out_f32 ? 4 : ts_);
                    f2.bias = bias ? vec(0, 2) + pk.row0 : nullptr;
                    f2.residual = residual ? f2.Y : nullptr;
                    f2.tid = pk.t;
                    launched[j] = true;
                    ZO_HIP(c, zo_launch_fq_gemm_fused_pair(f, f2, seed, pe.t, c->st));
                    continue;
                }
                ZO_HIP(c, zo_launch_fq_gemm_fused(f, seed, pe.t, c->st));
            }
            npend = 0;
            return ZO_OK;
        }
        if (w_codes != x_codes) {
            w_codes = x_codes = false;
            return fail(c, ZO_EUNSUPPORTED, "integer route: operands of one GEMM prepared differently");
        }
        if (w_codes) {
            w_codes = x_codes = false;
            if (ce_ids || w_shared || rope || (out_f32 && dt() != ZO_T_F32)) return fail(c, ZO_EUNSUPPORTED, "integer route: epilogue");
            zo_i8_gemm_args g{};
            char* x0 = at(c->L.br[0].*in);
            char* w0 = at(c->L.what[0]);
            g.X = (const int8_t*)x0; g.W = (const int8_t*)w0;
            g.xs = (const float*)(x0 + i8_xs_off()); g.xo = g.xs + M;
            g.ws = (const float*)(w0 + i8_ws_off()); g.wr = (const float*)(w0 + i8_wr_off());
            g.Y = at(c->L.br[0].*out);
            g.bias = bias ? vec(0, 2) : nullptr;
            g.residual = residual ? g.Y : nullptr;
            g.M = M; g.N = N; g.K = K; g.batch = nb;
            g.sgroup = c->cfg.w_group > 0 ? c->cfg.w_group : K;
            g.relu = relu;
            g.epi = swiglu ? 1 : 0;
            if (nb == 2) {
                const int64_t ts_ = (int64_t)zo_tsize(dt());
                g.strideX = (int64_t)(c->L.br[1].*in - c->L.br[0].*in);
                g.strideXs = g.strideX / 4;
                g.strideW = (int64_t)(c->L.what[1] - c->L.what[0]);
                g.strideWs = g.strideWr = g.strideW / 4;
                g.strideY = (int64_t)(c->L.br[1].*out - c->L.br[0].*out) / ts_;
                g.strideBias = (int64_t)(c->L.vec[1] - c->L.vec[0]) / 4;
                g.strideRes = g.strideY;
            }
            c->routes |= ZO_ROUTE_INT8_MMA;
            prof_scope ps(c, ZO_PROF_GEMM);
            ZO_HIP(c, zo_launch_gemm_i8(g, dt() == ZO_T_F32, c->st));
            return ZO_OK;
        }
        zo_gemm_args a{};
        a.X = at(c->L.br[0].*in);
        a.W = at(c->L.what[0]);
        a.Y = at(c->L.br[0].*out);
        a.bias = bias ? vec(0, 2) : nullptr;
        a.residual = residual ? at(c->L.br[0].*out) : nullptr;
        a.M = M; a.N = N; a.K = K;
        a.batch = nb;
        const int64_t ts = (int64_t)zo_tsize(dt());
        if (nb == 2) {
            a.strideX = (int64_t)(c->L.br[1].*in - c->L.br[0].*in) / ts;
            a.strideW = w_shared ? 0 : (int64_t)(c->L.what[1] - c->L.what[0]) / ts;
            a.strideY = (int64_t)(c->L.br[1].*out - c->L.br[0].*out) / (out_f32 ? 4 : ts);
            a.strideBias = (int64_t)(c->L.vec[1] - c->L.vec[0]) / 4;
            a.strideRes = a.strideY;
        }
        a.relu = relu;
        a.out_f32 = out_f32;
        a.dtype = dt();
        a.swiglu = swiglu ? 1 : 0;
        if (rope) {
            a.rope_cos = at<float>(c->L.rope_cos) + (size_t)pos0 * (c->cfg.d_model / c->cfg.n_heads / 2);
            a.rope_sin = at<float>(c->L.rope_sin) + (size_t)pos0 * (c->cfg.d_model / c->cfg.n_heads / 2);
            a.rope_cols = 2 * c->cfg.d_model;
            a.rope_S = S;
        }
        if (ce_ids) {                                    // `out` receives the partial results, then the target logits
            a.ce_part = at<float>(c->L.br[0].*out);
            a.ce_tgt = a.ce_part + zo_gemm_ce_part_floats(M, N);
            a.ce_ids = ce_ids;
            a.ce_S = S;
            a.stridePart = a.strideTgt = nb == 2 ? (int64_t)(c->L.br[1].*out - c->L.br[0].*out) / 4 : 0;
        }
        if (c->L.kpart_bytes && !swiglu && !rope && !ce_ids) {
            a.ks_part = at<float>(c->L.kpart);
            a.ks_part_bytes = c->L.kpart_bytes;
            const size_t need = zo_gemm_splitk_bytes(M, N, K, nb, dt());
            if (need && need <= a.ks_part_bytes) c->routes |= ZO_ROUTE_GEMM_SPLIT_K;
        }
        prof_scope ps(c, ZO_PROF_GEMM);
        ZO_HIP(c, zo_launch_gemm(a, c->st));
        return ZO_OK;
    }
};

#define ZO_TRY(x) do { zo_status s_ = (x); if (s_ != ZO_OK) return s_; } while (0)

// Generator mode (inf != NULL; one sequence, eps = 0, nb = 1): rows are positions pos0 .. pos0 + S - 1; every layer's keys (after
// the rotary embedding) and values are appended to the cache; with pos0 > 0 (S = 1) the query attends to the cached rows
// instead of the batch; no loss -- the logits of the LAST row go to logits_out.
struct infer_opts { char* kv; int kv_max_seq; int pos0; float* logits_out; };

zo_status run_forward(zo_ctx* c, const void* ids_or_x, const float* target, int B, int S, uint64_t seed,
                      float eps, int nb, float* loss_out /* dev fp32[nb] */, const infer_opts* inf = nullptr)
{
    const zo_config& cfg = c->cfg;
    using PB = layout::per_branch;
    c->routes = 0;
    fwd F{c, nb, eps, seed, 0, S};
    if (inf) F.pos0 = inf->pos0;
    const int dt = cfg.act_dtype;
    const size_t ts = zo_tsize(dt);
    if (cfg.arch == ZO_ARCH_LINEAR) {
        const int M = B, K = cfg.d_model, N = cfg.d_ffn;
        F.M = M;
        c->last_M = M;
        ZO_TRY(F.smooth_prepare(0));
        ZO_TRY(F.weights(0, 0, true));
        ZO_TRY(F.bias_shift(0, 0, false));
        // input X is given by the caller; quantize into hq (the same X^ for both branches unless the
        // perturbed smoothing makes them differ)
        if (F.i8_route(0)) {
            // integer route: codes of X (the same for both branches) into hq of branch 0 -- and of branch 1, which the batched
            // launch reads through its stride
            prof_scope ps(c, ZO_PROF_ACT_QUANT);
            for (int b = 0; b < nb; ++b) {
                char* hq = F.at(c->L.br[b].hq);
                ZO_HIP(c, zo_launch_act_codes_i8(ids_or_x, (int8_t*)hq, (float*)(hq + F.i8_xs_off()), (float*)(hq + F.i8_xs_off()) + M, M, K,
                                                 cfg.a_bits, cfg.a_sym, dt, c->st));
            }
            F.x_codes = true;
            ZO_TRY(F.gemm(&PB::hq, &PB::logits, N, K, false, false, false));
            prof_scope ps2(c, ZO_PROF_OTHER);
            for (int b = 0; b < nb; ++b) {
                ZO_HIP(c, zo_launch_sqerr_rows(F.at(c->L.br[b].logits), target, F.at<float>(c->L.br[b].rowloss), M, N, dt, c->st));
                ZO_HIP(c, zo_launch_reduce_loss(F.at<float>(c->L.br[b].rowloss), M, 1.0f / ((float)M * (float)N), loss_out + b, c->st));
            }
            ZO_HIP(c, zo_launch_i8_flag_to_loss(F.i8_flag(), loss_out, nb, c->st));
            return ZO_OK;
        }
        zo_gemm_args a{};
        const void* xin = ids_or_x;
        const bool two_x = nb == 2 && F.sm_on;
        if (cfg.a_bits < 16) {
            prof_scope ps(c, ZO_PROF_ACT_QUANT);
            for (int b = 0; b < (two_x ? 2 : 1); ++b)
                ZO_HIP(c, zo_launch_fq_act(ids_or_x, F.at(c->L.br[b].hq), M, K, cfg.a_bits, cfg.a_sym, dt, nullptr, nullptr, nullptr,
                                           F.sm_delta(b), F.sm_inv(b), c->st));
            xin = F.at(c->L.br[0].hq);
        }
        a.X = xin; a.W = F.at(c->L.what[0]); a.Y = F.at(c->L.br[0].logits);
        a.bias = F.sm_on ? F.vec(0, 2) : nullptr;
        a.M = M; a.N = N; a.K = K; a.batch = nb; a.dtype = dt;
        if (nb == 2) {
            a.strideX = two_x ? (int64_t)(c->L.br[1].hq - c->L.br[0].hq) / (int64_t)ts : 0;
            a.strideBias = (int64_t)(c->L.vec[1] - c->L.vec[0]) / 4;
            a.strideW = (int64_t)(c->L.what[1] - c->L.what[0]) / (int64_t)ts;
            a.strideY = (int64_t)(c->L.br[1].logits - c->L.br[0].logits) / (int64_t)ts;
        }
        if (F.npend > 0) {                               // small M: tiles of Q(W +- eps u) built inside the GEMM kernel
            zo_fused_args fa{};
            fa.X = a.X; fa.W = c->params[0].ptr; fa.wdtype = F.wd(); fa.Y = a.Y; fa.bias = a.bias;
            fa.M = M; fa.N = N; fa.K = K; fa.nb = nb; fa.ldY = N;
            fa.strideX = a.strideX; fa.strideY = a.strideY; fa.strideBias = a.strideBias;
            fa.bits = cfg.w_bits; fa.group = cfg.w_group; fa.eps = F.eps_of(0);
            F.npend = 0;
            c->routes |= ZO_ROUTE_FUSED_SMALL_M;
            if (M > 32 && zo_fused_relayout_bytes(M, K) <= c->L.what_bytes) {
                prof_scope ps(c, ZO_PROF_OTHER);
                fa.Xfrag = F.at(c->L.what[0]);
                fa.strideXfrag = (int64_t)(c->L.what[1] - c->L.what[0]) / 2;
                ZO_HIP(c, zo_launch_fused_relayout(fa.X, fa.strideX, M, K, nb, fa.bits, fa.group, F.at(c->L.what[0]), fa.strideXfrag, c->st));
            }
            prof_scope ps(c, ZO_PROF_FUSED);
            ZO_HIP(c, zo_launch_fq_gemm_fused(fa, seed, 0, c->st));
        } else {
            prof_scope ps(c, ZO_PROF_GEMM);
            ZO_HIP(c, zo_launch_gemm(a, c->st));
        }
        prof_scope ps(c, ZO_PROF_OTHER);
        for (int b = 0; b < nb; ++b) {
            ZO_HIP(c, zo_launch_sqerr_rows(F.at(c->L.br[b].logits), target, F.at<float>(c->L.br[b].rowloss), M, N, dt, c->st));
            ZO_HIP(c, zo_launch_reduce_loss(F.at<float>(c->L.br[b].rowloss), M, 1.0f / ((float)M * (float)N), loss_out + b, c->st));
        }
        return ZO_OK;
    }

    const int M = B * S, d = cfg.d_model, f = cfg.d_ffn, V = cfg.vocab, H = cfg.n_heads, dh = d / H;
    F.M = M;
    c->last_M = M;
    const bool llama = cfg.arch == ZO_ARCH_LLAMA;
    const int32_t* ids = (const int32_t*)ids_or_x;
    int t = 0;                                           // running tensor number
    // embedding
    {
        const int t_tok = t++;
        const int t_pos = llama ? -1 : t++;
        prof_scope ps(c, ZO_PROF_OTHER);
        for (int b = 0; b < nb; ++b) {
            const float sgn = (b == 0) ? 1.0f : -1.0f;
            const char* pos_tab = llama ? nullptr : (const char*)c->params[t_pos].ptr +
                                                     (size_t)F.pos0 * d * (F.wd() == ZO_W_F16 ? 2 : 4);   // (offset rows: eps = 0 there)
            ZO_HIP(c, zo_launch_embed(ids, c->params[t_tok].ptr, pos_tab,
                                      F.at(c->L.br[b].x), M, S, d, V, seed, t_tok, llama ? 0 : t_pos,
                                      sgn * F.eps_of(t_tok), llama ? 0.0f : sgn * F.eps_of(t_pos), dt, c->st, F.wd()));
        }
    }
    size_t PB::* xin;
    for (int l = 0; l < cfg.n_layers; ++l) {
        // ---- attention block
        ZO_TRY(F.vector(t++, 0));
        if (!llama) ZO_TRY(F.vector(t++, 1));
        ZO_TRY(F.smooth_prepare(t));                     // t: wq, which carries the pair of the q/k/v input
        ZO_TRY(F.norm_quant(&PB::x, !llama, &xin));
        const int tstep = llama ? 1 : 2;                 // OPT interleaves the biases
        bool sh = F.frozen(t) && F.frozen(t + tstep) && F.frozen(t + 2 * tstep);
        // one quantized linear: weights of tensor t into rows [row0, ..) of the operand buffer, its bias
        // (OPT-shaped) into slot 2, the smoothing term of Eq. 4 added to it
        auto linear = [&](int64_t row0, bool shared, int ilv = 0) -> zo_status {
            const int tw = t++;
            ZO_TRY(F.weights(tw, row0, true, shared, ilv));
            if (!llama) ZO_TRY(F.vector(t++, 2, row0));
            return F.bias_shift(tw, row0, !llama);
        };
        const bool bias = !llama || cfg.learn_smooth;
        const bool rope_fused = llama && F.rope_in_gemm(t);      // head blocks permuted in the operand, rotation in the epilogue
        F.gemm_N = 3 * d;
        for (int i = 0; i < 3; ++i) ZO_TRY(linear((int64_t)i * d, sh, rope_fused ? 3 : 0));
        ZO_TRY(F.gemm(xin, &PB::qkv, 3 * d, d, bias, false, false, false, sh, false, rope_fused));
        // a decoding step (one new row, rows cached before it): rotation, cache append, attention over key ranges and the
        // per-token quantizer of the attention output run in two launches further down
        const bool dec_split = inf && inf->pos0 > 0 && M == 1 && zo_decode_attention_split_supported(H, dh) &&
                               zo_decode_attention_split_bytes(inf->pos0 + 1, H, dh) <= c->L.what_bytes;
        for (int b = 0; b < nb && !dec_split; ++b) {
            prof_scope ps(c, ZO_PROF_ATTENTION);
            char* qkv = F.at(c->L.br[b].qkv);
            if (llama && !rope_fused)
                ZO_HIP(c, zo_launch_rope(qkv, qkv + (size_t)d * ts, F.at<float>(c->L.rope_cos) + (size_t)F.pos0 * (dh / 2),
                                         F.at<float>(c->L.rope_sin) + (size_t)F.pos0 * (dh / 2), M, S, H, dh, 3 * d, dt, c->st));
            if (inf) {
                // keys and values of these rows join the cache: [layer][K | V][kv_max_seq][d]
                char* kc = inf->kv + ((size_t)l * 2) * inf->kv_max_seq * d * ts;
                char* vc = kc + (size_t)inf->kv_max_seq * d * ts;
                ZO_HIP(c, hipMemcpy2DAsync(kc + (size_t)inf->pos0 * d * ts, (size_t)d * ts, qkv + (size_t)d * ts, (size_t)3 * d * ts,
                                           (size_t)d * ts, (size_t)M, hipMemcpyDeviceToDevice, c->st));
                ZO_HIP(c, hipMemcpy2DAsync(vc + (size_t)inf->pos0 * d * ts, (size_t)d * ts, qkv + (size_t)2 * d * ts, (size_t)3 * d * ts,
                                           (size_t)d * ts, (size_t)M, hipMemcpyDeviceToDevice, c->st));
                if (inf->pos0 > 0) {                     // one new query over everything cached so far
                    ZO_HIP(c, zo_launch_decode_attention(qkv, kc, vc, F.at(c->L.br[b].att), inf->pos0 + 1, H, dh, dt, c->st));
                    continue;
                }
            }
            if (zo_flash_attention_supported(dh, dt))
                ZO_HIP(c, zo_launch_flash_attention(qkv, qkv + (size_t)d * ts, qkv + (size_t)2 * d * ts, F.at(c->L.br[b].att),
                                                    B, S, H, dh, 3 * d, c->st));
            else
                ZO_HIP(c, zo_launch_attention(qkv, qkv + (size_t)d * ts, qkv + (size_t)2 * d * ts, F.at(c->L.br[b].att),
                                              B, S, H, dh, 3 * d, dt, c->st));
        }
        ZO_TRY(F.smooth_prepare(t));                     // wo
        if (dec_split) {
            prof_scope ps(c, ZO_PROF_ATTENTION);
            char* kc = inf->kv + ((size_t)l * 2) * inf->kv_max_seq * d * ts;
            char* vc = kc + (size_t)inf->kv_max_seq * d * ts;
            const bool aq = cfg.a_bits < 16;
            ZO_HIP(c, zo_launch_decode_attention_split(F.at(c->L.br[0].qkv), kc, vc,
                                                       llama ? F.at<float>(c->L.rope_cos) + (size_t)inf->pos0 * (dh / 2) : nullptr,
                                                       llama ? F.at<float>(c->L.rope_sin) + (size_t)inf->pos0 * (dh / 2) : nullptr,
                                                       F.at(c->L.what[1]), F.at(c->L.br[0].att), aq ? F.at(c->L.br[0].hq) : nullptr,
                                                       inf->pos0 + 1, H, dh, cfg.a_bits, cfg.a_sym, F.sm_delta(0), F.sm_inv(0), dt, c->st));
            xin = aq ? &PB::hq : &PB::att;
        } else {
            ZO_TRY(F.act_quant(&PB::att, d, &xin));
        }
        sh = F.frozen(t);
        F.gemm_N = d;
        ZO_TRY(linear(0, sh));
        ZO_TRY(F.gemm(xin, &PB::x, d, d, bias, false, true, false, sh));
        // ---- feed-forward block
        ZO_TRY(F.vector(t++, 0));
        if (!llama) ZO_TRY(F.vector(t++, 1));
        ZO_TRY(F.smooth_prepare(t));                     // w_gate / fc1
        ZO_TRY(F.norm_quant(&PB::x, !llama, &xin));
        bool act_done = false;
        if (llama && F.swiglu_in_gemm(t)) {
            // gate and up rows interleaved in the operand buffer; the GEMM writes silu(gate) * up
            sh = F.frozen(t) && F.frozen(t + 1);
            F.gemm_N = 2 * f;
            ZO_TRY(F.weights(t++, 0, true, sh, 1));
            ZO_TRY(F.weights(t++, 0, true, sh, 2));
            ZO_TRY(F.gemm(xin, &PB::act, 2 * f, d, false, false, false, false, sh, true));
        } else if (llama) {
            sh = F.frozen(t) && F.frozen(t + 1);
            F.gemm_N = 2 * f;
            ZO_TRY(linear(0, sh));
            ZO_TRY(linear(f, sh));
            ZO_TRY(F.gemm(xin, &PB::gu, 2 * f, d, bias, false, false, false, sh));
            ZO_TRY(F.smooth_prepare(t));                 // w_down: its input is the SwiGLU output
            act_done = cfg.a_bits < 16 && zo_swiglu_quant_supported(f);
            const bool i8 = act_done && F.i8_route(t);   // integer route: the same kernel leaves signed-byte codes
            prof_scope ps(c, act_done ? ZO_PROF_ACT_QUANT : ZO_PROF_OTHER);
            for (int b = 0; b < nb; ++b) {
                char* gu = F.at(c->L.br[b].gu);
                char* hq = F.at(c->L.br[b].hq);
                if (act_done)
                    ZO_HIP(c, zo_launch_swiglu_quant(gu, gu + (size_t)f * ts, hq, M, f, 2 * f,
                                                     cfg.a_bits, cfg.a_sym, dt, F.sm_delta(b), F.sm_inv(b), c->st,
                                                     i8 ? (int8_t*)hq : nullptr, i8 ? (float*)(hq + F.i8_xs_off()) : nullptr,
                                                     i8 ? (float*)(hq + F.i8_xs_off()) + M : nullptr));
                else
                    ZO_HIP(c, zo_launch_swiglu(gu, gu + (size_t)f * ts, F.at(c->L.br[b].act), M, f, 2 * f, dt, c->st));
            }
        } else {
            sh = F.frozen(t);
            F.gemm_N = f;
            ZO_TRY(linear(0, sh));
            ZO_TRY(F.gemm(xin, &PB::act, f, d, true, true, false, false, sh));
            ZO_TRY(F.smooth_prepare(t));                 // fc2
        }
        if (act_done) { xin = &PB::hq; F.x_codes = F.i8_route(t); }
        else ZO_TRY(F.act_quant(&PB::act, f, &xin));
        sh = F.frozen(t);
        F.gemm_N = d;
        ZO_TRY(linear(0, sh));
        ZO_TRY(F.gemm(xin, &PB::x, d, f, bias, false, true, false, sh));
    }
    // ---- head
    ZO_TRY(F.vector(t++, 0));
    if (!llama) ZO_TRY(F.vector(t++, 1));
    if (inf) {
        // generator: only the last row is normalised (into row 0 of h) and multiplied with the lm_head; fp32 logits out
        {
            prof_scope ps(c, ZO_PROF_OTHER);
            ZO_HIP(c, zo_launch_norm(F.at(c->L.br[0].x) + (size_t)(M - 1) * d * ts, F.vec(0, 0), llama ? nullptr : F.vec(0, 1),
                                     F.at(c->L.br[0].h), 1, d, 1e-5f, dt, c->st));
        }
        F.M = 1;
        ZO_TRY(F.weights(t++, 0, false));
        ZO_TRY(F.gemm(&PB::h, &PB::logits, V, d, false, false, false, true));
        F.M = M;
        ZO_HIP(c, hipMemcpyAsync(inf->logits_out, F.at(c->L.br[0].logits), (size_t)V * sizeof(float), hipMemcpyDeviceToDevice, c->st));
        return ZO_OK;
    }
    ZO_TRY(F.norm(&PB::x, &PB::h, !llama));
    ZO_TRY(F.weights(t++, 0, false));
    // large bf16 forwards: the logits are never stored, the GEMM's epilogue leaves per-tile (maximum, sum of exponentials)
    const bool ce_in_gemm = F.npend == 0 && zo_gemm_ce_supported(M, V, d, F.dt());
    ZO_TRY(F.gemm(&PB::h, &PB::logits, V, d, false, false, false, true, false, false, false, ce_in_gemm ? ids : nullptr));
    prof_scope ps(c, ZO_PROF_OTHER);
    for (int b = 0; b < nb; ++b) {
        if (ce_in_gemm) {
            const float* part = F.at<float>(c->L.br[b].logits);
            ZO_HIP(c, zo_launch_ce_combine(part, part + zo_gemm_ce_part_floats(M, V), F.at<float>(c->L.br[b].rowloss), M, S, V, c->st));
        } else
            ZO_HIP(c, zo_launch_ce_rows(F.at<float>(c->L.br[b].logits), ids, F.at<float>(c->L.br[b].rowloss), M, S, V, c->st));
        ZO_HIP(c, zo_launch_reduce_loss(F.at<float>(c->L.br[b].rowloss), M, 1.0f / ((float)B * (float)(S - 1)), loss_out + b, c->st));
    }
    if (c->routes & ZO_ROUTE_INT8_MMA) ZO_HIP(c, zo_launch_i8_flag_to_loss(F.i8_flag(), loss_out, nb, c->st));
    return ZO_OK;
}

zo_status check_batch(zo_ctx* c, const void* ids, const float* target, int B, int S)
{
    if (!c) return ZO_EINVAL;
    if (!ids) return fail(c, ZO_EINVAL, "ids / input is NULL");
    if (B <= 0 || S <= 0) return fail(c, ZO_EINVAL, "B and S must be positive");
    if (c->cfg.arch == ZO_ARCH_LINEAR) {
        if (!target) return fail(c, ZO_EINVAL, "target is NULL");
        if (S != 1) return fail(c, ZO_ESHAPE, "the linear arch takes S = 1");
        if (!aligned16(target)) return fail(c, ZO_EALIGN, "target not 16-byte aligned");
    } else {
        if (S < 2) return fail(c, ZO_ESHAPE, "next-token loss needs S >= 2");
        if (S > c->cfg.max_seq) return fail(c, ZO_ESHAPE, "S exceeds max_seq");
    }
    if (!aligned16(ids)) return fail(c, ZO_EALIGN, "ids / input not 16-byte aligned");
    for (size_t i = 0; i < c->params.size(); ++i)
        if (!c->params[i].ptr && !c->frozen[i].codes) return fail(c, ZO_EINVAL, "a tensor has neither fp32 nor packed storage");
    if ((int64_t)B * S > (int64_t)c->max_B * c->max_S || S > c->max_S)
        return fail(c, ZO_EWORKSPACE, "batch larger than the one the context was created for");
    return ZO_OK;
}

}  // namespace

// =============================================================================================
extern "C" {

int32_t zo_num_params(const zo_config* cfg)
{
    std::vector<param_desc> p;
    if (!cfg || !describe_params(*cfg, p)) return 0;
    return (int32_t)p.size();
}

int64_t zo_param_numel(const zo_config* cfg, int32_t index)
{
    std::vector<param_desc> p;
    if (!cfg || !describe_params(*cfg, p) || index < 0 || index >= (int32_t)p.size()) return -1;
    return p[index].rows * p[index].cols;
}

size_t zo_workspace_bytes(const zo_config* cfg, int32_t B, int32_t S)
{
    if (!cfg || B <= 0 || S <= 0 || check_config(*cfg) != ZO_OK) return 0;
    return make_layout(*cfg, B, S).total;
}

zo_status zo_init(const zo_config* cfg, const zo_tensor* params, int32_t n_params,
                  void* workspace, size_t workspace_bytes, int32_t max_B, int32_t max_S,
                  void* hip_stream, zo_ctx** out)
{
    if (!cfg || !params || !workspace || !out || max_B <= 0 || max_S <= 0) return ZO_EINVAL;
    *out = nullptr;
    zo_status s = check_config(*cfg);
    if (s != ZO_OK) return s;
    std::vector<param_desc> desc;
    describe_params(*cfg, desc);
    if (n_params != (int32_t)desc.size()) return ZO_EINVAL;
    for (int i = 0; i < n_params; ++i) {
        // a frozen linear of the lightweight variant may come without fp32 storage: its packed form
        // is attached afterwards (zo_attach_frozen_int4)
        const bool may_be_packed = cfg->lightweight && !params[i].trainable && desc[i].quantized;
        if (!params[i].ptr && !may_be_packed) return ZO_EINVAL;
        if (params[i].numel != desc[i].rows * desc[i].cols) return ZO_ESHAPE;
        if (!aligned16(params[i].ptr)) return ZO_EALIGN;
    }
    if (cfg->arch != ZO_ARCH_LINEAR && max_S > cfg->max_seq) return ZO_ESHAPE;
    if (cfg->arch == ZO_ARCH_LINEAR && max_S != 1) return ZO_ESHAPE;      // its workspace is sized for max_B rows
    if (!aligned16(workspace)) return ZO_EALIGN;
    layout L = make_layout(*cfg, max_B, max_S);
    if (workspace_bytes < L.total) return ZO_EWORKSPACE;
    zo_ctx* c = new zo_ctx();
    c->cfg = *cfg;
    c->params.assign(params, params + n_params);
    c->desc = desc;
    c->frozen.assign(n_params, zo_ctx::frozen_int4{nullptr, nullptr, nullptr, 0});
    c->ws = (char*)workspace;
    c->ws_bytes = workspace_bytes;
    c->max_B = max_B;
    c->max_S = max_S;
    c->st = (hipStream_t)hip_stream;
    c->L = L;
    c->last_M = 0;
    if (cfg->arch == ZO_ARCH_LLAMA) {
        // rotary angle table: cos / sin of pos * 10000^(-2i/dh), evaluated in fp64, stored fp32
        const int dh = cfg->d_model / cfg->n_heads, half = dh / 2;
        std::vector<float>&cs = c->rope_host[0], &sn = c->rope_host[1];
        cs.resize((size_t)cfg->max_seq * half);
        sn.resize((size_t)cfg->max_seq * half);
        for (int p = 0; p < cfg->max_seq; ++p)
            for (int i = 0; i < half; ++i) {
                const double ang = (double)p * std::pow(10000.0, -2.0 * (double)i / (double)dh);
                cs[(size_t)p * half + i] = (float)std::cos(ang);
                sn[(size_t)p * half + i] = (float)std::sin(ang);
            }
        // asynchronous: the host copies belong to the context, so nothing has to be waited for here
        hipError_t e = hipMemcpyAsync(c->ws + L.rope_cos, cs.data(), cs.size() * 4, hipMemcpyHostToDevice, c->st);
        if (e == hipSuccess) e = hipMemcpyAsync(c->ws + L.rope_sin, sn.data(), sn.size() * 4, hipMemcpyHostToDevice, c->st);
        if (e != hipSuccess) { delete c; return ZO_EHIP; }
    }
    if (cfg->mma == ZO_MMA_INT8) {
        // the integer route's overflow flag starts clear (afterwards the forward that reads it clears it again)
        if (hipMemsetAsync(c->ws + L.scalars + 15 * sizeof(float), 0, sizeof(int), c->st) != hipSuccess) { delete c; return ZO_EHIP; }
    }
    *out = c;
    return ZO_OK;
}

zo_status zo_attach_frozen_int4(zo_ctx* ctx, int32_t index, const void* codes, const void* step_f16, const int16_t* zp,
                                int32_t group)
{
    if (!ctx) return ZO_EINVAL;
    if (index < 0 || index >= (int32_t)ctx->params.size()) return fail(ctx, ZO_EINVAL, "tensor index out of range");
    if (!ctx->cfg.lightweight || ctx->params[index].trainable) return fail(ctx, ZO_EINVAL, "only frozen tensors of a lightweight configuration take packed storage");
    if (!ctx->desc[index].quantized) return fail(ctx, ZO_EINVAL, "only quantized linears take packed storage");
    if (!codes || !step_f16 || !zp) return fail(ctx, ZO_EINVAL, "NULL packed storage");
    if (!zo_int4_group_supported((int)ctx->desc[index].cols, group)) return fail(ctx, ZO_ESHAPE, "group must be a power of two in 8..512 dividing the in-features");
    if (!aligned16(codes) || ((uintptr_t)step_f16 & 1) || ((uintptr_t)zp & 1)) return fail(ctx, ZO_EALIGN, "packed storage misaligned");
    if (!ctx->frozen[index].codes) ctx->n_packed += 1;
    {
        const int cg = ctx->cfg.w_group > 0 ? ctx->cfg.w_group : 0;
        auto slab = [](int g) { return g >= 128 ? 128 : g; };
        if (ctx->cfg.w_bits == 0 || cg < 32 || cg > 128 || slab(cg) != slab(group)) ctx->packed_fusable = false;
    }
    ctx->frozen[index] = zo_ctx::frozen_int4{codes, step_f16, zp, group};
    return ZO_OK;
}

zo_status zo_destroy(zo_ctx* ctx)
{
    if (ctx)
        for (hipEvent_t e : ctx->ev_pool) (void)hipEventDestroy(e);
    delete ctx;
    return ZO_OK;
}

zo_status zo_profile_begin(zo_ctx* ctx) { return zo_profile_begin_mask(ctx, 0xFFFFFFFFu); }

zo_status zo_profile_begin_mask(zo_ctx* ctx, uint32_t category_mask)
{
    if (!ctx) return ZO_EINVAL;
    ctx->prof = true;
    ctx->prof_mask = category_mask;
    ctx->ev_used = 0;
    ctx->ev_cat.clear();
    return ZO_OK;
}

zo_status zo_profile_end(zo_ctx* ctx, float* ms, int32_t* launches)
{
    if (!ctx || !ms || !launches) return ZO_EINVAL;
    ctx->prof = false;
    for (int i = 0; i < ZO_PROF_CATEGORIES; ++i) { ms[i] = 0.0f; launches[i] = 0; }
    ZO_HIP(ctx, hipStreamSynchronize(ctx->st));
    for (size_t i = 0; i < ctx->ev_cat.size(); ++i) {
        float t = 0.0f;
        ZO_HIP(ctx, hipEventElapsedTime(&t, ctx->ev_pool[2 * i], ctx->ev_pool[2 * i + 1]));
        ms[ctx->ev_cat[i]] += t;
        launches[ctx->ev_cat[i]] += 1;
    }
    ctx->ev_used = 0;
    ctx->ev_cat.clear();
    return ZO_OK;
}

const char* zo_last_error(const zo_ctx* ctx) { return ctx ? ctx->err.c_str() : "null context"; }

zo_status zo_forward_quant(zo_ctx* ctx, const void* ids, const float* target, int32_t B, int32_t S,
                           uint64_t seed, float eps_signed, float* loss_dev)
{
    zo_status s = check_batch(ctx, ids, target, B, S);
    if (s != ZO_OK) return s;
    if (!loss_dev) return fail(ctx, ZO_EINVAL, "loss_dev is NULL");
    return run_forward(ctx, ids, target, B, S, seed, eps_signed, 1, loss_dev);
}

// ---- generator on the quantized model ----
size_t zo_kv_cache_bytes(const zo_config* cfg, int32_t kv_max_seq)
{
    if (!cfg || kv_max_seq <= 0 || cfg->arch == ZO_ARCH_LINEAR || check_config(*cfg) != ZO_OK) return 0;
    return (size_t)cfg->n_layers * 2 * (size_t)kv_max_seq * (size_t)cfg->d_model * zo_tsize(cfg->act_dtype);
}

namespace {
zo_status check_infer(zo_ctx* ctx, const void* ids, int S, int pos0, const void* kv, int kv_max_seq, const float* logits)
{
    if (!ctx) return ZO_EINVAL;
    if (ctx->cfg.arch == ZO_ARCH_LINEAR) return fail(ctx, ZO_EUNSUPPORTED, "the generator needs a decoder");
    if (ctx->cfg.learn_clip || ctx->cfg.learn_smooth) return fail(ctx, ZO_EUNSUPPORTED, "the generator runs the plain quantizer");
    if (!ids || !kv || !logits) return fail(ctx, ZO_EINVAL, "NULL argument");
    if (S < 1 || pos0 < 0 || kv_max_seq < 1) return fail(ctx, ZO_EINVAL, "S, pos, kv_max_seq must be positive");
    if (kv_max_seq > ctx->cfg.max_seq || pos0 + S > kv_max_seq) return fail(ctx, ZO_ESHAPE, "position beyond the cache / max_seq");
    if (S > ctx->max_B * ctx->max_S) return fail(ctx, ZO_EWORKSPACE, "prompt longer than the context was created for");
    if (!aligned16(kv) || !aligned16(logits) || ((uintptr_t)ids & 3)) return fail(ctx, ZO_EALIGN, "kv / logits / ids misaligned");
    for (size_t i = 0; i < ctx->params.size(); ++i)
        if (!ctx->params[i].ptr && !ctx->frozen[i].codes) return fail(ctx, ZO_EINVAL, "a tensor has neither fp32 nor packed storage");
    return ZO_OK;
}
}  // namespace

zo_status zo_prefill(zo_ctx* ctx, const int32_t* ids_dev, int32_t S, void* kv_dev, int32_t kv_max_seq, float* logits_dev)
{
    zo_status s = check_infer(ctx, ids_dev, S, 0, kv_dev, kv_max_seq, logits_dev);
    if (s != ZO_OK) return s;
    const infer_opts inf{(char*)kv_dev, kv_max_seq, 0, logits_dev};
    return run_forward(ctx, ids_dev, nullptr, 1, S, 0, 0.0f, 1, nullptr, &inf);
}

zo_status zo_decode(zo_ctx* ctx, const int32_t* token_dev, int32_t pos, void* kv_dev, int32_t kv_max_seq, float* logits_dev)
{
    zo_status s = check_infer(ctx, token_dev, 1, pos, kv_dev, kv_max_seq, logits_dev);
    if (s != ZO_OK) return s;
    const infer_opts inf{(char*)kv_dev, kv_max_seq, pos, logits_dev};
    return run_forward(ctx, token_dev, nullptr, 1, 1, 0, 0.0f, 1, nullptr, &inf);
}

zo_status zo_generate_greedy(zo_ctx* ctx, const int32_t* prompt_dev, int32_t S, int32_t n_new, void* kv_dev, int32_t kv_max_seq,
                             int32_t* tokens_dev, float* logits_dev)
{
    if (!ctx) return ZO_EINVAL;
    if (!tokens_dev || n_new < 1) return fail(ctx, ZO_EINVAL, "tokens_dev is NULL or n_new < 1");
    if (S + n_new - 1 > kv_max_seq) return fail(ctx, ZO_ESHAPE, "prompt + generated tokens exceed the cache");
    zo_status s = zo_prefill(ctx, prompt_dev, S, kv_dev, kv_max_seq, logits_dev);
    for (int i = 0; s == ZO_OK && i < n_new; ++i) {
        ZO_HIP(ctx, zo_launch_argmax(logits_dev, ctx->cfg.vocab, tokens_dev + i, ctx->st));
        if (i + 1 < n_new) s = zo_decode(ctx, tokens_dev + i, S + i, kv_dev, kv_max_seq, logits_dev);
    }
    return s;
}

namespace {
// coefficient of tensor i: coeff_dev[stride * group] if coeff_dev, else coeff_host[group]
zo_status update_all(zo_ctx* ctx, uint64_t seed, const float* coeff_dev, int stride, const float coeff_host[3])
{
    prof_scope ps(ctx, ZO_PROF_UPDATE);
    if (ctx->cfg.master_dtype == ZO_MASTER_F16) {          // binary16 masters: fp32 fma, one rounding
        zo_multi_seeds ms{};
        ms.k0[0] = (uint32_t)seed;
        ms.k1[0] = (uint32_t)(seed >> 32);
        for (int i = 0; i < (int)ctx->params.size(); ++i) {
            if (!trainable(ctx, i) || !ctx->params[i].ptr) continue;
            const int g = ctx->desc[i].lr_group;
            ms.c[0] = coeff_host ? coeff_host[g] : 0.0f;
            ZO_HIP(ctx, zo_launch_update_f16(ctx->params[i].ptr, ctx->params[i].numel, ms, 1, i, coeff_dev ? coeff_dev + stride * g : nullptr, 0,
                                             ctx->cfg.master_round, ctx->st));
        }
        return ZO_OK;
    }
    for (int i = 0; i < (int)ctx->params.size(); ++i) {
        if (!trainable(ctx, i) || !ctx->params[i].ptr) continue;
        const int g = ctx->desc[i].lr_group;
        ZO_HIP(ctx, zo_launch_update((float*)ctx->params[i].ptr, ctx->params[i].numel, seed, i,
                                     coeff_dev ? coeff_dev + stride * g : nullptr, coeff_host ? coeff_host[g] : 0.0f, ctx->st));
    }
    return ZO_OK;
}

zo_status step_impl(zo_ctx* ctx, const void* ids, const float* target, int32_t B, int32_t S, uint64_t seed, float eps,
                    const float lr[3], float* out_dev, int n_out)
{
    zo_status s = check_batch(ctx, ids, target, B, S);
    if (s != ZO_OK) return s;
    if (!out_dev) return fail(ctx, ZO_EINVAL, "out_dev is NULL");
    if (!(eps > 0.0f)) return fail(ctx, ZO_EINVAL, "eps must be positive");
    float* loss2 = (float*)(ctx->ws + ctx->L.scalars);
    float* out6 = loss2 + 2;
    s = run_forward(ctx, ids, target, B, S, seed, eps, 2, loss2);
    if (s != ZO_OK) return s;
    ZO_HIP(ctx, zo_launch_projected_grad(loss2, eps, lr, out6, out_dev, n_out, ctx->st));
    return update_all(ctx, seed, out6 + 3, 1, nullptr);
}
}  // namespace

namespace {
// q directions in one pass: coefficient of (direction d, group g) = coeff_dev[d * stride + g], or coeff_host[d * 3 + g]
zo_status update_all_multi(zo_ctx* ctx, const uint64_t* seeds, int q, const float* coeff_dev, int stride, const float* coeff_host)
{
    prof_scope ps(ctx, ZO_PROF_UPDATE);
    zo_multi_seeds ms{};
    for (int d = 0; d < q; ++d) { ms.k0[d] = (uint32_t)seeds[d]; ms.k1[d] = (uint32_t)(seeds[d] >> 32); }
    for (int i = 0; i < (int)ctx->params.size(); ++i) {
        if (!trainable(ctx, i) || !ctx->params[i].ptr) continue;
        const int g = ctx->desc[i].lr_group;
        if (!coeff_dev)
            for (int d = 0; d < q; ++d) ms.c[d] = coeff_host[d * 3 + g];
        if (ctx->cfg.master_dtype == ZO_MASTER_F16) {
            ZO_HIP(ctx, zo_launch_update_f16(ctx->params[i].ptr, ctx->params[i].numel, ms, q, i, coeff_dev ? coeff_dev + g : nullptr, stride,
                                             ctx->cfg.master_round, ctx->st));
            continue;
        }
        ZO_HIP(ctx, zo_launch_update_multi((float*)ctx->params[i].ptr, ctx->params[i].numel, ms, q, i, coeff_dev ? coeff_dev + g : nullptr,
                                           stride, ctx->st));
    }
    return ZO_OK;
}
}  // namespace

zo_status zo_step_multi(zo_ctx* ctx, const void* ids, const float* target, int32_t B, int32_t S, const uint64_t* seeds_host,
                        int32_t q, float eps, float lr_model, float lr_smooth, float lr_clip, float* out_dev)
{
    zo_status s = check_batch(ctx, ids, target, B, S);
    if (s != ZO_OK) return s;
    if (!out_dev || !seeds_host) return fail(ctx, ZO_EINVAL, "out_dev / seeds_host is NULL");
    if (q < 1 || q > ZO_MAX_DIRECTIONS) return fail(ctx, ZO_EINVAL, "q must be in 1..ZO_MAX_DIRECTIONS");
    if (!(eps > 0.0f)) return fail(ctx, ZO_EINVAL, "eps must be positive");
    // Eq. 2's factor 1/q, folded into the step sizes once (one fp32 division each)
    const float lrq[3] = {lr_model / (float)q, lr_smooth / (float)q, lr_clip / (float)q};
    float* scal = (float*)(ctx->ws + ctx->L.scalars) + 16;
    for (int d = 0; d < q; ++d) {                       // every direction at the same, not yet updated, W
        float* loss2 = scal + 8 * d;
        s = run_forward(ctx, ids, target, B, S, seeds_host[d], eps, 2, loss2);
        if (s != ZO_OK) return s;
        ZO_HIP(ctx, zo_launch_projected_grad(loss2, eps, lrq, loss2 + 2, out_dev + 6 * d, 6, ctx->st));
    }
    return update_all_multi(ctx, seeds_host, q, scal + 2 + 3, 8, nullptr);
}

zo_status zo_update_multi(zo_ctx* ctx, const uint64_t* seeds_host, int32_t q, const float* coeff_dev, const float* coeff_host)
{
    if (!ctx) return ZO_EINVAL;
    if (!seeds_host || (!coeff_dev && !coeff_host)) return fail(ctx, ZO_EINVAL, "seeds / coefficients missing");
    if (q < 1 || q > ZO_MAX_DIRECTIONS) return fail(ctx, ZO_EINVAL, "q must be in 1..ZO_MAX_DIRECTIONS");
    return update_all_multi(ctx, seeds_host, q, coeff_dev ? coeff_dev + 3 : nullptr, 6, coeff_host);
}

float zo_lr_linear_decay(float lr0, int64_t t, int64_t T)
{
    if (T <= 0) return lr0;
    return (float)((double)lr0 * (1.0 - (double)t / (double)T));
}

zo_status zo_update(zo_ctx* ctx, uint64_t seed, const float* coeff_dev, float coeff_host)
{
    if (!ctx) return ZO_EINVAL;
    const float h[3] = {coeff_host, coeff_host, coeff_host};
    return update_all(ctx, seed, coeff_dev, 0, h);
}

zo_status zo_update_groups(zo_ctx* ctx, uint64_t seed, const float* coeff_dev, const float* coeff_host)
{
    if (!ctx) return ZO_EINVAL;
    if (!coeff_dev && !coeff_host) return fail(ctx, ZO_EINVAL, "no coefficients");
    return update_all(ctx, seed, coeff_dev, 1, coeff_host);
}

zo_status zo_step(zo_ctx* ctx, const void* ids, const float* target, int32_t B, int32_t S,
                  uint64_t seed, float eps, float lr, float* out_dev)
{
    if (!ctx) return ZO_EINVAL;
    const float lrs[3] = {lr, lr, lr};
    return step_impl(ctx, ids, target, B, S, seed, eps, lrs, out_dev, 4);
}

zo_status zo_step_groups(zo_ctx* ctx, const void* ids, const float* target, int32_t B, int32_t S,
                         uint64_t seed, float eps, float lr_model, float lr_smooth, float lr_clip, float* out_dev)
{
    if (!ctx) return ZO_EINVAL;
    const float lrs[3] = {lr_model, lr_smooth, lr_clip};
    return step_impl(ctx, ids, target, B, S, seed, eps, lrs, out_dev, 6);
}

zo_status zo_init_learned_params(zo_ctx* ctx)
{
    if (!ctx) return ZO_EINVAL;
    const zo_config& c = ctx->cfg;
    if (!c.learn_clip && !c.learn_smooth) return ZO_OK;
    for (size_t t = 0; t < ctx->desc.size(); ++t) {
        const param_desc& p = ctx->desc[t];
        if (!p.quantized) continue;
        if (p.smooth >= 0 && p.owner == (int)t) {          // identity smoothing: s = 1, delta = 0
            ZO_HIP(ctx, zo_launch_fill((float*)ctx->params[p.smooth].ptr, p.cols, 1.0f, ctx->st));
            ZO_HIP(ctx, zo_launch_fill((float*)ctx->params[p.smooth + 1].ptr, p.cols, 0.0f, ctx->st));
        }
        if (p.clip >= 0) {                                  // the dynamic scheme's step and zero point; alpha 0, beta 1
            int32_t* scratch = (int32_t*)(ctx->ws + ctx->L.what[0]);
            ZO_HIP(ctx, zo_launch_init_learned((const float*)ctx->params[t].ptr, (int)p.rows, (int)p.cols, c.w_bits, c.w_group,
                                               (float*)ctx->params[p.clip].ptr, (float*)ctx->params[p.clip + 1].ptr,
                                               (float*)ctx->params[p.clip + 2].ptr, (float*)ctx->params[p.clip + 3].ptr, scratch, ctx->st));
        }
    }
    return ZO_OK;
}

uint32_t zo_debug_routes(const zo_ctx* ctx) { return ctx ? ctx->routes : 0u; }

zo_status zo_debug_buffer(zo_ctx* ctx, int32_t which, int32_t branch, void** ptr, size_t* bytes)
{
    if (!ctx || !ptr || !bytes || branch < 0 || branch > 1) return ZO_EINVAL;
    const zo_config& c = ctx->cfg;
    const size_t ts = zo_tsize(c.act_dtype);
    const layout::per_branch& r = ctx->L.br[branch];
    const size_t M = ctx->last_M;
    if (c.arch == ZO_ARCH_LINEAR) {
        if (which != 1) return ZO_EINVAL;
        *ptr = ctx->ws + r.logits;
        *bytes = M * c.d_ffn * ts;
        return ZO_OK;
    }
    switch (which) {
        case 0: *ptr = ctx->ws + r.h; *bytes = M * c.d_model * ts; return ZO_OK;
        case 1:
            if (ctx->routes & ZO_ROUTE_CE_IN_GEMM) return ZO_EUNSUPPORTED;   // that forward stored no logits
            *ptr = ctx->ws + r.logits; *bytes = M * (size_t)c.vocab * 4; return ZO_OK;
        case 2: *ptr = ctx->ws + r.x; *bytes = M * c.d_model * ts; return ZO_OK;
        case 3: *ptr = ctx->ws + r.qkv; *bytes = M * 3 * (size_t)c.d_model * ts; return ZO_OK;
        case 4: *ptr = ctx->ws + r.att; *bytes = M * c.d_model * ts; return ZO_OK;
        default: return ZO_EINVAL;
    }
}

// ---- stand-alone pieces -----------------------------------------------------------------------
zo_status zo_debug_philox_u32(uint64_t seed, int32_t tensor_id, int64_t nwords, uint32_t* out_dev, void* hip_stream)
{
    if (nwords < 0 || (nwords > 0 && !out_dev)) return ZO_EINVAL;
    return zo_launch_philox_words(seed, tensor_id, nwords, out_dev, (hipStream_t)hip_stream) == hipSuccess ? ZO_OK : ZO_EHIP;
}

zo_status zo_debug_normal(uint64_t seed, int32_t tensor_id, int64_t start, int64_t numel, float* out_dev, void* hip_stream)
{
    if (numel < 0 || start < 0 || (numel > 0 && !out_dev)) return ZO_EINVAL;
    return zo_launch_normal(seed, tensor_id, start, numel, out_dev, (hipStream_t)hip_stream) == hipSuccess ? ZO_OK : ZO_EHIP;
}

zo_status zo_update_tensor(float* w_dev, int64_t numel, uint64_t seed, int32_t tensor_id,
                           const float* coeff_dev, float coeff_host, void* hip_stream)
{
    if (numel < 0 || (numel > 0 && !w_dev)) return ZO_EINVAL;
    if (!aligned16(w_dev)) return ZO_EALIGN;
    return zo_launch_update(w_dev, numel, seed, tensor_id, coeff_dev, coeff_host, (hipStream_t)hip_stream) == hipSuccess ? ZO_OK : ZO_EHIP;
}

zo_status zo_update_tensor_f16(void* w_dev, int64_t numel, uint64_t seed, int32_t tensor_id, const float* coeff_dev, float coeff_host,
                               int32_t stochastic, void* hip_stream)
{
    if (numel < 0 || (numel > 0 && !w_dev)) return ZO_EINVAL;
    if (!aligned16(w_dev)) return ZO_EALIGN;
    zo_multi_seeds ms{};
    ms.k0[0] = (uint32_t)seed;
    ms.k1[0] = (uint32_t)(seed >> 32);
    ms.c[0] = coeff_host;
    return zo_launch_update_f16(w_dev, numel, ms, 1, tensor_id, coeff_dev, 0, stochastic ? 1 : 0, (hipStream_t)hip_stream) == hipSuccess
               ? ZO_OK : ZO_EHIP;
}

int64_t zo_master_bytes(const zo_config* cfg)
{
    std::vector<param_desc> p;
    if (!cfg || check_config(*cfg) != ZO_OK || !describe_params(*cfg, p)) return -1;
    int64_t total = 0;
    for (const param_desc& d : p) total += d.rows * d.cols * (cfg->master_dtype == ZO_MASTER_F16 ? 2 : 4);
    return total;
}

zo_status zo_debug_quant_weight(const float* W_dev, int32_t N, int32_t K, int32_t bits, int32_t group,
                                uint64_t seed, int32_t tensor_id, float eps_signed, int32_t out_dtype,
                                uint8_t* codes_dev, float* step_dev, int32_t* zp_dev, void* what_dev, void* hip_stream)
{
    if (!W_dev || N < 0 || K < 0) return ZO_EINVAL;
    if (out_dtype != ZO_ACT_FP32 && out_dtype != ZO_ACT_BF16) return ZO_EINVAL;
    if (bits < 0 || bits > 8 || group < 0) return ZO_EINVAL;
    if (!zo_fq_weight_supported(K, bits, group)) return ZO_ESHAPE;
    if (!aligned16(W_dev) || !aligned16(what_dev)) return ZO_EALIGN;
    hipError_t e = zo_launch_fq_weight(W_dev, N, K, bits, group, seed, tensor_id, eps_signed, out_dtype, what_dev, nullptr,
                                       codes_dev, step_dev, zp_dev, (hipStream_t)hip_stream);
    return e == hipSuccess ? ZO_OK : ZO_EHIP;
}

zo_status zo_debug_quant_weight_learned(const float* W_dev, int32_t N, int32_t K, int32_t bits, int32_t group,
                                        uint64_t seed, int32_t tensor_id, float eps_signed,
                                        const float* scale_dev, const float* step_dev, const float* zp_dev,
                                        const float* alpha_dev, const float* beta_dev, int32_t out_dtype,
                                        uint8_t* codes_dev, void* what_dev, void* hip_stream)
{
    if (!W_dev || !step_dev || !zp_dev || !alpha_dev || !beta_dev || !what_dev || N < 0 || K <= 0) return ZO_EINVAL;
    if (out_dtype != ZO_ACT_FP32 && out_dtype != ZO_ACT_BF16) return ZO_EINVAL;
    if (bits < 1 || bits > 8 || group < 0) return ZO_EINVAL;
    const int g = group ? group : K;
    if ((K & 7) || (g & 7) || K % g) return ZO_ESHAPE;
    if (!aligned16(W_dev) || !aligned16(what_dev) || !aligned16(scale_dev)) return ZO_EALIGN;
    const zo_learned p{step_dev, zp_dev, alpha_dev, beta_dev, scale_dev}, none{};
    hipError_t e = zo_launch_fq_weight_learned(W_dev, N, K, bits, group, seed, tensor_id, eps_signed, out_dtype, p, none, what_dev,
                                               nullptr, codes_dev, (hipStream_t)hip_stream);
    return e == hipSuccess ? ZO_OK : ZO_EHIP;
}

zo_status zo_debug_smooth_bias(const float* W_dev, int32_t N, int32_t K, uint64_t seed, int32_t tensor_id, float eps_signed,
                               const float* delta_dev, const float* bias_dev, float* out_dev, void* hip_stream)
{
    if (!W_dev || !delta_dev || !out_dev || N < 0 || K <= 0) return ZO_EINVAL;
    if (K & 7) return ZO_ESHAPE;
    if (!aligned16(W_dev) || !aligned16(delta_dev)) return ZO_EALIGN;
    hipError_t e = zo_launch_bias_shift(W_dev, N, K, seed, tensor_id, eps_signed, delta_dev, nullptr, bias_dev, nullptr, out_dev, nullptr,
                                        (hipStream_t)hip_stream);
    return e == hipSuccess ? ZO_OK : ZO_EHIP;
}

zo_status zo_debug_quant_act(const void* X_dev, int32_t M, int32_t K, int32_t bits, int32_t sym, int32_t dtype,
                             int16_t* codes_dev, float* step_dev, int32_t* zp_dev, void* xhat_dev, void* hip_stream)
{
    if (!X_dev || M < 0 || K <= 0) return ZO_EINVAL;
    if (dtype != ZO_ACT_FP32 && dtype != ZO_ACT_BF16) return ZO_EINVAL;
    if (bits < 2 || bits > 8) return ZO_EINVAL;
    if (K & 7) return ZO_ESHAPE;
    if (!aligned16(X_dev) || !aligned16(xhat_dev)) return ZO_EALIGN;
    hipError_t e = zo_launch_fq_act(X_dev, xhat_dev, M, K, bits, sym, dtype, codes_dev, step_dev, zp_dev, nullptr, nullptr,
                                    (hipStream_t)hip_stream);
    return e == hipSuccess ? ZO_OK : ZO_EHIP;
}

size_t zo_linear_scratch_bytes(int32_t M, int32_t N, int32_t K, int32_t dtype)
{
    if (M < 0 || N < 0 || K < 0) return 0;
    const size_t ts = zo_tsize(dtype);
    return align_up((size_t)M * K * ts) + align_up((size_t)N * K * ts);
}

zo_status zo_linear_fakequant(const void* X_dev, const float* W_dev, const float* bias_dev, void* Y_dev,
                              int32_t M, int32_t N, int32_t K, int32_t w_bits, int32_t w_group,
                              int32_t a_bits, int32_t a_sym, int32_t dtype,
                              uint64_t seed, int32_t tensor_id, float eps_signed, void* scratch_dev, void* hip_stream)
{
    if (!X_dev || !W_dev || !Y_dev || !scratch_dev || M < 0 || N < 0 || K <= 0) return ZO_EINVAL;
    if (dtype != ZO_ACT_FP32 && dtype != ZO_ACT_BF16) return ZO_EINVAL;
    if (w_bits < 0 || w_bits > 8 || w_group < 0) return ZO_EINVAL;
    if (!(a_bits == 16 || (a_bits >= 2 && a_bits <= 8))) return ZO_EINVAL;
    if (!zo_fq_weight_supported(K, w_bits, w_group)) return ZO_ESHAPE;
    if (!aligned16(X_dev) || !aligned16(W_dev) || !aligned16(Y_dev) || !aligned16(scratch_dev) || !aligned16(bias_dev)) return ZO_EALIGN;
    hipStream_t st = (hipStream_t)hip_stream;
    const size_t ts = zo_tsize(dtype);
    char* xhat = (char*)scratch_dev;
    char* what = xhat + align_up((size_t)M * K * ts);
    hipError_t e = zo_launch_fq_weight(W_dev, N, K, w_bits, w_group, seed, tensor_id, eps_signed, dtype, what, nullptr,
                                       nullptr, nullptr, nullptr, st);
    if (e != hipSuccess) return ZO_EHIP;
    const void* xin = X_dev;
    if (a_bits < 16) {
        e = zo_launch_fq_act(X_dev, xhat, M, K, a_bits, a_sym, dtype, nullptr, nullptr, nullptr, nullptr, nullptr, st);
        if (e != hipSuccess) return ZO_EHIP;
        xin = xhat;
    }
    zo_gemm_args a{};
    a.X = xin; a.W = what; a.Y = Y_dev; a.bias = bias_dev;
    a.M = M; a.N = N; a.K = K; a.batch = 1; a.dtype = dtype;
    return zo_launch_gemm(a, st) == hipSuccess ? ZO_OK : ZO_EHIP;
}

// scratch of the integer-code route: [0] activation codes, [1] token steps, [2] token offsets, [3] weight codes,
// [4] weight steps, [5] r, [6] per-group parts of r, [7] end
static void linear_i8_layout(int32_t M, int32_t N, int32_t K, int32_t w_group, size_t off[8])
{
    const size_t G = (size_t)(K / (w_group ? w_group : K));
    size_t o = 0;
    off[0] = o; o += align_up((size_t)M * K);
    off[1] = o; o += align_up((size_t)M * 4);
    off[2] = o; o += align_up((size_t)M * 4);
    off[3] = o; o += align_up((size_t)N * K);
    off[4] = o; o += align_up(zo_i8_scale_floats(N, K, w_group) * 4);
    off[5] = o; o += align_up((size_t)N * 4);
    off[6] = o; o += align_up((size_t)N * G * 4);
    off[7] = o;
}

size_t zo_linear_mma_scratch_bytes(int32_t M, int32_t N, int32_t K, int32_t w_group, int32_t dtype, int32_t mma, size_t* offsets_host)
{
    if (M < 0 || N < 0 || K <= 0 || w_group < 0) return 0;
    if (mma == ZO_MMA_BF16) return zo_linear_scratch_bytes(M, N, K, dtype);
    if (mma != ZO_MMA_INT8 || (w_group && K % w_group)) return 0;
    size_t off[8];
    linear_i8_layout(M, N, K, w_group, off);
    if (offsets_host) memcpy(offsets_host, off, sizeof(off));
    return off[7];
}

zo_status zo_linear_fakequant_mma(const void* X_dev, const float* W_dev, const float* bias_dev, void* Y_dev,
                                  int32_t M, int32_t N, int32_t K, int32_t w_bits, int32_t w_group,
                                  int32_t a_bits, int32_t a_sym, int32_t dtype, int32_t out_f32, int32_t mma,
                                  uint64_t seed, int32_t tensor_id, float eps_signed, void* scratch_dev, int32_t* flag_dev,
                                  void* hip_stream)
{
    if (mma == ZO_MMA_BF16) {
        if (out_f32 != (dtype == ZO_ACT_FP32)) return ZO_EUNSUPPORTED;
        return zo_linear_fakequant(X_dev, W_dev, bias_dev, Y_dev, M, N, K, w_bits, w_group, a_bits, a_sym, dtype, seed, tensor_id,
                                   eps_signed, scratch_dev, hip_stream);
    }
    if (mma != ZO_MMA_INT8) return ZO_EINVAL;
    if (!X_dev || !W_dev || !Y_dev || !scratch_dev || !flag_dev || M < 0 || N < 0 || K <= 0) return ZO_EINVAL;
    if (dtype != ZO_ACT_FP32 && dtype != ZO_ACT_BF16) return ZO_EINVAL;
    if (w_group < 0) return ZO_EINVAL;
    if (M == 0 || N == 0) return ZO_OK;
    if (!zo_i8_supported(M, N, K, w_bits, w_group, a_bits)) return ZO_EUNSUPPORTED;    // needs weight AND activation codes
    if (!aligned16(X_dev) || !aligned16(W_dev) || !aligned16(Y_dev) || !aligned16(scratch_dev) || !aligned16(bias_dev) ||
        ((uintptr_t)flag_dev & 3))
        return ZO_EALIGN;
    hipStream_t st = (hipStream_t)hip_stream;
    size_t off[8];
    linear_i8_layout(M, N, K, w_group, off);
    char* sc = (char*)scratch_dev;
    int8_t* xc = (int8_t*)(sc + off[0]);
    float* xs = (float*)(sc + off[1]);
    float* xo = (float*)(sc + off[2]);
    int8_t* wc = (int8_t*)(sc + off[3]);
    float* ws = (float*)(sc + off[4]);
    float* wr = (float*)(sc + off[5]);
    float* rpart = (float*)(sc + off[6]);
    if (zo_launch_act_codes_i8(X_dev, xc, xs, xo, M, K, a_bits, a_sym, dtype, st) != hipSuccess) return ZO_EHIP;
    if (zo_launch_weight_codes_i8(W_dev, N, K, w_bits, w_group, seed, tensor_id, eps_signed, ZO_W_F32, wc, nullptr, ws, nullptr, wr,
                                  nullptr, rpart, nullptr, flag_dev, st) != hipSuccess)
        return ZO_EHIP;
    zo_i8_gemm_args a{};
    a.X = xc; a.W = wc; a.xs = xs; a.xo = xo; a.ws = ws; a.wr = wr; a.Y = Y_dev; a.bias = bias_dev;
    a.M = M; a.N = N; a.K = K; a.batch = 1;
    a.sgroup = w_group ? w_group : K;
    return zo_launch_gemm_i8(a, out_f32, st) == hipSuccess ? ZO_OK : ZO_EHIP;
}

size_t zo_linear_fused_scratch_bytes(int32_t M, int32_t K)
{
    if (M <= 0 || K <= 0) return 0;
    return 2 * align_up(zo_fused_relayout_bytes(M, K));
}

zo_status zo_linear_fakequant_fused(const void* Xp_dev, const void* Xm_dev, const float* W_dev, const float* bias_dev,
                                    void* Yp_dev, void* Ym_dev, int32_t M, int32_t N, int32_t K, int32_t w_bits,
                                    int32_t w_group, uint64_t seed, int32_t tensor_id, float eps, int32_t out_f32,
                                    void* scratch_dev, void* hip_stream)
{
    if (!Xp_dev || !W_dev || !Yp_dev || M <= 0 || N <= 0 || K <= 0) return ZO_EINVAL;
    if (Ym_dev && !Xm_dev) return ZO_EINVAL;
    if (w_bits < 0 || w_bits > 8 || w_group < 0) return ZO_EINVAL;
    if (!zo_fused_supported(M, N, K, w_bits, w_group)) return ZO_ESHAPE;
    if (!aligned16(Xp_dev) || !aligned16(Xm_dev) || !aligned16(W_dev) || !aligned16(bias_dev) || !aligned16(Yp_dev) || !aligned16(Ym_dev))
        return ZO_EALIGN;
    zo_fused_args f{};
    f.X = Xp_dev; f.W = W_dev; f.Y = Yp_dev; f.bias = bias_dev;
    f.M = M; f.N = N; f.K = K; f.nb = Ym_dev ? 2 : 1; f.ldY = N;
    if (Ym_dev) {
        f.strideX = ((const char*)Xm_dev - (const char*)Xp_dev) / 2;
        f.strideY = ((const char*)Ym_dev - (const char*)Yp_dev) / (out_f32 ? 4 : 2);
    }
    f.bits = w_bits; f.group = w_group; f.eps = eps; f.out_f32 = out_f32 ? 1 : 0;
    if (scratch_dev) {
        if (!aligned16(scratch_dev)) return ZO_EALIGN;
        f.Xfrag = scratch_dev;
        f.strideXfrag = (int64_t)(align_up(zo_fused_relayout_bytes(M, K)) / 2);
        if (zo_launch_fused_relayout(f.X, f.strideX, M, K, f.nb, w_bits, w_group, scratch_dev, f.strideXfrag, (hipStream_t)hip_stream) != hipSuccess)
            return ZO_EHIP;
    }
    return zo_launch_fq_gemm_fused(f, seed, tensor_id, (hipStream_t)hip_stream) == hipSuccess ? ZO_OK : ZO_EHIP;
}

zo_status zo_pack_weight_int4(const float* W_dev, int32_t N, int32_t K, int32_t group,
                              void* codes_dev, void* step_f16_dev, int16_t* zp_dev, void* hip_stream)
{
    if (!W_dev || !codes_dev || !step_f16_dev || !zp_dev || N < 0 || K <= 0) return ZO_EINVAL;
    if (!zo_int4_group_supported(K, group)) return ZO_ESHAPE;
    if (!aligned16(W_dev) || !aligned16(codes_dev) || ((uintptr_t)step_f16_dev & 1) || ((uintptr_t)zp_dev & 1)) return ZO_EALIGN;
    return zo_launch_pack_int4(W_dev, N, K, group, codes_dev, step_f16_dev, zp_dev, (hipStream_t)hip_stream) == hipSuccess ? ZO_OK : ZO_EHIP;
}

zo_status zo_linear_frozen_int4(const void* X_dev, const void* codes_dev, const void* step_f16_dev, const int16_t* zp_dev,
                                const float* bias_dev, void* Y_dev, int32_t M, int32_t N, int32_t K, int32_t group,
                                int32_t a_bits, int32_t a_sym, int32_t dtype, void* scratch_dev, void* hip_stream)
{
    if (!X_dev || !codes_dev || !step_f16_dev || !zp_dev || !Y_dev || !scratch_dev || M < 0 || N < 0 || K <= 0) return ZO_EINVAL;
    if (dtype != ZO_ACT_FP32 && dtype != ZO_ACT_BF16) return ZO_EINVAL;
    if (!(a_bits == 16 || (a_bits >= 2 && a_bits <= 8))) return ZO_EINVAL;
    if (!zo_int4_group_supported(K, group)) return ZO_ESHAPE;
    if (!aligned16(X_dev) || !aligned16(codes_dev) || !aligned16(Y_dev) || !aligned16(scratch_dev) || !aligned16(bias_dev) ||
        ((uintptr_t)step_f16_dev & 1) || ((uintptr_t)zp_dev & 1))
        return ZO_EALIGN;
    hipStream_t st = (hipStream_t)hip_stream;
    const size_t ts = zo_tsize(dtype);
    char* xhat = (char*)scratch_dev;
    char* what = xhat + align_up((size_t)M * K * ts);
    hipError_t e = zo_launch_dequant_int4(codes_dev, step_f16_dev, zp_dev, N, K, group, dtype, what, nullptr, st);
    if (e != hipSuccess) return ZO_EHIP;
    const void* xin = X_dev;
    if (a_bits < 16) {
        e = zo_launch_fq_act(X_dev, xhat, M, K, a_bits, a_sym, dtype, nullptr, nullptr, nullptr, nullptr, nullptr, st);
        if (e != hipSuccess) return ZO_EHIP;
        xin = xhat;
    }
    zo_gemm_args a{};
    a.X = xin; a.W = what; a.Y = Y_dev; a.bias = bias_dev;
    a.M = M; a.N = N; a.K = K; a.batch = 1; a.dtype = dtype;
    return zo_launch_gemm(a, st) == hipSuccess ? ZO_OK : ZO_EHIP;
}

zo_status zo_linear_frozen_int4_fused(const void* Xp_dev, const void* Xm_dev, const void* codes_dev, const void* step_f16_dev,
                                      const int16_t* zp_dev, const float* bias_dev, void* Yp_dev, void* Ym_dev, int32_t M, int32_t N,
                                      int32_t K, int32_t group, int32_t out_f32, void* scratch_dev, void* hip_stream)
{
    if (!Xp_dev || !codes_dev || !step_f16_dev || !zp_dev || !Yp_dev || M <= 0 || N <= 0 || K <= 0) return ZO_EINVAL;
    if (Ym_dev && !Xm_dev) return ZO_EINVAL;
    if (!zo_int4_fused_supported(M, N, K, group)) return ZO_ESHAPE;
    if (!aligned16(Xp_dev) || !aligned16(Xm_dev) || !aligned16(codes_dev) || !aligned16(bias_dev) || !aligned16(Yp_dev) ||
        !aligned16(Ym_dev) || !aligned16(scratch_dev) || ((uintptr_t)step_f16_dev & 1) || ((uintptr_t)zp_dev & 1))
        return ZO_EALIGN;
    zo_fused_args f{};
    f.X = Xp_dev; f.codes = codes_dev; f.step16 = step_f16_dev; f.zp = zp_dev; f.Y = Yp_dev; f.bias = bias_dev;
    f.M = M; f.N = N; f.K = K; f.nb = Ym_dev ? 2 : 1; f.ldY = N; f.group = group; f.bits = 4; f.out_f32 = out_f32 ? 1 : 0;
    if (Ym_dev) {
        f.strideX = ((const char*)Xm_dev - (const char*)Xp_dev) / 2;
        f.strideY = ((const char*)Ym_dev - (const char*)Yp_dev) / (out_f32 ? 4 : 2);
    }
    if (scratch_dev) {
        // with scratch: fragment-ordered activations, 128 channels per workgroup, K split over workgroups
        f.Xfrag = scratch_dev;
        f.strideXfrag = (int64_t)(align_up(zo_fused_relayout_bytes(M, K)) / 2);
        if (zo_launch_fused_relayout(f.X, f.strideX, M, K, f.nb, 4, group, scratch_dev, f.strideXfrag, (hipStream_t)hip_stream) != hipSuccess)
            return ZO_EHIP;
        void* partials = (char*)scratch_dev + zo_linear_fused_scratch_bytes(M, K);
        return zo_launch_int4_gemm_splitk(f, partials, (hipStream_t)hip_stream) == hipSuccess ? ZO_OK : ZO_EHIP;
    }
    return zo_launch_int4_gemm_fused(f, (hipStream_t)hip_stream) == hipSuccess ? ZO_OK : ZO_EHIP;
}

zo_status zo_linear_frozen_int4_token(const void* x_dev, const void* codes_dev, const void* step_f16_dev, const int16_t* zp_dev,
                                      const float* bias_dev, const void* residual_dev, int32_t relu, void* y_dev, int32_t N, int32_t K,
                                      int32_t group, int32_t out_f32, void* hip_stream)
{
    if (!x_dev || !codes_dev || !step_f16_dev || !zp_dev || !y_dev || N <= 0 || K <= 0) return ZO_EINVAL;
    if (!zo_int4_gemv_supported(1, 1, N, K, group)) return ZO_ESHAPE;
    if (!aligned16(x_dev) || !aligned16(codes_dev) || ((uintptr_t)step_f16_dev & 1) || ((uintptr_t)zp_dev & 1) || ((uintptr_t)bias_dev & 3) ||
        ((uintptr_t)residual_dev & 1) || ((uintptr_t)y_dev & 3))
        return ZO_EALIGN;
    zo_fused_args f{};
    f.X = x_dev; f.codes = codes_dev; f.step16 = step_f16_dev; f.zp = zp_dev; f.Y = y_dev; f.bias = bias_dev; f.residual = residual_dev;
    f.M = 1; f.N = N; f.K = K; f.nb = 1; f.ldY = N; f.group = group; f.bits = 4; f.relu = relu ? 1 : 0; f.out_f32 = out_f32 ? 1 : 0;
    return zo_launch_int4_gemv(f, (hipStream_t)hip_stream) == hipSuccess ? ZO_OK : ZO_EHIP;
}

size_t zo_linear_frozen_fused_scratch_bytes(int32_t M, int32_t N, int32_t K, int32_t group)
{
    if (M <= 0 || N <= 0 || K <= 0 || group <= 0) return 0;
    return zo_linear_fused_scratch_bytes(M, K) + align_up(zo_int4_splitk_scratch_bytes(M, N, K, group));
}

size_t zo_attention_scratch_bytes(int32_t, int32_t, int32_t, int32_t, int32_t) { return 0; }   // no kernel needs one

zo_status zo_attention_causal(const void* q_dev, const void* k_dev, const void* v_dev, void* out_dev,
                              int32_t B, int32_t S, int32_t H, int32_t dh, int64_t row_stride, int32_t dtype,
                              void* scratch_dev, void* hip_stream)
{
    if (!q_dev || !k_dev || !v_dev || !out_dev || B < 0 || S < 0 || H <= 0) return ZO_EINVAL;
    if (dtype != ZO_ACT_FP32 && dtype != ZO_ACT_BF16) return ZO_EINVAL;
    if (dh != 16 && dh != 32 && dh != 64 && dh != 128) return ZO_EUNSUPPORTED;
    if (row_stride < (int64_t)H * dh || (row_stride & 7)) return ZO_ESHAPE;
    if (!aligned16(q_dev) || !aligned16(k_dev) || !aligned16(v_dev) || !aligned16(out_dev) || !aligned16(scratch_dev)) return ZO_EALIGN;
    hipStream_t st = (hipStream_t)hip_stream;
    hipError_t e;
    if (zo_flash_attention_supported(dh, dtype)) {
        e = zo_launch_flash_attention(q_dev, k_dev, v_dev, out_dev, B, S, H, dh, row_stride, st);
    } else {
        e = zo_launch_attention(q_dev, k_dev, v_dev, out_dev, B, S, H, dh, row_stride, dtype, st);
    }
    return e == hipSuccess ? ZO_OK : ZO_EHIP;
}

zo_status zo_gemm_nt(const void* X_dev, const void* W_dev, void* Y_dev, int32_t M, int32_t N, int32_t K,
                     int32_t dtype, void* hip_stream)
{
    if (!X_dev || !W_dev || !Y_dev || M < 0 || N < 0 || K <= 0) return ZO_EINVAL;
    if (dtype != ZO_ACT_FP32 && dtype != ZO_ACT_BF16) return ZO_EINVAL;
    if (K & 7) return ZO_ESHAPE;
    if (!aligned16(X_dev) || !aligned16(W_dev) || !aligned16(Y_dev)) return ZO_EALIGN;
    zo_gemm_args a{};
    a.X = X_dev; a.W = W_dev; a.Y = Y_dev;
    a.M = M; a.N = N; a.K = K; a.batch = 1; a.dtype = dtype;
    return zo_launch_gemm(a, (hipStream_t)hip_stream) == hipSuccess ? ZO_OK : ZO_EHIP;
}

zo_status zo_gemm_nt_swiglu(const void* X_dev, const void* W_dev, void* Y_dev, int32_t M, int32_t N2, int32_t K, void* hip_stream)
{
    if (!X_dev || !W_dev || !Y_dev || M <= 0 || N2 <= 0 || K <= 0) return ZO_EINVAL;
    if (!aligned16(X_dev) || !aligned16(W_dev) || !aligned16(Y_dev)) return ZO_EALIGN;
    if (!zo_gemm_swiglu_supported(M, N2, K, ZO_T_BF16)) return ZO_EUNSUPPORTED;
    zo_gemm_args a{};
    a.X = X_dev; a.W = W_dev; a.Y = Y_dev;
    a.M = M; a.N = N2; a.K = K; a.batch = 1; a.dtype = ZO_T_BF16; a.swiglu = 1;
    return zo_launch_gemm(a, (hipStream_t)hip_stream) == hipSuccess ? ZO_OK : ZO_EHIP;
}

size_t zo_gemm_nt_ce_scratch_bytes(int32_t M, int32_t N)
{
    if (M <= 0 || N <= 0) return 0;
    return (zo_gemm_ce_part_floats(M, N) + (size_t)M) * sizeof(float);
}

zo_status zo_gemm_nt_ce(const void* X_dev, const void* W_dev, const int32_t* ids_dev, float* row_loss_dev, int32_t M, int32_t S,
                        int32_t N, int32_t K, void* scratch_dev, void* hip_stream)
{
    if (!X_dev || !W_dev || !ids_dev || !row_loss_dev || !scratch_dev || M <= 0 || S <= 0 || N <= 0 || K <= 0) return ZO_EINVAL;
    if (M % S) return ZO_ESHAPE;
    if (!aligned16(X_dev) || !aligned16(W_dev) || !aligned16(scratch_dev)) return ZO_EALIGN;
    if (!zo_gemm_ce_supported(M, N, K, ZO_T_BF16)) return ZO_EUNSUPPORTED;
    zo_gemm_args a{};
    a.X = X_dev; a.W = W_dev;
    a.M = M; a.N = N; a.K = K; a.batch = 1; a.dtype = ZO_T_BF16; a.out_f32 = 1;
    a.ce_part = (float*)scratch_dev;
    a.ce_tgt = a.ce_part + zo_gemm_ce_part_floats(M, N);
    a.ce_ids = ids_dev;
    a.ce_S = S;
    if (zo_launch_gemm(a, (hipStream_t)hip_stream) != hipSuccess) return ZO_EHIP;
    return zo_launch_ce_combine(a.ce_part, a.ce_tgt, row_loss_dev, M, S, N, (hipStream_t)hip_stream) == hipSuccess ? ZO_OK : ZO_EHIP;
}

zo_status zo_gemm_nt_fused(const void* X_dev, const void* W_dev, const float* bias_dev, const void* residual_dev, int32_t relu,
                           void* Y_dev, int32_t M, int32_t N, int32_t K, int32_t dtype, void* hip_stream)
{
    if (!X_dev || !W_dev || !Y_dev || M < 0 || N < 0 || K <= 0) return ZO_EINVAL;
    if (dtype != ZO_ACT_FP32 && dtype != ZO_ACT_BF16) return ZO_EINVAL;
    if (K & 7) return ZO_ESHAPE;
    if (!aligned16(X_dev) || !aligned16(W_dev) || !aligned16(Y_dev) || !aligned16(bias_dev) || !aligned16(residual_dev)) return ZO_EALIGN;
    zo_gemm_args a{};
    a.X = X_dev; a.W = W_dev; a.Y = Y_dev; a.bias = bias_dev; a.residual = residual_dev; a.relu = relu ? 1 : 0;
    a.M = M; a.N = N; a.K = K; a.batch = 1; a.dtype = dtype;
    return zo_launch_gemm(a, (hipStream_t)hip_stream) == hipSuccess ? ZO_OK : ZO_EHIP;
}

size_t zo_gemm_nt_splitk_scratch_bytes(int32_t M, int32_t N, int32_t K, int32_t dtype)
{
    return zo_gemm_splitk_bytes(M, N, K, 1, dtype == ZO_ACT_BF16 ? ZO_T_BF16 : ZO_T_F32);
}

int32_t zo_gemm_nt_splitk_ranges(int32_t M, int32_t N, int32_t K, int32_t dtype)
{
    if (zo_gemm_splitk_bytes(M, N, K, 1, dtype == ZO_ACT_BF16 ? ZO_T_BF16 : ZO_T_F32) == 0) return 1;
    return zo_gemm_splitk(M, N, K, 1, ZO_T_BF16);
}

zo_status zo_gemm_nt_fused_splitk(const void* X_dev, const void* W_dev, const float* bias_dev, const void* residual_dev, int32_t relu,
                                  void* Y_dev, int32_t M, int32_t N, int32_t K, int32_t dtype, void* scratch_dev, size_t scratch_bytes,
                                  void* hip_stream)
{
    if (!X_dev || !W_dev || !Y_dev || M < 0 || N < 0 || K <= 0) return ZO_EINVAL;
    if (dtype != ZO_ACT_FP32 && dtype != ZO_ACT_BF16) return ZO_EINVAL;
    if (K & 7) return ZO_ESHAPE;
    if (!aligned16(X_dev) || !aligned16(W_dev) || !aligned16(Y_dev) || !aligned16(bias_dev) || !aligned16(residual_dev) ||
        !aligned16(scratch_dev))
        return ZO_EALIGN;
    zo_gemm_args a{};
    a.X = X_dev; a.W = W_dev; a.Y = Y_dev; a.bias = bias_dev; a.residual = residual_dev; a.relu = relu ? 1 : 0;
    a.M = M; a.N = N; a.K = K; a.batch = 1; a.dtype = dtype;
    a.ks_part = (float*)scratch_dev;
    a.ks_part_bytes = scratch_dev ? scratch_bytes : 0;
    return zo_launch_gemm(a, (hipStream_t)hip_stream) == hipSuccess ? ZO_OK : ZO_EHIP;
}

// ---- the K-split GEMM for callers that cannot allocate -------------------------------------------------------------
// The partial sums live in a file-scope device array instead of caller-provided scratch.  The array's name is a host-side
// stand-in only; its device address is looked up once per device (every GPU holds its own copy) and that pointer is
// what the kernels receive.
enum { ZO_STATIC_SCRATCH_BYTES = 32 << 20, ZO_STATIC_MAX_DEVICES = 64 };
static __device__ __align__(256) float zo_static_scratch[ZO_STATIC_SCRATCH_BYTES / sizeof(float)];
static float* zo_static_scratch_ptr[ZO_STATIC_MAX_DEVICES];
static std::mutex zo_static_scratch_mutex;

size_t zo_gemm_nt_splitk_static_max_bytes(void) { return (size_t)ZO_STATIC_SCRATCH_BYTES; }

zo_status zo_gemm_nt_fused_splitk_static(const void* X_dev, const void* W_dev, const float* bias_dev, const void* residual_dev,
                                         int32_t relu, void* Y_dev, int32_t M, int32_t N, int32_t K, int32_t dtype, void* hip_stream)
{
    if (!X_dev || !W_dev || !Y_dev || M < 0 || N < 0 || K <= 0) return ZO_EINVAL;
    if (dtype != ZO_ACT_FP32 && dtype != ZO_ACT_BF16) return ZO_EINVAL;
    if (K & 7) return ZO_ESHAPE;
    if (!aligned16(X_dev) || !aligned16(W_dev) || !aligned16(Y_dev) || !aligned16(bias_dev) || !aligned16(residual_dev))
        return ZO_EALIGN;
    const size_t need = zo_gemm_splitk_bytes(M, N, K, 1, dtype == ZO_ACT_BF16 ? ZO_T_BF16 : ZO_T_F32);
    if (need > (size_t)ZO_STATIC_SCRATCH_BYTES) return ZO_EWORKSPACE;     // the K ranges of this shape need more than the array holds
    float* scratch = nullptr;
    if (need) {
        int dev = -1;
        if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= ZO_STATIC_MAX_DEVICES) return ZO_EHIP;
        std::lock_guard<std::mutex> lock(zo_static_scratch_mutex);
        if (!zo_static_scratch_ptr[dev]) {
            void* p = nullptr;
            if (hipGetSymbolAddress(&p, HIP_SYMBOL(zo_static_scratch)) != hipSuccess || !p) return ZO_EHIP;
            zo_static_scratch_ptr[dev] = (float*)p;
        }
        scratch = zo_static_scratch_ptr[dev];
    }
    zo_gemm_args a{};
    a.X = X_dev; a.W = W_dev; a.Y = Y_dev; a.bias = bias_dev; a.residual = residual_dev; a.relu = relu ? 1 : 0;
    a.M = M; a.N = N; a.K = K; a.batch = 1; a.dtype = dtype;
    a.ks_part = scratch;                                   // every range's partial sums are written before they are read:
    a.ks_part_bytes = scratch ? need : 0;                  // nothing left by an earlier call is ever seen
    return zo_launch_gemm(a, (hipStream_t)hip_stream) == hipSuccess ? ZO_OK : ZO_EHIP;
}

}  // extern "C"
