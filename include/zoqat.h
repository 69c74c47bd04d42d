/*
 * zoqat.h -- C ABI of the MI355X (gfx950) library for one zeroth-order quantization-aware
 * training step of ZeroQAT:
 *
 *     draw u ~ N(0, I) from a seed                          (Eq. 2; never stored)
 *     L+ = L(Q(W + eps u)),  L- = L(Q(W - eps u))           (Eq. 2, two quantized forwards)
 *     g  = (L+ - L-) / (2 eps)                              (Eq. 2 with q = 1)
 *     W <- W - eta g u                                      (Eq. 3, full-precision masters)
 *
 * Q is the uniform asymmetric quantizer of the Background section applied per group of
 * `w_group` consecutive input features of every quantized linear layer; activations entering a
 * quantized linear are quantized per token (Appendix "Quantization settings").
 *
 * Conventions
 *   - plain C, no exceptions; every call returns a zo_status (ZO_OK = 0);
 *   - "dev" pointers are device (HBM) addresses, "host" pointers are host addresses;
 *   - the caller owns every device buffer (master weights, workspace, ids, outputs); the library
 *     never allocates or frees device memory, and it launches all work asynchronously on the
 *     hipStream_t given at zo_init / in the call (passed as void*); the only call that waits for the
 *     stream is zo_profile_end, which has to read its events;
 *   - matrices are row-major; a linear weight is W[N][K] (N outputs, K inputs, K contiguous) and
 *     Y[M][N] = X[M][K] * W^T;
 *   - element i (flat, row-major) of tensor number t under seed s always receives the same
 *     perturbation u(s, t, i), whichever call or kernel asks for it;
 *   - device pointers must be 16-byte aligned; K must be a multiple of 8 and of the group size.
 *   - one context per stream; a context is not thread-safe.
 */
#ifndef ZOQAT_H
#define ZOQAT_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    ZO_OK = 0,
    ZO_EINVAL = 1,        /* null pointer, negative size, unknown enum value */
    ZO_ESHAPE = 2,        /* a dimension violates a divisibility / size rule */
    ZO_EALIGN = 3,        /* device pointer not 16-byte aligned */
    ZO_EHIP = 4,          /* a HIP call failed; see zo_last_error */
    ZO_EUNSUPPORTED = 5,  /* valid request this build cannot run */
    ZO_EWORKSPACE = 6     /* workspace smaller than zo_workspace_bytes */
} zo_status;

enum { ZO_ARCH_LINEAR = 0, ZO_ARCH_LLAMA = 1, ZO_ARCH_OPT = 2 };
enum { ZO_ACT_FP32 = 0, ZO_ACT_BF16 = 1 };
enum { ZO_MASTER_F32 = 0, ZO_MASTER_F16 = 1 };

/* Model and quantization setting ("WxAy gN" of the appendix: w_bits, a_bits, w_group). */
typedef struct {
    int32_t arch;        /* ZO_ARCH_*: single linear (d_model inputs -> d_ffn outputs, MSE loss),
                            Llama-shaped (RMSNorm, RoPE, SwiGLU, no biases), OPT-shaped (LayerNorm,
                            learned positions, ReLU, biases); decoders use next-token cross entropy */
    int32_t n_layers, d_model, n_heads, d_ffn, vocab, max_seq;
    int32_t w_bits;      /* weight bits of the quantized linears, 1..8; 0 = no weight quantization */
    int32_t w_group;     /* group size along K; 0 = per output channel */
    int32_t a_bits;      /* activation bits, 2..8; 16 = activations not quantized */
    int32_t a_sym;       /* 0 = asymmetric min/max (the paper's choice), 1 = symmetric absmax */
    int32_t act_dtype;   /* ZO_ACT_*: storage type of activations and GEMM operands */
    int32_t lightweight; /* 0 = every tensor trainable; 1 = only tensors whose zo_tensor.trainable
                            is set are perturbed and updated (lightweight variant) */
    int32_t learn_clip;  /* 1 = adaptive weight quantizer (Eq. 5): every quantized linear gets four more
                            trainable fp32 tensors [N][K/w_group] -- step, zero point, alpha, beta -- used
                            instead of the per-forward min/max */
    int32_t learn_smooth;/* 1 = channel-wise smoothing (Eq. 4): every distinct input activation of the
                            quantized linears gets two more trainable fp32 tensors [K] -- s and delta;
                            needs learn_clip = 1 and a_bits < 16 */
    int32_t no_fused;    /* 0 = the linears of a forward over at most 128 tokens (bf16 storage, groups of 8..128 -- at most 64
                            tokens and groups of 32..128 when packed tensors are attached --, no learned tensors) build their weight tiles inside
                            the GEMM kernel, from the masters or from the packed codes; large bf16 Llama-shaped forwards
                            without smoothing interleave the gate and up rows in the operand buffer and take silu(gate) * up
                            in the GEMM epilogue, and (head dimension 128) permute the head blocks of q | k | v and apply
                            the rotary embedding there (zo_debug_routes tells which routes a forward took);
                            1 = always quantize once into the workspace and run the plain GEMM with the stand-alone kernels.
                            Independent of this flag, a large bf16 forward forms its cross entropy in the lm_head GEMM's
                            epilogue and stores no logits, and the bf16 GEMMs of a few hundred tokens onto a narrow output
                            split K into ranges whose fp32 partial sums a second kernel adds in order. */
    int32_t master_dtype;/* ZO_MASTER_*: storage type of every tensor of the parameter list.  ZO_MASTER_F16 = IEEE binary16,
                            the 2 bytes per parameter that the memory table of the efficiency section implies: a
                            forward reads the stored value (exactly widened to fp32) wherever it read the fp32 master;
                            the update of Eq. 3 computes fma(-c, u, w) in fp32 and rounds once to binary16.  Not
                            available together with learn_clip / learn_smooth. */
    int32_t master_round;/* binary16 masters only: 0 = round to nearest even (a step below half the spacing of
                            binary16 is lost entirely), 1 = stochastic rounding (upper neighbour with probability
                            (x - lo) / (hi - lo), integers from the stream (seed, element / 4, tensor, 1)) */
    int32_t mma;         /* contraction of the quantized linears (ZO_MMA_*, see zo_linear_fakequant_mma): 0 = ZO_MMA_BF16, de-quantized
                            operands rounded to the storage type; 1 = ZO_MMA_INT8, the integer codes themselves (Background/Quantization:
                            X_INT) on the int8 matrix instructions, steps and zero points applied in fp32, neither operand rounded.
                            ZO_MMA_INT8 needs activation codes (a_bits <= 8), w_bits 1..7, w_group 64 / 128 / 256 / 512 or 0 (per
                            channel: then the loop has no rescale and the linear runs about 1.5 times faster than in bf16), d_model and
                            d_ffn multiples of 256, no learned tensors, no lightweight variant -- zo_init returns ZO_EUNSUPPORTED
                            otherwise.  It applies to forwards that quantize once (more than 128 tokens, or no_fused = 1); the lm_head is
                            not quantized and keeps its bf16 contraction.  A weight group whose zero point lies so far outside its
                            range that code - zero point does not fit a signed byte cannot be represented: the forward then reports
                            NaN losses (use ZO_MMA_BF16 for such weights). */
} zo_config;

/* One parameter tensor.  The array given to zo_init lists them in the fixed order below; the
 * position in the array is the tensor number used by the perturbation stream.
 *   linear:  W[d_ffn][d_model]
 *   llama:   tok_emb[V][d]; per layer: attn_norm[d], wq, wk, wv, wo [d][d], ffn_norm[d],
 *            w_gate[f][d], w_up[f][d], w_down[d][f]; then final_norm[d], lm_head[V][d]
 *   opt:     tok_emb[V][d], pos_emb[max_seq][d]; per layer: ln1_g, ln1_b, wq, bq, wk, bk, wv, bv,
 *            wo, bo, ln2_g, ln2_b, fc1[f][d], b1[f], fc2[d][f], b2[d]; then final_ln_g,
 *            final_ln_b, lm_head[V][d]
 *   With learn_clip / learn_smooth the list continues, for every quantized linear in the order above:
 *   (learn_clip) step, zero point, alpha, beta, each [N][K/w_group] (per channel: [N][1]);
 *   (learn_smooth, only for the first linear of those that read the same activation: wq for wq/wk/wv,
 *   w_gate for w_gate/w_up, every other linear for itself) s[K], delta[K].
 *   Learning-rate groups: the model's tensors 0, smoothing tensors 1, quantizer tensors 2.         */
typedef struct {
    void*   ptr;        /* dev, master weights (fp32, or binary16 with ZO_MASTER_F16), updated in place by zo_update / zo_step; may be
                           NULL for a frozen quantized linear of a lightweight configuration whose
                           packed form is attached with zo_attach_frozen_int4 */
    int64_t numel;
    int32_t trainable;  /* used only when zo_config.lightweight = 1 */
    int32_t reserved;
} zo_tensor;

typedef struct zo_ctx zo_ctx;

/* Number of parameter tensors the configuration expects (0 if the configuration is invalid). */
int32_t zo_num_params(const zo_config* cfg);
/* Element count of parameter tensor `index` (-1 if out of range). */
int64_t zo_param_numel(const zo_config* cfg, int32_t index);

/* Bytes of device workspace a context needs to run B x S tokens (B rows for the linear arch). */
size_t zo_workspace_bytes(const zo_config* cfg, int32_t B, int32_t S);

/* Create a context.  `params` (host array) is copied; the tensors stay owned by the caller.
 * `workspace` (dev) must hold zo_workspace_bytes(cfg, max_B, max_S) bytes and stay valid until
 * zo_destroy.  Constant tables (rotary angles) are written into the workspace on `hip_stream`. */
zo_status zo_init(const zo_config* cfg, const zo_tensor* params, int32_t n_params,
                  void* workspace, size_t workspace_bytes, int32_t max_B, int32_t max_S,
                  void* hip_stream, zo_ctx** out);
zo_status zo_destroy(zo_ctx* ctx);
/* Text of the last error of this context (host string owned by the context). */
const char* zo_last_error(const zo_ctx* ctx);

/* One quantized forward at W + eps_signed * u(seed): L(Q(W + eps_signed u); batch) of Eq. 2.
 *   ids      dev int32 [B][S] token ids (decoders); for the linear arch: dev input X[B][d_model]
 *            in the activation storage type
 *   target   dev fp32 [B][d_ffn] regression target (linear arch only, else NULL)
 *   loss_dev dev fp32[1], written asynchronously
 * eps_signed = +eps, -eps, or 0 for the unperturbed quantized model. */
zo_status zo_forward_quant(zo_ctx* ctx, const void* ids, const float* target, int32_t B, int32_t S,
                           uint64_t seed, float eps_signed, float* loss_dev);

/* One full step: both forwards of Eq. 2 (sharing one pass over the weights), the projected
 * gradient, and the update of Eq. 3.  out_dev: dev fp32[4] = { L+, L-, g, eta*g }. */
zo_status zo_step(zo_ctx* ctx, const void* ids, const float* target, int32_t B, int32_t S,
                  uint64_t seed, float eps, float lr, float* out_dev);

/* Update of Eq. 3 alone: w_i <- w_i - c * u(seed, tensor, i) over every trainable tensor.
 * c is read from coeff_dev (dev fp32[1]) if non-NULL, else coeff_host is used. */
zo_status zo_update(zo_ctx* ctx, uint64_t seed, const float* coeff_dev, float coeff_host);

/* ---- q > 1 directions per step (Eq. 2 as printed: the average over q directions u_i), step-size schedule, replay ----
 * zo_step_multi: for i < q the pair of losses at W +- eps u(seeds[i]) -- every direction at the same, not yet
 * updated W -- gives g_i; then W <- W - sum_i (lr_group / q) g_i u(seeds[i]) in ONE pass over the masters, the q
 * terms applied in the order of the seeds, one fused multiply-add each (lr / q is one fp32 division).
 *   seeds_host  host uint64 [q], q in 1..ZO_MAX_DIRECTIONS
 *   out_dev     dev fp32 [q][6] = { L+, L-, g_i, (lr_model/q) g_i, (lr_smooth/q) g_i, (lr_clip/q) g_i }
 * q = 1 is zo_step_groups. */
enum { ZO_MAX_DIRECTIONS = 16 };
zo_status zo_step_multi(zo_ctx* ctx, const void* ids_dev, const float* target_dev, int32_t B, int32_t S,
                        const uint64_t* seeds_host, int32_t q, float eps, float lr_model, float lr_smooth, float lr_clip,
                        float* out_dev);
/* The update of zo_step_multi alone.  coeff_dev: dev fp32 [q][6] rows as zo_step_multi writes them (columns 3..5
 * are read), or NULL and coeff_host: host fp32 [q][3] = the three group coefficients of every direction.
 * A run is reproduced exactly, without any forward pass, by replaying its log of (seeds, coefficients). */
zo_status zo_update_multi(zo_ctx* ctx, const uint64_t* seeds_host, int32_t q, const float* coeff_dev, const float* coeff_host);
/* Step size of iteration t = 0 .. T-1 under the linear-decay schedule of the pre-training recipe (Appendix,
 * hyperparameter table): lr0 (1 - t/T), evaluated in double, returned as float.  Host function. */
float zo_lr_linear_decay(float lr0, int64_t t, int64_t T);

/* Per-launch timing of the context's own work with HIP events recorded on its stream (the
 * stream the kernels run on).  Between zo_profile_begin and zo_profile_end every group of launches
 * is bracketed by two events.  zo_profile_end synchronises the stream and returns, per category,
 * the summed elapsed milliseconds and the number of bracketed groups (host arrays of
 * ZO_PROF_CATEGORIES entries).  A "GEMM" group is exactly one launch of the GEMM kernel (both
 * branches of Eq. 2 batched in it). */
enum { ZO_PROF_GEMM = 0, ZO_PROF_WEIGHT_QUANT = 1, ZO_PROF_ACT_QUANT = 2, ZO_PROF_ATTENTION = 3,
       ZO_PROF_UPDATE = 4, ZO_PROF_OTHER = 5, ZO_PROF_FUSED = 6 /* a group = one launch of the fused small-M kernel (one parameter tensor) */,
       ZO_PROF_FUSED_INT4 = 7 /* a group = one launch of the small-M kernel that expands packed codes */,
       ZO_PROF_CATEGORIES = 8 };
zo_status zo_profile_begin(zo_ctx* ctx);
/* The same with only the categories whose bit (1 << ZO_PROF_*) is set in category_mask bracketed: an event pair costs a few
 * microseconds of idle stream between two kernels (about 1.5 % of a 7B-shaped step when every launch is bracketed), so a timed
 * region brackets only the kernel whose duration it needs. */
zo_status zo_profile_begin_mask(zo_ctx* ctx, uint32_t category_mask);
zo_status zo_profile_end(zo_ctx* ctx, float* ms_host, int32_t* launches_host);

/* ---- stand-alone pieces of the path (same device code as the step), for tests and benches ---- */

/* out[j] = word (j & 3) of Philox4x32-10 block (j >> 2) of the stream (seed, tensor_id). */
zo_status zo_debug_philox_u32(uint64_t seed, int32_t tensor_id, int64_t nwords, uint32_t* out_dev, void* hip_stream);
/* Measurement probe (for benchmarks; no part of the step -- it serves the measurement contract, not a passage of the paper):
 * `workgroups` workgroups of four waves issue iters * 8 bf16 matrix instructions (32 x 32 x 16) per wave on register-resident
 * operands, with no memory traffic: 4 * 8 * 32768 * iters flop per workgroup.  zero_operands = 1: all-zero operands; 0: random
 * mantissas (the power-managed clock depends on the data).  out_dev: dev fp32 [workgroups * 256], receives the accumulator sums.
 * The caller times the launch on hip_stream. */
zo_status zo_probe_mfma_only(float* out_dev, int32_t workgroups, int32_t iters, int32_t zero_operands, void* hip_stream);
/* out[i] = u(seed, tensor_id, start + i), i < numel: the perturbation of Eq. 2. */
zo_status zo_debug_normal(uint64_t seed, int32_t tensor_id, int64_t start, int64_t numel, float* out_dev, void* hip_stream);

/* Seeded in-place update of one tensor (Eq. 3): w_i <- w_i - c * u(seed, tensor_id, i). */
zo_status zo_update_tensor(float* w_dev, int64_t numel, uint64_t seed, int32_t tensor_id,
                           const float* coeff_dev, float coeff_host, void* hip_stream);

/* The same for a tensor kept in IEEE binary16: w_i <- round16(fma(-c, u(seed, tensor_id, i), w_i)), nearest even or
 * (stochastic != 0) stochastic rounding. */
zo_status zo_update_tensor_f16(void* w_dev, int64_t numel, uint64_t seed, int32_t tensor_id,
                               const float* coeff_dev, float coeff_host, int32_t stochastic, void* hip_stream);

/* Bytes of master-weight storage a configuration asks the caller for (all tensors of the parameter list in
 * master_dtype; -1 if the configuration is invalid): the "weights only, independent of the batch size" memory of
 * the efficiency section's table.  Host function. */
int64_t zo_master_bytes(const zo_config* cfg);

/* Q(W + eps_signed u) of one weight matrix W[N][K] (Eq. 2's argument of L for one linear):
 * perturb, group min/max, quantize, de-quantize.  bits = 0: perturb only.  Outputs (any may be
 * NULL): codes u8 [N][K]; step fp32 and zp int32 [N][K/group]; what [N][K] de-quantized weights in
 * storage type out_dtype (ZO_ACT_*).  group = 0 means K. */
zo_status zo_debug_quant_weight(const float* W_dev, int32_t N, int32_t K, int32_t bits, int32_t group,
                                uint64_t seed, int32_t tensor_id, float eps_signed, int32_t out_dtype,
                                uint8_t* codes_dev, float* step_dev, int32_t* zp_dev, void* what_dev,
                                void* hip_stream);

/* ---- adaptive weight quantizer (Eq. 5) and channel-wise smoothing (Eq. 4) as ZO-trained tensors ----
 * Eq. 5: code = clamp(round(w/step) + z, alpha Q_P, beta Q_P), w^ = (code - z) step, with step, z, alpha,
 * beta learnable per group.  The four are real-valued fp32 tensors that the step perturbs and updates;
 * inside a forward z and the two bounds are rounded half-to-even, the bounds kept inside [0, Q_P] and
 * ordered, the step floored at 1e-5.  Eq. 4: Y = [(X - delta) / s] [s (.) W] + [B + delta W]: the per-token
 * quantizer sees (x - delta) * (1/s) (one division per channel), the weight quantizer s (.) (W +- eps u),
 * and the bias gains delta (W +- eps u)^T. */

/* Fill the tensors of Eq. 5 / Eq. 4 of a context (caller's memory, on the context's stream): s = 1,
 * delta = 0; step and zero point as the default asymmetric scheme computes them from W, alpha = 0, beta = 1
 * (the initial values the paragraph on the adaptive weight quantizer, Eq. 5, prescribes).  Uses the workspace as scratch. */
zo_status zo_init_learned_params(zo_ctx* ctx);

/* zo_step with one learning rate per group (Appendix, hyperparameter table: model, smoothing, clipping).
 * out_dev fp32[6] = { L+, L-, g, lr_model g, lr_smooth g, lr_clip g }. */
zo_status zo_step_groups(zo_ctx* ctx, const void* ids_dev, const float* target_dev, int32_t B, int32_t S,
                         uint64_t seed, float eps, float lr_model, float lr_smooth, float lr_clip, float* out_dev);

/* zo_update with one coefficient per group: coeff_dev fp32[3] on the device, or (if NULL) coeff_host[3]. */
zo_status zo_update_groups(zo_ctx* ctx, uint64_t seed, const float* coeff_dev, const float* coeff_host);

/* Eq. 5 on scale (.) (W + eps_signed u) for one matrix W[N][K]; step/zp/alpha/beta dev fp32 [N][K/group]
 * (already perturbed), scale dev fp32 [K] or NULL.  Outputs: codes u8 [N][K] (may be NULL), what [N][K]
 * in storage type out_dtype. */
zo_status zo_debug_quant_weight_learned(const float* W_dev, int32_t N, int32_t K, int32_t bits, int32_t group,
                                        uint64_t seed, int32_t tensor_id, float eps_signed,
                                        const float* scale_dev, const float* step_dev, const float* zp_dev,
                                        const float* alpha_dev, const float* beta_dev, int32_t out_dtype,
                                        uint8_t* codes_dev, void* what_dev, void* hip_stream);

/* Bias term of Eq. 4: out[n] = bias[n] + sum_k delta[k] (W[n][k] + eps_signed u); bias may be NULL.
 * fp32 accumulation in a fixed order. */
zo_status zo_debug_smooth_bias(const float* W_dev, int32_t N, int32_t K, uint64_t seed, int32_t tensor_id, float eps_signed,
                               const float* delta_dev, const float* bias_dev, float* out_dev, void* hip_stream);

/* Per-token quantizer of the input of a quantized linear: every row of X[M][K] (storage type
 * dtype) is one group.  Outputs (any may be NULL): codes int16 [M][K], step fp32 [M], zp int32 [M],
 * xhat [M][K] de-quantized in the same storage type. */
zo_status zo_debug_quant_act(const void* X_dev, int32_t M, int32_t K, int32_t bits, int32_t sym, int32_t dtype,
                             int16_t* codes_dev, float* step_dev, int32_t* zp_dev, void* xhat_dev,
                             void* hip_stream);

/* One fake-quantized linear layer: Y = Q_A(X) * Q(W + eps_signed u)^T (+ bias).
 *   X  dev [M][K] storage type dtype;  W dev fp32 [N][K];  bias dev fp32 [N] or NULL (not perturbed)
 *   Y  dev [M][N] storage type dtype
 *   scratch dev, at least zo_linear_scratch_bytes(M, N, K, dtype) bytes */
size_t zo_linear_scratch_bytes(int32_t M, int32_t N, int32_t K, int32_t dtype);
zo_status zo_linear_fakequant(const void* X_dev, const float* W_dev, const float* bias_dev, void* Y_dev,
                              int32_t M, int32_t N, int32_t K, int32_t w_bits, int32_t w_group,
                              int32_t a_bits, int32_t a_sym, int32_t dtype,
                              uint64_t seed, int32_t tensor_id, float eps_signed,
                              void* scratch_dev, void* hip_stream);

/* The same layer with the contraction chosen by `mma`:
 *   ZO_MMA_BF16  zo_linear_fakequant as above: both operands de-quantized, rounded to the storage type, bf16 (or fp32) GEMM;
 *   ZO_MMA_INT8  the contraction runs on the integer codes (Background/Quantization: X_INT; Appendix/Quantization settings:
 *                per-token activation codes, per-group weight codes) with the int8 matrix instructions:
 *                    y[t][n] = step_x[t] * sum_g step_w[n][g] * sum_{k in g} (qx[t][k] - zx[t]) (qw[n][k] - zw[n][g])
 *                i.e. x^ w^^T with NEITHER operand rounded -- the inner sums are exact integers, one fp32 multiply-add per
 *                weight group.  Needs weight and activation codes (1 <= w_bits <= 7, 2 <= a_bits <= 8), K a multiple of
 *                128, w_group 64, 128, 256 or 512, or 0 / K = per channel (K <= 65536: the integer sums then run over all of K
 *                inside the matrix unit and the loop has no rescale at all); otherwise ZO_EUNSUPPORTED.  A weight group whose
 *                |qw - zw| exceeds 127 (a group far from zero compared with its own range: the zero point is not clamped)
 *                does not fit a signed byte: its operands are saturated and *flag_dev is OR-ed with 1 -- the caller clears
 *                the flag before the call and must discard Y if it is set.
 *   X dev [M][K] storage type dtype; Y dev [M][N], fp32 if out_f32 else bf16 (ZO_MMA_BF16: the storage type);
 *   scratch dev, zo_linear_mma_scratch_bytes(...) bytes; offsets_host (may be NULL) receives, for ZO_MMA_INT8, the byte
 *   offsets inside the scratch of: activation codes qx - O as int8 [M][K] (O = 2^(a_bits-1), 0 if a_sym), token steps fp32 [M],
 *   O - zx fp32 [M], weight operands qw - zw int8 [N][K], weight steps (kernel order), r[n] = sum_g step_w sum_k (qw - zw)
 *   fp32 [N], its per-group parts fp32 [N][K/w_group] (not written per channel), end -- for parity tests. */
enum { ZO_MMA_BF16 = 0, ZO_MMA_INT8 = 1 };
size_t zo_linear_mma_scratch_bytes(int32_t M, int32_t N, int32_t K, int32_t w_group, int32_t dtype, int32_t mma, size_t* offsets_host);
zo_status zo_linear_fakequant_mma(const void* X_dev, const float* W_dev, const float* bias_dev, void* Y_dev,
                                  int32_t M, int32_t N, int32_t K, int32_t w_bits, int32_t w_group,
                                  int32_t a_bits, int32_t a_sym, int32_t dtype, int32_t out_f32, int32_t mma,
                                  uint64_t seed, int32_t tensor_id, float eps_signed, void* scratch_dev, int32_t* flag_dev,
                                  void* hip_stream);

/* The same layer for both branches of Eq. 2 at once and a small token count (1 <= M <= 128), fused: one pass
 * over the fp32 master builds the tiles of Q(W + eps u) and Q(W - eps u) in registers, in matrix-core operand
 * layout, and multiplies them with the branches' (already quantized) inputs; neither set of weights is ever
 * written anywhere.  Yp = Xp Q(W + eps u)^T + bias, Ym = Xm Q(W - eps u)^T + bias.
 *   Xp, Xm  dev bf16 [M][K] (may be the same buffer); Ym = NULL: one branch only, at W + eps u (eps signed)
 *   W       dev fp32 [N][K]; bias dev fp32 [N] or NULL; Yp, Ym dev [M][N], fp32 if out_f32 else bf16
 *   w_bits 0..8 (0: perturbed, not quantized); w_group in {8, 16, 32, 64, 128} dividing K; N a multiple
 *   of 16, K of 32; otherwise ZO_ESHAPE.  Same arithmetic per weight as zo_debug_quant_weight; only the
 *   order of the fp32 accumulation differs from zo_linear_fakequant.
 *   scratch dev, NULL or zo_linear_fused_scratch_bytes(M, K) bytes: if given, the activations are first copied
 *   into it in the order the kernel consumes them (contiguous loads instead of 16-byte gathers; faster from
 *   M ~ 48 on, identical results). */
size_t zo_linear_fused_scratch_bytes(int32_t M, int32_t K);
zo_status zo_linear_fakequant_fused(const void* Xp_dev, const void* Xm_dev, const float* W_dev, const float* bias_dev,
                                    void* Yp_dev, void* Ym_dev, int32_t M, int32_t N, int32_t K, int32_t w_bits,
                                    int32_t w_group, uint64_t seed, int32_t tensor_id, float eps, int32_t out_f32,
                                    void* scratch_dev, void* hip_stream);

/* ---- frozen, pre-quantized weights (Section "Lightweight ZeroQAT for memory reduction"): most
 * parameters are frozen and stored quantized, only the query and value projections stay in full
 * precision and trainable.  Storage of one frozen linear W[N][K], groups of `group` consecutive k
 * (a power of two in 8..512 dividing K):
 *   codes     u8   [N][K/2]      4-bit codes, k = 2j in the low nibble of byte j, k = 2j+1 in the high
 *   step_f16  f16  [N][K/group]  group step, IEEE binary16
 *   zp        i16  [N][K/group]  group zero point
 * and the operand of the GEMM is w^[n][k] = (code - zp) * step, the same for both branches of
 * Eq. 2 (no perturbation, no update). ---- */

/* Pre-quantize an fp32 matrix into that form: the asymmetric 4-bit group quantizer of the Background
 * section at eps = 0, step rounded to binary16 (nearest even), zero point saturated to int16.
 * All pointers dev; codes 16-byte aligned.  ZO_ESHAPE if the group rule is violated. */
zo_status zo_pack_weight_int4(const float* W_dev, int32_t N, int32_t K, int32_t group,
                              void* codes_dev, void* step_f16_dev, int16_t* zp_dev, void* hip_stream);

/* Give tensor `index` of a lightweight context its packed storage (dev pointers, owned by the
 * caller, valid until zo_destroy).  The tensor must be a quantized linear with trainable = 0; its
 * zo_tensor.ptr is ignored from then on.  A forward fails with ZO_EINVAL while some tensor has
 * neither fp32 nor packed storage. */
zo_status zo_attach_frozen_int4(zo_ctx* ctx, int32_t index, const void* codes_dev, const void* step_f16_dev,
                                const int16_t* zp_dev, int32_t group);

/* One frozen linear layer alone: Y = Q_A(X) * w^^T (+ bias), X and Y [M][*] in storage type dtype,
 * a_bits = 16 skips the per-token quantizer.  scratch dev: zo_linear_scratch_bytes(M, N, K, dtype)
 * bytes; on return its second part (offset = M*K*sizeof(dtype) rounded up to 256) holds w^ [N][K]. */
zo_status zo_linear_frozen_int4(const void* X_dev, const void* codes_dev, const void* step_f16_dev, const int16_t* zp_dev,
                                const float* bias_dev, void* Y_dev, int32_t M, int32_t N, int32_t K, int32_t group,
                                int32_t a_bits, int32_t a_sym, int32_t dtype, void* scratch_dev, void* hip_stream);

/* The same layer for a small token count (1 <= M <= 128) and both branches at once, fused: the operand w^ is expanded
 * from the packed codes in registers, in matrix-core operand layout (0.5 B of HBM traffic per weight, nothing
 * written but Y); the two branches share it.  Also the linear of plain inference on the packed model.
 *   Xp, Xm dev bf16 [M][K] (already quantized per token if the configuration asks for it); Ym = NULL: one branch
 *   Yp, Ym dev [M][N], fp32 if out_f32 else bf16; bias dev fp32 [N] or NULL
 *   group in {32, 64, 128, 256, 512} dividing K, N a multiple of 16; otherwise ZO_ESHAPE
 *   scratch dev, NULL or zo_linear_frozen_fused_scratch_bytes(M, N, K, group) bytes.  Without scratch a workgroup covers
 *   16 channels and all of K (every workgroup then reads all of X: slow beyond a few tokens); with it the activations
 *   are copied into fragment order, a workgroup covers 128 channels and one of several K ranges, and the partial sums
 *   (fp32, in the scratch) are added in a fixed order by a second kernel.
 * Same arithmetic per weight as zo_linear_frozen_int4; only the order of the fp32 accumulation differs. */
size_t zo_linear_frozen_fused_scratch_bytes(int32_t M, int32_t N, int32_t K, int32_t group);
zo_status zo_linear_frozen_int4_fused(const void* Xp_dev, const void* Xm_dev, const void* codes_dev, const void* step_f16_dev,
                                      const int16_t* zp_dev, const float* bias_dev, void* Yp_dev, void* Ym_dev, int32_t M, int32_t N,
                                      int32_t K, int32_t group, int32_t out_f32, void* scratch_dev, void* hip_stream);

/* The frozen linear for ONE token (the linear of a decoding step of the generator below; Lightweight section: pre-quantized
 * weights): y[n] = relu?(sum_k x[k] (code[n][k] - zp[n][g]) step[n][g] + bias[n]) + residual[n], reading 0.5 B per weight.
 *   x dev bf16 [K]; y dev [N] bf16, or fp32 if out_f32; bias dev fp32 [N] or NULL; residual dev bf16 [N] or NULL (may be y)
 *   N a multiple of 4, K a multiple of 32, group a power of two >= 32 dividing K; otherwise ZO_ESHAPE.
 * The products x (code - zp) step are formed WITHOUT rounding the de-quantized weight to bf16 first (exact bf16 x integer
 * products summed in fp32, one multiplication by the step per 32 weights): closer to the quantizer's definition than the
 * bf16-rounded operand of zo_linear_frozen_int4, from which it differs by at most 2^-9 relative per weight. */
zo_status zo_linear_frozen_int4_token(const void* x_dev, const void* codes_dev, const void* step_f16_dev, const int16_t* zp_dev,
                                      const float* bias_dev, const void* residual_dev, int32_t relu, void* y_dev, int32_t N, int32_t K,
                                      int32_t group, int32_t out_f32, void* hip_stream);

/* Plain GEMM of the path, Y[M][N] = X[M][K] * W[N][K]^T with fp32 accumulation, operands and
 * output in storage type dtype (the contraction every quantized linear runs after both operands
 * have been de-quantized).  Exposed for roofline measurement and parity. */
zo_status zo_gemm_nt(const void* X_dev, const void* W_dev, void* Y_dev, int32_t M, int32_t N, int32_t K,
                     int32_t dtype, void* hip_stream);

/* The same GEMM with the epilogue the decoder layers fuse into it:
 *   Y = relu?(X * W^T + bias) + residual,   bias dev fp32 [N] or NULL, residual dev [M][N] in
 * storage type dtype or NULL (may be Y itself: the residual stream is updated in place), relu != 0
 * applies max(., 0) before the residual is added.  One rounding to the storage type at the end. */
zo_status zo_gemm_nt_fused(const void* X_dev, const void* W_dev, const float* bias_dev, const void* residual_dev, int32_t relu,
                           void* Y_dev, int32_t M, int32_t N, int32_t K, int32_t dtype, void* hip_stream);

/* The same fused GEMM with scratch memory that lets the library split K (the GEMM of the quantized linear layers at the
 * token counts of the paper's fine-tuning runs: a few hundred tokens and the narrow outputs of the attention-output
 * and down projections give too few tiles to occupy the chip).  zo_gemm_nt_splitk_ranges tells how many K ranges the shape
 * gets (1: computed exactly as zo_gemm_nt_fused does, scratch unused), zo_gemm_nt_splitk_scratch_bytes how much scratch
 * they need (0 for one range).  Every range's partial sums are kept in fp32 in the scratch and added in range order by a
 * second kernel, which applies the epilogue: the result does not depend on scheduling; it differs from the unsplit
 * kernel's only by the order of the fp32 additions.  scratch dev, 16-byte aligned, or NULL (no split); a scratch smaller
 * than asked for also means no split.  Errors as zo_gemm_nt_fused. */
int32_t zo_gemm_nt_splitk_ranges(int32_t M, int32_t N, int32_t K, int32_t dtype);
size_t zo_gemm_nt_splitk_scratch_bytes(int32_t M, int32_t N, int32_t K, int32_t dtype);
zo_status zo_gemm_nt_fused_splitk(const void* X_dev, const void* W_dev, const float* bias_dev, const void* residual_dev, int32_t relu,
                                  void* Y_dev, int32_t M, int32_t N, int32_t K, int32_t dtype, void* scratch_dev, size_t scratch_bytes,
                                  void* hip_stream);

/* zo_gemm_nt_fused_splitk for callers that cannot allocate device memory (code under HIP graph capture, tight
 * serving loops, harnesses that forbid hipMalloc): no scratch argument.  The partial sums of the K ranges go to a device
 * array that is part of the library (zo_gemm_nt_splitk_static_max_bytes() = 32 MiB, held on every GPU the library is
 * loaded on until the process ends); the call allocates and frees nothing, on the device or through any library.
 * Same kernels, same K ranges, bit-identical results to zo_gemm_nt_fused_splitk with a scratch of
 * zo_gemm_nt_splitk_scratch_bytes bytes.  ZO_EWORKSPACE (nothing launched) if the shape's K ranges need more than the
 * array holds; other errors as zo_gemm_nt_fused.  All calls on one GPU share the one array: calls that may overlap on a
 * GPU (different streams, different threads) race on it -- keep them on one stream or order them with events.  Nothing
 * has to be cleared between calls (every partial sum is written before it is read). */
size_t zo_gemm_nt_splitk_static_max_bytes(void);
zo_status zo_gemm_nt_fused_splitk_static(const void* X_dev, const void* W_dev, const float* bias_dev, const void* residual_dev,
                                         int32_t relu, void* Y_dev, int32_t M, int32_t N, int32_t K, int32_t dtype,
                                         void* hip_stream);

/* The gate / up GEMM of a SwiGLU block with the activation in its epilogue (what large bf16 Llama-shaped forwards run):
 *   W dev bf16 [N2][K]: rows of the gate and the up projection interleaved in blocks of 32 channels -- rows 64 i .. 64 i + 31
 *   = gate channels 32 i .., rows 64 i + 32 .. 64 i + 63 = up channels 32 i ..;  X dev bf16 [M][K];
 *   Y dev bf16 [M][N2/2] = rt(silu(rt(X gate^T)) * rt(X up^T)), silu(x) = x / (1 + exp(-x)), rt = rounding to bf16 (the
 *   same values as storing gate and up first).  ZO_EUNSUPPORTED unless M * N2 >= 2^23, N2 and K multiples of 64. */
zo_status zo_gemm_nt_swiglu(const void* X_dev, const void* W_dev, void* Y_dev, int32_t M, int32_t N2, int32_t K, void* hip_stream);

/* The lm_head GEMM with the next-token cross entropy formed in its epilogue (the loss of the ZO objective, Eq. 2, on a
 * decoder: the logits X W^T are never stored).  X dev bf16 [M][K] (M = B*S rows, S positions per sequence), W dev bf16
 * [N][K] (N = vocabulary), ids dev int32 [M]: row m's target is ids[m + 1], clamped to [0, N); rows at the last position of a
 * sequence have none.  row_loss dev fp32 [M] = log sum_n exp(logit[m][n]) - logit[m][target] (0 at last positions).
 * scratch dev, zo_gemm_nt_ce_scratch_bytes(M, N) bytes, 16-byte aligned, overwritten.  ZO_EUNSUPPORTED unless
 * M * N >= 2^23 and K a multiple of 64; ZO_ESHAPE unless S divides M. */
size_t zo_gemm_nt_ce_scratch_bytes(int32_t M, int32_t N);
zo_status zo_gemm_nt_ce(const void* X_dev, const void* W_dev, const int32_t* ids_dev, float* row_loss_dev, int32_t M, int32_t S,
                        int32_t N, int32_t K, void* scratch_dev, void* hip_stream);

/* Causal softmax attention of the decoder forward: for every batch b, head h and position s,
 * out[b,s,h,:] = sum_{j<=s} softmax_j(q[b,s,h,:].k[b,j,h,:] / sqrt(dh)) v[b,j,h,:].
 * q, k, v: dev, storage type dtype, element (b,s,h,i) at ((b*S + s) * row_stride + h*dh + i)
 * (row_stride lets them live inside one fused [B*S][3*H*dh] buffer); out: dev [B*S][H*dh].
 * dh must be 16, 32, 64 or 128 and row_stride a multiple of 8.  scratch: dev buffer of
 * zo_attention_scratch_bytes(...) bytes; no kernel uses one any more: the size is 0 and NULL is accepted. */
size_t zo_attention_scratch_bytes(int32_t B, int32_t S, int32_t H, int32_t dh, int32_t dtype);
zo_status zo_attention_causal(const void* q_dev, const void* k_dev, const void* v_dev, void* out_dev,
                              int32_t B, int32_t S, int32_t H, int32_t dh, int64_t row_stride, int32_t dtype,
                              void* scratch_dev, void* hip_stream);

/* ---- the quantized model as a generator (efficiency section, on-device table: inference on the quantized model,
 * prompts of a few hundred tokens, one token at a time afterwards) ----
 * The same quantized forward at eps = 0 on ONE sequence, with a key / value cache in caller-owned memory:
 *   kv_dev  dev, zo_kv_cache_bytes(cfg, kv_max_seq) bytes, 16-byte aligned, layout [n_layers][K | V][kv_max_seq][d_model] in the
 *           activation storage type; keys are stored after the rotary embedding.  kv_max_seq <= cfg.max_seq.
 * zo_prefill: rows 0 .. S-1 of the prompt ids_dev (dev int32 [S], S <= max_B * max_S of the context) fill the cache; logits_dev
 *   (dev fp32 [vocab]) receives the logits of the LAST position (the distribution of the first generated token).
 * zo_decode: one more token (*token_dev, dev int32 -- typically written by the previous step's arg max) at position pos
 *   (= number of cached rows): its keys / values are appended, its query attends to rows 0 .. pos; logits_dev as above.
 * zo_generate_greedy: zo_prefill, then n_new times { tokens_dev[i] = arg max of the logits (lowest index on ties);
 *   zo_decode(tokens_dev + i, S + i) } -- everything queued on the context's stream, no host round trip between tokens.
 * Works on any decoder context without learned quantizer tensors; meant for a lightweight context whose quantized linears
 * are all attached as packed 4-bit codes (zo_attach_frozen_int4), where a decoding step reads 0.5 B per weight. */
size_t zo_kv_cache_bytes(const zo_config* cfg, int32_t kv_max_seq);
zo_status zo_prefill(zo_ctx* ctx, const int32_t* ids_dev, int32_t S, void* kv_dev, int32_t kv_max_seq, float* logits_dev);
zo_status zo_decode(zo_ctx* ctx, const int32_t* token_dev, int32_t pos, void* kv_dev, int32_t kv_max_seq, float* logits_dev);
zo_status zo_generate_greedy(zo_ctx* ctx, const int32_t* prompt_dev, int32_t S, int32_t n_new, void* kv_dev, int32_t kv_max_seq,
                             int32_t* tokens_dev, float* logits_dev);

/* Which optional routes the context's last forward (or step) took: an OR of ZO_ROUTE_* bits.  Host function. */
enum { ZO_ROUTE_FUSED_SMALL_M = 1,    /* linears built from the masters inside the small-M kernel */
       ZO_ROUTE_FUSED_INT4 = 2,       /* frozen linears expanded from their packed codes inside the small-M kernel */
       ZO_ROUTE_SWIGLU_IN_GEMM = 4,   /* SwiGLU applied by the epilogue of the gate / up GEMM */
       ZO_ROUTE_ROPE_IN_GEMM = 8,     /* rotary embedding applied by the epilogue of the q | k | v GEMM */
       ZO_ROUTE_CE_IN_GEMM = 16,      /* cross entropy formed by the epilogue of the lm_head GEMM, no logits stored */
       ZO_ROUTE_GEMM_SPLIT_K = 32,    /* some linear's GEMM ran with K split into ranges (see zo_gemm_nt_fused_splitk) */
       ZO_ROUTE_INT8_MMA = 64 };      /* quantized linears contracted on their integer codes (zo_config.mma = ZO_MMA_INT8) */
uint32_t zo_debug_routes(const zo_ctx* ctx);

/* Device buffers of the context's last forward, for layer-level parity tests.
 * which: 0 = final hidden state [M][d], 1 = logits fp32 [M][V] (linear arch: output Y [M][N]; ZO_EUNSUPPORTED after a
 *        forward that took ZO_ROUTE_CE_IN_GEMM: it stored none),
 *        2 = residual stream after the last layer [M][d], 3 = q | k | v of the last layer [M][3d] (q and k after the
 *        rotary embedding where the architecture has one), 4 = attention output of the last layer [M][d].
 *        branch: 0 = '+' (or the single forward), 1 = '-'.  Returns the dev pointer in *ptr and its size in *bytes. */
zo_status zo_debug_buffer(zo_ctx* ctx, int32_t which, int32_t branch, void** ptr, size_t* bytes);

#ifdef __cplusplus
}
#endif
#endif /* ZOQAT_H */
