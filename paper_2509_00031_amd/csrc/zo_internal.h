// Host-side launchers of the HIP kernels (internal to the library; the public C ABI is zoqat.h).
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

enum { ZO_T_F32 = 0, ZO_T_BF16 = 1 };          // storage type of activations / GEMM operands
enum { ZO_W_F32 = 0, ZO_W_F16 = 1 };           // storage type of the master weights (IEEE binary32 / binary16)

static inline size_t zo_tsize(int dtype) { return dtype == ZO_T_BF16 ? 2 : 4; }

// ---- perturbation stream ---------------------------------------------------------------------
hipError_t zo_launch_philox_words(uint64_t seed, int32_t tid, int64_t nwords, uint32_t* out, hipStream_t st);
hipError_t zo_launch_normal(uint64_t seed, int32_t tid, int64_t start, int64_t n, float* out, hipStream_t st);

// ---- update (Eq. 3) ----------------------------------------------------------------------------
hipError_t zo_launch_update(float* w, int64_t numel, uint64_t seed, int32_t tid,
                            const float* coeff_dev, float coeff_host, hipStream_t st);

// q directions at once: terms applied in order d = 0 .. q-1; coefficient of direction d = coeff_dev[d * coeff_stride]
// (device) if coeff_dev, else ms.c[d]
#define ZO_MAX_DIRECTIONS_INTERNAL 16
struct zo_multi_seeds { uint32_t k0[ZO_MAX_DIRECTIONS_INTERNAL], k1[ZO_MAX_DIRECTIONS_INTERNAL]; float c[ZO_MAX_DIRECTIONS_INTERNAL]; };
hipError_t zo_launch_update_multi(float* w, int64_t numel, const zo_multi_seeds& ms, int32_t q, int32_t tid,
                                  const float* coeff_dev, int32_t coeff_stride, hipStream_t st);

// binary16 masters: the q terms in fp32, then one rounding (stochastic != 0: driven by the rounding stream of seed 0)
hipError_t zo_launch_update_f16(void* w, int64_t numel, const zo_multi_seeds& ms, int32_t q, int32_t tid,
                                const float* coeff_dev, int32_t coeff_stride, int32_t stochastic, hipStream_t st);

// ---- weight fake-quantizer ---------------------------------------------------------------------
// Emits Q(W + eps u) into out_plus and/or Q(W - eps u) into out_minus (storage type dtype); either
// may be NULL.  bits = 0: perturbed weights, not quantized.  Debug outputs describe the '+' branch.
bool zo_fq_weight_supported(int32_t K, int32_t bits, int32_t group);
hipError_t zo_launch_fq_weight(const void* W, int32_t N, int32_t K, int32_t bits, int32_t group,
                               uint64_t seed, int32_t tid, float eps, int dtype,
                               void* out_plus, void* out_minus,
                               uint8_t* codes, float* step, int32_t* zp, hipStream_t st, int wdtype = ZO_W_F32, int ilv = 0);
// ilv: 0 = rows written where they are read; 1 / 2 = rows of a gate / up projection written interleaved in blocks of 32
// channels (gate block, up block, ...) for the GEMM with SwiGLU in its epilogue (N a multiple of 32, groups <= 512);
// 3 = the 32-row blocks of every 128-row head written in the order [0, 2, 1, 3] for the GEMM with the rotary embedding
// in its epilogue (N a multiple of 128)

// ---- frozen weights (lightweight variant): packed 4-bit codes, binary16 steps, int16 zero points ----
// group: a power of two in 8 .. 512 that divides K
bool zo_int4_group_supported(int32_t K, int32_t group);
hipError_t zo_launch_pack_int4(const float* W, int32_t N, int32_t K, int32_t group, void* packed, void* step_f16, int16_t* zp,
                               hipStream_t st);
// w^ = (code - zp) * step into out0 (and out1 if not NULL), storage type dtype
hipError_t zo_launch_dequant_int4(const void* packed, const void* step_f16, const int16_t* zp, int32_t N, int32_t K, int32_t group,
                                  int dtype, void* out0, void* out1, hipStream_t st, int ilv = 0);

// ---- per-token activation fake-quantizer -------------------------------------------------------
// sm_delta / sm_inv (fp32 [K], or both NULL): the quantizer sees (x - delta) * inv (Eq. 4)
hipError_t zo_launch_fq_act(const void* X, void* Xhat, int32_t M, int32_t K, int32_t bits, int32_t sym, int dtype,
                            int16_t* codes, float* step, int32_t* zp, const float* sm_delta, const float* sm_inv, hipStream_t st);

// ---- adaptive weight quantizer (Eq. 5) / smoothing (Eq. 4) -------------------------------------
// per-group parameters [N][K/group] and the optional per-feature scale [K], all fp32, already perturbed
struct zo_learned { const float* step; const float* zp; const float* alpha; const float* beta; const float* scale; };
hipError_t zo_launch_fq_weight_learned(const float* W, int32_t N, int32_t K, int32_t bits, int32_t group, uint64_t seed, int32_t tid,
                                       float eps, int dtype, const zo_learned& pp, const zo_learned& pm, void* out_plus, void* out_minus,
                                       uint8_t* codes, hipStream_t st, int ilv = 0);
// initial parameters from the dynamic scheme on W; zp_scratch: int32 [N][K/group]
hipError_t zo_launch_init_learned(const float* W, int32_t N, int32_t K, int32_t bits, int32_t group, float* step, float* zp,
                                  float* alpha, float* beta, int32_t* zp_scratch, hipStream_t st);
hipError_t zo_launch_fill(float* out, int64_t n, float value, hipStream_t st);
hipError_t zo_launch_reciprocal(const float* in, float* out, int64_t n, hipStream_t st);
// out[n] = bias[n] + sum_k delta[k] * (w[n][k] +- eps u); the minus outputs may be NULL
hipError_t zo_launch_bias_shift(const float* W, int32_t N, int32_t K, uint64_t seed, int32_t tid, float eps,
                                const float* delta_p, const float* delta_m, const float* bias_p, const float* bias_m,
                                float* out_p, float* out_m, hipStream_t st);

// ---- GEMM: Y[b] = X[b] * W[b]^T (+bias[b]) (relu) (+residual[b]); batch over branches -----------
struct zo_gemm_args {
    const void* X; const void* W; void* Y;
    const float* bias;          // [N] fp32 or NULL
    const void* residual;       // [M][N] storage type or NULL
    int32_t M, N, K;
    int32_t batch;              // 1 or 2
    int64_t strideX, strideW, strideY, strideBias, strideRes;   // elements between batch entries
    int32_t relu;
    int32_t out_f32;            // 1: Y is fp32 whatever the operand type
    int dtype;                  // operand (and default output) storage type
    int32_t swiglu;             // 1: W holds gate and up rows interleaved in blocks of 32 channels; Y[M][N/2] = silu(gate) * up
                                //    (bf16, large shapes only: zo_gemm_swiglu_supported; no bias / residual / relu)
    // rotary embedding in the epilogue of the fused q | k | v GEMM (head dimension 128; rope_cos != NULL switches it on): W rows
    // with the 32-row blocks of every head in the order [0, 2, 1, 3]; columns < rope_cols rotated, position = row % rope_S
    const float* rope_cos; const float* rope_sin;   // fp32 [max_seq][64]
    int32_t rope_cols, rope_S;
    // cross entropy in the epilogue of the lm_head GEMM (ce_part != NULL switches it on; Y is not written): per row and
    // 256-column tile the maximum logit and the sum of exp(logit - maximum) go to ce_part[m][tiles_n][2]; the logit of
    // the row's target ce_ids[m + 1] (clamped to the vocabulary; no target at positions m % ce_S == ce_S - 1) to ce_tgt[m]
    float* ce_part; float* ce_tgt;
    const int32_t* ce_ids;      // shared by the batch entries
    int32_t ce_S;
    int64_t stridePart, strideTgt;   // floats between batch entries
    // K split of the 128 x 128-tile form (shapes that leave most CUs without a workgroup): ks_part = NULL, or fp32 scratch of
    // ks_part_bytes >= zo_gemm_splitk_bytes(M, N, K, batch); the launcher then gives every K range a workgroup of its own,
    // which writes its partial sums there, and a second kernel adds the ranges in order and applies the epilogue
    float* ks_part; size_t ks_part_bytes;
    int32_t kspl;               // set by the launcher: K ranges of this launch (0 / 1: none)
};
int zo_gemm_splitk(int32_t M, int32_t N, int32_t K, int32_t batch, int dtype);            // K ranges the launcher would use (1: no split)
size_t zo_gemm_splitk_bytes(int32_t M, int32_t N, int32_t K, int32_t batch, int dtype);   // scratch for them (0: no split)
bool zo_gemm_ce_supported(int32_t M, int32_t N, int32_t K, int dtype);
size_t zo_gemm_ce_part_floats(int32_t M, int32_t N);     // floats of ce_part for one batch entry
// row_loss[m] = log sum exp(logits[m][:]) - logits[m][target], from the partial results above; 0 at the last position
hipError_t zo_launch_ce_combine(const float* part, const float* tgt, float* row_loss, int32_t M, int32_t S, int32_t N, hipStream_t st);
bool zo_gemm_rope_supported(int32_t M, int32_t N, int32_t K, int dtype);
bool zo_gemm_swiglu_supported(int32_t M, int32_t N, int32_t K, int dtype);
hipError_t zo_launch_gemm(const zo_gemm_args& a, hipStream_t st);

// ---- fused fake-quantized linear for small M: Y[b] = X[b] * Q(W +- eps u)^T, tiles built in registers ----
#define ZO_FUSED_MAX_M 128
struct zo_fused_args {
    const void* X;              // bf16 [nb][M][K] (strideX elements between the branches, may be 0)
    const void* Xfrag;          // NULL, or the same activations re-laid out by zo_launch_fused_relayout (same bits / group)
    int64_t strideXfrag;
    const void* codes;          // frozen linear (zo_launch_int4_gemm_fused): 4-bit codes [N][K/2], binary16 steps and
    const void* step16;         // int16 zero points [N][K/group]
    const int16_t* zp;
    const void* W;              // master [N][K] of ONE tensor (element index = n*K + k in its stream), fp32 or binary16
    int32_t wdtype;             // ZO_W_*
    void* Y;                    // bf16 or fp32 [M][ldY], already offset to the tensor's first output column
    const float* bias;          // fp32 [N] (per branch: strideBias) or NULL
    const void* residual;       // bf16, same indexing as Y, or NULL
    int32_t M, N, K, nb;        // nb = 1: eps is signed; nb = 2: branch 0 at +eps, branch 1 at -eps
    int64_t strideX, strideY, strideBias, strideRes, ldY;
    int32_t bits, group;        // bits = 0: perturbed, not quantized; group in {8, 16, 32, 64, 128}
    float eps;
    int32_t relu, out_f32;
};
// M in 1..ZO_FUSED_MAX_M, N a multiple of 16, K a multiple of 32 and of the group
bool zo_fused_supported(int32_t M, int32_t N, int32_t K, int32_t bits, int32_t group);
hipError_t zo_launch_fq_gemm_fused(const zo_fused_args& a, uint64_t seed, int32_t tid, hipStream_t st);
// Two tensors of the same shape and settings (say the query and value projections) in one launch, so that their workgroups
// share the rounds over the CUs: `second` replaces W, Y, bias and residual of `a` for the second tensor (stream tid2).
struct zo_fused_second { const void* W; void* Y; const float* bias; const void* residual; int32_t tid; };
hipError_t zo_launch_fq_gemm_fused_pair(const zo_fused_args& a, const zo_fused_second& second, uint64_t seed, int32_t tid, hipStream_t st);
// Frozen, pre-quantized linear at small M: the operand is expanded from the packed codes in registers (a.codes /
// step16 / zp / group; W, bits, eps, seed unused).  group in {32, 64, 128, 256, 512}.  The fragment-ordered copy
// of the activations is laid out as for bits = 4 and the same group capped at 128.
bool zo_int4_fused_supported(int32_t M, int32_t N, int32_t K, int32_t group);
hipError_t zo_launch_int4_gemm_fused(const zo_fused_args& a, hipStream_t st);
// Split-K form (128 channels per workgroup, activations shared through LDS, partial sums reduced in a fixed order by
// a second kernel): needs zo_int4_splitk_scratch_bytes of fp32 scratch.  Same results up to the order of the fp32 sums.
size_t zo_int4_splitk_scratch_bytes(int32_t M, int32_t N, int32_t K, int32_t group);
hipError_t zo_launch_int4_gemm_splitk(const zo_fused_args& a, void* partials, hipStream_t st);
// Optional: activations in the order the fused kernel consumes them (contiguous wave-level loads instead of
// 16-byte gathers; pays from a few m-tiles on).  out: zo_fused_relayout_bytes(M, K) bytes per branch.
size_t zo_fused_relayout_bytes(int32_t M, int32_t K);
hipError_t zo_launch_fused_relayout(const void* X, int64_t strideX, int32_t M, int32_t K, int32_t nb, int32_t bits, int32_t group,
                                    void* out, int64_t strideOut, hipStream_t st);

// ---- the rest of the decoder forward -----------------------------------------------------------
// x[t] = rt(fma(eps, u(tok row), tok_emb[id]) (+ fma(eps, u(pos row), pos_emb[t % S])))
hipError_t zo_launch_embed(const int32_t* ids, const void* tok_emb, const void* pos_emb, void* out,
                           int32_t M, int32_t S, int32_t d, int32_t vocab, uint64_t seed, int32_t tid_tok, int32_t tid_pos,
                           float eps_tok, float eps_pos, int dtype, hipStream_t st, int wdtype = ZO_W_F32);
// RMSNorm (beta = NULL) or LayerNorm; gamma/beta are already perturbed fp32 vectors
hipError_t zo_launch_norm(const void* x, const float* gamma, const float* beta, void* out,
                          int32_t M, int32_t d, float eps, int dtype, hipStream_t st);
// norm fused with the per-token quantizer (row kept in registers): d <= 8192
bool zo_norm_quant_supported(int32_t d);
hipError_t zo_launch_norm_quant(const void* x, const float* gamma, const float* beta, void* xhat, int32_t M, int32_t d,
                                float eps, int32_t bits, int32_t sym, int dtype,
                                const float* sm_delta, const float* sm_inv, hipStream_t st,
                                int8_t* codes = nullptr, float* xs = nullptr, float* xo = nullptr);   // codes != NULL: integer route
// SwiGLU fused with the per-token quantizer: cols <= 16384; up = NULL: the quantizer alone on the rows of `gate`
bool zo_swiglu_quant_supported(int32_t cols);
hipError_t zo_launch_swiglu_quant(const void* gate, const void* up, void* xhat, int64_t rows, int32_t cols, int64_t in_stride,
                                  int32_t bits, int32_t sym, int dtype, const float* sm_delta, const float* sm_inv, hipStream_t st,
                                  int8_t* codes = nullptr, float* xs = nullptr, float* xo = nullptr);   // codes != NULL: integer route
hipError_t zo_launch_rope(void* q, void* k, const float* cos_tab, const float* sin_tab,
                          int32_t M, int32_t S, int32_t H, int32_t dh, int64_t row_stride, int dtype, hipStream_t st);
hipError_t zo_launch_attention(const void* q, const void* k, const void* v, void* out,
                               int32_t B, int32_t S, int32_t H, int32_t dh, int64_t row_stride, int dtype, hipStream_t st);
// bf16, head dimension 64 / 128: matrix-core kernel
bool zo_flash_attention_supported(int32_t dh, int dtype);
hipError_t zo_launch_flash_attention(const void* q, const void* k, const void* v, void* out,
                                     int32_t B, int32_t S, int32_t H, int32_t dh, int64_t row_stride, hipStream_t st);
hipError_t zo_launch_swiglu(const void* gate, const void* up, void* out, int64_t rows, int32_t cols,
                            int64_t in_stride, int dtype, hipStream_t st);
// row_loss[t] = logsumexp(logits[t]) - logits[t][ids[t+1]] (0 for the last position of a sequence)
hipError_t zo_launch_ce_rows(const float* logits, const int32_t* ids, float* row_loss,
                             int32_t M, int32_t S, int32_t V, hipStream_t st);
hipError_t zo_launch_sqerr_rows(const void* y, const float* target, float* row_loss, int32_t M, int32_t N, int dtype, hipStream_t st);
// loss = sum(row_loss) * scale, fixed summation order
hipError_t zo_launch_reduce_loss(const float* row_loss, int32_t M, float scale, float* loss, hipStream_t st);
// out6 = { L+, L-, g, lr[0]*g, lr[1]*g, lr[2]*g } from loss[0], loss[1]; the first n_user values also go to user_out
hipError_t zo_launch_projected_grad(const float* loss2, float eps, const float lr[3], float* out6, float* user_out, int n_user,
                                    hipStream_t st);

// ---- quantized linear on the integer codes (int8 matrix instructions) ----------------------------
// y = step_x (sum_g step_w S_g + (O - zx) r): see zo_i8.hip.  w_group 64, 128, 256, 512 or 0 / K (per channel), K a multiple of 128.
bool zo_i8_supported(int32_t M, int32_t N, int32_t K, int32_t w_bits, int32_t w_group, int32_t a_bits);
size_t zo_i8_scale_floats(int32_t N, int32_t K, int32_t w_group);       // floats of one branch's array of weight steps
hipError_t zo_launch_act_codes_i8(const void* X, int8_t* codes, float* xs, float* xo, int32_t M, int32_t K, int32_t bits, int32_t sym,
                                  int dtype, hipStream_t st);
hipError_t zo_launch_weight_codes_i8(const void* W, int32_t N, int32_t K, int32_t bits, int32_t group, uint64_t seed, int32_t tid, float eps,
                                     int wdtype, int8_t* cp, int8_t* cm, float* wsp, float* wsm, float* rp, float* rm, float* rpart_p,
                                     float* rpart_m, int* overflow, hipStream_t st, int32_t scale_row_tiles = 0,
                                     int32_t ilv = 0);   // ilv: rows interleaved for a pairing epilogue (see zo_i8.hip)
// the forward's overflow flag: a set flag turns the nb losses into NaN and is cleared for the next forward
hipError_t zo_launch_i8_flag_to_loss(int* flag, float* loss, int32_t nb, hipStream_t st);
struct zo_i8_gemm_args {
    const int8_t* X; const int8_t* W;        // codes [M][K], [N][K]
    const float* xs; const float* xo;        // per token: step, O - zero point
    const float* ws;                         // [K / sgroup][tiles_n * 256] weight steps
    const float* wr;                         // [N]
    void* Y; const float* bias; const void* residual;
    int32_t M, N, K, batch, sgroup;          // sgroup: k per weight step (64, or a multiple of 128)
    int64_t strideX, strideW, strideXs, strideWs, strideWr, strideY, strideBias, strideRes;
    int32_t relu;
    int32_t epi;                             // 1: SwiGLU on rows written interleaved (zo_launch_weight_codes_i8's ilv 1 / 2); Y is [M][N / 2]
};
hipError_t zo_launch_gemm_i8(const zo_i8_gemm_args& a, int out_f32, hipStream_t st);

// ---- generator on the quantized model (prompt pass + cached decoding) ----------------------------
// out[h*dh + i] = sum_j softmax_j(q_h . K[j]_h / sqrt(dh)) V[j]_h[i] over the n cached rows (row pitch H*dh); fp32 math
hipError_t zo_launch_decode_attention(const void* q, const void* Kc, const void* Vc, void* out, int32_t n, int32_t H, int32_t dh,
                                      int dtype, hipStream_t st);
bool zo_decode_attention_split_supported(int32_t H, int32_t dh);
size_t zo_decode_attention_split_bytes(int32_t n, int32_t H, int32_t dh);
hipError_t zo_launch_decode_attention_split(const void* qkv, void* Kc, void* Vc, const float* cos_row, const float* sin_row, void* scratch,
                                            void* att, void* xhat, int32_t n, int32_t H, int32_t dh, int32_t bits, int32_t sym,
                                            const float* sm_delta, const float* sm_inv, int dtype, hipStream_t st);
hipError_t zo_launch_argmax(const float* logits, int32_t V, int32_t* token, hipStream_t st);
// frozen (packed 4-bit) linear of ONE token (M = 1, one branch): a.X bf16 [K], a.Y [N] (bf16, or fp32 with out_f32), 0.5 B per weight
bool zo_int4_gemv_supported(int32_t M, int32_t nb, int32_t N, int32_t K, int32_t group);
hipError_t zo_launch_int4_gemv(const zo_fused_args& a, hipStream_t st);
// the same for up to four tensors that read the same token (same X, K, group, epilogue flags) in one launch
hipError_t zo_launch_int4_gemv_multi(const zo_fused_args* t, int nt, hipStream_t st);

