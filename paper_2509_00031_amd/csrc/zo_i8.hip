// Quantized linear on the integer codes themselves (int8 matrix instructions of gfx950):
//
//   y[t][n] = step_x[t] * ( sum_g step_w[g][n] * S_g[t][n]  +  (O - zx[t]) * r[n] ),
//   S_g[t][n] = sum_{k in g} (qx[t][k] - O) (qw[n][k] - zw[g][n]),   r[n] = sum_g step_w[g][n] sum_{k in g} (qw[n][k] - zw[g][n]),
//
// which is x^ w^^T with x^ = (qx - zx) step_x and w^ = (qw - zw) step_w, the de-quantized operands of the uniform
// quantizer of the Background section, evaluated without rounding either operand: the inner sums are exact 32-bit
// integers, one fp32 multiply-add per weight group carries them into the fp32 result.  O = 2^(a_bits - 1) re-centres
// the activation codes of the asymmetric per-token quantizer (0 .. 2^a_bits - 1) into a signed byte; O = 0 for the
// symmetric one.  Weight operands are qw - zw as signed bytes; a group whose |qw - zw| exceeds 127 (a group lying far
// from zero compared with its own range) cannot be represented: the quantizer saturates it and raises a flag.
#include "zo_device.h"
#include "zo_internal.h"

typedef int i32x4 __attribute__((ext_vector_type(4)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

static inline zo_stream make_stream_i8(uint64_t seed, int32_t tid)
{
    zo_stream s;
    s.k0 = (uint32_t)seed;
    s.k1 = (uint32_t)(seed >> 32);
    s.tensor_id = (uint32_t)tid;
    return s;
}

// position of output channel n inside its 256-channel tile's row of scales: the GEMM's wave wn (64 channels) reads, per
// lane j = n % 16, the four values of its 16-channel blocks tn = (n % 64) / 16 as one 16-byte piece
__host__ __device__ static inline int scale_slot(int n)
{
    const int c = n & 255;
    return (c & ~63) + ((c & 15) << 2) + ((c >> 4) & 3);
}

// Output row of input row n when the rows of a matrix go out interleaved for the GEMM epilogue that pairs channels: ilv = 1 / 2:
// the gate / up rows of a SwiGLU pair in alternating blocks of 32 channels (gate block, up block of the same channels, ...).
// The GEMM's 16-channel tiles j and j + 2 of a wave then hold the two partners in the same lane and register.
__host__ __device__ static inline uint32_t ilv_row(uint32_t n, int ilv)
{
    if (ilv == 0) return n;
    return ((n >> 5) << 6) + (n & 31) + (ilv == 2 ? 32 : 0);
}

// ---------------------------------------------------------------------------------------------
// per-token activation quantizer -> signed-byte codes: one wavefront per row, two sweeps
// ---------------------------------------------------------------------------------------------
template <typename T>
__global__ __launch_bounds__(256) void zo_act_codes_i8_kernel(const T* __restrict__ X, int8_t* __restrict__ C, float* __restrict__ xs,
                                                              float* __restrict__ xo, int M, int K, int bits, int sym)
{
    const int lane = threadIdx.x & 63;
    const int row = blockIdx.x * 4 + (threadIdx.x >> 6);
    if (row >= M) return;
    const T* x = X + (int64_t)row * K;
    float mn = INFINITY, mx = -INFINITY;
    for (int c = lane * 8; c < K; c += 512) {
        float v[8];
        zo_load8(x + c, v);
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            if (sym) mx = fmaxf(mx, fabsf(v[i]));
            else { mn = fminf(mn, v[i]); mx = fmaxf(mx, v[i]); }
        }
    }
    mn = zo_group_min<64>(mn);
    mx = zo_group_max<64>(mx);
    const zo_qparams q = sym ? zo_qparams_sym(mx, bits) : zo_qparams_asym(mn, mx, bits);
    const float off = sym ? 0.0f : (float)(1 << (bits - 1));
    if (lane == 0) { xs[row] = q.step; xo[row] = off - q.zp; }
    for (int c = lane * 8; c < K; c += 512) {
        float v[8];
        zo_load8(x + c, v);
        uint32_t w[2] = {0u, 0u};
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            const int cd = (int)(zo_code(q, v[i]) - off);              // in [-128, 127] by construction
            w[i >> 2] |= ((uint32_t)cd & 0xFFu) << (8 * (i & 3));
        }
        *reinterpret_cast<uint2*>(C + (int64_t)row * K + c) = make_uint2(w[0], w[1]);
    }
}

hipError_t zo_launch_act_codes_i8(const void* X, int8_t* codes, float* xs, float* xo, int32_t M, int32_t K, int32_t bits, int32_t sym,
                                  int dtype, hipStream_t st)
{
    if (M == 0) return hipSuccess;
    if (bits < 2 || bits > 8 || (K & 7)) return hipErrorInvalidValue;
    const int grid = (M + 3) / 4;
    if (dtype == ZO_T_BF16) zo_act_codes_i8_kernel<zo_bf16><<<grid, 256, 0, st>>>((const zo_bf16*)X, codes, xs, xo, M, K, bits, sym);
    else zo_act_codes_i8_kernel<float><<<grid, 256, 0, st>>>((const float*)X, codes, xs, xo, M, K, bits, sym);
    return hipGetLastError();
}

// ---------------------------------------------------------------------------------------------
// weight quantizer -> signed-byte operands qw - zw of Q(W + eps u) and Q(W - eps u), the group steps in the layout the
// GEMM reads, and step * (sum of the group's operands) per group for r[n].  One thread = 8 consecutive k (one block of
// the perturbation stream), a group = GL neighbouring lanes; u is generated once for both branches.
// ---------------------------------------------------------------------------------------------
struct zo_i8_rowdiv { int32_t kb; uint32_t magic; int32_t shift; };
static zo_i8_rowdiv make_rowdiv_i8(int kb)
{
    int l = 0;
    while ((1u << l) < (unsigned)kb) ++l;
    const int sh = 31 + l;
    return zo_i8_rowdiv{kb, (uint32_t)((((uint64_t)1 << sh) + (uint64_t)kb - 1) / (uint64_t)kb), sh};
}

// (b: output position of the lane's 8 codes in blocks of 8; n: output row)
template <int GL>
__device__ __forceinline__ void weight_codes_branch(const float v[8], int bits, bool active, int lane, int64_t b, uint32_t n, uint32_t g,
                                                    int G, int tiles_n, int8_t* codes, float* ws, float* rpart, int* overflow)
{
    float mn = v[0], mx = v[0];
#pragma unroll
    for (int i = 1; i < 8; ++i) { mn = fminf(mn, v[i]); mx = fmaxf(mx, v[i]); }
    mn = zo_group_min<GL>(mn);
    mx = zo_group_max<GL>(mx);
    const zo_qparams q = zo_qparams_asym(mn, mx, bits);
    float sum = 0.0f;
    uint32_t w[2] = {0u, 0u};
    bool over = false;
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        float d = zo_code(q, v[i]) - q.zp;                              // integer valued
        over = over || d > 127.0f || d < -128.0f;
        d = __builtin_amdgcn_fmed3f(d, -128.0f, 127.0f);
        sum += d;                                                       // exact: |sum| < 2^24
        w[i >> 2] |= ((uint32_t)(int)d & 0xFFu) << (8 * (i & 3));
    }
    sum = zo_group_sum<GL>(sum);
    if (!active) return;
    *reinterpret_cast<uint2*>(codes + 8 * b) = make_uint2(w[0], w[1]);
    if (over) atomicOr(overflow, 1);
    if ((lane & (GL - 1)) == 0) {
        ws[((int64_t)g * tiles_n + (n >> 8)) * 256 + scale_slot((int)n)] = q.step;
        rpart[(int64_t)n * G + g] = q.step * sum;
    }
}

template <typename TW, int GL>
__global__ __launch_bounds__(256) void zo_weight_codes_i8_kernel(const TW* __restrict__ W, int64_t nblk, zo_stream s, float eps, int bits,
                                                                 int8_t* cp, int8_t* cm, float* wsp, float* wsm, float* rp, float* rm,
                                                                 int* overflow, zo_i8_rowdiv kb, int tiles_n, int ilv)
{
    const int lane = threadIdx.x & 63;
    const int64_t b = (int64_t)blockIdx.x * 256 + threadIdx.x;
    const bool active = b < nblk;
    float w[8], z[8];
    if (active) {
        zo_load8(W + 8 * b, w);
        if (eps != 0.0f) zo_z8(s, (uint64_t)b, z);
    }
    if (!active || eps == 0.0f) {
#pragma unroll
        for (int i = 0; i < 8; ++i) { z[i] = 0.0f; if (!active) w[i] = 0.0f; }
    }
    const uint32_t n = (uint32_t)(((uint64_t)(uint32_t)b * kb.magic) >> kb.shift);
    const uint32_t kblk = (uint32_t)b - n * (uint32_t)kb.kb;
    const uint32_t g = kblk / GL;
    const int G = kb.kb / GL;
    const uint32_t no = ilv_row(n, ilv);                      // where the row goes
    const int64_t ob = (int64_t)no * kb.kb + kblk;
    {
        float v[8];
#pragma unroll
        for (int i = 0; i < 8; ++i) v[i] = __builtin_fmaf(eps, z[i], w[i]);
        weight_codes_branch<GL>(v, bits, active, lane, ob, no, g, G, tiles_n, cp, wsp, rp, overflow);
    }
    if (cm) {
        float v[8];
#pragma unroll
        for (int i = 0; i < 8; ++i) v[i] = __builtin_fmaf(-eps, z[i], w[i]);
        weight_codes_branch<GL>(v, bits, active, lane, ob, no, g, G, tiles_n, cm, wsm, rm, overflow);
    }
}

// r[n] = sum_g rpart[n][g], added in the order of g (one thread per channel of the matrix, at its output row; G is a few dozen)
__global__ __launch_bounds__(256) void zo_rowsum_kernel(const float* __restrict__ rpart, float* __restrict__ r, int N, int G, int ilv)
{
    const int n0 = blockIdx.x * 256 + threadIdx.x;
    if (n0 >= N) return;
    const int64_t n = ilv_row((uint32_t)n0, ilv);
    float acc = 0.0f;
    for (int g = 0; g < G; ++g) acc += rpart[n * G + g];
    r[n] = acc;
}

// Per-channel quantization (one group = one whole row of W, the weight setting of the W4A4 rows of the appendix's
// quantization settings): one workgroup per output channel, two sweeps over the row (range, then codes; the stream is
// generated again in the second sweep).  The channel's step goes to the same slot layout (a single row of steps) and
// r[n] = step * (sum of the row's operands) is written directly -- a sum of at most 65536 integers below 128 is exact in fp32.
// NB > 0: a thread's (at most NB) blocks of 8 weights and their perturbations stay in registers between the two sweeps
// (rows of up to 2048 NB weights), so the stream is generated once; NB = 0: any row length, stream generated in both sweeps.
template <typename TW, int NB>
__global__ __launch_bounds__(256) void zo_weight_codes_i8_row_kernel(const TW* __restrict__ W, int K, zo_stream s, float eps, int bits,
                                                                     int8_t* cp, int8_t* cm, float* wsp, float* wsm, float* rp, float* rm,
                                                                     int* overflow, int ilv)
{
    __shared__ float red[4][4];
    constexpr int HELD = NB > 0 ? NB : 1;
    const int n = blockIdx.x, nb = K / 8;
    const int no = (int)ilv_row((uint32_t)n, ilv);            // where the row goes
    const int64_t b0 = (int64_t)n * nb, ob0 = (int64_t)no * nb;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int sweeps = NB > 0 ? NB : (nb + 255) / 256;
    float wv[HELD][8], zv[HELD][8];
    auto fetch = [&](int j, float (&w)[8], float (&z)[8]) {
        zo_load8(W + 8 * (b0 + j), w);
        if (eps != 0.0f) zo_z8(s, (uint64_t)(b0 + j), z);
        else {
#pragma unroll
            for (int i = 0; i < 8; ++i) z[i] = 0.0f;
        }
    };
    float mnp = INFINITY, mxp = -INFINITY, mnm = INFINITY, mxm = -INFINITY;
#pragma unroll
    for (int u = 0; u < sweeps; ++u) {
        const int j = threadIdx.x + 256 * u;
        if (j < nb) {
            float wl[8], zl[8];
            float (&w)[8] = NB > 0 ? wv[NB > 0 ? u : 0] : wl;
            float (&z)[8] = NB > 0 ? zv[NB > 0 ? u : 0] : zl;
            fetch(j, w, z);
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                const float vp = __builtin_fmaf(eps, z[i], w[i]), vm = __builtin_fmaf(-eps, z[i], w[i]);
                mnp = fminf(mnp, vp); mxp = fmaxf(mxp, vp); mnm = fminf(mnm, vm); mxm = fmaxf(mxm, vm);
            }
        }
    }
    mnp = zo_group_min<64>(mnp); mxp = zo_group_max<64>(mxp);
    mnm = zo_group_min<64>(mnm); mxm = zo_group_max<64>(mxm);
    if (lane == 0) { red[wave][0] = mnp; red[wave][1] = mxp; red[wave][2] = mnm; red[wave][3] = mxm; }
    __syncthreads();
    mnp = fminf(fminf(red[0][0], red[1][0]), fminf(red[2][0], red[3][0]));
    mxp = fmaxf(fmaxf(red[0][1], red[1][1]), fmaxf(red[2][1], red[3][1]));
    mnm = fminf(fminf(red[0][2], red[1][2]), fminf(red[2][2], red[3][2]));
    mxm = fmaxf(fmaxf(red[0][3], red[1][3]), fmaxf(red[2][3], red[3][3]));
    __syncthreads();
    const zo_qparams qp = zo_qparams_asym(mnp, mxp, bits), qm = zo_qparams_asym(mnm, mxm, bits);
    float sump = 0.0f, summ = 0.0f;
    bool over = false;
#pragma unroll
    for (int u = 0; u < sweeps; ++u) {
        const int j = threadIdx.x + 256 * u;
        if (j < nb) {
            float wl[8], zl[8];
            float (&w)[8] = NB > 0 ? wv[NB > 0 ? u : 0] : wl;
            float (&z)[8] = NB > 0 ? zv[NB > 0 ? u : 0] : zl;
            if (NB == 0) fetch(j, w, z);
            uint32_t up[2] = {0u, 0u}, um[2] = {0u, 0u};
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                float d = zo_code(qp, __builtin_fmaf(eps, z[i], w[i])) - qp.zp;          // integer valued
                over = over || d > 127.0f || d < -128.0f;
                d = __builtin_amdgcn_fmed3f(d, -128.0f, 127.0f);
                sump += d;
                up[i >> 2] |= ((uint32_t)(int)d & 0xFFu) << (8 * (i & 3));
                if (cm) {
                    float dm = zo_code(qm, __builtin_fmaf(-eps, z[i], w[i])) - qm.zp;
                    over = over || dm > 127.0f || dm < -128.0f;
                    dm = __builtin_amdgcn_fmed3f(dm, -128.0f, 127.0f);
                    summ += dm;
                    um[i >> 2] |= ((uint32_t)(int)dm & 0xFFu) << (8 * (i & 3));
                }
            }
            *reinterpret_cast<uint2*>(cp + 8 * (ob0 + j)) = make_uint2(up[0], up[1]);
            if (cm) *reinterpret_cast<uint2*>(cm + 8 * (ob0 + j)) = make_uint2(um[0], um[1]);
        }
    }
    if (over) atomicOr(overflow, 1);
    sump = zo_group_sum<64>(sump);
    summ = zo_group_sum<64>(summ);
    if (lane == 0) { red[wave][0] = sump; red[wave][1] = summ; }
    __syncthreads();
    if (threadIdx.x == 0) {
        const int slot = (no >> 8) * 256 + scale_slot(no);
        wsp[slot] = qp.step;
        rp[no] = qp.step * (((red[0][0] + red[1][0]) + red[2][0]) + red[3][0]);
        if (cm) {
            wsm[slot] = qm.step;
            rm[no] = qm.step * (((red[0][1] + red[1][1]) + red[2][1]) + red[3][1]);
        }
    }
}

template <typename TW>
static hipError_t launch_weight_codes_row_t(const TW* W, int32_t N, int32_t K, int32_t bits, zo_stream s, float eps, int8_t* cp, int8_t* cm,
                                            float* wsp, float* wsm, float* rp, float* rm, int* overflow, hipStream_t st, int ilv)
{
#define ZO_ROWQ(NB) zo_weight_codes_i8_row_kernel<TW, NB><<<N, 256, 0, st>>>(W, K, s, eps, bits, cp, cm, wsp, wsm, rp, rm, overflow, ilv)
    if (K <= 4096) ZO_ROWQ(2); else if (K <= 8192) ZO_ROWQ(4); else if (K <= 12288) ZO_ROWQ(6); else if (K <= 16384) ZO_ROWQ(8); else ZO_ROWQ(0);
#undef ZO_ROWQ
    return hipGetLastError();
}

bool zo_i8_supported(int32_t M, int32_t N, int32_t K, int32_t w_bits, int32_t w_group, int32_t a_bits)
{
    if (M < 1 || N < 1 || K < 128 || (K & 127)) return false;
    if (w_bits < 1 || w_bits > 7 || a_bits < 2 || a_bits > 8) return false;        // 8-bit weight codes minus their zero point span 9 bits
    if (w_group == 0 || w_group == K) return K <= 65536;                            // per channel: integer sums over K stay below 2^31
    if (w_group != 64 && w_group != 128 && w_group != 256 && w_group != 512) return false;   // a step per 64 k, or per whole K tiles;
    if (K % w_group) return false;                                                           // at most 64 lanes per group in the quantizer
    return true;
}
size_t zo_i8_scale_floats(int32_t N, int32_t K, int32_t w_group)
{
    if (w_group == 0) w_group = K;
    return (size_t)(K / w_group) * (size_t)((N + 255) / 256) * 256;
}

template <typename TW>
static hipError_t launch_weight_codes_t(const TW* W, int32_t N, int32_t K, int32_t bits, int32_t group, zo_stream s, float eps, int8_t* cp,
                                        int8_t* cm, float* wsp, float* wsm, float* rpp, float* rpm, int* overflow, hipStream_t st,
                                        int scale_row_tiles, int ilv)
{
    const int kb = K / 8;
    const int64_t nblk = (int64_t)N * kb;
    if (nblk == 0) return hipSuccess;
    if (nblk >= ((int64_t)1 << 31)) return hipErrorInvalidValue;
    const int grid = (int)((nblk + 255) / 256);
    const zo_i8_rowdiv rd = make_rowdiv_i8(kb);
    // 256-channel tiles per row of steps: this matrix alone, or the fused operand it is a row block of (then wsp / wsm point at
    // the block's first tile inside the row of steps of group 0)
    const int tiles_n = scale_row_tiles > 0 ? scale_row_tiles : (N + 255) / 256;
    switch (group / 8) {
        case 8:  zo_weight_codes_i8_kernel<TW, 8><<<grid, 256, 0, st>>>(W, nblk, s, eps, bits, cp, cm, wsp, wsm, rpp, rpm, overflow, rd, tiles_n, ilv); break;
        case 16: zo_weight_codes_i8_kernel<TW, 16><<<grid, 256, 0, st>>>(W, nblk, s, eps, bits, cp, cm, wsp, wsm, rpp, rpm, overflow, rd, tiles_n, ilv); break;
        case 32: zo_weight_codes_i8_kernel<TW, 32><<<grid, 256, 0, st>>>(W, nblk, s, eps, bits, cp, cm, wsp, wsm, rpp, rpm, overflow, rd, tiles_n, ilv); break;
        case 64: zo_weight_codes_i8_kernel<TW, 64><<<grid, 256, 0, st>>>(W, nblk, s, eps, bits, cp, cm, wsp, wsm, rpp, rpm, overflow, rd, tiles_n, ilv); break;
        default: return hipErrorInvalidValue;
    }
    return hipGetLastError();
}

// codes / ws / r of the '+' branch (eps as given) and, if cm != NULL, of the '-' branch.  rpart: fp32 scratch [N][K / group]
// per branch.  *overflow (device int) is OR-ed with 1 if some |qw - zw| did not fit a signed byte.
hipError_t zo_launch_weight_codes_i8(const void* W, int32_t N, int32_t K, int32_t bits, int32_t group, uint64_t seed, int32_t tid, float eps,
                                     int wdtype, int8_t* cp, int8_t* cm, float* wsp, float* wsm, float* rp, float* rm, float* rpart_p,
                                     float* rpart_m, int* overflow, hipStream_t st, int32_t scale_row_tiles, int32_t ilv)
{
    if (ilv < 0 || ilv > 2 || (ilv != 0 && (N & 31))) return hipErrorInvalidValue;
    if (group == 0) group = K;
    const zo_stream s = make_stream_i8(seed, tid);
    if (group == K) {                                                               // per channel
        if (N == 0) return hipSuccess;
        if (wdtype == ZO_W_F16)
            return launch_weight_codes_row_t<zo_f16>((const zo_f16*)W, N, K, bits, s, eps, cp, cm, wsp, wsm, rp, rm, overflow, st, ilv);
        return launch_weight_codes_row_t<float>((const float*)W, N, K, bits, s, eps, cp, cm, wsp, wsm, rp, rm, overflow, st, ilv);
    }
    hipError_t e = wdtype == ZO_W_F16
        ? launch_weight_codes_t<zo_f16>((const zo_f16*)W, N, K, bits, group, s, eps, cp, cm, wsp, wsm, rpart_p, rpart_m, overflow, st, scale_row_tiles, ilv)
        : launch_weight_codes_t<float>((const float*)W, N, K, bits, group, s, eps, cp, cm, wsp, wsm, rpart_p, rpart_m, overflow, st, scale_row_tiles, ilv);
    if (e != hipSuccess) return e;
    const int G = K / group;
    zo_rowsum_kernel<<<(N + 255) / 256, 256, 0, st>>>(rpart_p, rp, N, G, ilv);
    if (cm) zo_rowsum_kernel<<<(N + 255) / 256, 256, 0, st>>>(rpart_m, rm, N, G, ilv);
    return hipGetLastError();
}

__global__ void zo_i8_flag_to_loss_kernel(int* flag, float* loss, int nb)
{
    if (threadIdx.x == 0 && blockIdx.x == 0 && *flag) {
        for (int b = 0; b < nb; ++b) loss[b] = __builtin_nanf("");
        *flag = 0;
    }
}
hipError_t zo_launch_i8_flag_to_loss(int* flag, float* loss, int32_t nb, hipStream_t st)
{
    zo_i8_flag_to_loss_kernel<<<1, 64, 0, st>>>(flag, loss, nb);
    return hipGetLastError();
}

// ---------------------------------------------------------------------------------------------
// GEMM on the codes.  256 x 256 block tile, 8 waves as 2 (m) x 4 (n), wave tile 128 x 64 = 8 x 4 tiles of
// v_mfma_i32_16x16x64_i8 (one 64-wide slice of K per instruction), K tile = 128 codes = 128 bytes per row.  Operand
// tiles and the tile's rows of weight steps are copied global -> LDS by the load unit (16 bytes per lane), two stages.
// X is the first operand, W the second: a lane holds 4 consecutive m of ONE channel n per 16 x 16 tile, so the step of
// its channel is one register: per 64 k and output,  acc = fma((float)S, step, acc)  -- a conversion and a multiply-add in
// the vector unit next to 64 multiply-adds in the matrix unit.  The integer tile of slice s + 1 is issued before the
// rescale of slice s, so the two units overlap.
// ---------------------------------------------------------------------------------------------
__device__ __forceinline__ uint32_t lds_offset_i8(const void* p)
{
    return (uint32_t)(uintptr_t)(__attribute__((address_space(3))) const void*)p;
}
__device__ __forceinline__ void lds_dma16_i8(const void* base, uint32_t voff, uint32_t dst)
{
    asm volatile("s_mov_b32 m0, %0\n\tglobal_load_lds_dwordx4 %1, %2\n" ::"s"(dst), "v"(voff), "s"(base) : "memory");
}
template <int N> __device__ __forceinline__ void wait_vmcnt_i8()
{
    __builtin_amdgcn_s_waitcnt(0x0F70 | (N & 15) | ((N >> 4) << 14));
}
__device__ __forceinline__ int swz128(int row) { return (row ^ (row >> 3)) & 7; }


template <typename TY, int SPT, int EPI>
__global__ __launch_bounds__(512) void zo_gemm_i8_kernel(zo_i8_gemm_args a)
{
    constexpr int BM = 256, BN = 256, BKB = 128;      // K tile in bytes (= codes)
    constexpr int OPER = (BM + BN) * BKB;             // 64 KB of operands per stage
    constexpr int STAGE = OPER + 8 * 1024;            // + one 1 KB row of steps per wave (SPT distinct ones are used)
    constexpr int DPW = 9;                            // copies per wave and stage: 8 operand row-blocks + 1 row of steps
    constexpr int TM = 8, TN = 4;
    extern __shared__ __attribute__((aligned(16))) unsigned char lds[];
    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm = wave >> 2, wn = wave & 3;
    const int M = a.M, N = a.N, K = a.K, bz = blockIdx.z;
    const int tiles_m = (M + BM - 1) / BM, tiles_n = (N + BN - 1) / BN;
    int vid = blockIdx.x;
    const int nblk = gridDim.x;
    if ((nblk & 7) == 0) vid = (vid & 7) * (nblk >> 3) + (vid >> 3);     // one contiguous range of tiles per XCD
    const int group_sz = 8 * tiles_n;
    const int grp = vid / group_sz;
    const int first_m = grp * 8;
    const int gm = (tiles_m - first_m) < 8 ? (tiles_m - first_m) : 8;
    const int tile_m = first_m + (vid % group_sz) % gm;
    const int tile_n = (vid % group_sz) / gm;
    const int m0 = tile_m * BM, n0 = tile_n * BN;
    const int8_t* X = a.X + bz * a.strideX;
    const int8_t* W = a.W + bz * a.strideW;
    const float* ws = a.ws + bz * a.strideWs + (int64_t)tile_n * 256;
    const int ws_row = tiles_n * 256;                 // floats between two groups' rows of steps
    const int tpr = SPT == 2 ? 1 : a.sgroup / 128;    // K tiles per row of steps

    // copy plan: wave w copies row-blocks (8 rows of 128 B) w*8 .. w*8+7 of the 64 (X rows first, then W rows)
    const int lrow = lane >> 3, slot = lane & 7;
    uint32_t voff[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        const int rb = wave * 8 + i;
        const bool isw = rb >= 32;
        const int trow = (isw ? rb - 32 : rb) * 8 + lrow;
        int grow = (isw ? n0 : m0) + trow;
        const int lim = isw ? N : M;
        grow = grow < lim ? grow : lim - 1;
        const int c = slot ^ swz128(trow);
        voff[i] = (uint32_t)((int64_t)grow * K + c * 16);
    }
    const uint32_t lds0 = __builtin_amdgcn_readfirstlane(lds_offset_i8(lds));
    auto issue = [&](int stage, int kt) {
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            const int rb = wave * 8 + i;
            lds_dma16_i8(rb >= 32 ? (const void*)(W + kt * BKB) : (const void*)(X + kt * BKB), voff[i], lds0 + stage * STAGE + rb * 1024);
        }
        if constexpr (SPT != 0) {
            // the steps of slice (wave % SPT) of this K tile, into this wave's own 1 KB slot (waves >= SPT duplicate)
            const int row = __builtin_amdgcn_readfirstlane(SPT == 2 ? kt * 2 + (wave & 1) : kt / tpr);
            lds_dma16_i8((const void*)(ws + (size_t)(uint32_t)(row * ws_row)), (uint32_t)(lane * 16), lds0 + stage * STAGE + OPER + wave * 1024);
        }
    };

    f32x4 acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j) acc[i][j] = f32x4{0.0f, 0.0f, 0.0f, 0.0f};

    // Fragment addresses.  Lane (j16 = lane % 16, q4 = lane / 16) reads row base + 16 i + j16, 16-byte chunk 4 ks + q4,
    // stored at chunk slot (4 ks + q4) ^ swz(row).  With row = 16 (...) + j16:  swz(row) = (j16 & 7) ^ (j16 >> 3) ^ (2 i & 7),
    // so the slot is a lane constant XOR one of four values per ks -- eight byte offsets per operand in all, the row
    // block 16 i being an immediate offset of the read.
    const int j16 = lane & 15, q4 = lane >> 4;
    const int lane_slot = q4 ^ (j16 & 7) ^ (j16 >> 3);
    // row base | lane's slot bits: the slot of (ks, i) is the lane constant XOR (4 ks ^ 2 (i & 3)), bits 4..6 of the address
    const uint32_t xlane = (uint32_t)((wm * 128 + j16) * BKB) | ((uint32_t)lane_slot << 4);
    const uint32_t wlane = (uint32_t)(BM * BKB + (wn * 64 + j16) * BKB) | ((uint32_t)lane_slot << 4);
    auto xaddr = [&](uint32_t stage_off, int ks, int i) { return (xlane ^ (uint32_t)(((4 * ks) ^ (2 * (i & 3))) << 4)) + stage_off; };
    auto waddr = [&](uint32_t stage_off, int ks, int j) { return (wlane ^ (uint32_t)(((4 * ks) ^ (2 * (j & 3))) << 4)) + stage_off; };
    const uint32_t soff = (uint32_t)(OPER + (wn * 16 + j16) * 16);

    const int nk = K / BKB;
    // Pipeline.  All fragments are single-buffered and refilled IN PLACE as they die: within a 64-wide slice the 32 tiles
    // run channel block by channel block (j outer, i inner), so wf[j] is dead after its eighth tile and xf[i] after tile
    // (i, 3); the read of the next slice's fragment is issued right behind the matrix instruction that used the old one
    // last, a whole block of tiles before it is needed.  The next slice of the LAST slice of a K tile lies in the other
    // stage: the workgroup synchronises once per K tile, behind the first channel block of that slice -- the next K
    // tile has landed for everybody, nobody reads the current stage any more -- and the copies of K tile kt + 2 into the
    // freed stage are issued there.  The integer tile of (idx + 1) is always issued before the rescale of tile idx, across
    // slices and K tiles, so the matrix unit and the vector unit never wait for each other.
    issue(0, 0);
    wait_vmcnt_i8<0>();
    __syncthreads();
    if (nk > 1) issue(1, 1);
    i32x4 xf[TM], wf[TN];
    f32x4 sc, sc_next;
    {
        const unsigned char* sb0 = lds;
#pragma unroll
        for (int j = 0; j < TN; ++j) wf[j] = *reinterpret_cast<const i32x4*>(lds + waddr(0, 0, j) + j * 16 * BKB);
#pragma unroll
        for (int i = 0; i < TM; ++i) xf[i] = *reinterpret_cast<const i32x4*>(lds + xaddr(0, 0, i) + i * 16 * BKB);
        sc = *reinterpret_cast<const f32x4*>(sb0 + soff);
        sc_next = sc;
    }
    const i32x4 zero = {0, 0, 0, 0};
    if constexpr (SPT == 0) {
        // One step per channel for the whole of K: the 32 integer tiles stay in the matrix unit's accumulators over all K
        // tiles (|sum| <= 128 * 128 * K < 2^31) and meet their step once, behind the loop -- nothing for the vector unit inside
        // it.  Fragments are refilled in place as they die (wf[j] behind tile (7, j), xf[i] behind tile (i, 3)); the workgroup
        // synchronises behind the first channel block of a K tile's second slice, as in the grouped form below.
        i32x4 iacc[TM][TN];
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int j = 0; j < TN; ++j) iacc[i][j] = zero;
        for (int kt = 0; kt < nk; ++kt) {
            const int cur = kt & 1;
#pragma unroll
            for (int ks = 0; ks < 2; ++ks) {
                const int nstage = ks == 0 ? cur : cur ^ 1, nks = ks ^ 1;
                uint32_t nsb = (uint32_t)(nstage * STAGE);
                asm volatile("" : "+s"(nsb));
#pragma unroll
                for (int idx = 0; idx < TM * TN; ++idx) {
                    const int j = idx / TM, i = idx % TM;
                    __builtin_amdgcn_sched_barrier(0);
                    iacc[i][j] = __builtin_amdgcn_mfma_i32_16x16x64_i8(xf[i], wf[j], iacc[i][j], 0, 0, 0);
                    __builtin_amdgcn_sched_barrier(0);
                    if (ks == 1 && idx == TM - 1) {
                        wait_vmcnt_i8<0>();                       // own copies of K tile kt + 1 have landed
                        __builtin_amdgcn_s_waitcnt(0xC07F);       // lgkmcnt(0): own reads of this stage have returned
                        __syncthreads();
                        issue(cur, kt + 2 < nk ? kt + 2 : nk - 1);
                        __builtin_amdgcn_sched_barrier(0);
                    }
                    if (i == TM - 1) wf[j] = *reinterpret_cast<const i32x4*>(lds + waddr(nsb, nks, j) + j * 16 * BKB);
                    if (j == TN - 1) xf[i] = *reinterpret_cast<const i32x4*>(lds + xaddr(nsb, nks, i) + i * 16 * BKB);
                }
            }
        }
        float stp[TN];
#pragma unroll
        for (int j = 0; j < TN; ++j) stp[j] = ws[scale_slot(wn * 64 + j * 16 + j16)];
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int j = 0; j < TN; ++j)
#pragma unroll
                for (int r = 0; r < 4; ++r) acc[i][j][r] = (float)iacc[i][j][r] * stp[j];
    } else {
    i32x4 t = __builtin_amdgcn_mfma_i32_16x16x64_i8(xf[0], wf[0], zero, 0, 0, 0);
    for (int kt = 0; kt < nk; ++kt) {
        const int cur = kt & 1;
#pragma unroll
        for (int ks = 0; ks < 2; ++ks) {
            // where the next slice's fragments lie: same stage, slice 1 -- or the other stage, slice 0
            const int nstage = ks == 0 ? cur : cur ^ 1, nks = ks ^ 1;
            uint32_t nsb = (uint32_t)(nstage * STAGE);
            asm volatile("" : "+s"(nsb));                     // opaque: the addresses below are formed where they are used,
            const unsigned char* nb = lds + nsb;              // not kept in registers across the loop
#pragma unroll
            for (int idx = 0; idx < TM * TN; ++idx) {
                const int j = idx / TM, i = idx % TM;
                const int n1 = (idx + 1) % (TM * TN), j1 = n1 / TM, i1 = n1 % TM;
                __builtin_amdgcn_sched_barrier(0);
                const i32x4 nxt = __builtin_amdgcn_mfma_i32_16x16x64_i8(xf[i1], wf[j1], zero, 0, 0, 0);
                __builtin_amdgcn_sched_barrier(0);
                if (ks == 1 && idx == TM - 2) {
                    wait_vmcnt_i8<0>();                       // own copies of K tile kt + 1 have landed
                    __builtin_amdgcn_s_waitcnt(0xC07F);       // lgkmcnt(0): own reads of this stage have returned
                    __syncthreads();
                    issue(cur, kt + 2 < nk ? kt + 2 : nk - 1);   // past the end: the last tile again, into a stage nobody reads (no branch here)
                    __builtin_amdgcn_sched_barrier(0);
                }
                if (i1 == TM - 1 && idx != TM * TN - 1) {     // tile (7, j1) was wf[j1]'s last use
                    wf[j1] = *reinterpret_cast<const i32x4*>(lds + waddr(nsb, nks, j1) + j1 * 16 * BKB);
                    if (j1 == 0) sc_next = *reinterpret_cast<const f32x4*>(nb + soff + (SPT == 2 ? nks : 0) * 1024);
                }
                if (j1 == TN - 1 && idx != TM * TN - 1)       // tile (i1, 3) was xf[i1]'s last use
                    xf[i1] = *reinterpret_cast<const i32x4*>(lds + xaddr(nsb, nks, i1) + i1 * 16 * BKB);
                __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                for (int r = 0; r < 4; ++r) acc[i][j][r] = __builtin_fmaf((float)t[r], sc[j], acc[i][j][r]);
                t = nxt;
            }
            sc = sc_next;
        }
    }
    }
    wait_vmcnt_i8<0>();
    __syncthreads();

    // epilogue: y = xs[m] * (acc + xo[m] * r[n]) + bias -> relu -> + residual, one rounding; fp32 values go through this
    // wave's 16 KB slice of LDS (two passes of 32 channels: rows of 128 B, 16-byte granule g stored at
    // g ^ (4 * ((row >> 2) & 1))) and leave as row pieces
    TY* Y = (TY*)a.Y + bz * a.strideY;
    const float* bias = a.bias ? a.bias + bz * a.strideBias : nullptr;
    const TY* res = a.residual ? (const TY*)a.residual + bz * a.strideRes : nullptr;     // the residual has the output's type
    const float* xs = a.xs + bz * a.strideXs;
    const float* xo = a.xo + bz * a.strideXs;
    const float* wr = a.wr + bz * a.strideWr;
    unsigned char* slice = lds + wave * 16384;
    float rn[TN], bn[TN];
#pragma unroll
    for (int j = 0; j < TN; ++j) {
        int n = n0 + wn * 64 + j * 16 + j16;
        n = n < N ? n : N - 1;
        rn[j] = wr[n];
        bn[j] = bias ? bias[n] : 0.0f;
    }
    // Pairing epilogue (epi 1; the weight rows were written interleaved, see ilv_row): tiles j and j + 2 of a wave hold the gate
    // and the up value of one (token, channel) -> silu(gate) * up, both rounded to the output type first (as if they had been
    // stored), one pass, N / 2 output columns.  (The rotary embedding was tried the same way and dropped: its table reads in
    // accumulator layout and the register pressure next to 128 live accumulators cost 390 us per q | k | v launch, the
    // stand-alone kernel 73.)
    constexpr int epi = EPI;
    const int c0 = n0 + wn * 64;                       // first (interleaved) channel of the wave
    constexpr int npass = epi == 1 ? 1 : 2;
#pragma unroll
    for (int pass = 0; pass < npass; ++pass) {
#pragma unroll
        for (int i = 0; i < TM; ++i) {
            float sx[4], ox[4];
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                int m = m0 + wm * 128 + i * 16 + q4 * 4 + r;
                m = m < M ? m : M - 1;
                sx[r] = xs[m];
                ox[r] = xo[m];
            }
#pragma unroll
            for (int jj = 0; jj < 2; ++jj) {
                const int j = epi == 0 ? pass * 2 + jj : jj;
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    float v;
                    if (epi == 0) {
                        v = sx[r] * __builtin_fmaf(ox[r], pass == 0 ? rn[jj] : rn[jj + 2], pass == 0 ? acc[i][jj][r] : acc[i][jj + 2][r]) +
                            (pass == 0 ? bn[jj] : bn[jj + 2]);
                    } else {
                        const float lo = zo_round_to<TY>(sx[r] * __builtin_fmaf(ox[r], rn[j], acc[i][j][r]) + bn[j]);
                        const float hi = zo_round_to<TY>(sx[r] * __builtin_fmaf(ox[r], rn[j + 2], acc[i][j + 2][r]) + bn[j + 2]);
                        v = (lo / (1.0f + __expf(-lo))) * hi;
                    }
                    if (a.relu) v = fmaxf(v, 0.0f);
                    const int row = i * 16 + q4 * 4 + r;
                    const int gsl = (jj * 4 + (j16 >> 2)) ^ (((row >> 2) & 1) << 2);
                    *reinterpret_cast<float*>(slice + row * 128 + gsl * 16 + (j16 & 3) * 4) = v;
                }
            }
        }
#pragma unroll 4
        for (int it = 0; it < 16; ++it) {
            const int row = it * 8 + (lane >> 3), g = lane & 7;
            const f32x4 v4 = *reinterpret_cast<const f32x4*>(slice + row * 128 + ((g ^ (((row >> 2) & 1) << 2)) << 4));
            float v[4] = {v4[0], v4[1], v4[2], v4[3]};
            const int m = m0 + wm * 128 + row;
            // output column and row pitch: as computed; SwiGLU: half as many columns
            const int NO = epi == 1 ? N / 2 : N;
            const int n = epi == 0 ? c0 + pass * 32 + g * 4 : c0 / 2 + g * 4;
            if (m >= M || n >= NO) continue;
            const int64_t off = (int64_t)m * NO + n;
            if ((NO & 3) == 0) {
                if (res) {
                    if constexpr (sizeof(TY) == 4) {
                        const float4 r4 = *reinterpret_cast<const float4*>(res + off);
                        v[0] += r4.x; v[1] += r4.y; v[2] += r4.z; v[3] += r4.w;
                    } else {
                        const uint2 r2 = *reinterpret_cast<const uint2*>(res + off);
                        v[0] += zo_bf16_lo(r2.x); v[1] += zo_bf16_hi(r2.x); v[2] += zo_bf16_lo(r2.y); v[3] += zo_bf16_hi(r2.y);
                    }
                }
                if constexpr (sizeof(TY) == 4) {
                    *reinterpret_cast<float4*>((float*)Y + off) = make_float4(v[0], v[1], v[2], v[3]);
                } else {
                    uint2 o;
                    o.x = zo_pack_bf16x2(v[0], v[1]);
                    o.y = zo_pack_bf16x2(v[2], v[3]);
                    *reinterpret_cast<uint2*>((zo_bf16*)Y + off) = o;
                }
            } else {
                for (int e = 0; e < 4 && n + e < NO; ++e) {
                    float t = v[e];
                    if (res) t += (float)res[off + e];
                    zo_store(Y + off + e, t);
                }
            }
        }
    }
}

template <typename TY, int SPT, int EPI>
static hipError_t launch_gemm_i8_e(const zo_i8_gemm_args& a, hipStream_t st)
{
    const int tiles = ((a.M + 255) / 256) * ((a.N + 255) / 256);
    constexpr int lds_bytes = 2 * (64 * 1024 + 8 * 1024);
    hipError_t e = hipFuncSetAttribute((const void*)zo_gemm_i8_kernel<TY, SPT, EPI>, hipFuncAttributeMaxDynamicSharedMemorySize, lds_bytes);
    if (e != hipSuccess) return e;
    zo_gemm_i8_kernel<TY, SPT, EPI><<<dim3(tiles, 1, a.batch), 512, lds_bytes, st>>>(a);
    return hipGetLastError();
}
template <typename TY, int SPT>
static hipError_t launch_gemm_i8_t(const zo_i8_gemm_args& a, hipStream_t st)
{
    if (a.epi == 0) return launch_gemm_i8_e<TY, SPT, 0>(a, st);
    if constexpr (sizeof(TY) == 2) {                  // the pairing epilogues exist for bf16 output
        return launch_gemm_i8_e<TY, SPT, 1>(a, st);
    }
    return hipErrorInvalidValue;
}

hipError_t zo_launch_gemm_i8(const zo_i8_gemm_args& a, int out_f32, hipStream_t st)
{
    if (a.M <= 0 || a.N <= 0) return hipSuccess;
    if (a.epi < 0 || a.epi > 1 || (a.epi != 0 && (a.relu || a.residual || (a.N & 127)))) return hipErrorInvalidValue;
    if (a.K < 128 || (a.K & 127) || (a.sgroup != 64 && (a.sgroup & 127)) || a.K % a.sgroup) return hipErrorInvalidValue;
    if (a.sgroup == a.K) return out_f32 ? launch_gemm_i8_t<float, 0>(a, st) : launch_gemm_i8_t<zo_bf16, 0>(a, st);
    if (a.sgroup == 64) return out_f32 ? launch_gemm_i8_t<float, 2>(a, st) : launch_gemm_i8_t<zo_bf16, 2>(a, st);
    return out_f32 ? launch_gemm_i8_t<float, 1>(a, st) : launch_gemm_i8_t<zo_bf16, 1>(a, st);
}
