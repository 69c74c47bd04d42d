// The rest of the decoder forward around the quantized linears, and the scalar tail of the step:
// perturbed embedding gather, RMSNorm / LayerNorm, rotary embedding, causal softmax attention,
// SwiGLU, cross-entropy / squared-error rows, fixed-order loss reduction, projected gradient.
// All kernels read and write activations in the storage type T (fp32 or bf16) and compute in fp32.
#include "zo_device.h"
#include "zo_internal.h"

static inline zo_stream make_stream(uint64_t seed, int32_t tid)
{
    zo_stream s;
    s.k0 = (uint32_t)seed;
    s.k1 = (uint32_t)(seed >> 32);
    s.tensor_id = (uint32_t)tid;
    return s;
}

// ---------------------------------------------------------------------------------------------
// embedding: x[t][:] = rt( theta'_tok[id[t]][:] (+ theta'_pos[t % S][:]) ), theta' = fma(eps, u, theta)
// Only the gathered rows are perturbed (the table itself is never rewritten).
// ---------------------------------------------------------------------------------------------
template <typename TW, typename T>
__global__ __launch_bounds__(256) void zo_embed_kernel(const int32_t* __restrict__ ids, const TW* __restrict__ tok,
                                                       const TW* __restrict__ pos, T* __restrict__ out, int M, int S, int d, int vocab,
                                                       zo_stream st, zo_stream sp, float eps_tok, float eps_pos)
{
    const int t = blockIdx.x;
    int id = ids[t];
    id = id < 0 ? 0 : (id >= vocab ? vocab - 1 : id);
    const int64_t tb = (int64_t)id * d, pb = (int64_t)(t % S) * d;
    for (int c = threadIdx.x * 8; c < d; c += 256 * 8) {
        float v[8], z[8];
        zo_load8(tok + tb + c, v);
        if (eps_tok != 0.0f) {
            zo_z8(st, (uint64_t)(tb + c) >> 3, z);
#pragma unroll
            for (int i = 0; i < 8; ++i) v[i] = __builtin_fmaf(eps_tok, z[i], v[i]);
        }
        if (pos) {
            float p[8];
            zo_load8(pos + pb + c, p);
            if (eps_pos != 0.0f) {
                zo_z8(sp, (uint64_t)(pb + c) >> 3, z);
#pragma unroll
                for (int i = 0; i < 8; ++i) p[i] = __builtin_fmaf(eps_pos, z[i], p[i]);
            }
#pragma unroll
            for (int i = 0; i < 8; ++i) v[i] += p[i];
        }
        zo_store8(out + (int64_t)t * d + c, v);
    }
}

template <typename TW>
static void launch_embed_w(const int32_t* ids, const void* tok_emb, const void* pos_emb, void* out, int32_t M, int32_t S, int32_t d,
                           int32_t vocab, uint64_t seed, int32_t tid_tok, int32_t tid_pos, float eps_tok, float eps_pos, int dtype,
                           hipStream_t st)
{
    if (dtype == ZO_T_BF16)
        zo_embed_kernel<TW, zo_bf16><<<M, 256, 0, st>>>(ids, (const TW*)tok_emb, (const TW*)pos_emb, (zo_bf16*)out, M, S, d, vocab,
                                                        make_stream(seed, tid_tok), make_stream(seed, tid_pos), eps_tok, eps_pos);
    else
        zo_embed_kernel<TW, float><<<M, 256, 0, st>>>(ids, (const TW*)tok_emb, (const TW*)pos_emb, (float*)out, M, S, d, vocab,
                                                      make_stream(seed, tid_tok), make_stream(seed, tid_pos), eps_tok, eps_pos);
}

hipError_t zo_launch_embed(const int32_t* ids, const void* tok_emb, const void* pos_emb, void* out,
                           int32_t M, int32_t S, int32_t d, int32_t vocab, uint64_t seed, int32_t tid_tok, int32_t tid_pos,
                           float eps_tok, float eps_pos, int dtype, hipStream_t st, int wdtype)
{
    if (M == 0) return hipSuccess;
    if (wdtype == ZO_W_F16) launch_embed_w<zo_f16>(ids, tok_emb, pos_emb, out, M, S, d, vocab, seed, tid_tok, tid_pos, eps_tok, eps_pos, dtype, st);
    else launch_embed_w<float>(ids, tok_emb, pos_emb, out, M, S, d, vocab, seed, tid_tok, tid_pos, eps_tok, eps_pos, dtype, st);
    return hipGetLastError();
}

// ---------------------------------------------------------------------------------------------
// RMSNorm / LayerNorm: one wavefront per row, fp32 statistics.
// ---------------------------------------------------------------------------------------------
template <typename T>
__global__ __launch_bounds__(256) void zo_norm_kernel(const T* __restrict__ x, const float* __restrict__ gamma,
                                                      const float* __restrict__ beta, T* __restrict__ out, int M, int d, float eps)
{
    const int lane = threadIdx.x & 63;
    const int row = blockIdx.x * 4 + (threadIdx.x >> 6);
    if (row >= M) return;
    const T* xr = x + (int64_t)row * d;
    float s1 = 0.0f, s2 = 0.0f;
    for (int c = lane * 8; c < d; c += 512) {
        float v[8];
        zo_load8(xr + c, v);
#pragma unroll
        for (int i = 0; i < 8; ++i) { s1 += v[i]; s2 = __builtin_fmaf(v[i], v[i], s2); }
    }
    s1 = zo_group_sum<64>(s1);
    s2 = zo_group_sum<64>(s2);
    float mean = 0.0f, var;
    if (beta) {                                       // LayerNorm: second sweep for the centred variance
        mean = s1 / (float)d;
        float sv = 0.0f;
        for (int c = lane * 8; c < d; c += 512) {
            float v[8];
            zo_load8(xr + c, v);
#pragma unroll
            for (int i = 0; i < 8; ++i) { float t = v[i] - mean; sv = __builtin_fmaf(t, t, sv); }
        }
        var = zo_group_sum<64>(sv) / (float)d;
    } else {
        var = s2 / (float)d;
    }
    const float rstd = 1.0f / __builtin_sqrtf(var + eps);
    for (int c = lane * 8; c < d; c += 512) {
        float v[8], g[8], o[8];
        zo_load8(xr + c, v);
        zo_load8(gamma + c, g);
        if (beta) {
            float b[8];
            zo_load8(beta + c, b);
#pragma unroll
            for (int i = 0; i < 8; ++i) o[i] = __builtin_fmaf((v[i] - mean) * rstd, g[i], b[i]);
        } else {
#pragma unroll
            for (int i = 0; i < 8; ++i) o[i] = (v[i] * rstd) * g[i];
        }
        zo_store8(out + (int64_t)row * d + c, o);
    }
}

hipError_t zo_launch_norm(const void* x, const float* gamma, const float* beta, void* out,
                          int32_t M, int32_t d, float eps, int dtype, hipStream_t st)
{
    if (M == 0) return hipSuccess;
    const int grid = (M + 3) / 4;
    if (dtype == ZO_T_BF16) zo_norm_kernel<zo_bf16><<<grid, 256, 0, st>>>((const zo_bf16*)x, gamma, beta, (zo_bf16*)out, M, d, eps);
    else zo_norm_kernel<float><<<grid, 256, 0, st>>>((const float*)x, gamma, beta, (float*)out, M, d, eps);
    return hipGetLastError();
}

// ---------------------------------------------------------------------------------------------
// RMSNorm / LayerNorm fused with the per-token quantizer of the linear that follows:
// x^ = rt(Q_A(rt(norm(x)))).  The row stays in registers: WPR = 1 wavefront per row for short rows
// (4 rows per workgroup), WPR = 4 (the whole workgroup, 16 bytes per thread and 4 KB chunk) for long
// ones; the four partial results of a row meet in LDS and are combined in a fixed order.
// ---------------------------------------------------------------------------------------------
template <typename T, int NC, int WPR>
__global__ __launch_bounds__(256) void zo_norm_quant_kernel(const T* __restrict__ x, const float* __restrict__ gamma,
                                                            const float* __restrict__ beta, T* __restrict__ xhat, int M, int d,
                                                            float eps, int bits, int sym,
                                                            const float* __restrict__ sm_delta, const float* __restrict__ sm_inv,
                                                            int8_t* __restrict__ codes, float* __restrict__ xs, float* __restrict__ xo)
{
    __shared__ float red[5][4];
    constexpr int TPR = 64 * WPR;                    // threads per row
    const int tr = threadIdx.x % TPR, wave = threadIdx.x >> 6;
    const int row = blockIdx.x * (4 / WPR) + threadIdx.x / TPR;
    if (row >= M) return;                            // a whole wavefront (WPR = 1) or workgroup (WPR = 4)
    const T* xr = x + (int64_t)row * d;
    float v[NC][8], g[NC][8];
    float s1 = 0.0f, s2 = 0.0f;
#pragma unroll
    for (int i = 0; i < NC; ++i) {
        const int c = tr * 8 + 8 * TPR * i;
        if (c < d) {
            zo_load8(xr + c, v[i]);
            zo_load8(gamma + c, g[i]);               // requested with the row: not needed before the statistics are known
        }
    }
#pragma unroll
    for (int i = 0; i < NC; ++i)
        if (tr * 8 + 8 * TPR * i < d) {
#pragma unroll
            for (int e = 0; e < 8; ++e) { s1 += v[i][e]; s2 = __builtin_fmaf(v[i][e], v[i][e], s2); }
        }
    s2 = zo_group_sum<64>(s2);
    if (beta) s1 = zo_group_sum<64>(s1);
    if (WPR == 4) {
        if ((threadIdx.x & 63) == 0) { red[0][wave] = s1; red[1][wave] = s2; }
        __syncthreads();
        s1 = (red[0][0] + red[0][1]) + (red[0][2] + red[0][3]);
        s2 = (red[1][0] + red[1][1]) + (red[1][2] + red[1][3]);
    }
    float mean = 0.0f, var;
    if (beta) {
        mean = s1 / (float)d;
        float sv = 0.0f;
#pragma unroll
        for (int i = 0; i < NC; ++i)
            if (tr * 8 + 8 * TPR * i < d) {
#pragma unroll
                for (int e = 0; e < 8; ++e) { float t = v[i][e] - mean; sv = __builtin_fmaf(t, t, sv); }
            }
        sv = zo_group_sum<64>(sv);
        if (WPR == 4) {
            if ((threadIdx.x & 63) == 0) red[2][wave] = sv;
            __syncthreads();
            sv = (red[2][0] + red[2][1]) + (red[2][2] + red[2][3]);
        }
        var = sv / (float)d;
    } else {
        var = s2 / (float)d;
    }
    const float rstd = 1.0f / __builtin_sqrtf(var + eps);
    float mn = INFINITY, mx = -INFINITY;
#pragma unroll
    for (int i = 0; i < NC; ++i) {
        const int c = tr * 8 + 8 * TPR * i;
        if (c < d) {
            if (beta) {
                float b[8];
                zo_load8(beta + c, b);
#pragma unroll
                for (int e = 0; e < 8; ++e) v[i][e] = zo_round_to<T>(__builtin_fmaf((v[i][e] - mean) * rstd, g[i][e], b[e]));
            } else {
#pragma unroll
                for (int e = 0; e < 8; ++e) v[i][e] = zo_round_to<T>((v[i][e] * rstd) * g[i][e]);
            }
            if (sm_delta) {                           // Eq. 4: the quantizer sees (x - delta) / s
                float dl[8], iv[8];
                zo_load8(sm_delta + c, dl);
                zo_load8(sm_inv + c, iv);
#pragma unroll
                for (int e = 0; e < 8; ++e) v[i][e] = (v[i][e] - dl[e]) * iv[e];
            }
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                if (sym) mx = fmaxf(mx, fabsf(v[i][e]));
                else { mn = fminf(mn, v[i][e]); mx = fmaxf(mx, v[i][e]); }
            }
        }
    }
    mn = zo_group_min<64>(mn);
    mx = zo_group_max<64>(mx);
    if (WPR == 4) {
        if ((threadIdx.x & 63) == 0) { red[3][wave] = mn; red[4][wave] = mx; }
        __syncthreads();
        mn = fminf(fminf(red[3][0], red[3][1]), fminf(red[3][2], red[3][3]));
        mx = fmaxf(fmaxf(red[4][0], red[4][1]), fmaxf(red[4][2], red[4][3]));
    }
    const zo_qparams q = sym ? zo_qparams_sym(mx, bits) : zo_qparams_asym(mn, mx, bits);
    if (codes) {
        // integer route: the codes themselves, re-centred into a signed byte, and the row's step and offset - zero point
        const float off = sym ? 0.0f : (float)(1 << (bits - 1));
        if (tr == 0) { xs[row] = q.step; xo[row] = off - q.zp; }
#pragma unroll
        for (int i = 0; i < NC; ++i) {
            const int c = tr * 8 + 8 * TPR * i;
            if (c < d) *reinterpret_cast<uint2*>(codes + (int64_t)row * d + c) = zo_pack_codes8(q, v[i], off);
        }
        return;
    }
#pragma unroll
    for (int i = 0; i < NC; ++i) {
        const int c = tr * 8 + 8 * TPR * i;
        if (c < d) {
            float o[8];
#pragma unroll
            for (int e = 0; e < 8; ++e) o[e] = zo_dequant(q, zo_code(q, v[i][e]));
            zo_store8(xhat + (int64_t)row * d + c, o);
        }
    }
}

bool zo_norm_quant_supported(int32_t d) { return d > 0 && (d & 7) == 0 && d <= 8192; }

hipError_t zo_launch_norm_quant(const void* x, const float* gamma, const float* beta, void* xhat, int32_t M, int32_t d,
                                float eps, int32_t bits, int32_t sym, int dtype,
                                const float* sm_delta, const float* sm_inv, hipStream_t st, int8_t* codes, float* xs, float* xo)
{
    if (M == 0) return hipSuccess;
    if (codes && (!xs || !xo)) return hipErrorInvalidValue;
    // rows up to 1024 elements: one wavefront each; longer ones: one workgroup each
#define ZO_NQ(T, NC, WPR) zo_norm_quant_kernel<T, NC, WPR><<<(WPR == 4 ? M : (M + 3) / 4), 256, 0, st>>>((const T*)x, gamma, beta, (T*)xhat, M, d, eps, bits, sym, sm_delta, sm_inv, codes, xs, xo)
#define ZO_NQ_ALL(T)                          \
    if (d <= 512) ZO_NQ(T, 1, 1);             \
    else if (d <= 1024) ZO_NQ(T, 2, 1);       \
    else if (d <= 2048) ZO_NQ(T, 1, 4);       \
    else if (d <= 4096) ZO_NQ(T, 2, 4);       \
    else ZO_NQ(T, 4, 4)
    if (dtype == ZO_T_BF16) { ZO_NQ_ALL(zo_bf16); } else { ZO_NQ_ALL(float); }
#undef ZO_NQ_ALL
#undef ZO_NQ
    return hipGetLastError();
}

// ---------------------------------------------------------------------------------------------
// rotary embedding on q and k, in place: pairs (i, i + dh/2) of every head, angle table [S][dh/2]
// ---------------------------------------------------------------------------------------------
template <typename T>
__global__ __launch_bounds__(256) void zo_rope_kernel(T* __restrict__ q, T* __restrict__ k, const float* __restrict__ ct,
                                                      const float* __restrict__ stab, int M, int S, int H, int dh, int64_t row_stride)
{
    const int half = dh / 2;
    const int64_t total = (int64_t)M * H * half;
    for (int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x; idx < total; idx += (int64_t)gridDim.x * 256) {
        const int i = (int)(idx % half);
        const int h = (int)((idx / half) % H);
        const int64_t t = idx / ((int64_t)half * H);
        const int pos = (int)(t % S);
        const float c = ct[pos * half + i], s = stab[pos * half + i];
        const int64_t o = t * row_stride + (int64_t)h * dh + i;
        float a = zo_load(q + o), b = zo_load(q + o + half);
        zo_store(q + o, __builtin_fmaf(a, c, -(b * s)));
        zo_store(q + o + half, __builtin_fmaf(b, c, a * s));
        a = zo_load(k + o); b = zo_load(k + o + half);
        zo_store(k + o, __builtin_fmaf(a, c, -(b * s)));
        zo_store(k + o + half, __builtin_fmaf(b, c, a * s));
    }
}

hipError_t zo_launch_rope(void* q, void* k, const float* cos_tab, const float* sin_tab,
                          int32_t M, int32_t S, int32_t H, int32_t dh, int64_t row_stride, int dtype, hipStream_t st)
{
    const int64_t total = (int64_t)M * H * (dh / 2);
    if (total == 0) return hipSuccess;
    int grid = (int)((total + 255) / 256 < 65535 * 4 ? (total + 255) / 256 : 65535 * 4);
    if (dtype == ZO_T_BF16) zo_rope_kernel<zo_bf16><<<grid, 256, 0, st>>>((zo_bf16*)q, (zo_bf16*)k, cos_tab, sin_tab, M, S, H, dh, row_stride);
    else zo_rope_kernel<float><<<grid, 256, 0, st>>>((float*)q, (float*)k, cos_tab, sin_tab, M, S, H, dh, row_stride);
    return hipGetLastError();
}

// ---------------------------------------------------------------------------------------------
// causal softmax attention, generic version: one wavefront per query row, keys in chunks of 64
// (one key per lane), online softmax, then P*V with lanes over the head dimension.
// ---------------------------------------------------------------------------------------------
template <typename T, int DH>
__global__ __launch_bounds__(256) void zo_attention_kernel(const T* __restrict__ q, const T* __restrict__ k, const T* __restrict__ v,
                                                           T* __restrict__ out, int B, int S, int H, int64_t row_stride, float scale)
{
    __shared__ float qs[4][DH];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int64_t qi = (int64_t)blockIdx.x * 4 + wave;           // over B*H*S, s fastest
    const bool valid = qi < (int64_t)B * H * S;
    const int s = (int)(qi % S);
    const int h = (int)((qi / S) % H);
    const int b = (int)(qi / ((int64_t)S * H));
    const int64_t rowq = ((int64_t)b * S + s) * row_stride + (int64_t)h * DH;
    if (valid)
        for (int i = lane; i < DH; i += 64) qs[wave][i] = zo_load(q + rowq + i) * scale;
    __syncthreads();
    if (!valid) return;
    constexpr int PER = (DH + 63) / 64;
    float o[PER];
#pragma unroll
    for (int i = 0; i < PER; ++i) o[i] = 0.0f;
    float mrun = -INFINITY, lrun = 0.0f;
    for (int j0 = 0; j0 <= s; j0 += 64) {
        const int j = j0 + lane;
        float sc = -INFINITY;
        if (j <= s) {
            const T* kr = k + ((int64_t)b * S + j) * row_stride + (int64_t)h * DH;
            float acc = 0.0f;
#pragma unroll 8
            for (int i = 0; i < DH; i += 8) {
                float kv[8];
                zo_load8(kr + i, kv);
#pragma unroll
                for (int e = 0; e < 8; ++e) acc = __builtin_fmaf(qs[wave][i + e], kv[e], acc);
            }
            sc = acc;
        }
        const float mnew = fmaxf(mrun, zo_group_max<64>(sc));
        const float p = (j <= s) ? __expf(sc - mnew) : 0.0f;
        const float corr = __expf(mrun - mnew);
        lrun = lrun * corr + zo_group_sum<64>(p);
        mrun = mnew;
        const int cnt = (s - j0 + 1) < 64 ? (s - j0 + 1) : 64;
#pragma unroll
        for (int i = 0; i < PER; ++i) o[i] *= corr;
        for (int jj = 0; jj < cnt; ++jj) {
            const float pj = __uint_as_float(__builtin_amdgcn_readlane(__float_as_uint(p), jj));
            const T* vr = v + ((int64_t)b * S + j0 + jj) * row_stride + (int64_t)h * DH;
#pragma unroll
            for (int i = 0; i < PER; ++i) {
                const int dcol = lane + 64 * i;
                if (dcol < DH) o[i] = __builtin_fmaf(pj, zo_load(vr + dcol), o[i]);
            }
        }
    }
    const float inv = 1.0f / lrun;
    T* orow = out + ((int64_t)b * S + s) * ((int64_t)H * DH) + (int64_t)h * DH;
#pragma unroll
    for (int i = 0; i < PER; ++i) {
        const int dcol = lane + 64 * i;
        if (dcol < DH) zo_store(orow + dcol, o[i] * inv);
    }
}

hipError_t zo_launch_attention(const void* q, const void* k, const void* v, void* out,
                               int32_t B, int32_t S, int32_t H, int32_t dh, int64_t row_stride, int dtype, hipStream_t st)
{
    const int64_t nq = (int64_t)B * S * H;
    if (nq == 0) return hipSuccess;
    const int grid = (int)((nq + 3) / 4);
    const float scale = 1.0f / sqrtf((float)dh);
#define ZO_ATT(T, D) zo_attention_kernel<T, D><<<grid, 256, 0, st>>>((const T*)q, (const T*)k, (const T*)v, (T*)out, B, S, H, row_stride, scale)
    if (dtype == ZO_T_BF16) {
        if (dh == 16) ZO_ATT(zo_bf16, 16); else if (dh == 32) ZO_ATT(zo_bf16, 32); else if (dh == 64) ZO_ATT(zo_bf16, 64);
        else if (dh == 128) ZO_ATT(zo_bf16, 128); else return hipErrorInvalidValue;
    } else {
        if (dh == 16) ZO_ATT(float, 16); else if (dh == 32) ZO_ATT(float, 32); else if (dh == 64) ZO_ATT(float, 64);
        else if (dh == 128) ZO_ATT(float, 128); else return hipErrorInvalidValue;
    }
#undef ZO_ATT
    return hipGetLastError();
}

// ---------------------------------------------------------------------------------------------
// SwiGLU: out = rt( silu(gate) * up )
// ---------------------------------------------------------------------------------------------
template <typename T>
__global__ __launch_bounds__(256) void zo_swiglu_kernel(const T* __restrict__ gate, const T* __restrict__ up, T* __restrict__ out,
                                                        int64_t rows, int cols, int64_t in_stride)
{
    const int64_t per_row = cols / 8;
    const int64_t total = rows * per_row;
    for (int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x; idx < total; idx += (int64_t)gridDim.x * 256) {
        const int64_t r = idx / per_row;
        const int c = (int)(idx % per_row) * 8;
        float g[8], u[8], o[8];
        zo_load8(gate + r * in_stride + c, g);
        zo_load8(up + r * in_stride + c, u);
#pragma unroll
        for (int i = 0; i < 8; ++i) o[i] = (g[i] / (1.0f + __expf(-g[i]))) * u[i];
        zo_store8(out + r * cols + c, o);
    }
}

hipError_t zo_launch_swiglu(const void* gate, const void* up, void* out, int64_t rows, int32_t cols,
                            int64_t in_stride, int dtype, hipStream_t st)
{
    const int64_t total = rows * (cols / 8);
    if (total == 0) return hipSuccess;
    int grid = (int)((total + 255) / 256 < 262144 ? (total + 255) / 256 : 262144);
    if (dtype == ZO_T_BF16) zo_swiglu_kernel<zo_bf16><<<grid, 256, 0, st>>>((const zo_bf16*)gate, (const zo_bf16*)up, (zo_bf16*)out, rows, cols, in_stride);
    else zo_swiglu_kernel<float><<<grid, 256, 0, st>>>((const float*)gate, (const float*)up, (float*)out, rows, cols, in_stride);
    return hipGetLastError();
}

// ---------------------------------------------------------------------------------------------
// SwiGLU fused with the per-token quantizer of the down projection:
// x^ = rt(Q_A(rt(silu(gate) * up))).  One workgroup per row, the row stays in registers.
// up = NULL: the per-token quantizer alone on the row `gate` (one read, one write per element).
// NT threads per row: 256, or 1024 where there are only a few rows (a decoding step), which shortens a lane's serial chain.
// ---------------------------------------------------------------------------------------------
template <typename T, int NC, int NT = 256>
__global__ __launch_bounds__(NT) void zo_swiglu_quant_kernel(const T* __restrict__ gate, const T* __restrict__ up, T* __restrict__ xhat,
                                                              int cols, int64_t in_stride, int bits, int sym,
                                                              const float* __restrict__ sm_delta, const float* __restrict__ sm_inv,
                                                              int8_t* __restrict__ codes, float* __restrict__ xs, float* __restrict__ xo)
{
    __shared__ float red[2][NT / 64];
    const int64_t row = blockIdx.x;
    float v[NC][8];
    float mn = INFINITY, mx = -INFINITY;
#pragma unroll
    for (int i = 0; i < NC; ++i) {
        const int c = threadIdx.x * 8 + NT * 8 * i;
        if (c < cols) {
            float g[8], u[8];
            zo_load8(gate + row * in_stride + c, g);
            if (up) zo_load8(up + row * in_stride + c, u);
            float dl[8], iv[8];
            if (sm_delta) { zo_load8(sm_delta + c, dl); zo_load8(sm_inv + c, iv); }
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                v[i][e] = up ? zo_round_to<T>((g[e] / (1.0f + __expf(-g[e]))) * u[e]) : g[e];
                if (sm_delta) v[i][e] = (v[i][e] - dl[e]) * iv[e];
                if (sym) mx = fmaxf(mx, fabsf(v[i][e]));
                else { mn = fminf(mn, v[i][e]); mx = fmaxf(mx, v[i][e]); }
            }
        }
    }
    mn = zo_group_min<64>(mn);
    mx = zo_group_max<64>(mx);
    if ((threadIdx.x & 63) == 0) { red[0][threadIdx.x >> 6] = mn; red[1][threadIdx.x >> 6] = mx; }
    __syncthreads();
    mn = red[0][0];
    mx = red[1][0];
#pragma unroll
    for (int w = 1; w < NT / 64; ++w) { mn = fminf(mn, red[0][w]); mx = fmaxf(mx, red[1][w]); }
    const zo_qparams q = sym ? zo_qparams_sym(mx, bits) : zo_qparams_asym(mn, mx, bits);
    if (codes) {                                     // integer route (see zo_norm_quant_kernel)
        const float off = sym ? 0.0f : (float)(1 << (bits - 1));
        if (threadIdx.x == 0) { xs[row] = q.step; xo[row] = off - q.zp; }
#pragma unroll
        for (int i = 0; i < NC; ++i) {
            const int c = threadIdx.x * 8 + NT * 8 * i;
            if (c < cols) *reinterpret_cast<uint2*>(codes + row * cols + c) = zo_pack_codes8(q, v[i], off);
        }
        return;
    }
#pragma unroll
    for (int i = 0; i < NC; ++i) {
        const int c = threadIdx.x * 8 + NT * 8 * i;
        if (c < cols) {
            float o[8];
#pragma unroll
            for (int e = 0; e < 8; ++e) o[e] = zo_dequant(q, zo_code(q, v[i][e]));
            zo_store8(xhat + row * cols + c, o);
        }
    }
}

bool zo_swiglu_quant_supported(int32_t cols) { return cols > 0 && (cols & 7) == 0 && cols <= 16384; }

hipError_t zo_launch_swiglu_quant(const void* gate, const void* up, void* xhat, int64_t rows, int32_t cols, int64_t in_stride,
                                  int32_t bits, int32_t sym, int dtype, const float* sm_delta, const float* sm_inv, hipStream_t st,
                                  int8_t* codes, float* xs, float* xo)
{
    if (rows == 0) return hipSuccess;
    if (codes && (!xs || !xo)) return hipErrorInvalidValue;
    if (rows > 0x7FFFFFFF) return hipErrorInvalidValue;
#define ZO_SQ(T, NC) zo_swiglu_quant_kernel<T, NC><<<(int)rows, 256, 0, st>>>((const T*)gate, (const T*)up, (T*)xhat, cols, in_stride, bits, sym, sm_delta, sm_inv, codes, xs, xo)
#define ZO_SQW(T, NC) zo_swiglu_quant_kernel<T, NC, 1024><<<(int)rows, 1024, 0, st>>>((const T*)gate, (const T*)up, (T*)xhat, cols, in_stride, bits, sym, sm_delta, sm_inv, codes, xs, xo)
    if (rows <= 16 && cols > 2048) {                 // too few rows to fill the chip anyway: more lanes per row
        if (dtype == ZO_T_BF16) { if (cols <= 8192) ZO_SQW(zo_bf16, 1); else ZO_SQW(zo_bf16, 2); }
        else { if (cols <= 8192) ZO_SQW(float, 1); else ZO_SQW(float, 2); }
        return hipGetLastError();
    }
    if (dtype == ZO_T_BF16) {
        if (cols <= 4096) ZO_SQ(zo_bf16, 2); else if (cols <= 12288) ZO_SQ(zo_bf16, 6); else ZO_SQ(zo_bf16, 8);
    } else {
        if (cols <= 4096) ZO_SQ(float, 2); else if (cols <= 12288) ZO_SQ(float, 6); else ZO_SQ(float, 8);
    }
#undef ZO_SQ
#undef ZO_SQW
    return hipGetLastError();
}

// ---------------------------------------------------------------------------------------------
// losses.  Cross entropy: one workgroup per token row of the fp32 logits; the row loss of the last
// position of every sequence is 0.  Squared error: one workgroup per row.  Reduction in fixed order.
// ---------------------------------------------------------------------------------------------
__device__ __forceinline__ float block_reduce_max(float v, float* sm)
{
    v = zo_group_max<64>(v);
    if ((threadIdx.x & 63) == 0) sm[threadIdx.x >> 6] = v;
    __syncthreads();
    v = fmaxf(fmaxf(sm[0], sm[1]), fmaxf(sm[2], sm[3]));
    __syncthreads();
    return v;
}
__device__ __forceinline__ float block_reduce_sum(float v, float* sm)
{
    v = zo_group_sum<64>(v);
    if ((threadIdx.x & 63) == 0) sm[threadIdx.x >> 6] = v;
    __syncthreads();
    v = (sm[0] + sm[1]) + (sm[2] + sm[3]);
    __syncthreads();
    return v;
}

__global__ __launch_bounds__(256) void zo_ce_rows_kernel(const float* __restrict__ logits, const int32_t* __restrict__ ids,
                                                         float* __restrict__ row_loss, int M, int S, int V)
{
    __shared__ float sm[4];
    const int t = blockIdx.x;
    if ((t % S) == S - 1) {
        if (threadIdx.x == 0) row_loss[t] = 0.0f;
        return;
    }
    const float* lg = logits + (int64_t)t * V;
    float mx = -INFINITY;
    for (int c = threadIdx.x; c < V; c += 256) mx = fmaxf(mx, lg[c]);
    mx = block_reduce_max(mx, sm);
    float se = 0.0f;
    for (int c = threadIdx.x; c < V; c += 256) se += expf(lg[c] - mx);
    se = block_reduce_sum(se, sm);
    if (threadIdx.x == 0) {
        int tgt = ids[t + 1];
        tgt = tgt < 0 ? 0 : (tgt >= V ? V - 1 : tgt);
        row_loss[t] = (logf(se) + mx) - lg[tgt];
    }
}

hipError_t zo_launch_ce_rows(const float* logits, const int32_t* ids, float* row_loss, int32_t M, int32_t S, int32_t V, hipStream_t st)
{
    if (M == 0) return hipSuccess;
    zo_ce_rows_kernel<<<M, 256, 0, st>>>(logits, ids, row_loss, M, S, V);
    return hipGetLastError();
}

template <typename T>
__global__ __launch_bounds__(256) void zo_sqerr_rows_kernel(const T* __restrict__ y, const float* __restrict__ target,
                                                            float* __restrict__ row_loss, int M, int N)
{
    __shared__ float sm[4];
    const int t = blockIdx.x;
    float s = 0.0f;
    for (int c = threadIdx.x; c < N; c += 256) {
        float dlt = zo_load(y + (int64_t)t * N + c) - target[(int64_t)t * N + c];
        s = __builtin_fmaf(dlt, dlt, s);
    }
    s = block_reduce_sum(s, sm);
    if (threadIdx.x == 0) row_loss[t] = s;
}

hipError_t zo_launch_sqerr_rows(const void* y, const float* target, float* row_loss, int32_t M, int32_t N, int dtype, hipStream_t st)
{
    if (M == 0) return hipSuccess;
    if (dtype == ZO_T_BF16) zo_sqerr_rows_kernel<zo_bf16><<<M, 256, 0, st>>>((const zo_bf16*)y, target, row_loss, M, N);
    else zo_sqerr_rows_kernel<float><<<M, 256, 0, st>>>((const float*)y, target, row_loss, M, N);
    return hipGetLastError();
}

// one workgroup; every thread sums a strided slice in fp64, then a fixed tree
__global__ __launch_bounds__(256) void zo_reduce_loss_kernel(const float* __restrict__ row_loss, int M, float scale, float* __restrict__ loss)
{
    __shared__ double sm[256];
    double s = 0.0;
    for (int i = threadIdx.x; i < M; i += 256) s += (double)row_loss[i];
    sm[threadIdx.x] = s;
    __syncthreads();
    for (int o = 128; o > 0; o >>= 1) {
        if (threadIdx.x < o) sm[threadIdx.x] += sm[threadIdx.x + o];
        __syncthreads();
    }
    if (threadIdx.x == 0) *loss = (float)(sm[0] * (double)scale);
}

hipError_t zo_launch_reduce_loss(const float* row_loss, int32_t M, float scale, float* loss, hipStream_t st)
{
    zo_reduce_loss_kernel<<<1, 256, 0, st>>>(row_loss, M, scale, loss);
    return hipGetLastError();
}

// g = (L+ - L-) / (2 eps) (Eq. 2, q = 1) and c = eta * g (Eq. 3), formed in fp64, stored as fp32
// out6 = { L+, L-, g, c_model, c_smoothing, c_clipping } (one coefficient per learning-rate group);
// the first n_user values are also written to user_out
__global__ void zo_projected_grad_kernel(const float* __restrict__ loss2, float eps, float lr0, float lr1, float lr2,
                                         float* __restrict__ out6, float* __restrict__ user_out, int n_user)
{
    const float lp = loss2[0], lm = loss2[1];
    const float g = (float)(((double)lp - (double)lm) / (2.0 * (double)eps));
    float v[6];
    v[0] = lp;
    v[1] = lm;
    v[2] = g;
    v[3] = (float)((double)lr0 * (double)g);
    v[4] = (float)((double)lr1 * (double)g);
    v[5] = (float)((double)lr2 * (double)g);
    for (int i = 0; i < 6; ++i) out6[i] = v[i];
    for (int i = 0; i < n_user; ++i) user_out[i] = v[i];
}

hipError_t zo_launch_projected_grad(const float* loss2, float eps, const float lr[3], float* out6, float* user_out, int n_user,
                                    hipStream_t st)
{
    zo_projected_grad_kernel<<<1, 1, 0, st>>>(loss2, eps, lr[0], lr[1], lr[2], out6, user_out, n_user);
    return hipGetLastError();
}
