// Kernels of the generator on the quantized model (prompt pass + cached decoding; efficiency section, on-device
// inference): attention of ONE new query over the cached keys / values of a sequence, and the arg max of a row of logits.
#include "zo_device.h"
#include "zo_internal.h"

// One workgroup per head, dh / 8 lanes per cached row (each lane owns 8 consecutive dimensions: one 16-byte load per row).
// scores[j] = q . K[j] / sqrt(dh): partial dot products of the lanes of a row are added with register-to-register
// exchanges; a numerically safe softmax in fp32 (fixed-order reductions); out = sum_j p_j V[j]: the 256 / (dh / 8) row
// groups accumulate their rows j = group, group + groups, ... and their partial sums are added in group order through
// LDS.  The row loops are unrolled so that several 16-byte loads are in flight per lane.
template <typename T, int LPK>
__global__ __launch_bounds__(256) void zo_decode_attention_kernel(const T* __restrict__ q, const T* __restrict__ Kc, const T* __restrict__ Vc,
                                                                  T* __restrict__ out, int n, int d, float scale)
{
    constexpr int DH = LPK * 8, KG = 256 / LPK;
    extern __shared__ float sm[];                     // [n] scores, [8] wave results, [KG][DH] partial outputs
    float* sc = sm;
    float* red = sm + n;
    float* part = red + 8;
    const int h = blockIdx.x, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int sub = tid % LPK, kg = tid / LPK;
    const int64_t hoff = (int64_t)h * DH + sub * 8;
    float qv[8];
    zo_load8(q + hoff, qv);
    float mx = -INFINITY;
#pragma unroll 4
    for (int j = kg; j < n; j += KG) {
        float v[8];
        zo_load8(Kc + (int64_t)j * d + hoff, v);
        float acc = 0.0f;
#pragma unroll
        for (int e = 0; e < 8; ++e) acc = __builtin_fmaf(v[e], qv[e], acc);
        acc = zo_group_sum<LPK>(acc) * scale;
        if (sub == 0) sc[j] = acc;
        mx = fmaxf(mx, acc);
    }
    mx = zo_group_max<64>(mx);
    if (lane == 0) red[wave] = mx;
    __syncthreads();
    mx = fmaxf(fmaxf(red[0], red[1]), fmaxf(red[2], red[3]));
    float sum = 0.0f;
    for (int j = tid; j < n; j += 256) {
        const float p = __expf(sc[j] - mx);
        sc[j] = p;
        sum += p;
    }
    sum = zo_group_sum<64>(sum);
    if (lane == 0) red[4 + wave] = sum;
    __syncthreads();
    sum = ((red[4] + red[5]) + red[6]) + red[7];
    float o[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) o[e] = 0.0f;
#pragma unroll 4
    for (int j = kg; j < n; j += KG) {
        float v[8];
        zo_load8(Vc + (int64_t)j * d + hoff, v);
        const float p = sc[j];
#pragma unroll
        for (int e = 0; e < 8; ++e) o[e] = __builtin_fmaf(p, v[e], o[e]);
    }
#pragma unroll
    for (int e = 0; e < 8; ++e) part[kg * DH + sub * 8 + e] = o[e];
    __syncthreads();
    if (tid < DH) {
        float t = part[tid];
        for (int g = 1; g < KG; ++g) t += part[g * DH + tid];
        zo_store(out + (int64_t)h * DH + tid, t / sum);
    }
}

template <typename T>
static hipError_t launch_decode_attention_t(const T* q, const T* Kc, const T* Vc, T* out, int n, int H, int dh, hipStream_t st)
{
    const int d = H * dh;
    const size_t lds = ((size_t)n + 8 + 2048) * sizeof(float);
    if (lds > 160 * 1024) return hipErrorInvalidValue;
    const float scale = 1.0f / sqrtf((float)dh);
#define ZO_DEC_ATT(L)                                                                                                              \
    do {                                                                                                                           \
        if (lds > 64 * 1024) {                                                                                                     \
            hipError_t e = hipFuncSetAttribute((const void*)zo_decode_attention_kernel<T, L>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds); \
            if (e != hipSuccess) return e;                                                                                         \
        }                                                                                                                          \
        zo_decode_attention_kernel<T, L><<<H, 256, lds, st>>>(q, Kc, Vc, out, n, d, scale);                                        \
    } while (0)
    switch (dh) {
        case 16:  ZO_DEC_ATT(2); break;
        case 32:  ZO_DEC_ATT(4); break;
        case 64:  ZO_DEC_ATT(8); break;
        default:  ZO_DEC_ATT(16); break;
    }
#undef ZO_DEC_ATT
    return hipGetLastError();
}

hipError_t zo_launch_decode_attention(const void* q, const void* Kc, const void* Vc, void* out, int32_t n, int32_t H, int32_t dh,
                                      int dtype, hipStream_t st)
{
    if (n <= 0 || H <= 0 || (dh != 16 && dh != 32 && dh != 64 && dh != 128)) return hipErrorInvalidValue;
    if (dtype == ZO_T_BF16)
        return launch_decode_attention_t<zo_bf16>((const zo_bf16*)q, (const zo_bf16*)Kc, (const zo_bf16*)Vc, (zo_bf16*)out, n, H, dh, st);
    return launch_decode_attention_t<float>((const float*)q, (const float*)Kc, (const float*)Vc, (float*)out, n, H, dh, st);
}

// token = lowest index of the largest logit (NaNs never win).  One workgroup.
__global__ __launch_bounds__(1024) void zo_argmax_kernel(const float* __restrict__ logits, int V, int32_t* __restrict__ token)
{
    __shared__ float bv[16];
    __shared__ int bi[16];
    float best = -INFINITY;
    int idx = 0x7FFFFFFF;
    for (int j = threadIdx.x; j < V; j += 1024) {
        const float v = logits[j];
        if (v > best || (v == best && j < idx)) { best = v; idx = j; }
    }
#pragma unroll
    for (int o = 32; o >= 1; o >>= 1) {
        const float ov = __shfl_xor(best, o);
        const int oi = __shfl_xor(idx, o);
        if (ov > best || (ov == best && oi < idx)) { best = ov; idx = oi; }
    }
    if ((threadIdx.x & 63) == 0) { bv[threadIdx.x >> 6] = best; bi[threadIdx.x >> 6] = idx; }
    __syncthreads();
    if (threadIdx.x == 0) {
        for (int w = 1; w < 16; ++w)
            if (bv[w] > best || (bv[w] == best && bi[w] < idx)) { best = bv[w]; idx = bi[w]; }
        *token = idx == 0x7FFFFFFF ? 0 : idx;
    }
}

hipError_t zo_launch_argmax(const float* logits, int32_t V, int32_t* token, hipStream_t st)
{
    if (V <= 0) return hipErrorInvalidValue;
    zo_argmax_kernel<<<1, 1024, 0, st>>>(logits, V, token);
    return hipGetLastError();
}

// ---------------------------------------------------------------------------------------------
// Frozen (packed 4-bit) linear for ONE token -- the linear of a decoding step: y[n] = sum_k x^[k] (code[n][k] - zp[n][g]) step[n][g].
// Bound by the 0.5 B per weight it reads.  A workgroup of two waves covers four output channels; the 128 lanes split K in
// chunks of 32 codes (one 16-byte load per channel and chunk; a chunk lies inside one group).  The activations of a chunk
// are loaded once (they are bf16 pairs as stored) and serve all four channels.  Codes are not converted one by one: a
// code dword holds k = 0..7 as nibbles; (w >> 4 j) & 0x000F000F picks codes j and j + 4 into the low bits of two half
// words, OR-ing 0x4300 into each makes them the bf16 values 128 + code exactly, and one packed dot-product instruction
// multiplies the pair with the activation pair (x_j, x_{j+4}) (built once per chunk by byte permutes) into an fp32 sum:
// about 1.5 vector instructions per weight.  The offset 128 and the zero point leave through the chunk's activation sum:
//   sum_k x (code - zp) = sum_k x (128 + code) - (128 + zp) sum_k x.
// The 128 partial sums of a channel are added in a fixed order (lanes, then the two waves).
// ---------------------------------------------------------------------------------------------
typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
typedef uint32_t u32x4_t __attribute__((ext_vector_type(4)));
__device__ __forceinline__ float dot2_bf16(uint32_t a, uint32_t b, float c)
{
    return __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2_t, a), __builtin_bit_cast(bf16x2_t, b), c, false);
}

// Up to four tensors that read the same token (query | key | value, gate | up) share one launch: tensor i owns the
// workgroups [wg_end[i-1], wg_end[i]).
struct zo_gemv_multi {
    int32_t nt;
    const void* codes[4]; const void* step16[4]; const int16_t* zp[4];
    void* Y[4]; const float* bias[4]; const void* residual[4];
    int32_t wg_end[4];
    const void* X;
    int32_t K, group, relu;
};

template <typename TY>
__global__ __launch_bounds__(128) void zo_int4_gemv_kernel(zo_gemv_multi mt)
{
    constexpr int R = 4;
    __shared__ float red[R];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    int ti = 0, wg0 = 0;
#pragma unroll
    for (int i = 1; i < 4; ++i)
        if (i < mt.nt && (int)blockIdx.x >= mt.wg_end[i - 1]) { ti = i; wg0 = mt.wg_end[i - 1]; }
    struct { const void* codes; const void* step16; const int16_t* zp; void* Y; const float* bias; const void* residual; int relu; } a;
    a.codes = mt.codes[0]; a.step16 = mt.step16[0]; a.zp = mt.zp[0]; a.Y = mt.Y[0]; a.bias = mt.bias[0]; a.residual = mt.residual[0];
#pragma unroll
    for (int i = 1; i < 4; ++i)
        if (ti == i) { a.codes = mt.codes[i]; a.step16 = mt.step16[i]; a.zp = mt.zp[i]; a.Y = mt.Y[i]; a.bias = mt.bias[i]; a.residual = mt.residual[i]; }
    a.relu = mt.relu;
    const int n0 = ((int)blockIdx.x - wg0) * R;
    const int K = mt.K, G = K / mt.group, gshift = __builtin_ctz(mt.group);
    const int chunks = K >> 5;
    const uint8_t* codes = (const uint8_t*)a.codes;
    const _Float16* step16 = (const _Float16*)a.step16;
    const uint4* xv = (const uint4*)mt.X;
    float acc[R];
#pragma unroll
    for (int r = 0; r < R; ++r) acc[r] = 0.0f;
    for (int ci = threadIdx.x; ci < chunks; ci += 128) {
        u32x4_t cw[R];                                     // read once: streaming loads
#pragma unroll
        for (int r = 0; r < R; ++r) cw[r] = __builtin_nontemporal_load((const u32x4_t*)(codes + ((int64_t)(n0 + r) * K >> 1)) + ci);
        uint32_t P[16];
        float sx = 0.0f;
#pragma unroll
        for (int m = 0; m < 4; ++m) {
            const uint4 x4 = xv[ci * 4 + m];               // x[32 ci + 8 m .. + 7] as four bf16 pairs
            P[4 * m + 0] = __builtin_amdgcn_perm(x4.z, x4.x, 0x05040100u);      // (x0, x4)
            P[4 * m + 1] = __builtin_amdgcn_perm(x4.z, x4.x, 0x07060302u);      // (x1, x5)
            P[4 * m + 2] = __builtin_amdgcn_perm(x4.w, x4.y, 0x05040100u);      // (x2, x6)
            P[4 * m + 3] = __builtin_amdgcn_perm(x4.w, x4.y, 0x07060302u);      // (x3, x7)
#pragma unroll
            for (int j = 0; j < 4; ++j) sx = dot2_bf16(P[4 * m + j], 0x3F803F80u, sx);
        }
        const int g = (ci << 5) >> gshift;
#pragma unroll
        for (int r = 0; r < R; ++r) {
            const uint32_t w4[4] = {cw[r][0], cw[r][1], cw[r][2], cw[r][3]};
            float part = 0.0f;
#pragma unroll
            for (int m = 0; m < 4; ++m)
#pragma unroll
                for (int j = 0; j < 4; ++j)
                    part = dot2_bf16(((w4[m] >> (4 * j)) & 0x000F000Fu) | 0x43004300u, P[4 * m + j], part);
            const float st = (float)step16[(int64_t)(n0 + r) * G + g];
            const float zp = (float)a.zp[(int64_t)(n0 + r) * G + g] + 128.0f;
            acc[r] = __builtin_fmaf(st, part - zp * sx, acc[r]);
        }
    }
#pragma unroll
    for (int r = 0; r < R; ++r) acc[r] = zo_group_sum<64>(acc[r]);
    if (wave == 1 && lane == 0) {
#pragma unroll
        for (int r = 0; r < R; ++r) red[r] = acc[r];
    }
    __syncthreads();
    if (wave == 0 && lane < R) {
        const int n = n0 + lane;
        float v = 0.0f;
#pragma unroll
        for (int r = 0; r < R; ++r) v = lane == r ? acc[r] + red[r] : v;
        if (a.bias) v += a.bias[n];
        if (a.relu) v = fmaxf(v, 0.0f);
        if (a.residual) v += (float)((const zo_bf16*)a.residual)[n];
        zo_store((TY*)a.Y + n, v);
    }
}

bool zo_int4_gemv_supported(int32_t M, int32_t nb, int32_t N, int32_t K, int32_t group)
{
    return M == 1 && nb == 1 && N >= 4 && (N & 3) == 0 && K >= 32 && (K & 31) == 0 && group >= 32 && (group & (group - 1)) == 0 && K % group == 0;
}

hipError_t zo_launch_int4_gemv_multi(const zo_fused_args* t, int nt, hipStream_t st)
{
    if (nt < 1 || nt > 4) return hipErrorInvalidValue;
    zo_gemv_multi mt{};
    mt.nt = nt;
    int wgs = 0;
    for (int i = 0; i < nt; ++i) {
        const zo_fused_args& a = t[i];
        if (!zo_int4_gemv_supported(a.M, a.nb, a.N, a.K, a.group) || !a.codes || !a.step16 || !a.zp || !a.X || !a.Y) return hipErrorInvalidValue;
        if (a.K != t[0].K || a.group != t[0].group || a.X != t[0].X || a.relu != t[0].relu || a.out_f32 != t[0].out_f32) return hipErrorInvalidValue;
        mt.codes[i] = a.codes; mt.step16[i] = a.step16; mt.zp[i] = a.zp; mt.Y[i] = a.Y; mt.bias[i] = a.bias; mt.residual[i] = a.residual;
        wgs += a.N / 4;
        mt.wg_end[i] = wgs;
    }
    for (int i = nt; i < 4; ++i) mt.wg_end[i] = wgs;
    mt.X = t[0].X; mt.K = t[0].K; mt.group = t[0].group; mt.relu = t[0].relu;
    if (t[0].out_f32) zo_int4_gemv_kernel<float><<<wgs, 128, 0, st>>>(mt);
    else zo_int4_gemv_kernel<zo_bf16><<<wgs, 128, 0, st>>>(mt);
    return hipGetLastError();
}

hipError_t zo_launch_int4_gemv(const zo_fused_args& a, hipStream_t st) { return zo_launch_int4_gemv_multi(&a, 1, st); }
