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

// ---------------------------------------------------------------------------------------------
// The same attention in two launches that fill the chip and do the bookkeeping of a decoding step on the way.
// Launch 1, one workgroup per (range of cached rows, head): the new row's query and key are rotated here (same
// arithmetic and rounding as the stand-alone rotary kernel; ROPE = false for learned positions), the workgroup of the last
// range appends the new key / value row to the cache and attends to it from registers; every row group runs a streaming
// softmax over its rows (four rows' loads in flight), the groups are merged in group order, and the workgroup leaves
// (maximum, sum of exponentials, un-normalised output) of its range.  Launch 2, one workgroup: merges the ranges of every
// head in range order, rounds the attention output to the storage type, and -- the row now sitting in registers --
// applies the per-token quantizer of the attention-output projection's input (same arithmetic as the stand-alone one).
// ---------------------------------------------------------------------------------------------
template <typename T, int LPK, bool ROPE>
__global__ __launch_bounds__(256) void zo_decode_attn_part_kernel(const T* __restrict__ qkv, T* __restrict__ Kc, T* __restrict__ Vc,
                                                                  const float* __restrict__ cosr, const float* __restrict__ sinr,
                                                                  float* __restrict__ po, float* __restrict__ ml, int n, int d, int rps,
                                                                  float scale)
{
    constexpr int DH = LPK * 8, KG = 256 / LPK, HL = LPK / 2;
    __shared__ float gm[KG], gl[KG];
    __shared__ float part[KG * DH];
    const int s = blockIdx.x, KS = gridDim.x, h = blockIdx.y, tid = threadIdx.x;
    const int sub = tid % LPK, kg = tid / LPK;
    const int64_t hbase = (int64_t)h * DH, hoff = hbase + sub * 8;
    float cs[8], sn[8];
    const bool first = sub < HL;
    if (ROPE) {
        zo_load8(cosr + (sub % HL) * 8, cs);
        zo_load8(sinr + (sub % HL) * 8, sn);
    }
    auto rotated = [&](const T* row, float out[8]) {
        zo_load8(row + hoff, out);
        if (ROPE) {
            float oth[8];
            zo_load8(row + hbase + (sub ^ HL) * 8, oth);
#pragma unroll
            for (int e = 0; e < 8; ++e)
                out[e] = zo_round_to<T>(first ? __builtin_fmaf(out[e], cs[e], -(oth[e] * sn[e])) : __builtin_fmaf(out[e], cs[e], oth[e] * sn[e]));
        }
    };
    float qv[8];
    rotated(qkv, qv);
    const int r0 = s * rps;
    const int r1 = r0 + rps < n ? r0 + rps : n;
    const int rc = r1 < n - 1 ? r1 : n - 1;              // cached rows of this range: [r0, rc); row n - 1 is the new one
    float m = -INFINITY, l = 0.0f, o[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) o[e] = 0.0f;
    auto absorb = [&](const float (&sc)[4], const float (&vv)[4][8]) {
        const float mnew = fmaxf(fmaxf(fmaxf(sc[0], sc[1]), fmaxf(sc[2], sc[3])), m);
        const float corr = __expf(m - mnew);             // 0 the first time (m = -inf, mnew finite)
        l *= corr;
#pragma unroll
        for (int e = 0; e < 8; ++e) o[e] *= corr;
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const float pr = __expf(sc[u] - mnew);        // 0 for a row that does not exist (score -inf)
            l += pr;
#pragma unroll
            for (int e = 0; e < 8; ++e) o[e] = __builtin_fmaf(pr, vv[u][e], o[e]);
        }
        m = mnew;
    };
    for (int j0 = r0 + kg; j0 < rc; j0 += 4 * KG) {
        float kv[4][8], vv[4][8], sc[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const int j = j0 + u * KG < rc ? j0 + u * KG : j0;
            zo_load8(Kc + (int64_t)j * d + hoff, kv[u]);
            zo_load8(Vc + (int64_t)j * d + hoff, vv[u]);
        }
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            float acc = 0.0f;
#pragma unroll
            for (int e = 0; e < 8; ++e) acc = __builtin_fmaf(kv[u][e], qv[e], acc);
            acc = zo_group_sum<LPK>(acc) * scale;
            sc[u] = j0 + u * KG < rc ? acc : -INFINITY;
        }
        absorb(sc, vv);
    }
    if (r1 == n) {
        // the new row: every row group computes its score (no divergence around the lane exchanges), the group whose turn
        // it is stores it into the cache and counts it
        const bool mine = kg == (n - 1 - r0) % KG;
        float kn[8], vv[4][8], sc[4] = {-INFINITY, -INFINITY, -INFINITY, -INFINITY};
        rotated(qkv + d, kn);
        zo_load8(qkv + 2 * (int64_t)d + hoff, vv[0]);
#pragma unroll
        for (int u = 1; u < 4; ++u)
#pragma unroll
            for (int e = 0; e < 8; ++e) vv[u][e] = 0.0f;
        float acc = 0.0f;
#pragma unroll
        for (int e = 0; e < 8; ++e) acc = __builtin_fmaf(kn[e], qv[e], acc);
        acc = zo_group_sum<LPK>(acc) * scale;
        if (mine) {
            zo_store8(Kc + (int64_t)(n - 1) * d + hoff, kn);
            zo_store8(Vc + (int64_t)(n - 1) * d + hoff, vv[0]);
            sc[0] = acc;
            absorb(sc, vv);
        }
    }
    if (sub == 0) { gm[kg] = m; gl[kg] = l; }
    __syncthreads();
    float mx = gm[0];
    for (int g = 1; g < KG; ++g) mx = fmaxf(mx, gm[g]);
    const float w = __expf(m - mx);                       // a group without rows: m = -inf, weight 0
#pragma unroll
    for (int e = 0; e < 8; ++e) part[kg * DH + sub * 8 + e] = o[e] * w;
    __syncthreads();
    const int64_t slot = (int64_t)h * KS + s;
    if (tid < DH) {
        float t = part[tid];
        for (int g = 1; g < KG; ++g) t += part[g * DH + tid];
        po[slot * DH + tid] = t;
    }
    if (tid == 0) {
        float lt = 0.0f;
        for (int g = 0; g < KG; ++g) lt += gl[g] * __expf(gm[g] - mx);
        ml[slot * 2] = mx;
        ml[slot * 2 + 1] = lt;
    }
}

// launch 2 (see above); 1024 lanes, NC chunks of 8192 columns, a lane's 8 columns lie in one head
template <typename T, int NC>
__global__ __launch_bounds__(1024) void zo_decode_attn_merge_kernel(const float* __restrict__ po, const float* __restrict__ ml, int KS, int H, int dh,
                                                                    T* __restrict__ att, T* __restrict__ xhat, int bits, int sym,
                                                                    const float* __restrict__ sm_delta, const float* __restrict__ sm_inv)
{
    __shared__ float wgt[512];                          // weight of (head, range): exp(m - head maximum) / head sum
    __shared__ float lsum[512];
    __shared__ float red[2][16];
    const int cols = H * dh, tid = threadIdx.x;
    if (tid < H * KS) { wgt[tid] = ml[tid * 2]; lsum[tid] = ml[tid * 2 + 1]; }
    __syncthreads();
    float mxh = 0.0f, inv = 0.0f;
    if (tid < H) {
        mxh = wgt[tid * KS];
        for (int s = 1; s < KS; ++s) mxh = fmaxf(mxh, wgt[tid * KS + s]);
        float lt = 0.0f;
        for (int s = 0; s < KS; ++s) lt += lsum[tid * KS + s] * __expf(wgt[tid * KS + s] - mxh);
        inv = 1.0f / lt;
    }
    __syncthreads();
    if (tid < H)
        for (int s = 0; s < KS; ++s) wgt[tid * KS + s] = __expf(wgt[tid * KS + s] - mxh) * inv;
    __syncthreads();
    float v[NC][8];
    float mn = INFINITY, mx = -INFINITY;
#pragma unroll
    for (int i = 0; i < NC; ++i) {
        const int c = tid * 8 + 8192 * i;
        if (c < cols) {
            const int h = c / dh, col = c - h * dh;
            float o[8];
#pragma unroll
            for (int e = 0; e < 8; ++e) o[e] = 0.0f;
            for (int s0 = 0; s0 < KS; s0 += 4) {          // four ranges' loads in flight
                float t[4][8], w[4];
#pragma unroll
                for (int u = 0; u < 4; ++u) {
                    const int s = s0 + u < KS ? s0 + u : s0;
                    zo_load8(po + ((int64_t)h * KS + s) * dh + col, t[u]);
                    w[u] = s0 + u < KS ? wgt[h * KS + s] : 0.0f;
                }
#pragma unroll
                for (int u = 0; u < 4; ++u)
#pragma unroll
                    for (int e = 0; e < 8; ++e) o[e] = __builtin_fmaf(w[u], t[u][e], o[e]);
            }
#pragma unroll
            for (int e = 0; e < 8; ++e) v[i][e] = zo_round_to<T>(o[e]);
            zo_store8(att + c, v[i]);
            if (xhat) {
                float dl[8], iv[8];
                if (sm_delta) { zo_load8(sm_delta + c, dl); zo_load8(sm_inv + c, iv); }
#pragma unroll
                for (int e = 0; e < 8; ++e) {
                    if (sm_delta) v[i][e] = (v[i][e] - dl[e]) * iv[e];
                    if (sym) mx = fmaxf(mx, fabsf(v[i][e]));
                    else { mn = fminf(mn, v[i][e]); mx = fmaxf(mx, v[i][e]); }
                }
            }
        }
    }
    if (!xhat) return;
    mn = zo_group_min<64>(mn);
    mx = zo_group_max<64>(mx);
    if ((tid & 63) == 0) { red[0][tid >> 6] = mn; red[1][tid >> 6] = mx; }
    __syncthreads();
    mn = red[0][0];
    mx = red[1][0];
#pragma unroll
    for (int w = 1; w < 16; ++w) { mn = fminf(mn, red[0][w]); mx = fmaxf(mx, red[1][w]); }
    const zo_qparams q = sym ? zo_qparams_sym(mx, bits) : zo_qparams_asym(mn, mx, bits);
#pragma unroll
    for (int i = 0; i < NC; ++i) {
        const int c = tid * 8 + 8192 * i;
        if (c < cols) {
            float o[8];
#pragma unroll
            for (int e = 0; e < 8; ++e) o[e] = zo_dequant(q, zo_code(q, v[i][e]));
            zo_store8(xhat + c, o);
        }
    }
}

// Ranges of cached rows per head: enough workgroups for two per CU, at least two rounds of row groups per range.
static int decode_attn_rows_per_range(int n, int H, int dh)
{
    const int kg = 256 / (dh / 8);
    int ks_max = 512 / H;
    ks_max = ks_max < 1 ? 1 : (ks_max > 16 ? 16 : ks_max);
    int rps = (n + ks_max - 1) / ks_max;
    rps = (rps + kg - 1) / kg * kg;
    return rps < 2 * kg ? 2 * kg : rps;
}

bool zo_decode_attention_split_supported(int32_t H, int32_t dh)
{
    return H >= 1 && H <= 256 && (dh == 16 || dh == 32 || dh == 64 || dh == 128) && H * dh <= 16384;
}

size_t zo_decode_attention_split_bytes(int32_t n, int32_t H, int32_t dh)
{
    const int rps = decode_attn_rows_per_range(n, H, dh);
    const int ks = (n + rps - 1) / rps;
    return (size_t)H * ks * (dh + 2) * sizeof(float);
}

template <typename T>
static hipError_t launch_decode_attention_split_t(const T* qkv, T* Kc, T* Vc, const float* cosr, const float* sinr, float* scratch, T* att,
                                                  T* xhat, int n, int H, int dh, int bits, int sym, const float* sm_delta,
                                                  const float* sm_inv, hipStream_t st)
{
    const int d = H * dh;
    const int rps = decode_attn_rows_per_range(n, H, dh);
    const int ks = (n + rps - 1) / rps;
    float* po = scratch;
    float* ml = scratch + (size_t)H * ks * dh;
    const float scale = 1.0f / sqrtf((float)dh);
    const dim3 grid(ks, H);
#define ZO_DEC_PART(L)                                                                                                                   \
    do {                                                                                                                                 \
        if (cosr) zo_decode_attn_part_kernel<T, L, true><<<grid, 256, 0, st>>>(qkv, Kc, Vc, cosr, sinr, po, ml, n, d, rps, scale);       \
        else zo_decode_attn_part_kernel<T, L, false><<<grid, 256, 0, st>>>(qkv, Kc, Vc, cosr, sinr, po, ml, n, d, rps, scale);           \
    } while (0)
    switch (dh) {
        case 16:  ZO_DEC_PART(2); break;
        case 32:  ZO_DEC_PART(4); break;
        case 64:  ZO_DEC_PART(8); break;
        default:  ZO_DEC_PART(16); break;
    }
#undef ZO_DEC_PART
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
#define ZO_DEC_MERGE(NC) zo_decode_attn_merge_kernel<T, NC><<<1, 1024, 0, st>>>(po, ml, ks, H, dh, att, xhat, bits, sym, sm_delta, sm_inv)
    if (d <= 8192) ZO_DEC_MERGE(1); else ZO_DEC_MERGE(2);
#undef ZO_DEC_MERGE
    return hipGetLastError();
}

// qkv: the new row (q | k | v, 3 H dh elements; q and k not yet rotated); Kc / Vc: this layer's cache, row n - 1 is written;
// cos_row / sin_row: the rotary table's row of position n - 1, or NULL (no rotation); scratch: zo_decode_attention_split_bytes;
// att: the attention output row; xhat: its per-token-quantized copy, or NULL.
hipError_t zo_launch_decode_attention_split(const void* qkv, void* Kc, void* Vc, const float* cos_row, const float* sin_row, void* scratch,
                                            void* att, void* xhat, int32_t n, int32_t H, int32_t dh, int32_t bits, int32_t sym,
                                            const float* sm_delta, const float* sm_inv, int dtype, hipStream_t st)
{
    if (n <= 0 || !zo_decode_attention_split_supported(H, dh) || (cos_row == nullptr) != (sin_row == nullptr)) return hipErrorInvalidValue;
    if (dtype == ZO_T_BF16)
        return launch_decode_attention_split_t<zo_bf16>((const zo_bf16*)qkv, (zo_bf16*)Kc, (zo_bf16*)Vc, cos_row, sin_row, (float*)scratch,
                                                        (zo_bf16*)att, (zo_bf16*)xhat, n, H, dh, bits, sym, sm_delta, sm_inv, st);
    return launch_decode_attention_split_t<float>((const float*)qkv, (float*)Kc, (float*)Vc, cos_row, sin_row, (float*)scratch, (float*)att,
                                                  (float*)xhat, n, H, dh, bits, sym, sm_delta, sm_inv, st);
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

template <typename TY, int U>
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
    // U chunks per lane and round, all their loads requested before the first is used (a chunk past the end repeats the
    // lane's first chunk and is weighted 0)
    for (int c0 = threadIdx.x; c0 < chunks; c0 += 128 * U) {
        u32x4_t cw[U][R];                                  // read once: streaming loads
        uint4 xr[U][4];
        float st[U][R], zq[U][R];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const bool ok = c0 + 128 * u < chunks;
            const int ci = ok ? c0 + 128 * u : c0;
            const int g = (ci << 5) >> gshift;
#pragma unroll
            for (int r = 0; r < R; ++r) {
                cw[u][r] = __builtin_nontemporal_load((const u32x4_t*)(codes + ((int64_t)(n0 + r) * K >> 1)) + ci);
                st[u][r] = ok ? (float)step16[(int64_t)(n0 + r) * G + g] : 0.0f;
                zq[u][r] = (float)a.zp[(int64_t)(n0 + r) * G + g] + 128.0f;
            }
#pragma unroll
            for (int m = 0; m < 4; ++m) xr[u][m] = xv[ci * 4 + m];      // x[32 ci + 8 m .. + 7] as four bf16 pairs
        }
#pragma unroll
        for (int u = 0; u < U; ++u) {
            uint32_t P[16];
            float sx = 0.0f;
#pragma unroll
            for (int m = 0; m < 4; ++m) {
                const uint4 x4 = xr[u][m];
                P[4 * m + 0] = __builtin_amdgcn_perm(x4.z, x4.x, 0x05040100u);      // (x0, x4)
                P[4 * m + 1] = __builtin_amdgcn_perm(x4.z, x4.x, 0x07060302u);      // (x1, x5)
                P[4 * m + 2] = __builtin_amdgcn_perm(x4.w, x4.y, 0x05040100u);      // (x2, x6)
                P[4 * m + 3] = __builtin_amdgcn_perm(x4.w, x4.y, 0x07060302u);      // (x3, x7)
#pragma unroll
                for (int j = 0; j < 4; ++j) sx = dot2_bf16(P[4 * m + j], 0x3F803F80u, sx);
            }
#pragma unroll
            for (int r = 0; r < R; ++r) {
                const uint32_t w4[4] = {cw[u][r][0], cw[u][r][1], cw[u][r][2], cw[u][r][3]};
                float part = 0.0f;
#pragma unroll
                for (int m = 0; m < 4; ++m)
#pragma unroll
                    for (int j = 0; j < 4; ++j)
                        part = dot2_bf16(((w4[m] >> (4 * j)) & 0x000F000Fu) | 0x43004300u, P[4 * m + j], part);
                acc[r] = __builtin_fmaf(st[u][r], part - zq[u][r] * sx, acc[r]);
            }
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
    const int chunks = mt.K >> 5;
#define ZO_GEMV(U)                                                                                    \
    do {                                                                                              \
        if (t[0].out_f32) zo_int4_gemv_kernel<float, U><<<wgs, 128, 0, st>>>(mt);                     \
        else zo_int4_gemv_kernel<zo_bf16, U><<<wgs, 128, 0, st>>>(mt);                                \
    } while (0)
    // (requesting two or three chunks per lane at once measured slower on the long rows of the down projection: 13.9 against
    // 10.7 us at K = 11008 -- the lanes then all compute at the same time instead of staggered behind one another's loads)
    (void)chunks;
    ZO_GEMV(1);
#undef ZO_GEMV
    return hipGetLastError();
}

hipError_t zo_launch_int4_gemv(const zo_fused_args& a, hipStream_t st) { return zo_launch_int4_gemv_multi(&a, 1, st); }
