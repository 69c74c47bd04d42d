// Kernels of the generator on the quantized model (prompt pass + cached decoding; efficiency section, on-device
// inference): attention of ONE new query over the cached keys / values of a sequence, and the arg max of a row of logits.
#include "zo_device.h"
#include "zo_internal.h"

// One workgroup per head.  scores[j] = q . K[j] / sqrt(dh) for the n cached positions (a thread per key, strided), a
// numerically safe softmax in fp32 (fixed-order reductions: lanes, then the four waves in order), then
// out[i] = sum_j p_j V[j][i] with the keys dealt to 256 / dh thread groups whose partial sums are added in group order.
template <typename T>
__global__ __launch_bounds__(256) void zo_decode_attention_kernel(const T* __restrict__ q, const T* __restrict__ Kc, const T* __restrict__ Vc,
                                                                  T* __restrict__ out, int n, int d, int dh, float scale)
{
    extern __shared__ float sm[];                     // [n] scores, then [dh] query, then [256] reduction scratch
    float* sc = sm;
    float* qs = sm + n;
    float* red = qs + dh;
    const int h = blockIdx.x, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int64_t hoff = (int64_t)h * dh;
    for (int i = tid; i < dh; i += 256) qs[i] = zo_load(q + hoff + i);
    __syncthreads();
    float mx = -INFINITY;
    for (int j = tid; j < n; j += 256) {
        const T* kr = Kc + (int64_t)j * d + hoff;
        float acc = 0.0f;
        for (int i = 0; i < dh; i += 8) {
            float v[8];
            zo_load8(kr + i, v);
#pragma unroll
            for (int e = 0; e < 8; ++e) acc = __builtin_fmaf(v[e], qs[i + e], acc);
        }
        acc *= scale;
        sc[j] = acc;
        mx = fmaxf(mx, acc);
    }
    mx = zo_group_max<64>(mx);
    if (lane == 0) red[wave] = mx;
    __syncthreads();
    mx = fmaxf(fmaxf(red[0], red[1]), fmaxf(red[2], red[3]));
    __syncthreads();
    float sum = 0.0f;
    for (int j = tid; j < n; j += 256) {
        const float p = __expf(sc[j] - mx);
        sc[j] = p;
        sum += p;
    }
    sum = zo_group_sum<64>(sum);
    if (lane == 0) red[wave] = sum;
    __syncthreads();
    sum = ((red[0] + red[1]) + red[2]) + red[3];
    __syncthreads();
    const int parts = 256 / dh, i = tid % dh, part = tid / dh;      // dh in {16, 32, 64, 128}
    float o = 0.0f;
    for (int j = part; j < n; j += parts) o = __builtin_fmaf(sc[j], zo_load(Vc + (int64_t)j * d + hoff + i), o);
    red[tid] = o;
    __syncthreads();
    if (tid < dh) {
        float t = red[tid];
        for (int p2 = 1; p2 < parts; ++p2) t += red[p2 * dh + tid];
        zo_store(out + hoff + tid, t / sum);
    }
}

hipError_t zo_launch_decode_attention(const void* q, const void* Kc, const void* Vc, void* out, int32_t n, int32_t H, int32_t dh,
                                      int dtype, hipStream_t st)
{
    if (n <= 0 || H <= 0 || (dh != 16 && dh != 32 && dh != 64 && dh != 128)) return hipErrorInvalidValue;
    const int d = H * dh;
    const size_t lds = ((size_t)n + dh + 256) * sizeof(float);
    if (lds > 160 * 1024) return hipErrorInvalidValue;
    const float scale = 1.0f / sqrtf((float)dh);
    if (dtype == ZO_T_BF16) {
        if (lds > 64 * 1024) {
            hipError_t e = hipFuncSetAttribute((const void*)zo_decode_attention_kernel<zo_bf16>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
            if (e != hipSuccess) return e;
        }
        zo_decode_attention_kernel<zo_bf16><<<H, 256, lds, st>>>((const zo_bf16*)q, (const zo_bf16*)Kc, (const zo_bf16*)Vc, (zo_bf16*)out, n, d, dh, scale);
    } else {
        if (lds > 64 * 1024) {
            hipError_t e = hipFuncSetAttribute((const void*)zo_decode_attention_kernel<float>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
            if (e != hipSuccess) return e;
        }
        zo_decode_attention_kernel<float><<<H, 256, lds, st>>>((const float*)q, (const float*)Kc, (const float*)Vc, (float*)out, n, d, dh, scale);
    }
    return hipGetLastError();
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
