// Fused form of the fake-quantized linear for small token counts (M <= 128): one pass over the fp32
// master matrix builds the tiles of Q(W + eps u) and Q(W - eps u) (Eq. 2) in registers, straight in
// matrix-core operand layout, and multiplies them with the two branches' activations.  Neither the
// perturbed nor the de-quantized weights ever reach LDS or HBM: traffic is 4 B per parameter.
//
// Work split (gfx950, wave64, v_mfma_f32_16x16x32_bf16):
//   workgroup = 16 output channels x all of K, 8 waves; wave w takes the K slabs w, w+8, ...
//   slab = 32*CH input features; lane (n = lane % 16, q = lane / 16) owns CH consecutive Philox
//   blocks (8 features each) of channel n, i.e. CH*32 contiguous bytes of W.  A quantization group
//   of g = 8*CH*GL features is GL neighbouring q lanes (cross-lane min/max).  The lane's de-quantized
//   block c is operand A of matrix instruction c of the slab as it stands; the activations are
//   fetched in the matching order (lane (m, q) reads X[m][slab + (q*CH + c)*8 ...]), so the
//   instruction's summation index is a permutation of k inside the slab -- the sum is the same.
//   The eight partial accumulators of a tile are added in wave order through LDS (fixed order, no
//   atomics), then bias / ReLU / residual and a single rounding.
// The tile build is plain-ALU work (the perturbation stream, two branches of range / code /
// de-quantize: ~65 lane-instructions per parameter), which bounds this kernel; at large M the
// same build would be repeated per m-tile, which is why the large-M path quantizes once instead.
#include "zo_device.h"
#include "zo_internal.h"

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

namespace {

constexpr int FW = 8;            // waves per workgroup

template <int GL> ZO_DEV float q_min(float v)
{
    if (GL >= 2) v = fminf(v, __shfl_xor(v, 16, 64));
    if (GL >= 4) v = fminf(v, __shfl_xor(v, 32, 64));
    return v;
}
template <int GL> ZO_DEV float q_max(float v)
{
    if (GL >= 2) v = fmaxf(v, __shfl_xor(v, 16, 64));
    if (GL >= 4) v = fmaxf(v, __shfl_xor(v, 32, 64));
    return v;
}

ZO_DEV bf16x8 pack8(const float o[8])
{
    typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
    u32x4 p = {zo_pack_bf16x2(o[0], o[1]), zo_pack_bf16x2(o[2], o[3]), zo_pack_bf16x2(o[4], o[5]), zo_pack_bf16x2(o[6], o[7])};
    return __builtin_bit_cast(bf16x8, p);
}

// One branch of the tile build for the lane's CH blocks: v = fma(se, z, w), group range over the lane's
// values and its GL - 1 neighbours, code, de-quantize, round to bf16.
template <int CH, int GL>
ZO_DEV void build_branch(const float (&w)[CH][8], const float (&z)[CH][8], float se, int bits, bf16x8 (&af)[CH])
{
    float v[CH][8];
#pragma unroll
    for (int c = 0; c < CH; ++c)
#pragma unroll
        for (int i = 0; i < 8; ++i) v[c][i] = __builtin_fmaf(se, z[c][i], w[c][i]);
    if (bits != 0) {
        float mn = v[0][0], mx = v[0][0];
#pragma unroll
        for (int c = 0; c < CH; ++c)
#pragma unroll
            for (int i = 0; i < 8; ++i) { mn = fminf(mn, v[c][i]); mx = fmaxf(mx, v[c][i]); }
        mn = q_min<GL>(mn);
        mx = q_max<GL>(mx);
        const zo_qparams qp = zo_qparams_asym(mn, mx, bits);
#pragma unroll
        for (int c = 0; c < CH; ++c)
#pragma unroll
            for (int i = 0; i < 8; ++i) v[c][i] = zo_dequant(qp, zo_code(qp, v[c][i]));
    }
#pragma unroll
    for (int c = 0; c < CH; ++c) af[c] = pack8(v[c]);
}

template <int CH, int GL, int J>
__global__ __launch_bounds__(FW * 64) void zo_fq_gemm_fused_kernel(zo_fused_args a, zo_stream s)
{
    extern __shared__ __attribute__((aligned(16))) unsigned char lds_raw[];
    f32x4* red = reinterpret_cast<f32x4*>(lds_raw);          // [FW][2 * J][64]
    constexpr int SLAB = 32 * CH;
    const int lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int n = lane & 15, q = lane >> 4;
    const int M = a.M, K = a.K, nb = a.nb;
    const int n0 = blockIdx.x * 16;
    const int nslab = K / SLAB;
    const int jn = (M + 15) >> 4;                             // m-tiles in use (<= J)
    const float* wrow = a.W + (int64_t)(n0 + n) * K + q * (CH * 8);
    const uint64_t blk_row = ((uint64_t)(n0 + n) * (uint64_t)K >> 3) + (uint64_t)(q * CH);
    const zo_bf16* X = (const zo_bf16*)a.X;

    f32x4 acc[2][J];
#pragma unroll
    for (int b = 0; b < 2; ++b)
#pragma unroll
        for (int j = 0; j < J; ++j) acc[b][j] = f32x4{0.0f, 0.0f, 0.0f, 0.0f};

    for (int sl = wave; sl < nslab; sl += FW) {
        const int k0 = sl * SLAB;
        float w[CH][8], z[CH][8];
#pragma unroll
        for (int c = 0; c < CH; ++c) zo_load8(wrow + k0 + c * 8, w[c]);
        if (a.eps != 0.0f) {
#pragma unroll
            for (int c = 0; c < CH; ++c) zo_z8(s, blk_row + (uint64_t)(k0 >> 3) + c, z[c]);
        } else {
#pragma unroll
            for (int c = 0; c < CH; ++c)
#pragma unroll
                for (int i = 0; i < 8; ++i) z[c][i] = 0.0f;
        }
        bf16x8 af[2][CH];
        build_branch<CH, GL>(w, z, a.eps, a.bits, af[0]);
        if (nb == 2) build_branch<CH, GL>(w, z, -a.eps, a.bits, af[1]);
#pragma unroll
        for (int j = 0; j < J; ++j) {
            if (j < jn) {
                int m = j * 16 + n;
                m = m < M ? m : M - 1;
                const zo_bf16* xr = X + (int64_t)m * K + k0 + q * (CH * 8);
#pragma unroll
                for (int b = 0; b < 2; ++b) {
                    if (b < nb) {
#pragma unroll
                        for (int c = 0; c < CH; ++c) {
                            const bf16x8 xf = *reinterpret_cast<const bf16x8*>(xr + b * a.strideX + c * 8);
                            acc[b][j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(af[b][c], xf, acc[b][j], 0, 0, 0);
                        }
                    }
                }
            }
        }
    }

    // partial accumulators -> LDS, then tile t = b * J + j is summed over the waves in order by wave t % FW
#pragma unroll
    for (int b = 0; b < 2; ++b)
#pragma unroll
        for (int j = 0; j < J; ++j)
            if (b < nb && j < jn) red[((wave * 2 + b) * J + j) * 64 + lane] = acc[b][j];
    __syncthreads();
    for (int t = wave; t < 2 * J; t += FW) {
        const int b = t / J, j = t % J;
        if (b >= nb || j >= jn) continue;
        f32x4 v = red[((0 * 2 + b) * J + j) * 64 + lane];
        for (int wv = 1; wv < FW; ++wv) {
            const f32x4 p = red[((wv * 2 + b) * J + j) * 64 + lane];
            v[0] += p[0]; v[1] += p[1]; v[2] += p[2]; v[3] += p[3];
        }
        // lane holds outputs (m, n0 + 4 q .. + 3)
        const int m = j * 16 + n;
        if (m >= M) continue;
        const int nn = n0 + 4 * q;
        if (a.bias) {
            const float4 b4 = *reinterpret_cast<const float4*>(a.bias + b * a.strideBias + nn);
            v[0] += b4.x; v[1] += b4.y; v[2] += b4.z; v[3] += b4.w;
        }
        if (a.relu) {
#pragma unroll
            for (int e = 0; e < 4; ++e) v[e] = fmaxf(v[e], 0.0f);
        }
        const int64_t off = (int64_t)m * a.ldY + nn;
        if (a.residual) {
            const uint2 r2 = *reinterpret_cast<const uint2*>((const zo_bf16*)a.residual + b * a.strideRes + off);
            v[0] += zo_bf16_lo(r2.x); v[1] += zo_bf16_hi(r2.x);
            v[2] += zo_bf16_lo(r2.y); v[3] += zo_bf16_hi(r2.y);
        }
        if (a.out_f32) {
            *reinterpret_cast<float4*>((float*)a.Y + b * a.strideY + off) = make_float4(v[0], v[1], v[2], v[3]);
        } else {
            uint2 o;
            o.x = zo_pack_bf16x2(v[0], v[1]);
            o.y = zo_pack_bf16x2(v[2], v[3]);
            *reinterpret_cast<uint2*>((zo_bf16*)a.Y + b * a.strideY + off) = o;
        }
    }
}

template <int CH, int GL>
hipError_t launch_j(const zo_fused_args& a, const zo_stream& s, hipStream_t st)
{
    const dim3 grid(a.N / 16);
    if (a.M <= 32) {
        constexpr int lds = FW * 2 * 2 * 1024;
        zo_fq_gemm_fused_kernel<CH, GL, 2><<<grid, FW * 64, lds, st>>>(a, s);
    } else {
        constexpr int lds = FW * 2 * 8 * 1024;
        hipError_t e = hipFuncSetAttribute((const void*)zo_fq_gemm_fused_kernel<CH, GL, 8>, hipFuncAttributeMaxDynamicSharedMemorySize, lds);
        if (e != hipSuccess) return e;
        zo_fq_gemm_fused_kernel<CH, GL, 8><<<grid, FW * 64, lds, st>>>(a, s);
    }
    return hipGetLastError();
}

}  // namespace

bool zo_fused_supported(int32_t M, int32_t N, int32_t K, int32_t bits, int32_t group)
{
    if (M < 1 || M > ZO_FUSED_MAX_M || N < 16 || (N & 15) || K < 32 || (K & 31)) return false;
    if (bits == 0) return true;
    if (bits < 1 || bits > 8) return false;
    if (group != 8 && group != 16 && group != 32 && group != 64 && group != 128) return false;
    return K % group == 0;
}

hipError_t zo_launch_fq_gemm_fused(const zo_fused_args& a, uint64_t seed, int32_t tid, hipStream_t st)
{
    if (!zo_fused_supported(a.M, a.N, a.K, a.bits, a.group) || (a.nb != 1 && a.nb != 2) || (a.ldY & 3)) return hipErrorInvalidValue;
    zo_stream s;
    s.k0 = (uint32_t)seed;
    s.k1 = (uint32_t)(seed >> 32);
    s.tensor_id = (uint32_t)tid;
    if (a.bits == 0) return launch_j<1, 1>(a, s, st);
    switch (a.group) {
        case 8:   return launch_j<1, 1>(a, s, st);
        case 16:  return launch_j<1, 2>(a, s, st);
        case 32:  return launch_j<1, 4>(a, s, st);
        case 64:  return launch_j<2, 4>(a, s, st);
        default:  return launch_j<4, 4>(a, s, st);
    }
}
