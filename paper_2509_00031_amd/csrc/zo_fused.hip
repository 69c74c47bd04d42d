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

template <typename TW, int CH, int GL, int J>
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
    // All J m-tiles are always computed (rows past M repeat row M - 1 and are never stored): the matrix
    // instructions sit in straight-line code, with no data-dependent branch between them and their readers.
    const TW* wrow = (const TW*)a.W + (int64_t)(n0 + n) * K + q * (CH * 8);
    const uint64_t blk_row = ((uint64_t)(n0 + n) * (uint64_t)K >> 3) + (uint64_t)(q * CH);
    const zo_bf16* X = (const zo_bf16*)a.X;

    f32x4 acc[2][J];
#pragma unroll
    for (int b = 0; b < 2; ++b)
#pragma unroll
        for (int j = 0; j < J; ++j) acc[b][j] = f32x4{0.0f, 0.0f, 0.0f, 0.0f};

    // Per slab: the activation fragments of a branch are requested before that branch's tile build (a few
    // thousand ALU cycles), so they have landed when its matrix instructions are issued; the master
    // weights of the next slab are requested one slab ahead.  Tiles beyond JP are fetched on the spot.
    constexpr int JPMAX = CH == 4 ? (J == 8 ? 1 : 2) : 8;                  // m-tiles whose fragments are preloaded (<= 64 VGPRs)
    constexpr int JP = JPMAX < J ? JPMAX : J;
    constexpr bool WPF = CH < 4;                             // register budget: no look-ahead with 32 features per lane
    float w[CH][8], wnext[WPF ? CH : 1][8];
    if (WPF && wave < nslab) {
#pragma unroll
        for (int c = 0; c < CH; ++c) zo_load8(wrow + wave * SLAB + c * 8, w[c]);
    }
    for (int sl = wave; sl < nslab; sl += FW) {
        const int k0 = sl * SLAB;
        const zo_bf16* xcol = X + k0 + q * (CH * 8);
        int mrow[J];
#pragma unroll
        for (int j = 0; j < J; ++j) {
            const int m = j * 16 + n;
            mrow[j] = m < M ? m : M - 1;
        }
        bf16x8 xf[JP][CH];
        // fragment (b, j, c) of this slab: gathered from the row-major activations (16 bytes of 16 different rows
        // per q), or, if the caller re-laid them out fragment by fragment, one contiguous 1 KB wave-level load
        const zo_bf16* xfrag = a.Xfrag ? (const zo_bf16*)a.Xfrag + ((int64_t)sl * J * CH * 64 + lane) * 8 : nullptr;
        auto fragment = [&](int b, int j, int c) -> bf16x8 {
            if (xfrag) return *reinterpret_cast<const bf16x8*>(xfrag + b * a.strideXfrag + (j * CH + c) * 512);
            return *reinterpret_cast<const bf16x8*>(xcol + b * a.strideX + (int64_t)mrow[j] * K + c * 8);
        };
        auto preload = [&](int b) {
#pragma unroll
            for (int j = 0; j < JP; ++j)
#pragma unroll
                for (int c = 0; c < CH; ++c) xf[j][c] = fragment(b, j, c);
        };
        auto contract = [&](int b, const bf16x8 (&af)[CH], f32x4 (&ac)[J]) {
#pragma unroll
            for (int j = 0; j < J; ++j)
#pragma unroll
                for (int c = 0; c < CH; ++c) {
                    const bf16x8 x = j < JP ? xf[j][c] : fragment(b, j, c);
                    ac[j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(af[c], x, ac[j], 0, 0, 0);
                }
        };
        preload(0);
        if constexpr (WPF) {
            if (sl + FW < nslab) {
#pragma unroll
                for (int c = 0; c < CH; ++c) zo_load8(wrow + k0 + FW * SLAB + c * 8, wnext[c]);
            }
        } else {
#pragma unroll
            for (int c = 0; c < CH; ++c) zo_load8(wrow + k0 + c * 8, w[c]);
        }
        __builtin_amdgcn_sched_barrier(0);
        float z[CH][8];
        if (a.eps != 0.0f) {
#pragma unroll
            for (int c = 0; c < CH; ++c) zo_z8(s, blk_row + (uint64_t)(k0 >> 3) + c, z[c]);
        } else {
#pragma unroll
            for (int c = 0; c < CH; ++c)
#pragma unroll
                for (int i = 0; i < 8; ++i) z[c][i] = 0.0f;
        }
        bf16x8 af[CH];
        build_branch<CH, GL>(w, z, a.eps, a.bits, af);
        __builtin_amdgcn_sched_barrier(0);
        contract(0, af, acc[0]);
        if (nb == 2) {
            __builtin_amdgcn_sched_barrier(0);
            preload(1);
            __builtin_amdgcn_sched_barrier(0);
            build_branch<CH, GL>(w, z, -a.eps, a.bits, af);
            __builtin_amdgcn_sched_barrier(0);
            contract(1, af, acc[1]);
        }
        if constexpr (WPF) {
#pragma unroll
            for (int c = 0; c < CH; ++c)
#pragma unroll
                for (int i = 0; i < 8; ++i) w[c][i] = wnext[c][i];
        }
    }

    // The accumulators are read next.  The compiler inserts the wait states between a matrix instruction and a
    // reader of its result; an earlier form of this loop, with the instructions of a tile under a run-time
    // condition and the accumulators copied right after the branch that joined the paths, returned three of
    // every four outputs stale.  The loop is straight-line now; the longest such wait (19 states) is spelled
    // out as well, once per launch.
    __builtin_amdgcn_sched_barrier(0);
    asm volatile("s_nop 15\n\ts_nop 7" ::: "memory");
    __builtin_amdgcn_sched_barrier(0);
    // partial accumulators -> LDS, then tile t = b * J + j is summed over the waves in order by wave t % FW
#pragma unroll
    for (int b = 0; b < 2; ++b)
#pragma unroll
        for (int j = 0; j < J; ++j)
            if (b < nb) red[((wave * 2 + b) * J + j) * 64 + lane] = acc[b][j];
    __syncthreads();
    for (int t = wave; t < 2 * J; t += FW) {
        const int b = t / J, j = t % J;
        if (b >= nb) continue;
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

// Activations re-laid out fragment by fragment for the kernel above: the 16-byte piece that lane (m % 16, q) feeds
// to matrix instruction c of m-tile j in slab sl goes to ((((sl * jn + j) * CH + c) * 64 + lane) * 16 bytes, jn = the
// number of m-tiles the kernel variant for this M computes.  Rows past M repeat row M - 1; their products are never stored.
__global__ __launch_bounds__(256) void zo_fused_relayout_kernel(const zo_bf16* __restrict__ X, int64_t strideX, int M, int K, int CH, int jn,
                                                                zo_bf16* __restrict__ out, int64_t strideOut)
{
    const int kchunks = K >> 3;
    const int64_t total = (int64_t)jn * 16 * kchunks;
    const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (i >= total) return;
    const int b = blockIdx.y;
    const int mp = (int)(i / kchunks), kc = (int)(i % kchunks);
    const int m = mp < M ? mp : M - 1;
    const uint4 v = *reinterpret_cast<const uint4*>(X + b * strideX + (int64_t)m * K + kc * 8);
    const int sl = kc / (4 * CH), r = kc % (4 * CH), q = r / CH, c = r % CH, j = mp >> 4, lane = q * 16 + (mp & 15);
    *reinterpret_cast<uint4*>(out + b * strideOut + ((((int64_t)sl * jn + j) * CH + c) * 64 + lane) * 8) = v;
}

// m-tiles computed by the kernel variant that serves M rows
int tiles_for(int M) { return M <= 16 ? 1 : M <= 32 ? 2 : M <= 64 ? 4 : 8; }

template <typename TW, int CH, int GL, int J>
hipError_t launch_w(const zo_fused_args& a, const zo_stream& s, hipStream_t st)
{
    constexpr int lds = FW * 2 * J * 1024;
    if (lds > 64 * 1024) {
        hipError_t e = hipFuncSetAttribute((const void*)zo_fq_gemm_fused_kernel<TW, CH, GL, J>, hipFuncAttributeMaxDynamicSharedMemorySize, lds);
        if (e != hipSuccess) return e;
    }
    zo_fq_gemm_fused_kernel<TW, CH, GL, J><<<dim3(a.N / 16), FW * 64, lds, st>>>(a, s);
    return hipGetLastError();
}

template <int CH, int GL, int J>
hipError_t launch_one(const zo_fused_args& a, const zo_stream& s, hipStream_t st)
{
    return a.wdtype == ZO_W_F16 ? launch_w<zo_f16, CH, GL, J>(a, s, st) : launch_w<float, CH, GL, J>(a, s, st);
}

template <int CH, int GL>
hipError_t launch_j(const zo_fused_args& a, const zo_stream& s, hipStream_t st)
{
    switch (tiles_for(a.M)) {
        case 1:  return launch_one<CH, GL, 1>(a, s, st);
        case 2:  return launch_one<CH, GL, 2>(a, s, st);
        case 4:  return launch_one<CH, GL, 4>(a, s, st);
        default: return launch_one<CH, GL, 8>(a, s, st);
    }
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

static int fused_ch(int bits, int group) { return bits == 0 || group <= 32 ? 1 : group / 32; }

size_t zo_fused_relayout_bytes(int32_t M, int32_t K) { return (size_t)tiles_for(M) * 16 * (size_t)K * 2; }

hipError_t zo_launch_fused_relayout(const void* X, int64_t strideX, int32_t M, int32_t K, int32_t nb, int32_t bits, int32_t group,
                                    void* out, int64_t strideOut, hipStream_t st)
{
    const int jn = tiles_for(M);
    const int64_t total = (int64_t)jn * 16 * (K / 8);
    const dim3 grid((unsigned)((total + 255) / 256), nb);
    zo_fused_relayout_kernel<<<grid, 256, 0, st>>>((const zo_bf16*)X, strideX, M, K, fused_ch(bits, group), jn, (zo_bf16*)out, strideOut);
    return hipGetLastError();
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
