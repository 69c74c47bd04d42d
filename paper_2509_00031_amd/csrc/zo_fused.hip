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

// min / max over the GL lanes lane % 16 + 16 q that share a quantization group: row swap (lane ^ 16), then half-wave
// swap (lane ^ 32), both register-to-register
template <int GL, typename OP> ZO_DEV float q_reduce(float v, OP op)
{
    if (GL >= 2) {
        const auto r = __builtin_amdgcn_permlane16_swap(__float_as_uint(v), __float_as_uint(v), false, false);
        v = op(__uint_as_float(r[0]), __uint_as_float(r[1]));
    }
    if (GL >= 4) {
        const auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(v), __float_as_uint(v), false, false);
        v = op(__uint_as_float(r[0]), __uint_as_float(r[1]));
    }
    return v;
}
template <int GL> ZO_DEV float q_min(float v)
{
    return q_reduce<GL>(v, [](float a, float b) { return fminf(a, b); });
}
template <int GL> ZO_DEV float q_max(float v)
{
    return q_reduce<GL>(v, [](float a, float b) { return fmaxf(a, b); });
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

// bias / ReLU / residual and one rounding for the four outputs (m, nn .. nn + 3) of branch b
__device__ __forceinline__ void store_outputs(const zo_fused_args& a, f32x4 v, int b, int m, int nn)
{
    if (m >= a.M) return;
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

// Tail shared by the two kernels of this file: the partial accumulators of the FW waves are added in wave order
// through LDS, then bias / ReLU / residual and one rounding.
template <int J>
__device__ __forceinline__ void reduce_and_store(const zo_fused_args& a, f32x4 (&acc)[2][J], f32x4* red, int wave, int lane, int n0)
{
    const int n = lane & 15, q = lane >> 4;
    const int nb = a.nb;
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
        store_outputs(a, v, b, j * 16 + n, n0 + 4 * q);
    }
}

template <typename TW, int CH, int GL, int J>
__global__ __launch_bounds__(FW * 64) void zo_fq_gemm_fused_kernel(zo_fused_args a, zo_stream s, zo_fused_second second)
{
    if (blockIdx.y) {                                        // second tensor of a paired launch
        a.W = second.W; a.Y = second.Y; a.bias = second.bias; a.residual = second.residual;
        s.tensor_id = (uint32_t)second.tid;
    }
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

    reduce_and_store<J>(a, acc, red, wave, lane, n0);
}

// ---------------------------------------------------------------------------------------------
// The same contraction for a frozen, pre-quantized linear (lightweight variant; also plain inference on the
// packed model): Y[b] = X[b] * w^^T with w^ = (code - zp) * step expanded from the 4-bit codes in registers, in
// operand layout, 0.5 B of HBM traffic per weight.  Both branches of Eq. 2 share the operand (no perturbation).
// Lane (n, q) owns CH consecutive 32-bit words of codes (8 features each); a slab of 32*CH features lies inside
// one quantization group (group = 32, 64 or a multiple of 128), whose binary16 step and int16 zero point every
// lane of the row reads.  Same arithmetic per weight as zo_dequant_int4_kernel.
// ---------------------------------------------------------------------------------------------
template <int CH> ZO_DEV void load_words(const uint32_t* p, uint32_t (&w)[CH])
{
    if constexpr (CH == 4) {
        const uint4 v = *reinterpret_cast<const uint4*>(p);
        w[0] = v.x; w[1] = v.y; w[2] = v.z; w[3] = v.w;
    } else if constexpr (CH == 2) {
        const uint2 v = *reinterpret_cast<const uint2*>(p);
        w[0] = v.x; w[1] = v.y;
    } else {
        w[0] = *p;
    }
}

template <int CH, int J>
__global__ __launch_bounds__(FW * 64) void zo_int4_gemm_fused_kernel(zo_fused_args a)
{
    extern __shared__ __attribute__((aligned(16))) unsigned char lds_raw[];
    f32x4* red = reinterpret_cast<f32x4*>(lds_raw);
    constexpr int SLAB = 32 * CH;
    const int lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int n = lane & 15, q = lane >> 4;
    const int M = a.M, K = a.K, nb = a.nb;
    const int n0 = blockIdx.x * 16;
    const int nslab = K / SLAB;
    const int G = K / a.group;
    const uint32_t* crow = (const uint32_t*)a.codes + (((int64_t)(n0 + n) * K) >> 3) + q * CH;
    const _Float16* srow = (const _Float16*)a.step16 + (int64_t)(n0 + n) * G;
    const int16_t* zrow = a.zp + (int64_t)(n0 + n) * G;
    const zo_bf16* X = (const zo_bf16*)a.X;

    f32x4 acc[2][J];
#pragma unroll
    for (int b = 0; b < 2; ++b)
#pragma unroll
        for (int j = 0; j < J; ++j) acc[b][j] = f32x4{0.0f, 0.0f, 0.0f, 0.0f};

    uint32_t words[CH], wnext[CH];
    if (wave < nslab) load_words<CH>(crow + wave * (SLAB / 8), words);
    for (int sl = wave; sl < nslab; sl += FW) {
        const int k0 = sl * SLAB;
        const zo_bf16* xcol = X + k0 + q * (CH * 8);
        int mrow[J];
#pragma unroll
        for (int j = 0; j < J; ++j) {
            const int m = j * 16 + n;
            mrow[j] = m < M ? m : M - 1;
        }
        const zo_bf16* xfrag = a.Xfrag ? (const zo_bf16*)a.Xfrag + ((int64_t)sl * J * CH * 64 + lane) * 8 : nullptr;
        auto fragment = [&](int b, int j, int c) -> bf16x8 {
            if (xfrag) return *reinterpret_cast<const bf16x8*>(xfrag + b * a.strideXfrag + (j * CH + c) * 512);
            return *reinterpret_cast<const bf16x8*>(xcol + b * a.strideX + (int64_t)mrow[j] * K + c * 8);
        };
        if (sl + FW < nslab) load_words<CH>(crow + (sl + FW) * (SLAB / 8), wnext);
        const int g = k0 / a.group;
        const float st = (float)srow[g];
        const int z = zrow[g];
        bf16x8 af[CH];
#pragma unroll
        for (int c = 0; c < CH; ++c) {
            float o[8];
#pragma unroll
            for (int i = 0; i < 8; ++i) o[i] = (float)((int)((words[c] >> (4 * i)) & 15u) - z) * st;
            af[c] = pack8(o);
        }
#pragma unroll
        for (int j = 0; j < J; ++j)
#pragma unroll
            for (int b = 0; b < 2; ++b)
                if (b < nb) {
#pragma unroll
                    for (int c = 0; c < CH; ++c)
                        acc[b][j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(af[c], fragment(b, j, c), acc[b][j], 0, 0, 0);
                }
#pragma unroll
        for (int c = 0; c < CH; ++c) words[c] = wnext[c];
    }
    reduce_and_store<J>(a, acc, red, wave, lane, n0);
}

// ---------------------------------------------------------------------------------------------
// Split-K form of the kernel above, for when the caller lends scratch memory.  With 16 channels per workgroup every
// workgroup reads all of X (N/16 times in total, far more than the 0.5 B per weight of the codes), and with one
// 16-channel operand per wave every matrix instruction needs a fresh 1 KB activation fragment.  Here
//   * a workgroup = 4 waves covers 256 or 128 channels (wave w: 64 or 32 of them = four or two 16-channel operands per K step, so a
//     fragment read from LDS feeds four or two matrix instructions) and one of KS ranges of K;
//   * the activation fragments of a slab (already in fragment order in a.Xfrag) are copied global -> LDS by the load
//     unit itself (16 B per lane, no staging registers), two stages, one barrier per slab;
//   * a workgroup handles MT <= 8 m-tiles: both branches together while they fit (MT = nb * J), else one branch per
//     workgroup (blockIdx.z), which expands the same codes twice;
//   * every wave owns its outputs over the workgroup's K range: KS = 1 stores them directly, otherwise partial sums go
//     to P[ks][b][m][n] (fp32) and zo_splitk_reduce_kernel adds the KS partials in order (no atomics).
// ---------------------------------------------------------------------------------------------
__device__ __forceinline__ uint32_t lds_offset_of(const void* p)
{
    return (uint32_t)(uintptr_t)(__attribute__((address_space(3))) const void*)p;
}
// one wave-level 1 KB copy: lane fetches 16 bytes at base + voff, LDS destination dst + lane * 16
__device__ __forceinline__ void lds_copy16(const void* base, uint32_t voff, uint32_t dst)
{
    asm volatile("s_mov_b32 m0, %0\n\tglobal_load_lds_dwordx4 %1, %2\n" ::"s"(dst), "v"(voff), "s"(base) : "memory");
}

constexpr int SW = 4;            // waves per workgroup of the split-K kernel

// SRG: 16-channel operands per wave.  KG: wave groups of SW waves each; the groups work on the same channels and deal the
// slabs of the workgroup's K range among themselves (group g takes slabs g, g + KG, ...), so that a SIMD holds KG waves that
// hide one another's waits; at the end the groups' accumulators are added through LDS in group order.
template <int CH, int MT, int SRG, int KG>
__global__ __launch_bounds__(SW * KG * 64) void zo_int4_gemm_splitk_kernel(zo_fused_args a, float* __restrict__ P, int KS, int J)
{
    extern __shared__ __attribute__((aligned(16))) unsigned char lds_raw[];
    constexpr int SLAB = 32 * CH;
    constexpr int NF = MT * CH;                              // 1 KB fragments per stage and wave group
    constexpr int STAGE = NF * 1024;
    const int lane = threadIdx.x & 63, wave_all = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int kg = wave_all / SW, wave = wave_all % SW;
    const int n = lane & 15, q = lane >> 4;
    const int M = a.M, N = a.N, K = a.K, nb = a.nb;
    const bool per_branch = gridDim.z > 1;                   // one branch per workgroup
    const int zb = blockIdx.z;
    const int nbase = blockIdx.x * (SW * SRG * 16) + wave * (SRG * 16);
    const int nslab = K / SLAB;
    const int per = (nslab + KS - 1) / KS;
    const int s_begin = blockIdx.y * per;
    const int s_end = s_begin + per < nslab ? s_begin + per : nslab;
    const int iters = s_end > s_begin ? (s_end - s_begin + KG - 1) / KG : 0;   // the same for every wave of the workgroup
    const int G = K / a.group;
    const uint32_t* crow[SRG];
    const _Float16* srow[SRG];
    const int16_t* zrow[SRG];
    bool rg_ok[SRG];
#pragma unroll
    for (int r = 0; r < SRG; ++r) {
        rg_ok[r] = nbase + 16 * r < N;                       // N is a multiple of 16
        const int ch = rg_ok[r] ? nbase + 16 * r + n : 0;
        crow[r] = (const uint32_t*)a.codes + (((int64_t)ch * K) >> 3) + q * CH;
        srow[r] = (const _Float16*)a.step16 + (int64_t)ch * G;
        zrow[r] = a.zp + (int64_t)ch * G;
    }
    const uint32_t lds0 = __builtin_amdgcn_readfirstlane(lds_offset_of(lds_raw));
    const zo_bf16* xf_base = (const zo_bf16*)a.Xfrag;
    // fragment fi = t * CH + c of slab sl: m-tile t is (branch, j) = (zb, t) or (t / J, t % J).  A group whose turn falls past the
    // end of the range copies the range's last slab again (finite values) and multiplies it by all-zero weights.
    auto issue = [&](int stage, int sl) {
        const int slc = sl < s_end ? sl : s_end - 1;
        for (int fi = wave; fi < NF; fi += SW) {
            const int t = fi / CH, c = fi % CH;
            const int b = per_branch ? zb : t / J, j = per_branch ? t : t % J;
            const zo_bf16* src = xf_base + b * a.strideXfrag + (((int64_t)slc * J + j) * CH + c) * 512;
            lds_copy16(src, (uint32_t)lane * 16u, lds0 + (stage * KG + kg) * STAGE + fi * 1024);
        }
    };

    f32x4 acc[SRG][MT];
#pragma unroll
    for (int r = 0; r < SRG; ++r)
#pragma unroll
        for (int t = 0; t < MT; ++t) acc[r][t] = f32x4{0.0f, 0.0f, 0.0f, 0.0f};

    uint32_t words[SRG][CH], wnext[SRG][CH];
#pragma unroll
    for (int r = 0; r < SRG; ++r)
#pragma unroll
        for (int c = 0; c < CH; ++c) words[r][c] = wnext[r][c] = 0u;
    float st[SRG], stn[SRG];
    int zq[SRG], zqn[SRG];
#pragma unroll
    for (int r = 0; r < SRG; ++r) { st[r] = stn[r] = 0.0f; zq[r] = zqn[r] = 0; }
    if (iters > 0) {
        const int sl0 = s_begin + kg;
        issue(0, sl0);
        if (sl0 < s_end) {
            const int g0 = sl0 * SLAB / a.group;
#pragma unroll
            for (int r = 0; r < SRG; ++r) {
                load_words<CH>(crow[r] + sl0 * (SLAB / 8), words[r]);
                st[r] = (float)srow[r][g0];
                zq[r] = zrow[r][g0];
            }
        }
    }
    __builtin_amdgcn_s_waitcnt(0x0F70);                      // vmcnt(0): this wave's copies have landed
    __syncthreads();
    int stage = 0;
    for (int it = 0; it < iters; ++it) {
        const int sln = s_begin + (it + 1) * KG + kg;        // this group's next slab
        if (it + 1 < iters) {                                // stage ^ 1 was last read before the barrier just passed
            issue(stage ^ 1, sln);
            if (sln < s_end) {                               // codes, step and zero point of the next slab: one slab ahead
                const int gn = sln * SLAB / a.group;
#pragma unroll
                for (int r = 0; r < SRG; ++r) {
                    load_words<CH>(crow[r] + sln * (SLAB / 8), wnext[r]);
                    stn[r] = (float)srow[r][gn];
                    zqn[r] = zrow[r][gn];
                }
            } else {
#pragma unroll
                for (int r = 0; r < SRG; ++r) {
                    stn[r] = 0.0f;
                    zqn[r] = 0;
#pragma unroll
                    for (int c = 0; c < CH; ++c) wnext[r][c] = 0u;
                }
            }
        }
        bf16x8 af[SRG][CH];
#pragma unroll
        for (int r = 0; r < SRG; ++r) {
#pragma unroll
            for (int c = 0; c < CH; ++c) {
                float o[8];
#pragma unroll
                for (int i = 0; i < 8; ++i) o[i] = (float)((int)((words[r][c] >> (4 * i)) & 15u) - zq[r]) * st[r];
                af[r][c] = pack8(o);
            }
        }
        // fragments are read from LDS two ahead of their use (ring of three), in the order c-major / t-minor so that
        // consecutive matrix instructions never wait for one another's accumulator
        const unsigned char* sb = lds_raw + (stage * KG + kg) * STAGE + lane * 16;
        auto frag = [&](int f) { return *reinterpret_cast<const bf16x8*>(sb + (((f % MT) * CH + f / MT) << 10)); };
        bf16x8 xq[3];
        xq[0] = frag(0);
        if (NF > 1) xq[1] = frag(1);
#pragma unroll
        for (int f = 0; f < NF; ++f) {
            if (f + 2 < NF) xq[(f + 2) % 3] = frag(f + 2);
            const int c = f / MT, t = f % MT;
#pragma unroll
            for (int r = 0; r < SRG; ++r) acc[r][t] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(af[r][c], xq[f % 3], acc[r][t], 0, 0, 0);
        }
        __builtin_amdgcn_s_waitcnt(0x0F70);                  // vmcnt(0): own copies of the next slab (and its codes) are in
        __syncthreads();
        stage ^= 1;
#pragma unroll
        for (int r = 0; r < SRG; ++r) {
            st[r] = stn[r];
            zq[r] = zqn[r];
#pragma unroll
            for (int c = 0; c < CH; ++c) words[r][c] = wnext[r][c];
        }
    }
    __builtin_amdgcn_sched_barrier(0);
    asm volatile("s_nop 15\n\ts_nop 7" ::: "memory");
    __builtin_amdgcn_sched_barrier(0);
    if constexpr (KG > 1) {
        // the last barrier of the loop is behind every wave: the stages are free.  Groups 1 .. KG-1 hand their sums to group 0.
        f32x4* red = reinterpret_cast<f32x4*>(lds_raw);      // [KG - 1][SW][SRG][MT][64]
        if (kg > 0) {
#pragma unroll
            for (int r = 0; r < SRG; ++r)
#pragma unroll
                for (int t = 0; t < MT; ++t) red[((((kg - 1) * SW + wave) * SRG + r) * MT + t) * 64 + lane] = acc[r][t];
        }
        __syncthreads();
        if (kg > 0) return;
#pragma unroll
        for (int g = 1; g < KG; ++g)
#pragma unroll
            for (int r = 0; r < SRG; ++r)
#pragma unroll
                for (int t = 0; t < MT; ++t) {
                    const f32x4 p = red[((((g - 1) * SW + wave) * SRG + r) * MT + t) * 64 + lane];
                    acc[r][t][0] += p[0]; acc[r][t][1] += p[1]; acc[r][t][2] += p[2]; acc[r][t][3] += p[3];
                }
    }
#pragma unroll
    for (int r = 0; r < SRG; ++r)
#pragma unroll
        for (int t = 0; t < MT; ++t) {
            const int b = per_branch ? zb : t / J, j = per_branch ? t : t % J;
            const int m = j * 16 + n, nn = nbase + 16 * r + 4 * q;
            if (!rg_ok[r] || b >= nb || j >= J) continue;
            if (P) {
                if (m < M)
                    *reinterpret_cast<float4*>(P + (((int64_t)blockIdx.y * nb + b) * M + m) * N + nn) =
                        make_float4(acc[r][t][0], acc[r][t][1], acc[r][t][2], acc[r][t][3]);
            } else {
                store_outputs(a, acc[r][t], b, m, nn);
            }
        }
}

// Y = epilogue(sum over ks of P[ks][b][m][n]), the KS terms added in order; one thread per four consecutive n
__global__ __launch_bounds__(256) void zo_splitk_reduce_kernel(zo_fused_args a, const float* __restrict__ P, int KS)
{
    const int64_t per_b = (int64_t)a.M * (a.N >> 2);
    const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (i >= per_b * a.nb) return;
    const int b = (int)(i / per_b);
    const int64_t r = i % per_b;
    const int m = (int)(r / (a.N >> 2)), nn = (int)(r % (a.N >> 2)) * 4;
    const int64_t plane = (int64_t)a.nb * a.M * a.N;
    const float* p = P + ((int64_t)b * a.M + m) * a.N + nn;
    f32x4 v = *reinterpret_cast<const f32x4*>(p);
    for (int ks = 1; ks < KS; ++ks) {
        const f32x4 t = *reinterpret_cast<const f32x4*>(p + ks * plane);
        v[0] += t[0]; v[1] += t[1]; v[2] += t[2]; v[3] += t[3];
    }
    store_outputs(a, v, b, m, nn);
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
hipError_t launch_w(const zo_fused_args& a, const zo_stream& s, const zo_fused_second* second, hipStream_t st)
{
    constexpr int lds = FW * 2 * J * 1024;
    if (lds > 64 * 1024) {
        hipError_t e = hipFuncSetAttribute((const void*)zo_fq_gemm_fused_kernel<TW, CH, GL, J>, hipFuncAttributeMaxDynamicSharedMemorySize, lds);
        if (e != hipSuccess) return e;
    }
    zo_fq_gemm_fused_kernel<TW, CH, GL, J><<<dim3(a.N / 16, second ? 2 : 1), FW * 64, lds, st>>>(a, s, second ? *second : zo_fused_second{});
    return hipGetLastError();
}

template <int CH, int GL, int J>
hipError_t launch_one(const zo_fused_args& a, const zo_stream& s, const zo_fused_second* second, hipStream_t st)
{
    return a.wdtype == ZO_W_F16 ? launch_w<zo_f16, CH, GL, J>(a, s, second, st) : launch_w<float, CH, GL, J>(a, s, second, st);
}

template <int CH, int GL>
hipError_t launch_j(const zo_fused_args& a, const zo_stream& s, const zo_fused_second* second, hipStream_t st)
{
    switch (tiles_for(a.M)) {
        case 1:  return launch_one<CH, GL, 1>(a, s, second, st);
        case 2:  return launch_one<CH, GL, 2>(a, s, second, st);
        case 4:  return launch_one<CH, GL, 4>(a, s, second, st);
        default: return launch_one<CH, GL, 8>(a, s, second, st);
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

template <int CH, int J>
static hipError_t launch_int4_one(const zo_fused_args& a, hipStream_t st)
{
    constexpr int lds = FW * 2 * J * 1024;
    if (lds > 64 * 1024) {
        hipError_t e = hipFuncSetAttribute((const void*)zo_int4_gemm_fused_kernel<CH, J>, hipFuncAttributeMaxDynamicSharedMemorySize, lds);
        if (e != hipSuccess) return e;
    }
    zo_int4_gemm_fused_kernel<CH, J><<<dim3(a.N / 16), FW * 64, lds, st>>>(a);
    return hipGetLastError();
}

template <int CH>
static hipError_t launch_int4_j(const zo_fused_args& a, hipStream_t st)
{
    switch (tiles_for(a.M)) {
        case 1:  return launch_int4_one<CH, 1>(a, st);
        case 2:  return launch_int4_one<CH, 2>(a, st);
        case 4:  return launch_int4_one<CH, 4>(a, st);
        default: return launch_int4_one<CH, 8>(a, st);
    }
}

// 16-channel operands per wave: four (256 channels per workgroup) where a workgroup carries 8 m-tiles, else two -- measured at
// the 13B shapes: half the partial sums for twice the activation re-reads pays at 32 tokens (36.5 against 41.7 us per launch)
// and costs at 128 (104 against 94 us)
static int splitk_srg(int MT) { return MT >= 8 ? 4 : 2; }
// Number of K ranges.  Timers inside the kernel: a workgroup spends about 0.9 us per slab and wave (operand expansion, LDS
// reads and matrix instructions mostly one after the other) and 30 % more waiting for the next slab, so a launch lasts about as
// long as the CU with the most slabs to work through: (rounds of workgroups over the 256 CUs) x (slabs per workgroup).  Every
// further range also adds a set of fp32 partial sums, written and read back (8 B per output at about 4 TB/s, in units of a
// slab's 0.9 us).  The count that minimises the sum is taken; at least two slabs per range, at most 16 ranges.  Against "one
// workgroup per CU, rounded up": 34.0 instead of 36.9 us per launch at 32 tokens, 86.8 instead of 94.7 at 128 (13B shapes).
static int splitk_ranges(int M, int nb, int N, int K, int group, int zdim, int MT)
{
    const int slab = group >= 128 ? 128 : group;
    const int chw = SW * splitk_srg(MT) * 16;
    const int tiles = ((N + chw - 1) / chw) * zdim, nslab = K / slab;
    const double per_range = 2.2e-6 * nb * (double)M * N;
    int best = 1;
    double best_cost = 0.0;
    for (int ks = 1; ks <= 16 && (ks == 1 || ks <= nslab / 2); ++ks) {
        const int rounds = (tiles * ks + 255) / 256, slabs = (nslab + ks - 1) / ks;
        const double cost = (double)rounds * slabs + (ks > 1 ? ks * per_range : 0.0);
        if (ks == 1 || cost < best_cost) { best = ks; best_cost = cost; }
    }
    return best;
}
// m-tiles per workgroup and workgroups along z for M rows and nb branches
static void splitk_shape(int M, int nb, int& MT, int& zdim)
{
    const int J = tiles_for(M);
    if (nb * J <= 8) { MT = nb * J; zdim = 1; } else { MT = J; zdim = nb; }
}

template <int CH, int MT>
static hipError_t launch_splitk_one(const zo_fused_args& a, float* P, int KS, int zdim, hipStream_t st)
{
    constexpr int SRG = MT >= 8 ? 4 : 2;             // = splitk_srg(MT)
    constexpr int KG = MT >= 8 ? 1 : 2;              // two wave groups (two waves per SIMD) while their registers fit
    constexpr int chw = SW * SRG * 16;
    constexpr int lds_stages = 2 * KG * MT * CH * 1024, lds_red = (KG - 1) * SW * SRG * MT * 1024;
    constexpr int lds = lds_stages > lds_red ? lds_stages : lds_red;
    static_assert(lds <= 160 * 1024, "LDS of the split-K kernel");
    if (lds > 64 * 1024) {
        hipError_t e = hipFuncSetAttribute((const void*)zo_int4_gemm_splitk_kernel<CH, MT, SRG, KG>, hipFuncAttributeMaxDynamicSharedMemorySize, lds);
        if (e != hipSuccess) return e;
    }
    zo_int4_gemm_splitk_kernel<CH, MT, SRG, KG><<<dim3((a.N + chw - 1) / chw, KS, zdim), SW * KG * 64, lds, st>>>(a, KS > 1 ? P : nullptr, KS, tiles_for(a.M));
    if (KS > 1) {
        const int64_t items = (int64_t)a.nb * a.M * (a.N / 4);
        zo_splitk_reduce_kernel<<<(unsigned)((items + 255) / 256), 256, 0, st>>>(a, P, KS);
    }
    return hipGetLastError();
}

template <int CH>
static hipError_t launch_splitk_mt(const zo_fused_args& a, float* P, int KS, int MT, int zdim, hipStream_t st)
{
    switch (MT) {
        case 1:  return launch_splitk_one<CH, 1>(a, P, KS, zdim, st);
        case 2:  return launch_splitk_one<CH, 2>(a, P, KS, zdim, st);
        case 4:  return launch_splitk_one<CH, 4>(a, P, KS, zdim, st);
        default: return launch_splitk_one<CH, 8>(a, P, KS, zdim, st);
    }
}

size_t zo_int4_splitk_scratch_bytes(int32_t M, int32_t N, int32_t K, int32_t group)
{
    return (size_t)16 * 2 * (size_t)M * (size_t)N * sizeof(float);      // KS <= 16, two branches
}

hipError_t zo_launch_int4_gemm_splitk(const zo_fused_args& a, void* partials, hipStream_t st)
{
    if (!zo_int4_fused_supported(a.M, a.N, a.K, a.group) || (a.nb != 1 && a.nb != 2) || (a.ldY & 3) || !a.codes || !a.step16 || !a.zp ||
        !partials || !a.Xfrag)
        return hipErrorInvalidValue;
    int MT, zdim;
    splitk_shape(a.M, a.nb, MT, zdim);
    const int KS = splitk_ranges(a.M, a.nb, a.N, a.K, a.group, zdim, MT);
    if (a.group == 32) return launch_splitk_mt<1>(a, (float*)partials, KS, MT, zdim, st);
    if (a.group == 64) return launch_splitk_mt<2>(a, (float*)partials, KS, MT, zdim, st);
    return launch_splitk_mt<4>(a, (float*)partials, KS, MT, zdim, st);
}

bool zo_int4_fused_supported(int32_t M, int32_t N, int32_t K, int32_t group)
{
    if (M < 1 || M > ZO_FUSED_MAX_M || N < 16 || (N & 15) || K <= 0) return false;
    if (group != 32 && group != 64 && group != 128 && group != 256 && group != 512) return false;
    return K % group == 0;
}

hipError_t zo_launch_int4_gemm_fused(const zo_fused_args& a, hipStream_t st)
{
    if (!zo_int4_fused_supported(a.M, a.N, a.K, a.group) || (a.nb != 1 && a.nb != 2) || (a.ldY & 3) || !a.codes || !a.step16 || !a.zp)
        return hipErrorInvalidValue;
    if (a.group == 32) return launch_int4_j<1>(a, st);
    if (a.group == 64) return launch_int4_j<2>(a, st);
    return launch_int4_j<4>(a, st);
}

static int fused_ch(int bits, int group) { return bits == 0 || group <= 32 ? 1 : group >= 128 ? 4 : group / 32; }

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

static hipError_t launch_fq_gemm_fused(const zo_fused_args& a, const zo_fused_second* second, uint64_t seed, int32_t tid, hipStream_t st)
{
    if (!zo_fused_supported(a.M, a.N, a.K, a.bits, a.group) || (a.nb != 1 && a.nb != 2) || (a.ldY & 3)) return hipErrorInvalidValue;
    zo_stream s;
    s.k0 = (uint32_t)seed;
    s.k1 = (uint32_t)(seed >> 32);
    s.tensor_id = (uint32_t)tid;
    if (a.bits == 0) return launch_j<1, 1>(a, s, second, st);
    switch (a.group) {
        case 8:   return launch_j<1, 1>(a, s, second, st);
        case 16:  return launch_j<1, 2>(a, s, second, st);
        case 32:  return launch_j<1, 4>(a, s, second, st);
        case 64:  return launch_j<2, 4>(a, s, second, st);
        default:  return launch_j<4, 4>(a, s, second, st);
    }
}
hipError_t zo_launch_fq_gemm_fused(const zo_fused_args& a, uint64_t seed, int32_t tid, hipStream_t st)
{
    return launch_fq_gemm_fused(a, nullptr, seed, tid, st);
}
hipError_t zo_launch_fq_gemm_fused_pair(const zo_fused_args& a, const zo_fused_second& second, uint64_t seed, int32_t tid, hipStream_t st)
{
    if (!second.W || !second.Y) return hipErrorInvalidValue;
    return launch_fq_gemm_fused(a, &second, seed, tid, st);
}
