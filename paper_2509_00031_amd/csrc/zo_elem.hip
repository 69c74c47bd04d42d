// Streaming (HBM-bound) kernels of the ZO-QAT step: the seeded update of Eq. 3, the weight
// fake-quantizer Q(W +- eps u) of Eq. 2, the per-token activation quantizer, and the debug
// materialisation of the perturbation stream.  gfx950, wave64.
#include "zo_device.h"
#include "zo_internal.h"
#include <cstdlib>

static inline zo_stream make_stream(uint64_t seed, int32_t tid)
{
    zo_stream s;
    s.k0 = (uint32_t)seed;
    s.k1 = (uint32_t)(seed >> 32);
    s.tensor_id = (uint32_t)tid;
    return s;
}

static inline int grid_for(int64_t items, int per_block, int max_blocks)
{
    int64_t b = (items + per_block - 1) / per_block;
    if (b < 1) b = 1;
    if (b > max_blocks) b = max_blocks;
    return (int)b;
}

// ---------------------------------------------------------------------------------------------
// perturbation stream, materialised (tests only)
// ---------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void zo_philox_words_kernel(zo_stream s, int64_t nwords, uint32_t* out)
{
    int64_t nblk = (nwords + 3) >> 2;
    for (int64_t b = (int64_t)blockIdx.x * 256 + threadIdx.x; b < nblk; b += (int64_t)gridDim.x * 256) {
        uint32_t w[4];
        zo_philox(s, (uint64_t)b, w);
#pragma unroll
        for (int i = 0; i < 4; ++i)
            if (4 * b + i < nwords) out[4 * b + i] = w[i];
    }
}

__global__ __launch_bounds__(256) void zo_normal_kernel(zo_stream s, int64_t start, int64_t n, float* out)
{
    for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < n; i += (int64_t)gridDim.x * 256)
        out[i] = zo_z1(s, (uint64_t)(start + i));
}

hipError_t zo_launch_philox_words(uint64_t seed, int32_t tid, int64_t nwords, uint32_t* out, hipStream_t st)
{
    if (nwords == 0) return hipSuccess;
    zo_philox_words_kernel<<<grid_for((nwords + 3) / 4, 256, 4096), 256, 0, st>>>(make_stream(seed, tid), nwords, out);
    return hipGetLastError();
}

hipError_t zo_launch_normal(uint64_t seed, int32_t tid, int64_t start, int64_t n, float* out, hipStream_t st)
{
    if (n == 0) return hipSuccess;
    zo_normal_kernel<<<grid_for(n, 256, 4096), 256, 0, st>>>(make_stream(seed, tid), start, n, out);
    return hipGetLastError();
}

// ---------------------------------------------------------------------------------------------
// update (Eq. 3): w_i <- fma(-c, u_i, w_i).  8 B of HBM traffic per parameter, u regenerated.
// Main kernel: a workgroup owns 4096 consecutive parameters; a wave sweeps 512 of them with two
// fully coalesced 16-byte accesses per lane (elements 4L..4L+3 and 256+4L..), then neighbouring
// lanes swap halves (DPP) so that every lane holds one whole Philox block of 8 parameters
// (even lane: block L/2 of the first half, odd lane: block 32 + L/2), and swap back for the store.
// The part of a tensor beyond the last multiple of 4096 goes through the simple tail kernel.
// ---------------------------------------------------------------------------------------------
__device__ __forceinline__ float swap_adjacent_lanes(float x)
{
    return __uint_as_float(__builtin_amdgcn_mov_dpp(__float_as_uint(x), 0xB1, 0xF, 0xF, true));   // quad_perm [1,0,3,2]
}

__global__ __launch_bounds__(256) void zo_update_kernel(float* __restrict__ w, zo_stream s,
                                                        const float* __restrict__ coeff_dev, float coeff_host)
{
    const float negc = -(coeff_dev ? *coeff_dev : coeff_host);
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const bool odd = lane & 1;
#pragma unroll
    for (int u = 0; u < 2; ++u) {
        const int64_t e0 = ((int64_t)blockIdx.x * 2 + u) * 2048 + wave * 512;
        float4* p = reinterpret_cast<float4*>(w + e0) + lane;
        typedef float f32x4_ __attribute__((ext_vector_type(4)));
        // every master is touched once per step: streaming (non-temporal) accesses, +8 % over cached ones
        const f32x4_ A_ = __builtin_nontemporal_load(reinterpret_cast<f32x4_*>(p)), B_ = __builtin_nontemporal_load(reinterpret_cast<f32x4_*>(p + 64));
        float4 A = make_float4(A_[0], A_[1], A_[2], A_[3]), B = make_float4(B_[0], B_[1], B_[2], B_[3]);
        float y0 = odd ? A.x : B.x, y1 = odd ? A.y : B.y, y2 = odd ? A.z : B.z, y3 = odd ? A.w : B.w;
        float n0 = swap_adjacent_lanes(y0), n1 = swap_adjacent_lanes(y1), n2 = swap_adjacent_lanes(y2), n3 = swap_adjacent_lanes(y3);
        float v[8], z[8];
        v[0] = odd ? n0 : A.x; v[1] = odd ? n1 : A.y; v[2] = odd ? n2 : A.z; v[3] = odd ? n3 : A.w;
        v[4] = odd ? B.x : n0; v[5] = odd ? B.y : n1; v[6] = odd ? B.z : n2; v[7] = odd ? B.w : n3;
        zo_z8(s, (uint64_t)(e0 >> 3) + (odd ? 32 : 0) + (lane >> 1), z);
#pragma unroll
        for (int i = 0; i < 8; ++i) v[i] = __builtin_fmaf(negc, z[i], v[i]);
        y0 = odd ? v[0] : v[4]; y1 = odd ? v[1] : v[5]; y2 = odd ? v[2] : v[6]; y3 = odd ? v[3] : v[7];
        n0 = swap_adjacent_lanes(y0); n1 = swap_adjacent_lanes(y1); n2 = swap_adjacent_lanes(y2); n3 = swap_adjacent_lanes(y3);
        A = odd ? make_float4(n0, n1, n2, n3) : make_float4(v[0], v[1], v[2], v[3]);
        B = odd ? make_float4(v[4], v[5], v[6], v[7]) : make_float4(n0, n1, n2, n3);
        const f32x4_ a_ = {A.x, A.y, A.z, A.w}, b_ = {B.x, B.y, B.z, B.w};
        __builtin_nontemporal_store(a_, reinterpret_cast<f32x4_*>(p));
        __builtin_nontemporal_store(b_, reinterpret_cast<f32x4_*>(p + 64));
    }
}

// elements [first, numel): one Philox block per thread, then the ragged end one element per thread
__global__ __launch_bounds__(256) void zo_update_tail_kernel(float* __restrict__ w, int64_t first, int64_t numel, zo_stream s,
                                                             const float* __restrict__ coeff_dev, float coeff_host)
{
    const float negc = -(coeff_dev ? *coeff_dev : coeff_host);
    const int64_t nblk = numel >> 3;
    const int64_t b = (first >> 3) + (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (b < nblk) {
        float v[8], z[8];
        zo_load8(w + 8 * b, v);
        zo_z8(s, (uint64_t)b, z);
#pragma unroll
        for (int i = 0; i < 8; ++i) v[i] = __builtin_fmaf(negc, z[i], v[i]);
        zo_store8(w + 8 * b, v);
    }
    if (blockIdx.x == 0) {
        const int64_t i = 8 * nblk + threadIdx.x;
        if (i < numel) w[i] = __builtin_fmaf(negc, zo_z1(s, (uint64_t)i), w[i]);
    }
}

hipError_t zo_launch_update(float* w, int64_t numel, uint64_t seed, int32_t tid,
                            const float* coeff_dev, float coeff_host, hipStream_t st)
{
    if (numel == 0) return hipSuccess;
    const zo_stream s = make_stream(seed, tid);
    const int64_t main_blocks = numel / 4096;
    if (main_blocks > 0x7FFFFFFF) return hipErrorInvalidValue;
    if (main_blocks > 0) zo_update_kernel<<<(int)main_blocks, 256, 0, st>>>(w, s, coeff_dev, coeff_host);
    const int64_t first = main_blocks * 4096;
    if (first < numel) {
        const int64_t tail_blk = ((numel >> 3) - (first >> 3) + 255) / 256;
        zo_update_tail_kernel<<<(int)(tail_blk > 0 ? tail_blk : 1), 256, 0, st>>>(w, first, numel, s, coeff_dev, coeff_host);
    }
    return hipGetLastError();
}

// ---------------------------------------------------------------------------------------------
// update with q directions (Eq. 2 with q > 1, Eq. 3): w_i <- fma(-c_{q-1}, u_i(seed_{q-1}), ... fma(-c_0, u_i(seed_0), w_i)),
// the terms applied in the order of the seeds, all in one pass over the masters (8 B per parameter whatever q).
// Same work split and lane-pair exchange as zo_update_kernel.
// ---------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void zo_update_multi_kernel(float* __restrict__ w, zo_multi_seeds ms, uint32_t tensor_id, int q,
                                                              const float* __restrict__ coeff_dev, int coeff_stride)
{
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const bool odd = lane & 1;
#pragma unroll 1
    for (int u = 0; u < 2; ++u) {
        const int64_t e0 = ((int64_t)blockIdx.x * 2 + u) * 2048 + wave * 512;
        float4* p = reinterpret_cast<float4*>(w + e0) + lane;
        typedef float f32x4_ __attribute__((ext_vector_type(4)));
        const f32x4_ A_ = __builtin_nontemporal_load(reinterpret_cast<f32x4_*>(p)), B_ = __builtin_nontemporal_load(reinterpret_cast<f32x4_*>(p + 64));
        float4 A = make_float4(A_[0], A_[1], A_[2], A_[3]), B = make_float4(B_[0], B_[1], B_[2], B_[3]);
        float y0 = odd ? A.x : B.x, y1 = odd ? A.y : B.y, y2 = odd ? A.z : B.z, y3 = odd ? A.w : B.w;
        float n0 = swap_adjacent_lanes(y0), n1 = swap_adjacent_lanes(y1), n2 = swap_adjacent_lanes(y2), n3 = swap_adjacent_lanes(y3);
        float v[8], z[8];
        v[0] = odd ? n0 : A.x; v[1] = odd ? n1 : A.y; v[2] = odd ? n2 : A.z; v[3] = odd ? n3 : A.w;
        v[4] = odd ? B.x : n0; v[5] = odd ? B.y : n1; v[6] = odd ? B.z : n2; v[7] = odd ? B.w : n3;
        const uint64_t blk = (uint64_t)(e0 >> 3) + (odd ? 32 : 0) + (lane >> 1);
#pragma unroll 1
        for (int d = 0; d < q; ++d) {
            const zo_stream s{ms.k0[d], ms.k1[d], tensor_id};
            const float negc = -(coeff_dev ? coeff_dev[d * coeff_stride] : ms.c[d]);
            zo_z8(s, blk, z);
#pragma unroll
            for (int i = 0; i < 8; ++i) v[i] = __builtin_fmaf(negc, z[i], v[i]);
        }
        y0 = odd ? v[0] : v[4]; y1 = odd ? v[1] : v[5]; y2 = odd ? v[2] : v[6]; y3 = odd ? v[3] : v[7];
        n0 = swap_adjacent_lanes(y0); n1 = swap_adjacent_lanes(y1); n2 = swap_adjacent_lanes(y2); n3 = swap_adjacent_lanes(y3);
        A = odd ? make_float4(n0, n1, n2, n3) : make_float4(v[0], v[1], v[2], v[3]);
        B = odd ? make_float4(v[4], v[5], v[6], v[7]) : make_float4(n0, n1, n2, n3);
        const f32x4_ a_ = {A.x, A.y, A.z, A.w}, b_ = {B.x, B.y, B.z, B.w};
        __builtin_nontemporal_store(a_, reinterpret_cast<f32x4_*>(p));
        __builtin_nontemporal_store(b_, reinterpret_cast<f32x4_*>(p + 64));
    }
}

__global__ __launch_bounds__(256) void zo_update_multi_tail_kernel(float* __restrict__ w, int64_t first, int64_t numel, zo_multi_seeds ms,
                                                                   uint32_t tensor_id, int q, const float* __restrict__ coeff_dev,
                                                                   int coeff_stride)
{
    const int64_t nblk = numel >> 3;
    const int64_t b = (first >> 3) + (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (b < nblk) {
        float v[8], z[8];
        zo_load8(w + 8 * b, v);
        for (int d = 0; d < q; ++d) {
            const zo_stream s{ms.k0[d], ms.k1[d], tensor_id};
            const float negc = -(coeff_dev ? coeff_dev[d * coeff_stride] : ms.c[d]);
            zo_z8(s, (uint64_t)b, z);
#pragma unroll
            for (int i = 0; i < 8; ++i) v[i] = __builtin_fmaf(negc, z[i], v[i]);
        }
        zo_store8(w + 8 * b, v);
    }
    if (blockIdx.x == 0) {
        const int64_t i = 8 * nblk + threadIdx.x;
        if (i < numel) {
            float x = w[i];
            for (int d = 0; d < q; ++d) {
                const zo_stream s{ms.k0[d], ms.k1[d], tensor_id};
                const float negc = -(coeff_dev ? coeff_dev[d * coeff_stride] : ms.c[d]);
                x = __builtin_fmaf(negc, zo_z1(s, (uint64_t)i), x);
            }
            w[i] = x;
        }
    }
}

hipError_t zo_launch_update_multi(float* w, int64_t numel, const zo_multi_seeds& ms, int32_t q, int32_t tid,
                                  const float* coeff_dev, int32_t coeff_stride, hipStream_t st)
{
    if (numel == 0 || q == 0) return hipSuccess;
    if (q < 0 || q > ZO_MAX_DIRECTIONS_INTERNAL) return hipErrorInvalidValue;
    const int64_t main_blocks = numel / 4096;
    if (main_blocks > 0x7FFFFFFF) return hipErrorInvalidValue;
    if (main_blocks > 0) zo_update_multi_kernel<<<(int)main_blocks, 256, 0, st>>>(w, ms, (uint32_t)tid, q, coeff_dev, coeff_stride);
    const int64_t first = main_blocks * 4096;
    if (first < numel) {
        const int64_t tail_blk = ((numel >> 3) - (first >> 3) + 255) / 256;
        zo_update_multi_tail_kernel<<<(int)(tail_blk > 0 ? tail_blk : 1), 256, 0, st>>>(w, first, numel, ms, (uint32_t)tid, q, coeff_dev,
                                                                                        coeff_stride);
    }
    return hipGetLastError();
}

// ---------------------------------------------------------------------------------------------
// update of binary16 masters: x = fma(-c_d, u(seed_d), w) over the q directions in fp32, then ONE rounding to
// binary16 (nearest even, or stochastic with the integers of the rounding stream of seeds[0]).  A lane's 16-byte
// access is exactly one Philox block of 8 parameters, so no lane exchange is needed; 4 B of HBM traffic per
// parameter.  The ragged end (numel % 8) goes one element per thread.
// ---------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void zo_update_f16_kernel(uint16_t* __restrict__ w, int64_t numel, zo_multi_seeds ms, uint32_t tensor_id,
                                                            int q, const float* __restrict__ coeff_dev, int coeff_stride, int stochastic)
{
    const int64_t nblk = numel >> 3;
    const int64_t b = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (b < nblk) {
        typedef uint32_t u32x4_ __attribute__((ext_vector_type(4)));
        u32x4_* p = reinterpret_cast<u32x4_*>(w + 8 * b);
        const u32x4_ raw = __builtin_nontemporal_load(p);
        float v[8], z[8];
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            v[2 * i] = zo_f16_value((uint16_t)(raw[i] & 0xFFFFu));
            v[2 * i + 1] = zo_f16_value((uint16_t)(raw[i] >> 16));
        }
#pragma unroll 1
        for (int d = 0; d < q; ++d) {
            const zo_stream s{ms.k0[d], ms.k1[d], tensor_id};
            const float negc = -(coeff_dev ? coeff_dev[d * coeff_stride] : ms.c[d]);
            zo_z8(s, (uint64_t)b, z);
#pragma unroll
            for (int i = 0; i < 8; ++i) v[i] = __builtin_fmaf(negc, z[i], v[i]);
        }
        uint16_t h[8];
        if (stochastic) {
            uint32_t r[8];
            zo_round_bits8(zo_stream{ms.k0[0], ms.k1[0], tensor_id}, (uint64_t)b, r);
#pragma unroll
            for (int i = 0; i < 8; ++i) h[i] = zo_f16_stochastic(v[i], r[i]);
        } else {
#pragma unroll
            for (int i = 0; i < 8; ++i) h[i] = zo_f16_bits(v[i]);
        }
        u32x4_ o;
#pragma unroll
        for (int i = 0; i < 4; ++i) o[i] = (uint32_t)h[2 * i] | ((uint32_t)h[2 * i + 1] << 16);
        __builtin_nontemporal_store(o, p);
    }
    if (blockIdx.x == 0) {
        const int64_t i = 8 * nblk + threadIdx.x;
        if (i < numel) {
            float x = zo_f16_value(w[i]);
            for (int d = 0; d < q; ++d) {
                const zo_stream s{ms.k0[d], ms.k1[d], tensor_id};
                const float negc = -(coeff_dev ? coeff_dev[d * coeff_stride] : ms.c[d]);
                x = __builtin_fmaf(negc, zo_z1(s, (uint64_t)i), x);
            }
            w[i] = stochastic ? zo_f16_stochastic(x, zo_round_bits1(zo_stream{ms.k0[0], ms.k1[0], tensor_id}, (uint64_t)i)) : zo_f16_bits(x);
        }
    }
}

hipError_t zo_launch_update_f16(void* w, int64_t numel, const zo_multi_seeds& ms, int32_t q, int32_t tid,
                                const float* coeff_dev, int32_t coeff_stride, int32_t stochastic, hipStream_t st)
{
    if (numel == 0 || q == 0) return hipSuccess;
    if (q < 0 || q > ZO_MAX_DIRECTIONS_INTERNAL) return hipErrorInvalidValue;
    const int64_t blocks = ((numel >> 3) + 255) / 256;
    if (blocks > 0x7FFFFFFF) return hipErrorInvalidValue;
    zo_update_f16_kernel<<<(int)(blocks > 0 ? blocks : 1), 256, 0, st>>>((uint16_t*)w, numel, ms, (uint32_t)tid, q, coeff_dev, coeff_stride,
                                                                         stochastic);
    return hipGetLastError();
}

// ---------------------------------------------------------------------------------------------
// weight fake-quantizer: Q(W + eps u) and/or Q(W - eps u), de-quantized, in GEMM operand type.
// One thread owns 8 consecutive k (one Philox block); a group of G consecutive k is G/8 = GL
// neighbouring lanes, reduced with cross-lane shuffles.  u is generated once for both branches.
// HBM traffic: 4 B read + sizeof(TO) written per branch and element.
// ---------------------------------------------------------------------------------------------
// Output position (in 8-element blocks) of input block b of a matrix with kb blocks per row when the rows go out
// interleaved for the gate / up GEMM with SwiGLU in its epilogue: blocks of 32 gate rows (ilv = 1) alternate with the
// 32 up rows (ilv = 2) of the same channels; or (ilv = 3) for the q | k | v GEMM with the rotary embedding in its epilogue.
// The row of a block is b / kb: a 64-bit division per thread would cost dozens of instructions, so the host passes the
// multiplier and shift that make it one multiply (exact for b < 2^31: m = ceil(2^(31 + l) / kb), l = ceil(log2 kb)).
struct zo_rowdiv { int32_t kb; uint32_t magic; int32_t shift; };
static zo_rowdiv make_rowdiv(int kb)
{
    int l = 0;
    while ((1u << l) < (unsigned)kb) ++l;
    const int sh = 31 + l;
    return zo_rowdiv{kb, (uint32_t)((((uint64_t)1 << sh) + (uint64_t)kb - 1) / (uint64_t)kb), sh};
}
__device__ __forceinline__ uint32_t zo_quot(uint32_t b, const zo_rowdiv& d)      // b / d.kb for b < 2^31
{
    return (uint32_t)(((uint64_t)b * d.magic) >> d.shift);
}
__device__ __forceinline__ int64_t interleaved_block(int64_t b, const zo_rowdiv& d, int ilv)
{
    if (ilv == 0) return b;
    const uint32_t n = zo_quot((uint32_t)b, d);
    const uint32_t kblk = (uint32_t)b - n * (uint32_t)d.kb;
    uint32_t row;
    if (ilv == 3) {                                  // blocks 1 and 2 of every 128-row head trade places
        const uint32_t blk = (n >> 5) & 3;
        row = (blk == 1) ? n + 32 : (blk == 2) ? n - 32 : n;
    } else {
        row = ((n >> 5) << 6) + (n & 31) + (ilv == 2 ? 32 : 0);
    }
    return (int64_t)row * d.kb + kblk;
}

template <typename TO, int GL, bool DEBUG>
__device__ __forceinline__ void fq_branch(const float v[8], int bits, TO* out, int64_t b, int64_t ob, bool active,
                                          uint8_t* codes, float* step, int32_t* zp, int lane)
{
    float o[8];
    if (bits == 0) {
#pragma unroll
        for (int i = 0; i < 8; ++i) o[i] = v[i];
    } else {
        float mn = v[0], mx = v[0];
#pragma unroll
        for (int i = 1; i < 8; ++i) { mn = fminf(mn, v[i]); mx = fmaxf(mx, v[i]); }
        mn = zo_group_min<GL>(mn);
        mx = zo_group_max<GL>(mx);
        zo_qparams q = zo_qparams_asym(mn, mx, bits);
        float c[8];
#pragma unroll
        for (int i = 0; i < 8; ++i) { c[i] = zo_code(q, v[i]); o[i] = zo_dequant(q, c[i]); }
        if (DEBUG && active) {
            if (codes) {
#pragma unroll
                for (int i = 0; i < 8; ++i) codes[8 * b + i] = (uint8_t)c[i];
            }
            if ((lane & (GL - 1)) == 0) {
                if (step) step[b / GL] = q.step;
                if (zp) zp[b / GL] = (int32_t)q.zp;
            }
        }
    }
    if (active && out) zo_store8(out + 8 * ob, o);
}

template <typename TW, typename TO, int GL, bool DEBUG>
__global__ __launch_bounds__(256) void zo_fq_weight_kernel(const TW* __restrict__ W, int64_t nblk, zo_stream s,
                                                           float eps, int bits, TO* __restrict__ out_p, TO* __restrict__ out_m,
                                                           uint8_t* codes, float* step, int32_t* zp, zo_rowdiv kb, int ilv)
{
    const int lane = threadIdx.x & 63;
    // one Philox block per thread; every lane of a wave takes part in the shuffles
    {
        const int64_t b = (int64_t)blockIdx.x * 256 + threadIdx.x;
        const bool active = b < nblk;
        const int64_t ob = interleaved_block(b, kb, ilv);
        float w[8], z[8];
        if (active) {
            zo_load8(W + 8 * b, w);
            if (eps != 0.0f) zo_z8(s, (uint64_t)b, z);
        }
        if (!active || eps == 0.0f) {
#pragma unroll
            for (int i = 0; i < 8; ++i) { z[i] = 0.0f; if (!active) w[i] = 0.0f; }
        }
        if (out_p || DEBUG) {
            float v[8];
#pragma unroll
            for (int i = 0; i < 8; ++i) v[i] = __builtin_fmaf(eps, z[i], w[i]);
            fq_branch<TO, GL, DEBUG>(v, bits, out_p, b, ob, active, codes, step, zp, lane);
        }
        if (out_m) {
            float v[8];
#pragma unroll
            for (int i = 0; i < 8; ++i) v[i] = __builtin_fmaf(-eps, z[i], w[i]);
            fq_branch<TO, GL, false>(v, bits, out_m, b, ob, active, nullptr, nullptr, nullptr, lane);
        }
    }
}

// Groups wider than 512 elements (per-channel quantization): one workgroup per group, two sweeps over it (range, then
// codes).  NB > 0: a thread's (at most NB) blocks of 8 weights and their perturbations stay in registers between the sweeps
// (groups of up to 2048 NB weights), so the stream is generated once; NB = 0: any group length, stream generated twice.
// The rows may go out interleaved for the GEMM epilogues (ilv, see interleaved_block).
template <typename TW, typename TO, bool DEBUG, int NB>
__global__ __launch_bounds__(256) void zo_fq_weight_row_kernel(const TW* __restrict__ W, int K, int group, zo_stream s,
                                                               float eps, int bits, TO* __restrict__ out_p, TO* __restrict__ out_m,
                                                               uint8_t* codes, float* step, int32_t* zp, zo_rowdiv kb, int ilv)
{
    __shared__ float red[4][4];
    constexpr int HELD = NB > 0 ? NB : 1;
    const int64_t grp = blockIdx.x;                 // group index over the whole matrix
    const int64_t b0 = grp * (group / 8);           // first Philox block of the group
    const int nb = group / 8;
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
                float vp = __builtin_fmaf(eps, z[i], w[i]), vm = __builtin_fmaf(-eps, z[i], w[i]);
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
    zo_qparams qp = zo_qparams_asym(mnp, mxp, bits), qm = zo_qparams_asym(mnm, mxm, bits);
    if (DEBUG && threadIdx.x == 0) {
        if (step) step[grp] = qp.step;
        if (zp) zp[grp] = (int32_t)qp.zp;
    }
#pragma unroll
    for (int u = 0; u < sweeps; ++u) {
        const int j = threadIdx.x + 256 * u;
        if (j < nb) {
            float wl[8], zl[8], o[8];
            float (&w)[8] = NB > 0 ? wv[NB > 0 ? u : 0] : wl;
            float (&z)[8] = NB > 0 ? zv[NB > 0 ? u : 0] : zl;
            if (NB == 0) fetch(j, w, z);
            const int64_t ob = interleaved_block(b0 + j, kb, ilv);
            if (out_p || DEBUG) {
#pragma unroll
                for (int i = 0; i < 8; ++i) {
                    float c = zo_code(qp, __builtin_fmaf(eps, z[i], w[i]));
                    o[i] = zo_dequant(qp, c);
                    if (DEBUG && codes) codes[8 * (b0 + j) + i] = (uint8_t)c;
                }
                if (out_p) zo_store8(out_p + 8 * ob, o);
            }
            if (out_m) {
#pragma unroll
                for (int i = 0; i < 8; ++i) o[i] = zo_dequant(qm, zo_code(qm, __builtin_fmaf(-eps, z[i], w[i])));
                zo_store8(out_m + 8 * ob, o);
            }
        }
    }
}

bool zo_fq_weight_supported(int32_t K, int32_t bits, int32_t group)
{
    if (K <= 0 || (K & 7)) return false;
    if (bits == 0) return true;
    if (bits < 1 || bits > 8) return false;
    if (group == 0) group = K;
    if (group <= 0 || (group & 7) || K % group) return false;
    return true;
}

template <typename TW, typename TO, int GL>
static hipError_t launch_fq_weight_gl(const TW* W, int64_t nblk, zo_stream s, float eps, int bits, TO* op, TO* om,
                                      uint8_t* codes, float* step, int32_t* zp, hipStream_t st, int kb = 1, int ilv = 0)
{
    if ((nblk + 255) / 256 > 0x7FFFFFFF || (ilv != 0 && nblk >= ((int64_t)1 << 31))) return hipErrorInvalidValue;
    const int grid = (int)((nblk + 255) / 256);
    const zo_rowdiv rd = make_rowdiv(kb);
    if (codes || step || zp)
        zo_fq_weight_kernel<TW, TO, GL, true><<<grid, 256, 0, st>>>(W, nblk, s, eps, bits, op, om, codes, step, zp, rd, ilv);
    else
        zo_fq_weight_kernel<TW, TO, GL, false><<<grid, 256, 0, st>>>(W, nblk, s, eps, bits, op, om, nullptr, nullptr, nullptr, rd, ilv);
    return hipGetLastError();
}

template <typename TW, typename TO>
static hipError_t launch_fq_weight_t(const TW* W, int32_t N, int32_t K, int32_t bits, int32_t group, zo_stream s, float eps,
                                     TO* op, TO* om, uint8_t* codes, float* step, int32_t* zp, hipStream_t st, int ilv)
{
    const int kb = K / 8;
    if (ilv != 0 && (N & (ilv == 3 ? 127 : 31))) return hipErrorInvalidValue;
    const int64_t nblk = (int64_t)N * K / 8;
    if (nblk == 0) return hipSuccess;
    if (bits == 0) return launch_fq_weight_gl<TW, TO, 1>(W, nblk, s, eps, 0, op, om, nullptr, nullptr, nullptr, st, kb, ilv);
    if (group == 0) group = K;
    const int gl = group / 8;
    const bool pow2 = (gl & (gl - 1)) == 0;
    if (pow2 && gl <= 64) {
        switch (gl) {
            case 1:  return launch_fq_weight_gl<TW, TO, 1>(W, nblk, s, eps, bits, op, om, codes, step, zp, st, kb, ilv);
            case 2:  return launch_fq_weight_gl<TW, TO, 2>(W, nblk, s, eps, bits, op, om, codes, step, zp, st, kb, ilv);
            case 4:  return launch_fq_weight_gl<TW, TO, 4>(W, nblk, s, eps, bits, op, om, codes, step, zp, st, kb, ilv);
            case 8:  return launch_fq_weight_gl<TW, TO, 8>(W, nblk, s, eps, bits, op, om, codes, step, zp, st, kb, ilv);
            case 16: return launch_fq_weight_gl<TW, TO, 16>(W, nblk, s, eps, bits, op, om, codes, step, zp, st, kb, ilv);
            case 32: return launch_fq_weight_gl<TW, TO, 32>(W, nblk, s, eps, bits, op, om, codes, step, zp, st, kb, ilv);
            default: return launch_fq_weight_gl<TW, TO, 64>(W, nblk, s, eps, bits, op, om, codes, step, zp, st, kb, ilv);
        }
    }
    const int64_t ngroups = (int64_t)N * (K / group);
    if (ngroups > 0x7FFFFFFF || (ilv != 0 && nblk >= ((int64_t)1 << 31))) return hipErrorInvalidValue;
    const zo_rowdiv rd = make_rowdiv(kb);
    if (codes || step || zp) {
        zo_fq_weight_row_kernel<TW, TO, true, 0><<<(int)ngroups, 256, 0, st>>>(W, K, group, s, eps, bits, op, om, codes, step, zp, rd, ilv);
        return hipGetLastError();
    }
#define ZO_ROWFQ(NB) zo_fq_weight_row_kernel<TW, TO, false, NB><<<(int)ngroups, 256, 0, st>>>(W, K, group, s, eps, bits, op, om, nullptr, nullptr, nullptr, rd, ilv)
    if (group <= 4096) ZO_ROWFQ(2); else if (group <= 8192) ZO_ROWFQ(4); else if (group <= 12288) ZO_ROWFQ(6); else if (group <= 16384) ZO_ROWFQ(8); else ZO_ROWFQ(0);
#undef ZO_ROWFQ
    return hipGetLastError();
}

hipError_t zo_launch_fq_weight(const void* W, int32_t N, int32_t K, int32_t bits, int32_t group,
                               uint64_t seed, int32_t tid, float eps, int dtype,
                               void* out_plus, void* out_minus,
                               uint8_t* codes, float* step, int32_t* zp, hipStream_t st, int wdtype, int ilv)
{
    zo_stream s = make_stream(seed, tid);
    if (wdtype == ZO_W_F16) {
        const zo_f16* Wh = (const zo_f16*)W;
        if (dtype == ZO_T_BF16)
            return launch_fq_weight_t<zo_f16, zo_bf16>(Wh, N, K, bits, group, s, eps, (zo_bf16*)out_plus, (zo_bf16*)out_minus, codes, step, zp, st, ilv);
        return launch_fq_weight_t<zo_f16, float>(Wh, N, K, bits, group, s, eps, (float*)out_plus, (float*)out_minus, codes, step, zp, st, ilv);
    }
    const float* Wf = (const float*)W;
    if (dtype == ZO_T_BF16)
        return launch_fq_weight_t<float, zo_bf16>(Wf, N, K, bits, group, s, eps, (zo_bf16*)out_plus, (zo_bf16*)out_minus, codes, step, zp, st, ilv);
    return launch_fq_weight_t<float, float>(Wf, N, K, bits, group, s, eps, (float*)out_plus, (float*)out_minus, codes, step, zp, st, ilv);
}

// ---------------------------------------------------------------------------------------------
// Adaptive weight quantizer (Eq. 5) with learnable per-group step, zero point and clipping
// coefficients, optionally on the smoothed weight s (.) W of Eq. 4.  The parameter arrays arrive
// already perturbed (one set per branch); there is no min/max reduction, so any group size that is
// a multiple of 8 works: gl = group / 8 threads share one parameter set.
//   code = clamp(rint(w * (1/step)) + rint(zp), rint(alpha Q_P), rint(beta Q_P)),  w^ = (code - rint(zp)) * step
// with the bounds kept inside [0, Q_P] and ordered, and the step floored at 1e-5.
// ---------------------------------------------------------------------------------------------
template <typename TO>
__device__ __forceinline__ void fq_learned_branch(const float w[8], const float z[8], float e, const zo_learned& p, int64_t g, int kb,
                                                  int bits, TO* out, int64_t b, int64_t ob, uint8_t* codes)
{
    float st = p.step[g];
    if (!(st >= 1e-5f)) st = 1e-5f;
    const float inv = 1.0f / st;
    const float qp = (float)((1 << bits) - 1);
    const float zr = rintf(p.zp[g]);
    float lo = rintf(p.alpha[g] * qp), hi = rintf(p.beta[g] * qp);
    lo = lo < 0.0f ? 0.0f : lo;
    lo = lo > qp ? qp : lo;
    hi = hi > qp ? qp : hi;
    hi = hi < lo ? lo : hi;
    float sc[8];
    if (p.scale) zo_load8(p.scale + kb, sc);
    float o[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        float v = __builtin_fmaf(e, z[i], w[i]);
        if (p.scale) v = sc[i] * v;
        float q = rintf(v * inv) + zr;
        q = q < lo ? lo : q;
        q = q > hi ? hi : q;
        if (codes) codes[8 * b + i] = (uint8_t)q;
        o[i] = (q - zr) * st;
    }
    zo_store8(out + 8 * ob, o);
}

template <typename TO>
__global__ __launch_bounds__(256) void zo_fq_weight_learned_kernel(const float* __restrict__ W, int64_t nblk, zo_rowdiv k8, zo_rowdiv gl, zo_stream s,
                                                                   float eps, int bits, zo_learned pp, zo_learned pm,
                                                                   TO* __restrict__ out_p, TO* __restrict__ out_m, uint8_t* codes, int ilv)
{
    const int64_t b = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (b >= nblk) return;
    const int64_t ob = interleaved_block(b, k8, ilv);          // rows interleaved for the GEMM epilogues (0: as stored)
    float w[8], z[8];
    zo_load8(W + 8 * b, w);
    if (eps != 0.0f) zo_z8(s, (uint64_t)b, z);
    else {
#pragma unroll
        for (int i = 0; i < 8; ++i) z[i] = 0.0f;
    }
    const int64_t g = zo_quot((uint32_t)b, gl);
    const int kb = (int)((uint32_t)b - zo_quot((uint32_t)b, k8) * (uint32_t)k8.kb) * 8;
    fq_learned_branch<TO>(w, z, eps, pp, g, kb, bits, out_p, b, ob, codes);
    if (out_m) fq_learned_branch<TO>(w, z, -eps, pm, g, kb, bits, out_m, b, ob, nullptr);
}

hipError_t zo_launch_fq_weight_learned(const float* W, int32_t N, int32_t K, int32_t bits, int32_t group, uint64_t seed, int32_t tid,
                                       float eps, int dtype, const zo_learned& pp, const zo_learned& pm, void* out_plus, void* out_minus,
                                       uint8_t* codes, hipStream_t st, int ilv)
{
    const int64_t nblk = (int64_t)N * K / 8;
    if (nblk == 0) return hipSuccess;
    if (group == 0) group = K;
    if ((K & 7) || (group & 7) || K % group || bits < 1 || bits > 8 || nblk >= ((int64_t)1 << 31)) return hipErrorInvalidValue;
    const int grid = (int)((nblk + 255) / 256);
    const zo_stream s = make_stream(seed, tid);
    if (dtype == ZO_T_BF16)
        zo_fq_weight_learned_kernel<zo_bf16><<<grid, 256, 0, st>>>(W, nblk, make_rowdiv(K / 8), make_rowdiv(group / 8), s, eps, bits, pp, pm, (zo_bf16*)out_plus,
                                                                   (zo_bf16*)out_minus, codes, ilv);
    else
        zo_fq_weight_learned_kernel<float><<<grid, 256, 0, st>>>(W, nblk, make_rowdiv(K / 8), make_rowdiv(group / 8), s, eps, bits, pp, pm, (float*)out_plus,
                                                                 (float*)out_minus, codes, ilv);
    return hipGetLastError();
}

// Initial values of Eq. 5's parameters from what the dynamic quantizer computes (zero point as a
// real number, alpha = 0, beta = 1).
__global__ __launch_bounds__(256) void zo_init_learned_kernel(const int32_t* __restrict__ zp_i, int64_t n, float* zp, float* alpha, float* beta)
{
    const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (i >= n) return;
    zp[i] = (float)zp_i[i];
    alpha[i] = 0.0f;
    beta[i] = 1.0f;
}

hipError_t zo_launch_init_learned(const float* W, int32_t N, int32_t K, int32_t bits, int32_t group, float* step, float* zp,
                                  float* alpha, float* beta, int32_t* zp_scratch, hipStream_t st)
{
    const int g = group ? group : K;
    const int64_t n = (int64_t)N * (K / g);
    if (n == 0) return hipSuccess;
    hipError_t e = zo_launch_fq_weight(W, N, K, bits, group, 0, 0, 0.0f, ZO_T_F32, nullptr, nullptr, nullptr, step, zp_scratch, st);
    if (e != hipSuccess) return e;
    zo_init_learned_kernel<<<(int)((n + 255) / 256), 256, 0, st>>>(zp_scratch, n, zp, alpha, beta);
    return hipGetLastError();
}

// out[i] = value (fill) / out[i] = 1 / in[i] (correctly rounded division): the small vectors of Eq. 4
__global__ __launch_bounds__(256) void zo_fill_kernel(float* out, int64_t n, float value)
{
    const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (i < n) out[i] = value;
}
__global__ __launch_bounds__(256) void zo_reciprocal_kernel(const float* __restrict__ in, float* __restrict__ out, int64_t n)
{
    const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (i < n) out[i] = 1.0f / in[i];
}
hipError_t zo_launch_fill(float* out, int64_t n, float value, hipStream_t st)
{
    if (n == 0) return hipSuccess;
    zo_fill_kernel<<<(int)((n + 255) / 256), 256, 0, st>>>(out, n, value);
    return hipGetLastError();
}
hipError_t zo_launch_reciprocal(const float* in, float* out, int64_t n, hipStream_t st)
{
    if (n == 0) return hipSuccess;
    zo_reciprocal_kernel<<<(int)((n + 255) / 256), 256, 0, st>>>(in, out, n);
    return hipGetLastError();
}

// Bias of the smoothed linear (Eq. 4): out[n] = bias[n] + sum_k delta[k] * w'[n][k], w' = w +- eps u, for both
// branches in one pass over W.  One wavefront per output row, lane-strided partial sums in k order, then a
// fixed xor tree: the result does not depend on the launch shape.
__global__ __launch_bounds__(256) void zo_bias_shift_kernel(const float* __restrict__ W, int N, int K, zo_stream s, float eps,
                                                            const float* __restrict__ delta_p, const float* __restrict__ delta_m,
                                                            const float* __restrict__ bias_p, const float* __restrict__ bias_m,
                                                            float* __restrict__ out_p, float* __restrict__ out_m)
{
    const int lane = threadIdx.x & 63;
    const int n = blockIdx.x * 4 + (threadIdx.x >> 6);
    if (n >= N) return;
    const int k8 = K / 8;
    float ap = 0.0f, am = 0.0f;
    for (int j = lane; j < k8; j += 64) {
        const int64_t b = (int64_t)n * k8 + j;
        float w[8], z[8], dp[8], dm[8];
        zo_load8(W + 8 * b, w);
        if (eps != 0.0f) zo_z8(s, (uint64_t)b, z);
        zo_load8(delta_p + 8 * j, dp);
        if (out_m) zo_load8(delta_m + 8 * j, dm);
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            const float zi = eps != 0.0f ? z[i] : 0.0f;
            ap = __builtin_fmaf(dp[i], __builtin_fmaf(eps, zi, w[i]), ap);
            if (out_m) am = __builtin_fmaf(dm[i], __builtin_fmaf(-eps, zi, w[i]), am);
        }
    }
    ap = zo_group_sum<64>(ap);
    am = zo_group_sum<64>(am);
    if (lane == 0) {
        out_p[n] = (bias_p ? bias_p[n] : 0.0f) + ap;
        if (out_m) out_m[n] = (bias_m ? bias_m[n] : 0.0f) + am;
    }
}

hipError_t zo_launch_bias_shift(const float* W, int32_t N, int32_t K, uint64_t seed, int32_t tid, float eps,
                                const float* delta_p, const float* delta_m, const float* bias_p, const float* bias_m,
                                float* out_p, float* out_m, hipStream_t st)
{
    if (N == 0) return hipSuccess;
    zo_bias_shift_kernel<<<(N + 3) / 4, 256, 0, st>>>(W, N, K, make_stream(seed, tid), eps, delta_p, delta_m, bias_p, bias_m, out_p, out_m);
    return hipGetLastError();
}

// ---------------------------------------------------------------------------------------------
// Frozen weights of the lightweight variant (Section "Lightweight ZeroQAT for memory reduction"):
// stored as 4-bit codes two per byte (low nibble = even k), one binary16 step and one int16 zero
// point per group.  zo_pack_int4_kernel pre-quantizes an fp32 matrix into that form (same
// arithmetic as the fake-quantizer at eps = 0); zo_dequant_int4_kernel expands it into the GEMM
// operand type: w^ = (code - zp) * step.  One thread owns 8 consecutive k = 4 packed bytes.
// ---------------------------------------------------------------------------------------------
template <int GL>
__global__ __launch_bounds__(256) void zo_pack_int4_kernel(const float* __restrict__ W, int64_t nblk, uint32_t* __restrict__ packed,
                                                           _Float16* __restrict__ step, int16_t* __restrict__ zp)
{
    const int lane = threadIdx.x & 63;
    const int64_t b = (int64_t)blockIdx.x * 256 + threadIdx.x;
    const bool active = b < nblk;
    float v[8];
    if (active) zo_load8(W + 8 * b, v);
    else {
#pragma unroll
        for (int i = 0; i < 8; ++i) v[i] = 0.0f;
    }
    float mn = v[0], mx = v[0];
#pragma unroll
    for (int i = 1; i < 8; ++i) { mn = fminf(mn, v[i]); mx = fmaxf(mx, v[i]); }
    mn = zo_group_min<GL>(mn);
    mx = zo_group_max<GL>(mx);
    const zo_qparams q = zo_qparams_asym(mn, mx, 4);
    uint32_t word = 0;
#pragma unroll
    for (int i = 0; i < 8; ++i) word |= ((uint32_t)zo_code(q, v[i]) & 15u) << (4 * i);
    if (!active) return;
    packed[b] = word;
    if ((lane & (GL - 1)) == 0) {
        step[b / GL] = (_Float16)q.step;                                  // round to nearest even, subnormals kept
        zp[b / GL] = (int16_t)fminf(fmaxf(q.zp, -32768.0f), 32767.0f);
    }
}

template <typename TO>
__global__ __launch_bounds__(256) void zo_dequant_int4_kernel(const uint32_t* __restrict__ packed, const _Float16* __restrict__ step,
                                                              const int16_t* __restrict__ zp, int64_t nblk, zo_rowdiv gl,
                                                              TO* __restrict__ out0, TO* __restrict__ out1, zo_rowdiv kb, int ilv)
{
    const int64_t b = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (b >= nblk) return;
    const int64_t ob = interleaved_block(b, kb, ilv);
    const uint32_t word = packed[b];
    const int64_t g = zo_quot((uint32_t)b, gl);
    const float st = (float)step[g];
    const int z = zp[g];
    float o[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) o[i] = (float)((int)((word >> (4 * i)) & 15u) - z) * st;
    zo_store8(out0 + 8 * ob, o);
    if (out1) zo_store8(out1 + 8 * ob, o);
}

bool zo_int4_group_supported(int32_t K, int32_t group)
{
    if (group < 8 || group > 512 || (group & (group - 1)) != 0) return false;
    return K > 0 && K % group == 0;
}

hipError_t zo_launch_pack_int4(const float* W, int32_t N, int32_t K, int32_t group, void* packed, void* step_f16, int16_t* zp,
                               hipStream_t st)
{
    const int64_t nblk = (int64_t)N * K / 8;
    if (nblk == 0) return hipSuccess;
    if (!zo_int4_group_supported(K, group) || (nblk + 255) / 256 > 0x7FFFFFFF) return hipErrorInvalidValue;
    const int grid = (int)((nblk + 255) / 256);
    uint32_t* pk = (uint32_t*)packed;
    _Float16* sp = (_Float16*)step_f16;
    switch (group / 8) {
        case 1:  zo_pack_int4_kernel<1><<<grid, 256, 0, st>>>(W, nblk, pk, sp, zp); break;
        case 2:  zo_pack_int4_kernel<2><<<grid, 256, 0, st>>>(W, nblk, pk, sp, zp); break;
        case 4:  zo_pack_int4_kernel<4><<<grid, 256, 0, st>>>(W, nblk, pk, sp, zp); break;
        case 8:  zo_pack_int4_kernel<8><<<grid, 256, 0, st>>>(W, nblk, pk, sp, zp); break;
        case 16: zo_pack_int4_kernel<16><<<grid, 256, 0, st>>>(W, nblk, pk, sp, zp); break;
        case 32: zo_pack_int4_kernel<32><<<grid, 256, 0, st>>>(W, nblk, pk, sp, zp); break;
        default: zo_pack_int4_kernel<64><<<grid, 256, 0, st>>>(W, nblk, pk, sp, zp); break;
    }
    return hipGetLastError();
}

hipError_t zo_launch_dequant_int4(const void* packed, const void* step_f16, const int16_t* zp, int32_t N, int32_t K, int32_t group,
                                  int dtype, void* out0, void* out1, hipStream_t st, int ilv)
{
    const int64_t nblk = (int64_t)N * K / 8;
    if (nblk == 0) return hipSuccess;
    if (!zo_int4_group_supported(K, group) || nblk >= ((int64_t)1 << 31) || (ilv != 0 && (N & (ilv == 3 ? 127 : 31)))) return hipErrorInvalidValue;
    const int grid = (int)((nblk + 255) / 256);
    if (dtype == ZO_T_BF16)
        zo_dequant_int4_kernel<zo_bf16><<<grid, 256, 0, st>>>((const uint32_t*)packed, (const _Float16*)step_f16, zp, nblk, make_rowdiv(group / 8),
                                                              (zo_bf16*)out0, (zo_bf16*)out1, make_rowdiv(K / 8), ilv);
    else
        zo_dequant_int4_kernel<float><<<grid, 256, 0, st>>>((const uint32_t*)packed, (const _Float16*)step_f16, zp, nblk, make_rowdiv(group / 8),
                                                            (float*)out0, (float*)out1, make_rowdiv(K / 8), ilv);
    return hipGetLastError();
}

// ---------------------------------------------------------------------------------------------
// per-token activation fake-quantizer: one wavefront per row; range sweep, then code sweep
// (the second sweep re-reads the row from cache).
// ---------------------------------------------------------------------------------------------
template <typename T, bool DEBUG>
__global__ __launch_bounds__(256) void zo_fq_act_kernel(const T* __restrict__ X, T* __restrict__ Xhat, int M, int K, int bits, int sym,
                                                        int16_t* codes, float* step, int32_t* zp,
                                                        const float* __restrict__ sm_delta, const float* __restrict__ sm_inv)
{
    const int lane = threadIdx.x & 63;
    const int row = blockIdx.x * 4 + (threadIdx.x >> 6);
    if (row >= M) return;                            // whole wave leaves together
    const T* x = X + (int64_t)row * K;
    float mn = INFINITY, mx = -INFINITY;
    // Eq. 4: with smoothing the quantizer sees (x - delta) / s
    auto smooth8 = [&](int c, float v[8]) {
        if (!sm_delta) return;
        float dl[8], iv[8];
        zo_load8(sm_delta + c, dl);
        zo_load8(sm_inv + c, iv);
#pragma unroll
        for (int i = 0; i < 8; ++i) v[i] = (v[i] - dl[i]) * iv[i];
    };
    for (int c = lane * 8; c < K; c += 512) {
        float v[8];
        zo_load8(x + c, v);
        smooth8(c, v);
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            if (sym) mx = fmaxf(mx, fabsf(v[i]));
            else { mn = fminf(mn, v[i]); mx = fmaxf(mx, v[i]); }
        }
    }
    mn = zo_group_min<64>(mn);
    mx = zo_group_max<64>(mx);
    zo_qparams q = sym ? zo_qparams_sym(mx, bits) : zo_qparams_asym(mn, mx, bits);
    if (DEBUG && lane == 0) {
        if (step) step[row] = q.step;
        if (zp) zp[row] = (int32_t)q.zp;
    }
    for (int c = lane * 8; c < K; c += 512) {
        float v[8], o[8];
        zo_load8(x + c, v);
        smooth8(c, v);
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            float cd = zo_code(q, v[i]);
            o[i] = zo_dequant(q, cd);
            if (DEBUG && codes) codes[(int64_t)row * K + c + i] = (int16_t)cd;
        }
        if (Xhat) zo_store8(Xhat + (int64_t)row * K + c, o);
    }
}

hipError_t zo_launch_fq_act(const void* X, void* Xhat, int32_t M, int32_t K, int32_t bits, int32_t sym, int dtype,
                            int16_t* codes, float* step, int32_t* zp, const float* sm_delta, const float* sm_inv, hipStream_t st)
{
    if (M == 0) return hipSuccess;
    const int grid = (M + 3) / 4;
    const bool dbg = codes || step || zp;
    if (dtype == ZO_T_BF16) {
        if (dbg) zo_fq_act_kernel<zo_bf16, true><<<grid, 256, 0, st>>>((const zo_bf16*)X, (zo_bf16*)Xhat, M, K, bits, sym, codes, step, zp, sm_delta, sm_inv);
        else zo_fq_act_kernel<zo_bf16, false><<<grid, 256, 0, st>>>((const zo_bf16*)X, (zo_bf16*)Xhat, M, K, bits, sym, nullptr, nullptr, nullptr, sm_delta, sm_inv);
    } else {
        if (dbg) zo_fq_act_kernel<float, true><<<grid, 256, 0, st>>>((const float*)X, (float*)Xhat, M, K, bits, sym, codes, step, zp, sm_delta, sm_inv);
        else zo_fq_act_kernel<float, false><<<grid, 256, 0, st>>>((const float*)X, (float*)Xhat, M, K, bits, sym, nullptr, nullptr, nullptr, sm_delta, sm_inv);
    }
    return hipGetLastError();
}
