// Causal softmax attention on the gfx950 matrix cores (bf16 storage, head dimension 64 or 128).
//
// One workgroup = 4 waves = 128 consecutive queries of one (batch, head); a wave owns 32 queries.
// Keys/values stream through LDS in tiles of 64.  Both matrix products are issued "transposed" so
// that a lane owns ONE query (column lane%32) in every accumulator:
//     S^T[key][query] = K[key][:] . Q[query][:]          (A = K tile rows, B = Q rows)
//     O^T[dh][query] += V^T[dh][key] . P^T[key][query]   (A = V^T tile rows, B = P, straight from
//                                                        the S accumulators, no cross-lane moves)
// so the running max / sum of the online softmax are per-lane scalars (the other half of a
// query's keys lives in lane^32).  V is transposed on its way into LDS; within each block of 16
// keys the order is permuted to match the accumulator layout of the S product.
#include "zo_device.h"
#include "zo_internal.h"

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

template <int CH> __device__ __forceinline__ int kswz(int row)
{
    return CH == 16 ? (row & 15) : ((row + (row >> 3)) & 7);
}
__device__ __forceinline__ int vswz(int row) { return (row + (row >> 3)) & 7; }

template <int DH>
__global__ __launch_bounds__(256) void zo_flash_attn_kernel(const zo_bf16* __restrict__ q, const zo_bf16* __restrict__ k,
                                                            const zo_bf16* __restrict__ v, zo_bf16* __restrict__ out,
                                                            int S, int H, int64_t row_stride, float scale_log2e)
{
    constexpr int CH = DH / 8;                    // 16-byte chunks per K row
    constexpr int KROW = DH * 2;                  // bytes per K row in LDS
    constexpr int KBYTES = 64 * KROW;
    constexpr int VBYTES = DH * 128;              // V^T tile: DH rows x 64 keys x 2 B
    constexpr int KIT = 64 * CH / 256;            // K chunks per thread
    constexpr int VIT = 32 * CH / 256;            // V key-pair chunks per thread
    __shared__ __attribute__((aligned(16))) unsigned char lds[2][KBYTES + VBYTES];

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int j = lane & 31, g = lane >> 5;
    const int nqt = (S + 127) / 128;
    const int qt = nqt - 1 - (int)blockIdx.x;     // longest rows first
    const int b = blockIdx.y / H, h = blockIdx.y % H;
    const int q0 = qt * 128 + wave * 32;
    const int qrow = q0 + j;
    const zo_bf16* qp = q + (int64_t)b * S * row_stride + (int64_t)h * DH;
    const zo_bf16* kp = k + (int64_t)b * S * row_stride + (int64_t)h * DH;
    const zo_bf16* vp = v + (int64_t)b * S * row_stride + (int64_t)h * DH;

    bf16x8 qf[DH / 16];
    {
        const int qr = qrow < S ? qrow : S - 1;
#pragma unroll
        for (int st = 0; st < DH / 16; ++st)
            qf[st] = *reinterpret_cast<const bf16x8*>(qp + (int64_t)qr * row_stride + 16 * st + 8 * g);
    }
    f32x16 o[DH / 32];
#pragma unroll
    for (int t = 0; t < DH / 32; ++t)
#pragma unroll
        for (int r = 0; r < 16; ++r) o[t][r] = 0.0f;
    float m_run = -INFINITY, l_run = 0.0f;

    const int kv_end = (qt * 128 + 128) < S ? (qt * 128 + 128) : S;
    const int ntiles = (kv_end + 63) / 64;

    uint4 kr[KIT], va[VIT], vb[VIT];
    auto fetch = [&](int t) {
#pragma unroll
        for (int i = 0; i < KIT; ++i) {
            const int id = tid + 256 * i, row = id / CH, c = id % CH;
            int key = t * 64 + row;
            key = key < S ? key : S - 1;
            kr[i] = *reinterpret_cast<const uint4*>(kp + (int64_t)key * row_stride + c * 8);
        }
#pragma unroll
        for (int i = 0; i < VIT; ++i) {
            const int id = tid + 256 * i, pr = id / CH, c = id % CH;
            int k0 = t * 64 + 2 * pr, k1 = k0 + 1;
            k0 = k0 < S ? k0 : S - 1;
            k1 = k1 < S ? k1 : S - 1;
            va[i] = *reinterpret_cast<const uint4*>(vp + (int64_t)k0 * row_stride + c * 8);
            vb[i] = *reinterpret_cast<const uint4*>(vp + (int64_t)k1 * row_stride + c * 8);
        }
    };
    auto stash = [&](int buf) {
        unsigned char* kb = lds[buf];
        unsigned char* vbuf = lds[buf] + KBYTES;
#pragma unroll
        for (int i = 0; i < KIT; ++i) {
            const int id = tid + 256 * i, row = id / CH, c = id % CH;
            *reinterpret_cast<uint4*>(kb + row * KROW + ((c ^ kswz<CH>(row)) << 4)) = kr[i];
        }
#pragma unroll
        for (int i = 0; i < VIT; ++i) {
            const int id = tid + 256 * i, pr = id / CH, c = id % CH;
            const int key = 2 * pr;                              // even key of the pair, 0..62
            const int w16 = key & 15;
            // position inside the block of 16: key = 8*hh + 4*gg + e  ->  8*gg + 4*hh + e
            const int pos = (key & ~15) + 8 * ((w16 >> 2) & 1) + 4 * ((w16 >> 3) & 1) + (w16 & 3);
            const int chunk = pos >> 3, inch = pos & 7;
            const u32x4 a4 = {va[i].x, va[i].y, va[i].z, va[i].w};
            const u32x4 b4 = {vb[i].x, vb[i].y, vb[i].z, vb[i].w};
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                const int dh = 8 * c + e;
                const uint32_t lo = (e & 1) ? (a4[e >> 1] >> 16) : (a4[e >> 1] & 0xFFFFu);
                const uint32_t hi = (e & 1) ? (b4[e >> 1] & 0xFFFF0000u) : (b4[e >> 1] << 16);
                *reinterpret_cast<uint32_t*>(vbuf + dh * 128 + ((chunk ^ vswz(dh)) << 4) + inch * 2) = lo | hi;
            }
        }
    };

    fetch(0);
    stash(0);
    __syncthreads();
    for (int t = 0; t < ntiles; ++t) {
        const int buf = t & 1;
        if (t + 1 < ntiles) fetch(t + 1);
        if (64 * t <= q0 + 31) {                                  // wave-uniform: tile not fully masked
            const unsigned char* kb = lds[buf];
            const unsigned char* vbuf = lds[buf] + KBYTES;
            f32x16 s[2];
#pragma unroll
            for (int kt = 0; kt < 2; ++kt) {
#pragma unroll
                for (int r = 0; r < 16; ++r) s[kt][r] = 0.0f;
                const int row = 32 * kt + j;
#pragma unroll
                for (int st = 0; st < DH / 16; ++st) {
                    const int c = 2 * st + g;
                    bf16x8 kf = *reinterpret_cast<const bf16x8*>(kb + row * KROW + ((c ^ kswz<CH>(row)) << 4));
                    s[kt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf, qf[st], s[kt], 0, 0, 0);
                }
            }
            const bool need_mask = 64 * t + 63 > q0;
            float mx = -INFINITY;
#pragma unroll
            for (int kt = 0; kt < 2; ++kt)
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const int key = 64 * t + 32 * kt + 8 * (r >> 2) + 4 * g + (r & 3);
                    float val = s[kt][r] * scale_log2e;
                    if (need_mask && key > qrow) val = -INFINITY;
                    s[kt][r] = val;
                    mx = fmaxf(mx, val);
                }
            mx = fmaxf(mx, __shfl_xor(mx, 32, 64));
            const float m_new = fmaxf(m_run, mx);
            const float alpha = __builtin_amdgcn_exp2f(m_run - m_new);
            float rs = 0.0f;
#pragma unroll
            for (int kt = 0; kt < 2; ++kt)
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const float p = __builtin_amdgcn_exp2f(s[kt][r] - m_new);
                    s[kt][r] = p;
                    rs += p;
                }
            rs += __shfl_xor(rs, 32, 64);
            l_run = l_run * alpha + rs;
            m_run = m_new;
#pragma unroll
            for (int tt = 0; tt < DH / 32; ++tt)
#pragma unroll
                for (int r = 0; r < 16; ++r) o[tt][r] *= alpha;
#pragma unroll
            for (int kt = 0; kt < 2; ++kt)
#pragma unroll
                for (int sp = 0; sp < 2; ++sp) {
                    u32x4 pu;
#pragma unroll
                    for (int e = 0; e < 4; ++e) pu[e] = zo_pack_bf16x2(s[kt][8 * sp + 2 * e], s[kt][8 * sp + 2 * e + 1]);
                    const bf16x8 pv = __builtin_bit_cast(bf16x8, pu);
                    const int chunk = 2 * (2 * kt + sp) + g;
#pragma unroll
                    for (int tt = 0; tt < DH / 32; ++tt) {
                        const int row = 32 * tt + j;
                        bf16x8 vf = *reinterpret_cast<const bf16x8*>(vbuf + row * 128 + ((chunk ^ vswz(row)) << 4));
                        o[tt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf, pv, o[tt], 0, 0, 0);
                    }
                }
        }
        if (t + 1 < ntiles) {
            stash(buf ^ 1);
            __syncthreads();
        }
    }
    if (qrow < S) {
        const float inv = 1.0f / l_run;
        zo_bf16* orow = out + ((int64_t)b * S + qrow) * ((int64_t)H * DH) + (int64_t)h * DH;
#pragma unroll
        for (int tt = 0; tt < DH / 32; ++tt)
#pragma unroll
            for (int rg = 0; rg < 4; ++rg) {
                const int dh = 32 * tt + 8 * rg + 4 * g;
                uint2 w;
                w.x = zo_pack_bf16x2(o[tt][4 * rg] * inv, o[tt][4 * rg + 1] * inv);
                w.y = zo_pack_bf16x2(o[tt][4 * rg + 2] * inv, o[tt][4 * rg + 3] * inv);
                *reinterpret_cast<uint2*>(orow + dh) = w;
            }
    }
}

bool zo_flash_attention_supported(int32_t dh, int dtype) { return dtype == ZO_T_BF16 && (dh == 64 || dh == 128); }

hipError_t zo_launch_flash_attention(const void* q, const void* k, const void* v, void* out,
                                     int32_t B, int32_t S, int32_t H, int32_t dh, int64_t row_stride, hipStream_t st)
{
    if (B == 0 || S == 0 || H == 0) return hipSuccess;
    const dim3 grid((S + 127) / 128, B * H);
    const float scale_log2e = (1.0f / sqrtf((float)dh)) * 1.4426950408889634f;
    if (dh == 128)
        zo_flash_attn_kernel<128><<<grid, 256, 0, st>>>((const zo_bf16*)q, (const zo_bf16*)k, (const zo_bf16*)v, (zo_bf16*)out, S, H, row_stride, scale_log2e);
    else if (dh == 64)
        zo_flash_attn_kernel<64><<<grid, 256, 0, st>>>((const zo_bf16*)q, (const zo_bf16*)k, (const zo_bf16*)v, (zo_bf16*)out, S, H, row_stride, scale_log2e);
    else
        return hipErrorInvalidValue;
    return hipGetLastError();
}
