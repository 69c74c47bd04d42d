// Causal softmax attention on the gfx950 matrix cores (bf16 storage, head dimension 64 or 128).
//
// One workgroup = 4 waves = 128 consecutive queries of one (batch, head); a wave owns 32 queries.
// Keys / values stream through LDS in tiles of 64 keys, copied global -> LDS by the load unit
// (16 bytes per lane, no staging registers), two stages.  Both matrix products are issued
// "transposed" so that a lane owns ONE query (column lane % 32) in every accumulator:
//     S^T[key][query] = K[key][:] . Q[query][:]          (A = K tile rows, B = Q rows in registers)
//     O^T[dh][query] += V^T[dh][key] . P^T[key][query]   (A = V^T tile rows, B = P)
// so the running max / sum of the online softmax are per-lane scalars (the other half of a
// query's keys lives in lane ^ 32).  The S accumulator of lane group g = lane / 32 holds keys
// 8*(r/4) + 4*g + r%4 of a 32-key block; one v_permlane32_swap per register pair regroups them
// into 8 consecutive keys per lane group, which is what the second product wants as its B operand.
// V is transposed once per call by a small kernel (V^T[b,h][dh][key], keys padded to a multiple of
// 64 with zeros) so that its tiles can be copied like the K tiles.
#include "zo_device.h"
#include "zo_internal.h"

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

namespace {

__device__ __forceinline__ uint32_t lds_offset(const void* p)
{
    return (uint32_t)(uintptr_t)(__attribute__((address_space(3))) const void*)p;
}
// one wave-level 1 KB copy: lane fetches 16 bytes at base + voff, LDS destination dst + lane*16
__device__ __forceinline__ void lds_dma16(const void* base, uint32_t voff, uint32_t dst)
{
    asm volatile("s_mov_b32 m0, %0\n\tglobal_load_lds_dwordx4 %1, %2\n" ::"s"(dst), "v"(voff), "s"(base) : "memory");
}
// chunk swizzles (16-byte chunks): K rows are 2*DH bytes, V^T rows 128 bytes
template <int CH> __device__ __forceinline__ int kswz(int row)
{
    return CH == 16 ? (row & 15) : ((row ^ (row >> 3)) & 7);
}
__device__ __forceinline__ int vswz(int row) { return (row ^ (row >> 3)) & 7; }

}  // namespace

// V[b*S + key][h*DH + i] (row stride in elements) -> VT[(b*H + h)*DH + i][key], key < S_pad, zero padded
template <int DH>
__global__ __launch_bounds__(256) void zo_transpose_v_kernel(const zo_bf16* __restrict__ v, zo_bf16* __restrict__ vt,
                                                             int S, int S_pad, int H, int64_t row_stride)
{
    __shared__ uint16_t tile[64][DH + 2];
    const int t0 = blockIdx.x * 64;
    const int b = blockIdx.y / H, h = blockIdx.y % H;
    const uint16_t* src = reinterpret_cast<const uint16_t*>(v) + (int64_t)b * S * row_stride + (int64_t)h * DH;
    for (int idx = threadIdx.x; idx < 64 * DH / 2; idx += 256) {
        const int r = idx / (DH / 2), c = (idx % (DH / 2)) * 2;
        uint32_t w = 0;
        if (t0 + r < S) w = *reinterpret_cast<const uint32_t*>(src + (int64_t)(t0 + r) * row_stride + c);
        tile[r][c] = (uint16_t)(w & 0xFFFFu);
        tile[r][c + 1] = (uint16_t)(w >> 16);
    }
    __syncthreads();
    uint16_t* dst = reinterpret_cast<uint16_t*>(vt) + (int64_t)blockIdx.y * DH * S_pad + t0;
    for (int idx = threadIdx.x; idx < DH * 32; idx += 256) {
        const int i = idx / 32, kk = (idx % 32) * 2;
        const uint32_t w = (uint32_t)tile[kk][i] | ((uint32_t)tile[kk + 1][i] << 16);
        *reinterpret_cast<uint32_t*>(dst + (int64_t)i * S_pad + kk) = w;
    }
}

template <int DH>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(2, 2)))
void zo_flash_attn_kernel(const zo_bf16* __restrict__ q, const zo_bf16* __restrict__ k, const zo_bf16* __restrict__ vt,
                          zo_bf16* __restrict__ out, int S, int S_pad, int H, int64_t row_stride, float scale_log2e)
{
    constexpr int CH = DH / 8;                    // 16-byte chunks per K row
    constexpr int KROW = DH * 2;                  // bytes per K row in LDS
    constexpr int KBYTES = 64 * KROW;
    constexpr int VBYTES = DH * 128;              // V^T tile: DH rows x 64 keys x 2 B
    constexpr int STAGE = KBYTES + VBYTES;
    constexpr int KRPD = 1024 / KROW;             // K rows per wave-level copy
    constexpr int KDPW = 64 / KRPD / 4;           // K copies per wave per tile
    constexpr int VDPW = DH / 8 / 4;              // V^T copies per wave per tile (8 rows each)
    __shared__ __attribute__((aligned(16))) unsigned char lds[2 * STAGE];

    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int j = lane & 31, g = lane >> 5;
    const int nqt = (S + 127) / 128;
    const int qt = nqt - 1 - (int)blockIdx.x;     // longest rows first
    const int b = blockIdx.y / H, h = blockIdx.y % H;
    const int q0 = qt * 128 + wave * 32;
    const int qrow = q0 + j;
    const zo_bf16* qp = q + (int64_t)b * S * row_stride + (int64_t)h * DH;
    const zo_bf16* kp = k + (int64_t)b * S * row_stride + (int64_t)h * DH;
    const zo_bf16* vp = vt + (int64_t)blockIdx.y * DH * S_pad;

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
    float m_run = -INFINITY, l_run = 0.0f;        // running max (raw scores) and sum

    const int kv_end = (qt * 128 + 128) < S ? (qt * 128 + 128) : S;
    const int ntiles = (kv_end + 63) / 64;

    // copy plan of this wave
    const uint32_t lds0 = __builtin_amdgcn_readfirstlane(lds_offset(lds));
    uint32_t voff_v[VDPW];
#pragma unroll
    for (int i = 0; i < VDPW; ++i) {
        const int row = (wave * VDPW + i) * 8 + (lane >> 3);       // dh row
        const int c = (lane & 7) ^ vswz(row);
        voff_v[i] = (uint32_t)(((int64_t)row * S_pad + c * 8) * 2);
    }
    auto issue = [&](int stage, int t) {
#pragma unroll
        for (int i = 0; i < KDPW; ++i) {
            const int rb = wave * KDPW + i;
            const int row = rb * KRPD + lane / CH;                 // key row inside the tile
            int key = t * 64 + row;
            key = key < S ? key : S - 1;
            const int c = (lane % CH) ^ kswz<CH>(row);
            const uint32_t voff = (uint32_t)(((int64_t)key * row_stride + c * 8) * 2);
            lds_dma16(kp, voff, lds0 + stage * STAGE + rb * 1024);
        }
        const zo_bf16* vb = vp + t * 64;
#pragma unroll
        for (int i = 0; i < VDPW; ++i)
            lds_dma16(vb, voff_v[i], lds0 + stage * STAGE + KBYTES + (wave * VDPW + i) * 1024);
    };

    issue(0, 0);
    __builtin_amdgcn_s_waitcnt(0x0F70);
    __syncthreads();
    for (int t = 0; t < ntiles; ++t) {
        const int buf = t & 1;
        if (t + 1 < ntiles) issue(buf ^ 1, t + 1);
        if (64 * t <= q0 + 31) {                                  // wave-uniform: tile not fully masked
            const unsigned char* kb = lds + buf * STAGE;
            const unsigned char* vbuf = kb + KBYTES;
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
            if (64 * t + 63 > q0) {                               // diagonal tile: causal mask (also keys >= S)
#pragma unroll
                for (int kt = 0; kt < 2; ++kt)
#pragma unroll
                    for (int r = 0; r < 16; ++r) {
                        const int key = 64 * t + 32 * kt + 8 * (r >> 2) + 4 * g + (r & 3);
                        if (key > qrow) s[kt][r] = -INFINITY;
                    }
            }
            float mx = fmaxf(s[0][0], s[1][0]);
#pragma unroll
            for (int r = 1; r < 16; ++r) mx = fmaxf(mx, fmaxf(s[0][r], s[1][r]));
            mx = fmaxf(mx, __shfl_xor(mx, 32, 64));
            const float m_new = fmaxf(m_run, mx);
            const float neg_m = -m_new * scale_log2e;
            float rs = 0.0f;
#pragma unroll
            for (int kt = 0; kt < 2; ++kt)
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const float p = __builtin_amdgcn_exp2f(__builtin_fmaf(s[kt][r], scale_log2e, neg_m));
                    s[kt][r] = p;
                    rs += p;
                }
            rs += __shfl_xor(rs, 32, 64);
            if (__builtin_amdgcn_ballot_w64(m_new != m_run) != 0) {   // some query's max moved: rescale
                const float alpha = __builtin_amdgcn_exp2f((m_run - m_new) * scale_log2e);
                l_run *= alpha;
#pragma unroll
                for (int tt = 0; tt < DH / 32; ++tt)
#pragma unroll
                    for (int r = 0; r < 16; ++r) o[tt][r] *= alpha;
            }
            l_run += rs;
            m_run = m_new;
#pragma unroll
            for (int kt = 0; kt < 2; ++kt)
#pragma unroll
                for (int sp = 0; sp < 2; ++sp) {
                    // registers 8sp..8sp+3 hold keys 16sp + 4g + e, registers 8sp+4..8sp+7 keys 16sp + 8 + 4g + e
                    const uint32_t a0 = zo_pack_bf16x2(s[kt][8 * sp + 0], s[kt][8 * sp + 1]);
                    const uint32_t a1 = zo_pack_bf16x2(s[kt][8 * sp + 2], s[kt][8 * sp + 3]);
                    const uint32_t b0 = zo_pack_bf16x2(s[kt][8 * sp + 4], s[kt][8 * sp + 5]);
                    const uint32_t b1 = zo_pack_bf16x2(s[kt][8 * sp + 6], s[kt][8 * sp + 7]);
                    // upper lanes of a* <-> lower lanes of b*: lane group g then holds keys 16sp + 8g .. + 7
                    const u32x2 x0 = __builtin_amdgcn_permlane32_swap(a0, b0, false, false);
                    const u32x2 x1 = __builtin_amdgcn_permlane32_swap(a1, b1, false, false);
                    const u32x4 pu = {x0[0], x1[0], x0[1], x1[1]};
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
        __builtin_amdgcn_s_waitcnt(0x0F70);       // vmcnt(0): own copies of tile t+1 have landed
        __syncthreads();
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

size_t zo_flash_attention_scratch_bytes(int32_t B, int32_t S, int32_t H, int32_t dh)
{
    const size_t s_pad = ((size_t)S + 63) / 64 * 64;
    return (size_t)B * H * dh * s_pad * 2;
}

hipError_t zo_launch_flash_attention(const void* q, const void* k, const void* v, void* out, void* scratch,
                                     int32_t B, int32_t S, int32_t H, int32_t dh, int64_t row_stride, hipStream_t st)
{
    if (B == 0 || S == 0 || H == 0) return hipSuccess;
    const int s_pad = (S + 63) / 64 * 64;
    // 32-bit byte offsets inside one (batch, head) slice
    if ((int64_t)S * row_stride * 2 >= ((int64_t)1 << 32) || (int64_t)dh * s_pad * 2 >= ((int64_t)1 << 32)) return hipErrorInvalidValue;
    const dim3 tgrid(s_pad / 64, B * H);
    const dim3 grid((S + 127) / 128, B * H);
    const float scale_log2e = (1.0f / sqrtf((float)dh)) * 1.4426950408889634f;
    if (dh == 128) {
        zo_transpose_v_kernel<128><<<tgrid, 256, 0, st>>>((const zo_bf16*)v, (zo_bf16*)scratch, S, s_pad, H, row_stride);
        zo_flash_attn_kernel<128><<<grid, 256, 0, st>>>((const zo_bf16*)q, (const zo_bf16*)k, (const zo_bf16*)scratch, (zo_bf16*)out,
                                                        S, s_pad, H, row_stride, scale_log2e);
    } else if (dh == 64) {
        zo_transpose_v_kernel<64><<<tgrid, 256, 0, st>>>((const zo_bf16*)v, (zo_bf16*)scratch, S, s_pad, H, row_stride);
        zo_flash_attn_kernel<64><<<grid, 256, 0, st>>>((const zo_bf16*)q, (const zo_bf16*)k, (const zo_bf16*)scratch, (zo_bf16*)out,
                                                       S, s_pad, H, row_stride, scale_log2e);
    } else {
        return hipErrorInvalidValue;
    }
    return hipGetLastError();
}
