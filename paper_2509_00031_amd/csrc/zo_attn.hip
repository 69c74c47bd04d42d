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
// V tiles lie in LDS as they lie in memory ([key][dh], copied like the K tiles); the V^T operand is
// read from them with the transposing LDS load of gfx950 (ds_read_b64_tr_b16: in a group of 16 lanes,
// source lane u points at 4 consecutive 16-bit elements of row u / 4, columns 4 (u % 4) ...; lane t
// receives column t of that 4 x 16 block), two loads per 8-key operand.  No transposed copy of V in HBM.
#include "zo_device.h"
#include "zo_internal.h"

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
typedef short s16x4 __attribute__((ext_vector_type(4)));

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
// chunk swizzles (16-byte chunks) of the 2*DH-byte K and V rows
template <int CH> __device__ __forceinline__ int kswz(int row)
{
    return CH == 16 ? (row & 15) : ((row ^ (row >> 3)) & 7);
}
// V: one transposing load touches keys k .. k+3 and k+8 .. k+11 (k a multiple of 4), 64 bytes of each; moving the
// 64-byte blocks of a row by the key spreads them over all banks (each 32-byte bank group is then hit twice, the minimum)
template <int CH> __device__ __forceinline__ int vswz(int row)
{
    return CH == 16 ? ((row & 3) << 2) : (((row >> 1) & 1) << 2);
}
// nested so that the compiler forms one v_max3_f32 (a flat max over pairs re-quiets every operand first)
__device__ __forceinline__ float max3(float a, float b, float c) { return fmaxf(fmaxf(a, b), c); }

}  // namespace

constexpr int HC = 8;    // heads per chunk of an XCD's work list (see the kernel)

template <int DH>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(2, 2)))
void zo_flash_attn_kernel(const zo_bf16* __restrict__ q, const zo_bf16* __restrict__ k, const zo_bf16* __restrict__ v,
                          zo_bf16* __restrict__ out, int S, int H, int BH, int64_t row_stride, float scale_log2e)
{
    constexpr int CH = DH / 8;                    // 16-byte chunks per K row
    constexpr int KROW = DH * 2;                  // bytes per K row in LDS
    constexpr int KBYTES = 64 * KROW;
    constexpr int STAGE = 2 * KBYTES;             // K tile, then V tile: 64 keys x DH each
    constexpr int KRPD = 1024 / KROW;             // rows per wave-level copy
    constexpr int KDPW = 64 / KRPD / 4;           // copies per wave, tile and operand
    __shared__ __attribute__((aligned(16))) unsigned char lds[2 * STAGE];

    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int j = lane & 31, g = lane >> 5;
    // Workgroups go round-robin over the 8 XCDs in launch order; the cost of a query tile grows with its index.
    // XCD x therefore takes (batch, head) pairs x, x + 8, ... whole (the query tiles of a head share its K / V
    // through that XCD's L2), in chunks of HC heads, within a chunk the longest query tiles first: every XCD gets
    // the same mix of tile lengths and the short tiles fill the tail.
    const int nqt = (S + 127) / 128;
    const int xcd = (int)blockIdx.x & 7, seq = (int)blockIdx.x >> 3;
    const int chunk = seq / (HC * nqt), rem = seq % (HC * nqt);
    const int qt = nqt - 1 - rem / HC;
    const int bh = (chunk * HC + rem % HC) * 8 + xcd;
    if (bh >= BH) return;                         // padding of the last chunk (whole workgroup, before any barrier)
    const int b = bh / H, h = bh % H;
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
    float m_run = -INFINITY, l_run = 0.0f;        // running max (raw scores) and sum

    const int kv_end = (qt * 128 + 128) < S ? (qt * 128 + 128) : S;
    const int ntiles = (kv_end + 63) / 64;

    // copy plan of this wave
    const uint32_t lds0 = __builtin_amdgcn_readfirstlane(lds_offset(lds));
    // V^T operand: lane = 16 G + u reads, as source lane u of its group, 4 dh of key 8 (G / 2) + u / 4 (+ 4 for the
    // second load) and receives 4 keys of dh 16 (G % 2) + u; the key's swizzle term is u / 4 whatever the tile row
    uint32_t vrd[DH / 32];
    {
        const int u = lane & 15, G = lane >> 4;
        const int krow = 8 * (G >> 1) + (u >> 2);
#pragma unroll
        for (int tt = 0; tt < DH / 32; ++tt) {
            const int c = 4 * tt + 2 * (G & 1) + ((u & 3) >> 1);
            vrd[tt] = (uint32_t)(krow * KROW + ((c ^ vswz<CH>(krow)) << 4) + (u & 1) * 8);
        }
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
#pragma unroll
        for (int i = 0; i < KDPW; ++i) {
            const int rb = wave * KDPW + i;
            const int row = rb * KRPD + lane / CH;
            int key = t * 64 + row;
            key = key < S ? key : S - 1;                           // such keys carry probability 0
            const int c = (lane % CH) ^ vswz<CH>(row);
            const uint32_t voff = (uint32_t)(((int64_t)key * row_stride + c * 8) * 2);
            lds_dma16(vp, voff, lds0 + stage * STAGE + KBYTES + rb * 1024);
        }
    };

    issue(0, 0);
    __builtin_amdgcn_s_waitcnt(0x0F70);
    __syncthreads();
    // The Q fragments are pinned here, before the loop: left to the compiler, their loads sink below the barrier and
    // the counter waits for them land inside the loop, where they would also wait for the copies of the next tile.
#pragma unroll
    for (int st = 0; st < DH / 16; ++st) asm volatile("" : "+v"(qf[st]));
    for (int t = 0; t < ntiles; ++t) {
        const int buf = t & 1;
        if (t + 1 < ntiles) issue(buf ^ 1, t + 1);
        if (64 * t <= q0 + 31) {                                  // wave-uniform: tile not fully masked
            const unsigned char* kb = lds + buf * STAGE;
            const unsigned char* vbuf = kb + KBYTES;
            f32x16 s[2];
            // Matrix phases run at raised wave priority: the SIMD's other wave (another workgroup, in another phase) then
            // slots its softmax arithmetic between this wave's matrix instructions instead of delaying them (+3..4 %).
            __builtin_amdgcn_s_setprio(2);
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
            __builtin_amdgcn_s_setprio(0);
            if (64 * t + 63 > q0) {                               // diagonal tile: causal mask (also keys >= S)
#pragma unroll
                for (int kt = 0; kt < 2; ++kt)
#pragma unroll
                    for (int r = 0; r < 16; ++r) {
                        const int key = 64 * t + 32 * kt + 8 * (r >> 2) + 4 * g + (r & 3);
                        if (key > qrow) s[kt][r] = -INFINITY;
                    }
            }
            // tile maximum of the lane's 32 scores, three operands per instruction, then over the query's two lanes
            float mx = max3(s[0][0], s[0][1], s[0][2]);
#pragma unroll
            for (int r = 3; r < 15; r += 2) mx = max3(mx, s[0][r], s[0][r + 1]);
            mx = max3(mx, s[0][15], s[1][0]);
#pragma unroll
            for (int r = 1; r < 15; r += 2) mx = max3(mx, s[1][r], s[1][r + 1]);
            mx = fmaxf(mx, s[1][15]);
            {
                const u32x2 h = __builtin_amdgcn_permlane32_swap(__float_as_uint(mx), __float_as_uint(mx), false, false);
                mx = fmaxf(__uint_as_float(h[0]), __uint_as_float(h[1]));
            }
            // The reference point m_run of the exponentials only follows the maximum when some query's maximum has
            // outgrown it by more than 2^8 (probabilities stay below 256; the reference cancels in O / l): the pass
            // over the output accumulators is then rare instead of once per tile.
            if (__builtin_amdgcn_ballot_w64((mx - m_run) * scale_log2e > 8.0f) != 0) {
                const float m_new = fmaxf(m_run, mx);
                const float alpha = __builtin_amdgcn_exp2f((m_run - m_new) * scale_log2e);
                l_run *= alpha;
#pragma unroll
                for (int tt = 0; tt < DH / 32; ++tt)
#pragma unroll
                    for (int r = 0; r < 16; ++r) o[tt][r] *= alpha;
                m_run = m_new;
            }
            const float neg_m = -m_run * scale_log2e;
            float rs = 0.0f;
#pragma unroll
            for (int kt = 0; kt < 2; ++kt)
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const float p = __builtin_amdgcn_exp2f(__builtin_fmaf(s[kt][r], scale_log2e, neg_m));
                    s[kt][r] = p;
                    rs += p;
                }
            {
                const u32x2 h = __builtin_amdgcn_permlane32_swap(__float_as_uint(rs), __float_as_uint(rs), false, false);
                rs = __uint_as_float(h[0]) + __uint_as_float(h[1]);
            }
            l_run += rs;
            __builtin_amdgcn_s_setprio(2);
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
                    const unsigned char* vk = vbuf + (32 * kt + 16 * sp) * KROW;
#pragma unroll
                    for (int tt = 0; tt < DH / 32; ++tt) {
                        typedef __attribute__((address_space(3))) s16x4 lds_s16x4;
                        const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4*)(vk + vrd[tt]));
                        const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4*)(vk + vrd[tt] + 4 * KROW));
                        const u32x4 vu = {__builtin_bit_cast(u32x2, lo)[0], __builtin_bit_cast(u32x2, lo)[1],
                                          __builtin_bit_cast(u32x2, hi)[0], __builtin_bit_cast(u32x2, hi)[1]};
                        o[tt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, vu), pv, o[tt], 0, 0, 0);
                    }
                }
            __builtin_amdgcn_s_setprio(0);
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

hipError_t zo_launch_flash_attention(const void* q, const void* k, const void* v, void* out,
                                     int32_t B, int32_t S, int32_t H, int32_t dh, int64_t row_stride, hipStream_t st)
{
    if (B == 0 || S == 0 || H == 0) return hipSuccess;
    // 32-bit byte offsets inside one (batch, head) slice
    if ((int64_t)S * row_stride * 2 >= ((int64_t)1 << 32)) return hipErrorInvalidValue;
    // 8 XCDs x chunks of HC heads x query tiles (the kernel's own numbering; pairs past B*H exit at once)
    const int64_t nwg = (int64_t)8 * (((int64_t)B * H + 8 * HC - 1) / (8 * HC)) * HC * ((S + 127) / 128);
    if (nwg >= ((int64_t)1 << 31)) return hipErrorInvalidValue;
    const dim3 grid((unsigned)nwg);
    const float scale_log2e = (1.0f / sqrtf((float)dh)) * 1.4426950408889634f;
    if (dh == 128)
        zo_flash_attn_kernel<128><<<grid, 256, 0, st>>>((const zo_bf16*)q, (const zo_bf16*)k, (const zo_bf16*)v, (zo_bf16*)out,
                                                        S, H, B * H, row_stride, scale_log2e);
    else if (dh == 64)
        zo_flash_attn_kernel<64><<<grid, 256, 0, st>>>((const zo_bf16*)q, (const zo_bf16*)k, (const zo_bf16*)v, (zo_bf16*)out,
                                                       S, H, B * H, row_stride, scale_log2e);
    else
        return hipErrorInvalidValue;
    return hipGetLastError();
}
