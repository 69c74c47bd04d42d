// GEMM of the quantized linears: Y[M][N] = X[M][K] * W[N][K]^T, both operands already
// de-quantized (X^ by the per-token quantizer, W^ = Q(W +- eps u) by the weight fake-quantizer).
// bf16 operands run on the gfx950 matrix cores (v_mfma_f32_32x32x16_bf16, fp32 accumulate);
// fp32 operands (parity mode) use a plain LDS-tiled FMA kernel.
#include "zo_device.h"
#include "zo_internal.h"
#include <cstdlib>
#include <type_traits>

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

// ---------------------------------------------------------------------------------------------
// bf16 MFMA kernel.
//   workgroup = 256 threads = 4 waves as 2 (m) x 2 (n); block tile BM x BN, K step 64.
//   LDS tile rows are 64 bf16 = 128 B = eight 16-byte chunks; chunk c of row r is stored at
//   chunk slot c ^ f(r), f(r) = (r + (r >> 3)) & 7, which spreads the 16-byte fragment reads of
//   32 consecutive rows over all banks.  Two LDS buffers: the next K tile is fetched from global
//   memory into registers while the current one feeds the matrix cores.
//   The matrix instruction is issued with W as its first operand and X as its second, so each
//   lane ends up with 4 consecutive n of one row m: outputs are stored as 8- or 16-byte vectors.
// ---------------------------------------------------------------------------------------------
template <int BM, int BN> struct gemm_cfg {
    static constexpr int BK = 64;
    static constexpr int WM = BM / 2, WN = BN / 2;
    static constexpr int TM = WM / 32, TN = WN / 32;
    static constexpr int XCH = BM * 8 / 256;         // 16-byte chunks per thread for the X tile
    static constexpr int WCH = BN * 8 / 256;
    static constexpr int LDS_BYTES = 2 * (BM + BN) * 128;
};

__device__ __forceinline__ int swz(int row) { return (row + (row >> 3)) & 7; }

template <int BM, int BN, typename TY>
__global__ __launch_bounds__(256) void zo_gemm_bf16_kernel(zo_gemm_args a)
{
    using C = gemm_cfg<BM, BN>;
    extern __shared__ __attribute__((aligned(16))) unsigned char lds[];
    // buffer b: X tile at b*(BM+BN)*128, W tile right after it
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave >> 1, wn = wave & 1;
    const int M = a.M, N = a.N, K = a.K;
    const int tiles_n = (N + BN - 1) / BN;
    const int tile_m = blockIdx.x / tiles_n, tile_n = blockIdx.x % tiles_n;
    const int m0 = tile_m * BM, n0 = tile_n * BN;
    const int bz = blockIdx.z;
    const zo_bf16* X = (const zo_bf16*)a.X + bz * a.strideX;
    const zo_bf16* W = (const zo_bf16*)a.W + bz * a.strideW;

    // global -> register staging: thread owns chunk (row = tid/8 + 32*i, c = tid%8)
    const int lrow = tid >> 3, lc = tid & 7;
    uint4 xr[C::XCH], wr[C::WCH];
    auto fetch = [&](int kt) {
        const int k = kt * C::BK + lc * 8;
        const bool kin = k < K;
#pragma unroll
        for (int i = 0; i < C::XCH; ++i) {
            int r = m0 + lrow + 32 * i;
            r = r < M ? r : M - 1;
            xr[i] = kin ? *reinterpret_cast<const uint4*>(X + (int64_t)r * K + k) : make_uint4(0, 0, 0, 0);
        }
#pragma unroll
        for (int i = 0; i < C::WCH; ++i) {
            int r = n0 + lrow + 32 * i;
            r = r < N ? r : N - 1;
            wr[i] = kin ? *reinterpret_cast<const uint4*>(W + (int64_t)r * K + k) : make_uint4(0, 0, 0, 0);
        }
    };
    auto stash = [&](int buf) {
        unsigned char* xb = lds + buf * (BM + BN) * 128;
        unsigned char* wb = xb + BM * 128;
#pragma unroll
        for (int i = 0; i < C::XCH; ++i) {
            int r = lrow + 32 * i;
            *reinterpret_cast<uint4*>(xb + r * 128 + ((lc ^ swz(r)) << 4)) = xr[i];
        }
#pragma unroll
        for (int i = 0; i < C::WCH; ++i) {
            int r = lrow + 32 * i;
            *reinterpret_cast<uint4*>(wb + r * 128 + ((lc ^ swz(r)) << 4)) = wr[i];
        }
    };

    f32x16 acc[C::TN][C::TM];
#pragma unroll
    for (int i = 0; i < C::TN; ++i)
#pragma unroll
        for (int j = 0; j < C::TM; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.0f;

    const int nk = (K + C::BK - 1) / C::BK;
    fetch(0);
    stash(0);
    __syncthreads();
    for (int kt = 0; kt < nk; ++kt) {
        const int buf = kt & 1;
        if (kt + 1 < nk) fetch(kt + 1);
        const unsigned char* xb = lds + buf * (BM + BN) * 128;
        const unsigned char* wb = xb + BM * 128;
#pragma unroll
        for (int ks = 0; ks < 4; ++ks) {
            const int c = 2 * ks + (lane >> 5);
            bf16x8 xf[C::TM], wf[C::TN];
#pragma unroll
            for (int j = 0; j < C::TM; ++j) {
                int r = wm * C::WM + j * 32 + (lane & 31);
                xf[j] = *reinterpret_cast<const bf16x8*>(xb + r * 128 + ((c ^ swz(r)) << 4));
            }
#pragma unroll
            for (int i = 0; i < C::TN; ++i) {
                int r = wn * C::WN + i * 32 + (lane & 31);
                wf[i] = *reinterpret_cast<const bf16x8*>(wb + r * 128 + ((c ^ swz(r)) << 4));
            }
#pragma unroll
            for (int i = 0; i < C::TN; ++i)
#pragma unroll
                for (int j = 0; j < C::TM; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wf[i], xf[j], acc[i][j], 0, 0, 0);
        }
        if (kt + 1 < nk) {
            stash(buf ^ 1);          // the other buffer was last read before the previous barrier
            __syncthreads();
        }
    }

    // epilogue: lane holds, per 32x32 tile, rows n = 8*(r/4) + 4*(lane/32) + r%4 of column m = lane%32
    TY* Y = (TY*)a.Y + bz * a.strideY;
    const float* bias = a.bias ? a.bias + bz * a.strideBias : nullptr;
    const zo_bf16* res = a.residual ? (const zo_bf16*)a.residual + bz * a.strideRes : nullptr;
    const bool vec_ok = (N & 3) == 0;
#pragma unroll
    for (int j = 0; j < C::TM; ++j) {
        const int m = m0 + wm * C::WM + j * 32 + (lane & 31);
        if (m >= M) continue;
#pragma unroll
        for (int i = 0; i < C::TN; ++i) {
#pragma unroll
            for (int rg = 0; rg < 4; ++rg) {
                const int n = n0 + wn * C::WN + i * 32 + rg * 8 + (lane >> 5) * 4;
                if (n >= N) continue;
                float v[4];
#pragma unroll
                for (int e = 0; e < 4; ++e) v[e] = acc[i][j][rg * 4 + e];
                const int64_t off = (int64_t)m * N + n;
                if (vec_ok && n + 3 < N) {
                    if (bias) {
                        float4 b4 = *reinterpret_cast<const float4*>(bias + n);
                        v[0] += b4.x; v[1] += b4.y; v[2] += b4.z; v[3] += b4.w;
                    }
                    if (a.relu) {
#pragma unroll
                        for (int e = 0; e < 4; ++e) v[e] = fmaxf(v[e], 0.0f);
                    }
                    if (res) {
                        uint2 r2 = *reinterpret_cast<const uint2*>(res + off);
                        v[0] += zo_bf16_lo(r2.x); v[1] += zo_bf16_hi(r2.x);
                        v[2] += zo_bf16_lo(r2.y); v[3] += zo_bf16_hi(r2.y);
                    }
                    if constexpr (sizeof(TY) == 4) {
                        *reinterpret_cast<float4*>((float*)Y + off) = make_float4(v[0], v[1], v[2], v[3]);
                    } else {
                        uint2 o;
                        o.x = zo_pack_bf16x2(v[0], v[1]);
                        o.y = zo_pack_bf16x2(v[2], v[3]);
                        *reinterpret_cast<uint2*>((zo_bf16*)Y + off) = o;
                    }
                } else {
                    for (int e = 0; e < 4 && n + e < N; ++e) {
                        float t = v[e];
                        if (bias) t += bias[n + e];
                        if (a.relu) t = fmaxf(t, 0.0f);
                        if (res) t += (float)res[off + e];
                        zo_store(Y + off + e, t);
                    }
                }
            }
        }
    }
}

// ---------------------------------------------------------------------------------------------
// bf16 MFMA kernel, large shapes (K a multiple of BK): 256 x 256 tile, NW waves, ST LDS stages.
// The K tiles are copied global -> LDS by the load unit itself (16 bytes per lane, no staging
// registers): one wave-level copy fills 1 KB of a stage = 1024 / (2 BK) tile rows, lane L landing
// in row L / CPR, chunk slot L % CPR (CPR = 16-byte chunks per row); the lane fetches global chunk
// slot ^ f(row) to realise the bank swizzle.  ST - 1 K tiles are in flight while one feeds the
// matrix cores; the wait at the end of a tile only covers the oldest of them.
// Workgroups are renumbered so that each of the 8 XCDs (blockIdx % 8) works on a contiguous
// range of tiles, visited in groups of 8 m-tiles, which keeps operand tiles hot in that XCD's L2.
// ---------------------------------------------------------------------------------------------
__device__ __forceinline__ uint32_t lds_offset(const void* p)
{
    return (uint32_t)(uintptr_t)(__attribute__((address_space(3))) const void*)p;
}
// one wave-level 1 KB copy: lane fetches 16 bytes at base + voff, LDS destination dst + lane*16
__device__ __forceinline__ void lds_dma16(const void* base, uint32_t voff, uint32_t dst)
{
    asm volatile("s_mov_b32 m0, %0\n\tglobal_load_lds_dwordx4 %1, %2\n" ::"s"(dst), "v"(voff), "s"(base) : "memory");
}
template <int BK> __device__ __forceinline__ int swz_bk(int row)
{
    return BK == 64 ? ((row ^ (row >> 3)) & 7) : (((row >> 1) & 3) ^ ((row >> 3) & 1));
}
// s_waitcnt vmcnt(n) only (expcnt / lgkmcnt left at their maxima)
template <int N> __device__ __forceinline__ void wait_vmcnt()
{
    __builtin_amdgcn_s_waitcnt(0x0F70 | (N & 15) | ((N >> 4) << 14));
}

// epilogue of one 32 x 32 accumulator tile: lane holds rows n = nb + 8*(r/4) + r%4 (nb includes
// the 4*(lane/32) term) of column m
template <typename TY>
__device__ __forceinline__ void store_tile(const f32x16& acc, const zo_gemm_args& a, TY* Y, const float* bias,
                                           const zo_bf16* res, int m, int nb)
{
    const int M = a.M, N = a.N;
    if (m >= M) return;
    const bool vec_ok = (N & 3) == 0;
#pragma unroll
    for (int rg = 0; rg < 4; ++rg) {
        const int n = nb + rg * 8;
        if (n >= N) continue;
        float v[4];
#pragma unroll
        for (int e = 0; e < 4; ++e) v[e] = acc[rg * 4 + e];
        const int64_t off = (int64_t)m * N + n;
        if (vec_ok && n + 3 < N) {
            if (bias) {
                float4 b4 = *reinterpret_cast<const float4*>(bias + n);
                v[0] += b4.x; v[1] += b4.y; v[2] += b4.z; v[3] += b4.w;
            }
            if (a.relu) {
#pragma unroll
                for (int e = 0; e < 4; ++e) v[e] = fmaxf(v[e], 0.0f);
            }
            if (res) {
                uint2 r2 = *reinterpret_cast<const uint2*>(res + off);
                v[0] += zo_bf16_lo(r2.x); v[1] += zo_bf16_hi(r2.x);
                v[2] += zo_bf16_lo(r2.y); v[3] += zo_bf16_hi(r2.y);
            }
            if constexpr (sizeof(TY) == 4) {
                *reinterpret_cast<float4*>((float*)Y + off) = make_float4(v[0], v[1], v[2], v[3]);
            } else {
                uint2 o;
                o.x = zo_pack_bf16x2(v[0], v[1]);
                o.y = zo_pack_bf16x2(v[2], v[3]);
                *reinterpret_cast<uint2*>((zo_bf16*)Y + off) = o;
            }
        } else {
            for (int e = 0; e < 4 && n + e < N; ++e) {
                float t = v[e];
                if (bias) t += bias[n + e];
                if (a.relu) t = fmaxf(t, 0.0f);
                if (res) t += (float)res[off + e];
                zo_store(Y + off + e, t);
            }
        }
    }
}

// SWIGLU (bf16 output only): the rows of W are the gate and up projections interleaved in blocks of 32 channels
// (32 gate rows, the 32 up rows of the same channels, ...), so the two 32 x 32 accumulator tiles a wave holds side
// by side along n are gate and up of the same (m, channel) in the same lane and register; the epilogue rounds both
// to the storage type (as if they had been stored), forms silu(gate) * up and writes Y[M][N/2].
// EPI = 2 (bf16 output, head dimension 128): the rows of W are the fused q | k | v projections with the four 32-row
// blocks of every head in the order [0, 2, 1, 3], so the two n-tiles of a wave hold dimensions i and i + 64 of the same
// head -- the pair the rotary embedding mixes -- in the same lane and register.  Columns below rope_cols (q and k) are
// rounded to the storage type, rotated by the angle table (position = row % rope_S) exactly as the stand-alone
// kernel does, and every column is written back in its natural place.
// EPI = 3 (lm_head): no output matrix at all.  A lane holds 32 logits of one token per 32-row block; per token and
// 256-column tile the maximum and the sum of exp(logit - maximum) are formed (lane, its partner half, then the four
// waves along n through LDS) and written to ce_part, and the lane that holds the token's target column writes that
// logit to ce_tgt.  The cross entropy of a row is then a 2 * tiles_n-float reduction instead of a pass over V logits.
// BT = 128 (4 waves, 64 x 64 per wave, two workgroups per CU) is the form for shapes with too few 256 x 256 tiles to
// fill the chip; it has the plain epilogue only.
template <typename TY, int NW, int BK, int ST, int EPI = 0, int BT = 256>
__global__ __launch_bounds__(NW * 64) void zo_gemm_bf16_dma_kernel(zo_gemm_args a)
{
    constexpr int BM = BT, BN = BT;
    static_assert(BT == 256 || (BT == 128 && NW == 4 && EPI == 0), "tile forms");
    constexpr int RB = BK * 2;                       // bytes per tile row
    constexpr int CPR = RB / 16;                     // 16-byte chunks per row
    constexpr int STAGE = (BM + BN) * RB;            // bytes per LDS stage
    constexpr int RPD = 1024 / RB;                   // tile rows per wave-level copy
    constexpr int DPW = (BM + BN) / RPD / NW;        // copies per wave per stage
    constexpr int WN_WAVES = NW / 2;                 // waves along n (2 along m)
    constexpr int WM = BM / 2, WN = BN / WN_WAVES;
    constexpr int TM = WM / 32, TN = WN / 32;
    constexpr int KS = BK / 16;                      // MFMA K steps per stage
    extern __shared__ __attribute__((aligned(16))) unsigned char lds[];
    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm = wave / WN_WAVES, wn = wave % WN_WAVES;
    const int M = a.M, N = a.N, LDK = a.K;            // LDK: row pitch of both operands
    int K = a.K, bz = blockIdx.z, krange = 0;         // K: length of this workgroup's K range
    if constexpr (BT == 128 && sizeof(TY) == 4) {
        if (a.kspl > 1) {                             // blockIdx.z = batch entry * kspl + range
            krange = __builtin_amdgcn_readfirstlane(bz % a.kspl);   // (divisions run in the vector unit)
            bz = __builtin_amdgcn_readfirstlane(bz / a.kspl);
            K = __builtin_amdgcn_readfirstlane(a.K / a.kspl);
        }
    }
    const int tiles_m = (M + BM - 1) / BM, tiles_n = (N + BN - 1) / BN;
    // XCD-aware renumbering, then grouped (8 m-tiles) ordering
    int vid = blockIdx.x;
    const int nblk = gridDim.x;
    if ((nblk & 7) == 0) vid = (vid & 7) * (nblk >> 3) + (vid >> 3);
    const int group_sz = 8 * tiles_n;
    const int grp = vid / group_sz;
    const int first_m = grp * 8;
    const int gm = (tiles_m - first_m) < 8 ? (tiles_m - first_m) : 8;
    const int tile_m = first_m + (vid % group_sz) % gm;
    const int tile_n = (vid % group_sz) / gm;
    const int m0 = tile_m * BM, n0 = tile_n * BN;
    const zo_bf16* X = (const zo_bf16*)a.X + bz * a.strideX + krange * K;
    const zo_bf16* W = (const zo_bf16*)a.W + bz * a.strideW + krange * K;

    // copy plan: (BM + BN) / RPD row-blocks per stage (X rows first, then W rows)
    const int lrow = lane / CPR, slot = lane % CPR;
    uint32_t voff[DPW];
#pragma unroll
    for (int i = 0; i < DPW; ++i) {
        const int rb = wave * DPW + i;
        const bool isw = rb >= BM / RPD;
        const int trow = (isw ? rb - BM / RPD : rb) * RPD + lrow;   // row inside the operand tile
        int grow = (isw ? n0 : m0) + trow;
        const int lim = isw ? N : M;
        grow = grow < lim ? grow : lim - 1;
        const int c = slot ^ swz_bk<BK>(trow);
        voff[i] = (uint32_t)(((int64_t)grow * LDK + c * 8) * 2);
    }
    const uint32_t lds0 = __builtin_amdgcn_readfirstlane(lds_offset(lds));
    auto issue = [&](int stage, int kt) {
        const zo_bf16* xb = X + kt * BK;
        const zo_bf16* wb = W + kt * BK;
#pragma unroll
        for (int i = 0; i < DPW; ++i) {
            const int rb = wave * DPW + i;
            const uint32_t dst = lds0 + stage * STAGE + rb * 1024;
            lds_dma16(rb >= BM / RPD ? (const void*)wb : (const void*)xb, voff[i], dst);
        }
    };

    f32x16 acc[TN][TM];
#pragma unroll
    for (int i = 0; i < TN; ++i)
#pragma unroll
        for (int j = 0; j < TM; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.0f;

    auto issue_one = [&](int stage, int kt, int i) {
        const int rb = wave * DPW + i;
        const uint32_t dst = lds0 + stage * STAGE + rb * 1024;
        lds_dma16(rb >= BM / RPD ? (const void*)(W + kt * BK) : (const void*)(X + kt * BK), voff[i], dst);
    };
    // Pipeline.  Stage t % ST holds K tile t.  Before the MFMAs of the LAST K step of tile t (whose
    // fragments are already in registers) the workgroup synchronises: tile t + 1 has landed for
    // everybody and stage t % ST is free.  The first fragments of tile t + 1 are read, and the
    // copies of tile t + ST into the freed stage are issued, while those last MFMAs run, so neither
    // the barrier nor the LDS latency after it leaves the matrix cores without issued work.
    // With two stages all copies of a tile are issued in that last K step (they are needed one tile
    // later); with more stages they are spread over the KS steps that follow the barrier.
    constexpr int SPAN = ST == 2 ? 1 : KS;            // K steps over which one tile's copies are issued
    constexpr int CPS = DPW / SPAN;                   // copies per K step
    constexpr int Q = CPS < TN * TM ? CPS : TN * TM;  // groups per K step: MPQ MFMAs, then CPQ copies
    constexpr int MPQ = TN * TM / Q;                  // MFMAs between two groups of copies
    constexpr int CPQ = CPS / Q;                      // copies per group
    static_assert(DPW % SPAN == 0 && (TN * TM) % Q == 0 && CPS % Q == 0 && KS % 2 == 0, "copy / MFMA interleave");
    const int nk = K / BK;
    auto tile_clamped = [&](int t) { return t < nk ? t : nk - 1; };   // past the end: refetch the last tile
#pragma unroll
    for (int s0 = 0; s0 < ST - 1; ++s0) issue(s0, tile_clamped(s0));
#pragma unroll
    for (int i = 0; i < CPS; ++i) issue_one(ST - 1, tile_clamped(ST - 1), i);
    wait_vmcnt<(ST - 2) * DPW + CPS>();               // tile 0 has landed (copies complete in order)
    __syncthreads();
    bf16x8 xf[2][TM], wf[2][TN];
    auto load_frags = [&](int stage, int ks, int sel) {
        const unsigned char* xb = lds + stage * STAGE;
        const unsigned char* wb = xb + BM * RB;
        const int c = 2 * ks + (lane >> 5);
#pragma unroll
        for (int j = 0; j < TM; ++j) {
            const int r = wm * WM + j * 32 + (lane & 31);
            xf[sel][j] = *reinterpret_cast<const bf16x8*>(xb + r * RB + ((c ^ swz_bk<BK>(r)) << 4));
        }
#pragma unroll
        for (int i = 0; i < TN; ++i) {
            const int r = wn * WN + i * 32 + (lane & 31);
            wf[sel][i] = *reinterpret_cast<const bf16x8*>(wb + r * RB + ((c ^ swz_bk<BK>(r)) << 4));
        }
    };
    int cur = 0, prev = ST - 1;                       // stage of tile kt / of tile kt-1 (= kt-1+ST)
    load_frags(0, 0, 0);
    for (int kt = 0; kt < nk; ++kt) {
        const int cur1 = cur + 1 == ST ? 0 : cur + 1;
        const int t_prev = tile_clamped(kt - 1 + ST), t_cur = tile_clamped(kt + ST);
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
            const int sel = ks & 1;                   // KS is even: every tile starts at sel 0
            const bool last = ks + 1 == KS;
            if (!last) {
                load_frags(cur, ks + 1, sel ^ 1);
            } else {
                __builtin_amdgcn_sched_barrier(0);
                wait_vmcnt<(ST - 2) * DPW>();         // own copies of tile kt+1 have landed
                __builtin_amdgcn_s_waitcnt(0xC07F);   // lgkmcnt(0): own reads of stage cur have returned
                __syncthreads();
                load_frags(cur1, 0, sel ^ 1);
            }
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int qq = 0; qq < Q; ++qq) {
#pragma unroll
                for (int e = 0; e < MPQ; ++e) {
                    const int idx = qq * MPQ + e, i = idx / TM, j = idx % TM;
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wf[sel][i], xf[sel][j], acc[i][j], 0, 0, 0);
                }
                __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                for (int cc = 0; cc < CPQ; ++cc) {
                    if (last) issue_one(cur, t_cur, qq * CPQ + cc);           // stage freed just above
                    else if (SPAN > 1) issue_one(prev, t_prev, CPS * (1 + ks) + qq * CPQ + cc);   // rest of the previous refill
                }
                __builtin_amdgcn_sched_barrier(0);
            }
        }
        prev = cur;
        cur = cur1;
    }
    wait_vmcnt<0>();

    // a K range writes its partial sums to plane [range][batch entry] of the scratch (the launcher has pointed Y there)
    TY* Y = (TY*)a.Y + (bz + krange * (int)(gridDim.z / (a.kspl > 1 ? a.kspl : 1))) * a.strideY;
    const float* bias = a.bias ? a.bias + bz * a.strideBias : nullptr;
    const zo_bf16* res = a.residual ? (const zo_bf16*)a.residual + bz * a.strideRes : nullptr;
    if constexpr (EPI == 3) {
        static_assert(TN == 2 && WN == 64 && WN_WAVES == 4, "a lane holds 32 of a wave's 64 columns");
        constexpr float LOG2E = 1.4426950408889634f;
        __syncthreads();                                    // the stages are idle: [2][4 waves along n][256 rows] floats
        float* red = reinterpret_cast<float*>(lds);
        const int g = lane >> 5;
        float* part = a.ce_part + bz * a.stridePart;
        float* tgt_out = a.ce_tgt + bz * a.strideTgt;
        const int col0 = n0 + wn * WN + g * 4;              // column of the lane's value (i, rg, e) = col0 + 32 i + 8 rg + e
#pragma unroll
        for (int j = 0; j < TM; ++j) {
            const int ml = wm * WM + j * 32 + (lane & 31);
            const int m = m0 + ml;
            float v[32];
#pragma unroll
            for (int i = 0; i < 2; ++i)
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const int col = col0 + 32 * i + 8 * (r >> 2) + (r & 3);
                    v[16 * i + r] = col < N ? acc[i][j][r] : -INFINITY;
                }
            float mx = fmaxf(fmaxf(v[0], v[1]), v[2]);
#pragma unroll
            for (int r = 3; r < 31; r += 2) mx = fmaxf(fmaxf(mx, v[r]), v[r + 1]);
            mx = fmaxf(mx, v[31]);
            {
                const auto h = __builtin_amdgcn_permlane32_swap(__float_as_uint(mx), __float_as_uint(mx), false, false);
                mx = fmaxf(__uint_as_float(h[0]), __uint_as_float(h[1]));
            }
            const float ref = mx == -INFINITY ? 0.0f : mx;  // a wave whose 64 columns all lie past N contributes (-inf, 0)
            float se = 0.0f;
#pragma unroll
            for (int r = 0; r < 32; ++r) se += __builtin_amdgcn_exp2f((v[r] - ref) * LOG2E);
            {
                const auto h = __builtin_amdgcn_permlane32_swap(__float_as_uint(se), __float_as_uint(se), false, false);
                se = __uint_as_float(h[0]) + __uint_as_float(h[1]);
            }
            if (g == 0) { red[wn * 256 + ml] = mx; red[(4 + wn) * 256 + ml] = se; }
            if (m < M && (m % a.ce_S) != a.ce_S - 1) {
                int t = a.ce_ids[m + 1];
                t = t < 0 ? 0 : (t >= N ? N - 1 : t);
                const int rel = t - col0;
                if (rel >= 0 && rel < 64 && (rel & 4) == 0) {
                    const int idx = (rel >> 5) * 16 + ((rel >> 3) & 3) * 4 + (rel & 3);
                    float tv = v[0];
#pragma unroll
                    for (int r = 1; r < 32; ++r) tv = idx == r ? v[r] : tv;
                    tgt_out[m] = tv;
                }
            }
        }
        __syncthreads();
        if (tid < 256 && m0 + tid < M) {
            float mw[4], sw[4];
#pragma unroll
            for (int w = 0; w < 4; ++w) { mw[w] = red[w * 256 + tid]; sw[w] = red[(4 + w) * 256 + tid]; }
            const float mt = fmaxf(fmaxf(mw[0], mw[1]), fmaxf(mw[2], mw[3]));   // finite: a tile has a column below N
            float st = 0.0f;
#pragma unroll
            for (int w = 0; w < 4; ++w) st += sw[w] * __builtin_amdgcn_exp2f((mw[w] - mt) * LOG2E);
            float2* dst = reinterpret_cast<float2*>(part) + (int64_t)(m0 + tid) * tiles_n + tile_n;
            *dst = make_float2(mt, st);
        }
        return;
    }
    if constexpr (EPI == 1) {
        static_assert(sizeof(TY) == 2 && TN == 2, "gate / up pairs need two n-tiles per wave and bf16 output");
        // each wave: 128 rows x 32 channels, staged through its LDS slice (64-byte rows, 8-byte granules XOR-swizzled by
        // the row) and written as whole 16-byte pieces, four lanes per row
        __syncthreads();
        constexpr int ROWB = 64;
        unsigned char* slice = lds + wave * (WM * ROWB);
#pragma unroll
        for (int j = 0; j < TM; ++j) {
            const int ml = j * 32 + (lane & 31);
#pragma unroll
            for (int rg = 0; rg < 4; ++rg) {
                const int g = rg * 2 + (lane >> 5);
                float v[4];
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    const float gt = zo_round_to<zo_bf16>(acc[0][j][rg * 4 + e]), up = zo_round_to<zo_bf16>(acc[1][j][rg * 4 + e]);
                    v[e] = (gt / (1.0f + __expf(-gt))) * up;
                }
                uint2 o;
                o.x = zo_pack_bf16x2(v[0], v[1]);
                o.y = zo_pack_bf16x2(v[2], v[3]);
                *reinterpret_cast<uint2*>(slice + ml * ROWB + ((g ^ (ml & 7)) << 3)) = o;
            }
        }
        const int No = N >> 1;
#pragma unroll 4
        for (int it = 0; it < WM / 16; ++it) {
            const int row = it * 16 + (lane >> 2), c = lane & 3, f = row & 7;
            uint4 v = *reinterpret_cast<const uint4*>(slice + row * ROWB + ((c ^ (f >> 1)) << 4));
            if (f & 1) v = make_uint4(v.z, v.w, v.x, v.y);
            const int m = m0 + wm * WM + row, n = (n0 >> 1) + wn * 32 + c * 8;
            // a wave's row piece is half a cache line (its n-neighbour writes the other half): cached stores, the
            // streaming hint is for whole lines only
            if (m < M && n < No) *reinterpret_cast<uint4*>((zo_bf16*)Y + (int64_t)m * No + n) = v;
        }
        return;
    }
    if constexpr (EPI == 2) {
        static_assert(sizeof(TY) == 2 && TN == 2 && WN == 64, "rotary pairs need two 32-column tiles per wave");
        __syncthreads();
        constexpr int ROWB = WN * 2;
        unsigned char* slice = lds + wave * (WM * ROWB);
        const bool rotate = n0 < a.rope_cols;               // a 256-column tile is two whole heads of q / k, or of v
        const int jh = wn & 1;                              // which 32 dimensions of the half head this wave holds
#pragma unroll
        for (int j = 0; j < TM; ++j) {
            const int ml = j * 32 + (lane & 31);
            int m = m0 + wm * WM + ml;
            m = m < M ? m : M - 1;
            const int64_t trow = (int64_t)(m % a.rope_S) * 64 + jh * 32 + (lane >> 5) * 4;
#pragma unroll
            for (int rg = 0; rg < 4; ++rg) {
                float x0[4], x1[4];
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    x0[e] = zo_round_to<zo_bf16>(acc[0][j][rg * 4 + e]);
                    x1[e] = zo_round_to<zo_bf16>(acc[1][j][rg * 4 + e]);
                }
                if (rotate) {
                    const float4 c4 = *reinterpret_cast<const float4*>(a.rope_cos + trow + rg * 8);
                    const float4 s4 = *reinterpret_cast<const float4*>(a.rope_sin + trow + rg * 8);
                    const float cc[4] = {c4.x, c4.y, c4.z, c4.w}, ss[4] = {s4.x, s4.y, s4.z, s4.w};
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        const float p = x0[e], r = x1[e];
                        x0[e] = __builtin_fmaf(p, cc[e], -(r * ss[e]));
                        x1[e] = __builtin_fmaf(r, cc[e], p * ss[e]);
                    }
                }
                const int g = rg * 2 + (lane >> 5);
                uint2 o;
                o.x = zo_pack_bf16x2(x0[0], x0[1]);
                o.y = zo_pack_bf16x2(x0[2], x0[3]);
                *reinterpret_cast<uint2*>(slice + ml * ROWB + ((g ^ (ml & 15)) << 3)) = o;
                o.x = zo_pack_bf16x2(x1[0], x1[1]);
                o.y = zo_pack_bf16x2(x1[2], x1[3]);
                *reinterpret_cast<uint2*>(slice + ml * ROWB + (((8 + g) ^ (ml & 15)) << 3)) = o;
            }
        }
        // read-back as in the plain path; chunk c < 4 is the first-half piece, c >= 4 the second-half piece of the row
#pragma unroll 4
        for (int it = 0; it < WM / 8; ++it) {
            const int row = it * 8 + (lane >> 3), c = lane & 7, f = row & 15;
            uint4 v = *reinterpret_cast<const uint4*>(slice + row * ROWB + ((c ^ (f >> 1)) << 4));
            if (f & 1) v = make_uint4(v.z, v.w, v.x, v.y);
            const int m = m0 + wm * WM + row;
            const int n = n0 + (wn >> 1) * 128 + (c >> 2) * 64 + jh * 32 + (c & 3) * 8;
            if (m < M && n < N) *reinterpret_cast<uint4*>((zo_bf16*)Y + (int64_t)m * N + n) = v;
        }
        return;
    }
    if constexpr (sizeof(TY) == 2) {
        if ((N & 7) == 0) {
            // bf16 output: each wave transposes its WM x WN tile through its own slice of the (now idle)
            // LDS, so that the global stores are whole 16-byte row segments, 128 contiguous bytes per
            // 8 lanes, instead of 8-byte pieces of 32 different rows.  A lane holds 4 consecutive n
            // (one 8-byte granule) of row m; granule g of row m is stored at granule slot
            // g ^ (m & 15): 16 lanes with consecutive m hit 16 different bank pairs.
            __syncthreads();                          // every wave's copies have landed, nobody reads the stages any more
            constexpr int ROWB = WN * 2;              // bytes per tile row
            unsigned char* slice = lds + wave * (WM * ROWB);
            auto stage = [&](auto fused_tag) {
                constexpr bool FUSED = decltype(fused_tag)::value;      // bias / ReLU / residual present
#pragma unroll
                for (int j = 0; j < TM; ++j) {
                    const int ml = j * 32 + (lane & 31);
                    const int m = m0 + wm * WM + ml;
                    uint2 r2[TN][4];
                    if constexpr (FUSED) {
                        // all residual pieces of this row block are requested before the first is used
#pragma unroll
                        for (int i = 0; i < TN; ++i)
#pragma unroll
                            for (int rg = 0; rg < 4; ++rg) {
                                const int n = n0 + wn * WN + (i * 8 + rg * 2 + (lane >> 5)) * 4;
                                r2[i][rg] = make_uint2(0, 0);
                                if (res && m < M && n < N) r2[i][rg] = *reinterpret_cast<const uint2*>(res + (int64_t)m * N + n);
                            }
                    }
#pragma unroll
                    for (int i = 0; i < TN; ++i)
#pragma unroll
                        for (int rg = 0; rg < 4; ++rg) {
                            const int g = i * 8 + rg * 2 + (lane >> 5);
                            float v[4];
#pragma unroll
                            for (int e = 0; e < 4; ++e) v[e] = acc[i][j][rg * 4 + e];
                            if constexpr (FUSED) {
                                const int n = n0 + wn * WN + g * 4;
                                if (bias && n < N) {
                                    float4 b4 = *reinterpret_cast<const float4*>(bias + n);
                                    v[0] += b4.x; v[1] += b4.y; v[2] += b4.z; v[3] += b4.w;
                                }
                                if (a.relu) {
#pragma unroll
                                    for (int e = 0; e < 4; ++e) v[e] = fmaxf(v[e], 0.0f);
                                }
                                if (res) {
                                    v[0] += zo_bf16_lo(r2[i][rg].x); v[1] += zo_bf16_hi(r2[i][rg].x);
                                    v[2] += zo_bf16_lo(r2[i][rg].y); v[3] += zo_bf16_hi(r2[i][rg].y);
                                }
                            }
                            uint2 o;
                            o.x = zo_pack_bf16x2(v[0], v[1]);
                            o.y = zo_pack_bf16x2(v[2], v[3]);
                            *reinterpret_cast<uint2*>(slice + ml * ROWB + ((g ^ (ml & 15)) << 3)) = o;
                        }
                }
            };
            if (bias || res || a.relu) stage(std::true_type{}); else stage(std::false_type{});
            constexpr int LPR = ROWB / 16;            // lanes per row in the read-back
            constexpr int RPI = 64 / LPR;             // rows per wave-level store
#pragma unroll 4
            for (int it = 0; it < WM / RPI; ++it) {
                const int row = it * RPI + lane / LPR, c = lane % LPR, f = row & 15;
                uint4 v = *reinterpret_cast<const uint4*>(slice + row * ROWB + ((c ^ (f >> 1)) << 4));
                if (f & 1) v = make_uint4(v.z, v.w, v.x, v.y);
                const int m = m0 + wm * WM + row, n = n0 + wn * WN + c * 8;
                if (m < M && n < N) {
                    typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
                    u32x4 vv = {v.x, v.y, v.z, v.w};
                    __builtin_nontemporal_store(vv, reinterpret_cast<u32x4*>((zo_bf16*)Y + (int64_t)m * N + n));
                }
            }
            return;
        }
    }
#pragma unroll
    for (int j = 0; j < TM; ++j)
#pragma unroll
        for (int i = 0; i < TN; ++i)
            store_tile<TY>(acc[i][j], a, Y, bias, res, m0 + wm * WM + j * 32 + (lane & 31),
                           n0 + wn * WN + i * 32 + (lane >> 5) * 4);
}

// ---------------------------------------------------------------------------------------------
// fp32 kernel (parity mode): 64 x 64 tile, K step 16, 256 threads x (4 x 4) outputs.
// ---------------------------------------------------------------------------------------------
template <typename TY>
__global__ __launch_bounds__(256) void zo_gemm_f32_kernel(zo_gemm_args a)
{
    __shared__ float xs[16][64 + 4];
    __shared__ float ws[16][64 + 4];
    const int tid = threadIdx.x;
    const int M = a.M, N = a.N, K = a.K;
    const int tiles_n = (N + 63) / 64;
    const int m0 = (blockIdx.x / tiles_n) * 64, n0 = (blockIdx.x % tiles_n) * 64;
    const int bz = blockIdx.z;
    const float* X = (const float*)a.X + bz * a.strideX;
    const float* W = (const float*)a.W + bz * a.strideW;
    const int tx = tid & 15, ty = tid >> 4;          // outputs m = ty*4.., n = tx*4..
    const int lr = tid >> 2, lk = (tid & 3) * 4;     // loader: row lr (0..63), k offset lk
    float acc[4][4] = {};
    for (int k0 = 0; k0 < K; k0 += 16) {
        float4 xv = make_float4(0, 0, 0, 0), wv = make_float4(0, 0, 0, 0);
        if (k0 + lk < K) {                            // K is a multiple of 4
            int rm = m0 + lr; rm = rm < M ? rm : M - 1;
            int rn = n0 + lr; rn = rn < N ? rn : N - 1;
            xv = *reinterpret_cast<const float4*>(X + (int64_t)rm * K + k0 + lk);
            wv = *reinterpret_cast<const float4*>(W + (int64_t)rn * K + k0 + lk);
        }
        __syncthreads();
        xs[lk + 0][lr] = xv.x; xs[lk + 1][lr] = xv.y; xs[lk + 2][lr] = xv.z; xs[lk + 3][lr] = xv.w;
        ws[lk + 0][lr] = wv.x; ws[lk + 1][lr] = wv.y; ws[lk + 2][lr] = wv.z; ws[lk + 3][lr] = wv.w;
        __syncthreads();
#pragma unroll
        for (int k = 0; k < 16; ++k) {
            float xm[4], wn[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) { xm[i] = xs[k][ty * 4 + i]; wn[i] = ws[k][tx * 4 + i]; }
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
                for (int j = 0; j < 4; ++j) acc[i][j] = __builtin_fmaf(xm[i], wn[j], acc[i][j]);
        }
    }
    TY* Y = (TY*)a.Y + bz * a.strideY;
    const float* bias = a.bias ? a.bias + bz * a.strideBias : nullptr;
    const float* res = a.residual ? (const float*)a.residual + bz * a.strideRes : nullptr;
    for (int i = 0; i < 4; ++i) {
        const int m = m0 + ty * 4 + i;
        if (m >= M) continue;
        for (int j = 0; j < 4; ++j) {
            const int n = n0 + tx * 4 + j;
            if (n >= N) continue;
            float t = acc[i][j];
            if (bias) t += bias[n];
            if (a.relu) t = fmaxf(t, 0.0f);
            if (res) t += res[(int64_t)m * N + n];
            Y[(int64_t)m * N + n] = t;
        }
    }
}

template <int BM, int BN>
static hipError_t launch_bf16(const zo_gemm_args& a, hipStream_t st)
{
    using C = gemm_cfg<BM, BN>;
    const int tiles = ((a.M + BM - 1) / BM) * ((a.N + BN - 1) / BN);
    dim3 grid(tiles, 1, a.batch);
    hipError_t e;
    if (a.out_f32) {
        e = hipFuncSetAttribute((const void*)zo_gemm_bf16_kernel<BM, BN, float>, hipFuncAttributeMaxDynamicSharedMemorySize, C::LDS_BYTES);
        if (e != hipSuccess) return e;
        zo_gemm_bf16_kernel<BM, BN, float><<<grid, 256, C::LDS_BYTES, st>>>(a);
    } else {
        e = hipFuncSetAttribute((const void*)zo_gemm_bf16_kernel<BM, BN, zo_bf16>, hipFuncAttributeMaxDynamicSharedMemorySize, C::LDS_BYTES);
        if (e != hipSuccess) return e;
        zo_gemm_bf16_kernel<BM, BN, zo_bf16><<<grid, 256, C::LDS_BYTES, st>>>(a);
    }
    return hipGetLastError();
}

// the gate / up GEMM with SwiGLU in its epilogue runs in the large-shape kernel only
bool zo_gemm_swiglu_supported(int32_t M, int32_t N, int32_t K, int dtype)
{
    if (dtype != ZO_T_BF16 || M <= 0 || N <= 0 || (N & 63) || (K & 63)) return false;
    if ((int64_t)M * N < (int64_t)256 * 256 * 128) return false;
    return (int64_t)M * K * 2 < ((int64_t)1 << 32) && (int64_t)N * K * 2 < ((int64_t)1 << 32);
}

// the lm_head GEMM with the cross entropy in its epilogue: the large-shape kernel
bool zo_gemm_ce_supported(int32_t M, int32_t N, int32_t K, int dtype)
{
    if (dtype != ZO_T_BF16 || M <= 0 || N <= 0 || (K & 63)) return false;
    if ((int64_t)M * N < (int64_t)256 * 256 * 128) return false;
    return (int64_t)M * K * 2 < ((int64_t)1 << 32) && (int64_t)N * K * 2 < ((int64_t)1 << 32);
}
size_t zo_gemm_ce_part_floats(int32_t M, int32_t N) { return (size_t)M * ((N + 255) / 256) * 2; }

// one wavefront per row: the tiles' (maximum, sum) pairs are merged in a fixed order
__global__ __launch_bounds__(256) void zo_ce_combine_kernel(const float* __restrict__ part, const float* __restrict__ tgt,
                                                            float* __restrict__ row_loss, int M, int S, int tiles_n)
{
    const int lane = threadIdx.x & 63;
    const int m = blockIdx.x * 4 + (threadIdx.x >> 6);
    if (m >= M) return;
    if ((m % S) == S - 1) {
        if (lane == 0) row_loss[m] = 0.0f;
        return;
    }
    const float2* p = reinterpret_cast<const float2*>(part) + (int64_t)m * tiles_n;
    float mx = -INFINITY;
    for (int t = lane; t < tiles_n; t += 64) mx = fmaxf(mx, p[t].x);
    mx = zo_group_max<64>(mx);
    float se = 0.0f;
    for (int t = lane; t < tiles_n; t += 64) se += p[t].y * __expf(p[t].x - mx);
    se = zo_group_sum<64>(se);
    if (lane == 0) row_loss[m] = (logf(se) + mx) - tgt[m];
}

hipError_t zo_launch_ce_combine(const float* part, const float* tgt, float* row_loss, int32_t M, int32_t S, int32_t N, hipStream_t st)
{
    if (M == 0) return hipSuccess;
    zo_ce_combine_kernel<<<(M + 3) / 4, 256, 0, st>>>(part, tgt, row_loss, M, S, (N + 255) / 256);
    return hipGetLastError();
}

// the fused q | k | v GEMM with the rotary embedding in its epilogue: large shapes, whole heads of 128 per half tile
bool zo_gemm_rope_supported(int32_t M, int32_t N, int32_t K, int dtype)
{
    if (dtype != ZO_T_BF16 || M <= 0 || N <= 0 || (N & 255) || (K & 63)) return false;
    if ((int64_t)M * N < (int64_t)256 * 256 * 128) return false;
    return (int64_t)M * K * 2 < ((int64_t)1 << 32) && (int64_t)N * K * 2 < ((int64_t)1 << 32);
}

// ---------------------------------------------------------------------------------------------
// K split of the 128 x 128-tile form.  A few hundred tokens times a narrow N (the attention output and down projections)
// give fewer workgroups than the chip has slots (two per CU), and each of them walks a long K with one tile in flight:
// the launch is bound by the latency of a tile's copies.  The launcher then cuts K into 2 / 4 / 8 ranges, every
// (tile, range) is a workgroup that writes fp32 partial sums P[range][batch entry][M][N], and the kernel below adds the
// ranges in order (no atomics: the result does not depend on scheduling) and applies bias / ReLU / residual / rounding.
// ---------------------------------------------------------------------------------------------
int zo_gemm_splitk(int32_t M, int32_t N, int32_t K, int32_t batch, int dtype)
{
    if (dtype != ZO_T_BF16 || M <= 0 || N <= 0 || (K & 63) || (N & 3)) return 1;
    if ((int64_t)((M + 255) / 256) * ((N + 255) / 256) * batch >= 160) return 1;      // the 256 x 256-tile form runs
    const int64_t wgs = (int64_t)((M + 127) / 128) * ((N + 127) / 128) * batch;
    const int64_t nk = K / 64;
    // Measured (128 x 128 tiles): an unsplit launch with no more workgroups than CUs takes about 0.62 us per K tile whatever
    // their number; split into ranges that together give every CU a workgroup it takes about 14 us (second kernel, shorter
    // pipelines) + 0.6 us x K tiles x workgroups / 256.  Split where that is the smaller figure ...
    if (wgs >= 256 || nk * (256 - wgs) <= 23 * 256) return 1;
    // ... into the fewest ranges that reach one and a half workgroups per CU (measured inside the step at 256 and 384 tokens:
    // better than one or two per CU; more ranges only add partial sums), at least 16 K tiles each
    int best = 1;
    for (int ks = 2; ks <= 8; ks <<= 1) {
        if (nk % ks != 0 || nk / ks < 16) break;
        best = ks;
        if (wgs * ks >= 384) break;
    }
    return best;
}
size_t zo_gemm_splitk_bytes(int32_t M, int32_t N, int32_t K, int32_t batch, int dtype)
{
    const int ks = zo_gemm_splitk(M, N, K, batch, dtype);
    return ks > 1 ? (size_t)ks * batch * M * N * sizeof(float) : 0;
}

// one thread per four consecutive n of one batch entry (blockIdx.y)
template <typename TY>
__global__ __launch_bounds__(256) void zo_gemm_splitk_reduce_kernel(zo_gemm_args a, const float* __restrict__ P, int KS)
{
    const int N4 = a.N >> 2;
    const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (i >= (int64_t)a.M * N4) return;
    const int b = blockIdx.y;
    const int m = (int)(i / N4), n = (int)(i % N4) * 4;
    const int64_t plane = (int64_t)a.M * a.N;
    const float* p = P + b * plane + (int64_t)m * a.N + n;
    f32x4 v = __builtin_nontemporal_load(reinterpret_cast<const f32x4*>(p));
    for (int ks = 1; ks < KS; ++ks) {
        const f32x4 t = __builtin_nontemporal_load(reinterpret_cast<const f32x4*>(p + (int64_t)ks * a.batch * plane));
        v[0] += t[0]; v[1] += t[1]; v[2] += t[2]; v[3] += t[3];
    }
    if (a.bias) {
        const float4 b4 = *reinterpret_cast<const float4*>(a.bias + b * a.strideBias + n);
        v[0] += b4.x; v[1] += b4.y; v[2] += b4.z; v[3] += b4.w;
    }
    if (a.relu) {
#pragma unroll
        for (int e = 0; e < 4; ++e) v[e] = fmaxf(v[e], 0.0f);
    }
    const int64_t off = (int64_t)m * a.N + n;
    if (a.residual) {
        const uint2 r2 = *reinterpret_cast<const uint2*>((const zo_bf16*)a.residual + b * a.strideRes + off);
        v[0] += zo_bf16_lo(r2.x); v[1] += zo_bf16_hi(r2.x);
        v[2] += zo_bf16_lo(r2.y); v[3] += zo_bf16_hi(r2.y);
    }
    if constexpr (sizeof(TY) == 4) {
        *reinterpret_cast<float4*>((float*)a.Y + b * a.strideY + off) = make_float4(v[0], v[1], v[2], v[3]);
    } else {
        uint2 o;
        o.x = zo_pack_bf16x2(v[0], v[1]);
        o.y = zo_pack_bf16x2(v[2], v[3]);
        *reinterpret_cast<uint2*>((zo_bf16*)a.Y + b * a.strideY + off) = o;
    }
}

hipError_t zo_launch_gemm(const zo_gemm_args& a, hipStream_t st)
{
    if (a.M == 0 || a.N == 0) return hipSuccess;
    if (a.dtype == ZO_T_BF16) {
        const bool large = (int64_t)a.M * a.N >= (int64_t)256 * 256 * 128;
        // operand bytes must be addressable with 32-bit offsets from the (batch) base pointers
        const bool off32 = (int64_t)a.M * a.K * 2 < ((int64_t)1 << 32) && (int64_t)a.N * a.K * 2 < ((int64_t)1 << 32);
        if (a.ce_part) {
            if (!zo_gemm_ce_supported(a.M, a.N, a.K, a.dtype) || a.bias || a.residual || a.relu || !a.ce_tgt || !a.ce_ids || a.ce_S <= 0)
                return hipErrorInvalidValue;
            const int tiles = ((a.M + 255) / 256) * ((a.N + 255) / 256);
            constexpr int lds_bytes = 2 * 512 * 64 * 2;
            hipError_t e_ = hipFuncSetAttribute((const void*)zo_gemm_bf16_dma_kernel<float, 8, 64, 2, 3>,
                                                hipFuncAttributeMaxDynamicSharedMemorySize, lds_bytes);
            if (e_ != hipSuccess) return e_;
            zo_gemm_bf16_dma_kernel<float, 8, 64, 2, 3><<<dim3(tiles, 1, a.batch), 8 * 64, lds_bytes, st>>>(a);
            return hipGetLastError();
        }
        if (a.rope_cos) {
            if (!zo_gemm_rope_supported(a.M, a.N, a.K, a.dtype) || a.bias || a.residual || a.relu || a.out_f32 || !a.rope_sin || a.rope_S <= 0 ||
                (a.rope_cols & 255))
                return hipErrorInvalidValue;
            const int tiles = ((a.M + 255) / 256) * ((a.N + 255) / 256);
            constexpr int lds_bytes = 2 * 512 * 64 * 2;
            hipError_t e_ = hipFuncSetAttribute((const void*)zo_gemm_bf16_dma_kernel<zo_bf16, 8, 64, 2, 2>,
                                                hipFuncAttributeMaxDynamicSharedMemorySize, lds_bytes);
            if (e_ != hipSuccess) return e_;
            zo_gemm_bf16_dma_kernel<zo_bf16, 8, 64, 2, 2><<<dim3(tiles, 1, a.batch), 8 * 64, lds_bytes, st>>>(a);
            return hipGetLastError();
        }
        if (a.swiglu) {
            if (!zo_gemm_swiglu_supported(a.M, a.N, a.K, a.dtype) || a.bias || a.residual || a.relu || a.out_f32) return hipErrorInvalidValue;
            const int tiles = ((a.M + 255) / 256) * ((a.N + 255) / 256);
            constexpr int lds_bytes = 2 * 512 * 64 * 2;
            hipError_t e_ = hipFuncSetAttribute((const void*)zo_gemm_bf16_dma_kernel<zo_bf16, 8, 64, 2, 1>,
                                                hipFuncAttributeMaxDynamicSharedMemorySize, lds_bytes);
            if (e_ != hipSuccess) return e_;
            zo_gemm_bf16_dma_kernel<zo_bf16, 8, 64, 2, 1><<<dim3(tiles, 1, a.batch), 8 * 64, lds_bytes, st>>>(a);
            return hipGetLastError();
        }
        // plain epilogue: 256 x 256 tiles once they give five eighths of the CUs a workgroup (both branches of a batched
        // launch count; measured crossover); below that the 128 x 128 form further down fills the chip better
        const bool fill256 = (int64_t)((a.M + 255) / 256) * ((a.N + 255) / 256) * a.batch >= 160;
        if (fill256 && (a.K & 63) == 0 && off32) {
            const int tiles = ((a.M + 255) / 256) * ((a.N + 255) / 256);
            const dim3 grid(tiles, 1, a.batch);
            constexpr int lds_bytes = 2 * 512 * 64 * 2;
            if (a.out_f32) {
                hipError_t e_ = hipFuncSetAttribute((const void*)zo_gemm_bf16_dma_kernel<float, 8, 64, 2>,
                                                    hipFuncAttributeMaxDynamicSharedMemorySize, lds_bytes);
                if (e_ != hipSuccess) return e_;
                zo_gemm_bf16_dma_kernel<float, 8, 64, 2><<<grid, 8 * 64, lds_bytes, st>>>(a);
            } else {
                hipError_t e_ = hipFuncSetAttribute((const void*)zo_gemm_bf16_dma_kernel<zo_bf16, 8, 64, 2>,
                                                    hipFuncAttributeMaxDynamicSharedMemorySize, lds_bytes);
                if (e_ != hipSuccess) return e_;
                zo_gemm_bf16_dma_kernel<zo_bf16, 8, 64, 2><<<grid, 8 * 64, lds_bytes, st>>>(a);
            }
            return hipGetLastError();
        }
        if ((a.K & 63) == 0 && off32 && a.K >= 128) {    // too few 256 x 256 tiles to fill the chip: 128 x 128 tiles, same pipeline
            const int tiles = ((a.M + 127) / 128) * ((a.N + 127) / 128);
            const dim3 grid(tiles, 1, a.batch);
            constexpr int lds_bytes = 2 * 256 * 64 * 2;
            const int ks = a.ks_part ? zo_gemm_splitk(a.M, a.N, a.K, a.batch, a.dtype) : 1;
            if (ks > 1 && a.ks_part_bytes >= zo_gemm_splitk_bytes(a.M, a.N, a.K, a.batch, a.dtype)) {
                zo_gemm_args p = a;                      // the partial-sum pass: fp32, no epilogue
                p.Y = a.ks_part;
                p.strideY = (int64_t)a.M * a.N;
                p.bias = nullptr; p.residual = nullptr; p.relu = 0; p.out_f32 = 1;
                p.kspl = ks;
                hipError_t e_ = hipFuncSetAttribute((const void*)zo_gemm_bf16_dma_kernel<float, 4, 64, 2, 0, 128>,
                                                    hipFuncAttributeMaxDynamicSharedMemorySize, lds_bytes);
                if (e_ != hipSuccess) return e_;
                zo_gemm_bf16_dma_kernel<float, 4, 64, 2, 0, 128><<<dim3(tiles, 1, a.batch * ks), 4 * 64, lds_bytes, st>>>(p);
                e_ = hipGetLastError();
                if (e_ != hipSuccess) return e_;
                const dim3 rgrid((unsigned)(((int64_t)a.M * (a.N >> 2) + 255) / 256), a.batch, 1);
                if (a.out_f32) zo_gemm_splitk_reduce_kernel<float><<<rgrid, 256, 0, st>>>(a, a.ks_part, ks);
                else zo_gemm_splitk_reduce_kernel<zo_bf16><<<rgrid, 256, 0, st>>>(a, a.ks_part, ks);
                return hipGetLastError();
            }
            if (a.out_f32) {
                hipError_t e_ = hipFuncSetAttribute((const void*)zo_gemm_bf16_dma_kernel<float, 4, 64, 2, 0, 128>,
                                                    hipFuncAttributeMaxDynamicSharedMemorySize, lds_bytes);
                if (e_ != hipSuccess) return e_;
                zo_gemm_bf16_dma_kernel<float, 4, 64, 2, 0, 128><<<grid, 4 * 64, lds_bytes, st>>>(a);
            } else {
                hipError_t e_ = hipFuncSetAttribute((const void*)zo_gemm_bf16_dma_kernel<zo_bf16, 4, 64, 2, 0, 128>,
                                                    hipFuncAttributeMaxDynamicSharedMemorySize, lds_bytes);
                if (e_ != hipSuccess) return e_;
                zo_gemm_bf16_dma_kernel<zo_bf16, 4, 64, 2, 0, 128><<<grid, 4 * 64, lds_bytes, st>>>(a);
            }
            return hipGetLastError();
        }
        if (large) return launch_bf16<256, 256>(a, st);     // K not a multiple of 64: the register-staged kernel
        return launch_bf16<128, 128>(a, st);
    }
    const int tiles = ((a.M + 63) / 64) * ((a.N + 63) / 64);
    zo_gemm_f32_kernel<float><<<dim3(tiles, 1, a.batch), 256, 0, st>>>(a);
    return hipGetLastError();
}
