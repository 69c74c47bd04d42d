// Device-side building blocks shared by the HIP kernels of the ZO-QAT step (gfx950 only).
//
//  * the perturbation stream u ~ N(0, I) of Eq. 2: Philox4x32-10 (Salmon et al., SC'11) keyed by
//    the step seed, counter = (element index / 8, tensor id), and a Box-Muller transform made of
//    a fixed sequence of correctly rounded fp32 operations, so that every kernel that asks for
//    element i of tensor t under seed s gets the same bits; the stream is never stored;
//  * the uniform quantizer of the Background section (asymmetric min/max, or symmetric absmax);
//  * bf16 storage conversion.
//
// Everything that decides an integer code is written one IEEE operation per statement; the
// translation unit is compiled with -ffp-contract=off and fused multiply-adds are explicit.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#define ZO_DEV __device__ __forceinline__

typedef __bf16 zo_bf16;
typedef __bf16 zo_bf16x2 __attribute__((ext_vector_type(2)));
typedef float zo_f32x2 __attribute__((ext_vector_type(2)));

// ---------------------------------------------------------------------------------------------
// storage types
// ---------------------------------------------------------------------------------------------
ZO_DEV float zo_load(const float* p) { return *p; }
ZO_DEV float zo_load(const zo_bf16* p) { return (float)*p; }
ZO_DEV void zo_store(float* p, float v) { *p = v; }
ZO_DEV void zo_store(zo_bf16* p, float v) { *p = (zo_bf16)v; }   // round to nearest even

ZO_DEV uint32_t zo_pack_bf16x2(float lo, float hi)
{
    zo_f32x2 v = {lo, hi};
    zo_bf16x2 b = __builtin_convertvector(v, zo_bf16x2);
    return __builtin_bit_cast(uint32_t, b);
}
ZO_DEV float zo_bf16_lo(uint32_t u) { return __uint_as_float(u << 16); }
ZO_DEV float zo_bf16_hi(uint32_t u) { return __uint_as_float(u & 0xFFFF0000u); }

// 8 consecutive elements of storage type T <-> 8 floats
ZO_DEV void zo_load8(const float* p, float v[8])
{
    float4 a = *reinterpret_cast<const float4*>(p);
    float4 b = *reinterpret_cast<const float4*>(p + 4);
    v[0] = a.x; v[1] = a.y; v[2] = a.z; v[3] = a.w; v[4] = b.x; v[5] = b.y; v[6] = b.z; v[7] = b.w;
}
ZO_DEV void zo_load8(const zo_bf16* p, float v[8])
{
    uint4 a = *reinterpret_cast<const uint4*>(p);
    v[0] = zo_bf16_lo(a.x); v[1] = zo_bf16_hi(a.x); v[2] = zo_bf16_lo(a.y); v[3] = zo_bf16_hi(a.y);
    v[4] = zo_bf16_lo(a.z); v[5] = zo_bf16_hi(a.z); v[6] = zo_bf16_lo(a.w); v[7] = zo_bf16_hi(a.w);
}
ZO_DEV void zo_store8(float* p, const float v[8])
{
    *reinterpret_cast<float4*>(p) = make_float4(v[0], v[1], v[2], v[3]);
    *reinterpret_cast<float4*>(p + 4) = make_float4(v[4], v[5], v[6], v[7]);
}
ZO_DEV void zo_store8(zo_bf16* p, const float v[8])
{
    uint4 a;
    a.x = zo_pack_bf16x2(v[0], v[1]); a.y = zo_pack_bf16x2(v[2], v[3]);
    a.z = zo_pack_bf16x2(v[4], v[5]); a.w = zo_pack_bf16x2(v[6], v[7]);
    *reinterpret_cast<uint4*>(p) = a;
}
// master weights kept in IEEE binary16: exact widening on load
typedef _Float16 zo_f16;
ZO_DEV void zo_load8(const zo_f16* p, float v[8])
{
    typedef _Float16 f16x8_ __attribute__((ext_vector_type(8)));
    const f16x8_ a = *reinterpret_cast<const f16x8_*>(p);
#pragma unroll
    for (int i = 0; i < 8; ++i) v[i] = (float)a[i];
}
ZO_DEV float zo_load(const zo_f16* p) { return (float)*p; }

// value as it will be read back from storage of type T
template <typename T> ZO_DEV float zo_round_to(float v);
template <> ZO_DEV float zo_round_to<float>(float v) { return v; }
template <> ZO_DEV float zo_round_to<zo_bf16>(float v) { return (float)(zo_bf16)v; }

// ---------------------------------------------------------------------------------------------
// Philox4x32-10
// ---------------------------------------------------------------------------------------------
struct zo_stream {          // uniform across a launch: lives in scalar registers
    uint32_t k0, k1;        // seed low / high
    uint32_t tensor_id;
};

ZO_DEV void zo_philox(const zo_stream& s, uint64_t blk, uint32_t out[4])
{
    uint32_t c0 = (uint32_t)blk, c1 = (uint32_t)(blk >> 32), c2 = s.tensor_id, c3 = 0u;
    uint32_t k0 = s.k0, k1 = s.k1;
#pragma unroll
    for (int r = 0; r < 10; ++r) {
        uint64_t p0 = (uint64_t)0xD2511F53u * (uint64_t)c0;
        uint64_t p1 = (uint64_t)0xCD9E8D57u * (uint64_t)c2;
        uint32_t n0 = (uint32_t)(p1 >> 32) ^ c1 ^ k0;
        uint32_t n2 = (uint32_t)(p0 >> 32) ^ c3 ^ k1;
        c1 = (uint32_t)p1;
        c3 = (uint32_t)p0;
        c0 = n0;
        c2 = n2;
        k0 += 0x9E3779B9u;
        k1 += 0xBB67AE85u;
    }
    out[0] = c0; out[1] = c1; out[2] = c2; out[3] = c3;
}

// Correctly rounded square root for 2^-96 < x < 2^96 (S below lies in [1.5e-5, 23.6]): the hardware estimate, whose
// error is below one ulp, moved to the neighbour that the exact residuals x - r * (r -+ ulp) ask for.  This is the
// sequence the compiler emits for sqrtf, without its rescaling of tiny inputs and its special cases for 0 and infinity.
ZO_DEV float zo_sqrt_in_range(float x)
{
    const float r = __builtin_amdgcn_sqrtf(x);
    const float dn = __uint_as_float(__float_as_uint(r) - 1u), up = __uint_as_float(__float_as_uint(r) + 1u);
    const float vd = __builtin_fmaf(-dn, r, x), vu = __builtin_fmaf(-up, r, x);
    float s = vd <= 0.0f ? dn : r;
    s = vu > 0.0f ? up : s;
    return s;
}

// One 32-bit word -> (r cos t, r sin t): low half is the radius uniform, high half the angle.
ZO_DEV void zo_word_to_normals(uint32_t w, float& z0, float& z1)
{
    // radius: u1 = (2a+1) / 2^17, S = -2 ln u1
    uint32_t a = w & 0xFFFFu;
    float f = (float)(2u * a + 1u);
    uint32_t x = __float_as_uint(f) - 0x3F3504F3u;
    int32_t e = (int32_t)x >> 23;
    float m = __uint_as_float((x & 0x007FFFFFu) + 0x3F3504F3u);
    float t = m - 1.0f;
    float p = -0x1.a91ca0p-4f;
    p = __builtin_fmaf(p, t, 0x1.4e9aecp-3f);
    p = __builtin_fmaf(p, t, -0x1.6082b2p-3f);
    p = __builtin_fmaf(p, t, 0x1.973aaap-3f);
    p = __builtin_fmaf(p, t, -0x1.ff6ae4p-3f);
    p = __builtin_fmaf(p, t, 0x1.555b4cp-2f);
    p = __builtin_fmaf(p, t, -0x1.000074p-1f);
    p = __builtin_fmaf(p, t, 0x1.fffffep-1f);
    float lnm = t * p;
    float E = (float)(e - 17);
    float ln_u1 = __builtin_fmaf(E, 0x1.62e430p-1f, lnm);
    float S = -2.0f * ln_u1;
    float r = zo_sqrt_in_range(S);                      // correctly rounded
    // angle: quadrant from the top two bits, x in (-pi/4, pi/4) from the other fourteen
    uint32_t b = w >> 16;
    int32_t j = (int32_t)((b & 0x3FFFu) << 1) - 16383;
    float xa = (float)j * 0x1.921fb6p-15f;
    float y = xa * xa;
    float sp = -0x1.99076cp-13f;
    sp = __builtin_fmaf(y, sp, 0x1.110630p-7f);
    sp = __builtin_fmaf(y, sp, -0x1.555540p-3f);
    float xy = xa * y;
    float sn = __builtin_fmaf(xy, sp, xa);
    float cp = -0x1.64257ep-10f;
    cp = __builtin_fmaf(y, cp, 0x1.553cecp-5f);
    cp = __builtin_fmaf(y, cp, -0x1.ffffa0p-2f);
    float cs = __builtin_fmaf(y, cp, 1.0f);
    // rotate by quadrant q: (c,s) -> q=0 (cs,sn) 1 (-sn,cs) 2 (-cs,-sn) 3 (sn,-cs)
    bool swap = (w >> 30) & 1u;
    float c = swap ? sn : cs;
    float s = swap ? cs : sn;
    uint32_t sign_s = w & 0x80000000u;                   // q >= 2
    uint32_t sign_c = (w ^ (w << 1)) & 0x80000000u;      // q == 1 or q == 2
    c = __uint_as_float(__float_as_uint(c) ^ sign_c);
    s = __uint_as_float(__float_as_uint(s) ^ sign_s);
    z0 = r * c;
    z1 = r * s;
}

// The eight perturbation elements 8*blk .. 8*blk+7 of the stream.
ZO_DEV void zo_z8(const zo_stream& s, uint64_t blk, float z[8])
{
    uint32_t w[4];
    zo_philox(s, blk, w);
#pragma unroll
    for (int i = 0; i < 4; ++i) zo_word_to_normals(w[i], z[2 * i], z[2 * i + 1]);
}

// Single element (ragged tails, gathers).
ZO_DEV float zo_z1(const zo_stream& s, uint64_t i)
{
    uint32_t w[4];
    zo_philox(s, i >> 3, w);
    uint32_t sel = (uint32_t)(i >> 1) & 3u;
    uint32_t word = sel == 0 ? w[0] : sel == 1 ? w[1] : sel == 2 ? w[2] : w[3];
    float z0, z1;
    zo_word_to_normals(word, z0, z1);
    return (i & 1) ? z1 : z0;
}

// ---------------------------------------------------------------------------------------------
// rounding of an updated master to binary16: nearest even, or stochastic (the stored value's expectation is
// the fp32 result even when the step is far below the spacing of binary16).  The random integers come from
// a second stream: same key, counter = (element index / 4, tensor id, 1).
// ---------------------------------------------------------------------------------------------
ZO_DEV uint16_t zo_f16_bits(float x) { return __builtin_bit_cast(uint16_t, (zo_f16)x); }      // round to nearest even
ZO_DEV float zo_f16_value(uint16_t h) { return (float)__builtin_bit_cast(zo_f16, h); }

// r: uniform 24-bit integer.  lo < x < hi neighbouring binary16 values: hi iff r (hi - lo) / 2^24 < x - lo.
ZO_DEV uint16_t zo_f16_stochastic(float x, uint32_t r)
{
    const uint16_t h = zo_f16_bits(x);
    if ((h & 0x7C00u) == 0x7C00u) return h;            // infinity / NaN
    const float f = zo_f16_value(h);
    if (f == x) return h;                              // representable
    const bool zero = (h & 0x7FFFu) == 0, neg = (h & 0x8000u) != 0;
    const uint16_t up = zero ? (uint16_t)0x0001u : (uint16_t)(neg ? h - 1 : h + 1);
    const uint16_t dn = zero ? (uint16_t)0x8001u : (uint16_t)(neg ? h + 1 : h - 1);
    const bool below = f < x;
    const uint16_t lo = below ? h : dn, hi = below ? up : h;
    const float flo = zo_f16_value(lo), fhi = zo_f16_value(hi);
    const float ulp = fhi - flo;
    const float d = x - flo;
    const float t = (float)r * (ulp * 0x1p-24f);
    return t < d ? hi : lo;
}

// the eight 24-bit integers of elements 8*blk .. 8*blk+7 (two blocks of the rounding stream)
ZO_DEV void zo_round_bits8(const zo_stream& s, uint64_t blk, uint32_t r[8])
{
#pragma unroll
    for (int half = 0; half < 2; ++half) {
        const uint64_t b = 2 * blk + half;
        uint32_t c0 = (uint32_t)b, c1 = (uint32_t)(b >> 32), c2 = s.tensor_id, c3 = 1u;
        uint32_t k0 = s.k0, k1 = s.k1;
#pragma unroll
        for (int rd = 0; rd < 10; ++rd) {
            uint64_t p0 = (uint64_t)0xD2511F53u * (uint64_t)c0;
            uint64_t p1 = (uint64_t)0xCD9E8D57u * (uint64_t)c2;
            uint32_t n0 = (uint32_t)(p1 >> 32) ^ c1 ^ k0;
            uint32_t n2 = (uint32_t)(p0 >> 32) ^ c3 ^ k1;
            c1 = (uint32_t)p1;
            c3 = (uint32_t)p0;
            c0 = n0;
            c2 = n2;
            k0 += 0x9E3779B9u;
            k1 += 0xBB67AE85u;
        }
        r[4 * half + 0] = c0 >> 8; r[4 * half + 1] = c1 >> 8; r[4 * half + 2] = c2 >> 8; r[4 * half + 3] = c3 >> 8;
    }
}
ZO_DEV uint32_t zo_round_bits1(const zo_stream& s, uint64_t i)
{
    uint32_t r[8];
    zo_round_bits8(s, i >> 3, r);
    uint32_t out = r[0];
#pragma unroll
    for (int k = 1; k < 8; ++k) out = ((uint32_t)(i & 7) == (uint32_t)k) ? r[k] : out;
    return out;
}

// ---------------------------------------------------------------------------------------------
// uniform quantizer (per group): parameters from the group's range, then code / de-quantize
// ---------------------------------------------------------------------------------------------
#define ZO_STEP_MIN 1e-5f

struct zo_qparams { float step, inv, zp, qn, qp; };

ZO_DEV zo_qparams zo_qparams_asym(float mn, float mx, int bits)
{
    zo_qparams q;
    q.qp = (float)((1 << bits) - 1);
    q.qn = 0.0f;
    float step = (mx - mn) / q.qp;
    q.step = step < ZO_STEP_MIN ? ZO_STEP_MIN : step;
    q.inv = 1.0f / q.step;
    q.zp = -__builtin_rintf(mn * q.inv);
    return q;
}
ZO_DEV zo_qparams zo_qparams_sym(float amax, int bits)
{
    zo_qparams q;
    q.qp = (float)((1 << (bits - 1)) - 1);
    q.qn = -(float)(1 << (bits - 1));
    float step = amax / q.qp;
    q.step = step < ZO_STEP_MIN ? ZO_STEP_MIN : step;
    q.inv = 1.0f / q.step;
    q.zp = 0.0f;
    return q;
}
ZO_DEV float zo_code(const zo_qparams& q, float x)
{
    const float c = __builtin_rintf(x * q.inv) + q.zp;
    return __builtin_amdgcn_fmed3f(c, q.qn, q.qp);       // clamp to [qn, qp] in one instruction
}
ZO_DEV float zo_dequant(const zo_qparams& q, float code) { return (code - q.zp) * q.step; }
// eight codes minus `off` (the re-centring of the integer route: the results lie in [-128, 127]) as eight signed bytes
ZO_DEV uint2 zo_pack_codes8(const zo_qparams& q, const float v[8], float off)
{
    uint32_t w[2] = {0u, 0u};
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        const int cd = (int)(zo_code(q, v[i]) - off);
        w[i >> 2] |= ((uint32_t)cd & 0xFFu) << (8 * (i & 3));
    }
    return make_uint2(w[0], w[1]);
}

// ---------------------------------------------------------------------------------------------
// wavefront helpers (64 lanes)
// ---------------------------------------------------------------------------------------------
// Reductions over aligned groups of WIDTH lanes (a power of two); every lane of a group gets the group's result.
// The exchanges are register-to-register: lane ^ 1 and lane ^ 2 by quad permutes, then the mirror images of the
// 8 and 16 lanes of a row (the lanes met there all hold their half's result already), then the row and half-wave
// swaps of gfx950 -- no trip through the LDS crossbar.  The association order is fixed, so sums are reproducible.
template <int CTRL> ZO_DEV float zo_dpp(float v)
{
    return __int_as_float(__builtin_amdgcn_mov_dpp(__float_as_int(v), CTRL, 0xF, 0xF, true));
}
template <int WIDTH, typename OP> ZO_DEV float zo_group_reduce(float v, OP op)
{
    static_assert(WIDTH >= 1 && WIDTH <= 64 && (WIDTH & (WIDTH - 1)) == 0, "group width");
    if (WIDTH >= 2) v = op(v, zo_dpp<0xB1>(v));      // quad_perm [1,0,3,2]
    if (WIDTH >= 4) v = op(v, zo_dpp<0x4E>(v));      // quad_perm [2,3,0,1]
    if (WIDTH >= 8) v = op(v, zo_dpp<0x141>(v));     // row_half_mirror: lane 7 - i of each 8
    if (WIDTH >= 16) v = op(v, zo_dpp<0x140>(v));    // row_mirror: lane 15 - i of each 16
    if (WIDTH >= 32) {                               // rows 1 and 3 of the first copy <-> rows 0 and 2 of the second
        const auto r = __builtin_amdgcn_permlane16_swap(__float_as_uint(v), __float_as_uint(v), false, false);
        v = op(__uint_as_float(r[0]), __uint_as_float(r[1]));
    }
    if (WIDTH >= 64) {                               // upper half of the first copy <-> lower half of the second
        const auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(v), __float_as_uint(v), false, false);
        v = op(__uint_as_float(r[0]), __uint_as_float(r[1]));
    }
    return v;
}
template <int WIDTH> ZO_DEV float zo_group_min(float v)
{
    return zo_group_reduce<WIDTH>(v, [](float a, float b) { return fminf(a, b); });
}
template <int WIDTH> ZO_DEV float zo_group_max(float v)
{
    return zo_group_reduce<WIDTH>(v, [](float a, float b) { return fmaxf(a, b); });
}
template <int WIDTH> ZO_DEV float zo_group_sum(float v)
{
    return zo_group_reduce<WIDTH>(v, [](float a, float b) { return a + b; });
}
