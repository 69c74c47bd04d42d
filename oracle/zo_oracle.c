/*
 * CPU oracle for the ZeroQAT zeroth-order quantization-aware training step.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, plain reference that the
 * HIP library is checked against.  It shares no code, header, table or
 * constant generator with the HIP path and is never called by it.
 *
 * What it computes, and where the paper defines it:
 *   - the uniform asymmetric / symmetric quantizer      (Background, "Quantization" equation)
 *   - group-wise weights, per-token activations          (Appendix "Quantization settings")
 *   - the two-point zeroth-order estimate, q = 1         (Eq. 2)
 *   - the ZO-SGD update on full-precision master weights (Eq. 3)
 *   - the adaptive weight quantizer with learnable step, zero point and
 *     clipping coefficients (Eq. 5) and the channel-wise smoothing (Eq. 4)
 *   - frozen, pre-quantized weights of the lightweight variant
 *                                 (Section "Lightweight ZeroQAT for memory reduction")
 *   - master weights kept in IEEE binary16, what the memory table of the
 *     efficiency section implies (2 bytes per parameter), with the update of
 *     Eq. 3 rounded to nearest even or stochastically
 * The paper only says u ~ N(0, I); the concrete counter-based stream used here
 * (Philox4x32-10 of Salmon et al. 2011 + a fixed-recipe Box-Muller) is this
 * build's reading.  The *choice* of generator is "parity unpinned": nothing in
 * the paper fixes it.  The generator itself is pinned by published
 * known-answer vectors (integers) and by distribution tests (normals).
 *
 * Floating point: every step that decides an integer code is done in fp32
 * with one IEEE operation per line (compile with -ffp-contract=off; fmaf is
 * the correctly rounded fused multiply-add).  Contractions accumulate in fp64.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

/* ------------------------------------------------------------------ */
/* Philox4x32-10 (Salmon, Moraes, Dror, Shaw, SC'11)                   */
/* ------------------------------------------------------------------ */
void zo_or_philox4x32_10(const uint32_t ctr[4], const uint32_t key[2], uint32_t out[4])
{
    uint32_t c0 = ctr[0], c1 = ctr[1], c2 = ctr[2], c3 = ctr[3];
    uint32_t k0 = key[0], k1 = key[1];
    for (int round = 0; round < 10; ++round) {
        uint64_t p0 = (uint64_t)0xD2511F53u * (uint64_t)c0;
        uint64_t p1 = (uint64_t)0xCD9E8D57u * (uint64_t)c2;
        uint32_t n0 = (uint32_t)(p1 >> 32) ^ c1 ^ k0;
        uint32_t n1 = (uint32_t)p1;
        uint32_t n2 = (uint32_t)(p0 >> 32) ^ c3 ^ k1;
        uint32_t n3 = (uint32_t)p0;
        c0 = n0; c1 = n1; c2 = n2; c3 = n3;
        k0 += 0x9E3779B9u;
        k1 += 0xBB67AE85u;
    }
    out[0] = c0; out[1] = c1; out[2] = c2; out[3] = c3;
}

/* Block `blk` of the stream of tensor `tensor_id` under `seed`:
 * key = (seed low, seed high), counter = (blk low, blk high, tensor_id, 0). */
static void stream_block(uint64_t seed, int32_t tensor_id, uint64_t blk, uint32_t out[4])
{
    uint32_t ctr[4] = { (uint32_t)blk, (uint32_t)(blk >> 32), (uint32_t)tensor_id, 0u };
    uint32_t key[2] = { (uint32_t)seed, (uint32_t)(seed >> 32) };
    zo_or_philox4x32_10(ctr, key, out);
}

/* out[j] = word (j & 3) of block (j >> 2), j = 0 .. nwords-1. */
void zo_or_philox_words(uint64_t seed, int32_t tensor_id, int64_t nwords, uint32_t* out)
{
    for (int64_t j = 0; j < nwords; ++j) {
        uint32_t w[4];
        stream_block(seed, tensor_id, (uint64_t)(j >> 2), w);
        out[j] = w[j & 3];
    }
}

/* ------------------------------------------------------------------ */
/* 32-bit word -> two standard normals (Box-Muller, fixed fp32 recipe) */
/* ------------------------------------------------------------------ */
static float u2f(uint32_t u) { float f; memcpy(&f, &u, 4); return f; }
static uint32_t f2u(float f) { uint32_t u; memcpy(&u, &f, 4); return u; }

/* Low 16 bits a -> u1 = (2a+1)/2^17 in (0,1); returns S = -2 ln(u1) in fp32.
 * ln is range-reduced to m in [sqrt(1/2), sqrt(2)) and a degree-7 polynomial
 * in t = m - 1 stands for ln(1+t)/t; the factor -2 is folded in afterwards. */
static float neg2_log_u1(uint32_t a)
{
    float    f    = (float)(2u * a + 1u);              /* exact: 17-bit integer */
    uint32_t x    = f2u(f) - 0x3F3504F3u;              /* bits relative to sqrt(1/2) */
    int32_t  e    = (int32_t)x >> 23;                  /* f = m * 2^e, arithmetic shift */
    float    m    = u2f((x & 0x007FFFFFu) + 0x3F3504F3u);
    float    t    = m - 1.0f;                          /* exact */
    float    p    = -0x1.a91ca0p-4f;
    p = fmaf(p, t,  0x1.4e9aecp-3f);
    p = fmaf(p, t, -0x1.6082b2p-3f);
    p = fmaf(p, t,  0x1.973aaap-3f);
    p = fmaf(p, t, -0x1.ff6ae4p-3f);
    p = fmaf(p, t,  0x1.555b4cp-2f);
    p = fmaf(p, t, -0x1.000074p-1f);
    p = fmaf(p, t,  0x1.fffffep-1f);
    float lnm = t * p;                                 /* ln(m) */
    float E   = (float)(e - 17);                       /* u1 = m * 2^(e-17) */
    float ln_u1 = fmaf(E, 0x1.62e430p-1f, lnm);        /* fp32(ln 2) */
    return -2.0f * ln_u1;                              /* exact scaling */
}

/* High 16 bits b -> (cos, sin) of theta = (pi/2) * (b>>14) + x, where
 * x = pi * (2*(b & 0x3FFF) - 16383) / 65536 lies in (-pi/4, pi/4). */
static void cos_sin_b(uint32_t b, float* c_out, float* s_out)
{
    int32_t j = (int32_t)((b & 0x3FFFu) << 1) - 16383;
    float x = (float)j * 0x1.921fb6p-15f;              /* fp32(pi / 65536) */
    float y = x * x;
    float sp = -0x1.99076cp-13f;
    sp = fmaf(y, sp,  0x1.110630p-7f);
    sp = fmaf(y, sp, -0x1.555540p-3f);
    float xy = x * y;
    float sn = fmaf(xy, sp, x);                        /* sin x */
    float cp = -0x1.64257ep-10f;
    cp = fmaf(y, cp,  0x1.553cecp-5f);
    cp = fmaf(y, cp, -0x1.ffffa0p-2f);
    float cs = fmaf(y, cp, 1.0f);                      /* cos x */
    switch (b >> 14) {
        case 0:  *c_out =  cs; *s_out =  sn; break;
        case 1:  *c_out = -sn; *s_out =  cs; break;
        case 2:  *c_out = -cs; *s_out = -sn; break;
        default: *c_out =  sn; *s_out = -cs; break;
    }
}

/* One 32-bit word gives the pair (r cos theta, r sin theta). */
void zo_or_word_to_normals(uint32_t w, float out[2])
{
    float S = neg2_log_u1(w & 0xFFFFu);
    float r = sqrtf(S);                                /* correctly rounded */
    float c, s;
    cos_sin_b(w >> 16, &c, &s);
    out[0] = r * c;
    out[1] = r * s;
}

/* Perturbation element i of tensor `tensor_id` under `seed`:
 * block i>>3, word (i>>1)&3, pair member i&1.  Depends on nothing else. */
float zo_or_z(uint64_t seed, int32_t tensor_id, int64_t i)
{
    uint32_t w[4];
    float pair[2];
    stream_block(seed, tensor_id, (uint64_t)i >> 3, w);
    zo_or_word_to_normals(w[(i >> 1) & 3], pair);
    return pair[i & 1];
}

void zo_or_normal(uint64_t seed, int32_t tensor_id, int64_t start, int64_t n, float* out)
{
    #pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < n; ++i) out[i] = zo_or_z(seed, tensor_id, start + i);
}

/* ------------------------------------------------------------------ */
/* bf16 storage rounding (round to nearest even on the top 16 bits)     */
/* ------------------------------------------------------------------ */
float zo_or_bf16_round(float v)
{
    uint32_t u = f2u(v);
    if ((u & 0x7F800000u) == 0x7F800000u) return v;    /* inf / nan unchanged */
    u += 0x7FFFu + ((u >> 16) & 1u);
    u &= 0xFFFF0000u;
    return u2f(u);
}

void zo_or_bf16_round_array(const float* in, int64_t n, float* out)
{
    for (int64_t i = 0; i < n; ++i) out[i] = zo_or_bf16_round(in[i]);
}

/* ------------------------------------------------------------------ */
/* Perturbation of a parameter tensor: theta' = theta + (s*eps) * z     */
/* (argument of Q in Eq. 2), one fused multiply-add in fp32.            */
/* ------------------------------------------------------------------ */
void zo_or_perturb(const float* w, int64_t n, uint64_t seed, int32_t tensor_id,
                   float eps_signed, float* out)
{
    #pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < n; ++i) {
        float z = (eps_signed == 0.0f) ? 0.0f : zo_or_z(seed, tensor_id, i);
        out[i] = fmaf(eps_signed, z, w[i]);
    }
}

/* ------------------------------------------------------------------ */
/* Uniform quantizer of one group (Background, "Quantization").         */
/*   asymmetric: Q_N = 0, Q_P = 2^b - 1, step = (max - min)/Q_P,        */
/*               zp = -round(min/step)                                  */
/*   symmetric:  Q_N = -2^(b-1), Q_P = 2^(b-1) - 1, step = max|x|/Q_P,  */
/*               zp = 0                                                 */
/*   code = clamp(round(x/step) + zp, Q_N, Q_P);  x^ = (code - zp)*step */
/* Readings: signed min/max (the printed |X| would clamp every negative */
/* value); round = half-to-even; x/step evaluated as x * (1/step) with  */
/* one division per group; step floored at 1e-5; zp not clamped.        */
/* ------------------------------------------------------------------ */
#define ZO_OR_STEP_MIN 1e-5f

/* float -> int32 for REPORTED integers (codes, zero points): saturating, NaN -> 0.  The zero point of the Background
 * section, -round(min / step), is unbounded (a constant group far from zero, whose step is the floor, can exceed 2^31);
 * the arithmetic keeps it as a float, only the integer handed back saturates. */
static int32_t sat_i32(float v)
{
    if (!(v == v)) return 0;
    if (v >= 2147483648.0f) return INT32_MAX;
    if (v <= -2147483648.0f) return INT32_MIN;
    return (int32_t)v;
}

void zo_or_quant_group(const float* x, int n, int bits, int sym,
                       float* step_out, int32_t* zp_out, int32_t* codes, float* xhat)
{
    float qn, qp, step, mn = 0.0f;
    if (sym) {
        float amax = 0.0f;
        for (int i = 0; i < n; ++i) { float a = fabsf(x[i]); if (a > amax) amax = a; }
        qp = (float)((1 << (bits - 1)) - 1);
        qn = -(float)(1 << (bits - 1));
        step = amax / qp;
    } else {
        float mx = x[0];
        mn = x[0];
        for (int i = 1; i < n; ++i) { if (x[i] < mn) mn = x[i]; if (x[i] > mx) mx = x[i]; }
        qp = (float)((1 << bits) - 1);
        qn = 0.0f;
        step = (mx - mn) / qp;
    }
    if (step < ZO_OR_STEP_MIN) step = ZO_OR_STEP_MIN;
    float inv = 1.0f / step;                           /* one division per group */
    float zpf = sym ? 0.0f : -rintf(mn * inv);
    for (int i = 0; i < n; ++i) {
        float q = rintf(x[i] * inv) + zpf;
        if (q < qn) q = qn;
        if (q > qp) q = qp;
        if (codes) codes[i] = sat_i32(q);
        if (xhat)  xhat[i]  = (q - zpf) * step;
    }
    if (step_out) *step_out = step;
    if (zp_out)   *zp_out   = sat_i32(zpf);
}

/* Weight fake-quantizer: W[N,K] row-major, groups of `group` consecutive k
 * inside one output channel (group == K is per-channel).  bits == 0 means the
 * tensor is perturbed but not quantized.  round_bf16 rounds w^ to bf16, the
 * storage type of the GEMM operand in bf16 mode.  Any output may be NULL. */
void zo_or_fakequant_weight(const float* W, int N, int K, int bits, int group,
                            uint64_t seed, int32_t tensor_id, float eps_signed, int round_bf16,
                            int32_t* codes, float* step, int32_t* zp, float* what)
{
    int G = (bits > 0) ? K / group : 0;
    #pragma omp parallel for schedule(static)
    for (int n = 0; n < N; ++n) {
        float* wp  = (float*)malloc(sizeof(float) * (size_t)K);   /* perturbed row */
        float* hat = (float*)malloc(sizeof(float) * (size_t)K);   /* de-quantized row */
        for (int k = 0; k < K; ++k) {
            int64_t i = (int64_t)n * K + k;
            float z = (eps_signed == 0.0f) ? 0.0f : zo_or_z(seed, tensor_id, i);
            wp[k] = fmaf(eps_signed, z, W[i]);
        }
        if (bits == 0) {
            memcpy(hat, wp, sizeof(float) * (size_t)K);
        } else {
            for (int k = 0; k < K; k += group) {
                int64_t gi = (int64_t)n * G + k / group;
                zo_or_quant_group(wp + k, group, bits, 0,
                                  step ? step + gi : NULL, zp ? zp + gi : NULL,
                                  codes ? codes + (int64_t)n * K + k : NULL, hat + k);
            }
        }
        if (what)
            for (int k = 0; k < K; ++k)
                what[(int64_t)n * K + k] = round_bf16 ? zo_or_bf16_round(hat[k]) : hat[k];
        free(wp);
        free(hat);
    }
}

/* ------------------------------------------------------------------ */
/* Adaptive weight quantizer (Eq. 5): learnable step, zero point and    */
/* clipping coefficients per group,                                     */
/*   code = clamp(round(w/step) + z, alpha*Q_P, beta*Q_P),              */
/*   w^   = (code - z) * step.                                          */
/* Readings: the four are real-valued fp32 tensors that the ZO step     */
/* perturbs and updates; inside the forward z and the two bounds are    */
/* rounded to integers (half to even) so that codes stay integers, the  */
/* bounds are kept inside [0, Q_P] and ordered, the step is floored at  */
/* 1e-5 and w/step is w * (1/step) as in the dynamic quantizer.         */
/* ------------------------------------------------------------------ */
void zo_or_quant_group_learned(const float* x, int n, int bits, float step, float zp,
                               float alpha, float beta, int32_t* codes, float* xhat)
{
    float qp = (float)((1 << bits) - 1);
    float st = step;
    if (!(st >= ZO_OR_STEP_MIN)) st = ZO_OR_STEP_MIN;
    float inv = 1.0f / st;
    float zr = rintf(zp);
    float lo = rintf(alpha * qp);
    float hi = rintf(beta * qp);
    if (lo < 0.0f) lo = 0.0f;
    if (lo > qp) lo = qp;
    if (hi > qp) hi = qp;
    if (hi < lo) hi = lo;
    for (int i = 0; i < n; ++i) {
        float q = rintf(x[i] * inv) + zr;
        if (q < lo) q = lo;
        if (q > hi) q = hi;
        if (codes) codes[i] = sat_i32(q);
        if (xhat)  xhat[i]  = (q - zr) * st;
    }
}

/* Weight side of a linear with learnable quantizer parameters, optionally
 * smoothed (Eq. 4: the weight operand is s (.) W, s per input feature):
 *   w'   = fma(eps_signed, u, w)                 (perturbed master)
 *   wbar = scale[k] * w'                         (scale == NULL: no smoothing)
 *   w^   = Eq. 5 on wbar with the group's (step, zp, alpha, beta)
 * scale and the four parameter arrays ([N][K/group]) are passed in already
 * perturbed.  Any output may be NULL. */
void zo_or_fakequant_weight_learned(const float* W, int N, int K, int bits, int group,
                                    uint64_t seed, int32_t tensor_id, float eps_signed,
                                    const float* scale, const float* step, const float* zp,
                                    const float* alpha, const float* beta, int round_bf16,
                                    int32_t* codes, float* what)
{
    int G = K / group;
    #pragma omp parallel for schedule(static)
    for (int n = 0; n < N; ++n) {
        float* wb  = (float*)malloc(sizeof(float) * (size_t)K);
        float* hat = (float*)malloc(sizeof(float) * (size_t)K);
        for (int k = 0; k < K; ++k) {
            int64_t i = (int64_t)n * K + k;
            float z = (eps_signed == 0.0f) ? 0.0f : zo_or_z(seed, tensor_id, i);
            float wp = fmaf(eps_signed, z, W[i]);
            wb[k] = scale ? scale[k] * wp : wp;
        }
        for (int g = 0; g < G; ++g) {
            int64_t gi = (int64_t)n * G + g;
            zo_or_quant_group_learned(wb + g * group, group, bits, step[gi], zp[gi], alpha[gi], beta[gi],
                                      codes ? codes + (int64_t)n * K + g * group : NULL, hat + g * group);
        }
        if (what)
            for (int k = 0; k < K; ++k)
                what[(int64_t)n * K + k] = round_bf16 ? zo_or_bf16_round(hat[k]) : hat[k];
        free(wb);
        free(hat);
    }
}

/* Initial values (Eq. 5: "initialized based on the default asymmetric
 * quantization scheme"): step and zero point of the dynamic quantizer on
 * scale (.) W, alpha = 0, beta = 1. */
void zo_or_init_learned(const float* W, int N, int K, int bits, int group, const float* scale,
                        float* step, float* zp, float* alpha, float* beta)
{
    int G = K / group;
    #pragma omp parallel for schedule(static)
    for (int n = 0; n < N; ++n) {
        float* wb = (float*)malloc(sizeof(float) * (size_t)K);
        for (int k = 0; k < K; ++k) wb[k] = scale ? scale[k] * W[(int64_t)n * K + k] : W[(int64_t)n * K + k];
        for (int g = 0; g < G; ++g) {
            int64_t gi = (int64_t)n * G + g;
            float st;
            int32_t z;
            zo_or_quant_group(wb + g * group, group, bits, 0, &st, &z, NULL, NULL);
            step[gi] = st;
            zp[gi] = (float)z;
            alpha[gi] = 0.0f;
            beta[gi] = 1.0f;
        }
        free(wb);
    }
}

/* Activation side of Eq. 4: xbar = (x - delta[k]) * (1 / s[k]), fp32, one
 * correctly rounded division per channel (inv_s is passed in). */
void zo_or_smooth_act(const float* X, int M, int K, const float* delta, const float* inv_s, float* out)
{
    #pragma omp parallel for schedule(static)
    for (int m = 0; m < M; ++m)
        for (int k = 0; k < K; ++k) {
            int64_t i = (int64_t)m * K + k;
            out[i] = (X[i] - delta[k]) * inv_s[k];
        }
}

/* ------------------------------------------------------------------ */
/* Frozen, pre-quantized weights (Section "Lightweight ZeroQAT"):       */
/* 4-bit codes packed two per byte + one fp16 step and one int16 zero   */
/* point per group.  The paper fixes no storage format; this one is the */
/* build's reading.                                                     */
/* ------------------------------------------------------------------ */

/* fp32 -> IEEE binary16 bits, round to nearest even, subnormals kept,
 * overflow to infinity.  Written with integer arithmetic only. */
uint16_t zo_or_f32_to_f16_bits(float v)
{
    uint32_t u;
    memcpy(&u, &v, 4);
    uint32_t sign = (u >> 16) & 0x8000u;
    uint32_t mag = u & 0x7FFFFFFFu;
    if (mag >= 0x7F800000u)                          /* inf / nan */
        return (uint16_t)(sign | 0x7C00u | ((mag > 0x7F800000u) ? 0x200u : 0u));
    int32_t e = (int32_t)(mag >> 23) - 127;          /* unbiased exponent */
    uint32_t m = (mag & 0x7FFFFFu) | 0x800000u;      /* 24-bit significand, 1.xxx */
    if (mag < 0x00800000u) return (uint16_t)sign;    /* fp32 subnormal: far below half's range */
    /* value = m * 2^(e-23).  half: normal needs e >= -14; below that the
     * spacing is fixed at 2^-24. */
    int shift;                                       /* bits dropped from m */
    uint32_t base;                                   /* exponent field contribution */
    if (e >= -14) { shift = 13; base = (uint32_t)(e + 15) << 10; }
    else          { shift = 13 + (-14 - e); base = 0; }
    if (shift > 25) return (uint16_t)sign;           /* rounds to zero */
    uint32_t keep = m >> shift;
    uint32_t rem  = m & ((1u << shift) - 1u);
    uint32_t half = 1u << (shift - 1);
    if (rem > half || (rem == half && (keep & 1u))) keep += 1u;
    /* normal: keep has the implicit bit at position 10; adding base-0x400
     * lets a carry out of the significand bump the exponent. */
    uint32_t h = (e >= -14) ? (base - 0x400u + keep) : keep;
    if (h >= 0x7C00u) h = 0x7C00u;                   /* overflow */
    return (uint16_t)(sign | h);
}

float zo_or_f16_bits_to_f32(uint16_t h)
{
    uint32_t sign = ((uint32_t)h & 0x8000u) << 16;
    int32_t e = (h >> 10) & 0x1F;
    uint32_t m = h & 0x3FFu;
    float mag;
    if (e == 0)       mag = ldexpf((float)m, -24);
    else if (e == 31) mag = m ? NAN : INFINITY;
    else              mag = ldexpf((float)(m | 0x400u), e - 25);
    uint32_t u;
    memcpy(&u, &mag, 4);
    u |= sign;
    memcpy(&mag, &u, 4);
    return mag;
}

/* Pre-quantize W[N,K] (no perturbation) with the asymmetric 4-bit group
 * quantizer above.  Outputs: packed[N][K/2], byte j of a row holds the code
 * of k = 2j in its low nibble and of k = 2j+1 in its high nibble;
 * step_f16[N][K/group] the group step rounded to binary16;
 * zp[N][K/group] the zero point saturated to int16. */
void zo_or_pack_int4(const float* W, int N, int K, int group,
                     uint8_t* packed, uint16_t* step_f16, int16_t* zp)
{
    int G = K / group;
    #pragma omp parallel for schedule(static)
    for (int n = 0; n < N; ++n) {
        int32_t* codes = (int32_t*)malloc(sizeof(int32_t) * (size_t)group);
        for (int g = 0; g < G; ++g) {
            float st;
            int32_t z;
            zo_or_quant_group(W + (int64_t)n * K + (int64_t)g * group, group, 4, 0, &st, &z, codes, NULL);
            step_f16[(int64_t)n * G + g] = zo_or_f32_to_f16_bits(st);
            zp[(int64_t)n * G + g] = (int16_t)(z < -32768 ? -32768 : (z > 32767 ? 32767 : z));
            for (int k = 0; k < group; k += 2)
                packed[((int64_t)n * K + (int64_t)g * group + k) / 2] =
                    (uint8_t)((codes[k] & 15) | ((codes[k + 1] & 15) << 4));
        }
        free(codes);
    }
}

/* w^[n,k] = (code - zp) * step, step read back from binary16, product in
 * fp32 (the integer difference is exact in fp32), optionally rounded to
 * bf16, the GEMM operand type. */
void zo_or_dequant_int4(const uint8_t* packed, const uint16_t* step_f16, const int16_t* zp,
                        int N, int K, int group, int round_bf16, float* what)
{
    int G = K / group;
    #pragma omp parallel for schedule(static)
    for (int n = 0; n < N; ++n)
        for (int k = 0; k < K; ++k) {
            int64_t i = (int64_t)n * K + k;
            uint8_t byte = packed[i / 2];
            int code = (k & 1) ? (byte >> 4) : (byte & 15);
            int64_t gi = (int64_t)n * G + k / group;
            float st = zo_or_f16_bits_to_f32(step_f16[gi]);
            float v = (float)(code - (int)zp[gi]) * st;
            what[i] = round_bf16 ? zo_or_bf16_round(v) : v;
        }
}

/* Per-token activation fake-quantizer: each row of X[M,K] is one group.
 * bits >= 16 means no quantization. */
void zo_or_fakequant_act(const float* X, int M, int K, int bits, int sym, int round_bf16,
                         int32_t* codes, float* step, int32_t* zp, float* xhat)
{
    #pragma omp parallel for schedule(static)
    for (int m = 0; m < M; ++m) {
        const float* x = X + (int64_t)m * K;
        float* h = xhat ? xhat + (int64_t)m * K : NULL;
        if (bits >= 16) {
            if (h) memcpy(h, x, sizeof(float) * (size_t)K);
        } else {
            zo_or_quant_group(x, K, bits, sym, step ? step + m : NULL, zp ? zp + m : NULL,
                              codes ? codes + (int64_t)m * K : NULL, h);
        }
        if (h && round_bf16) for (int k = 0; k < K; ++k) h[k] = zo_or_bf16_round(h[k]);
    }
}

/* y[m,n] = sum_k x[m,k] * w[n,k] + bias[n], accumulated in fp64. */
void zo_or_linear(const float* x, const float* w, const float* bias, int M, int N, int K, double* y)
{
    #pragma omp parallel for schedule(static)
    for (int m = 0; m < M; ++m)
        for (int n = 0; n < N; ++n) {
            double acc = 0.0;
            for (int k = 0; k < K; ++k) acc += (double)x[(int64_t)m * K + k] * (double)w[(int64_t)n * K + k];
            y[(int64_t)m * N + n] = acc + (bias ? (double)bias[n] : 0.0);
        }
}

/* Projected gradient (Eq. 2 with q = 1): g = (L+ - L-) / (2 eps), formed in
 * fp64 from the two fp32 losses and stored as fp32. */
float zo_or_projected_grad(float loss_plus, float loss_minus, float eps)
{
    return (float)(((double)loss_plus - (double)loss_minus) / (2.0 * (double)eps));
}

/* Step coefficient c = eta * g (Eq. 3), formed in fp64, stored as fp32. */
float zo_or_coeff(float lr, float g) { return (float)((double)lr * (double)g); }

/* Update (Eq. 3): w_i <- w_i - c * z_i with z regenerated from the seed. */
void zo_or_update(float* w, int64_t n, uint64_t seed, int32_t tensor_id, float c)
{
    #pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < n; ++i) w[i] = fmaf(-c, zo_or_z(seed, tensor_id, i), w[i]);
}


/* ------------------------------------------------------------------ */
/* Master weights stored in IEEE binary16 (memory table of the         */
/* efficiency section: the ZeroQAT rows are 2 bytes per parameter).    */
/* Forward: the stored value, converted exactly to fp32, takes the     */
/* place of w everywhere (w' = fma(s eps, u, w) in fp32, never stored).*/
/* Update (Eq. 3): x = fma(-c, u, w) in fp32, then one rounding to     */
/* binary16 -- to nearest even, or stochastically: x goes to its upper */
/* neighbour hi with probability (x - lo) / (hi - lo), else to lo, so  */
/* that the expectation of the stored value is x even when |c u| is    */
/* far below the spacing of binary16 (a reading: the paper does not    */
/* say how the 16-bit weights are rounded).                            */
/* ------------------------------------------------------------------ */

/* Uniform 24-bit integer of element i for the stochastic rounding: the top 24 bits of word (i & 3)
 * of block (i >> 2) of a second stream, counter = (block low, block high, tensor_id, 1) -- the
 * perturbation stream uses 0 in the last counter word, so the two never share a block. */
uint32_t zo_or_round_bits(uint64_t seed, int32_t tensor_id, int64_t i)
{
    uint64_t blk = (uint64_t)i >> 2;
    uint32_t ctr[4] = { (uint32_t)blk, (uint32_t)(blk >> 32), (uint32_t)tensor_id, 1u };
    uint32_t key[2] = { (uint32_t)seed, (uint32_t)(seed >> 32) };
    uint32_t w[4];
    zo_or_philox4x32_10(ctr, key, w);
    return w[i & 3] >> 8;
}

/* neighbours of a finite binary16 value on the real line (bit patterns) */
static uint16_t f16_next_up(uint16_t h)
{
    if ((h & 0x7FFFu) == 0) return 0x0001u;          /* +-0 -> smallest positive */
    return (h & 0x8000u) ? (uint16_t)(h - 1) : (uint16_t)(h + 1);
}
static uint16_t f16_next_down(uint16_t h)
{
    if ((h & 0x7FFFu) == 0) return 0x8001u;          /* +-0 -> smallest negative */
    return (h & 0x8000u) ? (uint16_t)(h + 1) : (uint16_t)(h - 1);
}

/* x -> binary16 with stochastic rounding driven by the 24-bit integer r: exactly representable
 * values, infinities, NaNs and values that round to infinity go through the nearest-even
 * conversion; otherwise lo < x < hi are the neighbouring binary16 values and the result is hi
 * iff r * (hi - lo) / 2^24 < x - lo (all three quantities exact in fp32). */
uint16_t zo_or_f32_to_f16_stochastic(float x, uint32_t r)
{
    uint16_t h = zo_or_f32_to_f16_bits(x);
    if ((h & 0x7C00u) == 0x7C00u) return h;
    float f = zo_or_f16_bits_to_f32(h);
    if (f == x) return h;
    uint16_t lo = (f < x) ? h : f16_next_down(h);
    uint16_t hi = (f < x) ? f16_next_up(h) : h;
    float flo = zo_or_f16_bits_to_f32(lo), fhi = zo_or_f16_bits_to_f32(hi);
    float ulp = fhi - flo;                           /* a power of two */
    float d = x - flo;                               /* exact: 0 < d < ulp */
    float t = (float)r * (ulp * 0x1p-24f);           /* exact: 24-bit integer times a power of two */
    return (t < d) ? hi : lo;
}

/* Update of binary16 masters: w_i <- round16(fma(-c, u_i, w_i)). */
void zo_or_update_f16(uint16_t* w, int64_t n, uint64_t seed, int32_t tensor_id, float c, int stochastic)
{
    #pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < n; ++i) {
        float x = fmaf(-c, zo_or_z(seed, tensor_id, i), zo_or_f16_bits_to_f32(w[i]));
        w[i] = stochastic ? zo_or_f32_to_f16_stochastic(x, zo_or_round_bits(seed, tensor_id, i))
                          : zo_or_f32_to_f16_bits(x);
    }
}

/* One rounding of fp32 values to binary16 (nearest even, or stochastic with the rounding stream of `seed`). */
void zo_or_round_array_f16(const float* x, int64_t n, uint64_t seed, int32_t tensor_id, int stochastic, uint16_t* out)
{
    #pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < n; ++i)
        out[i] = stochastic ? zo_or_f32_to_f16_stochastic(x[i], zo_or_round_bits(seed, tensor_id, i)) : zo_or_f32_to_f16_bits(x[i]);
}
