/* Driver for the host sanitizer pass over the oracle's C file (test infrastructure): every exported routine is called
 * on heap buffers of exactly the size its contract names, with ragged shapes, the degenerate groups (constant,
 * all-positive, huge range) and extreme inputs (infinities, NaN, subnormals, the largest element index), so that
 * AddressSanitizer sees any access past a buffer and UndefinedBehaviorSanitizer any overflowing shift, conversion or
 * index.  Build: gcc -O1 -g -fsanitize=address,undefined -fno-sanitize-recover=all -fopenmp zo_oracle.c sanitize_main.c -lm */
#include <math.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

void zo_or_philox4x32_10(const uint32_t ctr[4], const uint32_t key[2], uint32_t out[4]);
void zo_or_philox_words(uint64_t seed, int32_t tensor_id, int64_t nwords, uint32_t* out);
void zo_or_word_to_normals(uint32_t w, float out[2]);
float zo_or_z(uint64_t seed, int32_t tensor_id, int64_t i);
void zo_or_normal(uint64_t seed, int32_t tensor_id, int64_t start, int64_t n, float* out);
float zo_or_bf16_round(float v);
void zo_or_bf16_round_array(const float* in, int64_t n, float* out);
void zo_or_perturb(const float* w, int64_t n, uint64_t seed, int32_t tensor_id, float eps_signed, float* out);
void zo_or_quant_group(const float* x, int n, int bits, int sym, float* step_out, int32_t* zp_out, int32_t* codes, float* xhat);
void zo_or_fakequant_weight(const float* W, int N, int K, int bits, int group, uint64_t seed, int32_t tensor_id, float eps_signed,
                            int round_bf16, int32_t* codes, float* step, int32_t* zp, float* what);
void zo_or_quant_group_learned(const float* x, int n, int bits, float step, float zp, float alpha, float beta, int32_t* codes, float* xhat);
void zo_or_fakequant_weight_learned(const float* W, int N, int K, int bits, int group, uint64_t seed, int32_t tensor_id, float eps_signed,
                                    const float* scale, const float* step, const float* zp, const float* alpha, const float* beta,
                                    int round_bf16, int32_t* codes, float* what);
void zo_or_init_learned(const float* W, int N, int K, int bits, int group, const float* scale, float* step, float* zp, float* alpha, float* beta);
void zo_or_smooth_act(const float* X, int M, int K, const float* delta, const float* inv_s, float* out);
uint16_t zo_or_f32_to_f16_bits(float v);
float zo_or_f16_bits_to_f32(uint16_t h);
void zo_or_pack_int4(const float* W, int N, int K, int group, uint8_t* packed, uint16_t* step_f16, int16_t* zp);
void zo_or_dequant_int4(const uint8_t* packed, const uint16_t* step_f16, const int16_t* zp, int N, int K, int group, int round_bf16, float* what);
void zo_or_fakequant_act(const float* X, int M, int K, int bits, int sym, int round_bf16, int32_t* codes, float* step, int32_t* zp, float* xhat);
void zo_or_linear(const float* x, const float* w, const float* bias, int M, int N, int K, double* y);
float zo_or_projected_grad(float loss_plus, float loss_minus, float eps);
float zo_or_coeff(float lr, float g);
void zo_or_update(float* w, int64_t n, uint64_t seed, int32_t tensor_id, float c);
uint32_t zo_or_round_bits(uint64_t seed, int32_t tensor_id, int64_t i);
uint16_t zo_or_f32_to_f16_stochastic(float x, uint32_t r);
void zo_or_update_f16(uint16_t* w, int64_t n, uint64_t seed, int32_t tensor_id, float c, int stochastic);
void zo_or_round_array_f16(const float* x, int64_t n, uint64_t seed, int32_t tensor_id, int stochastic, uint16_t* out);

static float* fbuf(size_t n) { float* p = (float*)malloc(n * sizeof(float) + (n == 0)); if (!p) exit(2); return p; }
static uint32_t lcg = 12345u;
static float rnd(void) { lcg = lcg * 1664525u + 1013904223u; return ((float)(lcg >> 8) / 8388608.0f - 1.0f); }

int main(void)
{
    /* perturbation stream, including the largest representable element index and seed */
    uint32_t ctr[4] = {0xFFFFFFFFu, 0xFFFFFFFFu, 0xFFFFFFFFu, 0xFFFFFFFFu}, key[2] = {0xFFFFFFFFu, 0xFFFFFFFFu}, out4[4];
    zo_or_philox4x32_10(ctr, key, out4);
    uint32_t* words = (uint32_t*)malloc(37 * 4);
    zo_or_philox_words(UINT64_MAX, INT32_MAX, 37, words);
    free(words);
    float pair[2];
    zo_or_word_to_normals(0u, pair);
    zo_or_word_to_normals(0xFFFFFFFFu, pair);
    (void)zo_or_z(7, 3, INT64_MAX);
    (void)zo_or_z(UINT64_MAX, -1, 0);
    float* nrm = fbuf(1003);
    zo_or_normal(5, 2, ((int64_t)1 << 40) + 5, 1003, nrm);
    free(nrm);
    /* storage rounding on special values */
    const float specials[8] = {0.0f, -0.0f, INFINITY, -INFINITY, NAN, 1e-45f, 3.4e38f, -1.17549435e-38f};
    float* sp = fbuf(8); memcpy(sp, specials, sizeof(specials));
    float* spo = fbuf(8);
    zo_or_bf16_round_array(sp, 8, spo);
    for (int i = 0; i < 8; ++i) { (void)zo_or_f16_bits_to_f32(zo_or_f32_to_f16_bits(sp[i])); (void)zo_or_f32_to_f16_stochastic(sp[i], 0xFFFFFFu); }
    for (uint32_t h = 0; h < 65536u; h += 97u) (void)zo_or_f32_to_f16_bits(zo_or_f16_bits_to_f32((uint16_t)h));
    free(sp); free(spo);
    /* quantizer on ragged shapes and degenerate groups */
    const int N = 7, K = 96, group = 32, G = K / group;
    float* W = fbuf((size_t)N * K);
    for (int i = 0; i < N * K; ++i) W[i] = 0.02f * rnd();
    for (int k = 0; k < K; ++k) { W[0 * K + k] = 0.5f; W[1 * K + k] = 1.0f + 1e-3f * rnd(); W[2 * K + k] = (k & 1) ? 3e38f : -3e38f; W[3 * K + k] = 1e30f; }      /* constant, far from zero: the zero point exceeds int32 */
    for (int bits = 1; bits <= 8; ++bits) {
        int32_t* codes = (int32_t*)malloc((size_t)N * K * 4);
        float* step = fbuf((size_t)N * G); int32_t* zp = (int32_t*)malloc((size_t)N * G * 4); float* what = fbuf((size_t)N * K);
        zo_or_fakequant_weight(W, N, K, bits, group, 11, 4, 1e-3f, bits & 1, codes, step, zp, what);
        zo_or_fakequant_weight(W, N, K, bits, K, 11, 4, -1e-3f, 0, NULL, step, zp, what);      /* per channel, no codes */
        float* st = fbuf((size_t)N * G), *z = fbuf((size_t)N * G), *al = fbuf((size_t)N * G), *be = fbuf((size_t)N * G), *scale = fbuf(K);
        for (int k = 0; k < K; ++k) scale[k] = 1.0f + 0.1f * rnd();
        zo_or_init_learned(W, N, K, bits, group, scale, st, z, al, be);
        for (int i = 0; i < N * G; ++i) { al[i] += 0.6f * rnd(); be[i] += 0.6f * rnd(); z[i] += 300.0f * rnd(); }   /* crossed and out-of-range bounds */
        zo_or_fakequant_weight_learned(W, N, K, bits, group, 11, 4, 1e-3f, scale, st, z, al, be, 1, codes, what);
        zo_or_fakequant_weight_learned(W, N, K, bits, group, 11, 4, 1e-3f, NULL, st, z, al, be, 0, NULL, what);
        int32_t c1[5]; float x1[5] = {1.0f, 1.0f, 1.0f, 1.0f, 1.0f}, xh[5], s1; int32_t z1;
        zo_or_quant_group(x1, 5, bits, 0, &s1, &z1, c1, xh);
        if (bits >= 2) zo_or_quant_group(x1, 5, bits, 1, &s1, &z1, c1, xh);
        zo_or_quant_group_learned(x1, 5, bits, 1e-9f, -1e9f, 2.0f, -1.0f, c1, xh);
        free(codes); free(step); free(zp); free(what); free(st); free(z); free(al); free(be); free(scale);
    }
    zo_or_fakequant_weight(W, N, K, 0, 0, 11, 4, 1e-3f, 1, NULL, NULL, NULL, W);              /* bits 0: perturb only, in place */
    /* activations: per-token quantizer (asymmetric / symmetric), smoothing, linear */
    const int M = 5;
    float* X = fbuf((size_t)M * K);
    for (int i = 0; i < M * K; ++i) X[i] = rnd();
    for (int k = 0; k < K; ++k) X[3 * K + k] = 0.0f;
    for (int bits = 2; bits <= 8; bits += 3)
        for (int sym = 0; sym < 2; ++sym) {
            int32_t* codes = (int32_t*)malloc((size_t)M * K * 4); float* step = fbuf(M); int32_t* zp = (int32_t*)malloc(M * 4); float* xhat = fbuf((size_t)M * K);
            zo_or_fakequant_act(X, M, K, bits, sym, sym, codes, step, zp, xhat);
            free(codes); free(step); free(zp); free(xhat);
        }
    float* xh16 = fbuf((size_t)M * K);
    zo_or_fakequant_act(X, M, K, 16, 0, 1, NULL, NULL, NULL, xh16);
    float* delta = fbuf(K), *inv = fbuf(K), *sm = fbuf((size_t)M * K);
    for (int k = 0; k < K; ++k) { delta[k] = 0.1f * rnd(); inv[k] = 1.0f + 0.1f * rnd(); }
    zo_or_smooth_act(X, M, K, delta, inv, sm);
    double* y = (double*)malloc((size_t)M * N * 8); float* bias = fbuf(N);
    for (int n = 0; n < N; ++n) bias[n] = rnd();
    zo_or_linear(xh16, W, bias, M, N, K, y);
    zo_or_linear(xh16, W, NULL, M, N, K, y);
    free(xh16); free(delta); free(inv); free(sm); free(y); free(bias);
    /* packed 4-bit storage */
    for (int g = 8; g <= 32; g *= 2) {
        const int Gp = K / g;
        uint8_t* packed = (uint8_t*)malloc((size_t)N * K / 2); uint16_t* st16 = (uint16_t*)malloc((size_t)N * Gp * 2); int16_t* zp16 = (int16_t*)malloc((size_t)N * Gp * 2);
        float* what = fbuf((size_t)N * K);
        zo_or_pack_int4(W, N, K, g, packed, st16, zp16);
        zo_or_dequant_int4(packed, st16, zp16, N, K, g, g == 16, what);
        free(packed); free(st16); free(zp16); free(what);
    }
    /* estimator and updates */
    (void)zo_or_projected_grad(6.5f, 6.4f, 1e-3f);
    (void)zo_or_projected_grad(INFINITY, 1.0f, 1e-3f);
    (void)zo_or_coeff(1e-6f, -3.0f);
    float* w = fbuf(1001);
    for (int i = 0; i < 1001; ++i) w[i] = rnd();
    zo_or_update(w, 1001, 9, 1, 2.5e-4f);
    zo_or_update(w, 0, 9, 1, 2.5e-4f);
    uint16_t* w16 = (uint16_t*)malloc(1001 * 2);
    zo_or_round_array_f16(w, 1001, 9, 1, 0, w16);
    zo_or_round_array_f16(w, 1001, 9, 1, 1, w16);
    zo_or_update_f16(w16, 1001, 9, 1, 1e-5f, 0);
    zo_or_update_f16(w16, 1001, 9, 1, 1e-5f, 1);
    (void)zo_or_round_bits(UINT64_MAX, INT32_MAX, INT64_MAX);
    free(w); free(w16); free(W); free(X);
    puts("oracle sanitizer pass: ok");
    return 0;
}
