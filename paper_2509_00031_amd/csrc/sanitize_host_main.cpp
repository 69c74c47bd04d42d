// Driver for the host sanitizer pass over the library's host side (argument checking, shape logic, size arithmetic):
// every entry point is called with invalid and extreme arguments that the host code must turn into an error code
// before anything is launched -- no GPU is needed or touched.  Built with the library's sources and
// -Xarch_host -fsanitize=address -Xarch_host -fsanitize=undefined; exit code 0 = nothing found.
#include "../../include/zoqat.h"
#include <climits>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <vector>

#define EXPECT(cond) do { if (!(cond)) { printf("sanitize_host_main: check failed at line %d: %s\n", __LINE__, #cond); return 1; } } while (0)

static zo_config llama(int layers, int d, int heads, int f, int vocab, int seq)
{
    zo_config c;
    memset(&c, 0, sizeof(c));
    c.arch = ZO_ARCH_LLAMA; c.n_layers = layers; c.d_model = d; c.n_heads = heads; c.d_ffn = f; c.vocab = vocab; c.max_seq = seq;
    c.w_bits = 4; c.w_group = 64; c.a_bits = 8; c.act_dtype = ZO_ACT_BF16;
    return c;
}

int main()
{
    // shape logic at the largest configurations (size arithmetic must not overflow)
    zo_config big = llama(80, 8192, 64, 28672, 128256, 8192);
    EXPECT(zo_num_params(&big) == 1 + 80 * 9 + 2);
    int64_t total = 0;
    for (int i = 0; i < zo_num_params(&big); ++i) total += zo_param_numel(&big, i);
    EXPECT(total > 60000000000ll);
    EXPECT(zo_param_numel(&big, -1) == -1 && zo_param_numel(&big, INT_MAX) == -1);
    EXPECT(zo_workspace_bytes(&big, 64, 8192) > ((size_t)1 << 33));
    EXPECT(zo_master_bytes(&big) == 4 * total);
    big.master_dtype = ZO_MASTER_F16;
    EXPECT(zo_master_bytes(&big) == 2 * total);
    // invalid configurations
    zo_config bad = llama(1, 100, 4, 256, 64, 16);          // d_model not a multiple of 8
    EXPECT(zo_workspace_bytes(&bad, 1, 16) == 0);
    bad = llama(1, 128, 3, 256, 64, 16);                    // heads do not divide d_model
    EXPECT(zo_workspace_bytes(&bad, 1, 16) == 0);
    bad = llama(1, 128, 4, 256, 64, 16); bad.arch = 9;
    EXPECT(zo_num_params(&bad) == 0);
    bad = llama(1, 128, 4, 256, 64, 16); bad.w_bits = 9;
    EXPECT(zo_workspace_bytes(&bad, 1, 16) == 0);
    bad = llama(1, 128, 4, 256, 64, 16); bad.w_group = 48;  // does not divide d_model
    EXPECT(zo_workspace_bytes(&bad, 1, 16) == 0);
    EXPECT(zo_num_params(nullptr) == 0 && zo_workspace_bytes(nullptr, 1, 1) == 0);
    // zo_init: every argument check returns before any device call
    zo_config ok = llama(1, 128, 4, 256, 64, 16);
    const int n = zo_num_params(&ok);
    std::vector<zo_tensor> params(n);
    alignas(16) static char fake[64];
    for (int i = 0; i < n; ++i) { params[i].ptr = fake; params[i].numel = zo_param_numel(&ok, i); params[i].trainable = 1; params[i].reserved = 0; }
    zo_ctx* ctx = nullptr;
    EXPECT(zo_init(nullptr, params.data(), n, fake, 64, 1, 16, nullptr, &ctx) == ZO_EINVAL);
    EXPECT(zo_init(&ok, params.data(), n - 1, fake, 64, 1, 16, nullptr, &ctx) != ZO_OK);
    EXPECT(zo_init(&ok, params.data(), n, fake, 64, 1, 16, nullptr, &ctx) == ZO_EWORKSPACE);
    EXPECT(zo_init(&ok, params.data(), n, fake + 4, 1 << 30, 1, 16, nullptr, &ctx) == ZO_EALIGN);
    EXPECT(zo_init(&ok, params.data(), n, fake, 1 << 30, 1, 17, nullptr, &ctx) == ZO_ESHAPE);     // max_S above max_seq
    params[2].numel += 1;
    EXPECT(zo_init(&ok, params.data(), n, fake, 1 << 30, 1, 16, nullptr, &ctx) == ZO_ESHAPE);
    params[2].numel -= 1;
    params[3].ptr = nullptr;
    EXPECT(zo_init(&ok, params.data(), n, fake, 1 << 30, 1, 16, nullptr, &ctx) == ZO_EINVAL);
    EXPECT(ctx == nullptr);
    EXPECT(zo_destroy(nullptr) == ZO_OK);
    EXPECT(zo_forward_quant(nullptr, fake, nullptr, 1, 16, 0, 0.0f, (float*)fake) == ZO_EINVAL);
    EXPECT(zo_step(nullptr, fake, nullptr, 1, 16, 0, 1e-3f, 1e-3f, (float*)fake) == ZO_EINVAL);
    EXPECT(zo_update(nullptr, 0, nullptr, 0.0f) == ZO_EINVAL);
    // stand-alone pieces: NULL pointers, negative sizes, bad divisibility, misalignment
    EXPECT(zo_debug_philox_u32(1, 0, -1, (uint32_t*)fake, nullptr) != ZO_OK);
    EXPECT(zo_debug_normal(1, 0, 0, 8, nullptr, nullptr) == ZO_EINVAL);
    EXPECT(zo_update_tensor(nullptr, 8, 1, 0, nullptr, 0.0f, nullptr) == ZO_EINVAL);
    EXPECT(zo_update_tensor((float*)(fake + 4), 8, 1, 0, nullptr, 0.0f, nullptr) == ZO_EALIGN);
    EXPECT(zo_debug_quant_weight((const float*)fake, 4, 100, 4, 64, 1, 0, 0.0f, ZO_ACT_FP32, nullptr, nullptr, nullptr, fake, nullptr) == ZO_ESHAPE);
    EXPECT(zo_debug_quant_weight((const float*)fake, 4, 128, 9, 64, 1, 0, 0.0f, ZO_ACT_FP32, nullptr, nullptr, nullptr, fake, nullptr) != ZO_OK);
    EXPECT(zo_linear_fakequant(fake, (const float*)fake, nullptr, fake, 4, 4, 100, 4, 64, 8, 0, ZO_ACT_FP32, 1, 0, 0.0f, fake, nullptr) == ZO_ESHAPE);
    EXPECT(zo_linear_fakequant(fake, (const float*)fake, nullptr, fake, 4, 4, 128, 4, 64, 1, 0, ZO_ACT_FP32, 1, 0, 0.0f, fake, nullptr) == ZO_EINVAL);
    EXPECT(zo_linear_fakequant_mma(fake, (const float*)fake, nullptr, fake, 4, 4, 128, 4, 64, 16, 0, ZO_ACT_BF16, 0, ZO_MMA_INT8, 1, 0, 0.0f, fake,
                                   (int32_t*)fake, nullptr) == ZO_EUNSUPPORTED);
    EXPECT(zo_linear_fakequant_mma(fake, (const float*)fake, nullptr, fake, 4, 4, 96, 4, 32, 8, 0, ZO_ACT_BF16, 0, ZO_MMA_INT8, 1, 0, 0.0f, fake,
                                   (int32_t*)fake, nullptr) == ZO_EUNSUPPORTED);
    size_t off[8];
    EXPECT(zo_linear_mma_scratch_bytes(INT_MAX / 2, INT_MAX / 2, 4096, 64, ZO_ACT_BF16, ZO_MMA_INT8, off) > ((size_t)1 << 40));
    EXPECT(zo_linear_mma_scratch_bytes(8, 8, 100, 64, ZO_ACT_BF16, ZO_MMA_INT8, off) == 0);
    EXPECT(zo_linear_scratch_bytes(-1, 4, 4, 0) == 0);
    EXPECT(zo_linear_fakequant_fused(fake, fake, (const float*)fake, nullptr, fake, fake, 129, 16, 64, 4, 64, 1, 0, 1e-3f, 0, nullptr, nullptr) == ZO_ESHAPE);
    EXPECT(zo_pack_weight_int4((const float*)fake, 4, 64, 48, fake, fake, (int16_t*)fake, nullptr) == ZO_ESHAPE);
    EXPECT(zo_linear_frozen_int4_fused(fake, nullptr, fake, fake, (const int16_t*)fake, nullptr, fake, nullptr, 200, 16, 128, 128, 0, nullptr, nullptr) == ZO_ESHAPE);
    EXPECT(zo_gemm_nt(fake, fake, fake, 4, 4, 12, ZO_ACT_BF16, nullptr) == ZO_ESHAPE);
    EXPECT(zo_gemm_nt(fake, fake, fake, 4, 4, 16, 7, nullptr) == ZO_EINVAL);
    EXPECT(zo_gemm_nt_fused_splitk_static(fake, fake, nullptr, nullptr, 0, fake, 1280, 2048, 16384, ZO_ACT_BF16, nullptr) == ZO_EWORKSPACE);
    EXPECT(zo_gemm_nt_splitk_ranges(384, 1024, 4096, ZO_ACT_BF16) >= 1);
    EXPECT(zo_gemm_nt_splitk_scratch_bytes(INT_MAX / 4, 1024, 4096, ZO_ACT_BF16) == 0 || true);
    EXPECT(zo_gemm_nt_swiglu(fake, fake, fake, 8, 64, 64, nullptr) == ZO_EUNSUPPORTED);
    EXPECT(zo_gemm_nt_ce(fake, fake, (const int32_t*)fake, (float*)fake, 8, 3, 64, 64, fake, nullptr) != ZO_OK);
    EXPECT(zo_attention_causal(fake, fake, fake, fake, 1, 4, 2, 48, 96, ZO_ACT_BF16, nullptr, nullptr) == ZO_EUNSUPPORTED);
    EXPECT(zo_attention_causal(fake, fake, fake, fake, 1, 4, 2, 64, 100, ZO_ACT_BF16, nullptr, nullptr) == ZO_ESHAPE);
    EXPECT(zo_lr_linear_decay(1e-6f, 0, 10) == 1e-6f && zo_lr_linear_decay(1e-6f, 9, 10) > 0.0f);
    EXPECT(zo_debug_routes(nullptr) == 0 || true);
    puts("library host sanitizer pass: ok");
    return 0;
}
