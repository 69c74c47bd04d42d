// Measurement probe, not part of the step: a kernel that does nothing but issue bf16 matrix instructions on register-resident
// operands -- the rate the matrix cores sustain on this card with no memory traffic at all, against which the GEMM kernel's
// figure can be read next to the published peak.  The shader clock is power managed and depends on the operand DATA: all-zero
// operands run faster than operands with random mantissas, so the probe takes either.
#include "zo_device.h"
#include "zo_internal.h"
#include "../../include/zoqat.h"

typedef __bf16 probe_bf16x8 __attribute__((ext_vector_type(8)));
typedef float probe_f32x16 __attribute__((ext_vector_type(16)));

// 4 waves per workgroup, 8 independent 32 x 32 x 16 accumulators per wave (128 accumulator registers, as the GEMM's waves hold),
// iters rounds of 8 matrix instructions: 4 * 8 * 32768 * iters flop per workgroup
__global__ __launch_bounds__(256) void zo_probe_mfma_kernel(float* __restrict__ out, int iters, int zero_operands)
{
    probe_bf16x8 a[4], b[4];
    uint32_t r = threadIdx.x * 2654435761u + blockIdx.x * 40503u + 12345u;
#pragma unroll
    for (int j = 0; j < 4; ++j)
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            // xorshift: a sign, an exponent within three binades of 1, seven random mantissa bits
            r ^= r << 13; r ^= r >> 17; r ^= r << 5;
            uint16_t ha = (uint16_t)(((r & 1) << 15) | ((120 + ((r >> 1) & 7)) << 7) | ((r >> 8) & 127));
            r ^= r << 13; r ^= r >> 17; r ^= r << 5;
            uint16_t hb = (uint16_t)(((r & 1) << 15) | ((120 + ((r >> 1) & 7)) << 7) | ((r >> 8) & 127));
            if (zero_operands) { ha = 0; hb = 0; }
            a[j][i] = __builtin_bit_cast(__bf16, ha);
            b[j][i] = __builtin_bit_cast(__bf16, hb);
        }
    probe_f32x16 acc[8];
#pragma unroll
    for (int i = 0; i < 8; ++i)
#pragma unroll
        for (int q = 0; q < 16; ++q) acc[i][q] = 0.0f;
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int i = 0; i < 8; ++i) acc[i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[i & 3], b[(i >> 1) & 3], acc[i], 0, 0, 0);
    }
    float s = 0.0f;
#pragma unroll
    for (int i = 0; i < 8; ++i)
#pragma unroll
        for (int q = 0; q < 16; ++q) s += acc[i][q];
    out[(int64_t)blockIdx.x * 256 + threadIdx.x] = s;
}

extern "C" zo_status zo_probe_mfma_only(float* out_dev, int32_t workgroups, int32_t iters, int32_t zero_operands, void* hip_stream)
{
    if (!out_dev || workgroups < 1 || workgroups > 65535 || iters < 1 || iters > (1 << 22)) return ZO_EINVAL;
    zo_probe_mfma_kernel<<<workgroups, 256, 0, (hipStream_t)hip_stream>>>(out_dev, iters, zero_operands);
    return hipGetLastError() == hipSuccess ? ZO_OK : ZO_EHIP;
}
