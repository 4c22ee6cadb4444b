// 4-bit quantisation of parameter tensors at create time (MXFP4, weight-only).
// Part of the tn_linear library's single translation unit: included by tn_linear.hip inside its
// anonymous namespace, after kernels/common.hpp.
#pragma once

// ---------------------------------------------------------------------------------------------
// The paper names 4-bit quantisation of the tensor-network cores as the step after factorisation (Section 6) and
// gives no scheme. The one taken here is the OCP microscaling format MXFP4: blocks of 32 consecutive elements of
// a tensor's row-major flattening share a power-of-two scale X = 2^(floor(log2 max|v|) - 2) (an E8M0 exponent,
// clamped to -127 .. 127; -127 for an all-zero block), and an element is v / X rounded to the nearest E2M1 value
// {0, 0.5, 1, 1.5, 2, 3, 4, 6} (ties to the value with an even mantissa bit, saturating at 6) with a sign bit.
// One thread per block: block maximum, exponent, the eight-way comparison that picks the code, the packed codes
// (two per byte, the even element in the low nibble), the exponent byte and the dequantised values, which are
// exact in bf16 (three significant bits) and are what the contraction kernels multiply with.
// ---------------------------------------------------------------------------------------------
__global__ void __launch_bounds__(256) mxfp4_quantize_kernel(const bf16_t* src, int64_t n, unsigned char* codes,
                                                             signed char* exps, bf16_t* deq) {
    const int64_t n_blocks = (n + 31) / 32;
    for (int64_t b = int64_t(blockIdx.x) * 256 + threadIdx.x; b < n_blocks; b += int64_t(gridDim.x) * 256) {
        const int64_t base = b * 32;
        const int len = int(min(int64_t(32), n - base));
        float v[32];
        float amax = 0.f;
#pragma unroll
        for (int i = 0; i < 32; ++i) {
            v[i] = i < len ? float(src[base + i]) : 0.f;
            amax = fmaxf(amax, fabsf(v[i]));
        }
        int ex = 0;
        (void)frexpf(amax, &ex);                       // amax = m * 2^ex with m in [0.5, 1)
        int e = amax > 0.f ? ex - 1 - 2 : -127;
        e = max(-127, min(127, e));
        const float inv = ldexpf(1.f, -e);
        exps[b] = static_cast<signed char>(e);
        unsigned char nib[32];
#pragma unroll
        for (int i = 0; i < 32; ++i) {
            const float q = fabsf(v[i]) * inv;         // exact: a power-of-two scaling
            const int code = int(q > 0.25f) + int(q >= 0.75f) + int(q > 1.25f) + int(q >= 1.75f) + int(q > 2.5f) +
                             int(q >= 3.5f) + int(q > 5.0f);
            const int sign = (v[i] < 0.f && code > 0) ? 1 : 0;
            nib[i] = static_cast<unsigned char>(code | (sign << 3));
            // grid value: 0, 0.5, then 1 .. 6 = (2 + (code & 1)) * 2^((code >> 1) - 1) / 2 ... written out
            const float mag = code == 0 ? 0.f : (code == 1 ? 0.5f : ldexpf(1.f + 0.5f * float(code & 1), (code >> 1) - 1));
            if (i < len) deq[base + i] = bf16_t(ldexpf(sign ? -mag : mag, e));
        }
#pragma unroll
        for (int i = 0; i < 32; i += 2)
            if (i < len) codes[(base + i) >> 1] = static_cast<unsigned char>(nib[i] | (nib[i + 1] << 4));
    }
}
