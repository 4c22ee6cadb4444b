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

// ---------------------------------------------------------------------------------------------
// The 4-bit form as decode-size kernels stream it. A step whose contraction index walks the caller's tensor in
// memory order (K consecutive elements per column, K a multiple of 32, every column starting at a block boundary)
// reads one block of 32 codes per lane and load: the stream is cut into pieces of 32 columns x 64 k, piece
// (cb, chunk) holding for lane l the 16 bytes of block 2*chunk + l/32 of column 32*cb + l%32, followed in a second
// array by that block's exponent as a biased byte (e + 127: shifted left by 23 it is the float 2^e). Four MFMA
// k-steps are fed from one such load: k-step u takes codes 8u .. 8u+7 of the lane's block, so lanes 0-31 supply
// k = 64*chunk + 8u .. and lanes 32-63 k = 64*chunk + 32 + 8u ..; the other operand is fetched in the same order.
// Blocks past K and columns past C are zero codes with a zero scale.
// ---------------------------------------------------------------------------------------------
struct Q4PackArgs {
    const unsigned char* codes;    // the tensor's codes in the caller's order, 16 bytes per block
    const signed char* exps;       // one exponent per block
    uint4* out_codes;              // [col_blocks][n_chunks][64]
    unsigned char* out_scales;     // [col_blocks][n_chunks][64]
    int32_t C, K, n_chunks, col_blocks, nc;
    int64_t cext[tn::kMaxGatherDims], cstr[tn::kMaxGatherDims];      // digits of c: extent, stride in elements
};

__global__ void __launch_bounds__(256) q4_stream_pack_kernel(Q4PackArgs a) {
    const int64_t total = int64_t(a.col_blocks) * a.n_chunks * 64;
    for (int64_t i = int64_t(blockIdx.x) * 256 + threadIdx.x; i < total; i += int64_t(gridDim.x) * 256) {
        const int lane = int(i & 63);
        const int64_t piece = i >> 6;
        const int chunk = int(piece % a.n_chunks);
        const int cb = int(piece / a.n_chunks);
        const int c = cb * 32 + (lane & 31);
        const int blk = 2 * chunk + (lane >> 5);
        uint4 v = make_uint4(0u, 0u, 0u, 0u);
        unsigned char sc = 0;
        if (c < a.C && blk * 32 < a.K) {
            int64_t rem = c, off = 0;
            for (int j = a.nc - 1; j >= 0; --j) {
                off += (rem % a.cext[j]) * a.cstr[j];
                rem /= a.cext[j];
            }
            const int64_t b = (off >> 5) + blk;
            v = reinterpret_cast<const uint4*>(a.codes)[b];
            sc = static_cast<unsigned char>(int(a.exps[b]) + 127);
        }
        a.out_codes[i] = v;
        a.out_scales[i] = sc;
    }
}

typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));

// One lane's block of 32 codes times 2^e as the four MFMA operands it feeds (8 values each). The conversion
// instruction takes two codes (one byte, the even element in the low nibble) and the scale as a float.
__device__ __forceinline__ void q4_dequant_block(const uint4& codes, unsigned scale_byte, bf16x8 (&out)[4]) {
    const float scale = __uint_as_float(scale_byte << 23);
    const unsigned w[4] = {codes.x, codes.y, codes.z, codes.w};
#pragma unroll
    for (int u = 0; u < 4; ++u) {
        const bf16x2_t p0 = __builtin_amdgcn_cvt_scalef32_pk_bf16_fp4(w[u], scale, 0);
        const bf16x2_t p1 = __builtin_amdgcn_cvt_scalef32_pk_bf16_fp4(w[u], scale, 1);
        const bf16x2_t p2 = __builtin_amdgcn_cvt_scalef32_pk_bf16_fp4(w[u], scale, 2);
        const bf16x2_t p3 = __builtin_amdgcn_cvt_scalef32_pk_bf16_fp4(w[u], scale, 3);
        out[u][0] = p0[0]; out[u][1] = p0[1];
        out[u][2] = p1[0]; out[u][3] = p1[1];
        out[u][4] = p2[0]; out[u][5] = p2[1];
        out[u][6] = p3[0]; out[u][7] = p3[1];
    }
}
