// Device-side argument blocks, vector types, the fragment-major packing map and small helpers.
// Part of the tn_linear library's single translation unit: included by tn_linear.hip inside its
// anonymous namespace, after <hip/hip_runtime.h> and tn_plan.hpp.
#pragma once

// ---------------------------------------------------------------------------------------------
// device-side argument blocks
// ---------------------------------------------------------------------------------------------
struct StepArgs {
    const void* A;
    const void* B;
    void* Out;
    const int32_t* arow;   // gather tables for A (null when A is plain)
    const int32_t* acol;
    const int32_t* crow;   // scatter tables for Out
    const int32_t* ccol;
    int64_t a_tok_stride;
    int64_t c_tok_stride;
    uint32_t total_rows;   // tokens * R
    uint32_t R;
    int32_t K, Kp, C, Cp;
    const void* Bs = nullptr;   // 4-bit stream: the block scales (B then holds the codes)
};

struct PackArgs {
    const void* src;
    void* dst;
    int32_t K, Kp, C, Cp;
    int32_t nk, nc;
    int64_t kext[tn::kMaxGatherDims], kstr[tn::kMaxGatherDims];
    int64_t cext[tn::kMaxGatherDims], cstr[tn::kMaxGatherDims];
    int64_t trace_extent, trace_stride;
};

typedef __bf16 bf16_t;
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float floatx16 __attribute__((ext_vector_type(16)));
typedef float floatx4 __attribute__((ext_vector_type(4)));

// Packed parameter tensors are stored "fragment-major": the [Cp][Kp] matrix is cut into blocks of
// 32 columns x 16 k; a block is 64 chunks of 8 consecutive k (16 bytes in bf16), chunk l holding
// column l%32 and k offset 8*(l/32) - exactly the operand one lane of v_mfma_f32_32x32x16_bf16
// wants. A wave that reads a block with one 16-byte load per lane therefore fetches 1 KB of
// contiguous memory straight into MFMA operand registers (decode path), and the tiled kernels
// read whole 1 KB blocks as well. Element (c, k) lives at:
__host__ __device__ __forceinline__ int64_t bfrag_offset(int c, int k, int nks /* Kp / 16 */) {
    return (int64_t(c >> 5) * nks + (k >> 4)) * 512 + ((c & 31) + 32 * ((k >> 3) & 1)) * 8 + (k & 7);
}

__device__ __forceinline__ float to_float(float v) { return v; }
__device__ __forceinline__ float to_float(bf16_t v) { return float(v); }
template <typename T> __device__ __forceinline__ T from_float(float v);
template <> __device__ __forceinline__ float from_float<float>(float v) { return v; }
template <> __device__ __forceinline__ bf16_t from_float<bf16_t>(float v) { return bf16_t(v); }

