// Create-time repacking of the caller's tensors (Section 3.5: contiguous, kernel-friendly parameter storage).
// Part of the tn_linear library's single translation unit: included by tn_linear.hip inside its
// anonymous namespace, after <hip/hip_runtime.h> and tn_plan.hpp.
#pragma once

// ---------------------------------------------------------------------------------------------
// create-time repack: Bp(c, k) = sum_a src[off_c(c) + off_k(k) + a*trace_stride], zero padded to
// [Cp][Kp] and stored fragment-major
// ---------------------------------------------------------------------------------------------
template <typename T>
__global__ void __launch_bounds__(256) pack_kernel(PackArgs p) {
    int64_t total = int64_t(p.Cp) * p.Kp;
    for (int64_t i = int64_t(blockIdx.x) * blockDim.x + threadIdx.x; i < total;
         i += int64_t(gridDim.x) * blockDim.x) {
        int32_t c = int32_t(i / p.Kp);
        int32_t k = int32_t(i - int64_t(c) * p.Kp);
        float v = 0.f;
        if (c < p.C && k < p.K) {
            int64_t off = 0;
            int32_t rem = k;
            for (int j = p.nk - 1; j >= 0; --j) {
                int32_t e = int32_t(p.kext[j]);
                int32_t q = rem / e;
                off += int64_t(rem - q * e) * p.kstr[j];
                rem = q;
            }
            rem = c;
            for (int j = p.nc - 1; j >= 0; --j) {
                int32_t e = int32_t(p.cext[j]);
                int32_t q = rem / e;
                off += int64_t(rem - q * e) * p.cstr[j];
                rem = q;
            }
            const T* s = static_cast<const T*>(p.src);
            if (p.trace_extent == 1) {
                static_cast<T*>(p.dst)[bfrag_offset(c, k, p.Kp >> 4)] = s[off];
                continue;
            }
            for (int64_t a = 0; a < p.trace_extent; ++a) v += to_float(s[off + a * p.trace_stride]);
        }
        static_cast<T*>(p.dst)[bfrag_offset(c, k, p.Kp >> 4)] = from_float<T>(v);
    }
}

