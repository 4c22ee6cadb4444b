// Gradients with respect to the parameter tensors: the contraction step with the token index contracted.
// Part of the tn_linear library's single translation unit: included by tn_linear.hip inside its
// anonymous namespace, after kernels/stream.hpp.
#pragma once

// ---------------------------------------------------------------------------------------------
// A forward step computes Out[t, r, c] = sum_k In[t, r, k] P[c][k]. With dOut the gradient of the loss with
// respect to the step's output (Section 3.4: the factors are fine-tuned, so the loss is back-propagated through
// every contraction), the gradient with respect to the step's parameter tensor is the same contraction with the
// rows (tokens and row indices) summed instead of k:
//     dP[c][k] = sum_{t, r} dOut[t, r, c] * In[t, r, k]
// and the gradient with respect to its input, dIn[t, r, k] = sum_c dOut[t, r, c] P[c][k], is an ordinary step
// with the packed tensor transposed, which the step kernels run as they are (dOut is read through the forward
// step's scatter tables as gather tables).
// grad_param_kernel: a workgroup owns a 64 x 64 tile of (c, k) and a range of rows; rows go through LDS 16 at a
// time, plain fp32 FMA, any dtype, any addressing. The row range is split over workgroups when C*K alone would not
// fill the chip; every split writes its own fp32 tile and grad_reduce_kernel adds them in split order (no
// atomics: results are bit-reproducible) and scatters the sum to the caller's tensor layout.
// ---------------------------------------------------------------------------------------------
struct GradArgs {
    const void* dOut;
    const void* In;
    float* partial;            // [n_split][C][K]
    const int32_t* crow;       // position of (r, c) in a token of dOut: crow[r] + ccol[c]
    const int32_t* ccol;
    const int32_t* arow;       // position of (r, k) in a token of In: arow[r] + acol[k]; null: r*K + k
    const int32_t* acol;
    int64_t c_tok_stride, a_tok_stride;
    uint32_t total_rows, R;
    int32_t K, C;
    uint32_t rows_per_split;
};

template <typename T>
__global__ void __launch_bounds__(256) grad_param_kernel(GradArgs a) {
    constexpr int BC = 64, BK = 64, BG = 16;
    __shared__ float sD[BG][BC + 4];
    __shared__ float sI[BG][BK + 4];
    const T* dOut = static_cast<const T*>(a.dOut);
    const T* In = static_cast<const T*>(a.In);
    const int tid = threadIdx.x;
    const int c0 = blockIdx.x * BC, k0 = blockIdx.y * BK;
    const uint32_t g_begin = blockIdx.z * a.rows_per_split;
    const uint32_t g_end = min(a.total_rows, g_begin + a.rows_per_split);
    const int tx = tid & 15, ty = tid >> 4;            // thread: c = c0 + 4*ty .. +3, k = k0 + 4*tx .. +3
    float acc[4][4] = {};
    for (uint32_t g0 = g_begin; g0 < g_end; g0 += BG) {
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int e = tid + 256 * j;
            const int gg = e >> 6, cc = e & 63;
            const uint32_t g = g0 + gg;
            float vd = 0.f, vi = 0.f;
            if (g < g_end) {
                const uint32_t t = g / a.R;
                const uint32_t r = g - t * a.R;
                if (c0 + cc < a.C) vd = to_float(dOut[int64_t(t) * a.c_tok_stride + a.crow[r] + a.ccol[c0 + cc]]);
                if (k0 + cc < a.K)
                    vi = to_float(In[int64_t(t) * a.a_tok_stride +
                                     (a.arow ? int64_t(a.arow[r]) + a.acol[k0 + cc] : int64_t(r) * a.K + k0 + cc)]);
            }
            sD[gg][cc] = vd;
            sI[gg][cc] = vi;
        }
        __syncthreads();
#pragma unroll
        for (int gg = 0; gg < BG; ++gg) {
            float dv[4], iv[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) dv[i] = sD[gg][ty * 4 + i];
#pragma unroll
            for (int j = 0; j < 4; ++j) iv[j] = sI[gg][tx * 4 + j];
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
                for (int j = 0; j < 4; ++j) acc[i][j] = fmaf(dv[i], iv[j], acc[i][j]);
        }
        __syncthreads();
    }
    float* out = a.partial + int64_t(blockIdx.z) * a.C * a.K;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int c = c0 + ty * 4 + i;
        if (c >= a.C) continue;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int k = k0 + tx * 4 + j;
            if (k < a.K) out[int64_t(c) * a.K + k] = acc[i][j];
        }
    }
}

// grad[position of (c, k) in the caller's tensor] (+)= sum over splits of partial[split][c][k]. The position follows the
// step's packing recipe (PackArgs: digits of k and c times their strides); a tensor with a traced index pair (a
// ring of one core) receives the value at every diagonal position and keeps zeros elsewhere (the caller's buffer
// is cleared first by grad_fill_kernel).
struct GradOutArgs {
    const float* partial;
    float* grad;
    int32_t C, K, n_split, accumulate;
    int32_t nk, nc;
    int64_t kext[tn::kMaxGatherDims], kstr[tn::kMaxGatherDims];
    int64_t cext[tn::kMaxGatherDims], cstr[tn::kMaxGatherDims];
    int64_t trace_extent, trace_stride;
};

__global__ void __launch_bounds__(256) grad_reduce_kernel(GradOutArgs a) {
    const int64_t total = int64_t(a.C) * a.K;
    for (int64_t e = int64_t(blockIdx.x) * 256 + threadIdx.x; e < total; e += int64_t(gridDim.x) * 256) {
        float sum = 0.f;
        for (int s = 0; s < a.n_split; ++s) sum += a.partial[int64_t(s) * total + e];
        int64_t c = e / a.K, k = e - c * a.K, off = 0;
        for (int j = a.nk - 1; j >= 0; --j) {
            off += (k % a.kext[j]) * a.kstr[j];
            k /= a.kext[j];
        }
        for (int j = a.nc - 1; j >= 0; --j) {
            off += (c % a.cext[j]) * a.cstr[j];
            c /= a.cext[j];
        }
        for (int64_t d = 0; d < a.trace_extent; ++d) {
            float* p = a.grad + off + d * a.trace_stride;
            *p = a.accumulate ? *p + sum : sum;
        }
    }
}

__global__ void __launch_bounds__(256) grad_fill_kernel(float* p, int64_t n) {
    for (int64_t e = int64_t(blockIdx.x) * 256 + threadIdx.x; e < n; e += int64_t(gridDim.x) * 256) p[e] = 0.f;
}
