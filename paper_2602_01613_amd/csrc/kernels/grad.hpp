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
    int32_t c_tiles, k_tiles, n_split;      // grad_param_mfma_kernel: a one-dimensional grid of c_tiles * k_tiles * n_split workgroups
    int32_t d_mode, i_mode;                 // grad_param_mfma_kernel: how dOut and In are loaded (see there)
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

// The same contraction on the matrix cores, for bf16 layers: a workgroup owns a 128 x 128 tile of (c, k), each of
// its four waves a 64 x 64 quarter (2 x 2 MFMA tiles, fp32 accumulators). The contracted index is the row g, which
// is the slow index of both operands in memory, while an MFMA lane supplies 8 consecutive values of the contracted
// index: so the rows go through LDS 32 at a time, stored transposed ([column][g]), and a fragment is one 16-byte LDS
// read. Waves 0-1 bring the 128 x 32 block of dOut, waves 2-3 that of In, each through the forward step's own tables,
// in the widest pieces the operand's layout allows (GradArgs::d_mode, i_mode):
//   1  8 consecutive columns of a row are one aligned 16-byte piece: a thread loads 4 rows x 8 columns, transposes
//      them in registers and writes 8 pieces of 4 consecutive g;
//   2  8 consecutive rows of a column are one aligned 16-byte piece (dOut of a step whose output runs along the row
//      index; R % 8 == 0): such a piece is 8 consecutive g as it stands;
//   0  neither: one element per lane and load, lanes along the columns of one row (the row of a load is the same
//      for the whole wave, so its token and table entry sit in scalar registers).
// The loads of the next 32 rows are requested before the current ones are multiplied. Row ranges start at multiples
// of 32. Partial tiles as in grad_param_kernel.
__global__ void __launch_bounds__(256) grad_param_mfma_kernel(GradArgs a) {
    // LDS row of column x: 32 + 8 bf16 (80 bytes), and every 8 columns 16 bytes more, so that the 8-byte writes of
    // mode 1 (lanes 8 columns = 640 bytes apart) do not all fall on one bank
    constexpr int BT = 128, BG = 32, PITCH = BG + 8, LDS_ELEMS = BT * PITCH + (BT / 8) * 8;
    auto row_of = [](int x) { return x * PITCH + ((x >> 3) << 3); };
    __shared__ __attribute__((aligned(16))) bf16_t sD[LDS_ELEMS];
    __shared__ __attribute__((aligned(16))) bf16_t sI[LDS_ELEMS];
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    // workgroup -> (tile, split). With a multiple of 8 splits, all tiles of one split run on one XCD (workgroups are
    // dealt to the 8 XCDs in turn): the rows of a split then come from memory once, into that XCD's L2, for all of its
    // tiles, instead of once per XCD.
    const int tiles = a.c_tiles * a.k_tiles;
    int tile, split;
    if ((a.n_split & 7) == 0) {
        const int xcd = blockIdx.x & 7, j = blockIdx.x >> 3;
        tile = j % tiles;
        split = (j / tiles) * 8 + xcd;
    } else {
        tile = blockIdx.x % tiles;
        split = blockIdx.x / tiles;
    }
    const int c0 = (tile % a.c_tiles) * BT, k0 = (tile / a.c_tiles) * BT;
    const uint32_t g_begin = min(a.total_rows, uint32_t(split) * a.rows_per_split);
    const uint32_t g_end = min(a.total_rows, g_begin + a.rows_per_split);

    // ---- this wave's operand (wave-uniform)
    const bool is_d = wave < 2;
    const bf16_t* src = static_cast<const bf16_t*>(is_d ? a.dOut : a.In);
    const int32_t* rowtab = is_d ? a.crow : a.arow;             // null: plain In, row r at r*K
    const int32_t* coltab = is_d ? a.ccol : a.acol;             // null: plain In, column k at k
    const int64_t tok_stride = is_d ? a.c_tok_stride : a.a_tok_stride;
    const int mode = is_d ? a.d_mode : a.i_mode;
    const int ext = is_d ? a.C : a.K, x0 = is_d ? c0 : k0;
    bf16_t* sdst = is_d ? sD : sI;
    const int u = tid & 127;
    // modes 0 and 2: thread -> column u; mode 1: thread -> (columns 8*(u%16) .. +7, rows 4*(u/16) .. +3 of the 32)
    const int col = x0 + (mode == 1 ? 8 * (u & 15) : u);
    const bool vcol = col < ext;                                // mode 1: ext % 8 == 0, the whole piece is inside
    // table entries are offsets inside one token: non-negative, below 2^31 (checked when the plan is built)
    const uint32_t coff = vcol ? (coltab ? uint32_t(coltab[col]) : uint32_t(col)) : 0u;
    bf16x8 reg[4];
    auto request = [&](uint32_t g0) {
        bf16x8 zero;
#pragma unroll
        for (int e = 0; e < 8; ++e) zero[e] = bf16_t(0.f);
        if (mode == 1) {
            // per-lane rows: g0 + 4*(u/16) + j
            uint32_t g = g0 + 4u * uint32_t(u >> 4);
            uint32_t t = g / a.R, r = g - t * a.R;
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                reg[j] = zero;
                if (g + uint32_t(j) < g_end && vcol) {
                    const int64_t ro = rowtab ? int64_t(rowtab[r]) : int64_t(r) * a.K;
                    reg[j] = *reinterpret_cast<const bf16x8*>(src + int64_t(t) * tok_stride + ro + coff);
                }
                if (++r == a.R) {
                    r = 0;
                    ++t;
                }
            }
        } else if (mode == 2) {
            // rows g0 + 8q .. +7: one token, one aligned run of the row table (R % 8 == 0, g0 % 8 == 0)
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const uint32_t g = g0 + 8u * uint32_t(q);       // wave-uniform
                reg[q] = zero;
                if (g < g_end && vcol) {
                    const uint32_t t = g / a.R, r = g - t * a.R;
                    reg[q] = *reinterpret_cast<const bf16x8*>(src + (int64_t(t) * tok_stride + rowtab[r]) + coff);
                }
            }
        } else {
            uint32_t t = g0 / a.R, r = g0 - t * a.R;            // wave-uniform
            // all 32 row offsets first (scalar table reads, one wait), then the loads back to back
            int64_t ro[BG];
#pragma unroll
            for (int j = 0; j < BG; ++j) {
                ro[j] = g0 + uint32_t(j) < g_end ? int64_t(t) * tok_stride + (rowtab ? int64_t(rowtab[r]) : int64_t(r) * a.K) : -1;
                if (++r == a.R) {
                    r = 0;
                    ++t;
                }
            }
#pragma unroll
            for (int j = 0; j < BG; ++j)
                reg[j >> 3][j & 7] = (ro[j] >= 0 && vcol) ? (src + ro[j])[coff] : bf16_t(0.f);
        }
    };
    auto deposit = [&]() {
        if (mode == 1) {
            typedef __bf16 bf16x4_t __attribute__((ext_vector_type(4)));
            const int cl = 8 * (u & 15), gq = 4 * (u >> 4);
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                bf16x4_t v;
#pragma unroll
                for (int j = 0; j < 4; ++j) v[j] = reg[j][e];
                *reinterpret_cast<bf16x4_t*>(sdst + row_of(cl + e) + gq) = v;
            }
        } else {
#pragma unroll
            for (int q = 0; q < 4; ++q) *reinterpret_cast<bf16x8*>(sdst + row_of(u) + 8 * q) = reg[q];
        }
    };
    // wave -> quarter (wc, wk); MFMA row operand: c, column operand: k; lane l supplies g = 8*(l/32) .. +7 of a k-step
    const int wc = wave >> 1, wk = wave & 1;
    floatx16 acc[2][2];
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;
    if (g_begin < g_end) request(g_begin);
    for (uint32_t g0 = g_begin; g0 < g_end; g0 += BG) {
        deposit();
        __syncthreads();
        if (g0 + BG < g_end) request(g0 + BG);
#pragma unroll
        for (int ks = 0; ks < 2; ++ks) {
            bf16x8 fd[2], fi[2];
#pragma unroll
            for (int i = 0; i < 2; ++i) {
                fd[i] = *reinterpret_cast<const bf16x8*>(sD + row_of(64 * wc + 32 * i + (lane & 31)) + 16 * ks + 8 * (lane >> 5));
                fi[i] = *reinterpret_cast<const bf16x8*>(sI + row_of(64 * wk + 32 * i + (lane & 31)) + 16 * ks + 8 * (lane >> 5));
            }
#pragma unroll
            for (int i = 0; i < 2; ++i)
#pragma unroll
                for (int j = 0; j < 2; ++j) acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fd[i], fi[j], acc[i][j], 0, 0, 0);
        }
        __syncthreads();                                        // everyone has read the group before it is overwritten
    }
    // lane l, register v of acc[i][j]: c = c0 + 64*wc + 32*i + 8*(v/4) + 4*(l/32) + v%4, k = k0 + 64*wk + 32*j + l%32
    float* out = a.partial + int64_t(split) * a.C * a.K;
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j) {
            const int k = k0 + 64 * wk + 32 * j + (lane & 31);
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int c = c0 + 64 * wc + 32 * i + 8 * (v >> 2) + 4 * (lane >> 5) + (v & 3);
                if (c < a.C && k < a.K) out[int64_t(c) * a.K + k] = acc[i][j][v];
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
