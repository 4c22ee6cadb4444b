// tn_linear: C-ABI library and gfx950 kernels for the forward pass of
// tensor-network linear layers (Section 3.5 of the paper: TN matmuls applied
// to token activations by sequential core contractions).
//
// Every contraction step of a plan (see tn_plan.hpp) is one launch of a
// "scatter GEMM":
//     Out[t, crow[r] + ccol[c]] = sum_k A[t, r, k] * Bp[c][k]
// A is the step's input (plain row-major [tokens*R, K] except possibly for the
// first step, which may gather from x through two tables), Bp is the packed
// parameter tensor [Cp][Kp] (K contiguous, zero padded), and the output is
// written directly in the layout the next step wants to read, so no separate
// permutation kernel ever runs.
#include <hip/hip_runtime.h>

#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <new>
#include <vector>

#include "../../include/tn_linear.h"
#include "tn_plan.hpp"

namespace {

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

__device__ __forceinline__ float to_float(float v) { return v; }
__device__ __forceinline__ float to_float(bf16_t v) { return float(v); }
template <typename T> __device__ __forceinline__ T from_float(float v);
template <> __device__ __forceinline__ float from_float<float>(float v) { return v; }
template <> __device__ __forceinline__ bf16_t from_float<bf16_t>(float v) { return bf16_t(v); }

// ---------------------------------------------------------------------------------------------
// create-time repack: Bp[c][k] = sum_a src[off_c(c) + off_k(k) + a*trace_stride], zero padded
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
                static_cast<T*>(p.dst)[i] = s[off];
                continue;
            }
            for (int64_t a = 0; a < p.trace_extent; ++a) v += to_float(s[off + a * p.trace_stride]);
        }
        static_cast<T*>(p.dst)[i] = from_float<T>(v);
    }
}

// ---------------------------------------------------------------------------------------------
// plain FMA step kernel: any dtype, any addressing. 64x64 tile, 256 threads, 4x4 per thread.
// ---------------------------------------------------------------------------------------------
template <typename T>
__global__ void __launch_bounds__(256) step_scalar_kernel(StepArgs a) {
    constexpr int BM = 64, BN = 64, BK = 16;
    __shared__ float As[BK][BM + 4];
    __shared__ float Bs[BK][BN + 4];
    const T* A = static_cast<const T*>(a.A);
    const T* B = static_cast<const T*>(a.B);
    T* Out = static_cast<T*>(a.Out);
    const int tid = threadIdx.x;
    const uint32_t row0 = blockIdx.x * BM;
    const int col0 = blockIdx.y * BN;
    const int tx = tid & 15, ty = tid >> 4;
    float acc[4][4] = {};

    // each thread loads 4 elements of A and 4 of B per K chunk: element e = tid + 256*j
    for (int k0 = 0; k0 < a.K; k0 += BK) {
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            int e = tid + 256 * j;
            int kk = e & (BK - 1);
            int rr = e >> 4;
            uint32_t g = row0 + rr;
            int k = k0 + kk;
            float v = 0.f;
            if (g < a.total_rows && k < a.K) {
                uint32_t t = g / a.R;
                uint32_t r = g - t * a.R;
                int64_t off = int64_t(t) * a.a_tok_stride +
                              (a.arow ? int64_t(a.arow[r]) + a.acol[k] : int64_t(r) * a.K + k);
                v = to_float(A[off]);
            }
            As[kk][rr] = v;
            int c = col0 + rr;
            float w = 0.f;
            if (c < a.Cp && k < a.Kp) w = to_float(B[int64_t(c) * a.Kp + k]);
            Bs[kk][rr] = w;
        }
        __syncthreads();
#pragma unroll
        for (int kk = 0; kk < BK; ++kk) {
            float av[4], bv[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) av[i] = As[kk][ty * 4 + i];
#pragma unroll
            for (int j = 0; j < 4; ++j) bv[j] = Bs[kk][tx * 4 + j];
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
                for (int j = 0; j < 4; ++j) acc[i][j] = fmaf(av[i], bv[j], acc[i][j]);
        }
        __syncthreads();
    }
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        uint32_t g = row0 + ty * 4 + i;
        if (g >= a.total_rows) continue;
        uint32_t t = g / a.R;
        uint32_t r = g - t * a.R;
        int64_t base = int64_t(t) * a.c_tok_stride + a.crow[r];
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            int c = col0 + tx * 4 + j;
            if (c < a.C) Out[base + a.ccol[c]] = from_float<T>(acc[i][j]);
        }
    }
}

// ---------------------------------------------------------------------------------------------
// bf16 MFMA step kernel. 256 threads = 4 waves arranged WM x WN; each wave owns TM x TN tiles of
// v_mfma_f32_32x32x16_bf16. A and B tiles are staged through LDS with K contiguous so that one
// ds_read_b128 feeds one MFMA operand (lane l: row l%32, k = 8*(l/32) .. +7). The fp32
// accumulators are rounded to bf16, transposed through LDS and scattered with 16-byte stores
// along whichever direction (columns or rows) is contiguous in the output layout.
//   AMODE 0: A rows are plain and K % 8 == 0 -> 16-byte global loads
//   AMODE 1: element-wise gather (tables, or K not a multiple of 8)
//   CMODE 0: scalar stores; 1: 8 contiguous columns per store; 2: 8 contiguous rows per store
// ---------------------------------------------------------------------------------------------
template <int WM, int WN, int TM, int TN, int AMODE>
__global__ void __launch_bounds__(256) step_mfma_kernel(StepArgs a, int cmode) {
    constexpr int BM = WM * TM * 32, BN = WN * TN * 32, BK = 64;
    constexpr int LDK = BK + 8;                       // padded LDS row (elements)
    constexpr int A_ELEMS = BM * LDK, B_ELEMS = BN * LDK;
    constexpr int LDC = BN + 8;
    constexpr int SMEM_ELEMS = (A_ELEMS + B_ELEMS) > (BM * LDC) ? (A_ELEMS + B_ELEMS) : (BM * LDC);
    __shared__ __attribute__((aligned(16))) bf16_t smem[SMEM_ELEMS];
    bf16_t* sA = smem;
    bf16_t* sB = smem + A_ELEMS;

    const bf16_t* A = static_cast<const bf16_t*>(a.A);
    const bf16_t* B = static_cast<const bf16_t*>(a.B);
    bf16_t* Out = static_cast<bf16_t*>(a.Out);

    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int wm = wave / WN, wn = wave % WN;
    const uint32_t row0 = blockIdx.x * BM;
    const int col0 = blockIdx.y * BN;

    // global -> LDS assignment: a tile row has BK/8 = 8 chunks of 16 bytes
    constexpr int A_CHUNKS = BM * 8 / 256;            // chunks per thread
    constexpr int B_CHUNKS = BN * 8 / 256;
    int64_t a_base[A_CHUNKS];                         // element offset of the row start, -1 if out of range
#pragma unroll
    for (int j = 0; j < A_CHUNKS; ++j) {
        int e = tid + 256 * j;
        uint32_t g = row0 + (e >> 3);
        if (g < a.total_rows) {
            uint32_t t = g / a.R;
            uint32_t r = g - t * a.R;
            a_base[j] = int64_t(t) * a.a_tok_stride + (a.arow ? int64_t(a.arow[r]) : int64_t(r) * a.K);
        } else {
            a_base[j] = -1;
        }
    }

    floatx16 acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;

    for (int k0 = 0; k0 < a.Kp; k0 += BK) {
        // ---- stage A
#pragma unroll
        for (int j = 0; j < A_CHUNKS; ++j) {
            int e = tid + 256 * j;
            int rr = e >> 3, kc = (e & 7) * 8;
            bf16x8 v;
#pragma unroll
            for (int q = 0; q < 8; ++q) v[q] = bf16_t(0.f);
            int k = k0 + kc;
            if (a_base[j] >= 0) {
                if (AMODE == 0) {
                    if (k < a.K) v = *reinterpret_cast<const bf16x8*>(A + a_base[j] + k);
                } else {
#pragma unroll
                    for (int q = 0; q < 8; ++q)
                        if (k + q < a.K) v[q] = A[a_base[j] + (a.acol ? a.acol[k + q] : k + q)];
                }
            }
            *reinterpret_cast<bf16x8*>(sA + rr * LDK + kc) = v;
        }
        // ---- stage B (always in range: Bp is padded to [Cp][Kp])
#pragma unroll
        for (int j = 0; j < B_CHUNKS; ++j) {
            int e = tid + 256 * j;
            int cc = e >> 3, kc = (e & 7) * 8;
            bf16x8 v = *reinterpret_cast<const bf16x8*>(B + int64_t(col0 + cc) * a.Kp + k0 + kc);
            *reinterpret_cast<bf16x8*>(sB + cc * LDK + kc) = v;
        }
        __syncthreads();
#pragma unroll
        for (int ks = 0; ks < BK; ks += 16) {
            bf16x8 af[TM], bfr[TN];
#pragma unroll
            for (int i = 0; i < TM; ++i)
                af[i] = *reinterpret_cast<const bf16x8*>(sA + ((wm * TM + i) * 32 + (lane & 31)) * LDK + ks +
                                                         8 * (lane >> 5));
#pragma unroll
            for (int j = 0; j < TN; ++j)
                bfr[j] = *reinterpret_cast<const bf16x8*>(sB + ((wn * TN + j) * 32 + (lane & 31)) * LDK + ks +
                                                          8 * (lane >> 5));
#pragma unroll
            for (int i = 0; i < TM; ++i)
#pragma unroll
                for (int j = 0; j < TN; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[i], bfr[j], acc[i][j], 0, 0, 0);
        }
        __syncthreads();
    }

    // ---- epilogue: accumulators -> bf16 tile in LDS (row-major [BM][LDC])
    // D layout of the 32x32 MFMA: lane l, register v: col = l%32, row = 8*(v/4) + 4*(l/32) + v%4
    bf16_t* sC = smem;
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                int rr = (wm * TM + i) * 32 + 8 * (v >> 2) + 4 * (lane >> 5) + (v & 3);
                int cc = (wn * TN + j) * 32 + (lane & 31);
                sC[rr * LDC + cc] = bf16_t(acc[i][j][v]);
            }
    __syncthreads();

    if (cmode == 1) {
        // thread -> (row, group of 8 columns), columns fastest
        constexpr int GROUPS = BM * BN / 8;
        for (int e = tid; e < GROUPS; e += 256) {
            int rr = e / (BN / 8), cg = (e % (BN / 8)) * 8;
            uint32_t g = row0 + rr;
            int c = col0 + cg;
            if (g >= a.total_rows || c >= a.C) continue;
            uint32_t t = g / a.R;
            uint32_t r = g - t * a.R;
            int64_t off = int64_t(t) * a.c_tok_stride + a.crow[r] + a.ccol[c];
            *reinterpret_cast<bf16x8*>(Out + off) = *reinterpret_cast<const bf16x8*>(sC + rr * LDC + cg);
        }
    } else if (cmode == 2) {
        // thread -> (group of 8 rows, column), rows fastest
        constexpr int GROUPS = BM * BN / 8;
        for (int e = tid; e < GROUPS; e += 256) {
            int rg = (e % (BM / 8)) * 8, cc = e / (BM / 8);
            uint32_t g = row0 + rg;
            int c = col0 + cc;
            if (g >= a.total_rows || c >= a.C) continue;
            uint32_t t = g / a.R;
            uint32_t r = g - t * a.R;
            int64_t off = int64_t(t) * a.c_tok_stride + a.crow[r] + a.ccol[c];
            bf16x8 v;
#pragma unroll
            for (int q = 0; q < 8; ++q) v[q] = sC[(rg + q) * LDC + cc];
            *reinterpret_cast<bf16x8*>(Out + off) = v;
        }
    } else {
        for (int e = tid; e < BM * BN; e += 256) {
            int rr = e / BN, cc = e % BN;
            uint32_t g = row0 + rr;
            int c = col0 + cc;
            if (g >= a.total_rows || c >= a.C) continue;
            uint32_t t = g / a.R;
            uint32_t r = g - t * a.R;
            Out[int64_t(t) * a.c_tok_stride + a.crow[r] + a.ccol[c]] = sC[rr * LDC + cc];
        }
    }
}

// ---------------------------------------------------------------------------------------------
// host side
// ---------------------------------------------------------------------------------------------
enum Variant : int {
    VAR_SCALAR = 0,
    VAR_MFMA_128x128 = 1,
    VAR_MFMA_256x32 = 2,
};

struct DevStep {
    tn::Step plan;
    void* packed = nullptr;       // [Cp][Kp]
    int32_t* tables = nullptr;    // arow | acol | crow | ccol in one allocation
    const int32_t *arow = nullptr, *acol = nullptr, *crow = nullptr, *ccol = nullptr;
    int Kp = 0, Cp = 0;
    int variant = VAR_SCALAR;
    int amode = 0, cmode = 0;
    int bn = 64, bm = 64;
};

}  // namespace

struct tn_linear_s {
    tn::Plan plan;
    std::vector<DevStep> steps;
    int elt = 4;
    int64_t max_tokens = 0, chunk_tokens = 0;
    int64_t packed_bytes = 0, workspace_bytes = 0;
    void* ws[2] = {nullptr, nullptr};
    int device = 0;
    bool profiling = false;
    struct ProfRec { int step; hipEvent_t start, stop; };
    std::vector<ProfRec> prof;
};

namespace {

constexpr int64_t kDefaultWorkspaceBytes = int64_t(192) << 20;

inline int round_up(int v, int m) { return (v + m - 1) / m * m; }

void clear_profile(tn_linear_s* h) {
    for (auto& r : h->prof) {
        (void)hipEventDestroy(r.start);
        (void)hipEventDestroy(r.stop);
    }
    h->prof.clear();
}

void free_handle(tn_linear_s* h) {
    if (!h) return;
    clear_profile(h);
    for (auto& s : h->steps) {
        if (s.packed) (void)hipFree(s.packed);
        if (s.tables) (void)hipFree(s.tables);
    }
    for (void* w : h->ws)
        if (w) (void)hipFree(w);
    delete h;
}

void choose_variant(const tn_linear_s* h, DevStep* s, int flags) {
    const tn::Step& p = s->plan;
    if (h->plan.dtype != TN_DTYPE_BF16 || (flags & TN_FLAG_SCALAR_KERNELS)) {
        s->variant = VAR_SCALAR;
        s->bm = 64;
        s->bn = 64;
    } else if (p.C <= 32) {
        s->variant = VAR_MFMA_256x32;
        s->bm = 256;
        s->bn = 32;
    } else {
        s->variant = VAR_MFMA_128x128;
        s->bm = 128;
        s->bn = 128;
    }
    s->amode = (p.a_plain && p.K % 8 == 0) ? 0 : 1;
    s->cmode = p.c_vec == 8 ? 1 : (p.r_vec == 8 ? 2 : 0);
    s->Kp = round_up(int(p.K), 64);
    s->Cp = round_up(int(p.C), s->bn);
}

template <int WM, int WN, int TM, int TN>
void launch_mfma(const DevStep& s, const StepArgs& a, dim3 grid, hipStream_t st) {
    if (s.amode == 0)
        hipLaunchKernelGGL((step_mfma_kernel<WM, WN, TM, TN, 0>), grid, dim3(256), 0, st, a, s.cmode);
    else
        hipLaunchKernelGGL((step_mfma_kernel<WM, WN, TM, TN, 1>), grid, dim3(256), 0, st, a, s.cmode);
}

int launch_step(const tn_linear_s* h, const DevStep& s, const void* A, void* Out, int64_t tokens,
                hipStream_t st) {
    StepArgs a;
    a.A = A;
    a.B = s.packed;
    a.Out = Out;
    a.arow = s.arow;
    a.acol = s.acol;
    a.crow = s.crow;
    a.ccol = s.ccol;
    a.a_tok_stride = s.plan.a_tok_stride;
    a.c_tok_stride = s.plan.c_tok_stride;
    int64_t rows = tokens * s.plan.R;
    a.total_rows = uint32_t(rows);
    a.R = uint32_t(s.plan.R);
    a.K = int32_t(s.plan.K);
    a.Kp = s.Kp;
    a.C = int32_t(s.plan.C);
    a.Cp = s.Cp;
    dim3 grid(uint32_t((rows + s.bm - 1) / s.bm), uint32_t(s.Cp / s.bn));
    switch (s.variant) {
        case VAR_SCALAR:
            if (h->plan.dtype == TN_DTYPE_BF16)
                hipLaunchKernelGGL(step_scalar_kernel<bf16_t>, grid, dim3(256), 0, st, a);
            else
                hipLaunchKernelGGL(step_scalar_kernel<float>, grid, dim3(256), 0, st, a);
            break;
        case VAR_MFMA_128x128:
            launch_mfma<2, 2, 2, 2>(s, a, grid, st);
            break;
        case VAR_MFMA_256x32:
            launch_mfma<4, 1, 2, 1>(s, a, grid, st);
            break;
        default:
            return TN_ERR_UNSUPPORTED;
    }
    return hipGetLastError() == hipSuccess ? TN_OK : TN_ERR_HIP;
}

int plan_value(const tn::Plan& p, int32_t what, int64_t* value) {
    switch (what) {
        case TN_QUERY_PARAM_COUNT: *value = p.params; return TN_OK;
        case TN_QUERY_FLOPS_PER_TOKEN: *value = p.flops; return TN_OK;
        case TN_QUERY_NUM_STEPS: *value = int64_t(p.steps.size()); return TN_OK;
        case TN_QUERY_MAX_INTERMEDIATE: *value = p.max_intermediate; return TN_OK;
        case TN_QUERY_OUT_FEATURES: *value = p.M; return TN_OK;
        case TN_QUERY_IN_FEATURES: *value = p.N; return TN_OK;
        default: break;
    }
    if (what >= TN_QUERY_STEP_BASE) {
        int s = (what - TN_QUERY_STEP_BASE) / 10, f = (what - TN_QUERY_STEP_BASE) % 10;
        if (s >= int(p.steps.size())) return TN_ERR_INVALID_ARG;
        const tn::Step& st = p.steps[size_t(s)];
        switch (f) {
            case 0: *value = st.R; return TN_OK;
            case 1: *value = st.K; return TN_OK;
            case 2: *value = st.C; return TN_OK;
            case 3: *value = st.flops; return TN_OK;
            case 4: *value = st.slot; return TN_OK;
            default: return TN_ERR_INVALID_ARG;
        }
    }
    return TN_ERR_INVALID_ARG;
}

}  // namespace

extern "C" {

int tn_linear_version(void) { return 1; }

const char* tn_linear_strerror(int status) {
    switch (status) {
        case TN_OK: return "success";
        case TN_ERR_INVALID_ARG: return "invalid argument";
        case TN_ERR_UNSUPPORTED: return "unsupported configuration";
        case TN_ERR_ALLOC: return "allocation failed";
        case TN_ERR_HIP: return "HIP runtime error";
        default: return "unknown status";
    }
}

int tn_linear_plan_query(const tn_linear_desc* desc, int32_t what, int64_t* value) {
    if (!desc || !value) return TN_ERR_INVALID_ARG;
    tn::Plan p;
    int rc = tn::make_plan(desc, &p);
    if (rc != TN_OK) return rc;
    if (what == TN_QUERY_WORKSPACE_BYTES || what == TN_QUERY_CHUNK_TOKENS) {
        *value = 0;
        return TN_OK;
    }
    if (what == TN_QUERY_PACKED_BYTES) {
        int64_t elt = desc->dtype == TN_DTYPE_BF16 ? 2 : 4, total = 0;
        for (const auto& s : p.steps)
            total += int64_t(round_up(int(s.K), 64)) * round_up(int(s.C), 32) * elt;
        *value = total;   // lower bound: the tile width used for padding is chosen at create
        return TN_OK;
    }
    if (what >= TN_QUERY_STEP_BASE && (what - TN_QUERY_STEP_BASE) % 10 == 5) {
        *value = 0;
        return TN_OK;
    }
    return plan_value(p, what, value);
}

int tn_linear_create(tn_linear_t* out, const tn_linear_desc* desc) {
    if (!out || !desc || !desc->tensors) return TN_ERR_INVALID_ARG;
    tn_linear_s* h = new (std::nothrow) tn_linear_s;
    if (!h) return TN_ERR_ALLOC;
    int rc = tn::make_plan(desc, &h->plan);
    if (rc != TN_OK) {
        delete h;
        return rc;
    }
    for (int i = 0; i < desc->n_tensors; ++i)
        if (!desc->tensors[i]) {
            delete h;
            return TN_ERR_INVALID_ARG;
        }
    if (hipGetDevice(&h->device) != hipSuccess) {
        delete h;
        return TN_ERR_HIP;
    }
    {
        hipDeviceProp_t prop;
        if (hipGetDeviceProperties(&prop, h->device) != hipSuccess) {
            delete h;
            return TN_ERR_HIP;
        }
        if (strncmp(prop.gcnArchName, "gfx950", 6) != 0) {
            delete h;
            return TN_ERR_UNSUPPORTED;
        }
    }
    hipStream_t st = static_cast<hipStream_t>(desc->stream);
    h->elt = desc->dtype == TN_DTYPE_BF16 ? 2 : 4;
    h->max_tokens = desc->max_tokens;
    h->steps.resize(h->plan.steps.size());
    for (size_t i = 0; i < h->steps.size(); ++i) {
        DevStep& s = h->steps[i];
        s.plan = h->plan.steps[i];
        choose_variant(h, &s, desc->flags);
        const tn::Step& p = s.plan;
        // offset tables
        size_t n_tab = p.arow.size() + p.acol.size() + p.crow.size() + p.ccol.size();
        std::vector<int32_t> host_tab;
        host_tab.reserve(n_tab);
        host_tab.insert(host_tab.end(), p.arow.begin(), p.arow.end());
        host_tab.insert(host_tab.end(), p.acol.begin(), p.acol.end());
        host_tab.insert(host_tab.end(), p.crow.begin(), p.crow.end());
        host_tab.insert(host_tab.end(), p.ccol.begin(), p.ccol.end());
        if (hipMalloc(reinterpret_cast<void**>(&s.tables), n_tab * sizeof(int32_t)) != hipSuccess) {
            free_handle(h);
            return TN_ERR_ALLOC;
        }
        // pageable source: the copy is staged before the call returns, so host_tab may go away
        if (hipMemcpyAsync(s.tables, host_tab.data(), n_tab * sizeof(int32_t), hipMemcpyHostToDevice, st) !=
            hipSuccess) {
            free_handle(h);
            return TN_ERR_HIP;
        }
        if (hipStreamSynchronize(st) != hipSuccess) {
            free_handle(h);
            return TN_ERR_HIP;
        }
        const int32_t* t = s.tables;
        if (!p.a_plain) {
            s.arow = t;
            s.acol = t + p.arow.size();
        }
        s.crow = t + p.arow.size() + p.acol.size();
        s.ccol = s.crow + p.crow.size();
        // packed parameter tensor
        int64_t bytes = int64_t(s.Cp) * s.Kp * h->elt;
        if (hipMalloc(&s.packed, size_t(bytes)) != hipSuccess) {
            free_handle(h);
            return TN_ERR_ALLOC;
        }
        h->packed_bytes += bytes;
        PackArgs pa;
        memset(&pa, 0, sizeof(pa));
        pa.src = desc->tensors[p.slot];
        pa.dst = s.packed;
        pa.K = int32_t(p.K);
        pa.Kp = s.Kp;
        pa.C = int32_t(p.C);
        pa.Cp = s.Cp;
        pa.nk = int32_t(p.kdims.size());
        pa.nc = int32_t(p.cdims.size());
        for (int j = 0; j < pa.nk; ++j) {
            pa.kext[j] = p.kdims[size_t(j)].extent;
            pa.kstr[j] = p.kdims[size_t(j)].stride;
        }
        for (int j = 0; j < pa.nc; ++j) {
            pa.cext[j] = p.cdims[size_t(j)].extent;
            pa.cstr[j] = p.cdims[size_t(j)].stride;
        }
        pa.trace_extent = p.trace_extent;
        pa.trace_stride = p.trace_stride;
        int64_t total = int64_t(s.Cp) * s.Kp;
        uint32_t blocks = uint32_t(std::min<int64_t>((total + 255) / 256, 65535));
        if (h->elt == 2)
            hipLaunchKernelGGL(pack_kernel<bf16_t>, dim3(blocks), dim3(256), 0, st, pa);
        else
            hipLaunchKernelGGL(pack_kernel<float>, dim3(blocks), dim3(256), 0, st, pa);
        if (hipGetLastError() != hipSuccess) {
            free_handle(h);
            return TN_ERR_HIP;
        }
    }
    // workspace: two ping-pong buffers, each chunk_tokens * max_intermediate elements
    int64_t per_token = h->plan.max_intermediate * h->elt;
    int64_t limit = desc->workspace_limit_bytes > 0 ? desc->workspace_limit_bytes : kDefaultWorkspaceBytes;
    int64_t chunk = h->max_tokens;
    if (per_token > 0) {
        chunk = std::max<int64_t>(1, std::min<int64_t>(h->max_tokens, limit / (2 * per_token)));
        // rows of a pass are indexed with 32 bits
        int64_t max_r = 1;
        for (const auto& s : h->steps) max_r = std::max(max_r, s.plan.R);
        chunk = std::max<int64_t>(1, std::min<int64_t>(chunk, ((int64_t(1) << 31) - 1024) / max_r));
        for (int b = 0; b < 2; ++b) {
            if (hipMalloc(&h->ws[b], size_t(chunk * per_token)) != hipSuccess) {
                free_handle(h);
                return TN_ERR_ALLOC;
            }
        }
        h->workspace_bytes = 2 * chunk * per_token;
    } else {
        int64_t max_r = 1;
        for (const auto& s : h->steps) max_r = std::max(max_r, s.plan.R);
        chunk = std::max<int64_t>(1, std::min<int64_t>(chunk, ((int64_t(1) << 31) - 1024) / max_r));
    }
    h->chunk_tokens = chunk;
    *out = h;
    return TN_OK;
}

int tn_linear_forward(tn_linear_t h, const void* x, void* y, int64_t tokens, void* stream) {
    if (!h || tokens < 0) return TN_ERR_INVALID_ARG;
    if (tokens == 0) return TN_OK;
    if (!x || !y) return TN_ERR_INVALID_ARG;
    hipStream_t st = static_cast<hipStream_t>(stream);
    const char* xb = static_cast<const char*>(x);
    char* yb = static_cast<char*>(y);
    size_t ns = h->steps.size();
    for (int64_t t0 = 0; t0 < tokens; t0 += h->chunk_tokens) {
        int64_t nt = std::min(h->chunk_tokens, tokens - t0);
        for (size_t s = 0; s < ns; ++s) {
            const void* A = (s == 0) ? static_cast<const void*>(xb + t0 * h->plan.N * h->elt) : h->ws[(s - 1) & 1];
            void* Out = (s == ns - 1) ? static_cast<void*>(yb + t0 * h->plan.M * h->elt) : h->ws[s & 1];
            tn_linear_s::ProfRec rec{int(s), nullptr, nullptr};
            if (h->profiling) {
                if (hipEventCreate(&rec.start) != hipSuccess || hipEventCreate(&rec.stop) != hipSuccess)
                    return TN_ERR_HIP;
                (void)hipEventRecord(rec.start, st);
            }
            int rc = launch_step(h, h->steps[s], A, Out, nt, st);
            if (h->profiling) {
                (void)hipEventRecord(rec.stop, st);
                h->prof.push_back(rec);
            }
            if (rc != TN_OK) return rc;
        }
    }
    return TN_OK;
}

int tn_linear_profile(tn_linear_t h, int32_t enable) {
    if (!h) return TN_ERR_INVALID_ARG;
    if (enable) clear_profile(h);
    h->profiling = enable != 0;
    return TN_OK;
}

int tn_linear_profile_read(tn_linear_t h, int32_t step, double* total_ms, int64_t* launches) {
    if (!h || !total_ms || !launches || step < 0 || step >= int(h->steps.size())) return TN_ERR_INVALID_ARG;
    double ms = 0;
    int64_t n = 0;
    for (auto& r : h->prof) {
        if (r.step != step) continue;
        if (hipEventSynchronize(r.stop) != hipSuccess) return TN_ERR_HIP;
        float e = 0;
        if (hipEventElapsedTime(&e, r.start, r.stop) != hipSuccess) return TN_ERR_HIP;
        ms += e;
        ++n;
    }
    *total_ms = ms;
    *launches = n;
    return TN_OK;
}

int tn_linear_destroy(tn_linear_t h) {
    free_handle(h);
    return TN_OK;
}

int tn_linear_query(tn_linear_t h, int32_t what, int64_t* value) {
    if (!h || !value) return TN_ERR_INVALID_ARG;
    switch (what) {
        case TN_QUERY_PACKED_BYTES: *value = h->packed_bytes; return TN_OK;
        case TN_QUERY_WORKSPACE_BYTES: *value = h->workspace_bytes; return TN_OK;
        case TN_QUERY_CHUNK_TOKENS: *value = h->chunk_tokens; return TN_OK;
        default: break;
    }
    if (what >= TN_QUERY_STEP_BASE && (what - TN_QUERY_STEP_BASE) % 10 == 5) {
        int s = (what - TN_QUERY_STEP_BASE) / 10;
        if (s >= int(h->steps.size())) return TN_ERR_INVALID_ARG;
        *value = h->steps[size_t(s)].variant;
        return TN_OK;
    }
    return plan_value(h->plan, what, value);
}

}  // extern "C"
