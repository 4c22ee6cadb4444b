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
#include <type_traits>
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
            if (c < a.Cp && k < a.Kp) w = to_float(B[bfrag_offset(c, k, a.Kp >> 4)]);
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
            bf16x8 v = *reinterpret_cast<const bf16x8*>(B + bfrag_offset(col0 + cc, k0 + kc, a.Kp >> 4));
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
// Pipelined bf16 MFMA step kernel for the FLOP-heavy steps (wide C, plain A with K % 8 == 0 or
// gathered A). Differences from the kernel above:
//   * the next K tile is fetched from global memory into registers while the current one is
//     multiplied (and, with STAGES == 2, written to the other LDS buffer: one barrier per tile);
//   * the MFMA operands are swapped (packed tensor first), so a lane ends up with 4 consecutive
//     columns of one row and the epilogue writes 8-byte pieces to LDS;
//   * tiles are numbered so that the column tiles of one row tile run back to back on the same
//     XCD (workgroup i goes to XCD i % 8): the second read of an A tile hits that XCD's L2;
//   * per-row output offsets are computed once per tile and kept in LDS;
//   * TRANS = 1 serves outputs whose contiguous direction is along rows (CMODE 2): the operands
//     are not swapped, a lane holds 4 consecutive rows of one column, and the tile is staged in LDS
//     column-major so that the stores again move 16 contiguous bytes per lane.
// ---------------------------------------------------------------------------------------------
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));

// Workgroup -> output tile, XCD-aware. Workgroup i runs on XCD i % 8 (round-robin dispatch) and an
// XCD runs about 32 of these workgroups at a time, all reading through its own 4 MB L2. XCD x owns the
// row tiles x, x+8, x+16, ...; its workgroups walk them in bands of 4 row tiles, row fastest, so
// that the 32 tiles in flight are 4 row tiles x 8 column tiles: 4 + 8 operand panels move through the
// L2 at a time instead of 1 + 32 (a band of one row tile per XCD streams the whole packed tensor
// from the fabric once per row tile, which bounded the large-K launches).
__device__ __forceinline__ void tile_of_workgroup(int id, int nrow_tiles, int ncol_tiles, int* row_tile, int* col_tile) {
    constexpr int BAND = 4;
    const int xcd = id & 7, slot = id >> 3;
    const int rows_per_xcd = (nrow_tiles + 7) >> 3;                  // the grid is padded to whole XCD rows
    const int band = slot / (BAND * ncol_tiles);
    const int in_band = slot - band * (BAND * ncol_tiles);
    const int band_rows = min(BAND, rows_per_xcd - band * BAND);
    const int col = in_band / band_rows;
    const int r = in_band - col * band_rows;
    *row_tile = (band * BAND + r) * 8 + xcd;
    *col_tile = col;
}


template <int WM, int WN, int TM, int TN, int AMODE, int STAGES, int MINB, int TRANS>
__global__ void __launch_bounds__(WM * WN * 64, MINB)
step_mfma_pipe_kernel(StepArgs a, int cmode, int nrow_tiles, int ncol_tiles) {
    constexpr int BM = WM * TM * 32, BN = WN * TN * 32, BK = 64;
    constexpr int LDK = BK + 8;
    constexpr int A_ELEMS = BM * LDK, B_ELEMS = BN * LDK, STAGE_ELEMS = A_ELEMS + B_ELEMS;
    constexpr int LDC = BN + 8;
    constexpr int NT = WM * WN * 64;                 // threads per workgroup
    constexpr int RPP = NT / 8;                       // tile rows covered by one pass of 16-byte loads
    constexpr int A_CHUNKS = BM / RPP, B_CHUNKS = BN / RPP;
    extern __shared__ __attribute__((aligned(16))) unsigned char dyn_smem[];
    bf16_t* smem = reinterpret_cast<bf16_t*>(dyn_smem);

    int row_tile, col_tile;
    tile_of_workgroup(blockIdx.x, nrow_tiles, ncol_tiles, &row_tile, &col_tile);
    if (row_tile >= nrow_tiles) return;
    const uint32_t row0 = uint32_t(row_tile) * BM;
    const int col0 = col_tile * BN;

    const bf16_t* A = static_cast<const bf16_t*>(a.A);
    const bf16_t* B = static_cast<const bf16_t*>(a.B);
    bf16_t* Out = static_cast<bf16_t*>(a.Out);
    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int wm = wave / WN, wn = wave % WN;
    const int lrow = tid >> 3, lkc = (tid & 7) * 8;      // this thread's row (mod 32) and k offset in a tile

    // A addressing: AMODE 0 -> one pointer, rows 32*j apart; AMODE 1 -> per-row element offsets
    const bf16_t* a_ptr = A + int64_t(row0 + lrow) * a.K + lkc;
    int64_t a_base[AMODE == 1 ? A_CHUNKS : 1];
    if (AMODE == 1) {
#pragma unroll
        for (int j = 0; j < A_CHUNKS; ++j) {
            uint32_t g = row0 + lrow + RPP * j;
            a_base[j] = -1;
            if (g < a.total_rows) {
                uint32_t t = g / a.R;
                uint32_t r = g - t * a.R;
                a_base[j] = int64_t(t) * a.a_tok_stride + (a.arow ? int64_t(a.arow[r]) : int64_t(r) * a.K);
            }
        }
    }
    // B: chunk e = tid + NT*j of a K tile is lane e%64 of block e/64; block b = (column block b/4,
    // k-step b%4): every wave reads whole 1 KB blocks
    const int nks = a.Kp >> 4;
    const bf16_t* b_ptr = B + (int64_t(col0 >> 5) * nks) * 512 + (tid & 63) * 8;

    bf16x8 ra[A_CHUNKS], rb[B_CHUNKS];
    auto load_tile = [&](int k0) {
#pragma unroll
        for (int j = 0; j < A_CHUNKS; ++j) {
            bf16x8 v;
#pragma unroll
            for (int q = 0; q < 8; ++q) v[q] = bf16_t(0.f);
            int k = k0 + lkc;
            if (AMODE == 0) {
                if (row0 + lrow + RPP * j < a.total_rows && k < a.K)
                    v = *reinterpret_cast<const bf16x8*>(a_ptr + int64_t(RPP * j) * a.K + k0);
            } else if (a_base[j] >= 0) {
#pragma unroll
                for (int q = 0; q < 8; ++q)
                    if (k + q < a.K) v[q] = A[a_base[j] + (a.acol ? a.acol[k + q] : k + q)];
            }
            ra[j] = v;
        }
#pragma unroll
        for (int j = 0; j < B_CHUNKS; ++j)
        {
            int blk = (tid >> 6) + (NT / 64) * j;
            rb[j] = *reinterpret_cast<const bf16x8*>(b_ptr + (int64_t(blk >> 2) * nks + (k0 >> 4) + (blk & 3)) * 512);
        }
    };
    auto store_tile = [&](int stage) {
        bf16_t* sA = smem + stage * STAGE_ELEMS;
        bf16_t* sB = sA + A_ELEMS;
#pragma unroll
        for (int j = 0; j < A_CHUNKS; ++j)
            *reinterpret_cast<bf16x8*>(sA + (lrow + RPP * j) * LDK + lkc) = ra[j];
#pragma unroll
        for (int j = 0; j < B_CHUNKS; ++j) {
            int blk = (tid >> 6) + (NT / 64) * j;
            int col = (blk >> 2) * 32 + (lane & 31), kc = (blk & 3) * 16 + 8 * (lane >> 5);
            *reinterpret_cast<bf16x8*>(sB + col * LDK + kc) = rb[j];
        }
    };

    floatx16 acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;

    const int nk = a.Kp / BK;
    load_tile(0);
    store_tile(0);
    __syncthreads();
    for (int kt = 0; kt < nk; ++kt) {
        const int cur = (STAGES == 2) ? (kt & 1) : 0;
        if (kt + 1 < nk) load_tile((kt + 1) * BK);
        const bf16_t* sA = smem + cur * STAGE_ELEMS + ((wm * TM) * 32 + (lane & 31)) * LDK + 8 * (lane >> 5);
        const bf16_t* sB = smem + cur * STAGE_ELEMS + A_ELEMS + ((wn * TN) * 32 + (lane & 31)) * LDK + 8 * (lane >> 5);
#pragma unroll
        for (int ks = 0; ks < BK; ks += 16) {
            bf16x8 af[TM], bfr[TN];
#pragma unroll
            for (int i = 0; i < TM; ++i) af[i] = *reinterpret_cast<const bf16x8*>(sA + i * 32 * LDK + ks);
#pragma unroll
            for (int j = 0; j < TN; ++j) bfr[j] = *reinterpret_cast<const bf16x8*>(sB + j * 32 * LDK + ks);
#pragma unroll
            for (int i = 0; i < TM; ++i)
#pragma unroll
                for (int j = 0; j < TN; ++j)
                    acc[i][j] = TRANS ? __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[i], bfr[j], acc[i][j], 0, 0, 0)
                                      : __builtin_amdgcn_mfma_f32_32x32x16_bf16(bfr[j], af[i], acc[i][j], 0, 0, 0);
        }
        if (STAGES == 1) __syncthreads();
        if (kt + 1 < nk) store_tile((STAGES == 2) ? (cur ^ 1) : 0);
        __syncthreads();
    }

    // ---- epilogue. Operands swapped (TRANS = 0): lane l, register v of a tile holds
    //      row = l%32, col = 8*(v/4) + 4*(l/32) + v%4; staged row-major [BM][LDC].
    //      Not swapped (TRANS = 1): col = l%32, row = 8*(v/4) + 4*(l/32) + v%4; staged
    //      column-major [BN][LDR].
    constexpr int LDR = BM + 8;
    constexpr size_t C_ELEMS = size_t(BM) * LDC > size_t(BN) * LDR ? size_t(BM) * LDC : size_t(BN) * LDR;
    bf16_t* sC = smem;
    int64_t* sBase = reinterpret_cast<int64_t*>(dyn_smem + C_ELEMS * sizeof(bf16_t));
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                bf16x4 pk;
#pragma unroll
                for (int u = 0; u < 4; ++u) pk[u] = bf16_t(acc[i][j][4 * q + u]);
                if (TRANS) {
                    int cc = (wn * TN + j) * 32 + (lane & 31);
                    int rr = (wm * TM + i) * 32 + 8 * q + 4 * (lane >> 5);
                    *reinterpret_cast<bf16x4*>(sC + cc * LDR + rr) = pk;
                } else {
                    int rr = (wm * TM + i) * 32 + (lane & 31);
                    int cc = (wn * TN + j) * 32 + 8 * q + 4 * (lane >> 5);
                    *reinterpret_cast<bf16x4*>(sC + rr * LDC + cc) = pk;
                }
            }
    for (int rr = tid; rr < BM; rr += NT) {
        uint32_t g = row0 + rr;
        int64_t base = -1;
        if (g < a.total_rows) {
            uint32_t t = g / a.R;
            uint32_t r = g - t * a.R;
            base = int64_t(t) * a.c_tok_stride + a.crow[r];
        }
        sBase[rr] = base;
    }
    __syncthreads();

    constexpr int GROUPS = BM * BN / 8;
    if (TRANS) {
        // rows come in aligned contiguous runs of 8: thread -> (group of 8 rows, column), rows fastest
#pragma unroll 4
        for (int e = tid; e < GROUPS; e += NT) {
            int rg = (e % (BM / 8)) * 8, cc = e / (BM / 8);
            int c = col0 + cc;
            int64_t base = sBase[rg];
            if (base < 0 || c >= a.C) continue;
            *reinterpret_cast<bf16x8*>(Out + base + a.ccol[c]) = *reinterpret_cast<const bf16x8*>(sC + cc * LDR + rg);
        }
    } else if (cmode == 1) {
#pragma unroll 4
        for (int e = tid; e < GROUPS; e += NT) {
            int rr = e / (BN / 8), cg = (e % (BN / 8)) * 8;
            int c = col0 + cg;
            int64_t base = sBase[rr];
            if (base < 0 || c >= a.C) continue;
            *reinterpret_cast<bf16x8*>(Out + base + a.ccol[c]) = *reinterpret_cast<const bf16x8*>(sC + rr * LDC + cg);
        }
    } else {
        for (int e = tid; e < BM * BN; e += NT) {
            int rr = e / BN, cc = e % BN;
            int c = col0 + cc;
            int64_t base = sBase[rr];
            if (base < 0 || c >= a.C) continue;
            Out[base + a.ccol[c]] = sC[rr * LDC + cc];
        }
    }
}

// ---------------------------------------------------------------------------------------------
// Direct-to-LDS bf16 MFMA step kernel (the fastest tiled kernel; needs a plain A with K % 32 == 0).
//   * K tiles of 32 travel from global memory straight into LDS with global_load_lds_dwordx4
//     (16 bytes per lane, no staging registers, no LDS write instructions) into a ring of NS
//     stages; a wave waits on its own loads with s_waitcnt vmcnt(n) and a workgroup barrier makes
//     the other waves' loads visible;
//   * tile kt+1 is known to have landed before tile kt is multiplied, and the MFMA operand
//     fragments are double-buffered in registers, so the LDS reads of the next k-step are in
//     flight while the current MFMAs run, across the barrier as well;
//   * an LDS tile row is 64 bytes (4 chunks of 16 B); chunk c of row r sits at chunk position
//     c ^ ((r >> 2) & 3), which makes the fragment reads of 16 consecutive rows conflict-free. The
//     swizzle costs nothing: each lane simply fetches the global chunk that belongs at its LDS slot.
// Tile numbering (XCD-aware), epilogue (CMODE 1, TRANS, scalar) and tables are those of the kernel
// above. Rows past the end are clamped to the last row when loading and masked when storing.
// ---------------------------------------------------------------------------------------------
template <int N> __device__ __forceinline__ void wait_vmcnt() {
    // s_waitcnt immediate on gfx9: vmcnt[3:0] | expcnt[6:4] | lgkmcnt[11:8] | vmcnt[5:4] at [15:14]
    constexpr int imm = (N & 0xF) | (0x7 << 4) | (0xF << 8) | ((N >> 4) << 14);
    __builtin_amdgcn_s_waitcnt(imm);
}

template <int WM, int WN, int TM, int TN, int NS, int MINB, int TRANS>
__global__ void __launch_bounds__(WM * WN * 64, MINB)
step_mfma_dlds_kernel(StepArgs a, int cmode, int nrow_tiles, int ncol_tiles) {
    constexpr int NT = WM * WN * 64, NWAVE = WM * WN;
    constexpr int BM = WM * TM * 32, BN = WN * TN * 32, BK = 32;
    constexpr int ROWB = BK * 2;                       // bytes per LDS tile row
    constexpr int A_BYTES = BM * ROWB, STAGE_BYTES = (BM + BN) * ROWB;
    constexpr int A_PER_WAVE = BM / 16 / NWAVE, B_PER_WAVE = BN / 16 / NWAVE;   // 1 KB loads per wave and stage
    constexpr int L = A_PER_WAVE + B_PER_WAVE;
    constexpr int LDC = BN + 8, LDR = BM + 8;
    static_assert((BM / 16) % NWAVE == 0 && (BN / 16) % NWAVE == 0, "16-row blocks per wave");
    static_assert(NS >= 3 && NS <= 4 && 2 * L <= 63, "ring depth / vmcnt range");
    extern __shared__ __attribute__((aligned(16))) unsigned char dyn_smem[];

    int row_tile, col_tile;
    tile_of_workgroup(blockIdx.x, nrow_tiles, ncol_tiles, &row_tile, &col_tile);
    if (row_tile >= nrow_tiles) return;
    const uint32_t row0 = uint32_t(row_tile) * BM;
    const int col0 = col_tile * BN;

    const bf16_t* A = static_cast<const bf16_t*>(a.A);
    const bf16_t* B = static_cast<const bf16_t*>(a.B);
    bf16_t* Out = static_cast<bf16_t*>(a.Out);
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm = wave / WN, wn = wave % WN;
    const int nks = a.Kp >> 4;

    // per-lane sources: lane l of a 1 KB load fills LDS row l/4, chunk position l%4 of its block
    const int lr = lane >> 2, lpc = lane & 3;
    const bf16_t* a_src[A_PER_WAVE];
    const bf16_t* b_src[B_PER_WAVE];
#pragma unroll
    for (int j = 0; j < A_PER_WAVE; ++j) {
        int r = (j * NWAVE + wave) * 16 + lr;
        int c = lpc ^ ((r >> 2) & 3);
        uint32_t g = row0 + r;
        if (g >= a.total_rows) g = a.total_rows - 1;
        a_src[j] = A + int64_t(g) * a.K + c * 8;
    }
#pragma unroll
    for (int j = 0; j < B_PER_WAVE; ++j) {
        int r = (j * NWAVE + wave) * 16 + lr;              // column within the tile
        int c = lpc ^ ((r >> 2) & 3);                       // logical chunk: k = kt*32 + c*8
        int col = col0 + r;
        // fragment-major: block (col/32, k/16), chunk (col%32) + 32*((k/8)%2)
        b_src[j] = B + (int64_t(col >> 5) * nks + (c >> 1)) * 512 + ((col & 31) + 32 * (c & 1)) * 8;
    }
    auto issue = [&](int kt, int stage) {
        unsigned char* sbase = dyn_smem + stage * STAGE_BYTES;
#pragma unroll
        for (int j = 0; j < A_PER_WAVE; ++j)
            __builtin_amdgcn_global_load_lds(
                (const void __attribute__((address_space(1)))*)(a_src[j] + kt * BK),
                (void __attribute__((address_space(3)))*)(sbase + (j * NWAVE + wave) * 1024), 16, 0, 0);
#pragma unroll
        for (int j = 0; j < B_PER_WAVE; ++j)
            __builtin_amdgcn_global_load_lds(
                (const void __attribute__((address_space(1)))*)(b_src[j] + int64_t(kt) * 2 * 512),
                (void __attribute__((address_space(3)))*)(sbase + A_BYTES + (j * NWAVE + wave) * 1024), 16, 0, 0);
    };
    auto wait_outstanding_tiles = [&](int n) {            // n is wave-uniform, at most NS - 2
        if (n <= 0) wait_vmcnt<0>();
        else if (n == 1) wait_vmcnt<L>();
        else if (n == 2 || NS <= 4) wait_vmcnt<2 * L>();
        else wait_vmcnt<3 * L>();
    };

    floatx16 acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;

    // fragment read offsets: lane reads row lane%32, logical chunk ks*2 + lane/32
    int a_off[TM][2], b_off[TN][2];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int ks = 0; ks < 2; ++ks) {
            int r = (wm * TM + i) * 32 + (lane & 31);
            a_off[i][ks] = r * ROWB + (((ks * 2 + (lane >> 5)) ^ ((r >> 2) & 3)) * 16);
        }
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
        for (int ks = 0; ks < 2; ++ks) {
            int r = (wn * TN + j) * 32 + (lane & 31);
            b_off[j][ks] = A_BYTES + r * ROWB + (((ks * 2 + (lane >> 5)) ^ ((r >> 2) & 3)) * 16);
        }

    const int nk = a.Kp / BK;                            // K % 32 == 0, so tiles past K are all padding
    const int nk_real = a.K / BK;                        // only these hold data; B is zero beyond
    int issued = 0;
    for (; issued < NS - 1 && issued < nk_real; ++issued) issue(issued, issued);
    wait_outstanding_tiles(min(issued - 1, NS - 2));     // tile 0 has landed
    __syncthreads();
    bf16x8 af[2][TM], bfr[2][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i) af[0][i] = *reinterpret_cast<const bf16x8*>(dyn_smem + a_off[i][0]);
#pragma unroll
    for (int j = 0; j < TN; ++j) bfr[0][j] = *reinterpret_cast<const bf16x8*>(dyn_smem + b_off[j][0]);
    (void)nk;

    for (int kt = 0; kt < nk_real; ++kt) {
        if (kt + 1 < nk_real) wait_outstanding_tiles(issued - (kt + 2));   // tile kt+1 has landed
        __syncthreads();       // everyone is done with tile kt-1: its stage may be refilled
        if (issued < nk_real) {
            issue(issued, issued % NS);
            ++issued;
        }
        const unsigned char* scur = dyn_smem + (kt % NS) * STAGE_BYTES;
        const unsigned char* snxt = dyn_smem + ((kt + 1) % NS) * STAGE_BYTES;
#pragma unroll
        for (int ks = 0; ks < 2; ++ks) {
            const int cb = ks & 1, nb = cb ^ 1;
            if (ks == 0) {
#pragma unroll
                for (int i = 0; i < TM; ++i) af[nb][i] = *reinterpret_cast<const bf16x8*>(scur + a_off[i][1]);
#pragma unroll
                for (int j = 0; j < TN; ++j) bfr[nb][j] = *reinterpret_cast<const bf16x8*>(scur + b_off[j][1]);
            } else if (kt + 1 < nk_real) {
#pragma unroll
                for (int i = 0; i < TM; ++i) af[nb][i] = *reinterpret_cast<const bf16x8*>(snxt + a_off[i][0]);
#pragma unroll
                for (int j = 0; j < TN; ++j) bfr[nb][j] = *reinterpret_cast<const bf16x8*>(snxt + b_off[j][0]);
            }
#pragma unroll
            for (int i = 0; i < TM; ++i)
#pragma unroll
                for (int j = 0; j < TN; ++j)
                    acc[i][j] = TRANS ? __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[cb][i], bfr[cb][j], acc[i][j], 0, 0, 0)
                                      : __builtin_amdgcn_mfma_f32_32x32x16_bf16(bfr[cb][j], af[cb][i], acc[i][j], 0, 0, 0);
        }
    }
    __syncthreads();

    // ---- epilogue (see step_mfma_pipe_kernel)
    constexpr size_t C_ELEMS = size_t(BM) * LDC > size_t(BN) * LDR ? size_t(BM) * LDC : size_t(BN) * LDR;
    bf16_t* sC = reinterpret_cast<bf16_t*>(dyn_smem);
    int64_t* sBase = reinterpret_cast<int64_t*>(dyn_smem + C_ELEMS * sizeof(bf16_t));
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                bf16x4 pk;
#pragma unroll
                for (int u = 0; u < 4; ++u) pk[u] = bf16_t(acc[i][j][4 * q + u]);
                if (TRANS) {
                    int cc = (wn * TN + j) * 32 + (lane & 31);
                    int rr = (wm * TM + i) * 32 + 8 * q + 4 * (lane >> 5);
                    *reinterpret_cast<bf16x4*>(sC + cc * LDR + rr) = pk;
                } else {
                    int rr = (wm * TM + i) * 32 + (lane & 31);
                    int cc = (wn * TN + j) * 32 + 8 * q + 4 * (lane >> 5);
                    *reinterpret_cast<bf16x4*>(sC + rr * LDC + cc) = pk;
                }
            }
    for (int rr = tid; rr < BM; rr += NT) {
        uint32_t g = row0 + rr;
        int64_t base = -1;
        if (g < a.total_rows) {
            uint32_t t = g / a.R;
            uint32_t r = g - t * a.R;
            base = int64_t(t) * a.c_tok_stride + a.crow[r];
        }
        sBase[rr] = base;
    }
    __syncthreads();
    constexpr int GROUPS = BM * BN / 8;
    if (TRANS) {
#pragma unroll 4
        for (int e = tid; e < GROUPS; e += NT) {
            int rg = (e % (BM / 8)) * 8, cc = e / (BM / 8);
            int c = col0 + cc;
            int64_t base = sBase[rg];
            if (base < 0 || c >= a.C) continue;
            *reinterpret_cast<bf16x8*>(Out + base + a.ccol[c]) = *reinterpret_cast<const bf16x8*>(sC + cc * LDR + rg);
        }
    } else if (cmode == 1) {
#pragma unroll 4
        for (int e = tid; e < GROUPS; e += NT) {
            int rr = e / (BN / 8), cg = (e % (BN / 8)) * 8;
            int c = col0 + cg;
            int64_t base = sBase[rr];
            if (base < 0 || c >= a.C) continue;
            *reinterpret_cast<bf16x8*>(Out + base + a.ccol[c]) = *reinterpret_cast<const bf16x8*>(sC + rr * LDC + cg);
        }
    } else {
        for (int e = tid; e < BM * BN; e += NT) {
            int rr = e / BN, cc = e % BN;
            int c = col0 + cc;
            int64_t base = sBase[rr];
            if (base < 0 || c >= a.C) continue;
            Out[base + a.ccol[c]] = sC[rr * LDC + cc];
        }
    }
}

template <int WM, int WN, int TM, int TN, int NS>
constexpr size_t dlds_smem_bytes() {
    constexpr int BM = WM * TM * 32, BN = WN * TN * 32;
    constexpr size_t stage = size_t(BM + BN) * 64 * NS;
    constexpr size_t c_elems = size_t(BM) * (BN + 8) > size_t(BN) * (BM + 8) ? size_t(BM) * (BN + 8) : size_t(BN) * (BM + 8);
    constexpr size_t epi = c_elems * 2 + size_t(BM) * 8;
    return stage > epi ? stage : epi;
}

template <int WM, int WN, int TM, int TN, int STAGES>
constexpr size_t pipe_smem_bytes() {
    constexpr int BM = WM * TM * 32, BN = WN * TN * 32;
    constexpr size_t stage = size_t(BM + BN) * (64 + 8) * 2 * STAGES;
    constexpr size_t c_elems = size_t(BM) * (BN + 8) > size_t(BN) * (BM + 8) ? size_t(BM) * (BN + 8) : size_t(BN) * (BM + 8);
    constexpr size_t epi = c_elems * 2 + size_t(BM) * 8;
    return stage > epi ? stage : epi;
}

// ---------------------------------------------------------------------------------------------
// Short-K kernel (K <= 64): steps such as the first contraction of a chain read little and write
// a lot, so they are bound by the store stream. A workgroup owns 128 rows and walks over all
// columns, 128 at a time. The A fragments of its rows (the whole K) stay in registers for the whole
// walk; the packed tensor's fragment blocks are loaded from memory straight into MFMA operand
// registers (double-buffered across column iterations); each wave turns its 64x64 result into
// row-contiguous 16-byte pieces through a private LDS patch and stores it. No workgroup barrier
// is used anywhere, so the stores of one wave overlap the loads and MFMAs of the others.
// Requires Kp == 64, aligned runs of 8 columns in the output (CMODE 1) and Cp % 128 == 0.
// ---------------------------------------------------------------------------------------------
template <int AMODE, int TMW, int DBUF, int MINB>
__global__ void __launch_bounds__(256, MINB) step_shortk_kernel(StepArgs a) {
    // TMW = 32-row tiles per wave (1 or 2): the workgroup covers 4 * TMW * 32 / 2 ... rows, see below
    constexpr int LDP = 64 + 8;                          // padded row of the wave's LDS patch
    constexpr int WROWS = TMW * 32;                      // rows per wave
    __shared__ __attribute__((aligned(16))) bf16_t patch[4][WROWS * LDP];
    const bf16_t* A = static_cast<const bf16_t*>(a.A);
    const bf16_t* B = static_cast<const bf16_t*>(a.B);
    bf16_t* Out = static_cast<bf16_t*>(a.Out);
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave >> 1, wn = wave & 1;             // 2 x 2 waves: rows wm, 64-column half wn
    const uint32_t row0 = blockIdx.x * (2 * WROWS) + wm * WROWS;
    bf16_t* sP = patch[wave];

    // A fragments for the wave's rows and all 4 k-steps
    bf16x8 af[TMW][4];
#pragma unroll
    for (int i = 0; i < TMW; ++i) {
        uint32_t g = row0 + i * 32 + (lane & 31);
        int64_t base = -1;
        if (g < a.total_rows) {
            uint32_t t = g / a.R;
            uint32_t r = g - t * a.R;
            base = int64_t(t) * a.a_tok_stride + (a.arow ? int64_t(a.arow[r]) : int64_t(r) * a.K);
        }
#pragma unroll
        for (int ks = 0; ks < 4; ++ks) {
            bf16x8 v;
#pragma unroll
            for (int q = 0; q < 8; ++q) v[q] = bf16_t(0.f);
            int k = ks * 16 + 8 * (lane >> 5);
            if (base >= 0) {
                if (AMODE == 0) {
                    if (k < a.K) v = *reinterpret_cast<const bf16x8*>(A + base + k);
                } else {
#pragma unroll
                    for (int q = 0; q < 8; ++q)
                        if (k + q < a.K) v[q] = A[base + (a.acol ? a.acol[k + q] : k + q)];
                }
            }
            af[i][ks] = v;
        }
    }
    // output bases of the rows this lane stores per iteration (row p*8 + lane/8), in units of 8
    // elements (every run of 8 columns is 16-byte aligned), so that they fit 32 bits
    constexpr int NP = WROWS / 8;
    uint32_t obase8[NP];
    bool ovalid[NP];
#pragma unroll
    for (int p = 0; p < NP; ++p) {
        uint32_t g = row0 + p * 8 + (lane >> 3);
        ovalid[p] = g < a.total_rows;
        obase8[p] = 0;
        if (ovalid[p]) {
            uint32_t t = g / a.R;
            uint32_t r = g - t * a.R;
            obase8[p] = uint32_t((int64_t(t) * a.c_tok_stride + a.crow[r]) >> 3);
        }
    }
    const int ncol_iters = a.Cp >> 7;
    const bf16_t* bp = B + lane * 8;                     // Kp == 64: 4 k-step blocks per column block
    auto load_b = [&](int it, bf16x8 (&bf)[2][4]) {
        int cb = it * 4 + wn * 2;
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int ks = 0; ks < 4; ++ks)
                bf[j][ks] = *reinterpret_cast<const bf16x8*>(bp + (int64_t(cb + j) * 4 + ks) * 512);
    };
    // column iterations are dealt round-robin over gridDim.y workgroups (1 when there are enough
    // row tiles to fill the chip)
    const int it_step = gridDim.y;
    bf16x8 bcur[2][4], bnext[2][4];
    if (DBUF && int(blockIdx.y) < ncol_iters) load_b(blockIdx.y, bcur);
    for (int it = blockIdx.y; it < ncol_iters; it += it_step) {
        if (DBUF) {
            if (it + it_step < ncol_iters) load_b(it + it_step, bnext);
        } else {
            load_b(it, bcur);
        }
        floatx16 acc[TMW][2];
#pragma unroll
        for (int i = 0; i < TMW; ++i)
#pragma unroll
            for (int j = 0; j < 2; ++j)
#pragma unroll
                for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;
#pragma unroll
        for (int ks = 0; ks < 4; ++ks)
#pragma unroll
            for (int i = 0; i < TMW; ++i)
#pragma unroll
                for (int j = 0; j < 2; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(bcur[j][ks], af[i][ks], acc[i][j], 0, 0, 0);
        // lane l, register v: row l%32, column 8*(v/4) + 4*(l/32) + v%4
#pragma unroll
        for (int i = 0; i < TMW; ++i)
#pragma unroll
            for (int j = 0; j < 2; ++j)
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    bf16x4 pk;
#pragma unroll
                    for (int u = 0; u < 4; ++u) pk[u] = bf16_t(acc[i][j][4 * q + u]);
                    *reinterpret_cast<bf16x4*>(sP + (i * 32 + (lane & 31)) * LDP + j * 32 + 8 * q + 4 * (lane >> 5)) = pk;
                }
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
        const int c = it * 128 + wn * 64 + (lane & 7) * 8;
        if (c < a.C) {
            const uint32_t coff8 = uint32_t(a.ccol[c]) >> 3;
#pragma unroll
            for (int p = 0; p < NP; ++p) {
                bf16x8 v = *reinterpret_cast<const bf16x8*>(sP + (p * 8 + (lane >> 3)) * LDP + (lane & 7) * 8);
                if (ovalid[p]) *reinterpret_cast<bf16x8*>(Out + (int64_t(obase8[p] + coff8) << 3)) = v;
            }
        }
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        if (DBUF) {
#pragma unroll
            for (int j = 0; j < 2; ++j)
#pragma unroll
                for (int ks = 0; ks < 4; ++ks) bcur[j][ks] = bnext[j][ks];
        }
    }
}

// ---------------------------------------------------------------------------------------------
// Split-K kernel for launches whose output has too few tiles to fill the chip: decode (1-64
// tokens) and small batches. Grid = (row tiles of TM*32 rows) x (32-column blocks) x (K splits).
// The NW waves of a workgroup (4, 8 or 16: more waves keep more of the weight stream in flight)
// take the 16-wide k-steps of the split round-robin; each wave loads
// the packed tensor's 1 KB fragment blocks straight from memory into MFMA operand registers (no
// LDS staging, fully coalesced: this is the stream that is HBM-bound at decode) and the matching
// A fragments (a few rows) from global memory. The per-wave accumulators are summed through LDS
// in a fixed order. With one split the result is stored through the scatter tables; otherwise it
// goes to an fp32 partial buffer that step_split_reduce_kernel sums in split order, so results
// stay bit-reproducible (no atomics). A single-pass variant in which the last workgroup to arrive
// at a tile does the sum was measured 8x slower: a device-scope fence on this chip writes back the
// L2 of the workgroup's XCD.
// ---------------------------------------------------------------------------------------------
template <int TM, int AMODE, int NW>
__global__ void __launch_bounds__(NW * 64) step_split_kernel(StepArgs a, float* partial, int ksteps_per_split) {
    __shared__ float red[NW][TM][16][64];
    const bf16_t* A = static_cast<const bf16_t*>(a.A);
    const bf16_t* B = static_cast<const bf16_t*>(a.B);
    bf16_t* Out = static_cast<bf16_t*>(a.Out);
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const uint32_t row0 = blockIdx.x * (TM * 32);
    const int cb = blockIdx.y, split = blockIdx.z, nsplit = gridDim.z;
    const int nks = a.Kp >> 4;
    const int ks_begin = split * ksteps_per_split;
    const int ks_end = min(nks, ks_begin + ksteps_per_split);

    int64_t a_base[TM];
#pragma unroll
    for (int i = 0; i < TM; ++i) {
        uint32_t g = row0 + i * 32 + (lane & 31);
        a_base[i] = -1;
        if (g < a.total_rows) {
            uint32_t t = g / a.R;
            uint32_t r = g - t * a.R;
            a_base[i] = int64_t(t) * a.a_tok_stride + (a.arow ? int64_t(a.arow[r]) : int64_t(r) * a.K);
        }
    }
    const bf16_t* bp = B + (int64_t(cb) * nks) * 512 + lane * 8;
    floatx16 acc[TM];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[i][v] = 0.f;

    // U k-steps per batch and two batches in registers: the next batch is requested before the current
    // one is multiplied, so a wave always has loads in flight (a decode-size launch is a pure stream of
    // the packed tensor; with one batch the stream would drain at every wait)
    constexpr int U = 4;
    auto load_batch = [&](int ks0, bf16x8 (&bf)[U], bf16x8 (&af)[U][TM]) {
#pragma unroll
        for (int u = 0; u < U; ++u) {
            int ks = ks0 + NW * u;
#pragma unroll
            for (int q = 0; q < 8; ++q) bf[u][q] = bf16_t(0.f);
            if (ks < ks_end) bf[u] = *reinterpret_cast<const bf16x8*>(bp + int64_t(ks) * 512);
            int k = ks * 16 + 8 * (lane >> 5);
#pragma unroll
            for (int i = 0; i < TM; ++i) {
                bf16x8 v;
#pragma unroll
                for (int q = 0; q < 8; ++q) v[q] = bf16_t(0.f);
                if (ks < ks_end && a_base[i] >= 0) {
                    if (AMODE == 0) {
                        if (k < a.K) v = *reinterpret_cast<const bf16x8*>(A + a_base[i] + k);
                    } else {
#pragma unroll
                        for (int q = 0; q < 8; ++q)
                            if (k + q < a.K) v[q] = A[a_base[i] + (a.acol ? a.acol[k + q] : k + q)];
                    }
                }
                af[u][i] = v;
            }
        }
    };
    auto multiply = [&](const bf16x8 (&bf)[U], const bf16x8 (&af)[U][TM]) {
#pragma unroll
        for (int u = 0; u < U; ++u)
#pragma unroll
            for (int i = 0; i < TM; ++i)
                acc[i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(bf[u], af[u][i], acc[i], 0, 0, 0);
    };
    {
        bf16x8 bf0[U], af0[U][TM], bf1[U], af1[U][TM];
        constexpr int STEP = NW * U;
        int ks0 = ks_begin + wave;
        load_batch(ks0, bf0, af0);                       // batches past the end load nothing and multiply zeros
        for (; ks0 < ks_end; ks0 += 2 * STEP) {
            load_batch(ks0 + STEP, bf1, af1);
            multiply(bf0, af0);
            load_batch(ks0 + 2 * STEP, bf0, af0);
            multiply(bf1, af1);
        }
    }
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int v = 0; v < 16; ++v) red[wave][i][v][lane] = acc[i][v];
    __syncthreads();
    // operands swapped: lane l, register v holds row l%32, column 8*(v/4) + 4*(l/32) + v%4
    const uint32_t rows_pad = gridDim.x * (TM * 32);
    const float* rw = &red[0][0][0][0];
    for (int e = tid; e < TM * 1024; e += NW * 64) {
        int i = e >> 10, v = (e >> 6) & 15, l = e & 63;
        float sum = 0.f;
#pragma unroll
        for (int w = 0; w < NW; ++w) sum += rw[w * TM * 1024 + e];
        uint32_t g = row0 + i * 32 + (l & 31);
        int c = cb * 32 + 8 * (v >> 2) + 4 * (l >> 5) + (v & 3);
        if (g >= a.total_rows || c >= a.C) continue;
        if (nsplit == 1) {
            uint32_t t = g / a.R;
            uint32_t r = g - t * a.R;
            Out[int64_t(t) * a.c_tok_stride + a.crow[r] + a.ccol[c]] = bf16_t(sum);
        } else {
            partial[(int64_t(split) * rows_pad + g) * a.Cp + c] = sum;
        }
    }
}

// Sums the partial results of the split-K kernel in split order and stores through the tables.
__global__ void __launch_bounds__(256) step_split_reduce_kernel(StepArgs a, const float* partial, int nsplit,
                                                                uint32_t rows_pad) {
    bf16_t* Out = static_cast<bf16_t*>(a.Out);
    int64_t total = int64_t(a.total_rows) * a.C;
    for (int64_t e = int64_t(blockIdx.x) * 256 + threadIdx.x; e < total; e += int64_t(gridDim.x) * 256) {
        uint32_t g = uint32_t(e / a.C);
        int c = int(e - int64_t(g) * a.C);
        // 8 loads in flight at a time; the additions keep the split order
        float sum = 0.f;
        const float* src = partial + int64_t(g) * a.Cp + c;
        const int64_t sstride = int64_t(rows_pad) * a.Cp;
        for (int s0 = 0; s0 < nsplit; s0 += 8) {
            float v[8];
#pragma unroll
            for (int q = 0; q < 8; ++q) v[q] = s0 + q < nsplit ? src[int64_t(s0 + q) * sstride] : 0.f;
#pragma unroll
            for (int q = 0; q < 8; ++q) sum += v[q];
        }
        uint32_t t = g / a.R;
        uint32_t r = g - t * a.R;
        Out[int64_t(t) * a.c_tok_stride + a.crow[r] + a.ccol[c]] = bf16_t(sum);
    }
}

// ---------------------------------------------------------------------------------------------
// Fused pair of small steps (e.g. the two out-factor or the two in-factor products of a Tucker
// layer): when one token's input of the first step and its intermediate fit in LDS, a workgroup
// takes tokens one at a time, stages the token's [R1, K1] input in LDS, runs step 1 with MFMA into
// an LDS copy of the intermediate (written through step 1's scatter tables, i.e. already in the
// layout step 2 reads), runs step 2 from LDS and stores its result through step 2's tables. Each
// wave owns up to two 32-column tiles of either packed tensor and keeps their fragment blocks in
// registers for all the tokens of the workgroup (K <= 96, C <= 256); the next token's input is
// prefetched into registers while the current one is computed. The intermediate never touches HBM and one launch
// replaces two. Needs K1 % 16 == 0 and K2 % 16 == 0 (no padded k-steps are ever read).
// CM2 = 1: step 2's columns come in aligned runs of 8 -> 16-byte stores via a per-wave LDS patch;
// CM2 = 0: scalar stores.
// ---------------------------------------------------------------------------------------------
struct Fused2Args {
    StepArgs s1, s2;
    int32_t tokens;
    int32_t in_elems;     // LDS elements reserved for the staged input: roundup(R1, 32) * (K1 + 8)
    int32_t mid_elems;    // LDS elements reserved for the intermediate: roundup(R2, 32) * K2
};

template <int CM2>
__global__ void __launch_bounds__(256, 2) step_fused2_kernel(Fused2Args f) {
    extern __shared__ __attribute__((aligned(16))) unsigned char dyn_smem[];
    const StepArgs& a1 = f.s1;
    const StepArgs& a2 = f.s2;
    const int R1 = int(a1.R), K1 = a1.K, C1 = a1.C, R2 = int(a2.R), K2 = a2.K, C2 = a2.C;
    const int LD1 = K1 + 8;
    bf16_t* sIn = reinterpret_cast<bf16_t*>(dyn_smem);
    bf16_t* sMid = sIn + f.in_elems;
    bf16_t* sPatch = sMid + f.mid_elems;                       // 4 waves x 32 x 40
    int32_t* sTab = reinterpret_cast<int32_t*>(sPatch + 4 * 32 * 40);
    int32_t* t_crow1 = sTab;
    int32_t* t_ccol1 = t_crow1 + R1;
    int32_t* t_crow2 = t_ccol1 + C1;
    int32_t* t_ccol2 = t_crow2 + R2;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    for (int i = tid; i < R1; i += 256) t_crow1[i] = a1.crow[i];
    for (int i = tid; i < C1; i += 256) t_ccol1[i] = a1.ccol[i];
    for (int i = tid; i < R2; i += 256) t_crow2[i] = a2.crow[i];
    for (int i = tid; i < C2; i += 256) t_ccol2[i] = a2.ccol[i];
    // rows past R1 / R2 of the last row tile are read by the MFMAs (their results are dropped):
    // give them defined contents once
    for (int i = tid; i < f.in_elems; i += 256) sIn[i] = bf16_t(0.f);
    for (int i = tid; i < f.mid_elems; i += 256) sMid[i] = bf16_t(0.f);
    __syncthreads();

    const bf16_t* A = static_cast<const bf16_t*>(a1.A);
    const bf16_t* B1 = static_cast<const bf16_t*>(a1.B);
    const bf16_t* B2 = static_cast<const bf16_t*>(a2.B);
    bf16_t* Out = static_cast<bf16_t*>(a2.Out);
    const int nks1 = K1 >> 4, nks2 = K2 >> 4;                  // real k-steps (<= 6)
    const int bks1 = a1.Kp >> 4, bks2 = a2.Kp >> 4;            // k-steps per column block in the packed tensors
    const int nrt1 = (R1 + 31) >> 5, nct1 = (C1 + 31) >> 5;
    const int nrt2 = (R2 + 31) >> 5, nct2 = (C2 + 31) >> 5;     // nct <= 8: column tiles j = wave, wave + 4
    const int chunks_per_row = K1 >> 3;
    bf16_t* myPatch = sPatch + wave * 32 * 40;

    // the wave's column tiles of both packed tensors stay in registers for all of its tokens
    bf16x8 bw1[2][6], bw2[2][6];
#pragma unroll
    for (int jj = 0; jj < 2; ++jj)
#pragma unroll
        for (int ks = 0; ks < 6; ++ks) {
            bf16x8 z;
#pragma unroll
            for (int q = 0; q < 8; ++q) z[q] = bf16_t(0.f);
            int j = wave + 4 * jj;
            bw1[jj][ks] = (j < nct1 && ks < nks1)
                              ? *reinterpret_cast<const bf16x8*>(B1 + (int64_t(j) * bks1 + ks) * 512 + lane * 8) : z;
            bw2[jj][ks] = (j < nct2 && ks < nks2)
                              ? *reinterpret_cast<const bf16x8*>(B2 + (int64_t(j) * bks2 + ks) * 512 + lane * 8) : z;
        }

    // the next token's input is fetched into registers while the current token is computed
    // (at most 6 chunks of 16 bytes per thread: R1 * K1 <= 12288)
    const int n_chunks = R1 * chunks_per_row;
    int my_off[6];                                             // LDS element offset of each of my chunks
#pragma unroll
    for (int q = 0; q < 6; ++q) {
        int e = tid + 256 * q;
        int r = e / chunks_per_row;
        my_off[q] = e < n_chunks ? r * LD1 + (e - r * chunks_per_row) * 8 : -1;
    }
    bf16x8 pre[6];
    auto fetch_in = [&](int t) {
        const bf16_t* in = A + int64_t(t) * a1.a_tok_stride + tid * 8;
#pragma unroll
        for (int q = 0; q < 6; ++q)
            if (my_off[q] >= 0) pre[q] = *reinterpret_cast<const bf16x8*>(in + 2048 * q);
    };
    if (int(blockIdx.x) < f.tokens) fetch_in(blockIdx.x);
    for (int t = blockIdx.x; t < f.tokens; t += gridDim.x) {
        // ---- stage the token's input
#pragma unroll
        for (int q = 0; q < 6; ++q)
            if (my_off[q] >= 0) *reinterpret_cast<bf16x8*>(sIn + my_off[q]) = pre[q];
        __syncthreads();
        if (t + int(gridDim.x) < f.tokens) fetch_in(t + gridDim.x);
        // ---- step 1
#pragma unroll
        for (int jj = 0; jj < 2; ++jj) {
            const int j = wave + 4 * jj;
            if (j >= nct1) continue;
            for (int i = 0; i < nrt1; ++i) {
                floatx16 acc;
#pragma unroll
                for (int v = 0; v < 16; ++v) acc[v] = 0.f;
                const bf16_t* ap = sIn + (i * 32 + (lane & 31)) * LD1 + 8 * (lane >> 5);
                bf16x8 af[6];                 // all fragment reads first, then the MFMA chain
#pragma unroll
                for (int ks = 0; ks < 6; ++ks)
                    if (ks < nks1) af[ks] = *reinterpret_cast<const bf16x8*>(ap + ks * 16);
#pragma unroll
                for (int ks = 0; ks < 6; ++ks)
                    if (ks < nks1) acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(bw1[jj][ks], af[ks], acc, 0, 0, 0);
                // lane l, register v: row l%32, column 8*(v/4) + 4*(l/32) + v%4
                int r = i * 32 + (lane & 31);
                if (r < R1) {
                    int rbase = t_crow1[r];
#pragma unroll
                    for (int v = 0; v < 16; ++v) {
                        int c = j * 32 + 8 * (v >> 2) + 4 * (lane >> 5) + (v & 3);
                        if (c < C1) sMid[rbase + t_ccol1[c]] = bf16_t(acc[v]);
                    }
                }
            }
        }
        __syncthreads();
        // ---- step 2 from the LDS intermediate
        bf16_t* out_t = Out + int64_t(t) * a2.c_tok_stride;
#pragma unroll
        for (int jj = 0; jj < 2; ++jj) {
            const int j = wave + 4 * jj;
            if (j >= nct2) continue;
            for (int i = 0; i < nrt2; ++i) {
                floatx16 acc;
#pragma unroll
                for (int v = 0; v < 16; ++v) acc[v] = 0.f;
                const bf16_t* ap = sMid + (i * 32 + (lane & 31)) * K2 + 8 * (lane >> 5);
                bf16x8 af[6];
#pragma unroll
                for (int ks = 0; ks < 6; ++ks)
                    if (ks < nks2) af[ks] = *reinterpret_cast<const bf16x8*>(ap + ks * 16);
#pragma unroll
                for (int ks = 0; ks < 6; ++ks)
                    if (ks < nks2) acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(bw2[jj][ks], af[ks], acc, 0, 0, 0);
                if (CM2 == 1) {
#pragma unroll
                    for (int q = 0; q < 4; ++q) {
                        bf16x4 pk;
#pragma unroll
                        for (int u = 0; u < 4; ++u) pk[u] = bf16_t(acc[4 * q + u]);
                        *reinterpret_cast<bf16x4*>(myPatch + (lane & 31) * 40 + 8 * q + 4 * (lane >> 5)) = pk;
                    }
                    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
                    __builtin_amdgcn_wave_barrier();
                    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
                    int c = j * 32 + (lane & 3) * 8;
#pragma unroll
                    for (int h = 0; h < 2; ++h) {
                        int rr = h * 16 + (lane >> 2);
                        int r = i * 32 + rr;
                        bf16x8 v = *reinterpret_cast<const bf16x8*>(myPatch + rr * 40 + (lane & 3) * 8);
                        if (r < R2 && c < C2) *reinterpret_cast<bf16x8*>(out_t + t_crow2[r] + t_ccol2[c]) = v;
                    }
                    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
                    __builtin_amdgcn_wave_barrier();
                } else {
                    int r = i * 32 + (lane & 31);
                    if (r < R2) {
                        int rbase = t_crow2[r];
#pragma unroll
                        for (int v = 0; v < 16; ++v) {
                            int c = j * 32 + 8 * (v >> 2) + 4 * (lane >> 5) + (v & 3);
                            if (c < C2) out_t[rbase + t_ccol2[c]] = bf16_t(acc[v]);
                        }
                    }
                }
            }
        }
        __syncthreads();   // sIn and sMid are rewritten for the next token
    }
}

// ---------------------------------------------------------------------------------------------
// Chained pair kernel: a short-K step followed by a long-K step whose K is (rows of the first
// step) x (a bond of 64), the shape a tensor train takes once its end cores are contracted into
// their neighbours (Section 3.5: fuse core contractions, specialise for shared ranks):
//     Z[t][j][a][b] = sum_k  X[t][a*64 + k] * B0[j*64 + b][k]          K0 = 64, bond b < 64
//     Y[t][yrow[j] + ycol[c]] = sum_{a, b} Z[t][j][a][b] * B1[c][a*64 + b]      c < C1 <= 128
// Unfused, Z (A*J*64 values per token) is written to and read back from HBM and both launches are
// bound by that traffic. Here Z never leaves the registers: a workgroup owns 32 tokens and 8
// values of j (two per wave) and walks over a. For one a, a wave computes Z^T[b][t] for its two j
// with the packed tensor of the first step as the row operand (kept in registers for the whole
// walk) and the tokens as MFMA columns; the result lands in the accumulator layout (lane: token
// l%32, b = 8*(v/4) + 4*(l/32) + v%4), which after rounding to bf16 IS the column operand of the
// second contraction when that step's packed tensor is stored with the same permutation of b
// inside each k-step of 16 (done once at create time by pair_repack_kernel). Per a the workgroup
// streams a 16 KB slice of B1 and 4 KB of X into a ring of LDS stages with direct-to-LDS loads.
// The 32 x C1 x 8 results of the workgroup are transposed through LDS and stored as 16-byte
// pieces (8 consecutive j). Workgroups that share a token tile run back to back on one XCD, so
// that their reads of X and their pieces of the same output lines meet in that XCD's L2.
// ---------------------------------------------------------------------------------------------
struct PairArgs {
    const void* X;
    void* Y;
    const void* B0;        // first step's packed tensor, fragment-major [J*64][64]
    const void* B1f;       // second step's packed tensor in the chained layout (pair_repack_kernel)
    const int32_t* yrow;   // output offset of j (J entries, aligned runs of 8)
    const int32_t* ycol;   // output offset of c (C1 entries, multiples of 8)
    int64_t N, M;          // elements per token of X and Y
    int32_t tokens, A, J, C1;
    int32_t n_tok_tiles, n_jsets;
};

// B1f[((a*16 + ct*4 + s)*64 + l)*8 + e] = B1[c = 32*ct + l%32][k = a*64 + 16*s + 8*(e/4) + 4*(l/32) + e%4]
__global__ void __launch_bounds__(256) pair_repack_kernel(const bf16_t* src, bf16_t* dst, int A, int nks, int Cp) {
    int64_t total = int64_t(A) * 8192;
    for (int64_t i = int64_t(blockIdx.x) * 256 + threadIdx.x; i < total; i += int64_t(gridDim.x) * 256) {
        int e = int(i & 7), l = int(i >> 3) & 63, blk = int(i >> 9) & 15;
        int a = int(i >> 13);
        int c = 32 * (blk >> 2) + (l & 31);
        int k = a * 64 + 16 * (blk & 3) + 8 * (e >> 2) + 4 * (l >> 5) + (e & 3);
        dst[i] = c < Cp ? src[bfrag_offset(c, k, nks)] : bf16_t(0.f);      // columns past Cp do not exist
    }
}

template <int NS>
__global__ void __launch_bounds__(256, 1) step_pair_kernel(PairArgs p) {
    constexpr int L = 5;                               // NS ring stages; L direct-to-LDS loads per wave and stage
    constexpr int STAGE_BYTES = 20 * 1024, X_OFF = 16 * 1024;
    extern __shared__ __attribute__((aligned(16))) unsigned char dyn_smem[];

    const int id = blockIdx.x;
    const int xcd = id & 7, slot = id >> 3;
    const int tok_tile = (slot / p.n_jsets) * 8 + xcd;
    const int jset = slot % p.n_jsets;
    if (tok_tile >= p.n_tok_tiles) return;
    const int t0 = tok_tile * 32;

    const bf16_t* X = static_cast<const bf16_t*>(p.X);
    const bf16_t* B0 = static_cast<const bf16_t*>(p.B0);
    const bf16_t* B1f = static_cast<const bf16_t*>(p.B1f);
    bf16_t* Y = static_cast<bf16_t*>(p.Y);
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int j0 = jset * 8 + wave * 2;
    const int A = p.A;

    // the wave's rows of the first packed tensor: [jj][32-row half of the bond][k-step]
    bf16x8 p0[2][2][4];
#pragma unroll
    for (int jj = 0; jj < 2; ++jj)
#pragma unroll
        for (int rt = 0; rt < 2; ++rt)
#pragma unroll
            for (int s = 0; s < 4; ++s)
                p0[jj][rt][s] = *reinterpret_cast<const bf16x8*>(B0 + (int64_t((j0 + jj) * 2 + rt) * 4 + s) * 512 + lane * 8);

    // direct-to-LDS sources: wave w brings blocks w, w+4, w+8, w+12 of the B1 slice and k-step w of X
    const int tl = min(t0 + (lane & 31), p.tokens - 1);             // rows past the end repeat the last token
    const bf16_t* x_src = X + int64_t(tl) * p.N + 16 * wave + 8 * (lane >> 5);
    const bf16_t* b_src = B1f + lane * 8;
    auto issue = [&](int a, int stage) {
        unsigned char* sbase = dyn_smem + stage * STAGE_BYTES;
#pragma unroll
        for (int q = 0; q < 4; ++q)
            __builtin_amdgcn_global_load_lds(
                (const void __attribute__((address_space(1)))*)(b_src + (int64_t(a) * 16 + wave + 4 * q) * 512),
                (void __attribute__((address_space(3)))*)(sbase + (wave + 4 * q) * 1024), 16, 0, 0);
        __builtin_amdgcn_global_load_lds(
            (const void __attribute__((address_space(1)))*)(x_src + int64_t(a) * 64),
            (void __attribute__((address_space(3)))*)(sbase + X_OFF + wave * 1024), 16, 0, 0);
    };
    auto wait_outstanding_tiles = [&](int n) {            // n is wave-uniform, at most NS - 2
        if (n <= 0) wait_vmcnt<0>();
        else if (n == 1) wait_vmcnt<L>();
        else if (n == 2 || NS <= 4) wait_vmcnt<2 * L>();
        else if (n == 3 || NS <= 5) wait_vmcnt<3 * L>();
        else wait_vmcnt<4 * L>();
    };

    floatx16 acc[2][4];
#pragma unroll
    for (int jj = 0; jj < 2; ++jj)
#pragma unroll
        for (int ct = 0; ct < 4; ++ct)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[jj][ct][v] = 0.f;

    int issued = 0;
    for (; issued < NS - 1 && issued < A; ++issued) issue(issued, issued);
    wait_outstanding_tiles(min(issued - 1, NS - 2));     // tile 0 has landed
    __syncthreads();
    bf16x8 xb[4];
#pragma unroll
    for (int s = 0; s < 4; ++s) xb[s] = *reinterpret_cast<const bf16x8*>(dyn_smem + X_OFF + s * 1024 + lane * 16);

    // first contraction for one j: Z^T[b][t], two 32-row halves of the bond
    auto contract0 = [&](const bf16x8 (&w)[2][4], const bf16x8 (&x)[4], floatx16 (&z)[2]) {
#pragma unroll
        for (int rt = 0; rt < 2; ++rt)
#pragma unroll
            for (int v = 0; v < 16; ++v) z[rt][v] = 0.f;
#pragma unroll
        for (int s = 0; s < 4; ++s)
#pragma unroll
            for (int rt = 0; rt < 2; ++rt)
                z[rt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(w[rt][s], x[s], z[rt], 0, 0, 0);
    };
    // second contraction for one j: Y^T[c][t] += B1[c][(a, b)] Z^T[b][t]. Registers 8*(s%2) .. +7 of
    // half s/2 of z are the 8 values this lane supplies to k-step s.
    auto contract1 = [&](const bf16x8 (&w)[4][4], const floatx16 (&z)[2], floatx16 (&y)[4]) {
        bf16x8 zb[4];
#pragma unroll
        for (int s = 0; s < 4; ++s)
#pragma unroll
            for (int e = 0; e < 8; ++e) zb[s][e] = bf16_t(z[s >> 1][8 * (s & 1) + e]);
#pragma unroll
        for (int s = 0; s < 4; ++s)
#pragma unroll
            for (int ct = 0; ct < 4; ++ct)
                y[ct] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(w[ct][s], zb[s], y[ct], 0, 0, 0);
    };

    // software pipeline over (a, j): the first contraction of the next unit is issued before the
    // second contraction of the current one, so that reading back and rounding Z overlaps MFMAs
    floatx16 z0[2], z1[2];
    contract0(p0[0], xb, z0);
    auto iteration = [&](int a, auto last_tag) {
        constexpr bool LAST = decltype(last_tag)::value;
        if (!LAST) wait_outstanding_tiles(issued - (a + 2));       // tile a+1 has landed
        __syncthreads();       // everyone is done with tile a-1: its stage may be refilled
        if (issued < A) {
            issue(issued, issued % NS);
            ++issued;
        }
        const unsigned char* scur = dyn_smem + (a % NS) * STAGE_BYTES;
        const unsigned char* snxt = dyn_smem + ((a + 1) % NS) * STAGE_BYTES;
        bf16x8 p1[4][4];
#pragma unroll
        for (int ct = 0; ct < 4; ++ct)
#pragma unroll
            for (int s = 0; s < 4; ++s)
                p1[ct][s] = *reinterpret_cast<const bf16x8*>(scur + (ct * 4 + s) * 1024 + lane * 16);
        // the scheduler would otherwise sink each LDS read next to its first use and expose the LDS
        // latency 16 times per iteration
        __builtin_amdgcn_sched_barrier(0);
        contract0(p0[1], xb, z1);
        if (!LAST) {
#pragma unroll
            for (int s = 0; s < 4; ++s) xb[s] = *reinterpret_cast<const bf16x8*>(snxt + X_OFF + s * 1024 + lane * 16);
            __builtin_amdgcn_sched_barrier(0);
        }
        contract1(p1, z0, acc[0]);
        if (!LAST) contract0(p0[0], xb, z0);
        contract1(p1, z1, acc[1]);
        // keep the accumulators in the accumulation registers across the back edge (the register
        // allocator otherwise parks some of them in ordinary registers and copies them every
        // iteration)
#pragma unroll
        for (int jj = 0; jj < 2; ++jj)
#pragma unroll
            for (int ct = 0; ct < 4; ++ct) asm volatile("" : "+a"(acc[jj][ct]));
        if (!LAST) {
            asm volatile("" : "+a"(z0[0]));
            asm volatile("" : "+a"(z0[1]));
        }
    };
    for (int a = 0; a + 1 < A; ++a) iteration(a, std::false_type());
    iteration(A - 1, std::true_type());
    __syncthreads();

    // ---- epilogue: lane l, register v of acc[jj][ct] is token l%32, c = 32*ct + 8*(v/4) + 4*(l/32) + v%4.
    //      LDS holds [32 tokens][128 c] pieces of 16 bytes (the 8 j of the workgroup), the piece of
    //      (t, c) at position c ^ t of row t so that neither the 4-byte writes nor the 16-byte reads
    //      pile up on a bank.
    {
        const int t = lane & 31;
        typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
#pragma unroll
        for (int ct = 0; ct < 4; ++ct)
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                int c = 32 * ct + 8 * (v >> 2) + 4 * (lane >> 5) + (v & 3);
                bf16x2 pr;
                pr[0] = bf16_t(acc[0][ct][v]);
                pr[1] = bf16_t(acc[1][ct][v]);
                *reinterpret_cast<bf16x2*>(dyn_smem + (t * 128 + (c ^ t)) * 16 + wave * 4) = pr;
            }
    }
    __syncthreads();
    const int yj = p.yrow[jset * 8];
#pragma unroll 4
    for (int e = tid; e < 32 * 128; e += 256) {
        int t = e >> 7, c = e & 127;
        if (t0 + t >= p.tokens || c >= p.C1) continue;
        bf16x8 v = *reinterpret_cast<const bf16x8*>(dyn_smem + (t * 128 + (c ^ t)) * 16);
        *reinterpret_cast<bf16x8*>(Y + int64_t(t0 + t) * p.M + p.ycol[c] + yj) = v;
    }
}

// ---------------------------------------------------------------------------------------------
// Transposing chain of two small steps (the two in-factor or the two out-factor products of a
// Tucker layer): the second step contracts the ROW index r of the first and keeps its column index
// c1 as a row,
//     T[r][c1] = sum_k  In[t][r][k] * Ba[c1][k]                    R1 x K1 input per token
//     Out[t][off1[c1] + off2[c2]] = sum_r T[r][c1] * Bb[c2][r]
// A wave owns one token at a time. The token's input travels from memory straight into a
// wave-private LDS buffer in MFMA fragment order (direct-to-LDS loads, double buffered: the next
// token's input is in flight while the current one is computed; no workgroup barrier anywhere).
// For each tile of 32 values of c1 the wave computes T^T as accumulator tiles with r in the
// registers and c1 across the lanes, rounds them to bf16 and feeds them - without leaving the
// registers - to the second contraction, whose packed tensor is stored at create time with the
// matching permutation of r inside each k-step (chain2_repack_kernel) and stays in registers for
// all tokens. The intermediate T never exists in memory, one launch replaces two, and the HBM
// traffic drops to the first step's input plus the second step's output.
// RUN_C1 = 1: the output takes 8 consecutive c1 as an aligned 16-byte piece (T^T is the row operand
// of the second MFMA, so a lane ends up with 4 consecutive c1); RUN_C1 = 0: 8 consecutive c2 (T^T is
// the column operand). Either way the 32x32 result tiles pass through a wave-private LDS patch and
// leave as 16-byte stores.
// Limits: R1 <= 32*R1T, K1 <= 16*K1S, K1 % 8 == 0, C2 <= 32*C2T; any C1.
// ---------------------------------------------------------------------------------------------
struct Chain2Args {
    const void* In;
    void* Out;
    const void* Ba;         // first step's packed tensor (fragment-major, nks_a k-steps per column block)
    const void* Bbf;        // second step's packed tensor in the chained layout
    const int32_t* off1;    // output offset of c1 (the second step's row table)
    const int32_t* off2;    // output offset of c2 (the second step's column table)
    int64_t in_tok_stride, out_tok_stride;
    int32_t tokens, R1, K1, C1, C2;
    int32_t nks_a;
    int32_t c1_tiles;       // ceil(C1 / 32)
    int32_t tiles_per_item; // c1 tiles one wave handles per visit of a token (all of them for large
                            // batches; 1 spreads a single token over several waves)
};

// Bbf[((j*KS + s)*64 + l)*8 + e] = Bb[c2 = 32*j + l%32][r = 16*s + 8*(e/4) + 4*(l/32) + e%4], zero outside
__global__ void __launch_bounds__(256) chain2_repack_kernel(const bf16_t* src, bf16_t* dst, int C2T, int KS,
                                                            int nks_src, int Cp, int Kp) {
    int total = C2T * KS * 512;
    for (int i = blockIdx.x * 256 + threadIdx.x; i < total; i += gridDim.x * 256) {
        int e = i & 7, l = (i >> 3) & 63, blk = i >> 9;
        int j = blk / KS, sk = blk - j * KS;
        int c = 32 * j + (l & 31);
        int k = 16 * sk + 8 * (e >> 2) + 4 * (l >> 5) + (e & 3);
        dst[i] = (c < Cp && k < Kp) ? src[bfrag_offset(c, k, nks_src)] : bf16_t(0.f);
    }
}

template <int R1T, int K1S, int C2T>
constexpr size_t chain2_smem_bytes() {
    return size_t(4) * (R1T * K1S * 1024 + 2 * 32 * 80);
}

template <int R1T, int K1S, int C2T, int RUN_C1>
__global__ void __launch_bounds__(256, 1) step_chain2_kernel(Chain2Args p) {
    constexpr int IN_BYTES = R1T * K1S * 1024;           // one token's input in fragment order
    constexpr int KS2 = 2 * R1T;                         // k-steps of the second contraction
    constexpr int PATCH_LD = 80;                         // bytes per patch row (64 + 16 of padding)
    constexpr int PATCH_BYTES = 32 * PATCH_LD;
    extern __shared__ __attribute__((aligned(16))) unsigned char dyn_smem[];
    const bf16_t* In = static_cast<const bf16_t*>(p.In);
    const bf16_t* Ba = static_cast<const bf16_t*>(p.Ba);
    const bf16_t* Bbf = static_cast<const bf16_t*>(p.Bbf);
    bf16_t* Out = static_cast<bf16_t*>(p.Out);
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    unsigned char* my_in = dyn_smem + wave * IN_BYTES;
    unsigned char* my_patch = dyn_smem + 4 * IN_BYTES + wave * (2 * PATCH_BYTES);

    const int n_groups = (p.c1_tiles + p.tiles_per_item - 1) / p.tiles_per_item;
    const int64_t n_items = int64_t(p.tokens) * n_groups;
    const int64_t gw = int64_t(blockIdx.x) * 4 + wave, GW = int64_t(gridDim.x) * 4;
    if (gw >= n_items) return;                           // no workgroup barrier below: a wave may leave

    // lanes whose (row, k) lies outside the input never load: the fragment blocks they belong to are
    // zeroed once and keep those zeros
#pragma unroll
    for (int i = 0; i < R1T; ++i)
#pragma unroll
        for (int sk = 0; sk < K1S; ++sk)
            if (32 * i + 32 > p.R1 || 16 * sk + 16 > p.K1) {        // wave-uniform
                bf16x8 z;
#pragma unroll
                for (int q = 0; q < 8; ++q) z[q] = bf16_t(0.f);
                *reinterpret_cast<bf16x8*>(my_in + (i * K1S + sk) * 1024 + lane * 16) = z;
            }
    __builtin_amdgcn_s_waitcnt(0xc07f);                  // lgkmcnt(0): the zeros are in LDS before any load lands
    __builtin_amdgcn_wave_barrier();

    // the second packed tensor stays in registers for every token of the wave
    bf16x8 bb[C2T][KS2];
#pragma unroll
    for (int j = 0; j < C2T; ++j)
#pragma unroll
        for (int sk = 0; sk < KS2; ++sk)
            bb[j][sk] = *reinterpret_cast<const bf16x8*>(Bbf + (int64_t(j) * KS2 + sk) * 512 + lane * 8);

    const int nrt = (p.R1 + 31) >> 5, nks1 = (p.K1 + 15) >> 4;
    const int nj = (p.C2 + 31) >> 5;
    const int lrow = lane & 31, lk = 8 * (lane >> 5);
    auto issue_in = [&](int t) {
        const bf16_t* src = In + int64_t(t) * p.in_tok_stride + int64_t(lrow) * p.K1 + lk;
#pragma unroll
        for (int i = 0; i < R1T; ++i)
#pragma unroll
            for (int sk = 0; sk < K1S; ++sk) {
                if (i < nrt && sk < nks1) {                          // wave-uniform
                    if (32 * i + lrow < p.R1 && 16 * sk + lk < p.K1)
                        __builtin_amdgcn_global_load_lds(
                            (const void __attribute__((address_space(1)))*)(src + int64_t(32 * i) * p.K1 + 16 * sk),
                            (void __attribute__((address_space(3)))*)(my_in + (i * K1S + sk) * 1024), 16, 0, 0);
                }
            }
    };
    auto load_ba = [&](int ct1, bf16x8 (&ba)[K1S]) {
#pragma unroll
        for (int sk = 0; sk < K1S; ++sk)      // k-steps past the packed tensor's padding meet zero input: any finite block will do
            ba[sk] = *reinterpret_cast<const bf16x8*>(Ba + (int64_t(ct1) * p.nks_a + min(sk, p.nks_a - 1)) * 512 + lane * 8);
    };

    // output offsets of the two 16-byte pieces a lane stores per 32x32 tile (patch row lane/4 + 16h,
    // piece lane%4): those along c2 never change; those along c1 are fetched a tile ahead. -1 = outside.
    const int prow = lane >> 2, pchunk = lane & 3;
    int o2[C2T][2];
#pragma unroll
    for (int j = 0; j < C2T; ++j)
#pragma unroll
        for (int h = 0; h < 2; ++h) {
            int c2 = 32 * j + (RUN_C1 ? prow + 16 * h : 8 * pchunk);
            o2[j][h] = c2 < p.C2 ? p.off2[c2] : -1;
        }
    auto load_o1 = [&](int ct1, int (&o1)[2]) {
#pragma unroll
        for (int h = 0; h < 2; ++h) {
            int c1 = 32 * ct1 + (RUN_C1 ? 8 * pchunk : prow + 16 * h);
            o1[h] = c1 < p.C1 ? p.off1[c1] : -1;
        }
    };

    // Vector memory operations a full item issues after its input request (the packed-tensor loads and
    // the stores of every tile but a possibly ragged last one, a lower bound). Loads complete in issue
    // order, so once at most 63 operations are in flight an input request older than that has landed,
    // without waiting for the latest stores to be acknowledged.
    const int ops_after = max(0, p.tiles_per_item - ((p.C1 & 31) ? 1 : 0)) * (K1S + 2 * (p.C2 >> 5));
    issue_in(int(gw / n_groups));
    for (int64_t item = gw; item < n_items; item += GW) {
        const int t = int(item / n_groups);
        const int g = int(item - int64_t(t) * n_groups);
        const int tile_begin = g * p.tiles_per_item;
        const int tile_end = min(p.c1_tiles, tile_begin + p.tiles_per_item);
        bf16x8 ba_next[K1S];
        int o1_next[2];
        load_ba(tile_begin, ba_next);
        load_o1(tile_begin, o1_next);
        if (item == gw || ops_after < 66 + K1S) wait_vmcnt<0>();
        else wait_vmcnt<61 - K1S>();                                  // the loads above are younger still
        // the token's input moves to registers; its LDS buffer then takes the next item's input,
        // which travels while this item is computed
        bf16x8 inf[R1T][K1S];
#pragma unroll
        for (int i = 0; i < R1T; ++i)
#pragma unroll
            for (int sk = 0; sk < K1S; ++sk)      // slots outside the input hold zeros
                inf[i][sk] = *reinterpret_cast<const bf16x8*>(my_in + (i * K1S + sk) * 1024 + lane * 16);
        __builtin_amdgcn_s_waitcnt(0xc07f);                          // the reads are done before the buffer is refilled
        if (item + GW < n_items) issue_in(int((item + GW) / n_groups));
        bf16_t* out_t = Out + int64_t(t) * p.out_tok_stride;
        for (int ct1 = tile_begin; ct1 < tile_end; ++ct1) {
            bf16x8 ba[K1S];
#pragma unroll
            for (int sk = 0; sk < K1S; ++sk) ba[sk] = ba_next[sk];
            const int o1[2] = {o1_next[0], o1_next[1]};
            if (ct1 + 1 < tile_end) {
                load_ba(ct1 + 1, ba_next);
                load_o1(ct1 + 1, o1_next);
            }
            // first contraction: accumulator tile i holds T^T for r in [32i, 32i+32): lane l has c1 = l%32,
            // register v has r = 32i + 8*(v/4) + 4*(l/32) + v%4
            floatx16 d[R1T];
#pragma unroll
            for (int i = 0; i < R1T; ++i)
#pragma unroll
                for (int v = 0; v < 16; ++v) d[i][v] = 0.f;
#pragma unroll
            for (int sk = 0; sk < K1S; ++sk)
#pragma unroll
                for (int i = 0; i < R1T; ++i)
                    d[i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(inf[i][sk], ba[sk], d[i], 0, 0, 0);
            bf16x8 zb[KS2];
#pragma unroll
            for (int i = 0; i < R1T; ++i)
#pragma unroll
                for (int u = 0; u < 2; ++u)
#pragma unroll
                    for (int e = 0; e < 8; ++e) zb[2 * i + u][e] = bf16_t(d[i][8 * u + e]);
            // second contraction: all tiles of c2 (independent accumulators), then their way out
            floatx16 acc[C2T];
#pragma unroll
            for (int j = 0; j < C2T; ++j)
#pragma unroll
                for (int v = 0; v < 16; ++v) acc[j][v] = 0.f;
#pragma unroll
            for (int sk = 0; sk < KS2; ++sk)
#pragma unroll
                for (int j = 0; j < C2T; ++j)
                        acc[j] = RUN_C1 ? __builtin_amdgcn_mfma_f32_32x32x16_bf16(zb[sk], bb[j][sk], acc[j], 0, 0, 0)
                                        : __builtin_amdgcn_mfma_f32_32x32x16_bf16(bb[j][sk], zb[sk], acc[j], 0, 0, 0);
            // RUN_C1: lane l holds c2 = 32j + l%32 and, in registers 4q..4q+3, c1 = 32*ct1 + 8q + 4*(l/32) + 0..3
            // else  : lane l holds c1 = 32*ct1 + l%32 and c2 = 32j + 8q + 4*(l/32) + 0..3
            // The 32x32 tiles pass through two alternating wave-private LDS patches and leave as 16-byte
            // pieces; a patch is rewritten two tiles later, after the wave barrier of the tile between.
#pragma unroll
            for (int j = 0; j < C2T; ++j) {
                if (j >= nj) continue;                                 // wave-uniform
                unsigned char* patch = my_patch + (j & 1) * PATCH_BYTES;
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    bf16x4 pk;
#pragma unroll
                    for (int u = 0; u < 4; ++u) pk[u] = bf16_t(acc[j][4 * q + u]);
                    *reinterpret_cast<bf16x4*>(patch + (lane & 31) * PATCH_LD + (8 * q + 4 * (lane >> 5)) * 2) = pk;
                }
                __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
                __builtin_amdgcn_wave_barrier();
                __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
#pragma unroll
                for (int h = 0; h < 2; ++h) {
                    bf16x8 v = *reinterpret_cast<const bf16x8*>(patch + (prow + 16 * h) * PATCH_LD + pchunk * 16);
                    if (o1[h] >= 0 && o2[j][h] >= 0) *reinterpret_cast<bf16x8*>(out_t + o1[h] + o2[j][h]) = v;
                }
            }
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
            __builtin_amdgcn_wave_barrier();
        }
    }
}

// ---------------------------------------------------------------------------------------------
// host side
// ---------------------------------------------------------------------------------------------
enum Variant : int {
    VAR_SCALAR = 0,
    VAR_MFMA_256x32 = 2,      // narrow outputs (<= 32 columns)
    VAR_PIPE_128x256 = 3,     // register-prefetch tiles, 4 waves, 2 workgroups per CU, one LDS stage
    VAR_PIPE_256x128 = 8,     // same, 4 waves stacked along rows
    VAR_SHORTK = 9,           // K <= 64, store-bound: registers-only operands, barrier-free
    VAR_DLDS8_256x256 = 12,   // direct-to-LDS ring, 8 waves, 4 stages, 1 workgroup per CU
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
    bool fuse_next = false;       // this step and the next run as one launch
    int fuse_kind = 0;            // 1 step_fused2_kernel (opt-in), 2 step_chain2_kernel
    void* chain_bbf = nullptr;    // chain2: the next step's packed tensor in the chained layout
    int chain_cfg = 0;            // chain2 instantiation: 0 <3,6,5>, 1 <2,8,2>
    int chain_run_c1 = 0;         // chain2: output pieces run along c1 (else along c2)
    int fused_in_elems = 0, fused_mid_elems = 0;
    size_t fused_smem = 0;
};

}  // namespace

struct tn_linear_s {
    tn::Plan plan;
    std::vector<DevStep> steps;
    int elt = 4;
    int64_t max_tokens = 0, chunk_tokens = 0;
    int64_t packed_bytes = 0, workspace_bytes = 0;
    void* ws[2] = {nullptr, nullptr};
    void* partial = nullptr;          // fp32 partial sums of the split-K kernel
    int64_t partial_bytes = 0;
    int flags = 0;
    bool owns_workspace = true;
    int device = 0;
    int num_cus = 256;
    bool profiling = false;
    // chained pair kernel (two-step plans of the train shape): second packed tensor in its layout
    bool pair = false;
    void* pair_b1f = nullptr;
    int64_t pair_min_tokens = 0;
    struct ProfRec { int step; hipEvent_t start, stop; };
    std::vector<ProfRec> prof;
};

namespace {

constexpr int64_t kDefaultWorkspaceBytes = int64_t(16) << 30;

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
        if (s.chain_bbf) (void)hipFree(s.chain_bbf);
    }
    if (h->pair_b1f) (void)hipFree(h->pair_b1f);
    if (h->owns_workspace) {
        for (void* w : h->ws)
            if (w) (void)hipFree(w);
        if (h->partial) (void)hipFree(h->partial);
    }
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
        int forced = (flags >> TN_FLAG_VARIANT_SHIFT) & 0xff;
        // default: the tile width that wastes the fewest padded columns (256 on a tie); the
        // register-only kernel for short-K, wide steps
        const bool shortk_ok = p.K <= 64 && p.c_vec == 8;
        int v = round_up(int(p.C), 128) < round_up(int(p.C), 256) ? VAR_PIPE_256x128 : VAR_PIPE_128x256;
        // direct-to-LDS tiles where A is a plain matrix whose K is a whole number of 32-wide tiles
        const bool dlds_ok = p.a_plain && p.K % 32 == 0 && p.K >= 64;
        // (measured: the 8-wave 256x256 ring beats the register-prefetch tiles on every shape it
        // fits without extra column padding; the 4-wave direct-to-LDS tiles do not)
        if (dlds_ok && p.C >= 256 && round_up(int(p.C), 256) == round_up(int(p.C), 128)) v = VAR_DLDS8_256x256;
        if (shortk_ok && p.C >= 256) v = VAR_SHORTK;
        if (forced == VAR_PIPE_128x256 || forced == VAR_PIPE_256x128 || (forced == VAR_SHORTK && shortk_ok) ||
            (forced == VAR_DLDS8_256x256 && dlds_ok))
            v = forced;
        s->variant = v;
        switch (v) {
            case VAR_SHORTK: s->bm = 128; s->bn = 128; break;
            case VAR_PIPE_128x256: s->bm = 128; s->bn = 256; break;
            case VAR_PIPE_256x128: s->bm = 256; s->bn = 128; break;
            default: s->bm = 256; s->bn = 256; break;      // VAR_DLDS8_256x256
        }
    }
    s->amode = (p.a_plain && p.K % 8 == 0) ? 0 : 1;
    s->cmode = p.c_vec == 8 ? 1 : (p.r_vec == 8 ? 2 : 0);
    s->Kp = round_up(int(p.K), 64);
    s->Cp = round_up(int(p.C), s->bn);
}

struct SplitCfg {
    bool use = false;
    int tm = 1, nw = 4, row_tiles = 0, col_blocks = 0, nsplit = 1, ksteps_per_split = 0;
    int64_t partial_bytes = 0;
};

constexpr int64_t kMaxPartialBytes = int64_t(64) << 20;

// Decide whether a launch of `rows` rows runs on the split-K kernel: when the tiled kernel would
// start fewer workgroups than there are compute units and K is long enough to share out.
SplitCfg split_config(const DevStep& s, int64_t rows) {
    SplitCfg c;
    if (s.variant == VAR_SCALAR || rows <= 0) return c;
    int64_t tiles = ((rows + s.bm - 1) / s.bm) * (s.Cp / s.bn);
    int nks = s.Kp / 16;
    // the narrow tile keeps 4 waves of a CU busy at best: it needs twice as many tiles to fill the chip
    if (tiles >= (s.variant == VAR_MFMA_256x32 ? 512 : 128) || nks < 8) return c;
    c.tm = rows > 32 ? 2 : 1;
    c.row_tiles = int((rows + 32 * c.tm - 1) / (32 * c.tm));
    c.col_blocks = int((s.plan.C + 31) / 32);
    int64_t base = int64_t(c.row_tiles) * c.col_blocks;
    // long K: wide workgroups (16 waves for up to 32 rows, 8 for up to 64), so that one split per
    // tile is enough to keep the weight stream busy and no reduction pass is needed
    c.nw = nks >= 64 ? 8 : 4;
    int64_t target_wgs = 3072 / c.nw;
    int want = int(std::max<int64_t>(1, target_wgs / base));
    int max_split = std::max(1, nks / (2 * c.nw));      // at least 2 k-steps per wave
    c.nsplit = std::min(want, max_split);
    for (;;) {
        c.ksteps_per_split = (nks + c.nsplit - 1) / c.nsplit;
        c.nsplit = (nks + c.ksteps_per_split - 1) / c.ksteps_per_split;      // no empty split
        c.partial_bytes = c.nsplit > 1 ? int64_t(c.nsplit) * c.row_tiles * 32 * c.tm * s.Cp * 4 : 0;
        if (c.partial_bytes <= kMaxPartialBytes || c.nsplit == 1) break;
        c.nsplit = std::max(1, c.nsplit / 2);
    }
    c.use = true;
    return c;
}

template <int WM, int WN, int TM, int TN>
void launch_mfma(const DevStep& s, const StepArgs& a, dim3 grid, hipStream_t st) {
    if (s.amode == 0)
        hipLaunchKernelGGL((step_mfma_kernel<WM, WN, TM, TN, 0>), grid, dim3(256), 0, st, a, s.cmode);
    else
        hipLaunchKernelGGL((step_mfma_kernel<WM, WN, TM, TN, 1>), grid, dim3(256), 0, st, a, s.cmode);
}

template <int WM, int WN, int TM, int TN, int STAGES, int MINB>
int launch_pipe(const DevStep& s, const StepArgs& a, int64_t rows, hipStream_t st) {
    constexpr int BM = WM * TM * 32, BN = WN * TN * 32;
    constexpr size_t smem = pipe_smem_bytes<WM, WN, TM, TN, STAGES>();
    int nrow = int((rows + BM - 1) / BM), ncol = s.Cp / BN;
    int nrow_pad = (nrow + 7) / 8 * 8;
    dim3 grid(uint32_t(nrow_pad) * uint32_t(ncol));
    using kern_t = void (*)(StepArgs, int, int, int);
    static const kern_t kerns[4] = {
        step_mfma_pipe_kernel<WM, WN, TM, TN, 0, STAGES, MINB, 0>, step_mfma_pipe_kernel<WM, WN, TM, TN, 1, STAGES, MINB, 0>,
        step_mfma_pipe_kernel<WM, WN, TM, TN, 0, STAGES, MINB, 1>, step_mfma_pipe_kernel<WM, WN, TM, TN, 1, STAGES, MINB, 1>};
    if (!s.packed) {                       // configuration call (create time): raise the kernels' LDS limit
        for (kern_t k : kerns)
            if (hipFuncSetAttribute(reinterpret_cast<const void*>(k), hipFuncAttributeMaxDynamicSharedMemorySize,
                                    int(smem)) != hipSuccess)
                return TN_ERR_HIP;
        return TN_OK;
    }
    kern_t k = kerns[(s.cmode == 2 ? 2 : 0) + (s.amode == 0 ? 0 : 1)];
    hipLaunchKernelGGL(k, grid, dim3(WM * WN * 64), smem, st, a, s.cmode, nrow, ncol);
    return TN_OK;
}

template <int WM, int WN, int TM, int TN, int NS, int MINB>
int launch_dlds(const DevStep& s, const StepArgs& a, int64_t rows, hipStream_t st) {
    constexpr int BM = WM * TM * 32, BN = WN * TN * 32;
    constexpr size_t smem = dlds_smem_bytes<WM, WN, TM, TN, NS>();
    int nrow = int((rows + BM - 1) / BM), ncol = s.Cp / BN;
    int nrow_pad = (nrow + 7) / 8 * 8;
    dim3 grid(uint32_t(nrow_pad) * uint32_t(ncol));
    using kern_t = void (*)(StepArgs, int, int, int);
    static const kern_t kerns[2] = {step_mfma_dlds_kernel<WM, WN, TM, TN, NS, MINB, 0>,
                                    step_mfma_dlds_kernel<WM, WN, TM, TN, NS, MINB, 1>};
    if (!s.packed) {                       // configuration call (create time)
        for (kern_t k : kerns)
            if (hipFuncSetAttribute(reinterpret_cast<const void*>(k), hipFuncAttributeMaxDynamicSharedMemorySize,
                                    int(smem)) != hipSuccess)
                return TN_ERR_HIP;
        return TN_OK;
    }
    hipLaunchKernelGGL(kerns[s.cmode == 2 ? 1 : 0], grid, dim3(WM * WN * 64), smem, st, a, s.cmode, nrow, ncol);
    return TN_OK;
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
    SplitCfg sc = (h->flags & TN_FLAG_NO_SPLIT_K) ? SplitCfg() : split_config(s, rows);
    if (sc.use && (sc.partial_bytes == 0 || (h->partial && sc.partial_bytes <= h->partial_bytes))) {
        dim3 sgrid(uint32_t(sc.row_tiles), uint32_t(sc.col_blocks), uint32_t(sc.nsplit));
        float* part = static_cast<float*>(h->partial);
        using split_t = void (*)(StepArgs, float*, int);
        split_t k;
        if (sc.tm == 1)
            k = sc.nw == 8 ? (s.amode == 0 ? step_split_kernel<1, 0, 8> : step_split_kernel<1, 1, 8>)
                           : (s.amode == 0 ? step_split_kernel<1, 0, 4> : step_split_kernel<1, 1, 4>);
        else
            k = sc.nw == 8 ? (s.amode == 0 ? step_split_kernel<2, 0, 8> : step_split_kernel<2, 1, 8>)
                           : (s.amode == 0 ? step_split_kernel<2, 0, 4> : step_split_kernel<2, 1, 4>);
        hipLaunchKernelGGL(k, sgrid, dim3(uint32_t(sc.nw * 64)), 0, st, a, part, sc.ksteps_per_split);
        if (sc.nsplit > 1) {
            int64_t total = rows * s.plan.C;
            uint32_t blocks = uint32_t(std::min<int64_t>((total + 255) / 256, 2048));
            hipLaunchKernelGGL(step_split_reduce_kernel, dim3(blocks), dim3(256), 0, st, a, part, sc.nsplit,
                               uint32_t(sc.row_tiles * 32 * sc.tm));
        }
        return hipGetLastError() == hipSuccess ? TN_OK : TN_ERR_HIP;
    }
    dim3 grid(uint32_t((rows + s.bm - 1) / s.bm), uint32_t(s.Cp / s.bn));
    switch (s.variant) {
        case VAR_SCALAR:
            if (h->plan.dtype == TN_DTYPE_BF16)
                hipLaunchKernelGGL(step_scalar_kernel<bf16_t>, grid, dim3(256), 0, st, a);
            else
                hipLaunchKernelGGL(step_scalar_kernel<float>, grid, dim3(256), 0, st, a);
            break;
        case VAR_MFMA_256x32:
            launch_mfma<4, 1, 2, 1>(s, a, grid, st);
            break;
        case VAR_PIPE_128x256: {
            int rc = launch_pipe<2, 2, 2, 4, 1, 2>(s, a, rows, st);
            if (rc != TN_OK) return rc;
            break;
        }
        case VAR_DLDS8_256x256: {
            int rc = launch_dlds<4, 2, 2, 4, 4, 1>(s, a, rows, st);
            if (rc != TN_OK) return rc;
            break;
        }
        case VAR_SHORTK: {
            // forms (tuning override in flag bits 16..19, value = form + 1): 0 = 64 rows per wave with
            // double-buffered packed fragments, 1 = 64 rows single-buffered, 2 = 32 rows single-buffered
            if (tokens * s.plan.c_tok_stride >= (int64_t(1) << 35)) {
                // output offsets would not fit the kernel's 32-bit (x8) row bases: use the tiled kernel
                int rc = launch_pipe<4, 1, 2, 4, 1, 2>(s, a, rows, st);
                if (rc != TN_OK) return rc;
                break;
            }
            // measured: 32 rows per wave at 4 workgroups per CU streams best when A is a plain matrix
            // (4.7 TB/s stored); with a gathered A the 64-row double-buffered form is slightly ahead
            int mode = (h->flags >> 16) & 0xf;
            mode = mode ? mode - 1 : (s.amode == 0 ? 2 : 0);
            const int wrows = mode == 2 ? 32 : 64;
            int64_t row_tiles = (rows + 2 * wrows - 1) / (2 * wrows);
            int col_iters = s.Cp / 128;
            int groups = int(std::min<int64_t>(col_iters, std::max<int64_t>(1, 1024 / row_tiles)));
            dim3 g{uint32_t(row_tiles), uint32_t(groups)};
            using k_t = void (*)(StepArgs);
            k_t k;
            if (mode == 2)
                k = s.amode == 0 ? step_shortk_kernel<0, 1, 0, 4> : step_shortk_kernel<1, 1, 0, 4>;
            else if (mode == 1)
                k = s.amode == 0 ? step_shortk_kernel<0, 2, 0, 3> : step_shortk_kernel<1, 2, 0, 3>;
            else
                k = s.amode == 0 ? step_shortk_kernel<0, 2, 1, 2> : step_shortk_kernel<1, 2, 1, 2>;
            hipLaunchKernelGGL(k, g, dim3(256), 0, st, a);
            break;
        }
        case VAR_PIPE_256x128: {
            int rc = launch_pipe<4, 1, 2, 4, 1, 2>(s, a, rows, st);
            if (rc != TN_OK) return rc;
            break;
        }
        default:
            return TN_ERR_UNSUPPORTED;
    }
    return hipGetLastError() == hipSuccess ? TN_OK : TN_ERR_HIP;
}

// Can steps s and s+1 run as one fused launch? (small per-token tensors, k-steps without padding)
void plan_fusion(tn_linear_s* h) {
    // opt-in: measured slower than the two separate launches on MI355X (the per-token work is a
    // chain of small dependent LDS reads and MFMAs that 8 waves per CU cannot overlap)
    if (h->plan.dtype != TN_DTYPE_BF16 || (h->flags & TN_FLAG_SCALAR_KERNELS) || !(h->flags & TN_FLAG_FUSE_SMALL_STEPS)) return;
    for (size_t s = 0; s + 1 < h->steps.size(); ++s) {
        DevStep& a = h->steps[s];
        DevStep& b = h->steps[s + 1];
        if (s > 0 && h->steps[s - 1].fuse_next) continue;
        const tn::Step& p1 = a.plan;
        const tn::Step& p2 = b.plan;
        if (!p1.a_plain || !p2.a_plain || p1.K % 16 || p2.K % 16) continue;
        if (p1.K > 96 || p2.K > 96 || p1.C > 256 || p2.C > 256) continue;      // register-resident packed tensors
        if (p1.R * p1.K > 12288) continue;                                      // register-prefetched input
        if (p1.c_tok_stride != p2.R * p2.K) continue;
        int64_t in_elems = int64_t((p1.R + 31) / 32 * 32) * (p1.K + 8);
        int64_t mid_elems = int64_t((p2.R + 31) / 32 * 32) * p2.K;
        int64_t tab = p1.R + p1.C + p2.R + p2.C;
        int64_t smem = (in_elems + mid_elems + 4 * 32 * 40) * 2 + tab * 4 + 64;
        if (smem > 72 * 1024) continue;
        if (int64_t(a.Cp) * a.Kp > 65536 || int64_t(b.Cp) * b.Kp > 65536) continue;
        a.fuse_next = true;
        a.fuse_kind = 1;
        a.fused_in_elems = int(in_elems);
        a.fused_mid_elems = int((mid_elems + 7) / 8 * 8);
        a.fused_smem = size_t((a.fused_in_elems + a.fused_mid_elems + 4 * 32 * 40) * 2 + tab * 4 + 64);
    }
}

void fill_args(const DevStep& s, const void* A, void* Out, int64_t tokens, StepArgs* a) {
    a->A = A;
    a->B = s.packed;
    a->Out = Out;
    a->arow = s.arow;
    a->acol = s.acol;
    a->crow = s.crow;
    a->ccol = s.ccol;
    a->a_tok_stride = s.plan.a_tok_stride;
    a->c_tok_stride = s.plan.c_tok_stride;
    a->total_rows = uint32_t(tokens * s.plan.R);
    a->R = uint32_t(s.plan.R);
    a->K = int32_t(s.plan.K);
    a->Kp = s.Kp;
    a->C = int32_t(s.plan.C);
    a->Cp = s.Cp;
}

int launch_fused2(const DevStep& s1, const DevStep& s2, const void* A, void* Out, int64_t tokens, hipStream_t st) {
    Fused2Args f;
    fill_args(s1, A, nullptr, tokens, &f.s1);
    fill_args(s2, nullptr, Out, tokens, &f.s2);
    f.tokens = int32_t(tokens);
    f.in_elems = s1.fused_in_elems;
    f.mid_elems = s1.fused_mid_elems;
    dim3 grid(uint32_t(std::min<int64_t>(tokens, 1024)));
    if (s2.cmode == 1)
        hipLaunchKernelGGL(step_fused2_kernel<1>, grid, dim3(256), s1.fused_smem, st, f);
    else
        hipLaunchKernelGGL(step_fused2_kernel<0>, grid, dim3(256), s1.fused_smem, st, f);
    return hipGetLastError() == hipSuccess ? TN_OK : TN_ERR_HIP;
}

// Token count from which the chained pair kernel replaces the two separate launches (below it a
// launch has too few workgroups: 8 per 32 tokens).
constexpr int64_t kPairMinTokens = 256;
constexpr int kPairStages = 4;
constexpr size_t kPairSmemBytes = kPairStages * 20 * 1024;

int prepare_pair(tn_linear_s* h, hipStream_t st) {
    if ((h->flags & (TN_FLAG_NO_PAIR_CHAIN | TN_FLAG_SCALAR_KERNELS)) || !tn::pair_chainable(h->plan)) return TN_OK;
    const DevStep& s0 = h->steps[0];
    const DevStep& s1 = h->steps[1];
    if (s0.Kp != 64 || s0.Cp < s0.plan.C || s1.Kp != s1.plan.K) return TN_OK;
    const int A = int(s0.plan.R);
    if (hipMalloc(&h->pair_b1f, size_t(A) * 8192 * sizeof(bf16_t)) != hipSuccess) return TN_ERR_ALLOC;
    h->packed_bytes += int64_t(A) * 8192 * int64_t(sizeof(bf16_t));
    uint32_t blocks = uint32_t(std::min<int64_t>((int64_t(A) * 8192 + 255) / 256, 4096));
    hipLaunchKernelGGL(pair_repack_kernel, dim3(blocks), dim3(256), 0, st, static_cast<const bf16_t*>(s1.packed),
                       static_cast<bf16_t*>(h->pair_b1f), A, s1.Kp >> 4, s1.Cp);
    if (hipGetLastError() != hipSuccess) return TN_ERR_HIP;
    h->pair = true;
    h->pair_min_tokens = kPairMinTokens;
    return TN_OK;
}

int launch_pair(const tn_linear_s* h, const void* x, void* y, int64_t tokens, hipStream_t st) {
    const DevStep& s0 = h->steps[0];
    const DevStep& s1 = h->steps[1];
    PairArgs p;
    p.X = x;
    p.Y = y;
    p.B0 = s0.packed;
    p.B1f = h->pair_b1f;
    p.yrow = s1.crow;
    p.ycol = s1.ccol;
    p.N = h->plan.N;
    p.M = h->plan.M;
    p.tokens = int32_t(tokens);
    p.A = int32_t(s0.plan.R);
    p.J = int32_t(s1.plan.R);
    p.C1 = int32_t(s1.plan.C);
    p.n_tok_tiles = int32_t((tokens + 31) / 32);
    p.n_jsets = p.J / 8;
    int64_t grid = int64_t((p.n_tok_tiles + 7) / 8 * 8) * p.n_jsets;
    hipLaunchKernelGGL(step_pair_kernel<kPairStages>, dim3(uint32_t(grid)), dim3(256), kPairSmemBytes, st, p);
    return hipGetLastError() == hipSuccess ? TN_OK : TN_ERR_HIP;
}

// Pairs of steps the transposing chain kernel can run (see step_chain2_kernel): both plain, the
// first step's output stored transposed ([c1][r], which is what the second step reads as rows c1
// with K = r), the output in aligned runs of 8 along c1 or along c2, and sizes within one of the
// two instantiations.
int plan_chain2(tn_linear_s* h, hipStream_t st) {
    if (h->plan.dtype != TN_DTYPE_BF16 || (h->flags & (TN_FLAG_SCALAR_KERNELS | TN_FLAG_NO_CHAIN2 | TN_FLAG_FUSE_SMALL_STEPS)) ||
        h->pair)
        return TN_OK;
    for (size_t i = 0; i + 1 < h->steps.size(); ++i) {
        DevStep& a = h->steps[i];
        DevStep& b = h->steps[i + 1];
        if (i > 0 && h->steps[i - 1].fuse_next) continue;
        if (a.variant == VAR_SCALAR || b.variant == VAR_SCALAR) continue;
        int cfg = 0, run_c1 = 0;
        if (!tn::chain2_shape(h->plan, a.plan, b.plan, &cfg, &run_c1)) continue;
        const int C2T = cfg == 0 ? 5 : 2, KS = cfg == 0 ? 6 : 4;
        size_t elems = size_t(C2T) * KS * 512;
        if (hipMalloc(&a.chain_bbf, elems * sizeof(bf16_t)) != hipSuccess) return TN_ERR_ALLOC;
        h->packed_bytes += int64_t(elems * sizeof(bf16_t));
        hipLaunchKernelGGL(chain2_repack_kernel, dim3(uint32_t((elems + 255) / 256)), dim3(256), 0, st,
                           static_cast<const bf16_t*>(b.packed), static_cast<bf16_t*>(a.chain_bbf), C2T, KS, b.Kp >> 4,
                           b.Cp, b.Kp);
        if (hipGetLastError() != hipSuccess) return TN_ERR_HIP;
        a.fuse_next = true;
        a.fuse_kind = 2;
        a.chain_cfg = cfg;
        a.chain_run_c1 = run_c1;
    }
    return TN_OK;
}

int launch_chain2(const tn_linear_s* h, const DevStep& s1, const DevStep& s2, const void* A, void* Out, int64_t tokens,
                  hipStream_t st) {
    using k_t = void (*)(Chain2Args);
    static const k_t kerns[4] = {step_chain2_kernel<3, 6, 5, 0>, step_chain2_kernel<3, 6, 5, 1>,
                                 step_chain2_kernel<2, 8, 2, 0>, step_chain2_kernel<2, 8, 2, 1>};
    static const size_t smem[2] = {chain2_smem_bytes<3, 6, 5>(), chain2_smem_bytes<2, 8, 2>()};
    if (!s1.packed) {                      // configuration call (create time)
        for (int i = 0; i < 4; ++i)
            if (hipFuncSetAttribute(reinterpret_cast<const void*>(kerns[i]), hipFuncAttributeMaxDynamicSharedMemorySize,
                                    int(smem[i / 2])) != hipSuccess)
                return TN_ERR_HIP;
        return TN_OK;
    }
    Chain2Args p;
    p.In = A;
    p.Out = Out;
    p.Ba = s1.packed;
    p.Bbf = s1.chain_bbf;
    p.off1 = s2.crow;
    p.off2 = s2.ccol;
    p.in_tok_stride = s1.plan.a_tok_stride;
    p.out_tok_stride = s2.plan.c_tok_stride;
    p.tokens = int32_t(tokens);
    p.R1 = int32_t(s1.plan.R);
    p.K1 = int32_t(s1.plan.K);
    p.C1 = int32_t(s1.plan.C);
    p.C2 = int32_t(s2.plan.C);
    p.nks_a = s1.Kp >> 4;
    p.c1_tiles = (p.C1 + 31) / 32;
    // a wave per token when there are tokens enough to fill the chip, else a wave per (token, c1 tile)
    const int64_t waves = int64_t(h->num_cus) * 4;
    p.tiles_per_item = tokens >= waves ? p.c1_tiles : 1;
    const int64_t n_groups = (p.c1_tiles + p.tiles_per_item - 1) / p.tiles_per_item;
    const int64_t items = tokens * n_groups;
    dim3 grid(uint32_t(std::min<int64_t>((items + 3) / 4, h->num_cus)));
    hipLaunchKernelGGL(kerns[s1.chain_cfg * 2 + s1.chain_run_c1], grid, dim3(256), smem[s1.chain_cfg], st, p);
    return hipGetLastError() == hipSuccess ? TN_OK : TN_ERR_HIP;
}

// Kernels that use more than 64 KB of LDS need their limit raised once per device. Done at create
// time (never inside tn_linear_forward, which must stay legal under stream capture from its first
// call). The launchers double as configurators: called with an empty step they set the attribute of
// every kernel they can launch and return.
int configure_kernels(int device) {
    static bool done[64] = {};
    if (device >= 0 && device < 64 && done[device]) return TN_OK;
    const DevStep none;                    // packed == nullptr: configuration call
    const StepArgs a{};
    const tn_linear_s* no_handle = nullptr;
    int rc = launch_pipe<2, 2, 2, 4, 1, 2>(none, a, 0, nullptr);
    if (rc == TN_OK) rc = launch_pipe<4, 1, 2, 4, 1, 2>(none, a, 0, nullptr);
    if (rc == TN_OK) rc = launch_dlds<4, 2, 2, 4, 4, 1>(none, a, 0, nullptr);
    if (rc == TN_OK) rc = launch_chain2(no_handle, none, none, nullptr, nullptr, 0, nullptr);
    if (rc == TN_OK &&
        (hipFuncSetAttribute(reinterpret_cast<const void*>(step_fused2_kernel<0>),
                             hipFuncAttributeMaxDynamicSharedMemorySize, 72 * 1024) != hipSuccess ||
         hipFuncSetAttribute(reinterpret_cast<const void*>(step_fused2_kernel<1>),
                             hipFuncAttributeMaxDynamicSharedMemorySize, 72 * 1024) != hipSuccess ||
         hipFuncSetAttribute(reinterpret_cast<const void*>(step_pair_kernel<kPairStages>),
                             hipFuncAttributeMaxDynamicSharedMemorySize, int(kPairSmemBytes)) != hipSuccess))
        rc = TN_ERR_HIP;
    if (rc == TN_OK && device >= 0 && device < 64) done[device] = true;
    return rc;
}

int plan_value(const tn::Plan& p, int32_t what, int64_t* value) {
    switch (what) {
        case TN_QUERY_PARAM_COUNT: *value = p.params; return TN_OK;
        case TN_QUERY_FLOPS_PER_TOKEN: *value = p.flops; return TN_OK;
        case TN_QUERY_NUM_STEPS: *value = int64_t(p.steps.size()); return TN_OK;
        case TN_QUERY_MAX_INTERMEDIATE: *value = p.max_intermediate; return TN_OK;
        case TN_QUERY_OUT_FEATURES: *value = p.M; return TN_OK;
        case TN_QUERY_IN_FEATURES: *value = p.N; return TN_OK;
        case TN_QUERY_NUM_MERGES: *value = int64_t(p.merges.size()); return TN_OK;
        case TN_QUERY_PAIR_CHAINABLE: *value = tn::pair_chainable(p) ? 1 : 0; return TN_OK;
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
            case 7: {
                int cfg = 0, run_c1 = 0;
                *value = (size_t(s) + 1 < p.steps.size() && !tn::pair_chainable(p) &&
                          tn::chain2_shape(p, st, p.steps[size_t(s) + 1], &cfg, &run_c1)) ? 1 + cfg : 0;
                return TN_OK;
            }
            default: return TN_ERR_INVALID_ARG;
        }
    }
    return TN_ERR_INVALID_ARG;
}

// Offsets of every flat index over `dims` (outer -> inner) as an int32 table.
std::vector<int32_t> gather_table(const std::vector<tn::GatherDim>& dims, int64_t total) {
    std::vector<int32_t> tab(static_cast<size_t>(total));
    for (int64_t f = 0; f < total; ++f) {
        int64_t off = 0, rem = f;
        for (int j = int(dims.size()) - 1; j >= 0; --j) {
            off += (rem % dims[size_t(j)].extent) * dims[size_t(j)].stride;
            rem /= dims[size_t(j)].extent;
        }
        tab[size_t(f)] = int32_t(off);
    }
    return tab;
}

void fill_pack_dims(PackArgs* pa, const std::vector<tn::GatherDim>& kd, const std::vector<tn::GatherDim>& cd) {
    pa->nk = int32_t(kd.size());
    pa->nc = int32_t(cd.size());
    for (int j = 0; j < pa->nk; ++j) {
        pa->kext[j] = kd[size_t(j)].extent;
        pa->kstr[j] = kd[size_t(j)].stride;
    }
    for (int j = 0; j < pa->nc; ++j) {
        pa->cext[j] = cd[size_t(j)].extent;
        pa->cstr[j] = cd[size_t(j)].stride;
    }
}

void launch_pack(const PackArgs& pa, int elt, hipStream_t st) {
    int64_t total = int64_t(pa.Cp) * pa.Kp;
    uint32_t blocks = uint32_t(std::min<int64_t>((total + 255) / 256, 65535));
    if (elt == 2)
        hipLaunchKernelGGL(pack_kernel<bf16_t>, dim3(blocks), dim3(256), 0, st, pa);
    else
        hipLaunchKernelGGL(pack_kernel<float>, dim3(blocks), dim3(256), 0, st, pa);
}

// Contract pairs of parameter tensors at create time (tn::MergeOp) with the plain FMA kernel
// (fp32 accumulate, one rounding to the storage type). `virt` receives one device buffer per merge;
// `temps` receives scratch buffers the caller frees once the stream has drained.
int materialise_merges(const tn::Plan& plan, const tn_linear_desc* desc, int elt, hipStream_t st,
                       std::vector<void*>* virt, std::vector<void*>* temps) {
    auto source = [&](int slot) -> const void* {
        return slot < plan.n_caller_tensors ? desc->tensors[slot] : (*virt)[size_t(slot - plan.n_caller_tensors)];
    };
    for (const tn::MergeOp& m : plan.merges) {
        void* out = nullptr;
        if (hipMalloc(&out, size_t(m.R * m.C) * elt) != hipSuccess) return TN_ERR_ALLOC;
        virt->push_back(out);
        int Kp = round_up(int(m.K), 64), Cp = round_up(int(m.C), 64);
        void* packed = nullptr;
        if (hipMalloc(&packed, size_t(Kp) * Cp * elt) != hipSuccess) return TN_ERR_ALLOC;
        temps->push_back(packed);
        PackArgs pa;
        memset(&pa, 0, sizeof(pa));
        pa.src = source(m.q_slot);
        pa.dst = packed;
        pa.K = int32_t(m.K);
        pa.Kp = Kp;
        pa.C = int32_t(m.C);
        pa.Cp = Cp;
        fill_pack_dims(&pa, m.kq, m.cdims);
        pa.trace_extent = 1;
        launch_pack(pa, elt, st);
        // tables: arow | acol | crow | ccol
        std::vector<int32_t> tab = gather_table(m.rdims, m.R);
        std::vector<int32_t> acol = gather_table(m.kp, m.K);
        tab.insert(tab.end(), acol.begin(), acol.end());
        for (int64_t r = 0; r < m.R; ++r) tab.push_back(int32_t(r * m.C));
        for (int64_t c = 0; c < m.C; ++c) tab.push_back(int32_t(c));
        int32_t* dtab = nullptr;
        if (hipMalloc(reinterpret_cast<void**>(&dtab), tab.size() * sizeof(int32_t)) != hipSuccess) return TN_ERR_ALLOC;
        temps->push_back(dtab);
        if (hipMemcpyAsync(dtab, tab.data(), tab.size() * sizeof(int32_t), hipMemcpyHostToDevice, st) != hipSuccess ||
            hipStreamSynchronize(st) != hipSuccess)
            return TN_ERR_HIP;
        StepArgs a;
        a.A = source(m.p_slot);
        a.B = packed;
        a.Out = out;
        a.arow = dtab;
        a.acol = dtab + m.R;
        a.crow = dtab + m.R + m.K;
        a.ccol = dtab + m.R + m.K + m.R;
        a.a_tok_stride = 0;
        a.c_tok_stride = 0;
        a.total_rows = uint32_t(m.R);
        a.R = uint32_t(m.R);
        a.K = int32_t(m.K);
        a.Kp = Kp;
        a.C = int32_t(m.C);
        a.Cp = Cp;
        dim3 grid(uint32_t((m.R + 63) / 64), uint32_t(Cp / 64));
        if (elt == 2)
            hipLaunchKernelGGL(step_scalar_kernel<bf16_t>, grid, dim3(256), 0, st, a);
        else
            hipLaunchKernelGGL(step_scalar_kernel<float>, grid, dim3(256), 0, st, a);
        if (hipGetLastError() != hipSuccess) return TN_ERR_HIP;
    }
    return TN_OK;
}

}  // namespace

extern "C" {

int tn_linear_version(void) { return 2; }

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
    if (what >= TN_QUERY_STEP_BASE && (what - TN_QUERY_STEP_BASE) % 10 >= 5 &&
        (what - TN_QUERY_STEP_BASE) % 10 <= 6) {
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
        h->num_cus = std::max(1, prop.multiProcessorCount);
        if (configure_kernels(h->device) != TN_OK) {
            delete h;
            return TN_ERR_HIP;
        }
    }
    hipStream_t st = static_cast<hipStream_t>(desc->stream);
    h->elt = desc->dtype == TN_DTYPE_BF16 ? 2 : 4;
    h->max_tokens = desc->max_tokens;
    h->flags = desc->flags;
    h->steps.resize(h->plan.steps.size());
    std::vector<void*> virt, temps;     // merged tensors and scratch: freed before create returns
    auto release_temps = [&]() {
        for (void* v : virt) (void)hipFree(v);
        for (void* v : temps) (void)hipFree(v);
    };
    rc = materialise_merges(h->plan, desc, h->elt, st, &virt, &temps);
    if (rc != TN_OK) {
        (void)hipStreamSynchronize(st);
        release_temps();
        free_handle(h);
        return rc;
    }
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
            (void)hipStreamSynchronize(st);
            release_temps();
            free_handle(h);
            return TN_ERR_ALLOC;
        }
        // pageable source: the copy is staged before the call returns, so host_tab may go away
        if (hipMemcpyAsync(s.tables, host_tab.data(), n_tab * sizeof(int32_t), hipMemcpyHostToDevice, st) !=
            hipSuccess) {
            (void)hipStreamSynchronize(st);
            release_temps();
            free_handle(h);
            return TN_ERR_HIP;
        }
        if (hipStreamSynchronize(st) != hipSuccess) {
            (void)hipStreamSynchronize(st);
            release_temps();
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
            (void)hipStreamSynchronize(st);
            release_temps();
            free_handle(h);
            return TN_ERR_ALLOC;
        }
        h->packed_bytes += bytes;
        PackArgs pa;
        memset(&pa, 0, sizeof(pa));
        pa.src = p.slot < h->plan.n_caller_tensors ? desc->tensors[p.slot]
                                                    : virt[size_t(p.slot - h->plan.n_caller_tensors)];
        pa.dst = s.packed;
        pa.K = int32_t(p.K);
        pa.Kp = s.Kp;
        pa.C = int32_t(p.C);
        pa.Cp = s.Cp;
        fill_pack_dims(&pa, p.kdims, p.cdims);
        pa.trace_extent = p.trace_extent;
        pa.trace_stride = p.trace_stride;
        launch_pack(pa, h->elt, st);
        if (hipGetLastError() != hipSuccess) {
            (void)hipStreamSynchronize(st);
            release_temps();
            free_handle(h);
            return TN_ERR_HIP;
        }
    }
    if (!virt.empty() || !temps.empty()) {
        // the pack kernels read the merged tensors: wait for them before the buffers go away
        if (hipStreamSynchronize(st) != hipSuccess) {
            release_temps();
            free_handle(h);
            return TN_ERR_HIP;
        }
        release_temps();
    }
    plan_fusion(h);
    rc = prepare_pair(h, st);
    if (rc == TN_OK) rc = plan_chain2(h, st);
    if (rc != TN_OK) {
        (void)hipStreamSynchronize(st);
        free_handle(h);
        return rc;
    }
    // workspace: two ping-pong buffers, each chunk_tokens * max_intermediate elements, and the
    // partial-sum buffer of the split-K kernel; allocated here, or carved out of the caller's block
    int64_t per_token = h->plan.max_intermediate * h->elt;
    int64_t max_r = 1;
    for (const auto& s : h->steps) max_r = std::max(max_r, s.plan.R);
    const int64_t row_cap = ((int64_t(1) << 31) - 1024) / max_r;      // rows of a pass are indexed with 32 bits
    const bool split_ok = !(desc->flags & TN_FLAG_NO_SPLIT_K) && h->elt == 2;
    auto partial_need = [&](int64_t chunk) {
        int64_t need = 0;
        if (!split_ok) return need;
        for (const auto& s : h->steps)
            for (int64_t t = 1; t <= chunk; ++t) {
                SplitCfg c = split_config(s, t * s.plan.R);
                if (!c.use) break;          // larger passes only add tiles
                need = std::max(need, c.partial_bytes);
            }
        return need;
    };
    // with the chained pair kernel only calls below its token threshold use the workspace
    const int64_t ws_tokens = h->pair ? std::min<int64_t>(h->max_tokens, h->pair_min_tokens - 1) : h->max_tokens;
    int64_t chunk = ws_tokens;
    if (desc->workspace) {
        // caller-owned block: [partial sums | buffer 0 | buffer 1], 256-byte aligned pieces
        h->owns_workspace = false;
        char* base = static_cast<char*>(desc->workspace);
        int64_t avail = desc->workspace_bytes;
        int64_t part = split_ok ? std::min<int64_t>(kMaxPartialBytes, avail / 4) & ~int64_t(255) : 0;
        int64_t half = ((avail - part) / 2) & ~int64_t(255);
        if (per_token > 0) {
            chunk = std::min<int64_t>(std::min<int64_t>(ws_tokens, half / per_token), row_cap);
            if (chunk < 1) {
                free_handle(h);
                return TN_ERR_INVALID_ARG;      // the block cannot hold one token's intermediates
            }
            h->ws[0] = base + part;
            h->ws[1] = base + part + half;
        } else {
            chunk = std::max<int64_t>(1, std::min<int64_t>(chunk, row_cap));
        }
        if (part > 0) {
            h->partial = base;
            h->partial_bytes = part;
        }
        h->workspace_bytes = 0;
    } else {
        int64_t limit = desc->workspace_limit_bytes > 0 ? desc->workspace_limit_bytes : kDefaultWorkspaceBytes;
        if (per_token > 0) {
            chunk = std::max<int64_t>(1, std::min<int64_t>(ws_tokens, limit / (2 * per_token)));
            chunk = std::max<int64_t>(1, std::min<int64_t>(chunk, row_cap));
            for (int b = 0; b < 2; ++b) {
                if (hipMalloc(&h->ws[b], size_t(chunk * per_token)) != hipSuccess) {
                    free_handle(h);
                    return TN_ERR_ALLOC;
                }
            }
            h->workspace_bytes = 2 * chunk * per_token;
        } else {
            chunk = std::max<int64_t>(1, std::min<int64_t>(chunk, row_cap));
        }
        int64_t need = partial_need(chunk);
        if (need > 0) {
            if (hipMalloc(&h->partial, size_t(need)) != hipSuccess) {
                free_handle(h);
                return TN_ERR_ALLOC;
            }
            h->partial_bytes = need;
            h->workspace_bytes += need;
        }
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
    if (h->pair && tokens >= h->pair_min_tokens) {
        // both steps in one launch, no intermediate in memory; passes only bound the 32-bit token index
        const int64_t pass = int64_t(1) << 24;
        for (int64_t t0 = 0; t0 < tokens; t0 += pass) {
            int64_t nt = std::min(pass, tokens - t0);
            tn_linear_s::ProfRec rec{0, nullptr, nullptr};
            if (h->profiling) {
                if (hipEventCreate(&rec.start) != hipSuccess || hipEventCreate(&rec.stop) != hipSuccess)
                    return TN_ERR_HIP;
                (void)hipEventRecord(rec.start, st);
            }
            int rc = launch_pair(h, xb + t0 * h->plan.N * h->elt, yb + t0 * h->plan.M * h->elt, nt, st);
            if (h->profiling) {
                (void)hipEventRecord(rec.stop, st);
                h->prof.push_back(rec);
            }
            if (rc != TN_OK) return rc;
        }
        return TN_OK;
    }
    for (int64_t t0 = 0; t0 < tokens; t0 += h->chunk_tokens) {
        int64_t nt = std::min(h->chunk_tokens, tokens - t0);
        for (size_t s = 0; s < ns; ++s) {
            const bool fused = h->steps[s].fuse_next;
            const size_t so = fused ? s + 1 : s;                 // step whose output this launch writes
            const void* A = (s == 0) ? static_cast<const void*>(xb + t0 * h->plan.N * h->elt) : h->ws[(s - 1) & 1];
            void* Out = (so == ns - 1) ? static_cast<void*>(yb + t0 * h->plan.M * h->elt) : h->ws[so & 1];
            tn_linear_s::ProfRec rec{int(s), nullptr, nullptr};
            if (h->profiling) {
                if (hipEventCreate(&rec.start) != hipSuccess || hipEventCreate(&rec.stop) != hipSuccess)
                    return TN_ERR_HIP;
                (void)hipEventRecord(rec.start, st);
            }
            int rc = !fused ? launch_step(h, h->steps[s], A, Out, nt, st)
                     : h->steps[s].fuse_kind == 2 ? launch_chain2(h, h->steps[s], h->steps[s + 1], A, Out, nt, st)
                                                  : launch_fused2(h->steps[s], h->steps[s + 1], A, Out, nt, st);
            if (h->profiling) {
                (void)hipEventRecord(rec.stop, st);
                h->prof.push_back(rec);
            }
            if (rc != TN_OK) return rc;
            if (fused) ++s;
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
    if (what >= TN_QUERY_STEP_BASE && (what - TN_QUERY_STEP_BASE) % 10 == 6) {
        int s = (what - TN_QUERY_STEP_BASE) / 10;
        if (s >= int(h->steps.size())) return TN_ERR_INVALID_ARG;
        *value = h->steps[size_t(s)].fuse_next ? 1 : ((h->pair && s == 0) ? 2 : 0);
        return TN_OK;
    }
    return plan_value(h->plan, what, value);
}

}  // extern "C"
