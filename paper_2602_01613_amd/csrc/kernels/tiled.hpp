// Tiled contraction-step kernels: plain FMA (any dtype), bf16 MFMA tiles with register prefetch, and the direct-to-LDS ring kernel.
// Part of the tn_linear library's single translation unit: included by tn_linear.hip inside its
// anonymous namespace, after <hip/hip_runtime.h> and tn_plan.hpp.
#pragma once

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
//   AMODE 2 (step_mfma_pipe_kernel only): rows through the tables, the k of a row in aligned contiguous runs of 8
//            (tn::Step::a_vec): 16-byte loads at arow[r] + acol[k]
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
    int64_t a_base[AMODE != 0 ? A_CHUNKS : 1];
    if (AMODE != 0) {
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
            } else if (AMODE == 2) {
                if (a_base[j] >= 0 && k < a.K) v = *reinterpret_cast<const bf16x8*>(A + a_base[j] + a.acol[k]);
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
// Ping-pong bf16 MFMA step kernel (the fastest tiled kernel; needs a plain A with K % 32 == 0, 8 waves).
//   * Two groups of four waves (one wave of each group on every SIMD) run half a period apart: while one group
//     multiplies K tile kt out of registers (16 MFMAs per wave, raised priority), the other fetches its fragments
//     of the next tile from LDS, stores the tile after that into LDS and issues the global loads of the one after,
//     so a SIMD's matrix core always has a wave with work ready. Each wave alternates a memory phase M(kt) and a
//     compute phase C(kt) with a workgroup barrier after each; group 1 passes one barrier more before its first
//     phase and group 0 one more after its last, so all waves execute 2 * nk + 1 barriers in the loop. With the
//     phases numbered so that group 0 runs M(kt) in phase 2kt and group 1 in phase 2kt + 1:
//       - a K tile of 32 travels global memory -> registers (issued in M(kt-1) for tile kt+1, 16 registers per
//         wave) -> LDS stage (kt+1) % NS (written in M(kt)) -> fragments (read in M(kt+1));
//       - that stage is written in phase 2kt at the earliest; its last readers (tile kt+1-NS) finished in phase
//         2(kt+1-NS)+1 < 2kt for NS >= 2, with lgkmcnt(0) before their barrier;
//       - tile kt+1 is written by phase 2kt+1 and read from phase 2kt+2 on.
//     (Measured against the same loop fed by global_load_lds, and against a single-phase loop with one barrier
//     per tile: 6 % faster than either. The barriers of the loop are bare s_barrier: a fence there makes the
//     compiler drain the global loads in flight.)
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
step_mfma_pingpong_kernel(StepArgs a, int cmode, int nrow_tiles, int ncol_tiles, int slot_base, int halves) {
    constexpr int NT = WM * WN * 64, NWAVE = WM * WN;
    constexpr int BM = WM * TM * 32, BN = WN * TN * 32, BK = 32;
    constexpr int ROWB = BK * 2;                       // bytes per LDS tile row
    constexpr int A_BYTES = BM * ROWB, STAGE_BYTES = (BM + BN) * ROWB;
    constexpr int A_PER_WAVE = BM / 16 / NWAVE, B_PER_WAVE = BN / 16 / NWAVE;   // 1 KB loads per wave and stage
    constexpr int L = A_PER_WAVE + B_PER_WAVE;
    constexpr int LDC = BN + 8, LDR = BM + 8;
    static_assert(NWAVE == 8, "two groups of four waves");
    static_assert((BM / 16) % NWAVE == 0 && (BN / 16) % NWAVE == 0, "16-row blocks per wave");
    static_assert(NS >= 2, "a stage is refilled while its neighbour is read");
    extern __shared__ __attribute__((aligned(16))) unsigned char dyn_smem[];

    // A launch covers the tiles of slots slot_base .. of every XCD's walk (see tile_of_workgroup); with
    // halves = 1 the walk is that of tiles twice as wide as this kernel's (ncol_tiles counts those) and two
    // consecutive workgroups of an XCD take the two halves of one of them: the host runs the last, partly
    // filled round of a launch that way, on twice as many workgroups for half as long.
    int row_tile, col_tile;
    {
        const int xcd = blockIdx.x & 7;
        int slot = blockIdx.x >> 3, half = 0;
        if (halves) {
            half = slot & 1;
            slot >>= 1;
        }
        slot += slot_base;
        if (slot >= ((nrow_tiles + 7) >> 3) * ncol_tiles) return;
        tile_of_workgroup((slot << 3) | xcd, nrow_tiles, ncol_tiles, &row_tile, &col_tile);
        if (halves) col_tile = 2 * col_tile + half;
    }
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

    // per-lane sources: lane l of a 1 KB block fills LDS row l/4, chunk position l%4 of the block
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
    bf16x8 stg[L];                                       // the tile on its way from global memory to LDS
    auto load_tile = [&](int kt) {
#pragma unroll
        for (int j = 0; j < A_PER_WAVE; ++j) stg[j] = *reinterpret_cast<const bf16x8*>(a_src[j] + kt * BK);
#pragma unroll
        for (int j = 0; j < B_PER_WAVE; ++j)
            stg[A_PER_WAVE + j] = *reinterpret_cast<const bf16x8*>(b_src[j] + int64_t(kt) * 2 * 512);
    };
    auto store_tile = [&](int stage) {
        unsigned char* sbase = dyn_smem + stage * STAGE_BYTES + lane * 16;
#pragma unroll
        for (int j = 0; j < A_PER_WAVE; ++j) *reinterpret_cast<bf16x8*>(sbase + (j * NWAVE + wave) * 1024) = stg[j];
#pragma unroll
        for (int j = 0; j < B_PER_WAVE; ++j)
            *reinterpret_cast<bf16x8*>(sbase + A_BYTES + (j * NWAVE + wave) * 1024) = stg[A_PER_WAVE + j];
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

    const int nk_real = a.K / BK;                        // K % 32 == 0: only these tiles hold data; B is zero beyond
    const int grp = wave >> 2;
    load_tile(0);
    store_tile(0);
    if (nk_real > 1) load_tile(1);
    __syncthreads();
    bf16x8 af[2][TM], bfr[2][TN];
    if (grp == 1) __builtin_amdgcn_s_barrier();
    for (int kt = 0; kt < nk_real; ++kt) {
        // ---- M(kt)
        const unsigned char* scur = dyn_smem + (kt % NS) * STAGE_BYTES;
#pragma unroll
        for (int ks = 0; ks < 2; ++ks) {
#pragma unroll
            for (int i = 0; i < TM; ++i) af[ks][i] = *reinterpret_cast<const bf16x8*>(scur + a_off[i][ks]);
#pragma unroll
            for (int j = 0; j < TN; ++j) bfr[ks][j] = *reinterpret_cast<const bf16x8*>(scur + b_off[j][ks]);
        }
        if (kt + 1 < nk_real) store_tile((kt + 1) % NS);
        if (kt + 2 < nk_real) load_tile(kt + 2);
        __builtin_amdgcn_sched_barrier(0);
        __builtin_amdgcn_s_waitcnt(0xC07F);              // lgkmcnt(0): fragment reads and tile stores are done
        __builtin_amdgcn_s_barrier();
        __builtin_amdgcn_sched_barrier(0);
        // ---- C(kt)
        __builtin_amdgcn_s_setprio(1);
#pragma unroll
        for (int ks = 0; ks < 2; ++ks)
#pragma unroll
            for (int i = 0; i < TM; ++i)
#pragma unroll
                for (int j = 0; j < TN; ++j)
                    acc[i][j] = TRANS ? __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[ks][i], bfr[ks][j], acc[i][j], 0, 0, 0)
                                      : __builtin_amdgcn_mfma_f32_32x32x16_bf16(bfr[ks][j], af[ks][i], acc[i][j], 0, 0, 0);
        __builtin_amdgcn_s_setprio(0);
        __builtin_amdgcn_sched_barrier(0);
        __builtin_amdgcn_s_barrier();
    }
    if (grp == 0) __builtin_amdgcn_s_barrier();
    __syncthreads();

    // ---- epilogue (see step_mfma_pipe_kernel)
    constexpr size_t C_ELEMS = size_t(BM) * LDC > size_t(BN) * LDR ? size_t(BM) * LDC : size_t(BN) * LDR;
    bf16_t* sC = reinterpret_cast<bf16_t*>(dyn_smem);
    int64_t* sBase = reinterpret_cast<int64_t*>(dyn_smem + C_ELEMS * sizeof(bf16_t));
    int32_t* sCol = reinterpret_cast<int32_t*>(sBase + BM);    // output offsets of the tile's columns (-1: no such column)
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
    // (looked up once per tile: inside the store loops every lookup would sit between two stores)
    for (int cc = tid; cc < BN; cc += NT) sCol[cc] = col0 + cc < a.C ? a.ccol[col0 + cc] : -1;
    __syncthreads();
    constexpr int GROUPS = BM * BN / 8;
    if (TRANS) {
#pragma unroll 4
        for (int e = tid; e < GROUPS; e += NT) {
            int rg = (e % (BM / 8)) * 8, cc = e / (BM / 8);
            int64_t base = sBase[rg];
            const int co = sCol[cc];
            if (base < 0 || co < 0) continue;
            *reinterpret_cast<bf16x8*>(Out + base + co) = *reinterpret_cast<const bf16x8*>(sC + cc * LDR + rg);
        }
    } else if (cmode == 1) {
#pragma unroll 4
        for (int e = tid; e < GROUPS; e += NT) {
            int rr = e / (BN / 8), cg = (e % (BN / 8)) * 8;
            int64_t base = sBase[rr];
            const int co = sCol[cg];
            if (base < 0 || co < 0) continue;
            *reinterpret_cast<bf16x8*>(Out + base + co) = *reinterpret_cast<const bf16x8*>(sC + rr * LDC + cg);
        }
    } else {
        for (int e = tid; e < BM * BN; e += NT) {
            int rr = e / BN, cc = e % BN;
            int64_t base = sBase[rr];
            const int co = sCol[cc];
            if (base < 0 || co < 0) continue;
            Out[base + co] = sC[rr * LDC + cc];
        }
    }
}

template <int WM, int WN, int TM, int TN, int NS>
constexpr size_t pingpong_smem_bytes() {
    constexpr int BM = WM * TM * 32, BN = WN * TN * 32;
    constexpr size_t stage = size_t(BM + BN) * 64 * NS;
    constexpr size_t c_elems = size_t(BM) * (BN + 8) > size_t(BN) * (BM + 8) ? size_t(BM) * (BN + 8) : size_t(BN) * (BM + 8);
    constexpr size_t epi = c_elems * 2 + size_t(BM) * 8 + size_t(BN) * 4;
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

