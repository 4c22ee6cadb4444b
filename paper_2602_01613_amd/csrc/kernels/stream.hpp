// Store-bound and decode-size step kernels: short-K, split-K with its reduction, and the whole-chain kernel for small layers.
// Part of the tn_linear library's single translation unit: included by tn_linear.hip inside its
// anonymous namespace, after <hip/hip_runtime.h> and tn_plan.hpp.
#pragma once

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
// End of a split-K workgroup: the per-wave accumulators are summed through LDS in wave order; with one split the
// result is stored through the scatter tables, else into the fp32 partial buffer.
template <int TM, int NW>
__device__ __forceinline__ void split_finish(const StepArgs& a, float* partial, float* red, const floatx16 (&acc)[TM],
                                             uint32_t row0, int cb, int split, int nsplit, uint32_t rows_pad) {
    bf16_t* Out = static_cast<bf16_t*>(a.Out);
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int v = 0; v < 16; ++v) red[((wave * TM + i) * 16 + v) * 64 + lane] = acc[i][v];
    __syncthreads();
    // operands swapped: lane l, register v holds row l%32, column 8*(v/4) + 4*(l/32) + v%4
    const float* rw = red;
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

// The work of one workgroup (row tile bx, column block cb, split `split` of nsplit). red is NW * TM * 1024 floats of
// LDS. A may be memory or LDS (generic address).
template <int TM, int AMODE, int NW>
__device__ __forceinline__ void split_run(const StepArgs& a, float* partial, int ksteps_per_split, float* red, int bx,
                                          int cb, int split, int nsplit, uint32_t rows_pad) {
    const bf16_t* A = static_cast<const bf16_t*>(a.A);
    const bf16_t* B = static_cast<const bf16_t*>(a.B);
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const uint32_t row0 = uint32_t(bx) * (TM * 32);
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
    split_finish<TM, NW>(a, partial, red, acc, row0, cb, split, nsplit, rows_pad);
}

template <int TM, int AMODE, int NW>
__global__ void __launch_bounds__(NW * 64) step_split_kernel(StepArgs a, float* partial, int ksteps_per_split) {
    __shared__ float red[NW * TM * 1024];
    split_run<TM, AMODE, NW>(a, partial, ksteps_per_split, red, blockIdx.x, blockIdx.y, blockIdx.z, gridDim.z,
                             gridDim.x * (TM * 32));
}

// The same workgroup with the packed tensor read in its 4-bit form (see q4_stream_pack_kernel): a lane's 16-byte load
// is one block of 32 codes, converted in registers to the operands of four k-steps. A wave takes whole pieces of 64 k
// (wave, wave + NW, ...) of its split; ksteps_per_split is a multiple of 4. The weight stream is a quarter of the
// bf16 one, so the pieces in flight per wave are what keeps it busy: UC pieces per batch, two batches in registers.
template <int TM, int AMODE, int NW>
__device__ __forceinline__ void split_run_q4(const StepArgs& a, float* partial, int ksteps_per_split, float* red, int bx,
                                             int cb, int split, int nsplit, uint32_t rows_pad) {
    const bf16_t* A = static_cast<const bf16_t*>(a.A);
    const uint4* Q = static_cast<const uint4*>(a.B);
    const unsigned char* S = static_cast<const unsigned char*>(a.Bs);
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const uint32_t row0 = uint32_t(bx) * (TM * 32);
    const int n_chunks = a.Kp >> 6;
    const int ch_begin = split * (ksteps_per_split >> 2);
    const int ch_end = min(n_chunks, ch_begin + (ksteps_per_split >> 2));

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
    const int64_t piece0 = int64_t(cb) * n_chunks;
    floatx16 acc[TM];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[i][v] = 0.f;

    constexpr int UC = TM == 1 ? 4 : 2;
    auto load_batch = [&](int c0, uint4 (&q)[UC], unsigned (&sc)[UC], bf16x8 (&af)[UC][4][TM]) {
#pragma unroll
        for (int u = 0; u < UC; ++u) {
            const int ch = c0 + NW * u;
            const bool live = ch < ch_end;
            q[u] = make_uint4(0u, 0u, 0u, 0u);
            sc[u] = 0u;
            if (live) {
                q[u] = Q[(piece0 + ch) * 64 + lane];
                sc[u] = S[(piece0 + ch) * 64 + lane];
            }
#pragma unroll
            for (int ks = 0; ks < 4; ++ks) {
                const int k = 64 * ch + 32 * (lane >> 5) + 8 * ks;
#pragma unroll
                for (int i = 0; i < TM; ++i) {
                    bf16x8 v;
#pragma unroll
                    for (int e = 0; e < 8; ++e) v[e] = bf16_t(0.f);
                    if (live && a_base[i] >= 0) {
                        if (AMODE == 0) {
                            if (k < a.K) v = *reinterpret_cast<const bf16x8*>(A + a_base[i] + k);
                        } else {
#pragma unroll
                            for (int e = 0; e < 8; ++e)
                                if (k + e < a.K) v[e] = A[a_base[i] + (a.acol ? a.acol[k + e] : k + e)];
                        }
                    }
                    af[u][ks][i] = v;
                }
            }
        }
    };
    auto multiply = [&](const uint4 (&q)[UC], const unsigned (&sc)[UC], const bf16x8 (&af)[UC][4][TM]) {
#pragma unroll
        for (int u = 0; u < UC; ++u) {
            bf16x8 bf[4];
            q4_dequant_block(q[u], sc[u], bf);
#pragma unroll
            for (int ks = 0; ks < 4; ++ks)
#pragma unroll
                for (int i = 0; i < TM; ++i)
                    acc[i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(bf[ks], af[u][ks][i], acc[i], 0, 0, 0);
        }
    };
    {
        uint4 q0[UC], q1[UC];
        unsigned sc0[UC], sc1[UC];
        bf16x8 af0[UC][4][TM], af1[UC][4][TM];
        constexpr int STEP = NW * UC;
        int c0 = ch_begin + wave;
        load_batch(c0, q0, sc0, af0);                    // batches past the end load nothing and multiply zeros
        for (; c0 < ch_end; c0 += 2 * STEP) {
            load_batch(c0 + STEP, q1, sc1, af1);
            multiply(q0, sc0, af0);
            load_batch(c0 + 2 * STEP, q0, sc0, af0);
            multiply(q1, sc1, af1);
        }
    }
    split_finish<TM, NW>(a, partial, red, acc, row0, cb, split, nsplit, rows_pad);
}

// Split-K with the rows of A in LDS, for launches of one row tile (up to 32 * TM rows: decode, verification
// batches; the host uses TM = 1 only: with two row tiles the splits needed to fit the rows cost more than they save). The rows of A that the workgroup's split needs are copied to LDS once (rows * K-range bf16
// values, x_ld elements per row; the host raises the number of splits until they fit), so that the loop's only
// vector-memory traffic is the parameter stream: a ring of D pieces of 64 k per wave is requested up front and each
// slot is requested again as soon as it has been multiplied, while the other operand comes from LDS on its own
// counter. With A fetched from memory (one 16-byte gather per k-step and row tile, behind which the in-order return
// of loads makes the stream wait) the 4-bit launches ran at a third of the bandwidth. Q4: the stream is the 4-bit form (see q4_stream_pack_kernel), else the fragment-major bf16 tensor.
// The reduction buffer shares the LDS of the rows (they are dead by then).
template <int TM, int AMODE, int NW, int Q4>
__global__ void __launch_bounds__(NW * 64) step_split_lds_kernel(StepArgs a, float* partial, int ksteps_per_split,
                                                                 int x_ld) {
    extern __shared__ __attribute__((aligned(16))) unsigned char dyn_smem[];
    float* red = reinterpret_cast<float*>(dyn_smem);                           // NW x TM x 1024, after the loop
    bf16_t* xs = reinterpret_cast<bf16_t*>(dyn_smem);                          // [rows][x_ld], during the loop
    const bf16_t* A = static_cast<const bf16_t*>(a.A);
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int cb = blockIdx.y, split = blockIdx.z, nsplit = gridDim.z;
    const int n_chunks = a.Kp >> 6;
    const int ch_begin = split * (ksteps_per_split >> 2);
    const int ch_end = min(n_chunks, ch_begin + (ksteps_per_split >> 2));
    const int rows = int(a.total_rows);                                        // <= 32 * TM: one row tile
    constexpr int D = Q4 ? 8 : 4;
    uint4 q[Q4 ? D : 1];
    unsigned sc[Q4 ? D : 1];
    bf16x8 bf[Q4 ? 1 : D][4];
    const uint4* Q = static_cast<const uint4*>(a.B) + int64_t(cb) * n_chunks * 64 + lane;
    const unsigned char* S = static_cast<const unsigned char*>(a.Bs) + int64_t(cb) * n_chunks * 64 + lane;
    const bf16_t* Bp = static_cast<const bf16_t*>(a.B) + int64_t(cb) * n_chunks * 2048 + lane * 8;
    auto request = [&](int u, int ch) {
        if (Q4) {
            q[Q4 ? u : 0] = Q[int64_t(ch) * 64];
            sc[Q4 ? u : 0] = S[int64_t(ch) * 64];
        } else {
#pragma unroll
            for (int ks = 0; ks < 4; ++ks) bf[Q4 ? 0 : u][ks] = *reinterpret_cast<const bf16x8*>(Bp + (int64_t(ch) * 4 + ks) * 512);
        }
    };
    // pieces past the split re-read its last piece (never used)
#pragma unroll
    for (int u = 0; u < D; ++u) request(u, min(ch_begin + wave + NW * u, ch_end - 1));
    // the rows of A over the split's k range, zero past K
    {
        const int k0 = ch_begin * 64, kn = (ch_end - ch_begin) * 64;
        const int pieces_per_row = kn >> 3;
        for (int e = tid; e < rows * pieces_per_row; e += NW * 64) {
            const int g = e / pieces_per_row, k = k0 + 8 * (e - g * pieces_per_row);
            const uint32_t t = uint32_t(g) / a.R, r = uint32_t(g) - t * a.R;
            const int64_t base = int64_t(t) * a.a_tok_stride + (a.arow ? int64_t(a.arow[r]) : int64_t(r) * a.K);
            bf16x8 v;
#pragma unroll
            for (int i = 0; i < 8; ++i) v[i] = bf16_t(0.f);
            if (AMODE == 0) {
                if (k < a.K) v = *reinterpret_cast<const bf16x8*>(A + base + k);
            } else {
#pragma unroll
                for (int i = 0; i < 8; ++i)
                    if (k + i < a.K) v[i] = A[base + (a.acol ? a.acol[k + i] : k + i)];
            }
            *reinterpret_cast<bf16x8*>(xs + int64_t(g) * x_ld + (k - k0)) = v;
        }
    }
    __syncthreads();
    floatx16 acc[TM];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[i][v] = 0.f;
    // lane l supplies row 32i + l%32 and, in k-step u of a piece, k = 64*piece + (Q4 ? 32*(l/32) + 8u : 16u + 8*(l/32)) ..
    bool tv[TM];
    const bf16_t* xrow[TM];
#pragma unroll
    for (int i = 0; i < TM; ++i) {
        tv[i] = 32 * i + (lane & 31) < rows;
        xrow[i] = xs + int64_t(tv[i] ? 32 * i + (lane & 31) : 0) * x_ld + (Q4 ? 32 : 8) * (lane >> 5);
    }
    bf16x8 zero;
#pragma unroll
    for (int i = 0; i < 8; ++i) zero[i] = bf16_t(0.f);
    for (int idx0 = 0; ch_begin + wave + NW * idx0 < ch_end; idx0 += D) {
#pragma unroll
        for (int u = 0; u < D; ++u) {
            const int ch = ch_begin + wave + NW * (idx0 + u);
            if (ch < ch_end) {                                                 // wave-uniform
                bf16x8 w[4];
                if (Q4) {
                    q4_dequant_block(q[Q4 ? u : 0], sc[Q4 ? u : 0], w);
                } else {
#pragma unroll
                    for (int ks = 0; ks < 4; ++ks) w[ks] = bf[Q4 ? 0 : u][ks];
                }
#pragma unroll
                for (int ks = 0; ks < 4; ++ks)
#pragma unroll
                    for (int i = 0; i < TM; ++i) {
                        const bf16x8 x = tv[i] ? *reinterpret_cast<const bf16x8*>(xrow[i] + (ch - ch_begin) * 64 + (Q4 ? 8 : 16) * ks)
                                               : zero;
                        acc[i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(w[ks], x, acc[i], 0, 0, 0);
                    }
            }
            const int nxt = ch + NW * D;
            if (nxt < ch_end) request(u, nxt);                                 // wave-uniform
        }
    }
    __syncthreads();                                                           // the rows are dead: their LDS becomes red
    split_finish<TM, NW>(a, partial, red, acc, 0u, cb, split, nsplit, uint32_t(32 * TM));
}

// One row tile of up to 64 rows against 256 columns per workgroup ("skinny" launches: small serving batches, 5 to 64
// rows). The rows of A over the split's k range sit in LDS as in step_split_lds_kernel, but here they are shared by
// eight column blocks: wave w streams ALL pieces of column block 8 * blockIdx.y + w (ring of D pieces in flight) and
// owns its 32 columns outright, so there is no reduction across waves, and A is copied once per 256 columns instead
// of once per 32 (at 64 rows the copies of the one-block kernel moved twice the bytes of the parameter stream).
// With one split the wave stores through the scatter tables (out_vec4: columns come in aligned runs of four, stored
// as 8-byte pieces); else fp32 partial sums [split][row][Cp] that step_split_reduce_kernel adds in split order.
template <int TM, int AMODE, int Q4>
__global__ void __launch_bounds__(512) step_skinny_kernel(StepArgs a, float* partial, int ksteps_per_split, int x_ld,
                                                          int out_vec4) {
    extern __shared__ __attribute__((aligned(16))) unsigned char dyn_smem[];
    bf16_t* xs = reinterpret_cast<bf16_t*>(dyn_smem);                          // [rows][x_ld]
    const bf16_t* A = static_cast<const bf16_t*>(a.A);
    bf16_t* Out = static_cast<bf16_t*>(a.Out);
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int cb = blockIdx.y * 8 + wave, split = blockIdx.z, nsplit = gridDim.z;
    const bool has_cols = cb * 32 < a.C;                                       // wave-uniform
    const int n_chunks = a.Kp >> 6;
    const int ch_begin = split * (ksteps_per_split >> 2);
    const int ch_end = min(n_chunks, ch_begin + (ksteps_per_split >> 2));
    const int rows = int(a.total_rows);                                        // <= 32 * TM
    constexpr int D = Q4 ? 8 : 4;
    uint4 q[Q4 ? D : 1];
    unsigned sc[Q4 ? D : 1];
    bf16x8 bf[Q4 ? 1 : D][4];
    const int cbc = has_cols ? cb : 0;                                         // a wave without columns streams nothing it uses
    const uint4* Q = static_cast<const uint4*>(a.B) + int64_t(cbc) * n_chunks * 64 + lane;
    const unsigned char* S = static_cast<const unsigned char*>(a.Bs) + int64_t(cbc) * n_chunks * 64 + lane;
    const bf16_t* Bp = static_cast<const bf16_t*>(a.B) + int64_t(cbc) * n_chunks * 2048 + lane * 8;
    auto request = [&](int u, int ch) {
        if (Q4) {
            q[Q4 ? u : 0] = Q[int64_t(ch) * 64];
            sc[Q4 ? u : 0] = S[int64_t(ch) * 64];
        } else {
#pragma unroll
            for (int ks = 0; ks < 4; ++ks) bf[Q4 ? 0 : u][ks] = *reinterpret_cast<const bf16x8*>(Bp + (int64_t(ch) * 4 + ks) * 512);
        }
    };
    if (has_cols) {
#pragma unroll
        for (int u = 0; u < D; ++u) request(u, min(ch_begin + u, ch_end - 1));    // pieces past the split: its last one, unused
    }
    // the rows of A over the split's k range, zero past K
    {
        const int k0 = ch_begin * 64, kn = (ch_end - ch_begin) * 64;
        const int pieces_per_row = kn >> 3;
        for (int e = tid; e < rows * pieces_per_row; e += 512) {
            const int g = e / pieces_per_row, k = k0 + 8 * (e - g * pieces_per_row);
            const uint32_t t = uint32_t(g) / a.R, r = uint32_t(g) - t * a.R;
            const int64_t base = int64_t(t) * a.a_tok_stride + (a.arow ? int64_t(a.arow[r]) : int64_t(r) * a.K);
            bf16x8 v;
#pragma unroll
            for (int i = 0; i < 8; ++i) v[i] = bf16_t(0.f);
            if (AMODE == 0) {
                if (k < a.K) v = *reinterpret_cast<const bf16x8*>(A + base + k);
            } else {
#pragma unroll
                for (int i = 0; i < 8; ++i)
                    if (k + i < a.K) v[i] = A[base + (a.acol ? a.acol[k + i] : k + i)];
            }
            *reinterpret_cast<bf16x8*>(xs + int64_t(g) * x_ld + (k - k0)) = v;
        }
    }
    __syncthreads();
    if (!has_cols) return;
    floatx16 acc[TM];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[i][v] = 0.f;
    bool tv[TM];
    const bf16_t* xrow[TM];
#pragma unroll
    for (int i = 0; i < TM; ++i) {
        tv[i] = 32 * i + (lane & 31) < rows;
        xrow[i] = xs + int64_t(tv[i] ? 32 * i + (lane & 31) : 0) * x_ld + (Q4 ? 32 : 8) * (lane >> 5);
    }
    bf16x8 zero;
#pragma unroll
    for (int i = 0; i < 8; ++i) zero[i] = bf16_t(0.f);
    for (int c0 = ch_begin; c0 < ch_end; c0 += D) {
#pragma unroll
        for (int u = 0; u < D; ++u) {
            const int ch = c0 + u;
            if (ch < ch_end) {                                                 // wave-uniform
                bf16x8 w[4];
                if (Q4) {
                    q4_dequant_block(q[Q4 ? u : 0], sc[Q4 ? u : 0], w);
                } else {
#pragma unroll
                    for (int ks = 0; ks < 4; ++ks) w[ks] = bf[Q4 ? 0 : u][ks];
                }
#pragma unroll
                for (int ks = 0; ks < 4; ++ks)
#pragma unroll
                    for (int i = 0; i < TM; ++i) {
                        const bf16x8 x = tv[i] ? *reinterpret_cast<const bf16x8*>(xrow[i] + (ch - ch_begin) * 64 + (Q4 ? 8 : 16) * ks)
                                               : zero;
                        acc[i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(w[ks], x, acc[i], 0, 0, 0);
                    }
            }
            if (ch + D < ch_end) request(u, ch + D);                           // wave-uniform
        }
    }
    // lane l, register v of acc[i]: row 32i + l%32, column 32*cb + 8*(v/4) + 4*(l/32) + v%4: registers 4q .. 4q+3 are
    // four consecutive columns, stored as one piece where the layout allows (always for the partial sums)
#pragma unroll
    for (int i = 0; i < TM; ++i) {
        const uint32_t g = uint32_t(32 * i + (lane & 31));
        if (g >= a.total_rows) continue;
        const uint32_t t = g / a.R, r = g - t * a.R;
        const int64_t obase = int64_t(t) * a.c_tok_stride + a.crow[r];
#pragma unroll
        for (int qd = 0; qd < 4; ++qd) {
            const int c = cb * 32 + 8 * qd + 4 * (lane >> 5);
            if (c >= a.C) continue;
            if (nsplit > 1) {                      // Cp is a multiple of 32: the four columns exist in the buffer
                floatx4 v4;
#pragma unroll
                for (int e = 0; e < 4; ++e) v4[e] = acc[i][4 * qd + e];
                *reinterpret_cast<floatx4*>(partial + (int64_t(split) * (32 * TM) + g) * a.Cp + c) = v4;
            } else if (out_vec4 && c + 3 < a.C) {
                bf16x4 pk;
#pragma unroll
                for (int e = 0; e < 4; ++e) pk[e] = bf16_t(acc[i][4 * qd + e]);
                *reinterpret_cast<bf16x4*>(Out + obase + a.ccol[c]) = pk;
            } else {
#pragma unroll
                for (int e = 0; e < 4; ++e)
                    if (c + e < a.C) Out[obase + a.ccol[c + e]] = bf16_t(acc[i][4 * qd + e]);
            }
        }
    }
}

template <int TM, int AMODE, int NW>
__global__ void __launch_bounds__(NW * 64) step_split_q4_kernel(StepArgs a, float* partial, int ksteps_per_split) {
    __shared__ float red[NW * TM * 1024];
    split_run_q4<TM, AMODE, NW>(a, partial, ksteps_per_split, red, blockIdx.x, blockIdx.y, blockIdx.z, gridDim.z,
                                gridDim.x * (TM * 32));
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
// Whole-chain kernel for small layers: when every packed tensor of the plan and two copies of the
// largest per-token tensor fit in LDS together (the small fp32 train: 19 KB of cores, 8 KB per
// intermediate), one launch runs all steps. At create time the tensors (as fp32, rows padded) and
// the offset tables of all steps are laid out as one contiguous image (small_chain_image_kernel); a
// workgroup copies that image into LDS with 16-byte loads, then takes tokens one at a time: the
// token's input goes to an LDS buffer, every step reads one buffer and scatters into the other
// through its tables - the same tables the one-launch-per-step kernels use - and the last step
// stores to memory. Plain fp32 FMA, 256 threads over the R*C outputs of a step (consecutive threads
// take consecutive columns, so the input value is an LDS broadcast and the tensor rows of a wave are
// 4 banks apart). Intermediates are rounded to the storage type between steps, as on the other
// paths. For layers this small the cost is launch latency, and this is one launch instead of one
// per step.
// ---------------------------------------------------------------------------------------------
constexpr int kSmallChainMaxSteps = 8;
struct SmallChainStep {
    const void* B;                         // packed tensor (fragment-major); read by the image kernel only
    const int32_t *arow, *acol;            // gather tables of the step's input (null: plain); image kernel only
    const int32_t *crow, *ccol;            // scatter tables of its output; image kernel only
    int32_t R, K, C, nks;                  // nks = Kp / 16 of the packing
    int32_t b_off;                         // offset of the tensor in the image, in 4-byte words (a multiple of 4)
    int32_t ldb;                           // its row length: K + 4 when K % 4 == 0 (16-byte reads), else K + 1
    int32_t t_off;                         // offset of the tables in the image: crow[R], ccol[C], then arow[R],
                                           // acol[K] when the input is gathered
    int32_t gathered;
};
struct SmallChainArgs {
    const void* X;
    void* Y;
    const float* image;                    // tensors and tables of all steps, image_words long (a multiple of 4)
    int64_t N, M;
    int32_t tokens, nsteps, image_words;
    int32_t buf_off[2];                    // offsets of the two per-token buffers in LDS, in words
    SmallChainStep st[kSmallChainMaxSteps];
};

template <typename T>
__global__ void __launch_bounds__(256) small_chain_image_kernel(SmallChainArgs a, float* image) {
    int32_t* imagei = reinterpret_cast<int32_t*>(image);
    for (int i = blockIdx.x * 256 + threadIdx.x; i < a.image_words; i += gridDim.x * 256) image[i] = 0.f;
    __syncthreads();                       // single workgroup launch: zero fill before the pieces
    for (int s = 0; s < a.nsteps; ++s) {
        const SmallChainStep& st = a.st[s];
        const T* B = static_cast<const T*>(st.B);
        for (int i = threadIdx.x; i < st.C * st.K; i += 256) {
            int c = i / st.K, k = i - c * st.K;
            image[st.b_off + c * st.ldb + k] = to_float(B[bfrag_offset(c, k, st.nks)]);
        }
        int32_t* tab = imagei + st.t_off;
        for (int i = threadIdx.x; i < st.R; i += 256) tab[i] = st.crow[i];
        for (int i = threadIdx.x; i < st.C; i += 256) tab[st.R + i] = st.ccol[i];
        if (st.gathered) {
            for (int i = threadIdx.x; i < st.R; i += 256) tab[st.R + st.C + i] = st.arow[i];
            for (int i = threadIdx.x; i < st.K; i += 256) tab[2 * st.R + st.C + i] = st.acol[i];
        }
    }
}

template <typename T>
__global__ void __launch_bounds__(256) small_chain_kernel(SmallChainArgs a) {
    extern __shared__ __attribute__((aligned(16))) unsigned char dyn_smem[];
    float* lds = reinterpret_cast<float*>(dyn_smem);
    const int32_t* ldsi = reinterpret_cast<const int32_t*>(dyn_smem);
    const int tid = threadIdx.x;
    {
        const floatx4* src = reinterpret_cast<const floatx4*>(a.image);
        floatx4* dst = reinterpret_cast<floatx4*>(lds);
#pragma unroll 4
        for (int i = tid; i < (a.image_words >> 2); i += 256) dst[i] = src[i];
    }
    const T* X = static_cast<const T*>(a.X);
    T* Y = static_cast<T*>(a.Y);
    for (int t = blockIdx.x; t < a.tokens; t += gridDim.x) {
        __syncthreads();                   // image loaded / previous token's buffers no longer read
        float* in = lds + a.buf_off[0];
        float* out = lds + a.buf_off[1];
        for (int i = tid; i < int(a.N); i += 256) in[i] = to_float(X[int64_t(t) * a.N + i]);
        __syncthreads();
        for (int s = 0; s < a.nsteps; ++s) {
            const SmallChainStep& st = a.st[s];
            const float* Bs = lds + st.b_off;
            const int32_t* t_crow = ldsi + st.t_off;
            const int32_t* t_ccol = t_crow + st.R;
            const int32_t* t_arow = t_ccol + st.C;
            const int32_t* t_acol = t_arow + st.R;
            const bool last = s + 1 == a.nsteps;
            for (int i = tid; i < st.R * st.C; i += 256) {
                int r = i / st.C, c = i - r * st.C;
                const float* brow = Bs + c * st.ldb;
                float acc = 0.f;
                if (st.gathered) {
                    const int base = t_arow[r];
                    for (int k = 0; k < st.K; ++k) acc = fmaf(in[base + t_acol[k]], brow[k], acc);
                } else if ((st.K & 3) == 0) {
                    // 16-byte LDS reads, several in flight
                    const floatx4* a4 = reinterpret_cast<const floatx4*>(in + r * st.K);
                    const floatx4* b4 = reinterpret_cast<const floatx4*>(brow);
                    float acc1 = 0.f, acc2 = 0.f, acc3 = 0.f;
#pragma unroll 4
                    for (int k = 0; k < (st.K >> 2); ++k) {
                        floatx4 av = a4[k], bv = b4[k];
                        acc = fmaf(av[0], bv[0], acc);
                        acc1 = fmaf(av[1], bv[1], acc1);
                        acc2 = fmaf(av[2], bv[2], acc2);
                        acc3 = fmaf(av[3], bv[3], acc3);
                    }
                    acc = (acc + acc1) + (acc2 + acc3);
                } else {
                    const float* arow = in + r * st.K;
                    for (int k = 0; k < st.K; ++k) acc = fmaf(arow[k], brow[k], acc);
                }
                const int o = t_crow[r] + t_ccol[c];
                if (last) Y[int64_t(t) * a.M + o] = from_float<T>(acc);
                else out[o] = to_float(from_float<T>(acc));
            }
            __syncthreads();
            float* tmp = in;
            in = out;
            out = tmp;
        }
    }
}
