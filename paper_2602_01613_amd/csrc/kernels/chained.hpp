// Chained kernels: two contraction steps in one launch with the intermediate kept in the MFMA register layout.
// Part of the tn_linear library's single translation unit: included by tn_linear.hip inside its
// anonymous namespace, after <hip/hip_runtime.h> and tn_plan.hpp.
#pragma once

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
    // few token tiles: the range of a is split over n_splits workgroups per (token tile, j set), each of which
    // writes fp32 partial sums [split][tokens][M] to `partial`; a second kernel adds them in split order
    int32_t n_splits, a_per_split;
    float* partial;
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

template <int NS, int BAR>
__global__ void __launch_bounds__(256, 1) step_pair_kernel(PairArgs p) {
    // A ring of NS LDS stages, one value of a each; L direct-to-LDS loads per wave and stage. Stages are requested
    // BAR at a time, with one workgroup barrier per BAR values of a.
    constexpr int L = 5;
    static_assert(NS >= 2 * BAR + 1 && NS - 2 * BAR - 1 <= 4, "ring depth");
    constexpr int STAGE_BYTES = 20 * 1024, X_OFF = 16 * 1024;
    extern __shared__ __attribute__((aligned(16))) unsigned char dyn_smem[];

    int id = blockIdx.x;
    const int split = id % p.n_splits;                  // n_splits = 1: no split
    id /= p.n_splits;
    int tok_tile, jset;
    if (p.n_splits > 1) {
        // few token tiles: an exact grid (a workgroup that only returns still costs a CU's worth of LDS and registers)
        tok_tile = id / p.n_jsets;
        jset = id % p.n_jsets;
    } else {
        const int xcd = id & 7, slot = id >> 3;
        tok_tile = (slot / p.n_jsets) * 8 + xcd;
        jset = slot % p.n_jsets;
    }
    if (tok_tile >= p.n_tok_tiles) return;
    const int t0 = tok_tile * 32;
    const int a_begin = split * p.a_per_split;          // this workgroup's values of a: a_begin .. a_begin + A - 1

    const bf16_t* X = static_cast<const bf16_t*>(p.X);
    const bf16_t* B0 = static_cast<const bf16_t*>(p.B0);
    const bf16_t* B1f = static_cast<const bf16_t*>(p.B1f);
    bf16_t* Y = static_cast<bf16_t*>(p.Y);
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int j0 = jset * 8 + wave * 2;
    const int A = min(p.A, a_begin + p.a_per_split) - a_begin;          // >= 1 by construction of the grid

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
    auto issue = [&](int a_rel, int stage) {             // a_rel counts from a_begin, as everything below does
        const int a = a_begin + a_rel;
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
    auto wait_outstanding_tiles = [&](int n) {            // n is wave-uniform
        if (n <= 0) wait_vmcnt<0>();
        else if (n == 1) wait_vmcnt<L>();
        else if (n == 2) wait_vmcnt<2 * L>();
        else if (n == 3) wait_vmcnt<3 * L>();
        else wait_vmcnt<4 * L>();
    };

    floatx16 acc[2][4];
#pragma unroll
    for (int jj = 0; jj < 2; ++jj)
#pragma unroll
        for (int ct = 0; ct < 4; ++ct)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[jj][ct][v] = 0.f;

    // Stage of a is a % NS. At the barrier before a group of BAR values a .. a+BAR-1 the stages of a+1 .. a+BAR must
    // have landed (they are read while the group is computed: see the refills below), and the stages requested
    // there, those of a+NS-BAR .. a+NS-1, are the ones of a-BAR .. a-1, whose last reads were issued a full group
    // earlier.
    int issued = 0;
    for (; issued < NS - BAR && issued < A; ++issued) issue(issued, issued);
    wait_outstanding_tiles(min(issued - 1, 4));          // tile 0 has landed
    __syncthreads();
    bf16x8 xb[4];
#pragma unroll
    for (int s = 0; s < 4; ++s) xb[s] = *reinterpret_cast<const bf16x8*>(dyn_smem + X_OFF + s * 1024 + lane * 16);
    // the B1 slice of the current tile, in registers: p1[ct][s]. Each fragment is used twice per tile (once per j
    // of the wave); right after its second use it is refilled from the NEXT tile's stage, so that the LDS reads of
    // a tile are spread over the MFMAs of the tile before and none of them is waited for after the barrier.
    bf16x8 p1[4][4];
#pragma unroll
    for (int ct = 0; ct < 4; ++ct)
#pragma unroll
        for (int s = 0; s < 4; ++s)
            p1[ct][s] = *reinterpret_cast<const bf16x8*>(dyn_smem + (ct * 4 + s) * 1024 + lane * 16);

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
    // half s/2 of z are the 8 values this lane supplies to k-step s. With REFILL, the four fragments of a k-step
    // are reloaded from `next` (the following tile's slice in LDS) as soon as their MFMAs have been issued.
    auto contract1 = [&](const floatx16 (&z)[2], floatx16 (&y)[4], const unsigned char* next, auto refill_tag) {
        constexpr bool REFILL = decltype(refill_tag)::value;
        bf16x8 zb[4];
#pragma unroll
        for (int s = 0; s < 4; ++s)
#pragma unroll
            for (int e = 0; e < 8; ++e) zb[s][e] = bf16_t(z[s >> 1][8 * (s & 1) + e]);
#pragma unroll
        for (int s = 0; s < 4; ++s) {
#pragma unroll
            for (int ct = 0; ct < 4; ++ct)
                y[ct] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(p1[ct][s], zb[s], y[ct], 0, 0, 0);
            if (REFILL) {
#pragma unroll
                for (int ct = 0; ct < 4; ++ct)
                    p1[ct][s] = *reinterpret_cast<const bf16x8*>(next + (ct * 4 + s) * 1024 + lane * 16);
            }
        }
    };

    // software pipeline over (a, j): the first contraction of the next unit is issued before the
    // second contraction of the current one, so that reading back and rounding Z overlaps MFMAs
    floatx16 z0[2], z1[2];
    contract0(p0[0], xb, z0);
    auto iteration = [&](int a, auto last_tag) {
        constexpr bool LAST = decltype(last_tag)::value;
        if (BAR == 1 || a % BAR == 0) {                      // wave-uniform
            wait_outstanding_tiles(min(max(issued - 1 - (a + BAR), 0), 4));       // tiles a+1 .. a+BAR have landed
            __syncthreads();   // ... for every wave; everyone's reads of the stages refilled now were issued long ago
#pragma unroll
            for (int g = 0; g < BAR; ++g)
                if (issued < A) {
                    issue(issued, issued % NS);
                    ++issued;
                }
        }
        const unsigned char* snxt = dyn_smem + ((a + 1) % NS) * STAGE_BYTES;
        __builtin_amdgcn_sched_barrier(0);
        contract0(p0[1], xb, z1);
        if (!LAST) {
#pragma unroll
            for (int s = 0; s < 4; ++s) xb[s] = *reinterpret_cast<const bf16x8*>(snxt + X_OFF + s * 1024 + lane * 16);
            __builtin_amdgcn_sched_barrier(0);
        }
        contract1(z0, acc[0], snxt, std::false_type());
        if (!LAST) contract0(p0[0], xb, z0);
        if (!LAST) contract1(z1, acc[1], snxt, std::true_type());
        else contract1(z1, acc[1], snxt, std::false_type());
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

    if (p.n_splits > 1) {
        // Partial sums of this workgroup's range of a: fp32, in the output's own layout, [split][tokens][M]. As in the
        // epilogue below the tiles are transposed through LDS so that the stores run along j: in two passes (waves
        // 0-1, then waves 2-3), each leaving 16-byte pieces of 4 consecutive j per (token, c).
        const int t = lane & 31;
        const int yj = p.yrow[jset * 8];
        float* dst = p.partial + int64_t(split) * p.tokens * p.M;
#pragma unroll
        for (int half = 0; half < 2; ++half) {
            if (half) __syncthreads();                  // the first pass has been read out
            if ((wave >> 1) == half) {
#pragma unroll
                for (int jj = 0; jj < 2; ++jj)
#pragma unroll
                    for (int ct = 0; ct < 4; ++ct)
#pragma unroll
                        for (int v = 0; v < 16; ++v) {
                            const int c = 32 * ct + 8 * (v >> 2) + 4 * (lane >> 5) + (v & 3);
                            *reinterpret_cast<float*>(dyn_smem + (t * 128 + (c ^ t)) * 16 + ((wave & 1) * 2 + jj) * 4) = acc[jj][ct][v];
                        }
            }
            __syncthreads();
#pragma unroll 4
            for (int e = tid; e < 32 * 128; e += 256) {
                const int tt = e >> 7, c = e & 127;
                if (t0 + tt >= p.tokens || c >= p.C1) continue;
                const floatx4 v4 = *reinterpret_cast<const floatx4*>(dyn_smem + (tt * 128 + (c ^ tt)) * 16);
                *reinterpret_cast<floatx4*>(dst + int64_t(t0 + tt) * p.M + p.ycol[c] + yj + 4 * half) = v4;
            }
        }
        return;
    }
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

// The work of one wave: items gw, gw + GW, ... of the tokens * (c1 tile groups) items. `smem` is the area of
// chain2_smem_bytes: wave slot `wave` (0..3) uses its own input buffer and patches in it. Out may be memory or
// LDS (generic address). No workgroup barrier inside: waves come and go independently.
template <int R1T, int K1S, int C2T, int RUN_C1>
__device__ __forceinline__ void chain2_run(const Chain2Args& p, unsigned char* smem, int wave, int64_t gw, int64_t GW) {
    constexpr int IN_BYTES = R1T * K1S * 1024;           // one token's input in fragment order
    constexpr int KS2 = 2 * R1T;                         // k-steps of the second contraction
    constexpr int PATCH_LD = 80;                         // bytes per patch row (64 + 16 of padding)
    constexpr int PATCH_BYTES = 32 * PATCH_LD;
    const bf16_t* In = static_cast<const bf16_t*>(p.In);
    const bf16_t* Ba = static_cast<const bf16_t*>(p.Ba);
    const bf16_t* Bbf = static_cast<const bf16_t*>(p.Bbf);
    bf16_t* Out = static_cast<bf16_t*>(p.Out);
    const int lane = threadIdx.x & 63;
    unsigned char* my_in = smem + wave * IN_BYTES;
    unsigned char* my_patch = smem + 4 * IN_BYTES + wave * (2 * PATCH_BYTES);

    const int n_groups = (p.c1_tiles + p.tiles_per_item - 1) / p.tiles_per_item;
    const int64_t n_items = int64_t(p.tokens) * n_groups;
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

template <int R1T, int K1S, int C2T, int RUN_C1>
__global__ void __launch_bounds__(256, 1) step_chain2_kernel(Chain2Args p) {
    extern __shared__ __attribute__((aligned(16))) unsigned char dyn_smem[];
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    chain2_run<R1T, K1S, C2T, RUN_C1>(p, dyn_smem, wave, int64_t(blockIdx.x) * 4 + wave, int64_t(gridDim.x) * 4);
}

// ---------------------------------------------------------------------------------------------
// Decode-size fusion of a chained factor pair with the wide step that follows it (a Tucker layer's two in-factor
// products and its core): one launch instead of two, for calls of a few tokens. Every workgroup of the wide
// step's grid (one per block of 32 columns, 8 waves, the whole K) recomputes the pair's small result for the
// call's tokens (2304 values per token for the up_proj layer) instead of reading it from memory:
//   1. the waves that have an item (token, tile of 32 values of c1) request that item's operands - the token's
//      input rows, the two small packed tensors, the offsets of its outputs - straight into registers;
//   2. every wave requests ALL its k-steps of the wide step's packed tensor (KPW fragments of 1 KB per wave, the
//      workgroup's whole block): from here on the parameter stream, which is what bounds a call this small, is
//      in flight, and everything below runs in its shadow;
//   3. the item waves wait for their operands only (they were requested first, and loads return in order), run
//      the two chained MFMA contractions as step_chain2_kernel does and store the rounded result to LDS;
//   4. after one barrier every wave multiplies its fragments with the LDS buffer as the other operand, and the
//      eight partial tiles are summed through LDS in wave order (as in step_split_kernel).
// Limits (checked by the host): R1 <= 64, C2 <= 64, K1 <= 16*K1S, tokens * ceil(C1/32) <= 8 items, K of the wide
// step <= 128 * KPW, its rows are the tokens (R = 1), output offsets in aligned runs of 8.
// ---------------------------------------------------------------------------------------------
// One (token, tile of 32 values of c1) item of a chained pair with every operand requested up front, straight into
// registers: nothing is staged through LDS and there is a single memory round trip before the MFMAs, which is what
// a call of a few tokens needs (step_chain2_kernel pipelines tokens through LDS instead, which pays once a wave has
// many of them). Register layouts as in chain2_run.
template <int R1T, int K1S, int C2T, int RUN_C1>
struct Chain2Item {
    static constexpr int KS2 = 2 * R1T;
    bf16x8 inf[R1T][K1S], ba[K1S], bb[C2T][KS2];
    int o_lane[C2T];             // offset of the index this lane holds one value of (c2 when RUN_C1; else c1, entry 0 only)
    int o_run[C2T][4];           // offsets of the runs of 4 it holds in its registers (c1 when RUN_C1, entries [0][q]; else c2)
    int t, ct1, j0;              // the item covers the c2 tiles j0 .. j0 + C2T - 1

    __device__ __forceinline__ void load(const Chain2Args& c, int token, int tile, int first_c2_tile = 0) {
        const bf16_t* In = static_cast<const bf16_t*>(c.In);
        const bf16_t* Ba = static_cast<const bf16_t*>(c.Ba);
        const bf16_t* Bbf = static_cast<const bf16_t*>(c.Bbf);
        const int lane = threadIdx.x & 63, lrow = lane & 31, lhalf = lane >> 5;
        t = token;
        ct1 = tile;
        j0 = first_c2_tile;
        const bf16_t* in_t = In + int64_t(t) * c.in_tok_stride;
        // straight-line loads from clamped addresses; what lies outside the input is replaced by zeros later
#pragma unroll
        for (int i = 0; i < R1T; ++i) {
            const int r = min(32 * i + lrow, c.R1 - 1);
#pragma unroll
            for (int sk = 0; sk < K1S; ++sk) {
                const int k = min(16 * sk + 8 * lhalf, c.K1 - 8);
                inf[i][sk] = *reinterpret_cast<const bf16x8*>(in_t + int64_t(r) * c.K1 + k);
            }
        }
#pragma unroll
        for (int sk = 0; sk < K1S; ++sk)      // k-steps past the packed tensor's padding meet zero input: any finite block will do
            ba[sk] = *reinterpret_cast<const bf16x8*>(Ba + (int64_t(ct1) * c.nks_a + min(sk, c.nks_a - 1)) * 512 + lane * 8);
#pragma unroll
        for (int j = 0; j < C2T; ++j)
#pragma unroll
            for (int sk = 0; sk < KS2; ++sk)
                bb[j][sk] = *reinterpret_cast<const bf16x8*>(Bbf + (int64_t(j0 + j) * KS2 + sk) * 512 + lane * 8);
        // output offsets come in aligned runs of 8 along the direction the pieces run (checked by the planner)
        if (RUN_C1) {
#pragma unroll
            for (int j = 0; j < C2T; ++j) o_lane[j] = c.off2[min(32 * (j0 + j) + lrow, c.C2 - 1)];
#pragma unroll
            for (int q = 0; q < 4; ++q) o_run[0][q] = c.off1[min(32 * ct1 + 8 * q, c.C1 - 1)] + 4 * lhalf;
        } else {
            o_lane[0] = c.off1[min(32 * ct1 + lrow, c.C1 - 1)];
#pragma unroll
            for (int j = 0; j < C2T; ++j)
#pragma unroll
                for (int q = 0; q < 4; ++q) o_run[j][q] = c.off2[min(32 * (j0 + j) + 8 * q, c.C2 - 1)] + 4 * lhalf;
        }
    }

    // Both contractions; the result goes to out (memory or LDS) in 8-byte pieces of 4 consecutive values.
    __device__ __forceinline__ void compute(const Chain2Args& c, bf16_t* out) const {
        const int lane = threadIdx.x & 63, lrow = lane & 31, lhalf = lane >> 5;
        bf16x8 zero;
#pragma unroll
        for (int e = 0; e < 8; ++e) zero[e] = bf16_t(0.f);
        floatx16 d[R1T];
#pragma unroll
        for (int i = 0; i < R1T; ++i) {
#pragma unroll
            for (int v = 0; v < 16; ++v) d[i][v] = 0.f;
            const bool rv = 32 * i + lrow < c.R1;
#pragma unroll
            for (int sk = 0; sk < K1S; ++sk) {
                const bf16x8 x = (rv && 16 * sk + 8 * lhalf < c.K1) ? inf[i][sk] : zero;
                d[i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(x, ba[sk], d[i], 0, 0, 0);
            }
        }
        bf16x8 zb[KS2];
#pragma unroll
        for (int i = 0; i < R1T; ++i)
#pragma unroll
            for (int u = 0; u < 2; ++u)
#pragma unroll
                for (int e = 0; e < 8; ++e) zb[2 * i + u][e] = bf16_t(d[i][8 * u + e]);
        bf16_t* out_t = out + int64_t(t) * c.out_tok_stride;
#pragma unroll
        for (int j = 0; j < C2T; ++j) {
            if (32 * (j0 + j) >= c.C2) continue;                           // wave-uniform
            floatx16 acc;
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[v] = 0.f;
#pragma unroll
            for (int sk = 0; sk < KS2; ++sk)
                acc = RUN_C1 ? __builtin_amdgcn_mfma_f32_32x32x16_bf16(zb[sk], bb[j][sk], acc, 0, 0, 0)
                             : __builtin_amdgcn_mfma_f32_32x32x16_bf16(bb[j][sk], zb[sk], acc, 0, 0, 0);
            // RUN_C1: lane l holds c2 = 32(j0+j) + l%32 and, in registers 4q..4q+3, c1 = 32*ct1 + 8q + 4*(l/32) + 0..3
            // else  : lane l holds c1 = 32*ct1 + l%32 and c2 = 32(j0+j) + 8q + 4*(l/32) + 0..3
            const bool lane_ok = RUN_C1 ? 32 * (j0 + j) + lrow < c.C2 : 32 * ct1 + lrow < c.C1;
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const bool run_ok = RUN_C1 ? 32 * ct1 + 8 * q < c.C1 : 32 * (j0 + j) + 8 * q < c.C2;   // runs of 8 are whole
                if (!lane_ok || !run_ok) continue;
                const int base = RUN_C1 ? o_lane[j] + o_run[0][q] : o_lane[0] + o_run[j][q];
                bf16x4 pk;
#pragma unroll
                for (int u = 0; u < 4; ++u) pk[u] = bf16_t(acc[4 * q + u]);
                *reinterpret_cast<bf16x4*>(out_t + base) = pk;
            }
        }
    }
};

// A chained pair for a few tokens: one wave per (token, c1 tile) item, four items per workgroup. With two
// argument blocks (two layers applied to the same input, e.g. the gate and up projections of an MLP) the
// workgroups of blockIdx.y = 1 work on the second layer: one launch serves both.
template <int R1T, int K1S, int C2T, int RUN_C1>
__global__ void __launch_bounds__(256) step_chain2_small_kernel(Chain2Args c0, Chain2Args c1) {
    const Chain2Args& c = blockIdx.y ? c1 : c0;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int item = blockIdx.x * 4 + wave;
    if (item >= c.tokens * c.c1_tiles) return;
    Chain2Item<R1T, K1S, C2T, RUN_C1> it;
    it.load(c, item / c.c1_tiles, item % c.c1_tiles);
    it.compute(c, static_cast<bf16_t*>(c.Out));
}

// The same with one wave per (token, c1 tile, c2 tile): five times as many items for the out-factor pair of the
// up_proj layer (each repeats the first contraction, 18 MFMAs, and requests 30 KB instead of 54), one wave per
// workgroup so that they spread over as many compute units. A call of a few tokens is one memory round trip and a
// short MFMA chain either way: what this form cuts is the bytes each CU's memory pipeline delivers in that trip.
template <int R1T, int K1S, int RUN_C1>
__global__ void __launch_bounds__(64) step_chain2_fine_kernel(Chain2Args c0, Chain2Args c1) {
    const Chain2Args& c = blockIdx.y ? c1 : c0;
    const int c2_tiles = (c.C2 + 31) / 32;
    const int item = blockIdx.x;
    if (item >= c.tokens * c.c1_tiles * c2_tiles) return;
    const int j = item % c2_tiles, rest = item / c2_tiles;
    Chain2Item<R1T, K1S, 1, RUN_C1> it;
    it.load(c, rest / c.c1_tiles, rest % c.c1_tiles, j);
    it.compute(c, static_cast<bf16_t*>(c.Out));
}

// KPW: pieces of 64 k per wave. Q4: the wide step's tensor is read in its 4-bit form (see q4_stream_pack_kernel), one
// 16-byte load of codes and one scale byte per lane and piece instead of four fragment loads.
template <int K1S, int RUN_C1, int KPW, int Q4>
__global__ void __launch_bounds__(512) step_chain2_split_kernel(Chain2Args c0, StepArgs a0, int z_bytes0, Chain2Args c1,
                                                                StepArgs a1, int z_bytes1) {
    constexpr int NW = 8;
    extern __shared__ __attribute__((aligned(16))) unsigned char dyn_smem[];
    // blockIdx.y = 1: the second of two layers applied to the same input (see step_chain2_small_kernel)
    const Chain2Args& c = blockIdx.y ? c1 : c0;
    const StepArgs& a = blockIdx.y ? a1 : a0;
    const int z_bytes = blockIdx.y ? z_bytes1 : z_bytes0;
    bf16_t* z = reinterpret_cast<bf16_t*>(dyn_smem);                       // [tokens][a.a_tok_stride]
    float* red = reinterpret_cast<float*>(dyn_smem + z_bytes);             // NW x 1024
    const bf16_t* B = static_cast<const bf16_t*>(a.B);
    bf16_t* Out = static_cast<bf16_t*>(a.Out);
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int cb = blockIdx.x;
    if (cb * 32 >= a.C) return;                                            // the two layers' grids may differ
    const int nks = a.Kp >> 4;
    const int lrow = lane & 31, lhalf = lane >> 5;
    bf16x8 zero;
#pragma unroll
    for (int e = 0; e < 8; ++e) zero[e] = bf16_t(0.f);

    // ---- 1. operands of this wave's item
    const bool has_item = wave < c.tokens * c.c1_tiles;                    // wave-uniform
    Chain2Item<2, K1S, 2, RUN_C1> item;
    if (has_item) item.load(c, wave / c.c1_tiles, wave % c.c1_tiles);
    __builtin_amdgcn_sched_barrier(0);
    // ---- 2. the wave's share of the parameter stream: pieces of 64 k (four k-steps) wave, wave + 8, ..., the same
    //         assignment and order of summation as step_split_lds_kernel, so that a call gives the same bits whether
    //         it runs fused or as separate launches
    bf16x8 bf[Q4 ? 1 : KPW][4];
    uint4 qc[Q4 ? KPW : 1];
    unsigned qs[Q4 ? KPW : 1];
    const int n_chunks = nks >> 2;
    if (Q4) {
        const uint4* qp = static_cast<const uint4*>(a.B) + int64_t(cb) * n_chunks * 64 + lane;
        const unsigned char* sp = static_cast<const unsigned char*>(a.Bs) + int64_t(cb) * n_chunks * 64 + lane;
#pragma unroll
        for (int u = 0; u < KPW; ++u) {
            const int ch = min(wave + NW * u, n_chunks - 1);
            qc[u] = qp[int64_t(ch) * 64];
            qs[u] = sp[int64_t(ch) * 64];
        }
    } else {
        const bf16_t* bp = B + (int64_t(cb) * nks) * 512 + lane * 8;
#pragma unroll
        for (int u = 0; u < KPW; ++u) {
            const int ch = min(wave + NW * u, n_chunks - 1);
#pragma unroll
            for (int ks = 0; ks < 4; ++ks) bf[u][ks] = *reinterpret_cast<const bf16x8*>(bp + (int64_t(ch) * 4 + ks) * 512);
        }
    }
    __builtin_amdgcn_sched_barrier(0);
    // ---- 3. the chained pair for the item, into LDS
    if (has_item) item.compute(c, z);
    __syncthreads();
    // ---- 4. the wide step: lane l supplies token l%32, k = 16*ks + 8*(l/32) .. +7 from the LDS buffer
    floatx16 acc;
#pragma unroll
    for (int v = 0; v < 16; ++v) acc[v] = 0.f;
    {
        const bool tv = lrow < int(a.total_rows);
        const bf16_t* zrow = z + int64_t(tv ? lrow : 0) * a.a_tok_stride + 8 * lhalf;
        if (Q4) {
            // lanes 0-31 hold block 2*ch, lanes 32-63 block 2*ch + 1: k-step u of a piece takes k = 64*ch + 32*(l/32) + 8u ..
            const bf16_t* zq = z + int64_t(tv ? lrow : 0) * a.a_tok_stride + 32 * lhalf;
#pragma unroll
            for (int u = 0; u < KPW; ++u) {
                const int ch = wave + NW * u;
                if (ch < n_chunks) {                                           // wave-uniform
                    bf16x8 w[4];
                    q4_dequant_block(qc[u], qs[u], w);
#pragma unroll
                    for (int ks = 0; ks < 4; ++ks) {
                        const int k = 64 * ch + 8 * ks;
                        const bf16x8 x = (tv && k + 32 * lhalf < a.K) ? *reinterpret_cast<const bf16x8*>(zq + k) : zero;
                        acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(w[ks], x, acc, 0, 0, 0);
                    }
                }
            }
        } else {
#pragma unroll
            for (int u = 0; u < KPW; ++u) {
                const int ch = wave + NW * u;
                if (ch < n_chunks) {                                           // wave-uniform
#pragma unroll
                    for (int ks = 0; ks < 4; ++ks) {
                        const int k = 64 * ch + 16 * ks;
                        const bf16x8 x = (tv && k + 8 * lhalf < a.K) ? *reinterpret_cast<const bf16x8*>(zrow + k) : zero;
                        acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(bf[u][ks], x, acc, 0, 0, 0);
                    }
                }
            }
        }
    }
#pragma unroll
    for (int v = 0; v < 16; ++v) red[(wave * 16 + v) * 64 + lane] = acc[v];
    __syncthreads();
    // lane l, register v holds row (token) l%32, column 8*(v/4) + 4*(l/32) + v%4
    for (int e = tid; e < 1024; e += NW * 64) {
        const int v = (e >> 6) & 15, l = e & 63;
        float sum = 0.f;
#pragma unroll
        for (int w = 0; w < NW; ++w) sum += red[w * 1024 + e];
        const uint32_t g = uint32_t(l & 31);
        const int col = cb * 32 + 8 * (v >> 2) + 4 * (l >> 5) + (v & 3);
        if (g >= a.total_rows || col >= a.C) continue;
        Out[int64_t(g) * a.c_tok_stride + a.crow[0] + a.ccol[col]] = bf16_t(sum);
    }
}

