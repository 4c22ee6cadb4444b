// Kronecker-sum kernel: both steps of a two-tensor plan in one launch, per token, with the intermediate in
// MFMA registers. Part of the tn_linear library's single translation unit: included by tn_linear.hip inside
// its anonymous namespace, after kernels/tiled.hpp.
#pragma once

// ---------------------------------------------------------------------------------------------
// A network of two parameter tensors that share a bond rho (a tensor ring whose cores were contracted
// in pairs at create time into two half rings, a tensor train of two cores) is a sum over rho of
// Kronecker products: with the token's input seen as a matrix X_t[k][a],
//     Y_t[o1][o2] = sum_rho sum_a ( sum_k X_t[k][a] * B0[(o1, rho)][k] ) * B1[o2][(a, rho)]
// As two launches the intermediate Z[t][o1][a][rho] (A*O1*P values per token, 21 MB for the ring
// 25600 -> 5120 at rank 32) crosses HBM twice and both launches are bound by it (Section 3.5: the time
// goes to memory locality, not to FLOPs). Here every term of the sum over rho is finished on chip:
//   * a wave owns one token and a chunk of 32*O1T values of o1; X_t sits in its registers as MFMA row
//     operands (a along the rows, k contracted) for the whole launch;
//   * per rho the workgroup (4 waves = 4 tokens) streams the two slices B0[(o1 chunk, rho)][:] and
//     B1[:][(:, rho)] (tens of KB, stored contiguously per rho at create time by the repack kernels) into
//     a ring of 3 LDS stages with direct-to-LDS loads;
//   * D[a][o1] = X_t^T B0_rho^T lands in the accumulator layout (lane: o1 = l%32, a = 8*(v/4) + 4*(l/32)
//     + v%4), which after rounding to bf16 IS the column operand of the second contraction
//     Y^T[o2][o1] += B1_rho[o2][a] D[a][o1] when B1's slice is stored with the same permutation of a
//     inside each k-step of 16.
// The slices are the same for every token, so the workgroups of an XCD, which walk rho in step, read
// them from that XCD's L2; HBM sees X once, Y once and the packed tensors once per XCD.
// Few tokens: the range of rho is split over workgroups, each writes fp32 partial sums, and a second
// small kernel adds them in a fixed order. One or two tokens: a wave per token would leave three of a CU's four
// matrix cores idle while one wave works through 16 * AT * O1T MFMAs per value of the bond (six times the time the
// slices take to arrive), so the four waves share the token (KronArgs::share).
// Template: AT tiles of 32 values of a, KS0 k-steps of 16 in the first contraction, O2T tiles of 32
// values of o2, O1T tiles of 32 values of o1 per chunk; smaller shapes run on zero padding (the repacked
// slices hold zeros there).
// ---------------------------------------------------------------------------------------------
struct KronArgs {
    const void* X;
    void* Y;               // bf16 output, or fp32 partial sums [split][tokens][M] when n_splits > 1
    const void* H0f;       // [o1 chunk][rho][o1 tile (O1T)][k-step (KS0)] blocks of 512
    const void* H1f;       // [rho][o2 tile (O2T)][a k-step (2*AT)] blocks of 512
    const int32_t* xrow;   // offset of a in a token of x (null: a*K0)
    const int32_t* xcol;   // offset of k (null: k)
    const int32_t* yrow;   // output offset of o1
    const int32_t* ycol;   // output offset of o2
    int64_t N, M;          // elements per token of X and Y
    int32_t tokens, A, K0, O1, C1, P;
    int32_t n_chunks;      // ceil(O1 / (32*O1T))
    int32_t n_splits;      // workgroups sharing one (token quad, chunk): each takes rho_per_split values of rho
    int32_t rho_per_split;
    int32_t x_vec8;        // 8 consecutive k of one a are one aligned 16-byte piece of x
    int32_t tpw;           // tokens per wave (the TPW instantiation): 1 or 2
    int32_t share;         // one token (the SHARE instantiation): the four waves of a workgroup share ONE token (the workgroup's index
                           // counts tokens, not quads): per value of the bond its (o1 tile, a tile) units are dealt
                           // round-robin to the waves, whose sums are added through LDS in wave order at the end
};

template <int AT, int KS0, int O2T, int O1T>
struct KronShape {
    static constexpr int NB0 = O1T * KS0;               // blocks of 1 KB per rho: first slice
    static constexpr int NB1 = O2T * 2 * AT;            // second slice
    static constexpr int L = (NB0 + NB1 + 3) / 4;       // direct-to-LDS loads per wave and stage
    static constexpr int STAGE_BYTES = 4 * L * 1024;
    static constexpr int NS = 3;
    static constexpr size_t SMEM = size_t(NS) * STAGE_BYTES;
};

// H0f[((chunk*P + rho)*O1T*KS0 + o1t*KS0 + ks)*512 + l*8 + e] = B0[c = o1*P + rho][k = 16*ks + 8*(l/32) + e],
// o1 = 32*O1T*chunk + 32*o1t + l%32; zero outside the tensor.
__global__ void __launch_bounds__(256) kron_repack0_kernel(const bf16_t* src, bf16_t* dst, int n_chunks, int P, int KS0,
                                                           int O1T, int O1, int K0, int nks_src) {
    const int64_t total = int64_t(n_chunks) * P * O1T * KS0 * 512;
    for (int64_t i = int64_t(blockIdx.x) * 256 + threadIdx.x; i < total; i += int64_t(gridDim.x) * 256) {
        int e = int(i & 7), l = int(i >> 3) & 63;
        int64_t blk = i >> 9;
        int ks = int(blk % KS0);
        blk /= KS0;
        int o1t = int(blk % O1T);
        blk /= O1T;
        int rho = int(blk % P);
        int chunk = int(blk / P);
        int o1 = 32 * O1T * chunk + 32 * o1t + (l & 31);
        int k = 16 * ks + 8 * (l >> 5) + e;
        dst[i] = (o1 < O1 && k < K0) ? src[bfrag_offset(o1 * P + rho, k, nks_src)] : bf16_t(0.f);
    }
}

// H1f[((rho*O2T + j)*2*AT + 2*i + s)*512 + l*8 + e] = B1[c = 32*j + l%32][k = a*P + rho],
// a = 32*i + 16*s + 8*(e/4) + 4*(l/32) + e%4; zero outside the tensor.
__global__ void __launch_bounds__(256) kron_repack1_kernel(const bf16_t* src, bf16_t* dst, int P, int O2T, int AT, int C1,
                                                           int A, int nks_src) {
    const int64_t total = int64_t(P) * O2T * 2 * AT * 512;
    for (int64_t i = int64_t(blockIdx.x) * 256 + threadIdx.x; i < total; i += int64_t(gridDim.x) * 256) {
        int e = int(i & 7), l = int(i >> 3) & 63;
        int64_t blk = i >> 9;
        int is = int(blk % (2 * AT));
        blk /= 2 * AT;
        int j = int(blk % O2T);
        int rho = int(blk / O2T);
        int c = 32 * j + (l & 31);
        int a = 16 * is + 8 * (e >> 2) + 4 * (l >> 5) + (e & 3);
        dst[i] = (c < C1 && a < A) ? src[bfrag_offset(c, a * P + rho, nks_src)] : bf16_t(0.f);
    }
}

// SHARE: the one-token form (KronArgs::share): a compile-time switch, so that the loop of the many-token form stays
// one straight line of MFMAs and LDS reads (with the test inside it that loop ran 7 % slower).
// TPW: tokens per wave (1 or 2). With two, a wave reads every slice fragment from LDS once for both tokens and has
// two independent MFMA chains per unit to interleave: used for the instantiations whose slices are small against their
// MFMA work per token (fewer than 100 MFMAs per 32 KB of slice), where one token per wave left the matrix cores
// waiting on LDS, and only for calls with tokens enough to fill the chip in groups of eight.
template <int AT, int KS0, int O2T, int O1T, int SHARE, int TPW>
__global__ void __launch_bounds__(256, 1) step_kronsum_kernel(KronArgs p) {
    static_assert(TPW == 1 || !SHARE, "the shared form is for one token");
    using S = KronShape<AT, KS0, O2T, O1T>;
    constexpr int L = S::L, NS = S::NS, NB0 = S::NB0, NB1 = S::NB1, STAGE_BYTES = S::STAGE_BYTES;
    extern __shared__ __attribute__((aligned(16))) unsigned char dyn_smem[];

    const bf16_t* X = static_cast<const bf16_t*>(p.X);
    const bf16_t* H0f = static_cast<const bf16_t*>(p.H0f);
    const bf16_t* H1f = static_cast<const bf16_t*>(p.H1f);
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);

    // workgroup -> (token quad, chunk of o1, split of rho)
    int id = blockIdx.x;
    const int split = id % p.n_splits;
    id /= p.n_splits;
    const int chunk = id % p.n_chunks;
    const int quad = id / p.n_chunks;
    const int t = SHARE ? quad : (quad * 4 + wave) * TPW;      // the wave's first token (its second is t + 1)
    // waves past the end repeat the last token and store nothing
    const int rho_begin = split * p.rho_per_split;
    const int rho_end = min(p.P, rho_begin + p.rho_per_split);
    const int n_rho = rho_end - rho_begin;               // >= 1 by construction of the grid

    // the token's input as row operands of the first contraction: tile i, k-step ks: lane l holds
    // a = 32*i + l%32, k = 16*ks + 8*(l/32) .. +7
    bf16x8 xa[TPW][AT][KS0];
#pragma unroll
    for (int tp = 0; tp < TPW; ++tp) {
        const bf16_t* xt = X + int64_t(min(t + tp, p.tokens - 1)) * p.N;
        if (p.x_vec8) {
            // Straight-line code: offsets first (clamped into the tables), then all AT * KS0 loads back to back,
            // values outside the matrix replaced by zeros afterwards. With a branch around every load each one
            // waited for the one before, which cost a small call more than its contractions.
            int ro[AT], co[KS0];
            bool va[AT], vk[KS0];
#pragma unroll
            for (int i = 0; i < AT; ++i) {
                const int a = 32 * i + (lane & 31);
                va[i] = a < p.A;
                const int ac = min(a, p.A - 1);
                ro[i] = p.xrow ? p.xrow[ac] : ac * p.K0;
            }
#pragma unroll
            for (int ks = 0; ks < KS0; ++ks) {
                const int k = 16 * ks + 8 * (lane >> 5);
                vk[ks] = k < p.K0;                       // K0 % 8 == 0: then k + 8 <= K0 as well
                const int kc = min(k, p.K0 - 8);
                co[ks] = p.xcol ? p.xcol[kc] : kc;
            }
            bf16x8 zero;
#pragma unroll
            for (int e = 0; e < 8; ++e) zero[e] = bf16_t(0.f);
#pragma unroll
            for (int i = 0; i < AT; ++i)
#pragma unroll
                for (int ks = 0; ks < KS0; ++ks) {
                    const bf16x8 v = *reinterpret_cast<const bf16x8*>(xt + ro[i] + co[ks]);
                    xa[tp][i][ks] = (va[i] && vk[ks]) ? v : zero;
                }
        } else {
            // element-wise gather (the k of one a are not contiguous in x); the straight-line form measured slower here
#pragma unroll
            for (int i = 0; i < AT; ++i) {
                const int a = 32 * i + (lane & 31);
                const int ro = a < p.A ? (p.xrow ? p.xrow[a] : a * p.K0) : -1;
#pragma unroll
                for (int ks = 0; ks < KS0; ++ks) {
                    const int k = 16 * ks + 8 * (lane >> 5);
                    bf16x8 v;
#pragma unroll
                    for (int e = 0; e < 8; ++e) v[e] = bf16_t(0.f);
                    if (ro >= 0 && k < p.K0) {
#pragma unroll
                        for (int e = 0; e < 8; ++e) v[e] = xt[ro + p.xcol[k + e]];
                    }
                    xa[tp][i][ks] = v;
                }
            }
        }
    }

    // direct-to-LDS: wave w brings blocks w, w+4, ... of a stage (L each; blocks past the two slices repeat the
    // last one into the stage's padding so that every wave has the same number of loads in flight)
    const bf16_t* h0_src = H0f + (int64_t(chunk) * p.P) * (NB0 * 512) + lane * 8;
    const bf16_t* h1_src = H1f + lane * 8;
    auto issue = [&](int rho, int stage) {
        unsigned char* sbase = dyn_smem + stage * STAGE_BYTES;
#pragma unroll
        for (int q = 0; q < L; ++q) {
            const int b = wave + 4 * q;                  // wave-uniform
            const int bs = min(b, NB0 + NB1 - 1);
            const bf16_t* src = bs < NB0 ? h0_src + (int64_t(rho) * NB0 + bs) * 512
                                         : h1_src + (int64_t(rho) * NB1 + (bs - NB0)) * 512;
            __builtin_amdgcn_global_load_lds((const void __attribute__((address_space(1)))*)src,
                                             (void __attribute__((address_space(3)))*)(sbase + b * 1024), 16, 0, 0);
        }
    };

    floatx16 acc[TPW][O2T][O1T];
#pragma unroll
    for (int tp = 0; tp < TPW; ++tp)
#pragma unroll
        for (int j = 0; j < O2T; ++j)
#pragma unroll
            for (int o = 0; o < O1T; ++o)
#pragma unroll
                for (int v = 0; v < 16; ++v) acc[tp][j][o][v] = 0.f;

    issue(rho_begin, 0);
    if (n_rho > 1) issue(rho_begin + 1, 1);
    for (int r = 0; r < n_rho; ++r) {
        if (r + 1 < n_rho) wait_vmcnt<L>();              // stage r has landed (r+1 may be in flight)
        else wait_vmcnt<0>();
        __syncthreads();                                 // ... for every wave, and stage r-1 is free
        if (r + 2 < n_rho) issue(rho_begin + r + 2, (r + 2) % NS);
        const unsigned char* sb = dyn_smem + (r % NS) * STAGE_BYTES + lane * 16;
#pragma unroll
        for (int o = 0; o < O1T; ++o) {
            bf16x8 h0[KS0];
#pragma unroll
            for (int ks = 0; ks < KS0; ++ks) h0[ks] = *reinterpret_cast<const bf16x8*>(sb + (o * KS0 + ks) * 1024);
#pragma unroll
            for (int i = 0; i < AT; ++i) {
                if (SHARE && ((o * AT + i) & 3) != wave) continue;         // wave-uniform: another wave's unit
                bf16x8 h1[O2T][2];
#pragma unroll
                for (int j = 0; j < O2T; ++j)
#pragma unroll
                    for (int s = 0; s < 2; ++s)
                        h1[j][s] = *reinterpret_cast<const bf16x8*>(sb + (NB0 + (j * AT + i) * 2 + s) * 1024);
                floatx16 d[TPW];
#pragma unroll
                for (int tp = 0; tp < TPW; ++tp)
#pragma unroll
                    for (int v = 0; v < 16; ++v) d[tp][v] = 0.f;
#pragma unroll
                for (int ks = 0; ks < KS0; ++ks)
#pragma unroll
                    for (int tp = 0; tp < TPW; ++tp)
                        d[tp] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(xa[tp][i][ks], h0[ks], d[tp], 0, 0, 0);
                // registers 8s .. 8s+7 are the 8 values of a this lane supplies to k-step s
                bf16x8 zb[TPW][2];
#pragma unroll
                for (int tp = 0; tp < TPW; ++tp)
#pragma unroll
                    for (int s = 0; s < 2; ++s)
#pragma unroll
                        for (int e = 0; e < 8; ++e) zb[tp][s][e] = bf16_t(d[tp][8 * s + e]);
#pragma unroll
                for (int s = 0; s < 2; ++s)
#pragma unroll
                    for (int j = 0; j < O2T; ++j)
#pragma unroll
                        for (int tp = 0; tp < TPW; ++tp)
                            acc[tp][j][o] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(h1[j][s], zb[tp][s], acc[tp][j][o], 0, 0, 0);
            }
        }
        // keep the accumulators in the accumulation registers across the back edge
#pragma unroll
        for (int tp = 0; tp < TPW; ++tp)
#pragma unroll
            for (int j = 0; j < O2T; ++j)
#pragma unroll
                for (int o = 0; o < O1T; ++o) asm volatile("" : "+a"(acc[tp][j][o]));
    }

    if (SHARE) {
        // the four waves hold sums over disjoint sets of a: add them in wave order in LDS (the stages are dead), then
        // every wave takes back the tiles it stores (tile j*O1T + o belongs to wave (j*O1T + o) % 4)
        static_assert(size_t(O2T) * O1T * 4096 <= S::SMEM, "the shared sums fit the stages' LDS");
        float* red = reinterpret_cast<float*>(dyn_smem);
        __syncthreads();
        for (int w = 0; w < 4; ++w) {
            if (wave == w) {
#pragma unroll
                for (int j = 0; j < O2T; ++j)
#pragma unroll
                    for (int o = 0; o < O1T; ++o)
#pragma unroll
                        for (int v = 0; v < 16; ++v) {
                            float* q = red + ((j * O1T + o) * 16 + v) * 64 + lane;
                            *q = w == 0 ? acc[0][j][o][v] : *q + acc[0][j][o][v];
                        }
            }
            __syncthreads();
        }
#pragma unroll
        for (int j = 0; j < O2T; ++j)
#pragma unroll
            for (int o = 0; o < O1T; ++o)
                if (((j * O1T + o) & 3) == wave) {
#pragma unroll
                    for (int v = 0; v < 16; ++v) acc[0][j][o][v] = red[((j * O1T + o) * 16 + v) * 64 + lane];
                }
    }
    // lane l, register v of acc[j][o]: o2 = 32*j + 8*(v/4) + 4*(l/32) + v%4, o1 = 32*O1T*chunk + 32*o + l%32
    int yr[O1T];
#pragma unroll
    for (int o = 0; o < O1T; ++o) {
        const int o1 = 32 * O1T * chunk + 32 * o + (lane & 31);
        yr[o] = o1 < p.O1 ? p.yrow[o1] : -1;
    }
#pragma unroll
    for (int tp = 0; tp < TPW; ++tp) {
        if (t + tp >= p.tokens) break;
        bf16_t* yb = static_cast<bf16_t*>(p.Y) + int64_t(t + tp) * p.M;
        float* yf = static_cast<float*>(p.Y) + (int64_t(split) * p.tokens + t + tp) * p.M;
#pragma unroll
        for (int j = 0; j < O2T; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int o2 = 32 * j + 8 * (v >> 2) + 4 * (lane >> 5) + (v & 3);
                if (o2 >= p.C1) continue;
                const int yc = p.ycol[o2];
#pragma unroll
                for (int o = 0; o < O1T; ++o) {
                    if (yr[o] < 0 || (SHARE && ((j * O1T + o) & 3) != wave)) continue;
                    if (p.n_splits > 1) yf[yr[o] + yc] = acc[tp][j][o][v];
                    else yb[yr[o] + yc] = bf16_t(acc[tp][j][o][v]);
                }
            }
    }
}

// Y[i] = bf16( sum_s partial[s][i] ) for n = tokens * M values (n % 4 == 0). A workgroup owns 64 consecutive
// values: thread (g, q) adds the splits q, q+16, ... of values 4g .. 4g+3, then the 16 partial sums are added in
// the order of q. The order of the additions depends only on n_splits.
__global__ void __launch_bounds__(256) kron_reduce_kernel(const float* partial, bf16_t* Y, int64_t n, int n_splits) {
    __shared__ floatx4 part[16][16];
    const int g = threadIdx.x & 15, q = threadIdx.x >> 4;
    const int64_t i = (int64_t(blockIdx.x) * 16 + g) * 4;
    floatx4 s = {0.f, 0.f, 0.f, 0.f};
    if (i < n) {
#pragma unroll 4
        for (int k = q; k < n_splits; k += 16) s += *reinterpret_cast<const floatx4*>(partial + int64_t(k) * n + i);
    }
    part[q][g] = s;
    __syncthreads();
    if (q == 0 && i < n) {
        floatx4 t = part[0][g];
#pragma unroll
        for (int k = 1; k < 16; ++k) t += part[k][g];
        typedef __bf16 bf16x4_t __attribute__((ext_vector_type(4)));
        bf16x4_t o;
#pragma unroll
        for (int e = 0; e < 4; ++e) o[e] = bf16_t(t[e]);
        *reinterpret_cast<bf16x4_t*>(Y + i) = o;
    }
}

// ---------------------------------------------------------------------------------------------
// The two slice arrays above, computed from the caller's tensors instead of read from a stored merged
// tensor: each element is one entry of the contraction of two tensors P and Q over the indices they
// share (a half ring: two neighbouring cores over their common bond),
//     merged[r][c] = sum_s P[off_r(r) + off_s(s)] * Q[off_c(c) + off_s'(s)]        row-major [R][C],
// taken at the position the step's packing and the slice layout assign to it. This lets a layer keep
// only its compact tensors: the slices (tens of MB) are rebuilt in the shared workspace by every large
// call, which costs a fraction of a millisecond against the milliseconds of the call itself.
// The library keeps P and Q as matrices with the shared indices innermost (Pc[r][s], Qc[c][s], rows padded
// with zeros to a multiple of 8), written once at create time by kron_source_kernel, so that an entry is
// the dot product of two contiguous rows.
// ---------------------------------------------------------------------------------------------
struct GenDims {
    int32_t n;
    int32_t ext[tn::kMaxGatherDims];
    int64_t str[tn::kMaxGatherDims];
};

__host__ __device__ __forceinline__ int64_t gen_offset(const GenDims& d, int64_t idx) {
    int64_t off = 0;
    for (int j = d.n - 1; j >= 0; --j) {
        int64_t q = idx / d.ext[j];
        off += (idx - q * d.ext[j]) * d.str[j];
        idx = q;
    }
    return off;
}

// dst[r*Sp + s] = src[off_free(r) + off_shared(s)], zero for s >= S
__global__ void __launch_bounds__(256) kron_source_kernel(const bf16_t* src, bf16_t* dst, GenDims free_dims, GenDims shared_dims,
                                                          int64_t rows, int32_t S, int32_t Sp) {
    const int64_t total = rows * Sp;
    for (int64_t i = int64_t(blockIdx.x) * 256 + threadIdx.x; i < total; i += int64_t(gridDim.x) * 256) {
        const int64_t r = i / Sp;
        const int32_t sidx = int32_t(i - r * Sp);
        dst[i] = sidx < S ? src[gen_offset(free_dims, r) + gen_offset(shared_dims, sidx)] : bf16_t(0.f);
    }
}

struct KronGenArgs {
    const void* Pc;        // [R][Sp]
    const void* Qc;        // [C][Sp]
    void* dst;
    GenDims sc, sk;        // the step's column / k index -> offset in the merged tensor (row-major [R][C])
    int64_t merged_C;
    int32_t Sp;            // padded length of the shared indices, a multiple of 8
    int32_t which;         // 0: first slice array (H0f), 1: second (H1f)
    int32_t n_chunks, P, KS0, O1T, O1, K0;   // layout of H0f
    int32_t O2T, AT, C1, A;                  // layout of H1f
};

// One thread per 16-byte piece (8 consecutive elements) of a slice array.
__global__ void __launch_bounds__(256) kron_generate_kernel(KronGenArgs p) {
    const int64_t pieces = p.which == 0 ? int64_t(p.n_chunks) * p.P * p.O1T * p.KS0 * 64 : int64_t(p.P) * p.O2T * 2 * p.AT * 64;
    const bf16_t* Pc = static_cast<const bf16_t*>(p.Pc);
    const bf16_t* Qc = static_cast<const bf16_t*>(p.Qc);
    bf16x8* dst = static_cast<bf16x8*>(p.dst);
    for (int64_t i = int64_t(blockIdx.x) * 256 + threadIdx.x; i < pieces; i += int64_t(gridDim.x) * 256) {
        const int l = int(i & 63);
        int64_t blk = i >> 6;
        // position of the piece's 8 elements in the step's packed matrix B[c][k]
        int64_t c0, k0;
        int64_t k_step4, k_step1;              // element e: c = c0, k = k0 + (e/4)*k_step4 + (e%4)*k_step1
        int n_inside = 8;                      // first array: elements e < n_inside are inside the tensor
        bool row_inside;
        int limit_a = 0;
        if (p.which == 0) {
            int ks = int(blk % p.KS0);
            blk /= p.KS0;
            int o1t = int(blk % p.O1T);
            blk /= p.O1T;
            int rho = int(blk % p.P);
            int chunk = int(blk / p.P);
            int o1 = 32 * p.O1T * chunk + 32 * o1t + (l & 31);
            k0 = 16 * ks + 8 * (l >> 5);
            c0 = int64_t(o1) * p.P + rho;
            row_inside = o1 < p.O1;
            k_step4 = 4;
            k_step1 = 1;
            n_inside = int(max(int64_t(0), min(int64_t(8), int64_t(p.K0) - k0)));
        } else {
            int is = int(blk % (2 * p.AT));
            blk /= 2 * p.AT;
            int j = int(blk % p.O2T);
            int rho = int(blk / p.O2T);
            c0 = 32 * j + (l & 31);
            int a0 = 16 * is + 4 * (l >> 5);            // a = a0 + 8*(e/4) + e%4
            k0 = int64_t(a0) * p.P + rho;
            row_inside = c0 < p.C1;
            k_step4 = 8 * int64_t(p.P);
            k_step1 = p.P;
            limit_a = a0;
        }
        bf16x8 out;
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            float v = 0.f;
            bool inside = row_inside;
            if (p.which == 0) inside = inside && e < n_inside;
            else inside = inside && (limit_a + 8 * (e >> 2) + (e & 3)) < p.A;
            if (inside) {
                const int64_t k = k0 + (e >> 2) * k_step4 + (e & 3) * k_step1;
                const int64_t m = gen_offset(p.sc, c0) + gen_offset(p.sk, k);
                const int64_t r = m / p.merged_C, cc = m - r * p.merged_C;
                const bf16x8* pr = reinterpret_cast<const bf16x8*>(Pc + r * p.Sp);
                const bf16x8* qr = reinterpret_cast<const bf16x8*>(Qc + cc * p.Sp);
                for (int j = 0; j < (p.Sp >> 3); ++j) {
                    const bf16x8 a = pr[j], b = qr[j];
#pragma unroll
                    for (int q = 0; q < 8; ++q) v += float(a[q]) * float(b[q]);
                }
            }
            out[e] = bf16_t(v);
        }
        dst[i] = out;
    }
}

// ---------------------------------------------------------------------------------------------
// The same slices by MFMA, one workgroup per value rho of the shared bond. For a fixed rho the entries of
// a slice array are all products of one row of one source matrix with one row of the other: with r numbering
// the rows that occur of the "row-side" matrix Rc (rho's own contribution taken out) and c those of the
// "column-side" matrix Cc,
//     G[r][c] = sum_s Rc[rhoR[rho] + rowR[r]][s] * Cc[rhoC[rho] + rowC[c]][s]
// is a small matrix product (at most 160 x 160 x 128). The workgroup computes it in 32x32 tiles straight
// from the two source matrices (their rows are MFMA operand fragments as they lie in memory), writes the
// tiles to LDS as a bf16 matrix (a lane holds one r and runs of 4 consecutive c: 8-byte writes), and then
// assembles the slice's 16-byte pieces from it: a table made at create time gives, for each piece of one
// rho, the LDS positions of its 8 elements (the map does not depend on rho). The host picks which of the
// merge's two tensors is the column side, and the order in which the kernels number k and a, such that the 8
// elements of a piece are consecutive columns of G wherever the shapes allow (contig 1: one 16-byte read;
// contig 2: two runs of 4, for the slice whose k-steps are permuted; 0: eight 2-byte reads). 40-120 MFMAs
// replace the 10^4 dot products of 32-96 terms that the scalar kernel above spends per rho, which matters for
// calls of tens of tokens at high rank.
// ---------------------------------------------------------------------------------------------
struct KronGenMfmaArgs {
    const void* Rc;            // row-side source matrix [rows][Sp], Sp a multiple of 16, zero padded
    const void* Cc;            // column-side source matrix
    void* dst;                 // the slice array, in 16-byte pieces
    const int32_t* rowR;       // NR row numbers of Rc (for rho = 0)
    const int32_t* rowC;       // NC row numbers of Cc
    const int32_t* rhoR;       // P row offsets: what rho adds to a row number of Rc
    const int32_t* rhoC;
    const void* tab;           // per piece of one rho: 8 x uint16 positions r*LDC + c in the LDS matrix, 0xFFFF = zero
    int32_t NR, NC, LDC, Sp;   // LDC >= NC rounded up to 32, a multiple of 8
    int32_t pieces_per_rho;    // over all chunks
    int32_t pieces_per_chunk;  // blocks per rho and chunk x 64
    int32_t P;
    int32_t contig;
};

// One 16-byte piece from the product matrix in LDS.
__device__ __forceinline__ bf16x8 kron_gather_piece(const bf16_t* G, const unsigned (&t)[4], int contig) {
    typedef __bf16 bf16x4_t __attribute__((ext_vector_type(4)));
    bf16x8 out;
    const unsigned p0 = t[0] & 0xFFFFu, p4 = t[2] & 0xFFFFu;
    if (contig == 1) {
        if (p0 == 0xFFFFu) {
#pragma unroll
            for (int e = 0; e < 8; ++e) out[e] = bf16_t(0.f);
        } else {
            out = *reinterpret_cast<const bf16x8*>(G + p0);
        }
    } else if (contig == 2) {
        bf16x4_t lo, hi;
#pragma unroll
        for (int e = 0; e < 4; ++e) lo[e] = hi[e] = bf16_t(0.f);
        if (p0 != 0xFFFFu) lo = *reinterpret_cast<const bf16x4_t*>(G + p0);
        if (p4 != 0xFFFFu) hi = *reinterpret_cast<const bf16x4_t*>(G + p4);
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            out[e] = lo[e];
            out[4 + e] = hi[e];
        }
    } else {
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            const unsigned pos = (t[e >> 1] >> (16 * (e & 1))) & 0xFFFFu;
            out[e] = pos == 0xFFFFu ? bf16_t(0.f) : G[pos];
        }
    }
    return out;
}

template <int KSS /* k-steps of 16 along the shared bond */>
__device__ __forceinline__ void kron_generate_mfma_body(const KronGenMfmaArgs& p, int rho) {
    extern __shared__ __attribute__((aligned(16))) unsigned char dyn_smem[];
    typedef __bf16 bf16x4_t __attribute__((ext_vector_type(4)));
    bf16_t* G = reinterpret_cast<bf16_t*>(dyn_smem);
    const bf16_t* Rc = static_cast<const bf16_t*>(p.Rc);
    const bf16_t* Cc = static_cast<const bf16_t*>(p.Cc);
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int RT = (p.NR + 31) >> 5, CT = (p.NC + 31) >> 5;
    const int64_t baseR = p.rhoR[rho], baseC = p.rhoC[rho];
    const int kofs = 8 * (lane >> 5);
    bf16x8 zero;
#pragma unroll
    for (int e = 0; e < 8; ++e) zero[e] = bf16_t(0.f);

    // tiles (ct, rt): wave w takes the row tiles rt = w, w+4, ...; the MFMA's row operand is the column side, so
    // that a lane ends up with one r (l%32) and, in registers 4q..4q+3, the columns 32*ct + 8q + 4*(l/32) + 0..3
    for (int rt = wave; rt < RT; rt += 4) {
        const int r = 32 * rt + (lane & 31);
        bf16x8 b[KSS];
        {
            const bf16_t* row = Rc + (baseR + (r < p.NR ? p.rowR[r] : 0)) * p.Sp + kofs;
#pragma unroll
            for (int ks = 0; ks < KSS; ++ks)
                b[ks] = (r < p.NR && 16 * ks < p.Sp) ? *reinterpret_cast<const bf16x8*>(row + 16 * ks) : zero;
        }
        for (int ct = 0; ct < CT; ++ct) {
            const int c = 32 * ct + (lane & 31);
            const bf16_t* row = Cc + (baseC + (c < p.NC ? p.rowC[c] : 0)) * p.Sp + kofs;
            floatx16 acc;
#pragma unroll
            for (int i = 0; i < 16; ++i) acc[i] = 0.f;
#pragma unroll
            for (int ks = 0; ks < KSS; ++ks) {
                const bf16x8 a = (c < p.NC && 16 * ks < p.Sp) ? *reinterpret_cast<const bf16x8*>(row + 16 * ks) : zero;
                acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b[ks], acc, 0, 0, 0);
            }
            if (r < p.NR) {
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    bf16x4_t pk;
#pragma unroll
                    for (int j = 0; j < 4; ++j) pk[j] = bf16_t(acc[4 * q + j]);
                    *reinterpret_cast<bf16x4_t*>(G + r * p.LDC + 32 * ct + 8 * q + 4 * (lane >> 5)) = pk;
                }
            }
        }
    }
    __syncthreads();
    typedef unsigned int uintx4 __attribute__((ext_vector_type(4)));
    const uintx4* tab = static_cast<const uintx4*>(p.tab);
    bf16x8* dst = static_cast<bf16x8*>(p.dst);
    for (int lp = tid; lp < p.pieces_per_rho; lp += 256) {
        const uintx4 tv = tab[lp];
        const unsigned t[4] = {tv[0], tv[1], tv[2], tv[3]};
        const bf16x8 out = kron_gather_piece(G, t, p.contig);
        const int chunk = lp / p.pieces_per_chunk, rem = lp - chunk * p.pieces_per_chunk;
        dst[(int64_t(chunk) * p.P + rho) * p.pieces_per_chunk + rem] = out;
    }
}

template <int KSS>
__global__ void __launch_bounds__(256) kron_generate_mfma_kernel(KronGenMfmaArgs p) {
    kron_generate_mfma_body<KSS>(p, blockIdx.x);
}

// Both halves in one launch (the usual case): workgroups 0 .. P0-1 build the first half's slices, the others the second's.
template <int KSS>
__global__ void __launch_bounds__(256) kron_generate_mfma_both_kernel(KronGenMfmaArgs p0, KronGenMfmaArgs p1) {
    if (int(blockIdx.x) < p0.P) kron_generate_mfma_body<KSS>(p0, blockIdx.x);
    else kron_generate_mfma_body<KSS>(p1, int(blockIdx.x) - p0.P);
}
