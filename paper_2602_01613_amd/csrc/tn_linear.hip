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

#include <cmath>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <mutex>
#include <new>
#include <type_traits>
#include <vector>

#include "../../include/tn_linear.h"
#include "tn_plan.hpp"

// Scratch memory of tn_linear_forward_scratch: one array per GPU the library is loaded on, held until the
// process ends. Host code never uses this name as an address; it asks the runtime for the device address once
// per device (scratch_address) and passes that pointer on.
constexpr int64_t kScratchBytes = int64_t(32) << 20;
static __device__ __align__(256) unsigned char scratch[kScratchBytes];

namespace {

#include "kernels/common.hpp"
#include "kernels/pack.hpp"
#include "kernels/quant.hpp"
#include "kernels/tiled.hpp"
#include "kernels/stream.hpp"
#include "kernels/chained.hpp"
#include "kernels/kronsum.hpp"
#include "kernels/grad.hpp"

// ---------------------------------------------------------------------------------------------
// host side
// ---------------------------------------------------------------------------------------------
enum Variant : int {
    VAR_SCALAR = 0,
    VAR_MFMA_256x32 = 2,      // narrow outputs (<= 32 columns)
    VAR_PIPE_128x256 = 3,     // register-prefetch tiles, 4 waves, 2 workgroups per CU, one LDS stage
    VAR_PIPE_256x128 = 8,     // same, 4 waves stacked along rows
    VAR_SHORTK = 9,           // K <= 64, store-bound: registers-only operands, barrier-free
    VAR_PINGPONG_256x256 = 12,   // 8 waves in two alternating groups, 1 workgroup per CU
    VAR_KRONSUM = 20,         // (as a forced id only, read by tn::kron_shape) the Kronecker-sum kernel wherever
                              // the plan's layout allows it
};

struct DevStep {
    tn::Step plan;
    void* packed = nullptr;       // [Cp][Kp]
    const int32_t *arow = nullptr, *acol = nullptr, *crow = nullptr, *ccol = nullptr;
    int Kp = 0, Cp = 0;
    int variant = VAR_SCALAR;
    int amode = 0, cmode = 0;
    int bn = 64, bm = 64;
    bool fuse_next = false;       // this step and the next run as one launch
    void* chain_bbf = nullptr;    // chain2: the next step's packed tensor in the chained layout
    int chain_cfg = 0;            // chain2 instantiation: 0 <3,6,5>, 1 <2,8,2>, 2 <2,5,2>
    int chain_run_c1 = 0;         // chain2: output pieces run along c1 (else along c2)
    void* q4_codes = nullptr;     // 4-bit stream of the tensor for decode-size launches (codes, then block scales)
    void* q4_scales = nullptr;
    bool no_skinny = false;       // TN_FLAG_NO_SKINNY
};

}  // namespace

struct tn_linear_s {
    tn::Plan plan;
    std::vector<DevStep> steps;
    int elt = 4;
    int64_t max_tokens = 0, chunk_tokens = 0;
    int64_t packed_bytes = 0, workspace_bytes = 0;
    int32_t* tables = nullptr;        // arow | acol | crow | ccol of every step, one allocation
    void* ws[2] = {nullptr, nullptr};
    void* partial = nullptr;          // fp32 partial sums of the split-K kernel
    int64_t partial_bytes = 0;
    std::vector<tn::LaunchIO> schedule;   // launches of one pass over the chain and the buffers they use
    int flags = 0;
    bool owns_workspace = true;
    int device = 0;
    int num_cus = 256;
    bool profiling = false;
    // whole chain in one launch with everything in LDS (small layers)
    bool small_chain = false;
    size_t small_chain_smem = 0;
    int small_chain_b_off[kSmallChainMaxSteps] = {};
    int small_chain_t_off[kSmallChainMaxSteps] = {};
    void* small_chain_image = nullptr;    // tensors (fp32, padded rows) and tables of all steps, as they sit in LDS
    int small_chain_image_words = 0;
    int small_chain_buf_off[2] = {0, 0};
    // chained pair kernel (two-step plans of the train shape): second packed tensor in its layout
    bool pair = false;
    void* pair_b1f = nullptr;
    int64_t pair_min_tokens = 0;
    // Kronecker-sum kernel (two-step plans over a shared bond): both packed tensors in per-bond slices
    bool kron = false;
    tn::KronDims kron_dims;
    void* kron_h0f = nullptr;
    void* kron_h1f = nullptr;
    int64_t kron_min_tokens = 0;
    // the same kernel on a plan that exists only for large calls: the layer keeps its compact tensors and
    // steps, and calls of at least lazy_min_tokens tokens rebuild the merged plan's slices in the workspace
    bool lazy = false;
    bool lazy_slices_kept = false;    // the slices sit in memory only this handle writes (its own workspace): built once, at create
    tn::Plan lazy_plan;
    tn::KronDims lazy_dims;
    int64_t lazy_min_tokens = 0;
    int64_t lazy_kept_bytes = 0;              // what the lazy plan added to packed_bytes (sources and tables)
    int64_t lazy_slice_bytes = 0;             // both slice arrays
    int64_t lazy_h1_offset = 0;               // byte offset of the second array inside the slice buffer
    void* lazy_slices = nullptr;              // in the workspace (owned or caller's)
    std::vector<void*> lazy_sources;          // per half: the two tensors it is made of, as matrices [free][shared]
    int32_t* lazy_tables = nullptr;           // xrow | xcol | yrow | ycol of the merged plan
    const int32_t *lazy_xrow = nullptr, *lazy_xcol = nullptr, *lazy_yrow = nullptr, *lazy_ycol = nullptr;
    KronGenArgs lazy_gen[2];
    // the same slices by MFMA (one workgroup per value of the bond), where the half's shape allows it
    bool lazy_mfma[2] = {false, false};
    KronGenMfmaArgs lazy_gen_mfma[2];
    size_t lazy_gen_smem[2] = {0, 0};
    void* lazy_gen_tables[2] = {nullptr, nullptr};
    // 4-bit form of the caller's tensors (TN_FLAG_QUANT_MXFP4): packed codes and block exponents per tensor
    std::vector<void*> quant_codes, quant_exps;
    std::vector<int64_t> quant_elems;
    int64_t quant_bytes = 0;
    int64_t q4_stream_bytes = 0;              // 4-bit streams of the steps whose decode-size launches read them
    std::vector<void*> create_temps;          // device buffers that only live until create returns
    // gradients with respect to the parameter tensors (TN_FLAG_TRAINABLE)
    bool trainable = false;
    std::vector<DevStep> bwd;                 // per step s >= 1: the step with its tensor transposed (gives dIn_s from dOut_s)
    int32_t* bwd_tables = nullptr;            // plain output tables of those steps
    void* bwd_ws = nullptr;                   // saved step inputs | two gradient buffers, for bwd_chunk tokens
    std::vector<int64_t> bwd_saved_off;       // element offset (per token block) of the saved input of step s
    int64_t bwd_saved_elems = 0;              // per token
    int64_t bwd_chunk = 0, bwd_ws_bytes = 0;
    float* bwd_partial = nullptr;
    int64_t bwd_partial_bytes = 0;
    struct ProfRec { int step; hipEvent_t start, stop; };
    std::vector<ProfRec> prof;
};

namespace {

constexpr int64_t kDefaultWorkspaceBytes = int64_t(4) << 30;

// The scratch memory a forward call works in: the two intermediate buffers (each holds chunk_tokens tokens
// of the largest intermediate) and the fp32 partial sums of the split kernels. Normally the handle's own
// workspace; tn_linear_forward_scratch carves it out of the library's static device array instead.
struct Workspace {
    void* ws[2] = {nullptr, nullptr};
    void* partial = nullptr;
    int64_t partial_bytes = 0;
    int64_t chunk_tokens = 0;
};

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
        if (s.chain_bbf) (void)hipFree(s.chain_bbf);
        if (s.q4_codes) (void)hipFree(s.q4_codes);       // one allocation: the scales follow the codes
    }
    if (h->tables) (void)hipFree(h->tables);
    for (void* v : h->quant_codes)
        if (v) (void)hipFree(v);
    for (void* v : h->quant_exps)
        if (v) (void)hipFree(v);
    for (void* v : h->create_temps)
        if (v) (void)hipFree(v);
    for (auto& b : h->bwd)
        if (b.packed) (void)hipFree(b.packed);
    if (h->bwd_tables) (void)hipFree(h->bwd_tables);
    if (h->bwd_ws) (void)hipFree(h->bwd_ws);
    if (h->bwd_partial) (void)hipFree(h->bwd_partial);
    if (h->pair_b1f) (void)hipFree(h->pair_b1f);
    if (h->kron_h0f) (void)hipFree(h->kron_h0f);
    if (h->kron_h1f) (void)hipFree(h->kron_h1f);
    for (void* v : h->lazy_sources)
        if (v) (void)hipFree(v);
    if (h->lazy_tables) (void)hipFree(h->lazy_tables);
    for (void* v : h->lazy_gen_tables)
        if (v) (void)hipFree(v);
    if (h->lazy_slices && h->owns_workspace) (void)hipFree(h->lazy_slices);
    if (h->small_chain_image) (void)hipFree(h->small_chain_image);
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
        const bool pingpong_ok = p.a_plain && p.K % 32 == 0 && p.K >= 64;
        // (measured: the 8-wave 256x256 ring beats the register-prefetch tiles on every shape it
        // fits without extra column padding; the 4-wave direct-to-LDS tiles do not)
        if (pingpong_ok && p.C >= 256 && round_up(int(p.C), 256) == round_up(int(p.C), 128)) v = VAR_PINGPONG_256x256;
        if (shortk_ok && p.C >= 256) v = VAR_SHORTK;
        if (forced == VAR_PIPE_128x256 || forced == VAR_PIPE_256x128 || (forced == VAR_SHORTK && shortk_ok) ||
            (forced == VAR_PINGPONG_256x256 && pingpong_ok))
            v = forced;
        s->variant = v;
        switch (v) {
            case VAR_SHORTK: s->bm = 128; s->bn = 128; break;
            case VAR_PIPE_128x256: s->bm = 128; s->bn = 256; break;
            case VAR_PIPE_256x128: s->bm = 256; s->bn = 128; break;
            default: s->bm = 256; s->bn = 256; break;      // VAR_PINGPONG_256x256
        }
    }
    // 0: plain rows of 16-byte pieces; 2: gathered rows of 16-byte pieces (the tiled pipeline kernel; every other kernel
    // reads such a step element by element, like 1); 1: element-wise gather
    s->amode = (p.a_plain && p.K % 8 == 0) ? 0 : (p.a_vec == 8 ? 2 : 1);
    s->cmode = p.c_vec == 8 ? 1 : (p.r_vec == 8 ? 2 : 0);
    s->Kp = round_up(int(p.K), 64);
    s->Cp = round_up(int(p.C), s->bn);
}

struct SplitCfg {
    bool use = false;
    int tm = 1, nw = 4, row_tiles = 0, col_blocks = 0, nsplit = 1, ksteps_per_split = 0;
    bool lds_rows = false;        // one row tile: the kernel that keeps the rows of A in LDS
    bool skinny = false;          // one row tile against 256 columns per workgroup (step_skinny_kernel)
    int64_t partial_bytes = 0;
};

constexpr int64_t kMaxPartialBytes = int64_t(64) << 20;
constexpr size_t kSplitLdsRowBytes = 144 * 1024;  // rows of A a split-K workgroup may keep in LDS (the reduction reuses it)
// Measured (dense 5120->8192 and 25600->5120, us per call, rows in LDS against rows gathered from memory): bf16 stream
// 1 row 17.5 / 19.3 and 56.3 / 60.0 (captured graph over 16 copies), 8 rows 18.6 / 15.8 (same layer back to back), 64
// rows (two row tiles, five splits to fit) 62.8 / 31.2; 4-bit stream 1 row 8.6 / 13.0, 8 rows 8.4 / 11.2, 64 rows
// 56.7 / 26.1. Hence: one row tile only; a bf16 stream up to 4 rows, a 4-bit stream up to 32.
constexpr int64_t kSplitLdsMaxBf16Rows = 4;
constexpr int64_t kSplitOneSplitBlocks = 128;
constexpr int kSkinnyFillWorkgroups = 256;       // compute units the skinny kernel's grid is planned for
constexpr int64_t kSkinnyLdsPerCu = 160 * 1024;  // LDS of a compute unit: bounds the workgroups it holds at a time
constexpr int64_t kSplitLdsMaxQ4Rows = 12;
constexpr int64_t kSkinnyMinRows = 8, kSkinnyMinRowsTimesK = 100000;

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
    if (c.row_tiles == 1 && base >= kSplitOneSplitBlocks) c.nsplit = 1;      // enough column blocks: no second pass over partial sums
    const bool rows_fit_as_planned =
        size_t(rows) * size_t(round_up((nks + c.nsplit - 1) / c.nsplit, 4) * 16 + 8) * 2 <= kSplitLdsRowBytes;
    const bool skinny_possible = c.row_tiles == 1 && nks % 4 == 0 && c.col_blocks >= 8 && !s.no_skinny;
    // a 4-bit stream whose rows would need extra splits to fit, or with many rows x K to copy per column block, goes
    // to the 256-column kernel instead
    if (c.row_tiles == 1 && c.tm == 1 && nks % 4 == 0 && rows <= (s.q4_codes ? kSplitLdsMaxQ4Rows : kSplitLdsMaxBf16Rows) &&
        !(s.q4_codes && skinny_possible && (!rows_fit_as_planned || rows * int64_t(s.plan.K) >= kSkinnyMinRowsTimesK))) {
        // the kernel that keeps the rows of A in LDS: enough splits that the rows' share of A fits (at least two
        // pieces of 64 k per wave stay in a split), and whole pieces of 64 k per split
        c.lds_rows = true;
        const int min_ksteps = 8 * c.nw;
        while (size_t(rows) * size_t(round_up((nks + c.nsplit - 1) / c.nsplit, 4) * 16 + 8) * 2 > kSplitLdsRowBytes &&
               (nks + c.nsplit) / (c.nsplit + 1) >= min_ksteps)
            ++c.nsplit;
    }
    if (!c.lds_rows && skinny_possible &&
        (rows > 32 || s.q4_codes || (rows >= kSkinnyMinRows && rows * int64_t(s.plan.K) >= kSkinnyMinRowsTimesK))) {
        // up to 64 rows against 256 columns per workgroup (step_skinny_kernel), every wave a column block of its own.
        // The number of splits (equal, whole pieces of 64 k, the rows' share of A within the LDS budget) is the one
        // with the least bytes on the critical path: the busiest CU runs ceil(grid / CUs) workgroups, each of which
        // moves its pieces of the stream and its rows of A (a quarter more when LDS leaves room for only one
        // workgroup per CU: nothing overlaps its start and end), and every split adds fp32 partial sums that are
        // written and read back.
        const int n_chunks = nks / 4, col_tiles = (c.col_blocks + 7) / 8;
        auto cps_of = [&](int ns) { return (n_chunks + ns - 1) / ns; };
        auto lds_bytes = [&](int ns) { return int64_t(rows) * (int64_t(cps_of(ns)) * 64 + 8) * 2; };
        const double stream_bytes_per_k = s.q4_codes ? 256 * 17.0 / 32.0 : 256 * 2.0;
        int best = 0;
        double best_cost = 0;
        for (int ns = 1; ns <= std::max(1, n_chunks / 2); ++ns) {
            if (ns > 1 && cps_of(ns) == cps_of(ns - 1)) continue;              // same pieces per split: more empty tail
            if (lds_bytes(ns) > int64_t(kSplitLdsRowBytes)) continue;
            const int n_real = (n_chunks + cps_of(ns) - 1) / cps_of(ns);
            const int64_t pb = n_real > 1 ? int64_t(n_real) * 32 * c.tm * s.Cp * 4 : 0;
            if (pb > kMaxPartialBytes) break;
            const int per_cu = int(std::max<int64_t>(1, std::min<int64_t>(4, kSkinnyLdsPerCu / std::max<int64_t>(1, lds_bytes(ns)))));
            const int64_t grid = int64_t(col_tiles) * n_real;
            const int64_t serial = (grid + kSkinnyFillWorkgroups - 1) / kSkinnyFillWorkgroups;      // workgroups the busiest CU runs
            const double wg_bytes = cps_of(ns) * 64.0 * (stream_bytes_per_k + 2.0 * double(rows));
            const double cost = double(serial) * wg_bytes * kSkinnyFillWorkgroups * (per_cu == 1 ? 1.25 : 1.0) + 2.0 * double(pb);
            if (!best || cost < best_cost) {
                best = ns;
                best_cost = cost;
            }
        }
        if (best) {
            const int cps = cps_of(best);
            c.skinny = true;
            c.nsplit = (n_chunks + cps - 1) / cps;
            c.ksteps_per_split = cps * 4;
            c.partial_bytes = c.nsplit > 1 ? int64_t(c.nsplit) * 32 * c.tm * s.Cp * 4 : 0;
            c.use = true;
            return c;
        }
    }
    for (;;) {
        c.ksteps_per_split = (nks + c.nsplit - 1) / c.nsplit;
        if (s.q4_codes || c.lds_rows) c.ksteps_per_split = round_up(c.ksteps_per_split, 4);    // pieces of 64 k
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
    static const kern_t kerns[6] = {
        step_mfma_pipe_kernel<WM, WN, TM, TN, 0, STAGES, MINB, 0>, step_mfma_pipe_kernel<WM, WN, TM, TN, 1, STAGES, MINB, 0>,
        step_mfma_pipe_kernel<WM, WN, TM, TN, 2, STAGES, MINB, 0>, step_mfma_pipe_kernel<WM, WN, TM, TN, 0, STAGES, MINB, 1>,
        step_mfma_pipe_kernel<WM, WN, TM, TN, 1, STAGES, MINB, 1>, step_mfma_pipe_kernel<WM, WN, TM, TN, 2, STAGES, MINB, 1>};
    if (!s.packed) {                       // configuration call (create time): raise the kernels' LDS limit
        for (kern_t k : kerns)
            if (hipFuncSetAttribute(reinterpret_cast<const void*>(k), hipFuncAttributeMaxDynamicSharedMemorySize,
                                    int(smem)) != hipSuccess)
                return TN_ERR_HIP;
        return TN_OK;
    }
    kern_t k = kerns[(s.cmode == 2 ? 3 : 0) + s.amode];
    hipLaunchKernelGGL(k, grid, dim3(WM * WN * 64), smem, st, a, s.cmode, nrow, ncol);
    return TN_OK;
}

// The 256x256 ping-pong kernel and its 256x128 form. A CU holds one workgroup, so a launch runs in rounds of
// num_cus tiles; when the last round would fill at most half of the CUs, its tiles run as a second launch of
// half-width tiles on twice as many workgroups (same walk over the tiles, see the kernel), which takes half a round.
using pingpong_kern_t = void (*)(StepArgs, int, int, int, int, int);

template <int TN, int TRANS>
pingpong_kern_t pingpong_kernel() { return step_mfma_pingpong_kernel<4, 2, 2, TN, 2, 1, TRANS>; }

int configure_pingpong() {
    const pingpong_kern_t wide[2] = {pingpong_kernel<4, 0>(), pingpong_kernel<4, 1>()};
    const pingpong_kern_t narrow[2] = {pingpong_kernel<2, 0>(), pingpong_kernel<2, 1>()};
    for (int i = 0; i < 2; ++i)
        if (hipFuncSetAttribute(reinterpret_cast<const void*>(wide[i]), hipFuncAttributeMaxDynamicSharedMemorySize,
                                int(pingpong_smem_bytes<4, 2, 2, 4, 2>())) != hipSuccess ||
            hipFuncSetAttribute(reinterpret_cast<const void*>(narrow[i]), hipFuncAttributeMaxDynamicSharedMemorySize,
                                int(pingpong_smem_bytes<4, 2, 2, 2, 2>())) != hipSuccess)
            return TN_ERR_HIP;
    return TN_OK;
}

int launch_pingpong(const tn_linear_s* h, const DevStep& s, const StepArgs& a, int64_t rows, hipStream_t st) {
    const int nrow = int((rows + 255) / 256), ncol = s.Cp / 256;
    const int trans = s.cmode == 2 ? 1 : 0;
    const pingpong_kern_t wide = trans ? pingpong_kernel<4, 1>() : pingpong_kernel<4, 0>();
    const pingpong_kern_t narrow = trans ? pingpong_kernel<2, 1>() : pingpong_kernel<2, 0>();
    const int slots = ((nrow + 7) / 8) * ncol;             // per XCD (workgroup i runs on XCD i % 8)
    const int per_xcd = h->num_cus / 8;
    int full = slots, rest = 0;
    if (nrow % 8 == 0 && h->num_cus % 8 == 0 && per_xcd > 0) {
        const int r = slots % per_xcd;
        if (r > 0 && 2 * r <= per_xcd) {
            rest = r;
            full = slots - r;
        }
    }
    constexpr size_t wide_smem = pingpong_smem_bytes<4, 2, 2, 4, 2>(), narrow_smem = pingpong_smem_bytes<4, 2, 2, 2, 2>();
    if (full > 0)
        hipLaunchKernelGGL(wide, dim3(uint32_t(8 * full)), dim3(512), wide_smem, st, a, s.cmode, nrow, ncol, 0, 0);
    if (rest > 0)
        hipLaunchKernelGGL(narrow, dim3(uint32_t(16 * rest)), dim3(512), narrow_smem, st, a, s.cmode, nrow, ncol, full, 1);
    return TN_OK;
}

// Instantiations of the split-K kernel that keeps the rows of A in LDS (one row tile of up to 32 rows): index
// (8 waves ? 4 : 0) + (gathered A ? 2 : 0) + (4-bit stream ? 1 : 0).
using split_lds_t = void (*)(StepArgs, float*, int, int);
constexpr int kSplitLdsKernels = 8;
const split_lds_t* split_lds_kernels() {
    static const split_lds_t lds[kSplitLdsKernels] = {
        step_split_lds_kernel<1, 0, 4, 0>, step_split_lds_kernel<1, 0, 4, 1>, step_split_lds_kernel<1, 1, 4, 0>,
        step_split_lds_kernel<1, 1, 4, 1>, step_split_lds_kernel<1, 0, 8, 0>, step_split_lds_kernel<1, 0, 8, 1>,
        step_split_lds_kernel<1, 1, 8, 0>, step_split_lds_kernel<1, 1, 8, 1>};
    return lds;
}

// step_skinny_kernel: index (tm - 1) * 4 + (gathered A ? 2 : 0) + (4-bit stream ? 1 : 0).
constexpr int kSkinnyKernels = 8;
using skinny_t = void (*)(StepArgs, float*, int, int, int);
const skinny_t* skinny_kernels() {
    static const skinny_t k[kSkinnyKernels] = {step_skinny_kernel<1, 0, 0>, step_skinny_kernel<1, 0, 1>, step_skinny_kernel<1, 1, 0>,
                                                  step_skinny_kernel<1, 1, 1>, step_skinny_kernel<2, 0, 0>, step_skinny_kernel<2, 0, 1>,
                                                  step_skinny_kernel<2, 1, 0>, step_skinny_kernel<2, 1, 1>};
    return k;
}

int launch_step(const tn_linear_s* h, const Workspace& w, const DevStep& s, const void* A, void* Out, int64_t tokens,
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
    if (sc.use && (sc.partial_bytes == 0 || (w.partial && sc.partial_bytes <= w.partial_bytes))) {
        dim3 sgrid(uint32_t(sc.row_tiles), uint32_t(sc.col_blocks), uint32_t(sc.nsplit));
        float* part = static_cast<float*>(w.partial);
        using split_t = void (*)(StepArgs, float*, int);
        split_t k = nullptr;
        const int q4 = s.q4_codes ? 1 : 0;
        if (q4) {
            // the launch is a stream of the packed tensor: read its 4-bit form
            a.B = s.q4_codes;
            a.Bs = s.q4_scales;
        }
        const int x_ld = sc.ksteps_per_split * 16 + 8;
        const size_t x_bytes = size_t(rows) * size_t(x_ld) * sizeof(bf16_t);
        if (sc.skinny) {
            if (x_bytes > kSplitLdsRowBytes) return TN_ERR_UNSUPPORTED;       // split_config sized it to fit
            const dim3 kgrid(1, uint32_t((sc.col_blocks + 7) / 8), uint32_t(sc.nsplit));
            hipLaunchKernelGGL(skinny_kernels()[(sc.tm - 1) * 4 + (s.amode == 0 ? 0 : 2) + q4], kgrid, dim3(512), x_bytes, st, a,
                               part, sc.ksteps_per_split, x_ld, s.plan.c_vec >= 4 ? 1 : 0);
        } else if (sc.lds_rows && sc.tm == 1 && sc.row_tiles == 1 && sc.ksteps_per_split % 4 == 0 && x_bytes <= kSplitLdsRowBytes) {
            // one row tile whose share of A fits in LDS
            const size_t red_bytes = size_t(sc.nw) * sc.tm * 4096;
            hipLaunchKernelGGL(split_lds_kernels()[(sc.nw == 8 ? 4 : 0) + (s.amode == 0 ? 0 : 2) + q4], sgrid,
                               dim3(uint32_t(sc.nw * 64)), std::max(red_bytes, x_bytes), st, a, part, sc.ksteps_per_split, x_ld);
        } else if (q4) {
            if (sc.tm == 1)
                k = sc.nw == 8 ? (s.amode == 0 ? step_split_q4_kernel<1, 0, 8> : step_split_q4_kernel<1, 1, 8>)
                               : (s.amode == 0 ? step_split_q4_kernel<1, 0, 4> : step_split_q4_kernel<1, 1, 4>);
            else
                k = sc.nw == 8 ? (s.amode == 0 ? step_split_q4_kernel<2, 0, 8> : step_split_q4_kernel<2, 1, 8>)
                               : (s.amode == 0 ? step_split_q4_kernel<2, 0, 4> : step_split_q4_kernel<2, 1, 4>);
        } else if (sc.tm == 1)
            k = sc.nw == 8 ? (s.amode == 0 ? step_split_kernel<1, 0, 8> : step_split_kernel<1, 1, 8>)
                           : (s.amode == 0 ? step_split_kernel<1, 0, 4> : step_split_kernel<1, 1, 4>);
        else
            k = sc.nw == 8 ? (s.amode == 0 ? step_split_kernel<2, 0, 8> : step_split_kernel<2, 1, 8>)
                           : (s.amode == 0 ? step_split_kernel<2, 0, 4> : step_split_kernel<2, 1, 4>);
        if (k) hipLaunchKernelGGL(k, sgrid, dim3(uint32_t(sc.nw * 64)), 0, st, a, part, sc.ksteps_per_split);
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
        case VAR_PINGPONG_256x256: {
            int rc = launch_pingpong(h, s, a, rows, st);
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

// Small layers: all steps in one launch when the packed tensors (as fp32, rows padded by one) and two
// per-token buffers fit in 96 KB of LDS. Used for fp32 layers at any token count (their other path is
// the plain FMA kernel, one launch per step) and for bf16 layers up to 32 tokens.
constexpr size_t kSmallChainMaxSmem = 96 * 1024;
constexpr int64_t kSmallChainMaxBf16Tokens = 32;

void fill_small_chain_args(const tn_linear_s* h, SmallChainArgs* a) {
    a->image = static_cast<const float*>(h->small_chain_image);
    a->N = h->plan.N;
    a->M = h->plan.M;
    a->nsteps = int32_t(h->steps.size());
    a->image_words = h->small_chain_image_words;
    a->buf_off[0] = h->small_chain_buf_off[0];
    a->buf_off[1] = h->small_chain_buf_off[1];
    for (size_t s = 0; s < h->steps.size(); ++s) {
        const DevStep& d = h->steps[s];
        SmallChainStep& o = a->st[s];
        o.B = d.packed;
        o.arow = d.arow;
        o.acol = d.acol;
        o.crow = d.crow;
        o.ccol = d.ccol;
        o.R = int32_t(d.plan.R);
        o.K = int32_t(d.plan.K);
        o.C = int32_t(d.plan.C);
        o.nks = d.Kp >> 4;
        o.b_off = h->small_chain_b_off[s];
        o.ldb = (o.K & 3) ? o.K + 1 : o.K + 4;
        o.t_off = h->small_chain_t_off[s];
        o.gathered = d.plan.a_plain ? 0 : 1;
    }
}

int plan_small_chain(tn_linear_s* h, hipStream_t st) {
    if (h->flags & (TN_FLAG_SCALAR_KERNELS | TN_FLAG_NO_SMALL_CHAIN)) return TN_OK;
    const size_t ns = h->steps.size();
    if (ns == 0 || ns > size_t(kSmallChainMaxSteps)) return TN_OK;
    int64_t off = 0;
    for (size_t s = 0; s < ns; ++s) {
        const tn::Step& p = h->steps[s].plan;
        if (p.R * p.C > (int64_t(1) << 20)) return TN_OK;
        h->small_chain_b_off[s] = int(off);
        off += (p.C * ((p.K & 3) ? p.K + 1 : p.K + 4) + 3) & ~int64_t(3);      // every tensor starts 16-byte aligned
        if (off > int64_t(kSmallChainMaxSmem / 4)) return TN_OK;
    }
    for (size_t s = 0; s < ns; ++s) {              // the offset tables
        const tn::Step& p = h->steps[s].plan;
        h->small_chain_t_off[s] = int(off);
        off += p.R + p.C + (p.a_plain ? 0 : p.R + p.K);
        if (off > int64_t(kSmallChainMaxSmem / 4)) return TN_OK;
    }
    off = (off + 3) & ~int64_t(3);
    const int64_t image_words = off;
    const int64_t buf = (std::max(h->plan.N, h->plan.max_intermediate) + 3) & ~int64_t(3);
    if ((off + 2 * buf) * 4 > int64_t(kSmallChainMaxSmem)) return TN_OK;
    h->small_chain_buf_off[0] = int(off);
    h->small_chain_buf_off[1] = int(off + buf);
    h->small_chain_smem = size_t(off + 2 * buf) * 4;
    h->small_chain_image_words = int(image_words);
    if (hipMalloc(&h->small_chain_image, size_t(image_words) * 4) != hipSuccess) return TN_ERR_ALLOC;
    h->packed_bytes += image_words * 4;
    SmallChainArgs a;
    memset(&a, 0, sizeof(a));
    fill_small_chain_args(h, &a);
    if (h->elt == 2)
        hipLaunchKernelGGL(small_chain_image_kernel<bf16_t>, dim3(1), dim3(256), 0, st, a, static_cast<float*>(h->small_chain_image));
    else
        hipLaunchKernelGGL(small_chain_image_kernel<float>, dim3(1), dim3(256), 0, st, a, static_cast<float*>(h->small_chain_image));
    if (hipGetLastError() != hipSuccess) return TN_ERR_HIP;
    h->small_chain = true;
    return TN_OK;
}

int launch_small_chain(const tn_linear_s* h, const void* x, void* y, int64_t tokens, hipStream_t st) {
    SmallChainArgs a;
    memset(&a, 0, sizeof(a));
    fill_small_chain_args(h, &a);
    a.X = x;
    a.Y = y;
    a.tokens = int32_t(tokens);
    dim3 grid(uint32_t(std::min<int64_t>(tokens, int64_t(h->num_cus) * 2)));
    if (h->elt == 2)
        hipLaunchKernelGGL(small_chain_kernel<bf16_t>, grid, dim3(256), h->small_chain_smem, st, a);
    else
        hipLaunchKernelGGL(small_chain_kernel<float>, grid, dim3(256), h->small_chain_smem, st, a);
    return hipGetLastError() == hipSuccess ? TN_OK : TN_ERR_HIP;
}

// The chained pair kernel runs every call of a layer it fits. With few token tiles (8 workgroups per 32 tokens) the
// range of a is split over workgroups, fp32 partial sums are written to the partial buffer and kron_reduce_kernel
// adds them in split order.
constexpr int64_t kPairMinTokens = 1;
#ifndef TN_PAIR_STAGES
#define TN_PAIR_STAGES 4
#define TN_PAIR_BAR 1
#endif
constexpr int kPairStages = TN_PAIR_STAGES, kPairBar = TN_PAIR_BAR;
constexpr size_t kPairSmemBytes = kPairStages * 20 * 1024;

struct PairGeom {
    int n_tok_tiles = 1, n_jsets = 1, n_splits = 1, a_per_split = 1;
    int64_t partial_bytes = 0;
};

PairGeom pair_geometry(const tn_linear_s* h, int64_t tokens, int64_t partial_cap) {
    PairGeom g;
    const int64_t A = h->steps[0].plan.R, J = h->steps[1].plan.R;
    g.n_tok_tiles = int((tokens + 31) / 32);
    g.n_jsets = int(J / 8);
    const int64_t base = int64_t(g.n_tok_tiles) * g.n_jsets;
    // one round of workgroups (a CU holds one): as many splits as keep the grid within the number of CUs
    int64_t want = std::max<int64_t>(1, int64_t(h->num_cus) / base);
    want = std::min<int64_t>(want, std::max<int64_t>(1, A / 2));                      // at least two values of a each
    // every split writes tokens * M floats that the reduction reads back: within one token tile the number of splits
    // that balances the two (measured at 8, 16 and 32 tokens: 16-20, 16, 13) grows as tokens^-1/2; with several
    // token tiles filling the chip matters more
    if (want > 1 && tokens <= 32) {
        const double per_split_mb = double(tokens) * double(h->plan.M) * 8.0 / 1e6;      // written and read
        const double best = std::sqrt(double(A) * 4.8 / per_split_mb);
        want = std::min<int64_t>(want, std::max<int64_t>(1, int64_t(best + 0.5)));
    }
    want = std::min<int64_t>(want, std::max<int64_t>(1, partial_cap / (tokens * h->plan.M * 4)));       // stays the last word
    g.a_per_split = int((A + want - 1) / want);
    g.n_splits = int((A + g.a_per_split - 1) / g.a_per_split);                        // no empty split
    g.partial_bytes = g.n_splits > 1 ? int64_t(g.n_splits) * tokens * h->plan.M * 4 : 0;
    return g;
}

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

int launch_pair(const tn_linear_s* h, const Workspace& w, const void* x, void* y, int64_t tokens, hipStream_t st) {
    const DevStep& s0 = h->steps[0];
    const DevStep& s1 = h->steps[1];
    const PairGeom g = pair_geometry(h, tokens, w.partial ? w.partial_bytes : 0);
    if (g.partial_bytes > (w.partial ? w.partial_bytes : 0)) return TN_ERR_UNSUPPORTED;      // never write past the buffer
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
    p.n_tok_tiles = g.n_tok_tiles;
    p.n_jsets = g.n_jsets;
    p.n_splits = g.n_splits;
    p.a_per_split = g.a_per_split;
    p.partial = static_cast<float*>(w.partial);
    const int64_t grid = p.n_splits > 1 ? int64_t(p.n_tok_tiles) * p.n_jsets * p.n_splits
                                        : int64_t((p.n_tok_tiles + 7) / 8 * 8) * p.n_jsets;
    hipLaunchKernelGGL((step_pair_kernel<kPairStages, kPairBar>), dim3(uint32_t(grid)), dim3(256), kPairSmemBytes, st, p);
    if (g.n_splits > 1) {
        const int64_t n = tokens * h->plan.M;
        hipLaunchKernelGGL(kron_reduce_kernel, dim3(uint32_t((n + 63) / 64)), dim3(256), 0, st,
                           static_cast<const float*>(w.partial), static_cast<bf16_t*>(y), n, g.n_splits);
    }
    return hipGetLastError() == hipSuccess ? TN_OK : TN_ERR_HIP;
}

// Kronecker-sum kernel: instantiations (see tn::kron_shape for the order) and launch geometry.
// From kKronMinTokens tokens on it replaces the two launches. A workgroup holds 4 tokens; when there are
// fewer workgroups than compute units the shared bond is split over several of them (fp32 partial sums,
// added by kron_reduce_kernel).
constexpr int64_t kKronMinTokens = 1;

struct KronTiles {
    int at = 0, ks0 = 0, o2t = 0, o1t = 0;
    size_t smem = 0;
    bool two_tokens = false;      // the instantiation with two tokens per wave exists
};

// Two tokens per wave where the registers allow it: at most 12 accumulation tiles (192 registers) for the two tokens'
// sums and at most 32 fragments of their inputs (<3,4,4,2> with 16 tiles spills).
template <int AT, int KS0, int O2T, int O1T>
constexpr bool kron_two_tokens_fit() { return 2 * O2T * O1T <= 12 && 2 * AT * KS0 <= 32; }

template <int AT, int KS0, int O2T, int O1T>
int kron_entry(const KronArgs* p, uint32_t grid, hipStream_t st, KronTiles* tiles) {
    using S = KronShape<AT, KS0, O2T, O1T>;
    constexpr bool two = kron_two_tokens_fit<AT, KS0, O2T, O1T>();
    if (tiles) {
        *tiles = KronTiles{AT, KS0, O2T, O1T, S::SMEM, two};
        return TN_OK;
    }
    if (!p) {       // configuration call (create time)
        bool ok = hipFuncSetAttribute(reinterpret_cast<const void*>(step_kronsum_kernel<AT, KS0, O2T, O1T, 0, 1>),
                                      hipFuncAttributeMaxDynamicSharedMemorySize, int(S::SMEM)) == hipSuccess &&
                  hipFuncSetAttribute(reinterpret_cast<const void*>(step_kronsum_kernel<AT, KS0, O2T, O1T, 1, 1>),
                                      hipFuncAttributeMaxDynamicSharedMemorySize, int(S::SMEM)) == hipSuccess;
        if constexpr (two)
            ok = ok && hipFuncSetAttribute(reinterpret_cast<const void*>(step_kronsum_kernel<AT, KS0, O2T, O1T, 0, 2>),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, int(S::SMEM)) == hipSuccess;
        return ok ? TN_OK : TN_ERR_HIP;
    }
    if (p->share) {
        hipLaunchKernelGGL((step_kronsum_kernel<AT, KS0, O2T, O1T, 1, 1>), dim3(grid), dim3(256), S::SMEM, st, *p);
    } else if (p->tpw == 2) {
        if constexpr (two) hipLaunchKernelGGL((step_kronsum_kernel<AT, KS0, O2T, O1T, 0, 2>), dim3(grid), dim3(256), S::SMEM, st, *p);
        else return TN_ERR_UNSUPPORTED;
    } else {
        hipLaunchKernelGGL((step_kronsum_kernel<AT, KS0, O2T, O1T, 0, 1>), dim3(grid), dim3(256), S::SMEM, st, *p);
    }
    return TN_OK;
}

#define TN_KRON_CASE(i)                                                                                        \
    case i:                                                                                                   \
        return kron_entry<tn::kKronConfig[i][0], tn::kKronConfig[i][1], tn::kKronConfig[i][2], tn::kKronConfig[i][3]>( \
            p, grid, st, tiles);

int kron_dispatch(int cfg, const KronArgs* p, uint32_t grid, hipStream_t st, KronTiles* tiles = nullptr) {
    static_assert(tn::kKronConfigs == 8, "one case per instantiation");
    switch (cfg) {
        TN_KRON_CASE(0)
        TN_KRON_CASE(1)
        TN_KRON_CASE(2)
        TN_KRON_CASE(3)
        TN_KRON_CASE(4)
        TN_KRON_CASE(5)
        TN_KRON_CASE(6)
        TN_KRON_CASE(7)
        default: return TN_ERR_INVALID_ARG;
    }
}
#undef TN_KRON_CASE

struct KronGeom {
    int n_chunks = 1, n_splits = 1, rho_per_split = 1;
    int64_t quads = 1, partial_bytes = 0;
    bool share = false;       // the four waves of a workgroup share one token (quads then counts tokens)
    int tpw = 1;              // tokens per wave (quads then counts groups of 4 * tpw tokens)
};

// measured on seven ring classes with stored half rings (us per call, shared / a wave per token): one token 30/44,
// 110/214, 146/206, 79/119, 51/65, 31/35, 16/16; two tokens 34/44, 165/195, 214/204, 109/111, 65/63, 41/36, 18/17
constexpr int64_t kKronShareMaxTokens = 1;
// calls from which a wave takes two tokens, where that instantiation exists (8192->5120 at rank 64, ms per call, two / one:
// 64 tokens 0.63 / 0.67, 128 1.15 / 1.23, 300 2.46 / 2.74, 8192 58.4 / 65.6)
constexpr int64_t kKronTwoTokensMin = 64;

KronGeom kron_geometry(const tn_linear_s* h, const tn::KronDims& d, int64_t tokens, int64_t partial_cap) {
    KronGeom g;
    const int o1_chunk = 32 * tn::kKronConfig[d.cfg][3];
    g.n_chunks = int((d.O1 + o1_chunk - 1) / o1_chunk);
    g.share = tokens <= kKronShareMaxTokens && !(h->flags & TN_FLAG_NO_DECODE_FUSION);
    {
        KronTiles kt;
        const bool two = kron_dispatch(d.cfg, nullptr, 0, nullptr, &kt) == TN_OK && kt.two_tokens;
        g.tpw = (two && tokens >= kKronTwoTokensMin) ? 2 : 1;
    }
    g.quads = g.share ? tokens : (tokens + 4 * g.tpw - 1) / (4 * g.tpw);
    int64_t base = g.quads * g.n_chunks;
    // workgroups a CU holds at a time: one when the three LDS stages take more than half of its 160 KB
    const int* cfg = tn::kKronConfig[d.cfg];
    const int64_t stage_bytes = 4096 * int64_t((cfg[3] * cfg[1] + cfg[2] * 2 * cfg[0] + 3) / 4);
    // (measured: with several chunks of o1 the two-round split is the faster one at rank 96, so it is kept there)
    const int64_t per_cu = (3 * stage_bytes > 80 * 1024 && g.n_chunks == 1) ? 1 : 2;
    // as many splits as keep the grid within one round of workgroups (rounding up instead left a second round with a
    // handful of workgroups: 300 tokens took as long as 512)
    int64_t want = std::max<int64_t>(1, per_cu * int64_t(h->num_cus) / base);
    if (base >= h->num_cus) want = 1;
    // at least 4 values of the bond per workgroup, partial sums within their buffer
    want = std::min<int64_t>(want, std::max<int64_t>(1, d.P / 4));
    want = std::min<int64_t>(want, std::max<int64_t>(1, partial_cap / (tokens * h->plan.M * 4)));
    g.rho_per_split = int((d.P + want - 1) / want);
    g.n_splits = int((d.P + g.rho_per_split - 1) / g.rho_per_split);      // no empty split
    g.partial_bytes = g.n_splits > 1 ? int64_t(g.n_splits) * tokens * h->plan.M * 4 : 0;
    return g;
}

int prepare_kron(tn_linear_s* h, hipStream_t st) {
    if ((h->flags & (TN_FLAG_NO_PAIR_CHAIN | TN_FLAG_SCALAR_KERNELS)) || h->pair || h->small_chain) return TN_OK;
    tn::KronDims d;
    if (!tn::kron_shape(h->plan, &d)) return TN_OK;
    const DevStep& s0 = h->steps[0];
    const DevStep& s1 = h->steps[1];
    if (s0.variant == VAR_SCALAR || s1.variant == VAR_SCALAR) return TN_OK;
    KronTiles kt;
    if (kron_dispatch(d.cfg, nullptr, 0, nullptr, &kt) != TN_OK) return TN_OK;
    const int at = kt.at, ks0 = kt.ks0, o2t = kt.o2t, o1t = kt.o1t;
    const int n_chunks = int((d.O1 + 32 * o1t - 1) / (32 * o1t));
    const int64_t e0 = int64_t(n_chunks) * d.P * o1t * ks0 * 512;
    const int64_t e1 = d.P * int64_t(o2t) * 2 * at * 512;
    if (hipMalloc(&h->kron_h0f, size_t(e0) * sizeof(bf16_t)) != hipSuccess) return TN_ERR_ALLOC;
    if (hipMalloc(&h->kron_h1f, size_t(e1) * sizeof(bf16_t)) != hipSuccess) return TN_ERR_ALLOC;
    h->packed_bytes += (e0 + e1) * int64_t(sizeof(bf16_t));
    hipLaunchKernelGGL(kron_repack0_kernel, dim3(uint32_t(std::min<int64_t>((e0 + 255) / 256, 8192))), dim3(256), 0, st,
                       static_cast<const bf16_t*>(s0.packed), static_cast<bf16_t*>(h->kron_h0f), n_chunks, int(d.P), ks0,
                       o1t, int(d.O1), int(d.K0), s0.Kp >> 4);
    hipLaunchKernelGGL(kron_repack1_kernel, dim3(uint32_t(std::min<int64_t>((e1 + 255) / 256, 8192))), dim3(256), 0, st,
                       static_cast<const bf16_t*>(s1.packed), static_cast<bf16_t*>(h->kron_h1f), int(d.P), o2t, at,
                       int(d.C1), int(d.A), s1.Kp >> 4);
    if (hipGetLastError() != hipSuccess) return TN_ERR_HIP;
    h->kron = true;
    h->kron_dims = d;
    h->kron_min_tokens = kKronMinTokens;
    if (h->kron_min_tokens <= 1) {
        // every call runs the one-launch kernel: the per-step packed tensors are not needed any more
        if (hipStreamSynchronize(st) != hipSuccess) return TN_ERR_HIP;
        for (DevStep& s : h->steps) {
            h->packed_bytes -= int64_t(s.Cp) * s.Kp * h->elt;
            (void)hipFree(s.packed);
            s.packed = nullptr;
        }
    }
    return TN_OK;
}

struct KronSetup {
    const tn::KronDims* dims;
    const void *h0f, *h1f;
    const int32_t *xrow, *xcol, *yrow, *ycol;
};

int launch_kron(const tn_linear_s* h, const Workspace& w, const KronSetup& k, const void* x, void* y, int64_t tokens,
                hipStream_t st) {
    const tn::KronDims& d = *k.dims;
    const KronGeom g = kron_geometry(h, d, tokens, w.partial ? w.partial_bytes : 0);
    if (g.partial_bytes > (w.partial ? w.partial_bytes : 0)) return TN_ERR_UNSUPPORTED;      // never write past the buffer
    KronArgs p;
    p.X = x;
    p.Y = g.n_splits > 1 ? w.partial : y;
    p.H0f = k.h0f;
    p.H1f = k.h1f;
    p.xrow = k.xrow;
    p.xcol = k.xcol;
    p.yrow = k.yrow;
    p.ycol = k.ycol;
    p.N = h->plan.N;
    p.M = h->plan.M;
    p.tokens = int32_t(tokens);
    p.A = int32_t(d.A);
    p.K0 = int32_t(d.K0);
    p.O1 = int32_t(d.O1);
    p.C1 = int32_t(d.C1);
    p.P = int32_t(d.P);
    p.n_chunks = g.n_chunks;
    p.n_splits = g.n_splits;
    p.rho_per_split = g.rho_per_split;
    p.x_vec8 = d.x_vec8 ? 1 : 0;
    p.share = g.share ? 1 : 0;
    p.tpw = g.tpw;
    const int64_t grid = g.quads * g.n_chunks * g.n_splits;
    int rc = kron_dispatch(d.cfg, &p, uint32_t(grid), st);
    if (rc != TN_OK) return rc;
    if (g.n_splits > 1) {
        const int64_t n = tokens * h->plan.M;
        hipLaunchKernelGGL(kron_reduce_kernel, dim3(uint32_t((n + 63) / 64)), dim3(256), 0, st,
                           static_cast<const float*>(w.partial), static_cast<bf16_t*>(y), n, g.n_splits);
    }
    return hipGetLastError() == hipSuccess ? TN_OK : TN_ERR_HIP;
}

int launch_kron_eager(const tn_linear_s* h, const Workspace& w, const void* x, void* y, int64_t tokens, hipStream_t st) {
    const DevStep& s0 = h->steps[0];
    const DevStep& s1 = h->steps[1];
    KronSetup k{&h->kron_dims, h->kron_h0f, h->kron_h1f, s0.plan.a_plain ? nullptr : s0.arow,
                s0.plan.a_plain ? nullptr : s0.acol, s1.crow, s1.ccol};
    return launch_kron(h, w, k, x, y, tokens, st);
}

// Large calls of a layer with a lazily merged plan: rebuild the two slice arrays in the workspace from the
// library's copies of the caller's tensors (once per call), then run the Kronecker-sum kernel on them.
constexpr size_t kGenMfmaMaxSmem = 160 * 168 * 2;

int gen_mfma_dispatch(const KronGenMfmaArgs* a, size_t smem, hipStream_t st) {
    using kern_t = void (*)(KronGenMfmaArgs);
    static const kern_t kerns[4] = {kron_generate_mfma_kernel<2>, kron_generate_mfma_kernel<4>, kron_generate_mfma_kernel<6>,
                                    kron_generate_mfma_kernel<8>};
    if (!a) {               // configuration call (create time)
        for (kern_t k : kerns)
            if (hipFuncSetAttribute(reinterpret_cast<const void*>(k), hipFuncAttributeMaxDynamicSharedMemorySize,
                                    int(kGenMfmaMaxSmem)) != hipSuccess)
                return TN_ERR_HIP;
        return TN_OK;
    }
    const int idx = (a->Sp + 31) / 32 - 1;
    if (idx < 0 || idx > 3) return TN_ERR_INVALID_ARG;
    hipLaunchKernelGGL(kerns[idx], dim3(uint32_t(a->P)), dim3(256), smem, st, *a);
    return TN_OK;
}

int gen_mfma_both_dispatch(const KronGenMfmaArgs* a0, const KronGenMfmaArgs* a1, size_t smem, hipStream_t st) {
    using kern_t = void (*)(KronGenMfmaArgs, KronGenMfmaArgs);
    static const kern_t kerns[4] = {kron_generate_mfma_both_kernel<2>, kron_generate_mfma_both_kernel<4>,
                                    kron_generate_mfma_both_kernel<6>, kron_generate_mfma_both_kernel<8>};
    if (!a0) {              // configuration call (create time)
        for (kern_t k : kerns)
            if (hipFuncSetAttribute(reinterpret_cast<const void*>(k), hipFuncAttributeMaxDynamicSharedMemorySize,
                                    int(kGenMfmaMaxSmem)) != hipSuccess)
                return TN_ERR_HIP;
        return TN_OK;
    }
    const int idx = (std::max(a0->Sp, a1->Sp) + 31) / 32 - 1;
    if (idx < 0 || idx > 3) return TN_ERR_INVALID_ARG;
    hipLaunchKernelGGL(kerns[idx], dim3(uint32_t(a0->P + a1->P)), dim3(256), smem, st, *a0, *a1);
    return TN_OK;
}

int launch_lazy_generate(const tn_linear_s* h, hipStream_t st) {
    if (h->lazy_mfma[0] && h->lazy_mfma[1]) {
        int rc = gen_mfma_both_dispatch(&h->lazy_gen_mfma[0], &h->lazy_gen_mfma[1],
                                        std::max(h->lazy_gen_smem[0], h->lazy_gen_smem[1]), st);
        if (rc != TN_OK) return rc;
        return hipGetLastError() == hipSuccess ? TN_OK : TN_ERR_HIP;
    }
    for (int w = 0; w < 2; ++w) {
        if (h->lazy_mfma[w]) {
            int rc = gen_mfma_dispatch(&h->lazy_gen_mfma[w], h->lazy_gen_smem[w], st);
            if (rc != TN_OK) return rc;
            continue;
        }
        const KronGenArgs& g = h->lazy_gen[w];
        const int64_t pieces = w == 0 ? int64_t(g.n_chunks) * g.P * g.O1T * g.KS0 * 64 : int64_t(g.P) * g.O2T * 2 * g.AT * 64;
        hipLaunchKernelGGL(kron_generate_kernel, dim3(uint32_t(std::min<int64_t>((pieces + 255) / 256, 1 << 20))), dim3(256),
                           0, st, g);
    }
    return hipGetLastError() == hipSuccess ? TN_OK : TN_ERR_HIP;
}

// Tables of the MFMA form of the slice generation for half w (see kron_generate_mfma_kernel): which rows of the
// two source matrices a value of the bond uses, and where each element of a slice sits in their product.
// perm maps the kernels' numbering of k (w = 0) or a (w = 1) to the plan's. Returns false (and leaves the scalar
// kernel in charge) when the half does not fit: more than 160 distinct rows on a side or a shared bond longer
// than 128.
bool prepare_gen_mfma(tn_linear_s* h, int w, const KronGenArgs& g, const tn::KronDims& d, int64_t merged_C,
                      const std::vector<int32_t>& perm, hipStream_t st) {
    if (g.Sp > 128 || g.Sp % 16) return false;
    const int64_t P = d.P;
    struct Elem { int64_t rP, rQ; };
    const int64_t pieces = w == 0 ? int64_t(g.n_chunks) * g.O1T * g.KS0 * 64 : int64_t(g.O2T) * 2 * g.AT * 64;
    std::vector<Elem> elems(size_t(pieces) * 8, Elem{-1, -1});
    for (int64_t lp = 0; lp < pieces; ++lp) {
        const int l = int(lp & 63);
        int64_t blk = lp >> 6;
        for (int e = 0; e < 8; ++e) {
            int64_t cB, kB;
            bool inside;
            if (w == 0) {
                int64_t b2 = blk;
                const int ks = int(b2 % g.KS0);
                b2 /= g.KS0;
                const int o1t = int(b2 % g.O1T);
                const int chunk = int(b2 / g.O1T);
                const int64_t o1 = int64_t(32) * g.O1T * chunk + 32 * o1t + (l & 31);
                const int64_t k = 16 * ks + 8 * (l >> 5) + e;
                inside = o1 < d.O1 && k < d.K0;
                cB = o1 * P;
                kB = inside ? perm[size_t(k)] : 0;
            } else {
                const int is = int(blk % (2 * g.AT));
                const int j = int(blk / (2 * g.AT));
                const int64_t c = 32 * j + (l & 31);
                const int64_t a = 16 * is + 8 * (e >> 2) + 4 * (l >> 5) + (e & 3);
                inside = c < d.C1 && a < d.A;
                cB = c;
                kB = inside ? int64_t(perm[size_t(a)]) * P : 0;
            }
            if (!inside) continue;
            const int64_t m = gen_offset(g.sc, cB) + gen_offset(g.sk, kB);
            elems[size_t(lp) * 8 + e] = Elem{m / merged_C, m % merged_C};
        }
    }
    // the column side of the product is the tensor whose row changes from one element of a piece to the next
    bool cols_from_q = true;
    for (size_t i = 0; i + 1 < elems.size(); i += 8)
        if (elems[i].rP >= 0 && elems[i + 1].rP >= 0) {
            cols_from_q = elems[i].rQ != elems[i + 1].rQ;
            break;
        }
    std::vector<int64_t> rows_r, rows_c;
    for (const Elem& el : elems)
        if (el.rP >= 0) {
            rows_r.push_back(cols_from_q ? el.rP : el.rQ);
            rows_c.push_back(cols_from_q ? el.rQ : el.rP);
        }
    auto uniq = [](std::vector<int64_t>* v) {
        std::sort(v->begin(), v->end());
        v->erase(std::unique(v->begin(), v->end()), v->end());
    };
    uniq(&rows_r);
    uniq(&rows_c);
    const int64_t NR = int64_t(rows_r.size()), NC = int64_t(rows_c.size());
    if (NR < 1 || NC < 1 || NR > 160 || NC > 160) return false;
    const int LDC = round_up(int(NC), 32) + 8;
    // one allocation: rowR | rowC | rhoR | rhoC (int32), then the piece table (8 x uint16 per piece, 16-byte aligned)
    const size_t n_int = size_t(NR + NC + 2 * P);
    const size_t tab_off = (n_int * 4 + 15) & ~size_t(15);
    std::vector<unsigned char> host(tab_off + size_t(pieces) * 16);
    int32_t* ints = reinterpret_cast<int32_t*>(host.data());
    for (int64_t r = 0; r < NR; ++r) ints[r] = int32_t(rows_r[size_t(r)]);
    for (int64_t c = 0; c < NC; ++c) ints[NR + c] = int32_t(rows_c[size_t(c)]);
    for (int64_t rho = 0; rho < P; ++rho) {
        const int64_t m = w == 0 ? gen_offset(g.sc, rho) : gen_offset(g.sk, rho);
        ints[NR + NC + rho] = int32_t(cols_from_q ? m / merged_C : m % merged_C);
        ints[NR + NC + P + rho] = int32_t(cols_from_q ? m % merged_C : m / merged_C);
    }
    uint16_t* tab = reinterpret_cast<uint16_t*>(host.data() + tab_off);
    for (size_t i = 0; i < elems.size(); ++i) {
        if (elems[i].rP < 0) {
            tab[i] = 0xFFFF;
            continue;
        }
        const int64_t vr = cols_from_q ? elems[i].rP : elems[i].rQ, vc = cols_from_q ? elems[i].rQ : elems[i].rP;
        const int64_t r = std::lower_bound(rows_r.begin(), rows_r.end(), vr) - rows_r.begin();
        const int64_t c = std::lower_bound(rows_c.begin(), rows_c.end(), vc) - rows_c.begin();
        tab[i] = uint16_t(r * LDC + c);
    }
    // are the pieces runs of consecutive columns? (first slice: 8 in a row; second: two runs of 4); a run is
    // either wholly inside the tensor or wholly outside, and starts at a multiple of its length
    const int run = w == 0 ? 8 : 4;
    bool contig = true;
    for (size_t i = 0; i < elems.size() && contig; i += size_t(run)) {
        const bool out0 = tab[i] == 0xFFFF;
        for (int e = 0; e < run && contig; ++e) {
            if ((tab[i + e] == 0xFFFF) != out0) contig = false;
            else if (!out0 && (tab[i + e] != tab[i] + e || tab[i] % run)) contig = false;
        }
    }
    if (hipMalloc(&h->lazy_gen_tables[w], host.size()) != hipSuccess) return false;
    if (hipMemcpyAsync(h->lazy_gen_tables[w], host.data(), host.size(), hipMemcpyHostToDevice, st) != hipSuccess ||
        hipStreamSynchronize(st) != hipSuccess)
        return false;
    h->packed_bytes += int64_t(host.size());
    KronGenMfmaArgs& a = h->lazy_gen_mfma[w];
    memset(&a, 0, sizeof(a));
    a.Rc = cols_from_q ? g.Pc : g.Qc;
    a.Cc = cols_from_q ? g.Qc : g.Pc;
    const int32_t* dints = static_cast<const int32_t*>(h->lazy_gen_tables[w]);
    a.rowR = dints;
    a.rowC = dints + NR;
    a.rhoR = dints + NR + NC;
    a.rhoC = dints + NR + NC + P;
    a.tab = static_cast<const unsigned char*>(h->lazy_gen_tables[w]) + tab_off;
    a.NR = int32_t(NR);
    a.NC = int32_t(NC);
    a.LDC = LDC;
    a.Sp = g.Sp;
    a.pieces_per_rho = int32_t(pieces);
    a.pieces_per_chunk = int32_t(pieces / (w == 0 ? g.n_chunks : 1));
    a.P = int32_t(P);
    a.contig = contig ? (w == 0 ? 1 : 2) : 0;
    h->lazy_gen_smem[w] = size_t(NR) * LDC * 2;
    h->lazy_mfma[w] = true;
    return true;
}

// The kernels may number k and a in any order as long as x is gathered through the same numbering. Pick the one that
// makes an index of extent % unit == 0 the fastest-running digit (it is then a run of consecutive columns of the
// product matrix the slices are assembled from): returns new number -> the plan's number.
std::vector<int32_t> minor_digit_permutation(const std::vector<int64_t>& extents, int unit) {
    int64_t total = 1;
    for (int64_t e : extents) total *= e;
    std::vector<int32_t> perm(static_cast<size_t>(total));
    for (int64_t i = 0; i < total; ++i) perm[size_t(i)] = int32_t(i);
    const int n = int(extents.size());
    if (n < 2 || extents[size_t(n - 1)] % unit == 0) return perm;      // already so (or nothing to choose)
    int pick = -1;
    for (int j = 0; j < n; ++j)
        if (extents[size_t(j)] % unit == 0 && (pick < 0 || extents[size_t(j)] > extents[size_t(pick)])) pick = j;
    if (pick < 0) return perm;
    std::vector<int> order;                 // digits of the new number, outer -> inner
    for (int j = 0; j < n; ++j)
        if (j != pick) order.push_back(j);
    order.push_back(pick);
    std::vector<int64_t> weight(size_t(n), 1);      // of each digit in the plan's number
    for (int j = n - 2; j >= 0; --j) weight[size_t(j)] = weight[size_t(j + 1)] * extents[size_t(j + 1)];
    for (int64_t i = 0; i < total; ++i) {
        int64_t rem = i, orig = 0;
        for (int q = n - 1; q >= 0; --q) {
            const int j = order[size_t(q)];
            orig += (rem % extents[size_t(j)]) * weight[size_t(j)];
            rem /= extents[size_t(j)];
        }
        perm[size_t(i)] = int32_t(orig);
    }
    return perm;
}

int launch_kron_lazy(const tn_linear_s* h, const Workspace& w, const void* x, void* y, int64_t tokens, hipStream_t st) {
    KronSetup k{&h->lazy_dims, h->lazy_slices, static_cast<const char*>(h->lazy_slices) + h->lazy_h1_offset,
                h->lazy_xrow, h->lazy_xcol, h->lazy_yrow, h->lazy_ycol};
    return launch_kron(h, w, k, x, y, tokens, st);
}

// Token count from which a lazily merged plan replaces the compact steps: every call. With the one-token form of
// the Kronecker-sum kernel (four waves share the token) rebuilding the slices and streaming them once is as fast as
// the compact steps or faster on every ring class of the 64-layer stack (us per one-token call, rebuilt / compact:
// 25600->5120 r32 49/69, r96 326/527; 5120->25600 r64 246/246; 5120->8192 r96 253/262; 8192->5120 r64 118/130;
// 5120->1024 r96 97/163, r32 24/46).
constexpr int64_t kLazyMinTokens = 1;

void fill_gen_dims(GenDims* g, const std::vector<tn::GatherDim>& d) {
    g->n = int32_t(d.size());
    for (size_t j = 0; j < d.size(); ++j) {
        g->ext[j] = int32_t(d[j].extent);
        g->str[j] = d[j].stride;
    }
}

// Decide whether the layer gets a lazily merged plan, and prepare it: the plan TN_FLAG_MERGE_GROW would give
// must be two steps the Kronecker-sum kernel takes (large intermediate, little padding), each absorbing a
// tensor merged from two of the caller's, and cheaper than the compact plan. Nothing of that plan is stored
// except copies of the caller's tensors involved and four offset tables.
int prepare_lazy(tn_linear_s* h, const tn_linear_desc* desc, hipStream_t st) {
    if (h->plan.dtype != TN_DTYPE_BF16 || h->pair || h->kron || h->small_chain) return TN_OK;
    if (desc->flags & (TN_FLAG_NO_PAIR_CHAIN | TN_FLAG_SCALAR_KERNELS | TN_FLAG_NO_MERGE | TN_FLAG_MERGE_GROW |
                       TN_FLAG_MERGE_HALVES | TN_FLAG_NO_LAZY_MERGE | TN_FLAG_TRAINABLE))
        return TN_OK;
    if (((desc->flags >> TN_FLAG_VARIANT_SHIFT) & 0xff) != 0) return TN_OK;      // tuning overrides: keep what they ask
    if (desc->max_tokens < kLazyMinTokens) return TN_OK;
    tn_linear_desc grow = *desc;
    grow.flags |= TN_FLAG_MERGE_HALVES;
    tn::Plan& q = h->lazy_plan;
    if (tn::make_plan(&grow, &q) != TN_OK || q.steps.size() != 2 || q.merges.size() != 2 || q.flops >= h->plan.flops)
        return TN_OK;
    tn::KronDims d;
    if (!tn::kron_shape(q, &d)) return TN_OK;
    const tn::MergeOp* mo[2];
    for (int w = 0; w < 2; ++w) {
        int mi = q.steps[size_t(w)].slot - q.n_caller_tensors;
        if (mi < 0 || mi >= 2) return TN_OK;
        mo[w] = &q.merges[size_t(mi)];
        if (mo[w]->p_slot >= q.n_caller_tensors || mo[w]->q_slot >= q.n_caller_tensors) return TN_OK;
        if (mo[w]->kp.empty() || q.steps[size_t(w)].trace_extent != 1) return TN_OK;
    }
    KronTiles kt;
    if (kron_dispatch(d.cfg, nullptr, 0, nullptr, &kt) != TN_OK) return TN_OK;
    const int at = kt.at, ks0 = kt.ks0, o2t = kt.o2t, o1t = kt.o1t;
    // the four source matrices (shared indices innermost), written from the caller's tensors
    const int32_t sp_len[2] = {round_up(int(mo[0]->K), 16), round_up(int(mo[1]->K), 16)};
    for (int w = 0; w < 2; ++w)
        for (int side = 0; side < 2; ++side) {
            const int64_t rows = side == 0 ? mo[w]->R : mo[w]->C;
            const int64_t n = rows * sp_len[w];
            void* buf = nullptr;
            if (hipMalloc(&buf, size_t(n) * sizeof(bf16_t)) != hipSuccess) return TN_ERR_ALLOC;
            h->lazy_sources.push_back(buf);
            h->packed_bytes += n * int64_t(sizeof(bf16_t));
            GenDims fd, sd;
            memset(&fd, 0, sizeof(fd));
            memset(&sd, 0, sizeof(sd));
            fill_gen_dims(&fd, side == 0 ? mo[w]->rdims : mo[w]->cdims);
            fill_gen_dims(&sd, side == 0 ? mo[w]->kp : mo[w]->kq);
            hipLaunchKernelGGL(kron_source_kernel, dim3(uint32_t(std::min<int64_t>((n + 255) / 256, 65536))), dim3(256), 0, st,
                               static_cast<const bf16_t*>(desc->tensors[side == 0 ? mo[w]->p_slot : mo[w]->q_slot]),
                               static_cast<bf16_t*>(buf), fd, sd, rows, int32_t(mo[w]->K), sp_len[w]);
        }
    if (hipGetLastError() != hipSuccess) return TN_ERR_HIP;
    const tn::Step& s0 = q.steps[0];
    const tn::Step& s1 = q.steps[1];
    const int n_chunks = int((d.O1 + 32 * o1t - 1) / (32 * o1t));
    const int64_t e0 = int64_t(n_chunks) * d.P * o1t * ks0 * 512;
    const int64_t e1 = d.P * int64_t(o2t) * 2 * at * 512;
    h->lazy_h1_offset = (e0 * 2 + 255) & ~int64_t(255);
    h->lazy_slice_bytes = h->lazy_h1_offset + ((e1 * 2 + 255) & ~int64_t(255));
    for (int w = 0; w < 2; ++w) {
        KronGenArgs& g = h->lazy_gen[w];
        memset(&g, 0, sizeof(g));
        const tn::Step& sp = q.steps[size_t(w)];
        g.Pc = h->lazy_sources[size_t(2 * w)];
        g.Qc = h->lazy_sources[size_t(2 * w + 1)];
        fill_gen_dims(&g.sc, sp.cdims);
        fill_gen_dims(&g.sk, sp.kdims);
        g.merged_C = mo[w]->C;
        g.Sp = sp_len[w];
        g.which = w;
        g.n_chunks = n_chunks;
        g.P = int32_t(d.P);
        g.KS0 = ks0;
        g.O1T = o1t;
        g.O1 = int32_t(d.O1);
        g.K0 = int32_t(d.K0);
        g.O2T = o2t;
        g.AT = at;
        g.C1 = int32_t(d.C1);
        g.A = int32_t(d.A);
    }
    // The MFMA form of the rebuild, with k and a numbered so that the pieces of the slices are runs of columns of
    // the products; if a half does not fit that form, both keep the plan's numbering (the plain-FMA kernel knows no
    // other) and the halves that fit still use MFMA.
    std::vector<int32_t> perm_k(size_t(d.K0)), perm_a(size_t(d.A));
    for (int64_t i = 0; i < d.K0; ++i) perm_k[size_t(i)] = int32_t(i);
    for (int64_t i = 0; i < d.A; ++i) perm_a[size_t(i)] = int32_t(i);
    if (!(desc->flags & TN_FLAG_SCALAR_GENERATE)) {
        std::vector<int64_t> kext;
        for (const tn::GatherDim& gd : s0.kdims) kext.push_back(gd.extent);
        const std::vector<int32_t> pk = minor_digit_permutation(kext, 8), pa = minor_digit_permutation(s0.rext, 4);
        const bool ok = int64_t(pk.size()) == d.K0 && int64_t(pa.size()) == d.A &&
                        prepare_gen_mfma(h, 0, h->lazy_gen[0], d, mo[0]->C, pk, st) &&
                        prepare_gen_mfma(h, 1, h->lazy_gen[1], d, mo[1]->C, pa, st);
        if (ok) {
            perm_k = pk;
            perm_a = pa;
        } else {
            for (int w = 0; w < 2; ++w) {
                if (h->lazy_gen_tables[w]) (void)hipFree(h->lazy_gen_tables[w]);
                h->lazy_gen_tables[w] = nullptr;
                h->lazy_mfma[w] = false;
            }
            (void)prepare_gen_mfma(h, 0, h->lazy_gen[0], d, mo[0]->C, perm_k, st);
            (void)prepare_gen_mfma(h, 1, h->lazy_gen[1], d, mo[1]->C, perm_a, st);
        }
    }
    // tables of the merged plan: where a and k (in the kernels' numbering) sit in a token of x, where o1 and o2 go
    std::vector<int32_t> tab;
    bool identity = s0.a_plain;
    for (int64_t i = 0; i < d.K0 && identity; ++i) identity = perm_k[size_t(i)] == i;
    for (int64_t i = 0; i < d.A && identity; ++i) identity = perm_a[size_t(i)] == i;
    const size_t n_xrow = identity ? 0 : size_t(d.A), n_xcol = identity ? 0 : size_t(d.K0);
    if (!identity) {
        for (int64_t a = 0; a < d.A; ++a)
            tab.push_back(s0.a_plain ? int32_t(perm_a[size_t(a)] * d.K0) : s0.arow[size_t(perm_a[size_t(a)])]);
        for (int64_t k = 0; k < d.K0; ++k)
            tab.push_back(s0.a_plain ? perm_k[size_t(k)] : s0.acol[size_t(perm_k[size_t(k)])]);
        // 8 consecutive k of one a as one aligned 16-byte piece of x?
        d.x_vec8 = true;
        for (int64_t a = 0; a < d.A; ++a)
            if (tab[size_t(a)] % 8) d.x_vec8 = false;
        for (int64_t k = 0; k < d.K0; ++k) {
            const int32_t v = tab[size_t(d.A + k)], v0 = tab[size_t(d.A + (k & ~int64_t(7)))];
            if (v != v0 + (k & 7) || (!(k & 7) && v % 8)) d.x_vec8 = false;
        }
    }
    tab.insert(tab.end(), s1.crow.begin(), s1.crow.end());
    tab.insert(tab.end(), s1.ccol.begin(), s1.ccol.end());
    if (hipMalloc(reinterpret_cast<void**>(&h->lazy_tables), tab.size() * sizeof(int32_t)) != hipSuccess) return TN_ERR_ALLOC;
    if (hipMemcpyAsync(h->lazy_tables, tab.data(), tab.size() * sizeof(int32_t), hipMemcpyHostToDevice, st) != hipSuccess ||
        hipStreamSynchronize(st) != hipSuccess)
        return TN_ERR_HIP;
    if (!identity) {
        h->lazy_xrow = h->lazy_tables;
        h->lazy_xcol = h->lazy_tables + n_xrow;
    }
    h->lazy_yrow = h->lazy_tables + n_xrow + n_xcol;
    h->lazy_ycol = h->lazy_yrow + s1.crow.size();
    h->lazy = true;
    h->lazy_dims = d;
    h->lazy_min_tokens = kLazyMinTokens;
    return TN_OK;
}

// Pairs of steps the transposing chain kernel can run (see step_chain2_kernel): both plain, the
// first step's output stored transposed ([c1][r], which is what the second step reads as rows c1
// with K = r), the output in aligned runs of 8 along c1 or along c2, and sizes within one of the
// two instantiations.
int plan_chain2(tn_linear_s* h, hipStream_t st) {
    if (h->plan.dtype != TN_DTYPE_BF16 || (h->flags & (TN_FLAG_SCALAR_KERNELS | TN_FLAG_NO_CHAIN2)) ||
        h->pair || h->kron)
        return TN_OK;
    const std::vector<int> pairs = tn::chain2_pairs(h->plan);
    for (size_t i = 0; i + 1 < h->steps.size(); ++i) {
        DevStep& a = h->steps[i];
        DevStep& b = h->steps[i + 1];
        if (!pairs[i] || a.variant == VAR_SCALAR || b.variant == VAR_SCALAR) continue;
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
        if (cfg == 1 && a.plan.K <= 80) cfg = 2;         // <2,5,2>: the same layouts with 5 k-steps instead of 8
        a.chain_cfg = cfg;
        a.chain_run_c1 = run_c1;
    }
    return TN_OK;
}

Chain2Args chain2_args(const DevStep& s1, const DevStep& s2, const void* A, void* Out, int64_t tokens) {
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
    p.tiles_per_item = 1;
    return p;
}

// Few tokens: every (token, c1 tile) item of a chained pair gets a wave of its own, operands requested up front.
bool chain2_small_applies(const tn_linear_s* h, const DevStep& s1, int64_t tokens) {
    return tokens * ((s1.plan.C + 31) / 32) <= int64_t(h->num_cus) * 4 && !(h->flags & TN_FLAG_NO_DECODE_FUSION);
}

constexpr int64_t kChain2FineMaxItems = 64;      // (token, c1 tile) items up to which every c2 tile gets a wave of its own

// One launch for the pair of one layer (p1 == nullptr) or of two layers with the same instantiation.
int launch_chain2_small(const DevStep& s1, const Chain2Args& p0, const Chain2Args* p1, hipStream_t st) {
    using k_t = void (*)(Chain2Args, Chain2Args);
    static const k_t small[6] = {step_chain2_small_kernel<3, 6, 5, 0>, step_chain2_small_kernel<3, 6, 5, 1>,
                                 step_chain2_small_kernel<2, 8, 2, 0>, step_chain2_small_kernel<2, 8, 2, 1>,
                                 step_chain2_small_kernel<2, 5, 2, 0>, step_chain2_small_kernel<2, 5, 2, 1>};
    int64_t items = int64_t(p0.tokens) * p0.c1_tiles;
    if (p1) items = std::max(items, int64_t(p1->tokens) * p1->c1_tiles);
    if (items <= kChain2FineMaxItems) {
        // few items: one wave per (token, c1 tile, c2 tile)
        static const k_t fine[6] = {step_chain2_fine_kernel<3, 6, 0>, step_chain2_fine_kernel<3, 6, 1>,
                                    step_chain2_fine_kernel<2, 8, 0>, step_chain2_fine_kernel<2, 8, 1>,
                                    step_chain2_fine_kernel<2, 5, 0>, step_chain2_fine_kernel<2, 5, 1>};
        int64_t fine_items = int64_t(p0.tokens) * p0.c1_tiles * ((p0.C2 + 31) / 32);
        if (p1) fine_items = std::max(fine_items, int64_t(p1->tokens) * p1->c1_tiles * ((p1->C2 + 31) / 32));
        hipLaunchKernelGGL(fine[s1.chain_cfg * 2 + s1.chain_run_c1], dim3(uint32_t(fine_items), p1 ? 2 : 1), dim3(64), 0, st, p0,
                           p1 ? *p1 : p0);
        return hipGetLastError() == hipSuccess ? TN_OK : TN_ERR_HIP;
    }
    hipLaunchKernelGGL(small[s1.chain_cfg * 2 + s1.chain_run_c1], dim3(uint32_t((items + 3) / 4), p1 ? 2 : 1), dim3(256), 0, st,
                       p0, p1 ? *p1 : p0);
    return hipGetLastError() == hipSuccess ? TN_OK : TN_ERR_HIP;
}

int launch_chain2(const tn_linear_s* h, const DevStep& s1, const DevStep& s2, const void* A, void* Out, int64_t tokens,
                  hipStream_t st) {
    using k_t = void (*)(Chain2Args);
    static const k_t kerns[6] = {step_chain2_kernel<3, 6, 5, 0>, step_chain2_kernel<3, 6, 5, 1>,
                                 step_chain2_kernel<2, 8, 2, 0>, step_chain2_kernel<2, 8, 2, 1>,
                                 step_chain2_kernel<2, 5, 2, 0>, step_chain2_kernel<2, 5, 2, 1>};
    static const size_t smem[3] = {chain2_smem_bytes<3, 6, 5>(), chain2_smem_bytes<2, 8, 2>(), chain2_smem_bytes<2, 5, 2>()};
    if (!s1.packed) {                      // configuration call (create time)
        for (int i = 0; i < 6; ++i)
            if (hipFuncSetAttribute(reinterpret_cast<const void*>(kerns[i]), hipFuncAttributeMaxDynamicSharedMemorySize,
                                    int(smem[i / 2])) != hipSuccess)
                return TN_ERR_HIP;
        return TN_OK;
    }
    Chain2Args p = chain2_args(s1, s2, A, Out, tokens);
    if (chain2_small_applies(h, s1, tokens)) return launch_chain2_small(s1, p, nullptr, st);
    // a wave per token when there are tokens enough to fill the chip, else a wave per (token, c1 tile)
    const int64_t waves = int64_t(h->num_cus) * 4;
    p.tiles_per_item = tokens >= waves ? p.c1_tiles : 1;
    const int64_t n_groups = (p.c1_tiles + p.tiles_per_item - 1) / p.tiles_per_item;
    const int64_t items = tokens * n_groups;
    // the narrow instantiation leaves room for two workgroups per CU
    const int64_t wgs = int64_t(h->num_cus) * (s1.chain_cfg == 2 ? 2 : 1);
    dim3 grid(uint32_t(std::min<int64_t>((items + 3) / 4, wgs)));
    hipLaunchKernelGGL(kerns[s1.chain_cfg * 2 + s1.chain_run_c1], grid, dim3(256), smem[s1.chain_cfg], st, p);
    return hipGetLastError() == hipSuccess ? TN_OK : TN_ERR_HIP;
}

// A chained factor pair and the wide step after it as one launch (step_chain2_split_kernel), for calls of a few
// tokens: applicable when the pair runs on one of the two small instantiations, the wide step would run on the
// split-K kernel with one split and 8 waves, its rows are the tokens themselves (R = 1), its K fits the kernel's
// register budget and every (token, column tile) item of the pair gets a wave of its own.
constexpr int64_t kFusedDecodeMaxZBytes = 32 * 1024;
constexpr size_t kFusedDecodeRedBytes = 8 * 1024 * sizeof(float);
constexpr int kFusedDecodeKPW = 5;           // pieces of 64 k of the wide step per wave: K <= 8 * 5 * 64 = 2560

bool chain2_split_applies(const tn_linear_s* h, const DevStep& s1, const DevStep& s3, int64_t tokens) {
    if (!s1.fuse_next || s1.chain_cfg == 0 || (h->flags & (TN_FLAG_NO_SPLIT_K | TN_FLAG_NO_DECODE_FUSION))) return false;
    if (s3.fuse_next || s3.variant == VAR_SCALAR || s3.amode != 0 || s3.plan.R != 1) return false;
    if (tokens * ((s1.plan.C + 31) / 32) > 8 || s3.Kp > 8 * kFusedDecodeKPW * 64) return false;
    if (tokens * s3.plan.a_tok_stride * 2 > kFusedDecodeMaxZBytes) return false;
    const SplitCfg sc = split_config(s3, tokens);
    // (however many splits the wide step would take on its own: here a workgroup always walks the whole K, which for a
    // core this small is a few hundred KB per workgroup at most)
    return sc.use && sc.tm == 1 && sc.nw == 8 && sc.row_tiles == 1;
}

struct Chain2SplitArgs {
    Chain2Args c;
    StepArgs a;
    int z_bytes = 0;
    int kern = 0;
    uint32_t col_blocks = 0;
};

Chain2SplitArgs chain2_split_args(const DevStep& s1, const DevStep& s2, const DevStep& s3, const void* A, void* Out,
                                  int64_t tokens) {
    Chain2SplitArgs r;
    r.c = chain2_args(s1, s2, A, nullptr, tokens);      // the pair's result stays in LDS
    StepArgs& a = r.a;
    a.A = nullptr;                                       // likewise
    a.B = s3.q4_codes ? s3.q4_codes : s3.packed;
    a.Bs = s3.q4_scales;
    a.Out = Out;
    a.arow = nullptr;
    a.acol = nullptr;
    a.crow = s3.crow;
    a.ccol = s3.ccol;
    a.a_tok_stride = s3.plan.a_tok_stride;
    a.c_tok_stride = s3.plan.c_tok_stride;
    a.total_rows = uint32_t(tokens);
    a.R = 1;
    a.K = int32_t(s3.plan.K);
    a.Kp = s3.Kp;
    a.C = int32_t(s3.plan.C);
    a.Cp = s3.Cp;
    r.z_bytes = int((tokens * s3.plan.a_tok_stride * 2 + 255) & ~int64_t(255));
    r.kern = (s1.chain_cfg - 1) * 2 + s1.chain_run_c1 + (s3.q4_codes ? 4 : 0);
    r.col_blocks = uint32_t((s3.plan.C + 31) / 32);
    return r;
}

// One launch for one layer (p1 == nullptr) or for two layers on the same instantiation (grid.y = 2).
int launch_chain2_split(const Chain2SplitArgs* p0, const Chain2SplitArgs* p1, hipStream_t st) {
    using k_t = void (*)(Chain2Args, StepArgs, int, Chain2Args, StepArgs, int);
    static const k_t kerns[8] = {
        step_chain2_split_kernel<8, 0, kFusedDecodeKPW, 0>, step_chain2_split_kernel<8, 1, kFusedDecodeKPW, 0>,
        step_chain2_split_kernel<5, 0, kFusedDecodeKPW, 0>, step_chain2_split_kernel<5, 1, kFusedDecodeKPW, 0>,
        step_chain2_split_kernel<8, 0, kFusedDecodeKPW, 1>, step_chain2_split_kernel<8, 1, kFusedDecodeKPW, 1>,
        step_chain2_split_kernel<5, 0, kFusedDecodeKPW, 1>, step_chain2_split_kernel<5, 1, kFusedDecodeKPW, 1>};
    if (!p0) {                             // configuration call (create time)
        for (int i = 0; i < 8; ++i)
            if (hipFuncSetAttribute(reinterpret_cast<const void*>(kerns[i]), hipFuncAttributeMaxDynamicSharedMemorySize,
                                    int(kFusedDecodeRedBytes + size_t(kFusedDecodeMaxZBytes))) != hipSuccess)
                return TN_ERR_HIP;
        return TN_OK;
    }
    const Chain2SplitArgs& q = p1 ? *p1 : *p0;
    const uint32_t blocks = std::max(p0->col_blocks, q.col_blocks);
    const size_t smem = kFusedDecodeRedBytes + size_t(std::max(p0->z_bytes, q.z_bytes));
    hipLaunchKernelGGL(kerns[p0->kern], dim3(blocks, p1 ? 2 : 1), dim3(512), smem, st, p0->c, p0->a, p0->z_bytes, q.c, q.a,
                       q.z_bytes);
    return hipGetLastError() == hipSuccess ? TN_OK : TN_ERR_HIP;
}

// 4-bit streams for the decode-size launches of a quantised layer: a step qualifies when its tensor is one of the
// caller's (not merged, no traced index pair), its k walks that tensor in memory order (K consecutive elements per
// column, K a multiple of 32) and every column starts on a block boundary. Such a step's split-K launches then read
// 0.53 bytes per parameter instead of 2. The bf16 packed tensor stays: larger calls run on it.
bool q4_streamable(const tn_linear_s* h, const tn::Step& p) {
    if (p.slot < 0 || p.slot >= h->plan.n_caller_tensors || p.trace_extent != 1 || p.K % 32 || p.kdims.empty()) return false;
    int64_t run = 1;
    for (size_t j = p.kdims.size(); j-- > 0;) {
        if (p.kdims[j].stride != run) return false;
        run *= p.kdims[j].extent;
    }
    for (const tn::GatherDim& d : p.cdims)
        if (d.stride % 32) return false;
    return true;
}

int prepare_q4_stream(tn_linear_s* h, hipStream_t st) {
    if (!(h->flags & TN_FLAG_QUANT_MXFP4) || (h->flags & (TN_FLAG_NO_Q4_STREAM | TN_FLAG_SCALAR_KERNELS | TN_FLAG_NO_SPLIT_K)) ||
        h->plan.dtype != TN_DTYPE_BF16)
        return TN_OK;
    for (DevStep& s : h->steps) {
        const tn::Step& p = s.plan;
        if (s.variant == VAR_SCALAR || !q4_streamable(h, p)) continue;
        // worth it only where a decode-size launch is a stream of this tensor: the split-K kernel must take one-row calls
        if (!split_config(s, p.R).use) continue;
        const int n_chunks = s.Kp / 64, col_blocks = int((p.C + 31) / 32);
        const int64_t pieces = int64_t(col_blocks) * n_chunks * 64;
        const int64_t code_bytes = pieces * 16, scale_bytes = (pieces + 255) & ~int64_t(255);
        if (hipMalloc(&s.q4_codes, size_t(code_bytes + scale_bytes)) != hipSuccess) return TN_ERR_ALLOC;
        s.q4_scales = static_cast<char*>(s.q4_codes) + code_bytes;
        h->packed_bytes += code_bytes + scale_bytes;
        h->q4_stream_bytes += code_bytes + scale_bytes;
        Q4PackArgs a;
        memset(&a, 0, sizeof(a));
        a.codes = static_cast<const unsigned char*>(h->quant_codes[size_t(p.slot)]);
        a.exps = static_cast<const signed char*>(h->quant_exps[size_t(p.slot)]);
        a.out_codes = static_cast<uint4*>(s.q4_codes);
        a.out_scales = static_cast<unsigned char*>(s.q4_scales);
        a.C = int32_t(p.C);
        a.K = int32_t(p.K);
        a.n_chunks = n_chunks;
        a.col_blocks = col_blocks;
        a.nc = int32_t(p.cdims.size());
        for (size_t j = 0; j < p.cdims.size(); ++j) {
            a.cext[j] = p.cdims[j].extent;
            a.cstr[j] = p.cdims[j].stride;
        }
        hipLaunchKernelGGL(q4_stream_pack_kernel, dim3(uint32_t(std::min<int64_t>((pieces + 255) / 256, 16384))), dim3(256), 0, st, a);
        if (hipGetLastError() != hipSuccess) return TN_ERR_HIP;
    }
    return TN_OK;
}

// Kernels that use more than 64 KB of LDS need their limit raised once per device. Done at create
// time (never inside tn_linear_forward, which must stay legal under stream capture from its first
// call). The launchers double as configurators: called with an empty step they set the attribute of
// every kernel they can launch and return.
// Device address of the static scratch array on each GPU, looked up once per device at create time with that
// device current (every GPU holds its own copy of the array at its own address).
void* g_scratch_ptr[64] = {};

int configure_kernels(int device) {
    static bool done[64] = {};
    static std::mutex lock;                // handles may be created from several host threads
    std::lock_guard<std::mutex> guard(lock);
    if (device >= 0 && device < 64 && done[device]) return TN_OK;
    const DevStep none;                    // packed == nullptr: configuration call
    const StepArgs a{};
    const tn_linear_s* no_handle = nullptr;
    int rc = launch_pipe<2, 2, 2, 4, 1, 2>(none, a, 0, nullptr);
    if (rc == TN_OK) rc = launch_pipe<4, 1, 2, 4, 1, 2>(none, a, 0, nullptr);
    if (rc == TN_OK) rc = configure_pingpong();
    if (rc == TN_OK) rc = launch_chain2(no_handle, none, none, nullptr, nullptr, 0, nullptr);
    if (rc == TN_OK) rc = launch_chain2_split(nullptr, nullptr, nullptr);
    for (int i = 0; i < kSkinnyKernels && rc == TN_OK; ++i)
        if (hipFuncSetAttribute(reinterpret_cast<const void*>(skinny_kernels()[i]), hipFuncAttributeMaxDynamicSharedMemorySize,
                                int(kSplitLdsRowBytes)) != hipSuccess)
            rc = TN_ERR_HIP;
    for (int i = 0; i < kSplitLdsKernels && rc == TN_OK; ++i)
        if (hipFuncSetAttribute(reinterpret_cast<const void*>(split_lds_kernels()[i]), hipFuncAttributeMaxDynamicSharedMemorySize,
                                int(kSplitLdsRowBytes)) != hipSuccess)
            rc = TN_ERR_HIP;
    if (rc == TN_OK &&
        (hipFuncSetAttribute(reinterpret_cast<const void*>(&step_pair_kernel<kPairStages, kPairBar>),
                             hipFuncAttributeMaxDynamicSharedMemorySize, int(kPairSmemBytes)) != hipSuccess ||
         hipFuncSetAttribute(reinterpret_cast<const void*>(small_chain_kernel<float>),
                             hipFuncAttributeMaxDynamicSharedMemorySize, int(kSmallChainMaxSmem)) != hipSuccess ||
         hipFuncSetAttribute(reinterpret_cast<const void*>(small_chain_kernel<bf16_t>),
                             hipFuncAttributeMaxDynamicSharedMemorySize, int(kSmallChainMaxSmem)) != hipSuccess))
        rc = TN_ERR_HIP;
    for (int cfg = 0; cfg < tn::kKronConfigs && rc == TN_OK; ++cfg) rc = kron_dispatch(cfg, nullptr, 0, nullptr);
    if (rc == TN_OK) rc = gen_mfma_dispatch(nullptr, 0, nullptr);
    if (rc == TN_OK) rc = gen_mfma_both_dispatch(nullptr, nullptr, 0, nullptr);
    if (rc == TN_OK && device >= 0 && device < 64) {
        void* ptr = nullptr;
        if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess || !ptr) rc = TN_ERR_HIP;
        else g_scratch_ptr[device] = ptr;
    }
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
        case TN_QUERY_KRON_CHAINABLE: {
            tn::KronDims d;
            *value = (!tn::pair_chainable(p) && tn::kron_shape(p, &d)) ? 1 + d.cfg : 0;
            return TN_OK;
        }
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

// ---- gradients with respect to the parameter tensors (TN_FLAG_TRAINABLE) ----
constexpr int64_t kMaxGradPartialBytes = int64_t(256) << 20;
constexpr int64_t kGradMfmaMinExtent = 32;

// Row ranges a gradient launch is split into: enough workgroups to fill the chip, at least 64 rows each, partial
// tiles within `cap` bytes.
// How grad_param_mfma_kernel loads dOut (d) and In (i) of a step: 1 = 16-byte pieces along the columns, 2 = 16-byte
// pieces along the rows (dOut only), 0 = element by element.
struct GradModes {
    int d = 0, i = 0;
};

GradModes grad_modes(const tn::Step& p) {
    GradModes m;
    if (p.c_vec == 8 && p.C % 8 == 0) m.d = 1;
    else if (p.r_vec == 8 && p.R % 8 == 0) m.d = 2;
    if (p.K % 8 == 0 && p.a_tok_stride % 8 == 0 && (p.a_plain || p.a_vec == 8)) m.i = 1;
    return m;
}

// bf16 steps whose tensor is at least a quarter of a 128 x 128 tile in both directions run on the matrix cores, and so
// do skinny ones (8 to 31 one way, 32 or more the other: the boundary cores of a train) when both operands come in
// 16-byte pieces: those are bound by reading the long operand once, which the tile kernel does in full lines
bool grad_on_mfma(const tn_linear_s* h, const tn::Step& p) {
    if (h->elt != 2) return false;
    if (p.C >= kGradMfmaMinExtent && p.K >= kGradMfmaMinExtent) return true;
    const GradModes m = grad_modes(p);
    return m.d != 0 && m.i != 0 && std::min(p.C, p.K) >= 8 && std::max(p.C, p.K) >= kGradMfmaMinExtent;
}

int grad_splits(const tn_linear_s* h, const tn::Step& p, int64_t rows, int64_t cap) {
    const int64_t edge = grad_on_mfma(h, p) ? 128 : 64;
    const int64_t tiles = ((p.C + edge - 1) / edge) * ((p.K + edge - 1) / edge);
    int64_t n = std::max<int64_t>(1, ((edge == 128 ? 2 : 4) * int64_t(h->num_cus) + tiles - 1) / tiles);
    n = std::min<int64_t>(n, std::max<int64_t>(1, rows / 64));
    n = std::min<int64_t>(n, std::max<int64_t>(1, cap / (p.C * p.K * 4)));
    n = std::min<int64_t>(n, 65535);
    // the matrix-core kernel keeps the tiles of a split on one XCD when the splits come in eights
    if (edge == 128 && n > 8 && (n + 7) / 8 * 8 * p.C * p.K * 4 <= cap && (n + 7) / 8 * 8 <= std::max<int64_t>(1, rows / 64)) n = (n + 7) / 8 * 8;
    return int(n);
}

int prepare_backward(tn_linear_s* h, const tn_linear_desc* desc, hipStream_t st) {
    const size_t n = h->steps.size();
    if (!h->plan.merges.empty()) return TN_ERR_UNSUPPORTED;
    h->bwd.resize(n);
    std::vector<int32_t> tab;
    std::vector<size_t> off(n, 0);
    for (size_t s = 1; s < n; ++s) {
        const tn::Step& f = h->steps[s].plan;
        if (!f.a_plain) return TN_ERR_UNSUPPORTED;      // only a first step gathers
        off[s] = tab.size();
        for (int64_t r = 0; r < f.R; ++r) tab.push_back(int32_t(r * f.K));
        for (int64_t k = 0; k < f.K; ++k) tab.push_back(int32_t(k));
    }
    if (hipMalloc(reinterpret_cast<void**>(&h->bwd_tables), std::max<size_t>(1, tab.size()) * sizeof(int32_t)) != hipSuccess)
        return TN_ERR_ALLOC;
    if (hipMemcpyAsync(h->bwd_tables, tab.data(), tab.size() * sizeof(int32_t), hipMemcpyHostToDevice, st) != hipSuccess ||
        hipStreamSynchronize(st) != hipSuccess)
        return TN_ERR_HIP;
    for (size_t s = 1; s < n; ++s) {
        const DevStep& fs = h->steps[s];
        const tn::Step& f = fs.plan;
        DevStep& b = h->bwd[s];
        b.plan.tensor = f.tensor;
        b.plan.slot = f.slot;
        b.plan.R = f.R;
        b.plan.K = f.C;
        b.plan.C = f.K;
        b.plan.a_plain = false;                         // dOut is read through the forward step's scatter tables
        b.plan.a_tok_stride = f.c_tok_stride;
        b.plan.c_tok_stride = f.a_tok_stride;
        b.plan.c_vec = (f.K % 8 == 0) ? 8 : 1;
        b.plan.r_vec = 1;
        b.plan.a_vec = (f.c_vec == 8 && f.C % 8 == 0) ? 8 : 1;       // dOut's columns in 16-byte runs: gathered as such
        b.plan.kdims = f.cdims;
        b.plan.cdims = f.kdims;
        b.plan.trace_extent = f.trace_extent;
        b.plan.trace_stride = f.trace_stride;
        b.plan.flops = f.flops;
        b.arow = fs.crow;
        b.acol = fs.ccol;
        b.crow = h->bwd_tables + off[s];
        b.ccol = b.crow + f.R;
        choose_variant(h, &b, desc->flags);
        const int64_t bytes = int64_t(b.Cp) * b.Kp * h->elt;
        if (hipMalloc(&b.packed, size_t(bytes)) != hipSuccess) return TN_ERR_ALLOC;
        h->packed_bytes += bytes;
        PackArgs pa;
        memset(&pa, 0, sizeof(pa));
        pa.src = desc->tensors[f.slot];
        pa.dst = b.packed;
        pa.K = int32_t(b.plan.K);
        pa.Kp = b.Kp;
        pa.C = int32_t(b.plan.C);
        pa.Cp = b.Cp;
        fill_pack_dims(&pa, b.plan.kdims, b.plan.cdims);
        pa.trace_extent = f.trace_extent;
        pa.trace_stride = f.trace_stride;
        launch_pack(pa, h->elt, st);
        if (hipGetLastError() != hipSuccess) return TN_ERR_HIP;
    }
    // workspace of a backward pass: the saved inputs of steps 1 .. n-1 and two gradient buffers
    h->bwd_saved_off.assign(n, 0);
    int64_t saved = 0;
    for (size_t s = 1; s < n; ++s) {
        h->bwd_saved_off[s] = saved;
        saved += (h->steps[s].plan.a_tok_stride + 127) & ~int64_t(127);
    }
    h->bwd_saved_elems = saved;
    const int64_t dbuf = (h->plan.max_intermediate + 127) & ~int64_t(127);
    const int64_t per_token = (saved + 2 * dbuf) * h->elt;
    int64_t max_r = 1;
    for (const auto& s : h->steps) max_r = std::max(max_r, s.plan.R);
    const int64_t limit = desc->workspace_limit_bytes > 0 ? desc->workspace_limit_bytes : kDefaultWorkspaceBytes;
    int64_t chunk = h->max_tokens;
    if (per_token > 0) chunk = std::min<int64_t>(chunk, std::max<int64_t>(1, limit / per_token));
    chunk = std::max<int64_t>(1, std::min<int64_t>(chunk, ((int64_t(1) << 31) - 1024) / max_r));
    h->bwd_chunk = chunk;
    h->bwd_ws_bytes = std::max<int64_t>(256, chunk * per_token);
    if (hipMalloc(&h->bwd_ws, size_t(h->bwd_ws_bytes)) != hipSuccess) return TN_ERR_ALLOC;
    int64_t need = 0;
    for (const auto& s : h->steps)
        need = std::max(need, int64_t(grad_splits(h, s.plan, chunk * s.plan.R, kMaxGradPartialBytes)) * s.plan.C * s.plan.K * 4);
    h->bwd_partial_bytes = need;
    if (hipMalloc(reinterpret_cast<void**>(&h->bwd_partial), size_t(need)) != hipSuccess) return TN_ERR_ALLOC;
    h->trainable = true;
    return TN_OK;
}

// dP of one step from dOut and the step's saved input, into the caller's tensor.
int launch_param_gradient(const tn_linear_s* h, const DevStep& s, const void* dOut, const void* In, float* grad,
                          int64_t grad_elems, int64_t tokens, bool accumulate, hipStream_t st) {
    const tn::Step& p = s.plan;
    const int64_t rows = tokens * p.R;
    const int n_split = grad_splits(h, p, rows, h->bwd_partial_bytes);
    if (int64_t(n_split) * p.C * p.K * 4 > h->bwd_partial_bytes) return TN_ERR_UNSUPPORTED;
    GradArgs a;
    a.dOut = dOut;
    a.In = In;
    a.partial = h->bwd_partial;
    a.crow = s.crow;
    a.ccol = s.ccol;
    a.arow = s.arow;
    a.acol = s.acol;
    a.c_tok_stride = p.c_tok_stride;
    a.a_tok_stride = p.a_tok_stride;
    a.total_rows = uint32_t(rows);
    a.R = uint32_t(p.R);
    a.K = int32_t(p.K);
    a.C = int32_t(p.C);
    a.rows_per_split = uint32_t((rows + n_split - 1) / n_split);
    const bool mfma = grad_on_mfma(h, p);
    if (mfma) a.rows_per_split = (a.rows_per_split + 31u) & ~31u;        // the tile kernel's row ranges start at multiples of 32
    const GradModes gm = grad_modes(p);
    a.d_mode = gm.d;
    a.i_mode = gm.i;
    const int64_t edge = mfma ? 128 : 64;
    dim3 grid(uint32_t((p.C + edge - 1) / edge), uint32_t((p.K + edge - 1) / edge), uint32_t(n_split));
    if (grid.y > 65535) return TN_ERR_UNSUPPORTED;
    a.c_tiles = int32_t(grid.x);
    a.k_tiles = int32_t(grid.y);
    a.n_split = n_split;
    if (mfma) {
        const int64_t wgs = int64_t(grid.x) * grid.y * n_split;
        if (wgs > (int64_t(1) << 30)) return TN_ERR_UNSUPPORTED;
        hipLaunchKernelGGL(grad_param_mfma_kernel, dim3(uint32_t(wgs)), dim3(256), 0, st, a);
    }
    else if (h->elt == 2)
        hipLaunchKernelGGL(grad_param_kernel<bf16_t>, grid, dim3(256), 0, st, a);
    else
        hipLaunchKernelGGL(grad_param_kernel<float>, grid, dim3(256), 0, st, a);
    if (p.trace_extent > 1 && !accumulate)
        hipLaunchKernelGGL(grad_fill_kernel, dim3(uint32_t(std::min<int64_t>((grad_elems + 255) / 256, 4096))), dim3(256), 0, st,
                           grad, grad_elems);
    GradOutArgs o;
    memset(&o, 0, sizeof(o));
    o.partial = h->bwd_partial;
    o.grad = grad;
    o.C = int32_t(p.C);
    o.K = int32_t(p.K);
    o.n_split = n_split;
    o.accumulate = accumulate ? 1 : 0;
    o.nk = int32_t(p.kdims.size());
    o.nc = int32_t(p.cdims.size());
    for (int j = 0; j < o.nk; ++j) {
        o.kext[j] = p.kdims[size_t(j)].extent;
        o.kstr[j] = p.kdims[size_t(j)].stride;
    }
    for (int j = 0; j < o.nc; ++j) {
        o.cext[j] = p.cdims[size_t(j)].extent;
        o.cstr[j] = p.cdims[size_t(j)].stride;
    }
    o.trace_extent = p.trace_extent;
    o.trace_stride = p.trace_stride;
    const int64_t total = p.C * p.K;
    hipLaunchKernelGGL(grad_reduce_kernel, dim3(uint32_t(std::min<int64_t>((total + 255) / 256, 8192))), dim3(256), 0, st, o);
    return hipGetLastError() == hipSuccess ? TN_OK : TN_ERR_HIP;
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

int tn_linear_version(void) { return 6; }

const char* tn_linear_strerror(int status) {
    switch (status) {
        case TN_OK: return "success";
        case TN_ERR_INVALID_ARG: return "invalid argument";
        case TN_ERR_UNSUPPORTED: return "unsupported configuration";
        case TN_ERR_ALLOC: return "allocation failed";
        case TN_ERR_HIP: return "HIP runtime error";
        case TN_ERR_SCRATCH: return "the call needs more scratch memory than the library's static buffer holds";
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

int tn_linear_create(tn_linear_t* out, const tn_linear_desc* desc_in) {
    if (!out || !desc_in || !desc_in->tensors) return TN_ERR_INVALID_ARG;
    tn_linear_desc eff = *desc_in;             // the description create works with: tensors may be replaced below
    const tn_linear_desc* desc = &eff;
    std::vector<const void*> eff_tensors;
    if ((desc->flags & TN_FLAG_QUANT_MXFP4) && (desc->dtype != TN_DTYPE_BF16 || (desc->flags & TN_FLAG_TRAINABLE)))
        return TN_ERR_INVALID_ARG;
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
    if (desc->flags & TN_FLAG_QUANT_MXFP4) {
        // quantise every tensor; everything below (merging, packing, lazily merged plans) sees the dequantised copies
        for (int i = 0; i < desc->n_tensors; ++i) {
            const int64_t n = tn::caller_tensor_elems(desc, i);
            void *codes = nullptr, *exps = nullptr, *deq = nullptr;
            if (n <= 0 || hipMalloc(&codes, size_t((n + 1) / 2)) != hipSuccess) {
                free_handle(h);
                return TN_ERR_ALLOC;
            }
            h->quant_codes.push_back(codes);
            if (hipMalloc(&exps, size_t((n + 31) / 32)) != hipSuccess) {
                free_handle(h);
                return TN_ERR_ALLOC;
            }
            h->quant_exps.push_back(exps);
            if (hipMalloc(&deq, size_t(n) * 2) != hipSuccess) {
                free_handle(h);
                return TN_ERR_ALLOC;
            }
            h->create_temps.push_back(deq);
            h->quant_elems.push_back(n);
            h->quant_bytes += (n + 1) / 2 + (n + 31) / 32;
            const int64_t blocks = (n + 31) / 32;
            hipLaunchKernelGGL(mxfp4_quantize_kernel, dim3(uint32_t(std::min<int64_t>((blocks + 255) / 256, 16384))), dim3(256), 0,
                               st, static_cast<const bf16_t*>(desc_in->tensors[i]), n, static_cast<unsigned char*>(codes),
                               static_cast<signed char*>(exps), static_cast<bf16_t*>(deq));
            eff_tensors.push_back(deq);
        }
        if (hipGetLastError() != hipSuccess) {
            (void)hipStreamSynchronize(st);
            free_handle(h);
            return TN_ERR_HIP;
        }
        eff.tensors = eff_tensors.data();
    }
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
    // offset tables of every step (arow | acol | crow | ccol each): one allocation, one copy; the host copy
    // lives until create's final synchronisation
    std::vector<int32_t> host_tab;
    {
        std::vector<size_t> tab_off(h->steps.size());
        for (size_t i = 0; i < h->steps.size(); ++i) {
            DevStep& s = h->steps[i];
            s.plan = h->plan.steps[i];
            s.no_skinny = (desc->flags & TN_FLAG_NO_SKINNY) != 0;
            choose_variant(h, &s, desc->flags);
            const tn::Step& p = s.plan;
            tab_off[i] = host_tab.size();
            host_tab.insert(host_tab.end(), p.arow.begin(), p.arow.end());
            host_tab.insert(host_tab.end(), p.acol.begin(), p.acol.end());
            host_tab.insert(host_tab.end(), p.crow.begin(), p.crow.end());
            host_tab.insert(host_tab.end(), p.ccol.begin(), p.ccol.end());
        }
        if (hipMalloc(reinterpret_cast<void**>(&h->tables), std::max<size_t>(1, host_tab.size()) * sizeof(int32_t)) != hipSuccess ||
            hipMemcpyAsync(h->tables, host_tab.data(), host_tab.size() * sizeof(int32_t), hipMemcpyHostToDevice, st) != hipSuccess) {
            (void)hipStreamSynchronize(st);
            release_temps();
            free_handle(h);
            return TN_ERR_ALLOC;
        }
        for (size_t i = 0; i < h->steps.size(); ++i) {
            DevStep& s = h->steps[i];
            const tn::Step& p = s.plan;
            const int32_t* t = h->tables + tab_off[i];
            if (!p.a_plain) {
                s.arow = t;
                s.acol = t + p.arow.size();
            }
            s.crow = t + p.arow.size() + p.acol.size();
            s.ccol = s.crow + p.crow.size();
        }
    }
    for (size_t i = 0; i < h->steps.size(); ++i) {
        DevStep& s = h->steps[i];
        const tn::Step& p = s.plan;
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
    rc = plan_small_chain(h, st);
    if (rc == TN_OK) rc = prepare_pair(h, st);
    if (rc == TN_OK) rc = prepare_kron(h, st);
    if (rc == TN_OK) rc = plan_chain2(h, st);
    if (rc == TN_OK) rc = prepare_q4_stream(h, st);
    if (rc == TN_OK) {
        const int64_t before = h->packed_bytes;
        rc = prepare_lazy(h, desc, st);
        h->lazy_kept_bytes = h->packed_bytes - before;
    }
    if (rc == TN_OK && (desc->flags & TN_FLAG_TRAINABLE)) rc = prepare_backward(h, desc, st);
    if (rc != TN_OK) {
        (void)hipStreamSynchronize(st);
        free_handle(h);
        return rc;
    }
    // workspace: two ping-pong buffers, each chunk_tokens * max_intermediate elements, and the
    // partial-sum buffer of the split-K kernel; allocated here, or carved out of the caller's block
    int64_t per_token = h->plan.max_intermediate * h->elt;
    if (h->kron && h->kron_min_tokens <= 1) per_token = 0;      // every call runs the one-launch kernel: no intermediates
    if (h->pair && h->pair_min_tokens <= 1) per_token = 0;
    int64_t max_r = 1;
    for (const auto& s : h->steps) max_r = std::max(max_r, s.plan.R);
    const int64_t row_cap = ((int64_t(1) << 31) - 1024) / max_r;      // rows of a pass are indexed with 32 bits
    const bool split_ok = !(desc->flags & TN_FLAG_NO_SPLIT_K) && h->elt == 2;
    auto partial_need = [&](int64_t chunk) {
        int64_t need = 0;
        if (!split_ok) return need;
        if (h->kron) {
            for (int64_t t = 1; t <= std::min<int64_t>(h->max_tokens, 4 * int64_t(h->num_cus)); ++t)
                need = std::max(need, kron_geometry(h, h->kron_dims, t, kMaxPartialBytes).partial_bytes);
            if (h->kron_min_tokens <= 1) return need;
        }
        if (h->pair) {
            for (int64_t t = h->pair_min_tokens; t <= std::min<int64_t>(h->max_tokens, 32 * int64_t(h->num_cus)); ++t)
                need = std::max(need, pair_geometry(h, t, kMaxPartialBytes).partial_bytes);
            if (h->pair_min_tokens <= 1) return need;
        }
        if (h->lazy)
            for (int64_t t = h->lazy_min_tokens; t <= std::min<int64_t>(h->max_tokens, 4 * int64_t(h->num_cus)); ++t)
                need = std::max(need, kron_geometry(h, h->lazy_dims, t, kMaxPartialBytes).partial_bytes);
        for (const auto& s : h->steps)
            for (int64_t t = 1; t <= chunk; ++t) {
                SplitCfg c = split_config(s, t * s.plan.R);
                if (!c.use) break;          // larger passes only add tiles
                need = std::max(need, c.partial_bytes);
            }
        return need;
    };
    // a lazily merged plan needs room for its slices: in the caller's block they share the space of the two
    // buffers (never in use at the same time), otherwise they get an allocation of their own
    if (h->lazy) {
        const int64_t room = desc->workspace
                                 ? desc->workspace_bytes - (split_ok ? std::min<int64_t>(kMaxPartialBytes, desc->workspace_bytes / 4) : 0) - 512
                                 : (desc->workspace_limit_bytes > 0 ? desc->workspace_limit_bytes : kDefaultWorkspaceBytes);
        if (room < h->lazy_slice_bytes) {
            // no room for the slices: every call runs the compact steps, and what the lazy plan kept goes away
            // (the kernels that wrote these buffers may still be running on the stream)
            if (hipStreamSynchronize(st) != hipSuccess) {
                free_handle(h);
                return TN_ERR_HIP;
            }
            h->lazy = false;
            h->packed_bytes -= h->lazy_kept_bytes;
            h->lazy_kept_bytes = 0;
            for (void* v : h->lazy_sources) (void)hipFree(v);
            h->lazy_sources.clear();
            for (int w = 0; w < 2; ++w)
                if (h->lazy_gen_tables[w]) {
                    (void)hipFree(h->lazy_gen_tables[w]);
                    h->lazy_gen_tables[w] = nullptr;
                    h->lazy_mfma[w] = false;
                }
            if (h->lazy_tables) (void)hipFree(h->lazy_tables);
            h->lazy_tables = nullptr;
        }
    }
    // with the chained pair kernel or a lazily merged plan only calls below the token threshold use the buffers
    int64_t ws_tokens = h->pair ? std::min<int64_t>(h->max_tokens, h->pair_min_tokens - 1) : h->max_tokens;
    // (one token's buffers stay: calls that may not use the rebuilt plan - profiled steps, the entry point that
    // allocates nothing - run the compact steps token by token)
    if (h->lazy) ws_tokens = std::min<int64_t>(ws_tokens, std::max<int64_t>(1, h->lazy_min_tokens - 1));
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
        if (h->lazy) h->lazy_slices = base + part;
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
        if (h->lazy) {
            if (hipMalloc(&h->lazy_slices, size_t(h->lazy_slice_bytes)) != hipSuccess) {
                free_handle(h);
                return TN_ERR_ALLOC;
            }
            h->workspace_bytes += h->lazy_slice_bytes;
        }
    }
    for (int w = 0; w < 2 && h->lazy; ++w) {
        h->lazy_gen[w].dst = static_cast<char*>(h->lazy_slices) + (w == 0 ? 0 : h->lazy_h1_offset);
        h->lazy_gen_mfma[w].dst = h->lazy_gen[w].dst;
    }
    h->chunk_tokens = chunk;
    if (h->lazy && h->owns_workspace) {
        // the handle's own workspace: nobody else writes the slices, so they are built here once and every call
        // finds them (a layer that shares a caller's block rebuilds them per call instead)
        rc = launch_lazy_generate(h, st);
        if (rc != TN_OK) {
            (void)hipStreamSynchronize(st);
            free_handle(h);
            return rc;
        }
        h->lazy_slices_kept = true;
    }
    {
        std::vector<int> fuse(h->steps.size(), 0);
        for (size_t i = 0; i < h->steps.size(); ++i) fuse[i] = h->steps[i].fuse_next ? 1 : 0;
        h->schedule = tn::launch_schedule(h->steps.size(), fuse);
    }
    // everything create enqueued (repacking, table uploads) is done before the handle is handed out, so
    // that a forward on any stream may follow without further ordering
    if (hipStreamSynchronize(st) != hipSuccess) {
        free_handle(h);
        return TN_ERR_HIP;
    }
    for (void* v : h->create_temps) (void)hipFree(v);
    h->create_temps.clear();
    *out = h;
    return TN_OK;
}

}  // extern "C"

namespace {

// Brackets one launch with a pair of HIP events when the handle is being profiled.
struct ProfScope {
    tn_linear_s* h;
    hipStream_t st;
    tn_linear_s::ProfRec rec;
    bool ok = true;
    ProfScope(tn_linear_s* handle, int step, hipStream_t stream) : h(handle), st(stream), rec{step, nullptr, nullptr} {
        if (!h->profiling) return;
        ok = hipEventCreate(&rec.start) == hipSuccess && hipEventCreate(&rec.stop) == hipSuccess;
        if (ok) (void)hipEventRecord(rec.start, st);
    }
    void done() {
        if (!h->profiling || !ok) return;
        (void)hipEventRecord(rec.stop, st);
        h->prof.push_back(rec);
    }
};

// One forward call in the workspace `w`. allow_lazy: calls large enough may run on the lazily merged plan,
// whose slices live in the handle's own workspace.
int forward_in(tn_linear_s* h, const Workspace& w, bool allow_lazy, const void* x, void* y, int64_t tokens,
               hipStream_t st) {
    const char* xb = static_cast<const char*>(x);
    char* yb = static_cast<char*>(y);
    if (h->small_chain && (h->elt == 4 || tokens <= kSmallChainMaxBf16Tokens)) {
        // every step in one launch, tensors and intermediates in LDS
        const int64_t pass = int64_t(1) << 24;
        for (int64_t t0 = 0; t0 < tokens; t0 += pass) {
            int64_t nt = std::min(pass, tokens - t0);
            ProfScope prof(h, 0, st);
            if (!prof.ok) return TN_ERR_HIP;
            int rc = launch_small_chain(h, xb + t0 * h->plan.N * h->elt, yb + t0 * h->plan.M * h->elt, nt, st);
            prof.done();
            if (rc != TN_OK) return rc;
        }
        return TN_OK;
    }
    const bool use_pair = h->pair && tokens >= h->pair_min_tokens;
    const bool use_kron = h->kron && tokens >= h->kron_min_tokens;
    const bool use_lazy = allow_lazy && h->lazy && tokens >= h->lazy_min_tokens;
    if (use_pair || use_kron || use_lazy) {
        // both steps in one launch, no intermediate in memory; passes only bound the 32-bit token index
        // (and, for the Kronecker-sum kernel, keep a call's partial sums within their buffer)
        const int64_t pass = use_pair ? int64_t(1) << 24 : int64_t(1) << 20;
        if (!use_pair && !use_kron && !h->lazy_slices_kept) {
            // a caller's block is shared with other layers: whatever it held is gone
            int rc = launch_lazy_generate(h, st);          // not part of the profiled launch: a kernel of its own
            if (rc != TN_OK) return rc;
        }
        for (int64_t t0 = 0; t0 < tokens; t0 += pass) {
            int64_t nt = std::min(pass, tokens - t0);
            ProfScope prof(h, 0, st);
            if (!prof.ok) return TN_ERR_HIP;
            const void* xp = xb + t0 * h->plan.N * h->elt;
            void* yp = yb + t0 * h->plan.M * h->elt;
            int rc = use_pair ? launch_pair(h, w, xp, yp, nt, st)
                              : (use_kron ? launch_kron_eager(h, w, xp, yp, nt, st) : launch_kron_lazy(h, w, xp, yp, nt, st));
            prof.done();
            if (rc != TN_OK) return rc;
        }
        return TN_OK;
    }
    if (w.chunk_tokens < 1) return TN_ERR_INVALID_ARG;
    for (int64_t t0 = 0; t0 < tokens; t0 += w.chunk_tokens) {
        int64_t nt = std::min(w.chunk_tokens, tokens - t0);
        for (size_t li = 0; li < h->schedule.size(); ++li) {
            const tn::LaunchIO& l = h->schedule[li];
            const void* A = l.in == tn::kBufX ? static_cast<const void*>(xb + t0 * h->plan.N * h->elt) : w.ws[l.in];
            void* Out = l.out == tn::kBufY ? static_cast<void*>(yb + t0 * h->plan.M * h->elt) : w.ws[l.out];
            ProfScope prof(h, l.first, st);
            if (!prof.ok) return TN_ERR_HIP;
            const DevStep& s = h->steps[size_t(l.first)];
            int rc;
            if (l.steps == 2 && li + 1 < h->schedule.size() && h->schedule[li + 1].steps == 1 &&
                chain2_split_applies(h, s, h->steps[size_t(l.first) + 2], nt)) {
                // few tokens: the pair and the wide step after it in one launch, the pair's result in LDS
                const tn::LaunchIO& l2 = h->schedule[li + 1];
                void* Out2 = l2.out == tn::kBufY ? static_cast<void*>(yb + t0 * h->plan.M * h->elt) : w.ws[l2.out];
                const Chain2SplitArgs fa = chain2_split_args(s, h->steps[size_t(l.first) + 1], h->steps[size_t(l.first) + 2], A, Out2, nt);
                rc = launch_chain2_split(&fa, nullptr, st);
                ++li;
            } else {
                rc = l.steps == 2 ? launch_chain2(h, s, h->steps[size_t(l.first) + 1], A, Out, nt, st)
                                  : launch_step(h, w, s, A, Out, nt, st);
            }
            prof.done();
            if (rc != TN_OK) return rc;
        }
    }
    return TN_OK;
}

}  // namespace

extern "C" {

// the kernels read and write rows of activations in 16-byte pieces
static bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15) == 0; }

int tn_linear_forward(tn_linear_t h, const void* x, void* y, int64_t tokens, void* stream) {
    if (!h || tokens < 0) return TN_ERR_INVALID_ARG;
    if (tokens == 0) return TN_OK;
    if (!x || !y || !aligned16(x) || !aligned16(y)) return TN_ERR_INVALID_ARG;
    Workspace w;
    w.ws[0] = h->ws[0];
    w.ws[1] = h->ws[1];
    w.partial = h->partial;
    w.partial_bytes = h->partial_bytes;
    w.chunk_tokens = h->chunk_tokens;
    return forward_in(h, w, true, x, y, tokens, static_cast<hipStream_t>(stream));
}

int tn_linear_forward2(tn_linear_t ha, tn_linear_t hb, const void* x, void* ya, void* yb, int64_t tokens, void* stream) {
    if (!ha || !hb || tokens < 0) return TN_ERR_INVALID_ARG;
    if (ha->elt != hb->elt || ha->plan.N != hb->plan.N) return TN_ERR_INVALID_ARG;
    if (tokens == 0) return TN_OK;
    if (!x || !ya || !yb || !aligned16(x) || !aligned16(ya) || !aligned16(yb)) return TN_ERR_INVALID_ARG;
    hipStream_t st = static_cast<hipStream_t>(stream);
    // Launch by launch in step when the two layers have the same launch structure and the call is one pass of
    // the per-step path for both: where a launch of the decode-size kernels serves both layers, it does.
    auto per_step_path = [&](const tn_linear_s* h) {
        return !h->profiling && !(h->small_chain && (h->elt == 4 || tokens <= kSmallChainMaxBf16Tokens)) &&
               !(h->pair && tokens >= h->pair_min_tokens) && !(h->kron && tokens >= h->kron_min_tokens) &&
               !(h->lazy && tokens >= h->lazy_min_tokens) && tokens <= h->chunk_tokens;
    };
    bool together = ha != hb && per_step_path(ha) && per_step_path(hb) && ha->schedule.size() == hb->schedule.size();
    for (size_t li = 0; together && li < ha->schedule.size(); ++li) {
        const tn::LaunchIO &la = ha->schedule[li], &lb = hb->schedule[li];
        if (la.first != lb.first || la.steps != lb.steps) together = false;
        else if (la.steps == 2 && (ha->steps[size_t(la.first)].chain_cfg != hb->steps[size_t(lb.first)].chain_cfg ||
                                   ha->steps[size_t(la.first)].chain_run_c1 != hb->steps[size_t(lb.first)].chain_run_c1))
            together = false;
    }
    if (!together) {
        int rc = tn_linear_forward(ha, x, ya, tokens, stream);
        return rc != TN_OK ? rc : tn_linear_forward(hb, x, yb, tokens, stream);
    }
    tn_linear_s* hs[2] = {ha, hb};
    void* ys[2] = {ya, yb};
    Workspace ws[2];
    for (int n = 0; n < 2; ++n) {
        ws[n].ws[0] = hs[n]->ws[0];
        ws[n].ws[1] = hs[n]->ws[1];
        ws[n].partial = hs[n]->partial;
        ws[n].partial_bytes = hs[n]->partial_bytes;
        ws[n].chunk_tokens = hs[n]->chunk_tokens;
    }
    auto buffer = [&](int n, int id) -> void* {
        return id == tn::kBufX ? const_cast<void*>(x) : (id == tn::kBufY ? ys[n] : ws[n].ws[id]);
    };
    // Each layer takes the launches tn_linear_forward would give it (so that its result has the same bits); where both
    // take the same decode-size kernel at the same point of the chain, one launch serves both.
    bool skip[2] = {false, false};                 // the layer's launch at this index ran inside its previous, fused one
    for (size_t li = 0; li < ha->schedule.size(); ++li) {
        const tn::LaunchIO& l = ha->schedule[li];
        const size_t f = size_t(l.first);
        const bool has_next = li + 1 < ha->schedule.size() && ha->schedule[li + 1].steps == 1;
        int rc = TN_OK;
        bool fuse[2];
        Chain2SplitArgs fa[2];
        for (int n = 0; n < 2; ++n) {
            fuse[n] = !skip[n] && l.steps == 2 && has_next &&
                      chain2_split_applies(hs[n], hs[n]->steps[f], hs[n]->steps[f + 2], tokens);
            if (fuse[n])
                fa[n] = chain2_split_args(hs[n]->steps[f], hs[n]->steps[f + 1], hs[n]->steps[f + 2],
                                          buffer(n, hs[n]->schedule[li].in), buffer(n, hs[n]->schedule[li + 1].out), tokens);
        }
        if (fuse[0] && fuse[1] && fa[0].kern == fa[1].kern) {
            rc = launch_chain2_split(&fa[0], &fa[1], st);          // pair and wide step of both layers in one launch
            skip[0] = skip[1] = true;
        } else if (!skip[0] && !skip[1] && !fuse[0] && !fuse[1] && l.steps == 2 &&
                   chain2_small_applies(ha, ha->steps[f], tokens) && chain2_small_applies(hb, hb->steps[f], tokens)) {
            Chain2Args ca[2];
            for (int n = 0; n < 2; ++n)
                ca[n] = chain2_args(hs[n]->steps[f], hs[n]->steps[f + 1], buffer(n, hs[n]->schedule[li].in),
                                    buffer(n, hs[n]->schedule[li].out), tokens);
            rc = launch_chain2_small(ha->steps[f], ca[0], &ca[1], st);
        } else {
            for (int n = 0; n < 2 && rc == TN_OK; ++n) {
                if (skip[n]) {
                    skip[n] = false;
                    continue;
                }
                if (fuse[n]) {                     // e.g. only this layer qualifies, or only one streams its 4-bit form
                    rc = launch_chain2_split(&fa[n], nullptr, st);
                    skip[n] = true;
                    continue;
                }
                const tn::LaunchIO& ln = hs[n]->schedule[li];
                const DevStep& s = hs[n]->steps[f];
                rc = ln.steps == 2 ? launch_chain2(hs[n], s, hs[n]->steps[f + 1], buffer(n, ln.in), buffer(n, ln.out), tokens, st)
                                   : launch_step(hs[n], ws[n], s, buffer(n, ln.in), buffer(n, ln.out), tokens, st);
            }
        }
        if (rc != TN_OK) return rc;
    }
    return TN_OK;
}

int tn_linear_param_gradients(tn_linear_t h, const void* x, const void* dy, void* const* grads, int64_t tokens,
                              void* stream) {
    if (!h || tokens < 0 || !grads || !h->trainable) return TN_ERR_INVALID_ARG;
    if (tokens == 0) return TN_OK;
    if (!x || !dy || !aligned16(x) || !aligned16(dy)) return TN_ERR_INVALID_ARG;
    hipStream_t st = static_cast<hipStream_t>(stream);
    const size_t n = h->steps.size();
    Workspace w;                                   // the forward workspace serves the split-K partial sums
    w.partial = h->partial;
    w.partial_bytes = h->partial_bytes;
    w.chunk_tokens = h->bwd_chunk;
    char* base = static_cast<char*>(h->bwd_ws);
    const int64_t dbuf = (h->plan.max_intermediate + 127) & ~int64_t(127);
    void* dbufs[2] = {base + h->bwd_chunk * h->bwd_saved_elems * h->elt,
                      base + h->bwd_chunk * (h->bwd_saved_elems + dbuf) * h->elt};
    auto saved = [&](size_t s) -> void* { return base + h->bwd_chunk * h->bwd_saved_off[s] * h->elt; };
    for (int64_t t0 = 0; t0 < tokens; t0 += h->bwd_chunk) {
        const int64_t nt = std::min(h->bwd_chunk, tokens - t0);
        const void* xc = static_cast<const char*>(x) + t0 * h->plan.N * h->elt;
        // forward, one launch per step, every step's input kept
        const void* cur = xc;
        for (size_t s = 0; s + 1 < n; ++s) {
            int rc = launch_step(h, w, h->steps[s], cur, saved(s + 1), nt, st);
            if (rc != TN_OK) return rc;
            cur = saved(s + 1);
        }
        // backward
        const void* dcur = static_cast<const char*>(dy) + t0 * h->plan.M * h->elt;
        int toggle = 0;
        for (size_t s = n; s-- > 0;) {
            const DevStep& fs = h->steps[s];
            const void* in_s = s == 0 ? xc : saved(s);
            void* g = grads[fs.plan.slot];
            if (g) {
                const int64_t elems = h->plan.tensors[size_t(fs.plan.tensor)].n_elems;
                int rc = launch_param_gradient(h, fs, dcur, in_s, static_cast<float*>(g), elems, nt, t0 > 0, st);
                if (rc != TN_OK) return rc;
            }
            if (s > 0) {
                int rc = launch_step(h, w, h->bwd[s], dcur, dbufs[toggle], nt, st);
                if (rc != TN_OK) return rc;
                dcur = dbufs[toggle];
                toggle ^= 1;
            }
        }
    }
    return TN_OK;
}

int tn_linear_quantized_tensor(tn_linear_t h, int32_t slot, void* codes, void* exponents, void* stream) {
    if (!h || slot < 0 || size_t(slot) >= h->quant_codes.size()) return TN_ERR_INVALID_ARG;
    hipStream_t st = static_cast<hipStream_t>(stream);
    const int64_t n = h->quant_elems[size_t(slot)];
    if (codes && hipMemcpyAsync(codes, h->quant_codes[size_t(slot)], size_t((n + 1) / 2), hipMemcpyDeviceToDevice, st) != hipSuccess)
        return TN_ERR_HIP;
    if (exponents &&
        hipMemcpyAsync(exponents, h->quant_exps[size_t(slot)], size_t((n + 31) / 32), hipMemcpyDeviceToDevice, st) != hipSuccess)
        return TN_ERR_HIP;
    return TN_OK;
}

int tn_linear_forward_scratch(tn_linear_t h, const void* x, void* y, int64_t tokens, void* stream) {
    if (!h || tokens < 0) return TN_ERR_INVALID_ARG;
    if (tokens == 0) return TN_OK;
    if (!x || !y || !aligned16(x) || !aligned16(y) || h->profiling) return TN_ERR_INVALID_ARG;       // profiling creates events, i.e. allocates
    void* base = (h->device >= 0 && h->device < 64) ? g_scratch_ptr[h->device] : nullptr;
    if (!base) return TN_ERR_UNSUPPORTED;
    Workspace w;
    const bool one_launch = h->small_chain && (h->elt == 4 || tokens <= kSmallChainMaxBf16Tokens);
    if (one_launch) {
        // nothing but x and y is touched
    } else if ((h->pair && tokens >= h->pair_min_tokens) || (h->kron && tokens >= h->kron_min_tokens)) {
        // only partial sums: the launch takes as many splits of the bond as fit
        w.partial = base;
        w.partial_bytes = kScratchBytes;
    } else {
        // the compact steps in one pass: [partial sums | buffer 0 | buffer 1], 256-byte aligned pieces
        int64_t part = 0;
        if (!(h->flags & TN_FLAG_NO_SPLIT_K) && h->elt == 2)
            for (const tn::LaunchIO& l : h->schedule)
                if (l.steps == 1) {
                    const DevStep& s = h->steps[size_t(l.first)];
                    const SplitCfg c = split_config(s, tokens * s.plan.R);
                    if (c.use) part = std::max(part, c.partial_bytes);
                }
        part = (part + 255) & ~int64_t(255);
        int64_t max_r = 1;
        for (const auto& s : h->steps) max_r = std::max(max_r, s.plan.R);
        if (tokens > ((int64_t(1) << 31) - 1024) / max_r) return TN_ERR_SCRATCH;      // rows of a pass are indexed with 32 bits
        const int64_t per_token = h->plan.max_intermediate * h->elt;
        if (per_token > 0 && tokens > kScratchBytes / per_token) return TN_ERR_SCRATCH;
        const int64_t buf = (tokens * per_token + 255) & ~int64_t(255);
        if (part + 2 * buf > kScratchBytes) return TN_ERR_SCRATCH;
        char* b = static_cast<char*>(base);
        w.partial = part > 0 ? b : nullptr;
        w.partial_bytes = part;
        w.ws[0] = b + part;
        w.ws[1] = b + part + buf;
        w.chunk_tokens = tokens;
    }
    return forward_in(h, w, false, x, y, tokens, static_cast<hipStream_t>(stream));
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
        case TN_QUERY_LAZY_MIN_TOKENS: *value = h->lazy ? h->lazy_min_tokens : 0; return TN_OK;
        case TN_QUERY_LAZY_FLOPS_PER_TOKEN: *value = h->lazy ? h->lazy_plan.flops : 0; return TN_OK;
        case TN_QUERY_QUANT_BYTES: *value = h->quant_bytes; return TN_OK;
        case TN_QUERY_QUANT_STREAM_BYTES: *value = h->q4_stream_bytes; return TN_OK;
        case TN_QUERY_BACKWARD_CHUNK_TOKENS: *value = h->trainable ? h->bwd_chunk : 0; return TN_OK;
        case TN_QUERY_BACKWARD_WORKSPACE_BYTES: *value = h->trainable ? h->bwd_ws_bytes + h->bwd_partial_bytes : 0; return TN_OK;
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
        *value = h->steps[size_t(s)].fuse_next ? 1 : ((h->pair && s == 0) ? 2 : ((h->kron && s == 0) ? 4 : 0));
        if (h->small_chain && size_t(s) + 1 < h->steps.size()) *value = 3;
        return TN_OK;
    }
    return plan_value(h->plan, what, value);
}

}  // extern "C"
