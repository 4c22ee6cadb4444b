/*
 * tn_linear: forward pass of tensor-network-structured linear layers on one
 * MI355X (gfx950).
 *
 * y = W x with W [M, N] held as dense, tensor-train (TT), tensor-ring (TR) or
 * Tucker factors (the formats of the paper's Stage 2, Section 3.3) and applied
 * to a batch of token activations by sequential contraction of the factors
 * (the kernels of Stage 4, Section 3.5). The paper names the formats without
 * formulas; the standard definitions are used:
 *
 *   TT     W[i, j] = G_1[:, i_1, j_1, :] G_2[:, i_2, j_2, :] ... G_d[:, i_d, j_d, :]   (r_0 = r_d = 1)
 *   TR     W[i, j] = trace of the same matrix product                                  (r_0 = r_d = r)
 *   Tucker W[(i_1..i_p), (j_1..j_q)] = sum_{a, c} C[a_1..a_p, c_1..c_q]
 *                                      prod_a U_a[i_a, a_a]  prod_b V_b[j_b, c_b]
 *   dense  W given directly
 *
 * M = prod m_k, N = prod n_k. Flat index <-> mode digits is C order, first
 * mode most significant: i = ((i_1 m_2 + i_2) m_3 + i_3)... All tensors are
 * contiguous row-major. X is [tokens, N], Y is [tokens, M],
 * Y[t, i] = sum_j W[i, j] X[t, j]; no bias.
 *
 * Every pointer named "device" is GPU memory of the current HIP device; every
 * other pointer is host memory. No function throws; all return an int status
 * (TN_OK = 0, errors negative). The library keeps no global state besides the
 * handles it returns.
 */
#ifndef TN_LINEAR_H
#define TN_LINEAR_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* status codes */
#define TN_OK                 0
#define TN_ERR_INVALID_ARG   (-1)   /* NULL pointer, bad extent, inconsistent ranks ... */
#define TN_ERR_UNSUPPORTED   (-2)   /* valid request this build cannot run (e.g. too many modes) */
#define TN_ERR_ALLOC         (-3)   /* host or device allocation failed */
#define TN_ERR_HIP           (-4)   /* a HIP runtime call or kernel launch failed */
#define TN_ERR_SCRATCH       (-5)   /* tn_linear_forward_scratch: the call needs more scratch memory than the
                                       library's static buffer holds (use tn_linear_forward) */

/* desc.format */
#define TN_FORMAT_DENSE   0
#define TN_FORMAT_TT      1
#define TN_FORMAT_TR      2
#define TN_FORMAT_TUCKER  3

/* desc.dtype: storage type of tensors, X and Y. Accumulation is always fp32. */
#define TN_DTYPE_F32   0    /* fp32 storage, fp32 FMA arithmetic, fp32 intermediates */
#define TN_DTYPE_BF16  1    /* bf16 storage, bf16 MFMA with fp32 accumulate, bf16 intermediates */

/*
 * desc.flags, part 1: what the layer is and how much memory it may trade for speed. These are the interface.
 */
#define TN_FLAG_NO_MERGE        2   /* keep every parameter tensor separate: do not contract adjacent
                                       tensors into one at create time even where that is free */
#define TN_FLAG_MERGE_GROW     16   /* trade memory for speed: also contract parameter tensors at create time
                                       when that ADDS parameters, as long as the layer stays under a quarter
                                       of the dense matrix (e.g. a ring of 4 cores becomes two half-rings) */
#define TN_FLAG_MERGE_HALVES  (1 << 22)  /* like TN_FLAG_MERGE_GROW, but whatever the size (up to 1e9 elements): contract
                                       parameter tensors at create time until two are left (a ring of four cores
                                       becomes two half rings), and keep them. This is the plan large calls of a
                                       default layer run on with the merged tensors rebuilt per call
                                       (TN_QUERY_LAZY_MIN_TOKENS); with this flag every call runs on it. */
#define TN_FLAG_TRANSPOSE      128   /* apply W^T instead of W: X is [tokens, M], Y is [tokens, N],
                                       Y[t, j] = sum_i W[i, j] X[t, i]. Same tensors, same description; this is
                                       the gradient of the forward pass with respect to its input, which the
                                       fine-tuning of the factors (Section 3.4) back-propagates through every
                                       layer. TN_QUERY_IN_FEATURES / OUT_FEATURES then report M / N. */
#define TN_FLAG_TRAINABLE (1 << 25)      /* the layer can also give the gradients of a loss with respect to its tensors
                                       (tn_linear_param_gradients, Section 3.4): every parameter tensor of the caller
                                       stays separate (as with TN_FLAG_NO_MERGE; no lazily merged plan either) and the
                                       handle holds a second workspace for the saved intermediates of a backward pass */
#define TN_FLAG_QUANT_MXFP4 (1 << 26)    /* 4-bit tensors (Section 6: 4-bit quantisation of the cores; the paper gives no scheme,
                                       the one taken is the OCP microscaling format MXFP4, weight-only): at create every
                                       tensor of the caller is quantised in blocks of 32 consecutive elements of its
                                       row-major flattening (last block shorter): shared scale 2^(floor(log2 max|v|) - 2)
                                       (E8M0 exponent, clamped to -127..127, -127 for a zero block), element = v / scale
                                       rounded to the nearest of 0, 0.5, 1, 1.5, 2, 3, 4, 6 (ties to an even mantissa bit,
                                       saturating) with a sign. The layer then applies the DEQUANTISED tensors (exact in
                                       bf16) and keeps codes and exponents (tn_linear_quantized_tensor,
                                       TN_QUERY_QUANT_BYTES). Calls of up to 64 rows read a tensor in its 4-bit form
                                       (0.53 bytes per parameter, converted in registers: same values, a quarter of the
                                       memory traffic) where the contraction walks the caller's tensor in memory order
                                       and K is a multiple of 32 - a dense matrix, the core of a Tucker layer
                                       (TN_QUERY_QUANT_STREAM_BYTES); larger calls and all other tensors use the bf16
                                       copies. bf16 layers only; not with TN_FLAG_TRAINABLE. */

/*
 * desc.flags, part 2: switches that take a kernel path away, and tuning overrides. They exist for the library's own
 * tests and measurements (every fused or specialised path is compared with the plain one it replaces); results
 * stay within tolerance under any of them, only speed changes. Not meant for applications; bit 3 is unused.
 */
#define TN_FLAG_SCALAR_KERNELS  1   /* run every contraction step on the plain FMA kernel */
#define TN_FLAG_NO_SPLIT_K      4   /* never use the split-K kernel for small launches */
#define TN_FLAG_NO_PAIR_CHAIN   32   /* never run a two-step plan as one chained launch (see TN_QUERY_PAIR_CHAINABLE):
                                       always two launches with the intermediate in the workspace */
#define TN_FLAG_NO_CHAIN2       64   /* never run two small transposing steps (Tucker factor products) as one
                                       chained launch: always one launch per step */
#define TN_FLAG_NO_SMALL_CHAIN (1 << 20) /* never run a small layer as one launch with all its tensors in LDS */
#define TN_FLAG_NO_LAZY_MERGE (1 << 21)  /* never run large calls on a merged plan rebuilt in the workspace (see
                                       TN_QUERY_LAZY_MIN_TOKENS): every call runs the compact steps */
#define TN_FLAG_SCALAR_GENERATE (1 << 23) /* rebuild the slices of a lazily merged plan with the plain FMA kernel
                                       instead of the MFMA one */
#define TN_FLAG_NO_DECODE_FUSION (1 << 24) /* none of the forms kept for calls of a few tokens: a chained factor pair and the
                                       wide step after it as one launch (the in-factor products and the core of a Tucker
                                       layer), chained pairs on the kernels that request their operands up front, the
                                       Kronecker-sum kernel with the four waves of a workgroup sharing one token */
#define TN_FLAG_NO_Q4_STREAM (1 << 27)   /* a TN_FLAG_QUANT_MXFP4 layer never reads the 4-bit form in its kernels: every call
                                       multiplies with the bf16 copies of the dequantised tensors */
#define TN_FLAG_NO_SKINNY (1 << 28)      /* never run a launch of 5 to 64 rows on the kernel that keeps the rows in LDS and
                                       gives a workgroup 256 columns: such launches use the split-K kernel of one column block */
#define TN_FLAG_VARIANT_SHIFT   8   /* bits 8..15: kernel variant id for the wide bf16 steps (0 = library's choice):
                                       3 = 128x256 and 8 = 256x128 register-prefetch tiles, 9 = short-K store kernel,
                                       12 = 256x256 ping-pong kernel; 20 = the Kronecker-sum kernel for every two-step
                                       plan whose layout allows it, whatever its size (see TN_QUERY_KRON_CHAINABLE);
                                       ignored where the variant cannot run the step */
#define TN_FLAG_SHORTK_SHIFT   16   /* bits 16..19: form of the short-K kernel (0 = library's choice) */

/* tn_linear_query / tn_linear_plan_query: what */
#define TN_QUERY_PARAM_COUNT        0   /* number of parameters in the caller's tensors */
#define TN_QUERY_PACKED_BYTES       1   /* bytes of the library's packed copy (padding included) */
#define TN_QUERY_FLOPS_PER_TOKEN    2   /* 2 * multiply-adds of the chosen contraction order, per token */
#define TN_QUERY_WORKSPACE_BYTES    3   /* device workspace held by the handle (0 from plan_query) */
#define TN_QUERY_NUM_STEPS          4   /* contraction steps = kernel launches per token chunk */
#define TN_QUERY_CHUNK_TOKENS       5   /* tokens processed per pass over the chain (0 from plan_query) */
#define TN_QUERY_MAX_INTERMEDIATE   6   /* largest per-token intermediate, in elements */
#define TN_QUERY_OUT_FEATURES       7   /* M */
#define TN_QUERY_IN_FEATURES        8   /* N */
#define TN_QUERY_NUM_MERGES         9   /* parameter-tensor pairs contracted into one at create time */
#define TN_QUERY_PAIR_CHAINABLE    10   /* 1 if the plan is a short-K step feeding a long-K step over a bond of 64
                                           (a train whose end cores were merged into their neighbours): from
                                           256 tokens on, forward runs both steps as one launch that keeps the
                                           intermediate in registers */
#define TN_QUERY_KRON_CHAINABLE   11   /* 0, or 1 + instantiation when the plan is two steps over a shared bond
                                           that the Kronecker-sum kernel runs as one launch with the
                                           intermediate in registers (e.g. a ring contracted into two half
                                           rings under TN_FLAG_MERGE_GROW) */
#define TN_QUERY_LAZY_MIN_TOKENS   12   /* handle only: 0, or the token count from which a call runs on a lazily
                                           merged plan: the plan TN_FLAG_MERGE_HALVES would give (two half rings for
                                           a ring of four cores) is cheaper and fits the Kronecker-sum kernel, so
                                           such calls run that one launch on its tensors, rebuilt in the workspace
                                           from the caller's compact ones (microseconds): per call when the
                                           workspace is a caller's block shared with other layers, once at create
                                           when it is the handle's own; 1 since the kernel has a one-token form */
#define TN_QUERY_LAZY_FLOPS_PER_TOKEN 13 /* handle only: FLOPs per token of that plan (0 if none) */
#define TN_QUERY_BACKWARD_CHUNK_TOKENS 14 /* handle only: tokens per pass of tn_linear_param_gradients (0: not trainable) */
#define TN_QUERY_BACKWARD_WORKSPACE_BYTES 15 /* handle only: device memory held for those passes */
#define TN_QUERY_QUANT_BYTES       16   /* handle only: bytes of the 4-bit codes and block exponents of all tensors (0: not quantised) */
#define TN_QUERY_QUANT_STREAM_BYTES 17  /* handle only: bytes of the 4-bit streams that decode-size calls read instead of the
                                           bf16 tensors (0: no step of the layer qualifies, or not quantised) */
#define TN_QUERY_STEP_BASE        100   /* 100 + 10*s + f: field f of step s:
                                           f=0 rows per token, 1 K, 2 columns, 3 FLOPs per token,
                                           4 id of the absorbed tensor (index into desc.tensors; ids >=
                                             n_tensors name tensors merged at create time),
                                           5 kernel variant chosen (0 plain FMA, 2 narrow 256x32 tile, else
                                             the ids listed at TN_FLAG_VARIANT_SHIFT),
                                           6 1 if this step and the next run as one fused launch, 2 if they
                                             do so from 256 tokens on (chained pair kernel), 3 if the whole chain
                                             runs as one launch with its tensors in LDS (small layers: fp32 at any
                                             token count, bf16 up to 32 tokens), 4 if both steps run as one launch
                                             of the Kronecker-sum kernel at every token count,
                                           7 shape test only (also from plan_query): 0, or 1 + the instantiation
                                             of the transposing chain kernel that could run this step with the
                                             next one (consecutive qualifying pairs overlap: create takes them
                                             left to right) */

typedef struct tn_linear_s* tn_linear_t;

/*
 * Layer description.
 *
 *  format, dtype      see above.
 *  out_modes[n_out_modes], in_modes[n_in_modes]
 *                     m_1..m_p and n_1..n_q, all >= 1. TT/TR need p == q = d.
 *                     dense: any factorisation is accepted, only M and N matter.
 *  ranks[n_ranks]     TT/TR: d+1 bond sizes r_0..r_d (TT: r_0 = r_d = 1; TR: r_0 = r_d);
 *                     Tucker: p+q ranks R_1..R_p, S_1..S_q; dense: ignored (n_ranks may be 0).
 *  tensors[n_tensors] DEVICE pointers to contiguous row-major arrays of `dtype`:
 *                     dense : 1 tensor  W[M, N]
 *                     TT/TR : d cores   G_k[r_{k-1}, m_k, n_k, r_k]
 *                     Tucker: core C[R_1..R_p, S_1..S_q], then U_1..U_p as [m_a, R_a],
 *                             then V_1..V_q as [n_b, S_b]
 *                     The array of pointers itself is host memory.
 *  max_tokens         largest token count a single pass will be sized for (>= 1); larger
 *                     forward calls are processed in several passes.
 *  workspace_limit_bytes
 *                     upper bound for the handle's device workspace; 0 = library default
 *                     (4 GiB): the handle allocates what max_tokens needs, up to this bound; with less,
 *                     a call is processed in passes of as many tokens as fit.
 *  flags              TN_FLAG_* bits.
 *  stream             hipStream_t on which create enqueues its repacking work.
 *  workspace, workspace_bytes
 *                     optional DEVICE block owned by the caller (NULL = the library allocates its
 *                     own, bounded by workspace_limit_bytes). The handle then keeps its intermediates,
 *                     split-K partial sums and the per-call tensors of a lazily merged plan
 *                     (TN_QUERY_LAZY_MIN_TOKENS; switched off if they do not fit) inside this block and
 *                     allocates no workspace; the block
 *                     must outlive the handle and be 256-byte aligned. Several handles may share one
 *                     block as long as their forwards never overlap in time (e.g. all layers of a model
 *                     run on one stream). Too small for one token's intermediates: TN_ERR_INVALID_ARG.
 */
typedef struct tn_linear_desc {
    int32_t format;
    int32_t dtype;
    int32_t n_out_modes;
    const int32_t* out_modes;
    int32_t n_in_modes;
    const int32_t* in_modes;
    int32_t n_ranks;
    const int32_t* ranks;
    int32_t n_tensors;
    const void* const* tensors;
    int64_t max_tokens;
    int64_t workspace_limit_bytes;
    int32_t flags;
    void* stream;
    void* workspace;
    int64_t workspace_bytes;
} tn_linear_desc;

/*
 * Build a layer (Section 3.5: contiguous, kernel-friendly parameter storage).
 * Validates the description, chooses the contraction order with the fewest
 * FLOPs, copies the caller's tensors into library-owned packed device buffers
 * (one per contraction step, K-contiguous, zero-padded to the MFMA tile) by
 * kernels enqueued on desc->stream, and allocates the workspace. The caller
 * keeps ownership of its tensors and may free them once desc->stream has
 * drained. On success *out receives the handle; on failure *out is untouched.
 * May wait for desc->stream while uploading its tables; allocates device memory
 * (not capturable).
 */
int tn_linear_create(tn_linear_t* out, const tn_linear_desc* desc);

/*
 * Y = X W^T for `tokens` rows (Section 3.5, the TN matmul).
 *  x  DEVICE [tokens, N] of the handle's dtype, read only
 *  y  DEVICE [tokens, M] of the handle's dtype, fully overwritten
 *  x and y must not overlap each other and must be 16-byte aligned (device allocations are; TN_ERR_INVALID_ARG
 *  otherwise: rows are read and written in 16-byte pieces). Enqueues kernels on `stream`
 *  (hipStream_t) and returns without synchronising or allocating; with
 *  profiling off it makes no other HIP call than kernel launches, so it may be
 *  recorded into a HIP graph (stream capture) from the handle's first call on.
 *  tokens == 0 is a no-op. One forward per handle may be in flight at a time (the
 *  workspace is shared); different handles are independent. Results are
 *  bit-identical from call to call for the same handle, inputs and token count.
 */
int tn_linear_forward(tn_linear_t h, const void* x, void* y, int64_t tokens, void* stream);

/*
 * Two layers applied to the same activations in one call (Section 3.5: fuse core contractions and factor
 * multiplications where possible), e.g. the gate and up projections of an MLP block:
 *   ya = X Wa^T, yb = X Wb^T for `tokens` rows of x [tokens, N]; both handles must have the same dtype and N.
 * Where the two layers have the same launch structure, calls of a few tokens run each decode-size launch once for
 * both layers (a Tucker pair's in-factor products + cores are one launch, its out-factor products another: two
 * launches for two layers instead of six); every other case runs the two forwards back to back on `stream`, the
 * second of which finds x in the last-level cache. Same conditions as tn_linear_forward (asynchronous, no
 * allocation, capturable); each result agrees with that of tn_linear_forward on its handle (bit for bit where the
 * same kernels run).
 */
int tn_linear_forward2(tn_linear_t ha, tn_linear_t hb, const void* x, void* ya, void* yb, int64_t tokens, void* stream);

/*
 * Gradients with respect to the parameter tensors (Section 3.4: after compression the factors are fine-tuned, so a
 * loss is back-propagated through every factorised layer). For L = sum_{t,i} dY[t,i] Y[t,i] with Y = X W^T:
 *   grads[s]  DEVICE fp32 array of the shape of desc.tensors[s] (canonical layout), overwritten with dL/d tensors[s];
 *             a NULL entry skips that tensor. The array of pointers is host memory, n_tensors entries.
 *   x  DEVICE [tokens, N], dy DEVICE [tokens, M], of the handle's dtype, read only, 16-byte aligned.
 * The call re-runs the contraction steps keeping every intermediate, then walks them backwards: for each step the
 * gradient of its parameter tensor is the step's own contraction with the token and row indices summed (fp32
 * accumulation, partial sums over row ranges added in a fixed order: bit-reproducible), and the gradient handed to
 * the step before is the step with its tensor transposed. Intermediates are rounded to the handle's dtype as in the
 * forward pass. Needs a handle created with TN_FLAG_TRAINABLE (else TN_ERR_INVALID_ARG); tokens beyond the backward
 * workspace are processed in passes whose gradients are added. The gradient with respect to x is what a handle
 * created with TN_FLAG_TRANSPOSE computes. Asynchronous on `stream`, no allocation.
 */
int tn_linear_param_gradients(tn_linear_t h, const void* x, const void* dy, void* const* grads, int64_t tokens,
                              void* stream);

/*
 * The 4-bit form of tensor `slot` of a layer created with TN_FLAG_QUANT_MXFP4, copied on `stream`:
 *   codes      DEVICE, ceil(n / 2) bytes: element 2i in the low nibble of byte i, 2i + 1 in the high one; a nibble is
 *              sign (bit 3) and the index of its magnitude in 0, 0.5, 1, 1.5, 2, 3, 4, 6 (bits 0..2)
 *   exponents  DEVICE, ceil(n / 32) signed bytes: block b scales elements 32b .. 32b + 31 by 2^exponents[b]
 * n is the element count of desc.tensors[slot]. Either pointer may be NULL.
 */
int tn_linear_quantized_tensor(tn_linear_t h, int32_t slot, void* codes, void* exponents, void* stream);

/*
 * tn_linear_forward for callers that cannot allocate and want no workspace tied to the handle: code under
 * HIP graph capture, tight serving loops, harnesses that forbid hipMalloc. Same arguments, same result bits
 * as tn_linear_forward for calls that take the same kernels; the intermediates between contraction steps and
 * the fp32 partial sums of the split kernels live in a static device array of the library
 * (TN_SCRATCH_BYTES = 32 MiB per GPU, held until the process ends) instead of the handle's workspace, which
 * this call never touches. It calls no allocating routine and no HIP call other than kernel launches.
 *   - The whole call runs as one pass: it needs tokens * 2 * (largest per-token intermediate) bytes plus the
 *     partial sums of its split launches. More than TN_SCRATCH_BYTES: TN_ERR_SCRATCH, nothing is launched.
 *     Calls that run as one launch with no intermediate in memory (small layers, the chained pair kernel)
 *     need none and are never refused; a layer on the Kronecker-sum kernel takes as many splits as fit.
 *   - A lazily merged ring (TN_QUERY_LAZY_MIN_TOKENS) runs its compact steps here: the rebuilt slices belong to
 *     the handle's workspace.
 *   - Every call on one GPU, from any handle, shares that GPU's array: calls that overlap in time on one GPU
 *     race. Nothing in it needs to start at zero (every element is written before it is read within a call).
 *   - A handle with profiling enabled is refused (TN_ERR_INVALID_ARG): profiling creates events.
 */
#define TN_SCRATCH_BYTES (32 << 20)
int tn_linear_forward_scratch(tn_linear_t h, const void* x, void* y, int64_t tokens, void* stream);

/* Free packed tensors and workspace. No forward may be in flight. NULL is accepted. */
int tn_linear_destroy(tn_linear_t h);

/* Read a property of a built layer (TN_QUERY_*). */
int tn_linear_query(tn_linear_t h, int32_t what, int64_t* value);

/*
 * Host-only planning: the same validation and contraction-order search as
 * create, with no GPU call and no tensor access (desc->tensors may be NULL).
 */
int tn_linear_plan_query(const tn_linear_desc* desc, int32_t what, int64_t* value);

/*
 * Per-step timing for measurement (Section 3.5 gives no kernel-level numbers; these are
 * ours). While enabled, every kernel launch of tn_linear_forward on this handle is
 * bracketed by a pair of HIP events on the caller's stream (events are created as needed,
 * so an enabled handle allocates and must not be used under graph capture). Enabling
 * clears earlier records; disabling keeps them readable.
 */
int tn_linear_profile(tn_linear_t h, int32_t enable);

/*
 * Sum of the recorded kernel durations of contraction step `step` in milliseconds and the
 * number of launches recorded. Waits for the recorded events (host-blocking). total_ms and
 * launches are host pointers.
 */
int tn_linear_profile_read(tn_linear_t h, int32_t step, double* total_ms, int64_t* launches);

/* Static, NUL-terminated description of a status code. */
const char* tn_linear_strerror(int status);

/* Library ABI version (incremented when a signature or struct changes). */
int tn_linear_version(void);

#ifdef __cplusplus
}
#endif
#endif /* TN_LINEAR_H */
