// Host-side planner for tensor-network linear layers (no GPU calls).
//
// A layer is a small tensor network: the activation tensor x[n_1..n_q] and a
// set of parameter tensors (TT/TR cores, Tucker core and factors, or one dense
// matrix; formats of Section 3.3). The forward pass absorbs one parameter
// tensor per step into a running intermediate Z (Section 3.5: sequential core
// contractions). Absorbing tensor P contracts every index of P that is live in
// Z and introduces every other index of P, which as a matrix product reads
//     rows = all other live indices of Z   (times tokens)
//     K    = indices shared by Z and P
//     cols = indices of P not in Z
// The planner picks the absorption order with the fewest multiply-adds by a
// dynamic programme over subsets of absorbed tensors, then assigns a memory
// layout to every intermediate such that each step reads a plain row-major
// [rows, K] matrix, and the index permutation between steps happens in the
// store of the previous step through two small offset tables.
#pragma once

#include <algorithm>
#include <cstdint>
#include <limits>
#include <string>
#include <vector>

#include "../../include/tn_linear.h"

namespace tn {

constexpr int kMaxTensors = 16;
constexpr int kMaxGatherDims = 8;

struct GatherDim {
    int64_t extent;
    int64_t stride;   // in elements of the caller's tensor
};

struct NetTensor {
    int slot;                       // index into desc.tensors
    std::vector<int> idx;           // index ids, outer -> inner, canonical layout (trace pair removed)
    std::vector<int64_t> stride;    // element stride of each idx entry
    int64_t trace_extent = 1;       // >1: sum over a repeated index (single-core ring)
    int64_t trace_stride = 0;
    int64_t n_elems = 0;
};

struct Step {
    int tensor = -1;                // network tensor absorbed
    int slot = -1;                  // desc.tensors slot of that tensor
    int64_t R = 1, K = 1, C = 1;    // rows per token, contraction length, columns
    std::vector<GatherDim> kdims, cdims;   // decomposition of k and c into source strides
    int64_t trace_extent = 1, trace_stride = 0;
    bool a_plain = true;            // A is row-major [tokens*R, K] with leading dimension K
    std::vector<int32_t> arow, acol;       // gather tables when !a_plain
    std::vector<int64_t> rext;             // extents of the indices the row number runs over, outer -> inner
    int64_t a_tok_stride = 0;       // elements per token of the step's input
    std::vector<int32_t> crow, ccol;       // scatter tables of the output
    int64_t c_tok_stride = 0;       // elements per token of the step's output
    int c_vec = 1;                  // columns come in aligned contiguous runs of this many (1, 4 or 8)
    int r_vec = 1;                  // rows come in aligned contiguous runs of this many (1 or 8)
    int a_vec = 1;                  // !a_plain: 8 when the k of one row come in aligned contiguous runs of 8 (acol in runs,
                                    // arow and a_tok_stride multiples of 8), i.e. a row is gathered in 16-byte pieces
    int64_t flops = 0;              // 2*R*K*C
};

// Create-time contraction of two parameter tensors into one (a "virtual" tensor):
//   out[p_free..., q_free...] = sum_shared P[...] * Q[...]
// taken when the result is no larger than the two tensors together, e.g. a TT boundary core whose
// bond already has the full rank m*n of that core carries no compression and is absorbed into its
// neighbour (Section 3.5: "fuse core contractions ... where possible").
struct MergeOp {
    int p_slot = -1, q_slot = -1;           // sources: caller slots, or n_caller + index of an earlier merge
    std::vector<GatherDim> rdims;           // free indices of P: extent, stride in P
    std::vector<GatherDim> kp, kq;          // shared indices: extent and stride in P / in Q
    std::vector<GatherDim> cdims;           // free indices of Q: extent, stride in Q
    int64_t R = 1, K = 1, C = 1;            // out is row-major [R, C]
};

struct Plan {
    int format = 0, dtype = 0;
    int flags = 0;                  // the description's flags
    int n_caller_tensors = 0;
    std::vector<MergeOp> merges;
    int64_t M = 1, N = 1;
    int64_t params = 0;
    int64_t flops = 0;
    int64_t max_intermediate = 0;   // elements per token, over all step inputs and outputs except x and y
    std::vector<int64_t> extent;    // per index id
    std::vector<NetTensor> tensors;
    std::vector<int> x_idx, y_idx;  // index ids of x and y, outer -> inner
    std::vector<Step> steps;
};

namespace detail {

inline bool mul_overflow(int64_t a, int64_t b, int64_t* out) {
    return __builtin_mul_overflow(a, b, out);
}

inline int64_t prod_extents(const std::vector<int>& ids, const std::vector<int64_t>& ext) {
    int64_t p = 1;
    for (int i : ids) p *= ext[i];
    return p;
}

inline bool contains(const std::vector<int>& v, int x) {
    return std::find(v.begin(), v.end(), x) != v.end();
}

}  // namespace detail

// Validate the description and build the index network of y = W x. Returns TN_OK or an error.
inline int build_network_forward(const tn_linear_desc* d, Plan* p) {
    using detail::mul_overflow;
    if (!d) return TN_ERR_INVALID_ARG;
    if (d->format < TN_FORMAT_DENSE || d->format > TN_FORMAT_TUCKER) return TN_ERR_INVALID_ARG;
    if (d->dtype != TN_DTYPE_F32 && d->dtype != TN_DTYPE_BF16) return TN_ERR_INVALID_ARG;
    if (d->n_out_modes < 1 || d->n_in_modes < 1 || !d->out_modes || !d->in_modes) return TN_ERR_INVALID_ARG;
    if (d->n_out_modes > kMaxTensors || d->n_in_modes > kMaxTensors) return TN_ERR_UNSUPPORTED;
    if (d->max_tokens < 1) return TN_ERR_INVALID_ARG;
    if (d->workspace_limit_bytes < 0) return TN_ERR_INVALID_ARG;
    if (d->workspace && d->workspace_bytes < 512) return TN_ERR_INVALID_ARG;
    p->format = d->format;
    p->dtype = d->dtype;
    int64_t M = 1, N = 1;
    for (int i = 0; i < d->n_out_modes; ++i) {
        if (d->out_modes[i] < 1) return TN_ERR_INVALID_ARG;
        if (mul_overflow(M, d->out_modes[i], &M)) return TN_ERR_INVALID_ARG;
    }
    for (int i = 0; i < d->n_in_modes; ++i) {
        if (d->in_modes[i] < 1) return TN_ERR_INVALID_ARG;
        if (mul_overflow(N, d->in_modes[i], &N)) return TN_ERR_INVALID_ARG;
    }
    // int32 offset tables address positions inside one token's tensors.
    if (M > (int64_t(1) << 30) || N > (int64_t(1) << 30)) return TN_ERR_UNSUPPORTED;
    p->M = M;
    p->N = N;
    auto new_index = [&](int64_t e) {
        p->extent.push_back(e);
        return int(p->extent.size()) - 1;
    };
    auto add_tensor = [&](int slot, const std::vector<int>& idx) -> int {
        NetTensor t;
        t.slot = slot;
        int n = int(idx.size());
        std::vector<int64_t> st(n, 1);
        int64_t total = 1;
        for (int i = n - 1; i >= 0; --i) {
            st[i] = total;
            if (mul_overflow(total, p->extent[idx[i]], &total)) return TN_ERR_INVALID_ARG;
        }
        if (total > (int64_t(1) << 40)) return TN_ERR_UNSUPPORTED;
        t.n_elems = total;
        // a repeated index inside one tensor (ring of one core) becomes a partial trace
        std::vector<bool> drop(n, false);
        for (int i = 0; i < n; ++i)
            for (int j = i + 1; j < n; ++j)
                if (idx[i] == idx[j] && !drop[i] && !drop[j]) {
                    if (t.trace_extent != 1) return TN_ERR_UNSUPPORTED;
                    t.trace_extent = p->extent[idx[i]];
                    t.trace_stride = st[i] + st[j];
                    drop[i] = drop[j] = true;
                }
        for (int i = 0; i < n; ++i)
            if (!drop[i]) {
                t.idx.push_back(idx[i]);
                t.stride.push_back(st[i]);
            }
        p->params += total;
        p->tensors.push_back(t);
        p->n_caller_tensors = int(p->tensors.size());
        return TN_OK;
    };

    if (d->format == TN_FORMAT_DENSE) {
        // one index per side: only M and N matter for a dense matrix
        int mi = new_index(M), ni = new_index(N);
        p->y_idx = {mi};
        p->x_idx = {ni};
        if (d->tensors && d->n_tensors != 1) return TN_ERR_INVALID_ARG;
        return add_tensor(0, {mi, ni});
    }
    if (d->format == TN_FORMAT_TT || d->format == TN_FORMAT_TR) {
        int dd = d->n_out_modes;
        if (d->n_in_modes != dd) return TN_ERR_INVALID_ARG;
        if (d->n_ranks != dd + 1 || !d->ranks) return TN_ERR_INVALID_ARG;
        for (int i = 0; i <= dd; ++i)
            if (d->ranks[i] < 1) return TN_ERR_INVALID_ARG;
        if (d->format == TN_FORMAT_TT && (d->ranks[0] != 1 || d->ranks[dd] != 1)) return TN_ERR_INVALID_ARG;
        if (d->format == TN_FORMAT_TR && d->ranks[0] != d->ranks[dd]) return TN_ERR_INVALID_ARG;
        if (d->tensors && d->n_tensors != dd) return TN_ERR_INVALID_ARG;
        std::vector<int> mi(dd), ni(dd), bi(dd + 1);
        for (int k = 0; k < dd; ++k) mi[k] = new_index(d->out_modes[k]);
        for (int k = 0; k < dd; ++k) ni[k] = new_index(d->in_modes[k]);
        for (int k = 0; k <= dd; ++k) bi[k] = new_index(d->ranks[k]);
        if (d->format == TN_FORMAT_TR) bi[dd] = bi[0];   // the ring bond is one index with two owners
        p->y_idx = mi;
        p->x_idx = ni;
        for (int k = 0; k < dd; ++k) {
            // the two boundary bonds of a train have extent 1 and no second owner: leave them
            // out (strides are unchanged by an extent-1 axis)
            std::vector<int> idx;
            if (!(d->format == TN_FORMAT_TT && k == 0)) idx.push_back(bi[k]);
            idx.push_back(mi[k]);
            idx.push_back(ni[k]);
            if (!(d->format == TN_FORMAT_TT && k == dd - 1)) idx.push_back(bi[k + 1]);
            int rc = add_tensor(k, idx);
            if (rc != TN_OK) return rc;
        }
        return TN_OK;
    }
    // Tucker
    int pp = d->n_out_modes, qq = d->n_in_modes;
    if (pp + qq + 1 > kMaxTensors) return TN_ERR_UNSUPPORTED;
    if (d->n_ranks != pp + qq || !d->ranks) return TN_ERR_INVALID_ARG;
    for (int i = 0; i < pp + qq; ++i)
        if (d->ranks[i] < 1) return TN_ERR_INVALID_ARG;
    if (d->tensors && d->n_tensors != pp + qq + 1) return TN_ERR_INVALID_ARG;
    std::vector<int> mi(pp), ni(qq), ri(pp), si(qq);
    for (int a = 0; a < pp; ++a) mi[a] = new_index(d->out_modes[a]);
    for (int b = 0; b < qq; ++b) ni[b] = new_index(d->in_modes[b]);
    for (int a = 0; a < pp; ++a) ri[a] = new_index(d->ranks[a]);
    for (int b = 0; b < qq; ++b) si[b] = new_index(d->ranks[pp + b]);
    p->y_idx = mi;
    p->x_idx = ni;
    std::vector<int> core_idx = ri;
    core_idx.insert(core_idx.end(), si.begin(), si.end());
    int rc = add_tensor(0, core_idx);
    if (rc != TN_OK) return rc;
    for (int a = 0; a < pp; ++a) {
        rc = add_tensor(1 + a, {mi[a], ri[a]});
        if (rc != TN_OK) return rc;
    }
    for (int b = 0; b < qq; ++b) {
        rc = add_tensor(1 + pp + b, {ni[b], si[b]});
        if (rc != TN_OK) return rc;
    }
    return TN_OK;
}

// Element count of the caller's tensor `slot` (canonical layouts of tn_linear_desc); 0 for a slot that does not exist.
inline int64_t caller_tensor_elems(const tn_linear_desc* d, int slot) {
    int64_t M = 1, N = 1;
    for (int i = 0; i < d->n_out_modes; ++i) M *= d->out_modes[i];
    for (int i = 0; i < d->n_in_modes; ++i) N *= d->in_modes[i];
    if (slot < 0) return 0;
    if (d->format == TN_FORMAT_DENSE) return slot == 0 ? M * N : 0;
    if (d->format == TN_FORMAT_TT || d->format == TN_FORMAT_TR) {
        if (slot >= d->n_out_modes) return 0;
        return int64_t(d->ranks[slot]) * d->out_modes[slot] * d->in_modes[slot] * d->ranks[slot + 1];
    }
    const int p = d->n_out_modes, q = d->n_in_modes;
    if (slot == 0) {
        int64_t n = 1;
        for (int i = 0; i < p + q; ++i) n *= d->ranks[i];
        return n;
    }
    if (slot <= p) return int64_t(d->out_modes[slot - 1]) * d->ranks[slot - 1];
    if (slot <= p + q) return int64_t(d->in_modes[slot - 1 - p]) * d->ranks[slot - 1];
    return 0;
}

// The network of the layer: y = W x, or with TN_FLAG_TRANSPOSE y = W^T x, which is the same network
// with the roles of the out-modes and the in-modes exchanged (the activation then carries the
// out-modes). The second form is the gradient of the first with respect to its input.
inline int build_network(const tn_linear_desc* d, Plan* p) {
    int rc = build_network_forward(d, p);
    if (rc != TN_OK) return rc;
    if (d->flags & TN_FLAG_TRANSPOSE) {
        std::swap(p->x_idx, p->y_idx);
        std::swap(p->M, p->N);
    }
    return TN_OK;
}

// Live indices after absorbing the tensors in `mask`: an index is live when it is
// carried by x or an absorbed tensor, and also by y or a tensor not yet absorbed.
inline std::vector<int> live_after(const Plan& p, uint32_t mask) {
    int ni = int(p.extent.size());
    std::vector<int> in_done(ni, 0), in_todo(ni, 0);
    for (int i : p.x_idx) in_done[i] = 1;
    for (int i : p.y_idx) in_todo[i] = 1;
    for (size_t t = 0; t < p.tensors.size(); ++t)
        for (int i : p.tensors[t].idx) {
            if (mask & (1u << t)) in_done[i] = 1;
            else in_todo[i] = 1;
        }
    std::vector<int> live;
    for (int i = 0; i < ni; ++i)
        if (in_done[i] && in_todo[i]) live.push_back(i);
    return live;
}

// Fewest-FLOP absorption order by dynamic programming over subsets.
inline int choose_order(const Plan& p, std::vector<int>* order) {
    int n = int(p.tensors.size());
    if (n > kMaxTensors) return TN_ERR_UNSUPPORTED;
    uint32_t full = (n == 32) ? 0xffffffffu : ((1u << n) - 1);
    struct Cost {
        double flops = std::numeric_limits<double>::infinity();
        double penalty = 0;      // first step cannot read x as a plain matrix
        double peak = 0;         // largest intermediate
        int prev = -1;
        bool better(const Cost& o) const {
            if (flops != o.flops) return flops < o.flops;
            if (penalty != o.penalty) return penalty < o.penalty;
            return peak < o.peak;
        }
    };
    std::vector<Cost> best(size_t(full) + 1);
    best[0].flops = 0;
    for (uint32_t mask = 0; mask <= full; ++mask) {
        if (best[mask].flops == std::numeric_limits<double>::infinity()) {
            if (mask == full) break;
            continue;
        }
        if (mask == full) break;
        std::vector<int> live = live_after(p, mask);
        double live_sz = 1;
        for (int i : live) live_sz *= double(p.extent[i]);
        for (int t = 0; t < n; ++t) {
            if (mask & (1u << t)) continue;
            const NetTensor& T = p.tensors[t];
            double ksz = 1, csz = 1;
            int nk = 0;
            for (int i : T.idx) {
                if (detail::contains(live, i)) { ksz *= double(p.extent[i]); ++nk; }
                else csz *= double(p.extent[i]);
            }
            if (nk == 0) continue;    // an outer product is never a useful step here
            Cost c;
            c.flops = best[mask].flops + 2.0 * live_sz * csz;   // rows*K = live_sz
            double out_sz = live_sz / ksz * csz;
            c.peak = std::max(best[mask].peak, (mask | (1u << t)) == full ? 0.0 : out_sz);
            c.penalty = best[mask].penalty;
            if (mask == 0) {
                // plain first step: the contracted in-modes are the innermost of x
                size_t q = p.x_idx.size();
                bool suffix = true;
                for (int j = 0; j < nk; ++j)
                    if (!detail::contains(T.idx, p.x_idx[q - 1 - j])) suffix = false;
                c.penalty = suffix ? 0 : 1;
            }
            c.prev = t;
            uint32_t nm = mask | (1u << t);
            if (c.better(best[nm])) best[nm] = c;
        }
    }
    if (best[full].prev < 0 && n > 0) return TN_ERR_INVALID_ARG;
    order->clear();
    uint32_t mask = full;
    while (mask) {
        int t = best[mask].prev;
        order->push_back(t);
        mask &= ~(1u << t);
    }
    std::reverse(order->begin(), order->end());
    return TN_OK;
}

// Offsets of every multi-index over `ids` (outer -> inner) inside a layout.
inline std::vector<int32_t> offset_table(const std::vector<int>& ids, const std::vector<int64_t>& ext,
                                         const std::vector<int>& layout) {
    // stride of each layout index
    std::vector<int64_t> lst(layout.size(), 1);
    int64_t s = 1;
    for (int i = int(layout.size()) - 1; i >= 0; --i) {
        lst[i] = s;
        s *= ext[layout[i]];
    }
    std::vector<int64_t> st(ids.size(), 0);
    for (size_t j = 0; j < ids.size(); ++j)
        for (size_t i = 0; i < layout.size(); ++i)
            if (layout[i] == ids[j]) st[j] = lst[i];
    int64_t total = detail::prod_extents(ids, ext);
    std::vector<int32_t> tab(static_cast<size_t>(total), 0);
    std::vector<int64_t> digit(ids.size(), 0);
    int64_t off = 0;
    for (int64_t f = 0; f < total; ++f) {
        tab[size_t(f)] = int32_t(off);
        for (int j = int(ids.size()) - 1; j >= 0; --j) {
            off += st[j];
            if (++digit[j] < ext[ids[j]]) break;
            off -= st[j] * ext[ids[j]];
            digit[j] = 0;
        }
    }
    return tab;
}

inline int run_length(const std::vector<int32_t>& tab, int want) {
    // largest v in {want, 4, 1} such that the table is made of aligned runs of v consecutive offsets
    for (int v : {want, 4}) {
        if (v > want) continue;
        if (tab.size() % size_t(v)) continue;
        bool ok = true;
        for (size_t i = 0; i < tab.size() && ok; i += size_t(v)) {
            if (tab[i] % v) ok = false;
            for (int j = 1; j < v && ok; ++j)
                if (tab[i + j] != tab[i] + j) ok = false;
        }
        if (ok) return v;
    }
    return 1;
}

inline bool all_multiple_of(const std::vector<int32_t>& tab, int v) {
    for (int32_t x : tab)
        if (x % v) return false;
    return true;
}

// Build the steps (layouts, tables, packing recipes) for the chosen order.
inline int build_steps(Plan* p, const std::vector<int>& order) {
    using detail::contains;
    const auto& ext = p->extent;
    int n = int(order.size());
    // time at which each index is contracted (n = never, i.e. an output mode)
    std::vector<int> when(ext.size(), n);
    {
        uint32_t mask = 0;
        for (int s = 0; s < n; ++s) {
            std::vector<int> live = live_after(*p, mask);
            for (int i : p->tensors[order[s]].idx)
                if (contains(live, i)) when[i] = s;
            mask |= 1u << order[s];
        }
    }
    std::vector<int> layout = p->x_idx;
    uint32_t mask = 0;
    p->steps.clear();
    p->flops = 0;
    p->max_intermediate = 0;
    for (int s = 0; s < n; ++s) {
        const NetTensor& T = p->tensors[order[s]];
        Step st;
        st.tensor = order[s];
        st.slot = T.slot;
        st.trace_extent = T.trace_extent;
        st.trace_stride = T.trace_stride;
        std::vector<int> kset, rows, cset;
        for (int i : layout) (contains(T.idx, i) ? kset : rows).push_back(i);
        for (int i : T.idx)
            if (!contains(layout, i)) cset.push_back(i);
        if (kset.empty()) return TN_ERR_INVALID_ARG;
        if (s == 0 && n > 1) {
            // x arrives in a fixed layout, but the order in which the first step walks its rows is
            // free: put the indices the next step contracts innermost (and later-contracted ones
            // outermost) so that the rows of one tile store next to each other; A is then gathered
            // through the tables, which is cheap because x is small
            const NetTensor& Tn = p->tensors[order[1]];
            std::vector<int> outer, inner;
            for (int i : rows) (contains(Tn.idx, i) ? inner : outer).push_back(i);
            std::stable_sort(outer.begin(), outer.end(), [&](int a, int b) {
                if (when[a] != when[b]) return when[a] > when[b];
                return a < b;
            });
            rows = outer;
            rows.insert(rows.end(), inner.begin(), inner.end());
        }
        // plain when the layout is exactly [rows..., contracted indices...]
        bool plain = true;
        for (size_t j = 0; j < kset.size(); ++j)
            if (layout[layout.size() - kset.size() + j] != kset[j]) plain = false;
        for (size_t j = 0; j < rows.size() && plain; ++j)
            if (layout[j] != rows[j]) plain = false;
        st.a_plain = plain;
        st.R = detail::prod_extents(rows, ext);
        for (int i : rows) st.rext.push_back(ext[size_t(i)]);
        st.K = detail::prod_extents(kset, ext);
        st.a_tok_stride = detail::prod_extents(layout, ext);
        if (!plain) {
            st.arow = offset_table(rows, ext, layout);
            st.acol = offset_table(kset, ext, layout);
        }
        // next layout
        std::vector<int> next;
        uint32_t nmask = mask | (1u << order[s]);
        bool last = (s == n - 1);
        if (last) {
            next = p->y_idx;
            // everything else must be gone
            std::vector<int> live = rows;
            live.insert(live.end(), cset.begin(), cset.end());
            if (live.size() != next.size()) return TN_ERR_INVALID_ARG;
            for (int i : live)
                if (!contains(next, i)) return TN_ERR_INVALID_ARG;
        } else {
            const NetTensor& Tn = p->tensors[order[s + 1]];
            std::vector<int> live = rows;
            live.insert(live.end(), cset.begin(), cset.end());
            std::vector<int> nk_rows, nk_cols, nrows;
            for (int i : live) {
                if (contains(Tn.idx, i)) (contains(cset, i) ? nk_cols : nk_rows).push_back(i);
                else nrows.push_back(i);
            }
            // rows of the next step: later-contracted indices outermost, output modes first and
            // in output order, so that consecutive rows of a tile land close together when stored
            std::stable_sort(nrows.begin(), nrows.end(), [&](int a, int b) {
                if (when[a] != when[b]) return when[a] > when[b];
                return a < b;
            });
            next = nrows;
            if (p->flags & TN_FLAG_QUANT_MXFP4) {
                // a 4-bit tensor is streamed in blocks of 32 consecutive elements of the caller's flattening: the
                // indices the next tensor contracts run in that tensor's own axis order, so that the k of the next
                // step walks its memory and a block is 32 consecutive k of one column
                std::vector<int> nk = nk_rows;
                nk.insert(nk.end(), nk_cols.begin(), nk_cols.end());
                std::stable_sort(nk.begin(), nk.end(), [&](int a, int b) {
                    auto pa = std::find(Tn.idx.begin(), Tn.idx.end(), a) - Tn.idx.begin();
                    auto pb = std::find(Tn.idx.begin(), Tn.idx.end(), b) - Tn.idx.begin();
                    return pa < pb;
                });
                next.insert(next.end(), nk.begin(), nk.end());
            } else {
                next.insert(next.end(), nk_rows.begin(), nk_rows.end());
                next.insert(next.end(), nk_cols.begin(), nk_cols.end());
            }
        }
        // column order follows the position of the new indices in the next layout
        std::stable_sort(cset.begin(), cset.end(), [&](int a, int b) {
            auto pa = std::find(next.begin(), next.end(), a) - next.begin();
            auto pb = std::find(next.begin(), next.end(), b) - next.begin();
            return pa < pb;
        });
        st.C = detail::prod_extents(cset, ext);
        st.c_tok_stride = detail::prod_extents(next, ext);
        st.crow = offset_table(rows, ext, next);
        st.ccol = offset_table(cset, ext, next);
        st.c_vec = run_length(st.ccol, 8);
        if (st.c_vec > 1 && (!all_multiple_of(st.crow, st.c_vec) || st.c_tok_stride % st.c_vec)) st.c_vec = 1;
        st.r_vec = run_length(st.crow, 8) == 8 ? 8 : 1;
        if (st.r_vec > 1 && (!all_multiple_of(st.ccol, 8) || st.c_tok_stride % 8)) st.r_vec = 1;
        if (!st.a_plain && st.K % 8 == 0 && run_length(st.acol, 8) == 8 && all_multiple_of(st.arow, 8) && st.a_tok_stride % 8 == 0)
            st.a_vec = 8;
        // packing recipe: B[c][k] = tensor[sum of digit*stride]
        auto dims_of = [&](const std::vector<int>& ids, std::vector<GatherDim>* out) {
            for (int i : ids) {
                int64_t stride = 0;
                for (size_t j = 0; j < T.idx.size(); ++j)
                    if (T.idx[j] == i) stride = T.stride[j];
                out->push_back({ext[i], stride});
            }
        };
        dims_of(kset, &st.kdims);
        dims_of(cset, &st.cdims);
        if (int(st.kdims.size()) > kMaxGatherDims || int(st.cdims.size()) > kMaxGatherDims) return TN_ERR_UNSUPPORTED;
        int64_t f;
        if (detail::mul_overflow(st.R, st.K, &f) || detail::mul_overflow(f, st.C, &f) ||
            detail::mul_overflow(f, 2, &f))
            return TN_ERR_UNSUPPORTED;
        st.flops = f;
        p->flops += f;
        if (st.a_tok_stride > (int64_t(1) << 31) - 1 || st.c_tok_stride > (int64_t(1) << 31) - 1)
            return TN_ERR_UNSUPPORTED;
        if (s > 0) p->max_intermediate = std::max(p->max_intermediate, st.a_tok_stride);
        if (!last) p->max_intermediate = std::max(p->max_intermediate, st.c_tok_stride);
        p->steps.push_back(std::move(st));
        layout = next;
        mask = nmask;
    }
    return TN_OK;
}

// Merge pairs of parameter tensors whose contraction is no larger than the pair. Returns the
// number of merges made. Only indices owned by exactly these two tensors are summed.
inline int merge_pass(Plan* p, double budget_elems = 0, int min_tensors = 1) {
    int made = 0;
    for (;;) {
        if (int(p->tensors.size()) <= min_tensors) break;
        int best_a = -1, best_b = -1;
        double best_ratio = 1e300;
        int n = int(p->tensors.size());
        double total_now = 0;
        for (const NetTensor& T : p->tensors) total_now += double(T.n_elems);
        for (int a = 0; a < n; ++a)
            for (int b = 0; b < n; ++b) {
                if (a == b) continue;
                const NetTensor& P = p->tensors[size_t(a)];
                const NetTensor& Q = p->tensors[size_t(b)];
                if (P.trace_extent != 1 || Q.trace_extent != 1) continue;
                std::vector<int> shared;
                for (int i : P.idx)
                    if (detail::contains(Q.idx, i)) shared.push_back(i);
                if (shared.empty()) continue;
                bool ok = true;
                for (int i : shared) {
                    if (detail::contains(p->x_idx, i) || detail::contains(p->y_idx, i)) ok = false;
                    for (int c = 0; c < n && ok; ++c)
                        if (c != a && c != b && detail::contains(p->tensors[size_t(c)].idx, i)) ok = false;
                }
                if (!ok) continue;
                double merged = 1;
                for (int i : P.idx)
                    if (!detail::contains(shared, i)) merged *= double(p->extent[size_t(i)]);
                for (int i : Q.idx)
                    if (!detail::contains(shared, i)) merged *= double(p->extent[size_t(i)]);
                double ratio = merged / double(P.n_elems + Q.n_elems);
                // free merges always; growing ones only inside the caller's parameter budget
                bool ok_size = ratio <= 1.0 ||
                               (budget_elems > 0 && total_now - double(P.n_elems + Q.n_elems) + merged <= budget_elems);
                // a < b keeps P's free indices (the earlier tensor's) outermost in the result
                if (ok_size && a < b && ratio < best_ratio) {
                    best_ratio = ratio;
                    best_a = a;
                    best_b = b;
                }
            }
        if (best_a < 0) break;
        const NetTensor P = p->tensors[size_t(best_a)];
        const NetTensor Q = p->tensors[size_t(best_b)];
        MergeOp m;
        m.p_slot = P.slot;
        m.q_slot = Q.slot;
        NetTensor out;
        out.slot = p->n_caller_tensors + int(p->merges.size());
        for (size_t j = 0; j < P.idx.size(); ++j) {
            int i = P.idx[j];
            if (detail::contains(Q.idx, i)) {
                m.kp.push_back({p->extent[size_t(i)], P.stride[j]});
                int64_t qs = 0;
                for (size_t l = 0; l < Q.idx.size(); ++l)
                    if (Q.idx[l] == i) qs = Q.stride[l];
                m.kq.push_back({p->extent[size_t(i)], qs});
                m.K *= p->extent[size_t(i)];
            } else {
                m.rdims.push_back({p->extent[size_t(i)], P.stride[j]});
                m.R *= p->extent[size_t(i)];
                out.idx.push_back(i);
            }
        }
        for (size_t j = 0; j < Q.idx.size(); ++j) {
            int i = Q.idx[j];
            if (detail::contains(P.idx, i)) continue;
            m.cdims.push_back({p->extent[size_t(i)], Q.stride[j]});
            m.C *= p->extent[size_t(i)];
            out.idx.push_back(i);
        }
        if (int(m.rdims.size()) > kMaxGatherDims || int(m.cdims.size()) > kMaxGatherDims ||
            int(m.kp.size()) > kMaxGatherDims || m.R * m.C > (int64_t(1) << 31) - 1 ||
            P.n_elems > (int64_t(1) << 31) - 1 || Q.n_elems > (int64_t(1) << 31) - 1)
            break;
        out.n_elems = m.R * m.C;
        out.stride.assign(out.idx.size(), 1);
        int64_t s = 1;
        for (int j = int(out.idx.size()) - 1; j >= 0; --j) {
            out.stride[size_t(j)] = s;
            s *= p->extent[size_t(out.idx[size_t(j)])];
        }
        p->merges.push_back(m);
        // replace P by the merged tensor, drop Q
        p->tensors[size_t(best_a)] = out;
        p->tensors.erase(p->tensors.begin() + best_b);
        ++made;
    }
    return made;
}

// Is the plan a short-K step feeding a long-K step over a bond of 64, laid out the way the chained
// pair kernel walks it?  Z[t][j][a][b]: rows a of step 0 (plain x, K0 = 64), columns (j, b) of
// step 0 with b < 64 innermost; step 1 reads rows j with K = (a, b) and has at most 128 columns;
// the output takes 8 consecutive j as one aligned 16-byte piece. Checked on the tables themselves.
inline bool pair_chainable(const Plan& p) {
    if (p.dtype != TN_DTYPE_BF16 || p.steps.size() != 2) return false;
    const Step& s0 = p.steps[0];
    const Step& s1 = p.steps[1];
    const int64_t B = 64;
    if (!s0.a_plain || s0.K != 64 || s0.C % B) return false;
    const int64_t J = s0.C / B, A = s0.R;
    if (J % 8 || A < 1 || A > (int64_t(1) << 20)) return false;
    if (!s1.a_plain || s1.R != J || s1.K != A * B || s1.C > 128) return false;
    if (s0.c_tok_stride != J * A * B || s0.a_tok_stride != A * 64) return false;
    for (int64_t r = 0; r < A; ++r)
        if (s0.crow[size_t(r)] != r * B) return false;
    for (int64_t c = 0; c < s0.C; ++c)
        if (s0.ccol[size_t(c)] != (c / B) * (A * B) + c % B) return false;
    return s1.r_vec == 8;
}

// Is the plan two steps of the form  Z[t][o1][a][rho] = sum_k X_t[k][a] B0[(o1, rho)][k],
// Y[t][o1][o2] = sum_{a, rho} Z[t][o1][a][rho] B1[o2][(a, rho)]  (a sum over the shared bond rho of Kronecker
// products), laid out the way the Kronecker-sum kernel walks it? Rows a of step 0 (K0 a multiple of 8; x plain
// or gathered), columns (o1, rho) with rho innermost; step 1 reads rows
// o1 with K = (a, rho). cfg names the instantiation <AT tiles of a, KS0 k-steps, O2T tiles of o2, O1T tiles of
// o1 per chunk> that holds the shape with the least padding. Unless the flags force the kernel (variant id 20) the shape must also be one
// where it pays: an intermediate of at least 32768 values per token, a bond of at least 8, and at least 35 %
// of the padded MFMA work real.
struct KronDims {
    int64_t A = 0, K0 = 0, O1 = 0, C1 = 0, P = 0;
    int cfg = -1;
    bool x_vec8 = true;
};

constexpr int kKronConfigs = 8;
constexpr int kKronConfig[kKronConfigs][4] = {{5, 10, 3, 2}, {3, 4, 5, 2}, {4, 4, 3, 2}, {2, 5, 5, 2},
                                              {2, 8, 2, 3}, {2, 5, 1, 1}, {3, 4, 4, 2}, {2, 5, 5, 1}};

inline bool kron_shape(const Plan& p, KronDims* d) {
    if (p.dtype != TN_DTYPE_BF16 || p.steps.size() != 2) return false;
    if (p.flags & (TN_FLAG_NO_PAIR_CHAIN | TN_FLAG_SCALAR_KERNELS)) return false;
    const bool any_size = ((p.flags >> TN_FLAG_VARIANT_SHIFT) & 0xff) == 20;      // forced (tests)
    const Step& s0 = p.steps[0];
    const Step& s1 = p.steps[1];
    const int64_t A = s0.R, K0 = s0.K, O1 = s1.R, C1 = s1.C;
    if (!s1.a_plain || A < 1 || s1.K % A || K0 % 8 || p.N % 8 || p.M % 4) return false;
    const int64_t P = s1.K / A;
    if (P < 2 || s0.C != O1 * P || s0.c_tok_stride != O1 * A * P || s1.a_tok_stride != O1 * A * P) return false;
    if (s0.C > (int64_t(1) << 30) || s1.K > (int64_t(1) << 30)) return false;
    for (int64_t r = 0; r < A; ++r)
        if (s0.crow[size_t(r)] != r * P) return false;
    for (int64_t c = 0; c < s0.C; ++c)
        if (s0.ccol[size_t(c)] != (c / P) * (A * P) + c % P) return false;
    bool x_vec8 = true;             // 8 consecutive k of one a are one aligned 16-byte piece of x
    if (!s0.a_plain) {
        for (int64_t r = 0; r < A; ++r)
            if (s0.arow[size_t(r)] % 8) x_vec8 = false;
        for (int64_t k = 0; k < K0; ++k)
            if (s0.acol[size_t(k)] != s0.acol[size_t(k & ~int64_t(7))] + (k & 7) || (!(k & 7) && s0.acol[size_t(k)] % 8))
                x_vec8 = false;
    }
    int cfg = -1;
    int64_t best = 0;
    for (int c = 0; c < kKronConfigs; ++c) {
        const int64_t at = kKronConfig[c][0], ks0 = kKronConfig[c][1], o2t = kKronConfig[c][2], o1t = kKronConfig[c][3];
        if (A > 32 * at || K0 > 16 * ks0 || C1 > 32 * o2t) continue;
        const int64_t n_chunks = (O1 + 32 * o1t - 1) / (32 * o1t);
        const int64_t mfmas = n_chunks * o1t * at * (ks0 + 2 * o2t);
        if (cfg < 0 || mfmas < best) {
            cfg = c;
            best = mfmas;
        }
    }
    if (cfg < 0) return false;
    if (!any_size) {
        const double real = double(A) * double(O1) * double(K0 + C1);
        if (A * O1 * P < 32768 || P < 8 || real < 0.35 * double(best) * 16384.0) return false;
    }
    d->A = A;
    d->K0 = K0;
    d->O1 = O1;
    d->C1 = C1;
    d->P = P;
    d->cfg = cfg;
    d->x_vec8 = x_vec8;
    return true;
}

// Can steps a and b (consecutive) run on the transposing chain kernel? Both plain; b contracts a's row
// index and keeps a's column index as its row index, i.e. a's output is stored transposed ([c1][r]);
// the output takes 8 consecutive c1 (run_c1 = 1) or 8 consecutive c2 (run_c1 = 0) as one aligned piece;
// sizes within one of the two instantiations (cfg 1: R1 <= 64, K1 <= 128, C2 <= 64; cfg 0: R1 <= 96,
// K1 <= 96, C2 <= 160).
inline bool chain2_shape(const Plan& p, const Step& a, const Step& b, int* cfg, int* run_c1) {
    if (p.dtype != TN_DTYPE_BF16) return false;
    if (!a.a_plain || !b.a_plain || a.K % 8) return false;
    if (b.K != a.R || b.R != a.C || a.c_tok_stride != a.C * a.R) return false;
    if (a.R <= 64 && a.K <= 128 && b.C <= 64) *cfg = 1;
    else if (a.R <= 96 && a.K <= 96 && b.C <= 160) *cfg = 0;
    else return false;
    for (int64_t r = 0; r < a.R; ++r)
        if (a.crow[size_t(r)] != r) return false;
    for (int64_t c = 0; c < a.C; ++c)
        if (a.ccol[size_t(c)] != c * a.R) return false;
    if (b.r_vec == 8) *run_c1 = 1;
    else if (b.c_vec == 8) *run_c1 = 0;
    else return false;
    return true;
}

// Which consecutive step pairs run as one launch of the transposing chain kernel: qualifying pairs are
// taken left to right, a step belongs to at most one pair. fuse[i] = 1 + instantiation when steps i and
// i + 1 are one launch, else 0.
inline std::vector<int> chain2_pairs(const Plan& p) {
    std::vector<int> fuse(p.steps.size(), 0);
    if (p.dtype != TN_DTYPE_BF16 || (p.flags & (TN_FLAG_SCALAR_KERNELS | TN_FLAG_NO_CHAIN2))) return fuse;
    for (size_t i = 0; i + 1 < p.steps.size(); ++i) {
        if (i > 0 && fuse[i - 1]) continue;
        int cfg = 0, run_c1 = 0;
        if (chain2_shape(p, p.steps[i], p.steps[i + 1], &cfg, &run_c1)) fuse[i] = 1 + cfg;
    }
    return fuse;
}

// Buffers of the launches of one pass over the chain. A launch covers step `first` (and `first + 1` when
// fused) and reads `in`, writes `out`: kBufX is the caller's x, kBufY the caller's y, 0 and 1 the two
// workspace buffers. The buffer alternates per LAUNCH, not per step, so that a launch never writes the
// buffer it reads, wherever fused pairs sit in the chain.
constexpr int kBufX = -1, kBufY = -2;
struct LaunchIO {
    int first = 0, steps = 1, in = kBufX, out = kBufY;
};

inline std::vector<LaunchIO> launch_schedule(size_t n_steps, const std::vector<int>& fuse) {
    std::vector<LaunchIO> out;
    int in = kBufX, next = 0;
    for (size_t s = 0; s < n_steps;) {
        LaunchIO l;
        l.first = int(s);
        l.steps = (s < fuse.size() && fuse[s] && s + 1 < n_steps) ? 2 : 1;
        l.in = in;
        s += size_t(l.steps);
        l.out = s >= n_steps ? kBufY : next;
        out.push_back(l);
        in = l.out;
        next ^= 1;
    }
    return out;
}

// TN_FLAG_MERGE_HALVES: merges may grow up to kMaxHalvesElems elements in total but stop at two parameter tensors.
constexpr double kMaxHalvesElems = 1.0e9;

inline int make_plan(const tn_linear_desc* d, Plan* p) {
    const double halves_budget = (d->flags & TN_FLAG_MERGE_HALVES) ? kMaxHalvesElems : 0.0;
    int rc = build_network(d, p);
    if (rc != TN_OK) return rc;
    p->flags = d->flags;
    std::vector<int> order;
    rc = choose_order(*p, &order);
    if (rc != TN_OK) return rc;
    rc = build_steps(p, order);
    if (rc != TN_OK) return rc;
    // a trainable layer keeps every parameter tensor of the caller separate: gradients are taken with respect to those
    if (!(d->flags & (TN_FLAG_NO_MERGE | TN_FLAG_TRAINABLE))) {
        Plan q = *p;
        q.steps.clear();
        // TN_FLAG_MERGE_GROW: merges may add parameters up to a quarter of the dense matrix
        double budget = (d->flags & TN_FLAG_MERGE_GROW) ? double(p->M) * double(p->N) / 4.0 : 0.0;
        if (halves_budget > 0) budget = halves_budget;
        if (merge_pass(&q, budget, halves_budget > 0 ? 2 : 1) > 0) {
            std::vector<int> qorder;
            if (choose_order(q, &qorder) == TN_OK && build_steps(&q, qorder) == TN_OK && q.flops < p->flops)
                *p = q;
        }
    }
    return TN_OK;
}

}  // namespace tn
