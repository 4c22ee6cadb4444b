// Test-only host executor of a contraction plan, in double precision.
//
// It walks the planner's steps exactly as the GPU kernels do - pack the
// parameter tensor as B[c][k] from the gather recipe, read A through the plain
// or table addressing, scatter the result through crow/ccol - so that the CPU
// test-suite can check the planner's order, layouts, tables and packing recipes
// against the oracle without a GPU. Never linked into the product library.
#include <cstdint>
#include <vector>

#include "../paper_2602_01613_amd/csrc/tn_plan.hpp"

extern "C" int plan_host_forward(const tn_linear_desc* d, const double* const* tensors, const double* x,
                                 double* y, int64_t tokens) {
    tn::Plan p;
    int rc = tn::make_plan(d, &p);
    if (rc != TN_OK) return rc;
    // tensors merged at create time, in double
    std::vector<std::vector<double>> virt;
    auto source = [&](int slot) -> const double* {
        return slot < p.n_caller_tensors ? tensors[slot] : virt[size_t(slot - p.n_caller_tensors)].data();
    };
    auto offset_of = [](int64_t flat, const std::vector<tn::GatherDim>& dims) {
        int64_t off = 0;
        for (int j = int(dims.size()) - 1; j >= 0; --j) {
            off += (flat % dims[size_t(j)].extent) * dims[size_t(j)].stride;
            flat /= dims[size_t(j)].extent;
        }
        return off;
    };
    for (const tn::MergeOp& m : p.merges) {
        const double* P = source(m.p_slot);
        const double* Q = source(m.q_slot);
        std::vector<double> out(size_t(m.R * m.C), 0.0);
        for (int64_t r = 0; r < m.R; ++r)
            for (int64_t c = 0; c < m.C; ++c) {
                double acc = 0;
                for (int64_t k = 0; k < m.K; ++k)
                    acc += P[offset_of(r, m.rdims) + offset_of(k, m.kp)] * Q[offset_of(c, m.cdims) + offset_of(k, m.kq)];
                out[size_t(r * m.C + c)] = acc;
            }
        virt.push_back(std::move(out));
    }
    std::vector<double> cur(x, x + tokens * p.N), nxt;
    for (size_t s = 0; s < p.steps.size(); ++s) {
        const tn::Step& st = p.steps[s];
        std::vector<double> B(size_t(st.C * st.K), 0.0);
        for (int64_t c = 0; c < st.C; ++c)
            for (int64_t k = 0; k < st.K; ++k) {
                int64_t off = 0, rem = k;
                for (int j = int(st.kdims.size()) - 1; j >= 0; --j) {
                    off += (rem % st.kdims[j].extent) * st.kdims[j].stride;
                    rem /= st.kdims[j].extent;
                }
                rem = c;
                for (int j = int(st.cdims.size()) - 1; j >= 0; --j) {
                    off += (rem % st.cdims[j].extent) * st.cdims[j].stride;
                    rem /= st.cdims[j].extent;
                }
                double v = 0;
                for (int64_t a = 0; a < st.trace_extent; ++a) v += source(st.slot)[off + a * st.trace_stride];
                B[size_t(c * st.K + k)] = v;
            }
        nxt.assign(size_t(tokens * st.c_tok_stride), 0.0);
        // every output position must be written exactly once
        std::vector<char> hit(nxt.size(), 0);
        for (int64_t t = 0; t < tokens; ++t)
            for (int64_t r = 0; r < st.R; ++r)
                for (int64_t c = 0; c < st.C; ++c) {
                    double acc = 0;
                    for (int64_t k = 0; k < st.K; ++k) {
                        int64_t ao = t * st.a_tok_stride + (st.a_plain ? r * st.K + k : int64_t(st.arow[r]) + st.acol[k]);
                        acc += cur[size_t(ao)] * B[size_t(c * st.K + k)];
                    }
                    int64_t oo = t * st.c_tok_stride + st.crow[r] + st.ccol[c];
                    if (oo < 0 || oo >= int64_t(nxt.size()) || hit[size_t(oo)]) return -100 - int(s);
                    hit[size_t(oo)] = 1;
                    nxt[size_t(oo)] = acc;
                }
        for (char h : hit)
            if (!h) return -200 - int(s);
        cur.swap(nxt);
    }
    if (int64_t(cur.size()) != tokens * p.M) return -300;
    for (size_t i = 0; i < cur.size(); ++i) y[i] = cur[i];
    return 0;
}

// vectorisation hints of a step, for the tests: field 0 c_vec, 1 r_vec, 2 a_plain, 3 merges in the plan
extern "C" int plan_host_step_hint(const tn_linear_desc* d, int step, int field, int64_t* value) {
    tn::Plan p;
    int rc = tn::make_plan(d, &p);
    if (rc != TN_OK) return rc;
    if (step < 0 || step >= int(p.steps.size())) return TN_ERR_INVALID_ARG;
    const tn::Step& st = p.steps[size_t(step)];
    *value = field == 0 ? st.c_vec : field == 1 ? st.r_vec : field == 2 ? int64_t(st.a_plain) : int64_t(p.merges.size());
    return 0;
}

// Buffers of the launches of one pass (see tn::launch_schedule) with the chained factor pairs the plan
// allows: in_buf / out_buf receive one entry per launch (-1 = x, -2 = y, 0 / 1 = workspace buffers),
// steps the number of steps each launch covers. Returns the number of launches, or a negative status.
extern "C" int plan_host_launch_buffers(const tn_linear_desc* d, int cap, int* in_buf, int* out_buf, int* steps) {
    tn::Plan p;
    int rc = tn::make_plan(d, &p);
    if (rc != TN_OK) return rc;
    const std::vector<tn::LaunchIO> sched = tn::launch_schedule(p.steps.size(), tn::chain2_pairs(p));
    if (int(sched.size()) > cap) return TN_ERR_INVALID_ARG;
    for (size_t i = 0; i < sched.size(); ++i) {
        in_buf[i] = sched[i].in;
        out_buf[i] = sched[i].out;
        steps[i] = sched[i].steps;
    }
    return int(sched.size());
}
