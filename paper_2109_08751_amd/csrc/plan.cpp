// Schedule builder: per-step (dst, src, slot-list) tables for p virtual ranks.
//
// Sparbit (Section III-B of the paper, Algorithm 1).  The tables are produced
// from the stripe view of the algorithm rather than from its bit mask: after
// the step with distance d every rank r holds the comb of slots
// { (r - k d) mod p : 0 <= k < ceil(p / d) } -- the ranks r is reached from in
// the p rank-shifted binomial trees.  Going from the stride-2d comb to the
// stride-d comb needs the odd multiples (2j + 1) d < p, which the partner
// r - d holds as its own even multiples 2 j d.  Hence, with q = ceil(p / d):
//   blocks sent     n      = floor(q / 2)            (= data - ignore)
//   stripe dropped  ignore = q mod 2                 (the bit of ignore_steps)
//   send slots of r        = (r - 2 j d) mod p,  j < n,  to rank (r + d) mod p
//   they land in the same slot indices of the receiver.
//
// Ring, Recursive Doubling and Bruck follow Section II-A.
#include "plan.hpp"

#include <new>

#include "../../include/sparbit.h"

namespace sparbit {

int ceil_log2(int p)
{
    int l = 0;
    while ((int64_t(1) << l) < int64_t(p)) ++l;
    return l;
}

static inline int32_t wrap(int64_t x, int p)
{
    int64_t m = x % p;
    return int32_t(m < 0 ? m + p : m);
}

static void size_step(Step& st, int p, int distance, int nblocks, int ignore)
{
    st.distance = distance;
    st.nblocks = nblocks;
    st.ignore = ignore;
    st.dst.resize(p);
    st.src.resize(p);
    st.send_slot.resize(size_t(p) * nblocks);
    st.recv_slot.resize(size_t(p) * nblocks);
}

// Phase for a step whose messages stay inside one buffer: the j-th block rank
// r sends lands in the j-th receive slot of dst[r].
static Phase phase_from_step(const Step& st, int p, int step, Buffer buf)
{
    Phase ph;
    ph.step = step;
    ph.src_buf = ph.dst_buf = buf;
    ph.copies.reserve(size_t(p) * st.nblocks);
    for (int r = 0; r < p; ++r) {
        const int to = st.dst[r];
        for (int j = 0; j < st.nblocks; ++j) {
            Copy c;
            c.src_block = uint32_t(r) * uint32_t(p) + uint32_t(st.send_slot[size_t(r) * st.nblocks + j]);
            c.dst_block = uint32_t(to) * uint32_t(p) + uint32_t(st.recv_slot[size_t(to) * st.nblocks + j]);
            ph.copies.push_back(c);
        }
    }
    return ph;
}

static Phase own_block_phase(int p, Buffer dst_buf, bool rotated)
{
    Phase ph;
    ph.step = -1;
    ph.src_buf = BUF_SEND;
    ph.dst_buf = dst_buf;
    ph.skip_in_place = true;
    for (int r = 0; r < p; ++r)
        ph.copies.push_back(Copy{uint32_t(r), uint32_t(r) * uint32_t(p) + uint32_t(rotated ? 0 : r)});
    return ph;
}

static void build_sparbit(int p, Plan& out)
{
    const int L = ceil_log2(p);
    out.phases.push_back(own_block_phase(p, BUF_RECV, false));
    for (int s = 0; s < L; ++s) {
        const int d = 1 << (L - 1 - s);
        const int q = (p + d - 1) / d;  // comb size after this step
        Step st;
        size_step(st, p, d, q / 2, q & 1);
        for (int r = 0; r < p; ++r) {
            st.dst[r] = wrap(int64_t(r) + d, p);
            st.src[r] = wrap(int64_t(r) - d, p);
            for (int j = 0; j < st.nblocks; ++j) {
                st.send_slot[size_t(r) * st.nblocks + j] = wrap(int64_t(r) - int64_t(2 * j) * d, p);
                st.recv_slot[size_t(r) * st.nblocks + j] = wrap(int64_t(r) - int64_t(2 * j + 1) * d, p);
            }
        }
        out.phases.push_back(phase_from_step(st, p, s, BUF_RECV));
        out.steps.push_back(std::move(st));
    }
}

static void build_ring(int p, Plan& out)
{
    out.phases.push_back(own_block_phase(p, BUF_RECV, false));
    for (int s = 0; s < p - 1; ++s) {
        Step st;
        size_step(st, p, 1, 1, 0);
        for (int r = 0; r < p; ++r) {
            st.dst[r] = wrap(r + 1, p);
            st.src[r] = wrap(r - 1, p);
            st.send_slot[r] = wrap(int64_t(r) - s, p);      // own block first, then the last one received
            st.recv_slot[r] = wrap(int64_t(r) - 1 - s, p);
        }
        out.phases.push_back(phase_from_step(st, p, s, BUF_RECV));
        out.steps.push_back(std::move(st));
    }
}

static void build_recursive_doubling(int p, Plan& out)
{
    const int L = ceil_log2(p);
    out.phases.push_back(own_block_phase(p, BUF_RECV, false));
    for (int s = 0; s < L; ++s) {
        const int w = 1 << s;
        Step st;
        size_step(st, p, w, w, 0);
        for (int r = 0; r < p; ++r) {
            const int peer = r ^ w;
            st.dst[r] = st.src[r] = peer;
            for (int j = 0; j < w; ++j) {
                st.send_slot[size_t(r) * w + j] = (r & ~(w - 1)) + j;  // everything received so far
                st.recv_slot[size_t(r) * w + j] = (peer & ~(w - 1)) + j;
            }
        }
        out.phases.push_back(phase_from_step(st, p, s, BUF_RECV));
        out.steps.push_back(std::move(st));
    }
}

static void build_bruck(int p, Plan& out)
{
    const int L = ceil_log2(p);
    out.phases.push_back(own_block_phase(p, BUF_WORK, true));
    int have = 1;  // working slots filled so far
    for (int s = 0; s < L; ++s) {
        const int w = 1 << s;
        const int n = (w < p - w) ? w : p - w;  // last step of a non-power-of-two p is short
        Step st;
        size_step(st, p, w, n, 0);
        for (int r = 0; r < p; ++r) {
            st.dst[r] = wrap(int64_t(r) - w, p);
            st.src[r] = wrap(int64_t(r) + w, p);
            for (int j = 0; j < n; ++j) {
                st.send_slot[size_t(r) * n + j] = j;
                st.recv_slot[size_t(r) * n + j] = have + j;
            }
        }
        have += n;
        out.phases.push_back(phase_from_step(st, p, s, BUF_WORK));
        out.steps.push_back(std::move(st));
    }
    // final memory shift: working slot i of rank r is block (r + i) mod p
    Phase rot;
    rot.step = L;
    rot.src_buf = BUF_WORK;
    rot.dst_buf = BUF_RECV;
    for (int r = 0; r < p; ++r)
        for (int i = 0; i < p; ++i)
            rot.copies.push_back(Copy{uint32_t(r) * uint32_t(p) + uint32_t(i),
                                      uint32_t(r) * uint32_t(p) + uint32_t(wrap(int64_t(r) + i, p))});
    out.phases.push_back(std::move(rot));
}

static void build_direct(int p, Plan& out)
{
    Phase a;  // out of place: every slot straight from the send buffer
    a.step = -1;
    a.src_buf = BUF_SEND;
    a.dst_buf = BUF_RECV;
    a.skip_in_place = true;
    Phase b;  // in place: slot k of rank k is the source
    b.step = -1;
    b.src_buf = BUF_RECV;
    b.dst_buf = BUF_RECV;
    b.only_in_place = true;
    for (int r = 0; r < p; ++r)
        for (int k = 0; k < p; ++k) {
            a.copies.push_back(Copy{uint32_t(k), uint32_t(r) * uint32_t(p) + uint32_t(k)});
            if (r != k)
                b.copies.push_back(Copy{uint32_t(k) * uint32_t(p) + uint32_t(k),
                                        uint32_t(r) * uint32_t(p) + uint32_t(k)});
        }
    out.phases.push_back(std::move(a));
    out.phases.push_back(std::move(b));
}

// Step 0 of every schedule sends each rank's own block.  For a whole
// out-of-place call that block can be read from the send buffer, which makes
// step 0 independent of the own-block placement: both become one batch (one
// launch less).  The state after the fused phase is the state after step 0.
static void add_fused_first_phase(int p, Plan& out)
{
    if (out.steps.empty() || out.phases.size() < 2) return;
    Phase& own = out.phases[0];
    Phase& first = out.phases[1];
    if (own.step != -1 || first.step != 0 || own.src_buf != BUF_SEND || own.dst_buf != first.src_buf) return;
    std::vector<int64_t> owner(size_t(p) * size_t(p), -1);  // block index in the working buffer -> rank whose own block it is
    for (const Copy& c : own.copies) owner[c.dst_block] = c.src_block;
    Phase fused;
    fused.step = 0;
    fused.src_buf = BUF_SEND;
    fused.dst_buf = own.dst_buf;
    fused.skip_in_place = true;
    fused.fused_first = true;
    fused.copies = own.copies;
    for (const Copy& c : first.copies) {
        if (owner[c.src_block] < 0) return;  // step 0 forwards something else: leave the plan unfused
        fused.copies.push_back(Copy{uint32_t(owner[c.src_block]), c.dst_block});
    }
    own.covered_by_fused = true;
    first.covered_by_fused = true;
    out.phases.insert(out.phases.begin(), std::move(fused));  // runs first where it is used
}

int build_plan(int p, int algo, Plan& out)
{
    if (p < 1 || p > SPARBIT_MAX_P) return SPARBIT_ERR_ARG;
    out = Plan();
    out.p = p;
    out.algo = algo;
    switch (algo) {
    case SPARBIT_ALGO_SPARBIT: build_sparbit(p, out); break;
    case SPARBIT_ALGO_RING: build_ring(p, out); break;
    case SPARBIT_ALGO_RECURSIVE_DOUBLING:
        if (p & (p - 1)) return SPARBIT_ERR_UNSUPPORTED;
        build_recursive_doubling(p, out);
        break;
    case SPARBIT_ALGO_BRUCK: build_bruck(p, out); break;
    case SPARBIT_ALGO_DIRECT: build_direct(p, out); break;
    default: return SPARBIT_ERR_ARG;
    }
    if (algo != SPARBIT_ALGO_DIRECT) add_fused_first_phase(p, out);
    return SPARBIT_OK;
}

}  // namespace sparbit

extern "C" {

int sparbit_plan_create(int p, int algo, sparbit_plan_t** out)
{
    if (!out) return SPARBIT_ERR_ARG;
    *out = nullptr;
    sparbit_plan* h = new (std::nothrow) sparbit_plan();
    if (!h) return SPARBIT_ERR_NOMEM;
    int rc;
    try {
        rc = sparbit::build_plan(p, algo, h->plan);
    } catch (const std::bad_alloc&) {
        rc = SPARBIT_ERR_NOMEM;
    }
    if (rc != SPARBIT_OK) {
        delete h;
        return rc;
    }
    *out = h;
    return SPARBIT_OK;
}

int sparbit_plan_num_steps(const sparbit_plan_t* plan)
{
    return plan ? int(plan->plan.steps.size()) : SPARBIT_ERR_ARG;
}

int sparbit_plan_step(const sparbit_plan_t* plan, int step, sparbit_step_t* out)
{
    if (!plan || !out || step < 0 || step >= int(plan->plan.steps.size())) return SPARBIT_ERR_ARG;
    const sparbit::Step& st = plan->plan.steps[step];
    out->distance = st.distance;
    out->nblocks = st.nblocks;
    out->ignore = st.ignore;
    out->dst = st.dst.data();
    out->src = st.src.data();
    out->send_slot = st.send_slot.data();
    out->recv_slot = st.recv_slot.data();
    return SPARBIT_OK;
}

void sparbit_plan_destroy(sparbit_plan_t* plan) { delete plan; }

}  // extern "C"
