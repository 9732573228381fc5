// Host-side schedule tables (integer only, no HIP).
#pragma once
#include <cstdint>
#include <vector>

namespace sparbit {

// One communication step: every rank sends `nblocks` single blocks to dst[r]
// and receives as many from src[r].
struct Step {
    int distance = 0;
    int nblocks = 0;
    int ignore = 0;
    std::vector<int32_t> dst, src;              // [p]
    std::vector<int32_t> send_slot, recv_slot;  // [p * nblocks]
};

// Which buffer a copy phase reads or writes.
enum Buffer : int { BUF_SEND = 0, BUF_RECV = 1, BUF_WORK = 2 };

// One block copy: block indices (units of block_bytes) into the phase's source
// and destination buffers.
struct Copy {
    uint32_t src_block;
    uint32_t dst_block;
};

// A phase is what one launch (or one barrier-delimited section of the
// persistent kernel) executes: a batch of independent block copies.
struct Phase {
    int step = -1;  // -1: own-block placement; num_steps: Bruck's final rotation; else the step
    Buffer src_buf = BUF_RECV, dst_buf = BUF_RECV;
    bool skip_in_place = false;      // phase is dropped when sendbufs == NULL
    bool only_in_place = false;      // phase exists only when sendbufs == NULL
    bool fused_first = false;        // own-block placement and step 0 in one batch, step 0 reading the send buffer
    bool covered_by_fused = false;   // own-block and step-0 phases: dropped where the fused phase runs
    std::vector<Copy> copies;
};

struct Plan {
    int p = 0;
    int algo = 0;
    std::vector<Step> steps;
    std::vector<Phase> phases;
};

int ceil_log2(int p);
// Returns 0 or a negative SPARBIT_ERR_* code.
int build_plan(int p, int algo, Plan& out);

}  // namespace sparbit

struct sparbit_plan {
    sparbit::Plan plan;
};
