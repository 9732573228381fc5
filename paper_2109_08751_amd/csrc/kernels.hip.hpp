// gfx950 copy kernels: every phase of a schedule is a batch of independent
// block copies  dst_base[dst_block * B ..] <- src_base[src_block * B ..].
// Nothing here is a contraction: the kernels are plain HBM streams built from
// 16-byte (or 4- / 1-byte) global loads and stores.
#pragma once
#include <hip/hip_runtime.h>

#include <cstdint>

#include "plan.hpp"

namespace sparbit {

constexpr int WG = 256;  // 4 wavefronts of 64 lanes

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

template <typename V, bool NT>
__device__ __forceinline__ V ld(const V* p)
{
    if constexpr (NT)
        return __builtin_nontemporal_load(p);
    else
        return *p;
}

// Streaming store.  For 16-byte vectors that cover whole 128-byte lines the fastest form measured on MI355X is a
// write-through store at system scope (sc0 sc1): a linear copy runs at 6.69 TB/s with it against 6.45 TB/s with
// the non-temporal hint alone, block copies of 4 KiB .. 16 MiB gain 2 .. 20 %; on lines covered piecewise it
// loses to the hint, so the host picks.  The compiler has no builtin that emits it for 16 bytes, hence the one-instruction asm; the
// data operand comes from a tracked load, so the wait for that load is still the compiler's.
template <typename V, bool NT, bool WRITE_THROUGH = true>
__device__ __forceinline__ void st(V* p, V v)
{
    if constexpr (NT && WRITE_THROUGH && sizeof(V) == 16)
        asm volatile("global_store_dwordx4 %0, %1, off sc0 sc1" ::"v"(p), "v"(v) : "memory");
    else if constexpr (NT)
        __builtin_nontemporal_store(v, p);  // narrower stores fill a line piecewise: write-through is slower there
    else
        *p = v;
}

// ---------------------------------------------------------------------------
// The per-step kernel.  One workgroup of T lanes moves one tile of T * U
// vectors of one block copy and exits: no loop, and the table entry, both base
// addresses and the bound are wave-uniform (scalar registers).  V is the
// access width the call's alignment allows (16, 4 or 1 bytes); Index is 32-bit
// unless a block holds 2^32 vectors or more.  On MI355X the best rate comes
// from the smallest footprint per wave (U = 1: one load and one store per
// lane) with the parallelism left to the dispatcher; for blocks shorter than
// a tile the host picks a smaller T.
//
// XCD-aware mapping.  The dispatcher deals consecutive workgroups round-robin
// to the 8 XCDs, each with its own L2 and its own address-translation caches.
// The copies of a phase are far apart (stripes of 1 block every 2d blocks), so
// if the tiles of one block were dealt to all XCDs, every XCD would have to
// translate every block's pages and would see only every 8th tile.  Instead
// blockIdx.x interleaves G = 2^lg_g copies: copy = group * G + (x mod G),
// tile = x / G.  With G = 8 each XCD streams one whole block by itself.
// ---------------------------------------------------------------------------
template <typename V, typename Index, int T, int U, bool NT, bool LOOP, bool WT = true>
__global__ __launch_bounds__(T) void copy_tiles_kernel(const uint8_t* __restrict__ src_base,
                                                       uint8_t* __restrict__ dst_base,
                                                       const Copy* __restrict__ copies, uint32_t ncopies,
                                                       uint64_t block_bytes, uint32_t lg_g)
{
    const uint32_t group = blockIdx.z * gridDim.y + blockIdx.y;
    const uint32_t c = (group << lg_g) + (blockIdx.x & ((1u << lg_g) - 1u));
    if (c >= ncopies) return;
    const Copy cp = copies[c];
    const V* __restrict__ s = reinterpret_cast<const V*>(src_base + uint64_t(cp.src_block) * block_bytes);
    V* __restrict__ d = reinterpret_cast<V*>(dst_base + uint64_t(cp.dst_block) * block_bytes);
    const Index vpb = Index(block_bytes / sizeof(V));
    const Index v0 = Index(blockIdx.x >> lg_g) * Index(T * U) + threadIdx.x;
    auto move = [&](Index v) {
        V x[U];
#pragma unroll
        for (int u = 0; u < U; ++u)
            if (v + Index(u * T) < vpb) x[u] = ld<V, NT>(s + v + Index(u * T));
#pragma unroll
        for (int u = 0; u < U; ++u)
            if (v + Index(u * T) < vpb) st<V, NT, WT>(d + v + Index(u * T), x[u]);
    };
    if constexpr (LOOP) {  // blocks so long that their tiles exceed the grid's x extent: several trips
        const Index stride = Index(gridDim.x >> lg_g) * Index(T * U);
        for (Index v = v0; v < vpb; v += stride) move(v);
    } else {
        move(v0);
    }
}

// ---------------------------------------------------------------------------
// Copy table of a Sparbit call, written on the device from the stripe closed
// form (the host passes, per step, the distance d and the blocks per rank n):
// entries 0 .. p-1 place the own blocks, then step s holds, for every rank r and
// j < n, the copy of slot (r - 2 j d) mod p from rank r to rank (r + d) mod p.
// Same layout as the tables the host builds for the other entry points.
// ---------------------------------------------------------------------------
struct StaticSteps {
    uint32_t nsteps;
    uint32_t d[12];
    uint32_t n[12];
    uint32_t first[13];  // first[s]: table index of step s; first[nsteps]: one past the end
};

__global__ __launch_bounds__(WG) void static_tables_kernel(Copy* __restrict__ out, uint32_t p, const StaticSteps st)
{
    const uint32_t t = blockIdx.x * WG + threadIdx.x;
    if (t >= st.first[st.nsteps]) return;
    if (t < p) {
        out[t] = Copy{t, t * p + t};
        return;
    }
    uint32_t s = 0;
    while (t >= st.first[s + 1]) ++s;  // ends: t < first[nsteps]
    const uint32_t e = t - st.first[s];
    const uint32_t r = e / st.n[s], j = e - r * st.n[s];
    const uint32_t back = (2u * j * st.d[s]) % p;
    const uint32_t slot = r >= back ? r - back : r + p - back;
    uint32_t to = r + st.d[s];
    if (to >= p) to -= p;
    out[t] = Copy{r * p + slot, to * p + slot};
}

// ---------------------------------------------------------------------------
// Tree form of Sparbit (Section III-B: p binomial trees, the tree of block b
// shifted by b, all advancing together).  The trees never touch each other's
// data -- tree b only reads and writes slot b of the receive buffers -- and
// neither do different byte ranges of one block, so one wavefront can carry
// one piece of one block through its whole tree with no flag, no barrier and
// no table: lane l moves the same 16 bytes of the piece in every message, and
// a load that follows the same lane's store to the same address sees that
// store (program order of one thread).
//
// The messages of tree b, in relative ranks rho = (rank - b) mod p: the step
// with distance d sends from every rho that is a multiple of 2d to rho + d, as
// long as rho + d < p (that bound is the "ignore" rule: the stripe kept back is
// the one whose destination would pass the root again).  So rho received the
// block in the step whose distance is the lowest set bit of rho, and forwards it
// to rho + d' for every smaller power of two d' with rho + d' < p.  A forwarder
// is read once, when its turn comes, and the value is stored to all of its
// destinations: the reads that its forwards of different steps would make of
// the same slot are merged.
//
// Order.  Any order in which a rank is read after it was written is valid; the
// parent of rho is rho minus its lowest set bit, so increasing rho is one.  The
// kernel walks runs of K = 2^lg_k consecutive relative ranks; inside a run it
// goes level by level (the run's first rank, then +K/2, then +K/4 and +3K/4,
// ...), loading a batch of forwarders at once, and the next run's first rank is
// loaded ahead, while the current run is served.  Small K keeps the distance
// between the write and the read of a slot short (the read hits the cache that
// holds the write); K >= p is the step order of Algorithm 1 (all forwards of a
// step before the next step), which has the fewest dependent round trips.
//
// Workgroups are single wavefronts (teams and gangs, below, hold several);
// blockIdx.x interleaves 2^lg_g trees so that each XCD streams through the
// pieces of one tree at a time.
// ---------------------------------------------------------------------------
struct TreeArgs {
    const uint8_t* send;  // nullptr: in place, slot r of rank r already holds rank r's block
    uint8_t* recv;
    uint64_t block_bytes;  // equal blocks: slot k at byte k * block_bytes of a row
    uint64_t vpb;          // equal blocks: vectors per block
    uint64_t row_bytes;    // distance between two ranks' receive buffers
    // Blocks of different sizes (Allgatherv): bytes of slot k and its offset in a row (and of rank k's block in the
    // send buffer); nullptr for equal blocks.
    const uint64_t* counts;
    const uint64_t* displs;
    uint32_t p;
    uint32_t top;   // distance of the first step: 2^(ceil(log2 p) - 1), 0 for p = 1
    uint32_t lg_k;
    uint32_t lg_g;
    uint32_t lg_s;  // gangs: the pieces of a workgroup's wavefronts lie 2^lg_s pieces apart
};

// Store forms of the tree kernel (ST), for 16-byte vectors.  0: plain, the line is allocated in the XCD's L2 and
// written back later.  2: write-through at system scope (sc0 sc1), the line goes straight to the memory side.
// 3: by destination -- plain for a rank that forwards and is read again soon, write-through for the others.
// 1: plain stores, and a run of 8 is walked so that every forwarder is read back right after it was stored, while
// its lines are still in the caches, and held in registers until its turn to forward; so are the first ranks of the
// runs 8, 16 and 32 ranks ahead (the form for calls that the caches hold a good part of: no read leaves the XCD but
// that of every eighth run's first rank, and the write-back of such a call is cheap).
// 4: the walk of 1 with the stores of 3 -- plain where the rank is read back at once, write-through for the ranks that
// only receive and for the first ranks of far runs (the form for the largest calls).
// The 16-byte accesses are raw buffer loads and stores: the base of a slot's piece is wave-uniform and sits in
// scalar registers (no per-lane 64-bit address arithmetic), the piece's length is the buffer's size, so lanes past
// a block's ragged end are dropped by the bounds check, and the cache-policy bits are an operand of the
// instruction the compiler knows, so it counts these stores like any others when it places its waits (stores
// issued from inline assembly are invisible to it, and it then waits for everything before every access).
constexpr int kBufferSc0Sc1 = 1 | 16;  // cache-policy operand: bit 0 = sc0, bit 4 = sc1

__device__ __forceinline__ __amdgpu_buffer_rsrc_t piece_buffer(const uint8_t* base, uint32_t bytes)
{
    // stride 0 (raw), `bytes` addressable, third descriptor word for untyped 32-bit accesses on gfx9-class targets
    return __builtin_amdgcn_make_buffer_rsrc(const_cast<uint8_t*>(base), 0, int(bytes), 0x00020000);
}

// s_waitcnt vmcnt(0): every vector-memory access issued so far has completed (loads and stores count together and
// complete in order on this target).  The operand leaves the export and scalar/LDS counters at "no wait".
__device__ __forceinline__ void wait_for_loads() { __builtin_amdgcn_s_waitcnt(0x0F70); }

// What a lane holds of one rank's piece: U vectors and, in the ANY form, one byte of the piece's ragged end.
template <typename V, int U>
struct Held {
    V v[U];
    uint8_t tail;
};

// PF: the first rank of the next run is loaded ahead, while the current run is served.
// ANY (16-byte vectors, U = 1): blocks of any length at any byte address.  Which bytes of a block a lane moves must
// not depend on the rank (the lane reads back what it wrote itself), so the pieces are cut in block offsets, the same
// at every rank: piece 0 ends where the block, as it lies in its own rank's receive buffer, reaches a 128-byte line
// (a 1 KiB boundary where the rows are a multiple of 1 KiB apart), the others follow in steps of 1 KiB.  Where all ranks' slots have that same position relative to the lines (rows
// a multiple of 128 bytes apart) every store covers whole lines; elsewhere the same accesses are unaligned, which the
// target's buffer loads and stores accept.  A piece is a run of 16-byte chunks, one per lane, and, at the block's
// first and last piece, up to 15 single bytes, one per lane.
//
// WALK 1 (DOUBLING): the same form for Recursive Doubling (Section II-A; p a power of two).  Seen by block, that schedule is
// a binomial tree as well, with the distances in the opposite order and the rank found by exclusive-or: with rho =
// rank xor b, step s sends from every rho < 2^s to rho + 2^s.  So rho receives in the step of its highest set bit and
// forwards in every later step, i.e. every rho below p/2 forwards and its destinations are far away.  The walk is
// the step order: the ranks that received in one step are loaded in batches and each is stored to all its
// destinations.  With store forms 1 and 4 it is walked like Sparbit's tree instead: under sigma = rho with its
// log2(p) bits reversed the two trees are the same (rho < 2^s means sigma is a multiple of 2^(L - s), and rho + 2^s is
// sigma + 2^(L - 1 - s), a distance below sigma's lowest set bit), so the runs and the read-back-at-once walk below
// serve with the rank found as b xor the reversed bits of the walk's relative rank.
//
// TEAM: several wavefronts per workgroup share one piece of one tree, for calls so small that the time is one
// wavefront's walk through all p ranks (its address arithmetic alone is ~100 ns per rank).  The tree is cut into
// runs of K = 2^lg_k relative ranks, one per wavefront; a run's first rank receives from the first rank of an earlier
// run, so the wavefront of that run stores it, waits until the store is done, and raises a flag in LDS, which the
// receiving wavefront polls before it loads its first rank and walks its run as above.  The chain of such hand-overs
// is log2(wavefronts) long.  A wavefront only ever waits for a wavefront of its own workgroup that waits for nothing
// it has not received yet (the first run waits for nothing), so every wait ends; it is bounded all the same.
// Recursive Doubling's tree is cut by the low bits of the relative rank instead (see the kernel).
constexpr uint32_t kTeamSpinLimit = 1u << 22;  // polls of ~100 cycles each

//
// WALK 2, Ring (Section II-A) in the same form: per block a chain, relative rank rho forwards to rho + 1, so the
// wavefront stores a rank and reads it back at once, p - 1 times.
constexpr int kWalkSparbit = 0, kWalkDoubling = 1, kWalkChain = 2;

// GANG: the workgroup holds GANG wavefronts that each carry a piece of their own through the same tree, the pieces
// 2^lg_s KiB apart (16 or 32), and meet at a barrier before every run.  What the memory side then sees at one time are
// stores to one rank's slot that lie 16 or 32 KiB apart, which it takes at a higher rate than stores to unrelated
// places (a stream of nothing but such stores, 16 GiB: 6.4-6.6 TB/s with 32 KiB against 5.7 TB/s with adjacent or
// unrelated pieces; 16 KiB apart 6.2-6.4, 64 KiB 6.2-6.3, 8 KiB and less or 256 KiB and more: no gain).  The counters
// say why: every store of a wavefront goes to another rank's receive buffer, megabytes from the one before, so a
// compute unit's first-level address translation cache misses on nearly every store of independent wavefronts (cfg4:
// 13.4 M misses per call, 0.8 per store); the wavefronts of a gang store into the same 64 or 128 KiB at the same time
// and share one miss (gangs of 4: 4.0 M; cfg5 8.7 M against 2.1 M).  GANG is 4 (two gangs per compute unit) or 8 (one).
// A piece index past the block's end leaves its wavefront with an empty buffer: its accesses are dropped by the
// bounds check and it still meets every barrier.

template <typename V, int U, int NB, int ST, bool PF, bool VAR = false, bool ANY = false, int WALK = kWalkSparbit,
          bool TEAM = false, int GANG = 1>
__global__ __launch_bounds__(TEAM ? 1024 : 64 * GANG) void tree_kernel(const TreeArgs a)
{
    static_assert(GANG == 1 || (!TEAM && (ST == 1 || ST == 4 || WALK == kWalkChain) && sizeof(V) == 16 && U == 1),
                  "gangs walk 16-byte vectors, one per lane, in the read-back-at-once forms or along Ring's chain");
    constexpr bool DOUBLING = WALK == kWalkDoubling, CHAIN = WALK == kWalkChain;
    static_assert(!CHAIN || (!PF && !TEAM), "a chain has nothing to look ahead of and nothing to share");
    static_assert(!ANY || (U == 1 && sizeof(V) == 16), "the any-alignment form moves one 16-byte chunk per lane");
    constexpr bool REVERSED = DOUBLING && (ST == 1 || ST == 4);  // the doubling tree walked as Sparbit's, bits reversed
    static_assert(!DOUBLING || !PF || REVERSED, "the step-order doubling walk has no run to look ahead of");
    static_assert(!REVERSED || !TEAM, "teams walk the doubling tree by the low bits of the relative rank");
    static_assert(!TEAM || (!PF && U == 1), "a team's wavefronts walk one part of the tree each, one vector per lane");
    const uint32_t lane = TEAM || GANG > 1 ? (threadIdx.x & 63u) : threadIdx.x;
    const uint32_t wave = TEAM || GANG > 1 ? uint32_t(__builtin_amdgcn_readfirstlane(int(threadIdx.x >> 6))) : 0u;
    const uint32_t group = blockIdx.z * gridDim.y + blockIdx.y;
    // The tree (origin rank = slot) and the piece of it.  A last group of fewer than 2^lg_g trees interleaves just
    // those, so that its pieces still go round all XCDs (p = 257: the last tree alone would run on one of them).
    const uint32_t p = a.p;
    const uint32_t first = group << a.lg_g;
    uint32_t b = first + (blockIdx.x & ((1u << a.lg_g) - 1u));
    uint32_t piece_index = blockIdx.x >> a.lg_g;
    if (first >= p) return;
    if (p - first < (1u << a.lg_g)) {
        const uint32_t t = p - first;
        b = first + blockIdx.x % t;
        piece_index = blockIdx.x / t;
        if (piece_index >= (gridDim.x >> a.lg_g)) return;  // the grid holds 2^lg_g trees' pieces
    }
    uint64_t offset = uint64_t(b) * a.block_bytes;  // this tree's block inside a row
    if constexpr (VAR) offset = a.displs[b];
    if constexpr (GANG > 1)  // the workgroup's number counts groups of GANG << lg_s pieces and a place in one
        piece_index = (piece_index >> a.lg_s) * (uint32_t(GANG) << a.lg_s) + (piece_index & ((1u << a.lg_s) - 1u)) + (wave << a.lg_s);
    uint32_t piece_vectors;  // V's in this wavefront's piece
    uint32_t tail_bytes = 0;  // ANY: single bytes after them
    bool part_of_a_line = false;  // ANY: the piece starts or ends inside a 128-byte line (a block's first and last piece)
    if constexpr (ANY) {
        const uint64_t bytes = VAR ? a.counts[b] : a.block_bytes;
        const uint64_t own = reinterpret_cast<uint64_t>(a.recv) + uint64_t(b) * a.row_bytes + offset;
        uint64_t at, hi;
        bool none;  // uniform: no such piece in this block
        if ((a.row_bytes & 1023u) == 0) {
            // Rows a multiple of 1 KiB apart: the pieces are the block's parts in the cells of the 1 KiB grid of
            // addresses, which are the same cells at every rank (per-slot sizes of 0.5-1.5 MiB on 128 ranks, rows rounded
            // up to 1 KiB, against the cut below, in turn on the same buffers: 3.00 against 3.13 ms, 3.40 against 3.43 ms).
            // piece_index counts cells from the block's first one; in gangs, where the rows are a multiple of the GANG <<
            // lg_s KiB apart that a gang spans, from the start of the group of that many cells that holds it, so that a
            // gang's pieces lie in one such group of the address grid at every rank.
            uint64_t cell = own >> 10;
            if constexpr (GANG > 1) {
                const uint64_t group = uint64_t(GANG) << a.lg_s;  // cells
                if ((a.row_bytes & ((group << 10) - 1u)) == 0) cell &= ~(group - 1u);
            }
            cell += piece_index;
            const uint64_t lo = cell << 10 > own ? cell << 10 : own;
            const uint64_t end = own + bytes, up = (cell + 1) << 10 < end ? (cell + 1) << 10 : end;
            none = lo >= up;
            at = none ? 0 : lo - own;
            hi = none ? 0 : up - own;
        } else {
            // other rows: the block bytes ahead of the first line boundary, then 1 KiB pieces (the cells' cut costs 0-3 %
            // here)
            const uint64_t to_line = (0 - own) & 127u;
            const uint64_t i = piece_index;
            at = i ? to_line + (i - 1) * 1024u : 0;
            hi = to_line + i * 1024u;
            if (hi > bytes) hi = bytes;
            none = at >= hi;
            if (none) at = hi = 0;
        }
        if (none) {
            if constexpr (GANG == 1) return;  // in a gang it stays for the barriers, with an empty buffer
        }
        offset += at;
        piece_vectors = uint32_t(hi - at) >> 4;
        tail_bytes = uint32_t(hi - at) & 15u;
        part_of_a_line = hi - at != 1024u || ((own + at) & 127u) != 0;
    } else {
        const uint64_t vectors = VAR ? a.counts[b] / sizeof(V) : a.vpb;
        uint64_t piece_at = uint64_t(piece_index) * uint64_t(64 * U);  // first vector of the piece
        bool no_piece = piece_at >= vectors;  // uniform: a shorter block has no such piece
        if (no_piece) {
            if constexpr (GANG == 1) return;
            piece_at = 0;  // stays for the barriers, with an empty buffer
        }
        offset += piece_at * sizeof(V);
        const uint64_t left = vectors - piece_at;
        piece_vectors = no_piece ? 0u : left < uint64_t(64 * U) ? uint32_t(left) : uint32_t(64 * U);
    }
    bool ok[U];
#pragma unroll
    for (int u = 0; u < U; ++u) ok[u] = lane + uint32_t(u * 64) < piece_vectors;
    typedef Held<V, U> H;
    // The piece of slot b held by the rank at relative rank rho (wave-uniform).  No __restrict__ anywhere: a slot
    // is written and later read.
    auto slot = [&](uint32_t rho) -> uint8_t* {
        uint32_t r;
        if constexpr (REVERSED) r = b ^ (__builtin_bitreverse32(rho) >> __builtin_clz(a.top | 1u));  // a.top = p / 2 (0: one rank)
        else r = DOUBLING ? (b ^ rho) : b + rho;
        if (r >= p) r -= p;
        return a.recv + uint64_t(r) * a.row_bytes + offset;
    };
    auto load = [&](const uint8_t* s, H& x) {
        if constexpr (sizeof(V) == 16) {
            const __amdgpu_buffer_rsrc_t rs = piece_buffer(s, piece_vectors * 16u);
#pragma unroll
            for (int u = 0; u < U; ++u)
                x.v[u] = __builtin_bit_cast(V, __builtin_amdgcn_raw_buffer_load_b128(rs, int(lane * 16u + u * 1024u), 0, 0));
            if constexpr (ANY) {
                if (tail_bytes)
                    x.tail = __builtin_amdgcn_raw_buffer_load_b8(piece_buffer(s + piece_vectors * 16u, tail_bytes), int(lane), 0, 0);
            }
        } else {
            const V* sv = reinterpret_cast<const V*>(s) + lane;
#pragma unroll
            for (int u = 0; u < U; ++u)
                if (ok[u]) x.v[u] = sv[u * 64];
        }
    };
    auto store = [&](uint8_t* d, const H& x, bool read_again_soon) {
        if constexpr (sizeof(V) == 16) {
            const __amdgpu_buffer_rsrc_t rd = piece_buffer(d, piece_vectors * 16u);
            typedef uint32_t raw4 __attribute__((ext_vector_type(4)));
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const int at = int(lane * 16u + u * 1024u);
                const raw4 v = __builtin_bit_cast(raw4, x.v[u]);
                // Write-through stores that cover part of a line are slow (the any-alignment form on 256 ranks with
                // 4 KiB + 4 byte blocks, where two pieces in six are such: 328 us all write-through, 141 us this way).
                if (ST == 0 || ST == 1 || ((ST == 3 || ST == 4) && read_again_soon) || (ANY && part_of_a_line))
                    __builtin_amdgcn_raw_buffer_store_b128(v, rd, at, 0, 0);
                else
                    __builtin_amdgcn_raw_buffer_store_b128(v, rd, at, 0, kBufferSc0Sc1);
            }
            if constexpr (ANY) {
                if (tail_bytes)
                    __builtin_amdgcn_raw_buffer_store_b8(x.tail, piece_buffer(d + piece_vectors * 16u, tail_bytes), int(lane), 0,
                                                         0);
            }
        } else {
            V* dv = reinterpret_cast<V*>(d) + lane;
#pragma unroll
            for (int u = 0; u < U; ++u)
                if (ok[u]) dv[u * 64] = x.v[u];
        }
    };
    const uint32_t K = 1u << a.lg_k;
    // From relative rank rho to rho + d.  The destination is read again soon if it forwards (d >= 2: it is even)
    // and belongs to this run or is the first rank of the next one.
    auto send_to = [&](uint32_t rho, uint32_t d, const H& x) { store(slot(rho + d), x, d >= 2 && d <= K); };
    // A rank forwards if it is even in the tree and the next relative rank exists (its nearest destination).
    auto forwards = [&](uint32_t rho) { return (rho & 1u) == 0 && rho + 1 < p; };
    if constexpr (TEAM && DOUBLING) {
        // Recursive Doubling's tree splits by the low bits of rho: the ranks with rho mod W = c form the sub-tree of
        // rho = c (every forward of a rank >= W adds a power of two >= W), W = 2^lg_k wavefronts, c = this one's
        // number.  Rank c receives from rank c minus its highest set bit, which belongs to an earlier wavefront.
        __shared__ uint32_t arrived[16];  // per wavefront: its sub-tree's first rank has been stored
        if (lane == 0) arrived[wave] = 0;
        __syncthreads();
        const uint32_t W = 1u << a.lg_k, c = wave;
        if (c >= W || 2 * W > p) return;  // the host launches W wavefronts, W <= p / 2
        H xt;
        if (c == 0) {
            if (a.send) {
                load(a.send + offset, xt);
                store(slot(0), xt, false);
            } else {
                load(slot(0), xt);
            }
        } else {
            uint32_t polls = 0;
            while (__hip_atomic_load(&arrived[c], __ATOMIC_ACQUIRE, __HIP_MEMORY_SCOPE_WORKGROUP) == 0) {
                if (++polls > kTeamSpinLimit) return;
                __builtin_amdgcn_s_sleep(1);
            }
            load(slot(c), xt);
        }
        bool handed = false;
        for (uint32_t d = 1; d < W; d <<= 1)  // the steps after the one c received in, while they leave the sub-tree
            if (d > c) {
                store(slot(c + d), xt, false);
                handed = true;
            }
        if (handed) {
            wait_for_loads();  // those stores are done
            for (uint32_t d = 1; d < W; d <<= 1)
                if (d > c && lane == 0)
                    __hip_atomic_store(&arrived[c + d], 1u, __ATOMIC_RELEASE, __HIP_MEMORY_SCOPE_WORKGROUP);
        }
        for (uint32_t d = W; d < p; d <<= 1) store(slot(c + d), xt, false);
        for (uint32_t lvl = W; 2 * lvl < p; lvl <<= 1) {  // the sub-tree's ranks that received at distance lvl
            for (uint32_t n0 = c + lvl; n0 < 2 * lvl; n0 += W * NB) {
                H x[NB];
#pragma unroll
                for (int i = 0; i < NB; ++i)
                    if (n0 + W * i < 2 * lvl) load(slot(n0 + W * i), x[i]);
                wait_for_loads();
#pragma unroll
                for (int i = 0; i < NB; ++i)
                    if (n0 + W * i < 2 * lvl)
                        for (uint32_t d = 2 * lvl; d < p; d <<= 1) store(slot(n0 + W * i + d), x[i], false);
            }
        }
        return;
    } else if constexpr (TEAM) {
        __shared__ uint32_t arrived[16];  // per run of the team: its first rank has been stored
        if (lane == 0) arrived[wave] = 0;
        __syncthreads();
        const uint32_t first = wave << a.lg_k;  // this wavefront's run starts here
        if (first >= p || (first != 0 && !forwards(first))) return;  // no such run, or nothing to forward in it
        if (first != 0) {
            uint32_t polls = 0;
            while (__hip_atomic_load(&arrived[wave], __ATOMIC_ACQUIRE, __HIP_MEMORY_SCOPE_WORKGROUP) == 0) {
                if (++polls > kTeamSpinLimit) return;
                __builtin_amdgcn_s_sleep(1);
            }
        }
        // After its first rank's forwards a run's wavefront tells the runs whose first ranks it stored to.
        auto hand_over = [&](uint32_t h, uint32_t dmax) {
            if (dmax < K) return;
            wait_for_loads();  // the stores are done
            for (uint32_t d = dmax; d >= K; d >>= 1)
                if (d < p - h && lane == 0)
                    __hip_atomic_store(&arrived[(h + d) >> a.lg_k], 1u, __ATOMIC_RELEASE, __HIP_MEMORY_SCOPE_WORKGROUP);
        };
        H xt;
        if (first == 0) {
            if (a.send) {
                load(a.send + offset, xt);
                store(slot(0), xt, false);
            } else {
                load(slot(0), xt);
            }
        } else {
            load(slot(first), xt);
        }
        // The first ranks of other runs first: their wavefronts are waiting.
        const uint32_t dmax = first ? ((first & (0u - first)) >> 1) : a.top;
        uint32_t d = dmax;
        for (; d >= K; d >>= 1)
            if (d < p - first) send_to(first, d, xt);
        hand_over(first, dmax);
        for (; d >= 1; d >>= 1)
            if (d < p - first) send_to(first, d, xt);
        const uint32_t end = (p - first < K) ? p : first + K;
        for (uint32_t st = K >> 1; st >= 2; st >>= 1) {
            for (uint32_t n0 = first + st; n0 < end; n0 += 2 * st * NB) {
                H x[NB];
#pragma unroll
                for (int i = 0; i < NB; ++i) {
                    const uint32_t n = n0 + 2 * st * i;
                    if (n < end && forwards(n)) load(slot(n), x[i]);
                }
                wait_for_loads();
#pragma unroll
                for (int i = 0; i < NB; ++i) {
                    const uint32_t n = n0 + 2 * st * i;
                    if (n < end)
                        for (uint32_t d = st >> 1; d >= 1; d >>= 1)
                            if (d < p - n) send_to(n, d, x[i]);
                }
            }
        }
        return;
    }
    H xh;  // the block as the run's first rank holds it
    if (a.send) {
        load(a.send + offset, xh);
        store(slot(0), xh, false);  // own-block placement; read again only in an in-place call
    } else {
        load(slot(0), xh);
    }
    if constexpr (CHAIN) {
        for (uint32_t rho = 1; rho < p; ++rho) {
            if constexpr (GANG > 1) {
                if ((rho & 3u) == 1u) __syncthreads();  // every wavefront of the gang takes every turn of this loop
            }
            store(slot(rho), xh, true);
            if (rho + 1 < p) {
                load(slot(rho), xh);  // what rho forwards is what it received
                wait_for_loads();
            }
        }
        return;
    }
    if constexpr (DOUBLING && !REVERSED) {
        for (uint32_t d = 1; d < p; d <<= 1) store(slot(d), xh, false);  // the origin sends in every step
        for (uint32_t lvl = 1; 2 * lvl < p; lvl <<= 1) {  // rho in [lvl, 2 lvl) received in the step with distance lvl
            for (uint32_t n0 = lvl; n0 < 2 * lvl; n0 += NB) {
                H x[NB];
#pragma unroll
                for (int i = 0; i < NB; ++i)
                    if (n0 + i < 2 * lvl) load(slot(n0 + i), x[i]);
                wait_for_loads();
#pragma unroll
                for (int i = 0; i < NB; ++i)
                    if (n0 + i < 2 * lvl)
                        for (uint32_t d = 2 * lvl; d < p; d <<= 1) store(slot(n0 + i + d), x[i], false);
            }
        }
        return;
    }
    H y16, y32;  // store forms 1 and 4: the first ranks of the runs 16 and 32 ranks ahead, read back when they were stored
    for (uint32_t h = 0; h < p; h += K) {  // h: first relative rank of the run; its lowest set bit is >= K
        const uint32_t end = (p - h < K) ? p : h + K;
        if constexpr (GANG > 1) __syncthreads();  // every wavefront of the gang takes every turn of this loop
        if constexpr (ST == 1 || ST == 4) {  // K = 8 (the host sees to it); PF: xh is this run's first rank, loaded by the run before
            static_assert(PF && U == 1, "the read-back-at-once walk keeps the next run's first rank in registers");
            auto to = [&](uint32_t n, uint32_t d, const H& x) {  // a forward, if both ranks exist
                if (n < p && d < p - n) send_to(n, d, x);
            };
            auto back = [&](uint32_t n, H& x) {  // read a forwarder back
                if (n < p && forwards(n)) load(slot(n), x);
            };
            const uint32_t dmax = h ? ((h & (0u - h)) >> 1) : a.top;
            for (uint32_t d = dmax; d > 32; d >>= 1) to(h, d, xh);
            // The first ranks of the runs at +32 and +16 are read back at once as well and kept until those runs
            // begin, so that only every eighth run starts with a load of what an earlier run stored long ago.
            if (dmax >= 32) {
                if (h + 32 < p) store(slot(h + 32), xh, true);
                back(h + 32, y32);
            }
            if (dmax >= 16) {
                if (h + 16 < p) store(slot(h + 16), xh, true);
                back(h + 16, y16);
            }
            H x4, x2, x6, xn;
            if (dmax >= 8) {
                to(h, 8, xh);
                back(h + 8, xn);
            }
            to(h, 4, xh);
            back(h + 4, x4);
            to(h, 2, xh);
            back(h + 2, x2);
            to(h, 1, xh);
            wait_for_loads();
            if constexpr (GANG > 1) __syncthreads();  // the gang's stores stay together (p = 125, 64 KiB: 163 against 171 us)
            to(h + 4, 2, x4);
            back(h + 6, x6);
            to(h + 4, 1, x4);
            to(h + 2, 1, x2);
            wait_for_loads();
            to(h + 6, 1, x6);
            if (dmax < 8) {  // the next run's first rank was stored by an earlier run
                const uint32_t hn = h + 8;
                if ((hn & 31u) == 16u) xn = y16;       // ... 16 ranks back, which kept it
                else if ((hn & 63u) == 32u) xn = y32;  // ... 32 ranks back
                else back(hn, xn);
            }
            xh = xn;
            continue;
        }
        if (!PF && h != 0 && forwards(h)) load(slot(h), xh);
        for (uint32_t d = h ? ((h & (0u - h)) >> 1) : a.top; d >= 1; d >>= 1)
            if (d < p - h) send_to(h, d, xh);
        // The next run's first rank got the block from this run's first rank (just above) or from an earlier run,
        // so its load can already travel while this run's other forwarders are served.
        H xn;
        const uint32_t hn = h + K;
        if (PF && hn < p && forwards(hn)) load(slot(hn), xn);
        for (uint32_t st = K >> 1; st >= 2; st >>= 1) {  // forwarders whose lowest set bit is st
            for (uint32_t n0 = h + st; n0 < end; n0 += 2 * st * NB) {
                H x[NB];
#pragma unroll
                for (int i = 0; i < NB; ++i) {
                    const uint32_t n = n0 + 2 * st * i;
                    if (n < end && forwards(n)) load(slot(n), x[i]);
                }
                // One wait for the whole batch, stated here: behind the conditions above the compiler would
                // otherwise wait before each forwarder's stores, i.e. for the previous forwarder's stores.
                wait_for_loads();
#pragma unroll
                for (int i = 0; i < NB; ++i) {
                    const uint32_t n = n0 + 2 * st * i;
                    if (n < end)
                        for (uint32_t d = st >> 1; d >= 1; d >>= 1)
                            if (d < p - n) send_to(n, d, x[i]);
                }
            }
        }
        if constexpr (PF) xh = xn;
    }
}

// ---------------------------------------------------------------------------
// Blocks of different sizes (Allgatherv): every copy carries its own byte
// offsets and length.  Same shape as copy_tiles_kernel -- one tile per
// workgroup, copies dealt round-robin to consecutive workgroups -- with the
// grid's x extent sized for the longest block of the launch; workgroups past
// the end of a shorter block exit at once (the host groups the copies of a
// phase into launches of similar length, so at most half of them do).  V is
// the access width that all offsets, lengths and base addresses allow.
// ---------------------------------------------------------------------------
// Offsets and the length are below 2^40 (the host checks), so an entry packs into 16 bytes: one scalar load per
// workgroup, and half the table memory of three 64-bit fields (p = 4096: 16.7 million entries).
struct VarCopy {
    uint64_t a;  // bits 0..39: byte offset from the phase's source base; bits 40..63: length bits 0..23
    uint64_t b;  // bits 0..39: byte offset from the phase's destination base; bits 40..55: length bits 24..39
};
constexpr uint64_t kVarFieldMask = (uint64_t(1) << 40) - 1;

__host__ __device__ inline VarCopy pack_var_copy(uint64_t src_off, uint64_t dst_off, uint64_t len)
{
    return VarCopy{src_off | ((len & 0xffffffull) << 40), dst_off | ((len >> 24) << 40)};
}
__host__ __device__ inline uint64_t var_src_off(const VarCopy& c) { return c.a & kVarFieldMask; }
__host__ __device__ inline uint64_t var_dst_off(const VarCopy& c) { return c.b & kVarFieldMask; }
__host__ __device__ inline uint64_t var_len(const VarCopy& c) { return (c.a >> 40) | ((c.b >> 40) << 24); }

template <typename V, bool NT, bool WT = false>
__global__ __launch_bounds__(WG) void copy_var_kernel(const uint8_t* __restrict__ src_base,
                                                      uint8_t* __restrict__ dst_base,
                                                      const VarCopy* __restrict__ copies, uint32_t ncopies,
                                                      uint32_t lg_g)
{
    const uint32_t group = blockIdx.z * gridDim.y + blockIdx.y;
    const uint32_t c = (group << lg_g) + (blockIdx.x & ((1u << lg_g) - 1u));
    if (c >= ncopies) return;
    const VarCopy cp = copies[c];
    const uint64_t src_off = var_src_off(cp), dst_off = var_dst_off(cp), len = var_len(cp);
    const uint64_t v = uint64_t(blockIdx.x >> lg_g) * WG + threadIdx.x;
    if (v < len / sizeof(V)) {
        const V* __restrict__ s = reinterpret_cast<const V*>(src_base + src_off);
        V* __restrict__ d = reinterpret_cast<V*>(dst_base + dst_off);
        // The host picks the store form: the non-temporal hint for long blocks (128 ranks x 1 MiB: 6.5 TB/s against
        // 6.4 TB/s with the write-through form that serves copy_tiles_kernel better), write-through for whole-line
        // blocks below 128 KiB.
        st<V, NT, WT>(d + v, ld<V, NT>(s + v));
    }
}

// ---------------------------------------------------------------------------
// Blocks whose ends do not fall on 16-byte boundaries.  Moving them with 4- or
// 1-byte accesses costs 2x to 6x of the 16-byte rate, so the body of such a copy
// is moved in 16-byte vectors all the same: stores are aligned on the
// destination (whole-line writes), loads take whatever alignment the source then
// has -- global loads on this target accept any byte address, which is what the
// compiler itself assumes when it is handed an under-aligned vector type -- and
// the first workgroup of the copy also moves the bytes before the first aligned
// vector and the up to 15 bytes after the last, one byte per lane.
// Same shape as the kernels above: one tile per workgroup, copies dealt
// round-robin to consecutive workgroups; the trip loop only matters for blocks
// longer than the grid's x extent.
// ---------------------------------------------------------------------------
typedef u32x4 u32x4_any_align __attribute__((aligned(1)));

template <int T, bool NT>
__device__ __forceinline__ void realign_copy(const uint8_t* __restrict__ s, uint8_t* __restrict__ d, uint64_t n,
                                             uint64_t tile, uint64_t tiles_in_grid)
{
    // Long blocks start their vectors on a 128-byte line of the destination, so that every wavefront's store
    // covers whole lines (measured: 5.5 against 5.3 TB/s on 256 KiB blocks); short ones settle for 16 bytes.
    const uint32_t align_mask = n >= 32768u ? 127u : 15u;
    uint32_t head = uint32_t(0u - uint32_t(reinterpret_cast<uintptr_t>(d))) & align_mask;
    if (head > n) head = uint32_t(n);
    const uint64_t nvec = (n - head) >> 4;
    const uint32_t tail = uint32_t(n - head) & 15u;
    if (tile == 0) {
        for (uint32_t l = threadIdx.x; l < head; l += T) d[l] = s[l];
        if (threadIdx.x < tail) {
            const uint64_t o = head + (nvec << 4) + threadIdx.x;
            d[o] = s[o];
        }
    }
    const u32x4_any_align* __restrict__ sv = reinterpret_cast<const u32x4_any_align*>(s + head);
    u32x4* __restrict__ dv = reinterpret_cast<u32x4*>(d + head);
    for (uint64_t v = tile * T + threadIdx.x; v < nvec; v += tiles_in_grid * T) {
        u32x4 x;
        if constexpr (NT)
            x = __builtin_nontemporal_load(sv + v);
        else
            x = sv[v];
        st<u32x4, NT, false>(dv + v, x);  // write-through is slower here (4.4-5.5 against 5.3-6.4 TB/s)
    }
}

template <int T, bool NT>
__global__ __launch_bounds__(T) void copy_tiles_realign_kernel(const uint8_t* __restrict__ src_base,
                                                               uint8_t* __restrict__ dst_base,
                                                               const Copy* __restrict__ copies, uint32_t ncopies,
                                                               uint64_t block_bytes, uint32_t lg_g)
{
    const uint32_t group = blockIdx.z * gridDim.y + blockIdx.y;
    const uint32_t c = (group << lg_g) + (blockIdx.x & ((1u << lg_g) - 1u));
    if (c >= ncopies) return;
    const Copy cp = copies[c];
    realign_copy<T, NT>(src_base + uint64_t(cp.src_block) * block_bytes, dst_base + uint64_t(cp.dst_block) * block_bytes,
                        block_bytes, blockIdx.x >> lg_g, gridDim.x >> lg_g);
}

template <bool NT>
__global__ __launch_bounds__(WG) void copy_var_realign_kernel(const uint8_t* __restrict__ src_base,
                                                              uint8_t* __restrict__ dst_base,
                                                              const VarCopy* __restrict__ copies, uint32_t ncopies,
                                                              uint32_t lg_g)
{
    const uint32_t group = blockIdx.z * gridDim.y + blockIdx.y;
    const uint32_t c = (group << lg_g) + (blockIdx.x & ((1u << lg_g) - 1u));
    if (c >= ncopies) return;
    const VarCopy cp = copies[c];
    realign_copy<WG, NT>(src_base + var_src_off(cp), dst_base + var_dst_off(cp), var_len(cp), blockIdx.x >> lg_g,
                         gridDim.x >> lg_g);
}

// ---------------------------------------------------------------------------
// Flattened tiles: the (copy, element) space of a phase is one index range and
// every lane finds its copy by one division, so a tile may span many short
// blocks.  Used by the persistent kernel's grid-stride loop and, as a kernel of
// its own, for blocks shorter than one wavefront's worth of vectors, where a
// tile per block would leave most lanes idle and scatter partial-line writes
// over the XCDs.  (For longer blocks copy_tiles_kernel wins at every size: the
// per-lane division and table look-up cost more than a few idle lanes.)
// ---------------------------------------------------------------------------
template <typename V, typename Index, int UNROLL, bool NT>
__device__ __forceinline__ void copy_flat_tile(const uint8_t* __restrict__ src_base,
                                               uint8_t* __restrict__ dst_base,
                                               const Copy* __restrict__ copies, uint64_t block_bytes,
                                               Index vpb, Index total, Index tile)
{
    V x[UNROLL];
    const V* sp[UNROLL];
    V* dp[UNROLL];
    bool ok[UNROLL];
    const Index g0 = tile * Index(WG * UNROLL) + threadIdx.x;
#pragma unroll
    for (int u = 0; u < UNROLL; ++u) {
        const Index g = g0 + Index(u * WG);
        ok[u] = g < total;
        if (ok[u]) {
            const Index c = g / vpb;
            const Index o = g - c * vpb;
            const Copy cp = copies[c];
            sp[u] = reinterpret_cast<const V*>(src_base + uint64_t(cp.src_block) * block_bytes) + o;
            dp[u] = reinterpret_cast<V*>(dst_base + uint64_t(cp.dst_block) * block_bytes) + o;
            x[u] = ld<V, NT>(sp[u]);
        }
    }
#pragma unroll
    for (int u = 0; u < UNROLL; ++u)
        if (ok[u]) st<V, NT>(dp[u], x[u]);
}

template <typename V, typename Index, int UNROLL, bool NT>
__global__ __launch_bounds__(WG) void copy_flat_kernel(const uint8_t* __restrict__ src_base,
                                                       uint8_t* __restrict__ dst_base,
                                                       const Copy* __restrict__ copies,
                                                       uint64_t block_bytes, Index vpb, Index total)
{
    copy_flat_tile<V, Index, UNROLL, NT>(src_base, dst_base, copies, block_bytes, vpb, total,
                                         Index(blockIdx.x));
}

// ---------------------------------------------------------------------------
// Persistent form: all phases of one call in one launch.  The Waitall between
// steps is a device-wide barrier: thread 0 of every workgroup releases its
// workgroup's stores at agent scope (write-back of this XCD's L2), counts in,
// and acquires (invalidate) once all workgroups of the grid have arrived.  The
// grid is sized by the host so that every workgroup is resident.
// ---------------------------------------------------------------------------
struct DevPhase {
    uint32_t first_copy;  // offset into the plan's copy array
    uint32_t ncopies;
    int32_t src_buf;  // Buffer
    int32_t dst_buf;
    uint32_t copies_before;  // copies of the earlier phases of the same call (dataflow item numbering)
    uint32_t pad;
};

struct BarrierState {
    uint32_t arrived;  // monotonic within a launch; reset by the last workgroup to leave
    uint32_t left;
    uint32_t abort;   // set when a bounded wait expired in this launch; reset like `arrived`
    uint32_t errors;  // sticky count of launches that aborted (read by the host on request)
};

struct PersistentArgs {
    const uint8_t* base[3];  // BUF_SEND, BUF_RECV, BUF_WORK (const cast away for dst)
    const Copy* copies;
    const DevPhase* phases;
    BarrierState* bar;
    uint32_t* note;  // host-visible word: receives the stream's count of aborted launches when this one aborts
    uint64_t block_bytes;
    uint64_t spin_limit_ticks;  // bounded wait, in 100 MHz wall-clock ticks
    uint32_t nphases;
};

__device__ __forceinline__ bool grid_barrier(BarrierState* bar, uint32_t target, uint64_t limit)
{
    __shared__ uint32_t failed;
    __syncthreads();
    if (threadIdx.x == 0) {
        uint32_t f = 0;
        __hip_atomic_fetch_add(&bar->arrived, 1u, __ATOMIC_RELEASE, __HIP_MEMORY_SCOPE_AGENT);
        const uint64_t t0 = wall_clock64();
        // Spin on relaxed loads (no cache maintenance per poll); one acquire fence at the end.
        while (__hip_atomic_load(&bar->arrived, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) < target) {
            __builtin_amdgcn_s_sleep(1);
            if (uint64_t(wall_clock64()) - t0 > limit ||
                __hip_atomic_load(&bar->abort, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT)) {
                __hip_atomic_store(&bar->abort, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                f = 1;
                break;
            }
        }
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "agent");
        failed = f;
    }
    __syncthreads();
    return failed == 0;
}

template <typename V, int UNROLL, bool NT>
__global__ __launch_bounds__(WG) void persistent_kernel(const PersistentArgs a)
{
    const uint32_t nwg = gridDim.x;
    bool ok = true;
    for (uint32_t ph = 0; ph < a.nphases && ok; ++ph) {
        const DevPhase P = a.phases[ph];
        const uint8_t* src = a.base[P.src_buf];
        uint8_t* dst = const_cast<uint8_t*>(a.base[P.dst_buf]);
        const uint64_t vpb = a.block_bytes / sizeof(V);
        const uint64_t total = vpb * P.ncopies;
        const uint64_t ntiles = (total + WG * UNROLL - 1) / (WG * UNROLL);
        if (total + WG * UNROLL <= 0xffffffffull) {  // lane indices of the last tile stay below 2^32
            for (uint32_t t = blockIdx.x; t < uint32_t(ntiles); t += nwg)
                copy_flat_tile<V, uint32_t, UNROLL, NT>(src, dst, a.copies + P.first_copy, a.block_bytes,
                                                        uint32_t(vpb), uint32_t(total), t);
        } else {
            for (uint64_t t = blockIdx.x; t < ntiles; t += nwg)
                copy_flat_tile<V, uint64_t, UNROLL, NT>(src, dst, a.copies + P.first_copy, a.block_bytes,
                                                        vpb, total, t);
        }
        if (ph + 1 < a.nphases) ok = grid_barrier(a.bar, (ph + 1) * nwg, a.spin_limit_ticks);
    }
    // Leave: the last workgroup out puts the counters back to zero for the next
    // launch on this stream (nobody waits on `arrived` any more by then).
    __syncthreads();
    if (threadIdx.x == 0) {
        const uint32_t n = __hip_atomic_fetch_add(&a.bar->left, 1u, __ATOMIC_ACQ_REL, __HIP_MEMORY_SCOPE_AGENT);
        if (n == nwg - 1) {
            if (__hip_atomic_load(&a.bar->abort, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT)) {
                const uint32_t n_aborted =
                    __hip_atomic_fetch_add(&a.bar->errors, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) + 1u;
                __hip_atomic_store(a.note, n_aborted, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM);  // the host's next call sees it
                __hip_atomic_store(&a.bar->abort, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            }
            __hip_atomic_store(&a.bar->arrived, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            __hip_atomic_store(&a.bar->left, 0u, __ATOMIC_RELEASE, __HIP_MEMORY_SCOPE_AGENT);
        }
    }
}

// ---------------------------------------------------------------------------
// Dataflow form (the non-blocking variant the paper names as future work in
// its conclusion): one launch, no device-wide barrier.  The unit of work is
// one piece of one block copy (a block is cut into round(block_bytes / chunk_bytes) equal pieces); every chunk of a receive slot
// has a ready flag that holds the number of the call that last filled it.
// Items are numbered in phase order, one workgroup per item; a workgroup waits
// for the flag of its item's source chunk (unless the source is the send buffer
// or, in place, a rank's own slot), copies, and publishes the flag of the
// destination chunk.  An item only waits for an item of an earlier phase, i.e.
// a lower-numbered workgroup, and workgroups are started in increasing order,
// so whatever a resident workgroup waits for is itself resident or done: the
// grid makes progress whatever part of it is resident.  Waits are bounded all
// the same.
//
// What this machine makes expensive, and how the kernel avoids it:
//  - a device-scope atomic read-modify-write on one address costs ~70 ns and
//    serialises, so there is no ticket or arrival counter on the fast path;
//  - an agent-scope release / acquire is a write-back / invalidate of the whole
//    L2 of the XCD (~300 ns each, serialised per XCD), far too much per chunk.
//    Instead every data access is itself coherent at agent scope (relaxed
//    atomic loads and stores of 4 or 1 bytes, sc1 on the 16-byte ones: past the XCD's L2 to
//    the memory side), so no cache maintenance is needed: a wave waits for its
//    own stores to be acknowledged (s_waitcnt vmcnt(0)), the workgroup meets at
//    a barrier, and one lane stores the flag.
// ---------------------------------------------------------------------------
template <typename V>
__device__ __forceinline__ V coherent_ld(const V* p)
{
    return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

template <typename V>
__device__ __forceinline__ void coherent_st(V* p, V v)
{
    __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// 16-byte forms of the same coherent accesses.  The language offers no 16-byte atomic, and none is needed: the
// flag protocol orders the data, the accesses only have to go past the XCD's L2 like the ones above, which is the
// sc1 bit on the plain 16-byte instructions.  The compiler does not track loads issued from asm, so a group of
// four is issued and waited for inside one statement.
__device__ __forceinline__ void coherent_ld4(const u32x4* p0, const u32x4* p1, const u32x4* p2, const u32x4* p3,
                                             u32x4& x0, u32x4& x1, u32x4& x2, u32x4& x3)
{
    asm volatile(
        "global_load_dwordx4 %0, %4, off sc1\n\t"
        "global_load_dwordx4 %1, %5, off sc1\n\t"
        "global_load_dwordx4 %2, %6, off sc1\n\t"
        "global_load_dwordx4 %3, %7, off sc1\n\t"
        "s_waitcnt vmcnt(0)"
        : "=&v"(x0), "=&v"(x1), "=&v"(x2), "=&v"(x3)
        : "v"(p0), "v"(p1), "v"(p2), "v"(p3)
        : "memory");
}

template <>
__device__ __forceinline__ u32x4 coherent_ld<u32x4>(const u32x4* p)
{
    u32x4 x;
    asm volatile("global_load_dwordx4 %0, %1, off sc1\n\ts_waitcnt vmcnt(0)" : "=&v"(x) : "v"(p) : "memory");
    return x;
}

template <>
__device__ __forceinline__ void coherent_st<u32x4>(u32x4* p, u32x4 v)
{
    asm volatile("global_store_dwordx4 %0, %1, off sc1" ::"v"(p), "v"(v) : "memory");
}

struct FlowState {
    uint32_t abort;   // number of the last call in which a bounded wait expired
    uint32_t errors;  // sticky count of such calls
};

struct FlowArgs {
    const uint8_t* base[3];
    const Copy* copies;
    const DevPhase* phases;
    FlowState* state;
    uint32_t* note;          // host-visible word: receives this call's number when one of its waits expires
    uint32_t* flags;         // [2][p * p * chunks_per_block]: receive buffer, then the working buffer
    uint64_t block_bytes;
    uint64_t spin_limit_ticks;
    uint32_t nphases;
    uint32_t chunks_per_block;
    uint32_t chunk_vecs;     // chunk size in units of sizeof(V)
    uint32_t flags_per_buf;
    uint32_t epoch;          // number of this call on its stream, never 0
    uint32_t total_items;
    uint32_t p;
    uint32_t in_place;       // 1: slot r of rank r was filled by the caller before the call; nobody flags it
};

// One chunk whose ends are not on 16-byte boundaries, with the same coherent accesses: bytes up to the first
// 16-byte boundary of the destination and after the last one singly, the body in 16-byte vectors (aligned stores,
// loads at the source's alignment).
__device__ __forceinline__ void coherent_realign_chunk(const uint8_t* __restrict__ s, uint8_t* __restrict__ d, uint32_t n)
{
    uint32_t head = (0u - uint32_t(reinterpret_cast<uintptr_t>(d))) & 15u;
    if (head > n) head = n;
    const uint32_t nvec = (n - head) >> 4;
    const uint32_t tail = (n - head) & 15u;
    // The single bytes are loaded first and stored last, so that their round trips overlap the body's.
    const bool has_head = threadIdx.x < head;
    const bool has_tail = threadIdx.x >= 32u && threadIdx.x - 32u < tail;
    const uint32_t tail_at = head + (nvec << 4) + (threadIdx.x - 32u);
    uint8_t head_byte = 0, tail_byte = 0;
    if (has_head) head_byte = coherent_ld<uint8_t>(s + threadIdx.x);
    if (has_tail) tail_byte = coherent_ld<uint8_t>(s + tail_at);
    const u32x4* sv = reinterpret_cast<const u32x4*>(s + head);  // any alignment: only handed to the asm loads
    u32x4* dv = reinterpret_cast<u32x4*>(d + head);
    uint32_t v = 0;
    for (; nvec - v >= 4u * WG; v += 4u * WG) {
        const uint32_t l = v + threadIdx.x;
        u32x4 x0, x1, x2, x3;
        coherent_ld4(sv + l, sv + l + WG, sv + l + 2 * WG, sv + l + 3 * WG, x0, x1, x2, x3);
        coherent_st<u32x4>(dv + l, x0);
        coherent_st<u32x4>(dv + l + WG, x1);
        coherent_st<u32x4>(dv + l + 2 * WG, x2);
        coherent_st<u32x4>(dv + l + 3 * WG, x3);
    }
    for (v += threadIdx.x; v < nvec; v += WG) coherent_st<u32x4>(dv + v, coherent_ld<u32x4>(sv + v));
    if (has_head) coherent_st<uint8_t>(d + threadIdx.x, head_byte);
    if (has_tail) coherent_st<uint8_t>(d + tail_at, tail_byte);
}

// Thread 0 polls `flag` until it holds this call's number; the whole workgroup learns the outcome.  False: a
// bounded wait expired here or elsewhere in the launch, and the workgroup must leave.
__device__ __forceinline__ bool flow_wait(const FlowArgs& a, const uint32_t* flag)
{
    __shared__ uint32_t s_ok;
    if (threadIdx.x == 0) {
        uint32_t good = 1;
        const uint64_t t0 = wall_clock64();
        while (__hip_atomic_load(flag, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) != a.epoch) {
            __builtin_amdgcn_s_sleep(1);
            const bool expired = uint64_t(wall_clock64()) - t0 > a.spin_limit_ticks;
            if (expired || __hip_atomic_load(&a.state->abort, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) == a.epoch) {
                if (expired && __hip_atomic_exchange(&a.state->abort, a.epoch, __ATOMIC_RELAXED,
                                                     __HIP_MEMORY_SCOPE_AGENT) != a.epoch) {
                    __hip_atomic_fetch_add(&a.state->errors, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                    __hip_atomic_store(a.note, a.epoch, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM);  // the host's next call sees it
                }
                good = 0;
                break;
            }
        }
        s_ok = good;
    }
    __syncthreads();
    return s_ok != 0;  // the next write of s_ok comes after the barrier in flow_publish
}

// Own stores acknowledged by the memory side, then the workgroup meets, then the flag.
__device__ __forceinline__ void flow_publish(const FlowArgs& a, uint32_t* flag)
{
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __syncthreads();
    if (threadIdx.x == 0) coherent_st<uint32_t>(flag, a.epoch);
}

// One chunk of n 16-byte vectors, both ends on the 16-byte grid.
__device__ __forceinline__ void coherent_copy_vectors(const u32x4* __restrict__ s, u32x4* __restrict__ d, uint32_t n)
{
    uint32_t v = 0;
    for (; n - v >= 4u * WG; v += 4u * WG) {  // whole groups: four vectors per lane in flight
        const uint32_t l = v + threadIdx.x;
        u32x4 x0, x1, x2, x3;
        coherent_ld4(s + l, s + l + WG, s + l + 2 * WG, s + l + 3 * WG, x0, x1, x2, x3);
        coherent_st<u32x4>(d + l, x0);
        coherent_st<u32x4>(d + l + WG, x1);
        coherent_st<u32x4>(d + l + 2 * WG, x2);
        coherent_st<u32x4>(d + l + 3 * WG, x3);
    }
    for (v += threadIdx.x; v < n; v += WG) coherent_st<u32x4>(d + v, coherent_ld<u32x4>(s + v));
}

// The phase that copy ordinal k (counted over the call) belongs to: the last one that starts at or before k.
__device__ __forceinline__ uint32_t phase_of_copy(const DevPhase* __restrict__ phases, uint32_t nphases, uint32_t k)
{
    uint32_t lo = 0, hi = nphases - 1;
    while (lo < hi) {
        const uint32_t mid = (lo + hi + 1) >> 1;
        if (phases[mid].copies_before <= k) lo = mid; else hi = mid - 1;
    }
    return lo;
}

// One workgroup per item.  REALIGN (with V = uint8_t): chunks of blocks that are off the 16-byte grid move through
// coherent_realign_chunk.
template <typename V, bool REALIGN = false>
__global__ __launch_bounds__(WG) void dataflow_kernel(const FlowArgs a)
{
    const uint32_t vpb = uint32_t(a.block_bytes / sizeof(V));
    const uint32_t item = blockIdx.x;
    if (item >= a.total_items) return;
    const uint32_t k = item / a.chunks_per_block;  // copy ordinal within the call
    const uint32_t q = item - k * a.chunks_per_block;
    const DevPhase P = a.phases[phase_of_copy(a.phases, a.nphases, k)];
    const Copy cp = a.copies[P.first_copy + (k - P.copies_before)];
    const uint32_t v0 = q * a.chunk_vecs;
    if (v0 >= vpb) return;  // uniform; only with pieces of a few vectors, where rounding them up can use the block up early
    const uint32_t v1 = (q + 1 == a.chunks_per_block || vpb - v0 < a.chunk_vecs) ? vpb : v0 + a.chunk_vecs;
    // Sources that were complete before the launch need no wait: the send buffer, and in an in-place call
    // the own slot of every rank (block index rank * p + rank of the receive buffer).
    const bool own_slot = a.in_place != 0 && P.src_buf == BUF_RECV && cp.src_block / a.p == cp.src_block % a.p;
    if (P.src_buf != BUF_SEND && !own_slot &&
        !flow_wait(a, a.flags + (P.src_buf == BUF_WORK ? a.flags_per_buf : 0u) + cp.src_block * a.chunks_per_block + q))
        return;  // uniform: the whole workgroup leaves
    const V* __restrict__ s = reinterpret_cast<const V*>(a.base[P.src_buf] + uint64_t(cp.src_block) * a.block_bytes);
    V* __restrict__ d = reinterpret_cast<V*>(const_cast<uint8_t*>(a.base[P.dst_buf]) + uint64_t(cp.dst_block) * a.block_bytes);
    if constexpr (REALIGN) {
        static_assert(sizeof(V) == 1, "chunk bounds are byte offsets");
        coherent_realign_chunk(reinterpret_cast<const uint8_t*>(s) + v0, reinterpret_cast<uint8_t*>(d) + v0, v1 - v0);
    } else if constexpr (sizeof(V) == 16) {
        coherent_copy_vectors(s + v0, d + v0, v1 - v0);
    } else {
        constexpr int U = 8;
        for (uint32_t v = v0 + threadIdx.x; v < v1; v += WG * U) {
            V x[U];
#pragma unroll
            for (int u = 0; u < U; ++u)
                if (v + u * WG < v1) x[u] = coherent_ld<V>(s + v + u * WG);
#pragma unroll
            for (int u = 0; u < U; ++u)
                if (v + u * WG < v1) coherent_st<V>(d + v + u * WG, x[u]);
        }
    }
    flow_publish(a, a.flags + (P.dst_buf == BUF_WORK ? a.flags_per_buf : 0u) + cp.dst_block * a.chunks_per_block + q);
}

// ---------------------------------------------------------------------------
// The dataflow form for blocks of different sizes (Allgatherv): same items,
// flags and waits; a copy's offsets and length come from its slot's entry in
// the call's count and displacement arrays.  Every copy is given the chunk
// count of the longest block; the items past the end of a shorter block have
// nothing to move and nobody waits for them.  ON_GRID: every offset and length
// is a multiple of 16.
// ---------------------------------------------------------------------------
struct FlowVarArgs {
    FlowArgs f;              // block_bytes unused; chunk_vecs = chunk size in bytes
    const uint64_t* counts;  // [p] bytes per slot
    const uint64_t* displs;  // [p] byte offset of a slot in a receive buffer (and of a rank's block in the send buffer)
    uint64_t row_bytes;
};

template <bool ON_GRID>
__global__ __launch_bounds__(WG) void dataflow_var_kernel(const FlowVarArgs va)
{
    const FlowArgs& a = va.f;
    const uint32_t item = blockIdx.x;
    if (item >= a.total_items) return;
    const uint32_t k = item / a.chunks_per_block;
    const uint32_t q = item - k * a.chunks_per_block;
    const DevPhase P = a.phases[phase_of_copy(a.phases, a.nphases, k)];
    const Copy cp = a.copies[P.first_copy + (k - P.copies_before)];
    const uint32_t dst_rank = cp.dst_block / a.p, slot = cp.dst_block - dst_rank * a.p;
    const uint64_t len = va.counts[slot];
    // The block's own number of pieces: round(len / chunk), at least one, at most what the longest block has.
    uint64_t npieces = (len + a.chunk_vecs / 2) / a.chunk_vecs;
    npieces = npieces > a.chunks_per_block ? a.chunks_per_block : (npieces ? npieces : (len ? 1u : 0u));
    if (q >= npieces) return;  // uniform: this block has no piece q
    const uint64_t piece = ((len + npieces - 1) / npieces + 15) / 16 * 16;  // equal pieces, whole 16-byte vectors
    const uint64_t at = uint64_t(q) * piece;
    if (at >= len) return;
    const uint32_t n = uint32_t((q + 1 == npieces || len - at < piece ? len : at + piece) - at);  // below 1.5 chunks
    const bool own_slot = a.in_place != 0 && P.src_buf == BUF_RECV && cp.src_block / a.p == cp.src_block % a.p;
    if (P.src_buf != BUF_SEND && !own_slot && !flow_wait(a, a.flags + cp.src_block * a.chunks_per_block + q)) return;
    const uint64_t src_off = P.src_buf == BUF_SEND
                                 ? va.displs[cp.src_block]
                                 : uint64_t(cp.src_block / a.p) * va.row_bytes + va.displs[cp.src_block % a.p];
    const uint8_t* __restrict__ s = a.base[P.src_buf] + src_off + at;
    uint8_t* __restrict__ d = const_cast<uint8_t*>(a.base[P.dst_buf]) + uint64_t(dst_rank) * va.row_bytes + va.displs[slot] + at;
    if constexpr (ON_GRID)
        coherent_copy_vectors(reinterpret_cast<const u32x4*>(s), reinterpret_cast<u32x4*>(d), n >> 4);
    else
        coherent_realign_chunk(s, d, n);
    flow_publish(a, a.flags + cp.dst_block * a.chunks_per_block + q);
}

}  // namespace sparbit
