// C-ABI of the library: argument checks, per-device caches of the schedule
// tables, and the launches.  See include/sparbit.h for the contract.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <atomic>
#include <cstdarg>
#include <cstdio>
#include <cstring>
#include <map>
#include <memory>
#include <mutex>
#include <new>
#include <utility>
#include <vector>

#include "../../include/sparbit.h"
#include "kernels.hip.hpp"
#include "plan.hpp"

// Table memory of sparbit_allgather_static, the entry point that allocates nothing: room for the p own-block
// copies and the p (p - 1) forwarding copies of a Sparbit call with p <= SPARBIT_STATIC_MAX_P.  Every GPU the
// library runs on holds its own copy of this array, at its own address, until the process ends.  In host code the
// name below is only a handle for hipGetSymbolAddress; the address it yields (per device) is what kernels get.
static __device__ __align__(256) unsigned char scratch[size_t(SPARBIT_STATIC_MAX_P) * SPARBIT_STATIC_MAX_P * sizeof(sparbit::Copy)];

namespace sparbit {
namespace {

thread_local int tl_last_hip_error = 0;

// What the current call of this thread has enqueued so far (sparbit_last_launch_info).
struct LaunchInfo {
    int launches = 0;
    uint64_t most_bytes = 0;
    char kernel[256] = "";
};
thread_local LaunchInfo tl_launch_info;

template <typename V>
constexpr const char* type_label()
{
    if constexpr (sizeof(V) == 16) return "unsigned int __vector(4)";
    else if constexpr (sizeof(V) == 8) return "unsigned long";
    else if constexpr (sizeof(V) == 4) return "unsigned int";
    else return "unsigned char";
}

constexpr const char* bool_label(bool b) { return b ? "true" : "false"; }

// Records one launch that moves `bytes`; the name is kept if no earlier launch of the call moved more.
__attribute__((format(printf, 2, 3))) void note_launch(uint64_t bytes, const char* fmt, ...)
{
    LaunchInfo& li = tl_launch_info;
    ++li.launches;
    if (bytes < li.most_bytes || (li.launches > 1 && bytes == li.most_bytes)) return;
    li.most_bytes = bytes;
    va_list ap;
    va_start(ap, fmt);
    std::vsnprintf(li.kernel, sizeof li.kernel, fmt, ap);
    va_end(ap);
}

#define SB_HIP(expr)                                    \
    do {                                                \
        hipError_t e_ = (expr);                         \
        if (e_ != hipSuccess) {                         \
            tl_last_hip_error = int(e_);                \
            (void)hipGetLastError();                    \
            return SPARBIT_ERR_HIP;                     \
        }                                               \
    } while (0)

// True while `stream` records into a HIP graph.  A recorded call is replayed with the arguments it had at
// capture time and possibly next to other replays, so it may not allocate, may not build tables, and may not
// use the kernels that wait on themselves through per-stream device state.
bool stream_is_capturing(hipStream_t stream)
{
    hipStreamCaptureStatus status = hipStreamCaptureStatusNone;
    if (hipStreamIsCapturing(stream, &status) != hipSuccess) {
        (void)hipGetLastError();
        return false;
    }
    return status != hipStreamCaptureStatusNone;
}

// The C ABI never throws: host allocation failures inside the library become an error code.
template <typename F>
int no_throw(F&& body)
{
    try {
        return body();
    } catch (const std::bad_alloc&) {
        return SPARBIT_ERR_NOMEM;
    } catch (...) {
        return SPARBIT_ERR_NOMEM;
    }
}

// ---- tuning knobs ----------------------------------------------------------
std::atomic<long long> g_wg_threads{0};                       // lanes per workgroup of the tile kernel; 0 = by block size
std::atomic<long long> g_unroll{1};                           // vectors per lane of the tile kernel (2 and 4 only with 256 lanes)
std::atomic<long long> g_interleave_log2{3};                  // copies interleaved over consecutive workgroups: 2^3 = one per XCD
std::atomic<long long> g_nontemporal{1};
std::atomic<long long> g_persistent_max_bytes{4ll << 10};     // AUTO uses the persistent kernel up to this p*p*B
std::atomic<long long> g_dataflow_max_items{256};             // AUTO uses the dataflow kernel up to this many work items
std::atomic<long long> g_hybrid_max_items{512};               // AUTO: leading steps with at most this many items share one dataflow launch
std::atomic<long long> g_flow_chunk_bytes{16384};             // unit of work (and of readiness) of the dataflow kernel
std::atomic<long long> g_wgs_per_cu{1};
std::atomic<long long> g_spin_limit_ms{2000};
std::atomic<long long> g_line_align_min_bytes{64ll << 10};    // 16-byte-aligned blocks at least this long, off the 128-byte grid: same
std::atomic<long long> g_var_idle_max{131072};                // Allgatherv: idle workgroups one launch per step may cost before size classes pay
std::atomic<long long> g_realign_min_bytes{512};
std::atomic<long long> g_tree_auto{1};                        // AUTO runs Sparbit as the tree kernel where it applies
std::atomic<long long> g_tree_auto_doubling{1};               // ... and whole Recursive Doubling calls too
std::atomic<long long> g_tree_auto_ring{1};                   // ... and whole Ring calls (a chain per block)
std::atomic<long long> g_tree_gang_apart_log2{-1};            // ... 2^this KiB apart (-1: by the call)
std::atomic<long long> g_tree_gang{-1};                       // gangs of wavefronts: -1 = by size, 0 = never, 1 or 4 = gangs of 4 wherever the form allows, 8 = of 8 where they exist
std::atomic<long long> g_tree_hot{-1};                        // plain stores with forwarders read back at once: -1 = by size, 0 = never, 1 = always
std::atomic<long long> g_tree_team_log2{-1};                  // small calls: 2^this wavefronts share a tree's piece; -1 = by size
std::atomic<long long> g_tree_run_log2{-1};                   // tree kernel: relative ranks are walked in runs of 2^this; -1 = by size
std::atomic<long long> g_tree_small_bytes{96ll << 20};        // p*p*B up to this: the tree kernel walks in step order instead
std::atomic<long long> g_tree_unroll{1};                      // vectors per lane of the tree kernel (1, 2 or 4)
std::atomic<long long> g_tree_store{2};                       // its stores: 0 plain, 2 write-through, 3 by destination
std::atomic<long long> g_tree_prefetch{1};                    // it loads the next run's first rank ahead
std::atomic<long long> g_tree_any_align{1};                   // blocks of 512 bytes and more off the 128-byte grid: the any-alignment tree form
std::atomic<long long> g_tree_part_line_max_bytes{512ll << 20};  // ... with rows off that grid only for calls up to this size
std::atomic<long long> g_tree_lds_bytes{-1};                  // LDS each of its wavefronts reserves (unused: caps the wavefronts per CU); -1 = by size              // blocks at least this long, not 16-byte aligned: realigning kernel

struct DevicePlan {
    Plan host;
    Copy* d_copies = nullptr;
    DevPhase* d_phases = nullptr;          // phases of an out-of-place call
    DevPhase* d_phases_in_place = nullptr; // phases of an in-place call
    std::vector<uint32_t> first_copy;      // per host phase
    std::vector<DevPhase> out_of_place, in_place;
    DevicePlan() = default;
    DevicePlan(const DevicePlan&) = delete;
    DevicePlan& operator=(const DevicePlan&) = delete;
    ~DevicePlan()  // the owning device is current when plans are destroyed (finalize, or a failed build)
    {
        (void)hipFree(d_copies);
        (void)hipFree(d_phases);
        (void)hipFree(d_phases_in_place);
    }
};

// Per-stream state of the two kernels that wait on themselves (dataflow: ready flags; persistent: barrier).
struct StreamState {
    FlowState* flow = nullptr;
    uint32_t* flags = nullptr;
    size_t flag_capacity = 0;
    uint32_t epoch = 0;  // last dataflow call number handed out (0 is never used: fresh flags are 0)
    BarrierState* barrier = nullptr;
    // Two words of pinned host memory that the device writes when a bounded wait expires ([0] dataflow: the call's
    // number, [1] persistent: the stream's count of aborted launches), and the values the host has reported so far.
    uint32_t* note = nullptr;
    uint32_t* note_dev = nullptr;  // the same words as the device addresses them
    uint32_t reported[2] = {0, 0};
};

// Allgatherv: explicit byte-offset copy lists for one (schedule, p, counts, displs, row_bytes).
struct VarPhase {
    Buffer src_buf, dst_buf;
    uint32_t first, ncopies;
    uint64_t max_len;
    uint32_t host_phase;  // index of the schedule phase these copies belong to
};

struct VarPlan {
    int algo = 0, p = 0;
    size_t row_bytes = 0;
    std::vector<size_t> counts, displs;
    std::vector<VarPhase> out_of_place, in_place;
    VarCopy* d_copies = nullptr;
    uint64_t* d_geometry = nullptr;  // counts[p], then displs[p]: what the dataflow form reads
    uint64_t max_count = 0;
    uint64_t last_use = 0;
    VarPlan() = default;
    VarPlan(const VarPlan&) = delete;
    VarPlan& operator=(const VarPlan&) = delete;
    ~VarPlan()
    {
        (void)hipFree(d_copies);
        (void)hipFree(d_geometry);
    }
};

struct DeviceState {
    int device = -1;
    int num_cus = 0;
    std::map<const void*, int> occupancy;              // resident workgroups per CU, per kernel
    std::vector<std::unique_ptr<VarPlan>> var_plans;  // small most-recently-used cache
    uint64_t var_clock = 0;
    std::map<hipStream_t, StreamState> streams;
    std::map<std::pair<int, int>, std::unique_ptr<DevicePlan>> plans;  // (algo, p)
    void* work = nullptr;  // Bruck's rotated working buffer
    size_t work_bytes = 0;
    Copy* static_tables = nullptr;  // this device's address of `scratch` (sparbit_allgather_static)
};

std::mutex g_mutex;
std::map<int, std::unique_ptr<DeviceState>> g_devices;
std::atomic<int> g_stream_states{0};  // how many StreamState objects hold note words (0: nothing can have expired)

int get_device_state(DeviceState** out)
{
    int dev = 0;
    SB_HIP(hipGetDevice(&dev));
    auto it = g_devices.find(dev);
    if (it == g_devices.end()) {
        auto st = std::make_unique<DeviceState>();
        st->device = dev;
        // Attribute query, not hipGetDeviceProperties: the property struct's
        // layout differs between HIP releases and the process may carry another
        // runtime version than the headers this file was compiled with.
        SB_HIP(hipDeviceGetAttribute(&st->num_cus, hipDeviceAttributeMultiprocessorCount, dev));
        it = g_devices.emplace(dev, std::move(st)).first;
    }
    *out = it->second.get();
    return SPARBIT_OK;
}

int get_plan(DeviceState* ds, int algo, int p, bool may_build, DevicePlan** out)
{
    auto key = std::make_pair(algo, p);
    auto it = ds->plans.find(key);
    if (it != ds->plans.end()) {
        *out = it->second.get();
        return SPARBIT_OK;
    }
    if (!may_build) return SPARBIT_ERR_UNSUPPORTED;  // stream capture: the tables must exist already
    auto dp = std::make_unique<DevicePlan>();
    int rc = build_plan(p, algo, dp->host);
    if (rc != SPARBIT_OK) return rc;
    std::vector<Copy> all;
    for (const Phase& ph : dp->host.phases) {
        dp->first_copy.push_back(uint32_t(all.size()));
        all.insert(all.end(), ph.copies.begin(), ph.copies.end());
        DevPhase d{dp->first_copy.back(), uint32_t(ph.copies.size()), int32_t(ph.src_buf), int32_t(ph.dst_buf), 0u, 0u};
        if (d.ncopies == 0) continue;
        auto append = [&d](std::vector<DevPhase>& list) {
            d.copies_before = list.empty() ? 0u : list.back().copies_before + list.back().ncopies;
            list.push_back(d);
        };
        if (!ph.only_in_place && !ph.covered_by_fused) append(dp->out_of_place);
        if (!ph.skip_in_place) append(dp->in_place);
    }
    if (!all.empty()) {
        SB_HIP(hipMalloc(reinterpret_cast<void**>(&dp->d_copies), all.size() * sizeof(Copy)));
        SB_HIP(hipMemcpy(dp->d_copies, all.data(), all.size() * sizeof(Copy), hipMemcpyHostToDevice));
    }
    auto upload = [](const std::vector<DevPhase>& v, DevPhase** d) -> int {
        if (v.empty()) return SPARBIT_OK;
        SB_HIP(hipMalloc(reinterpret_cast<void**>(d), v.size() * sizeof(DevPhase)));
        SB_HIP(hipMemcpy(*d, v.data(), v.size() * sizeof(DevPhase), hipMemcpyHostToDevice));
        return SPARBIT_OK;
    };
    if ((rc = upload(dp->out_of_place, &dp->d_phases)) != SPARBIT_OK) return rc;
    if ((rc = upload(dp->in_place, &dp->d_phases_in_place)) != SPARBIT_OK) return rc;
    *out = dp.get();
    ds->plans.emplace(key, std::move(dp));
    return SPARBIT_OK;
}

// The first self-waiting launch on a stream allocates that stream's state (device memory and two pinned host words)
// and synchronises the device once; growing the flag array synchronises the stream.
int get_stream_state(DeviceState* ds, hipStream_t stream, StreamState** out)
{
    StreamState& ss = ds->streams[stream];
    if (!ss.note) {
        void* host = nullptr;
        SB_HIP(hipHostMalloc(&host, 2 * sizeof(uint32_t), hipHostMallocDefault));
        std::memset(host, 0, 2 * sizeof(uint32_t));
        void* dev = nullptr;
        if (hipHostGetDevicePointer(&dev, host, 0) != hipSuccess) {
            (void)hipGetLastError();
            (void)hipHostFree(host);
            return SPARBIT_ERR_HIP;
        }
        ss.note = static_cast<uint32_t*>(host);
        ss.note_dev = static_cast<uint32_t*>(dev);
        g_stream_states.fetch_add(1);
    }
    *out = &ss;
    return SPARBIT_OK;
}

int get_barrier(DeviceState* ds, hipStream_t stream, StreamState** out)
{
    StreamState* ss = nullptr;
    int rc = get_stream_state(ds, stream, &ss);
    if (rc != SPARBIT_OK) return rc;
    if (!ss->barrier) {
        SB_HIP(hipMalloc(reinterpret_cast<void**>(&ss->barrier), sizeof(BarrierState)));
        SB_HIP(hipMemset(ss->barrier, 0, sizeof(BarrierState)));
        SB_HIP(hipDeviceSynchronize());
    }
    *out = ss;
    return SPARBIT_OK;
}

int get_flow(DeviceState* ds, hipStream_t stream, size_t nflags, StreamState** out)
{
    StreamState* ss = nullptr;
    int rc = get_stream_state(ds, stream, &ss);
    if (rc != SPARBIT_OK) return rc;
    if (!ss->flow) {
        SB_HIP(hipMalloc(reinterpret_cast<void**>(&ss->flow), sizeof(FlowState)));
        SB_HIP(hipMemset(ss->flow, 0, sizeof(FlowState)));
        SB_HIP(hipDeviceSynchronize());
    }
    if (ss->flag_capacity < nflags) {
        if (ss->flags) {
            SB_HIP(hipStreamSynchronize(stream));
            SB_HIP(hipFree(ss->flags));
            ss->flags = nullptr;
            ss->flag_capacity = 0;
        }
        SB_HIP(hipMalloc(reinterpret_cast<void**>(&ss->flags), nflags * sizeof(uint32_t)));
        SB_HIP(hipMemset(ss->flags, 0, nflags * sizeof(uint32_t)));
        SB_HIP(hipDeviceSynchronize());
        ss->flag_capacity = nflags;
        // The call numbers go on counting: fresh flags are 0, which no call uses, and a number that an expired
        // wait of an earlier call left in FlowState::abort can then never be handed out again before the wrap.
    }
    *out = ss;
    return SPARBIT_OK;
}

// The number of the next call on this stream; flags hold the number of the call that last set them, 0 = never.
// After 2^32 calls the numbers start over, so the flags are cleared first (in stream order, ahead of the launch
// that uses the new number; a dataflow launch is never recorded into a graph, so the memset is not either).
int next_epoch(StreamState* ss, hipStream_t stream, uint32_t* epoch)
{
    if (++ss->epoch == 0) {
        SB_HIP(hipMemsetAsync(ss->flags, 0, ss->flag_capacity * sizeof(uint32_t), stream));
        SB_HIP(hipMemsetAsync(&ss->flow->abort, 0, sizeof(uint32_t), stream));
        ss->epoch = 1;
    }
    *epoch = ss->epoch;
    return SPARBIT_OK;
}

// SPARBIT_ERR_TIMEOUT once for every self-waiting launch on `stream` that ended with an expired wait since the
// last report.  Reads two words of host memory; no synchronisation.
int report_expired_waits(hipStream_t stream)
{
    if (g_stream_states.load() == 0) return SPARBIT_OK;
    std::lock_guard<std::mutex> lock(g_mutex);
    int dev = 0;
    SB_HIP(hipGetDevice(&dev));
    auto d = g_devices.find(dev);
    if (d == g_devices.end()) return SPARBIT_OK;
    auto it = d->second->streams.find(stream);
    if (it == d->second->streams.end() || !it->second.note) return SPARBIT_OK;
    StreamState& ss = it->second;
    bool moved = false;
    for (int i = 0; i < 2; ++i) {
        const uint32_t now = __atomic_load_n(&ss.note[i], __ATOMIC_RELAXED);
        if (now != ss.reported[i]) {
            ss.reported[i] = now;
            moved = true;
        }
    }
    return moved ? SPARBIT_ERR_TIMEOUT : SPARBIT_OK;
}

int get_work(DeviceState* ds, size_t bytes, bool may_allocate, void** out)
{
    if (ds->work_bytes < bytes) {
        if (!may_allocate) return SPARBIT_ERR_UNSUPPORTED;
        if (ds->work) {
            SB_HIP(hipDeviceSynchronize());
            SB_HIP(hipFree(ds->work));
            ds->work = nullptr;
            ds->work_bytes = 0;
        }
        SB_HIP(hipMalloc(&ds->work, bytes));
        ds->work_bytes = bytes;
    }
    *out = ds->work;
    return SPARBIT_OK;
}

// Widest access the pointers and the block size allow.
int access_width(const void* a, const void* b, const void* c, size_t block_bytes)
{
    uintptr_t bits = uintptr_t(a) | uintptr_t(b) | uintptr_t(c) | uintptr_t(block_bytes);
    if ((bits & 15) == 0) return 16;
    if ((bits & 3) == 0) return 4;
    return 1;
}

// Grid of one tile of T vectors per workgroup for `ncopies` copies of at most `max_vecs` vectors each, copies dealt
// round-robin in groups of 2^lg_g to consecutive workgroups.  Blocks with more tiles than the x extent allows get
// the largest extent and *capped = true (the kernels that accept such a grid loop).  False if the copies do not
// fit a grid at all.
bool tile_grid(uint64_t max_vecs, uint32_t ncopies, int T, dim3* grid, uint32_t* lg_g_out, bool* capped)
{
    uint64_t tiles = (max_vecs + uint64_t(T) - 1) / uint64_t(T);
    if (tiles == 0) tiles = 1;
    uint32_t lg_g = uint32_t(g_interleave_log2.load());
    while (lg_g > 0 && (1u << lg_g) > ncopies) --lg_g;  // a short phase has fewer copies than XCDs
    const uint32_t groups = (ncopies + (1u << lg_g) - 1) >> lg_g;
    const uint32_t gy = groups < 32768u ? groups : 32768u;
    const uint32_t gz = (groups + gy - 1) / gy;
    if (gz > 65535u) return false;
    const uint64_t max_tiles = (0x7fffffffull / uint64_t(T)) >> lg_g;  // grid x extent stays below 2^31 lanes
    *capped = tiles > max_tiles;
    if (*capped) tiles = max_tiles;
    *grid = dim3(uint32_t(tiles << lg_g), gy, gz);
    *lg_g_out = lg_g;
    return true;
}

template <typename V, typename Index, int T, int U>
int launch_tiles(const uint8_t* src, uint8_t* dst, const Copy* copies, uint32_t ncopies, size_t B, bool nt,
                 hipStream_t stream)
{
    const uint64_t vpb = B / sizeof(V);
    dim3 grid;
    uint32_t lg_g = 0;
    bool loop = false;  // blocks with more tiles than the grid holds: the kernel takes several trips
    if (!tile_grid((vpb + U - 1) / U, ncopies, T, &grid, &lg_g, &loop)) return SPARBIT_ERR_ARG;
    const bool plain_nt = nt && ((uintptr_t(dst) | uintptr_t(B)) & 127) != 0;
    note_launch(uint64_t(ncopies) * B, "sparbit::copy_tiles_kernel<%s, %s, %d, %d, %s, %s, %s>", type_label<V>(),
                type_label<Index>(), T, U, bool_label(loop || nt), bool_label(loop), bool_label(loop || !plain_nt));
    if (loop)
        hipLaunchKernelGGL((copy_tiles_kernel<V, Index, T, U, true, true>), grid, dim3(T), 0, stream, src, dst, copies,
                           ncopies, uint64_t(B), lg_g);
    else if (nt && ((uintptr_t(dst) | uintptr_t(B)) & 127) != 0)
        // Destinations off the 128-byte grid: write-through stores cover lines piecewise there and lose to the
        // plain non-temporal hint (p = 128, B = 4 KiB + 16: 53.5 against 48.9 us per call).
        hipLaunchKernelGGL((copy_tiles_kernel<V, Index, T, U, true, false, false>), grid, dim3(T), 0, stream, src, dst,
                           copies, ncopies, uint64_t(B), lg_g);
    else if (nt)
        hipLaunchKernelGGL((copy_tiles_kernel<V, Index, T, U, true, false>), grid, dim3(T), 0, stream, src, dst,
                           copies, ncopies, uint64_t(B), lg_g);
    else
        hipLaunchKernelGGL((copy_tiles_kernel<V, Index, T, U, false, false>), grid, dim3(T), 0, stream, src, dst,
                           copies, ncopies, uint64_t(B), lg_g);
    SB_HIP(hipGetLastError());
    return SPARBIT_OK;
}

template <typename V>
int launch_flat(const uint8_t* src, uint8_t* dst, const Copy* copies, uint32_t ncopies, size_t B, bool nt,
                hipStream_t stream)
{
    constexpr int U = 4;
    const uint32_t vpb = uint32_t(B / sizeof(V));  // < 64 here
    const uint64_t total = uint64_t(vpb) * ncopies;
    const uint64_t ntiles = (total + WG * U - 1) / (WG * U);
    if (total + WG * U > 0xffffffffull) return SPARBIT_ERR_ARG;  // cannot happen: ncopies < 2^25, vpb < 64
    note_launch(uint64_t(ncopies) * B, "sparbit::copy_flat_kernel<%s, unsigned int, %d, %s>", type_label<V>(), U, bool_label(nt));
    if (nt)
        hipLaunchKernelGGL((copy_flat_kernel<V, uint32_t, U, true>), dim3(uint32_t(ntiles)), dim3(WG), 0, stream, src,
                           dst, copies, uint64_t(B), vpb, uint32_t(total));
    else
        hipLaunchKernelGGL((copy_flat_kernel<V, uint32_t, U, false>), dim3(uint32_t(ntiles)), dim3(WG), 0, stream, src,
                           dst, copies, uint64_t(B), vpb, uint32_t(total));
    SB_HIP(hipGetLastError());
    return SPARBIT_OK;
}

template <int T>
int launch_realign_t(const uint8_t* src, uint8_t* dst, const Copy* copies, uint32_t ncopies, size_t B, bool nt,
                     hipStream_t stream)
{
    dim3 grid;
    uint32_t lg_g = 0;
    bool capped = false;  // the kernel loops, so a capped grid is fine
    if (!tile_grid(B >> 4, ncopies, T, &grid, &lg_g, &capped)) return SPARBIT_ERR_ARG;
    note_launch(uint64_t(ncopies) * B, "sparbit::copy_tiles_realign_kernel<%d, %s>", T, bool_label(nt));
    if (nt)
        hipLaunchKernelGGL((copy_tiles_realign_kernel<T, true>), grid, dim3(T), 0, stream, src, dst, copies, ncopies,
                           uint64_t(B), lg_g);
    else
        hipLaunchKernelGGL((copy_tiles_realign_kernel<T, false>), grid, dim3(T), 0, stream, src, dst, copies, ncopies,
                           uint64_t(B), lg_g);
    SB_HIP(hipGetLastError());
    return SPARBIT_OK;
}

int launch_realign(const uint8_t* src, uint8_t* dst, const Copy* copies, uint32_t ncopies, size_t B, bool nt,
                   hipStream_t stream)
{
    const uint64_t vecs = B >> 4;
    if (vecs <= 64) return launch_realign_t<64>(src, dst, copies, ncopies, B, nt, stream);
    if (vecs <= 128) return launch_realign_t<128>(src, dst, copies, ncopies, B, nt, stream);
    return launch_realign_t<256>(src, dst, copies, ncopies, B, nt, stream);
}

// Picks the workgroup size (no wider than the block, no wider than the "wg_threads" knob) and the index width.
template <typename V>
int launch_phase_v(const uint8_t* src, uint8_t* dst, const Copy* copies, uint32_t ncopies, size_t B, bool nt,
                   hipStream_t stream)
{
    const uint64_t vpb = B / sizeof(V);
    // Blocks shorter than one wavefront.  A tile per block leaves lanes idle and costs one workgroup per
    // block; flattened tiles keep the lanes busy and neighbouring blocks' writes coalesced, but every lane pays
    // a division and a table look-up.  Measured: with byte-wide accesses flattened tiles always win (p = 253,
    // B = 1: 43 us against 147 us); with 16-byte vectors a tile per block wins until a launch holds tens of
    // thousands of blocks (p = 125, B = 16..512: 31 us against 40 us per call; one launch of 65536 16-byte
    // blocks: 33 us against 14.5 us).
    if (vpb < 64 && (sizeof(V) < 16 || ncopies >= 16384u)) return launch_flat<V>(src, dst, copies, ncopies, B, nt, stream);
    if (2 * vpb > 0xffffffffull)  // lane index plus a grid-wide stride must not wrap
        return launch_tiles<V, uint64_t, 256, 1>(src, dst, copies, ncopies, B, nt, stream);
    long long t = g_wg_threads.load();
    // One wavefront per workgroup (1 KiB tiles) is 0.5-2.5 % ahead of four for 16-byte vectors and blocks of
    // 8 KiB .. 4 MiB (p = 128, B = 1 MiB: 5.128 against 5.160 ms per call); shorter blocks (more workgroups than
    // the launch can hide) and 16 MiB blocks are 1-2 % better off with 256 lanes.
    // Phases that read the send buffer (own-block placement, DIRECT) re-read a small, cache-resident source and
    // are bound by their stores; there four times as many workgroups only cost dispatch time (DIRECT, p = 32,
    // B = 512 KiB: 116 us with 64 lanes, 77 us with 256), so the rule is for forwarding steps only.
    if (t == 0) t = (sizeof(V) == 16 && B >= 8192 && B <= (size_t(4) << 20) && src == dst) ? 64 : 256;
    while (t > 64 && uint64_t(t / 2) >= vpb) t /= 2;
    const int u = int(g_unroll.load());
    if (u == 4 && t == 256) return launch_tiles<V, uint32_t, 256, 4>(src, dst, copies, ncopies, B, nt, stream);
    if (u == 2 && t == 256) return launch_tiles<V, uint32_t, 256, 2>(src, dst, copies, ncopies, B, nt, stream);
    switch (t) {
    case 64: return launch_tiles<V, uint32_t, 64, 1>(src, dst, copies, ncopies, B, nt, stream);
    case 128: return launch_tiles<V, uint32_t, 128, 1>(src, dst, copies, ncopies, B, nt, stream);
    case 512: return launch_tiles<V, uint32_t, 512, 1>(src, dst, copies, ncopies, B, nt, stream);
    case 1024: return launch_tiles<V, uint32_t, 1024, 1>(src, dst, copies, ncopies, B, nt, stream);
    default: return launch_tiles<V, uint32_t, 256, 1>(src, dst, copies, ncopies, B, nt, stream);
    }
}

// One phase as one launch.
int launch_phase(const uint8_t* src, uint8_t* dst, const Copy* copies, uint32_t ncopies, size_t B, int width,
                 hipStream_t stream)
{
    if (ncopies == 0) return SPARBIT_OK;
    const bool nt = g_nontemporal.load() != 0;
    if (width < 16 && B >= size_t(g_realign_min_bytes.load()))
        return launch_realign(src, dst, copies, ncopies, B, nt, stream);
    // Blocks on the 16-byte grid whose destinations do not all start on a 128-byte line: the tile kernel's
    // write-through stores would cover lines piecewise, which costs up to 20 % from 64 KiB blocks on (p = 128,
    // B = 256 KiB + 16: 4.64 TB/s against 5.85 TB/s through the realigning kernel, whose stores cover whole lines).
    if (((uintptr_t(dst) | uintptr_t(B)) & 127) != 0 && B >= size_t(g_line_align_min_bytes.load()))
        return launch_realign(src, dst, copies, ncopies, B, nt, stream);
    switch (width) {
    case 16: return launch_phase_v<u32x4>(src, dst, copies, ncopies, B, nt, stream);
    case 4: return launch_phase_v<uint32_t>(src, dst, copies, ncopies, B, nt, stream);
    default: return launch_phase_v<uint8_t>(src, dst, copies, ncopies, B, nt, stream);
    }
}

// Workgroups of `kernel` (WG lanes, no dynamic LDS) that fit on one compute unit; asked once per device.
template <typename Kernel>
int resident_per_cu(DeviceState* ds, Kernel kernel, int* out)
{
    const void* key = reinterpret_cast<const void*>(kernel);
    auto it = ds->occupancy.find(key);
    if (it == ds->occupancy.end()) {
        int n = 0;
        SB_HIP(hipOccupancyMaxActiveBlocksPerMultiprocessor(&n, kernel, WG, 0));
        it = ds->occupancy.emplace(key, n).first;
    }
    *out = it->second;
    return SPARBIT_OK;
}

// A grid of more than one workgroup meets at device-wide barriers, so all of it must be resident at once: it goes
// out as a cooperative launch, which the runtime co-schedules or refuses.  A single workgroup needs no such care.
template <typename V>
int launch_persistent_v(const PersistentArgs& a, DeviceState* ds, uint64_t max_tiles, hipStream_t stream)
{
    constexpr int U = 4;
    const int num_cus = ds->num_cus;
    const bool nt = g_nontemporal.load() != 0;
    int per_cu = 0;
    int rc = nt ? resident_per_cu(ds, persistent_kernel<V, U, true>, &per_cu)
                : resident_per_cu(ds, persistent_kernel<V, U, false>, &per_cu);
    if (rc != SPARBIT_OK) return rc;
    long long want = g_wgs_per_cu.load();
    if (want < 1) want = 1;
    if (per_cu < 1) return SPARBIT_ERR_HIP;
    if (want > per_cu) want = per_cu;
    uint64_t grid = uint64_t(num_cus) * uint64_t(want);
    if (grid > max_tiles) grid = max_tiles ? max_tiles : 1;  // no more workgroups than the largest phase has tiles
    note_launch(max_tiles * uint64_t(WG * U) * sizeof(V), "sparbit::persistent_kernel<%s, %d, %s>", type_label<V>(), U, bool_label(nt));
    const void* fn = nt ? reinterpret_cast<const void*>(persistent_kernel<V, U, true>)
                        : reinterpret_cast<const void*>(persistent_kernel<V, U, false>);
    if (grid == 1) {
        if (nt)
            hipLaunchKernelGGL((persistent_kernel<V, U, true>), dim3(1), dim3(WG), 0, stream, a);
        else
            hipLaunchKernelGGL((persistent_kernel<V, U, false>), dim3(1), dim3(WG), 0, stream, a);
        SB_HIP(hipGetLastError());
        return SPARBIT_OK;
    }
    PersistentArgs args = a;
    void* params[] = {&args};
    const hipError_t e = hipLaunchCooperativeKernel(fn, dim3(uint32_t(grid)), dim3(WG), params, 0, stream);
    if (e == hipErrorCooperativeLaunchTooLarge) {
        (void)hipGetLastError();
        return SPARBIT_ERR_UNSUPPORTED;
    }
    SB_HIP(e);
    return SPARBIT_OK;
}

// The dataflow grid has exactly one workgroup per work item.  An item only waits for an item with a lower number,
// and the dispatcher starts the workgroups of a grid in increasing order (each XCD its share of them), so whatever
// a resident workgroup waits for is resident too or has finished: the grid makes progress whatever part of it is
// resident and whatever else runs on the GPU, including other such grids.
constexpr uint64_t kMaxFlowItems = (uint64_t(1) << 32) / WG - 1;  // a grid's x extent times its block size stays below 2^32

template <typename V, bool REALIGN = false>
int launch_dataflow_v(const FlowArgs& a, hipStream_t stream)
{
    note_launch(uint64_t(a.total_items / a.chunks_per_block) * a.block_bytes, "sparbit::dataflow_kernel<%s, %s>", type_label<V>(),
                bool_label(REALIGN));
    hipLaunchKernelGGL((dataflow_kernel<V, REALIGN>), dim3(a.total_items), dim3(WG), 0, stream, a);
    SB_HIP(hipGetLastError());
    return SPARBIT_OK;
}

// The tree kernel: one wavefront, or with `team` > 1 that many, per (tree, piece of 64 * U vectors).
constexpr uint32_t kTreeGang = 4;     // wavefronts per workgroup in the gang form ...
constexpr uint32_t kTreeBigGang = 8;  // ... and in its second size: one such workgroup per compute unit (see choose_tree_walk)
constexpr uint32_t kLdsPerUnit = 160 * 1024;

// One gang launch.  A workgroup that is to have a compute unit to itself reserves more than half of the unit's LDS,
// which is more than a kernel may ask for unless the function's limit has been raised: once per function and device.
template <auto kernel>
int launch_gang(dim3 grid, uint32_t wavefronts, uint32_t lds, hipStream_t stream, const TreeArgs& a)
{
    if (lds > 65536u) {
        static std::atomic<uint64_t> raised{0};  // one per kernel (the kernel is a template argument); bit d = done on device d
        int device = 0;
        SB_HIP(hipGetDevice(&device));
        const uint64_t bit = uint64_t(1) << (device & 63);
        if (device >= 64 || !(raised.load() & bit)) {
            SB_HIP(hipFuncSetAttribute(reinterpret_cast<const void*>(kernel), hipFuncAttributeMaxDynamicSharedMemorySize, int(kLdsPerUnit)));
            raised.fetch_or(bit);
        }
    }
    hipLaunchKernelGGL(kernel, grid, dim3(64 * wavefronts), lds, stream, a);
    SB_HIP(hipGetLastError());
    return SPARBIT_OK;
}

template <typename V, int U, int NB, bool VAR, bool ANY = false, int WALK = kWalkSparbit>
int launch_tree_vu(const TreeArgs& a, dim3 grid, int store_kind, bool prefetch, uint32_t lds, uint64_t bytes, hipStream_t stream,
                   uint32_t team = 1, uint32_t gang = 1)
{
    if (sizeof(V) != 16) store_kind = 0;
    // Ring's chain has no runs: no look-ahead, plain or write-through stores.  Recursive Doubling's tree has them
    // only in store forms 1 and 4 (walked as Sparbit's tree with the bits of the relative rank reversed), on whole
    // 16-byte vectors, one per lane, without teams.
    const bool reversed = WALK == kWalkDoubling && (store_kind == 1 || store_kind == 4) && sizeof(V) == 16 && U == 1 && team == 1;
    const bool step_order_only = WALK != kWalkSparbit && !reversed;
    if (step_order_only || team > 1) prefetch = false;
    if ((step_order_only || team > 1) && store_kind == 3) store_kind = 2;
    if ((step_order_only || team > 1) && store_kind == 1) store_kind = 0;
    if ((step_order_only || team > 1) && store_kind == 4) store_kind = 2;
    if (store_kind == 1 || store_kind == 4) prefetch = true;
    if (WALK == kWalkChain) team = 1;
    if (sizeof(V) != 16 || U != 1 || team > 1 || (WALK != kWalkChain && store_kind != 1 && store_kind != 4)) gang = 1;
    // the larger gang: equal blocks of whole vectors, store form 4 or the chain (the caller sized the grid for it)
    if (gang == kTreeBigGang && (VAR || ANY || (WALK != kWalkChain && store_kind != 4))) return SPARBIT_ERR_ARG;
    note_launch(bytes, "sparbit::tree_kernel<%s, %d, %d, %d, %s, %s, %s, %d, %s, %d>", type_label<V>(), U, NB, store_kind,
                bool_label(prefetch), bool_label(VAR), bool_label(ANY), WALK, bool_label(team > 1), int(gang));
#define SB_TREE(ST, PF) hipLaunchKernelGGL((tree_kernel<V, U, NB, ST, PF, VAR, ANY, WALK>), grid, dim3(64), lds, stream, a)
#define SB_TEAM(ST) \
    hipLaunchKernelGGL((tree_kernel<V, U, NB, ST, false, VAR, ANY, WALK, true>), grid, dim3(64 * team), lds, stream, a)
    if constexpr (U == 1 && WALK == kWalkChain && sizeof(V) == 16 && !ANY) {
        if constexpr (!VAR)
            if (gang == kTreeBigGang)
                return launch_gang<&tree_kernel<V, U, NB, 0, false, VAR, ANY, WALK, false, kTreeBigGang>>(grid, gang, lds, stream, a);
        if (gang > 1)  // Ring's chain stores plain (see choose_tree_walk)
            return launch_gang<&tree_kernel<V, U, NB, 0, false, VAR, ANY, WALK, false, kTreeGang>>(grid, gang, lds, stream, a);
    }
    if constexpr (U == 1 && WALK != kWalkChain && sizeof(V) == 16) {
        if constexpr (!VAR && !ANY)
            if (gang == kTreeBigGang)
                return launch_gang<&tree_kernel<V, U, NB, 4, true, VAR, ANY, WALK, false, kTreeBigGang>>(grid, gang, lds, stream, a);
        if (gang > 1) {
            if (store_kind == 1)
                return launch_gang<&tree_kernel<V, U, NB, 1, true, VAR, ANY, WALK, false, kTreeGang>>(grid, gang, lds, stream, a);
            return launch_gang<&tree_kernel<V, U, NB, 4, true, VAR, ANY, WALK, false, kTreeGang>>(grid, gang, lds, stream, a);
        }
    }
    if constexpr (U == 1 && WALK != kWalkChain) {
        if (team > 1) {
            if (store_kind != 0) SB_TEAM(2);
            else SB_TEAM(0);
            SB_HIP(hipGetLastError());
            return SPARBIT_OK;
        }
    }
    if constexpr (WALK == kWalkDoubling && sizeof(V) == 16 && U == 1) {
        if (reversed) {
            if (store_kind == 1) SB_TREE(1, true);
            else SB_TREE(4, true);
            SB_HIP(hipGetLastError());
            return SPARBIT_OK;
        }
    }
    if constexpr (WALK != kWalkSparbit) {
        if (store_kind != 0) SB_TREE(2, false);
        else SB_TREE(0, false);
    } else if constexpr (ANY) {  // the store forms that lost on whole vectors are not built a second time
        if (store_kind == 1) SB_TREE(1, true);
        else if (store_kind == 4) SB_TREE(4, true);
        else if (store_kind != 0 && prefetch) SB_TREE(2, true);
        else if (store_kind != 0) SB_TREE(2, false);
        else if (prefetch) SB_TREE(0, true);
        else SB_TREE(0, false);
    } else if constexpr (sizeof(V) == 16) {
        if constexpr (U == 1) {
            if (store_kind == 1 || store_kind == 4) {
                if (store_kind == 1) SB_TREE(1, true);
                else SB_TREE(4, true);
                SB_HIP(hipGetLastError());
                return SPARBIT_OK;
            }
        }
        if (store_kind == 1) store_kind = 0;
        if (store_kind == 4) store_kind = 2;
        if (store_kind == 3 && prefetch) SB_TREE(3, true);
        else if (store_kind == 3) SB_TREE(3, false);
        else if (store_kind == 2 && prefetch) SB_TREE(2, true);
        else if (store_kind == 2) SB_TREE(2, false);
        else if (prefetch) SB_TREE(0, true);
        else SB_TREE(0, false);
    } else {
        if (prefetch) SB_TREE(0, true);
        else SB_TREE(0, false);
    }
#undef SB_TREE
#undef SB_TEAM
    SB_HIP(hipGetLastError());
    return SPARBIT_OK;
}

// The access form of one tree launch, chosen by launch_tree below.
struct TreeLaunch {
    dim3 grid;
    bool any;       // the any-alignment form
    int width;      // else: bytes per access, 16, 4 or 1
    int U;          // 16-byte vectors per lane
    int store_kind;
    bool prefetch;
    uint32_t lds;
    uint64_t bytes;
    hipStream_t stream;
    uint32_t team;
    uint32_t gang;  // wavefronts per workgroup in the gang form, else 1
};

template <bool VAR, int WALK>
int launch_tree_as(const TreeArgs& a, const TreeLaunch& h)
{
    if (h.any)
        return launch_tree_vu<u32x4, 1, 8, VAR, true, WALK>(a, h.grid, h.store_kind, h.prefetch, h.lds, h.bytes, h.stream, h.team, h.gang);
    if (h.width == 16) {
        if constexpr (WALK == kWalkSparbit) {
            if (h.U == 2) return launch_tree_vu<u32x4, 2, 8, VAR>(a, h.grid, h.store_kind, h.prefetch, h.lds, h.bytes, h.stream);
        }
        return launch_tree_vu<u32x4, 1, 8, VAR, false, WALK>(a, h.grid, h.store_kind, h.prefetch, h.lds, h.bytes, h.stream, h.team, h.gang);
    }
    if (h.width == 4)
        return launch_tree_vu<uint32_t, 1, 8, VAR, false, WALK>(a, h.grid, 0, h.prefetch, h.lds, h.bytes, h.stream, h.team);
    return launch_tree_vu<uint8_t, 1, 8, VAR, false, WALK>(a, h.grid, 0, h.prefetch, h.lds, h.bytes, h.stream, h.team);
}

// How launch_tree's wavefronts walk their trees, and how many of them a compute unit holds at once.
struct TreeWalk {
    uint32_t lg_k;  // runs of 2^lg_k relative ranks (with teams: one run per wavefront; Recursive Doubling: 2^lg_k sub-trees)
    uint32_t team;  // wavefronts per workgroup that share one piece of one tree
    int store;      // the kernel's store form
    uint32_t lds;   // bytes of LDS each wavefront reserves without using them: caps the resident wavefronts per unit
    uint32_t gang;  // 4 or 8: workgroups of that many wavefronts whose pieces lie 2^lg_s KiB apart; 0: none
    uint32_t lg_s;
};
struct TreeCall {
    int algo, p;
    size_t B;         // the (longest) block
    bool any;         // the any-alignment form ...
    bool part_lines;  // ... in rows that are not a multiple of 128 bytes apart: stores cover parts of lines at most ranks
    bool var;         // per-slot sizes
    bool rows_64k;    // rows a multiple of 64 KiB apart
    int width, U;     // bytes per access (any: 0) and 16-byte vectors per lane
    uint64_t total_bytes, waves;  // receive bytes of the call; wavefronts (teams) of the grid
};

// Every figure below was measured on an MI355X; the kernel's comment explains the terms.  LDS is handed out in
// granules of 1280 bytes (measured with a kernel that only sleeps): 10240 bytes per wavefront leave room for 16
// wavefronts per compute unit, 14336 bytes (12 granules) for 10, 8192 bytes (7 granules) for 18.
//
// Without the knobs, by receive bytes of the call:
//  - up to 96 MiB (tree_small_bytes): step order, the fewest dependent round trips of a latency-bound call; from 33
//    ranks on a team of 4 wavefronts, from 65 on of 8, walks a piece's tree (p = 256, 128-byte blocks: 9.9 us of kernel
//    time against 27 us; what is left is the depth of the tree, ceil(log2 p) dependent hops of ~1.2 us).  Otherwise:
//  - grids of fewer than 4096 wavefronts: runs of 32, 16 or 8 ranks as the grid has fewer than 1024, 2048 or more
//    wavefronts, for more loads in flight per wavefront (p = 256, 2 KiB: 38 us with runs of 32, 43 us with 16, 54 us
//    with 4; p = 256, 4 KiB: 55 us with runs of 16, 64 us with 4); larger grids: runs of 4, write-through stores;
//  - Sparbit and Recursive Doubling (the same tree, see the kernel), whole 16-byte vectors or the any-alignment form:
//    from 48 MiB (96 MiB from 65 ranks on) to 336 MiB store form 1, uncapped: plain stores, runs of 8, every
//    forwarder read back right after it was stored (against the write-through walk: p = 16, 1 MiB: 48 against 57 us;
//    p = 64, 64 KiB: 42 against 48 us; p = 128, 16 KiB (256 MiB): 46 against 52 us);
//  - beyond 336 MiB store form 4 (that walk, write-through for the stores that are not read back) on a capped grid.
//    16 wavefronts per unit up to 48 ranks, up to 1.25 GiB on 49 .. 64 ranks and up to 480 MiB beyond, else 10 (p = 64,
//    128 KiB: 99 us with 16, 110 us with 10, uncapped 114 us; p = 48, 768 MiB: 156 / 161 / 166 us; p = 16, 4 MiB: 223 /
//    282 / 241 us; p = 33, 2 GiB: 415 / 433 / 419 us; p = 80, 762 MiB: 162 / 153 / 169 us; p = 125, 885 MiB: 185 / 178 /
//    194 us; p = 256, 24 KiB: 326 / 320 / 337 us; cfg4 3.21 / 3.07 / 3.48 ms, 3.11-3.15 ms with the write-through walk
//    on 10 per unit; cfg5 3.33 / 3.21 / 3.52 ms, 3.25 ms).  A cap turns the grid into rounds of 4096 or 2560
//    wavefronts, and a last round of a few wavefronts costs a whole round: with fewer than three rounds the preferred
//    cap is taken only if its last round is 3/8 full (3/5 with fewer than two rounds), else the other cap on the same
//    condition, else none (p = 125, 504 MiB, 4125 wavefronts on 4096 places: 118 us, uncapped 103 us; p = 253, 750 MiB,
//    3036 wavefronts on 2560 places: 186 against 161 us; 875 MiB, 3542 wavefronts: 193 against 183 us);
//  - the any-alignment form in rows on the lines takes form 4 from blocks of 10 KiB on (p = 256, 6 KiB + 4: 151 us
//    against 132 us with the write-through walk) and below 8 GiB (beyond: level, or 1 % behind with per-slot sizes),
//    with 16 per unit or no cap, and a cap only from three rounds on: its first and last pieces are short, so its
//    rounds are uneven anyway (p = 32, 2 MiB + 4: 403 us with 16 per unit, 453 us with the write-through walk; p = 256,
//    24 KiB + 4: 370 us uncapped, 413 / 478 us with 16 / 10 per unit; p = 128, 64 KiB + 4: 237 / 266 us with 16 / 10);
//  - the any-alignment form in other rows: plain stores, since a piece's stores cover part-lines at most ranks, which
//    write-through stores do badly (p = 61, B = 64 KiB + 16: 54 us plain, 57-60 us write-through; on jobs of several
//    GiB 5.6-6.1 ms against 6.5-8.6 ms), and form 1 by the earlier rule (48 MiB .. 768 MiB up to 64 ranks, any size
//    above 48 MiB below 32 ranks, 96 .. 384 MiB beyond 64 ranks);
//  - what is left of the large calls (the knobs switch the forms above off, narrow accesses): the write-through walk
//    in runs of 8 on 10 wavefronts per unit when the grid has 8192 wavefronts and more on more than 32 ranks (p = 128,
//    1 MiB: 3.12 ms; uncapped 3.45 ms; capped at 16 with runs of 4: 3.23 ms; a shorter tree is walked too quickly for
//    that to pay: p = 16, 1 MiB: 58.6 us uncapped with runs of 4, 66.6 us capped with runs of 8);
//  - Ring: plain stores always (the chain reads a rank back right after storing it, and a plain store leaves the line
//    in the L2 for that read: p = 128, 1 MiB: 3.23 ms; a write-through store makes every hop wait for the memory side:
//    13.3 ms); beyond 336 MiB 16 wavefronts per unit (p = 64, 128 KiB: 93 against 103 us; p = 128, 1 GiB: 195 against
//    206 us; 16 GiB: level with 10), so that a comparison of the schedules compares tuned forms;
//  - Recursive Doubling where it still walks in step order beyond 336 MiB: below 8 GiB 10 per unit from 32 ranks on
//    (p = 128, 64 KiB: 239 against 290 us; p = 64, 1 MiB: 936 against 1116 us); on 16 GiB uncapped up to 64 ranks (3.97
//    against 4.56 ms), 18 per unit beyond (p = 128, 1 MiB: 4.61 ms; 10 per unit 4.99 ms; uncapped 4.66 ms).
TreeWalk choose_tree_walk(const TreeCall& c)
{
    const int p = c.p;
    const uint64_t MiB = uint64_t(1) << 20, total_bytes = c.total_bytes, waves = c.waves;
    const bool doubling = c.algo == SPARBIT_ALGO_RECURSIVE_DOUBLING, ring = c.algo == SPARBIT_ALGO_RING;
    const long long run_knob = g_tree_run_log2.load(), lds_knob = g_tree_lds_bytes.load(), hot_knob = g_tree_hot.load();
    const long long team_knob = g_tree_team_log2.load();
    const bool untouched = run_knob < 0 && lds_knob < 0 && g_tree_store.load() == 2 && team_knob < 0;
    const bool small = total_bytes <= uint64_t(g_tree_small_bytes.load());
    const bool capped = waves >= 8192 && p > 32;
    TreeWalk w;
    w.lg_k = run_knob >= 0 ? uint32_t(run_knob)
                           : small ? uint32_t(ceil_log2(p))
                           : waves < 1024 ? 5u : waves < 2048 ? 4u : waves < 4096 ? 3u : capped ? 3u : 2u;
    w.team = 1;
    if (c.U == 1 && !ring) {
        const int lg_p = ceil_log2(p);
        int lg_team = team_knob >= 0 ? int(team_knob) : (small && run_knob < 0 && p > 32) ? (p > 64 ? 3 : 2) : 0;
        if (lg_team > lg_p - 1) lg_team = lg_p > 1 ? lg_p - 1 : 0;  // at least 2 ranks per wavefront
        if (lg_team > 0) {
            w.team = 1u << lg_team;
            // Sparbit: runs of 2^lg_k ranks, one per wavefront; Recursive Doubling: 2^lg_k sub-trees, by low bits
            w.lg_k = doubling ? uint32_t(lg_team) : uint32_t(lg_p - lg_team);
        }
    }
    w.lds = lds_knob >= 0 ? uint32_t(lds_knob) : capped ? (doubling ? 8192u : 14336u) : 0u;
    w.store = int(g_tree_store.load());
    if (c.part_lines && w.store != 1) w.store = 0;
    struct Cap { uint32_t lds; uint64_t places; };
    const Cap c16{10240u, 16 * 256}, c10{14336u, 10 * 256}, none{0u, 0};
    const bool lines16 = c.width == 16 && !c.any, lines_any = c.any && !c.part_lines;
    auto whole_rounds = [&](const Cap& cap, bool from_three_rounds_only) {  // no last round that leaves most of the GPU idle
        if (cap.places == 0) return true;
        const uint64_t last = waves % cap.places;
        if (waves <= cap.places || waves >= 3 * cap.places || last == 0) return true;
        if (from_three_rounds_only) return false;
        return waves < 2 * cap.places ? last * 5 >= cap.places * 3 : last * 8 >= cap.places * 3;
    };
    if ((c.algo == SPARBIT_ALGO_SPARBIT || doubling) && (c.width == 16 || c.any) && c.U == 1) {
        const bool hot_size = lines16 || lines_any ? total_bytes > (p <= 64 ? 48 : 96) * MiB && total_bytes <= 336 * MiB
                              : p < 32             ? total_bytes > 48 * MiB
                              : p <= 64            ? total_bytes > 48 * MiB && total_bytes <= 768 * MiB
                                                   : total_bytes > 96 * MiB && total_bytes <= 384 * MiB;
        if (hot_knob > 0 || (hot_knob < 0 && hot_size && untouched)) {
            w.store = 1;
            if (lds_knob < 0) w.lds = 0;
        } else if (hot_knob < 0 && untouched && total_bytes > 336 * MiB &&
                   (lines16 || (lines_any && c.B >= 10240 && total_bytes < 8192 * MiB))) {
            w.store = 4;
            const bool prefer16 = lines_any || p <= 48 || total_bytes < (p <= 64 ? 1280 : 480) * MiB;
            const Cap first = prefer16 ? c16 : c10, second = lines_any || p <= 32 ? none : prefer16 ? c10 : c16;
            w.lds = whole_rounds(first, lines_any) ? first.lds : whole_rounds(second, lines_any) ? second.lds : 0u;
        }
        if (w.store == 1 || w.store == 4) {  // those walks are runs of 8 by one wavefront
            w.team = 1;
            w.lg_k = 3;
        }
    }
    if (ring) w.store = 0;
    if (untouched && hot_knob < 0 && total_bytes > 336 * MiB && w.store != 1 && w.store != 4 && (ring || doubling)) {
        auto rounds_fit = [&](const Cap& cap) {
            const uint64_t last = waves % cap.places;
            return waves <= cap.places || waves >= 3 * cap.places || last == 0 || last * 5 >= cap.places * 3;
        };
        if (ring)
            w.lds = rounds_fit(c16) ? c16.lds : (p > 32 && rounds_fit(c10)) ? c10.lds : 0u;
        else if (total_bytes < 8192 * MiB)
            w.lds = (p >= 32 && rounds_fit(c10)) ? c10.lds : 0u;
        else
            w.lds = p <= 64 ? 0u : 8192u;
    }
    // Gangs (the kernel's GANG): where form 4 was chosen above for whole 16-byte vectors and the blocks are a multiple
    // of 64 KiB, so that the 64 or 128 KiB that a gang's four pieces span start on such a boundary at every rank, or
    // are 16 KiB and more (then the gain is smaller: 3-10 %).  Against the choice above: cfg5 2.70 against 3.21 ms, cfg4 2.66
    // against 3.07 ms, p = 64 with 1 MiB blocks 683 against 777 us, p = 16 with 4 MiB blocks 192 against 222 us, p = 128
    // with 64 KiB blocks 183 against 214 us; blocks off those boundaries: p = 125 with 1073 KiB blocks 2.55 against
    // 2.75 ms, p = 33 with 1925 KiB blocks 394 against 417 us, p = 257 with 254 KiB blocks 3.11 against 3.13 ms.  Few
    // pieces per block leave most of a gang idle (p = 125, 6 KiB blocks: 56 against 22 us).  Pieces 32 KiB apart, 16 KiB
    // from 64 ranks on for blocks of 1 MiB and more or off the 128 KiB boundaries (cfg4 2.66 against 2.77 ms, cfg5 2.75
    // against 2.70 ms).  Resident wavefronts per unit: 16 up to 16 ranks, 12 up to 48 and up to 768 MiB, else 8 (two
    // gangs), again only where the grid's last round is at least half full or there are six rounds and more; and one
    // gang of 8 per unit from 48 ranks on where the blocks are a multiple of 128 KiB (below).
    const long long gang_knob = g_tree_gang.load(), apart_knob = g_tree_gang_apart_log2.load();
    const bool on_boundaries = c.B % 65536 == 0;
    w.gang = gang_knob == 1 ? kTreeGang : gang_knob > 1 ? uint32_t(gang_knob) : 0u;
    w.lg_s = apart_knob >= 0 ? uint32_t(apart_knob) : p >= 64 && (c.B >= MiB || c.B % 131072 != 0) ? 4u : 5u;
    // (The any-alignment form in rows that are not a multiple of 64 KiB apart can run in gangs too, by the knob: its
    // pieces cannot lie on such boundaries at every rank, and gain 0-6 %: p = 128, 1 MiB + 4: 3.18 against 3.23 ms; p =
    // 64, 128 KiB + 4: 125 against 121 us.  In rows that are: at the end of this function.)
    // Form 1's calls gain where they no longer fit the last-level cache and the blocks are long: from 240 MiB on with
    // blocks of 128 KiB and more, no cap (p = 16 with 1 MiB blocks 43.7 against 47.5 us, p = 8 with 4 MiB 52 against
    // 61-65 us, p = 20 with 768 KiB 58 against 63 us, p = 24 with 512 KiB 48.9 against 52 us, p = 48 with 128 KiB 49.2
    // against 50.3 us, p = 5 with 12 MiB 64 against 74 us; below 240 MiB or with shorter blocks 0 +- 1 %: p = 29 with
    // 256 KiB 34.8 us either way, p = 96 with 32 KiB 46.7-47.4 against 46.5 us; blocks under 512 KiB off the 64 KiB
    // boundaries lose: p = 40 with 160 KiB 43.6 against 42.4 us).  Ring's chain by the same rule (p = 16 with 1 MiB 43.5
    // against 45.8 us, p = 8 with 4 MiB 48.5 against 53 us, p = 20 with 768 KiB 54.5 against 58 us).
    const bool hot_gangs = (ring ? total_bytes <= 336 * MiB : w.store == 1) && total_bytes >= 240 * MiB && c.B >= 128 * 1024 &&
                           (on_boundaries || c.B >= 512 * 1024);
    if (gang_knob < 0 && untouched && hot_knob < 0 && apart_knob < 0 && lines16 &&
        (ring ? (total_bytes > 336 * MiB || hot_gangs) : (w.store == 4 || hot_gangs)) && (on_boundaries || c.B >= 16 * 1024)) {
        w.gang = kTreeGang;
        const bool short_blocks = c.B < 48 * 1024;
        if (c.B % 131072 != 0 && on_boundaries && c.B < MiB) w.lg_s = 4;  // 64 KiB on its boundaries: two pieces of 32 KiB do not fit
        if (!on_boundaries && c.B < 400 * 1024) {  // few pieces: the spacing that leaves fewer wavefronts without one
            const uint64_t pieces = (c.B + 1023) / 1024;
            const uint64_t room4 = (pieces + 63) / 64 * 64, room5 = (pieces + 127) / 128 * 128;
            w.lg_s = room4 < room5 ? 4u : room5 < room4 ? 5u : w.lg_s;
            uint64_t room = room4 < room5 ? room4 : room5;
            if (short_blocks) {  // 16 or 32 KiB: closer together, so that a gang's four all lie inside a block
                // (p = 256, 32 KiB: 393 us with 8 KiB between them, 401 us with 16, 429 us without gangs; p = 256, 16 KiB:
                // 200 / 311 / 213 us with 4 / 16 KiB / none; p = 128, 32 KiB: 100 against 105 us; 8 KiB blocks: no gain;
                // blocks that are not a multiple of the 16 or 32 KiB a gang spans lose: p = 200, 20 KiB: 196 against
                // 162 us; p = 96, 40 KiB: 94 against 73 us)
                w.lg_s = pieces >= 32 ? 3u : 2u;
                const uint64_t group = uint64_t(4) << w.lg_s;
                room = (pieces + group - 1) / group * group;
                if (room != pieces) w.gang = 0;
            }
            // ... and none where two in five would be (p = 253, 65 KiB blocks: 908 against 820 us)
            if (pieces * 5 < room * 3) w.gang = 0;
        }
        const Cap g16{10240u, 16 * 256}, g12{12800u, 12 * 256}, g8{14336u, 8 * 256};  // per wavefront; a gang reserves four times that
        auto rounds_fit = [&](const Cap& cap) {
            const uint64_t last = waves % cap.places;
            return waves <= cap.places || waves >= 6 * cap.places || last == 0 || last * 2 >= cap.places;
        };
        // (per-slot sizes: 12, the blocks' lengths differ; p = 128 with blocks of 0.5-1.5 MiB: 3.17 against 3.38 ms with 8)
        const Cap order[3] = {short_blocks ? g8 : p <= 16 ? g16 : (p <= 48 || total_bytes <= 768 * MiB || c.var) ? g12 : g8,
                              short_blocks ? g12 : p <= 16 ? g12 : g16, short_blocks ? g16 : p <= 48 ? g8 : g12};
        if (w.gang && hot_gangs) {
            w.lds = 0;
        } else if (w.gang) {  // ... and no gangs where no cap fits (p = 257, 16 KiB, 4112 wavefronts: 255 against 220 us)
            const uint32_t none = ~0u;
            uint32_t fit = none;
            for (int i = 2; i >= 0; --i)
                if (rounds_fit(order[i])) fit = order[i].lds;
            if (fit == none) w.gang = 0;
            else w.lds = fit;
            // One gang of 8 per unit instead of two of 4, pieces 16 KiB apart, where the blocks are a multiple of the 128 KiB
            // that such a gang spans and there are 48 ranks and more: one address translation serves eight stores instead
            // of four (cfg5 2.61 against 2.69 ms, cfg4 2.68 against 2.71 ms; p = 64 with 1 MiB blocks 650 against 684 us,
            // with 128 KiB blocks 87 against 90 us; p = 128 with 512 KiB blocks 1.30 against 1.35 ms; p = 200 with 384 KiB
            // blocks 2.42 against 2.49 ms; p = 32 with 1 MiB 181 against 176 us, p = 16 with 4 MiB 202 against 185 us;
            // 8 KiB apart in blocks of 64 KiB: 2.75 ms on cfg4's size).  Two gangs of 8 per unit, or a gang of 16: slower
            // than the gangs of 4 (cfg4 2.84, 2.78 ms).  Ring's chain by the same rule (cfg4's size 2.63 against 2.68 ms,
            // p = 64 with 1 MiB blocks 659 against 673 us, cfg5's size level).
            if (w.gang && rounds_fit(g8) && !c.var && c.B % 131072 == 0 && p >= 48) {
                w.gang = kTreeBigGang;
                w.lg_s = 4;
                w.lds = kLdsPerUnit / 2 / kTreeBigGang + 256;  // more than half of the unit's LDS per gang
            }
        }
    }
    // The any-alignment form in rows a multiple of 64 KiB apart: its pieces are the cells of the 1 KiB grid of addresses
    // and a gang's four lie in one 64 KiB group of that grid at every rank, whatever the blocks' lengths and places
    // (the kernel's ANY), so long blocks gain as aligned ones do, less the part-filled groups at a block's two ends
    // (per-slot sizes of 0.5-1.5 MiB at 1-byte granularity on 128 ranks, rows rounded up to 64 KiB: 3.08 against 3.43 ms
    // with 16 wavefronts per unit, 3.17 ms with 12; 128 ranks with blocks of 1 MiB + 512 bytes from a base 16 bytes off
    // the lines: 3.02 ms with 12 per unit, 3.11 ms with 8, 3.31 ms without gangs).
    if (gang_knob < 0 && untouched && hot_knob < 0 && apart_knob < 0 && lines_any && c.rows_64k && !ring && total_bytes > 336 * MiB &&
        c.B >= 512 * 1024) {
        const Cap cap = c.var ? Cap{10240u, 16 * 256} : Cap{12800u, 12 * 256};
        const uint64_t last = waves % cap.places;
        if (waves >= 6 * cap.places || last == 0 || last * 2 >= cap.places) {
            w.store = 4;
            w.lg_k = 3;
            w.team = 1;
            w.gang = kTreeGang;
            w.lg_s = 4;
            w.lds = cap.lds;
        }
    }
    return w;
}

// Equal blocks of B bytes (counts == nullptr; slot k at k * B of a row) or blocks of different sizes (device arrays
// counts / displs; `B` is then the longest block).  Rows are row_bytes apart.  `width` is the access width the
// call's addresses and lengths allow; 0 asks for the any-alignment form (16-byte chunks cut relative to the
// 128-byte lines, single bytes at a block's ends).  *eligible stays false when the piece count does not fit a grid
// (blocks of several GiB): the caller falls back to per-step launches.
int launch_tree(int algo, const void* sendbufs, void* recvbufs, int p, size_t B, size_t row_bytes, const uint64_t* counts,
                const uint64_t* displs, uint64_t total_bytes, int width, hipStream_t stream, bool* eligible)
{
    *eligible = false;
    if (p == 1 && !sendbufs) {  // in place with one rank: nothing moves
        *eligible = true;
        return SPARBIT_OK;
    }
    const bool any = width == 0;
    int U = width == 16 && algo == SPARBIT_ALGO_SPARBIT ? int(g_tree_unroll.load()) : 1;
    const uint64_t vpb = any ? 0 : B / size_t(width);
    while (U > 1 && vpb <= uint64_t(64 * (U / 2))) U /= 2;  // short blocks: no lanes that only idle
    // any-alignment form: up to 127 bytes ahead of the first line boundary, then 1 KiB pieces
    const uint64_t pieces = any ? 1 + (uint64_t(B) + 1023) / 1024 : (vpb + uint64_t(64 * U) - 1) / uint64_t(64 * U);
    uint32_t lg_g = uint32_t(g_interleave_log2.load());
    while (lg_g > 0 && (1u << lg_g) > uint32_t(p)) --lg_g;
    if ((pieces << lg_g) > 0x7fffffffull / 64) return SPARBIT_OK;  // the grid's x extent stays below 2^31 lanes
    const uint32_t groups = (uint32_t(p) + (1u << lg_g) - 1) >> lg_g;  // at most 4096: fits the y extent
    TreeArgs a;
    std::memset(&a, 0, sizeof a);
    a.send = static_cast<const uint8_t*>(sendbufs);
    a.recv = static_cast<uint8_t*>(recvbufs);
    a.block_bytes = B;
    a.vpb = vpb;
    a.row_bytes = row_bytes;
    a.counts = counts;
    a.displs = displs;
    a.p = uint32_t(p);
    a.top = p > 1 ? 1u << (ceil_log2(p) - 1) : 0u;
    a.lg_g = lg_g;
    const uint64_t waves = pieces * uint64_t(p);
    const TreeWalk walk = choose_tree_walk(TreeCall{algo, p, B, any, any && row_bytes % 128 != 0, counts != nullptr, row_bytes % 65536 == 0, width, U, total_bytes, waves});
    a.lg_k = walk.lg_k;
    const uint32_t team = walk.team;
    const int st = walk.store;
    const bool doubling = algo == SPARBIT_ALGO_RECURSIVE_DOUBLING;
    // Gangs: a workgroup of kTreeGang wavefronts per kTreeGang pieces that lie `apart` pieces apart, i.e. per
    // group of kTreeGang * apart pieces `apart` workgroups; a block's last group may be part empty.
    const bool ring = algo == SPARBIT_ALGO_RING;
    const bool in_gangs = walk.gang && U == 1 && team == 1 && (ring ? width == 16 && !any : (width == 16 || any) && (st == 1 || st == 4));
    // the larger gang exists for equal blocks of whole vectors in store form 4 and for the chain
    const bool big = walk.gang == kTreeBigGang && !any && !counts && (ring || st == 4);
    const uint32_t gang = !in_gangs ? 1u : big ? kTreeBigGang : kTreeGang;
    a.lg_s = walk.lg_s;
    const uint64_t apart = uint64_t(1) << walk.lg_s, per_group = uint64_t(gang) * apart;
    // (the any-alignment form in rows a multiple of a gang's span apart counts a gang's pieces from the boundary of the
    // address grid below the block: up to a group less one of places ahead of the block's first piece stay empty)
    const uint64_t places = any && row_bytes % (per_group * 1024) == 0 ? pieces + per_group - 1 : pieces;
    const uint64_t x_items = in_gangs ? (places + per_group - 1) / per_group * apart : pieces;
    // per workgroup: a gang of 4 may reserve 64 KiB at most (16384 bytes per wavefront: 2 gangs per unit), a gang of 8
    // the unit's whole LDS
    const uint32_t most = big ? kLdsPerUnit : 65536u;
    const uint32_t lds = in_gangs ? (walk.lds * gang > most ? most : walk.lds * gang) : walk.lds;
    const dim3 grid(uint32_t(x_items << lg_g), groups, 1);
    const bool pf = g_tree_prefetch.load() != 0;
    *eligible = true;
    const TreeLaunch how{grid, any, width, U, st, pf, lds, total_bytes, stream, team, gang};
    if (algo == SPARBIT_ALGO_RING) return counts ? launch_tree_as<true, kWalkChain>(a, how) : launch_tree_as<false, kWalkChain>(a, how);
    if (doubling) return counts ? launch_tree_as<true, kWalkDoubling>(a, how) : launch_tree_as<false, kWalkDoubling>(a, how);
    return counts ? launch_tree_as<true, kWalkSparbit>(a, how) : launch_tree_as<false, kWalkSparbit>(a, how);
}

// AUTO runs whole calls of this schedule as the tree kernel where tree_form() finds a form for them.
bool auto_takes_tree_form(int algo)
{
    if (algo == SPARBIT_ALGO_SPARBIT) return g_tree_auto.load() != 0;
    if (algo == SPARBIT_ALGO_RECURSIVE_DOUBLING) return g_tree_auto.load() != 0 && g_tree_auto_doubling.load() != 0;
    if (algo == SPARBIT_ALGO_RING) return g_tree_auto.load() != 0 && g_tree_auto_ring.load() != 0;
    return false;
}

// Which form of the tree kernel serves a whole Sparbit call: 16, 4 or 1 = that access width with the pieces cut
// from the block's start, 0 = the any-alignment form, -1 = none (the call goes out step by step).  `w` is the
// access width the call's addresses and lengths allow, `whole_lines` says that every block starts and ends on a
// 128-byte line as it is, `longest` is the longest block, `asked_for` an explicit SPARBIT_MODE_TREE.
int tree_form(int algo, bool asked_for, int w, bool whole_lines, uint64_t row_bytes, size_t longest, uint64_t total_bytes, int p)
{
    const bool longish = longest >= size_t(g_realign_min_bytes.load());
    if (w == 16 && whole_lines) {
        // Long blocks on the lines but off the 64 KiB boundaries, in rows that are a multiple of 64 KiB apart: cut from
        // their starts, a gang's pieces straddle those boundaries; the any-alignment form cuts them by the address grid
        // and counts a gang's pieces from its boundaries (see choose_tree_walk; p = 128, blocks of 1 MiB + 512 bytes:
        // 3.02 against 3.27 ms).
        const bool by_the_grid = g_tree_any_align.load() != 0 && algo != SPARBIT_ALGO_RING && row_bytes % 65536 == 0 &&
                                 longest % 65536 != 0 && longest >= (size_t(512) << 10) && total_bytes > (uint64_t(336) << 20);
        if (!by_the_grid) return 16;
    }
    if (g_tree_any_align.load() != 0 && longish) {
        // Rows a multiple of 128 bytes apart: every rank's copy of a slot lies the same way relative to the lines,
        // so the any-alignment form writes whole lines everywhere (p = 128, B = 1 MiB + 4: 3.23 ms against 5.32 ms
        // step by step; p = 256, B = 4100: 72 against 125 us).
        if (row_bytes % 128 == 0) return 0;
        // Other rows: its stores cover part-lines at every piece's ends.  With plain stores it is still ahead
        // while the job is small (p = 61, B = 64 KiB + 16: 54 against 95 us; p = 253, B = 4100: 88 against 117
        // us), level from about 1 GiB (p = 125, B = 64 KiB + 16: 350 against 343 us), behind on several GiB (p =
        // 125, B = 1 MiB + 4: 5.6 against 5.0 ms).
        if (total_bytes <= uint64_t(g_tree_part_line_max_bytes.load())) return 0;
    }
    // On the 16-byte grid but off the lines, and not taken above: with write-through stores of part-lines the tree
    // form loses to one launch per step (p = 253, B = 16 KiB + 16, 1 GiB: 526 against 389 us).
    if (w == 16) {
        const bool as_before = g_tree_any_align.load() == 0 && longest < size_t(g_line_align_min_bytes.load());
        return (asked_for || !longish || as_before) ? 16 : -1;
    }
    // single-byte accesses only up to 1024 ranks (a lane walks its tree byte by byte; in a team of wavefronts p = 256,
    // B = 1..7: 12-13 us against 34-40 us step by step, p = 1000: 53-55 against 56-67 us, p = 4096: 660-1430 against
    // 130-470 us)
    if (!longish) return (asked_for || w == 4 || p <= 1024) ? w : -1;
    return asked_for ? w : -1;
}

bool ranges_overlap(const void* a, size_t na, const void* b, size_t nb);
int run(const void* sendbufs, void* recvbufs, int p, size_t B, int algo, int mode, bool whole, int first_step,
        int last_step, void* stream_v);

constexpr size_t kVarPlanCacheSize = 8;

// Look up or build the copy lists of an Allgatherv geometry.  Block index b of a
// receive-side buffer means (rank b / p, slot b % p); of the send buffer, rank b.
int get_var_plan(DeviceState* ds, DevicePlan* dp, int algo, int p, const size_t* counts, const size_t* displs,
                 size_t row_bytes, bool may_build, VarPlan** out)
{
    for (auto& vp : ds->var_plans) {
        if (vp->algo == algo && vp->p == p && vp->row_bytes == row_bytes &&
            std::memcmp(vp->counts.data(), counts, size_t(p) * sizeof(size_t)) == 0 &&
            std::memcmp(vp->displs.data(), displs, size_t(p) * sizeof(size_t)) == 0) {
            vp->last_use = ++ds->var_clock;
            *out = vp.get();
            return SPARBIT_OK;
        }
    }
    if (!may_build) return SPARBIT_ERR_UNSUPPORTED;
    auto vp = std::make_unique<VarPlan>();
    vp->algo = algo;
    vp->p = p;
    vp->row_bytes = row_bytes;
    vp->counts.assign(counts, counts + p);
    vp->displs.assign(displs, displs + p);
    std::vector<VarCopy> all;
    for (size_t host_phase = 0; host_phase < dp->host.phases.size(); ++host_phase) {
        const Phase& ph = dp->host.phases[host_phase];
        // The copies of a phase are independent, so they may be regrouped.  Lengths within a factor of four
        // share one launch (workgroups past the end of a shorter block exit at once), and so do phases whose
        // skew costs few idle workgroups; any other phase goes out as one launch per size class (factor of
        // two), so that it neither wastes dispatches on tiny blocks nor overflows the grid.
        std::vector<VarCopy> bucket[65], in_order;
        uint64_t longest = 0, shortest = ~uint64_t(0);
        for (const Copy& c : ph.copies) {
            const uint32_t slot = c.dst_block % uint32_t(p);  // the destination always names the slot
            if (counts[slot] == 0) continue;
            const uint64_t src_off = ph.src_buf == BUF_SEND
                                         ? displs[c.src_block]
                                         : uint64_t(c.src_block / uint32_t(p)) * row_bytes + displs[c.src_block % uint32_t(p)];
            const uint64_t dst_off = uint64_t(c.dst_block / uint32_t(p)) * row_bytes + displs[slot];
            const uint64_t len = counts[slot];
            const VarCopy vc = pack_var_copy(src_off, dst_off, len);  // all three below 2^40: checked by the caller
            int cls = 0;
            while ((uint64_t(1) << cls) < len) ++cls;  // ceil(log2 len)
            bucket[cls].push_back(vc);
            in_order.push_back(vc);
            if (len > longest) longest = len;
            if (len < shortest) shortest = len;
        }
        // Workgroups that a single launch, sized for the longest block, would start past the end of shorter blocks
        // (4 KiB tiles).  They exit at once, so up to ~10^5 of them are cheaper than the extra launches (measured:
        // p = 64, blocks of 1-64 KiB: 107 us with size classes, 41 us without; beyond ~10^6 idle workgroups the
        // single launch loses).
        uint64_t idle = 0;
        for (const VarCopy& vc : in_order) idle += (longest + 4095) / 4096 - (var_len(vc) + 4095) / 4096;
        if (longest != 0 && (longest <= 4 * shortest || idle <= uint64_t(g_var_idle_max.load()))) {  // one launch, schedule order
            for (int cls = 0; cls <= 64; ++cls) bucket[cls].clear();
            bucket[64].swap(in_order);
        }
        for (int cls = 64; cls >= 0; --cls) {
            if (bucket[cls].empty()) continue;
            VarPhase v{ph.src_buf, ph.dst_buf, uint32_t(all.size()), uint32_t(bucket[cls].size()), 0u, uint32_t(host_phase)};
            for (const VarCopy& vc : bucket[cls])
                if (var_len(vc) > v.max_len) v.max_len = var_len(vc);
            all.insert(all.end(), bucket[cls].begin(), bucket[cls].end());
            if (!ph.only_in_place && !ph.covered_by_fused) vp->out_of_place.push_back(v);
            if (!ph.skip_in_place) vp->in_place.push_back(v);
        }
    }
    if (!all.empty()) {
        SB_HIP(hipMalloc(reinterpret_cast<void**>(&vp->d_copies), all.size() * sizeof(VarCopy)));
        SB_HIP(hipMemcpy(vp->d_copies, all.data(), all.size() * sizeof(VarCopy), hipMemcpyHostToDevice));
    }
    {
        std::vector<uint64_t> geometry(size_t(2) * size_t(p));
        for (int k = 0; k < p; ++k) {
            geometry[size_t(k)] = counts[k];
            geometry[size_t(p) + size_t(k)] = displs[k];
            if (counts[k] > vp->max_count) vp->max_count = counts[k];
        }
        SB_HIP(hipMalloc(reinterpret_cast<void**>(&vp->d_geometry), geometry.size() * sizeof(uint64_t)));
        SB_HIP(hipMemcpy(vp->d_geometry, geometry.data(), geometry.size() * sizeof(uint64_t), hipMemcpyHostToDevice));
    }
    if (ds->var_plans.size() >= kVarPlanCacheSize) {
        // Evict the least recently used geometry; its table may still be read by queued launches.
        SB_HIP(hipDeviceSynchronize());
        size_t victim = 0;
        for (size_t i = 1; i < ds->var_plans.size(); ++i)
            if (ds->var_plans[i]->last_use < ds->var_plans[victim]->last_use) victim = i;
        ds->var_plans.erase(ds->var_plans.begin() + victim);
    }
    vp->last_use = ++ds->var_clock;
    *out = vp.get();
    ds->var_plans.push_back(std::move(vp));
    return SPARBIT_OK;
}

int launch_var_realign(const uint8_t* src, uint8_t* dst, const VarCopy* copies, uint32_t ncopies, uint64_t max_len,
                       hipStream_t stream)
{
    dim3 grid;
    uint32_t lg_g = 0;
    bool capped = false;  // the kernel loops, so a capped grid is fine
    if (!tile_grid(max_len >> 4, ncopies, WG, &grid, &lg_g, &capped)) return SPARBIT_ERR_ARG;
    note_launch(uint64_t(ncopies) * max_len, "sparbit::copy_var_realign_kernel<%s>", bool_label(g_nontemporal.load() != 0));
    if (g_nontemporal.load() != 0)
        hipLaunchKernelGGL((copy_var_realign_kernel<true>), grid, dim3(WG), 0, stream, src, dst, copies, ncopies, lg_g);
    else
        hipLaunchKernelGGL((copy_var_realign_kernel<false>), grid, dim3(WG), 0, stream, src, dst, copies, ncopies, lg_g);
    SB_HIP(hipGetLastError());
    return SPARBIT_OK;
}

template <typename V>
int launch_var(const uint8_t* src, uint8_t* dst, const VarCopy* copies, uint32_t ncopies, uint64_t max_len,
               bool write_through, hipStream_t stream)
{
    const uint64_t tiles = (max_len / sizeof(V) + WG - 1) / WG;
    if (tiles == 0 || ncopies == 0) return SPARBIT_OK;
    if (sizeof(V) < 16 && max_len >= uint64_t(g_realign_min_bytes.load()))
        return launch_var_realign(src, dst, copies, ncopies, max_len, stream);
    dim3 grid;
    uint32_t lg_g = 0;
    bool capped = false;
    if (!tile_grid(max_len / sizeof(V), ncopies, WG, &grid, &lg_g, &capped)) return SPARBIT_ERR_ARG;
    if (capped)  // a block too long for one tile per workgroup: the looping kernel
        return launch_var_realign(src, dst, copies, ncopies, max_len, stream);
    note_launch(uint64_t(ncopies) * max_len, "sparbit::copy_var_kernel<%s, %s, %s>", type_label<V>(),
                bool_label(g_nontemporal.load() != 0), bool_label(g_nontemporal.load() != 0 && write_through));
    if (g_nontemporal.load() != 0 && write_through)
        hipLaunchKernelGGL((copy_var_kernel<V, true, true>), grid, dim3(WG), 0, stream, src, dst, copies, ncopies, lg_g);
    else if (g_nontemporal.load() != 0)
        hipLaunchKernelGGL((copy_var_kernel<V, true>), grid, dim3(WG), 0, stream, src, dst, copies, ncopies, lg_g);
    else
        hipLaunchKernelGGL((copy_var_kernel<V, false>), grid, dim3(WG), 0, stream, src, dst, copies, ncopies, lg_g);
    SB_HIP(hipGetLastError());
    return SPARBIT_OK;
}

// AUTO's use of the dataflow launch.  `phases` are the phases the call runs (cumulative copy counts inside),
// `block` the block size (the longest one for Allgatherv).  Items are (copy, chunk) pairs, one workgroup each.
//   - a call of at most "dataflow_max_items" items at the base chunk size: the whole call in one launch;
//   - else the whole call if it fits "hybrid_max_items" items at up to four times that chunk (the smallest such
//     chunk: more workgroups move the data);
//   - else the leading phases that fit that limit at four times the base chunk (64 KiB), if there are at least two
//     of them to merge; the large late phases stay with the per-step kernel, which moves bulk data faster
//     (p = 16, B = 256 KiB: three of four phases merged 27.4 us, all four 33.3 us, none 36.0 us).
struct FlowChoice {
    size_t chunk = 0;    // bytes per work item (the last item of a block also takes the remainder)
    uint64_t cpb = 1;    // items per block
    size_t phases = 0;   // leading phases that go out as the dataflow launch (0: none)
    bool few_items = false;  // the first rule applied
};

// A block of `bytes` is cut into round(bytes / chunk) equal pieces (at least one), so that no item is much
// longer than the others: an item's copy is a serial chain of round trips inside one workgroup.
uint64_t pieces_per_block(uint64_t bytes, size_t chunk)
{
    const uint64_t n = (bytes + chunk / 2) / chunk;
    return n ? n : 1;
}

size_t base_flow_chunk()
{
    size_t c = size_t(g_flow_chunk_bytes.load());
    c -= c % 16;
    return c < 16 ? 16 : c;
}

FlowChoice choose_flow(const std::vector<DevPhase>& phases, uint64_t block)
{
    FlowChoice fc;
    if (phases.empty()) return fc;
    const size_t c0 = base_flow_chunk();
    const uint64_t total = phases.back().copies_before + phases.back().ncopies;
    auto per_block = [block](size_t c) -> uint64_t { return pieces_per_block(block, c); };
    if (total * per_block(c0) <= uint64_t(g_dataflow_max_items.load())) {
        fc.chunk = c0, fc.cpb = per_block(c0), fc.phases = phases.size(), fc.few_items = true;
        return fc;
    }
    const uint64_t limit = uint64_t(g_hybrid_max_items.load());
    for (size_t c = c0; c <= 4 * c0; c *= 2) {
        if (total * per_block(c) <= limit) {
            fc.chunk = c, fc.cpb = per_block(c), fc.phases = phases.size();
            return fc;
        }
    }
    const size_t c = 4 * c0;
    size_t n = 0;
    while (n < phases.size() && (phases[n].copies_before + phases[n].ncopies) * per_block(c) <= limit) ++n;
    if (n >= 2) fc.chunk = c, fc.cpb = per_block(c), fc.phases = n;
    return fc;
}

template <bool ON_GRID>
int launch_dataflow_var(const FlowVarArgs& a, hipStream_t stream)
{
    note_launch(uint64_t(a.f.total_items) * a.f.chunk_vecs, "sparbit::dataflow_var_kernel<%s>", bool_label(ON_GRID));
    hipLaunchKernelGGL((dataflow_var_kernel<ON_GRID>), dim3(a.f.total_items), dim3(WG), 0, stream, a);
    SB_HIP(hipGetLastError());
    return SPARBIT_OK;
}

int run_v(const void* sendbufs, void* recvbufs, int p, const size_t* counts, const size_t* displs, size_t row_bytes,
          int algo, void* stream_v)
{
    tl_launch_info = LaunchInfo();
    if (p < 1 || p > SPARBIT_MAX_P || !recvbufs || !counts || !displs) return SPARBIT_ERR_ARG;
    if (algo < SPARBIT_ALGO_SPARBIT || algo > SPARBIT_ALGO_DIRECT) return SPARBIT_ERR_ARG;
    if (algo == SPARBIT_ALGO_BRUCK) return SPARBIT_ERR_UNSUPPORTED;  // its rotated buffer assumes equal blocks
    if (algo == SPARBIT_ALGO_RECURSIVE_DOUBLING && (p & (p - 1))) return SPARBIT_ERR_UNSUPPORTED;
    // the copy lists hold byte offsets into the p receive buffers in 40 bits (1 TiB; the GPU has 288 GB)
    if ((unsigned __int128)row_bytes * unsigned(p) > (unsigned __int128)kVarFieldMask) return SPARBIT_ERR_ARG;
    uintptr_t bits = uintptr_t(sendbufs) | uintptr_t(recvbufs) | uintptr_t(row_bytes);
    std::vector<std::pair<size_t, size_t>> spans;  // (start, end) of the non-empty blocks
    for (int k = 0; k < p; ++k) {
        if (displs[k] > row_bytes || counts[k] > row_bytes - displs[k]) return SPARBIT_ERR_ARG;
        if (counts[k]) {
            bits |= uintptr_t(displs[k]) | uintptr_t(counts[k]);
            spans.emplace_back(displs[k], displs[k] + counts[k]);
        }
    }
    std::sort(spans.begin(), spans.end());
    for (size_t i = 1; i < spans.size(); ++i)  // blocks of one receive buffer must not overlap
        if (spans[i].first < spans[i - 1].second) return SPARBIT_ERR_ARG;
    const bool any = !spans.empty();
    const bool in_place = sendbufs == nullptr;
    if (!in_place && ranges_overlap(sendbufs, row_bytes, recvbufs, size_t(p) * row_bytes)) return SPARBIT_ERR_ALIAS;
    if (!any) return SPARBIT_OK;
    // Equal blocks packed back to back are a plain Allgather: same layout, and the equal-block path has the
    // faster kernels and the single-launch forms for small jobs.
    bool packed = counts[0] != 0 && row_bytes == size_t(p) * counts[0];
    for (int k = 0; k < p && packed; ++k) packed = counts[k] == counts[0] && displs[k] == size_t(k) * counts[0];
    if (packed) return run(sendbufs, recvbufs, p, counts[0], algo, SPARBIT_MODE_AUTO, true, 0, 0, stream_v);
    hipStream_t stream = static_cast<hipStream_t>(stream_v);
    const bool capturing = stream_is_capturing(stream);
    if (!capturing) {
        const int erc = report_expired_waits(stream);
        if (erc != SPARBIT_OK) return erc;
    }
    const int width = (bits & 15) == 0 ? 16 : (bits & 3) == 0 ? 4 : 1;
    size_t longest = 0;
    uint64_t total_bytes = 0;
    for (int k = 0; k < p; ++k) {
        if (counts[k] > longest) longest = counts[k];
        total_bytes += counts[k];
    }
    total_bytes *= uint64_t(p);
    // Sparbit as the tree kernel, by the same rules as for equal blocks.
    const int form = auto_takes_tree_form(algo) ? tree_form(algo, false, width, (bits & 127) == 0, row_bytes, longest, total_bytes, p)
                                                : -1;
    const bool tree = form >= 0;
    // Equal blocks at their packed positions in rows that are longer than p blocks (padded rows): the equal-block
    // tree kernel takes the row length as it is, and needs no table at all.
    bool padded = tree && counts[0] != 0 && row_bytes > size_t(p) * counts[0];
    for (int k = 0; k < p && padded; ++k) padded = counts[k] == counts[0] && displs[k] == size_t(k) * counts[0];
    if (padded) {
        tl_launch_info = LaunchInfo();
        bool eligible = false;
        const int trc = launch_tree(algo, sendbufs, recvbufs, p, counts[0], row_bytes, nullptr, nullptr, total_bytes, form,
                                    stream, &eligible);
        if (trc != SPARBIT_OK || eligible) return trc;
    }

    std::lock_guard<std::mutex> lock(g_mutex);
    DeviceState* ds = nullptr;
    int rc = get_device_state(&ds);
    if (rc != SPARBIT_OK) return rc;
    DevicePlan* dp = nullptr;
    if ((rc = get_plan(ds, algo, p, !capturing, &dp)) != SPARBIT_OK) return rc;
    VarPlan* vp = nullptr;
    if ((rc = get_var_plan(ds, dp, algo, p, counts, displs, row_bytes, !capturing, &vp)) != SPARBIT_OK) return rc;
    const uint8_t* base[3] = {static_cast<const uint8_t*>(sendbufs), static_cast<const uint8_t*>(recvbufs), nullptr};
    const bool on_lines = (bits & 127) == 0;  // every block starts and ends on a 128-byte line
    if (tree) {  // sizes and offsets come from the geometry's device copy
        bool eligible = false;
        const int trc = launch_tree(algo, sendbufs, recvbufs, p, longest, row_bytes, vp->d_geometry, vp->d_geometry + p,
                                    total_bytes, form, stream, &eligible);
        if (trc != SPARBIT_OK || eligible) return trc;
    }

    // As for equal blocks: a call of a few work items goes out as one dataflow launch, and in a larger one the
    // leading small steps share one.  A copy of an empty block still counts as an item (it exits at once).
    const std::vector<DevPhase>& phases = in_place ? dp->in_place : dp->out_of_place;
    size_t flow_phases = 0;  // leading phases done by the dataflow launch
    if (!capturing && !phases.empty()) {
        const FlowChoice fc = choose_flow(phases, vp->max_count);
        const size_t chunk = fc.chunk;
        const uint64_t cpb = fc.cpb;
        flow_phases = fc.phases;
        const uint64_t flags_per_buf = uint64_t(p) * uint64_t(p) * cpb;
        if (flow_phases && flags_per_buf <= 0x3fffffffull &&
            (phases[flow_phases - 1].copies_before + phases[flow_phases - 1].ncopies) * cpb <= kMaxFlowItems) {
            StreamState* fs = nullptr;
            if ((rc = get_flow(ds, stream, size_t(flags_per_buf), &fs)) != SPARBIT_OK) return rc;
            FlowVarArgs a;
            std::memset(&a, 0, sizeof a);
            a.f.base[0] = base[0];
            a.f.base[1] = base[1];
            a.f.copies = dp->d_copies;
            a.f.phases = in_place ? dp->d_phases_in_place : dp->d_phases;
            a.f.state = fs->flow;
            a.f.note = fs->note_dev;
            a.f.flags = fs->flags;
            a.f.spin_limit_ticks = uint64_t(g_spin_limit_ms.load()) * 100000ull;
            a.f.nphases = uint32_t(flow_phases);
            a.f.chunks_per_block = uint32_t(cpb);
            a.f.chunk_vecs = uint32_t(chunk);
            a.f.flags_per_buf = uint32_t(flags_per_buf);
            if ((rc = next_epoch(fs, stream, &a.f.epoch)) != SPARBIT_OK) return rc;
            a.f.total_items = uint32_t((phases[flow_phases - 1].copies_before + phases[flow_phases - 1].ncopies) * cpb);
            a.f.p = uint32_t(p);
            a.f.in_place = in_place ? 1u : 0u;
            a.counts = vp->d_geometry;
            a.displs = vp->d_geometry + p;
            a.row_bytes = row_bytes;
            rc = width == 16 ? launch_dataflow_var<true>(a, stream) : launch_dataflow_var<false>(a, stream);
            if (rc != SPARBIT_OK) return rc;
        } else {
            flow_phases = 0;
        }
    }
    // Which schedule phases the dataflow launch covered: the first `flow_phases` of those that this call runs.
    std::vector<char> covered(dp->host.phases.size(), 0);
    for (size_t i = 0, active = 0; i < dp->host.phases.size() && active < flow_phases; ++i) {
        const Phase& ph = dp->host.phases[i];
        if (in_place ? ph.skip_in_place : ph.only_in_place) continue;
        if (!in_place ? ph.covered_by_fused : ph.fused_first) continue;
        if (ph.copies.empty()) continue;
        covered[i] = 1;
        ++active;
    }
    for (const VarPhase& ph : in_place ? vp->in_place : vp->out_of_place) {
        if (covered[ph.host_phase]) continue;
        const uint8_t* src = base[ph.src_buf];
        uint8_t* dst = const_cast<uint8_t*>(base[ph.dst_buf]);
        const VarCopy* copies = vp->d_copies + ph.first;
        // Write-through stores where they were measured ahead of the non-temporal hint in this kernel: whole-line
        // blocks below 128 KiB (p = 128, 32..96 KiB: 6.2 against 5.96 TB/s; p = 61: 6.1 against 5.2); longer
        // blocks and blocks that cover lines piecewise are faster with the hint (1 MiB: 6.5 against 6.36 TB/s).
        const bool wt = on_lines && ph.max_len < (128u << 10);
        switch (width) {
        case 16: rc = launch_var<u32x4>(src, dst, copies, ph.ncopies, ph.max_len, wt, stream); break;
        case 4: rc = launch_var<uint32_t>(src, dst, copies, ph.ncopies, ph.max_len, false, stream); break;
        default: rc = launch_var<uint8_t>(src, dst, copies, ph.ncopies, ph.max_len, false, stream); break;
        }
        if (rc != SPARBIT_OK) return rc;
    }
    return SPARBIT_OK;
}

bool ranges_overlap(const void* a, size_t na, const void* b, size_t nb)
{
    const uintptr_t a0 = uintptr_t(a), b0 = uintptr_t(b);
    return a0 < b0 + nb && b0 < a0 + na;
}

// first_step / last_step as in sparbit_allgather_steps; `whole` = full call.
int run(const void* sendbufs, void* recvbufs, int p, size_t B, int algo, int mode, bool whole, int first_step,
        int last_step, void* stream_v)
{
    tl_launch_info = LaunchInfo();
    if (p < 1 || p > SPARBIT_MAX_P || !recvbufs) return SPARBIT_ERR_ARG;
    if (algo < SPARBIT_ALGO_SPARBIT || algo > SPARBIT_ALGO_DIRECT) return SPARBIT_ERR_ARG;
    if (mode < SPARBIT_MODE_AUTO || mode > SPARBIT_MODE_TREE) return SPARBIT_ERR_ARG;
    const unsigned __int128 total128 = (unsigned __int128)(uint64_t(p) * uint64_t(p)) * B;
    if (total128 > (unsigned __int128)0x7fffffffffffffffull) return SPARBIT_ERR_ARG;
    const size_t recv_bytes = size_t(p) * size_t(p) * B;
    const bool in_place = sendbufs == nullptr;
    if (!in_place && ranges_overlap(sendbufs, size_t(p) * B, recvbufs, recv_bytes)) return SPARBIT_ERR_ALIAS;
    if (algo == SPARBIT_ALGO_RECURSIVE_DOUBLING && (p & (p - 1))) return SPARBIT_ERR_UNSUPPORTED;
    if (algo == SPARBIT_ALGO_BRUCK && in_place) return SPARBIT_ERR_UNSUPPORTED;
    hipStream_t stream = static_cast<hipStream_t>(stream_v);
    if (B == 0) {  // zero-size blocks: only the step range is still validated
        if (!whole) {
            const int nsteps = (algo == SPARBIT_ALGO_RING) ? p - 1 : (algo == SPARBIT_ALGO_DIRECT) ? 0 : ceil_log2(p);
            if (first_step < -1 || last_step < -1 || first_step > last_step || last_step >= nsteps) return SPARBIT_ERR_ARG;
        }
        return SPARBIT_OK;
    }

    const bool capturing = stream_is_capturing(stream);
    const bool explicit_mode = mode != SPARBIT_MODE_AUTO;
    // A self-waiting launch on this stream that gave up since the last report: say so now, and enqueue nothing.
    if (!capturing) {
        const int erc = report_expired_waits(stream);
        if (erc != SPARBIT_OK) return erc;
    }

    // The tree kernel needs no table, no flag and no state, so it is decided before anything is looked up or built
    // (and a capturing stream can record it like any other launch).
    const bool has_tree_form = algo == SPARBIT_ALGO_SPARBIT || algo == SPARBIT_ALGO_RECURSIVE_DOUBLING || algo == SPARBIT_ALGO_RING;
    if (mode == SPARBIT_MODE_TREE && (!has_tree_form || !whole)) return SPARBIT_ERR_UNSUPPORTED;
    if (whole && has_tree_form && (mode == SPARBIT_MODE_TREE || (mode == SPARBIT_MODE_AUTO && auto_takes_tree_form(algo)))) {
        const int w = access_width(sendbufs, recvbufs, nullptr, B);
        const bool whole_lines = ((uintptr_t(recvbufs) | uintptr_t(B)) & 127) == 0;
        const int form = tree_form(algo, mode == SPARBIT_MODE_TREE, w, whole_lines, uint64_t(p) * B, B, recv_bytes, p);
        if (form >= 0) {
            bool eligible = false;
            const int trc = launch_tree(algo, sendbufs, recvbufs, p, B, size_t(p) * B, nullptr, nullptr, recv_bytes, form,
                                        stream, &eligible);
            if (trc != SPARBIT_OK || eligible) return trc;
            if (mode == SPARBIT_MODE_TREE) return SPARBIT_ERR_UNSUPPORTED;  // blocks of several GiB
        }
    }

    if (capturing) {
        if (mode == SPARBIT_MODE_PERSISTENT || mode == SPARBIT_MODE_DATAFLOW) return SPARBIT_ERR_UNSUPPORTED;
        mode = SPARBIT_MODE_PER_STEP;
    }

    std::lock_guard<std::mutex> lock(g_mutex);
    DeviceState* ds = nullptr;
    int rc = get_device_state(&ds);
    if (rc != SPARBIT_OK) return rc;
    DevicePlan* dp = nullptr;
    if ((rc = get_plan(ds, algo, p, !capturing, &dp)) != SPARBIT_OK) return rc;
    const int nsteps = int(dp->host.steps.size());
    if (!whole) {
        if (first_step < -1 || last_step < -1 || first_step > last_step || last_step >= nsteps) return SPARBIT_ERR_ARG;
        if (algo == SPARBIT_ALGO_BRUCK && !(first_step == -1 && last_step == nsteps - 1)) return SPARBIT_ERR_ARG;
    } else {
        first_step = -1;
        last_step = nsteps - 1;
    }

    void* work = nullptr;
    if (algo == SPARBIT_ALGO_BRUCK && (rc = get_work(ds, recv_bytes, !capturing, &work)) != SPARBIT_OK) return rc;
    const uint8_t* base[3] = {static_cast<const uint8_t*>(sendbufs), static_cast<const uint8_t*>(recvbufs),
                              static_cast<const uint8_t*>(work)};
    const int width = access_width(sendbufs, recvbufs, work, B);

    const std::vector<DevPhase>& phases = in_place ? dp->in_place : dp->out_of_place;
    size_t flow_chunk = base_flow_chunk();
    // Dataflow work items (and ready flags) per block.
    uint64_t cpb = pieces_per_block(B, flow_chunk);
    size_t flow_prefix = 0;  // leading phases that go out as one dataflow launch ahead of per-step launches
    if (mode == SPARBIT_MODE_AUTO) {
        // The single-launch dataflow form only where the whole job is a handful of workgroups: a grid that
        // waits on itself while it holds much of the machine starves whatever else runs on the GPU (and is
        // starved by it).  Anything larger goes out as one launch per step, which never waits on the device --
        // except that the first steps of a log-step schedule are small, so as many leading phases as fit in
        // one workgroup per item share one dataflow launch (a flag hand-over costs less than a kernel boundary).
        // With one workgroup per item an item only waits for lower-numbered workgroups, which are dispatched
        // first, so such a grid does not depend on its own residency; and at 512 workgroups, a quarter of the
        // GPU's workgroup slots, the grids of four calls running at once (HIP's default number of hardware
        // queues per process) are all resident together, so they cannot hold one another's slots either.
        const FlowChoice fc = choose_flow(phases, B);
        const bool whole_call = !phases.empty() && fc.phases == phases.size();
        if (whole_call && fc.few_items) {
            mode = SPARBIT_MODE_DATAFLOW;
            flow_chunk = fc.chunk, cpb = fc.cpb;
        } else if (recv_bytes <= size_t(g_persistent_max_bytes.load())) {
            mode = SPARBIT_MODE_PERSISTENT;  // a single workgroup of flattened tiles: the barrier costs next to nothing
        } else if (whole_call) {
            mode = SPARBIT_MODE_DATAFLOW;
            flow_chunk = fc.chunk, cpb = fc.cpb;
        } else {
            mode = SPARBIT_MODE_PER_STEP;
            if (fc.phases) flow_prefix = fc.phases, flow_chunk = fc.chunk, cpb = fc.cpb;
        }
    }

    // Dataflow form (flags instead of barriers) for the first `nph` phases of the call.
    auto launch_flow = [&](size_t nph, bool* launched) -> int {
        *launched = false;
        // Blocks off the 16-byte grid that are long enough to have a body: byte units, realigned 16-byte accesses.
        const bool realign = width < 16 && B >= size_t(g_realign_min_bytes.load());
        const size_t unit = realign ? 1 : size_t(width);
        const uint64_t items = (phases[nph - 1].copies_before + phases[nph - 1].ncopies) * cpb;
        const uint64_t flags_per_buf = uint64_t(p) * uint64_t(p) * cpb;
        if (items > kMaxFlowItems || flags_per_buf > 0x3fffffffull || B / unit > 0xffffffffull)
            return SPARBIT_OK;  // too many items for one grid, or offsets inside a block beyond the kernel's 32 bits
        StreamState* fs = nullptr;
        int frc = get_flow(ds, stream, size_t(2 * flags_per_buf), &fs);
        if (frc != SPARBIT_OK) return frc;
        FlowArgs a;
        std::memset(&a, 0, sizeof a);
        a.base[0] = base[0];
        a.base[1] = base[1];
        a.base[2] = base[2];
        a.copies = dp->d_copies;
        a.phases = in_place ? dp->d_phases_in_place : dp->d_phases;
        a.state = fs->flow;
        a.note = fs->note_dev;
        a.flags = fs->flags;
        a.block_bytes = B;
        a.spin_limit_ticks = uint64_t(g_spin_limit_ms.load()) * 100000ull;
        a.nphases = uint32_t(nph);
        a.chunks_per_block = uint32_t(cpb);
        a.chunk_vecs = uint32_t((((B + cpb - 1) / cpb + 15) / 16 * 16) / unit);  // equal pieces, whole 16-byte vectors
        a.flags_per_buf = uint32_t(flags_per_buf);
        if ((frc = next_epoch(fs, stream, &a.epoch)) != SPARBIT_OK) return frc;
        a.total_items = uint32_t(items);
        a.p = uint32_t(p);
        a.in_place = in_place ? 1u : 0u;
        *launched = true;
        if (realign) return launch_dataflow_v<uint8_t, true>(a, stream);
        switch (width) {
        case 16: return launch_dataflow_v<u32x4>(a, stream);
        case 4: return launch_dataflow_v<uint32_t>(a, stream);
        default: return launch_dataflow_v<uint8_t>(a, stream);
        }
    };
    if (whole && mode == SPARBIT_MODE_DATAFLOW && !phases.empty()) {
        bool launched = false;
        if ((rc = launch_flow(phases.size(), &launched)) != SPARBIT_OK || launched) return rc;
        if (explicit_mode) return SPARBIT_ERR_UNSUPPORTED;  // more work items than one grid holds
        mode = SPARBIT_MODE_PER_STEP;
    }
    if (flow_prefix) {
        bool launched = false;
        if ((rc = launch_flow(flow_prefix, &launched)) != SPARBIT_OK) return rc;
        if (!launched) flow_prefix = 0;
    }

    if (whole && mode == SPARBIT_MODE_PERSISTENT && !phases.empty()) {
        PersistentArgs a;
        std::memset(&a, 0, sizeof a);
        a.base[0] = base[0];
        a.base[1] = base[1];
        a.base[2] = base[2];
        a.copies = dp->d_copies;
        a.phases = in_place ? dp->d_phases_in_place : dp->d_phases;
        a.block_bytes = B;
        a.nphases = uint32_t(phases.size());
        a.spin_limit_ticks = uint64_t(g_spin_limit_ms.load()) * 100000ull;  // 100 MHz counter
        StreamState* bs = nullptr;
        if ((rc = get_barrier(ds, stream, &bs)) != SPARBIT_OK) return rc;
        a.bar = bs->barrier;
        a.note = bs->note_dev + 1;
        uint64_t max_tiles = 1;
        for (const DevPhase& ph : phases) {
            const uint64_t t = ((B / size_t(width)) * ph.ncopies + WG * 4 - 1) / (WG * 4);
            if (t > max_tiles) max_tiles = t;
        }
        switch (width) {
        case 16: return launch_persistent_v<u32x4>(a, ds, max_tiles, stream);
        case 4: return launch_persistent_v<uint32_t>(a, ds, max_tiles, stream);
        default: return launch_persistent_v<uint8_t>(a, ds, max_tiles, stream);
        }
    }

    // One launch per phase; stream order is the Waitall.
    size_t active = 0;  // index of the phase in `phases` (the list the single-launch kernels walk)
    for (size_t i = 0; i < dp->host.phases.size(); ++i) {
        const Phase& ph = dp->host.phases[i];
        if (in_place ? ph.skip_in_place : ph.only_in_place) continue;
        if (whole && !in_place ? ph.covered_by_fused : ph.fused_first) continue;
        const int step = (ph.step >= nsteps) ? nsteps - 1 : ph.step;  // Bruck's rotation rides with the last step
        if (step < first_step || step > last_step) continue;
        if (ph.copies.empty()) continue;
        if (active++ < flow_prefix) continue;  // already done by the dataflow launch above
        rc = launch_phase(base[ph.src_buf], const_cast<uint8_t*>(base[ph.dst_buf]), dp->d_copies + dp->first_copy[i],
                          uint32_t(ph.copies.size()), B, width, stream);
        if (rc != SPARBIT_OK) return rc;
    }
    return SPARBIT_OK;
}

// ---- the entry point that allocates nothing -----------------------------------------------------------------
// Per-step form with the copy table in the file-scope device array instead of library-allocated memory.  The
// table is rebuilt on the device, from the stripe closed form, by a small kernel at the head of every call (the
// array keeps the last call's contents and every call on a GPU shares it), then the own-block placement and one
// launch per step read it exactly as they read the cached tables of the other entry points.
int run_static(const void* sendbufs, void* recvbufs, int p, size_t B, void* stream_v)
{
    tl_launch_info = LaunchInfo();
    if (p < 1 || !recvbufs) return SPARBIT_ERR_ARG;
    if (p > SPARBIT_STATIC_MAX_P) return SPARBIT_ERR_TOO_LARGE;
    const size_t recv_bytes = size_t(p) * size_t(p) * B;  // p <= 512: no overflow below 2^45-byte blocks
    if (B > (size_t(1) << 45)) return SPARBIT_ERR_ARG;
    const bool in_place = sendbufs == nullptr;
    if (!in_place && ranges_overlap(sendbufs, size_t(p) * B, recvbufs, recv_bytes)) return SPARBIT_ERR_ALIAS;
    if (B == 0) return SPARBIT_OK;
    hipStream_t stream = static_cast<hipStream_t>(stream_v);

    Copy* tables = nullptr;
    {
        std::lock_guard<std::mutex> lock(g_mutex);
        DeviceState* ds = nullptr;
        const int rc = get_device_state(&ds);
        if (rc != SPARBIT_OK) return rc;
        if (!ds->static_tables) {  // once per device, with that device current
            void* ptr = nullptr;
            SB_HIP(hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)));
            ds->static_tables = static_cast<Copy*>(ptr);
        }
        tables = ds->static_tables;
    }

    StaticSteps st;
    std::memset(&st, 0, sizeof st);
    const int L = ceil_log2(p);
    st.nsteps = uint32_t(L);
    st.first[0] = uint32_t(p);  // entries 0 .. p - 1: own-block placement
    for (int s = 0; s < L; ++s) {
        const uint32_t d = 1u << (L - 1 - s);
        const uint32_t q = (uint32_t(p) + d - 1) / d;  // comb size after this step
        st.d[s] = d;
        st.n[s] = q / 2;
        st.first[s + 1] = st.first[s] + uint32_t(p) * st.n[s];
    }
    const uint32_t total = st.first[L];  // p + p (p - 1) = p^2
    hipLaunchKernelGGL(static_tables_kernel, dim3((total + WG - 1) / WG), dim3(WG), 0, stream, tables, uint32_t(p), st);
    SB_HIP(hipGetLastError());

    const uint8_t* send = static_cast<const uint8_t*>(sendbufs);
    uint8_t* recv = static_cast<uint8_t*>(recvbufs);
    const int width = access_width(sendbufs, recvbufs, nullptr, B);
    int rc = SPARBIT_OK;
    if (!in_place && (rc = launch_phase(send, recv, tables, uint32_t(p), B, width, stream)) != SPARBIT_OK) return rc;
    for (int s = 0; s < L; ++s)
        if ((rc = launch_phase(recv, recv, tables + st.first[s], uint32_t(p) * st.n[s], B, width, stream)) != SPARBIT_OK)
            return rc;
    return SPARBIT_OK;
}

}  // namespace
}  // namespace sparbit

extern "C" {

int sparbit_allgather(const void* sendbufs, void* recvbufs, int p, size_t block_bytes, void* stream)
{
    return sparbit::no_throw([&] {
        return sparbit::run(sendbufs, recvbufs, p, block_bytes, SPARBIT_ALGO_SPARBIT, SPARBIT_MODE_AUTO, true, 0, 0,
                            stream);
    });
}

int sparbit_allgather_algo(const void* sendbufs, void* recvbufs, int p, size_t block_bytes, int algo, void* stream)
{
    return sparbit::no_throw(
        [&] { return sparbit::run(sendbufs, recvbufs, p, block_bytes, algo, SPARBIT_MODE_AUTO, true, 0, 0, stream); });
}

int sparbit_allgather_mode(const void* sendbufs, void* recvbufs, int p, size_t block_bytes, int algo, int mode,
                           void* stream)
{
    return sparbit::no_throw(
        [&] { return sparbit::run(sendbufs, recvbufs, p, block_bytes, algo, mode, true, 0, 0, stream); });
}

int sparbit_allgatherv(const void* sendbufs, void* recvbufs, int p, const size_t* counts, const size_t* displs,
                       size_t row_bytes, int algo, void* stream)
{
    return sparbit::no_throw(
        [&] { return sparbit::run_v(sendbufs, recvbufs, p, counts, displs, row_bytes, algo, stream); });
}

int sparbit_allgather_steps(const void* sendbufs, void* recvbufs, int p, size_t block_bytes, int algo, int first_step,
                            int last_step, void* stream)
{
    return sparbit::no_throw([&] {
        return sparbit::run(sendbufs, recvbufs, p, block_bytes, algo, SPARBIT_MODE_PER_STEP, false, first_step,
                            last_step, stream);
    });
}

int sparbit_allgather_static(const void* sendbufs, void* recvbufs, int p, size_t block_bytes, void* stream)
{
    return sparbit::no_throw([&] { return sparbit::run_static(sendbufs, recvbufs, p, block_bytes, stream); });
}

void sparbit_finalize(void)
{
    std::lock_guard<std::mutex> lock(sparbit::g_mutex);
    int current = 0;
    const bool have_dev = hipGetDevice(&current) == hipSuccess;
    for (auto& kv : sparbit::g_devices) {
        sparbit::DeviceState* ds = kv.second.get();
        if (hipSetDevice(ds->device) != hipSuccess) continue;
        (void)hipDeviceSynchronize();  // queued launches may still read the tables
        ds->plans.clear();  // frees the device tables while this device is current
        ds->var_plans.clear();
        for (auto& sk : ds->streams) {
            (void)hipFree(sk.second.barrier);
            (void)hipFree(sk.second.flow);
            (void)hipFree(sk.second.flags);
            if (sk.second.note) {
                (void)hipHostFree(sk.second.note);
                sparbit::g_stream_states.fetch_sub(1);
            }
        }
        if (ds->work) (void)hipFree(ds->work);
    }
    sparbit::g_devices.clear();
    if (have_dev) (void)hipSetDevice(current);
}

const char* sparbit_strerror(int code)
{
    switch (code) {
    case SPARBIT_OK: return "success";
    case SPARBIT_ERR_ARG: return "invalid argument";
    case SPARBIT_ERR_ALIAS: return "send and receive buffers overlap (pass NULL sendbufs for in-place)";
    case SPARBIT_ERR_UNSUPPORTED: return "schedule does not support this call";
    case SPARBIT_ERR_HIP: return "HIP runtime error";
    case SPARBIT_ERR_NOMEM: return "out of host memory";
    case SPARBIT_ERR_TOO_LARGE: return "beyond the fixed capacity of the entry point that allocates nothing";
    case SPARBIT_ERR_TIMEOUT: return "an earlier self-waiting launch on this stream gave up a bounded wait; its results are incomplete";
    default: return "unknown error";
    }
}

int sparbit_last_hip_error(void) { return sparbit::tl_last_hip_error; }

int sparbit_last_launch_info(char* kernel, size_t cap, int* launches)
{
    const sparbit::LaunchInfo& li = sparbit::tl_launch_info;
    if (launches) *launches = li.launches;
    if (kernel && cap) {
        std::strncpy(kernel, li.kernel, cap - 1);
        kernel[cap - 1] = '\0';
    }
    return SPARBIT_OK;
}

// Test hook, deliberately absent from sparbit.h: moves the 32-bit call counter of the dataflow launches of every
// known stream forward to `value` (they wrap at 2^32), so that a test reaches the wrap without 2^32 calls.  Only
// forward: a number already handed out may still sit in a ready flag.
int sparbit_test_set_flow_call_number(long long value)
{
    using namespace sparbit;
    if (value < 0 || value > 0xffffffffll) return SPARBIT_ERR_ARG;
    std::lock_guard<std::mutex> lock(g_mutex);
    DeviceState* ds = nullptr;
    int rc = get_device_state(&ds);
    if (rc != SPARBIT_OK) return rc;
    for (auto& sk : ds->streams)
        if (sk.second.flow && sk.second.epoch > uint32_t(value)) return SPARBIT_ERR_ARG;
    for (auto& sk : ds->streams)
        if (sk.second.flow) sk.second.epoch = uint32_t(value);
    return SPARBIT_OK;
}

int sparbit_barrier_timeouts(void* stream_v, uint64_t* count)
{
    using namespace sparbit;
    if (!count) return SPARBIT_ERR_ARG;
    *count = 0;
    hipStream_t stream = static_cast<hipStream_t>(stream_v);
    return no_throw([&]() -> int {
        std::lock_guard<std::mutex> lock(g_mutex);
        DeviceState* ds = nullptr;
        int rc = get_device_state(&ds);
        if (rc != SPARBIT_OK) return rc;
        SB_HIP(hipStreamSynchronize(stream));
        auto it = ds->streams.find(stream);
        if (it != ds->streams.end() && it->second.barrier) {
            BarrierState host;
            SB_HIP(hipMemcpy(&host, it->second.barrier, sizeof host, hipMemcpyDeviceToHost));
            *count += host.errors;
        }
        if (it != ds->streams.end() && it->second.flow) {
            FlowState host;
            SB_HIP(hipMemcpy(&host, it->second.flow, sizeof host, hipMemcpyDeviceToHost));
            *count += host.errors;
        }
        return SPARBIT_OK;
    });
}

int sparbit_tune(const char* key, long long value)
{
    using namespace sparbit;
    if (!key) return SPARBIT_ERR_ARG;
    if (!std::strcmp(key, "wg_threads")) {
        if (value != 0 && value != 64 && value != 128 && value != 256 && value != 512 && value != 1024) return SPARBIT_ERR_ARG;
        g_wg_threads = value;
    } else if (!std::strcmp(key, "interleave_log2")) {
        if (value < 0 || value > 8) return SPARBIT_ERR_ARG;
        g_interleave_log2 = value;
    } else if (!std::strcmp(key, "unroll")) {
        if (value != 1 && value != 2 && value != 4) return SPARBIT_ERR_ARG;
        g_unroll = value;
    } else if (!std::strcmp(key, "persistent_max_bytes")) {
        if (value < 0) return SPARBIT_ERR_ARG;
        g_persistent_max_bytes = value;
    } else if (!std::strcmp(key, "hybrid_max_items")) {
        if (value < 0 || value > 1024) return SPARBIT_ERR_ARG;
        g_hybrid_max_items = value;
    } else if (!std::strcmp(key, "dataflow_max_items")) {
        if (value < 0) return SPARBIT_ERR_ARG;
        g_dataflow_max_items = value;
    } else if (!std::strcmp(key, "flow_chunk_bytes")) {
        if (value < 16 || (value & 15)) return SPARBIT_ERR_ARG;
        g_flow_chunk_bytes = value;
    } else if (!std::strcmp(key, "nontemporal")) {
        g_nontemporal = value ? 1 : 0;
    } else if (!std::strcmp(key, "wgs_per_cu")) {
        if (value < 1 || value > 16) return SPARBIT_ERR_ARG;
        g_wgs_per_cu = value;
    } else if (!std::strcmp(key, "line_align_min_bytes")) {
        if (value < 16) return SPARBIT_ERR_ARG;
        g_line_align_min_bytes = value;
    } else if (!std::strcmp(key, "var_idle_max")) {
        if (value < 0) return SPARBIT_ERR_ARG;
        g_var_idle_max = value;
    } else if (!std::strcmp(key, "realign_min_bytes")) {
        if (value < 16) return SPARBIT_ERR_ARG;
        g_realign_min_bytes = value;
    } else if (!std::strcmp(key, "tree_auto")) {
        g_tree_auto = value ? 1 : 0;
    } else if (!std::strcmp(key, "tree_auto_doubling")) {
        g_tree_auto_doubling = value ? 1 : 0;
    } else if (!std::strcmp(key, "tree_auto_ring")) {
        g_tree_auto_ring = value ? 1 : 0;
    } else if (!std::strcmp(key, "tree_gang_apart_log2")) {
        if (value < -1 || value > 10) return SPARBIT_ERR_ARG;
        g_tree_gang_apart_log2 = value;
    } else if (!std::strcmp(key, "tree_gang")) {
        if (value < -1 || (value > 1 && value != kTreeGang && value != kTreeBigGang)) return SPARBIT_ERR_ARG;
        g_tree_gang = value;
    } else if (!std::strcmp(key, "tree_hot")) {
        if (value < -1 || value > 1) return SPARBIT_ERR_ARG;
        g_tree_hot = value;
    } else if (!std::strcmp(key, "tree_team_log2")) {
        if (value < -1 || value > 4) return SPARBIT_ERR_ARG;
        g_tree_team_log2 = value;
    } else if (!std::strcmp(key, "tree_run_log2")) {
        if (value < -1 || value > 12) return SPARBIT_ERR_ARG;
        g_tree_run_log2 = value;
    } else if (!std::strcmp(key, "tree_small_bytes")) {
        if (value < 0) return SPARBIT_ERR_ARG;
        g_tree_small_bytes = value;
    } else if (!std::strcmp(key, "tree_unroll")) {
        if (value != 1 && value != 2) return SPARBIT_ERR_ARG;
        g_tree_unroll = value;
    } else if (!std::strcmp(key, "tree_store")) {
        if (value < 0 || value > 4) return SPARBIT_ERR_ARG;
        g_tree_store = value;
    } else if (!std::strcmp(key, "tree_prefetch")) {
        g_tree_prefetch = value ? 1 : 0;
    } else if (!std::strcmp(key, "tree_any_align")) {
        g_tree_any_align = value ? 1 : 0;
    } else if (!std::strcmp(key, "tree_part_line_max_bytes")) {
        if (value < 0) return SPARBIT_ERR_ARG;
        g_tree_part_line_max_bytes = value;
    } else if (!std::strcmp(key, "tree_lds_bytes")) {
        if (value < -1 || value > 65536) return SPARBIT_ERR_ARG;
        g_tree_lds_bytes = value;
    } else if (!std::strcmp(key, "spin_limit_ms")) {
        if (value < 0 || value > 60000) return SPARBIT_ERR_ARG;
        g_spin_limit_ms = value;
    } else {
        return SPARBIT_ERR_ARG;
    }
    return SPARBIT_OK;
}

}  // extern "C"
