// libbcsched: round-optimal broadcast schedules on a circulant graph, built on gfx950.
//
// Method: J. L. Traff, arXiv 2205.10072, Section 2 (Alg. 1, 2, 4, 5; index arithmetic of Alg. 6).
// One lane owns one rank.  Everything is 32-bit integer work on the vector ALU; block sets are
// 32-bit masks (q <= 31); the skips of a uniform-p launch live in scalar registers.
//
// The per-rank construction is in bcs_core.h, the kernels in bcs_kernels_*.h; this file holds the launch and
// timing helpers, the host logic and the C ABI.
#include <hip/hip_runtime.h>
#include <hip/hip_ext.h>
#include <stdint.h>
#include <mutex>
#include <utility>

#include "bcsched.h"
#include "bcs_core.h"
#include "bcs_kernels_common.h"

namespace {

thread_local int g_last_hip = 0;

inline int hip_fail(hipError_t e) {
    g_last_hip = (int)e;
    return BCS_EHIP;
}

// Optional per-kernel device timing (bcs_timing_begin / bcs_timing_end): while it is on, a launch is
// given a start and a stop event from a fixed pool, so its duration is the device's own.
enum KernelId {
    kRecv = 0, kSendLookup, kSendRecompute, kBatch, kExpand, kFill, kValuPeak, kAllgather, kPackPlan, kPackCopy,
    kRecvExpand, kSendExpand, kExpandRows, kRowsToBytes, kDigits, kPartnerTables, kKernelCount
};
static_assert(kKernelCount == BCS_KERNEL_COUNT, "header and kernel list disagree");
const char *const kKernelNames[kKernelCount] = {"k_recv_uniform", "k_send_lookup", "k_send_recompute", "k_batch",
                                                "k_expand",       "k_fill",        "k_valu_peak",   "k_allgather_tables",
                                                "k_pack_plan",    "k_pack_copy",   "k_recv_expand", "k_send_expand",
                                                "k_expand_rows",  "k_rows_to_bytes", "k_digits",     "k_partner_tables"};
struct Timing {
    bool on = false;
    int used = 0;
    int created = 0;
    hipEvent_t start[BCS_TIMING_MAX_LAUNCHES];
    hipEvent_t stop[BCS_TIMING_MAX_LAUNCHES];
    int kid[BCS_TIMING_MAX_LAUNCHES];
};
Timing g_timing;

template <class... KArgs, class... Args>
void launch_lds(int kid, void (*kernel)(KArgs...), dim3 grid, dim3 block, unsigned lds_bytes, hipStream_t st,
                Args... args) {
    Timing &t = g_timing;
    if (t.on && t.used < BCS_TIMING_MAX_LAUNCHES) {
        if (t.used == t.created) {
            if (hipEventCreate(&t.start[t.created]) == hipSuccess) {
                if (hipEventCreate(&t.stop[t.created]) == hipSuccess) ++t.created;
                else (void)hipEventDestroy(t.start[t.created]);
            }
        }
        if (t.used < t.created) {
            const int slot = t.used++;
            t.kid[slot] = kid;
            hipExtLaunchKernelGGL(kernel, grid, block, lds_bytes, st, t.start[slot], t.stop[slot], 0, args...);
            return;
        }
    }
    hipLaunchKernelGGL(kernel, grid, block, lds_bytes, st, args...);
}

template <class... KArgs, class... Args>
void launch(int kid, void (*kernel)(KArgs...), dim3 grid, dim3 block, hipStream_t st, Args... args) {
    launch_lds(kid, kernel, grid, block, 0u, st, args...);
}

}  // namespace

#include "bcs_kernels_sched.h"
#include "bcs_kernels_expand.h"
#include "bcs_kernels_allgather.h"

namespace {

// Measurement aid: the practical ceiling the `alu` roofline is set against.  kValuChains independent chains of
// full-rate 32-bit integer vector ops of the kinds the construction is made of (add, xor, min, subtract), written
// as instructions so that the count is exact: `iters` rounds of 4 ops per chain and lane, no memory traffic
// until one word per lane at the end.
constexpr int kValuChains = 8;
static_assert(4 * kValuChains == BCS_VALU_PEAK_OPS_PER_ITER, "header and calibration kernel disagree");

__global__ __launch_bounds__(kBlock) void k_valu_peak(uint32_t iters, uint32_t seed, uint32_t *__restrict__ sink) {
    uint32_t x[kValuChains];
#pragma unroll
    for (int c = 0; c < kValuChains; ++c) x[c] = seed + threadIdx.x * (2u * c + 1u) + blockIdx.x;
    const uint32_t k1 = seed | 1u, k2 = seed ^ 0x9e3779b9u, k3 = 0xfffffff1u;
#pragma unroll 1
    for (uint32_t it = 0; it < iters; ++it) {
#pragma unroll
        for (int c = 0; c < kValuChains; ++c) asm volatile("v_add_u32 %0, %1, %0" : "+v"(x[c]) : "s"(k1));
#pragma unroll
        for (int c = 0; c < kValuChains; ++c) asm volatile("v_xor_b32 %0, %1, %0" : "+v"(x[c]) : "s"(k2));
#pragma unroll
        for (int c = 0; c < kValuChains; ++c) asm volatile("v_min_u32 %0, %1, %0" : "+v"(x[c]) : "s"(k3));
#pragma unroll
        for (int c = 0; c < kValuChains; ++c) asm volatile("v_subrev_u32 %0, %1, %0" : "+v"(x[c]) : "s"(k1));
    }
    uint32_t acc = 0;
#pragma unroll
    for (int c = 0; c < kValuChains; ++c) acc ^= x[c];
    sink[(size_t)blockIdx.x * kBlock + threadIdx.x] = acc;
}

__global__ void k_fill(int32_t *__restrict__ out, uint64_t n, int32_t value) {
    const uint64_t stride = (uint64_t)gridDim.x * blockDim.x;
    for (uint64_t e = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x; e < n; e += stride) out[e] = value;
}

// ----------------------------------------------------------------------------------------------
// Host side
// ----------------------------------------------------------------------------------------------
int host_q(int32_t p) {
    int q = 0;
    while (((int64_t)1 << q) < (int64_t)p) ++q;
    return q;
}

// The skips of Alg. 1 by the closed form its halving produces: skips[k] = ceil(p / 2^(q-k)).
int host_skips(int32_t p, SkipTab &t) {
    const int q = host_q(p);
    for (int k = 0; k <= q; ++k) t.s[k] = (((uint32_t)p - 1u) >> (q - k)) + 1u;
    for (int j = q + 1; j < kMaxQ + 2; ++j) t.s[j] = (uint32_t)p;
    t.odd = odd_levels((uint32_t)p, q);
    return q;
}

// Fills g_lowtab on first use per device.  The fill is enqueued on the first caller's stream; until
// it has finished, callers on other streams are made to wait for it on the device.
struct LowTabState {
    bool launched = false;
    bool done = false;
    hipStream_t stream = nullptr;
    hipEvent_t ready = nullptr;
};
constexpr int kMaxDevices = 64;
LowTabState g_lowtab_state[kMaxDevices];
std::mutex g_lowtab_mutex;

int ensure_lowtab(hipStream_t st) {
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return hip_fail(e);
    if (dev < 0 || dev >= kMaxDevices) return BCS_EINVAL;
    std::lock_guard<std::mutex> lock(g_lowtab_mutex);
    LowTabState &s = g_lowtab_state[dev];
    if (s.done) return BCS_OK;
    if (!s.launched) {
        e = hipEventCreateWithFlags(&s.ready, hipEventDisableTiming);
        if (e != hipSuccess) return hip_fail(e);
        hipLaunchKernelGGL(k_build_lowtab, dim3((kLowTableBytes + kBlock - 1) / kBlock), dim3(kBlock), 0, st);
        e = hipGetLastError();
        if (e != hipSuccess) return hip_fail(e);
        e = hipEventRecord(s.ready, st);
        if (e != hipSuccess) return hip_fail(e);
        s.launched = true;
        s.stream = st;
        return BCS_OK;
    }
    if (hipEventQuery(s.ready) == hipSuccess) {
        s.done = true;
        return BCS_OK;
    }
    (void)hipGetLastError();                       // hipErrorNotReady is not an error here
    if (st != s.stream) {
        e = hipStreamWaitEvent(st, s.ready, 0);
        if (e != hipSuccess) return hip_fail(e);
    }
    return BCS_OK;
}

// The per-device scratch of the plain calls.  One allocation serves every plain call on the device, so two of
// them on different streams must not overlap: when a call comes on another stream than the one before it, that
// earlier stream's work is made a dependency of the new one (an event recorded there now covers everything
// the earlier call enqueued).
struct Scratch {
    void *ptr = nullptr;
    size_t bytes = 0;
    bool used = false;
    hipStream_t last = nullptr;
    hipEvent_t order = nullptr;
};
Scratch g_scratch[kMaxDevices];
std::mutex g_scratch_mutex;

int scratch_get(size_t bytes, hipStream_t st, void **out) {
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return hip_fail(e);
    if (dev < 0 || dev >= kMaxDevices) return BCS_EINVAL;
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    Scratch &s = g_scratch[dev];
    if (s.bytes < bytes) {
        if (s.ptr) {
            e = hipDeviceSynchronize();            // the one place a call waits: work may still use the old block
            if (e != hipSuccess) return hip_fail(e);
            e = hipFree(s.ptr);
            s.ptr = nullptr;
            s.bytes = 0;
            s.used = false;
            if (e != hipSuccess) return hip_fail(e);
        }
        e = hipMalloc(&s.ptr, bytes);
        if (e != hipSuccess) {
            s.ptr = nullptr;
            (void)hipGetLastError();
            g_last_hip = (int)e;
            return BCS_ENOMEM;
        }
        s.bytes = bytes;
    }
    if (s.used && s.last != st) {
        if (!s.order) {
            e = hipEventCreateWithFlags(&s.order, hipEventDisableTiming);
            if (e != hipSuccess) return hip_fail(e);
        }
        e = hipEventRecord(s.order, s.last);
        if (e == hipSuccess) {
            e = hipStreamWaitEvent(st, s.order, 0);
        } else {                                   // the earlier stream is gone: wait for whatever it left behind
            (void)hipGetLastError();
            e = hipDeviceSynchronize();
        }
        if (e != hipSuccess) return hip_fail(e);
    }
    s.used = true;
    s.last = st;
    *out = s.ptr;
    return BCS_OK;
}

inline uint64_t round_up(uint64_t v, uint64_t m) { return (v + m - 1) / m * m; }

// row length of the slot-major receive table (rows start on 256-byte boundaries)
inline uint64_t slot_ld(int32_t p) { return round_up((uint64_t)p, 256); }

template <int Q>
int launch_sched(const SkipTab &tab, uint32_t root, uint32_t r0, uint32_t r1, int32_t *recv_out, int32_t *send_out,
                 slot_t *recvT, uint64_t ldT, int8_t *recvB, int8_t *sendB, uint32_t *dtab, hipStream_t st) {
    const uint64_t count = (uint64_t)r1 - r0;
    const unsigned blocks = (unsigned)((count + kBlock - 1) / kBlock);
    const bool full = (r0 == 0 && r1 == tab.s[Q]);
    // the slot-major copy feeds the send look-up; with neither table asked for it is the only output
    const bool want_t = full && recvT && (send_out || !recv_out);
    if (recv_out || want_t) {
        const bool tabbed = dtab != nullptr;     // one walk a rank (all p of them) into the table, the rows read it
        if (tabbed)
            launch(kDigits, k_digits<Q>, dim3((unsigned)(((uint64_t)tab.s[Q] + kBlock - 1) / kBlock)), dim3(kBlock), st,
                   tab, dtab);
        slot_t *const t_out = want_t ? recvT : (slot_t *)nullptr;
        const uint32_t *const d_in = dtab;
        if (full && recvB && recv_out) {
            if (tabbed)
                launch(kRecv, k_recv_uniform<Q, true, true>, dim3(blocks), dim3(kBlock), st, tab, root, r0, r1,
                       recv_out, t_out, ldT, recvB, d_in);
            else
                launch(kRecv, k_recv_uniform<Q, true, false>, dim3(blocks), dim3(kBlock), st, tab, root, r0, r1,
                       recv_out, t_out, ldT, recvB, d_in);
        } else {
            if (tabbed)
                launch(kRecv, k_recv_uniform<Q, false, true>, dim3(blocks), dim3(kBlock), st, tab, root, r0, r1,
                       recv_out, t_out, ldT, (int8_t *)nullptr, d_in);
            else
                launch(kRecv, k_recv_uniform<Q, false, false>, dim3(blocks), dim3(kBlock), st, tab, root, r0, r1,
                       recv_out, t_out, ldT, (int8_t *)nullptr, d_in);
        }
    }
    if (send_out) {
        if (full) {
            constexpr int G = Q >= kLookupBigMinQ ? kLookupBigG : kLookupSmallG;
            launch(kSendLookup, k_send_lookup<Q, G>, dim3((unsigned)((count + G - 1) / G)), dim3(kLookupLanes), st, tab,
                   (const slot_t *)recvT, ldT, send_out, sendB);
        } else if (dtab) {
            if (!recv_out)                      // no receive rows asked for: the table has not been filled yet
                launch(kDigits, k_digits<Q>, dim3((unsigned)(((uint64_t)tab.s[Q] + kBlock - 1) / kBlock)), dim3(kBlock),
                       st, tab, dtab);
            launch(kSendRecompute, k_send_recompute<Q, true>, dim3(blocks), dim3(kBlock), st, tab, root, r0, r1, send_out,
                   (const uint32_t *)dtab);
        } else {
            launch(kSendRecompute, k_send_recompute<Q, false>, dim3(blocks), dim3(kBlock), st, tab, root, r0, r1,
                   send_out, (const uint32_t *)nullptr);
        }
    }
    hipError_t e = hipGetLastError();
    return e == hipSuccess ? BCS_OK : hip_fail(e);
}

typedef int (*LaunchFn)(const SkipTab &, uint32_t, uint32_t, uint32_t, int32_t *, int32_t *, slot_t *, uint64_t,
                        int8_t *, int8_t *, uint32_t *, hipStream_t);

template <int... Qs>
constexpr void fill_table(LaunchFn *t, std::integer_sequence<int, Qs...>) {
    ((t[Qs] = &launch_sched<Qs + 1>), ...);
}

LaunchFn launch_for_q(int q) {
    struct Table {
        LaunchFn fn[kMaxQ];
        Table() { fill_table(fn, std::make_integer_sequence<int, kMaxQ>{}); }
    };
    static const Table table;                  // initialised once, thread-safe
    return table.fn[q - 1];
}

ExpandArgs expand_args(uint64_t rows, uint64_t R, int q, int32_t n, const void *out) {
    ExpandArgs ea;
    ea.total = rows * R;
    ea.rows = rows;
    ea.R = (uint32_t)R;
    ea.q = (uint32_t)q;
    ea.x = (uint32_t)((q - (int)(R % (uint64_t)q)) % q);
    ea.nm1 = n - 1;
    ea.step_rows = (uint32_t)((kBlock * 4u) / R);
    ea.step_j = (uint32_t)((kBlock * 4u) % R);
    ea.step_k = ea.step_j % (uint32_t)q;
    ea.wrap_k = (uint32_t)q - (uint32_t)(R % (uint64_t)q);
    ea.aligned = (((uintptr_t)out) & 15u) == 0 ? 1 : 0;
    ea.magic_R = (uint32_t)((1ull << 32) / R + 1ull);
    ea.magic_q = q >= 2 ? (uint32_t)((1ull << 32) / (uint64_t)q + 1ull) : 0u;
    ea.magic_w = (uint32_t)((1ull << 32) / (uint64_t)(q + kExpPad) + 1ull);
    return ea;
}

// Fused construction + expansion of all ranks (tiles of 256 rows).  Measured on MI355X against the
// separate kernels for p = 2^12 .. 2^22 and n = 1 .. 1024: 15-40 % less time while rows are short (the
// schedule rows are a large share of the traffic, and two launches replace four); for longer rows the
// flat stream of k_expand, whose workgroups are small and many, writes faster than a tile at a time.
constexpr uint64_t kFusedShortR = 96;              // rows up to this length: fused for any p
constexpr uint64_t kFusedMaxR = 128;               // rows up to this length: fused when p >= kFusedMinP
constexpr uint32_t kFusedMinP = 1u << 16;

inline bool use_fused(int32_t p, int q, uint64_t R, bool aligned) {
    if (q < (int)kExpMinQ || R < kExpMinR || !aligned) return false;
    return R <= kFusedShortR || (R <= kFusedMaxR && (uint32_t)p >= kFusedMinP);
}

template <int Q>
int launch_fused(const SkipTab &tab, uint32_t root, const ExpandArgs &ea, int32_t *recv_out, int32_t *send_out,
                 slot_t *recvT, uint64_t ldT, int32_t *recv_blocks, int32_t *send_blocks, hipStream_t st) {
    if constexpr (Q >= (int)kExpMinQ) {
        const unsigned blocks = (unsigned)(((uint64_t)tab.s[Q] + kBlock - 1) / kBlock);
        launch(kRecvExpand, k_recv_expand<Q>, dim3(blocks), dim3(kBlock), st, tab, root, ea, recv_out, recvT, ldT,
               recv_blocks);
        launch(kSendExpand, k_send_expand<Q>, dim3(blocks), dim3(kBlock), st, tab, ea, (const slot_t *)recvT, ldT,
               send_out, send_blocks);
        hipError_t e = hipGetLastError();
        return e == hipSuccess ? BCS_OK : hip_fail(e);
    } else {
        return BCS_EINVAL;
    }
}

typedef int (*FusedFn)(const SkipTab &, uint32_t, const ExpandArgs &, int32_t *, int32_t *, slot_t *, uint64_t,
                       int32_t *, int32_t *, hipStream_t);

template <int... Qs>
constexpr void fill_fused(FusedFn *t, std::integer_sequence<int, Qs...>) {
    ((t[Qs] = &launch_fused<Qs + 1>), ...);
}

FusedFn fused_for_q(int q) {
    struct Table {
        FusedFn fn[kMaxQ];
        Table() { fill_fused(fn, std::make_integer_sequence<int, kMaxQ>{}); }
    };
    static const Table table;
    return table.fn[q - 1];
}

int check_range(int32_t p, int32_t root, int32_t r0, int32_t r1) {
    if (p < 1 || root < 0 || root >= p || r0 < 0 || r0 > r1 || r1 > p) return BCS_EINVAL;
    return BCS_OK;
}

}  // namespace

extern "C" {

int bcs_q(int32_t p) { return p < 1 ? BCS_EINVAL : host_q(p); }

int bcs_skips(int32_t p, int32_t *skips_host) {
    if (p < 1 || !skips_host) return BCS_EINVAL;
    SkipTab t;
    const int q = host_skips(p, t);
    for (int k = 0; k <= q; ++k) skips_host[k] = (int32_t)t.s[k];
    return q;
}

int64_t bcs_rounds(int32_t p, int32_t n) {
    if (p < 1 || n < 1) return BCS_EINVAL;
    return (int64_t)n - 1 + host_q(p);
}

// Scratch of a launch over all ranks with a send table: the slot-major receive table, then the digit masks of
// all ranks (one word each).
inline uint64_t slot_table_bytes(int32_t p, int q) { return slot_ld(p) * (uint64_t)q * sizeof(slot_t); }
// The digit table pays at every size (measured on MI355X: receive rows of all ranks in 0.57-0.73 of the walking
// kernel's time from 2^18 to 2^27 ranks, table pass included), with all of a row's reads issued up front.
inline uint64_t digit_table_bytes(int32_t p) { return round_up((uint64_t)p * sizeof(uint32_t), 256); }

// A part of the ranks with send rows (Alg. 5) takes the digit table when filling it (p walks) costs less than the
// walks it saves (about q^2 / 2 a rank).  Measured: 2^20 ranks of 2^20+1 gain 0.27 ms, 2^20 ranks of 2^27-1
// (q^2 (r1 - r0) = 5.7 p) lose 0.02 ms to the 0.32 ms the table of 2^27 ranks takes.
inline bool partial_range_tabled(int32_t p, int q, int32_t r0, int32_t r1) {
    return (uint64_t)(r1 - r0) * (uint64_t)(q * q) >= 8ull * (uint64_t)p;
}

int64_t bcs_sched_workspace_bytes(int32_t p, int32_t r0, int32_t r1, int want_send) {
    if (check_range(p, 0, r0, r1) != BCS_OK) return BCS_EINVAL;
    const int q = host_q(p);
    if (!want_send || q == 0) return 0;
    if (!(r0 == 0 && r1 == p)) return partial_range_tabled(p, q, r0, r1) ? (int64_t)digit_table_bytes(p) : 0;
    return (int64_t)(slot_table_bytes(p, q) + digit_table_bytes(p));
}

int bcs_sched_rooted_ws(int32_t p, int32_t root, int32_t r0, int32_t r1, int32_t *recv_out, int32_t *send_out,
                        void *workspace, size_t workspace_bytes, void *stream) {
    int rc = check_range(p, root, r0, r1);
    if (rc != BCS_OK) return rc;
    if (!recv_out && !send_out) return BCS_EINVAL;
    const int q = host_q(p);
    if (q == 0 || r0 == r1) return BCS_OK;
    const int64_t need = bcs_sched_workspace_bytes(p, r0, r1, send_out != nullptr);
    if (need > 0 && (!workspace || workspace_bytes < (size_t)need)) return BCS_ENOMEM;
    if (need > 0 && (((uintptr_t)workspace) & 255u)) return BCS_EINVAL;     // tables are read 4 and 16 bytes at a time
    SkipTab tab;
    host_skips(p, tab);
    rc = ensure_lowtab((hipStream_t)stream);
    if (rc != BCS_OK) return rc;
    const uint64_t ld = slot_ld(p);
    // all ranks: the digit table sits behind the slot-major table; a call for receive rows alone needs no
    // workspace, and uses one that holds the digit table if it is given
    const bool full = (r0 == 0 && r1 == p);
    uint32_t *dtab = nullptr;
    const uint64_t dbytes = digit_table_bytes(p);
    if (need > 0 && dbytes > 0) dtab = (uint32_t *)((char *)workspace + (full ? slot_table_bytes(p, q) : 0));
    else if (need == 0 && dbytes > 0 && full && workspace && workspace_bytes >= dbytes &&
             ((uintptr_t)workspace & 3u) == 0)
        dtab = (uint32_t *)workspace;
    return launch_for_q(q)(tab, (uint32_t)root, (uint32_t)r0, (uint32_t)r1, recv_out, send_out,
                           need > 0 && full ? (slot_t *)workspace : nullptr, ld, nullptr, nullptr, dtab,
                           (hipStream_t)stream);
}

int bcs_sched_rooted(int32_t p, int32_t root, int32_t r0, int32_t r1, int32_t *recv_out, int32_t *send_out,
                     void *stream) {
    int rc = check_range(p, root, r0, r1);
    if (rc != BCS_OK) return rc;
    if (!recv_out && !send_out) return BCS_EINVAL;
    const int64_t need = bcs_sched_workspace_bytes(p, r0, r1, send_out != nullptr);
    void *ws = nullptr;
    if (need > 0 && r0 != r1) {
        rc = scratch_get((size_t)need, (hipStream_t)stream, &ws);
        if (rc != BCS_OK) return rc;
    }
    return bcs_sched_rooted_ws(p, root, r0, r1, recv_out, send_out, ws, (size_t)need, stream);
}

}  // extern "C"

namespace {
// Scratch of bcs_sched_rooted_static: a fixed array in the code object, one copy per GPU.  In host code the
// array's name is only a handle for hipGetSymbolAddress; kernels and every other use take the address that
// call returns for the current device.
static __device__ __align__(256) unsigned char scratch[BCS_STATIC_SCRATCH_BYTES];

struct StaticScratch {
    void *ptr = nullptr;
    bool ready = false;
};
StaticScratch g_static[kMaxDevices];
std::mutex g_static_mutex;

int static_scratch(void **out) {
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return hip_fail(e);
    if (dev < 0 || dev >= kMaxDevices) return BCS_EINVAL;
    std::lock_guard<std::mutex> lock(g_static_mutex);
    StaticScratch &s = g_static[dev];
    if (!s.ready) {
        void *ptr = nullptr;
        e = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));      // this device's copy
        if (e != hipSuccess) return hip_fail(e);
        if (!ptr || (((uintptr_t)ptr) & 255u)) return BCS_EINVAL;
        s.ptr = ptr;
        s.ready = true;
    }
    *out = s.ptr;
    return BCS_OK;
}
}  // namespace

extern "C" {

int bcs_sched_rooted_static(int32_t p, int32_t root, int32_t r0, int32_t r1, int32_t *recv_out, int32_t *send_out,
                            void *stream) {
    int rc = check_range(p, root, r0, r1);
    if (rc != BCS_OK) return rc;
    if (!recv_out && !send_out) return BCS_EINVAL;
    const int64_t need = bcs_sched_workspace_bytes(p, r0, r1, send_out != nullptr);
    if (need < 0) return (int)need;
    if ((uint64_t)need > (uint64_t)BCS_STATIC_SCRATCH_BYTES) return BCS_ETOOBIG;
    void *ws = nullptr;
    if (need > 0 && r0 != r1) {
        rc = static_scratch(&ws);
        if (rc != BCS_OK) return rc;
    }
    return bcs_sched_rooted_ws(p, root, r0, r1, recv_out, send_out, ws, ws ? (size_t)need : 0, stream);
}

int bcs_sched(int32_t p, int32_t r0, int32_t r1, int32_t *recv_out, int32_t *send_out, void *stream) {
    return bcs_sched_rooted(p, 0, r0, r1, recv_out, send_out, stream);
}

int bcs_sched_batch(int64_t count, const int32_t *p, const int32_t *r, const int32_t *root, int32_t *recv_out,
                    int32_t *send_out, int32_t *q_out, void *stream) {
    if (count < 0 || !p || !r || !root) return BCS_EINVAL;
    if (!recv_out && !send_out && !q_out) return BCS_EINVAL;
    if (count == 0) return BCS_OK;
    const uint64_t blocks = ((uint64_t)count + kBatchBlock - 1) / kBatchBlock;
    if (blocks > 0x7fffffffull) return BCS_EINVAL;
    const int rc = ensure_lowtab((hipStream_t)stream);
    if (rc != BCS_OK) return rc;
    launch(kBatch, k_batch, dim3((unsigned)blocks), dim3(kBatchBlock), (hipStream_t)stream, count, p, r, root,
                       recv_out, send_out, q_out);
    hipError_t e = hipGetLastError();
    return e == hipSuccess ? BCS_OK : hip_fail(e);
}

int bcs_expand(int32_t p, int32_t n, int32_t r0, int32_t r1, const int32_t *recv, const int32_t *send,
               int32_t *recv_blocks, int32_t *send_blocks, void *stream) {
    if (check_range(p, 0, r0, r1) != BCS_OK || n < 1 || n > BCS_MAX_N) return BCS_EINVAL;
    const int q = host_q(p);
    if (q == 0) {                      // rows of the input tables are empty: only the outputs count
        recv = recv_blocks;
        send = send_blocks;
    }
    if ((recv == nullptr) != (recv_blocks == nullptr)) return BCS_EINVAL;
    if ((send == nullptr) != (send_blocks == nullptr)) return BCS_EINVAL;
    if (!recv && !send) return BCS_EINVAL;
    const uint64_t rows = (uint64_t)r1 - r0;
    const uint64_t R = (uint64_t)n - 1 + q;
    if (rows == 0 || R == 0) return BCS_OK;
    hipStream_t st = (hipStream_t)stream;
    const int32_t *ins[2] = {recv, send};
    int32_t *outs[2] = {recv_blocks, send_blocks};
    for (int t = 0; t < 2; ++t) {
        if (!ins[t]) continue;
        if (q == 0) {
            launch(kFill, k_fill, dim3(1024), dim3(kBlock), st, outs[t], rows * R, (int32_t)BCS_NO_BLOCK);
            continue;
        }
        const ExpandArgs ea = expand_args(rows, R, q, n, outs[t]);
        const uint64_t blocks = (ea.total + kExpChunk - 1) / kExpChunk;
        if (blocks > 0x7fffffffull) return BCS_EINVAL;
        if (R >= kExpMinR && (uint32_t)q >= kExpMinQ) {
            // rows a chunk can touch, plus one that a lane past the end may address but never uses
            const uint64_t max_rows = (R - 1 + kExpChunk - 1) / R + 2;
            const unsigned lds_bytes = (unsigned)(max_rows * (uint64_t)(q + kExpPad) * sizeof(int32_t));
            if (R <= kExpNtMaxR)
                launch_lds(kExpand, k_expand<true>, dim3((unsigned)blocks), dim3(kBlock), lds_bytes, st, ea, ins[t],
                           outs[t]);
            else
                launch_lds(kExpand, k_expand<false>, dim3((unsigned)blocks), dim3(kBlock), lds_bytes, st, ea, ins[t],
                           outs[t]);
        } else {
            launch(kExpand, k_expand_small, dim3((unsigned)blocks), dim3(kBlock), st, ea, ins[t], outs[t]);
        }
    }
    hipError_t e = hipGetLastError();
    return e == hipSuccess ? BCS_OK : hip_fail(e);
}

namespace {
// bytes of one rank-major byte table (p rows and one spare that the last row's lanes may read)
inline uint64_t byte_rows_bytes(int32_t p, int q) { return round_up(((uint64_t)p + 1) * byte_row_stride(q), 256); }
inline bool byte_rows_apply(int32_t p, int q, uint64_t R) {
    return q >= (int)kExpMinQ && R >= kExpMinR && byte_rows_bytes(p, q) <= kByteRowsMax;
}
}  // namespace

namespace {
// rows of the caller's tables from which an expansion through byte rows pays: the conversion is one more
// pass over the table and one more launch
constexpr uint64_t kExpandWsMinR = 256;
inline bool expand_ws_applies(int32_t rows, int q, uint64_t R) {
    return q >= (int)kExpMinQ && R >= kExpandWsMinR && rows > 0;
}
// rows converted and expanded at a time: their byte table fits kByteRowsMax; a multiple of 4, so that every
// chunk's piece of the output starts on a 16-byte boundary
inline uint32_t expand_ws_chunk_rows(uint32_t rows, int q) {
    const uint32_t fit = (uint32_t)(kByteRowsMax / (uint64_t)byte_row_stride(q) - 1) & ~3u;
    return rows < fit ? rows : fit;
}

ExpandRowsArgs expand_rows_args(uint64_t rows, uint64_t R, int q, int32_t n) {
    ExpandRowsArgs ra;
    ra.total = rows * R;
    ra.magic_R64 = ~0ull / R + 1ull;
    ra.magic_R32 = (uint32_t)((1ull << 32) / R + 1ull);
    ra.magic_q = (uint32_t)((1ull << 32) / (uint64_t)q + 1ull);
    ra.R = (uint32_t)R;
    ra.q = (uint32_t)q;
    ra.x = (uint32_t)((q - (int)(R % (uint64_t)q)) % q);
    ra.RS = (uint32_t)byte_row_stride(q);
    ra.nm1 = n - 1;
    return ra;
}
}  // namespace

int64_t bcs_expand_workspace_bytes(int32_t p, int32_t n, int32_t r0, int32_t r1) {
    if (check_range(p, 0, r0, r1) != BCS_OK || n < 1 || n > BCS_MAX_N) return BCS_EINVAL;
    const int q = host_q(p);
    if (!expand_ws_applies(r1 - r0, q, (uint64_t)n - 1 + q)) return 0;
    return (int64_t)byte_rows_bytes((int32_t)expand_ws_chunk_rows((uint32_t)(r1 - r0), q), q);
}

int bcs_expand_ws(int32_t p, int32_t n, int32_t r0, int32_t r1, const int32_t *recv, const int32_t *send,
                  int32_t *recv_blocks, int32_t *send_blocks, void *workspace, size_t workspace_bytes, void *stream) {
    if (check_range(p, 0, r0, r1) != BCS_OK || n < 1 || n > BCS_MAX_N) return BCS_EINVAL;
    const int q = host_q(p);
    const uint64_t R = (uint64_t)n - 1 + q;
    const int64_t need = bcs_expand_workspace_bytes(p, n, r0, r1);
    const bool aligned = ((recv_blocks ? (uintptr_t)recv_blocks : 0) | (send_blocks ? (uintptr_t)send_blocks : 0)) % 16 == 0;
    const bool tables_ok = (recv == nullptr) == (recv_blocks == nullptr) && (send == nullptr) == (send_blocks == nullptr) &&
                           (recv || send);
    if (need <= 0 || !aligned || !tables_ok || !workspace || workspace_bytes < (size_t)need ||
        (((uintptr_t)workspace) & 15u))
        return bcs_expand(p, n, r0, r1, recv, send, recv_blocks, send_blocks, stream);
    hipStream_t st = (hipStream_t)stream;
    const uint32_t rows = (uint32_t)(r1 - r0);
    const uint32_t chunk = expand_ws_chunk_rows(rows, q);
    const uint32_t RS = (uint32_t)byte_row_stride(q), w4 = RS / 4;
    const int32_t *ins[2] = {recv, send};
    int32_t *outs[2] = {recv_blocks, send_blocks};
    // the one workspace serves every chunk of both tables in turn (same stream: a conversion follows the
    // expansion that read the previous contents)
    for (int t = 0; t < 2; ++t) {
        if (!ins[t]) continue;
        for (uint32_t c0 = 0; c0 < rows; c0 += chunk) {
            const uint32_t rc = rows - c0 < chunk ? rows - c0 : chunk;
            const ExpandRowsArgs ra = expand_rows_args(rc, R, q, n);
            const uint64_t pieces = (ra.total + kBlock * 4 - 1) / (kBlock * 4);
            if (pieces > 0x7fffffffull) return BCS_EINVAL;
            launch(kRowsToBytes, k_rows_to_bytes, dim3((rc * w4 + kBlock - 1) / kBlock), dim3(kBlock), st, rc, (uint32_t)q,
                   RS, (uint32_t)((1ull << 32) / w4 + 1ull), ins[t] + (uint64_t)c0 * q, (int8_t *)workspace);
            launch(kExpandRows, k_expand_rows, dim3((unsigned)pieces), dim3(kBlock), st, ra, (const int8_t *)workspace,
                   outs[t] + (uint64_t)c0 * R);
        }
    }
    hipError_t e = hipGetLastError();
    return e == hipSuccess ? BCS_OK : hip_fail(e);
}

int64_t bcs_sched_expand_workspace_bytes(int32_t p, int32_t n) {
    if (p < 1 || n < 1 || n > BCS_MAX_N) return BCS_EINVAL;
    const int q = host_q(p);
    const int64_t base = bcs_sched_workspace_bytes(p, 0, p, 1);
    if (byte_rows_apply(p, q, (uint64_t)n - 1 + q)) return base + (int64_t)(2 * byte_rows_bytes(p, q));
    // too many ranks for byte tables that stay in cache: the tables are expanded chunk by chunk (bcs_expand_ws)
    const int64_t extra = bcs_expand_workspace_bytes(p, n, 0, p);
    return base + (extra > 0 ? extra : 0);
}

int bcs_sched_expand_ws(int32_t p, int32_t root, int32_t n, int32_t *recv_out, int32_t *send_out,
                        int32_t *recv_blocks, int32_t *send_blocks, void *workspace, size_t workspace_bytes,
                        void *stream) {
    if (p < 1 || root < 0 || root >= p || n < 1 || n > BCS_MAX_N) return BCS_EINVAL;
    const int q = host_q(p);
    const uint64_t R = (uint64_t)n - 1 + q;
    if (R == 0) return BCS_OK;                     // one process, one block: every table is empty
    if (!recv_blocks || !send_blocks) return BCS_EINVAL;
    if (q > 0 && (!recv_out || !send_out)) return BCS_EINVAL;
    if (workspace && workspace_bytes > 0 && (((uintptr_t)workspace) & 255u)) return BCS_EINVAL;
    const bool aligned = ((((uintptr_t)recv_blocks) | ((uintptr_t)send_blocks)) & 15u) == 0;
    if (!use_fused(p, q, R, aligned)) {
        const int64_t base = q > 0 ? bcs_sched_workspace_bytes(p, 0, p, 1) : 0;
        const uint64_t rows_bytes = q > 0 ? byte_rows_bytes(p, q) : 0;
        if (byte_rows_apply(p, q, R) && aligned && workspace && workspace_bytes >= (size_t)base + 2 * rows_bytes) {
            // long rows: the schedule kernels also leave byte rows, which the expansion then reads from cache
            SkipTab tab;
            host_skips(p, tab);
            int rc = ensure_lowtab((hipStream_t)stream);
            if (rc != BCS_OK) return rc;
            const ExpandRowsArgs ra = expand_rows_args((uint64_t)p, R, q, n);
            const uint64_t pieces = (ra.total + kBlock * 4 - 1) / (kBlock * 4);
            if (pieces > 0x7fffffffull) return BCS_EINVAL;
            int8_t *recvB = (int8_t *)workspace + base, *sendB = recvB + rows_bytes;
            rc = launch_for_q(q)(tab, (uint32_t)root, 0u, (uint32_t)p, recv_out, send_out, (slot_t *)workspace,
                                 slot_ld(p), recvB, sendB,
                                 digit_table_bytes(p) ? (uint32_t *)((char *)workspace + slot_table_bytes(p, q)) : nullptr,
                                 (hipStream_t)stream);
            if (rc != BCS_OK) return rc;
            int32_t *outs[2] = {recv_blocks, send_blocks};
            const int8_t *srcs[2] = {recvB, sendB};
            for (int t = 0; t < 2; ++t) {
                launch(kExpandRows, k_expand_rows, dim3((unsigned)pieces), dim3(kBlock), (hipStream_t)stream, ra,
                       srcs[t], outs[t]);
            }
            hipError_t e = hipGetLastError();
            return e == hipSuccess ? BCS_OK : hip_fail(e);
        }
        if (q > 0) {
            const int rc = bcs_sched_rooted_ws(p, root, 0, p, recv_out, send_out, workspace, workspace_bytes, stream);
            if (rc != BCS_OK) return rc;
        }
        // what the workspace holds beyond the schedules' scratch serves the expansion (chunks of byte rows)
        const bool more = workspace && workspace_bytes > (size_t)base;
        return bcs_expand_ws(p, n, 0, p, recv_out, send_out, recv_blocks, send_blocks,
                             more ? (char *)workspace + base : nullptr, more ? workspace_bytes - (size_t)base : 0, stream);
    }
    const int64_t need = bcs_sched_workspace_bytes(p, 0, p, 1);
    if (!workspace || workspace_bytes < (size_t)need) return BCS_ENOMEM;
    SkipTab tab;
    host_skips(p, tab);
    const int rc = ensure_lowtab((hipStream_t)stream);
    if (rc != BCS_OK) return rc;
    const ExpandArgs ea = expand_args((uint64_t)p, R, q, n, recv_blocks);
    return fused_for_q(q)(tab, (uint32_t)root, ea, recv_out, send_out, (slot_t *)workspace,
                          slot_ld(p), recv_blocks, send_blocks, (hipStream_t)stream);
}

int bcs_sched_expand(int32_t p, int32_t root, int32_t n, int32_t *recv_out, int32_t *send_out, int32_t *recv_blocks,
                     int32_t *send_blocks, void *stream) {
    if (p < 1 || root < 0 || root >= p || n < 1 || n > BCS_MAX_N) return BCS_EINVAL;
    if ((uint64_t)n - 1 + host_q(p) > 0) {         // nothing is required of an empty result
        if (!recv_blocks || !send_blocks) return BCS_EINVAL;
        if (p > 1 && (!recv_out || !send_out)) return BCS_EINVAL;
    }
    const int64_t need = bcs_sched_expand_workspace_bytes(p, n);
    void *ws = nullptr;
    if (need > 0) {
        const int rc = scratch_get((size_t)need, (hipStream_t)stream, &ws);
        if (rc != BCS_OK) return rc;
    }
    return bcs_sched_expand_ws(p, root, n, recv_out, send_out, recv_blocks, send_blocks, ws, (size_t)need, stream);
}

int bcs_release(void) {
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return hip_fail(e);
    if (dev < 0 || dev >= kMaxDevices) return BCS_EINVAL;
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    Scratch &s = g_scratch[dev];
    if (s.ptr) {
        e = hipDeviceSynchronize();
        if (e != hipSuccess) return hip_fail(e);
        e = hipFree(s.ptr);
        s.ptr = nullptr;
        s.bytes = 0;
        s.used = false;
        if (e != hipSuccess) return hip_fail(e);
    }
    return BCS_OK;
}

int64_t bcs_allgather_workspace_bytes(int32_t p) {
    if (p < 1) return BCS_EINVAL;
    return bcs_sched_workspace_bytes(p, 0, p, 1);
}

int bcs_allgather_tables_ws(int32_t p, int32_t n, int32_t r, int32_t *pack_idx, int32_t *unpack_idx, void *workspace,
                            size_t workspace_bytes, void *stream) {
    if (p < 1 || n < 1 || n > BCS_MAX_N || r < 0 || r >= p) return BCS_EINVAL;
    if (!pack_idx && !unpack_idx) return BCS_EINVAL;
    const int q = host_q(p);
    const uint64_t R = (uint64_t)n - 1 + q;
    if (R == 0) return BCS_OK;
    hipStream_t st = (hipStream_t)stream;
    if (q == 0) {                                  // one process: nothing ever moves
        if (pack_idx) launch(kFill, k_fill, dim3(64), dim3(kBlock), st, pack_idx, R, (int32_t)BCS_NO_BLOCK);
        if (unpack_idx) launch(kFill, k_fill, dim3(64), dim3(kBlock), st, unpack_idx, R, (int32_t)BCS_NO_BLOCK);
        hipError_t e0 = hipGetLastError();
        return e0 == hipSuccess ? BCS_OK : hip_fail(e0);
    }
    const int64_t need = bcs_allgather_workspace_bytes(p);
    if (!workspace || workspace_bytes < (size_t)need) return BCS_ENOMEM;
    if (((uintptr_t)workspace) & 255u) return BCS_EINVAL;
    SkipTab tab;
    host_skips(p, tab);
    int rc = ensure_lowtab(st);
    if (rc != BCS_OK) return rc;
    const uint64_t ld = slot_ld(p);
    slot_t *recvT = (slot_t *)workspace;
    uint32_t *dtab = digit_table_bytes(p) ? (uint32_t *)((char *)workspace + slot_table_bytes(p, q)) : nullptr;
    rc = launch_for_q(q)(tab, 0u, 0u, (uint32_t)p, nullptr, nullptr, recvT, ld, nullptr, nullptr, dtab, st);
    if (rc != BCS_OK) return rc;
    const unsigned bx = (unsigned)(((uint64_t)p + kAgChunk - 1) / kAgChunk);
    const uint32_t x = (uint32_t)((q - (int)(R % (uint64_t)q)) % q);
    const bool vec = ((((uintptr_t)pack_idx) | ((uintptr_t)unpack_idx)) & 15u) == 0;
    if (vec) {
        AgFlatArgs fa;
        fa.total = R * (uint64_t)p;
        fa.magic_p = ~0ull / (uint64_t)p + 1ull;
        fa.p = (uint32_t)p;
        fa.q = (uint32_t)q;
        fa.r = (uint32_t)r;
        fa.x = x;
        fa.nm1 = n - 1;
        fa.magic_q = (uint32_t)((1ull << 32) / (uint64_t)q + 1ull);
        const uint64_t pieces = (fa.total + kBlock * 4 - 1) / (kBlock * 4);
        if (pieces > 0x7fffffffull) return BCS_EINVAL;
        launch(kAllgather, k_allgather_tables_flat, dim3((unsigned)pieces, (pack_idx && unpack_idx) ? 2u : 1u),
               dim3(kBlock), st, tab, fa, (const slot_t *)recvT, ld, pack_idx, unpack_idx);
    } else {
        launch(kAllgather, k_allgather_tables, dim3(bx, (unsigned)q), dim3(kBlock), st, tab, q, (uint32_t)r, x,
               (int32_t)(n - 1), R, (const slot_t *)recvT, ld, pack_idx, unpack_idx);
    }
    hipError_t e = hipGetLastError();
    return e == hipSuccess ? BCS_OK : hip_fail(e);
}

int bcs_allgather_tables(int32_t p, int32_t n, int32_t r, int32_t *pack_idx, int32_t *unpack_idx, void *stream) {
    if (p < 1 || n < 1 || n > BCS_MAX_N || r < 0 || r >= p) return BCS_EINVAL;
    if (!pack_idx && !unpack_idx) return BCS_EINVAL;
    const int64_t need = bcs_allgather_workspace_bytes(p);
    void *ws = nullptr;
    if (need > 0) {
        const int rc = scratch_get((size_t)need, (hipStream_t)stream, &ws);
        if (rc != BCS_OK) return rc;
    }
    return bcs_allgather_tables_ws(p, n, r, pack_idx, unpack_idx, ws, (size_t)need, stream);
}

int bcs_allgather_plan(int32_t p, int32_t r, int32_t *to, int32_t *from, int32_t *count, int32_t *recv_first) {
    if (p < 1 || r < 0 || r >= p || !to || !from || !count || !recv_first) return BCS_EINVAL;
    SkipTab t;
    const int q = host_skips(p, t);
    for (int k = 0; k < q; ++k) {
        const uint32_t s = t.s[k];
        to[k] = (int32_t)((uint32_t)r >= s ? (uint32_t)r - s : (uint32_t)r + (uint32_t)p - s);
        const uint32_t f = (uint32_t)r + s;
        from[k] = (int32_t)(f >= (uint32_t)p ? f - (uint32_t)p : f);
        count[k] = (int32_t)(t.s[k + 1] - s);
        recv_first[k] = (int32_t)s;
    }
    return q;
}

int bcs_census_plan(int32_t p, int32_t r, int32_t *to, int32_t *from, int32_t *own) {
    if (p < 1 || r < 0 || r >= p || !to || !from || !own) return BCS_EINVAL;
    SkipTab t;
    const int q = host_skips(p, t);
    for (int k = 0; k < q; ++k) {
        const bool odd = ((t.odd >> k) & 1u) != 0;             // 2 skips[k] - skips[k+1] = 1
        const uint32_t s = t.s[k] - (odd ? 1u : 0u);            // partner distance
        to[k] = (int32_t)((uint32_t)r >= s ? (uint32_t)r - s : (uint32_t)r + (uint32_t)p - s);
        const uint32_t f = (uint32_t)r + s;
        from[k] = (int32_t)(f >= (uint32_t)p ? f - (uint32_t)p : f);
        own[k] = odd ? 0 : 1;
    }
    return q;
}

}  // extern "C"

namespace {
int partner_tables(int32_t p, int32_t r0, int32_t r1, uint32_t census, int32_t *to, int32_t *from, void *stream) {
    if (p < 1 || r0 < 0 || r0 > r1 || r1 > p) return BCS_EINVAL;
    const int q = host_q(p);
    const uint64_t total = (uint64_t)(r1 - r0) * (uint64_t)q;
    if (total == 0) return BCS_OK;                                          // p = 1 or an empty range
    if (!to && !from) return BCS_EINVAL;
    const uint64_t blocks = (total + kBlock * 4 - 1) / (kBlock * 4);       // at most 2^31 * 31 / 1024
    const bool vec = ((((uintptr_t)to) | ((uintptr_t)from)) & 15u) == 0;
    if (vec)
        launch(kPartnerTables, k_partner_tables<true>, dim3((unsigned)blocks), dim3(kBlock), (hipStream_t)stream,
               (uint32_t)p, (uint32_t)q, census, (uint32_t)r0, total, to, from);
    else
        launch(kPartnerTables, k_partner_tables<false>, dim3((unsigned)blocks), dim3(kBlock), (hipStream_t)stream,
               (uint32_t)p, (uint32_t)q, census, (uint32_t)r0, total, to, from);
    hipError_t e = hipGetLastError();
    return e == hipSuccess ? BCS_OK : hip_fail(e);
}
}  // namespace

extern "C" {

int bcs_allgather_partners(int32_t p, int32_t r0, int32_t r1, int32_t *to, int32_t *from, void *stream) {
    return partner_tables(p, r0, r1, 0u, to, from, stream);
}

int bcs_census_partners(int32_t p, int32_t r0, int32_t r1, int32_t *to, int32_t *from, void *stream) {
    return partner_tables(p, r0, r1, 1u, to, from, stream);
}

int64_t bcs_pack_workspace_bytes(int32_t p) {
    if (p < 1) return BCS_EINVAL;
    const uint64_t groups = ((uint64_t)p + kPlanRoots - 1) / kPlanRoots;
    return (int64_t)(((uint64_t)p + groups + 1) * sizeof(int64_t));
}

namespace {
int pack_plan(int32_t p, int32_t n, const int32_t *idx, const int64_t *displs, int64_t *offsets, void *workspace,
              size_t workspace_bytes, hipStream_t st, PackPlan &plan) {
    if (p < 1 || n < 1 || !idx || !displs || !offsets) return BCS_EINVAL;
    const int64_t need = bcs_pack_workspace_bytes(p);
    if (!workspace || workspace_bytes < (size_t)need || (((uintptr_t)workspace) & 7u)) return BCS_ENOMEM;
    const uint32_t groups = (uint32_t)(((uint64_t)p + kPlanRoots - 1) / kPlanRoots);
    plan.offsets = offsets;
    plan.src = (int64_t *)workspace;
    plan.totals = plan.src + p;
    if ((uint32_t)p <= kPlanOneMaxP) {
        launch(kPackPlan, k_pack_plan_one, dim3(1), dim3(kBlock), st, (uint32_t)p, (uint32_t)n, idx, displs, plan);
    } else {
        launch(kPackPlan, k_pack_plan_local, dim3(groups), dim3(kBlock), st, (uint32_t)p, (uint32_t)n, idx, displs,
               plan);
        launch(kPackPlan, k_pack_plan_totals, dim3(1), dim3(kBlock), st, (uint32_t)p, groups, plan);
        launch(kPackPlan, k_pack_plan_finish, dim3(((unsigned)p + kBlock - 1) / kBlock), dim3(kBlock), st, (uint32_t)p,
               plan);
    }
    hipError_t e = hipGetLastError();
    return e == hipSuccess ? BCS_OK : hip_fail(e);
}
}  // namespace

}  // extern "C"

namespace {
// the payload kernel of one round: PACK moves blocks into the message, !PACK the message into the blocks
template <bool PACK>
int launch_copy(int32_t p, int64_t limit, const int64_t *offsets, const int64_t *src, int32_t *data, int32_t *message,
                hipStream_t st) {
    const int aligned = (int)((((uintptr_t)message) & 15u) == 0);
    if (limit < kCopyShort) {
        const uint64_t blocks = ((uint64_t)limit + kBlock * 4 - 1) / (kBlock * 4);
        launch(kPackCopy, k_pack_copy<PACK, 1>, dim3((unsigned)blocks), dim3(kBlock), st, (uint32_t)p, limit, offsets, src,
               data, message, aligned);
    } else {
        const uint64_t chunk = (uint64_t)kCopyIter * kBlock * 4;
        const uint64_t blocks = ((uint64_t)limit + chunk - 1) / chunk;
        launch(kPackCopy, k_pack_copy<PACK, kCopyIter>, dim3((unsigned)blocks), dim3(kBlock), st, (uint32_t)p, limit,
               offsets, src, data, message, aligned);
    }
    hipError_t e = hipGetLastError();
    return e == hipSuccess ? BCS_OK : hip_fail(e);
}
inline bool copy_size_ok(int64_t limit) { return ((uint64_t)limit + kBlock * 4 - 1) / (kBlock * 4) <= 0x7fffffffull; }
}  // namespace

extern "C" {

int bcs_pack_round(int32_t p, int32_t n, const int32_t *idx, const int64_t *displs, const int32_t *data,
                   int32_t *packed, int64_t capacity, int64_t *offsets, void *workspace, size_t workspace_bytes,
                   void *stream) {
    if (!data || capacity < 0 || (!packed && capacity > 0)) return BCS_EINVAL;
    if (!copy_size_ok(capacity)) return BCS_EINVAL;
    PackPlan plan;
    const int rc = pack_plan(p, n, idx, displs, offsets, workspace, workspace_bytes, (hipStream_t)stream, plan);
    if (rc != BCS_OK || capacity == 0) return rc;
    return launch_copy<true>(p, capacity, offsets, plan.src, const_cast<int32_t *>(data), packed, (hipStream_t)stream);
}

int bcs_unpack_round(int32_t p, int32_t n, const int32_t *idx, const int64_t *displs, int32_t *data,
                     const int32_t *packed, int64_t length, int64_t *offsets, void *workspace, size_t workspace_bytes,
                     void *stream) {
    if (!data || length < 0 || (!packed && length > 0)) return BCS_EINVAL;
    if (!copy_size_ok(length)) return BCS_EINVAL;
    PackPlan plan;
    const int rc = pack_plan(p, n, idx, displs, offsets, workspace, workspace_bytes, (hipStream_t)stream, plan);
    if (rc != BCS_OK || length == 0) return rc;
    return launch_copy<false>(p, length, offsets, plan.src, data, const_cast<int32_t *>(packed), (hipStream_t)stream);
}

int bcs_pack_plan_rounds(int32_t p, int32_t n, int64_t rounds, const int32_t *idx_table, const int64_t *displs,
                         int64_t *offsets_all, int64_t *src_all, void *stream) {
    if (p < 1 || n < 1 || rounds < 0 || rounds > 0x7fffffffll || !idx_table || !displs || !offsets_all || !src_all)
        return BCS_EINVAL;
    if ((((uintptr_t)offsets_all) | ((uintptr_t)src_all)) & 7u) return BCS_EINVAL;
    if (rounds == 0) return BCS_OK;
    PackPlan all;
    all.offsets = offsets_all;
    all.src = src_all;
    all.totals = nullptr;
    launch(kPackPlan, k_pack_plan_one, dim3((unsigned)rounds), dim3(kBlock), (hipStream_t)stream, (uint32_t)p, (uint32_t)n,
           idx_table, displs, all);
    hipError_t e = hipGetLastError();
    return e == hipSuccess ? BCS_OK : hip_fail(e);
}

int bcs_pack_round_planned(int32_t p, const int64_t *offsets, const int64_t *src, const int32_t *data, int32_t *packed,
                           int64_t capacity, void *stream) {
    if (p < 1 || !offsets || !src || !data || capacity < 0 || (!packed && capacity > 0)) return BCS_EINVAL;
    if (!copy_size_ok(capacity)) return BCS_EINVAL;
    if (capacity == 0) return BCS_OK;
    return launch_copy<true>(p, capacity, offsets, src, const_cast<int32_t *>(data), packed, (hipStream_t)stream);
}

int bcs_unpack_round_planned(int32_t p, const int64_t *offsets, const int64_t *src, int32_t *data,
                             const int32_t *packed, int64_t length, void *stream) {
    if (p < 1 || !offsets || !src || !data || length < 0 || (!packed && length > 0)) return BCS_EINVAL;
    if (!copy_size_ok(length)) return BCS_EINVAL;
    if (length == 0) return BCS_OK;
    return launch_copy<false>(p, length, offsets, src, data, const_cast<int32_t *>(packed), (hipStream_t)stream);
}

int bcs_valu_peak_launch(uint32_t blocks, uint32_t iters, uint32_t *sink, void *stream) {
    if (blocks == 0 || iters == 0 || !sink) return BCS_EINVAL;
    launch(kValuPeak, k_valu_peak, dim3(blocks), dim3(kBlock), (hipStream_t)stream, iters, 0x2205u, sink);
    hipError_t e = hipGetLastError();
    return e == hipSuccess ? BCS_OK : hip_fail(e);
}

int bcs_timing_begin(void) {
    g_timing.used = 0;
    g_timing.on = true;
    return BCS_OK;
}

int bcs_timing_stats(double *ms_sum, int64_t *launches, double *ms_min, double *ms_max) {
    Timing &t = g_timing;
    t.on = false;
    if (!ms_sum || !launches) return BCS_EINVAL;
    for (int k = 0; k < kKernelCount; ++k) {
        ms_sum[k] = 0.0;
        launches[k] = 0;
        if (ms_min) ms_min[k] = 0.0;
        if (ms_max) ms_max[k] = 0.0;
    }
    for (int i = 0; i < t.used; ++i) {
        hipError_t e = hipEventSynchronize(t.stop[i]);
        if (e != hipSuccess) return hip_fail(e);
        float ms = 0.f;
        e = hipEventElapsedTime(&ms, t.start[i], t.stop[i]);
        if (e != hipSuccess) return hip_fail(e);
        const int k = t.kid[i];
        if (ms_min && (launches[k] == 0 || (double)ms < ms_min[k])) ms_min[k] = (double)ms;
        if (ms_max && (launches[k] == 0 || (double)ms > ms_max[k])) ms_max[k] = (double)ms;
        ms_sum[k] += (double)ms;
        launches[k] += 1;
    }
    t.used = 0;
    return BCS_OK;
}

int bcs_timing_end(double *ms_sum, int64_t *launches) { return bcs_timing_stats(ms_sum, launches, nullptr, nullptr); }

const char *bcs_kernel_name(int id) { return (id >= 0 && id < kKernelCount) ? kKernelNames[id] : "?"; }

const char *bcs_strerror(int code) {
    switch (code) {
        case BCS_OK: return "success";
        case BCS_EINVAL: return "invalid argument";
        case BCS_EHIP: return "HIP call failed (see bcs_last_hip_error)";
        case BCS_ENOMEM: return "scratch memory unavailable or workspace too small";
        case BCS_ETOOBIG: return "problem needs more scratch than the fixed array of the no-allocation call holds";
        default: return "unknown bcsched error code";
    }
}

int bcs_last_hip_error(void) { return g_last_hip; }

}  // extern "C"
