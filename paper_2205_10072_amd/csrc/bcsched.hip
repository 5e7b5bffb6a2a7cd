// libbcsched: round-optimal broadcast schedules on a circulant graph, built on gfx950.
//
// Method: J. L. Traff, arXiv 2205.10072, Section 2 (Alg. 1, 2, 4, 5; index arithmetic of Alg. 6).
// One lane owns one rank.  Everything is 32-bit integer work on the vector ALU; block sets are
// 32-bit masks (q <= 31); the skips of a uniform-p launch live in scalar registers.
//
// The per-rank construction is in bcs_core.h; this file holds the kernels and the C ABI.
#include <hip/hip_runtime.h>
#include <hip/hip_ext.h>
#include <stdint.h>
#include <mutex>
#include <utility>

#include "bcsched.h"
#include "bcs_core.h"

namespace {

using namespace bcs;
typedef int v4i __attribute__((ext_vector_type(4)));
// An entry of the slot-major receive table kept in scratch memory: schedule entries lie in [-q, q-1], q <= 31.
typedef int8_t slot_t;
// Rank-major byte rows for the expansion of long rows (scratch as well): row r holds T[k] = entry[k] - k for the q
// slots, then T[0..2] once more, padded to a multiple of 4 bytes.  T lies in [-2q, q), q <= 31.
constexpr int byte_row_stride(int q) { return (q + 3 + 3) & ~3; }
// The byte rows pay while a table of them stays in cache (measured: 25 MB at p = 2^20+1 gives 0.83-0.93 of the
// separate kernels' time for every row length, 50 MB at p = 2^21+1 gives 1.08-1.2).
constexpr uint64_t kByteRowsMax = 32ull << 20;
static_assert(kMaxQ == BCS_MAX_Q, "header and core disagree");
constexpr int kBlock = 256;              // lanes (= ranks) per workgroup

thread_local int g_last_hip = 0;

inline int hip_fail(hipError_t e) {
    g_last_hip = (int)e;
    return BCS_EHIP;
}

// Optional per-kernel device timing (bcs_timing_begin / bcs_timing_end): while it is on, a launch is
// given a start and a stop event from a fixed pool, so its duration is the device's own.
enum KernelId {
    kRecv = 0, kSendLookup, kSendRecompute, kBatch, kExpand, kFill, kValuPeak, kAllgather, kPackPlan, kPackCopy,
    kRecvExpand, kSendExpand, kExpandRows, kRowsToBytes, kKernelCount
};
static_assert(kKernelCount == BCS_KERNEL_COUNT, "header and kernel list disagree");
const char *const kKernelNames[kKernelCount] = {"k_recv_uniform", "k_send_lookup", "k_send_recompute", "k_batch",
                                                "k_expand",       "k_fill",        "k_valu_peak",   "k_allgather_tables",
                                                "k_pack_plan",    "k_pack_copy",   "k_recv_expand", "k_send_expand",
                                                "k_expand_rows",  "k_rows_to_bytes"};
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

// ----------------------------------------------------------------------------------------------
// The low-level table of bcs_core.h lives in the code object; k_build_lowtab fills it once per device
// and process (one thread per entry, by the level walk).
// ----------------------------------------------------------------------------------------------
__device__ uint8_t g_lowtab[kLowTableBytes];

__global__ __launch_bounds__(kBlock) void k_build_lowtab() {
    const int e = blockIdx.x * kBlock + threadIdx.x;
    if (e >= kLowTableBytes) return;
    const int shape = e / kLowShapeBytes;
    const int rest = e - shape * kLowShapeBytes;
    g_lowtab[e] = (uint8_t)low_table_entry(shape, rest >> 7, rest & 127);
}

// copies one shape of the table (kLowShapeBytes, a multiple of 4) into LDS; callers synchronise
__device__ __forceinline__ void stage_lowtab(uint32_t *dst, int shape) {
    const uint32_t *src = reinterpret_cast<const uint32_t *>(g_lowtab + (size_t)shape * kLowShapeBytes);
    for (int i = threadIdx.x; i < kLowShapeBytes / 4; i += kBlock) dst[i] = src[i];
}

// A lane completes its byte row (the three mirrored slots and the padding) ...
template <int Q>
__device__ __forceinline__ void byte_row_finish(int8_t *row) {
    constexpr int kRS = byte_row_stride(Q);
#pragma unroll
    for (int m = 0; m < kRS - Q; ++m) row[Q + m] = (m < 3 && m < Q) ? row[m] : (int8_t)0;
}

// ... and the workgroup's byte rows leave for the table as 16-byte pieces (after a barrier)
template <int Q>
__device__ __forceinline__ void byte_rows_out(const int8_t *tileB, uint32_t rows, int8_t *__restrict__ dst) {
    constexpr int kRS = byte_row_stride(Q);
    const uint32_t n4 = rows * (kRS / 4);                         // dwords
    const uint32_t n16 = n4 >> 2;
    for (uint32_t g = threadIdx.x; g < n16; g += kBlock)
        reinterpret_cast<v4i *>(dst)[g] = reinterpret_cast<const v4i *>(tileB)[g];
    const uint32_t e = (n16 << 2) + threadIdx.x;
    if (e < n4) reinterpret_cast<int32_t *>(dst)[e] = reinterpret_cast<const int32_t *>(tileB)[e];
}

// The byte rows of a workgroup packed straight from its int32 tile (row stride Q | 1), four entries a dword:
// for a kernel that has vector-ALU time to spare and should not spend LDS on a byte tile.
template <int Q>
__device__ __forceinline__ void byte_rows_from_tile(const int32_t *tile, uint32_t rows, int8_t *__restrict__ dst) {
    constexpr int kStride = Q | 1;
    constexpr int kW4 = byte_row_stride(Q) / 4;                   // dwords per byte row
    const uint32_t n4 = rows * kW4;
    for (uint32_t g = threadIdx.x; g < n4; g += kBlock) {
        const uint32_t row = g / kW4, w = g - row * kW4;
        const int32_t *src = tile + row * kStride;
        uint32_t packed = 0;
#pragma unroll
        for (int c = 0; c < 4; ++c) {
            const uint32_t pos = 4u * w + c;
            const bool slot_ok = pos < (uint32_t)(Q + 3);          // the row's slots and its three mirrors
            const uint32_t slot = pos < (uint32_t)Q ? pos : (slot_ok ? pos - Q : 0u);
            const int32_t t = slot_ok ? src[slot] - (int32_t)slot : 0;
            packed |= ((uint32_t)t & 0xffu) << (8 * c);
        }
        reinterpret_cast<uint32_t *>(dst)[g] = packed;
    }
}

// Rows of a workgroup's LDS tile (row stride Q | 1) to their place in a rank-major table.  For odd Q the tile is
// already laid out like the table, so it leaves as 16-byte pieces with no index arithmetic.
template <int Q>
__device__ __forceinline__ void tile_to_rows(const int32_t *tile, uint32_t rows, int32_t *__restrict__ dst) {
    constexpr int kStride = Q | 1;
    const uint32_t n = rows * Q;
    if constexpr (kStride == Q) {
        if ((reinterpret_cast<uintptr_t>(dst) & 15u) == 0) {
            const uint32_t n4 = n >> 2;
            for (uint32_t g = threadIdx.x; g < n4; g += kBlock)
                reinterpret_cast<v4i *>(dst)[g] = reinterpret_cast<const v4i *>(tile)[g];
            const uint32_t e = (n4 << 2) + threadIdx.x;
            if (e < n) dst[e] = tile[e];
            return;
        }
    }
    for (uint32_t e = threadIdx.x; e < n; e += kBlock) {
        const uint32_t row = e / Q, col = e - row * Q;
        dst[e] = tile[row * kStride + col];
    }
}

// ----------------------------------------------------------------------------------------------
// K1: receive rows of ranks [r0, r1), uniform p.  Lane = rank.  Rows are staged in LDS (odd stride,
// conflict-free) and leave as contiguous dwords; optionally each entry is also stored slot-major
// (recvT[k][r - r0]) for the send look-up that follows.
// ----------------------------------------------------------------------------------------------
template <int Q, bool BYTES>
__global__ __launch_bounds__(kBlock) void k_recv_uniform(const SkipTab tab, uint32_t root, uint32_t r0, uint32_t r1,
                                                         int32_t *__restrict__ recv_out,
                                                         slot_t *__restrict__ recvT, uint64_t ldT,
                                                         int8_t *__restrict__ rowsB) {
    constexpr int kStride = Q | 1;
    constexpr int kRS = byte_row_stride(Q);
    __shared__ __align__(16) int32_t tile[kBlock * kStride];
    __shared__ __align__(16) int8_t tileB[BYTES ? kBlock * kRS : 16];   // only the variant that leaves byte rows pays for it
    __shared__ uint32_t lowtab[kLowShapeBytes / 4];
    Uniform<Q> pol;
#pragma unroll
    for (int k = 0; k <= Q; ++k) pol.S[k] = tab.s[k];
    pol.tab = &tab;
    pol.low = reinterpret_cast<const uint8_t *>(lowtab);
    const uint32_t p = pol.p();
    stage_lowtab(lowtab, low_shape(p, Q));
    __syncthreads();
    const uint64_t first = (uint64_t)blockIdx.x * kBlock;       // offset of this tile inside [r0, r1)
    const uint64_t idx = first + threadIdx.x;
    const uint64_t count = (uint64_t)r1 - r0;
    const bool live = idx < count;
    const uint32_t r = live ? (uint32_t)(r0 + idx) : root;       // idle lanes replay the root (cheap, valid)
    const uint32_t v = r >= root ? r - root : r + p - root;
    int32_t *my = tile + threadIdx.x * kStride;
    int8_t *myB = tileB + (BYTES ? threadIdx.x * kRS : 0);
    recv_row(pol, v, Q - 1, [&](int i, int val) {
        my[i] = val;
        if (recvT && live) recvT[(uint64_t)i * ldT + idx] = (slot_t)val;
        if constexpr (BYTES) myB[i] = (int8_t)(val - i);
    });
    if (!recv_out) return;
    if constexpr (BYTES) byte_row_finish<Q>(myB);
    __syncthreads();
    const uint64_t rows = (count - first) < (uint64_t)kBlock ? (count - first) : (uint64_t)kBlock;
    tile_to_rows<Q>(tile, (uint32_t)rows, recv_out + first * Q);
    if constexpr (BYTES) byte_rows_out<Q>(tileB, (uint32_t)rows, rowsB + first * kRS);
}

// K2: send rows from the slot-major receive table of ALL ranks (Alg. 9, second loop):
// send[r][k] = recv[(r + skips[k]) mod p][k].  Reads are contiguous per slot, rows leave through LDS.
template <int Q>
__global__ __launch_bounds__(kBlock) void k_send_lookup(const SkipTab tab, const slot_t *__restrict__ recvT,
                                                        uint64_t ldT, int32_t *__restrict__ send_out,
                                                        int8_t *__restrict__ rowsB) {
    constexpr int kStride = Q | 1;
    constexpr int kRS = byte_row_stride(Q);
    __shared__ __align__(16) int32_t tile[kBlock * kStride];
    const uint32_t p = tab.s[Q];
    const uint64_t first = (uint64_t)blockIdx.x * kBlock;
    const uint64_t idx = first + threadIdx.x;
    const bool live = idx < p;
    int32_t *my = tile + threadIdx.x * kStride;
    if (live) {
#pragma unroll
        for (int k = 0; k < Q; ++k) {
            uint32_t t = (uint32_t)idx + tab.s[k];
            t = t >= p ? t - p : t;
            my[k] = recvT[(uint64_t)k * ldT + t];
        }
    }
    __syncthreads();
    const uint64_t rows = ((uint64_t)p - first) < (uint64_t)kBlock ? ((uint64_t)p - first) : (uint64_t)kBlock;
    tile_to_rows<Q>(tile, (uint32_t)rows, send_out + first * Q);
    if (rowsB) byte_rows_from_tile<Q>(tile, (uint32_t)rows, rowsB + first * kRS);
}

// K1b: send rows of ranks [r0, r1) with no neighbour rows at hand (Alg. 5): entry i is entry i of the
// receive schedule of the to-neighbour, which costs that neighbour's rounds 0..i.
template <int Q>
__global__ __launch_bounds__(kBlock) void k_send_recompute(const SkipTab tab, uint32_t root, uint32_t r0, uint32_t r1,
                                                           int32_t *__restrict__ send_out) {
    constexpr int kStride = Q | 1;
    __shared__ __align__(16) int32_t tile[kBlock * kStride];
    __shared__ uint32_t lowtab[kLowShapeBytes / 4];
    Uniform<Q> pol;
#pragma unroll
    for (int k = 0; k <= Q; ++k) pol.S[k] = tab.s[k];
    pol.tab = &tab;
    pol.low = reinterpret_cast<const uint8_t *>(lowtab);
    const uint32_t p = pol.p();
    stage_lowtab(lowtab, low_shape(p, Q));
    __syncthreads();
    const uint64_t first = (uint64_t)blockIdx.x * kBlock;
    const uint64_t idx = first + threadIdx.x;
    const uint64_t count = (uint64_t)r1 - r0;
    const bool live = idx < count;
    const uint32_t r = live ? (uint32_t)(r0 + idx) : root;
    const uint32_t v = r >= root ? r - root : r + p - root;
    int32_t *my = tile + threadIdx.x * kStride;
#pragma unroll 1
    for (int i = 0; i < Q; ++i) {
        uint32_t t = v + tab.s[i];
        t = t >= p ? t - p : t;
        const uint32_t dt = digits(pol, t);
        int32_t keep = dt ? __builtin_ctz(dt) : 0;
        // Round i is the neighbour's home round when its highest digit is i: then the entry is its baseblock and
        // none of its earlier rounds matters.  A wave of consecutive ranks below skips[i+1] - skips[i] is in that
        // case as a whole (half of all waves for the last slot, a quarter for the one before, ...).
        const bool home_round = dt != 0u && (31 - __clz((int)dt)) == i;
        if (__any(!home_round)) {
            int32_t got = 0;
            recv_row_from(pol, t, dt, i, [&](int j, int val) { got = (j == i) ? val : got; });
            keep = got;
        }
        my[i] = keep;
    }
    __syncthreads();
    const uint64_t rows = (count - first) < (uint64_t)kBlock ? (count - first) : (uint64_t)kBlock;
    tile_to_rows<Q>(tile, (uint32_t)rows, send_out + first * Q);
}

// K3: unrelated (p, r, root) triples; rows of BCS_BATCH_STRIDE ints (one 128-byte line each), padded.
// A workgroup takes kBatchBlock triples and first orders them by q in LDS (counting sort), because a
// wave runs its level loops to the largest q among its lanes and the work grows like q^3: after the
// sort a wave holds neighbouring q only.  Each lane then builds the rows of its triple and stores
// them entry by entry into the triple's own line.
constexpr int kBatchBlock = 1024;

__global__ __launch_bounds__(kBatchBlock) void k_batch(int64_t count, const int32_t *__restrict__ pv,
                                                       const int32_t *__restrict__ rv,
                                                       const int32_t *__restrict__ rootv,
                                                       int32_t *__restrict__ recv_out, int32_t *__restrict__ send_out,
                                                       int32_t *__restrict__ q_out) {
    __shared__ uint32_t bins[33];                 // bins[q] for valid triples, bins[32] for the rest
    __shared__ uint32_t start[33];
    __shared__ uint32_t s_p[kBatchBlock], s_v[kBatchBlock], s_slot[kBatchBlock];
    const int64_t first = (int64_t)blockIdx.x * kBatchBlock;
    {
        const int64_t idx = first + threadIdx.x;
        const bool live = idx < count;
        const int32_t pi = live ? pv[idx] : 1, ri = live ? rv[idx] : 0, rooti = live ? rootv[idx] : 0;
        const bool valid = live && pi >= 1 && ri >= 0 && ri < pi && rooti >= 0 && rooti < pi;
        const uint32_t p = valid ? (uint32_t)pi : 1u;
        const int q = ceil_log2(p);
        const uint32_t v = !valid ? 0u
                           : ((uint32_t)ri >= (uint32_t)rooti ? (uint32_t)(ri - rooti)
                                                              : (uint32_t)ri + p - (uint32_t)rooti);
        if (threadIdx.x < 33) bins[threadIdx.x] = 0u;
        __syncthreads();
        const int bin = valid ? q : 32;
        const uint32_t rank_in_bin = atomicAdd(&bins[bin], 1u);
        __syncthreads();
        if (threadIdx.x == 0) {
            uint32_t acc = 0;
            for (int k = 0; k < 33; ++k) {
                start[k] = acc;
                acc += bins[k];
            }
        }
        __syncthreads();
        const uint32_t pos = start[bin] + rank_in_bin;
        s_p[pos] = p;
        s_v[pos] = v;
        s_slot[pos] = threadIdx.x | (valid ? 0u : 0x80000000u) | (live ? 0u : 0x40000000u);
        __syncthreads();
    }
    // from here on this lane works on the triple that the sort put at its position
    const uint32_t p = s_p[threadIdx.x];
    const uint32_t v = s_v[threadIdx.x];
    const uint32_t slot = s_slot[threadIdx.x];
    const bool valid = (slot & 0x80000000u) == 0u;
    const bool live = (slot & 0x40000000u) == 0u;
    const int64_t idx = first + (slot & 0xffffu);
    const int q = ceil_log2(p);
    if (live && q_out) q_out[idx] = valid ? q : -1;
    // largest q in this wave bounds the level loops of all its lanes
    int qmax = q;
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) {
        const int other = __shfl_xor(qmax, off, 64);
        qmax = other > qmax ? other : qmax;
    }
    PerLane pol;
    pol.pm1 = p - 1u;
    pol.ql = q;
    pol.wave_top = qmax - 1;
    pol.odd = odd_levels(p, q);
    pol.low = g_lowtab + (size_t)low_shape(p, q) * kLowShapeBytes;
    if (recv_out) {
        int32_t *row = recv_out + idx * BCS_BATCH_STRIDE;
        recv_row(pol, v, qmax - 1, [&](int i, int val) { if (live) row[i] = val; });
        if (live)
            for (int k = q; k < BCS_BATCH_STRIDE; ++k) row[k] = BCS_BATCH_PAD;
    }
    if (send_out) {
        int32_t *row = send_out + idx * BCS_BATCH_STRIDE;
#pragma unroll 1
        for (int i = 0; i < qmax; ++i) {
            uint32_t t = v + (i < q ? pol.s(i) : 0u);
            t = t >= p ? t - p : t;
            int32_t keep = 0;
            recv_row(pol, t, i, [&](int j, int val) { keep = (j == i) ? val : keep; });
            if (live && i < q) row[i] = keep;
        }
        if (live)
            for (int k = q; k < BCS_BATCH_STRIDE; ++k) row[k] = BCS_BATCH_PAD;
    }
}

// ----------------------------------------------------------------------------------------------
// K4: expansion (Alg. 6 index arithmetic).  Real round j uses slot k = (x+j) mod q; by then the slot
// has been advanced floor((x+j)/q) times by q and shifted by -x, and q*floor((x+j)/q) = x+j-k, so
// the block is sched[k] + j - k.  Negative -> BCS_NO_BLOCK, above n-1 -> n-1 (caption of Alg. 6).
//
// The output is one contiguous int32 stream of rows*R entries and the kernels treat it as such: a
// workgroup owns kExpChunk consecutive entries (16 KiB), a lane writes 16 bytes per 4 KiB piece.
// The schedule rows the chunk touches are staged in LDS as T[k] = sched[k] - k, so an entry is
// T[k] + j, clamped.  Wave-uniform steps come precomputed from the host.
//
// k_expand (R >= 16, q >= 3): a lane's four consecutive entries use four consecutive slots.  So that
// they are four consecutive LDS words whatever happens in between, a staged row of q+9 words holds
//   T[0..q-1] | T[0..2] | T[q-3..q-1] | T'[x..x+2] - R      (T' = next row's T, slots mod q)
// A row always ends on slot q-1 (x + R is a multiple of q).  A lane that stays inside its row starts at
// word k and may run into the second group (slot wraps to 0, round keeps counting); a lane whose
// piece crosses into the next row starts 6 words further and runs into the fourth group, whose
// "- R" makes T + (j + c) come out as the next row's T + (c - entries left).  One select per lane,
// none per entry.  Small divisions use exact multiply-high reciprocals.
// k_expand_small: the same stream for tiny R or q = 1, advancing slot and round entry by entry.
// ----------------------------------------------------------------------------------------------
constexpr int kExpIter = 4;                         // 16-byte pieces per lane (measured best of 1..16)
constexpr int kExpChunk = kExpIter * kBlock * 4;    // entries per workgroup
constexpr int kExpSmallLds = kExpChunk + 2 * (kMaxQ + 1);
constexpr uint32_t kExpMinR = 16;
constexpr uint32_t kExpMinQ = 3;
constexpr uint64_t kExpNtMaxR = 640;                // rows up to this length use streaming stores
constexpr uint32_t kExpPad = 9;                      // extra words per staged row

struct ExpandArgs {
    uint64_t total;                       // rows * R
    uint64_t rows;
    uint32_t R;
    uint32_t step_rows;                   // (kBlock*4) / R
    uint32_t step_j;                      // (kBlock*4) % R
    uint32_t step_k;                      // step_j % q
    uint32_t wrap_k;                      // q - R % q
    uint32_t q;
    uint32_t x;
    int32_t nm1;                          // n - 1
    int aligned;                          // output is 16-byte aligned
    uint32_t magic_R;                     // floor(2^32 / R) + 1       (dividends below 2^14, R < 8192)
    uint32_t magic_q;                     // floor(2^32 / q) + 1       (dividends below 2^16)
    uint32_t magic_w;                     // floor(2^32 / (q+9)) + 1   (dividends below 2^14)
};

__device__ __forceinline__ void expand_store(int32_t *__restrict__ out, uint64_t e, const int32_t (&v)[4],
                                             bool vec, bool full, uint64_t total) {
    if (vec && (full || e + 4 <= total)) {
        *reinterpret_cast<int4 *>(out + e) = make_int4(v[0], v[1], v[2], v[3]);
    } else {
#pragma unroll
        for (int c = 0; c < 4; ++c)
            if (full || e + c < total) out[e + c] = v[c];
    }
}

// NT: streaming (non-temporal) stores.  Measured on MI355X they win while the schedule reads are a
// visible share of the traffic (short rows) and lose to plain stores for long rows.
template <bool NT>
__global__ __launch_bounds__(kBlock) void k_expand(const ExpandArgs a, const int32_t *__restrict__ in,
                                                   int32_t *__restrict__ out) {
    extern __shared__ int32_t tile[];     // (rows touched + 1) x (q + 9)
    const uint32_t q = a.q, R = a.R, w = q + kExpPad;
    const uint64_t e0 = (uint64_t)blockIdx.x * kExpChunk;          // first entry of this workgroup
    uint64_t row0;
    uint32_t j0;
    if ((a.total >> 32) == 0) {
        const uint32_t e32 = (uint32_t)e0, r32 = e32 / R;
        row0 = r32;
        j0 = e32 - r32 * R;
    } else {
        row0 = e0 / R;
        j0 = (uint32_t)(e0 - row0 * R);
    }
    uint32_t nrows = (j0 + (uint32_t)kExpChunk - 1u) / R + 1u;
    if (row0 + nrows > a.rows) nrows = (uint32_t)(a.rows - row0);
    const bool has_next = row0 + nrows < a.rows;                    // a row after the last touched one
    const uint32_t staged = nrows * w;
    const int32_t *src = in + row0 * q;
    const uint32_t last_row = has_next ? nrows : nrows - 1u;        // highest row index that may be read
    // loads of a group are issued together (indices clamped, no branch) so their latencies overlap
    constexpr int kGroup = 4;
    for (uint32_t base = 0; base < staged; base += kGroup * kBlock) {
        int32_t got[kGroup];
#pragma unroll
        for (int u = 0; u < kGroup; ++u) {
            uint32_t i = base + u * kBlock + threadIdx.x;
            i = i < staged ? i : staged - 1u;
            const uint32_t rr = __umulhi(i, a.magic_w);
            const uint32_t pos = i - rr * w;
            // which slot of which row this word mirrors
            const bool g1 = pos >= q, g2 = pos >= q + 3u, g3 = pos >= q + 6u;
            uint32_t slot = g3 ? pos - (q + 6u) + a.x : (g2 ? pos - 6u : (g1 ? pos - q : pos));
            slot = slot >= q ? slot - q : slot;
            uint32_t row = g3 ? rr + 1u : rr;
            row = row > last_row ? last_row : row;
            const int32_t shift = g3 ? (int32_t)(slot + R) : (int32_t)slot;
            got[u] = src[row * q + slot] - shift;
        }
#pragma unroll
        for (int u = 0; u < kGroup; ++u) {
            const uint32_t i = base + u * kBlock + threadIdx.x;
            if (i < staged) tile[i] = got[u];
        }
    }
    __syncthreads();

    // this lane's first entry: chunk-relative t = j0 + 4*lane lies in row row0 + t / R
    const uint32_t t = j0 + threadIdx.x * 4u;
    uint32_t rd = R >= 8192u ? (t >= R ? 1u : 0u) : __umulhi(t, a.magic_R);
    uint32_t j = t - rd * R;
    const uint32_t kb = (a.x + j0) % q;
    const uint32_t kv = kb + threadIdx.x * 4u + rd * a.wrap_k;     // congruent to x + j mod q
    uint32_t k = kv - q * __umulhi(kv, a.magic_q);
    const bool full = e0 + kExpChunk <= a.total;
    const bool vec = a.aligned != 0;
    uint64_t e = e0 + threadIdx.x * 4u;
    const int32_t lo = -1, hi = a.nm1;
    const unsigned char *lds = reinterpret_cast<const unsigned char *>(tile);
#pragma unroll 1
    for (int it = 0; it < kExpIter; ++it) {
        if (!full && e >= a.total) break;
        const uint32_t left = R - j;                                // entries left in this row
        const uint32_t word = rd * w + k + (left < 4u ? 6u : 0u);
        const int32_t *wp = reinterpret_cast<const int32_t *>(lds + word * 4u);
        int32_t v[4];
#pragma unroll
        for (int c = 0; c < 4; ++c) {
            const int32_t raw = wp[c] + (int32_t)(j + c);
            const int32_t m = raw > lo ? raw : lo;
            v[c] = m < hi ? m : hi;
        }
        if (vec && (full || e + 4 <= a.total)) {
            v4i pack = {v[0], v[1], v[2], v[3]};
            if constexpr (NT) __builtin_nontemporal_store(pack, reinterpret_cast<v4i *>(out + e));
            else *reinterpret_cast<v4i *>(out + e) = pack;
        } else {
#pragma unroll
            for (int c = 0; c < 4; ++c)
                if (full || e + c < a.total) out[e + c] = v[c];
        }
        e += (uint64_t)kBlock * 4u;
        rd += a.step_rows;
        j += a.step_j;
        k += a.step_k;
        if (j >= R) {
            j -= R;
            ++rd;
            k += a.wrap_k;
        }
        k = k >= q ? k - q : k;
        k = k >= q ? k - q : k;
    }
}

// k_expand_rows: the same stream from the rank-major byte rows that the schedule kernels leave in scratch
// memory when the expansion follows in the same call (T[0..q-1] | T[0..2] per row, 4 p bytes at q = 21: it stays
// in cache).  No staging and no barrier: a workgroup writes one piece of 1024 entries (4 KiB) and ends; a lane
// resolves row and round of its four entries by itself (exact division by R: multiply-high and one correction),
// reads the four bytes at its slot and the four at slot x of the next row -- those serve the entries past the end
// of its row -- and stores 16 bytes.  Measured on MI355X: 0.159 ms a table at the bench size against 0.181 ms
// for k_expand; short workgroups dispatched in address order are what the memory system likes best.  Streaming
// stores for every row length (plain stores were 1.3 times slower from 640 rounds up).
struct ExpandRowsArgs {
    uint64_t total;                       // rows * R
    uint64_t magic_R64;                   // floor(2^64 / R) + 1
    uint32_t magic_R32;                   // floor(2^32 / R) + 1
    uint32_t magic_q;                     // floor(2^32 / q) + 1
    uint32_t R, q, x, RS;                 // RS: bytes per row of the byte table
    int32_t nm1;
};

__global__ __launch_bounds__(kBlock) void k_expand_rows(const ExpandRowsArgs a, const int8_t *__restrict__ rowsB,
                                                        int32_t *__restrict__ out) {
    const uint64_t e = ((uint64_t)blockIdx.x * kBlock + threadIdx.x) * 4u;
    if (e >= a.total) return;
    const uint32_t q = a.q, R = a.R;
    uint64_t row;
    uint32_t j;
    if ((a.total >> 32) == 0) {
        const uint32_t e32 = (uint32_t)e;
        uint32_t r32 = __umulhi(e32, a.magic_R32);                 // exact or one too large
        int32_t jj = (int32_t)(e32 - r32 * R);
        if (jj < 0) { jj += (int32_t)R; --r32; }
        row = r32;
        j = (uint32_t)jj;
    } else {
        uint64_t r64 = __umul64hi(e, a.magic_R64);
        int64_t jj = (int64_t)(e - r64 * R);
        if (jj < 0) { jj += R; --r64; }
        row = r64;
        j = (uint32_t)jj;
    }
    const uint32_t i = a.x + j;
    uint32_t k = i - q * __umulhi(i, a.magic_q);
    k = (int32_t)k < 0 ? k + q : k;                                // the multiply-high may be one too large
    const int8_t *src = rowsB + row * a.RS;
    uint32_t here, next;                                           // the table has one more row than ranks
    __builtin_memcpy(&here, src + k, 4);
    __builtin_memcpy(&next, src + a.RS + a.x, 4);
    const uint32_t left = R - j;                                   // entries left in this row
    const int32_t lo = -1, hi = a.nm1;
    int32_t v[4];
#pragma unroll
    for (int c = 0; c < 4; ++c) {
        const int32_t cur = (int32_t)(int8_t)(here >> (8 * c)) + (int32_t)(j + c);
        const uint32_t over = (uint32_t)c - left;                  // round in the next row, when c >= left
        const int32_t nxt = (int32_t)(int8_t)(next >> (8 * (over & 3u))) + (int32_t)over;
        const int32_t raw = (uint32_t)c < left ? cur : nxt;
        const int32_t m = raw > lo ? raw : lo;
        v[c] = m < hi ? m : hi;
    }
    if (e + 4 <= a.total) {
        const v4i pack = {v[0], v[1], v[2], v[3]};
        __builtin_nontemporal_store(pack, reinterpret_cast<v4i *>(out + e));
    } else {
#pragma unroll
        for (int c = 0; c < 4; ++c)
            if (e + c < a.total) out[e + c] = v[c];
    }
}

// int32 schedule rows -> byte rows (for an expansion whose tables come from the caller): one dword of four
// packed bytes a lane.  Byte tables are at most kByteRowsMax bytes, so 32-bit indices do.
__global__ __launch_bounds__(kBlock) void k_rows_to_bytes(uint32_t rows, uint32_t q, uint32_t RS, uint32_t magic_w4,
                                                          const int32_t *__restrict__ in, int8_t *__restrict__ rowsB) {
    const uint32_t w4 = RS >> 2;                                    // dwords per byte row
    const uint32_t g = blockIdx.x * kBlock + threadIdx.x;
    if (g >= rows * w4) return;
    uint32_t row = __umulhi(g, magic_w4);                           // exact or one too large
    int32_t w = (int32_t)(g - row * w4);
    if (w < 0) { w += (int32_t)w4; --row; }
    const int32_t *src = in + (uint64_t)row * q;
    uint32_t packed = 0;
#pragma unroll
    for (int c = 0; c < 4; ++c) {
        const uint32_t pos = 4u * (uint32_t)w + c;
        const bool slot_ok = pos < q + 3u;                          // the row's slots and its three mirrors
        const uint32_t slot = pos < q ? pos : (slot_ok ? pos - q : 0u);
        const int32_t t = slot_ok ? src[slot] - (int32_t)slot : 0;
        packed |= ((uint32_t)t & 0xffu) << (8 * c);
    }
    reinterpret_cast<uint32_t *>(rowsB)[g] = packed;
}

// ----------------------------------------------------------------------------------------------
// K1+K4 and K2+K4 fused: a workgroup that has just built (or looked up) the schedule rows of its 256
// ranks expands them straight from LDS, so the rows are not read back from memory and the integer
// work of the construction overlaps with the stores of the expansion.  The tile is kept in the
// mirrored T layout of k_expand (row stride odd, so the lanes' row writes do not collide); the 256
// rows of a tile are one contiguous piece of the expanded table that starts on a 16-byte boundary.
// Used for short rows (see use_fused).
// ----------------------------------------------------------------------------------------------
template <int Q>
struct FusedTile {
    static constexpr int kWidth = (Q + (int)kExpPad) | 1;
};

// after the rows T[k] = entry - k are in place: add the three mirrors of every row (see k_expand)
template <int Q>
__device__ __forceinline__ void tile_mirrors(int32_t *tile, uint32_t x, uint32_t R) {
    constexpr int W = FusedTile<Q>::kWidth;
    static_assert(Q >= (int)kExpMinQ, "the mirrored layout needs three slots");
    int32_t *my = tile + threadIdx.x * W;
#pragma unroll
    for (int m = 0; m < 3; ++m) {
        my[Q + m] = my[m];
        my[Q + 3 + m] = my[Q - 3 + m];
    }
    __syncthreads();
    if (threadIdx.x + 1 < kBlock) {
        const int32_t *next = my + W;
#pragma unroll
        for (int m = 0; m < 3; ++m) {
            uint32_t slot = x + m;
            slot = slot >= (uint32_t)Q ? slot - (uint32_t)Q : slot;
            my[Q + 6 + m] = next[slot] - (int32_t)R;
        }
    }
    __syncthreads();
}

// rank-major schedule rows of the tile: entry = T + slot
template <int Q>
__device__ __forceinline__ void tile_rows_out(const int32_t *tile, uint32_t rows, int32_t *__restrict__ dst) {
    constexpr int W = FusedTile<Q>::kWidth;
    const uint32_t n = rows * Q;
    for (uint32_t e = threadIdx.x; e < n; e += kBlock) {
        const uint32_t row = e / Q, col = e - row * Q;
        dst[e] = tile[row * W + col] + (int32_t)col;
    }
}

// the expanded entries of the tile's rows: `rows` x R entries starting at flat index first_row * R
template <int Q, bool NT>
__device__ __forceinline__ void tile_expand(const int32_t *tile, uint32_t rows, uint64_t first_row,
                                            const ExpandArgs &a, int32_t *__restrict__ out) {
    constexpr uint32_t W = FusedTile<Q>::kWidth;
    const uint32_t R = a.R;
    const uint64_t count = (uint64_t)rows * R;
    int32_t *dst = out + first_row * R;
    const uint32_t t = threadIdx.x * 4u;
    uint32_t rd = __umulhi(t, a.magic_R);                             // t < 2^14, R <= kFusedMaxR
    uint32_t j = t - rd * R;
    const uint32_t kv = a.x + t + rd * a.wrap_k;                    // congruent to x + j mod q
    uint32_t k = kv - (uint32_t)Q * __umulhi(kv, a.magic_q);
    const int32_t lo = -1, hi = a.nm1;
#pragma unroll 1
    for (uint64_t e = t; e < count; e += (uint64_t)kBlock * 4u) {
        const uint32_t left = R - j;
        const int32_t *wp = tile + rd * W + k + (left < 4u ? 6u : 0u);
        int32_t v[4];
#pragma unroll
        for (int c = 0; c < 4; ++c) {
            const int32_t raw = wp[c] + (int32_t)(j + c);
            const int32_t m = raw > lo ? raw : lo;
            v[c] = m < hi ? m : hi;
        }
        if (e + 4 <= count) {
            const v4i pack = {v[0], v[1], v[2], v[3]};
            if constexpr (NT) __builtin_nontemporal_store(pack, reinterpret_cast<v4i *>(dst + e));
            else *reinterpret_cast<v4i *>(dst + e) = pack;
        } else {
            for (int c = 0; c < 4; ++c)
                if (e + c < count) dst[e + c] = v[c];
        }
        rd += a.step_rows;
        j += a.step_j;
        k += a.step_k;
        if (j >= R) {
            j -= R;
            ++rd;
            k += a.wrap_k;
        }
        k = k >= (uint32_t)Q ? k - (uint32_t)Q : k;
        k = k >= (uint32_t)Q ? k - (uint32_t)Q : k;
    }
}

template <int Q>
__global__ __launch_bounds__(kBlock) void k_recv_expand(const SkipTab tab, uint32_t root, const ExpandArgs ea,
                                                        int32_t *__restrict__ recv_out, slot_t *__restrict__ recvT,
                                                        uint64_t ldT, int32_t *__restrict__ blocks_out) {
    constexpr int W = FusedTile<Q>::kWidth;
    __shared__ int32_t tile[kBlock * W];
    __shared__ uint32_t lowtab[kLowShapeBytes / 4];
    Uniform<Q> pol;
#pragma unroll
    for (int k = 0; k <= Q; ++k) pol.S[k] = tab.s[k];
    pol.tab = &tab;
    pol.low = reinterpret_cast<const uint8_t *>(lowtab);
    const uint32_t p = pol.p();
    stage_lowtab(lowtab, low_shape(p, Q));
    __syncthreads();
    const uint64_t first = (uint64_t)blockIdx.x * kBlock;
    const uint64_t idx = first + threadIdx.x;
    const bool live = idx < p;
    const uint32_t r = live ? (uint32_t)idx : root;
    const uint32_t v = r >= root ? r - root : r + p - root;
    int32_t *my = tile + threadIdx.x * W;
    recv_row(pol, v, Q - 1, [&](int i, int val) {
        my[i] = val - i;
        if (live) recvT[(uint64_t)i * ldT + idx] = (slot_t)val;
    });
    tile_mirrors<Q>(tile, ea.x, ea.R);
    const uint32_t rows = (uint32_t)(((uint64_t)p - first) < (uint64_t)kBlock ? ((uint64_t)p - first) : (uint64_t)kBlock);
    tile_rows_out<Q>(tile, rows, recv_out + first * Q);
    tile_expand<Q, true>(tile, rows, first, ea, blocks_out);
}

template <int Q>
__global__ __launch_bounds__(kBlock) void k_send_expand(const SkipTab tab, const ExpandArgs ea,
                                                        const slot_t *__restrict__ recvT, uint64_t ldT,
                                                        int32_t *__restrict__ send_out,
                                                        int32_t *__restrict__ blocks_out) {
    constexpr int W = FusedTile<Q>::kWidth;
    __shared__ int32_t tile[kBlock * W];
    const uint32_t p = tab.s[Q];
    const uint64_t first = (uint64_t)blockIdx.x * kBlock;
    const uint64_t idx = first + threadIdx.x;
    const uint32_t me = idx < p ? (uint32_t)idx : 0u;               // idle lanes replay rank 0
    int32_t *my = tile + threadIdx.x * W;
#pragma unroll
    for (int k = 0; k < Q; ++k) {
        uint32_t t = me + tab.s[k];
        t = t >= p ? t - p : t;
        my[k] = recvT[(uint64_t)k * ldT + t] - k;
    }
    tile_mirrors<Q>(tile, ea.x, ea.R);
    const uint32_t rows = (uint32_t)(((uint64_t)p - first) < (uint64_t)kBlock ? ((uint64_t)p - first) : (uint64_t)kBlock);
    tile_rows_out<Q>(tile, rows, send_out + first * Q);
    tile_expand<Q, true>(tile, rows, first, ea, blocks_out);
}

__global__ __launch_bounds__(kBlock) void k_expand_small(const ExpandArgs a, const int32_t *__restrict__ in,
                                                         int32_t *__restrict__ out) {
    __shared__ int32_t tile[kExpSmallLds];
    const uint32_t q = a.q, R = a.R;
    const uint64_t e0 = (uint64_t)blockIdx.x * kExpChunk;
    const uint64_t row0 = e0 / R;
    const uint32_t j0 = (uint32_t)(e0 - row0 * R);
    uint64_t row_last = (e0 + kExpChunk - 1) / R;
    if (row_last >= a.rows) row_last = a.rows - 1;
    const uint32_t staged = (uint32_t)(row_last - row0 + 1) * q;   // <= kExpSmallLds since q <= R
    const int32_t *src = in + row0 * q;
    for (uint32_t i = threadIdx.x; i < staged; i += kBlock) tile[i] = src[i] - (int32_t)(i % q);
    __syncthreads();
    const uint32_t t = j0 + threadIdx.x * 4u;
    uint32_t rd = t / R;
    uint32_t j = t - rd * R;
    uint32_t k = (a.x + j) % q;
    const bool full = e0 + kExpChunk <= a.total;
    const bool vec = a.aligned != 0;
    uint64_t e = e0 + threadIdx.x * 4u;
#pragma unroll 1
    for (int it = 0; it < kExpIter; ++it) {
        if (!full && e >= a.total) break;
        uint32_t ro = rd * q, jj = j, kk = k;
        int32_t v[4];
#pragma unroll
        for (int c = 0; c < 4; ++c) {
            uint32_t idx = ro + kk;
            idx = idx < staged ? idx : 0u;            // past the table's end; such entries are never stored
            const int32_t raw = tile[idx] + (int32_t)jj;
            v[c] = raw < 0 ? -1 : (raw > a.nm1 ? a.nm1 : raw);
            ++kk;
            ++jj;
            kk = kk == q ? 0u : kk;
            const bool wj = jj == R;                  // next row: round 0, slot x
            jj = wj ? 0u : jj;
            kk = wj ? a.x : kk;
            ro = wj ? ro + q : ro;
        }
        expand_store(out, e, v, vec, full, a.total);
        e += (uint64_t)kBlock * 4u;
        rd += a.step_rows;
        j += a.step_j;
        k += a.step_k;
        if (j >= R) {
            j -= R;
            ++rd;
            k += a.wrap_k;
        }
        k = k >= q ? k - q : k;
        k = k >= q ? k - q : k;
    }
}

// ----------------------------------------------------------------------------------------------
// K5: pack / unpack index tables of the irregular allgather for one process r (Alg. 9, its per-round
// loops over the roots).  For root j the process acts as virtual rank r' = (r - j + p) mod p of a
// broadcast rooted at 0, so unpack[round][j] is the expanded receive entry of r' and pack[round][j]
// that of its to-neighbour's receive row: both come from the slot-major receive table recvT[k][rank].
// k_allgather_tables (outputs at any 4-byte alignment): all rounds that use slot k differ by a multiple
// of q only, so a workgroup takes one slot and kAgChunk consecutive roots, reads its 2 x kAgChunk
// schedule entries once and walks down the rounds k-x, k-x+q, ..., writing one contiguous piece of
// kAgChunk entries per table and round; lanes are consecutive roots, so every store of a wave is one
// contiguous 256-byte piece.  k_allgather_tables_flat (16-byte aligned outputs) is described with it.
// ----------------------------------------------------------------------------------------------
constexpr int kAgRootsPerLane = 16;
constexpr int kAgChunk = kAgRootsPerLane * kBlock;

__global__ __launch_bounds__(kBlock) void k_allgather_tables(const SkipTab tab, int q, uint32_t r, uint32_t x,
                                                             int32_t nm1, uint64_t R,
                                                             const slot_t *__restrict__ recvT, uint64_t ldT,
                                                             int32_t *__restrict__ pack,
                                                             int32_t *__restrict__ unpack) {
    const uint32_t p = tab.s[q];
    const uint32_t k = blockIdx.y;
    const uint32_t sk = tab.s[k];
    const slot_t *row = recvT + (uint64_t)k * ldT;
    const uint64_t first = (uint64_t)blockIdx.x * kAgChunk + threadIdx.x;   // this lane's first root
    int32_t tu[kAgRootsPerLane], tp[kAgRootsPerLane];                        // entry - k for unpack / pack
#pragma unroll
    for (int u = 0; u < kAgRootsPerLane; ++u) {
        const uint64_t j64 = first + (uint64_t)u * kBlock;
        const uint32_t j = j64 < p ? (uint32_t)j64 : 0u;
        const uint32_t vr = r >= j ? r - j : r + p - j;                      // virtual rank of r under root j
        uint32_t to = vr + sk;
        to = to >= p ? to - p : to;
        tu[u] = row[vr] - (int32_t)k;
        tp[u] = row[to] - (int32_t)k;
    }
    // first real round that uses slot k: k - x, or one phase later when that is a dummy round
    for (uint64_t j = k >= x ? k - x : k + (uint32_t)q - x; j < R; j += (uint32_t)q) {
        int32_t *up = unpack ? unpack + j * p + first : nullptr;
        int32_t *pp = pack ? pack + j * p + first : nullptr;
#pragma unroll
        for (int u = 0; u < kAgRootsPerLane; ++u) {
            if (first + (uint64_t)u * kBlock >= p) break;
            if (up) {
                const int32_t raw = tu[u] + (int32_t)j;
                up[u * kBlock] = raw < 0 ? -1 : (raw > nm1 ? nm1 : raw);
            }
            if (pp) {
                const int32_t raw = tp[u] + (int32_t)j;
                pp[u * kBlock] = raw < 0 ? -1 : (raw > nm1 ? nm1 : raw);
            }
        }
    }
}

// K5 with 16-byte stores for any p.  Rows of p entries start on every possible 4-byte phase of a
// 16-byte line, so the schedule entries of the workgroup's roots are staged in LDS and each round
// reads them back at that round's phase: single entries up to the next 128-byte line, aligned groups
// of four (a wave stores whole lines), up to three single entries.  Needs 16-byte aligned tables (else the kernel above runs).
// The same tables as ONE flat stream of R * p entries each, for 16-byte aligned outputs: a workgroup writes one
// piece of 1024 consecutive entries (4 KiB, whole lines whatever p is) and ends; a lane resolves round and root
// of its four entries by itself (exact division by p with a multiply-high and one correction), reads the four
// one-byte table entries -- consecutive ranks, descending -- with one unaligned load, and stores 16 bytes.  No
// staging and no barrier: measured on MI355X, short workgroups that are dispatched in address order write
// 7.0 TB/s where a workgroup that walks down the rounds of one slot reaches 5.2 TB/s.
struct AgFlatArgs {
    uint64_t total;                       // R * p
    uint64_t magic_p;                     // floor(2^64 / p) + 1
    uint32_t p, q, r, x;
    int32_t nm1;
    uint32_t magic_q;                     // floor(2^32 / q) + 1; x + j can pass 2^16, the quotient is corrected
};

__device__ __forceinline__ int32_t ag_entry(const AgFlatArgs &a, const SkipTab &tab, const slot_t *__restrict__ recvT,
                                            uint64_t ldT, bool packing, uint64_t e) {
    uint64_t j = __umul64hi(e, a.magic_p);
    int64_t root = (int64_t)(e - j * a.p);
    if (root < 0) { root += a.p; --j; }
    const uint32_t i = a.x + (uint32_t)j;
    const uint32_t k = i % a.q;
    const uint32_t vr = a.r >= (uint32_t)root ? a.r - (uint32_t)root : a.r + a.p - (uint32_t)root;
    uint32_t from = vr + (packing ? tab.s[k] : 0u);
    from = from >= a.p ? from - a.p : from;
    const int32_t raw = (int32_t)recvT[(uint64_t)k * ldT + from] - (int32_t)k + (int32_t)j;
    return raw < 0 ? -1 : (raw > a.nm1 ? a.nm1 : raw);
}

__global__ __launch_bounds__(kBlock) void k_allgather_tables_flat(const SkipTab tab, const AgFlatArgs a,
                                                                  const slot_t *__restrict__ recvT, uint64_t ldT,
                                                                  int32_t *__restrict__ pack,
                                                                  int32_t *__restrict__ unpack) {
    const bool packing = unpack == nullptr || blockIdx.y == 1;
    int32_t *__restrict__ out = packing ? pack : unpack;
    const uint64_t e = ((uint64_t)blockIdx.x * kBlock + threadIdx.x) * 4u;
    if (e >= a.total) return;
    // round j = e / p and root = e mod p of the first entry
    uint64_t j = __umul64hi(e, a.magic_p);
    int64_t root64 = (int64_t)(e - j * a.p);
    if (root64 < 0) { root64 += a.p; --j; }
    const uint32_t root = (uint32_t)root64;
    // slot k = (x + j) mod q
    const uint32_t i = a.x + (uint32_t)j;
    uint32_t k = i - a.q * __umulhi(i, a.magic_q);
    k = (int32_t)k < 0 ? k + a.q : k;                              // the multiply-high may be one too large
    const uint32_t vr = a.r >= root ? a.r - root : a.r + a.p - root;   // virtual rank towards `root`
    uint32_t from = vr + (packing ? tab.s[k] : 0u);                // the pack entry is the to-neighbour's
    from = from >= a.p ? from - a.p : from;
    if (e + 4 <= a.total && root + 3u < a.p && from >= 3u) {
        // entries root .. root+3 of round j read ranks from, from-1, from-2, from-3 of row k
        const slot_t *src = recvT + (uint64_t)k * ldT + (from - 3u);
        uint32_t four;
        __builtin_memcpy(&four, src, 4);
        const int32_t shift = (int32_t)j - (int32_t)k;
        const int32_t lo = -1, hi = a.nm1;
        v4i v;
#pragma unroll
        for (int c = 0; c < 4; ++c) {
            const int32_t raw = (int32_t)(int8_t)(four >> (8 * (3 - c))) + shift;
            const int32_t m = raw > lo ? raw : lo;
            v[c] = m < hi ? m : hi;
        }
        __builtin_nontemporal_store(v, reinterpret_cast<v4i *>(out + e));
    } else {
        // the end of a row, a wrap of the ranks, or the end of the table: entry by entry
        for (int c = 0; c < 4; ++c)
            if (e + c < a.total) out[e + c] = ag_entry(a, tab, recvT, ldT, packing, e + c);
    }
}

// ----------------------------------------------------------------------------------------------
// K6: pack / unpack of one round of the irregular allgather (Alg. 9, its "Pack" and "Unpack" loops).
// The message is the concatenation, root by root, of one block of each buffer; buffers have any
// sizes (Section 3.2 uses (r mod 3) * floor(m/p)), a buffer of m elements is cut into n blocks at
// floor(b*m/n).  Three small kernels make the plan -- each root's block length and source offset, an
// exclusive scan of the lengths (1024 roots per workgroup, then the workgroup totals, then the sum) --
// and one kernel moves the payload: it walks the MESSAGE in 16-byte pieces (aligned on that side), a
// lane finds the root of its piece by a search that starts where its previous piece ended, and the
// buffer side is read or written with whatever alignment the block happens to have.
// ----------------------------------------------------------------------------------------------
constexpr int kPlanRoots = 1024;                     // roots per workgroup in the scan (4 per lane)

struct PackPlan {
    int64_t *offsets;                                // [p+1] message offset of each root's block; [p] = length
    int64_t *src;                                    // [p]   element offset of that block inside `data`
    int64_t *totals;                                 // [ceil(p / kPlanRoots) + 1] workgroup totals, then their scan
};

// four consecutive roots of one lane: block lengths into len[], block positions into plan.src; returns their sum
__device__ __forceinline__ int64_t plan_roots(uint32_t p, uint32_t n, const int32_t *__restrict__ idx,
                                              const int64_t *__restrict__ displs, const PackPlan &plan,
                                              uint64_t first, int64_t (&len)[4]) {
    int64_t mine = 0;
#pragma unroll
    for (int c = 0; c < 4; ++c) {
        const uint64_t j = first + c;
        len[c] = 0;
        if (j < p) {
            const int64_t begin = displs[j], m = displs[j + 1] - begin;
            int64_t b = idx[j];
            b = b > (int64_t)n - 1 ? (int64_t)n - 1 : b;             // caption of Alg. 9: beyond n-1 means n-1
            int64_t lo = 0, hi = 0;
            if (b >= 0 && m > 0) {
                lo = (int64_t)(((uint64_t)b * (uint64_t)m) / n);
                hi = (int64_t)((((uint64_t)b + 1u) * (uint64_t)m) / n);
            }
            plan.src[j] = begin + lo;
            len[c] = hi - lo;
        }
        mine += len[c];
    }
    return mine;
}

// exclusive scan of `mine` over the workgroup: inside a wave by shuffles, across the four waves through LDS
// (wave_sum: kBlock / 64 entries; contains a barrier)
__device__ __forceinline__ int64_t plan_scan(int64_t mine, int64_t *wave_sum) {
    int64_t incl = mine;
    const int lane = threadIdx.x & 63;
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) {
        const int64_t up = __shfl_up(incl, off, 64);
        if (lane >= off) incl += up;
    }
    if (lane == 63) wave_sum[threadIdx.x >> 6] = incl;
    __syncthreads();
    int64_t before = incl - mine;
    for (int w = 0; w < (int)(threadIdx.x >> 6); ++w) before += wave_sum[w];
    return before;
}

__global__ __launch_bounds__(kBlock) void k_pack_plan_local(uint32_t p, uint32_t n, const int32_t *__restrict__ idx,
                                                            const int64_t *__restrict__ displs, PackPlan plan) {
    __shared__ int64_t wave_sum[kBlock / 64];
    const uint64_t first = (uint64_t)blockIdx.x * kPlanRoots + threadIdx.x * 4u;
    int64_t len[4];
    const int64_t mine = plan_roots(p, n, idx, displs, plan, first, len);
    int64_t before = plan_scan(mine, wave_sum);
    if (threadIdx.x == kBlock - 1) plan.totals[blockIdx.x] = before + mine;
#pragma unroll
    for (int c = 0; c < 4; ++c) {
        const uint64_t j = first + c;
        if (j < p) plan.offsets[j] = before;
        before += len[c];
    }
}

// The whole plan in one workgroup, for the few thousand processes of the paper's runs: one launch instead
// of three (a round is launch-latency bound at those sizes).
constexpr uint32_t kPlanOneMaxP = 8 * kPlanRoots;

__global__ __launch_bounds__(kBlock) void k_pack_plan_one(uint32_t p, uint32_t n, const int32_t *__restrict__ idx,
                                                          const int64_t *__restrict__ displs, PackPlan plan) {
    __shared__ int64_t wave_sum[kBlock / 64];
    __shared__ int64_t carry_s;
    if (threadIdx.x == 0) carry_s = 0;
    __syncthreads();
    for (uint64_t base = 0; base < p; base += kPlanRoots) {
        const uint64_t first = base + threadIdx.x * 4u;
        int64_t len[4];
        const int64_t mine = plan_roots(p, n, idx, displs, plan, first, len);
        const int64_t carry = carry_s;
        int64_t before = carry + plan_scan(mine, wave_sum);
        const int64_t end = before + mine;
#pragma unroll
        for (int c = 0; c < 4; ++c) {
            const uint64_t j = first + c;
            if (j < p) plan.offsets[j] = before;
            before += len[c];
        }
        __syncthreads();                                            // everyone has read carry_s and wave_sum
        if (threadIdx.x == kBlock - 1) carry_s = end;
        __syncthreads();
    }
    if (threadIdx.x == 0) plan.offsets[p] = carry_s;
}

// one workgroup: exclusive scan of the workgroup totals in place; the grand total goes to offsets[p]
__global__ __launch_bounds__(kBlock) void k_pack_plan_totals(uint32_t p, uint32_t groups, PackPlan plan) {
    __shared__ int64_t wave_sum[kBlock / 64];
    __shared__ int64_t carry_s;
    if (threadIdx.x == 0) carry_s = 0;
    __syncthreads();
    const int lane = threadIdx.x & 63;
    for (uint32_t base = 0; base < groups; base += kBlock) {
        const uint32_t g = base + threadIdx.x;
        const int64_t mine = g < groups ? plan.totals[g] : 0;
        int64_t incl = mine;
#pragma unroll
        for (int off = 1; off < 64; off <<= 1) {
            const int64_t up = __shfl_up(incl, off, 64);
            if (lane >= off) incl += up;
        }
        if (lane == 63) wave_sum[threadIdx.x >> 6] = incl;
        __syncthreads();
        int64_t before = carry_s + incl - mine;
        for (int w = 0; w < (int)(threadIdx.x >> 6); ++w) before += wave_sum[w];
        if (g < groups) plan.totals[g] = before;
        __syncthreads();
        if (threadIdx.x == kBlock - 1) carry_s = before + mine;
        __syncthreads();
    }
    if (threadIdx.x == 0) plan.offsets[p] = carry_s;
}

__global__ __launch_bounds__(kBlock) void k_pack_plan_finish(uint32_t p, PackPlan plan) {
    const uint64_t j = (uint64_t)blockIdx.x * kBlock + threadIdx.x;
    if (j < p) plan.offsets[j] += plan.totals[j / kPlanRoots];
}

constexpr int kCopyIter = 4;                          // 16-byte pieces per lane, long messages
constexpr int64_t kCopyShort = 4 << 20;               // message elements below which a lane takes one piece

// PACK: data -> message.  !PACK: message -> data.  `limit` = capacity (pack) or message length (unpack).
// A wave first finds the root of its first element together (64 probes of `offsets` per step), each lane then
// walks on from there; the roots of a lane's ITER pieces are all found before any payload is touched, so
// that the payload loads of the pieces are in flight together.
// Short messages (a few hundred KB in the paper's runs) take one piece a lane, which gives four times the
// workgroups: 6 us against 16 us for 241 KB; long ones take kCopyIter (0.10 ms against 0.15 ms for 239 MB).
template <bool PACK, int ITER>
__global__ __launch_bounds__(kBlock) void k_pack_copy(uint32_t p, int64_t limit, const int64_t *__restrict__ offsets,
                                                      const int64_t *__restrict__ src, int32_t *data,
                                                      int32_t *message, int msg_aligned) {
    int64_t end = offsets[p];
    end = end < limit ? end : limit;
    const int64_t e0 = (int64_t)blockIdx.x * (ITER * kBlock * 4) + threadIdx.x * 4;
    const int64_t e_wave = (int64_t)blockIdx.x * (ITER * kBlock * 4) + (threadIdx.x & ~63u) * 4;
    if (e_wave >= end) return;                                      // the whole wave leaves together
    // root of the wave's first element: the last j with offsets[j] <= e_wave, answer in [lo, hi)
    uint32_t lo = 0, hi = p;
    const uint32_t lane = threadIdx.x & 63u;
    while (hi - lo > 1u) {
        const uint32_t step = (hi - lo + 63u) >> 6;
        const uint64_t probe = (uint64_t)lo + (uint64_t)(lane + 1u) * step;
        const bool below = probe < hi && offsets[probe] <= e_wave;  // true for a prefix of the lanes
        const uint32_t c = (uint32_t)__popcll(__ballot(below));
        const uint64_t nlo = (uint64_t)lo + (uint64_t)c * step;
        const uint64_t nhi = nlo + step;
        lo = (uint32_t)nlo;
        hi = nhi < hi ? (uint32_t)nhi : hi;
    }
    uint32_t j = lo;
    // the pieces of this lane: 0 = none, 1 = whole piece inside one root's block, 2 = crosses a boundary
    int kind[ITER];
    int32_t *inner[ITER];
    uint32_t first_root[ITER];
#pragma unroll
    for (int it = 0; it < ITER; ++it) {
        const int64_t e = e0 + (int64_t)it * kBlock * 4;
        kind[it] = 0;
        inner[it] = data;
        first_root[it] = j;
        if (e >= end) continue;
        // move on to the root that holds element e: gallop, then bisect
        if (offsets[j + 1] <= e) {
            uint32_t step = 1, a = j + 1;                           // offsets[a] <= e
            while (a + step < p && offsets[a + step] <= e) { a += step; step <<= 1; }
            uint32_t b = a + step < p ? a + step : p;               // offsets[b] > e or b == p
            while (b - a > 1u) {
                const uint32_t mid = a + ((b - a) >> 1);
                if (offsets[mid] <= e) a = mid; else b = mid;
            }
            j = a;
        }
        const int64_t seg_begin = offsets[j], seg_end = offsets[j + 1];
        first_root[it] = j;
        if (e + 4 <= seg_end && e + 4 <= end) {
            kind[it] = 1;
            inner[it] = data + src[j] + (e - seg_begin);
        } else {
            kind[it] = 2;
        }
    }
    v4i val[ITER];
#pragma unroll
    for (int it = 0; it < ITER; ++it) {
        if (kind[it] != 1) continue;
        const int64_t e = e0 + (int64_t)it * kBlock * 4;
        if (PACK) {
            const int32_t *d = inner[it];
            val[it] = (v4i){d[0], d[1], d[2], d[3]};
        } else if (msg_aligned) {
            val[it] = *reinterpret_cast<const v4i *>(message + e);
        } else {
            val[it] = (v4i){message[e], message[e + 1], message[e + 2], message[e + 3]};
        }
    }
#pragma unroll
    for (int it = 0; it < ITER; ++it) {
        if (kind[it] != 1) continue;
        const int64_t e = e0 + (int64_t)it * kBlock * 4;
        const v4i v = val[it];
        if (PACK) {
            if (msg_aligned) __builtin_nontemporal_store(v, reinterpret_cast<v4i *>(message + e));
            else { message[e] = v[0]; message[e + 1] = v[1]; message[e + 2] = v[2]; message[e + 3] = v[3]; }
        } else {
            int32_t *d = inner[it];
            d[0] = v[0]; d[1] = v[1]; d[2] = v[2]; d[3] = v[3];
        }
    }
    // pieces that cross into other roots' blocks (or the end): element by element
#pragma unroll
    for (int it = 0; it < ITER; ++it) {
        if (kind[it] != 2) continue;
        const int64_t e = e0 + (int64_t)it * kBlock * 4;
        uint32_t jj = first_root[it];
        for (int c = 0; c < 4; ++c) {
            const int64_t ee = e + c;
            if (ee >= end) break;
            while (offsets[jj + 1] <= ee) ++jj;                     // ends: offsets[p] = length > ee
            int32_t *d = data + src[jj] + (ee - offsets[jj]);
            if (PACK) message[ee] = *d; else *d = message[ee];
        }
    }
}

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

// Alg. 1
int host_skips(int32_t p, SkipTab &t) {
    const int q = host_q(p);
    int k = q;
    uint32_t v = (uint32_t)p;
    while (v > 1u) {
        t.s[k] = v;
        v = v / 2u + v % 2u;
        --k;
    }
    t.s[k] = v;
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

struct Scratch {
    void *ptr = nullptr;
    size_t bytes = 0;
};
Scratch g_scratch[kMaxDevices];
std::mutex g_scratch_mutex;

int scratch_get(size_t bytes, void **out) {
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return hip_fail(e);
    if (dev < 0 || dev >= kMaxDevices) return BCS_EINVAL;
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    Scratch &s = g_scratch[dev];
    if (s.bytes < bytes) {
        if (s.ptr) {
            e = hipDeviceSynchronize();
            if (e != hipSuccess) return hip_fail(e);
            e = hipFree(s.ptr);
            s.ptr = nullptr;
            s.bytes = 0;
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
    *out = s.ptr;
    return BCS_OK;
}

inline uint64_t round_up(uint64_t v, uint64_t m) { return (v + m - 1) / m * m; }

// row length of the slot-major receive table (rows start on 256-byte boundaries)
inline uint64_t slot_ld(int32_t p) { return round_up((uint64_t)p, 256); }

template <int Q>
int launch_sched(const SkipTab &tab, uint32_t root, uint32_t r0, uint32_t r1, int32_t *recv_out, int32_t *send_out,
                 slot_t *recvT, uint64_t ldT, int8_t *recvB, int8_t *sendB, hipStream_t st) {
    const uint64_t count = (uint64_t)r1 - r0;
    const unsigned blocks = (unsigned)((count + kBlock - 1) / kBlock);
    const bool full = (r0 == 0 && r1 == tab.s[Q]);
    // the slot-major copy feeds the send look-up; with neither table asked for it is the only output
    const bool want_t = full && recvT && (send_out || !recv_out);
    if (recv_out || want_t) {
        if (full && recvB && recv_out)
            launch(kRecv, k_recv_uniform<Q, true>, dim3(blocks), dim3(kBlock), st, tab, root, r0, r1, recv_out,
                   want_t ? recvT : (slot_t *)nullptr, ldT, recvB);
        else
            launch(kRecv, k_recv_uniform<Q, false>, dim3(blocks), dim3(kBlock), st, tab, root, r0, r1, recv_out,
                   want_t ? recvT : (slot_t *)nullptr, ldT, (int8_t *)nullptr);
    }
    if (send_out) {
        if (full) {
            launch(kSendLookup, k_send_lookup<Q>, dim3(blocks), dim3(kBlock), st, tab, (const slot_t *)recvT, ldT,
                   send_out, sendB);
        } else {
            launch(kSendRecompute, k_send_recompute<Q>, dim3(blocks), dim3(kBlock), st, tab, root, r0, r1, send_out);
        }
    }
    hipError_t e = hipGetLastError();
    return e == hipSuccess ? BCS_OK : hip_fail(e);
}

typedef int (*LaunchFn)(const SkipTab &, uint32_t, uint32_t, uint32_t, int32_t *, int32_t *, slot_t *, uint64_t,
                        int8_t *, int8_t *, hipStream_t);

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
constexpr uint64_t kFusedMaxR = 160;               // rows up to this length: fused when p >= kFusedMinP
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

int64_t bcs_sched_workspace_bytes(int32_t p, int32_t r0, int32_t r1, int want_send) {
    if (check_range(p, 0, r0, r1) != BCS_OK) return BCS_EINVAL;
    const int q = host_q(p);
    if (!want_send || q == 0 || !(r0 == 0 && r1 == p)) return 0;
    const uint64_t ld = slot_ld(p);
    return (int64_t)(ld * (uint64_t)q * sizeof(slot_t));
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
    SkipTab tab;
    host_skips(p, tab);
    rc = ensure_lowtab((hipStream_t)stream);
    if (rc != BCS_OK) return rc;
    const uint64_t ld = slot_ld(p);
    return launch_for_q(q)(tab, (uint32_t)root, (uint32_t)r0, (uint32_t)r1, recv_out, send_out,
                           need > 0 ? (slot_t *)workspace : nullptr, ld, nullptr, nullptr, (hipStream_t)stream);
}

int bcs_sched_rooted(int32_t p, int32_t root, int32_t r0, int32_t r1, int32_t *recv_out, int32_t *send_out,
                     void *stream) {
    int rc = check_range(p, root, r0, r1);
    if (rc != BCS_OK) return rc;
    if (!recv_out && !send_out) return BCS_EINVAL;
    const int64_t need = bcs_sched_workspace_bytes(p, r0, r1, send_out != nullptr);
    void *ws = nullptr;
    if (need > 0 && r0 != r1) {
        rc = scratch_get((size_t)need, &ws);
        if (rc != BCS_OK) return rc;
    }
    return bcs_sched_rooted_ws(p, root, r0, r1, recv_out, send_out, ws, (size_t)need, stream);
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
                                 slot_ld(p), recvB, sendB, (hipStream_t)stream);
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
        const int rc = scratch_get((size_t)need, &ws);
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
    SkipTab tab;
    host_skips(p, tab);
    int rc = ensure_lowtab(st);
    if (rc != BCS_OK) return rc;
    const uint64_t ld = slot_ld(p);
    slot_t *recvT = (slot_t *)workspace;
    rc = launch_for_q(q)(tab, 0u, 0u, (uint32_t)p, nullptr, nullptr, recvT, ld, nullptr, nullptr, st);
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
        const int rc = scratch_get((size_t)need, &ws);
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

int bcs_pack_round(int32_t p, int32_t n, const int32_t *idx, const int64_t *displs, const int32_t *data,
                   int32_t *packed, int64_t capacity, int64_t *offsets, void *workspace, size_t workspace_bytes,
                   void *stream) {
    if (!data || capacity < 0 || (!packed && capacity > 0)) return BCS_EINVAL;
    if (((uint64_t)capacity + kBlock * 4 - 1) / (kBlock * 4) > 0x7fffffffull) return BCS_EINVAL;
    PackPlan plan;
    const int rc = pack_plan(p, n, idx, displs, offsets, workspace, workspace_bytes, (hipStream_t)stream, plan);
    if (rc != BCS_OK || capacity == 0) return rc;
    const int aligned = (int)((((uintptr_t)packed) & 15u) == 0);
    if (capacity < kCopyShort) {
        const uint64_t blocks = ((uint64_t)capacity + kBlock * 4 - 1) / (kBlock * 4);
        launch(kPackCopy, k_pack_copy<true, 1>, dim3((unsigned)blocks), dim3(kBlock), (hipStream_t)stream, (uint32_t)p,
               capacity, (const int64_t *)offsets, (const int64_t *)plan.src, const_cast<int32_t *>(data), packed,
               aligned);
    } else {
        const uint64_t chunk = (uint64_t)kCopyIter * kBlock * 4;
        const uint64_t blocks = ((uint64_t)capacity + chunk - 1) / chunk;
        launch(kPackCopy, k_pack_copy<true, kCopyIter>, dim3((unsigned)blocks), dim3(kBlock), (hipStream_t)stream,
               (uint32_t)p, capacity, (const int64_t *)offsets, (const int64_t *)plan.src,
               const_cast<int32_t *>(data), packed, aligned);
    }
    hipError_t e = hipGetLastError();
    return e == hipSuccess ? BCS_OK : hip_fail(e);
}

int bcs_unpack_round(int32_t p, int32_t n, const int32_t *idx, const int64_t *displs, int32_t *data,
                     const int32_t *packed, int64_t length, int64_t *offsets, void *workspace, size_t workspace_bytes,
                     void *stream) {
    if (!data || length < 0 || (!packed && length > 0)) return BCS_EINVAL;
    if (((uint64_t)length + kBlock * 4 - 1) / (kBlock * 4) > 0x7fffffffull) return BCS_EINVAL;
    PackPlan plan;
    const int rc = pack_plan(p, n, idx, displs, offsets, workspace, workspace_bytes, (hipStream_t)stream, plan);
    if (rc != BCS_OK || length == 0) return rc;
    const int aligned = (int)((((uintptr_t)packed) & 15u) == 0);
    if (length < kCopyShort) {
        const uint64_t blocks = ((uint64_t)length + kBlock * 4 - 1) / (kBlock * 4);
        launch(kPackCopy, k_pack_copy<false, 1>, dim3((unsigned)blocks), dim3(kBlock), (hipStream_t)stream, (uint32_t)p,
               length, (const int64_t *)offsets, (const int64_t *)plan.src, data, const_cast<int32_t *>(packed),
               aligned);
    } else {
        const uint64_t chunk = (uint64_t)kCopyIter * kBlock * 4;
        const uint64_t blocks = ((uint64_t)length + chunk - 1) / chunk;
        launch(kPackCopy, k_pack_copy<false, kCopyIter>, dim3((unsigned)blocks), dim3(kBlock), (hipStream_t)stream,
               (uint32_t)p, length, (const int64_t *)offsets, (const int64_t *)plan.src, data,
               const_cast<int32_t *>(packed), aligned);
    }
    hipError_t e = hipGetLastError();
    return e == hipSuccess ? BCS_OK : hip_fail(e);
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
        default: return "unknown bcsched error code";
    }
}

int bcs_last_hip_error(void) { return g_last_hip; }

}  // extern "C"
