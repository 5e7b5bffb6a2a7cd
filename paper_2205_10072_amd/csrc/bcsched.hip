// libbcsched: round-optimal broadcast schedules on a circulant graph, built on gfx950.
//
// Method: J. L. Traff, arXiv 2205.10072, Section 2 (Alg. 1, 2, 4, 5; index arithmetic of Alg. 6).
// One lane owns one rank.  Everything is 32-bit integer work on the vector ALU; block sets are
// 32-bit masks (q <= 31); the skips of a uniform-p launch live in scalar registers.
//
// The per-rank construction is in bcs_core.h; this file holds the kernels and the C ABI.
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <utility>

#include "bcsched.h"
#include "bcs_core.h"

namespace {

using namespace bcs;
static_assert(kMaxQ == BCS_MAX_Q, "header and core disagree");
constexpr int kBlock = 256;              // lanes (= ranks) per workgroup

thread_local int g_last_hip = 0;

inline int hip_fail(hipError_t e) {
    g_last_hip = (int)e;
    return BCS_EHIP;
}

// ----------------------------------------------------------------------------------------------
// K1: receive rows of ranks [r0, r1), uniform p.  Lane = rank.  Rows are staged in LDS (odd stride,
// conflict-free) and leave as contiguous dwords; optionally each entry is also stored slot-major
// (recvT[k][r - r0]) for the send look-up that follows.
// ----------------------------------------------------------------------------------------------
template <int Q>
__global__ __launch_bounds__(kBlock) void k_recv_uniform(const SkipTab tab, uint32_t root, uint32_t r0, uint32_t r1,
                                                         int32_t *__restrict__ recv_out,
                                                         int32_t *__restrict__ recvT, uint64_t ldT) {
    constexpr int kStride = Q | 1;
    __shared__ int32_t tile[kBlock * kStride];
    Uniform<Q> pol;
#pragma unroll
    for (int k = 0; k <= Q; ++k) pol.S[k] = tab.s[k];
    pol.tab = &tab;
    const uint32_t p = pol.p();
    const uint64_t first = (uint64_t)blockIdx.x * kBlock;       // offset of this tile inside [r0, r1)
    const uint64_t idx = first + threadIdx.x;
    const uint64_t count = (uint64_t)r1 - r0;
    const bool live = idx < count;
    const uint32_t r = live ? (uint32_t)(r0 + idx) : root;       // idle lanes replay the root (cheap, valid)
    const uint32_t v = r >= root ? r - root : r + p - root;
    int32_t *my = tile + threadIdx.x * kStride;
    recv_row(pol, v, Q - 1, [&](int i, int val) {
        my[i] = val;
        if (recvT && live) recvT[(uint64_t)i * ldT + idx] = val;
    });
    if (!recv_out) return;
    __syncthreads();
    const uint64_t rows = (count - first) < (uint64_t)kBlock ? (count - first) : (uint64_t)kBlock;
    const uint32_t n = (uint32_t)rows * Q;
    int32_t *dst = recv_out + first * Q;
    for (uint32_t e = threadIdx.x; e < n; e += kBlock) {
        const uint32_t row = e / Q, col = e - row * Q;
        dst[e] = tile[row * kStride + col];
    }
}

// K2: send rows from the slot-major receive table of ALL ranks (Alg. 9, second loop):
// send[r][k] = recv[(r + skips[k]) mod p][k].  Reads are contiguous per slot, rows leave through LDS.
template <int Q>
__global__ __launch_bounds__(kBlock) void k_send_lookup(const SkipTab tab, const int32_t *__restrict__ recvT,
                                                        uint64_t ldT, int32_t *__restrict__ send_out) {
    constexpr int kStride = Q | 1;
    __shared__ int32_t tile[kBlock * kStride];
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
    const uint32_t n = (uint32_t)rows * Q;
    int32_t *dst = send_out + first * Q;
    for (uint32_t e = threadIdx.x; e < n; e += kBlock) {
        const uint32_t row = e / Q, col = e - row * Q;
        dst[e] = tile[row * kStride + col];
    }
}

// K1b: send rows of ranks [r0, r1) with no neighbour rows at hand (Alg. 5): entry i is entry i of the
// receive schedule of the to-neighbour, which costs that neighbour's rounds 0..i.
template <int Q>
__global__ __launch_bounds__(kBlock) void k_send_recompute(const SkipTab tab, uint32_t root, uint32_t r0, uint32_t r1,
                                                           int32_t *__restrict__ send_out) {
    constexpr int kStride = Q | 1;
    __shared__ int32_t tile[kBlock * kStride];
    Uniform<Q> pol;
#pragma unroll
    for (int k = 0; k <= Q; ++k) pol.S[k] = tab.s[k];
    pol.tab = &tab;
    const uint32_t p = pol.p();
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
        int32_t keep = 0;
        recv_row(pol, t, i, [&](int j, int val) { keep = (j == i) ? val : keep; });
        my[i] = keep;
    }
    __syncthreads();
    const uint64_t rows = (count - first) < (uint64_t)kBlock ? (count - first) : (uint64_t)kBlock;
    const uint32_t n = (uint32_t)rows * Q;
    int32_t *dst = send_out + first * Q;
    for (uint32_t e = threadIdx.x; e < n; e += kBlock) {
        const uint32_t row = e / Q, col = e - row * Q;
        dst[e] = tile[row * kStride + col];
    }
}

// K3: unrelated (p, r, root) triples, one per lane; rows of BCS_BATCH_STRIDE ints, padded.
__global__ __launch_bounds__(kBlock) void k_batch(int64_t count, const int32_t *__restrict__ pv,
                                                  const int32_t *__restrict__ rv, const int32_t *__restrict__ rootv,
                                                  int32_t *__restrict__ recv_out, int32_t *__restrict__ send_out,
                                                  int32_t *__restrict__ q_out) {
    constexpr int kStride = BCS_BATCH_STRIDE + 1;
    __shared__ int32_t tile[kBlock * kStride];
    const int64_t first = (int64_t)blockIdx.x * kBlock;
    const int64_t idx = first + threadIdx.x;
    const bool live = idx < count;
    int32_t pi = live ? pv[idx] : 1, ri = live ? rv[idx] : 0, rooti = live ? rootv[idx] : 0;
    const bool valid = live && pi >= 1 && ri >= 0 && ri < pi && rooti >= 0 && rooti < pi;
    if (!valid) { pi = 1; ri = 0; rooti = 0; }
    const uint32_t p = (uint32_t)pi;
    const int q = p > 1u ? 32 - __clz((int)(p - 1u)) : 0;
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
    const uint32_t v = (uint32_t)ri >= (uint32_t)rooti ? (uint32_t)(ri - rooti) : (uint32_t)ri + p - (uint32_t)rooti;
    int32_t *my = tile + threadIdx.x * kStride;
    const int64_t rows = (count - first) < (int64_t)kBlock ? (count - first) : (int64_t)kBlock;
    const uint32_t n = (uint32_t)rows * BCS_BATCH_STRIDE;

    if (recv_out) {
#pragma unroll
        for (int k = 0; k < BCS_BATCH_STRIDE; ++k) my[k] = BCS_BATCH_PAD;
        recv_row(pol, v, qmax - 1, [&](int i, int val) { my[i] = val; });
        __syncthreads();
        int32_t *dst = recv_out + first * BCS_BATCH_STRIDE;
        for (uint32_t e = threadIdx.x; e < n; e += kBlock)
            dst[e] = tile[(e >> 5) * kStride + (e & 31u)];
        __syncthreads();
    }
    if (send_out) {
#pragma unroll
        for (int k = 0; k < BCS_BATCH_STRIDE; ++k) my[k] = BCS_BATCH_PAD;
#pragma unroll 1
        for (int i = 0; i < qmax; ++i) {
            uint32_t t = v + (i < q ? pol.s(i) : 0u);
            t = t >= p ? t - p : t;
            int32_t keep = 0;
            recv_row(pol, t, i, [&](int j, int val) { keep = (j == i) ? val : keep; });
            if (i < q) my[i] = keep;
        }
        __syncthreads();
        int32_t *dst = send_out + first * BCS_BATCH_STRIDE;
        for (uint32_t e = threadIdx.x; e < n; e += kBlock)
            dst[e] = tile[(e >> 5) * kStride + (e & 31u)];
    }
}

// ----------------------------------------------------------------------------------------------
// K4: expansion (Alg. 6 index arithmetic).  Real round j uses slot k = (x+j) mod q and the value
// sched[k] + q*floor((x+j)/q) - x: slots below x were advanced once by the x dummy rounds, which
// the floor term already counts.  Negative -> BCS_NO_BLOCK, above n-1 -> n-1.  A workgroup owns a
// panel of kExpCols rounds and walks down the rows; lanes are consecutive rounds, so stores are
// contiguous and each lane keeps its slot and offset in registers for the whole walk.
// ----------------------------------------------------------------------------------------------
constexpr int kExpCols = kBlock;          // rounds per panel (one per lane)
constexpr int kExpRows = 64;              // rows staged in LDS per step

__global__ __launch_bounds__(kBlock) void k_expand(int q, uint32_t x, int32_t nm1, uint64_t rows, uint64_t R,
                                                   uint32_t rows_per_block,
                                                   const int32_t *__restrict__ in, int32_t *__restrict__ out) {
    __shared__ int32_t tile[kExpRows * (kMaxQ + 1)];
    const uint64_t j = (uint64_t)blockIdx.x * kExpCols + threadIdx.x;
    const bool col_live = j < R;
    const uint64_t i = (uint64_t)x + j;
    const uint32_t phase = (uint32_t)(i / (uint32_t)q);
    const int k = (int)(i - (uint64_t)phase * q);
    const int64_t off64 = (int64_t)phase * q - (int64_t)x;
    const uint64_t row_begin = (uint64_t)blockIdx.y * rows_per_block;
    uint64_t row_end = row_begin + rows_per_block;
    if (row_end > rows) row_end = rows;
    for (uint64_t rb = row_begin; rb < row_end; rb += kExpRows) {
        const uint32_t nr = (uint32_t)((row_end - rb) < (uint64_t)kExpRows ? (row_end - rb) : (uint64_t)kExpRows);
        const uint32_t cnt = nr * (uint32_t)q;
        __syncthreads();
        const int32_t *src = in + rb * (uint64_t)q;
        for (uint32_t e = threadIdx.x; e < cnt; e += kBlock) tile[e] = src[e];
        __syncthreads();
        if (col_live) {
            int32_t *dst = out + rb * R + j;
            for (uint32_t rr = 0; rr < nr; ++rr) {
                int64_t val = (int64_t)tile[rr * (uint32_t)q + k] + off64;
                val = val < 0 ? -1 : (val > nm1 ? nm1 : val);
                dst[(uint64_t)rr * R] = (int32_t)val;
            }
        }
    }
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
    return q;
}

struct Scratch {
    void *ptr = nullptr;
    size_t bytes = 0;
};
constexpr int kMaxDevices = 64;
Scratch g_scratch[kMaxDevices];

int scratch_get(size_t bytes, void **out) {
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return hip_fail(e);
    if (dev < 0 || dev >= kMaxDevices) return BCS_EINVAL;
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

template <int Q>
int launch_sched(const SkipTab &tab, uint32_t root, uint32_t r0, uint32_t r1, int32_t *recv_out, int32_t *send_out,
                 int32_t *recvT, uint64_t ldT, hipStream_t st) {
    const uint64_t count = (uint64_t)r1 - r0;
    const unsigned blocks = (unsigned)((count + kBlock - 1) / kBlock);
    const bool full = (r0 == 0 && r1 == tab.s[Q]);
    if (recv_out || (send_out && full)) {
        hipLaunchKernelGGL(k_recv_uniform<Q>, dim3(blocks), dim3(kBlock), 0, st, tab, root, r0, r1, recv_out,
                           (send_out && full) ? recvT : (int32_t *)nullptr, ldT);
    }
    if (send_out) {
        if (full) {
            hipLaunchKernelGGL(k_send_lookup<Q>, dim3(blocks), dim3(kBlock), 0, st, tab, (const int32_t *)recvT, ldT,
                               send_out);
        } else {
            hipLaunchKernelGGL(k_send_recompute<Q>, dim3(blocks), dim3(kBlock), 0, st, tab, root, r0, r1, send_out);
        }
    }
    hipError_t e = hipGetLastError();
    return e == hipSuccess ? BCS_OK : hip_fail(e);
}

typedef int (*LaunchFn)(const SkipTab &, uint32_t, uint32_t, uint32_t, int32_t *, int32_t *, int32_t *, uint64_t,
                        hipStream_t);

template <int... Qs>
constexpr void fill_table(LaunchFn *t, std::integer_sequence<int, Qs...>) {
    ((t[Qs] = &launch_sched<Qs + 1>), ...);
}

LaunchFn launch_for_q(int q) {
    static LaunchFn table[kMaxQ] = {};
    static bool ready = false;
    if (!ready) {
        fill_table(table, std::make_integer_sequence<int, kMaxQ>{});
        ready = true;
    }
    return table[q - 1];
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
    const uint64_t ld = round_up((uint64_t)p, 64);
    return (int64_t)(ld * (uint64_t)q * sizeof(int32_t));
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
    const uint64_t ld = round_up((uint64_t)p, 64);
    return launch_for_q(q)(tab, (uint32_t)root, (uint32_t)r0, (uint32_t)r1, recv_out, send_out,
                           need > 0 ? (int32_t *)workspace : nullptr, ld, (hipStream_t)stream);
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
    const uint64_t blocks = ((uint64_t)count + kBlock - 1) / kBlock;
    if (blocks > 0x7fffffffull) return BCS_EINVAL;
    hipLaunchKernelGGL(k_batch, dim3((unsigned)blocks), dim3(kBlock), 0, (hipStream_t)stream, count, p, r, root,
                       recv_out, send_out, q_out);
    hipError_t e = hipGetLastError();
    return e == hipSuccess ? BCS_OK : hip_fail(e);
}

int bcs_expand(int32_t p, int32_t n, int32_t r0, int32_t r1, const int32_t *recv, const int32_t *send,
               int32_t *recv_blocks, int32_t *send_blocks, void *stream) {
    if (check_range(p, 0, r0, r1) != BCS_OK || n < 1) return BCS_EINVAL;
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
            hipLaunchKernelGGL(k_fill, dim3(1024), dim3(kBlock), 0, st, outs[t], rows * R, (int32_t)BCS_NO_BLOCK);
            continue;
        }
        const uint32_t x = (uint32_t)((q - (int)(R % (uint64_t)q)) % q);
        const uint64_t panels = (R + kExpCols - 1) / kExpCols;
        // enough workgroups to fill 256 CUs several times over, rows split in multiples of the LDS step
        uint64_t want_y = (8192 + panels - 1) / panels;
        uint64_t rpb = (rows + want_y - 1) / want_y;
        rpb = round_up(rpb < 1 ? 1 : rpb, kExpRows);
        const uint64_t gy = (rows + rpb - 1) / rpb;
        if (panels > 0x7fffffffull || gy > 65535ull) {
            // fall back to fewer, taller workgroups
            rpb = round_up((rows + 65534ull) / 65535ull, kExpRows);
        }
        const uint64_t gy2 = (rows + rpb - 1) / rpb;
        hipLaunchKernelGGL(k_expand, dim3((unsigned)panels, (unsigned)gy2), dim3(kBlock), 0, st, q, x, (int32_t)(n - 1),
                           rows, R, (uint32_t)rpb, ins[t], outs[t]);
    }
    hipError_t e = hipGetLastError();
    return e == hipSuccess ? BCS_OK : hip_fail(e);
}

int bcs_release(void) {
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return hip_fail(e);
    if (dev < 0 || dev >= kMaxDevices) return BCS_EINVAL;
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
