// Irregular allgather (Alg. 9; Section 2.4): the pack / unpack index tables of one process and the packing and
// unpacking of one round's message.
#ifndef BCS_KERNELS_ALLGATHER_H
#define BCS_KERNELS_ALLGATHER_H

#include "bcs_kernels_common.h"

namespace {

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

// The whole plan of a round in one workgroup, for the few thousand processes of the paper's runs: one launch
// instead of three (a round is launch-latency bound at those sizes).  A grid of several workgroups plans as many
// rounds at once: workgroup b takes row b of an index table (rows of p entries, as bcs_allgather_tables writes
// them) and fills row b of the offsets (p + 1 entries a row) and of the block positions (p entries a row).
constexpr uint32_t kPlanOneMaxP = 8 * kPlanRoots;

__global__ __launch_bounds__(kBlock) void k_pack_plan_one(uint32_t p, uint32_t n, const int32_t *__restrict__ idx_rows,
                                                          const int64_t *__restrict__ displs, PackPlan all) {
    __shared__ int64_t wave_sum[kBlock / 64];
    __shared__ int64_t carry_s;
    const int32_t *idx = idx_rows + (uint64_t)blockIdx.x * p;
    PackPlan plan;
    plan.offsets = all.offsets + (uint64_t)blockIdx.x * ((uint64_t)p + 1u);
    plan.src = all.src + (uint64_t)blockIdx.x * p;
    plan.totals = nullptr;
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

// ----------------------------------------------------------------------------------------------
// Partner tables of the regular allgather (Alg. 7) and of the census (Alg. 8) for a range of processes:
// to[(r - r0) q + k] = (r - dist_k + p) mod p, from[(r - r0) q + k] = (r + dist_k) mod p, where dist_k = skips[k]
// for Alg. 7 and skips[k] minus one at the odd levels (2 skips[k] > skips[k+1]) for Alg. 8.  Pure stores: a
// workgroup writes one 4 KB piece of each table (a lane 16 bytes of each), the shape in which store-only kernels
// come closest to the HBM's rate on this GPU.  The skips come from Alg. 1's halving in closed form,
// skips[k] = ((p-1) >> (q-k)) + 1, and level k is odd when bit q-1-k of p-1 is clear.
// ----------------------------------------------------------------------------------------------
template <bool VEC>
__global__ __launch_bounds__(kBlock) void k_partner_tables(uint32_t p, uint32_t q, uint32_t census, uint32_t r0,
                                                           uint64_t total, int32_t *__restrict__ to,
                                                           int32_t *__restrict__ from) {
    const uint64_t e0 = ((uint64_t)blockIdx.x * kBlock + threadIdx.x) * 4;
    if (e0 >= total) return;
    const uint64_t row = e0 / q;
    uint32_t k = (uint32_t)(e0 - row * q);
    uint32_t r = r0 + (uint32_t)row;
    const uint32_t pm1 = p - 1u;
    v4i vt, vf;
#pragma unroll
    for (int c = 0; c < 4; ++c) {
        const uint32_t odd = census & ~(pm1 >> (q - 1u - k)) & 1u;
        const uint32_t dist = (pm1 >> (q - k)) + 1u - odd;           // k < q <= 31: shifts of 1..31
        vt[c] = (int32_t)(r >= dist ? r - dist : r + (p - dist));
        const uint32_t f = r + dist;                                  // < 2^32: r, dist < 2^31
        vf[c] = (int32_t)(f >= p ? f - p : f);
        if (++k == q) { k = 0; ++r; }                                 // entries past the end are never stored
    }
    if (VEC && e0 + 4 <= total) {
        if (to) __builtin_nontemporal_store(vt, reinterpret_cast<v4i *>(to + e0));
        if (from) __builtin_nontemporal_store(vf, reinterpret_cast<v4i *>(from + e0));
    } else {
        for (int c = 0; c < 4 && e0 + c < total; ++c) {
            if (to) to[e0 + c] = vt[c];
            if (from) from[e0 + c] = vf[c];
        }
    }
}

}  // namespace

#endif  // BCS_KERNELS_ALLGATHER_H
