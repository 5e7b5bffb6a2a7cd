// Schedule construction kernels: the low-level table, receive rows (Alg. 4), send rows by look-up (Alg. 9,
// second loop) and by recomputation (Alg. 5), and the batch of unrelated (p, r, root) triples.
#ifndef BCS_KERNELS_SCHED_H
#define BCS_KERNELS_SCHED_H

#include "bcs_kernels_common.h"

namespace {

// ----------------------------------------------------------------------------------------------
// The low-level table of bcs_core.h lives in the code object; k_build_lowtab fills it once per device
// and process (one thread per entry, by the level walk).
// ----------------------------------------------------------------------------------------------
__device__ __align__(16) uint8_t g_lowtab[kLowTableBytes];   // read a dword at a time by stage_lowtab

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

// Rows of a workgroup's LDS tile of bytes (rank-major, Q bytes a rank, so the tile is the table's piece with one byte
// an entry) to their place in the rank-major int32 table: a lane reads four bytes, widens them and writes 16 bytes.
template <int Q>
__device__ __forceinline__ void byte_tile_to_rows(const int8_t *tile, uint32_t rows, int32_t *__restrict__ dst) {
    const uint32_t n = rows * Q;
    if ((reinterpret_cast<uintptr_t>(dst) & 15u) == 0) {
        const uint32_t n4 = n >> 2;
        for (uint32_t g = threadIdx.x; g < n4; g += kBlock) {
            const int32_t w = reinterpret_cast<const int32_t *>(tile)[g];
            const v4i pack = {(int32_t)(int8_t)w, (int32_t)(int8_t)(w >> 8), (int32_t)(int8_t)(w >> 16), w >> 24};
            __builtin_nontemporal_store(pack, reinterpret_cast<v4i *>(dst) + g);
        }
        const uint32_t e = (n4 << 2) + threadIdx.x;
        if (e < n) dst[e] = tile[e];
        return;
    }
    for (uint32_t e = threadIdx.x; e < n; e += kBlock) dst[e] = tile[e];
}

// ----------------------------------------------------------------------------------------------
// K1: receive rows of ranks [r0, r1), uniform p.  Lane = rank.  Rows are staged in LDS as bytes, laid out like
// the table, and leave widened to int32 in 16-byte pieces; optionally the entries are also kept slot-major
// (recvT[k][r - r0], one byte each) for the send look-up that follows, staged the same way and written as one
// aligned 256-byte piece a slot.  Bytes instead of int32 in LDS is what lets eight workgroups share a compute unit.
// ----------------------------------------------------------------------------------------------
// K0: the digit mask of every rank (one walk each), for launches over all ranks: every end point of every
// window of Alg. 4 is some rank, so K1 then reads its digit masks instead of walking (q+2 walks a row otherwise).
template <int Q>
__global__ __launch_bounds__(kBlock) void k_digits(const SkipTab tab, uint32_t *__restrict__ dtab) {
    __shared__ uint32_t lowtab[kLowShapeBytes / 4];
    Uniform<Q> pol;
#pragma unroll
    for (int k = 0; k <= Q; ++k) pol.S[k] = tab.s[k];
    pol.tab = &tab;
    pol.low = reinterpret_cast<const uint8_t *>(lowtab);
    const uint32_t p = pol.p();
    stage_lowtab(lowtab, low_shape(p, Q));
    __syncthreads();
    const uint64_t y = (uint64_t)blockIdx.x * kBlock + threadIdx.x;
    const uint32_t d = digits(pol, y < p ? (uint32_t)y : 0u);
    if (y < p) dtab[y] = d;
}

constexpr uint64_t kSlotTableCached = 128ull << 20;   // slot-major tables up to this size are written for the caches
template <int Q, bool BYTES, bool TAB = false>
__global__ __launch_bounds__(kBlock) void k_recv_uniform(const SkipTab tab, uint32_t root, uint32_t r0, uint32_t r1,
                                                         int32_t *__restrict__ recv_out,
                                                         slot_t *__restrict__ recvT, uint64_t ldT,
                                                         int8_t *__restrict__ rowsB,
                                                         const uint32_t *__restrict__ dtab) {
    constexpr int kRS = byte_row_stride(Q);
    __shared__ __align__(16) int8_t tile[kBlock * Q + 16];
    __shared__ __align__(16) int8_t tileB[BYTES ? kBlock * kRS : 16];   // only the variant that leaves byte rows pays for it
    // the tile's part of the slot-major table, slot by slot; the variant with byte rows (tables that the caches
    // hold) has no room for it beside them and stores the entries one by one
    __shared__ __align__(16) slot_t tileT[BYTES ? 16 : Q * kBlock];
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
    const uint32_t r = live ? (uint32_t)(r0 + idx) : root;
    const uint32_t v = r >= root ? r - root : r + p - root;
    int8_t *my = tile + threadIdx.x * Q;
    int8_t *myB = tileB + (BYTES ? threadIdx.x * kRS : 0);
    auto emit = [&](int i, int val) {
        my[i] = (int8_t)val;
        if constexpr (BYTES) {
            if (recvT) recvT[(uint64_t)i * ldT + idx] = (slot_t)val;
            myB[i] = (int8_t)(val - i);
        } else {
            if (recvT) tileT[i * kBlock + threadIdx.x] = (slot_t)val;
        }
    };
    if (live) {                                                  // lanes past the end sit the row out
        if constexpr (TAB) recv_row_tab(pol, dtab, v, emit);
        else recv_row(pol, v, Q - 1, emit);
    }
    if constexpr (BYTES) byte_row_finish<Q>(myB);
    __syncthreads();
    if (!BYTES && recvT) {
        // Each slot's kBlock bytes are one aligned piece of the table (its rows are padded to a multiple of
        // kBlock, so the last tile writes its idle lanes' bytes into the padding): 16 bytes a lane.
        static_assert(kBlock % 16 == 0, "16-byte pieces");
        // A table that the caches hold is left there for the look-up that follows; a larger one is streamed out.
        const bool stream_out = ldT * Q > kSlotTableCached;
        for (int g = threadIdx.x; g < Q * (kBlock / 16); g += kBlock) {
            const int k = g / (kBlock / 16), part = g % (kBlock / 16);
            const v4i piece = *reinterpret_cast<const v4i *>(tileT + k * kBlock + part * 16);
            v4i *dst = reinterpret_cast<v4i *>(recvT + (uint64_t)k * ldT + first + part * 16);
            if (stream_out) __builtin_nontemporal_store(piece, dst);
            else *dst = piece;
        }
    }
    if (!recv_out) return;
    const uint64_t rows = (count - first) < (uint64_t)kBlock ? (count - first) : (uint64_t)kBlock;
    byte_tile_to_rows<Q>(tile, (uint32_t)rows, recv_out + first * Q);
    if constexpr (BYTES) byte_rows_out<Q>(tileB, (uint32_t)rows, rowsB + first * kRS);
}

// K2: send rows from the slot-major receive table of ALL ranks (Alg. 9, second loop):
// send[r][k] = recv[(r + skips[k]) mod p][k].
// One wave (a workgroup of 64 lanes) takes G consecutive ranks.  Reading: a lane fetches the entries of FOUR
// consecutive ranks in one slot with one (unaligned) 4-byte load -- the table is slot-major bytes, so the four
// neighbours' entries are adjacent -- and the 64 lanes cover 64 / (G/4) slots at a time; all loads of a wave are in
// flight together.  Byte loads, one rank a lane, cost the address path of the memory pipeline four times as many
// instructions for the same bytes, and that path, not the HBM, was the limit (measured on MI355X at p = 2^27-1:
// 3.8 ms against 18.1 GB / 8 TB/s = 2.3 ms).  The words go to an LDS tile of bytes, slot-major with padded rows;
// then the wave writes its ranks' rows -- one contiguous piece of G q int32 -- as 16-byte streaming stores in
// address order, each lane gathering the four entries of its store from the tile.
// Measured at p = 2^27-1 (18.1 GB): 3.24 ms with G = 256, 3.38 ms with G = 128, 4.35 ms with G = 64 (4.3 KB of
// loads in flight per wave are too few); at p = 2^20+1: 0.0212, 0.0199, 0.0231 ms.  So many ranks take G = 256
// and fewer take G = 128 (more waves to spread over the device).  The reading side alone (no stores) takes
// 0.65 ms and the stores alone 2.6 ms (a wave streaming 27 KB: 5.5 TB/s; a store-only kernel whose workgroups
// write one aligned 4 KB piece each reaches 6.6-7.0 TB/s, but a workgroup that short cannot keep enough loads in
// flight: measured 4.4-5.4 ms in that shape); the whole kernel takes about their sum, reads and writes do not
// overlap in the memory system.
constexpr int kLookupLanes = 64;
constexpr int kLookupBigG = 256, kLookupSmallG = 128;
constexpr int kLookupBigMinQ = 22;                      // p > 2^21: a wave takes kLookupBigG ranks

template <int Q, int G>
__global__ __launch_bounds__(kLookupLanes) void k_send_lookup(const SkipTab tab, const slot_t *__restrict__ recvT,
                                                              uint64_t ldT, int32_t *__restrict__ send_out,
                                                              int8_t *__restrict__ rowsB) {
    static_assert(G % 4 == 0 && kLookupLanes % (G / 4) == 0 && G <= 4 * kLookupLanes, "a lane takes four ranks of one slot");
    constexpr int kQuads = G / 4;                                  // lanes that cover one slot of the group
    constexpr int kSlotsPerLoad = kLookupLanes / kQuads;
    constexpr int kLoads = (Q + kSlotsPerLoad - 1) / kSlotsPerLoad;
    constexpr int kRS = G + 4;                                     // bytes per slot row of the tile (padded: banks)
    constexpr int kStores = (G * Q + 4 * kLookupLanes - 1) / (4 * kLookupLanes);
    __shared__ __align__(16) int8_t tile[Q * kRS];
    const uint32_t p = tab.s[Q];
    const uint64_t first = (uint64_t)blockIdx.x * G;               // < p: the grid has ceil(p / G) workgroups
    const uint32_t lane = threadIdx.x;
    const uint32_t j4 = (lane % kQuads) * 4u;                      // this lane's four ranks within the group
    const uint32_t kk = lane / kQuads;
    uint32_t got[kLoads];
#pragma unroll
    for (int it = 0; it < kLoads; ++it) {
        const uint32_t k = it * kSlotsPerLoad + kk;
        const uint32_t kc = k < (uint32_t)Q ? k : (uint32_t)Q - 1u;    // lanes past the last slot repeat it; never stored
        const uint32_t sk = ((p - 1u) >> (Q - kc)) + 1u;           // skips[k]: the closed form of Alg. 1's halving
        const uint64_t r = first + j4;
        uint32_t word = 0;
        if (r < p) {
            uint32_t t = (uint32_t)r + sk;                         // below 2p < 2^32
            t = t >= p ? t - p : t;
            const slot_t *row = recvT + (uint64_t)kc * ldT;
            if (t + 3u < p) {
                __builtin_memcpy(&word, row + t, 4);
            } else {                                               // the ranks wrap inside these four (one lane per slot)
#pragma unroll
                for (int c = 0; c < 4; ++c) {
                    uint32_t tc = t + c;
                    tc = tc >= p ? tc - p : tc;
                    word |= (uint32_t)(uint8_t)row[tc] << (8 * c);
                }
            }
        }
        got[it] = word;
    }
#pragma unroll
    for (int it = 0; it < kLoads; ++it) {
        const uint32_t k = it * kSlotsPerLoad + kk;
        if (k < (uint32_t)Q) *reinterpret_cast<uint32_t *>(tile + k * kRS + j4) = got[it];
    }
    __syncthreads();
    const uint32_t rows = ((uint64_t)p - first) < (uint64_t)G ? (uint32_t)((uint64_t)p - first) : (uint32_t)G;
    const uint32_t n = rows * Q;                                   // entries of this group
    int32_t *dst = send_out + first * Q;
    const bool vec = (reinterpret_cast<uintptr_t>(dst) & 15u) == 0;
#pragma unroll
    for (int it = 0; it < kStores; ++it) {
        const uint32_t e = (uint32_t)it * 4u * kLookupLanes + lane * 4u;
        if (e < n) {
            uint32_t R = e / Q, k = e - R * Q;                     // divisions by a constant
            int32_t v[4];
#pragma unroll
            for (int c = 0; c < 4; ++c) {
                const uint32_t Rc = R < (uint32_t)G ? R : (uint32_t)G - 1u;   // past the group's end: read in bounds, not stored
                v[c] = tile[k * kRS + Rc];
                ++k;
                const bool wrap = k == (uint32_t)Q;
                k = wrap ? 0u : k;
                R += wrap ? 1u : 0u;
            }
            if (vec && e + 4u <= n) {
                const v4i pack = {v[0], v[1], v[2], v[3]};
                __builtin_nontemporal_store(pack, reinterpret_cast<v4i *>(dst + e));
            } else {
#pragma unroll
                for (int c = 0; c < 4; ++c)
                    if (e + c < n) dst[e + c] = v[c];
            }
        }
    }
    if (rowsB) {
        // the same rows as bytes for the expansion that follows: T[k] = entry[k] - k, the first three once more
        constexpr int kRSB = byte_row_stride(Q);
        constexpr uint32_t kW4 = kRSB / 4;
        uint32_t *out4 = reinterpret_cast<uint32_t *>(rowsB + first * kRSB);
        for (uint32_t w = lane; w < rows * kW4; w += kLookupLanes) {
            const uint32_t row = w / kW4, pos0 = 4u * (w - row * kW4);
            uint32_t packed = 0;
#pragma unroll
            for (int c = 0; c < 4; ++c) {
                const uint32_t pos = pos0 + c;
                const bool slot_ok = pos < (uint32_t)(Q + 3);
                const uint32_t slot = pos < (uint32_t)Q ? pos : (slot_ok ? pos - Q : 0u);
                const int32_t t = slot_ok && slot < (uint32_t)Q ? (int32_t)tile[slot * kRS + row] - (int32_t)slot : 0;
                packed |= ((uint32_t)t & 0xffu) << (8 * c);
            }
            out4[w] = packed;
        }
    }
}

// K1b: send rows of ranks [r0, r1) with no neighbour rows at hand (Alg. 5): entry i is entry i of the
// receive schedule of the to-neighbour, which costs that neighbour's rounds 0..i.
// Work lists for send entries left to Alg. 5 (k_send_recompute, k_batch).  Each lane working down its own entries
// makes a wave run as many turns as its unluckiest lane has entries, each turn as far as the largest k any lane asked
// for; so the entries named by the lanes' masks (bit k of lane L: entry (L, k)) are made one list of the workgroup,
// ranked by k and then by lane, and handed out one entry a lane: neighbouring places hold entries of the same k (and,
// in the batch kernel, whose lanes are in the order of q, of neighbouring q), and a wave's loops run about as far as
// each of its lanes needs.  Entry (L, k) goes to place
// kstart[k] + (entries for k in earlier waves) + (earlier lanes of L's wave with bit k), found with ballots.  The
// list is filled and handed out QUEUE entries at a time (QUEUE a multiple of BLOCK, the workgroup's lanes), one entry a lane: fn(has, who, k) runs in every lane of
// every wave that has an entry.  All lanes of the workgroup must call this (it synchronises them).
template <int BLOCK, int QUEUE, class Fn>
__device__ __forceinline__ void work_list(uint32_t mask, uint32_t (*wcnt)[32], uint32_t *kstart, uint16_t *queue, Fn fn) {
    static_assert(QUEUE % BLOCK == 0 && BLOCK % 64 == 0 && BLOCK <= 2048, "whole waves; a lane index and k share 16 bits");
    const int wave = threadIdx.x >> 6;
    // the k for which any lane of this wave has an entry (wave-uniform): the loops below visit only these
    uint32_t any_k = mask;
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) any_k |= (uint32_t)__shfl_xor((int)any_k, off, 64);
    any_k = __builtin_amdgcn_readfirstlane(any_k);
    __syncthreads();                                        // earlier users of wcnt / kstart / queue are done
    {
        uint32_t mine = 0;                                  // lane k of a wave: the wave's entries for k
        for (uint32_t m = any_k; m != 0u; m &= m - 1u) {
            const int k = __builtin_ctz(m);
            const uint32_t c = (uint32_t)__popcll(__ballot((mask >> k) & 1u));
            mine = (threadIdx.x & 63u) == (uint32_t)k ? c : mine;
        }
        if ((threadIdx.x & 63u) < 32u) wcnt[wave][threadIdx.x & 63u] = mine;
    }
    __syncthreads();
    if (threadIdx.x < 32) {                                 // entries for k = threadIdx.x: running count over the waves
        uint32_t acc = 0;
        for (int w = 0; w < BLOCK / 64; ++w) {
            const uint32_t c = wcnt[w][threadIdx.x];
            wcnt[w][threadIdx.x] = acc;
            acc += c;
        }
        kstart[threadIdx.x] = acc;
    }
    __syncthreads();
    if (threadIdx.x == 0) {
        uint32_t acc = 0;
        for (int k = 0; k < 32; ++k) {
            const uint32_t c = kstart[k];
            kstart[k] = acc;
            acc += c;
        }
        kstart[32] = acc;
    }
    __syncthreads();
    const uint32_t total = kstart[32];
    for (uint32_t base = 0; base < total; base += QUEUE) {
        for (uint32_t m = any_k; m != 0u; m &= m - 1u) {
            const int k = __builtin_ctz(m);
            const uint64_t bal = __ballot((mask >> k) & 1u);
            const uint32_t before = __builtin_amdgcn_mbcnt_hi((uint32_t)(bal >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)bal, 0u));
            const uint32_t place = kstart[k] + wcnt[wave][k] + before - base;
            if (((mask >> k) & 1u) && place < (uint32_t)QUEUE) queue[place] = (uint16_t)((threadIdx.x << 5) | (uint32_t)k);
        }
        __syncthreads();
        const uint32_t n = total - base < (uint32_t)QUEUE ? total - base : (uint32_t)QUEUE;
        for (uint32_t e0 = 0; e0 < n; e0 += BLOCK) {   // workgroup-uniform
            if (e0 + (threadIdx.x & ~63u) >= n) continue;    // a wave with no entry left (wave-uniform)
            const uint32_t e = e0 + threadIdx.x;
            const bool has = e < n;
            const uint32_t entry = has ? queue[e] : 0u;
            fn(has, entry >> 5, has ? (int)(entry & 31u) : -1);
        }
        __syncthreads();                                    // the next part of the list overwrites the queue
    }
}

constexpr int kRecomputeQueue = 4 * kBlock;                // entries of k_send_recompute's work list held at a time

template <int Q, bool TAB>
__global__ __launch_bounds__(kBlock) void k_send_recompute(const SkipTab tab, uint32_t root, uint32_t r0, uint32_t r1,
                                                           int32_t *__restrict__ send_out,
                                                           const uint32_t *__restrict__ dtab) {
    __shared__ __align__(16) int8_t tile[kBlock * Q + 16];   // one byte an entry, laid out like the table
    __shared__ uint32_t lowtab[kLowShapeBytes / 4];
    __shared__ uint32_t wcnt[kBlock / 64][32], kstart[33];    // the work list of the entries left to Alg. 5
    __shared__ uint16_t queue[kRecomputeQueue];
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
    int8_t *my = tile + threadIdx.x * Q;
    // the entries that need none of the to-neighbour's rounds (bcs_core.h); for consecutive ranks and large p
    // that is nearly all of them
    auto digits_of = [&](uint32_t y) -> uint32_t {
        if constexpr (TAB) return dtab[y];                // digit masks of all ranks from k_digits
        else return digits(pol, y);
    };
    uint32_t pending = send_row_direct(pol, v, digits_of(v), digits_of, [&](int k, int val) { my[k] = (int8_t)val; });
    pending = live ? pending : 0u;                            // lanes past the end replay the root and ask for nothing
    // Alg. 5 for the rest, as a work list of the workgroup: a lane takes one entry (of any rank of the tile), the
    // wave computes rounds 0..(its largest k) of each lane's to-neighbour and a lane keeps the entry of its own k
    work_list<kBlock, kRecomputeQueue>(pending, wcnt, kstart, queue, [&](bool has, uint32_t who, int kk) {
        int kmax = kk;
#pragma unroll
        for (int off = 32; off >= 1; off >>= 1) {
            const int other = __shfl_xor(kmax, off, 64);
            kmax = other > kmax ? other : kmax;
        }
        kmax = __builtin_amdgcn_readfirstlane(kmax);
        // the rank the entry belongs to: the tile's ranks are consecutive
        const uint64_t idx2 = first + (has ? who : threadIdx.x);
        const uint32_t r2 = idx2 < count ? (uint32_t)(r0 + idx2) : root;
        const uint32_t v2 = r2 >= root ? r2 - root : r2 + p - root;
        // skips[kk] by the closed form of Alg. 1's halving (kk differs from lane to lane)
        uint32_t t = v2 + (kk >= 0 ? ((p - 1u) >> (Q - kk)) + 1u : 0u);
        t = t >= p ? t - p : t;
        int32_t got = 0;
        auto own_entry = [&](int j, int val) { got = (j == kk) ? val : got; };
        if constexpr (TAB) recv_row_tab_upto(pol, dtab, t, dtab[t], kmax, own_entry);
        else recv_row(pol, t, kmax, own_entry);
        if (has) tile[who * Q + kk] = (int8_t)got;
    });
    __syncthreads();
    const uint64_t rows = (count - first) < (uint64_t)kBlock ? (count - first) : (uint64_t)kBlock;
    byte_tile_to_rows<Q>(tile, (uint32_t)rows, send_out + first * Q);
}

// K3: unrelated (p, r, root) triples; rows of BCS_BATCH_STRIDE ints (one 128-byte line each), padded.
// A workgroup takes kBatchBlock triples and first orders them by q in LDS (counting sort), because a
// wave runs its level loops to the largest q among its lanes and the work grows like q^3: after the
// sort a wave holds neighbouring q only.  Each lane then builds the rows of its triple into an LDS tile of
// bytes (entries lie in [-31, 30]; a byte of -128 stands for the padding), at the triple's place in the
// input order; the workgroup then writes the tile out as whole 128-byte lines, eight lanes a row and 16 bytes
// a lane.  (Storing each entry straight into its row, 4 bytes at a time into a line of the lane's own, made the
// memory system write five times the table's bytes as partial lines, and a call for receive rows alone was
// bound by those stores: measured 0.254 ms with the vector ALU busy 28 % of the time.)
constexpr int kBatchBlock = 1024;
constexpr int kBatchRowBytes = BCS_BATCH_STRIDE + 4;       // LDS row stride: nine words, so lanes' rows spread over the banks
constexpr int8_t kBatchPadByte = -128;
constexpr int kQueue = 4 * kBatchBlock;                    // entries of the Alg. 5 work list held at a time

// the workgroup's byte tile -> rows of the table (after a barrier); `rows` = triples of this workgroup that exist
__device__ __forceinline__ void batch_rows_out(const int8_t *tileB, uint32_t rows, int32_t *__restrict__ dst) {
    const bool vec = (reinterpret_cast<uintptr_t>(dst) & 15u) == 0;
#pragma unroll
    for (int it = 0; it < BCS_BATCH_STRIDE / 4; ++it) {
        const uint32_t g = (uint32_t)it * kBatchBlock + threadIdx.x;
        const uint32_t row = g >> 3, part = g & 7u;
        if (row >= rows) continue;
        const uint32_t four = *reinterpret_cast<const uint32_t *>(tileB + row * kBatchRowBytes + part * 4u);
        int32_t v[4];
#pragma unroll
        for (int c = 0; c < 4; ++c) {
            const int32_t b = (int32_t)(int8_t)(four >> (8 * c));
            v[c] = b == (int32_t)kBatchPadByte ? BCS_BATCH_PAD : b;
        }
        int32_t *out = dst + (uint64_t)row * BCS_BATCH_STRIDE + part * 4u;
        if (vec) {
            const v4i pack = {v[0], v[1], v[2], v[3]};
            *reinterpret_cast<v4i *>(out) = pack;
        } else {
#pragma unroll
            for (int c = 0; c < 4; ++c) out[c] = v[c];
        }
    }
}

// One entry of a work list of the batch kernel, as the lane that works on it sees it: the triple `who` of the
// workgroup (its p and rank from the sorted arrays), the entry's k, the to-neighbour t = (v + skips[k]) mod p, and
// a policy whose level loops run as far as the wave's largest q; kmax is the wave's largest k.  Lanes without an
// entry (has = false, kk = -1) stand in with p = 1.
struct BatchLane {
    PerLane pol;
    uint32_t t, orig;
    int kmax;
};
__device__ __forceinline__ BatchLane batch_lane(bool has, uint32_t who, int kk, const uint32_t *s_p, const uint32_t *s_v,
                                                const uint32_t *s_slot) {
    BatchLane e;
    const uint32_t p = has ? s_p[who] : 1u, v = has ? s_v[who] : 0u;
    e.orig = s_slot[who] & 0xffffu;
    const int q = ceil_log2(p);
    int kmax = kk, qtop = q;
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) {
        const int ok = __shfl_xor(kmax, off, 64), oq = __shfl_xor(qtop, off, 64);
        kmax = ok > kmax ? ok : kmax;
        qtop = oq > qtop ? oq : qtop;
    }
    e.kmax = __builtin_amdgcn_readfirstlane(kmax);
    e.pol.pm1 = p - 1u;
    e.pol.ql = q;
    e.pol.wave_top = __builtin_amdgcn_readfirstlane(qtop) - 1;
    e.pol.odd = odd_levels(p, q);
    e.pol.low = g_lowtab + (size_t)low_shape(p, q) * kLowShapeBytes;
    const uint32_t t = v + (kk >= 0 ? e.pol.s(kk) : 0u);
    e.t = t >= p ? t - p : t;
    return e;
}

__global__ __launch_bounds__(kBatchBlock) void k_batch(int64_t count, const int32_t *__restrict__ pv,
                                                       const int32_t *__restrict__ rv,
                                                       const int32_t *__restrict__ rootv,
                                                       int32_t *__restrict__ recv_out, int32_t *__restrict__ send_out,
                                                       int32_t *__restrict__ q_out) {
    __shared__ uint32_t bins[33];                 // bins[q] for valid triples, bins[32] for the rest
    __shared__ uint32_t start[33];
    __shared__ uint32_t s_p[kBatchBlock], s_v[kBatchBlock], s_slot[kBatchBlock];
    __shared__ __align__(16) int8_t tileB[kBatchBlock * kBatchRowBytes];
    __shared__ uint32_t wcnt[kBatchBlock / 64][32];            // send entries left to Alg. 5: per wave and k, then their offsets
    __shared__ uint32_t kstart[33];
    __shared__ uint16_t queue[kQueue];                         // the work list: (lane << 5) | k
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
    const uint32_t orig = slot & 0xffffu;                     // the triple's place among the workgroup's 1024
    const int64_t idx = first + orig;
    const int q = ceil_log2(p);
    if (live && q_out) q_out[idx] = valid ? q : -1;
    // largest q in this wave bounds the level loops of all its lanes
    int qmax = q;
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) {
        const int other = __shfl_xor(qmax, off, 64);
        qmax = other > qmax ? other : qmax;
    }
    qmax = __builtin_amdgcn_readfirstlane(qmax);   // the same in every lane: a scalar, so the loops it bounds are scalar loops
    PerLane pol;
    pol.pm1 = p - 1u;
    pol.ql = q;
    pol.wave_top = qmax - 1;
    pol.odd = odd_levels(p, q);
    pol.low = g_lowtab + (size_t)low_shape(p, q) * kLowShapeBytes;
    const uint32_t rows = (count - first) < (int64_t)kBatchBlock ? (uint32_t)(count - first) : (uint32_t)kBatchBlock;
    int8_t *my = tileB + orig * kBatchRowBytes;
    uint32_t *my4 = reinterpret_cast<uint32_t *>(my);
    const uint32_t pad4 = 0x80808080u;
    if (recv_out) {
#pragma unroll
        for (int w = 0; w < BCS_BATCH_STRIDE / 4; ++w) my4[w] = pad4;
        recv_row(pol, v, qmax - 1, [&](int i, int val) { my[i] = (int8_t)val; });
        __syncthreads();
        batch_rows_out(tileB, rows, recv_out + first * BCS_BATCH_STRIDE);
        __syncthreads();
    }
    if (send_out) {
#pragma unroll
        for (int w = 0; w < BCS_BATCH_STRIDE / 4; ++w) my4[w] = pad4;
        // the entries that need none of the to-neighbour's rounds (send_row_direct); the others are left in `pending`
        const uint32_t pending = send_row_direct(pol, v, digits(pol, v), [&](uint32_t y) { return digits(pol, y); },
                                                 [&](int k, int val) { my[k] = (int8_t)val; });
        // Those are worked off as one list of the whole workgroup, one entry a lane.  (Each lane working down its
        // own entries made a wave run as many turns as its unluckiest lane has entries, each turn as far as the
        // largest k any lane asked for: five times the lane-operations the entries themselves need, by a count on
        // the C5 triples, where a triple leaves 1.8 entries on average, nearly all below level 8.)
        // Alg. 5 for the rest: rounds 0..k of the to-neighbour's receive row, of which entry k is kept (a wave
        // computes as many rounds as its largest k; receive rows are prefix-stable, the extra rounds change nothing)
        work_list<kBatchBlock, kQueue>(pending, wcnt, kstart, queue, [&](bool has, uint32_t who, int kk) {
            const BatchLane e = batch_lane(has, who, kk, s_p, s_v, s_slot);
            int32_t keep = 0;
            recv_row(e.pol, e.t, e.kmax, [&](int j, int val) { keep = (j == kk) ? val : keep; });
            if (has) tileB[e.orig * kBatchRowBytes + kk] = (int8_t)keep;
        });
        __syncthreads();
        batch_rows_out(tileB, rows, send_out + first * BCS_BATCH_STRIDE);
    }
}

}  // namespace

#endif  // BCS_KERNELS_SCHED_H
