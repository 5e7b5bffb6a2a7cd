// Expansion kernels (the index arithmetic of Alg. 6): block tables from int32 schedule rows, from byte rows,
// and fused with the construction of the rows for short rows.
#ifndef BCS_KERNELS_EXPAND_H
#define BCS_KERNELS_EXPAND_H

#include "bcs_kernels_common.h"
#include "bcs_kernels_sched.h"

namespace {

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

}  // namespace

#endif  // BCS_KERNELS_EXPAND_H
