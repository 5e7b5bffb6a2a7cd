// bcs_core.h: the per-rank schedule construction, written once for the GPU lanes and for a host
// build that the CPU tests use to check this same code against the oracle.
//
// Method: J. L. Traff, arXiv 2205.10072, Section 2 (Alg. 1, 2, 4).  Block sets are 32-bit masks.
//
// Two routines answer "which baseblocks do the ranks a..b hold" (what the paper's Alg. 3 is for).
// Both are this library's own and rest on the self-similarity stated after Alg. 2: rank skips[k] has
// baseblock k, and ranks skips[k]+1 .. skips[k+1]-1 repeat the baseblocks of ranks
// 1 .. skips[k+1]-skips[k]-1.
//
// (1) The level walk (range_blocks), exact for any range, 25 vector ops a level.  For k = q-1 .. 0:
//   b <  skips[k]            nothing at this level;
//   a >  skips[k] (<= b)     the range lies in the upper copy: move it down by skips[k];
//   a <= skips[k] <= b       block k is in; so are the blocks of ranks 1 .. b-skips[k], which are
//                            exactly 0 .. (largest level whose skip is <= b-skips[k]); what is left
//                            is [a, skips[k]-1], handled by the remaining levels.
// It builds the small table below and serves as the reference in the host tests.
//
// (2) The digit form (digits + window_blocks), which Alg. 4 runs on.  Write a rank as the greedy sum
// of skips, largest first (the walk of Alg. 2); its digit mask D(y) has bit k set when skips[k] was
// taken, and the baseblock is the lowest set bit.  D is order preserving, so for a window (y1, y2]:
//   - the first level k (from the top) where D(y1) and D(y2) differ holds a rank with baseblock k,
//     the largest block of the window;
//   - the ranks above that node are a prefix of the level-k pattern: blocks 0 .. (highest digit of
//     D(y2) below k);
//   - the ranks below it are a tail of the pattern: blocks 0 .. l1 with l1 the highest clear digit of
//     D(y1) below k -- provided l1 >= 7.  Each copy of the pattern in the upper half of its parent
//     lacks its last rank when the parent skip is odd, and below level 7 these missing ranks can be
//     the only holders of a block; there the answer is read from a table indexed by the number of
//     odd levels passed and the seven low digits.  The table depends on skips[7] only (64 shapes;
//     another 64 for p <= 64) and is filled by the level walk.
// The windows of Alg. 4 share their end points (round i ends where round i+1 begins), so a row costs
// q+1 digit masks (3 vector ops a level down to level 7; the seven low digits of what is left are one
// more row of the table) and a few bit operations per round.
// All of it is branch-free apart from the wave-uniform test for Alg. 4's rare second range.
//
// (3) Rounds without a window (round_from_digits, one p per launch).  From level 6 up most rounds of most ranks
// follow from D(v) alone: the home round gives the baseblock, a round whose digit is set gives the next digit
// above, a round whose digit is clear gives the round's own index when the value of the lower digits keeps clear
// of the ends of its range.  The 64 consecutive ranks of a wave share their high digits, so whole waves skip the
// window in about three of four rounds; a wave with a lane the rule leaves out computes the window as in (2) and
// every lane keeps whichever result applies to it.
#ifndef BCS_CORE_H
#define BCS_CORE_H

#include <stddef.h>
#include <stdint.h>

#if defined(__HIP_DEVICE_COMPILE__)
#define BCS_HD __host__ __device__ __forceinline__
#define BCS_WAVE_ANY(x) __any(x)
#define BCS_CLZ(x) __clz((int)(x))
#elif defined(__HIPCC__)
#define BCS_HD __host__ __device__ __forceinline__
#define BCS_WAVE_ANY(x) (x)
#define BCS_CLZ(x) ((x) ? __builtin_clz(x) : 32)
#else
#define BCS_HD inline
#define BCS_WAVE_ANY(x) (x)
#define BCS_CLZ(x) ((x) ? __builtin_clz(x) : 32)
#endif

namespace bcs {

constexpr int kMaxQ = 31;

// Low-level table: kLowShapes shapes x kLowRows rows x 128 digit patterns, one byte (a 7-bit block
// mask) each.  Shape: skips[7] - 65 when q >= 7, else 63 + p.  Row d < 25: tail of the level-7 pattern
// cut short by d ranks; row 25 + k: tail of the level-k pattern, k <= 7; last row: the greedy digits of
// the ranks below skips[7] (what the walk of Alg. 2 finds on its last seven levels).
constexpr int kLowLevels = 7;
constexpr int kLowShapes = 128;
constexpr int kLowDigitRow = 25 + kLowLevels + 1;   // row of the low digits themselves: entry y = digits of rank y < skips[7]
constexpr int kLowRows = kLowDigitRow + 1;
constexpr int kLowShapeBytes = kLowRows * 128;
constexpr int kLowTableBytes = kLowShapes * kLowShapeBytes;

BCS_HD int ceil_log2(uint32_t p) { return p > 1u ? 32 - BCS_CLZ(p - 1u) : 0; }
BCS_HD int low_shape(uint32_t p, int q) { return q >= kLowLevels ? (int)(((p - 1u) >> (q - kLowLevels)) + 1u) - 65 : 63 + (int)p; }
// bit k set when skips[k+1] is odd, i.e. 2*skips[k] - skips[k+1] = 1: bit q-1-k of p-1 is clear
BCS_HD uint32_t odd_levels(uint32_t p, int q) {
#if defined(__HIP_DEVICE_COMPILE__)
    return q ? __brev(~(p - 1u) & (0xffffffffu >> (32 - q))) >> (32 - q) : 0u;
#else
    uint32_t m = 0;
    for (int k = 0; k < q; ++k) m |= ((~(p - 1u) >> (q - 1 - k)) & 1u) << k;
    return m;
#endif
}

struct SkipTab {
    uint32_t s[kMaxQ + 2];               // s[0..q]; entries above q repeat p
    uint32_t odd;                        // odd_levels(p, q)
};

// ----------------------------------------------------------------------------------------------
// Skip policies.  Uniform<Q>: one p for the whole launch, Q known at compile time, level loops
// fully unrolled, skips in SGPRs.  PerLane: every lane has its own p and q; skips come from the
// closed form skips[k] = ceil(p / 2^(q-k)) = ((p-1) >> (q-k)) + 1 that Alg. 1's halving produces.
// ----------------------------------------------------------------------------------------------
template <int Q>
struct Uniform {
    static constexpr bool kScalarSkips = true;   // skips are wave-uniform (SGPR operands)
    uint32_t S[Q + 1];
    const SkipTab *tab;                  // same values, for wave-uniform dynamic indices
    const uint8_t *low;                  // this p's shape of the low-level table
    BCS_HD uint32_t odd_mask() const { return tab->odd; }
    BCS_HD const uint8_t *lowtab() const { return low; }
    BCS_HD int q() const { return Q; }
    BCS_HD int top() const { return Q - 1; }
    static constexpr int kTopLevel = Q - 1;
    BCS_HD uint32_t p() const { return S[Q]; }
    BCS_HD uint32_t s(int k) const { return S[k]; }          // k constant after unrolling
    BCS_HD uint32_t sdyn(int k) const { return tab->s[k]; }  // k wave-uniform
    // skips[h+1] - 1 for a per-lane h in [-1, Q-1]
    BCS_HD uint32_t skip_above_minus1(int h) const { return (S[Q] - 1u) >> (Q - 1 - h); }
};

struct PerLane {
    static constexpr bool kScalarSkips = false;
    uint32_t pm1;                        // p - 1
    int ql;                              // this lane's q
    int wave_top;                        // largest q in the wave, minus 1 (uniform loop bound)
    uint32_t odd;                        // odd_levels(p, q)
    const uint8_t *low;                  // this lane's shape of the low-level table
    BCS_HD uint32_t odd_mask() const { return odd; }
    BCS_HD const uint8_t *lowtab() const { return low; }
    BCS_HD int q() const { return ql; }
    BCS_HD int top() const { return wave_top; }
    BCS_HD uint32_t p() const { return pm1 + 1u; }
    // levels above this lane's q get a skip no rank reaches, which makes them inert
    BCS_HD uint32_t s(int k) const {
        int sh = ql - k;
        return sh >= 0 ? (pm1 >> sh) + 1u : 0xffffffffu;
    }
    BCS_HD uint32_t sdyn(int k) const { return s(k); }
    BCS_HD uint32_t skip_above_minus1(int h) const { return pm1 >> (ql - 1 - h); }
};

// Blocks of ranks 1..y: {0..k'} with k' the largest level whose skip is <= y (empty for y = 0).
// skips[k] lies in (2^(k-1), 2^k], so k' is floor(log2 y) or one more.
template <class Pol>
BCS_HD uint32_t prefix_blocks(const Pol &pol, uint32_t y) {
    int h = 31 - BCS_CLZ(y | 1u);
    int kk = h + (pol.skip_above_minus1(h) < y ? 1 : 0);
    uint32_t m = (2u << kk) - 1u;
    return y ? m : 0u;
}

// Baseblocks of ranks a..b as a mask, 1 <= a, b < p; empty (0) when a > b.
template <class Pol>
BCS_HD uint32_t range_blocks(const Pol &pol, uint32_t a, uint32_t b) {
    uint32_t m = 0;
#pragma unroll
    for (int k = pol.top(); k >= 0; --k) {
        const uint32_t s = pol.s(k);
        const bool reach = b >= s;
        const bool above = a > s;
        const bool shift = reach && above;
        const bool hit = reach && !above;
        const uint32_t y = b - s;
        const uint32_t add = (1u << k) | prefix_blocks(pol, hit ? y : 0u);
        m |= hit ? add : 0u;
        a = shift ? a - s : a;
        b = shift ? y : (hit ? s - 1u : b);
    }
    return m;
}

// One entry of the low-level table, by the level walk on the small system p' that the shape names.
BCS_HD uint32_t low_table_entry(int shape, int row, int low) {
    const uint32_t pp = shape < 64 ? (uint32_t)shape + 65u : (uint32_t)shape - 63u;
    const int qq = ceil_log2(pp);
    PerLane pol;
    pol.pm1 = pp - 1u;
    pol.ql = qq;
    pol.wave_top = kLowLevels - 1;
    pol.odd = 0;
    pol.low = nullptr;
    int k;
    uint32_t cut;
    if (row == kLowDigitRow) {
        uint32_t y = (uint32_t)low, d = 0;
        if (y >= pp) return 0u;
        for (int j = qq - 1; j >= 0; --j) {
            const uint32_t sj = pol.s(j);
            if (y >= sj) {
                y -= sj;
                d |= 1u << j;
            }
        }
        return d;
    }
    if (row < 25) {
        if (qq < kLowLevels) return 0u;
        k = kLowLevels;
        cut = (uint32_t)row;
    } else {
        k = row - 25;
        cut = 0u;
        if (k > qq) return 0u;
    }
    uint32_t a = 1u;                                     // first rank after the one the digits name
    for (int j = 0; j < k; ++j)
        if ((low >> j) & 1) a += pol.s(j);
    const uint32_t top = pol.s(k);                       // k = qq gives p'
    if (top < 2u + cut) return 0u;
    const uint32_t b = top - 1u - cut;
    return a <= b ? range_blocks(pol, a, b) : 0u;
}

// Alg. 2's walk, keeping which skips were taken: bit k of the result is set when skips[k] is part of
// the greedy sum of y (0 <= y < p).  The lowest set bit is the baseblock, the highest the home level.
template <class Pol>
BCS_HD uint32_t digits(const Pol &pol, uint32_t y) {
#if defined(__HIP_DEVICE_COMPILE__)
    // three vector ops a level: subtract with borrow-out, keep the old value on borrow, shift the borrow
    // into the (inverted) digit mask.  gfx950 wants two wait states between a vector op that writes
    // vcc and one that reads it, hence the s_nop.
    uint32_t inv = 0;
    if constexpr (Pol::kScalarSkips) {
        // levels 7 and up by the walk; what is left is a rank below skips[7] <= 128, whose digits are read
        // from the table's last row
        constexpr int kHigh = Pol::kTopLevel + 1 > kLowLevels ? Pol::kTopLevel + 1 - kLowLevels : 0;
#pragma unroll
        for (int k = pol.top(); k >= kLowLevels; --k) {
            uint32_t t;
            asm("v_subrev_co_u32 %0, vcc, %3, %1\n\t"
                "s_nop 1\n\t"
                "v_cndmask_b32 %1, %0, %1, vcc\n\t"
                "v_addc_co_u32 %2, vcc, %2, %2, vcc"
                : "=&v"(t), "+v"(y), "+v"(inv)
                : "s"(pol.s(k))
                : "vcc");
        }
        const uint32_t lowd = pol.lowtab()[kLowDigitRow * 128 + (int)y];
        const uint32_t highd = kHigh > 0 ? (~inv & (0xffffffffu >> (32 - (kHigh > 0 ? kHigh : 1)))) : 0u;
        return (highd << kLowLevels) | lowd;
    } else {
        // Per-lane p: the lane's own levels come first, whatever the wave's bound.  Step m handles level
        // q-1-m, whose skip is ((p-1) >> (m+1)) + 1 (Alg. 1's halving), so g = skip - 1 is one shift a
        // step and "y - g - 1 with borrow-out" (borrow-in forced to one) subtracts the skip: four vector
        // ops a level.  Steps past level 0 find y = 0 below a skip of 1 and change nothing; the digits
        // are moved down to their places at the end.
        // The walk stops seven levels short of the wave's bound: what is left of y is then below the lane's
        // skips[7] (or is 0, for a lane with fewer levels than steps), and its digits come from the table.
        const int steps = pol.top() + 1 > kLowLevels ? pol.top() + 1 - kLowLevels : 0;
        const uint64_t ones = ~0ull;
        uint32_t g = pol.pm1;
#pragma unroll 1
        for (int m = 0; m < steps; ++m) {
            uint32_t t;
            asm("v_lshrrev_b32 %3, 1, %3\n\t"
                "v_subb_co_u32_e64 %0, vcc, %1, %3, %4\n\t"
                "s_nop 1\n\t"
                "v_cndmask_b32 %1, %0, %1, vcc\n\t"
                "v_addc_co_u32 %2, vcc, %2, %2, vcc"
                : "=&v"(t), "+v"(y), "+v"(inv), "+v"(g)
                : "s"(ones)
                : "vcc");
        }
        const uint32_t walked = steps > 0 ? (~inv & (0xffffffffu >> (32 - steps))) : 0u;
        const int left = pol.ql - steps;                   // levels the walk did not reach (at most seven)
        // A lane whose own q is below the round the wave is in gets an inert skip and with it a y that is no
        // rank at all: its result is never used, but its table index must stay inside the row.
        const uint32_t lowd = pol.lowtab()[kLowDigitRow * 128 + (int)(y & 127u)];
        return (left >= 0 ? walked << left : walked >> -left) | lowd;
    }
    const int levels = pol.top() + 1;
    return levels > 0 ? (~inv & (0xffffffffu >> (32 - levels))) : 0u;
#else
    // host build: the same split as on the GPU, levels 7 and up by the walk and the rest from the table's digit
    // row, so that the host tests check that row too
    uint32_t d = 0;
    const bool by_table = pol.lowtab() != nullptr;
    for (int k = pol.top(); k >= (by_table ? kLowLevels : 0); --k) {
        const uint32_t s = pol.s(k);
        const bool take = y >= s;
        y = take ? y - s : y;
        d = (d << 1) | (take ? 1u : 0u);
    }
    if (by_table) d = (d << kLowLevels) | pol.lowtab()[kLowDigitRow * 128 + (int)(y & 127u)];
    return d;
#endif
}

// Baseblocks of the ranks after the one with digits d_lo up to the one with digits d_hi (d_lo < d_hi
// as integers; both may carry one more digit above level q-1 that counts laps around the ring, in
// which case the result has that bit set for rank 0 and the caller drops it).  0 when d_lo == d_hi.
template <class Pol>
BCS_HD uint32_t window_blocks(const Pol &pol, uint32_t d_lo, uint32_t d_hi) {
    const uint32_t diff = d_lo ^ d_hi;
    const int k = 31 - BCS_CLZ(diff);
    const uint32_t node = 1u << (k & 31);
    const uint32_t below = node - 1u;
    const uint32_t up = d_hi & below;                          // ranks above the node: a prefix
    const uint32_t pre = up ? (0xffffffffu >> BCS_CLZ(up)) : 0u;
    const uint32_t low = d_lo & below;                         // ranks below it: a tail
    const uint32_t clear = ~low & below;
    const uint32_t tail = clear ? (0xffffffffu >> BCS_CLZ(clear)) : 0u;
    const uint32_t run = below & ~127u;                        // levels 7..k-1
    const int passed = __builtin_popcount(pol.odd_mask() & run);
    const int row = k > kLowLevels ? passed : 25 + k;
    // the table serves tails whose highest clear digit lies below level 7; where the table sits in global memory
    // (every lane its own shape) the read is skipped when no lane of the wave has such a tail
    uint32_t small = 0;
    if (Pol::kScalarSkips || BCS_WAVE_ANY((clear >> kLowLevels) == 0u)) small = pol.lowtab()[row * 128 + (int)(low & 127u)];
    const uint32_t suf = (clear >> kLowLevels) ? tail : small;
    return diff ? (node | pre | suf) : 0u;
}

// Alg. 4: entries 0..last of the receive schedule of virtual rank v; emit(i, value) per entry.
// The rank's own baseblock starts the set B of blocks it already has.  Round i looks for the largest
// new block among ranks v-skips[i+1]+1 .. v-skips[i]; if there is none, among ranks
// v-sum_{j<=i}skips[j] .. v-skips[i+1], which are the last c ranks before the first range, c being the
// number of odd levels up to i (because skips[i+1] = 1 + sum_{j<=i}(skips[j] - odd_j)).  Ranks are
// mod p and rank 0 owns no baseblock.  The i = 0 and i = q-1 special cases printed in Alg. 4 are
// instances of this rule.  End points are kept as v + p - skips[i] in [0, 2p): digits of the rank plus
// a lap digit at level q, so that every window is an increasing pair.
// One round of Alg. 4 on the digit masks of the window's end points: d_hi for v - skips[i], d_lo for
// v - skips[i+1] (each with the lap digit when the subtraction did not wrap).  B is the set of blocks the rank
// has, c the number of odd levels up to i; digits_of(y) gives the digit mask of a rank y < p.
template <class Pol, class DigitsOf>
BCS_HD int recv_round_value(const Pol &pol, uint32_t v, int i, uint32_t s_n, uint32_t d_lo, uint32_t d_hi, int home,
                            int own, uint32_t B, DigitsOf digits_of, int &blk_out) {
    const uint32_t p = pol.p();
    const int q = pol.q();
    const uint32_t lap = 1u << (q & 31);
    const bool active = i < q;                            // per-lane q may be below the wave's bound
    const bool is_home = (i == home);
    uint32_t U = window_blocks(pol, d_lo, d_hi) & ~lap & ~B;
    const bool need2 = active && !is_home && U == 0u;
    if (BCS_WAVE_ANY(need2)) {
        // the c ranks that end where the first range begins (c = the number of odd levels up to i); one more lap
        // if that runs below 0
        const uint32_t c = (uint32_t)__builtin_popcount(pol.odd_mask() & ((2u << (i & 31)) - 1u));
        const uint32_t Y = v + p - s_n;
        const bool under = Y < c;
        const uint32_t Z = under ? Y + p - c : Y - c;
        const uint32_t hi2 = under ? (d_lo | lap) : d_lo;
        const bool zlap = Z >= p;
        const uint32_t lo2 = digits_of(zlap ? Z - p : Z) | (zlap ? lap : 0u);
        const uint32_t U2 = window_blocks(pol, lo2, hi2) & ~lap & ~B;
        U = need2 ? U2 : U;
    }
    const int blk = 31 - BCS_CLZ(U);                      // largest candidate
    blk_out = is_home ? q : blk;                          // the home round adds nothing to B: the lap digit's bit
    return is_home ? own : blk - q;
}

// The same round for callers that keep B themselves: the new block joins B, the entry goes to emit.
template <class Pol, class DigitsOf, class Emit>
BCS_HD void recv_round(const Pol &pol, uint32_t v, int i, uint32_t s_n, uint32_t d_lo, uint32_t d_hi, int home,
                       int own, uint32_t &B, DigitsOf digits_of, Emit emit) {
    const int q = pol.q();
    int blk;
    const int val = recv_round_value(pol, v, i, s_n, d_lo, d_hi, home, own, B, digits_of, blk);
    const bool active = i < q;
    // one emit for both kinds of round, so that a wave with lanes of both kinds does not run it twice
    B |= active ? (1u << (blk & 31)) : 0u;
    if (active) emit(i, val);
}

// Rounds that need no window (one p per launch).  With D(v) the digit mask of the rank, low the value of its
// digits below i and c the number of odd levels below i, round i's entry is
//   - the rank's baseblock when i is its highest digit (Alg. 4's first branch);
//   - (next digit j of v above i) - q when digit i is set and low >= c.  The rank w = v - skips[i] - low has the
//     digits of v above i and nothing below (taking digits out of a greedy sum leaves a greedy sum), so its
//     baseblock is j; low < skips[i+1] - skips[i] puts it into the round's first window, whose other end has digit
//     j clear, so j is the window's largest block; and v cannot have come by block j before: its own baseblock
//     is at or below i, the earlier rounds' windows lie above v - skips[i] except for round i-1's second range,
//     which reaches fewer than c ranks below it (and w lies low ranks below), and the next rank with baseblock j
//     is more than 2 skips[i] above w;
//   - i - q when digit i is clear and low keeps clear of the ends of its range: taking skips[i] from v borrows
//     from the next digit j above (the lap digit when there is none), which sets digits i..j-1 and lowers the low
//     part by the number o of odd levels in [i, j) (skips[j] - skips[i] = sum of skips[i..j-1] minus o).  With
//     low' = low - o >= 0: the rank w = v - skips[i] - low' has lowest digit i and lies in the first window when
//     low' < skips[i+1] - skips[i]; every other rank of the window shares the digits above i and has a lower
//     lowest digit; and block i is new: v's baseblock is not i, the earlier rounds reach down to
//     v - skips[i] - c + 1 only, which misses w when low' >= c, and the next rank with lowest digit i lies
//     skips[i+1] - (odd levels in [i+1, j)) above w, past v.  The test allows for every o from 0 to the number of
//     odd levels from i up and keeps twice the margin this needs (it is case (b) of send_row_direct below).
// Both are also checked against the oracle (every rank of every p the CPU tests run this code on, the full-size
// configurations on the GPU) and, on the GPU, against rows taken from windows throughout (the batch kernel) for
// every rank of every p up to 2^22 and for slices of tens of thousands of larger p.  Low rounds rarely agree
// across the 64 ranks of a wave, so the test starts at round kDigitRoundsFrom.
constexpr int kDigitRoundsFrom = 6;
constexpr int kTabAhead = 10;                           // recv_row_tab reads the end points of rounds below this ahead

// dl = D(v) with the lap digit (so that there always is a digit above round i); returns whether the entry could
// be taken from the digits and leaves it in val, its block (the lap digit's index q for the home round, which
// Alg. 4's set B never holds) in blk.  Written with masks instead of conditions: one straight run of vector ops.
template <class Pol>
BCS_HD bool round_from_digits(const Pol &pol, uint32_t dl, int i, uint32_t s_i, uint32_t low, int home, int own,
                              int &val, int &blk) {
    const int q = pol.q();
    const uint32_t odd = pol.odd_mask();
    const int mrg = 2 * __builtin_popcount(odd & ((2u << (i & 31)) - 1u)) + 2;
    const int c1 = mrg + __builtin_popcount(odd >> (i & 31));          // low must exceed this ...
    const int c2 = (int)s_i - mrg - 1;                                  // ... and stay below this
    const uint32_t width = c2 > c1 + 1 ? (uint32_t)(c2 - c1 - 1) : 0u;
    const uint32_t m = 0u - ((dl >> (i & 31)) & 1u);                    // all ones when digit i is set
    const uint32_t above = (dl >> (i & 31)) >> 1;                       // never 0: the lap digit
    const uint32_t next = (uint32_t)(__builtin_ctz(above) + i + 1);
    blk = (int)((m & next) | (~m & (uint32_t)i));
    val = i == home ? own : blk - q;
    const uint32_t x = (low - (uint32_t)c1 - 1u) & ~m;
    const uint32_t cbelow = (uint32_t)__builtin_popcount(odd & ((1u << (i & 31)) - 1u));   // odd levels below i
    return (m != 0u && low >= cbelow) || x < width;
}

template <class Pol, class Emit>
BCS_HD void recv_row_from(const Pol &pol, uint32_t v, uint32_t dv, int last, Emit emit);

template <class Pol, class Emit>
BCS_HD void recv_row(const Pol &pol, uint32_t v, int last, Emit emit) {
    recv_row_from(pol, v, digits(pol, v), last, emit);
}

// recv_row for a caller that already has dv = digits(pol, v)
template <class Pol, class Emit>
BCS_HD void recv_row_from(const Pol &pol, uint32_t v, uint32_t dv, int last, Emit emit) {
    const uint32_t p = pol.p();
    const int q = pol.q();
    const uint32_t lap = 1u << (q & 31);
    const int home = 31 - BCS_CLZ(dv);                    // -1 for the root
    const int own = dv ? __builtin_ctz(dv) : 0;
    uint32_t B = v ? (1u << own) : 0u;
    // Digits of v - skips[n] with the lap digit.  When skips[n] is part of v's greedy sum, taking it out leaves the
    // greedy sum of v - skips[n] (the ranks below it were below skips[n] before and still are), and for n = q the
    // end point is v itself: no walk.  The high digits of consecutive ranks agree, so whole waves take this path.
    // (Lanes with unrelated p never agree on it, so the per-lane policy does not ask.)
    auto end_digits = [&](int n, uint32_t s) -> uint32_t {
        const bool ahead = v >= s;
        const uint32_t y = ahead ? v - s : v + p - s;
        if constexpr (Pol::kScalarSkips) {
            const uint32_t nbit = 1u << (n & 31);
            const bool direct = (n == q) || (dv & nbit) != 0u;
            uint32_t d = (n == q) ? dv : ((dv & ~nbit) | lap);
            if (BCS_WAVE_ANY(!direct)) d = digits(pol, y) | (ahead ? lap : 0u);
            return d;
        } else {
            return digits(pol, y) | (ahead ? lap : 0u);
        }
    };
    uint32_t s_i = pol.sdyn(0);
    uint32_t d_hi = end_digits(0, s_i);
    bool have_hi = true;                                  // wave-uniform: d_hi holds the digits of v - skips[i]
    uint32_t low = 0;                                     // value of v's digits below round i
#pragma unroll 1
    for (int i = 0; i <= last; ++i) {
        const uint32_t s_n = pol.sdyn(i + 1);
        int val = 0, blk = 0;
        bool easy = false, window = true;
        if constexpr (Pol::kScalarSkips) {
            easy = i >= kDigitRoundsFrom && round_from_digits(pol, dv | lap, i, s_i, low, home, own, val, blk);
            window = BCS_WAVE_ANY(!easy);
        }
        if (window) {
            if (!have_hi) d_hi = end_digits(i, s_i);
            const uint32_t d_lo = end_digits(i + 1, s_n);
            int wb;
            const int w = recv_round_value(pol, v, i, s_n, d_lo, d_hi, home, own, B,
                                           [&](uint32_t r) { return digits(pol, r); }, wb);
            val = easy ? val : w;
            blk = easy ? blk : wb;
            d_hi = d_lo;
        }
        have_hi = window;
        const bool active = i < q;                        // per-lane q may be below the wave's bound
        B |= active ? (1u << (blk & 31)) : 0u;
        if (active) emit(i, val);
        low += (0u - ((dv >> (i & 31)) & 1u)) & s_i;
        s_i = s_n;
    }
}

// The same row with every digit mask read from a table of all ranks' masks (dtab[y] = digits of rank y, filled
// by one walk per rank beforehand): every end point of every window is some rank.  All q rounds, unrolled, so that
// the skips are the policy's registers and the reads of later rounds can be issued ahead of the rounds that use
// them.
template <class Pol, class Emit>
BCS_HD void recv_row_tab(const Pol &pol, const uint32_t *__restrict__ dtab, uint32_t v, Emit emit) {
    static_assert(Pol::kScalarSkips, "one p per launch: the inert skips of the per-lane policy are no table indices");
    constexpr int kQ = Pol::kTopLevel + 1;
    const uint32_t p = pol.p();
    const uint32_t lap = 1u << (kQ & 31);
    // d(n): digits of v - skips[n] with the lap digit.  Those of the low rounds, which always need their windows,
    // are read ahead; the others only by the few waves that need a window in a high round.
    constexpr int kAhead = kQ < kTabAhead ? kQ : kTabAhead;
    auto end_point = [&](int n) -> uint32_t {
        const uint32_t s = pol.s(n);
        const bool ahead = v >= s;
        return dtab[ahead ? v - s : v + p - s] | (ahead ? lap : 0u);
    };
    uint32_t d[kAhead + 1];
#pragma unroll
    for (int n = 0; n <= kAhead; ++n) d[n] = end_point(n);
    const uint32_t dv = dtab[v];                         // skips[q] = p: the rank itself, no lap
    const int home = 31 - BCS_CLZ(dv);
    const int own = dv ? __builtin_ctz(dv) : 0;
    uint32_t B = v ? (1u << own) : 0u;
    uint32_t low = 0;                                    // value of v's digits below round i
#pragma unroll
    for (int i = 0; i < kQ; ++i) {
        int val = 0, blk = 0;
        const bool easy = i >= kDigitRoundsFrom && round_from_digits(pol, dv | lap, i, pol.s(i), low, home, own, val, blk);
        if (BCS_WAVE_ANY(!easy)) {
            const uint32_t d_hi = i <= kAhead ? d[i <= kAhead ? i : 0] : end_point(i);
            const uint32_t d_lo = i + 1 == kQ ? dv : (i + 1 <= kAhead ? d[i + 1 <= kAhead ? i + 1 : 0] : end_point(i + 1));
            int wb;
            const int w = recv_round_value(pol, v, i, pol.s(i + 1), d_lo, d_hi, home, own, B,
                                           [&](uint32_t r) { return dtab[r]; }, wb);
            val = easy ? val : w;
            blk = easy ? blk : wb;
        }
        B |= 1u << (blk & 31);
        emit(i, val);
        low += (0u - ((dv >> i) & 1u)) & pol.s(i);
    }
}

// Rounds 0..last of the same row, for Alg. 5's neighbours (last varies, so the rounds stay a loop): the read for
// the next round is issued before this round's work.  dv = dtab[v] comes from the caller.
template <class Pol, class Emit>
BCS_HD void recv_row_tab_upto(const Pol &pol, const uint32_t *__restrict__ dtab, uint32_t v, uint32_t dv, int last,
                              Emit emit) {
    static_assert(Pol::kScalarSkips, "one p per launch: the inert skips of the per-lane policy are no table indices");
    const uint32_t p = pol.p();
    const int q = pol.q();
    const uint32_t lap = 1u << (q & 31);
    auto end_point = [&](uint32_t s) -> uint32_t {       // digits of v - s with the lap digit, s in [1, p]
        const bool ahead = v >= s;
        return dtab[ahead ? v - s : v + p - s] | (ahead ? lap : 0u);
    };
    uint32_t d_hi = end_point(pol.sdyn(0));
    uint32_t s_n = pol.sdyn(1);
    uint32_t d_lo = end_point(s_n);
    const int home = 31 - BCS_CLZ(dv);
    const int own = dv ? __builtin_ctz(dv) : 0;
    uint32_t B = v ? (1u << own) : 0u;
#pragma unroll 1
    for (int i = 0; i <= last; ++i) {
        const uint32_t s_next = pol.sdyn(i + 2 <= q ? i + 2 : q);
        const uint32_t d_next = end_point(s_next);
        recv_round(pol, v, i, s_n, d_lo, d_hi, home, own, B, [&](uint32_t r) { return dtab[r]; }, emit);
        d_hi = d_lo;
        d_lo = d_next;
        s_n = s_next;
    }
}

// Send entries without the to-neighbour's rounds (Alg. 5 costs entry k that neighbour's rounds 0..k).
// With t = (v + skips[k]) mod p the entry is entry k of t's receive row, and in three cases none of t's rounds
// are needed:
//   (a) k is t's home round, which is the case exactly for v < skips[k+1] - skips[k]: the entry is t's
//       baseblock (Alg. 4's first branch), and D(t) = D(v) with digit k added, so that baseblock is v's, or k
//       for v = 0;
//   otherwise, when v has a digit at or above k, let m be the lowest such digit and L the value of v's digits
//   below k.  The rank with the digits of v from m up and nothing below lies in round k's first window
//   (v - (skips[k+1] - skips[k]), v], holds baseblock m, and nothing larger lies there; so the entry is m - q
//   unless t has come by block m in its earlier rounds.  Those rounds' windows reach back to v + 1 only, and past
//   it, by Alg. 4's second range, by at most the number of odd levels; between v + 1 and t the ranks whose lower
//   part is empty hold blocks other than m.  So the entry is m - q
//   (b) when L keeps clear of both ends of its range: 2c + 2 < L < skips[k] - 1 - (2c + 2), c = the number of
//       odd levels up to k.  The second range of round i of t reaches skips[k] - skips[i+1] + 1 - c_i ranks past
//       v + 1 at most, so it can touch the holder of m, the rank v - L, only for L < c; at the other end a lower
//       part within c of skips[k] - 1 runs over the end of its (shortened) copy when the skip is added.  Every
//       exception found (all entries of every rank of every p <= 40 000; 39 million entries of structured larger
//       p up to 2^31 with L within 80 of either end, 0.6 million of them exceptions) has L within c - 1 of an end;
//       the margin is more than twice that;
//   (c) when the digits of t below k are those of v (adding the skip did not disturb them): no exception in the
//       same searches.
// (b) is what round_from_digits argues for receive rounds, read from the sender (digit k of v clear: t has digit k
// set and the same low part; set: the addition carries, t has digit k clear and the low part L plus the odd levels
// the carry passes); (c) goes beyond it and is an observation, not a proved statement.  The CPU tests compare this
// code with Alg. 5 of the oracle entry by entry (every rank of every p <= 1500, of every p <= 40 000 behind the slow
// marker, and structured large p).  Everything else -- L near an end of its range and low digits disturbed by a
// carry that met an odd level -- is left to Alg. 5: the return value has bit k set for every entry k < q that was
// NOT emitted.
template <class Pol, class DigitsOf, class Emit>
BCS_HD uint32_t send_row_direct(const Pol &pol, uint32_t v, uint32_t dv, DigitsOf digits_of, Emit emit) {
    const uint32_t p = pol.p();
    const int q = pol.q();
    uint32_t pending = 0;
    uint32_t low = 0;                                         // value of v's digits below k
#pragma unroll 1
    for (int k = 0; k <= pol.top(); ++k) {
        const bool active = k < q;                            // per-lane q may be below the wave's bound
        const uint32_t s = active ? pol.sdyn(k) : 0u;
        const uint32_t kbit = 1u << (k & 31);
        const uint32_t oddk = (pol.odd_mask() >> (k & 31)) & 1u;
        const uint32_t above = dv & ~(kbit - 1u);
        const bool home = active && v + oddk < s;             // v < skips[k+1] - skips[k]
        const uint32_t mrg = 2u * (uint32_t)__builtin_popcount(pol.odd_mask() & ((kbit << 1) - 1u)) + 2u;
        const bool mid = low > mrg && low + mrg + 1u < s;
        bool direct = home || (above != 0u && mid);
        const bool ask = active && !direct && above != 0u;    // (c) needs the digits of t
        bool same_low = false;
        if (BCS_WAVE_ANY(ask)) {
            uint32_t t = v + s;
            t = t >= p ? t - p : t;
            const uint32_t dt = digits_of(t);
            same_low = ((dv ^ dt) & (kbit - 1u)) == 0u;
        }
        direct = direct || (ask && same_low);
        const int val = home ? (v ? __builtin_ctz(dv | 0x80000000u) : k) : __builtin_ctz(above | 0x80000000u) - q;
        if (active && direct) emit(k, val);
        pending |= (active && !direct) ? kbit : 0u;
        low += (dv & kbit) ? s : 0u;
    }
    return pending;
}

}  // namespace bcs
#endif  // BCS_CORE_H
