// bcs_core.h: the per-rank schedule construction, written once for the GPU lanes and for a host
// build that the CPU tests use to check this same code against the oracle.
//
// Method: J. L. Traff, arXiv 2205.10072, Section 2 (Alg. 1, 2, 4).  Block sets are 32-bit masks.
//
// How a lane finds the baseblocks of a rank range [a, b] (what the paper's Alg. 3 is for) is this
// library's own routine.  It rests on the self-similarity stated after Alg. 2: rank skips[k] has
// baseblock k, and ranks skips[k]+1 .. skips[k+1]-1 repeat the baseblocks of ranks
// 1 .. skips[k+1]-skips[k]-1.  Walking the levels k = q-1 .. 0 once:
//   b <  skips[k]            nothing at this level;
//   a >  skips[k] (<= b)     the range lies in the upper copy: move it down by skips[k];
//   a <= skips[k] <= b       block k is in; so are the blocks of ranks 1 .. b-skips[k], which are
//                            exactly 0 .. (largest level whose skip is <= b-skips[k]); what is left
//                            is [a, skips[k]-1], handled by the remaining levels.
// The walk is branch-free (compare / select), so the lanes of a wave never diverge in it.
#ifndef BCS_CORE_H
#define BCS_CORE_H

#include <stdint.h>

#if defined(__HIP_DEVICE_COMPILE__)
#define BCS_HD __device__ __forceinline__
#define BCS_WAVE_ANY(x) __any(x)
#define BCS_CLZ(x) __clz((int)(x))
#elif defined(__HIPCC__)
#define BCS_HD __device__ __forceinline__
#define BCS_WAVE_ANY(x) (x)
#define BCS_CLZ(x) ((x) ? __builtin_clz(x) : 32)
#else
#define BCS_HD inline
#define BCS_WAVE_ANY(x) (x)
#define BCS_CLZ(x) ((x) ? __builtin_clz(x) : 32)
#endif

namespace bcs {

constexpr int kMaxQ = 31;

struct SkipTab {
    uint32_t s[kMaxQ + 2];               // s[0..q]; entries above q repeat p
};

// ----------------------------------------------------------------------------------------------
// Skip policies.  Uniform<Q>: one p for the whole launch, Q known at compile time, level loops
// fully unrolled, skips in SGPRs.  PerLane: every lane has its own p and q; skips come from the
// closed form skips[k] = ceil(p / 2^(q-k)) = ((p-1) >> (q-k)) + 1 that Alg. 1's halving produces.
// ----------------------------------------------------------------------------------------------
template <int Q>
struct Uniform {
    uint32_t S[Q + 1];
    const SkipTab *tab;                  // same values, for wave-uniform dynamic indices
    BCS_HD int q() const { return Q; }
    BCS_HD int top() const { return Q - 1; }
    BCS_HD uint32_t p() const { return S[Q]; }
    BCS_HD uint32_t s(int k) const { return S[k]; }          // k constant after unrolling
    BCS_HD uint32_t sdyn(int k) const { return tab->s[k]; }  // k wave-uniform
    // skips[h+1] - 1 for a per-lane h in [-1, Q-1]
    BCS_HD uint32_t skip_above_minus1(int h) const { return (S[Q] - 1u) >> (Q - 1 - h); }
};

struct PerLane {
    uint32_t pm1;                        // p - 1
    int ql;                              // this lane's q
    int wave_top;                        // largest q in the wave, minus 1 (uniform loop bound)
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

// Alg. 2 as a level walk (largest skip first, subtract while it fits): returns the baseblock of
// v > 0 and, in `home`, the level h with skips[h] <= v < skips[h+1] (-1 for the root).
template <class Pol>
BCS_HD int baseblock_and_home(const Pol &pol, uint32_t v, int &home) {
    int own = 0, h = -1;
    uint32_t y = v;
#pragma unroll
    for (int k = pol.top(); k >= 0; --k) {
        const uint32_t s = pol.s(k);
        const bool fits = s <= y;
        h = (fits && h < 0) ? k : h;
        own = fits ? k : own;
        y = fits ? y - s : y;
    }
    home = h;
    return own;
}

// Alg. 4: entries 0..last of the receive schedule of virtual rank v; emit(i, value) per entry.
// The rank's own baseblock starts the set B of blocks it already has.  Round i looks for the largest
// new block among ranks v-skips[i+1]+1 .. v-skips[i]; if there is none, among ranks
// v-sum_{j<=i}skips[j] .. v-skips[i+1].  Ranks are mod p and rank 0 owns no baseblock.  The i = 0 and
// i = q-1 special cases printed in Alg. 4 are instances of this rule.
template <class Pol, class Emit>
BCS_HD void recv_row(const Pol &pol, uint32_t v, int last, Emit emit) {
    const uint32_t p = pol.p();
    const int q = pol.q();
    int home;
    const int own = baseblock_and_home(pol, v, home);
    uint32_t B = v ? (1u << own) : 0u;
    const uint32_t all = (q >= 32) ? 0xffffffffu : ((1u << q) - 1u);
    uint32_t psum = 0;
    uint32_t s_i = pol.sdyn(0);
#pragma unroll 1
    for (int i = 0; i <= last; ++i) {
        const uint32_t s_n = pol.sdyn(i + 1);
        psum += s_i;
        const bool active = i < q;                       // per-lane q may be below the wave's bound
        const bool is_home = (i == home);
        // first range; for i > home it wraps below rank 0 and is taken p higher
        const uint32_t base = (v >= s_n) ? v : v + p;
        uint32_t a = base - s_n + 1u, b = base - s_i;
        if (is_home || !active) { a = 1u; b = 0u; }
        uint32_t U = range_blocks(pol, a, b) & ~B;
        const bool need2 = active && !is_home && U == 0u;
        if (BCS_WAVE_ANY(need2)) {
            // second range, possibly cut in two by rank 0
            int64_t lo = (int64_t)v - (int64_t)psum, hi = (int64_t)v - (int64_t)s_n;
            const bool whole = (hi - lo + 1) >= (int64_t)p;
            if (hi < 0) { lo += p; hi += p; }
            uint32_t a1, b1, a2 = 1u, b2 = 0u;
            if (lo >= 1) { a1 = (uint32_t)lo; b1 = (uint32_t)hi; }
            else { a1 = (uint32_t)(lo + p); b1 = p - 1u; a2 = 1u; b2 = (uint32_t)hi; if (lo == 0) { a1 = 1u; b1 = 0u; } }
            if (!need2 || whole) { a1 = 1u; b1 = 0u; a2 = 1u; b2 = 0u; }
            uint32_t U2 = whole ? all : 0u;
#pragma unroll 1
            for (int piece = 0; piece < 2; ++piece) {
                U2 |= range_blocks(pol, piece ? a2 : a1, piece ? b2 : b1);
            }
            U = need2 ? (U2 & ~B) : U;
        }
        const int blk = 31 - BCS_CLZ(U);             // largest candidate
        if (active) {
            if (is_home) emit(i, own);
            else { B |= 1u << (blk & 31); emit(i, blk - q); }
        }
        s_i = s_n;
    }
}

}  // namespace bcs
#endif  // BCS_CORE_H
