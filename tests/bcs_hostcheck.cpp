// Host build of the per-rank construction in bcs_core.h, one "lane" at a time, so that CPU tests can
// compare the code the GPU lanes run with the oracle.  Test support; not part of libbcsched.
#include <stddef.h>
#include <stdint.h>

#include "bcs_core.h"

using namespace bcs;

namespace {

int host_q(int32_t p) {
    int q = 0;
    while (((int64_t)1 << q) < (int64_t)p) ++q;
    return q;
}

void fill_skips(int32_t p, SkipTab &t) {
    const int q = host_q(p);
    for (int k = 0; k <= q; ++k) t.s[k] = (((uint32_t)p - 1u) >> (q - k)) + 1u;
    for (int k = q + 1; k < kMaxQ + 2; ++k) t.s[k] = (uint32_t)p;
    t.odd = odd_levels((uint32_t)p, q);
}

// the low-level table, filled on the host by the same entry function the GPU's fill kernel runs
uint8_t g_low[kLowTableBytes];
bool g_low_ready = false;
const uint8_t *low_for(int32_t p) {
    if (!g_low_ready) {
        for (int e = 0; e < kLowTableBytes; ++e) {
            const int shape = e / kLowShapeBytes, rest = e - shape * kLowShapeBytes;
            g_low[e] = (uint8_t)low_table_entry(shape, rest >> 7, rest & 127);
        }
        g_low_ready = true;
    }
    return g_low + (size_t)low_shape((uint32_t)p, host_q(p)) * kLowShapeBytes;
}

template <int Q>
void row_uniform(const SkipTab &t, uint32_t v, int last, int32_t *out) {
    Uniform<Q> pol;
    for (int k = 0; k <= Q; ++k) pol.S[k] = t.s[k];
    pol.tab = &t;
    pol.low = low_for((int32_t)t.s[Q]);
    recv_row(pol, v, last, [&](int i, int val) { out[i] = val; });
}

// the same row from a table of all ranks' digit masks, as the kernels for whole rank ranges build it
template <int Q>
void row_from_table(const SkipTab &t, const uint32_t *dtab, uint32_t v, int last, int32_t *out) {
    Uniform<Q> pol;
    for (int k = 0; k <= Q; ++k) pol.S[k] = t.s[k];
    pol.tab = &t;
    pol.low = low_for((int32_t)t.s[Q]);
    if (!dtab) {
        *reinterpret_cast<uint32_t *>(out) = digits(pol, v);      // table entry of rank v
        return;
    }
    if (last == Q - 1) recv_row_tab(pol, dtab, v, [&](int i, int val) { out[i] = val; });
    else recv_row_tab_upto(pol, dtab, v, dtab[v], last, [&](int i, int val) { out[i] = val; });
}

template <int Q>
uint32_t range_uniform(const SkipTab &t, uint32_t a, uint32_t b) {
    Uniform<Q> pol;
    for (int k = 0; k <= Q; ++k) pol.S[k] = t.s[k];
    pol.tab = &t;
    pol.low = nullptr;
    return range_blocks(pol, a, b);
}

typedef void (*RowFn)(const SkipTab &, uint32_t, int, int32_t *);
typedef uint32_t (*RangeFn)(const SkipTab &, uint32_t, uint32_t);
typedef void (*TabRowFn)(const SkipTab &, const uint32_t *, uint32_t, int, int32_t *);

template <int Q>
struct Fill {
    static void go(RowFn *r, RangeFn *g, TabRowFn *t) {
        r[Q] = &row_uniform<Q>;
        g[Q] = &range_uniform<Q>;
        t[Q] = &row_from_table<Q>;
        Fill<Q - 1>::go(r, g, t);
    }
};
template <>
struct Fill<0> {
    static void go(RowFn *, RangeFn *, TabRowFn *) {}
};

RowFn g_row[kMaxQ + 1];
RangeFn g_range[kMaxQ + 1];
TabRowFn g_tabrow[kMaxQ + 1];
bool g_ready = false;
void ready() {
    if (!g_ready) {
        Fill<kMaxQ>::go(g_row, g_range, g_tabrow);
        g_ready = true;
    }
}

}  // namespace

extern "C" {

// entries 0..last of the receive row of virtual rank v, uniform-p code path
int hc_recv_row(int32_t p, int32_t v, int last, int32_t *out) {
    if (p < 2 || v < 0 || v >= p) return -1;
    ready();
    SkipTab t;
    fill_skips(p, t);
    g_row[host_q(p)](t, (uint32_t)v, last, out);
    return 0;
}

// the same through the per-lane-p code path; wave_q >= q plays the largest q of the wave
int hc_recv_row_perlane(int32_t p, int32_t v, int last, int wave_q, int32_t *out) {
    if (p < 1 || v < 0 || v >= p) return -1;
    PerLane pol;
    pol.pm1 = (uint32_t)p - 1u;
    pol.ql = host_q(p);
    pol.wave_top = wave_q - 1;
    pol.odd = odd_levels((uint32_t)p, pol.ql);
    pol.low = low_for(p);
    recv_row(pol, (uint32_t)v, last, [&](int i, int val) { out[i] = val; });
    return 0;
}

// all p receive rows (uniform-p code path), rank-major with q entries a row
int hc_recv_rows_all(int32_t p, int32_t *out) {
    if (p < 2) return -1;
    ready();
    SkipTab t;
    fill_skips(p, t);
    const int q = host_q(p);
    for (int32_t v = 0; v < p; ++v) g_row[q](t, (uint32_t)v, q - 1, out + (size_t)v * q);
    return 0;
}

// all p receive rows through the table of digit masks: dtab (p words of scratch) is filled first, one walk a rank
int hc_recv_rows_all_tab(int32_t p, uint32_t *dtab, int32_t *out) {
    if (p < 2) return -1;
    ready();
    SkipTab t;
    fill_skips(p, t);
    const int q = host_q(p);
    for (int32_t v = 0; v < p; ++v) {
        int32_t word;
        g_tabrow[q](t, nullptr, (uint32_t)v, 0, &word);
        dtab[v] = (uint32_t)word;
    }
    for (int32_t v = 0; v < p; ++v) g_tabrow[q](t, dtab, (uint32_t)v, q - 1, out + (size_t)v * q);
    return 0;
}

// entries 0..last of one row from a filled table of digit masks (what Alg. 5 asks of a neighbour's row)
int hc_recv_row_tab(int32_t p, const uint32_t *dtab, int32_t v, int last, int32_t *out) {
    if (p < 2 || v < 0 || v >= p || !dtab) return -1;
    ready();
    SkipTab t;
    fill_skips(p, t);
    g_tabrow[host_q(p)](t, dtab, (uint32_t)v, last, out);
    return 0;
}

// full receive rows of the listed virtual ranks, out[i * 32 + k]; perlane != 0: through the per-lane-p path with
// a wave bound of min(q + 2, 31)
int hc_recv_rows_list(int32_t p, const int32_t *v, int64_t count, int perlane, int32_t *out) {
    if (p < 2 || !v || !out) return -1;
    ready();
    SkipTab t;
    fill_skips(p, t);
    const int q = host_q(p);
    for (int64_t i = 0; i < count; ++i) {
        if (v[i] < 0 || v[i] >= p) return -1;
        if (perlane) {
            const int wq = q + 2 < 31 ? q + 2 : 31;
            if (hc_recv_row_perlane(p, v[i], wq - 1, wq, out + i * 32)) return -1;
        } else {
            g_row[q](t, (uint32_t)v[i], q - 1, out + i * 32);
        }
    }
    return 0;
}

// send rows of the listed virtual ranks as the batch kernel builds them: the entries that need no rounds of the
// to-neighbour directly, the rest by Alg. 5 on the lane code; out[i * 32 + k]; direct_mask[i] (may be NULL) gets the
// bits of the entries that were taken directly
int hc_send_rows_list(int32_t p, const int32_t *v, int64_t count, int wave_q, int32_t *out, uint32_t *direct_mask) {
    if (p < 1 || !v || !out) return -1;
    for (int64_t i = 0; i < count; ++i) {
        if (v[i] < 0 || v[i] >= p) return -1;
        PerLane pol;
        pol.pm1 = (uint32_t)p - 1u;
        pol.ql = host_q(p);
        pol.wave_top = (wave_q > pol.ql ? wave_q : pol.ql) - 1;
        pol.odd = odd_levels((uint32_t)p, pol.ql);
        pol.low = low_for(p);
        int32_t *row = out + i * 32;
        const uint32_t dv = digits(pol, (uint32_t)v[i]);
        uint32_t pending = send_row_direct(pol, (uint32_t)v[i], dv, [&](uint32_t y) { return digits(pol, y); },
                                           [&](int k, int val) { row[k] = val; });
        if (direct_mask) direct_mask[i] = ~pending & (pol.ql >= 32 ? 0xffffffffu : ((1u << pol.ql) - 1u));
        while (pending) {
            const int k = 31 - __builtin_clz(pending);
            pending &= ~(1u << k);
            uint32_t t = (uint32_t)v[i] + pol.s(k);
            t = t >= (uint32_t)p ? t - (uint32_t)p : t;
            recv_row(pol, t, k, [&](int j, int val) { if (j == k) row[k] = val; });
        }
    }
    return 0;
}

// mask of baseblocks of ranks a..b (1 <= a, b < p), uniform-p code path
uint32_t hc_range_blocks(int32_t p, uint32_t a, uint32_t b) {
    ready();
    SkipTab t;
    fill_skips(p, t);
    return g_range[host_q(p)](t, a, b);
}
}
