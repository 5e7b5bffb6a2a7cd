// Driver for the sanitizer test (test support): the C oracle and the host build of the lane code, both compiled
// with -fsanitize=address,undefined, run over small problems and compared.  Exits 0 when every comparison holds
// (a sanitizer report aborts the run with its own non-zero status).
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include <vector>

extern "C" {
int orc_q(int32_t p);
int orc_skips(int32_t p, int32_t *skips);
int orc_baseblocks_linear(int32_t p, int32_t *bb);
uint32_t orc_rangeblocks_scan(int32_t p, const int32_t *bb, int64_t a, int64_t b);
uint32_t orc_rangeblocks(int32_t p, int64_t a, int64_t b);
int orc_recvsched(int32_t p, int32_t r, int k, int mode, int32_t *out);
int orc_sendsched(int32_t p, int32_t r, int32_t *out);
int orc_sched_definition(int32_t p, int general_only, int32_t *bb_out, int32_t *recv, int32_t *send);
int orc_sched_range(int32_t p, int32_t root, int32_t r0, int32_t r1, int32_t *recv, int32_t *send, int threads);
int orc_sched_batch(int64_t count, const int32_t *p, const int32_t *r, const int32_t *root, int32_t *recv,
                    int32_t *send, int32_t *q_out, int threads);
int orc_expand(int32_t p, int32_t n, int64_t rows, const int32_t *in, int32_t *out, int threads);
int orc_allgather_tables(int32_t p, int32_t n, int32_t r, int32_t *pack, int32_t *unpack);
int64_t orc_pack_round(int32_t p, int32_t n, const int32_t *idx, const int64_t *displs, const int32_t *data,
                       int32_t *packed, int64_t capacity, int64_t *offsets);
int64_t orc_unpack_round(int32_t p, int32_t n, const int32_t *idx, const int64_t *displs, int32_t *data,
                         const int32_t *packed, int64_t length, int64_t *offsets);
int orc_allgather_plan(int32_t p, int32_t r, int32_t *to, int32_t *from, int32_t *count, int32_t *recv_first);
int orc_census_plan(int32_t p, int32_t r, int32_t *to, int32_t *from, int32_t *own);

int hc_recv_row(int32_t p, int32_t v, int last, int32_t *out);
int hc_recv_row_perlane(int32_t p, int32_t v, int last, int wave_q, int32_t *out);
int hc_recv_rows_all(int32_t p, int32_t *out);
int hc_recv_rows_all_tab(int32_t p, uint32_t *dtab, int32_t *out);
int hc_recv_row_tab(int32_t p, const uint32_t *dtab, int32_t v, int last, int32_t *out);
uint32_t hc_range_blocks(int32_t p, uint32_t a, uint32_t b);
}

static int fail(const char *what, long a, long b) {
    fprintf(stderr, "sanitize_driver: mismatch in %s at (%ld, %ld)\n", what, a, b);
    return 1;
}

static int one_p(int32_t p) {
    const int q = orc_q(p);
    std::vector<int32_t> recv((size_t)p * q + 1), send((size_t)p * q + 1), got((size_t)p * q + 1), bb(p);
    std::vector<uint32_t> dtab(p);
    if (orc_sched_range(p, 0, 0, p, recv.data(), send.data(), 1)) return fail("orc_sched_range", p, 0);
    if (p < 2) return 0;
    orc_baseblocks_linear(p, bb.data());
    if (hc_recv_rows_all(p, got.data()) || memcmp(got.data(), recv.data(), sizeof(int32_t) * p * q)) return fail("hc_recv_rows_all", p, 0);
    if (hc_recv_rows_all_tab(p, dtab.data(), got.data()) || memcmp(got.data(), recv.data(), sizeof(int32_t) * p * q))
        return fail("hc_recv_rows_all_tab", p, 0);
    for (int32_t v = 0; v < p; v += (p > 200 ? 7 : 1)) {
        int32_t row[33], srow[33];
        for (int wq = q; wq <= 31; wq += 5) {
            for (int i = 0; i < 33; ++i) row[i] = 4242;
            if (hc_recv_row_perlane(p, v, wq - 1, wq, row) || memcmp(row, &recv[(size_t)v * q], sizeof(int32_t) * q)) return fail("perlane row", p, v);
            if (row[q] != 4242) return fail("perlane row writes past q", p, v);
        }
        if (orc_sendsched(p, v, srow) || memcmp(srow, &send[(size_t)v * q], sizeof(int32_t) * q)) return fail("Alg. 5 against look-up", p, v);
        const int last = (v * 7 + 3) % q;
        if (hc_recv_row_tab(p, dtab.data(), v, last, row) || memcmp(row, &recv[(size_t)v * q], sizeof(int32_t) * (last + 1))) return fail("row prefix from table", p, v);
        if (orc_recvsched(p, v, q - 1, 3, row) || memcmp(row, &recv[(size_t)v * q], sizeof(int32_t) * q)) return fail("definition row", p, v);
    }
    if (p <= 64)
        for (uint32_t a = 1; a < (uint32_t)p; ++a)
            for (uint32_t b = a; b < (uint32_t)p; ++b)
                if (hc_range_blocks(p, a, b) != orc_rangeblocks_scan(p, bb.data(), a, b) ||
                    orc_rangeblocks(p, a, b) != orc_rangeblocks_scan(p, bb.data(), a, b))
                    return fail("range blocks", a, b);
    for (int32_t n : {1, 2, q, q + 3, 40}) {
        if (n < 1) continue;
        const int64_t R = (int64_t)n - 1 + q;
        std::vector<int32_t> blocks((size_t)p * R + 1);
        if (orc_expand(p, n, p, recv.data(), blocks.data(), 1)) return fail("orc_expand", p, n);
        if (p <= 40) {
            std::vector<int32_t> pack((size_t)R * p + 1), unpack((size_t)R * p + 1);
            if (orc_allgather_tables(p, n, p / 2, pack.data(), unpack.data())) return fail("orc_allgather_tables", p, n);
            // one round of packing and unpacking with sizes (r mod 3) * 5
            std::vector<int64_t> displs(p + 1, 0), offs(p + 1);
            for (int j = 0; j < p; ++j) displs[j + 1] = displs[j] + (j % 3) * 5;
            std::vector<int32_t> data(displs[p] + 1), msg(displs[p] + 1);
            for (size_t i = 0; i < data.size(); ++i) data[i] = (int32_t)i;
            const int64_t len = orc_pack_round(p, n, pack.data() + (R / 2) * p, displs.data(), data.data(), msg.data(), (int64_t)msg.size(), offs.data());
            if (len < 0) return fail("orc_pack_round", p, n);
            if (orc_unpack_round(p, n, pack.data() + (R / 2) * p, displs.data(), data.data(), msg.data(), len, offs.data()) != len)
                return fail("orc_unpack_round", p, n);
        }
    }
    int32_t a[33], b2[33], c[33], d[33];
    if (orc_allgather_plan(p, p - 1, a, b2, c, d) != q || orc_census_plan(p, p / 3, a, b2, c) != q) return fail("plans", p, 0);
    return 0;
}

int main(int argc, char **argv) {
    const int pmax = argc > 1 ? atoi(argv[1]) : 260;
    for (int32_t p = 1; p <= pmax; ++p)
        if (one_p(p)) return 1;
    for (int32_t p : {511, 512, 513, 1000, 1023, 1025, 4097, 65537})
        if (one_p(p)) return 1;
    // single rows of large p through both lane-code paths, and a small batch through the oracle
    const int32_t big[] = {1048577, 134217727, 2147483647, 1073741824, 1073741825, 1500000001};
    for (int32_t p : big) {
        const int q = orc_q(p);
        for (int32_t v : {0, 1, 2, p - 1, p / 2, p / 3, (int32_t)(p * 0.61803)}) {
            int32_t want[33], row[33];
            if (orc_recvsched(p, v, q - 1, 0, want)) return fail("orc_recvsched", p, v);
            if (hc_recv_row(p, v, q - 1, row) || memcmp(row, want, sizeof(int32_t) * q)) return fail("uniform row, large p", p, v);
            if (hc_recv_row_perlane(p, v, 30, 31, row) || memcmp(row, want, sizeof(int32_t) * q)) return fail("perlane row, large p", p, v);
        }
    }
    {
        const int32_t bp[] = {1, 2, 3, 20, 33, 1000, 2147483647}, br[] = {0, 1, 2, 19, 0, 999, 2147483646}, bo[] = {0, 0, 1, 7, 32, 500, 5};
        int32_t rr[7 * 32], ss[7 * 32], qq[7];
        if (orc_sched_batch(7, bp, br, bo, rr, ss, qq, 1)) return fail("orc_sched_batch", 0, 0);
    }
    printf("sanitize_driver: ok (p <= %d and samples)\n", pmax);
    return 0;
}
