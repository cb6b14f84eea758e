// Host-side check of the LDS geometry that stage 1 bakes into the candidate
// entries and stage 2 relies on.  Built and run by tests/test_host_geometry.py
// (no GPU needed).  Every property is stated from the layout's definition, not
// from the formulas under test:
//   wide kernel   copy m of a row holds cell t at byte PAD + 2t - 2m of the copy;
//                 a lane element starts at a cell t0 that is a multiple of the
//                 element's cells, and adding an entry's shift to the element's
//                 place in copy 0 must land, aligned, on cell t0 - lt of some copy;
//   narrow kernel dword j of copy A holds cells (2j, 2j+1), of copy B (2j+1, 2j+2),
//                 each copy behind one wavefront's worth of padding.
#include <cstdio>
#include <cstdlib>

#include "themis_internal.h"

using namespace themis;

static int failures = 0;
#define CHECK(cond, ...)                                  \
    do {                                                  \
        if (!(cond)) {                                    \
            if (failures < 20) {                          \
                std::printf("FAIL %s: ", #cond);          \
                std::printf(__VA_ARGS__);                 \
                std::printf("\n");                        \
            }                                             \
            ++failures;                                   \
        }                                                 \
    } while (0)

static void check_wide()
{
    const int copies = WIDE_COPIES;
    const int elt = 4;  // bytes per lane element
    for (int c = 0; c < N_WIDE_CLS; ++c) {
        const int csb = wide_copy_bytes(CLS_WAVES[c]);
        const int cells = CLS_WAVES[c] * WIDE_CHUNK;
        CHECK(csb % elt == 0 && WIDE_PAD_BYTES % elt == 0, "class %d", c);
        for (int lt = 0; lt < cells; ++lt) {
            const uint32_t shift = wide_shift((uint32_t)lt, csb);
            CHECK(wide_lt_of_shift(shift, csb) == (uint32_t)lt, "class %d copies %d lt %d", c,
                  copies, lt);
            // elements of the position the entry's bucket starts in, of the last
            // position, and one straddling lt
            const int first = (lt / BUCKET_CELLS) * BUCKET_CELLS;
            const int probes[4] = {first, (lt / (elt / 2)) * (elt / 2), first + BUCKET_CELLS - elt / 2,
                                   cells - elt / 2};
            for (int t0 : probes) {
                if (t0 >= cells) continue;
                const long addr = (long)WIDE_PAD_BYTES + 2L * t0 + (long)(int32_t)shift;
                CHECK(addr >= 0 && addr % elt == 0, "class %d copies %d lt %d t0 %d addr %ld", c,
                      copies, lt, t0, addr);
                const long m = addr / csb, off = addr - m * csb;
                CHECK(m >= 0 && m < copies && off + elt <= csb, "class %d copies %d lt %d t0 %d", c,
                      copies, lt, t0);
                // the element's first cell, by the layout of copy m
                const long cell = (off - WIDE_PAD_BYTES) / 2 + m;
                CHECK((off - WIDE_PAD_BYTES) % 2 == 0 && cell == (long)t0 - lt,
                      "class %d copies %d lt %d t0 %d reads cell %ld", c, copies, lt, t0, cell);
                // reads below cell 0 stay inside the copy's padding
                CHECK(off >= 0, "class %d copies %d lt %d t0 %d", c, copies, lt, t0);
            }
        }
    }
}

static void check_narrow()
{
    const int cells = 2 * NAR_WAVES * NAR_CHUNK_DW;
    for (int lt = 0; lt < cells; ++lt) {
        const uint32_t shift = narrow_shift((uint32_t)lt);
        CHECK(shift % 4 == 0, "lt %d", lt);
        CHECK(narrow_lt_of_shift(shift) == (uint32_t)lt, "lt %d", lt);
        const int probes[3] = {lt / 2, (lt + 1) / 2 + 7, NAR_WAVES * NAR_CHUNK_DW - 1};
        for (int j : probes) {  // output dword j = cells (2j, 2j+1)
            if (j >= NAR_WAVES * NAR_CHUNK_DW || 2 * j + 1 < lt) continue;
            // LDS addresses are 32 bits wide: shifts below zero wrap back into range
            const long d = (long)((uint32_t)(shift + 4u * (uint32_t)j) / 4u);
            long first_cell;
            if (d < NAR_COPY_DW) {
                first_cell = 2 * (d - NAR_CHUNK_DW);  // copy A, behind its padding
                CHECK(d >= 0, "lt %d j %d", lt, j);
            } else {
                first_cell = 2 * (d - NAR_COPY_DW - NAR_CHUNK_DW) + 1;  // copy B
                CHECK(d < 2 * NAR_COPY_DW && d >= NAR_COPY_DW, "lt %d j %d", lt, j);
            }
            CHECK(first_cell == 2L * j - lt, "lt %d j %d reads cell %ld", lt, j, first_cell);
        }
    }
}

static void check_classes()
{
    for (int T = 0; T <= THEMIS_MAX_TICKS; ++T) {
        const int c = class_of_budget(T), cells = T + 1;
        if (cells > WIDE_MAX_CELLS) {
            CHECK(c == NARROW_CLS, "T %d", T);
            continue;
        }
        CHECK(c >= 0 && c < N_WIDE_CLS && cells <= CLS_WAVES[c] * WIDE_CHUNK, "T %d class %d", T, c);
        CHECK(c == 0 || cells > CLS_WAVES[c - 1] * WIDE_CHUNK, "T %d class %d is not the smallest", T, c);
    }
    for (int c = 1; c < N_WIDE_CLS; ++c) CHECK(CLS_WAVES[c] > CLS_WAVES[c - 1], "class %d", c);
    CHECK(CLS_WAVES[N_WIDE_CLS - 1] * WIDE_CHUNK == WIDE_MAX_CELLS, "top class");
    CHECK(2 * NAR_WAVES * NAR_CHUNK_DW > THEMIS_MAX_TICKS, "the narrow kernel holds the longest row");

    // groups: heads at classes 9, 5 and 2
    uint64_t map = 0;
    const int heads[N_WIDE_CLS] = {2, 2, 2, 5, 5, 5, 9, 9, 9, 9};
    for (int c = 0; c < N_WIDE_CLS; ++c) map |= (uint64_t)heads[c] << (4 * c);
    for (int c = 0; c < N_WIDE_CLS; ++c) CHECK(head_of_class(c, map) == heads[c], "class %d", c);
    CHECK(head_of_class(NARROW_CLS, map) == NARROW_CLS, "narrow");
    CHECK(effective_class(0, map) == 2 && effective_class(3 * WIDE_CHUNK, map) == 5 &&
              effective_class(WIDE_MAX_CELLS - 1, map) == 9 &&
              effective_class(WIDE_MAX_CELLS, map) == NARROW_CLS,
          "effective classes");
    // an entry is decoded with the geometry of the class that serves the instance
    const int T = 700;  // class 0, served by class 2
    CHECK(lt_of_entry(wide_shift(345u, wide_copy_bytes(CLS_WAVES[2])), T, map) == 345u, "wide entry");
    CHECK(lt_of_entry(narrow_shift(20001u), 30000, map) == 20001u, "narrow entry");
}

static void check_layout()
{
    const int shapes[][6] = {  // N, S, c_max, n_batch, slo_max_us, tick_us
        {1, 1, 1, 1, 0, 1},        {64, 3, 8, 5, 300000, 1000},   {4096, 5, 16, 7, 1000000, 250},
        {65536, 8, 32, 8, 4000000, 250}, {7, 2, 512, 16, 32767, 1}, {1000, 4, 3, 3, 8191999, 250}};
    for (const auto& sh : shapes) {
        themis_problem_t p{};
        p.n_inst = sh[0], p.n_stage = sh[1], p.c_max = sh[2], p.n_batch = sh[3];
        p.slo_max_us = sh[4], p.tick_us = sh[5];
        const Layout L = make_layout(p);
        const size_t rows = (size_t)L.N * L.S;
        const int T = sh[4] / sh[5];
        CHECK(L.K == sh[2] * sh[3] && L.Kp >= L.K && L.Kp % 8 == 0 && L.Kp < L.K + 8, "N %d", sh[0]);
        CHECK(L.t_max == T && L.nb == T / BUCKET_CELLS + 1 && L.nbs >= L.nb + 1 && L.nbs % 2 == 0,
              "N %d", sh[0]);
        // a lane stores up to four cells at once from any cell <= T; rows stay 256-byte aligned
        CHECK(L.row_stride >= T + 4 && L.row_stride % 128 == 0, "N %d stride %d", sh[0], L.row_stride);
        const size_t off[8] = {L.step_off, L.bcum_off, L.frow_off, L.tmeta_off,
                               L.ans_off,  L.order_off, L.ctrl_off, L.total};
        const size_t need[7] = {rows * L.Kp * 8,
                                rows * L.nbs * 2,
                                rows * (size_t)L.row_stride * 2,
                                (size_t)L.N * 4,
                                (size_t)L.N * 8,
                                (size_t)N_CLS * L.N * 4,
                                (size_t)2 * N_CLS * 4};
        CHECK(off[0] == 0, "N %d", sh[0]);
        for (int r = 0; r < 7; ++r) {
            CHECK(off[r] % 256 == 0, "N %d region %d", sh[0], r);
            CHECK(off[r + 1] >= off[r] + need[r] && off[r + 1] < off[r] + need[r] + 256,
                  "N %d region %d", sh[0], r);
        }
    }
    // the shortcut rule: entries times positions against 24 per wavefront
    CHECK(worth_shortcut(24, 1, 1) && !worth_shortcut(23, 1, 1) && worth_shortcut(12, 8, 4) &&
              !worth_shortcut(11, 8, 4) && !worth_shortcut(0, 32, 1),
          "shortcut rule");
}

int main()
{
    check_layout();
    check_wide();
    check_narrow();
    check_classes();
    if (failures) {
        std::printf("%d checks failed\n", failures);
        return 1;
    }
    std::printf("geometry ok\n");
    return 0;
}
