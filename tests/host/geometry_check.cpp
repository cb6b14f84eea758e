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

static void check_wide(int copies)
{
    const int elt = copies == 4 ? 8 : 4;  // bytes per lane element
    for (int c = 0; c < N_WIDE_CLS; ++c) {
        const int csb = wide_copy_bytes(CLS_WAVES[c]);
        const int cells = CLS_WAVES[c] * WIDE_CHUNK;
        CHECK(csb % elt == 0 && WIDE_PAD_BYTES % elt == 0, "class %d", c);
        for (int lt = 0; lt < cells; ++lt) {
            const uint32_t shift = wide_shift((uint32_t)lt, copies, csb);
            CHECK(wide_lt_of_shift(shift, copies, csb) == (uint32_t)lt, "class %d copies %d lt %d", c,
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
    for (int copies_mask : {0x3FF, 0}) {
        const int copies = class_copies(2, copies_mask);
        const uint32_t shift = wide_shift(345u, copies, wide_copy_bytes(CLS_WAVES[2]));
        CHECK(lt_of_entry(shift, T, map, copies_mask) == 345u, "copies %d", copies);
    }
    CHECK(lt_of_entry(narrow_shift(20001u), 30000, map, 0x3FF) == 20001u, "narrow entry");
    CHECK(class_copies(3, 0x3FF) == 2 && class_copies(3, 0) == 4, "copies mask");
}

int main()
{
    check_wide(2);
    check_wide(4);
    check_narrow();
    check_classes();
    if (failures) {
        std::printf("%d checks failed\n", failures);
        return 1;
    }
    std::printf("geometry ok\n");
    return 0;
}
