// Host-side check of the level-walk kernels' LDS layouts (csrc/lc_walk_layout.h): for every launch
// shape the launchers can produce, every array lies inside the allocation, arrays do not overlap,
// arrays read with 16-byte vector loads are 16-byte aligned, and the limits the entry points report
// are the ones the layout implies.  Prints "ok <cases>" or the first violation.
#include <cstdio>
#include <cstdlib>
#include <vector>
#include <algorithm>
#include "lc_walk_layout.h"

static int fail(const char* what, int a, int b) {
    std::printf("FAIL %s (%d, %d)\n", what, a, b);
    return 1;
}

int main() {
    long cases = 0;
    // ---- exact walk: every (internal nodes, chunks) the host lets through
    const int max_nodes = lc_upper_max_internal_nodes();
    if (lc_upper_lds_bytes(max_nodes, 64) > (size_t)LC_WALK_LDS_LIMIT) return fail("limit too high", max_nodes, 0);
    if (lc_upper_lds_bytes(max_nodes + 64, 64) <= (size_t)LC_WALK_LDS_LIMIT) return fail("limit too low", max_nodes, 0);
    for (int upper = 0; upper <= max_nodes + 200; upper += (upper < 300 ? 1 : 37)) {
        for (int M = 0; M <= 70000; M += (M < 300 ? 1 : 997)) {
            int UC, PC;
            const bool fits = lc_upper_launch_shape(upper, M, &UC, &PC);
            if (upper <= max_nodes && !fits) return fail("a shape within the reported limit does not fit", upper, M);
            if (upper > ((max_nodes + 63) / 64) * 64 && fits) return fail("a shape beyond the limit fits", upper, M);
            if (!fits) continue;
            ++cases;
            if (UC % 64 || PC % 64 || UC < 64 || PC < 64) return fail("slots not multiples of 64", UC, PC);
            if (UC < upper) return fail("fewer node slots than nodes", UC, upper);
            const LcUpperLayout y = lc_upper_layout(UC, PC);
            if ((size_t)y.total > (size_t)LC_WALK_LDS_LIMIT) return fail("over the LDS limit", UC, PC);
            if (y.sc < UC || y.sc * 4 < PC) return fail("staging buffer too short for a level or for the flag bytes", UC, PC);
            struct Arr { int off, bytes, align; };
            const std::vector<Arr> arrs = {
                {y.ukey, 4 * UC, 4}, {y.untok, 4 * UC, 4}, {y.upar, 4 * UC, 4}, {y.kp, UC, 1},
                {y.ekA, 4 * y.sc, 16}, {y.ewA, 4 * y.sc, 16}, {y.ekB, 4 * y.sc, 16}, {y.ewB, 4 * y.sc, 16},
                {y.plist, 4 * PC, 4}, {y.plen, 4 * PC, 16}, {y.pkey, 4 * PC, 16}};
            int end = 0;
            for (const Arr& a : arrs) {
                if (a.off < end) return fail("arrays overlap", UC, PC);
                if (a.off % a.align) return fail("array misaligned for its vector loads", UC, PC);
                end = a.off + a.bytes;
            }
            if (end != y.total) return fail("total does not cover the arrays", UC, PC);
            // the zero padding behind a list of n entries (n rounded up to 4) stays inside its array
            if (((UC + 3) & ~3) > y.sc || ((PC + 3) & ~3) > PC) return fail("padding leaves the array", UC, PC);
        }
    }
    // ---- top-k per level: list slots for any node count
    for (int n = 0; n <= 200000; n += (n < 300 ? 1 : 613)) {
        const int CL = lc_beam_list_slots(n);
        ++cases;
        if (CL % 64 || CL < 64 || CL > LC_BEAM_LIST_MAX) return fail("list slots", n, CL);
        if (n <= LC_BEAM_LIST_MAX && CL < n) return fail("list shorter than the level", n, CL);
        const LcBeamLayout y = lc_beam_layout(CL);
        const int offs[5] = {y.cid, y.nxt, y.key, y.wgt, y.flg};
        const int sizes[5] = {4 * CL, 4 * CL, 4 * CL, 4 * CL, CL};
        int end = 0;
        for (int i = 0; i < 5; ++i) {
            if (offs[i] < end) return fail("beam arrays overlap", n, i);
            if (i >= 2 && i <= 3 && offs[i] % 16) return fail("beam key/weight arrays misaligned", n, i);
            end = offs[i] + sizes[i];
        }
        if (end != y.total || (size_t)y.total > (size_t)LC_WALK_LDS_LIMIT) return fail("beam total", n, y.total);
    }
    std::printf("ok %ld\n", cases);
    return 0;
}
