// LDS layouts of the two level-walk kernels, as plain functions of the launch parameters: the
// kernels carve their dynamic LDS with them, the launchers size it with them, and a host-side test
// enumerates the parameters the launchers can produce and checks every array's extent and alignment.
// Plain C++ (no HIP types), so that the test can compile it with the host compiler alone.
#pragma once

#include <stddef.h>

#ifdef __HIPCC__
#define LC_LAYOUT_FN __host__ __device__ inline
#else
#define LC_LAYOUT_FN inline
#endif

#define LC_WALK_LDS_LIMIT (150 * 1024)    // dynamic LDS a walking workgroup may take (a gfx950 workgroup has 160 KiB)

// ---- exact walk (lc_upper_kernel).  UC = slots for internal nodes (all levels of one (sequence,
// head) together), PC = slots of the probe chunk list; both multiples of 64.  Offsets in bytes.
struct LcUpperLayout {
    int sc;          // entries of each of the four select staging buffers
    int ukey, untok, upar, kp;             // per internal node: key, subtree tokens, parent, kept flag (1 byte)
    int ekA, ewA, ekB, ewB;                // two (key, weight) staging buffers; the tau step parks PC flag bytes in ekA
    int plist, plen, pkey;                 // probe chunks: id, length, key
    int total;
};
LC_LAYOUT_FN int lc_upper_scratch_entries(int UC, int PC) {
    const int q = ((PC / 4 + 63) / 64) * 64;            // PC flag bytes must fit the first staging buffer
    return UC > q ? UC : q;
}
LC_LAYOUT_FN LcUpperLayout lc_upper_layout(int UC, int PC) {
    LcUpperLayout y;
    y.sc = lc_upper_scratch_entries(UC, PC);
    int o = 0;
    y.ukey = o; o += 4 * UC;
    y.untok = o; o += 4 * UC;
    y.upar = o; o += 4 * UC;
    y.kp = o; o += UC;
    y.ekA = o; o += 4 * y.sc;
    y.ewA = o; o += 4 * y.sc;
    y.ekB = o; o += 4 * y.sc;
    y.ewB = o; o += 4 * y.sc;
    y.plist = o; o += 4 * PC;
    y.plen = o; o += 4 * PC;
    y.pkey = o; o += 4 * PC;
    y.total = o;
    return y;
}
LC_LAYOUT_FN size_t lc_upper_lds_bytes(int UC, int PC) { return (size_t)lc_upper_layout(UC, PC).total; }

// What the launcher does with the node and chunk counts of the batch: slots for the internal
// nodes, then as long a probe list as fits beside them.  Returns false if even the shortest list
// does not fit (the caller answers with LC_ERR_CAPACITY or a flat scan before any launch).
LC_LAYOUT_FN bool lc_upper_launch_shape(int max_upper, int max_M, int* UC, int* PC) {
    int uc = ((max_upper > 0 ? max_upper : 0) + 63) / 64 * 64;
    if (uc < 64) uc = 64;
    int pc = ((max_M > 0 ? max_M : 0) + 63) / 64 * 64;
    if (pc < 64) pc = 64;
    while (pc > 64 && lc_upper_lds_bytes(uc, pc) > (size_t)LC_WALK_LDS_LIMIT) pc -= 64;
    *UC = uc;
    *PC = pc;
    return lc_upper_lds_bytes(uc, pc) <= (size_t)LC_WALK_LDS_LIMIT;
}
// Most internal nodes of one (sequence, head) that the exact walk holds in LDS.
LC_LAYOUT_FN int lc_upper_max_internal_nodes() {
    int uc = 64;
    while (lc_upper_lds_bytes(uc + 64, 64) <= (size_t)LC_WALK_LDS_LIMIT) uc += 64;
    return uc;
}

// ---- top-k per level (lc_beam_kernel).  CL = slots of each candidate list, a multiple of 64.
struct LcBeamLayout {
    int cid, nxt, key, wgt, flg;           // candidate ids (two lists), keys, weights, kept flags (1 byte each)
    int total;
};
#define LC_BEAM_LIST_MAX 4096             // longer candidate lists go to the workspace
LC_LAYOUT_FN LcBeamLayout lc_beam_layout(int CL) {
    LcBeamLayout y;
    int o = 0;
    y.cid = o; o += 4 * CL;
    y.nxt = o; o += 4 * CL;
    y.key = o; o += 4 * CL;
    y.wgt = o; o += 4 * CL;
    y.flg = o; o += CL;
    y.total = o;
    return y;
}
LC_LAYOUT_FN int lc_beam_list_slots(int max_nodes) {
    int cl = ((max_nodes > 0 ? max_nodes : 1) + 63) / 64 * 64;
    return cl > LC_BEAM_LIST_MAX ? LC_BEAM_LIST_MAX : cl;
}
