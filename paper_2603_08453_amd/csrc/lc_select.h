// Budget selection of one (sequence, head) from the chunk score keys, by one workgroup whose lanes
// keep the chunks in registers.  Used by every workgroup of the select+attend kernel of a decode
// step.  (One 1024-thread workgroup per (sequence, head) running it as a kernel of its own behind
// the scoring kernel was measured too: no faster than the last scoring workgroup selecting from
// staged keys -- 12.5 against 11.4 us at 2.3 K chunks per head, 26 against 22 us at 11 K: a single
// compute unit's instruction rate bounds both -- so lc_retrieve keeps the one-kernel form.)
#pragma once

#include "lc_device.h"
#include "lc_internal.h"

#define LC_SEL_CAND 64            // chunks of the cutoff bin that are ranked directly
#define LC_SEL_BINS_MAX 1024      // most bins of the selection histogram

// Workgroup barrier that orders LDS accesses only: global loads issued before it stay in flight
// (a plain __syncthreads() also waits for every outstanding global load of the wavefront).
__device__ __forceinline__ void lc_barrier_lds() {
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup", "local");
    __builtin_amdgcn_s_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup", "local");
}
__device__ __forceinline__ int lc_readlane(int v, int l) { return __builtin_amdgcn_readlane(v, l); }
__device__ __forceinline__ int lc_wave_sum_i(int v) {                       // all 64 lanes active
    return lc_readlane(lc_wave_scan_incl(v), 63);
}

// LDS of the fused step's selection (the general select routine, used when the cutoff bin
// overflows its short list, has its own block)
template <int NT>
struct LcFusedSh {
    int hw[LC_SEL_BINS_MAX + 4];     // chunk lengths per bin; the slot after the last bin takes what is no candidate
    int4 cand[LC_SEL_CAND];          // chunks of the cutoff bin: key, length, id
    int n_cand;
    uint32_t kmin[NT / 64], kmax[NT / 64];
    int wtok[NT / 64], wcnt[NT / 64];
};
// min / max over a wavefront, uniform result: DPP within the four 16-lane rows, then the rows' values by lane reads
__device__ __forceinline__ uint32_t lc_wave_min_uniform(uint32_t v) {
    v = min(v, lc_dpp_u<0xB1>(v)); v = min(v, lc_dpp_u<0x4E>(v));
    v = min(v, lc_dpp_u<0x141>(v)); v = min(v, lc_dpp_u<0x140>(v));
    const uint32_t r0 = (uint32_t)lc_readlane((int)v, 0), r1 = (uint32_t)lc_readlane((int)v, 16);
    const uint32_t r2 = (uint32_t)lc_readlane((int)v, 32), r3 = (uint32_t)lc_readlane((int)v, 48);
    return min(min(r0, r1), min(r2, r3));
}
__device__ __forceinline__ uint32_t lc_wave_max_uniform(uint32_t v) {
    v = max(v, lc_dpp_u<0xB1>(v)); v = max(v, lc_dpp_u<0x4E>(v));
    v = max(v, lc_dpp_u<0x141>(v)); v = max(v, lc_dpp_u<0x140>(v));
    const uint32_t r0 = (uint32_t)lc_readlane((int)v, 0), r1 = (uint32_t)lc_readlane((int)v, 16);
    const uint32_t r2 = (uint32_t)lc_readlane((int)v, 32), r3 = (uint32_t)lc_readlane((int)v, 48);
    return max(max(r0, r1), max(r2, r3));
}
// number of set bits of `mask` below this lane
__device__ __forceinline__ int lc_mbcnt(unsigned long long mask) {
    return (int)__builtin_amdgcn_mbcnt_hi((uint32_t)(mask >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)mask, 0u));
}

// What the selection leaves in every lane: its chunks' first rows, lengths (0 unless selected) and
// token offsets among its wavefront's selected tokens, and the workgroup-wide totals.
template <int EC>
struct LcChunkSel {
    int cst[EC], stok[EC], coff[EC];
    int base_tok;        // selected tokens of the wavefronts before this one
    int n_sel_tok;       // selected tokens of the (sequence, head), without the open tail
    int n_sel;           // selected chunks (only counted when the chunk list is written)
    int tail_st, tail_ln;
    int n_tok;           // n_sel_tok + tail_ln
    int T, M;
};

// Wavefront w owns the chunks [64 EC w, 64 EC (w + 1)), lane l of it the chunks (EC w + e) * 64 + l
// for e < EC, so every load is coalesced and the id order is (wavefront, e, lane): prefix sums in id
// order are EC independent wavefront scans on the vector ALU plus one exchange of the wavefront
// totals.  The loops over e carry no branches, so that the EC copies of each step overlap in the
// pipeline (one wavefront per SIMD has nothing else to hide a dependent instruction's latency behind).
//   1. range of the candidate keys (one exchange), histogram of chunk lengths over it (LDS
//      atomics), every wavefront scans all bins from the top: cutoff bin, budget left for it;
//   2. chunks in bins above the cutoff bin are selected; the few in the cutoff bin go to a short
//      list and their owners rank them against each other (key descending, id ascending) -- or,
//      if the list overflows (a crowded or tied bin), the general select routine runs on them;
//   3. token offsets of the selected chunks by the scans above.
// `keys_all`: [B][H][cap0] score keys (0 = not a candidate); chunks whose first token lies below
// `sink` are pinned: always selected, not charged to the budget.  With `ids_out` (per (sequence,
// head) `cap` entries) the selected ids are also written in ascending order and their number to
// counts_out[bh].  `lds_dyn`: 8 * EC * NT bytes, touched only when the cutoff bin overflows.
// All NT threads must call; NT / 64 wavefronts; holds up to EC * NT chunks.
template <int NT, int EC>
__device__ __forceinline__ void lc_select_chunks(const LcDev& ix, int b, int bh, const uint32_t* keys_all, int budget,
                                                 int sink, int32_t* ids_out, int32_t* counts_out, int cap,
                                                 LcLeafSelSh& sel_sh, LcFusedSh<NT>& fs, int* lds_dyn,
                                                 LcChunkSel<EC>& o) {
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int* bnd = ix.bounds + (size_t)b * (ix.cap[0] + 1);
    o.base_tok = 0;
    o.n_sel_tok = 0;
    o.n_sel = 0;
    // bins of the histogram: about one per four chunks, so that the cutoff bin holds a handful
    constexpr int BITS = EC * NT <= 1024 ? 8 : (EC * NT <= 2560 ? 9 : 10);
    constexpr int BINS = 1 << BITS;
    const int cap0 = ix.cap[0];
    // ---- every load of the selection goes out at once, before the chunk count is known (reads
    // past the arrays' ends return 0; what lies past the count is masked below)
    const __amdgpu_buffer_rsrc_t keys_r = lc_buffer(keys_all + (size_t)bh * cap0, cap0 * 4);
    const __amdgpu_buffer_rsrc_t bnd_r = lc_buffer(bnd, (cap0 + 1) * 4);
    const int j0 = wave * (EC * 64) + lane;                      // this lane's chunk e is j0 + 64 e
    uint32_t ck[EC];
    int cend[EC];
#pragma unroll
    for (int e = 0; e < EC; ++e) {
        ck[e] = (uint32_t)__builtin_amdgcn_raw_buffer_load_b32(keys_r, j0 * 4, e * 256, 0);
        o.cst[e] = __builtin_amdgcn_raw_buffer_load_b32(bnd_r, j0 * 4, e * 256, 0);
        cend[e] = __builtin_amdgcn_raw_buffer_load_b32(bnd_r, j0 * 4, e * 256 + 4, 0);
    }
    o.T = ix.state[bh * 4 + 0];
    const int M_all = ix.state[bh * 4 + 1];
    // meanwhile: empty histograms and list (their first use is behind the barrier of the key range)
    for (int i = tid; i < BINS + 4; i += NT) fs.hw[i] = 0;
    if (tid < LC_SEL_CAND) fs.cand[tid] = make_int4(0, 0, 0, 0);
    if (tid == 0) fs.n_cand = 0;
    o.M = min(M_all, EC * NT);
    o.tail_st = bnd[M_all];
    const int W = budget > 0 ? budget : 0;
    // ---- lengths; what is past the count or pinned is no candidate (key 0), pinned chunks are selected
    int cln[EC];
    uint32_t kmin1 = 0xffffffffu, kmax = 0u;                    // (lowest candidate key) - 1, highest
#pragma unroll
    for (int e = 0; e < EC; ++e) {
        const bool valid = j0 + 64 * e < o.M;
        cln[e] = valid ? max(0, cend[e] - o.cst[e]) : 0;
        const bool pinned = valid && o.cst[e] < sink;
        const int len_p = cln[e];
        o.stok[e] = pinned ? len_p : 0;
        ck[e] = (valid && !pinned) ? ck[e] : 0u;
        kmin1 = min(kmin1, ck[e] - 1u);                         // key 0 wraps to the largest value: ignored
        kmax = max(kmax, ck[e]);
    }
    {
        const uint32_t wmin = lc_wave_min_uniform(kmin1), wmax = lc_wave_max_uniform(kmax);
        if (lane == 0) { fs.kmin[wave] = wmin; fs.kmax[wave] = wmax; }
    }
    lc_barrier_lds();
    kmin1 = fs.kmin[0];
    kmax = fs.kmax[0];
#pragma unroll
    for (int w = 1; w < NT / 64; ++w) { kmin1 = min(kmin1, fs.kmin[w]); kmax = max(kmax, fs.kmax[w]); }
    if (kmax != 0u) {                                           // (uniform) there are candidates
        const uint32_t kmin = kmin1 + 1u;
        const uint32_t span = kmax - kmin;
        const int bits = span ? 32 - __clz(span) : 0;
        const int shift = bits > BITS ? bits - BITS : 0;        // (span >> shift) < BINS
        // bin of every chunk: -1 = no candidate (those add their length to a slot nobody reads)
        int cbin[EC];
#pragma unroll
        for (int e = 0; e < EC; ++e) {
            const int bin = (int)((ck[e] - kmin) >> shift);
            cbin[e] = ck[e] != 0u ? bin : -1;
            const int slot = (int)min((uint32_t)cbin[e], (uint32_t)BINS);
            atomicAdd(&fs.hw[slot], cln[e]);
        }
        lc_barrier_lds();
        // ---- every wavefront scans all bins from the top: lane l holds bins BINS - 1 - PER l - i, i < PER
        constexpr int PER = BINS / 64;
        int fb = -1, remW = W;                                  // cutoff bin (-1: every candidate fits), budget left for it
        {
            int pw[PER];                                        // inclusive prefix sums within the lane, bins descending
            const int4* hw4 = reinterpret_cast<const int4*>(fs.hw + BINS - PER * (lane + 1));
#pragma unroll
            for (int v = 0; v < PER / 4; ++v) {
                const int4 x = hw4[PER / 4 - 1 - v];
                pw[4 * v + 0] = x.w; pw[4 * v + 1] = x.z; pw[4 * v + 2] = x.y; pw[4 * v + 3] = x.x;
            }
#pragma unroll
            for (int i = 1; i < PER; ++i) pw[i] += pw[i - 1];
            const int cw = lc_wave_scan_incl(pw[PER - 1]) - pw[PER - 1];      // length of all higher lanes' bins
            // bins of this lane that still fit (prefix sums grow, so they are the first `fit` ones) and their total
            int fit = 0, fitw = 0;
#pragma unroll
            for (int i = 0; i < PER; ++i) {
                const bool ok = cw + pw[i] <= W;
                fit += ok ? 1 : 0;
                fitw = ok ? pw[i] : fitw;
            }
            const unsigned long long bal = __ballot(fit < PER); // the prefix ends in the first bin that no longer fits
            if (bal != 0ull) {
                const int fl = __ffsll((long long)bal) - 1;     // lowest lane = highest bins
                fb = BINS - 1 - (PER * fl + lc_readlane(fit, fl));
                remW = W - (lc_readlane(cw, fl) + lc_readlane(fitw, fl));
            }
        }
        // ---- chunks above the cutoff bin are in; those in it go to the short list
        unsigned long long cutm[EC];
        unsigned long long anycut = 0ull;
#pragma unroll
        for (int e = 0; e < EC; ++e) {
            const int len_e = cln[e], old_e = o.stok[e];          // (values first: a select of two array slots keeps both arrays in memory)
            o.stok[e] = cbin[e] > fb ? len_e : old_e;
            cutm[e] = __ballot(fb >= 0 && cbin[e] == fb);
            anycut |= cutm[e];
        }
        int cpos[EC];
        if (anycut != 0ull) {                                   // (uniform per wavefront)
            int n_mine = 0;
#pragma unroll
            for (int e = 0; e < EC; ++e) {
                cpos[e] = n_mine + lc_mbcnt(cutm[e]);
                n_mine += __popcll(cutm[e]);
            }
            int base = 0;
            if (lane == 0) base = atomicAdd(&fs.n_cand, n_mine);
            base = lc_readlane(base, 0);
#pragma unroll
            for (int e = 0; e < EC; ++e) {
                cpos[e] += base;
                if (((cutm[e] >> lane) & 1ull) && cpos[e] < LC_SEL_CAND)
                    fs.cand[cpos[e]] = make_int4((int)ck[e], cln[e], j0 + 64 * e, 0);
            }
        }
        lc_barrier_lds();
        const int nc = fs.n_cand;
        if (nc <= LC_SEL_CAND) {
            // ---- each owner ranks its chunk against the list: length and number of the chunks before it
            // (the list is padded with key 0 entries, which come before nothing)
            if (anycut != 0ull) {
#pragma unroll
                for (int e = 0; e < EC; ++e) {
                    if (cutm[e] != 0ull) {                      // (uniform per wavefront)
                        const uint32_t km = ck[e];
                        const int im = j0 + 64 * e;
                        int wb = 0;
                        for (int t = 0; t < nc; t += 4) {
#pragma unroll
                            for (int u = 0; u < 4; ++u) {
                                const int4 o = fs.cand[t + u];
                                const bool before = (uint32_t)o.x > km || ((uint32_t)o.x == km && o.z < im);
                                wb += before ? o.y : 0;
                            }
                        }
                        const int len_e = cln[e], old_e = o.stok[e];
                        const bool in = ((cutm[e] >> lane) & 1ull) && wb + len_e <= remW;
                        o.stok[e] = in ? len_e : old_e;
                    }
                }
            }
        } else {
            // ---- a crowded or tied cutoff bin: the general select routine on its chunks alone
            uint32_t* skey = reinterpret_cast<uint32_t*>(lds_dyn);
            int* slen = lds_dyn + EC * NT;
            lc_leaf_select_prepare<NT>(sel_sh);
            lc_barrier_lds();
            uint32_t bmin = 0xffffffffu, bmax = 0u;
#pragma unroll
            for (int e = 0; e < EC; ++e) {
                const int j = j0 + 64 * e;
                const bool cnd = (cutm[e] >> lane) & 1ull;
                const uint32_t k = cnd ? (ck[e] == 0xffffffffu ? 0xfffffffeu : ck[e]) : 0u;     // the mark is reserved
                skey[j] = k;
                slen[j] = cln[e];
                if (cnd) { bmin = min(bmin, k); bmax = max(bmax, k); }
            }
            lc_leaf_select_range(bmin, bmax, sel_sh);
            lc_barrier_lds();
            const uint32_t thr = lc_leaf_select<NT>(o.M, skey, slen, (long long)remW, 0x7fffffffLL, sel_sh);
            __syncthreads();
#pragma unroll
            for (int e = 0; e < EC; ++e) {
                const int len_e = cln[e], old_e = o.stok[e];
                const bool in = ((cutm[e] >> lane) & 1ull) && skey[j0 + 64 * e] > thr;
                o.stok[e] = in ? len_e : old_e;
            }
        }
    }
    // ---- token offsets in id order: EC independent wavefront scans, their totals chained, then
    // the four wavefront totals
    {
        int inc[EC], tot[EC];
#pragma unroll
        for (int e = 0; e < EC; ++e) inc[e] = lc_wave_scan_incl(o.stok[e]);
#pragma unroll
        for (int e = 0; e < EC; ++e) tot[e] = lc_readlane(inc[e], 63);
        int run = 0;
#pragma unroll
        for (int e = 0; e < EC; ++e) {
            o.coff[e] = run + inc[e] - o.stok[e];
            run += tot[e];
        }
        if (lane == 0) fs.wtok[wave] = run;
    }
    const bool want_ids = ids_out != nullptr;
    int crank[EC];
    if (want_ids) {                                             // (uniform) the same for the chunk counts
        int inc[EC], tot[EC];
#pragma unroll
        for (int e = 0; e < EC; ++e) inc[e] = lc_wave_scan_incl(o.stok[e] > 0 ? 1 : 0);
#pragma unroll
        for (int e = 0; e < EC; ++e) tot[e] = lc_readlane(inc[e], 63);
        int run = 0;
#pragma unroll
        for (int e = 0; e < EC; ++e) {
            crank[e] = run + inc[e] - (o.stok[e] > 0 ? 1 : 0);
            run += tot[e];
        }
        if (lane == 0) fs.wcnt[wave] = run;
    }
    lc_barrier_lds();
#pragma unroll
    for (int w = 0; w < NT / 64; ++w) {
        const int wt = fs.wtok[w];
        if (w < wave) o.base_tok += wt;
        o.n_sel_tok += wt;
    }
    o.tail_ln = max(0, o.T - o.tail_st);
    o.n_tok = o.n_sel_tok + o.tail_ln;
    if (want_ids) {                                             // the chunk list, for callers that want it
        int base_cnt = 0;
#pragma unroll
        for (int w = 0; w < NT / 64; ++w) {
            const int wc = fs.wcnt[w];
            if (w < wave) base_cnt += wc;
            o.n_sel += wc;
        }
        int32_t* io = ids_out + (size_t)bh * cap;
#pragma unroll
        for (int e = 0; e < EC; ++e) {
            const int r = base_cnt + crank[e];
            if (o.stok[e] > 0 && r < cap) io[r] = j0 + 64 * e;
        }
        if (tid == 0 && counts_out != nullptr) counts_out[bh] = min(o.n_sel, cap);
    }
}
