// Retrieval kernels: Eq. 2 node scoring, level-by-level pruning, budget selection.
//
// lc_upper_kernel (EXACT policy with the level walk on): one workgroup per (sequence, KV head).
// It stages the internal nodes' small arrays (parents, subtree token counts) in LDS with a few
// batched loads, scores every internal node (levels >= 1), and walks the levels top-down with
// the frontier held in LDS: a probe pass gives a lower bound tau0 of the selection cutoff, the
// verify pass keeps every node whose bound reaches tau0.  It leaves one byte per level-1 node:
// score the chunks below it or not.
//
// lc_beam_kernel (BEAM policy, Algorithm 1): one workgroup per (sequence, KV head) does the whole
// retrieval -- per level score the candidates, keep the beam[l] best, gather their children; at
// the chunk level cut by the token budget and write the ids.
//
// lc_leaf_kernel (lc_retrieve, and the decode step beyond what its selecting workgroups hold):
// many workgroups per (sequence, KV head) score the wanted chunks; the last workgroup to finish
// for a (sequence, head) pulls the keys into LDS, runs the weighted histogram select (weights =
// chunk lengths) and emits the ids in ascending order.
//
// lc_score_kernel (first kernel of a decode step): the scoring half of lc_leaf_kernel alone.
//
// The kernels are latency-bound at batch 1, so global loads are issued in batches
// and nothing reads global memory element by element inside a dependent loop.
#include "lc_device.h"
#include "lc_internal.h"
#include "lc_walk_layout.h"

#define LC_TAU_SLACK 1e-3f
#define LC_COUNT_SELECT_MAX 1024         // up to this many candidates the O(n^2 / threads) rank is used


struct LcRetrieveArgs {
    LcDev ix;
    const uint16_t* q;       // [B][H_q][d]
    uint32_t* keys;          // [B][H][cap0]
    uint8_t* want;           // [B][H][cap0], first N_1 entries used: 1 = this level-1 node was kept, i.e. the
                             // chunks below it are to be scored (the chunk kernel looks its chunks' parents up)
    float* scores;           // [B][H][cap0] or null
    int32_t* ids;            // [B][H][cap]
    int32_t* counts;         // [B][H]
    int* scratch;            // [B][H][4 * cap0] ints: chunk-level staging when it does not fit in LDS
    int cap;
    int budget;
    int policy;
    int sink;
    int beam[LC_MAX_LEVELS];
    int upper_cap;           // LDS entries for internal nodes
    int walk;                // 1 = the internal levels were walked and `want` is valid
    int chunk_cap;           // upper kernel: LDS entries of the probe list; leaf kernel: LDS entries for
                             // the select's staging, 0 = stage in `scratch` (global memory)
    int score_only;          // 1 = only the score keys are wanted (lc_score_kernel; the fused decode step selects)
};

// Selection among n <= LC_COUNT_SELECT_MAX candidates whose keys / weights sit in 16-byte aligned,
// zero-padded LDS arrays.
//   mode 0: keep the longest prefix with weight <= W and count <= C  (exact ties by index)
//   mode 1: keep the shortest prefix whose weight reaches W (everything if it never does)
// Writes flags[i] for i < n.  With REDUCE it also returns, in every thread, the smallest kept key
// (0 if nothing kept) and whether the kept weight reached W (mode 1); that costs three barriers.
template <int NT, bool REDUCE>
__device__ __forceinline__ void lc_small_select(int n, int mode, long long W, long long C, const uint32_t* keys,
                                                const int* wgts, uint8_t* flags, int* sh, uint32_t* min_kept,
                                                int* reached) {
    uint32_t mk = 0xffffffffu;
    int hit = 0;
    const int part = threadIdx.x & 15;
    for (int base = 0; base < n; base += NT / 16) {           // NT/16 items per round, 16 lanes each
        const int i = base + (threadIdx.x >> 4);
        const uint32_t ki = i < n ? keys[i] : 0u;
        int cb, wb;
        lc_rank_before16(ki != 0u ? n : 0, keys, wgts, i, ki, part, &cb, &wb);
        int keep = 0;
        if (ki != 0u) {
            const int wi = wgts[i];
            if (mode == 0) keep = ((long long)wb + wi <= W && (long long)cb + 1 <= C) ? 1 : 0;
            else {
                keep = ((long long)wb < W) ? 1 : 0;
                if (keep && (long long)wb + wi >= W) hit = 1;
            }
        }
        if (part == 0 && i < n) flags[i] = (uint8_t)keep;
        if (keep) mk = min(mk, ki);
    }
    if (!REDUCE) {                   // flags only: the caller synchronises before it reads them
        *min_kept = 0u;
        *reached = 0;
        return;
    }
    mk = lc_wave_min_u(mk);
    hit = (int)lc_wave_max_u((uint32_t)(hit != 0));
    __syncthreads();
    if ((threadIdx.x & 63) == 0) { sh[threadIdx.x >> 6] = (int)mk; sh[32 + (threadIdx.x >> 6)] = hit; }
    __syncthreads();
#pragma unroll
    for (int w = 0; w < NT / 64; ++w) { mk = min(mk, (uint32_t)sh[w]); hit |= sh[32 + w]; }
    __syncthreads();
    *min_kept = (mk == 0xffffffffu) ? 0u : mk;
    *reached = hit;
}

// ---------------------------------------------------------------------------------
// lc_upper_kernel: internal levels (EXACT walk)
// ---------------------------------------------------------------------------------
// (LDS layout: lc_walk_layout.h: 13 bytes per internal-node slot, 16 per select-scratch slot, 12 per probe-list slot)

// One workgroup of 1024 threads (64 groups of 16 lanes) per (sequence, head).  All
// global loads of a phase are issued before any of them is used: at batch 1 the
// kernel's duration is a chain of memory round trips, not bandwidth.
#define LC_UP_THREADS 1024
#define LC_UP_GROUPS (LC_UP_THREADS / 16)
#define LC_UP_PER_THREAD 4

template <int G>
__global__ void __launch_bounds__(LC_UP_THREADS)
lc_upper_kernel(const LcRetrieveArgs a) {
    extern __shared__ int lds_dyn[];
    __shared__ int sel_sh[LC_SEL_SH];
    __shared__ int off_sh[LC_MAX_LEVELS + 1];
    constexpr int NB = (G <= 4) ? 4 : 2;          // nodes in flight per group

    const LcDev& ix = a.ix;
    const int h = blockIdx.x, b = blockIdx.y;
    const int bh = b * ix.H + h;
    const int tid = threadIdx.x;
    const int sub = tid & 15, grp = tid >> 4;
    const int L = ix.L;
    const int M = ix.state[bh * 4 + 1];

    if (tid == 0) {
        int o = 0;
        for (int l = 1; l < L; ++l) { off_sh[l] = o; o += ix.nlev[b * LC_MAX_LEVELS + l]; }
        off_sh[L] = o;
        off_sh[0] = 0;
    }
    // LDS carve-up: internal nodes (UC entries each), select scratch, probe list (PC entries each)
    const int UC = a.upper_cap, PC = a.chunk_cap;
    const LcUpperLayout ly = lc_upper_layout(UC, PC);
    char* const lds_b = reinterpret_cast<char*>(lds_dyn);
    uint32_t* ukey = reinterpret_cast<uint32_t*>(lds_b + ly.ukey);
    int* untok = reinterpret_cast<int*>(lds_b + ly.untok);
    int* upar = reinterpret_cast<int*>(lds_b + ly.upar);
    uint8_t* kp = reinterpret_cast<uint8_t*>(lds_b + ly.kp);
    // two (key, weight) staging buffers for the per-level selects, used alternately
    uint32_t* ekA = reinterpret_cast<uint32_t*>(lds_b + ly.ekA);
    int* ewA = reinterpret_cast<int*>(lds_b + ly.ewA);
    uint32_t* ekB = reinterpret_cast<uint32_t*>(lds_b + ly.ekB);
    int* ewB = reinterpret_cast<int*>(lds_b + ly.ewB);
    int* plist = reinterpret_cast<int*>(lds_b + ly.plist);
    int* plen = reinterpret_cast<int*>(lds_b + ly.plen);
    uint32_t* pkey = reinterpret_cast<uint32_t*>(lds_b + ly.pkey);

    // Query fragments: widened once for small groups; for large ones kept as packed bfloat16 words
    // and widened per node, which keeps this 1024-thread kernel within its 128 registers per lane.
    constexpr bool QP = G > 4;
    float qf[QP ? 1 : G][8], qn[G];
    uint32_t qp[QP ? G : 1][4];
    if constexpr (QP) lc_load_query_packed<G>(a.q + (size_t)b * ix.H * G * LC_D, h, sub, qp, qn);
    else lc_load_query_frags<G>(a.q + (size_t)b * ix.H * G * LC_D, h, sub, qf, qn);
    auto score_node = [&](const LcNodeFrag& f, float R) -> float {
        if constexpr (QP) return lc_score_frag_packed<G>(f, R, qp, qn);
        else return lc_score_frag<G>(f, R, qf, qn);
    };
    // prefetch what the chunk pass will need much later (parents and boundaries of this thread's
    // first LC_UP_PER_THREAD chunks): the arrays are cap[0] long, so no count is needed to load them
    int pf_p[LC_UP_PER_THREAD], pf_s[LC_UP_PER_THREAD + 1];
    {
        const int* bnd_e = ix.bounds + (size_t)b * (ix.cap[0] + 1);
        const int* par_e = ix.parent[0] + (size_t)bh * ix.cap[0];
        const int j0 = tid * LC_UP_PER_THREAD;
#pragma unroll
        for (int k = 0; k < LC_UP_PER_THREAD; ++k) pf_p[k] = par_e[min(j0 + k, ix.cap[0] - 1)];
#pragma unroll
        for (int k = 0; k <= LC_UP_PER_THREAD; ++k) pf_s[k] = bnd_e[min(j0 + k, ix.cap[0])];
    }
    __syncthreads();
    const int NU = off_sh[L];

    // ---- internal nodes, all levels as one list: parents, token counts, scores
    auto level_of = [&](int u) -> int {
        int l = 1;
        while (l + 1 < L && u >= off_sh[l + 1]) ++l;
        return l;
    };
    for (int u = tid; u < NU; u += LC_UP_THREADS) {
        const int l = level_of(u);
        const size_t n = (size_t)bh * ix.cap[l] + (u - off_sh[l]);
        untok[u] = ix.ntok[l][n];
        upar[u] = ix.parent[l][n];
    }
    for (int u0 = grp; u0 < NU; u0 += NB * LC_UP_GROUPS) {
        LcNodeFrag f[NB];
        float R[NB];
        int nc[NB];
#pragma unroll
        for (int k = 0; k < NB; ++k) {
            const int u = min(u0 + k * LC_UP_GROUPS, NU - 1);
            const int l = level_of(u);
            const size_t n = (size_t)bh * ix.cap[l] + (u - off_sh[l]);
            f[k] = lc_load_node(ix.center[l] + n * LC_D, sub);
            R[k] = ix.radius[l][n];
            nc[k] = ix.nchunk[l][n];
        }
#pragma unroll
        for (int k = 0; k < NB; ++k) {
            const int u = u0 + k * LC_UP_GROUPS;
            float s = score_node(f[k], R[k]);
            if (nc[k] <= 0) s = LC_NEG_INF;
            if (sub == 0 && u < NU) ukey[u] = lc_score_key(s);
        }
    }
    __syncthreads();

    uint8_t* want = a.want + (size_t)bh * ix.cap[0];
    const int* bnd = ix.bounds + (size_t)b * (ix.cap[0] + 1);
    const int* par0 = ix.parent[0] + (size_t)bh * ix.cap[0];
    const int o1 = off_sh[1];
    const int n_1 = (L > 2 ? off_sh[2] : off_sh[L]) - o1;
    if (a.budget <= 0) {
        for (int i = tid; i < n_1; i += LC_UP_THREADS) want[i] = 0;
        return;
    }

    // the outcome of the walk: which level-1 nodes were kept (the chunk kernel maps chunks to them)
    auto write_want = [&]() {
        for (int i = tid; i < n_1; i += LC_UP_THREADS) want[i] = kp[o1 + i];
    };
    // Per-level selection.  The candidates of a level (frontier nodes: key, weight; others: 0) sit in
    // one staging buffer; the select writes kept flags; the children of the kept nodes are staged into
    // the other buffer for the next level.  Two barriers per level.
    uint32_t* ek = ekA;
    int* ew = ewA;
    uint32_t* ek_next = ekB;
    int* ew_next = ewB;
    const bool with_tokens = true;
    {
        const int o = off_sh[L - 1], n_l = off_sh[L] - o;
        for (int i = tid; i < ((n_l + 3) & ~3); i += LC_UP_THREADS) {
            ek[i] = i < n_l ? ukey[o + i] : 0u;
            ew[i] = (i < n_l && with_tokens) ? untok[o + i] : 0;
        }
        __syncthreads();
    }
    for (int l = L - 1; l >= 1; --l) {
        const int o = off_sh[l], n_l = off_sh[l + 1] - o;
        uint32_t mk;
        int reached;
        {
            // EXACT, probe pass: keep the best frontier nodes until their subtree token counts reach the budget
            if (n_l <= LC_COUNT_SELECT_MAX) {
                lc_small_select<LC_UP_THREADS, false>(n_l, 1, (long long)a.budget, 0x7fffffffLL, ek, ew, kp + o, sel_sh, &mk, &reached);
            } else {
                auto keyf = [&](int i) -> uint32_t { return ek[i]; };
                auto wf = [&](int i) -> int { return ew[i]; };
                const LcSel r = lc_block_select<LC_UP_THREADS>(n_l, (long long)a.budget - 1, 0x7fffffffLL, keyf, wf, sel_sh);
                for (int i = tid; i < n_l; i += LC_UP_THREADS)
                    kp[o + i] = (ek[i] != 0u && (r.all || ek[i] >= r.kstar)) ? 1 : 0;      // whole tie group
            }
        }
        __syncthreads();
        if (l >= 2) {                 // stage the children of the kept nodes as the next level's candidates
            const int ob = off_sh[l - 1], n_b = off_sh[l] - ob;
            for (int n = tid; n < ((n_b + 3) & ~3); n += LC_UP_THREADS) {
                const bool in = n < n_b && kp[o + upar[ob + n]];
                ek_next[n] = in ? ukey[ob + n] : 0u;
                ew_next[n] = (in && with_tokens) ? untok[ob + n] : 0;
            }
            __syncthreads();
            uint32_t* tk = ek; ek = ek_next; ek_next = tk;
            int* tw = ew; ew = ew_next; ew_next = tw;
        }
    }
    // ---- compact the probe's chunks (children of the kept level-1 nodes, not pinned) into LDS.
    // The list holds at most PC chunks; dropping the rest only weakens tau0, never the result.
    int n_probe = 0;
    for (int base = 0; base < M; base += LC_UP_THREADS * LC_UP_PER_THREAD) {
        const int j0 = base + tid * LC_UP_PER_THREAD;
        int p[LC_UP_PER_THREAD], s0[LC_UP_PER_THREAD + 1];
        if (base == 0) {
#pragma unroll
            for (int k = 0; k < LC_UP_PER_THREAD; ++k) p[k] = pf_p[k];
#pragma unroll
            for (int k = 0; k <= LC_UP_PER_THREAD; ++k) s0[k] = pf_s[k];
        } else {
#pragma unroll
            for (int k = 0; k < LC_UP_PER_THREAD; ++k) p[k] = par0[max(0, min(j0 + k, M - 1))];
#pragma unroll
            for (int k = 0; k <= LC_UP_PER_THREAD; ++k) s0[k] = bnd[min(j0 + k, M)];
        }
        int f[LC_UP_PER_THREAD], cnt = 0;
#pragma unroll
        for (int k = 0; k < LC_UP_PER_THREAD; ++k) {
            f[k] = (j0 + k < M && s0[k] >= a.sink && kp[o1 + p[k]]) ? 1 : 0;
            cnt += f[k];
        }
        int tot;
        int pos = n_probe + lc_block_scan<LC_UP_THREADS>(cnt, sel_sh, &tot);
#pragma unroll
        for (int k = 0; k < LC_UP_PER_THREAD; ++k) {
            if (f[k]) {
                if (pos < PC) { plist[pos] = j0 + k; plen[pos] = s0[k + 1] - s0[k]; }
                ++pos;
            }
        }
        n_probe += tot;
    }
    n_probe = min(n_probe, PC);
    __syncthreads();
    // ---- score them
    {
        const size_t cb = (size_t)bh * ix.cap[0];
        const bool c0b = ix.c0_bf16 != 0;
        for (int i0 = grp; i0 < n_probe; i0 += NB * LC_UP_GROUPS) {
            LcNodeFrag f[NB];
            float R[NB];
#pragma unroll
            for (int k = 0; k < NB; ++k) {
                const int j = plist[min(i0 + k * LC_UP_GROUPS, n_probe - 1)];
                f[k] = lc_load_chunk_node(ix.center[0], c0b, cb + j, sub);
                R[k] = ix.radius[0][cb + j];
            }
#pragma unroll
            for (int k = 0; k < NB; ++k) {
                const int i = i0 + k * LC_UP_GROUPS;
                const float s = score_node(c0b ? lc_widen_chunk_frag(f[k]) : f[k], R[k]);
                if (sub == 0 && i < n_probe) pkey[i] = lc_score_key(s);
            }
        }
        // zero padding for the vector reads of the select
        if (tid < 4 && n_probe + tid < ((n_probe + 3) & ~3)) { pkey[n_probe + tid] = 0u; plen[n_probe + tid] = 0; }
    }
    __syncthreads();
    // ---- tau0: the score at which the probe chunks' cumulative length reaches the budget
    uint32_t tau_key = 1u;                  // keep everything unless the probe proves a cutoff
    {
        uint32_t cut = 0u;
        int reached = 0;
        if (n_probe <= LC_COUNT_SELECT_MAX) {
            lc_small_select<LC_UP_THREADS, true>(n_probe, 1, (long long)a.budget, 0x7fffffffLL, pkey, plen,
                                                 reinterpret_cast<uint8_t*>(ekA), sel_sh, &cut, &reached);
        } else {
            auto keyf = [&](int i) -> uint32_t { return pkey[i]; };
            auto wf = [&](int i) -> int { return plen[i]; };
            const LcSel r = lc_block_select<LC_UP_THREADS>(n_probe, (long long)a.budget - 1, 0x7fffffffLL, keyf, wf, sel_sh);
            reached = r.all ? 0 : 1;
            cut = r.kstar;
        }
        if (reached && cut != 0u) {
            const float tau = lc_key_score(cut);
            tau_key = lc_score_key(tau - LC_TAU_SLACK * fmaxf(1.0f, fabsf(tau)));
            if (tau_key == 0u) tau_key = 1u;
        }
    }
    // ---- verify pass: keep every node whose bound reaches tau0 and whose parent was kept
    {
        const int o = off_sh[L - 1], n_l = off_sh[L] - o;
        for (int i = tid; i < n_l; i += LC_UP_THREADS) kp[o + i] = (ukey[o + i] >= tau_key) ? 1 : 0;
        __syncthreads();
    }
    for (int l = L - 2; l >= 1; --l) {
        const int o = off_sh[l], n_l = off_sh[l + 1] - o, oa = off_sh[l + 1];
        for (int i = tid; i < n_l; i += LC_UP_THREADS)
            kp[o + i] = (ukey[o + i] >= tau_key && kp[oa + upar[o + i]]) ? 1 : 0;
        __syncthreads();
    }
    write_want();
}


// ---------------------------------------------------------------------------------
// top-k per level (Algorithm 1): the whole retrieval in one workgroup per (sequence, head)
// ---------------------------------------------------------------------------------
// Only the children of the kept nodes are ever scored, so the work follows the beam sizes, not the
// size of the index: per level, score the candidate list (ascending node order, so that equal
// scores fall to the lower id), rank it, mark the kept nodes in a bitmap, gather their children.
// The chunks under the kept level-1 nodes are scored the same way, cut by the token budget (and the
// chunk-count limit beam[0]) and written out in ascending order behind the pinned chunks.
// The lists live in LDS while a level's candidates number at most `chunk_cap`; a longer list goes
// to the workspace (same code through generic pointers, slower).
#define LC_BM_THREADS 1024
#define LC_BM_GROUPS (LC_BM_THREADS / 16)
#define LC_BM_KEPT_WORDS 2048             // kept bitmap: up to 65536 nodes per internal level
#define LC_BM_MAX_LEVEL_NODES (LC_BM_KEPT_WORDS * 32)
#define LC_BM_PF 4                       // chunks per thread whose parent and boundary are fetched at kernel start
#define LC_BM_RANK_MAX 128               // chunk lists up to this length are ranked directly, longer ones by histogram


template <int G>
__global__ void __launch_bounds__(LC_BM_THREADS)
lc_beam_kernel(const LcRetrieveArgs a) {
    extern __shared__ int lds_dyn[];
    __shared__ LcLeafSelSh leaf_sh;
    __shared__ int sel_sh[LC_SEL_SH];
    __shared__ uint32_t kept[LC_BM_KEPT_WORDS];
    constexpr int NB = G <= 6 ? 2 : 1;            // nodes in flight per group (the lists are short; 128 registers per lane)

    const LcDev& ix = a.ix;
    const int h = blockIdx.x, b = blockIdx.y;
    const int bh = b * ix.H + h;
    const int tid = threadIdx.x;
    const int sub = tid & 15, grp = tid >> 4;
    const int L = ix.L;
    const int cap0 = ix.cap[0];
    const int M = min(ix.state[bh * 4 + 1], cap0);
    const int* bnd = ix.bounds + (size_t)b * (cap0 + 1);

    // candidate lists: ids of the current level, ids of the next, keys, weights, kept flags
    const int CL = a.chunk_cap;
    const LcBeamLayout ly = lc_beam_layout(CL);
    char* const lds_b = reinterpret_cast<char*>(lds_dyn);
    int* const l_cid = reinterpret_cast<int*>(lds_b + ly.cid);
    int* const l_nxt = reinterpret_cast<int*>(lds_b + ly.nxt);
    uint32_t* const l_key = reinterpret_cast<uint32_t*>(lds_b + ly.key);
    int* const l_wgt = reinterpret_cast<int*>(lds_b + ly.wgt);
    uint8_t* const l_flg = reinterpret_cast<uint8_t*>(lds_b + ly.flg);
    int* const gs = a.scratch + (size_t)bh * 4 * cap0;
    int* const g_cid = gs;
    int* const g_nxt = gs + cap0;
    uint32_t* const g_key = reinterpret_cast<uint32_t*>(gs + 2 * cap0);
    int* const g_wgt = gs + 3 * cap0;
    uint8_t* const g_flg = a.want + (size_t)bh * cap0;

    constexpr bool QP = G > 2;                   // (see lc_upper_kernel; this kernel waits for memory, not for the ALU)
    float qf[QP ? 1 : G][8], qn[G];
    uint32_t qp[QP ? G : 1][4];
    if constexpr (QP) lc_load_query_packed<G>(a.q + (size_t)b * ix.H * G * LC_D, h, sub, qp, qn);
    else lc_load_query_frags<G>(a.q + (size_t)b * ix.H * G * LC_D, h, sub, qf, qn);
    auto score_node = [&](const LcNodeFrag& f, float R) -> float {
        if constexpr (QP) return lc_score_frag_packed<G>(f, R, qp, qn);
        else return lc_score_frag<G>(f, R, qf, qn);
    };

    // What the chunk stage will need much later -- parents and boundaries of this thread's first
    // LC_BM_PF chunks (thread t looks at the chunks [t E, t E + E), E = ceil(M / threads)) -- is
    // fetched now: the arrays are cap0 long, so only the count has to arrive first.
    const int* par0 = ix.parent[0] + (size_t)bh * cap0;
    const int EM = (M + LC_BM_THREADS - 1) / LC_BM_THREADS;
    const int j_lo = min(M, tid * EM), j_hi = min(M, j_lo + EM);
    int pf_p[LC_BM_PF], pf_s[LC_BM_PF];
#pragma unroll
    for (int k = 0; k < LC_BM_PF; ++k) {
        const int j = min(j_lo + k, cap0 - 1);
        pf_p[k] = L > 1 ? par0[j] : 0;
        pf_s[k] = bnd[j];
    }

    // optional score output: everything that is never scored reads -inf
    float* scores = a.scores ? a.scores + (size_t)bh * cap0 : nullptr;
    if (scores)
        for (int j = tid; j < M; j += LC_BM_THREADS) scores[j] = LC_NEG_INF;

    // ---- top level: every node is a candidate
    int n_c = L > 1 ? ix.nlev[b * LC_MAX_LEVELS + (L - 1)] : 0;
    bool in_lds = n_c <= CL;
    int* cid = in_lds ? l_cid : g_cid;
    for (int i = tid; i < n_c; i += LC_BM_THREADS) cid[i] = i;
    __syncthreads();

    for (int l = L - 1; l >= 1; --l) {
        uint32_t* key = in_lds ? l_key : g_key;
        int* wgt = in_lds ? l_wgt : g_wgt;
        uint8_t* flg = in_lds ? l_flg : g_flg;
        // ---- score the candidates of this level
        for (int i0 = grp; i0 < n_c; i0 += NB * LC_BM_GROUPS) {
            LcNodeFrag f[NB];
            float R[NB];
            int nc[NB];
#pragma unroll
            for (int k = 0; k < NB; ++k) {
                const size_t n = (size_t)bh * ix.cap[l] + cid[min(i0 + k * LC_BM_GROUPS, n_c - 1)];
                f[k] = lc_load_node(ix.center[l] + n * LC_D, sub);
                R[k] = ix.radius[l][n];
                nc[k] = ix.nchunk[l][n];
            }
#pragma unroll
            for (int k = 0; k < NB; ++k) {
                const int i = i0 + k * LC_BM_GROUPS;
                float sc = score_node(f[k], R[k]);
                if (nc[k] <= 0) sc = LC_NEG_INF;
                if (sub == 0 && i < n_c) { key[i] = lc_score_key(sc); wgt[i] = 0; }
            }
        }
        if (in_lds && tid < 4 && n_c + tid < ((n_c + 3) & ~3)) { key[n_c + tid] = 0u; wgt[n_c + tid] = 0; }
        __syncthreads();
        // ---- keep the beam[l] best
        const long long C = a.beam[l] > 0 ? a.beam[l] : 0x7fffffffLL;
        if (in_lds && n_c <= LC_COUNT_SELECT_MAX) {
            uint32_t mk;
            int reached;
            lc_small_select<LC_BM_THREADS, false>(n_c, 0, 0x7fffffffffffLL, C, key, wgt, flg, sel_sh, &mk, &reached);
        } else {
            auto keyf = [&](int i) -> uint32_t { return key[i]; };
            auto wf = [&](int) -> int { return 0; };
            const LcSel r = lc_block_select<LC_BM_THREADS>(n_c, 0x7fffffffffffLL, C, keyf, wf, sel_sh);
            int tie_c = 0;
            for (int t0 = 0; t0 < n_c; t0 += LC_BM_THREADS) {
                const int i = t0 + tid;
                const uint32_t k = (i < n_c) ? key[i] : 0u;
                const int eq = (!r.all && k != 0u && k == r.kstar) ? 1 : 0;
                int tot;
                const int ex = lc_block_scan<LC_BM_THREADS>(eq, sel_sh, &tot);
                if (i < n_c) flg[i] = (k != 0u && (k > r.kstar || (eq && tie_c + ex + 1 <= r.remC))) ? 1 : 0;
                tie_c += tot;
            }
        }
        // ---- bitmap of the kept nodes
        const int n_l = ix.nlev[b * LC_MAX_LEVELS + l];
        for (int i = tid; i < (n_l + 31) / 32; i += LC_BM_THREADS) kept[i] = 0u;
        __syncthreads();
        for (int i = tid; i < n_c; i += LC_BM_THREADS)
            if (flg[i]) atomicOr(&kept[cid[i] >> 5], 1u << (cid[i] & 31));
        __syncthreads();
        if (l == 1) break;
        // ---- the kept nodes' children, in ascending order: count them, pick where the list goes, write it
        const int n_b = ix.nlev[b * LC_MAX_LEVELS + (l - 1)];
        const int* par = ix.parent[l - 1] + (size_t)bh * ix.cap[l - 1];
        auto is_child = [&](int i) -> int {
            if (i >= n_b) return 0;
            const int p = par[i];
            return (p >= 0 && p < n_l && ((kept[p >> 5] >> (p & 31)) & 1u)) ? 1 : 0;
        };
        // (thread t looks at the nodes [t E, t E + E): one count, one scan, one write pass.  The parent
        // pointers are fetched in batches of eight with no branch around the loads -- a memory round
        // trip per batch, not per node -- and the verdicts of the first 32 nodes stay in a register mask.)
        const int E = (n_b + LC_BM_THREADS - 1) / LC_BM_THREADS;
        const int i_lo = min(n_b, tid * E), i_hi = min(n_b, i_lo + E);
        const int i_last = max(n_b - 1, 0);
        unsigned vmask = 0u;
        const int E_b = E > 4 ? min(E, 32) : 0;                   // short runs: node by node below
        for (int k0 = 0; k0 < E_b; k0 += 8) {
            int pv[8];
#pragma unroll
            for (int k = 0; k < 8; ++k) pv[k] = par[min(i_lo + k0 + k, i_last)];
#pragma unroll
            for (int k = 0; k < 8; ++k) {
                const int pp = pv[k];
                const bool in = i_lo + k0 + k < i_hi && pp >= 0 && pp < n_l;
                const uint32_t w = kept[in ? pp >> 5 : 0];
                vmask |= (in && ((w >> (pp & 31)) & 1u)) ? 1u << (k0 + k) : 0u;
            }
        }
        int n_new = 0, mine = __popc(vmask);
        for (int i = i_lo + E_b; i < i_hi; ++i) mine += is_child(i);
        int pos = lc_block_scan<LC_BM_THREADS>(mine, sel_sh, &n_new);
        const bool nxt_lds = n_new <= CL;
        int* nxt = nxt_lds ? (cid == l_cid ? l_nxt : l_cid) : (cid == g_cid ? g_nxt : g_cid);
        if (mine > 0) {
            while (vmask != 0u) {
                nxt[pos++] = i_lo + __ffs((int)vmask) - 1;
                vmask &= vmask - 1u;
            }
            for (int i = i_lo + E_b; i < i_hi; ++i)
                if (is_child(i)) nxt[pos++] = i;
        }
        __syncthreads();
        cid = nxt;
        in_lds = nxt_lds;
        n_c = n_new;
    }

    // ---- chunks: children of the kept level-1 nodes (every chunk if the index has no level above
    // them), without the pinned ones; the pinned chunks are the leading ones and are counted here
    const int W = a.budget > 0 ? a.budget : 0;
    const int n_1 = L > 1 ? ix.nlev[b * LC_MAX_LEVELS + 1] : 0;
    auto chunk_state_of = [&](int j, int start, int p) -> int {        // 0 = not a candidate, 1 = candidate, 2 = pinned
        if (j >= M) return 0;
        if (start < a.sink) return 2;
        if (W <= 0) return 0;
        if (L == 1) return 1;
        return (p >= 0 && p < n_1 && ((kept[p >> 5] >> (p & 31)) & 1u)) ? 1 : 0;
    };
    auto chunk_state = [&](int j) -> int { return j < M ? chunk_state_of(j, bnd[j], L > 1 ? par0[j] : 0) : 0; };
    int n_pin = 0;
    n_c = 0;
    {
        // (the verdicts of a thread's first 32 chunks stay in a register mask: those of the prefetched
        // chunks, then batches of eight whose parents and boundaries are fetched together with no
        // branch around the loads; longer runs read memory chunk by chunk)
        unsigned cand = 0u;
        int pins = 0;
#pragma unroll
        for (int k = 0; k < LC_BM_PF; ++k) {
            const int st = j_lo + k < j_hi ? chunk_state_of(j_lo + k, pf_s[k], pf_p[k]) : 0;
            cand |= st == 1 ? 1u << k : 0u;
            pins += st == 2 ? 1 : 0;
        }
        const int j_last = max(M - 1, 0);
        for (int k0 = LC_BM_PF; k0 < min(EM, 32); k0 += 8) {
            int pv[8], sv[8];
#pragma unroll
            for (int k = 0; k < 8; ++k) {
                const int j = min(j_lo + k0 + k, j_last);
                pv[k] = L > 1 ? par0[j] : 0;
                sv[k] = bnd[j];
            }
#pragma unroll
            for (int k = 0; k < 8; ++k) {
                const int st = (k0 + k < 32 && j_lo + k0 + k < j_hi) ? chunk_state_of(j_lo + k0 + k, sv[k], pv[k]) : 0;
                cand |= st == 1 ? 1u << (k0 + k) : 0u;
                pins += st == 2 ? 1 : 0;
            }
        }
        int mine = __popc(cand);
        for (int j = j_lo + 32; j < j_hi; ++j) {
            const int st = chunk_state(j);
            mine += st == 1 ? 1 : 0;
            pins += st == 2 ? 1 : 0;
        }
        int pos, e1;
        lc_block_scan2<LC_BM_THREADS>(mine, pins, sel_sh, &pos, &e1, &n_c, &n_pin);
        in_lds = n_c <= CL;
        int* nxt = in_lds ? (cid == l_cid ? l_nxt : l_cid) : (cid == g_cid ? g_nxt : g_cid);
        if (mine > 0) {
            while (cand != 0u) {
                nxt[pos++] = j_lo + __ffs((int)cand) - 1;
                cand &= cand - 1u;
            }
            for (int j = j_lo + 32; j < j_hi; ++j)
                if (chunk_state(j) == 1) nxt[pos++] = j;
        }
        cid = nxt;
    }
    lc_leaf_select_prepare<LC_BM_THREADS>(leaf_sh);
    __syncthreads();
    uint32_t* key = in_lds ? l_key : g_key;
    int* wgt = in_lds ? l_wgt : g_wgt;
    // ---- score them: key and length per candidate
    {
        const size_t cb = (size_t)bh * cap0;
        const bool c0b = ix.c0_bf16 != 0;
        uint32_t kmin = 0xffffffffu, kmax = 0u;
        constexpr int NBC = G <= 2 ? 4 : (G <= 4 ? 3 : NB);     // (little else is live here)
        for (int i0 = grp; i0 < n_c; i0 += NBC * LC_BM_GROUPS) {
            LcNodeFrag f[NBC];
            float R[NBC];
            int s0[NBC], s1[NBC], jj[NBC];
#pragma unroll
            for (int k = 0; k < NBC; ++k) {
                const int j = cid[min(i0 + k * LC_BM_GROUPS, n_c - 1)];
                jj[k] = j;
                f[k] = lc_load_chunk_node(ix.center[0], c0b, cb + j, sub);
                R[k] = ix.radius[0][cb + j];
                s0[k] = bnd[j];
                s1[k] = bnd[j + 1];
            }
#pragma unroll
            for (int k = 0; k < NBC; ++k) {
                const int i = i0 + k * LC_BM_GROUPS;
                const float sc = score_node(c0b ? lc_widen_chunk_frag(f[k]) : f[k], R[k]);
                uint32_t kk = lc_score_key(sc);
                if (kk == 0xffffffffu) kk = 0xfffffffeu;           // the select routine's mark is reserved
                if (sub == 0 && i < n_c) {
                    key[i] = kk;
                    wgt[i] = max(0, s1[k] - s0[k]);
                    if (scores) scores[jj[k]] = sc;
                }
                if (i < n_c && kk != 0u) { kmin = min(kmin, kk); kmax = max(kmax, kk); }
            }
        }
        lc_leaf_select_range(kmin, kmax, leaf_sh);
    }
    if (in_lds && tid < 4 && n_c + tid < ((n_c + 3) & ~3)) { key[n_c + tid] = 0u; wgt[n_c + tid] = 0; }
    __syncthreads();
    const long long C0 = a.beam[0] > 0 ? a.beam[0] : 0x7fffffffLL;
    uint8_t* flg = in_lds ? l_flg : g_flg;
    if (in_lds && n_c <= LC_BM_RANK_MAX) {
        // a short list: every chunk is ranked against the others directly
        uint32_t mk;
        int reached;
        lc_small_select<LC_BM_THREADS, false>(n_c, 0, (long long)W, C0, key, wgt, flg, sel_sh, &mk, &reached);
    } else {
        const uint32_t thr = lc_leaf_select<LC_BM_THREADS>(n_c, key, wgt, (long long)W, C0, leaf_sh);
        __syncthreads();
        for (int i = tid; i < n_c; i += LC_BM_THREADS) flg[i] = key[i] > thr ? 1 : 0;
    }
    __syncthreads();
    // ---- the chunk list: pinned chunks (ids 0 .. n_pin - 1), then the selected candidates in ascending order
    int32_t* ids = a.ids + (size_t)bh * a.cap;
    for (int j = tid; j < min(n_pin, a.cap); j += LC_BM_THREADS) ids[j] = j;
    int n_sel = 0;
    {
        const int E = (n_c + LC_BM_THREADS - 1) / LC_BM_THREADS;
        const int i_lo = min(n_c, tid * E), i_hi = min(n_c, i_lo + E);
        int mine = 0;
        for (int i = i_lo; i < i_hi; ++i) mine += flg[i] ? 1 : 0;
        int pos = n_pin + lc_block_scan<LC_BM_THREADS>(mine, sel_sh, &n_sel);
        for (int i = i_lo; i < i_hi; ++i) {
            if (flg[i]) {
                if (pos < a.cap) ids[pos] = cid[i];
                ++pos;
            }
        }
    }
    const int pos0 = n_pin + n_sel;
    if (tid == 0) a.counts[bh] = min(pos0, a.cap);
}

template <int G>
static int launch_beam_g(LcRetrieveArgs& a, int max_nodes, hipStream_t stream) {
    // LDS lists for up to LC_BEAM_LIST_MAX candidates per level (more go to the workspace)
    const int cl = lc_beam_list_slots(max_nodes);
    a.chunk_cap = cl;
    const size_t lds = (size_t)lc_beam_layout(cl).total;
    if (lds + sizeof(LcLeafSelSh) + LC_SEL_SH * 4 + LC_BM_KEPT_WORDS * 4 + 256 > 48 * 1024)
        LC_HIP_CHECK(hipFuncSetAttribute(reinterpret_cast<const void*>(&lc_beam_kernel<G>),
                                         hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));
    hipLaunchKernelGGL(lc_beam_kernel<G>, dim3(a.ix.H, a.ix.B), dim3(LC_BM_THREADS), lds, stream, a);
    LC_HIP_CHECK(hipGetLastError());
    return LC_OK;
}

// lc_leaf_kernel runs 1024 threads = 64 groups: one chunk per group while scoring; the last workgroup
// has enough threads to hold a few keys each during the select.
#define LC_LF_THREADS 1024
#define LC_LF_THREADS_MAX LC_LF_THREADS
#define LC_LF_GROUPS (LC_LF_THREADS / 16)

// ---------------------------------------------------------------------------------
// lc_leaf_kernel: chunk scoring + budget selection by the last workgroup
// ---------------------------------------------------------------------------------
// BF16: how the chunk-level centers are stored (a compile-time copy of the index's flag).
template <int G, int R, bool BF16>
__global__ void __launch_bounds__(LC_LF_THREADS)
lc_leaf_kernel(const LcRetrieveArgs a) {
    extern __shared__ int lds_dyn[];
    __shared__ LcLeafSelSh sel_sh;
    __shared__ int last_sh;

    const LcDev& ix = a.ix;
    const int h = blockIdx.y, b = blockIdx.z;
    const int bh = b * ix.H + h;
    const int tid = threadIdx.x;
    const int sub = tid & 15, grp = tid >> 4;
    const size_t cb = (size_t)bh * ix.cap[0];
    constexpr bool c0b = BF16;
    const int cap0 = ix.cap[0];
    const int* bnd = ix.bounds + (size_t)b * (cap0 + 1);
    uint32_t* keys = a.keys + cb;
    float* scores = a.scores ? a.scores + cb : nullptr;
    // the per-chunk arrays of the scoring part through range-checked buffer resources (an index
    // derived from stored values -- a parent pointer -- cannot reach memory outside its array)
    const __amdgpu_buffer_rsrc_t bnd_r = lc_buffer(bnd, (cap0 + 1) * 4);
    const __amdgpu_buffer_rsrc_t want_r = lc_buffer(a.want + cb, cap0);
    const __amdgpu_buffer_rsrc_t par_r = lc_buffer(ix.parent[0] + cb, cap0 * 4);
    const __amdgpu_buffer_rsrc_t rad_r = lc_buffer(ix.radius[0] + cb, cap0 * 4);
    const bool have_want = a.walk != 0;

    // loads that do not depend on M are issued together with it (the arrays are cap0 long)
    const int j_lo = blockIdx.x * (R * LC_LF_GROUPS);
    int jj[R];
    int wv[R];
    float rv[R];
#pragma unroll
    for (int r = 0; r < R; ++r) {
        const int j = min(j_lo + r * LC_LF_GROUPS + grp, cap0 - 1);
        jj[r] = j;
        // (rows past the chunk count hold whatever the buffer held: the result is unused)
        wv[r] = (lc_buf_load_i32(bnd_r, j) >= a.sink ? 1 : 0) & (have_want ? lc_buf_load_u8(want_r, lc_buf_load_i32(par_r, j)) : 1);
        rv[r] = lc_buf_load_f32(rad_r, j);
    }
    // Without a level walk every chunk below M is scored, so its center can be fetched right away
    // instead of one memory round trip later (with a walk the centers of pruned chunks are the
    // traffic the walk exists to save, so there the load waits for the verdict).
    constexpr bool kSpec = R <= 2 || (R == 4 && G <= 7);      // as far as the registers of a 1024-thread workgroup go
    LcNodeFrag pre[kSpec ? R : 1];
    if (kSpec && !have_want) {
#pragma unroll
        for (int r = 0; r < (kSpec ? R : 1); ++r) pre[r] = lc_load_chunk_node(ix.center[0], c0b, cb + jj[r], sub);
    }
    // (group size 7 with four speculative centers per group: the query stays packed, see lc_upper_kernel)
    constexpr bool QP = kSpec && R == 4 && G >= 7;
    float qf[QP ? 1 : G][8], qn[G];
    uint32_t qp[QP ? G : 1][4];
    if constexpr (QP) lc_load_query_packed<G>(a.q + (size_t)b * ix.H * G * LC_D, h, sub, qp, qn);
    else lc_load_query_frags<G>(a.q + (size_t)b * ix.H * G * LC_D, h, sub, qf, qn);
    auto score_chunk = [&](const LcNodeFrag& raw, float Rv) -> float {
        if constexpr (QP) return lc_score_frag_packed<G>(c0b ? lc_widen_chunk_frag(raw) : raw, Rv, qp, qn);
        else return lc_score_chunk_frag<G>(raw, c0b, Rv, qf, qn);
    };
    const int M = ix.state[bh * 4 + 1];

    if (j_lo < M) {
        if (a.budget > 0) {
            float sv[R];
#pragma unroll
            for (int r = 0; r < R; ++r) {
                const int j = j_lo + r * LC_LF_GROUPS + grp;
                sv[r] = LC_NEG_INF;
                if (j < M && wv[r]) {
                    if (kSpec && !have_want) sv[r] = score_chunk(pre[kSpec ? r : 0], rv[r]);
                    else sv[r] = score_chunk(lc_load_chunk_node(ix.center[0], c0b, cb + jj[r], sub), rv[r]);
                }
            }
#pragma unroll
            for (int r = 0; r < R; ++r) {
                const int j = j_lo + r * LC_LF_GROUPS + grp;
                if (j < M && sub == 0) {
                    lc_store_agent(&keys[j], lc_score_key(sv[r]));
                    if (scores) scores[j] = sv[r];
                }
            }
        } else {
            for (int j = j_lo + tid; j < min(M, j_lo + (R * LC_LF_GROUPS)); j += LC_LF_THREADS) {
                lc_store_agent(&keys[j], 0u);
                if (scores) scores[j] = LC_NEG_INF;
            }
        }
    }

    // ---- last workgroup of this (sequence, head) selects
    // (every workgroup empties its select histogram on the way: whichever turns out to be the last
    // finds it ready behind the barriers of the arrival)
    lc_leaf_select_prepare<LC_LF_THREADS>(sel_sh);
    if (!lc_arrive_last(&ix.sync[bh * 4 + 0], (int)gridDim.x, &last_sh)) return;

    // stage keys and lengths (pinned chunks get length -1) in LDS, or fall back to global scratch
    uint32_t* skey;
    int* slen;
    if (a.chunk_cap > 0) {
        skey = reinterpret_cast<uint32_t*>(lds_dyn);
        slen = lds_dyn + a.chunk_cap;
    } else {
        int* g = a.scratch + (size_t)bh * 4 * ix.cap[0];
        skey = reinterpret_cast<uint32_t*>(g);
        slen = g + ix.cap[0];
    }
    uint32_t kmin = 0xffffffffu, kmax = 0u;
    // (batches of eight chunks per thread, all their loads in flight together: a memory round trip
    // per batch instead of one per chunk)
    constexpr int SB = 8;
    for (int j0 = tid; j0 < M; j0 += SB * LC_LF_THREADS) {
        int s0[SB], s1[SB];
        uint32_t kv[SB];
#pragma unroll
        for (int e = 0; e < SB; ++e) {
            const int j = min(j0 + e * LC_LF_THREADS, M - 1);
            s0[e] = bnd[j];
            s1[e] = bnd[j + 1];
            kv[e] = lc_load_agent(&keys[j]);
        }
#pragma unroll
        for (int e = 0; e < SB; ++e) {
            const int j = j0 + e * LC_LF_THREADS;
            if (j < M) {
                skey[j] = kv[e];
                slen[j] = (s0[e] < a.sink) ? -1 : (s1[e] - s0[e]);
                if (kv[e] != 0u) { kmin = min(kmin, kv[e]); kmax = max(kmax, kv[e]); }
            }
        }
    }
    lc_leaf_select_range(kmin, kmax, sel_sh);
    __syncthreads();

    const long long C = (a.policy == LC_POLICY_BEAM && a.beam[0] > 0) ? a.beam[0] : 0x7fffffffLL;
    const uint32_t thr = lc_leaf_select<LC_LF_THREADS>(M, skey, slen, a.budget > 0 ? (long long)a.budget : 0LL, C,
                                                       sel_sh);

    // each thread owns a contiguous run of chunks, so the ids come out ascending: count, scan, write
    int E = (M + LC_LF_THREADS - 1) / LC_LF_THREADS;
    E |= 1;                                             // odd stride: no LDS bank conflicts
    const int lo = min(M, tid * E), hi = min(M, lo + E);
    // (the verdicts of up to 64 chunks stay in a register mask; longer runs read LDS again)
    unsigned long long mask = 0ull;
    int my_sel = 0;
    for (int i = lo; i < hi; ++i) {
        const bool sel = slen[i] < 0 || skey[i] > thr;
        if (sel && i - lo < 64) mask |= 1ull << (i - lo);
        my_sel += sel ? 1 : 0;
    }
    int tot_s;
    int pos = lc_block_scan<LC_LF_THREADS>(my_sel, sel_sh.scan, &tot_s);
    int32_t* ids = a.ids + (size_t)bh * a.cap;
    while (mask) {
        const int k = __ffsll((long long)mask) - 1;
        mask &= mask - 1ull;
        if (pos < a.cap) ids[pos] = lo + k;
        ++pos;
    }
    for (int i = lo + 64; i < hi; ++i) {
        if (slen[i] < 0 || skey[i] > thr) {
            if (pos < a.cap) ids[pos] = i;
            ++pos;
        }
    }
    if (tid == 0) {
        a.counts[bh] = min(tot_s, a.cap);
        ix.sync[bh * 4 + 0] = 0;                 // ready for the next call
    }
}

// ---------------------------------------------------------------------------------
// launcher
// ---------------------------------------------------------------------------------
// ---------------------------------------------------------------------------------
// lc_score_kernel: chunk scoring only (the decode step's second kernel selects by itself)
// ---------------------------------------------------------------------------------
// The same scoring as lc_leaf_kernel without the selection behind it, so without its LDS and its
// 1024-thread workgroups: NT threads = NT/16 groups, R chunks per group.
#define LC_SC_THREADS 256
#define LC_SCORE_MAX_WGS 1024          // measured flat between 512 and 2048 workgroups
// BF16: how the chunk-level centers are stored (a compile-time copy of the index's flag).
template <int G, int R, bool BF16>
__global__ void __launch_bounds__(LC_SC_THREADS)
lc_score_kernel(const LcRetrieveArgs a) {
    constexpr int GROUPS = LC_SC_THREADS / 16;
    const LcDev& ix = a.ix;
    const int h = blockIdx.y, b = blockIdx.z;
    const int bh = b * ix.H + h;
    const int tid = threadIdx.x;
    const int sub = tid & 15, grp = tid >> 4;
    const size_t cb = (size_t)bh * ix.cap[0];
    constexpr bool c0b = BF16;
    const int cap0 = ix.cap[0];
    // the per-chunk arrays through range-checked buffer resources (an index derived from stored
    // values -- a parent pointer -- cannot reach memory outside its array)
    const __amdgpu_buffer_rsrc_t bnd_r = lc_buffer(ix.bounds + (size_t)b * (cap0 + 1), (cap0 + 1) * 4);
    const __amdgpu_buffer_rsrc_t keys_r = lc_buffer(a.keys + cb, cap0 * 4);
    const __amdgpu_buffer_rsrc_t want_r = lc_buffer(a.want + cb, cap0);
    const __amdgpu_buffer_rsrc_t par_r = lc_buffer(ix.parent[0] + cb, cap0 * 4);
    const __amdgpu_buffer_rsrc_t rad_r = lc_buffer(ix.radius[0] + cb, cap0 * 4);
    const bool have_want = a.walk != 0;
    const int j_lo = blockIdx.x * (R * GROUPS);
    int jj[R], wv[R];
    float rv[R];
#pragma unroll
    for (int r = 0; r < R; ++r) {
        const int j = min(j_lo + r * GROUPS + grp, cap0 - 1);
        jj[r] = j;
        // (rows past the chunk count hold whatever the buffer held: the result is unused)
        wv[r] = (lc_buf_load_i32(bnd_r, j) >= a.sink ? 1 : 0) & (have_want ? lc_buf_load_u8(want_r, lc_buf_load_i32(par_r, j)) : 1);
        rv[r] = lc_buf_load_f32(rad_r, j);
    }
    LcNodeFrag pre[R];
    if (!have_want) {
#pragma unroll
        for (int r = 0; r < R; ++r) pre[r] = lc_load_chunk_node(ix.center[0], c0b, cb + jj[r], sub);
    }
    float qf[G][8], qn[G];
    lc_load_query_frags<G>(a.q + (size_t)b * ix.H * G * LC_D, h, sub, qf, qn);
    const int M = ix.state[bh * 4 + 1];
    if (j_lo >= M) return;
#pragma unroll
    for (int r = 0; r < R; ++r) {
        const int j = j_lo + r * GROUPS + grp;
        float sv = LC_NEG_INF;
        if (a.budget > 0 && j < M && wv[r]) {
            if (!have_want) sv = lc_score_chunk_frag<G>(pre[r], c0b, rv[r], qf, qn);
            else sv = lc_score_chunk_frag<G>(lc_load_chunk_node(ix.center[0], c0b, cb + jj[r], sub), c0b, rv[r], qf, qn);
        }
        if (j < M && sub == 0) lc_buf_store_u32(keys_r, j, lc_score_key(sv));
    }
}


template <int G, int R>
static int launch_score(const LcRetrieveArgs& a, int max_M, hipStream_t stream) {
    const int per = R * (LC_SC_THREADS / 16);
    const int nblk = max_M > 0 ? (max_M + per - 1) / per : 1;
    if (a.ix.c0_bf16)
        hipLaunchKernelGGL((lc_score_kernel<G, R, true>), dim3(nblk, a.ix.H, a.ix.B), dim3(LC_SC_THREADS), 0, stream, a);
    else
        hipLaunchKernelGGL((lc_score_kernel<G, R, false>), dim3(nblk, a.ix.H, a.ix.B), dim3(LC_SC_THREADS), 0, stream, a);
    LC_HIP_CHECK(hipGetLastError());
    return LC_OK;
}

template <int G, int R, bool BF16>
static int launch_leaf_t(const LcRetrieveArgs& a, int max_M, size_t lds, hipStream_t stream) {
    if (lds + sizeof(LcLeafSelSh) + 1024 > 48 * 1024)             // static + dynamic beyond the default allowance
        LC_HIP_CHECK(hipFuncSetAttribute(reinterpret_cast<const void*>(&lc_leaf_kernel<G, R, BF16>),
                                         hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));
    const int per = R * LC_LF_GROUPS;
    const int nblk = max_M > 0 ? (max_M + per - 1) / per : 1;
    hipLaunchKernelGGL((lc_leaf_kernel<G, R, BF16>), dim3(nblk, a.ix.H, a.ix.B), dim3(LC_LF_THREADS), lds, stream, a);
    LC_HIP_CHECK(hipGetLastError());
    return LC_OK;
}
template <int G, int R>
static int launch_leaf(const LcRetrieveArgs& a, int max_M, size_t lds, hipStream_t stream) {
    return a.ix.c0_bf16 ? launch_leaf_t<G, R, true>(a, max_M, lds, stream) : launch_leaf_t<G, R, false>(a, max_M, lds, stream);
}

template <int G>
static int launch_retrieve_g(LcRetrieveArgs& a, int max_M, hipStream_t stream) {
    const LcDev& ix = a.ix;
    const int mc = ((max_M + 63) / 64) * 64;
    const size_t lds_limit = LC_WALK_LDS_LIMIT;
    if (a.policy == LC_POLICY_BEAM) return launch_beam_g<G>(a, a.upper_cap > max_M ? a.upper_cap : max_M, stream);
    if (a.walk) {
        // as long a probe list as LDS holds next to the internal-node slots (the host has checked that one fits)
        int uc, pc;
        if (!lc_upper_launch_shape(a.upper_cap, max_M, &uc, &pc)) return LC_ERR_CAPACITY;
        a.upper_cap = uc;
        a.chunk_cap = pc;
        const size_t lds = lc_upper_lds_bytes(uc, pc);
        if (lds > 48 * 1024)
            LC_HIP_CHECK(hipFuncSetAttribute(reinterpret_cast<const void*>(&lc_upper_kernel<G>),
                                             hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));
        hipLaunchKernelGGL(lc_upper_kernel<G>, dim3(ix.H, ix.B), dim3(LC_UP_THREADS), lds, stream, a);
        LC_HIP_CHECK(hipGetLastError());
    }
    if (a.score_only) {
        // chunks per group: enough work per workgroup without leaving compute units idle
        int rs = 1;
        while (rs < 4 && (long long)((max_M + 16 * rs - 1) / (16 * rs)) * ix.H * ix.B > LC_SCORE_MAX_WGS) rs *= 2;
        if (rs == 1) return launch_score<G, 1>(a, max_M, stream);
        if (rs == 2) return launch_score<G, 2>(a, max_M, stream);
        return launch_score<G, 4>(a, max_M, stream);
    }
    a.chunk_cap = ((size_t)mc * 8 + sizeof(LcLeafSelSh) + 1024 <= lds_limit) ? mc : 0;
    const size_t lds2 = (size_t)a.chunk_cap * 8;
    // chunks per group: the fewest for which there is at most one workgroup per compute unit
    // (measured: beyond that the kernel gets slower, not faster)
    int r = 1;
#ifdef LC_LEAF_FORCE_R
    r = LC_LEAF_FORCE_R;
#else
    while (r < 8 && (long long)((max_M + 64 * r - 1) / (64 * r)) * ix.H * ix.B > 256) r *= 2;
#endif
    if (r == 1) return launch_leaf<G, 1>(a, max_M, lds2, stream);
    if (r == 2) return launch_leaf<G, 2>(a, max_M, lds2, stream);
    if (r == 4) return launch_leaf<G, 4>(a, max_M, lds2, stream);
    return launch_leaf<G, 8>(a, max_M, lds2, stream);
}

// Most internal nodes of one (sequence, head) that the exact level walk holds in LDS (with the shortest probe list).
int lc_walk_max_internal_nodes() { return lc_upper_max_internal_nodes(); }
int lc_beam_max_level_nodes() { return LC_BM_MAX_LEVEL_NODES; }

int lc_launch_retrieve(const lc_index* idx, const LcWs& ws, const void* q, int G, int budget,
                       int32_t* ids, int32_t* counts, float* scores, int cap,
                       int max_M, int max_upper, int score_only, hipStream_t stream) {
    LcRetrieveArgs a;
    a.score_only = score_only;
    a.ix = idx->dev;
    a.q = static_cast<const uint16_t*>(q);
    a.keys = ws.keys;
    a.want = ws.want;
    a.scores = scores;
    a.ids = ids;
    a.counts = counts;
    a.scratch = ws.scratch;
    a.cap = cap;
    a.budget = budget;
    a.policy = idx->cfg.policy;
    a.sink = idx->cfg.sink_tokens;
    for (int l = 0; l < LC_MAX_LEVELS; ++l) a.beam[l] = idx->cfg.beam[l];
    a.walk = (max_upper >= 0 && idx->cfg.levels > 1) ? 1 : 0;
    if (max_upper < 0) max_upper = 0;
    a.upper_cap = ((max_upper + 63) / 64) * 64;
    if (a.upper_cap < 64) a.upper_cap = 64;
    a.chunk_cap = 0;
    switch (G) {
        case 1: return launch_retrieve_g<1>(a, max_M, stream);
        case 2: return launch_retrieve_g<2>(a, max_M, stream);
        case 3: return launch_retrieve_g<3>(a, max_M, stream);
        case 4: return launch_retrieve_g<4>(a, max_M, stream);
        case 5: return launch_retrieve_g<5>(a, max_M, stream);
        case 6: return launch_retrieve_g<6>(a, max_M, stream);
        case 7: return launch_retrieve_g<7>(a, max_M, stream);
        case 8: return launch_retrieve_g<8>(a, max_M, stream);
    }
    return LC_ERR_BAD_SHAPE;
}
