// Retrieval kernels: Eq. 2 node scoring, level-by-level pruning, budget selection.
//
// Kernel 1 (lc_upper_kernel): one workgroup per (sequence, KV head).  Scores every
// internal node (levels >= 1), keeps score keys and frontier flags in LDS, and
// walks the levels top-down:
//   EXACT  probe pass  -> a lower bound tau0 of the selection cutoff,
//          verify pass -> every node whose bound reaches tau0 stays;
//   BEAM   keep the beam[l] best frontier nodes per level (Algorithm 1).
// It leaves a byte map of the level-1 nodes whose chunks must be scored.
//
// Kernel 2 (lc_leaf_kernel): many workgroups per (sequence, KV head) score the
// surviving chunks; the last workgroup to finish for a (sequence, head) runs the
// weighted radix select over the chunk keys (weights = chunk lengths) and emits
// the ids in ascending order.
#include "lc_device.h"
#include "lc_internal.h"

#define LC_RT_THREADS 256
#define LC_RT_GROUPS (LC_RT_THREADS / 16)
#define LC_LEAF_CHUNKS_PER_BLOCK 32
#define LC_TAU_SLACK 1e-3f

struct LcRetrieveArgs {
    LcDev ix;
    const uint16_t* q;       // [B][H_q][d]
    uint32_t* keys;          // [B][H][cap0]
    uint8_t* kept1;          // [B][H][cap1]
    float* scores;           // [B][H][cap0] or null
    int32_t* ids;            // [B][H][cap]
    int32_t* counts;         // [B][H]
    int cap;
    int budget;
    int policy;
    int sink;
    int beam[LC_MAX_LEVELS];
    int upper_cap;           // LDS entries available for internal nodes
};

// ---------------------------------------------------------------------------------
// kernel 1: internal levels
// ---------------------------------------------------------------------------------
template <int G>
__global__ void __launch_bounds__(LC_RT_THREADS)
lc_upper_kernel(const LcRetrieveArgs a) {
    extern __shared__ int lds_dyn[];
    __shared__ int sel_sh[516];
    __shared__ int off_sh[LC_MAX_LEVELS + 1];

    const LcDev& ix = a.ix;
    const int h = blockIdx.x, b = blockIdx.y;
    const int bh = b * ix.H + h;
    const int tid = threadIdx.x;
    const int sub = tid & 15, grp = tid >> 4;
    const int L = ix.L;
    const int M = ix.state[bh * 4 + 1];

    // LDS: keys[NU] (uint32) | flag arrays fr[NU], kp[NU] (bytes)
    if (tid == 0) {
        int o = 0;
        for (int l = 1; l < L; ++l) { off_sh[l] = o; o += ix.nlev[b * LC_MAX_LEVELS + l]; }
        off_sh[L] = o;
        off_sh[0] = 0;
    }
    __syncthreads();
    const int NU = off_sh[L];
    uint32_t* ukey = reinterpret_cast<uint32_t*>(lds_dyn);
    uint8_t* fr = reinterpret_cast<uint8_t*>(ukey + a.upper_cap);
    uint8_t* kp = fr + a.upper_cap;

    float qf[G][8], qn[G];
    lc_load_query_frags<G>(a.q + (size_t)b * ix.H * G * LC_D, h, sub, qf, qn);

    // ---- score every internal node
    for (int l = 1; l < L; ++l) {
        const int n_l = off_sh[l + 1] - off_sh[l];
        const size_t base = (size_t)bh * ix.cap[l];
        for (int n = grp; n < n_l; n += LC_RT_GROUPS) {
            const float R = ix.radius[l][base + n];
            const int nch = ix.nchunk[l][base + n];
            float s = lc_score_node<G>(ix.center[l] + (base + n) * LC_D, R, sub, qf, qn);
            if (nch <= 0) s = LC_NEG_INF;
            if (sub == 0) ukey[off_sh[l] + n] = lc_score_key(s);
        }
    }
    __syncthreads();

    uint8_t* kept1_out = a.kept1 + (size_t)bh * ix.cap[1];
    const int n1 = off_sh[2] - off_sh[1];

    if (a.budget <= 0) {
        for (int n = tid; n < n1; n += LC_RT_THREADS) kept1_out[n] = 0;
        return;
    }

    if (a.policy == LC_POLICY_BEAM) {
        // frontier of the top level: every node
        for (int n = tid; n < NU; n += LC_RT_THREADS) fr[n] = (n >= off_sh[L - 1]) ? 1 : 0;
        __syncthreads();
        for (int l = L - 1; l >= 1; --l) {
            const int o = off_sh[l], n_l = off_sh[l + 1] - o;
            const long long C = a.beam[l] > 0 ? a.beam[l] : 0x7fffffffLL;
            auto keyf = [&](int i) -> uint32_t { return fr[o + i] ? ukey[o + i] : 0u; };
            auto wf = [&](int) -> int { return 0; };
            const LcSel r = lc_block_select<LC_RT_THREADS>(n_l, 0x7fffffffffffLL, C, keyf, wf, sel_sh);
            // ties at kstar: ascending id while the count allows
            int tie_c = 0;
            for (int t0 = 0; t0 < n_l; t0 += LC_RT_THREADS) {
                const int i = t0 + tid;
                const uint32_t k = (i < n_l) ? keyf(i) : 0u;
                const int eq = (!r.all && k != 0u && k == r.kstar) ? 1 : 0;
                int tot;
                const int ex = lc_block_scan<LC_RT_THREADS>(eq, sel_sh, &tot);
                if (i < n_l) kp[o + i] = (k != 0u && (k > r.kstar || (eq && tie_c + ex + 1 <= r.remC))) ? 1 : 0;
                tie_c += tot;
            }
            __syncthreads();
            if (l >= 2) {
                const int ob = off_sh[l - 1], n_b = off_sh[l] - ob;
                const size_t pb = (size_t)bh * ix.cap[l - 1];
                for (int n = tid; n < n_b; n += LC_RT_THREADS) fr[ob + n] = kp[o + ix.parent[l - 1][pb + n]];
                __syncthreads();
            }
        }
        for (int n = tid; n < n1; n += LC_RT_THREADS) kept1_out[n] = kp[off_sh[1] + n];
        return;
    }

    // ---- EXACT, probe pass: going down, keep the best frontier nodes until their
    // subtree token counts reach the budget (whole tie groups are kept).
    for (int n = tid; n < NU; n += LC_RT_THREADS) fr[n] = (n >= off_sh[L - 1]) ? 1 : 0;
    __syncthreads();
    for (int l = L - 1; l >= 1; --l) {
        const int o = off_sh[l], n_l = off_sh[l + 1] - o;
        const size_t nb = (size_t)bh * ix.cap[l];
        auto keyf = [&](int i) -> uint32_t { return fr[o + i] ? ukey[o + i] : 0u; };
        auto wf = [&](int i) -> int { return ix.ntok[l][nb + i]; };
        const LcSel r = lc_block_select<LC_RT_THREADS>(n_l, (long long)a.budget - 1, 0x7fffffffLL, keyf, wf, sel_sh);
        for (int i = tid; i < n_l; i += LC_RT_THREADS) {
            const uint32_t k = keyf(i);
            kp[o + i] = (k != 0u && (r.all || k >= r.kstar)) ? 1 : 0;
        }
        __syncthreads();
        if (l >= 2) {
            const int ob = off_sh[l - 1], n_b = off_sh[l] - ob;
            const size_t pb = (size_t)bh * ix.cap[l - 1];
            for (int n = tid; n < n_b; n += LC_RT_THREADS) fr[ob + n] = kp[o + ix.parent[l - 1][pb + n]];
            __syncthreads();
        }
    }
    // score the probe's chunks (children of the kept level-1 nodes)
    uint32_t* pkeys = a.keys + (size_t)bh * ix.cap[0];
    {
        const size_t cb = (size_t)bh * ix.cap[0];
        const int* bnd = ix.bounds + (size_t)b * (ix.cap[0] + 1);
        const int o1 = off_sh[1];
        for (int j0 = 0; j0 < M; j0 += LC_RT_GROUPS) {
            const int j = j0 + grp;
            if (j < M) {
                uint32_t key = 0u;
                const int p = ix.parent[0][cb + j];
                if (kp[o1 + p] && bnd[j] >= a.sink) {
                    const float s = lc_score_node<G>(ix.center[0] + (cb + j) * LC_D, ix.radius[0][cb + j], sub, qf, qn);
                    key = lc_score_key(s);
                }
                if (sub == 0) pkeys[j] = key;
            }
        }
    }
    __syncthreads();
    uint32_t tau_key;
    {
        const int* bnd = ix.bounds + (size_t)b * (ix.cap[0] + 1);
        auto keyf = [&](int i) -> uint32_t { return pkeys[i]; };
        auto wf = [&](int i) -> int { return bnd[i + 1] - bnd[i]; };
        const LcSel r = lc_block_select<LC_RT_THREADS>(M, (long long)a.budget - 1, 0x7fffffffLL, keyf, wf, sel_sh);
        if (r.all) {
            tau_key = 1u;                                 // fewer than `budget` probe tokens: keep everything
        } else {
            const float tau = lc_key_score(r.kstar);
            tau_key = lc_score_key(tau - LC_TAU_SLACK * fmaxf(1.0f, fabsf(tau)));
            if (tau_key == 0u) tau_key = 1u;
        }
    }
    // ---- verify pass: keep every node whose bound reaches tau0 and whose parent was kept
    {
        const int o = off_sh[L - 1], n_l = off_sh[L] - o;
        for (int i = tid; i < n_l; i += LC_RT_THREADS) kp[o + i] = (ukey[o + i] >= tau_key) ? 1 : 0;
        __syncthreads();
    }
    for (int l = L - 2; l >= 1; --l) {
        const int o = off_sh[l], n_l = off_sh[l + 1] - o, oa = off_sh[l + 1];
        const size_t pb = (size_t)bh * ix.cap[l];
        for (int i = tid; i < n_l; i += LC_RT_THREADS)
            kp[o + i] = (ukey[o + i] >= tau_key && kp[oa + ix.parent[l][pb + i]]) ? 1 : 0;
        __syncthreads();
    }
    for (int n = tid; n < n1; n += LC_RT_THREADS) kept1_out[n] = kp[off_sh[1] + n];
}

// ---------------------------------------------------------------------------------
// kernel 2: chunk scoring + budget selection by the last workgroup
// ---------------------------------------------------------------------------------
template <int G>
__global__ void __launch_bounds__(LC_RT_THREADS)
lc_leaf_kernel(const LcRetrieveArgs a) {
    __shared__ int sel_sh[516];
    __shared__ int last_sh;

    const LcDev& ix = a.ix;
    const int h = blockIdx.y, b = blockIdx.z;
    const int bh = b * ix.H + h;
    const int tid = threadIdx.x;
    const int sub = tid & 15, grp = tid >> 4;
    const int M = ix.state[bh * 4 + 1];
    const size_t cb = (size_t)bh * ix.cap[0];
    const int* bnd = ix.bounds + (size_t)b * (ix.cap[0] + 1);
    uint32_t* keys = a.keys + cb;
    float* scores = a.scores ? a.scores + cb : nullptr;
    const uint8_t* kept1 = (ix.L > 1) ? a.kept1 + (size_t)bh * ix.cap[1] : nullptr;

    const int j_lo = blockIdx.x * LC_LEAF_CHUNKS_PER_BLOCK;
    if (j_lo < M && a.budget > 0) {
        float qf[G][8], qn[G];
        lc_load_query_frags<G>(a.q + (size_t)b * ix.H * G * LC_D, h, sub, qf, qn);
#pragma unroll
        for (int r = 0; r < LC_LEAF_CHUNKS_PER_BLOCK / LC_RT_GROUPS; ++r) {
            const int j = j_lo + r * LC_RT_GROUPS + grp;
            if (j < M) {
                bool want = bnd[j] >= a.sink;
                if (want && kept1) want = kept1[ix.parent[0][cb + j]] != 0;
                float s = LC_NEG_INF;
                if (want) s = lc_score_node<G>(ix.center[0] + (cb + j) * LC_D, ix.radius[0][cb + j], sub, qf, qn);
                if (sub == 0) {
                    keys[j] = lc_score_key(s);
                    if (scores) scores[j] = s;
                }
            }
        }
    } else if (j_lo < M) {
        for (int j = j_lo + tid; j < min(M, j_lo + LC_LEAF_CHUNKS_PER_BLOCK); j += LC_RT_THREADS) {
            keys[j] = 0u;
            if (scores) scores[j] = LC_NEG_INF;
        }
    }

    // ---- last workgroup of this (sequence, head) selects
    __threadfence();
    __syncthreads();
    if (tid == 0) {
        const int old = atomicAdd(&ix.sync[bh * 4 + 0], 1);
        last_sh = (old == (int)gridDim.x - 1) ? 1 : 0;
    }
    __syncthreads();
    if (!last_sh) return;
    __threadfence();

    auto keyf = [&](int i) -> uint32_t { return __builtin_nontemporal_load(&keys[i]); };
    auto wf = [&](int i) -> int { return bnd[i + 1] - bnd[i]; };
    const long long C = (a.policy == LC_POLICY_BEAM && a.beam[0] > 0) ? a.beam[0] : 0x7fffffffLL;
    const LcSel r = lc_block_select<LC_RT_THREADS>(M, a.budget > 0 ? (long long)a.budget : 0LL, C, keyf, wf, sel_sh);

    int32_t* ids = a.ids + (size_t)bh * a.cap;
    int base = 0, tie_w = 0, tie_c = 0;
    for (int t0 = 0; t0 < M; t0 += LC_RT_THREADS) {
        const int i = t0 + tid;
        const bool valid = i < M;
        const uint32_t k = valid ? keyf(i) : 0u;
        const bool pinned = valid && bnd[i] < a.sink;
        const int eq = (!r.all && k != 0u && k == r.kstar) ? 1 : 0;
        const int w = eq ? wf(i) : 0;
        int sel = (pinned || (k != 0u && k > r.kstar)) ? 1 : 0;
        if (__syncthreads_or(eq)) {
            int tot_w, tot_c;
            const int ex_w = lc_block_scan<LC_RT_THREADS>(w, sel_sh, &tot_w);
            const int ex_c = lc_block_scan<LC_RT_THREADS>(eq, sel_sh, &tot_c);
            if (eq && (long long)tie_w + ex_w + w <= r.remW && tie_c + ex_c + 1 <= r.remC) sel = 1;
            tie_w += tot_w;
            tie_c += tot_c;
        }
        int tot_s;
        const int ex_s = lc_block_scan<LC_RT_THREADS>(sel, sel_sh, &tot_s);
        if (sel && base + ex_s < a.cap) ids[base + ex_s] = i;
        base += tot_s;
    }
    if (tid == 0) {
        a.counts[bh] = min(base, a.cap);
        ix.sync[bh * 4 + 0] = 0;                 // ready for the next call
    }
}

// ---------------------------------------------------------------------------------
// launcher
// ---------------------------------------------------------------------------------
template <int G>
static int launch_retrieve_g(const LcRetrieveArgs& a, int max_M, int max_upper, hipStream_t stream) {
    const LcDev& ix = a.ix;
    if (ix.L > 1) {
        const size_t lds = (size_t)a.upper_cap * 4 + 2 * (size_t)a.upper_cap;
        hipLaunchKernelGGL(lc_upper_kernel<G>, dim3(ix.H, ix.B), dim3(LC_RT_THREADS), lds, stream, a);
        LC_HIP_CHECK(hipGetLastError());
    }
    const int nblk = max_M > 0 ? (max_M + LC_LEAF_CHUNKS_PER_BLOCK - 1) / LC_LEAF_CHUNKS_PER_BLOCK : 1;
    hipLaunchKernelGGL(lc_leaf_kernel<G>, dim3(nblk, ix.H, ix.B), dim3(LC_RT_THREADS), 0, stream, a);
    LC_HIP_CHECK(hipGetLastError());
    (void)max_upper;
    return LC_OK;
}

int lc_launch_retrieve(const lc_index* idx, const LcWs& ws, const void* q, int G, int budget,
                       int32_t* ids, int32_t* counts, float* scores, int cap,
                       int max_M, int max_upper, hipStream_t stream) {
    LcRetrieveArgs a;
    a.ix = idx->dev;
    a.q = static_cast<const uint16_t*>(q);
    a.keys = ws.keys;
    a.kept1 = ws.kept1;
    a.scores = scores;
    a.ids = ids;
    a.counts = counts;
    a.cap = cap;
    a.budget = budget;
    a.policy = idx->cfg.policy;
    a.sink = idx->cfg.sink_tokens;
    for (int l = 0; l < LC_MAX_LEVELS; ++l) a.beam[l] = idx->cfg.beam[l];
    a.upper_cap = ((max_upper + 63) / 64) * 64;
    if (a.upper_cap < 64) a.upper_cap = 64;
    switch (G) {
        case 1: return launch_retrieve_g<1>(a, max_M, max_upper, stream);
        case 2: return launch_retrieve_g<2>(a, max_M, max_upper, stream);
        case 3: return launch_retrieve_g<3>(a, max_M, max_upper, stream);
        case 4: return launch_retrieve_g<4>(a, max_M, max_upper, stream);
        case 5: return launch_retrieve_g<5>(a, max_M, max_upper, stream);
        case 6: return launch_retrieve_g<6>(a, max_M, max_upper, stream);
        case 7: return launch_retrieve_g<7>(a, max_M, max_upper, stream);
        case 8: return launch_retrieve_g<8>(a, max_M, max_upper, stream);
    }
    return LC_ERR_BAD_SHAPE;
}
