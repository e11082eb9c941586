// Sparse attention for one decode step: split-K flash-decode over the selected
// chunks (plus the open tail), merged by the last split to finish.
//
// Grid (split, KV head, sequence), 256 threads = 16 groups of 16 lanes.  A group
// owns a contiguous run of the split's tokens and handles them U at a time.
//   Q.K^T runs on the matrix cores: the 4 groups of a wavefront together hold 16
//   tokens, whose K rows form the 16 x 128 A operand of four 16x16x32 bf16 MFMAs;
//   the B operand is the query block (head n in column n).  The result leaves lane
//   (group, n) with the logits of the group's own tokens for head n, so each lane
//   keeps the online softmax (base 2) of one head and the probabilities reach the
//   other 15 lanes of the group by DPP row broadcasts.
//   P.V stays on the vector ALU: lane n of a group holds columns [8n, 8n + 8) of a
//   V row (one 16-byte load), four rows make a full 1 KiB wavefront load.
#include <type_traits>

#include "lc_device.h"
#include "lc_internal.h"
#include "lc_select.h"

#ifndef LC_DEC_THREADS
#define LC_DEC_THREADS 256
#endif
#define LC_DEC_GROUPS (LC_DEC_THREADS / 16)
#define LC_DEC_MIN_TOKENS_PER_SPLIT 64
#define LC_DEC_MAX_SPLITS 256
#define LC_DEC_TILE 1024          // tokens of a split whose cache rows are resolved into LDS at a time
#define LC_DEC_WIN 2048           // slots of the entry window of a tile: a power of two above LC_DEC_TILE + 2
#define LC_DEC_E 2                // selected ids per thread and pass of the row resolution
#define LC_LOG2E 1.4426950408889634f
#define LC_LN2 0.6931471805599453f

typedef __bf16 lc_bf16x8 __attribute__((ext_vector_type(8)));
typedef float lc_f32x4 __attribute__((ext_vector_type(4)));


struct LcDecodeArgs {
    LcDev ix;
    const uint16_t* q;
    const uint16_t* K;
    const uint16_t* V;
    long long ks_seq, ks_head, ks_tok;
    const int32_t* ids;
    const int32_t* counts;
    int cap;
    float* part_acc;      // [B][H][S][G][d]
    float* part_ml;       // [B][H][S][G][2]
    float* out;           // [B][H*G][d]
    float* lse;           // [B][H*G] or null
    // fused step only (the kernel selects the chunks itself from their score keys):
    const uint32_t* keys; // [B][H][cap0] score keys of the chunks (0 = not a candidate)
    int32_t* ids_out;     // [B][H][cap] selected ids, ascending, or null
    int32_t* counts_out;  // [B][H] or null
    int budget, sink;     // token budget, tokens of the pinned prefix
    int ew;               // fused step: rows of 64 chunks per wavefront that hold the longest sequence (host side: picks EC)
    int max_tokens;       // rows of one (sequence, head) slab of K and V
};

// Value of lane `src` (0..15) of the caller's 16-lane row, in every lane of the row.
template <int SRC>
__device__ __forceinline__ float lc_row_bcast(float v) {
    return lc_dpp<0x150 + SRC>(v);
}
__device__ __forceinline__ float lc_row_bcast_n(float v, int src) {      // src folds to a constant once unrolled
    switch (src) {
        case 0: return lc_row_bcast<0>(v);
        case 1: return lc_row_bcast<1>(v);
        case 2: return lc_row_bcast<2>(v);
        case 3: return lc_row_bcast<3>(v);
        case 4: return lc_row_bcast<4>(v);
        case 5: return lc_row_bcast<5>(v);
        case 6: return lc_row_bcast<6>(v);
        default: return lc_row_bcast<7>(v);
    }
}
// exp2 of (x - ref) where x may be -inf (gives 0); ref is finite.
__device__ __forceinline__ float lc_exp2_rel(float x, float ref) { return exp2f(x - ref); }

// FUSED = false: the chunk list comes from a.ids / a.counts.  FUSED = true: every workgroup first
// repeats the budget selection of its (sequence, head) from the chunk score keys -- the same
// deterministic routine on the same keys, so all splits agree -- and never reads a chunk list.
//
// The fused selection (lc_select_chunks) keeps the chunks in registers and leaves every lane with
// the first rows, lengths and token offsets of its selected chunks; the wavefronts then write the
// cache row of every token of the split's tile into LDS, 64 lanes per overlapping chunk.
template <int G, bool FUSED, int EC>
__global__ void __launch_bounds__(LC_DEC_THREADS)
lc_decode_kernel(const LcDecodeArgs a) {
    extern __shared__ int lds_dyn[];             // FUSED: key and length of every chunk, for the overflow path only
    using SelStore = typename std::conditional<FUSED, LcLeafSelSh, int>::type;
    using FusedStore = typename std::conditional<FUSED, LcFusedSh<LC_DEC_THREADS>, int>::type;
    constexpr int WIN = FUSED ? 1 : LC_DEC_WIN;
    __shared__ __attribute__((aligned(16))) SelStore sel_store;
    __shared__ __attribute__((aligned(16))) FusedStore fused_store;
    __shared__ int scan_sh[8];
    __shared__ int rows[LC_DEC_TILE];
    __shared__ int win_off[WIN];                  // first token position of the entries that overlap the tile
    __shared__ int win_st[WIN];                   // and their first cache row
    __shared__ int win_hd[2];                     // indices of the entries holding the tile's first / last token
    __shared__ int last_sh;
    __shared__ float comb_ml[LC_DEC_THREADS / 64][G][2];
    __shared__ __attribute__((aligned(16))) float comb_acc[LC_DEC_THREADS / 64][G][LC_D];
    __shared__ float mrg_m[LC_DEC_MAX_SPLITS * G];
    __shared__ float mrg_l[LC_DEC_MAX_SPLITS * G];
    __shared__ float mrg_hd[2 * G];
    __shared__ float4 mrg_red[LC_DEC_THREADS];

    // tokens per group and batch of loads; two batches are in flight per group (the next one is
    // issued before the current one is consumed)
    constexpr int U = (G <= 4) ? 4 : 2;
    constexpr int E = LC_DEC_E;
    const LcDev& ix = a.ix;
    const int s = blockIdx.x, S = gridDim.x, h = blockIdx.y, b = blockIdx.z;
    const int bh = b * ix.H + h;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int sub = tid & 15, grp = tid >> 4, q4 = lane >> 4;

    const int* bnd = ix.bounds + (size_t)b * (ix.cap[0] + 1);
    // the query block in MFMA B layout (lane (q4, n): head n, columns 8 q4 + 32 j + [0, 8))
    uint4 qb[4];
    {
        const uint16_t* qh = a.q + ((size_t)b * ix.H * G + (size_t)h * G + min(sub, G - 1)) * LC_D + 8 * q4;
#pragma unroll
        for (int j = 0; j < 4; ++j) qb[j] = *reinterpret_cast<const uint4*>(qh + 32 * j);
    }

    // ---- the attended tokens are the selected chunks in ascending id order, then the open tail.
    // Entry i of that list is (first cache row, length).  Both variants end up with: n_runs entries,
    // n_tok tokens, and a way to find the cache row of every token of a tile.
    int n_runs, n_tok, T;
    // FUSED = false: thread t of a pass owns entries [E t, E t + E); the first pass stays in registers
    const int32_t* ids = nullptr;
    int n_ids = 0, M = 0;
    int idv[E], st0[E], ln0[E];
    int ex0 = 0, tot0 = 0;
    // FUSED = true: this lane's chunks and the totals of the selection
    LcChunkSel<EC> cs;

    auto entries = [&](int base, bool preloaded, int (&st)[E], int (&ln)[E]) -> int {
        int sum = 0;
#pragma unroll
        for (int e = 0; e < E; ++e) {
            const int i = base + tid * E + e;
            st[e] = 0;
            ln[e] = 0;
            if (i < n_ids) {
                const int id = max(0, min(preloaded ? idv[e] : ids[i], M - 1));
                st[e] = bnd[id];
                ln[e] = max(0, bnd[id + 1] - st[e]);
            } else if (i == n_ids) {
                st[e] = bnd[M];
                ln[e] = max(0, T - st[e]);
            }
            sum += ln[e];
        }
        return sum;
    };

    if constexpr (!FUSED) {
        ids = a.ids + (size_t)bh * a.cap;
        // independent loads first: the ids a thread will need are fetched before the count is known
#pragma unroll
        for (int e = 0; e < E; ++e) idv[e] = (tid * E + e < a.cap) ? ids[tid * E + e] : 0;
        T = ix.state[bh * 4 + 0];
        M = ix.state[bh * 4 + 1];
        n_ids = a.counts[bh];
        n_ids = (M > 0) ? max(0, min(n_ids, a.cap)) : 0;
        n_runs = n_ids + 1;
        ex0 = lc_block_scan<LC_DEC_THREADS>(entries(0, true, st0, ln0), scan_sh, &tot0);
        n_tok = tot0;
        for (int base = LC_DEC_THREADS * E; base < n_runs; base += LC_DEC_THREADS * E) {
            int st[E], ln[E], tot;
            lc_block_scan<LC_DEC_THREADS>(entries(base, false, st, ln), scan_sh, &tot);
            n_tok += tot;
        }
    } else {
        lc_select_chunks<LC_DEC_THREADS, EC>(ix, b, bh, a.keys, a.budget, a.sink, s == 0 ? a.ids_out : nullptr,
                                             a.counts_out, a.cap, sel_store, fused_store, lds_dyn, cs);
        T = cs.T;
        M = cs.M;
        n_tok = cs.n_tok;
        n_runs = cs.n_sel + 1;
    }
    int S_eff = (n_tok + LC_DEC_MIN_TOKENS_PER_SPLIT - 1) / LC_DEC_MIN_TOKENS_PER_SPLIT;
    S_eff = max(1, min(S, S_eff));

    if (s < S_eff) {
        const int lo = (int)(((long long)n_tok * s) / S_eff);
        const int hi = (int)(((long long)n_tok * (s + 1)) / S_eff);
        const float scale = 0.08838834764831845f * LC_LOG2E;     // log2(e) / sqrt(128)
        // softmax state of head `sub` over this group's tokens (lanes sub >= G repeat head G-1)
        float m_run = LC_NEG_INF, l_run = 0.f;
        float acc[G][8];
#pragma unroll
        for (int g = 0; g < G; ++g) {
#pragma unroll
            for (int i = 0; i < 8; ++i) acc[g][i] = 0.f;
        }
        // K and V of this (sequence, head) as buffer resources: one 32-bit byte offset per row
        // (the host has checked that the slab spans less than 2 GiB)
        // (the resources end with the last row the index may ever hold, so a wrong row cannot fault)
        const int row_bytes = (int)a.ks_tok * 2;
        const int slab_bytes = (a.max_tokens - 1) * row_bytes + LC_D * 2;
        const __amdgpu_buffer_rsrc_t Kr = lc_buffer(a.K + (size_t)b * a.ks_seq + (size_t)h * a.ks_head, slab_bytes);
        const __amdgpu_buffer_rsrc_t Vr = lc_buffer(a.V + (size_t)b * a.ks_seq + (size_t)h * a.ks_head, slab_bytes);

        // A lane loads K for token (sub & 3) of group (sub >> 2) of its wavefront -- row `sub` of the
        // MFMA A operand -- and V for the tokens of its own group.
        const int gk = (wave << 2) + (sub >> 2), uk = sub & 3;
        int tv = 0, tv_end = 0, tk = 0, tk_end = 0;
        // Branch-free: a branch around a load would put each row lookup (an LDS read) and its load in a
        // basic block of its own, waited for one after the other.  All row lookups go out together
        // (slot 0 stands in where there is no token) and a load without a token gets an offset past
        // the resource's end, which the range check answers with zeros.
        auto issue = [&](int it, lc_v4i (&kv)[4], lc_v4i (&vv)[U]) {
            const int k_tok = tk + it * U + uk;
            const bool k_in = uk < U && k_tok < tk_end;
            const int k_row = rows[k_in ? k_tok : 0];
            int v_row[U];
            bool v_in[U];
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const int v_tok = tv + it * U + u;
                v_in[u] = v_tok < tv_end;
                v_row[u] = rows[v_in[u] ? v_tok : 0];
            }
            const int ko = k_in ? k_row * row_bytes + 16 * q4 : slab_bytes;
#pragma unroll
            for (int j = 0; j < 4; ++j) kv[j] = __builtin_amdgcn_raw_buffer_load_b128(Kr, ko + 64 * j, 0, 0);
#pragma unroll
            for (int u = 0; u < U; ++u)
                vv[u] = __builtin_amdgcn_raw_buffer_load_b128(Vr, v_in[u] ? v_row[u] * row_bytes + 16 * sub : slab_bytes, 0, 0);
        };
        // logits of the wavefront's 16 tokens for all heads (MFMA), one online-softmax update of
        // this lane's head, then P.V for every head with the broadcast probabilities
        auto consume = [&](int it, const lc_v4i (&kv)[4], const lc_v4i (&vv)[U]) {
            lc_f32x4 d = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int j = 0; j < 4; ++j)
                d = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(lc_bf16x8, kv[j]),
                                                            __builtin_bit_cast(lc_bf16x8, qb[j]), d, 0, 0, 0);
            // d[i]: token 4 q4 + i of the wavefront = token i of this lane's group, head `sub`
            float x[U];
            float mx = m_run;
#pragma unroll
            for (int u = 0; u < U; ++u) {
                x[u] = (tv + it * U + u < tv_end) ? d[u] * scale : LC_NEG_INF;
                mx = fmaxf(mx, x[u]);
            }
            const float ref = (mx == LC_NEG_INF) ? 0.f : mx;
            const float sc = lc_exp2_rel(m_run, ref);
            float p[U];
            float psum = 0.f;
#pragma unroll
            for (int u = 0; u < U; ++u) {
                p[u] = lc_exp2_rel(x[u], ref);
                psum += p[u];
            }
            l_run = fmaf(l_run, sc, psum);
            m_run = mx;
#pragma unroll
            for (int g = 0; g < G; ++g) {
                const float sg = lc_row_bcast_n(sc, g);
#pragma unroll
                for (int i = 0; i < 8; ++i) acc[g][i] *= sg;
            }
#pragma unroll
            for (int u = 0; u < U; ++u) {
                float vf[8];
                {
                    const int v0 = vv[u].x, v1 = vv[u].y, v2 = vv[u].z, v3 = vv[u].w;
                    lc_unpack8(make_uint4((uint32_t)v0, (uint32_t)v1, (uint32_t)v2, (uint32_t)v3), vf);
                }
#pragma unroll
                for (int g = 0; g < G; ++g) {
                    const float pg = lc_row_bcast_n(p[u], g);
#pragma unroll
                    for (int i = 0; i < 8; ++i) acc[g][i] = fmaf(pg, vf[i], acc[g][i]);
                }
            }
        };

        // The split's tokens are handled in tiles; for each tile the workgroup first writes the cache
        // row of every token into LDS, then every group streams a contiguous slice of the tile.
        for (int tile0 = lo; tile0 < hi; tile0 += LC_DEC_TILE) {
            const int tl = min(LC_DEC_TILE, hi - tile0);
            const int row_max = max(T - 1, 0);
            if constexpr (FUSED) {
                // 64 lanes per selected chunk that overlaps the tile (its owner's values are read by lane)
                if (tile0 != lo) lc_barrier_lds();                  // the previous tile's rows have been used
                auto fill = [&](int o, int st, int ln) {
                    const int k0 = max(o, tile0), k1 = min(o + ln, tile0 + tl);
                    for (int k = k0 + lane; k < k1; k += 64) rows[k - tile0] = max(0, min(st + (k - o), row_max));
                };
#pragma unroll
                for (int e = 0; e < EC; ++e) {
                    const int off = cs.base_tok + cs.coff[e];
                    unsigned long long mask = __ballot(cs.stok[e] > 0 && off < tile0 + tl && tile0 < off + cs.stok[e]);
                    while (mask != 0ull) {
                        const int l = __ffsll((long long)mask) - 1;
                        mask &= mask - 1ull;
                        fill(lc_readlane(off, l), lc_readlane(cs.cst[e], l), lc_readlane(cs.stok[e], l));
                    }
                }
                if (wave == 0 && cs.tail_ln > 0 && cs.n_sel_tok < tile0 + tl && tile0 < cs.n_sel_tok + cs.tail_ln)
                    fill(cs.n_sel_tok, cs.tail_st, cs.tail_ln);
                lc_barrier_lds();
            } else {
                // The few entries that overlap the tile go into a window at slot (entry index mod window
                // size) -- overlapping entries are consecutive and fewer than the window is long -- and the
                // entries that hold the tile's first and last token leave their indices; then one small
                // binary search per token, in parallel.
                __syncthreads();
                {
                    auto entry = [&](int i, int off, int st, int ln) {
                        if (ln > 0 && off < tile0 + tl && tile0 < off + ln) {
                            win_off[i & (LC_DEC_WIN - 1)] = off;
                            win_st[i & (LC_DEC_WIN - 1)] = st;
                            if (off <= tile0) win_hd[0] = i;
                            if (tile0 + tl <= off + ln) win_hd[1] = i;
                        }
                    };
                    auto visit = [&](int base, int off, const int (&st)[E], const int (&ln)[E]) {
#pragma unroll
                        for (int e = 0; e < E; ++e) {
                            entry(base + tid * E + e, off, st[e], ln[e]);
                            off += ln[e];
                        }
                    };
                    visit(0, ex0, st0, ln0);
                    int carry = tot0;
                    for (int base = LC_DEC_THREADS * E; base < n_runs; base += LC_DEC_THREADS * E) {
                        int st[E], ln[E], tot;
                        const int ex = lc_block_scan<LC_DEC_THREADS>(entries(base, false, st, ln), scan_sh, &tot);
                        visit(base, carry + ex, st, ln);
                        carry += tot;
                    }
                }
                __syncthreads();
                {
                    const int w_first = win_hd[0], w_last = win_hd[1];
                    for (int i = tid; i < tl; i += LC_DEC_THREADS) {
                        const int tok = tile0 + i;
                        int lo_w = w_first, hi_w = w_last + 1;   // off[lo_w] <= tok < off[hi_w]
                        while (hi_w - lo_w > 1) {
                            const int mid = (lo_w + hi_w) >> 1;
                            if (win_off[mid & (LC_DEC_WIN - 1)] <= tok) lo_w = mid; else hi_w = mid;
                        }
                        const int sl = lo_w & (LC_DEC_WIN - 1);
                        rows[i] = max(0, min(win_st[sl] + (tok - win_off[sl]), row_max));
                    }
                }
                __syncthreads();
            }
            const int per = (tl + LC_DEC_GROUPS - 1) / LC_DEC_GROUPS;
            const int n_it = (per + U - 1) / U;            // the same for every wavefront: the MFMA needs all lanes
            tv = min(tl, grp * per);
            tv_end = min(tl, tv + per);
            tk = min(tl, gk * per);
            tk_end = min(tl, tk + per);
            lc_v4i kA[4], vA[U], kB[4], vB[U];
            issue(0, kA, vA);
            for (int it = 0; it < n_it; it += 2) {
                if (it + 1 < n_it) issue(it + 1, kB, vB);
                consume(it, kA, vA);
                if (it + 1 >= n_it) break;
                if (it + 2 < n_it) issue(it + 2, kA, vA);
                consume(it + 1, kB, vB);
            }
        }

        // ---- combine the 4 groups of a wave (xor 16, 32), then the waves through LDS
#pragma unroll
        for (int off = 16; off < 64; off <<= 1) {
            const float m_o = __shfl_xor(m_run, off);
            const float l_o = __shfl_xor(l_run, off);
            const float mx = fmaxf(m_run, m_o);
            const float ref = (mx == LC_NEG_INF) ? 0.f : mx;
            const float sa = lc_exp2_rel(m_run, ref);
            const float sb = lc_exp2_rel(m_o, ref);
            l_run = l_run * sa + l_o * sb;
            m_run = mx;
#pragma unroll
            for (int g = 0; g < G; ++g) {
                const float sag = lc_row_bcast_n(sa, g), sbg = lc_row_bcast_n(sb, g);
#pragma unroll
                for (int i = 0; i < 8; ++i) {
                    const float a_o = __shfl_xor(acc[g][i], off);
                    acc[g][i] = acc[g][i] * sag + a_o * sbg;
                }
            }
        }
        if (lane < 16) {
            if (lane < G) { comb_ml[wave][lane][0] = m_run; comb_ml[wave][lane][1] = l_run; }
#pragma unroll
            for (int g = 0; g < G; ++g) {
#pragma unroll
                for (int i = 0; i < 8; ++i) comb_acc[wave][g][8 * lane + i] = acc[g][i];
            }
        }
        __syncthreads();
        // one float4 slot of the split's partial per thread, stored at agent scope
        float* pml = a.part_ml + ((size_t)bh * S + s) * G * 2;
        const __amdgpu_buffer_rsrc_t pacc_w = lc_buffer(a.part_acc + ((size_t)bh * S + s) * G * LC_D);
        for (int v = tid; v < G * (LC_D / 4); v += LC_DEC_THREADS) {
            const int g = v / (LC_D / 4), c4 = v % (LC_D / 4);
            float mx = LC_NEG_INF;
#pragma unroll
            for (int w = 0; w < LC_DEC_THREADS / 64; ++w) mx = fmaxf(mx, comb_ml[w][g][0]);
            float4 num = make_float4(0.f, 0.f, 0.f, 0.f);
            float den = 0.f;
#pragma unroll
            for (int w = 0; w < LC_DEC_THREADS / 64; ++w) {
                const float mw = comb_ml[w][g][0];
                const float sc = (mw == LC_NEG_INF) ? 0.f : exp2f(mw - mx);
                const float4 x = *reinterpret_cast<const float4*>(&comb_acc[w][g][4 * c4]);
                num.x = fmaf(x.x, sc, num.x); num.y = fmaf(x.y, sc, num.y);
                num.z = fmaf(x.z, sc, num.z); num.w = fmaf(x.w, sc, num.w);
                den = fmaf(comb_ml[w][g][1], sc, den);
            }
            lc_store_agent4(pacc_w, v * 16, num);
            if (c4 == 0) { lc_store_agent(&pml[2 * g], mx); lc_store_agent(&pml[2 * g + 1], den); }
        }
    }

    // ---- the last split to arrive merges (log-sum-exp merge of the partial results)
    if (!lc_arrive_last(&ix.sync[bh * 4 + 1], S, &last_sh)) return;

    // The accumulator partials do not depend on the scales, so their loads go out first and fly
    // while the (m, l) pairs are fetched and turned into per-split scales.
    const __amdgpu_buffer_rsrc_t pacc_r = lc_buffer(a.part_acc + (size_t)bh * S * G * LC_D);
    const float* pml = a.part_ml + (size_t)bh * S * G * 2;
    const int n_part = (n_tok > 0) ? S_eff : 0;
    constexpr int NV = G * (LC_D / 4);                       // float4 slots of the output
    constexpr int WAYS = (LC_DEC_THREADS / NV) > 0 ? (LC_DEC_THREADS / NV) : 1;
    constexpr int MR = (G <= 4) ? 16 : 8;                    // partials per round and thread
    const int v = tid % NV, wy = tid / NV;
    const int g = v / (LC_D / 4), c4 = v % (LC_D / 4);
    float4 x[MR];
    auto load_round = [&](int sp0) {
#pragma unroll
        for (int k = 0; k < MR; ++k) {
            const int spc = min(sp0 + k * WAYS, n_part - 1);
            x[k] = lc_load_agent4(pacc_r, ((spc * G + g) * LC_D + 4 * c4) * 4);
        }
    };
    if (wy < WAYS && n_part > 0) load_round(wy);
    // partial (m, l) of every split -> LDS; per head: global max, scale of each split, denominator
    for (int e = tid; e < n_part * G; e += LC_DEC_THREADS) {
        mrg_m[e] = lc_load_agent(pml + 2 * e);
        mrg_l[e] = lc_load_agent(pml + 2 * e + 1);
    }
    __syncthreads();
    for (int gg = wave; gg < G; gg += LC_DEC_THREADS / 64) {
        float mx = LC_NEG_INF;
        for (int sp = lane; sp < n_part; sp += 64) mx = fmaxf(mx, mrg_m[sp * G + gg]);
        mx = lc_max64(mx);
        float den = 0.f;
        for (int sp = lane; sp < n_part; sp += 64) {
            const float ms = mrg_m[sp * G + gg];
            const float sc = (ms == LC_NEG_INF) ? 0.f : exp2f(ms - mx);
            mrg_m[sp * G + gg] = sc;                    // from here on: the split's scale
            den = fmaf(mrg_l[sp * G + gg], sc, den);
        }
        den = lc_sum64(den);
        if (lane == 0) { mrg_hd[2 * gg] = mx; mrg_hd[2 * gg + 1] = den; }
    }
    __syncthreads();
    float4 acc4 = make_float4(0.f, 0.f, 0.f, 0.f);
    if (wy < WAYS) {
        for (int sp0 = wy; sp0 < n_part; sp0 += MR * WAYS) {
            if (sp0 != wy) load_round(sp0);
#pragma unroll
            for (int k = 0; k < MR; ++k) {
                const int sp = sp0 + k * WAYS;
                const float sc = sp < n_part ? mrg_m[sp * G + g] : 0.f;
                acc4.x = fmaf(x[k].x, sc, acc4.x);
                acc4.y = fmaf(x[k].y, sc, acc4.y);
                acc4.z = fmaf(x[k].z, sc, acc4.z);
                acc4.w = fmaf(x[k].w, sc, acc4.w);
            }
        }
        if (WAYS > 1 && wy > 0) mrg_red[(wy - 1) * NV + v] = acc4;
    }
    __syncthreads();
    if (wy == 0) {
#pragma unroll
        for (int k = 1; k < WAYS; ++k) {
            const float4 o4 = mrg_red[(k - 1) * NV + v];
            acc4.x += o4.x; acc4.y += o4.y; acc4.z += o4.z; acc4.w += o4.w;
        }
        const float mx = mrg_hd[2 * g], den = mrg_hd[2 * g + 1];
        const float inv = den > 0.f ? 1.0f / den : 0.f;
        const size_t o = ((size_t)b * ix.H * G + (size_t)h * G + g);
        *reinterpret_cast<float4*>(a.out + o * LC_D + 4 * c4) =
            make_float4(acc4.x * inv, acc4.y * inv, acc4.z * inv, acc4.w * inv);
        if (a.lse && c4 == 0) a.lse[o] = den > 0.f ? (mx + log2f(den)) * LC_LN2 : LC_NEG_INF;
    }
    if (tid == 0) ix.sync[bh * 4 + 1] = 0;
}

template <int G>
static int launch_decode_g(const LcDecodeArgs& a, int splits, hipStream_t stream) {
    hipLaunchKernelGGL((lc_decode_kernel<G, false, 1>), dim3(splits, a.ix.H, a.ix.B), dim3(LC_DEC_THREADS), 0, stream, a);
    LC_HIP_CHECK(hipGetLastError());
    return LC_OK;
}

static void fill_common(LcDecodeArgs& a, const lc_index* idx, const LcWs& ws, const void* q, const void* K,
                        const void* V, const int64_t ks[3], float* out, float* lse) {
    a.ix = idx->dev;
    a.q = static_cast<const uint16_t*>(q);
    a.K = static_cast<const uint16_t*>(K);
    a.V = static_cast<const uint16_t*>(V);
    a.ks_seq = ks[0];
    a.ks_head = ks[1];
    a.ks_tok = ks[2];
    a.ids = nullptr;
    a.counts = nullptr;
    a.cap = 0;
    a.part_acc = ws.part_acc;
    a.part_ml = ws.part_ml;
    a.out = out;
    a.lse = lse;
    a.keys = nullptr;
    a.ids_out = nullptr;
    a.counts_out = nullptr;
    a.budget = 0;
    a.sink = 0;
    a.ew = 0;
    a.max_tokens = idx->cfg.max_tokens;
}

int lc_launch_decode(const lc_index* idx, const LcWs& ws, const void* q, const void* K, const void* V,
                     const int64_t ks[3], const int32_t* ids, const int32_t* counts, int cap, int G,
                     int splits, float* out, float* lse, hipStream_t stream) {
    LcDecodeArgs a;
    fill_common(a, idx, ws, q, K, V, ks, out, lse);
    a.ids = ids;
    a.counts = counts;
    a.cap = cap;
    switch (G) {
        case 1: return launch_decode_g<1>(a, splits, stream);
        case 2: return launch_decode_g<2>(a, splits, stream);
        case 3: return launch_decode_g<3>(a, splits, stream);
        case 4: return launch_decode_g<4>(a, splits, stream);
        case 5: return launch_decode_g<5>(a, splits, stream);
        case 6: return launch_decode_g<6>(a, splits, stream);
        case 7: return launch_decode_g<7>(a, splits, stream);
        case 8: return launch_decode_g<8>(a, splits, stream);
    }
    return LC_ERR_BAD_SHAPE;
}

// ---- fused step
// Rows of 64 chunks per wavefront that the kernel instances hold in registers: a (sequence, head)
// with up to 256 * EC chunks runs in the smallest instance that holds it.
#define LC_DEC_EC_MAX 16

bool lc_decode_fused_fits(int G, int max_M) {
    return G >= 1 && G <= LC_MAX_GROUP && max_M <= LC_DEC_THREADS * LC_DEC_EC_MAX;
}

template <int G, int EC>
static int launch_fused_ge(const LcDecodeArgs& a, int splits, hipStream_t stream) {
    // key and length of every chunk, touched only when the cutoff bin overflows its short list
    const size_t lds = (size_t)EC * LC_DEC_THREADS * 8;
    if (lds > 16 * 1024)        // static + dynamic may pass the default per-workgroup allowance
        LC_HIP_CHECK(hipFuncSetAttribute(reinterpret_cast<const void*>(&lc_decode_kernel<G, true, EC>),
                                         hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));
    hipLaunchKernelGGL((lc_decode_kernel<G, true, EC>), dim3(splits, a.ix.H, a.ix.B), dim3(LC_DEC_THREADS), lds, stream, a);
    LC_HIP_CHECK(hipGetLastError());
    return LC_OK;
}
template <int G>
static int launch_fused_g(const LcDecodeArgs& a, int splits, hipStream_t stream) {
    if (a.ew <= 2) return launch_fused_ge<G, 2>(a, splits, stream);
    if (a.ew <= 4) return launch_fused_ge<G, 4>(a, splits, stream);
    if (a.ew <= 6) return launch_fused_ge<G, 6>(a, splits, stream);
    if (a.ew <= 10) return launch_fused_ge<G, 10>(a, splits, stream);
    return launch_fused_ge<G, LC_DEC_EC_MAX>(a, splits, stream);
}

int lc_launch_decode_fused(const lc_index* idx, const LcWs& ws, const void* q, const void* K, const void* V,
                           const int64_t ks[3], int G, int splits, int budget, int32_t* ids_out,
                           int32_t* counts_out, int cap, int max_M, float* out, float* lse, hipStream_t stream) {
    LcDecodeArgs a;
    fill_common(a, idx, ws, q, K, V, ks, out, lse);
    a.keys = ws.keys;
    a.ids_out = ids_out;
    a.counts_out = counts_out;
    a.cap = cap;
    a.budget = budget;
    a.sink = idx->cfg.sink_tokens;
    a.ew = ((max_M > 0 ? max_M : 1) + LC_DEC_THREADS - 1) / LC_DEC_THREADS;
    if (a.ew > LC_DEC_EC_MAX) return LC_ERR_CAPACITY;
    switch (G) {
        case 1: return launch_fused_g<1>(a, splits, stream);
        case 2: return launch_fused_g<2>(a, splits, stream);
        case 3: return launch_fused_g<3>(a, splits, stream);
        case 4: return launch_fused_g<4>(a, splits, stream);
        case 5: return launch_fused_g<5>(a, splits, stream);
        case 6: return launch_fused_g<6>(a, splits, stream);
        case 7: return launch_fused_g<7>(a, splits, stream);
        case 8: return launch_fused_g<8>(a, splits, stream);
    }
    return LC_ERR_BAD_SHAPE;
}
