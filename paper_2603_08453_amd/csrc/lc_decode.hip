// Sparse attention for one decode step: split-K flash-decode over the selected
// chunks (plus the open tail), merged by the last split to finish.
//
// Grid (split, KV head, sequence), 256 threads = 16 groups of 16 lanes.  A group
// owns a contiguous run of the split's tokens; its 16 lanes each hold 8 of the
// 128 columns, so one K (or V) row is one 16-byte load per lane and four rows
// make a full 1 KiB wavefront load.  Logits for the G query heads of the group
// are reduced across the 16 lanes; the softmax is kept online in base 2.
#include "lc_device.h"
#include "lc_internal.h"

#define LC_DEC_THREADS 256
#define LC_DEC_GROUPS 16
#define LC_DEC_MIN_TOKENS_PER_SPLIT 64
#define LC_DEC_MAX_SPLITS 256
#define LC_DEC_TILE 2048          // tokens of a split whose cache rows are resolved into LDS at a time
#define LC_LOG2E 1.4426950408889634f
#define LC_LN2 0.6931471805599453f

LC_STAMP_DECL(lc_dbg_decode)

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
    int id_cap_lds;       // entries of the LDS run table
};

template <int G>
__global__ void __launch_bounds__(LC_DEC_THREADS)
lc_decode_kernel(const LcDecodeArgs a) {
    extern __shared__ int lds_dyn[];
    __shared__ int scan_sh[8];
    __shared__ int rows[LC_DEC_TILE];
    __shared__ int last_sh;
    __shared__ float comb_ml[LC_DEC_THREADS / 64][G][2];
    __shared__ __attribute__((aligned(16))) float comb_acc[LC_DEC_THREADS / 64][G][LC_D];
    __shared__ float mrg_m[LC_DEC_MAX_SPLITS * G];
    __shared__ float mrg_l[LC_DEC_MAX_SPLITS * G];
    __shared__ float mrg_hd[2 * G];
    __shared__ float4 mrg_red[LC_DEC_THREADS];

    // tokens per batch of loads; two batches are in flight per group (the next one is issued
    // before the current one is consumed)
    constexpr int U = (G <= 4) ? 4 : 2;
    const LcDev& ix = a.ix;
    const int s = blockIdx.x, S = gridDim.x, h = blockIdx.y, b = blockIdx.z;
    const int bh = b * ix.H + h;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int sub = tid & 15, grp = tid >> 4;

    LC_STAMP0(lc_dbg_decode, 0);
    const int* bnd = ix.bounds + (size_t)b * (ix.cap[0] + 1);
    const int32_t* ids = a.ids + (size_t)bh * a.cap;
    // independent loads first: the id a thread will need is fetched before the count is known,
    // and so are the query fragments (lane `sub` holds columns [8 sub, 8 sub + 8) of each head)
    const int id_first = (tid < a.cap) ? ids[tid] : 0;
    uint4 qraw[G];
    {
        const uint16_t* qb = a.q + ((size_t)b * ix.H * G + (size_t)h * G) * LC_D;
#pragma unroll
        for (int g = 0; g < G; ++g) qraw[g] = *reinterpret_cast<const uint4*>(qb + g * LC_D + 8 * sub);
    }
    const int T = ix.state[bh * 4 + 0];
    const int M = ix.state[bh * 4 + 1];
    int n_ids = a.counts[bh];
    n_ids = max(0, min(n_ids, min(a.cap, a.id_cap_lds)));

    // ---- run table in LDS: start row and exclusive token prefix of each selected chunk,
    // then the open tail as the last run.
    int* run_start = lds_dyn;                       // [n_ids + 1]
    int* run_off = lds_dyn + a.id_cap_lds + 1;      // [n_ids + 2]
    int carry = 0;
    for (int t0 = 0; t0 < n_ids + 1; t0 += LC_DEC_THREADS) {
        const int i = t0 + tid;
        int st = 0, ln = 0;
        if (i < n_ids) {
            const int id = max(0, min(t0 == 0 ? id_first : ids[i], M - 1));
            st = bnd[id];
            ln = bnd[id + 1] - st;
        } else if (i == n_ids) {
            st = bnd[M];
            ln = T - st;
        }
        int tot;
        const int ex = lc_block_scan<LC_DEC_THREADS>(ln, scan_sh, &tot);
        if (i <= n_ids) { run_start[i] = st; run_off[i] = carry + ex; }
        carry += tot;
    }
    LC_STAMP0(lc_dbg_decode, 1);
    const int n_runs = n_ids + 1;
    const int n_tok = carry;
    if (tid == 0) run_off[n_runs] = n_tok;
    __syncthreads();

    int S_eff = (n_tok + LC_DEC_MIN_TOKENS_PER_SPLIT - 1) / LC_DEC_MIN_TOKENS_PER_SPLIT;
    S_eff = max(1, min(S, S_eff));

    if (s < S_eff) {
        const int lo = (int)(((long long)n_tok * s) / S_eff);
        const int hi = (int)(((long long)n_tok * (s + 1)) / S_eff);
        float qf[G][8];
        {
            const float scale = 0.08838834764831845f * LC_LOG2E;     // log2(e) / sqrt(128)
#pragma unroll
            for (int g = 0; g < G; ++g) {
                lc_unpack8(qraw[g], qf[g]);
#pragma unroll
                for (int i = 0; i < 8; ++i) qf[g][i] *= scale;
            }
        }
        float m[G], l[G], acc[G][8];
#pragma unroll
        for (int g = 0; g < G; ++g) {
            m[g] = LC_NEG_INF;
            l[g] = 0.f;
#pragma unroll
            for (int i = 0; i < 8; ++i) acc[g][i] = 0.f;
        }
        const uint16_t* Kb = a.K + (size_t)b * a.ks_seq + (size_t)h * a.ks_head;
        const uint16_t* Vb = a.V + (size_t)b * a.ks_seq + (size_t)h * a.ks_head;

        // K and V rows of up to U tokens starting at position tt of the tile, all loads issued at once
        int t_end = 0;
        auto issue = [&](int tt, uint4 (&kv)[U], uint4 (&vv)[U]) {
#pragma unroll
            for (int u = 0; u < U; ++u) {
                if (tt + u < t_end) {
                    const long long row = rows[tt + u];
                    kv[u] = *reinterpret_cast<const uint4*>(Kb + row * a.ks_tok + 8 * sub);
                    vv[u] = *reinterpret_cast<const uint4*>(Vb + row * a.ks_tok + 8 * sub);
                }
            }
        };
        // logits of the U tokens for the G heads, one online-softmax update, then P.V
        auto consume = [&](int tt, const uint4 (&kv)[U], const uint4 (&vv)[U]) {
            float x[U][G];
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const bool live = tt + u < t_end;
                float kf[8];
                if (live) lc_unpack8(kv[u], kf);
#pragma unroll
                for (int g = 0; g < G; ++g) {
                    float p = 0.f;
                    if (live) {
#pragma unroll
                        for (int i = 0; i < 8; ++i) p = fmaf(kf[i], qf[g][i], p);
                    }
                    p = lc_sum16(p);
                    x[u][g] = live ? p : LC_NEG_INF;
                }
            }
#pragma unroll
            for (int g = 0; g < G; ++g) {
                float mx = m[g];
#pragma unroll
                for (int u = 0; u < U; ++u) mx = fmaxf(mx, x[u][g]);
                const float sc = exp2f(m[g] - mx);          // m = -inf, mx finite: 0
                m[g] = mx;
                l[g] *= sc;
#pragma unroll
                for (int i = 0; i < 8; ++i) acc[g][i] *= sc;
            }
#pragma unroll
            for (int u = 0; u < U; ++u) {
                if (tt + u < t_end) {
                    float vf[8];
                    lc_unpack8(vv[u], vf);
#pragma unroll
                    for (int g = 0; g < G; ++g) {
                        const float p = exp2f(x[u][g] - m[g]);
                        l[g] += p;
#pragma unroll
                        for (int i = 0; i < 8; ++i) acc[g][i] = fmaf(p, vf[i], acc[g][i]);
                    }
                }
            }
        };

        LC_STAMP0(lc_dbg_decode, 8);
        // The split's tokens are handled in tiles; for each tile the workgroup first writes the cache
        // row of every token into LDS (one binary search over the run table per token, in parallel),
        // then every group streams a contiguous slice of the tile with two batches of loads in flight.
        for (int tile0 = lo; tile0 < hi; tile0 += LC_DEC_TILE) {
            const int tl = min(LC_DEC_TILE, hi - tile0);
            __syncthreads();
            for (int i = tid; i < tl; i += LC_DEC_THREADS) {
                const int tok = tile0 + i;
                int lo_r = 0, hi_r = n_runs;            // run_off[lo_r] <= tok < run_off[hi_r]
                while (hi_r - lo_r > 1) {
                    const int mid = (lo_r + hi_r) >> 1;
                    if (run_off[mid] <= tok) lo_r = mid; else hi_r = mid;
                }
                rows[i] = run_start[lo_r] + (tok - run_off[lo_r]);
            }
            __syncthreads();
            const int per = (tl + LC_DEC_GROUPS - 1) / LC_DEC_GROUPS;
            int t = min(tl, grp * per);
            t_end = min(tl, t + per);
            uint4 kA[U], vA[U], kB[U], vB[U];
            if (t < t_end) issue(t, kA, vA);
            while (t < t_end) {
                if (t + U < t_end) issue(t + U, kB, vB);
                consume(t, kA, vA);
                t += U;
                if (t >= t_end) break;
                if (t + U < t_end) issue(t + U, kA, vA);
                consume(t, kB, vB);
                t += U;
            }
        }

        LC_STAMP0(lc_dbg_decode, 2);
        // ---- combine the 4 groups of a wave (xor 16, 32), then the waves through LDS
#pragma unroll
        for (int off = 16; off < 64; off <<= 1) {
#pragma unroll
            for (int g = 0; g < G; ++g) {
                const float m_o = __shfl_xor(m[g], off);
                const float l_o = __shfl_xor(l[g], off);
                const float mx = fmaxf(m[g], m_o);
                const float sa = (m[g] == LC_NEG_INF) ? 0.f : exp2f(m[g] - mx);
                const float sb = (m_o == LC_NEG_INF) ? 0.f : exp2f(m_o - mx);
                l[g] = l[g] * sa + l_o * sb;
#pragma unroll
                for (int i = 0; i < 8; ++i) {
                    const float a_o = __shfl_xor(acc[g][i], off);
                    acc[g][i] = acc[g][i] * sa + a_o * sb;
                }
                m[g] = mx;
            }
        }
        if (lane < 16) {
#pragma unroll
            for (int g = 0; g < G; ++g) {
                if (lane == 0) { comb_ml[wave][g][0] = m[g]; comb_ml[wave][g][1] = l[g]; }
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

    LC_STAMP0(lc_dbg_decode, 3);
    // ---- the last split to arrive merges (log-sum-exp merge of the partial results)
    if (!lc_arrive_last(&ix.sync[bh * 4 + 1], S, &last_sh)) return;

    LC_STAMP(lc_dbg_decode, 4);
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
    LC_STAMP(lc_dbg_decode, 5);
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
    LC_STAMP(lc_dbg_decode, 6);
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
    LC_STAMP(lc_dbg_decode, 7);
    if (tid == 0) ix.sync[bh * 4 + 1] = 0;
}

template <int G>
static int launch_decode_g(const LcDecodeArgs& a, int splits, hipStream_t stream) {
    const size_t lds = (size_t)(2 * a.id_cap_lds + 4) * sizeof(int);
    if (lds > 48 * 1024)
        LC_HIP_CHECK(hipFuncSetAttribute(reinterpret_cast<const void*>(&lc_decode_kernel<G>),
                                         hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));
    hipLaunchKernelGGL(lc_decode_kernel<G>, dim3(splits, a.ix.H, a.ix.B), dim3(LC_DEC_THREADS), lds, stream, a);
    LC_HIP_CHECK(hipGetLastError());
    return LC_OK;
}

int lc_launch_decode(const lc_index* idx, const LcWs& ws, const void* q, const void* K, const void* V,
                     const int64_t ks[3], const int32_t* ids, const int32_t* counts, int cap, int G,
                     int splits, float* out, float* lse, hipStream_t stream) {
    LcDecodeArgs a;
    a.ix = idx->dev;
    a.q = static_cast<const uint16_t*>(q);
    a.K = static_cast<const uint16_t*>(K);
    a.V = static_cast<const uint16_t*>(V);
    a.ks_seq = ks[0];
    a.ks_head = ks[1];
    a.ks_tok = ks[2];
    a.ids = ids;
    a.counts = counts;
    a.cap = cap;
    a.part_acc = ws.part_acc;
    a.part_ml = ws.part_ml;
    a.out = out;
    a.lse = lse;
    int max_M = 0;
    for (int b = 0; b < idx->B; ++b)
        if (idx->M[b] > max_M) max_M = idx->M[b];
    a.id_cap_lds = cap < max_M ? cap : max_M;          // a (sequence, head) never lists more ids than it has chunks
    if (a.id_cap_lds < 1) a.id_cap_lds = 1;
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
