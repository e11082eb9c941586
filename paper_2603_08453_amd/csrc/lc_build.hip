// Index construction (prefill side) and the lazy update for streamed tokens.
//
// Build, per (sequence, KV head):
//   lc_pool_kernel    chunk representative = mean-pooled keys; covering radius; unit direction
//   lc_kmeans_*       spherical k-means on unit directions: strided init, then
//                     `iters` x (assign by largest inner product, normalised-sum update)
//   lc_anc_kernel     chunk -> ancestor at the new level
//   lc_node_kernel    node center, radius over all descendant chunks' balls, counts, direction
// Append: lc_append_kernel writes the token's k, v; on a chunk close it pools the
// open tail, finds the level-1 node of nearest direction and updates the path to the top.
//
// Every reduction runs in a fixed order, so results are reproducible run to run.
#include "lc_device.h"
#include "lc_internal.h"

#define LC_BT 256                 // threads per block
#define LC_BG (LC_BT / 16)        // 16-lane groups per block
#define LC_RADIUS_PAD 4e-6f       // stored radii are inflated by this relative amount so that
                                  // float32 rounding in the distance never leaves a member outside

__device__ __forceinline__ float lc_pad_radius(float r) { return r > 0.f ? r * (1.0f + LC_RADIUS_PAD) : r; }

// ---------------------------------------------------------------------------------
// pooling of rows [lo, hi) of one (sequence, head) key cache; block-wide.
// On return every lane holds, for its 8 columns [8 sub, 8 sub + 8), the stored center
// `mu` (rounded to bfloat16 first if the chunk level is stored that way, so that the radius
// covers the tokens around the value that is stored), and all threads hold the stored radius.
// sh: LC_BG * 128 + LC_BG floats.
// ---------------------------------------------------------------------------------
#define LC_POOL_KEEP 8            // rows per 16-lane group that stay in registers between the two passes (chunks up to 128 tokens are read once)
__device__ __forceinline__ void lc_pool_rows(const uint16_t* __restrict__ Kbh, long long ks_tok, int lo, int hi,
                                             int geometry, bool round_bf16, float* sh, float (&mu)[8], float* radius) {
    const int tid = threadIdx.x, sub = tid & 15, grp = tid >> 4;
    float sum[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) sum[i] = 0.f;
    uint4 keep[LC_POOL_KEEP];
#pragma unroll
    for (int k = 0; k < LC_POOL_KEEP; ++k) {
        const int r = lo + grp + k * LC_BG;
        keep[k] = make_uint4(0u, 0u, 0u, 0u);
        if (r < hi) keep[k] = *reinterpret_cast<const uint4*>(Kbh + (long long)r * ks_tok + 8 * sub);
    }
#pragma unroll
    for (int k = 0; k < LC_POOL_KEEP; ++k) {          // (rows past the chunk hold zeros: they add nothing)
        float f[8];
        lc_unpack8(keep[k], f);
#pragma unroll
        for (int i = 0; i < 8; ++i) sum[i] += f[i];
    }
    for (int r = lo + grp + LC_POOL_KEEP * LC_BG; r < hi; r += LC_BG) {
        const uint4 v = *reinterpret_cast<const uint4*>(Kbh + (long long)r * ks_tok + 8 * sub);
        float f[8];
        lc_unpack8(v, f);
#pragma unroll
        for (int i = 0; i < 8; ++i) sum[i] += f[i];
    }
    __syncthreads();
#pragma unroll
    for (int i = 0; i < 8; ++i) sh[grp * LC_D + 8 * sub + i] = sum[i];
    __syncthreads();
    const float inv_n = 1.0f / (float)(hi - lo);
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        float s = 0.f;
        for (int g = 0; g < LC_BG; ++g) s += sh[g * LC_D + 8 * sub + i];
        mu[i] = s * inv_n;
    }
    if (geometry == LC_GEOMETRY_PAPER_UNIT) {
        float n2 = 0.f;
#pragma unroll
        for (int i = 0; i < 8; ++i) n2 = fmaf(mu[i], mu[i], n2);
        n2 = lc_sum16(n2);
        if (n2 > 0.f) {
            const float inv = 1.0f / sqrtf(n2);
#pragma unroll
            for (int i = 0; i < 8; ++i) mu[i] *= inv;
        } else {
#pragma unroll
            for (int i = 0; i < 8; ++i) mu[i] = (sub == 0 && i == 0) ? 1.f : 0.f;
        }
        if (round_bf16) {
#pragma unroll
            for (int i = 0; i < 8; ++i) mu[i] = lc_round_bf16(mu[i]);
        }
        *radius = 0.f;
        __syncthreads();
        return;
    }
    if (round_bf16) {
#pragma unroll
        for (int i = 0; i < 8; ++i) mu[i] = lc_round_bf16(mu[i]);
    }
    float far2 = 0.f;
    auto reach = [&](const uint4& v) {
        float f[8];
        lc_unpack8(v, f);
        float d2 = 0.f;
#pragma unroll
        for (int i = 0; i < 8; ++i) { const float t = f[i] - mu[i]; d2 = fmaf(t, t, d2); }
        d2 = lc_sum16(d2);
        far2 = fmaxf(far2, d2);
    };
#pragma unroll
    for (int k = 0; k < LC_POOL_KEEP; ++k)
        if (lo + grp + k * LC_BG < hi) reach(keep[k]);
    for (int r = lo + grp + LC_POOL_KEEP * LC_BG; r < hi; r += LC_BG)
        reach(*reinterpret_cast<const uint4*>(Kbh + (long long)r * ks_tok + 8 * sub));
    __syncthreads();
    if (sub == 0) sh[grp] = far2;
    __syncthreads();
    float mx = 0.f;
    for (int g = 0; g < LC_BG; ++g) mx = fmaxf(mx, sh[g]);
    *radius = lc_pad_radius(sqrtf(mx));
    __syncthreads();
}

// unit direction of the 8-column fragments (zero vector -> e_0)
__device__ __forceinline__ void lc_unit_frag(const float (&v)[8], int sub, float (&u)[8]) {
    float n2 = 0.f;
#pragma unroll
    for (int i = 0; i < 8; ++i) n2 = fmaf(v[i], v[i], n2);
    n2 = lc_sum16(n2);
    if (n2 > 0.f) {
        const float inv = 1.0f / sqrtf(n2);
#pragma unroll
        for (int i = 0; i < 8; ++i) u[i] = v[i] * inv;
    } else {
#pragma unroll
        for (int i = 0; i < 8; ++i) u[i] = (sub == 0 && i == 0) ? 1.f : 0.f;
    }
}

__device__ __forceinline__ void lc_store8(float* p, const float (&v)[8]) {
    *reinterpret_cast<float4*>(p) = make_float4(v[0], v[1], v[2], v[3]);
    *reinterpret_cast<float4*>(p + 4) = make_float4(v[4], v[5], v[6], v[7]);
}
__device__ __forceinline__ void lc_load8(const float* p, float (&v)[8]) {
    const float4 a = *reinterpret_cast<const float4*>(p);
    const float4 b = *reinterpret_cast<const float4*>(p + 4);
    v[0] = a.x; v[1] = a.y; v[2] = a.z; v[3] = a.w;
    v[4] = b.x; v[5] = b.y; v[6] = b.z; v[7] = b.w;
}

// Chunk-level center of node n, columns [8 sub, 8 sub + 8), in the index's storage format.
// (`v` already holds bfloat16-representable values when the level is stored as bfloat16.)
__device__ __forceinline__ void lc_c0_store8(const LcDev& ix, size_t n, int sub, const float (&v)[8]) {
    if (ix.c0_bf16) {
        uint4 w;
        w.x = (__float_as_uint(v[0]) >> 16) | (__float_as_uint(v[1]) & 0xffff0000u);
        w.y = (__float_as_uint(v[2]) >> 16) | (__float_as_uint(v[3]) & 0xffff0000u);
        w.z = (__float_as_uint(v[4]) >> 16) | (__float_as_uint(v[5]) & 0xffff0000u);
        w.w = (__float_as_uint(v[6]) >> 16) | (__float_as_uint(v[7]) & 0xffff0000u);
        *reinterpret_cast<uint4*>(reinterpret_cast<uint16_t*>(ix.center[0]) + n * LC_D + 8 * sub) = w;
    } else {
        lc_store8(ix.center[0] + n * LC_D + 8 * sub, v);
    }
}
__device__ __forceinline__ void lc_c0_load8(const LcDev& ix, size_t n, int sub, float (&v)[8]) {
    if (ix.c0_bf16) {
        const uint4 w = *reinterpret_cast<const uint4*>(reinterpret_cast<const uint16_t*>(ix.center[0]) + n * LC_D + 8 * sub);
        lc_unpack8(w, v);
    } else {
        lc_load8(ix.center[0] + n * LC_D + 8 * sub, v);
    }
}

// ---------------------------------------------------------------------------------
// level 0: one wavefront per chunk
// ---------------------------------------------------------------------------------
// The four 16-lane groups of a wavefront take the chunk's rows in turn (lane `sub` of a group holds
// columns [8 sub, 8 sub + 8) of a row); the first LC_POOLW_KEEP rows of every group stay in registers
// between the mean pass and the radius pass, so chunks of up to 4 * LC_POOLW_KEEP tokens are read
// once (longer ones find their other rows in the L2 cache the second time).
// No workgroup barrier: the groups' partial sums meet through wavefront shuffles.
#define LC_POOLW_KEEP 8
__device__ __forceinline__ float lc_sum_groups4(float v) { v += __shfl_xor(v, 16); v += __shfl_xor(v, 32); return v; }
__global__ void __launch_bounds__(LC_BT)
lc_pool_kernel(LcDev ix, const uint16_t* K, long long ks_seq, long long ks_head, long long ks_tok,
               int geometry, float* dirs) {
    const int h = blockIdx.y, b = blockIdx.z;
    const int bh = b * ix.H + h;
    const int lane = threadIdx.x & 63, sub = lane & 15, g4 = lane >> 4;
    const int j = blockIdx.x * (LC_BT / 64) + (threadIdx.x >> 6);
    const int M = ix.state[bh * 4 + 1];
    if (j >= M) return;                                            // (whole wavefronts leave: nothing below waits across them)
    const int* bnd = ix.bounds + (size_t)b * (ix.cap[0] + 1);
    const int lo = bnd[j], hi = bnd[j + 1];
    const uint16_t* Kbh = K + b * ks_seq + h * ks_head;
    const bool round_bf16 = ix.c0_bf16 != 0;
    // a batch = LC_POOLW_KEEP rows per group, all loads in flight together (rows past the chunk read as zeros)
    auto load_batch = [&](int base, uint4 (&buf)[LC_POOLW_KEEP]) {
#pragma unroll
        for (int k = 0; k < LC_POOLW_KEEP; ++k) {
            // (no branch around the load -- the compiler would wait for one load before issuing the
            // next; a row past the chunk re-reads the chunk's last row and is zeroed afterwards)
            const int r = base + g4 + 4 * k;
            const uint4 v = *reinterpret_cast<const uint4*>(Kbh + (long long)max(min(r, hi - 1), lo) * ks_tok + 8 * sub);
            buf[k] = r < hi ? v : make_uint4(0u, 0u, 0u, 0u);
        }
    };
    uint4 keep[LC_POOLW_KEEP];
    load_batch(lo, keep);
    float sum[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) sum[i] = 0.f;
    auto add_batch = [&](const uint4 (&buf)[LC_POOLW_KEEP]) {
#pragma unroll
        for (int k = 0; k < LC_POOLW_KEEP; ++k) {                   // (zero rows add nothing)
            float f[8];
            lc_unpack8(buf[k], f);
#pragma unroll
            for (int i = 0; i < 8; ++i) sum[i] += f[i];
        }
    };
    add_batch(keep);
    for (int base = lo + 4 * LC_POOLW_KEEP; base < hi; base += 4 * LC_POOLW_KEEP) {
        uint4 more[LC_POOLW_KEEP];
        load_batch(base, more);
        add_batch(more);
    }
    // The rows stay packed (four registers each) across the two passes: an empty statement that
    // claims to rewrite them keeps the compiler from holding their unpacked copies as well, which
    // would double the registers per row and halve the resident wavefronts.
#pragma unroll
    for (int k = 0; k < LC_POOLW_KEEP; ++k)
        asm volatile("" : "+v"(keep[k].x), "+v"(keep[k].y), "+v"(keep[k].z), "+v"(keep[k].w));
    float mu[8];
    const float inv_n = 1.0f / (float)(hi - lo);
#pragma unroll
    for (int i = 0; i < 8; ++i) mu[i] = lc_sum_groups4(sum[i]) * inv_n;
    float radius = 0.f;
    if (geometry == LC_GEOMETRY_PAPER_UNIT) {
        float un[8];
        lc_unit_frag(mu, sub, un);
#pragma unroll
        for (int i = 0; i < 8; ++i) mu[i] = round_bf16 ? lc_round_bf16(un[i]) : un[i];
    } else {
        if (round_bf16) {
#pragma unroll
            for (int i = 0; i < 8; ++i) mu[i] = lc_round_bf16(mu[i]);
        }
        float far2 = 0.f;
        auto reach = [&](const uint4& v) {
            float f[8];
            lc_unpack8(v, f);
            float d2 = 0.f;
#pragma unroll
            for (int i = 0; i < 8; ++i) { const float t = f[i] - mu[i]; d2 = fmaf(t, t, d2); }
            d2 = lc_sum16(d2);
            far2 = fmaxf(far2, d2);
        };
#pragma unroll
        for (int k = 0; k < LC_POOLW_KEEP; ++k)
            if (lo + g4 + 4 * k < hi) reach(keep[k]);
        for (int base = lo + 4 * LC_POOLW_KEEP; base < hi; base += 4 * LC_POOLW_KEEP) {
            uint4 more[LC_POOLW_KEEP];
            load_batch(base, more);
#pragma unroll
            for (int k = 0; k < LC_POOLW_KEEP; ++k)
                if (base + g4 + 4 * k < hi) reach(more[k]);
        }
        far2 = fmaxf(far2, __shfl_xor(far2, 16));
        far2 = fmaxf(far2, __shfl_xor(far2, 32));
        radius = lc_pad_radius(sqrtf(far2));
    }
    const size_t n = (size_t)bh * ix.cap[0] + j;
    if (g4 == 0) {
        lc_c0_store8(ix, n, sub, mu);
        float u[8];
        lc_unit_frag(mu, sub, u);
        lc_store8(dirs + n * LC_D + 8 * sub, u);
        if (sub == 0) {
            ix.radius[0][n] = radius;
            ix.parent[0][n] = -1;
            ix.ntok[0][n] = hi - lo;
            ix.nchunk[0][n] = 1;
        }
    }
}

// Re-clustering starts from the chunk nodes already in the index: unit directions of their centers.
__global__ void __launch_bounds__(LC_BT)
lc_dirs_kernel(LcDev ix, float* dirs) {
    const int h = blockIdx.y, b = blockIdx.z;
    const int bh = b * ix.H + h;
    const int M = ix.state[bh * 4 + 1];
    const int sub = threadIdx.x & 15;
    const int j = blockIdx.x * LC_BG + (threadIdx.x >> 4);
    if (j >= M) return;
    const size_t n = (size_t)bh * ix.cap[0] + j;
    float mu[8], u[8];
    lc_c0_load8(ix, n, sub, mu);
    lc_unit_frag(mu, sub, u);
    lc_store8(dirs + n * LC_D + 8 * sub, u);
    if (sub == 0) ix.parent[0][n] = -1;
}

// ---------------------------------------------------------------------------------
// spherical k-means
// ---------------------------------------------------------------------------------
// Number of points / clusters of sequence b when clustering level `l` into level l+1.
__device__ __forceinline__ int lc_level_count(const LcDev& ix, int b, int bh, int l) {
    return l == 0 ? ix.state[bh * 4 + 1] : ix.nlev[b * LC_MAX_LEVELS + l];
}

// centroid c starts at point floor(c * N / k)
__global__ void __launch_bounds__(LC_D)
lc_kmeans_init_kernel(LcDev ix, int l, const float* pts, int pts_cap, float* cent, int cent_cap, int* flags) {
    const int c = blockIdx.x, h = blockIdx.y, b = blockIdx.z;
    const int bh = b * ix.H + h;
    if (c == 0 && flags && threadIdx.x < LC_KM_FLAGS) flags[bh * LC_KM_FLAGS + threadIdx.x] = 0;
    const int N = lc_level_count(ix, b, bh, l);
    const int k = ix.nlev[b * LC_MAX_LEVELS + l + 1];
    if (c >= k) return;
    float v = (threadIdx.x == 0) ? 1.f : 0.f;
    if (N > 0) {
        const long long src = ((long long)c * N) / k;
        v = pts[((size_t)bh * pts_cap + src) * LC_D + threadIdx.x];
    }
    cent[((size_t)bh * cent_cap + c) * LC_D + threadIdx.x] = v;
}

// label(i) = argmax_c <x_i, m_c>, ties to the lower c: the one dense contraction of the build
// (N x k x 128 per iteration), on the matrix cores in float32 (v_mfma_f32_16x16x4_f32).
// A wavefront takes 16 points (the A operand, in registers for the whole kernel), the workgroup's
// four wavefronts share centroid tiles staged in LDS (the B operand).  Both operands walk the 128
// dimensions in the same permuted order -- step (t, u) pairs dimension 16 t + 4 kk + u of a point
// with the same dimension of a centroid, kk = lane / 16 being the instruction's K index -- so that
// each lane fetches its share of a row as eight 16-byte pieces.  The result tile leaves lane (q, j)
// with the similarities of points 4 q + r (r < 4) to centroid j of the block; every lane keeps the
// best of its column per point, and the 16 lanes of a row merge (value, then lower id) at the end.
#define LC_AS_PTS 64              // points per workgroup
#define LC_AS_TILE 64             // centroids per LDS tile
#define LC_AS_ROW (LC_D + 4)      // floats per staged centroid row (the pad spreads the 16 rows of a block over the banks)
typedef float lc_f32x4_b __attribute__((ext_vector_type(4)));
// One 16 x 16 block of similarities: the wavefront's 16 points (xa, the A operand) against the 16
// centroid rows of which `brow` is this lane's (already offset by 4 * kk); lane j's centroid has id c.
__device__ __forceinline__ void lc_assign_block(const float4 (&xa)[8], const float* brow, int c, int k,
                                                float (&best)[4], int (&arg)[4]) {
    lc_f32x4_b d = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int t = 0; t < 8; ++t) {
        const float4 mb = *reinterpret_cast<const float4*>(brow + 16 * t);
        d = __builtin_amdgcn_mfma_f32_16x16x4f32(xa[t].x, mb.x, d, 0, 0, 0);
        d = __builtin_amdgcn_mfma_f32_16x16x4f32(xa[t].y, mb.y, d, 0, 0, 0);
        d = __builtin_amdgcn_mfma_f32_16x16x4f32(xa[t].z, mb.z, d, 0, 0, 0);
        d = __builtin_amdgcn_mfma_f32_16x16x4f32(xa[t].w, mb.w, d, 0, 0, 0);
    }
    if (c < k) {
#pragma unroll
        for (int r = 0; r < 4; ++r)
            if (d[r] > best[r]) { best[r] = d[r]; arg[r] = c; }
    }
}
// Two blocks at once: the two accumulators are independent chains, so the matrix pipe is not left
// waiting for one instruction's result before the next can start (a wavefront is alone on its
// SIMD here).  Each block's own sum runs in the same order as in lc_assign_block: same bits.
__device__ __forceinline__ void lc_assign_block2(const float4 (&xa)[8], const float* brow0, const float* brow1,
                                                 int c0, int c1, int k, float (&best)[4], int (&arg)[4]) {
    lc_f32x4_b d0 = {0.f, 0.f, 0.f, 0.f}, d1 = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int t = 0; t < 8; ++t) {
        const float4 m0 = *reinterpret_cast<const float4*>(brow0 + 16 * t);
        const float4 m1 = *reinterpret_cast<const float4*>(brow1 + 16 * t);
        d0 = __builtin_amdgcn_mfma_f32_16x16x4f32(xa[t].x, m0.x, d0, 0, 0, 0);
        d1 = __builtin_amdgcn_mfma_f32_16x16x4f32(xa[t].x, m1.x, d1, 0, 0, 0);
        d0 = __builtin_amdgcn_mfma_f32_16x16x4f32(xa[t].y, m0.y, d0, 0, 0, 0);
        d1 = __builtin_amdgcn_mfma_f32_16x16x4f32(xa[t].y, m1.y, d1, 0, 0, 0);
        d0 = __builtin_amdgcn_mfma_f32_16x16x4f32(xa[t].z, m0.z, d0, 0, 0, 0);
        d1 = __builtin_amdgcn_mfma_f32_16x16x4f32(xa[t].z, m1.z, d1, 0, 0, 0);
        d0 = __builtin_amdgcn_mfma_f32_16x16x4f32(xa[t].w, m0.w, d0, 0, 0, 0);
        d1 = __builtin_amdgcn_mfma_f32_16x16x4f32(xa[t].w, m1.w, d1, 0, 0, 0);
    }
    if (c0 < k) {
#pragma unroll
        for (int r = 0; r < 4; ++r)
            if (d0[r] > best[r]) { best[r] = d0[r]; arg[r] = c0; }
    }
    if (c1 < k) {
#pragma unroll
        for (int r = 0; r < 4; ++r)
            if (d1[r] > best[r]) { best[r] = d1[r]; arg[r] = c1; }
    }
}
// merge the 16 columns of a row: larger similarity wins, equal ones go to the lower centroid id
__device__ __forceinline__ int lc_assign_merge(float bv, int ba) {
    auto merge = [&](float ov, int oa) {
        if (ov > bv || (ov == bv && oa < ba)) { bv = ov; ba = oa; }
    };
    merge(lc_dpp<0xB1>(bv), __builtin_amdgcn_update_dpp(0, ba, 0xB1, 0xF, 0xF, true));
    merge(lc_dpp<0x4E>(bv), __builtin_amdgcn_update_dpp(0, ba, 0x4E, 0xF, 0xF, true));
    merge(lc_dpp<0x141>(bv), __builtin_amdgcn_update_dpp(0, ba, 0x141, 0xF, 0xF, true));
    merge(lc_dpp<0x140>(bv), __builtin_amdgcn_update_dpp(0, ba, 0x140, 0xF, 0xF, true));
    return ba;
}
// `flags` (may be null): flags[bh][t] = iteration t moved a point.  An iteration that moves none is a
// fixed point -- the update would rebuild the same centroids from the same members and every later
// iteration would repeat it -- so from then on the kernels of this (sequence, head) return at once:
// iteration `it` assigns only if it <= 1 or iteration it - 1 moved a point, and leaves its own flag
// at zero otherwise, which passes the verdict on.
__global__ void __launch_bounds__(LC_BT)
lc_kmeans_assign_kernel(LcDev ix, int l, const float* pts, int pts_cap, const float* cent, int cent_cap, int it,
                        int* flags) {
    __shared__ __attribute__((aligned(16))) float tile[LC_AS_TILE * LC_AS_ROW];
    const int h = blockIdx.y, b = blockIdx.z;
    const int bh = b * ix.H + h;
    if (flags && it >= 2 && flags[bh * LC_KM_FLAGS + it - 1] == 0) return;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int j = lane & 15, kk = lane >> 4;
    const int N = lc_level_count(ix, b, bh, l);
    const int k = ix.nlev[b * LC_MAX_LEVELS + l + 1];
    const int i0 = blockIdx.x * LC_AS_PTS + wave * 16;             // this wavefront's first point
    if ((int)blockIdx.x * LC_AS_PTS >= N) return;
    // A operand: point i0 + j, dimensions 16 t + 4 kk + (0..3)
    float4 xa[8];
    {
        const float* row = pts + ((size_t)bh * pts_cap + min(i0 + j, N - 1)) * LC_D + 4 * kk;
#pragma unroll
        for (int t = 0; t < 8; ++t) xa[t] = *reinterpret_cast<const float4*>(row + 16 * t);
    }
    const float* cb = cent + (size_t)bh * cent_cap * LC_D;
    float best[4];
    int arg[4];
#pragma unroll
    for (int r = 0; r < 4; ++r) { best[r] = LC_NEG_INF; arg[r] = 0x7fffffff; }
    // a tile's rows travel global memory -> registers -> LDS; the next tile's loads are issued
    // before the current tile's products, so their latency is covered by the matrix work
    constexpr int PF = LC_AS_TILE * (LC_D / 4) / LC_BT;             // float4 pieces per thread and tile
    float4 pf[PF];
    auto fetch = [&](int c0) {
        const int nc = min(LC_AS_TILE, k - c0);
#pragma unroll
        for (int e = 0; e < PF; ++e) {
            const int v = tid + e * LC_BT;
            const int c = v / (LC_D / 4), q = v % (LC_D / 4);
            pf[e] = make_float4(0.f, 0.f, 0.f, 0.f);
            if (c < nc) pf[e] = *reinterpret_cast<const float4*>(cb + (size_t)(c0 + c) * LC_D + 4 * q);
        }
    };
    fetch(0);
    for (int c0 = 0; c0 < k; c0 += LC_AS_TILE) {
        const int nc = min(LC_AS_TILE, k - c0);
        __syncthreads();                                            // the previous tile has been used
#pragma unroll
        for (int e = 0; e < PF; ++e) {
            const int v = tid + e * LC_BT;
            *reinterpret_cast<float4*>(tile + (v / (LC_D / 4)) * LC_AS_ROW + 4 * (v % (LC_D / 4))) = pf[e];
        }
        if (c0 + LC_AS_TILE < k) fetch(c0 + LC_AS_TILE);
        __syncthreads();
        int cj = 0;
        for (; cj + 16 < nc; cj += 32)
            lc_assign_block2(xa, tile + (cj + j) * LC_AS_ROW + 4 * kk, tile + (cj + 16 + j) * LC_AS_ROW + 4 * kk,
                             c0 + cj + j, c0 + cj + 16 + j, k, best, arg);
        if (cj < nc) lc_assign_block(xa, tile + (cj + j) * LC_AS_ROW + 4 * kk, c0 + cj + j, k, best, arg);
    }
#pragma unroll
    for (int r = 0; r < 4; ++r) {
        const int ba = lc_assign_merge(best[r], arg[r]);
        const int i = i0 + 4 * kk + r;
        if (j == 0 && i < N) {
            int* lab = ix.parent[l] + (size_t)bh * ix.cap[l] + i;
            if (flags && *lab != ba) flags[bh * LC_KM_FLAGS + it] = 1;     // (every writer stores the same value)
            *lab = ba;
        }
    }
}

// Ascending list, in LDS, of the i in [base, base + LC_MEM_WIN) below n with lab[i] == c; returns its
// length in every thread.  Every label is loaded once, coalesced, all loads in flight together;
// positions come from wavefront ballots and one scan of the 64 (row, wavefront) counts, so the order
// is fixed.  cnt: 2 * 64 + 1 ints of LDS; mem: LC_MEM_WIN ints.  All LC_BT threads must call.
#define LC_MEM_WIN 4096
__device__ __forceinline__ int lc_collect_members(const int* __restrict__ lab, int n, int base, int c, int* mem, int* cnt) {
    constexpr int E = LC_MEM_WIN / LC_BT;
    constexpr int W = LC_BT / 64;
    static_assert(E * W == 64, "one wavefront scans the (row, wavefront) counts");
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    int lv[E];
#pragma unroll
    for (int e = 0; e < E; ++e) {
        const int i = base + e * LC_BT + tid;
        lv[e] = i < n ? lab[i] : -1;
    }
    unsigned long long m[E];
#pragma unroll
    for (int e = 0; e < E; ++e) {
        m[e] = __ballot(lv[e] == c);
        if (lane == 0) cnt[e * W + wave] = __popcll(m[e]);
    }
    __syncthreads();
    if (wave == 0) {
        const int v = cnt[lane];
        const int inc = lc_wave_scan_incl(v);
        cnt[64 + lane] = inc - v;
        if (lane == 63) cnt[128] = inc;
    }
    __syncthreads();
#pragma unroll
    for (int e = 0; e < E; ++e) {
        if (lv[e] == c) {
            const unsigned long long below = m[e] & ((1ull << lane) - 1ull);
            mem[cnt[64 + e * W + wave] + __popcll(below)] = base + e * LC_BT + tid;
        }
    }
    __syncthreads();
    return cnt[128];
}

// m_c = normalise(sum of members); a cluster without members (or with a zero sum) keeps m_c.
// One workgroup per cluster: it lists its members (above), then the 16 groups add them up in turn.
__global__ void __launch_bounds__(LC_BT)
lc_kmeans_update_kernel(LcDev ix, int l, const float* pts, int pts_cap, float* cent, int cent_cap, int it,
                        const int* flags) {
    __shared__ float sh[LC_BG * LC_D];
    __shared__ int mem[LC_MEM_WIN];
    __shared__ int cnt[2 * 64 + 1];
    const int c = blockIdx.x, h = blockIdx.y, b = blockIdx.z;
    const int bh = b * ix.H + h;
    if (flags && it >= 1 && flags[bh * LC_KM_FLAGS + it] == 0) return;      // no point moved: the centroids stand
    const int sub = threadIdx.x & 15, grp = threadIdx.x >> 4;
    const int N = lc_level_count(ix, b, bh, l);
    const int k = ix.nlev[b * LC_MAX_LEVELS + l + 1];
    if (c >= k) return;
    const int* lab = ix.parent[l] + (size_t)bh * ix.cap[l];
    float sum[8];
#pragma unroll
    for (int t = 0; t < 8; ++t) sum[t] = 0.f;
    for (int base = 0; base < N; base += LC_MEM_WIN) {
        const int nm = lc_collect_members(lab, N, base, c, mem, cnt);
#pragma unroll 4
        for (int t0 = grp; t0 < nm; t0 += LC_BG) {
            float x[8];
            lc_load8(pts + ((size_t)bh * pts_cap + mem[t0]) * LC_D + 8 * sub, x);
#pragma unroll
            for (int t = 0; t < 8; ++t) sum[t] += x[t];
        }
        __syncthreads();                                            // the list is rewritten by the next window
    }
#pragma unroll
    for (int t = 0; t < 8; ++t) sh[grp * LC_D + 8 * sub + t] = sum[t];
    __syncthreads();
    if (threadIdx.x < 16) {
        float s[8];
#pragma unroll
        for (int t = 0; t < 8; ++t) {
            float a = 0.f;
            for (int g = 0; g < LC_BG; ++g) a += sh[g * LC_D + 8 * sub + t];
            s[t] = a;
        }
        float n2 = 0.f;
#pragma unroll
        for (int t = 0; t < 8; ++t) n2 = fmaf(s[t], s[t], n2);
        n2 = lc_sum16(n2);
        if (n2 > 0.f) {
            const float inv = 1.0f / sqrtf(n2);
#pragma unroll
            for (int t = 0; t < 8; ++t) s[t] *= inv;
            lc_store8(cent + ((size_t)bh * cent_cap + c) * LC_D + 8 * sub, s);
        }
    }
}

// The whole clustering of a small level (up to LC_KS_MAX_N points into up to LC_KS_MAX_K clusters)
// in one kernel, one workgroup per (sequence, head): centroids and labels live in LDS, the
// iterations are separated by workgroup barriers instead of kernel boundaries.  Same steps as the
// three kernels above: strided start, assign (ties to the lower id), normalised member sums (members
// added in ascending order; a cluster without members or with a zero sum keeps its centroid).
#define LC_KS_MAX_N 224
#define LC_KS_MAX_K 64
static inline size_t lc_kmeans_small_lds(int N, int k) {
    return (size_t)((N > 0 ? N : 1) + ((k + 15) & ~15)) * LC_AS_ROW * sizeof(float);
}
__global__ void __launch_bounds__(LC_BT)
lc_kmeans_small_kernel(LcDev ix, int l, const float* pts, int pts_cap, float* cent, int cent_cap, int iters,
                       int x_rows) {
    extern __shared__ __attribute__((aligned(16))) float ks_dyn[];   // x_rows point rows, then the centroid rows
    __shared__ int lab[LC_KS_MAX_N];
    __shared__ int moff[LC_KS_MAX_K + 1];
    __shared__ unsigned short mem[LC_KS_MAX_N];
    __shared__ int changed[2];                    // labels changed in this iteration (one flag per parity of `it`)
    const int h = blockIdx.x, b = blockIdx.y;
    const int bh = b * ix.H + h;
    const int tid = threadIdx.x, sub = tid & 15, grp = tid >> 4, lane = tid & 63, wave = tid >> 6;
    const int j = lane & 15, kk = lane >> 4;
    const int N = min(min(lc_level_count(ix, b, bh, l), LC_KS_MAX_N), x_rows);
    const int k = min(ix.nlev[b * LC_MAX_LEVELS + l + 1], LC_KS_MAX_K);
    const int k16 = (k + 15) & ~15;
    const int rounds = (N + 63) >> 6;
    const float* P = pts + (size_t)bh * pts_cap * LC_D;
    float* X = ks_dyn;
    float* cs = ks_dyn + (size_t)x_rows * LC_AS_ROW;
    for (int v = tid; v < N * (LC_D / 4); v += LC_BT) {
        const int i = v / (LC_D / 4), q = v % (LC_D / 4);
        *reinterpret_cast<float4*>(X + i * LC_AS_ROW + 4 * q) = *reinterpret_cast<const float4*>(P + (size_t)i * LC_D + 4 * q);
    }
    for (int i = tid; i < N; i += LC_BT) lab[i] = 0;
    if (tid < 2) changed[tid] = 0;
    __syncthreads();
    for (int v = tid; v < k16 * LC_D; v += LC_BT) {
        const int c = v / LC_D, t = v % LC_D;
        float m = 0.f;
        if (c < k) m = N > 0 ? X[(int)(((long long)c * N) / k) * LC_AS_ROW + t] : (t == 0 ? 1.f : 0.f);
        cs[c * LC_AS_ROW + t] = m;
    }
    __syncthreads();
    for (int it = 0; it < iters; ++it) {
        for (int i0 = 16 * wave; i0 < N; i0 += 16 * (LC_BT / 64)) {
            float4 xa[8];
            const float* row = X + min(i0 + j, N - 1) * LC_AS_ROW + 4 * kk;
#pragma unroll
            for (int t = 0; t < 8; ++t) xa[t] = *reinterpret_cast<const float4*>(row + 16 * t);
            float best[4];
            int arg[4];
#pragma unroll
            for (int r = 0; r < 4; ++r) { best[r] = LC_NEG_INF; arg[r] = 0x7fffffff; }
            int cj = 0;
            for (; cj + 16 < k; cj += 32)
                lc_assign_block2(xa, cs + (cj + j) * LC_AS_ROW + 4 * kk, cs + (cj + 16 + j) * LC_AS_ROW + 4 * kk,
                                 cj + j, cj + 16 + j, k, best, arg);
            if (cj < k) lc_assign_block(xa, cs + (cj + j) * LC_AS_ROW + 4 * kk, cj + j, k, best, arg);
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                const int ba = lc_assign_merge(best[r], arg[r]);
                const int i = i0 + 4 * kk + r;
                if (j == 0 && i < N) {
                    if (lab[i] != ba) changed[it & 1] = 1;
                    lab[i] = ba;
                }
            }
        }
        if (tid == 0) changed[(it + 1) & 1] = 0;                    // (last read before the previous barrier)
        __syncthreads();
        // An iteration that moves no point is a fixed point: the update would rebuild the same
        // centroids from the same members and every later iteration would repeat it, so the
        // remaining iterations are skipped (the first iteration always runs its update).
        if (it > 0 && changed[it & 1] == 0) break;
        // members of every cluster, ascending, as one list ordered by cluster: counts, offsets, ids
        for (int c = wave; c < k; c += LC_BT / 64) {
            int n = 0;
            for (int r = 0; r < rounds; ++r) {
                const int i = lane + 64 * r;
                n += __popcll(__ballot(i < N && lab[i] == c));
            }
            if (lane == 0) moff[c + 1] = n;
        }
        if (tid == 0) moff[0] = 0;
        __syncthreads();
        if (wave == 0) {
            int v = lane < k ? moff[lane + 1] : 0;
            v = lc_wave_scan_incl(v);
            if (lane < k) moff[lane + 1] = v;
        }
        __syncthreads();
        for (int c = wave; c < k; c += LC_BT / 64) {
            int at = moff[c];
            for (int r = 0; r < rounds; ++r) {
                const int i = lane + 64 * r;
                const bool in = i < N && lab[i] == c;
                const unsigned long long m = __ballot(in);
                if (in) mem[at + __popcll(m & ((1ull << lane) - 1ull))] = (unsigned short)i;
                at += __popcll(m);
            }
        }
        __syncthreads();
        for (int c = grp; c < k; c += LC_BG) {
            float sum[8];
#pragma unroll
            for (int t = 0; t < 8; ++t) sum[t] = 0.f;
            const int j1 = moff[c + 1];
#pragma unroll 4
            for (int jm = moff[c]; jm < j1; ++jm) {
                float x[8];
                lc_load8(X + (int)mem[jm] * LC_AS_ROW + 8 * sub, x);
#pragma unroll
                for (int t = 0; t < 8; ++t) sum[t] += x[t];
            }
            float n2 = 0.f;
#pragma unroll
            for (int t = 0; t < 8; ++t) n2 = fmaf(sum[t], sum[t], n2);
            n2 = lc_sum16(n2);
            if (n2 > 0.f) {
                const float inv = 1.0f / sqrtf(n2);
#pragma unroll
                for (int t = 0; t < 8; ++t) sum[t] *= inv;
                lc_store8(cs + c * LC_AS_ROW + 8 * sub, sum);
            }
        }
        __syncthreads();
    }
    for (int i = tid; i < N; i += LC_BT) ix.parent[l][(size_t)bh * ix.cap[l] + i] = lab[i];
    for (int v = tid; v < k * LC_D; v += LC_BT)
        cent[(size_t)bh * cent_cap * LC_D + v] = cs[(v / LC_D) * LC_AS_ROW + (v % LC_D)];
}

// anc[j] <- label of anc[j] at the level just clustered (anc starts as identity)
__global__ void lc_anc_kernel(LcDev ix, int l, int* anc) {
    const int h = blockIdx.y, b = blockIdx.z;
    const int bh = b * ix.H + h;
    const int M = ix.state[bh * 4 + 1];
    const int j = blockIdx.x * blockDim.x + threadIdx.x;
    if (j >= M) return;
    int* a = anc + (size_t)bh * ix.cap[0];
    const int cur = (l == 0) ? j : a[j];
    a[j] = ix.parent[l][(size_t)bh * ix.cap[l] + cur];
}

// node u of level l+1: center, radius over all descendant chunks, counts, direction
#define LC_NODE_BATCH 8
__global__ void __launch_bounds__(LC_BT)
lc_node_kernel(LcDev ix, int l, const int* anc, const float* cent, int cent_cap, int geometry,
               float* next_pts, int next_cap) {
    __shared__ float sh[LC_BG * LC_D + LC_BG];
    __shared__ int shi[2 * LC_BG];
    __shared__ int mem[LC_MEM_WIN];
    __shared__ int mcnt[2 * 64 + 1];
    const int u = blockIdx.x, h = blockIdx.y, b = blockIdx.z;
    const int bh = b * ix.H + h;
    const int sub = threadIdx.x & 15, grp = threadIdx.x >> 4;
    const int k = ix.nlev[b * LC_MAX_LEVELS + l + 1];
    if (u >= k) return;
    const int M = ix.state[bh * 4 + 1];
    const int* a = anc + (size_t)bh * ix.cap[0];
    const size_t cb = (size_t)bh * ix.cap[0];
    // the node's chunks are listed window by window (lc_collect_members); the 16 groups take them in turn
    float sum[8];
#pragma unroll
    for (int t = 0; t < 8; ++t) sum[t] = 0.f;
    int cnt = 0, tok = 0;
    int nm = 0;
    for (int base = 0; base < M; base += LC_MEM_WIN) {
        nm = lc_collect_members(a, M, base, u, mem, mcnt);
        for (int t0 = grp; t0 < nm; t0 += LC_NODE_BATCH * LC_BG) {  // a batch of rows in flight per group
            float c[LC_NODE_BATCH][8];
            int nt[LC_NODE_BATCH];
#pragma unroll
            for (int q = 0; q < LC_NODE_BATCH; ++q) {
                const int t1 = t0 + q * LC_BG;
                const bool in = t1 < nm;
                nt[q] = -1;
                if (in) {
                    const int j = mem[t1];
                    lc_c0_load8(ix, cb + j, sub, c[q]);
                    nt[q] = ix.ntok[0][cb + j];
                }
            }
#pragma unroll
            for (int q = 0; q < LC_NODE_BATCH; ++q) {
                if (nt[q] >= 0) {
#pragma unroll
                    for (int t = 0; t < 8; ++t) sum[t] += c[q][t];
                    cnt += 1;
                    tok += nt[q];
                }
            }
        }
        if (base + LC_MEM_WIN < M) __syncthreads();                 // the list is rewritten by the next window
    }
#pragma unroll
    for (int t = 0; t < 8; ++t) sh[grp * LC_D + 8 * sub + t] = sum[t];
    if (sub == 0) { shi[grp] = cnt; shi[LC_BG + grp] = tok; }
    __syncthreads();
    int nch = 0, ntk = 0;
    for (int g = 0; g < LC_BG; ++g) { nch += shi[g]; ntk += shi[LC_BG + g]; }
    float mu[8];
    if (nch > 0 && geometry == LC_GEOMETRY_TOKEN_BALL) {
        const float inv = 1.0f / (float)nch;
#pragma unroll
        for (int t = 0; t < 8; ++t) {
            float s = 0.f;
            for (int g = 0; g < LC_BG; ++g) s += sh[g * LC_D + 8 * sub + t];
            mu[t] = s * inv;
        }
    } else {
        lc_load8(cent + ((size_t)bh * cent_cap + u) * LC_D + 8 * sub, mu);
    }
    __syncthreads();
    float far = LC_NEG_INF;
    for (int base = 0; base < M; base += LC_MEM_WIN) {
        if (M > LC_MEM_WIN) nm = lc_collect_members(a, M, base, u, mem, mcnt);    // (a single window still holds its list)
        for (int t0 = grp; t0 < nm; t0 += LC_NODE_BATCH * LC_BG) {
            float c[LC_NODE_BATCH][8];
            float r0[LC_NODE_BATCH];
#pragma unroll
            for (int q = 0; q < LC_NODE_BATCH; ++q) {
                const int t1 = t0 + q * LC_BG;
                const bool in = t1 < nm;
#pragma unroll
                for (int t = 0; t < 8; ++t) c[q][t] = mu[t];
                r0[q] = LC_NEG_INF;                                 // (a slot past the list reaches nothing)
                if (in) {
                    const int j = mem[t1];
                    lc_c0_load8(ix, cb + j, sub, c[q]);
                    r0[q] = ix.radius[0][cb + j];
                }
            }
#pragma unroll
            for (int q = 0; q < LC_NODE_BATCH; ++q) {
                float d2 = 0.f;
#pragma unroll
                for (int t = 0; t < 8; ++t) { const float e = c[q][t] - mu[t]; d2 = fmaf(e, e, d2); }
                d2 = lc_sum16(d2);
                far = fmaxf(far, lc_pad_radius(sqrtf(d2)) + r0[q]);
            }
        }
        if (base + LC_MEM_WIN < M) __syncthreads();
    }
    if (sub == 0) sh[grp] = far;
    __syncthreads();
    float R = LC_NEG_INF;
    for (int g = 0; g < LC_BG; ++g) R = fmaxf(R, sh[g]);
    const size_t n = (size_t)bh * ix.cap[l + 1] + u;
    if (threadIdx.x < 16) {
        lc_store8(ix.center[l + 1] + n * LC_D + 8 * sub, mu);
        float d[8];
        lc_unit_frag(mu, sub, d);
        lc_store8(next_pts + ((size_t)bh * next_cap + u) * LC_D + 8 * sub, d);
        if (sub == 0) {
            const float R_st = nch > 0 ? lc_pad_radius(R) : LC_NEG_INF;
            ix.radius[l + 1][n] = R_st;
            ix.rbuild[l + 1][n] = R_st;          // the baseline that lc_index_drift measures growth against
            ix.parent[l + 1][n] = -1;
            ix.ntok[l + 1][n] = ntk;
            ix.nchunk[l + 1][n] = nch;
        }
    }
}

// K == nullptr: keep the chunk nodes (level 0) as they are and rebuild only the levels above them.
int lc_launch_build(const lc_index* idx, const LcWs& ws, const void* Kp, const int64_t ks[3],
                    int max_M, hipStream_t stream) {
    const LcDev& ix = idx->dev;
    const uint16_t* K = static_cast<const uint16_t*>(Kp);
    const int geometry = idx->cfg.geometry;
    const int B = ix.B, H = ix.H, L = ix.L;
    int* const kflags = idx->cfg.kmeans_iters < LC_KM_FLAGS ? ws.kflags : nullptr;   // (more iterations: no early exit)
    if (max_M > 0 && K != nullptr) {
        hipLaunchKernelGGL(lc_pool_kernel, dim3((max_M + LC_BT / 64 - 1) / (LC_BT / 64), H, B), dim3(LC_BT), 0, stream, ix, K,
                           (long long)ks[0], (long long)ks[1], (long long)ks[2], geometry, ws.dirs);
        LC_HIP_CHECK(hipGetLastError());
    } else if (max_M > 0) {
        hipLaunchKernelGGL(lc_dirs_kernel, dim3((max_M + LC_BG - 1) / LC_BG, H, B), dim3(LC_BT), 0, stream, ix, ws.dirs);
        LC_HIP_CHECK(hipGetLastError());
    }
    // per-level maxima over the batch (host mirror)
    float* pts = ws.dirs;
    int pts_cap = ix.cap[0];
    float* other = ws.cent_b;
    int other_cap = ix.cap[1];
    for (int l = 0; l + 1 < L; ++l) {
        int maxN = 0, maxK = 0;
        for (int b = 0; b < B; ++b) {
            maxN = idx->N[b * LC_MAX_LEVELS + l] > maxN ? idx->N[b * LC_MAX_LEVELS + l] : maxN;
            maxK = idx->N[b * LC_MAX_LEVELS + l + 1] > maxK ? idx->N[b * LC_MAX_LEVELS + l + 1] : maxK;
        }
        const int cent_cap = ix.cap[1];
        const bool small = maxN <= LC_KS_MAX_N && maxK <= LC_KS_MAX_K;      // the whole clustering in one kernel
        if (small) {
            const int x_rows = maxN > 0 ? maxN : 1;
            const size_t lds = lc_kmeans_small_lds(x_rows, maxK);
            LC_HIP_CHECK(hipFuncSetAttribute(reinterpret_cast<const void*>(&lc_kmeans_small_kernel),
                                             hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));
            hipLaunchKernelGGL(lc_kmeans_small_kernel, dim3(H, B), dim3(LC_BT), lds, stream, ix, l, (const float*)pts,
                               pts_cap, ws.cent_a, cent_cap, idx->cfg.kmeans_iters, x_rows);
        } else {
            hipLaunchKernelGGL(lc_kmeans_init_kernel, dim3(maxK, H, B), dim3(LC_D), 0, stream, ix, l,
                               (const float*)pts, pts_cap, ws.cent_a, cent_cap, kflags);
        }
        LC_HIP_CHECK(hipGetLastError());
        if (maxN > 0) {
            for (int it = 0; it < (small ? 0 : idx->cfg.kmeans_iters); ++it) {
                hipLaunchKernelGGL(lc_kmeans_assign_kernel, dim3((maxN + LC_AS_PTS - 1) / LC_AS_PTS, H, B), dim3(LC_BT), 0,
                                   stream, ix, l, (const float*)pts, pts_cap, (const float*)ws.cent_a, cent_cap, it, kflags);
                hipLaunchKernelGGL(lc_kmeans_update_kernel, dim3(maxK, H, B), dim3(LC_BT), 0, stream, ix, l,
                                   (const float*)pts, pts_cap, ws.cent_a, cent_cap, it, (const int*)kflags);
            }
            LC_HIP_CHECK(hipGetLastError());
            if (max_M > 0) {
                hipLaunchKernelGGL(lc_anc_kernel, dim3((max_M + 255) / 256, H, B), dim3(256), 0, stream, ix, l, ws.anc);
                LC_HIP_CHECK(hipGetLastError());
            }
        }
        hipLaunchKernelGGL(lc_node_kernel, dim3(maxK, H, B), dim3(LC_BT), 0, stream, ix, l, (const int*)ws.anc,
                           (const float*)ws.cent_a, cent_cap, geometry, other, other_cap);
        LC_HIP_CHECK(hipGetLastError());
        float* t = pts; pts = other; other = t;
        const int tc = pts_cap; pts_cap = other_cap; other_cap = tc;
    }
    return LC_OK;
}

// ---------------------------------------------------------------------------------
// drift of one level's radii since the last (re)build
// ---------------------------------------------------------------------------------
// One workgroup per (sequence, head): over the nodes with a finite radius at build time, the sum of
// those radii, the sum of the radii now, the largest growth and the count (fixed reduction order).
__global__ void __launch_bounds__(LC_BT)
lc_drift_kernel(LcDev ix, int level, float* out) {
    __shared__ float sh[4][LC_BT / 64];
    const int h = blockIdx.x, b = blockIdx.y;
    const int bh = b * ix.H + h;
    const int n_l = min(ix.nlev[b * LC_MAX_LEVELS + level], ix.cap[level]);
    const size_t base = (size_t)bh * ix.cap[level];
    float s_then = 0.f, s_now = 0.f, grow = 0.f, cnt = 0.f;
    for (int n = threadIdx.x; n < n_l; n += LC_BT) {
        const float r0 = ix.rbuild[level][base + n], r1 = ix.radius[level][base + n];
        if (r0 > LC_NEG_INF) {
            s_then += r0;
            s_now += r1;
            grow = fmaxf(grow, r1 - r0);
            cnt += 1.f;
        }
    }
    s_then = lc_sum64(s_then);
    s_now = lc_sum64(s_now);
    grow = lc_max64(grow);
    cnt = lc_sum64(cnt);
    if ((threadIdx.x & 63) == 0) {
        const int w = threadIdx.x >> 6;
        sh[0][w] = s_then; sh[1][w] = s_now; sh[2][w] = grow; sh[3][w] = cnt;
    }
    __syncthreads();
    if (threadIdx.x == 0) {
        float a = 0.f, c = 0.f, g = 0.f, k = 0.f;
        for (int w = 0; w < LC_BT / 64; ++w) { a += sh[0][w]; c += sh[1][w]; g = fmaxf(g, sh[2][w]); k += sh[3][w]; }
        out[bh * 4 + 0] = a; out[bh * 4 + 1] = c; out[bh * 4 + 2] = g; out[bh * 4 + 3] = k;
    }
}

// staged = [state: B*H*4 | nlev: B*LC_MAX_LEVELS | boundaries: M_0 + 1, M_1 + 1, ...]; block b < B
// moves sequence b's boundaries, block B the counts (and clears the arrival counters).
__global__ void __launch_bounds__(LC_BT)
lc_place_state_kernel(LcDev ix, const int32_t* staged, int B) {
    const int b = blockIdx.x, tid = threadIdx.x;
    const int n_state = B * ix.H * 4, n_nlev = B * LC_MAX_LEVELS;
    if (b == B) {
        for (int i = tid; i < n_state; i += LC_BT) { ix.state[i] = staged[i]; ix.sync[i] = 0; }
        for (int i = tid; i < n_nlev; i += LC_BT) ix.nlev[i] = staged[n_state + i];
        return;
    }
    int off = n_state + n_nlev;
    for (int s = 0; s < b; ++s) off += staged[s * ix.H * 4 + 1] + 1;
    const int n = staged[b * ix.H * 4 + 1] + 1;
    int* dst = ix.bounds + (size_t)b * (ix.cap[0] + 1);
    for (int i = tid; i < n; i += LC_BT) dst[i] = staged[off + i];
}

int lc_launch_place_state(const lc_index* idx, const int32_t* staged, hipStream_t stream) {
    hipLaunchKernelGGL(lc_place_state_kernel, dim3(idx->B + 1), dim3(LC_BT), 0, stream, idx->dev, staged, idx->B);
    LC_HIP_CHECK(hipGetLastError());
    return LC_OK;
}

int lc_launch_drift(const lc_index* idx, int level, float* out, hipStream_t stream) {
    hipLaunchKernelGGL(lc_drift_kernel, dim3(idx->dev.H, idx->dev.B), dim3(LC_BT), 0, stream, idx->dev, level, out);
    LC_HIP_CHECK(hipGetLastError());
    return LC_OK;
}

// ---------------------------------------------------------------------------------
// lazy update
// ---------------------------------------------------------------------------------
struct LcCloseBits { uint32_t w[32]; };       // one bit per sequence (B <= 1024)

__global__ void __launch_bounds__(LC_BT)
lc_append_kernel(LcDev ix, uint16_t* K, uint16_t* V, long long ks_seq, long long ks_head, long long ks_tok,
                 const uint16_t* k_new, const uint16_t* v_new, LcCloseBits close, int geometry, int max_tokens) {
    __shared__ float sh[LC_BG * LC_D + LC_BG];
    __shared__ float best_sim[LC_BG];
    __shared__ int best_arg[LC_BG];
    const int h = blockIdx.x, b = blockIdx.y;
    const int bh = b * ix.H + h;
    const int tid = threadIdx.x, sub = tid & 15, grp = tid >> 4;
    const int T = ix.state[bh * 4 + 0];
    const int M = ix.state[bh * 4 + 1];
    // The host checks the capacities against its own counts before it launches; these guards are for
    // a caller who replays the launch from a captured graph, where the host is not asked again.
    if (T >= max_tokens) return;
    uint16_t* Kbh = K + b * ks_seq + h * ks_head;
    uint16_t* Vbh = V + b * ks_seq + h * ks_head;
    if (tid < 16) {
        *reinterpret_cast<uint4*>(Kbh + (long long)T * ks_tok + 8 * sub) =
            *reinterpret_cast<const uint4*>(k_new + (size_t)bh * LC_D + 8 * sub);
    } else if (tid < 32) {
        *reinterpret_cast<uint4*>(Vbh + (long long)T * ks_tok + 8 * sub) =
            *reinterpret_cast<const uint4*>(v_new + (size_t)bh * LC_D + 8 * sub);
    }
    const bool do_close = ((close.w[b >> 5] >> (b & 31)) & 1u) && M < ix.cap[0];
    if (!do_close) {
        if (tid == 0) ix.state[bh * 4 + 0] = T + 1;
        return;
    }
    __threadfence_block();
    __syncthreads();

    int* bnd = ix.bounds + (size_t)b * (ix.cap[0] + 1);
    const int lo = bnd[M], hi = T + 1;
    float mu_x[8], r_x;
    lc_pool_rows(Kbh, ks_tok, lo, hi, geometry, ix.c0_bf16 != 0, sh, mu_x, &r_x);
    const int n_x = hi - lo;
    int p = -1;
    if (ix.L > 1) {
        float xh[8];
        lc_unit_frag(mu_x, sub, xh);
        const float xh0 = __shfl(xh[0], (tid & 48), 64);        // first component, from the group's lane 0
        const int n1 = ix.nlev[b * LC_MAX_LEVELS + 1];
        const size_t b1 = (size_t)bh * ix.cap[1];
        float bs = LC_NEG_INF;
        int ba = 0x7fffffff;
        for (int c = grp; c < n1; c += LC_BG) {
            float m[8];
            lc_load8(ix.center[1] + (b1 + c) * LC_D + 8 * sub, m);
            float dot = 0.f, n2 = 0.f;
#pragma unroll
            for (int t = 0; t < 8; ++t) { dot = fmaf(xh[t], m[t], dot); n2 = fmaf(m[t], m[t], n2); }
            dot = lc_sum16(dot);
            n2 = lc_sum16(n2);
            const float sim = n2 > 0.f ? dot / sqrtf(n2) : xh0;
            if (sim > bs) { bs = sim; ba = c; }
        }
        if (sub == 0) { best_sim[grp] = bs; best_arg[grp] = ba; }
        __syncthreads();
        float s = LC_NEG_INF;
        p = 0x7fffffff;
        for (int g = 0; g < LC_BG; ++g) {
            const float sg = best_sim[g];
            const int ag = best_arg[g];
            if (sg > s || (sg == s && ag < p)) { s = sg; p = ag; }
        }
        // path to the top: moving-average centers, monotone radii
        if (tid < 16) {
            int a = p;
            for (int l = 1; l < ix.L; ++l) {
                const size_t n = (size_t)bh * ix.cap[l] + a;
                const int n_a = ix.nchunk[l][n];
                float mu_a[8], nw[8];
                lc_load8(ix.center[l] + n * LC_D + 8 * sub, mu_a);
                const float inv = 1.0f / (float)(n_a + 1);
#pragma unroll
                for (int t = 0; t < 8; ++t) nw[t] = fmaf((float)n_a, mu_a[t], mu_x[t]) * inv;
                if (geometry == LC_GEOMETRY_PAPER_UNIT) {
                    float un[8];
                    lc_unit_frag(nw, sub, un);
#pragma unroll
                    for (int t = 0; t < 8; ++t) nw[t] = un[t];
                }
                float sh2 = 0.f, re2 = 0.f;
#pragma unroll
                for (int t = 0; t < 8; ++t) {
                    const float e = nw[t] - mu_a[t];
                    const float f = mu_x[t] - nw[t];
                    sh2 = fmaf(e, e, sh2);
                    re2 = fmaf(f, f, re2);
                }
                sh2 = lc_sum16(sh2);
                re2 = lc_sum16(re2);
                const float R_old = ix.radius[l][n];
                const float grown = R_old + lc_pad_radius(sqrtf(sh2));
                const float reach = lc_pad_radius(sqrtf(re2)) + r_x;
                const int next = ix.parent[l][n];
                lc_store8(ix.center[l] + n * LC_D + 8 * sub, nw);
                if (sub == 0) {
                    ix.radius[l][n] = lc_pad_radius(fmaxf(grown, reach));
                    ix.ntok[l][n] += n_x;
                    ix.nchunk[l][n] = n_a + 1;
                }
                a = next;
            }
        }
    }
    const size_t n0 = (size_t)bh * ix.cap[0] + M;
    if (tid < 16) {
        lc_c0_store8(ix, n0, sub, mu_x);
        if (sub == 0) {
            ix.radius[0][n0] = r_x;
            ix.parent[0][n0] = p;
            ix.ntok[0][n0] = n_x;
            ix.nchunk[0][n0] = 1;
            if (h == 0) bnd[M + 1] = hi;
            ix.state[bh * 4 + 0] = T + 1;
            ix.state[bh * 4 + 1] = M + 1;
        }
    }
}

int lc_launch_append(const lc_index* idx, void* K, void* V, const int64_t ks[3],
                     const void* k_new, const void* v_new, const uint8_t* close_host,
                     uint32_t, hipStream_t stream) {
    const LcDev& ix = idx->dev;
    LcCloseBits bits;
    for (int i = 0; i < 32; ++i) bits.w[i] = 0u;
    if (close_host)
        for (int b = 0; b < ix.B; ++b)
            if (close_host[b]) bits.w[b >> 5] |= 1u << (b & 31);
    hipLaunchKernelGGL(lc_append_kernel, dim3(ix.H, ix.B), dim3(LC_BT), 0, stream, ix,
                       static_cast<uint16_t*>(K), static_cast<uint16_t*>(V),
                       (long long)ks[0], (long long)ks[1], (long long)ks[2],
                       static_cast<const uint16_t*>(k_new), static_cast<const uint16_t*>(v_new), bits,
                       idx->cfg.geometry, idx->cfg.max_tokens);
    LC_HIP_CHECK(hipGetLastError());
    return LC_OK;
}
