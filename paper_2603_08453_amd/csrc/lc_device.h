// Device-side building blocks shared by the kernels (wave64, gfx950).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#define LC_D 128                  // head dimension the kernels are written for

#define LC_NEG_INF (-__builtin_huge_valf())

// ---------------------------------------------------------------- bf16 unpacking
// A 32-bit word holds two bf16 values; widening is a shift or a mask.
__device__ __forceinline__ float lc_bf16_lo(uint32_t w) { return __uint_as_float(w << 16); }
__device__ __forceinline__ float lc_bf16_hi(uint32_t w) { return __uint_as_float(w & 0xffff0000u); }

__device__ __forceinline__ void lc_unpack8(const uint4& v, float (&f)[8]) {
    f[0] = lc_bf16_lo(v.x); f[1] = lc_bf16_hi(v.x);
    f[2] = lc_bf16_lo(v.y); f[3] = lc_bf16_hi(v.y);
    f[4] = lc_bf16_lo(v.z); f[5] = lc_bf16_hi(v.z);
    f[6] = lc_bf16_lo(v.w); f[7] = lc_bf16_hi(v.w);
}

// ---------------------------------------------------------------- reductions
// Sum over the 16 consecutive lanes that share (lane >> 4): exactly one DPP row, so the
// butterfly runs on the vector ALU (quad permutes, then half-row and full-row mirrors)
// instead of going through the LDS crossbar as a generic shuffle would.
template <int CTRL>
__device__ __forceinline__ float lc_dpp(float v) {
    return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), CTRL, 0xF, 0xF, true));
}
__device__ __forceinline__ float lc_sum16(float v) {
    v += lc_dpp<0xB1>(v);      // quad_perm [1,0,3,2]: lane ^ 1
    v += lc_dpp<0x4E>(v);      // quad_perm [2,3,0,1]: lane ^ 2
    v += lc_dpp<0x141>(v);     // row_half_mirror: the other quad of the same half-row
    v += lc_dpp<0x140>(v);     // row_mirror: the other half-row
    return v;
}
__device__ __forceinline__ float lc_sum64(float v) {
    v = lc_sum16(v);
    v += __shfl_xor(v, 16);
    v += __shfl_xor(v, 32);
    return v;
}
__device__ __forceinline__ float lc_max64(float v) {
    v = fmaxf(v, lc_dpp<0xB1>(v));
    v = fmaxf(v, lc_dpp<0x4E>(v));
    v = fmaxf(v, lc_dpp<0x141>(v));
    v = fmaxf(v, lc_dpp<0x140>(v));
    v = fmaxf(v, __shfl_xor(v, 16));
    v = fmaxf(v, __shfl_xor(v, 32));
    return v;
}

// ---------------------------------------------------------------- cross-workgroup hand-off
// Several workgroups produce partial results and the last one to arrive consumes them.
// A device-scope fence (__threadfence) writes back the whole L2 of the XCD on this chip,
// which costs tens of microseconds when hundreds of workgroups do it.  Instead the
// hand-off data itself is stored and loaded at agent scope (relaxed atomics: the
// accesses are performed at the device-coherent level and leave no dirty L2 lines),
// the producer waits for its stores to complete (s_waitcnt vmcnt(0)) before it bumps the
// arrival counter, and the consumer reads only after it has seen
// the final count.
__device__ __forceinline__ void lc_store_agent(float* p, float v) {
    __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ void lc_store_agent(uint32_t* p, uint32_t v) {
    __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ float lc_load_agent(const float* p) {
    return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ uint32_t lc_load_agent(const uint32_t* p) {
    return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
// 16-byte versions through buffer instructions with the agent-scope cache policy (sc1).
typedef int lc_v4i __attribute__((ext_vector_type(4)));
__device__ __forceinline__ __amdgpu_buffer_rsrc_t lc_buffer(const void* base, int bytes = 0x7fffffff) {
    // `bytes` is the extent the hardware checks offsets against: a load past it returns 0, a store is dropped
    return __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(base), 0, bytes, 0x00020000);
}
__device__ __forceinline__ float4 lc_load_agent4(__amdgpu_buffer_rsrc_t r, int byte_offset) {
    const lc_v4i v = __builtin_amdgcn_raw_buffer_load_b128(r, byte_offset, 0, 16);
    const int x = v.x, y = v.y, z = v.z, w = v.w;         // element values first, then reinterpret
    return make_float4(__int_as_float(x), __int_as_float(y), __int_as_float(z), __int_as_float(w));
}
__device__ __forceinline__ void lc_store_agent4(__amdgpu_buffer_rsrc_t r, int byte_offset, float4 f) {
    lc_v4i v;
    v.x = __float_as_int(f.x); v.y = __float_as_int(f.y);
    v.z = __float_as_int(f.z); v.w = __float_as_int(f.w);
    __builtin_amdgcn_raw_buffer_store_b128(v, r, byte_offset, 0, 16);
}
// 4-byte and 1-byte reads and 4-byte writes through a range-checked buffer resource: an index outside
// [0, extent) reads 0 / writes nothing instead of touching memory that is not the array's.
__device__ __forceinline__ int lc_buf_load_i32(__amdgpu_buffer_rsrc_t r, int index) {
    return __builtin_amdgcn_raw_buffer_load_b32(r, index * 4, 0, 0);
}
__device__ __forceinline__ float lc_buf_load_f32(__amdgpu_buffer_rsrc_t r, int index) {
    return __int_as_float(__builtin_amdgcn_raw_buffer_load_b32(r, index * 4, 0, 0));
}
__device__ __forceinline__ int lc_buf_load_u8(__amdgpu_buffer_rsrc_t r, int index) {
    return (int)(unsigned char)__builtin_amdgcn_raw_buffer_load_b8(r, index, 0, 0);
}
__device__ __forceinline__ void lc_buf_store_u32(__amdgpu_buffer_rsrc_t r, int index, uint32_t v) {
    __builtin_amdgcn_raw_buffer_store_b32((int)v, r, index * 4, 0, 0);
}
// Returns true in every thread of the last workgroup to arrive at `counter` (of `expected`).
__device__ __forceinline__ bool lc_arrive_last(int* counter, int expected, int* flag_sh) {
    // Wait until this thread's hand-off stores have been acknowledged (they are write-through, so
    // the acknowledgement means they are visible device-wide).  A workgroup-scope fence alone does
    // not wait for stores to complete, so the counters are drained explicitly.
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
    __builtin_amdgcn_s_waitcnt(0);
    __syncthreads();
    if (threadIdx.x == 0) {
        const int old = __hip_atomic_fetch_add(counter, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        *flag_sh = (old == expected - 1) ? 1 : 0;
    }
    __syncthreads();
    const bool last = *flag_sh != 0;
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup");
    return last;
}

// ---------------------------------------------------------------- score keys
// Order-preserving map float -> uint32 (larger score = larger key).  -inf (empty
// or pruned node) maps to 0, which no finite score produces: key 0 = "not a candidate".
__device__ __forceinline__ uint32_t lc_score_key(float s) {
    if (s == LC_NEG_INF) return 0u;
    s += 0.0f;                                        // -0 -> +0 so equal scores share a key
    uint32_t u = __float_as_uint(s);
    return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}
__device__ __forceinline__ float lc_key_score(uint32_t k) {
    if (k == 0u) return LC_NEG_INF;
    uint32_t u = (k & 0x80000000u) ? (k & 0x7fffffffu) : ~k;
    return __uint_as_float(u);
}

// ---------------------------------------------------------------- Eq. 2 for one node
// Called by the 16 lanes of a group; lane `sub` holds the query fragments for
// floats [4 sub, 4 sub + 4) and [64 + 4 sub, 64 + 4 sub + 4) of each of the G heads.
// Returns max_g (q_g . mu + |q_g| R) / sqrt(d) in every lane of the group.
// The operation order is fixed (explicit fma chain) so that every kernel that
// scores the same node obtains the same bits.
struct LcNodeFrag {
    float4 a, b;        // floats [4 sub, 4 sub + 4) and [64 + 4 sub, 64 + 4 sub + 4) of the center
};
__device__ __forceinline__ LcNodeFrag lc_load_node(const float* __restrict__ center, int sub) {
    LcNodeFrag f;
    f.a = *reinterpret_cast<const float4*>(center + 4 * sub);
    f.b = *reinterpret_cast<const float4*>(center + 64 + 4 * sub);
    return f;
}
// Chunk-level centers may be stored as bfloat16.  Loading and widening are separate steps so that a
// kernel can issue the loads early and touch the data only where it scores: the loaded fragment
// holds the raw words (float32 storage: the eight values; bfloat16 storage: four packed pairs in
// a.x, a.y, b.x, b.y) and lc_score_chunk_frag widens them.  Same columns per lane either way.
__device__ __forceinline__ LcNodeFrag lc_load_chunk_node(const float* center0, bool bf16, size_t n, int sub) {
    if (!bf16) return lc_load_node(center0 + n * LC_D, sub);
    const uint16_t* row = reinterpret_cast<const uint16_t*>(center0) + n * LC_D;
    const uint2 a = *reinterpret_cast<const uint2*>(row + 4 * sub);
    const uint2 b = *reinterpret_cast<const uint2*>(row + 64 + 4 * sub);
    LcNodeFrag f;
    f.a = make_float4(__uint_as_float(a.x), __uint_as_float(a.y), 0.f, 0.f);
    f.b = make_float4(__uint_as_float(b.x), __uint_as_float(b.y), 0.f, 0.f);
    return f;
}
__device__ __forceinline__ LcNodeFrag lc_widen_chunk_frag(const LcNodeFrag& r) {
    const uint32_t a0 = __float_as_uint(r.a.x), a1 = __float_as_uint(r.a.y);
    const uint32_t b0 = __float_as_uint(r.b.x), b1 = __float_as_uint(r.b.y);
    LcNodeFrag f;
    f.a = make_float4(lc_bf16_lo(a0), lc_bf16_hi(a0), lc_bf16_lo(a1), lc_bf16_hi(a1));
    f.b = make_float4(lc_bf16_lo(b0), lc_bf16_hi(b0), lc_bf16_lo(b1), lc_bf16_hi(b1));
    return f;
}
// float -> nearest bfloat16, ties to even (finite inputs)
__device__ __forceinline__ uint32_t lc_f32_to_bf16_bits(float f) {
    const uint32_t u = __float_as_uint(f);
    return (u + 0x7fffu + ((u >> 16) & 1u)) >> 16;
}
__device__ __forceinline__ float lc_round_bf16(float f) { return __uint_as_float(lc_f32_to_bf16_bits(f) << 16); }

template <int G>
__device__ __forceinline__ float lc_score_frag(const LcNodeFrag& f, float R, const float (&qf)[G][8],
                                               const float (&qn)[G]) {
    float best = LC_NEG_INF;
#pragma unroll
    for (int g = 0; g < G; ++g) {
        float p = f.a.x * qf[g][0];
        p = fmaf(f.a.y, qf[g][1], p);
        p = fmaf(f.a.z, qf[g][2], p);
        p = fmaf(f.a.w, qf[g][3], p);
        p = fmaf(f.b.x, qf[g][4], p);
        p = fmaf(f.b.y, qf[g][5], p);
        p = fmaf(f.b.z, qf[g][6], p);
        p = fmaf(f.b.w, qf[g][7], p);
        p = lc_sum16(p);
        const float ub = fmaf(qn[g], R, p) * 0.08838834764831845f;      // 1/sqrt(128)
        best = fmaxf(best, ub);
    }
    return best;
}
template <int G>
__device__ __forceinline__ float lc_score_node(const float* __restrict__ center, float R, int sub,
                                               const float (&qf)[G][8], const float (&qn)[G]) {
    return lc_score_frag<G>(lc_load_node(center, sub), R, qf, qn);
}
// Eq. 2 for a chunk node from its loaded fragment (see lc_load_chunk_node).
template <int G>
__device__ __forceinline__ float lc_score_chunk_frag(const LcNodeFrag& raw, bool bf16, float R,
                                                     const float (&qf)[G][8], const float (&qn)[G]) {
    return lc_score_frag<G>(bf16 ? lc_widen_chunk_frag(raw) : raw, R, qf, qn);
}

// The same with the query fragments kept as the packed bfloat16 words they arrive in (half the
// registers; the widening is redone per node).  Same operands in the same order: same bits.
template <int G>
__device__ __forceinline__ float lc_score_frag_packed(const LcNodeFrag& f, float R, const uint32_t (&qp)[G][4],
                                                      const float (&qn)[G]) {
    float best = LC_NEG_INF;
#pragma unroll
    for (int g = 0; g < G; ++g) {
        // (the empty asm makes the words opaque here, so that the widening is not hoisted out of the
        // caller's loops and kept in registers after all)
        uint32_t w0 = qp[g][0], w1 = qp[g][1], w2 = qp[g][2], w3 = qp[g][3];
        asm volatile("" : "+v"(w0), "+v"(w1), "+v"(w2), "+v"(w3));
        float p = f.a.x * lc_bf16_lo(w0);
        p = fmaf(f.a.y, lc_bf16_hi(w0), p);
        p = fmaf(f.a.z, lc_bf16_lo(w1), p);
        p = fmaf(f.a.w, lc_bf16_hi(w1), p);
        p = fmaf(f.b.x, lc_bf16_lo(w2), p);
        p = fmaf(f.b.y, lc_bf16_hi(w2), p);
        p = fmaf(f.b.z, lc_bf16_lo(w3), p);
        p = fmaf(f.b.w, lc_bf16_hi(w3), p);
        p = lc_sum16(p);
        const float ub = fmaf(qn[g], R, p) * 0.08838834764831845f;      // 1/sqrt(128)
        best = fmaxf(best, ub);
    }
    return best;
}
template <int G>
__device__ __forceinline__ void lc_load_query_packed(const uint16_t* __restrict__ q, int h, int sub,
                                                     uint32_t (&qp)[G][4], float (&qn)[G]) {
#pragma unroll
    for (int g = 0; g < G; ++g) {
        const uint16_t* row = q + (size_t)(h * G + g) * LC_D;
        const uint2 a = *reinterpret_cast<const uint2*>(row + 4 * sub);
        const uint2 b = *reinterpret_cast<const uint2*>(row + 64 + 4 * sub);
        qp[g][0] = a.x; qp[g][1] = a.y; qp[g][2] = b.x; qp[g][3] = b.y;
        float s = 0.f;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            s = fmaf(lc_bf16_lo(qp[g][i]), lc_bf16_lo(qp[g][i]), s);
            s = fmaf(lc_bf16_hi(qp[g][i]), lc_bf16_hi(qp[g][i]), s);
        }
        qn[g] = sqrtf(lc_sum16(s));
    }
}

// Load the query group of KV head h into registers (fragments as above) and
// compute the norms.  q: bf16 [H_q][d] of this sequence.
template <int G>
__device__ __forceinline__ void lc_load_query_frags(const uint16_t* __restrict__ q, int h, int sub,
                                                    float (&qf)[G][8], float (&qn)[G]) {
#pragma unroll
    for (int g = 0; g < G; ++g) {
        const uint16_t* row = q + (size_t)(h * G + g) * LC_D;
        const uint2 a = *reinterpret_cast<const uint2*>(row + 4 * sub);
        const uint2 b = *reinterpret_cast<const uint2*>(row + 64 + 4 * sub);
        qf[g][0] = lc_bf16_lo(a.x); qf[g][1] = lc_bf16_hi(a.x);
        qf[g][2] = lc_bf16_lo(a.y); qf[g][3] = lc_bf16_hi(a.y);
        qf[g][4] = lc_bf16_lo(b.x); qf[g][5] = lc_bf16_hi(b.x);
        qf[g][6] = lc_bf16_lo(b.y); qf[g][7] = lc_bf16_hi(b.y);
        float s = 0.f;
#pragma unroll
        for (int i = 0; i < 8; ++i) s = fmaf(qf[g][i], qf[g][i], s);
        qn[g] = sqrtf(lc_sum16(s));
    }
}

// ---------------------------------------------------------------- block scan
// Exclusive prefix sum of one int per thread over a block of NT threads.
// `sh` needs NT/64 + 1 ints.  Returns the exclusive prefix; *total = block sum.
// Inclusive prefix sum over the 64 lanes of a wavefront (all of them active), on the vector ALU:
// four shifted adds inside each 16-lane row, then the row totals are carried over by the two
// row-broadcast adds (last lane of row 0 -> row 1 and of row 2 -> row 3; last lane of row 1 ->
// rows 2 and 3).  A generic shuffle would take a trip through the LDS crossbar per step.
__device__ __forceinline__ int lc_wave_scan_incl(int v) {
    v += __builtin_amdgcn_update_dpp(0, v, 0x111, 0xF, 0xF, true);   // row_shr:1
    v += __builtin_amdgcn_update_dpp(0, v, 0x112, 0xF, 0xF, true);   // row_shr:2
    v += __builtin_amdgcn_update_dpp(0, v, 0x114, 0xF, 0xF, true);   // row_shr:4
    v += __builtin_amdgcn_update_dpp(0, v, 0x118, 0xF, 0xF, true);   // row_shr:8
    v += __builtin_amdgcn_update_dpp(0, v, 0x142, 0xA, 0xF, true);   // row_bcast:15 -> rows 1, 3
    v += __builtin_amdgcn_update_dpp(0, v, 0x143, 0xC, 0xF, true);   // row_bcast:31 -> rows 2, 3
    return v;
}

template <int NT>
__device__ __forceinline__ int lc_block_scan(int v, int* sh, int* total) {
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int inc = lc_wave_scan_incl(v);
    __syncthreads();                 // protect sh from the previous use
    if (lane == 63) sh[wave] = inc;
    __syncthreads();
    int base = 0, tot = 0;
#pragma unroll
    for (int w = 0; w < NT / 64; ++w) {
        const int s = sh[w];
        if (w < wave) base += s;
        tot += s;
    }
    *total = tot;
    return base + inc - v;
}

// ---------------------------------------------------------------- weighted radix select
// Items i in [0, n) with key(i) != 0, ordered by (key descending, i ascending).
// Finds the longest prefix whose weights sum to <= W and that holds <= C items.
// Result: items with key > kstar are in; items with key == kstar are in while,
// taken in ascending i, their running weight stays <= remW and their running
// count <= remC; `all` set = every candidate fits (kstar = 0).
//
// The digits are taken from the highest bit in which the keys differ downward
// (scores of one query sit in a narrow range, so their top bits agree): at most
// four 8-bit passes, and the LDS histogram atomics spread over many bins.
struct LcSel {
    uint32_t kstar;
    int remW;
    int remC;
    int all;
};

// Min / max over the 64 lanes of a wave: DPP within the 16-lane rows, then two cross-row steps.
template <int CTRL>
__device__ __forceinline__ uint32_t lc_dpp_u(uint32_t v) {
    return (uint32_t)__builtin_amdgcn_update_dpp((int)v, (int)v, CTRL, 0xF, 0xF, false);
}
__device__ __forceinline__ uint32_t lc_wave_min_u(uint32_t v) {
    v = min(v, lc_dpp_u<0xB1>(v)); v = min(v, lc_dpp_u<0x4E>(v));
    v = min(v, lc_dpp_u<0x141>(v)); v = min(v, lc_dpp_u<0x140>(v));
    v = min(v, (uint32_t)__shfl_xor((int)v, 16)); v = min(v, (uint32_t)__shfl_xor((int)v, 32));
    return v;
}
__device__ __forceinline__ uint32_t lc_wave_max_u(uint32_t v) {
    v = max(v, lc_dpp_u<0xB1>(v)); v = max(v, lc_dpp_u<0x4E>(v));
    v = max(v, lc_dpp_u<0x141>(v)); v = max(v, lc_dpp_u<0x140>(v));
    v = max(v, (uint32_t)__shfl_xor((int)v, 16)); v = max(v, (uint32_t)__shfl_xor((int)v, 32));
    return v;
}

// sh: LC_SEL_SH ints of LDS.  All NT threads must call.  `kmin` / `kmax`: this thread's partial
// range of the candidate keys it has already seen (0xffffffff / 0 if none); with have_range false
// the routine scans the keys itself.
#define LC_SEL_SH 584
template <int NT, typename KeyF, typename WgtF>
__device__ __forceinline__ LcSel lc_block_select(int n, long long W, long long C, KeyF key, WgtF wgt, int* sh,
                                                 bool have_range = false, uint32_t kmin = 0xffffffffu,
                                                 uint32_t kmax = 0u) {
    int* hw = sh;
    int* hc = sh + 256;
    int* res = sh + 512;
    int* mm = sh + 520;                          // 2 x 32 ints, used by nothing else
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    LcSel out;
    out.all = 0;
    out.kstar = 0u;
    out.remW = 0;
    out.remC = 0;
    // ---- range of the candidate keys
    if (!have_range) {
        for (int i = threadIdx.x; i < n; i += NT) {
            const uint32_t k = key(i);
            if (k != 0u) { kmin = min(kmin, k); kmax = max(kmax, k); }
        }
    }
    kmin = lc_wave_min_u(kmin);
    kmax = lc_wave_max_u(kmax);
    if (lane == 0) { mm[wave] = (int)kmin; mm[32 + wave] = (int)kmax; }
    __syncthreads();
#pragma unroll
    for (int w = 0; w < NT / 64; ++w) { kmin = min(kmin, (uint32_t)mm[w]); kmax = max(kmax, (uint32_t)mm[32 + w]); }
    if (kmax == 0u) { out.all = 1; __syncthreads(); return out; }            // no candidate at all
    const uint32_t diff = kmin ^ kmax;
    int top = diff ? 32 - __clz(diff) : 0;                   // bits [0, top) may differ
    uint32_t mask = top >= 32 ? 0u : ~((1u << top) - 1u);
    uint32_t prefix = kmax & mask;
    long long remW = W, remC = C;
    const bool count_c = C < 0x7fffffffLL;
    bool first = true;
    int npass = 0;
    (void)npass;
    while (top > 0) {
        const int width = top >= 8 ? 8 : top;
        const int shift = top - width;
        for (int i = threadIdx.x; i < 256; i += NT) { hw[i] = 0; hc[i] = 0; }
        __syncthreads();
        for (int i = threadIdx.x; i < n; i += NT) {
            const uint32_t k = key(i);
            if (k != 0u && (k & mask) == prefix) {
                const int b = (k >> shift) & ((1 << width) - 1);
                atomicAdd(&hw[b], wgt(i));
                if (count_c) atomicAdd(&hc[b], 1);
            }
        }
        __syncthreads();
        if (threadIdx.x < 64) {
            const int l = threadIdx.x;
            int w[4], c[4];
#pragma unroll
            for (int j = 0; j < 4; ++j) { w[j] = hw[255 - (4 * l + j)]; c[j] = hc[255 - (4 * l + j)]; }
            long long sw = (long long)w[0] + w[1] + w[2] + w[3];
            long long sc = (long long)c[0] + c[1] + c[2] + c[3];
            // (the histogram holds ints: the sums of a pass fit 32 bits, so the scan can run on the vector ALU)
            const long long iw = lc_wave_scan_incl((int)sw), ic = lc_wave_scan_incl((int)sc);
            long long cw = iw - sw, cc = ic - sc;           // weight / count of all higher bins
            int found = -1;
            long long fw = 0, fc = 0;
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                if (found < 0) {
                    if (cw + w[j] > remW || cc + c[j] > remC) { found = 255 - (4 * l + j); fw = cw; fc = cc; }
                    else { cw += w[j]; cc += c[j]; }
                }
            }
            const unsigned long long bal = __ballot(found >= 0);
            if (bal == 0ull) {
                if (l == 0) res[0] = -1;
            } else {
                const int firstl = __ffsll((long long)bal) - 1;       // lowest lane = highest bins
                if (l == firstl) { res[0] = found; res[1] = (int)fw; res[2] = (int)fc; }
            }
        }
        __syncthreads();
        ++npass;
        const int found = res[0];
        if (found < 0) {            // everything in scope fits: only possible in the first pass
            out.all = first ? 1 : 0;
            break;
        }
        remW -= res[1];
        remC -= res[2];
        prefix |= (uint32_t)found << shift;
        mask |= (uint32_t)((1 << width) - 1) << shift;
        top = shift;
        first = false;
        __syncthreads();
    }
    __syncthreads();
    // all keys equal (top == 0 from the start): the single key group is the tie group
    out.kstar = out.all ? 0u : prefix;
    out.remW = (int)(remW > 0x7fffffffLL ? 0x7fffffffLL : (remW < 0 ? -1 : remW));
    out.remC = (int)(remC > 0x7fffffffLL ? 0x7fffffffLL : (remC < 0 ? -1 : remC));
    return out;
}

// ---------------------------------------------------------------- counting select (small n)
// For item i among n candidates: number and total weight of the items that precede it in the
// (key descending, index ascending) order.  `keys` and `wgts` are 16-byte aligned LDS arrays,
// zero-padded to a multiple of 4 entries (key 0 = not a candidate; it never precedes anything).
// The 16 lanes of a group share one item: lane `part` scans every 16th vector of four entries
// (neighbouring lanes read neighbouring vectors, the four groups of a wave read the same ones),
// and the partial counts are summed over the DPP row.  Returned in every lane of the group.
__device__ __forceinline__ int lc_sum16_i(int v) {
    v += __builtin_amdgcn_update_dpp(0, v, 0xB1, 0xF, 0xF, true);
    v += __builtin_amdgcn_update_dpp(0, v, 0x4E, 0xF, 0xF, true);
    v += __builtin_amdgcn_update_dpp(0, v, 0x141, 0xF, 0xF, true);
    v += __builtin_amdgcn_update_dpp(0, v, 0x140, 0xF, 0xF, true);
    return v;
}
__device__ __forceinline__ void lc_rank_before16(int n, const uint32_t* keys, const int* wgts, int i, uint32_t ki,
                                                 int part, int* count_before, int* weight_before) {
    int cb = 0, wb = 0;
    const int nv = (n + 3) >> 2;
    for (int jv = part; jv < nv; jv += 16) {
        const int j = 4 * jv;
        const uint4 k = *reinterpret_cast<const uint4*>(keys + j);
        const int4 w = *reinterpret_cast<const int4*>(wgts + j);
        const bool b0 = k.x > ki || (k.x == ki && j + 0 < i);
        const bool b1 = k.y > ki || (k.y == ki && j + 1 < i);
        const bool b2 = k.z > ki || (k.z == ki && j + 2 < i);
        const bool b3 = k.w > ki || (k.w == ki && j + 3 < i);
        cb += (int)b0 + (int)b1 + (int)b2 + (int)b3;
        wb += (b0 ? w.x : 0) + (b1 ? w.y : 0) + (b2 ? w.z : 0) + (b3 ? w.w : 0);
    }
    *count_before = lc_sum16_i(cb);
    *weight_before = lc_sum16_i(wb);
}

#define LC_SELECT_THREADS_MAX 1024
// ---------------------------------------------------------------------------------
// budget selection over the staged chunk keys (used by the chunk-scoring kernel's last workgroup and by the fused decode step)
// ---------------------------------------------------------------------------------
// Candidates are the chunks with key != 0, ordered by (key descending, id ascending); the
// selection is the longest prefix with total length <= W and at most C chunks.
//   1. One histogram pass over 1024 bins that span [lowest, highest] candidate key linearly
//      (length and count per bin), a descending scan finds the bin in which the prefix ends.
//   2. That bin usually holds a handful of chunks: they are copied to a short list and ranked
//      against each other directly (16 lanes per chunk), which decides each of them exactly.
//      A bin with more chunks than the list holds is split again (step 1 on its key range); a
//      bin that is a single key value is a tie group and is cut by a scan in id order.
// On return chunk i is selected iff skey[i] > thr: the chunks of the last bin have had their key
// replaced by 0xffffffff (selected) or 0 (not).
#define LC_LS_BITS 10
#define LC_LS_BINS (1 << LC_LS_BITS)
#define LC_LS_CAND 256
struct LcLeafSelSh {
    int hw[LC_LS_BINS];
    int hc[LC_LS_BINS];
    uint32_t ck[LC_LS_CAND];
    int cl[LC_LS_CAND];
    int ci[LC_LS_CAND];
    int scan[2 * (LC_SELECT_THREADS_MAX / 64)];
    int mm[2];                     // lowest / highest candidate key
    int res[4];
    int ncand;
};

// exclusive prefix sums of two values over the workgroup, sharing the barriers
template <int NT>
__device__ __forceinline__ void lc_block_scan2(int a, int b, int* sh, int* ea, int* eb, int* ta = nullptr,
                                               int* tb = nullptr) {
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int ia = lc_wave_scan_incl(a), ib = lc_wave_scan_incl(b);
    __syncthreads();                 // protect sh from the previous use
    if (lane == 63) { sh[wave] = ia; sh[NT / 64 + wave] = ib; }
    __syncthreads();
    int ba = 0, bb = 0, sa = 0, sb = 0;
#pragma unroll
    for (int w = 0; w < NT / 64; ++w) {
        const int xa = sh[w], xb = sh[NT / 64 + w];
        if (w < wave) { ba += xa; bb += xb; }
        sa += xa;
        sb += xb;
    }
    *ea = ba + ia - a;
    *eb = bb + ib - b;
    if (ta) *ta = sa;
    if (tb) *tb = sb;
}

// Called by every thread before the keys are staged: empties the histogram and the key range.
template <int NT>
__device__ __forceinline__ void lc_leaf_select_prepare(LcLeafSelSh& sh) {
    for (int i = threadIdx.x; i < LC_LS_BINS; i += NT) { sh.hw[i] = 0; sh.hc[i] = 0; }
    if (threadIdx.x == 0) { sh.res[0] = -1; sh.ncand = 0; sh.mm[0] = (int)0xffffffffu; sh.mm[1] = 0; }
}
// Called by every thread with the range of the candidate keys it staged (0xffffffff / 0 if none);
// a barrier must follow before lc_leaf_select.
__device__ __forceinline__ void lc_leaf_select_range(uint32_t kmin, uint32_t kmax, LcLeafSelSh& sh) {
    kmin = min(kmin, lc_dpp_u<0xB1>(kmin)); kmin = min(kmin, lc_dpp_u<0x4E>(kmin));
    kmin = min(kmin, lc_dpp_u<0x141>(kmin)); kmin = min(kmin, lc_dpp_u<0x140>(kmin));
    kmax = max(kmax, lc_dpp_u<0xB1>(kmax)); kmax = max(kmax, lc_dpp_u<0x4E>(kmax));
    kmax = max(kmax, lc_dpp_u<0x141>(kmax)); kmax = max(kmax, lc_dpp_u<0x140>(kmax));
    if ((threadIdx.x & 15) == 0 && kmax != 0u) {
        atomicMin(reinterpret_cast<unsigned int*>(&sh.mm[0]), kmin);
        atomicMax(reinterpret_cast<unsigned int*>(&sh.mm[1]), kmax);
    }
}

template <int NT>
__device__ __forceinline__ uint32_t lc_leaf_select(int n, uint32_t* skey, const int* slen, long long W, long long C,
                                                   LcLeafSelSh& sh) {
    const int tid = threadIdx.x;
    const uint32_t kmin = (uint32_t)sh.mm[0], kmax = (uint32_t)sh.mm[1];
    if (kmax == 0u) return 0u;                                   // no candidate at all
    int remW = (int)(W > 0x7fffffffLL ? 0x7fffffffLL : (W < 0 ? 0 : W));
    int remC = (int)(C > 0x7fffffffLL ? 0x7fffffffLL : (C < 0 ? 0 : C));
    const bool count_c = C < 0x7fffffffLL;                       // chunk counts matter only with a count limit
    uint32_t lo = kmin, hi = kmax;
    int pass = 0;
    for (;;) {
        const uint32_t span = hi - lo;
        const int bits = span ? 32 - __clz(span) : 0;
        const int shift = bits > LC_LS_BITS ? bits - LC_LS_BITS : 0;     // (span >> shift) < LC_LS_BINS
        if (pass > 0) {                                                  // the first pass was prepared by the caller
            for (int i = tid; i < LC_LS_BINS; i += NT) { sh.hw[i] = 0; sh.hc[i] = 0; }
            if (tid == 0) { sh.res[0] = -1; sh.ncand = 0; }
            __syncthreads();
        }
#pragma unroll 4
        for (int i = tid; i < n; i += NT) {
            const uint32_t k = skey[i];
            if (k >= lo && k <= hi) {
                const int bin = (int)((k - lo) >> shift);
                atomicAdd(&sh.hw[bin], slen[i]);
                if (count_c) atomicAdd(&sh.hc[bin], 1);
            }
        }
        __syncthreads();
        // descending scan: thread t looks at bin 1023 - t (at PER consecutive bins with fewer threads)
        constexpr int PER = LC_LS_BINS / NT;
        int w[PER], c[PER], sw = 0, sc = 0;
#pragma unroll
        for (int j = 0; j < PER; ++j) {
            const int bin = LC_LS_BINS - 1 - (tid * PER + j);
            w[j] = sh.hw[bin];
            c[j] = count_c ? sh.hc[bin] : 0;
            sw += w[j];
            sc += c[j];
        }
        int cw, cc = 0;                                      // length / count of all higher bins
        if (count_c) {
            lc_block_scan2<NT>(sw, sc, sh.scan, &cw, &cc);
        } else {
            int total;
            cw = lc_block_scan<NT>(sw, sh.scan, &total);
        }
#pragma unroll
        for (int j = 0; j < PER; ++j) {
            // the prefix ends in the first bin that no longer fits: everything above it fits, it does not
            if (cw <= remW && cc <= remC && ((long long)cw + w[j] > remW || cc + c[j] > remC)) {
                sh.res[0] = LC_LS_BINS - 1 - (tid * PER + j);
                sh.res[1] = cw;
                sh.res[2] = cc;
            }
            cw += w[j];
            cc += c[j];
        }
        __syncthreads();
        const int fb = sh.res[0];
        if (fb < 0) return lo - 1u;                               // every candidate in scope fits
        remW -= sh.res[1];
        remC -= sh.res[2];
        const uint32_t blo = lo + ((uint32_t)fb << shift);
        const unsigned long long bend = (unsigned long long)blo + ((1ull << shift) - 1ull);
        const uint32_t bhi = bend < (unsigned long long)hi ? (uint32_t)bend : hi;
        // the chunks of that bin go to the short list (as many as it holds; the counter tells how many there are)
#pragma unroll 4
        for (int i = tid; i < n; i += NT) {
            const uint32_t k = skey[i];
            if (k >= blo && k <= bhi) {
                const int pos = atomicAdd(&sh.ncand, 1);
                if (pos < LC_LS_CAND) { sh.ck[pos] = k; sh.cl[pos] = slen[i]; sh.ci[pos] = i; }
            }
        }
        __syncthreads();
        const int nc = sh.ncand;
        if (nc <= LC_LS_CAND) {
            // ---- ranked directly
            const int part = tid & 15;
            for (int c0 = 0; c0 < nc; c0 += NT / 16) {
                const int me = c0 + (tid >> 4);
                const bool valid = me < nc;
                const uint32_t km = valid ? sh.ck[me] : 0u;
                const int im = valid ? sh.ci[me] : 0;
                const int lm = valid ? sh.cl[me] : 0;
                int wb = 0, cb = 0;
                for (int j = part; j < nc; j += 16) {
                    const uint32_t kj = sh.ck[j];
                    const bool before = kj > km || (kj == km && sh.ci[j] < im);
                    wb += before ? sh.cl[j] : 0;
                    cb += before ? 1 : 0;
                }
                wb = lc_sum16_i(wb);
                cb = lc_sum16_i(cb);
                if (valid && part == 0) skey[im] = ((long long)wb + lm <= remW && cb + 1 <= remC) ? 0xffffffffu : 0u;
            }
            __syncthreads();
            return bhi;
        }
        if (blo == bhi) {
            // ---- a tie group too large for the list: cut it in id order
            int E = (n + NT - 1) / NT;
            E |= 1;                                               // odd stride: no LDS bank conflicts
            const int i0 = min(n, tid * E), i1 = min(n, i0 + E);
            int my_w = 0, my_c = 0;
            for (int i = i0; i < i1; ++i)
                if (skey[i] == blo) { my_w += slen[i]; my_c += 1; }
            int tw, tc;
            lc_block_scan2<NT>(my_w, my_c, sh.scan, &tw, &tc);
            long long rw = tw;
            int rc = tc;
            for (int i = i0; i < i1; ++i) {
                if (skey[i] == blo) {
                    rw += slen[i];
                    rc += 1;
                    skey[i] = (rw <= remW && rc <= remC) ? 0xffffffffu : 0u;
                }
            }
            __syncthreads();
            return bhi;
        }
        lo = blo;
        hi = bhi;
        ++pass;
        __syncthreads();                                          // everyone has read the list counter
    }
}

