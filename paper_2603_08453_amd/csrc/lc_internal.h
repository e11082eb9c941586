// Host-side structures shared by the translation units of liblychee.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stddef.h>

#include <vector>

#include "lychee.h"

// Device-side view of an index, passed to kernels by value.
// Per-level arrays are indexed [(b * H + h) * cap[l] + n]; centers carry d floats per node, except that
// center[0] points at rows of d bfloat16 values when c0_bf16 is set (read it through lc_c0_*).
struct LcDev {
    int B, H, d, L, F;
    int c0_bf16;
    int cap[LC_MAX_LEVELS];
    int* state;      // [B][H][4]: {T, M, 0, 0}: tokens written, closed chunks (one copy per head)
    int* nlev;       // [B][LC_MAX_LEVELS]: nodes per level (entry 0 unused: level 0 has M nodes)
    int* bounds;     // [B][cap[0] + 1]: chunk boundaries (shared by the heads of a sequence)
    int* sync;       // [B][H][4]: arrival counters of the fused kernels; zero between calls
    float* center[LC_MAX_LEVELS];
    float* radius[LC_MAX_LEVELS];
    int* parent[LC_MAX_LEVELS];
    int* ntok[LC_MAX_LEVELS];
    int* nchunk[LC_MAX_LEVELS];
    float* rbuild[LC_MAX_LEVELS];   // levels >= 1: the radius as the last (re)build left it (baseline of lc_index_drift)
};

struct lc_index {
    lc_config cfg;
    int B, H_kv, d;
    int device;
    void* buf;
    size_t bytes;
    LcDev dev;
    std::vector<int> T;      // host mirror, per sequence
    std::vector<int> M;      // host mirror, per sequence
    std::vector<int> N;      // [B][LC_MAX_LEVELS] nodes per level (N[b][0] mirrors M)
};

// Layout of the index buffer: fills dev pointers from base; returns total bytes.
size_t lc_layout_index(const lc_config* cfg, int B, int H, int d, void* base, LcDev* dev);

// Workspace carve-up (all offsets 256-byte aligned).
#define LC_KM_FLAGS 64       // k-means iterations whose progress flags the workspace holds
struct LcWs {
    // retrieval
    uint32_t* keys;      // [B][H][cap0] order-preserving score keys of the chunks (0 = not a candidate)
    uint8_t* want;       // [B][H][cap0] 1 = this chunk's score is needed
    int* scratch;        // [B][H][4 * cap0] chunk-level staging when it does not fit in LDS
    int32_t* ids_tmp;    // [B][H][cap0] chunk list of a decode step that has to run as two kernels
    int32_t* counts_tmp; // [B][H]
    // decode
    float* part_acc;     // [B][H][S][G][d]
    float* part_ml;      // [B][H][S][G][2]
    // build
    float* dirs;         // [B][H][cap0][d] unit directions of the level being clustered
    float* cent_a;       // [B][H][cap1][d] centroids (ping)
    float* cent_b;       // [B][H][cap1][d] centroids (pong)
    int* anc;            // [B][H][cap0] chunk -> ancestor at the level being built
    int* kflags;         // [B][H][LC_KM_FLAGS] "iteration t of the k-means moved a point" (tiled kernels only)
    size_t total;
};
// with_build = false leaves out the build scratch (dirs, centroids, ancestors): what a decode step needs.
size_t lc_layout_ws(const lc_config* cfg, int B, int H_q, int H, int d, int splits, void* base, LcWs* ws,
                    bool with_build = true);
int lc_auto_splits(const lc_config* cfg, int B, int H);

void lc_set_hip_error(hipError_t e);
#define LC_HIP_CHECK(expr)                       \
    do {                                         \
        hipError_t _e = (expr);                  \
        if (_e != hipSuccess) {                  \
            lc_set_hip_error(_e);                \
            return LC_ERR_HIP;                   \
        }                                        \
    } while (0)

// lc_decode_step with a switch for the measurement aid that launches its second kernel alone
// (C linkage: it is defined among the entry points).
extern "C" int lc_decode_step_impl(const lc_index* idx, const void* q, const void* K, const void* V,
                                   const int64_t kv_strides[3], int H_q, int budget, float* out, float* lse,
                                   int32_t* chunk_ids, int32_t* counts, int cap, void* ws, size_t ws_bytes,
                                   void* stream, bool second_kernel_only);

// Limits of the two level walks (pure host functions).
int lc_walk_max_internal_nodes();   // exact walk: internal nodes of one (sequence, head), all levels together
int lc_beam_max_level_nodes();      // top-k per level: nodes of one internal level of one (sequence, head)

// Launchers (each enqueues on `stream` and returns LC_OK or LC_ERR_HIP).
int lc_launch_build(const lc_index* idx, const LcWs& ws, const void* K, const int64_t ks[3],
                    int max_M, hipStream_t stream);
int lc_launch_retrieve(const lc_index* idx, const LcWs& ws, const void* q, int G, int budget,
                       int32_t* ids, int32_t* counts, float* scores, int cap,
                       int max_M, int max_upper, int score_only, hipStream_t stream);
int lc_launch_decode(const lc_index* idx, const LcWs& ws, const void* q, const void* K, const void* V,
                     const int64_t ks[3], const int32_t* ids, const int32_t* counts, int cap, int G,
                     int splits, float* out, float* lse, hipStream_t stream);
// Fused step: selection from ws.keys (written by lc_launch_retrieve with score_only) + attention.
// lc_decode_fused_fits tells whether the staged chunk arrays of max_M chunks fit into LDS.
bool lc_decode_fused_fits(int G, int max_M);
int lc_launch_decode_fused(const lc_index* idx, const LcWs& ws, const void* q, const void* K, const void* V,
                           const int64_t ks[3], int G, int splits, int budget, int32_t* ids_out,
                           int32_t* counts_out, int cap, int max_M, float* out, float* lse, hipStream_t stream);
// out (device): [B][H][4] floats: sum of radii at build, sum now, largest growth, nodes counted
int lc_launch_drift(const lc_index* idx, int level, float* out, hipStream_t stream);
// Puts a staged [state | nlev | chunk boundaries of all sequences] block (device memory) in place
// and zeroes the arrival counters.
int lc_launch_place_state(const lc_index* idx, const int32_t* staged, hipStream_t stream);
int lc_launch_append(const lc_index* idx, void* K, void* V, const int64_t ks[3],
                     const void* k_new, const void* v_new, const uint8_t* close_dev_flags_or_null,
                     uint32_t close_mask_lo, hipStream_t stream);
