// C ABI of liblychee: argument validation, buffer layout, handle management.
// All checks that do not need the GPU happen before the first HIP call.
#include <string.h>

#include <mutex>
#include <new>
#include <string>

#include "lc_internal.h"

namespace {

thread_local hipError_t g_last_hip = hipSuccess;

inline size_t align_up(size_t x, size_t a = 256) { return (x + a - 1) / a * a; }

bool config_ok(const lc_config* c) {
    if (!c) return false;
    if (c->levels < 1 || c->levels > LC_MAX_LEVELS) return false;
    if (c->fanout < 1) return false;
    if (c->kmeans_iters < 0) return false;
    if (c->geometry != LC_GEOMETRY_TOKEN_BALL && c->geometry != LC_GEOMETRY_PAPER_UNIT) return false;
    if (c->policy != LC_POLICY_EXACT && c->policy != LC_POLICY_BEAM) return false;
    if (c->sink_tokens < 0) return false;
    if (c->max_chunks < 1 || c->max_tokens < 1) return false;
    if (c->max_chunks > c->max_tokens) return false;
    if (c->max_tokens > (1 << 30)) return false;
    if (c->decode_splits < 0 || c->decode_splits > 256) return false;
    if (c->prune != LC_PRUNE_AUTO && c->prune != LC_PRUNE_ALWAYS && c->prune != LC_PRUNE_NEVER) return false;
    if (c->center_dtype != LC_CENTER_F32 && c->center_dtype != LC_CENTER_BF16) return false;
    for (int l = 0; l < LC_MAX_LEVELS; ++l)
        if (c->fanouts[l] < 0) return false;
    return true;
}

// average children of a level-l node (l >= 1)
int level_fanout(const lc_config* c, int l) { return c->fanouts[l] > 0 ? c->fanouts[l] : c->fanout; }

void level_caps(const lc_config* c, int* cap) {
    cap[0] = c->max_chunks;
    for (int l = 1; l < LC_MAX_LEVELS; ++l) {
        cap[l] = l < c->levels ? (cap[l - 1] + level_fanout(c, l) - 1) / level_fanout(c, l) : 0;
        if (l < c->levels && cap[l] < 1) cap[l] = 1;
    }
}

struct Carver {
    char* base;
    size_t off;
    template <typename T>
    T* take(size_t count) {
        off = align_up(off);
        T* p = base ? reinterpret_cast<T*>(base + off) : nullptr;
        off += count * sizeof(T);
        return p;
    }
};

}  // namespace

void lc_set_hip_error(hipError_t e) { g_last_hip = e; }

size_t lc_layout_index(const lc_config* cfg, int B, int H, int d, void* base, LcDev* dev) {
    LcDev tmp;
    LcDev* D = dev ? dev : &tmp;
    memset(D, 0, sizeof(LcDev));
    D->B = B; D->H = H; D->d = d; D->L = cfg->levels; D->F = cfg->fanout;
    D->c0_bf16 = cfg->center_dtype == LC_CENTER_BF16 ? 1 : 0;
    level_caps(cfg, D->cap);
    Carver c{static_cast<char*>(base), 0};
    const size_t BH = (size_t)B * H;
    D->state = c.take<int>(BH * 4);
    D->sync = c.take<int>(BH * 4);
    D->nlev = c.take<int>((size_t)B * LC_MAX_LEVELS);
    D->bounds = c.take<int>((size_t)B * (D->cap[0] + 1));
    for (int l = 0; l < cfg->levels; ++l) {
        const size_t n = BH * D->cap[l];
        if (l == 0 && D->c0_bf16) D->center[l] = reinterpret_cast<float*>(c.take<uint16_t>(n * d));   // rows of d bfloat16
        else D->center[l] = c.take<float>(n * d);
        D->radius[l] = c.take<float>(n);
        D->parent[l] = c.take<int>(n);
        D->ntok[l] = c.take<int>(n);
        D->nchunk[l] = c.take<int>(n);
        D->rbuild[l] = l >= 1 ? c.take<float>(n) : nullptr;
    }
    return align_up(c.off);
}

int lc_auto_splits(const lc_config* cfg, int B, int H) {
    if (cfg->decode_splits > 0) return cfg->decode_splits;
    // about two workgroups per compute unit (512 in all): at small batch the kernel is a chain of memory
    // round trips and every extra split lengthens the merge
    int s = (512 + B * H - 1) / (B * H);
    if (s < 1) s = 1;
    if (s > 32) s = 32;
    return s;
}

size_t lc_layout_ws(const lc_config* cfg, int B, int H_q, int H, int d, int splits, void* base, LcWs* ws,
                    bool with_build) {
    LcWs tmp;
    LcWs* W = ws ? ws : &tmp;
    int cap[LC_MAX_LEVELS];
    level_caps(cfg, cap);
    const int cap1 = cfg->levels > 1 ? cap[1] : 1;
    const size_t BH = (size_t)B * H;
    Carver c{static_cast<char*>(base), 0};
    W->keys = c.take<uint32_t>(BH * cap[0]);
    W->want = c.take<uint8_t>(BH * cap[0]);
    W->scratch = c.take<int>(BH * 4 * cap[0]);
    W->ids_tmp = c.take<int32_t>(BH * cap[0]);
    W->counts_tmp = c.take<int32_t>(BH);
    W->part_acc = c.take<float>((size_t)B * H_q * splits * d);
    W->part_ml = c.take<float>((size_t)B * H_q * splits * 2);
    W->dirs = W->cent_a = W->cent_b = nullptr;
    W->anc = nullptr;
    W->kflags = nullptr;
    if (with_build) {
        W->dirs = c.take<float>(BH * cap[0] * d);
        W->cent_a = c.take<float>(BH * cap1 * d);
        W->cent_b = c.take<float>(BH * cap1 * d);
        W->anc = c.take<int>(BH * cap[0]);
        W->kflags = c.take<int>(BH * LC_KM_FLAGS);
    }
    W->total = align_up(c.off);
    return W->total;
}

extern "C" {

void lc_config_default(lc_config* cfg) {
    if (!cfg) return;
    memset(cfg, 0, sizeof(*cfg));
    cfg->levels = 3;
    cfg->fanout = 16;
    cfg->kmeans_iters = 10;
    cfg->geometry = LC_GEOMETRY_TOKEN_BALL;
    cfg->policy = LC_POLICY_EXACT;
}

const char* lc_strerror(int code) {
    switch (code) {
        case LC_OK: return "ok";
        case LC_ERR_INVALID_ARG: return "invalid argument";
        case LC_ERR_BAD_SHAPE: return "unsupported shape (need d = 128, H_q a multiple of H_kv, group size <= 8, strides multiple of 8)";
        case LC_ERR_WORKSPACE_TOO_SMALL: return "index buffer or workspace too small";
        case LC_ERR_CAPACITY: return "capacity exceeded";
        case LC_ERR_HIP: return "HIP runtime error";
        case LC_ERR_BAD_BLOB: return "malformed index blob";
    }
    return "unknown error";
}

const char* lc_last_hip_error(void) { return hipGetErrorString(g_last_hip); }

size_t lc_index_bytes(const lc_config* cfg, int B, int H_kv, int d) {
    if (!config_ok(cfg) || B < 1 || H_kv < 1 || d != LC_HEAD_DIM) return 0;
    return lc_layout_index(cfg, B, H_kv, d, nullptr, nullptr);
}

size_t lc_workspace_bytes(const lc_config* cfg, int B, int H_q, int H_kv, int d) {
    if (!config_ok(cfg) || B < 1 || H_kv < 1 || H_q < H_kv || H_q % H_kv != 0 || d != LC_HEAD_DIM) return 0;
    if (H_q / H_kv > LC_MAX_GROUP) return 0;
    return lc_layout_ws(cfg, B, H_q, H_kv, d, lc_auto_splits(cfg, B, H_kv), nullptr, nullptr);
}

}  // extern "C"

namespace {

int check_shape(int B, int H_kv, int d) {
    if (B < 1 || H_kv < 1) return LC_ERR_INVALID_ARG;
    if (d != LC_HEAD_DIM) return LC_ERR_BAD_SHAPE;
    return LC_OK;
}

int check_strides(const int64_t s[3]) {
    if (!s) return LC_ERR_INVALID_ARG;
    for (int i = 0; i < 3; ++i)
        if (s[i] < 0 || s[i] % 8 != 0) return LC_ERR_BAD_SHAPE;
    if (s[2] < LC_HEAD_DIM) return LC_ERR_BAD_SHAPE;
    return LC_OK;
}

bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

lc_index* new_handle(const lc_config* cfg, int B, int H, int d, void* buf, size_t bytes) {
    lc_index* h = new (std::nothrow) lc_index();
    if (!h) return nullptr;
    h->cfg = *cfg;
    h->B = B; h->H_kv = H; h->d = d;
    h->device = 0;
    h->buf = buf;
    h->bytes = bytes;
    lc_layout_index(cfg, B, H, d, buf, &h->dev);
    h->T.assign(B, 0);
    h->M.assign(B, 0);
    h->N.assign((size_t)B * LC_MAX_LEVELS, 0);
    return h;
}

void fill_level_counts(lc_index* h) {
    for (int b = 0; b < h->B; ++b) {
        int n = h->M[b];
        h->N[(size_t)b * LC_MAX_LEVELS + 0] = n;
        for (int l = 1; l < h->cfg.levels; ++l) {
            n = (n + level_fanout(&h->cfg, l) - 1) / level_fanout(&h->cfg, l);
            if (n < 1) n = 1;
            h->N[(size_t)b * LC_MAX_LEVELS + l] = n;
        }
    }
}

// Host side of the small uploads (counts, chunk boundaries): one pinned buffer per device, kept for
// the life of the process and grown on demand, so that an upload is one asynchronous copy and no
// wait for the stream.  The event marks the last copy that read the buffer; it is waited for before
// the buffer is written again (long done, normally).
struct LcStage {
    int32_t* host = nullptr;
    size_t ints = 0;
    hipEvent_t read = nullptr;
};
constexpr int LC_STAGE_DEVICES = 64;
LcStage g_stage[LC_STAGE_DEVICES];
std::mutex g_stage_mutex;

// Returns the current device's buffer with room for `ints` values (the lock must be held).
int stage_reserve(size_t ints, LcStage** out) {
    int dev = 0;
    LC_HIP_CHECK(hipGetDevice(&dev));
    if (dev < 0 || dev >= LC_STAGE_DEVICES) return LC_ERR_INVALID_ARG;
    LcStage& st = g_stage[dev];
    if (!st.read) LC_HIP_CHECK(hipEventCreateWithFlags(&st.read, hipEventDisableTiming));
    else LC_HIP_CHECK(hipEventSynchronize(st.read));
    if (st.ints < ints) {
        if (st.host) LC_HIP_CHECK(hipHostFree(st.host));
        st.host = nullptr;
        st.ints = 0;
        const size_t want = ints < 16384 ? 16384 : ints + ints / 2;
        LC_HIP_CHECK(hipHostMalloc(reinterpret_cast<void**>(&st.host), want * sizeof(int32_t), hipHostMallocDefault));
        st.ints = want;
    }
    *out = &st;
    return LC_OK;
}

// state, nlev, zeroed arrival counters and chunk boundaries -> device: staged as
// [state | nlev | boundaries of all sequences], copied once into `dev_stage` (workspace memory the
// build overwrites later) and put in place by one kernel.
int upload_state(lc_index* h, const int32_t* bounds_concat, void* dev_stage, hipStream_t stream) {
    const int B = h->B, H = h->H_kv;
    const size_t n_state = (size_t)B * H * 4, n_nlev = (size_t)B * LC_MAX_LEVELS;
    size_t n_bounds = 0;
    for (int b = 0; b < B; ++b) n_bounds += (size_t)h->M[b] + 1;
    const size_t total = n_state + n_nlev + n_bounds;
    std::lock_guard<std::mutex> lock(g_stage_mutex);
    LcStage* st = nullptr;
    const int rc = stage_reserve(total, &st);
    if (rc != LC_OK) return rc;
    int32_t* p = st->host;
    memset(p, 0, n_state * sizeof(int32_t));
    for (int b = 0; b < B; ++b) {
        for (int hh = 0; hh < H; ++hh) {
            p[((size_t)b * H + hh) * 4 + 0] = h->T[b];
            p[((size_t)b * H + hh) * 4 + 1] = h->M[b];
        }
    }
    for (size_t i = 0; i < n_nlev; ++i) p[n_state + i] = h->N[i];
    memcpy(p + n_state + n_nlev, bounds_concat, n_bounds * sizeof(int32_t));
    LC_HIP_CHECK(hipMemcpyAsync(dev_stage, p, total * sizeof(int32_t), hipMemcpyHostToDevice, stream));
    LC_HIP_CHECK(hipEventRecord(st->read, stream));
    return lc_launch_place_state(h, static_cast<const int32_t*>(dev_stage), stream);
}

// nodes per level -> device (lc_recluster)
int upload_level_counts(lc_index* h, hipStream_t stream) {
    const size_t n_nlev = (size_t)h->B * LC_MAX_LEVELS;
    std::lock_guard<std::mutex> lock(g_stage_mutex);
    LcStage* st = nullptr;
    const int rc = stage_reserve(n_nlev, &st);
    if (rc != LC_OK) return rc;
    for (size_t i = 0; i < n_nlev; ++i) st->host[i] = h->N[i];
    LC_HIP_CHECK(hipMemcpyAsync(h->dev.nlev, st->host, n_nlev * sizeof(int32_t), hipMemcpyHostToDevice, stream));
    LC_HIP_CHECK(hipEventRecord(st->read, stream));
    return LC_OK;
}

}  // namespace

extern "C" {

int lc_build_index(lc_index** out, const lc_config* cfg, const void* K, const int64_t k_strides[3],
                   const int32_t* seq_lens, const int32_t* chunk_bounds, const int32_t* chunk_counts,
                   int B, int H_kv, int d, void* index_buf, size_t index_bytes, void* ws, size_t ws_bytes,
                   void* stream) {
    if (!out || !cfg || !K || !seq_lens || !chunk_bounds || !chunk_counts || !index_buf || !ws)
        return LC_ERR_INVALID_ARG;
    if (!config_ok(cfg)) return LC_ERR_INVALID_ARG;
    int rc = check_shape(B, H_kv, d);
    if (rc) return rc;
    rc = check_strides(k_strides);
    if (rc) return rc;
    if (!aligned16(K) || (reinterpret_cast<uintptr_t>(index_buf) & 255u) || (reinterpret_cast<uintptr_t>(ws) & 255u))
        return LC_ERR_INVALID_ARG;
    size_t off = 0;
    for (int b = 0; b < B; ++b) {
        const int M = chunk_counts[b], T = seq_lens[b];
        if (M < 0 || T < 0) return LC_ERR_INVALID_ARG;
        if (M > cfg->max_chunks || T > cfg->max_tokens) return LC_ERR_CAPACITY;
        const int32_t* bd = chunk_bounds + off;
        if (bd[0] != 0) return LC_ERR_INVALID_ARG;
        for (int j = 0; j < M; ++j)
            if (bd[j + 1] <= bd[j]) return LC_ERR_INVALID_ARG;
        if (bd[M] > T) return LC_ERR_INVALID_ARG;
        off += (size_t)M + 1;
    }
    if (index_bytes < lc_layout_index(cfg, B, H_kv, d, nullptr, nullptr)) return LC_ERR_WORKSPACE_TOO_SMALL;
    // the build does not depend on the number of query heads: size with G = 1
    LcWs w;
    if (ws_bytes < lc_layout_ws(cfg, B, H_kv, H_kv, d, 1, nullptr, nullptr)) return LC_ERR_WORKSPACE_TOO_SMALL;
    lc_layout_ws(cfg, B, H_kv, H_kv, d, 1, ws, &w);

    lc_index* h = new_handle(cfg, B, H_kv, d, index_buf, index_bytes);
    if (!h) return LC_ERR_INVALID_ARG;
    int max_M = 0;
    for (int b = 0; b < B; ++b) {
        h->T[b] = seq_lens[b];
        h->M[b] = chunk_counts[b];
        if (h->M[b] > max_M) max_M = h->M[b];
    }
    fill_level_counts(h);
    hipStream_t s = static_cast<hipStream_t>(stream);
    rc = upload_state(h, chunk_bounds, w.dirs, s);
    if (rc == LC_OK) rc = lc_launch_build(h, w, K, k_strides, max_M, s);
    if (rc != LC_OK) {
        delete h;
        return rc;
    }
    *out = h;
    return LC_OK;
}

int lc_recluster(lc_index* idx, void* ws, size_t ws_bytes, void* stream) {
    if (!idx || !ws || (reinterpret_cast<uintptr_t>(ws) & 255u)) return LC_ERR_INVALID_ARG;
    LcWs w;
    if (ws_bytes < lc_layout_ws(&idx->cfg, idx->B, idx->H_kv, idx->H_kv, idx->d, 1, nullptr, nullptr))
        return LC_ERR_WORKSPACE_TOO_SMALL;
    lc_layout_ws(&idx->cfg, idx->B, idx->H_kv, idx->H_kv, idx->d, 1, ws, &w);
    hipStream_t s = static_cast<hipStream_t>(stream);
    fill_level_counts(idx);                       // nodes per level follow the current chunk counts
    const int rc = upload_level_counts(idx, s);
    if (rc != LC_OK) return rc;
    int max_M = 0;
    for (int b = 0; b < idx->B; ++b)
        if (idx->M[b] > max_M) max_M = idx->M[b];
    const int64_t no_strides[3] = {0, 0, 0};
    return lc_launch_build(idx, w, nullptr, no_strides, max_M, s);
}

int lc_set_policy(lc_index* idx, int policy, const int32_t* beam, int sink_tokens) {
    if (!idx) return LC_ERR_INVALID_ARG;
    if (policy != LC_POLICY_EXACT && policy != LC_POLICY_BEAM) return LC_ERR_INVALID_ARG;
    if (sink_tokens < 0) return LC_ERR_INVALID_ARG;
    idx->cfg.policy = policy;
    idx->cfg.sink_tokens = sink_tokens;
    for (int l = 0; l < LC_MAX_LEVELS; ++l) idx->cfg.beam[l] = beam ? beam[l] : 0;
    return LC_OK;
}

int lc_set_prune(lc_index* idx, int prune) {
    if (!idx) return LC_ERR_INVALID_ARG;
    if (prune != LC_PRUNE_AUTO && prune != LC_PRUNE_ALWAYS && prune != LC_PRUNE_NEVER) return LC_ERR_INVALID_ARG;
    idx->cfg.prune = prune;
    return LC_OK;
}

int lc_index_drift(const lc_index* idx, int level, float* drift, void* ws, size_t ws_bytes, void* stream) {
    if (!idx || !drift || !ws || (reinterpret_cast<uintptr_t>(ws) & 255u)) return LC_ERR_INVALID_ARG;
    if (level < 1 || level >= idx->cfg.levels) return LC_ERR_INVALID_ARG;
    const size_t n = (size_t)idx->B * idx->H_kv * 4;
    if (ws_bytes < n * sizeof(float)) return LC_ERR_WORKSPACE_TOO_SMALL;
    hipStream_t s = static_cast<hipStream_t>(stream);
    int rc = lc_launch_drift(idx, level, static_cast<float*>(ws), s);
    if (rc) return rc;
    LC_HIP_CHECK(hipMemcpyAsync(drift, ws, n * sizeof(float), hipMemcpyDeviceToHost, s));
    LC_HIP_CHECK(hipStreamSynchronize(s));
    return LC_OK;
}

void lc_walk_limits(int32_t* exact_walk_internal_nodes, int32_t* beam_level_nodes) {
    if (exact_walk_internal_nodes) *exact_walk_internal_nodes = lc_walk_max_internal_nodes();
    if (beam_level_nodes) *beam_level_nodes = lc_beam_max_level_nodes();
}

int lc_index_info(const lc_index* idx, int b, int32_t* T, int32_t* M, int32_t* n_per_level) {
    if (!idx || b < 0 || b >= idx->B) return LC_ERR_INVALID_ARG;
    if (T) *T = idx->T[b];
    if (M) *M = idx->M[b];
    if (n_per_level)
        for (int l = 0; l < LC_MAX_LEVELS; ++l)
            n_per_level[l] = l < idx->cfg.levels ? idx->N[(size_t)b * LC_MAX_LEVELS + l] : 0;
    return LC_OK;
}

static int common_decode_checks(const lc_index* idx, const void* q, int H_q, int cap) {
    if (!idx || !q) return LC_ERR_INVALID_ARG;
    if (H_q < idx->H_kv || H_q % idx->H_kv != 0) return LC_ERR_BAD_SHAPE;
    if (H_q / idx->H_kv > LC_MAX_GROUP) return LC_ERR_BAD_SHAPE;
    if (cap < 1) return LC_ERR_INVALID_ARG;
    if (!aligned16(q)) return LC_ERR_INVALID_ARG;
    return LC_OK;
}

#define LC_STEP_FUSED_MAX_CHUNKS 4096

namespace {
// What a retrieval over the current index needs: sizes, the capacity check, walk or flat scan.
struct RetrievePlan {
    int max_M = 0;
    int max_upper = 0;          // internal nodes of one (sequence, head), all levels together
    int max_level = 0;          // nodes of one internal level
    bool walk = false;
};
int plan_retrieve(const lc_index* idx, int budget, int cap, bool check_cap, RetrievePlan* p) {
    long long leaf_bytes = 0;
    for (int b = 0; b < idx->B; ++b) {
        const int M = idx->M[b];
        if (M > p->max_M) p->max_M = M;
        leaf_bytes += (long long)M * idx->H_kv * (idx->d * (idx->dev.c0_bf16 ? 2 : 4) + 8);
        // every chunk holds >= 1 token: at most `budget` chunks fit, plus the pinned ones
        long long need = (long long)budget + idx->cfg.sink_tokens;
        if (need > M) need = M;
        if (check_cap && cap < need) return LC_ERR_CAPACITY;
        int up = 0;
        for (int l = 1; l < idx->cfg.levels; ++l) {
            const int n = idx->N[(size_t)b * LC_MAX_LEVELS + l];
            up += n;
            if (n > p->max_level) p->max_level = n;
        }
        if (up > p->max_upper) p->max_upper = up;
    }
    // walk the internal levels?  BEAM: always.  EXACT: by mode; the result does not depend on it.
    p->walk = idx->cfg.levels > 1;
    if (p->walk && idx->cfg.policy == LC_POLICY_EXACT) {
        if (idx->cfg.prune == LC_PRUNE_NEVER) p->walk = false;
        else if (idx->cfg.prune == LC_PRUNE_AUTO) p->walk = leaf_bytes > (long long)LC_PRUNE_AUTO_BYTES;
    }
    // What the walks hold on chip: the exact walk keeps every internal node of a (sequence, head) in
    // LDS; top-k per level keeps a kept-bit per node of a level.  A flat scan reads no internal node.
    if (idx->cfg.policy == LC_POLICY_BEAM) {
        if (p->max_level > lc_beam_max_level_nodes()) return LC_ERR_CAPACITY;
    } else if (p->walk) {
        if (p->max_upper > lc_walk_max_internal_nodes()) {
            if (idx->cfg.prune == LC_PRUNE_ALWAYS) return LC_ERR_CAPACITY;
            p->walk = false;                      // AUTO: the flat scan gives the same selection
        }
    }
    return LC_OK;
}
}  // namespace

int lc_retrieve(const lc_index* idx, const void* q, int H_q, int budget, int32_t* chunk_ids, int32_t* counts,
                float* scores, int cap, void* ws, size_t ws_bytes, void* stream) {
    int rc = common_decode_checks(idx, q, H_q, cap);
    if (rc) return rc;
    if (!chunk_ids || !counts || !ws) return LC_ERR_INVALID_ARG;
    if (budget < 0) return LC_ERR_INVALID_ARG;
    if (reinterpret_cast<uintptr_t>(ws) & 255u) return LC_ERR_INVALID_ARG;
    const int splits = lc_auto_splits(&idx->cfg, idx->B, idx->H_kv);
    if (ws_bytes < lc_layout_ws(&idx->cfg, idx->B, H_q, idx->H_kv, idx->d, splits, nullptr, nullptr))
        return LC_ERR_WORKSPACE_TOO_SMALL;
    RetrievePlan p;
    rc = plan_retrieve(idx, budget, cap, true, &p);
    if (rc) return rc;
    LcWs w;
    lc_layout_ws(&idx->cfg, idx->B, H_q, idx->H_kv, idx->d, splits, ws, &w);
    return lc_launch_retrieve(idx, w, q, H_q / idx->H_kv, budget, chunk_ids, counts, scores, cap, p.max_M,
                              p.walk ? p.max_upper : -1, 0, static_cast<hipStream_t>(stream));
}

namespace {
// Argument checks of a decode step that need neither the workspace nor the GPU.
int decode_step_checks(const lc_index* idx, const void* q, const void* K, const void* V, const int64_t kv_strides[3],
                       int H_q, int budget, float* out, int32_t* chunk_ids, int32_t* counts, int cap) {
    const bool want_ids = chunk_ids != nullptr;
    int rc = common_decode_checks(idx, q, H_q, want_ids ? cap : 1);
    if (rc) return rc;
    if (!K || !V || !out || budget < 0) return LC_ERR_INVALID_ARG;
    if (want_ids != (counts != nullptr)) return LC_ERR_INVALID_ARG;
    rc = check_strides(kv_strides);
    if (rc) return rc;
    if (!aligned16(K) || !aligned16(V)) return LC_ERR_INVALID_ARG;
    if ((long long)idx->cfg.max_tokens * kv_strides[2] * 2 >= (1LL << 31)) return LC_ERR_BAD_SHAPE;
    return LC_OK;
}

// The step itself on a laid-out workspace (every check has passed).
int decode_step_run(const lc_index* idx, const LcWs& w, const RetrievePlan& p, int splits, const void* q,
                    const void* K, const void* V, const int64_t kv_strides[3], int H_q, int budget, float* out,
                    float* lse, int32_t* chunk_ids, int32_t* counts, int cap, hipStream_t st,
                    bool second_kernel_only = false) {
    const bool want_ids = chunk_ids != nullptr;
    const int G = H_q / idx->H_kv;
    int rc;
    // Every workgroup of the fused kernel repeats the selection with 256 threads: with a few thousand
    // chunks that is cheaper than the hand-off through a chunk list, with more it is not.
    if (idx->cfg.policy != LC_POLICY_BEAM && p.max_M <= LC_STEP_FUSED_MAX_CHUNKS && lc_decode_fused_fits(G, p.max_M)) {
        // kernel 1 (and the level walk before it) leaves the chunk score keys in the workspace;
        // kernel 2 selects from them in every workgroup and attends
        if (!second_kernel_only) {
            rc = lc_launch_retrieve(idx, w, q, G, budget, nullptr, nullptr, nullptr, 1, p.max_M,
                                    p.walk ? p.max_upper : -1, 1, st);
            if (rc) return rc;
        }
        return lc_launch_decode_fused(idx, w, q, K, V, kv_strides, G, splits, budget, chunk_ids, counts,
                                      want_ids ? cap : 0, p.max_M, out, lse, st);
    }
    if (second_kernel_only) return LC_ERR_CAPACITY;
    // too many chunks for the registers of the selecting workgroups: the two kernels of lc_retrieve + lc_sparse_decode, with the
    // chunk list in the caller's buffer or, without one, in the workspace
    int32_t* ids = want_ids ? chunk_ids : w.ids_tmp;
    int32_t* cnt = want_ids ? counts : w.counts_tmp;
    int icap = cap;
    if (!want_ids) {
        int cap0 = idx->cfg.max_chunks;
        icap = cap0 < 1 ? 1 : cap0;
    }
    rc = lc_launch_retrieve(idx, w, q, G, budget, ids, cnt, nullptr, icap, p.max_M, p.walk ? p.max_upper : -1, 0, st);
    if (rc) return rc;
    return lc_launch_decode(idx, w, q, K, V, kv_strides, ids, cnt, icap, G, splits, out, lse, st);
}
}  // namespace

int lc_decode_step(const lc_index* idx, const void* q, const void* K, const void* V, const int64_t kv_strides[3],
                   int H_q, int budget, float* out, float* lse, int32_t* chunk_ids, int32_t* counts, int cap,
                   void* ws, size_t ws_bytes, void* stream) {
    return lc_decode_step_impl(idx, q, K, V, kv_strides, H_q, budget, out, lse, chunk_ids, counts, cap, ws, ws_bytes,
                               stream, false);
}

int lc_decode_step_impl(const lc_index* idx, const void* q, const void* K, const void* V, const int64_t kv_strides[3],
                        int H_q, int budget, float* out, float* lse, int32_t* chunk_ids, int32_t* counts, int cap,
                        void* ws, size_t ws_bytes, void* stream, bool second_kernel_only) {
    int rc = decode_step_checks(idx, q, K, V, kv_strides, H_q, budget, out, chunk_ids, counts, cap);
    if (rc) return rc;
    if (!ws || (reinterpret_cast<uintptr_t>(ws) & 255u)) return LC_ERR_INVALID_ARG;
    const int splits = lc_auto_splits(&idx->cfg, idx->B, idx->H_kv);
    if (ws_bytes < lc_layout_ws(&idx->cfg, idx->B, H_q, idx->H_kv, idx->d, splits, nullptr, nullptr))
        return LC_ERR_WORKSPACE_TOO_SMALL;
    RetrievePlan p;
    rc = plan_retrieve(idx, budget, cap, chunk_ids != nullptr, &p);
    if (rc) return rc;
    LcWs w;
    lc_layout_ws(&idx->cfg, idx->B, H_q, idx->H_kv, idx->d, splits, ws, &w);
    return decode_step_run(idx, w, p, splits, q, K, V, kv_strides, H_q, budget, out, lse, chunk_ids, counts, cap,
                           static_cast<hipStream_t>(stream), second_kernel_only);
}

// ---------------------------------------------------------------------------------
// decode step without a caller workspace
// ---------------------------------------------------------------------------------
// The workspace of a decode step (score keys, kept flags, select staging, chunk list, split-K
// partials) in a file-scope device array instead of a caller buffer, for callers that cannot
// allocate.  In host code the array's name is only a stand-in: its device address is asked for
// once per device and kept; kernels and layout code only ever see that address.
static __device__ __align__(256) unsigned char lc_static_scratch[LC_STATIC_SCRATCH_BYTES];

namespace {
constexpr int kMaxDevices = 64;
void* g_scratch_ptr[kMaxDevices] = {};
std::mutex g_scratch_mutex;

// Device address of the static scratch array on the current device (asked for on first use).
int static_scratch(void** out) {
    int dev = -1;
    LC_HIP_CHECK(hipGetDevice(&dev));
    if (dev < 0 || dev >= kMaxDevices) return LC_ERR_CAPACITY;
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (g_scratch_ptr[dev] == nullptr) {
        void* ptr = nullptr;
        LC_HIP_CHECK(hipGetSymbolAddress(&ptr, HIP_SYMBOL(lc_static_scratch)));
        if (ptr == nullptr || (reinterpret_cast<uintptr_t>(ptr) & 255u)) return LC_ERR_HIP;
        g_scratch_ptr[dev] = ptr;
    }
    *out = g_scratch_ptr[dev];
    return LC_OK;
}
}  // namespace

size_t lc_static_workspace_bytes(void) { return (size_t)LC_STATIC_SCRATCH_BYTES; }

size_t lc_decode_workspace_bytes(const lc_config* cfg, int B, int H_q, int H_kv, int d) {
    if (!config_ok(cfg) || B < 1 || H_kv < 1 || H_q < H_kv || H_q % H_kv != 0 || d != LC_HEAD_DIM) return 0;
    if (H_q / H_kv > LC_MAX_GROUP) return 0;
    return lc_layout_ws(cfg, B, H_q, H_kv, d, lc_auto_splits(cfg, B, H_kv), nullptr, nullptr, false);
}

int lc_decode_step_static(const lc_index* idx, const void* q, const void* K, const void* V,
                          const int64_t kv_strides[3], int H_q, int budget, float* out, float* lse,
                          int32_t* chunk_ids, int32_t* counts, int cap, void* stream) {
    int rc = decode_step_checks(idx, q, K, V, kv_strides, H_q, budget, out, chunk_ids, counts, cap);
    if (rc) return rc;
    const int splits = lc_auto_splits(&idx->cfg, idx->B, idx->H_kv);
    if (lc_layout_ws(&idx->cfg, idx->B, H_q, idx->H_kv, idx->d, splits, nullptr, nullptr, false) >
        (size_t)LC_STATIC_SCRATCH_BYTES)
        return LC_ERR_CAPACITY;
    RetrievePlan p;
    rc = plan_retrieve(idx, budget, cap, chunk_ids != nullptr, &p);
    if (rc) return rc;
    void* base = nullptr;
    rc = static_scratch(&base);
    if (rc) return rc;
    LcWs w;
    lc_layout_ws(&idx->cfg, idx->B, H_q, idx->H_kv, idx->d, splits, base, &w, false);
    return decode_step_run(idx, w, p, splits, q, K, V, kv_strides, H_q, budget, out, lse, chunk_ids, counts, cap,
                           static_cast<hipStream_t>(stream));
}

int lc_sparse_decode(const lc_index* idx, const void* q, const void* K, const void* V, const int64_t kv_strides[3],
                     const int32_t* chunk_ids, const int32_t* counts, int cap, int H_q, float* out, float* lse,
                     void* ws, size_t ws_bytes, void* stream) {
    int rc = common_decode_checks(idx, q, H_q, cap);
    if (rc) return rc;
    if (!K || !V || !chunk_ids || !counts || !out || !ws) return LC_ERR_INVALID_ARG;
    rc = check_strides(kv_strides);
    if (rc) return rc;
    if (!aligned16(K) || !aligned16(V) || (reinterpret_cast<uintptr_t>(ws) & 255u)) return LC_ERR_INVALID_ARG;
    const int splits = lc_auto_splits(&idx->cfg, idx->B, idx->H_kv);
    if (ws_bytes < lc_layout_ws(&idx->cfg, idx->B, H_q, idx->H_kv, idx->d, splits, nullptr, nullptr))
        return LC_ERR_WORKSPACE_TOO_SMALL;
    // the kernel addresses the rows of one (sequence, head) with 32-bit byte offsets
    if ((long long)idx->cfg.max_tokens * kv_strides[2] * 2 >= (1LL << 31)) return LC_ERR_BAD_SHAPE;
    LcWs w;
    lc_layout_ws(&idx->cfg, idx->B, H_q, idx->H_kv, idx->d, splits, ws, &w);
    return lc_launch_decode(idx, w, q, K, V, kv_strides, chunk_ids, counts, cap, H_q / idx->H_kv, splits, out, lse,
                            static_cast<hipStream_t>(stream));
}

int lc_append(lc_index* idx, void* K, void* V, const int64_t kv_strides[3], const void* k_new, const void* v_new,
              const uint8_t* close_chunk, void* ws, size_t ws_bytes, void* stream) {
    (void)ws; (void)ws_bytes;
    if (!idx || !K || !V || !k_new || !v_new) return LC_ERR_INVALID_ARG;
    int rc = check_strides(kv_strides);
    if (rc) return rc;
    if (!aligned16(K) || !aligned16(V) || !aligned16(k_new) || !aligned16(v_new)) return LC_ERR_INVALID_ARG;
    if (idx->B > 1024) return LC_ERR_CAPACITY;
    for (int b = 0; b < idx->B; ++b) {
        if (idx->T[b] + 1 > idx->cfg.max_tokens) return LC_ERR_CAPACITY;
        if (close_chunk && close_chunk[b] && idx->M[b] + 1 > idx->cfg.max_chunks) return LC_ERR_CAPACITY;
    }
    rc = lc_launch_append(idx, K, V, kv_strides, k_new, v_new, close_chunk, 0u, static_cast<hipStream_t>(stream));
    if (rc != LC_OK) return rc;
    for (int b = 0; b < idx->B; ++b) {
        idx->T[b] += 1;
        if (close_chunk && close_chunk[b]) {
            idx->M[b] += 1;
            idx->N[(size_t)b * LC_MAX_LEVELS + 0] = idx->M[b];
        }
    }
    return LC_OK;
}

// ---------------------------------------------------------------------------------
// export / import
// ---------------------------------------------------------------------------------
static const int32_t kMagic = 0x5849434C;    // 'L','C','I','X'

static size_t blob_size(const lc_index* idx) {
    size_t n = 16 * 4;
    const int L = idx->cfg.levels;
    for (int b = 0; b < idx->B; ++b) {
        n += (size_t)(2 + (L - 1)) * 4 + ((size_t)idx->M[b] + 1) * 4;
        for (int l = 0; l < L; ++l) {
            const size_t nl = idx->N[(size_t)b * LC_MAX_LEVELS + l];
            n += (size_t)idx->H_kv * nl * ((size_t)idx->d * 4 + 16);
        }
    }
    return n;
}

int lc_index_export(const lc_index* idx, void* blob, size_t* bytes, void* stream) {
    if (!idx || !bytes) return LC_ERR_INVALID_ARG;
    const size_t need = blob_size(idx);
    if (!blob) { *bytes = need; return LC_OK; }
    if (*bytes < need) { *bytes = need; return LC_ERR_WORKSPACE_TOO_SMALL; }
    *bytes = need;
    hipStream_t s = static_cast<hipStream_t>(stream);
    LC_HIP_CHECK(hipStreamSynchronize(s));
    char* p = static_cast<char*>(blob);
    int32_t hdr[16] = {kMagic, 1, idx->B, idx->H_kv, idx->d, idx->cfg.levels, idx->cfg.fanout, idx->cfg.geometry,
                       idx->cfg.center_dtype};
    for (int l = 1; l < LC_MAX_LEVELS; ++l) hdr[8 + l] = idx->cfg.fanouts[l];
    memcpy(p, hdr, sizeof(hdr));
    p += sizeof(hdr);
    const int L = idx->cfg.levels;
    const LcDev& D = idx->dev;
    for (int b = 0; b < idx->B; ++b) {
        int32_t rec[2 + LC_MAX_LEVELS];
        rec[0] = idx->T[b];
        rec[1] = idx->M[b];
        for (int l = 1; l < L; ++l) rec[1 + l] = idx->N[(size_t)b * LC_MAX_LEVELS + l];
        memcpy(p, rec, (size_t)(2 + (L - 1)) * 4);
        p += (size_t)(2 + (L - 1)) * 4;
        const size_t nb = ((size_t)idx->M[b] + 1) * 4;
        LC_HIP_CHECK(hipMemcpy(p, D.bounds + (size_t)b * (D.cap[0] + 1), nb, hipMemcpyDeviceToHost));
        p += nb;
    }
    for (int b = 0; b < idx->B; ++b)
        for (int h = 0; h < idx->H_kv; ++h)
            for (int l = 0; l < L; ++l) {
                const size_t nl = idx->N[(size_t)b * LC_MAX_LEVELS + l];
                const size_t base = ((size_t)b * idx->H_kv + h) * D.cap[l];
                if (nl == 0) continue;
                if (l == 0 && D.c0_bf16) {
                    // the blob always carries float32 centers: widen the stored bfloat16 values
                    std::vector<uint16_t> half(nl * idx->d);
                    LC_HIP_CHECK(hipMemcpy(half.data(), reinterpret_cast<const uint16_t*>(D.center[0]) + base * idx->d,
                                           nl * idx->d * 2, hipMemcpyDeviceToHost));
                    for (size_t i = 0; i < half.size(); ++i) {
                        const uint32_t w = (uint32_t)half[i] << 16;
                        memcpy(p + 4 * i, &w, 4);
                    }
                } else {
                    LC_HIP_CHECK(hipMemcpy(p, D.center[l] + base * idx->d, nl * idx->d * 4, hipMemcpyDeviceToHost));
                }
                p += nl * idx->d * 4;
                LC_HIP_CHECK(hipMemcpy(p, D.radius[l] + base, nl * 4, hipMemcpyDeviceToHost)); p += nl * 4;
                LC_HIP_CHECK(hipMemcpy(p, D.parent[l] + base, nl * 4, hipMemcpyDeviceToHost)); p += nl * 4;
                LC_HIP_CHECK(hipMemcpy(p, D.ntok[l] + base, nl * 4, hipMemcpyDeviceToHost)); p += nl * 4;
                LC_HIP_CHECK(hipMemcpy(p, D.nchunk[l] + base, nl * 4, hipMemcpyDeviceToHost)); p += nl * 4;
            }
    return LC_OK;
}

int lc_index_import(lc_index** out, const lc_config* cfg, const void* blob, size_t blob_bytes, void* index_buf,
                    size_t index_bytes, void* stream) {
    if (!out || !cfg || !blob || !index_buf) return LC_ERR_INVALID_ARG;
    if (!config_ok(cfg)) return LC_ERR_INVALID_ARG;
    if (reinterpret_cast<uintptr_t>(index_buf) & 255u) return LC_ERR_INVALID_ARG;
    if (blob_bytes < 64) return LC_ERR_BAD_BLOB;
    const char* p = static_cast<const char*>(blob);
    const char* end = p + blob_bytes;
    int32_t hdr[16];
    memcpy(hdr, p, sizeof(hdr));
    p += sizeof(hdr);
    if (hdr[0] != kMagic || hdr[1] != 1) return LC_ERR_BAD_BLOB;
    const int B = hdr[2], H = hdr[3], d = hdr[4], L = hdr[5], F = hdr[6], geo = hdr[7];
    if (B < 1 || H < 1) return LC_ERR_BAD_BLOB;
    if (d != LC_HEAD_DIM) return LC_ERR_BAD_SHAPE;
    if (L != cfg->levels || F != cfg->fanout || geo != cfg->geometry) return LC_ERR_BAD_BLOB;
    for (int l = 1; l < L; ++l)
        if ((hdr[8 + l] > 0 ? hdr[8 + l] : F) != level_fanout(cfg, l)) return LC_ERR_BAD_BLOB;
    if (hdr[8] != cfg->center_dtype) return LC_ERR_BAD_BLOB;     // radii are only valid for the centers they were measured against
    if (index_bytes < lc_layout_index(cfg, B, H, d, nullptr, nullptr)) return LC_ERR_WORKSPACE_TOO_SMALL;

    lc_index* h = new_handle(cfg, B, H, d, index_buf, index_bytes);
    if (!h) return LC_ERR_INVALID_ARG;
    std::vector<int32_t> bounds_concat;
    int rc = LC_OK;
    for (int b = 0; b < B && rc == LC_OK; ++b) {
        const size_t rec_bytes = (size_t)(2 + (L - 1)) * 4;
        if (p + rec_bytes > end) { rc = LC_ERR_BAD_BLOB; break; }
        int32_t rec[2 + LC_MAX_LEVELS];
        memcpy(rec, p, rec_bytes);
        p += rec_bytes;
        const int T = rec[0], M = rec[1];
        if (M < 0 || T < 0) { rc = LC_ERR_BAD_BLOB; break; }
        if (M > cfg->max_chunks || T > cfg->max_tokens) { rc = LC_ERR_CAPACITY; break; }
        h->T[b] = T;
        h->M[b] = M;
        h->N[(size_t)b * LC_MAX_LEVELS] = M;
        for (int l = 1; l < L; ++l) {
            const int n = rec[1 + l];
            if (n < 1 || n > h->dev.cap[l]) { rc = LC_ERR_BAD_BLOB; break; }
            h->N[(size_t)b * LC_MAX_LEVELS + l] = n;
        }
        if (rc != LC_OK) break;
        const size_t nb = ((size_t)M + 1) * 4;
        if (p + nb > end) { rc = LC_ERR_BAD_BLOB; break; }
        const size_t at = bounds_concat.size();
        bounds_concat.resize(at + M + 1);
        memcpy(bounds_concat.data() + at, p, nb);
        p += nb;
        const int32_t* bd = bounds_concat.data() + at;
        if (bd[0] != 0 || bd[M] > T) { rc = LC_ERR_BAD_BLOB; break; }
        for (int j = 0; j < M; ++j)
            if (bd[j + 1] <= bd[j]) { rc = LC_ERR_BAD_BLOB; break; }
    }
    if (rc == LC_OK) {
        // validate the node records before touching the GPU
        const char* r = p;
        for (int b = 0; b < B && rc == LC_OK; ++b)
            for (int hh = 0; hh < H && rc == LC_OK; ++hh)
                for (int l = 0; l < L; ++l) {
                    const size_t nl = h->N[(size_t)b * LC_MAX_LEVELS + l];
                    const size_t sz = nl * ((size_t)d * 4 + 16);
                    if (r + sz > end) { rc = LC_ERR_BAD_BLOB; break; }
                    const int32_t* par = reinterpret_cast<const int32_t*>(r + nl * (size_t)d * 4 + nl * 4);
                    if (l + 1 < L) {
                        const int up = h->N[(size_t)b * LC_MAX_LEVELS + l + 1];
                        for (size_t n = 0; n < nl; ++n) {
                            int32_t pv;
                            memcpy(&pv, par + n, 4);
                            if (pv < 0 || pv >= up) { rc = LC_ERR_BAD_BLOB; break; }
                        }
                    }
                    r += sz;
                }
    }
    hipStream_t s = static_cast<hipStream_t>(stream);
    // staged through the chunk centers' memory, which the copies below overwrite once the stream has drained
    if (rc == LC_OK) rc = upload_state(h, bounds_concat.data(), h->dev.center[0], s);
    if (rc == LC_OK && hipStreamSynchronize(s) != hipSuccess) rc = LC_ERR_HIP;
    if (rc == LC_OK) {
        const LcDev& D = h->dev;
        for (int b = 0; b < B && rc == LC_OK; ++b)
            for (int hh = 0; hh < H && rc == LC_OK; ++hh)
                for (int l = 0; l < L && rc == LC_OK; ++l) {
                    const size_t nl = h->N[(size_t)b * LC_MAX_LEVELS + l];
                    if (nl == 0) continue;
                    const size_t base = ((size_t)b * H + hh) * D.cap[l];
                    hipError_t e;
                    if (l == 0 && D.c0_bf16) {
                        // values of a bfloat16 index are bfloat16-representable; anything else is rounded to nearest even
                        std::vector<uint16_t> half(nl * d);
                        for (size_t i = 0; i < half.size(); ++i) {
                            uint32_t w;
                            memcpy(&w, p + 4 * i, 4);
                            half[i] = (uint16_t)((w + 0x7fffu + ((w >> 16) & 1u)) >> 16);
                        }
                        e = hipMemcpy(reinterpret_cast<uint16_t*>(D.center[0]) + base * d, half.data(), nl * d * 2,
                                      hipMemcpyHostToDevice);
                    } else {
                        e = hipMemcpy(D.center[l] + base * d, p, nl * d * 4, hipMemcpyHostToDevice);
                    }
                    p += nl * d * 4;
                    if (e == hipSuccess) e = hipMemcpy(D.radius[l] + base, p, nl * 4, hipMemcpyHostToDevice);
                    if (e == hipSuccess && l >= 1) e = hipMemcpy(D.rbuild[l] + base, p, nl * 4, hipMemcpyHostToDevice);
                    p += nl * 4;
                    if (e == hipSuccess) e = hipMemcpy(D.parent[l] + base, p, nl * 4, hipMemcpyHostToDevice);
                    p += nl * 4;
                    if (e == hipSuccess) e = hipMemcpy(D.ntok[l] + base, p, nl * 4, hipMemcpyHostToDevice);
                    p += nl * 4;
                    if (e == hipSuccess) e = hipMemcpy(D.nchunk[l] + base, p, nl * 4, hipMemcpyHostToDevice);
                    p += nl * 4;
                    if (e != hipSuccess) { lc_set_hip_error(e); rc = LC_ERR_HIP; }
                }
    }
    if (rc != LC_OK) {
        delete h;
        return rc;
    }
    *out = h;
    return LC_OK;
}

void lc_index_destroy(lc_index* idx) { delete idx; }

}  // extern "C"
