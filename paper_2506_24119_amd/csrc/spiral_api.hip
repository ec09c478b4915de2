// Host side of the C ABI: argument checking, the paged-KV bookkeeping, workspace carving and the
// fixed kernel sequence of a prefill / decode step.  No device memory is allocated here.
#include <algorithm>
#include <cmath>
#include <cstdarg>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <new>
#include <string>
#include <vector>

#include "spiral_internal.h"

using namespace spiral;

// ---------------------------------------------------------------------------------------------
// errors
// ---------------------------------------------------------------------------------------------
static thread_local char g_err[512] = "";

static int fail(int code, const char* fmt, ...) {
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof(g_err), fmt, ap);
    va_end(ap);
    return code;
}

#define HIP_TRY(expr)                                                                        \
    do {                                                                                     \
        hipError_t e_ = (expr);                                                              \
        if (e_ != hipSuccess) return fail(SPIRAL_ERR_HIP, "%s: %s", #expr, hipGetErrorString(e_)); \
    } while (0)

extern "C" const char* spiral_last_error(void) { return g_err; }
int spiral_set_error(int code, const char* text) { return fail(code, "%s", text); }
extern "C" const char* spiral_version(void) {
    return "spiral-mi355x 0.1 (gfx950; bf16 weights, f16 activations/KV cache, f16 MFMA, f32 accumulate)";
}

// ---------------------------------------------------------------------------------------------
// objects
// ---------------------------------------------------------------------------------------------
struct Tune {
    // weight rows per workgroup and K splits of the narrow projections; 0 = chosen from the shape
    int bn_qkv = 0, s_qkv = 0;
    int bn_o = 0, s_o = 0;
    int bn_gu = 0;                 // 0: waves per workgroup chosen from the shape
    int bn_down = 0, s_down = 0;
    int bn_lm = 128;
    int chunk_pages = 16;          // decode attention: least (row, kv head, page) units per workgroup
    int attn_wgs = 0;              // workgroups of the decode attention; 0 = 3 per compute unit (its occupancy)
    int frag = 1;                  // 0: ignore spiral_model_repack (weights stay row-major; for A/B measurements)
    int fuse_qkv = 1;              // 0: large-M q/k/v projection and its post-processing as two kernels (for A/B measurements)
    int fail_after = 0;            // test hook: the n-th timed launch from now reports a launch failure instead of running
};
constexpr int kMaxSplit = 16;
constexpr int kScoreSplits = 64;       // vocabulary ranges of the scoring pass (partial log-sum-exp pairs per row)

struct Profiler {
    bool active = false;
    int kclass = -1, used = 0;
    std::vector<hipEvent_t> ev;       // start/stop pairs
};

struct spiral_model {
    Profiler prof;
    spiral_model_config cfg;
    std::vector<const void*> w;
    bool w_bf16;
    RopeFreq freq;
    Tune tune;
    int n_cus = 256;
    // fragment-ordered copies of the projection matrices (spiral_model_repack), null until then
    std::vector<const void*> f_qkv, f_o, f_gu, f_down;
    const void* f_lm = nullptr;
    const void* lw(int layer, int slot) const { return w[3 + layer * SPIRAL_LAYER_SLOTS + slot]; }
};

struct spiral_kv_pool {
    const spiral_model* m;
    int32_t* d_block_table;
    int32_t* d_status;                        // [0]: count of activations that left the 16-bit range
    uint16_t* d_pages;
    int n_pages, max_seqs, max_blocks;
    size_t layer_elems;                       // elements between consecutive layers' page arrays
    std::vector<int32_t> free_list;           // back = next page handed out
    std::vector<int32_t> h_lens;
    std::vector<std::vector<int32_t>> h_pages;
};

static size_t align256(size_t x) { return (x + 255) & ~(size_t)255; }

static void parse_tune(Tune& t, const char* e) {
    std::string s(e);
    size_t i = 0;
    while (i < s.size()) {
        size_t j = s.find(',', i);
        if (j == std::string::npos) j = s.size();
        std::string kv = s.substr(i, j - i);
        size_t eq = kv.find('=');
        if (eq != std::string::npos) {
            std::string k = kv.substr(0, eq);
            int a = 0, b = 0;
            int n = sscanf(kv.c_str() + eq + 1, "%d:%d", &a, &b);
            if (n >= 1) {
                if (k == "qkv") { t.bn_qkv = a; if (n == 2) t.s_qkv = b; }
                else if (k == "o") { t.bn_o = a; if (n == 2) t.s_o = b; }
                else if (k == "gu") { t.bn_gu = a; }
                else if (k == "down") { t.bn_down = a; if (n == 2) t.s_down = b; }
                else if (k == "lm") { t.bn_lm = a; }
                else if (k == "chunk") { t.chunk_pages = a; }
                else if (k == "wgs") { t.attn_wgs = a; }
                else if (k == "frag") { t.frag = a; }
                else if (k == "fuse_qkv") { t.fuse_qkv = a; }
                else if (k == "fail_after") { t.fail_after = a; }
            }
        }
        i = j + 1;
    }
    auto clampi = [](int& v, int lo, int hi) { v = v < lo ? lo : (v > hi ? hi : v); };
    clampi(t.s_qkv, 0, kMaxSplit); clampi(t.s_o, 0, kMaxSplit); clampi(t.s_down, 0, kMaxSplit);
    clampi(t.chunk_pages, 1, 1 << 20);
}

extern "C" int spiral_model_tune(spiral_model* m, const char* spec) {
    if (!m) return fail(SPIRAL_ERR_NOT_LOADED, "model_tune: null model");
    if (!spec) return fail(SPIRAL_ERR_INVALID_ARG, "model_tune: null spec");
    Tune t = m->tune;
    parse_tune(t, spec);
    if (t.frag != m->tune.frag && m->f_lm) return fail(SPIRAL_ERR_INVALID_ARG, "model_tune: frag must be set before spiral_model_repack");
    m->tune = t;
    return SPIRAL_OK;
}

extern "C" int spiral_model_load(const spiral_model_config* cfg, const void* const* host_dev_weights,
                                 int n_weights, spiral_model** out) {
    if (!cfg || !host_dev_weights || !out) return fail(SPIRAL_ERR_INVALID_ARG, "model_load: null argument");
    *out = nullptr;
    const spiral_model_config& c = *cfg;
    if (c.n_layers < 1 || c.d_model < 1 || c.n_q_heads < 1 || c.n_kv_heads < 1 || c.ffn_dim < 1 || c.vocab < 1)
        return fail(SPIRAL_ERR_SHAPE, "model_load: non-positive dimension");
    if (c.head_dim != 32 && c.head_dim != 64 && c.head_dim != 128)
        return fail(SPIRAL_ERR_SHAPE, "model_load: head_dim %d not in {32,64,128}", c.head_dim);
    if (c.n_q_heads % c.n_kv_heads != 0 || c.n_q_heads / c.n_kv_heads > kMaxGroup)
        return fail(SPIRAL_ERR_SHAPE, "model_load: %d query heads per kv head unsupported", c.n_q_heads / std::max(1, c.n_kv_heads));
    if (c.kv_block_tokens != kPageTokens) return fail(SPIRAL_ERR_SHAPE, "model_load: kv_block_tokens must be 16");
    if (c.weight_dtype != SPIRAL_WEIGHT_FP32 && c.weight_dtype != SPIRAL_WEIGHT_BF16)
        return fail(SPIRAL_ERR_SHAPE, "model_load: unknown weight_dtype %d", c.weight_dtype);
    if (!(c.rope_theta > 0.f) || !(c.rms_eps >= 0.f)) return fail(SPIRAL_ERR_INVALID_ARG, "model_load: bad rope_theta / rms_eps");
    if (c.weight_dtype == SPIRAL_WEIGHT_BF16) {
        const int qw = c.n_q_heads * c.head_dim;
        if (c.d_model % 32 || qw % 32 || c.ffn_dim % 32)
            return fail(SPIRAL_ERR_SHAPE, "model_load: d_model, Hq*hd and ffn_dim must be multiples of 32 for bf16 weights");
        if (c.vocab % 4) return fail(SPIRAL_ERR_SHAPE, "model_load: vocab must be a multiple of 4 for bf16 weights");
    }
    if (n_weights != 3 + SPIRAL_LAYER_SLOTS * c.n_layers)
        return fail(SPIRAL_ERR_INVALID_ARG, "model_load: expected %d weight pointers, got %d", 3 + SPIRAL_LAYER_SLOTS * c.n_layers, n_weights);
    auto need = [&](int idx, bool required) -> bool {
        const void* p = host_dev_weights[idx];
        if (!p) return !required;
        return ((uintptr_t)p & 15) == 0;
    };
    for (int i = 0; i < 3; ++i)
        if (!need(i, true)) return fail(SPIRAL_ERR_INVALID_ARG, "model_load: weight %d null or not 16-byte aligned", i);
    for (int l = 0; l < c.n_layers; ++l)
        for (int s = 0; s < SPIRAL_LAYER_SLOTS; ++s) {
            bool req = true;
            if (s == SPIRAL_W_BQ || s == SPIRAL_W_BK || s == SPIRAL_W_BV) req = c.qkv_bias != 0;
            if (s == SPIRAL_W_Q_NORM || s == SPIRAL_W_K_NORM) req = c.qk_norm != 0;
            if (!need(3 + l * SPIRAL_LAYER_SLOTS + s, req))
                return fail(SPIRAL_ERR_INVALID_ARG, "model_load: layer %d slot %d null or not 16-byte aligned", l, s);
        }
    spiral_model* m = new (std::nothrow) spiral_model();
    if (!m) return fail(SPIRAL_ERR_INVALID_ARG, "model_load: out of host memory");
    m->cfg = c;
    m->w.assign(host_dev_weights, host_dev_weights + n_weights);
    m->w_bf16 = c.weight_dtype == SPIRAL_WEIGHT_BF16;
    for (int j = 0; j < 64; ++j)
        m->freq.inv_freq[j] = j < c.head_dim / 2 ? std::pow((double)c.rope_theta, -2.0 * j / c.head_dim) : 0.0;
    {
        // compute units of the current device (the stream attention kernel launches 3 workgroups on each);
        // without a device the default stays, model_load itself touches no GPU state
        int dev = 0, cus = 0;
        if (hipGetDevice(&dev) == hipSuccess &&
            hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) == hipSuccess && cus > 0)
            m->n_cus = cus;
        else
            (void)hipGetLastError();
    }
    *out = m;
    return SPIRAL_OK;
}

static void drop_events(Profiler& p) {
    for (hipEvent_t e : p.ev) (void)hipEventDestroy(e);
    p.ev.clear();
    p.active = false;
    p.used = 0;
}

extern "C" void spiral_model_free(spiral_model* m) {
    if (m) drop_events(m->prof);
    delete m;
}

// ---------------------------------------------------------------------------------------------
// weight repack into fragment order
// ---------------------------------------------------------------------------------------------
struct RepackPlan { size_t qkv, o, gu, down, lm, per_layer, total; bool ok; };

static RepackPlan repack_plan(const spiral_model* m) {
    const spiral_model_config& c = m->cfg;
    const size_t d = c.d_model, qw = (size_t)c.n_q_heads * c.head_dim, kw = (size_t)c.n_kv_heads * c.head_dim, F = c.ffn_dim;
    auto pad32 = [](size_t n) { return (n + 31) / 32 * 32; };
    RepackPlan r;
    r.ok = m->w_bf16 && d % 16 == 0 && qw % 16 == 0 && F % 16 == 0 && qw % 32 == 0 && kw % 32 == 0;
    r.qkv = align256(pad32(qw + 2 * kw) * d * 2);
    r.o = align256(pad32(d) * qw * 2);
    r.gu = align256(2 * F * d * 2);
    r.down = align256(pad32(d) * F * 2);
    r.lm = align256(pad32(c.vocab) * d * 2);
    r.per_layer = r.qkv + r.o + r.gu + r.down;
    r.total = r.per_layer * c.n_layers + r.lm;
    return r;
}

extern "C" size_t spiral_model_repack_bytes(const spiral_model* m) {
    if (!m) return 0;
    const RepackPlan r = repack_plan(m);
    return r.ok ? r.total : 0;
}

extern "C" int spiral_model_repack(spiral_model* m, void* dev_buffer, size_t bytes, void* stream) {
    if (!m) return fail(SPIRAL_ERR_NOT_LOADED, "model_repack: null model");
    const RepackPlan r = repack_plan(m);
    if (!r.ok) return fail(SPIRAL_ERR_SHAPE, "model_repack: needs 16-bit weights and d_model, Hq*hd, Hkv*hd, ffn_dim multiples of 32 / 16");
    if (!dev_buffer || ((uintptr_t)dev_buffer & 255) || bytes < r.total)
        return fail(SPIRAL_ERR_INVALID_ARG, "model_repack: buffer null, not 256-byte aligned or smaller than %zu bytes", r.total);
    if (!m->tune.frag) return SPIRAL_OK;
    const spiral_model_config& c = m->cfg;
    const int d = c.d_model, qw = c.n_q_heads * c.head_dim, kw = c.n_kv_heads * c.head_dim, F = c.ffn_dim;
    hipStream_t s = (hipStream_t)stream;
    char* base = (char*)dev_buffer;
    std::vector<const void*> fq(c.n_layers), fo(c.n_layers), fg(c.n_layers), fd(c.n_layers);
    for (int l = 0; l < c.n_layers; ++l) {
        char* p = base + (size_t)l * r.per_layer;
        fq[l] = p; fo[l] = p + r.qkv; fg[l] = p + r.qkv + r.o; fd[l] = p + r.qkv + r.o + r.gu;
        HIP_TRY(launch_repack(m->lw(l, SPIRAL_W_Q), m->lw(l, SPIRAL_W_K), m->lw(l, SPIRAL_W_V), qw, kw, kw, d, false, (void*)fq[l], s));
        HIP_TRY(launch_repack(m->lw(l, SPIRAL_W_O), nullptr, nullptr, d, 0, 0, qw, false, (void*)fo[l], s));
        HIP_TRY(launch_repack(m->lw(l, SPIRAL_W_GATE), m->lw(l, SPIRAL_W_UP), nullptr, F, F, 0, d, true, (void*)fg[l], s));
        HIP_TRY(launch_repack(m->lw(l, SPIRAL_W_DOWN), nullptr, nullptr, d, 0, 0, F, false, (void*)fd[l], s));
    }
    char* lm = base + (size_t)c.n_layers * r.per_layer;
    HIP_TRY(launch_repack(m->w[2], nullptr, nullptr, c.vocab, 0, 0, d, false, lm, s));
    m->f_qkv = fq; m->f_o = fo; m->f_gu = fg; m->f_down = fd; m->f_lm = lm;
    return SPIRAL_OK;
}

extern "C" int spiral_profile_begin(spiral_model* m, int kernel_class, int max_launches) {
    if (!m) return fail(SPIRAL_ERR_NOT_LOADED, "profile_begin: null model");
    if (kernel_class < 0 || kernel_class >= SPIRAL_K_CLASSES || max_launches < 1 || max_launches > (1 << 20))
        return fail(SPIRAL_ERR_INVALID_ARG, "profile_begin: bad kernel class or launch count");
    if (m->prof.active) return fail(SPIRAL_ERR_INVALID_ARG, "profile_begin: already active");
    m->prof.ev.reserve((size_t)2 * max_launches);
    for (int i = 0; i < 2 * max_launches; ++i) {
        hipEvent_t e;
        hipError_t rc = hipEventCreate(&e);
        if (rc != hipSuccess) { drop_events(m->prof); return fail(SPIRAL_ERR_HIP, "profile_begin: %s", hipGetErrorString(rc)); }
        m->prof.ev.push_back(e);
    }
    m->prof.kclass = kernel_class;
    m->prof.used = 0;
    m->prof.active = true;
    return SPIRAL_OK;
}

extern "C" int spiral_profile_end(spiral_model* m, double* host_total_ms, int* host_n_launches) {
    if (!m) return fail(SPIRAL_ERR_NOT_LOADED, "profile_end: null model");
    if (!m->prof.active) return fail(SPIRAL_ERR_INVALID_ARG, "profile_end: not active");
    if (!host_total_ms || !host_n_launches) return fail(SPIRAL_ERR_INVALID_ARG, "profile_end: null output");
    double total = 0.0;
    const int n = m->prof.used;
    if (n > 0) {
        hipError_t rc = hipEventSynchronize(m->prof.ev[2 * n - 1]);
        if (rc != hipSuccess) { drop_events(m->prof); return fail(SPIRAL_ERR_HIP, "profile_end: %s", hipGetErrorString(rc)); }
        for (int i = 0; i < n; ++i) {
            float ms = 0.f;
            rc = hipEventElapsedTime(&ms, m->prof.ev[2 * i], m->prof.ev[2 * i + 1]);
            if (rc != hipSuccess) { drop_events(m->prof); return fail(SPIRAL_ERR_HIP, "profile_end: %s", hipGetErrorString(rc)); }
            total += ms;
        }
    }
    *host_total_ms = total;
    *host_n_launches = n;
    drop_events(m->prof);
    return SPIRAL_OK;
}

extern "C" int spiral_probe_stream_read(const void* dev_buf, size_t bytes, int iters, double* host_ms_per_pass, void* stream) {
    if (!dev_buf || ((uintptr_t)dev_buf & 15) || bytes < (1u << 20) || iters < 1 || iters > 10000 || !host_ms_per_pass)
        return fail(SPIRAL_ERR_INVALID_ARG, "probe_stream_read: needs a 16-byte aligned buffer of at least 1 MiB, 1 <= iters <= 10000 and an output");
    hipStream_t s = (hipStream_t)stream;
    int dev = 0, cus = 256;
    if (hipGetDevice(&dev) == hipSuccess) (void)hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev);
    hipEvent_t e0, e1;
    HIP_TRY(hipEventCreate(&e0));
    hipError_t rc = hipEventCreate(&e1);
    if (rc != hipSuccess) { (void)hipEventDestroy(e0); return fail(SPIRAL_ERR_HIP, "probe_stream_read: %s", hipGetErrorString(rc)); }
    auto done = [&](hipError_t e) { (void)hipEventDestroy(e0); (void)hipEventDestroy(e1); return e; };
    rc = launch_stream_read(dev_buf, bytes, 3 * cus, s);                       // untimed first pass
    if (rc == hipSuccess) rc = hipEventRecord(e0, s);
    for (int i = 0; i < iters && rc == hipSuccess; ++i) rc = launch_stream_read(dev_buf, bytes, 3 * cus, s);
    if (rc == hipSuccess) rc = hipEventRecord(e1, s);
    if (rc == hipSuccess) rc = hipEventSynchronize(e1);
    float ms = 0.f;
    if (rc == hipSuccess) rc = hipEventElapsedTime(&ms, e0, e1);
    if (done(rc) != hipSuccess) return fail(SPIRAL_ERR_HIP, "probe_stream_read: %s", hipGetErrorString(rc));
    *host_ms_per_pass = (double)ms / iters;
    return SPIRAL_OK;
}

// Runs one launch, bracketed by events when its class is being profiled.
template <typename F>
static hipError_t timed(spiral_model* m, int kclass, hipStream_t s, F&& launch) {
    if (m->tune.fail_after > 0 && --m->tune.fail_after == 0) return hipErrorLaunchFailure;     // host-forced, nothing is launched
    Profiler& p = m->prof;
    const bool on = p.active && p.kclass == kclass && 2 * (p.used + 1) <= (int)p.ev.size();
    if (on) { hipError_t e = hipEventRecord(p.ev[2 * p.used], s); if (e != hipSuccess) return e; }
    hipError_t rc = launch();
    if (rc != hipSuccess) return rc;
    if (on) { hipError_t e = hipEventRecord(p.ev[2 * p.used + 1], s); if (e != hipSuccess) return e; ++p.used; }
    return hipSuccess;
}

// ---------------------------------------------------------------------------------------------
// workspace
// ---------------------------------------------------------------------------------------------
struct Workspace {
    float* x; void* h; float* qkv; uint16_t* q; void* o; float* proj; void* mlp; void* hf;
    float* attn_part; float2* rope;
    int32_t *row_seq, *row_pos, *seq_ids, *cu_rows, *base_pos, *last_rows, *page_start;
    int2* row_page;                           // (page, position) that takes each row's k and v
    float *score_part, *score_tgt;
    uint64_t* s_keys; float2* s_part;         // fused sampler: row keys, per-tile winners
    size_t bytes;
};

static int decode_chunks(const spiral_model* m, int max_context) {
    const int pages = (max_context + kPageTokens - 1) / kPageTokens;
    return std::max(1, (pages + m->tune.chunk_pages - 1) / m->tune.chunk_pages);
}
// partial-result slots per (row, kv head): the stream kernel gives a workgroup at least chunk_pages
// units, so a pair of n pages is cut into at most n / chunk_pages + 2 pieces
static int decode_slots(const spiral_model* m, int max_context) { return decode_chunks(m, max_context) + 2; }

static Workspace carve(const spiral_model* m, char* base, int rows, int max_context) {
    const spiral_model_config& c = m->cfg;
    const size_t act = m->w_bf16 ? 2 : 4;
    const size_t R = (size_t)rows;
    const size_t brows = (size_t)std::min(rows, SPIRAL_MAX_BATCH);
    const size_t nqkv = (size_t)(c.n_q_heads + 2 * c.n_kv_heads) * c.head_dim;
    const size_t qw = (size_t)c.n_q_heads * c.head_dim;
    const int G = c.n_q_heads / c.n_kv_heads;
    // projection outputs: up to kMaxSplit K-split partials while rows <= 128, one copy beyond that;
    // sized so that a workspace for R rows also serves any smaller row count
    const size_t split_rows = std::max(R, std::min<size_t>(R, 128) * kMaxSplit);
    size_t off = 0;
    auto take = [&](size_t bytes) { char* p = base ? base + off : nullptr; off += align256(bytes); return p; };
    Workspace w;
    // the per-call id arrays come first so that their addresses do not depend on rows / context
    w.seq_ids = (int32_t*)take(SPIRAL_MAX_BATCH * 4);
    w.cu_rows = (int32_t*)take((SPIRAL_MAX_BATCH + 1) * 4);
    w.base_pos = (int32_t*)take(SPIRAL_MAX_BATCH * 4);
    w.last_rows = (int32_t*)take(SPIRAL_MAX_BATCH * 4);
    w.page_start = (int32_t*)take((SPIRAL_MAX_BATCH + 1) * 4);
    w.x = (float*)take(R * c.d_model * 4);
    w.h = take(R * c.d_model * act);
    w.qkv = (float*)take(split_rows * nqkv * 4);
    w.q = (uint16_t*)take(R * qw * 2);
    w.o = take(R * qw * act);
    w.proj = (float*)take(split_rows * c.d_model * 4);
    w.mlp = take(R * c.ffn_dim * act);
    w.hf = take(brows * c.d_model * act);
    w.rope = (float2*)take(R * (c.head_dim / 2) * 8);
    w.row_seq = (int32_t*)take(R * 4);
    w.row_pos = (int32_t*)take(R * 4);
    w.row_page = (int2*)take(R * 8);
    w.attn_part = (float*)take(brows * c.n_kv_heads * decode_slots(m, max_context) * G * (c.head_dim + 2) * 4);
    w.score_part = (float*)take(R * kScoreSplits * 8);
    w.score_tgt = (float*)take(R * 4);
    w.s_keys = (uint64_t*)take(SPIRAL_MAX_BATCH * 8);
    w.s_part = (float2*)take(brows * (size_t)((c.vocab + 63) / 64) * 8);
    w.bytes = off;
    return w;
}

extern "C" size_t spiral_workspace_bytes(const spiral_model* m, int max_rows, int max_context) {
    if (!m || max_rows < 1 || max_context < 1) return 0;
    return carve(m, nullptr, max_rows, max_context).bytes;
}

// ---------------------------------------------------------------------------------------------
// KV pool
// ---------------------------------------------------------------------------------------------
static size_t pool_header_bytes(int max_seqs, int max_blocks) {
    return align256((size_t)max_seqs * max_blocks * 4) + 256;          // block table, status block
}
static size_t page_layer_elems(const spiral_model* m) {      // elements of one page in one layer
    return (size_t)m->cfg.n_kv_heads * 2 * kPageTokens * m->cfg.head_dim;
}

extern "C" size_t spiral_kv_pool_bytes(const spiral_model* m, int n_pages, int max_seqs, int max_blocks_per_seq) {
    if (!m || n_pages < 1 || max_seqs < 1 || max_blocks_per_seq < 1) return 0;
    return pool_header_bytes(max_seqs, max_blocks_per_seq) +
           (size_t)m->cfg.n_layers * n_pages * page_layer_elems(m) * 2;
}

extern "C" int spiral_kv_pool_create(const spiral_model* m, void* dev_mem, size_t bytes, int n_pages, int max_seqs,
                                     int max_blocks_per_seq, const int32_t* host_page_order, void* stream,
                                     spiral_kv_pool** out) {
    if (!out) return fail(SPIRAL_ERR_INVALID_ARG, "kv_pool_create: null out");
    *out = nullptr;
    if (!m) return fail(SPIRAL_ERR_NOT_LOADED, "kv_pool_create: null model");
    if (!dev_mem || ((uintptr_t)dev_mem & 255)) return fail(SPIRAL_ERR_INVALID_ARG, "kv_pool_create: dev_mem null or not 256-byte aligned");
    const size_t need = spiral_kv_pool_bytes(m, n_pages, max_seqs, max_blocks_per_seq);
    if (need == 0) return fail(SPIRAL_ERR_INVALID_ARG, "kv_pool_create: non-positive size argument");
    if (bytes < need) return fail(SPIRAL_ERR_OOM_KV, "kv_pool_create: %zu bytes given, %zu needed", bytes, need);
    std::vector<int32_t> order(n_pages);
    if (host_page_order) {
        std::vector<char> seen(n_pages, 0);
        for (int i = 0; i < n_pages; ++i) {
            const int p = host_page_order[i];
            if (p < 0 || p >= n_pages || seen[p]) return fail(SPIRAL_ERR_INVALID_ARG, "kv_pool_create: page order is not a permutation");
            seen[p] = 1;
            order[i] = p;
        }
    } else {
        for (int i = 0; i < n_pages; ++i) order[i] = i;
    }
    spiral_kv_pool* p = new (std::nothrow) spiral_kv_pool();
    if (!p) return fail(SPIRAL_ERR_INVALID_ARG, "kv_pool_create: out of host memory");
    p->m = m;
    char* base = (char*)dev_mem;
    p->d_block_table = (int32_t*)base;
    p->d_status = (int32_t*)(base + align256((size_t)max_seqs * max_blocks_per_seq * 4));
    p->d_pages = (uint16_t*)(base + pool_header_bytes(max_seqs, max_blocks_per_seq));
    p->n_pages = n_pages; p->max_seqs = max_seqs; p->max_blocks = max_blocks_per_seq;
    p->layer_elems = (size_t)n_pages * page_layer_elems(m);
    p->free_list.assign(order.rbegin(), order.rend());     // order[0] is handed out first
    p->h_lens.assign(max_seqs, 0);
    p->h_pages.assign(max_seqs, std::vector<int32_t>());
    hipError_t e = launch_fill_zero(dev_mem, need, (hipStream_t)stream);
    if (e != hipSuccess) { delete p; return fail(SPIRAL_ERR_HIP, "kv_pool_create: fill: %s", hipGetErrorString(e)); }
    *out = p;
    return SPIRAL_OK;
}

extern "C" void spiral_kv_pool_free(spiral_kv_pool* p) { delete p; }

extern "C" long long spiral_kv_pool_status_offset(const spiral_kv_pool* p) {
    if (!p) return fail(SPIRAL_ERR_NOT_LOADED, "kv_pool_status_offset: null pool");
    return (long long)((const char*)p->d_status - (const char*)p->d_block_table);
}

static int check_ids(const spiral_kv_pool* p, const int32_t* ids, int n, const char* who) {
    if (!ids) return fail(SPIRAL_ERR_INVALID_ARG, "%s: null sequence ids", who);
    if (n < 1 || n > SPIRAL_MAX_BATCH) return fail(SPIRAL_ERR_INVALID_ARG, "%s: batch %d outside [1, %d]", who, n, SPIRAL_MAX_BATCH);
    std::vector<char> seen(p->max_seqs, 0);
    for (int i = 0; i < n; ++i) {
        if (ids[i] < 0 || ids[i] >= p->max_seqs) return fail(SPIRAL_ERR_INVALID_ARG, "%s: sequence id %d out of range", who, ids[i]);
        if (seen[ids[i]]) return fail(SPIRAL_ERR_INVALID_ARG, "%s: sequence id %d listed twice", who, ids[i]);
        seen[ids[i]] = 1;
    }
    return SPIRAL_OK;
}

extern "C" int spiral_seq_reset(spiral_kv_pool* p, const int32_t* host_seq_ids, int n, void* stream) {
    if (!p) return fail(SPIRAL_ERR_NOT_LOADED, "seq_reset: null pool");
    if (n == 0) return SPIRAL_OK;
    int rc = check_ids(p, host_seq_ids, n, "seq_reset");
    if (rc) return rc;
    (void)stream;                              // lengths live on the host: nothing to enqueue
    for (int i = 0; i < n; ++i) {
        std::vector<int32_t>& pg = p->h_pages[host_seq_ids[i]];
        for (size_t k = pg.size(); k-- > 0;) p->free_list.push_back(pg[k]);
        pg.clear();
        p->h_lens[host_seq_ids[i]] = 0;
    }
    return SPIRAL_OK;
}

extern "C" int spiral_seq_truncate(spiral_kv_pool* p, const int32_t* host_seq_ids, const int32_t* host_new_lens,
                                   int n, void* stream) {
    if (!p) return fail(SPIRAL_ERR_NOT_LOADED, "seq_truncate: null pool");
    if (n == 0) return SPIRAL_OK;
    int rc = check_ids(p, host_seq_ids, n, "seq_truncate");
    if (rc) return rc;
    if (!host_new_lens) return fail(SPIRAL_ERR_INVALID_ARG, "seq_truncate: null lengths");
    for (int i = 0; i < n; ++i)
        if (host_new_lens[i] < 0 || host_new_lens[i] > p->h_lens[host_seq_ids[i]])
            return fail(SPIRAL_ERR_INVALID_ARG, "seq_truncate: length %d outside [0, %d] for sequence %d",
                        host_new_lens[i], p->h_lens[host_seq_ids[i]], host_seq_ids[i]);
    (void)stream;
    for (int i = 0; i < n; ++i) {
        std::vector<int32_t>& pg = p->h_pages[host_seq_ids[i]];
        const size_t keep = (size_t)(host_new_lens[i] + kPageTokens - 1) / kPageTokens;
        while (pg.size() > keep) { p->free_list.push_back(pg.back()); pg.pop_back(); }
        p->h_lens[host_seq_ids[i]] = host_new_lens[i];
    }
    return SPIRAL_OK;
}

extern "C" int spiral_seq_len(const spiral_kv_pool* p, int seq_id) {
    if (!p) return fail(SPIRAL_ERR_NOT_LOADED, "seq_len: null pool");
    if (seq_id < 0 || seq_id >= p->max_seqs) return fail(SPIRAL_ERR_INVALID_ARG, "seq_len: id %d out of range", seq_id);
    return p->h_lens[seq_id];
}

extern "C" int spiral_kv_free_pages(const spiral_kv_pool* p) {
    if (!p) return fail(SPIRAL_ERR_NOT_LOADED, "kv_free_pages: null pool");
    return (int)p->free_list.size();
}

// Checks that every listed sequence can grow by add[i] tokens, then takes the pages and enqueues the
// block-table updates.  Nothing is modified when the check fails.  `before` receives the page counts the
// sequences had, for ungrow().
static int grow(spiral_kv_pool* p, const int32_t* ids, const int32_t* add, int n, hipStream_t s, const char* who,
                std::vector<size_t>& before) {
    size_t need_pages = 0;
    for (int i = 0; i < n; ++i) {
        const long long new_len = (long long)p->h_lens[ids[i]] + add[i];
        const long long blocks = (new_len + kPageTokens - 1) / kPageTokens;
        if (blocks > p->max_blocks)
            return fail(SPIRAL_ERR_OOM_KV, "%s: sequence %d would need %lld pages, block table holds %d", who, ids[i], blocks, p->max_blocks);
        need_pages += (size_t)blocks - p->h_pages[ids[i]].size();
    }
    if (need_pages > p->free_list.size())
        return fail(SPIRAL_ERR_OOM_KV, "%s: %zu pages needed, %zu free", who, need_pages, p->free_list.size());
    std::vector<int32_t> idx, val;
    before.resize(n);
    for (int i = 0; i < n; ++i) {
        const int new_len = p->h_lens[ids[i]] + add[i];
        const size_t blocks = (size_t)(new_len + kPageTokens - 1) / kPageTokens;
        std::vector<int32_t>& pg = p->h_pages[ids[i]];
        before[i] = pg.size();
        while (pg.size() < blocks) {
            const int32_t page = p->free_list.back();
            p->free_list.pop_back();
            idx.push_back(ids[i] * p->max_blocks + (int32_t)pg.size());
            val.push_back(page);
            pg.push_back(page);
        }
    }
    if (!idx.empty()) {
        hipError_t e = launch_scatter(p->d_block_table, idx.data(), val.data(), (int)idx.size(), s);
        if (e != hipSuccess) {
            // nothing was enqueued for the failed chunk onwards; give the pages back
            for (int i = n; i-- > 0;) {
                std::vector<int32_t>& pg = p->h_pages[ids[i]];
                while (pg.size() > before[i]) { p->free_list.push_back(pg.back()); pg.pop_back(); }
            }
            return fail(SPIRAL_ERR_HIP, "%s: block-table update: %s", who, hipGetErrorString(e));
        }
    }
    return SPIRAL_OK;
}

// Undoes grow() on the host after a later step of the same call failed: pages return to the free list in the
// order they were taken from it, lengths were not advanced yet.  Block-table entries already written on the
// device lie beyond the sequences' lengths and are overwritten by the next grow.
static void ungrow(spiral_kv_pool* p, const int32_t* ids, int n, const std::vector<size_t>& before) {
    for (int i = n; i-- > 0;) {
        std::vector<int32_t>& pg = p->h_pages[ids[i]];
        while (pg.size() > before[i]) { p->free_list.push_back(pg.back()); pg.pop_back(); }
    }
}

// ---------------------------------------------------------------------------------------------
// the layer stack (shared by prefill and decode)
// ---------------------------------------------------------------------------------------------
struct StepCtx {
    spiral_model* m; spiral_kv_pool* p; Workspace w; hipStream_t s;
    int rows;            // activation rows
    int B;               // sequences
    bool decode;
    int max_new;         // prefill: longest appended run
    int n_chunks;        // decode: context chunks
    float* logits;
    int total_units = 0, units_per_wg = 0, n_slots = 0;   // decode, stream kernel
    const int32_t* score_targets = nullptr;                // scoring pass: per-row targets and output
    float* score_out = nullptr;
    bool sample = false;                                   // fused LM head + sampler (no logits written)
    float temperature = 0.f;
    int32_t* out_tokens = nullptr;
};

static int run_layers(StepCtx& c) {
    spiral_model* m = c.m;
    const spiral_model_config& cfg = m->cfg;
    const bool act32 = !m->w_bf16;
    const Tune& t = m->tune;
    const int d = cfg.d_model, hd = cfg.head_dim;
    const int qw = cfg.n_q_heads * hd, kw = cfg.n_kv_heads * hd, nqkv = qw + 2 * kw;
    const bool wide = c.rows > 128 || act32;      // many row tiles already fill the GPU: no K split
    // A narrow projection is split along K until its workgroups fill the 256 compute units in one
    // round (at least two 128-wide k chunks per split); 64-row workgroups when 128-row ones cannot.
    struct Shape { int bn, splits; };
    auto shape = [&](int bn, int s, int N, int K) {
        auto fit = [&](int rows) {
            const int tiles = (N + rows - 1) / rows;
            return std::max(1, std::min({256 / std::max(tiles, 1), kMaxSplit, K / 256}));
        };
        if (bn == 0) {
            const int t128 = (N + 127) / 128, t64 = (N + 63) / 64;
            bn = (t128 * fit(128) < 160 && t64 * fit(64) > t128 * fit(128)) ? 64 : 128;
        }
        if (s == 0) s = fit(bn);
        if (wide) s = 1;
        return Shape{bn, std::max(1, std::min(s, K / 128))};
    };
    const Shape sh_qkv = shape(t.bn_qkv, t.s_qkv, nqkv, d), sh_o = shape(t.bn_o, t.s_o, d, qw),
                sh_down = shape(t.bn_down, t.s_down, d, cfg.ffn_dim);
    const int s_qkv = sh_qkv.splits, s_o = sh_o.splits, s_down = sh_down.splits;
    int pending = 0;            // projection partials waiting to be added to the residual
    int32_t* sat = c.p->d_status;

    for (int l = 0; l < cfg.n_layers; ++l) {
        if (l > 0) {
            NormArgs n = {c.w.x, c.w.proj, (const float*)m->lw(l, SPIRAL_W_ATTN_NORM), c.w.h, nullptr, c.rows, c.rows, d, pending, cfg.rms_eps, sat};
            HIP_TRY(timed(m, SPIRAL_K_NORM, c.s, [&] { return launch_add_norm(n, act32, c.s); }));
        }
        GemmArgs g = {};
        g.A = c.w.h; g.w[0] = m->lw(l, SPIRAL_W_Q); g.w[1] = m->lw(l, SPIRAL_W_K); g.w[2] = m->lw(l, SPIRAL_W_V);
        g.rows[0] = qw; g.rows[1] = kw; g.rows[2] = kw;
        g.M = c.rows; g.N = nqkv; g.K = d; g.out = c.w.qkv; g.splits = s_qkv;
        g.wf = m->f_lm ? m->f_qkv[l] : nullptr;
        uint16_t* pages = c.p->d_pages + (size_t)l * c.p->layer_elems;
        QkvPostArgs qa = {c.w.qkv, m->lw(l, SPIRAL_W_BQ), m->lw(l, SPIRAL_W_BK), m->lw(l, SPIRAL_W_BV),
                          (const float*)m->lw(l, SPIRAL_W_Q_NORM), (const float*)m->lw(l, SPIRAL_W_K_NORM),
                          c.w.rope, c.w.row_page, c.w.q, pages,
                          c.rows, s_qkv, cfg.n_q_heads, cfg.n_kv_heads, hd, cfg.rms_eps, sat};
        if (t.fuse_qkv && s_qkv == 1 && sh_qkv.bn != 1 && gemm_tile_qkv_usable(g, qa, m->w_bf16)) {
            // thousands of rows (prefill, scoring): the projection's epilogue does the post-processing, the fp32 product
            // never reaches memory
            HIP_TRY(timed(m, SPIRAL_K_GEMM_QKV, c.s, [&] { return launch_gemm_tile_qkv(g, qa, c.s); }));
        } else {
            HIP_TRY(timed(m, SPIRAL_K_GEMM_QKV, c.s, [&] { return launch_gemm(g, EPI_STORE_F32, m->w_bf16, sh_qkv.bn, c.s); }));
            HIP_TRY(timed(m, SPIRAL_K_QKV_POST, c.s, [&] { return launch_qkv_post(qa, m->w_bf16, c.s); }));
        }

        AttnArgs aa = {};
        aa.q = c.w.q; aa.pages = pages; aa.block_table = c.p->d_block_table; aa.row_seq = c.w.row_seq;
        aa.row_pos = c.w.row_pos; aa.cu_rows = c.w.cu_rows; aa.part = c.w.attn_part; aa.out = c.w.o;
        aa.n_rows = c.rows; aa.n_q_heads = cfg.n_q_heads; aa.n_kv_heads = cfg.n_kv_heads;
        aa.max_blocks = c.p->max_blocks; aa.chunk_pages = t.chunk_pages; aa.n_chunks = c.n_chunks;
        aa.scale_log2e = (float)(1.4426950408889634 / std::sqrt((double)hd));
        if (c.decode) {
            aa.row_page_start = c.w.page_start; aa.units_per_wg = c.units_per_wg; aa.total_units = c.total_units;
            aa.n_chunks = c.n_slots;
            HIP_TRY(timed(m, SPIRAL_K_ATTN_DECODE, c.s, [&] { return launch_attn_stream(aa, hd, act32, c.s); }));
            HIP_TRY(timed(m, SPIRAL_K_ATTN_COMBINE, c.s, [&] { return launch_attn_stream_combine(aa, hd, act32, c.s); }));
        } else {
            HIP_TRY(timed(m, SPIRAL_K_ATTN_PREFILL, c.s, [&] { return launch_attn_prefill(aa, hd, c.B, c.max_new, act32, c.s); }));
        }

        GemmArgs go = {};
        go.A = c.w.o; go.w[0] = m->lw(l, SPIRAL_W_O); go.rows[0] = d;
        go.M = c.rows; go.N = d; go.K = qw; go.out = c.w.proj; go.splits = s_o;
        go.wf = m->f_lm ? m->f_o[l] : nullptr;
        HIP_TRY(timed(m, SPIRAL_K_GEMM_O, c.s, [&] { return launch_gemm(go, EPI_STORE_F32, m->w_bf16, sh_o.bn, c.s); }));

        NormArgs n2 = {c.w.x, c.w.proj, (const float*)m->lw(l, SPIRAL_W_MLP_NORM), c.w.h, nullptr, c.rows, c.rows, d, s_o, cfg.rms_eps, sat};
        HIP_TRY(timed(m, SPIRAL_K_NORM, c.s, [&] { return launch_add_norm(n2, act32, c.s); }));

        GemmArgs gu = {};
        gu.A = c.w.h; gu.w[0] = m->lw(l, SPIRAL_W_GATE); gu.w[1] = m->lw(l, SPIRAL_W_UP);
        gu.rows[0] = cfg.ffn_dim; gu.rows[1] = cfg.ffn_dim;
        gu.M = c.rows; gu.N = cfg.ffn_dim; gu.K = d; gu.out = c.w.mlp; gu.splits = 1;
        gu.wf = m->f_lm ? m->f_gu[l] : nullptr;
        gu.sat_count = sat;
        HIP_TRY(timed(m, SPIRAL_K_GEMM_GATE_UP, c.s, [&] { return launch_gemm(gu, EPI_SWIGLU, m->w_bf16, t.bn_gu, c.s); }));

        GemmArgs gd = {};
        gd.A = c.w.mlp; gd.w[0] = m->lw(l, SPIRAL_W_DOWN); gd.rows[0] = d;
        gd.M = c.rows; gd.N = d; gd.K = cfg.ffn_dim; gd.out = c.w.proj; gd.splits = s_down;
        gd.wf = m->f_lm ? m->f_down[l] : nullptr;
        HIP_TRY(timed(m, SPIRAL_K_GEMM_DOWN, c.s, [&] { return launch_gemm(gd, EPI_STORE_F32, m->w_bf16, sh_down.bn, c.s); }));
        pending = s_down;
    }
    if (c.score_out) {
        // scoring pass: final norm on every row, then the LM head fused with log-softmax and the target gather
        NormArgs na = {c.w.x, c.w.proj, (const float*)m->w[1], c.w.h, nullptr, c.rows, c.rows, d, pending, cfg.rms_eps, sat};
        HIP_TRY(timed(m, SPIRAL_K_NORM, c.s, [&] { return launch_add_norm(na, act32, c.s); }));
        const int n_tiles = (cfg.vocab + 127) / 128;
        ScoreArgs sa = {};
        sa.A = c.w.h; sa.W = m->w[2]; sa.Wf = m->f_lm; sa.targets = c.score_targets; sa.part = c.w.score_part; sa.tgt_logit = c.w.score_tgt;
        sa.M = c.rows; sa.V = cfg.vocab; sa.K = d;
        sa.tiles_per_split = (n_tiles + kScoreSplits - 1) / kScoreSplits;
        sa.n_splits = (n_tiles + sa.tiles_per_split - 1) / sa.tiles_per_split;
        HIP_TRY(timed(m, SPIRAL_K_GEMM_LM_HEAD, c.s, [&] { return launch_score(sa, c.score_out, c.s); }));
        return SPIRAL_OK;
    }
    // final norm on one row per sequence, then the LM head
    NormArgs nf = {c.w.x, c.w.proj, (const float*)m->w[1], c.w.hf, c.decode ? nullptr : c.w.last_rows,
                   c.rows, c.B, d, pending, cfg.rms_eps, sat};
    HIP_TRY(timed(m, SPIRAL_K_NORM, c.s, [&] { return launch_add_norm(nf, act32, c.s); }));
    GemmArgs gl = {};
    gl.A = c.w.hf; gl.w[0] = m->w[2]; gl.rows[0] = cfg.vocab;
    gl.M = c.B; gl.N = cfg.vocab; gl.K = d; gl.out = c.logits; gl.splits = 1;
    gl.wf = m->f_lm;
    if (c.sample) {
        // the LM head keeps the best (score, index) of each 128-column tile per row; a small kernel picks the winner
        const int cols = gemm_sample_tile_cols(c.B, t.bn_lm);
        gl.out = nullptr; gl.s_keys = c.w.s_keys; gl.s_part = c.w.s_part; gl.s_temperature = c.temperature;
        gl.s_tiles = (cfg.vocab + cols - 1) / cols;
        HIP_TRY(timed(m, SPIRAL_K_GEMM_LM_HEAD, c.s, [&] { return launch_gemm(gl, EPI_SAMPLE, m->w_bf16, t.bn_lm, c.s); }));
        HIP_TRY(timed(m, SPIRAL_K_SAMPLE, c.s, [&] { return launch_sample_pick(c.w.s_part, c.B, gl.s_tiles, c.out_tokens, c.s); }));
        return SPIRAL_OK;
    }
    HIP_TRY(timed(m, SPIRAL_K_GEMM_LM_HEAD, c.s, [&] { return launch_gemm(gl, EPI_STORE_F32, m->w_bf16, t.bn_lm, c.s); }));
    return SPIRAL_OK;
}

static int check_common(spiral_model* m, spiral_kv_pool* p, const void* toks, void* ws, float* logits, const char* who) {
    if (!m) return fail(SPIRAL_ERR_NOT_LOADED, "%s: null model", who);
    if (!p) return fail(SPIRAL_ERR_NOT_LOADED, "%s: null pool", who);
    if (p->m != m) return fail(SPIRAL_ERR_INVALID_ARG, "%s: pool belongs to another model", who);
    if (!toks || !logits) return fail(SPIRAL_ERR_INVALID_ARG, "%s: null token or output pointer", who);
    if (!ws || ((uintptr_t)ws & 255)) return fail(SPIRAL_ERR_INVALID_ARG, "%s: workspace null or not 256-byte aligned", who);
    if ((uintptr_t)logits & 15) return fail(SPIRAL_ERR_INVALID_ARG, "%s: logits not 16-byte aligned", who);
    return SPIRAL_OK;
}

// prefill and score share everything up to the output: last-row logits, or per-row log-probabilities
static int prefill_or_score(spiral_model* m, spiral_kv_pool* p, const int32_t* host_seq_ids, const int32_t* host_lens,
                            int B, const int32_t* dev_tokens_packed, void* dev_ws, size_t ws_bytes, float* dev_logits,
                            const int32_t* dev_targets, float* dev_logp, void* stream) {
    int rc = check_ids(p, host_seq_ids, B, "prefill");
    if (rc) return rc;
    if (!host_lens) return fail(SPIRAL_ERR_INVALID_ARG, "prefill: null lengths");
    long long rows = 0;
    int max_new = 0, max_ctx = 0;
    for (int i = 0; i < B; ++i) {
        if (host_lens[i] < 1) return fail(SPIRAL_ERR_INVALID_ARG, "prefill: length %d of sequence %d is not positive", host_lens[i], host_seq_ids[i]);
        rows += host_lens[i];
        max_new = std::max(max_new, host_lens[i]);
        const long long ctx = (long long)p->h_lens[host_seq_ids[i]] + host_lens[i];
        if (ctx > (long long)p->max_blocks * kPageTokens)
            return fail(SPIRAL_ERR_OOM_KV, "prefill: sequence %d would exceed its block table", host_seq_ids[i]);
        max_ctx = std::max(max_ctx, (int)ctx);
    }
    if (rows > (1ll << 30)) return fail(SPIRAL_ERR_SHAPE, "prefill: too many tokens");
    const size_t need = carve(m, nullptr, (int)rows, max_ctx).bytes;
    if (ws_bytes < need) return fail(SPIRAL_ERR_OOM_KV, "prefill: workspace of %zu bytes given, %zu needed", ws_bytes, need);
    hipStream_t s = (hipStream_t)stream;
    std::vector<size_t> before;
    rc = grow(p, host_seq_ids, host_lens, B, s, "prefill", before);
    if (rc) return rc;

    Workspace w = carve(m, (char*)dev_ws, (int)rows, max_ctx);
    std::vector<int32_t> cu(B + 1), base(B), last(B), ids(host_seq_ids, host_seq_ids + B);
    cu[0] = 0;
    for (int i = 0; i < B; ++i) {
        cu[i + 1] = cu[i] + host_lens[i];
        base[i] = p->h_lens[ids[i]];
        last[i] = cu[i + 1] - 1;
    }
    // everything that can fail runs before the lengths advance; on failure the pages go back
    auto enqueue = [&]() -> int {
        int32_t* dst[4] = {w.seq_ids, w.cu_rows, w.base_pos, w.last_rows};
        const int32_t* src[4] = {ids.data(), cu.data(), base.data(), last.data()};
        const int cnt[4] = {B, B + 1, B, B};
        HIP_TRY(launch_upload_multi(dst, src, cnt, 4, s));
        HIP_TRY(launch_prefill_meta(w.cu_rows, w.base_pos, w.seq_ids, B, (int)rows, w.row_seq, w.row_pos, s));
        EmbedArgs e = {dev_tokens_packed, m->w[0], (const float*)m->lw(0, SPIRAL_W_ATTN_NORM), w.x, w.h,
                       w.row_pos, w.rope, (int)rows, m->cfg.d_model, m->cfg.head_dim / 2, m->cfg.vocab, m->cfg.rms_eps,
                       w.row_seq, p->d_block_table, p->max_blocks, w.row_page};
        HIP_TRY(launch_embed_norm(e, m->freq, m->w_bf16, !m->w_bf16, s));
        StepCtx c = {m, p, w, s, (int)rows, B, false, max_new, 1, dev_logits};
        c.score_targets = dev_targets;
        c.score_out = dev_logp;
        return run_layers(c);
    };
    rc = enqueue();
    if (rc) { ungrow(p, host_seq_ids, B, before); return rc; }
    for (int i = 0; i < B; ++i) p->h_lens[ids[i]] = base[i] + host_lens[i];
    return SPIRAL_OK;
}

extern "C" int spiral_prefill(spiral_model* m, spiral_kv_pool* p, const int32_t* host_seq_ids, const int32_t* host_lens,
                              int B, const int32_t* dev_tokens_packed, void* dev_ws, size_t ws_bytes, float* dev_logits,
                              void* stream) {
    int rc = check_common(m, p, dev_tokens_packed, dev_ws, dev_logits, "prefill");
    if (rc) return rc;
    return prefill_or_score(m, p, host_seq_ids, host_lens, B, dev_tokens_packed, dev_ws, ws_bytes, dev_logits, nullptr, nullptr, stream);
}

extern "C" int spiral_score(spiral_model* m, spiral_kv_pool* p, const int32_t* host_seq_ids, const int32_t* host_lens,
                            int B, const int32_t* dev_tokens_packed, const int32_t* dev_targets, void* dev_ws,
                            size_t ws_bytes, float* dev_logp, void* stream) {
    if (!dev_targets) return fail(SPIRAL_ERR_INVALID_ARG, "score: null targets");
    int rc = check_common(m, p, dev_tokens_packed, dev_ws, dev_logp, "score");
    if (rc) return rc;
    if (!m->w_bf16) return fail(SPIRAL_ERR_SHAPE, "score: 16-bit weights only");
    if (m->cfg.d_model % 128) return fail(SPIRAL_ERR_SHAPE, "score: d_model must be a multiple of 128");
    return prefill_or_score(m, p, host_seq_ids, host_lens, B, dev_tokens_packed, dev_ws, ws_bytes, nullptr, dev_targets, dev_logp, stream);
}

extern "C" int spiral_policy_objective(const float* dev_logp_new, const float* dev_logp_old, const float* dev_advantage,
                                       const int32_t* dev_mask, long long n, float clip_eps, double* dev_out2, void* stream) {
    if (!dev_logp_new || !dev_logp_old || !dev_advantage || !dev_out2) return fail(SPIRAL_ERR_INVALID_ARG, "policy_objective: null pointer");
    if (n < 0 || !(clip_eps >= 0.f) || !std::isfinite(clip_eps)) return fail(SPIRAL_ERR_INVALID_ARG, "policy_objective: bad n or clip parameter");
    HIP_TRY(launch_score_objective(dev_logp_new, dev_logp_old, dev_advantage, dev_mask, n, clip_eps, dev_out2, (hipStream_t)stream));
    return SPIRAL_OK;
}

static uint64_t mix64_host(uint64_t z) {
    z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
    z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
    return z ^ (z >> 31);
}
// the generator key of (seed, sequence, step): see the sampler's description in spiral.h
static uint64_t row_key(uint64_t seed, int32_t seq_id, int32_t step) {
    const uint64_t k0 = mix64_host(seed ^ 0x9E3779B97F4A7C15ull);
    return mix64_host(k0 + (((uint64_t)(uint32_t)seq_id << 32) | (uint64_t)(uint32_t)step));
}

struct SampleSpec { float temperature; uint64_t seed; const int32_t* host_steps; int32_t* dev_out_tokens; };

// One decode step; with `sp` the LM head feeds the sampler directly and no logits are written.
static int decode_impl(spiral_model* m, spiral_kv_pool* p, const int32_t* host_seq_ids, int B, const int32_t* dev_in_tokens,
                       void* dev_ws, size_t ws_bytes, float* dev_logits, const SampleSpec* sp, void* stream, const char* who) {
    int rc = check_ids(p, host_seq_ids, B, who);
    if (rc) return rc;
    if (sp) {
        if (!(sp->temperature >= 0.f) || !std::isfinite(sp->temperature))
            return fail(SPIRAL_ERR_INVALID_ARG, "%s: temperature must be finite and >= 0", who);
        if (sp->temperature > 0.f) {
            if (!sp->host_steps) return fail(SPIRAL_ERR_INVALID_ARG, "%s: steps are needed to generate noise", who);
            for (int i = 0; i < B; ++i)
                if (sp->host_steps[i] < 0) return fail(SPIRAL_ERR_INVALID_ARG, "%s: negative step", who);
        }
        if (!m->w_bf16 || !m->f_lm || (m->cfg.d_model & 127) || (m->cfg.vocab & 15))
            return fail(SPIRAL_ERR_SHAPE, "%s: needs repacked 16-bit weights, d_model %% 128 == 0 and vocab %% 16 == 0", who);
    }
    int max_ctx = 0;
    for (int i = 0; i < B; ++i) max_ctx = std::max(max_ctx, p->h_lens[host_seq_ids[i]] + 1);
    const size_t need = carve(m, nullptr, B, max_ctx).bytes;
    if (ws_bytes < need) return fail(SPIRAL_ERR_OOM_KV, "%s: workspace of %zu bytes given, %zu needed", who, ws_bytes, need);
    hipStream_t s = (hipStream_t)stream;
    std::vector<int32_t> ones(B, 1);
    std::vector<size_t> before;
    rc = grow(p, host_seq_ids, ones.data(), B, s, who, before);
    if (rc) return rc;
    Workspace w = carve(m, (char*)dev_ws, B, max_ctx);

    // per-call host arrays, one by-value upload: sequence and position of every row, the prefix sum of the rows'
    // page counts after this step's append, and (sampling) the rows' generator keys as pairs of 32-bit halves
    std::vector<int32_t> pos(B), start(B + 1, 0), keys;
    for (int i = 0; i < B; ++i) {
        pos[i] = p->h_lens[host_seq_ids[i]];
        start[i + 1] = start[i] + (pos[i] + 1 + kPageTokens - 1) / kPageTokens;
    }
    if (sp && sp->temperature > 0.f) {
        keys.resize((size_t)2 * B);
        for (int i = 0; i < B; ++i) {
            const uint64_t k = row_key(sp->seed, host_seq_ids[i], sp->host_steps[i]);
            keys[2 * i] = (int32_t)(uint32_t)k;
            keys[2 * i + 1] = (int32_t)(uint32_t)(k >> 32);
        }
    }
    auto enqueue = [&]() -> int {
        int32_t* dst[4] = {w.row_seq, w.row_pos, w.page_start, (int32_t*)w.s_keys};
        const int32_t* src[4] = {host_seq_ids, pos.data(), start.data(), keys.data()};
        const int cnt[4] = {B, B, B + 1, (int)keys.size()};
        HIP_TRY(launch_upload_multi(dst, src, cnt, keys.empty() ? 3 : 4, s));
        EmbedArgs e = {dev_in_tokens, m->w[0], (const float*)m->lw(0, SPIRAL_W_ATTN_NORM), w.x, w.h,
                       w.row_pos, w.rope, B, m->cfg.d_model, m->cfg.head_dim / 2, m->cfg.vocab, m->cfg.rms_eps,
                       w.row_seq, p->d_block_table, p->max_blocks, w.row_page};
        HIP_TRY(launch_embed_norm(e, m->freq, m->w_bf16, !m->w_bf16, s));
        StepCtx c = {m, p, w, s, B, B, true, 1, decode_chunks(m, max_ctx), dev_logits};
        {
            const int wgs = m->tune.attn_wgs > 0 ? m->tune.attn_wgs : 3 * m->n_cus;
            c.total_units = start[B] * m->cfg.n_kv_heads;
            c.units_per_wg = std::max(m->tune.chunk_pages, (c.total_units + wgs - 1) / wgs);
            c.n_slots = decode_slots(m, max_ctx);
        }
        if (sp) { c.sample = true; c.temperature = sp->temperature; c.out_tokens = sp->dev_out_tokens; }
        return run_layers(c);
    };
    rc = enqueue();
    if (rc) { ungrow(p, host_seq_ids, B, before); return rc; }
    for (int i = 0; i < B; ++i) p->h_lens[host_seq_ids[i]] += 1;
    return SPIRAL_OK;
}

extern "C" int spiral_decode_step(spiral_model* m, spiral_kv_pool* p, const int32_t* host_seq_ids, int B,
                                  const int32_t* dev_in_tokens, void* dev_ws, size_t ws_bytes, float* dev_logits,
                                  void* stream) {
    int rc = check_common(m, p, dev_in_tokens, dev_ws, dev_logits, "decode_step");
    if (rc) return rc;
    return decode_impl(m, p, host_seq_ids, B, dev_in_tokens, dev_ws, ws_bytes, dev_logits, nullptr, stream, "decode_step");
}

extern "C" int spiral_decode_sample_step(spiral_model* m, spiral_kv_pool* p, const int32_t* host_seq_ids, int B,
                                         const int32_t* dev_in_tokens, void* dev_ws, size_t ws_bytes, float temperature,
                                         uint64_t seed, const int32_t* host_steps, int32_t* dev_out_tokens, void* stream) {
    int rc = check_common(m, p, dev_in_tokens, dev_ws, (float*)dev_out_tokens, "decode_sample_step");
    if (rc) return rc;
    const SampleSpec sp = {temperature, seed, host_steps, dev_out_tokens};
    return decode_impl(m, p, host_seq_ids, B, dev_in_tokens, dev_ws, ws_bytes, nullptr, &sp, stream, "decode_sample_step");
}

// Entry points for other translation units of the library: the workspace a decode step over the listed
// sequences needs, and the step itself on a given workspace.
int spiral_decode_workspace_need(spiral_model* m, spiral_kv_pool* p, const int32_t* host_seq_ids, int B, const char* who,
                                 size_t* need) {
    if (!m) return fail(SPIRAL_ERR_NOT_LOADED, "%s: null model", who);
    if (!p) return fail(SPIRAL_ERR_NOT_LOADED, "%s: null pool", who);
    if (p->m != m) return fail(SPIRAL_ERR_INVALID_ARG, "%s: pool belongs to another model", who);
    int rc = check_ids(p, host_seq_ids, B, who);
    if (rc) return rc;
    int max_ctx = 0;
    for (int i = 0; i < B; ++i) max_ctx = std::max(max_ctx, p->h_lens[host_seq_ids[i]] + 1);
    *need = carve(m, nullptr, B, max_ctx).bytes;
    return SPIRAL_OK;
}
int spiral_decode_on_workspace(spiral_model* m, spiral_kv_pool* p, const int32_t* host_seq_ids, int B, const int32_t* dev_in_tokens,
                               void* dev_ws, size_t ws_bytes, float* dev_logits, void* stream, const char* who) {
    int rc = check_common(m, p, dev_in_tokens, dev_ws, dev_logits, who);
    if (rc) return rc;
    return decode_impl(m, p, host_seq_ids, B, dev_in_tokens, dev_ws, ws_bytes, dev_logits, nullptr, stream, who);
}

// ---------------------------------------------------------------------------------------------
// sampling
// ---------------------------------------------------------------------------------------------
extern "C" int spiral_sample(const float* dev_logits, int B, int V, float temperature, uint64_t seed,
                             const int32_t* host_seq_ids, const int32_t* host_steps, const float* dev_noise,
                             int32_t* dev_out_tokens, void* stream) {
    if (!dev_logits || !dev_out_tokens) return fail(SPIRAL_ERR_INVALID_ARG, "sample: null logits or output");
    if (B < 1 || B > SPIRAL_MAX_BATCH || V < 1) return fail(SPIRAL_ERR_INVALID_ARG, "sample: bad B=%d or V=%d", B, V);
    if (!(temperature >= 0.f) || !std::isfinite(temperature)) return fail(SPIRAL_ERR_INVALID_ARG, "sample: temperature must be finite and >= 0");
    std::vector<uint64_t> keys(B, 0);
    if (temperature > 0.f && !dev_noise) {
        if (!host_seq_ids || !host_steps) return fail(SPIRAL_ERR_INVALID_ARG, "sample: seq ids and steps are needed to generate noise");
        for (int i = 0; i < B; ++i) {
            if (host_seq_ids[i] < 0 || host_steps[i] < 0) return fail(SPIRAL_ERR_INVALID_ARG, "sample: negative seq id or step");
            keys[i] = row_key(seed, host_seq_ids[i], host_steps[i]);
        }
    }
    HIP_TRY(launch_sample(dev_logits, B, V, temperature, keys.data(), temperature > 0.f ? dev_noise : nullptr,
                          dev_out_tokens, (hipStream_t)stream));
    return SPIRAL_OK;
}

static int sample_truncated_impl(const float* dev_logits, int B, int V, float temperature, int top_k, float top_p,
                                 uint64_t seed, const int32_t* host_seq_ids, const int32_t* host_steps,
                                 const float* dev_noise, int32_t* dev_out_tokens, float* dev_threshold_out,
                                 void* dev_workspace, size_t workspace_bytes, bool with_workspace, void* stream) {
    if (!(top_p > 0.f) || !(top_p <= 1.f)) return fail(SPIRAL_ERR_INVALID_ARG, "sample_truncated: top_p must be in (0, 1] (1 disables)");
    if (!(temperature >= 0.f) || !std::isfinite(temperature)) return fail(SPIRAL_ERR_INVALID_ARG, "sample_truncated: temperature must be finite and >= 0");
    if (temperature == 0.f && dev_threshold_out) return fail(SPIRAL_ERR_INVALID_ARG, "sample_truncated: greedy decoding has no threshold to report");
    if (with_workspace) {
        if (B < 1 || B > SPIRAL_MAX_BATCH || V < 1) return fail(SPIRAL_ERR_INVALID_ARG, "sample_truncated: bad B=%d or V=%d", B, V);
        if (!dev_workspace || ((uintptr_t)dev_workspace & 255)) return fail(SPIRAL_ERR_INVALID_ARG, "sample_truncated: workspace is null or not 256-byte aligned");
        const size_t need = sample_truncated_workspace_bytes(B, V);
        if (workspace_bytes < need) return fail(SPIRAL_ERR_INVALID_ARG, "sample_truncated: workspace of %zu bytes, %zu needed", workspace_bytes, need);
    }
    const bool cut = temperature > 0.f && ((top_k > 0 && top_k < V) || top_p < 1.f);
    if (!cut && !dev_threshold_out)      // nothing is truncated: the plain sampler is the same draw
        return spiral_sample(dev_logits, B, V, temperature, seed, host_seq_ids, host_steps, dev_noise, dev_out_tokens, stream);
    if (!dev_logits || !dev_out_tokens) return fail(SPIRAL_ERR_INVALID_ARG, "sample_truncated: null logits or output");
    if (B < 1 || B > SPIRAL_MAX_BATCH || V < 1) return fail(SPIRAL_ERR_INVALID_ARG, "sample_truncated: bad B=%d or V=%d", B, V);
    std::vector<uint64_t> keys(B, 0);
    if (!dev_noise) {
        if (!host_seq_ids || !host_steps) return fail(SPIRAL_ERR_INVALID_ARG, "sample_truncated: seq ids and steps are needed to generate noise");
        for (int i = 0; i < B; ++i) {
            if (host_seq_ids[i] < 0 || host_steps[i] < 0) return fail(SPIRAL_ERR_INVALID_ARG, "sample_truncated: negative seq id or step");
            keys[i] = row_key(seed, host_seq_ids[i], host_steps[i]);
        }
    }
    // short rows leave nothing to share between workgroups; without a cut the single kernel needs two sweeps only
    if (with_workspace && cut && V >= 16384)
        HIP_TRY(launch_sample_truncated_ws(dev_logits, B, V, temperature, top_k, top_p < 1.f ? top_p : 1.f, keys.data(), dev_noise,
                                           dev_out_tokens, dev_threshold_out, dev_workspace, (hipStream_t)stream));
    else
        HIP_TRY(launch_sample_truncated(dev_logits, B, V, temperature, top_k, top_p < 1.f ? top_p : 1.f, keys.data(), dev_noise,
                                        dev_out_tokens, dev_threshold_out, (hipStream_t)stream));
    return SPIRAL_OK;
}

extern "C" int spiral_sample_truncated(const float* dev_logits, int B, int V, float temperature, int top_k, float top_p,
                                       uint64_t seed, const int32_t* host_seq_ids, const int32_t* host_steps,
                                       const float* dev_noise, int32_t* dev_out_tokens, float* dev_threshold_out,
                                       void* stream) {
    return sample_truncated_impl(dev_logits, B, V, temperature, top_k, top_p, seed, host_seq_ids, host_steps, dev_noise,
                                 dev_out_tokens, dev_threshold_out, nullptr, 0, false, stream);
}

extern "C" size_t spiral_sample_truncated_workspace_bytes(int B, int V) {
    if (B < 1 || B > SPIRAL_MAX_BATCH || V < 1) return 0;
    return sample_truncated_workspace_bytes(B, V);
}

extern "C" int spiral_sample_truncated_ws(const float* dev_logits, int B, int V, float temperature, int top_k, float top_p,
                                          uint64_t seed, const int32_t* host_seq_ids, const int32_t* host_steps,
                                          const float* dev_noise, int32_t* dev_out_tokens, float* dev_threshold_out,
                                          void* dev_workspace, size_t workspace_bytes, void* stream) {
    return sample_truncated_impl(dev_logits, B, V, temperature, top_k, top_p, seed, host_seq_ids, host_steps, dev_noise,
                                 dev_out_tokens, dev_threshold_out, dev_workspace, workspace_bytes, true, stream);
}
