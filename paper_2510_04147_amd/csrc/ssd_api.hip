// Host side of the C ABI: validation, workspace carve-up, the forward driver
// (one pass of the transformer over a list of node groups) and the decoding
// loop of Algorithm 1.  All arithmetic of the method runs in the kernels; the
// host only decides which forward to launch next.
#include <algorithm>
#include <chrono>
#include <cmath>
#include <cstdarg>
#include <cstdio>
#include <cstring>
#include <new>

#include "ssd_internal.h"
#include "../../include/ssd_kernels.h"

#define HIPCHK(ctx, call)                                                                   \
    do {                                                                                    \
        hipError_t e_ = (call);                                                             \
        if (e_ != hipSuccess) {                                                             \
            set_err(ctx, "%s failed: %s (%s:%d)", #call, hipGetErrorString(e_), __FILE__, __LINE__); \
            return SSD_EHIP;                                                                \
        }                                                                                   \
    } while (0)

static void set_err(ssd_ctx* c, const char* fmt, ...) {
    if (!c) return;
    char buf[512];
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(buf, sizeof buf, fmt, ap);
    va_end(ap);
    c->err = buf;
}

static thread_local std::string g_create_err;

// ------------------------------------------------------------------ static scratch
// Device memory of the allocation-free entry point (ssd_k_lm_head_static): one array per GPU the
// library runs on, held until the process ends.  `scratch` is a host-side stand-in for the symbol;
// the device address comes from hipGetSymbolAddress, once per device, and only that pointer is
// ever handed to kernels or copies.
static __device__ __align__(256) unsigned char scratch[SSD_STATIC_SCRATCH_BYTES];
#define SSD_MAX_DEVICES 64
static void* g_scratch_ptr[SSD_MAX_DEVICES];          // per device, nullptr until resolved

// Resolves the array's address on `device` (which must be the current device).
static hipError_t resolve_scratch(int device) {
    if (device < 0 || device >= SSD_MAX_DEVICES) return hipErrorInvalidDevice;
    if (g_scratch_ptr[device]) return hipSuccess;
    void* p = nullptr;
    hipError_t e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
    if (e != hipSuccess) return e;
    if (!p) return hipErrorInvalidSymbol;
    g_scratch_ptr[device] = p;
    return hipSuccess;
}

extern "C" __attribute__((visibility("default"))) const char* ssd_strerror(int code) {
    switch (code) {
        case SSD_OK: return "ok";
        case SSD_EINVAL: return "invalid argument";
        case SSD_ERANGE: return "size or index out of range for this context";
        case SSD_ENOMEM: return "workspace too small";
        case SSD_EHIP: return "HIP runtime error";
        case SSD_ESTATE: return "call does not fit the cached prefix";
        default: return "unknown error";
    }
}

extern "C" __attribute__((visibility("default"))) const char* ssd_last_error(const ssd_ctx* c) { return c ? c->err.c_str() : g_create_err.c_str(); }

// ------------------------------------------------------------------ config
static int check_config(const ssd_config* cfg, std::string* why) {
    auto bad = [&](int code, const char* m) { *why = m; return code; };
    if (!cfg) return bad(SSD_EINVAL, "null config");
    if (cfg->n_layers < 1 || cfg->d_model < 8 || cfg->n_q_heads < 1 || cfg->n_kv_heads < 1 || cfg->d_ffn < 8 ||
        cfg->vocab < 2 || cfg->max_seqs < 1 || cfg->max_seq_len < 1 || cfg->block < 1 || cfg->max_draft < 0 ||
        cfg->max_rows < 1)
        return bad(SSD_EINVAL, "non-positive dimension");
    if (cfg->dtype != SSD_F32 && cfg->dtype != SSD_BF16) return bad(SSD_EINVAL, "dtype must be SSD_F32 or SSD_BF16");
    if (cfg->n_q_heads % cfg->n_kv_heads) return bad(SSD_EINVAL, "n_q_heads must be a multiple of n_kv_heads");
    if (cfg->head_dim != 64 && cfg->head_dim != 128) return bad(SSD_ERANGE, "head_dim must be 64 or 128");
    if (cfg->d_model % 8 || cfg->d_ffn % 8) return bad(SSD_EINVAL, "d_model and d_ffn must be multiples of 8");
    if (cfg->d_model > 8192) return bad(SSD_ERANGE, "d_model exceeds 8192");
    if (cfg->mask_id < 0 || cfg->mask_id >= cfg->vocab) return bad(SSD_EINVAL, "mask_id outside the vocabulary");
    if (cfg->block > SSD_MAX_BLOCK) return bad(SSD_ERANGE, "block exceeds SSD_MAX_BLOCK");
    if (cfg->max_draft > SSD_MAX_DRAFT) return bad(SSD_ERANGE, "max_draft exceeds SSD_MAX_DRAFT");
    if (cfg->max_seqs > SSD_MAX_SEQS) return bad(SSD_ERANGE, "max_seqs exceeds 16");
    if ((long long)cfg->max_seqs * (cfg->max_draft + 1) * cfg->block > cfg->max_rows)
        return bad(SSD_EINVAL, "max_rows smaller than max_seqs*(max_draft+1)*block");
    if (!(cfg->rope_theta > 0.f) || !(cfg->rms_eps >= 0.f)) return bad(SSD_EINVAL, "bad rope_theta / rms_eps");
    return SSD_OK;
}

static Dims dims_of(const ssd_config* c) {
    Dims d;
    d.L = c->n_layers; d.d = c->d_model; d.Hq = c->n_q_heads; d.Hkv = c->n_kv_heads; d.dh = c->head_dim;
    d.F = c->d_ffn; d.V = c->vocab; d.mask_id = c->mask_id; d.dtype = c->dtype; d.eps = c->rms_eps;
    d.max_seqs = c->max_seqs; d.max_seq_len = c->max_seq_len; d.block = c->block; d.max_draft = c->max_draft;
    d.max_rows = c->max_rows;
    return d;
}

// the finest vocabulary tiling of any kernel path is 32 columns per partial
static int lm_tiles_for(const Dims& d) { return (d.V + 31) / 32; }

static bool packable(const Dims& d, size_t N, size_t K) { return d.dtype == SSD_BF16 && N % 32 == 0 && K % 16 == 0; }

// Bytes of the fragment-order weight copies (bf16 models; shapes that do not tile stay unpacked).
static size_t packed_bytes(const Dims& d) {
    if (d.dtype != SSD_BF16) return 0;
    auto sz = [&](size_t N, size_t K) { return packable(d, N, K) ? ((N * K * 2 + 255) & ~(size_t)255) : 0; };
    return (sz(d.nqkv(), d.d) + sz(d.d, d.nq()) + sz(2 * (size_t)d.F, d.d) + sz(d.d, d.F)) * d.L + sz(d.V, d.d);
}

// Walks the workspace layout; with base == nullptr it only measures.
static size_t carve(const Dims& d, char* base, Buffers* b) {
    size_t off = 0;
    auto take = [&](size_t bytes) -> void* {
        off = (off + 255) & ~(size_t)255;
        void* p = base ? base + off : nullptr;
        off += bytes;
        return p;
    };
    const size_t R = d.max_rows, e = d.esz();
    const int tiles = lm_tiles_for(d);
    Buffers t;
    t.h = (float*)take(R * d.d * 4);
    t.xn = take(R * d.d * e);
    t.q = take(R * d.nq() * e);
    t.kown = take((size_t)d.nkv() * d.vt_rows() * e);
    t.vown = take((size_t)d.nkv() * d.vt_rows() * e);
    t.attn = take(R * d.nq() * e);
    t.act = take(R * d.F * e);
    const size_t pc = d.nqkv() > d.d ? d.nqkv() : d.d;
    t.part = (float*)take((size_t)SSD_MAX_SPLIT * R * pc * 4);
    t.packed = take(packed_bytes(d));
    t.lm_part = (float*)take(R * (size_t)tiles * 3 * 4);
    t.row_max = (float*)take(R * 4);
    t.row_arg = (int*)take(R * 4);
    t.row_conf = (float*)take(R * 4);
    t.row_tok = (int*)take(R * 4);
    t.row_pos = (int*)take(R * 4);
    t.row_node = (int*)take(R * 4);
    t.raw_tok = (int*)take(R * 4);
    const size_t cache = (size_t)d.L * d.max_seqs * d.Hkv * d.seq_stride() * d.dh * e;
    t.kcache = take(cache);
    t.vcache = take(cache);
    t.rope_cos = (float*)take((size_t)d.max_seq_len * (d.dh / 2) * 4);
    t.rope_sin = (float*)take((size_t)d.max_seq_len * (d.dh / 2) * 4);
    t.fwd = (FwdHeader*)take(sizeof(FwdHeader));
    t.state = (SeqState*)take(sizeof(SeqState) * SSD_MAX_SEQS);
    t.result = (StepResult*)take(sizeof(StepResult) * SSD_MAX_SEQS);
    t.out_tok = (int*)take((size_t)d.max_seqs * d.max_seq_len * 4);
    t.ref_conf = (float*)take((size_t)d.max_seqs * d.max_seq_len * 4);
    t.ref_arg = (int*)take((size_t)d.max_seqs * d.max_seq_len * 4);
    t.probe_logits = (float*)take((size_t)d.block * d.V * 4);
    t.probe_rank = (int*)take((SSD_MAX_DRAFT + 1) * 4);
    t.lm_tiles = tiles;
    if (b) *b = t;
    return (off + 255) & ~(size_t)255;
}

extern "C" __attribute__((visibility("default"))) size_t ssd_workspace_bytes(const ssd_config* cfg) {
    std::string why;
    if (check_config(cfg, &why) != SSD_OK) return 0;
    return carve(dims_of(cfg), nullptr, nullptr);
}

extern "C" __attribute__((visibility("default"))) int ssd_create(const ssd_config* cfg, const ssd_weights* w, void* workspace, size_t ws_bytes,
                          void* hip_stream, ssd_ctx** out) {
    std::string why;
    int rc = check_config(cfg, &why);
    if (rc != SSD_OK) { g_create_err = why; return rc; }
    if (!w || !out || !workspace) { g_create_err = "null weights / workspace / out"; return SSD_EINVAL; }
    if (!w->embed || !w->lm_head || !w->final_norm || !w->wqkv || !w->wo || !w->wgu || !w->wdown || !w->norm1 ||
        !w->norm2) { g_create_err = "null weight pointer"; return SSD_EINVAL; }
    if (((uintptr_t)workspace) & 255) { g_create_err = "workspace must be 256-byte aligned"; return SSD_EINVAL; }
    const Dims d = dims_of(cfg);
    const size_t need = carve(d, nullptr, nullptr);
    if (ws_bytes < need) { g_create_err = "workspace smaller than ssd_workspace_bytes()"; return SSD_ENOMEM; }
    for (int l = 0; l < d.L; ++l)
        if (!w->wqkv[l] || !w->wo[l] || !w->wgu[l] || !w->wdown[l] || !w->norm1[l] || !w->norm2[l]) {
            g_create_err = "null per-layer weight pointer";
            return SSD_EINVAL;
        }
    // The repack kernels below read the weights on `hip_stream`; whatever wrote them, on any stream
    // of this device, has to be complete first.  Creation is a one-time set-up call: wait for the device.
    {
        hipError_t es = hipDeviceSynchronize();
        if (es != hipSuccess) { g_create_err = std::string("hipDeviceSynchronize: ") + hipGetErrorString(es); return SSD_EHIP; }
    }
    ssd_ctx* c = new (std::nothrow) ssd_ctx();
    if (!c) { g_create_err = "host allocation failed"; return SSD_ENOMEM; }
    c->dm = d;
    carve(d, (char*)workspace, &c->b);
    c->stream = (hipStream_t)hip_stream;
    c->part_cols = d.nqkv() > d.d ? d.nqkv() : d.d;
    c->device = -1;
    {
        // the context lives on the current device; the static scratch array of that device is
        // resolved here, at set-up, so that the allocation-free entry point only looks it up
        hipError_t e0 = hipGetDevice(&c->device);
        if (e0 == hipSuccess) e0 = resolve_scratch(c->device);
        if (e0 != hipSuccess) {
            g_create_err = std::string("static scratch: ") + hipGetErrorString(e0);
            delete c;
            return SSD_EHIP;
        }
    }
    // weights: keep the caller's pointers, and repack what tiles into MFMA fragment order
    {
        char* pk = (char*)c->b.packed;
        auto mk = [&](const void* raw, int N, int K, int gate_rows = 0) {
            Wt t{raw, nullptr, N, K};
            if (packable(d, N, K)) {
                t.packed = pk;
                launch_pack_weights(raw, pk, N, K, gate_rows, c->stream);
                pk += ((size_t)N * K * 2 + 255) & ~(size_t)255;
            }
            return t;
        };
        c->lw.resize(d.L);
        for (int l = 0; l < d.L; ++l)
            c->lw[l] = LayerW{mk(w->wqkv[l], d.nqkv(), d.d), mk(w->wo[l], d.d, d.nq()), mk(w->wgu[l], 2 * d.F, d.d, d.F),
                              mk(w->wdown[l], d.d, d.F), w->norm1[l], w->norm2[l]};
        c->lm_head = mk(w->lm_head, d.V, d.d);
    }
    c->embed = w->embed; c->final_norm = w->final_norm;
    c->kernel_path = 1;
    c->fuse_boundary = 1;
    c->tree_mode = 0;
    c->cross_block = 0;
    c->spill_over = 0;
    c->cache_mode = 0;
    c->refresh_interval = 0;
    memset(c->total_len, 0, sizeof c->total_len);
    c->use_graphs = 0;
    memset(c->cached_len, 0, sizeof c->cached_len);
    c->profiling = false; c->ev_used = 0;
    memset(c->prof_ms, 0, sizeof c->prof_ms); memset(c->prof_n, 0, sizeof c->prof_n);
    c->stage_next = 0;
    c->stage_bytes = sizeof(FwdHeader) + (size_t)d.max_rows * 4 + sizeof(SeqState) * SSD_MAX_SEQS;
    for (int i = 0; i < ssd_ctx::kSlots; ++i) { c->stage[i] = nullptr; c->stage_ev[i] = nullptr; c->stage_used[i] = false; }
    c->host_result = nullptr;
    auto fail = [&](hipError_t e, const char* what) {
        g_create_err = std::string(what) + ": " + hipGetErrorString(e);
        ssd_destroy(c);
        return SSD_EHIP;
    };
    hipError_t e;
    for (int i = 0; i < ssd_ctx::kSlots; ++i) {
        if ((e = hipHostMalloc((void**)&c->stage[i], c->stage_bytes, hipHostMallocDefault)) != hipSuccess)
            return fail(e, "hipHostMalloc(staging)");
        if ((e = hipEventCreateWithFlags(&c->stage_ev[i], hipEventDisableTiming)) != hipSuccess)
            return fail(e, "hipEventCreate");
    }
    if ((e = hipHostMalloc((void**)&c->host_result, sizeof(StepResult) * SSD_MAX_SEQS, hipHostMallocDefault)) != hipSuccess)
        return fail(e, "hipHostMalloc(result)");
    // rotary table in double precision: angle(pos, i) = pos * theta^(-2i/dh)
    {
        const int half = d.dh / 2;
        std::vector<float> cs((size_t)d.max_seq_len * half), sn((size_t)d.max_seq_len * half);
        for (int i = 0; i < half; ++i) {
            const double inv = std::pow((double)cfg->rope_theta, -2.0 * i / d.dh);
            for (int p = 0; p < d.max_seq_len; ++p) {
                const double a = (double)p * inv;
                cs[(size_t)p * half + i] = (float)std::cos(a);
                sn[(size_t)p * half + i] = (float)std::sin(a);
            }
        }
        if ((e = hipMemcpy(c->b.rope_cos, cs.data(), cs.size() * 4, hipMemcpyHostToDevice)) != hipSuccess)
            return fail(e, "hipMemcpy(rope)");
        if ((e = hipMemcpy(c->b.rope_sin, sn.data(), sn.size() * 4, hipMemcpyHostToDevice)) != hipSuccess)
            return fail(e, "hipMemcpy(rope)");
        if ((e = hipMemset(c->b.state, 0, sizeof(SeqState) * SSD_MAX_SEQS)) != hipSuccess) return fail(e, "hipMemset");
        if ((e = hipMemset(c->b.result, 0, sizeof(StepResult) * SSD_MAX_SEQS)) != hipSuccess) return fail(e, "hipMemset");
    }
    *out = c;
    return SSD_OK;
}

extern "C" __attribute__((visibility("default"))) int ssd_destroy(ssd_ctx* c) {
    if (!c) return SSD_EINVAL;
    (void)hipStreamSynchronize(c->stream);
    for (int i = 0; i < ssd_ctx::kSlots; ++i) {
        if (c->stage[i]) (void)hipHostFree(c->stage[i]);
        if (c->stage_ev[i]) (void)hipEventDestroy(c->stage_ev[i]);
    }
    if (c->host_result) (void)hipHostFree(c->host_result);
    for (auto ev : c->ev_pool) (void)hipEventDestroy(ev);
    for (auto& g : c->graphs)
        if (g.exec) (void)hipGraphExecDestroy(g.exec);
    delete c;
    return SSD_OK;
}

extern "C" __attribute__((visibility("default"))) int ssd_reset(ssd_ctx* c, int seq) {
    if (!c) return SSD_EINVAL;
    if (seq < 0 || seq >= c->dm.max_seqs) { set_err(c, "seq %d out of range", seq); return SSD_ERANGE; }
    c->cached_len[seq] = 0;
    c->total_len[seq] = 0;
    return SSD_OK;
}

extern "C" __attribute__((visibility("default"))) int ssd_cached_len(ssd_ctx* c, int seq) {
    if (!c) return SSD_EINVAL;
    if (seq < 0 || seq >= c->dm.max_seqs) { set_err(c, "seq %d out of range", seq); return SSD_ERANGE; }
    return c->cached_len[seq];
}

extern "C" __attribute__((visibility("default"))) int ssd_set_kernel_path(ssd_ctx* c, int path) {
    if (!c || path < 0 || path > 2) return SSD_EINVAL;
    const int old = c->kernel_path;
    c->kernel_path = path;
    return old;
}

extern "C" __attribute__((visibility("default"))) int ssd_set_boundary_fusion(ssd_ctx* c, int on) {
    if (!c || (on != 0 && on != 1)) return SSD_EINVAL;
    const int old = c->fuse_boundary;
    c->fuse_boundary = on;
    return old;
}

extern "C" __attribute__((visibility("default"))) int ssd_set_cross_block(ssd_ctx* c, int on) {
    if (!c || (on != 0 && on != 1)) return SSD_EINVAL;
    const int old = c->cross_block;
    c->cross_block = on;
    return old;
}

extern "C" __attribute__((visibility("default"))) int ssd_set_spill_over(ssd_ctx* c, int on) {
    if (!c || (on != 0 && on != 1)) return SSD_EINVAL;
    const int old = c->spill_over;
    c->spill_over = on;
    return old;
}

extern "C" __attribute__((visibility("default"))) int ssd_set_cache_mode(ssd_ctx* c, int mode, int refresh_interval) {
    if (!c || (mode != 0 && mode != 1) || refresh_interval < 0) return SSD_EINVAL;
    const int old = c->cache_mode;
    c->cache_mode = mode;
    c->refresh_interval = refresh_interval;
    return old;
}

extern "C" __attribute__((visibility("default"))) int ssd_set_tree_mode(ssd_ctx* c, int mode) {
    if (!c || (mode != 0 && mode != 1)) return SSD_EINVAL;
    const int old = c->tree_mode;
    c->tree_mode = mode;
    return old;
}

extern "C" __attribute__((visibility("default"))) int ssd_set_graphs(ssd_ctx* c, int on) {
    if (!c || (on != 0 && on != 1)) return SSD_EINVAL;
    const int old = c->use_graphs;
    c->use_graphs = on;
    return old;
}

// --------------------------------------------------------------- profiling
static const char* kClassNames[KC_COUNT] = {"build_rows+embed", "rmsnorm", "gemm_qkv", "rope", "attention", "gemm_o",
                                            "gemm_gate_up_swiglu", "gemm_down", "lm_head_reduce", "lm_merge",
                                            "accept"};

struct ProfScope {
    ssd_ctx* c;
    bool on;
    size_t idx;
    ProfScope(ssd_ctx* c_, int cls) : c(c_), on(c_->profiling), idx(0) {
        if (!on) return;
        while (c->ev_pool.size() < c->ev_used + 2) {
            hipEvent_t ev;
            if (hipEventCreate(&ev) != hipSuccess) { on = false; return; }
            c->ev_pool.push_back(ev);
            c->ev_class.push_back(0);
        }
        idx = c->ev_used;
        c->ev_used += 2;
        c->ev_class[idx] = cls;
        (void)hipEventRecord(c->ev_pool[idx], c->stream);
    }
    ~ProfScope() {
        if (on) (void)hipEventRecord(c->ev_pool[idx + 1], c->stream);
    }
};

static void prof_collect(ssd_ctx* c) {
    (void)hipStreamSynchronize(c->stream);
    for (size_t i = 0; i + 1 < c->ev_used; i += 2) {
        float ms = 0.f;
        if (hipEventElapsedTime(&ms, c->ev_pool[i], c->ev_pool[i + 1]) == hipSuccess) {
            c->prof_ms[c->ev_class[i]] += ms;
            c->prof_n[c->ev_class[i]] += 1;
        }
    }
    c->ev_used = 0;
}

extern "C" __attribute__((visibility("default"))) int ssd_profile_begin(ssd_ctx* c) {
    if (!c) return SSD_EINVAL;
    (void)hipStreamSynchronize(c->stream);
    c->profiling = true;
    c->ev_used = 0;
    memset(c->prof_ms, 0, sizeof c->prof_ms);
    memset(c->prof_n, 0, sizeof c->prof_n);
    return SSD_OK;
}

extern "C" __attribute__((visibility("default"))) int ssd_profile_read(ssd_ctx* c, int* n_classes, const char** names, int64_t* launches, double* ms) {
    if (!c || !n_classes) return SSD_EINVAL;
    prof_collect(c);
    const int cap = *n_classes;
    for (int i = 0; i < KC_COUNT && i < cap; ++i) {
        if (names) names[i] = kClassNames[i];
        if (launches) launches[i] = c->prof_n[i];
        if (ms) ms[i] = c->prof_ms[i];
    }
    *n_classes = KC_COUNT;
    return SSD_OK;
}

extern "C" __attribute__((visibility("default"))) int ssd_profile_end(ssd_ctx* c) {
    if (!c) return SSD_EINVAL;
    prof_collect(c);
    c->profiling = false;
    return SSD_OK;
}

// ---------------------------------------------------------- forward driver
struct Upload {           // block state to push before the forward (stateless API)
    int seq;
    SeqState st;
};

// out = X * W^T.  EPI_F32 writes *n_split partial sums (the consumer adds them in order);
// EPI_SWIGLU treats W as [gate; up] and writes silu(gate)*up; EPI_LMHEAD writes *n_split
// per-tile (max, arg, sumexp) triples per row.
static void gemm(ssd_ctx* c, int cls, int epi, const void* X, const Wt& W, void* out, int M, int* n_split) {
    ProfScope ps(c, cls);
    *n_split = 1;
    if (c->kernel_path >= 1 && c->dm.dtype == SSD_BF16 && launch_gemm_mfma(c, epi, X, W, out, M, n_split, c->stream))
        return;
    const int N = epi == EPI_SWIGLU ? W.N / 2 : W.N;
    *n_split = epi == EPI_LMHEAD ? lm_tiles_plain(N) : 1;
    launch_gemm_plain(c, epi, X, W.raw, out, M, N, W.K, c->stream);
}

// Copies a forward's descriptor, its raw tokens and the block states to upload to the device through
// the pinned staging ring (asynchronous on the context's stream).
static int stage_forward(ssd_ctx* c, const FwdHeader& hd, const int32_t* raw, int n_raw, const Upload* ups, int n_ups,
                         const ssd_step_out* out) {
    const Dims& d = c->dm;
    hipStream_t st = c->stream;
    // ---- stage and upload the descriptor
    const int slot = c->stage_next;
    c->stage_next = (slot + 1) % ssd_ctx::kSlots;
    if (c->stage_used[slot]) HIPCHK(c, hipEventSynchronize(c->stage_ev[slot]));
    char* sp = c->stage[slot];
    memcpy(sp, &hd, sizeof hd);
    if (out) ((FwdHeader*)sp)->out = *out;
    HIPCHK(c, hipMemcpyAsync(c->b.fwd, sp, sizeof hd, hipMemcpyHostToDevice, st));
    if (n_raw > 0) {
        int* sr = (int*)(sp + sizeof(FwdHeader));
        memcpy(sr, raw, (size_t)n_raw * 4);
        HIPCHK(c, hipMemcpyAsync(c->b.raw_tok, sr, (size_t)n_raw * 4, hipMemcpyHostToDevice, st));
    }
    if (n_ups > 0) {
        SeqState* ss = (SeqState*)(sp + sizeof(FwdHeader) + (size_t)d.max_rows * 4);
        for (int i = 0; i < n_ups; ++i) {
            ss[i] = ups[i].st;
            HIPCHK(c, hipMemcpyAsync(&c->b.state[ups[i].seq], &ss[i], sizeof(SeqState), hipMemcpyHostToDevice, st));
        }
    }
    HIPCHK(c, hipEventRecord(c->stage_ev[slot], st));
    c->stage_used[slot] = true;

    return SSD_OK;
}

// Runs one forward over the groups in `hd` (decode groups first).  raw / n_raw:
// tokens of GM_RAW groups; ups: block states to upload first.
static int run_forward(ssd_ctx* c, const FwdHeader& hd, const int32_t* raw, int n_raw, const Upload* ups, int n_ups,
                       const ssd_step_out* out, const float* k_conf = nullptr, const int32_t* k_arg = nullptr) {
    hipStream_t st = c->stream;
    {
        const int rc = stage_forward(c, hd, raw, n_raw, ups, n_ups, out);
        if (rc != SSD_OK) return rc;
    }
    const Dims& d = c->dm;
    const int M = hd.M, ML = hd.M_logits;
    if (k_conf) {
        // kernel-level entry: the caller supplies every row's confidence and arg-max; only the
        // acceptance kernel runs
        HIPCHK(c, hipMemcpyAsync(c->b.row_conf, k_conf, (size_t)ML * 4, hipMemcpyDeviceToDevice, st));
        HIPCHK(c, hipMemcpyAsync(c->b.row_arg, k_arg, (size_t)ML * 4, hipMemcpyDeviceToDevice, st));
        HIPCHK(c, hipMemsetAsync(c->b.row_max, 0, (size_t)ML * 4, st));
        launch_accept(c, hd.n_groups, st);
        HIPCHK(c, hipGetLastError());
        return SSD_OK;
    }
    int max_blen = 0;
    bool any_write_kv = false, any_suffix = false;
    for (int i = 0; i < hd.n_nodes; ++i) {
        max_blen = std::max(max_blen, hd.nodes[i].blen);
        any_write_kv |= hd.nodes[i].write_kv != 0;
        any_suffix |= hd.nodes[i].T > hd.nodes[i].S + hd.nodes[i].blen;
    }

    // nodes per sequence, if every sequence of the forward has equally many, consecutive in the node list
    // (the attention launch then keeps the nodes and query heads that share a sequence's KV head on one XCD)
    int nodes_per_seq = 0;
    {
        int run = 0, first_run = 0;
        bool uniform = true;
        for (int i = 0; i < hd.n_nodes; ++i) {
            ++run;
            if (i + 1 == hd.n_nodes || hd.nodes[i + 1].seq != hd.nodes[i].seq) {
                if (first_run == 0) first_run = run;
                uniform &= run == first_run;
                run = 0;
            }
        }
        // a sequence may appear only once as a run (decode groups first, then its KV-append group: not uniform)
        bool seen[SSD_MAX_SEQS] = {};
        for (int i = 0; uniform && i < hd.n_nodes; i += first_run) {
            uniform &= !seen[hd.nodes[i].seq];
            seen[hd.nodes[i].seq] = true;
        }
        if (uniform) nodes_per_seq = first_run;
    }

    // ---- the kernel sequence: a function of (M, ML, n_nodes, n_groups, max_blen, kernel path) only
    auto launch_all = [&]() {
        {
            ProfScope ps(c, KC_ROWS);
            launch_build_rows(c, st, hd.n_nodes);
            launch_embed(c, M, st);
        }
        int n_part = 0, ns = 1;
        for (int l = 0; l < d.L; ++l) {
            const LayerW& w = c->lw[l];
            { ProfScope ps(c, KC_NORM); launch_norm(c, M, w.norm1, n_part, st); }
            n_part = 0;
            gemm(c, KC_GEMM_QKV, EPI_F32, c->b.xn, w.wqkv, c->b.part, M, &ns);
            // blocks of at most 32 rows: the attention kernel sums the partial sums and applies the
            // rotary embedding itself; a pure KV pass needs only the last layer's K and V, not its attention
            const bool last_kv_only = l == d.L - 1 && ML == 0;
            // (not in a forward that appends KV: with block-boundary fusion the next block's node reads
            // those cache entries in the same layer, so they must be written by an earlier kernel)
            const bool fused = c->kernel_path == 1 && !last_kv_only && !any_write_kv &&
                               attn_mfma_can_fuse_rope(c, max_blen);
            if (!fused) { ProfScope ps(c, KC_ROPE); launch_rope(c, hd.n_nodes, max_blen, l, ns, st); }
            if (last_kv_only) break;
            {
                ProfScope ps(c, KC_ATTN);
                if (!(c->kernel_path >= 1 && d.dtype == SSD_BF16 &&
                      launch_attn_mfma(c, hd.n_nodes, nodes_per_seq, max_blen, l, fused ? ns : -1, any_suffix, st)))
                    launch_attn_plain(c, M, l, st);
            }
            gemm(c, KC_GEMM_O, EPI_F32, c->b.attn, w.wo, c->b.part, M, &ns);
            { ProfScope ps(c, KC_NORM); launch_norm(c, M, w.norm2, ns, st); }
            gemm(c, KC_GEMM_GU, EPI_SWIGLU, c->b.xn, w.wgu, c->b.act, M, &ns);
            gemm(c, KC_GEMM_DOWN, EPI_F32, c->b.act, w.wdown, c->b.part, M, &ns);
            n_part = ns;
        }
        if (ML > 0) {
            { ProfScope ps(c, KC_NORM); launch_norm(c, ML, c->final_norm, n_part, st); }
            int tiles = 0;
            gemm(c, KC_LMHEAD, EPI_LMHEAD, c->b.xn, c->lm_head, c->b.lm_part, ML, &tiles);
            { ProfScope ps(c, KC_LMMERGE); launch_lm_merge(c, ML, tiles, st); }
            { ProfScope ps(c, KC_ACCEPT); launch_accept(c, hd.n_groups, st); }
        }
    };

    ssd_ctx::FwdGraph* fg = nullptr;
    const int gflags = (any_write_kv ? 1 : 0) | (any_suffix ? 2 : 0);
    if (c->use_graphs && !c->profiling && st != nullptr) {      // the legacy default stream cannot be captured
        for (auto& g : c->graphs)
            if (g.M == M && g.ML == ML && g.n_nodes == hd.n_nodes && g.n_groups == hd.n_groups &&
                g.max_blen == max_blen && g.kernel_path == c->kernel_path && g.flags == gflags) { fg = &g; break; }
        if (!fg && c->graphs.size() < 64) {
            c->graphs.push_back({M, ML, hd.n_nodes, hd.n_groups, max_blen, c->kernel_path, gflags, 0, nullptr});
            fg = &c->graphs.back();
        }
    }
    if (fg && fg->exec) {
        HIPCHK(c, hipGraphLaunch(fg->exec, st));
        return SSD_OK;
    }
    if (fg && fg->seen >= 1) {
        // second forward of this shape: every kernel it launches has run once (function attributes
        // are set), so the sequence can be recorded.  A failed capture leaves the shape eager.
        hipGraph_t graph = nullptr;
        if (hipStreamBeginCapture(st, hipStreamCaptureModeThreadLocal) == hipSuccess) {
            launch_all();
            hipError_t e = hipStreamEndCapture(st, &graph);
            if (e == hipSuccess && graph && hipGraphInstantiate(&fg->exec, graph, nullptr, nullptr, 0) == hipSuccess) {
                (void)hipGraphDestroy(graph);
                HIPCHK(c, hipGraphLaunch(fg->exec, st));
                return SSD_OK;
            }
            if (graph) (void)hipGraphDestroy(graph);
            fg->exec = nullptr;
        }
        (void)hipGetLastError();                     // a refused capture must not poison later error checks
        fg->seen = -1;                               // do not try again
    }
    launch_all();
    if (fg && fg->seen >= 0) fg->seen++;
    HIPCHK(c, hipGetLastError());
    return SSD_OK;
}

// Mix-order nodes of a chain with n_draft drafts (Section 5.2): one per non-leaf chain node but the last.
static int mix_nodes(const ssd_ctx* c, int n_draft) { return c->tree_mode == 1 && n_draft >= 2 ? n_draft - 1 : 0; }

// Appends a group to a header: n_chain chain nodes (node j holds drafts 1..j), then n_extra mix-order
// nodes (node m holds drafts 1..m and m+2); returns the rows it takes.
static int add_group(FwdHeader& hd, int seq, int mode, int blen, int S, int n_chain, int n_extra, int n_draft_next,
                     int fresh, int raw_off, int out_off, int allow_full = 0, bool leaf_writes_kv = false,
                     int T = 0) {
    GroupDesc& g = hd.groups[hd.n_groups];
    const int n_nodes = n_chain + n_extra;
    g.seq = seq; g.row0 = hd.M; g.blen = blen; g.S = S; g.n_nodes = n_nodes; g.mode = mode; g.raw_off = raw_off;
    g.n_draft_next = n_draft_next; g.fresh = fresh; g.out_off = out_off; g.node0 = hd.n_nodes; g.n_chain = n_chain;
    g.spec_next1 = 0; g.spec_of1 = 0; g.allow_full = allow_full;
    g.from_refresh = 0; g.leafless = 0; g.keep_ref = 0; g.pad[0] = g.pad[1] = 0;
    int vrows = hd.n_nodes ? hd.nodes[hd.n_nodes - 1].vrow0 + ((hd.nodes[hd.n_nodes - 1].blen + 63) & ~63) : 0;
    for (int j = 0; j < n_nodes; ++j) {
        NodeDesc& nd = hd.nodes[hd.n_nodes++];
        nd.seq = seq; nd.row0 = hd.M + j * blen; nd.blen = blen; nd.S = S; nd.group = hd.n_groups;
        nd.j = j < n_chain ? j : j - n_chain;
        nd.extra = j < n_chain ? -1 : j - n_chain + 1;
        nd.write_kv = mode != GM_DECODE || (leaf_writes_kv && j == n_chain - 1);
        nd.vrow0 = vrows;
        nd.T = T;
        vrows += (blen + 63) & ~63;
    }
    hd.n_groups++;
    hd.M += n_nodes * blen;
    if (mode == GM_DECODE) hd.M_logits = hd.M;
    return n_nodes * blen;
}

extern "C" __attribute__((visibility("default"))) int ssd_prefill_kv(ssd_ctx* c, int seq, const int32_t* tokens, int n, int pos0) {
    if (!c) return SSD_EINVAL;
    const Dims& d = c->dm;
    if (!tokens || n < 1 || pos0 < 0) { set_err(c, "prefill: null tokens, n < 1 or pos0 < 0"); return SSD_EINVAL; }
    if (seq < 0 || seq >= d.max_seqs) { set_err(c, "prefill: seq %d out of range", seq); return SSD_ERANGE; }
    if (n > d.max_rows) { set_err(c, "prefill: %d rows exceed max_rows %d", n, d.max_rows); return SSD_ERANGE; }
    if ((long long)pos0 + n > d.max_seq_len) { set_err(c, "prefill: pos0+n exceeds max_seq_len"); return SSD_ERANGE; }
    if (pos0 > c->cached_len[seq]) {
        set_err(c, "prefill: pos0 %d beyond the cached prefix %d", pos0, c->cached_len[seq]);
        return SSD_ESTATE;
    }
    for (int i = 0; i < n; ++i)
        if (tokens[i] < 0 || tokens[i] >= d.V) { set_err(c, "prefill: token id %d out of range", tokens[i]); return SSD_ERANGE; }
    FwdHeader hd;
    memset(&hd, 0, sizeof hd);
    add_group(hd, seq, GM_RAW, n, pos0, 1, 0, 0, 0, 0, -1);
    int rc = run_forward(c, hd, tokens, n, nullptr, 0, nullptr);
    if (rc == SSD_OK) { c->cached_len[seq] = pos0 + n; c->total_len[seq] = 0; }   // prefix-only cache again
    return rc;
}

static int popcount64(uint64_t x) { return __builtin_popcountll(x); }

static int step_common(ssd_ctx* c, const char* who, int n, const int* seqs, const int32_t* block_tok,
                       const uint64_t* masked, const int* pos0, const int* block_len, const int32_t* draft_pos,
                       const int32_t* draft_tok, const int* n_draft, int n_draft_next, const ssd_step_out* out,
                       const float* k_conf = nullptr, const int32_t* k_arg = nullptr) {
    if (!c) return SSD_EINVAL;
    const Dims& d = c->dm;
    const bool accept_only = k_conf != nullptr;          // no forward: prefix lengths play no part
    if (n < 1 || !seqs || !block_tok || !masked || (!pos0 && !accept_only)) { set_err(c, "%s: null argument or n < 1", who); return SSD_EINVAL; }
    if (n > d.max_seqs) { set_err(c, "%s: n %d exceeds max_seqs", who, n); return SSD_ERANGE; }
    if (n_draft_next < 0 || n_draft_next > d.max_draft) { set_err(c, "%s: n_draft_next out of range", who); return SSD_ERANGE; }
    FwdHeader hd;
    memset(&hd, 0, sizeof hd);
    Upload ups[SSD_MAX_SEQS];
    bool seen[SSD_MAX_SEQS] = {};
    for (int i = 0; i < n; ++i) {
        const int seq = seqs[i];
        if (seq < 0 || seq >= d.max_seqs) { set_err(c, "%s: seq %d out of range", who, seq); return SSD_ERANGE; }
        if (seen[seq]) { set_err(c, "%s: seq %d listed twice", who, seq); return SSD_EINVAL; }
        seen[seq] = true;
        const int bl = block_len ? block_len[i] : d.block;
        if (bl < 1 || bl > d.block) { set_err(c, "%s: block_len %d out of range", who, bl); return SSD_ERANGE; }
        const int p0 = accept_only ? 0 : pos0[i];
        if (!accept_only && p0 != c->cached_len[seq]) {
            set_err(c, "%s: pos0 %d is not the cached prefix length %d of seq %d", who, p0, c->cached_len[seq], seq);
            return SSD_ESTATE;
        }
        if ((long long)p0 + bl > d.max_seq_len) { set_err(c, "%s: block exceeds max_seq_len", who); return SSD_ERANGE; }
        const uint64_t mk = masked[i];
        if (bl < 64 && (mk >> bl)) { set_err(c, "%s: masked bits beyond block_len", who); return SSD_EINVAL; }
        const int nm = popcount64(mk);
        if (nm < 1) { set_err(c, "%s: no masked position in the block", who); return SSD_EINVAL; }
        const int nd = n_draft ? n_draft[i] : 0;
        if (nd < 0 || nd > d.max_draft) { set_err(c, "%s: n_draft %d out of range", who, nd); return SSD_ERANGE; }
        if (nd > nm - 1) { set_err(c, "%s: n_draft %d leaves the leaf no masked position (%d masked)", who, nd, nm); return SSD_EINVAL; }
        if (nd > 0 && (!draft_pos || !draft_tok)) { set_err(c, "%s: null drafts", who); return SSD_EINVAL; }
        SeqState& s = ups[i].st;
        memset(&s, 0, sizeof s);
        ups[i].seq = seq;
        s.masked = mk;
        s.n_draft = nd;
        for (int p = 0; p < bl; ++p) {
            const int t = block_tok[(size_t)i * d.block + p];
            if (t < 0 || t >= d.V) { set_err(c, "%s: token id %d out of range", who, t); return SSD_ERANGE; }
            s.tok[p] = ((mk >> p) & 1) ? d.mask_id : t;
        }
        uint64_t used = 0;
        for (int j = 0; j < nd; ++j) {
            const int q = draft_pos[(size_t)i * d.max_draft + j], t = draft_tok[(size_t)i * d.max_draft + j];
            if (q < 0 || q >= bl || !((mk >> q) & 1)) { set_err(c, "%s: draft position %d is not a masked position", who, q); return SSD_EINVAL; }
            if ((used >> q) & 1) { set_err(c, "%s: draft position %d listed twice", who, q); return SSD_EINVAL; }
            if (t < 0 || t >= d.V || t == d.mask_id) { set_err(c, "%s: draft token %d out of range", who, t); return SSD_ERANGE; }
            used |= 1ull << q;
            s.draft_pos[j] = q;
            s.draft_tok[j] = t;
        }
        if (hd.M + (nd + 1 + mix_nodes(c, nd)) * bl > d.max_rows) { set_err(c, "%s: forward exceeds max_rows", who); return SSD_ERANGE; }
        add_group(hd, seq, GM_DECODE, bl, p0, nd + 1, mix_nodes(c, nd), n_draft_next, 0, 0, -1, 0, false,
                  accept_only ? 0 : c->total_len[seq]);
    }
    return run_forward(c, hd, nullptr, 0, ups, n, out, k_conf, k_arg);
}

extern "C" __attribute__((visibility("default"))) int ssd_draft(ssd_ctx* c, int n, const int* seqs, const int32_t* block_tok, const uint64_t* masked,
                         const int* pos0, const int* block_len, int n_draft_next, const ssd_step_out* out) {
    return step_common(c, "ssd_draft", n, seqs, block_tok, masked, pos0, block_len, nullptr, nullptr, nullptr,
                       n_draft_next, out);
}

extern "C" __attribute__((visibility("default"))) int ssd_verify_tree(ssd_ctx* c, int n, const int* seqs, const int32_t* block_tok, const uint64_t* masked,
                               const int* pos0, const int* block_len, const int32_t* draft_pos,
                               const int32_t* draft_tok, const int* n_draft, int n_draft_next,
                               const ssd_step_out* out) {
    if (c && !n_draft) { set_err(c, "ssd_verify_tree: null n_draft"); return SSD_EINVAL; }
    return step_common(c, "ssd_verify_tree", n, seqs, block_tok, masked, pos0, block_len, draft_pos, draft_tok,
                       n_draft, n_draft_next, out);
}

// ------------------------------------------------ dual cache (Section 4.1)
// The three segments of a cache refresh for one sequence: the current block (a decode group whose one
// node also writes its KV), then, as raw-token groups appended by refresh_tail, everything before and
// everything behind it.  All three write their keys and values in each layer's rotary kernel, before
// that layer's attention kernel, and read every other position from the cache (NodeDesc::T): together
// one forward over the whole sequence with full bidirectional attention.
static void refresh_head(FwdHeader& hd, int seq, int pos0, int bl, int T, int n_draft_next, int fresh) {
    add_group(hd, seq, GM_DECODE, bl, pos0, 1, 0, n_draft_next, fresh, 0, -1, 0, true, T);
}
static void refresh_tail(FwdHeader& hd, int seq, const int32_t* tokens, int pos0, int bl, int T,
                         std::vector<int32_t>& raw) {
    if (pos0 > 0) {
        add_group(hd, seq, GM_RAW, pos0, 0, 1, 0, 0, 0, (int)raw.size(), -1, 0, false, T);
        raw.insert(raw.end(), tokens, tokens + pos0);
    }
    if (T > pos0 + bl) {
        add_group(hd, seq, GM_RAW, T - pos0 - bl, pos0 + bl, 1, 0, 0, 0, (int)raw.size(), -1, 0, false, T);
        raw.insert(raw.end(), tokens + pos0 + bl, tokens + T);
    }
}

extern "C" __attribute__((visibility("default"))) int ssd_refresh_kv(ssd_ctx* c, int seq, const int32_t* tokens, int total_len, int pos0,
                                                                     int block_len, int n_draft_next, const ssd_step_out* out) {
    if (!c) return SSD_EINVAL;
    const Dims& d = c->dm;
    if (!tokens || total_len < 1 || pos0 < 0 || block_len < 1) { set_err(c, "refresh: null tokens or bad lengths"); return SSD_EINVAL; }
    if (seq < 0 || seq >= d.max_seqs) { set_err(c, "refresh: seq %d out of range", seq); return SSD_ERANGE; }
    if (block_len > d.block || (long long)pos0 + block_len > total_len) { set_err(c, "refresh: block [%d, %d+%d) does not fit", pos0, pos0, block_len); return SSD_ERANGE; }
    if (total_len > d.max_rows || total_len > d.max_seq_len) { set_err(c, "refresh: %d positions exceed max_rows / max_seq_len", total_len); return SSD_ERANGE; }
    if (n_draft_next < 0 || n_draft_next > d.max_draft) { set_err(c, "refresh: n_draft_next out of range"); return SSD_ERANGE; }
    for (int i = 0; i < total_len; ++i)
        if (tokens[i] < 0 || tokens[i] >= d.V) { set_err(c, "refresh: token id %d out of range", tokens[i]); return SSD_ERANGE; }
    Upload up;
    memset(&up, 0, sizeof up);
    up.seq = seq;
    for (int p = 0; p < block_len; ++p) {
        up.st.tok[p] = tokens[pos0 + p];
        if (tokens[pos0 + p] == d.mask_id) up.st.masked |= 1ull << p;
    }
    if (!up.st.masked) { set_err(c, "refresh: no masked position in the block"); return SSD_EINVAL; }
    FwdHeader hd;
    memset(&hd, 0, sizeof hd);
    std::vector<int32_t> raw;
    refresh_head(hd, seq, pos0, block_len, total_len, n_draft_next, 0);
    refresh_tail(hd, seq, tokens, pos0, block_len, total_len, raw);
    int rc = run_forward(c, hd, raw.data(), (int)raw.size(), &up, 1, out);
    if (rc == SSD_OK) { c->cached_len[seq] = pos0; c->total_len[seq] = total_len; }
    return rc;
}

// The two timing events of a decoding loop, destroyed on every way out of it.
struct EventPair {
    hipEvent_t a = nullptr, b = nullptr;
    hipError_t create() {
        hipError_t e = hipEventCreate(&a);
        return e != hipSuccess ? e : hipEventCreate(&b);
    }
    ~EventPair() {
        if (a) (void)hipEventDestroy(a);
        if (b) (void)hipEventDestroy(b);
    }
};

// ssd_generate with the dual cache: a forward over the whole sequence renews the cache at the start
// and whenever refresh_interval tokens have been decoded since (0: the block length), and is itself the
// decoding step of that moment; a chain carries no more drafts than fit before the next refresh, so
// stepwise decoding and SSD refresh at the same states.  The host mirrors the sequences (the accepted
// (position, token) pairs come back with every round) because a refresh feeds all of them in again.
static int generate_dual(ssd_ctx* c, int n, const int32_t* const* prompts, const int* prompt_len, int gen_len, int block,
                         int draft_depth, int32_t* out_tokens, ssd_stats* stats) {
    const Dims& d = c->dm;
    const int R = c->refresh_interval > 0 ? c->refresh_interval : block;
    // Spill-over (Section 3.2.2): while a next block exists the chain may hold drafts for every remaining
    // position of the current block and then goes on in the next block, whose drafts are read off the last
    // refresh; a block nobody has predicted yet starts with such drafts too.  Between refreshes a block's
    // forward sees all other positions through the cache, so both blocks' nodes run in one forward.
    const bool spill = c->spill_over != 0;
    long long rows_all = 0;
    for (int i = 0; i < n; ++i) rows_all += prompt_len[i] + gen_len;
    if (rows_all > d.max_rows) {
        set_err(c, "generate: the dual cache refreshes whole sequences: %lld rows exceed max_rows %d", rows_all, d.max_rows);
        return SSD_ERANGE;
    }
    const auto t_begin = std::chrono::steady_clock::now();
    ssd_stats sta;
    memset(&sta, 0, sizeof sta);
    EventPair evp;
    HIPCHK(c, evp.create());
    const hipEvent_t ev0 = evp.a, ev1 = evp.b;
    const int n_blocks = (gen_len + block - 1) / block;
    std::vector<std::vector<int32_t>> x(n);
    int blk[SSD_MAX_SEQS], n_masked[SSD_MAX_SEQS], n_dr[SSD_MAX_SEQS], since[SSD_MAX_SEQS];
    bool start[SSD_MAX_SEQS], live_seq[SSD_MAX_SEQS], refresh_now[SSD_MAX_SEQS];
    for (int i = 0; i < n; ++i) {
        x[i].assign(prompts[i], prompts[i] + prompt_len[i]);
        x[i].resize((size_t)prompt_len[i] + gen_len, d.mask_id);
        blk[i] = 0; n_masked[i] = 0; n_dr[i] = 0; since[i] = R; start[i] = true; live_seq[i] = true;
        c->total_len[i] = 0;
    }
    auto block_len = [&](int b) { return std::min(block, gen_len - b * block); };
    int live = n, rc;
    std::vector<int32_t> raw;
    while (live > 0) {
        FwdHeader hd;
        memset(&hd, 0, sizeof hd);
        raw.clear();
        int master_of[SSD_MAX_SEQS], keep_end[SSD_MAX_SEQS];
        for (int i = 0; i < n; ++i) {                       // decode groups first: their rows get logits
            master_of[i] = -1;
            keep_end[i] = 0;
            if (!live_seq[i]) continue;
            const int S = prompt_len[i] + blk[i] * block, bl = block_len(blk[i]);
            const int T = prompt_len[i] + gen_len;
            const bool has_next = blk[i] + 1 < n_blocks;
            if (start[i]) { n_masked[i] = bl; n_dr[i] = 0; }
            refresh_now[i] = since[i] >= R;
            c->cached_len[i] = S;
            master_of[i] = hd.n_groups;
            if (refresh_now[i]) {
                refresh_head(hd, i, S, bl, T, draft_depth, start[i]);
                hd.groups[master_of[i]].allow_full = spill && has_next;
                continue;
            }
            const int budget = std::min(draft_depth, R - since[i] - 1);
            if (!spill) {
                const int ndr = std::max(0, std::min(std::min(n_dr[i], n_masked[i] - 1), budget));
                add_group(hd, i, GM_DECODE, bl, S, ndr + 1, 0, draft_depth, start[i], 0, -1, 0, false, T);
                continue;
            }
            // drafts at hand: the last node's, or (a block nobody predicted yet) all positions ranked by the refresh
            const int avail = start[i] ? bl : n_dr[i];
            const int a = std::max(0, std::min(std::min(avail, budget), has_next ? n_masked[i] : n_masked[i] - 1));
            const bool crossing = has_next && a == n_masked[i];
            add_group(hd, i, GM_DECODE, bl, S, crossing ? a : a + 1, 0, draft_depth, start[i], 0, -1, has_next, false, T);
            hd.groups[master_of[i]].from_refresh = start[i];
            hd.groups[master_of[i]].leafless = crossing;
            if (crossing) {
                const int bln = block_len(blk[i] + 1);
                const int b = std::max(0, std::min(budget - a, bln - 1));
                hd.groups[master_of[i]].spec_next1 = hd.n_groups + 1;
                add_group(hd, i, GM_DECODE, bln, S + bl, b + 1, 0, draft_depth, 1, 0, -1, blk[i] + 2 < n_blocks, false, T);
                hd.groups[hd.n_groups - 1].from_refresh = 1;
                hd.groups[hd.n_groups - 1].spec_of1 = master_of[i] + 1;
            }
        }
        // refreshes: the positions right behind the block, as far as decoding can get before the next refresh,
        // keep their predictions (the drafts of the blocks entered until then); they need logits, so they follow
        // the decode groups directly.  (Also without spill-over: how a refresh is cut into segments fixes the
        // summation order of its attention rows, and the switch must not change a single bit of the tokens.)
        for (int i = 0; i < n; ++i) {
            if (!live_seq[i] || !refresh_now[i]) continue;
            const int S = prompt_len[i] + blk[i] * block, bl = block_len(blk[i]), T = prompt_len[i] + gen_len;
            const int from = S + bl, upto = std::min(T, from + ((R + block - 1) / block + 1) * block);
            if (upto <= from) continue;
            add_group(hd, i, GM_RAW, upto - from, from, 1, 0, 0, 0, (int)raw.size(), -1, 0, false, T);
            hd.groups[hd.n_groups - 1].keep_ref = 1;
            raw.insert(raw.end(), x[i].begin() + from, x[i].begin() + upto);
            hd.M_logits = hd.M;
            keep_end[i] = upto;
        }
        for (int i = 0; i < n; ++i) {
            if (!live_seq[i] || !refresh_now[i]) continue;
            const int S = prompt_len[i] + blk[i] * block, bl = block_len(blk[i]), T = prompt_len[i] + gen_len;
            if (keep_end[i] > 0) {
                // everything before the block, then what lies behind the kept positions
                if (S > 0) {
                    add_group(hd, i, GM_RAW, S, 0, 1, 0, 0, 0, (int)raw.size(), -1, 0, false, T);
                    raw.insert(raw.end(), x[i].begin(), x[i].begin() + S);
                }
                if (T > keep_end[i]) {
                    add_group(hd, i, GM_RAW, T - keep_end[i], keep_end[i], 1, 0, 0, 0, (int)raw.size(), -1, 0, false, T);
                    raw.insert(raw.end(), x[i].begin() + keep_end[i], x[i].begin() + T);
                }
            } else {
                refresh_tail(hd, i, x[i].data(), S, bl, T, raw);
            }
            c->total_len[i] = T;
        }
        if (hd.M > d.max_rows) { set_err(c, "generate: forward exceeds max_rows"); return SSD_ERANGE; }
        (void)hipEventRecord(ev0, c->stream);
        if ((rc = run_forward(c, hd, raw.data(), (int)raw.size(), nullptr, 0, nullptr)) != SSD_OK) return rc;
        HIPCHK(c, hipMemcpyAsync(c->host_result, c->b.result, sizeof(StepResult) * d.max_seqs, hipMemcpyDeviceToHost, c->stream));
        (void)hipEventRecord(ev1, c->stream);
        if (hipEventSynchronize(ev1) != hipSuccess) { set_err(c, "generate: sync failed: %s", hipGetErrorString(hipGetLastError())); return SSD_EHIP; }
        float ms = 0; (void)hipEventElapsedTime(&ms, ev0, ev1);
        sta.decode_ms += ms;
        sta.forwards++;
        for (int i = 0; i < n; ++i) {
            if (master_of[i] < 0) continue;
            const GroupDesc& g = hd.groups[master_of[i]];
            const StepResult& r = c->host_result[i];
            const int bln = g.spec_next1 ? hd.groups[g.spec_next1 - 1].blen : 0;
            const int chain_next = g.spec_next1 ? hd.groups[g.spec_next1 - 1].n_chain : 0;
            const bool crossed = r.completed != 0;
            bool ok = r.n_accept >= 1 && r.n_accept <= SSD_MAX_DRAFT + 1;
            if (crossed)
                ok = ok && g.spec_next1 != 0 && g.leafless && r.n_in_next >= 1 && r.n_in_next <= chain_next &&
                     r.n_accept == n_masked[i] + r.n_in_next;
            else
                ok = ok && r.n_accept <= g.n_chain && r.n_accept <= n_masked[i] && r.n_in_next == 0;
            if (!ok) {
                set_err(c, "generate: acceptance kernel returned %d tokens (%d in the next block) for a chain of %d + %d nodes",
                        r.n_accept, r.n_in_next, g.n_chain, chain_next);
                return SSD_EHIP;
            }
            for (int k = 0; k < r.n_accept; ++k) {
                if (r.acc_pos[k] < 0 || r.acc_pos[k] >= g.blen + (crossed ? bln : 0)) { set_err(c, "generate: accepted position out of range"); return SSD_EHIP; }
                x[i][(size_t)g.S + r.acc_pos[k]] = r.acc_tok[k];
            }
            sta.accept_hist[r.n_accept]++;
            sta.tokens += r.n_accept;
            if (refresh_now[i]) { since[i] = 0; sta.kv_passes++; }
            since[i] += r.n_accept;
            n_dr[i] = r.n_next;
            start[i] = false;
            if (crossed) {
                blk[i]++;
                n_masked[i] = bln - r.n_in_next;
            } else {
                n_masked[i] -= r.n_accept;
            }
            if (n_masked[i] == 0) {
                blk[i]++;
                start[i] = true;
                if (blk[i] >= n_blocks) { live_seq[i] = false; live--; }
            }
        }
    }
    for (int i = 0; i < n; ++i)
        memcpy(out_tokens + (size_t)i * gen_len, x[i].data() + prompt_len[i], (size_t)gen_len * 4);
    sta.total_ms = std::chrono::duration<double, std::milli>(std::chrono::steady_clock::now() - t_begin).count();
    if (stats) *stats = sta;
    return SSD_OK;
}

// ------------------------------------------------------------- Algorithm 1
extern "C" __attribute__((visibility("default"))) int ssd_generate(ssd_ctx* c, int n, const int32_t* const* prompts, const int* prompt_len, int gen_len,
                            int block, int draft_depth, int32_t* out_tokens, ssd_stats* stats) {
    if (!c) return SSD_EINVAL;
    const Dims& d = c->dm;
    if (n < 1 || !prompts || !prompt_len || !out_tokens || gen_len < 1) { set_err(c, "generate: bad argument"); return SSD_EINVAL; }
    if (n > d.max_seqs) { set_err(c, "generate: n exceeds max_seqs"); return SSD_ERANGE; }
    if (block < 1 || block > d.block) { set_err(c, "generate: block %d out of range", block); return SSD_ERANGE; }
    if (draft_depth < 0 || draft_depth > d.max_draft) { set_err(c, "generate: draft_depth out of range"); return SSD_ERANGE; }
    for (int i = 0; i < n; ++i) {
        if (!prompts[i] || prompt_len[i] < 1) { set_err(c, "generate: empty prompt %d", i); return SSD_EINVAL; }
        if (prompt_len[i] > d.max_rows || (long long)prompt_len[i] + gen_len > d.max_seq_len) {
            set_err(c, "generate: prompt %d (+gen_len) exceeds max_rows / max_seq_len", i);
            return SSD_ERANGE;
        }
    }
    if (c->cache_mode == 1) return generate_dual(c, n, prompts, prompt_len, gen_len, block, draft_depth, out_tokens, stats);
    const auto t_begin = std::chrono::steady_clock::now();
    ssd_stats sta;
    memset(&sta, 0, sizeof sta);
    EventPair evp;
    HIPCHK(c, evp.create());
    const hipEvent_t ev0 = evp.a, ev1 = evp.b;
    auto done = [&](int rc) { return rc; };
    int rc;
    // prompt prefill, one segment per forward
    for (int i = 0; i < n; ++i) {
        c->cached_len[i] = 0;
        (void)hipEventRecord(ev0, c->stream);
        if ((rc = ssd_prefill_kv(c, i, prompts[i], prompt_len[i], 0)) != SSD_OK) return done(rc);
        (void)hipEventRecord(ev1, c->stream);
        if (hipEventSynchronize(ev1) != hipSuccess) { set_err(c, "generate: sync failed"); return done(SSD_EHIP); }
        float ms = 0; (void)hipEventElapsedTime(&ms, ev0, ev1);
        sta.kv_ms += ms; sta.kv_passes++;
    }
    const int n_blocks = (gen_len + block - 1) / block;
    enum { FRESH, DECODE, APPEND, DONE };
    int phase[SSD_MAX_SEQS], blk[SSD_MAX_SEQS], n_masked[SSD_MAX_SEQS], n_dr[SSD_MAX_SEQS];
    for (int i = 0; i < n; ++i) { phase[i] = FRESH; blk[i] = 0; n_masked[i] = 0; n_dr[i] = 0; }
    int live = n;
    while (live > 0) {
        FwdHeader hd;
        memset(&hd, 0, sizeof hd);
        bool any_decode = false;
        // Block-boundary fusion: the KV append of a finished block and the block-start draft of the
        // next block of the same sequence share one forward.  The append node's keys and values
        // reach the cache in each layer's rotary kernel, before that layer's attention kernel, so the
        // next block's node simply reads a prefix that is one block longer.  Fused only while the
        // forward still fits max_rows.
        bool fuse[SSD_MAX_SEQS] = {}, reach[SSD_MAX_SEQS] = {};
        const bool cross = c->cross_block && c->tree_mode == 0;
        {
            int rows = 0;
            for (int i = 0; i < n; ++i) {
                if (phase[i] == DONE) continue;
                const int bl = std::min(block, gen_len - blk[i] * block);
                const int ndr = phase[i] == FRESH ? 0 : n_dr[i];
                rows += phase[i] == APPEND ? bl : (ndr + 1 + mix_nodes(c, ndr)) * bl;
            }
            // extra rows, granted while the forward still fits max_rows: the next block behind a leaf that
            // holds a finished block (see below), then the next block's draft next to a KV append
            for (int i = 0; i < n; ++i) {
                if (!cross || phase[i] != DECODE || blk[i] + 1 >= n_blocks || n_dr[i] != n_masked[i]) continue;
                const int bln = std::min(block, gen_len - (blk[i] + 1) * block);
                if (rows + bln <= d.max_rows) { reach[i] = true; rows += bln; }
            }
            for (int i = 0; c->fuse_boundary && i < n; ++i) {
                if (phase[i] != APPEND || blk[i] + 1 >= n_blocks) continue;
                const int bln = std::min(block, gen_len - (blk[i] + 1) * block);
                if (rows + bln <= d.max_rows) { fuse[i] = true; rows += bln; }
            }
        }
        // A round across the block boundary (Section 3.2.2): while a next block exists the drafts may
        // cover every masked position of the current block (allow_full); when they do, the chain's leaf
        // holds the finished block, writes its KV, and a group for the next block, all masked, runs behind
        // it in the same forward.  The acceptance kernel uses that group only if every draft verifies.
        int spec_master[SSD_MAX_SEQS];
        for (int i = 0; i < n; ++i) spec_master[i] = -1;
        for (int pass = 0; pass < 2; ++pass)          // decode groups first, then KV appends
            for (int i = 0; i < n; ++i) {
                if (phase[i] == DONE) continue;
                const int bl = std::min(block, gen_len - blk[i] * block);
                const bool has_next = blk[i] + 1 < n_blocks;
                if (pass == 0 && phase[i] != APPEND) {
                    if (phase[i] == FRESH) { n_masked[i] = bl; n_dr[i] = 0; }
                    int ndr = n_dr[i];
                    const int bln = has_next ? std::min(block, gen_len - (blk[i] + 1) * block) : 0;
                    if (!reach[i] && ndr >= n_masked[i]) ndr = n_masked[i] - 1;   // the leaf must keep a position to predict
                    const int master = hd.n_groups;
                    add_group(hd, i, GM_DECODE, bl, c->cached_len[i], ndr + 1, mix_nodes(c, ndr), draft_depth,
                              phase[i] == FRESH, 0, reach[i] ? blk[i] * block : -1, cross && has_next, reach[i]);
                    if (reach[i]) {
                        const bool next_has_next = blk[i] + 2 < n_blocks;
                        hd.groups[master].spec_next1 = hd.n_groups + 1;
                        add_group(hd, i, GM_DECODE, bln, c->cached_len[i] + bl, 1, 0, draft_depth, 1, 0, -1,
                                  cross && next_has_next);
                        hd.groups[hd.n_groups - 1].spec_of1 = master + 1;
                        spec_master[i] = master;
                    }
                    any_decode = true;
                } else if (pass == 0 && fuse[i]) {
                    const int bln = std::min(block, gen_len - (blk[i] + 1) * block);
                    n_masked[i] = bln;
                    n_dr[i] = 0;
                    const bool next_has_next = blk[i] + 2 < n_blocks;
                    add_group(hd, i, GM_DECODE, bln, c->cached_len[i] + bl, 1, 0, draft_depth, 1, 0, -1, cross && next_has_next);
                    any_decode = true;
                } else if (pass == 1 && phase[i] == APPEND) {
                    add_group(hd, i, GM_APPEND, bl, c->cached_len[i], 1, 0, 0, 0, 0, blk[i] * block);
                }
            }
        if (hd.M > d.max_rows) { set_err(c, "generate: forward exceeds max_rows"); return done(SSD_ERANGE); }
        (void)hipEventRecord(ev0, c->stream);
        if ((rc = run_forward(c, hd, nullptr, 0, nullptr, 0, nullptr)) != SSD_OK) return done(rc);
        if (any_decode)
            HIPCHK(c, hipMemcpyAsync(c->host_result, c->b.result, sizeof(StepResult) * d.max_seqs, hipMemcpyDeviceToHost, c->stream));
        (void)hipEventRecord(ev1, c->stream);
        if (hipEventSynchronize(ev1) != hipSuccess) { set_err(c, "generate: sync failed: %s", hipGetErrorString(hipGetLastError())); return done(SSD_EHIP); }
        float ms = 0; (void)hipEventElapsedTime(&ms, ev0, ev1);
        if (any_decode) { sta.decode_ms += ms; sta.forwards++; } else { sta.kv_ms += ms; sta.kv_passes++; }
        for (int gi = 0; gi < hd.n_groups; ++gi) {
            const GroupDesc& g = hd.groups[gi];
            const int i = g.seq;
            if (g.mode == GM_DECODE && g.spec_of1 != 0) continue;     // reported through its master group
            if (g.mode == GM_DECODE) {
                const StepResult& r = c->host_result[i];
                if (r.completed) {
                    // the round verified drafts for every masked position: the block is finished, its tokens
                    // are in the output and its KV in the cache; the next block has its first token already
                    const int got_next = g.spec_next1 != 0 ? 1 : 0;
                    if (spec_master[i] != gi || r.n_accept != n_masked[i] + got_next) {
                        set_err(c, "generate: acceptance kernel finished a block with %d tokens, %d were masked", r.n_accept, n_masked[i]);
                        return done(SSD_EHIP);
                    }
                    sta.accept_hist[r.n_accept]++;
                    sta.tokens += r.n_accept;
                    c->cached_len[i] += g.blen;
                    blk[i]++;
                    if (blk[i] == n_blocks) { phase[i] = DONE; live--; continue; }
                    n_masked[i] = std::min(block, gen_len - blk[i] * block) - 1;
                    n_dr[i] = r.n_next;
                    phase[i] = n_masked[i] == 0 ? APPEND : DECODE;
                    continue;
                }
                if (r.n_accept < 1 || r.n_accept > g.n_chain || r.n_accept > n_masked[i]) {
                    set_err(c, "generate: acceptance kernel returned %d for a chain of %d nodes", r.n_accept, g.n_chain);
                    return done(SSD_EHIP);
                }
                sta.accept_hist[r.n_accept]++;
                sta.tokens += r.n_accept;
                n_masked[i] -= r.n_accept;
                n_dr[i] = r.n_next;
                phase[i] = n_masked[i] == 0 ? APPEND : DECODE;
            } else {
                c->cached_len[i] += g.blen;
                blk[i]++;
                if (blk[i] == n_blocks) { phase[i] = DONE; live--; }
                else if (!fuse[i]) phase[i] = FRESH;     // a fused sequence is already decoding its next block
            }
        }
    }
    for (int i = 0; i < n; ++i)
        HIPCHK(c, hipMemcpy(out_tokens + (size_t)i * gen_len, c->b.out_tok + (size_t)i * d.max_seq_len, (size_t)gen_len * 4,
                            hipMemcpyDeviceToHost));
    sta.total_ms = std::chrono::duration<double, std::milli>(std::chrono::steady_clock::now() - t_begin).count();
    if (stats) *stats = sta;
    return done(SSD_OK);
}

// ------------------------------------------- acceptance-rate limit (Section 5.1, Table 2)
extern "C" __attribute__((visibility("default"))) int ssd_acceptance_limit(ssd_ctx* c, const int32_t* prompt, int prompt_len, int gen_len,
                                                                           int block, int n_draft, int k_max, int32_t* out_tokens,
                                                                           int64_t* matched, int64_t* forwards, int64_t* rounds,
                                                                           double* reduction) {
    if (!c) return SSD_EINVAL;
    const Dims& d = c->dm;
    if (!prompt || prompt_len < 1 || gen_len < 1 || !matched || !forwards || k_max < 1) { set_err(c, "acceptance_limit: bad argument"); return SSD_EINVAL; }
    if (block < 1 || block > d.block) { set_err(c, "acceptance_limit: block %d out of range", block); return SSD_ERANGE; }
    if (n_draft < 0 || n_draft > SSD_MAX_DRAFT) { set_err(c, "acceptance_limit: n_draft out of range"); return SSD_ERANGE; }
    if (prompt_len > d.max_rows || (long long)prompt_len + gen_len > d.max_seq_len) { set_err(c, "acceptance_limit: prompt (+gen_len) exceeds max_rows / max_seq_len"); return SSD_ERANGE; }
    for (int k = 0; k < k_max; ++k) matched[k] = forwards[k] = 0;
    int64_t n_rounds = 0;
    int rc;
    c->cached_len[0] = 0;
    if ((rc = ssd_prefill_kv(c, 0, prompt, prompt_len, 0)) != SSD_OK) return rc;
    std::vector<int32_t> blk_tok(d.block);
    RankPairs pairs;
    int rank[SSD_MAX_DRAFT + 1];
    // ranks of a finished round against its first logits -> matched tokens and forwards of an ideal tree
    auto close_round = [&]() -> int {
        if (pairs.n == 0) return SSD_OK;
        launch_token_rank(c->b.probe_logits, d.V, d.mask_id, pairs, c->b.probe_rank, c->stream);
        HIPCHK(c, hipMemcpyAsync(rank, c->b.probe_rank, (size_t)pairs.n * 4, hipMemcpyDeviceToHost, c->stream));
        HIPCHK(c, hipStreamSynchronize(c->stream));
        for (int k = 1; k <= k_max; ++k) {
            int m = 0;
            for (int i = 0; i < pairs.n; ++i) m += rank[i] < k;
            matched[k - 1] += m;
            forwards[k - 1] += pairs.n - m + (m > 0 ? 1 : 0);
        }
        n_rounds++;
        pairs.n = 0;
        return SSD_OK;
    };
    const int n_blocks = (gen_len + block - 1) / block;
    for (int b = 0; b < n_blocks; ++b) {
        const int S = prompt_len + b * block, bl = std::min(block, gen_len - b * block);
        pairs.n = 0;
        for (int step = 0; step < bl; ++step) {
            FwdHeader hd;
            memset(&hd, 0, sizeof hd);
            add_group(hd, 0, GM_DECODE, bl, S, 1, 0, 0, step == 0, 0, -1);
            if ((rc = run_forward(c, hd, nullptr, 0, nullptr, 0, nullptr)) != SSD_OK) return rc;
            if (pairs.n == 0)   // a round's first forward: keep its logits (the normed rows are still in place)
                launch_gemm_plain(c, EPI_F32, c->b.xn, c->lm_head.raw, c->b.probe_logits, bl, d.V, d.d, c->stream);
            HIPCHK(c, hipMemcpyAsync(c->host_result, c->b.result, sizeof(StepResult), hipMemcpyDeviceToHost, c->stream));
            HIPCHK(c, hipStreamSynchronize(c->stream));
            const StepResult& r = c->host_result[0];
            if (r.n_accept != 1 || r.acc_pos[0] < 0 || r.acc_pos[0] >= bl || r.acc_tok[0] < 0 || r.acc_tok[0] >= d.V) {
                set_err(c, "acceptance_limit: a stepwise forward accepted %d tokens", r.n_accept);
                return SSD_EHIP;
            }
            blk_tok[r.acc_pos[0]] = r.acc_tok[0];
            pairs.pos[pairs.n] = r.acc_pos[0];
            pairs.tok[pairs.n] = r.acc_tok[0];
            pairs.n++;
            if (pairs.n == n_draft + 1 && (rc = close_round()) != SSD_OK) return rc;
        }
        if ((rc = close_round()) != SSD_OK) return rc;          // a block's last round may be short
        if (out_tokens) memcpy(out_tokens + (size_t)b * block, blk_tok.data(), (size_t)bl * 4);
        if (b + 1 < n_blocks && (rc = ssd_prefill_kv(c, 0, blk_tok.data(), bl, S)) != SSD_OK) return rc;
    }
    if (rounds) *rounds = n_rounds;
    // Table 2's quantity: the share of stepwise forwards an ideal verification tree would save
    if (reduction)
        for (int k = 0; k < k_max; ++k) reduction[k] = 1.0 - (double)forwards[k] / (double)gen_len;
    return SSD_OK;
}

// ---------------------------------------------------------- kernel-level entry
extern "C" __attribute__((visibility("default"))) int ssd_k_accept(ssd_ctx* c, int n, const int* seqs, const int32_t* block_tok,
                                                                   const uint64_t* masked, const int* block_len,
                                                                   const int32_t* draft_pos, const int32_t* draft_tok,
                                                                   const int* n_draft, int n_draft_next,
                                                                   const float* row_conf, const int32_t* row_argmax,
                                                                   const ssd_step_out* out) {
    if (!c) return SSD_EINVAL;
    if (!n_draft || !row_conf || !row_argmax) { set_err(c, "ssd_k_accept: null argument"); return SSD_EINVAL; }
    return step_common(c, "ssd_k_accept", n, seqs, block_tok, masked, nullptr, block_len, draft_pos, draft_tok, n_draft,
                       n_draft_next, out, row_conf, row_argmax);
}

extern "C" __attribute__((visibility("default"))) int ssd_k_write_cache(ssd_ctx* c, int seq, int layer, int pos0, int n,
                                                                        const void* k, const void* v) {
    if (!c) return SSD_EINVAL;
    const Dims& d = c->dm;
    if (!k || !v || n < 1 || pos0 < 0) { set_err(c, "k_write_cache: null pointer, n < 1 or pos0 < 0"); return SSD_EINVAL; }
    if (seq < 0 || seq >= d.max_seqs || layer < 0 || layer >= d.L) { set_err(c, "k_write_cache: seq or layer out of range"); return SSD_ERANGE; }
    if ((long long)pos0 + n > d.max_seq_len) { set_err(c, "k_write_cache: positions exceed max_seq_len"); return SSD_ERANGE; }
    launch_write_cache(c, seq, layer, pos0, n, k, v, c->stream);
    HIPCHK(c, hipGetLastError());
    return SSD_OK;
}

extern "C" __attribute__((visibility("default"))) int ssd_k_attention(ssd_ctx* c, int layer, int n_nodes, const ssd_k_node* nodes,
                                                                      const float* qkv, int n_part, int fused, void* out_attn,
                                                                      void* out_q, void* out_k, void* out_v) {
    if (!c) return SSD_EINVAL;
    const Dims& d = c->dm;
    if (!nodes || !qkv || !out_attn || n_nodes < 1 || n_part < 1) { set_err(c, "k_attention: null pointer, no node or no partial sum"); return SSD_EINVAL; }
    if (layer < 0 || layer >= d.L || n_nodes > d.max_nodes() || n_nodes > SSD_MAX_GROUPS || n_part > SSD_MAX_SPLIT) {
        set_err(c, "k_attention: layer, node count or partial-sum count out of range");
        return SSD_ERANGE;
    }
    FwdHeader hd;
    memset(&hd, 0, sizeof hd);
    int max_blen = 0;
    bool any_suffix = false;
    for (int i = 0; i < n_nodes; ++i) {
        const ssd_k_node& nd = nodes[i];
        if (nd.seq < 0 || nd.seq >= d.max_seqs || nd.blen < 1 || nd.S < 0 || (long long)nd.S + nd.blen > d.max_seq_len ||
            (nd.T != 0 && (nd.T < nd.S + nd.blen || nd.T > d.max_seq_len)) || hd.M + nd.blen > d.max_rows) {
            set_err(c, "k_attention: node %d does not fit the context (seq %d, S %d, blen %d, T %d)", i, nd.seq, nd.S, nd.blen, nd.T);
            return SSD_ERANGE;
        }
        add_group(hd, nd.seq, GM_RAW, nd.blen, nd.S, 1, 0, 0, 0, hd.M, -1, 0, false, nd.T);
        hd.nodes[hd.n_nodes - 1].write_kv = 0;           // the cache is the caller's: nothing is appended
        max_blen = std::max(max_blen, nd.blen);
        any_suffix |= nd.T > nd.S + nd.blen;
    }
    const int M = hd.M;
    const bool mfma = c->kernel_path >= 1 && d.dtype == SSD_BF16;
    if (fused && !(mfma && c->kernel_path == 1 && attn_mfma_can_fuse_rope(c, max_blen))) {
        set_err(c, "k_attention: the fused rotary stage needs bf16, kernel path 1, head size 128 and nodes of at most 32 rows");
        return SSD_EINVAL;
    }
    if (fused && (out_q || out_k || out_v)) { set_err(c, "k_attention: the fused kernel keeps q, k and v on chip"); return SSD_EINVAL; }
    std::vector<int32_t> zeros((size_t)M, 0);
    int rc = stage_forward(c, hd, zeros.data(), M, nullptr, 0, nullptr);
    if (rc != SSD_OK) return rc;
    hipStream_t st = c->stream;
    const size_t stride = (size_t)d.max_rows * c->part_cols;
    for (int sp = 0; sp < n_part; ++sp)
        HIPCHK(c, hipMemcpyAsync(c->b.part + sp * stride, qkv + (size_t)sp * M * d.nqkv(), (size_t)M * d.nqkv() * 4,
                                 hipMemcpyDeviceToDevice, st));
    launch_build_rows(c, st, hd.n_nodes);
    if (!fused) launch_rope(c, hd.n_nodes, max_blen, layer, n_part, st);
    if (!(mfma && launch_attn_mfma(c, hd.n_nodes, 0, max_blen, layer, fused ? n_part : -1, any_suffix, st)))
        launch_attn_plain(c, M, layer, st);
    HIPCHK(c, hipMemcpyAsync(out_attn, c->b.attn, (size_t)M * d.nq() * d.esz(), hipMemcpyDeviceToDevice, st));
    if (out_q) HIPCHK(c, hipMemcpyAsync(out_q, c->b.q, (size_t)M * d.nq() * d.esz(), hipMemcpyDeviceToDevice, st));
    if (out_k && out_v) launch_read_own_kv(c, M, out_k, out_v, st);
    HIPCHK(c, hipGetLastError());
    return SSD_OK;
}

extern "C" __attribute__((visibility("default"))) int ssd_k_norm(ssd_ctx* c, float* h, const float* partials, int n_part,
                                                                 const float* gain, int M, void* out) {
    if (!c) return SSD_EINVAL;
    const Dims& d = c->dm;
    if (!h || !gain || !out || M < 1 || n_part < 0 || (n_part > 0 && !partials)) { set_err(c, "k_norm: null pointer, M < 1 or n_part < 0"); return SSD_EINVAL; }
    if (M > d.max_rows || n_part > SSD_MAX_SPLIT) { set_err(c, "k_norm: M or n_part out of range"); return SSD_ERANGE; }
    hipStream_t st = c->stream;
    const size_t stride = (size_t)d.max_rows * c->part_cols;
    HIPCHK(c, hipMemcpyAsync(c->b.h, h, (size_t)M * d.d * 4, hipMemcpyDeviceToDevice, st));
    for (int sp = 0; sp < n_part; ++sp)
        HIPCHK(c, hipMemcpyAsync(c->b.part + sp * stride, partials + (size_t)sp * M * d.d, (size_t)M * d.d * 4,
                                 hipMemcpyDeviceToDevice, st));
    launch_norm(c, M, gain, n_part, st);
    HIPCHK(c, hipMemcpyAsync(h, c->b.h, (size_t)M * d.d * 4, hipMemcpyDeviceToDevice, st));
    HIPCHK(c, hipMemcpyAsync(out, c->b.xn, (size_t)M * d.d * d.esz(), hipMemcpyDeviceToDevice, st));
    HIPCHK(c, hipGetLastError());
    return SSD_OK;
}

extern "C" __attribute__((visibility("default"))) int ssd_k_lm_head_static(ssd_ctx* c, const void* x, int M,
                                                                           void* out) {
    if (!c) return SSD_EINVAL;
    const Dims& d = c->dm;
    if (!x || !out || M < 1) { set_err(c, "k_lm_head_static: null pointer or M < 1"); return SSD_EINVAL; }
    // per-tile partials [M, tiles, 3] fp32, then the rows' arg-max as integers [M]; the finest tiling of
    // any kernel path bounds the tile count
    const size_t tiles_max = (size_t)lm_tiles_for(d);
    const size_t part_bytes = (((size_t)M * tiles_max * 3 * 4) + 255) & ~(size_t)255;
    const size_t need = part_bytes + (size_t)M * 4;
    if (M > d.max_rows || need > SSD_STATIC_SCRATCH_BYTES) {
        set_err(c, "k_lm_head_static: %d rows of a %d-token vocabulary need %zu bytes of scratch, the static array holds %u",
                M, d.V, need, (unsigned)SSD_STATIC_SCRATCH_BYTES);
        return SSD_ERANGE;
    }
    void* sp = c->device >= 0 && c->device < SSD_MAX_DEVICES ? g_scratch_ptr[c->device] : nullptr;
    if (!sp) { set_err(c, "k_lm_head_static: the static scratch of device %d was never resolved", c->device); return SSD_EHIP; }
    float* part = (float*)sp;
    int* row_arg = (int*)((char*)sp + part_bytes);
    float* o = (float*)out;
    int tiles = 1;
    if (!(c->kernel_path >= 1 && d.dtype == SSD_BF16 &&
          launch_gemm_mfma(c, EPI_LMHEAD, x, c->lm_head, part, M, &tiles, c->stream))) {
        tiles = lm_tiles_plain(d.V);
        launch_gemm_plain(c, EPI_LMHEAD, x, c->lm_head.raw, part, M, d.V, d.d, c->stream);
    }
    launch_lm_merge_to(c, M, tiles, part, o, row_arg, o + 2 * (size_t)M, c->stream);
    launch_int_to_float(row_arg, o + M, M, c->stream);
    HIPCHK(c, hipGetLastError());
    return SSD_OK;
}

extern "C" __attribute__((visibility("default"))) int ssd_k_linear(ssd_ctx* c, int which, int layer, const void* x,
                                                                   int M, void* out) {
    if (!c) return SSD_EINVAL;
    const Dims& d = c->dm;
    if (!x || !out || M < 1) { set_err(c, "k_linear: null pointer or M < 1"); return SSD_EINVAL; }
    if (M > d.max_rows) { set_err(c, "k_linear: M exceeds max_rows"); return SSD_ERANGE; }
    if (which != SSD_LIN_LM && (layer < 0 || layer >= d.L)) { set_err(c, "k_linear: layer out of range"); return SSD_ERANGE; }
    int ns = 1;
    switch (which) {
        case SSD_LIN_QKV:
        case SSD_LIN_O:
        case SSD_LIN_DOWN: {
            const LayerW& w = c->lw[layer];
            const Wt& W = which == SSD_LIN_QKV ? w.wqkv : which == SSD_LIN_O ? w.wo : w.wdown;
            gemm(c, KC_GEMM_QKV, EPI_F32, x, W, c->b.part, M, &ns);
            launch_sum_partials(c, M, W.N, ns, (float*)out, c->stream);
            break;
        }
        case SSD_LIN_GU:
            gemm(c, KC_GEMM_GU, EPI_SWIGLU, x, c->lw[layer].wgu, out, M, &ns);
            break;
        case SSD_LIN_LM: {
            int tiles = 0;
            gemm(c, KC_LMHEAD, EPI_LMHEAD, x, c->lm_head, c->b.lm_part, M, &tiles);
            launch_lm_merge(c, M, tiles, c->stream);
            HIPCHK(c, hipMemcpyAsync(out, c->b.row_max, (size_t)M * 4, hipMemcpyDeviceToDevice, c->stream));
            launch_int_to_float(c->b.row_arg, (float*)out + M, M, c->stream);
            HIPCHK(c, hipMemcpyAsync((float*)out + 2 * (size_t)M, c->b.row_conf, (size_t)M * 4, hipMemcpyDeviceToDevice, c->stream));
            break;
        }
        default:
            set_err(c, "k_linear: unknown step %d", which);
            return SSD_EINVAL;
    }
    HIPCHK(c, hipGetLastError());
    return SSD_OK;
}
