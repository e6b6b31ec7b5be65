// C ABI of libmukv (declared in include/mukv.h): argument validation, context lifetime,
// and dispatch to the kernel launchers.  No torch types, no exceptions across the boundary.
#include <cmath>
#include <cstdio>
#include <cstring>
#include <mutex>
#include <new>
#include <vector>

#include "mukv_internal.h"

using mukv::Ctx;

struct mukv_ctx {
    Ctx c;
};

namespace {

constexpr double kDefaultRefineMargin = 1e-5;

bool pow2(int x) { return x > 0 && (x & (x - 1)) == 0; }

// Makes the context's device current for the duration of a call and gives the caller's back.
struct DeviceScope {
    int prev = -1;
    bool ok = false;
    explicit DeviceScope(int device) {
        if (hipGetDevice(&prev) != hipSuccess) prev = -1;
        ok = hipSetDevice(device) == hipSuccess;
    }
    ~DeviceScope() {
        if (prev >= 0) (void)hipSetDevice(prev);
    }
};

template <typename T>
hipError_t dalloc(T **p, size_t count) {
    *p = nullptr;
    if (count == 0) count = 1;
    return hipMalloc(reinterpret_cast<void **>(p), count * sizeof(T));
}

int validate_config(const mukv_config *cfg) {
    if (!cfg) return MUKV_ERR_INVALID_ARG;
    if (cfg->n_layers < 1 || cfg->n_q_heads < 1 || cfg->n_kv_heads < 1 || cfg->head_dim < 1 ||
        cfg->tokens_per_frame < 1 || cfg->frames_per_segment < 1 || cfg->superpatches_per_frame < 1 ||
        cfg->max_frames < 1 || cfg->max_chunk_frames < 1 || cfg->max_questions < 1 || cfg->device_id < 0)
        return MUKV_ERR_INVALID_ARG;
    if (cfg->dtype != MUKV_BF16 && cfg->dtype != MUKV_F32) return MUKV_ERR_INVALID_ARG;
    if (!(cfg->keep_ratio > 0.0) || cfg->keep_ratio > 1.0) return MUKV_ERR_INVALID_ARG;
    if (!(cfg->alpha >= 0.0) || cfg->alpha > 1.0) return MUKV_ERR_INVALID_ARG;
    if (cfg->n_q_heads % cfg->n_kv_heads) return MUKV_ERR_SHAPE;
    if (cfg->superpatches_per_frame > cfg->tokens_per_frame) return MUKV_ERR_SHAPE;
    if (cfg->score_layer < -1 || cfg->score_layer >= cfg->n_layers) return MUKV_ERR_SHAPE;
    if (cfg->att_path < MUKV_ATT_AUTO || cfg->att_path > MUKV_ATT_MFMA) return MUKV_ERR_INVALID_ARG;
    if (cfg->batch_chunks < 0) return MUKV_ERR_INVALID_ARG;
    if (cfg->overlap_copy != 0 && cfg->overlap_copy != 1) return MUKV_ERR_INVALID_ARG;
    if (cfg->freq_axis != MUKV_FREQ_FEATURE && cfg->freq_axis != MUKV_FREQ_TOKEN) return MUKV_ERR_INVALID_ARG;
    if (cfg->batch_chunks > mukv::kMaxSlots) return MUKV_ERR_UNSUPPORTED;
    const int kappa = (int)std::floor(cfg->keep_ratio * cfg->tokens_per_frame + 1e-9);
    if (kappa < 1) return MUKV_ERR_INVALID_ARG;
    if (!pow2(cfg->head_dim) || cfg->head_dim < 16 || cfg->head_dim > 128) return MUKV_ERR_UNSUPPORTED;
    if (cfg->tokens_per_frame > mukv::kMaxUnit) return MUKV_ERR_UNSUPPORTED;
    // a unit of several frames: ranked as one, attention signal from the caller, feature-axis indicator
    const bool large_unit = cfg->tokens_per_frame > mukv::kMaxP;
    if (large_unit && cfg->freq_axis != MUKV_FREQ_FEATURE) return MUKV_ERR_UNSUPPORTED;
    if ((int64_t)cfg->n_kv_heads * cfg->head_dim > 1024) return MUKV_ERR_UNSUPPORTED;
    if (cfg->n_q_heads / cfg->n_kv_heads > 1024) return MUKV_ERR_UNSUPPORTED; // the question pooling holds 4 * G partial sums per feature in LDS
    const int esz = cfg->dtype == MUKV_BF16 ? 2 : 4;
    if (!large_unit &&
        mukv::att_generic_lds_bytes(cfg->tokens_per_frame, cfg->head_dim, sizeof(double), sizeof(float)) > 160 * 1024)
        return MUKV_ERR_UNSUPPORTED;
    if ((cfg->head_dim * esz) % 16) return MUKV_ERR_UNSUPPORTED;
    if (((int64_t)cfg->max_frames + cfg->frames_per_segment - 1) / cfg->frames_per_segment > 65536)
        return MUKV_ERR_UNSUPPORTED;
    // block numbers (frame * S + s) and batch token offsets are 32-bit in the kernels
    if ((int64_t)cfg->max_frames * cfg->superpatches_per_frame > 0x7fffffff ||
        (int64_t)cfg->max_frames * cfg->tokens_per_frame > 0x7fffffff)
        return MUKV_ERR_UNSUPPORTED;
    return MUKV_OK;
}

bool mfma_supported(const mukv_config &c) { return mukv::att_mfma_supported(c); }

// Scratch of mukv_prefill_attend_static, for callers that may not allocate: one array per GPU in the
// library's device image, held until the process ends.  `scratch` itself is only the host-side
// handle of the symbol; the array's device address differs from GPU to GPU and is looked up once per
// device (with that device current) and kept in g_scratch_ptr, which is what the kernels are given.
static __device__ __align__(256) unsigned char scratch[MUKV_STATIC_SCRATCH_BYTES];
void *g_scratch_ptr[mukv::kMaxDevices];
std::mutex g_scratch_lock;

// The calling thread's current device must be `device`.
hipError_t static_scratch(int device, void **ptr) {
    if (device < 0 || device >= mukv::kMaxDevices) return hipErrorInvalidDevice;
    std::lock_guard<std::mutex> hold(g_scratch_lock);
    if (!g_scratch_ptr[device]) {
        void *p = nullptr;
        const hipError_t e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess) return e;
        if (!p) return hipErrorInvalidSymbol;
        g_scratch_ptr[device] = p;
    }
    *ptr = g_scratch_ptr[device];
    return hipSuccess;
}

// most kept tokens one super-patch can hold: the last super-patch is the longest
int patch_cap(const Ctx &c) {
    const int P = c.cfg.tokens_per_frame, S = c.cfg.superpatches_per_frame;
    const int longest = P - (S - 1) * (P / S);
    return longest < c.kappa ? longest : c.kappa;
}

void free_all(Ctx &c) {
    void *ptrs[] = {c.store_k,    c.store_v,    c.kept_idx,  c.rep_frame_k, c.rep_frame_v, c.rep_patch_k,
                    c.rep_patch_v, c.rep_seg_k, c.rep_seg_v, c.cnt_patch,   c.fsum_k,      c.fsum_v,
                    c.ssum_k,      c.ssum_v,    c.margin,      c.refined,   c.att_part[0], c.att_part[1], c.fft_sig[0], c.fft_sig[1],     c.att64,       c.fft64,
                    c.src_tok[0],  c.src_tok[1],   c.src_tok2,    c.flag_list[0], c.flag_list[1], c.flag_count, c.qbar,      c.qq,        c.s_frm,       c.s_seg,       c.seg_tail,
                    c.u_mask,      c.u_entry,     c.u_count,   c.attend_part, c.tw32, c.tw64, c.tok_part, c.m_entry, c.m_count, c.dft_tab};
    // nothing of the library's own may still be running on what is freed below
    if (c.side) (void)hipStreamSynchronize(c.side);
    for (void *p : ptrs)
        if (p) (void)hipFree(p);
    if (c.side) (void)hipStreamDestroy(c.side);
    for (hipEvent_t ev : c.ev_keep)
        if (ev) (void)hipEventDestroy(ev);
    if (c.ev_fork) (void)hipEventDestroy(c.ev_fork);
    for (hipEvent_t ev : c.ev_join)
        if (ev) (void)hipEventDestroy(ev);
    delete[] c.deferred;
    if (c.ev_copy) (void)hipEventDestroy(c.ev_copy);
}

} // namespace

// ---- snapshot of the cache: header, then every table trimmed to the frames it holds ----
namespace {
struct SnapHeader {
    char magic[8]; // "MUKVSNP1"
    int32_t n_layers, n_q_heads, n_kv_heads, head_dim, tokens_per_frame, frames_per_segment, superpatches_per_frame, dtype;
    int32_t kappa, score_layer;
    int64_t n_frames;
};

// the pieces of the cache in file order: device pointer, bytes used by n frames, stride between
// `count` such pieces on the device (the store is one piece per (layer, head) slab)
struct SnapPiece {
    void *dev;
    size_t bytes, stride;
    int count;
};

std::vector<SnapPiece> snap_pieces(const Ctx &c, int64_t n) {
    const size_t C = c.c_kv, S = c.cfg.superpatches_per_frame, row_b = (size_t)c.cfg.head_dim * c.esz;
    const size_t ns = (size_t)((n + c.cfg.frames_per_segment - 1) / c.cfg.frames_per_segment);
    const int slabs = c.cfg.n_layers * c.cfg.n_kv_heads;
    const size_t un = (size_t)n;
    return {
        {c.store_k, un * c.kappa * row_b, (size_t)c.store_cap * row_b, slabs},
        {c.store_v, un * c.kappa * row_b, (size_t)c.store_cap * row_b, slabs},
        {c.kept_idx, un * c.kappa * 4, 0, 1},
        {c.rep_frame_k, un * C * 4, 0, 1},
        {c.rep_frame_v, un * C * 4, 0, 1},
        {c.rep_patch_k, un * S * C * 4, 0, 1},
        {c.rep_patch_v, un * S * C * 4, 0, 1},
        {c.cnt_patch, un * S * 4, 0, 1},
        {c.rep_seg_k, ns * C * 4, 0, 1},
        {c.rep_seg_v, ns * C * 4, 0, 1},
        {c.fsum_k, un * C * 8, 0, 1},
        {c.fsum_v, un * C * 8, 0, 1},
        {c.ssum_k, ns * C * 8, 0, 1},
        {c.ssum_v, ns * C * 8, 0, 1},
        {c.margin, un * 4, 0, 1},
        {c.refined, un * 4, 0, 1},
    };
}

int64_t snap_bytes(const Ctx &c, int64_t n) {
    int64_t total = (int64_t)sizeof(SnapHeader);
    for (const SnapPiece &p : snap_pieces(c, n)) total += (int64_t)p.bytes * p.count;
    return total;
}

SnapHeader snap_header(const Ctx &c) {
    SnapHeader h;
    std::memset(&h, 0, sizeof h);
    std::memcpy(h.magic, "MUKVSNP1", 8);
    h.n_layers = c.cfg.n_layers;
    h.n_q_heads = c.cfg.n_q_heads;
    h.n_kv_heads = c.cfg.n_kv_heads;
    h.head_dim = c.cfg.head_dim;
    h.tokens_per_frame = c.cfg.tokens_per_frame;
    h.frames_per_segment = c.cfg.frames_per_segment;
    h.superpatches_per_frame = c.cfg.superpatches_per_frame;
    h.dtype = c.cfg.dtype;
    h.kappa = c.kappa;
    h.score_layer = c.ls;
    h.n_frames = c.n_frames;
    return h;
}
} // namespace

extern "C" {

const char *mukv_strerror(int status) {
    switch (status) {
    case MUKV_OK: return "ok";
    case MUKV_ERR_INVALID_ARG: return "invalid argument";
    case MUKV_ERR_SHAPE: return "shape inconsistent with the configuration";
    case MUKV_ERR_CAPACITY: return "capacity exceeded";
    case MUKV_ERR_UNSUPPORTED: return "unsupported shape or alignment";
    case MUKV_ERR_HIP: return "HIP runtime error";
    default: return "unknown status";
    }
}

int mukv_create(const mukv_config *cfg, mukv_ctx **out) {
    if (!out) return MUKV_ERR_INVALID_ARG;
    int rc = validate_config(cfg);
    if (rc != MUKV_OK) return rc;
    if (cfg->att_path == MUKV_ATT_MFMA && !mfma_supported(*cfg)) return MUKV_ERR_UNSUPPORTED;
    int n_dev = 0;
    if (hipGetDeviceCount(&n_dev) != hipSuccess || cfg->device_id >= n_dev) return MUKV_ERR_HIP;
    DeviceScope dev(cfg->device_id);
    if (!dev.ok) return MUKV_ERR_HIP;

    {
        void *unused = nullptr; // the static scratch's address on this device, resolved once here
        if (static_scratch(cfg->device_id, &unused) != hipSuccess) return MUKV_ERR_HIP;
    }
    mukv_ctx *h = new (std::nothrow) mukv_ctx();
    if (!h) return MUKV_ERR_HIP;
    Ctx &c = h->c;
    std::memset(&c, 0, sizeof(c));
    c.cfg = *cfg;
    c.kappa = (int)std::floor(cfg->keep_ratio * cfg->tokens_per_frame + 1e-9);
    c.ls = cfg->score_layer < 0 ? cfg->n_layers - 1 : cfg->score_layer;
    c.c_kv = cfg->n_kv_heads * cfg->head_dim;
    c.group = cfg->n_q_heads / cfg->n_kv_heads;
    c.esz = cfg->dtype == MUKV_BF16 ? 2 : 4;
    c.max_segments = (cfg->max_frames + cfg->frames_per_segment - 1) / cfg->frames_per_segment;
    c.use_mfma = cfg->att_path != MUKV_ATT_GENERIC && mfma_supported(*cfg);
    c.margin_thr = cfg->refine_margin < 0.0 ? kDefaultRefineMargin : cfg->refine_margin;
    c.n_frames = 0;
    c.n_done = 0;
    c.batch_chunks = cfg->batch_chunks < 1 ? 1 : cfg->batch_chunks;
    c.max_batch_frames = c.batch_chunks * cfg->max_chunk_frames;
    c.pending = new (std::nothrow) std::vector<mukv::PendingChunk>();
    c.p_stream = nullptr;
    c.store_cap = (int64_t)cfg->max_frames * c.kappa;
    c.profiling = false;
    c.prof = new (std::nothrow) std::vector<mukv::ProfEntry>();

    const size_t store_bytes = (size_t)cfg->n_layers * cfg->n_kv_heads * c.store_cap * cfg->head_dim * c.esz;
    const size_t MF = cfg->max_frames, C = c.c_kv, S = cfg->superpatches_per_frame, P = cfg->tokens_per_frame;
    const size_t MC = c.max_batch_frames, MQ = cfg->max_questions, Hq = cfg->n_q_heads;
    hipError_t e = hipSuccess;
    auto ok = [&](hipError_t r) {
        if (e == hipSuccess) e = r;
    };
    ok(dalloc(reinterpret_cast<unsigned char **>(&c.store_k), store_bytes));
    ok(dalloc(reinterpret_cast<unsigned char **>(&c.store_v), store_bytes));
    ok(dalloc(&c.kept_idx, MF * c.kappa));
    ok(dalloc(&c.rep_frame_k, MF * C));
    ok(dalloc(&c.rep_frame_v, MF * C));
    ok(dalloc(&c.rep_patch_k, MF * S * C));
    ok(dalloc(&c.rep_patch_v, MF * S * C));
    ok(dalloc(&c.rep_seg_k, (size_t)c.max_segments * C));
    ok(dalloc(&c.rep_seg_v, (size_t)c.max_segments * C));
    ok(dalloc(&c.cnt_patch, MF * S));
    ok(dalloc(&c.fsum_k, MF * C));
    ok(dalloc(&c.fsum_v, MF * C));
    ok(dalloc(&c.ssum_k, (size_t)c.max_segments * C));
    ok(dalloc(&c.ssum_v, (size_t)c.max_segments * C));
    ok(dalloc(&c.margin, MF));
    ok(dalloc(&c.refined, MF));
    // partial rows per frame; none for a unit of several frames, whose attention signal is the caller's
    const size_t n_part_max = P > (size_t)mukv::kMaxP ? 0 : Hq * ((P + 31) / 32 > 2 ? (P + 31) / 32 : 2);
    for (int par = 0; par < 2; ++par) {
        ok(dalloc(&c.att_part[par], MC * n_part_max * P));
        ok(dalloc(&c.fft_sig[par], MC * P * (c.use_mfma ? (size_t)cfg->n_kv_heads : 1)));
        ok(dalloc(&c.src_tok[par], MC * c.kappa));
        ok(hipEventCreateWithFlags(&c.ev_join[par], hipEventDisableTiming));
    }
    if (c.use_mfma && cfg->freq_axis == MUKV_FREQ_FEATURE) {
        const std::vector<uint16_t> tab = mukv::dft_operand_table();
        ok(dalloc(&c.dft_tab, tab.size()));
        if (e == hipSuccess) ok(hipMemcpy(c.dft_tab, tab.data(), tab.size() * sizeof(uint16_t), hipMemcpyHostToDevice));
    }
    ok(dalloc(&c.att64, MC * n_part_max * P));
    ok(dalloc(&c.fft64, MC * P));
    ok(dalloc(&c.src_tok2, MC * c.kappa));
    ok(dalloc(&c.flag_list[0], MC));
    ok(dalloc(&c.flag_list[1], MC));
    ok(dalloc(&c.flag_count, 2));
    if (e == hipSuccess) ok(hipMemset(c.flag_count, 0, 2 * sizeof(int32_t)));
    ok(hipStreamCreateWithFlags(&c.side, hipStreamNonBlocking));
    c.split_side = cfg->overlap_copy != 0 && cfg->tokens_per_frame <= mukv::kMaxP;
    if (c.split_side)
        for (int par = 0; par < 2; ++par) ok(hipEventCreateWithFlags(&c.ev_keep[par], hipEventDisableTiming));
    ok(hipEventCreateWithFlags(&c.ev_fork, hipEventDisableTiming));
    c.deferred = new (std::nothrow) mukv::ChunkArgs[2];
    ok(hipEventCreateWithFlags(&c.ev_copy, hipEventDisableTiming));
    ok(dalloc(&c.qbar, MQ * C));
    ok(dalloc(&c.qq, MQ * cfg->n_kv_heads * (size_t)(cfg->head_dim / mukv::pool_slice(c.group, cfg->head_dim))));
    ok(dalloc(&c.s_frm, MQ * MF * S)); // room for the super-patch level
    ok(dalloc(&c.s_seg, MQ * (size_t)c.max_segments));
    ok(dalloc(&c.seg_tail, MQ * C));
    ok(dalloc(&c.u_mask, MQ * MF));
    ok(dalloc(&c.u_entry, MQ * MF * 3));
    ok(dalloc(&c.u_count, MQ * 2));
    ok(dalloc(&c.m_entry, MQ * (size_t)mukv::kMaxMultiEntries * 3));
    ok(dalloc(&c.m_count, MQ * 2));
    ok(dalloc(&c.attend_part, MQ * mukv::kAttendMaxTokens * cfg->n_q_heads * mukv::kAttendMaxSplit * (size_t)(cfg->head_dim + 2)));
    if (cfg->freq_axis == MUKV_FREQ_TOKEN) {
        // rows 0..P/2 of the DFT matrix over the frame's tokens, columns 0..P/2 (the others mirror
        // them), as (cos, -sin) pairs, rounded once from double for the fp32 pass.  The sine of
        // column 0 and, for even P, of column P/2 is exactly zero.
        const int P = cfg->tokens_per_frame, hc = P / 2 + 1;
        std::vector<double> t64((size_t)hc * hc * 2);
        std::vector<float> t32(t64.size());
        for (int m = 0; m < hc; ++m)
            for (int j = 0; j < hc; ++j) {
                const int r = (int)(((int64_t)m * j) % P);
                const double ang = 2.0 * 3.14159265358979323846 * (double)r / (double)P;
                t64[((size_t)m * hc + j) * 2] = std::cos(ang);
                t64[((size_t)m * hc + j) * 2 + 1] = (j == 0 || 2 * j == P) ? 0.0 : -std::sin(ang);
            }
        for (size_t i = 0; i < t64.size(); ++i) t32[i] = (float)t64[i];
        ok(dalloc(&c.tw32, t32.size()));
        ok(dalloc(&c.tw64, t64.size()));
        if (e == hipSuccess) ok(hipMemcpy(c.tw32, t32.data(), t32.size() * sizeof(float), hipMemcpyHostToDevice));
        if (e == hipSuccess) ok(hipMemcpy(c.tw64, t64.data(), t64.size() * sizeof(double), hipMemcpyHostToDevice));
        const size_t n_groups = ((size_t)cfg->n_kv_heads * cfg->head_dim + 63) / 64;
        c.tok_part_half = (size_t)c.max_batch_frames * n_groups * hc * sizeof(float);
        c.tok_part_half = (c.tok_part_half + 255) & ~(size_t)255;
        ok(dalloc(&c.tok_part, c.tok_part_half + (size_t)c.max_batch_frames * n_groups * hc * sizeof(double)));
    }
    if (e != hipSuccess || !c.prof || !c.pending || !c.deferred) {
        free_all(c);
        delete c.prof;
        delete c.pending;
        delete h;
        (void)hipGetLastError();
        return MUKV_ERR_HIP;
    }
    *out = h;
    return MUKV_OK;
}

int mukv_destroy(mukv_ctx *ctx) {
    if (!ctx) return MUKV_OK;
    DeviceScope dev(ctx->c.cfg.device_id);
    free_all(ctx->c);
    if (ctx->c.prof) {
        for (auto &p : *ctx->c.prof) {
            (void)hipEventDestroy(p.start);
            (void)hipEventDestroy(p.stop);
        }
        delete ctx->c.prof;
    }
    delete ctx->c.pending;
    delete ctx;
    return MUKV_OK;
}

int mukv_profile_begin(mukv_ctx *ctx) {
    if (!ctx) return MUKV_ERR_INVALID_ARG;
    ctx->c.profiling = true;
    return MUKV_OK;
}

int mukv_profile_end(mukv_ctx *ctx, mukv_profile *out) {
    if (!ctx || !out) return MUKV_ERR_INVALID_ARG;
    Ctx &c = ctx->c;
    c.profiling = false;
    std::memset(out, 0, sizeof(*out));
    int rc = MUKV_OK;
    for (auto &p : *c.prof) {
        float ms = 0.f;
        if (hipEventSynchronize(p.stop) != hipSuccess || hipEventElapsedTime(&ms, p.start, p.stop) != hipSuccess)
            rc = MUKV_ERR_HIP;
        out->ms[p.kid] += (double)ms;
        out->launches[p.kid] += 1;
        (void)hipEventDestroy(p.start);
        (void)hipEventDestroy(p.stop);
    }
    c.prof->clear();
    return rc;
}

int mukv_reset(mukv_ctx *ctx) {
    if (!ctx) return MUKV_ERR_INVALID_ARG;
    ctx->c.n_frames = 0;
    ctx->c.n_done = 0;
    ctx->c.pending->clear();
    if (ctx->c.n_deferred) { // the rows they would have copied are forgotten with the rest
        DeviceScope dev(ctx->c.cfg.device_id);
        if (!dev.ok || mukv::drop_deferred(ctx->c) != hipSuccess) return MUKV_ERR_HIP;
    }
    return MUKV_OK;
}

// Chunks that make the next batch.  (Shorter first batches -- they have no copy to run beside yet -- were
// measured on the 1-hour stream: 1/4, 3/8 and 1/2 of batch_chunks for the first two took 3.70, 3.67 and 3.67 ms
// per step against 3.64 with every batch alike.)
static int batch_limit(const Ctx &c) { return c.batch_chunks; }

// Enqueues the kernels for every chunk gathered so far (on the stream they were submitted with).
// join: also order `join_stream` after the work outstanding on the library's own streams.
static int flush_pending(Ctx &c, bool join, hipStream_t join_stream) {
    if (c.pending->empty()) {
        if (!join) return MUKV_OK;
        DeviceScope dev(c.cfg.device_id);
        if (!dev.ok) return MUKV_ERR_HIP;
        return mukv::join_streams(c, join_stream) == hipSuccess ? MUKV_OK : MUKV_ERR_HIP;
    }
    mukv::ChunkArgs a;
    std::memset(&a, 0, sizeof(a));
    int nf = 0, s = 0;
    for (const mukv::PendingChunk &pc : *c.pending) {
        a.k.p[s] = pc.k;
        a.v.p[s] = pc.v;
        a.q.p[s] = pc.q;
        a.att_in.p[s] = pc.att_in;
        a.dbg_att.p[s] = pc.sig.att;
        a.dbg_fft.p[s] = pc.sig.fft;
        a.dbg_fused.p[s] = pc.sig.fused;
        a.have_dbg = a.have_dbg || pc.sig.att || pc.sig.fft || pc.sig.fused;
        a.map.fstart[s] = nf;
        nf += pc.n_frames;
        ++s;
    }
    a.map.fstart[s] = nf;
    a.map.n_slots = s;
    a.have_q = c.pending->front().q != nullptr;
    a.have_att_in = c.pending->front().att_in != nullptr;
    a.kv_sl = c.p_kv_sl;
    a.kv_sh = c.p_kv_sh;
    a.kv_st = c.p_kv_st;
    a.q_sh = c.p_q_sh;
    a.q_st = c.p_q_st;
    a.n_frames = nf;
    a.frame0 = c.n_done;
    a.parity = c.batch_parity;
    c.batch_parity ^= 1;
    c.pending->clear();
    c.n_done += nf;
    DeviceScope dev(c.cfg.device_id);
    if (!dev.ok) return MUKV_ERR_HIP;
    if (mukv::launch_compress(c, a, c.p_stream) != hipSuccess) return MUKV_ERR_HIP;
    if (join && mukv::join_streams(c, join_stream) != hipSuccess) return MUKV_ERR_HIP;
    return MUKV_OK;
}

int mukv_flush(mukv_ctx *ctx) {
    if (!ctx) return MUKV_ERR_INVALID_ARG;
    return flush_pending(ctx->c, true, ctx->c.p_stream);
}

int mukv_compress_chunk(mukv_ctx *ctx, const void *k, const void *v, const mukv_strides *kv_strides,
                        const void *q_last, const mukv_strides *q_strides, const float *att_signal,
                        int32_t n_frames, void *stream, const mukv_signals_out *sig) {
    if (!ctx || !k || !v || !kv_strides) return MUKV_ERR_INVALID_ARG;
    Ctx &c = ctx->c;
    if (c.cfg.alpha != 0.0) {
        if ((q_last != nullptr) == (att_signal != nullptr)) return MUKV_ERR_INVALID_ARG;
        if (q_last && !q_strides) return MUKV_ERR_INVALID_ARG;
    }
    if (c.cfg.tokens_per_frame > mukv::kMaxP && c.cfg.alpha != 0.0 && !att_signal) return MUKV_ERR_UNSUPPORTED;
    if (n_frames < 1) return MUKV_ERR_SHAPE;
    if (n_frames > c.cfg.max_chunk_frames) return MUKV_ERR_CAPACITY;
    if (c.n_frames + n_frames > c.cfg.max_frames) return MUKV_ERR_CAPACITY;
    const int64_t D = c.cfg.head_dim;
    if (kv_strides->token < D || kv_strides->head < 0 || kv_strides->layer < 0) return MUKV_ERR_SHAPE;
    const int64_t unit = 16 / c.esz; // elements per 16 bytes
    if (kv_strides->token % unit || kv_strides->head % unit || kv_strides->layer % unit ||
        (reinterpret_cast<uintptr_t>(k) & 15) || (reinterpret_cast<uintptr_t>(v) & 15))
        return MUKV_ERR_UNSUPPORTED;
    int64_t q_sh = 0, q_st = 0;
    const bool use_q = c.cfg.alpha != 0.0 && q_last;
    if (use_q) {
        if (q_strides->token < D || q_strides->head < 0) return MUKV_ERR_SHAPE;
        if (q_strides->token % unit || q_strides->head % unit || (reinterpret_cast<uintptr_t>(q_last) & 15))
            return MUKV_ERR_UNSUPPORTED;
        if (q_strides->token * c.esz >= (int64_t)1 << 24) return MUKV_ERR_UNSUPPORTED; // 24-bit offset arithmetic
        q_sh = q_strides->head;
        q_st = q_strides->token;
    }
    hipStream_t st = reinterpret_cast<hipStream_t>(stream);
    const bool use_att_in = c.cfg.alpha != 0.0 && att_signal;
    if (!c.pending->empty()) {
        // a batch shares one stream, one set of strides and one attention source
        const mukv::PendingChunk &p0 = c.pending->front();
        const bool same = c.p_stream == st && c.p_kv_sl == kv_strides->layer && c.p_kv_sh == kv_strides->head &&
                          c.p_kv_st == kv_strides->token && c.p_q_sh == q_sh && c.p_q_st == q_st &&
                          (p0.q != nullptr) == use_q && (p0.att_in != nullptr) == use_att_in;
        if (!same) {
            const int rc = flush_pending(c, true, c.p_stream);
            if (rc != MUKV_OK) return rc;
        }
    }
    mukv::PendingChunk pc;
    pc.k = k;
    pc.v = v;
    pc.q = use_q ? q_last : nullptr;
    pc.att_in = use_att_in ? att_signal : nullptr;
    pc.sig = mukv_signals_out{nullptr, nullptr, nullptr};
    if (sig) pc.sig = *sig;
    pc.n_frames = n_frames;
    c.p_stream = st;
    c.p_kv_sl = kv_strides->layer;
    c.p_kv_sh = kv_strides->head;
    c.p_kv_st = kv_strides->token;
    c.p_q_sh = q_sh;
    c.p_q_st = q_st;
    c.pending->push_back(pc);
    c.n_frames += n_frames;
    if ((int)c.pending->size() >= batch_limit(c)) return flush_pending(c, false, nullptr);
    return MUKV_OK;
}

static int retrieve_any(mukv_ctx *ctx, const void *q_tokens, const int32_t *q_offsets, const int32_t *n_visible, int32_t B,
                        const mukv_retrieve_params *params, bool patches, int32_t *seg_idx_out, float *seg_score_out,
                        int32_t *fine_idx_out, float *fine_score_out, void *stream) {
    if (!ctx || !q_tokens || !q_offsets || !params || !fine_idx_out) return MUKV_ERR_INVALID_ARG;
    Ctx &c = ctx->c;
    if (B < 1) return MUKV_ERR_INVALID_ARG;
    if (B > c.cfg.max_questions) return MUKV_ERR_CAPACITY;
    if (params->mode < MUKV_SEMI || params->mode > MUKV_PARALLEL) return MUKV_ERR_INVALID_ARG;
    if (params->k_seg < 1 || params->k_frame < 1 || params->n_global < 0) return MUKV_ERR_INVALID_ARG;
    if (!(params->lambda_frame >= 0.0) || params->lambda_frame > 1.0) return MUKV_ERR_INVALID_ARG;
    if (2 * params->k_seg > mukv::kMaxCand || 2 * params->k_frame > mukv::kMaxCand) return MUKV_ERR_UNSUPPORTED;
    {
        const int rc = flush_pending(c, true, reinterpret_cast<hipStream_t>(stream));
        if (rc != MUKV_OK) return rc;
    }
    mukv::RetrieveArgs a;
    a.q_tokens = q_tokens;
    a.q_offsets = q_offsets;
    a.B = B;
    a.p = *params;
    int64_t nv = params->n_visible_frames < 0 ? c.n_frames : params->n_visible_frames;
    if (nv > c.n_frames || n_visible) nv = c.n_frames; // per-question timestamps: every ingested frame is scored
    a.nv_q = n_visible;
    a.nv = (int)nv;
    a.ns = (int)((nv + c.cfg.frames_per_segment - 1) / c.cfg.frames_per_segment);
    a.patches = patches;
    a.units = 0;
    a.g_in = nullptr;
    a.g_out = nullptr;
    a.seg_idx = seg_idx_out;
    a.seg_score = seg_score_out;
    a.frm_idx = fine_idx_out;
    a.frm_score = fine_score_out;
    DeviceScope dev(c.cfg.device_id);
    if (!dev.ok) return MUKV_ERR_HIP;
    return mukv::launch_retrieve(c, a, reinterpret_cast<hipStream_t>(stream)) == hipSuccess ? MUKV_OK : MUKV_ERR_HIP;
}

int mukv_retrieve(mukv_ctx *ctx, const void *q_tokens, const int32_t *q_offsets, int32_t B,
                  const mukv_retrieve_params *params, int32_t *seg_idx_out, float *seg_score_out,
                  int32_t *frame_idx_out, float *frame_score_out, void *stream) {
    if (!seg_idx_out) return MUKV_ERR_INVALID_ARG;
    return retrieve_any(ctx, q_tokens, q_offsets, nullptr, B, params, false, seg_idx_out, seg_score_out, frame_idx_out,
                        frame_score_out, stream);
}

int mukv_retrieve_patches(mukv_ctx *ctx, const void *q_tokens, const int32_t *q_offsets, int32_t B,
                          const mukv_retrieve_params *params, int32_t *patch_idx_out, float *patch_score_out,
                          void *stream) {
    return retrieve_any(ctx, q_tokens, q_offsets, nullptr, B, params, true, nullptr, nullptr, patch_idx_out,
                        patch_score_out, stream);
}

int mukv_retrieve_at(mukv_ctx *ctx, const void *q_tokens, const int32_t *q_offsets, const int32_t *n_visible, int32_t B,
                     const mukv_retrieve_params *params, int32_t level, int32_t *seg_idx_out, float *seg_score_out,
                     int32_t *fine_idx_out, float *fine_score_out, void *stream) {
    if (!n_visible || (level != 0 && level != 1)) return MUKV_ERR_INVALID_ARG;
    return retrieve_any(ctx, q_tokens, q_offsets, n_visible, B, params, level == 1, seg_idx_out, seg_score_out, fine_idx_out,
                        fine_score_out, stream);
}

int mukv_gather_patches(mukv_ctx *ctx, const int32_t *patch_idx, int32_t B, int32_t k_patch, int32_t order,
                        void *k_out, void *v_out, int32_t *n_tokens_out, void *stream) {
    if (!ctx || !patch_idx || !k_out || !v_out) return MUKV_ERR_INVALID_ARG;
    Ctx &c = ctx->c;
    if (B < 1 || k_patch < 1) return MUKV_ERR_INVALID_ARG;
    if (order != MUKV_TEMPORAL && order != MUKV_AS_GIVEN) return MUKV_ERR_INVALID_ARG;
    if (B > c.cfg.max_questions) return MUKV_ERR_CAPACITY;
    if (k_patch > mukv::kMaxGatherK) return MUKV_ERR_UNSUPPORTED;
    if ((reinterpret_cast<uintptr_t>(k_out) & 15) || (reinterpret_cast<uintptr_t>(v_out) & 15))
        return MUKV_ERR_UNSUPPORTED;
    {
        const int rc = flush_pending(c, true, reinterpret_cast<hipStream_t>(stream));
        if (rc != MUKV_OK) return rc;
    }
    DeviceScope dev(c.cfg.device_id);
    if (!dev.ok) return MUKV_ERR_HIP;
    return mukv::launch_gather_patches(c, patch_idx, B, k_patch, order, k_patch * patch_cap(c), k_out, v_out,
                                       n_tokens_out, reinterpret_cast<hipStream_t>(stream)) == hipSuccess
               ? MUKV_OK
               : MUKV_ERR_HIP;
}

int mukv_retrieve_units(mukv_ctx *ctx, const void *q_tokens, const int32_t *q_offsets, int32_t B, int32_t k,
                        double lambda_g, int32_t n_visible_units, const double *global_query_in, int32_t n_global,
                        double *global_query_out, int32_t *idx_out, float *score_out, void *stream) {
    if (!ctx || !q_tokens || !q_offsets || !idx_out) return MUKV_ERR_INVALID_ARG;
    Ctx &c = ctx->c;
    if (B < 1 || k < 1 || n_global < 0) return MUKV_ERR_INVALID_ARG;
    if (!(lambda_g >= 0.0) || lambda_g > 1.0) return MUKV_ERR_INVALID_ARG;
    if (global_query_in && global_query_out) return MUKV_ERR_INVALID_ARG; // a store either supplies the global query or takes it
    if (B > c.cfg.max_questions) return MUKV_ERR_CAPACITY;
    if (2 * k > mukv::kMaxCand) return MUKV_ERR_UNSUPPORTED;
    if ((reinterpret_cast<uintptr_t>(global_query_in) & 7) || (reinterpret_cast<uintptr_t>(global_query_out) & 7))
        return MUKV_ERR_UNSUPPORTED;
    {
        const int rc = flush_pending(c, true, reinterpret_cast<hipStream_t>(stream));
        if (rc != MUKV_OK) return rc;
    }
    mukv::RetrieveArgs a;
    a.q_tokens = q_tokens;
    a.q_offsets = q_offsets;
    a.B = B;
    a.p.mode = MUKV_SEMI;
    a.p.k_seg = 1;
    a.p.k_frame = k;
    a.p.n_global = n_global;
    a.p.n_visible_frames = n_visible_units;
    a.p.lambda_frame = lambda_g;
    int64_t nv = n_visible_units < 0 ? c.n_frames : n_visible_units;
    if (nv > c.n_frames) nv = c.n_frames;
    a.nv_q = nullptr;
    a.nv = (int)nv;
    a.ns = 0; // the blocks are this store's units; its own segment level takes no part
    a.patches = false;
    a.units = global_query_in ? 2 : 1;
    a.g_in = global_query_in;
    a.g_out = global_query_out;
    a.seg_idx = nullptr;
    a.seg_score = nullptr;
    a.frm_idx = idx_out;
    a.frm_score = score_out;
    DeviceScope dev(c.cfg.device_id);
    if (!dev.ok) return MUKV_ERR_HIP;
    return mukv::launch_retrieve(c, a, reinterpret_cast<hipStream_t>(stream)) == hipSuccess ? MUKV_OK : MUKV_ERR_HIP;
}

int mukv_gather_multi(mukv_ctx *const *ctxs, int32_t n_ctx, const int32_t *const *unit_idx, const int32_t *k,
                      const int32_t *units_per_step, int32_t B, int32_t rows_cap, void *k_out, void *v_out,
                      int32_t *n_tokens_out, void *stream) {
    if (!ctxs || !unit_idx || !k || !units_per_step || !k_out || !v_out) return MUKV_ERR_INVALID_ARG;
    if (n_ctx < 1 || n_ctx > mukv::kMaxStores || B < 1 || rows_cap < 1) return MUKV_ERR_INVALID_ARG;
    int64_t total = 0;
    for (int i = 0; i < n_ctx; ++i) {
        if (!ctxs[i] || k[i] < 0 || units_per_step[i] < 1 || (k[i] > 0 && !unit_idx[i])) return MUKV_ERR_INVALID_ARG;
        total += k[i];
    }
    if (total > mukv::kMaxMultiEntries) return MUKV_ERR_UNSUPPORTED;
    Ctx &c0 = ctxs[0]->c;
    if (B > c0.cfg.max_questions) return MUKV_ERR_CAPACITY;
    for (int i = 1; i < n_ctx; ++i) { // one decode context: the stores hold rows of one model on one device
        const mukv_config &x = ctxs[i]->c.cfg;
        if (x.n_layers != c0.cfg.n_layers || x.n_kv_heads != c0.cfg.n_kv_heads || x.head_dim != c0.cfg.head_dim ||
            x.dtype != c0.cfg.dtype)
            return MUKV_ERR_SHAPE;
        if (x.device_id != c0.cfg.device_id) return MUKV_ERR_UNSUPPORTED;
    }
    if ((reinterpret_cast<uintptr_t>(k_out) & 15) || (reinterpret_cast<uintptr_t>(v_out) & 15)) return MUKV_ERR_UNSUPPORTED;
    hipStream_t st = reinterpret_cast<hipStream_t>(stream);
    for (int i = 0; i < n_ctx; ++i) {
        const int rc = flush_pending(ctxs[i]->c, true, st);
        if (rc != MUKV_OK) return rc;
    }
    mukv::MultiArgs a;
    a.n_ctx = n_ctx;
    for (int i = 0; i < n_ctx; ++i) {
        a.c[i] = &ctxs[i]->c;
        a.idx[i] = k[i] > 0 ? unit_idx[i] : nullptr;
        a.k[i] = k[i];
        a.ups[i] = units_per_step[i];
    }
    a.B = B;
    a.rows_cap = rows_cap;
    a.k_out = k_out;
    a.v_out = v_out;
    a.n_tokens_out = n_tokens_out;
    DeviceScope dev(c0.cfg.device_id);
    if (!dev.ok) return MUKV_ERR_HIP;
    return mukv::launch_gather_multi(a, st) == hipSuccess ? MUKV_OK : MUKV_ERR_HIP;
}

int mukv_gather_kv(mukv_ctx *ctx, const int32_t *frame_idx, int32_t B, int32_t k_frame, int32_t order,
                   void *k_out, void *v_out, int32_t *n_tokens_out, void *stream) {
    if (!ctx || !frame_idx || !k_out || !v_out) return MUKV_ERR_INVALID_ARG;
    Ctx &c = ctx->c;
    if (B < 1 || k_frame < 1) return MUKV_ERR_INVALID_ARG;
    if (order != MUKV_TEMPORAL && order != MUKV_AS_GIVEN) return MUKV_ERR_INVALID_ARG;
    if (B > c.cfg.max_questions) return MUKV_ERR_CAPACITY;
    if (k_frame > mukv::kMaxGatherK) return MUKV_ERR_UNSUPPORTED;
    if ((reinterpret_cast<uintptr_t>(k_out) & 15) || (reinterpret_cast<uintptr_t>(v_out) & 15))
        return MUKV_ERR_UNSUPPORTED;
    {
        const int rc = flush_pending(c, true, reinterpret_cast<hipStream_t>(stream));
        if (rc != MUKV_OK) return rc;
    }
    DeviceScope dev(c.cfg.device_id);
    if (!dev.ok) return MUKV_ERR_HIP;
    return mukv::launch_gather(c, frame_idx, B, k_frame, order, k_out, v_out, n_tokens_out,
                               reinterpret_cast<hipStream_t>(stream)) == hipSuccess
               ? MUKV_OK
               : MUKV_ERR_HIP;
}

int mukv_attend(mukv_ctx *ctx, int32_t layer, const void *q, int32_t n_q, const int32_t *frame_idx, int32_t k_frame,
                const void *k_local, const void *v_local, const int32_t *local_offsets, int32_t B, int32_t causal_local,
                void *out, void *stream) {
    if (!ctx || !q || !out) return MUKV_ERR_INVALID_ARG;
    Ctx &c = ctx->c;
    if (B < 1 || n_q < 1 || k_frame < 0 || layer < 0 || layer >= c.cfg.n_layers) return MUKV_ERR_INVALID_ARG;
    if (causal_local != 0 && causal_local != 1) return MUKV_ERR_INVALID_ARG;
    if (k_frame > 0 && !frame_idx) return MUKV_ERR_INVALID_ARG;
    const int n_local_args = (k_local != nullptr) + (v_local != nullptr) + (local_offsets != nullptr);
    if (n_local_args != 0 && n_local_args != 3) return MUKV_ERR_INVALID_ARG;
    if (B > c.cfg.max_questions) return MUKV_ERR_CAPACITY;
    if (n_q > mukv::kAttendMaxTokens || k_frame > mukv::kMaxGatherK) return MUKV_ERR_UNSUPPORTED;
    if ((reinterpret_cast<uintptr_t>(q) & 15) || (reinterpret_cast<uintptr_t>(out) & 15) ||
        (reinterpret_cast<uintptr_t>(k_local) & 15) || (reinterpret_cast<uintptr_t>(v_local) & 15))
        return MUKV_ERR_UNSUPPORTED;
    {
        const int rc = flush_pending(c, true, reinterpret_cast<hipStream_t>(stream));
        if (rc != MUKV_OK) return rc;
    }
    DeviceScope dev(c.cfg.device_id);
    if (!dev.ok) return MUKV_ERR_HIP;
    return mukv::launch_attend(c, layer, q, n_q, frame_idx, k_frame, k_local, v_local, local_offsets, B, causal_local, out,
                               nullptr, nullptr, reinterpret_cast<hipStream_t>(stream)) == hipSuccess
               ? MUKV_OK
               : MUKV_ERR_HIP;
}

static int prefill_shape_check(const Ctx &c, int32_t n_q, int32_t k_frame, int32_t B) {
    if (B < 1 || n_q < 1 || k_frame < 0) return MUKV_ERR_INVALID_ARG;
    if (B > c.cfg.max_questions) return MUKV_ERR_CAPACITY;
    if (n_q > mukv::kPrefillMaxTokens || k_frame > mukv::kMaxGatherK) return MUKV_ERR_UNSUPPORTED;
    // grid limits: (KV head, query tile) pairs along y, one merge workgroup per (question, token, head) along x
    const int64_t n_qtiles = ((int64_t)n_q * c.group + 7) / 8;
    if (n_qtiles * c.cfg.n_kv_heads > 65535 || (int64_t)B * n_q * c.cfg.n_q_heads > 0x7fffffff) return MUKV_ERR_UNSUPPORTED;
    return MUKV_OK;
}

int mukv_prefill_workspace_size(const mukv_ctx *ctx, int32_t n_q, int32_t k_frame, int32_t B, int64_t *bytes_out) {
    if (!ctx || !bytes_out) return MUKV_ERR_INVALID_ARG;
    const int rc = prefill_shape_check(ctx->c, n_q, k_frame, B);
    if (rc != MUKV_OK) return rc;
    *bytes_out = mukv::prefill_workspace_bytes(ctx->c, n_q, B, k_frame);
    return MUKV_OK;
}

int mukv_prefill_attend(mukv_ctx *ctx, int32_t layer, const void *q, int32_t n_q, const int32_t *frame_idx,
                        int32_t k_frame, const void *k_local, const void *v_local, const int32_t *local_offsets,
                        int32_t B, int32_t causal_local, void *out, float *att_signal_out, void *workspace,
                        int64_t workspace_bytes, void *stream) {
    if (!ctx || !q || !out || !att_signal_out || !workspace || !k_local || !v_local || !local_offsets)
        return MUKV_ERR_INVALID_ARG;
    Ctx &c = ctx->c;
    if (layer < 0 || layer >= c.cfg.n_layers) return MUKV_ERR_INVALID_ARG;
    if (causal_local != 0 && causal_local != 1) return MUKV_ERR_INVALID_ARG;
    if (k_frame > 0 && !frame_idx) return MUKV_ERR_INVALID_ARG;
    const int rc0 = prefill_shape_check(c, n_q, k_frame, B);
    if (rc0 != MUKV_OK) return rc0;
    if (workspace_bytes < mukv::prefill_workspace_bytes(c, n_q, B, k_frame)) return MUKV_ERR_CAPACITY;
    if ((reinterpret_cast<uintptr_t>(q) & 15) || (reinterpret_cast<uintptr_t>(out) & 15) ||
        (reinterpret_cast<uintptr_t>(k_local) & 15) || (reinterpret_cast<uintptr_t>(v_local) & 15) ||
        (reinterpret_cast<uintptr_t>(workspace) & 15))
        return MUKV_ERR_UNSUPPORTED;
    {
        const int rc = flush_pending(c, true, reinterpret_cast<hipStream_t>(stream));
        if (rc != MUKV_OK) return rc;
    }
    DeviceScope dev(c.cfg.device_id);
    if (!dev.ok) return MUKV_ERR_HIP;
    return mukv::launch_attend(c, layer, q, n_q, frame_idx, k_frame, k_local, v_local, local_offsets, B, causal_local, out,
                               att_signal_out, static_cast<float *>(workspace),
                               reinterpret_cast<hipStream_t>(stream)) == hipSuccess
               ? MUKV_OK
               : MUKV_ERR_HIP;
}

int mukv_prefill_attend_static(mukv_ctx *ctx, int32_t layer, const void *q, int32_t n_q, const int32_t *frame_idx,
                               int32_t k_frame, const void *k_local, const void *v_local, const int32_t *local_offsets,
                               int32_t B, int32_t causal_local, void *out, float *att_signal_out, void *stream) {
    if (!ctx || !q || !out || !att_signal_out || !k_local || !v_local || !local_offsets) return MUKV_ERR_INVALID_ARG;
    Ctx &c = ctx->c;
    if (layer < 0 || layer >= c.cfg.n_layers) return MUKV_ERR_INVALID_ARG;
    if (causal_local != 0 && causal_local != 1) return MUKV_ERR_INVALID_ARG;
    if (k_frame > 0 && !frame_idx) return MUKV_ERR_INVALID_ARG;
    const int rc0 = prefill_shape_check(c, n_q, k_frame, B);
    if (rc0 != MUKV_OK) return rc0;
    if (mukv::prefill_workspace_bytes(c, n_q, B, k_frame) > (int64_t)MUKV_STATIC_SCRATCH_BYTES) return MUKV_ERR_CAPACITY;
    if ((reinterpret_cast<uintptr_t>(q) & 15) || (reinterpret_cast<uintptr_t>(out) & 15) ||
        (reinterpret_cast<uintptr_t>(k_local) & 15) || (reinterpret_cast<uintptr_t>(v_local) & 15))
        return MUKV_ERR_UNSUPPORTED;
    {
        const int rc = flush_pending(c, true, reinterpret_cast<hipStream_t>(stream));
        if (rc != MUKV_OK) return rc;
    }
    DeviceScope dev(c.cfg.device_id);
    if (!dev.ok) return MUKV_ERR_HIP;
    void *ws = nullptr; // this device's copy of the array (resolved at mukv_create; a look-up here)
    if (static_scratch(c.cfg.device_id, &ws) != hipSuccess) return MUKV_ERR_HIP;
    // every float of the scratch that a kernel of this call reads was written by an earlier kernel of
    // the same call, so what the previous call left behind needs no clearing
    return mukv::launch_attend(c, layer, q, n_q, frame_idx, k_frame, k_local, v_local, local_offsets, B, causal_local, out,
                               att_signal_out, static_cast<float *>(ws), reinterpret_cast<hipStream_t>(stream)) == hipSuccess
               ? MUKV_OK
               : MUKV_ERR_HIP;
}

int mukv_gather_union(mukv_ctx *ctx, const int32_t *seg_idx, int32_t k_seg, const int32_t *frame_idx, int32_t k_frame,
                      const int32_t *patch_idx, int32_t k_patch, int32_t B, int32_t rows_cap, void *k_out, void *v_out,
                      int32_t *n_tokens_out, void *stream) {
    if (!ctx || !k_out || !v_out) return MUKV_ERR_INVALID_ARG;
    Ctx &c = ctx->c;
    if (B < 1 || rows_cap < 1 || k_seg < 0 || k_frame < 0 || k_patch < 0) return MUKV_ERR_INVALID_ARG;
    if (k_seg > 65536 || k_frame > (1 << 24) || k_patch > (1 << 24)) return MUKV_ERR_UNSUPPORTED;
    if ((k_seg > 0 && !seg_idx) || (k_frame > 0 && !frame_idx) || (k_patch > 0 && !patch_idx)) return MUKV_ERR_INVALID_ARG;
    if (B > c.cfg.max_questions) return MUKV_ERR_CAPACITY;
    if (c.cfg.superpatches_per_frame > 32) return MUKV_ERR_UNSUPPORTED; // one mask bit per super-patch
    if ((reinterpret_cast<uintptr_t>(k_out) & 15) || (reinterpret_cast<uintptr_t>(v_out) & 15))
        return MUKV_ERR_UNSUPPORTED;
    {
        const int rc = flush_pending(c, true, reinterpret_cast<hipStream_t>(stream));
        if (rc != MUKV_OK) return rc;
    }
    mukv::UnionArgs a;
    a.seg_idx = k_seg > 0 ? seg_idx : nullptr;
    a.frame_idx = k_frame > 0 ? frame_idx : nullptr;
    a.patch_idx = k_patch > 0 ? patch_idx : nullptr;
    a.k_seg = k_seg;
    a.k_frame = k_frame;
    a.k_patch = k_patch;
    a.B = B;
    a.rows_cap = rows_cap;
    a.k_out = k_out;
    a.v_out = v_out;
    a.n_tokens_out = n_tokens_out;
    DeviceScope dev(c.cfg.device_id);
    if (!dev.ok) return MUKV_ERR_HIP;
    return mukv::launch_gather_union(c, a, reinterpret_cast<hipStream_t>(stream)) == hipSuccess ? MUKV_OK : MUKV_ERR_HIP;
}

int mukv_snapshot_size(const mukv_ctx *ctx, int64_t *bytes_out) {
    if (!ctx || !bytes_out) return MUKV_ERR_INVALID_ARG;
    *bytes_out = snap_bytes(ctx->c, ctx->c.n_frames);
    return MUKV_OK;
}

int mukv_snapshot_save(mukv_ctx *ctx, void *host_dst, int64_t bytes, void *stream) {
    if (!ctx || !host_dst) return MUKV_ERR_INVALID_ARG;
    Ctx &c = ctx->c;
    hipStream_t st = reinterpret_cast<hipStream_t>(stream);
    {
        const int rc = flush_pending(c, true, st);
        if (rc != MUKV_OK) return rc;
    }
    if (bytes < snap_bytes(c, c.n_frames)) return MUKV_ERR_CAPACITY;
    DeviceScope dev(c.cfg.device_id);
    if (!dev.ok) return MUKV_ERR_HIP;
    unsigned char *out = static_cast<unsigned char *>(host_dst);
    const SnapHeader h = snap_header(c);
    std::memcpy(out, &h, sizeof h);
    out += sizeof h;
    for (const SnapPiece &p : snap_pieces(c, c.n_frames))
        for (int i = 0; i < p.count; ++i) {
            if (p.bytes &&
                hipMemcpyAsync(out, static_cast<unsigned char *>(p.dev) + (size_t)i * p.stride, p.bytes,
                               hipMemcpyDeviceToHost, st) != hipSuccess)
                return MUKV_ERR_HIP;
            out += p.bytes;
        }
    return hipStreamSynchronize(st) == hipSuccess ? MUKV_OK : MUKV_ERR_HIP;
}

int mukv_snapshot_load(mukv_ctx *ctx, const void *host_src, int64_t bytes, void *stream) {
    if (!ctx || !host_src || bytes < (int64_t)sizeof(SnapHeader)) return MUKV_ERR_INVALID_ARG;
    Ctx &c = ctx->c;
    hipStream_t st = reinterpret_cast<hipStream_t>(stream);
    SnapHeader h;
    std::memcpy(&h, host_src, sizeof h);
    const SnapHeader mine = snap_header(c);
    if (std::memcmp(h.magic, mine.magic, 8) != 0) return MUKV_ERR_INVALID_ARG;
    if (h.n_layers != mine.n_layers || h.n_q_heads != mine.n_q_heads || h.n_kv_heads != mine.n_kv_heads ||
        h.head_dim != mine.head_dim || h.tokens_per_frame != mine.tokens_per_frame ||
        h.frames_per_segment != mine.frames_per_segment || h.superpatches_per_frame != mine.superpatches_per_frame ||
        h.dtype != mine.dtype || h.kappa != mine.kappa || h.score_layer != mine.score_layer)
        return MUKV_ERR_SHAPE;
    if (h.n_frames < 0 || h.n_frames > c.cfg.max_frames) return MUKV_ERR_CAPACITY;
    if (bytes < snap_bytes(c, h.n_frames)) return MUKV_ERR_INVALID_ARG;
    {
        const int rc = mukv_reset(ctx); // drops gathered chunks and a copy that was put off
        if (rc != MUKV_OK) return rc;
    }
    DeviceScope dev(c.cfg.device_id);
    if (!dev.ok) return MUKV_ERR_HIP;
    // earlier kernels of this context, on whichever stream, may still write the tables
    if (mukv::join_streams(c, st) != hipSuccess || hipDeviceSynchronize() != hipSuccess) return MUKV_ERR_HIP;
    const unsigned char *in = static_cast<const unsigned char *>(host_src) + sizeof h;
    for (const SnapPiece &p : snap_pieces(c, h.n_frames))
        for (int i = 0; i < p.count; ++i) {
            if (p.bytes &&
                hipMemcpyAsync(static_cast<unsigned char *>(p.dev) + (size_t)i * p.stride, in, p.bytes,
                               hipMemcpyHostToDevice, st) != hipSuccess)
                return MUKV_ERR_HIP;
            in += p.bytes;
        }
    if (hipStreamSynchronize(st) != hipSuccess) return MUKV_ERR_HIP;
    c.n_frames = h.n_frames;
    c.n_done = h.n_frames;
    return MUKV_OK;
}

int mukv_plain_copy(void *dst, const void *src, int64_t bytes, void *stream) {
    if (!dst || !src || bytes < 0 || (bytes & 15)) return MUKV_ERR_INVALID_ARG;
    if ((reinterpret_cast<uintptr_t>(dst) & 15) || (reinterpret_cast<uintptr_t>(src) & 15)) return MUKV_ERR_UNSUPPORTED;
    if (bytes / 16 / 1024 > 0x7fffffff) return MUKV_ERR_UNSUPPORTED;
    return mukv::launch_plain_copy(dst, src, bytes, reinterpret_cast<hipStream_t>(stream)) == hipSuccess ? MUKV_OK
                                                                                                         : MUKV_ERR_HIP;
}

int mukv_get_state(const mukv_ctx *ctx, mukv_state *out) {
    if (!ctx || !out) return MUKV_ERR_INVALID_ARG;
    const Ctx &c = ctx->c;
    const int F = c.cfg.frames_per_segment;
    out->n_frames = c.n_frames;
    out->n_segments = (c.n_frames + F - 1) / F;
    out->n_kept_tokens = c.n_frames * c.kappa;
    out->store_token_capacity = c.store_cap;
    out->kappa = c.kappa;
    out->c_kv = c.c_kv;
    out->store_k = c.store_k;
    out->store_v = c.store_v;
    out->kept_idx = c.kept_idx;
    out->rep_frame_k = c.rep_frame_k;
    out->rep_frame_v = c.rep_frame_v;
    out->rep_patch_k = c.rep_patch_k;
    out->rep_patch_v = c.rep_patch_v;
    out->cnt_patch = c.cnt_patch;
    out->rep_seg_k = c.rep_seg_k;
    out->rep_seg_v = c.rep_seg_v;
    out->margin = c.margin;
    out->refined = c.refined;
    out->patch_cap = patch_cap(c);
    return MUKV_OK;
}

} // extern "C"
