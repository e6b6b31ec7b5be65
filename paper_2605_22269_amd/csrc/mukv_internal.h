// Internal declarations shared by the HIP translation units of libmukv.
// Nothing here is part of the public ABI (see include/mukv.h).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include <vector>

#include "mukv.h"
#include "mukv_measure.h"

namespace mukv {

constexpr int kWave = 64;
constexpr int kMaxP = 256;        // tokens per frame the per-frame kernels are built for
constexpr int kMaxUnit = 8192;    // tokens of a unit of several frames ranked as one (attention signal handed over)
constexpr int kMaxCand = 1024;    // stage-1 candidates (2*k) held in LDS by the rerank kernel
constexpr int kMaxGatherK = 1024; // selected frames per question the gather kernel can plan
constexpr int kMaxStores = 4;         // stores searched together (the paper has three: segment, frame, patch)
constexpr int kMaxMultiEntries = 3072; // units per question the gather over several stores can plan

// one chunk handed to mukv_compress_chunk and not yet launched
struct PendingChunk {
    const void *k, *v, *q;
    const float *att_in;
    mukv_signals_out sig;
    int n_frames;
};

struct ProfEntry {
    int kid;
    hipEvent_t start, stop;
};

struct ChunkArgs;

constexpr int kAttendMaxTokens = 16; // query tokens per question in one mukv_attend call
constexpr int kAttendMaxSplit = 8;   // workgroups sharing the frame list of one (question, KV head)
constexpr int kPrefillMaxTokens = 8192; // new tokens per question in one mukv_prefill_attend call

struct Ctx {
    mukv_config cfg;
    bool profiling;
    std::vector<ProfEntry> *prof; // event pairs recorded since mukv_profile_begin
    int kappa, ls, c_kv, group, esz, max_segments;
    bool use_mfma;
    double margin_thr;
    int64_t n_frames;  // frames submitted so far (host-side append position)
    int64_t n_done;    // frames whose kernels have been enqueued
    int batch_chunks;  // chunks gathered before a chain of launches goes out
    int max_batch_frames;
    std::vector<PendingChunk> *pending;
    int64_t p_kv_sl, p_kv_sh, p_kv_st, p_q_sh, p_q_st; // strides shared by the pending chunks
    hipStream_t p_stream;
    int batch_parity;
    int64_t store_cap; // tokens per (layer, head) slab of the store
    // cache (device)
    void *store_k, *store_v;
    int32_t *kept_idx;
    float *rep_frame_k, *rep_frame_v, *rep_patch_k, *rep_patch_v, *rep_seg_k, *rep_seg_v;
    int32_t *cnt_patch;
    double *fsum_k, *fsum_v; // [max_frames][c_kv] exact sums of the kept scoring-layer rows
    double *ssum_k, *ssum_v; // [max_segments][c_kv] running sums of fsum over each segment
    float *margin;
    int32_t *refined;
    // per-chunk scratch (device)
    // (two of each, by batch parity: with overlap_copy the keep of a batch runs beside the next
    // batch's kernels)
    float *att_part[2]; // [max_batch_frames][n_part][P]
    float *fft_sig[2];  // [max_batch_frames][P], or [max_batch_frames][Hkv][P] per-head sums (matrix-core path)
    uint16_t *dft_tab;  // matrix-core operands of the feature-axis transform (matrix-core attention, D = 128), or null
    double *att64;    // [max_chunk_frames][Hq][P] partial fp64 attention of re-scored frames
    double *fft64;    // [max_chunk_frames][P]
    int32_t *src_tok[2]; // [max_batch_frames*kappa] chunk-local token of every kept row
    int32_t *src_tok2;                // the same for the frames re-scored in fp64
    int32_t *flag_list[2], *flag_count; // batch frames to re-score in fp64 and how many, by batch parity
    hipStream_t side;                 // re-scoring chain (with overlap_copy also the keep) runs here
    hipEvent_t ev_fork;               // the batch's signals are enqueued on the caller's stream
    hipEvent_t ev_join[2];            // the side stream's work for the batch of that parity is enqueued
    hipEvent_t ev_copy;               // the copies that were put off are enqueued (orders another stream after them)
    bool side_pending[2];             // ev_join recorded and not yet waited for by the caller's stream
    // overlap_copy with frames as units: `side` carries the keep of a batch and then its fp64 re-scoring
    // chain; ev_keep marks the end of the keep, so that the copy of the batch's rows (two batches later,
    // on the caller's stream) waits for the keep alone; the re-scored frames' rows and the segment keys
    // follow with the fp64 chain
    bool split_side;
    hipEvent_t ev_keep[2];            // the keep of the batch of that parity is enqueued
    bool keep_pending[2];             // ev_keep recorded and not yet waited for by the caller's stream
    ChunkArgs *deferred;              // overlap_copy: the (at most two) batches whose row copy is still to be
    int n_deferred;                   // launched, the older one first
    hipStream_t deferred_stream;      // stream those batches were submitted on
    // retrieval scratch (device)
    double *qbar;    // [max_questions][c_kv]  group-summed mean query
    double *qq;      // [max_questions][Hkv * D / pool_slice]   partial squared norms of the mean query
    double *s_frm;   // [max_questions][max_frames]
    double *s_seg;   // [max_questions][max_segments]
    float *seg_tail; // [max_questions][c_kv] key of the segment cut by a question's timestamp
    // combined gather scratch (device)
    uint32_t *u_mask;  // [max_questions][max_frames] super-patches of a frame chosen at any level
    int32_t *u_entry;  // [max_questions][max_frames][3] chosen frames in time order: frame, mask, first output row
    int32_t *u_count;  // [max_questions][2] entries, rows
    // gather over several stores (this context being the first of them): chosen units in temporal order
    int32_t *m_entry;  // [max_questions][kMaxMultiEntries][3] store, unit, first output row
    int32_t *m_count;  // [max_questions][2] entries, rows
    // token-axis frequency signal: cos and -sin of 2*pi*m*j/P for rows and token pairs 0..P/2,
    // [P/2+1][P/2+1][2]; per (batch frame, group of 64 features, row) sums of |Z|: the fp32 pass
    // uses the first tok_part_half bytes, the fp64 pass the rest
    float *tw32;
    double *tw64;
    unsigned char *tok_part;
    size_t tok_part_half;
    // attention over the retrieved context: per (question, token, head, split) maximum, normaliser, output
    float *attend_part; // [max_questions][kAttendMaxTokens][Hq][kAttendMaxSplit][D+2]
};

// ---- a batch of chunks processed by one chain of launches ----
// Every chunk handed to mukv_compress_chunk occupies one slot; the kernels see the batch as
// frames 0..n_frames-1 and resolve a frame to (slot, frame inside the chunk) with FrameMap.
// The tables travel by value in the kernel arguments, so a captured HIP graph replays them as is.
constexpr int kMaxSlots = 64;
struct PtrTable {
    const void *p[kMaxSlots];
};
struct OutTable {
    float *p[kMaxSlots];
};
struct FrameMap {
    int fstart[kMaxSlots + 1]; // first batch frame of every slot; fstart[n_slots] = n_frames
    int n_slots;
};
// slot of batch frame f (f is uniform over the workgroup at every call site, so this is scalar code)
__device__ __forceinline__ int find_slot(const FrameMap &m, int f) {
    int s = 0;
    while (s + 1 < m.n_slots && f >= m.fstart[s + 1]) ++s;
    return s;
}

struct ChunkArgs {
    PtrTable k, v, q, att_in;      // per slot: chunk base pointers (att_in: float [n][P] or null)
    OutTable dbg_att, dbg_fft, dbg_fused;
    FrameMap map;
    bool have_q, have_att_in, have_dbg;
    int64_t kv_sl, kv_sh, kv_st; // element strides layer / head / token (same for every slot)
    int64_t q_sh, q_st;
    int n_frames;                // frames in the batch
    int64_t frame0;              // cache position of batch frame 0
    int parity;                  // which set of per-batch scratch (signals, row list, re-scoring list) this batch uses
};


hipError_t launch_compress(Ctx &c, const ChunkArgs &a, hipStream_t st);
// launches the copy that was put off (overlap_copy) and orders `st` after it and after the
// re-scoring chain still outstanding on the side stream
hipError_t join_streams(Ctx &c, hipStream_t st);
// forgets the copy that was put off (mukv_reset) and leaves the re-scoring list empty
hipError_t drop_deferred(Ctx &c);

struct RetrieveArgs {
    const void *q_tokens;
    const int32_t *q_offsets;
    int B;
    mukv_retrieve_params p;
    int nv;      // visible frames
    int ns;      // visible segments
    bool patches; // fine level of the search: super-patches instead of frames (k_frame, lambda_frame apply to it)
    const int32_t *nv_q; // device [B] per-question timestamps, or null (then nv / ns hold for every question)
    int units;           // 0: segments and frames of this context; 1 / 2: the context's units as the blocks of one of
                         // several stores (1: ranked by stage 1, global query out; 2: reranked with g_in), ns = 0
    const double *g_in;  // device [B][C_kv]
    double *g_out;       // device [B][C_kv] or null
    int32_t *seg_idx;
    float *seg_score;
    int32_t *frm_idx;
    float *frm_score;
};

hipError_t launch_retrieve(Ctx &c, const RetrieveArgs &a, hipStream_t st);
int pool_slice(int G, int D); // features per workgroup of the question pooling

hipError_t launch_gather(Ctx &c, const int32_t *frame_idx, int B, int k_frame, int order, void *k_out,
                         void *v_out, int32_t *n_tokens_out, hipStream_t st);

hipError_t launch_gather_patches(Ctx &c, const int32_t *patch_idx, int B, int k_patch, int order, int rows_cap,
                                 void *k_out, void *v_out, int32_t *n_tokens_out, hipStream_t st);

struct UnionArgs {
    const int32_t *seg_idx, *frame_idx, *patch_idx; // [B][k] each, any may be null
    int k_seg, k_frame, k_patch;
    int B, rows_cap;
    void *k_out, *v_out;
    int32_t *n_tokens_out;
};
hipError_t launch_gather_union(Ctx &c, const UnionArgs &a, hipStream_t st);

struct MultiArgs {
    const Ctx *c[kMaxStores];
    const int32_t *idx[kMaxStores]; // device [B][k[i]] or null
    int k[kMaxStores], ups[kMaxStores];
    int n_ctx, B, rows_cap;
    void *k_out, *v_out;
    int32_t *n_tokens_out;
};
hipError_t launch_gather_multi(const MultiArgs &a, hipStream_t st);

// Brackets the launches of one scope with HIP events when the context is profiling.
struct ProfScope {
    Ctx &c;
    hipStream_t st;
    ProfEntry e;
    bool on;
    ProfScope(Ctx &ctx, int kid, hipStream_t s) : c(ctx), st(s), on(ctx.profiling) {
        if (!on) return;
        e.kid = kid;
        on = hipEventCreate(&e.start) == hipSuccess && hipEventCreate(&e.stop) == hipSuccess &&
             hipEventRecord(e.start, st) == hipSuccess;
    }
    ~ProfScope() {
        if (!on) return;
        (void)hipEventRecord(e.stop, st);
        c.prof->push_back(e);
    }
};

hipError_t launch_plain_copy(void *dst, const void *src, int64_t bytes, hipStream_t st);

// Kernels that use more than 64 KB of dynamic LDS have to ask for it once per device; `done` is
// the caller's per-kernel table of devices already served.
constexpr int kMaxDevices = 64;
inline hipError_t allow_dynamic_lds(const void *kernel, size_t bytes, int device, bool (&done)[kMaxDevices]) {
    if (device < 0 || device >= kMaxDevices) return hipErrorInvalidDevice;
    if (done[device]) return hipSuccess;
    const hipError_t e = hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize, (int)bytes);
    if (e == hipSuccess) done[device] = true;
    return e;
}

// True when the matrix-core attention kernel covers this configuration.
bool att_mfma_supported(const mukv_config &c);
// The length-128 transform's matrix as matrix-core operands (bf16 bits), for the frequency indicator
// that the matrix-core attention workgroups compute on the way.
std::vector<uint16_t> dft_operand_table();
hipError_t launch_attend(const Ctx &c, int layer, const void *q, int n_q, const int32_t *frame_idx, int k_frame,
                         const void *k_local, const void *v_local, const int32_t *local_offsets, int B, int causal,
                         void *out, float *signal, float *workspace, hipStream_t st);
int64_t prefill_workspace_bytes(const Ctx &c, int n_q, int B, int k_frame);

// LDS bytes the generic attention kernel needs for P tokens of D features when it accumulates
// in a type of r_size bytes and keeps the keys as elements of key_size bytes.
size_t att_generic_lds_bytes(int P, int D, size_t r_size, size_t key_size);
// bytes of the staged keys: rows of D + 16 / key_size elements, rounded up to 8 bytes
__host__ __device__ inline size_t att_generic_key_bytes(int P, int D, size_t key_size) {
    return ((size_t)P * (D + 16 / key_size) * key_size + 7) & ~(size_t)7;
}

// ---- small device helpers ----
__device__ __forceinline__ float to_float(uint16_t bits) { return __uint_as_float((uint32_t)bits << 16); }
__device__ __forceinline__ float to_float(float x) { return x; }

// Cross-lane helpers that stay in the vector ALU (no LDS traffic).
// dpp_lane: value of another lane of the same 16-lane row, chosen by a DPP control word.
template <int CTRL>
__device__ __forceinline__ float dpp_lane(float v) {
    return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), CTRL, 0xF, 0xF, true));
}
constexpr int kDppQuadSwap1 = 0xB1;     // quad_perm [1,0,3,2]
constexpr int kDppQuadSwap2 = 0x4E;     // quad_perm [2,3,0,1]
constexpr int kDppRowHalfMirror = 0x141;
constexpr int kDppRowMirror = 0x140;

// sum / max over the 16 lanes of a row, result in every lane of the row
__device__ __forceinline__ float row16_sum(float v) {
    v += dpp_lane<kDppQuadSwap1>(v);
    v += dpp_lane<kDppQuadSwap2>(v);
    v += dpp_lane<kDppRowHalfMirror>(v);
    v += dpp_lane<kDppRowMirror>(v);
    return v;
}
__device__ __forceinline__ float row16_max(float v) {
    v = fmaxf(v, dpp_lane<kDppQuadSwap1>(v));
    v = fmaxf(v, dpp_lane<kDppQuadSwap2>(v));
    v = fmaxf(v, dpp_lane<kDppRowHalfMirror>(v));
    v = fmaxf(v, dpp_lane<kDppRowMirror>(v));
    return v;
}
// sum / max over the four lanes that share lane % 16 (one per row), result in all four:
// v_permlane16_swap exchanges odd rows of one operand with even rows of the other,
// v_permlane32_swap the upper half-wave of one with the lower half-wave of the other.
__device__ __forceinline__ float xrow_sum(float v) {
    auto a = __builtin_amdgcn_permlane16_swap(__float_as_uint(v), __float_as_uint(v), false, false);
    v = __uint_as_float(a[0]) + __uint_as_float(a[1]);
    auto b = __builtin_amdgcn_permlane32_swap(__float_as_uint(v), __float_as_uint(v), false, false);
    return __uint_as_float(b[0]) + __uint_as_float(b[1]);
}
__device__ __forceinline__ float xrow_max(float v) {
    auto a = __builtin_amdgcn_permlane16_swap(__float_as_uint(v), __float_as_uint(v), false, false);
    v = fmaxf(__uint_as_float(a[0]), __uint_as_float(a[1]));
    auto b = __builtin_amdgcn_permlane32_swap(__float_as_uint(v), __float_as_uint(v), false, false);
    return fmaxf(__uint_as_float(b[0]), __uint_as_float(b[1]));
}
// value of lane (lane ^ H), H a power of two below 64, without going through LDS:
// quad permutes for 1 and 2, mirror pairs for 4 (i^7 then i^3) and 8 (i^15 then i^7), row /
// half-wave swaps for 16 and 32.
constexpr int kDppQuadReverse = 0x1B; // quad_perm [3,2,1,0]
template <int H>
__device__ __forceinline__ float lane_xor(float v) {
    static_assert(H == 1 || H == 2 || H == 4 || H == 8 || H == 16 || H == 32, "lane distance");
    if constexpr (H == 1) {
        return dpp_lane<kDppQuadSwap1>(v);
    } else if constexpr (H == 2) {
        return dpp_lane<kDppQuadSwap2>(v);
    } else if constexpr (H == 4) {
        return dpp_lane<kDppQuadReverse>(dpp_lane<kDppRowHalfMirror>(v));
    } else if constexpr (H == 8) {
        return dpp_lane<kDppRowHalfMirror>(dpp_lane<kDppRowMirror>(v));
    } else if constexpr (H == 16) {
        auto a = __builtin_amdgcn_permlane16_swap(__float_as_uint(v), __float_as_uint(v), false, false);
        const bool odd_row = (__lane_id() >> 4) & 1;
        return __uint_as_float(odd_row ? a[0] : a[1]);
    } else {
        auto b = __builtin_amdgcn_permlane32_swap(__float_as_uint(v), __float_as_uint(v), false, false);
        return __uint_as_float(__lane_id() < 32 ? b[1] : b[0]);
    }
}
template <int H>
__device__ __forceinline__ double lane_xor(double v) {
    const float lo = lane_xor<H>(__int_as_float(__double2loint(v)));
    const float hi = lane_xor<H>(__int_as_float(__double2hiint(v)));
    return __hiloint2double(__float_as_int(hi), __float_as_int(lo));
}

__device__ __forceinline__ double row16_sum(double v) {
    v += lane_xor<1>(v);
    v += lane_xor<2>(v);
    v += lane_xor<4>(v);
    v += lane_xor<8>(v);
    return v;
}

__device__ __forceinline__ float wave_max(float x) { return xrow_max(row16_max(x)); }
__device__ __forceinline__ float wave_sum(float x) { return xrow_sum(row16_sum(x)); }
__device__ __forceinline__ int wave_sum(int v) {
    v += __builtin_amdgcn_update_dpp(0, v, kDppQuadSwap1, 0xF, 0xF, true);
    v += __builtin_amdgcn_update_dpp(0, v, kDppQuadSwap2, 0xF, 0xF, true);
    v += __builtin_amdgcn_update_dpp(0, v, kDppRowHalfMirror, 0xF, 0xF, true);
    v += __builtin_amdgcn_update_dpp(0, v, kDppRowMirror, 0xF, 0xF, true);
    auto a = __builtin_amdgcn_permlane16_swap((unsigned)v, (unsigned)v, false, false);
    v = (int)(a[0] + a[1]);
    auto b = __builtin_amdgcn_permlane32_swap((unsigned)v, (unsigned)v, false, false);
    return (int)(b[0] + b[1]);
}
__device__ __forceinline__ double wave_sum(double x) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) x += __shfl_xor(x, o);
    return x;
}
__device__ __forceinline__ double wave_max(double x) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) x = fmax(x, __shfl_xor(x, o));
    return x;
}

} // namespace mukv
