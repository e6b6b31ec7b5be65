// traffic_probe: a torch-free driver of libmukv for hardware-counter runs.
//
// rocprofv3 --pmc is run on this small program instead of bench.py: it streams pseudo-random
// bf16 chunks of the 1-hour shape (L=28, Hq=28, Hkv=4, D=128, P=196, keep 24/196) through
// mukv_compress_chunk in 8-frame chunks gathered 64 at a time with overlap_copy (the launch
// configuration bench.py times; every chunk has its own resident buffers), asks one question
// (mukv_retrieve + mukv_gather_kv), and runs the library's plain copy kernel on 1 GiB as the
// reference whose HBM traffic is known (1 GiB read, 1 GiB written).  Counter values do not
// depend on the data, only on the access pattern, so the filler is a cheap LCG.
//
//   traffic_probe [n_frames=2048]
#include <hip/hip_runtime.h>

#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <vector>

#include "mukv.h"
#include "mukv_measure.h"

#define CK(x)                                                                          \
    do {                                                                               \
        hipError_t e_ = (x);                                                           \
        if (e_ != hipSuccess) {                                                        \
            std::printf("HIP error %s at line %d\n", hipGetErrorString(e_), __LINE__); \
            return 1;                                                                  \
        }                                                                              \
    } while (0)
#define MK(x)                                                                      \
    do {                                                                           \
        int r_ = (x);                                                              \
        if (r_ != MUKV_OK) {                                                       \
            std::printf("mukv error %s at line %d\n", mukv_strerror(r_), __LINE__); \
            return 1;                                                              \
        }                                                                          \
    } while (0)

int main(int argc, char **argv) {
    const int L = 28, Hq = 28, Hkv = 4, D = 128, P = 196, chunk = 8, batch = 64;
    const int n_frames = argc > 1 ? std::atoi(argv[1]) : 2048;
    const int n_chunks = n_frames / chunk;
    mukv_config cfg;
    std::memset(&cfg, 0, sizeof cfg);
    cfg.n_layers = L;
    cfg.n_q_heads = Hq;
    cfg.n_kv_heads = Hkv;
    cfg.head_dim = D;
    cfg.tokens_per_frame = P;
    cfg.frames_per_segment = 32;
    cfg.superpatches_per_frame = 4;
    cfg.dtype = MUKV_BF16;
    cfg.keep_ratio = 0.125;
    cfg.alpha = 0.7;
    cfg.causal = 1;
    cfg.score_layer = -1;
    cfg.max_frames = n_chunks * chunk;
    cfg.max_chunk_frames = chunk;
    cfg.max_questions = 1;
    cfg.batch_chunks = batch;
    cfg.refine_margin = -1.0;
    cfg.overlap_copy = 1;
    mukv_ctx *ctx = nullptr;
    MK(mukv_create(&cfg, &ctx));

    const size_t kv_elems = (size_t)L * Hkv * chunk * P * D, q_elems = (size_t)Hq * chunk * P * D;
    uint16_t *K, *V, *Q;
    CK(hipMalloc(&K, kv_elems * 2 * n_chunks));
    CK(hipMalloc(&V, kv_elems * 2 * n_chunks));
    CK(hipMalloc(&Q, q_elems * 2 * n_chunks));
    std::vector<uint16_t> h(kv_elems + 64);
    uint32_t lcg = 12345u;
    for (size_t i = 0; i < h.size(); ++i) { // bf16 values in (-2, 2)
        lcg = lcg * 1664525u + 1013904223u;
        const float f = (float)((int)(lcg >> 8) % 2001 - 1000) / 500.f;
        uint32_t u;
        std::memcpy(&u, &f, 4);
        h[i] = (uint16_t)(u >> 16);
    }
    for (int c = 0; c < n_chunks; ++c) { // every chunk: the same filler at a different offset
        const int o = c % 32;
        CK(hipMemcpy(K + c * kv_elems, h.data() + o, kv_elems * 2, hipMemcpyHostToDevice));
        CK(hipMemcpy(V + c * kv_elems, h.data() + 32 + o, kv_elems * 2, hipMemcpyHostToDevice));
        CK(hipMemcpy(Q + c * q_elems, h.data() + 16 + o, q_elems * 2, hipMemcpyHostToDevice));
    }
    const mukv_strides ks = {(int64_t)Hkv * chunk * P * D, (int64_t)chunk * P * D, D};
    const mukv_strides qs = {0, (int64_t)chunk * P * D, D};
    hipStream_t st;
    CK(hipStreamCreate(&st));
    for (int c = 0; c < n_chunks; ++c)
        MK(mukv_compress_chunk(ctx, K + c * kv_elems, V + c * kv_elems, &ks, Q + c * q_elems, &qs, nullptr, chunk, st,
                               nullptr));
    MK(mukv_flush(ctx));

    // one 32-token question, top-8 segments / top-32 frames, then the gather
    const int nq = 32, k_seg = 8, k_frame = 32, kappa = 24;
    int32_t offs_h[2] = {0, nq}, *offs, *seg_idx, *frm_idx, *n_tok;
    float *seg_sc, *frm_sc;
    void *k_out, *v_out;
    CK(hipMalloc(&offs, 8));
    CK(hipMemcpy(offs, offs_h, 8, hipMemcpyHostToDevice));
    CK(hipMalloc(&seg_idx, k_seg * 4));
    CK(hipMalloc(&frm_idx, k_frame * 4));
    CK(hipMalloc(&seg_sc, k_seg * 4));
    CK(hipMalloc(&frm_sc, k_frame * 4));
    CK(hipMalloc(&n_tok, 4));
    const size_t g_bytes = (size_t)L * Hkv * k_frame * kappa * D * 2;
    CK(hipMalloc(&k_out, g_bytes));
    CK(hipMalloc(&v_out, g_bytes));
    mukv_retrieve_params prm;
    std::memset(&prm, 0, sizeof prm);
    prm.mode = MUKV_SEMI;
    prm.k_seg = k_seg;
    prm.k_frame = k_frame;
    prm.n_visible_frames = -1;
    prm.lambda_frame = 0.3;
    MK(mukv_retrieve(ctx, Q, offs, 1, &prm, seg_idx, seg_sc, frm_idx, frm_sc, st));
    MK(mukv_gather_kv(ctx, frm_idx, 1, k_frame, MUKV_TEMPORAL, k_out, v_out, n_tok, st));

    // reference: 1 GiB plain copy (source: the first GiB of K, destination: scratch)
    const int64_t gib = (int64_t)1 << 30;
    void *scratch;
    CK(hipMalloc(&scratch, gib));
    MK(mukv_plain_copy(scratch, K, gib, st));
    CK(hipStreamSynchronize(st));
    std::printf("traffic_probe: %d frames compressed in %d chunks, 1 question retrieved, 1 GiB reference copy done\n",
                n_chunks * chunk, n_chunks);
    mukv_destroy(ctx);
    return 0;
}
