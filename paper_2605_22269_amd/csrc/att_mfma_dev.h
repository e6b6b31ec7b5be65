// Eq. 1 (attention received per token) on the CDNA4 matrix cores: bf16 payload, D = 128,
// P <= 208 tokens per frame.
//
// One workgroup per (frame, part) where a part is `hpw` consecutive query heads of one KV
// group.  The frame's keys are staged once in LDS: rows of 256 B whose 16-byte pieces are
// stored at piece ^ (row % 16), so the 16-byte operand reads of 16 consecutive rows fall into
// different banks without padding.  The score tile S = Q K^T is computed with
// v_mfma_f32_16x16x32_bf16: the A operand is a 16-query x 32-dim slice of Q, the B operand a
// 32-dim x 16-key slice of K from LDS.  Every Q element is used exactly once; a wave's next
// 16-query strip is fetched by the global-to-LDS load (no registers held while it is in flight)
// into the wave's own 4 KB buffer, in the same swizzled layout, while the current strip -- already
// in registers -- is processed.  In the accumulator layout a lane owns one key column
// (lane % 16) and the four query rows 4*(lane/16)..+3 of each tile, so the softmax statistics of
// a query row are an in-lane pass over its tiles plus a 16-lane reduction, and the per-key
// column sums stay in registers (one per tile) across queries, strips and heads.
//
// A query strip is 16 queries.  With the causal mask strip s needs key tiles 0..s only, so
// wave w takes strips w and nt-1-w (nt = ceil(P/16)) to balance the work.
// The softmax is exact (whole key row in registers), evaluated as exp2((s - max) * log2(e)/sqrt(D)).
// This header holds the device code; att_mfma.hip wraps it in a kernel of its own and compress.hip in
// the launch that also carries the copy of an earlier batch's kept rows.
#pragma once
#include "mukv_internal.h"

namespace mukv {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(4))) unsigned int u32x4;

constexpr int kMaxTiles = 13;  // 13 * 16 = 208 >= P
constexpr int kHeadDim = 128;
constexpr int kRowB = kHeadDim * 2;   // bytes of one key / query row in LDS
constexpr int kTileB = 16 * kRowB;    // one 16-row tile: 4 KB
constexpr size_t kAttMfmaMaxLds = (size_t)(kMaxTiles + (kMaxTiles + 1) / 2) * kTileB; // most LDS a workgroup asks for
#define MUKV_GLOBAL_PTR(p) ((const void __attribute__((address_space(1))) *)(p))
#define MUKV_LDS_PTR(p) ((void __attribute__((address_space(3))) *)(p))

struct JobArgs {
    const unsigned char *k_lds; // LDS key tile 0
    int off[4];                 // this lane's byte offset inside a tile for feature slices 0..3
    int t;                      // last tile: query row r of this lane sees the lane's key iff t <= r
    int rows;                   // query rows r < rows of this lane exist (position < P)
    bool mask;                  // the last tile holds the causal diagonal or keys past P
    float scale_log2e;
};

// Maximum over the 16 lanes of a row for four values at once.  The four chains are interleaved so
// that a value is read (through the lane permute) three instructions after it was written, which
// covers the two wait states the permute needs; the leading s_nop covers the instruction before
// the block.  All lanes are active and every permutation stays inside the row.
__device__ __forceinline__ void row16_max4(float &a, float &b, float &c, float &d) {
#define MUKV_MAX4(CTRL)                                                  \
    "v_max_f32_dpp %0, %0, %0 " CTRL " row_mask:0xf bank_mask:0xf\n\t" \
    "v_max_f32_dpp %1, %1, %1 " CTRL " row_mask:0xf bank_mask:0xf\n\t" \
    "v_max_f32_dpp %2, %2, %2 " CTRL " row_mask:0xf bank_mask:0xf\n\t" \
    "v_max_f32_dpp %3, %3, %3 " CTRL " row_mask:0xf bank_mask:0xf\n\t"
    asm("s_nop 1\n\t" MUKV_MAX4("quad_perm:[1,0,3,2]") MUKV_MAX4("quad_perm:[2,3,0,1]") MUKV_MAX4("row_half_mirror")
            MUKV_MAX4("row_mirror")
        : "+v"(a), "+v"(b), "+v"(c), "+v"(d));
#undef MUKV_MAX4
}

// One (head, strip) job over the first NTL key tiles, fully unrolled for that count so that no
// arithmetic is spent on tiles above the causal diagonal.  Score tiles S = Q K^T (A operand: the
// strip's Q, B operand: a key tile from LDS): a lane then owns one key column (lane % 16) and the
// four query rows 4*(lane/16)..+3 of every tile.  The key operands of tile c+1 are requested from
// LDS before the matrix instructions of tile c are issued.  Row statistics of the exact softmax
// are an in-lane pass over the tiles plus a 16-lane reduction; the normalised probabilities of
// the lane's four rows are added into ONE accumulator per tile (13 registers for the whole frame).
template <int NTL>
__device__ __forceinline__ void strip_job(const JobArgs &ja, const bf16x8 *qv, float *acc) {
    f32x4 st[NTL];
    bf16x8 kf[2][4];
#pragma unroll
    for (int kk = 0; kk < 4; ++kk) kf[0][kk] = *reinterpret_cast<const bf16x8 *>(ja.k_lds + ja.off[kk]);
#pragma unroll
    for (int c = 0; c < NTL; ++c) {
        if (c + 1 < NTL) {
#pragma unroll
            for (int kk = 0; kk < 4; ++kk)
                kf[(c + 1) & 1][kk] = *reinterpret_cast<const bf16x8 *>(ja.k_lds + (c + 1) * kTileB + ja.off[kk]);
        }
        __builtin_amdgcn_sched_barrier(0); // keeps the requests of tile c+1 ahead of the matrix instructions of tile c
        f32x4 d = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int kk = 0; kk < 4; ++kk) d = __builtin_amdgcn_mfma_f32_16x16x32_bf16(qv[kk], kf[c & 1][kk], d, 0, 0, 0);
        st[c] = d;
        __builtin_amdgcn_sched_barrier(0);
    }
    if (ja.mask) { // only the last tile can need masking
        constexpr int c = NTL - 1;
#pragma unroll
        for (int r = 0; r < 4; ++r) st[c][r] = (ja.t <= r) ? st[c][r] : -INFINITY;
    }
    float m[4];
#pragma unroll
    for (int r = 0; r < 4; ++r) m[r] = st[0][r];
#pragma unroll
    for (int c = 1; c < NTL; ++c)
#pragma unroll
        for (int r = 0; r < 4; ++r) m[r] = fmaxf(m[r], st[c][r]);
    row16_max4(m[0], m[1], m[2], m[3]); // every query row sees at least its own key: finite
    float mb[4], z[4] = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int r = 0; r < 4; ++r) mb[r] = m[r] * ja.scale_log2e;
#pragma unroll
    for (int c = 0; c < NTL; ++c)
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            const float p = __builtin_amdgcn_exp2f(st[c][r] * ja.scale_log2e - mb[r]);
            st[c][r] = p;
            z[r] += p;
        }
    float inv[4];
#pragma unroll
    for (int r = 0; r < 4; ++r) {
        // 1 <= z <= P (the largest term is 1): reciprocal estimate + one Newton step
        const float zr = row16_sum(z[r]);
        float rc = __builtin_amdgcn_rcpf(zr);
        rc = fmaf(fmaf(-zr, rc, 1.0f), rc, rc);
        inv[r] = (r < ja.rows) ? rc : 0.0f;
    }
#pragma unroll
    for (int c = 0; c < NTL; ++c) {
        float t = acc[c];
#pragma unroll
        for (int r = 0; r < 4; ++r) t += st[c][r] * inv[r];
        acc[c] = t;
    }
}

// What the attention workgroups need besides the batch's pointer tables.
struct AttMfmaArgs {
    int64_t k_off, q_sh, q_st, k_sh, k_st; // element offset of the scoring layer's keys; head / token strides
    int P, nt, G, hpw, causal, pair, n_split, n_part;
    float scale_log2e;
    float *out; // [batch frame][n_part][P] partial column sums
    // Eq. 2-3 on the way (layout with a KV group per workgroup only): the frequency indicator of the
    // staged keys, per KV head, to fft_out [batch frame][Hkv][P] as sum_m |Z[m]| (not yet divided by
    // Hkv * D); dft = the transform's matrix as bf16 operands (see dft_operand_table).  Null: not computed.
    const uint16_t *dft;
    float *fft_out;
};

// Eq. 2-3 for the frame's keys of one KV head, from the key tiles already staged in LDS, as a matrix
// product on the matrix cores: Z = K W with W [128 features x 128 columns], column c <= 64 the cosine
// of bin c, column 64 + m the sine of bin m (1 <= m <= 63); the keys are real, so bins m and 128 - m
// have the same magnitude and sum_m |Z[m]| = |Z[0]| + |Z[64]| + 2 sum_{0<m<64} |Z[m]|.
// The keys are bf16 and go in as they are; W is split into three bf16 terms (hi + mid + lo carry 24
// bits of every entry) and the three products accumulate in fp32, every single product being exact.
// A key tile is the A operand exactly as the attention reads it as its B operand (lane = row lr, 8
// features from 8 * lg of every 32); the W operands come from a table in memory that every workgroup
// shares (lane-major: one 16-byte load per lane and operand).  In the result a lane holds bin column
// lr of four tokens; the cosine tile ct and the sine tile ct + 4 put a bin's real and imaginary part
// in the same lane (bin 0's lane gets Re Z[0] and Re Z[64]).  Wave w takes token tiles w and
// w + n_waves and loads every W operand once for both.
constexpr int kDftSplits = 3;
constexpr int kDftOperand = 64 * 8; // bf16 elements of one operand: 64 lanes x 8
__device__ __forceinline__ void freq_mfma_phase(const unsigned char *Ks, const int (&off)[4], const uint16_t *__restrict__ dft,
                                                int w, int n_waves, int lane, int nt, int P, float *__restrict__ out) {
    const int lr = lane & 15, lg = lane >> 4;
    const int tA = w, tB = w + n_waves;
    if (tA >= nt) return;
    const bool two = tB < nt;
    bf16x8 ka[2][4];
#pragma unroll
    for (int kk = 0; kk < 4; ++kk) {
        ka[0][kk] = *reinterpret_cast<const bf16x8 *>(Ks + tA * kTileB + off[kk]);
        ka[1][kk] = *reinterpret_cast<const bf16x8 *>(Ks + (two ? tB : tA) * kTileB + off[kk]);
    }
    float tok[2][4] = {{0.f, 0.f, 0.f, 0.f}, {0.f, 0.f, 0.f, 0.f}};
    const bf16x8 *tab = reinterpret_cast<const bf16x8 *>(dft) + lane;
#pragma unroll 1
    for (int ct = 0; ct < 4; ++ct) {
        f32x4 re[2] = {{0.f, 0.f, 0.f, 0.f}, {0.f, 0.f, 0.f, 0.f}}, im[2] = {{0.f, 0.f, 0.f, 0.f}, {0.f, 0.f, 0.f, 0.f}};
#pragma unroll
        for (int sp = kDftSplits - 1; sp >= 0; --sp) { // the smallest terms first
            bf16x8 wr[4], wi[4];
#pragma unroll
            for (int kk = 0; kk < 4; ++kk) {
                wr[kk] = tab[((sp * 8 + ct) * 4 + kk) * 64];
                wi[kk] = tab[((sp * 8 + ct + 4) * 4 + kk) * 64];
            }
#pragma unroll
            for (int kk = 0; kk < 4; ++kk) {
#pragma unroll
                for (int t = 0; t < 2; ++t) {
                    re[t] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(ka[t][kk], wr[kk], re[t], 0, 0, 0);
                    im[t] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(ka[t][kk], wi[kk], im[t], 0, 0, 0);
                }
            }
        }
        const bool ends = ct == 0 && lr == 0; // this lane holds Re Z[0] and Re Z[64]
#pragma unroll
        for (int t = 0; t < 2; ++t)
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                const float x = re[t][r], y = im[t][r];
                const float mid = 2.0f * __builtin_sqrtf(fmaf(x, x, y * y));
                tok[t][r] += ends ? fabsf(x) + fabsf(y) : mid;
            }
    }
#pragma unroll
    for (int t = 0; t < 2; ++t)
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            const float v = row16_sum(tok[t][r]);
            const int token = 16 * (t ? tB : tA) + 4 * lg + r;
            if (lr == 0 && token < P && (t == 0 || two)) out[token] = v;
        }
}

// The same with the transform's matrix passing through LDS: read straight from memory, every wave fetches all
// 96 KB of operands for its two token tiles, 24 dependent rounds of loads with 16 matrix instructions each.
// Here the workgroup stages the 24 KB of one cosine / sine tile pair (all three terms) at a time in `wlds`
// (lane-major operands, 1 KB each, in the order [term][re | im][feature slice]), the next pair's pieces being
// on their way in registers meanwhile, and every wave reads its operands from there.  All waves of the
// workgroup must call it; `wlds` (24 KB) must not be in use by anyone, and is free again on return.
constexpr int kDftStageB = kDftSplits * 2 * 4 * 1024;
__device__ __forceinline__ void freq_mfma_phase_lds(const unsigned char *Ks, const int (&off)[4], const uint16_t *__restrict__ dft,
                                                    unsigned char *wlds, int w, int n_waves, int tid, int n_threads, int nt,
                                                    int P, float *__restrict__ out) {
    const int lane = tid & 63, lr = lane & 15, lg = lane >> 4;
    const int tA = w < nt ? w : nt - 1, tB = w + n_waves;
    const bool any = w < nt, two = tB < nt;
    bf16x8 ka[2][4];
#pragma unroll
    for (int kk = 0; kk < 4; ++kk) {
        ka[0][kk] = *reinterpret_cast<const bf16x8 *>(Ks + tA * kTileB + off[kk]);
        ka[1][kk] = *reinterpret_cast<const bf16x8 *>(Ks + (two ? tB : tA) * kTileB + off[kk]);
    }
    float tok[2][4] = {{0.f, 0.f, 0.f, 0.f}, {0.f, 0.f, 0.f, 0.f}};
    // piece i of a tile pair's 1536 16-byte pieces: block i / 256 = term * 2 + (re | im), 256 pieces each
    constexpr int kPieces = kDftStageB / 16, kMaxPer = 4; // up to 4 pieces per thread (384 threads and more)
    const u32x4 *tab = reinterpret_cast<const u32x4 *>(dft);
    u32x4 wst[kMaxPer];
    auto fetch = [&](int ct) {
#pragma unroll
        for (int j = 0; j < kMaxPer; ++j) {
            int i = tid + j * n_threads;
            i = i < kPieces ? i : kPieces - 1;
            const int blk = i >> 8, within = i & 255, sp = blk >> 1, ri = blk & 1;
            wst[j] = tab[((sp * 8 + ct + 4 * ri) * 4) * 64 + within];
        }
    };
    fetch(0);
#pragma unroll 1
    for (int ct = 0; ct < 4; ++ct) {
        if (ct > 0) __syncthreads(); // everybody has read the pair before
#pragma unroll
        for (int j = 0; j < kMaxPer; ++j) {
            const int i = tid + j * n_threads;
            if (i < kPieces) *reinterpret_cast<u32x4 *>(wlds + 16 * i) = wst[j];
        }
        __syncthreads();
        if (ct + 1 < 4) fetch(ct + 1);
        f32x4 re[2] = {{0.f, 0.f, 0.f, 0.f}, {0.f, 0.f, 0.f, 0.f}}, im[2] = {{0.f, 0.f, 0.f, 0.f}, {0.f, 0.f, 0.f, 0.f}};
#pragma unroll
        for (int sp = kDftSplits - 1; sp >= 0; --sp) { // the smallest terms first
#pragma unroll
            for (int kk = 0; kk < 4; ++kk) {
                const bf16x8 wr = *reinterpret_cast<const bf16x8 *>(wlds + ((sp * 2 + 0) * 4 + kk) * 1024 + 16 * lane);
                const bf16x8 wi = *reinterpret_cast<const bf16x8 *>(wlds + ((sp * 2 + 1) * 4 + kk) * 1024 + 16 * lane);
#pragma unroll
                for (int t = 0; t < 2; ++t) {
                    re[t] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(ka[t][kk], wr, re[t], 0, 0, 0);
                    im[t] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(ka[t][kk], wi, im[t], 0, 0, 0);
                }
            }
        }
        const bool ends = ct == 0 && lr == 0; // this lane holds Re Z[0] and Re Z[64]
#pragma unroll
        for (int t = 0; t < 2; ++t)
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                const float x = re[t][r], y = im[t][r];
                const float mid = 2.0f * __builtin_sqrtf(fmaf(x, x, y * y));
                tok[t][r] += ends ? fabsf(x) + fabsf(y) : mid;
            }
    }
#pragma unroll
    for (int t = 0; t < 2; ++t)
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            const float v = row16_sum(tok[t][r]);
            const int token = 16 * (t ? tB : tA) + 4 * lg + r;
            if (any && lr == 0 && token < P && (t == 0 || two)) out[token] = v;
        }
}

// True when a batch is long enough for the layout with a whole KV group per workgroup.
bool att_mfma_many(const Ctx &c, int n_frames);
// Fills in the launch shape for a batch: workgroup layout, waves per workgroup, LDS bytes.
void att_mfma_plan(const Ctx &c, const ChunkArgs &a, float *out, AttMfmaArgs *aa, int *waves, size_t *lds);

// Work of workgroup (f, by) of the (frames, n_part) grid; blockDim.x = 64 * waves.
// LDS (smem_raw, (nt + waves) * 4 KB): key tiles [nt][16 rows][256 B], then one 4 KB query buffer per
// wave.  After the last job the key region is reused for the per-wave column sums.
__device__ __forceinline__ void att_mfma_body(const PtrTable &qtab, const PtrTable &ktab, const FrameMap &map,
                                              const AttMfmaArgs &aa, int f, int by, unsigned char *smem_raw) {
    const int64_t k_off = aa.k_off, q_sh = aa.q_sh, q_st = aa.q_st, k_sh = aa.k_sh, k_st = aa.k_st;
    const int P = aa.P, nt = aa.nt, G = aa.G, hpw = aa.hpw, causal = aa.causal, pair = aa.pair, n_split = aa.n_split;
    const int n_part = aa.n_part;
    const float scale_log2e = aa.scale_log2e;
    float *__restrict__ out = aa.out;
    unsigned char *Ks = smem_raw;
    const int part = by / n_split, sp = by - part * n_split;
    const int h0 = part * hpw, g = h0 / G;
    const int tid = threadIdx.x, lane = tid & 63;
    const int w = __builtin_amdgcn_readfirstlane(tid >> 6); // wave-uniform: strip choices become scalar branches
    const int n_threads = blockDim.x;
    const int lr = lane & 15, lg = lane >> 4;
    unsigned char *Qs = smem_raw + (size_t)nt * kTileB + (size_t)w * kTileB;

    // pair = 1: wave w takes strips w and nt-1-w (balanced under the causal mask, for throughput).
    // pair = 0: one strip per wave and the strips of a (frame, part) split over n_split workgroups
    // (shortest critical path, for calls with few frames); a workgroup then stages only the keys
    // its strips can see.
    const int wps = (nt + n_split - 1) / n_split; // strips per workgroup when not paired
    const int sA = pair ? w : sp * wps + w, sB = nt - 1 - w;
    const int n_strips = (pair && sA != sB) ? 2 : 1;
    const bool active = sA < nt && (pair || w < wps);
    int k_tiles = nt;
    if (!pair && causal) k_tiles = (sp + 1) * wps < nt ? (sp + 1) * wps : nt;
    const int slot = find_slot(map, f);
    const int lf = f - map.fstart[slot];
    const uint16_t *qf = reinterpret_cast<const uint16_t *>(qtab.p[slot]) + ((int64_t)lf * P) * q_st;
    // Request of one (head, strip) into the wave's query buffer: four 1 KB instructions, lane i of
    // instruction j fills 16-byte slot 64*j + i = (row 4*j + i/16, position i%16), which holds
    // piece position ^ row of that row.  Rows past P are clamped (masked later).
    const unsigned q_st2 = (unsigned)q_st * 2u; // token stride in bytes
    auto request_q = [&](int h, int s) {
        // wave-uniform 64-bit base + a 32-bit per-lane byte offset: the token stride is below
        // 2^24 bytes (checked on the host), so position * stride is one 24-bit multiply-add
        const unsigned char *base = reinterpret_cast<const unsigned char *>(qf + (int64_t)h * q_sh);
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int row = 4 * j + lg;
            const int qi = 16 * s + row;
            const unsigned off = __umul24((unsigned)(qi < P ? qi : P - 1), q_st2) + (unsigned)((lr ^ row) << 4);
            __builtin_amdgcn_global_load_lds(MUKV_GLOBAL_PTR(base + off), MUKV_LDS_PTR(Qs + 1024 * j), 16, 0, 0);
        }
    };
    const int n_jobs = active ? hpw * n_strips : 0; // (head, strip) pairs of this wave, strip fastest
    if (n_jobs > 0) request_q(h0, sA);              // job 0: in flight while K is staged

    // stage K of (frame, KV head) in LDS; rows past P are zero.  Loads are unconditional on a
    // clamped row and issued in batches of 8 before the LDS stores.
    const uint16_t *kf = reinterpret_cast<const uint16_t *>(ktab.p[slot]) + k_off + (int64_t)g * k_sh + (int64_t)lf * P * k_st;
    const int n_units = k_tiles * 16 * 16;
    for (int i0 = tid; i0 < n_units; i0 += 8 * n_threads) {
        u32x4 val[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) {
            int idx = i0 + u * n_threads;
            idx = idx < n_units ? idx : n_units - 1;
            const int row = idx >> 4;
            val[u] = *reinterpret_cast<const u32x4 *>(kf + (int64_t)(row < P ? row : P - 1) * k_st + (idx & 15) * 8);
        }
#pragma unroll
        for (int u = 0; u < 8; ++u) {
            const int idx = i0 + u * n_threads;
            if (idx < n_units) {
                const int row = idx >> 4, piece = idx & 15;
                *reinterpret_cast<u32x4 *>(Ks + row * kRowB + ((piece ^ (row & 15)) << 4)) =
                    row < P ? val[u] : u32x4{0u, 0u, 0u, 0u};
            }
        }
    }
    __syncthreads();

    JobArgs ja;
    ja.k_lds = Ks;
#pragma unroll
    for (int kk = 0; kk < 4; ++kk) ja.off[kk] = lr * kRowB + (((4 * kk + lg) ^ lr) << 4);
    // Eq. 2-3 from the staged keys (pair: every key tile is staged and this workgroup is the only one of its
    // (frame, KV head)): through LDS once the query buffers are free, if together they hold a staged tile
    // pair; else straight from memory, now
    const bool fft_here = aa.fft_out && pair;
    const bool fft_lds = fft_here && (size_t)(n_threads >> 6) * kTileB >= (size_t)kDftStageB && n_threads * 4 >= kDftStageB / 16;
    float *fft_dst = fft_here ? aa.fft_out + ((int64_t)f * (aa.n_part / n_split) + g) * P : nullptr;
    if (fft_here && !fft_lds) freq_mfma_phase(Ks, ja.off, aa.dft, w, n_threads >> 6, lane, nt, P, fft_dst);

    float acc[kMaxTiles];
#pragma unroll
    for (int c = 0; c < kMaxTiles; ++c) acc[c] = 0.f;

    ja.scale_log2e = scale_log2e;
    const bool tail = (P & 15) != 0;
    for (int job = 0; job < n_jobs; ++job) {
        const int hh = job / n_strips, si = job - hh * n_strips;
        const int s = si ? sB : sA;
        const int ntl = __builtin_amdgcn_readfirstlane(causal ? s + 1 : nt); // key tiles this strip sees
        const int q0 = 16 * s + 4 * lg;   // first of this lane's four query positions
        const int j = 16 * (ntl - 1) + lr; // this lane's key in the last tile
        ja.t = j < P ? (causal ? j - q0 : -1) : 4;
        ja.rows = P - q0;
        ja.mask = causal || (tail && ntl == nt);
        // this job's queries have arrived in the wave's buffer: move them to registers, and once
        // they are there let the buffer take the next job's queries, which then have this whole
        // job (and the other resident waves) to arrive
        bf16x8 qv[4];
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
#pragma unroll
        for (int kk = 0; kk < 4; ++kk) qv[kk] = *reinterpret_cast<const bf16x8 *>(Qs + ja.off[kk]);
        asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
        if (job + 1 < n_jobs) {
            const int hn = (job + 1) / n_strips, sn = (job + 1) - hn * n_strips;
            request_q(h0 + hn, sn ? sB : sA);
        }
        switch (ntl) {
#define MUKV_JOB_CASE(N) case N: strip_job<N>(ja, qv, acc); break;
            MUKV_JOB_CASE(1) MUKV_JOB_CASE(2) MUKV_JOB_CASE(3) MUKV_JOB_CASE(4) MUKV_JOB_CASE(5)
            MUKV_JOB_CASE(6) MUKV_JOB_CASE(7) MUKV_JOB_CASE(8) MUKV_JOB_CASE(9) MUKV_JOB_CASE(10)
            MUKV_JOB_CASE(11) MUKV_JOB_CASE(12) MUKV_JOB_CASE(13)
#undef MUKV_JOB_CASE
        default: break;
        }
    }
    __syncthreads(); // the query buffers are free
    if (fft_lds) {
        freq_mfma_phase_lds(Ks, ja.off, aa.dft, smem_raw + (size_t)nt * kTileB, w, n_threads >> 6, tid, n_threads, nt, P, fft_dst);
        __syncthreads(); // the key tiles are free
    }
    // column sums: add the four lane groups (the other query rows), then the waves in a fixed
    // order; the key tiles are no longer needed and give room for the per-wave sums
    float *red = reinterpret_cast<float *>(smem_raw); // [waves][nt*16]
    const int ld = nt * 16;
#pragma unroll
    for (int c = 0; c < kMaxTiles; ++c) {
        if (c < nt) {
            const float v = xrow_sum(acc[c]);
            if (lg == 0) red[w * ld + 16 * c + lr] = v;
        }
    }
    __syncthreads();
    const int n_waves = n_threads >> 6;
    for (int j = tid; j < P; j += n_threads) {
        float s = 0.f;
        for (int ww = 0; ww < n_waves; ++ww) s += red[ww * ld + j];
        out[((int64_t)f * n_part + by) * P + j] = s;
    }
}


} // namespace mukv
