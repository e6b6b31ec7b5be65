// Eq. 1 (attention received per token) on the CDNA4 matrix cores: bf16 payload, D = 128,
// P <= 208 tokens per frame.
//
// One workgroup per (frame, part) where a part is `hpw` consecutive query heads of one KV
// group.  The frame's keys are staged once in LDS (row stride 272 B, so the 16-byte operand
// reads of 8 consecutive rows fall into different banks).  The score tile is computed
// transposed, S^T = K Q^T, with v_mfma_f32_16x16x32_bf16: the A operand is a 16-key x 32-dim
// slice of K from LDS, the B operand a 32-dim x 16-query slice of Q read straight from global
// memory (every Q element is used exactly once).  In the accumulator layout a lane owns one
// query column (lane % 16) and the four key rows 4*(lane/16)..+3 of each 16-key tile, so the
// softmax statistics of a query are an in-lane reduction over its tiles plus two cross-lane
// steps, and the per-key column sums can stay in registers across queries, strips and heads;
// they are reduced over the 16 query lanes once at the end.
//
// A query strip is 16 queries.  With the causal mask strip s needs key tiles 0..s only, so
// wave w takes strips w and nt-1-w (nt = ceil(P/16)) to balance the work.
// The softmax is exact (whole key row in registers), evaluated as exp2((s - max) * log2(e)/sqrt(D)).
#include "mukv_internal.h"

namespace mukv {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(4))) unsigned int u32x4;

constexpr int kMaxTiles = 13;  // 13 * 16 = 208 >= P
constexpr int kLdsRow = 136;   // bf16 elements per LDS key row: 128 + 8 of padding (272 B)
constexpr int kHeadDim = 128;

struct JobArgs {
    const uint16_t *a_base; // this lane's key-operand address in LDS key tile 0
    int q0;                 // first of this lane's four query positions in the frame
    int lr;                 // lane % 16
    int P;
    bool diag;              // causal: the last tile holds the diagonal
    bool tail;              // the last tile holds keys past P
    float scale_log2e;
};

// One (head, strip) job over the first NTL key tiles, fully unrolled for that count so that no
// arithmetic is spent on tiles above the causal diagonal.  Score tiles S = Q K^T (A operand: the
// strip's Q, B operand: a key tile from LDS): a lane then owns one key column (lane % 16) and the
// four query rows 4*(lane/16)..+3 of every tile.  Row statistics of the exact softmax are an
// in-lane pass over the tiles plus a 16-lane DPP reduction; the normalised probabilities of the
// lane's four rows are added into ONE accumulator per tile (13 registers for the whole frame).
// `after_mfma` runs once the Q operand registers are free again.
template <int NTL, typename F>
__device__ __forceinline__ void strip_job(const JobArgs &ja, const bf16x8 *qv, float *acc, F after_mfma) {
    f32x4 st[NTL];
#pragma unroll
    for (int c = 0; c < NTL; ++c) {
        f32x4 d = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int kk = 0; kk < 4; ++kk) {
            const bf16x8 kf = *reinterpret_cast<const bf16x8 *>(ja.a_base + c * 16 * kLdsRow + 32 * kk);
            d = __builtin_amdgcn_mfma_f32_16x16x32_bf16(qv[kk], kf, d, 0, 0, 0);
        }
        st[c] = d;
    }
    after_mfma();
    if (ja.diag || ja.tail) { // only the last tile can need masking
        constexpr int c = NTL - 1;
        const int j = 16 * c + ja.lr;
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            const bool ok = (j < ja.P) && (!ja.diag || j <= ja.q0 + r);
            st[c][r] = ok ? st[c][r] : -INFINITY;
        }
    }
    float m[4] = {-INFINITY, -INFINITY, -INFINITY, -INFINITY};
#pragma unroll
    for (int c = 0; c < NTL; ++c)
#pragma unroll
        for (int r = 0; r < 4; ++r) m[r] = fmaxf(m[r], st[c][r]);
    float mb[4], z[4] = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int r = 0; r < 4; ++r) mb[r] = row16_max(m[r]) * ja.scale_log2e;
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
    for (int r = 0; r < 4; ++r) inv[r] = (ja.q0 + r < ja.P) ? 1.0f / row16_sum(z[r]) : 0.0f;
#pragma unroll
    for (int c = 0; c < NTL; ++c) {
        float t = acc[c];
#pragma unroll
        for (int r = 0; r < 4; ++r) t += st[c][r] * inv[r];
        acc[c] = t;
    }
}

__global__ __launch_bounds__(448) __attribute__((amdgpu_waves_per_eu(4, 4))) void att_mfma_kernel(PtrTable qtab, PtrTable ktab, FrameMap map, int64_t k_off,
                                                       int64_t q_sh, int64_t q_st, int64_t k_sh, int64_t k_st,
                                                       int P, int nt, int G, int hpw, int causal, int pair, int n_split,
                                                       float scale_log2e, int n_part, float *__restrict__ out) {
    extern __shared__ __align__(16) unsigned char smem_raw[];
    uint16_t *Ks = reinterpret_cast<uint16_t *>(smem_raw);                           // [nt*16][kLdsRow]
    float *red = reinterpret_cast<float *>(smem_raw + (size_t)nt * 16 * kLdsRow * 2); // [waves][nt*16]
    const int f = blockIdx.x, part = blockIdx.y / n_split, sp = blockIdx.y - part * n_split;
    const int h0 = part * hpw, g = h0 / G;
    const int tid = threadIdx.x, lane = tid & 63;
    const int w = __builtin_amdgcn_readfirstlane(tid >> 6); // wave-uniform: strip choices become scalar branches
    const int n_threads = blockDim.x;
    const int lr = lane & 15, lg = lane >> 4;

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
    const uint16_t *qf = reinterpret_cast<const uint16_t *>(qtab.p[slot]) + ((int64_t)lf * P) * q_st + 8 * lg;
    // B operand of one (head, strip): 4 x 16 bytes per lane, rows past P clamped (masked later)
    auto load_q = [&](int h, int s, bf16x8 *dst) {
        const int qi = 16 * s + lr;
        const uint16_t *qp = qf + (int64_t)h * q_sh + (int64_t)(qi < P ? qi : P - 1) * q_st;
#pragma unroll
        for (int kk = 0; kk < 4; ++kk) dst[kk] = *reinterpret_cast<const bf16x8 *>(qp + 32 * kk);
    };
    const int n_jobs = active ? hpw * n_strips : 0; // (head, strip) pairs of this wave, strip fastest
    bf16x8 qv[4];
    load_q(h0, active ? sA : 0, qv); // job 0: in flight while K is staged

    // stage K of (frame, KV head) in LDS; rows past P are zero.  Loads are unconditional on a
    // clamped row and issued in batches of 4 before the LDS stores.
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
                const int row = idx >> 4;
                *reinterpret_cast<u32x4 *>(Ks + row * kLdsRow + (idx & 15) * 8) = row < P ? val[u] : u32x4{0u, 0u, 0u, 0u};
            }
        }
    }
    __syncthreads();

    float acc[kMaxTiles];
#pragma unroll
    for (int c = 0; c < kMaxTiles; ++c) acc[c] = 0.f;

    const uint16_t *a_base = Ks + lr * kLdsRow + 8 * lg;
    const bool tail = (P & 15) != 0;
    for (int job = 0; job < n_jobs; ++job) {
        const int hh = job / n_strips, si = job - hh * n_strips;
        const int s = si ? sB : sA;
        const int ntl = __builtin_amdgcn_readfirstlane(causal ? s + 1 : nt); // key tiles this strip sees
        JobArgs ja;
        ja.a_base = a_base;
        ja.q0 = 16 * s + 4 * lg;
        ja.lr = lr;
        ja.P = P;
        ja.diag = causal != 0;
        ja.tail = tail && ntl == nt;
        ja.scale_log2e = scale_log2e;
        // as soon as the MFMAs of this job are done its Q registers take the next job's Q; the
        // softmax below and the other resident waves cover the load latency
        auto next_q = [&]() {
            if (job + 1 < n_jobs) {
                const int hn = (job + 1) / n_strips, sn = (job + 1) - hn * n_strips;
                load_q(h0 + hn, sn ? sB : sA, qv);
            }
        };
        switch (ntl) {
#define MUKV_JOB_CASE(N) case N: strip_job<N>(ja, qv, acc, next_q); break;
            MUKV_JOB_CASE(1) MUKV_JOB_CASE(2) MUKV_JOB_CASE(3) MUKV_JOB_CASE(4) MUKV_JOB_CASE(5)
            MUKV_JOB_CASE(6) MUKV_JOB_CASE(7) MUKV_JOB_CASE(8) MUKV_JOB_CASE(9) MUKV_JOB_CASE(10)
            MUKV_JOB_CASE(11) MUKV_JOB_CASE(12) MUKV_JOB_CASE(13)
#undef MUKV_JOB_CASE
        default: break;
        }
    }
    // column sums: add the four lane groups (the other query rows), then the waves in a fixed order
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
        out[((int64_t)f * n_part + blockIdx.y) * P + j] = s;
    }
}

bool att_mfma_supported(const mukv_config &c) {
    return c.dtype == MUKV_BF16 && c.head_dim == kHeadDim && c.tokens_per_frame <= kMaxTiles * 16;
}

hipError_t launch_att_mfma(const Ctx &c, const ChunkArgs &a, float *out, int *n_part, hipStream_t st) {
    const int P = c.cfg.tokens_per_frame, Hq = c.cfg.n_q_heads, G = c.group;
    const int nt = (P + 15) / 16;
    // few frames: one head per workgroup and one strip per wave (fills the chip, shortest critical
    // path); many frames: a whole KV group per workgroup, two strips per wave (K staged once per
    // group, balanced waves)
    const bool many = (int64_t)a.n_frames * Hq > 4096;
    const int hpw = many ? G : 1;
    const int pair = many ? 1 : 0;
    const int n_split = (!pair && nt > 7) ? 2 : 1;
    const int waves = pair ? (nt + 1) / 2 : (nt + n_split - 1) / n_split;
    *n_part = (Hq / hpw) * n_split;
    const size_t lds = (size_t)nt * 16 * kLdsRow * 2 + (size_t)waves * nt * 16 * sizeof(float);
    const float scale_log2e = 1.4426950408889634f / sqrtf((float)c.cfg.head_dim);
    hipLaunchKernelGGL(att_mfma_kernel, dim3(a.n_frames, *n_part), dim3(waves * 64), lds, st, a.q, a.k, a.map,
                       (int64_t)c.ls * a.kv_sl, a.q_sh, a.q_st, a.kv_sh, a.kv_st, P, nt, G, hpw, c.cfg.causal, pair,
                       n_split, scale_log2e, *n_part, out);
    return hipGetLastError();
}

} // namespace mukv
