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

constexpr int kMaxTiles = 13;  // 13 * 16 = 208 >= P
constexpr int kLdsRow = 136;   // bf16 elements per LDS key row: 128 + 8 of padding (272 B)
constexpr int kHeadDim = 128;

__global__ __launch_bounds__(448) void att_mfma_kernel(const uint16_t *__restrict__ q, int64_t q_sh, int64_t q_st,
                                                       const uint16_t *__restrict__ k, int64_t k_sh, int64_t k_st,
                                                       int P, int nt, int G, int hpw, int causal,
                                                       float scale_log2e, int n_part, float *__restrict__ out) {
    extern __shared__ __align__(16) unsigned char smem_raw[];
    uint16_t *Ks = reinterpret_cast<uint16_t *>(smem_raw);                           // [nt*16][kLdsRow]
    float *red = reinterpret_cast<float *>(smem_raw + (size_t)nt * 16 * kLdsRow * 2); // [waves][nt*16]
    const int f = blockIdx.x, part = blockIdx.y;
    const int h0 = part * hpw, g = h0 / G;
    const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
    const int n_threads = blockDim.x;
    const int lr = lane & 15, lg = lane >> 4;

    // stage K of (frame, KV head) in LDS; rows past P are zero
    const uint16_t *kf = k + (int64_t)g * k_sh + (int64_t)f * P * k_st;
    for (int idx = tid; idx < nt * 16 * 16; idx += n_threads) {
        const int row = idx >> 4, u = idx & 15;
        uint4 val = make_uint4(0u, 0u, 0u, 0u);
        if (row < P) val = *reinterpret_cast<const uint4 *>(kf + (int64_t)row * k_st + u * 8);
        *reinterpret_cast<uint4 *>(Ks + row * kLdsRow + u * 8) = val;
    }
    __syncthreads();

    const int sA = w, sB = nt - 1 - w;
    const int n_strips = (sA == sB) ? 1 : 2;
    f32x4 acc[kMaxTiles];
#pragma unroll
    for (int c = 0; c < kMaxTiles; ++c) acc[c] = f32x4{0.f, 0.f, 0.f, 0.f};

    const uint16_t *a_base = Ks + lr * kLdsRow + 8 * lg;
    const bool tail = (P & 15) != 0;
    for (int hh = 0; hh < hpw; ++hh) {
        const int h = h0 + hh;
        for (int si = 0; si < n_strips; ++si) {
            const int s = si ? sB : sA;
            const int qi = 16 * s + lr;
            const int qrow = qi < P ? qi : P - 1;
            const uint16_t *qp = q + (int64_t)h * q_sh + ((int64_t)f * P + qrow) * q_st + 8 * lg;
            bf16x8 qv[4];
#pragma unroll
            for (int kk = 0; kk < 4; ++kk) qv[kk] = *reinterpret_cast<const bf16x8 *>(qp + 32 * kk);
            const int cmax = causal ? s : nt - 1;
            f32x4 st[kMaxTiles];
#pragma unroll
            for (int c = 0; c < kMaxTiles; ++c) {
                if (c <= cmax) {
                    f32x4 d = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
                    for (int kk = 0; kk < 4; ++kk) {
                        const bf16x8 a = *reinterpret_cast<const bf16x8 *>(a_base + c * 16 * kLdsRow + 32 * kk);
                        d = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, qv[kk], d, 0, 0, 0);
                    }
                    st[c] = d;
                }
            }
            // masks: keys after the query on the diagonal tile, keys past P on the last tile
            float m = -INFINITY;
#pragma unroll
            for (int c = 0; c < kMaxTiles; ++c) {
                if (c <= cmax) {
                    const bool diag = causal && c == s;
                    const bool last = tail && c == nt - 1;
                    if (diag || last) {
#pragma unroll
                        for (int r = 0; r < 4; ++r) {
                            const int j = 16 * c + 4 * lg + r;
                            const bool ok = (j < P) && (!diag || j <= qi);
                            st[c][r] = ok ? st[c][r] : -INFINITY;
                        }
                    }
#pragma unroll
                    for (int r = 0; r < 4; ++r) m = fmaxf(m, st[c][r]);
                }
            }
            m = fmaxf(m, __shfl_xor(m, 16));
            m = fmaxf(m, __shfl_xor(m, 32));
            const float mb = m * scale_log2e;
            float z = 0.f;
#pragma unroll
            for (int c = 0; c < kMaxTiles; ++c) {
                if (c <= cmax) {
#pragma unroll
                    for (int r = 0; r < 4; ++r) {
                        const float p = __builtin_amdgcn_exp2f(st[c][r] * scale_log2e - mb);
                        st[c][r] = p;
                        z += p;
                    }
                }
            }
            z += __shfl_xor(z, 16);
            z += __shfl_xor(z, 32);
            const float inv = (qi < P) ? 1.0f / z : 0.0f;
#pragma unroll
            for (int c = 0; c < kMaxTiles; ++c) {
                if (c <= cmax) {
#pragma unroll
                    for (int r = 0; r < 4; ++r) acc[c][r] += st[c][r] * inv;
                }
            }
        }
    }
    // column sums over the 16 query lanes, then over the waves in a fixed order
    const int ld = nt * 16;
#pragma unroll
    for (int c = 0; c < kMaxTiles; ++c) {
        if (c < nt) {
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                float v = acc[c][r];
                v += __shfl_xor(v, 1);
                v += __shfl_xor(v, 2);
                v += __shfl_xor(v, 4);
                v += __shfl_xor(v, 8);
                if (lr == 0) red[w * ld + 16 * c + 4 * lg + r] = v;
            }
        }
    }
    __syncthreads();
    const int n_waves = n_threads >> 6;
    for (int j = tid; j < P; j += n_threads) {
        float s = 0.f;
        for (int ww = 0; ww < n_waves; ++ww) s += red[ww * ld + j];
        out[((int64_t)f * n_part + part) * P + j] = s;
    }
}

bool att_mfma_supported(const mukv_config &c) {
    return c.dtype == MUKV_BF16 && c.head_dim == kHeadDim && c.tokens_per_frame <= kMaxTiles * 16;
}

hipError_t launch_att_mfma(const Ctx &c, const ChunkArgs &a, float *out, int *n_part, hipStream_t st) {
    const int P = c.cfg.tokens_per_frame, Hq = c.cfg.n_q_heads, G = c.group;
    const int nt = (P + 15) / 16;
    const int waves = (nt + 1) / 2;
    // few frames: one head per workgroup to fill the chip; many frames: a whole KV group per
    // workgroup so that K is staged once per group
    const int hpw = ((int64_t)a.n_frames * Hq > 4096) ? G : 1;
    *n_part = Hq / hpw;
    const size_t lds = (size_t)nt * 16 * kLdsRow * 2 + (size_t)waves * nt * 16 * sizeof(float);
    const float scale_log2e = 1.4426950408889634f / sqrtf((float)c.cfg.head_dim);
    const uint16_t *k = reinterpret_cast<const uint16_t *>(a.k) + (int64_t)c.ls * a.kv_sl;
    hipLaunchKernelGGL(att_mfma_kernel, dim3(a.n_frames, *n_part), dim3(waves * 64), lds, st,
                       reinterpret_cast<const uint16_t *>(a.q), a.q_sh, a.q_st, k, a.kv_sh, a.kv_st, P, nt, G, hpw,
                       c.cfg.causal, scale_log2e, *n_part, out);
    return hipGetLastError();
}

} // namespace mukv
