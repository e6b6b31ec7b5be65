// Eq. 1 (attention received per token) on the CDNA4 matrix cores as a launch of its own: the kernel
// around att_mfma_body (att_mfma_dev.h) and its launcher.
#include <cmath>
#include <cstring>
#include <vector>

#include "att_mfma_dev.h"

namespace mukv {

__global__ __launch_bounds__(448) __attribute__((amdgpu_waves_per_eu(4, 4))) void att_mfma_kernel(PtrTable qtab, PtrTable ktab, FrameMap map,
                                                                                                 AttMfmaArgs aa) {
    extern __shared__ __align__(16) unsigned char smem_raw[];
    att_mfma_body(qtab, ktab, map, aa, blockIdx.x, blockIdx.y, smem_raw);
}

bool att_mfma_supported(const mukv_config &c) {
    return c.dtype == MUKV_BF16 && c.head_dim == kHeadDim && c.tokens_per_frame <= kMaxTiles * 16;
}

bool att_mfma_many(const Ctx &c, int n_frames) { return (int64_t)n_frames * c.cfg.n_q_heads >= 1792; }

void att_mfma_plan(const Ctx &c, const ChunkArgs &a, float *out, AttMfmaArgs *aa, int *waves, size_t *lds) {
    const int P = c.cfg.tokens_per_frame, Hq = c.cfg.n_q_heads, G = c.group;
    const int nt = (P + 15) / 16;
    // few frames: one head per workgroup and one strip per wave (fills the chip, shortest critical
    // path); many frames: a whole KV group per workgroup, two strips per wave (K staged once per
    // group, balanced waves)
    const bool many = att_mfma_many(c, a.n_frames);
    aa->hpw = many ? G : 1;
    aa->pair = many ? 1 : 0;
    aa->n_split = (!aa->pair && nt > 7) ? 2 : 1;
    *waves = aa->pair ? (nt + 1) / 2 : (nt + aa->n_split - 1) / aa->n_split;
    aa->n_part = (Hq / aa->hpw) * aa->n_split;
    *lds = (size_t)(nt + *waves) * kTileB; // key tiles + one query buffer per wave (>= the per-wave sums)
    aa->k_off = (int64_t)c.ls * a.kv_sl;
    aa->q_sh = a.q_sh;
    aa->q_st = a.q_st;
    aa->k_sh = a.kv_sh;
    aa->k_st = a.kv_st;
    aa->P = P;
    aa->nt = nt;
    aa->G = G;
    aa->causal = c.cfg.causal;
    aa->scale_log2e = 1.4426950408889634f / sqrtf((float)c.cfg.head_dim);
    aa->out = out;
    aa->dft = nullptr;
    aa->fft_out = nullptr;
}

// The matrix of the length-128 transform of real keys as matrix-core B operands (see freq_mfma_phase):
// [split 3][column tile 8][feature slice 4][lane 64][8] bf16; entry j of lane (lr, lg) of (tile ct,
// slice kk) is W[d = 32 kk + 8 lg + j][c = 16 ct + lr], W[d][c] = cos(2 pi c d / 128) for c <= 64 and
// sin(2 pi (c - 64) d / 128) above; split 0 is W rounded to bf16, split 1 the rounded rest, split 2
// the rounded rest of that.
static uint16_t bf16_rne(float x) {
    uint32_t u;
    std::memcpy(&u, &x, 4);
    return (uint16_t)((u + 0x7FFFu + ((u >> 16) & 1u)) >> 16);
}
static float bf16_to_float(uint16_t b) {
    const uint32_t u = (uint32_t)b << 16;
    float x;
    std::memcpy(&x, &u, 4);
    return x;
}
std::vector<uint16_t> dft_operand_table() {
    std::vector<uint16_t> t((size_t)kDftSplits * 8 * 4 * kDftOperand);
    for (int ct = 0; ct < 8; ++ct)
        for (int kk = 0; kk < 4; ++kk)
            for (int lane = 0; lane < 64; ++lane)
                for (int j = 0; j < 8; ++j) {
                    const int d = 32 * kk + 8 * (lane >> 4) + j, col = 16 * ct + (lane & 15);
                    const int m = col <= 64 ? col : col - 64;
                    const int r = (m * d) % 128; // the angle, reduced exactly
                    const double ang = 2.0 * 3.14159265358979323846 * (double)r / 128.0;
                    double w = col <= 64 ? std::cos(ang) : std::sin(ang);
                    if (col <= 64 && (r % 32) == 0) w = (r == 0) ? 1.0 : (r == 64 ? -1.0 : 0.0); // exact zeros and ones
                    if (col > 64 && (r % 64) == 0) w = 0.0;
                    for (int sp = 0; sp < kDftSplits; ++sp) {
                        const uint16_t b = bf16_rne((float)w);
                        t[((((size_t)sp * 8 + ct) * 4 + kk) * 64 + lane) * 8 + j] = b;
                        w -= (double)bf16_to_float(b);
                    }
                }
    return t;
}

hipError_t launch_att_mfma(const Ctx &c, const ChunkArgs &a, float *out, int *n_part, hipStream_t st) {
    AttMfmaArgs aa;
    int waves;
    size_t lds;
    att_mfma_plan(c, a, out, &aa, &waves, &lds);
    *n_part = aa.n_part;
    static bool lds_ok[kMaxDevices];
    const hipError_t ea = allow_dynamic_lds(reinterpret_cast<const void *>(&att_mfma_kernel), kAttMfmaMaxLds,
                                            c.cfg.device_id, lds_ok);
    if (ea != hipSuccess) return ea;
    hipLaunchKernelGGL(att_mfma_kernel, dim3(a.n_frames, aa.n_part), dim3(waves * 64), lds, st, a.q, a.k, a.map, aa);
    return hipGetLastError();
}

} // namespace mukv
