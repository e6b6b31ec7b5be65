// Eq. 1 (attention received per token) on the CDNA4 matrix cores as a launch of its own: the kernel
// around att_mfma_body (att_mfma_dev.h) and its launcher.
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
