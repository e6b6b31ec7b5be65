// Offline half of MuKV (Sec. 3.3 of the paper): token scoring, per-frame keep,
// KV compaction and block-key pooling for one chunk of frames.
//
// Kernel chain enqueued by launch_compress (all on the caller's stream):
//   att_generic<float> | att_mfma      Eq. 1   partial attention received per (frame, head group)
//   freq_signal<float>                 Eq. 2-3 length-D DFT magnitudes of every key
//   select_pool<float>                 Eq. 4 fusion, keep of the kappa best, Eq. 5 frame / super-patch keys
//   att_generic<double>, freq_signal<double>, select_pool<double>
//                                      the same three steps in fp64, only for frames whose
//                                      fp32 selection margin is below the threshold
//   compact                            copy of the kept rows of all layers; segment keys
#include <cstring>

#include "att_mfma_dev.h"
#include "mukv_internal.h"

namespace mukv {

// ------------------------------------------------------------------------------------------
// Eq. 2-3: frequency indicator.  A real length-D transform is done as a complex transform of
// length N = D/2 spread over N lanes (lane p holds x[2p] + i*x[2p+1]), radix-2 decimation in
// frequency with lane exchanges, then the usual split into the spectra of the even and odd
// samples.  Bins m and D-m have equal magnitude, so sum_m |X[m]| = |X[0]| + |X[D/2]| +
// 2*sum_{0<m<D/2} |X[m]|.  One wave handles 64/N tokens at a time and loops over the KV heads.
// R is the arithmetic type (float for the main path, double for re-scored frames).
// ------------------------------------------------------------------------------------------
template <typename T>
struct __align__(2 * sizeof(T)) Pair2 {
    T a, b;
};

template <int N>
__device__ __forceinline__ int bitrev(int x) {
    int r = 0;
#pragma unroll
    for (int b = 1; b < N; b <<= 1) {
        r = (r << 1) | (x & 1);
        x >>= 1;
    }
    return r;
}

__device__ __forceinline__ void sincospi_t(float x, float *s, float *c) { sincospif(x, s, c); }
__device__ __forceinline__ void sincospi_t(double x, double *s, double *c) { sincospi(x, s, c); }
__device__ __forceinline__ float sqrt_t(float x) { return sqrtf(x); }
__device__ __forceinline__ double sqrt_t(double x) { return sqrt(x); }
__device__ __forceinline__ float fma_t(float a, float b, float c) { return fmaf(a, b, c); }
__device__ __forceinline__ double fma_t(double a, double b, double c) { return fma(a, b, c); }
__device__ __forceinline__ float abs_t(float x) { return fabsf(x); }
__device__ __forceinline__ double abs_t(double x) { return fabs(x); }

// Workgroups that share the tokens of one frame (grid.y of the frequency kernel): 7 for a frame of
// up to kMaxP tokens, and as many per 196 tokens for a unit of several frames.
static inline int freq_blocks_per_frame(int P) { return P <= kMaxP ? 7 : 7 * ((P + 195) / 196); }

// sum over the N consecutive lanes of a transform (N a power of two <= 64), result in every lane
template <int N, typename R>
__device__ __forceinline__ R group_sum(R v) {
    if constexpr (N > 1) {
        v += lane_xor<N / 2>(v);
        return group_sum<N / 2>(v);
    } else {
        return v;
    }
}

// Radix-2 decimation-in-frequency stages S..LOG-1 of the N-point transform held one point per
// lane, for GH independent transforms at once.  Stage S pairs lanes N >> (S+1) apart.
template <int N, int S, int LOG, typename R, int GH>
__device__ __forceinline__ void fft_stages(R (&zr)[GH], R (&zi)[GH], const R *sg, const R *twr, const R *twi) {
    if constexpr (S < LOG) {
        constexpr int h = N >> (S + 1);
        R pr[GH], pi[GH];
#pragma unroll
        for (int u = 0; u < GH; ++u) {
            pr[u] = lane_xor<h>(zr[u]);
            pi[u] = lane_xor<h>(zi[u]);
        }
#pragma unroll
        for (int u = 0; u < GH; ++u) {
            const R tr = pr[u] + sg[S] * zr[u], ti = pi[u] + sg[S] * zi[u];
            zr[u] = tr * twr[S] - ti * twi[S];
            zi[u] = tr * twi[S] + ti * twr[S];
        }
        fft_stages<N, S + 1, LOG, R, GH>(zr, zi, sg, twr, twi);
    }
}
// grid.x of the fp64 re-scoring kernels: listed frames handled side by side (the kernels loop
// over the list from their slot).  The attention kernel's workgroups hold ~100 KB of LDS each,
// so it gets fewer slots: its idle ones still have to be placed before they can leave.
constexpr int kRescoreSlots = 4;
constexpr int kRescoreSlotsAtt = 2;
// A unit of several frames is tens of frames' worth of work and a batch holds few of them: one slot each.
static inline int rescore_slots(int P, int n_frames) { return P > kMaxP ? n_frames : kRescoreSlots; }

// Work of workgroup (bx, by) of a (gx, bpf) grid.
template <typename T, typename R, int D>
__device__ __forceinline__ void freq_body(const PtrTable &ktab, const FrameMap &map, int64_t k_off, int64_t sh,
                                          int64_t st, int Hkv, int P, const int32_t *__restrict__ flag_list,
                                          const int32_t *__restrict__ flag_count, R *__restrict__ out, int bx, int by,
                                          int gx, int bpf) {
    constexpr int N = D / 2;
    constexpr int GROUPS = kWave / N;
    constexpr int LOG = (N == 64) ? 6 : (N == 32) ? 5 : (N == 16) ? 4 : 3;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int p = lane % N, sub = lane / N;

    // Per stage and lane: the butterfly is written branch-free as (partner + sg*own) * w, with
    // sg = +1, w = 1 on the lanes that take the sum and sg = -1, w = twiddle on the others.
    R twr[LOG], twi[LOG], sg[LOG];
#pragma unroll
    for (int s = 0; s < LOG; ++s) {
        const int h = N >> (s + 1);
        sincospi_t(-(R)(p & (h - 1)) / (R)h, &twi[s], &twr[s]);
        const bool lower = (p & h) != 0;
        sg[s] = lower ? (R)-1 : (R)1;
        twr[s] = lower ? twr[s] : (R)1;
        twi[s] = lower ? twi[s] : (R)0;
    }
    const int kb = bitrev<N>(p);
    const int partner = bitrev<N>((N - kb) & (N - 1)) + sub * N;
    R uwr, uwi;
    sincospi_t(-(R)kb / (R)N, &uwi, &uwr);

    // frames: every batch frame (grid.x = n_frames), or the entries of the re-scoring list
    const int n_e = flag_list ? *flag_count : gx;
    for (int e = bx; e < n_e; e += gx) {
    const int f = flag_list ? flag_list[e] : e;
    const int slot = find_slot(map, f);
    const T *k = reinterpret_cast<const T *>(ktab.p[slot]) + k_off + (int64_t)(f - map.fstart[slot]) * P * st;
    // the workgroup's waves walk over the frame's tokens, GROUPS tokens per wave and step
    const int n_waves = blockDim.x >> 6;
    const int stride = bpf * n_waves * GROUPS;
    // Up to four heads of a token are transformed together (independent butterflies hide the
    // lane-exchange latency), and the key elements of the next group are loaded before the
    // current group is computed.
    constexpr int GH = 4;
    const int t_first = (by * n_waves + wave) * GROUPS;
    auto load_group = [&](int t0, int g0, T *a0, T *a1) {
        const int tok = t0 + sub < P ? t0 + sub : P - 1;
        const T *r = k + (int64_t)tok * st + 2 * p;
#pragma unroll
        for (int u = 0; u < GH; ++u) { // both elements of the lane in one load
            const Pair2<T> pr = *reinterpret_cast<const Pair2<T> *>(r + (int64_t)(g0 + u < Hkv ? g0 + u : Hkv - 1) * sh);
            a0[u] = pr.a;
            a1[u] = pr.b;
        }
    };
    T n0[GH], n1[GH];
    if (t_first < P) load_group(t_first, 0, n0, n1);
    for (int t0 = t_first; t0 < P; t0 += stride) {
        const int tok = t0 + sub;
        const bool valid = tok < P;
        R total = 0;
        for (int g0 = 0; g0 < Hkv; g0 += GH) {
            R zr[GH], zi[GH];
#pragma unroll
            for (int u = 0; u < GH; ++u) {
                zr[u] = (R)to_float(n0[u]);
                zi[u] = (R)to_float(n1[u]);
            }
            {   // next group: further heads of this token, else the first heads of the wave's next token
                const bool wrap = g0 + GH >= Hkv;
                const int tn = wrap ? t0 + stride : t0;
                load_group(tn < P ? tn : t0, wrap ? 0 : g0 + GH, n0, n1);
            }
            fft_stages<N, 0, LOG, R, GH>(zr, zi, sg, twr, twi);
            // lane p now holds Z[kb]; fetch Z[(N-kb) mod N]
            R pr[GH], pi[GH];
#pragma unroll
            for (int u = 0; u < GH; ++u) {
                pr[u] = __shfl(zr[u], partner);
                pi[u] = __shfl(zi[u], partner);
            }
#pragma unroll
            for (int u = 0; u < GH; ++u) {
                const R er = (R)0.5 * (zr[u] + pr[u]), ei = (R)0.5 * (zi[u] - pi[u]);
                const R odr = (R)0.5 * (zi[u] + pi[u]), odi = (R)-0.5 * (zr[u] - pr[u]);
                const R xr = er + (odr * uwr - odi * uwi);
                const R xi = ei + (odr * uwi + odi * uwr);
                const R c_mid = (R)2 * sqrt_t(xr * xr + xi * xi);
                const R c_end = abs_t(zr[u] + zi[u]) + abs_t(zr[u] - zi[u]); // bins 0 and D/2 (lane with kb = 0)
                const R c = (kb == 0) ? c_end : c_mid;
                total += (g0 + u < Hkv) ? c : (R)0;
            }
        }
        total = group_sum<N>(total);
        if (p == 0 && valid) out[(int64_t)f * P + tok] = total / (R)(Hkv * D);
    }
    }
}

template <typename T, typename R, int D>
__global__ __launch_bounds__(256) void freq_signal_kernel(PtrTable ktab, FrameMap map, int64_t k_off, int64_t sh,
                                                          int64_t st, int Hkv, int P,
                                                          const int32_t *__restrict__ flag_list,
                                                          const int32_t *__restrict__ flag_count,
                                                          R *__restrict__ out) {
    freq_body<T, R, D>(ktab, map, k_off, sh, st, Hkv, P, flag_list, flag_count, out, blockIdx.x, blockIdx.y, gridDim.x,
                       gridDim.y);
}

// ------------------------------------------------------------------------------------------
// Eq. 2-3 with the transform along the TOKEN axis of the frame (the other reading of Eq. 2):
//   Z[m][c] = sum_j K[j][c] exp(-2 pi i m j / P),  I[m] = mean_c |Z[m][c]|,  c over Hkv*D features.
// A direct DFT: P is any number up to 256 (196 = 4*7*7 in the paper's setting).  The keys are real,
// so rows m and P-m have the same magnitude: rows 0..P/2 are evaluated and the rows above copy
// their mirror row, which keeps that tie exact.  For the same reason tokens j and P-j share their
// factors up to a sign: with e_j = k_j + k_{P-j}, o_j = k_j - k_{P-j} (1 <= j < P/2)
//   Re Z[m] = k_0 + sum_j e_j cos(2 pi m j/P) (+ k_{P/2} cos(pi m)),  Im Z[m] = -sum_j o_j sin(2 pi m j/P),
// half the multiply-adds of the plain sum.
// freq_token_kernel: one workgroup per (frame, group of 64 features).  The frame's [P][64] slice is
// staged in LDS (as R) and folded in place (slot j: e_j, slot P-j: o_j, slot P: zero); lane =
// feature, wave w owns rows m = w, w+4, ..., kTokBins of them at a time, so a staged value is read
// once per kTokBins rows; the (cos, -sin) factors of a (row, token) pair are the same for the whole
// wave and come from a table through scalar loads.  |Z| is summed over the lanes.
// freq_token_finish_kernel adds the feature groups in order and writes both mirror rows.
// ------------------------------------------------------------------------------------------
constexpr int kTokBins = 4;
constexpr int kTokStep = 8; // tokens per batch of loads
template <typename T, typename R>
__global__ __launch_bounds__(256) void freq_token_kernel(PtrTable ktab, FrameMap map, int64_t k_off, int64_t sh,
                                                         int64_t st, int Hkv, int D, int P,
                                                         const R *__restrict__ tw, // [P/2+1][P/2+1][2]
                                                         const int32_t *__restrict__ flag_list,
                                                         const int32_t *__restrict__ flag_count,
                                                         R *__restrict__ part, // [frame][group][P/2+1]
                                                         int n_frames) {
    extern __shared__ __align__(16) unsigned char smem_tok[];
    R *X = reinterpret_cast<R *>(smem_tok); // [P+1][64]
    const int lane = threadIdx.x & 63;
    const int w = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int C = Hkv * D, hc = P / 2 + 1, n_groups = gridDim.y, grp = blockIdx.y;
    const int c = grp * 64 + lane;
    const bool live = c < C;
    const int cc = live ? c : C - 1; // loads stay unconditional
    const int n_e = flag_list ? *flag_count : n_frames;
    for (int e = blockIdx.x; e < n_e; e += gridDim.x) {
        const int f = flag_list ? flag_list[e] : e;
        const int slot = find_slot(map, f);
        const T *col = reinterpret_cast<const T *>(ktab.p[slot]) + k_off + (int64_t)(f - map.fstart[slot]) * P * st +
                       (int64_t)(cc / D) * sh + (cc % D);
        for (int j0 = w; j0 < P; j0 += 4 * 8) { // 8 independent loads per lane
            T v[8];
#pragma unroll
            for (int u = 0; u < 8; ++u) v[u] = col[(int64_t)(j0 + 4 * u < P ? j0 + 4 * u : P - 1) * st];
#pragma unroll
            for (int u = 0; u < 8; ++u)
                if (j0 + 4 * u < P) X[(j0 + 4 * u) * 64 + lane] = live ? (R)to_float(v[u]) : (R)0;
        }
        if (w == 0) X[P * 64 + lane] = (R)0;
        __syncthreads();
        for (int j = 1 + w; 2 * j < P; j += 4) { // fold: a pair of slots belongs to one wave
            const R a = X[j * 64 + lane], b = X[(P - j) * 64 + lane];
            X[j * 64 + lane] = a + b;
            X[(P - j) * 64 + lane] = a - b;
        }
        __syncthreads();
        for (int m0 = w; m0 < hc; m0 += 4 * kTokBins) {
            R re[kTokBins], im[kTokBins];
            const R *row[kTokBins];
#pragma unroll
            for (int b = 0; b < kTokBins; ++b) {
                re[b] = im[b] = (R)0;
                const int m = m0 + 4 * b < hc ? m0 + 4 * b : hc - 1; // a row past the end repeats the last one
                row[b] = tw + (size_t)m * hc * 2;
            }
            // token pairs in batches of kTokStep: their staged values and the factors (scalar
            // loads of consecutive table entries) are requested together; then the remaining ones
            int j0 = 0;
            for (; j0 + kTokStep <= hc; j0 += kTokStep) {
                R xe[kTokStep], xo[kTokStep];
#pragma unroll
                for (int u = 0; u < kTokStep; ++u) {
                    xe[u] = X[(j0 + u) * 64 + lane];
                    xo[u] = X[(P - j0 - u) * 64 + lane];
                }
#pragma unroll
                for (int b = 0; b < kTokBins; ++b) {
                    const R *t = row[b] + 2 * j0;
#pragma unroll
                    for (int u = 0; u < kTokStep; ++u) {
                        re[b] = fma_t(xe[u], t[2 * u], re[b]);
                        im[b] = fma_t(xo[u], t[2 * u + 1], im[b]);
                    }
                }
            }
            for (int j = j0; j < hc; ++j) {
                const R xe = X[j * 64 + lane], xo = X[(P - j) * 64 + lane];
#pragma unroll
                for (int b = 0; b < kTokBins; ++b) {
                    re[b] = fma_t(xe, row[b][2 * j], re[b]);
                    im[b] = fma_t(xo, row[b][2 * j + 1], im[b]);
                }
            }
#pragma unroll
            for (int b = 0; b < kTokBins; ++b) {
                const R mag = wave_sum(sqrt_t(re[b] * re[b] + im[b] * im[b])); // dead lanes hold zeros
                if (lane == 0 && m0 + 4 * b < hc) part[((int64_t)f * n_groups + grp) * hc + m0 + 4 * b] = mag;
            }
        }
        __syncthreads(); // the slice is restaged for the next listed frame
    }
}

template <typename R>
__global__ __launch_bounds__(256) void freq_token_finish_kernel(const R *__restrict__ part, int n_groups, int P, int C,
                                                                const int32_t *__restrict__ flag_list,
                                                                const int32_t *__restrict__ flag_count,
                                                                R *__restrict__ out, int n_frames) {
    const int hc = P / 2 + 1;
    const int n_e = flag_list ? *flag_count : n_frames;
    for (int e = blockIdx.x; e < n_e; e += gridDim.x) {
        const int f = flag_list ? flag_list[e] : e;
        for (int m = threadIdx.x; m < hc; m += 256) {
            R s = (R)0;
            for (int g = 0; g < n_groups; ++g) s += part[((int64_t)f * n_groups + g) * hc + m];
            const R val = s / (R)C;
            out[(int64_t)f * P + m] = val;
            if (m > 0 && P - m > m) out[(int64_t)f * P + P - m] = val;
        }
    }
}

// ------------------------------------------------------------------------------------------
// Eq. 1, generic path (any dtype, any D, P <= 256), also the fp64 re-scoring path.
// Grid (frame, query head, query range): a workgroup stages the frame's keys in LDS as float
// (exact for bf16 and fp32 payloads) and handles kGenQ consecutive queries per round, four per
// wave at once: lanes own keys j = lane + 64*t, every LDS key value read is used for four
// queries, the row softmax uses wave reductions, and each lane accumulates the probabilities of
// its keys.  Per-wave partial column sums are combined in a fixed order, so results are
// run-to-run identical.
// out: [frame][Hq * gridDim.z][P] (R) partial sums over this workgroup's query rows.
// ------------------------------------------------------------------------------------------
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

// 16 bytes of payload -> floats in LDS (8 bf16 or 4 fp32 values)
template <typename T>
__device__ __forceinline__ void unpack_to_float(u32x4 raw, float *dst);
template <>
__device__ __forceinline__ void unpack_to_float<uint16_t>(u32x4 raw, float *dst) {
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        dst[2 * i] = __uint_as_float(raw[i] << 16);
        dst[2 * i + 1] = __uint_as_float(raw[i] & 0xffff0000u);
    }
}
template <>
__device__ __forceinline__ void unpack_to_float<float>(u32x4 raw, float *dst) {
#pragma unroll
    for (int i = 0; i < 4; ++i) dst[i] = __uint_as_float(raw[i]);
}

__device__ __forceinline__ float exp_t(float x) { return expf(x); }
__device__ __forceinline__ double exp_t(double x) { return exp(x); }

constexpr int kGenQ = 16; // queries per round of a workgroup: 4 waves x 4

// How the generic attention kernel keeps a frame's keys in LDS.  The fp32 pass, which runs on every
// frame, keeps them expanded to float (its inner loop lives on LDS bandwidth).  The fp64 pass runs on a
// few listed frames beside the next batch's kernels, whose workgroups leave less than half of a compute
// unit's LDS free: it keeps bf16 keys as they are (half the room; the expansion is a shift).
template <typename T, typename R>
struct KeyStage {
    typedef float type;
    static constexpr int pad = 4;
};
template <>
struct KeyStage<uint16_t, double> {
    typedef uint16_t type;
    static constexpr int pad = 8;
};
__device__ __forceinline__ float4 key4(const float *p) { return *reinterpret_cast<const float4 *>(p); }
__device__ __forceinline__ float4 key4(const uint16_t *p) {
    const uint2 raw = *reinterpret_cast<const uint2 *>(p);
    return make_float4(__uint_as_float(raw.x << 16), __uint_as_float(raw.x & 0xffff0000u), __uint_as_float(raw.y << 16),
                       __uint_as_float(raw.y & 0xffff0000u));
}
__device__ __forceinline__ void stage_keys(u32x4 raw, uint16_t *dst) { *reinterpret_cast<u32x4 *>(dst) = raw; }

template <typename T, typename R>
__global__ __launch_bounds__(256) void att_generic_kernel(PtrTable qtab, PtrTable ktab, FrameMap map, int64_t k_off,
                                                          int64_t q_sh, int64_t q_st, int64_t k_sh, int64_t k_st,
                                                          int P, int D, int G, int Hq, int causal, int q_per_block,
                                                          const int32_t *__restrict__ flag_list,
                                                          const int32_t *__restrict__ flag_count,
                                                          R *__restrict__ out) {
    extern __shared__ __align__(16) unsigned char smem_raw[];
    const int h = blockIdx.y, z = blockIdx.z;
    // frames: every batch frame (grid.x = n_frames), or the entries of the re-scoring list
    const int n_e = flag_list ? *flag_count : (int)gridDim.x;
    for (int e_idx = blockIdx.x; e_idx < n_e; e_idx += gridDim.x) {
    const int f = flag_list ? flag_list[e_idx] : e_idx;
    typedef typename KeyStage<T, R>::type KT;
    const int ldk = D + KeyStage<T, R>::pad; // 16-byte aligned rows; 4-word lane stride keeps 16 lanes on distinct banks
    KT *Ks = reinterpret_cast<KT *>(smem_raw);          // [P][ldk]
    float *qs = reinterpret_cast<float *>(smem_raw + att_generic_key_bytes(P, D, sizeof(KT))); // [kGenQ][D]
    R *part = reinterpret_cast<R *>(qs + kGenQ * D);    // [4][P], 8-byte aligned
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int slot = find_slot(map, f);
    const int lf = f - map.fstart[slot];
    const T *kf = reinterpret_cast<const T *>(ktab.p[slot]) + k_off + (int64_t)(h / G) * k_sh + (int64_t)lf * P * k_st;
    const T *qf = reinterpret_cast<const T *>(qtab.p[slot]) + (int64_t)h * q_sh + (int64_t)lf * P * q_st;
    const int i_lo = z * q_per_block;
    const int i_hi = (i_lo + q_per_block < P) ? i_lo + q_per_block : P;
    const int n_keys = causal ? i_hi : P; // keys any query of this workgroup can see
    // stage keys: 16-byte units, eight loads in flight per thread
    constexpr int EPU = 16 / sizeof(T);          // elements per unit
    const int upr = D / EPU;                      // units per row (D*sizeof(T) is a multiple of 16)
    const int n_ku = n_keys * upr;
    for (int u0 = tid; u0 < n_ku; u0 += 8 * 256) {
        u32x4 raw[8];
#pragma unroll
        for (int b = 0; b < 8; ++b) {
            const int u = u0 + b * 256 < n_ku ? u0 + b * 256 : n_ku - 1;
            const int j = u / upr, c = u - j * upr;
            raw[b] = *reinterpret_cast<const u32x4 *>(kf + (int64_t)j * k_st + c * EPU);
        }
#pragma unroll
        for (int b = 0; b < 8; ++b) {
            const int u = u0 + b * 256;
            if (u < n_ku) {
                const int j = u / upr, c = u - j * upr;
                if constexpr (sizeof(KT) == sizeof(float))
                    unpack_to_float<T>(raw[b], reinterpret_cast<float *>(Ks) + j * ldk + c * EPU);
                else
                    stage_keys(raw[b], Ks + j * ldk + c * EPU);
            }
        }
    }
    const R scale = (R)1 / sqrt_t((R)D);
    R acc[4] = {0, 0, 0, 0};
    for (int i0 = i_lo; i0 < i_hi; i0 += kGenQ) {
        __syncthreads();
        for (int u = tid; u < kGenQ * upr; u += 256) {
            const int qi = u / upr, c = u - qi * upr;
            const int i = i0 + qi < i_hi ? i0 + qi : i_hi - 1;
            const u32x4 raw = *reinterpret_cast<const u32x4 *>(qf + (int64_t)i * q_st + c * EPU);
            unpack_to_float<T>(raw, qs + qi * D + c * EPU);
        }
        __syncthreads();
        const int iw = i0 + 4 * wave; // this wave's four queries: iw .. iw+3
        if (iw >= i_hi) continue;
        const int i_last = iw + 3 < i_hi ? iw + 3 : i_hi - 1;
        const int nj_max = causal ? i_last + 1 : P;
        R s[4][4];
#pragma unroll
        for (int u = 0; u < 4; ++u)
#pragma unroll
            for (int t = 0; t < 4; ++t) s[u][t] = 0;
        const float *qr = qs + (4 * wave) * D;
        int jrow[4];
#pragma unroll
        for (int t = 0; t < 4; ++t) {
            const int j = lane + 64 * t;
            jrow[t] = (j < nj_max ? j : nj_max - 1) * ldk;
        }
        for (int d = 0; d < D; d += 4) { // 8 x 16-byte LDS reads feed 64 multiply-adds
            float4 qv[4], kv[4];
#pragma unroll
            for (int u = 0; u < 4; ++u) qv[u] = *reinterpret_cast<const float4 *>(qr + u * D + d);
#pragma unroll
            for (int t = 0; t < 4; ++t) kv[t] = key4(Ks + jrow[t] + d);
#pragma unroll
            for (int t = 0; t < 4; ++t)
#pragma unroll
                for (int u = 0; u < 4; ++u) {
                    R a = s[u][t];
                    a += (R)qv[u].x * (R)kv[t].x;
                    a += (R)qv[u].y * (R)kv[t].y;
                    a += (R)qv[u].z * (R)kv[t].z;
                    a += (R)qv[u].w * (R)kv[t].w;
                    s[u][t] = a;
                }
        }
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const int i = iw + u;
            if (i >= i_hi) break;
            const int nj = causal ? i + 1 : P;
            R m = -INFINITY;
#pragma unroll
            for (int t = 0; t < 4; ++t) {
                const int j = lane + 64 * t;
                s[u][t] = (j < nj) ? s[u][t] * scale : (R)-INFINITY;
                m = s[u][t] > m ? s[u][t] : m;
            }
            m = wave_max(m);
            R zsum = 0;
#pragma unroll
            for (int t = 0; t < 4; ++t) {
                const int j = lane + 64 * t;
                s[u][t] = (j < nj) ? exp_t(s[u][t] - m) : (R)0;
                zsum += s[u][t];
            }
            zsum = wave_sum(zsum);
#pragma unroll
            for (int t = 0; t < 4; ++t) acc[t] += s[u][t] / zsum;
        }
    }
    __syncthreads();
#pragma unroll
    for (int t = 0; t < 4; ++t) {
        const int j = lane + 64 * t;
        if (j < P) part[wave * P + j] = acc[t];
    }
    __syncthreads();
    const int n_part = Hq * gridDim.z;
    for (int j = tid; j < P; j += 256)
        out[((int64_t)f * n_part + h * gridDim.z + z) * P + j] = ((part[j] + part[P + j]) + part[2 * P + j]) + part[3 * P + j];
    __syncthreads();
    }
}

// ------------------------------------------------------------------------------------------
// Eq. 4 fusion, per-frame keep (Sec. 3.3, granularity-adaptive compression with the frame as
// the unit) and Eq. 5 block keys for the frame and its super-patches.  One workgroup of 256
// threads per frame, thread j owns token j (P <= 256).
// Ranking is by counting: rank(j) = #{i : I[i] > I[j] or (I[i] == I[j] and i < j)}, so equal
// scores resolve to the lowest position; token j is kept iff rank(j) < kappa.
// Pooled sums are accumulated in fp64 (exact for bf16 / fp32 payloads of ordinary dynamic
// range), divided once and rounded once to float.
// ------------------------------------------------------------------------------------------
template <typename R>
struct SelectArgs {
    const R *att;       // [n_frames][n_part][P] partial sums, or NULL (alpha == 0)
    int n_part;
    R att_scale;        // 1/(Hq*P) for partial sums, 1 for a caller-supplied signal
    PtrTable att_in;    // per slot: caller-supplied float [n][P]
    bool have_att_in;
    const R *fft;       // [n_frames][P], or NULL (alpha == 1)
    int fft_parts;      // > 0: fft is [n_frames][fft_parts][P] partial sums (one per KV head), to be added in order
    R fft_scale;        //      and scaled by this (1 / (Hkv * D))
    R alpha;
    int P, kappa, S, Hkv, D;
    int64_t frame0;
    PtrTable k, v;      // per slot: chunk base
    FrameMap map;
    int64_t k_off;      // element offset of the scoring layer
    int64_t sh, st;
    R margin_thr;
    int pass2;          // 1: fp64 pass over the frames listed by pass 1
    int32_t *flag_list; // batch frames whose fp32 margin is below the threshold (written by pass 1)
    int32_t *flag_count;
    int32_t *kept_idx;
    int32_t *src_tok;
    float *rep_frame_k, *rep_frame_v, *rep_patch_k, *rep_patch_v;
    int32_t *cnt_patch;
    double *fsum_k, *fsum_v;
    float *margin;
    int32_t *refined;
    OutTable dbg_att, dbg_fft, dbg_fused; // per slot, float [n][P], entries may be null
    bool have_dbg;
};

template <typename R>
__device__ __forceinline__ void block_minmax(R v, bool valid, R *red, R &lo, R &hi) {
    R mn = valid ? v : (R)INFINITY, mx = valid ? v : (R)-INFINITY;
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) {
        const R a = __shfl_xor(mn, o), b = __shfl_xor(mx, o);
        mn = a < mn ? a : mn;
        mx = b > mx ? b : mx;
    }
    const int wave = threadIdx.x >> 6;
    __syncthreads();
    if ((threadIdx.x & 63) == 0) {
        red[wave] = mn;
        red[4 + wave] = mx;
    }
    __syncthreads();
    lo = red[0];
    hi = red[4];
#pragma unroll
    for (int w = 1; w < 4; ++w) {
        lo = red[w] < lo ? red[w] : lo;
        hi = red[4 + w] > hi ? red[4 + w] : hi;
    }
}

template <typename T, typename R>
__global__ __launch_bounds__(256) void select_pool_kernel(SelectArgs<R> a) {
    __shared__ R sc[kMaxP];
    __shared__ R red[8];
    __shared__ R vk[2];
    __shared__ int kl[kMaxP];
    __shared__ int wcnt[4];
    const int j = threadIdx.x;
    const int P = a.P, kappa = a.kappa;
    const int n_e = a.pass2 ? *a.flag_count : (int)gridDim.x;
    for (int e_idx = blockIdx.x; e_idx < n_e; e_idx += gridDim.x) {
    const int f = a.pass2 ? a.flag_list[e_idx] : e_idx;
    const int64_t gf = a.frame0 + f;
    const bool valid = j < P;
    const int slot = find_slot(a.map, f);
    const int lf = f - a.map.fstart[slot];
    float *dbg_att = a.have_dbg ? a.dbg_att.p[slot] : nullptr;
    float *dbg_fft = a.have_dbg ? a.dbg_fft.p[slot] : nullptr;
    float *dbg_fused = a.have_dbg ? a.dbg_fused.p[slot] : nullptr;

    R av = 0, fv = 0;
    if (valid && a.alpha != (R)0) {
        if (a.have_att_in) {
            av = (R) reinterpret_cast<const float *>(a.att_in.p[slot])[(int64_t)lf * P + j];
        } else {
            const R *pp = a.att + (int64_t)f * a.n_part * P + j;
            constexpr int kPB = 16;
            for (int n0 = 0; n0 < a.n_part; n0 += kPB) { // fixed summation order, kPB loads in flight
                R t[kPB];
#pragma unroll
                for (int u = 0; u < kPB; ++u) t[u] = pp[(int64_t)(n0 + u < a.n_part ? n0 + u : a.n_part - 1) * P];
#pragma unroll
                for (int u = 0; u < kPB; ++u)
                    if (n0 + u < a.n_part) av += t[u];
            }
            av *= a.att_scale;
        }
    }
    if (valid && a.alpha != (R)1) {
        if (a.fft_parts > 0) {
            R sum = 0;
            for (int pt = 0; pt < a.fft_parts; ++pt) sum += a.fft[((int64_t)f * a.fft_parts + pt) * P + j];
            fv = sum * a.fft_scale;
        } else {
            fv = a.fft[(int64_t)f * P + j];
        }
    }
    if (valid && dbg_att) dbg_att[(int64_t)lf * P + j] = (float)av;
    if (valid && dbg_fft) dbg_fft[(int64_t)lf * P + j] = (float)fv;

    R lo, hi;
    R fused = 0;
    if (a.alpha != (R)0) {
        block_minmax(av, valid, red, lo, hi);
        const R an = (hi > lo) ? (av - lo) / (hi - lo) : (R)0;
        fused = a.alpha * an;
    }
    if (a.alpha != (R)1) {
        block_minmax(fv, valid, red, lo, hi);
        const R fn = (hi > lo) ? (fv - lo) / (hi - lo) : (R)0;
        fused += ((R)1 - a.alpha) * fn;
    }
    if (valid) {
        sc[j] = fused;
        if (dbg_fused) dbg_fused[(int64_t)lf * P + j] = (float)fused;
    }
    if (j < 2) vk[j] = 0;
    __syncthreads();

    int rank = 0;
    if (valid) {
        for (int i = 0; i < P; ++i) {
            const R o = sc[i];
            rank += (o > fused) || (o == fused && i < j);
        }
        if (rank == kappa - 1) vk[0] = fused;
        if (rank == kappa) vk[1] = fused;
    }
    {   // position of a kept token among the kept ones: ballot prefix inside the wave + wave offsets
        const bool kept = valid && rank < kappa;
        const uint64_t bal = __ballot(kept);
        if ((j & 63) == 0) wcnt[j >> 6] = __popcll(bal);
        __syncthreads();
        int pos = __popcll(bal & ((1ull << (j & 63)) - 1ull));
        for (int w = 0; w < (j >> 6); ++w) pos += wcnt[w];
        // selection margin: gap between the last kept and the first dropped fused score.  A pass-1
        // frame whose margin is below the threshold goes on the re-scoring list; its rows are
        // marked -1 so that the main copy leaves them to the fp64 pass.
        const R mg = (kappa < P) ? vk[0] - vk[1] : (R)INFINITY;
        const bool flag = !a.pass2 && a.margin_thr > (R)0 && mg < a.margin_thr;
        if (kept) {
            kl[pos] = j;
            a.kept_idx[gf * kappa + pos] = j;
            a.src_tok[(int64_t)f * kappa + pos] = flag ? -1 : lf * P + j; // token inside the slot's chunk
        }
        if (j == 0) {
            a.margin[gf] = (float)mg;
            a.refined[gf] = (a.pass2 || flag) ? 1 : 0;
            if (flag) a.flag_list[atomicAdd(a.flag_count, 1)] = f; // order is irrelevant: frames are independent
        }
    }
    __syncthreads();

    // Eq. 5 for the frame and its S super-patches, K and V together.  A thread owns two adjacent
    // channels (one 4- or 8-byte load per row) and fetches the kept rows in batches of kBatch
    // independent loads; kl is ascending, so a super-patch ends when a position reaches its end.
    constexpr int kBatch = 12;
    const int C = a.Hkv * a.D;
    const int len = P / a.S;
    const T *xk = reinterpret_cast<const T *>(a.k.p[slot]) + a.k_off;
    const T *xv = reinterpret_cast<const T *>(a.v.p[slot]) + a.k_off;
    for (int cp = j; cp < C / 2; cp += 256) {
        const int c = 2 * cp;
        const int g = c / a.D, d = c - g * a.D;
        const int64_t col = (int64_t)g * a.sh + d + (int64_t)lf * P * a.st;
        double run[4] = {0.0, 0.0, 0.0, 0.0}, tot[4] = {0.0, 0.0, 0.0, 0.0}; // k0 k1 v0 v1
        int cnt = 0, s = 0;
        int end = (a.S == 1) ? P : len;
        auto flush = [&]() {
            const int64_t o = (gf * a.S + s) * C + c;
            a.rep_patch_k[o] = cnt ? (float)(run[0] / (double)cnt) : 0.0f;
            a.rep_patch_k[o + 1] = cnt ? (float)(run[1] / (double)cnt) : 0.0f;
            a.rep_patch_v[o] = cnt ? (float)(run[2] / (double)cnt) : 0.0f;
            a.rep_patch_v[o + 1] = cnt ? (float)(run[3] / (double)cnt) : 0.0f;
            if (c == 0) a.cnt_patch[gf * a.S + s] = cnt;
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                tot[e] += run[e];
                run[e] = 0.0;
            }
            cnt = 0;
            ++s;
            end = (s == a.S - 1) ? P : (s + 1) * len;
        };
        for (int r0 = 0; r0 < kappa; r0 += kBatch) {
            Pair2<T> vk[kBatch], vv[kBatch];
#pragma unroll
            for (int u = 0; u < kBatch; ++u) {
                const int r = r0 + u < kappa ? r0 + u : kappa - 1; // clamped: loads stay unconditional
                const int64_t off = col + (int64_t)kl[r] * a.st;
                vk[u] = *reinterpret_cast<const Pair2<T> *>(xk + off);
                vv[u] = *reinterpret_cast<const Pair2<T> *>(xv + off);
            }
#pragma unroll
            for (int u = 0; u < kBatch; ++u) {
                if (r0 + u < kappa) {
                    const int pos = kl[r0 + u];
                    while (pos >= end) flush();
                    run[0] += (double)to_float(vk[u].a);
                    run[1] += (double)to_float(vk[u].b);
                    run[2] += (double)to_float(vv[u].a);
                    run[3] += (double)to_float(vv[u].b);
                    ++cnt;
                }
            }
        }
        while (s < a.S) flush();
        const int64_t o = gf * C + c;
        a.fsum_k[o] = tot[0];
        a.fsum_k[o + 1] = tot[1];
        a.fsum_v[o] = tot[2];
        a.fsum_v[o + 1] = tot[3];
        a.rep_frame_k[o] = (float)(tot[0] / (double)kappa);
        a.rep_frame_k[o + 1] = (float)(tot[1] / (double)kappa);
        a.rep_frame_v[o] = (float)(tot[2] / (double)kappa);
        a.rep_frame_v[o + 1] = (float)(tot[3] / (double)kappa);
    }
    __syncthreads();
    }
}

// ------------------------------------------------------------------------------------------
// Units of more than kMaxP tokens: several frames, up to a segment, ranked as ONE unit of Eq. 4
// (Sec. 3.3 at the coarsest granularity keeps a fraction of the segment's tokens wherever they
// lie).  P <= kMaxUnit.  The attention signal of such a unit is the caller's: the prefill that
// produced the keys has it.  Two kernels take the place of select_pool_kernel.
//
// select_large_kernel: one workgroup of 1024 threads per unit, thread t owns the kUnitTok
// consecutive tokens from kUnitTok * t.  Fused scores become order-preserving unsigned keys
// (a padding token gets key 0, below every real one).  The kappa-th largest key is built bit by
// bit from the top: the largest value x with #{key >= x} >= kappa.  Tokens above it are kept;
// of those equal to it the lowest positions, by a prefix count; a second prefix count gives each
// kept token its row.  Same outputs as select_pool_kernel up to the kept list.
//
// pool_large_kernel: Eq. 5 for the unit and its S super-patches.  Grid (unit, group of 64 channel
// pairs); the unit's kept list sits in LDS; the kept rows of a super-patch are a run of that list
// (positions ascend), found by bisection; the 16 waves take every 16th row of the run, a batch of
// independent loads at a time, and their fp64 sums are joined in wave order.
// ------------------------------------------------------------------------------------------
constexpr int kUnitThreads = 1024;
constexpr int kUnitTok = kMaxUnit / kUnitThreads;
constexpr int kUnitWaves = kUnitThreads / kWave;

template <typename R>
struct OrdKey;
template <>
struct OrdKey<float> {
    using U = uint32_t;
    static constexpr int kBits = 32;
    static __device__ __forceinline__ U of(float x) {
        const uint32_t b = __float_as_uint(x);
        return (b >> 31) ? ~b : (b | 0x80000000u);
    }
    static __device__ __forceinline__ float back(U k) { return __uint_as_float((k >> 31) ? (k & 0x7fffffffu) : ~k); }
};
template <>
struct OrdKey<double> {
    using U = uint64_t;
    static constexpr int kBits = 64;
    static __device__ __forceinline__ U of(double x) {
        const uint64_t b = (uint64_t)__double_as_longlong(x);
        return (b >> 63) ? ~b : (b | 0x8000000000000000ull);
    }
    static __device__ __forceinline__ double back(U k) {
        return __longlong_as_double((long long)((k >> 63) ? (k & 0x7fffffffffffffffull) : ~k));
    }
};

// Sum of v over the 16 waves.  buf: kUnitWaves ints; two calls in a row use different buffers.
__device__ __forceinline__ int unit_sum(int v, int *buf) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o);
    if ((threadIdx.x & 63) == 0) buf[threadIdx.x >> 6] = v;
    __syncthreads();
    int s = 0;
#pragma unroll
    for (int w = 0; w < kUnitWaves; ++w) s += buf[w];
    return s;
}

// Exclusive prefix of v in thread order and the total; buf as for unit_sum.
__device__ __forceinline__ int unit_scan(int v, int *buf, int &total) {
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    int inc = v;
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) {
        const int t = __shfl_up(inc, o);
        inc += lane >= o ? t : 0;
    }
    if (lane == 63) buf[wave] = inc;
    __syncthreads();
    int base = 0;
    total = 0;
#pragma unroll
    for (int w = 0; w < kUnitWaves; ++w) {
        const int c = buf[w];
        base += w < wave ? c : 0;
        total += c;
    }
    return base + inc - v;
}

template <typename R>
__device__ __forceinline__ void unit_minmax(R mn, R mx, R *red, R &lo, R &hi) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) {
        const R a = __shfl_xor(mn, o), b = __shfl_xor(mx, o);
        mn = a < mn ? a : mn;
        mx = b > mx ? b : mx;
    }
    __syncthreads(); // the previous use of red is over
    if ((threadIdx.x & 63) == 0) {
        red[threadIdx.x >> 6] = mn;
        red[kUnitWaves + (threadIdx.x >> 6)] = mx;
    }
    __syncthreads();
    lo = red[0];
    hi = red[kUnitWaves];
#pragma unroll
    for (int w = 1; w < kUnitWaves; ++w) {
        lo = red[w] < lo ? red[w] : lo;
        hi = red[kUnitWaves + w] > hi ? red[kUnitWaves + w] : hi;
    }
}

template <typename R>
__global__ __launch_bounds__(kUnitThreads) void select_large_kernel(SelectArgs<R> a) {
    using K = OrdKey<R>;
    using U = typename K::U;
    __shared__ R red[2 * kUnitWaves];
    __shared__ U kred[kUnitWaves];
    __shared__ int cnt[2][kUnitWaves];
    const int tid = threadIdx.x;
    const int P = a.P, kappa = a.kappa;
    const int j0 = tid * kUnitTok;
    const int n_e = a.pass2 ? *a.flag_count : (int)gridDim.x;
    for (int e_idx = blockIdx.x; e_idx < n_e; e_idx += gridDim.x) {
        const int f = a.pass2 ? a.flag_list[e_idx] : e_idx;
        const int64_t gf = a.frame0 + f;
        const int slot = find_slot(a.map, f);
        const int lf = f - a.map.fstart[slot];
        float *dbg_att = a.have_dbg ? a.dbg_att.p[slot] : nullptr;
        float *dbg_fft = a.have_dbg ? a.dbg_fft.p[slot] : nullptr;
        float *dbg_fused = a.have_dbg ? a.dbg_fused.p[slot] : nullptr;
        const float *att_in = a.have_att_in ? reinterpret_cast<const float *>(a.att_in.p[slot]) + (int64_t)lf * P : nullptr;
        const R *fft = a.fft ? a.fft + (int64_t)f * P : nullptr;

        R av[kUnitTok], fv[kUnitTok];
#pragma unroll
        for (int u = 0; u < kUnitTok; ++u) {
            const int j = j0 + u < P ? j0 + u : P - 1;
            av[u] = att_in ? (R)att_in[j] : (R)0;
            fv[u] = fft ? fft[j] : (R)0;
        }
#pragma unroll
        for (int u = 0; u < kUnitTok; ++u) {
            if (j0 + u < P) {
                if (dbg_att) dbg_att[(int64_t)lf * P + j0 + u] = (float)av[u];
                if (dbg_fft) dbg_fft[(int64_t)lf * P + j0 + u] = (float)fv[u];
            }
        }
        R fused[kUnitTok];
#pragma unroll
        for (int u = 0; u < kUnitTok; ++u) fused[u] = 0;
        if (a.alpha != (R)0) { // clamped tokens repeat token P-1: they change neither bound
            R mn = av[0], mx = av[0], lo, hi;
#pragma unroll
            for (int u = 1; u < kUnitTok; ++u) {
                mn = av[u] < mn ? av[u] : mn;
                mx = av[u] > mx ? av[u] : mx;
            }
            unit_minmax(mn, mx, red, lo, hi);
#pragma unroll
            for (int u = 0; u < kUnitTok; ++u) fused[u] = a.alpha * ((hi > lo) ? (av[u] - lo) / (hi - lo) : (R)0);
        }
        if (a.alpha != (R)1) {
            R mn = fv[0], mx = fv[0], lo, hi;
#pragma unroll
            for (int u = 1; u < kUnitTok; ++u) {
                mn = fv[u] < mn ? fv[u] : mn;
                mx = fv[u] > mx ? fv[u] : mx;
            }
            unit_minmax(mn, mx, red, lo, hi);
#pragma unroll
            for (int u = 0; u < kUnitTok; ++u)
                fused[u] += ((R)1 - a.alpha) * ((hi > lo) ? (fv[u] - lo) / (hi - lo) : (R)0);
        }
        U key[kUnitTok];
#pragma unroll
        for (int u = 0; u < kUnitTok; ++u) {
            const bool valid = j0 + u < P;
            key[u] = valid ? K::of(fused[u]) : (U)0;
            if (valid && dbg_fused) dbg_fused[(int64_t)lf * P + j0 + u] = (float)fused[u];
        }

        // the kappa-th largest key
        U kth = 0;
        for (int b = K::kBits - 1; b >= 0; --b) {
            const U cand = kth | ((U)1 << b);
            int n = 0;
#pragma unroll
            for (int u = 0; u < kUnitTok; ++u) n += key[u] >= cand;
            if (unit_sum(n, cnt[b & 1]) >= kappa) kth = cand;
        }
        // ties at the threshold go to the lowest positions
        int n_gt = 0, n_eq = 0;
#pragma unroll
        for (int u = 0; u < kUnitTok; ++u) {
            n_gt += key[u] > kth;
            n_eq += key[u] == kth;
        }
        const int tot_gt = unit_sum(n_gt, cnt[1]); // the loop's last call used cnt[0]
        const int need = kappa - tot_gt;
        int tot_eq;
        int eq_rank = unit_scan(n_eq, cnt[0], tot_eq);
        unsigned kept_mask = 0;
        int n_kept = 0;
#pragma unroll
        for (int u = 0; u < kUnitTok; ++u) {
            const bool eq = key[u] == kth;
            const bool kept = key[u] > kth || (eq && eq_rank < need);
            eq_rank += eq;
            kept_mask |= (unsigned)kept << u;
            n_kept += kept;
        }
        int tot_kept;
        int pos = unit_scan(n_kept, cnt[1], tot_kept); // tot_kept == kappa

        // selection margin: the kappa-th largest score minus the next one in rank order
        R mg = (R)INFINITY;
        if (kappa < P) {
            U below = 0;
            if (tot_gt + tot_eq > kappa) {
                below = kth; // a token equal to the threshold was dropped
            } else {
#pragma unroll
                for (int u = 0; u < kUnitTok; ++u) below = (key[u] < kth && key[u] > below) ? key[u] : below;
#pragma unroll
                for (int o = 32; o > 0; o >>= 1) {
                    const U t = __shfl_xor(below, o);
                    below = t > below ? t : below;
                }
                if ((tid & 63) == 0) kred[tid >> 6] = below;
                __syncthreads();
                below = kred[0];
#pragma unroll
                for (int w = 1; w < kUnitWaves; ++w) below = kred[w] > below ? kred[w] : below;
            }
            mg = K::back(kth) - K::back(below);
        }
        const bool flag = !a.pass2 && a.margin_thr > (R)0 && mg < a.margin_thr;
#pragma unroll
        for (int u = 0; u < kUnitTok; ++u) {
            if ((kept_mask >> u) & 1u) {
                a.kept_idx[gf * kappa + pos] = j0 + u;
                a.src_tok[(int64_t)f * kappa + pos] = flag ? -1 : lf * P + j0 + u;
                ++pos;
            }
        }
        if (tid == 0) {
            a.margin[gf] = (float)mg;
            a.refined[gf] = (a.pass2 || flag) ? 1 : 0;
            if (flag) a.flag_list[atomicAdd(a.flag_count, 1)] = f;
        }
        __syncthreads(); // kred and cnt are reused by the next unit
    }
}

constexpr int kPoolBatch = 8;
constexpr int kPoolSlices = kUnitWaves;
template <typename T, typename R>
__global__ __launch_bounds__(kUnitThreads) void pool_large_kernel(SelectArgs<R> a) {
    __shared__ int kl[kMaxUnit];
    __shared__ double part[kPoolSlices][64][4];
    const int lane = threadIdx.x & 63, slice = threadIdx.x >> 6;
    const int P = a.P, kappa = a.kappa, S = a.S;
    const int C = a.Hkv * a.D;
    const int cp = blockIdx.y * 64 + lane;
    const bool live = cp < C / 2;
    const int c = live ? 2 * cp : 0;
    const int g = c / a.D, d = c - g * a.D;
    const int len = P / S;
    const int n_e = a.pass2 ? *a.flag_count : (int)gridDim.x;
    for (int e_idx = blockIdx.x; e_idx < n_e; e_idx += gridDim.x) {
        const int f = a.pass2 ? a.flag_list[e_idx] : e_idx;
        const int64_t gf = a.frame0 + f;
        if (!a.pass2 && a.refined[gf]) continue; // on the re-scoring list: its keys come from the fp64 pass
        const int slot = find_slot(a.map, f);
        const int lf = f - a.map.fstart[slot];
        for (int r = threadIdx.x; r < kappa; r += kUnitThreads) kl[r] = a.kept_idx[gf * kappa + r];
        __syncthreads();
        const T *xk = reinterpret_cast<const T *>(a.k.p[slot]) + a.k_off;
        const T *xv = reinterpret_cast<const T *>(a.v.p[slot]) + a.k_off;
        const int64_t col = (int64_t)g * a.sh + d + (int64_t)lf * P * a.st;
        double tot[4] = {0.0, 0.0, 0.0, 0.0}; // k0 k1 v0 v1, used by wave 0
        int b = 0;
        for (int s = 0; s < S; ++s) {
            int e = kappa;
            if (s < S - 1) { // first kept row at or beyond the next super-patch
                const int bound = (s + 1) * len;
                int lo = b, hi = kappa;
                while (lo < hi) {
                    const int mid = (lo + hi) >> 1;
                    if (kl[mid] < bound) lo = mid + 1; else hi = mid;
                }
                e = lo;
            }
            double run[4] = {0.0, 0.0, 0.0, 0.0};
            for (int r0 = b + slice; r0 < e; r0 += kPoolSlices * kPoolBatch) {
                Pair2<T> yk[kPoolBatch], yv[kPoolBatch];
#pragma unroll
                for (int u = 0; u < kPoolBatch; ++u) {
                    const int r = r0 + kPoolSlices * u < e ? r0 + kPoolSlices * u : e - 1; // clamped: loads stay unconditional
                    const int64_t off = col + (int64_t)kl[r] * a.st;
                    yk[u] = *reinterpret_cast<const Pair2<T> *>(xk + off);
                    yv[u] = *reinterpret_cast<const Pair2<T> *>(xv + off);
                }
#pragma unroll
                for (int u = 0; u < kPoolBatch; ++u) {
                    if (r0 + kPoolSlices * u < e) {
                        run[0] += (double)to_float(yk[u].a);
                        run[1] += (double)to_float(yk[u].b);
                        run[2] += (double)to_float(yv[u].a);
                        run[3] += (double)to_float(yv[u].b);
                    }
                }
            }
#pragma unroll
            for (int q = 0; q < 4; ++q) part[slice][lane][q] = run[q];
            __syncthreads();
            if (slice == 0 && live) {
                const int n = e - b;
                double sum[4];
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    sum[q] = part[0][lane][q];
#pragma unroll
                    for (int w = 1; w < kPoolSlices; ++w) sum[q] += part[w][lane][q];
                    tot[q] += sum[q];
                }
                const int64_t o = (gf * S + s) * C + c;
                a.rep_patch_k[o] = n ? (float)(sum[0] / (double)n) : 0.0f;
                a.rep_patch_k[o + 1] = n ? (float)(sum[1] / (double)n) : 0.0f;
                a.rep_patch_v[o] = n ? (float)(sum[2] / (double)n) : 0.0f;
                a.rep_patch_v[o + 1] = n ? (float)(sum[3] / (double)n) : 0.0f;
                if (c == 0) a.cnt_patch[gf * S + s] = n;
            }
            __syncthreads();
            b = e;
        }
        if (slice == 0 && live) {
            const int64_t o = gf * C + c;
            a.fsum_k[o] = tot[0];
            a.fsum_k[o + 1] = tot[1];
            a.fsum_v[o] = tot[2];
            a.fsum_v[o + 1] = tot[3];
            a.rep_frame_k[o] = (float)(tot[0] / (double)kappa);
            a.rep_frame_k[o + 1] = (float)(tot[1] / (double)kappa);
            a.rep_frame_v[o] = (float)(tot[2] / (double)kappa);
            a.rep_frame_v[o + 1] = (float)(tot[3] / (double)kappa);
        }
    }
}

// ------------------------------------------------------------------------------------------
// Storage of the kept KV rows of every layer (Sec. 3.3, last paragraph) and segment keys.
// grid.y < n_slab: slab (layer, K|V, KV head); grid.x = (slot of the batch, part of the slot).
// A slot's destination inside the slab is one dense run of its frames' kappa rows, so unit u of
// the slot goes to dst + u*VEC and comes from row src_tok[u / units_per_row] of the slot's chunk.  Each thread moves ITER units: loads first, then
// stores.  grid.y >= n_slab: one workgroup per segment touched by the chunk adds the chunk's
// exact per-frame sums to the segment's running fp64 sum and refreshes the segment's keys; the
// sums are exact for bf16 / fp32 payloads of ordinary dynamic range, so any chunking gives the
// same bits.
// ------------------------------------------------------------------------------------------
struct CompactArgs {
    PtrTable k, v;               // per slot: chunk base
    FrameMap map;
    int bps;                     // workgroups per slot along grid.x
    int64_t sl_b, sh_b, st_b;    // byte strides layer / head / token
    unsigned char *store_k, *store_v;
    int64_t slab_b;              // bytes of one (layer, head) slab of the store
    int64_t dst_off_b;           // byte offset of frame0's first row inside a slab
    const int32_t *src_tok;
    int units_per_frame;         // kappa * units per row
    int log_upr;                 // log2(units per row)
    int Hkv, n_slab;
    // segment update
    int seg_first, F, kappa, C;
    int64_t n_total;             // frames in the cache after this chunk
    const double *fsum_k, *fsum_v;
    double *ssum_k, *ssum_v;     // running exact sums per segment
    int64_t frame0;
    float *rep_seg_k, *rep_seg_v;
    // copy by runs (copy_run_body): the batch's slots all hold fpc frames (the last one may hold fewer)
    int n_frames, fpc;
    uint32_t magic_kappa, magic_fpc; // floor(2^32 / d) + 1: n / d = umulhi(n, magic) while n * d < 2^32
};

// Adds the batch's exact per-frame sums to a segment's running fp64 sums and refreshes its keys.
// Job j = (segment, group of 64 channels): 64 channel lanes x 4 frame slices per workgroup, each
// slice one batch of independent loads, the four partial sums joined through LDS (the sums are
// exact, so their order does not matter).
constexpr int kSegChan = 64;
constexpr int kSegLdsDoubles = 2 * 4 * kSegChan; // LDS the caller lends: part_k[4][64], part_v[4][64]
__device__ __forceinline__ void segment_update(const CompactArgs &a, int job, double *lds) {
    double(*part_k)[kSegChan] = reinterpret_cast<double(*)[kSegChan]>(lds);
    double(*part_v)[kSegChan] = reinterpret_cast<double(*)[kSegChan]>(lds + 4 * kSegChan);
    const int n_cg = (a.C + kSegChan - 1) / kSegChan;
    const int s = a.seg_first + job / n_cg;
    const int c = (job % n_cg) * kSegChan + (threadIdx.x & (kSegChan - 1));
    // up to four slices of frames side by side: the first 256 threads of the workgroup, or all of a smaller one
    const int slice = threadIdx.x / kSegChan;
    const int n_slices = blockDim.x >= 4 * kSegChan ? 4 : (int)blockDim.x / kSegChan;
    const int64_t f0 = (int64_t)s * a.F;
    const int64_t f1 = (f0 + a.F < a.n_total) ? f0 + a.F : a.n_total;
    const int64_t fa = f0 > a.frame0 ? f0 : a.frame0; // first frame of the segment in this batch
    const bool fresh = f0 >= a.frame0;                // the segment starts in this batch
    const double den = (double)(f1 - f0) * (double)a.kappa;
    const int cc = c < a.C ? c : a.C - 1;
    double sk = 0.0, sv = 0.0;
    for (int64_t fb = fa + slice; slice < n_slices && fb < f1; fb += 8 * n_slices) {
        double tk[8], tv[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) {
            const int64_t fr = fb + n_slices * u < f1 ? fb + n_slices * u : f1 - 1; // clamped: loads stay unconditional
            tk[u] = a.fsum_k[fr * a.C + cc];
            tv[u] = a.fsum_v[fr * a.C + cc];
        }
#pragma unroll
        for (int u = 0; u < 8; ++u) {
            if (fb + n_slices * u < f1) {
                sk += tk[u];
                sv += tv[u];
            }
        }
    }
    if (slice < 4) { // slices that do not exist contribute zeros
        part_k[slice][threadIdx.x & (kSegChan - 1)] = sk;
        part_v[slice][threadIdx.x & (kSegChan - 1)] = sv;
    }
    if (n_slices < 4 && threadIdx.x < kSegChan)
        for (int sl = n_slices; sl < 4; ++sl) part_k[sl][threadIdx.x] = part_v[sl][threadIdx.x] = 0.0;
    __syncthreads();
    if (slice == 0 && c < a.C) {
        sk = (fresh ? 0.0 : a.ssum_k[(int64_t)s * a.C + c]) + ((part_k[0][threadIdx.x] + part_k[1][threadIdx.x]) + (part_k[2][threadIdx.x] + part_k[3][threadIdx.x]));
        sv = (fresh ? 0.0 : a.ssum_v[(int64_t)s * a.C + c]) + ((part_v[0][threadIdx.x] + part_v[1][threadIdx.x]) + (part_v[2][threadIdx.x] + part_v[3][threadIdx.x]));
        a.ssum_k[(int64_t)s * a.C + c] = sk;
        a.ssum_v[(int64_t)s * a.C + c] = sv;
        a.rep_seg_k[(int64_t)s * a.C + c] = (float)(sk / den);
        a.rep_seg_v[(int64_t)s * a.C + c] = (float)(sv / den);
    }
}

// Work of workgroup (gx_i, y) of compact_kernel's grid.
template <typename V, int ITER>
__device__ __forceinline__ void compact_body(const CompactArgs &a, int gx_i, int y, double *seg_lds, int NT = 256) {
    if (y >= a.n_slab) {
        if (gx_i == 0) segment_update(a, y - a.n_slab, seg_lds);
        return;
    }
    const int l = y / (2 * a.Hkv), rem = y - l * 2 * a.Hkv;
    const int kv = rem / a.Hkv, g = rem - kv * a.Hkv;
    const int slot = gx_i / a.bps, bx = gx_i - slot * a.bps;
    const int f_lo = a.map.fstart[slot];
    const int n_units = (a.map.fstart[slot + 1] - f_lo) * a.units_per_frame;
    if (bx * (NT * ITER) >= n_units) return;
    const unsigned char *src = reinterpret_cast<const unsigned char *>(kv ? a.v.p[slot] : a.k.p[slot]) +
                               (int64_t)l * a.sl_b + (int64_t)g * a.sh_b;
    unsigned char *dst = (kv ? a.store_v : a.store_k) + ((int64_t)l * a.Hkv + g) * a.slab_b + a.dst_off_b +
                         (int64_t)f_lo * a.units_per_frame * sizeof(V);
    const int32_t *src_tok = a.src_tok + (int64_t)f_lo * (a.units_per_frame >> a.log_upr);
    const int mask = (1 << a.log_upr) - 1;
    // Loads are issued unconditionally on clamped unit numbers (first all row lookups, then all
    // row reads) so that they overlap; only the stores are predicated.
    V tmp[ITER];
    int row_tok[ITER];
    const int u0 = bx * (NT * ITER) + threadIdx.x;
#pragma unroll
    for (int it = 0; it < ITER; ++it) {
        int u = u0 + it * NT;
        u = u < n_units ? u : n_units - 1;
        row_tok[it] = src_tok[u >> a.log_upr];
    }
#pragma unroll
    for (int it = 0; it < ITER; ++it) {
        int u = u0 + it * NT;
        u = u < n_units ? u : n_units - 1;
        const int tok = row_tok[it] < 0 ? 0 : row_tok[it]; // -1: a frame left to the fp64 pass
        tmp[it] = *reinterpret_cast<const V *>(src + (int64_t)tok * a.st_b + (int64_t)(u & mask) * sizeof(V));
    }
#pragma unroll
    for (int it = 0; it < ITER; ++it) {
        const int u = u0 + it * NT;
        if (u < n_units && row_tok[it] >= 0) *reinterpret_cast<V *>(dst + (int64_t)u * sizeof(V)) = tmp[it];
    }
}

// The same copy cut into runs of blockDim.x * ITER consecutive 16-byte units of a slab's destination,
// whatever slots they come from: workgroup (run, y) moves units run * blockDim.x * ITER ... of slab y.
// For batches whose slots hold the same number of frames (a stream fed in equal chunks), so that a unit's
// slot is a division; a lane looks up its row and its chunk's base pointer (the tables are kernel
// arguments: a load from the argument block) side by side, then all its rows are in flight together.
// (A workgroup that walks several such runs as a software pipeline -- look-ups two rounds ahead of the
// stores, two rounds of rows in flight -- was measured beside the attention workgroups and was slower
// for every pipeline length: 497-577 us against 466-483 us for the launch with a full copy.)
template <int ITER>
__device__ __forceinline__ void copy_run_body(const CompactArgs &a, int run, int y) {
    typedef u32x4 V;
    const int NT = blockDim.x;
    const int l = y / (2 * a.Hkv), rem = y - l * 2 * a.Hkv;
    const int kv = rem / a.Hkv, g = rem - kv * a.Hkv;
    const int n_units = a.n_frames * a.units_per_frame;
    const int u0 = run * (NT * ITER) + threadIdx.x;
    if (run * (NT * ITER) >= n_units) return;
    const int64_t slab_src = (int64_t)l * a.sl_b + (int64_t)g * a.sh_b;
    unsigned char *dst = (kv ? a.store_v : a.store_k) + ((int64_t)l * a.Hkv + g) * a.slab_b + a.dst_off_b;
    const void *const *tab = kv ? a.v.p : a.k.p;
    const int mask = (1 << a.log_upr) - 1;
    int row_tok[ITER];
    const unsigned char *base[ITER];
    V tmp[ITER];
#pragma unroll
    for (int it = 0; it < ITER; ++it) {
        int u = u0 + it * NT;
        u = u < n_units ? u : n_units - 1;
        const unsigned row = (unsigned)u >> a.log_upr;       // kept row of the batch: frame * kappa + rank
        row_tok[it] = a.src_tok[row];
        const unsigned f = __umulhi(row, a.magic_kappa);     // batch frame
        const unsigned slot = __umulhi(f, a.magic_fpc);
        base[it] = static_cast<const unsigned char *>(tab[slot]);
    }
#pragma unroll
    for (int it = 0; it < ITER; ++it) {
        int u = u0 + it * NT;
        u = u < n_units ? u : n_units - 1;
        const int tok = row_tok[it] < 0 ? 0 : row_tok[it];
        tmp[it] = *reinterpret_cast<const V *>(base[it] + slab_src + (int64_t)tok * a.st_b + (int64_t)(u & mask) * sizeof(V));
    }
#pragma unroll
    for (int it = 0; it < ITER; ++it) {
        const int u = u0 + it * NT;
        if (u < n_units && row_tok[it] >= 0) *reinterpret_cast<V *>(dst + (int64_t)u * sizeof(V)) = tmp[it];
    }
}

template <typename V, int ITER>
__global__ __launch_bounds__(256) void compact_kernel(CompactArgs a) {
    __shared__ double seg_lds[kSegLdsDoubles];
    compact_body<V, ITER>(a, blockIdx.x, blockIdx.y, seg_lds);
}

// overlap_copy: the copy of the previous batch's kept rows (HBM bound) and the frequency signal of
// the new batch (arithmetic bound) in one launch, so that both kinds of work are resident on every
// compute unit together.  1-D grid of n_copy + n_freq workgroups; every `period`-th one is a
// frequency workgroup, the others walk compact_kernel's (copy_gx, y) grid in its own order.
constexpr int kFusedCopyIter = 4; // 16-byte loads in flight per lane of a copy workgroup
struct FreqPart {
    PtrTable k;
    FrameMap map;
    int64_t k_off, sh, st;
    int Hkv, P;
    float *out;
    int n_frames; // grid.x of the stand-alone frequency kernel
    int bpf;      // grid.y of the stand-alone frequency kernel
    int n_wg;     // n_frames * bpf
};

// kUnit: the unit is several frames (P > kMaxP), whose frequency workgroups per unit are a run-time
// number; a frame's are the constant 7.  (The two cases also show up under their own names in a
// kernel trace.)
template <typename T, int D, bool kUnit>
__global__ __launch_bounds__(256) void copy_freq_kernel(CompactArgs ca, int copy_gx, FreqPart fp, int period) {
    __shared__ double seg_lds[kSegLdsDoubles];
    const int b = blockIdx.x;
    const int q = b / period, r = b - q * period;
    if (r == 0 && q < fp.n_wg) {
        freq_body<T, float, D>(fp.k, fp.map, fp.k_off, fp.sh, fp.st, fp.Hkv, fp.P, nullptr, nullptr, fp.out,
                               q % fp.n_frames, q / fp.n_frames, fp.n_frames, kUnit ? fp.bpf : 7);
    } else {
        const int before = q + (r > 0) < fp.n_wg ? q + (r > 0) : fp.n_wg; // frequency workgroups with a lower number
        const int cid = b - before;
        const int n_rows = copy_gx * ca.n_slab; // then one workgroup per segment job
        if (cid < n_rows)
            compact_body<u32x4, kFusedCopyIter>(ca, cid % copy_gx, cid / copy_gx, seg_lds);
        else
            segment_update(ca, cid - n_rows, seg_lds);
    }
}

// overlap_copy with the matrix-core attention kernel: ONE launch per batch carries the copy of an earlier
// batch's kept rows (HBM bound), the frequency signal of the new batch (arithmetic bound, little
// traffic) and the attention signal of the new batch (arithmetic and issue bound while it streams all
// the queries), so that on every compute unit waves waiting for memory and waves busy with arithmetic
// are resident together and the launch as a whole runs at the pace of its HBM traffic.
// The attention workgroup fixes the launch shape: its block size (64 * waves) and its LDS (80 KB for
// 196 tokens), so two workgroups of any kind share a compute unit; the copy workgroups make up for
// their small number with ITER 16-byte loads in flight per lane.  No workgroup here owns static LDS: the
// segment jobs borrow the dynamic block.
// 1-D grid.  Attention workgroups -- by far the longest -- sit at multiples of att_period inside the
// first part of the grid so that the last of them starts well before the end; among the others every
// freq_period-th is a frequency workgroup.  Both periods are odd: workgroup b lands on XCD b % 8, and an
// even period would put a whole kind of work on half of the chip.
struct ChainMap {
    int n_att, att_period;   // attention workgroups at b = i * att_period, i < n_att
    int n_freq, freq_period; // among the rest (in order): frequency workgroups at r = i * freq_period, i < n_freq
    int copy_gx, n_copy_rows; // then compact_kernel's (copy_gx, n_slab) grid, then the segment jobs
};

template <int ITER, bool RUNS>
__global__ __launch_bounds__(448) __attribute__((amdgpu_waves_per_eu(4, 4))) void chain_kernel(CompactArgs ca, FreqPart fp, PtrTable qtab,
                                                                                              AttMfmaArgs aa, ChainMap cm) {
    extern __shared__ __align__(16) unsigned char smem_raw[];
    const int b = blockIdx.x;
    const int ia = b / cm.att_period;
    if (ia < cm.n_att && b == ia * cm.att_period) {
        att_mfma_body(qtab, fp.k, fp.map, aa, ia / aa.n_part, ia % aa.n_part, smem_raw);
        return;
    }
    // attention workgroups with a lower number: those at 0, att_period, ... below b
    const int a_before = ia + 1 < cm.n_att ? ia + 1 : cm.n_att;
    const int r = b - a_before;
    const int jf = r / cm.freq_period;
    if (jf < cm.n_freq && r == jf * cm.freq_period) {
        freq_body<uint16_t, float, 128>(fp.k, fp.map, fp.k_off, fp.sh, fp.st, fp.Hkv, fp.P, nullptr, nullptr, fp.out,
                                        jf % fp.n_frames, jf / fp.n_frames, fp.n_frames, fp.bpf);
        return;
    }
    const int f_before = jf + 1 < cm.n_freq ? jf + 1 : cm.n_freq;
    const int cid = r - f_before;
    double *seg_lds = reinterpret_cast<double *>(smem_raw);
    if (cid < cm.n_copy_rows) {
        if constexpr (RUNS)
            copy_run_body<ITER>(ca, cid % cm.copy_gx, cid / cm.copy_gx);
        else
            compact_body<u32x4, ITER>(ca, cid % cm.copy_gx, cid / cm.copy_gx, seg_lds, blockDim.x);
    } else {
        segment_update(ca, cid - cm.n_copy_rows, seg_lds);
    }
}

// Copy of the kept rows of the re-scored frames (rows chosen by the fp64 pass), list driven like
// the other re-scoring kernels; the extra workgroups in grid.y update the batch's segments, which
// need the final per-frame sums of every frame.
template <typename V>
__global__ __launch_bounds__(256) void compact_listed_kernel(CompactArgs a, const int32_t *__restrict__ flag_list,
                                                             const int32_t *__restrict__ flag_count) {
    const int y = blockIdx.y;
    if (y >= a.n_slab) {
        __shared__ double seg_lds[kSegLdsDoubles];
        if (blockIdx.x == 0 && blockIdx.z == 0) segment_update(a, y - a.n_slab, seg_lds);
        return;
    }
    const int l = y / (2 * a.Hkv), rem = y - l * 2 * a.Hkv;
    const int kv = rem / a.Hkv, g = rem - kv * a.Hkv;
    const int mask = (1 << a.log_upr) - 1;
    const int n_e = *flag_count;
    for (int e = blockIdx.x; e < n_e; e += gridDim.x) {
        const int f = flag_list[e];
        const int slot = find_slot(a.map, f);
        const unsigned char *src = reinterpret_cast<const unsigned char *>(kv ? a.v.p[slot] : a.k.p[slot]) +
                                   (int64_t)l * a.sl_b + (int64_t)g * a.sh_b;
        unsigned char *dst = (kv ? a.store_v : a.store_k) + ((int64_t)l * a.Hkv + g) * a.slab_b + a.dst_off_b +
                             (int64_t)f * a.units_per_frame * sizeof(V);
        const int32_t *src_tok = a.src_tok + (int64_t)f * (a.units_per_frame >> a.log_upr);
        for (int u0 = blockIdx.z * (2 * 256) + threadIdx.x; u0 < a.units_per_frame; u0 += gridDim.z * (2 * 256)) {
            V tmp[2];
            int row_tok[2];
#pragma unroll
            for (int it = 0; it < 2; ++it) {
                const int u = u0 + it * 256 < a.units_per_frame ? u0 + it * 256 : a.units_per_frame - 1;
                row_tok[it] = src_tok[u >> a.log_upr];
            }
#pragma unroll
            for (int it = 0; it < 2; ++it) {
                const int u = u0 + it * 256 < a.units_per_frame ? u0 + it * 256 : a.units_per_frame - 1;
                tmp[it] = *reinterpret_cast<const V *>(src + (int64_t)row_tok[it] * a.st_b + (int64_t)(u & mask) * sizeof(V));
            }
#pragma unroll
            for (int it = 0; it < 2; ++it) {
                const int u = u0 + it * 256;
                if (u < a.units_per_frame) *reinterpret_cast<V *>(dst + (int64_t)u * sizeof(V)) = tmp[it];
            }
        }
    }
}

__global__ void clear_count_kernel(int32_t *count) { *count = 0; }

// Puts every unit of the batch on the re-scoring list (units of several frames go straight to the fp64 pass).
__global__ void list_all_kernel(int32_t *list, int32_t *count, int n) {
    for (int i = threadIdx.x; i < n; i += blockDim.x) list[i] = i;
    if (threadIdx.x == 0) *count = n;
}

// A unit of several frames ranks thousands of min-max-normalised scores: the gap at the keep boundary is
// below the re-scoring threshold for practically every unit, so an fp32 keep would be overruled every
// time.  With re-scoring on, such units skip the fp32 pass: every unit is listed and the fp64 pass decides.
static bool direct_fp64(const Ctx &c) { return c.cfg.tokens_per_frame > kMaxP && c.margin_thr > 0.0; }

// ------------------------------------------------------------------------------------------
// host side
// ------------------------------------------------------------------------------------------
static const float *token_table(const Ctx &c, float) { return c.tw32; }
static const double *token_table(const Ctx &c, double) { return c.tw64; }

template <typename T, typename R>
static hipError_t launch_freq_token(const Ctx &c, const ChunkArgs &a, bool listed, R *out, hipStream_t st) {
    const int P = c.cfg.tokens_per_frame, C = c.cfg.n_kv_heads * c.cfg.head_dim;
    const int n_groups = (C + 63) / 64;
    const size_t lds = (size_t)(P + 1) * 64 * sizeof(R);
    static bool lds_ok[kMaxDevices];
    const hipError_t ea = allow_dynamic_lds(reinterpret_cast<const void *>(&freq_token_kernel<T, R>),
                                            (size_t)(kMaxP + 1) * 64 * sizeof(R), c.cfg.device_id, lds_ok);
    if (ea != hipSuccess) return ea;
    const int32_t *fl = listed ? c.flag_list[a.parity] : nullptr, *fc = listed ? c.flag_count + a.parity : nullptr;
    // the two passes (fp32 on the caller's stream, fp64 on the side stream) may run at the same
    // time: each has its own half of the partial-sum scratch
    R *part = reinterpret_cast<R *>(c.tok_part + (sizeof(R) == 8 ? c.tok_part_half : 0));
    hipLaunchKernelGGL((freq_token_kernel<T, R>), dim3(listed ? kRescoreSlots : a.n_frames, n_groups), dim3(256), lds, st,
                       a.k, a.map, (int64_t)c.ls * a.kv_sl, a.kv_sh, a.kv_st, c.cfg.n_kv_heads, c.cfg.head_dim, P,
                       token_table(c, R()), fl, fc, part, a.n_frames);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL((freq_token_finish_kernel<R>), dim3(listed ? kRescoreSlots : a.n_frames), dim3(256), 0, st, part,
                       n_groups, P, C, fl, fc, out, a.n_frames);
    return hipGetLastError();
}

template <typename T, typename R>
static hipError_t launch_freq(const Ctx &c, const ChunkArgs &a, bool listed, R *out, hipStream_t st) {
    if (c.cfg.freq_axis == MUKV_FREQ_TOKEN) return launch_freq_token<T, R>(c, a, listed, out, st);
    const int P = c.cfg.tokens_per_frame, D = c.cfg.head_dim, Hkv = c.cfg.n_kv_heads;
    const int64_t k_off = (int64_t)c.ls * a.kv_sl;
    const dim3 grid(listed ? rescore_slots(P, a.n_frames) : a.n_frames, freq_blocks_per_frame(P));
    const int32_t *fl = listed ? c.flag_list[a.parity] : nullptr, *fc = listed ? c.flag_count + a.parity : nullptr;
#define MUKV_FREQ(DD)                                                                                         \
    hipLaunchKernelGGL((freq_signal_kernel<T, R, DD>), grid, dim3(256), 0, st, a.k, a.map, k_off, a.kv_sh, \
                       a.kv_st, Hkv, P, fl, fc, out)
    switch (D) {
    case 128: MUKV_FREQ(128); break;
    case 64: MUKV_FREQ(64); break;
    case 32: MUKV_FREQ(32); break;
    case 16: MUKV_FREQ(16); break;
    default: return hipErrorInvalidValue;
    }
#undef MUKV_FREQ
    return hipGetLastError();
}

size_t att_generic_lds_bytes(int P, int D, size_t r_size, size_t key_size) {
    return att_generic_key_bytes(P, D, key_size) + (size_t)kGenQ * D * 4 + (size_t)4 * P * r_size;
}

template <typename T, typename R>
static hipError_t launch_att_generic(const Ctx &c, const ChunkArgs &a, bool listed, R *out, int *n_part,
                                     hipStream_t st) {
    const int P = c.cfg.tokens_per_frame, D = c.cfg.head_dim;
    const int q_per_block = 2 * kGenQ; // two rounds per workgroup
    const int qsplit = (P + q_per_block - 1) / q_per_block;
    *n_part = c.cfg.n_q_heads * qsplit;
    const size_t lds = att_generic_lds_bytes(P, D, sizeof(R), sizeof(typename KeyStage<T, R>::type));
    static bool lds_ok[kMaxDevices]; // per instantiation
    const hipError_t ea = allow_dynamic_lds(reinterpret_cast<const void *>(&att_generic_kernel<T, R>), 160 * 1024,
                                            c.cfg.device_id, lds_ok);
    if (ea != hipSuccess) return ea;
    hipLaunchKernelGGL((att_generic_kernel<T, R>), dim3(listed ? kRescoreSlotsAtt : a.n_frames, c.cfg.n_q_heads, qsplit),
                       dim3(256), lds, st, a.q, a.k, a.map, (int64_t)c.ls * a.kv_sl, a.q_sh, a.q_st, a.kv_sh, a.kv_st, P,
                       D, c.group, c.cfg.n_q_heads, c.cfg.causal, q_per_block, listed ? c.flag_list[a.parity] : nullptr,
                       listed ? c.flag_count + a.parity : nullptr, out);
    return hipGetLastError();
}

hipError_t launch_att_mfma(const Ctx &c, const ChunkArgs &a, float *out, int *n_part, hipStream_t st);

template <typename T, typename R>
static hipError_t launch_select(const Ctx &c, const ChunkArgs &a, const R *att, int n_part, const R *fft, int pass2,
                                hipStream_t st, int fft_parts = 0) {
    SelectArgs<R> s;
    const bool need_att = c.cfg.alpha != 0.0;
    s.att = (need_att && !a.have_att_in) ? att : nullptr;
    s.n_part = n_part;
    s.att_scale = (R)(1.0 / ((double)c.cfg.n_q_heads * (double)c.cfg.tokens_per_frame));
    s.att_in = a.att_in;
    s.have_att_in = need_att && a.have_att_in;
    s.fft = (c.cfg.alpha != 1.0) ? fft : nullptr;
    s.fft_parts = fft_parts;
    s.fft_scale = (R)(1.0 / ((double)c.cfg.n_kv_heads * (double)c.cfg.head_dim));
    s.alpha = (R)c.cfg.alpha;
    s.P = c.cfg.tokens_per_frame;
    s.kappa = c.kappa;
    s.S = c.cfg.superpatches_per_frame;
    s.Hkv = c.cfg.n_kv_heads;
    s.D = c.cfg.head_dim;
    s.frame0 = a.frame0;
    s.k = a.k;
    s.v = a.v;
    s.map = a.map;
    s.k_off = (int64_t)c.ls * a.kv_sl;
    s.sh = a.kv_sh;
    s.st = a.kv_st;
    s.margin_thr = (R)c.margin_thr;
    s.pass2 = pass2;
    s.flag_list = c.flag_list[a.parity];
    s.flag_count = c.flag_count + a.parity;
    s.kept_idx = c.kept_idx;
    // with overlap_copy the rows chosen by the fp64 pass replace the marks of the first pass: the
    // copy, which comes later, then takes every frame in one go
    // (a batch's main copy comes after its fp64 pass only with overlap_copy on units of several frames)
    s.src_tok = (pass2 && (!c.cfg.overlap_copy || c.split_side)) ? c.src_tok2 : c.src_tok[a.parity];
    s.rep_frame_k = c.rep_frame_k;
    s.rep_frame_v = c.rep_frame_v;
    s.rep_patch_k = c.rep_patch_k;
    s.rep_patch_v = c.rep_patch_v;
    s.cnt_patch = c.cnt_patch;
    s.fsum_k = c.fsum_k;
    s.fsum_v = c.fsum_v;
    s.margin = c.margin;
    s.refined = c.refined;
    s.dbg_att = a.dbg_att;
    s.dbg_fft = a.dbg_fft;
    s.dbg_fused = a.dbg_fused;
    s.have_dbg = a.have_dbg;
    const int gx = pass2 ? rescore_slots(s.P, a.n_frames) : a.n_frames;
    if (s.P > kMaxP) { // a unit of several frames: the keep and the block keys in two launches
        const int n_cg = (s.Hkv * s.D / 2 + 63) / 64;
        hipLaunchKernelGGL((select_large_kernel<R>), dim3(gx), dim3(kUnitThreads), 0, st, s);
        hipLaunchKernelGGL((pool_large_kernel<T, R>), dim3(gx, n_cg), dim3(kUnitThreads), 0, st, s);
        return hipGetLastError();
    }
    hipLaunchKernelGGL((select_pool_kernel<T, R>), dim3(gx), dim3(256), 0, st, s);
    return hipGetLastError();
}

static int ilog2(int x) {
    int l = 0;
    while ((1 << l) < x) ++l;
    return l;
}

// mode 0: every frame + segment update (no re-scoring, or a copy that comes after it); 1: main copy, frames on the re-scoring
// list skipped, no segment update; 2: listed frames only (rows from the fp64 pass) + segment update
constexpr int kCompactIter = 4;
static void compact_args(const Ctx &c, const ChunkArgs &a, int mode, int iter, CompactArgs &k, int &gx, int &gy,
                         int threads = 256) {
    const int esz = c.esz, D = c.cfg.head_dim;
    const int row_b = D * esz;
    k.k = a.k;
    k.v = a.v;
    k.map = a.map;
    k.sl_b = a.kv_sl * esz;
    k.sh_b = a.kv_sh * esz;
    k.st_b = a.kv_st * esz;
    k.store_k = reinterpret_cast<unsigned char *>(c.store_k);
    k.store_v = reinterpret_cast<unsigned char *>(c.store_v);
    k.slab_b = c.store_cap * row_b;
    k.dst_off_b = a.frame0 * c.kappa * (int64_t)row_b;
    k.src_tok = mode == 2 ? c.src_tok2 : c.src_tok[a.parity];
    const int upr = row_b / 16; // rows are whole 16-byte units (validated at create)
    k.log_upr = ilog2(upr);
    k.units_per_frame = c.kappa * upr;
    k.Hkv = c.cfg.n_kv_heads;
    k.n_slab = c.cfg.n_layers * 2 * c.cfg.n_kv_heads;
    k.F = c.cfg.frames_per_segment;
    k.kappa = c.kappa;
    k.C = c.c_kv;
    k.n_total = a.frame0 + a.n_frames;
    k.seg_first = (int)(a.frame0 / k.F);
    const int seg_last = (int)((k.n_total - 1) / k.F);
    k.fsum_k = c.fsum_k;
    k.fsum_v = c.fsum_v;
    k.ssum_k = c.ssum_k;
    k.ssum_v = c.ssum_v;
    k.frame0 = a.frame0;
    k.rep_seg_k = c.rep_seg_k;
    k.rep_seg_v = c.rep_seg_v;
    const int n_seg_jobs = (seg_last - k.seg_first + 1) * ((k.C + kSegChan - 1) / kSegChan);
    if (mode == 2) {
        k.bps = 0;
        gx = rescore_slots(c.cfg.tokens_per_frame, a.n_frames);
        gy = k.n_slab + n_seg_jobs;
        return;
    }
    int max_slot_frames = 0;
    for (int s = 0; s < a.map.n_slots; ++s) {
        const int n = a.map.fstart[s + 1] - a.map.fstart[s];
        max_slot_frames = n > max_slot_frames ? n : max_slot_frames;
    }
    k.bps = (max_slot_frames * k.units_per_frame + threads * iter - 1) / (threads * iter);
    gx = k.bps * a.map.n_slots;
    gy = k.n_slab + (mode == 0 ? n_seg_jobs : 0);
}

static hipError_t launch_compact(const Ctx &c, const ChunkArgs &a, int mode, hipStream_t st) {
    CompactArgs k;
    int gx, gy;
    compact_args(c, a, mode, kCompactIter, k, gx, gy);
    if (mode == 2) { // grid.z: a listed frame's rows are shared so that a workgroup makes at most 8 rounds
        const int gz = (k.units_per_frame + 8 * 512 - 1) / (8 * 512);
        hipLaunchKernelGGL((compact_listed_kernel<u32x4>), dim3(gx, gy, gz < 64 ? gz : 64), dim3(256), 0, st, k,
                           c.flag_list[a.parity], c.flag_count + a.parity);
    }
    else
        hipLaunchKernelGGL((compact_kernel<u32x4, kCompactIter>), dim3(gx, gy), dim3(256), 0, st, k);
    return hipGetLastError();
}

// One launch for the copy of batch `prev` (mode as for launch_compact) and Eq. 2-3 of batch `a`.
template <typename T>
static hipError_t launch_copy_freq(const Ctx &c, const ChunkArgs &prev, int mode, const ChunkArgs &a, hipStream_t st) {
    CompactArgs k;
    int gx, gy;
    compact_args(c, prev, mode, kFusedCopyIter, k, gx, gy);
    FreqPart fp;
    fp.k = a.k;
    fp.map = a.map;
    fp.k_off = (int64_t)c.ls * a.kv_sl;
    fp.sh = a.kv_sh;
    fp.st = a.kv_st;
    fp.Hkv = c.cfg.n_kv_heads;
    fp.P = c.cfg.tokens_per_frame;
    fp.out = c.fft_sig[a.parity];
    fp.n_frames = a.n_frames;
    fp.bpf = freq_blocks_per_frame(fp.P);
    fp.n_wg = a.n_frames * fp.bpf;
    const int64_t n_copy = (int64_t)gx * k.n_slab + (gy - k.n_slab); // row copies, then the segment jobs
    const int64_t total = n_copy + fp.n_wg;
    if (total > 0x7fffffff) return hipErrorInvalidValue;
    const int period = (int)(total / fp.n_wg); // >= 1; frequency workgroups at 0, period, 2*period, ...
#define MUKV_COPY_FREQ(DD)                                                                                         \
    do {                                                                                                           \
        if (fp.P > kMaxP)                                                                                          \
            hipLaunchKernelGGL((copy_freq_kernel<T, DD, true>), dim3((unsigned)total), dim3(256), 0, st, k, gx, fp, \
                               period);                                                                            \
        else                                                                                                       \
            hipLaunchKernelGGL((copy_freq_kernel<T, DD, false>), dim3((unsigned)total), dim3(256), 0, st, k, gx,   \
                               fp, period);                                                                        \
    } while (0)
    switch (c.cfg.head_dim) {
    case 128: MUKV_COPY_FREQ(128); break;
    case 64: MUKV_COPY_FREQ(64); break;
    case 32: MUKV_COPY_FREQ(32); break;
    case 16: MUKV_COPY_FREQ(16); break;
    default: return hipErrorInvalidValue;
    }
#undef MUKV_COPY_FREQ
    return hipGetLastError();
}

// One launch for the copy of batch `prev` (null: none is due yet), Eq. 2-3 and Eq. 1 of batch `a`.
static bool chain_supported(const Ctx &c, const ChunkArgs &a) {
    // the matrix-core attention in its many-frames layout (a KV group per workgroup), the feature-axis
    // indicator, frames as units
    return c.use_mfma && c.cfg.freq_axis == MUKV_FREQ_FEATURE && c.cfg.tokens_per_frame <= kMaxP &&
           att_mfma_many(c, a.n_frames);
}

static int odd_at_most(int64_t x) { // largest odd number <= x, at least 1
    if (x < 1) return 1;
    if (x > 0x3fffffff) x = 0x3fffffff;
    return (int)((x & 1) ? x : x - 1);
}

static hipError_t launch_chain(const Ctx &c, const ChunkArgs *prev, int copy_mode, const ChunkArgs &a, bool need_fft,
                               int *n_part, int *fft_parts, hipStream_t st) {
    AttMfmaArgs aa;
    int waves;
    size_t lds;
    att_mfma_plan(c, a, c.att_part[a.parity], &aa, &waves, &lds);
    *n_part = aa.n_part;
    // Eq. 2-3 by the attention workgroups themselves, from the keys they have staged anyway: no second read
    // of the keys, no frequency workgroups
    const bool fused_fft = need_fft && c.dft_tab != nullptr;
    if (fused_fft) {
        aa.dft = c.dft_tab;
        aa.fft_out = c.fft_sig[a.parity];
    }
    *fft_parts = fused_fft ? c.cfg.n_kv_heads : 0;
    const int threads = waves * 64;
    CompactArgs k;
    std::memset(&k, 0, sizeof(k));
    int gx = 0, gy = 0, iter = 4;
    bool runs = false;
    if (prev) {
        // equal slots (all but the last): the copy is cut into runs of the destination, 16 units per lane
        const int fpc = prev->map.fstart[1] - prev->map.fstart[0];
        runs = fpc > 1 && c.kappa > 1; // (the reciprocal of 1 does not fit the 32-bit multiplier)
        for (int s = 0; s < prev->map.n_slots && runs; ++s) {
            const int n = prev->map.fstart[s + 1] - prev->map.fstart[s];
            runs = s + 1 < prev->map.n_slots ? n == fpc : (n >= 1 && n <= fpc);
        }
        runs = runs && (int64_t)prev->n_frames * c.kappa * c.kappa < (1ll << 32) && (int64_t)prev->n_frames * fpc < (1ll << 32);
    }
    if (prev && runs) {
        iter = 16;
        compact_args(c, *prev, copy_mode, iter, k, gx, gy, threads);
        k.n_frames = prev->n_frames;
        k.fpc = prev->map.fstart[1] - prev->map.fstart[0];
        k.magic_kappa = (uint32_t)((1ull << 32) / (uint32_t)c.kappa) + 1u;
        k.magic_fpc = (uint32_t)((1ull << 32) / (uint32_t)k.fpc) + 1u;
        const int64_t per_wg = (int64_t)threads * iter;
        gx = (int)(((int64_t)k.n_frames * k.units_per_frame + per_wg - 1) / per_wg);
    } else if (prev) {
        // 16-byte units a lane moves: as many as the longest slot gives every lane of one workgroup,
        // within what the attention kernel's register budget leaves (16)
        int max_slot_frames = 0;
        for (int s = 0; s < prev->map.n_slots; ++s) {
            const int n = prev->map.fstart[s + 1] - prev->map.fstart[s];
            max_slot_frames = n > max_slot_frames ? n : max_slot_frames;
        }
        const int64_t units = (int64_t)max_slot_frames * c.kappa * (c.cfg.head_dim * c.esz / 16);
        const int cand[3] = {16, 7, 4};
        int64_t best = -1;
        for (int ci = 0; ci < 3; ++ci) {
            const int64_t per_wg = (int64_t)threads * cand[ci];
            const int64_t lanes = (units + per_wg - 1) / per_wg * per_wg; // unit slots launched per (slot, slab)
            if (best < 0 || lanes * 20 < best * 19) { // a smaller count only when it saves more than 5 % of the lanes
                best = lanes;
                iter = cand[ci];
            }
        }
        compact_args(c, *prev, copy_mode, iter, k, gx, gy, threads);
    }
    FreqPart fp;
    fp.k = a.k;
    fp.map = a.map;
    fp.k_off = (int64_t)c.ls * a.kv_sl;
    fp.sh = a.kv_sh;
    fp.st = a.kv_st;
    fp.Hkv = c.cfg.n_kv_heads;
    fp.P = c.cfg.tokens_per_frame;
    fp.out = c.fft_sig[a.parity];
    fp.n_frames = a.n_frames;
    fp.bpf = 4; // with 7 waves per workgroup: 28 tokens of a frame side by side, as in the kernel of its own
    fp.n_wg = (need_fft && !fused_fft) ? a.n_frames * fp.bpf : 0;
    ChainMap cm;
    cm.n_att = a.n_frames * aa.n_part;
    cm.n_freq = fp.n_wg;
    cm.copy_gx = gx > 0 ? gx : 1;
    cm.n_copy_rows = gx * k.n_slab;
    const int64_t n_copy = (int64_t)cm.n_copy_rows + (prev ? gy - k.n_slab : 0);
    const int64_t total = (int64_t)cm.n_att + cm.n_freq + n_copy;
    if (total > 0x7fffffff) return hipErrorInvalidValue;
    // attention workgroups over the first 7/8 of the grid: the last one to start still has an eighth of
    // the launch to finish in
    cm.att_period = odd_at_most(total * 7 / 8 / cm.n_att);
    cm.freq_period = cm.n_freq ? odd_at_most((total - cm.n_att) / cm.n_freq) : 1;
#define MUKV_CHAIN(IT, RUNS)                                                                                          \
    do {                                                                                                              \
        static bool lds_ok[kMaxDevices];                                                                              \
        const hipError_t ea = allow_dynamic_lds(reinterpret_cast<const void *>(&chain_kernel<IT, RUNS>),              \
                                                kAttMfmaMaxLds, c.cfg.device_id, lds_ok);                             \
        if (ea != hipSuccess) return ea;                                                                              \
        hipLaunchKernelGGL((chain_kernel<IT, RUNS>), dim3((unsigned)total), dim3(threads), lds, st, k, fp, a.q, aa,   \
                           cm);                                                                                       \
    } while (0)
    if (runs) {
        MUKV_CHAIN(16, true);
    } else {
        switch (iter) {
        case 16: MUKV_CHAIN(16, false); break;
        case 7: MUKV_CHAIN(7, false); break;
        default: MUKV_CHAIN(4, false); break;
        }
    }
#undef MUKV_CHAIN
    return hipGetLastError();
}

static hipError_t wait_side(Ctx &c, int parity, hipStream_t st) {
    if (c.side_pending[parity]) {
        hipError_t e = hipStreamWaitEvent(st, c.ev_join[parity], 0);
        if (e != hipSuccess) return e;
        c.side_pending[parity] = false;
    }
    return hipSuccess;
}

static hipError_t wait_keep(Ctx &c, int parity, hipStream_t st) {
    if (c.keep_pending[parity]) {
        hipError_t e = hipStreamWaitEvent(st, c.ev_keep[parity], 0);
        if (e != hipSuccess) return e;
        c.keep_pending[parity] = false;
    }
    return hipSuccess;
}

static hipError_t wait_side_all(Ctx &c, hipStream_t st) {
    hipError_t e;
    for (int par = 0; par < 2; ++par) {
        if ((e = wait_keep(c, par, st)) != hipSuccess) return e;
        if ((e = wait_side(c, par, st)) != hipSuccess) return e;
    }
    return hipSuccess;
}

// split_side: on `side`, behind ev_fork, the keep of batch `a` -- ev_keep marks its end, which is all
// the copy of the batch's rows waits for -- and then, with re-scoring on, the fp64 chain: Eq. 1-4 redone
// for the listed frames, their rows copied (the main copy skips them), the batch's segment keys, the
// list emptied.  One stream for both: the next batch's keep is enqueued behind this chain, which has
// that batch's whole launch to finish in.  (A second library stream for the chain, forked from `side`
// inside a stream capture, ended a capture with a crash in the runtime and is not used.)
template <typename T>
static hipError_t launch_split_side(Ctx &c, const ChunkArgs &a, int n_part, int fft_parts = 0) {
    hipError_t e;
    const int par = a.parity;
    const bool need_att = c.cfg.alpha != 0.0 && !a.have_att_in;
    const bool need_fft = c.cfg.alpha != 1.0;
    if ((e = hipStreamWaitEvent(c.side, c.ev_fork, 0)) != hipSuccess) return e;
    {
        ProfScope ps(c, MUKV_K_SELECT, c.side);
        if ((e = launch_select<T, float>(c, a, c.att_part[par], n_part, c.fft_sig[par], 0, c.side, fft_parts)) != hipSuccess) return e;
    }
    if ((e = hipEventRecord(c.ev_keep[par], c.side)) != hipSuccess) return e;
    c.keep_pending[par] = true;
    if (c.margin_thr > 0.0) {
        ProfScope ps(c, MUKV_K_REFINE, c.side);
        int n_part64 = c.cfg.n_q_heads;
        if (need_att)
            if ((e = launch_att_generic<T, double>(c, a, true, c.att64, &n_part64, c.side)) != hipSuccess) return e;
        if (need_fft)
            if ((e = launch_freq<T, double>(c, a, true, c.fft64, c.side)) != hipSuccess) return e;
        if ((e = launch_select<T, double>(c, a, c.att64, n_part64, c.fft64, 1, c.side)) != hipSuccess) return e;
        if ((e = launch_compact(c, a, 2, c.side)) != hipSuccess) return e;
        hipLaunchKernelGGL(clear_count_kernel, dim3(1), dim3(1), 0, c.side, c.flag_count + par);
        if ((e = hipGetLastError()) != hipSuccess) return e;
    }
    if ((e = hipEventRecord(c.ev_join[par], c.side)) != hipSuccess) return e;
    c.side_pending[par] = true;
    return hipSuccess;
}

// The side stream's share of a batch, behind ev_fork (recorded on the caller's stream once the
// batch's signals are enqueued):
//  - with overlap_copy the keep itself (Eq. 4, top-kappa, block keys), so that the caller's stream
//    goes straight on to the next batch;
//  - with re-scoring on, the fp64 chain: frames with a near-tie at the keep boundary are on the
//    re-scoring list; Eq. 1-4 are redone for them in fp64 and the keep repeated.  Without
//    overlap_copy their rows are copied here, beside the main copy that skips them; with it the
//    copy has not been launched yet and will find the final rows of every frame.
// ev_join[parity] marks its end.
template <typename T>
static hipError_t launch_side(Ctx &c, const ChunkArgs &a, bool with_keep, int n_part) {
    hipError_t e;
    const bool need_att = c.cfg.alpha != 0.0 && !a.have_att_in;
    const bool need_fft = c.cfg.alpha != 1.0;
    if ((e = hipStreamWaitEvent(c.side, c.ev_fork, 0)) != hipSuccess) return e;
    if (direct_fp64(c)) {
        hipLaunchKernelGGL(list_all_kernel, dim3(1), dim3(256), 0, c.side, c.flag_list[a.parity], c.flag_count + a.parity,
                           a.n_frames);
        if ((e = hipGetLastError()) != hipSuccess) return e;
    } else if (with_keep) {
        ProfScope ps(c, MUKV_K_SELECT, c.side);
        if ((e = launch_select<T, float>(c, a, c.att_part[a.parity], n_part, c.fft_sig[a.parity], 0, c.side)) != hipSuccess)
            return e;
    }
    if (c.margin_thr > 0.0) {
        ProfScope ps(c, MUKV_K_REFINE, c.side);
        int n_part64 = c.cfg.n_q_heads;
        if (need_att)
            if ((e = launch_att_generic<T, double>(c, a, true, c.att64, &n_part64, c.side)) != hipSuccess) return e;
        if (need_fft)
            if ((e = launch_freq<T, double>(c, a, true, c.fft64, c.side)) != hipSuccess) return e;
        if ((e = launch_select<T, double>(c, a, c.att64, n_part64, c.fft64, 1, c.side)) != hipSuccess) return e;
        if (!with_keep)
            if ((e = launch_compact(c, a, 2, c.side)) != hipSuccess) return e;
        // empty the list for the next batch (a one-thread kernel: memset nodes are avoided in graphs)
        hipLaunchKernelGGL(clear_count_kernel, dim3(1), dim3(1), 0, c.side, c.flag_count + a.parity);
        if ((e = hipGetLastError()) != hipSuccess) return e;
    }
    if ((e = hipEventRecord(c.ev_join[a.parity], c.side)) != hipSuccess) return e;
    c.side_pending[a.parity] = true;
    return hipSuccess;
}

// The copy of a batch that was put off, launched on its own (no new batch to share a launch with):
// its keep, on the side stream, must have finished.
static hipError_t launch_deferred_copy(Ctx &c, const ChunkArgs &d, hipStream_t st) {
    hipError_t e;
    if (c.split_side) { // the keep is enough; re-scored frames and segment keys are the fp64 chain's
        if ((e = wait_keep(c, d.parity, st)) != hipSuccess) return e;
        ProfScope ps(c, MUKV_K_COMPACT, st);
        return launch_compact(c, d, c.margin_thr > 0.0 ? 1 : 0, st);
    }
    if ((e = wait_side(c, d.parity, st)) != hipSuccess) return e;
    ProfScope ps(c, MUKV_K_COMPACT, st);
    return launch_compact(c, d, 0, st);
}

// mukv_reset: the copies that were put off are forgotten.  What the side stream still does for
// those batches is harmless (the cache is empty again) and is waited for, by parity, before its
// scratch is used again.
hipError_t drop_deferred(Ctx &c) {
    c.n_deferred = 0;
    return hipSuccess;
}

hipError_t join_streams(Ctx &c, hipStream_t st) {
    hipError_t e;
    if (c.n_deferred) {
        hipStream_t ds = c.deferred_stream;
        for (int i = 0; i < c.n_deferred; ++i)
            if ((e = launch_deferred_copy(c, c.deferred[i], ds)) != hipSuccess) return e;
        c.n_deferred = 0;
        if (ds != st) {
            if ((e = hipEventRecord(c.ev_copy, ds)) != hipSuccess) return e;
            if ((e = hipStreamWaitEvent(st, c.ev_copy, 0)) != hipSuccess) return e;
        }
    }
    return wait_side_all(c, st);
}

// One batch.  Without overlap_copy, on the caller's stream: signals, keep, copy, with the fp64
// chain beside the copy.  With overlap_copy the caller's stream carries only
//     [copy of batch n-2 + frequency signal of batch n] (one launch), attention signal of batch n
// and the side stream the keep of batch n (and its fp64 chain) meanwhile: the keep of a batch has
// the next batch's launches to finish in, the copy of its rows follows two batches later.
template <typename T>
static hipError_t compress_typed(Ctx &c, const ChunkArgs &a, hipStream_t st) {
    hipError_t e;
    const bool need_att = c.cfg.alpha != 0.0 && !a.have_att_in;
    const bool direct64 = direct_fp64(c); // no fp32 pass at all: its frequency signal is not needed either
    const bool need_fft = c.cfg.alpha != 1.0 && !direct64;
    const bool overlap = c.cfg.overlap_copy != 0;
    const bool rescoring = c.margin_thr > 0.0;
    int n_part = c.cfg.n_q_heads, fft_parts = 0;
    // copies put off on another stream cannot share a launch with this batch
    if (c.n_deferred && c.deferred_stream != st)
        if ((e = join_streams(c, st)) != hipSuccess) return e;
    // This batch's parity was last used two batches ago: that batch's keep and fp64 chain must be
    // through with the scratch (they have had a whole batch of launches to do so), and its rows
    // may now be copied.
    // (split_side: the keep alone -- the fp64 chain has streams and scratch of its own)
    if ((e = c.split_side ? wait_keep(c, a.parity, st) : wait_side(c, a.parity, st)) != hipSuccess) return e;
    const bool have_old = c.n_deferred == 2;
    // split_side: the main copy skips the frames on the re-scoring list and leaves the segment keys to the fp64 chain
    const int copy_mode = (c.split_side && rescoring) ? 1 : 0;
    if (overlap && need_att && chain_supported(c, a)) {
        // one launch: the rows of batch n-2, both signals of this batch
        {
            ProfScope ps(c, MUKV_K_CHAIN, st);
            if ((e = launch_chain(c, have_old ? &c.deferred[0] : nullptr, copy_mode, a, need_fft, &n_part, &fft_parts, st)) != hipSuccess) return e;
        }
        if (have_old) {
            c.deferred[0] = c.deferred[1];
            c.n_deferred = 1;
        }
        if ((e = hipEventRecord(c.ev_fork, st)) != hipSuccess) return e;
        if ((e = launch_split_side<T>(c, a, n_part, fft_parts)) != hipSuccess) return e;
        c.deferred[c.n_deferred++] = a;
        c.deferred_stream = st;
        return hipSuccess;
    }
    if (have_old && need_fft && c.cfg.freq_axis == MUKV_FREQ_FEATURE) {
        // the copy shares its launch with this batch's frequency kernel: HBM-bound beside
        // arithmetic-bound work (the attention kernel streams all the queries and gains nothing
        // beside a copy)
        ProfScope ps(c, MUKV_K_COPY_FREQ, st);
        if ((e = launch_copy_freq<T>(c, c.deferred[0], copy_mode, a, st)) != hipSuccess) return e;
    } else {
        if (have_old)
            if ((e = launch_deferred_copy(c, c.deferred[0], st)) != hipSuccess) return e;
        if (need_fft) {
            ProfScope ps(c, MUKV_K_FREQ, st);
            if ((e = launch_freq<T, float>(c, a, false, c.fft_sig[a.parity], st)) != hipSuccess) return e;
        }
    }
    if (have_old) {
        c.deferred[0] = c.deferred[1];
        c.n_deferred = 1;
    }
    if (need_att) {
        ProfScope ps(c, MUKV_K_ATT, st);
        if (c.use_mfma) {
            if ((e = launch_att_mfma(c, a, c.att_part[a.parity], &n_part, st)) != hipSuccess) return e;
        } else {
            if ((e = launch_att_generic<T, float>(c, a, false, c.att_part[a.parity], &n_part, st)) != hipSuccess) return e;
        }
    }
    if (overlap) { // keep on the side stream; the copy waits for the batch after next (or a flush / retrieve / gather call)
        if ((e = hipEventRecord(c.ev_fork, st)) != hipSuccess) return e;
        if ((e = c.split_side ? launch_split_side<T>(c, a, n_part) : launch_side<T>(c, a, true, n_part)) != hipSuccess) return e;
        c.deferred[c.n_deferred++] = a;
        c.deferred_stream = st;
        return hipSuccess;
    }
    if (direct64) { // everything of this batch is the fp64 chain's: keep, rows of every unit, segment keys
        if ((e = hipEventRecord(c.ev_fork, st)) != hipSuccess) return e;
        if ((e = launch_side<T>(c, a, false, n_part)) != hipSuccess) return e;
        return wait_side(c, a.parity, st);
    }
    {
        ProfScope ps(c, MUKV_K_SELECT, st);
        if ((e = launch_select<T, float>(c, a, c.att_part[a.parity], n_part, c.fft_sig[a.parity], 0, st)) != hipSuccess) return e;
    }
    if (rescoring) {
        if ((e = hipEventRecord(c.ev_fork, st)) != hipSuccess) return e;
        if ((e = launch_side<T>(c, a, false, n_part)) != hipSuccess) return e;
    }
    {
        ProfScope ps(c, MUKV_K_COMPACT, st);
        if ((e = launch_compact(c, a, rescoring ? 1 : 0, st)) != hipSuccess) return e;
    }
    return wait_side(c, a.parity, st);
}

hipError_t launch_compress(Ctx &c, const ChunkArgs &a, hipStream_t st) {
    return c.cfg.dtype == MUKV_BF16 ? compress_typed<uint16_t>(c, a, st) : compress_typed<float>(c, a, st);
}

} // namespace mukv
