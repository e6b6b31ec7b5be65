// Attention of new tokens over the retrieved context at one layer (Sec. 3.5, Eq. 9): queries
// W_Q X against keys [R_k, W_K X] and values [R_v, W_V X], where R are the kept rows of the
// frames chosen by the retrieval -- read in place from the store, no gathered copy -- and X the
// caller's own ("local") rows.
//
// attend_partial_kernel: one workgroup per (question, KV head, tile of up to 8 queries, split of
// the frame list).  A query of the tile is a (token, head of the KV group) pair, so a key / value
// row is read once for all the heads that share it.  Rows are taken in chunks of up to 512:
//   1. a table of where each row of the chunk lives (store row or local row) and which token is
//      the first to see it;
//   2. the scores of the chunk, kept in LDS, and their maximum per query.  bf16 rows of 32, 64 or
//      128 features: S^T = K Q^T with v_mfma_f32_16x16x32_bf16, 16 key rows per wave and step,
//      the A operand loaded straight from the row (lane % 16 = row, 8 features from
//      8 * (lane / 16) of every 32).  Otherwise: a row spread over D/E lanes (E = elements in 16
//      bytes), dot products reduced over those lanes;
//   3. with that maximum fixed, the weights exp2(score - maximum), once per (row, query), and their sums --
//      so the running sums are rescaled once per chunk, not once per row;
//   4. the value accumulation.  bf16 rows of 32, 64 or 128 features: O = P V on the matrix cores -- the
//      weights as bf16 pairs hi + lo (two products, nothing of the fp32 weight is lost) are the A operand,
//      the value rows pass through LDS 64 at a time, row-major as they come from memory, and the LDS
//      transpose read (ds_read_b64_tr_b16) hands every lane the 8 rows of one feature that the B operand
//      wants; a wave owns 16-feature tiles of the output, so nothing is left to add across lanes.
//      Otherwise: a value row spread over D/E lanes, 256*E/D rows per pass, multiply-adds on the VALU and a
//      sum over the lanes that hold the same piece of different rows.
// The split's (maximum, normaliser, unnormalised output) per query go to a scratch table;
// attend_combine_kernel merges the splits and writes the output in the payload type.
// Everything is summed in a fixed order: the result does not depend on timing.
//
// The prefill of new tokens (Sec. 3.2: they attend to the past cache and to themselves) is the same
// computation with many query tokens, and yields Eq. 1 -- the attention each new token receives --
// on the way: the merge also writes every query's log-sum-exp; prefill_colsum_kernel recomputes the
// scores of a tile's queries against the new tokens' keys, turns them into softmax weights with
// that log-sum-exp and adds them over the tile; prefill_signal_kernel adds the tiles and KV heads in
// order and divides by Hq * n_q.  Scratch for it comes from the caller (a workspace argument).
#include <climits>

#include "mukv_internal.h"

namespace mukv {

namespace {

constexpr int kTileQ = 8;    // queries per workgroup
constexpr int kChunk = 512;  // rows whose scores are held in LDS at a time
constexpr int kThreads = 256;
constexpr int kUnroll = 4;   // rows a lane has in flight
constexpr int kStepsA = 2;   // matrix path: 16-row steps of a wave whose loads are issued together

struct AttendArgs {
    const void *q;            // [B][n_q][Hq][D]
    const int32_t *frame_idx; // [B][k_frame] or null
    const void *k_local, *v_local; // [n_local_total][Hkv][D] or null
    const int32_t *local_offsets;  // [B+1] or null
    const void *store_k, *store_v; // the layer's slabs: [Hkv][store_cap][D]
    float *part;                   // [B][n_q*Hq][n_split][D+2]
    int64_t store_cap;
    int n_q, Hq, Hkv, G, k_frame, kappa, n_frames, n_split, frames_per_split, n_qtiles, causal;
    float scale_log2e;
};

template <typename T>
struct Row16;
typedef __attribute__((ext_vector_type(4))) unsigned int raw16; // 16 bytes as they come from memory
template <>
struct Row16<uint16_t> { // eight bf16
    static constexpr int E = 8;
    __device__ static void expand(raw16 u, float *x) {
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            x[2 * i] = __uint_as_float(u[i] << 16);
            x[2 * i + 1] = __uint_as_float(u[i] & 0xFFFF0000u);
        }
    }
};
template <>
struct Row16<float> {
    static constexpr int E = 4;
    __device__ static void expand(raw16 u, float *x) {
#pragma unroll
        for (int i = 0; i < 4; ++i) x[i] = __uint_as_float(u[i]);
    }
};
template <typename T>
__device__ __forceinline__ raw16 load16(const T *p) {
    return *reinterpret_cast<const raw16 *>(p);
}

// sum over the LPR consecutive lanes that hold one row; result in all of them
template <int LPR>
__device__ __forceinline__ float row_lanes_sum(float v) {
    if constexpr (LPR >= 2) v += lane_xor<1>(v);
    if constexpr (LPR >= 4) v += lane_xor<2>(v);
    if constexpr (LPR >= 8) v += lane_xor<4>(v);
    if constexpr (LPR >= 16) v += lane_xor<8>(v);
    if constexpr (LPR >= 32) v += lane_xor<16>(v);
    return v;
}
// sum over the lanes of a wave that hold the same piece of different rows; result in all of them
template <int LPR>
__device__ __forceinline__ float same_piece_sum(float v) {
    if constexpr (LPR <= 1) v += lane_xor<1>(v);
    if constexpr (LPR <= 2) v += lane_xor<2>(v);
    if constexpr (LPR <= 4) v += lane_xor<4>(v);
    if constexpr (LPR <= 8) v += lane_xor<8>(v);
    // across rows of 16 lanes: the LDS crossbar shuffle (the register-swap instructions, used 72
    // times in a row at the end of the kernel, cost it ~70 registers)
    if constexpr (LPR <= 16) v += __shfl_xor(v, 16);
    if constexpr (LPR <= 32) v += __shfl_xor(v, 32);
    return v;
}

__device__ __forceinline__ uint16_t bf16_round(float x) { // round to nearest even; inputs are finite
    const uint32_t u = __float_as_uint(x);
    return (uint16_t)((u + 0x7FFFu + ((u >> 16) & 1u)) >> 16);
}
__device__ __forceinline__ void store_out(uint16_t *p, float x) { *p = bf16_round(x); }
__device__ __forceinline__ void store_out(float *p, float x) { *p = x; }

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(2))) float f32x2;
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
typedef __attribute__((ext_vector_type(4))) int i32x4;
typedef __attribute__((ext_vector_type(2))) unsigned int u32x2;
typedef __attribute__((ext_vector_type(4))) short i16x4;
typedef __attribute__((ext_vector_type(8))) short i16x8;
// ds_read_b64_tr_b16, the LDS transpose read of 16-bit elements: every lane names 8 bytes; within each block
// of 16 lanes, result[t] of lane i is element i % 4 of the 8 bytes named by lane 4 * t + i / 4 of the block,
// t = 0..3 (lane layout checked by an in-bounds probe on the device).
__device__ __forceinline__ i16x4 lds_read_tr16(const unsigned char *p) {
    return __builtin_amdgcn_ds_read_tr16_b64_v4i16((i16x4 __attribute__((address_space(3))) *)(p));
}

template <typename T, int D>
__global__ __launch_bounds__(kThreads) __attribute__((amdgpu_waves_per_eu(3))) void attend_partial_kernel(AttendArgs a) {
    constexpr int E = Row16<T>::E, LPR = D / E, RPP = kThreads / LPR; // lanes per row, rows per pass
    // bf16 rows whose length is a multiple of 32: the scores come from the matrix cores
    constexpr bool kMfma = sizeof(T) == 2 && D % 32 == 0;
    constexpr int kWaves = kThreads / 64;
    static_assert(LPR >= 1 && LPR <= 32, "a row fits in half a wave");
    // Matrix path, value side: the chunk's value rows pass through LDS kSub at a time (row-major, padded rows) and
    // come back as B operands by the LDS transpose read; the weights are bf16 pairs (hi + lo, so that nothing of
    // the fp32 weight is lost) as A operands; a wave owns TPW 16-feature tiles of the output.
    constexpr int kSub = 64, kVStride = D * 2 + 16;
    constexpr int NP = kMfma ? kSub / RPP : 1; // 16-byte pieces of kSub rows per thread
    constexpr int NT = D / 16, TPW = NT >= kWaves ? NT / kWaves : 1;
    constexpr int kPRow = kChunk * 2 + 16; // bytes of a query's row of bf16 weights
    // scores of the chunk, log2 units (rows padded by 8 floats).  VALU path: after the last chunk the same memory
    // takes the per-wave outputs.  Matrix path: the weight pass rewrites it as the hi rows, then the lo rows.
    __shared__ __align__(16) float s_sc[kTileQ][kChunk + 8];
    static_assert(kWaves * (D > 64 ? D : 64) <= kChunk, "the per-wave outputs fit where the scores were");
    static_assert(2 * kTileQ * kPRow <= (int)sizeof(s_sc), "hi and lo weights fit where the scores were");
    unsigned char *const s_ph = reinterpret_cast<unsigned char *>(&s_sc[0][0]);
    unsigned char *const s_pl = s_ph + kTileQ * kPRow;
    __shared__ int s_row[kChunk]; // where row i of the chunk lives: >= 0 store row, <= -2 local row -2 - code, -1 nowhere
    __shared__ int s_ft[kChunk];  // first token that sees the row (INT_MAX: nobody does)
    __shared__ float s_wmax[kWaves][kTileQ]; // per-wave maxima of the chunk
    __shared__ float s_run[kTileQ];  // running maximum of every query over the chunks so far
    __shared__ float s_corr[kTileQ]; // factor that brings the sums so far to the new maximum
    __shared__ float s_ref[kTileQ];  // what the exponent subtracts: the running maximum, or 0 while nothing was seen
    __shared__ float s_zq[kTileQ];
    // VALU path: softmax weights of the chunk (unnormalised), row-major.  Matrix path: kSub staged value rows.
    __shared__ __align__(16) unsigned char s_u[kMfma ? kSub * kVStride : kChunk * kTileQ * 4];
    float(*const s_p)[kTileQ] = reinterpret_cast<float(*)[kTileQ]>(s_u);
    unsigned char *const s_v = s_u;
    __shared__ int s_frame[kMaxGatherK]; // this split's frames; -1: names no frame of the cache
    const int sp = blockIdx.x, g = blockIdx.y % a.Hkv, qt = blockIdx.y / a.Hkv, b = blockIdx.z;
    const int tid = threadIdx.x, li = tid % LPR, rg = tid / LPR, wave = tid >> 6, lane = tid & 63;
    const int lr = lane & 15, lg = lane >> 4;
    const int n_queries = a.n_q * a.G; // of this KV head: (token, head in group), token-major
    const T *q = static_cast<const T *>(a.q);
    auto query_row = [&](int n, bool *ok) { // element offset of query n of the tile
        const int qq = qt * kTileQ + n;
        *ok = n < kTileQ && qq < n_queries;
        const int i = *ok ? qq / a.G : 0, h = g * a.G + (*ok ? qq % a.G : 0);
        return (((int64_t)b * a.n_q + i) * a.Hq + h) * D;
    };
    auto token_of = [&](int n) { // INT_MIN: no such query, sees nothing
        const int qq = qt * kTileQ + n;
        return (n < kTileQ && qq < n_queries) ? qq / a.G : INT_MIN;
    };

    // VALU path: this lane's piece of every query of the tile, scaled so that scores come out in
    // log2 units.  Matrix path: the queries as the B operand (column lane % 16 = query, 8 features
    // from 8 * (lane / 16) of every 32), unscaled.
    float qr[kMfma ? 1 : kTileQ][E];
    if constexpr (!kMfma) {
#pragma unroll
        for (int n = 0; n < kTileQ; ++n) {
            bool ok;
            const int64_t off = query_row(n, &ok);
            float x[E];
            Row16<T>::expand(load16(q + off + li * E), x);
#pragma unroll
            for (int e = 0; e < E; ++e) qr[n][e] = ok ? x[e] * a.scale_log2e : 0.f;
        }
    }

    bf16x8 qb[kMfma ? D / 32 : 1]; // requested before anything else, needed after the first tables
    if constexpr (kMfma) {
        bool ok;
        const int64_t off = query_row(lr, &ok);
#pragma unroll
        for (int kk = 0; kk < D / 32; ++kk) {
            raw16 u = load16(q + off + kk * 32 + lg * 8);
            if (!ok) u = raw16{0u, 0u, 0u, 0u};
            qb[kk] = __builtin_bit_cast(bf16x8, u);
        }
    }

    // rows of this split: kept rows of its frames, then (last split only) the local rows
    const int f_lo = sp * a.frames_per_split;
    const int f_hi = f_lo + a.frames_per_split < a.k_frame ? f_lo + a.frames_per_split : a.k_frame;
    const int n_ret = f_hi > f_lo ? (f_hi - f_lo) * a.kappa : 0;
    int l0 = 0, n_loc = 0;
    if (a.local_offsets && sp == a.n_split - 1) {
        l0 = a.local_offsets[b];
        n_loc = a.local_offsets[b + 1] - l0;
        if (n_loc < 0) n_loc = 0;
    }
    const int total = n_ret + n_loc;
    for (int i = tid; i < f_hi - f_lo; i += kThreads) {
        const int f = a.frame_idx[(int64_t)b * a.k_frame + f_lo + i];
        s_frame[i] = (f >= 0 && f < a.n_frames) ? f : -1;
    }
    __syncthreads();
    const T *sk = static_cast<const T *>(a.store_k) + (int64_t)g * a.store_cap * D;
    const T *sv = static_cast<const T *>(a.store_v) + (int64_t)g * a.store_cap * D;
    const T *lk = static_cast<const T *>(a.k_local), *lv = static_cast<const T *>(a.v_local);
    // address of a row from its code; a row that lives nowhere reads the slab's first row (valid
    // memory, the result is masked)
    auto row_ptr = [&](const T *store, const T *local, int code) -> const T * {
        if (code >= 0) return store + (int64_t)code * D;
        if (code <= -2) return local + ((int64_t)(-2 - code) * a.Hkv + g) * D;
        return store;
    };

    float o[kMfma ? 1 : kTileQ][E]; // VALU path: this lane's 16-byte piece of the output of every query
    f32x4 acc[TPW];                 // matrix path: queries 4 * (lane / 16) + r, feature 16 * tile + lane % 16
    float zq = 0.f; // this thread's share of the normaliser of query tid / 32
    static_assert(kThreads / 32 == kTileQ, "32 threads per query in the weight pass");
    if (tid < kTileQ) s_run[tid] = -INFINITY; // read again only after the barriers of the first chunk
#pragma unroll
    for (int n = 0; n < (kMfma ? 1 : kTileQ); ++n) {
#pragma unroll
        for (int e = 0; e < E; ++e) o[n][e] = 0.f;
    }
#pragma unroll
    for (int t = 0; t < TPW; ++t) acc[t] = f32x4{0.f, 0.f, 0.f, 0.f};

    // matrix path: this thread's pieces of kSub value rows, on their way while the rows before them are used.
    // Loads are unconditional (a row that lives nowhere, or past the chunk, reads the slab's first row); what
    // was loaded instead of a row becomes zeros (its weights are zero, but zero times anything must stay zero).
    raw16 vx[NP];
    int n_rows = 0;
    auto load_sub = [&](raw16(&vreg)[NP], int sub) {
#pragma unroll
        for (int p = 0; p < NP; ++p) {
            const int i = sub * kSub + p * RPP + rg;
            const int code = i < n_rows ? s_row[i] : -1;
            const raw16 x = load16(row_ptr(sv, lv, code) + li * E);
            vreg[p] = code == -1 ? raw16{0u, 0u, 0u, 0u} : x;
        }
    };

    for (int c0 = 0; c0 < total; c0 += kChunk) {
        n_rows = (c0 + kChunk < total ? c0 + kChunk : total) - c0;
        // ---- where the rows of the chunk live and who sees them ----
        for (int i = tid; i < n_rows; i += kThreads) {
            const int r = c0 + i;
            int code, ft = 0;
            if (r < n_ret) {
                const int slot = r / a.kappa;
                const int f = s_frame[slot];
                code = f < 0 ? -1 : f * a.kappa + (r - slot * a.kappa);
            } else {
                const int j = r - n_ret;
                code = -2 - (l0 + j);
                if (a.causal) ft = j - (n_loc - a.n_q); // token i sees local row j iff j <= n_loc - n_q + i
            }
            s_row[i] = code;
            s_ft[i] = code == -1 ? INT_MAX : ft;
        }
        __syncthreads();
        // ---- scores of the chunk and their maxima ----
        if constexpr (kMfma) {
            // 16 rows per wave and step: S^T = K Q^T, so a lane ends up with one query (lane % 16)
            // and the four rows 4 * (lane / 16) .. +3 of the step
            const int my_tok = token_of(lr);
            float m_q = -INFINITY;
            // the key rows of kStepsA steps are requested together (rows past the chunk read its last row again:
            // loads stay unconditional).  Requesting the next batch before this one is used, and larger batches,
            // were measured and changed nothing: the launch moves its rows at the pace of the memory
            constexpr int kBatch = kStepsA * 16 * kWaves;
            auto load_k = [&](raw16(&ka)[kStepsA][D / 32], int R0) {
#pragma unroll
                for (int t = 0; t < kStepsA; ++t) {
                    const int i = R0 + t * 16 * kWaves + lr;
                    const T *kp = row_ptr(sk, lk, s_row[i < n_rows ? i : n_rows - 1]) + lg * 8;
#pragma unroll
                    for (int kk = 0; kk < D / 32; ++kk) ka[t][kk] = load16(kp + kk * 32);
                }
            };
            auto use_k = [&](const raw16(&ka)[kStepsA][D / 32], int R0) {
#pragma unroll
                for (int t = 0; t < kStepsA; ++t) {
                    const int R = R0 + t * 16 * kWaves;
                    if (R >= n_rows) break;
                    f32x4 d = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
                    for (int kk = 0; kk < D / 32; ++kk)
                        d = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, ka[t][kk]), qb[kk], d, 0, 0, 0);
#pragma unroll
                    for (int r = 0; r < 4; ++r) {
                        const int i2 = R + 4 * lg + r;
                        if (i2 < n_rows && lr < kTileQ) {
                            const float sc = my_tok >= s_ft[i2] ? d[r] * a.scale_log2e : -INFINITY;
                            s_sc[lr][i2] = sc;
                            m_q = fmaxf(m_q, sc);
                        }
                    }
                }
            };
            raw16 kx[kStepsA][D / 32];
            for (int R0 = 16 * wave; R0 < n_rows; R0 += kBatch) {
                load_k(kx, R0);
                use_k(kx, R0);
            }
            m_q = xrow_max(m_q);
            if (lg == 0 && lr < kTileQ) s_wmax[wave][lr] = m_q;
        } else {
            int tok[kTileQ];
            float m_loc[kTileQ];
#pragma unroll
            for (int n = 0; n < kTileQ; ++n) {
                tok[n] = token_of(n);
                m_loc[n] = -INFINITY;
            }
            for (int i0 = rg; i0 < n_rows; i0 += kUnroll * RPP) {
                // all loads of the batch first, each from an address that is valid whatever the row is
                raw16 kr[kUnroll];
#pragma unroll
                for (int u = 0; u < kUnroll; ++u) {
                    const int i = i0 + u * RPP;
                    kr[u] = load16(row_ptr(sk, lk, s_row[i < n_rows ? i : n_rows - 1]) + li * E);
                }
#pragma unroll
                for (int u = 0; u < kUnroll; ++u) {
                    const int i = i0 + u * RPP;
                    if (i >= n_rows) break;
                    const int ft = s_ft[i];
                    float kx[E];
                    Row16<T>::expand(kr[u], kx);
#pragma unroll
                    for (int n = 0; n < kTileQ; ++n) {
                        float sc = 0.f;
#pragma unroll
                        for (int e = 0; e < E; ++e) sc = fmaf(qr[n][e], kx[e], sc);
                        sc = row_lanes_sum<LPR>(sc);
                        if (tok[n] < ft) sc = -INFINITY;
                        if (li == 0) s_sc[n][i] = sc;
                        m_loc[n] = fmaxf(m_loc[n], sc);
                    }
                }
            }
#pragma unroll
            for (int n = 0; n < kTileQ; ++n) {
                const float m = wave_max(m_loc[n]);
                if (lane == 0) s_wmax[wave][n] = m;
            }
        }
        if constexpr (kMfma) load_sub(vx, 0); // the first value rows are on their way while the maxima are agreed on
        __syncthreads();
        // ---- new running maximum: rescale what has been summed so far (once per chunk) ----
        if (tid < kTileQ) {
            float m = s_wmax[0][tid];
#pragma unroll
            for (int w = 1; w < kWaves; ++w) m = fmaxf(m, s_wmax[w][tid]);
            const float m_old = s_run[tid], m_new = fmaxf(m_old, m);
            s_corr[tid] = m_old == -INFINITY ? 0.f : __builtin_amdgcn_exp2f(m_old - m_new);
            s_run[tid] = m_new;
            s_ref[tid] = m_new == -INFINITY ? 0.f : m_new;
        }
        __syncthreads();
        if constexpr (kMfma) {
            if (c0 > 0) {
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    const float corr = s_corr[(4 * lg + r) & (kTileQ - 1)];
#pragma unroll
                    for (int t = 0; t < TPW; ++t) acc[t][r] *= corr;
                }
            }
            // ---- the weights, once per (row, query): 32 threads per query walk the rows; their sums.  The
            // scores are taken into registers first, then the same memory receives the weights as bf16 pairs;
            // rows up to the next multiple of kSub get zero weights ----
            const int n = tid >> 5;
            const float ref = s_ref[n];
            if (c0 > 0) zq *= s_corr[n];
            const int n_pad = (n_rows + kSub - 1) / kSub * kSub;
            float sreg[kChunk / 32];
#pragma unroll
            for (int k = 0; k < kChunk / 32; ++k) {
                const int i = (tid & 31) + 32 * k;
                sreg[k] = i < n_rows ? s_sc[n][i] : -INFINITY;
            }
            __syncthreads();
#pragma unroll
            for (int k = 0; k < kChunk / 32; ++k) {
                if (32 * k >= n_pad) break;
                const int i = (tid & 31) + 32 * k;
                const float p = __builtin_amdgcn_exp2f(sreg[k] - ref); // exp2(-inf) = 0 for a masked row
                zq += p;
                const uint16_t hi = bf16_round(p);
                const uint16_t lo = bf16_round(p - __uint_as_float((uint32_t)hi << 16));
                *reinterpret_cast<uint16_t *>(s_ph + n * kPRow + 2 * i) = hi;
                *reinterpret_cast<uint16_t *>(s_pl + n * kPRow + 2 * i) = lo;
            }
            // ---- value accumulation on the matrix cores, kSub rows at a time ----
            const int n_sub = n_pad / kSub;
            // stage the rows held in vreg, request the next ones, multiply (two sets of rows in flight, like
            // larger sets, were measured and changed nothing)
            auto do_sub = [&](raw16(&vreg)[NP], int sub) {
                __syncthreads(); // the rows staged before have been used (first time round: the weights are written)
#pragma unroll
                for (int p = 0; p < NP; ++p)
                    *reinterpret_cast<raw16 *>(s_v + (p * RPP + rg) * kVStride + li * 16) = vreg[p];
                __syncthreads();
                if (sub + 1 < n_sub) load_sub(vreg, sub + 1);
                if (wave * TPW < NT) {
#pragma unroll
                    for (int st = 0; st < kSub / 32; ++st) {
                        const int r0 = sub * kSub + 32 * st;
                        if (r0 >= n_rows) break;
                        const unsigned char *pa = s_ph + (lr & (kTileQ - 1)) * kPRow + 2 * (r0 + 8 * lg);
                        const bf16x8 ah = __builtin_bit_cast(bf16x8, *reinterpret_cast<const raw16 *>(pa));
                        const bf16x8 al = __builtin_bit_cast(bf16x8, *reinterpret_cast<const raw16 *>(pa + kTileQ * kPRow));
#pragma unroll
                        for (int t = 0; t < TPW; ++t) {
                            const unsigned char *vp = s_v + (32 * st + 8 * lg + (lr >> 2)) * kVStride +
                                                      2 * (16 * (wave * TPW + t) + 4 * (lr & 3));
                            const i16x4 v0 = lds_read_tr16(vp), v1 = lds_read_tr16(vp + 4 * kVStride);
                            const bf16x8 bv = __builtin_bit_cast(bf16x8, i16x8{v0[0], v0[1], v0[2], v0[3], v1[0], v1[1], v1[2], v1[3]});
                            acc[t] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(ah, bv, acc[t], 0, 0, 0);
                            acc[t] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(al, bv, acc[t], 0, 0, 0);
                        }
                    }
                }
            };
            for (int sub = 0; sub < n_sub; ++sub) do_sub(vx, sub);
        } else {
            if (c0 > 0) {
#pragma unroll
                for (int n = 0; n < kTileQ; ++n) {
                    const float corr = s_corr[n];
#pragma unroll
                    for (int e = 0; e < E; ++e) o[n][e] *= corr;
                }
            }
            // ---- the weights, once per (row, query): 32 threads per query walk the rows; their sums ----
            {
                const int n = tid >> 5;
                const float ref = s_ref[n];
                if (c0 > 0) zq *= s_corr[n];
                for (int i = tid & 31; i < n_rows; i += 32) {
                    const float p = __builtin_amdgcn_exp2f(s_sc[n][i] - ref); // exp2(-inf) = 0 for a masked row
                    s_p[i][n] = p;
                    zq += p;
                }
            }
            __syncthreads();
            // ---- value accumulation: a value row spread over LPR lanes, kUnroll rows per lane in flight ----
            for (int i0 = rg; i0 < n_rows; i0 += kUnroll * RPP) {
                raw16 vr[kUnroll];
#pragma unroll
                for (int u = 0; u < kUnroll; ++u) {
                    const int i = i0 + u * RPP;
                    vr[u] = load16(row_ptr(sv, lv, s_row[i < n_rows ? i : n_rows - 1]) + li * E);
                }
#pragma unroll
                for (int u = 0; u < kUnroll; ++u) {
                    const int i = i0 + u * RPP;
                    if (i >= n_rows || s_row[i] == -1) continue; // what was loaded instead of a row is not a value
                    float vx[E];
                    Row16<T>::expand(vr[u], vx);
                    const f32x4 p0 = *reinterpret_cast<const f32x4 *>(&s_p[i][0]);
                    const f32x4 p1 = *reinterpret_cast<const f32x4 *>(&s_p[i][4]);
#pragma unroll
                    for (int n = 0; n < kTileQ; ++n) {
                        const float p = n < 4 ? p0[n & 3] : p1[n & 3];
#pragma unroll
                        for (int e = 0; e < E; ++e) o[n][e] = fmaf(p, vx[e], o[n][e]);
                    }
                }
            }
        }
        __syncthreads(); // the tables are rewritten by the next chunk
    }

    zq += lane_xor<1>(zq); // the 32 threads of a query are half a wave
    zq += lane_xor<2>(zq);
    zq += lane_xor<4>(zq);
    zq += lane_xor<8>(zq);
    zq += __shfl_xor(zq, 16);
    if ((tid & 31) == 0) s_zq[tid >> 5] = zq;
    // the split's record of a query: [0] running maximum, [1] normaliser, [2..] unnormalised output
    // (merged by a launch of its own: a merge by the last workgroup to finish, with records that cross the
    // XCDs' L2 caches as device-scope atomics, took as long as that launch for 64 questions and longer for one)
    auto record = [&](int n) -> float * { // of query n of the tile; null: no such query
        const int qq = qt * kTileQ + n;
        if (qq >= n_queries) return nullptr;
        const int i = qq / a.G, h = g * a.G + qq % a.G;
        return a.part + ((((int64_t)b * a.n_q + i) * a.Hq + h) * a.n_split + sp) * (D + 2);
    };
    if constexpr (kMfma) {
        // the matrix cores have added all rows already: a lane writes what it holds (lanes 32.. hold copies)
        if (lg < 2 && wave * TPW < NT) {
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                float *rec = record(4 * lg + r);
                if (!rec) continue;
#pragma unroll
                for (int t = 0; t < TPW; ++t) rec[2 + 16 * (wave * TPW + t) + lr] = acc[t][r];
            }
        }
        __syncthreads();
    } else {
        // ---- add the rows held by different lanes: inside a wave, then across the waves ----
#pragma unroll
        for (int n = 0; n < kTileQ; ++n) {
#pragma unroll
            for (int e = 0; e < E; ++e) o[n][e] = same_piece_sum<LPR>(o[n][e]);
        }
        __syncthreads(); // (every wave is done with the chunk's scores)
        if (lane < LPR) {
#pragma unroll
            for (int n = 0; n < kTileQ; ++n)
#pragma unroll
                for (int e = 0; e < E; ++e) s_sc[n][wave * (D > 64 ? D : 64) + li * E + e] = o[n][e];
        }
        __syncthreads();
        for (int idx = tid; idx < kTileQ * D; idx += kThreads) {
            const int n = idx / D, d = idx - n * D;
            float *rec = record(n);
            if (!rec) continue;
            float val = 0.f;
#pragma unroll
            for (int w = 0; w < kWaves; ++w) val += s_sc[n][w * (D > 64 ? D : 64) + d];
            rec[2 + d] = val;
        }
    }
    if (tid < kTileQ) {
        float *rec = record(tid);
        if (rec) {
            rec[0] = s_run[tid];
            rec[1] = s_zq[tid];
        }
    }
}

// out[b][i][h][:] = sum_s o_s 2^(m_s - m) / sum_s z_s 2^(m_s - m), m = max_s m_s; zero if no split saw a key
// lse (may be null): log2 of the query's softmax denominator, in the scores' log2 units; +inf for a
// query that sees no key, so that every weight computed from it is zero.
template <typename T, int D>
__global__ void attend_combine_kernel(const float *__restrict__ part, int n_split, T *__restrict__ out,
                                      float *__restrict__ lse) {
    const int64_t row = blockIdx.x;
    const float *p = part + row * n_split * (D + 2);
    for (int d = threadIdx.x; d < D; d += blockDim.x) {
        // every record's maximum, normaliser and this thread's element requested before any is used
        float ms[kAttendMaxSplit], zz[kAttendMaxSplit], oo[kAttendMaxSplit];
#pragma unroll
        for (int s = 0; s < kAttendMaxSplit; ++s) {
            const float *ps = p + (s < n_split ? s : 0) * (D + 2);
            ms[s] = ps[0];
            zz[s] = ps[1];
            oo[s] = ps[2 + d];
        }
        float m = -INFINITY;
#pragma unroll
        for (int s = 0; s < kAttendMaxSplit; ++s)
            if (s < n_split) m = fmaxf(m, ms[s]);
        float zs = 0.f, os = 0.f;
        if (m > -INFINITY) {
#pragma unroll
            for (int s = 0; s < kAttendMaxSplit; ++s) {
                if (s >= n_split) break;
                const float w = ms[s] == -INFINITY ? 0.f : __builtin_amdgcn_exp2f(ms[s] - m);
                zs = fmaf(zz[s], w, zs);
                os = fmaf(oo[s], w, os);
            }
        }
        store_out(out + row * D + d, zs > 0.f ? os / zs : 0.f);
        if (lse && d == 0) lse[row] = zs > 0.f ? m + __builtin_amdgcn_logf(zs) : INFINITY;
    }
}

// Softmax weights of a tile's queries on the new tokens (the last n_q local rows of the question),
// added over the tile.  Grid (query tile, KV head, question).  The tile's queries sit in LDS as
// scaled floats; a thread takes new token j, j + 256, ...: its key row against all queries of the tile.
// colpart [B][Hkv][n_qtiles][n_q].
template <typename T, int D>
__global__ __launch_bounds__(kThreads) void prefill_colsum_kernel(AttendArgs a, const float *__restrict__ lse,
                                                                  float *__restrict__ colpart) {
    constexpr int E = Row16<T>::E;
    __shared__ float s_q[kTileQ][D];
    __shared__ float s_l[kTileQ];
    __shared__ int s_tok[kTileQ];
    const int qt = blockIdx.x, g = blockIdx.y, b = blockIdx.z, tid = threadIdx.x;
    const int n_queries = a.n_q * a.G;
    const T *q = static_cast<const T *>(a.q);
    for (int idx = tid; idx < kTileQ * D; idx += kThreads) {
        const int n = idx / D, d = idx - n * D;
        const int qq = qt * kTileQ + n;
        float x = 0.f;
        if (qq < n_queries) {
            const int i = qq / a.G, h = g * a.G + qq % a.G;
            float one[E];
            Row16<T>::expand(load16(q + (((int64_t)b * a.n_q + i) * a.Hq + h) * D + (d / E) * E), one);
            x = one[d % E] * a.scale_log2e;
        }
        s_q[n][d] = x;
    }
    if (tid < kTileQ) {
        const int qq = qt * kTileQ + tid;
        const bool ok = qq < n_queries;
        const int i = ok ? qq / a.G : 0, h = g * a.G + (ok ? qq % a.G : 0);
        s_l[tid] = ok ? lse[((int64_t)b * a.n_q + i) * a.Hq + h] : INFINITY;
        s_tok[tid] = ok ? i : INT_MIN;
    }
    __syncthreads();
    const int l0 = a.local_offsets[b];
    int n_loc = a.local_offsets[b + 1] - l0;
    if (n_loc < 0) n_loc = 0;
    // the last token of the tile: with the causal mask no later new token gets anything from it
    const int last_q = (qt * kTileQ + kTileQ - 1 < n_queries ? qt * kTileQ + kTileQ - 1 : n_queries - 1) / a.G;
    const T *lk = static_cast<const T *>(a.k_local);
    float *dst = colpart + (((int64_t)b * a.Hkv + g) * a.n_qtiles + qt) * a.n_q;
    for (int j = tid; j < a.n_q; j += kThreads) {
        const int r = n_loc - a.n_q + j; // local row of new token j
        float acc = 0.f;
        if (r >= 0 && !(a.causal && j > last_q)) {
            const T *kp = lk + ((int64_t)(l0 + r) * a.Hkv + g) * D;
            float sc[kTileQ];
#pragma unroll
            for (int n = 0; n < kTileQ; ++n) sc[n] = 0.f;
#pragma unroll 4
            for (int d0 = 0; d0 < D; d0 += E) {
                float kx[E];
                Row16<T>::expand(load16(kp + d0), kx);
#pragma unroll
                for (int n = 0; n < kTileQ; ++n)
#pragma unroll
                    for (int e = 0; e < E; ++e) sc[n] = fmaf(s_q[n][d0 + e], kx[e], sc[n]);
            }
#pragma unroll
            for (int n = 0; n < kTileQ; ++n) { // token i sees new token j iff j <= i (or always, without the mask)
                const bool sees = a.causal ? s_tok[n] >= j : s_tok[n] >= 0;
                acc += sees ? __builtin_amdgcn_exp2f(sc[n] - s_l[n]) : 0.f;
            }
        }
        dst[j] = acc;
    }
}

// signal[b][j] = (sum over KV heads and query tiles of colpart) / (Hq * n_q), in a fixed order: 32 columns
// per workgroup, the terms of a column split into 8 contiguous runs (one per group of 32 threads, 8 loads
// in flight), the runs joined in order.
constexpr int kSigCols = 32, kSigRuns = kThreads / kSigCols;
__global__ __launch_bounds__(kThreads) void prefill_signal_kernel(const float *__restrict__ colpart, int n_terms, int n_q,
                                                                  float inv, float *__restrict__ signal) {
    __shared__ float s_run[kSigRuns][kSigCols];
    const int b = blockIdx.y, col = threadIdx.x % kSigCols, run = threadIdx.x / kSigCols;
    const int j = blockIdx.x * kSigCols + col;
    const int per = (n_terms + kSigRuns - 1) / kSigRuns;
    const int t0 = run * per, t1 = t0 + per < n_terms ? t0 + per : n_terms;
    float s = 0.f;
    if (j < n_q) {
        const float *p = colpart + (int64_t)b * n_terms * n_q + j;
        for (int t = t0; t < t1; t += 8) {
            float v[8];
#pragma unroll
            for (int u = 0; u < 8; ++u) v[u] = p[(int64_t)(t + u < t1 ? t + u : t1 - 1) * n_q];
#pragma unroll
            for (int u = 0; u < 8; ++u) s += t + u < t1 ? v[u] : 0.f;
        }
    }
    s_run[run][col] = s;
    __syncthreads();
    if (run == 0 && j < n_q) {
        float tot = s_run[0][col];
#pragma unroll
        for (int r = 1; r < kSigRuns; ++r) tot += s_run[r][col];
        signal[(int64_t)b * n_q + j] = tot * inv;
    }
}

// ------------------------------------------------------------------------------------------
// The prefill on the matrix cores (bf16 rows of 128 features): both products of the attention are
// dense contractions here, 64 queries -- (token, head of the KV group) pairs -- against every row.
// One workgroup of four waves per (64 queries, KV head, question); rows in steps of 32, staged
// through LDS (double-buffered, the next step's rows are in flight in registers meanwhile):
//   scores   wave w owns queries 16w..16w+15: S^T = K Q^T with v_mfma_f32_16x16x32_bf16, the keys as
//            the A operand from LDS (a lane: one key row, 8 features), the queries as the B operand in
//            registers.  A lane then holds ONE query (lane % 16) and eight rows of the step
//            (16 kb + 4 * (lane / 16) + r), so the softmax statistics of a query are mostly in-lane
//            work, joined over the four lanes that share the query by two register swaps.
//            Running maximum and normaliser stay in that wave's registers; the weights go to LDS as
//            bf16 (four of a query at a time), the factor that rescales what was summed so far as float.
//   values   wave w owns output features 32w..32w+31 of all 64 queries: O += P V with the weights as
//            the A operand (a lane: one query, 8 rows) and the values as the B operand (a lane: one
//            feature, 8 rows, fetched from LDS as eight 2-byte reads).
// Rows of padded strides 272 B (keys, values) and 80 B (weights) keep the 16-byte operand reads
// free of bank conflicts.
// Second loop, Eq. 1: with maximum and normaliser final, the scores against the NEW tokens' keys are
// formed once more and their softmax weights added over the workgroup's queries: one row of
// colpart [B][Hkv][query tile][n_q] per workgroup, summed later in a fixed order.
// ------------------------------------------------------------------------------------------
constexpr int kFK = 32, kFD = 128;
constexpr float kHidden = -1e30f, kFloor = -1e20f; // score of a row a query may not see; least running maximum
constexpr int kRowStride = kFD * 2 + 16; // bytes of a staged key / value row
constexpr int kPStride = kFK * 2 + 16;   // bytes of a row of weights

// QB: blocks of 16 queries per wave (64 * QB queries per workgroup).  With two blocks a key or value
// operand fetched from LDS serves twice the matrix instructions; with one there are twice the
// workgroups, which is what a short prefill needs.
// MODE 0: all of it in one launch.  A short prefill has too few tiles to fill the chip, so its rows are
// split over n_split workgroups per tile -- MODE 1: the split's (maximum, normaliser, unnormalised output)
// go to the records attend_combine_kernel merges (aux = records), no second loop -- and the second loop
// runs as a launch of its own once the merged log-sum-exps exist -- MODE 2 (aux = log-sum-exps), its
// steps split over the same number of workgroups.
template <int QB, int MODE>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(QB == 1 ? 3 : 2, QB == 1 ? 3 : 2))) void prefill_flash_kernel(
    AttendArgs a, uint16_t *__restrict__ out, float *__restrict__ colpart, int n_tiles, float *__restrict__ aux, int n_split) {
    using T = uint16_t;
    constexpr int kFQ = 64 * QB, NQB = 4 * QB; // queries, blocks of 16 queries per workgroup
    __shared__ __align__(16) unsigned char s_k[2][kFK * kRowStride];
    __shared__ __align__(16) unsigned char s_v[2][kFK * kRowStride];
    __shared__ __align__(16) unsigned char s_p[kFQ * kPStride];
    __shared__ __align__(16) int s_ft[2][kFK];
    __shared__ float s_corr[kFQ];
    __shared__ int s_chg[NQB]; // per block of 16 queries: did a running maximum move in this step
    __shared__ float s_fin[2][kFQ];
    __shared__ float s_col[4][kFK];
    __shared__ int s_frame[kMaxGatherK]; // the question's frames; -1: names no frame of the cache
    __shared__ int64_t s_toff[2][kFK];   // where the rows of the next two steps live
    __shared__ int s_tft[2][kFK];
    const int qt = MODE == 0 ? blockIdx.x : blockIdx.x / n_split, sp = MODE == 0 ? 0 : blockIdx.x % n_split;
    const int g = blockIdx.y, b = blockIdx.z;
    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63, lr = lane & 15, lg = lane >> 4;
    const int n_queries = a.n_q * a.G;
    const T *q = static_cast<const T *>(a.q);
    for (int i = tid; i < a.k_frame; i += 256) {
        const int f = a.frame_idx[(int64_t)b * a.k_frame + i];
        s_frame[i] = (f >= 0 && f < a.n_frames) ? f : -1;
    }
    __syncthreads();

    // the wave's 16 queries as the A operand; token of the four queries this lane holds scores for
    // the wave's blocks are QB * wave + i; block n holds queries 16 n .. 16 n + 15 of the tile
    bf16x8 qa[QB][kFD / 32];
    int tokq[QB]; // token of the query this lane holds scores for (nothing is visible to a query that does not exist)
    float lse_in[QB];
#pragma unroll
    for (int i = 0; i < QB; ++i) {
        const int qq = qt * kFQ + 16 * (QB * wave + i) + lr;
        const bool ok = qq < n_queries;
        const int ti = ok ? qq / a.G : 0, h = g * a.G + (ok ? qq % a.G : 0);
        const T *qp = q + (((int64_t)b * a.n_q + ti) * a.Hq + h) * kFD + 8 * lg;
#pragma unroll
        for (int kk = 0; kk < kFD / 32; ++kk) {
            raw16 u = load16(qp + 32 * kk);
            if (!ok) u = raw16{0u, 0u, 0u, 0u};
            qa[i][kk] = __builtin_bit_cast(bf16x8, u);
        }
        tokq[i] = ok ? ti : INT_MIN;
        if constexpr (MODE == 2) lse_in[i] = ok ? aux[((int64_t)b * a.n_q + ti) * a.Hq + h] : INFINITY;
    }

    const int n_ret = a.k_frame * a.kappa;
    const int l0 = a.local_offsets[b];
    int n_loc = a.local_offsets[b + 1] - l0;
    if (n_loc < 0) n_loc = 0;
    const int total = n_ret + n_loc;
    const T *sk = static_cast<const T *>(a.store_k) + (int64_t)g * a.store_cap * kFD;
    const T *sv = static_cast<const T *>(a.store_v) + (int64_t)g * a.store_cap * kFD;
    const T *lk = static_cast<const T *>(a.k_local), *lv = static_cast<const T *>(a.v_local);

    // Row r of [retrieved rows, local rows]: where it lives and the first token that sees it, worked out
    // by one thread per row two steps ahead and handed to the staging threads through a small table.
    // Entry: element offset in the store slab (>= 0) or ~offset in the local rows (< 0).  A row that
    // lives nowhere (or below r_min) reads the slab's first row and is seen by nobody.
    auto tabulate = [&](int set, int r, int r_min) { // threads tid < kFK, r = first row of the step + tid
        int64_t off = 0;
        int ft = INT_MAX;
        if (r >= r_min && r < n_ret) {
            const int slot = r / a.kappa;
            const int f = s_frame[slot];
            if (f >= 0) {
                off = ((int64_t)f * a.kappa + (r - slot * a.kappa)) * kFD;
                ft = 0;
            }
        } else if (r >= r_min && r < total) {
            const int j = r - n_ret;
            off = ~(((int64_t)(l0 + j) * a.Hkv + g) * kFD);
            ft = a.causal ? j - (n_loc - a.n_q) : 0;
        }
        s_toff[set][tid] = off;
        s_tft[set][tid] = ft;
    };
    // staging: thread -> rows tid / 16 and tid / 16 + 16 of the step, 16-byte piece tid % 16
    const int st_row = tid >> 4, st_piece = tid & 15;
    // the next step's rows are in flight in registers while a step is computed (a deeper queue of
    // loads cost occupancy and gained nothing)
    raw16 pk[2], pv[2];
    int pft[2];
    auto fetch = [&](int set, bool with_v) {
#pragma unroll
        for (int u = 0; u < 2; ++u) {
            const int64_t e = s_toff[set][st_row + 16 * u];
            pft[u] = s_tft[set][st_row + 16 * u];
            const bool local = e < 0;
            const int64_t off = (local ? ~e : e) + 8 * st_piece;
            pk[u] = load16((local ? lk : sk) + off);
            if (with_v) pv[u] = load16((local ? lv : sv) + off);
        }
    };
    auto put = [&](int buf, bool with_v) {
#pragma unroll
        for (int u = 0; u < 2; ++u) {
            const int off = (st_row + 16 * u) * kRowStride + 16 * st_piece;
            *reinterpret_cast<raw16 *>(s_k[buf] + off) = pk[u];
            if (with_v) *reinterpret_cast<raw16 *>(s_v[buf] + off) = pv[u];
            if (st_piece == 0) s_ft[buf][st_row + 16 * u] = pft[u];
        }
    };
    // scores of the wave's queries against the step's 32 rows: sc[i][kb][r] for row 16 kb + 4 lg + r, query lr of block i
    auto scores = [&](int buf, f32x4 (&sc)[QB][2]) {
#pragma unroll
        for (int kb = 0; kb < 2; ++kb) {
#pragma unroll
            for (int i = 0; i < QB; ++i) sc[i][kb] = f32x4{0.f, 0.f, 0.f, 0.f};
            const unsigned char *kp = s_k[buf] + (16 * kb + lr) * kRowStride + 16 * lg;
#pragma unroll
            for (int kk = 0; kk < kFD / 32; ++kk) {
                const bf16x8 bk = __builtin_bit_cast(bf16x8, *reinterpret_cast<const raw16 *>(kp + 64 * kk));
#pragma unroll
                for (int i = 0; i < QB; ++i) sc[i][kb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(bk, qa[i][kk], sc[i][kb], 0, 0, 0);
            }
        }
    };

    float m_run[QB], l_run[QB]; // of query lr of the wave's blocks
#pragma unroll
    for (int i = 0; i < QB; ++i) {
        m_run[i] = kFloor;
        l_run[i] = 0.f;
    }
    f32x4 o[NQB][2];
#pragma unroll
    for (int qb = 0; qb < NQB; ++qb)
#pragma unroll
        for (int db = 0; db < 2; ++db) o[qb][db] = f32x4{0.f, 0.f, 0.f, 0.f};

    // with the causal mask the rows after the workgroup's last token are seen by none of its queries
    const int last_q = (qt * kFQ + kFQ - 1 < n_queries ? qt * kFQ + kFQ - 1 : n_queries - 1) / a.G;
    int n_seen = total;
    if (a.causal) {
        // local rows up to the tile's last token; the retrieved rows are seen by every token, also by
        // tokens that have no local row of their own (fewer local rows than new tokens)
        int ns = n_ret + n_loc - a.n_q + last_q + 1;
        if (ns < n_ret) ns = n_ret;
        if (ns < total) n_seen = ns;
    }
    const int n_steps_all = n_seen > 0 ? (n_seen + kFK - 1) / kFK : 0;
    // this workgroup's steps: all of them, or its share of them
    const int per_split = MODE == 1 ? (n_steps_all + n_split - 1) / n_split : n_steps_all;
    const int t_lo = MODE == 1 ? sp * per_split : 0;
    const int n_steps = MODE == 2 ? 0 : (t_lo + per_split < n_steps_all ? t_lo + per_split : n_steps_all);
    if (MODE != 2 && tid < kFK) {
        tabulate(0, t_lo * kFK + tid, 0);
        tabulate(1, (t_lo + 1) * kFK + tid, 0);
    }
    __syncthreads();
    if (t_lo < n_steps) fetch(0, true);
    for (int t = t_lo; t < n_steps; ++t) {
        const int buf = (t - t_lo) & 1;
        put(buf, true);
        __syncthreads(); // step t is staged; every wave is done with step t-1
        if (t + 1 < n_steps) fetch(buf ^ 1, true);
        if (tid < kFK && t + 2 < n_steps) tabulate(buf, (t + 2) * kFK + tid, 0);
        f32x4 sc[QB][2];
        scores(buf, sc);
        // Scores stay unscaled (the factor to log2 units sits in the exponent's multiply-add); a row a query
        // may not see scores kHidden, and running maxima never drop below kFloor: exp2 of the difference is an
        // exact zero for hidden rows, no select needed, and a query that has seen nothing yet sums zeros.
        const i32x4 f0 = *reinterpret_cast<const i32x4 *>(&s_ft[buf][4 * lg]);
        const i32x4 f1 = *reinterpret_cast<const i32x4 *>(&s_ft[buf][16 + 4 * lg]);
#pragma unroll
        for (int i = 0; i < QB; ++i) {
            float sv[8];
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                sv[r] = tokq[i] >= f0[r] ? sc[i][0][r] : kHidden;
                sv[4 + r] = tokq[i] >= f1[r] ? sc[i][1][r] : kHidden;
            }
            const float mx = fmaxf(fmaxf(fmaxf(sv[0], sv[1]), fmaxf(sv[2], sv[3])), fmaxf(fmaxf(sv[4], sv[5]), fmaxf(sv[6], sv[7])));
            const float m_new = fmaxf(m_run[i], xrow_max(mx) * a.scale_log2e);
            const float corr = __builtin_amdgcn_exp2f(m_run[i] - m_new);
            float pw[8];
#pragma unroll
            for (int e = 0; e < 8; ++e) pw[e] = __builtin_amdgcn_exp2f(fmaf(sv[e], a.scale_log2e, -m_new));
            l_run[i] = l_run[i] * corr + xrow_sum(((pw[0] + pw[1]) + (pw[2] + pw[3])) + ((pw[4] + pw[5]) + (pw[6] + pw[7])));
            const bool moved = m_new != m_run[i];
            m_run[i] = m_new;
            const int qrow = 16 * (QB * wave + i) + lr;
            if (lg == 0) s_corr[qrow] = corr;
            // rows 4 lg .. 4 lg + 3 and 16 + 4 lg .. of the query's weights, rounded to bf16 two at a time
            u32x2 w0, w1;
            w0[0] = __builtin_bit_cast(uint32_t, __builtin_convertvector(f32x2{pw[0], pw[1]}, bf16x2));
            w0[1] = __builtin_bit_cast(uint32_t, __builtin_convertvector(f32x2{pw[2], pw[3]}, bf16x2));
            w1[0] = __builtin_bit_cast(uint32_t, __builtin_convertvector(f32x2{pw[4], pw[5]}, bf16x2));
            w1[1] = __builtin_bit_cast(uint32_t, __builtin_convertvector(f32x2{pw[6], pw[7]}, bf16x2));
            *reinterpret_cast<u32x2 *>(s_p + qrow * kPStride + 8 * lg) = w0;
            *reinterpret_cast<u32x2 *>(s_p + qrow * kPStride + 32 + 8 * lg) = w1;
            // most steps leave the running maxima of a block's 16 queries where they were: nothing to rescale then
            const bool any_moved = __builtin_amdgcn_ballot_w64(moved) != 0;
            if (lane == 0) s_chg[QB * wave + i] = any_moved;
        }
        __syncthreads(); // weights and factors of step t are in LDS
        // The B operand wants 8 rows of ONE feature per lane while the staged values are row-major: the LDS
        // transpose read hands lane n of a 16-lane block column n of a 4 x 16 tile whose row t is named by
        // lanes 4t .. 4t+3 of the block, 4 features each -- two such reads per operand.
        bf16x8 bv[2];
#pragma unroll
        for (int db = 0; db < 2; ++db) {
            const unsigned char *vp = s_v[buf] + (8 * lg + (lr >> 2)) * kRowStride + 2 * (32 * wave + 16 * db + 4 * (lr & 3));
            const i16x4 lo = lds_read_tr16(vp), hi = lds_read_tr16(vp + 4 * kRowStride);
            bv[db] = __builtin_bit_cast(bf16x8, i16x8{lo[0], lo[1], lo[2], lo[3], hi[0], hi[1], hi[2], hi[3]});
        }
#pragma unroll
        for (int qb = 0; qb < NQB; ++qb) {
            const bf16x8 ap = __builtin_bit_cast(bf16x8, *reinterpret_cast<const raw16 *>(s_p + (16 * qb + lr) * kPStride + 16 * lg));
            if (s_chg[qb]) {
                float corr[4];
#pragma unroll
                for (int r = 0; r < 4; ++r) corr[r] = s_corr[16 * qb + 4 * lg + r];
#pragma unroll
                for (int db = 0; db < 2; ++db)
#pragma unroll
                    for (int r = 0; r < 4; ++r) o[qb][db][r] *= corr[r];
            }
#pragma unroll
            for (int db = 0; db < 2; ++db) o[qb][db] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(ap, bv[db], o[qb][db], 0, 0, 0);
        }
    }
    float lse[QB]; // of query lr of the wave's blocks
    if constexpr (MODE != 2) {
        // ---- final statistics to LDS, output ----
        __syncthreads();
        if (lg == 0) {
#pragma unroll
            for (int i = 0; i < QB; ++i) {
                s_fin[0][16 * (QB * wave + i) + lr] = m_run[i];
                s_fin[1][16 * (QB * wave + i) + lr] = l_run[i];
            }
        }
        __syncthreads();
        if constexpr (MODE == 1) { // the split's record of every query: [0] maximum, [1] normaliser, [2..] unnormalised output
            if (tid < kFQ && qt * kFQ + tid < n_queries) {
                const int qq = qt * kFQ + tid;
                const int i = qq / a.G, h = g * a.G + qq % a.G;
                float *rec = aux + ((((int64_t)b * a.n_q + i) * a.Hq + h) * n_split + sp) * (kFD + 2);
                rec[0] = s_fin[0][tid];
                rec[1] = s_fin[1][tid];
            }
        }
#pragma unroll
        for (int qb = 0; qb < NQB; ++qb) {
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                const int n = 16 * qb + 4 * lg + r;
                const int qq = qt * kFQ + n;
                if (qq >= n_queries) continue;
                const int i = qq / a.G, h = g * a.G + qq % a.G;
                if constexpr (MODE == 1) {
                    float *rec = aux + ((((int64_t)b * a.n_q + i) * a.Hq + h) * n_split + sp) * (kFD + 2) + 2 + 32 * wave + lr;
                    rec[0] = o[qb][0][r];
                    rec[16] = o[qb][1][r];
                } else {
                    const float l = s_fin[1][n];
                    const float inv = l > 0.f ? 1.0f / l : 0.f;
                    uint16_t *op = out + (((int64_t)b * a.n_q + i) * a.Hq + h) * kFD + 32 * wave + lr;
                    op[0] = bf16_round(o[qb][0][r] * inv);
                    op[16] = bf16_round(o[qb][1][r] * inv);
                }
            }
        }
        if (MODE == 1 || !colpart) return;
#pragma unroll
        for (int i = 0; i < QB; ++i) lse[i] = l_run[i] > 0.f ? m_run[i] + __builtin_amdgcn_logf(l_run[i]) : INFINITY;
    } else {
#pragma unroll
        for (int i = 0; i < QB; ++i) lse[i] = lse_in[i];
    }

    // ---- Eq. 1: weights on the new tokens, added over the workgroup's queries ----
    float *dst = colpart + (((int64_t)b * a.Hkv + g) * n_tiles + qt) * a.n_q;
    // new token j is local row n_loc - n_q + j, i.e. row r_new0 + j of the row sequence (it may not exist)
    const int r_new0 = n_ret + n_loc - a.n_q;
    const int j_end = a.causal ? (last_q + 1 < a.n_q ? last_q + 1 : a.n_q) : a.n_q; // later tokens get nothing from here
    if (sp == 0)
        for (int j = j_end + tid; j < a.n_q; j += 256) dst[j] = 0.f;
    const int n_steps2_all = (j_end + kFK - 1) / kFK;
    const int per2 = MODE == 2 ? (n_steps2_all + n_split - 1) / n_split : n_steps2_all;
    const int t2_lo = MODE == 2 ? sp * per2 : 0;
    const int n_steps2 = t2_lo + per2 < n_steps2_all ? t2_lo + per2 : n_steps2_all;
    __syncthreads(); // the staging buffers and the row table are free again
    // rows below n_ret would be retrieved rows: a new token without a row of its own is seen by nobody
    if (tid < kFK) {
        tabulate(0, r_new0 + t2_lo * kFK + tid, n_ret);
        tabulate(1, r_new0 + (t2_lo + 1) * kFK + tid, n_ret);
    }
    __syncthreads();
    if (t2_lo < n_steps2) fetch(0, false);
    for (int t = t2_lo; t < n_steps2; ++t) {
        const int buf = (t - t2_lo) & 1;
        put(buf, false);
        __syncthreads();
        if (t + 1 < n_steps2) fetch(buf ^ 1, false);
        if (tid < kFK && t + 2 < n_steps2) tabulate(buf, r_new0 + (t + 2) * kFK + tid, n_ret);
        f32x4 sc[QB][2];
        scores(buf, sc);
        {   // the lane's weights on rows 16 kb + 4 lg + r, added over the queries of the wave (its blocks, the lanes of a row)
            const i32x4 f0 = *reinterpret_cast<const i32x4 *>(&s_ft[buf][4 * lg]);
            const i32x4 f1 = *reinterpret_cast<const i32x4 *>(&s_ft[buf][16 + 4 * lg]);
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                float c0 = 0.f, c1 = 0.f;
#pragma unroll
                for (int i = 0; i < QB; ++i) {
                    c0 += tokq[i] >= f0[r] ? __builtin_amdgcn_exp2f(fmaf(sc[i][0][r], a.scale_log2e, -lse[i])) : 0.f;
                    c1 += tokq[i] >= f1[r] ? __builtin_amdgcn_exp2f(fmaf(sc[i][1][r], a.scale_log2e, -lse[i])) : 0.f;
                }
                c0 = row16_sum(c0);
                c1 = row16_sum(c1);
                if (lr == 0) {
                    s_col[wave][4 * lg + r] = c0;
                    s_col[wave][16 + 4 * lg + r] = c1;
                }
            }
        }
        __syncthreads();
        if (tid < kFK && t * kFK + tid < j_end)
            dst[t * kFK + tid] = (s_col[0][tid] + s_col[1][tid]) + (s_col[2][tid] + s_col[3][tid]);
    }
}

struct PrefillOut { // all null for the plain attention call
    float *lse, *colpart, *signal;
};

template <typename T, int D>
hipError_t launch_typed(const AttendArgs &a, int B, void *out, const PrefillOut &po, hipStream_t st) {
    hipLaunchKernelGGL((attend_partial_kernel<T, D>), dim3(a.n_split, a.Hkv * a.n_qtiles, B), dim3(kThreads), 0, st, a);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL((attend_combine_kernel<T, D>), dim3((unsigned)(B * a.n_q * a.Hq)), dim3(D < 64 ? 64 : D), 0, st,
                       a.part, a.n_split, static_cast<T *>(out), po.lse);
    if ((e = hipGetLastError()) != hipSuccess || !po.signal) return e;
    hipLaunchKernelGGL((prefill_colsum_kernel<T, D>), dim3(a.n_qtiles, a.Hkv, B), dim3(kThreads), 0, st, a, po.lse,
                       po.colpart);
    if ((e = hipGetLastError()) != hipSuccess) return e;
    hipLaunchKernelGGL(prefill_signal_kernel, dim3((a.n_q + kSigCols - 1) / kSigCols, B), dim3(kThreads), 0, st, po.colpart,
                       a.Hkv * a.n_qtiles, a.n_q, 1.0f / ((float)a.Hq * (float)a.n_q), po.signal);
    return hipGetLastError();
}

template <typename T>
hipError_t launch_by_dim(const AttendArgs &a, int D, int B, void *out, const PrefillOut &po, hipStream_t st) {
    switch (D) {
    case 16: return launch_typed<T, 16>(a, B, out, po, st);
    case 32: return launch_typed<T, 32>(a, B, out, po, st);
    case 64: return launch_typed<T, 64>(a, B, out, po, st);
    case 128: return launch_typed<T, 128>(a, B, out, po, st);
    default: return hipErrorInvalidValue;
    }
}

int split_count(int B, int Hkv, int n_qtiles, int k_frame, int *frames_per_split) {
    // about three workgroups per compute unit (what fits at once): a workgroup walks its rows in
    // dependent batches of loads, so shorter lists finish sooner; at most kAttendMaxSplit splits,
    // at least one frame each
    // (64 questions of the 1-hour shape: 2 or 3 per compute unit take the same 28 us, 1 takes 37, 4 / 6 / 8 take
    // 34 / 38 / 43 -- every workgroup pays its chain of dependent steps once more)
    int64_t n_split = (3 * 256 + (int64_t)B * Hkv * n_qtiles - 1) / ((int64_t)B * Hkv * n_qtiles);
    if (n_split > kAttendMaxSplit) n_split = kAttendMaxSplit;
    if (n_split > k_frame) n_split = k_frame;
    if (n_split < 1) n_split = 1;
    *frames_per_split = k_frame > 0 ? (int)((k_frame + n_split - 1) / n_split) : 0;
    if (k_frame > 0) n_split = (k_frame + *frames_per_split - 1) / *frames_per_split;
    return (int)n_split;
}

} // namespace

static bool flash_shape(const Ctx &c) { return c.cfg.dtype == MUKV_BF16 && c.cfg.head_dim == kFD; }
static bool flash_wide(const Ctx &c, int n_q, int B) { // 128-query tiles once they still fill the chip about twice over
    return (((int64_t)n_q * c.group + 127) / 128) * c.cfg.n_kv_heads * B >= 2 * 256;
}
// Workgroups that share the rows of one 64-query tile of the matrix-core prefill: 1 unless the tiles alone
// leave most of the chip idle (about three workgroups per compute unit are wanted, at least four steps each).
// (Sharing the rows of a tile between workgroups also when the tiles fill the chip -- to even out the causal
// triangle -- was measured on the 1568-token chunk: 2 / 3 / 4 ways took 212 / 210 / 221 us against 207.)
static int flash_split(const Ctx &c, int n_q, int B, int k_frame) {
    if (flash_wide(c, n_q, B)) return 1;
    const int64_t wgs = (((int64_t)n_q * c.group + 63) / 64) * c.cfg.n_kv_heads * B;
    if (wgs >= 384) return 1;
    const int64_t steps = ((int64_t)(k_frame > 0 ? k_frame : 0) * c.kappa + n_q + kFK - 1) / kFK;
    int64_t n = (768 + wgs - 1) / wgs;
    if (n > kAttendMaxSplit) n = kAttendMaxSplit;
    if (n > steps / 4) n = steps / 4;
    return n < 1 ? 1 : (int)n;
}

// Workspace of the prefill call, in floats: the splits' records, the log-sum-exps, the tiles' column sums.
static void prefill_layout(const Ctx &c, int n_q, int B, int k_frame, int64_t *part, int64_t *lse, int64_t *colpart) {
    const int n_qtiles = (n_q * c.group + kTileQ - 1) / kTileQ;
    int n_split;
    if (flash_shape(c)) {
        n_split = flash_split(c, n_q, B, k_frame);
        if (n_split == 1) n_split = 0; // one launch does it all: no records
    } else {
        int fps;
        n_split = split_count(B, c.cfg.n_kv_heads, n_qtiles, k_frame > 0 ? k_frame : 0, &fps);
    }
    *part = (int64_t)B * n_q * c.cfg.n_q_heads * n_split * (c.cfg.head_dim + 2);
    *lse = (int64_t)B * n_q * c.cfg.n_q_heads;
    // column sums per (KV head, query tile): the matrix-core prefill has tiles of 64 (or 128) queries
    const int64_t n_coltiles = flash_shape(c) ? ((int64_t)n_q * c.group + 63) / 64 : n_qtiles;
    *colpart = (int64_t)B * c.cfg.n_kv_heads * n_coltiles * n_q;
}

int64_t prefill_workspace_bytes(const Ctx &c, int n_q, int B, int k_frame) {
    int64_t p, l, cp;
    prefill_layout(c, n_q, B, k_frame, &p, &l, &cp);
    return (p + l + cp) * (int64_t)sizeof(float);
}

// workspace == null: the plain attention call, records in the context's scratch, no signal.
hipError_t launch_attend(const Ctx &c, int layer, const void *q, int n_q, const int32_t *frame_idx, int k_frame,
                         const void *k_local, const void *v_local, const int32_t *local_offsets, int B, int causal,
                         void *out, float *signal, float *workspace, hipStream_t st) {
    AttendArgs a;
    a.q = q;
    a.frame_idx = k_frame > 0 ? frame_idx : nullptr;
    a.k_local = k_local;
    a.v_local = v_local;
    a.local_offsets = local_offsets;
    const int64_t slab = (int64_t)c.store_cap * c.cfg.head_dim * c.esz; // bytes of one (layer, head) slab
    a.store_k = static_cast<const unsigned char *>(c.store_k) + (int64_t)layer * c.cfg.n_kv_heads * slab;
    a.store_v = static_cast<const unsigned char *>(c.store_v) + (int64_t)layer * c.cfg.n_kv_heads * slab;
    a.part = c.attend_part;
    a.store_cap = c.store_cap;
    a.n_q = n_q;
    a.Hq = c.cfg.n_q_heads;
    a.Hkv = c.cfg.n_kv_heads;
    a.G = c.group;
    a.k_frame = k_frame > 0 ? k_frame : 0;
    a.kappa = c.kappa;
    a.n_frames = (int)c.n_frames;
    a.n_qtiles = (n_q * c.group + kTileQ - 1) / kTileQ;
    a.causal = causal;
    a.scale_log2e = 1.4426950408889634f / sqrtf((float)c.cfg.head_dim);
    a.n_split = split_count(B, a.Hkv, a.n_qtiles, a.k_frame, &a.frames_per_split);
    PrefillOut po{nullptr, nullptr, nullptr};
    if (workspace) {
        int64_t p, l, cp;
        prefill_layout(c, n_q, B, k_frame, &p, &l, &cp);
        a.part = workspace;
        po.lse = workspace + p;
        po.colpart = workspace + p + l;
        po.signal = signal;
    }
    if (workspace && flash_shape(c)) { // the prefill on the matrix cores
        const int64_t n_queries = (int64_t)n_q * c.group;
        const bool wide = flash_wide(c, n_q, B);
        const int n_fs = flash_split(c, n_q, B, k_frame);
        const int n_tiles = (int)((n_queries + (wide ? 127 : 63)) / (wide ? 128 : 64));
        uint16_t *o16 = static_cast<uint16_t *>(out);
        hipError_t e;
        if (wide) {
            hipLaunchKernelGGL((prefill_flash_kernel<2, 0>), dim3(n_tiles, a.Hkv, B), dim3(256), 0, st, a, o16, po.colpart,
                               n_tiles, nullptr, 1);
        } else if (n_fs == 1) {
            hipLaunchKernelGGL((prefill_flash_kernel<1, 0>), dim3(n_tiles, a.Hkv, B), dim3(256), 0, st, a, o16, po.colpart,
                               n_tiles, nullptr, 1);
        } else { // rows shared by n_fs workgroups per tile, merged, then the column sums from the merged log-sum-exps
            hipLaunchKernelGGL((prefill_flash_kernel<1, 1>), dim3(n_tiles * n_fs, a.Hkv, B), dim3(256), 0, st, a, o16,
                               nullptr, n_tiles, workspace, n_fs);
            if ((e = hipGetLastError()) != hipSuccess) return e;
            hipLaunchKernelGGL((attend_combine_kernel<uint16_t, kFD>), dim3((unsigned)(B * n_q * a.Hq)), dim3(kFD), 0, st,
                               workspace, n_fs, o16, po.lse);
            if ((e = hipGetLastError()) != hipSuccess) return e;
            hipLaunchKernelGGL((prefill_flash_kernel<1, 2>), dim3(n_tiles * n_fs, a.Hkv, B), dim3(256), 0, st, a, o16,
                               po.colpart, n_tiles, po.lse, n_fs);
        }
        if ((e = hipGetLastError()) != hipSuccess) return e;
        hipLaunchKernelGGL(prefill_signal_kernel, dim3((n_q + kSigCols - 1) / kSigCols, B), dim3(kThreads), 0, st, po.colpart,
                           a.Hkv * n_tiles, n_q, 1.0f / ((float)a.Hq * (float)n_q), po.signal);
        return hipGetLastError();
    }
    return c.cfg.dtype == MUKV_BF16 ? launch_by_dim<uint16_t>(a, c.cfg.head_dim, B, out, po, st)
                                    : launch_by_dim<float>(a, c.cfg.head_dim, B, out, po, st);
}

} // namespace mukv
