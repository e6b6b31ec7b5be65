// Online half of MuKV (Sec. 3.4-3.5 of the paper): question pooling, cosine scoring of the
// block keys, two-stage semi-hierarchical selection, and the gather of the selected KV.
//
// Kernel chain of launch_retrieve:
//   pool_question   Eq. 6   mean query per question, summed over each KV head's query group
//   score_blocks    Eq. 7   cosine of every visible frame / segment key with every question
//   select_rerank   stage-1 top-2k, global query, Eq. 8, final top-k   (one workgroup / question)
// launch_gather: gather_kv  copies the kept rows of the selected frames into the decode context.
//
// All scores are evaluated in fp64 from the float32 key tables, so that the selections agree
// with an fp64 evaluation of the same definitions except for ties closer than ~1e-15.
#include "mukv_internal.h"

namespace mukv {

typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef unsigned int cp_u32x4 __attribute__((ext_vector_type(4)));
constexpr int kSelThreads = 512;

// ------------------------------------------------------------------------------------------
// Eq. 6.  grid (B, Hkv, D / dz).  Each workgroup averages the question's tokens for a slice of dz
// features of the G query heads of one KV head, then sums those heads: with keys repeated G times
// over their group (grouped query attention), q . expand(r) = sum_g (sum_{h in g} q_h) . r_g.
// Also the slice's share of |q|^2.  dz is chosen so that G * dz elements are one pass of the
// workgroup's 256 element lanes: the call is a chain of dependent memory round trips, and the fewer
// a workgroup makes the sooner the scores can start.
// ------------------------------------------------------------------------------------------
template <typename T>
__global__ __launch_bounds__(1024) void pool_question_kernel(const T *__restrict__ q_tokens,
                                                             const int32_t *__restrict__ q_off, int Hq, int Hkv, int D,
                                                             int G, int dz, double *__restrict__ qbar,
                                                             double *__restrict__ qq) {
    // threads: 256 element lanes x 4 token slices; slice t takes tokens t, t+4, ... in batches of
    // 8 independent loads.  Token sums are exact in fp64, so the split does not change the result.
    extern __shared__ __align__(16) unsigned char smem_raw[];
    double *part = reinterpret_cast<double *>(smem_raw); // [4][G*dz]
    __shared__ double red[16];
    const int b = blockIdx.x, g = blockIdx.y, z = blockIdx.z, tid = threadIdx.x;
    const int el = tid & 255, ts = tid >> 8;
    const int t0 = q_off[b], t1 = q_off[b + 1];
    const int nq = t1 - t0;
    const int GD = G * dz, d0 = z * dz;
    const int64_t tstride = (int64_t)Hq * D;
    for (int e = el; e < GD; e += 256) {
        const int hl = e / dz, dd = e - hl * dz;
        const T *p = q_tokens + ((int64_t)t0 * Hq + (int64_t)g * G + hl) * D + d0 + dd;
        double s = 0.0;
        for (int tb = ts; tb < nq; tb += 32) {
            float v[8];
#pragma unroll
            for (int u = 0; u < 8; ++u) {
                const int t = tb + 4 * u < nq ? tb + 4 * u : nq - 1; // clamped: loads stay unconditional
                v[u] = to_float(p[(int64_t)t * tstride]);
            }
#pragma unroll
            for (int u = 0; u < 8; ++u)
                if (tb + 4 * u < nq) s += (double)v[u];
        }
        part[ts * GD + e] = s;
    }
    __syncthreads();
    double sq = 0.0;
    if (ts == 0) {
        for (int e = el; e < GD; e += 256) {
            const double s = ((part[e] + part[GD + e]) + part[2 * GD + e]) + part[3 * GD + e];
            const double m = nq > 0 ? s / (double)nq : 0.0;
            part[e] = m;
            sq += m * m;
        }
    }
    sq = wave_sum(sq);
    if ((tid & 63) == 0) red[tid >> 6] = sq;
    __syncthreads();
    if (tid == 0) qq[((int64_t)b * Hkv + g) * gridDim.z + z] = ((red[0] + red[1]) + red[2]) + red[3];
    for (int dd = tid; dd < dz; dd += 1024) {
        double s = 0.0;
        for (int hl = 0; hl < G; ++hl) s += part[hl * dz + dd];
        qbar[((int64_t)b * Hkv + g) * D + d0 + dd] = s;
    }
}

// ------------------------------------------------------------------------------------------
// Eq. 7.  One wave per block key (frames first, then segments).  The key row stays in
// registers while the wave loops over the questions.  cos(q, expand(r)) =
// (qbar . r) / (|q| * sqrt(G) * |r|); a zero key or zero query scores 0.
// A segment cut by the question's timestamp (only the last visible one can be) gets its key
// from the exact per-frame sums of its visible frames; that key is also left in seg_tail for
// the rerank kernel.
// ------------------------------------------------------------------------------------------
struct ScoreArgs {
    const float *rep_frame, *rep_seg;
    const double *fsum;
    const double *qbar, *qq;
    double *s_frm, *s_seg;
    float *seg_tail;
    int nv, ns, B, C, Hkv, G, F, kappa;
    int n_qq; // partial squared norms of the pooled query per question
    int nf; // keys of the fine level in rep_frame / s_frm: the visible frames, or their super-patches
    int tail_cut; // 1: segment ns-1 must be rebuilt from frames [ (ns-1)*F, nv )
    int64_t ld_frm, ld_seg;
};

__global__ __launch_bounds__(256) void score_blocks_kernel(ScoreArgs a) {
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int r = blockIdx.x * 4 + wave;
    if (r >= a.nf + a.ns) return;
    const bool is_seg = r >= a.nf;
    const int idx = is_seg ? r - a.nf : r;
    const int C = a.C;
    float row[16];
    if (is_seg && a.tail_cut && idx == a.ns - 1) {
        const int f0 = idx * a.F;
        const double den = (double)(a.nv - f0) * (double)a.kappa;
#pragma unroll
        for (int t = 0; t < 16; ++t) {
            const int c = lane + 64 * t;
            row[t] = 0.f;
            if (c < C) {
                double s = 0.0;
                for (int f = f0; f < a.nv; ++f) s += a.fsum[(int64_t)f * C + c];
                row[t] = (float)(s / den);
                a.seg_tail[c] = row[t];
            }
        }
    } else {
        const float *src = (is_seg ? a.rep_seg : a.rep_frame) + (int64_t)idx * C;
#pragma unroll
        for (int t = 0; t < 16; ++t) {
            const int c = lane + 64 * t;
            const float x = src[c < C ? c : C - 1]; // clamped: loads stay unconditional
            row[t] = (c < C) ? x : 0.f;
        }
    }
    double rr = 0.0;
#pragma unroll
    for (int t = 0; t < 16; ++t) rr += (double)row[t] * (double)row[t];
    rr = wave_sum(rr);
    // four questions per round: their pooled queries are loaded together (independent loads),
    // the four dot products reduced side by side, and lanes 0..3 finish one question each
    for (int b0 = 0; b0 < a.B; b0 += 4) {
        double dot[4] = {0.0, 0.0, 0.0, 0.0};
        const double *qb[4];
#pragma unroll
        for (int j = 0; j < 4; ++j) qb[j] = a.qbar + (int64_t)(b0 + j < a.B ? b0 + j : a.B - 1) * C;
#pragma unroll
        for (int t = 0; t < 16; ++t) {
            if (64 * t < C) { // uniform
                const int c = lane + 64 * t;
                const int cc = c < C ? c : C - 1; // row[t] is 0 past C
#pragma unroll
                for (int j = 0; j < 4; ++j)
                    if (b0 + j < a.B) dot[j] += (double)row[t] * qb[j][cc]; // uniform
            }
        }
#pragma unroll
        for (int j = 0; j < 4; ++j) dot[j] = wave_sum(dot[j]);
        const int b = b0 + lane;
        if (lane < 4 && b < a.B) {
            const double d = lane == 0 ? dot[0] : (lane == 1 ? dot[1] : (lane == 2 ? dot[2] : dot[3]));
            double qn = 0.0;
            for (int g = 0; g < a.n_qq; ++g) qn += a.qq[(int64_t)b * a.n_qq + g];
            double sc = 0.0;
            if (rr > 0.0 && qn > 0.0) sc = d / (sqrt(qn) * sqrt((double)a.G * rr));
            if (is_seg)
                a.s_seg[(int64_t)b * a.ld_seg + idx] = sc;
            else
                a.s_frm[(int64_t)b * a.ld_frm + idx] = sc;
        }
    }
}

// Eq. 7 when many questions are asked at once: the scores are a [keys x C] x [C x questions]
// product, done on the fp64 matrix cores.  A wave owns a tile of 16 keys x 16 questions and
// walks the channels 16 at a time: lane l holds channels c0 + 4*(l/16) .. +3 of key l%16 (one
// 16-byte load) and of question l%16 (two 16-byte loads)
// and issues four v_mfma_f64_16x16x4_f64, element e of the lane's four channels being reduction
// index l/16 of the e-th.  Operand / result layout (checked on the device): A[row = l%16][k = l/16],
// B[k = l/16][col = l%16], D register r of lane l = D[row = 4*r + l/16][col = l%16].
typedef double f64x4 __attribute__((ext_vector_type(4)));
typedef double f64x2 __attribute__((ext_vector_type(2)));
// Key of a segment cut by the question's timestamp, from the exact per-frame sums of its visible
// frames (the wave-per-key kernel does this inline; the matrix-core kernel reads the result).
__global__ __launch_bounds__(256) void seg_tail_kernel(ScoreArgs a) {
    const int f0 = (a.ns - 1) * a.F;
    const double den = (double)(a.nv - f0) * (double)a.kappa;
    for (int c = blockIdx.x * 256 + threadIdx.x; c < a.C; c += gridDim.x * 256) {
        double s = 0.0;
        for (int f = f0; f < a.nv; ++f) s += a.fsum[(int64_t)f * a.C + c];
        a.seg_tail[c] = (float)(s / den);
    }
}

// Per-question timestamps: the scoring kernels have scored every ingested block with its full
// key; question b, which sees frames < nv_q[b], may cut one segment.  One workgroup per question
// rebuilds that segment's key from the exact per-frame sums of its visible frames (kept for the
// rerank kernel in seg_tail[b]) and replaces its score.
struct TailArgs {
    const int32_t *nv_q;
    int n_all, F, kappa, C, Hkv, G, n_qq;
    const double *fsum, *qbar, *qq;
    double *s_seg;
    int64_t ld_seg;
    float *seg_tail;
};

__global__ __launch_bounds__(256) void tail_fix_kernel(TailArgs a) {
    __shared__ double red[8];
    const int b = blockIdx.x, tid = threadIdx.x;
    int nvb = a.nv_q[b];
    nvb = (nvb < 0 || nvb > a.n_all) ? a.n_all : nvb;
    const int ns = (nvb + a.F - 1) / a.F;
    const int seg_end = ns * a.F < a.n_all ? ns * a.F : a.n_all;
    if (ns == 0 || nvb >= seg_end) return; // uniform over the workgroup
    const int f0 = (ns - 1) * a.F;
    const double den = (double)(nvb - f0) * (double)a.kappa;
    double dot = 0.0, rr = 0.0;
    for (int c = tid; c < a.C; c += 256) {
        double s = 0.0;
        for (int f = f0; f < nvb; ++f) s += a.fsum[(int64_t)f * a.C + c];
        const float key = (float)(s / den);
        a.seg_tail[(int64_t)b * a.C + c] = key;
        dot += (double)key * a.qbar[(int64_t)b * a.C + c];
        rr += (double)key * (double)key;
    }
    dot = wave_sum(dot);
    rr = wave_sum(rr);
    if ((tid & 63) == 0) {
        red[tid >> 6] = dot;
        red[4 + (tid >> 6)] = rr;
    }
    __syncthreads();
    if (tid == 0) {
        dot = (red[0] + red[1]) + (red[2] + red[3]);
        rr = (red[4] + red[5]) + (red[6] + red[7]);
        double qn = 0.0;
        for (int g = 0; g < a.n_qq; ++g) qn += a.qq[(int64_t)b * a.n_qq + g];
        double sc = 0.0;
        if (rr > 0.0 && qn > 0.0) sc = dot / (sqrt(qn) * sqrt((double)a.G * rr));
        a.s_seg[(int64_t)b * a.ld_seg + ns - 1] = sc;
    }
}

// grid.x: the frame tiles, then the segment tiles (16 keys each)
__global__ __launch_bounds__(256) void score_blocks_mfma_kernel(ScoreArgs a) {
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int lr = lane & 15, kq = lane >> 4;
    const int C = a.C;
    const int n_ft = (a.nf + 15) / 16;
    const bool is_seg = (int)blockIdx.x >= n_ft;
    const int row0 = (is_seg ? (int)blockIdx.x - n_ft : (int)blockIdx.x) * 16;
    const int n_rows = is_seg ? a.ns : a.nf;
    const int rw_in = row0 + lr < n_rows ? row0 + lr : n_rows - 1;
    const float *kp = (is_seg ? ((a.tail_cut && rw_in == a.ns - 1) ? a.seg_tail : a.rep_seg + (int64_t)rw_in * C)
                              : a.rep_frame + (int64_t)rw_in * C) + 4 * kq;
    double *s_out = is_seg ? a.s_seg : a.s_frm;
    const int64_t ld_out = is_seg ? a.ld_seg : a.ld_frm;
    for (int q0 = 16 * wave; q0 < a.B; q0 += 64) {
        const int bq = q0 + lr < a.B ? q0 + lr : a.B - 1;
        const double *qp = a.qbar + (int64_t)bq * C + 4 * kq;
        f64x4 acc = {0.0, 0.0, 0.0, 0.0};
        double rr = 0.0;
        for (int c0 = 0; c0 < C; c0 += 64) { // four steps of 16 channels, their loads issued together
            f32x4 kv[4];
            f64x2 qlo[4], qhi[4];
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const int c = c0 + 16 * u < C ? c0 + 16 * u : C - 16;
                kv[u] = *reinterpret_cast<const f32x4 *>(kp + c);
                qlo[u] = *reinterpret_cast<const f64x2 *>(qp + c);
                qhi[u] = *reinterpret_cast<const f64x2 *>(qp + c + 2);
            }
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                if (c0 + 16 * u < C) { // uniform
                    const double k0 = (double)kv[u][0], k1 = (double)kv[u][1], k2 = (double)kv[u][2], k3 = (double)kv[u][3];
                    rr += (k0 * k0 + k1 * k1) + (k2 * k2 + k3 * k3);
                    acc = __builtin_amdgcn_mfma_f64_16x16x4f64(k0, qlo[u][0], acc, 0, 0, 0);
                    acc = __builtin_amdgcn_mfma_f64_16x16x4f64(k1, qlo[u][1], acc, 0, 0, 0);
                    acc = __builtin_amdgcn_mfma_f64_16x16x4f64(k2, qhi[u][0], acc, 0, 0, 0);
                    acc = __builtin_amdgcn_mfma_f64_16x16x4f64(k3, qhi[u][1], acc, 0, 0, 0);
                }
            }
        }
        // |r|^2 of key lr: add the four lanes that hold its channels
        rr += lane_xor<16>(rr);
        rr += lane_xor<32>(rr);
        double qn = 0.0;
        for (int g = 0; g < a.n_qq; ++g) qn += a.qq[(int64_t)bq * a.n_qq + g];
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            const int rw = 4 * r + kq; // tile row of result register r
            const double rr_row = __shfl(rr, rw);
            double sc = 0.0;
            if (rr_row > 0.0 && qn > 0.0) sc = acc[r] / (sqrt(qn) * sqrt((double)a.G * rr_row));
            if (row0 + rw < n_rows && q0 + lr < a.B) s_out[(int64_t)(q0 + lr) * ld_out + row0 + rw] = sc;
        }
    }
}

// ------------------------------------------------------------------------------------------
// Selection helpers.  Scores map to 64-bit keys whose unsigned order is "better first"
// (descending score); ~0 marks an entry that may not be chosen.
// ------------------------------------------------------------------------------------------
__device__ __forceinline__ uint64_t desc_key(double s) {
    if (s == 0.0) s = 0.0; // -0 and +0 are the same score
    const uint64_t u = (uint64_t)__double_as_longlong(s);
    const uint64_t asc = (u >> 63) ? ~u : (u | 0x8000000000000000ull);
    return ~asc;
}
constexpr uint64_t kNoKey = ~0ull;

struct SelShared {
    unsigned hist[256];
    uint64_t sel_key[kMaxCand];
    int sel_idx[kMaxCand];
    uint64_t loc_key[kSelThreads];
    int wtot[kSelThreads / 64];
    int count;
    int need;
    unsigned digit;
    int n_cand;
    uint64_t thr;
};

constexpr int kDirectN = 512; // up to this many entries are ranked against each other directly

// Rank by counting: for every entry t < n of keys[] (ties broken by ids[], or by the entry
// number when ids is null) the number of entries ahead of it.  The n*n comparisons are spread
// over the workgroup: `per` adjacent lanes share one entry, each counting over a stride of the
// entries, and add their counts with lane exchanges.  fn(t, rank) runs in one lane per entry.
// All threads of the workgroup must call it; keys / ids are LDS arrays complete before the call.
template <typename Fn>
__device__ __forceinline__ void block_rank(const uint64_t *keys, const int *ids, int n, Fn fn) {
    int p2 = 1;
    while (p2 < n) p2 <<= 1;
    int per = kSelThreads / p2;
    per = per < 1 ? 1 : (per > 64 ? 64 : per);
    const int tid = threadIdx.x, part = tid & (per - 1);
    for (int t0 = 0; t0 < n; t0 += kSelThreads / per) {
        const int t = t0 + tid / per;
        const bool live = t < n;
        const uint64_t kt = keys[live ? t : 0];
        const int it = ids ? ids[live ? t : 0] : t;
        int cnt = 0;
        for (int u0 = part; u0 < n; u0 += 8 * per) { // 8 independent LDS reads, then branch-free compares
            uint64_t ku[8];
            int iu[8];
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                const int u = u0 + j * per;
                const int uc = u < n ? u : n - 1;
                ku[j] = keys[uc];
                iu[j] = ids ? ids[uc] : uc;
            }
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                const int ahead = (int)(ku[j] < kt) | ((int)(ku[j] == kt) & (int)(iu[j] < it));
                cnt += (u0 + j * per < n) ? ahead : 0;
            }
        }
        for (int o = 1; o < per; o <<= 1) cnt += __shfl_xor(cnt, o);
        if (live && part == 0) fn(t, cnt);
    }
}

// Chooses the m best of entries 0..n-1 (smallest key; equal keys: lowest entry number) and
// writes their entry numbers to out[0..m_eff) in rank order.  Returns m_eff = min(m, number of
// entries whose key is not kNoKey).  All threads of the workgroup must call it.
// The keys of the first `cap` entries are computed once (batches of independent loads) and kept
// in the LDS array `cache`; entries past `cap` are recomputed from `key` on every pass.
// Three routes, all giving the same (key, entry)-ordered result:
//  * n <= kDirectN: every entry counts the entries ahead of it (rank by counting);
//  * otherwise a pre-filter: the entries are dealt to at least 2*m_eff groups of threads, each
//    group keeps its best key, the m_eff-th best of the group keys bounds the m_eff-th best
//    key overall from above, and the (usually few) entries at or below that bound are ranked
//    by counting;
//  * when the pre-filter leaves more than kMaxCand entries (many equal keys, or m_eff larger
//    than the thread count): 8-bit radix select of the m_eff-th key (LDS histograms, the digit
//    found by a wave-parallel prefix sum), one pass collecting everything better than it, an
//    ordered scan handing the remaining places to the first entries equal to it, then a
//    rank-by-counting sort of the survivors.
template <typename KeyFn>
__device__ int block_topk(KeyFn key, int n, int m, int *out, SelShared &sh, uint64_t *cache, int cap) {
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    __syncthreads();
    if (tid == 0) {
        sh.count = 0;
        sh.n_cand = 0;
    }
    __syncthreads();
    int mine = 0;
    uint64_t best = kNoKey;
    const int n_c = n < cap ? n : cap;
    for (int i0 = tid; i0 < n_c; i0 += 8 * kSelThreads) {
        uint64_t kk[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) {
            const int i = i0 + u * kSelThreads;
            kk[u] = key(i < n_c ? i : n_c - 1); // clamped: loads stay unconditional
        }
#pragma unroll
        for (int u = 0; u < 8; ++u) {
            const int i = i0 + u * kSelThreads;
            if (i < n_c) {
                cache[i] = kk[u];
                mine += kk[u] != kNoKey;
                best = kk[u] < best ? kk[u] : best;
            }
        }
    }
    for (int i = n_c + tid; i < n; i += kSelThreads) {
        const uint64_t k = key(i);
        mine += k != kNoKey;
        best = k < best ? k : best;
    }
    auto get = [&](int i) { return i < n_c ? cache[i] : key(i); };
    mine = wave_sum(mine);
    if (lane == 0 && mine) atomicAdd(&sh.count, mine);
    __syncthreads();
    const int m_eff = min(m, sh.count);
    if (m_eff == 0) return 0;

    if (n <= kDirectN && n <= n_c) {
        // entries without a key rank behind every entry that has one, so they never reach out[]
        block_rank(cache, nullptr, n, [&](int t, int rank) {
            if (rank < m_eff) out[rank] = t;
        });
        __syncthreads();
        return m_eff;
    }
    if (m_eff <= kSelThreads) {
        int n_grp = 8;
        while (n_grp < 2 * m_eff && n_grp < kSelThreads) n_grp <<= 1;
        const int grp = kSelThreads / n_grp; // adjacent lanes per group, a power of two <= 64
        for (int o = 1; o < grp; o <<= 1) {
            const uint64_t other = (uint64_t)__shfl_xor((unsigned long long)best, o);
            best = other < best ? other : best;
        }
        if ((tid & (grp - 1)) == 0) sh.loc_key[tid / grp] = best;
        __syncthreads();
        block_rank(sh.loc_key, nullptr, n_grp, [&](int t, int rank) {
            if (rank == m_eff - 1) sh.thr = sh.loc_key[t];
        });
        __syncthreads();
        const uint64_t bound = sh.thr;
        for (int i = tid; i < n; i += kSelThreads) {
            const uint64_t k = get(i);
            if (k <= bound && k != kNoKey) {
                const int pos = atomicAdd(&sh.n_cand, 1);
                if (pos < kMaxCand) {
                    sh.sel_key[pos] = k;
                    sh.sel_idx[pos] = i;
                }
            }
        }
        __syncthreads();
        const int n_cand = sh.n_cand;
        if (n_cand <= kMaxCand) {
            block_rank(sh.sel_key, sh.sel_idx, n_cand, [&](int t, int rank) {
                if (rank < m_eff) out[rank] = sh.sel_idx[t];
            });
            __syncthreads();
            return m_eff;
        }
    }
    __syncthreads();

    uint64_t prefix = 0;
    if (tid == 0) sh.need = m_eff;
    for (int pb = 7; pb >= 0; --pb) {
        for (int d = tid; d < 256; d += kSelThreads) sh.hist[d] = 0;
        __syncthreads();
        for (int i = tid; i < n; i += kSelThreads) {
            const uint64_t k = get(i);
            if (k == kNoKey) continue;
            const bool match = (pb == 7) || ((k >> (8 * (pb + 1))) == prefix);
            if (match) atomicAdd(&sh.hist[(unsigned)(k >> (8 * pb)) & 255u], 1u);
        }
        __syncthreads();
        if (wave == 0) {
            // lane owns bins 4*lane..4*lane+3; find the bin where the running count reaches need
            const int need = sh.need;
            const int h0 = (int)sh.hist[4 * lane], h1 = (int)sh.hist[4 * lane + 1];
            const int h2 = (int)sh.hist[4 * lane + 2], h3 = (int)sh.hist[4 * lane + 3];
            const int loc = h0 + h1 + h2 + h3;
            int inc = loc;
#pragma unroll
            for (int o = 1; o < 64; o <<= 1) {
                const int t = __shfl_up(inc, o);
                if (lane >= o) inc += t;
            }
            const int before = inc - loc;
            if (before < need && need <= inc) {
                int cum = before;
                unsigned d = 4 * lane;
                if (cum + h0 < need) {
                    cum += h0;
                    ++d;
                    if (cum + h1 < need) {
                        cum += h1;
                        ++d;
                        if (cum + h2 < need) {
                            cum += h2;
                            ++d;
                        }
                    }
                }
                sh.digit = d;
                sh.need = need - cum;
            }
        }
        __syncthreads();
        prefix = (prefix << 8) | sh.digit;
    }
    const uint64_t thr = prefix;      // the m_eff-th best key
    const int n_equal = sh.need;      // how many entries equal to it are still wanted (>= 1)
    const int n_less = m_eff - n_equal;
    __syncthreads();
    if (tid == 0) sh.count = 0;
    __syncthreads();
    for (int i = tid; i < n; i += kSelThreads) {
        const uint64_t k = get(i);
        if (k < thr) {
            const int pos = atomicAdd(&sh.count, 1);
            sh.sel_key[pos] = k;
            sh.sel_idx[pos] = i;
        }
    }
    // entries equal to the threshold, in entry order
    int running = 0;
    for (int base = 0; base < n && running < n_equal; base += kSelThreads) {
        const int i = base + tid;
        const bool flag = i < n && get(i) == thr;
        const uint64_t bal = __ballot(flag);
        const int below = __popcll(bal & ((1ull << lane) - 1ull));
        __syncthreads();
        if (lane == 0) sh.wtot[wave] = __popcll(bal);
        __syncthreads();
        int before = 0, total = 0;
        for (int w = 0; w < kSelThreads / 64; ++w) {
            if (w < wave) before += sh.wtot[w];
            total += sh.wtot[w];
        }
        const int ord = running + before + below;
        if (flag && ord < n_equal) {
            sh.sel_key[n_less + ord] = thr;
            sh.sel_idx[n_less + ord] = i;
        }
        running += total;
    }
    __syncthreads();
    // order the m_eff survivors by (key, entry)
    int my_rank[kMaxCand / kSelThreads], my_idx[kMaxCand / kSelThreads];
#pragma unroll
    for (int s = 0; s < kMaxCand / kSelThreads; ++s) {
        const int t = tid + s * kSelThreads;
        my_rank[s] = -1;
        if (t < m_eff) {
            const uint64_t kt = sh.sel_key[t];
            const int it = sh.sel_idx[t];
            int rank = 0;
            for (int u = 0; u < m_eff; ++u) {
                const uint64_t ku = sh.sel_key[u];
                rank += (ku < kt) || (ku == kt && sh.sel_idx[u] < it);
            }
            my_rank[s] = rank;
            my_idx[s] = it;
        }
    }
    __syncthreads();
#pragma unroll
    for (int s = 0; s < kMaxCand / kSelThreads; ++s)
        if (my_rank[s] >= 0) out[my_rank[s]] = my_idx[s];
    __syncthreads();
    return m_eff;
}

// ------------------------------------------------------------------------------------------
// Stage 1 / stage 2 of Sec. 3.4 for one question per workgroup.
// ------------------------------------------------------------------------------------------
struct RerankArgs {
    const double *s_frm, *s_seg;
    int64_t ld_frm, ld_seg;
    const float *rep_frame, *rep_seg, *seg_tail;
    int nv, ns, C, F, tail_cut;
    int mode, k_seg, k_frame, n_global;
    const int32_t *cnt; // fine level = super-patches: kept tokens per super-patch (empty ones are never chosen); else null
    const int32_t *nv_q; // per-question timestamps (visible frames), or null: nv / ns / tail_cut above hold for all
    int n_all, kpf, Ff;  // ingested frames, fine keys per frame, frames per segment (used with nv_q)
    int cache_cap; // entries of the LDS key cache (dynamic shared memory)
    // one store's units as the blocks (several stores searched together): 0 = off; 1 = the coarsest
    // store: top k_frame units by their stage-1 scores, and their first n_global keys' mean to g_out;
    // 2 = a finer store: stage 1, then Eq. 8 with the global query g_in, final top k_frame
    int units;
    const double *g_in; // [B][C]
    double *g_out;      // [B][C] or null
    double lambda;
    int32_t *seg_idx, *frm_idx;
    float *seg_score, *frm_score;
};

constexpr int kMaxSegBitmapWords = 2048; // HIER mode: segments 0..65535

// kPatches: the fine level is the super-patch table (empty super-patches get no key).
template <bool kPatches>
__global__ __launch_bounds__(kSelThreads) void select_rerank_kernel(RerankArgs a) {
    __shared__ SelShared sh;
    __shared__ int cand_seg[kMaxCand];
    __shared__ int cand_frm[kMaxCand];
    __shared__ int order[kMaxCand];
    __shared__ double st[kMaxCand];
    __shared__ double gvec[1024];
    __shared__ unsigned seg_ok[kMaxSegBitmapWords];
    __shared__ double gg_sh;
    extern __shared__ __align__(16) unsigned char smem_raw[];
    uint64_t *kcache = reinterpret_cast<uint64_t *>(smem_raw); // [a.cache_cap]
    const int cap = a.cache_cap;
    const int b = blockIdx.x, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    if (a.nv_q) { // this question's own timestamp: what it sees, and whether it cuts a segment
        int nvb = a.nv_q[b];
        nvb = (nvb < 0 || nvb > a.n_all) ? a.n_all : nvb;
        a.nv = nvb * a.kpf;
        a.ns = (nvb + a.Ff - 1) / a.Ff;
        const int seg_end = a.ns * a.Ff < a.n_all ? a.ns * a.Ff : a.n_all;
        a.tail_cut = (a.ns > 0 && nvb < seg_end) ? 1 : 0;
        a.seg_tail += (int64_t)b * a.C;
    }
    const double *s_frm = a.s_frm + (int64_t)b * a.ld_frm;
    const double *s_seg = a.s_seg + (int64_t)b * a.ld_seg;
    int32_t *seg_out = a.seg_idx + (int64_t)b * a.k_seg;
    int32_t *frm_out = a.frm_idx + (int64_t)b * a.k_frame;
    float *seg_sc = a.seg_score ? a.seg_score + (int64_t)b * a.k_seg : nullptr;
    float *frm_sc = a.frm_score ? a.frm_score + (int64_t)b * a.k_frame : nullptr;

    auto seg_key = [&](int i) { return desc_key(s_seg[i]); };
    auto frm_key = [&](int i) { // both loads unconditional, the choice afterwards
        const uint64_t k = desc_key(s_frm[i]);
        if constexpr (kPatches) {
            const int n_kept = a.cnt[i];
            return n_kept == 0 ? kNoKey : k;
        } else {
            return k;
        }
    };

    if (a.units == 1) {
        const int m_u = block_topk(frm_key, a.nv, a.k_frame, cand_frm, sh, kcache, cap);
        for (int r = tid; r < a.k_frame; r += kSelThreads) {
            frm_out[r] = r < m_u ? cand_frm[r] : -1;
            if (frm_sc) frm_sc[r] = r < m_u ? (float)s_frm[cand_frm[r]] : 0.f;
        }
        if (a.g_out) { // the global query for the finer stores: mean of the first n_glob chosen keys
            int n_glob = a.n_global > 0 ? a.n_global : a.k_frame;
            n_glob = min(n_glob, m_u);
            for (int c = tid; c < a.C; c += kSelThreads) {
                double sum = 0.0;
                for (int r0 = 0; r0 < n_glob; r0 += 8) { // batches of 8 independent loads, summed in list order
                    float x[8];
#pragma unroll
                    for (int u = 0; u < 8; ++u)
                        x[u] = a.rep_frame[(int64_t)cand_frm[r0 + u < n_glob ? r0 + u : n_glob - 1] * a.C + c];
#pragma unroll
                    for (int u = 0; u < 8; ++u)
                        if (r0 + u < n_glob) sum += (double)x[u];
                }
                a.g_out[(int64_t)b * a.C + c] = n_glob > 0 ? sum / (double)n_glob : 0.0;
            }
        }
        return;
    }
    if (a.mode != MUKV_SEMI) {
        const int m_s = block_topk(seg_key, a.ns, a.k_seg, cand_seg, sh, kcache, cap);
        for (int r = tid; r < a.k_seg && a.seg_idx; r += kSelThreads) {
            seg_out[r] = r < m_s ? cand_seg[r] : -1;
            if (seg_sc) seg_sc[r] = r < m_s ? (float)s_seg[cand_seg[r]] : 0.f;
        }
        int m_f;
        if (a.mode == MUKV_HIER) {
            for (int w = tid; w < kMaxSegBitmapWords; w += kSelThreads) seg_ok[w] = 0u;
            __syncthreads();
            for (int r = tid; r < m_s; r += kSelThreads) atomicOr(&seg_ok[cand_seg[r] >> 5], 1u << (cand_seg[r] & 31));
            __syncthreads();
            auto hier_key = [&](int i) {
                const int s = i / a.F;
                return ((seg_ok[s >> 5] >> (s & 31)) & 1u) ? frm_key(i) : kNoKey;
            };
            m_f = block_topk(hier_key, a.nv, a.k_frame, cand_frm, sh, kcache, cap);
        } else {
            m_f = block_topk(frm_key, a.nv, a.k_frame, cand_frm, sh, kcache, cap);
        }
        for (int r = tid; r < a.k_frame; r += kSelThreads) {
            frm_out[r] = r < m_f ? cand_frm[r] : -1;
            if (frm_sc) frm_sc[r] = r < m_f ? (float)s_frm[cand_frm[r]] : 0.f;
        }
        return;
    }

    // ---- semi-hierarchical ----
    int m_s = 0;
    if (a.units == 0) {
        m_s = block_topk(seg_key, a.ns, 2 * a.k_seg, cand_seg, sh, kcache, cap);
        for (int r = tid; r < a.k_seg && a.seg_idx; r += kSelThreads) { // lambda = 0 for segments: stage-1 order stands
            seg_out[r] = r < m_s ? cand_seg[r] : -1;
            if (seg_sc) seg_sc[r] = r < m_s ? (float)s_seg[cand_seg[r]] : 0.f;
        }
    }
    const int m_f = block_topk(frm_key, a.nv, 2 * a.k_frame, order, sh, kcache, cap);
    // candidates in ascending frame order, so that equal reranked scores resolve to the lowest frame
    for (int t = tid; t < m_f; t += kSelThreads) {
        const int me = order[t];
        int pos = 0;
        for (int u = 0; u < m_f; ++u) pos += order[u] < me;
        cand_frm[pos] = me;
    }
    // global query: handed over (it comes from a coarser store), or the mean of the first n_glob stage-1 segment keys
    int n_glob = a.n_global > 0 ? a.n_global : a.k_seg;
    n_glob = min(n_glob, m_s);
    for (int c = tid; c < a.C; c += kSelThreads) {
        if (a.units == 2) {
            gvec[c] = a.g_in[(int64_t)b * a.C + c];
            continue;
        }
        double s = 0.0;
        for (int r0 = 0; r0 < n_glob; r0 += 8) { // batches of 8 independent loads, summed in list order
            float x[8];
#pragma unroll
            for (int u = 0; u < 8; ++u) {
                const int sgi = cand_seg[r0 + u < n_glob ? r0 + u : n_glob - 1];
                const float *rep = (a.tail_cut && sgi == a.ns - 1) ? a.seg_tail : a.rep_seg + (int64_t)sgi * a.C;
                x[u] = rep[c];
            }
#pragma unroll
            for (int u = 0; u < 8; ++u)
                if (r0 + u < n_glob) s += (double)x[u];
        }
        gvec[c] = n_glob > 0 ? s / (double)n_glob : 0.0;
    }
    __syncthreads();
    if (wave == 0) {
        double gg = 0.0;
        for (int c = lane; c < a.C; c += 64) gg += gvec[c] * gvec[c];
        gg = wave_sum(gg);
        if (lane == 0) gg_sh = gg;
    }
    __syncthreads();
    const double gg = gg_sh;
    // Eq. 8: a 16-lane row per candidate, 4 candidates per wave and round, two rounds' key loads
    // (16-byte pieces, lane r of the row takes pieces r, r+16, ...) in flight before any use
    constexpr int kWaves = kSelThreads / 64;
    const int row = lane >> 4, rl = lane & 15;
    const int n_piece = a.C >> 2; // C is a multiple of 16
    for (int t0 = 0; t0 < m_f; t0 += 8 * kWaves) {
        double dot[2] = {0.0, 0.0}, rr[2] = {0.0, 0.0};
        int tc[2];
        const f32x4 *rep[2];
#pragma unroll
        for (int u = 0; u < 2; ++u) {
            tc[u] = t0 + (2 * wave + u) * 4 + row;
            rep[u] = reinterpret_cast<const f32x4 *>(a.rep_frame + (int64_t)cand_frm[tc[u] < m_f ? tc[u] : m_f - 1] * a.C);
        }
        for (int p0 = 0; p0 < n_piece; p0 += 64) {
            f32x4 x[2][4];
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const int pc = p0 + rl + 16 * j;
                const int pcc = pc < n_piece ? pc : n_piece - 1;
#pragma unroll
                for (int u = 0; u < 2; ++u) x[u][j] = rep[u][pcc];
            }
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const int pc = p0 + rl + 16 * j;
                if (pc < n_piece) {
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        const double g = gvec[4 * pc + e];
#pragma unroll
                        for (int u = 0; u < 2; ++u) {
                            const double xv = (double)x[u][j][e];
                            dot[u] += xv * g;
                            rr[u] += xv * xv;
                        }
                    }
                }
            }
        }
#pragma unroll
        for (int u = 0; u < 2; ++u) {
            dot[u] = row16_sum(dot[u]);
            rr[u] = row16_sum(rr[u]);
            if (rl == 0 && tc[u] < m_f) {
                const double gamma = (rr[u] > 0.0 && gg > 0.0) ? dot[u] / (sqrt(rr[u]) * sqrt(gg)) : 0.0;
                st[tc[u]] = (1.0 - a.lambda) * s_frm[cand_frm[tc[u]]] + a.lambda * gamma;
            }
        }
    }
    __syncthreads();
    auto st_key = [&](int i) { return desc_key(st[i]); };
    const int m_o = block_topk(st_key, m_f, a.k_frame, order, sh, kcache, cap);
    for (int r = tid; r < a.k_frame; r += kSelThreads) {
        frm_out[r] = r < m_o ? cand_frm[order[r]] : -1;
        if (frm_sc) frm_sc[r] = r < m_o ? (float)st[order[r]] : 0.f;
    }
}

// ------------------------------------------------------------------------------------------
// Gather (Sec. 3.5): grid (x, slab = (layer, K|V, KV head), question).  Every workgroup first
// turns the question's frame list into slot -> frame (ascending frame number for TEMPORAL,
// list order for AS_GIVEN; -1 and out-of-range entries dropped) -- lists of up to 64 frames inside
// each wave (a lane per entry, ranks by counting over lane reads, the slot's frame handed to the
// slot's lane by a lane permute; no LDS, no barrier), longer lists in LDS -- then moves its share
// of the slab: slot s of the output is the dense run of kappa rows of frame slot_frame[s] in the
// store.  Slots past the last selected frame are zero-filled.
// ------------------------------------------------------------------------------------------
struct GatherArgs {
    const int32_t *frame_idx;
    int k_frame, order;
    const unsigned char *store_k, *store_v;
    unsigned char *k_out, *v_out;
    int32_t *n_tokens_out;
    int64_t slab_b;       // bytes of one (layer, head) slab of the store
    int64_t frame_b;      // bytes of one frame's kept rows in a slab (kappa*D*esz)
    int units_per_frame;  // frame_b / 16
    int L, Hkv, kappa;
    int64_t n_frames;
};

template <int ITER, int ROUNDS>
__global__ __launch_bounds__(256) void gather_kv_kernel(GatherArgs a) {
    __shared__ int slot_frame[kMaxGatherK];
    __shared__ int n_valid_sh;
    __shared__ int raw[kMaxGatherK];
    const int tid = threadIdx.x, lane = tid & 63, b = blockIdx.z, y = blockIdx.y;
    const int32_t *idx = a.frame_idx + (int64_t)b * a.k_frame;
    const bool in_wave = a.k_frame <= 64; // the whole plan fits a wave: no LDS, no barrier
    int n_valid, sf_lane = -1;            // in_wave: lane s holds the frame of slot s (-1: empty)
    if (in_wave) {
        int me = -1;
        if (lane < a.k_frame) {
            const int x = idx[lane];
            me = (x < 0 || x >= a.n_frames) ? -1 : x;
        }
        const bool ok = me >= 0;
        const uint64_t okmask = __ballot(ok);
        const int ok_before = __popcll(okmask & ((1ull << lane) - 1ull));
        n_valid = __popcll(okmask);
        int pos = ok_before; // AS_GIVEN: list order
        if (a.order == MUKV_TEMPORAL) {
            pos = 0;
            for (int j = 0; j < a.k_frame; ++j) {
                const int o = __builtin_amdgcn_readlane(me, j);
                pos += (int)(o >= 0) & ((int)(o < me) | ((int)(o == me) & (int)(j < lane)));
            }
        }
        // every lane sends to a lane of its own: entries that name a frame to their slot, the others
        // to the places behind
        const int target = ok ? pos : n_valid + (lane - ok_before);
        sf_lane = __builtin_amdgcn_ds_permute(target << 2, me + 1) - 1;
    } else {
        if (tid == 0) n_valid_sh = 0;
        for (int t = tid; t < a.k_frame; t += 256) {
            slot_frame[t] = -1;
            const int me = idx[t];
            raw[t] = (me < 0 || me >= a.n_frames) ? -1 : me;
        }
        __syncthreads();
        int cnt = 0;
        for (int t = tid; t < a.k_frame; t += 256) {
            const int me = raw[t];
            if (me < 0) continue;
            int pos = 0;
            if (a.order == MUKV_TEMPORAL) {
#pragma unroll 4
                for (int u = 0; u < a.k_frame; ++u) {
                    const int o = raw[u];
                    pos += (o >= 0) && (o < me || (o == me && u < t));
                }
            } else {
#pragma unroll 4
                for (int u = 0; u < t; ++u) pos += raw[u] >= 0;
            }
            slot_frame[pos] = me;
            ++cnt;
        }
        if (cnt) atomicAdd(&n_valid_sh, cnt);
        __syncthreads();
        n_valid = n_valid_sh;
    }
    if (a.n_tokens_out && blockIdx.x == 0 && y == 0 && tid == 0) a.n_tokens_out[b] = n_valid * a.kappa;

    const int l = y / (2 * a.Hkv), rem = y - l * 2 * a.Hkv;
    const int kv = rem / a.Hkv, g = rem - kv * a.Hkv;
    const unsigned char *src = (kv ? a.store_v : a.store_k) + ((int64_t)l * a.Hkv + g) * a.slab_b;
    unsigned char *dst = (kv ? a.v_out : a.k_out) + (((int64_t)b * a.L + l) * a.Hkv + g) * (a.k_frame * a.frame_b);
    const int n_units = a.k_frame * a.units_per_frame;
    // ROUNDS rounds of ITER 16-byte pieces per lane; the loads of round r+1 are issued before the stores of
    // round r, so that reads and writes of the launch overlap (its workgroups all start together and would
    // otherwise all read, then all write).  Loads are unconditional (a piece past the end reads the last
    // slot, an empty slot reads slot 0's frame), the zero for an empty slot is selected afterwards.
    // A lane's pieces are 256 apart: (slot, piece in the frame) of the first by one division, the others by
    // adding 256 in mixed radix.
    cp_u32x4 tmp[2][ITER];
    const int fr_any = n_valid > 0 ? (in_wave ? __builtin_amdgcn_readlane(sf_lane, 0) : slot_frame[0]) : 0;
    const int upf = a.units_per_frame;
    const int dq = 256 / upf, dr = 256 - dq * upf;
    const int u_first = blockIdx.x * ROUNDS * (256 * ITER) + tid;
    int slot = u_first / upf, part = u_first - slot * upf;
    auto load_round = [&](cp_u32x4(&t)[ITER]) {
#pragma unroll
        for (int it = 0; it < ITER; ++it) {
            const int sc = slot < a.k_frame ? slot : a.k_frame - 1;
            const int fr = in_wave ? __builtin_amdgcn_ds_bpermute(sc << 2, sf_lane) : slot_frame[sc];
            const cp_u32x4 x = *reinterpret_cast<const cp_u32x4 *>(src + (int64_t)(fr >= 0 ? fr : fr_any) * a.frame_b + (int64_t)part * 16);
            t[it] = fr >= 0 ? x : cp_u32x4{0u, 0u, 0u, 0u};
            slot += dq;
            part += dr;
            const int carry = part >= upf;
            slot += carry;
            part -= carry ? upf : 0;
        }
    };
    auto store_round = [&](int r, const cp_u32x4(&t)[ITER]) {
        const int u0 = (blockIdx.x * ROUNDS + r) * (256 * ITER) + tid;
#pragma unroll
        for (int it = 0; it < ITER; ++it) {
            const int u = u0 + it * 256;
            if (u < n_units) *reinterpret_cast<cp_u32x4 *>(dst + (int64_t)u * 16) = t[it];
        }
    };
    load_round(tmp[0]);
#pragma unroll
    for (int r = 0; r < ROUNDS; ++r) {
        if (r + 1 < ROUNDS) load_round(tmp[(r + 1) & 1]);
        store_round(r, tmp[r & 1]);
    }
}

// Gather at super-patch granularity.  Patch id = frame * S + s; its kept rows are the dense run
// [offset, offset + count) inside the frame's kappa rows, offset = the counts of the frame's
// earlier super-patches (kept positions are ascending, super-patches index-contiguous).  Grid as
// for gather_kv.  Every workgroup plans the question's list in LDS: valid patches in ascending id
// (TEMPORAL) or list order, their source row and the running output row; rows are then copied
// 16 bytes per lane, the slot of an output row found by bisection of the running offsets.  The
// output holds rows_cap rows per (layer, head); rows past the last copied one are zero-filled.
struct GatherPatchArgs {
    const int32_t *patch_idx;
    int k_patch, order, S;
    const int32_t *cnt_patch;
    const unsigned char *store_k, *store_v;
    unsigned char *k_out, *v_out;
    int32_t *n_tokens_out;
    int64_t slab_b;
    int row_b, upr_log; // bytes per row, log2(16-byte units per row)
    int rows_cap;       // output rows per (layer, head)
    int L, Hkv, kappa;
    int64_t n_patches;  // n_frames * S
};

__global__ __launch_bounds__(256) void gather_patches_kernel(GatherPatchArgs a) {
    __shared__ int raw[kMaxGatherK], s_src[kMaxGatherK], s_cnt[kMaxGatherK], s_off[kMaxGatherK + 1];
    const int tid = threadIdx.x, b = blockIdx.z, y = blockIdx.y;
    const int32_t *idx = a.patch_idx + (int64_t)b * a.k_patch;
    for (int t = tid; t < a.k_patch; t += 256) {
        const int me = idx[t];
        raw[t] = (me < 0 || me >= a.n_patches) ? -1 : me;
        s_cnt[t] = 0;
        s_src[t] = 0;
    }
    __syncthreads();
    for (int t = tid; t < a.k_patch; t += 256) {
        const int me = raw[t];
        if (me < 0) continue;
        int pos = 0;
        for (int u = 0; u < a.k_patch; ++u) {
            const int o = raw[u];
            pos += (o >= 0) && ((a.order == MUKV_TEMPORAL) ? (o < me || (o == me && u < t)) : (u < t));
        }
        const int f = me / a.S, sp = me - f * a.S;
        int before = 0;
        for (int q = 0; q < sp; ++q) before += a.cnt_patch[(int64_t)f * a.S + q];
        s_src[pos] = f * a.kappa + before;
        s_cnt[pos] = a.cnt_patch[me];
    }
    __syncthreads();
    if (tid == 0) { // running output rows (k_patch <= 1024: a short serial scan)
        int run = 0;
        for (int t = 0; t < a.k_patch; ++t) {
            s_off[t] = run;
            run += s_cnt[t];
        }
        s_off[a.k_patch] = run;
    }
    __syncthreads();
    const int n_rows = s_off[a.k_patch];
    if (a.n_tokens_out && blockIdx.x == 0 && y == 0 && tid == 0) a.n_tokens_out[b] = n_rows;
    const int l = y / (2 * a.Hkv), rem = y - l * 2 * a.Hkv;
    const int kv = rem / a.Hkv, g = rem - kv * a.Hkv;
    const unsigned char *src = (kv ? a.store_v : a.store_k) + ((int64_t)l * a.Hkv + g) * a.slab_b;
    unsigned char *dst = (kv ? a.v_out : a.k_out) + (((int64_t)b * a.L + l) * a.Hkv + g) * ((int64_t)a.rows_cap * a.row_b);
    const int n_units = a.rows_cap << a.upr_log;
    const int mask = (1 << a.upr_log) - 1;
    for (int u = blockIdx.x * 256 + tid; u < n_units; u += gridDim.x * 256) {
        const int row = u >> a.upr_log;
        cp_u32x4 val = {0u, 0u, 0u, 0u};
        if (row < n_rows) {
            int lo = 0, hi = a.k_patch - 1; // last slot whose first output row is <= row
            while (lo < hi) {
                const int mid = (lo + hi + 1) >> 1;
                if (s_off[mid] <= row) lo = mid; else hi = mid - 1;
            }
            const int64_t srow = (int64_t)s_src[lo] + (row - s_off[lo]);
            val = *reinterpret_cast<const cp_u32x4 *>(src + srow * a.row_b + (int64_t)(u & mask) * 16);
        }
        *reinterpret_cast<cp_u32x4 *>(dst + (int64_t)u * 16) = val;
    }
}

// Combined gather over the three granularities (Sec. 3.4): the union of the kept rows of every
// frame of the chosen segments, of the chosen frames and of the chosen super-patches, each row
// once, in temporal order.  Two kernels.  union_plan: one workgroup per question marks, per
// frame, the super-patches chosen at any level (a 32-bit mask in the context's scratch; a whole
// frame sets all S bits), counts the rows behind every mask from the per-super-patch counts,
// and scans the frames in time order into a list of entries (frame, mask, first output row).
// gather_union: workgroups walk the entries; inside a frame the rows of a chosen super-patch are
// a dense run (kept positions ascend, super-patches are index-contiguous).
struct UnionPlanArgs {
    const int32_t *seg_idx, *frame_idx, *patch_idx;
    int k_seg, k_frame, k_patch;
    int S, F, kappa;
    int n_frames;
    int64_t ld; // max_frames
    const int32_t *cnt_patch;
    uint32_t *mask;
    int32_t *entry, *count;
};

constexpr int kPlanThreads = 512;
__global__ __launch_bounds__(kPlanThreads) void union_plan_kernel(UnionPlanArgs a) {
    __shared__ int sh_sel[kPlanThreads], sh_rows[kPlanThreads];
    const int b = blockIdx.x, tid = threadIdx.x;
    uint32_t *mask = a.mask + (int64_t)b * a.ld;
    int32_t *entry = a.entry + (int64_t)b * a.ld * 3;
    const uint32_t full = a.S >= 32 ? 0xffffffffu : ((1u << a.S) - 1u);
    for (int f = tid; f < a.n_frames; f += kPlanThreads) mask[f] = 0u;
    __syncthreads();
    for (int i = tid; i < a.k_seg * a.F; i += kPlanThreads) {
        const int sg = a.seg_idx[(int64_t)b * a.k_seg + i / a.F];
        const int64_t f = (int64_t)sg * a.F + i % a.F;
        if (sg >= 0 && f < a.n_frames) atomicOr(&mask[f], full);
    }
    for (int i = tid; i < a.k_frame; i += kPlanThreads) {
        const int f = a.frame_idx[(int64_t)b * a.k_frame + i];
        if (f >= 0 && f < a.n_frames) atomicOr(&mask[f], full);
    }
    for (int i = tid; i < a.k_patch; i += kPlanThreads) {
        const int p = a.patch_idx[(int64_t)b * a.k_patch + i];
        if (p >= 0 && p / a.S < a.n_frames) atomicOr(&mask[p / a.S], 1u << (p % a.S));
    }
    __syncthreads();
    // every thread owns a contiguous range of frames; rows behind a mask from the super-patch counts
    const int per = (a.n_frames + kPlanThreads - 1) / kPlanThreads;
    const int f_lo = tid * per < a.n_frames ? tid * per : a.n_frames;
    const int f_hi = f_lo + per < a.n_frames ? f_lo + per : a.n_frames;
    auto rows_of = [&](int f, uint32_t m) {
        if (m == full) return a.kappa;
        int r = 0;
        for (int sp = 0; sp < a.S; ++sp)
            if ((m >> sp) & 1u) r += a.cnt_patch[(int64_t)f * a.S + sp];
        return r;
    };
    int n_sel = 0, n_rows = 0;
    for (int f = f_lo; f < f_hi; ++f) {
        const uint32_t m = mask[f];
        if (m) {
            ++n_sel;
            n_rows += rows_of(f, m);
        }
    }
    sh_sel[tid] = n_sel;
    sh_rows[tid] = n_rows;
    __syncthreads();
    if (tid == 0) { // exclusive scan over the threads' ranges (512 short steps)
        int rs = 0, rr = 0;
        for (int t = 0; t < kPlanThreads; ++t) {
            const int s0 = sh_sel[t], r0 = sh_rows[t];
            sh_sel[t] = rs;
            sh_rows[t] = rr;
            rs += s0;
            rr += r0;
        }
        a.count[2 * b] = rs;
        a.count[2 * b + 1] = rr;
    }
    __syncthreads();
    int e = sh_sel[tid], row = sh_rows[tid];
    for (int f = f_lo; f < f_hi; ++f) {
        const uint32_t m = mask[f];
        if (m) {
            entry[3 * e] = f;
            entry[3 * e + 1] = (int32_t)m;
            entry[3 * e + 2] = row;
            row += rows_of(f, m);
            ++e;
        }
    }
}

struct UnionGatherArgs {
    const int32_t *entry, *count;
    int64_t ld;
    const int32_t *cnt_patch;
    int S, kappa;
    const unsigned char *store_k, *store_v;
    unsigned char *k_out, *v_out;
    int32_t *n_tokens_out;
    int64_t slab_b;
    int row_b, upr_log, rows_cap;
    int L, Hkv;
};

__global__ __launch_bounds__(256) void gather_union_kernel(UnionGatherArgs a) {
    const int tid = threadIdx.x, b = blockIdx.z, y = blockIdx.y;
    const int n_ent = a.count[2 * b], n_rows = a.count[2 * b + 1];
    if (a.n_tokens_out && blockIdx.x == 0 && y == 0 && tid == 0) a.n_tokens_out[b] = n_rows;
    const int32_t *entry = a.entry + (int64_t)b * a.ld * 3;
    const int l = y / (2 * a.Hkv), rem = y - l * 2 * a.Hkv;
    const int kv = rem / a.Hkv, g = rem - kv * a.Hkv;
    const unsigned char *src = (kv ? a.store_v : a.store_k) + ((int64_t)l * a.Hkv + g) * a.slab_b;
    unsigned char *dst = (kv ? a.v_out : a.k_out) + (((int64_t)b * a.L + l) * a.Hkv + g) * ((int64_t)a.rows_cap * a.row_b);
    const int upr = 1 << a.upr_log;
    for (int e = blockIdx.x; e < n_ent; e += gridDim.x) {
        const int f = entry[3 * e];
        const uint32_t m = (uint32_t)entry[3 * e + 1];
        int out_row = entry[3 * e + 2];
        int before = 0; // kept rows of the frame in earlier super-patches
        for (int sp = 0; sp < a.S; ++sp) {
            const int c = a.cnt_patch[(int64_t)f * a.S + sp];
            if ((m >> sp) & 1u) {
                const int c_fit = out_row + c <= a.rows_cap ? c : (a.rows_cap > out_row ? a.rows_cap - out_row : 0);
                const unsigned char *s0 = src + ((int64_t)f * a.kappa + before) * a.row_b;
                unsigned char *d0 = dst + (int64_t)out_row * a.row_b;
                for (int u = tid; u < c_fit * upr; u += 256)
                    *reinterpret_cast<cp_u32x4 *>(d0 + (int64_t)u * 16) = *reinterpret_cast<const cp_u32x4 *>(s0 + (int64_t)u * 16);
                out_row += c;
            }
            before += c;
        }
    }
    // rows past the union are zero
    const int first = n_rows < a.rows_cap ? n_rows : a.rows_cap;
    const int64_t n_zero = (int64_t)(a.rows_cap - first) * upr;
    unsigned char *z0 = dst + (int64_t)first * a.row_b;
    for (int64_t u = (int64_t)blockIdx.x * 256 + tid; u < n_zero; u += (int64_t)gridDim.x * 256)
        *reinterpret_cast<cp_u32x4 *>(z0 + u * 16) = cp_u32x4{0u, 0u, 0u, 0u};
}

// The decode context from several independently compressed stores (Sec. 3.3: one cache per granularity;
// Sec. 3.5: what was retrieved is loaded as the context): the kept rows of the chosen units of every
// store in temporal order -- ascending time step (unit u of store i belongs to step u / ups[i]), within
// a step the stores in the order given and a store's units ascending; a unit listed twice is taken
// once, entries that name no unit are skipped.  multi_plan: one workgroup per question orders the
// entries by counting (key = step, store, unit) and adds up the rows in front of each; multi_gather:
// workgroups walk the ordered entries, each a dense run of kappa_i rows of its store's slab.
struct MultiStore {
    const unsigned char *store_k, *store_v;
    int64_t slab_b;  // bytes of one (layer, head) slab
    int64_t n_units; // units held
    int kappa;
};
struct MultiPlanArgs {
    const int32_t *idx[kMaxStores];
    int k[kMaxStores], ups[kMaxStores], kappa[kMaxStores];
    int64_t n_units[kMaxStores];
    int n_ctx;
    int32_t *entry, *count;
};

__global__ __launch_bounds__(kPlanThreads) void multi_plan_kernel(MultiPlanArgs a) {
    __shared__ uint64_t key[kMaxMultiEntries]; // (step, store, unit), or kNoKey for an entry that is skipped
    __shared__ bool repeat[kMaxMultiEntries];
    __shared__ int n_sh, rows_sh;
    const int b = blockIdx.x, tid = threadIdx.x;
    int n = 0;
    for (int i = 0; i < a.n_ctx; ++i) n += a.k[i];
    if (tid == 0) n_sh = rows_sh = 0;
    int base = 0;
    for (int i = 0; i < a.n_ctx; ++i) {
        for (int t = tid; t < a.k[i]; t += kPlanThreads) {
            const int u = a.idx[i][(int64_t)b * a.k[i] + t];
            const bool ok = u >= 0 && u < a.n_units[i];
            key[base + t] = ok ? ((uint64_t)(unsigned)(u / a.ups[i]) << 34) | ((uint64_t)i << 32) | (unsigned)u : kNoKey;
        }
        base += a.k[i];
    }
    __syncthreads();
    // a unit listed twice is taken once: later repeats leave the list
    for (int t = tid; t < n; t += kPlanThreads) {
        const uint64_t kt = key[t];
        bool rep = false;
        for (int u = 0; u < t; ++u) rep |= key[u] == kt;
        repeat[t] = rep;
    }
    __syncthreads();
    for (int t = tid; t < n; t += kPlanThreads)
        if (repeat[t]) key[t] = kNoKey;
    __syncthreads();
    int32_t *entry = a.entry + (int64_t)b * kMaxMultiEntries * 3;
    int mine = 0, mine_rows = 0;
    for (int t = tid; t < n; t += kPlanThreads) {
        const uint64_t kt = key[t];
        if (kt == kNoKey) continue;
        int pos = 0, row = 0;
        for (int u = 0; u < n; ++u) { // entries ahead of this one, and the rows they bring
            const uint64_t ku = key[u];
            const bool ahead = ku < kt; // (kNoKey is the largest key: skipped entries are ahead of nobody)
            pos += ahead;
            row += ahead ? a.kappa[(int)((ku >> 32) & 3u)] : 0;
        }
        const int st = (int)((kt >> 32) & 3u);
        entry[3 * pos] = st;
        entry[3 * pos + 1] = (int)(unsigned)(kt & 0xffffffffu);
        entry[3 * pos + 2] = row;
        ++mine;
        mine_rows += a.kappa[st];
    }
    if (mine) {
        atomicAdd(&n_sh, mine);
        atomicAdd(&rows_sh, mine_rows);
    }
    __syncthreads();
    if (tid == 0) {
        a.count[2 * b] = n_sh;
        a.count[2 * b + 1] = rows_sh;
    }
}

struct MultiGatherArgs {
    MultiStore s[kMaxStores];
    const int32_t *entry, *count;
    unsigned char *k_out, *v_out;
    int32_t *n_tokens_out;
    int row_b, upr_log, rows_cap;
    int L, Hkv;
};

// Grid (x, slab = (layer, K|V, KV head), question): workgroup x moves output rows x * rows_per_wg ... of its slab,
// whatever entries they belong to (a segment unit's hundreds of rows are shared by several workgroups, a
// super-patch unit's four rows are a fraction of one): the entries' first output rows sit in LDS, a lane finds
// the entry of its first row by bisection and walks on from there; a lane holds one 16-byte piece of
// kMultiIter rows, all requested before the first is stored.  Rows past the context are zero.
constexpr int kMultiIter = 8;
__global__ __launch_bounds__(256) void multi_gather_kernel(MultiGatherArgs a, int rows_per_wg) {
    __shared__ int e_start[kMaxMultiEntries + 1];
    const int tid = threadIdx.x, b = blockIdx.z, y = blockIdx.y;
    const int n_ent = a.count[2 * b], n_rows = a.count[2 * b + 1];
    if (a.n_tokens_out && blockIdx.x == 0 && y == 0 && tid == 0) a.n_tokens_out[b] = n_rows;
    const int32_t *entry = a.entry + (int64_t)b * kMaxMultiEntries * 3;
    for (int e = tid; e < n_ent; e += 256) e_start[e] = entry[3 * e + 2];
    if (tid == 0) e_start[n_ent] = n_rows;
    __syncthreads();
    const int l = y / (2 * a.Hkv), rem = y - l * 2 * a.Hkv;
    const int kv = rem / a.Hkv, g = rem - kv * a.Hkv;
    unsigned char *dst = (kv ? a.v_out : a.k_out) + (((int64_t)b * a.L + l) * a.Hkv + g) * ((int64_t)a.rows_cap * a.row_b);
    const int64_t slab = (int64_t)l * a.Hkv + g;
    const int upr = 1 << a.upr_log, rpp = 256 >> a.upr_log; // pieces per row, rows per pass of the workgroup
    const int piece = tid & (upr - 1), rsub = tid >> a.upr_log;
    const int r_lo = blockIdx.x * rows_per_wg;
    const int r_hi = r_lo + rows_per_wg < a.rows_cap ? r_lo + rows_per_wg : a.rows_cap;
    const int n_copy = n_ent > 0 ? (n_rows < a.rows_cap ? n_rows : a.rows_cap) : 0; // rows that hold something
    for (int r0 = r_lo + rsub; r0 < r_hi; r0 += kMultiIter * rpp) {
        // entry of the lane's first row: the last one that starts at or before it
        int e = 0;
        if (r0 < n_copy) {
            int lo = 0, hi = n_ent - 1;
            while (lo < hi) {
                const int mid = (lo + hi + 1) >> 1;
                if (e_start[mid] <= r0)
                    lo = mid;
                else
                    hi = mid - 1;
            }
            e = lo;
        }
        cp_u32x4 x[kMultiIter];
        bool live[kMultiIter];
#pragma unroll
        for (int it = 0; it < kMultiIter; ++it) {
            const int r = r0 + it * rpp;
            live[it] = r < r_hi && r < n_copy;
            x[it] = cp_u32x4{0u, 0u, 0u, 0u};
            if (n_copy > 0) { // (uniform) loads are unconditional on a clamped row
                const int rc = live[it] ? r : n_copy - 1;
                while (e + 1 < n_ent && e_start[e + 1] <= rc) ++e;
                const MultiStore &ms = a.s[entry[3 * e]];
                const unsigned char *src = (kv ? ms.store_v : ms.store_k) + slab * ms.slab_b +
                                           ((int64_t)entry[3 * e + 1] * ms.kappa + (rc - e_start[e])) * a.row_b + piece * 16;
                x[it] = *reinterpret_cast<const cp_u32x4 *>(src);
            }
        }
#pragma unroll
        for (int it = 0; it < kMultiIter; ++it) {
            const int r = r0 + it * rpp;
            if (r < r_hi)
                *reinterpret_cast<cp_u32x4 *>(dst + (int64_t)r * a.row_b + piece * 16) =
                    live[it] ? x[it] : cp_u32x4{0u, 0u, 0u, 0u};
        }
    }
}

// Plain streaming copy, 4 x 16 bytes per thread: the calibration kernel for traffic counters.
__global__ __launch_bounds__(256) void plain_copy_kernel(const cp_u32x4 *__restrict__ src, cp_u32x4 *__restrict__ dst,
                                                         int64_t n_units) {
    const int64_t u0 = (int64_t)blockIdx.x * 1024 + threadIdx.x;
    cp_u32x4 t[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int64_t u = u0 + i * 256;
        t[i] = src[u < n_units ? u : n_units - 1];
    }
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int64_t u = u0 + i * 256;
        if (u < n_units) dst[u] = t[i];
    }
}

hipError_t launch_plain_copy(void *dst, const void *src, int64_t bytes, hipStream_t st) {
    const int64_t n_units = bytes / 16;
    if (n_units == 0) return hipSuccess;
    hipLaunchKernelGGL(plain_copy_kernel, dim3((unsigned)((n_units + 1023) / 1024)), dim3(256), 0, st,
                       reinterpret_cast<const cp_u32x4 *>(src), reinterpret_cast<cp_u32x4 *>(dst), n_units);
    return hipGetLastError();
}

// ------------------------------------------------------------------------------------------
// host side
// ------------------------------------------------------------------------------------------
// Features per workgroup of the question pooling: the largest power of two with G * dz <= 256 (one pass
// of the workgroup's element lanes), at least 1, at most D.
int pool_slice(int G, int D) {
    int dz = 1;
    while (dz * 2 <= D && G * dz * 2 <= 256) dz *= 2;
    return dz;
}

hipError_t launch_retrieve(Ctx &c, const RetrieveArgs &a, hipStream_t st) {
    const int Hq = c.cfg.n_q_heads, Hkv = c.cfg.n_kv_heads, D = c.cfg.head_dim, G = c.group;
    const int dz = pool_slice(G, D), n_z = D / dz;
    const size_t lds = (size_t)4 * G * dz * sizeof(double);
    hipError_t e;
    {
    ProfScope ps(c, MUKV_K_POOLQ, st);
    if (c.cfg.dtype == MUKV_BF16)
        hipLaunchKernelGGL((pool_question_kernel<uint16_t>), dim3(a.B, Hkv, n_z), dim3(1024), lds, st,
                           reinterpret_cast<const uint16_t *>(a.q_tokens), a.q_offsets, Hq, Hkv, D, G, dz, c.qbar, c.qq);
    else
        hipLaunchKernelGGL((pool_question_kernel<float>), dim3(a.B, Hkv, n_z), dim3(1024), lds, st,
                           reinterpret_cast<const float *>(a.q_tokens), a.q_offsets, Hq, Hkv, D, G, dz, c.qbar, c.qq);
    e = hipGetLastError();
    }
    if (e != hipSuccess) return e;

    const int F = c.cfg.frames_per_segment;
    const int64_t seg_end = (int64_t)a.ns * F < c.n_frames ? (int64_t)a.ns * F : c.n_frames;
    // per-question timestamps (a.nv_q): a.nv / a.ns cover every ingested frame, all keys are scored
    // in full and tail_fix_kernel repairs the one segment each question may cut
    const int tail_cut = (!a.nv_q && a.ns > 0 && a.nv < seg_end) ? 1 : 0;
    // fine level: the frames, or (a.patches) their super-patches -- the same kernels on the other
    // key table, S keys per frame
    const int kpf = a.patches ? c.cfg.superpatches_per_frame : 1;
    const int nf = a.nv * kpf;
    const float *rep_fine = a.patches ? c.rep_patch_k : c.rep_frame_k;
    const int64_t ld_fine = (int64_t)c.cfg.max_frames * kpf;
    if (a.nv + a.ns > 0) {
        ScoreArgs s;
        s.rep_frame = rep_fine;
        s.nf = nf;
        s.rep_seg = c.rep_seg_k;
        s.fsum = c.fsum_k;
        s.qbar = c.qbar;
        s.qq = c.qq;
        s.n_qq = Hkv * n_z;
        s.s_frm = c.s_frm;
        s.s_seg = c.s_seg;
        s.seg_tail = c.seg_tail;
        s.nv = a.nv;
        s.ns = a.ns;
        s.B = a.B;
        s.C = c.c_kv;
        s.Hkv = Hkv;
        s.G = G;
        s.F = F;
        s.kappa = c.kappa;
        s.tail_cut = tail_cut;
        s.ld_frm = ld_fine;
        s.ld_seg = c.max_segments;
        ProfScope ps(c, MUKV_K_SCORE, st);
        // many questions: the scores are a small matrix product for the fp64 matrix cores
        if (a.B >= 16) {
            if (tail_cut) hipLaunchKernelGGL(seg_tail_kernel, dim3((s.C + 255) / 256), dim3(256), 0, st, s);
            hipLaunchKernelGGL(score_blocks_mfma_kernel, dim3((nf + 15) / 16 + (a.ns + 15) / 16), dim3(256), 0, st, s);
        } else {
            hipLaunchKernelGGL(score_blocks_kernel, dim3((nf + a.ns + 3) / 4), dim3(256), 0, st, s);
        }
        if ((e = hipGetLastError()) != hipSuccess) return e;
        if (a.nv_q) {
            TailArgs t;
            t.nv_q = a.nv_q;
            t.n_all = (int)c.n_frames;
            t.F = F;
            t.kappa = c.kappa;
            t.C = c.c_kv;
            t.Hkv = Hkv;
            t.G = G;
            t.fsum = c.fsum_k;
            t.qbar = c.qbar;
            t.qq = c.qq;
            t.n_qq = Hkv * n_z;
            t.s_seg = c.s_seg;
            t.ld_seg = c.max_segments;
            t.seg_tail = c.seg_tail;
            hipLaunchKernelGGL(tail_fix_kernel, dim3(a.B), dim3(256), 0, st, t);
            if ((e = hipGetLastError()) != hipSuccess) return e;
        }
    }
    RerankArgs r;
    r.s_frm = c.s_frm;
    r.s_seg = c.s_seg;
    r.ld_frm = ld_fine;
    r.ld_seg = c.max_segments;
    r.rep_frame = rep_fine;
    r.rep_seg = c.rep_seg_k;
    r.seg_tail = c.seg_tail;
    r.nv = nf;
    r.ns = a.ns;
    r.C = c.c_kv;
    r.F = F * kpf; // fine keys per segment
    r.cnt = a.patches ? c.cnt_patch : nullptr;
    r.nv_q = a.nv_q;
    r.n_all = (int)c.n_frames;
    r.kpf = kpf;
    r.Ff = F;
    r.tail_cut = tail_cut;
    r.units = a.units;
    r.g_in = a.g_in;
    r.g_out = a.g_out;
    r.mode = a.units ? (int)MUKV_SEMI : a.p.mode;
    r.k_seg = a.p.k_seg;
    r.k_frame = a.p.k_frame;
    r.n_global = a.p.n_global;
    r.lambda = a.p.lambda_frame;
    r.seg_idx = a.seg_idx;
    r.frm_idx = a.frm_idx;
    r.seg_score = a.seg_score;
    r.frm_score = a.frm_score;
    // key cache: as many of the frame scores as fit beside the kernel's static LDS
    constexpr int kMaxCache = 11 * 1024; // 88 KB of 8-byte keys
    int n_max = nf > a.ns ? nf : a.ns;
    if (n_max < 2 * kMaxCand) n_max = 2 * kMaxCand;
    r.cache_cap = n_max < kMaxCache ? n_max : kMaxCache;
    static bool lds_ok[kMaxDevices];
    static bool lds_ok_p[kMaxDevices];
    if ((e = a.patches ? allow_dynamic_lds(reinterpret_cast<const void *>(&select_rerank_kernel<true>),
                                           (size_t)kMaxCache * 8, c.cfg.device_id, lds_ok_p)
                       : allow_dynamic_lds(reinterpret_cast<const void *>(&select_rerank_kernel<false>),
                                           (size_t)kMaxCache * 8, c.cfg.device_id, lds_ok)) != hipSuccess)
        return e;
    ProfScope ps(c, MUKV_K_RERANK, st);
    if (a.patches)
        hipLaunchKernelGGL(select_rerank_kernel<true>, dim3(a.B), dim3(kSelThreads), (size_t)r.cache_cap * 8, st, r);
    else
        hipLaunchKernelGGL(select_rerank_kernel<false>, dim3(a.B), dim3(kSelThreads), (size_t)r.cache_cap * 8, st, r);
    return hipGetLastError();
}

hipError_t launch_gather(Ctx &c, const int32_t *frame_idx, int B, int k_frame, int order, void *k_out, void *v_out,
                         int32_t *n_tokens_out, hipStream_t st) {
    GatherArgs g;
    const int row_b = c.cfg.head_dim * c.esz;
    g.frame_idx = frame_idx;
    g.k_frame = k_frame;
    g.order = order;
    g.store_k = reinterpret_cast<const unsigned char *>(c.store_k);
    g.store_v = reinterpret_cast<const unsigned char *>(c.store_v);
    g.k_out = reinterpret_cast<unsigned char *>(k_out);
    g.v_out = reinterpret_cast<unsigned char *>(v_out);
    g.n_tokens_out = n_tokens_out;
    g.slab_b = c.store_cap * row_b;
    g.frame_b = (int64_t)c.kappa * row_b;
    g.units_per_frame = (int)(g.frame_b / 16);
    g.L = c.cfg.n_layers;
    g.Hkv = c.cfg.n_kv_heads;
    g.kappa = c.kappa;
    g.n_frames = c.n_frames;
    const int n_units = k_frame * g.units_per_frame;
    // 16-byte pieces per thread: 4 rounds of 4, two rounds in flight; fewer, longer workgroups amortise the slot plan
    // (shapes from 1 x 8 to 8 x 2 pieces x rounds all took within 3 us of each other for one question of the
    // 1-hour stream)
    constexpr int ITER = 4, ROUNDS = 4;
    const int gx = (n_units + 256 * ITER * ROUNDS - 1) / (256 * ITER * ROUNDS);
    ProfScope ps(c, MUKV_K_GATHER, st);
    hipLaunchKernelGGL((gather_kv_kernel<ITER, ROUNDS>), dim3(gx, c.cfg.n_layers * 2 * c.cfg.n_kv_heads, B), dim3(256), 0, st, g);
    return hipGetLastError();
}

hipError_t launch_gather_patches(Ctx &c, const int32_t *patch_idx, int B, int k_patch, int order, int rows_cap,
                                 void *k_out, void *v_out, int32_t *n_tokens_out, hipStream_t st) {
    GatherPatchArgs g;
    g.patch_idx = patch_idx;
    g.k_patch = k_patch;
    g.order = order;
    g.S = c.cfg.superpatches_per_frame;
    g.cnt_patch = c.cnt_patch;
    g.store_k = reinterpret_cast<const unsigned char *>(c.store_k);
    g.store_v = reinterpret_cast<const unsigned char *>(c.store_v);
    g.k_out = reinterpret_cast<unsigned char *>(k_out);
    g.v_out = reinterpret_cast<unsigned char *>(v_out);
    g.n_tokens_out = n_tokens_out;
    g.row_b = c.cfg.head_dim * c.esz;
    g.slab_b = c.store_cap * g.row_b;
    int upr = g.row_b / 16, lg = 0;
    while ((1 << lg) < upr) ++lg;
    g.upr_log = lg;
    g.rows_cap = rows_cap;
    g.L = c.cfg.n_layers;
    g.Hkv = c.cfg.n_kv_heads;
    g.kappa = c.kappa;
    g.n_patches = c.n_frames * g.S;
    const int n_units = rows_cap * upr;
    int gx = (n_units + 256 * 8 - 1) / (256 * 8);
    gx = gx < 1 ? 1 : gx;
    ProfScope ps(c, MUKV_K_GATHER, st);
    hipLaunchKernelGGL(gather_patches_kernel, dim3(gx, c.cfg.n_layers * 2 * c.cfg.n_kv_heads, B), dim3(256), 0, st, g);
    return hipGetLastError();
}

hipError_t launch_gather_union(Ctx &c, const UnionArgs &a, hipStream_t st) {
    UnionPlanArgs p;
    p.seg_idx = a.seg_idx;
    p.frame_idx = a.frame_idx;
    p.patch_idx = a.patch_idx;
    p.k_seg = a.seg_idx ? a.k_seg : 0;
    p.k_frame = a.frame_idx ? a.k_frame : 0;
    p.k_patch = a.patch_idx ? a.k_patch : 0;
    p.S = c.cfg.superpatches_per_frame;
    p.F = c.cfg.frames_per_segment;
    p.kappa = c.kappa;
    p.n_frames = (int)c.n_frames;
    p.ld = c.cfg.max_frames;
    p.cnt_patch = c.cnt_patch;
    p.mask = c.u_mask;
    p.entry = c.u_entry;
    p.count = c.u_count;
    ProfScope ps(c, MUKV_K_GATHER, st);
    hipLaunchKernelGGL(union_plan_kernel, dim3(a.B), dim3(kPlanThreads), 0, st, p);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    UnionGatherArgs g;
    g.entry = c.u_entry;
    g.count = c.u_count;
    g.ld = c.cfg.max_frames;
    g.cnt_patch = c.cnt_patch;
    g.S = p.S;
    g.kappa = c.kappa;
    g.store_k = reinterpret_cast<const unsigned char *>(c.store_k);
    g.store_v = reinterpret_cast<const unsigned char *>(c.store_v);
    g.k_out = reinterpret_cast<unsigned char *>(a.k_out);
    g.v_out = reinterpret_cast<unsigned char *>(a.v_out);
    g.n_tokens_out = a.n_tokens_out;
    g.row_b = c.cfg.head_dim * c.esz;
    g.slab_b = c.store_cap * g.row_b;
    int upr = g.row_b / 16, lg = 0;
    while ((1 << lg) < upr) ++lg;
    g.upr_log = lg;
    g.rows_cap = a.rows_cap;
    g.L = c.cfg.n_layers;
    g.Hkv = c.cfg.n_kv_heads;
    hipLaunchKernelGGL(gather_union_kernel, dim3(64, c.cfg.n_layers * 2 * c.cfg.n_kv_heads, a.B), dim3(256), 0, st, g);
    return hipGetLastError();
}

hipError_t launch_gather_multi(const MultiArgs &a, hipStream_t st) {
    const Ctx &c0 = *a.c[0];
    MultiPlanArgs p;
    MultiGatherArgs g;
    for (int i = 0; i < kMaxStores; ++i) {
        const bool on = i < a.n_ctx;
        p.idx[i] = on ? a.idx[i] : nullptr;
        p.k[i] = on && a.idx[i] ? a.k[i] : 0;
        p.ups[i] = on ? a.ups[i] : 1;
        p.kappa[i] = on ? a.c[i]->kappa : 0;
        p.n_units[i] = on ? a.c[i]->n_frames : 0;
        g.s[i].store_k = on ? reinterpret_cast<const unsigned char *>(a.c[i]->store_k) : nullptr;
        g.s[i].store_v = on ? reinterpret_cast<const unsigned char *>(a.c[i]->store_v) : nullptr;
        g.s[i].slab_b = on ? a.c[i]->store_cap * (int64_t)(c0.cfg.head_dim * c0.esz) : 0;
        g.s[i].n_units = p.n_units[i];
        g.s[i].kappa = p.kappa[i];
    }
    p.n_ctx = a.n_ctx;
    p.entry = c0.m_entry;
    p.count = c0.m_count;
    hipLaunchKernelGGL(multi_plan_kernel, dim3(a.B), dim3(kPlanThreads), 0, st, p);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    g.entry = c0.m_entry;
    g.count = c0.m_count;
    g.k_out = reinterpret_cast<unsigned char *>(a.k_out);
    g.v_out = reinterpret_cast<unsigned char *>(a.v_out);
    g.n_tokens_out = a.n_tokens_out;
    g.row_b = c0.cfg.head_dim * c0.esz;
    int upr = g.row_b / 16, lg = 0;
    while ((1 << lg) < upr) ++lg;
    g.upr_log = lg;
    g.rows_cap = a.rows_cap;
    g.L = c0.cfg.n_layers;
    g.Hkv = c0.cfg.n_kv_heads;
    // one pass of kMultiIter rows per lane and workgroup, where the output is short enough for the grid
    const int rpp = 256 >> lg;
    int rows_per_wg = kMultiIter * rpp;
    if ((a.rows_cap + rows_per_wg - 1) / rows_per_wg > 4096) rows_per_wg = (a.rows_cap + 4095) / 4096;
    const int gx = a.rows_cap > 0 ? (a.rows_cap + rows_per_wg - 1) / rows_per_wg : 1;
    hipLaunchKernelGGL(multi_gather_kernel, dim3(gx, c0.cfg.n_layers * 2 * c0.cfg.n_kv_heads, a.B), dim3(256), 0, st, g,
                       rows_per_wg);
    return hipGetLastError();
}

} // namespace mukv
