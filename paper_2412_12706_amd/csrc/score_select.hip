// Prefill-time token selection (paper Section 3, "KV Pruning": keep s < n
// tokens chosen at prefill; the paper uses an attention-score method from the
// literature with the most recent tokens retained, Section 4 / Appendix B).
// The rule implemented is stated in kvqp.h at kvqp_compress:
//   votes  = column sums, over the W window rows of all query heads of a KV
//            head's group, of the causal Softmax(sm_scale q k^T) rows;
//   pooled = 1-D max-pool of the votes over the prefix;
//   keep   = the n_kept highest pooled scores, ties to the lower position,
//            listed in ascending position.
//
// Kernels.  The score matrix is a dense [Gq*W x D] x [D x L] contraction per
// KV head, so it runs on the matrix cores (v_mfma_f32_16x16x32_f16, binary32
// accumulation); everything after it is a bandwidth- or latency-bound sweep.
//   score_pass<STATS>  row maxima and exp-sums of every window row (pass 1)
//   stats_combine      merges the per-workgroup row statistics
//   score_pass<VOTES>  recomputes the tiles, normalises, sums columns (pass 2)
//   select_topk        pool, radix-select the cut, ordered compaction; scores
//                      within a relative 1e-4 of the cut are first re-scored in
//                      binary64 so that binary32 rounding cannot move the cut
// Keys stream through LDS once per pass in 128-key chunks shared by the four
// waves of a workgroup; query rows stay in registers as MFMA operands.
#include "kvqp_internal.h"

namespace kvqp {
namespace {

typedef _Float16 h8v __attribute__((ext_vector_type(8)));
typedef float f4v __attribute__((ext_vector_type(4)));
union Frag {
    h8v v;
    uint4 q;
};

constexpr int kThreads = 256;
constexpr int kRowsPerWave = 64;        // query rows one wave owns (4 MFMA row tiles)
constexpr int kMT = kRowsPerWave / 16;
constexpr int kKeyStride = kHeadDim * 2 + 16;  // LDS bytes per key row; +16 B skews banks
constexpr float kLog2e = 1.4426950408889634f;
constexpr float kNegBig = -1.0e30f;

enum { PASS_STATS = 0, PASS_VOTES = 1 };

struct ScoreArgs {
    const uint16_t* q_obs;  // [B, Hq, W, D]
    const uint16_t* k;      // [B, Hkv, L, D]
    float2* stats_part;     // [heads, n_parts, rows_pad]  (m, Z) in the log2 domain
    const float2* stats;    // [heads, rows_pad]           (m, 1/Z)
    float* vote;            // [heads, P]
    int L, W, P, gq, n_q_heads, n_kv_heads;
    int rows, rows_pad;     // Gq*W and its multiple of 64
    int chunks_per_wg, n_chunks, n_parts;
    float scale_log2;       // sm_scale * log2(e)
};

// NRW = number of 64-row slabs (1, 2, 4); the 4 waves are NRW row slabs x KS key strips.
template <int NRW> struct ScoreGeom {
    static constexpr int KS = 4 / NRW;
    static constexpr int CK = (KS == 1) ? 64 : 128;   // keys per chunk
    static constexpr int KT = CK / (16 * KS);         // key tiles per wave per chunk
};

template <int NRW, int PASS>
__global__ __launch_bounds__(kThreads) void score_pass(const ScoreArgs a) {
    using Gm = ScoreGeom<NRW>;
    constexpr int KS = Gm::KS, CK = Gm::CK, KT = Gm::KT;
    __shared__ __align__(16) unsigned char sk[CK * kKeyStride];
    __shared__ float svote[(PASS == PASS_VOTES) ? NRW * CK : 1];

    const int head = blockIdx.y;
    const int b = head / a.n_kv_heads, g = head % a.n_kv_heads;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int n = lane & 15, kb = lane >> 4;
    const int rw = wave % NRW, ks = wave / NRW;
    const uint16_t* kh = a.k + (size_t)head * a.L * kHeadDim;

    // Query operand: rows 64*rw + 16*mt + (lane & 15), channels 32*s + 8*kb .. +8.
    Frag qf[kMT][4];
#pragma unroll
    for (int mt = 0; mt < kMT; ++mt) {
        const int r = kRowsPerWave * rw + 16 * mt + n;
        const bool live = r < a.rows;
        const int hl = live ? r / a.W : 0, i = live ? r % a.W : 0;
        const uint16_t* qp = a.q_obs + (((size_t)b * a.n_q_heads + g * a.gq + hl) * a.W + i) * kHeadDim + 8 * kb;
#pragma unroll
        for (int s = 0; s < 4; ++s) {
            qf[mt][s].q = live ? *reinterpret_cast<const uint4*>(qp + 32 * s) : make_uint4(0, 0, 0, 0);
        }
    }
    // Window position of each accumulator row this lane holds: row 64rw+16mt+4kb+i.
    int wrow[kMT][4];
#pragma unroll
    for (int mt = 0; mt < kMT; ++mt)
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int r = kRowsPerWave * rw + 16 * mt + 4 * kb + i;
            wrow[mt][i] = (r < a.rows) ? r % a.W : -1;   // -1: padding row, sees nothing beyond the prefix
        }

    float m_run[kMT][4], z_run[kMT][4];   // STATS: running max / sum.  VOTES: m and 1/Z of the row.
#pragma unroll
    for (int mt = 0; mt < kMT; ++mt)
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            if (PASS == PASS_STATS) {
                m_run[mt][i] = kNegBig; z_run[mt][i] = 0.f;
            } else {
                const int r = kRowsPerWave * rw + 16 * mt + 4 * kb + i;
                const float2 st = a.stats[(size_t)head * a.rows_pad + r];
                m_run[mt][i] = st.x; z_run[mt][i] = (r < a.rows) ? st.y : 0.f;
            }
        }

    const int c_begin = blockIdx.x * a.chunks_per_wg;
    const int c_end = min(a.n_chunks, c_begin + a.chunks_per_wg);

    // The chunk after the one being computed is already on its way from HBM into registers;
    // it is parked in LDS only when every wave has finished reading the current one.
    constexpr int NPRE = CK * 16 / kThreads;
    typedef uint32_t u4v __attribute__((ext_vector_type(4)));
    u4v pre[NPRE];
    const int pre_row = threadIdx.x >> 4, pre_col = threadIdx.x & 15;   // item i of a thread: key row pre_row + 16 i
#define KVQP_ISSUE(chunk_)                                                                             \
    _Pragma("unroll") for (int i_ = 0; i_ < NPRE; ++i_) {                                              \
        const int key_ = min((chunk_) * CK + pre_row + 16 * i_, a.L - 1); /* rows past the end are masked */ \
        pre[i_] = *reinterpret_cast<const u4v*>(kh + (size_t)key_ * kHeadDim + pre_col * 8);        \
    }
#define KVQP_COMMIT()                                                                                  \
    _Pragma("unroll") for (int i_ = 0; i_ < NPRE; ++i_)                                                \
        *reinterpret_cast<u4v*>(sk + (pre_row + 16 * i_) * kKeyStride + pre_col * 16) = pre[i_];
    KVQP_ISSUE(min(c_begin, a.n_chunks - 1))
    KVQP_COMMIT()
    __syncthreads();

    for (int chunk = c_begin; chunk < c_end; ++chunk) {
        const int key0 = chunk * CK;
        KVQP_ISSUE(min(chunk + 1, c_end - 1))

        f4v acc[kMT][KT];
#pragma unroll
        for (int kt = 0; kt < KT; ++kt) {
            Frag kf[4];
            const unsigned char* kp = sk + (16 * (ks * KT + kt) + n) * kKeyStride + 16 * kb;
#pragma unroll
            for (int s = 0; s < 4; ++s) kf[s].q = *reinterpret_cast<const uint4*>(kp + 64 * s);
#pragma unroll
            for (int mt = 0; mt < kMT; ++mt) {
                f4v c = (f4v){0.f, 0.f, 0.f, 0.f};
#pragma unroll
                for (int s = 0; s < 4; ++s) c = __builtin_amdgcn_mfma_f32_16x16x32_f16(qf[mt][s].v, kf[s].v, c, 0, 0, 0);
                acc[mt][kt] = c;
            }
        }
        // causal mask only where the chunk reaches the window (raw scores; the scale is positive)
        if (key0 + CK > a.P) {
#pragma unroll
            for (int mt = 0; mt < kMT; ++mt)
#pragma unroll
                for (int kt = 0; kt < KT; ++kt)
#pragma unroll
                    for (int i = 0; i < 4; ++i) {
                        const int key = key0 + 16 * (ks * KT + kt) + n;
                        if (key > a.P + wrow[mt][i] || key >= a.L) acc[mt][kt][i] = -INFINITY;
                    }
        }

        if (PASS == PASS_STATS) {
#pragma unroll
            for (int mt = 0; mt < kMT; ++mt)
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    float raw = acc[mt][0][i];
#pragma unroll
                    for (int kt = 1; kt < KT; ++kt) raw = fmaxf(raw, acc[mt][kt][i]);
                    const float mx = fmaxf(m_run[mt][i], raw * a.scale_log2);   // log2-domain running maximum
                    float z = z_run[mt][i] * __builtin_amdgcn_exp2f(m_run[mt][i] - mx);
#pragma unroll
                    for (int kt = 0; kt < KT; ++kt) z += __builtin_amdgcn_exp2f(__builtin_fmaf(acc[mt][kt][i], a.scale_log2, -mx));
                    m_run[mt][i] = mx; z_run[mt][i] = z;
                }
            __syncthreads();                 // all waves are done with this chunk's keys
        } else {
            // normalised probabilities summed over this wave's 64 rows, per key
#pragma unroll
            for (int kt = 0; kt < KT; ++kt) {
                float col = 0.f;
#pragma unroll
                for (int mt = 0; mt < kMT; ++mt)
#pragma unroll
                    for (int i = 0; i < 4; ++i)
                        col = __builtin_fmaf(__builtin_amdgcn_exp2f(__builtin_fmaf(acc[mt][kt][i], a.scale_log2, -m_run[mt][i])),
                                             z_run[mt][i], col);
                // rows 4kb+i of all four lane quads
                col += __shfl_xor(col, 16);
                col += __shfl_xor(col, 32);
                if (kb == 0) svote[rw * CK + 16 * (ks * KT + kt) + n] = col;
            }
            __syncthreads();                 // votes of all row slabs parked; keys of this chunk consumed
            for (int kk = threadIdx.x; kk < CK; kk += kThreads) {
                float v = 0.f;
#pragma unroll
                for (int r = 0; r < NRW; ++r) v += svote[r * CK + kk];
                if (key0 + kk < a.P) a.vote[(size_t)head * a.P + key0 + kk] = v;
            }
        }
        KVQP_COMMIT()
        __syncthreads();
    }
#undef KVQP_ISSUE
#undef KVQP_COMMIT

    if (PASS == PASS_STATS) {
        // merge the 16 key columns a row is spread over, then one lane per row writes
#pragma unroll
        for (int mt = 0; mt < kMT; ++mt)
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                float m = m_run[mt][i], z = z_run[mt][i];
#pragma unroll
                for (int off = 1; off < 16; off <<= 1) {
                    const float mo = __shfl_xor(m, off), zo = __shfl_xor(z, off);
                    const float mn = fmaxf(m, mo);
                    z = z * __builtin_amdgcn_exp2f(m - mn) + zo * __builtin_amdgcn_exp2f(mo - mn);
                    m = mn;
                }
                if (n == 0) {
                    const int r = kRowsPerWave * rw + 16 * mt + 4 * kb + i;
                    a.stats_part[((size_t)head * a.n_parts + blockIdx.x * KS + ks) * a.rows_pad + r] = make_float2(m, z);
                }
            }
    }
}

// Merge the per-part row statistics; Z is accumulated in binary64.
__global__ void stats_combine(const float2* __restrict__ part, float2* __restrict__ stats, double* __restrict__ zsum,
                              int n_parts, int rows_pad) {
    const int head = blockIdx.x;
    for (int r = threadIdx.x; r < rows_pad; r += blockDim.x) {
        const float2* p = part + (size_t)head * n_parts * rows_pad + r;
        float M = kNegBig;
        for (int s = 0; s < n_parts; ++s) M = fmaxf(M, p[(size_t)s * rows_pad].x);
        double Z = 0.0;
        for (int s = 0; s < n_parts; ++s) {
            const float2 v = p[(size_t)s * rows_pad];
            Z += (double)v.y * (double)exp2f(v.x - M);
        }
        stats[(size_t)head * rows_pad + r] = make_float2(M, Z > 0.0 ? (float)(1.0 / Z) : 0.f);
        zsum[(size_t)head * rows_pad + r] = Z;
    }
}

// ---------------------------------------------------------------------------
// Selection: pool, find the cut with a radix select on the binary32 patterns,
// refine the candidates next to the cut in binary64, compact in position order.
// One workgroup per (batch, kv head); the data (<= a few hundred KB of scores)
// stays in L2.
// ---------------------------------------------------------------------------
constexpr int kSelThreads = 1024;
constexpr int kMaxBand = 512;         // candidates re-scored per head; beyond that binary32 decides
constexpr float kBandRel = 1.0e-4f;

struct SelectArgs {
    const float* vote;      // [heads, P]
    float* pooled;          // [heads, P]
    int32_t* idx;           // [heads, n_kept]
    const uint16_t* q_obs;
    const uint16_t* k;
    const float2* stats;    // (m, 1/Z) binary32
    const double* zsum;     // Z binary64
    int P, L, W, n_kept, pool, gq, n_q_heads, n_kv_heads, rows, rows_pad;
    float scale_log2;
    float sm_scale;
};

__device__ __forceinline__ uint32_t score_key(float v) { return __float_as_uint(v); }  // scores are >= 0: bits order like values

// Block-wide exclusive scan of one int per thread (kSelThreads threads).
__device__ int block_exclusive_scan(int v, int* total, int* swarp) {
    const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
    int inc = v;
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) {
        const int o = __shfl_up(inc, off);
        if (lane >= off) inc += o;
    }
    __syncthreads();
    if (lane == 63) swarp[w] = inc;
    __syncthreads();
    if (threadIdx.x == 0) {
        int run = 0;
        for (int i = 0; i < kSelThreads / 64; ++i) { const int t = swarp[i]; swarp[i] = run; run += t; }
        swarp[kSelThreads / 64] = run;
    }
    __syncthreads();
    *total = swarp[kSelThreads / 64];
    return swarp[w] + inc - v;
}

// binary64 vote of one prefix key: sum over the group's window rows of
// exp2(logit - m_r) / Z_r with exact products and the pass-1 statistics.
__device__ double vote_f64(const SelectArgs& a, int head, int key) {
    const int b = head / a.n_kv_heads, g = head % a.n_kv_heads;
    const uint16_t* kr = a.k + ((size_t)head * a.L + key) * kHeadDim;
    const int lane = threadIdx.x & 63;
    double acc = 0.0;
    for (int r = lane; r < a.rows; r += 64) {
        const int hl = r / a.W, i = r % a.W;
        const uint16_t* qr = a.q_obs + (((size_t)b * a.n_q_heads + g * a.gq + hl) * a.W + i) * kHeadDim;
        double s = 0.0;
        for (int d = 0; d < kHeadDim; ++d)
            s += (double)__half2float(__ushort_as_half(qr[d])) * (double)__half2float(__ushort_as_half(kr[d]));
        const double m = (double)a.stats[(size_t)head * a.rows_pad + r].x;
        acc += exp2(s * ((double)a.sm_scale * 1.4426950408889634074) - m) / a.zsum[(size_t)head * a.rows_pad + r];
    }
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) acc += __shfl_xor(acc, off);
    return acc;
}

__global__ __launch_bounds__(kSelThreads) void select_topk(const SelectArgs a) {
    __shared__ int hist[256];
    __shared__ int swarp[kSelThreads / 64 + 1];
    __shared__ uint32_t s_prefix;
    __shared__ int s_need, s_nband, s_sure;
    __shared__ int band_idx[kMaxBand];
    __shared__ double band_score[kMaxBand];
    __shared__ unsigned char band_take[kMaxBand];

    const int head = blockIdx.x;
    const int P = a.P, k = a.n_kept;
    const float* vote = a.vote + (size_t)head * P;
    float* pooled = a.pooled + (size_t)head * P;
    int32_t* idx = a.idx + (size_t)head * k;
    const int r = (a.pool - 1) / 2;

    if (k >= P) {  // budget covers the prefix: identity, no scores were computed
        for (int j = threadIdx.x; j < k; j += kSelThreads) idx[j] = j;
        return;
    }

    // ---- max-pool, clipped at both ends ----
    for (int j = threadIdx.x; j < P; j += kSelThreads) {
        float best = vote[j];
        for (int t = 1; t <= r; ++t) {
            if (j - t >= 0) best = fmaxf(best, vote[j - t]);
            if (j + t < P) best = fmaxf(best, vote[j + t]);
        }
        pooled[j] = best;
    }
    __syncthreads();

    // ---- radix select: bit pattern of the k-th largest pooled score ----
    if (threadIdx.x == 0) { s_prefix = 0u; s_need = k; }
    __syncthreads();
    for (int shift = 24; shift >= 0; shift -= 8) {
        if (threadIdx.x < 256) hist[threadIdx.x] = 0;
        __syncthreads();
        const uint32_t prefix = s_prefix;
        const uint32_t himask = (shift == 24) ? 0u : (0xffffffffu << (shift + 8));
        for (int j = threadIdx.x; j < P; j += kSelThreads) {
            const uint32_t key = score_key(pooled[j]);
            if ((key & himask) == prefix) atomicAdd(&hist[(key >> shift) & 255], 1);
        }
        __syncthreads();
        if (threadIdx.x == 0) {
            int need = s_need, bin = 255;
            for (; bin > 0; --bin) {
                if (hist[bin] >= need) break;
                need -= hist[bin];
            }
            s_need = need;                      // how many of this bin (and, at the end, of the cut value) are taken
            s_prefix = prefix | ((uint32_t)bin << shift);
        }
        __syncthreads();
    }
    const float cut = __uint_as_float(s_prefix);
    // band of scores that binary32 rounding could move across the cut
    const float lo = cut * (1.0f - kBandRel), hi = cut * (1.0f + kBandRel);

    // ---- collect the band (position order) and count the sure survivors ----
    int my_band = 0, my_sure = 0;
    const int per = (P + kSelThreads - 1) / kSelThreads;
    const int j0 = threadIdx.x * per, j1 = min(P, j0 + per);
    for (int j = j0; j < j1; ++j) {
        const float v = pooled[j];
        my_sure += (v > hi);
        my_band += (v >= lo && v <= hi);
    }
    int tot_band, tot_sure;
    const int band_off = block_exclusive_scan(my_band, &tot_band, swarp);
    (void)block_exclusive_scan(my_sure, &tot_sure, swarp);
    const bool refine = tot_band <= kMaxBand;
    if (refine) {
        int o = band_off;
        for (int j = j0; j < j1; ++j) {
            const float v = pooled[j];
            if (v >= lo && v <= hi) band_idx[o++] = j;
        }
    }
    __syncthreads();

    if (refine) {
        // ---- binary64 re-scoring of the band: one wave per candidate ----
        const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
        for (int c = wave; c < tot_band; c += kSelThreads / 64) {
            const int j = band_idx[c];
            double best = -1.0;
            for (int t = -r; t <= r; ++t) {
                if (j + t < 0 || j + t >= P) continue;
                const double v = vote_f64(a, head, j + t);
                best = v > best ? v : best;
            }
            if (lane == 0) band_score[c] = best;
        }
        __syncthreads();
        // rank inside the band by (score desc, position asc); band_idx is ascending
        const int take = k - tot_sure;
        for (int c = threadIdx.x; c < tot_band; c += kSelThreads) {
            const double sc = band_score[c];
            int rank = 0;
            for (int o = 0; o < tot_band; ++o) rank += (band_score[o] > sc) || (band_score[o] == sc && o < c);
            band_take[c] = rank < take;
        }
        __syncthreads();
    }

    // ---- ordered compaction ----
    int my_keep = 0;
    if (refine) {
        int bo = band_off;
        for (int j = j0; j < j1; ++j) {
            const float v = pooled[j];
            if (v > hi) ++my_keep;
            else if (v >= lo) my_keep += band_take[bo++];
        }
    } else {
        // binary32 decides: everything above the cut, then the first s_need equal to it
        int my_eq = 0;
        for (int j = j0; j < j1; ++j) my_eq += (pooled[j] == cut);
        int tot_eq;
        int eq_off = block_exclusive_scan(my_eq, &tot_eq, swarp);
        const int need = s_need;
        for (int j = j0; j < j1; ++j) {
            const float v = pooled[j];
            if (v > cut) ++my_keep;
            else if (v == cut) my_keep += (eq_off++ < need);
        }
    }
    int tot_keep;
    int out = block_exclusive_scan(my_keep, &tot_keep, swarp);
    if (refine) {
        int bo = band_off;
        for (int j = j0; j < j1; ++j) {
            const float v = pooled[j];
            bool keep = v > hi;
            if (!keep && v >= lo) keep = band_take[bo++];
            if (keep && out < k) idx[out++] = j;
        }
    } else {
        int my_eq = 0;
        for (int j = j0; j < j1; ++j) my_eq += (pooled[j] == cut);
        int tot_eq;
        int eq_off = block_exclusive_scan(my_eq, &tot_eq, swarp);
        const int need = s_need;
        for (int j = j0; j < j1; ++j) {
            const float v = pooled[j];
            bool keep = v > cut;
            if (!keep && v == cut) keep = (eq_off++ < need);
            if (keep && out < k) idx[out++] = j;
        }
    }
}

size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

int n_row_slabs(const kvqp_cfg& cfg) {
    const int rows = (cfg.n_q_heads / cfg.n_kv_heads) * cfg.window;
    const int slabs = (rows + kRowsPerWave - 1) / kRowsPerWave;
    return slabs <= 1 ? 1 : slabs == 2 ? 2 : 4;
}

template <int NRW>
hipError_t launch_scores(const ScoreArgs& a, int n_wg, int heads, hipStream_t stream, float2* stats, double* zsum) {
    ScoreArgs s1 = a;
    hipLaunchKernelGGL((score_pass<NRW, PASS_STATS>), dim3(n_wg, heads), dim3(kThreads), 0, stream, s1);
    hipLaunchKernelGGL(stats_combine, dim3(heads), dim3(256), 0, stream, (const float2*)a.stats_part, stats, zsum,
                       a.n_parts, a.rows_pad);
    hipLaunchKernelGGL((score_pass<NRW, PASS_VOTES>), dim3(n_wg, heads), dim3(kThreads), 0, stream, s1);
    return hipGetLastError();
}

}  // namespace

CompressPlan plan_compress(const kvqp_cfg& cfg) {
    CompressPlan p{};
    p.P = cfg.seq_len - cfg.window;
    p.n_kept = cfg.budget < p.P ? cfg.budget : p.P;
    p.rows = (cfg.n_q_heads / cfg.n_kv_heads) * cfg.window;
    const int nrw = n_row_slabs(cfg);
    const int rows_pad = nrw * kRowsPerWave;
    const int ks = 4 / nrw, ck = (ks == 1) ? 64 : 128;
    const int heads = cfg.batch * cfg.n_kv_heads;
    p.n_chunks = (cfg.seq_len + ck - 1) / ck;
    // enough workgroups to fill the chip a few times over, at least 2 chunks each
    int n_wg = (2048 + heads - 1) / heads;
    if (n_wg > (p.n_chunks + 1) / 2) n_wg = (p.n_chunks + 1) / 2;
    if (n_wg < 1) n_wg = 1;
    p.chunks_per_wg = (p.n_chunks + n_wg - 1) / n_wg;
    p.n_wg = (p.n_chunks + p.chunks_per_wg - 1) / p.chunks_per_wg;
    p.n_row_slabs = nrw;
    const size_t n_parts = (size_t)p.n_wg * ks;
    size_t off = 0;
    p.off_stats_part = off; off = align_up(off + (size_t)heads * n_parts * rows_pad * sizeof(float2), 256);
    p.off_stats = off;      off = align_up(off + (size_t)heads * rows_pad * (sizeof(float2) + sizeof(double)), 256);
    p.off_vote = off;       off = align_up(off + (size_t)heads * (p.P > 0 ? p.P : 1) * sizeof(float), 256);
    p.off_pooled = off;     off = align_up(off + (size_t)heads * (p.P > 0 ? p.P : 1) * sizeof(float), 256);
    p.off_sel = off;
    p.off_idx = off;        off = align_up(off + (size_t)heads * (p.n_kept > 0 ? p.n_kept : 1) * sizeof(int32_t), 256);
    p.total = off;
    return p;
}

hipError_t launch_select(const kvqp_cfg& cfg, const void* q_obs, const void* k, int32_t* idx, void* ws,
                         const CompressPlan& plan, hipStream_t stream) {
    char* base = static_cast<char*>(ws);
    const int heads = cfg.batch * cfg.n_kv_heads;
    const int nrw = plan.n_row_slabs;
    const int ks = 4 / nrw;
    const int n_wg = plan.n_wg, cpw = plan.chunks_per_wg;

    ScoreArgs a;
    a.q_obs = (const uint16_t*)q_obs; a.k = (const uint16_t*)k;
    a.stats_part = reinterpret_cast<float2*>(base + plan.off_stats_part);
    float2* stats = reinterpret_cast<float2*>(base + plan.off_stats);
    a.rows = plan.rows; a.rows_pad = nrw * kRowsPerWave;
    double* zsum = reinterpret_cast<double*>(base + plan.off_stats + (size_t)heads * a.rows_pad * sizeof(float2));
    a.stats = stats;
    a.vote = reinterpret_cast<float*>(base + plan.off_vote);
    a.L = cfg.seq_len; a.W = cfg.window; a.P = plan.P; a.gq = cfg.n_q_heads / cfg.n_kv_heads;
    a.n_q_heads = cfg.n_q_heads; a.n_kv_heads = cfg.n_kv_heads;
    a.chunks_per_wg = cpw; a.n_chunks = plan.n_chunks; a.n_parts = n_wg * ks;
    a.scale_log2 = cfg.sm_scale * kLog2e;

    hipError_t e;
    if (plan.n_kept < plan.P) {   // scores are needed only when something is dropped
        switch (nrw) {
            case 1: e = launch_scores<1>(a, n_wg, heads, stream, stats, zsum); break;
            case 2: e = launch_scores<2>(a, n_wg, heads, stream, stats, zsum); break;
            default: e = launch_scores<4>(a, n_wg, heads, stream, stats, zsum); break;
        }
        if (e != hipSuccess) return e;
    }
    SelectArgs s;
    s.vote = a.vote; s.pooled = reinterpret_cast<float*>(base + plan.off_pooled); s.idx = idx;
    s.q_obs = a.q_obs; s.k = a.k; s.stats = stats; s.zsum = zsum;
    s.P = plan.P; s.L = cfg.seq_len; s.W = cfg.window; s.n_kept = plan.n_kept; s.pool = cfg.pool_kernel;
    s.gq = a.gq; s.n_q_heads = cfg.n_q_heads; s.n_kv_heads = cfg.n_kv_heads; s.rows = a.rows; s.rows_pad = a.rows_pad;
    s.scale_log2 = a.scale_log2; s.sm_scale = cfg.sm_scale;
    hipLaunchKernelGGL(select_topk, dim3(heads), dim3(kSelThreads), 0, stream, s);
    return hipGetLastError();
}

}  // namespace kvqp
