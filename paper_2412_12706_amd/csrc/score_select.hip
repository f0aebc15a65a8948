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
//   score_pass<STATS>  a reference and the exp-sum of every window row (pass 1)
//   stats_combine      merges the per-wave row statistics
//   score_pass<VOTES>  recomputes the tiles, normalises, sums columns (pass 2)
//   select_topk        pool, radix-select the cut, ordered compaction; scores
//                      within a relative 2e-5 of the cut are first re-scored in
//                      binary64 so that binary32 rounding cannot move the cut
// Keys stream through LDS once per pass in 64- or 128-key chunks shared by the
// four waves of a workgroup; query rows stay in registers as MFMA operands.
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
// Query rows one wave owns (its MFMA A operands, register-resident): 32 when the group has up to
// 128 window rows (small register footprint, four waves per SIMD), else 64.
constexpr int rows_per_wave(int rows) { return rows <= 128 ? 32 : 64; }
constexpr int kKeyStride = kHeadDim * 2 + 16;  // LDS bytes per key row; +16 B skews banks
constexpr float kLog2e = 1.4426950408889634f;
constexpr float kNegBig = -1.0e30f;
constexpr float kLazy = 8.0f;           // pass 1 moves a row's reference only when a score beats it by 2^8

enum { PASS_STATS = 0, PASS_VOTES = 1 };

struct ScoreArgs {
    const uint16_t* q_obs;  // [B, Hq, W, D]
    const uint16_t* k;      // [B, Hkv, L, D]
    float2* stats_part;     // [heads, n_parts, rows_pad]  (m, Z) in the log2 domain
    const float2* stats;    // [heads, rows_pad]           (m, 1/Z)
    float* vote;            // [heads, P]
    int L, W, P, gq, n_q_heads, n_kv_heads;
    int rows, rows_pad;     // Gq*W and the rows the waves cover (a multiple of 32 or 64)
    int chunks_per_wg, n_chunks, n_parts;
    float scale_log2;       // sm_scale * log2(e)
};

// NRW = number of row slabs (1, 2, 4) of RPW rows; the 4 waves are NRW row slabs x KS key strips.
template <int NRW> struct ScoreGeom {
    static constexpr int KS = 4 / NRW;
    static constexpr int CK = (KS == 1) ? 64 : 128;   // keys per chunk
    static constexpr int KT = CK / (16 * KS);         // key tiles per wave per chunk
};

template <int RPW, int NRW, int PASS>
__global__ __launch_bounds__(kThreads, RPW == 32 ? 4 : 2) void score_pass(const ScoreArgs a) {
    constexpr int kRowsPerWave = RPW, kMT = RPW / 16;
    using Gm = ScoreGeom<NRW>;
    constexpr int KS = Gm::KS, CK = Gm::CK, KT = Gm::KT;
    __shared__ __align__(16) unsigned char sk[CK * kKeyStride];
    __shared__ float svote[(PASS == PASS_VOTES) ? NRW * CK : 1];

    const int head = blockIdx.y;
    const int b = head / a.n_kv_heads, g = head % a.n_kv_heads;
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);   // scalar: tile positions stay uniform
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
    float m_run[kMT][4], z_run[kMT][4];   // STATS: reference (log2 domain) and sum of exp2(score - reference).  VOTES: m and 1/Z of the row.
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
        const u4v* src_ = reinterpret_cast<const u4v*>(kh + (size_t)key_ * kHeadDim + pre_col * 8);    \
        pre[i_] = (PASS == PASS_VOTES) ? __builtin_nontemporal_load(src_) : *src_; /* last read of a key: streamed */ \
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

        // one 16-key tile at a time keeps the accumulators at 16 registers
#pragma unroll
        for (int kt = 0; kt < KT; ++kt) {
            Frag kf[4];
            const unsigned char* kp = sk + (16 * (ks * KT + kt) + n) * kKeyStride + 16 * kb;
#pragma unroll
            for (int s = 0; s < 4; ++s) kf[s].q = *reinterpret_cast<const uint4*>(kp + 64 * s);
            f4v acc[kMT];
#pragma unroll
            for (int mt = 0; mt < kMT; ++mt) {
                f4v c = (f4v){0.f, 0.f, 0.f, 0.f};
#pragma unroll
                for (int s = 0; s < 4; ++s) c = __builtin_amdgcn_mfma_f32_16x16x32_f16(qf[mt][s].v, kf[s].v, c, 0, 0, 0);
                acc[mt] = c;
            }
            // causal mask only where the tile reaches the window (raw scores; the scale is positive)
            const int tile0 = key0 + 16 * (ks * KT + kt);
            if (tile0 + 16 > a.P) {
                const int key = tile0 + n;
                int w = a.W;
                asm volatile("" : "+s"(w));   // keeps the window positions out of the loop's live registers
#pragma unroll
                for (int mt = 0; mt < kMT; ++mt)
#pragma unroll
                    for (int i = 0; i < 4; ++i) {
                        const int r = kRowsPerWave * rw + 16 * mt + 4 * kb + i;
                        const int wr = (r < a.rows) ? r % w : -1;   // padding rows see the prefix only
                        if (key > a.P + wr || key >= a.L) acc[mt][i] = -INFINITY;
                    }
            }
            if (PASS == PASS_STATS) {
                // m_run is a reference, not the exact maximum: it moves only when a score beats it
                // by more than 2^kLazy, so the common path is one fused multiply-add and one exp2
                float e[kMT][4];
                float big = -INFINITY;
#pragma unroll
                for (int mt = 0; mt < kMT; ++mt)
#pragma unroll
                    for (int i = 0; i < 4; ++i) {
                        e[mt][i] = __builtin_fmaf(acc[mt][i], a.scale_log2, -m_run[mt][i]);
                        big = fmaxf(big, e[mt][i]);
                    }
                if (__builtin_amdgcn_ballot_w64(big > kLazy) != 0ull) {   // rare after the first tiles
#pragma unroll
                    for (int mt = 0; mt < kMT; ++mt)
#pragma unroll
                        for (int i = 0; i < 4; ++i) {
                            const float sc = acc[mt][i] * a.scale_log2;
                            if (sc > m_run[mt][i]) {
                                z_run[mt][i] *= __builtin_amdgcn_exp2f(m_run[mt][i] - sc);
                                m_run[mt][i] = sc;
                            }
                            e[mt][i] = __builtin_fmaf(acc[mt][i], a.scale_log2, -m_run[mt][i]);
                        }
                }
#pragma unroll
                for (int mt = 0; mt < kMT; ++mt)
#pragma unroll
                    for (int i = 0; i < 4; ++i) z_run[mt][i] += __builtin_amdgcn_exp2f(e[mt][i]);
            } else {
                // normalised probabilities summed over this wave's 64 rows, per key
                float c0 = 0.f, c1 = 0.f;
#pragma unroll
                for (int mt = 0; mt < kMT; ++mt)
#pragma unroll
                    for (int i = 0; i < 4; i += 2) {
                        c0 = __builtin_fmaf(__builtin_amdgcn_exp2f(__builtin_fmaf(acc[mt][i], a.scale_log2, -m_run[mt][i])),
                                            z_run[mt][i], c0);
                        c1 = __builtin_fmaf(__builtin_amdgcn_exp2f(__builtin_fmaf(acc[mt][i + 1], a.scale_log2, -m_run[mt][i + 1])),
                                            z_run[mt][i + 1], c1);
                    }
                float col = c0 + c1;
                // rows 4kb+i of all four lane quads
                col += __shfl_xor(col, 16);
                col += __shfl_xor(col, 32);
                if (kb == 0) svote[rw * CK + 16 * (ks * KT + kt) + n] = col;
            }
        }
        __syncthreads();                 // all waves are done with this chunk's keys (and votes are parked)
        if (PASS == PASS_VOTES) {
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

// Merge the per-part row statistics; Z is accumulated in binary64.  One wave per row (four rows
// per workgroup): lanes stride over the parts, then a fixed-order butterfly.
__global__ __launch_bounds__(256) void stats_combine(const float2* __restrict__ part, float2* __restrict__ stats,
                                                     double* __restrict__ zsum, int n_parts, int rows_pad) {
    const int head = blockIdx.x;
    const int lane = threadIdx.x & 63;
    const int r = 4 * blockIdx.y + (threadIdx.x >> 6);
    if (r >= rows_pad) return;
    const float2* p = part + (size_t)head * n_parts * rows_pad + r;
    float M = kNegBig;
    for (int s = lane; s < n_parts; s += 64) M = fmaxf(M, p[(size_t)s * rows_pad].x);
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) M = fmaxf(M, __shfl_xor(M, off));
    double Z = 0.0;
    for (int s = lane; s < n_parts; s += 64) {
        const float2 v = p[(size_t)s * rows_pad];
        Z += (double)v.y * (double)exp2f(v.x - M);
    }
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) Z += __shfl_xor(Z, off);
    if (lane == 0) {
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
constexpr int kSelWaves = kSelThreads / 64;
constexpr int kMaxRows = 128;         // rows of 1024 candidates: prefixes up to 131072 tokens
constexpr int kRegRows = 32;          // rows whose pooled scores stay in registers (prefixes up to 32768)
constexpr int kMaxBand = 512;         // candidates re-scored per head; beyond that binary32 decides (and the caller is told)
constexpr int kVoteSlots = 2048;       // binary64 votes (distinct positions) held in LDS during the re-scoring
constexpr int kStageRows = 4;          // rows of votes staged in LDS per pooling step
constexpr int kMaxPoolRadius = 31;     // pool_kernel <= 63
constexpr float kBandRel = 2.0e-5f;   // >> the binary32 error of a vote (a few 1e-7 relative)

struct SelectArgs {
    const float* vote;      // [heads, P]
    float* pooled;          // [heads, P]
    int32_t* idx;           // [heads, n_kept]
    int32_t* unrefined;     // [heads] or NULL: candidates near the cut that binary32 decided (0: all re-scored)
    const int32_t* head_n;  // a head's own cut (<= n_kept), or NULL for n_kept everywhere
    const uint16_t* q_obs;
    const uint16_t* k;
    const float2* stats;    // (m, 1/Z) binary32
    const double* zsum;     // Z binary64
    int P, L, W, n_kept, pool, gq, n_q_heads, n_kv_heads, rows, rows_pad;
    float scale_log2;
    float sm_scale;
};

__device__ __forceinline__ uint32_t score_key(float v) { return __float_as_uint(v); }  // scores are >= 0: bits order like values

// Exclusive scan, in place, of a table of n <= 2 * kSelThreads ints in LDS; returns the total.
__device__ int scan_table(int* tab, int n, int* swave) {
    const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
    const int e0 = 2 * threadIdx.x, e1 = e0 + 1;
    const int v0 = e0 < n ? tab[e0] : 0, v1 = e1 < n ? tab[e1] : 0;
    int inc = v0 + v1;
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) {
        const int o = __shfl_up(inc, off);
        if (lane >= off) inc += o;
    }
    __syncthreads();
    if (lane == 63) swave[w] = inc;
    __syncthreads();
    int base = 0, total = 0;
#pragma unroll
    for (int i = 0; i < kSelWaves; ++i) {
        const int t = swave[i];
        if (i < w) base += t;
        total += t;
    }
    const int excl = base + inc - (v0 + v1);
    if (e0 < n) tab[e0] = excl;
    if (e1 < n) tab[e1] = excl + v0;
    __syncthreads();
    return total;
}

__device__ __forceinline__ float half_lo(uint32_t w) { return __half2float(__ushort_as_half((uint16_t)(w & 0xffffu))); }
__device__ __forceinline__ float half_hi(uint32_t w) { return __half2float(__ushort_as_half((uint16_t)(w >> 16))); }

// Part of the binary64 vote of one prefix key, computed by one wave: the sum over 32 of the group's
// window rows (row_base + lane/2; the two lanes of a row split the channels) of
// exp2(logit - m_r) / Z_r with the pass-1 statistics.  A product of two binary16 values is exact in
// binary32; the products are summed in binary64.
__device__ double vote_f64_part(const SelectArgs& a, int head, int key, int row_base) {
    const int b = head / a.n_kv_heads, g = head % a.n_kv_heads;
    const int lane = threadIdx.x & 63, half = lane & 1;
    const int r = row_base + (lane >> 1);
    const bool live = r < a.rows;
    const int rc = live ? r : 0;
    const int hl = rc / a.W, i = rc % a.W;
    const uint4* kr = reinterpret_cast<const uint4*>(a.k + ((size_t)head * a.L + key) * kHeadDim) + 8 * half;
    const uint4* qr = reinterpret_cast<const uint4*>(a.q_obs + (((size_t)b * a.n_q_heads + g * a.gq + hl) * a.W + i) * kHeadDim) + 8 * half;
    const double m = (double)a.stats[(size_t)head * a.rows_pad + rc].x;
    const double z = a.zsum[(size_t)head * a.rows_pad + rc];
    double s0 = 0.0, s1 = 0.0;
#pragma unroll
    for (int c0 = 0; c0 < 8; c0 += 4) {
        uint4 qv[4], kv[4];
#pragma unroll
        for (int c = 0; c < 4; ++c) { qv[c] = qr[c0 + c]; kv[c] = kr[c0 + c]; }
#pragma unroll
        for (int c = 0; c < 4; ++c) {
            const uint32_t qw[4] = {qv[c].x, qv[c].y, qv[c].z, qv[c].w}, kw[4] = {kv[c].x, kv[c].y, kv[c].z, kv[c].w};
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                s0 += (double)(half_lo(qw[e]) * half_lo(kw[e]));
                s1 += (double)(half_hi(qw[e]) * half_hi(kw[e]));
            }
        }
    }
    double s = s0 + s1;
    s += __shfl_xor(s, 1);
    double acc = (live && half == 0) ? exp2(s * ((double)a.sm_scale * 1.4426950408889634074) - m) / z : 0.0;
#pragma unroll
    for (int off = 32; off >= 2; off >>= 1) acc += __shfl_xor(acc, off);
    return acc;
}

// Visit every candidate of this thread: j = row * 1024 + thread, v = its pooled score (-1 past the
// end).  The first kRegRows rows come from registers, the rest from the pooled array.
#define KVQP_FOR_ROWS(...)                                                            \
    _Pragma("unroll") for (int row = 0; row < kRegRows; ++row) {                      \
        if (row < n_rows) {                                                           \
            const int j = row * kSelThreads + (int)threadIdx.x;                       \
            const float v = pv[row];                                                  \
            __VA_ARGS__                                                               \
        }                                                                             \
    }                                                                                 \
    for (int row = kRegRows; row < n_rows; ++row) {                                   \
        const int j = row * kSelThreads + (int)threadIdx.x;                           \
        const float v = j < P ? pooled[j] : -1.0f;                                    \
        __VA_ARGS__                                                                   \
    }

// One workgroup per (batch, kv head).  Candidate j lives at (row j / 1024, thread j % 1024), so
// every sweep is coalesced and "position order" is (row, wave, lane): ordered compaction needs only
// per-(row, wave) counts (one ballot each), one table scan, and a popcount below the lane.  The
// pooled scores of prefixes up to 32768 tokens never leave the registers.
__global__ __launch_bounds__(kSelThreads) void select_topk(const SelectArgs a) {
    __shared__ __align__(16) int hist[kSelWaves][256];   // later reused for the binary64 partial votes (2048 doubles)
    __shared__ int tab_a[kMaxRows * kSelWaves];   // per (row, wave): survivors that need no second look
    __shared__ int tab_b[kMaxRows * kSelWaves];   // per (row, wave): band members (or ties at the cut)
    __shared__ int swave[kSelWaves];
    __shared__ uint32_t s_red[2 * kSelWaves];
    __shared__ uint32_t s_prefix;
    __shared__ int s_need;
    __shared__ int band_idx[kMaxBand];
    __shared__ int band_start[kMaxBand];          // first position whose vote this member owns
    __shared__ int band_off[kMaxBand + 1];        // offset of its owned votes in the vote list
    __shared__ double band_score[kMaxBand];
    __shared__ int band_take[kMaxBand + 1];       // after the scan: taken band members before position c
    __shared__ __align__(16) float stage[kStageRows * kSelThreads + 2 * kMaxPoolRadius];   // votes of a few rows plus halo; later the binary64 votes

    const int head = blockIdx.x;
    const int P = a.P, k = a.head_n ? a.head_n[head] : a.n_kept;
    const float* vote = a.vote + (size_t)head * P;
    float* pooled = a.pooled + (size_t)head * P;
    int32_t* idx = a.idx + (size_t)head * a.n_kept;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int n_rows = (P + kSelThreads - 1) / kSelThreads;
    const unsigned long long lt_mask = (1ull << lane) - 1ull;

    if (a.unrefined && threadIdx.x == 0) a.unrefined[head] = 0;   // (overwritten below by the same thread if binary32 decides)
    if (k <= 0) return;   // (a head-level count may be zero)
    if (k >= P) {  // budget covers the prefix: identity, the scores are not looked at
        for (int j = threadIdx.x; j < k; j += kSelThreads) idx[j] = j;
        return;
    }

    // ---- max-pool (clipped at both ends) and the range of the pooled scores ----
    const int r = (a.pool - 1) / 2;
    uint32_t kmin = 0xffffffffu, kmax = 0u;
    float pv[kRegRows];
#pragma unroll
    for (int row = 0; row < kRegRows; ++row) pv[row] = -1.0f;
    // A step stages kStageRows * 1024 consecutive votes plus r on either side in LDS (-1, below any
    // vote, outside the prefix); every thread then takes the maximum over its window per row.  The
    // votes of the next step are requested before this step's are pooled, so only the first step
    // waits for memory.
    float nx[kStageRows + 1];
    auto fetch = [&](int row0) {
        const int base = row0 * kSelThreads - r;
#pragma unroll
        for (int u = 0; u <= kStageRows; ++u) {
            const int i = (int)threadIdx.x + u * kSelThreads, j = base + i;
            nx[u] = (i < kStageRows * kSelThreads + 2 * r && j >= 0 && j < P) ? vote[j] : -1.0f;
        }
    };
#define KVQP_POOL_STEP(ROW0, STORE)                                                                \
    {                                                                                              \
        _Pragma("unroll") for (int u = 0; u <= kStageRows; ++u) {                                  \
            const int i = (int)threadIdx.x + u * kSelThreads;                                      \
            if (i < kStageRows * kSelThreads + 2 * r) stage[i] = nx[u];                            \
        }                                                                                          \
        __syncthreads();                                                                           \
        if ((ROW0) + kStageRows < n_rows) fetch((ROW0) + kStageRows);                              \
        _Pragma("unroll") for (int q = 0; q < kStageRows; ++q) {                                   \
            const int row = (ROW0) + q;                                                            \
            const int j = row * kSelThreads + (int)threadIdx.x;                                    \
            if (j < P) {                                                                           \
                const float* w = stage + q * kSelThreads + threadIdx.x;                            \
                float best = w[0];                                                                 \
                for (int t = 1; t <= 2 * r; ++t) best = fmaxf(best, w[t]);                         \
                STORE;                                                                             \
                kmin = min(kmin, score_key(best)); kmax = max(kmax, score_key(best));              \
            }                                                                                      \
        }                                                                                          \
        __syncthreads();                                                                           \
    }
    fetch(0);
#pragma unroll
    for (int row0 = 0; row0 < kRegRows; row0 += kStageRows)
        if (row0 < n_rows) KVQP_POOL_STEP(row0, pv[row] = best)
    for (int row0 = kRegRows; row0 < n_rows; row0 += kStageRows) KVQP_POOL_STEP(row0, pooled[j] = best)
#undef KVQP_POOL_STEP
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) {
        kmin = min(kmin, (uint32_t)__shfl_xor((int)kmin, off));
        kmax = max(kmax, (uint32_t)__shfl_xor((int)kmax, off));
    }
    if (lane == 0) { s_red[wave] = kmin; s_red[kSelWaves + wave] = kmax; }
    __syncthreads();   // also orders the pooled[] writes before the sweeps below (same workgroup)
    kmin = s_red[0]; kmax = s_red[kSelWaves];
#pragma unroll
    for (int i = 1; i < kSelWaves; ++i) { kmin = min(kmin, s_red[i]); kmax = max(kmax, s_red[kSelWaves + i]); }

    // ---- radix select of the k-th largest score, on keys relative to the minimum so that the
    // digits that all candidates share (sign, exponent) do not pile into one histogram bin ----
    const uint32_t span = kmax - kmin;
    int top_shift = 24;
    while (top_shift > 0 && (span >> top_shift) == 0) top_shift -= 8;
    if (threadIdx.x == 0) { s_prefix = 0u; s_need = k; }
    for (int shift = top_shift; shift >= 0; shift -= 8) {
        for (int i = threadIdx.x; i < kSelWaves * 256; i += kSelThreads) (&hist[0][0])[i] = 0;
        __syncthreads();
        // (scalar copies: nothing in the sweep below then waits on LDS, so its atomics overlap)
        const uint32_t prefix = __builtin_amdgcn_readfirstlane(s_prefix);
        const int need = __builtin_amdgcn_readfirstlane(s_need);
        const uint32_t himask = (shift == 24) ? 0u : (0xffffffffu << (shift + 8));
        KVQP_FOR_ROWS(
            const uint32_t key = score_key(v) - kmin;
            const bool act = j < P && (key & himask) == prefix;
            const int bin = (key >> shift) & 255;
            // (an LDS atomic costs the CU a fixed time even with no lane active: skip those)
            if (__builtin_amdgcn_ballot_w64(act) != 0ull)
                if (act) atomicAdd(&hist[wave][bin], 1);
        )
        __syncthreads();
        // bins summed over the waves, then "how many candidates in bins above mine" per bin
        if (wave < 4) {
            const int bin = threadIdx.x;                  // 256 threads, one bin each
            int c = 0;
#pragma unroll
            for (int w = 0; w < kSelWaves; ++w) c += hist[w][bin];
            // suffix sum within the wave (bins descend with rank), then across the four waves
            int suf = c;
#pragma unroll
            for (int off = 1; off < 64; off <<= 1) {
                const int o = __shfl_down(suf, off);
                if (lane + off < 64) suf += o;
            }
            if (lane == 0) swave[wave] = suf;             // total of this wave's 64 bins
            hist[0][bin] = c;                             // (own column only: no other thread reads hist[0][bin])
            tab_a[bin] = suf;
        }
        __syncthreads();
        if (wave < 4) {
            const int bin = threadIdx.x;
            int above = tab_a[bin] - hist[0][bin];        // candidates in higher bins of this wave's 64
            for (int w = wave + 1; w < 4; ++w) above += swave[w];
            if (above < need && above + hist[0][bin] >= need) {   // exactly one bin satisfies this
                s_need = need - above;
                s_prefix = prefix | ((uint32_t)bin << shift);
            }
        }
        __syncthreads();
    }
    const float cut = __uint_as_float(s_prefix + kmin);
    const int need_at_cut = s_need;   // how many candidates equal to the cut are taken (binary32 rule)
    // band of scores that binary32 rounding could move across the cut
    const float lo = cut * (1.0f - kBandRel), hi = cut * (1.0f + kBandRel);

    // ---- per-(row, wave) counts: sure survivors (> hi) and band members ----
    KVQP_FOR_ROWS(
        const unsigned long long bs = __builtin_amdgcn_ballot_w64(v > hi);
        const unsigned long long bb = __builtin_amdgcn_ballot_w64(v >= lo && v <= hi);
        if (lane == 0) { tab_a[row * kSelWaves + wave] = __popcll(bs); tab_b[row * kSelWaves + wave] = __popcll(bb); }
        (void)j;
    )
    __syncthreads();
    const int tot_sure = scan_table(tab_a, n_rows * kSelWaves, swave);
    const int tot_band = scan_table(tab_b, n_rows * kSelWaves, swave);
    const int n_parts = (a.rows + 31) / 32;       // a wave re-scores 32 window rows of one position
    bool refine = tot_band <= kMaxBand;
    double* part_vote = reinterpret_cast<double*>(&hist[0][0]);   // kVoteSlots partial votes of a batch of positions
    double* pos_vote = reinterpret_cast<double*>(&stage[0]);        // kVoteSlots votes, one per distinct position
    int n_pos = 0;

    if (refine) {
        // ---- band members in position order ----
        KVQP_FOR_ROWS(
            const bool inb = v >= lo && v <= hi;
            const unsigned long long bb = __builtin_amdgcn_ballot_w64(inb);
            if (inb) band_idx[tab_b[row * kSelWaves + wave] + __popcll(bb & lt_mask)] = j;
        )
        __syncthreads();
        // ---- the positions whose votes are needed, each once: member c owns those of its pool
        // window that no earlier member's window covers ----
        for (int c = threadIdx.x; c < tot_band; c += kSelThreads) {
            const int jc = band_idx[c];
            int st = jc - r > 0 ? jc - r : 0;
            if (c > 0) st = max(st, band_idx[c - 1] + r + 1);
            const int en = min(jc + r, P - 1);
            band_start[c] = st;
            band_off[c] = en >= st ? en - st + 1 : 0;
        }
        __syncthreads();
        if (threadIdx.x == 0) {   // exclusive prefix over at most kMaxBand counts
            int run = 0;
            for (int c = 0; c < tot_band; ++c) { const int t = band_off[c]; band_off[c] = run; run += t; }
            band_off[tot_band] = run;
        }
        __syncthreads();
        n_pos = band_off[tot_band];
        refine = n_pos <= kVoteSlots;
    }
    if (refine) {
        // ---- binary64 re-scoring: one wave per (position, 32 window rows); the parts of a position land
        // in the histogram's LDS and are summed in ascending order into the position's vote, which is kept
        // in the pooling stage's LDS (both are free by now).  Positions go in batches that fit the parts. ----
        const int batch = kVoteSlots / n_parts;           // positions per batch (n_parts <= 8)
        for (int p0 = 0; p0 < n_pos; p0 += batch) {
            const int np = min(batch, n_pos - p0);
            for (int item = wave; item < np * n_parts; item += kSelWaves) {
                const int pos = p0 + item / n_parts, part = item % n_parts;
                int lo_c = 0, hi_c = tot_band - 1;           // owner: last member with band_off <= pos
                while (lo_c < hi_c) {
                    const int mid = (lo_c + hi_c + 1) >> 1;
                    if (band_off[mid] <= pos) lo_c = mid; else hi_c = mid - 1;
                }
                const int j = band_start[lo_c] + (pos - band_off[lo_c]);
                const double v = vote_f64_part(a, head, j, 32 * part);
                if (lane == 0) part_vote[item] = v;
            }
            __syncthreads();
            for (int i = threadIdx.x; i < np; i += kSelThreads) {
                double sum = 0.0;
                for (int q = 0; q < n_parts; ++q) sum += part_vote[i * n_parts + q];
                pos_vote[p0 + i] = sum;
            }
            __syncthreads();
        }
        // ---- pooled binary64 score of each member ----
        for (int c = threadIdx.x; c < tot_band; c += kSelThreads) {
            const int jc = band_idx[c];
            double best = 0.0;                            // votes are >= 0
            int o = c;
            for (int t = r; t >= -r; --t) {               // descending positions: the owner index only falls
                const int j = jc + t;
                if (j < 0 || j >= P) continue;
                while (o > 0 && j < band_start[o]) --o;
                best = fmax(best, pos_vote[band_off[o] + (j - band_start[o])]);
            }
            band_score[c] = best;
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
        if (threadIdx.x == 0) {
            int run = 0;
            for (int c = 0; c < tot_band; ++c) { const int t = band_take[c]; band_take[c] = run; run += t; }
            band_take[tot_band] = run;
        }
        __syncthreads();
        // ---- ordered compaction ----
        KVQP_FOR_ROWS(
            const bool sure = v > hi, inb = v >= lo && v <= hi;
            const unsigned long long bs = __builtin_amdgcn_ballot_w64(sure);
            const unsigned long long bb = __builtin_amdgcn_ballot_w64(inb);
            const int sure_before = tab_a[row * kSelWaves + wave] + __popcll(bs & lt_mask);
            const int band_before = tab_b[row * kSelWaves + wave] + __popcll(bb & lt_mask);
            bool keep = sure;
            if (inb) keep = band_take[band_before + 1] > band_take[band_before];
            if (keep) idx[sure_before + band_take[band_before]] = j;
        )
    } else {
        // binary32 decides: everything above the cut, then the first need_at_cut equal to it
        if (a.unrefined && threadIdx.x == 0) a.unrefined[head] = tot_band;
        KVQP_FOR_ROWS(
            const unsigned long long bs = __builtin_amdgcn_ballot_w64(v > cut);
            const unsigned long long bb = __builtin_amdgcn_ballot_w64(v == cut);
            if (lane == 0) { tab_a[row * kSelWaves + wave] = __popcll(bs); tab_b[row * kSelWaves + wave] = __popcll(bb); }
            (void)j;
        )
        __syncthreads();
        (void)scan_table(tab_a, n_rows * kSelWaves, swave);
        (void)scan_table(tab_b, n_rows * kSelWaves, swave);
        KVQP_FOR_ROWS(
            const bool above = v > cut, eq = v == cut;
            const unsigned long long bs = __builtin_amdgcn_ballot_w64(above);
            const unsigned long long bb = __builtin_amdgcn_ballot_w64(eq);
            const int above_before = tab_a[row * kSelWaves + wave] + __popcll(bs & lt_mask);
            const int eq_before = tab_b[row * kSelWaves + wave] + __popcll(bb & lt_mask);
            if (above) idx[above_before + min(eq_before, need_at_cut)] = j;
            else if (eq && eq_before < need_at_cut) idx[above_before + eq_before] = j;
        )
    }
}
#undef KVQP_FOR_ROWS

size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

int n_row_slabs(const kvqp_cfg& cfg) {
    const int rows = (cfg.n_q_heads / cfg.n_kv_heads) * cfg.window;
    const int rpw = rows_per_wave(rows);
    const int slabs = (rows + rpw - 1) / rpw;
    return slabs <= 1 ? 1 : slabs == 2 ? 2 : 4;
}

template <int RPW, int NRW>
hipError_t launch_scores(const ScoreArgs& a, int n_wg, int heads, hipStream_t stream, float2* stats, double* zsum) {
    ScoreArgs s1 = a;
    hipLaunchKernelGGL((score_pass<RPW, NRW, PASS_STATS>), dim3(n_wg, heads), dim3(kThreads), 0, stream, s1);
    hipLaunchKernelGGL(stats_combine, dim3(heads, (a.rows_pad + 3) / 4), dim3(256), 0, stream, (const float2*)a.stats_part, stats, zsum,
                       a.n_parts, a.rows_pad);
    hipLaunchKernelGGL((score_pass<RPW, NRW, PASS_VOTES>), dim3(n_wg, heads), dim3(kThreads), 0, stream, s1);
    return hipGetLastError();
}

}  // namespace

CompressPlan plan_compress(const kvqp_cfg& cfg) {
    CompressPlan p{};
    p.P = cfg.seq_len - cfg.window;
    p.n_kept = cfg.budget < p.P ? cfg.budget : p.P;
    p.rows = (cfg.n_q_heads / cfg.n_kv_heads) * cfg.window;
    const int nrw = n_row_slabs(cfg);
    const int rows_pad = nrw * rows_per_wave(p.rows);
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

hipError_t launch_select(const kvqp_cfg& cfg, const void* q_obs, const void* k, int32_t* idx, int32_t* unrefined, void* ws,
                         const CompressPlan& plan, const int32_t* head_n, bool score, hipStream_t stream) {
    char* base = static_cast<char*>(ws);
    const int heads = cfg.batch * cfg.n_kv_heads;
    const int nrw = plan.n_row_slabs;
    const int ks = 4 / nrw;
    const int n_wg = plan.n_wg, cpw = plan.chunks_per_wg;

    ScoreArgs a;
    a.q_obs = (const uint16_t*)q_obs; a.k = (const uint16_t*)k;
    a.stats_part = reinterpret_cast<float2*>(base + plan.off_stats_part);
    float2* stats = reinterpret_cast<float2*>(base + plan.off_stats);
    a.rows = plan.rows; a.rows_pad = nrw * rows_per_wave(plan.rows);
    double* zsum = reinterpret_cast<double*>(base + plan.off_stats + (size_t)heads * a.rows_pad * sizeof(float2));
    a.stats = stats;
    a.vote = reinterpret_cast<float*>(base + plan.off_vote);
    a.L = cfg.seq_len; a.W = cfg.window; a.P = plan.P; a.gq = cfg.n_q_heads / cfg.n_kv_heads;
    a.n_q_heads = cfg.n_q_heads; a.n_kv_heads = cfg.n_kv_heads;
    a.chunks_per_wg = cpw; a.n_chunks = plan.n_chunks; a.n_parts = n_wg * ks;
    a.scale_log2 = cfg.sm_scale * kLog2e;

    hipError_t e;
    if (score) {   // scores are needed only when something is dropped
        if (rows_per_wave(plan.rows) == 32) {
            switch (nrw) {
                case 1: e = launch_scores<32, 1>(a, n_wg, heads, stream, stats, zsum); break;
                case 2: e = launch_scores<32, 2>(a, n_wg, heads, stream, stats, zsum); break;
                default: e = launch_scores<32, 4>(a, n_wg, heads, stream, stats, zsum); break;
            }
        } else {
            e = launch_scores<64, 4>(a, n_wg, heads, stream, stats, zsum);   // 129..256 rows: four 64-row slabs
        }
        if (e != hipSuccess) return e;
    }
    SelectArgs s;
    s.vote = a.vote; s.pooled = reinterpret_cast<float*>(base + plan.off_pooled); s.idx = idx; s.unrefined = unrefined; s.head_n = head_n;
    s.q_obs = a.q_obs; s.k = a.k; s.stats = stats; s.zsum = zsum;
    s.P = plan.P; s.L = cfg.seq_len; s.W = cfg.window; s.n_kept = plan.n_kept; s.pool = cfg.pool_kernel;
    s.gq = a.gq; s.n_q_heads = cfg.n_q_heads; s.n_kv_heads = cfg.n_kv_heads; s.rows = a.rows; s.rows_pad = a.rows_pad;
    s.scale_log2 = a.scale_log2; s.sm_scale = cfg.sm_scale;
    hipLaunchKernelGGL(select_topk, dim3(heads), dim3(kSelThreads), 0, stream, s);
    return hipGetLastError();
}

}  // namespace kvqp
