// Decode attention over the packed cache (paper Section 3: the attention of
// Eq. (3), Softmax(h_Q X_K^T) X_V, evaluated on the dequantized survivors
// G' = Q(G) s + z, plus the full-precision tail).  This is the fused
// dequantize-and-multiply the paper's Limitations section leaves as future work.
//
// Design for gfx950.  The step is HBM-bound (every packed byte is read once
// per step and used for only Gq query heads), but at 2-4 bits the plain vector
// ALUs cannot even expand the codes and multiply them at HBM speed, so both
// products run on the matrix cores with the *codes themselves* as one operand:
//   QK:  S^T[token, row] = sum_d code[token, d] * (q[row, d] * s[group, d])
//        + sum_d q[row, d] z[group, d]          (scale folded into q, per group)
//   PV:  O[row, d] = sum_t (p[row, t] * s[t, cg(d)]) * code[t, d]
//        + sum_t p[row, t] z[t, cg(d)]           (scale folded into p)
// A b-bit field masked out of a packed word is, read as binary16, the
// subnormal code * 2^-24 (times a power of two given by its bit position), and
// v_mfma_f32_16x16x32_f16 takes subnormal inputs exactly; so "dequantization"
// is one AND per two codes and the power of two is folded into the other
// operand.  The folded operands q*s and p*s are split into binary16 hi + lo
// parts that occupy separate rows of the 16-row MFMA tile (Gq <= 8 heads leave
// room), which keeps them exact to ~2^-22 instead of 2^-11.
// The value codes are stored tile-transposed (kvqp.h) so that the lane that
// holds probabilities of tokens {4kb+i} after the QK product is the lane that
// needs them as the P operand: nothing moves between lanes or through LDS
// inside the token loop.  A workgroup streams a contiguous token range in
// 64-token chunks.  When the launch has enough (batch, kv head) pairs to fill
// the chip, a head is one workgroup of 8 or 12 waves that merges through LDS
// and writes the output itself; otherwise a head is split over several
// workgroups whose partial (m, l, O) go to the workspace, and the last one to
// arrive merges them (no second kernel).
#include <mutex>

#include "kvqp_internal.h"

// ---- library-owned decode workspace, for callers that cannot allocate device memory ----
// One array per device that runs the library, held until the process ends.  In host code the
// array's name is only a handle: its device address is asked for once per device
// (hipGetSymbolAddress, with that device current) and that pointer is what kernels and fills get.
// Each device's copy starts all zero (static storage) and every completed launch leaves the
// arrival counters at its head zero again; they are nevertheless zeroed by a fill kernel when a
// device's address is first taken.  Calls that use it share it: they must not overlap on one device.
static __device__ __align__(256) unsigned char scratch[KVQP_STATIC_SCRATCH_BYTES];

namespace kvqp {
namespace {

typedef _Float16 h2v __attribute__((ext_vector_type(2)));
typedef _Float16 h8v __attribute__((ext_vector_type(8)));
typedef float f4v __attribute__((ext_vector_type(4)));

union Frag {  // one MFMA 16x16x32 f16 input operand of a lane: 8 halves
    h8v v;
    uint32_t u[4];
    h2v h[4];
};

constexpr int kWaves = 4;
constexpr int kThreads = 64 * kWaves;
constexpr int kChunk = 64;          // tokens per wave iteration
constexpr float kLog2e = 1.4426950408889634f;
constexpr float kNegBig = -1.0e30f; // finite stand-in for -inf in running maxima
// Waves per SIMD the pipelined kernel is compiled for: the 2- and 4-bit variants fit 168 registers
// (three waves) up to four query heads per KV head; wider code words or eight heads need more (two waves).
constexpr int pipe_waves(int bits, int gq, bool out = false) { return (bits <= 4 && gq <= 4 && !out) ? 3 : 2; }
constexpr float kLazyLog2 = 4.0f;   // slack of the lazily updated softmax reference
// Probabilities are formed 2^kPBoost times too large (the factor sits in the exponent, at no cost,
// and a wave hands over its reference lowered by as much, so sums, outputs and merges are all
// consistent).  The weights p * s of the value product travel as binary16 hi + lo parts, cut off
// towards zero; a weight below 2^-14 has a subnormal hi part and loses up to 2^-24 of itself, and
// in a peaked softmax that is most tokens, all losing in the same direction: measured, outputs of
// quantized caches were off by 1e-4 and more where a 16-bit cache is off by 1e-6.  With the slack
// above, p stays below 2^(kLazyLog2 + kPBoost) = 2^8, the bound it always had.  (A smaller slack
// with a larger factor is more exact still, but moves the reference about once per row and wave.)
constexpr float kPBoost = 4.0f;
constexpr int kPartStride = kHeadDim + 2;  // floats per (wave, head) of the tail states in LDS: m, l, acc[128]
// A split's partial result in the workspace, per query head: 64 x {m, l, o[2j], o[2j+1]} -- the
// reference and the sum repeated beside every channel pair, so that the workgroup that merges
// fetches all it needs of one partial with a single 16-byte load per thread.
constexpr int kPartPairs = kHeadDim / 2;
constexpr int kPartFloats = 4 * kPartPairs;

__device__ __forceinline__ float xor16_max(float v) {
    auto r = __builtin_amdgcn_permlane16_swap(__float_as_uint(v), __float_as_uint(v), false, false);
    return fmaxf(__uint_as_float(r[0]), __uint_as_float(r[1]));
}
__device__ __forceinline__ float xor32_max(float v) {
    auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(v), __float_as_uint(v), false, false);
    return fmaxf(__uint_as_float(r[0]), __uint_as_float(r[1]));
}
__device__ __forceinline__ float xor16_add(float v) {
    auto r = __builtin_amdgcn_permlane16_swap(__float_as_uint(v), __float_as_uint(v), false, false);
    return __uint_as_float(r[0]) + __uint_as_float(r[1]);
}
__device__ __forceinline__ float xor32_add(float v) {
    auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(v), __float_as_uint(v), false, false);
    return __uint_as_float(r[0]) + __uint_as_float(r[1]);
}
// sum / max over the four lanes that share (lane & 15)
__device__ __forceinline__ float quad_rows_add(float v) { return xor32_add(xor16_add(v)); }
__device__ __forceinline__ float quad_rows_max(float v) { return xor32_max(xor16_max(v)); }
// value of the neighbouring lane (lane ^ 1)
__device__ __forceinline__ float pair_other(float v) {
    return __uint_as_float(__builtin_amdgcn_mov_dpp(__float_as_uint(v), 0xB1 /*quad_perm [1,0,3,2]*/, 0xf, 0xf, true));
}

// value of the lane eight further round the row of 16 (lane ^ 8)
__device__ __forceinline__ float row_ror8(float v) {
    return __uint_as_float(__builtin_amdgcn_mov_dpp(__float_as_uint(v), 0x128 /*row_ror:8*/, 0xf, 0xf, true));
}

// A load of cache data, which a launch reads exactly once.
typedef uint32_t u4v __attribute__((ext_vector_type(4)));
typedef uint32_t u2v __attribute__((ext_vector_type(2)));
template <typename T, bool NT>
__device__ __forceinline__ T stream_load(const char* p) {
    if constexpr (NT) return __builtin_nontemporal_load(reinterpret_cast<const T*>(p));
    else return *reinterpret_cast<const T*>(p);
}
template <bool B> struct BoolC { static constexpr bool value = B; };
template <int I> struct BoolI { static constexpr int value = I; };

__device__ __forceinline__ h2v as_h2(uint32_t u) { union { uint32_t u; h2v h; } c; c.u = u; return c.h; }
__device__ __forceinline__ uint32_t as_u32(h2v h) { union { uint32_t u; h2v h; } c; c.h = h; return c.u; }
// two binary32 values cut (toward zero) to binary16, (lo, hi) half-words
__device__ __forceinline__ uint32_t pack_rtz(float lo, float hi) {
    typedef __fp16 fp16x2 __attribute__((ext_vector_type(2)));
    union { fp16x2 h; uint32_t u; } c; c.h = __builtin_amdgcn_cvt_pkrtz(lo, hi); return c.u;
}

// ---- key codes: BITS words per lane per 16-token tile (the lane's 32 channels) ----
template <int BITS> struct KWords { uint32_t w[BITS]; };

// MFMA operand for contraction step s (8 of the lane's 32 channels, natural order).
// Fields are left in place; their power-of-two position factor is KPosLog2.
template <int BITS>
__device__ __forceinline__ Frag k_frag(const KWords<BITS>& k, int s) {
    Frag f;
    if constexpr (BITS == 16) {
        f.u[0] = k.w[4 * s]; f.u[1] = k.w[4 * s + 1]; f.u[2] = k.w[4 * s + 2]; f.u[3] = k.w[4 * s + 3];
    } else if constexpr (BITS == 8) {
        const uint32_t a = k.w[2 * s], b = k.w[2 * s + 1];
        f.u[0] = a & 0x00FF00FFu; f.u[1] = (a >> 8) & 0x00FF00FFu;
        f.u[2] = b & 0x00FF00FFu; f.u[3] = (b >> 8) & 0x00FF00FFu;
    } else if constexpr (BITS == 4) {
        const uint32_t a = k.w[s], b = a >> 8;
        f.u[0] = a & 0x000F000Fu; f.u[1] = a & 0x00F000F0u;
        f.u[2] = b & 0x000F000Fu; f.u[3] = b & 0x00F000F0u;
    } else {
        const uint32_t a = k.w[s >> 1];
        if ((s & 1) == 0) {
            f.u[0] = a & 0x00030003u; f.u[1] = a & 0x000C000Cu; f.u[2] = a & 0x00300030u; f.u[3] = a & 0x00C000C0u;
        } else {
            const uint32_t b = a >> 10;
            f.u[0] = a & 0x03000300u; f.u[1] = b & 0x00030003u; f.u[2] = b & 0x000C000Cu; f.u[3] = b & 0x00300030u;
        }
    }
    return f;
}
// log2 of the factor by which register r of step s is too large.
template <int BITS>
__device__ __forceinline__ constexpr int k_pos_log2(int s, int r) {
    if (BITS == 4) return (r & 1) ? 4 : 0;
    if (BITS == 2) return (s & 1) == 0 ? 2 * r : (r == 0 ? 8 : 2 * (r - 1));
    return 0;
}

// ---- value codes: words per lane per 32-token block ----
template <int BITS> struct VGeom {
    static constexpr int kWpt = v_words_per_tile(BITS);
    static constexpr int kWordsPerLoad = 8 * kWpt;                 // words a lane holds per superblock
    static constexpr int kLoadsPerChunk = (BITS == 2) ? 1 : 2;     // superblocks per 64-token chunk
};
template <int BITS> struct VWords { uint32_t w[VGeom<BITS>::kWordsPerLoad]; };

// MFMA operand of (block-in-superblock, channel tile): registers i = 0..3 hold
// the token pairs (16H + 4kb + i, H = 0/1) in the (low, high) halves.
template <int BITS>
__device__ __forceinline__ Frag v_frag(const VWords<BITS>& v, int blk, int tile) {
    Frag f;
    if constexpr (BITS == 16) {
        f.u[0] = v.w[4 * tile]; f.u[1] = v.w[4 * tile + 1]; f.u[2] = v.w[4 * tile + 2]; f.u[3] = v.w[4 * tile + 3];
    } else if constexpr (BITS == 8) {
        const uint32_t a = v.w[2 * tile], b = v.w[2 * tile + 1];
        f.u[0] = a & 0x00FF00FFu; f.u[1] = (a >> 8) & 0x00FF00FFu;
        f.u[2] = b & 0x00FF00FFu; f.u[3] = (b >> 8) & 0x00FF00FFu;
    } else if constexpr (BITS == 4) {
        const uint32_t a = v.w[tile], b = a >> 8;
        f.u[0] = a & 0x000F000Fu; f.u[1] = a & 0x00F000F0u;
        f.u[2] = b & 0x000F000Fu; f.u[3] = b & 0x00F000F0u;
    } else {
        const uint32_t a = v.w[tile];
        if (blk == 0) {
            f.u[0] = a & 0x00030003u; f.u[1] = a & 0x000C000Cu; f.u[2] = a & 0x00300030u; f.u[3] = a & 0x00C000C0u;
        } else {
            const uint32_t b = a >> 10;
            f.u[0] = a & 0x03000300u; f.u[1] = b & 0x00030003u; f.u[2] = b & 0x000C000Cu; f.u[3] = b & 0x00300030u;
        }
    }
    return f;
}
template <int BITS>
__device__ __forceinline__ constexpr int v_pos_log2(int blk, int i) {
    if (BITS == 4) return (i & 1) ? 4 : 0;
    if (BITS == 2) return blk == 0 ? 2 * i : (i == 0 ? 8 : 2 * (i - 1));
    return 0;
}

// binary16 hi / lo parts of the binary32 value x: hi = rn(x), lo = rn(x - hi).
__device__ __forceinline__ uint32_t split_half(float x, bool want_lo) {
    const _Float16 hi = (_Float16)x;
    const _Float16 lo = (_Float16)(x - (float)hi);
    union { _Float16 h; uint16_t u; } c;
    c.h = want_lo ? lo : hi;
    return c.u;
}

struct DecodeArgs {
    const uint16_t* q;        // [B, Hq, D]
    const uint32_t* k_codes;
    const uint32_t* v_codes;
    const uint16_t* k_scale;
    const uint16_t* k_zero;
    const uint16_t* v_scale;
    const uint16_t* v_zero;
    const uint16_t* tail_k;
    const uint16_t* tail_v;
    float* part;              // [B*Hkv, n_partials, GQ, D+2]
    unsigned int* arrivals;   // [B*Hkv] arrival counters at the head of the workspace, zero between launches
    uint16_t* out;            // [B, Hq, D]
    int n_kept, tail_len, tail_cap;
    int n_cap;                // tokens the packed buffers are laid out for (head strides); >= n_kept
    const int32_t* head_n_kept;   // per (batch, kv head) token counts under the bound n_kept, or NULL
    const uint32_t* k_out;        // outlier slots [B*Hkv, n_cap, 4] (filtering on), else NULL
    const uint32_t* v_out;
    const uint32_t* k_ovf;        // overflow buffers [B*Hkv, ovf_words(n_cap, ovf_cap)] (filtering on), else NULL
    const uint32_t* v_ovf;
    int ovf_cap;                  // entries of a head's overflow list
    int n_q_heads, n_kv_heads;
    int n_splits, chunks_per_split, n_partials;
    int n_waves;              // waves per workgroup of the pipelined kernel
    int group;                // G
    int stream_from;          // chunks from this one on are loaded with the non-temporal hint
    float sm_scale;
};

// Tokens of one head: the launch's count, or the head's own, cut to the bound so that no value found
// in memory can lead a load past the buffers (they are laid out for the bound in whole blocks).
// Uniform over the workgroup.
__device__ __forceinline__ int head_tokens(const DecodeArgs& a, int bh) {
    if (!a.head_n_kept) return a.n_kept;
    const int n = a.head_n_kept[bh];
    return n < 0 ? 0 : (n > a.n_kept ? a.n_kept : n);
}
// Workgroups a head is cut into.  Every workgroup takes the plan's range of 64-token chunks
// (chunks_per_split); with per-head token counts a head uses only as many of the launch's n_splits
// ranges as its own chunks fill -- at least one, which also takes the tail rows of a head that has
// no packed token -- and the workgroups beyond that leave at once.  Heads of different lengths are
// so cut into pieces of about equal work, and a head that fits one range skips the merge across
// workgroups altogether.
__device__ __forceinline__ int head_splits(const DecodeArgs& a, int n_chunks) {
    if (!a.head_n_kept) return a.n_splits;
    const int cps = a.chunks_per_split > 0 ? a.chunks_per_split : 1;
    const int ns = (n_chunks + cps - 1) / cps;
    return ns < 1 ? 1 : (ns > a.n_splits ? a.n_splits : ns);
}

// Partials cross workgroups (and XCDs, whose L2 caches are not coherent with each other inside a
// kernel) without device-wide fences, which would write back / invalidate whole L2s: they are
// written and read with device-scope accesses that go to the coherence point directly.
// They move 16 bytes at a time: buffer accesses with the device-scope bit (sc1) of the cache policy
// -- the instruction form of a relaxed atomic load / store at agent scope, which only comes in 4 and
// 8 bytes -- through a descriptor over one head's partials (offsets in bytes; accesses outside the
// descriptor's range read zero / are dropped).  No atomicity across the 16 bytes is needed: a
// partial is complete and acknowledged before its workgroup bumps the arrival counter.
constexpr int kAuxDevScope = 16;   // sc1
__device__ __forceinline__ __amdgpu_buffer_rsrc_t part_rsrc(float* base, unsigned bytes) {
    // stride 0 (raw byte offsets), `bytes` as the range that is checked, and the descriptor's last
    // word as raw buffers take it on gfx9-family parts: 32-bit data format, no swizzle, no tiling
    return __builtin_amdgcn_make_buffer_rsrc(base, 0, (int)bytes, 0x00020000);
}
__device__ __forceinline__ void st_dev16(__amdgpu_buffer_rsrc_t r, unsigned off, float x, float y, float z, float w) {
    u4v v; v[0] = __float_as_uint(x); v[1] = __float_as_uint(y); v[2] = __float_as_uint(z); v[3] = __float_as_uint(w);
    __builtin_amdgcn_raw_buffer_store_b128(v, r, (int)off, 0, kAuxDevScope);
}
__device__ __forceinline__ u4v ld_dev16(__amdgpu_buffer_rsrc_t r, unsigned off) {
    return __builtin_amdgcn_raw_buffer_load_b128(r, (int)off, 0, kAuxDevScope);
}

// Arrival counters, one per (batch, kv head), at the head of the call's workspace.  Every workgroup
// of a head bumps its counter after its partial is written; the last one to arrive merges the
// head's partials and puts the counter back to zero, so the counters are all zero again when the
// launch has drained (kvqp_decode_workspace_init zeroes them once, before the first use).  Calls
// with different workspaces share nothing and may overlap in time.
// Merge the splits of one KV head's query heads and round once to binary16 (last workgroup only).
template <int GQ>
__device__ void merge_if_last(const DecodeArgs& a, int bh, int n_parts) {
    __shared__ int s_last;
    // Ordering of the partials before the counter, without an agent-scope release fence (which
    // writes back the whole L2).  What this relies on, all of it stated for gfx942 / gfx950 in the
    // AMDGPU memory model: (1) a store with the device-scope policy bit (what a relaxed atomic store
    // at agent scope is) is a write-through store: it is performed at the device's coherence point,
    // not left dirty in the XCD's L2; (2) vmcnt counts
    // stores, and s_waitcnt vmcnt(0) returns only when every earlier store of the wave has been
    // acknowledged from there; (3) the barrier after it orders every wave's wait before thread 0's
    // read-modify-write, which is performed at the same coherence point.  A workgroup that sees the
    // bumped counter therefore finds the partials with device-scope loads (which do not hit in its L2).
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __syncthreads();
    if (threadIdx.x == 0) {
        const unsigned prev = __hip_atomic_fetch_add(&a.arrivals[bh], 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        const int last = prev == (unsigned)(n_parts - 1);
        if (last) __hip_atomic_store(&a.arrivals[bh], 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        s_last = last;
    }
    __syncthreads();
    if (!s_last) return;
    const int b = bh / a.n_kv_heads, g = bh % a.n_kv_heads;
    const unsigned head_bytes = (unsigned)a.n_partials * GQ * kPartFloats * 4u;
    const __amdgpu_buffer_rsrc_t rs = part_rsrc(a.part + (size_t)bh * a.n_partials * GQ * kPartFloats, head_bytes);
    // Device-scope loads are slow (they go to the coherence point), so a whole batch of partials is
    // put in flight per round trip: one 16-byte load per partial and thread, a thread owning one
    // pair of output channels.
    constexpr int kMergeBatch = 32;
    for (int item = threadIdx.x; item < GQ * kPartPairs; item += blockDim.x) {
        const int h = item / kPartPairs, j = item % kPartPairs;
        float M = kNegBig, acc0 = 0.f, acc1 = 0.f, L = 0.f;
        for (int s0 = 0; s0 < n_parts; s0 += kMergeBatch) {
            u4v v[kMergeBatch];
#pragma unroll
            for (int u4 = 0; u4 < kMergeBatch; u4 += 4) {
                if (s0 + u4 < n_parts) {          // (uniform: whole groups of four beyond the last partial are not fetched)
#pragma unroll
                    for (int u = u4; u < u4 + 4; ++u)
                        v[u] = ld_dev16(rs, (unsigned)((min(s0 + u, n_parts - 1) * GQ + h) * kPartPairs + j) * 16u);
                } else {
#pragma unroll
                    for (int u = u4; u < u4 + 4; ++u) { v[u][0] = __float_as_uint(kNegBig); v[u][1] = 0u; v[u][2] = 0u; v[u][3] = 0u; }
                }
            }
            float Mn = M;
#pragma unroll
            for (int u = 0; u < kMergeBatch; ++u) Mn = fmaxf(Mn, __uint_as_float(v[u][0]));
            const float keep = __builtin_amdgcn_exp2f(M - Mn);
            acc0 *= keep; acc1 *= keep; L *= keep;
#pragma unroll
            for (int u = 0; u < kMergeBatch; ++u) {
                const float wgt = (s0 + u < n_parts) ? __builtin_amdgcn_exp2f(__uint_as_float(v[u][0]) - Mn) : 0.f;
                acc0 = __builtin_fmaf(wgt, __uint_as_float(v[u][2]), acc0);
                acc1 = __builtin_fmaf(wgt, __uint_as_float(v[u][3]), acc1);
                L = __builtin_fmaf(wgt, __uint_as_float(v[u][1]), L);
            }
            M = Mn;
        }
        const uint32_t lo = __half_as_ushort(__float2half_rn(acc0 / L)), hi = __half_as_ushort(__float2half_rn(acc1 / L));
        reinterpret_cast<uint32_t*>(a.out + ((size_t)b * a.n_q_heads + g * GQ + h) * kHeadDim)[j] = lo | (hi << 16);
    }
}

// Value of lane ^ 16 / lane ^ 32.
__device__ __forceinline__ float xor16_get(float v) {
    const auto r = __builtin_amdgcn_permlane16_swap(__float_as_uint(v), __float_as_uint(v), false, false);
    return __uint_as_float((threadIdx.x & 16) ? r[0] : r[1]);
}
__device__ __forceinline__ float xor32_get(float v) {
    const auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(v), __float_as_uint(v), false, false);
    return __uint_as_float((threadIdx.x & 32) ? r[0] : r[1]);
}
// Sum over the 16 lanes of a DPP row, result in every lane of the row.
__device__ __forceinline__ float row16_add(float v) {
    v += __uint_as_float(__builtin_amdgcn_update_dpp(0u, __float_as_uint(v), 0xB1, 0xF, 0xF, true));    // quad_perm [1,0,3,2]
    v += __uint_as_float(__builtin_amdgcn_update_dpp(0u, __float_as_uint(v), 0x4E, 0xF, 0xF, true));    // quad_perm [2,3,0,1]
    v += __uint_as_float(__builtin_amdgcn_update_dpp(0u, __float_as_uint(v), 0x141, 0xF, 0xF, true));   // row_half_mirror
    v += __uint_as_float(__builtin_amdgcn_update_dpp(0u, __float_as_uint(v), 0x140, 0xF, 0xF, true));   // row_mirror
    return v;
}

// Full-precision tail rows [t0, t1) of one KV head, shared by the four waves of a workgroup, every
// wave taking part.  The 16 lanes of a DPP row hold one (query head, tail row) pair, 8 channels
// each: with four or more query heads per KV head the four DPP rows of a wave are four heads side by
// side and the wave walks its rows one at a time (wave w: rows t0 + w, t0 + w + 4, ...), so nothing
// is merged across lanes; with two heads (one head) a wave takes two (four) rows per step and the
// row groups of a head are merged at the end.  Eight heads go in two passes (rows re-read from
// cache).  Each wave leaves its softmax state in LDS, sT[wave][head] = {reference m (log2 domain),
// sum l, unnormalised o[128]}.
// The query rows come from their plain copy in LDS (sq); the lane's first row, tail_first_row(),
// has been requested by the caller before anything waited on memory and arrives in k_first /
// v_first: when a head is split over many workgroups that row is all a wave has, and a round trip
// to memory after the staging barrier would sit on every workgroup's path.
template <int GQ> struct TailGeom {
    static constexpr int HB = GQ < 4 ? GQ : 4;   // heads side by side in a wave
    static constexpr int RP = 4 / HB;            // rows side by side in a wave
};
template <int GQ>
__device__ __forceinline__ int tail_first_row(int t0, int t1, int wave, int lane) {
    const int r = t0 + wave * TailGeom<GQ>::RP + (lane >> 4) / TailGeom<GQ>::HB;
    return (wave < kWaves && r < t1) ? r : -1;
}
template <int GQ>
__device__ void tail_rows(const DecodeArgs& a, int bh, int t0, int t1, float* sT, const uint16_t* sq, uint4 k_first, uint4 v_first) {
    constexpr int HB = TailGeom<GQ>::HB, RP = TailGeom<GQ>::RP;
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int seg = lane & 15, hb = (lane >> 4) % HB;
    const uint16_t* tk = a.tail_k + (size_t)bh * a.tail_cap * kHeadDim + 8 * seg;
    const uint16_t* tv = a.tail_v + (size_t)bh * a.tail_cap * kHeadDim + 8 * seg;
    const int r_first = tail_first_row<GQ>(t0, t1, wave, lane);
    const float c_q = a.sm_scale * kLog2e;
#pragma unroll 1
    for (int h0 = 0; h0 < GQ; h0 += HB) {
        float m = kNegBig, l = 0.f, o[8];
#pragma unroll
        for (int j = 0; j < 8; ++j) o[j] = 0.f;
        if (t0 + wave * RP < t1) {   // (wave-uniform: the wave has a row)
            float qf[8];
            {
                const uint4 u = *reinterpret_cast<const uint4*>(sq + (h0 + hb) * kHeadDim + 8 * seg);
                const uint32_t w[4] = {u.x, u.y, u.z, u.w};
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    const h2v qq = as_h2(w[j]);
                    qf[2 * j] = (float)qq[0] * c_q; qf[2 * j + 1] = (float)qq[1] * c_q;
                }
            }
            auto row_step = [&](uint4 ku, uint4 vu) {
                const uint32_t kw[4] = {ku.x, ku.y, ku.z, ku.w}, vw[4] = {vu.x, vu.y, vu.z, vu.w};
                float sc = 0.f, vf[8];
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    const h2v kk = as_h2(kw[j]), vv = as_h2(vw[j]);
                    sc = __builtin_fmaf(qf[2 * j], (float)kk[0], sc);
                    sc = __builtin_fmaf(qf[2 * j + 1], (float)kk[1], sc);
                    vf[2 * j] = (float)vv[0]; vf[2 * j + 1] = (float)vv[1];
                }
                sc = row16_add(sc);
                const float mn = fmaxf(m, sc);
                const float alpha = __builtin_amdgcn_exp2f(m - mn), pr = __builtin_amdgcn_exp2f(sc - mn);
                l = __builtin_fmaf(l, alpha, pr);
#pragma unroll
                for (int j = 0; j < 8; ++j) o[j] = __builtin_fmaf(o[j], alpha, pr * vf[j]);
                m = mn;
            };
            if (r_first >= 0) row_step(k_first, v_first);   // whole DPP rows are in or out together
            // the lane's further rows, four requested per round trip
            constexpr int kStep = 4 * RP, kBatch = 4;
            for (int r = r_first + kStep; r_first >= 0 && r < t1; r += kBatch * kStep) {
                uint4 ku[kBatch], vu[kBatch];
#pragma unroll
                for (int u = 0; u < kBatch; ++u) {
                    const int ru = (r + u * kStep < t1) ? r + u * kStep : r;
                    ku[u] = *reinterpret_cast<const uint4*>(tk + (size_t)ru * kHeadDim);
                    vu[u] = *reinterpret_cast<const uint4*>(tv + (size_t)ru * kHeadDim);
                }
#pragma unroll
                for (int u = 0; u < kBatch; ++u)
                    if (r + u * kStep < t1) row_step(ku[u], vu[u]);
            }
            if constexpr (RP > 1) {
                // merge the row groups of a head: lanes ^ 32 (two heads), then also lanes ^ 16 (one head)
#pragma unroll
                for (int step = 0; step < (RP == 4 ? 2 : 1); ++step) {
                    const float mo = step ? xor16_get(m) : xor32_get(m);
                    const float lo = step ? xor16_get(l) : xor32_get(l);
                    const float mn = fmaxf(m, mo);
                    const float ws = __builtin_amdgcn_exp2f(m - mn), wo = __builtin_amdgcn_exp2f(mo - mn);
                    l = l * ws + lo * wo;
#pragma unroll
                    for (int j = 0; j < 8; ++j) {
                        const float oo = step ? xor16_get(o[j]) : xor32_get(o[j]);
                        o[j] = o[j] * ws + oo * wo;
                    }
                    m = mn;
                }
            }
        }
        if ((lane >> 4) < HB) {
            float* row = sT + (wave * GQ + h0 + hb) * kPartStride;
            if (seg == 0) { row[0] = m; row[1] = l; }
#pragma unroll
            for (int j = 0; j < 8; ++j) row[2 + 8 * seg + j] = o[j];
        }
    }
}

// the binary32 difference an outlier slot word carries (0 for an unused slot)
__device__ __forceinline__ float slot_delta(uint32_t w) { return __uint_as_float(w & 0xFFFFFF00u); }

// ---------------------------------------------------------------------------
// The decode kernel.  Beyond the arithmetic described at the top of the file,
// its structure is all about keeping HBM, the texture-address path and the
// vector ALU busy at once:
//   * every global load of a 32-token block is issued ahead into a second
//     register set (A = first block of a 64-token chunk, B = second): the next
//     chunk's blocks are requested while the current chunk's second block is
//     computed;
//   * waves claim chunks from a workgroup counter instead of owning a fixed
//     interleave, so late or slower waves take fewer and all finish together;
//   * scales and zero-points are needed replicated (every row lane of a quad
//     multiplies by the same 32 key scales; every row lane of a slot by the same
//     token scales).  Loading them replicated costs a full 1 KB trip through the
//     texture path per instruction, so each wave instead fetches every scale row
//     once, one dword per lane, parks it in a wave-private LDS strip and reads
//     it back with broadcast ds_read_b128;
//   * the key zero-point term sum_d q[d] z[group, d] of a chunk's groups comes
//     from one extra MFMA whose token rows are the z rows themselves;
//   * the hi/lo parts of q*s come from a packed binary16 multiply and a fused
//     multiply-add of the residual; those of p*s from one binary32 product,
//     a mask, an exact subtraction and a truncating pack.
// ---------------------------------------------------------------------------
// LDS bytes of one wave's staging strip in the pipelined kernel: key scale row | key zero rows |
// value scales | value zeros of the block in flight.
// (with outlier slots: also the block's key and value slot words, 512 bytes each)
template <int BITS, int NCG, bool OUT = false> struct PipeGeom {
    static constexpr bool QUANT = BITS != 16;
    static constexpr int G = kHeadDim / NCG;
    static constexpr int NGRP = (QUANT && G == 32) ? 2 : 1;   // key groups per 64-token chunk
    static constexpr int VROW = 64 * NCG;                     // bytes of value scales of one 32-token block
    static constexpr int OFF_KS = 0, OFF_KZ = 256, OFF_VS = OFF_KZ + 256 * NGRP, OFF_VZ = OFF_VS + VROW;
    static constexpr int OFF_KO = OFF_VZ + VROW, OFF_VO = OFF_KO + 512;
    static constexpr int STRIP = QUANT ? (OUT ? OFF_VO + 512 : OFF_VZ + VROW) : 0;
};
// LDS of the pipelined kernel, bytes.  While the chunks stream: the group's query rows twice
// (plain for the z-term product, operand layout for the scale fold) and one staging strip per wave.
// Afterwards the same bytes hold every wave's state for the merge: 8 output rows (hi + lo parts
// already added) of 128 floats and 16 x (m, l, oz[4]).  The tail rows' states have their own
// region behind both (they are produced first and merged last).
constexpr int kPipeQueryLds = 8 * kHeadDim * 2 + 2 * 4 * 64 * 16;   // plain rows + up to two operand-layout copies
constexpr int kPipeStateLds = 8 * kHeadDim * 4 + 16 * 6 * 4 + 2 * 8 * 4 + 8 * 4;   // per wave: rows, stats, merge weights (+ references)
constexpr int pipe_tail_lds(int gq) { return kWaves * gq * kPartStride * 4; }
constexpr int pipe_lds_bytes(int nw, int strip, int gq, bool out = false) {
    const int loop = kPipeQueryLds + nw * strip, merge = nw * kPipeStateLds;
    return (loop > merge ? loop : merge) + pipe_tail_lds(gq) + (out ? nw * 8 * kHeadDim * 4 : 0);   // + per-wave outlier terms
}
constexpr int pipe_tail_offset(int nw, int strip) {
    const int loop = kPipeQueryLds + nw * strip, merge = nw * kPipeStateLds;
    return loop > merge ? loop : merge;
}
constexpr int pipe_max_waves(int bits, int gq, bool out = false) { return 4 * pipe_waves(bits, gq, out); }

// KT (per-token key groups, AXIS = 1): the key scales have the shape of the value scales, [token][NCG],
// and travel the same way (one dword per lane per block, parked in the strip, read back as the
// scales of four consecutive tokens).  The query operand is then the same for every block: column
// n of the product holds q masked to ONE channel group -- the columns of a head, (slot, hi/lo),
// are free for that because q needs no scale folded in and so no hi/lo split: group 2 slot + hi/lo
// at four groups, hi/lo at two -- so one pass of the usual eight matrix instructions yields every
// group's partial sum; each lane scales its own by the token's scale, adds zero x sum(q of the
// group), and two DPP exchanges add the columns of the head up.  With eight query heads per KV head
// a head has only its hi / lo columns, and four groups take two passes.
// OUT (the cache carries outlier slots): an outlier has code 0, so the products see its group's
// zero; what is missing, q[ch] * delta in the logit of its token and p * delta in channel ch of the
// output, is added outside them.  The slot words of a block travel like its scales (two dwords per
// lane and tensor, parked in the strip).  The logit term is added by the lanes that hold the
// token's logit (the hi / lo lane pair splits the four slots; q is looked up in its plain copy in
// LDS); the output term goes with LDS float atomics into a per-wave [8 rows][128] binary32 array
// that is rescaled with its row whenever the row's reference maximum moves, and folded in at the merge.
template <int BITS, int GQ, int NCG, int AXIS, bool OUT>
__global__ __launch_bounds__(64 * pipe_max_waves(BITS, GQ, OUT), 1) void decode_attn_pipe(const DecodeArgs a) {
    constexpr int SLOTS = (GQ <= 4) ? 2 : 1;
    constexpr int NT = (SLOTS == 2) ? 1 : 2;
    constexpr bool QUANT = BITS != 16;
    constexpr bool KT = QUANT && AXIS == KVQP_KEY_PER_TOKEN;
    constexpr int KP = (KT && SLOTS == 1 && NCG == 4) ? 2 : 1;   // passes of the key product: eight heads leave two columns per head, four groups take two passes
    constexpr float kCodeUnit = QUANT ? 16777216.0f : 1.0f;
    constexpr int G = kHeadDim / NCG;
    constexpr int NGRP = (QUANT && !KT && G == 32) ? 2 : 1;   // key groups per 64-token chunk
    using Geo = PipeGeom<BITS, NCG, OUT>;
    constexpr int OFF_KO = Geo::OFF_KO, OFF_VO = Geo::OFF_VO;
    constexpr int VROW = Geo::VROW;
    constexpr int VSTRIP = 8 * NCG;                           // bytes of value scales of 4 consecutive tokens
    constexpr int OFF_KS = Geo::OFF_KS, OFF_KZ = Geo::OFF_KZ, OFF_VS = Geo::OFF_VS, OFF_VZ = Geo::OFF_VZ;
    constexpr int STRIP = Geo::STRIP;

    // A workgroup is nw = 4, 8 or 12 waves (blockDim.x / 64, a multiple of four): all of them stream
    // chunks; the merge at the end is done by the first 256 threads.
    extern __shared__ __align__(16) unsigned char pipe_lds[];
    const int nw = blockDim.x >> 6;
    uint16_t* sq = reinterpret_cast<uint16_t*>(pipe_lds);                      // the group's query rows (zero rows past GQ), for the z-term product
    uint4* sqpos = reinterpret_cast<uint4*>(pipe_lds + 8 * kHeadDim * 2);      // [slice s][lane]
    unsigned char* stage_all = pipe_lds + kPipeQueryLds;
    float* sO = reinterpret_cast<float*>(pipe_lds);                            // after the loop: [wave][8 rows][128]
    float* sS = reinterpret_cast<float*>(pipe_lds + nw * (8 * kHeadDim * 4));  //                 [wave][16 rows][m, l, oz[4]]
    float* sT = reinterpret_cast<float*>(pipe_lds + pipe_tail_offset(nw, STRIP));   // tail states [wave < 4][head][m, l, o[128]]
    float* s_oc = reinterpret_cast<float*>(pipe_lds + pipe_tail_offset(nw, STRIP) + pipe_tail_lds(GQ));   // OUT: [wave][8 rows][128]

    const int bh = blockIdx.y;

    const int b = bh / a.n_kv_heads, g = bh % a.n_kv_heads;
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int n = lane & 15, kb = lane >> 4;
    const int part = n & 1;
    const int slot = (SLOTS == 2) ? (n >> 3) : 0;
    const int h = (SLOTS == 2) ? ((n & 7) >> 1) : (n >> 1);
    const bool live_row = h < GQ;
    unsigned char* stage = stage_all + (QUANT ? wave * STRIP : 0);

    // head bases (wave-uniform) and per-lane 32-bit byte offsets
    const char* kc = reinterpret_cast<const char*>(a.k_codes) + (size_t)bh * ((size_t)a.n_cap * kHeadDim * BITS / 8);
    const char* vc = reinterpret_cast<const char*>(a.v_codes) +
                     (size_t)bh * v_superblock_words(BITS) * 4 * ((a.n_cap + v_superblock(BITS) - 1) / v_superblock(BITS));
    const size_t k_meta_head = KT ? (size_t)a.n_cap * NCG * 2 : (size_t)((a.n_cap + G - 1) / G) * kHeadDim * 2;   // bytes per head
    const char* ks = QUANT ? reinterpret_cast<const char*>(a.k_scale) + (size_t)bh * k_meta_head : nullptr;
    const char* kz = QUANT ? reinterpret_cast<const char*>(a.k_zero) + (size_t)bh * k_meta_head : nullptr;
    const char* vs = QUANT ? reinterpret_cast<const char*>(a.v_scale) + (size_t)bh * a.n_cap * NCG * 2 : nullptr;
    const char* vz = QUANT ? reinterpret_cast<const char*>(a.v_zero) + (size_t)bh * a.n_cap * NCG * 2 : nullptr;
    // within a 16-token key tile.  Quantized rows: the lane's 32 channels are one contiguous piece.
    // 16-bit rows: contraction step s takes the 64-byte stretch s of the row, 16 bytes per lane, so
    // that one load instruction covers whole half-lines of 16 rows (the channel order inside the
    // contraction is free as long as the query operand follows it).
    const uint32_t k_lane = (uint32_t)n * (16 * BITS) + (uint32_t)kb * (QUANT ? 4 * BITS : 16);
    const uint32_t v_lane = (uint32_t)lane * 16;
    const uint32_t row_lane = (uint32_t)lane * 4;                                     // dword of a 256-byte scale row
    const uint32_t vrow_lane = (uint32_t)min(lane, VROW / 4 - 1) * 4;                 // dword of a block's value scales
    const int n_kept = head_tokens(a, bh);
    const int n_chunks = (n_kept + kChunk - 1) / kChunk;
    const int n_parts = head_splits(a, n_chunks);                     // workgroups of this head (uniform over the workgroup)
    if ((int)blockIdx.x >= n_parts) return;
    const int n_kgroups = QUANT ? max((n_kept + G - 1) / G, 1) : 0;   // (the last group may hold fewer than G tokens)
    // The loads of the pipeline are unconditional; when a wave has no further chunk they are pointed
    // at one 16-byte spot (lane offsets zeroed) instead of re-reading a whole chunk.
    uint32_t k_off = k_lane, v_off = v_lane, row_off = row_lane, vrow_off = vrow_lane;
    // outlier slots: 16 bytes per token and tensor, a block's 512 bytes as two dwords per lane
    const char* ko = OUT ? reinterpret_cast<const char*>(a.k_out) + (size_t)bh * a.n_cap * 16 : nullptr;
    const char* vo = OUT ? reinterpret_cast<const char*>(a.v_out) + (size_t)bh * a.n_cap * 16 : nullptr;
    uint32_t slot_off = (uint32_t)lane * 8;
    // a row's outliers beyond its four slots: the head's overflow lists, prefix counts per 32 tokens in front
    const uint32_t* kov = OUT ? a.k_ovf + (size_t)bh * ovf_words(a.n_cap, a.ovf_cap) : nullptr;
    const uint32_t* vov = OUT ? a.v_ovf + (size_t)bh * ovf_words(a.n_cap, a.ovf_cap) : nullptr;
    const uint32_t* kov_e = OUT ? kov + ovf_start_words(a.n_cap) : nullptr;
    const uint32_t* vov_e = OUT ? vov + ovf_start_words(a.n_cap) : nullptr;
    uint32_t a_kov = 0, a_vov = 0, b_kov = 0, b_vov = 0;   // lanes 0, 1: the block's range in the list (requested with its codes)
    const uint32_t ovf_lane = (uint32_t)min(lane, 1) * 4;   // lane 0: entry of the block, other lanes: the entry after it (always inside the array)
    (void)kov_e; (void)vov_e; (void)ovf_lane;
    const int row8 = (SLOTS == 2) ? slot * 4 + h : h;                  // the lane's row of the wave's outlier terms
    float* oc = s_oc + (OUT ? wave * 8 * kHeadDim : 0);
    (void)ko; (void)vo; (void)slot_off; (void)row8; (void)oc;

    // lane constants of the p*s operand: lo rows subtract the leading bits; a value lands in the
    // half-word of the lane's token slot (byte selectors for v_perm_b32: 0x0c gives a zero byte)
    const uint32_t lo_mask = part ? 0xFFFFE000u : 0u;
    const uint32_t slot_mask = slot ? 0xFFFF0000u : 0x0000FFFFu;
    const uint32_t sel_even = slot ? 0x01000C0Cu : 0x0C0C0100u;   // low half-word of the pair
    const uint32_t sel_odd = slot ? 0x03020C0Cu : 0x0C0C0302u;    // high half-word of the pair
    (void)lo_mask; (void)slot_mask; (void)sel_even; (void)sel_odd;
    uint32_t zrow_mask = (n < NGRP) ? 0xFFFFFFFFu : 0u;   // rows of the zero-term product that hold a key group
    asm volatile("" : "+v"(zrow_mask));                    // (kept opaque: as a known select the sixteen ANDs become half-rate selects)
    (void)zrow_mask;
    const float c_logit = a.sm_scale * kLog2e * kCodeUnit;
    const float c_bias = a.sm_scale * kLog2e;
    // per-token keys: the channel group of the lane's column, whether the lane's 32 channels lie in
    // it, the byte selector that picks that group's half out of a pair of strip words, and (set once
    // q is staged) the sum of q over the group, in code units
    // (per pass where the product takes two)
    bool kt_mine[KP];
    uint32_t kt_sel[KP];
    float kt_qs[KP];
#pragma unroll
    for (int ps = 0; ps < KP; ++ps) {
        const int c = (NCG == 4) ? ((SLOTS == 2) ? 2 * slot + part : 2 * ps + part) : (NCG == 2 ? part : 0);
        kt_mine[ps] = (NCG > 1 || part == 0) && (kb / (4 / NCG)) == c;
        const uint32_t bsel = (NCG == 4) ? 4u * (c >> 1) + 2u * (c & 1) : 2u * (uint32_t)c;
        kt_sel[ps] = 0x0C0C0000u | ((bsel + 1u) << 8) | bsel;
        kt_qs[ps] = 0.f;
    }
    (void)kt_mine; (void)kt_sel;

    f4v O[8];
#pragma unroll
    for (int t = 0; t < 8; ++t) O[t] = (f4v){0.f, 0.f, 0.f, 0.f};
    float oz[NCG];
#pragma unroll
    for (int c = 0; c < NCG; ++c) oz[c] = 0.f;
    float m_run = kNegBig, l_run = 0.f;
    Frag bq[4];                       // query-times-scale operand of the current key group (KT: masked q, set once)

    // ---- the two register sets (codes as MFMA operands; one dword per lane of every scale row) ----
    KWords<BITS> ak0, ak1, bk0, bk1;
    VWords<BITS> av, bv;
    uint32_t a_ks = 0, a_kz[NGRP], a_vs = 0, a_vz = 0, b_ks = 0, b_kz = 0, b_vs = 0, b_vz = 0;
    uint2 a_ko = make_uint2(0u, 0u), a_vo = a_ko, b_ko = a_ko, b_vo = a_ko;   // OUT: slot words of the blocks in flight
#pragma unroll
    for (int i = 0; i < NGRP; ++i) a_kz[i] = 0;

    auto load_k = [&](int tok, KWords<BITS>& dst, auto nt) {
        constexpr bool NT = decltype(nt)::value;
        const char* p = kc + (size_t)tok * (16 * BITS) + k_off;
        if constexpr (BITS == 2) {
            const u2v v = stream_load<u2v, NT>(p);
            dst.w[0] = v[0]; dst.w[1] = v[1];
        } else {
#pragma unroll
            for (int i = 0; i < BITS / 4; ++i) {
                const u4v v = stream_load<u4v, NT>(p + (QUANT ? 16 : 64) * i);
                dst.w[4 * i] = v[0]; dst.w[4 * i + 1] = v[1]; dst.w[4 * i + 2] = v[2]; dst.w[4 * i + 3] = v[3];
            }
        }
    };
    auto load_v = [&](int sb, VWords<BITS>& dst, auto nt) {
        constexpr bool NT = decltype(nt)::value;
        const char* p = vc + (size_t)sb * (v_superblock_words(BITS) * 4) + v_off;
#pragma unroll
        for (int q = 0; q < VGeom<BITS>::kWordsPerLoad / 4; ++q) {
            const u4v v = stream_load<u4v, NT>(p + q * 1024);
            dst.w[4 * q] = v[0]; dst.w[4 * q + 1] = v[1]; dst.w[4 * q + 2] = v[2]; dst.w[4 * q + 3] = v[3];
        }
    };
    auto dword_at = [](const char* base, uint32_t off, auto nt) { return stream_load<uint32_t, decltype(nt)::value>(base + off); };
    // Loads are unconditional (indices clamped to valid blocks) so that the loop body is
    // straight-line code and the hardware wait counters can be tracked exactly.
    // A block's loads come in two parts: the key side (codes, key scales / zeros, key outlier slots)
    // and the value side (codes, value scales / zeros, value outlier slots).
    auto load_Ak_as = [&](int chunk, auto nt) {
        const int tb = chunk * kChunk;
        load_k(tb + 0, ak0, nt); load_k(tb + 16, ak1, nt);
        if constexpr (QUANT) {
            if constexpr (KT) {
                a_ks = dword_at(ks, (uint32_t)tb * (2 * NCG) + vrow_off, nt);
                a_kz[0] = dword_at(kz, (uint32_t)tb * (2 * NCG) + vrow_off, nt);
            } else {
                const int u = tb / G;
                a_ks = dword_at(ks, (uint32_t)u * 256 + row_off, nt);
#pragma unroll
                for (int i = 0; i < NGRP; ++i) a_kz[i] = dword_at(kz, (uint32_t)min(u + i, n_kgroups - 1) * 256 + row_off, nt);
            }
        }
        if constexpr (OUT) {
            const u2v w = stream_load<u2v, decltype(nt)::value>(ko + (size_t)tb * 16 + slot_off); a_ko = make_uint2(w[0], w[1]);
            a_kov = kov[tb / 32 + ovf_lane / 4];
        }
    };
    auto load_Av_as = [&](int chunk, auto nt) {
        const int tb = chunk * kChunk;
        if constexpr (QUANT) {
            a_vs = dword_at(vs, (uint32_t)tb * (2 * NCG) + vrow_off, nt);
            a_vz = dword_at(vz, (uint32_t)tb * (2 * NCG) + vrow_off, nt);
        }
        if constexpr (OUT) {
            const u2v w = stream_load<u2v, decltype(nt)::value>(vo + (size_t)tb * 16 + slot_off); a_vo = make_uint2(w[0], w[1]);
            a_vov = vov[tb / 32 + ovf_lane / 4];
        }
        load_v((BITS == 2) ? chunk : 2 * chunk, av, nt);
    };
    auto load_Bk_as = [&](int chunk, bool two, auto nt) {
        const int tb = chunk * kChunk + (two ? 32 : 0);
        load_k(tb + 0, bk0, nt); load_k(tb + 16, bk1, nt);
        if constexpr (QUANT) {
            if constexpr (KT) {
                b_ks = dword_at(ks, (uint32_t)tb * (2 * NCG) + vrow_off, nt);
                b_kz = dword_at(kz, (uint32_t)tb * (2 * NCG) + vrow_off, nt);
            } else if constexpr (NGRP == 2) b_ks = dword_at(ks, (uint32_t)(tb / G) * 256 + row_off, nt);
        }
        if constexpr (OUT) {
            const u2v w = stream_load<u2v, decltype(nt)::value>(ko + (size_t)tb * 16 + slot_off); b_ko = make_uint2(w[0], w[1]);
            b_kov = kov[tb / 32 + ovf_lane / 4];
        }
    };
    auto load_Bv_as = [&](int chunk, bool two, auto nt) {
        const int tb = chunk * kChunk + (two ? 32 : 0);
        if constexpr (QUANT) {
            b_vs = dword_at(vs, (uint32_t)tb * (2 * NCG) + vrow_off, nt);
            b_vz = dword_at(vz, (uint32_t)tb * (2 * NCG) + vrow_off, nt);
        }
        if constexpr (OUT) {
            const u2v w = stream_load<u2v, decltype(nt)::value>(vo + (size_t)tb * 16 + slot_off); b_vo = make_uint2(w[0], w[1]);
            b_vov = vov[tb / 32 + ovf_lane / 4];
        }
        if constexpr (BITS != 2) load_v(2 * chunk + (two ? 1 : 0), bv, nt);
    };
    // Chunks from a.stream_from on are read with the non-temporal hint (wave-uniform choice; a 16-bit
    // cache never is).  The empty statements keep the two arms apart: merged, the loads would lose
    // the hint.
    constexpr bool MIX = true;
    auto streamed = [&](int chunk) { return MIX && chunk >= a.stream_from; };
    auto load_Ak = [&](int chunk) {
        if (streamed(chunk)) { asm volatile("; streamed"); load_Ak_as(chunk, BoolC<true>{}); asm volatile("; streamed"); }
        else load_Ak_as(chunk, BoolC<false>{});
    };
    auto load_Av = [&](int chunk) {
        if (streamed(chunk)) { asm volatile("; streamed"); load_Av_as(chunk, BoolC<true>{}); asm volatile("; streamed"); }
        else load_Av_as(chunk, BoolC<false>{});
    };
    auto load_Bk = [&](int chunk, bool two) {
        if (streamed(chunk)) { asm volatile("; streamed"); load_Bk_as(chunk, two, BoolC<true>{}); asm volatile("; streamed"); }
        else load_Bk_as(chunk, two, BoolC<false>{});
    };
    auto load_Bv = [&](int chunk, bool two) {
        if (streamed(chunk)) { asm volatile("; streamed"); load_Bv_as(chunk, two, BoolC<true>{}); asm volatile("; streamed"); }
        else load_Bv_as(chunk, two, BoolC<false>{});
    };
    auto load_A = [&](int chunk) {
        if (streamed(chunk)) { asm volatile("; streamed"); load_Ak_as(chunk, BoolC<true>{}); load_Av_as(chunk, BoolC<true>{}); asm volatile("; streamed"); }
        else { load_Ak_as(chunk, BoolC<false>{}); load_Av_as(chunk, BoolC<false>{}); }
    };
    auto load_B = [&](int chunk, bool two) {
        if (streamed(chunk)) { asm volatile("; streamed"); load_Bk_as(chunk, two, BoolC<true>{}); load_Bv_as(chunk, two, BoolC<true>{}); asm volatile("; streamed"); }
        else { load_Bk_as(chunk, two, BoolC<false>{}); load_Bv_as(chunk, two, BoolC<false>{}); }
    };
    auto lds_put = [&](int off, uint32_t v) { *reinterpret_cast<uint32_t*>(stage + off + row_lane) = v; };
    auto lds_put_v = [&](int off, uint32_t v) { if (lane < VROW / 4) *reinterpret_cast<uint32_t*>(stage + off + row_lane) = v; };
    auto lds_get16 = [&](int off, uint32_t* dst) {   // 64 bytes -> 16 registers
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const uint4 v = *reinterpret_cast<const uint4*>(stage + off + 16 * i);
            dst[4 * i] = v.x; dst[4 * i + 1] = v.y; dst[4 * i + 2] = v.z; dst[4 * i + 3] = v.w;
        }
    };
    auto lds_get_strip = [&](int off, uint32_t* dst) {  // the scales of 4 consecutive tokens
        if constexpr (VSTRIP == 32) {
            const uint4 x = *reinterpret_cast<const uint4*>(stage + off), y = *reinterpret_cast<const uint4*>(stage + off + 16);
            dst[0] = x.x; dst[1] = x.y; dst[2] = x.z; dst[3] = x.w; dst[4] = y.x; dst[5] = y.y; dst[6] = y.z; dst[7] = y.w;
        } else if constexpr (VSTRIP == 16) {
            const uint4 x = *reinterpret_cast<const uint4*>(stage + off);
            dst[0] = x.x; dst[1] = x.y; dst[2] = x.z; dst[3] = x.w;
        } else {
            const uint2 x = *reinterpret_cast<const uint2*>(stage + off);
            dst[0] = x.x; dst[1] = x.y;
        }
    };

    // Move the softmax reference when a row maximum (already reduced over the row's lanes) asks for it.
    auto advance_reference = [&](float mx) {
        // The running maximum is only a scaling reference: it is moved (and O, l rescaled) when
        // some row's maximum has grown by more than 2^kLazyLog2, so probabilities stay below that.
        const float m_new = fmaxf(m_run, mx);
        if (__builtin_amdgcn_ballot_w64(m_new > m_run + kLazyLog2) != 0ull) {
            const float alpha = __builtin_amdgcn_exp2f(m_run - m_new);
            l_run *= alpha;
#pragma unroll
            for (int c = 0; c < NCG; ++c) oz[c] *= alpha;
            float ar[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) ar[i] = __shfl(alpha, 4 * kb + i);
#pragma unroll
            for (int t = 0; t < 8; ++t)
#pragma unroll
                for (int i = 0; i < 4; ++i) O[t][i] *= ar[i];
            m_run = m_new;
            if constexpr (OUT) {
                // the eight lanes of a row (hi / lo pair x four kb) rescale 16 channels each of its outlier terms
                if (live_row && alpha != 1.0f) {
                    float* p16 = oc + row8 * kHeadDim + (part * 4 + kb) * 16;
#pragma unroll
                    for (int c = 0; c < 16; c += 4) {
                        float4 v = *reinterpret_cast<float4*>(p16 + c);
                        v.x *= alpha; v.y *= alpha; v.z *= alpha; v.w *= alpha;
                        *reinterpret_cast<float4*>(p16 + c) = v;
                    }
                }
                __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");   // (LDS serves a wave in order; this only pins the compiler)
            }
        }
    };

    // one 32-token block: QK product, online softmax update, PV product.  mode 0: all of it; mode 1:
    // the logits only (into lgio); mode 2: the rest, from the logits in lgio, the reference having
    // been moved by the caller for both blocks of the chunk at once.
    auto compute = [&](auto mode, float (&lgio)[NT][4], const KWords<BITS>& k0, const KWords<BITS>& k1, uint32_t r_ks, uint32_t r_kz,
                       bool new_group, float bias, const VWords<BITS>& vv, int vblk, uint32_t r_vs, uint32_t r_vz, uint2 r_ko,
                       uint2 r_vo, uint32_t r_kov, uint32_t r_vov, int tok0) {
        constexpr int MODE = decltype(mode)::value;
        uint32_t vsr[QUANT ? NT * 2 * NCG : 1], vzr[QUANT ? NT * 2 * NCG : 1];
        if constexpr (QUANT && MODE != 2) {
            if constexpr (KT) { lds_put_v(OFF_KS, r_ks); lds_put_v(OFF_KZ, r_kz); }
            else if (new_group) lds_put(OFF_KS, r_ks);
            if constexpr (OUT) *reinterpret_cast<uint2*>(stage + OFF_KO + lane * 8) = r_ko;
        }
        if constexpr (QUANT && MODE != 1) {
            lds_put_v(OFF_VS, r_vs); lds_put_v(OFF_VZ, r_vz);
            if constexpr (OUT) *reinterpret_cast<uint2*>(stage + OFF_VO + lane * 8) = r_vo;
        }
        if constexpr (QUANT && MODE != 2) {
            if constexpr (KT) {
                // (the masked query operand is re-read from LDS inside the pass loop below)
            } else if (new_group) {
                uint32_t sw[16], qw[16];
                lds_get16(OFF_KS + 64 * kb, sw);
#pragma unroll
                for (int s = 0; s < 4; ++s) {
                    const uint4 v = sqpos[s * 64 + lane];
                    qw[4 * s] = v.x; qw[4 * s + 1] = v.y; qw[4 * s + 2] = v.z; qw[4 * s + 3] = v.w;
                }
#pragma unroll
                for (int s = 0; s < 4; ++s)
#pragma unroll
                    for (int r = 0; r < 4; ++r) bq[s].h[r] = as_h2(qw[4 * s + r]) * as_h2(sw[4 * s + r]);
                if (part) {
#pragma unroll
                    for (int s = 0; s < 4; ++s)
#pragma unroll
                        for (int r = 0; r < 4; ++r)
                            bq[s].h[r] = __builtin_elementwise_fma(as_h2(qw[4 * s + r]), as_h2(sw[4 * s + r]), -bq[s].h[r]);
                }
            }
        }
        if constexpr (QUANT && MODE != 1) {
#pragma unroll
            for (int t = 0; t < NT; ++t) {
                const int th = (SLOTS == 2) ? slot : t;
                lds_get_strip(OFF_VS + (16 * th + 4 * kb) * (2 * NCG), vsr + t * 2 * NCG);
                lds_get_strip(OFF_VZ + (16 * th + 4 * kb) * (2 * NCG), vzr + t * 2 * NCG);
            }
        }
        float lg[NT][4];
        if constexpr (MODE == 2) {
#pragma unroll
            for (int t = 0; t < NT; ++t)
#pragma unroll
                for (int i = 0; i < 4; ++i) lg[t][i] = lgio[t][i];
        } else {
            f4v acc0 = (f4v){0.f, 0.f, 0.f, 0.f}, acc1 = acc0;
            if constexpr (!KT) {
#pragma unroll
                for (int s = 0; s < 4; ++s) {
                    acc0 = __builtin_amdgcn_mfma_f32_16x16x32_f16(k_frag<BITS>(k0, s).v, bq[s].v, acc0, 0, 0, 0);
                    acc1 = __builtin_amdgcn_mfma_f32_16x16x32_f16(k_frag<BITS>(k1, s).v, bq[s].v, acc1, 0, 0, 0);
                }
            }
            const float bias_l2 = bias * c_bias;
            if constexpr (KT) {
                // The lane's column holds one channel group (per pass): the product with the masked query,
                // re-read from LDS rather than kept (16 registers), then scale by the token's scale of that
                // group and add its zero term.  One tile's strips at a time (16 registers), and only the
                // slot's own tile where the other one is not needed.
                constexpr bool kBothTiles = SLOTS == 1 || NCG == 4;
                float tt[2][4];
#pragma unroll
                for (int t = 0; t < 2; ++t)
#pragma unroll
                    for (int i = 0; i < 4; ++i) tt[t][i] = 0.f;
#pragma unroll
                for (int ps = 0; ps < KP; ++ps) {
                    acc0 = (f4v){0.f, 0.f, 0.f, 0.f}; acc1 = acc0;
#pragma unroll
                    for (int s = 0; s < 4; ++s) {
                        const uint4 v = sqpos[(ps * 4 + s) * 64 + lane];
                        Frag bqs;
                        bqs.u[0] = v.x; bqs.u[1] = v.y; bqs.u[2] = v.z; bqs.u[3] = v.w;
                        acc0 = __builtin_amdgcn_mfma_f32_16x16x32_f16(k_frag<BITS>(k0, s).v, bqs.v, acc0, 0, 0, 0);
                        acc1 = __builtin_amdgcn_mfma_f32_16x16x32_f16(k_frag<BITS>(k1, s).v, bqs.v, acc1, 0, 0, 0);
                    }
#pragma unroll
                    for (int t = 0; t < 2; ++t) {
                        if (!kBothTiles && t != 0) continue;
                        const int tile = kBothTiles ? t : slot;
                        uint32_t ksr[2 * NCG], kzr[2 * NCG];
                        lds_get_strip(OFF_KS + (16 * tile + 4 * kb) * (2 * NCG), ksr);
                        lds_get_strip(OFF_KZ + (16 * tile + 4 * kb) * (2 * NCG), kzr);
                        auto at = [&](const uint32_t* w, int i) -> float {   // half (token i, the column's group) of the strip
                            if constexpr (NCG == 4) {
                                return (float)as_h2(__builtin_amdgcn_perm(w[2 * i + 1], w[2 * i], kt_sel[ps]))[0];
                            } else if constexpr (NCG == 2) {
                                return (float)as_h2(__builtin_amdgcn_perm(w[i], w[i], kt_sel[ps]))[0];
                            } else {
                                return (float)as_h2(w[i >> 1])[i & 1];
                            }
                        };
#pragma unroll
                        for (int i = 0; i < 4; ++i) {
                            const float acc = kBothTiles ? (t ? acc1[i] : acc0[i]) : (slot ? acc1[i] : acc0[i]);
                            tt[t][i] += __builtin_fmaf(acc, at(ksr, i), at(kzr, i) * kt_qs[ps]);
                        }
                    }
                }
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    if constexpr (SLOTS == 2 && NCG == 4) {          // four columns per head: both tiles are summed, then the slot's is kept
                        float t0 = tt[0][i], t1 = tt[1][i];
                        t0 += pair_other(t0); t1 += pair_other(t1);
                        t0 += row_ror8(t0); t1 += row_ror8(t1);
                        lg[0][i] = (slot ? t1 : t0) * c_logit;
                    } else if constexpr (SLOTS == 2) {
                        float s = tt[0][i];
                        s += pair_other(s);
                        lg[0][i] = s * c_logit;
                    } else {
                        float t0 = tt[0][i], t1 = tt[1][i];
                        t0 += pair_other(t0); t1 += pair_other(t1);
                        lg[0][i] = t0 * c_logit; lg[NT - 1][i] = t1 * c_logit;
                    }
                }
            } else
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                if constexpr (SLOTS == 2) {
                    float s = slot ? acc1[i] : acc0[i];
                    s += pair_other(s);
                    lg[0][i] = __builtin_fmaf(s, c_logit, bias_l2);
                } else {
                    float s0 = acc0[i], s1 = acc1[i];
                    s0 += pair_other(s0); s1 += pair_other(s1);
                    lg[0][i] = __builtin_fmaf(s0, c_logit, bias_l2);
                    lg[NT - 1][i] = __builtin_fmaf(s1, c_logit, bias_l2);
                }
            }
            if constexpr (OUT) {
                // key outliers of the lane's tokens: this lane takes slots 2 part, 2 part + 1, its pair the other two
                const uint16_t* qrow = sq + h * kHeadDim;
#pragma unroll
                for (int t = 0; t < NT; ++t) {
                    const int th = (SLOTS == 2) ? slot : t;
#pragma unroll
                    for (int i = 0; i < 4; ++i) {
                        const uint2 w = *reinterpret_cast<const uint2*>(stage + OFF_KO + (16 * th + 4 * kb + i) * 16 + part * 8);
                        float c = slot_delta(w.x) * __half2float(__ushort_as_half(qrow[w.x & 127u]));
                        c = __builtin_fmaf(slot_delta(w.y), __half2float(__ushort_as_half(qrow[w.y & 127u])), c);
                        c += pair_other(c);
                        lg[t][i] = __builtin_fmaf(c, c_bias, lg[t][i]);
                    }
                }
                // key outliers beyond the rows' slots (rare): the block's stretch of the head's overflow list;
                // both lanes of a hi / lo pair hold the token's logit and both add the whole term
                const uint32_t e0 = (uint32_t)__builtin_amdgcn_readlane((int)r_kov, 0);
                const uint32_t e1 = min((uint32_t)__builtin_amdgcn_readlane((int)r_kov, 1), (uint32_t)a.ovf_cap);
                for (uint32_t e = e0; e < e1; ++e) {
                    const uint32_t w = kov_e[2 * (size_t)e];
                    const int tl = (int)kov_e[2 * (size_t)e + 1] - tok0;          // token within the block
                    if (tl < 0 || tl >= 32) continue;                             // (never, for a list the library wrote)
                    const float term = slot_delta(w) * __half2float(__ushort_as_half(qrow[w & 127u])) * c_bias;
                    const bool mine = ((tl >> 2) & 3) == kb && ((SLOTS == 2) ? (tl >> 4) == slot : true);
#pragma unroll
                    for (int t = 0; t < NT; ++t)
#pragma unroll
                        for (int i = 0; i < 4; ++i)
                            if (mine && (tl & 3) == i && ((SLOTS == 2) || (tl >> 4) == t)) lg[t][i] += term;
                }
            }
        }
        if constexpr (MODE != 2) {
            // the head's last block may be partly filled: tokens past the count take no part
            if (tok0 + 32 > n_kept) {   // (wave-uniform, and false for all but one block of a head)
#pragma unroll
                for (int t = 0; t < NT; ++t) {
                    const int th = (SLOTS == 2) ? slot : t;
#pragma unroll
                    for (int i = 0; i < 4; ++i)
                        if (tok0 + 16 * th + 4 * kb + i >= n_kept) lg[t][i] = -INFINITY;   // weight exactly 0 (references stay finite)
                }
            }
        }
        if constexpr (MODE == 1) {
#pragma unroll
            for (int t = 0; t < NT; ++t)
#pragma unroll
                for (int i = 0; i < 4; ++i) lgio[t][i] = lg[t][i];
            return;
        }
        if constexpr (MODE == 0) {
            float mx = lg[0][0];
#pragma unroll
            for (int t = 0; t < NT; ++t)
#pragma unroll
                for (int i = 0; i < 4; ++i) mx = fmaxf(mx, lg[t][i]);
            advance_reference(quad_rows_max(mx));
        }
        float p[NT][4];
#pragma unroll
        for (int t = 0; t < NT; ++t)
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const int e = v_pos_log2<BITS>(vblk, i);
                p[t][i] = __builtin_amdgcn_exp2f(lg[t][i] - (m_run + ((float)e - kPBoost)));
                l_run = __builtin_fmaf(p[t][i], (float)(1 << e), l_run);
            }
        if constexpr (OUT) {
            // value outliers of the lane's tokens: weight x delta into channel ch of the lane's row
            if (live_row) {
#pragma unroll
                for (int t = 0; t < NT; ++t) {
                    const int th = (SLOTS == 2) ? slot : t;
#pragma unroll
                    for (int i = 0; i < 4; ++i) {
                        const uint2 w = *reinterpret_cast<const uint2*>(stage + OFF_VO + (16 * th + 4 * kb + i) * 16 + part * 8);
                        const float pw = p[t][i] * (float)(1 << v_pos_log2<BITS>(vblk, i));
                        // (an LDS atomic costs the CU a fixed time even with no lane active: skip those)
                        if (__builtin_amdgcn_ballot_w64(w.x != 0u) != 0ull)
                            if (w.x) atomicAdd(oc + row8 * kHeadDim + (w.x & 127u), pw * slot_delta(w.x));
                        if (__builtin_amdgcn_ballot_w64(w.y != 0u) != 0ull)
                            if (w.y) atomicAdd(oc + row8 * kHeadDim + (w.y & 127u), pw * slot_delta(w.y));
                    }
                }
            }
            // value outliers beyond the rows' slots (rare): one lane per (row, token) -- the hi lane of the pair
            {
                const uint32_t e0 = (uint32_t)__builtin_amdgcn_readlane((int)r_vov, 0);
                const uint32_t e1 = min((uint32_t)__builtin_amdgcn_readlane((int)r_vov, 1), (uint32_t)a.ovf_cap);
                for (uint32_t e = e0; e < e1; ++e) {
                    const uint32_t w = vov_e[2 * (size_t)e];
                    const int tl = (int)vov_e[2 * (size_t)e + 1] - tok0;
                    if (tl < 0 || tl >= 32) continue;
                    const bool mine = live_row && part == 0 && ((tl >> 2) & 3) == kb && ((SLOTS == 2) ? (tl >> 4) == slot : true);
                    float pw = 0.f;
#pragma unroll
                    for (int t = 0; t < NT; ++t)
#pragma unroll
                        for (int i = 0; i < 4; ++i)
                            if ((tl & 3) == i && ((SLOTS == 2) || (tl >> 4) == t)) pw = p[t][i] * (float)(1 << v_pos_log2<BITS>(vblk, i));
                    if (mine) atomicAdd(oc + row8 * kHeadDim + (w & 127u), pw * slot_delta(w));
                }
            }
            __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
        }
        Frag pa[NCG];
        if constexpr (!QUANT) {
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                uint32_t w = 0;
#pragma unroll
                for (int t = 0; t < NT; ++t) {
                    const int th = (SLOTS == 2) ? slot : t;
                    w |= split_half(p[t][i], part) << (16 * th);
                }
                pa[0].u[i] = w;
            }
        } else {
            // x = p * s in binary32; the hi rows take x, the lo rows x minus its leading 11 bits (an
            // exact difference); both are then cut to binary16 by the same truncating conversion,
            // so hi + lo reproduces x to ~2^-22.
            float xv[NT][4][NCG];
#pragma unroll
            for (int t = 0; t < NT; ++t)
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    const float pz = p[t][i] * (float)(1 << v_pos_log2<BITS>(vblk, i));
#pragma unroll
                    for (int c = 0; c < NCG; ++c) {
                        const int e = i * NCG + c;                       // half index inside the lane's 4-token strip
                        const h2v sv2 = as_h2(vsr[t * 2 * NCG + (e >> 1)]), zv2 = as_h2(vzr[t * 2 * NCG + (e >> 1)]);
                        const float x = __builtin_fmaf(p[t][i], (float)sv2[e & 1], 0.0f);
                        xv[t][i][c] = x - __uint_as_float(__float_as_uint(x) & lo_mask);
                        oz[c] = __builtin_fmaf(pz, (float)zv2[e & 1], oz[c]);
                    }
                }
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                if constexpr (SLOTS == 1) {          // both token halves are this lane's: (t = 0 | t = 1)
#pragma unroll
                    for (int c = 0; c < NCG; ++c)
                        pa[c].u[i] = pack_rtz(xv[0][i][c], xv[NT - 1][i][c]);
                } else if constexpr (NCG == 1) {     // one value, parked in the half of this lane's token slot
                    pa[0].u[i] = pack_rtz(xv[0][i][0], xv[0][i][0]) & slot_mask;
                } else {                             // two channel groups per conversion, each moved to the slot's half
#pragma unroll
                    for (int c = 0; c < NCG; c += 2) {
                        const uint32_t pk = pack_rtz(xv[0][i][c], xv[0][i][c + 1]);
                        pa[c].u[i] = __builtin_amdgcn_perm(pk, pk, sel_even);
                        pa[c + 1].u[i] = __builtin_amdgcn_perm(pk, pk, sel_odd);
                    }
                }
            }
        }
#pragma unroll
        for (int t8 = 0; t8 < 8; ++t8)
            O[t8] = __builtin_amdgcn_mfma_f32_16x16x32_f16(pa[(t8 * 16) / G].v, v_frag<BITS>(vv, vblk, t8).v, O[t8], 0, 0, 0);
    };

    const int cps = a.chunks_per_split;
    const int c_begin = blockIdx.x * cps;
    const int c_end = min(n_chunks, c_begin + cps);
    // Chunks are claimed, not dealt: a wave takes its first chunk by index and every later one from
    // a workgroup counter, so waves that start late (the tail rows) or run slower (the SIMD favours
    // its oldest wave) simply take fewer and all of them finish together.
    __shared__ int s_next_chunk;
    if (threadIdx.x == 0) s_next_chunk = c_begin + nw;
    auto claim = [&]() {
        int v = 0;
        if (lane == 0) v = atomicAdd(&s_next_chunk, 1);
        return __builtin_amdgcn_readfirstlane(v);
    };
    int chunk = c_begin + wave;
    bool two = chunk < c_end && n_kept - chunk * kChunk > 32;        // the chunk reaches into its second 32-token block
    // The second block of a chunk is requested right after the previous chunk's second block has
    // been consumed (quantized variants: more bytes in flight, and the first chunk's blocks are both
    // on their way before anything waits); the 16-bit variant, whose blocks are four times larger,
    // runs faster when it asks at the top of the chunk's own iteration.
    constexpr bool kEarlyB = QUANT;
    constexpr bool kJoint = QUANT && !OUT && !(KT && BITS == 2);   // (where it measured faster: see the loop)
    if (chunk < c_end) { load_A(chunk); if (kEarlyB) load_B(chunk, two); }   // issued before anything else waits on memory
    // ... and with them the wave's first step of this workgroup's share of the full-precision tail rows
    const int tail_t0 = (int)(((long long)a.tail_len * blockIdx.x) / n_parts);
    const int tail_t1 = (int)(((long long)a.tail_len * (blockIdx.x + 1)) / n_parts);
    uint4 tail_k0 = make_uint4(0u, 0u, 0u, 0u), tail_v0 = tail_k0;
    {
        const int r = tail_first_row<GQ>(tail_t0, tail_t1, wave, lane);
        if (r >= 0) {
            const size_t at = ((size_t)bh * a.tail_cap + r) * kHeadDim + 8 * (lane & 15);
            tail_k0 = *reinterpret_cast<const uint4*>(a.tail_k + at);
            tail_v0 = *reinterpret_cast<const uint4*>(a.tail_v + at);
        }
    }
    // Query rows with each register's field-position factor folded in: MFMA operand layout, lane
    // (head row, channel block kb).  The quantized variants park them in LDS (same for every wave)
    // and re-read them when a key group's scales arrive; that frees 16 registers in the loop.
    h2v qpos[QUANT ? 1 : 16];
    if (!QUANT || wave == 0) {
        h2v qn[16];
        // (16-bit rows: step i of the contraction covers channels 32 i + 8 kb .. + 8, see k_lane)
        const uint16_t* qp = a.q + ((size_t)b * a.n_q_heads + g * GQ + (live_row ? h : 0)) * kHeadDim + (QUANT ? 32 : 8) * kb;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const uint4 v = *reinterpret_cast<const uint4*>(qp + (QUANT ? 8 : 32) * i);
            qn[4 * i] = as_h2(live_row ? v.x : 0u); qn[4 * i + 1] = as_h2(live_row ? v.y : 0u);
            qn[4 * i + 2] = as_h2(live_row ? v.z : 0u); qn[4 * i + 3] = as_h2(live_row ? v.w : 0u);
        }
#pragma unroll
        for (int s = 0; s < 4; ++s) {
            h2v t[4];
#pragma unroll
            for (int r = 0; r < 4; ++r) t[r] = qn[4 * s + r] * (_Float16)(1.0f / (float)(1 << k_pos_log2<BITS>(s, r)));
            if constexpr (QUANT) {
                // (per-token keys: the operand is q masked to the channel group of the lane's column, per pass)
#pragma unroll
                for (int ps = 0; ps < KP; ++ps) {
                    const bool keep = !KT || kt_mine[ps];
                    sqpos[(ps * 4 + s) * 64 + lane] = keep ? make_uint4(as_u32(t[0]), as_u32(t[1]), as_u32(t[2]), as_u32(t[3])) : make_uint4(0u, 0u, 0u, 0u);
                }
            } else {
#pragma unroll
                for (int r = 0; r < 4; ++r) qpos[4 * s + r] = t[r];
            }
        }
    }
    {   // plain copy (every variant: the tail rows read it too)
        for (int item = threadIdx.x; item < 8 * kHeadDim / 2; item += blockDim.x) {
            const int hh = item / (kHeadDim / 2), w = item % (kHeadDim / 2);
            const uint32_t v = hh < GQ ? reinterpret_cast<const uint32_t*>(a.q + ((size_t)b * a.n_q_heads + g * GQ + hh) * kHeadDim)[w] : 0u;
            reinterpret_cast<uint32_t*>(sq)[item] = v;
        }
    }
    if constexpr (OUT)
        for (int item = threadIdx.x; item < nw * 8 * kHeadDim; item += blockDim.x) s_oc[item] = 0.f;
    __syncthreads();   // query rows staged, chunk counter set
#pragma unroll
    for (int s = 0; s < 4; ++s)
#pragma unroll
        for (int r = 0; r < 4; ++r) bq[s].h[r] = (QUANT || part) ? (h2v){0, 0} : qpos[QUANT ? 0 : 4 * s + r];   // 16-bit cache: plain q in the hi rows
    if constexpr (KT) {
        float own = 0.f;                                  // sum of q over the lane's 32 channels
        const uint16_t* qrow = sq + h * kHeadDim + 32 * kb;
#pragma unroll
        for (int s = 0; s < 4; ++s) {
            const uint4 w = *reinterpret_cast<const uint4*>(qrow + 8 * s);
            const h2v a0 = as_h2(w.x), a1 = as_h2(w.y), a2 = as_h2(w.z), a3 = as_h2(w.w);
            own += ((float)a0[0] + (float)a0[1]) + ((float)a1[0] + (float)a1[1]) + ((float)a2[0] + (float)a2[1]) + ((float)a3[0] + (float)a3[1]);
        }
#pragma unroll
        for (int ps = 0; ps < KP; ++ps) kt_qs[ps] = quad_rows_add(kt_mine[ps] ? own : 0.f) * (1.0f / kCodeUnit);
    }
    // the tail rows go first, while the first blocks are on their way (their state waits in LDS)
    if (wave < kWaves) tail_rows<GQ>(a, bh, tail_t0, tail_t1, sT, sq, tail_k0, tail_v0);
    while (chunk < c_end) {
        if (!kEarlyB) load_B(chunk, two);
        const int next = claim();                            // used half an iteration later
        // key zero-point terms of this chunk's groups: token rows = z rows, unscaled q as the other operand
        float bias0 = 0.f, bias1 = 0.f;
        if constexpr (QUANT && !KT) {
#pragma unroll
            for (int i = 0; i < NGRP; ++i) lds_put(OFF_KZ + 256 * i, a_kz[i]);
            uint32_t zw[16], qw[16];
            lds_get16(OFF_KZ + 256 * min(n, NGRP - 1) + 64 * kb, zw);
            {
                // re-read q every chunk rather than pinning 16 registers for the whole loop
                const uint16_t* qrow = sq + h * kHeadDim + 32 * kb;
                asm volatile("" : "+v"(qrow));
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    const uint4 v = *reinterpret_cast<const uint4*>(qrow + 8 * i);
                    qw[4 * i] = v.x; qw[4 * i + 1] = v.y; qw[4 * i + 2] = v.z; qw[4 * i + 3] = v.w;
                }
            }
            f4v zc = (f4v){0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int s = 0; s < 4; ++s) {
                Frag zf, qf;
#pragma unroll
                for (int r = 0; r < 4; ++r) { zf.u[r] = zw[4 * s + r] & zrow_mask; qf.u[r] = qw[4 * s + r]; }
                zc = __builtin_amdgcn_mfma_f32_16x16x32_f16(zf.v, qf.v, zc, 0, 0, 0);
            }
            bias0 = quad_rows_add(zc[0]);                     // rows >= NGRP are zero, so the sum is a broadcast
            if constexpr (NGRP == 2) bias1 = quad_rows_add(zc[1]);
        }
        const bool has_next = next < c_end;
        const int nx = has_next ? next : chunk;
        const bool two_nx = n_kept - nx * kChunk > 32;
        float lgA[NT][4], lgB[NT][4];
        const uint2 no_slots = make_uint2(0u, 0u);
        if constexpr (kJoint) {
            // Both blocks' logits first, one move of the reference for the whole chunk, then both
            // blocks' softmax and PV products: one check per chunk instead of two, and each half of
            // the next chunk's loads leaves as soon as its registers are free.
            compute(BoolI<1>{}, lgA, ak0, ak1, a_ks, a_kz[0], true, bias0, av, 0, 0u, 0u, no_slots, no_slots, 0u, 0u, chunk * kChunk);
            if (!has_next) { k_off = 0; v_off = 0; row_off = 0; vrow_off = 0; slot_off = 0; }   // (wave-uniform; the loop ends after this pass)
            load_Ak(nx);
            float mx = lgA[0][0];
#pragma unroll
            for (int t = 0; t < NT; ++t)
#pragma unroll
                for (int i = 0; i < 4; ++i) mx = fmaxf(mx, lgA[t][i]);
            if (two) {
                compute(BoolI<1>{}, lgB, bk0, bk1, b_ks, b_kz, NGRP == 2, (NGRP == 2) ? bias1 : bias0, bv, 0, 0u, 0u, no_slots, no_slots, 0u, 0u, chunk * kChunk + 32);
#pragma unroll
                for (int t = 0; t < NT; ++t)
#pragma unroll
                    for (int i = 0; i < 4; ++i) mx = fmaxf(mx, lgB[t][i]);
            }
            load_Bk(nx, two_nx);
            advance_reference(quad_rows_max(mx));
            compute(BoolI<2>{}, lgA, ak0, ak1, 0u, 0u, true, 0.f, av, 0, a_vs, a_vz, no_slots, no_slots, 0u, 0u, 0);
            if constexpr (BITS == 2) bv = av;   // one 2-bit value word spans both blocks; keep it past the next prefetch
            load_Av(nx);
            if (two) compute(BoolI<2>{}, lgB, bk0, bk1, 0u, 0u, false, 0.f, bv, (BITS == 2) ? 1 : 0, b_vs, b_vz, no_slots, no_slots, 0u, 0u, 0);
            load_Bv(nx, two_nx);
        } else {
            compute(BoolI<0>{}, lgA, ak0, ak1, a_ks, a_kz[0], true, bias0, av, 0, a_vs, a_vz, a_ko, a_vo, a_kov, a_vov, chunk * kChunk);
            if constexpr (BITS == 2) bv = av;   // one 2-bit value word spans both blocks; keep it past the next prefetch
            // both blocks of the wave's next chunk are requested while this chunk's second block is computed
            if (!has_next) { k_off = 0; v_off = 0; row_off = 0; vrow_off = 0; slot_off = 0; }   // (wave-uniform; the loop ends after this pass)
            load_A(nx);
            if (two) compute(BoolI<0>{}, lgB, bk0, bk1, b_ks, b_kz, NGRP == 2, (NGRP == 2) ? bias1 : bias0, bv, (BITS == 2) ? 1 : 0, b_vs, b_vz, b_ko, b_vo, b_kov, b_vov,
                             chunk * kChunk + 32);
            if (kEarlyB) load_B(nx, two_nx);
        }
        chunk = next; two = two_nx;
    }

    // ---- merge the waves through LDS (one round), add the tail rows, write ----
    l_run = quad_rows_add(l_run);
#pragma unroll
    for (int c = 0; c < NCG; ++c) oz[c] = quad_rows_add(oz[c]);
    __syncthreads();                     // every wave has left the loop: its LDS is free for the states
    // rows 4kb+i come in (hi, lo) pairs i = (0,1), (2,3) with a common reference: add them here
#pragma unroll
    for (int t8 = 0; t8 < 8; ++t8) {
        sO[(wave * 8 + 2 * kb) * kHeadDim + 16 * t8 + n] = O[t8][0] + O[t8][1];
        sO[(wave * 8 + 2 * kb + 1) * kHeadDim + 16 * t8 + n] = O[t8][2] + O[t8][3];
    }
    if (kb == 0) {
        float* st = sS + (wave * 16 + n) * 6;
        st[0] = m_run - kPBoost; st[1] = l_run;   // (the reference the sums are relative to)
#pragma unroll
        for (int c = 0; c < NCG; ++c) st[2 + c] = oz[c];
    }
    __syncthreads();
    // One pair of output channels (head hh, channels d, d + 1) per thread: the common reference over
    // the waves' states and this workgroup's share of the full-precision tail rows (the first four
    // waves' states in sT), then one pass that weighs and adds them.  All threads of a head read the
    // same references and sums (LDS broadcasts); nw is a multiple of 4.
    const __amdgpu_buffer_rsrc_t part_rs = part_rsrc(a.part + (size_t)bh * a.n_partials * GQ * kPartFloats, (unsigned)a.n_partials * GQ * kPartFloats * 4u);
    for (int item = threadIdx.x; item < GQ * kPartPairs; item += blockDim.x) {
        const int hh = item / kPartPairs, d = 2 * (item % kPartPairs);
        const int cg = d / G;
        float M = kNegBig;
        for (int w0 = 0; w0 < nw; w0 += kWaves)
#pragma unroll
            for (int w = 0; w < kWaves; ++w)
#pragma unroll
                for (int sl = 0; sl < SLOTS; ++sl) M = fmaxf(M, sS[((w0 + w) * 16 + sl * 8 + 2 * hh) * 6]);
#pragma unroll
        for (int w = 0; w < kWaves; ++w) M = fmaxf(M, sT[(w * GQ + hh) * kPartStride]);
        float acc0 = 0.f, acc1 = 0.f, L = 0.f;
        for (int w0 = 0; w0 < nw; w0 += kWaves)
#pragma unroll
            for (int w = 0; w < kWaves; ++w)
#pragma unroll
                for (int sl = 0; sl < SLOTS; ++sl) {
                    const float* st = sS + ((w0 + w) * 16 + sl * 8 + 2 * hh) * 6;
                    const float2 ml = *reinterpret_cast<const float2*>(st);
                    const float wgt = __builtin_amdgcn_exp2f(ml.x - M);
                    const float2 o2 = *reinterpret_cast<const float2*>(sO + ((w0 + w) * 8 + sl * 4 + hh) * kHeadDim + d);
                    float o0 = o2.x * kCodeUnit + st[2 + cg], o1 = o2.y * kCodeUnit + st[2 + cg];
                    if constexpr (OUT) {
                        const float2 c2 = *reinterpret_cast<const float2*>(s_oc + ((w0 + w) * 8 + sl * 4 + hh) * kHeadDim + d);
                        o0 += c2.x; o1 += c2.y;
                    }
                    acc0 = __builtin_fmaf(wgt, o0, acc0);
                    acc1 = __builtin_fmaf(wgt, o1, acc1);
                    L = __builtin_fmaf(wgt, ml.y, L);
                }
#pragma unroll
        for (int w = 0; w < kWaves; ++w) {
            const float* row = sT + (w * GQ + hh) * kPartStride;
            const float2 ml = *reinterpret_cast<const float2*>(row);
            const float2 o2 = *reinterpret_cast<const float2*>(row + 2 + d);
            const float wgt = __builtin_amdgcn_exp2f(ml.x - M);
            acc0 = __builtin_fmaf(wgt, o2.x, acc0);
            acc1 = __builtin_fmaf(wgt, o2.y, acc1);
            L = __builtin_fmaf(wgt, ml.y, L);
        }
        if (n_parts == 1) {      // the whole head was here: normalise, round once, done
            const uint32_t lo = __half_as_ushort(__float2half_rn(acc0 / L)), hi = __half_as_ushort(__float2half_rn(acc1 / L));
            reinterpret_cast<uint32_t*>(a.out + ((size_t)b * a.n_q_heads + g * GQ + hh) * kHeadDim)[d >> 1] = lo | (hi << 16);
        } else {                 // this split's record of the pair, reference and sum beside it
            st_dev16(part_rs, (unsigned)((blockIdx.x * GQ + hh) * kPartPairs + (d >> 1)) * 16u, M, L, acc0, acc1);
        }
    }
    if (n_parts == 1) return;
    merge_if_last<GQ>(a, bh, n_parts);
}

// Which chunks of every head a launch reads with the non-temporal hint (streamed round the 256 MB
// memory-side cache) -- chunks from the returned index on.  A decode step reads every layer's cache
// exactly once and a model's weights pass through the chip between two steps, so nothing of a cache
// survives there until it is read again; loads that merely pass through that cache run slower than
// loads that go round it (measured with launches that rotate over several caches: 4 bits 65.2 ->
// 60.4 us, 8 bits 57.3 -> 53.8 us, 16 bits 55.6 -> 52.9 us per 256-head launch).  So the library
// streams everything unless the caller says the cache will still be resident (KVQP_CACHE_KEEP).
constexpr int kNoStream = 0x7fffffff;
static int stream_from_chunk(const kvqp_cfg& cfg, int n_kept) {
    (void)n_kept;
    return cfg.decode_cache_hint == KVQP_CACHE_KEEP ? kNoStream : 0;
}

template <int BITS, int GQ, int NCG>
hipError_t launch_axis(const kvqp_cfg& cfg, const DecodeArgs& a, hipStream_t stream) {
    const dim3 grid(a.n_partials, cfg.batch * cfg.n_kv_heads);
    const bool out = BITS != 16 && a.k_out != nullptr;
    const bool token_keys = BITS != 16 && cfg.key_axis == KVQP_KEY_PER_TOKEN;
    const unsigned lds_bytes = (out ? pipe_lds_bytes(a.n_waves, PipeGeom<BITS, NCG, true>::STRIP, GQ, true)
                                    : pipe_lds_bytes(a.n_waves, PipeGeom<BITS, NCG, false>::STRIP, GQ, false)) + 16;
    const dim3 block(64 * a.n_waves);
    // (more than 64 KB of dynamic LDS has to be asked for: the variants with outlier terms can need it)
    auto go = [&](auto kernel) {
        if (lds_bytes > 65536u &&
            hipFuncSetAttribute(reinterpret_cast<const void*>(kernel), hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds_bytes) != hipSuccess)
            return;
        hipLaunchKernelGGL(kernel, grid, block, lds_bytes, stream, a);
    };
    if constexpr (BITS != 16) {
        if (out && token_keys) go(decode_attn_pipe<BITS, GQ, NCG, 1, true>);
        else if (out) go(decode_attn_pipe<BITS, GQ, NCG, 0, true>);
        else if (token_keys) go(decode_attn_pipe<BITS, GQ, NCG, 1, false>);
        else go(decode_attn_pipe<BITS, GQ, NCG, 0, false>);
    } else {
        go(decode_attn_pipe<BITS, GQ, NCG, 0, false>);
    }
    return hipGetLastError();
}
template <int BITS, int GQ>
hipError_t launch_group(const kvqp_cfg& cfg, const DecodeArgs& a, hipStream_t stream) {
    if (BITS == 16) return launch_axis<BITS, GQ, 1>(cfg, a, stream);
    switch (cfg.group_size) {
        case 32: return launch_axis<BITS, GQ, 4>(cfg, a, stream);
        case 64: return launch_axis<BITS, GQ, 2>(cfg, a, stream);
        default: return launch_axis<BITS, GQ, 1>(cfg, a, stream);
    }
}
template <int BITS>
hipError_t launch_gq(const kvqp_cfg& cfg, const DecodeArgs& a, hipStream_t stream) {
    switch (cfg.n_q_heads / cfg.n_kv_heads) {
        case 1: return launch_group<BITS, 1>(cfg, a, stream);
        case 2: return launch_group<BITS, 2>(cfg, a, stream);
        case 4: return launch_group<BITS, 4>(cfg, a, stream);
        default: return launch_group<BITS, 8>(cfg, a, stream);
    }
}

}  // namespace

static int cu_count() {
    static const int n_cu = [] {
        int dev = 0, v = 0;
        if (hipGetDevice(&dev) != hipSuccess || hipDeviceGetAttribute(&v, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || v <= 0) v = 256;
        return v;
    }();
    return n_cu;
}

// Workspace that covers the plan of every cache of this cfg's batch, heads and bits, whatever its
// token count: no plan has more splits than the head's share of the chip in four-wave workgroups
// (or the caller's decode_splits).
size_t decode_ws_header_bytes(const kvqp_cfg& cfg) {
    return ((size_t)cfg.batch * cfg.n_kv_heads * sizeof(unsigned int) + 255) / 256 * 256;
}

size_t decode_ws_bound(const kvqp_cfg& cfg) {
    const int heads = cfg.batch * cfg.n_kv_heads, gq = cfg.n_q_heads / cfg.n_kv_heads;
    const int share = (cu_count() * pipe_max_waves(cfg.bits, gq, outliers_on(cfg))) / heads;
    int splits = (share + kWaves - 1) / kWaves;
    if (cfg.decode_splits > splits) splits = cfg.decode_splits;
    if (splits < 1) splits = 1;
    return decode_ws_header_bytes(cfg) + (size_t)heads * splits * gq * kPartFloats * sizeof(float);
}

DecodePlan plan_decode(const kvqp_cfg& cfg, int n_kept, int tail_len) {
    DecodePlan p;
    const int heads = cfg.batch * cfg.n_kv_heads;
    const int n_chunks = (n_kept + kChunk - 1) / kChunk;
    const int gq = cfg.n_q_heads / cfg.n_kv_heads;
    {
        // Every workgroup takes a token range and a share of the tail rows.  By default the launch
        // is one resident round: as many workgroups as the chip holds at the kernel's occupancy.
        const int n_cu = cu_count();
        // Waves a head may use: its share of what the chip holds at this kernel's occupancy, but no
        // more than it has 64-token chunks.
        const int max_nw = pipe_max_waves(cfg.bits, gq, outliers_on(cfg));
        int waves = (n_cu * max_nw) / heads;
        if (waves > n_chunks) waves = n_chunks;
        int splits, nw;
        if (cfg.decode_splits > 0) {            // caller's choice: that many four-wave workgroups
            splits = cfg.decode_splits < n_chunks ? cfg.decode_splits : n_chunks;
            nw = kWaves;
        } else if (waves <= max_nw) {           // one workgroup per head: no partials, no merge across workgroups
            splits = 1;
            nw = waves / kWaves * kWaves;
        } else {                                // several workgroups per head: small ones while CUs are left over
            nw = (int)((long long)waves * heads / n_cu) / kWaves * kWaves;
            // (a head is kept within sixteen partials by making the workgroups larger rather than more:
            // the last workgroup fetches 1 KB per partial and query head through its own CU, and 32
            // four-wave workgroups per head measured slower than 16 of eight waves)
            const int nw16 = ((waves + 15) / 16 + kWaves - 1) / kWaves * kWaves;
            if (nw < nw16) nw = nw16;
            if (nw > max_nw) nw = max_nw;
            if (nw < kWaves) nw = kWaves;
            splits = (waves + nw - 1) / nw;
        }
        if (splits < 1) splits = 1;
        if (nw < kWaves) nw = kWaves;
        p.n_waves = nw;
        p.chunks_per_split = (n_chunks + splits - 1) / splits;
        p.n_splits = p.chunks_per_split ? (n_chunks + p.chunks_per_split - 1) / p.chunks_per_split : 1;
        p.n_partials = p.n_splits;
    }
    // (a head that stays in one workgroup writes no partial: the counters' bytes are all the launch touches)
    p.ws_bytes = decode_ws_header_bytes(cfg) + (p.n_splits > 1 ? (size_t)heads * (size_t)p.n_partials * gq * kPartFloats * sizeof(float) : 0);
    return p;
}

// Zeroes the arrival counters of a workspace (a fill kernel, not a memset node: callers may capture it).
__global__ void zero_words(unsigned int* p, int n) {
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) p[i] = 0u;
}
hipError_t launch_ws_init(const kvqp_cfg& cfg, void* ws, hipStream_t stream) {
    const int n = (int)(decode_ws_header_bytes(cfg) / sizeof(unsigned int));
    hipLaunchKernelGGL(zero_words, dim3((n + 255) / 256), dim3(256), 0, stream, (unsigned int*)ws, n);
    return hipGetLastError();
}

// ---- the library-owned decode workspace (the array `scratch` at the top of this file) ----
namespace {
constexpr int kMaxDevices = 64;
std::mutex g_scratch_mutex;
void* g_scratch_ptr[kMaxDevices];     // per device: the address of its copy of `scratch`, or NULL
}

hipError_t static_scratch(const kvqp_cfg& cfg, void** ptr, hipStream_t stream) {
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    if (dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice;
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
        void* p = nullptr;
        e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess) return e;
        if (!p) return hipErrorInvalidSymbol;
        // counters for the largest head count the launches accept (a fill kernel: the call may be under capture)
        constexpr int n = 65536;
        static_assert((size_t)n * sizeof(unsigned int) <= kStaticScratchBytes, "counters fit the array");
        hipLaunchKernelGGL(zero_words, dim3(n / 256), dim3(256), 0, stream, (unsigned int*)p, n);
        e = hipGetLastError();
        if (e != hipSuccess) return e;
        g_scratch_ptr[dev] = p;
    }
    (void)cfg;
    *ptr = g_scratch_ptr[dev];
    return hipSuccess;
}

hipError_t launch_decode(const kvqp_cfg& cfg, const void* q, const kvqp_cache& c, void* out, void* ws,
                         const DecodePlan& plan, hipStream_t stream) {
    DecodeArgs a;
    a.q = (const uint16_t*)q;
    a.k_codes = (const uint32_t*)c.k_codes; a.v_codes = (const uint32_t*)c.v_codes;
    a.k_scale = (const uint16_t*)c.k_scale; a.k_zero = (const uint16_t*)c.k_zero;
    a.v_scale = (const uint16_t*)c.v_scale; a.v_zero = (const uint16_t*)c.v_zero;
    a.tail_k = (const uint16_t*)c.tail_k; a.tail_v = (const uint16_t*)c.tail_v;
    a.arrivals = (unsigned int*)ws;
    a.part = (float*)(static_cast<char*>(ws) + decode_ws_header_bytes(cfg));
    a.out = (uint16_t*)out;
    a.n_kept = c.n_kept; a.tail_len = c.tail_len; a.tail_cap = c.tail_cap;
    a.n_cap = layout_tokens(c, c.n_kept);
    a.head_n_kept = c.head_n_kept;
    a.k_out = outliers_on(cfg) ? (const uint32_t*)c.k_out : nullptr;
    a.v_out = outliers_on(cfg) ? (const uint32_t*)c.v_out : nullptr;
    a.k_ovf = outliers_on(cfg) ? (const uint32_t*)c.k_ovf : nullptr;
    a.v_ovf = outliers_on(cfg) ? (const uint32_t*)c.v_ovf : nullptr;
    a.ovf_cap = cfg.outlier_overflow_cap;
    a.n_q_heads = cfg.n_q_heads; a.n_kv_heads = cfg.n_kv_heads;
    a.n_splits = plan.n_splits; a.chunks_per_split = plan.chunks_per_split; a.n_partials = plan.n_partials;
    a.n_waves = plan.n_waves;
    a.group = cfg.group_size; a.sm_scale = cfg.sm_scale;
    a.stream_from = stream_from_chunk(cfg, c.n_kept);
    hipError_t e;
    switch (cfg.bits) {
        case 2: e = launch_gq<2>(cfg, a, stream); break;
        case 4: e = launch_gq<4>(cfg, a, stream); break;
        case 8: e = launch_gq<8>(cfg, a, stream); break;
        default: e = launch_gq<16>(cfg, a, stream); break;
    }
    return e;
}

}  // namespace kvqp
