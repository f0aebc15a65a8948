// Gather the surviving tokens, quantize them group by group and write the
// packed cache (paper Section 3, "KV Quantization": z = min, m = max,
// s = (m - z)/(2^B - 1), Q(G) = round((G - z)/s); grouping axes of Section 2 /
// Section 6.3).  Every survivor row is read once (2 x 256 B, scattered) and
// k*bpt bytes are written; there is no reuse to exploit.  What bounds it on
// the MI355X, measured: not the scattered rows (contiguous survivors take the
// same time) and not the instruction count alone (order keys, the quantizer's
// individually rounded binary32 steps, field packing: ~18 lane operations per
// element), but a workgroup's own chain of waits -- two memory round trips,
// three barriers -- that the six workgroups a CU holds at 78 registers do not
// fully hide; it moves ~4.7 TB/s of gathers and stores.
//
// One workgroup owns TB consecutive kept tokens of one (batch, kv head): whole
// key groups (G | TB) and whole value superblocks (SB | TB).  Thread
// (r = tid / 16, c8 = tid % 16) keeps channels 8 c8 .. 8 c8 + 7 of rows
// r, r + 16, r + 32, ... in registers from the gather to the packed words:
//   * minima / maxima are taken on packed 16-bit order keys (two channels per
//     register), across lanes with DPP / permlane exchanges and across waves
//     through a few hundred bytes of LDS;
//   * key words are assembled in registers and stored straight from them
//     (a word holds consecutive channels of one token);
//   * value words hold one channel of several tokens (the tile-transposed
//     layout of kvqp.h): wave kb owns tokens 4 kb + i, lanes OR their fields
//     together, and the finished superblocks leave through LDS as 16-byte
//     coalesced stores.
#include "kvqp_internal.h"

namespace kvqp {
namespace {

constexpr int kThreads = 256;

// One launch of the quantize-and-pack kernel: n_tok rows per head of (k, v) -- rows idx[...] or, with
// idx == NULL, rows 0 .. n_tok-1 -- land at tokens dst_base .. of a cache laid out for n_cap tokens.
struct QuantPackJob {
    const kvqp_cache& c;
    const void* k; const void* v; const int32_t* idx;
    const int32_t* head_n;   // device: rows of each head (<= n_tok, whole groups), or NULL for n_tok everywhere
    uint32_t tau_bits;       // outlier filtering: |x| is above the threshold iff its binary16 pattern exceeds this
    bool outliers;
    int heads, src_rows, window, n_tok, dst_base, n_cap, bits, group_size, key_axis;
    bool copy_tail;
    const int32_t* head_base = nullptr;   // device: first destination token of each head in place of dst_base, or NULL
    int base_quantum = 1;                 // what every head_base entry is a multiple of
    int ovf_cap = 0;                      // outlier filtering: entries of a head's overflow list
};

typedef unsigned short us2v __attribute__((ext_vector_type(2)));
__device__ __forceinline__ uint32_t pk_min(uint32_t a, uint32_t b) {
    union { uint32_t u; us2v v; } x, y, z; x.u = a; y.u = b; z.v = __builtin_elementwise_min(x.v, y.v); return z.u;
}
__device__ __forceinline__ uint32_t pk_max(uint32_t a, uint32_t b) {
    union { uint32_t u; us2v v; } x, y, z; x.u = a; y.u = b; z.v = __builtin_elementwise_max(x.v, y.v); return z.u;
}

// binary16 bit pattern -> key that orders like the value (-0 below +0).
__device__ __forceinline__ uint32_t order_key(uint16_t h) { return (h & 0x8000u) ? (uint16_t)~h : (uint16_t)(h | 0x8000u); }
// the same on both halves of a word
__device__ __forceinline__ uint32_t order_key2(uint32_t w) {
    const uint32_t neg = (w >> 15) & 0x00010001u;
    return w ^ (0x80008000u | (neg * 0x7fffu));
}
__device__ __forceinline__ uint16_t key_to_half(uint32_t key) { return (key & 0x8000u) ? (uint16_t)(key & 0x7fffu) : (uint16_t)~key; }
__device__ __forceinline__ float half_bits_to_float(uint16_t h) { return __half2float(__ushort_as_half(h)); }

// The quantizer's binary32 sequence; every operation individually rounded.
struct GroupParams {
    uint16_t scale_h, zero_h;
    float zf, inv;   // inv == 0 marks the degenerate group (all codes 0)
};
template <int BITS>
__device__ __forceinline__ GroupParams group_params(uint32_t kmin, uint32_t kmax) {
    GroupParams g;
    g.zero_h = key_to_half(kmin);
    const uint16_t mh = key_to_half(kmax);
    g.zf = half_bits_to_float(g.zero_h);
    const float r = __fsub_rn(half_bits_to_float(mh), g.zf);
    const float s32 = __fdiv_rn(r, (float)((1 << BITS) - 1));
    const __half sh = __float2half_rn(s32);
    g.scale_h = __half_as_ushort(sh);
    const float sf = __half2float(sh);
    g.inv = (sf == 0.0f) ? 0.0f : __fdiv_rn(1.0f, sf);
    return g;
}
template <int BITS>
__device__ __forceinline__ uint32_t encode(uint16_t xh, const GroupParams& g) {
    // a degenerate group needs no branch: (x - z) * 0 rounds and clamps to code 0
    float c = rintf(__fmul_rn(__fsub_rn(half_bits_to_float(xh), g.zf), g.inv));
    c = fminf(fmaxf(c, 0.0f), (float)((1 << BITS) - 1));
    return (uint32_t)c;
}

// lane exchanges: partner lane ^ 16 / ^ 32 (both values come back, combine them with any symmetric op)
#define KVQP_SWAP16(v) __builtin_amdgcn_permlane16_swap((v), (v), false, false)
#define KVQP_SWAP32(v) __builtin_amdgcn_permlane32_swap((v), (v), false, false)
template <int CTRL> __device__ __forceinline__ uint32_t dpp(uint32_t v) { return __builtin_amdgcn_update_dpp(0u, v, CTRL, 0xF, 0xF, true); }
constexpr int kQuadXor1 = 0xB1, kQuadXor2 = 0x4E, kRowHalfMirror = 0x141, kRowMirror = 0x140;

// min / max over the LANES consecutive lanes (4, 8 or 16) that share a per-token group
template <int LANES> __device__ __forceinline__ void group_minmax(uint32_t& mn, uint32_t& mx) {
    mn = min(mn, dpp<kQuadXor1>(mn)); mx = max(mx, dpp<kQuadXor1>(mx));
    mn = min(mn, dpp<kQuadXor2>(mn)); mx = max(mx, dpp<kQuadXor2>(mx));
    if (LANES >= 8) { mn = min(mn, dpp<kRowHalfMirror>(mn)); mx = max(mx, dpp<kRowHalfMirror>(mx)); }
    if (LANES >= 16) { mn = min(mn, dpp<kRowMirror>(mn)); mx = max(mx, dpp<kRowMirror>(mx)); }
}

// codes of a thread's eight channels of one row
template <int BITS>
__device__ __forceinline__ void encode8(const uint32_t (&w)[4], const float (&zf)[8], const float (&inv)[8], uint32_t (&c)[8]) {
#pragma unroll
    for (int q = 0; q < 4; ++q) {
        GroupParams g0, g1;
        g0.zf = zf[2 * q]; g0.inv = inv[2 * q]; g1.zf = zf[2 * q + 1]; g1.inv = inv[2 * q + 1];
        c[2 * q] = encode<BITS>((uint16_t)(w[q] & 0xffffu), g0);
        c[2 * q + 1] = encode<BITS>((uint16_t)(w[q] >> 16), g1);
    }
}

// the same when all eight channels share one group
template <int BITS>
__device__ __forceinline__ void encode8(const uint32_t (&w)[4], float zf, float inv, uint32_t (&c)[8]) {
    GroupParams g; g.zf = zf; g.inv = inv;
#pragma unroll
    for (int q = 0; q < 4; ++q) {
        c[2 * q] = encode<BITS>((uint16_t)(w[q] & 0xffffu), g);
        c[2 * q + 1] = encode<BITS>((uint16_t)(w[q] >> 16), g);
    }
}

// Key words of one row from the thread's eight codes (row-major layout of kvqp.h: channel d sits in
// word d / E at half-word r % 2, field r / 2, r = d % E) and their store.  krow points at the row.
// keep: all ones, or 0 for a padding row (its words are stored as zeros).
template <int BITS>
__device__ __forceinline__ void store_key_words(uint32_t* krow, int c8, const uint32_t (&c)[8], uint32_t keep = 0xFFFFFFFFu) {
    constexpr int E = 32 / BITS;
    if constexpr (E == 8) {
        uint32_t w = 0;
#pragma unroll
        for (int dd = 0; dd < 8; ++dd) w |= c[dd] << (16 * (dd & 1) + BITS * (dd >> 1));
        krow[c8] = w & keep;
    } else if constexpr (E == 4) {
        uint32_t w0 = 0, w1 = 0;
#pragma unroll
        for (int dd = 0; dd < 4; ++dd) {
            w0 |= c[dd] << (16 * (dd & 1) + BITS * (dd >> 1));
            w1 |= c[4 + dd] << (16 * (dd & 1) + BITS * (dd >> 1));
        }
        *reinterpret_cast<uint2*>(krow + 2 * c8) = make_uint2(w0 & keep, w1 & keep);
    } else {   // E == 16: the word spans this lane's channels and its neighbour's
        uint32_t w = 0;
#pragma unroll
        for (int dd = 0; dd < 8; ++dd) {
            const int r = dd;   // position inside the lane's half of the word
            w |= c[dd] << (16 * (r & 1) + BITS * (r >> 1));
        }
        // odd lanes hold channels 8..15 of the word: fields 4..7 of each half-word
        if (c8 & 1) w <<= 4 * BITS;
        w |= dpp<kQuadXor1>(w);
        if (!(c8 & 1)) krow[c8 >> 1] = w & keep;
    }
}

// all 16 lanes of a row of lanes (one token row) get the largest value among them
__device__ __forceinline__ uint32_t row16_max(uint32_t v) {
    v = max(v, dpp<kQuadXor1>(v)); v = max(v, dpp<kQuadXor2>(v));
    v = max(v, dpp<kRowHalfMirror>(v)); v = max(v, dpp<kRowMirror>(v));
    return v;
}
// sum over the 16 lanes of a row, in every lane; and the sum over the lanes before this one
__device__ __forceinline__ uint32_t row16_sum(uint32_t v) {
    v += dpp<kQuadXor1>(v); v += dpp<kQuadXor2>(v); v += dpp<kRowHalfMirror>(v); v += dpp<kRowMirror>(v);
    return v;
}
__device__ __forceinline__ uint32_t row16_before(uint32_t v) {
    uint32_t s = v;
    s += dpp<0x111>(s); s += dpp<0x112>(s); s += dpp<0x114>(s); s += dpp<0x118>(s);   // row_shr 1, 2, 4, 8 (zeros shifted in)
    return s - v;
}
// 0xFFFF in the half-words whose bit (bit 0: low half, bit 1: high half) is set
__device__ __forceinline__ uint32_t half_mask(uint32_t b) { return ((0u - (b & 1u)) & 0xFFFFu) | ((0u - ((b >> 1) & 1u)) << 16); }

template <int BITS, int G, bool OUT>
__global__ __launch_bounds__(kThreads) void gather_quant_pack(
    const uint16_t* __restrict__ k, const uint16_t* __restrict__ v, const int32_t* __restrict__ idx,
    uint32_t* __restrict__ k_codes, uint32_t* __restrict__ v_codes, uint16_t* __restrict__ k_scale,
    uint16_t* __restrict__ k_zero, uint16_t* __restrict__ v_scale, uint16_t* __restrict__ v_zero,
    uint16_t* __restrict__ tail_k, uint16_t* __restrict__ tail_v, int L, int W, int n_kept, int key_axis,
    int tail_cap, int n_tok_blocks, int n_cap, int dst_base, const int32_t* __restrict__ head_n,
    uint32_t* __restrict__ k_out, uint32_t* __restrict__ v_out, uint32_t tau_bits,
    const int32_t* __restrict__ head_base, int base_quantum, uint32_t* __restrict__ k_ovf,
    uint32_t* __restrict__ v_ovf, int ovf_cap) {
    // L: rows per head of the source tensors.  idx: source row of every token of this call
    // ([heads, n_kept]), or NULL for rows 0 .. n_kept-1.  The tokens land at positions dst_base ..
    // dst_base + n_kept - 1 of a cache whose buffers are laid out for n_cap tokens per head.
    // head_n: a head's own token count in place of n_kept (idx keeps its stride of n_kept), or NULL.
    // head_base: a head's own first position in place of dst_base, or NULL; it is cut to dst_base and
    // rounded down to a multiple of base_quantum, so whatever the array holds the stores stay inside
    // the buffers and on group and superblock boundaries.
    // OUT: outlier filtering; k_out / v_out receive four slot words per token row, and the number of
    // a block's further outliers is left at entry (block + 1) of the head's overflow prefix array
    // (k_ovf / v_ovf), which ovf_scan then turns into prefix counts and ovf_fill completes.
    constexpr bool QUANT = BITS != 16;
    constexpr int TB = (QUANT && G == 128) ? 128 : 64;   // tokens per workgroup
    constexpr int R = TB / 16;                            // rows per thread
    constexpr int NG = TB / G > 0 ? TB / G : 1;           // per-channel key groups per workgroup
    constexpr int JPG = G / 16;                           // a thread's rows per key group
    constexpr int CPT = kHeadDim / G;                     // per-token groups per row
    constexpr int GL = G / 8;                             // lanes per per-token group
    constexpr int E = 32 / BITS;
    constexpr int SB = v_superblock(BITS);
    constexpr int WPT = v_words_per_tile(BITS);
    constexpr int SBW = v_superblock_words(BITS);
    constexpr int NSB = TB / SB;
    __shared__ __align__(16) uint32_t s_words[NSB * SBW];                 // finished value superblocks
    __shared__ __align__(16) uint16_t s_min[QUANT ? 4 * NG * kHeadDim : 8];   // per wave: channel minima / maxima (order keys)
    __shared__ __align__(16) uint16_t s_max[QUANT ? 4 * NG * kHeadDim : 8];
    __shared__ __align__(16) float2 s_par[QUANT ? NG * kHeadDim : 1];     // (z, 1/s) per (key group, channel)
    __shared__ int s_cnt[2][OUT ? TB / 32 : 1];                           // OUT: outliers beyond the slots per 32-token block (keys, values)

    const int head = blockIdx.y;
    const uint16_t* kh = k + (size_t)head * L * kHeadDim;
    const uint16_t* vh = v + (size_t)head * L * kHeadDim;

    if ((int)blockIdx.x >= n_tok_blocks) {
        // Tail: the last W prompt rows stay at full precision.
        const int P = L - W;
        for (int item = threadIdx.x; item < W * 16; item += kThreads) {
            const int t = item >> 4, c = item & 15;
            const size_t src = (size_t)(P + t) * kHeadDim + c * 8, dst = ((size_t)head * tail_cap + t) * kHeadDim + c * 8;
            *reinterpret_cast<uint4*>(tail_k + dst) = *reinterpret_cast<const uint4*>(kh + src);
            *reinterpret_cast<uint4*>(tail_v + dst) = *reinterpret_cast<const uint4*>(vh + src);
        }
        return;
    }

    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int c8 = threadIdx.x & 15, r = threadIdx.x >> 4, i4 = (threadIdx.x >> 4) & 3;
    const int t0 = blockIdx.x * TB;
    int base = dst_base;
    if (head_base) {
        base = min(max(head_base[head], 0), dst_base);
        base -= base % base_quantum;
    }
    const int d0 = base + t0;                // first destination token: a multiple of the group and superblock sizes
    const int n_head = head_n ? head_n[head] : n_kept;
    if (t0 >= n_head) return;                // (the whole workgroup: nothing of this head left)
    const int ntok = min(TB, n_head - t0);   // any count: the head's last block and last key group may be partly filled
    const int ntok_pad = rows32(ntok);       // rows of the last block past the count are written as zeros
    if constexpr (OUT) {
        if (threadIdx.x < 2 * (TB / 32)) (&s_cnt[0][0])[threadIdx.x] = 0;
        __syncthreads();
    }

    // ---- gather: all of the thread's rows of both tensors are requested before anything is used.
    // The row numbers come first, all of them, and then every row load leaves without waiting for
    // another (two round trips to memory instead of one per row); a row past the count reads the
    // block's last row instead, so no load depends on a branch, and is cleared afterwards. ----
    uint32_t kw[R][4], vw[R][4];
    bool live[R];
    int pos[R];
#pragma unroll
    for (int j = 0; j < R; ++j) {
        live[j] = r + 16 * j < ntok;      // (the same for the 16 lanes of a token row)
        pos[j] = t0 + min(r + 16 * j, ntok - 1);
    }
    if (idx) {                            // (uniform)
        const int32_t* rows = idx + (size_t)head * n_kept;
#pragma unroll
        for (int j = 0; j < R; ++j) pos[j] = rows[pos[j]];
    }
#pragma unroll
    for (int j = 0; j < R; ++j) {
        // (prompt rows are read once: non-temporal)
        typedef uint32_t u4v __attribute__((ext_vector_type(4)));
        const u4v a = __builtin_nontemporal_load(reinterpret_cast<const u4v*>(kh + (size_t)pos[j] * kHeadDim + 8 * c8));
        const u4v b = __builtin_nontemporal_load(reinterpret_cast<const u4v*>(vh + (size_t)pos[j] * kHeadDim + 8 * c8));
        kw[j][0] = a[0]; kw[j][1] = a[1]; kw[j][2] = a[2]; kw[j][3] = a[3];
        vw[j][0] = b[0]; vw[j][1] = b[1]; vw[j][2] = b[2]; vw[j][3] = b[3];
    }
    if (ntok < TB) {                      // (uniform) the head's last block: rows past the count are zeros
#pragma unroll
        for (int j = 0; j < R; ++j)
            if (!live[j]) {
#pragma unroll
                for (int q = 0; q < 4; ++q) { kw[j][q] = 0u; vw[j][q] = 0u; }
            }
    }

    // Outlier marking (OUT): om gets a bit per own element whose magnitude is above the threshold --
    // every such element of the row is an outlier (Section 6.3 item (1): no limit per row).
    auto mark = [&](const uint32_t (&w)[R][4], uint32_t (&om)[R]) {
#pragma unroll
        for (int j = 0; j < R; ++j) {
            uint32_t cand = 0u;
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                const uint32_t mag = (w[j][e >> 1] >> (16 * (e & 1))) & 0x7fffu;
                cand |= mag > tau_bits ? (1u << e) : 0u;
            }
            om[j] = cand;
        }
    };
    // slot word of element x (binary16 pattern) in channel ch given its group's zero
    auto slot_word = [](uint32_t xh, uint32_t ch, float zf) -> uint32_t {
        const float diff = __fsub_rn(half_bits_to_float((uint16_t)xh), zf);
        return (__float_as_uint(diff) & 0xFFFFFF00u) | 0x80u | ch;
    };
    // Slot words of the rows: an outlier's index is the number of outliers before it in the row
    // (lanes before this one, then the lane's own earlier elements); the first four go to the row's
    // slots in that (ascending channel) order, lanes 0-3 of the row clear the unused slots.  Outliers
    // beyond the fourth belong to the head's overflow list, which a later kernel fills; here they are
    // only counted per block of 32 tokens (cnt, in LDS).  zero_of(j, e): the zero of element e's group in row j.
    auto store_slots = [&](uint32_t* out, int* cnt, const uint32_t (&w)[R][4], const uint32_t (&om)[R], auto zero_of) {
#pragma unroll
        for (int j = 0; j < R; ++j) {
            if (!live[j]) {                                           // (uniform over the row's 16 lanes)
                if (r + 16 * j < ntok_pad && c8 < 4) out[((size_t)head * n_cap + d0 + r + 16 * j) * 4 + c8] = 0u;   // padding row: no outliers
                continue;
            }
            const uint32_t mine = (uint32_t)__builtin_popcount(om[j]);
            const uint32_t total = row16_sum(mine);
            uint32_t at = row16_before(mine);
            uint32_t* row = out + ((size_t)head * n_cap + d0 + r + 16 * j) * 4;
            if (c8 < 4 && (uint32_t)c8 >= total) row[c8] = 0u;
            if (__builtin_amdgcn_ballot_w64(om[j] != 0u) == 0ull) continue;
            if (c8 == 0 && total > 4u) atomicAdd(&cnt[j >> 1], (int)(total - 4u));
#pragma unroll
            for (int e = 0; e < 8; ++e)
                if ((om[j] >> e) & 1u) {
                    const uint32_t xh = (w[j][e >> 1] >> (16 * (e & 1))) & 0xffffu;
                    if (at < 4u) row[at] = slot_word(xh, (uint32_t)(8 * c8 + e), zero_of(j, e));
                    ++at;
                }
        }
    };

    // Per-token groups (values always, keys on that axis): every row is complete inside GL lanes.
    // Fills the codes of all rows and stores scale / zero.  Lane q of a quad derives the parameters
    // of rows q, q + 4, ... and hands them to the other three.  om: outlier bits (OUT); zrow: float
    // bits of the zero of the lane's own group, per row.
    auto per_token = [&](const uint32_t (&w)[R][4], uint16_t* scale, uint16_t* zero, uint32_t (&codes)[R][8],
                         const uint32_t (&om)[R], uint32_t (&zrow)[R]) {
        uint32_t mn[R], mx[R];
#pragma unroll
        for (int j = 0; j < R; ++j) {
            uint32_t lo = 0xffffffffu, hi = 0u;
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const uint32_t a = order_key2(w[j][q]);
                const uint32_t ex = OUT ? half_mask(om[j] >> (2 * q)) : 0u;   // excluded halves: neutral for min and max
                lo = pk_min(lo, a | ex); hi = pk_max(hi, a & ~ex);
            }
            mn[j] = min(lo & 0xffffu, lo >> 16); mx[j] = max(hi & 0xffffu, hi >> 16);
            group_minmax<GL>(mn[j], mx[j]);
            if (OUT && mn[j] > mx[j]) { mn[j] = 0x8000u; mx[j] = 0x8000u; }   // nothing left in the group: zero +0, scale 0
        }
        const int q4 = c8 & 3;
#pragma unroll
        for (int jj = 0; jj < R / 4; ++jj) {
            const uint32_t a = q4 == 0 ? mn[4 * jj] : q4 == 1 ? mn[4 * jj + 1] : q4 == 2 ? mn[4 * jj + 2] : mn[4 * jj + 3];
            const uint32_t b = q4 == 0 ? mx[4 * jj] : q4 == 1 ? mx[4 * jj + 1] : q4 == 2 ? mx[4 * jj + 2] : mx[4 * jj + 3];
            const GroupParams gp = group_params<BITS>(a, b);
            const int t = r + 16 * (4 * jj + q4);
            if (t < ntok_pad && (c8 & (GL - 1)) < 4) {               // (a padding row of the last block was loaded as zeros: scale 0, zero +0)
                const size_t m = ((size_t)head * n_cap + d0 + t) * CPT + c8 / GL;
                scale[m] = gp.scale_h; zero[m] = gp.zero_h;
            }
            const uint32_t zb = __float_as_uint(gp.zf), ib = __float_as_uint(gp.inv);
            const uint32_t zq[4] = {dpp<0x00>(zb), dpp<0x55>(zb), dpp<0xAA>(zb), dpp<0xFF>(zb)};
            const uint32_t iq[4] = {dpp<0x00>(ib), dpp<0x55>(ib), dpp<0xAA>(ib), dpp<0xFF>(ib)};
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                encode8<BITS>(w[4 * jj + u], __uint_as_float(zq[u]), __uint_as_float(iq[u]), codes[4 * jj + u]);
                zrow[4 * jj + u] = zq[u];
                if constexpr (OUT) {
#pragma unroll
                    for (int e = 0; e < 8; ++e) codes[4 * jj + u][e] &= ((om[4 * jj + u] >> e) & 1u) - 1u;   // outliers: code 0
                }
            }
        }
    };
    // ---------------- keys ----------------
    uint32_t* kc_head = k_codes + (size_t)head * ((size_t)n_cap * kHeadDim / E);
    uint32_t om[R], zrow[R];   // outlier bits of the tensor at hand (OUT); zero of the lane's own per-token group
#pragma unroll
    for (int j = 0; j < R; ++j) om[j] = 0u;
    if constexpr (OUT) mark(kw, om);
    if constexpr (!QUANT) {
#pragma unroll
        for (int j = 0; j < R; ++j)
            if (r + 16 * j < ntok_pad)     // (rows past the count were loaded as zeros)
                *reinterpret_cast<uint4*>(kc_head + (size_t)(d0 + r + 16 * j) * (kHeadDim / 2) + 4 * c8) = make_uint4(kw[j][0], kw[j][1], kw[j][2], kw[j][3]);
    } else if (key_axis == KVQP_KEY_PER_CHANNEL) {
        // minima / maxima per channel over the G tokens of a group: own rows, the four row lanes of
        // the wave (lane ^ 16, ^ 32), then the four waves through LDS
        uint32_t pmin[NG][4], pmax[NG][4];
#pragma unroll
        for (int ug = 0; ug < NG; ++ug)
#pragma unroll
            for (int q = 0; q < 4; ++q) { pmin[ug][q] = 0xffffffffu; pmax[ug][q] = 0u; }
#pragma unroll
        for (int j = 0; j < R; ++j)
            if (live[j]) {
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    const uint32_t a = order_key2(kw[j][q]);
                    const uint32_t ex = OUT ? half_mask(om[j] >> (2 * q)) : 0u;
                    pmin[j / JPG][q] = pk_min(pmin[j / JPG][q], a | ex); pmax[j / JPG][q] = pk_max(pmax[j / JPG][q], a & ~ex);
                }
            }
#pragma unroll
        for (int ug = 0; ug < NG; ++ug)
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                auto s1 = KVQP_SWAP16(pmin[ug][q]); uint32_t a = pk_min(s1[0], s1[1]);
                auto s2 = KVQP_SWAP32(a); pmin[ug][q] = pk_min(s2[0], s2[1]);
                auto s3 = KVQP_SWAP16(pmax[ug][q]); uint32_t b = pk_max(s3[0], s3[1]);
                auto s4 = KVQP_SWAP32(b); pmax[ug][q] = pk_max(s4[0], s4[1]);
            }
        if (lane < 16) {
#pragma unroll
            for (int ug = 0; ug < NG; ++ug) {
                *reinterpret_cast<uint4*>(s_min + (wave * NG + ug) * kHeadDim + 8 * c8) = make_uint4(pmin[ug][0], pmin[ug][1], pmin[ug][2], pmin[ug][3]);
                *reinterpret_cast<uint4*>(s_max + (wave * NG + ug) * kHeadDim + 8 * c8) = make_uint4(pmax[ug][0], pmax[ug][1], pmax[ug][2], pmax[ug][3]);
            }
        }
        __syncthreads();
        for (int item = threadIdx.x; item < NG * kHeadDim; item += kThreads) {   // one (group, channel) each
            const int ug = item / kHeadDim, d = item % kHeadDim;
            uint32_t a = 0xffffu, b = 0u;
#pragma unroll
            for (int w = 0; w < 4; ++w) {
                a = min(a, (uint32_t)s_min[(w * NG + ug) * kHeadDim + d]);
                b = max(b, (uint32_t)s_max[(w * NG + ug) * kHeadDim + d]);
            }
            if (OUT && a > b) { a = 0x8000u; b = 0x8000u; }   // every token of the group is an outlier here: zero +0, scale 0
            const GroupParams gp = group_params<BITS>(a, b);
            s_par[item] = make_float2(gp.zf, gp.inv);
            if (ug * G < ntok) {
                const size_t m = ((size_t)head * ((n_cap + G - 1) / G) + (d0 / G + ug)) * kHeadDim + d;
                k_scale[m] = gp.scale_h; k_zero[m] = gp.zero_h;
            }
        }
        __syncthreads();
#pragma unroll
        for (int ug = 0; ug < NG; ++ug) {
            float zf[8], inv[8];
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const float4 pr = *reinterpret_cast<const float4*>(&s_par[ug * kHeadDim + 8 * c8 + 2 * q]);
                zf[2 * q] = pr.x; inv[2 * q] = pr.y; zf[2 * q + 1] = pr.z; inv[2 * q + 1] = pr.w;
            }
#pragma unroll
            for (int jl = 0; jl < JPG && ug * JPG + jl < R; ++jl) {
                const int j = ug * JPG + jl;
                uint32_t c[8];
                encode8<BITS>(kw[j], zf, inv, c);
                if constexpr (OUT) {
#pragma unroll
                    for (int e = 0; e < 8; ++e) c[e] &= ((om[j] >> e) & 1u) - 1u;
                }
                // (padding rows of the last block hold code 0)
                if (r + 16 * j < ntok_pad) store_key_words<BITS>(kc_head + (size_t)(d0 + r + 16 * j) * (kHeadDim / E), c8, c, live[j] ? 0xFFFFFFFFu : 0u);
            }
        }
        if constexpr (OUT)   // the zero of (row j's key group, own channel 8 c8 + e) from the table the codes were made with
            store_slots(k_out, s_cnt[0], kw, om, [&](int j, int e) { return s_par[(j / JPG) * kHeadDim + 8 * c8 + e].x; });
    } else {
        uint32_t codes[R][8];
        per_token(kw, k_scale, k_zero, codes, om, zrow);
        if constexpr (OUT) store_slots(k_out, s_cnt[0], kw, om, [&](int j, int) { return __uint_as_float(zrow[j]); });
#pragma unroll
        for (int j = 0; j < R; ++j)      // (a padding row was loaded as zeros: scale 0, all codes 0)
            if (r + 16 * j < ntok_pad) store_key_words<BITS>(kc_head + (size_t)(d0 + r + 16 * j) * (kHeadDim / E), c8, codes[j]);
    }

    // ---------------- values ----------------
    // Token t = r + 16 j = 32 (j / 2) + 16 (j % 2) + 4 wave + i4: half-word H = j % 2, 32-token block
    // j / 2, kb = wave, i = i4.  A lane's field of word (superblock, kb, channel, wl) sits at
    // 16 H + BITS p with run = 4 blk + i4 = wl (E/2) + p; lanes of equal wl OR their fields together.
    {
        uint32_t part[NSB][8];
#pragma unroll
        for (int sb = 0; sb < NSB; ++sb)
#pragma unroll
            for (int dd = 0; dd < 8; ++dd) part[sb][dd] = 0u;
        if constexpr (QUANT) {
            uint32_t codes[R][8];
            if constexpr (OUT) mark(vw, om);
            per_token(vw, v_scale, v_zero, codes, om, zrow);
            if constexpr (OUT) store_slots(v_out, s_cnt[1], vw, om, [&](int j, int) { return __uint_as_float(zrow[j]); });
#pragma unroll
            for (int j = 0; j < R; ++j) {
                const int b32 = j >> 1, H = j & 1;
                const int sb = (32 * b32) / SB, blk = b32 % (SB / 32);
                const int p = (4 * blk + i4) % (E / 2);
#pragma unroll
                for (int dd = 0; dd < 8; ++dd) part[sb][dd] |= codes[j][dd] << (16 * H + BITS * p);   // (a padding row's codes are all 0)
            }
        } else {
#pragma unroll
            for (int j = 0; j < R; ++j) {
                const int sb = j >> 1, H = j & 1;
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    part[sb][2 * q] |= (vw[j][q] & 0xffffu) << (16 * H);
                    part[sb][2 * q + 1] |= (vw[j][q] >> 16) << (16 * H);
                }
            }
        }
        constexpr int LANES_PER_WORD = (E / 2 >= 4) ? 4 : E / 2;   // row lanes whose fields share a word
#pragma unroll
        for (int sb = 0; sb < NSB; ++sb)
#pragma unroll
            for (int dd = 0; dd < 8; ++dd) {
                if (LANES_PER_WORD >= 2) { auto s1 = KVQP_SWAP16(part[sb][dd]); part[sb][dd] = s1[0] | s1[1]; }
                if (LANES_PER_WORD >= 4) { auto s2 = KVQP_SWAP32(part[sb][dd]); part[sb][dd] = s2[0] | s2[1]; }
            }
        const int wl = (E / 2 >= 4) ? 0 : i4 / (E / 2);          // run / (E/2) with blk = 0 (SB = 32 whenever E/2 < 4)
        const bool writer = (i4 % LANES_PER_WORD) == 0;
        if (writer) {
            const int tile = c8 >> 1, y = tile * WPT + wl;
#pragma unroll
            for (int sb = 0; sb < NSB; ++sb)
#pragma unroll
                for (int dd = 0; dd < 8; ++dd) {
                    const int n = 8 * (c8 & 1) + dd;
                    s_words[sb * SBW + ((y >> 2) * 64 + wave * 16 + n) * 4 + (y & 3)] = part[sb][dd];
                }
        }
        __syncthreads();
        const int n_sb = (ntok + SB - 1) / SB;
        uint32_t* vc = v_codes + (size_t)head * SBW * ((n_cap + SB - 1) / SB) + (size_t)(d0 / SB) * SBW;
        for (int item = threadIdx.x; item < n_sb * SBW / 4; item += kThreads)
            reinterpret_cast<uint4*>(vc)[item] = reinterpret_cast<const uint4*>(s_words)[item];
    }
    if constexpr (OUT) {   // (the barrier before the value store orders every row's count before this)
        const int tensor = threadIdx.x / (TB / 32), blk = threadIdx.x % (TB / 32);
        if (threadIdx.x < 2 * (TB / 32) && 32 * blk < ntok) {
            uint32_t* ovf = (tensor ? v_ovf : k_ovf) + (size_t)head * ovf_words(n_cap, ovf_cap);
            ovf[d0 / 32 + blk + 1] = (uint32_t)s_cnt[tensor][blk];
        }
    }
}

// Raw block counts -> prefix counts, in place: entry b + 1 of a head's prefix array holds the
// number of overflow outliers of block b (left there by the quantizer) for blocks first .. first +
// n - 1, and entry `first` the prefix so far (set to 0 here when first == 0).  One wave per (head,
// tensor); 64 blocks per round.
__global__ __launch_bounds__(64) void ovf_scan(uint32_t* __restrict__ k_ovf, uint32_t* __restrict__ v_ovf, int n_cap, int ovf_cap,
                                               int dst_base, int n_tok, const int32_t* __restrict__ head_n,
                                               const int32_t* __restrict__ head_base, int base_quantum) {
    const int head = blockIdx.x, lane = threadIdx.x;
    uint32_t* start = (blockIdx.y ? v_ovf : k_ovf) + (size_t)head * ovf_words(n_cap, ovf_cap);
    int base = dst_base;
    if (head_base) {
        base = min(max(head_base[head], 0), dst_base);
        base -= base % base_quantum;
    }
    const int n_head = head_n ? min(max(head_n[head], 0), n_tok) : n_tok;
    const int first = base / 32, n = (n_head + 31) / 32;
    if (first == 0 && lane == 0) start[0] = 0u;
    __syncthreads();
    uint32_t carry = start[first];
    for (int b0 = 0; b0 < n; b0 += 64) {
        const int b = b0 + lane;
        uint32_t v = b < n ? start[first + b + 1] : 0u;
#pragma unroll
        for (int off = 1; off < 64; off <<= 1) {
            const uint32_t o = __shfl_up(v, off);
            if (lane >= off) v += o;
        }
        if (b < n) start[first + b + 1] = carry + v;
        carry += __shfl(v, 63);
    }
}

// The overflow entries of one block of 32 tokens (one wave): the block's rows are read again, the
// outliers beyond a row's fourth found in channel order, and written as (word, token) at the block's
// place in the head's list -- position = prefix count of the block + entries of the block's earlier
// rows -- unless they lie beyond the list's capacity.  Most blocks have none and leave at once.
template <int G>
__global__ __launch_bounds__(64) void ovf_fill(const uint16_t* __restrict__ k, const uint16_t* __restrict__ v,
                                               const int32_t* __restrict__ idx, const uint16_t* __restrict__ k_zero,
                                               const uint16_t* __restrict__ v_zero, uint32_t* __restrict__ k_ovf,
                                               uint32_t* __restrict__ v_ovf, int L, int n_kept, int key_axis, int n_cap,
                                               int dst_base, const int32_t* __restrict__ head_n, uint32_t tau_bits,
                                               const int32_t* __restrict__ head_base, int base_quantum, int ovf_cap) {
    const int head = blockIdx.y, lane = threadIdx.x, tensor = blockIdx.z;
    int base = dst_base;
    if (head_base) {
        base = min(max(head_base[head], 0), dst_base);
        base -= base % base_quantum;
    }
    const int n_head = head_n ? min(max(head_n[head], 0), n_kept) : n_kept;
    const int t0 = 32 * blockIdx.x;
    if (t0 >= n_head) return;
    uint32_t* ovf = (tensor ? v_ovf : k_ovf) + (size_t)head * ovf_words(n_cap, ovf_cap);
    const int blk = (base + t0) / 32;
    uint32_t at = ovf[blk];
    if (ovf[blk + 1] == at) return;                  // (wave-uniform) nothing beyond the slots in this block
    uint32_t* entries = ovf + ovf_start_words(n_cap);
    const uint16_t* src = (tensor ? v : k) + (size_t)head * L * kHeadDim;
    const unsigned long long lt_mask = (1ull << lane) - 1ull;
    for (int t = t0; t < min(t0 + 32, n_head); ++t) {
        const int pos = idx ? idx[(size_t)head * n_kept + t] : t;
        const uint32_t w = *reinterpret_cast<const uint32_t*>(src + (size_t)pos * kHeadDim + 2 * lane);   // channels 2 lane, 2 lane + 1
        const bool c0 = (w & 0x7fffu) > tau_bits, c1 = ((w >> 16) & 0x7fffu) > tau_bits;
        const unsigned long long b0 = __builtin_amdgcn_ballot_w64(c0), b1 = __builtin_amdgcn_ballot_w64(c1);
        const uint32_t total = (uint32_t)(__popcll(b0) + __popcll(b1));
        if (total <= 4u) continue;                   // (wave-uniform)
        const uint32_t r0 = (uint32_t)(__popcll(b0 & lt_mask) + __popcll(b1 & lt_mask)), r1 = r0 + (c0 ? 1u : 0u);
        const int tok = base + t;                    // the token's position in the head
#pragma unroll
        for (int e = 0; e < 2; ++e) {
            const bool is = e ? c1 : c0;
            const uint32_t rank = e ? r1 : r0;
            if (is && rank >= 4u) {
                const int d = 2 * lane + e;
                const size_t m = (tensor == 0 && key_axis == KVQP_KEY_PER_CHANNEL)
                                     ? ((size_t)head * ((n_cap + G - 1) / G) + tok / G) * kHeadDim + d
                                     : ((size_t)head * n_cap + tok) * (kHeadDim / G) + d / G;
                const float zf = half_bits_to_float((tensor ? v_zero : k_zero)[m]);
                const uint32_t xh = e ? (w >> 16) : (w & 0xffffu);
                const float diff = __fsub_rn(half_bits_to_float((uint16_t)xh), zf);
                const uint32_t e_at = at + rank - 4u;
                if (e_at < (uint32_t)ovf_cap) {
                    entries[2 * (size_t)e_at] = (__float_as_uint(diff) & 0xFFFFFF00u) | 0x80u | (uint32_t)d;
                    entries[2 * (size_t)e_at + 1] = (uint32_t)tok;
                }
            }
        }
        at += total - 4u;
    }
}
#undef KVQP_SWAP16
#undef KVQP_SWAP32

template <int BITS, int G, bool OUT>
hipError_t launch_bits_g(const QuantPackJob& j, hipStream_t stream) {
    constexpr int TB = (BITS != 16 && G == 128) ? 128 : 64;
    const int nblk = (j.n_tok + TB - 1) / TB;
    dim3 grid(nblk + (j.copy_tail ? 1 : 0), j.heads);
    if (grid.x == 0) return hipSuccess;
    hipLaunchKernelGGL((gather_quant_pack<BITS, G, OUT>), grid, dim3(kThreads), 0, stream, (const uint16_t*)j.k,
                       (const uint16_t*)j.v, j.idx, (uint32_t*)j.c.k_codes, (uint32_t*)j.c.v_codes, (uint16_t*)j.c.k_scale,
                       (uint16_t*)j.c.k_zero, (uint16_t*)j.c.v_scale, (uint16_t*)j.c.v_zero, (uint16_t*)j.c.tail_k,
                       (uint16_t*)j.c.tail_v, j.src_rows, j.window, j.n_tok, j.key_axis, j.c.tail_cap, nblk, j.n_cap,
                       j.dst_base, j.head_n, (uint32_t*)j.c.k_out, (uint32_t*)j.c.v_out, j.tau_bits, j.head_base,
                       j.base_quantum, (uint32_t*)j.c.k_ovf, (uint32_t*)j.c.v_ovf, j.ovf_cap);
    hipError_t e = hipGetLastError();
    if constexpr (OUT) {
        if (e != hipSuccess || j.n_tok == 0) return e;
        hipLaunchKernelGGL(ovf_scan, dim3(j.heads, 2), dim3(64), 0, stream, (uint32_t*)j.c.k_ovf, (uint32_t*)j.c.v_ovf, j.n_cap,
                           j.ovf_cap, j.dst_base, j.n_tok, j.head_n, j.head_base, j.base_quantum);
        hipLaunchKernelGGL((ovf_fill<G>), dim3((j.n_tok + 31) / 32, j.heads, 2), dim3(64), 0, stream, (const uint16_t*)j.k,
                           (const uint16_t*)j.v, j.idx, (const uint16_t*)j.c.k_zero, (const uint16_t*)j.c.v_zero,
                           (uint32_t*)j.c.k_ovf, (uint32_t*)j.c.v_ovf, j.src_rows, j.n_tok, j.key_axis, j.n_cap, j.dst_base,
                           j.head_n, j.tau_bits, j.head_base, j.base_quantum, j.ovf_cap);
        e = hipGetLastError();
    }
    return e;
}
template <int BITS>
hipError_t launch_bits(const QuantPackJob& j, hipStream_t stream) {
    if constexpr (BITS == 16) {
        return launch_bits_g<BITS, 32, false>(j, stream);
    } else {
        if (j.outliers) {
            switch (j.group_size) {
                case 32: return launch_bits_g<BITS, 32, true>(j, stream);
                case 64: return launch_bits_g<BITS, 64, true>(j, stream);
                default: return launch_bits_g<BITS, 128, true>(j, stream);
            }
        }
        switch (j.group_size) {
            case 32: return launch_bits_g<BITS, 32, false>(j, stream);
            case 64: return launch_bits_g<BITS, 64, false>(j, stream);
            default: return launch_bits_g<BITS, 128, false>(j, stream);
        }
    }
}

// Rows [n_shift, tail_len) of both tail tensors move down to [0, tail_len - n_shift).  One workgroup
// per head; 16 rows per round go through registers (all reads of a round before its writes, rounds
// in ascending order, so overlapping ranges are safe).
__global__ __launch_bounds__(kThreads) void tail_shift(uint16_t* __restrict__ tail_k, uint16_t* __restrict__ tail_v,
                                                       int tail_cap, int n_shift, int tail_len) {
    const int head = blockIdx.x;
    uint16_t* tk = tail_k + (size_t)head * tail_cap * kHeadDim;
    uint16_t* tv = tail_v + (size_t)head * tail_cap * kHeadDim;
    const int r = threadIdx.x >> 4, c8 = threadIdx.x & 15;
    for (int r0 = n_shift; r0 < tail_len; r0 += 16) {
        const int row = r0 + r;
        const bool live = row < tail_len;
        uint4 a = make_uint4(0, 0, 0, 0), b = a;
        if (live) {
            a = *reinterpret_cast<const uint4*>(tk + (size_t)row * kHeadDim + 8 * c8);
            b = *reinterpret_cast<const uint4*>(tv + (size_t)row * kHeadDim + 8 * c8);
        }
        __syncthreads();
        if (live) {
            *reinterpret_cast<uint4*>(tk + (size_t)(row - n_shift) * kHeadDim + 8 * c8) = a;
            *reinterpret_cast<uint4*>(tv + (size_t)(row - n_shift) * kHeadDim + 8 * c8) = b;
        }
        __syncthreads();
    }
}

hipError_t launch_job(const QuantPackJob& j, hipStream_t stream) {
    switch (j.bits) {
        case 2: return launch_bits<2>(j, stream);
        case 4: return launch_bits<4>(j, stream);
        case 8: return launch_bits<8>(j, stream);
        default: return launch_bits<16>(j, stream);
    }
}

}  // namespace

// Largest binary16 magnitude pattern whose value does not exceed tau (> 0): |x| > tau iff the
// pattern of |x| is greater (patterns of non-negative halves order like their values).
static uint32_t threshold_bits(float tau) {
    auto value = [](uint32_t h) -> double {   // finite non-negative binary16 pattern -> value
        const int e = (int)(h >> 10), m = (int)(h & 0x3ff);
        return e == 0 ? m * (1.0 / 16777216.0) : (double)(1024 + m) * (e >= 25 ? (double)(1 << (e - 25)) : 1.0 / (double)(1 << (25 - e)));
    };
    uint32_t lo = 0, hi = 0x7BFF;
    while (lo < hi) {
        const uint32_t mid = (lo + hi + 1) / 2;
        if (value(mid) <= (double)tau) lo = mid; else hi = mid - 1;
    }
    return lo;
}
static void set_outliers(QuantPackJob& j, const kvqp_cfg& cfg) {
    j.outliers = outliers_on(cfg);
    j.ovf_cap = cfg.outlier_overflow_cap;
    j.tau_bits = j.outliers ? threshold_bits(cfg.outlier_threshold) : 0x7fffu;
}

hipError_t launch_quant_pack(const kvqp_cfg& cfg, const void* k, const void* v, const int32_t* idx, int n_kept,
                             const int32_t* head_n, const kvqp_cache& cache, hipStream_t stream) {
    QuantPackJob j{cache};
    set_outliers(j, cfg);
    j.k = k; j.v = v; j.idx = idx; j.head_n = head_n;
    j.heads = cfg.batch * cfg.n_kv_heads; j.src_rows = cfg.seq_len; j.window = cfg.window;
    j.n_tok = n_kept; j.dst_base = 0; j.n_cap = layout_tokens(cache, n_kept);
    j.bits = cfg.bits; j.group_size = cfg.group_size; j.key_axis = cfg.key_axis; j.copy_tail = true;
    return launch_job(j, stream);
}

// Host counts -> device array, carried in kernel arguments (copied when the launch is enqueued, so
// the caller's array may go away as soon as the call returns; no staging copy, no synchronisation).
struct CountBatch { int32_t v[kCountsPerLaunch]; };
__global__ void store_counts(int32_t* __restrict__ dst, CountBatch b, int n) {
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) dst[i] = b.v[i];
}
hipError_t upload_counts(int32_t* dst, const int32_t* src_host, int n, hipStream_t stream, int add) {
    for (int i0 = 0; i0 < n; i0 += kCountsPerLaunch) {
        CountBatch b;
        const int m = n - i0 < kCountsPerLaunch ? n - i0 : kCountsPerLaunch;
        for (int i = 0; i < m; ++i) b.v[i] = (src_host ? src_host[i0 + i] : 0) + add;
        for (int i = m; i < kCountsPerLaunch; ++i) b.v[i] = 0;
        hipLaunchKernelGGL(store_counts, dim3((m + 255) / 256), dim3(256), 0, stream, dst + i0, b, m);
        const hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
    }
    return hipSuccess;
}

// The n_tokens oldest tail rows are quantized onto the end of the packed part, then the tail closes up.
// base_quantum > 0: every head at its own count (cache.head_n_kept), counts being multiples of it.
hipError_t launch_append_tail(const kvqp_cfg& cfg, const kvqp_cache& cache, int n_tokens, int base_quantum, hipStream_t stream) {
    QuantPackJob j{cache};
    set_outliers(j, cfg);
    j.k = cache.tail_k; j.v = cache.tail_v; j.idx = nullptr; j.head_n = nullptr;
    if (base_quantum > 0) { j.head_base = cache.head_n_kept; j.base_quantum = base_quantum; }
    j.heads = cfg.batch * cfg.n_kv_heads; j.src_rows = cache.tail_cap; j.window = 0;
    j.n_tok = n_tokens; j.dst_base = cache.n_kept; j.n_cap = layout_tokens(cache, cache.n_kept);
    j.bits = cfg.bits; j.group_size = cfg.group_size; j.key_axis = cfg.key_axis; j.copy_tail = false;
    hipError_t e = launch_job(j, stream);
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(tail_shift, dim3(j.heads), dim3(kThreads), 0, stream, (uint16_t*)cache.tail_k, (uint16_t*)cache.tail_v,
                       cache.tail_cap, n_tokens, cache.tail_len);
    return hipGetLastError();
}

}  // namespace kvqp
