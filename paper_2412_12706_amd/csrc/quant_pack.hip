// Gather the surviving tokens, quantize them group by group and write the
// packed cache (paper Section 3, "KV Quantization": z = min, m = max,
// s = (m - z)/(2^B - 1), Q(G) = round((G - z)/s); grouping axes of Section 2 /
// Section 5.4).  Memory-bound: every survivor row is read once (2 x 256 B) and
// k*bpt bytes are written; there is no reuse to exploit, so the kernel's job
// is coalesced 16-byte row gathers and fully coalesced word stores.
//
// One workgroup owns TB consecutive kept tokens of one (batch, kv head):
// whole key groups (G | TB) and whole value superblocks (SB | TB).
#include "kvqp_internal.h"

namespace kvqp {
namespace {

constexpr int kThreads = 256;
constexpr int kRowPad = kHeadDim + 2;  // halves; odd dword stride -> conflict-free column walks

// binary16 bit pattern -> key that orders like the value (-0 below +0).
__device__ __forceinline__ uint32_t order_key(uint16_t h) { return (h & 0x8000u) ? (uint16_t)~h : (uint16_t)(h | 0x8000u); }
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
    if (g.inv == 0.0f) return 0u;
    float c = rintf(__fmul_rn(__fsub_rn(half_bits_to_float(xh), g.zf), g.inv));
    c = fminf(fmaxf(c, 0.0f), (float)((1 << BITS) - 1));
    return (uint32_t)c;
}

template <int BITS> struct CodeT { using type = uint8_t; };
template <> struct CodeT<16> { using type = uint16_t; };

// Gather ntok rows (positions sidx[t]) of one head into the LDS tile.
__device__ __forceinline__ void gather_rows(const uint16_t* __restrict__ src_head, const int* sidx, int ntok,
                                            uint16_t* tile) {
    for (int item = threadIdx.x; item < ntok * 16; item += kThreads) {
        const int t = item >> 4, c = item & 15;
        const uint4 v = *reinterpret_cast<const uint4*>(src_head + (size_t)sidx[t] * kHeadDim + c * 8);
        uint32_t* dst = reinterpret_cast<uint32_t*>(tile + t * kRowPad + c * 8);  // 4-byte aligned (kRowPad even)
        dst[0] = v.x; dst[1] = v.y; dst[2] = v.z; dst[3] = v.w;
    }
}

template <int BITS, int TB>
__global__ __launch_bounds__(kThreads) void gather_quant_pack(
    const uint16_t* __restrict__ k, const uint16_t* __restrict__ v, const int32_t* __restrict__ idx,
    uint32_t* __restrict__ k_codes, uint32_t* __restrict__ v_codes, uint16_t* __restrict__ k_scale,
    uint16_t* __restrict__ k_zero, uint16_t* __restrict__ v_scale, uint16_t* __restrict__ v_zero,
    uint16_t* __restrict__ tail_k, uint16_t* __restrict__ tail_v, int L, int W, int n_kept, int G, int key_axis,
    int tail_cap, int n_tok_blocks) {
    using code_t = typename CodeT<BITS>::type;
    constexpr int E = 32 / BITS;
    constexpr int SB = v_superblock(BITS);
    constexpr int WPT = v_words_per_tile(BITS);
    constexpr int SBW = v_superblock_words(BITS);
    __shared__ __align__(16) uint16_t tile[TB * kRowPad];
    __shared__ __align__(16) code_t cbuf[TB * kHeadDim];
    __shared__ int sidx[TB];

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

    const int t0 = blockIdx.x * TB;
    const int ntok = min(TB, n_kept - t0);
    for (int t = threadIdx.x; t < ntok; t += kThreads) sidx[t] = idx[(size_t)head * n_kept + t0 + t];
    __syncthreads();

    // ---------------- keys ----------------
    gather_rows(kh, sidx, ntok, tile);
    __syncthreads();
    uint32_t* kc_head = k_codes + (size_t)head * ((size_t)n_kept * kHeadDim / E);
    if constexpr (BITS == 16) {
        for (int item = threadIdx.x; item < ntok * (kHeadDim / 2); item += kThreads) {
            const int t = item / (kHeadDim / 2), w = item % (kHeadDim / 2);
            kc_head[(size_t)(t0 + t) * (kHeadDim / 2) + w] = *reinterpret_cast<const uint32_t*>(tile + t * kRowPad + 2 * w);
        }
    } else {
        if (key_axis == KVQP_KEY_PER_CHANNEL) {
            const int d = threadIdx.x & (kHeadDim - 1);
            for (int ug = threadIdx.x / kHeadDim; ug < ntok / G; ug += kThreads / kHeadDim) {
                uint32_t kmin = 0xffffu, kmax = 0u;
                for (int e = 0; e < G; ++e) {
                    const uint32_t key = order_key(tile[(ug * G + e) * kRowPad + d]);
                    kmin = min(kmin, key); kmax = max(kmax, key);
                }
                const GroupParams gp = group_params<BITS>(kmin, kmax);
                const size_t m = ((size_t)head * (n_kept / G) + (t0 / G + ug)) * kHeadDim + d;
                k_scale[m] = gp.scale_h; k_zero[m] = gp.zero_h;
                for (int e = 0; e < G; ++e)
                    cbuf[(ug * G + e) * kHeadDim + d] = (code_t)encode<BITS>(tile[(ug * G + e) * kRowPad + d], gp);
            }
        } else {
            const int cpt = kHeadDim / G;
            for (int item = threadIdx.x; item < ntok * cpt; item += kThreads) {
                const int t = item / cpt, cg = item % cpt;
                uint32_t kmin = 0xffffu, kmax = 0u;
                for (int e = 0; e < G; ++e) {
                    const uint32_t key = order_key(tile[t * kRowPad + cg * G + e]);
                    kmin = min(kmin, key); kmax = max(kmax, key);
                }
                const GroupParams gp = group_params<BITS>(kmin, kmax);
                const size_t m = ((size_t)head * n_kept + t0 + t) * cpt + cg;
                k_scale[m] = gp.scale_h; k_zero[m] = gp.zero_h;
                for (int e = 0; e < G; ++e)
                    cbuf[t * kHeadDim + cg * G + e] = (code_t)encode<BITS>(tile[t * kRowPad + cg * G + e], gp);
            }
        }
        __syncthreads();
        constexpr int WPR = kHeadDim / E;  // words per key row
        for (int item = threadIdx.x; item < ntok * WPR; item += kThreads) {
            const int t = item / WPR, w = item % WPR;
            uint32_t word = 0;
#pragma unroll
            for (int r = 0; r < E; ++r)
                word |= (uint32_t)cbuf[t * kHeadDim + w * E + r] << (16 * (r & 1) + BITS * (r >> 1));
            kc_head[(size_t)(t0 + t) * WPR + w] = word;
        }
    }
    __syncthreads();

    // ---------------- values ----------------
    gather_rows(vh, sidx, ntok, tile);
    __syncthreads();
    if constexpr (BITS == 16) {
        for (int item = threadIdx.x; item < ntok * kHeadDim; item += kThreads)
            cbuf[item] = tile[(item / kHeadDim) * kRowPad + (item % kHeadDim)];
    } else {
        const int cpt = kHeadDim / G;
        for (int item = threadIdx.x; item < ntok * cpt; item += kThreads) {
            const int t = item / cpt, cg = item % cpt;
            uint32_t kmin = 0xffffu, kmax = 0u;
            for (int e = 0; e < G; ++e) {
                const uint32_t key = order_key(tile[t * kRowPad + cg * G + e]);
                kmin = min(kmin, key); kmax = max(kmax, key);
            }
            const GroupParams gp = group_params<BITS>(kmin, kmax);
            const size_t m = ((size_t)head * n_kept + t0 + t) * cpt + cg;
            v_scale[m] = gp.scale_h; v_zero[m] = gp.zero_h;
            for (int e = 0; e < G; ++e)
                cbuf[t * kHeadDim + cg * G + e] = (code_t)encode<BITS>(tile[t * kRowPad + cg * G + e], gp);
        }
    }
    __syncthreads();
    {
        const int n_sb = (ntok + SB - 1) / SB;
        uint32_t* vc = v_codes + (size_t)head * v_superblock_words(BITS) * ((n_kept + SB - 1) / SB) + (size_t)(t0 / SB) * SBW;
        for (int item = threadIdx.x; item < n_sb * SBW; item += kThreads) {
            const int sbl = item / SBW, wsb = item % SBW;
            const int y = 4 * (wsb >> 8) + (wsb & 3), lane = (wsb >> 2) & 63;
            const int kb = lane >> 4, n = lane & 15, tl = y / WPT, wl = y % WPT;
            const int d = 16 * tl + n;
            uint32_t word = 0;
#pragma unroll
            for (int H = 0; H < 2; ++H)
#pragma unroll
                for (int p = 0; p < E / 2; ++p) {
                    const int run = wl * (E / 2) + p;
                    const int t = sbl * SB + 32 * (run >> 2) + 16 * H + 4 * kb + (run & 3);
                    const uint32_t c = (t < ntok) ? (uint32_t)cbuf[t * kHeadDim + d] : 0u;
                    word |= c << (16 * H + BITS * p);
                }
            vc[item] = word;
        }
    }
}

template <int BITS>
hipError_t launch_bits(const kvqp_cfg& cfg, const void* k, const void* v, const int32_t* idx, int n_kept,
                       const kvqp_cache& c, hipStream_t stream) {
    const int heads = cfg.batch * cfg.n_kv_heads;
    auto go = [&](auto tb_tag) {
        constexpr int TB = decltype(tb_tag)::value;
        const int nblk = (n_kept + TB - 1) / TB;
        dim3 grid(nblk + 1, heads);
        hipLaunchKernelGGL((gather_quant_pack<BITS, TB>), grid, dim3(kThreads), 0, stream, (const uint16_t*)k,
                           (const uint16_t*)v, idx, (uint32_t*)c.k_codes, (uint32_t*)c.v_codes, (uint16_t*)c.k_scale,
                           (uint16_t*)c.k_zero, (uint16_t*)c.v_scale, (uint16_t*)c.v_zero, (uint16_t*)c.tail_k,
                           (uint16_t*)c.tail_v, cfg.seq_len, cfg.window, n_kept, cfg.group_size, cfg.key_axis,
                           c.tail_cap, nblk);
    };
    if (cfg.bits != 16 && cfg.group_size == 128) go(std::integral_constant<int, 128>{});
    else go(std::integral_constant<int, 64>{});
    return hipGetLastError();
}

}  // namespace

hipError_t launch_quant_pack(const kvqp_cfg& cfg, const void* k, const void* v, const int32_t* idx, int n_kept,
                             const kvqp_cache& cache, hipStream_t stream) {
    switch (cfg.bits) {
        case 2: return launch_bits<2>(cfg, k, v, idx, n_kept, cache, stream);
        case 4: return launch_bits<4>(cfg, k, v, idx, n_kept, cache, stream);
        case 8: return launch_bits<8>(cfg, k, v, idx, n_kept, cache, stream);
        default: return launch_bits<16>(cfg, k, v, idx, n_kept, cache, stream);
    }
}

}  // namespace kvqp
