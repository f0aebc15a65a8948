// Internal declarations shared by the translation units of libkvqp.so.
// Not part of the public ABI (that is include/kvqp.h).
#pragma once
#include <hip/hip_runtime.h>
#include <hip/hip_fp16.h>
#include <stdint.h>
#include <stddef.h>

#include "kvqp.h"

namespace kvqp {

constexpr int kHeadDim = 128;  // the only head size built

// Value-code storage geometry (format statement in kvqp.h, "Value codes").
__host__ __device__ constexpr int v_superblock(int bits) { return bits == 2 ? 64 : 32; }
__host__ __device__ constexpr int v_words_per_tile(int bits) { return bits == 16 ? 4 : bits == 8 ? 2 : 1; }
__host__ __device__ constexpr int v_superblock_words(int bits) { return 64 * (kHeadDim / 16) * v_words_per_tile(bits); }

// Outlier filtering is on (format statement in kvqp.h, "Outlier filtering").
inline bool outliers_on(const kvqp_cfg& c) { return c.outlier_threshold > 0.0f; }

// Token counts need not fill whole blocks: the per-token arrays of a head (key code rows, per-token
// scales and zeros, outlier slots) are laid out for the count rounded up to 32, zeros past the count.
__host__ __device__ constexpr int rows32(int n) { return (n + 31) / 32 * 32; }
// Tokens a cache's buffers are laid out for: its capacity, or its own count in whole blocks.
inline int layout_tokens(const kvqp_cache& c, int n_kept) { return c.n_cap > 0 ? c.n_cap : rows32(n_kept); }

inline size_t k_code_words(int n_kept, int bits) { return (size_t)rows32(n_kept) * kHeadDim * bits / 32; }
inline size_t v_code_words(int n_kept, int bits) {
    const int sb = v_superblock(bits);
    return (size_t)((n_kept + sb - 1) / sb) * v_superblock_words(bits);
}

// Overflow buffer of one head and tensor (format statement in kvqp.h, "Outlier filtering"): the
// prefix counts per 32 tokens, padded to a multiple of four words, then `cap` entries of two words.
__host__ __device__ constexpr size_t ovf_start_words(int n_tok) { return ((size_t)((n_tok + 31) / 32 + 1) + 3) / 4 * 4; }
__host__ __device__ constexpr size_t ovf_words(int n_tok, int cap) { return ovf_start_words(n_tok) + 2 * (size_t)cap; }

// Element counts of scale/zero arrays per (batch, kv-head).
inline size_t k_meta_elems(int n_kept, int bits, int G, int key_axis) {
    if (bits == 16) return 0;
    // (per channel: the last group may hold fewer than G tokens)
    return key_axis == KVQP_KEY_PER_CHANNEL ? (size_t)((n_kept + G - 1) / G) * kHeadDim : (size_t)rows32(n_kept) * (kHeadDim / G);
}
inline size_t v_meta_elems(int n_kept, int bits, int G) { return bits == 16 ? 0 : (size_t)rows32(n_kept) * (kHeadDim / G); }

// Decode split-K geometry, a pure function of the problem so that the
// workspace query and the launch agree.
struct DecodePlan {
    int n_splits;        // token-axis splits of the packed part
    int chunks_per_split;// 64-token chunks handled by one workgroup
    int n_partials;      // n_splits (+1 when a tail partial is written)
    int n_waves;         // waves per decode workgroup
    size_t ws_bytes;
};
DecodePlan plan_decode(const kvqp_cfg& cfg, int n_kept, int tail_len);
size_t decode_ws_bound(const kvqp_cfg& cfg);   // >= plan_decode(cfg, n, t).ws_bytes for every n and t
size_t decode_ws_header_bytes(const kvqp_cfg& cfg);   // arrival counters at the head of a decode workspace
hipError_t launch_ws_init(const kvqp_cfg& cfg, void* ws, hipStream_t stream);   // zeroes them
// The library's own decode workspace (a static device array): its address on the current device,
// prepared on first use.  KVQP_STATIC_SCRATCH_BYTES in kvqp.h is its size.
constexpr size_t kStaticScratchBytes = KVQP_STATIC_SCRATCH_BYTES;
hipError_t static_scratch(const kvqp_cfg& cfg, void** ptr, hipStream_t stream);

// Compress workspace layout (bytes offsets), pure function of cfg.
struct CompressPlan {
    int P, n_kept, rows;          // rows = Gq * W query rows per kv head
    int n_chunks;                 // key chunks of the scoring passes
    int n_wg, chunks_per_wg;      // scoring workgroups per kv head and their share
    int n_row_slabs;              // 64-row slabs of query rows (1, 2 or 4)
    size_t off_stats_part, off_stats, off_vote, off_pooled, off_sel, off_idx, total;
};
CompressPlan plan_compress(const kvqp_cfg& cfg);

// head_n (device, or NULL): every head's own token count under n_kept
hipError_t launch_quant_pack(const kvqp_cfg& cfg, const void* k, const void* v, const int32_t* idx,
                             int n_kept, const int32_t* head_n, const kvqp_cache& cache, hipStream_t stream);
hipError_t launch_decode(const kvqp_cfg& cfg, const void* q, const kvqp_cache& cache, void* out,
                         void* ws, const DecodePlan& plan, hipStream_t stream);
// n host integers into a device array, enqueued on the stream; src_host is read before the call returns.
constexpr int kCountsPerLaunch = 768;   // (kernel arguments: 3 KB per launch)
hipError_t upload_counts(int32_t* dst, const int32_t* src_host, int n, hipStream_t stream, int add = 0);   // dst[i] = src_host[i] + add (src_host == NULL: zeros)
hipError_t launch_append_tail(const kvqp_cfg& cfg, const kvqp_cache& cache, int n_tokens, int base_quantum, hipStream_t stream);
// head_n (device, or NULL): every head's own cut under plan.n_kept; score says whether any head drops a token
// unrefined (device [heads], or NULL): per head, how many candidates near the cut binary32 had to decide
hipError_t launch_select(const kvqp_cfg& cfg, const void* q_obs, const void* k, int32_t* idx, int32_t* unrefined,
                         void* ws, const CompressPlan& plan, const int32_t* head_n, bool score, hipStream_t stream);

}  // namespace kvqp
