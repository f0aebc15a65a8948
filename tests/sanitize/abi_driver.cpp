// Memory- and undefined-behaviour check of the C ABI's host side (csrc/kvqp_api.cpp: argument
// validation, size arithmetic, reading of the caller's host arrays, order of launches).  This
// program is linked with that one file, built under -fsanitize=address,undefined, and with the
// stand-ins below for everything that would touch a GPU, so it runs anywhere.  The stand-ins count
// what reaches them: a rejected call must reach none, an accepted call the expected ones, and the
// host arrays handed to upload_counts are read over exactly the length the ABI states (they are
// heap blocks of exactly that length, so reading past them stops the run).
// The launch planning (how many workgroups, workspace sizes) lives next to the kernels and is not
// covered here; the stand-in plans are fixed numbers.
// Test infrastructure only.
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <vector>

#include "kvqp_internal.h"

static int g_launches = 0;      // calls that would have enqueued work
static long long g_count_sum = 0;

namespace kvqp {
DecodePlan plan_decode(const kvqp_cfg& cfg, int, int) {
    DecodePlan p{};
    p.n_splits = p.n_partials = 2;
    p.chunks_per_split = 1;
    p.n_waves = 4;
    p.ws_bytes = decode_ws_header_bytes(cfg) + 4096;
    return p;
}
size_t decode_ws_header_bytes(const kvqp_cfg& cfg) { return ((size_t)cfg.batch * cfg.n_kv_heads * 4 + 255) / 256 * 256; }
size_t decode_ws_bound(const kvqp_cfg& cfg) { return decode_ws_header_bytes(cfg) + 8192; }
hipError_t launch_ws_init(const kvqp_cfg&, void*, hipStream_t) { ++g_launches; return hipSuccess; }
hipError_t static_scratch(const kvqp_cfg&, void** ptr, hipStream_t) { *ptr = (void*)0x2000; return hipSuccess; }
CompressPlan plan_compress(const kvqp_cfg& cfg) {
    CompressPlan p{};
    p.P = cfg.seq_len - cfg.window;
    p.n_kept = cfg.budget < p.P ? cfg.budget : p.P;
    p.off_idx = 1024;
    p.total = 1 << 20;
    return p;
}
hipError_t launch_quant_pack(const kvqp_cfg&, const void*, const void*, const int32_t*, int, const int32_t*, const kvqp_cache&,
                             hipStream_t) { ++g_launches; return hipSuccess; }
hipError_t launch_decode(const kvqp_cfg&, const void*, const kvqp_cache&, void*, void*, const DecodePlan&, hipStream_t) {
    ++g_launches;
    return hipSuccess;
}
hipError_t upload_counts(int32_t*, const int32_t* src_host, int n, hipStream_t, int add) {
    ++g_launches;
    for (int i = 0; i < n; ++i) g_count_sum += (src_host ? src_host[i] : 0) + add;
    return hipSuccess;
}
hipError_t launch_append_tail(const kvqp_cfg&, const kvqp_cache&, int, int, hipStream_t) { ++g_launches; return hipSuccess; }
hipError_t launch_select(const kvqp_cfg&, const void*, const void*, int32_t*, int32_t*, void*, const CompressPlan&, const int32_t*,
                         bool, hipStream_t) { ++g_launches; return hipSuccess; }
}  // namespace kvqp

extern "C" hipError_t hipMemcpyAsync(void*, const void*, size_t, hipMemcpyKind, hipStream_t) { ++g_launches; return hipSuccess; }

static int g_failed = 0;
#define EXPECT(cond)                                                                   \
    do {                                                                               \
        if (!(cond)) { std::fprintf(stderr, "abi_driver: line %d: %s\n", __LINE__, #cond); ++g_failed; } \
    } while (0)

static kvqp_cfg base_cfg() {
    kvqp_cfg c{};
    c.batch = 2; c.n_q_heads = 8; c.n_kv_heads = 2; c.head_dim = 128; c.seq_len = 800; c.window = 32; c.pool_kernel = 7;
    c.budget = 256; c.bits = 4; c.group_size = 64; c.key_axis = KVQP_KEY_PER_CHANNEL; c.sm_scale = 0.088f;
    return c;
}
static void* const kDev = (void*)0x1000;    // stands for device memory: never dereferenced on the host
static kvqp_cache full_cache(bool counts, bool outliers) {
    kvqp_cache k{};
    k.k_codes = k.v_codes = k.k_scale = k.k_zero = k.v_scale = k.v_zero = k.tail_k = k.tail_v = kDev;
    if (counts) k.head_n_kept = (int32_t*)kDev;
    if (outliers) k.k_out = k.v_out = k.k_ovf = k.v_ovf = kDev;
    k.tail_cap = 96;
    return k;
}
// a heap array of exactly n counts
static int32_t* counts(std::initializer_list<int> v) {
    int32_t* p = (int32_t*)std::malloc(v.size() * sizeof(int32_t));
    int i = 0;
    for (int x : v) p[i++] = x;
    return p;
}

static void sizes_sweep() {
    // every size query over the whole supported grid; the results must be consistent with each other
    for (int bits : {2, 4, 8, 16})
        for (int G : {32, 64, 128})
            for (int axis : {0, 1})
                for (int budget : {0, 1, 31, 32, 37, 64, 1000, 4096, 131072, 1 << 30})
                    for (int batch : {1, 3, 8191}) {
                        kvqp_cfg c = base_cfg();
                        c.bits = bits; c.group_size = G; c.key_axis = axis; c.budget = budget; c.batch = batch;
                        c.seq_len = 131072 + 32;
                        size_t s[8], s2[8], o[4], cw = 0, dw = 0;
                        EXPECT(kvqp_cache_sizes(&c, 32, s) == KVQP_OK);
                        const int n = budget < 131072 ? budget : 131072;
                        const size_t heads = (size_t)batch * 2, R = (size_t)(n + 31) / 32 * 32;
                        EXPECT(s[0] == heads * R * 128 * bits / 8);
                        EXPECT(s[6] == heads * 32 * 128 * 2 && s[7] == s[6]);
                        EXPECT(s[2] == s[3] && s[4] == s[5]);
                        if (bits == 16) EXPECT(s[2] == 0 && s[4] == 0);
                        else EXPECT(s[4] == heads * R * (128 / G) * 2);
                        EXPECT(kvqp_workspace_bytes(&c, &cw, &dw) == KVQP_OK && cw > 0 && dw > 0);
                        EXPECT(kvqp_workspace_bytes(&c, nullptr, nullptr) == KVQP_OK);
                        const int cap = (n + 127) / 128 * 128;
                        EXPECT(kvqp_cache_sizes_cap(&c, cap, 40, s2) == KVQP_OK);
                        for (int i = 0; i < 6; ++i) EXPECT(s2[i] >= s[i]);
                        if (bits != 16) {
                            c.outlier_threshold = 6.0f; c.outlier_overflow_cap = 1000;
                            EXPECT(kvqp_outlier_sizes(&c, 0, o) == KVQP_OK);
                            EXPECT(o[0] == heads * R * 16 && o[1] == o[0]);
                            EXPECT(o[2] == o[3] && o[2] >= heads * (R / 32 + 1 + 2000) * 4);
                            c.outlier_threshold = 0.0f;
                            EXPECT(kvqp_outlier_sizes(&c, 0, o) == KVQP_OK && o[0] == 0 && o[2] == 0);
                        }
                    }
}

static void rejected_configurations() {
    struct Patch { void (*f)(kvqp_cfg&); int code; };
    const Patch bad[] = {
        {[](kvqp_cfg& c) { c.bits = 3; }, -1},           {[](kvqp_cfg& c) { c.bits = 0; }, -1},
        {[](kvqp_cfg& c) { c.group_size = 48; }, -1},    {[](kvqp_cfg& c) { c.group_size = 16; }, -2},
        {[](kvqp_cfg& c) { c.group_size = 0; }, -1},     {[](kvqp_cfg& c) { c.head_dim = 64; }, -2},
        {[](kvqp_cfg& c) { c.n_q_heads = 7; }, -1},      {[](kvqp_cfg& c) { c.n_q_heads = 32; }, -2},
        {[](kvqp_cfg& c) { c.n_kv_heads = 0; }, -1},     {[](kvqp_cfg& c) { c.pool_kernel = 4; }, -1},
        {[](kvqp_cfg& c) { c.pool_kernel = 65; }, -2},   {[](kvqp_cfg& c) { c.window = 0; }, -1},
        {[](kvqp_cfg& c) { c.window = 5000; }, -1},      {[](kvqp_cfg& c) { c.budget = -1; }, -1},
        {[](kvqp_cfg& c) { c.key_axis = 2; }, -1},       {[](kvqp_cfg& c) { c.batch = 0; }, -1},
        {[](kvqp_cfg& c) { c.batch = 1 << 30; }, -2},    {[](kvqp_cfg& c) { c.decode_splits = -1; }, -1},
        {[](kvqp_cfg& c) { c.sm_scale = 0.0f; }, -1},    {[](kvqp_cfg& c) { c.sm_scale = -1.0f; }, -1},
        {[](kvqp_cfg& c) { c.decode_cache_hint = 3; }, -1}, {[](kvqp_cfg& c) { c.outlier_overflow_cap = -1; }, -1},
        {[](kvqp_cfg& c) { c.outlier_threshold = -1.0f; }, -1},
        {[](kvqp_cfg& c) { c.seq_len = 1 << 30; }, -2},
    };
    for (const Patch& p : bad) {
        kvqp_cfg c = base_cfg();
        p.f(c);
        size_t s[8];
        kvqp_cache k = full_cache(false, false);
        g_launches = 0;
        EXPECT(kvqp_cache_sizes(&c, 5000, s) == p.code);
        EXPECT(kvqp_compress(&c, kDev, kDev, kDev, &k, nullptr, nullptr, kDev, (size_t)1 << 40, nullptr) == p.code);
        EXPECT(g_launches == 0);
    }
    EXPECT(kvqp_cache_sizes(nullptr, 32, nullptr) == -1);
    kvqp_cfg c = base_cfg();
    EXPECT(kvqp_cache_sizes(&c, 32, nullptr) == -1);
    size_t s[8];
    EXPECT(kvqp_cache_sizes(&c, 31, s) == -1);          // tail shorter than the window
    EXPECT(kvqp_cache_sizes_cap(&c, 100, 32, s) == -1);  // capacity not a multiple of 64
    EXPECT(kvqp_cache_sizes_cap(&c, -64, 32, s) == -1);
    EXPECT(std::strcmp(kvqp_strerror(0), "ok") == 0 && kvqp_strerror(-99) != nullptr && kvqp_version() >= 100);
}

static void compress_and_quantize() {
    kvqp_cfg c = base_cfg();
    kvqp_cache k = full_cache(false, false);
    g_launches = 0;
    EXPECT(kvqp_compress(&c, nullptr, kDev, kDev, &k, nullptr, nullptr, kDev, 1 << 20, nullptr) == -1);
    EXPECT(kvqp_compress(&c, kDev, kDev, kDev, nullptr, nullptr, nullptr, kDev, 1 << 20, nullptr) == -1);
    EXPECT(kvqp_compress(&c, kDev, kDev, kDev, &k, nullptr, nullptr, nullptr, 1 << 20, nullptr) == -3);
    EXPECT(kvqp_compress(&c, kDev, kDev, kDev, &k, nullptr, nullptr, kDev, 100, nullptr) == -3);
    EXPECT(kvqp_compress(&c, kDev, kDev, kDev, &k, nullptr, nullptr, (void*)0x1004, 1 << 20, nullptr) == -1);   // misaligned
    kvqp_cache missing = k;
    missing.v_zero = nullptr;
    EXPECT(kvqp_compress(&c, kDev, kDev, kDev, &missing, nullptr, nullptr, kDev, 1 << 20, nullptr) == -1);
    EXPECT(g_launches == 0 && k.n_kept == 0 && k.tail_len == 0);
    EXPECT(kvqp_compress(&c, kDev, kDev, kDev, &k, (int32_t*)kDev, (int32_t*)kDev, kDev, 1 << 20, nullptr) == 0);
    EXPECT(g_launches == 3 && k.n_kept == 256 && k.tail_len == 32);     // select, copy of the indices, quantizer
    // outlier filtering asks for its four buffers
    c.outlier_threshold = 6.0f;
    EXPECT(kvqp_compress(&c, kDev, kDev, kDev, &k, nullptr, nullptr, kDev, 1 << 20, nullptr) == -1);
    kvqp_cache ko = full_cache(false, true);
    EXPECT(kvqp_compress(&c, kDev, kDev, kDev, &ko, nullptr, nullptr, kDev, 1 << 20, nullptr) == 0);
    c.outlier_threshold = 0.0f;

    // head-level counts: the host array has exactly batch * Hkv = 4 entries
    kvqp_cache kr = full_cache(true, false);
    int32_t* good = counts({256, 0, 37, 1});
    int32_t* high = counts({256, 0, 37, 257});
    int32_t* neg = counts({256, -1, 37, 1});
    g_launches = 0; g_count_sum = 0;
    EXPECT(kvqp_compress_ragged(&c, kDev, kDev, kDev, high, &kr, nullptr, nullptr, kDev, 1 << 20, nullptr) == -1);
    EXPECT(kvqp_compress_ragged(&c, kDev, kDev, kDev, neg, &kr, nullptr, nullptr, kDev, 1 << 20, nullptr) == -1);
    EXPECT(kvqp_compress_ragged(&c, kDev, kDev, kDev, nullptr, &kr, nullptr, nullptr, kDev, 1 << 20, nullptr) == -1);
    EXPECT(kvqp_compress_ragged(&c, kDev, kDev, kDev, good, &k, nullptr, nullptr, kDev, 1 << 20, nullptr) == -1);   // cache without counts
    EXPECT(kvqp_compress(&c, kDev, kDev, kDev, &kr, nullptr, nullptr, kDev, 1 << 20, nullptr) == -1);               // and the reverse
    EXPECT(g_launches == 0);
    EXPECT(kvqp_compress_ragged(&c, kDev, kDev, kDev, good, &kr, nullptr, nullptr, kDev, 1 << 20, nullptr) == 0);
    EXPECT(g_launches == 3 && g_count_sum == 294 && kr.n_kept == 256);   // counts, select, quantizer
    g_launches = 0; g_count_sum = 0;
    EXPECT(kvqp_quantize_selected_ragged(&c, kDev, kDev, (int32_t*)kDev, 256, high, &kr, nullptr) == -1);
    EXPECT(kvqp_quantize_selected_ragged(&c, kDev, kDev, (int32_t*)kDev, 256, nullptr, &kr, nullptr) == -1);
    EXPECT(kvqp_quantize_selected(&c, kDev, kDev, (int32_t*)kDev, 256, &kr, nullptr) == -1);
    EXPECT(kvqp_quantize_selected(&c, kDev, kDev, nullptr, 256, &k, nullptr) == -1);
    EXPECT(kvqp_quantize_selected(&c, kDev, kDev, (int32_t*)kDev, 769, &k, nullptr) == -1);   // more than the prefix holds
    EXPECT(g_launches == 0);
    EXPECT(kvqp_quantize_selected_ragged(&c, kDev, kDev, (int32_t*)kDev, 256, good, &kr, nullptr) == 0 && g_count_sum == 294);
    EXPECT(kvqp_quantize_selected(&c, kDev, kDev, (int32_t*)kDev, 100, &k, nullptr) == 0 && k.n_kept == 100);
    // a budget of zero tokens: nothing is selected, the cut counts are zeroed
    c.budget = 0;
    g_launches = 0;
    EXPECT(kvqp_compress(&c, kDev, kDev, kDev, &k, nullptr, (int32_t*)kDev, kDev, 1 << 20, nullptr) == 0 && k.n_kept == 0);
    EXPECT(g_launches == 2);
    std::free(good); std::free(high); std::free(neg);
}

static void append_and_decode() {
    kvqp_cfg c = base_cfg();
    kvqp_cache k = full_cache(false, false);
    k.n_kept = 256; k.tail_len = 96; k.n_cap = 384;
    g_launches = 0;
    EXPECT(kvqp_append_tail(nullptr, &k, 64, nullptr) == -1);
    EXPECT(kvqp_append_tail(&c, nullptr, 64, nullptr) == -1);
    EXPECT(kvqp_append_tail(&c, &k, 0, nullptr) == -1);
    EXPECT(kvqp_append_tail(&c, &k, 32, nullptr) == -1);     // not whole key groups of 64
    EXPECT(kvqp_append_tail(&c, &k, 128, nullptr) == -1);    // more than the tail holds
    k.tail_cap = 256; k.tail_len = 256;
    EXPECT(kvqp_append_tail(&c, &k, 192, nullptr) == -1);    // beyond the capacity
    EXPECT(g_launches == 0 && k.n_kept == 256 && k.tail_len == 256);
    EXPECT(kvqp_append_tail(&c, &k, 128, nullptr) == 0 && k.n_kept == 384 && k.tail_len == 128 && g_launches == 1);
    kvqp_cache kr = full_cache(true, false);
    kr.n_kept = 256; kr.tail_len = 64; kr.n_cap = 320;
    int32_t* cur = counts({256, 0, 64, 128});
    int32_t* odd = counts({256, 0, 37, 128});
    g_launches = 0; g_count_sum = 0;
    EXPECT(kvqp_append_tail(&c, &kr, 64, nullptr) == -2);
    EXPECT(kvqp_append_tail_ragged(&c, &kr, 64, nullptr, nullptr) == -1);
    EXPECT(kvqp_append_tail_ragged(&c, &kr, 64, odd, nullptr) == -1);
    EXPECT(kvqp_append_tail_ragged(&c, &k, 64, cur, nullptr) == -1);
    EXPECT(g_launches == 0);
    EXPECT(kvqp_append_tail_ragged(&c, &kr, 64, cur, nullptr) == 0 && g_count_sum == 448 + 4 * 64 && kr.n_kept == 320);
    std::free(cur); std::free(odd);

    // decode: both entry points share their checks
    kvqp_cache d = full_cache(false, false);
    d.n_kept = 1000; d.tail_len = 32;
    const size_t need = 256 + 4096;
    g_launches = 0;
    EXPECT(kvqp_decode_attn(&c, nullptr, &d, kDev, kDev, need, nullptr) == -1);
    EXPECT(kvqp_decode_attn(&c, kDev, nullptr, kDev, kDev, need, nullptr) == -1);
    EXPECT(kvqp_decode_attn(&c, kDev, &d, nullptr, kDev, need, nullptr) == -1);
    EXPECT(kvqp_decode_attn(&c, kDev, &d, kDev, nullptr, need, nullptr) == -3);
    EXPECT(kvqp_decode_attn(&c, kDev, &d, kDev, kDev, need - 1, nullptr) == -3);
    EXPECT(kvqp_decode_attn(&c, kDev, &d, kDev, (void*)0x1008, need, nullptr) == -1);
    d.tail_len = 97;
    EXPECT(kvqp_decode_attn(&c, kDev, &d, kDev, kDev, need, nullptr) == -1);
    EXPECT(kvqp_decode_attn_static(&c, kDev, &d, kDev, nullptr) == -1);
    d.tail_len = 0; d.n_kept = 0;
    EXPECT(kvqp_decode_attn(&c, kDev, &d, kDev, kDev, need, nullptr) == -1);
    d.n_kept = -5; d.tail_len = 32;
    EXPECT(kvqp_decode_attn(&c, kDev, &d, kDev, kDev, need, nullptr) == -1);
    EXPECT(g_launches == 0);
    d.n_kept = 1000;
    EXPECT(kvqp_decode_attn(&c, kDev, &d, kDev, kDev, need, nullptr) == 0 && g_launches == 1);
    EXPECT(kvqp_decode_attn_static(&c, kDev, &d, kDev, nullptr) == 0 && g_launches == 2);
    d.n_kept = 0;          // only tail rows: the packed buffers may be absent
    d.k_codes = d.v_codes = d.k_scale = d.k_zero = d.v_scale = d.v_zero = nullptr;
    EXPECT(kvqp_decode_attn(&c, kDev, &d, kDev, kDev, need, nullptr) == 0);
    g_launches = 0;
    EXPECT(kvqp_decode_workspace_init(&c, nullptr, 256, nullptr) == -3);
    EXPECT(kvqp_decode_workspace_init(&c, kDev, 255, nullptr) == -3);
    EXPECT(kvqp_decode_workspace_init(nullptr, kDev, 256, nullptr) == -1);
    EXPECT(g_launches == 0);
    EXPECT(kvqp_decode_workspace_init(&c, kDev, 256, nullptr) == 0 && g_launches == 1);
}

int main() {
    sizes_sweep();
    rejected_configurations();
    compress_and_quantize();
    append_and_decode();
    if (g_failed) { std::fprintf(stderr, "abi_driver: %d checks failed\n", g_failed); return 1; }
    std::printf("abi_driver: clean\n");
    return 0;
}
