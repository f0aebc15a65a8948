/*
 * kvqp_oracle.c -- CPU oracle for the quantized-pruned KV cache.
 *
 * THIS IS TEST INFRASTRUCTURE, NOT PRODUCT CODE.  It is a plain, slow,
 * step-by-step statement of what the hot path computes, written from the
 * paper (arXiv 2412.12706, "More Tokens, Lower Precision"), used only by the
 * tests, the smoke check and the benchmark's CPU-baseline leg.  It shares no
 * code, header, table or helper with the HIP library and must never be
 * called from the product path.
 *
 * Parity pins (tests/test_oracle_*.py): identity selection when the budget
 * covers the prefix; top-k of raw logits when W=1, pool=1, Gq=1; brute force
 * on tiny L; quantization closed forms (ramp, constant, two-valued groups,
 * end codes, scale/2 error bound, exact rational cross-check); 16-bit mode
 * equal to textbook softmax attention computed by an independent library
 * routine; half<->float conversions against numpy.  No function here is
 * "parity unpinned"; what is *defined* rather than derived (window votes,
 * pooling, tie rule, bit layout) is listed with each function.
 *
 * Arithmetic: float64 everywhere a real-valued result is produced (votes,
 * attention).  Quantized codes are integers decided by floating point, so
 * that decision is taken in the precision the kernel uses: a fixed IEEE
 * binary32 operation sequence, round-to-nearest-even, no fused multiply-add
 * (build with -ffp-contract=off, never -ffast-math).
 *
 * Notation follows the paper, Section 3 (Methods): X_K, X_V are the cached
 * keys/values, s the token budget, B the bit width, G_i a quantization
 * group with minimum z_i, maximum m_i and scale s_i.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

/* ------------------------------------------------------------------ */
/* binary16 <-> binary32/64, written out bit by bit (gcc 11 has no      */
/* _Float16 on x86-64).  Pinned against numpy's float16 in the tests.   */
/* ------------------------------------------------------------------ */

double orc_half_to_double(uint16_t h)
{
    int sign = (h >> 15) & 1;
    int e = (h >> 10) & 0x1f;
    int m = h & 0x3ff;
    double v;
    if (e == 0)
        v = ldexp((double)m, -24); /* zero and subnormals */
    else if (e == 31)
        v = m ? NAN : INFINITY;
    else
        v = ldexp((double)(1024 + m), e - 25);
    return sign ? -v : v;
}

/* binary32 -> binary16, round to nearest, ties to even. */
uint16_t orc_float_to_half(float f)
{
    uint32_t x;
    memcpy(&x, &f, 4);
    uint16_t sign = (uint16_t)((x >> 16) & 0x8000u);
    uint32_t a = x & 0x7fffffffu;
    if (a >= 0x7f800000u) /* inf / nan */
        return (uint16_t)(sign | 0x7c00u | (a > 0x7f800000u ? 0x200u : 0));
    if (a >= 0x477ff000u) /* >= 65520 rounds to inf */
        return (uint16_t)(sign | 0x7c00u);
    if (a < 0x33000000u) /* below 2^-25: rounds to zero (2^-25 itself is handled below) */
        return sign;
    int e = (int)(a >> 23) - 127; /* unbiased */
    uint32_t man = (a & 0x7fffffu) | 0x800000u; /* 24-bit significand */
    int shift; /* number of low bits dropped */
    uint32_t base;
    if (e < -14) { /* result is subnormal: value = man * 2^(e-23), unit 2^-24 */
        shift = -1 - e; /* (e-23) - (-24) = e+1 -> drop -(e+1) bits */
        base = 0;
    } else {
        shift = 13;
        base = (uint32_t)(e + 15) << 10;
        man &= 0x7fffffu;
    }
    uint32_t q = man >> shift;
    uint32_t rem = man & ((1u << shift) - 1);
    uint32_t half = 1u << (shift - 1);
    if (rem > half || (rem == half && (q & 1)))
        q += 1; /* carry may roll into the exponent, which is the right answer */
    return (uint16_t)(sign | (base + q));
}

void orc_float_to_half_array(const float *in, uint16_t *out, size_t n)
{
    for (size_t i = 0; i < n; ++i)
        out[i] = orc_float_to_half(in[i]);
}

void orc_half_to_double_array(const uint16_t *in, double *out, size_t n)
{
    for (size_t i = 0; i < n; ++i)
        out[i] = orc_half_to_double(in[i]);
}

static float half_to_float(uint16_t h) { return (float)orc_half_to_double(h); /* exact */ }

/* ------------------------------------------------------------------ */
/* Selection (KV pruning, Section 3 "KV Pruning": pick s < n tokens at  */
/* prefill).  The paper cites an attention-score method and keeps the   */
/* last 32 tokens (Appendix B); the scoring details below -- window     */
/* votes, causal mask inside the window, sum over the query-head group, */
/* one max-pool, (score desc, index asc) order -- are this build's      */
/* stated reading, since the paper is silent on them.                   */
/* ------------------------------------------------------------------ */

/*
 * Window votes.  For KV head g and each query head h of its group, each of
 * the last W prompt positions i (absolute position P+i, P = L-W) attends
 * causally over keys 0..P+i with Softmax(sm_scale * q k^T) (the decode
 * attention form of Section 3, Eq. "attno", with an explicit scale); the
 * vote of prefix key j < P is the sum of those probabilities over the group's
 * heads and the W rows.
 *   q_obs [B,Hq,W,D] half, k [B,Hkv,L,D] half -> vote [B,Hkv,P] double
 */
int orc_window_votes(int B, int Hq, int Hkv, int D, int L, int W, double sm_scale,
                     const uint16_t *q_obs, const uint16_t *k, double *vote)
{
    if (B < 1 || Hkv < 1 || Hq % Hkv || W < 1 || W > L || D < 1)
        return -1;
    const int Gq = Hq / Hkv, P = L - W;
    int status = 0;
#pragma omp parallel for collapse(2) schedule(dynamic)
    for (int b = 0; b < B; ++b)
        for (int g = 0; g < Hkv; ++g) {
            double *a = (double *)malloc(sizeof(double) * (size_t)L);
            double *kd = (double *)malloc(sizeof(double) * (size_t)L * D);
            if (!a || !kd) {
                status = -2;
                free(a);
                free(kd);
                continue;
            }
            const uint16_t *kh = k + ((size_t)b * Hkv + g) * (size_t)L * D;
            for (size_t e = 0; e < (size_t)L * D; ++e)
                kd[e] = orc_half_to_double(kh[e]);
            double *vt = vote + ((size_t)b * Hkv + g) * (size_t)P;
            for (int j = 0; j < P; ++j)
                vt[j] = 0.0;
            for (int h = g * Gq; h < (g + 1) * Gq; ++h)
                for (int i = 0; i < W; ++i) {
                    const uint16_t *qr = q_obs + (((size_t)b * Hq + h) * W + i) * (size_t)D;
                    const int last = P + i; /* causal: keys 0..P+i */
                    double mx = -INFINITY;
                    for (int j = 0; j <= last; ++j) {
                        double s = 0.0;
                        for (int d = 0; d < D; ++d)
                            s += orc_half_to_double(qr[d]) * kd[(size_t)j * D + d];
                        a[j] = sm_scale * s;
                        if (a[j] > mx)
                            mx = a[j];
                    }
                    double Z = 0.0;
                    for (int j = 0; j <= last; ++j)
                        Z += exp(a[j] - mx);
                    for (int j = 0; j < P; ++j)
                        vt[j] += exp(a[j] - mx) / Z;
                }
            free(a);
            free(kd);
        }
    return status;
}

/* 1-D max-pool, stride 1, same length, window clipped at both ends (a kernel
 * of 1 is the identity).  Applied to the prefix votes only. */
int orc_max_pool(int rows, int P, int pool, const double *vote, double *pooled)
{
    if (pool < 1 || pool % 2 == 0)
        return -1;
    const int r = (pool - 1) / 2;
    for (int row = 0; row < rows; ++row)
        for (int j = 0; j < P; ++j) {
            double best = -INFINITY;
            for (int t = -r; t <= r; ++t)
                if (j + t >= 0 && j + t < P && vote[(size_t)row * P + j + t] > best)
                    best = vote[(size_t)row * P + j + t];
            pooled[(size_t)row * P + j] = best;
        }
    return 0;
}

typedef struct {
    double score;
    int32_t index;
} scored;

static int by_score_desc_index_asc(const void *pa, const void *pb)
{
    const scored *a = (const scored *)pa, *b = (const scored *)pb;
    if (a->score > b->score)
        return -1;
    if (a->score < b->score)
        return 1;
    return (a->index > b->index) - (a->index < b->index);
}

static int by_int_asc(const void *pa, const void *pb)
{
    int32_t a = *(const int32_t *)pa, b = *(const int32_t *)pb;
    return (a > b) - (a < b);
}

/* The k highest pooled scores of one head; equal scores go to the lower
 * position; the result is listed in ascending position. */
int orc_topk(int P, int k, const double *pooled, int32_t *idx)
{
    if (k < 0 || k > P)
        return -1;
    scored *c = (scored *)malloc(sizeof(scored) * (size_t)(P > 0 ? P : 1));
    if (!c)
        return -2;
    for (int j = 0; j < P; ++j) {
        c[j].score = pooled[j];
        c[j].index = j;
    }
    qsort(c, (size_t)P, sizeof(scored), by_score_desc_index_asc);
    for (int t = 0; t < k; ++t)
        idx[t] = c[t].index;
    qsort(idx, (size_t)k, sizeof(int32_t), by_int_asc);
    free(c);
    return 0;
}

/* ------------------------------------------------------------------ */
/* Quantization (Section 3 "KV Quantization"):                          */
/*   z = min G, m = max G, s = (m - z)/(2^B - 1), Q(G) = round((G-z)/s) */
/* and G' = Q(G)*s + z.  The stored s is binary16, rounded before the   */
/* codes are formed so that codes and dequantization agree; z is an     */
/* input value, hence exact in binary16.                                */
/* ------------------------------------------------------------------ */

/*
 * One group of n binary16 values x[0], x[stride], ...  Writes the stored
 * scale and zero (binary16 bit patterns) and n codes in [0, 2^bits).
 * binary32 sequence: r = m - z; s32 = r / (2^bits - 1); s_h = half(s32);
 * if s_h == 0 every code is 0 (constant group, or range below half
 * resolution); else inv = 1 / float(s_h); code = clamp(rint((x - z) * inv)).
 * Ties in rint go to even.  When the group holds both -0 and +0 as extremes
 * the minimum is -0 (IEEE minimum ordering).
 */
static int quantize_group_excl(const uint16_t *x, int n, int stride, int bits, const uint8_t *excl,
                               int excl_stride, uint16_t *scale, uint16_t *zero, uint8_t *codes)
{
    if (n < 1 || !(bits == 2 || bits == 4 || bits == 8))
        return -1;
    int have = 0;
    uint16_t zb = 0, mb = 0; /* +0: what a group with nothing left to quantize stores */
    for (int i = 0; i < n; ++i) {
        if (excl && excl[(size_t)i * excl_stride])
            continue;
        uint16_t xb = x[(size_t)i * stride];
        if (!have) {
            zb = mb = xb;
            have = 1;
            continue;
        }
        double v = orc_half_to_double(xb), lo = orc_half_to_double(zb), hi = orc_half_to_double(mb);
        if (v < lo || (v == lo && (xb & 0x8000) && !(zb & 0x8000)))
            zb = xb;
        if (v > hi || (v == hi && !(xb & 0x8000) && (mb & 0x8000)))
            mb = xb;
    }
    const float zf = half_to_float(zb), mf = half_to_float(mb);
    const float levels = (float)((1 << bits) - 1);
    volatile float r = mf - zf;
    volatile float s32 = r / levels;
    const uint16_t sh = orc_float_to_half(s32);
    const float sf = half_to_float(sh);
    *scale = sh;
    *zero = zb;
    if (sf == 0.0f) {
        for (int i = 0; i < n; ++i)
            codes[i] = 0;
        return 0;
    }
    volatile float inv = 1.0f / sf;
    for (int i = 0; i < n; ++i) {
        if (excl && excl[(size_t)i * excl_stride]) {
            codes[i] = 0;
            continue;
        }
        volatile float diff = half_to_float(x[(size_t)i * stride]) - zf;
        volatile float scaled = diff * inv;
        float c = rintf(scaled);
        if (c < 0.0f)
            c = 0.0f;
        if (c > levels)
            c = levels;
        codes[i] = (uint8_t)c;
    }
    return 0;
}

int orc_quantize_group(const uint16_t *x, int n, int stride, int bits, uint16_t *scale,
                       uint16_t *zero, uint8_t *codes)
{
    return quantize_group_excl(x, n, stride, bits, NULL, 0, scale, zero, codes);
}

/* ------------------------------------------------------------------ */
/* Outlier filtering (Section 6.3, item (1); Appendix B "KV             */
/* quantization": numbers whose absolute value exceeds a threshold, 6   */
/* in the paper, about 1 % of them, are excluded from quantization).    */
/* Every element of a kept token's key row or value row with |x| > tau  */
/* is an outlier -- there is no limit per row.  An outlier takes no     */
/* part in its group's min / max, gets code 0, and is kept at full      */
/* precision beside the codes as a 32-bit word: the top 24 bits of the  */
/* binary32 difference float(x) - float(z) (z the stored zero-point of  */
/* the element's group), a valid bit (bit 7) and the channel (bits      */
/* 0-6); the element dequantizes to float(z) + difference.  A group     */
/* left with no element stores scale 0, zero +0.                        */
/* Where the words go is storage format (the paper gives none): a       */
/* row's first ORC_OUT_SLOTS outliers in ascending channel order sit    */
/* in the row's slots (unused slots are 0); a row's further outliers    */
/* go, in ascending (token, channel) order, to the head's overflow      */
/* list as entries (word, token), with a prefix count per block of 32   */
/* tokens in front of it:                                               */
/*   int32  start[ceil(n_tok/32) + 1], padded to a multiple of 4 ints:  */
/*          start[b] = overflow entries of tokens before 32 b           */
/*   uint32 entry[ovf_cap][2] = (word, token index in the head)         */
/* Entries beyond ovf_cap are not stored (start[] still counts them, so  */
/* the shortfall is visible); such an element dequantizes to z.         */
/* ------------------------------------------------------------------ */
#define ORC_OUT_SLOTS 4

/* is_out[d] = 1 + (number of outliers of the row in lower channels) for the row's outliers,
 * 0 elsewhere (D <= 128, so the count fits a byte).  Returns how many there are. */
int orc_mark_outliers(const uint16_t *row, int D, double tau, uint8_t *is_out)
{
    int n = 0;
    for (int d = 0; d < D; ++d) {
        double mag = fabs(orc_half_to_double(row[d]));
        is_out[d] = mag > tau ? (uint8_t)(++n) : 0;
    }
    return n;
}

int orc_rows(int n_tok); /* the token count rounded up to whole blocks of 32 (defined with the layouts) */

/* Words of one head's overflow buffer laid out for n_tok tokens and cap entries (format above). */
size_t orc_ovf_words(int n_tok, int cap)
{
    size_t start = ((size_t)(orc_rows(n_tok) / 32 + 1) + 3) / 4 * 4;
    return start + 2 * (size_t)cap;
}

/* Slot word of an outlier x in channel d whose group stores zero-point zb. */
uint32_t orc_outlier_slot(uint16_t x, uint16_t zb, int d)
{
    volatile float diff = half_to_float(x) - half_to_float(zb);
    float f = diff;
    uint32_t u;
    memcpy(&u, &f, 4);
    return (u & 0xFFFFFF00u) | 0x80u | (uint32_t)d;
}

/* The value a slot word stands for, given its group's zero-point. */
double orc_outlier_value(uint32_t slot, uint16_t zb)
{
    uint32_t u = slot & 0xFFFFFF00u;
    float f;
    memcpy(&f, &u, 4);
    return orc_half_to_double(zb) + (double)f;
}

/* ------------------------------------------------------------------ */
/* Bit layout of the packed cache.  The paper gives none; this is the   */
/* library's storage format, restated here from its specification.      */
/*                                                                      */
/* A 32-bit word holds E = 32/bits fields.  Field p of the low half     */
/* (bits [bits*p, bits*p+bits)) and field p of the high half (16 bits   */
/* higher) always hold a *pair*.                                        */
/*  Keys: row-major [token][channel]; word (t, d / E); within the word  */
/*    the pair is two adjacent channels: r = d % E, p = r / 2,          */
/*    half = r % 2.  At 16 bits this is plain little-endian binary16.   */
/*  Values: tokens are taken in blocks of 32; token t = 32*blk + 16*H   */
/*    + 4*kb + i (H in {0,1}, kb, i in 0..3); channel d = 16*tile + n.  */
/*    The pair is (H=0, H=1): tokens 16 apart.  For fixed (kb, d) the   */
/*    fields with running index 4*blk + i fill successive low halves    */
/*    (and the H=1 partners the high halves), E/2 per word.  A          */
/*    superblock is SB = max(32, 2E) tokens and holds, per lane         */
/*    (kb, n), nw = (D/16) * (SB/2) / (E/2) ... words, ordered          */
/*    y = tile * wpt + (word within tile); the word sits at             */
/*    ((y / 4) * 64 + kb * 16 + n) * 4 + y % 4 inside the superblock.   */
/*    Tokens past n_kept inside the last superblock hold code 0.        */
/* ------------------------------------------------------------------ */

static int fields_per_word(int bits) { return 32 / bits; }

/* Token counts need not fill whole blocks or groups (Section 3: any s < n).  The per-token arrays
 * of a head (key code rows, per-token scales and zeros, outlier slots) are laid out for the count
 * rounded up to whole blocks of 32 tokens, the rows past the count holding zeros; per-channel key
 * groups number ceil(n / G), the last one having fewer than G members when G does not divide n. */
int orc_rows(int n_tok) { return (n_tok + 31) / 32 * 32; }
int orc_key_groups(int n_tok, int G) { return (n_tok + G - 1) / G; }

size_t orc_k_words(int n_tok, int D, int bits) { return (size_t)orc_rows(n_tok) * D * bits / 32; }

static void k_locate(int D, int bits, int t, int d, size_t *word, int *shift)
{
    const int E = fields_per_word(bits);
    const int r = d % E;
    *word = (size_t)t * (D / E) + d / E;
    *shift = 16 * (r % 2) + bits * (r / 2);
}

static int v_superblock(int bits) { return bits == 2 ? 64 : 32; }

/* words one lane (kb, n) holds per tile per superblock */
static int v_words_per_tile(int bits) { return bits == 16 ? 4 : bits == 8 ? 2 : 1; }

size_t orc_v_words(int n_tok, int D, int bits)
{
    const int SB = v_superblock(bits);
    const size_t nsb = ((size_t)n_tok + SB - 1) / SB;
    return nsb * 64 * (size_t)(D / 16) * v_words_per_tile(bits);
}

static void v_locate(int D, int bits, int t, int d, size_t *word, int *shift)
{
    const int E = fields_per_word(bits);
    const int SB = v_superblock(bits);
    const int wpt = v_words_per_tile(bits);
    const int sb = t / SB, ts = t % SB;
    const int blk = ts / 32, H = (ts % 32) / 16, kb = (ts % 16) / 4, i = ts % 4;
    const int tile = d / 16, n = d % 16;
    const int run = 4 * blk + i;    /* running field index inside the superblock */
    const int wl = run / (E / 2);   /* word within the tile                       */
    const int p = run % (E / 2);    /* field within the half                      */
    const int y = tile * wpt + wl;
    const size_t sb_words = 64 * (size_t)(D / 16) * wpt;
    *word = sb * sb_words + ((size_t)(y / 4) * 64 + kb * 16 + n) * 4 + y % 4;
    *shift = 16 * H + bits * p;
}

static uint32_t field_mask(int bits) { return bits == 16 ? 0xffffu : ((1u << bits) - 1u); }

uint32_t orc_k_code_get(const uint32_t *codes, int D, int bits, int t, int d)
{
    size_t w;
    int sh;
    k_locate(D, bits, t, d, &w, &sh);
    return (codes[w] >> sh) & field_mask(bits);
}

uint32_t orc_v_code_get(const uint32_t *codes, int D, int bits, int t, int d)
{
    size_t w;
    int sh;
    v_locate(D, bits, t, d, &w, &sh);
    return (codes[w] >> sh) & field_mask(bits);
}

static void k_code_put(uint32_t *codes, int D, int bits, int t, int d, uint32_t c)
{
    size_t w;
    int sh;
    k_locate(D, bits, t, d, &w, &sh);
    codes[w] |= (c & field_mask(bits)) << sh;
}

static void v_code_put(uint32_t *codes, int D, int bits, int t, int d, uint32_t c)
{
    size_t w;
    int sh;
    v_locate(D, bits, t, d, &w, &sh);
    codes[w] |= (c & field_mask(bits)) << sh;
}

/* ------------------------------------------------------------------ */
/* Quantized pruning of given survivors (Section 3 "Quantized Pruning": */
/* prune first, then quantize the preserved states).  idx lists, per    */
/* (b, g), n_kept ascending prefix positions.  Keys: key_axis 0 groups  */
/* G consecutive *kept tokens* of one channel (per-channel, the KIVI    */
/* axis); key_axis 1 groups G consecutive channels of one token         */
/* (per-token, the FlexGen axis).  Values are always per-token.  The    */
/* last W prompt rows are copied unquantized into the tail.             */
/*   k_scale/k_zero: [B,Hkv,ceil(n_kept/G),D] (axis 0) or              */
/*                   [B,Hkv,rows,D/G], rows = orc_rows(n_kept)          */
/*   v_scale/v_zero: [B,Hkv,rows,D/G]                                   */
/* When G does not divide n_kept the last per-channel key group has the */
/* remaining n_kept mod G tokens: the same quantizer on fewer members.  */
/*   tail_k/tail_v : [B,Hkv,tail_cap,D], first W rows written           */
/* ------------------------------------------------------------------ */
/* tau < 0: no outlier filtering (k_out, v_out, k_ovf, v_ovf unused).  Otherwise k_out, v_out
 * [B,Hkv,rows,ORC_OUT_SLOTS] receive the slot words and k_ovf, v_ovf
 * [B,Hkv,orc_ovf_words(n_kept, ovf_cap)] the overflow buffers (bits 2, 4, 8 only). */
static int quantize_selected_impl(int B, int Hkv, int D, int L, int W, int n_kept, int bits, int G,
                                  int key_axis, int tail_cap, const uint16_t *k, const uint16_t *v,
                                  const int32_t *idx, uint32_t *k_codes, uint32_t *v_codes,
                                  uint16_t *k_scale, uint16_t *k_zero, uint16_t *v_scale,
                                  uint16_t *v_zero, uint16_t *tail_k, uint16_t *tail_v, double tau,
                                  uint32_t *k_out, uint32_t *v_out, int ovf_cap, uint32_t *k_ovf,
                                  uint32_t *v_ovf)
{
    if (!(bits == 2 || bits == 4 || bits == 8 || bits == 16) || D % 64 || W > tail_cap || W > L)
        return -1;
    const int filt = tau >= 0.0;
    if (filt && (bits == 16 || !k_out || !v_out || !k_ovf || !v_ovf || ovf_cap < 0 || D > 128))
        return -1;
    if (bits != 16 && (G < 1 || D % G))
        return -1;
    const int rows = orc_rows(n_kept), n_groups = bits == 16 ? 0 : orc_key_groups(n_kept, G);
    const int P = L - W;
    const size_t kw = orc_k_words(n_kept, D, bits), vw = orc_v_words(n_kept, D, bits);
    uint8_t *codes = (uint8_t *)malloc((size_t)(G > D ? G : D) + 1);
    uint8_t *kmask = filt ? (uint8_t *)malloc((size_t)(n_kept > 0 ? n_kept : 1) * D) : NULL;
    uint8_t *vmask = filt ? (uint8_t *)malloc((size_t)(n_kept > 0 ? n_kept : 1) * D) : NULL;
    if (!codes || (filt && (!kmask || !vmask))) {
        free(codes);
        free(kmask);
        free(vmask);
        return -2;
    }
    for (int b = 0; b < B; ++b)
        for (int g = 0; g < Hkv; ++g) {
            const size_t head = (size_t)b * Hkv + g;
            const uint16_t *kh = k + head * (size_t)L * D, *vh = v + head * (size_t)L * D;
            const int32_t *id = idx + head * (size_t)n_kept;
            uint32_t *kc = k_codes + head * kw, *vc = v_codes + head * vw;
            memset(kc, 0, kw * 4);
            memset(vc, 0, vw * 4);
            for (int t = 0; t < n_kept; ++t)
                if (id[t] < 0 || id[t] >= P) {
                    free(codes);
                    free(kmask);
                    free(vmask);
                    return -3;
                }
            if (filt)
                for (int t = 0; t < n_kept; ++t) {
                    orc_mark_outliers(kh + (size_t)id[t] * D, D, tau, kmask + (size_t)t * D);
                    orc_mark_outliers(vh + (size_t)id[t] * D, D, tau, vmask + (size_t)t * D);
                }
            if (bits == 16) {
                for (int t = 0; t < n_kept; ++t)
                    for (int d = 0; d < D; ++d) {
                        k_code_put(kc, D, 16, t, d, kh[(size_t)id[t] * D + d]);
                        v_code_put(vc, D, 16, t, d, vh[(size_t)id[t] * D + d]);
                    }
            } else {
                if (key_axis == 0) {
                    uint16_t *gath = (uint16_t *)malloc(sizeof(uint16_t) * (size_t)G);
                    for (int u = 0; u < n_groups; ++u) {
                        const int members = n_kept - u * G < G ? n_kept - u * G : G; /* the last group may be short */
                        for (int d = 0; d < D; ++d) {
                            for (int e = 0; e < members; ++e)
                                gath[e] = kh[(size_t)id[u * G + e] * D + d];
                            size_t m = (head * (size_t)n_groups + u) * D + d;
                            quantize_group_excl(gath, members, 1, bits,
                                                filt ? kmask + (size_t)u * G * D + d : NULL, D,
                                                &k_scale[m], &k_zero[m], codes);
                            for (int e = 0; e < members; ++e)
                                k_code_put(kc, D, bits, u * G + e, d, codes[e]);
                        }
                    }
                    free(gath);
                } else {
                    for (int t = 0; t < n_kept; ++t)
                        for (int c = 0; c < D / G; ++c) {
                            size_t m = (head * (size_t)rows + t) * (D / G) + c;
                            quantize_group_excl(kh + (size_t)id[t] * D + c * G, G, 1, bits,
                                                filt ? kmask + (size_t)t * D + c * G : NULL, 1,
                                                &k_scale[m], &k_zero[m], codes);
                            for (int e = 0; e < G; ++e)
                                k_code_put(kc, D, bits, t, c * G + e, codes[e]);
                        }
                }
                for (int t = 0; t < n_kept; ++t)
                    for (int c = 0; c < D / G; ++c) {
                        size_t m = (head * (size_t)rows + t) * (D / G) + c;
                        quantize_group_excl(vh + (size_t)id[t] * D + c * G, G, 1, bits,
                                            filt ? vmask + (size_t)t * D + c * G : NULL, 1,
                                            &v_scale[m], &v_zero[m], codes);
                        for (int e = 0; e < G; ++e)
                            v_code_put(vc, D, bits, t, c * G + e, codes[e]);
                    }
            }
            if (filt) {
                const size_t ow = orc_ovf_words(n_kept, ovf_cap);
                const size_t n_start = ow - 2 * (size_t)ovf_cap;
                uint32_t *kov = k_ovf + head * ow, *vov = v_ovf + head * ow;
                memset(kov, 0, ow * 4);
                memset(vov, 0, ow * 4);
                int32_t nko = 0, nvo = 0; /* overflow entries so far */
                for (int t = 0; t < n_kept; ++t) {
                    uint32_t *ko = k_out + (head * (size_t)rows + t) * ORC_OUT_SLOTS;
                    uint32_t *vo = v_out + (head * (size_t)rows + t) * ORC_OUT_SLOTS;
                    memset(ko, 0, sizeof(uint32_t) * ORC_OUT_SLOTS);
                    memset(vo, 0, sizeof(uint32_t) * ORC_OUT_SLOTS);
                    if (t % 32 == 0) {
                        kov[t / 32] = (uint32_t)nko;
                        vov[t / 32] = (uint32_t)nvo;
                    }
                    for (int d = 0; d < D; ++d) { /* ascending channel */
                        size_t mk = key_axis == 0 ? (head * (size_t)n_groups + t / G) * D + d
                                                  : (head * (size_t)rows + t) * (D / G) + d / G;
                        size_t mv = (head * (size_t)rows + t) * (D / G) + d / G;
                        const int rk = kmask[(size_t)t * D + d], rv = vmask[(size_t)t * D + d];
                        if (rk) {
                            uint32_t w = orc_outlier_slot(kh[(size_t)id[t] * D + d], k_zero[mk], d);
                            if (rk <= ORC_OUT_SLOTS)
                                ko[rk - 1] = w;
                            else {
                                if (nko < ovf_cap) {
                                    kov[n_start + 2 * (size_t)nko] = w;
                                    kov[n_start + 2 * (size_t)nko + 1] = (uint32_t)t;
                                }
                                ++nko;
                            }
                        }
                        if (rv) {
                            uint32_t w = orc_outlier_slot(vh[(size_t)id[t] * D + d], v_zero[mv], d);
                            if (rv <= ORC_OUT_SLOTS)
                                vo[rv - 1] = w;
                            else {
                                if (nvo < ovf_cap) {
                                    vov[n_start + 2 * (size_t)nvo] = w;
                                    vov[n_start + 2 * (size_t)nvo + 1] = (uint32_t)t;
                                }
                                ++nvo;
                            }
                        }
                    }
                }
                kov[rows / 32] = (uint32_t)nko;
                vov[rows / 32] = (uint32_t)nvo;
            }
            for (int i = 0; i < W; ++i) {
                memcpy(tail_k + (head * tail_cap + i) * (size_t)D, kh + (size_t)(P + i) * D,
                       sizeof(uint16_t) * (size_t)D);
                memcpy(tail_v + (head * tail_cap + i) * (size_t)D, vh + (size_t)(P + i) * D,
                       sizeof(uint16_t) * (size_t)D);
            }
        }
    free(codes);
    free(kmask);
    free(vmask);
    return 0;
}

int orc_quantize_selected(int B, int Hkv, int D, int L, int W, int n_kept, int bits, int G,
                          int key_axis, int tail_cap, const uint16_t *k, const uint16_t *v,
                          const int32_t *idx, uint32_t *k_codes, uint32_t *v_codes,
                          uint16_t *k_scale, uint16_t *k_zero, uint16_t *v_scale,
                          uint16_t *v_zero, uint16_t *tail_k, uint16_t *tail_v)
{
    return quantize_selected_impl(B, Hkv, D, L, W, n_kept, bits, G, key_axis, tail_cap, k, v, idx,
                                  k_codes, v_codes, k_scale, k_zero, v_scale, v_zero, tail_k,
                                  tail_v, -1.0, NULL, NULL, 0, NULL, NULL);
}

/* The same with outlier filtering at threshold tau >= 0. */
int orc_quantize_selected_outliers(int B, int Hkv, int D, int L, int W, int n_kept, int bits,
                                   int G, int key_axis, int tail_cap, double tau,
                                   const uint16_t *k, const uint16_t *v, const int32_t *idx,
                                   uint32_t *k_codes, uint32_t *v_codes, uint16_t *k_scale,
                                   uint16_t *k_zero, uint16_t *v_scale, uint16_t *v_zero,
                                   uint16_t *tail_k, uint16_t *tail_v, uint32_t *k_out,
                                   uint32_t *v_out, int ovf_cap, uint32_t *k_ovf, uint32_t *v_ovf)
{
    if (tau < 0.0)
        return -1;
    return quantize_selected_impl(B, Hkv, D, L, W, n_kept, bits, G, key_axis, tail_cap, k, v, idx,
                                  k_codes, v_codes, k_scale, k_zero, v_scale, v_zero, tail_k,
                                  tail_v, tau, k_out, v_out, ovf_cap, k_ovf, v_ovf);
}

/*
 * Prefill-time compression of one layer, start to end: votes, pool, top-k
 * with k = min(budget, P), then quantize the survivors.  idx [B,Hkv,k] and,
 * when not NULL, pooled [B,Hkv,P] (the scores the selection was made on) are
 * returned for the tests.
 */
int orc_compress(int B, int Hq, int Hkv, int D, int L, int W, int pool, int budget, int bits,
                 int G, int key_axis, double sm_scale, int tail_cap, const uint16_t *q_obs,
                 const uint16_t *k, const uint16_t *v, int32_t *idx, double *pooled_out,
                 uint32_t *k_codes, uint32_t *v_codes, uint16_t *k_scale, uint16_t *k_zero,
                 uint16_t *v_scale, uint16_t *v_zero, uint16_t *tail_k, uint16_t *tail_v)
{
    if (W < 1 || W > L)
        return -1;
    const int P = L - W;
    const int n_kept = budget < P ? budget : P;
    const size_t heads = (size_t)B * Hkv;
    double *vote = (double *)malloc(sizeof(double) * heads * (size_t)(P > 0 ? P : 1));
    double *pooled = (double *)malloc(sizeof(double) * heads * (size_t)(P > 0 ? P : 1));
    if (!vote || !pooled) {
        free(vote);
        free(pooled);
        return -2;
    }
    int rc = orc_window_votes(B, Hq, Hkv, D, L, W, sm_scale, q_obs, k, vote);
    if (!rc)
        rc = orc_max_pool((int)heads, P, pool, vote, pooled);
    for (size_t h = 0; h < heads && !rc; ++h)
        rc = orc_topk(P, n_kept, pooled + h * P, idx + h * n_kept);
    if (!rc && pooled_out)
        memcpy(pooled_out, pooled, sizeof(double) * heads * (size_t)P);
    free(vote);
    free(pooled);
    if (rc)
        return rc;
    return orc_quantize_selected(B, Hkv, D, L, W, n_kept, bits, G, key_axis, tail_cap, k, v, idx,
                                 k_codes, v_codes, k_scale, k_zero, v_scale, v_zero, tail_k,
                                 tail_v);
}

/* ------------------------------------------------------------------ */
/* Decode (Section 3: G' = Q(G)*s + z, then Softmax(h_Q X_K'^T) X_V'    */
/* over the n_kept dequantized survivors followed by tail_len exact     */
/* binary16 rows; no mask, every cached token precedes the query).      */
/* ------------------------------------------------------------------ */

/* Dequantize one head into dense rows: Kd, Vd [n_kept + tail_len, D]. */
/* ko, vo: the head's outlier slots [n_kept, ORC_OUT_SLOTS], or NULL; kov, vov: its overflow
 * buffers for n_kept tokens and ovf_cap entries (with ko, vo). */
static void dequantize_head(int D, int n_kept, int bits, int G, int key_axis, int tail_len,
                            const uint32_t *kc, const uint32_t *vc, const uint16_t *ks,
                            const uint16_t *kz, const uint16_t *vs, const uint16_t *vz,
                            const uint16_t *tk, const uint16_t *tv, const uint32_t *ko,
                            const uint32_t *vo, int ovf_cap, const uint32_t *kov,
                            const uint32_t *vov, double *Kd, double *Vd)
{
    for (int t = 0; t < n_kept; ++t)
        for (int d = 0; d < D; ++d) {
            uint32_t ck = orc_k_code_get(kc, D, bits, t, d), cv = orc_v_code_get(vc, D, bits, t, d);
            if (bits == 16) {
                Kd[(size_t)t * D + d] = orc_half_to_double((uint16_t)ck);
                Vd[(size_t)t * D + d] = orc_half_to_double((uint16_t)cv);
            } else {
                size_t mk = key_axis == 0 ? (size_t)(t / G) * D + d : (size_t)t * (D / G) + d / G;
                size_t mv = (size_t)t * (D / G) + d / G;
                Kd[(size_t)t * D + d] =
                    (double)ck * orc_half_to_double(ks[mk]) + orc_half_to_double(kz[mk]);
                Vd[(size_t)t * D + d] =
                    (double)cv * orc_half_to_double(vs[mv]) + orc_half_to_double(vz[mv]);
            }
        }
    for (int t = 0; t < n_kept && ko && vo; ++t)
        for (int j = 0; j < ORC_OUT_SLOTS; ++j) {
            uint32_t a = ko[(size_t)t * ORC_OUT_SLOTS + j], c = vo[(size_t)t * ORC_OUT_SLOTS + j];
            if (a & 0x80u) {
                int d = (int)(a & 0x7Fu);
                size_t mk = key_axis == 0 ? (size_t)(t / G) * D + d : (size_t)t * (D / G) + d / G;
                Kd[(size_t)t * D + d] = orc_outlier_value(a, kz[mk]);
            }
            if (c & 0x80u) {
                int d = (int)(c & 0x7Fu);
                Vd[(size_t)t * D + d] = orc_outlier_value(c, vz[(size_t)t * (D / G) + d / G]);
            }
        }
    if (ko && vo && kov && vov) { /* the rows' further outliers */
        const size_t n_start = orc_ovf_words(n_kept, ovf_cap) - 2 * (size_t)ovf_cap;
        const uint32_t nk = kov[orc_rows(n_kept) / 32], nv = vov[orc_rows(n_kept) / 32];
        for (uint32_t e = 0; e < nk && e < (uint32_t)ovf_cap; ++e) {
            uint32_t a = kov[n_start + 2 * (size_t)e];
            int t = (int)kov[n_start + 2 * (size_t)e + 1], d = (int)(a & 0x7Fu);
            size_t mk = key_axis == 0 ? (size_t)(t / G) * D + d : (size_t)t * (D / G) + d / G;
            Kd[(size_t)t * D + d] = orc_outlier_value(a, kz[mk]);
        }
        for (uint32_t e = 0; e < nv && e < (uint32_t)ovf_cap; ++e) {
            uint32_t c = vov[n_start + 2 * (size_t)e];
            int t = (int)vov[n_start + 2 * (size_t)e + 1], d = (int)(c & 0x7Fu);
            Vd[(size_t)t * D + d] = orc_outlier_value(c, vz[(size_t)t * (D / G) + d / G]);
        }
    }
    for (int t = 0; t < tail_len; ++t)
        for (int d = 0; d < D; ++d) {
            Kd[(size_t)(n_kept + t) * D + d] = orc_half_to_double(tk[(size_t)t * D + d]);
            Vd[(size_t)(n_kept + t) * D + d] = orc_half_to_double(tv[(size_t)t * D + d]);
        }
}

/* q [B,Hq,D] half -> out [B,Hq,D] double.  Query head h reads KV head h/Gq. */
static int decode_attn_impl(int B, int Hq, int Hkv, int D, int n_kept, int bits, int G, int key_axis,
                            double sm_scale, int tail_len, int tail_cap, const uint16_t *q,
                            const uint32_t *k_codes, const uint32_t *v_codes,
                            const uint16_t *k_scale, const uint16_t *k_zero,
                            const uint16_t *v_scale, const uint16_t *v_zero, const uint16_t *tail_k,
                            const uint16_t *tail_v, const uint32_t *k_out, const uint32_t *v_out,
                            int ovf_cap, const uint32_t *k_ovf, const uint32_t *v_ovf, double *out)
{
    if (Hq % Hkv || tail_len > tail_cap || n_kept + tail_len < 1)
        return -1;
    const size_t ow = k_out ? orc_ovf_words(n_kept, ovf_cap) : 0;
    const int Gq = Hq / Hkv, T = n_kept + tail_len;
    const size_t kw = orc_k_words(n_kept, D, bits), vw = orc_v_words(n_kept, D, bits);
    const size_t rows = (size_t)orc_rows(n_kept);
    const size_t kmeta = bits == 16 ? 0
                         : key_axis == 0 ? (size_t)orc_key_groups(n_kept, G) * D
                                         : rows * (D / G);
    const size_t vmeta = bits == 16 ? 0 : rows * (D / G);
    int status = 0;
#pragma omp parallel for collapse(2) schedule(dynamic)
    for (int b = 0; b < B; ++b)
        for (int g = 0; g < Hkv; ++g) {
            const size_t head = (size_t)b * Hkv + g;
            double *Kd = (double *)malloc(sizeof(double) * (size_t)T * D);
            double *Vd = (double *)malloc(sizeof(double) * (size_t)T * D);
            double *a = (double *)malloc(sizeof(double) * (size_t)T);
            if (!Kd || !Vd || !a) {
                status = -2;
                free(Kd);
                free(Vd);
                free(a);
                continue;
            }
            dequantize_head(D, n_kept, bits, G, key_axis, tail_len, k_codes + head * kw,
                            v_codes + head * vw, k_scale + head * kmeta, k_zero + head * kmeta,
                            v_scale + head * vmeta, v_zero + head * vmeta,
                            tail_k + head * (size_t)tail_cap * D,
                            tail_v + head * (size_t)tail_cap * D,
                            k_out ? k_out + head * rows * ORC_OUT_SLOTS : NULL,
                            v_out ? v_out + head * rows * ORC_OUT_SLOTS : NULL, ovf_cap,
                            k_out ? k_ovf + head * ow : NULL, k_out ? v_ovf + head * ow : NULL, Kd, Vd);
            for (int h = g * Gq; h < (g + 1) * Gq; ++h) {
                const uint16_t *qr = q + ((size_t)b * Hq + h) * (size_t)D;
                double mx = -INFINITY;
                for (int t = 0; t < T; ++t) {
                    double s = 0.0;
                    for (int d = 0; d < D; ++d)
                        s += orc_half_to_double(qr[d]) * Kd[(size_t)t * D + d];
                    a[t] = sm_scale * s;
                    if (a[t] > mx)
                        mx = a[t];
                }
                double Z = 0.0;
                for (int t = 0; t < T; ++t) {
                    a[t] = exp(a[t] - mx);
                    Z += a[t];
                }
                double *o = out + ((size_t)b * Hq + h) * (size_t)D;
                for (int d = 0; d < D; ++d) {
                    double acc = 0.0;
                    for (int t = 0; t < T; ++t)
                        acc += a[t] * Vd[(size_t)t * D + d];
                    o[d] = acc / Z;
                }
            }
            free(Kd);
            free(Vd);
            free(a);
        }
    return status;
}

int orc_decode_attn(int B, int Hq, int Hkv, int D, int n_kept, int bits, int G, int key_axis,
                    double sm_scale, int tail_len, int tail_cap, const uint16_t *q,
                    const uint32_t *k_codes, const uint32_t *v_codes, const uint16_t *k_scale,
                    const uint16_t *k_zero, const uint16_t *v_scale, const uint16_t *v_zero,
                    const uint16_t *tail_k, const uint16_t *tail_v, double *out)
{
    return decode_attn_impl(B, Hq, Hkv, D, n_kept, bits, G, key_axis, sm_scale, tail_len, tail_cap,
                            q, k_codes, v_codes, k_scale, k_zero, v_scale, v_zero, tail_k, tail_v,
                            NULL, NULL, 0, NULL, NULL, out);
}

/* The same over a cache with outlier slots k_out, v_out [B,Hkv,n_kept,ORC_OUT_SLOTS] and overflow
 * buffers k_ovf, v_ovf [B,Hkv,orc_ovf_words(n_kept, ovf_cap)]. */
int orc_decode_attn_outliers(int B, int Hq, int Hkv, int D, int n_kept, int bits, int G,
                             int key_axis, double sm_scale, int tail_len, int tail_cap,
                             const uint16_t *q, const uint32_t *k_codes, const uint32_t *v_codes,
                             const uint16_t *k_scale, const uint16_t *k_zero,
                             const uint16_t *v_scale, const uint16_t *v_zero,
                             const uint16_t *tail_k, const uint16_t *tail_v, const uint32_t *k_out,
                             const uint32_t *v_out, int ovf_cap, const uint32_t *k_ovf,
                             const uint32_t *v_ovf, double *out)
{
    if (!k_out || !v_out || !k_ovf || !v_ovf || ovf_cap < 0)
        return -1;
    return decode_attn_impl(B, Hq, Hkv, D, n_kept, bits, G, key_axis, sm_scale, tail_len, tail_cap,
                            q, k_codes, v_codes, k_scale, k_zero, v_scale, v_zero, tail_k, tail_v,
                            k_out, v_out, ovf_cap, k_ovf, v_ovf, out);
}

/* Dense dequantized K', V' of one head, for tests of the error bound
 * (ko, vo: the head's outlier slots or NULL). */
int orc_dequantize_head(int D, int n_kept, int bits, int G, int key_axis, const uint32_t *kc,
                        const uint32_t *vc, const uint16_t *ks, const uint16_t *kz,
                        const uint16_t *vs, const uint16_t *vz, double *Kd, double *Vd)
{
    dequantize_head(D, n_kept, bits, G, key_axis, 0, kc, vc, ks, kz, vs, vz, NULL, NULL, NULL, NULL,
                    0, NULL, NULL, Kd, Vd);
    return 0;
}

int orc_dequantize_head_outliers(int D, int n_kept, int bits, int G, int key_axis,
                                 const uint32_t *kc, const uint32_t *vc, const uint16_t *ks,
                                 const uint16_t *kz, const uint16_t *vs, const uint16_t *vz,
                                 const uint32_t *ko, const uint32_t *vo, int ovf_cap,
                                 const uint32_t *kov, const uint32_t *vov, double *Kd, double *Vd)
{
    dequantize_head(D, n_kept, bits, G, key_axis, 0, kc, vc, ks, kz, vs, vz, NULL, NULL, ko, vo,
                    ovf_cap, kov, vov, Kd, Vd);
    return 0;
}

int orc_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/* Number of OpenMP threads the loops over (batch, KV head) may use from now on
 * (plumbing for the benchmark's single-thread timing; no arithmetic). */
void orc_set_threads(int n)
{
#ifdef _OPENMP
    if (n >= 1)
        omp_set_num_threads(n);
#else
    (void)n;
#endif
}
