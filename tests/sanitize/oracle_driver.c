/* Memory- and undefined-behaviour check of the CPU checker (oracle/kvqp_oracle.c): this program is
 * built together with that file under -fsanitize=address,undefined and walks its entry points over
 * small caches whose buffers have exactly the sizes the checker's own size functions state, so that
 * any access past them, any misaligned or overflowing arithmetic, stops the run.  Values are not
 * judged here (the pins do that) beyond a few sanity checks that keep the calls honest.
 * Test infrastructure only. */
#include <math.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

uint16_t orc_float_to_half(float f);
double orc_half_to_double(uint16_t h);
int orc_rows(int n_tok);
int orc_key_groups(int n_tok, int G);
size_t orc_k_words(int n_tok, int D, int bits);
size_t orc_v_words(int n_tok, int D, int bits);
size_t orc_ovf_words(int n_tok, int cap);
void orc_set_threads(int n);
int orc_compress(int B, int Hq, int Hkv, int D, int L, int W, int pool, int budget, int bits, int G, int key_axis,
                 double sm_scale, int tail_cap, const uint16_t *q_obs, const uint16_t *k, const uint16_t *v, int32_t *idx,
                 double *pooled_out, uint32_t *k_codes, uint32_t *v_codes, uint16_t *k_scale, uint16_t *k_zero,
                 uint16_t *v_scale, uint16_t *v_zero, uint16_t *tail_k, uint16_t *tail_v);
int orc_quantize_selected_outliers(int B, int Hkv, int D, int L, int W, int n_kept, int bits, int G, int key_axis,
                                   int tail_cap, double tau, const uint16_t *k, const uint16_t *v, const int32_t *idx,
                                   uint32_t *k_codes, uint32_t *v_codes, uint16_t *k_scale, uint16_t *k_zero,
                                   uint16_t *v_scale, uint16_t *v_zero, uint16_t *tail_k, uint16_t *tail_v,
                                   uint32_t *k_out, uint32_t *v_out, int ovf_cap, uint32_t *k_ovf, uint32_t *v_ovf);
int orc_decode_attn(int B, int Hq, int Hkv, int D, int n_kept, int bits, int G, int key_axis, double sm_scale,
                    int tail_len, int tail_cap, const uint16_t *q, const uint32_t *k_codes, const uint32_t *v_codes,
                    const uint16_t *k_scale, const uint16_t *k_zero, const uint16_t *v_scale, const uint16_t *v_zero,
                    const uint16_t *tail_k, const uint16_t *tail_v, double *out);
int orc_decode_attn_outliers(int B, int Hq, int Hkv, int D, int n_kept, int bits, int G, int key_axis, double sm_scale,
                             int tail_len, int tail_cap, const uint16_t *q, const uint32_t *k_codes,
                             const uint32_t *v_codes, const uint16_t *k_scale, const uint16_t *k_zero,
                             const uint16_t *v_scale, const uint16_t *v_zero, const uint16_t *tail_k,
                             const uint16_t *tail_v, const uint32_t *k_out, const uint32_t *v_out, int ovf_cap,
                             const uint32_t *k_ovf, const uint32_t *v_ovf, double *out);
int orc_dequantize_head_outliers(int D, int n_kept, int bits, int G, int key_axis, const uint32_t *kc, const uint32_t *vc,
                                 const uint16_t *ks, const uint16_t *kz, const uint16_t *vs, const uint16_t *vz,
                                 const uint32_t *ko, const uint32_t *vo, int ovf_cap, const uint32_t *kov,
                                 const uint32_t *vov, double *Kd, double *Vd);

static uint64_t rng = 0x9E3779B97F4A7C15ull;
static double uni(void)
{
    rng ^= rng << 13; rng ^= rng >> 7; rng ^= rng << 17;
    return (double)(rng >> 11) / 9007199254740992.0;
}
static double gauss(void) { return sqrt(-2.0 * log(uni() + 1e-300)) * cos(6.283185307179586 * uni()); }

/* exact-size heap blocks (never 0 bytes, so that every pointer is a real allocation) */
static void *blk(size_t n, size_t elem) { void *p = calloc(n ? n : 1, elem); if (!p) abort(); return p; }

static uint16_t *halves(size_t n, double spike_every, double spike)
{
    uint16_t *p = blk(n, sizeof *p);
    for (size_t i = 0; i < n; ++i) {
        double x = gauss();
        if (spike_every > 0 && uni() < 1.0 / spike_every) x *= spike;
        p[i] = orc_float_to_half((float)x);
    }
    return p;
}

static int fail(const char *what, int a, int b, int c, int d)
{
    fprintf(stderr, "oracle_driver: %s (bits %d G %d axis %d n %d)\n", what, a, b, c, d);
    return 1;
}

static int one_case(int B, int Hq, int Hkv, int L, int W, int pool, int budget, int bits, int G, int axis, double tau)
{
    const int D = 128, P = L - W, n = budget < P ? budget : P, tail_cap = W + 3, R = orc_rows(n);
    const int heads = B * Hkv, cap = 5 * n + 1;
    const double sm = 1.0 / sqrt((double)D);
    uint16_t *q_obs = halves((size_t)B * Hq * W * D, 0, 0), *k = halves((size_t)heads * L * D, 40, 9.0),
             *v = halves((size_t)heads * L * D, 60, 9.0), *q = halves((size_t)B * Hq * D, 0, 0);
    const size_t kw = orc_k_words(n, D, bits), vw = orc_v_words(n, D, bits);
    const size_t km = bits == 16 ? 0 : axis == 0 ? (size_t)orc_key_groups(n, G) * D : (size_t)R * (D / G);
    const size_t vm = bits == 16 ? 0 : (size_t)R * (D / G);
    int32_t *idx = blk((size_t)heads * n, sizeof *idx);
    double *pooled = blk((size_t)heads * P, sizeof *pooled);
    uint32_t *kc = blk(heads * kw, 4), *vc = blk(heads * vw, 4);
    uint16_t *ks = blk(heads * km, 2), *kz = blk(heads * km, 2), *vs = blk(heads * vm, 2), *vz = blk(heads * vm, 2);
    uint16_t *tk = blk((size_t)heads * tail_cap * D, 2), *tv = blk((size_t)heads * tail_cap * D, 2);
    double *out = blk((size_t)B * Hq * D, sizeof *out), *out2 = blk((size_t)B * Hq * D, sizeof *out2);
    int rc = orc_compress(B, Hq, Hkv, D, L, W, pool, budget, bits, G, axis, sm, tail_cap, q_obs, k, v, idx, pooled, kc, vc, ks,
                          kz, vs, vz, tk, tv);
    if (rc) return fail("compress returned an error", bits, G, axis, n);
    for (int h = 0; h < heads; ++h)
        for (int i = 0; i < n; ++i) {
            const int32_t a = idx[(size_t)h * n + i];
            if (a < 0 || a >= P || (i && a <= idx[(size_t)h * n + i - 1])) return fail("indices not ascending in range", bits, G, axis, n);
        }
    rc = orc_decode_attn(B, Hq, Hkv, D, n, bits, G, axis, sm, W, tail_cap, q, kc, vc, ks, kz, vs, vz, tk, tv, out);
    if (rc) return fail("decode returned an error", bits, G, axis, n);
    for (size_t i = 0; i < (size_t)B * Hq * D; ++i)
        if (!isfinite(out[i])) return fail("decode output not finite", bits, G, axis, n);
    if (bits != 16 && tau > 0) {
        uint32_t *ko = blk((size_t)heads * R * 4, 4), *vo = blk((size_t)heads * R * 4, 4);
        const size_t ow = orc_ovf_words(n, cap);
        uint32_t *kov = blk(heads * ow, 4), *vov = blk(heads * ow, 4);
        rc = orc_quantize_selected_outliers(B, Hkv, D, L, W, n, bits, G, axis, tail_cap, tau, k, v, idx, kc, vc, ks, kz, vs, vz,
                                            tk, tv, ko, vo, cap, kov, vov);
        if (rc) return fail("quantize with outliers returned an error", bits, G, axis, n);
        rc = orc_decode_attn_outliers(B, Hq, Hkv, D, n, bits, G, axis, sm, W, tail_cap, q, kc, vc, ks, kz, vs, vz, tk, tv, ko,
                                      vo, cap, kov, vov, out2);
        if (rc) return fail("decode with outliers returned an error", bits, G, axis, n);
        double *Kd = blk((size_t)(n ? n : 1) * D, sizeof *Kd), *Vd = blk((size_t)(n ? n : 1) * D, sizeof *Vd);
        rc = orc_dequantize_head_outliers(D, n, bits, G, axis, kc, vc, ks, kz, vs, vz, ko, vo, cap, kov, vov, Kd, Vd);
        if (rc) return fail("dequantize returned an error", bits, G, axis, n);
        for (size_t i = 0; i < (size_t)n * D; ++i)
            if (!isfinite(Kd[i]) || !isfinite(Vd[i])) return fail("dequantized value not finite", bits, G, axis, n);
        /* a list with room for a single entry: the writer must stop at the capacity */
        const size_t ow1 = orc_ovf_words(n, 1);
        uint32_t *kov1 = blk(heads * ow1, 4), *vov1 = blk(heads * ow1, 4);
        rc = orc_quantize_selected_outliers(B, Hkv, D, L, W, n, bits, G, axis, tail_cap, tau, k, v, idx, kc, vc, ks, kz, vs, vz,
                                            tk, tv, ko, vo, 1, kov1, vov1);
        if (rc) return fail("quantize with a one-entry list returned an error", bits, G, axis, n);
        rc = orc_decode_attn_outliers(B, Hq, Hkv, D, n, bits, G, axis, sm, W, tail_cap, q, kc, vc, ks, kz, vs, vz, tk, tv, ko,
                                      vo, 1, kov1, vov1, out2);
        if (rc) return fail("decode with a one-entry list returned an error", bits, G, axis, n);
        free(ko); free(vo); free(kov); free(vov); free(kov1); free(vov1); free(Kd); free(Vd);
    }
    free(q_obs); free(k); free(v); free(q); free(idx); free(pooled); free(kc); free(vc); free(ks); free(kz); free(vs);
    free(vz); free(tk); free(tv); free(out); free(out2);
    return 0;
}

int main(void)
{
    static const int bits_of[] = {2, 4, 8, 16}, groups[] = {32, 64, 128};
    /* budgets: whole blocks, a ragged count, one token, more than the prefix holds */
    static const int budgets[] = {64, 37, 1, 160, 1000};
    int n_cases = 0;
    orc_set_threads(2);
    for (int bi = 0; bi < 4; ++bi)
        for (int gi = 0; gi < 3; ++gi)
            for (int axis = 0; axis < 2; ++axis)
                for (int ni = 0; ni < 5; ++ni) {
                    const int bits = bits_of[bi], G = groups[gi];
                    if (bits == 16 && (gi || axis)) continue;
                    const int L = 200 + 13 * ni, W = 1 + 7 * ni, pool = 1 + 2 * (ni % 4);
                    const int Hkv = 1 + (ni & 1), Hq = Hkv * (1 << (gi % 3));
                    if (one_case(1 + (ni == 2), Hq, Hkv, L, W, pool, budgets[ni], bits, G, axis, ni % 2 ? 0.0 : 2.5)) return 1;
                    ++n_cases;
                }
    printf("oracle_driver: %d cases clean\n", n_cases);
    return 0;
}
