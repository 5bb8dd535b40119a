/*
 * xq_oracle.c -- CPU oracle for the XQuant quantized-KV decode path.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is a plain, slow, step-by-step CPU
 * statement of what the path computes.  It is called only from tests/, from
 * __graft_entry__.smoke() and from bench.py's cpu_baseline leg.  The product
 * (the HIP library) never links, loads or imports anything in this folder, and
 * this file includes nothing from the product.
 *
 * What each function follows (XQuant paper, arXiv 2510.11236):
 *   xqo_quantize_group  Sec. 3.1 Eq. 1-2 (asymmetric min/max B-bit quantization,
 *                       round to nearest) + Sec. 3.2 Eq. 12 (data-free
 *                       calibration of zero-point and scale; the codes are
 *                       computed with the uncalibrated z, s).
 *   xqo_quantize_k/_v   Sec. 4.1 "Baselines and Implementations": keys grouped
 *                       per channel, values per token, group size g, the most
 *                       recent tokens kept in fp16 (residual length R).
 *                       store_codes = 0 is Appendix Alg. 2 "PseudoQuantize":
 *                       the subordinate layer of a pair (Sec. 3.3.4) computes
 *                       only its calibrated scale and zero-point.
 *   xqo_dequant_k/_v    Sec. 3.2 / 3.3.3 dequantization X^ = X_Q * s^ + z^.
 *   xqo_attention       softmax(sigma q K^T) V over the dequantized cache plus
 *                       the fp16 residual rows (the textbook definition; the
 *                       paper dequantizes and then calls ordinary attention).
 *   xqo_prefill_attention_row  causal attention of the prompt on its fp16 K/V (the
 *                       paper is silent on it: textbook definition).
 *   xqo_pack_k/_v_words bit layout of the packed code words.  The layout is
 *                       this build's, not the paper's: parity unpinned by the
 *                       paper; it is pinned by the written specification in
 *                       include/xq.h and by an unpack round trip.
 *   xqo_equivalent_bits Appendix C worked example (codes only).
 *
 * Readings taken where the paper is silent or inconsistent:
 *   - ties round half to even in fp32 (agrees with Eq. 4: 0.5 -> 0);
 *   - a constant group (max == min) has s = 0, codes 0, s^ = 0, z^ = min;
 *   - calibrated zero-point follows Eq. 12 (z + eta*s*(2^B-1)), not the
 *     Appendix Alg. 2 "Calibrate" listing, which drops the (2^B-1) factor;
 *   - scale arithmetic is fp32 in the order written below, metadata is stored
 *     as fp16 (round to nearest even);
 *   - T_q = g * ceil(max(T - R, 0) / g) tokens are quantized, the rest
 *     (the newest r tokens, R - g < r <= R once T >= R) stay fp16.
 *
 * Build: gcc -O2 -ffp-contract=off -fno-fast-math -fPIC -shared (see build.py).
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

/* ---------------------------------------------------------------- fp16 <-> fp32
 * IEEE binary16, written out from the format definition (1 sign, 5 exponent,
 * 10 fraction bits, bias 15, gradual underflow).  Pinned against numpy.float16
 * in the tests. */
float xqo_half_to_float(uint16_t h) {
    int sign = (h >> 15) & 1;
    int e = (h >> 10) & 0x1f;
    int f = h & 0x3ff;
    double v;
    if (e == 0) v = ldexp((double)f, -24);            /* zero / subnormal */
    else if (e == 31) v = f ? NAN : INFINITY;
    else v = ldexp((double)(1024 + f), e - 25);
    return (float)(sign ? -v : v);
}

uint16_t xqo_float_to_half(float x) {
    uint16_t sign = signbit(x) ? 0x8000u : 0u;
    double a = fabs((double)x);
    if (isnan(x)) return (uint16_t)(sign | 0x7e00u);
    if (isinf(x)) return (uint16_t)(sign | 0x7c00u);
    if (a == 0.0) return sign;
    int e;
    (void)frexp(a, &e);          /* a = m * 2^e, m in [0.5, 1)  -> leading bit 2^(e-1) */
    int lead = e - 1;
    if (lead < -14) lead = -14;  /* subnormal range: fixed quantum 2^-24 */
    double quantum = ldexp(1.0, lead - 10);
    double r = rint(a / quantum);            /* exact quotient; ties to even */
    double v = r * quantum;
    if (v >= 65536.0) return (uint16_t)(sign | 0x7c00u);
    if (v < ldexp(1.0, -14)) return (uint16_t)(sign | (uint16_t)r);   /* r <= 1023 */
    (void)frexp(v, &e);
    lead = e - 1;
    int frac = (int)(v / ldexp(1.0, lead - 10)) - 1024;
    return (uint16_t)(sign | ((lead + 15) << 10) | frac);
}

/* ------------------------------------------------------------------ split rule */
int xqo_quantized_len(int T, int g, int R) {
    int over = T - R;
    if (over <= 0) return 0;
    return g * ((over + g - 1) / g);
}

/* ------------------------------------------------------- one group (Eq. 1, 2, 12)
 * x[i*stride], i < g are the fp16 values of the group.  B in {1,2}.
 * codes (may be NULL) receives one byte per element at codes[i*cstride].
 * s_hat / z_hat receive the calibrated scale and zero-point as fp16 bits. */
void xqo_quantize_group(const uint16_t *x, long stride, int g, int B, float eta,
                        uint8_t *codes, long cstride, uint16_t *s_hat, uint16_t *z_hat) {
    float mn = xqo_half_to_float(x[0]), mx = mn;
    for (int i = 1; i < g; ++i) {
        float v = xqo_half_to_float(x[i * stride]);
        if (v < mn) mn = v;
        if (v > mx) mx = v;
    }
    /* the sign of a zero minimum / maximum is not the paper's concern: taken as +0, so
     * that the stored zero-point does not depend on the order of -0 and +0 in the group */
    mn = mn + 0.0f;
    mx = mx + 0.0f;
    int n = (1 << B) - 1;
    volatile float range = mx - mn;                         /* Eq. 1 */
    volatile float s = (mx == mn) ? 0.0f : range / (float)n;
    if (codes) {
        for (int i = 0; i < g; ++i) {
            int c = 0;
            if (s != 0.0f) {
                volatile float d = xqo_half_to_float(x[i * stride]) - mn;   /* Eq. 2 */
                volatile float t = d / s;
                float r = rintf(t);                         /* nearest, ties to even */
                if (r < 0.0f) r = 0.0f;
                if (r > (float)n) r = (float)n;
                c = (int)r;
            }
            codes[i * cstride] = (uint8_t)c;
        }
    }
    /* Eq. 12: z^ = z + eta*s*(2^B-1),  s^ = (1-2eta)*s ; fp32, one rounding per op */
    volatile float c1 = eta * (float)n;
    volatile float two_eta = 2.0f * eta;
    volatile float c2 = 1.0f - two_eta;
    volatile float shift = c1 * s;
    volatile float zc = mn + shift;
    volatile float sc = c2 * s;
    *z_hat = xqo_float_to_half(zc);
    *s_hat = xqo_float_to_half(sc);
}

/* ----------------------------------------------------- keys: groups along tokens
 * k: [T][D] fp16.  Quantizes tokens [0, T_q).  Group (G, d) = tokens
 * [G*g, (G+1)*g) of channel d.  codes: [T_q][D] bytes or NULL (store_codes=0),
 * scale/zero: [T_q/g][D] fp16 bits.  Returns T_q. */
int xqo_quantize_k(const uint16_t *k, int T, int D, int g, int R, int B, float eta,
                   int store_codes, uint8_t *codes, uint16_t *scale, uint16_t *zero) {
    int Tq = xqo_quantized_len(T, g, R);
    for (int G = 0; G < Tq / g; ++G)
        for (int d = 0; d < D; ++d)
            xqo_quantize_group(k + (long)G * g * D + d, D, g, B, eta,
                               store_codes ? codes + (long)G * g * D + d : NULL, D,
                               scale + (long)G * D + d, zero + (long)G * D + d);
    return Tq;
}

/* -------------------------------------------------- values: groups along channels
 * v: [T][D] fp16.  Group (t, j) = channels [j*g, (j+1)*g) of token t.
 * codes: [T_q][D] bytes or NULL, scale/zero: [T_q][D/g]. */
int xqo_quantize_v(const uint16_t *v, int T, int D, int g, int R, int B, float eta,
                   int store_codes, uint8_t *codes, uint16_t *scale, uint16_t *zero) {
    int Tq = xqo_quantized_len(T, g, R);
    int J = D / g;
    for (int t = 0; t < Tq; ++t)
        for (int j = 0; j < J; ++j)
            xqo_quantize_group(v + (long)t * D + j * g, 1, g, B, eta,
                               store_codes ? codes + (long)t * D + j * g : NULL, 1,
                               scale + (long)t * J + j, zero + (long)t * J + j);
    return Tq;
}

/* --------------------------------------------------------------- dequantization
 * X^ = X_Q * s^ + z^ in double from the stored fp16 metadata. out: [T_q][D]. */
void xqo_dequant_k(const uint8_t *codes, const uint16_t *scale, const uint16_t *zero,
                   int Tq, int D, int g, double *out) {
    for (int t = 0; t < Tq; ++t)
        for (int d = 0; d < D; ++d) {
            long m = (long)(t / g) * D + d;
            out[(long)t * D + d] = (double)codes[(long)t * D + d] * (double)xqo_half_to_float(scale[m])
                                 + (double)xqo_half_to_float(zero[m]);
        }
}

void xqo_dequant_v(const uint8_t *codes, const uint16_t *scale, const uint16_t *zero,
                   int Tq, int D, int g, double *out) {
    int J = D / g;
    for (int t = 0; t < Tq; ++t)
        for (int d = 0; d < D; ++d) {
            long m = (long)t * J + d / g;
            out[(long)t * D + d] = (double)codes[(long)t * D + d] * (double)xqo_half_to_float(scale[m])
                                 + (double)xqo_half_to_float(zero[m]);
        }
}

/* fp16 rows -> double (the residual window is used as it is) */
void xqo_half_rows_to_double(const uint16_t *x, long n, double *out) {
    for (long i = 0; i < n; ++i) out[i] = (double)xqo_half_to_float(x[i]);
}

/* ------------------------------------------------------------------- attention
 * One query (fp16, [D]) against T rows of K^ and V^ (double, [T][D]):
 * u_t = sigma * <q, K^_t>,  p = softmax(u),  o = sum_t p_t V^_t.  out: fp32 [D]. */
void xqo_attention(const uint16_t *q, const double *Kh, const double *Vh, int T, int D,
                   double sigma, float *out) {
    double *u = (double *)malloc(sizeof(double) * (size_t)(T > 0 ? T : 1));
    double m = -INFINITY;
    for (int t = 0; t < T; ++t) {
        double acc = 0.0;
        for (int d = 0; d < D; ++d) acc += (double)xqo_half_to_float(q[d]) * Kh[(long)t * D + d];
        u[t] = sigma * acc;
        if (u[t] > m) m = u[t];
    }
    double denom = 0.0;
    for (int t = 0; t < T; ++t) { u[t] = exp(u[t] - m); denom += u[t]; }
    for (int d = 0; d < D; ++d) {
        double acc = 0.0;
        for (int t = 0; t < T; ++t) acc += u[t] * Vh[(long)t * D + d];
        out[d] = (float)(acc / denom);
    }
    free(u);
}

/* ------------------------------------------------------- prefill (causal) attention
 * The paper's procedure quantizes the prompt's K/V (Appendix Alg. 1, first loop) and reads the
 * quantized cache from the first decode step on (second loop); the attention of the prompt itself
 * is not described, so it is taken to be the ordinary causal attention of the model on the fp16
 * K/V it has just computed: query t attends to keys 0..t,
 *   o_t = softmax(sigma q_t K_{0..t}^T) V_{0..t}.
 * One query row per call (q: fp16 [D]; K, V: fp16 [T][D] with T > t); out: fp32 [D]. */
void xqo_prefill_attention_row(const uint16_t *q, const uint16_t *K, const uint16_t *V, int t, int D,
                               double sigma, float *out) {
    int n = t + 1;
    double *u = (double *)malloc(sizeof(double) * (size_t)n);
    double m = -INFINITY;
    for (int j = 0; j < n; ++j) {
        double acc = 0.0;
        for (int d = 0; d < D; ++d)
            acc += (double)xqo_half_to_float(q[d]) * (double)xqo_half_to_float(K[(long)j * D + d]);
        u[j] = sigma * acc;
        if (u[j] > m) m = u[j];
    }
    double denom = 0.0;
    for (int j = 0; j < n; ++j) { u[j] = exp(u[j] - m); denom += u[j]; }
    for (int d = 0; d < D; ++d) {
        double acc = 0.0;
        for (int j = 0; j < n; ++j) acc += u[j] * (double)xqo_half_to_float(V[(long)j * D + d]);
        out[d] = (float)(acc / denom);
    }
    free(u);
}

/* ------------------------------------------------------------ packed word layout
 * Written from the layout specification in include/xq.h ("Packed layout").
 * Keys: tokens in blocks of 32.  A token's code row is W = D*B/32 words; element d
 * sits in row word d/(32/B) at bit B*(d mod (32/B)).  A block stores its rows in
 * chunks of CW = min(4, W) words: [chunk][token in block][CW words]. */
void xqo_pack_k_words(const uint8_t *codes, int Tq, int D, int B, uint32_t *words) {
    int per = 32 / B, W = D / per, CW = W < 4 ? W : 4;
    memset(words, 0, sizeof(uint32_t) * (size_t)(Tq / 32) * 32 * W);
    for (int t = 0; t < Tq; ++t)
        for (int d = 0; d < D; ++d) {
            int wi = d / per, bit = B * (d % per);
            long addr = (long)(t / 32) * 32 * W + (long)(wi / CW) * 32 * CW + (long)(t % 32) * CW + wi % CW;
            words[addr] |= (uint32_t)codes[(long)t * D + d] << bit;
        }
}

/* Values: tokens in blocks of 32.  Channel d belongs to slot d / CPL (CPL = D/64
 * channels per slot).  A slot holds, per block, the 32*CPL codes ordered
 * e = (token in block)*CPL + (d mod CPL), packed B bits each, LSB first, into
 * WS = CPL*B words.  A block is [slot 0..63][WS words]. */
void xqo_pack_v_words(const uint8_t *codes, int Tq, int D, int B, uint32_t *words) {
    int CPL = D / 64, WS = CPL * B;
    memset(words, 0, sizeof(uint32_t) * (size_t)(Tq / 32) * 64 * WS);
    for (int t = 0; t < Tq; ++t)
        for (int d = 0; d < D; ++d) {
            int slot = d / CPL, e = (t % 32) * CPL + d % CPL;
            long addr = (long)(t / 32) * 64 * WS + (long)slot * WS + (e * B) / 32;
            words[addr] |= (uint32_t)codes[(long)t * D + d] << ((e * B) % 32);
        }
}

/* ------------------------------------------------ merged codes of a pair (Appendix E)
 * e0, e1: the two layers' own B-bit codes at the same positions (e0 = first layer, weight
 * gamma0).  mode 1: e_m = round-to-nearest(gamma0 e0 + (1 - gamma0) e1), computed as
 * floor(x + 1/2) (the paper leaves the boundary values of gamma0, where x is an exact half,
 * out of its six intervals).  mode 2 / 3: gamma0 = 1/2 with floor / ceil (the "Flooring" and
 * "Ceiling" rows of the ablation table).  mode 0: e_m = e0 (Sec. 3.3.4). */
void xqo_merge_codes(const uint8_t *e0, const uint8_t *e1, long count, int B, int mode, float gamma0,
                     uint8_t *out) {
    int n = (1 << B) - 1;
    for (long i = 0; i < count; ++i) {
        double x;
        if (mode == 1) x = floor((double)gamma0 * e0[i] + (1.0 - (double)gamma0) * e1[i] + 0.5);
        else if (mode == 2) x = floor(0.5 * e0[i] + 0.5 * e1[i]);
        else if (mode == 3) x = ceil(0.5 * e0[i] + 0.5 * e1[i]);
        else x = e0[i];
        int em = (int)x;
        if (em < 0) em = 0;
        if (em > n) em = n;
        out[i] = (uint8_t)em;
    }
}

/* --------------------------------------------------- equivalent bit-width (App. C)
 * Codes only (metadata and the fp16 window are excluded, as the appendix says):
 * a layer below q holds 2-bit codes, else 1-bit; a layer stores codes iff it is
 * below m or is the first (even) layer of its pair.  Stored code bits per element,
 * averaged over all L layers; then the mean of keys and values. */
double xqo_equivalent_bits_one(int L, int q, int m) {
    double bits = 0.0;
    for (int l = 0; l < L; ++l)
        if (l < m || l % 2 == 0) bits += (l < q) ? 2.0 : 1.0;
    return bits / L;
}

double xqo_equivalent_bits(int L, int kq, int vq, int km, int vm) {
    return 0.5 * (xqo_equivalent_bits_one(L, kq, km) + xqo_equivalent_bits_one(L, vq, vm));
}
