/*
 * tkv_oracle.c -- CPU oracle for the TriAxialKV decode/append hot path.
 *
 * THIS IS TEST INFRASTRUCTURE, NOT PRODUCT CODE.  It is a plain, slow, scalar
 * implementation used only by the tests, the smoke check and the CPU-baseline
 * leg of the benchmark.  It shares no code, header, table or helper with the
 * HIP library, and nothing in the product path may call it.
 *
 * What it implements (paper passages):
 *   - asymmetric groupwise min/max quantisation with group size G = 32, one
 *     (scale, zero-point) pair per group of channels of one token and head
 *     (Sec. 3.2.1, "Bitwidths and quantization axes"; the per-token axis is
 *     used for keys and values at both widths);
 *   - the paper's own scheme for INT2 keys (Sec. 3.2.1): per-channel groups, the
 *     32 tokens of a block sharing one (scale, zero-point) pair per channel; the
 *     residual policy (tokens that do not fill a block go to INT4) is the few
 *     lines of route_residual in tkv_oracle.py;
 *   - sub-byte packing of the codes plus scales and zero-points into paged
 *     UINT8 buffers, one pool per bitwidth in a shared index space split by
 *     an offset (Sec. 3.2.1 "Buffer layout", Sec. 3.2.2 "Shared address
 *     space"); the byte order inside a page follows this build's own layout
 *     specification, re-implemented here from its formulas;
 *   - the prefill gather (Sec. 3.2.3 "Prefill"): the cached rows of a matched
 *     prefix dequantised into FP16, value = binary16 nearest-even rounding of
 *     the exact code * scale + zero (one rounding);
 *   - decode attention softmax(q K^T / sqrt(d)) V over the dequantised cache
 *     (Sec. 3.2.3 "Decode"): the flash-decoding splits and the log-sum-exp
 *     merge reach exactly this value, so the oracle is the plain definition,
 *     unsplit, in fp64, tokens in their original order.
 *
 * Readings where the paper is silent (each listed in the design notes):
 * scale and zero are fp16; zero-point is the group minimum; codes are
 * round-half-even of (x - zero) * (1/scale) against the STORED fp16 values;
 * fp32 arithmetic without fused multiply-add; a zero scale gives all-zero
 * codes.
 *
 * Parity pins live in tests/test_oracle_*.py: conversions against numpy /
 * torch casts, hand-worked groups, nearest-code brute force, the scale/2
 * round-trip bound, exactly-representable inputs against unquantised fp64
 * attention, brute force on tiny heads, closed forms, codec bijectivity and
 * hand-derived bit positions; the FP16 dequantisation against numpy's
 * float64 -> float16 cast and exact rational arithmetic; the per-channel keys
 * against a hand-worked block, numpy reductions over the token axis, exact
 * nearest-code search and the per-token path on the transposed block
 * (tests/test_oracle_kchannel.py).  No function here
 * is "parity unpinned".
 *
 * Build: gcc -O2 -std=c11 -ffp-contract=off -fopenmp -shared -fPIC
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

/* ------------------------------------------------------------------ */
/* number formats: hand-written bit code, pinned against numpy/torch   */
/* ------------------------------------------------------------------ */

static inline float bits_to_f32(uint32_t u) { float f; memcpy(&f, &u, 4); return f; }
static inline uint32_t f32_to_bits(float f) { uint32_t u; memcpy(&u, &f, 4); return u; }

/* bf16 is the upper half of an IEEE binary32: widening is exact. */
float tkvo_bf16_to_f32(uint16_t h) { return bits_to_f32((uint32_t)h << 16); }

/* IEEE binary16 -> binary32, exact (subnormals, infinities, NaN kept). */
float tkvo_f16_to_f32(uint16_t h)
{
    uint32_t sign = (uint32_t)(h & 0x8000u) << 16;
    uint32_t ex = (h >> 10) & 0x1fu;
    uint32_t man = h & 0x3ffu;
    if (ex == 0) {
        if (man == 0) return bits_to_f32(sign);
        /* subnormal: man * 2^-24 */
        float v = (float)man * 5.9604644775390625e-8f; /* 2^-24, exact product */
        return sign ? -v : v;
    }
    if (ex == 31) return bits_to_f32(sign | 0x7f800000u | (man << 13));
    return bits_to_f32(sign | ((ex + 112u) << 23) | (man << 13));
}

/* binary32 -> binary16, round to nearest, ties to even; overflow -> inf,
 * results below the smallest subnormal round to zero or to that subnormal. */
uint16_t tkvo_f32_to_f16(float f)
{
    uint32_t u = f32_to_bits(f);
    uint16_t sign = (uint16_t)((u >> 16) & 0x8000u);
    uint32_t ex = (u >> 23) & 0xffu;
    uint32_t man = u & 0x7fffffu;
    if (ex == 255) return (uint16_t)(sign | 0x7c00u | (man ? (0x200u | (man >> 13)) : 0u));
    int e = (int)ex - 127;              /* unbiased exponent of the input   */
    if (e > 15) return (uint16_t)(sign | 0x7c00u);
    if (e >= -14) {                     /* normal range of binary16          */
        uint32_t keep = man >> 13, rest = man & 0x1fffu;
        uint32_t h = ((uint32_t)(e + 15) << 10) | keep;
        if (rest > 0x1000u || (rest == 0x1000u && (keep & 1u))) h += 1u; /* may carry into exponent / inf */
        return (uint16_t)(sign | h);
    }
    if (e < -25) return sign;           /* below half of the smallest subnormal */
    /* subnormal result: value = m * 2^-24 with m = round(full * 2^(e+24-23)) */
    uint32_t full = man | 0x800000u;    /* 24-bit significand, value full * 2^(e-23) */
    int shift = -e - 1;                 /* 14..24: m = full >> shift, rounded        */
    uint32_t keep = full >> shift;
    uint32_t rest = full & ((1u << shift) - 1u);
    uint32_t half = 1u << (shift - 1);
    if (rest > half || (rest == half && (keep & 1u))) keep += 1u;
    return (uint16_t)(sign | keep);
}

/* binary64 -> binary16, round to nearest even, ONE rounding (no detour through binary32). */
uint16_t tkvo_f64_to_f16(double d)
{
    uint64_t u;
    memcpy(&u, &d, sizeof u);
    uint16_t sign = (uint16_t)((u >> 48) & 0x8000u);
    uint32_t ex = (uint32_t)((u >> 52) & 0x7ffu);
    uint64_t man = u & 0xfffffffffffffull;
    if (ex == 2047) return (uint16_t)(sign | 0x7c00u | (man ? 0x200u : 0u));
    if (ex == 0) return sign;           /* zero or a binary64 subnormal: far below 2^-25 */
    int e = (int)ex - 1023;
    if (e > 15) return (uint16_t)(sign | 0x7c00u);
    if (e >= -14) {
        uint32_t keep = (uint32_t)(man >> 42);
        uint64_t rest = man & ((1ull << 42) - 1ull), half = 1ull << 41;
        uint32_t h = ((uint32_t)(e + 15) << 10) | keep;
        if (rest > half || (rest == half && (keep & 1u))) h += 1u;   /* may carry into the exponent / to inf */
        return (uint16_t)(sign | h);
    }
    if (e < -25) return sign;
    uint64_t full = man | (1ull << 52);  /* value full * 2^(e-52) = m * 2^-24 with m = full * 2^(e-28) */
    int shift = 28 - e;                  /* 42..53 */
    uint64_t keep = full >> shift;
    uint64_t rest = full & ((1ull << shift) - 1ull), half = 1ull << (shift - 1);
    if (rest > half || (rest == half && (keep & 1ull))) keep += 1ull;
    return (uint16_t)(sign | (uint16_t)keep);
}
void tkvo_f64_to_f16_array(const double *in, uint16_t *out, int64_t n)
{ for (int64_t i = 0; i < n; ++i) out[i] = tkvo_f64_to_f16(in[i]); }

void tkvo_bf16_to_f32_array(const uint16_t *in, float *out, int64_t n)
{ for (int64_t i = 0; i < n; ++i) out[i] = tkvo_bf16_to_f32(in[i]); }
void tkvo_f16_to_f32_array(const uint16_t *in, float *out, int64_t n)
{ for (int64_t i = 0; i < n; ++i) out[i] = tkvo_f16_to_f32(in[i]); }
void tkvo_f32_to_f16_array(const float *in, uint16_t *out, int64_t n)
{ for (int64_t i = 0; i < n; ++i) out[i] = tkvo_f32_to_f16(in[i]); }

/* ------------------------------------------------------------------ */
/* quantiser (Sec. 3.2.1): one group of G channels of one token/head   */
/* ------------------------------------------------------------------ */

/* The volatile stores keep every intermediate in binary32 and stop the
 * compiler from fusing or re-associating; -ffp-contract=off does the same. */
void tkvo_quantize_group(const uint16_t *x, int G, int bits,
                         uint8_t *codes, uint16_t *scale_h, uint16_t *zero_h)
{
    const int L = (1 << bits) - 1;
    float mn = tkvo_bf16_to_f32(x[0]), mx = mn;
    for (int i = 1; i < G; ++i) {
        float f = tkvo_bf16_to_f32(x[i]);
        if (f < mn) mn = f;
        if (f > mx) mx = f;
    }
    if (mn == 0.0f) mn = 0.0f;          /* -0 -> +0, so the stored zero-point has one spelling */
    volatile float r = mx - mn;
    volatile float s32 = r / (float)L;
    *scale_h = tkvo_f32_to_f16(s32);
    *zero_h = tkvo_f32_to_f16(mn);
    const float s = tkvo_f16_to_f32(*scale_h);
    const float z = tkvo_f16_to_f32(*zero_h);
    if (s == 0.0f) { memset(codes, 0, (size_t)G); return; }
    volatile float inv = 1.0f / s;
    for (int i = 0; i < G; ++i) {
        volatile float d = tkvo_bf16_to_f32(x[i]) - z;
        volatile float t = d * inv;
        float c = rintf(t);             /* default rounding mode: ties to even */
        if (c < 0.0f) c = 0.0f;
        if (c > (float)L) c = (float)L;
        codes[i] = (uint8_t)(int)c;
    }
}

/* x: bf16 [T, H, D]; bits: u8 [T] (2 or 4 per token, from the token's tag,
 * Sec. 3.2.3 "Tagging").  Outputs are the canonical per-token arrays:
 * codes u8 [T,H,D], scale/zero fp16 bit patterns [T,H,D/G].
 * Returns 0, or -1 on a bad bitwidth / shape. */
int tkvo_quantize(const uint16_t *x, int64_t T, int H, int D, int G, const uint8_t *bits,
                  uint8_t *codes, uint16_t *scale, uint16_t *zero)
{
    if (G <= 0 || D % G) return -1;
    for (int64_t t = 0; t < T; ++t) if (bits[t] != 2 && bits[t] != 4) return -1;
    const int NG = D / G;
#pragma omp parallel for schedule(static)
    for (int64_t t = 0; t < T; ++t)
        for (int h = 0; h < H; ++h)
            for (int g = 0; g < NG; ++g) {
                int64_t e = (t * H + h) * (int64_t)D + (int64_t)g * G;
                int64_t m = (t * H + h) * (int64_t)NG + g;
                tkvo_quantize_group(x + e, G, bits[t], codes + e, scale + m, zero + m);
            }
    return 0;
}

/* Per-channel key quantisation (Sec. 3.2.1, quantisation axes of the INT2 keys): the G tokens of a
 * block share one (scale, zero-point) pair FOR EACH CHANNEL, i.e. the quantisation group is the column of G
 * token values of one channel and head; the arithmetic of a group is the one above.
 * x: bf16 [T, H, D]; tok: i64 [nb, G], the token rows of each block in slot order.
 * codes: u8 [T, H, D], only the rows named by tok are written; bscale, bzero: fp16 bit patterns [nb, H, D].
 * Returns 0, -1 on a bad argument (bitwidth, G > 64, a row outside [0, T)). */
int tkvo_quantize_k_channel(const uint16_t *x, int64_t T, int H, int D, int G, int bits,
                            const int64_t *tok, int64_t nb,
                            uint8_t *codes, uint16_t *bscale, uint16_t *bzero)
{
    if ((bits != 2 && bits != 4) || G <= 0 || G > 64) return -1;
    for (int64_t i = 0; i < nb * G; ++i) if (tok[i] < 0 || tok[i] >= T) return -1;
#pragma omp parallel for schedule(static)
    for (int64_t b = 0; b < nb; ++b)
        for (int h = 0; h < H; ++h)
            for (int c = 0; c < D; ++c) {
                uint16_t col[64];
                uint8_t cc[64];
                for (int i = 0; i < G; ++i) col[i] = x[(tok[b * G + i] * H + h) * (int64_t)D + c];
                int64_t m = (b * H + h) * (int64_t)D + c;
                tkvo_quantize_group(col, G, bits, cc, bscale + m, bzero + m);
                for (int i = 0; i < G; ++i) codes[(tok[b * G + i] * H + h) * (int64_t)D + c] = cc[i];
            }
    return 0;
}

/* x_hat = code * scale + zero, evaluated in fp64 (exact: 4-bit x 11-bit
 * product plus an 11-bit addend fits a double with room to spare). */
void tkvo_dequantize(const uint8_t *codes, const uint16_t *scale, const uint16_t *zero,
                     int64_t T, int H, int D, int G, double *out)
{
    const int NG = D / G;
#pragma omp parallel for schedule(static)
    for (int64_t th = 0; th < T * H; ++th)
        for (int c = 0; c < D; ++c) {
            double s = (double)tkvo_f16_to_f32(scale[th * NG + c / G]);
            double z = (double)tkvo_f16_to_f32(zero[th * NG + c / G]);
            out[th * D + c] = (double)codes[th * D + c] * s + z;
        }
}

/* Prefill gather (Sec. 3.2.3 "Prefill"): the cached rows dequantised into FP16.  code * scale has at most
 * 15 significant bits and both terms lie on the binary16 exponent range, so the binary64 sum below is the
 * exact value; it is rounded to binary16 once. */
void tkvo_dequantize_f16(const uint8_t *codes, const uint16_t *scale, const uint16_t *zero,
                         int64_t T, int H, int D, int G, uint16_t *out)
{
    const int NG = D / G;
#pragma omp parallel for schedule(static)
    for (int64_t th = 0; th < T * H; ++th)
        for (int c = 0; c < D; ++c) {
            double s = (double)tkvo_f16_to_f32(scale[th * NG + c / G]);
            double z = (double)tkvo_f16_to_f32(zero[th * NG + c / G]);
            out[th * D + c] = tkvo_f64_to_f16((double)codes[th * D + c] * s + z);
        }
}

/* ------------------------------------------------------------------ */
/* attention: the plain definition, fp64 (Sec. 3.2.3 "Decode")         */
/* ------------------------------------------------------------------ */

/* One query head against n tokens of dequantised K, V (row stride D). */
static void attend_one(const double *q, const double *K, const double *V, int64_t n, int D,
                       double sm_scale, double *logit, double *out)
{
    for (int c = 0; c < D; ++c) out[c] = 0.0;
    if (n == 0) return;                 /* empty context: zeros, not NaN */
    double m = -INFINITY;
    for (int64_t t = 0; t < n; ++t) {
        double acc = 0.0;
        for (int c = 0; c < D; ++c) acc += q[c] * K[t * D + c];
        logit[t] = acc * sm_scale;
        if (logit[t] > m) m = logit[t];
    }
    double denom = 0.0;
    for (int64_t t = 0; t < n; ++t) {
        double p = exp(logit[t] - m);
        denom += p;
        for (int c = 0; c < D; ++c) out[c] += p * V[t * D + c];
    }
    for (int c = 0; c < D; ++c) out[c] /= denom;
}

/* Dense fp64 attention over real-valued K, V.
 * q: f64 [B, Hq, D]; K, V: f64 [T, Hkv, D] (sequences concatenated);
 * seq_indptr: i64 [B+1]; query head h reads kv head h / (Hq/Hkv).
 * out: f64 [B, Hq, D]. */
int tkvo_attention_f64(const double *q, const double *K, const double *V,
                       const int64_t *seq_indptr, int B, int Hq, int Hkv, int D,
                       double sm_scale, double *out)
{
    if (Hkv <= 0 || Hq % Hkv) return -1;
    const int R = Hq / Hkv;
    int err = 0;
#pragma omp parallel for schedule(dynamic, 1) collapse(2)
    for (int b = 0; b < B; ++b)
        for (int kh = 0; kh < Hkv; ++kh) {
            int64_t t0 = seq_indptr[b], n = seq_indptr[b + 1] - t0;
            double *Kb = (double *)malloc(sizeof(double) * (size_t)(n ? n : 1) * D);
            double *Vb = (double *)malloc(sizeof(double) * (size_t)(n ? n : 1) * D);
            double *lg = (double *)malloc(sizeof(double) * (size_t)(n ? n : 1));
            if (!Kb || !Vb || !lg) { err = 1; free(Kb); free(Vb); free(lg); continue; }
            for (int64_t t = 0; t < n; ++t) {
                memcpy(Kb + t * D, K + ((t0 + t) * Hkv + kh) * (int64_t)D, sizeof(double) * D);
                memcpy(Vb + t * D, V + ((t0 + t) * Hkv + kh) * (int64_t)D, sizeof(double) * D);
            }
            for (int r = 0; r < R; ++r) {
                int h = kh * R + r;
                attend_one(q + ((int64_t)b * Hq + h) * D, Kb, Vb, n, D, sm_scale, lg,
                           out + ((int64_t)b * Hq + h) * D);
            }
            free(Kb); free(Vb); free(lg);
        }
    return err ? -2 : 0;
}

/* Attention over the quantised cache given as canonical arrays: dequantise
 * each (sequence, kv head) slice exactly, then the definition above.
 * q: bf16 [B, Hq, D]. */
int tkvo_attention_quantized(const uint16_t *q,
                             const uint8_t *Kc, const uint16_t *Ks, const uint16_t *Kz,
                             const uint8_t *Vc, const uint16_t *Vs, const uint16_t *Vz,
                             const int64_t *seq_indptr, int B, int Hq, int Hkv, int D, int G,
                             double sm_scale, double *out)
{
    if (Hkv <= 0 || Hq % Hkv || G <= 0 || D % G) return -1;
    const int R = Hq / Hkv, NG = D / G;
    int err = 0;
#pragma omp parallel for schedule(dynamic, 1) collapse(2)
    for (int b = 0; b < B; ++b)
        for (int kh = 0; kh < Hkv; ++kh) {
            int64_t t0 = seq_indptr[b], n = seq_indptr[b + 1] - t0;
            double *Kb = (double *)malloc(sizeof(double) * (size_t)(n ? n : 1) * D);
            double *Vb = (double *)malloc(sizeof(double) * (size_t)(n ? n : 1) * D);
            double *lg = (double *)malloc(sizeof(double) * (size_t)(n ? n : 1));
            double *qd = (double *)malloc(sizeof(double) * (size_t)D);
            if (!Kb || !Vb || !lg || !qd) { err = 1; free(Kb); free(Vb); free(lg); free(qd); continue; }
            for (int64_t t = 0; t < n; ++t) {
                int64_t th = (t0 + t) * Hkv + kh;
                for (int c = 0; c < D; ++c) {
                    int64_t m = th * NG + c / G;
                    Kb[t * D + c] = (double)Kc[th * D + c] * (double)tkvo_f16_to_f32(Ks[m])
                                    + (double)tkvo_f16_to_f32(Kz[m]);
                    Vb[t * D + c] = (double)Vc[th * D + c] * (double)tkvo_f16_to_f32(Vs[m])
                                    + (double)tkvo_f16_to_f32(Vz[m]);
                }
            }
            for (int r = 0; r < R; ++r) {
                int h = kh * R + r;
                for (int c = 0; c < D; ++c)
                    qd[c] = (double)tkvo_bf16_to_f32(q[((int64_t)b * Hq + h) * D + c]);
                attend_one(qd, Kb, Vb, n, D, sm_scale, lg, out + ((int64_t)b * Hq + h) * D);
            }
            free(Kb); free(Vb); free(lg); free(qd);
        }
    return err ? -2 : 0;
}

/* ------------------------------------------------------------------ */
/* page codec: this build's layout, re-implemented from its formulas   */
/* ------------------------------------------------------------------ */
/* Fixed geometry of the layout: 64 tokens per page, head_dim 128, G = 32.
 * A record holds one (page, kv head): six planes
 *   K codes | K scale | K zero | V codes | V scale | V zero.
 * Code planes are 64*128*bits/8 bytes, metadata planes 64*4 fp16 = 512 bytes.
 * Pages [0, P2) are INT2, [P2, P2+P4) INT4 (the offset split of Sec. 3.2.2). */
enum { TP = 64, HD = 128, GS = 32, NGR = 4 };

static inline int64_t code_plane_bytes(int bits) { return (int64_t)TP * HD * bits / 8; }
int64_t tkvo_record_bytes(int bits) { return 2 * (code_plane_bytes(bits) + 512 + 512); }

/* byte offsets of the planes inside a record */
static inline int64_t off_kc(int bits) { (void)bits; return 0; }
static inline int64_t off_ks(int bits) { return code_plane_bytes(bits); }
static inline int64_t off_kz(int bits) { return code_plane_bytes(bits) + 512; }
static inline int64_t off_vc(int bits) { return code_plane_bytes(bits) + 1024; }
static inline int64_t off_vs(int bits) { return 2 * code_plane_bytes(bits) + 1024; }
static inline int64_t off_vz(int bits) { return 2 * code_plane_bytes(bits) + 1536; }

/* K codes: token-major, arranged in 16-byte chunks of four 32-bit words, one
 * word per channel group.  INT4: a word holds 8 consecutive channels of a
 * group; INT2: 16 consecutive channels.  Chunks are ordered
 * [16-token tile][word-in-group][token-in-tile]. */
void tkvo_kcode_pos(int bits, int t, int c, int *word, int *shift)
{
    int tile = t / 16, row = t % 16, g = c / 32, cg = c % 32;
    if (bits == 4) {
        int wq = cg / 8, j = cg % 8;
        *word = ((tile * 4 + wq) * 16 + row) * 4 + g;
        *shift = 4 * j;
    } else {
        int hf = cg / 16, k = cg % 16;
        *word = ((tile * 2 + hf) * 16 + row) * 4 + g;
        *shift = 2 * k;
    }
}

/* V codes: channel-major, a 32-bit word holds several tokens of ONE channel:
 * INT4 8 tokens, INT2 16 tokens, always tokens that share quad = (t%16)/4.
 * Position of token t inside its word: with j = 4*((t/16)%2) + t%4,
 *   INT4: nibble (j%2)*4 + j/2                       (word covers block t/32)
 *   INT2: crumb  4*(t/32) + j/2 + 8*(j%2)            (word covers the page)
 * Words are ordered [block (INT4 only)][channel-tile/4][quad][channel%16][channel-tile%4]. */
void tkvo_vcode_pos(int bits, int t, int c, int *word, int *shift)
{
    int jt = c / 16, n = c % 16, jh = jt / 4, jl = jt % 4;
    int quad = (t % 16) / 4;
    int j = 4 * ((t / 16) % 2) + t % 4;
    if (bits == 4) {
        int blk = t / 32;
        *word = (((blk * 2 + jh) * 4 + quad) * 16 + n) * 4 + jl;
        *shift = 4 * ((j % 2) * 4 + j / 2);
    } else {
        *word = ((jh * 4 + quad) * 16 + n) * 4 + jl;
        *shift = 2 * (4 * (t / 32) + j / 2 + 8 * (j % 2));
    }
}

/* K scale / K zero: fp16 [token][group]. */
int tkvo_kmeta_index(int t, int g) { return t * 4 + g; }
/* K scale / K zero of a page whose INT2 keys are quantised per channel: fp16 [block t/32][position of the
 * channel], 128 positions per block.  The position lists the channels in the order the decode kernel's
 * matrix operand holds them: chunks of 8 values per (group c/32, quarter), quarter = 2*((c%32)/16) + (c%8)/4,
 * and inside a chunk the pair (c, c+8) of k = c%4 sits at 2k, 2k+1. */
int tkvo_kcmeta_index(int blk, int c)
{
    int g = c / 32, r = c % 32;
    int quarter = 2 * (r / 16) + (r % 8) / 4;
    int k = r % 4, hi = (r % 16) / 8;
    return ((blk * 4 + g) * 4 + quarter) * 8 + 2 * k + hi;
}
/* V scale / V zero: fp16 in chunks of 8 tokens [block t/32][quad][group][j]
 * with j as above (the order in which a word of V codes lists its tokens). */
int tkvo_vmeta_index(int t, int g)
{
    int quad = (t % 16) / 4, j = 4 * ((t / 16) % 2) + t % 4;
    return (((t / 32) * 4 + quad) * 4 + g) * 8 + j;
}

static inline void put_bits(uint8_t *plane, int word, int shift, int nbits, uint32_t v)
{
    uint32_t w; memcpy(&w, plane + 4 * (int64_t)word, 4);   /* little-endian words */
    uint32_t mask = ((1u << nbits) - 1u) << shift;
    w = (w & ~mask) | ((v << shift) & mask);
    memcpy(plane + 4 * (int64_t)word, &w, 4);
}
static inline uint32_t get_bits(const uint8_t *plane, int word, int shift, int nbits)
{
    uint32_t w; memcpy(&w, plane + 4 * (int64_t)word, 4);
    return (w >> shift) & ((1u << nbits) - 1u);
}
static inline void put_h(uint8_t *plane, int idx, uint16_t v) { memcpy(plane + 2 * (int64_t)idx, &v, 2); }
static inline uint16_t get_h(const uint8_t *plane, int idx) { uint16_t v; memcpy(&v, plane + 2 * (int64_t)idx, 2); return v; }

/* Write one token (all 128 channels, 4 groups, K and V) into slot t of a
 * record; bits of other slots are left as they are. */
void tkvo_record_put_token(uint8_t *rec, int bits, int t,
                           const uint8_t *kc, const uint16_t *ks, const uint16_t *kz,
                           const uint8_t *vc, const uint16_t *vs, const uint16_t *vz)
{
    int w, s;
    for (int c = 0; c < HD; ++c) {
        tkvo_kcode_pos(bits, t, c, &w, &s); put_bits(rec + off_kc(bits), w, s, bits, kc[c]);
        tkvo_vcode_pos(bits, t, c, &w, &s); put_bits(rec + off_vc(bits), w, s, bits, vc[c]);
    }
    for (int g = 0; g < NGR; ++g) {
        put_h(rec + off_ks(bits), tkvo_kmeta_index(t, g), ks[g]);
        put_h(rec + off_kz(bits), tkvo_kmeta_index(t, g), kz[g]);
        put_h(rec + off_vs(bits), tkvo_vmeta_index(t, g), vs[g]);
        put_h(rec + off_vz(bits), tkvo_vmeta_index(t, g), vz[g]);
    }
}

void tkvo_record_get_token(const uint8_t *rec, int bits, int t,
                           uint8_t *kc, uint16_t *ks, uint16_t *kz,
                           uint8_t *vc, uint16_t *vs, uint16_t *vz)
{
    int w, s;
    for (int c = 0; c < HD; ++c) {
        tkvo_kcode_pos(bits, t, c, &w, &s); kc[c] = (uint8_t)get_bits(rec + off_kc(bits), w, s, bits);
        tkvo_vcode_pos(bits, t, c, &w, &s); vc[c] = (uint8_t)get_bits(rec + off_vc(bits), w, s, bits);
    }
    for (int g = 0; g < NGR; ++g) {
        ks[g] = get_h(rec + off_ks(bits), tkvo_kmeta_index(t, g));
        kz[g] = get_h(rec + off_kz(bits), tkvo_kmeta_index(t, g));
        vs[g] = get_h(rec + off_vs(bits), tkvo_vmeta_index(t, g));
        vz[g] = get_h(rec + off_vz(bits), tkvo_vmeta_index(t, g));
    }
}

/* Per-channel key metadata of one 32-token block of an INT2 record: scale, zero fp16 [128]. */
void tkvo_record_put_kblock(uint8_t *rec, int blk, const uint16_t *ks, const uint16_t *kz)
{
    for (int c = 0; c < HD; ++c) {
        put_h(rec + off_ks(2), tkvo_kcmeta_index(blk, c), ks[c]);
        put_h(rec + off_kz(2), tkvo_kcmeta_index(blk, c), kz[c]);
    }
}
void tkvo_record_get_kblock(const uint8_t *rec, int blk, uint16_t *ks, uint16_t *kz)
{
    for (int c = 0; c < HD; ++c) {
        ks[c] = get_h(rec + off_ks(2), tkvo_kcmeta_index(blk, c));
        kz[c] = get_h(rec + off_kz(2), tkvo_kcmeta_index(blk, c));
    }
}

int64_t tkvo_pool_bytes(int Hkv, int64_t P2, int64_t P4)
{ return (P2 * tkvo_record_bytes(2) + P4 * tkvo_record_bytes(4)) * Hkv; }

/* byte offset of the record of (page, head); the page's width follows from
 * one comparison against the offset P2 (Sec. 3.2.2). */
int64_t tkvo_record_offset(int Hkv, int64_t P2, int64_t page, int head, int *bits_out)
{
    if (page < P2) { if (bits_out) *bits_out = 2; return (page * Hkv + head) * tkvo_record_bytes(2); }
    if (bits_out) *bits_out = 4;
    return P2 * Hkv * tkvo_record_bytes(2) + ((page - P2) * Hkv + head) * tkvo_record_bytes(4);
}

/* Scatter canonical per-token arrays into a pool.  slot_ids[t] = page*64+slot.
 * The token's width must match its page's pool.  bit_map[page] is set to the
 * width of every page that receives a token.  Returns 0, -1 on mismatch. */
int tkvo_pack_pool(uint8_t *pool, uint8_t *bit_map, int Hkv, int64_t P2, int64_t P4,
                   const int64_t *slot_ids, const uint8_t *bits, int64_t T,
                   const uint8_t *Kc, const uint16_t *Ks, const uint16_t *Kz,
                   const uint8_t *Vc, const uint16_t *Vs, const uint16_t *Vz)
{
    for (int64_t t = 0; t < T; ++t) {
        int64_t page = slot_ids[t] / TP;
        if (slot_ids[t] < 0 || page >= P2 + P4) return -1;
        if (bits[t] != (page < P2 ? 2 : 4)) return -1;
        bit_map[page] = bits[t];
    }
    /* records of different kv heads never share a byte: one thread per head */
#pragma omp parallel for schedule(static)
    for (int h = 0; h < Hkv; ++h)
        for (int64_t t = 0; t < T; ++t) {
            int64_t page = slot_ids[t] / TP; int slot = (int)(slot_ids[t] % TP);
            int64_t th = t * Hkv + h;
            uint8_t *rec = pool + tkvo_record_offset(Hkv, P2, page, h, NULL);
            tkvo_record_put_token(rec, bits[t], slot, Kc + th * HD, Ks + th * NGR, Kz + th * NGR,
                                  Vc + th * HD, Vs + th * NGR, Vz + th * NGR);
        }
    return 0;
}

/* Gather the canonical arrays of T tokens back out of a pool. */
int tkvo_unpack_pool(const uint8_t *pool, int Hkv, int64_t P2, int64_t P4,
                     const int64_t *slot_ids, int64_t T,
                     uint8_t *Kc, uint16_t *Ks, uint16_t *Kz,
                     uint8_t *Vc, uint16_t *Vs, uint16_t *Vz)
{
    for (int64_t t = 0; t < T; ++t)
        if (slot_ids[t] < 0 || slot_ids[t] / TP >= P2 + P4) return -1;
#pragma omp parallel for schedule(static)
    for (int64_t t = 0; t < T; ++t) {
        int64_t page = slot_ids[t] / TP; int slot = (int)(slot_ids[t] % TP);
        int pb;
        for (int h = 0; h < Hkv; ++h) {
            int64_t th = t * Hkv + h;
            const uint8_t *rec = pool + tkvo_record_offset(Hkv, P2, page, h, &pb);
            tkvo_record_get_token(rec, pb, slot, Kc + th * HD, Ks + th * NGR, Kz + th * NGR,
                                  Vc + th * HD, Vs + th * NGR, Vz + th * NGR);
        }
    }
    return 0;
}

int tkvo_num_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}
