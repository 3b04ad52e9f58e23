// tkv_decode_attention: split-K flash-decoding over the paged INT2 / INT4 KV
// pool with in-register dequantisation, and the cross-split reduction
// (paper Sec. 3.2.3 "Decode": KV processed as parallel contiguous splits,
// each running one dequantisation path, merged by online log-sum-exp).
//
// One wavefront owns one (work item, kv head): a contiguous range of one
// sequence's page list.  All query heads that share the kv head (up to 8)
// are processed together so the packed KV bytes are read from HBM once.
//
// Matrix cores do both contractions (v_mfma_f32_16x16x32_f16), fp32 accumulate,
// and the packed codes are never expanded by arithmetic: a masked 16-bit field
// with a code in its low ten bits *is* the fp16 subnormal code * 2^(pos-24), so
// unpacking is one AND per two codes, for K and for V.
//
//   QK^T  D[token, head] = sum_c code[token, c] * q[head, c]   one MFMA per
//         (16-token tile, group of 32 channels).  q is converted to fp16 once,
//         scaled by a power of two (exact) and by 2^-pos per slot; the K scale
//         (fp32, times the compensating power of two) multiplies the MFMA
//         result.  The zero-point term sum_g zero[token,g] * sum_{c in g} q[head,c]
//         is one more MFMA whose A operand is the stored fp16 zero plane.
//         Head columns 8..15 repeat heads 0..7.
//   PV    D[head, channel] = sum_token (P[head, token] * scale[token, g]) * code[token, channel]
//         The V scale multiplies P, not the codes.  The softmax weights must be
//         good to about 2^-17 (a group with outliers has |code * scale| and
//         |zero| of tens while the tolerance near 0 is 2e-3), so P is split into
//         two fp16 pieces that occupy the 16 MFMA rows (8 heads x {hi, lo});
//         row hi carries fp16(P_hi * scale), row lo carries P_lo * scale plus
//         the exact remainder of the hi product, and the epilogue adds the two
//         rows.  The zero-point term sum_token P * zero[token, g] and the
//         softmax denominator come from one extra MFMA of the same P pieces
//         against the zero plane and a column of ones.
//
// Every product the MFMAs see is exact; the roundings are fp32 accumulation,
// the fp32 K-scale multiply, the 22-bit split of P and the 2^-22 relative
// rounding of the lo row.
#include <hip/hip_runtime.h>
#include <hip/hip_fp16.h>

#include <mutex>
#include <type_traits>

#include "tkv_internal.h"
#include "tkv_layout.h"

namespace {

using namespace tkv;

typedef _Float16 half8 __attribute__((ext_vector_type(8)));
typedef _Float16 half2_t __attribute__((ext_vector_type(2)));
typedef float floatx4 __attribute__((ext_vector_type(4)));
typedef uint32_t uint4v __attribute__((ext_vector_type(4)));

#ifndef TKV_WAVES_PER_EU
#define TKV_WAVES_PER_EU 3
#endif

constexpr float kTau = 4.0f;   // rescale when a logit exceeds the reference maximum by this much (log2 units)
// Softmax weights are carried as W = P * 2^kPExp (P <= 2^kTau), so that the lo piece of a small weight
// stays clear of the fp16 subnormal grid; numerator and denominator share the factor.
constexpr int kPExp = 8;
// The V scale is staged as scale * 2^(kVExp - pos), pos = bit position of the code's field in its fp16 half; undone once in the epilogue.
constexpr int kVExp = -1;
// W * staged scale must stay finite in fp16: the staged scale is clamped to 65504 / 2^(kTau + kPExp)
constexpr uint32_t kVsClamp = 0x4bff4bffu;   // fp16 15.99 twice
// Per-channel INT2 keys: q'' (q normalised, times its slot factor) stays below 2^6 and is multiplied by the K scale in fp16; the scale saturates at 1023.
constexpr uint32_t kKcClamp = 0x63fe63feu;   // fp16 1023 twice
constexpr int kKcQExp = 9;   // the first slot factor is 2^-3, so q'' stays below 2^6

__device__ __forceinline__ half8 as_half8(uint32_t a, uint32_t b, uint32_t c, uint32_t d)
{
    uint4v v = {a, b, c, d};
    return __builtin_bit_cast(half8, v);
}
__device__ __forceinline__ uint32_t pk_mul(uint32_t x, uint32_t y)
{
    const half2_t r = __builtin_bit_cast(half2_t, x) * __builtin_bit_cast(half2_t, y);
    return __builtin_bit_cast(uint32_t, r);
}
__device__ __forceinline__ uint32_t pk_rem(uint32_t x, uint32_t y, uint32_t h)   // x * y - h per fp16 half, one rounding
{
    const half2_t r = __builtin_elementwise_fma(__builtin_bit_cast(half2_t, x), __builtin_bit_cast(half2_t, y),
                                                -__builtin_bit_cast(half2_t, h));
    return __builtin_bit_cast(uint32_t, r);
}
__device__ __forceinline__ uint32_t pk_min(uint32_t x, uint32_t y)
{
    const half2_t r = __builtin_elementwise_min(__builtin_bit_cast(half2_t, x), __builtin_bit_cast(half2_t, y));
    return __builtin_bit_cast(uint32_t, r);
}
// p - k * t where t is the fp16 value in the low (HALF = 0) or high (HALF = 1) half of `t2`
template <int HALF> __device__ __forceinline__ float residual(uint32_t t2, float negk, float p)
{
    float r;
    if (HALF == 0) asm("v_fma_mix_f32 %0, %1, %2, %3 op_sel:[0,0,0] op_sel_hi:[1,0,0]" : "=v"(r) : "v"(t2), "v"(negk), "v"(p));
    else asm("v_fma_mix_f32 %0, %1, %2, %3 op_sel:[1,0,0] op_sel_hi:[1,0,0]" : "=v"(r) : "v"(t2), "v"(negk), "v"(p));
    return r;
}
// One fp16 piece of (p0, p1): lanes with negk = 0 get the leading 11 bits (truncated), lanes with
// negk = -1 the next 11 bits of the remainder.  `hi` receives the leading piece in every lane.
__device__ __forceinline__ uint32_t p_piece(float p0, float p1, float negk, uint32_t &hi)
{
    hi = __builtin_bit_cast(uint32_t, __builtin_amdgcn_cvt_pkrtz(p0, p1));
    const float r0 = residual<0>(hi, negk, p0), r1 = residual<1>(hi, negk, p1);
    return __builtin_bit_cast(uint32_t, __builtin_amdgcn_cvt_pkrtz(r0, r1));
}
__device__ __forceinline__ uint32_t pk_fma(uint32_t x, uint32_t y, uint32_t z)   // x * y + z per fp16 half, one rounding
{
    const half2_t r = __builtin_elementwise_fma(__builtin_bit_cast(half2_t, x), __builtin_bit_cast(half2_t, y),
                                                __builtin_bit_cast(half2_t, z));
    return __builtin_bit_cast(uint32_t, r);
}
__device__ __forceinline__ uint32_t pack_h2(float a, float b)
{
    const half2_t v = {(_Float16)a, (_Float16)b};
    return __builtin_bit_cast(uint32_t, v);
}
__device__ __forceinline__ floatx4 mfma(half8 a, half8 b, floatx4 c)
{
    return __builtin_amdgcn_mfma_f32_16x16x32_f16(a, b, c, 0, 0, 0);
}
// The value of the lane eight columns on in the same row of 16 lanes.
__device__ __forceinline__ float row_ror8(float v)
{
    return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), 0x128 /* row_ror:8 */, 0xf, 0xf, false));
}
__device__ __forceinline__ float wave_max(float v)
{
#pragma unroll
    for (int o = 32; o; o >>= 1) v = fmaxf(v, __shfl_xor(v, o));
    return v;
}
// Orders this wavefront's LDS writes before its later LDS reads.  The workgroup is one wavefront
// and LDS operations of a wavefront execute in order, so no wait and no barrier instruction is needed.
__device__ __forceinline__ void lds_order()
{
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

struct WaveState {
    floatx4 acc[8];     // PV accumulators: tile jt (16 channels) x rows 4*q4 + i = (head, piece of P)
    floatx4 zacc;       // zero-term (cols 0..3 = groups) and denominator (col 4), same rows
    float m_ref;        // reference maximum of this lane's head column, log2 units, -inf before the first page
};


// Only the kernel for per-channel INT2 keys holds the second q operand.
template <bool KC> struct LdsExtra {};
template <> struct LdsExtra<true> {
    alignas(16) uint4 qp[kGroups][64];                   // q * 2^E in the slot order of qo, without the slot factors
};
template <bool KC> struct alignas(16) Lds : LdsExtra<KC> {
    // Per-channel INT2 keys reuse ks and kz while INT2 pages run: ks holds the K scale plane (512 B) and the
    // K zero plane (512 B) of the page as stored, kz a plane of zeros (the INT4 pages, which come later in
    // an item, overwrite all three with their own staging).
    alignas(16) float ks[kPageTokens * kGroups];         // K scale * F, fp32 [token][group]
    alignas(16) uint32_t vs[kPageTokens * kGroups / 2];  // V scale * 2^(kVExp - pos), fp16 pairs in plane order
    alignas(16) uint32_t vz[kPageTokens * kGroups / 2];  // V zero, fp16 pairs in plane order
    alignas(16) uint2 kz[kPageTokens];                   // K zero, four fp16 per token
    alignas(16) uint4 qo[kGroups][64];                   // B operand of the QK^T MFMAs per group and lane
    alignas(16) float alpha[16];
    alignas(16) float zl[8][8];
    __device__ __forceinline__ uint4 *kc_scale() { return reinterpret_cast<uint4 *>(ks); }
    __device__ __forceinline__ uint4 *kc_zero() { return reinterpret_cast<uint4 *>(ks) + 32; }
    __device__ __forceinline__ uint4 *kc_nil() { return reinterpret_cast<uint4 *>(kz); }
};

// B operand of the QK^T MFMAs for one width, kept in LDS: per group and lane, 4 registers of fp16
// pairs holding q' = q * 2^E * 2^-pos in the slot order the unpack produces.
template <int BITS, bool KC, class QF>
__device__ __forceinline__ void build_q_operand(const QF *qf /* this lane's head, 128 values q * 2^E in LDS */, int q4,
                                               int lane, Lds<KC> &lds)
{
#pragma unroll
    for (int g = 0; g < 4; ++g) {
        uint32_t r[4], rp[4] = {0, 0, 0, 0};
        (void)rp;
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            int c0, c1;
            float f;
            if (BITS == 4) {
                // registers: (n0,n4) (n1,n5)*16 (n2,n6) (n3,n7)*16 of the 8-channel word q4
                const int nib = (k & 1) + 2 * (k >> 1);
                c0 = 32 * g + 8 * q4 + nib;
                c1 = c0 + 4;
                f = (k & 1) ? 0.0625f : 1.0f;
            } else {
                // registers: (crumb 4*sub+k, crumb 8+4*sub+k) * 2^(2k+3) of the 16-channel word q4/2
                c0 = 32 * g + 16 * (q4 >> 1) + 4 * (q4 & 1) + k;
                c1 = c0 + 8;
                // the unpack leaves the field of slot k at bit 2k + 3 (see compute_page)
                f = 1.0f / (float)(1 << (2 * k + 3));
            }
            r[k] = pack_h2((float)qf[c0] * f, (float)qf[c1] * f);
            if constexpr (KC && BITS == 2) rp[k] = pack_h2((float)qf[c0], (float)qf[c1]);
        }
        lds.qo[g][lane] = make_uint4(r[0], r[1], r[2], r[3]);
        if constexpr (KC && BITS == 2) lds.qp[g][lane] = make_uint4(rp[0], rp[1], rp[2], rp[3]);
    }
}

// Everything one wavefront loads for one (page, kv head) record.
template <int BITS> struct PageRegs {
    uint4 kw[4];          // K codes: one 16-byte chunk per 16-token tile (four groups of this lane's channel slice)
    uint4 vw[BITS];       // V codes: 16-byte chunks, one word per 16-channel tile
    uint2 ksc, vsc, vzc;  // this lane's four entries of the K scale / V scale / V zero planes
    uint2 kzc;            // K zero of token `lane`, four groups
    uint32_t bm;          // bit_map entry of the page
};

// The loads of one record come in two parts, issued as soon as the registers they land in are free:
// part A (K codes, K zero, the three metadata planes, the bit_map entry) after the QK^T phase of the
// previous page, part B (V codes) after its PV phase.
template <int BITS>
__device__ __forceinline__ void load_page_a(PageRegs<BITS> &pr, const uint8_t *__restrict__ rec,
                                            const uint8_t *__restrict__ bit_map, int page, int lane)
{
    using R = Rec<BITS>;
    const int r16 = lane & 15, q4 = lane >> 4;
    const uint4 *kc = reinterpret_cast<const uint4 *>(rec + R::kKCodes);
    pr.ksc = reinterpret_cast<const uint2 *>(rec + R::kKScale)[lane];
    pr.vsc = reinterpret_cast<const uint2 *>(rec + R::kVScale)[lane];
    pr.vzc = reinterpret_cast<const uint2 *>(rec + R::kVZero)[lane];
    pr.bm = bit_map[page];
    pr.kzc = reinterpret_cast<const uint2 *>(rec + R::kKZero)[lane];
#pragma unroll
    for (int e = 0; e < 4; ++e) pr.kw[e] = BITS == 4 ? kc[e * 64 + lane] : kc[e * 32 + (q4 >> 1) * 16 + r16];
}
template <int BITS>
__device__ __forceinline__ void load_page_b(PageRegs<BITS> &pr, const uint8_t *__restrict__ rec, int lane)
{
    using R = Rec<BITS>;
    const uint4 *vc = reinterpret_cast<const uint4 *>(rec + R::kVCodes);
#pragma unroll
    for (int i = 0; i < BITS; ++i) pr.vw[i] = vc[i * 64 + lane];
}

// Lane constants of the page loop.
struct LaneConst {
    float F;              // 2^(24 - E): undoes the subnormal position and the power-of-two normalisation of q
    float kappa;          // sm_scale * log2(e)
    uint32_t vmul01, vmul23;   // fp16 pairs of the staging factor of the V scale
    float negk;           // 0 in head columns 0..7 (hi piece of P), -1 in columns 8..15 (lo piece)
    uint32_t lomask;      // 0 / all ones likewise
    float zmul;           // per-channel INT2 keys: 2^-24 in head columns 0..7, 0 in columns 8..15
};

// One page.  `after_qk` runs once the K codes, K zeros and metadata registers of `pr` are dead, `after_pv`
// once the V codes are: the caller reloads them there for the next page.
template <int BITS, bool KC, class AfterQK, class AfterPV>
__device__ __forceinline__ void compute_page(const PageRegs<BITS> &pr, int n_valid, int lane,
                                             half8 qz, const LaneConst &lc, WaveState &st, Lds<KC> &lds,
                                             AfterQK after_qk, AfterPV after_pv)
{
    constexpr bool kPerChannel = KC && BITS == 2;   // INT2 keys quantised per channel over 32-token blocks
    const int r16 = lane & 15, q4 = lane >> 4;
    const bool partial = n_valid < kPageTokens;   // wave-uniform: only the last page of a width can be partly filled

    // ---- stage metadata in LDS --------------------------------------------
    {
        uint2 vsc = pr.vsc, vzc = pr.vzc;
        if (partial) {
            // Tokens at or beyond n_valid (never-written slots) are masked by count, never by content:
            // their logits become -inf below (so P = 0) and their V scale and V zero become 0 here, so
            // the products with P = 0 cannot be NaN.
            // this lane holds plane entries 4*lane .. 4*lane+3: chunk lane/2, slots 4*(lane&1) + 0..3
            const int chunk = lane >> 1, blk = chunk >> 4, quad = (chunk >> 2) & 3, jb = 4 * (lane & 1);
            const int t0 = 32 * blk + 16 * (jb >> 2) + 4 * quad;   // tokens t0 .. t0+3
            const uint32_t m01 = (t0 < n_valid ? 0xffffu : 0u) | (t0 + 1 < n_valid ? 0xffff0000u : 0u);
            const uint32_t m23 = (t0 + 2 < n_valid ? 0xffffu : 0u) | (t0 + 3 < n_valid ? 0xffff0000u : 0u);
            vsc.x &= m01; vsc.y &= m23; vzc.x &= m01; vzc.y &= m23;
        }
        if constexpr (kPerChannel) {
            // the two key metadata planes as stored: fp16 [block][128 channel positions]
            reinterpret_cast<uint2 *>(lds.kc_scale())[lane] = make_uint2(pk_min(pr.ksc.x, kKcClamp), pk_min(pr.ksc.y, kKcClamp));
            reinterpret_cast<uint2 *>(lds.kc_zero())[lane] = pr.kzc;
        } else {
            const half2_t a = __builtin_bit_cast(half2_t, pr.ksc.x), b = __builtin_bit_cast(half2_t, pr.ksc.y);
            reinterpret_cast<float4 *>(lds.ks)[lane] =
                make_float4((float)a[0] * lc.F, (float)a[1] * lc.F, (float)b[0] * lc.F, (float)b[1] * lc.F);
            lds.kz[lane] = pr.kzc;
        }
        reinterpret_cast<uint2 *>(lds.vs)[lane] =
            make_uint2(pk_min(pk_mul(vsc.x, lc.vmul01), kVsClamp), pk_min(pk_mul(vsc.y, lc.vmul23), kVsClamp));
        reinterpret_cast<uint2 *>(lds.vz)[lane] = vzc;
    }
    lds_order();

    // ---- QK^T: S[e][i] = q . k_hat (unscaled) for token 16e + 4*q4 + i, head column r16
    floatx4 S[4];
    if constexpr (kPerChannel) {
        // score = sum_c (q_c s_c) code + sum_c q_c z_c with s, z of the token's block.  q s is formed per block
        // in two fp16 pieces, exactly (q has 8 significant bits, s 11): head columns 0..7 take
        // fp16(q s), columns 8..15 the remainder q s - fp16(q s); the columns of a head are added after the
        // MFMAs.  Lanes of the hi columns read their "rounded product to subtract" from a plane of zeros.
        const uint4 *sxp = r16 >= 8 ? lds.kc_scale() : lds.kc_nil();
        const uint32_t rot = (q4 & 1) ? 5u : 29u;   // this lane's 16 codes of a word are its upper / lower half
        // operands of both blocks first: the zero-term chains run on the matrix core while the VALU forms q s
        floatx4 z[2] = {{0.f, 0.f, 0.f, 0.f}, {0.f, 0.f, 0.f, 0.f}};
        uint32_t b[2][4][4];
#pragma unroll
        for (int g = 0; g < 4; ++g) {
            const uint4 qp = lds.qp[g][lane], qo = lds.qo[g][lane];
#pragma unroll
            for (int blk = 0; blk < 2; ++blk) {
                const int mi = (blk * 4 + g) * 4 + q4;
                const uint4 zc = lds.kc_zero()[mi];
                z[blk] = mfma(as_half8(zc.x, zc.y, zc.z, zc.w), as_half8(qp.x, qp.y, qp.z, qp.w), z[blk]);   // every row: sum_c q_c z_c
                const uint4 sc = lds.kc_scale()[mi], sx = sxp[mi];
                b[blk][g][0] = pk_rem(qo.x, sc.x, pk_mul(qo.x, sx.x));
                b[blk][g][1] = pk_rem(qo.y, sc.y, pk_mul(qo.y, sx.y));
                b[blk][g][2] = pk_rem(qo.z, sc.z, pk_mul(qo.z, sx.z));
                b[blk][g][3] = pk_rem(qo.w, sc.w, pk_mul(qo.w, sx.w));
            }
        }
#pragma unroll
        for (int e = 0; e < 4; ++e) S[e] = z[e >> 1] * lc.zmul;   // to the unit of the code products, hi columns only
        // four independent accumulation chains (one per 16-token tile)
#pragma unroll
        for (int g = 0; g < 4; ++g)
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const uint32_t wg = g == 0 ? pr.kw[e].x : g == 1 ? pr.kw[e].y : g == 2 ? pr.kw[e].z : pr.kw[e].w;
                // fields at bits 4:3, 6:5, 8:7, 10:9 of each half: q s spans more binades than q, and
                // the matrix core drops product bits that fall below its alignment window
                const uint32_t ws = __builtin_amdgcn_alignbit(wg, wg, rot);   // w >> 5 or w << 3, stray bits fall outside the masks
                const half8 a = as_half8(ws & 0x00180018u, ws & 0x00600060u, ws & 0x01800180u, ws & 0x06000600u);
                S[e] = mfma(a, as_half8(b[e >> 1][g][0], b[e >> 1][g][1], b[e >> 1][g][2], b[e >> 1][g][3]), S[e]);
            }
#pragma unroll
        for (int e = 0; e < 4; ++e) {
#pragma unroll
            for (int i = 0; i < 4; ++i) S[e][i] += row_ror8(S[e][i]);   // the two pieces of q s: columns h and h + 8
            asm volatile("" : "+v"(S[e]));
        }
        __builtin_amdgcn_sched_barrier(0);
    } else
#pragma unroll
    for (int e = 0; e < 4; ++e) {
        const uint2 kz = lds.kz[16 * e + r16];
        const half8 za = as_half8(kz.x, kz.y, kz.x, kz.y);
        floatx4 s = mfma(za, qz, floatx4{0.f, 0.f, 0.f, 0.f});   // zero-point term
        float4 sc[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) sc[i] = reinterpret_cast<const float4 *>(lds.ks)[16 * e + 4 * q4 + i];
        const uint32_t w[4] = {pr.kw[e].x, pr.kw[e].y, pr.kw[e].z, pr.kw[e].w};
#pragma unroll
        for (int g = 0; g < 4; ++g) {
            half8 a;
            if (BITS == 4) {
                const uint32_t w8 = w[g] >> 8;
                a = as_half8(w[g] & 0x000f000fu, w[g] & 0x00f000f0u, w8 & 0x000f000fu, w8 & 0x00f000f0u);
            } else {
                // this lane's 16 codes of the word are its upper or lower half; the rotate leaves the fields at bits
                // 4:3, 6:5, 8:7, 10:9 of each half (towards the top of the fp16 mantissa, as for V: the matrix core
                // drops product bits below its alignment window), stray bits fall outside the masks
                const uint32_t ws = __builtin_amdgcn_alignbit(w[g], w[g], (q4 & 1) ? 5u : 29u);
                a = as_half8(ws & 0x00180018u, ws & 0x00600060u, ws & 0x01800180u, ws & 0x06000600u);
            }
            const uint4 qb = lds.qo[g][lane];
            const half8 b = as_half8(qb.x, qb.y, qb.z, qb.w);
            const floatx4 p = mfma(a, b, floatx4{0.f, 0.f, 0.f, 0.f});
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const float scg = g == 0 ? sc[i].x : g == 1 ? sc[i].y : g == 2 ? sc[i].z : sc[i].w;
                s[i] = fmaf(scg, p[i], s[i]);
            }
        }
        asm volatile("" : "+v"(s));   // the scaled sums are formed here, not sunk next to their first use
        S[e] = s;
        __builtin_amdgcn_sched_barrier(0);   // one tile's LDS operands at a time (register pressure)
    }
    after_qk();
    if (partial) {
#pragma unroll
        for (int e = 0; e < 4; ++e)
#pragma unroll
            for (int i = 0; i < 4; ++i) S[e][i] = 16 * e + 4 * q4 + i < n_valid ? S[e][i] : -INFINITY;
    }

    // ---- online softmax with a lazily updated reference maximum ------------
    // The cheap test looks only at this lane's own 16 logits; the column maximum is formed across
    // lanes only when some lane needs a new reference.
    float mx = fmaxf(fmaxf(S[0][0], S[0][1]), fmaxf(S[0][2], S[0][3]));
#pragma unroll
    for (int e = 1; e < 4; ++e) mx = fmaxf(fmaxf(mx, S[e][0]), fmaxf(fmaxf(S[e][1], S[e][2]), S[e][3]));
    if (__any(mx * lc.kappa > st.m_ref + kTau)) {
        mx = fmaxf(mx, __shfl_xor(mx, 16));
        mx = fmaxf(mx, __shfl_xor(mx, 32));
        const float m_new = fmaxf(st.m_ref, mx * lc.kappa);
        const float alpha = m_new == -INFINITY ? 1.0f : __builtin_amdgcn_exp2f(st.m_ref - m_new);
        st.m_ref = m_new;
        if (q4 == 0) lds.alpha[r16] = alpha;   // columns r16 and r16 ^ 8 hold the same head
        lds_order();
        const float4 al = reinterpret_cast<const float4 *>(lds.alpha)[q4 & 1];   // rows 4*q4 .. 4*q4+3 -> heads (4*q4 + i) & 7
        const floatx4 av = {al.x, al.y, al.z, al.w};
#pragma unroll
        for (int jt = 0; jt < 8; ++jt) st.acc[jt] *= av;
        st.zacc *= av;
    }
    const float nmref = (float)kPExp - (st.m_ref == -INFINITY ? 0.0f : st.m_ref);
    uint32_t pa[2][4];   // this lane's piece of P (hi in head columns 0..7, lo in 8..15): A operand of the zero / denominator MFMA
    uint32_t py[2][4];   // the hi piece again in the lo columns, 0 in the hi columns
#pragma unroll
    for (int e = 0; e < 4; ++e) {
        float pv[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) pv[i] = __builtin_amdgcn_exp2f(fmaf(S[e][i], lc.kappa, nmref));
        uint32_t h01, h23;
        pa[e >> 1][2 * (e & 1)] = p_piece(pv[0], pv[1], lc.negk, h01);
        pa[e >> 1][2 * (e & 1) + 1] = p_piece(pv[2], pv[3], lc.negk, h23);
        py[e >> 1][2 * (e & 1)] = h01 & lc.lomask;
        py[e >> 1][2 * (e & 1) + 1] = h23 & lc.lomask;
    }

    // ---- PV ------------------------------------------------------------------
#pragma unroll
    for (int blk = 0; blk < 2; ++blk) {
        // zero term and denominator: columns 0..3 = groups, column 4 = ones
        {
            uint4 bz = reinterpret_cast<const uint4 *>(lds.vz)[(blk * 4 + q4) * 4 + (r16 & 3)];
            if (r16 >= 4) {
                const uint32_t c = r16 == 4 ? 0x3c003c00u : 0u;
                bz = make_uint4(c, c, c, c);
            }
            st.zacc = mfma(as_half8(pa[blk][0], pa[blk][1], pa[blk][2], pa[blk][3]), as_half8(bz.x, bz.y, bz.z, bz.w), st.zacc);
        }
#pragma unroll
        for (int g = 0; g < 4; ++g) {
            const uint4 vs = reinterpret_cast<const uint4 *>(lds.vs)[(blk * 4 + q4) * 4 + g];
            const uint32_t vsr[4] = {vs.x, vs.y, vs.z, vs.w};
            uint32_t ar[4];
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                // hi rows: fp16(P_hi * scale); lo rows: P_lo * scale + (P_hi * scale - fp16(P_hi * scale))
                const uint32_t t = pk_mul(py[blk][k], vsr[k]);
                ar[k] = pk_fma(pa[blk][k], vsr[k], pk_rem(py[blk][k], vsr[k], t));
            }
            const half8 a = as_half8(ar[0], ar[1], ar[2], ar[3]);
#pragma unroll
            for (int t2 = 0; t2 < 2; ++t2) {
                const int jt = 2 * g + t2;
                uint32_t w;
                {
                    const uint4 v = BITS == 4 ? pr.vw[blk * 2 + (jt >> 2)] : pr.vw[jt >> 2];
                    w = (jt & 3) == 0 ? v.x : (jt & 3) == 1 ? v.y : (jt & 3) == 2 ? v.z : v.w;
                }
                // Codes as fp16 subnormals, fields shifted towards the top of the mantissa (INT2: bits 4:3,
                // 6:5, 8:7, 10:9 of each half; INT4: bits 6:3 and 10:7): the matrix core aligns the products of
                // a lane's eight k-slots to the largest exponent *field* and drops what falls below a fixed
                // window, so leading zeros of a subnormal cost precision.  Bit 10 is the lowest exponent bit:
                // fp16 is linear through the first binade, so a field may reach it.  The slot's power of two
                // is undone in the staged V scale.
                half8 b;
                if (BITS == 4) {
                    const uint32_t wl = w << 3, wr = w >> 5;
                    b = as_half8(wl & 0x00780078u, wl & 0x07800780u, wr & 0x00780078u, wr & 0x07800780u);
                } else {
                    const uint32_t ws = blk ? (w >> 5) : (w << 3);
                    b = as_half8(ws & 0x00180018u, ws & 0x00600060u, ws & 0x01800180u, ws & 0x06000600u);
                }
                st.acc[jt] = mfma(a, b, st.acc[jt]);
            }
        }
    }
    after_pv();
}

// All pages [pb, pe) of one width (indices into the sequence's page list).
template <int BITS, bool KC>
__device__ __forceinline__ void run_pages(const uint8_t *__restrict__ pool, const uint8_t *__restrict__ bit_map,
                                          const int32_t *__restrict__ pages, int pb, int pe, int last_index,
                                          int last_valid, int page_lo, int page_hi, int n_pages_total, int kvh,
                                          int n_kv_heads, int n_pages_int2, int item_end, int item_pages, int lane, half8 qz,
                                          LaneConst lc, WaveState &st, Lds<KC> &lds, int32_t *status)
{
    // A V code enters the MFMA as code * 2^(pos - 24), pos = lowest bit of its field after the unpack shift; the
    // staged scale of the slot carries 2^(kVExp - pos).  This lane stages plane entries 4*lane .. 4*lane+3 =
    // k-slots 4*(lane&1) + 0..3, i.e. operand registers 2*(lane&1) (first pair) and 2*(lane&1) + 1 (second pair).
    {
        const int k0 = 2 * (lane & 1);
        const int p01 = BITS == 4 ? 3 : 3 + 2 * k0, p23 = BITS == 4 ? 7 : 5 + 2 * k0;
        const uint32_t h01 = (uint32_t)(15 + kVExp - p01) << 10, h23 = (uint32_t)(15 + kVExp - p23) << 10;
        lc.vmul01 = h01 | (h01 << 16);
        lc.vmul23 = h23 | (h23 << 16);
    }
    // Page id of list position pi and its number of valid tokens.  A page id outside its pool cannot be
    // addressed: it is flagged, a valid page is read instead and skipped.
    auto resolve = [&](int pi, int &page) -> int {
        page = __builtin_amdgcn_readfirstlane(pages[pi]);
        const bool ok = page >= page_lo && page < page_hi;
        if (!ok) {
            if (status && lane == 0)
                atomicOr(status, page < 0 || page >= n_pages_total ? TKV_STATUS_PAGE_RANGE : TKV_STATUS_BITMAP_MISMATCH);
            page = page_lo;
        }
        return ok ? (pi == last_index ? last_valid : kPageTokens) : 0;
    };
    // One register set: every part of the next record is requested as soon as the registers it lands in
    // are dead, so about one page per wavefront is in flight while the current one is computed.
    PageRegs<BITS> pr;
    int page = 0;
    int nv = resolve(pb, page), nv_next = 0;
    const uint8_t *rec = pool + record_offset(page, kvh, n_kv_heads, n_pages_int2);
    load_page_a<BITS>(pr, rec, bit_map, page, lane);
    load_page_b<BITS>(pr, rec, lane);
    int quartile = -1;
    for (int pi = pb; pi < pe; ++pi) {
        // Wavefronts that share a SIMD are served oldest first; left alone, the oldest finishes long before
        // the others and the SIMD ends its work with one wavefront.  The priority follows the share of the
        // item still to do, so the wavefronts of a SIMD advance together.
        const int q = (4 * (item_end - pi) - 1) / item_pages;   // 3 .. 0
        if (__builtin_expect(q != quartile, 0)) {
            quartile = q;
            if (q >= 3) __builtin_amdgcn_s_setprio(3);
            else if (q == 2) __builtin_amdgcn_s_setprio(2);
            else if (q == 1) __builtin_amdgcn_s_setprio(1);
            else __builtin_amdgcn_s_setprio(0);
        }
        // the last page requests its own record again: no branch around the loads
        const int pi_next = pi + 1 < pe ? pi + 1 : pi;
        const uint8_t *rec_next = rec;
        auto after_qk = [&]() {
            __builtin_amdgcn_sched_barrier(0);   // keep the reloads below the last use of the registers they overwrite
            int page_next;
            nv_next = resolve(pi_next, page_next);
            rec_next = pool + record_offset(page_next, kvh, n_kv_heads, n_pages_int2);
            load_page_a<BITS>(pr, rec_next, bit_map, page_next, lane);
        };
        auto after_pv = [&]() {
            __builtin_amdgcn_sched_barrier(0);
            load_page_b<BITS>(pr, rec_next, lane);
        };
        // the bit_map entry arrives with the page: a mismatch skips the whole page
        if (pr.bm != BITS && nv > 0) {
            if (status && lane == 0) atomicOr(status, TKV_STATUS_BITMAP_MISMATCH);
            nv = 0;
        }
        // a page with no valid token still runs (every token masked by count): no second path through the loop
        compute_page<BITS, KC>(pr, nv, lane, qz, lc, st, lds, after_qk, after_pv);
        rec = rec_next;
        nv = nv_next;
    }
}

// KC: the INT2 keys of the pool are quantised per channel over 32-token blocks (Sec. 3.2.1).
template <bool KC>
__global__ __launch_bounds__(64) __attribute__((amdgpu_waves_per_eu(TKV_WAVES_PER_EU, TKV_WAVES_PER_EU))) void tkv_decode_kernel(
    const uint8_t *__restrict__ pool, const uint8_t *__restrict__ bit_map, const uint16_t *__restrict__ q,
    const int32_t *__restrict__ page_indptr, const int32_t *__restrict__ page_ids,
    const int32_t *__restrict__ n_tok_int2, const int32_t *__restrict__ n_tok_int4,
    const int32_t *__restrict__ items, int batch, int n_kv_heads, int n_q_heads, int n_pages_int2, int n_pages_int4,
    float kappa, float *__restrict__ acc_ws, float *__restrict__ ml_ws, int32_t *status
    )
{
    using QF = typename std::conditional<KC, _Float16, float>::type;   // q * 2^E is exact in either type
    __shared__ Lds<KC> lds;
    // q * 2^E per head and channel, read while the MFMA operands are built.  The per-channel-key kernel keeps it
    // (2 KiB of fp16) in the page staging area ks | vs | vz, which is idle then, so that twelve wavefronts
    // still fit the LDS of a compute unit; it is written again before the INT4 operand is built.
    __shared__ QF qf_own[KC ? 1 : 8][kHeadDim];
    QF(*qf)[kHeadDim] = KC ? reinterpret_cast<QF(*)[kHeadDim]>(lds.ks) : qf_own;
    static_assert(sizeof(lds.ks) + sizeof(lds.vs) + sizeof(lds.vz) >= 8 * kHeadDim * sizeof(_Float16) && sizeof(lds.ks) % 16 == 0 &&
                  sizeof(lds.vs) % 16 == 0, "ks, vs, vz are consecutive members and together hold q for 8 heads");
    const int lane = threadIdx.x, r16 = lane & 15, q4 = lane >> 4;
    const int item = blockIdx.x / n_kv_heads, kvh = blockIdx.x % n_kv_heads;
    const int R = n_q_heads / n_kv_heads;
    const int seq = items[4 * item];
    if (seq < 0 || seq >= batch) return;   // malformed item: nothing is read or written for it
    const int n2 = n_tok_int2[seq], n4 = n_tok_int4[seq];
    const int np2 = (n2 + kPageTokens - 1) / kPageTokens, np4 = (n4 + kPageTokens - 1) / kPageTokens;
    const int seq_pages = page_indptr[seq + 1] - page_indptr[seq];
    const int np_all = np2 + np4 < seq_pages ? np2 + np4 : seq_pages;
    const int pb = items[4 * item + 1] > 0 ? items[4 * item + 1] : 0;
    const int pe = items[4 * item + 2] < np_all ? items[4 * item + 2] : np_all;
    const int32_t *pages = page_ids + page_indptr[seq];

    // ---- q: load the R heads, common power-of-two normalisation, group sums ----
    // lane l holds channels 2l, 2l+1 of every head
    float qv[8][2];
    float amax = 0.0f;
#pragma unroll
    for (int h = 0; h < 8; ++h) {
        uint32_t two = 0;
        if (h < R) two = reinterpret_cast<const uint32_t *>(q + ((size_t)seq * n_q_heads + kvh * R + h) * kHeadDim)[lane];
        qv[h][0] = __uint_as_float(two << 16);
        qv[h][1] = __uint_as_float(two & 0xffff0000u);
        amax = fmaxf(amax, fmaxf(fabsf(qv[h][0]), fabsf(qv[h][1])));
    }
    amax = wave_max(amax);
    // 2^E with max|q| * 2^E in [2^14, 2^15); E clamped so every factor stays a normal fp32
    int ex = 0;
    if (amax > 0.0f) { (void)frexpf(amax, &ex); }   // amax = m * 2^ex, m in [0.5, 1)
    int E = (KC ? kKcQExp : 15) - ex;
    E = E > 100 ? 100 : (E < -100 ? -100 : E);
    if (!(amax > 0.0f)) E = 0;
    const float two_e = ldexpf(1.0f, E);
    LaneConst lc;
    lc.F = ldexpf(1.0f, 24 - E);
    lc.kappa = kappa;
    lc.negk = r16 >= 8 ? -1.0f : 0.0f;
    lc.lomask = r16 >= 8 ? 0xffffffffu : 0u;
    lc.vmul01 = lc.vmul23 = 0;
    lc.zmul = r16 >= 8 ? 0.0f : 0x1p-24f;
    // q * 2^E to LDS; per-group sums of the unscaled q: lanes 16g .. 16g+15 hold group g
#pragma unroll
    for (int h = 0; h < 8; ++h) {
        if constexpr (KC) reinterpret_cast<uint32_t *>(qf[h])[lane] = pack_h2(qv[h][0] * two_e, qv[h][1] * two_e);
        else reinterpret_cast<float2 *>(qf[h])[lane] = make_float2(qv[h][0] * two_e, qv[h][1] * two_e);
        float sum = qv[h][0] + qv[h][1];
#pragma unroll
        for (int o = 1; o < 16; o <<= 1) sum += __shfl_xor(sum, o);
        if (r16 == 0) lds.zl[h][q4] = sum;   // [head][group]
    }
    lds_order();
    const int hcol = (r16 & 7) & (R - 1);   // head of this lane's column (columns beyond R repeat heads)
    half8 qz;
    {
        // Z-term B operand: slots 0..3 / 4..7 of chunk 0 = hi / mid pieces of the four group sums,
        // slots 0..3 of chunk 1 = lo pieces, everything else zero
        const float4 gs = reinterpret_cast<const float4 *>(lds.zl[hcol])[0];
        const float sums[4] = {gs.x, gs.y, gs.z, gs.w};
        float pc[8] = {0, 0, 0, 0, 0, 0, 0, 0};
#pragma unroll
        for (int g = 0; g < 4; ++g) {
            const _Float16 hi = (_Float16)sums[g];
            const float r1 = sums[g] - (float)hi;
            const _Float16 mid = (_Float16)r1;
            const _Float16 lo = (_Float16)(r1 - (float)mid);
            if (q4 == 0) { pc[g] = (float)hi; pc[4 + g] = (float)mid; }
            else if (q4 == 1) { pc[g] = (float)lo; }
        }
        qz = as_half8(pack_h2(pc[0], pc[1]), pack_h2(pc[2], pc[3]), pack_h2(pc[4], pc[5]), pack_h2(pc[6], pc[7]));
    }

    WaveState st;
#pragma unroll
    for (int jt = 0; jt < 8; ++jt) st.acc[jt] = floatx4{0.f, 0.f, 0.f, 0.f};
    st.zacc = floatx4{0.f, 0.f, 0.f, 0.f};
    st.m_ref = -INFINITY;

    const int n_pages_total = n_pages_int2 + n_pages_int4;
    // INT2 pages of the range, then INT4 pages: each page runs one dequantisation path
    const int e2 = pe < np2 ? pe : np2;
    if (pb < e2) {
        build_q_operand<2, KC>(qf[hcol], q4, lane, lds);
        LaneConst lc2 = lc;
        if constexpr (KC) {
            lc2.kappa = lc.kappa * lc.F;   // the power of two that the K scale carries otherwise
            lds.kc_nil()[lane & 31] = make_uint4(0u, 0u, 0u, 0u);
        }
        lds_order();
        run_pages<2, KC>(pool, bit_map, pages, pb, e2, np2 - 1, n2 - (np2 - 1) * kPageTokens, 0, n_pages_int2,
                         n_pages_total, kvh, n_kv_heads, n_pages_int2, pe, pe - pb, lane, qz, lc2, st, lds, status);
    }
    const int b4 = pb > np2 ? pb : np2;
    if (b4 < pe) {
        if constexpr (KC) {
            if (pb < e2) {   // the INT2 pages have used the staging area since
                lds_order();
#pragma unroll
                for (int h = 0; h < 8; ++h) {
                    uint32_t two = 0;
                    if (h < R) two = reinterpret_cast<const uint32_t *>(q + ((size_t)seq * n_q_heads + kvh * R + h) * kHeadDim)[lane];
                    reinterpret_cast<uint32_t *>(qf[h])[lane] = pack_h2(__uint_as_float(two << 16) * two_e, __uint_as_float(two & 0xffff0000u) * two_e);
                }
                lds_order();
            }
        }
        build_q_operand<4, KC>(qf[hcol], q4, lane, lds);
        lds_order();
        run_pages<4, KC>(pool, bit_map, pages, b4, pe, np2 + np4 - 1, n4 - (np4 - 1) * kPageTokens, n_pages_int2,
                     n_pages_total, n_pages_total, kvh, n_kv_heads, n_pages_int2, pe, pe - pb, lane, qz, lc, st, lds, status);
    }

    // ---- write the partial (m, l, acc) of this item ------------------------------
    // rows 0..7 carry the hi piece of P, rows 8..15 the lo piece: add lanes l and l^32
#pragma unroll
    for (int jt = 0; jt < 8; ++jt)
#pragma unroll
        for (int i = 0; i < 4; ++i) st.acc[jt][i] += __shfl_xor(st.acc[jt][i], 32);
#pragma unroll
    for (int i = 0; i < 4; ++i) st.zacc[i] += __shfl_xor(st.zacc[i], 32);
    lds_order();
    if (r16 < 8 && q4 < 2)
#pragma unroll
        for (int i = 0; i < 4; ++i) lds.zl[4 * q4 + i][r16] = st.zacc[i];   // [head][column]
    if (q4 == 0 && r16 < 8) lds.alpha[r16] = st.m_ref;
    lds_order();
    const float unscale = ldexpf(1.0f, 24 - kVExp);
    if (q4 < 2) {
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int head = 4 * q4 + i;
            if (head >= R) continue;
            const size_t ph = (size_t)item * n_q_heads + kvh * R + head;
            float *dst = acc_ws + ph * kHeadDim;
#pragma unroll
            for (int jt = 0; jt < 8; ++jt) dst[16 * jt + r16] = st.acc[jt][i] * unscale + lds.zl[head][jt >> 1];
            if (r16 == 0) {
                ml_ws[2 * ph] = lds.alpha[head];
                ml_ws[2 * ph + 1] = lds.zl[head][4];
            }
        }
    }
}

// D7: out = sum_i 2^(m_i - M) acc_i / sum_i 2^(m_i - M) l_i over the items of a sequence.
// One workgroup of 512 threads per (sequence, query head, slice of CH channels): the items' maxima are reduced in
// parallel, the weights go to LDS, then 512 / CH groups of CH threads (one thread per channel) each sum every
// (512 / CH)-th item.  CH = 128 (four groups) when a sequence has tens of items; CH = 16 (32 groups, eight
// workgroups per head) when it has hundreds, as a single long sequence with one kv head does.
constexpr int kReduceThreads = 512;
template <int CH>
__global__ __launch_bounds__(kReduceThreads) void tkv_reduce_kernel(
    const float *__restrict__ acc_ws, const float *__restrict__ ml_ws, const int32_t *__restrict__ seq_item_indptr,
    int n_q_heads, float *__restrict__ out)
{
    constexpr int kThreads = kReduceThreads, kChunk = 512, kParts = kThreads / CH, kSlices = kHeadDim / CH;
    __shared__ float w_s[kChunk];
    __shared__ float red[kThreads / 64];
    __shared__ float part_s[kParts][CH];
    __shared__ float den_s[kParts];
    const int bh = blockIdx.x / kSlices, slice = blockIdx.x % kSlices;
    const int b = bh / n_q_heads, h = bh % n_q_heads, tid = threadIdx.x;
    const int cl = tid % CH, c = slice * CH + cl, part = tid / CH;
    const int i0 = seq_item_indptr[b], i1 = seq_item_indptr[b + 1];
    // global maximum of the items' reference maxima
    float M = -INFINITY;
    for (int i = i0 + tid; i < i1; i += kThreads) M = fmaxf(M, ml_ws[2 * ((size_t)i * n_q_heads + h)]);
    M = wave_max(M);
    if ((tid & 63) == 0) red[tid >> 6] = M;
    __syncthreads();
    M = red[0];
#pragma unroll
    for (int k = 1; k < kThreads / 64; ++k) M = fmaxf(M, red[k]);
    float num = 0.0f, den = 0.0f;
    if (M != -INFINITY) {
        for (int base = i0; base < i1; base += kChunk) {
            const int n = i1 - base < kChunk ? i1 - base : kChunk;
            __syncthreads();
            if (tid < n) w_s[tid] = __builtin_amdgcn_exp2f(ml_ws[2 * ((size_t)(base + tid) * n_q_heads + h)] - M);
            __syncthreads();
#pragma unroll 4
            for (int k = part; k < n; k += kParts) {
                const size_t ph = (size_t)(base + k) * n_q_heads + h;
                num = fmaf(w_s[k], acc_ws[ph * kHeadDim + c], num);
                if (cl == 0) den = fmaf(w_s[k], ml_ws[2 * ph + 1], den);
            }
        }
    }
    part_s[part][cl] = num;
    if (cl == 0) den_s[part] = den;
    __syncthreads();
    if (part == 0) {
        float nsum = 0.0f, dsum = 0.0f;
#pragma unroll
        for (int k = 0; k < kParts; ++k) { nsum += part_s[k][cl]; dsum += den_s[k]; }
        out[((size_t)b * n_q_heads + h) * kHeadDim + c] = dsum > 0.0f ? nsum / dsum : 0.0f;
    }
}

} // namespace

int tkv_launch_decode_split(const tkv_desc *desc, const void *pool, const uint8_t *bit_map, const void *q,
                            const int32_t *page_indptr, const int32_t *page_ids, const int32_t *n_tok_int2,
                            const int32_t *n_tok_int4, const int32_t *items, int32_t n_items, int32_t batch,
                            int32_t n_q_heads, float sm_scale, void *workspace, int32_t *status, void *stream)
{
    if (n_items == 0) return TKV_OK;
    float *acc_ws = (float *)workspace;
    float *ml_ws = acc_ws + (size_t)n_items * n_q_heads * kHeadDim;
    const float kappa = sm_scale * 1.44269504088896340736f;
    auto kernel = desc->int2_key_axis == TKV_KEYS_PER_CHANNEL ? tkv_decode_kernel<true> : tkv_decode_kernel<false>;
    hipLaunchKernelGGL(kernel, dim3((unsigned)(n_items * desc->n_kv_heads)), dim3(64), 0,
                       (hipStream_t)stream, (const uint8_t *)pool, bit_map, (const uint16_t *)q, page_indptr,
                       page_ids, n_tok_int2, n_tok_int4, items, batch, desc->n_kv_heads, n_q_heads,
                       desc->n_pages_int2, desc->n_pages_int4, kappa, acc_ws, ml_ws, status
                       );
    return hipGetLastError() == hipSuccess ? TKV_OK : TKV_ERR_HIP;
}

int tkv_launch_decode_reduce(const tkv_desc *desc, const int32_t *seq_item_indptr, int32_t n_items, int32_t batch,
                             int32_t n_q_heads, float *out, const void *workspace, void *stream)
{
    (void)desc;
    const float *acc_ws = (const float *)workspace;
    const float *ml_ws = acc_ws + (size_t)n_items * n_q_heads * kHeadDim;
    // the item counts are on the device; the average per sequence picks the shape of the reduction
    if ((int64_t)n_items > 128 * (int64_t)batch)
        hipLaunchKernelGGL(tkv_reduce_kernel<16>, dim3((unsigned)(batch * n_q_heads * (kHeadDim / 16))), dim3(kReduceThreads), 0,
                           (hipStream_t)stream, acc_ws, ml_ws, seq_item_indptr, n_q_heads, out);
    else
        hipLaunchKernelGGL(tkv_reduce_kernel<128>, dim3((unsigned)(batch * n_q_heads)), dim3(kReduceThreads), 0,
                           (hipStream_t)stream, acc_ws, ml_ws, seq_item_indptr, n_q_heads, out);
    return hipGetLastError() == hipSuccess ? TKV_OK : TKV_ERR_HIP;
}

// ---- tkv_decode_attention_static: the same two launches with the partials in a file-scope device array ----
// For callers that cannot allocate (HIP graph capture, tight serving loops).  `scratch` is a host-side
// stand-in for the device array: its device address is looked up once per device and only that address
// is handed to kernels.
static __device__ __align__(256) unsigned char scratch[TKV_DECODE_STATIC_SCRATCH_BYTES];

namespace {
constexpr int kMaxDevices = 64;
std::mutex g_scratch_mutex;
void *g_scratch_ptr[kMaxDevices];   // device address of `scratch` on each device, null until first use there

// Device address of this device's copy of `scratch` (the current device), or null on failure.
void *scratch_address()
{
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return nullptr;
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
        void *p = nullptr;
        if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess) {
            (void)hipGetLastError();
            return nullptr;
        }
        g_scratch_ptr[dev] = p;
    }
    return g_scratch_ptr[dev];
}
} // namespace

extern "C" int tkv_decode_attention_static(const tkv_desc *desc, const void *pool, const uint8_t *bit_map,
                                           const void *q, const int32_t *page_indptr, const int32_t *page_ids,
                                           const int32_t *n_tok_int2, const int32_t *n_tok_int4,
                                           const int32_t *items, const int32_t *seq_item_indptr, int32_t n_items,
                                           int32_t batch, int32_t n_q_heads, float sm_scale, float *out,
                                           int32_t *status, void *stream)
{
    // the argument checks of tkv_decode_attention, with the fixed array as the workspace
    const size_t need = tkv_decode_workspace_bytes(desc, n_items, n_q_heads);
    if (desc && n_items > 0 && n_q_heads > 0 && need == 0) return TKV_ERR_BAD_SHAPE;
    if (need > (size_t)TKV_DECODE_STATIC_SCRATCH_BYTES) return TKV_ERR_WORKSPACE_TOO_SMALL;
    alignas(16) static const char placeholder[16] = {0};   // stands for the workspace in the host-side checks (non-null, aligned)
    if (int st = tkv_decode_check_args(desc, n_items, batch, n_q_heads, placeholder, TKV_DECODE_STATIC_SCRATCH_BYTES)) return st;
    if (batch == 0) return TKV_OK;
    if (!(sm_scale > 0.0f) || !(sm_scale < 3.0e38f)) return TKV_ERR_INVALID_ARG;
    if (!q || !out || !page_indptr || !n_tok_int2 || !n_tok_int4 || !seq_item_indptr) return TKV_ERR_INVALID_ARG;
    if (n_items > 0 && (!pool || !bit_map || !page_ids || !items)) return TKV_ERR_INVALID_ARG;
    if (((uintptr_t)pool & 255) || ((uintptr_t)q & 15) || ((uintptr_t)out & 15)) return TKV_ERR_INVALID_ARG;
    void *ws = scratch_address();
    if (!ws) return TKV_ERR_HIP;
    // every partial the reduction reads is written by the split kernel of this call: nothing to clear
    if (int st = tkv_launch_decode_split(desc, pool, bit_map, q, page_indptr, page_ids, n_tok_int2, n_tok_int4, items,
                                         n_items, batch, n_q_heads, sm_scale, ws, status, stream))
        return st;
    return tkv_launch_decode_reduce(desc, seq_item_indptr, n_items, batch, n_q_heads, out, ws, stream);
}
