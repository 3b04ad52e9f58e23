// tkv_decode_attention: split-K flash-decoding over the paged INT2 / INT4 KV
// pool with in-register dequantisation, and the cross-split reduction
// (paper Sec. 3.2.3 "Decode": KV processed as parallel contiguous splits,
// each running one dequantisation path, merged by online log-sum-exp).
//
// One wavefront owns one (work item, kv head): a contiguous range of one
// sequence's page list.  All query heads that share the kv head (up to 8)
// are processed together so the packed KV bytes are read from HBM once.
//
// Matrix cores do both contractions (v_mfma_f32_16x16x32_f16), fp32 accumulate:
//
//   QK^T  D[token, head] = sum_c code[token, c] * q[head, c]   one MFMA per
//         (16-token tile, group of 32 channels).  The codes enter the MFMA as
//         fp16 SUBNORMALS: a masked 16-bit field with the code in its low ten
//         bits *is* the fp16 number code * 2^(shift-24), so unpacking is one
//         AND per two codes.  q is converted to fp16 once, scaled by a power
//         of two (exact) and by 2^-shift per slot, and the K scale (fp32,
//         times the compensating power of two) multiplies the MFMA result.
//         The zero-point term sum_g zero[token,g] * sum_{c in g} q[head,c]
//         is one more MFMA whose A operand is the stored fp16 zero plane.
//   PV    D[head, channel] = sum_token P[head, token] * (code * scale)[token, channel]
//         P is split into two fp16 pieces (hi, lo) that occupy the 16 MFMA
//         rows (8 heads x 2 pieces); code*scale is formed exactly in fp16 as
//         two pieces as well (scale = 7-bit piece + remainder).  The zero
//         term sum_token P * zero and the softmax denominator come from one
//         extra MFMA against the staged zero plane and a column of constants.
//
// Every product the MFMAs see is exact; the only rounding is fp32
// accumulation, the fp32 K-scale multiply and the 22-bit split of P.
#include <hip/hip_runtime.h>
#include <hip/hip_fp16.h>

#include "tkv_internal.h"
#include "tkv_layout.h"

namespace {

using namespace tkv;

typedef _Float16 half8 __attribute__((ext_vector_type(8)));
typedef _Float16 half2_t __attribute__((ext_vector_type(2)));
typedef float floatx4 __attribute__((ext_vector_type(4)));
typedef uint32_t uint4v __attribute__((ext_vector_type(4)));

#ifndef TKV_WAVES_PER_EU
#define TKV_WAVES_PER_EU 2
#endif

constexpr float kTau = 4.0f;       // rescale when a logit exceeds the reference maximum by this much (log2 units)
constexpr float kOBase = 1.0f;     // common power-of-two factor on P: P = p * 2^(kOBase + o_slot)

__device__ __forceinline__ half8 as_half8(uint32_t a, uint32_t b, uint32_t c, uint32_t d)
{
    uint4v v = {a, b, c, d};
    return __builtin_bit_cast(half8, v);
}
__device__ __forceinline__ uint32_t pk_fma(uint32_t x, uint32_t s)   // (x - 1) * s per fp16 half, one rounding
{
    const half2_t xv = __builtin_bit_cast(half2_t, x), sv = __builtin_bit_cast(half2_t, s);
    const half2_t r = __builtin_elementwise_fma(xv, sv, -sv);
    return __builtin_bit_cast(uint32_t, r);
}
// (x & mask) | orv in one VALU op
__device__ __forceinline__ uint32_t and_or(uint32_t x, uint32_t mask, uint32_t orv)
{
    uint32_t r;
    asm("v_and_or_b32 %0, %1, %2, %3" : "=v"(r) : "v"(x), "s"(mask), "v"(orv));
    return r;
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
// negk = -1 the next 11 bits of the remainder.
__device__ __forceinline__ uint32_t p_piece(float p0, float p1, float negk)
{
    const uint32_t t2 = __builtin_bit_cast(uint32_t, __builtin_amdgcn_cvt_pkrtz(p0, p1));
    const float r0 = residual<0>(t2, negk, p0), r1 = residual<1>(t2, negk, p1);
    return __builtin_bit_cast(uint32_t, __builtin_amdgcn_cvt_pkrtz(r0, r1));
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
__device__ __forceinline__ float wave_max(float v)
{
#pragma unroll
    for (int o = 32; o; o >>= 1) v = fmaxf(v, __shfl_xor(v, o));
    return v;
}

// log2 of the power-of-two factor carried by slot j of the V operand
template <int BITS> __device__ __forceinline__ constexpr int o_slot(int j)
{
    return BITS == 4 ? ((j & 2) ? 6 : 10) : 10 - 2 * (j >> 1);
}

struct WaveState {
    floatx4 acc[8];     // PV accumulators: tile jt (16 channels) x rows (4*q4 + i)
    floatx4 zacc;       // zero-term (cols 0..3 = groups) and denominator (col 4)
    float m_ref;        // reference maximum of this lane's head column, log2 units, -inf before the first page
};

struct alignas(16) Lds {
    alignas(16) float ks[kPageTokens * kGroups];          // K scale * F, fp32 [token][group]
    alignas(16) uint32_t vs_hi[kPageTokens * kGroups / 2];  // V scale, 7-bit piece, fp16 pairs in plane order
    alignas(16) uint32_t vs_lo[kPageTokens * kGroups / 2];  // V scale, remainder
    alignas(16) uint32_t vz[kPageTokens * kGroups / 2];     // V zero * 2^-o_slot
    alignas(16) float alpha[16];
    alignas(16) float zl[16][8];
};

// B operand of the QK^T MFMAs for one width: per group, 4 registers of fp16
// pairs holding q' = q * 2^E * 2^-shift in the slot order the unpack produces.
struct QOperand { uint32_t r[4][4]; };

template <int BITS>
__device__ __forceinline__ void build_q_operand(const float *qf /* this lane's head, 128 floats in LDS */, int q4,
                                               float two_e, QOperand &qo)
{
#pragma unroll
    for (int g = 0; g < 4; ++g)
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
                // registers: (crumb 4*sub+k, crumb 8+4*sub+k) * 4^k of the 16-channel word q4/2
                c0 = 32 * g + 16 * (q4 >> 1) + 4 * (q4 & 1) + k;
                c1 = c0 + 8;
                f = 1.0f / (float)(1 << (2 * k));
            }
            qo.r[g][k] = pack_h2(qf[c0] * two_e * f, qf[c1] * two_e * f);
        }
}

// Everything one wavefront loads for one (page, kv head) record.
template <int BITS> struct PageRegs {
    uint4 kw[4];          // K codes: one 16-byte chunk per 16-token tile (four groups of this lane's channel slice)
    uint4 vw[BITS];       // V codes: 16-byte chunks, one word per 16-channel tile
    uint2 ksc, vsc, vzc;  // this lane's four entries of the K scale / V scale / V zero planes
    uint2 kz[4];          // K zero of token 16*e + lane%16, four groups
    uint32_t bm;          // bit_map entry of the page
};

template <int BITS>
__device__ __forceinline__ void load_page(PageRegs<BITS> &pr, const uint8_t *__restrict__ rec,
                                          const uint8_t *__restrict__ bit_map, int page, int lane)
{
    using R = Rec<BITS>;
    const int r16 = lane & 15, q4 = lane >> 4;
    const uint4 *kc = reinterpret_cast<const uint4 *>(rec + R::kKCodes);
    const uint4 *vc = reinterpret_cast<const uint4 *>(rec + R::kVCodes);
#pragma unroll
    for (int e = 0; e < 4; ++e)
        pr.kw[e] = BITS == 4 ? kc[e * 64 + lane] : kc[e * 32 + (q4 >> 1) * 16 + r16];
#pragma unroll
    for (int i = 0; i < BITS; ++i) pr.vw[i] = vc[i * 64 + lane];
    pr.ksc = reinterpret_cast<const uint2 *>(rec + R::kKScale)[lane];
    pr.vsc = reinterpret_cast<const uint2 *>(rec + R::kVScale)[lane];
    pr.vzc = reinterpret_cast<const uint2 *>(rec + R::kVZero)[lane];
#pragma unroll
    for (int e = 0; e < 4; ++e) pr.kz[e] = reinterpret_cast<const uint2 *>(rec + R::kKZero)[16 * e + r16];
    pr.bm = bit_map[page];
}

template <int BITS>
__device__ __forceinline__ void compute_page(const PageRegs<BITS> &pr, int n_valid, int lane,
                                             const QOperand &qo, half8 qz, float F, float kappa,
                                             float negk, WaveState &st, Lds &lds)
{
    const int r16 = lane & 15, q4 = lane >> 4;

    // ---- stage metadata in LDS --------------------------------------------
    __syncthreads();   // previous page's readers are done
    {
        // Tokens at or beyond n_valid (never-written slots of a partly filled page) are masked by count,
        // never by content: their K scale and K zero become 0 and -inf is added to their logits below;
        // their V scale and V zero become 0 (their P is 0, the product must not be NaN).  Full pages
        // run the same instructions with all-ones masks.
        uint2 vsc = pr.vsc, vzc = pr.vzc;
        const half2_t a = __builtin_bit_cast(half2_t, pr.ksc.x), b = __builtin_bit_cast(half2_t, pr.ksc.y);
        const float fk = lane < n_valid ? F : 0.0f;
        reinterpret_cast<float4 *>(lds.ks)[lane] = lane < n_valid
            ? make_float4((float)a[0] * fk, (float)a[1] * fk, (float)b[0] * fk, (float)b[1] * fk)
            : make_float4(0.f, 0.f, 0.f, 0.f);
        // this lane holds plane entries 4*lane .. 4*lane+3: chunk lane/2, slots 4*(lane&1) + 0..3
        {
            const int chunk = lane >> 1, blk = chunk >> 4, quad = (chunk >> 2) & 3, jb = 4 * (lane & 1);
            const int t0 = 32 * blk + 16 * (jb >> 2) + 4 * quad;   // tokens t0 .. t0+3
            const uint32_t m01 = (t0 < n_valid ? 0xffffu : 0u) | (t0 + 1 < n_valid ? 0xffff0000u : 0u);
            const uint32_t m23 = (t0 + 2 < n_valid ? 0xffffu : 0u) | (t0 + 3 < n_valid ? 0xffff0000u : 0u);
            vsc.x &= m01; vsc.y &= m23; vzc.x &= m01; vzc.y &= m23;
        }
        const uint32_t hx = vsc.x & 0xfff0fff0u, hy = vsc.y & 0xfff0fff0u;
        const half2_t lx = __builtin_bit_cast(half2_t, vsc.x) - __builtin_bit_cast(half2_t, hx);
        const half2_t ly = __builtin_bit_cast(half2_t, vsc.y) - __builtin_bit_cast(half2_t, hy);
        reinterpret_cast<uint2 *>(lds.vs_hi)[lane] = make_uint2(hx, hy);
        reinterpret_cast<uint2 *>(lds.vs_lo)[lane] =
            make_uint2(__builtin_bit_cast(uint32_t, lx), __builtin_bit_cast(uint32_t, ly));
        // zero plane times 2^-o_slot: slots 4*(lane&1)+{0,1} and +{2,3}
        const int j0 = 4 * (lane & 1);
        float f01, f23;
        if (BITS == 4) { f01 = 0x1p-10f; f23 = 0x1p-6f; }
        else { f01 = j0 ? 0x1p-6f : 0x1p-10f; f23 = j0 ? 0x1p-4f : 0x1p-8f; }
        const half2_t z01 = __builtin_bit_cast(half2_t, vzc.x) * (_Float16)f01;
        const half2_t z23 = __builtin_bit_cast(half2_t, vzc.y) * (_Float16)f23;
        reinterpret_cast<uint2 *>(lds.vz)[lane] =
            make_uint2(__builtin_bit_cast(uint32_t, z01), __builtin_bit_cast(uint32_t, z23));
    }
    __syncthreads();

    // ---- QK^T: S[e][i] = q . k_hat (unscaled) for token 16e + 4*q4 + i, head column r16
    floatx4 S[4];
#pragma unroll
    for (int e = 0; e < 4; ++e) {
        // zero-point term; slot 4 of channel-slice 1 carries the token's mask bias (0 or -inf) against a 1.0 in q's operand
        const bool tok_ok = 16 * e + r16 < n_valid;
        const uint32_t z01 = tok_ok ? pr.kz[e].x : 0u, z23 = tok_ok ? pr.kz[e].y : 0u;
        const uint32_t biased = (z01 & 0xffff0000u) | (tok_ok ? 0u : 0xfc00u);
        const half8 za = as_half8(z01, z23, q4 == 1 ? biased : z01, z23);
        floatx4 s = mfma(za, qz, floatx4{0.f, 0.f, 0.f, 0.f});
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
                const uint32_t ws = w[g] >> (8 * (q4 & 1));
                a = as_half8(ws & 0x00030003u, ws & 0x000c000cu, ws & 0x00300030u, ws & 0x00c000c0u);
            }
            const half8 b = as_half8(qo.r[g][0], qo.r[g][1], qo.r[g][2], qo.r[g][3]);
            const floatx4 p = mfma(a, b, floatx4{0.f, 0.f, 0.f, 0.f});
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const float scg = g == 0 ? sc[i].x : g == 1 ? sc[i].y : g == 2 ? sc[i].z : sc[i].w;
                s[i] = fmaf(scg, p[i], s[i]);
            }
        }
        S[e] = s;
    }

    // ---- online softmax with a lazily updated reference maximum ------------
    float mx = fmaxf(fmaxf(S[0][0], S[0][1]), fmaxf(S[0][2], S[0][3]));
#pragma unroll
    for (int e = 1; e < 4; ++e) mx = fmaxf(fmaxf(mx, S[e][0]), fmaxf(fmaxf(S[e][1], S[e][2]), S[e][3]));
    mx = fmaxf(mx, __shfl_xor(mx, 16));
    mx = fmaxf(mx, __shfl_xor(mx, 32));
    mx *= kappa;   // log2 units
    if (__any(mx > st.m_ref + kTau)) {
        const float m_new = fmaxf(st.m_ref, mx);
        const float alpha = m_new == -INFINITY ? 1.0f : __builtin_amdgcn_exp2f(st.m_ref - m_new);
        st.m_ref = m_new;
        __syncthreads();
        if (q4 == 0) lds.alpha[r16] = alpha;
        __syncthreads();
        const float4 al = reinterpret_cast<const float4 *>(lds.alpha)[q4];   // rows 4*q4 .. 4*q4+3
        const floatx4 av = {al.x, al.y, al.z, al.w};
#pragma unroll
        for (int jt = 0; jt < 8; ++jt) st.acc[jt] *= av;
        st.zacc *= av;
    }
    const float mref = st.m_ref == -INFINITY ? 0.0f : st.m_ref;
    uint32_t pa[2][4];   // A operand of the two PV contraction blocks
#pragma unroll
    for (int e = 0; e < 4; ++e) {
        float pv[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int j = 4 * (e & 1) + i;
            const float off = (kOBase + (float)o_slot<BITS>(j)) - mref;
            pv[i] = __builtin_amdgcn_exp2f(fmaf(S[e][i], kappa, off));
        }
        pa[e >> 1][2 * (e & 1)] = p_piece(pv[0], pv[1], negk);
        pa[e >> 1][2 * (e & 1) + 1] = p_piece(pv[2], pv[3], negk);
    }

    // ---- PV ------------------------------------------------------------------
    constexpr uint32_t kOne = 0x3c003c00u;
    uint32_t one = kOne;
    asm volatile("" : "+v"(one));   // keep the constant in a VGPR (operand of v_and_or_b32)
#pragma unroll
    for (int blk = 0; blk < 2; ++blk) {
        const half8 p8 = as_half8(pa[blk][0], pa[blk][1], pa[blk][2], pa[blk][3]);
        // zero term and denominator: columns 0..3 = groups, column 4 = constants 2^-o_slot
        {
            uint4 bz = reinterpret_cast<const uint4 *>(lds.vz)[(blk * 4 + q4) * 4 + (r16 & 3)];
            if (r16 >= 4) {
                if (BITS == 4) bz = make_uint4(0x14001400u, 0x24002400u, 0x14001400u, 0x24002400u);   // 2^-10, 2^-6
                else bz = make_uint4(0x14001400u, 0x1c001c00u, 0x24002400u, 0x2c002c00u);           // 2^-10 .. 2^-4
            }
            st.zacc = mfma(p8, as_half8(bz.x, bz.y, bz.z, bz.w), st.zacc);
        }
#pragma unroll
        for (int g = 0; g < 4; ++g) {
            const uint4 shi = reinterpret_cast<const uint4 *>(lds.vs_hi)[(blk * 4 + q4) * 4 + g];
            const uint4 slo = reinterpret_cast<const uint4 *>(lds.vs_lo)[(blk * 4 + q4) * 4 + g];
#pragma unroll
            for (int t2 = 0; t2 < 2; ++t2) {
                const int jt = 2 * g + t2;
                uint32_t w;
                {
                    const uint4 v = BITS == 4 ? pr.vw[blk * 2 + (jt >> 2)] : pr.vw[jt >> 2];
                    w = (jt & 3) == 0 ? v.x : (jt & 3) == 1 ? v.y : (jt & 3) == 2 ? v.z : v.w;
                }
                uint32_t x[4];
                if (BITS == 4) {
                    const uint32_t w8 = w >> 8;
                    x[0] = and_or(w, 0x000f000fu, one); x[1] = and_or(w, 0x00f000f0u, one);
                    x[2] = and_or(w8, 0x000f000fu, one); x[3] = and_or(w8, 0x00f000f0u, one);
                } else {
                    const uint32_t ws = blk ? (w >> 8) : w;
                    x[0] = and_or(ws, 0x00030003u, one); x[1] = and_or(ws, 0x000c000cu, one);
                    x[2] = and_or(ws, 0x00300030u, one); x[3] = and_or(ws, 0x00c000c0u, one);
                }
                const half8 bh = as_half8(pk_fma(x[0], shi.x), pk_fma(x[1], shi.y), pk_fma(x[2], shi.z), pk_fma(x[3], shi.w));
                const half8 bl = as_half8(pk_fma(x[0], slo.x), pk_fma(x[1], slo.y), pk_fma(x[2], slo.z), pk_fma(x[3], slo.w));
                st.acc[jt] = mfma(p8, bh, st.acc[jt]);
                st.acc[jt] = mfma(p8, bl, st.acc[jt]);
            }
        }
    }
}

// All pages [pb, pe) of one width (indices into the sequence's page list).
template <int BITS>
__device__ __forceinline__ void run_pages(const uint8_t *__restrict__ pool, const uint8_t *__restrict__ bit_map,
                                          const int32_t *__restrict__ pages, int pb, int pe, int last_index,
                                          int last_valid, int page_lo, int page_hi, int n_pages_total, int kvh,
                                          int n_kv_heads, int n_pages_int2, int lane, const QOperand &qo, half8 qz,
                                          float F, float kappa, float negk, WaveState &st, Lds &lds, int32_t *status)
{
    // Issue the loads of list position pi into pr and return its number of valid tokens.  A page id
    // outside its pool cannot be addressed: it is flagged, a valid page is read instead and masked out.
    auto fetch = [&](int pi, PageRegs<BITS> &pr) -> int {
        int page = __builtin_amdgcn_readfirstlane(pages[pi]);
        const bool ok = page >= page_lo && page < page_hi;
        if (!ok) {
            if (status && lane == 0)
                atomicOr(status, page < 0 || page >= n_pages_total ? TKV_STATUS_PAGE_RANGE : TKV_STATUS_BITMAP_MISMATCH);
            page = page_lo;
        }
        load_page<BITS>(pr, pool + record_offset(page, kvh, n_kv_heads, n_pages_int2), bit_map, page, lane);
        return ok ? (pi == last_index ? last_valid : kPageTokens) : 0;
    };
    // the bit_map entry arrives with the page: a mismatch masks the whole page
    auto step = [&](const PageRegs<BITS> &pr, int nv) {
        if (pr.bm != BITS && nv > 0) {
            if (status && lane == 0) atomicOr(status, TKV_STATUS_BITMAP_MISMATCH);
            nv = 0;
        }
        compute_page<BITS>(pr, nv, lane, qo, qz, F, kappa, negk, st, lds);
    };
    // Two register sets: while one page is computed the loads of the next are in flight.
    PageRegs<BITS> cur, nxt;
    int nv = fetch(pb, cur), nv_next = 0;
    nxt = cur;
    for (int pi = pb; pi < pe; ++pi) {
        if (pi + 1 < pe) nv_next = fetch(pi + 1, nxt);
        step(cur, nv);
        cur = nxt;
        nv = nv_next;
    }
}

__global__ __launch_bounds__(64) __attribute__((amdgpu_waves_per_eu(TKV_WAVES_PER_EU, TKV_WAVES_PER_EU))) void tkv_decode_kernel(
    const uint8_t *__restrict__ pool, const uint8_t *__restrict__ bit_map, const uint16_t *__restrict__ q,
    const int32_t *__restrict__ page_indptr, const int32_t *__restrict__ page_ids,
    const int32_t *__restrict__ n_tok_int2, const int32_t *__restrict__ n_tok_int4,
    const int32_t *__restrict__ items, int batch, int n_kv_heads, int n_q_heads, int n_pages_int2, int n_pages_int4,
    float kappa, float *__restrict__ acc_ws, float *__restrict__ ml_ws, int32_t *status)
{
    __shared__ Lds lds;
    __shared__ float qf[8][kHeadDim];
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
    float amax = 0.0f;
    for (int idx = lane; idx < R * kHeadDim; idx += 64) {
        const int h = idx / kHeadDim, c = idx % kHeadDim;
        const float v = __uint_as_float((uint32_t)q[((size_t)seq * n_q_heads + kvh * R + h) * kHeadDim + c] << 16);
        qf[h][c] = v;
        amax = fmaxf(amax, fabsf(v));
    }
    amax = wave_max(amax);
    // 2^E with max|q| * 2^E in [2^14, 2^15); E clamped so every factor stays a normal fp32
    int ex = 0;
    if (amax > 0.0f) { (void)frexpf(amax, &ex); }   // amax = m * 2^ex, m in [0.5, 1)
    int E = 15 - ex;
    E = E > 100 ? 100 : (E < -100 ? -100 : E);
    const float two_e = ldexpf(1.0f, amax > 0.0f ? E : 0);
    const float F = ldexpf(1.0f, 24 - (amax > 0.0f ? E : 0));
    __syncthreads();
    const int hcol = (r16 & 7) & (R - 1);   // head of this lane's column (columns beyond R repeat heads)
    const float negk = r16 >= 8 ? -1.0f : 0.0f;   // columns 8..15 carry the low piece of P
    half8 qz;
    {
        // Z-term B operand: slots 0..3 / 4..7 of chunk 0 = hi / mid pieces of the four group sums,
        // slots 0..3 of chunk 1 = lo pieces, everything else zero
        float pc[8] = {0, 0, 0, 0, 0, 0, 0, 0};
#pragma unroll
        for (int g = 0; g < 4; ++g) {
            double sum = 0.0;
            for (int c = 0; c < kGroup; ++c) sum += (double)qf[hcol][g * kGroup + c];
            const _Float16 hi = (_Float16)sum;
            const double r1 = sum - (double)(float)hi;
            const _Float16 mid = (_Float16)r1;
            const _Float16 lo = (_Float16)(r1 - (double)(float)mid);
            if (q4 == 0) { pc[g] = (float)hi; pc[4 + g] = (float)mid; }
            else if (q4 == 1) { pc[g] = (float)lo; }
        }
        if (q4 == 1) pc[4] = 1.0f;   // multiplies the mask bias of the token rows
        qz = as_half8(pack_h2(pc[0], pc[1]), pack_h2(pc[2], pc[3]), pack_h2(pc[4], pc[5]), pack_h2(pc[6], pc[7]));
    }

    WaveState st;
#pragma unroll
    for (int jt = 0; jt < 8; ++jt) st.acc[jt] = floatx4{0.f, 0.f, 0.f, 0.f};
    st.zacc = floatx4{0.f, 0.f, 0.f, 0.f};
    st.m_ref = -INFINITY;

    const int n_pages_total = n_pages_int2 + n_pages_int4;
    QOperand qo;
    // INT2 pages of the range, then INT4 pages: each page runs one dequantisation path
    const int e2 = pe < np2 ? pe : np2;
    if (pb < e2) {
        asm volatile("" ::: "memory");   // re-read q from LDS here instead of holding 128 values in registers
        build_q_operand<2>(qf[hcol], q4, two_e, qo);
        run_pages<2>(pool, bit_map, pages, pb, e2, np2 - 1, n2 - (np2 - 1) * kPageTokens, 0, n_pages_int2,
                     n_pages_total, kvh, n_kv_heads, n_pages_int2, lane, qo, qz, F, kappa, negk, st, lds, status);
    }
    const int b4 = pb > np2 ? pb : np2;
    if (b4 < pe) {
        asm volatile("" ::: "memory");
        build_q_operand<4>(qf[hcol], q4, two_e, qo);
        run_pages<4>(pool, bit_map, pages, b4, pe, np2 + np4 - 1, n4 - (np4 - 1) * kPageTokens, n_pages_int2,
                     n_pages_total, n_pages_total, kvh, n_kv_heads, n_pages_int2, lane, qo, qz, F, kappa, negk, st, lds,
                     status);
    }

    // ---- write the partial (m, l, acc) of this item ------------------------------
    // rows 0..7 carry the hi piece of P, rows 8..15 the lo piece: add lanes l and l^32
#pragma unroll
    for (int jt = 0; jt < 8; ++jt)
#pragma unroll
        for (int i = 0; i < 4; ++i) st.acc[jt][i] += __shfl_xor(st.acc[jt][i], 32);
#pragma unroll
    for (int i = 0; i < 4; ++i) st.zacc[i] += __shfl_xor(st.zacc[i], 32);
    __syncthreads();
    if (r16 < 8 && q4 < 2)
#pragma unroll
        for (int i = 0; i < 4; ++i) lds.zl[4 * q4 + i][r16] = st.zacc[i];   // [head row][column]
    if (q4 == 0 && r16 < 8) lds.alpha[r16] = st.m_ref;
    __syncthreads();
    if (q4 < 2) {
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int row = 4 * q4 + i;
            if (row >= R) continue;
            const size_t ph = (size_t)item * n_q_heads + kvh * R + row;
            float *dst = acc_ws + ph * kHeadDim;
#pragma unroll
            for (int jt = 0; jt < 8; ++jt) dst[16 * jt + r16] = st.acc[jt][i] + lds.zl[row][jt >> 1];
            if (r16 == 0) {
                ml_ws[2 * ph] = lds.alpha[row];
                ml_ws[2 * ph + 1] = lds.zl[row][4];
            }
        }
    }
}

// D7: out = sum_i 2^(m_i - M) acc_i / sum_i 2^(m_i - M) l_i over the items of a sequence.
// One workgroup per (sequence, query head): the items' maxima are reduced in parallel, the weights go
// to LDS, then four groups of 128 threads (one thread per channel) each sum every fourth item.
constexpr int kReduceParts = 4;
__global__ __launch_bounds__(kHeadDim * kReduceParts) void tkv_reduce_kernel(
    const float *__restrict__ acc_ws, const float *__restrict__ ml_ws, const int32_t *__restrict__ seq_item_indptr,
    int n_q_heads, float *__restrict__ out)
{
    constexpr int kThreads = kHeadDim * kReduceParts, kChunk = 512;
    __shared__ float w_s[kChunk];
    __shared__ float red[kThreads / 64];
    __shared__ float part_s[kReduceParts][kHeadDim];
    __shared__ float den_s[kReduceParts];
    const int b = blockIdx.x / n_q_heads, h = blockIdx.x % n_q_heads, tid = threadIdx.x;
    const int c = tid % kHeadDim, part = tid / kHeadDim;
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
            for (int k = part; k < n; k += kReduceParts) {
                const size_t ph = (size_t)(base + k) * n_q_heads + h;
                num = fmaf(w_s[k], acc_ws[ph * kHeadDim + c], num);
                if (c == 0) den = fmaf(w_s[k], ml_ws[2 * ph + 1], den);
            }
        }
    }
    part_s[part][c] = num;
    if (c == 0) den_s[part] = den;
    __syncthreads();
    if (part == 0) {
        float nsum = 0.0f, dsum = 0.0f;
#pragma unroll
        for (int k = 0; k < kReduceParts; ++k) { nsum += part_s[k][c]; dsum += den_s[k]; }
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
    hipLaunchKernelGGL(tkv_decode_kernel, dim3((unsigned)(n_items * desc->n_kv_heads)), dim3(64), 0,
                       (hipStream_t)stream, (const uint8_t *)pool, bit_map, (const uint16_t *)q, page_indptr,
                       page_ids, n_tok_int2, n_tok_int4, items, batch, desc->n_kv_heads, n_q_heads,
                       desc->n_pages_int2, desc->n_pages_int4, kappa, acc_ws, ml_ws, status);
    return hipGetLastError() == hipSuccess ? TKV_OK : TKV_ERR_HIP;
}

int tkv_launch_decode_reduce(const tkv_desc *desc, const int32_t *seq_item_indptr, int32_t n_items, int32_t batch,
                             int32_t n_q_heads, float *out, const void *workspace, void *stream)
{
    (void)desc;
    const float *acc_ws = (const float *)workspace;
    const float *ml_ws = acc_ws + (size_t)n_items * n_q_heads * kHeadDim;
    hipLaunchKernelGGL(tkv_reduce_kernel, dim3((unsigned)(batch * n_q_heads)), dim3(kHeadDim * kReduceParts), 0,
                       (hipStream_t)stream, acc_ws, ml_ws, seq_item_indptr, n_q_heads, out);
    return hipGetLastError() == hipSuccess ? TKV_OK : TKV_ERR_HIP;
}
