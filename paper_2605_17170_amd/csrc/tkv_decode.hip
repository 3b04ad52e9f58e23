// tkv_decode_attention: split-K flash-decoding over the paged INT2 / INT4 KV
// pool with in-register dequantisation, and the cross-split reduction
// (paper Sec. 3.2.3 "Decode").
//
// One wavefront owns one (work item, kv head): a contiguous range of one
// sequence's page list.  All query heads that share the kv head (up to 8)
// are processed together so the packed KV bytes are read from HBM once; the
// partials (m, l, acc) of the items are merged by tkv_reduce_rows_kernel.
//
// Matrix cores do both contractions (v_mfma_f32_16x16x32_f16), fp32 accumulate,
// and the packed codes are never expanded by arithmetic: a masked 16-bit field
// with a code in its low ten bits *is* the fp16 subnormal code * 2^(pos-24), so
// unpacking is one AND per two codes, for K and for V.
//
//   QK^T  D[token, head] = sum_c code[token, c] * q[head, c].  q is converted to fp16
//         once, scaled by a power of two (exact) and by 2^-pos per slot; the K scale
//         (fp32, times the compensating power of two) multiplies the MFMA result.  The
//         eight heads fill half of the 16 columns, so the columns carry two token sets:
//         row r of a 32-token block is token r in columns 0..7 and token 16 + r in
//         columns 8..15; an MFMA contracts half a group (16 channels) of both, the B
//         operand holding q in the k-slots of the column's own set and zeros in the
//         others.  Scale, exponential and weight pieces are then formed once per
//         (token, head).  The zero-point term sum_g zero[token,g] * sum_{c in g} q[head,c]
//         is one more MFMA per block whose A operand is the stored fp16 zero plane.
//         (Per-channel INT2 keys use the columns differently, see compute_page.)
//   PV    D[(head, half), channel] = sum_token a[head, token, g] * code[token, channel],
//         a = W * scale[token, g], W the softmax weight: the V scale multiplies the
//         weights, not the codes.  Rows 0..7 carry the weights of the heads for groups 0
//         and 1, rows 8..15 for groups 2 and 3; the 16 columns of an MFMA are 8 channels
//         of groups {0,1} and 8 channels of groups {2,3} (each lane loads its V words
//         accordingly), so every (head, token, group) product is formed once per
//         wavefront; the two cross quadrants of the result are never read.
//         The weights must be good to about 2^-17: a group with outlier channels has
//         |code * scale| and |zero| of tens that cancel, and the tolerance near zero is
//         2e-3.  W is therefore carried in two fp16 pieces (the leading 11 bits, then the
//         next 11), and a in two pieces as well: a_hi = fp16(W_hi * s), a_lo = W_lo * s +
//         the exact remainder of the hi product (packed fp16 FMAs); each V operand meets
//         both pieces (two MFMAs into the same accumulator).  The zero-point term
//         sum_t W * zero[t, g] and the softmax denominator sum_t W come from one more
//         pair of MFMAs per 32 tokens against the stored zero plane and a column of ones.
//
// Every product the MFMAs see is exact; the roundings are fp32 accumulation, the fp32
// K-scale multiply, the 22-bit softmax weight (common to numerator and denominator) and
// the two-piece a.
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
// Softmax weights are carried in fp16 as W = P * 2^kPExp (P <= 2^kTau), so that small weights stay clear
// of the fp16 subnormal grid; numerator and denominator share the factor.
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
// The value of the lane eight columns on in the same row of 16 lanes.  (In all DPP moves here every lane has a source;
// `bound_ctrl` says so to the compiler, which otherwise presets the destination register with a move of its own.)
__device__ __forceinline__ float row_ror8(float v)
{
    return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), 0x128 /* row_ror:8 */, 0xf, 0xf, true));
}
__device__ __forceinline__ uint32_t ror8_u32(uint32_t v)
{
    return (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x128 /* row_ror:8 */, 0xf, 0xf, true);
}
// The value of another lane of the same row of 16 lanes: CTRL is a DPP pattern under which every lane has a source.
template <int CTRL> __device__ __forceinline__ float row_dpp(float v)
{
    return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), CTRL, 0xf, 0xf, true));
}
// Sum / maximum over a row of 16 lanes, in every lane of the row: neighbours, pairs, quads, halves
// (quad_perm [1,0,3,2], quad_perm [2,3,0,1], row_half_mirror, row_mirror).
__device__ __forceinline__ float row_sum(float v)
{
    v += row_dpp<0xB1>(v);
    v += row_dpp<0x4E>(v);
    v += row_dpp<0x141>(v);
    v += row_dpp<0x140>(v);
    return v;
}
__device__ __forceinline__ float row_max(float v)
{
    v = fmaxf(v, row_dpp<0xB1>(v));
    v = fmaxf(v, row_dpp<0x4E>(v));
    v = fmaxf(v, row_dpp<0x141>(v));
    v = fmaxf(v, row_dpp<0x140>(v));
    return v;
}
__device__ __forceinline__ float wave_max(float v)
{
    v = row_max(v);
    const int b = __builtin_bit_cast(int, v);
    const float r0 = __builtin_bit_cast(float, __builtin_amdgcn_readlane(b, 0)), r1 = __builtin_bit_cast(float, __builtin_amdgcn_readlane(b, 16));
    const float r2 = __builtin_bit_cast(float, __builtin_amdgcn_readlane(b, 32)), r3 = __builtin_bit_cast(float, __builtin_amdgcn_readlane(b, 48));
    return fmaxf(fmaxf(r0, r1), fmaxf(r2, r3));
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
    // PV accumulators.  Lane (c = lane % 16, q4 = lane / 16) holds rows 4*q4 + i: head 4*(q4 & 1) + i of row half
    // q4 >> 1; its column of acc[chunk][comp] is channel 64*(c >> 3) + 16*comp + (chunk ? c ^ 8 : c) % 16.
    // Only the quadrants with q4 >> 1 == c >> 3 (row half = column half) are meaningful.
    floatx4 acc[2][4];
    floatx4 zp;         // sum_t W * zero[t, g] in columns 0..3 (groups), sum_t W in column 4
    uint32_t sat;       // non-zero once a staged scale was clamped (reported in the status word at the end)
    float m_ref;        // reference maximum of this lane's head column, log2 units, -inf before the first page
};

// q operands of the QK^T MFMAs with two token sets: per (group, half group) 16 entries (sub*8 + head) and two entries of
// zeros.  The 16 lanes that a 16-byte LDS read serves together hold eight lanes that read their own entries
// sub*8 .. sub*8+7 (32 consecutive banks) and eight that read zeros: the zero entry they use lies in the other 32
// banks (entry 16 for sub = 1, entry 24 for sub = 0; entries 17..23 are padding).
constexpr int kQyStride = 25, kQyZero0 = 24, kQyZero1 = 16;
constexpr int kPvZ = 0, kPvS = 32, kPvZero = 64, kPvOne = 65, kPvChunks = 66;

// What only one of the two kernels keeps in LDS: the staged q (per-token keys; the other kernel borrows the page
// staging area for it), the second q operand (per-channel INT2 keys).
template <bool KC> struct LdsExtra {
    alignas(16) _Float16 qf[8][kHeadDim + 8];            // q * 2^E per head and channel (qf_chunk), kept for the whole item
};
template <> struct LdsExtra<true> {
    alignas(16) uint4 qp[kGroups][64];                   // q * 2^E in the slot order of qo, without the slot factors
};
template <bool KC> struct alignas(16) Lds : LdsExtra<KC> {
    // Per-channel INT2 keys reuse ks and kz while INT2 pages run: ks holds the K scale plane (512 B) and the
    // K zero plane (512 B) of the page as stored, kz a plane of zeros (the INT4 pages, which come later in
    // an item, overwrite all three with their own staging).
    alignas(16) float ks[kPageTokens * kGroups];         // K scale * F, fp32 [token][group]
    // Operands of the PV phase, 16-byte chunks of eight fp16 (the tokens of one k-slot octet), one array so that
    // a lane-dependent index can choose between staged data and the constants:
    //   kPvZ + (blk*4 + quad)*4 + g   V zero, as stored
    //   kPvS + (blk*4 + quad)*4 + g   V scale * 2^(kVExp - pos)
    //   kPvZero   zeros;   kPvOne   ones
    alignas(16) uint4 pv[kPvChunks];
    // K zero, four fp16 per token (per-channel INT2 keys, which also use it as a plane of zeros; otherwise the K
    // zeros travel between lanes without a copy in LDS)
    alignas(16) uint2 kz[KC ? kPageTokens : 2];
    // B operands of the QK^T MFMAs: per group and lane (per-channel INT2 keys), or 8 x (16 entries + zeros) (build_q_operand)
    alignas(16) uint4 qo[KC ? kGroups : 2][KC ? 64 : 4 * kQyStride];
    alignas(16) float alpha[16];
    // [head][8] floats of the prologue (group sums of q) and the epilogue (zero-point sums, denominator): the q
    // operands are not live then
    __device__ __forceinline__ float (*zl())[8] { return reinterpret_cast<float(*)[8]>(qo); }
    __device__ __forceinline__ uint4 *kc_scale() { return reinterpret_cast<uint4 *>(ks); }
    __device__ __forceinline__ uint4 *kc_zero() { return reinterpret_cast<uint4 *>(ks) + 32; }
    __device__ __forceinline__ uint4 *kc_nil() { return reinterpret_cast<uint4 *>(kz); }
};

// q * 2^E is staged in LDS as fp16 [head][128 channels].  The operand build reads the same channels of all eight
// heads at once; with plain 256-byte rows those reads would all fall on the same banks.  The kernel for per-token
// keys, which has the room, makes the rows 272 bytes long; the kernel for per-channel INT2 keys keeps 256-byte rows
// (the staging area it borrows holds no more) and stores the 16-byte chunks of a row at chunk ^ head instead.
// Byte offset of 16-byte chunk `chunk` (8 channels) of head `h`:
template <bool KC> __device__ __forceinline__ int qf_chunk(int h, int chunk)
{
    return KC ? h * 256 + ((chunk ^ h) << 4) : h * 272 + (chunk << 4);
}
// lane l of a wavefront holds channels 2l, 2l+1 of a head as an fp16 pair
template <bool KC> __device__ __forceinline__ void qf_store(void *qf, int h, int lane, uint32_t pair)
{
    *reinterpret_cast<uint32_t *>(static_cast<char *>(qf) + qf_chunk<KC>(h, lane >> 2) + ((lane & 3) << 2)) = pair;
}

// B operand of the QK^T MFMAs for one width, kept in LDS: 4 registers of fp16 pairs holding
// q' = q * 2^E * 2^-pos in the slot order the unpack produces.
//  - per-channel INT2 keys: per group and lane (head columns 8..15 repeat heads 0..7), plus the copy without
//    slot factors;
//  - otherwise (two token sets, see compute_page): per (group, half group) one entry per (channel octet sub,
//    head) and an entry of zeros, which the lanes whose k-slots belong to the other token set read.
// The slot factors are powers of two and q * 2^E has 8 significant bits: the fp16 products are exact unless they
// fall into the subnormals, where they round once.
template <int BITS, bool KC>
__device__ __forceinline__ void build_q_operand(const void *qf /* the staged q (qf_chunk) */, int h /* this lane's head */,
                                               int q4, int lane, Lds<KC> &lds)
{
    const char *qb = static_cast<const char *>(qf);
    // INT2 words: registers (crumb 4*sub+k, crumb 8+4*sub+k) * 2^-(2k+3), k = 0..3, of 16-channel word hg of a group
    auto int2_pairs = [&](int g, int hg, int sub, uint32_t (&pr)[4]) {
        const uint2 x = *reinterpret_cast<const uint2 *>(qb + qf_chunk<KC>(h, g * 4 + 2 * hg) + 8 * sub);       // channels 4*sub + 0..3
        const uint2 y = *reinterpret_cast<const uint2 *>(qb + qf_chunk<KC>(h, g * 4 + 2 * hg + 1) + 8 * sub);   // channels 8 + 4*sub + 0..3
        pr[0] = __builtin_amdgcn_perm(y.x, x.x, 0x05040100u);
        pr[1] = __builtin_amdgcn_perm(y.x, x.x, 0x07060302u);
        pr[2] = __builtin_amdgcn_perm(y.y, x.y, 0x05040100u);
        pr[3] = __builtin_amdgcn_perm(y.y, x.y, 0x07060302u);
    };
    constexpr uint32_t kSlot2[4] = {0x30003000u, 0x28002800u, 0x20002000u, 0x18001800u};   // fp16 2^-3, 2^-5, 2^-7, 2^-9 twice
    if constexpr (KC && BITS == 2) {
#pragma unroll
        for (int g = 0; g < 4; ++g) {
            uint32_t rp[4];
            int2_pairs(g, q4 >> 1, q4 & 1, rp);   // the unpack leaves the field of slot k at bit 2k + 3 (see compute_page)
            lds.qo[g][lane] = make_uint4(pk_mul(rp[0], kSlot2[0]), pk_mul(rp[1], kSlot2[1]), pk_mul(rp[2], kSlot2[2]), pk_mul(rp[3], kSlot2[3]));
            lds.qp[g][lane] = make_uint4(rp[0], rp[1], rp[2], rp[3]);
        }
    } else {
        uint4 *qy = reinterpret_cast<uint4 *>(lds.qo);
        const int sub = q4 & 1, ent = sub * 8 + (lane & 7);   // lanes that differ in lane & 8 or q4 & 2 write the same entry
#pragma unroll
        for (int g = 0; g < 4; ++g)
#pragma unroll
            for (int hg = 0; hg < 2; ++hg) {
                uint32_t r[4];
                if (BITS == 4) {
                    // registers: (n0,n4) (n1,n5)/16 (n2,n6) (n3,n7)/16 of the 8-channel word 2*hg + sub of the group
                    const uint4 c = *reinterpret_cast<const uint4 *>(qb + qf_chunk<KC>(h, g * 4 + 2 * hg + sub));   // channels (0,1) (2,3) (4,5) (6,7)
                    r[0] = __builtin_amdgcn_perm(c.z, c.x, 0x05040100u);
                    r[1] = pk_mul(__builtin_amdgcn_perm(c.z, c.x, 0x07060302u), 0x2c002c00u);
                    r[2] = __builtin_amdgcn_perm(c.w, c.y, 0x05040100u);
                    r[3] = pk_mul(__builtin_amdgcn_perm(c.w, c.y, 0x07060302u), 0x2c002c00u);
                } else {
                    int2_pairs(g, hg, sub, r);
#pragma unroll
                    for (int k = 0; k < 4; ++k) r[k] = pk_mul(r[k], kSlot2[k]);
                }
                qy[(g * 2 + hg) * kQyStride + ent] = make_uint4(r[0], r[1], r[2], r[3]);
            }
        if (lane < 16) qy[(lane & 7) * kQyStride + (lane < 8 ? kQyZero0 : kQyZero1)] = make_uint4(0u, 0u, 0u, 0u);
    }
}

// Everything one wavefront loads for one (page, kv head) record.
template <int BITS> struct PageRegs {
    uint4 kw[4];          // K codes, 16-byte chunks of four group words: [blk*2 + half group] of this lane's token (two token
                          // sets), or one per 16-token tile (per-channel INT2 keys)
    uint4 vw[BITS];       // V codes: 16-byte chunks, one word per 16-channel tile; [blk*2 + chunk] (INT4), [chunk] (INT2)
    uint2 ksc, vsc, vzc;  // this lane's four entries of the K scale / V scale / V zero planes
    uint2 kzc;            // K zero of token `lane`, four groups
    uint32_t bm;          // bit_map entry of the page
};

// The loads of one record come in two parts, issued as soon as the registers they land in are free: the
// metadata planes and the K codes after the QK^T phase of the previous page, the V codes after its PV phase.
template <int BITS>
__device__ __forceinline__ void load_page_meta(PageRegs<BITS> &pr, const uint8_t *__restrict__ rec,
                                               const uint8_t *__restrict__ bit_map, int page, int lane, int opaque_zero)
{
    using R = Rec<BITS>;
    pr.ksc = reinterpret_cast<const uint2 *>(rec + R::kKScale)[lane];
    pr.vsc = reinterpret_cast<const uint2 *>(rec + R::kVScale)[lane];
    pr.vzc = reinterpret_cast<const uint2 *>(rec + R::kVZero)[lane];
    // `opaque_zero` is 0 in a register the compiler cannot see through: the load stays a per-lane load whose
    // result is waited for where it is used, not a scalar value that is fetched back right behind the request
    pr.bm = bit_map[page + opaque_zero];
    pr.kzc = reinterpret_cast<const uint2 *>(rec + R::kKZero)[lane];
}
// Index (16-byte chunks) of part i of this lane's K codes / V codes in the record's code plane.
template <int BITS, bool KC> __device__ __forceinline__ int kcode_chunk(int i, int lane)
{
    const int r16 = lane & 15, q4 = lane >> 4;
    if constexpr (KC && BITS == 2) return i * 32 + (q4 >> 1) * 16 + r16;   // tile i
    // k-slots 0..15 of an MFMA are the first token set (tile 2*blk), 16..31 the second (tile 2*blk + 1); a lane
    // holds eight channels: octet q4 & 1 of half group hg; i = blk*2 + hg
    const int tile = 2 * (i >> 1) + (q4 >> 1), hg = i & 1;
    return BITS == 4 ? tile * 64 + (2 * hg + (q4 & 1)) * 16 + r16 : (tile * 2 + hg) * 16 + r16;
}
template <int BITS> __device__ __forceinline__ int vcode_chunk(int i, int lane)
{
    // Columns 0..7 of the PV MFMAs are channels of groups 0 and 1, columns 8..15 of groups 2 and 3: lane
    // (c, quad) reads the chunks of channel half c >> 3, at its own column (even i) and at column c ^ 8 (odd i);
    // INT4: i = blk*2 + chunk, INT2: i = chunk (a word holds both blocks)
    const int base = ((lane & 8) << 3) + (lane & 48) + ((lane & 15) ^ ((i & 1) << 3));
    return BITS == 4 ? (i >> 1) * 128 + base : base;
}
template <int BITS, bool KC>
__device__ __forceinline__ void load_page_k(PageRegs<BITS> &pr, const uint8_t *__restrict__ rec, int lane)
{
    const uint4 *kc = reinterpret_cast<const uint4 *>(rec + Rec<BITS>::kKCodes);
#pragma unroll
    for (int i = 0; i < 4; ++i) pr.kw[i] = load_once(kc + kcode_chunk<BITS, KC>(i, lane));
}
template <int BITS>
__device__ __forceinline__ void load_page_v(PageRegs<BITS> &pr, const uint8_t *__restrict__ rec, int lane)
{
    const uint4 *vc = reinterpret_cast<const uint4 *>(rec + Rec<BITS>::kVCodes);
#pragma unroll
    for (int i = 0; i < BITS; ++i) pr.vw[i] = load_once(vc + vcode_chunk<BITS>(i, lane));
}
// Lane constants of the page loop.
struct LaneConst {
    float F;              // 2^(24 - E): undoes the subnormal position and the power-of-two normalisation of q
    float kappa;          // sm_scale * log2(e)
    uint32_t vmul01, vmul23;   // fp16 pairs of the staging factor of the V scale, 2^(kVExp - pos)
    int zp_idx[2];        // chunk of Lds::pv with this lane's B operand of the zero-point MFMA, per 32-token block
    int vs_idx;           // ... of the staged V scales of (block 0, this lane's quad, group 2*(c >> 3))
    int vs_st;            // 8-byte slot of Lds::pv (behind kPvS) where this lane stages its four V scales
    uint32_t vrot[2];     // INT4 V unpack: rotate amounts that bring registers 0, 1 / 2, 3 of the operand into place
    uint32_t vmask[4];    // INT2 V unpack: field masks of operand registers 0..3
    int opaque_zero;      // 0, opaque to the compiler
    int tok0;             // two token sets: first token of this lane's four within a 32-token block
    int qy_ent;           // ... entry of this lane in a q operand of the QK^T MFMAs (or one of the two zero entries)
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
    uint2 kzv[2] = {{0u, 0u}, {0u, 0u}};   // K zeros of this lane's MFMA row per 32-token block (two token sets)
    (void)kzv;
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
            // the two key metadata planes as stored: fp16 [block][128 channel positions]; lanes 0..31 hold block 0.
            // A block that was never written (a half-filled page) is masked by count like everything else: whatever
            // its planes hold is neither used nor reported as a saturated scale.
            const bool dead = partial && 32 * (lane >> 5) >= n_valid;
            const uint2 ks = dead ? make_uint2(0u, 0u) : pr.ksc, kz = dead ? make_uint2(0u, 0u) : pr.kzc;
            const uint32_t k01 = pk_min(ks.x, kKcClamp), k23 = pk_min(ks.y, kKcClamp);
            st.sat |= (k01 ^ ks.x) | (k23 ^ ks.y);
            reinterpret_cast<uint2 *>(lds.kc_scale())[lane] = make_uint2(k01, k23);
            reinterpret_cast<uint2 *>(lds.kc_zero())[lane] = kz;
        } else {
            const half2_t a = __builtin_bit_cast(half2_t, pr.ksc.x), b = __builtin_bit_cast(half2_t, pr.ksc.y);
            // K scale * F as fp32 [block][group][token of the block]: a lane reads the scales of its four tokens for
            // one group with one 16-byte read
            {
                float *kst = lds.ks + (lane >> 5) * 128 + (lane & 31);
                kst[0] = fmaf((float)a[0], lc.F, 0.0f);   // (one mixed-precision FMA converts and scales)
                kst[32] = fmaf((float)a[1], lc.F, 0.0f);
                kst[64] = fmaf((float)b[0], lc.F, 0.0f);
                kst[96] = fmaf((float)b[1], lc.F, 0.0f);
            }
            // K zeros: lane (r, q4) takes those of token 32*blk + 16*(q4 >> 1) + r, which lane number that token holds.
            // An MFMA row holds a token of either set: a never-written token's zero-point (any bit pattern) would
            // meet the zeros of the other set's columns in the same row and could make them NaN.
            const uint2 kzm = partial && lane >= n_valid ? make_uint2(0u, 0u) : pr.kzc;
#pragma unroll
            for (int blk = 0; blk < 2; ++blk) {
                const int src = 4 * (32 * blk + 16 * (q4 >> 1) + r16);
                kzv[blk] = make_uint2((uint32_t)__builtin_amdgcn_ds_bpermute(src, (int)kzm.x),
                                      (uint32_t)__builtin_amdgcn_ds_bpermute(src, (int)kzm.y));
            }
        }
        // V side, this lane's four (token, group) entries: the staged scale and the zero plane as stored
        {
            const uint32_t m01 = pk_mul(vsc.x, lc.vmul01), m23 = pk_mul(vsc.y, lc.vmul23);
            const uint32_t s01 = pk_min(m01, kVsClamp), s23 = pk_min(m23, kVsClamp);
            st.sat |= (s01 ^ m01) | (s23 ^ m23);
            reinterpret_cast<uint2 *>(lds.pv)[2 * kPvS + lc.vs_st] = make_uint2(s01, s23);
            reinterpret_cast<uint2 *>(lds.pv)[2 * kPvZ + lane] = vzc;
        }
    }
    lds_order();

    // ---- QK^T: S[blk][i] = q . k_hat (unscaled) of token 32*blk + 16*(r16 >> 3) + 4*q4 + i for the head of column
    // r16 (two token sets); the per-channel path works on the four 16-token tiles first and folds them at its end
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
        // Both column halves now hold the logits of all four tiles.  From here on the page is treated as with
        // per-token keys: columns 0..7 go on with tile 2*blk, columns 8..15 with tile 2*blk + 1 (two token sets), so
        // that exponentials and weight pieces are formed once per (token, head).
        if (r16 >= 8) { S[0] = S[1]; S[2] = S[3]; }
        S[1] = S[2];
        __builtin_amdgcn_sched_barrier(0);
    } else {
        // Per-token groups.  The eight heads fill only half of the 16 MFMA columns, so the columns carry two
        // token sets: rows r of a 32-token block are token 32*blk + r in columns 0..7 and token 32*blk + 16 + r in
        // columns 8..15.  An MFMA contracts 16 channels (half a group) of both sets: k-slots 0..15 hold the
        // codes of the first token, 16..31 those of the second, and the B operand holds q in the matching half
        // of its k-slots and zeros in the other.  All that follows the MFMAs (K scale, exponentials, weight
        // pieces) is then done once per (token, head).
        const uint4 *qy = reinterpret_cast<const uint4 *>(lds.qo);
        floatx4 s[2];
#pragma unroll
        for (int blk = 0; blk < 2; ++blk) {
            const half8 za = as_half8(kzv[blk].x, kzv[blk].y, kzv[blk].x, kzv[blk].y);
            s[blk] = mfma(za, qz, floatx4{0.f, 0.f, 0.f, 0.f});   // zero-point term
        }
        // group by group, both 32-token blocks against one read of the q operand: two independent MFMA chains
#pragma unroll
        for (int g = 0; g < 4; ++g) {
            floatx4 p[2] = {{0.f, 0.f, 0.f, 0.f}, {0.f, 0.f, 0.f, 0.f}};
#pragma unroll
            for (int hg = 0; hg < 2; ++hg) {
                const uint4 qb4 = qy[(g * 2 + hg) * kQyStride + lc.qy_ent];
                const half8 qb = as_half8(qb4.x, qb4.y, qb4.z, qb4.w);
#pragma unroll
                for (int blk = 0; blk < 2; ++blk) {
                    const uint4 kw = pr.kw[blk * 2 + hg];
                    const uint32_t w = g == 0 ? kw.x : g == 1 ? kw.y : g == 2 ? kw.z : kw.w;
                    half8 a;
                    if (BITS == 4) {
                        const uint32_t w8 = w >> 8;
                        a = as_half8(w & 0x000f000fu, w & 0x00f000f0u, w8 & 0x000f000fu, w8 & 0x00f000f0u);
                    } else {
                        // this lane's 8 codes of the word are its upper or lower half; the rotate leaves the fields at bits
                        // 4:3, 6:5, 8:7, 10:9 of each half (towards the top of the fp16 mantissa, as for V: the matrix core
                        // drops product bits below its alignment window), stray bits fall outside the masks
                        const uint32_t ws = __builtin_amdgcn_alignbit(w, w, (q4 & 1) ? 5u : 29u);
                        a = as_half8(ws & 0x00180018u, ws & 0x00600060u, ws & 0x01800180u, ws & 0x06000600u);
                    }
                    p[blk] = mfma(a, qb, p[blk]);
                }
            }
#pragma unroll
            for (int blk = 0; blk < 2; ++blk) {
                const float4 sc = reinterpret_cast<const float4 *>(lds.ks)[(blk * 4 + g) * 8 + (lc.tok0 >> 2)];
                s[blk][0] = fmaf(sc.x, p[blk][0], s[blk][0]);
                s[blk][1] = fmaf(sc.y, p[blk][1], s[blk][1]);
                s[blk][2] = fmaf(sc.z, p[blk][2], s[blk][2]);
                s[blk][3] = fmaf(sc.w, p[blk][3], s[blk][3]);
            }
        }
        S[0] = s[0];
        S[1] = s[1];
        asm volatile("" : "+v"(S[0]), "+v"(S[1]));   // the scaled sums are formed here, not sunk next to their first use
        __builtin_amdgcn_sched_barrier(0);
    }
    after_qk();
    constexpr int kS = 2;   // logit registers of this lane: its eight tokens of the page
    if (partial) {
#pragma unroll
        for (int e = 0; e < kS; ++e)
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const int t = 32 * e + lc.tok0 + i;
                S[e][i] = t < n_valid ? S[e][i] : -INFINITY;
            }
    }

    // ---- online softmax with a lazily updated reference maximum ------------
    // The cheap test looks only at this lane's own logits; the column maximum is formed across
    // lanes only when some lane needs a new reference.
    float mx = fmaxf(fmaxf(S[0][0], S[0][1]), fmaxf(S[0][2], S[0][3]));
#pragma unroll
    for (int e = 1; e < kS; ++e) mx = fmaxf(fmaxf(mx, S[e][0]), fmaxf(fmaxf(S[e][1], S[e][2]), S[e][3]));
    if (__any(mx * lc.kappa > st.m_ref + kTau)) {
        mx = fmaxf(mx, row_ror8(mx));   // the other token set of the head
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
        for (int j = 0; j < 8; ++j) st.acc[j >> 2][j & 3] *= av;
        st.zp *= av;
    }
    const float nmref = (float)kPExp - (st.m_ref == -INFINITY ? 0.0f : st.m_ref);
    // W = P * 2^kPExp in two fp16 pieces (leading 11 bits truncated, then the next 11): the eight tokens of this
    // lane's k-slot octet per 32-token block.  With two token sets a lane forms the pieces of its own four tokens
    // and takes the other four from the lane eight columns on: registers 0, 1 are its own, 2, 3 the other set's
    // (the V operand of columns 8..15 lists its tokens in that order too).
    uint32_t wh[2][4], wl[2][4];
#pragma unroll
    for (int e = 0; e < kS; ++e) {
        float pv[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) pv[i] = __builtin_amdgcn_exp2f(fmaf(S[e][i], lc.kappa, nmref));
#pragma unroll
        for (int k = 0; k < 2; ++k) {
            const uint32_t hi = __builtin_bit_cast(uint32_t, __builtin_amdgcn_cvt_pkrtz(pv[2 * k], pv[2 * k + 1]));
            const uint32_t lo = __builtin_bit_cast(
                uint32_t, __builtin_amdgcn_cvt_pkrtz(residual<0>(hi, -1.0f, pv[2 * k]), residual<1>(hi, -1.0f, pv[2 * k + 1])));
            wh[e][k] = hi;
            wl[e][k] = lo;
            wh[e][2 + k] = ror8_u32(hi);
            wl[e][2 + k] = ror8_u32(lo);
        }
    }

    // ---- PV ------------------------------------------------------------------
#pragma unroll
    for (int blk = 0; blk < 2; ++blk) {
        // zero-point term and denominator: columns 0..3 = V zero of the groups, column 4 = ones
        {
            const uint4 bz4 = lds.pv[lc.zp_idx[blk]];
            const half8 bz = as_half8(bz4.x, bz4.y, bz4.z, bz4.w);
            st.zp = mfma(as_half8(wh[blk][0], wh[blk][1], wh[blk][2], wh[blk][3]), bz, st.zp);
            st.zp = mfma(as_half8(wl[blk][0], wl[blk][1], wl[blk][2], wl[blk][3]), bz, st.zp);
        }
#pragma unroll
        for (int gg = 0; gg < 2; ++gg) {
            // a = W * scale for group 2*(c >> 3) + gg in two fp16 pieces: hi = fp16(W_hi s), lo = W_lo s + the exact
            // remainder of the hi product
            const uint4 vs = lds.pv[lc.vs_idx + 16 * blk + gg];
            const uint32_t vsr[4] = {vs.x, vs.y, vs.z, vs.w};
            uint32_t ah[4], al[4];
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                ah[k] = pk_mul(wh[blk][k], vsr[k]);
                al[k] = pk_fma(wl[blk][k], vsr[k], pk_rem(wh[blk][k], vsr[k], ah[k]));
            }
            const half8 a_hi = as_half8(ah[0], ah[1], ah[2], ah[3]), a_lo = as_half8(al[0], al[1], al[2], al[3]);
            half8 b[2][2];
#pragma unroll
            for (int chunk = 0; chunk < 2; ++chunk)
#pragma unroll
                for (int cc = 0; cc < 2; ++cc) {
                    const int comp = 2 * gg + cc;
                    const uint4 v = BITS == 4 ? pr.vw[blk * 2 + chunk] : pr.vw[chunk];
                    const uint32_t w = comp == 0 ? v.x : comp == 1 ? v.y : comp == 2 ? v.z : v.w;
                    // Codes as fp16 subnormals, fields shifted towards the top of the mantissa (INT2: bits 4:3,
                    // 6:5, 8:7, 10:9 of each half; INT4: bits 6:3 and 10:7): the matrix core aligns the products of
                    // a lane's eight k-slots to the largest exponent *field* and drops what falls below a fixed
                    // window, so leading zeros of a subnormal cost precision.  Bit 10 is the lowest exponent bit:
                    // fp16 is linear through the first binade, so a field may reach it.  The slot's power of two
                    // is undone in the staged V scale.
                    // Registers 0, 1 take the tokens of this lane's own set, 2, 3 those of the other set (see the
                    // weights): the rotate amounts (INT4) or the masks (INT2) differ between the column halves.
                    if (BITS == 4) {
                        const uint32_t wa = __builtin_amdgcn_alignbit(w, w, lc.vrot[0]), wb = __builtin_amdgcn_alignbit(w, w, lc.vrot[1]);
                        b[chunk][cc] = as_half8(wa & 0x00780078u, wa & 0x07800780u, wb & 0x00780078u, wb & 0x07800780u);
                    } else {
                        const uint32_t ws = blk ? (w >> 5) : (w << 3);
                        b[chunk][cc] = as_half8(ws & lc.vmask[0], ws & lc.vmask[1], ws & lc.vmask[2], ws & lc.vmask[3]);
                    }
                    st.acc[chunk][2 * gg + cc] = mfma(a_hi, b[chunk][cc], st.acc[chunk][2 * gg + cc]);
                }
#pragma unroll
            for (int chunk = 0; chunk < 2; ++chunk)
#pragma unroll
                for (int cc = 0; cc < 2; ++cc) st.acc[chunk][2 * gg + cc] = mfma(a_lo, b[chunk][cc], st.acc[chunk][2 * gg + cc]);
        }
    }
    after_pv();
}

// What stays the same for every page of a work item, and the pages of one width in it (positions in the
// sequence's page list).
struct ItemCtx {
    const uint8_t *__restrict__ pool;
    const uint8_t *__restrict__ bit_map;
    const int32_t *__restrict__ pages;   // the sequence's page list
    int kvh, n_kv_heads, n_pages_int2, n_pages_total, lane, opaque_zero;
    int32_t *status;
};
struct WidthRange {
    int pb, pe;                  // positions in the page list
    int last_index, last_valid;  // position of the width's last page in the sequence and its number of valid tokens
    int page_lo, page_hi;        // the pool's page ids
};
// Page id of list position pi (already loaded) and its number of valid tokens.  A page id outside its pool cannot
// be addressed: it is flagged, a valid page is read instead and skipped.
__device__ __forceinline__ int validate_page(const ItemCtx &cx, const WidthRange &wr, int pi, int &page)
{
    const bool ok = page >= wr.page_lo && page < wr.page_hi;
    if (!ok) {
        if (cx.status && cx.lane == 0)
            atomicOr(cx.status, page < 0 || page >= cx.n_pages_total ? TKV_STATUS_PAGE_RANGE : TKV_STATUS_BITMAP_MISMATCH);
        page = wr.page_lo;
    }
    return ok ? (pi == wr.last_index ? wr.last_valid : kPageTokens) : 0;
}
// State handed from start_pages to run_pages: the first record's registers, the next page's id.
template <int BITS> struct Started {
    PageRegs<BITS> pr;
    int nv, page_next, nv_next;
};
// Requests the first record of a width.
template <int BITS, bool KC>
__device__ __forceinline__ void start_pages(const ItemCtx &cx, const WidthRange &wr, Started<BITS> &s0)
{
    int page = __builtin_amdgcn_readfirstlane(cx.pages[wr.pb]);
    s0.nv = validate_page(cx, wr, wr.pb, page);
    const int pi1 = wr.pb + 1 < wr.pe ? wr.pb + 1 : wr.pb;
    s0.page_next = __builtin_amdgcn_readfirstlane(cx.pages[pi1]);
    s0.nv_next = validate_page(cx, wr, pi1, s0.page_next);
    const uint8_t *rec = cx.pool + record_offset(page, cx.kvh, cx.n_kv_heads, cx.n_pages_int2);
    load_page_meta<BITS>(s0.pr, rec, cx.bit_map, page, cx.lane, cx.opaque_zero);
    load_page_k<BITS, KC>(s0.pr, rec, cx.lane);
    load_page_v<BITS>(s0.pr, rec, cx.lane);
}

template <int BITS, bool KC>
__device__ __forceinline__ void run_pages(const ItemCtx &cx, const WidthRange &wr, Started<BITS> &s0, int item_end, int item_pages,
                                          half8 qz, LaneConst lc, WaveState &st, Lds<KC> &lds)
{
    const uint8_t *__restrict__ pool = cx.pool;
    const uint8_t *__restrict__ bit_map = cx.bit_map;
    const int32_t *__restrict__ pages = cx.pages;
    const int pb = wr.pb, pe = wr.pe, kvh = cx.kvh, n_kv_heads = cx.n_kv_heads, n_pages_int2 = cx.n_pages_int2, lane = cx.lane;
    int32_t *status = cx.status;
    // A V code enters the MFMA as code * 2^(pos - 24), pos = lowest bit of its field after the unpack shift; the
    // staged scale of the slot carries 2^(kVExp - pos).  This lane stages plane entries 4*lane .. 4*lane+3 =
    // k-slots 4*(lane&1) + 0..3, i.e. operand registers 2*(lane&1) (first pair) and 2*(lane&1) + 1 (second pair).
    {
        const int k0 = 2 * (lane & 1);
        const int p01 = BITS == 4 ? 3 : 3 + 2 * k0, p23 = BITS == 4 ? 7 : 5 + 2 * k0;
        const uint32_t h01 = (uint32_t)(15 + kVExp - p01) << 10, h23 = (uint32_t)(15 + kVExp - p23) << 10;
        lc.vmul01 = h01 | (h01 << 16);
        lc.vmul23 = h23 | (h23 << 16);
        // Order of the eight tokens of a k-slot octet in the PV operands: a lane lists its own token set first, which
        // for columns 8..15 (the rows and columns of groups 2 and 3) is tile 2*blk + 1: those lanes swap the register
        // pairs of the V operand, and the staged scales of groups 2 and 3 are stored with their 8-byte halves swapped.
        const bool swap = lane & 8;
        lc.vrot[0] = swap ? 5u : 29u;   // w >> 5 / w << 3 (stray bits fall outside the masks)
        lc.vrot[1] = swap ? 29u : 5u;
        const uint32_t m[4] = {0x00180018u, 0x00600060u, 0x01800180u, 0x06000600u};
#pragma unroll
        for (int k = 0; k < 4; ++k) lc.vmask[k] = m[swap ? k ^ 2 : k];
        lc.vs_st = (lane & 4) ? lane ^ 1 : lane;   // lane = ((blk*4 + quad)*4 + g)*2 + half
    }
    // One register set: every part of the next record is requested as soon as the registers it lands in
    // are dead, so about one page per wavefront is in flight while the current one is computed.
    PageRegs<BITS> &pr = s0.pr;
    int nv = s0.nv, page_next = s0.page_next, nv_next = s0.nv_next;
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
        // The id of the page after next is requested now, as a per-lane load (`opaque_zero`), and turned into a
        // scalar at the end of this page: its latency never stands between two pages.  The last page requests its
        // own record again: no branch around the loads.
        const int pi_next2 = pi + 2 < pe ? pi + 2 : pe - 1;
        const int pgv = pages[pi_next2 + lc.opaque_zero];
        const uint8_t *rec_next = pool + record_offset(page_next, kvh, n_kv_heads, n_pages_int2);
        const uint32_t bm = pr.bm;
        auto after_qk = [&]() {
            __builtin_amdgcn_sched_barrier(0);   // keep the reloads below the last use of the registers they overwrite
            load_page_meta<BITS>(pr, rec_next, bit_map, page_next, lane, lc.opaque_zero);
            load_page_k<BITS, KC>(pr, rec_next, lane);
        };
        auto after_pv = [&]() {
            __builtin_amdgcn_sched_barrier(0);
            load_page_v<BITS>(pr, rec_next, lane);
        };
        // the bit_map entry arrives with the page: a mismatch skips the whole page
        if (__any(bm != BITS) && nv > 0) {
            if (status && lane == 0) atomicOr(status, TKV_STATUS_BITMAP_MISMATCH);
            nv = 0;
        }
        // a page with no valid token still runs (every token masked by count): no second path through the loop
        compute_page<BITS, KC>(pr, nv, lane, qz, lc, st, lds, after_qk, after_pv);
        nv = nv_next;
        page_next = __builtin_amdgcn_readfirstlane(pgv);
        nv_next = validate_page(cx, wr, pi_next2, page_next);
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
    __shared__ Lds<KC> lds;
    // q * 2^E per head and channel (2 KiB of fp16), read while the MFMA operands are built.  With per-channel INT2
    // keys it lives in the page staging area ks | pv, which is idle then, so that twelve wavefronts fit the LDS of a
    // compute unit, and is written again before the INT4 operand is built; otherwise it has its own place.
    void *qf;
    if constexpr (KC) qf = lds.ks;
    else qf = lds.qf;
    const int lane = threadIdx.x, r16 = lane & 15, q4 = lane >> 4;
    const int item = blockIdx.x / n_kv_heads, kvh = blockIdx.x % n_kv_heads;
    const int R = n_q_heads / n_kv_heads;
    const int seq = items[4 * item];
    // The partial of this item goes to slot items[4*item + 3] of the workspace: items are listed in launch order,
    // the slots of a sequence are contiguous (the merge reads them by sequence).
    const int slot = items[4 * item + 3];
    const bool slot_ok = slot >= 0 && slot < (int)(gridDim.x / n_kv_heads);
    if (seq < 0 || seq >= batch || !slot_ok) {
        // malformed item: an empty partial (m = -inf, l = 0), which the merge ignores, and a status bit; with a slot
        // outside the workspace nothing can be written, and whoever owns the slot it should have named reads what
        // the workspace held before
        for (int h = 0; h < R && slot_ok; ++h) {
            const size_t ph = (size_t)slot * n_q_heads + kvh * R + h;
            reinterpret_cast<float2 *>(acc_ws + ph * kHeadDim)[lane] = make_float2(0.0f, 0.0f);
            if (lane == 0) reinterpret_cast<float2 *>(ml_ws)[ph] = make_float2(-INFINITY, 0.0f);
        }
        if (status && lane == 0) atomicOr(status, TKV_STATUS_BAD_ITEM);
        return;
    }
    const int n2 = n_tok_int2[seq], n4 = n_tok_int4[seq];
    const int np2 = (n2 + kPageTokens - 1) / kPageTokens, np4 = (n4 + kPageTokens - 1) / kPageTokens;
    const int seq_pages = page_indptr[seq + 1] - page_indptr[seq];
    const int np_all = np2 + np4 < seq_pages ? np2 + np4 : seq_pages;
    const int pb = items[4 * item + 1] > 0 ? items[4 * item + 1] : 0;
    const int pe = items[4 * item + 2] < np_all ? items[4 * item + 2] : np_all;
    const int32_t *pages = page_ids + page_indptr[seq];
    const int n_pages_total = n_pages_int2 + n_pages_int4;
    // INT2 pages of the range, then INT4 pages: each page runs one dequantisation path
    const int e2 = pe < np2 ? pe : np2, b4 = pb > np2 ? pb : np2;
    const bool has2 = pb < e2, has4 = b4 < pe;
    int opaque_zero;
    asm volatile("v_mov_b32 %0, 0" : "=v"(opaque_zero));
    const ItemCtx cx = {pool, bit_map, pages, kvh, n_kv_heads, n_pages_int2, n_pages_total, lane, opaque_zero, status};
    const WidthRange wr2 = {pb, e2, np2 - 1, n2 - (np2 - 1) * kPageTokens, 0, n_pages_int2};
    const WidthRange wr4 = {b4, pe, np2 + np4 - 1, n4 - (np4 - 1) * kPageTokens, n_pages_int2, n_pages_total};
    Started<2> s2;
    Started<4> s4;

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
    lc.vmul01 = lc.vmul23 = 0;
    lc.zmul = r16 >= 8 ? 0.0f : 0x1p-24f;
    lc.vs_idx = kPvS + q4 * 4 + 2 * (r16 >> 3);
    lc.vs_st = lane;
    lc.opaque_zero = opaque_zero;
    lc.vrot[0] = lc.vrot[1] = 0;
    lc.vmask[0] = lc.vmask[1] = lc.vmask[2] = lc.vmask[3] = 0;
    lc.tok0 = 16 * (r16 >> 3) + 4 * q4;
    lc.qy_ent = (r16 >> 3) == (q4 >> 1) ? (q4 & 1) * 8 + (r16 & 7) : ((q4 & 1) ? kQyZero1 : kQyZero0);
#pragma unroll
    for (int blk = 0; blk < 2; ++blk) {
        lc.zp_idx[blk] = r16 < 4 ? kPvZ + (blk * 4 + q4) * 4 + r16 : (r16 == 4 ? kPvOne : kPvZero);
    }
    if (lane < 2) {
        const uint32_t c = lane == 1 ? 0x3c003c00u : 0u;
        lds.pv[kPvZero + lane] = make_uint4(c, c, c, c);
    }
    // q * 2^E to LDS; per-group sums of the unscaled q: lanes 16g .. 16g+15 hold group g
#pragma unroll
    for (int h = 0; h < 8; ++h) {
        qf_store<KC>(qf, h, lane, pack_h2(qv[h][0] * two_e, qv[h][1] * two_e));   // exact: q has 8 significant bits
        const float sum = row_sum(qv[h][0] + qv[h][1]);
        if (r16 == 0) lds.zl()[h][q4] = sum;   // [head][group]
    }
    lds_order();
    const int hcol = (r16 & 7) & (R - 1);   // head of this lane's column (columns beyond R repeat heads)
    half8 qz;
    {
        // Z-term B operand (two token sets: the k-slots of a column's own set carry the pieces, the others zeros):
        // slots 0..3 / 4..7 of the first octet = hi / mid pieces of the four group sums, slots 0..3 of the second
        // octet = lo pieces
        const float4 gs = reinterpret_cast<const float4 *>(lds.zl()[hcol])[0];
        const float sums[4] = {gs.x, gs.y, gs.z, gs.w};
        float pc[8] = {0, 0, 0, 0, 0, 0, 0, 0};
        const bool own = (r16 >> 3) == (q4 >> 1);
#pragma unroll
        for (int g = 0; g < 4; ++g) {
            const _Float16 hi = (_Float16)sums[g];
            const float r1 = sums[g] - (float)hi;
            const _Float16 mid = (_Float16)r1;
            const _Float16 lo = (_Float16)(r1 - (float)mid);
            if (own && (q4 & 1) == 0) { pc[g] = (float)hi; pc[4 + g] = (float)mid; }
            else if (own) { pc[g] = (float)lo; }
        }
        qz = as_half8(pack_h2(pc[0], pc[1]), pack_h2(pc[2], pc[3]), pack_h2(pc[4], pc[5]), pack_h2(pc[6], pc[7]));
    }

    WaveState st;
#pragma unroll
    for (int j = 0; j < 8; ++j) st.acc[j >> 2][j & 3] = floatx4{0.f, 0.f, 0.f, 0.f};
    st.zp = floatx4{0.f, 0.f, 0.f, 0.f};
    st.m_ref = -INFINITY;
    st.sat = 0;

    if (has2) {
        build_q_operand<2, KC>(qf, hcol, q4, lane, lds);
        LaneConst lc2 = lc;
        if constexpr (KC) {
            lc2.kappa = lc.kappa * lc.F;   // the power of two that the K scale carries otherwise
            lds.kc_nil()[lane & 31] = make_uint4(0u, 0u, 0u, 0u);
        }
        start_pages<2, KC>(cx, wr2, s2);
        lds_order();
        run_pages<2, KC>(cx, wr2, s2, pe, pe - pb, qz, lc2, st, lds);
    }
    if (has4) {
        start_pages<4, KC>(cx, wr4, s4);
        if (KC && has2) {   // the INT2 pages have used that memory since
            lds_order();
#pragma unroll
            for (int h = 0; h < 8; ++h) {
                uint32_t two = 0;
                if (h < R) two = reinterpret_cast<const uint32_t *>(q + ((size_t)seq * n_q_heads + kvh * R + h) * kHeadDim)[lane];
                const float q0 = __uint_as_float(two << 16) * two_e, q1 = __uint_as_float(two & 0xffff0000u) * two_e;
                qf_store<KC>(qf, h, lane, pack_h2(q0, q1));
            }
            lds_order();
        }
        build_q_operand<4, KC>(qf, hcol, q4, lane, lds);
        lds_order();
        run_pages<4, KC>(cx, wr4, s4, pe, pe - pb, qz, lc, st, lds);
    }

    // ---- write the partial (m, l, acc) of this item ------------------------------
    if (status && __any(st.sat != 0) && lane == 0) atomicOr(status, TKV_STATUS_SCALE_SATURATED);
    // per head: columns 0..3 of zl = zero-point sums of the groups, 4 = denominator
    lds_order();
    if (q4 < 2 && r16 < 5)
#pragma unroll
        for (int i = 0; i < 4; ++i) lds.zl()[4 * q4 + i][r16] = st.zp[i];
    if (q4 == 0 && r16 < 8) lds.alpha[r16] = st.m_ref;
    lds_order();
    const float unscale = ldexpf(1.0f, 24 - kVExp);
    const int hb = r16 >> 3;
    // The accumulators go through an LDS tile [head][channel] so that every lane stores 16 bytes and a store
    // instruction covers two whole heads (a lane holds single channels of four heads).  The tile takes the start of
    // the LDS, which holds nothing the epilogue needs (q staging, page staging); rows are 16 bytes longer than a
    // head so that heads h and h + 4, written by the same instruction, fall on different banks.
    constexpr int kOutRow = kHeadDim + 4;
    static_assert(sizeof(LdsExtra<KC>) + sizeof(float) * kPageTokens * kGroups + sizeof(uint4) * kPvChunks >= 8 * kOutRow * sizeof(float),
                  "the output tile must fit in what precedes kz, qo (= zl()) and alpha in Lds");
    float *tile = reinterpret_cast<float *>(&lds);
    if ((q4 >> 1) == hb) {   // the quadrants whose rows and columns belong to the same pair of groups
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int head = 4 * (q4 & 1) + i;
#pragma unroll
            for (int gg = 0; gg < 2; ++gg) {
                const int g = 2 * hb + gg;
                const float zsum = lds.zl()[head][g];
#pragma unroll
                for (int chunk = 0; chunk < 2; ++chunk)
#pragma unroll
                    for (int cc = 0; cc < 2; ++cc) {
                        const int comp = 2 * gg + cc;
                        tile[head * kOutRow + 64 * hb + 16 * comp + (chunk ? r16 ^ 8 : r16)] = st.acc[chunk][comp][i] * unscale + zsum;
                    }
            }
        }
    }
    if (lane < 8 && lane < R) {
        const size_t ph = (size_t)slot * n_q_heads + kvh * R + lane;
        reinterpret_cast<float2 *>(ml_ws)[ph] = make_float2(lds.alpha[lane], lds.zl()[lane][4]);
    }
    lds_order();
#pragma unroll
    for (int k = 0; k < 4; ++k) {
        const int head = 2 * k + (lane >> 5), c4 = lane & 31;
        if (head < R) {
            const size_t ph = (size_t)slot * n_q_heads + kvh * R + head;
            reinterpret_cast<float4 *>(acc_ws + ph * kHeadDim)[c4] = reinterpret_cast<const float4 *>(tile + head * kOutRow)[c4];
        }
    }
}

// D7: out = sum_i 2^(m_i - M) acc_i / sum_i 2^(m_i - M) l_i over the items of a sequence (Sec. 3.2.3: the
// splits are merged by online log-sum-exp).
// One workgroup of TH threads per (sequence, query head, one of SL channel slices).  32 / SL lanes own an item at a
// time: their 16-byte loads are the item's accumulators of the slice, so every partial is read once with 128-bit
// loads and TH * SL / 32 items are in flight per workgroup round.  Each such lane group keeps a running (M, l, acc);
// the groups are merged through LDS by the first wavefront.  SL = 1, TH = 256 when a sequence has tens of items;
// SL = 4, TH = 512 (four workgroups per head, 64 item slots each) when it has hundreds, as a single long sequence
// with one kv head does.
template <int SL, int TH>
__global__ __launch_bounds__(TH) void tkv_reduce_rows_kernel(
    const float *__restrict__ acc_ws, const float *__restrict__ ml_ws, const int32_t *__restrict__ seq_item_indptr,
    int n_q_heads, float *__restrict__ out)
{
    constexpr int kLanes = 32 / SL;       // lanes per item: 16 bytes each
    constexpr int kSlots = TH / kLanes;   // items in flight
    constexpr int kSubsets = 64 / kLanes; // the first wavefront merges the slots in this many interleaved subsets
    __shared__ float4 num_s[kSlots][kLanes];
    __shared__ float2 ml_s[kSlots];
    const int bh = blockIdx.x / SL, slice = blockIdx.x % SL;
    const int b = bh / n_q_heads, h = bh % n_q_heads, tid = threadIdx.x;
    const int slot = tid / kLanes, ln = tid % kLanes, cq = slice * kLanes + ln;   // cq: which float4 of the 32 of a row
    const int i0 = seq_item_indptr[b], i1 = seq_item_indptr[b + 1];
    float M = -INFINITY, den = 0.0f;
    float4 num = make_float4(0.f, 0.f, 0.f, 0.f);
#pragma unroll 4
    for (int i = i0 + slot; i < i1; i += kSlots) {
        const size_t ph = (size_t)i * n_q_heads + h;
        const float2 ml = reinterpret_cast<const float2 *>(ml_ws)[ph];
        // a partial is read once, 512 contiguous bytes per item
        const uint4 au = load_once(reinterpret_cast<const uint4 *>(acc_ws + ph * kHeadDim) + cq);
        const float4 a = make_float4(__uint_as_float(au.x), __uint_as_float(au.y), __uint_as_float(au.z), __uint_as_float(au.w));
        // an item without tokens has m = -inf, l = 0 and weighs nothing; no branch, so the loads of several
        // rounds are in flight together
        const float Mn = fmaxf(M, ml.x);
        const float so = M == -INFINITY ? 0.0f : __builtin_amdgcn_exp2f(M - Mn);
        const float sn = ml.x == -INFINITY ? 0.0f : __builtin_amdgcn_exp2f(ml.x - Mn);
        den = den * so + sn * ml.y;
        num.x = num.x * so + sn * a.x;
        num.y = num.y * so + sn * a.y;
        num.z = num.z * so + sn * a.z;
        num.w = num.w * so + sn * a.w;
        M = Mn;
    }
    num_s[slot][ln] = num;
    if (ln == 0) ml_s[slot] = make_float2(M, den);
    __syncthreads();
    if (tid < 64) {
        // lane (subset, ln) of the first wavefront merges slots subset, subset + kSubsets, ...
        float Mg = -INFINITY;
#pragma unroll
        for (int k = slot; k < kSlots; k += kSubsets) Mg = fmaxf(Mg, ml_s[k].x);
#pragma unroll
        for (int o = kLanes; o < 64; o <<= 1) Mg = fmaxf(Mg, __shfl_xor(Mg, o));
        float4 n = make_float4(0.f, 0.f, 0.f, 0.f);
        float d = 0.0f;
#pragma unroll
        for (int k = slot; k < kSlots; k += kSubsets) {
            const float2 ml = ml_s[k];
            const float wk = ml.x == -INFINITY ? 0.0f : __builtin_amdgcn_exp2f(ml.x - Mg);
            const float4 a = num_s[k][ln];
            d += wk * ml.y;
            n.x += wk * a.x;
            n.y += wk * a.y;
            n.z += wk * a.z;
            n.w += wk * a.w;
        }
#pragma unroll
        for (int o = kLanes; o < 64; o <<= 1) {
            d += __shfl_xor(d, o);
            n.x += __shfl_xor(n.x, o);
            n.y += __shfl_xor(n.y, o);
            n.z += __shfl_xor(n.z, o);
            n.w += __shfl_xor(n.w, o);
        }
        const float r = d > 0.0f ? 1.0f / d : 0.0f;
        if (tid < kLanes)
            reinterpret_cast<float4 *>(out + ((size_t)b * n_q_heads + h) * kHeadDim)[cq] = make_float4(n.x * r, n.y * r, n.z * r, n.w * r);
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
    if ((int64_t)n_items <= 128 * (int64_t)batch)
        hipLaunchKernelGGL((tkv_reduce_rows_kernel<1, 256>), dim3((unsigned)(batch * n_q_heads)), dim3(256), 0,
                           (hipStream_t)stream, acc_ws, ml_ws, seq_item_indptr, n_q_heads, out);
    else
        hipLaunchKernelGGL((tkv_reduce_rows_kernel<4, 512>), dim3((unsigned)(batch * n_q_heads * 4)), dim3(512), 0,
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
