// tkv_quantize_append: quantise newly written bf16 K/V at a per-token width
// (INT2 / INT4) and pack codes, fp16 scales and fp16 zero-points into the
// paged pool (paper Sec. 3.2.1 for the quantisation scheme, Sec. 3.2.2-3.2.3
// for the two pools and the per-token bitwidth array).
//
// One workgroup of 256 threads owns one (destination page, kv head) record.
// Thread (slot = tid/4, group = tid%4) quantises one group of 32 channels of
// the token bound for that slot, for K and for V, entirely in registers: a
// group is 64 contiguous bytes of the input, so min/max need no cross-lane
// step.  K words go straight to HBM (a wavefront's stores for one word index
// are 256 contiguous bytes, written with non-temporal stores).  V codes are transposed through LDS, because
// the V plane packs tokens, not channels, into a word; for a page that arrives whole, the V words and the two V
// metadata planes, which are adjacent in the record, are put together in LDS and leave in 16-byte non-temporal
// stores, one KiB per instruction of a wavefront.
//
// Arithmetic is IEEE binary32 without fused multiply-add so that the codes,
// scales and zero-points match a scalar CPU evaluation bit for bit:
//   zero = fp16(min), scale = fp16((max - min) / (2^b - 1)),
//   code = clamp(rint((x - zero) * (1 / scale)), 0, 2^b - 1), 0 if scale == 0.
#include <hip/hip_runtime.h>
#include <hip/hip_fp16.h>

#include <type_traits>

#include "tkv_internal.h"
#include "tkv_layout.h"

#pragma clang fp contract(off)

namespace {

using namespace tkv;

struct GroupQ {
    uint32_t words[4];   // packed codes: INT4 uses 4 words (8 channels each), INT2 2 words (16 each)
    uint32_t bytes[8];   // the same 32 codes, one per byte (for the V transpose)
    uint16_t scale, zero;
};

// One quantisation group of 32 values: the channels of a group of one token, or (per-channel keys) the 32
// tokens of a block for one channel.
template <int BITS>
__device__ __forceinline__ GroupQ quantize_values(const float (&f)[32])
{
    constexpr int L = (1 << BITS) - 1;
    // Inputs are finite, so min / max instructions give the value a chain of comparisons gives; only the sign
    // of a zero can differ.  A zero minimum is stored as +0 anyway; a zero maximum takes the sign the scalar
    // definition gives it (the first element that is not below its predecessors' maximum), settled below.
    float mn = f[0], mx = f[0];
#pragma unroll
    for (int i = 1; i < 32; ++i) {
        mn = fminf(mn, f[i]);
        mx = fmaxf(mx, f[i]);
    }
    if (mn == 0.0f) mn = 0.0f;   // -0 -> +0
    if (__builtin_expect(mx == 0.0f, 0)) {
        mx = f[0];
#pragma unroll
        for (int i = 1; i < 32; ++i) mx = f[i] > mx ? f[i] : mx;
    }
    const float r = __fsub_rn(mx, mn);
    const float s32 = __fdiv_rn(r, (float)L);
    const __half sh = __float2half_rn(s32), zh = __float2half_rn(mn);
    const float s = __half2float(sh), z = __half2float(zh);
    GroupQ out;
    out.scale = __half_as_ushort(sh);
    out.zero = __half_as_ushort(zh);
    const float inv = s == 0.0f ? 0.0f : __fdiv_rn(1.0f, s);   // a zero scale gives t = 0 and code 0 for every element
    // clamp, then round by adding 1.5 * 2^23: the sum is rounded to an integer (nearest, ties to even, the
    // same result as rounding first and clamping after) and its bit pattern is kBias + code
    constexpr float kMagic = 12582912.0f;
    constexpr uint32_t kBias = 0x4b400000u;
    uint32_t c[32];
#pragma unroll
    for (int i = 0; i < 32; ++i) {
        const float t = __builtin_amdgcn_fmed3f(__fmul_rn(__fsub_rn(f[i], z), inv), 0.0f, (float)L);
        c[i] = __float_as_uint(__fadd_rn(t, kMagic));
    }
    // packed by shift-and-add; what the biases add up to (modulo 2^32) is one constant per word
    constexpr int per_word = 32 / BITS;
    uint32_t bias_word = 0, bias_byte = 0;
#pragma unroll
    for (int i = 0; i < per_word; ++i) bias_word += kBias << (BITS * i);
#pragma unroll
    for (int k = 0; k < 4; ++k) bias_byte += kBias << (8 * k);
#pragma unroll
    for (int w = 0; w < 4; ++w) out.words[w] = 0u - bias_word;
#pragma unroll
    for (int i = 0; i < 32; ++i) out.words[i / per_word] += c[i] << (BITS * (i % per_word));
#pragma unroll
    for (int w = 0; w < 8; ++w)
        out.bytes[w] = c[4 * w] + (c[4 * w + 1] << 8) + (c[4 * w + 2] << 16) + (c[4 * w + 3] << 24) - bias_byte;
    return out;
}

template <int BITS>
__device__ __forceinline__ GroupQ quantize_group(const uint4 *src)
{
    float f[32];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const uint4 v = src[i];
        const uint32_t u[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            f[8 * i + 2 * k] = __uint_as_float(u[k] << 16);
            f[8 * i + 2 * k + 1] = __uint_as_float(u[k] & 0xffff0000u);
        }
    }
    return quantize_values<BITS>(f);
}

// LDS of the per-channel key path: the bf16 keys of the page [slot][channel], then their codes one per byte.
struct KcLds {
    alignas(16) uint16_t kt[kPageTokens][kHeadDim];
    alignas(16) uint8_t kcodes[kPageTokens][kHeadDim];
    int n_in_block[2];
};
struct NoLds {};

// KC: keys per channel over each block of 32 slots (INT2 pages only); `valid` is then uniform over a block.
template <int BITS, bool KC, class KL>
__device__ __forceinline__ void append_record(uint8_t *rec, const uint16_t *K, const uint16_t *V, int src,
                                              bool valid, int head, int n_kv_heads,
                                              uint32_t (*lds_codes)[32], uint8_t *lds_valid, uint4 *lds_vout, KL &kl)
{
    using R = Rec<BITS>;
    const int tid = threadIdx.x, slot = tid >> 2, g = tid & 3;
    const int tile = slot >> 4, row = slot & 15;
    if (g == 0) lds_valid[slot] = valid;
    uint16_t v_scale = 0, v_zero = 0;
    if (valid) {
        const size_t e = ((size_t)src * n_kv_heads + head) * kHeadDim + g * kGroup;
        if constexpr (KC) {
            // the keys wait in LDS until the whole block is there
            const uint4 *ksrc = reinterpret_cast<const uint4 *>(K + e);
            uint4 *kdst = reinterpret_cast<uint4 *>(&kl.kt[slot][g * kGroup]);
#pragma unroll
            for (int i = 0; i < 4; ++i) kdst[i] = ksrc[i];
        } else {
            const GroupQ kq = quantize_group<BITS>(reinterpret_cast<const uint4 *>(K + e));
            uint32_t *kc = reinterpret_cast<uint32_t *>(rec + R::kKCodes);
            constexpr int words = BITS;   // 32-bit words of codes per group: 4 (INT4) or 2 (INT2)
            // these stores of a wavefront fill whole lines (256 contiguous bytes per word index, 128 per plane)
#pragma unroll
            for (int w = 0; w < words; ++w) store_once(&kc[((tile * words + w) * 16 + row) * 4 + g], kq.words[w]);
            store_once(&reinterpret_cast<uint16_t *>(rec + R::kKScale)[slot * 4 + g], kq.scale);
            store_once(&reinterpret_cast<uint16_t *>(rec + R::kKZero)[slot * 4 + g], kq.zero);
        }

        const GroupQ vq = quantize_group<BITS>(reinterpret_cast<const uint4 *>(V + e));
        const int mi = vmeta_index(slot, g);
        v_scale = vq.scale;
        v_zero = vq.zero;
        // the two V metadata planes (2 x 512 B) are put together behind the V words in the staging area
        uint16_t *meta = reinterpret_cast<uint16_t *>(lds_vout + R::kCodeBytes / 16);
        meta[mi] = vq.scale;
        meta[kMetaBytes / 2 + mi] = vq.zero;
        uint4 *dst = reinterpret_cast<uint4 *>(&lds_codes[slot][g * 8]);
        dst[0] = make_uint4(vq.bytes[0], vq.bytes[1], vq.bytes[2], vq.bytes[3]);
        dst[1] = make_uint4(vq.bytes[4], vq.bytes[5], vq.bytes[6], vq.bytes[7]);
    }
    const bool page_full = __syncthreads_and(valid);   // every slot of the page arrives in this call
    if constexpr (KC) {
        // thread (block, channel): the block's 32 token values of one channel are one quantisation group
        {
            const int blk = tid >> 7, c = tid & 127;
            if (kl.n_in_block[blk] == kGroup) {
                float f[32];
#pragma unroll
                for (int i = 0; i < 32; ++i) f[i] = __uint_as_float((uint32_t)kl.kt[32 * blk + i][c] << 16);
                const GroupQ kq = quantize_values<BITS>(f);
                const int mi = kcmeta_index(blk, c);
                reinterpret_cast<uint16_t *>(rec + R::kKScale)[mi] = kq.scale;
                reinterpret_cast<uint16_t *>(rec + R::kKZero)[mi] = kq.zero;
#pragma unroll
                for (int i = 0; i < 32; ++i) kl.kcodes[32 * blk + i][c] = (uint8_t)(kq.bytes[i >> 2] >> (8 * (i & 3)));
            }
        }
        __syncthreads();
        // thread (slot, group) again: its token's 32 codes of the group, packed as in the per-token layout
        if (valid) {
            const uint4 *cb = reinterpret_cast<const uint4 *>(&kl.kcodes[slot][g * kGroup]);
            uint32_t *kc = reinterpret_cast<uint32_t *>(rec + R::kKCodes);
            constexpr int words = BITS;
            constexpr int per_word = 32 / BITS;
            uint32_t wv[4] = {0, 0, 0, 0};
#pragma unroll
            for (int q = 0; q < 2; ++q) {
                const uint4 v = cb[q];
                const uint32_t b4[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
                for (int j = 0; j < 4; ++j)
#pragma unroll
                    for (int k = 0; k < 4; ++k) {
                        const int i = 16 * q + 4 * j + k;   // channel of the group
                        wv[i / per_word] |= ((b4[j] >> (8 * k)) & 0xffu) << (BITS * (i % per_word));
                    }
            }
#pragma unroll
            for (int w = 0; w < words; ++w) kc[((tile * words + w) * 16 + row) * 4 + g] = wv[w];
        }
    }
    // V codes: one 32-bit word = one channel x (8 | 16) tokens of one quad
    const uint8_t *codes = reinterpret_cast<const uint8_t *>(lds_codes);
    uint32_t *vc = reinterpret_cast<uint32_t *>(rec + R::kVCodes);
    constexpr int n_words = R::kCodeBytes / 4;
    if (page_full) {
        // Whole page: a thread transposes four adjacent channels x the (8 | 16) tokens of one word with 32-bit
        // LDS reads (a row of the byte tile holds the token's codes in channel order), merges 2 | 4 tokens per
        // byte and finishes with a 4 x 4 byte transpose; no read-modify-write.
        constexpr int n_units = n_words / 4;   // 256 (INT4) / 128 (INT2)
        if (tid < n_units) {
            const int k = tid & 3, n4 = (tid >> 2) & 3, quad = (tid >> 4) & 3, h = (tid >> 6) & 1;
            const int blk = tid >> 7;   // INT4 only (0 for INT2)
            const int c0 = 64 * h + 16 * k + 4 * n4;
            uint32_t m[4];
#pragma unroll
            for (int b = 0; b < 4; ++b) {
                m[b] = 0;
#pragma unroll
                for (int e = 0; e < 8 / BITS; ++e) {
                    const int p = (8 / BITS) * b + e;   // position of the token in the word
                    int t;
                    if (BITS == 4) {
                        const int j = 2 * (p & 3) + (p >> 2);
                        t = 32 * blk + 16 * (j >> 2) + 4 * quad + (j & 3);
                    } else {
                        const int j = 2 * (p & 3) + (p >> 3);
                        t = 32 * ((p & 7) >> 2) + 16 * (j >> 2) + 4 * quad + (j & 3);
                    }
                    m[b] |= *reinterpret_cast<const uint32_t *>(codes + t * kHeadDim + c0) << (BITS * e);
                }
            }
            // byte i of m[b] = byte b of the word of channel c0 + i
            const uint32_t t01 = __builtin_amdgcn_perm(m[1], m[0], 0x05010400u), u01 = __builtin_amdgcn_perm(m[1], m[0], 0x07030602u);
            const uint32_t t23 = __builtin_amdgcn_perm(m[3], m[2], 0x05010400u), u23 = __builtin_amdgcn_perm(m[3], m[2], 0x07030602u);
            const uint32_t wv[4] = {__builtin_amdgcn_perm(t23, t01, 0x05040100u), __builtin_amdgcn_perm(t23, t01, 0x07060302u),
                                    __builtin_amdgcn_perm(u23, u01, 0x05040100u), __builtin_amdgcn_perm(u23, u01, 0x07060302u)};
            const int base = (((BITS == 4 ? blk * 2 : 0) + h) * 4 + quad) * 64;
            uint32_t *vs = reinterpret_cast<uint32_t *>(lds_vout);
#pragma unroll
            for (int i = 0; i < 4; ++i) vs[base + (4 * n4 + i) * 4 + k] = wv[i];
        }
        __syncthreads();
        // The V words and the two V metadata planes are adjacent in the record: one run of 16-byte stores,
        // every instruction of a wavefront a whole KiB, written once
        constexpr int n_chunks = (R::kCodeBytes + 2 * kMetaBytes) / 16;   // 192 (INT2) / 320 (INT4)
        uint4 *dst = reinterpret_cast<uint4 *>(rec + R::kVCodes);
#pragma unroll
        for (int c = tid; c < n_chunks; c += 256) store_once(dst + c, lds_vout[c]);
        return;
    }
    if (valid) {
        const int mi = vmeta_index(slot, g);
        reinterpret_cast<uint16_t *>(rec + R::kVScale)[mi] = v_scale;
        reinterpret_cast<uint16_t *>(rec + R::kVZero)[mi] = v_zero;
    }
#pragma unroll
    for (int widx = tid; widx < n_words; widx += 256) {
        const int jl = widx & 3, n = (widx >> 2) & 15, quad = (widx >> 6) & 3, jh = (widx >> 8) & 1;
        const int blk = widx >> 9;   // INT4 only (0 for INT2)
        const int c = (jh * 4 + jl) * 16 + n;
        uint32_t val = 0, mask = 0;
#pragma unroll
        for (int p = 0; p < 32 / BITS; ++p) {
            int t;
            if (BITS == 4) {
                const int j = 2 * (p & 3) + (p >> 2);
                t = 32 * blk + 16 * (j >> 2) + 4 * quad + (j & 3);
            } else {
                const int j = 2 * (p & 3) + (p >> 3);
                t = 32 * ((p & 7) >> 2) + 16 * (j >> 2) + 4 * quad + (j & 3);
            }
            const uint32_t field = ((1u << BITS) - 1u) << (BITS * p);
            if (lds_valid[t]) {
                val |= (uint32_t)codes[t * kHeadDim + c] << (BITS * p);
                mask |= field;
            }
        }
        if (mask == 0xffffffffu) vc[widx] = val;
        else if (mask) vc[widx] = (vc[widx] & ~mask) | val;
    }
}

template <bool KC>
__global__ __launch_bounds__(256) void tkv_append_kernel(
    uint8_t *__restrict__ pool, uint8_t *__restrict__ bit_map, const uint16_t *__restrict__ K,
    const uint16_t *__restrict__ V, const uint8_t *__restrict__ tag_bits, int n_tokens,
    const int32_t *__restrict__ work_pages, const int32_t *__restrict__ work_src, int n_kv_heads,
    int n_pages_int2, int n_pages_int4, int32_t *status)
{
    __shared__ __attribute__((aligned(16))) uint32_t lds_codes[kPageTokens][32];
    __shared__ uint8_t lds_valid[kPageTokens];
    // a whole page's V words and V metadata planes in record order, on their way to 16-byte stores
    __shared__ uint4 lds_vout[(Rec<4>::kCodeBytes + 2 * kMetaBytes) / 16];
    __shared__ typename std::conditional<KC, KcLds, NoLds>::type kl;
    const int w = blockIdx.x / n_kv_heads, head = blockIdx.x % n_kv_heads;
    const int page = work_pages[w];
    if (page < 0 || page >= n_pages_int2 + n_pages_int4) {
        if (status && threadIdx.x == 0) atomicOr(status, TKV_STATUS_PAGE_RANGE);
        return;
    }
    const int bits = page < n_pages_int2 ? 2 : 4;
    const int slot = threadIdx.x >> 2;
    const int src = work_src[(size_t)w * kPageTokens + slot];
    bool valid = src >= 0 && src < n_tokens;
    if (valid && tag_bits[src] != bits) {
        valid = false;
        if (status && (threadIdx.x & 3) == 0) atomicOr(status, TKV_STATUS_TAG_MISMATCH);
    }
    uint8_t *rec = pool + record_offset(page, head, n_kv_heads, n_pages_int2);
    if constexpr (KC) {
        if (bits == 2) {
            // a block of 32 slots is quantised in one piece: it takes part whole or not at all
            if (threadIdx.x < 2) kl.n_in_block[threadIdx.x] = 0;
            __syncthreads();
            if ((threadIdx.x & 3) == 0 && valid) atomicAdd(&kl.n_in_block[slot >> 5], 1);
            __syncthreads();
            const int n = kl.n_in_block[slot >> 5];
            if (n != 0 && n != kGroup) {
                valid = false;
                if (status && (threadIdx.x & 127) == 0) atomicOr(status, TKV_STATUS_BLOCK_PARTIAL);
            }
            append_record<2, true>(rec, K, V, src, valid, head, n_kv_heads, lds_codes, lds_valid, lds_vout, kl);
        } else {
            append_record<4, false>(rec, K, V, src, valid, head, n_kv_heads, lds_codes, lds_valid, lds_vout, kl);
        }
    } else {
        if (bits == 2) append_record<2, false>(rec, K, V, src, valid, head, n_kv_heads, lds_codes, lds_valid, lds_vout, kl);
        else append_record<4, false>(rec, K, V, src, valid, head, n_kv_heads, lds_codes, lds_valid, lds_vout, kl);
    }
    if (head == 0 && __syncthreads_or(valid) && threadIdx.x == 0) bit_map[page] = (uint8_t)bits;
}

} // namespace

int tkv_launch_append(const tkv_desc *desc, void *pool, uint8_t *bit_map, const void *K, const void *V,
                      const uint8_t *tag_bits, int32_t n_tokens, const int32_t *work_pages,
                      const int32_t *work_src, int32_t n_work, int32_t *status, void *stream)
{
    const dim3 grid((unsigned)(n_work * desc->n_kv_heads)), block(256);
    const bool kc = desc->int2_key_axis == TKV_KEYS_PER_CHANNEL;
    auto kernel = kc ? tkv_append_kernel<true> : tkv_append_kernel<false>;
    // The kernel is bound by the memory system, which serves four resident workgroups per compute unit
    // slightly faster than the eight that would fit (cfg2: 282 vs 294 us; 3 -> 282, 2 -> 339, 6 -> 286): unused
    // dynamic LDS holds the residency at four.  The per-channel-key kernel's own 33 KB do the same.
    const size_t pad_lds = kc ? 0 : 24 * 1024;
    hipLaunchKernelGGL(kernel, grid, block, pad_lds, (hipStream_t)stream, (uint8_t *)pool, bit_map,
                       (const uint16_t *)K, (const uint16_t *)V, tag_bits, n_tokens, work_pages, work_src,
                       desc->n_kv_heads, desc->n_pages_int2, desc->n_pages_int4, status);
    return hipGetLastError() == hipSuccess ? TKV_OK : TKV_ERR_HIP;
}
