// tkv_gather_dequant: the prefill gather (paper Sec. 3.2.3 "Prefill"): reads the
// pages of a matched prefix from the mixed-precision pool, unpacks every
// listed slot, dequantises it into FP16 and writes dense K / V rows in the
// caller's token order, ready for an FP16 prefill attention kernel.
//
// One workgroup of 256 threads owns one (page, kv head) record, the mirror
// image of the append kernel.  Thread (slot = tid/4, part = tid%4) produces
// channels 32*i + 8*part .. +7 of its token for the four groups i: one
// 16-byte load fetches its K codes of all four groups, and each of its four
// 16-byte stores per tensor completes a 64-byte line together with the three
// neighbouring threads.  V is stored channel-major (a word holds several
// tokens of one channel), so the V words are expanded into an LDS byte tile
// first and each thread reads its token's codes back.
//
// Value: binary16 nearest-even of the exact code * scale + zero.  The fp16
// fused multiply-add gives exactly that: code, scale and zero are fp16
// numbers and the FMA rounds once.
#include <hip/hip_runtime.h>
#include <hip/hip_fp16.h>

#include "tkv_internal.h"
#include "tkv_layout.h"

namespace {

using namespace tkv;

typedef _Float16 half2_t __attribute__((ext_vector_type(2)));

// Two code bytes of w (BYTE and BYTE + 1) as a pair of fp16 numbers: the byte under the bit pattern 0x6400
// is 1024 + code (the fp16 spacing there is 1), and subtracting 1024 is exact.
template <int BYTE> __device__ __forceinline__ half2_t code_pair(uint32_t w)
{
    // v_perm_b32 picks bytes from {w, 0x64646464}: selector bytes 4..7 address w, 0 the constant
    constexpr uint32_t sel = (4u + BYTE) | (0u << 8) | ((5u + BYTE) << 16) | (0u << 24);
    const uint32_t biased = __builtin_amdgcn_perm(w, 0x64646464u, sel);
    const half2_t k = {(_Float16)1024.0f, (_Float16)1024.0f};
    return __builtin_bit_cast(half2_t, biased) - k;
}
// Eight codes (one per byte of lo, hi) times scale plus zero -> eight fp16 values.
__device__ __forceinline__ uint4 dequant8(uint32_t lo, uint32_t hi, _Float16 s, _Float16 z)
{
    const half2_t sv = {s, s}, zv = {z, z};
    return make_uint4(__builtin_bit_cast(uint32_t, __builtin_elementwise_fma(code_pair<0>(lo), sv, zv)),
                      __builtin_bit_cast(uint32_t, __builtin_elementwise_fma(code_pair<2>(lo), sv, zv)),
                      __builtin_bit_cast(uint32_t, __builtin_elementwise_fma(code_pair<0>(hi), sv, zv)),
                      __builtin_bit_cast(uint32_t, __builtin_elementwise_fma(code_pair<2>(hi), sv, zv)));
}
// The same with one (scale, zero) pair per code: s01 .. s67 and z01 .. z67 are fp16 pairs in code order.
__device__ __forceinline__ uint4 dequant8_each(uint32_t lo, uint32_t hi, const uint32_t (&sp)[4], const uint32_t (&zp)[4])
{
    auto f = [](half2_t c, uint32_t s, uint32_t z) {
        return __builtin_bit_cast(uint32_t, __builtin_elementwise_fma(c, __builtin_bit_cast(half2_t, s), __builtin_bit_cast(half2_t, z)));
    };
    return make_uint4(f(code_pair<0>(lo), sp[0], zp[0]), f(code_pair<2>(lo), sp[1], zp[1]),
                      f(code_pair<0>(hi), sp[2], zp[2]), f(code_pair<2>(hi), sp[3], zp[3]));
}
// Eight consecutive sub-byte codes starting at bit `shift` of w -> one code per byte.
template <int BITS> __device__ __forceinline__ void spread8(uint32_t w, int shift, uint32_t &lo, uint32_t &hi)
{
    constexpr uint32_t m = (1u << BITS) - 1u;
    const uint32_t v = w >> shift;
    lo = (v & m) | (((v >> BITS) & m) << 8) | (((v >> (2 * BITS)) & m) << 16) | (((v >> (3 * BITS)) & m) << 24);
    hi = ((v >> (4 * BITS)) & m) | (((v >> (5 * BITS)) & m) << 8) | (((v >> (6 * BITS)) & m) << 16) |
         (((v >> (7 * BITS)) & m) << 24);
}

// KC: the keys of this (INT2) record are quantised per channel over blocks of 32 slots.
template <int BITS, bool KC>
__device__ __forceinline__ void gather_record(const uint8_t *__restrict__ rec, uint16_t *__restrict__ K_out,
                                              uint16_t *__restrict__ V_out, int dst, bool valid, int head,
                                              int n_kv_heads, uint8_t (*codes)[kHeadDim], uint16_t *vmeta)
{
    using R = Rec<BITS>;
    const int tid = threadIdx.x, slot = tid >> 2, part = tid & 3;
    const int tile = slot >> 4, row = slot & 15;

    // ---- V planes -> LDS: scale and zero as stored, codes one per byte [token][channel]
    if (tid < 128) reinterpret_cast<uint2 *>(vmeta)[tid] = reinterpret_cast<const uint2 *>(rec + R::kVScale)[tid];   // 512 B scale, 512 B zero
    // four words of four adjacent channels at a time, so that a token's four codes go out as one 32-bit write
    const uint32_t *vc = reinterpret_cast<const uint32_t *>(rec + R::kVCodes);
    constexpr int n_quads = R::kCodeBytes / 16;   // 256 (INT4) / 128 (INT2)
    if (tid < n_quads) {
        const int jl = tid & 3, nq = (tid >> 2) & 3, quad = (tid >> 4) & 3, jh = (tid >> 6) & 1;
        const int blk = tid >> 7;   // INT4 only (0 for INT2)
        const int widx = jl + 16 * nq + 64 * quad + 256 * jh + 512 * blk;   // word of channel c0; c0 + k is 4*k words on
        const int c0 = (jh * 4 + jl) * 16 + 4 * nq;
        const uint32_t w0 = vc[widx], w1 = vc[widx + 4], w2 = vc[widx + 8], w3 = vc[widx + 12];
        constexpr uint32_t m = (1u << BITS) - 1u;
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
            const uint32_t four = ((w0 >> (BITS * p)) & m) | (((w1 >> (BITS * p)) & m) << 8) |
                                  (((w2 >> (BITS * p)) & m) << 16) | (((w3 >> (BITS * p)) & m) << 24);
            *reinterpret_cast<uint32_t *>(&codes[t][c0]) = four;
        }
    }

    // ---- K: this thread's 8 channels of each group
    if (valid) {
        const uint4 *kc = reinterpret_cast<const uint4 *>(rec + R::kKCodes);
        // INT4: chunk (tile*4 + part)*16 + row = word `part` (8 channels) of the four groups
        // INT2: chunk (tile*2 + part/2)*16 + row = word part/2 (16 channels); this thread takes half part%2
        const uint4 kw = BITS == 4 ? kc[(tile * 4 + part) * 16 + row] : kc[(tile * 2 + (part >> 1)) * 16 + row];
        const uint32_t w[4] = {kw.x, kw.y, kw.z, kw.w};
        uint4 *out = reinterpret_cast<uint4 *>(K_out + ((size_t)dst * n_kv_heads + head) * kHeadDim);
        if constexpr (KC) {
            // channels 32*i + 8*part + j: chunks (block, group i, quarter 2*(part/2) + j/4) of the planes, fp16
            // half part%2 of word j%4.  Each plane is 1 KiB per record and stays in cache.
            const uint4 *sp4 = reinterpret_cast<const uint4 *>(rec + R::kKScale) + (slot >> 5) * 16 + 2 * (part >> 1);
            const uint4 *zp4 = reinterpret_cast<const uint4 *>(rec + R::kKZero) + (slot >> 5) * 16 + 2 * (part >> 1);
            const uint32_t sel = (part & 1) ? 0x07060302u : 0x05040100u;   // v_perm: the chosen halves of (second, first)
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const uint4 s0 = sp4[4 * i], s1 = sp4[4 * i + 1], z0 = zp4[4 * i], z1 = zp4[4 * i + 1];
                const uint32_t sp[4] = {__builtin_amdgcn_perm(s0.y, s0.x, sel), __builtin_amdgcn_perm(s0.w, s0.z, sel),
                                        __builtin_amdgcn_perm(s1.y, s1.x, sel), __builtin_amdgcn_perm(s1.w, s1.z, sel)};
                const uint32_t zp[4] = {__builtin_amdgcn_perm(z0.y, z0.x, sel), __builtin_amdgcn_perm(z0.w, z0.z, sel),
                                        __builtin_amdgcn_perm(z1.y, z1.x, sel), __builtin_amdgcn_perm(z1.w, z1.z, sel)};
                uint32_t lo, hi;
                spread8<BITS>(w[i], 16 * (part & 1), lo, hi);
                out[4 * i + part] = dequant8_each(lo, hi, sp, zp);
            }
        } else {
        const uint2 ksc = reinterpret_cast<const uint2 *>(rec + R::kKScale)[slot];
        const uint2 kzc = reinterpret_cast<const uint2 *>(rec + R::kKZero)[slot];
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const uint32_t sc = i < 2 ? ksc.x : ksc.y, zc = i < 2 ? kzc.x : kzc.y;
            const _Float16 s = __builtin_bit_cast(_Float16, (uint16_t)(sc >> (16 * (i & 1))));
            const _Float16 z = __builtin_bit_cast(_Float16, (uint16_t)(zc >> (16 * (i & 1))));
            uint32_t lo, hi;
            spread8<BITS>(w[i], BITS == 4 ? 0 : 16 * (part & 1), lo, hi);
            out[4 * i + part] = dequant8(lo, hi, s, z);
        }
        }
    }
    __syncthreads();
    // ---- V: codes from the byte tile, scale / zero from the staged planes
    if (valid) {
        uint4 *out = reinterpret_cast<uint4 *>(V_out + ((size_t)dst * n_kv_heads + head) * kHeadDim);
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int mi = vmeta_index(slot, i);
            const _Float16 s = __builtin_bit_cast(_Float16, vmeta[mi]);
            const _Float16 z = __builtin_bit_cast(_Float16, vmeta[kPageTokens * kGroups + mi]);
            const uint2 cb = *reinterpret_cast<const uint2 *>(&codes[slot][32 * i + 8 * part]);
            out[4 * i + part] = dequant8(cb.x, cb.y, s, z);
        }
    }
}

template <bool KC>
__global__ __launch_bounds__(256) void tkv_gather_kernel(
    const uint8_t *__restrict__ pool, const uint8_t *__restrict__ bit_map, const int32_t *__restrict__ work_pages,
    const int32_t *__restrict__ work_dst, int n_kv_heads, int n_pages_int2, int n_pages_int4,
    uint16_t *__restrict__ K_out, uint16_t *__restrict__ V_out, int n_tokens, int32_t *status)
{
    __shared__ __attribute__((aligned(16))) uint8_t codes[kPageTokens][kHeadDim];
    __shared__ __attribute__((aligned(16))) uint16_t vmeta[2 * kPageTokens * kGroups];
    const int w = blockIdx.x / n_kv_heads, head = blockIdx.x % n_kv_heads;
    const int page = work_pages[w];
    if (page < 0 || page >= n_pages_int2 + n_pages_int4) {
        if (status && threadIdx.x == 0) atomicOr(status, TKV_STATUS_PAGE_RANGE);
        return;
    }
    const int bits = page < n_pages_int2 ? 2 : 4;
    if (bit_map[page] != bits) {   // never written, or written at another width: nothing to read
        if (status && threadIdx.x == 0) atomicOr(status, TKV_STATUS_BITMAP_MISMATCH);
        return;
    }
    const int slot = threadIdx.x >> 2;
    const int dst = work_dst[(size_t)w * kPageTokens + slot];
    const bool valid = dst >= 0 && dst < n_tokens;
    if (dst >= n_tokens && status && (threadIdx.x & 3) == 0) atomicOr(status, TKV_STATUS_DST_RANGE);
    const uint8_t *rec = pool + record_offset(page, head, n_kv_heads, n_pages_int2);
    if (bits == 2) gather_record<2, KC>(rec, K_out, V_out, dst, valid, head, n_kv_heads, codes, vmeta);
    else gather_record<4, false>(rec, K_out, V_out, dst, valid, head, n_kv_heads, codes, vmeta);
}

} // namespace

int tkv_launch_gather(const tkv_desc *desc, const void *pool, const uint8_t *bit_map, const int32_t *work_pages,
                      const int32_t *work_dst, int32_t n_work, void *K_out, void *V_out, int32_t n_tokens,
                      int32_t *status, void *stream)
{
    const dim3 grid((unsigned)(n_work * desc->n_kv_heads)), block(256);
    auto kernel = desc->int2_key_axis == TKV_KEYS_PER_CHANNEL ? tkv_gather_kernel<true> : tkv_gather_kernel<false>;
    hipLaunchKernelGGL(kernel, grid, block, 0, (hipStream_t)stream, (const uint8_t *)pool, bit_map,
                       work_pages, work_dst, desc->n_kv_heads, desc->n_pages_int2, desc->n_pages_int4,
                       (uint16_t *)K_out, (uint16_t *)V_out, n_tokens, status);
    return hipGetLastError() == hipSuccess ? TKV_OK : TKV_ERR_HIP;
}
