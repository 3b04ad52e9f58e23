// tkv_gather_dequant: the prefill gather (paper Sec. 3.2.3 "Prefill"): reads the
// pages of a matched prefix from the mixed-precision pool, unpacks every
// listed slot, dequantises it into FP16 and writes dense K / V rows in the
// caller's token order, ready for an FP16 prefill attention kernel.
//
// A workgroup of 256 threads handles one (page, kv head) record at a time, the
// mirror image of the append kernel, and loops over records with the next
// record's loads already in flight.  Thread (slot = tid/4, part = tid%4) produces
// channels 32*i + 8*part .. +7 of its token for the four groups i: one
// 16-byte load fetches its K codes of all four groups.  Its four 16-byte
// pieces of a row would each fill a quarter of a line; mirror-image threads of
// two neighbouring slots trade pieces instead, so that eight lanes write one
// whole 128-byte line per store instruction, and the stores are non-temporal
// (the output is written once).  V is stored channel-major (a word holds several
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

// Value of the lane that mirrors this one within its group of eight lanes (lane ^ 7).
__device__ __forceinline__ uint32_t half_mirror(uint32_t v)
{
    return (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x141, 0xf, 0xf, true);
}
__device__ __forceinline__ uint4 half_mirror(uint4 v)
{
    return make_uint4(half_mirror(v.x), half_mirror(v.y), half_mirror(v.z), half_mirror(v.w));
}
__device__ __forceinline__ uint4 pick(bool c, uint4 a, uint4 b) { return c ? a : b; }
// Stores the four 16-byte pieces v[i] (channels 32 i + 8 part .. + 7) of this thread's token row so that every
// store instruction of a wavefront writes whole 128-byte lines: thread (slot, part) and thread (slot ^ 1, 3 - part),
// mirror images within eight lanes, trade one piece per line, and the eight lanes write first the line of the even
// slot's row, then that of the odd slot's.
__device__ __forceinline__ void store_row(uint16_t *__restrict__ out, int dst, bool valid, const uint4 (&v)[4], int slot, int part,
                                          int head, int n_kv_heads)
{
    const bool odd = slot & 1;
    const int dst_other = (int)half_mirror((uint32_t)dst);
    const bool valid_other = half_mirror((uint32_t)valid) != 0;
    const bool valid_even = odd ? valid_other : valid, valid_odd = odd ? valid : valid_other;
    // (a row that is not written gets the address of row 0: no pointer is formed from an index that was never checked)
    const size_t dst_even = valid_even ? (size_t)(odd ? dst_other : dst) : 0, dst_odd = valid_odd ? (size_t)(odd ? dst : dst_other) : 0;
    uint4 *row_even = reinterpret_cast<uint4 *>(out + (dst_even * n_kv_heads + head) * kHeadDim);
    uint4 *row_odd = reinterpret_cast<uint4 *>(out + (dst_odd * n_kv_heads + head) * kHeadDim);
#pragma unroll
    for (int h = 0; h < 2; ++h) {
        const uint4 recv = half_mirror(pick(odd, v[2 * h], v[2 * h + 1]));
        if (valid_even) store_once(row_even + 8 * h + (odd ? 7 - part : part), pick(odd, recv, v[2 * h]));
        if (valid_odd) store_once(row_odd + 8 * h + (odd ? 4 + part : 3 - part), pick(odd, v[2 * h + 1], recv));
    }
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

// What one thread requests from HBM for one (page, kv head) record.  The requests of the next record are
// issued before the current one is processed, so that a compute unit always has loads and stores in flight
// (workgroups that start together would otherwise all read, then all compute, then all store).
struct Stage {
    uint4 kw;         // K codes of this thread's token: its 8 channels of each of the four groups
    uint2 ksc, kzc;   // K scale / K zero of the token, four groups (per-token keys)
    uint4 km;         // per-channel keys: 16 bytes of the K scale | K zero planes (threads 0..63)
    uint4 vw;         // V words of four adjacent channels (threads 0..n_quads-1)
    uint2 vm;         // 8 bytes of the V scale | V zero planes (threads 0..127)
    int dst;          // output row of this thread's slot, or -1
    int page;         // workgroup-uniform; -1 = page id outside the pool, nothing was requested
    int bm;           // bit_map entry of the page
};
static_assert(sizeof(Stage) % 4 == 0, "plain dwords");

// KC: the keys of an INT2 record are quantised per channel over blocks of 32 slots.
template <int BITS, bool KC>
__device__ __forceinline__ void load_planes(Stage &st, const uint8_t *__restrict__ rec)
{
    using R = Rec<BITS>;
    const int tid = threadIdx.x, slot = tid >> 2, part = tid & 3;
    const int tile = slot >> 4, row = slot & 15;
    const uint4 *kc = reinterpret_cast<const uint4 *>(rec + R::kKCodes);
    // INT4: chunk (tile*4 + part)*16 + row = word `part` (8 channels) of the four groups
    // INT2: chunk (tile*2 + part/2)*16 + row = word part/2 (16 channels); this thread takes half part%2
    // read once, and an instruction of a wavefront covers 1 KiB (INT4) or 512 B (INT2) of whole lines
    st.kw = load_once(kc + (BITS == 4 ? (tile * 4 + part) * 16 + row : (tile * 2 + (part >> 1)) * 16 + row));
    if constexpr (KC) {
        if (tid < 64) st.km = reinterpret_cast<const uint4 *>(rec + R::kKScale)[tid];   // 512 B scale, 512 B zero
    } else {
        st.ksc = reinterpret_cast<const uint2 *>(rec + R::kKScale)[slot];
        st.kzc = reinterpret_cast<const uint2 *>(rec + R::kKZero)[slot];
    }
    if (tid < 128) st.vm = reinterpret_cast<const uint2 *>(rec + R::kVScale)[tid];   // 512 B scale, 512 B zero
    constexpr int n_quads = R::kCodeBytes / 16;   // 256 (INT4) / 128 (INT2)
    if (tid < n_quads) {
        const uint32_t *vc = reinterpret_cast<const uint32_t *>(rec + R::kVCodes);
        const int jl = tid & 3, nq = (tid >> 2) & 3, quad = (tid >> 4) & 3, jh = (tid >> 6) & 1;
        const int blk = tid >> 7;   // INT4 only (0 for INT2)
        const int widx = jl + 16 * nq + 64 * quad + 256 * jh + 512 * blk;   // word of channel c0; c0 + k is 4*k words on
        st.vw = make_uint4(vc[widx], vc[widx + 4], vc[widx + 8], vc[widx + 12]);
    }
}

template <bool KC>
__device__ __forceinline__ void load_stage(Stage &st, int r, const uint8_t *__restrict__ pool,
                                           const uint8_t *__restrict__ bit_map, const int32_t *__restrict__ work_pages,
                                           const int32_t *__restrict__ work_dst, int n_kv_heads, int n_pages_int2,
                                           int n_pages_int4, int32_t *status)
{
    const int w = r / n_kv_heads, head = r % n_kv_heads;
    const int page = work_pages[w];
    if (page < 0 || page >= n_pages_int2 + n_pages_int4) {
        if (status && threadIdx.x == 0) atomicOr(status, TKV_STATUS_PAGE_RANGE);
        st = Stage{};
        st.page = -1;
        return;
    }
    st.page = page;
    st.dst = work_dst[(size_t)w * kPageTokens + (threadIdx.x >> 2)];
    st.bm = bit_map[page];
    const uint8_t *rec = pool + record_offset(page, head, n_kv_heads, n_pages_int2);
    if (page < n_pages_int2) load_planes<2, KC>(st, rec);
    else load_planes<4, false>(st, rec);
}

struct GatherLds {
    alignas(16) uint8_t codes[kPageTokens][kHeadDim];     // V codes, one per byte [token][channel]
    alignas(16) uint16_t vmeta[2 * kPageTokens * kGroups];   // V scale plane, V zero plane, as stored
    alignas(16) uint4 kmeta[64];                           // per-channel keys: K scale plane, K zero plane
};

template <int BITS, bool KC>
__device__ __forceinline__ void gather_record(const Stage &st, uint16_t *__restrict__ K_out, uint16_t *__restrict__ V_out,
                                              bool valid, int head, int n_kv_heads, GatherLds &lds)
{
    using R = Rec<BITS>;
    const int tid = threadIdx.x, slot = tid >> 2, part = tid & 3;

    // ---- V planes -> LDS: scale and zero as stored, codes one per byte [token][channel]
    if (tid < 128) reinterpret_cast<uint2 *>(lds.vmeta)[tid] = st.vm;
    if constexpr (KC) {
        if (tid < 64) lds.kmeta[tid] = st.km;
    }
    // four words of four adjacent channels at a time, so that a token's four codes go out as one 32-bit write
    constexpr int n_quads = R::kCodeBytes / 16;
    if (tid < n_quads) {
        const int jl = tid & 3, nq = (tid >> 2) & 3, quad = (tid >> 4) & 3, jh = (tid >> 6) & 1;
        const int blk = tid >> 7;
        const int c0 = (jh * 4 + jl) * 16 + 4 * nq;
        const uint32_t w0 = st.vw.x, w1 = st.vw.y, w2 = st.vw.z, w3 = st.vw.w;
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
            *reinterpret_cast<uint32_t *>(&lds.codes[t][c0]) = four;
        }
    }

    // ---- K: this thread's 8 channels of each group (per-token keys need nothing from LDS)
    const uint32_t w[4] = {st.kw.x, st.kw.y, st.kw.z, st.kw.w};
    if constexpr (!KC) {
        uint4 kv[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const uint32_t sc = i < 2 ? st.ksc.x : st.ksc.y, zc = i < 2 ? st.kzc.x : st.kzc.y;
            const _Float16 s = __builtin_bit_cast(_Float16, (uint16_t)(sc >> (16 * (i & 1))));
            const _Float16 z = __builtin_bit_cast(_Float16, (uint16_t)(zc >> (16 * (i & 1))));
            uint32_t lo, hi;
            spread8<BITS>(w[i], BITS == 4 ? 0 : 16 * (part & 1), lo, hi);
            kv[i] = dequant8(lo, hi, s, z);
        }
        store_row(K_out, st.dst, valid, kv, slot, part, head, n_kv_heads);
    }
    __syncthreads();
    if constexpr (KC) {
        {
            uint4 kv[4];
            // channels 32*i + 8*part + j: chunks (block, group i, quarter 2*(part/2) + j/4) of the planes, fp16
            // half part%2 of word j%4
            const uint4 *sp4 = lds.kmeta + (slot >> 5) * 16 + 2 * (part >> 1);
            const uint4 *zp4 = sp4 + 32;
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
                kv[i] = dequant8_each(lo, hi, sp, zp);
            }
            store_row(K_out, st.dst, valid, kv, slot, part, head, n_kv_heads);
        }
    }
    // ---- V: codes from the byte tile, scale / zero from the staged planes
    {
        uint4 vv[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int mi = vmeta_index(slot, i);
            const _Float16 s = __builtin_bit_cast(_Float16, lds.vmeta[mi]);
            const _Float16 z = __builtin_bit_cast(_Float16, lds.vmeta[kPageTokens * kGroups + mi]);
            const uint2 cb = *reinterpret_cast<const uint2 *>(&lds.codes[slot][32 * i + 8 * part]);
            vv[i] = dequant8(cb.x, cb.y, s, z);
        }
        store_row(V_out, st.dst, valid, vv, slot, part, head, n_kv_heads);
    }
}

// Workgroup b handles records b, b + gridDim.x, ... (record = work page * n_kv_heads + head).  The LDS tile is
// double-buffered: one barrier per record (a thread can be at most one record ahead of the slowest).
template <bool KC>
__global__ __launch_bounds__(256) void tkv_gather_kernel(
    const uint8_t *__restrict__ pool, const uint8_t *__restrict__ bit_map, const int32_t *__restrict__ work_pages,
    const int32_t *__restrict__ work_dst, int n_records, int n_kv_heads, int n_pages_int2, int n_pages_int4,
    uint16_t *__restrict__ K_out, uint16_t *__restrict__ V_out, int n_tokens, int32_t *status)
{
    __shared__ GatherLds lds[2];
    int r = blockIdx.x;
    if (r >= n_records) return;
    Stage cur{}, nxt{};
    load_stage<KC>(cur, r, pool, bit_map, work_pages, work_dst, n_kv_heads, n_pages_int2, n_pages_int4, status);
    nxt = cur;
    int buf = 0;
    for (; r < n_records; r += gridDim.x) {
        const int rn = r + gridDim.x;
        if (rn < n_records)
            load_stage<KC>(nxt, rn, pool, bit_map, work_pages, work_dst, n_kv_heads, n_pages_int2, n_pages_int4, status);
        if (cur.page >= 0) {
            const int bits = cur.page < n_pages_int2 ? 2 : 4;
            // a page that was never written, or written at another width, has been read (its address is valid)
            // and nothing of it is stored
            const bool written = cur.bm == bits;
            if (!written && status && threadIdx.x == 0) atomicOr(status, TKV_STATUS_BITMAP_MISMATCH);
            const bool valid = written && cur.dst >= 0 && cur.dst < n_tokens;
            if (written && cur.dst >= n_tokens && status && (threadIdx.x & 3) == 0) atomicOr(status, TKV_STATUS_DST_RANGE);
            const int head = r % n_kv_heads;
            if (bits == 2) gather_record<2, KC>(cur, K_out, V_out, valid, head, n_kv_heads, lds[buf]);
            else gather_record<4, false>(cur, K_out, V_out, valid, head, n_kv_heads, lds[buf]);
            buf ^= 1;
        }
        cur = nxt;
    }
}

} // namespace

int tkv_launch_gather(const tkv_desc *desc, const void *pool, const uint8_t *bit_map, const int32_t *work_pages,
                      const int32_t *work_dst, int32_t n_work, void *K_out, void *V_out, int32_t n_tokens,
                      int32_t *status, void *stream)
{
    // A few looping workgroups per compute unit, fewer than would fit: the kernel is bound by the HBM write
    // stream (82 % of its bytes are stores), and on MI355X that stream runs faster with few concurrent
    // writers (cfg2, per-token keys: 271 / 243 / 243 / 249 us with 2 / 3 / 4 / 6 workgroups per unit).
    const bool kc = desc->int2_key_axis == TKV_KEYS_PER_CHANNEL;
    auto kernel = kc ? tkv_gather_kernel<true> : tkv_gather_kernel<false>;
    int dev = 0, cus = 0, per_cu = 0;
    if (hipGetDevice(&dev) != hipSuccess ||
        hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus <= 0 ||
        hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, kernel, 256, 0) != hipSuccess || per_cu <= 0)
        return TKV_ERR_HIP;
    const int wanted = 3;
    per_cu = per_cu < wanted ? per_cu : wanted;
    const int n_records = n_work * desc->n_kv_heads;
    const int n_blocks = n_records < cus * per_cu ? n_records : cus * per_cu;
    const dim3 grid((unsigned)n_blocks), block(256);
    hipLaunchKernelGGL(kernel, grid, block, 0, (hipStream_t)stream, (const uint8_t *)pool, bit_map,
                       work_pages, work_dst, n_records, desc->n_kv_heads, desc->n_pages_int2, desc->n_pages_int4,
                       (uint16_t *)K_out, (uint16_t *)V_out, n_tokens, status);
    return hipGetLastError() == hipSuccess ? TKV_OK : TKV_ERR_HIP;
}
