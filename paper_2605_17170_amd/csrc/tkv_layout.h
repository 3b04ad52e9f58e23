// Device-side constants of the page layout (fixed geometry: 64 tokens per
// page, head_dim 128, groups of 32 channels).  A record holds one (page, kv
// head): K codes | K scale | K zero | V codes | V scale | V zero.  The INT2
// pool precedes the INT4 pool in one address space split by an offset
// (paper Sec. 3.2.2).
#ifndef TKV_LAYOUT_H
#define TKV_LAYOUT_H

#include <stdint.h>

namespace tkv {

constexpr int kPageTokens = 64;
constexpr int kHeadDim = 128;
constexpr int kGroup = 32;
constexpr int kGroups = kHeadDim / kGroup;       // 4
constexpr int kMetaBytes = kPageTokens * kGroups * 2;   // one fp16 plane: 512 B

template <int BITS> struct Rec {
    static constexpr int kCodeBytes = kPageTokens * kHeadDim * BITS / 8;   // 2048 / 4096
    static constexpr int kKCodes = 0;
    static constexpr int kKScale = kCodeBytes;
    static constexpr int kKZero = kCodeBytes + kMetaBytes;
    static constexpr int kVCodes = kCodeBytes + 2 * kMetaBytes;
    static constexpr int kVScale = 2 * kCodeBytes + 2 * kMetaBytes;
    static constexpr int kVZero = 2 * kCodeBytes + 3 * kMetaBytes;
    static constexpr int kBytes = 2 * kCodeBytes + 4 * kMetaBytes;         // 6144 / 10240
};

// Byte offset of the record of (page, head); the caller has checked the range.
__host__ __device__ inline int64_t record_offset(int page, int head, int n_kv_heads, int n_pages_int2)
{
    if (page < n_pages_int2) return ((int64_t)page * n_kv_heads + head) * Rec<2>::kBytes;
    return (int64_t)n_pages_int2 * n_kv_heads * Rec<2>::kBytes +
           ((int64_t)(page - n_pages_int2) * n_kv_heads + head) * Rec<4>::kBytes;
}

// fp16 index of (token t, group g) in the V scale / V zero planes: chunks of 8
// tokens [t/32][(t%16)/4][g][j], j = 4*((t/16)%2) + t%4.
__host__ __device__ inline int vmeta_index(int t, int g)
{
    return ((((t >> 5) * 4 + ((t & 15) >> 2)) * 4 + g) << 3) + (((t >> 4) & 1) << 2) + (t & 3);
}

// fp16 index of (block blk = t/32, channel c) in the K scale / K zero planes of an INT2 page whose keys are
// quantised per channel: 128 positions per block, in chunks of 8 per (group c/32, quarter); a chunk is what
// one lane of the decode kernel's q operand holds: the pair (c, c+8) of k = c%4 at 2k, 2k+1.
__host__ __device__ inline int kcmeta_index(int blk, int c)
{
    const int g = c >> 5, r = c & 31;
    const int quarter = 2 * (r >> 4) + ((r & 7) >> 2);
    return ((((blk * 4 + g) * 4 + quarter) << 3) + 2 * (r & 3) + ((r & 15) >> 3));
}

// A 16-byte load of data that is read once (the records of the packed cache: every byte is used once per call).
// Non-temporal: on MI355X a plain 800 MB read runs at 7.0 TB/s with such loads and at 6.3 TB/s with ordinary
// ones.  Only where one load instruction of a wavefront covers whole 128-byte lines: a line shared with a later
// instruction would be fetched again.
__device__ __forceinline__ uint4 load_once(const uint4 *p)
{
    typedef uint32_t u32x4_t __attribute__((ext_vector_type(4)));
    const u32x4_t t = __builtin_nontemporal_load(reinterpret_cast<const u32x4_t *>(p));
    return make_uint4(t.x, t.y, t.z, t.w);
}

// The counterpart for data that is written once and not read again by the same kernel.  Only where one store
// instruction of a wavefront fills whole 128-byte lines (a plain 1 : 4 read : write stream of such stores runs at
// 6.2 TB/s against 5.0 TB/s with ordinary ones); on lines filled by several instructions it is slower than an
// ordinary store.
__device__ __forceinline__ void store_once(uint4 *p, uint4 v)
{
    typedef uint32_t u32x4_t __attribute__((ext_vector_type(4)));
    const u32x4_t t = {v.x, v.y, v.z, v.w};
    __builtin_nontemporal_store(t, reinterpret_cast<u32x4_t *>(p));
}
__device__ __forceinline__ void store_once(uint32_t *p, uint32_t v) { __builtin_nontemporal_store(v, p); }
__device__ __forceinline__ void store_once(uint16_t *p, uint16_t v) { __builtin_nontemporal_store(v, p); }

} // namespace tkv
#endif
