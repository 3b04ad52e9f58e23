// Measurement probes: what the memory system of the device delivers to the access patterns of the kernels, with
// none of their arithmetic.  They compute nothing of the method.
//   tkv_probe_stream_read   a plain 128-bit streaming read of a device buffer (the decode kernel is a read-only scan
//                           of the packed pool: this is its ceiling beside the published HBM peak)
//   tkv_probe_decode_reads  the records a decode plan reads, fetched in the decode kernel's decomposition (one
//                           wavefront per (work item, kv head), whole records of 6 or 10 KiB, one in flight)
//   tkv_probe_stream_mix    a streaming read of one buffer and write of another in a fixed byte ratio (the append
//                           reads four bytes for every byte it writes, the prefill gather the reverse)
#include <hip/hip_runtime.h>

#include "tkv_internal.h"
#include "tkv_layout.h"

namespace {

using namespace tkv;

__global__ __launch_bounds__(256) void tkv_probe_read_kernel(const uint4 *__restrict__ buf, size_t n, uint32_t *sink)
{
    size_t i = blockIdx.x * (size_t)blockDim.x + threadIdx.x;
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    uint32_t acc = 0;
    for (; i < n; i += stride) {
        const uint4 v = load_once(buf + i);
        acc ^= v.x ^ v.y ^ v.z ^ v.w;
    }
    // keeps the loads alive; a lane's xor of its share hits this value once in 2^32
    if (acc == 0x5a17c0deu && sink) atomicOr(sink, 1u);
}

// One record = n16 16-byte chunks per lane.  The next record is asked for as soon as the current one has arrived,
// as in the decode kernel.
__device__ __forceinline__ uint32_t fold(uint4 v) { return v.x ^ v.y ^ v.z ^ v.w; }

// walk = 1: addresses come from the item and the page tables, as in the decode kernel (items -> token counts ->
// page ids -> record): the memory skeleton of that kernel.  walk = 0: wavefront w reads records w, w + W, w + 2W, ...
// of the pool (W wavefronts), addresses computed, nothing read but the records.
__global__ __launch_bounds__(64) void tkv_probe_records_kernel(
    const uint8_t *__restrict__ pool, const int32_t *__restrict__ page_indptr, const int32_t *__restrict__ page_ids,
    const int32_t *__restrict__ n_tok_int2, const int32_t *__restrict__ n_tok_int4, const int32_t *__restrict__ items,
    int batch, int n_kv_heads, int n_pages_int2, int n_pages_int4, int walk, uint32_t *sink)
{
    const int lane = threadIdx.x;
    const int n_total = n_pages_int2 + n_pages_int4;
    uint32_t acc = 0;
    auto read_record = [&](int page, int head, uint4 (&r)[10]) {
        const uint4 *rec = reinterpret_cast<const uint4 *>(pool + record_offset(page, head, n_kv_heads, n_pages_int2));
        const bool wide = page >= n_pages_int2;
#pragma unroll
        for (int i = 0; i < 10; ++i)
            if (i < 6 || wide) r[i] = load_once(rec + i * 64 + lane);
    };
    auto fold_record = [&](int page, const uint4 (&r)[10]) {
        const bool wide = page >= n_pages_int2;
#pragma unroll
        for (int i = 0; i < 10; ++i)
            if (i < 6 || wide) acc ^= fold(r[i]);
    };
    uint4 r[10];
    if (walk) {
        const int item = blockIdx.x / n_kv_heads, kvh = blockIdx.x % n_kv_heads;
        const int seq = items[4 * item];
        if (seq < 0 || seq >= batch) return;
        const int np2 = (n_tok_int2[seq] + kPageTokens - 1) / kPageTokens, np4 = (n_tok_int4[seq] + kPageTokens - 1) / kPageTokens;
        const int seq_pages = page_indptr[seq + 1] - page_indptr[seq];
        const int np_all = np2 + np4 < seq_pages ? np2 + np4 : seq_pages;
        const int pb = items[4 * item + 1] > 0 ? items[4 * item + 1] : 0;
        const int pe = items[4 * item + 2] < np_all ? items[4 * item + 2] : np_all;
        if (pb >= pe) return;
        const int32_t *pages = page_ids + page_indptr[seq];
        auto page_at = [&](int pi) {
            const int pg = __builtin_amdgcn_readfirstlane(pages[pi]);
            return pg >= 0 && pg < n_total ? pg : 0;   // an id outside the pool: read page 0 instead
        };
        int page = page_at(pb);
        read_record(page, kvh, r);
        for (int pi = pb; pi < pe; ++pi) {
            const int next = page_at(pi + 1 < pe ? pi + 1 : pi);
            fold_record(page, r);
            read_record(next, kvh, r);
            page = next;
        }
    } else {
        const int n_rec = n_total * n_kv_heads;
        int k = blockIdx.x;
        if (k >= n_rec) return;
        read_record(k / n_kv_heads, k % n_kv_heads, r);
        while (k < n_rec) {
            const int kn = k + (int)gridDim.x < n_rec ? k + (int)gridDim.x : k;
            fold_record(k / n_kv_heads, r);
            read_record(kn / n_kv_heads, kn % n_kv_heads, r);
            if (kn == k) break;
            k = kn;
        }
    }
    if (acc == 0x5a17c0deu && sink) atomicOr(sink, 1u);
}

// Reads 16 * RD bytes for every 16 * WR bytes written, both as grid-stride streams of 16-byte accesses; ordinary
// loads and non-temporal stores, the fastest of the four combinations at these ratios.
template <int RD, int WR>
__global__ __launch_bounds__(256) void tkv_probe_mix_kernel(const uint4 *__restrict__ src, uint4 *__restrict__ dst, size_t n_units)
{
    size_t u = blockIdx.x * (size_t)blockDim.x + threadIdx.x;
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    for (; u < n_units; u += stride) {
        uint4 a = make_uint4(0u, 0u, 0u, 0u);
#pragma unroll
        for (int i = 0; i < RD; ++i) {
            const uint4 v = src[(size_t)i * n_units + u];
            a.x ^= v.x; a.y ^= v.y; a.z ^= v.z; a.w ^= v.w;
        }
#pragma unroll
        for (int i = 0; i < WR; ++i) store_once(dst + (size_t)i * n_units + u, a);
    }
}

} // namespace

int tkv_launch_probe_records(const tkv_desc *desc, const void *pool, const int32_t *page_indptr, const int32_t *page_ids,
                             const int32_t *n_tok_int2, const int32_t *n_tok_int4, const int32_t *items, int32_t n_items,
                             int32_t batch, int32_t walk, uint32_t *sink, void *stream)
{
    hipLaunchKernelGGL(tkv_probe_records_kernel, dim3((unsigned)(n_items * desc->n_kv_heads)), dim3(64), 0, (hipStream_t)stream,
                       (const uint8_t *)pool, page_indptr, page_ids, n_tok_int2, n_tok_int4, items, batch, desc->n_kv_heads,
                       desc->n_pages_int2, desc->n_pages_int4, walk, sink);
    return hipGetLastError() == hipSuccess ? TKV_OK : TKV_ERR_HIP;
}

int tkv_launch_probe_mix(const void *src, void *dst, size_t n_units, int32_t read_parts, int32_t write_parts, void *stream)
{
    int dev = 0, cus = 0;
    if (hipGetDevice(&dev) != hipSuccess ||
        hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus <= 0)
        return TKV_ERR_HIP;
    const dim3 grid((unsigned)(cus * 8)), block(256);
    if (read_parts == 4 && write_parts == 1)
        hipLaunchKernelGGL((tkv_probe_mix_kernel<4, 1>), grid, block, 0, (hipStream_t)stream, (const uint4 *)src, (uint4 *)dst, n_units);
    else if (read_parts == 1 && write_parts == 4)
        hipLaunchKernelGGL((tkv_probe_mix_kernel<1, 4>), grid, block, 0, (hipStream_t)stream, (const uint4 *)src, (uint4 *)dst, n_units);
    else if (read_parts == 1 && write_parts == 1)
        hipLaunchKernelGGL((tkv_probe_mix_kernel<1, 1>), grid, block, 0, (hipStream_t)stream, (const uint4 *)src, (uint4 *)dst, n_units);
    else
        return TKV_ERR_INVALID_ARG;
    return hipGetLastError() == hipSuccess ? TKV_OK : TKV_ERR_HIP;
}

int tkv_launch_probe_read(const void *buf, size_t bytes, uint32_t *sink, void *stream)
{
    int dev = 0, cus = 0;
    if (hipGetDevice(&dev) != hipSuccess ||
        hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus <= 0)
        return TKV_ERR_HIP;
    const size_t n = bytes / 16;
    hipLaunchKernelGGL(tkv_probe_read_kernel, dim3((unsigned)(cus * 8)), dim3(256), 0, (hipStream_t)stream,
                       (const uint4 *)buf, n, sink);
    return hipGetLastError() == hipSuccess ? TKV_OK : TKV_ERR_HIP;
}
