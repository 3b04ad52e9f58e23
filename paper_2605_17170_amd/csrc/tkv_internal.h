// Internal interface between the host-side validation (tkv_host.cpp) and the
// kernel launchers (tkv_append.hip, tkv_gather.hip, tkv_decode.hip,
// tkv_probe.hip).  Arguments are already
// validated; the launchers return TKV_OK or TKV_ERR_HIP.
#ifndef TKV_INTERNAL_H
#define TKV_INTERNAL_H

#include "tkv.h"

int tkv_launch_append(const tkv_desc *desc, void *pool, uint8_t *bit_map, const void *K, const void *V,
                      const uint8_t *tag_bits, int32_t n_tokens, const int32_t *work_pages,
                      const int32_t *work_src, int32_t n_work, int32_t *status, void *stream);

int tkv_launch_gather(const tkv_desc *desc, const void *pool, const uint8_t *bit_map, const int32_t *work_pages,
                      const int32_t *work_dst, int32_t n_work, void *K_out, void *V_out, int32_t n_tokens,
                      int32_t *status, void *stream);

int tkv_launch_probe_read(const void *buf, size_t bytes, uint32_t *sink, void *stream);
int tkv_launch_probe_records(const tkv_desc *desc, const void *pool, const int32_t *page_indptr, const int32_t *page_ids,
                             const int32_t *n_tok_int2, const int32_t *n_tok_int4, const int32_t *items, int32_t n_items,
                             int32_t batch, int32_t walk, uint32_t *sink, void *stream);
int tkv_launch_probe_mix(const void *src, void *dst, size_t n_units, int32_t read_parts, int32_t write_parts, void *stream);

int tkv_launch_decode_split(const tkv_desc *desc, const void *pool, const uint8_t *bit_map, const void *q,
                            const int32_t *page_indptr, const int32_t *page_ids, const int32_t *n_tok_int2,
                            const int32_t *n_tok_int4, const int32_t *items, int32_t n_items, int32_t batch,
                            int32_t n_q_heads, float sm_scale, void *workspace, int32_t *status, void *stream);

int tkv_launch_decode_reduce(const tkv_desc *desc, const int32_t *seq_item_indptr, int32_t n_items, int32_t batch,
                             int32_t n_q_heads, float *out, const void *workspace, void *stream);


// Argument checks shared by the decode entry points (tkv_host.cpp); TKV_OK or a negative status.
int tkv_decode_check_args(const tkv_desc *desc, int32_t n_items, int32_t batch, int32_t n_q_heads,
                          const void *workspace, size_t workspace_bytes);

#endif
