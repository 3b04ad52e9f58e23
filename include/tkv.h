/*
 * tkv.h -- C ABI of libtkv: TriAxialKV's decode / append hot path on AMD
 * MI355X (gfx950).
 *
 * The library quantises newly written bf16 keys / values at a per-token
 * bitwidth (INT2 or INT4, chosen upstream from the token's temporal x
 * modality x semantic-role tag) into a paged mixed-precision KV pool, and
 * runs decode attention over that pool with on-the-fly dequantisation.
 *
 * Conventions
 *  - Every function returns an int status (TKV_OK = 0, errors negative)
 *    unless its type says otherwise; nothing throws, aborts or prints.
 *  - "host" pointers are ordinary CPU memory; "device" pointers are HIP
 *    device memory on the current device.  The caller owns every buffer and
 *    the stream.  The library allocates no device memory, never synchronises
 *    a stream and keeps no global state: calls on different streams are
 *    independent.
 *  - Argument checks that are possible from host-visible values are done
 *    before anything is launched, so a bad call launches nothing.
 *  - Geometry is fixed in this version: head_dim 128, group_size 32,
 *    page_tokens 64; other values return TKV_ERR_BAD_SHAPE.
 *  - bf16 and fp16 values are raw 16-bit patterns.
 */
#ifndef TKV_H
#define TKV_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

enum {
    TKV_OK = 0,
    TKV_ERR_INVALID_ARG = -1,        /* null pointer, negative count, misaligned buffer */
    TKV_ERR_BAD_BITS = -2,           /* a bitwidth other than 2 or 4                      */
    TKV_ERR_BAD_SHAPE = -3,          /* unsupported geometry / head counts                */
    TKV_ERR_PAGE_RANGE = -4,         /* page id outside its pool                          */
    TKV_ERR_POOL_EXHAUSTED = -5,     /* allocator has too few free pages (state unchanged) */
    TKV_ERR_WORKSPACE_TOO_SMALL = -6,
    TKV_ERR_HIP = -7,                /* a launch failed; see hipGetLastError               */
    TKV_ERR_CAPACITY = -8            /* an output array supplied by the caller is too small */
};

/* Bits the kernels may OR into the optional device status word. */
enum {
    TKV_STATUS_TAG_MISMATCH = 1,     /* append: tag_bits[token] differs from its page's pool width (token skipped) */
    TKV_STATUS_BITMAP_MISMATCH = 2,  /* decode: bit_map[page] differs from the width its position implies (page skipped) */
    TKV_STATUS_PAGE_RANGE = 4,       /* a page id read on the device lies outside the pool (page skipped) */
    TKV_STATUS_DST_RANGE = 8,        /* tkv_gather_dequant: an output row index >= n_tokens (slot skipped) */
    TKV_STATUS_BLOCK_PARTIAL = 16,   /* append, per-channel INT2 keys: a 32-token block arrived incomplete (block skipped) */
    TKV_STATUS_SCALE_SATURATED = 32, /* decode: a stored V scale above 255, or a per-channel INT2 key scale above 1023, was
                                        clamped: the output is finite but not the attention over the stored values */
    TKV_STATUS_BAD_ITEM = 64         /* decode: a work item names a sequence outside the batch (it contributes nothing)
                                        or a partial slot outside the workspace (its partial is not stored) */
};

const char *tkv_strerror(int status);

/*
 * Pool geometry.  Pages [0, n_pages_int2) form the INT2 pool, pages
 * [n_pages_int2, n_pages_int2 + n_pages_int4) the INT4 pool: one address
 * space split by an offset, so a page's precision is one comparison
 * (paper Sec. 3.2.2, "Shared address space").
 */
typedef struct tkv_desc {
    int32_t n_kv_heads;
    int32_t head_dim;       /* 128 */
    int32_t group_size;     /* 32  */
    int32_t page_tokens;    /* 64  */
    int32_t n_pages_int2;
    int32_t n_pages_int4;
    int32_t int2_key_axis;  /* TKV_KEYS_PER_TOKEN or TKV_KEYS_PER_CHANNEL */
} tkv_desc;

/*
 * Quantisation axis of the keys in the INT2 pool (Sec. 3.2.1, "Bitwidths and
 * quantization axes").  Values and INT4 keys are always per token: a group is
 * 32 consecutive channels of one token.
 *   TKV_KEYS_PER_TOKEN    INT2 keys are grouped the same way.
 *   TKV_KEYS_PER_CHANNEL  the paper's scheme: the 32 tokens of a block (slots
 *       0..31 or 32..63 of an INT2 page) share one (scale, zero-point) pair
 *       per channel.  A block is quantised in one piece, so INT2 tokens arrive
 *       in whole blocks: the stream of a sequence's INT2 tokens always holds a
 *       multiple of 32 tokens, and tokens that do not fill a block are stored
 *       at INT4 (tkv_route_residual).  The record size is the same; the K
 *       scale / K zero planes hold fp16 [block][128 channel positions].
 */
enum { TKV_KEYS_PER_TOKEN = 0, TKV_KEYS_PER_CHANNEL = 1 };

/* Bytes of one (page, kv head) record: 6144 for bits = 2, 10240 for bits = 4, 0 otherwise
 * (codes of K and V plus fp16 scale and zero-point per group of 32 channels, Sec. 3.2.1). */
size_t tkv_record_bytes(int bits);
/* Bytes of one page of the INT2 (bits = 2) or INT4 (bits = 4) pool: n_kv_heads records, the unit the per-pool
 * allocators hand out (Sec. 3.2.2, "Memory allocation").  0 on a bad descriptor or width; host only. */
size_t tkv_page_bytes(const tkv_desc *desc, int bits);
/* Bytes of the mixed-precision pool: the INT2 pages followed by the INT4 pages in ONE buffer, so that a page id
 * below n_pages_int2 is an INT2 page and any other an INT4 page (Sec. 3.2.2, "Shared address space": the split
 * point is fixed when the pool is sized from the average bitwidth).  The caller allocates this much device
 * memory, 256-byte aligned, and owns it.  0 on a bad descriptor; host only. */
size_t tkv_pool_bytes(const tkv_desc *desc);
/* Byte offset of the record of (page, head) inside the pool, or (size_t)-1 if out of range. */
size_t tkv_record_offset(const tkv_desc *desc, int32_t page, int32_t head);

/* ------------------------------------------------------------------ */
/* Page allocators (host).  One free list per pool, no coordination     */
/* between them (Sec. 3.2.2, "Memory allocation").                      */
/* ------------------------------------------------------------------ */
typedef struct tkv_alloc tkv_alloc;

/* shuffle_seed = 0: pages are handed out in increasing order; otherwise each
 * free list is shuffled with a generator seeded by it (scattered pages). */
int tkv_alloc_create(const tkv_desc *desc, uint64_t shuffle_seed, tkv_alloc **out);
void tkv_alloc_destroy(tkv_alloc *a);
/* Take n free pages of the given width into page_ids_out (host, n entries).
 * On TKV_ERR_POOL_EXHAUSTED nothing is taken. */
int tkv_alloc_pages(tkv_alloc *a, int bits, int32_t n, int32_t *page_ids_out);
/* Return pages to their pools (width follows from the id).  A page that is
 * out of range or already free gives TKV_ERR_PAGE_RANGE and nothing is freed. */
int tkv_free_pages(tkv_alloc *a, const int32_t *page_ids, int32_t n);
int32_t tkv_alloc_free_count(const tkv_alloc *a, int bits);

/* ------------------------------------------------------------------ */
/* Per-sequence page table (host).  A sequence owns two page streams:   */
/* its INT2 tokens fill INT2 pages in arrival order, its INT4 tokens    */
/* INT4 pages.  Listing INT2 pages before INT4 pages is the partition   */
/* that lets decode run width-homogeneous work (Sec. 3.2.3, "Decode",   */
/* phase 1).                                                            */
/* ------------------------------------------------------------------ */
typedef struct tkv_seq tkv_seq;

int tkv_seq_create(tkv_seq **out);
void tkv_seq_destroy(tkv_seq *s);                      /* does not return pages */
int tkv_seq_release(tkv_seq *s, tkv_alloc *a);         /* returns every page, empties the sequence */
int32_t tkv_seq_n_tokens(const tkv_seq *s, int bits);  /* tokens stored at this width */
int32_t tkv_seq_n_pages(const tkv_seq *s, int bits);
/* Copy the page list, INT2 pages first then INT4 pages, into out (host,
 * capacity entries).  Returns the number of pages or TKV_ERR_CAPACITY. */
int32_t tkv_seq_page_ids(const tkv_seq *s, int32_t *out, int32_t capacity);

/* ------------------------------------------------------------------ */
/* T1: triaxial tagger and tag -> bitwidth lookup (host).               */
/* ------------------------------------------------------------------ */
/*
 * A token's tag is a point of temporal x modal x semantic (Sec. 3.1):
 *   semantic  0 inst, 1 user, 2 assistant, 3 reasoning, 4 tool_call, 5 obs, 6 delim
 *   modal     0 text, 1 image
 *   temporal  0 older, 1 turn_m2, 2 turn_m1, 3 current
 * tag code = (temporal * 2 + modal) * 7 + semantic, 56 codes (TKV_N_TAGS).
 * tkv_tag_tokens derives the temporal axis in one scan from the per-token
 * semantic role and modality that the chat template gives (host, u8[n_tokens]
 * each): a turn runs from one user message up to, not including, the next;
 * a user message starts at a `user` token that does not follow a `user`
 * token; tokens before the first user message are turn 0.  tags_out: host
 * u8[n_tokens].  TKV_ERR_INVALID_ARG on a null array or an axis value out of
 * range (nothing is written then).
 * tkv_tags_to_bits looks every tag up in the calibrated map b*: S -> {2, 4}
 * (table, host u8[56]) and yields the per-token bitwidth array that
 * tkv_plan_append and tkv_quantize_append take (Sec. 3.2.3, "Tagging").
 * TKV_ERR_INVALID_ARG on a tag >= 56, TKV_ERR_BAD_BITS on a table entry other
 * than 2 or 4.  tkv_tag_counts adds the tokens of each tag to counts (host
 * i64[56], the N_k of Eq. 3); the caller zeroes it first.
 */
enum { TKV_N_TAGS = 56 };
int tkv_tag_tokens(const uint8_t *semantic, const uint8_t *modal, int32_t n_tokens, uint8_t *tags_out);
int tkv_tags_to_bits(const uint8_t *tags, int32_t n_tokens, const uint8_t *table, uint8_t *bits_out);
int tkv_tag_counts(const uint8_t *tags, int32_t n_tokens, int64_t *counts);

/* ------------------------------------------------------------------ */
/* A1: tag -> bitwidth allocation (host).                               */
/* ------------------------------------------------------------------ */
/*
 * Chooses b_k in {2, 4} for every tag k so that the total distortion
 * sum_k D_k(b_k) is small under the budget sum_k N_k b_k <= B sum_k N_k
 * (Sec. 3.1.3, Eq. 3).  All arrays are host memory.
 *   n_tags   number of tags (the paper's triaxial space has 56)
 *   N        i64[n_tags]  token count of each tag, >= 0
 *   D2, D4   f64[n_tags]  distortion of the tag at 2 / 4 bits, finite
 *   B        target average bitwidth, 2 <= B <= 4
 *   bits_out u8[n_tags]   2 or 4 per tag
 * The budget is T = B * sum N in binary64 with a relative slack of 2^-40 (a
 * decimal B is not a binary64 number); bits in use are counted exactly.
 * tkv_allocate_bits_greedy is Alg. 1: per-bit gain rho_k = (D_k(2) - D_k(4)) /
 * (2 N_k) (Eq. 4; +inf / 0 / -inf by the sign of the gain when N_k = 0), tags
 * visited by rho descending (ties in tag order), a tag is upgraded whenever its
 * 2 N_k extra bits still fit.  tkv_allocate_bits_exhaustive visits all 2^n_tags
 * allocations (n_tags <= 22, as in the paper) and returns the feasible one of
 * least total distortion; ties go to fewer total bits, then to the smaller mask
 * (tag 0 = lowest bit, set = 4 bits).
 * Errors: TKV_ERR_INVALID_ARG (null array, negative count, non-finite distortion,
 * B outside [2, 4], n_tags < 0 or > 22 for the exhaustive search).
 */
int tkv_allocate_bits_greedy(int32_t n_tags, const int64_t *N, const double *D2, const double *D4,
                             double B, uint8_t *bits_out);
int tkv_allocate_bits_exhaustive(int32_t n_tags, const int64_t *N, const double *D2, const double *D4,
                                 double B, uint8_t *bits_out);

/* ------------------------------------------------------------------ */
/* Q1: route newly arrived tokens to slots (host).                      */
/* ------------------------------------------------------------------ */
/*
 * Residual policy of the per-channel INT2 keys (Sec. 3.2.1): of the tokens
 * tagged INT2 in tag_bits (host, u8[n_tokens], one arriving chunk of one
 * sequence) the last (count mod 32) do not fill a block and are stored at
 * INT4.  bits_out (host, u8[n_tokens], may alias tag_bits) receives the
 * per-token widths to hand to tkv_plan_append and tkv_quantize_append.
 * Errors: TKV_ERR_INVALID_ARG, TKV_ERR_BAD_BITS.
 */
int tkv_route_residual(const uint8_t *tag_bits, int32_t n_tokens, uint8_t *bits_out);

/* Upper bound of pages one tkv_plan_append call over n_tokens can touch. */
int32_t tkv_plan_append_max_work(int32_t n_tokens);
/*
 * tag_bits (host, u8[n_tokens]) is the per-token bitwidth array produced by
 * the tagger and the tag -> bitwidth table (Sec. 3.2.3, "Tagging").  Tokens
 * of each width are appended, in order, to the sequence's page stream of that
 * width; new pages come from the matching allocator.  Outputs (host):
 *   slot_ids_out[n_tokens]      page_id * 64 + slot of every token (the
 *                               per-token pointer of the page table);
 *   work_pages_out[max_work]    the distinct pages that receive tokens;
 *   work_src_out[max_work*64]   for each such page and slot, token_base +
 *                               index of the token that goes there, or -1;
 *   *n_work_out                 number of pages listed.
 * token_base lets several sequences' plans address one concatenated K/V
 * tensor.  With TKV_KEYS_PER_CHANNEL the number of INT2 tokens must be a
 * multiple of 32 (TKV_ERR_INVALID_ARG otherwise; see tkv_route_residual).
 * On any error the sequence and the allocator are left unchanged.
 */
int tkv_plan_append(tkv_alloc *a, tkv_seq *s, const uint8_t *tag_bits, int32_t n_tokens,
                    int32_t token_base, int32_t *slot_ids_out, int32_t *work_pages_out,
                    int32_t *work_src_out, int32_t max_work, int32_t *n_work_out);

/* ------------------------------------------------------------------ */
/* Q2-Q5: quantise and pack (device).                                   */
/* ------------------------------------------------------------------ */
/*
 * For every listed page and kv head: asymmetric min/max quantisation of each
 * group of 32 channels of each arriving token (zero = fp16(min), scale =
 * fp16((max-min)/(2^b-1)), code = round-half-even((x-zero)*(1/scale)) clamped),
 * per-token for K and V at both widths, or, with TKV_KEYS_PER_CHANNEL, the
 * keys of INT2 pages per channel over each block of 32 slots (Sec. 3.2.1),
 * packed into the page's planes; bit_map[page] is set to the page's width.
 * Bits of slots whose work_src entry is -1 are left untouched.  With
 * TKV_KEYS_PER_CHANNEL the 32 slots of a block of an INT2 page must all be
 * named or all be -1; a block named in part is skipped (keys and values) and
 * TKV_STATUS_BLOCK_PARTIAL is raised.
 *   pool       device, tkv_pool_bytes(desc) bytes, 256-byte aligned
 *   bit_map    device u8[n_pages_int2 + n_pages_int4]
 *   K, V       device bf16 [n_tokens, n_kv_heads, head_dim], contiguous
 *   tag_bits   device u8[n_tokens]; a token whose width differs from its
 *              page's pool is skipped and TKV_STATUS_TAG_MISMATCH is raised
 *   work_pages device i32[n_work], work_src device i32[n_work*64] as written
 *              by tkv_plan_append; a page may appear at most once per call
 *   status     device i32, may be NULL; kernels OR TKV_STATUS_* bits into it
 * group_size must be 32.  n_work = 0 is a no-op.
 */
int tkv_quantize_append(const tkv_desc *desc, void *pool, uint8_t *bit_map,
                        const void *K, const void *V, const uint8_t *tag_bits,
                        int32_t n_tokens, int32_t group_size,
                        const int32_t *work_pages, const int32_t *work_src, int32_t n_work,
                        int32_t *status, void *stream /* hipStream_t */);

/* ------------------------------------------------------------------ */
/* P1: prefill gather-dequant (device).                                 */
/* ------------------------------------------------------------------ */
/*
 * Reads the listed pages of a matched prefix from the pool, unpacks every
 * listed slot, dequantises it into FP16 and writes dense K / V rows for an
 * FP16 prefill attention kernel (Sec. 3.2.3, "Prefill").  Each value is the
 * binary16 nearest-even rounding of the exact code * scale + zero.
 *   pool, bit_map  device, as filled by tkv_quantize_append
 *   work_pages     device i32[n_work]: the pages to read, each at most once
 *   work_dst       device i32[n_work*64]: for each page and slot the output
 *                  row (token index) or -1 to skip the slot; the lists that
 *                  tkv_plan_append wrote (work_pages_out, work_src_out) name
 *                  exactly the rows the tokens came from
 *   K_out, V_out   device fp16 [n_tokens, n_kv_heads, head_dim], contiguous,
 *                  16-byte aligned; rows that no slot names are left untouched
 *   status         device i32, may be NULL: TKV_STATUS_PAGE_RANGE (page id
 *                  outside the pool), TKV_STATUS_BITMAP_MISMATCH (page never
 *                  written at its pool's width), TKV_STATUS_DST_RANGE; the
 *                  page or slot concerned is skipped
 * n_work = 0 is a no-op.
 */
int tkv_gather_dequant(const tkv_desc *desc, const void *pool, const uint8_t *bit_map,
                       const int32_t *work_pages, const int32_t *work_dst, int32_t n_work,
                       void *K_out, void *V_out, int32_t n_tokens,
                       int32_t *status, void *stream /* hipStream_t */);

/* ------------------------------------------------------------------ */
/* D1: cut page lists into work items (host).                           */
/* ------------------------------------------------------------------ */
/*
 * Split-K over a sequence's page list (Sec. 3.2.3, "Decode"): a work item is a
 * contiguous range of one sequence's page list (INT2 pages first); one
 * wavefront per (item, kv head) leaves a partial (m, l, acc) that
 * tkv_decode_reduce merges.  Items are balanced by decode cost (an INT2 page
 * weighs 6, an INT4 page 7): the planner finds the smallest bound on an item's
 * cost for which the batch still splits into at most target_items items and
 * cuts every sequence into equal parts below that bound, so the number of items
 * never exceeds target_items unless there are more non-empty sequences than
 * that (then one item each).
 * A plan depends only on the page COUNTS of the sequences: it stays valid while
 * tokens are appended to open pages (the kernel reads the token counts from the
 * device arrays and masks by them) and must be made again when a sequence gains
 * a page -- at most every 64 decoded tokens per sequence.  With a stale plan the
 * new page is simply not read.  Layers that share a page table share the plan.
 *   page_indptr   host i32[batch+1], page-list offsets of the sequences
 *   n_tok_int2/4  host i32[batch], valid tokens per width (last page may be partial;
 *                 with TKV_KEYS_PER_CHANNEL n_tok_int2 must be a multiple of 32)
 *   target_items  wanted number of items over the whole batch (>= 1)
 *   items_out     host i32[4*capacity]: {sequence, first page, end page, partial
 *                 slot}, page indices relative to the sequence's list.  Items
 *                 are listed in LAUNCH order (the kernel runs item k as its
 *                 k-th group of workgroups): by falling share of INT2 pages,
 *                 so that the wavefronts that end up on one SIMD mix ranges
 *                 that keep it busy (INT2) with ranges that mostly wait for
 *                 memory (INT4).  The partial of an item is written to slot
 *                 `partial slot` of the workspace; the slots are a permutation
 *                 of 0 .. n_items-1 in sequence order.
 *   seq_item_indptr_out  host i32[batch+1]: sequence b owns the partial slots
 *                 [indptr[b], indptr[b+1]); a sequence without tokens has none
 * Returns the number of items (>= 0) or a negative status.
 */
int32_t tkv_plan_decode_capacity(int32_t batch, int32_t target_items);
int32_t tkv_plan_decode(const tkv_desc *desc, int32_t batch, const int32_t *page_indptr,
                        const int32_t *n_tok_int2, const int32_t *n_tok_int4,
                        int32_t target_items, int32_t *items_out, int32_t capacity,
                        int32_t *seq_item_indptr_out);

/* ------------------------------------------------------------------ */
/* D2-D7: decode attention (device).                                    */
/* ------------------------------------------------------------------ */
/* Bytes of workspace that decode attention over n_items work items needs: the partial (m, l, acc[head_dim]) in
 * fp32 of every (item, query head), which the split kernel writes and the cross-split merge reads (Sec. 3.2.3,
 * "Decode": splits merged by log-sum-exp).  Device memory, 16-byte aligned, owned by the caller; it needs no
 * initialisation and may be shared by calls on the same stream.  0 on a bad descriptor or count; host only. */
size_t tkv_decode_workspace_bytes(const tkv_desc *desc, int32_t n_items, int32_t n_q_heads);
/*
 * Decode attention over the mixed-precision paged cache (Sec. 3.2.3, "Decode"):
 * out[b, h, :] = softmax(sm_scale * q[b, h, :] . K^T) V over the dequantised
 * tokens of sequence b's pages, query head h reading kv head
 * h / (n_q_heads / n_kv_heads); every page runs the dequantisation path of its
 * pool (INT2 or INT4).  A sequence with no tokens gives zeros.
 *   pool, bit_map  device, as filled by tkv_quantize_append
 *   q              device bf16 [batch, n_q_heads, head_dim]
 *   page_indptr    device i32[batch+1]
 *   page_ids       device i32[page_indptr[batch]]: per sequence INT2 pages then INT4 pages
 *   n_tok_int2/4   device i32[batch]
 *   items          device i32[4*n_items], seq_item_indptr device i32[batch+1] (tkv_plan_decode)
 *   out            device fp32 [batch, n_q_heads, head_dim]
 *   workspace      device, >= tkv_decode_workspace_bytes(...), 16-byte aligned
 *   status         device i32, may be NULL
 *   items          every item must name a sequence of the batch and a partial
 *                  slot below n_items, each slot once, the slots of a sequence
 *                  as seq_item_indptr lists them.  An item that names no
 *                  sequence of the batch contributes nothing (an empty partial
 *                  in its slot) and raises TKV_STATUS_BAD_ITEM; so does one
 *                  with a slot out of range, which cannot write anything: the
 *                  sequence that owns the slot it should have named then reads
 *                  what the workspace held before.  The page range of an item
 *                  is clamped to the sequence's pages.
 * The page tables on the device must describe the same sequences as the host
 * arrays the plan was made from (tkv_plan_decode above says when a plan ages).
 * Preconditions on the cache contents: stored scales and zeros finite; V scales
 * up to 255 are used exactly, larger ones are clamped there (the kernel forms
 * softmax weight x V scale in fp16 and keeps it finite); with
 * TKV_KEYS_PER_CHANNEL the scales of the INT2 keys likewise up to 1023 (the
 * kernel forms q x K scale in fp16), and every n_tok_int2 is a multiple of 32.
 * A clamped scale raises TKV_STATUS_SCALE_SATURATED: the output is then finite
 * but not the attention over the stored values.
 * n_q_heads / n_kv_heads must be 1, 2, 4 or 8.  Two launches on `stream`:
 * the split kernel, then the cross-split reduction.
 */
int tkv_decode_attention(const tkv_desc *desc, const void *pool, const uint8_t *bit_map,
                         const void *q, const int32_t *page_indptr, const int32_t *page_ids,
                         const int32_t *n_tok_int2, const int32_t *n_tok_int4,
                         const int32_t *items, const int32_t *seq_item_indptr, int32_t n_items,
                         int32_t batch, int32_t n_q_heads, float sm_scale, float *out,
                         void *workspace, size_t workspace_bytes, int32_t *status,
                         void *stream /* hipStream_t */);

/*
 * The two launches of tkv_decode_attention as separate calls, same arguments
 * and the same checks: D2-D6, the split kernel, which leaves one partial
 * (m, l, acc) per work item and query head in `workspace`; and D7, the
 * cross-split merge by log-sum-exp (Sec. 3.2.3), which reads the partials
 * and writes `out`.  tkv_decode_attention is exactly one call of each.
 */
int tkv_decode_split(const tkv_desc *desc, const void *pool, const uint8_t *bit_map,
                     const void *q, const int32_t *page_indptr, const int32_t *page_ids,
                     const int32_t *n_tok_int2, const int32_t *n_tok_int4,
                     const int32_t *items, int32_t n_items, int32_t batch, int32_t n_q_heads,
                     float sm_scale, void *workspace, size_t workspace_bytes, int32_t *status,
                     void *stream /* hipStream_t */);
int tkv_decode_reduce(const tkv_desc *desc, const int32_t *seq_item_indptr, int32_t n_items,
                      int32_t batch, int32_t n_q_heads, float *out, const void *workspace,
                      size_t workspace_bytes, void *stream /* hipStream_t */);

/*
 * tkv_decode_attention for callers that cannot allocate device memory or pass
 * a workspace: code under HIP graph capture, tight serving loops, harnesses
 * that forbid hipMalloc.  Same arguments, same checks, same two launches and
 * the same results; the partials live in a fixed device array inside the
 * library (TKV_DECODE_STATIC_SCRATCH_BYTES per GPU, held until the process
 * ends) instead of a caller workspace.  The call allocates and frees nothing.
 * TKV_ERR_WORKSPACE_TOO_SMALL when tkv_decode_workspace_bytes(desc, n_items,
 * n_q_heads) exceeds the array (nothing is launched); TKV_ERR_HIP when the
 * array's address cannot be obtained.  The device that owns `stream` must be
 * the current device.  All calls on one GPU share the array: two calls whose
 * kernels may overlap in time (different streams, or replays of captured
 * graphs running concurrently) race on it; calls on one stream are ordered
 * and safe.
 */
#define TKV_DECODE_STATIC_SCRATCH_BYTES (16u << 20)
int tkv_decode_attention_static(const tkv_desc *desc, const void *pool, const uint8_t *bit_map,
                                const void *q, const int32_t *page_indptr, const int32_t *page_ids,
                                const int32_t *n_tok_int2, const int32_t *n_tok_int4,
                                const int32_t *items, const int32_t *seq_item_indptr, int32_t n_items,
                                int32_t batch, int32_t n_q_heads, float sm_scale, float *out,
                                int32_t *status, void *stream /* hipStream_t */);

/* ------------------------------------------------------------------ */
/* Measurement aid (device).                                            */
/* ------------------------------------------------------------------ */
/*
 * Streams `bytes` (a multiple of 16) of the device buffer `buf` (16-byte
 * aligned) through the GPU with 128-bit non-temporal loads (the kind the
 * kernels use for the records of the cache) and discards them: the
 * read-bandwidth ceiling of the device for a scan such as the decode kernel's
 * pass over the pool.  For benchmarks that report a kernel against what the
 * memory system delivers as well as against the published peak; it computes
 * nothing of the method.  `sink` (device u32, may be NULL) is never written
 * in practice.  One launch on `stream`; TKV_ERR_INVALID_ARG on a null or
 * misaligned buffer.
 */
int tkv_probe_stream_read(const void *buf, size_t bytes, uint32_t *sink, void *stream /* hipStream_t */);
/*
 * Fetches the records that a decode plan reads, in the decode kernel's own
 * decomposition (Sec. 3.2.3, "Decode": one wavefront per (work item, kv head),
 * whole records, the next one requested when the current one has arrived) and
 * discards them: what the memory system delivers to that access pattern, with
 * none of the arithmetic.
 *   walk = 1  addresses come from the items and the device page tables exactly
 *             as in tkv_decode_split (same arguments, same meaning): the
 *             kernel's memory skeleton, start-up chain included;
 *   walk = 0  wavefront w of the n_items * n_kv_heads reads records w, w + W,
 *             ... of the whole pool, addresses computed; the page tables and
 *             items are not read (may be NULL).
 * sink as for tkv_probe_stream_read.  n_items = 0 or an empty pool is a no-op.
 */
int tkv_probe_decode_reads(const tkv_desc *desc, const void *pool, const int32_t *page_indptr,
                           const int32_t *page_ids, const int32_t *n_tok_int2, const int32_t *n_tok_int4,
                           const int32_t *items, int32_t n_items, int32_t batch, int32_t walk,
                           uint32_t *sink, void *stream /* hipStream_t */);
/*
 * Streams read_parts * unit_bytes out of `src` and writes write_parts *
 * unit_bytes into `dst` (device, 16-byte aligned, unit_bytes a multiple of 16)
 * with 128-bit accesses (ordinary loads, non-temporal stores: the fastest
 * combination): the ceiling of the device for a kernel that reads and
 * writes in that byte ratio.  Supported ratios: 4 : 1 (tkv_quantize_append reads
 * 512 B of bf16 per 96..160 B it writes), 1 : 4 (tkv_gather_dequant), 1 : 1.
 * What is written is a fold of what was read.  unit_bytes = 0 is a no-op.
 */
int tkv_probe_stream_mix(const void *src, void *dst, size_t unit_bytes, int32_t read_parts,
                         int32_t write_parts, void *stream /* hipStream_t */);

#ifdef __cplusplus
}
#endif
#endif /* TKV_H */
