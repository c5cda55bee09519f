/*
 * omni_attn.h — C ABI of the MI355X (gfx950) paged decode-attention library.
 *
 * The operation is the decode-phase attention of the paper's Background
 * section ("Attention computation", Eq. 1): for every decoding request only
 * the query q of its last token takes part,
 *
 *     Attention(q, K, V) = softmax(q K^T / sqrt(d_k)) V ,
 *
 * against the request's cached keys and values, the current token's own k, v
 * included (the latency-model section counts a decode request's load as
 * l_j + 1 tokens).  The KV cache is paged (the paper's engine is a paged-
 * attention one).  Attention piggybacking computes parts of a request's
 * attention in different places (GPU-resident context, context held by CPU
 * hosts whose threads each compute a partial load and aggregate intermediate
 * results — System Implementation, "CPU Attention"); the results come back
 * through an output queue of per-layer attention rows and join the input of
 * the following projection (Asynchronous CPU-GPU interaction).  This library
 * is the GPU side of that data path:
 *
 *   omni_paged_decode_attn  attention of each sequence over a token range of
 *                           its paged context, cut into chunks; one partial
 *                           (O, LSE) per (sequence, chunk, query head);
 *   omni_merge_partials     exact combination of partials of a sequence that
 *                           come from up to four sources into the final row.
 *
 * General rules
 *   - Every data pointer is DEVICE memory owned by the caller.  The library
 *     allocates nothing, frees nothing and keeps no state between calls; the
 *     only scratch it ever uses is the optional workspace the caller passes
 *     (omni_paged_decode_attn_static: a fixed array of its own instead).
 *   - q, the pools, part_o and out_o must be 16-byte aligned (checked: SHAPE).
 *   - Calls enqueue work on `hip_stream` (a hipStream_t passed as void*, NULL =
 *     the default stream) and return without synchronising.
 *   - The return value reports what the host can see: NULL pointers, bad
 *     sizes, unsupported shapes, a failed launch.  Argument structs live in
 *     host memory and are read before the call returns.
 *   - Page indices are checked on the device: a block-table entry outside
 *     [0, num_blocks) makes its 16 tokens count as absent (no access is made);
 *     ctx_end is clamped to max_blocks_per_seq * block_size, ctx_begin to >= 0.
 *   - Supported: block_size 16; head_dim 64 or 128; dtype fp32 or bf16;
 *     num_q_heads a multiple of num_kv_heads with ratio G <= 16.
 *
 * Layouts (row-major, last index fastest)
 *   q            [batch, num_q_heads, head_dim]
 *   k_pool/v_pool[num_blocks, num_kv_heads, block_size, head_dim]
 *                so the 16 x head_dim tile of one (page, kv head) is one
 *                contiguous run (4 KiB for bf16, head_dim 128).  Pools must be
 *                16-byte aligned.
 *   block_table  [batch, max_blocks_per_seq] int32; logical token t of
 *                sequence i is in page block_table[i][t / 16], slot t % 16.
 *   query head j reads kv head j / G.
 *
 * Partials
 *   A partial over a token set R is O_R = sum_{t in R} softmax_R(s)_t v_t
 *   (normalised inside R) with LSE_R = ln sum_{t in R} exp(s_t), s_t =
 *   sm_scale * <q, k_t>, natural logarithm.  Empty R: LSE = -inf and O is not
 *   written.  Merging uses the identity of Eq. 1 over a disjoint union:
 *   w_p = exp(LSE_p - max LSE), O = sum w_p O_p / sum w_p,
 *   LSE = max LSE + ln sum w_p.  A partial with LSE = -inf has weight zero and
 *   its O row is never read; a row with no weight at all gives O = 0,
 *   LSE = -inf.
 */
#ifndef OMNI_ATTN_H
#define OMNI_ATTN_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    OMNI_OK = 0,
    OMNI_ERR_NULL = -1,        /* a required pointer is NULL                      */
    OMNI_ERR_SHAPE = -2,       /* non-positive size, G not integral, bad chunking */
    OMNI_ERR_DTYPE = -3,       /* dtype value not known                           */
    OMNI_ERR_UNSUPPORTED = -4, /* valid but outside the supported set             */
    OMNI_ERR_LAUNCH = -5,      /* HIP reported an error at launch                 */
    OMNI_ERR_TOO_LARGE = -6    /* problem exceeds a fixed limit of the entry point */
} omni_status;

typedef enum { OMNI_F32 = 0, OMNI_BF16 = 1 } omni_dtype;

/* kernel selection for omni_paged_decode_attn */
typedef enum {
    OMNI_KERNEL_AUTO = 0,      /* matrix-core kernel when the shape allows, else the vector one */
    OMNI_KERNEL_VECTOR = 1,    /* vector-ALU kernel, any supported shape                        */
    OMNI_KERNEL_MFMA = 2       /* matrix-core kernel: bf16, head_dim 128 (else UNSUPPORTED)      */
} omni_kernel;

/* One source of partial rows (for the merge, and for the decode call's fused form). */
typedef struct omni_partial_src_s {
    const float*   o;                  /* [n_rows, num_q_heads, head_dim] fp32                 */
    const float*   lse;                /* [n_rows, num_q_heads] fp32, natural log              */
    const int32_t* row_offsets;        /* [batch+1] CSR: rows of sequence i are
                                          row_offsets[i] .. row_offsets[i+1]-1; NULL = dense   */
    int32_t        dense_rows_per_seq; /* dense: rows i*n .. i*n+n-1 belong to sequence i      */
} omni_partial_src;

typedef struct {
    /* problem shape */
    int32_t batch, num_q_heads, num_kv_heads, head_dim, block_size, max_blocks_per_seq;
    int64_t num_blocks;            /* pages in each pool                                      */
    int32_t qkv_dtype;             /* omni_dtype of q, k_pool, v_pool                         */
    float   sm_scale;              /* multiplies q.k; 1/sqrt(head_dim) in Eq. 1               */
    /* inputs (device) */
    const void*    q;
    const void*    k_pool;
    const void*    v_pool;
    const int32_t* block_table;
    const int32_t* ctx_begin;      /* [batch] first token attended; NULL = all zero           */
    const int32_t* ctx_end;        /* [batch] one past the last token attended                */
    /* chunking: chunk c of sequence i covers tokens
     * [ctx_begin[i] + c*chunk_tokens, min(ctx_end[i], ctx_begin[i] + (c+1)*chunk_tokens)).
     * chunk_tokens = 0 means one chunk holding the whole range (max_chunks must be 1).
     * Otherwise chunk_tokens is a positive multiple of block_size and max_chunks >= 1 is the
     * chunk stride of the partial buffers; tokens beyond max_chunks chunks are NOT attended. */
    int32_t chunk_tokens;
    int32_t max_chunks;
    /* outputs (device) */
    float* part_o;                 /* [batch, max_chunks, num_q_heads, head_dim] fp32; may be
                                      NULL if out_o is given and max_chunks == 1              */
    float* part_lse;               /* [batch, max_chunks, num_q_heads] fp32                   */
    /* Final rows.  With out_o, a sequence whose (clamped) range fits one chunk - its only possibly
     * non-empty chunk is chunk 0 - gets its final row from this call: O to out_o [batch, num_q_heads,
     * head_dim] of out_dtype, LSE to out_lse if not NULL (an empty range: O = 0, LSE = -inf).  Such a
     * sequence writes no partial O, and its part_lse slots read -inf (with max_chunks == 1 and partial
     * buffers given, the partial is kept as well).  The other sequences write partials as without out_o
     * and their out_o rows are left alone; seq_final tells which is which.                         */
    void*  out_o;
    int32_t out_dtype;
    float* out_lse;
    int32_t kernel;                /* omni_kernel                                             */
    /* optional scratch for the call's work list (device memory, caller-owned,
     * at least omni_decode_workspace_bytes(batch, max_chunks, num_kv_heads) bytes, 16-byte aligned,
     * contents need not survive between calls).  With it the matrix-core kernel runs in its
     * persistent form: non-empty chunks are listed longest-first and drawn by resident workgroups;
     * the vector kernel launches one workgroup per list entry, in list order (longest first, empty
     * chunk slots last).  NULL selects the plain grid form of either.  Two calls that may overlap
     * in time (different streams) need distinct workspaces.  The 32-bit word at byte 20 of a workspace that
     * holds a list is a diagnostic: the list build zeroes it and a wave that gives a launch up
     * (its bounded wait for the next work item ran out, about a second) adds one; it stays zero
     * in every healthy run, and a non-zero value means rows of some launch since then are missing
     * (omni_decode_abandoned_waves reads and clears it).                                         */
    void*    workspace;
    uint64_t workspace_bytes;
    /* non-zero: the workspace already holds the work list of exactly these ranges and this
     * chunking, written by omni_decode_plan (or by an earlier call with the same ranges): the
     * list is reused instead of rebuilt.  The list depends only on batch, ctx_begin, ctx_end,
     * max_blocks_per_seq, chunk_tokens, max_chunks and num_kv_heads (and, if ext_srcs are named
     * without fuse_merge, on which sequences have rows there), so one plan serves the attention
     * calls of every layer of a decoding iteration.                                           */
    int32_t  workspace_planned;
    /* optional [batch] int32 output: 1 where this call wrote the sequence's final row to out_o /
     * out_lse, 0 where its partial rows still have to be merged (omni_merge_partials_masked takes
     * the array as its skip list).  Required (as are the partial buffers) when out_o is given,
     * fuse_merge == 0 and max_chunks > 1 or ext_srcs are named.                                */
    int32_t* seq_final;
    /* non-zero: every sequence's final row comes out of this call (persistent form of the
     * matrix-core kernel only: a workspace is required, else UNSUPPORTED; out_o is required).
     * Sequences with several non-empty chunks still write their partial rows to part_o / part_lse
     * (scratch in this form: which of their rows a later reader finds is unspecified); the
     * workgroup that finishes a (sequence, kv head)'s last chunk merges them in chunk order.
     * ext_srcs[0 .. n_ext_srcs) (host array of up to 3 sources, copied during the call; NULL / 0 =
     * none) are rows computed elsewhere for these sequences - the attention rows that come back
     * through the output queue - and are folded into the final rows by the same rule, so that a
     * hybrid batch needs no separate merge launch.
     * With fuse_merge == 0 and out_o given, ext_srcs only tell the call which sequences have rows
     * elsewhere (their row counts are read, their O and LSE are not): such a sequence is never
     * finished here - it writes its partial row and seq_final 0 even if its range fits one chunk -
     * so that the merge finds every part of it.  A planned work list records this: plan and call
     * must name the same sources, and the list holds while the row counts do.                  */
    int32_t  fuse_merge;
    const struct omni_partial_src_s* ext_srcs;
    int32_t  n_ext_srcs;
} omni_decode_args;

/*
 * Batched decode attention over a paged KV cache, emitting per-chunk partials
 * (Eq. 1 restricted to each chunk; see "Partials" above).
 * Errors: NULL (q, pools, block_table, ctx_end, or no output given), SHAPE
 * (also a workspace that is too small or misaligned), DTYPE, UNSUPPORTED,
 * LAUNCH.  A batch of zero is OK and does nothing.
 */
omni_status omni_paged_decode_attn(const omni_decode_args* a, void* hip_stream);

/*
 * omni_paged_decode_attn for callers that cannot allocate device memory or pass a workspace: code under
 * HIP graph capture, tight serving loops, harnesses that forbid allocation.  Same arguments, same
 * results and the same kernels in their persistent form, but the work list lives in a scratch array of
 * OMNI_STATIC_SCRATCH_BYTES that is part of the library (one copy per GPU, held until the process ends);
 * a->workspace, workspace_bytes and workspace_planned are ignored and the list is rebuilt by every call.
 * The call allocates nothing and frees nothing.  Limit: omni_decode_workspace_bytes(batch, max_chunks,
 * num_kv_heads) must not exceed OMNI_STATIC_SCRATCH_BYTES (2 MiB: 64 + 16 batch max_chunks + 4 batch
 * num_kv_heads bytes, e.g. batch * max_chunks <= 100 000 at 8 kv heads), else OMNI_ERR_TOO_LARGE and
 * nothing is launched.  Every call on a GPU uses that GPU's one array (each call rewrites all of it that
 * it reads): calls that may overlap in time on one GPU (different streams) race and must be ordered by the
 * caller, or use omni_paged_decode_attn with workspaces of their own.  Other errors as
 * omni_paged_decode_attn.
 */
#define OMNI_STATIC_SCRATCH_BYTES (2u * 1024u * 1024u)
omni_status omni_paged_decode_attn_static(const omni_decode_args* a, void* hip_stream);

/* Bytes of workspace the persistent form needs for this batch, chunk stride and kv-head count: the work
 * list and one arrival counter per (sequence, kv head) (0 if any of them is <= 0). */
uint64_t omni_decode_workspace_bytes(int32_t batch, int32_t max_chunks, int32_t num_kv_heads);

/* Name of the attention kernel omni_paged_decode_attn would launch for these arguments (a static string:
 * "decode_mfma_persistent_kernel", "decode_mfma_grid_kernel" or "decode_vector_kernel"; "" if the call
 * would be refused).  Host only, launches nothing: for measurement reports. */
const char* omni_decode_kernel_name(const omni_decode_args* a);

/*
 * Reads the diagnostic word of a workspace that holds a work list (see `workspace` above) into *count
 * (host memory) and puts it back to zero: the number of waves that gave a launch up since the list was
 * built or the word was last cleared; 0 in every healthy run, anything else means that rows of some
 * launch in between were not written.  workspace = NULL means the static scratch of
 * omni_paged_decode_attn_static on the current device.  Waits for the stream.  Errors: NULL, LAUNCH.
 */
omni_status omni_decode_abandoned_waves(void* workspace, uint32_t* count, void* hip_stream);

/*
 * Build the work list for `a` into a->workspace on the stream, without computing attention: the
 * non-empty (sequence, chunk) ranges in longest-first order.  Reads only the shape, chunking,
 * ctx_begin and ctx_end; a following omni_paged_decode_attn with the same ranges may set
 * workspace_planned.  Errors: as omni_paged_decode_attn, plus NULL if there is no workspace.
 */
omni_status omni_decode_plan(const omni_decode_args* a, void* hip_stream);

/*
 * Merge the partials of every (sequence, query head) found in srcs[0..n_srcs)
 * (1 <= n_srcs <= 4; e.g. split-KV chunks of this GPU, partials computed by
 * other hosts and returned through the output queue, GPU-computed tails) into
 * out_o [batch, num_q_heads, head_dim] of out_dtype and, if not NULL,
 * out_lse [batch, num_q_heads].  The srcs array is host memory, copied during
 * the call.  Errors: NULL, SHAPE (n_srcs out of range, head_dim not 64/128 ...),
 * DTYPE, LAUNCH.
 */
omni_status omni_merge_partials(int32_t batch, int32_t num_q_heads, int32_t head_dim,
                                const omni_partial_src* srcs, int32_t n_srcs,
                                void* out_o, int32_t out_dtype, float* out_lse,
                                void* hip_stream);
/* The same, leaving alone the out_o / out_lse rows of every sequence i with skip[i] != 0 (device int32
 * [batch]; NULL = none): the seq_final array of a decode call that already wrote those final rows. */
omni_status omni_merge_partials_masked(int32_t batch, int32_t num_q_heads, int32_t head_dim,
                                       const omni_partial_src* srcs, int32_t n_srcs, const int32_t* skip,
                                       void* out_o, int32_t out_dtype, float* out_lse,
                                       void* hip_stream);

/*
 * KV-cache data movement around the decode step.
 *
 * The paper's decode context includes the token being decoded (its load is l_j + 1), so the new token's
 * k, v are written into the paged cache before attention runs; and the KV cache of a request moves
 * between GPU and CPU memory as a one-shot swap (KV cache management: swap-out overlapped with compute,
 * delayed swap-in).  These three calls are the device side of both: pure copies, bit-exact.
 */
typedef struct {
    int32_t batch, num_kv_heads, head_dim, block_size, max_blocks_per_seq;
    int64_t num_blocks;
    int32_t dtype;                 /* omni_dtype of the pools                                   */
    void*   k_pool;                /* [num_blocks, num_kv_heads, block_size, head_dim], device  */
    void*   v_pool;
    const int32_t* block_table;    /* [batch, max_blocks_per_seq]; only omni_kv_append reads it  */
} omni_kv_cache;

/*
 * Write k_new / v_new [batch, num_kv_heads, head_dim] (pool dtype, device) into the slot of logical
 * token positions[i] (device int32 [batch]) of every sequence i: page block_table[i][pos/16], slot pos%16.
 * A negative position, one past the table, or a table entry outside [0, num_blocks) writes nothing for
 * that sequence.  Errors: NULL, SHAPE, DTYPE, UNSUPPORTED (block_size != 16, row bytes not a multiple of
 * 16), LAUNCH.
 */
omni_status omni_kv_append(const omni_kv_cache* c, const void* k_new, const void* v_new,
                           const int32_t* positions, void* hip_stream);

/*
 * Copy pages page_ids[0..n_pages) (device int32) of both pools to contiguous staging buffers
 * k_out / v_out [n_pages, num_kv_heads, block_size, head_dim] (swap-out), or back from such buffers into
 * the pools (swap-in).  A page id outside [0, num_blocks) reads as zeros / is skipped.  batch,
 * max_blocks_per_seq and block_table of `c` are not used; n_pages = 0 does nothing.  Errors: NULL, SHAPE, DTYPE, UNSUPPORTED, LAUNCH.
 */
omni_status omni_kv_gather_pages(const omni_kv_cache* c, const int32_t* page_ids, int64_t n_pages,
                                 void* k_out, void* v_out, void* hip_stream);
omni_status omni_kv_scatter_pages(const omni_kv_cache* c, const int32_t* page_ids, int64_t n_pages,
                                  const void* k_in, const void* v_in, void* hip_stream);

/*
 * Device-resident row queues and residual store (System Implementation: "CPU Attention queue" — the
 * input queue of q, k, v rows and the output queue of attention-result rows are tensors in GPU memory with
 * head and tail pointers, producer at the tail, consumer at the head; "Residual management" — a store
 * indexed by request and layer keeps the residual while the request's attention is computed elsewhere).
 * GPU-side operations only; all pointers are device memory, counts stay on the device.
 *
 * A queue is a ring of `capacity` rows of `row_bytes` bytes (a multiple of 16), an optional int32 tag per
 * row (e.g. the request id) and four uint32 state words {head, tail, 0, 0} that the caller zeroes once:
 * head / tail count rows popped / pushed since then, a row with count c lives in slot c % capacity.
 * The ring is at most 2 GiB - 1 bytes (capacity * row_bytes; UNSUPPORTED beyond).
 * Calls on one queue must be ordered (same stream).  Inside a call the rows are written (through the
 * caches, at device scope) before the pointer that announces them; what a later call on the stream sees
 * is ordered by the stream.
 */
typedef struct {
    void*     data;                /* [capacity, row_bytes]                                      */
    int32_t*  tags;                /* [capacity] or NULL                                         */
    uint32_t* state;               /* [4]                                                        */
    int32_t   capacity, row_bytes;
} omni_queue;

/*
 * Push n_rows rows (rows [n_rows, row_bytes], tags [n_rows] or NULL) at the tail — all of them, or, if
 * they do not all fit, none; *n_pushed (device int32, may be NULL) receives n_rows or 0.
 * Errors: NULL, SHAPE (capacity, row_bytes, n_rows), UNSUPPORTED (ring of 2 GiB or more), LAUNCH.
 */
omni_status omni_queue_push(const omni_queue* q, const void* rows, const int32_t* tags, int32_t n_rows,
                            int32_t* n_pushed, void* hip_stream);
/*
 * Pop up to max_rows rows from the head into rows_out [max_rows, row_bytes] (tags into tags_out, may be
 * NULL), oldest first; *n_popped (device int32, may be NULL) receives how many.
 */
omni_status omni_queue_pop(const omni_queue* q, void* rows_out, int32_t* tags_out, int32_t max_rows,
                           int32_t* n_popped, void* hip_stream);

/*
 * Row offsets for rows that came out of an output queue, so that they can be a CSR source of
 * omni_merge_partials without a trip to the host: tags [max_rows] (device) hold the sequence number of each
 * popped row, *n_rows (device int32, NULL = max_rows) how many there are; the tags must be non-decreasing
 * (rows of a sequence together, sequences in batch order: the order a producer that works through the batch
 * pushes them in).  Writes row_offsets [batch + 1] (device): row_offsets[i] = number of rows with a tag below
 * i.  Rows with tags outside [0, batch) fall outside every sequence's range.  Errors: NULL, SHAPE, LAUNCH.
 */
omni_status omni_csr_from_tags(const int32_t* tags, const int32_t* n_rows, int32_t max_rows, int32_t batch,
                               int32_t* row_offsets, void* hip_stream);

/*
 * Residual store [n_slots, row_bytes]: save rows [n_rows, row_bytes] to slots slot_ids[r] (the caller
 * maps (request, layer) to a slot), or load those slots into rows.  Slot ids outside [0, n_slots) are
 * skipped on save and give zero rows on load.  Errors: NULL, SHAPE, LAUNCH.
 */
omni_status omni_residual_save(void* store, int64_t n_slots, int32_t row_bytes, const int32_t* slot_ids,
                               int32_t n_rows, const void* rows, void* hip_stream);
omni_status omni_residual_load(const void* store, int64_t n_slots, int32_t row_bytes, const int32_t* slot_ids,
                               int32_t n_rows, void* rows_out, void* hip_stream);

/*
 * Host-side producer of partial rows: attention over KV held in HOST memory, computed on the host's
 * cores (the paper's System Implementation, "CPU Attention": threads across the cores each take a part
 * of the load and the intermediate results are aggregated; the inner loops are vectorised).  It makes
 * no GPU call.  Every pointer of this struct is HOST memory owned by the caller.
 *
 * Row r covers tokens [row_begin[r], row_end[r]) of sequence row_seq[r] (ranges clamped as for
 * omni_paged_decode_attn; a page index outside [0, num_blocks) removes its 16 tokens) and yields, for
 * every query head, the partial defined under "Partials" above: part_o[r][head][:] (fp32, normalised
 * inside the range) and part_lse[r][head].  Rows listed sequence by sequence are a CSR source for
 * omni_merge_partials once copied to the device.  An empty range writes LSE = -inf and O = 0.
 * Layouts of q, the pools and the block table are those of omni_decode_args.  Arithmetic: products and
 * sums in fp32, inputs fp32 or bf16.  The call returns when all rows are written; it runs n_threads
 * threads of its own (0 = one per hardware thread) and allocates host scratch of
 * (number of 512-token slices) x G x (head_dim + 2) floats.
 * Errors: NULL, SHAPE (also a row_seq outside [0, batch), an isa_level outside 0..3), DTYPE, UNSUPPORTED
 * (block_size != 16, head_dim not 64 / 128, G > 16, an isa_level the CPU lacks).  n_rows = 0 is OK and
 * does nothing.
 */
typedef struct {
    int32_t n_rows;
    int32_t batch, num_q_heads, num_kv_heads, head_dim, block_size, max_blocks_per_seq;
    int64_t num_blocks;
    int32_t qkv_dtype;             /* omni_dtype of q, k_pool, v_pool */
    float   sm_scale;
    const void*    q;              /* [batch, num_q_heads, head_dim]                         */
    const void*    k_pool;         /* [num_blocks, num_kv_heads, block_size, head_dim]       */
    const void*    v_pool;
    const int32_t* block_table;    /* [batch, max_blocks_per_seq]                            */
    const int32_t* row_seq;        /* [n_rows]                                               */
    const int32_t* row_begin;      /* [n_rows]; NULL = all zero                              */
    const int32_t* row_end;        /* [n_rows]                                               */
    float* part_o;                 /* [n_rows, num_q_heads, head_dim]                        */
    float* part_lse;               /* [n_rows, num_q_heads]                                  */
    int32_t n_threads;
    /* instruction-set level of the inner loops: 0 = the best this CPU reports; 1 = plain x86-64,
     * 2 = AVX2 + FMA, 3 = AVX-512 (F, VL, BW, DQ) - UNSUPPORTED if the CPU lacks the level asked
     * for.  Levels differ in rounding order only (all within the tolerances of the path).      */
    int32_t isa_level;
} omni_host_attn_args;

omni_status omni_host_partial_attn(const omni_host_attn_args* a);

/* Static, human-readable name of a status code. */
const char* omni_status_string(omni_status s);

/*
 * Test aid for the block-table gather: copies the K and V rows of tokens
 * [ctx_begin[seq], ctx_end[seq]) of one sequence (ranges clamped as above) to
 * k_out / v_out [n_tokens, num_kv_heads, head_dim] in the pool's dtype, bit for
 * bit.  Rows whose page index is out of range are filled with zero bytes.
 */
omni_status omni_debug_gather_kv(const omni_decode_args* a, int32_t seq, void* k_out, void* v_out,
                                 void* hip_stream);

/*
 * Measurement aids.  omni_debug_stream_read reads `bytes` (multiple of 16) of
 * device memory once with 16-byte loads and folds them into sink[0..3] (so the
 * reads cannot be dropped): the streaming-read ceiling the attention kernel is
 * compared with.  omni_debug_copy copies `bytes` (multiple of 16) from src to
 * dst: the known-size kernel that calibrates the HBM byte counters.
 */
omni_status omni_debug_stream_read(const void* src, size_t bytes, uint32_t* sink, void* hip_stream);
omni_status omni_debug_copy(void* dst, const void* src, size_t bytes, void* hip_stream);
/* The host-side counterpart (HOST pointers, no GPU call): n_threads threads (0 = one per hardware thread)
 * read `bytes` (multiple of 8) of host memory once, a contiguous slab each, folded into *sink: the
 * streaming-read reference omni_host_partial_attn is compared with.  Returns when done. */
omni_status omni_debug_host_stream_read(const void* src, size_t bytes, int32_t n_threads, uint64_t* sink);

/*
 * Where the time of a persistent launch goes.  omni_debug_decode_timeline is omni_paged_decode_attn through
 * an instance of the persistent matrix-core kernel that also stamps a constant-rate clock (100 MHz, the same
 * for every workgroup) into `stamps` (device, n_words 64-bit words, zeroed by the caller): per workgroup w,
 * words_per_workgroup words from stamps[w * words_per_workgroup]: [0] start, [1] first query rows in LDS,
 * [2] streaming waves done, [3] the workgroup's last store done, [4] tickets taken, [5] 32-token steps of wave 0,
 * [8 + k] the workgroup's meeting after its k-th ticket (the first words_per_workgroup - 8 tickets).  A
 * workgroup without work stamps [0] only.  omni_debug_decode_timeline_shape tells how many workgroups a
 * launch on the current device has and how many words each writes.  Outputs are those of the plain call.
 * Errors: as omni_paged_decode_attn; UNSUPPORTED unless the call runs the persistent form at head_dim 128
 * (workspace given); SHAPE if n_words is too small.
 */
omni_status omni_debug_decode_timeline_shape(int32_t* n_workgroups, int32_t* words_per_workgroup);
omni_status omni_debug_decode_timeline(const omni_decode_args* a, uint64_t* stamps, uint64_t n_words, void* hip_stream);

/*
 * Test aids for the persistent form's work list (host only, no GPU call; they run the functions the kernels
 * use).  omni_debug_sort_bin: the sort key (0 .. 255, smaller = earlier in the list) of a non-empty range of
 * `tokens` tokens in a call with `chunk_tokens` (0 = unchunked); 256 for tokens <= 0.
 * omni_debug_ticket_map: for a list of n_entries non-empty ranges whose first n_long_entries are longer
 * than 256 tokens, num_kv_heads items per entry and n_workgroups workgroups, writes for every ticket t and
 * streaming wave w (0..3) the pair items[(4 t + w) * 2 + 0] = list item (entry * num_kv_heads + kv head,
 * -1 = none) and [.. + 1] = 1 if the ticket stands for one item per wave, 0 if all waves share the item;
 * *n_tickets receives the number of tickets.  Pairs beyond `capacity` ints are not written.
 * Errors: NULL, SHAPE (num_kv_heads < 1, n_workgroups < 1, more than 2^31 - 1 items).
 */
int32_t omni_debug_sort_bin(int32_t tokens, int32_t chunk_tokens);
omni_status omni_debug_ticket_map(uint32_t n_entries, uint32_t n_long_entries, int32_t num_kv_heads,
                                  uint32_t n_workgroups, int32_t* items, uint64_t capacity, uint32_t* n_tickets);

#ifdef __cplusplus
}
#endif
#endif /* OMNI_ATTN_H */
