// C ABI of libomni_attn: argument checks, flattening, kernel choice.
#include <limits.h>

#include <mutex>

#include "omni_internal.hpp"

using namespace omni;

namespace {

bool dtype_ok(int32_t d) { return d == OMNI_F32 || d == OMNI_BF16; }

// Checks shared by the decode entry point and the gather aid; fills `p`.
omni_status flatten(const omni_decode_args* a, DecodeParams& p, bool need_outputs)
{
    if (!a) return OMNI_ERR_NULL;
    if (a->batch < 0 || a->num_q_heads <= 0 || a->num_kv_heads <= 0 || a->head_dim <= 0 ||
        a->block_size <= 0 || a->max_blocks_per_seq <= 0 || a->num_blocks <= 0)
        return OMNI_ERR_SHAPE;
    if (a->num_q_heads % a->num_kv_heads != 0) return OMNI_ERR_SHAPE;
    if (!dtype_ok(a->qkv_dtype)) return OMNI_ERR_DTYPE;
    if (a->chunk_tokens < 0 || a->max_chunks < 1) return OMNI_ERR_SHAPE;
    if (a->chunk_tokens == 0 && a->max_chunks != 1) return OMNI_ERR_SHAPE;
    if (a->chunk_tokens % a->block_size != 0) return OMNI_ERR_SHAPE;
    if (a->block_size != kBlockSize) return OMNI_ERR_UNSUPPORTED;
    if (a->head_dim != 64 && a->head_dim != 128) return OMNI_ERR_UNSUPPORTED;
    if (a->num_q_heads / a->num_kv_heads > 16) return OMNI_ERR_UNSUPPORTED;
    if (a->batch > 65535 || a->max_chunks > 65535) return OMNI_ERR_UNSUPPORTED;
    if ((long long)a->max_blocks_per_seq * kBlockSize > INT_MAX / 2) return OMNI_ERR_UNSUPPORTED;
    if (!a->q || !a->k_pool || !a->v_pool || !a->block_table || !a->ctx_end) return OMNI_ERR_NULL;
    if (a->n_ext_srcs < 0 || a->n_ext_srcs > 3) return OMNI_ERR_SHAPE;
    if (need_outputs) {
        if (!dtype_ok(a->out_dtype) && a->out_o) return OMNI_ERR_DTYPE;
        const bool partials = a->part_o && a->part_lse;
        if ((a->part_o == nullptr) != (a->part_lse == nullptr)) return OMNI_ERR_NULL;
        // without partial buffers every row must be a final row: a single chunk slot
        if (!partials && !(a->out_o && a->max_chunks == 1)) return OMNI_ERR_NULL;
        // final rows of part of the batch only: the caller must be told which
        const bool some_left = a->max_chunks > 1 || a->n_ext_srcs > 0;
        if (a->out_o && some_left && !a->fuse_merge && (!a->seq_final || !partials)) return OMNI_ERR_NULL;
        if (a->fuse_merge && !a->out_o) return OMNI_ERR_NULL;
        if (a->n_ext_srcs > 0) {
            if (!a->ext_srcs) return OMNI_ERR_NULL;
            for (int i = 0; i < a->n_ext_srcs; ++i) {
                if (!a->ext_srcs[i].o || !a->ext_srcs[i].lse) return OMNI_ERR_NULL;
                if (!a->ext_srcs[i].row_offsets && a->ext_srcs[i].dense_rows_per_seq < 0) return OMNI_ERR_SHAPE;
            }
        }
        // the kernels move q and the rows in 16-byte pieces (bf16 final rows in 8-byte ones)
        auto misaligned = [](const void* ptr) { return reinterpret_cast<uintptr_t>(ptr) % 16 != 0; };
        if (misaligned(a->q) || misaligned(a->k_pool) || misaligned(a->v_pool) || misaligned(a->part_o) ||
            misaligned(a->out_o))
            return OMNI_ERR_SHAPE;
        for (int i = 0; i < a->n_ext_srcs; ++i)
            if (misaligned(a->ext_srcs[i].o)) return OMNI_ERR_SHAPE;
    }
    p.batch = a->batch; p.hq = a->num_q_heads; p.hkv = a->num_kv_heads; p.d = a->head_dim;
    p.max_blocks = a->max_blocks_per_seq; p.group = a->num_q_heads / a->num_kv_heads;
    p.num_blocks = a->num_blocks; p.sm_scale = a->sm_scale;
    p.q = a->q; p.k_pool = a->k_pool; p.v_pool = a->v_pool; p.block_table = a->block_table;
    p.ctx_begin = a->ctx_begin; p.ctx_end = a->ctx_end;
    // "one chunk" = a chunk long enough for any clamped range
    p.chunk_tokens = a->chunk_tokens ? a->chunk_tokens : a->max_blocks_per_seq * kBlockSize;
    p.max_chunks = a->max_chunks;
    p.part_o = a->part_o; p.part_lse = a->part_lse;
    p.out_o = need_outputs ? a->out_o : nullptr;
    p.out_bf16 = a->out_dtype == OMNI_BF16;
    p.out_lse = p.out_o ? a->out_lse : nullptr;
    p.seq_final = need_outputs ? a->seq_final : nullptr;
    p.stamps = nullptr;
    // (the work list records which sequences the call can finish, so the plan call sees these as well)
    p.fuse = (a->out_o && a->fuse_merge) ? 1 : 0;
    p.n_ext = (a->out_o && a->ext_srcs) ? a->n_ext_srcs : 0;
    for (int i = 0; i < 3; ++i)
        p.ext[i] = i < p.n_ext ? a->ext_srcs[i] : omni_partial_src{nullptr, nullptr, nullptr, 0};
    return OMNI_OK;
}

// The decode call behind both of its entry points: `ws` / `ws_bytes` is the work-list scratch to use
// (the caller's workspace, or the library's own array), `planned` whether it already holds the list.
omni_status decode_attn(const omni_decode_args* a, void* ws_given, uint64_t ws_bytes, bool planned, void* hip_stream,
                        unsigned long long* stamps = nullptr)
{
    DecodeParams p;
    omni_status st = flatten(a, p, true);
    if (st != OMNI_OK) return st;
    p.stamps = stamps;
    if (a->kernel != OMNI_KERNEL_AUTO && a->kernel != OMNI_KERNEL_VECTOR && a->kernel != OMNI_KERNEL_MFMA)
        return OMNI_ERR_SHAPE;
    if (p.batch == 0) return OMNI_OK;
    const bool bf16 = a->qkv_dtype == OMNI_BF16;
    hipStream_t s = static_cast<hipStream_t>(hip_stream);
    bool mfma = decode_mfma_supports(p, bf16);
    if (a->kernel == OMNI_KERNEL_MFMA && !mfma) return OMNI_ERR_UNSUPPORTED;
    if (a->kernel == OMNI_KERNEL_VECTOR) mfma = false;
    void* ws = ws_given;
    if (ws) {
        if (ws_bytes < decode_workspace_bytes(p.batch, p.max_chunks, p.hkv)) return OMNI_ERR_SHAPE;
        if (reinterpret_cast<uintptr_t>(ws) % 16 != 0) return OMNI_ERR_SHAPE;
    }
    // only the persistent form finishes every sequence, and only at head_dim 128
    if (p.fuse && (!mfma || !ws || p.d != 128)) return OMNI_ERR_UNSUPPORTED;
    // the time-stamping instances are of the persistent form at head_dim 128
    if (p.stamps && (!mfma || !ws || p.d != 128)) return OMNI_ERR_UNSUPPORTED;
    hipError_t e = mfma ? launch_decode_mfma(p, ws, planned, s) : launch_decode_vector(p, bf16, ws, planned, s);
    return e == hipSuccess ? OMNI_OK : OMNI_ERR_LAUNCH;
}

}  // namespace

// Work-list scratch of omni_paged_decode_attn_static: one array per GPU, part of the loaded code object, so
// no call ever allocates it.  In host code the name below is only a handle; the array's device address is
// asked for once per device (static_scratch) and only that address is handed to kernels.
static __device__ __align__(256) unsigned char scratch[OMNI_STATIC_SCRATCH_BYTES];

namespace {

// Device address of `scratch` on the current device (every GPU has its own copy at its own address).
hipError_t static_scratch(void*& ptr)
{
    constexpr int kMaxDevices = 64;
    static void* ptrs[kMaxDevices] = {};
    static std::mutex mu;
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    if (dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice;
    std::lock_guard<std::mutex> lock(mu);
    if (!ptrs[dev]) {
        void* found = nullptr;
        e = hipGetSymbolAddress(&found, HIP_SYMBOL(scratch));
        if (e != hipSuccess) return e;
        if (!found) return hipErrorInvalidSymbol;
        ptrs[dev] = found;
    }
    ptr = ptrs[dev];
    return hipSuccess;
}

}  // namespace

extern "C" {

omni_status omni_paged_decode_attn(const omni_decode_args* a, void* hip_stream)
{
    if (!a) return OMNI_ERR_NULL;
    return decode_attn(a, a->workspace, a->workspace_bytes, a->workspace_planned != 0, hip_stream);
}

omni_status omni_paged_decode_attn_static(const omni_decode_args* a, void* hip_stream)
{
    if (!a) return OMNI_ERR_NULL;
    if (a->batch > 0 && a->max_chunks > 0 && a->num_kv_heads > 0 &&
        decode_workspace_bytes(a->batch, a->max_chunks, a->num_kv_heads) > (size_t)OMNI_STATIC_SCRATCH_BYTES)
        return OMNI_ERR_TOO_LARGE;
    void* ws = nullptr;
    if (static_scratch(ws) != hipSuccess) return OMNI_ERR_LAUNCH;
    // the list is always rebuilt: the array is shared by every call on this GPU
    return decode_attn(a, ws, OMNI_STATIC_SCRATCH_BYTES, false, hip_stream);
}

const char* omni_decode_kernel_name(const omni_decode_args* a)
{
    DecodeParams p;
    if (flatten(a, p, true) != OMNI_OK) return "";
    bool mfma = decode_mfma_supports(p, a->qkv_dtype == OMNI_BF16);
    if (a->kernel == OMNI_KERNEL_MFMA && !mfma) return "";
    if (a->kernel == OMNI_KERNEL_VECTOR) mfma = false;
    if (!mfma) return (p.fuse || a->kernel > OMNI_KERNEL_MFMA || a->kernel < 0) ? "" : "decode_vector_kernel";
    if (p.fuse && p.d != 128) return "";
    if (!a->workspace) return p.fuse ? "" : "decode_mfma_grid_kernel";
    return "decode_mfma_persistent_kernel";
}

omni_status omni_decode_abandoned_waves(void* workspace, uint32_t* count, void* hip_stream)
{
    if (!count) return OMNI_ERR_NULL;
    void* ws = workspace;
    if (!ws && static_scratch(ws) != hipSuccess) return OMNI_ERR_LAUNCH;
    hipStream_t s = static_cast<hipStream_t>(hip_stream);
    char* word = static_cast<char*>(ws) + 20;
    if (hipMemcpyAsync(count, word, sizeof(uint32_t), hipMemcpyDeviceToHost, s) != hipSuccess) return OMNI_ERR_LAUNCH;
    if (hipStreamSynchronize(s) != hipSuccess) return OMNI_ERR_LAUNCH;
    if (*count != 0 && hipMemsetAsync(word, 0, sizeof(uint32_t), s) != hipSuccess) return OMNI_ERR_LAUNCH;
    return OMNI_OK;
}

omni_status omni_decode_plan(const omni_decode_args* a, void* hip_stream)
{
    DecodeParams p;
    omni_status st = flatten(a, p, false);
    if (st != OMNI_OK) return st;
    if (!a->workspace) return OMNI_ERR_NULL;
    if (a->workspace_bytes < decode_workspace_bytes(p.batch, p.max_chunks, p.hkv)) return OMNI_ERR_SHAPE;
    if (reinterpret_cast<uintptr_t>(a->workspace) % 16 != 0) return OMNI_ERR_SHAPE;
    if (p.batch == 0) return OMNI_OK;
    hipError_t e = launch_decode_plan(p, a->workspace, static_cast<hipStream_t>(hip_stream));
    return e == hipSuccess ? OMNI_OK : OMNI_ERR_LAUNCH;
}

uint64_t omni_decode_workspace_bytes(int32_t batch, int32_t max_chunks, int32_t num_kv_heads)
{
    if (batch <= 0 || max_chunks <= 0 || num_kv_heads <= 0) return 0;
    return decode_workspace_bytes(batch, max_chunks, num_kv_heads);
}

omni_status omni_merge_partials(int32_t batch, int32_t num_q_heads, int32_t head_dim,
                                const omni_partial_src* srcs, int32_t n_srcs,
                                void* out_o, int32_t out_dtype, float* out_lse, void* hip_stream)
{
    return omni_merge_partials_masked(batch, num_q_heads, head_dim, srcs, n_srcs, nullptr, out_o, out_dtype, out_lse,
                                      hip_stream);
}

omni_status omni_merge_partials_masked(int32_t batch, int32_t num_q_heads, int32_t head_dim,
                                       const omni_partial_src* srcs, int32_t n_srcs, const int32_t* skip,
                                       void* out_o, int32_t out_dtype, float* out_lse, void* hip_stream)
{
    if (batch < 0 || num_q_heads <= 0 || n_srcs < 1 || n_srcs > 4) return OMNI_ERR_SHAPE;
    if (head_dim != 64 && head_dim != 128) return OMNI_ERR_SHAPE;
    if (!dtype_ok(out_dtype)) return OMNI_ERR_DTYPE;
    if (!srcs || !out_o) return OMNI_ERR_NULL;
    MergeParams p;
    for (int i = 0; i < n_srcs; ++i) {
        if (!srcs[i].o || !srcs[i].lse) return OMNI_ERR_NULL;
        if (!srcs[i].row_offsets && srcs[i].dense_rows_per_seq < 0) return OMNI_ERR_SHAPE;
        p.src[i] = srcs[i];
    }
    for (int i = n_srcs; i < 4; ++i) p.src[i] = omni_partial_src{nullptr, nullptr, nullptr, 0};
    p.n_srcs = n_srcs; p.batch = batch; p.hq = num_q_heads; p.d = head_dim;
    p.out_bf16 = out_dtype == OMNI_BF16; p.out_o = out_o; p.out_lse = out_lse; p.skip = skip;
    hipError_t e = launch_merge(p, static_cast<hipStream_t>(hip_stream));
    return e == hipSuccess ? OMNI_OK : OMNI_ERR_LAUNCH;
}

static omni_status flatten_kv(const omni_kv_cache* c, KvParams& k, bool need_table)
{
    if (!c) return OMNI_ERR_NULL;
    if (c->num_kv_heads <= 0 || c->head_dim <= 0 || c->block_size <= 0 || c->num_blocks <= 0) return OMNI_ERR_SHAPE;
    if (need_table && (c->batch < 0 || c->max_blocks_per_seq <= 0)) return OMNI_ERR_SHAPE;
    if (!dtype_ok(c->dtype)) return OMNI_ERR_DTYPE;
    if (c->block_size != kBlockSize) return OMNI_ERR_UNSUPPORTED;
    const int eb = c->dtype == OMNI_BF16 ? 2 : 4;
    if ((c->head_dim * eb) % 16 != 0) return OMNI_ERR_UNSUPPORTED;
    if (!c->k_pool || !c->v_pool || (need_table && !c->block_table)) return OMNI_ERR_NULL;
    k.batch = c->batch; k.hkv = c->num_kv_heads; k.d = c->head_dim; k.max_blocks = c->max_blocks_per_seq;
    k.elem_bytes = eb; k.num_blocks = c->num_blocks; k.k_pool = c->k_pool; k.v_pool = c->v_pool;
    k.block_table = c->block_table;
    return OMNI_OK;
}

omni_status omni_kv_append(const omni_kv_cache* c, const void* k_new, const void* v_new,
                           const int32_t* positions, void* hip_stream)
{
    KvParams k;
    omni_status st = flatten_kv(c, k, true);
    if (st != OMNI_OK) return st;
    if (!k_new || !v_new || !positions) return OMNI_ERR_NULL;
    hipError_t e = launch_kv_append(k, k_new, v_new, positions, static_cast<hipStream_t>(hip_stream));
    return e == hipSuccess ? OMNI_OK : OMNI_ERR_LAUNCH;
}

static omni_status kv_pages(const omni_kv_cache* c, const int32_t* page_ids, int64_t n_pages, void* ks, void* vs,
                            bool to_pool, void* hip_stream)
{
    KvParams k;
    omni_status st = flatten_kv(c, k, false);
    if (st != OMNI_OK) return st;
    if (n_pages < 0) return OMNI_ERR_SHAPE;
    if (n_pages == 0) return OMNI_OK;
    if (!page_ids || !ks || !vs) return OMNI_ERR_NULL;
    hipError_t e = launch_kv_pages(k, page_ids, n_pages, ks, vs, to_pool, static_cast<hipStream_t>(hip_stream));
    return e == hipSuccess ? OMNI_OK : OMNI_ERR_LAUNCH;
}

omni_status omni_kv_gather_pages(const omni_kv_cache* c, const int32_t* page_ids, int64_t n_pages,
                                 void* k_out, void* v_out, void* hip_stream)
{
    return kv_pages(c, page_ids, n_pages, k_out, v_out, false, hip_stream);
}

omni_status omni_kv_scatter_pages(const omni_kv_cache* c, const int32_t* page_ids, int64_t n_pages,
                                  const void* k_in, const void* v_in, void* hip_stream)
{
    return kv_pages(c, page_ids, n_pages, const_cast<void*>(k_in), const_cast<void*>(v_in), true, hip_stream);
}

static omni_status flatten_queue(const omni_queue* q, QueueParams& k, int32_t n_rows)
{
    if (!q) return OMNI_ERR_NULL;
    if (q->capacity <= 0 || q->row_bytes <= 0 || q->row_bytes % 16 != 0 || n_rows < 0) return OMNI_ERR_SHAPE;
    if ((long long)q->capacity * q->row_bytes > 0x7fffffffLL) return OMNI_ERR_UNSUPPORTED;       // 32-bit offsets in the ring
    if (!q->data || !q->state) return OMNI_ERR_NULL;
    k.data = q->data; k.tags = q->tags; k.state = q->state; k.capacity = q->capacity; k.row_bytes = q->row_bytes;
    return OMNI_OK;
}

omni_status omni_queue_push(const omni_queue* q, const void* rows, const int32_t* tags, int32_t n_rows,
                            int32_t* n_pushed, void* hip_stream)
{
    QueueParams k;
    omni_status st = flatten_queue(q, k, n_rows);
    if (st != OMNI_OK) return st;
    if (n_rows > 0 && !rows) return OMNI_ERR_NULL;
    hipError_t e = launch_queue(k, true, rows, tags, nullptr, nullptr, n_rows, n_pushed, static_cast<hipStream_t>(hip_stream));
    return e == hipSuccess ? OMNI_OK : OMNI_ERR_LAUNCH;
}

omni_status omni_queue_pop(const omni_queue* q, void* rows_out, int32_t* tags_out, int32_t max_rows,
                           int32_t* n_popped, void* hip_stream)
{
    QueueParams k;
    omni_status st = flatten_queue(q, k, max_rows);
    if (st != OMNI_OK) return st;
    if (max_rows > 0 && !rows_out) return OMNI_ERR_NULL;
    hipError_t e = launch_queue(k, false, nullptr, nullptr, rows_out, tags_out, max_rows, n_popped, static_cast<hipStream_t>(hip_stream));
    return e == hipSuccess ? OMNI_OK : OMNI_ERR_LAUNCH;
}

omni_status omni_csr_from_tags(const int32_t* tags, const int32_t* n_rows, int32_t max_rows, int32_t batch,
                               int32_t* row_offsets, void* hip_stream)
{
    if (max_rows < 0 || batch < 0) return OMNI_ERR_SHAPE;
    if (!row_offsets || (max_rows > 0 && !tags)) return OMNI_ERR_NULL;
    hipError_t e = launch_csr_from_tags(tags, n_rows, max_rows, batch, row_offsets, static_cast<hipStream_t>(hip_stream));
    return e == hipSuccess ? OMNI_OK : OMNI_ERR_LAUNCH;
}

static omni_status residual(void* store, int64_t n_slots, int32_t row_bytes, const int32_t* slot_ids, int32_t n_rows,
                            void* rows, bool save, void* hip_stream)
{
    if (n_slots <= 0 || row_bytes <= 0 || row_bytes % 16 != 0 || n_rows < 0) return OMNI_ERR_SHAPE;
    if (n_rows == 0) return OMNI_OK;
    if (!store || !slot_ids || !rows) return OMNI_ERR_NULL;
    hipError_t e = launch_store(store, n_slots, row_bytes, slot_ids, n_rows, rows, save, static_cast<hipStream_t>(hip_stream));
    return e == hipSuccess ? OMNI_OK : OMNI_ERR_LAUNCH;
}

omni_status omni_residual_save(void* store, int64_t n_slots, int32_t row_bytes, const int32_t* slot_ids,
                               int32_t n_rows, const void* rows, void* hip_stream)
{
    return residual(store, n_slots, row_bytes, slot_ids, n_rows, const_cast<void*>(rows), true, hip_stream);
}

omni_status omni_residual_load(const void* store, int64_t n_slots, int32_t row_bytes, const int32_t* slot_ids,
                               int32_t n_rows, void* rows_out, void* hip_stream)
{
    return residual(const_cast<void*>(store), n_slots, row_bytes, slot_ids, n_rows, rows_out, false, hip_stream);
}

const char* omni_status_string(omni_status s)
{
    switch (s) {
        case OMNI_OK: return "OMNI_OK";
        case OMNI_ERR_NULL: return "OMNI_ERR_NULL: a required pointer is NULL";
        case OMNI_ERR_SHAPE: return "OMNI_ERR_SHAPE: bad size, head ratio or chunking";
        case OMNI_ERR_DTYPE: return "OMNI_ERR_DTYPE: unknown dtype";
        case OMNI_ERR_UNSUPPORTED: return "OMNI_ERR_UNSUPPORTED: shape outside the supported set";
        case OMNI_ERR_LAUNCH: return "OMNI_ERR_LAUNCH: HIP launch failed";
        case OMNI_ERR_TOO_LARGE: return "OMNI_ERR_TOO_LARGE: batch x max_chunks exceeds the library's static scratch";
    }
    return "OMNI_ERR_?: unknown status";
}

omni_status omni_debug_gather_kv(const omni_decode_args* a, int32_t seq, void* k_out, void* v_out, void* hip_stream)
{
    DecodeParams p;
    omni_status st = flatten(a, p, false);
    if (st != OMNI_OK) return st;
    if (!k_out || !v_out) return OMNI_ERR_NULL;
    if (seq < 0 || seq >= p.batch) return OMNI_ERR_SHAPE;
    hipError_t e = launch_gather(p, a->qkv_dtype == OMNI_BF16, seq, k_out, v_out, static_cast<hipStream_t>(hip_stream));
    return e == hipSuccess ? OMNI_OK : OMNI_ERR_LAUNCH;
}

omni_status omni_debug_stream_read(const void* src, size_t bytes, uint32_t* sink, void* hip_stream)
{
    if (!src || !sink) return OMNI_ERR_NULL;
    if (bytes % 16 != 0) return OMNI_ERR_SHAPE;
    hipError_t e = launch_stream_read(src, bytes, sink, static_cast<hipStream_t>(hip_stream));
    return e == hipSuccess ? OMNI_OK : OMNI_ERR_LAUNCH;
}

omni_status omni_debug_copy(void* dst, const void* src, size_t bytes, void* hip_stream)
{
    if (!src || !dst) return OMNI_ERR_NULL;
    if (bytes % 16 != 0) return OMNI_ERR_SHAPE;
    hipError_t e = launch_copy(dst, src, bytes, static_cast<hipStream_t>(hip_stream));
    return e == hipSuccess ? OMNI_OK : OMNI_ERR_LAUNCH;
}

int32_t omni_debug_sort_bin(int32_t tokens, int32_t chunk_tokens)
{
    return omni::decode_list_sort_bin(tokens, chunk_tokens);
}

omni_status omni_debug_decode_timeline_shape(int32_t* n_workgroups, int32_t* words_per_workgroup)
{
    if (!n_workgroups || !words_per_workgroup) return OMNI_ERR_NULL;
    int n = 0, w = 0;
    if (omni::decode_timeline_shape(n, w) != hipSuccess) return OMNI_ERR_LAUNCH;
    *n_workgroups = n;
    *words_per_workgroup = w;
    return OMNI_OK;
}

omni_status omni_debug_decode_timeline(const omni_decode_args* a, uint64_t* stamps, uint64_t n_words, void* hip_stream)
{
    if (!a || !stamps) return OMNI_ERR_NULL;
    int n = 0, w = 0;
    if (omni::decode_timeline_shape(n, w) != hipSuccess) return OMNI_ERR_LAUNCH;
    if (n_words < (uint64_t)n * (uint64_t)w) return OMNI_ERR_SHAPE;
    static_assert(sizeof(unsigned long long) == sizeof(uint64_t), "stamp words are 64 bits");
    return decode_attn(a, a->workspace, a->workspace_bytes, a->workspace_planned != 0, hip_stream,
                             reinterpret_cast<unsigned long long*>(stamps));
}

omni_status omni_debug_ticket_map(uint32_t n_entries, uint32_t n_long_entries, int32_t num_kv_heads,
                                  uint32_t n_workgroups, int32_t* items, uint64_t capacity, uint32_t* n_tickets)
{
    if (!items || !n_tickets) return OMNI_ERR_NULL;
    if (num_kv_heads < 1 || n_workgroups < 1 || (uint64_t)n_entries * (uint64_t)num_kv_heads > 0x7fffffffull)
        return OMNI_ERR_SHAPE;
    *n_tickets = omni::decode_ticket_map(n_entries, n_long_entries, (unsigned)num_kv_heads, n_workgroups, items,
                                         (size_t)capacity);
    return OMNI_OK;
}

}  // extern "C"
