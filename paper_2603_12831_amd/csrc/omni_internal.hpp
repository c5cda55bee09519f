// Internal declarations shared by the translation units of libomni_attn.
// Device helpers are plain inline functions; launchers are defined next to
// their kernels and called from api.hip.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "omni_attn.h"

namespace omni {

constexpr int kBlockSize = 16;     // tokens per KV page
constexpr int kWave = 64;          // CDNA wavefront width

// Flattened, validated form of omni_decode_args handed to the kernels.
struct DecodeParams {
    int batch, hq, hkv, d, max_blocks, group;
    long long num_blocks;
    float sm_scale;
    const void* q;
    const void* k_pool;
    const void* v_pool;
    const int* block_table;
    const int* ctx_begin;          // may be null
    const int* ctx_end;
    int chunk_tokens;              // > 0 here: "one chunk" is expressed as the whole table width, max_blocks * 16
    int max_chunks;
    float* part_o;                 // may be null (only when every row is written as a final row)
    float* part_lse;               // may be null
    void* out_o;                   // may be null; final rows of the sequences that this call can finish
    int out_bf16;
    float* out_lse;                // may be null
    int* seq_final;                // may be null; [batch] 1 = the call wrote the sequence's final row
    unsigned long long* stamps;    // null, or the time stamps of omni_debug_decode_timeline (device)
    int fuse;                      // 1 = every sequence is finished in the attention launch (persistent form)
    int n_ext;                     // fused form: sources of rows computed elsewhere, folded into the final rows
    omni_partial_src ext[3];
};

// Rows of sequence `seq` in a source of partial rows.
__device__ __forceinline__ void src_rows(const omni_partial_src& s, int seq, int& r0, int& r1)
{
    if (s.row_offsets) { r0 = s.row_offsets[seq]; r1 = s.row_offsets[seq + 1]; }
    else { r0 = seq * s.dense_rows_per_seq; r1 = r0 + s.dense_rows_per_seq; }
}

// Flattened, validated form of omni_kv_cache.
struct KvParams {
    int batch, hkv, d, max_blocks, elem_bytes;
    long long num_blocks;
    void* k_pool;
    void* v_pool;
    const int* block_table;        // may be null for the page gather / scatter
};

// Flattened form of omni_queue.
struct QueueParams {
    void* data;
    int* tags;                     // may be null
    unsigned* state;               // head, tail, departed workgroups, unused
    int capacity, row_bytes;
};

struct MergeParams {
    omni_partial_src src[4];
    int n_srcs, batch, hq, d, out_bf16;
    void* out_o;
    float* out_lse;
    const int* skip;               // may be null; [batch] non-zero = leave the sequence's rows alone
};

// ---- device helpers -------------------------------------------------------
__device__ __forceinline__ float bf16_to_f32(uint16_t b) { return __uint_as_float(((uint32_t)b) << 16); }
__device__ __forceinline__ float bf16lo_to_f32(uint32_t w) { return __uint_as_float(w << 16); }
__device__ __forceinline__ float bf16hi_to_f32(uint32_t w) { return __uint_as_float(w & 0xffff0000u); }

// fp32 -> bf16, round to nearest even; NaN stays NaN (quiet).
__device__ __forceinline__ uint16_t f32_to_bf16(float f)
{
    uint32_t u = __float_as_uint(f);
    if ((u & 0x7fffffffu) > 0x7f800000u) return (uint16_t)((u >> 16) | 0x40u);
    u += 0x7fffu + ((u >> 16) & 1u);
    return (uint16_t)(u >> 16);
}

// Token range of sequence `seq`, clamped so that every touched table entry exists.
__device__ __forceinline__ void seq_range(const DecodeParams& p, int seq, int& b, int& e)
{
    b = p.ctx_begin ? p.ctx_begin[seq] : 0;
    e = p.ctx_end[seq];
    if (b < 0) b = 0;
    long long cap = (long long)p.max_blocks * kBlockSize;
    if (e > cap) e = (int)cap;
}

// Range of chunk c inside [b, e); empty ranges come back with ce <= cb.
__device__ __forceinline__ void chunk_range(const DecodeParams& p, int b, int e, int c, int& cb, int& ce)
{
    long long lo = (long long)b + (long long)c * p.chunk_tokens;
    long long hi = lo + p.chunk_tokens;
    cb = lo < e ? (int)lo : e;
    ce = hi < e ? (int)hi : e;
}

// Number of non-empty chunks of a sequence whose clamped range is [b, e): chunks 0 .. n-1 are the live ones.
__device__ __forceinline__ int live_chunks(const DecodeParams& p, int b, int e)
{
    if (e <= b) return 0;
    // (both terms are at most the table width, which the API keeps below 2^30: 32-bit arithmetic is exact)
    const unsigned n = ((unsigned)(e - b) + (unsigned)p.chunk_tokens - 1u) / (unsigned)p.chunk_tokens;
    return n < (unsigned)p.max_chunks ? (int)n : p.max_chunks;
}

// What a sequence's final row has to be put together from, as far as this call can tell: its non-empty
// chunks, and - in a call that is told of rows computed elsewhere but does not fold them in itself - one
// more part where the sequence has such rows (then at least two, so that the call never takes the row for
// finished).  A sequence of at most one part gets its final row from the call.
__device__ __forceinline__ int seq_parts(const DecodeParams& p, int seq, int b, int e)
{
    int n = live_chunks(p, b, e);
    if (!p.fuse && p.n_ext > 0) {
        bool rows = false;
        for (int s = 0; s < p.n_ext; ++s) {
            int r0, r1;
            src_rows(p.ext[s], seq, r0, r1);
            rows |= r1 > r0;
        }
        if (rows) n = (n > 1 ? n : 1) + 1;
    }
    return n;
}

// ---- the work list of a decode call (built by decode_list_kernel, see decode_mfma.hip) ---------------
// Workspace: kHeaderWords words of header, then batch * max_chunks entries - the non-empty (sequence, chunk)
// ranges longest first from the front, the empty ones from the back -, then one arrival counter per
// (sequence, kv head).  An entry is a token range [cb, ce) of one chunk; `chunk` carries the chunk index in
// its low 16 bits and the number of parts of the sequence (non-empty chunks, + 1 if other sources hold rows
// for it) in its high 16 bits (both are at most 65535).
constexpr int kHeaderWords = 16;
struct alignas(16) WorkEntry { int seq, chunk, cb, ce; };
__host__ __device__ __forceinline__ int pack_chunk(int chunk, int n_live) { return (int)((unsigned)chunk | ((unsigned)n_live << 16)); }
__host__ __device__ __forceinline__ int chunk_index(int packed) { return packed & 0xffff; }
__host__ __device__ __forceinline__ int chunk_live(int packed) { return (int)((unsigned)packed >> 16); }

// ---- launchers (each defined beside its kernel) ---------------------------
hipError_t launch_decode_vector(const DecodeParams& p, bool bf16, void* workspace, bool planned, hipStream_t s);
hipError_t launch_decode_mfma(const DecodeParams& p, void* workspace, bool planned, hipStream_t s);
hipError_t launch_decode_plan(const DecodeParams& p, void* workspace, hipStream_t s);
hipError_t decode_timeline_shape(int& n_workgroups, int& words_per_workgroup);
size_t decode_workspace_bytes(long long batch, long long max_chunks, long long hkv);
bool decode_mfma_supports(const DecodeParams& p, bool bf16);
int decode_list_sort_bin(int tokens, int chunk_tokens);
unsigned decode_ticket_map(unsigned n_entries, unsigned n_long_entries, unsigned hkv, unsigned n_workgroups,
                           int* items, size_t capacity);
hipError_t launch_merge(const MergeParams& p, hipStream_t s);
hipError_t launch_gather(const DecodeParams& p, bool bf16, int seq, void* k_out, void* v_out, hipStream_t s);
hipError_t launch_stream_read(const void* src, size_t bytes, uint32_t* sink, hipStream_t s);
hipError_t launch_copy(void* dst, const void* src, size_t bytes, hipStream_t s);
hipError_t launch_queue(const QueueParams& q, bool push, const void* src_rows, const int* src_tags, void* dst_rows,
                        int* dst_tags, int n_rows, int* n_done, hipStream_t s);
hipError_t launch_csr_from_tags(const int* tags, const int* n_rows, int max_rows, int batch, int* offsets, hipStream_t s);
hipError_t launch_store(void* store, long long n_slots, int row_bytes, const int* slot_ids, int n_rows, void* rows,
                        bool save, hipStream_t s);
hipError_t launch_kv_append(const KvParams& c, const void* k_new, const void* v_new, const int* positions, hipStream_t s);
hipError_t launch_kv_pages(const KvParams& c, const int* page_ids, long long n_pages, void* k_stage, void* v_stage,
                           bool to_pool, hipStream_t s);

}  // namespace omni
