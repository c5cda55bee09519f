// Device-resident row queues and the residual store of the piggybacking data path.
//
// The paper keeps the hand-over between the GPU stream and the CPU attention workers in GPU memory: an
// input queue (q, k, v rows of offloaded requests of one layer) and an output queue (their attention
// result rows), each a tensor with head and tail pointers, written at the tail by the producer and read
// from the head by the consumer; and a residual store indexed by (request, layer) that keeps a request's
// residual while its attention is computed elsewhere (System Implementation: CPU Attention queue, Residual
// management).  These kernels are the GPU-side operations on those structures: push rows, pop rows,
// save rows to store slots, load rows from store slots.  All are copies in 16-byte pieces; counts and
// pointers live on the device, nothing synchronises with the host.
//
// Queue state words: [0] head (rows popped so far), [1] tail (rows pushed so far), [2] departed
// workgroups of the running call (zero between calls), [3] unused.  Slot of counter value c: c % capacity.
#include "omni_internal.hpp"

namespace omni {
namespace {

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

// every workgroup reads head and tail before any workgroup can have published a new value: the publisher
// is the last workgroup to leave.  A workgroup moves a contiguous share of the rows, its lanes the share's
// 16-byte pieces, kQueueUnroll independent moves in flight per lane (few workgroups with much in flight each:
// every workgroup ends with an atomic on one word, and those are served one after the other - 70 ns each).
// Rows go into the ring with device-scope stores (written through this XCD's L2), so that "rows before
// pointer" needs no cache-wide write-back: the workgroup only waits until its stores have left.
constexpr int kQueueUnroll = 8;

template <bool push>
__global__ __launch_bounds__(256) void queue_kernel(QueueParams q, const u32x4* __restrict__ src_rows,
                                                    const int* __restrict__ src_tags, u32x4* dst_rows, int* dst_tags,
                                                    int n_rows, int* n_done)
{
    const unsigned head = q.state[0], tail = q.state[1];
    const unsigned used = tail - head;
    unsigned n;
    if (push) n = (used + (unsigned)n_rows <= (unsigned)q.capacity) ? (unsigned)n_rows : 0u;   // all or nothing
    else n = used < (unsigned)n_rows ? used : (unsigned)n_rows;
    const unsigned pieces = (unsigned)(q.row_bytes / 16);
    u32x4* ring = static_cast<u32x4*>(q.data);
    // this workgroup's rows [r0, r1); their pieces are numbered 0 .. count-1 (32-bit: a share is far below 2^32 pieces)
    const unsigned per = (n + gridDim.x - 1) / gridDim.x;
    const unsigned r0 = min(n, blockIdx.x * per), r1 = min(n, r0 + per);
    const unsigned long long count64 = (unsigned long long)(r1 - r0) * pieces;
    const unsigned count = count64 < 0xffffffffull ? (unsigned)count64 : 0xffffffffu;
    constexpr int kDeviceScope = 1 << 4;
    // (the API keeps a ring below 2 GiB: 32-bit byte offsets)
    const __amdgpu_buffer_rsrc_t ring_rs =
        __builtin_amdgcn_make_buffer_rsrc(ring, 0, (int)((unsigned)q.capacity * (unsigned)q.row_bytes), 0x00020000);
    for (unsigned base = threadIdx.x; base < count; base += blockDim.x * kQueueUnroll) {
        u32x4 v[kQueueUnroll];
        unsigned long long at[kQueueUnroll];               // piece index in the ring
#pragma unroll
        for (int u = 0; u < kQueueUnroll; ++u) {
            const unsigned i = base + u * blockDim.x;
            if (i < count) {
                const unsigned r = r0 + i / pieces, piece = i % pieces;
                const unsigned slot = ((push ? tail : head) + r) % (unsigned)q.capacity;
                at[u] = (unsigned long long)slot * pieces + piece;
                v[u] = push ? src_rows[(unsigned long long)r * pieces + piece] : ring[at[u]];
                if (piece == 0) {
                    if (push) { if (q.tags) q.tags[slot] = src_tags ? src_tags[r] : 0; }
                    else if (dst_tags) dst_tags[r] = q.tags ? q.tags[slot] : 0;
                }
            }
        }
#pragma unroll
        for (int u = 0; u < kQueueUnroll; ++u) {
            const unsigned i = base + u * blockDim.x;
            if (i < count) {
                if (push) {
                    __builtin_amdgcn_raw_buffer_store_b128(v[u], ring_rs, (int)(unsigned)(at[u] * 16u), 0, kDeviceScope);
                } else {
                    dst_rows[(unsigned long long)(r0 + i / pieces) * pieces + i % pieces] = v[u];
                }
            }
        }
    }
    // every store of this workgroup has left before it counts as departed
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __syncthreads();
    if (threadIdx.x == 0) {
        const unsigned gone = __hip_atomic_fetch_add(q.state + 2, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        if (gone == gridDim.x - 1) {
            atomicExch(q.state + 2, 0u);
            if (push) atomicExch(q.state + 1, tail + n);
            else atomicExch(q.state + 0, head + n);
            if (n_done) *n_done = (int)n;
        }
    }
}

// rows <-> store slots: slot_ids[r] names the store row of source/destination row r; ids outside
// [0, n_slots) are skipped (save) or give zero rows (load).  Whole rows per workgroup, as above.
template <bool save>
__global__ __launch_bounds__(256) void store_kernel(u32x4* store, long long n_slots, int row_bytes,
                                                    const int* __restrict__ slot_ids, int n_rows, u32x4* rows)
{
    const int pieces = row_bytes / 16;
    constexpr int kUnroll = 4;
    for (int r = blockIdx.x; r < n_rows; r += gridDim.x) {
        const long long slot = slot_ids[r];
        const bool ok = slot >= 0 && slot < n_slots;
        if (save && !ok) continue;
        const u32x4* from = save ? rows + (long long)r * pieces : store + (ok ? slot : 0) * pieces;
        u32x4* to = save ? store + slot * pieces : rows + (long long)r * pieces;
        for (int base = threadIdx.x; base < pieces; base += blockDim.x * kUnroll) {
            u32x4 v[kUnroll];
#pragma unroll
            for (int u = 0; u < kUnroll; ++u) {
                const int i = base + u * blockDim.x;
                v[u] = u32x4{0, 0, 0, 0};
                if (i < pieces && ok) v[u] = from[i];
            }
#pragma unroll
            for (int u = 0; u < kUnroll; ++u) {
                const int i = base + u * blockDim.x;
                if (i < pieces) to[i] = v[u];
            }
        }
    }
}

// CSR offsets of popped rows: tags[0 .. n) (n read on the device, at most max_rows) are the sequence numbers
// of the rows, non-decreasing (rows of one sequence together, sequences in order - the order in which a
// producer that works through the batch pushes them); offsets[i] = number of rows with a tag below i, so
// rows offsets[i] .. offsets[i+1]-1 are sequence i's.  One thread per offset, a binary search each.
__global__ __launch_bounds__(256) void csr_from_tags_kernel(const int* __restrict__ tags, const int* __restrict__ n_rows,
                                                            int max_rows, int batch, int* __restrict__ offsets)
{
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i > batch) return;
    int n = n_rows ? *n_rows : max_rows;
    n = n < 0 ? 0 : (n > max_rows ? max_rows : n);
    int lo = 0, hi = n;                                    // first row whose tag is >= i
    while (lo < hi) {
        const int mid = (lo + hi) >> 1;
        if (tags[mid] < i) lo = mid + 1;
        else hi = mid;
    }
    offsets[i] = lo;
}

#ifndef OMNI_QUEUE_GRID_CAP
#define OMNI_QUEUE_GRID_CAP 128
#endif
// workgroups of a queue call: enough for 32 KiB in flight each, at most the cap (see queue_kernel)
unsigned queue_grid(long long n_rows, int row_bytes)
{
    const long long want = (n_rows * row_bytes + 32767) / 32768;
    return (unsigned)(want < 1 ? 1 : (want < OMNI_QUEUE_GRID_CAP ? want : OMNI_QUEUE_GRID_CAP));
}
// one workgroup per row for the store (no shared word at the end), up to a few per CU
unsigned grid_for(long long rows)
{
    return (unsigned)(rows < 1 ? 1 : (rows < 1024 ? rows : 1024));
}

}  // namespace

hipError_t launch_queue(const QueueParams& q, bool push, const void* src_rows, const int* src_tags, void* dst_rows,
                        int* dst_tags, int n_rows, int* n_done, hipStream_t s)
{
    const unsigned grid = queue_grid(n_rows, q.row_bytes);
    if (push)
        hipLaunchKernelGGL((queue_kernel<true>), dim3(grid), dim3(256), 0, s, q, static_cast<const u32x4*>(src_rows),
                           src_tags, static_cast<u32x4*>(dst_rows), dst_tags, n_rows, n_done);
    else
        hipLaunchKernelGGL((queue_kernel<false>), dim3(grid), dim3(256), 0, s, q, static_cast<const u32x4*>(src_rows),
                           src_tags, static_cast<u32x4*>(dst_rows), dst_tags, n_rows, n_done);
    return hipGetLastError();
}

hipError_t launch_csr_from_tags(const int* tags, const int* n_rows, int max_rows, int batch, int* offsets, hipStream_t s)
{
    const unsigned grid = (unsigned)((batch + 1 + 255) / 256);
    hipLaunchKernelGGL(csr_from_tags_kernel, dim3(grid), dim3(256), 0, s, tags, n_rows, max_rows, batch, offsets);
    return hipGetLastError();
}

hipError_t launch_store(void* store, long long n_slots, int row_bytes, const int* slot_ids, int n_rows, void* rows,
                        bool save, hipStream_t s)
{
    if (n_rows == 0) return hipSuccess;
    const unsigned grid = grid_for(n_rows);
    if (save)
        hipLaunchKernelGGL((store_kernel<true>), dim3(grid), dim3(256), 0, s, static_cast<u32x4*>(store), n_slots,
                           row_bytes, slot_ids, n_rows, static_cast<u32x4*>(rows));
    else
        hipLaunchKernelGGL((store_kernel<false>), dim3(grid), dim3(256), 0, s, static_cast<u32x4*>(store), n_slots,
                           row_bytes, slot_ids, n_rows, static_cast<u32x4*>(rows));
    return hipGetLastError();
}

}  // namespace omni
