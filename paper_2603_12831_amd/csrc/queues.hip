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
// is the last workgroup to leave
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
    const int pieces = q.row_bytes / 16;
    const long long total = (long long)n * pieces;
    const long long step = (long long)gridDim.x * blockDim.x;
    u32x4* ring = static_cast<u32x4*>(q.data);
    constexpr int kUnroll = 4;                             // independent 16-byte moves in flight per lane
    for (long long base = (long long)blockIdx.x * blockDim.x + threadIdx.x; base < total; base += step * kUnroll) {
        u32x4 v[kUnroll];
        long long ring_idx[kUnroll];
#pragma unroll
        for (int u = 0; u < kUnroll; ++u) {
            const long long i = base + u * step;
            ring_idx[u] = -1;
            if (i < total) {
                const unsigned r = (unsigned)(i / pieces);
                const int piece = (int)(i - (long long)r * pieces);
                const unsigned slot = ((push ? tail : head) + r) % (unsigned)q.capacity;
                ring_idx[u] = (long long)slot * pieces + piece;
                v[u] = push ? src_rows[i] : ring[ring_idx[u]];
                if (piece == 0) {
                    if (push) { if (q.tags) q.tags[slot] = src_tags ? src_tags[r] : 0; }
                    else if (dst_tags) dst_tags[r] = q.tags ? q.tags[slot] : 0;
                }
            }
        }
#pragma unroll
        for (int u = 0; u < kUnroll; ++u) {
            const long long i = base + u * step;
            if (ring_idx[u] >= 0) {
                if (push) ring[ring_idx[u]] = v[u];
                else dst_rows[i] = v[u];
            }
        }
    }
    __threadfence();                                       // rows before pointers, for any other agent
    __syncthreads();
    if (threadIdx.x == 0) {
        const unsigned gone = atomicAdd(q.state + 2, 1u);
        if (gone == gridDim.x - 1) {
            atomicExch(q.state + 2, 0u);
            if (push) atomicExch(q.state + 1, tail + n);
            else atomicExch(q.state + 0, head + n);
            if (n_done) *n_done = (int)n;
        }
    }
}

// rows <-> store slots: slot_ids[r] names the store row of source/destination row r; ids outside
// [0, n_slots) are skipped (save) or give zero rows (load)
template <bool save>
__global__ __launch_bounds__(256) void store_kernel(u32x4* store, long long n_slots, int row_bytes,
                                                    const int* __restrict__ slot_ids, int n_rows, u32x4* rows)
{
    const int pieces = row_bytes / 16;
    const long long total = (long long)n_rows * pieces;
    const long long step = (long long)gridDim.x * blockDim.x;
    for (long long i = (long long)blockIdx.x * blockDim.x + threadIdx.x; i < total; i += step) {
        const int r = (int)(i / pieces);
        const int piece = (int)(i - (long long)r * pieces);
        const long long slot = slot_ids[r];
        const bool ok = slot >= 0 && slot < n_slots;
        if (save) {
            if (ok) store[slot * pieces + piece] = rows[i];
        } else {
            const u32x4 z = {0, 0, 0, 0};
            rows[i] = ok ? store[slot * pieces + piece] : z;
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

// few workgroups: every workgroup of a queue call ends with an atomic on one word, and those are served
// one after the other; the moves per lane are unrolled instead
unsigned grid_for(long long pieces)
{
    const long long want = (pieces + 1023) / 1024;
    return (unsigned)(want < 1 ? 1 : (want < 64 ? want : 64));
}

}  // namespace

hipError_t launch_queue(const QueueParams& q, bool push, const void* src_rows, const int* src_tags, void* dst_rows,
                        int* dst_tags, int n_rows, int* n_done, hipStream_t s)
{
    const unsigned grid = grid_for((long long)n_rows * (q.row_bytes / 16));
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
    const unsigned grid = grid_for((long long)n_rows * (row_bytes / 16));
    if (save)
        hipLaunchKernelGGL((store_kernel<true>), dim3(grid), dim3(256), 0, s, static_cast<u32x4*>(store), n_slots,
                           row_bytes, slot_ids, n_rows, static_cast<u32x4*>(rows));
    else
        hipLaunchKernelGGL((store_kernel<false>), dim3(grid), dim3(256), 0, s, static_cast<u32x4*>(store), n_slots,
                           row_bytes, slot_ids, n_rows, static_cast<u32x4*>(rows));
    return hipGetLastError();
}

}  // namespace omni
