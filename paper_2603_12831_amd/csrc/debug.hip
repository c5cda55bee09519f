// Test and measurement aids: block-table gather, streaming read, plain copy.
#include "omni_internal.hpp"

namespace omni {
namespace {

// One thread per 16-byte piece of an output row; rows are (token, kv head).
__global__ __launch_bounds__(256) void gather_kernel(DecodeParams p, int elem_bytes, int seq, uint4* k_out, uint4* v_out)
{
    int b, e;
    seq_range(p, seq, b, e);
    const int pieces = p.d * elem_bytes / 16;                 // 16-byte pieces per row
    const long long total = (long long)(e > b ? e - b : 0) * p.hkv * pieces;
    const long long i = (long long)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= total) return;
    const int piece = (int)(i % pieces);
    const long long rowi = i / pieces;
    const int h = (int)(rowi % p.hkv);
    const int t = b + (int)(rowi / p.hkv);
    const long long page = p.block_table[(long long)seq * p.max_blocks + (t >> 4)];
    uint4 kk = make_uint4(0, 0, 0, 0), vv = kk;
    if (page >= 0 && page < p.num_blocks) {
        long long src = (((page * p.hkv + h) * kBlockSize + (t & 15)) * pieces) + piece;
        kk = static_cast<const uint4*>(p.k_pool)[src];
        vv = static_cast<const uint4*>(p.v_pool)[src];
    }
    k_out[i] = kk;
    v_out[i] = vv;
}

constexpr int kStreamUnroll = 8;

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

__global__ __launch_bounds__(256) void stream_read_kernel(const u32x4* __restrict__ src, long long n_vec, uint32_t* sink)
{
    // each workgroup walks a contiguous slab of kStreamUnroll * 256 vectors per step
    u32x4 acc = {0, 0, 0, 0};
    const u32x4 zero = {0, 0, 0, 0};
    const long long step = (long long)gridDim.x * blockDim.x * kStreamUnroll;
    for (long long base = (long long)blockIdx.x * blockDim.x * kStreamUnroll; base < n_vec; base += step) {
        u32x4 v[kStreamUnroll];
#pragma unroll
        for (int u = 0; u < kStreamUnroll; ++u) {
            long long i = base + (long long)u * blockDim.x + threadIdx.x;
            v[u] = i < n_vec ? __builtin_nontemporal_load(src + i) : zero;
        }
#pragma unroll
        for (int u = 0; u < kStreamUnroll; ++u) acc ^= v[u];
    }
    // the fold depends on every loaded word, and is stored only for a value that never occurs by chance
    uint32_t f = acc.x ^ acc.y ^ acc.z ^ acc.w;
    if (f == 0x9e3779b9u) sink[threadIdx.x & 3] = f;
}

__global__ __launch_bounds__(256) void copy_kernel(uint4* __restrict__ dst, const uint4* __restrict__ src, long long n_vec)
{
    const long long step = (long long)gridDim.x * blockDim.x;
    for (long long i = (long long)blockIdx.x * blockDim.x + threadIdx.x; i < n_vec; i += step) dst[i] = src[i];
}

}  // namespace

hipError_t launch_gather(const DecodeParams& p, bool bf16, int seq, void* k_out, void* v_out, hipStream_t s)
{
    // the token count lives on the device; launch for the largest possible range
    const int elem_bytes = bf16 ? 2 : 4;
    long long total = (long long)p.max_blocks * kBlockSize * p.hkv * (p.d * elem_bytes / 16);
    unsigned grid = (unsigned)((total + 255) / 256);
    if (grid == 0) return hipSuccess;
    hipLaunchKernelGGL(gather_kernel, dim3(grid), dim3(256), 0, s, p, elem_bytes, seq,
                       static_cast<uint4*>(k_out), static_cast<uint4*>(v_out));
    return hipGetLastError();
}

hipError_t launch_stream_read(const void* src, size_t bytes, uint32_t* sink, hipStream_t s)
{
    long long n_vec = (long long)(bytes / 16);
    if (n_vec == 0) return hipSuccess;
    long long want = (n_vec + 256LL * kStreamUnroll - 1) / (256LL * kStreamUnroll);
    unsigned grid = (unsigned)(want < 256 * 16 ? want : 256 * 16);
    hipLaunchKernelGGL(stream_read_kernel, dim3(grid), dim3(256), 0, s, static_cast<const u32x4*>(src), n_vec, sink);
    return hipGetLastError();
}

hipError_t launch_copy(void* dst, const void* src, size_t bytes, hipStream_t s)
{
    long long n_vec = (long long)(bytes / 16);
    if (n_vec == 0) return hipSuccess;
    long long want = (n_vec + 255) / 256;
    unsigned grid = (unsigned)(want < 256 * 32 ? want : 256 * 32);
    hipLaunchKernelGGL(copy_kernel, dim3(grid), dim3(256), 0, s, static_cast<uint4*>(dst), static_cast<const uint4*>(src), n_vec);
    return hipGetLastError();
}

}  // namespace omni
