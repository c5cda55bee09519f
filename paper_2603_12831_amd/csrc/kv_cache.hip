// KV-cache data movement next to the attention path: appending the new token's k, v to its page before
// the decode step (the paper's decode context counts the current token), and gathering / scattering whole
// pages between the pools and a contiguous staging buffer, the device side of the one-shot KV swap-out /
// swap-in of a request (paper, KV cache management).  Pure copies: bit-exact, bound by HBM bandwidth.
#include "omni_internal.hpp"

namespace omni {
namespace {

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

// one thread per 16-byte piece of a (sequence, kv head) row, K and V
__global__ __launch_bounds__(256) void kv_append_kernel(KvParams c, const u32x4* __restrict__ k_new,
                                                        const u32x4* __restrict__ v_new,
                                                        const int* __restrict__ positions)
{
    const int pieces = c.d * c.elem_bytes / 16;
    const long long total = (long long)c.batch * c.hkv * pieces;
    const long long i = (long long)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= total) return;
    const int piece = (int)(i % pieces);
    const int h = (int)((i / pieces) % c.hkv);
    const int seq = (int)(i / ((long long)pieces * c.hkv));
    const int pos = positions[seq];
    if (pos < 0 || (pos >> 4) >= c.max_blocks) return;        // no slot for this position: nothing written
    const long long page = c.block_table[(long long)seq * c.max_blocks + (pos >> 4)];
    if (page < 0 || page >= c.num_blocks) return;
    const long long dst = (((page * c.hkv + h) * kBlockSize + (pos & 15)) * pieces) + piece;
    static_cast<u32x4*>(c.k_pool)[dst] = k_new[i];
    static_cast<u32x4*>(c.v_pool)[dst] = v_new[i];
}

// whole pages (all kv heads) between the pools and staging[n_pages][hkv][16][d]; grid-stride over 16-byte
// pieces, a page's pieces handled by consecutive threads
template <bool to_pool>
__global__ __launch_bounds__(256) void kv_pages_kernel(KvParams c, const int* __restrict__ page_ids,
                                                       long long n_pages, u32x4* k_stage, u32x4* v_stage)
{
    const long long per_page = (long long)c.hkv * kBlockSize * c.d * c.elem_bytes / 16;
    const long long total = n_pages * per_page;
    const long long step = (long long)gridDim.x * blockDim.x;
    for (long long i = (long long)blockIdx.x * blockDim.x + threadIdx.x; i < total; i += step) {
        const long long slot = i / per_page, piece = i - slot * per_page;
        const long long page = page_ids[slot];
        const bool ok = page >= 0 && page < c.num_blocks;
        const long long pool_idx = (ok ? page : 0) * per_page + piece;
        if (to_pool) {
            if (ok) {
                static_cast<u32x4*>(c.k_pool)[pool_idx] = __builtin_nontemporal_load(k_stage + i);
                static_cast<u32x4*>(c.v_pool)[pool_idx] = __builtin_nontemporal_load(v_stage + i);
            }
        } else {
            const u32x4 z = {0, 0, 0, 0};
            u32x4 kk = z, vv = z;
            if (ok) {
                kk = __builtin_nontemporal_load(static_cast<const u32x4*>(c.k_pool) + pool_idx);
                vv = __builtin_nontemporal_load(static_cast<const u32x4*>(c.v_pool) + pool_idx);
            }
            __builtin_nontemporal_store(kk, k_stage + i);
            __builtin_nontemporal_store(vv, v_stage + i);
        }
    }
}

}  // namespace

hipError_t launch_kv_append(const KvParams& c, const void* k_new, const void* v_new, const int* positions, hipStream_t s)
{
    const long long total = (long long)c.batch * c.hkv * (c.d * c.elem_bytes / 16);
    if (total == 0) return hipSuccess;
    hipLaunchKernelGGL(kv_append_kernel, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, s, c,
                       static_cast<const u32x4*>(k_new), static_cast<const u32x4*>(v_new), positions);
    return hipGetLastError();
}

hipError_t launch_kv_pages(const KvParams& c, const int* page_ids, long long n_pages, void* k_stage, void* v_stage,
                           bool to_pool, hipStream_t s)
{
    const long long total = n_pages * ((long long)c.hkv * kBlockSize * c.d * c.elem_bytes / 16);
    if (total == 0) return hipSuccess;
    const long long want = (total + 255) / 256;
    const unsigned grid = (unsigned)(want < 256 * 32 ? want : 256 * 32);
    if (to_pool)
        hipLaunchKernelGGL((kv_pages_kernel<true>), dim3(grid), dim3(256), 0, s, c, page_ids, n_pages,
                           static_cast<u32x4*>(k_stage), static_cast<u32x4*>(v_stage));
    else
        hipLaunchKernelGGL((kv_pages_kernel<false>), dim3(grid), dim3(256), 0, s, c, page_ids, n_pages,
                           static_cast<u32x4*>(k_stage), static_cast<u32x4*>(v_stage));
    return hipGetLastError();
}

}  // namespace omni
