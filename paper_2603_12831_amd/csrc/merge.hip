// Merge of partial attention rows from up to four sources (split-KV chunks,
// externally produced partials, GPU tails) into final rows.  The rule is the
// exact identity of Eq. 1 (paper, Background) over a disjoint union of token
// sets: w_p = exp(LSE_p - max LSE), O = sum w_p O_p / sum w_p,
// LSE = max LSE + ln sum w_p.  This is the GPU-side aggregation of the
// intermediate results that the paper's CPU attention threads produce.
//
// One thread owns four consecutive dims of one (sequence, head) row, so a row
// is read with 16-byte loads by head_dim/4 adjacent lanes.  A partial whose
// LSE is -inf is skipped without touching its O row.
#include "omni_internal.hpp"

namespace omni {
namespace {

constexpr int kMaxSrcs = (int)(sizeof(MergeParams{}.src) / sizeof(omni_partial_src));   // sources of one call

template <int D, int kBatch>
__global__ __launch_bounds__(256) void merge_kernel(MergeParams p)
{
    constexpr int kLanesPerRow = D / 4;
    constexpr int kRowsPerBlock = 256 / kLanesPerRow;
    const long long row = (long long)blockIdx.x * kRowsPerBlock + threadIdx.x / kLanesPerRow;
    const int quad = threadIdx.x % kLanesPerRow;
    if (row >= (long long)p.batch * p.hq) return;
    const int seq = (int)(row / p.hq), head = (int)(row % p.hq);
    // where the sequence's rows are in each source, requested together with the flag that may end the thread
    // here (offsets read after the flag would be one more memory round trip in a kernel that is a handful of them)
    int first[kMaxSrcs], last[kMaxSrcs];
#pragma unroll
    for (int s = 0; s < kMaxSrcs; ++s) {
        first[s] = last[s] = 0;
        if (s < p.n_srcs) src_rows(p.src[s], seq, first[s], last[s]);
    }
    if (p.skip && p.skip[seq] != 0) return;                // the decode call already wrote this sequence's final row

    // Rows are visited kBatch at a time so that kBatch independent loads are in flight per lane: the kernel
    // is a handful of dependent memory round trips, not a bandwidth problem.  The launcher picks kBatch by how
    // many rows a sequence can have (fewer, larger turns for many rows; small turns, i.e. few registers and
    // more resident workgroups, for two or three rows).
    float m = -INFINITY;
#pragma unroll
    for (int s = 0; s < kMaxSrcs; ++s) {
        if (s >= p.n_srcs) break;
        const int r0 = first[s], r1 = last[s];
        const float* lse = p.src[s].lse + head;
        for (int r = r0; r < r1; r += kBatch) {
            float l[kBatch];
#pragma unroll
            for (int u = 0; u < kBatch; ++u) l[u] = (r + u < r1) ? lse[(long long)(r + u) * p.hq] : -INFINITY;
#pragma unroll
            for (int u = 0; u < kBatch; ++u) m = fmaxf(m, l[u]);
        }
    }
    float4 acc = make_float4(0.f, 0.f, 0.f, 0.f);
    float wsum = 0.f;
    if (m != -INFINITY) {
#pragma unroll
        for (int s = 0; s < kMaxSrcs; ++s) {
            if (s >= p.n_srcs) break;
            const int r0 = first[s], r1 = last[s];
            const float* lse = p.src[s].lse + head;
            const float* orow = p.src[s].o + (long long)head * D + quad * 4;
            for (int r = r0; r < r1; r += kBatch) {
                float w[kBatch];
                float4 o[kBatch];
#pragma unroll
                for (int u = 0; u < kBatch; ++u) {
                    const float l = (r + u < r1) ? lse[(long long)(r + u) * p.hq] : -INFINITY;
                    w[u] = (l == -INFINITY) ? 0.f : expf(l - m);
                }
#pragma unroll
                for (int u = 0; u < kBatch; ++u) {       // a row without weight is not read at all
                    o[u] = make_float4(0.f, 0.f, 0.f, 0.f);
                    if (w[u] != 0.f) o[u] = *reinterpret_cast<const float4*>(orow + (long long)(r + u) * p.hq * D);
                }
#pragma unroll
                for (int u = 0; u < kBatch; ++u) {
                    wsum += w[u];
                    acc.x = fmaf(w[u], o[u].x, acc.x); acc.y = fmaf(w[u], o[u].y, acc.y);
                    acc.z = fmaf(w[u], o[u].z, acc.z); acc.w = fmaf(w[u], o[u].w, acc.w);
                }
            }
        }
        float inv = 1.f / wsum;
        acc.x *= inv; acc.y *= inv; acc.z *= inv; acc.w *= inv;
    }
    if (p.out_bf16) {
        uint2 pk;
        pk.x = (uint32_t)f32_to_bf16(acc.x) | ((uint32_t)f32_to_bf16(acc.y) << 16);
        pk.y = (uint32_t)f32_to_bf16(acc.z) | ((uint32_t)f32_to_bf16(acc.w) << 16);
        *reinterpret_cast<uint2*>(static_cast<uint16_t*>(p.out_o) + row * D + quad * 4) = pk;
    } else {
        *reinterpret_cast<float4*>(static_cast<float*>(p.out_o) + row * D + quad * 4) = acc;
    }
    if (p.out_lse && quad == 0) p.out_lse[row] = (m == -INFINITY) ? -INFINITY : m + logf(wsum);
}

}  // namespace

namespace {

template <int kBatch>
void launch_merge_batch(const MergeParams& p, long long rows, hipStream_t s)
{
    if (p.d == 64) {
        unsigned grid = (unsigned)((rows + 15) / 16);
        hipLaunchKernelGGL((merge_kernel<64, kBatch>), dim3(grid), dim3(256), 0, s, p);
    } else {
        unsigned grid = (unsigned)((rows + 7) / 8);
        hipLaunchKernelGGL((merge_kernel<128, kBatch>), dim3(grid), dim3(256), 0, s, p);
    }
}

}  // namespace

hipError_t launch_merge(const MergeParams& p, hipStream_t s)
{
    long long rows = (long long)p.batch * p.hq;
    if (rows == 0) return hipSuccess;
    // rows a sequence may have: what the dense sources say, two for a source with row offsets (measured:
    // turns of 4 / 8 / 32 rows are best for the hybrid batch / 8-chunk rows / 32-chunk rows, each by 1-3 us)
    long long hint = 0;
    for (int i = 0; i < p.n_srcs; ++i) hint += p.src[i].row_offsets ? 2 : p.src[i].dense_rows_per_seq;
    if (hint <= 4) launch_merge_batch<4>(p, rows, s);
    else if (hint <= 12) launch_merge_batch<8>(p, rows, s);
    else if (hint <= 24) launch_merge_batch<16>(p, rows, s);
    else launch_merge_batch<32>(p, rows, s);
    return hipGetLastError();
}

}  // namespace omni
