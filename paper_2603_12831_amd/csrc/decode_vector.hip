// Vector-ALU decode attention: the any-shape kernel (fp32 or bf16, head_dim 64
// or 128, any GQA ratio).  One workgroup of four waves per (sequence, chunk,
// query head).  A wave looks at four tokens at a time: sixteen lanes share a
// token row, each lane holding head_dim/16 consecutive dims, so a wave load
// covers whole contiguous rows.  Each 16-lane group keeps its own online-
// softmax state over the tokens it sees; the sixteen states of the workgroup
// are combined through LDS at the end with the same log-sum-exp rule the
// merge uses.  Computes Eq. 1 of the paper's Background section restricted to
// the chunk.
#include "omni_internal.hpp"

namespace omni {
namespace {

template <typename T, int E> struct RowVec;   // E consecutive elements widened to fp32
template <> struct RowVec<float, 4> {
    static __device__ __forceinline__ void load(const void* base, long long elem, float* out) {
        float4 v = *reinterpret_cast<const float4*>(static_cast<const float*>(base) + elem);
        out[0] = v.x; out[1] = v.y; out[2] = v.z; out[3] = v.w;
    }
};
template <> struct RowVec<float, 8> {
    static __device__ __forceinline__ void load(const void* base, long long elem, float* out) {
        RowVec<float, 4>::load(base, elem, out);
        RowVec<float, 4>::load(base, elem + 4, out + 4);
    }
};
template <> struct RowVec<uint16_t, 4> {
    static __device__ __forceinline__ void load(const void* base, long long elem, float* out) {
        uint2 v = *reinterpret_cast<const uint2*>(static_cast<const uint16_t*>(base) + elem);
        out[0] = bf16lo_to_f32(v.x); out[1] = bf16hi_to_f32(v.x);
        out[2] = bf16lo_to_f32(v.y); out[3] = bf16hi_to_f32(v.y);
    }
};
template <> struct RowVec<uint16_t, 8> {
    static __device__ __forceinline__ void load(const void* base, long long elem, float* out) {
        uint4 v = *reinterpret_cast<const uint4*>(static_cast<const uint16_t*>(base) + elem);
        out[0] = bf16lo_to_f32(v.x); out[1] = bf16hi_to_f32(v.x);
        out[2] = bf16lo_to_f32(v.y); out[3] = bf16hi_to_f32(v.y);
        out[4] = bf16lo_to_f32(v.z); out[5] = bf16hi_to_f32(v.z);
        out[6] = bf16lo_to_f32(v.w); out[7] = bf16hi_to_f32(v.w);
    }
};

constexpr int kWaves = 4;
constexpr int kGroups = kWaves * 4;            // 16-lane groups per workgroup

template <typename T, int D>
__global__ __launch_bounds__(kWaves * kWave) void decode_vector_kernel(DecodeParams p)
{
    constexpr int E = D / 16;
    const int head = blockIdx.x, chunk = blockIdx.y, seq = blockIdx.z;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int sub = lane & 15;                 // which E dims of the row
    const int grp = wave * 4 + (lane >> 4);    // which token of each 16-token step
    const int kvh = head / p.group;

    int b, e, cb, ce;
    seq_range(p, seq, b, e);
    chunk_range(p, b, e, chunk, cb, ce);
    // a sequence with at most one non-empty chunk (chunk 0) gets its final row from this kernel
    const bool seq_direct = p.out_o != nullptr && live_chunks(p, b, e) <= 1;
    if (p.seq_final && head == 0 && chunk == 0 && threadIdx.x == 0) p.seq_final[seq] = seq_direct ? 1 : 0;

    float q[E];
    RowVec<T, E>::load(p.q, ((long long)seq * p.hq + head) * D + sub * E, q);

    float m = -INFINITY, l = 0.f, acc[E];
#pragma unroll
    for (int i = 0; i < E; ++i) acc[i] = 0.f;

    const int* table = p.block_table + (long long)seq * p.max_blocks;
    for (int t = cb + grp; t < ce; t += kGroups) {
        long long page = table[t >> 4];
        if (page < 0 || page >= p.num_blocks) continue;      // absent page: its tokens do not exist
        long long row = ((page * p.hkv + kvh) * kBlockSize + (t & 15)) * D + sub * E;
        float kx[E], vx[E];
        RowVec<T, E>::load(p.k_pool, row, kx);
        RowVec<T, E>::load(p.v_pool, row, vx);
        float dot = 0.f;
#pragma unroll
        for (int i = 0; i < E; ++i) dot = fmaf(q[i], kx[i], dot);
        dot += __shfl_xor(dot, 1);
        dot += __shfl_xor(dot, 2);
        dot += __shfl_xor(dot, 4);
        dot += __shfl_xor(dot, 8);
        float s = dot * p.sm_scale;
        float m_new = fmaxf(m, s);
        float corr = expf(m - m_new);                        // exp(-inf) = 0 on the first token
        float w = expf(s - m_new);
        l = l * corr + w;
#pragma unroll
        for (int i = 0; i < E; ++i) acc[i] = acc[i] * corr + w * vx[i];
        m = m_new;
    }

    __shared__ float sh_m[kGroups], sh_l[kGroups], sh_acc[kGroups][D];
    if (sub == 0) { sh_m[grp] = m; sh_l[grp] = l; }
#pragma unroll
    for (int i = 0; i < E; ++i) sh_acc[grp][sub * E + i] = acc[i];
    __syncthreads();

    const int dim = threadIdx.x;
    if (dim >= D) return;
    float mm = -INFINITY;
#pragma unroll
    for (int g = 0; g < kGroups; ++g) mm = fmaxf(mm, sh_m[g]);
    const long long prow = ((long long)seq * p.max_chunks + chunk) * p.hq + head;
    const bool final_row = seq_direct && chunk == 0;
    const bool partial_row = !seq_direct || p.max_chunks == 1;     // a one-slot call keeps the partial as well
    const long long orow = (long long)seq * p.hq + head;
    float o = 0.f, lse = -INFINITY;
    if (mm != -INFINITY) {
        float ll = 0.f, oo = 0.f;
#pragma unroll
        for (int g = 0; g < kGroups; ++g) {
            float w = (sh_m[g] == -INFINITY) ? 0.f : expf(sh_m[g] - mm);
            ll += w * sh_l[g];
            oo += w * sh_acc[g][dim];
        }
        o = oo / ll;
        lse = mm + logf(ll);
        if (p.part_o && partial_row) p.part_o[prow * D + dim] = o;
    }
    if (p.part_lse && dim == 0) p.part_lse[prow] = partial_row ? lse : -INFINITY;
    if (final_row) {
        if (p.out_bf16) static_cast<uint16_t*>(p.out_o)[orow * D + dim] = f32_to_bf16(o);
        else static_cast<float*>(p.out_o)[orow * D + dim] = o;
        if (p.out_lse && dim == 0) p.out_lse[orow] = lse;
    }
}

}  // namespace

hipError_t launch_decode_vector(const DecodeParams& p, bool bf16, hipStream_t s)
{
    dim3 grid(p.hq, p.max_chunks, p.batch), block(kWaves * kWave);
    if (bf16) {
        if (p.d == 64) hipLaunchKernelGGL((decode_vector_kernel<uint16_t, 64>), grid, block, 0, s, p);
        else hipLaunchKernelGGL((decode_vector_kernel<uint16_t, 128>), grid, block, 0, s, p);
    } else {
        if (p.d == 64) hipLaunchKernelGGL((decode_vector_kernel<float, 64>), grid, block, 0, s, p);
        else hipLaunchKernelGGL((decode_vector_kernel<float, 128>), grid, block, 0, s, p);
    }
    return hipGetLastError();
}

}  // namespace omni
