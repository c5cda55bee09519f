// Vector-ALU decode attention: the any-shape kernel (fp32 or bf16, head_dim 64 or 128, any GQA ratio up to
// 16).  One workgroup of four waves per (sequence, chunk, kv head): every KV byte of the chunk is read once
// and serves all G query heads that share the kv head (Eq. 1 of the paper's Background section for G
// queries at a time, restricted to the chunk); with more than eight heads to a kv head, two workgroups
// take eight heads each (the register file holds the states of eight).
//
// A wave looks at four tokens at a time: sixteen lanes share a token row, each lane holding head_dim/16
// consecutive dims, so a wave load covers whole contiguous rows.  A lane takes kUnroll tokens per turn
// (their loads go out together), forms the G dot products of each (partial sums over its dims, then a
// sum over the sixteen lanes of the row), and updates the online-softmax state of its 16-lane group
// once per turn: one running maximum, sum and accumulator slice per head.  The sixteen group states of the
// workgroup are combined at the end with the same log-sum-exp rule the merge uses: the four groups of a wave
// by lane shuffles, the four waves through LDS.
#include <type_traits>

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

// Sum over the sixteen lanes that share a token row, left in every one of them: four adds whose second
// operand comes through the data-parallel lane permutes (neighbour in the pair, other pair of the quad,
// mirrored half row, mirrored row) - vector-ALU instructions, where lane shuffles would go through the LDS
// pipe, which four waves of a CU share (the shuffles were what bounded this kernel).
__device__ __forceinline__ float row16_sum(float x)
{
    constexpr int kQuadPerm1032 = 0xB1, kQuadPerm2301 = 0x4E, kRowHalfMirror = 0x141, kRowMirror = 0x140;
    auto from = [](float v, auto ctrl) {
        return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), decltype(ctrl)::value,
                                                                     0xf, 0xf, true));
    };
    x += from(x, std::integral_constant<int, kQuadPerm1032>{});
    x += from(x, std::integral_constant<int, kQuadPerm2301>{});
    x += from(x, std::integral_constant<int, kRowHalfMirror>{});
    x += from(x, std::integral_constant<int, kRowMirror>{});
    return x;
}

constexpr int kWaves = 4;
constexpr int kGroups = kWaves * 4;            // 16-lane groups per workgroup
constexpr int kUnroll = 4;                     // tokens a 16-lane group takes per turn

// GMAX: compile-time bound of the heads per kv head the instance serves (registers are sized for it).
// `listed`: the launch goes by a work list (`entries`: every (sequence, chunk) slot of the call, the non-empty
// ranges longest first, then the empty ones): the grid walks the entries in list order, so the hardware, which
// starts workgroups in grid order, deals the long ranges out first and the empty slots last - ragged batches
// with many empty chunk slots otherwise ran at two thirds of the rate of uniform ones.  Without a list the
// grid is (kv head, chunk slot, sequence) and every workgroup works its range out itself.
template <typename T, int D, int GMAX, bool listed>
__global__ __launch_bounds__(kWaves * kWave) void decode_vector_kernel(DecodeParams p, const WorkEntry* __restrict__ entries)
{
    constexpr int E = D / 16;
    const int splits = (p.group + GMAX - 1) / GMAX;             // workgroups that share a kv head's heads
    // (listed: a one-dimensional grid, the head blocks of an entry side by side as in the other form)
    const int head_blocks = p.hkv * splits;
    const int head_block = listed ? blockIdx.x % head_blocks : blockIdx.x;
    const int kvh = head_block / splits;
    const int head0 = kvh * p.group + (head_block % splits) * GMAX;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int sub = lane & 15;                 // which E dims of the row
    const int grp = wave * 4 + (lane >> 4);    // which token of each 16-token turn
    const int G = min(GMAX, (kvh + 1) * p.group - head0);       // heads of this workgroup: head0 .. head0 + G - 1

    int seq, chunk, cb, ce, n_parts;
    if (listed) {
        // (a list planned for these very ranges holds only values that pass unchanged; one reused against
        // the contract is forced into bounds, so that wrong rows are the worst that can come of it)
        const WorkEntry w = entries[blockIdx.x / head_blocks];
        seq = min(max(w.seq, 0), p.batch - 1);
        chunk = min(chunk_index(w.chunk), p.max_chunks - 1);
        n_parts = chunk_live(w.chunk);
        cb = max(w.cb, 0);
        ce = min(w.ce, p.max_blocks * kBlockSize);
    } else {
        seq = blockIdx.z;
        chunk = blockIdx.y;
        int b, e;
        seq_range(p, seq, b, e);
        chunk_range(p, b, e, chunk, cb, ce);
        n_parts = seq_parts(p, seq, b, e);
    }
    // a sequence with at most one non-empty chunk (chunk 0) gets its final row from this kernel
    const bool seq_direct = p.out_o != nullptr && n_parts <= 1;
    if (p.seq_final && head_block == 0 && chunk == 0 && threadIdx.x == 0) p.seq_final[seq] = seq_direct ? 1 : 0;

    // Logits in the log2 domain and the hardware's exp2 / log2 (about one ulp), for both input types: the
    // library's expf / logf on natural logits gave fp32 inputs no smaller errors (seeded fp32 batches: worst
    // 1.6e-6 of the 1e-5 bound either way, set by the fp32 sums of the products) at a quarter more instructions.
    constexpr float kLog2e = 1.4426950408889634f, kLn2 = 0.6931471805599453f;
    const float qscale = p.sm_scale * kLog2e;
    auto ex = [](float x) { return __builtin_amdgcn_exp2f(x); };
    float q[GMAX][E];
#pragma unroll
    for (int g = 0; g < GMAX; ++g) {
#pragma unroll
        for (int i = 0; i < E; ++i) q[g][i] = 0.f;
        if (g < G) {
            RowVec<T, E>::load(p.q, ((long long)seq * p.hq + head0 + g) * D + sub * E, q[g]);
#pragma unroll
            for (int i = 0; i < E; ++i) q[g][i] *= qscale;
        }
    }
    float m[GMAX], l[GMAX], acc[GMAX][E];
#pragma unroll
    for (int g = 0; g < GMAX; ++g) {
        m[g] = -INFINITY;
        l[g] = 0.f;
#pragma unroll
        for (int i = 0; i < E; ++i) acc[g][i] = 0.f;
    }

    // The pages of a turn's tokens are looked up one turn ahead (all of a turn's table entries in one go,
    // requested behind the previous turn's K / V rows), so that a turn is one memory round trip - its rows -
    // and not a chain of table entry, rows, table entry, rows ...
    const int* table = p.block_table + (long long)seq * p.max_blocks;
    auto page_of_token = [&](int t) { return t < ce ? table[t >> 4] : -1; };
    int pages[kUnroll];
#pragma unroll
    for (int u = 0; u < kUnroll; ++u) pages[u] = page_of_token(cb + grp + u * kGroups);
    for (int t0 = cb + grp; t0 < ce; t0 += kGroups * kUnroll) {
        float kx[kUnroll][E], vx[kUnroll][E];
        bool live[kUnroll];
#pragma unroll
        for (int u = 0; u < kUnroll; ++u) {
            const int t = t0 + u * kGroups;
            const long long page = pages[u];
            live[u] = page >= 0 && page < p.num_blocks;          // absent page: its tokens do not exist
            const long long row = live[u] ? ((page * p.hkv + kvh) * kBlockSize + (t & 15)) * D + sub * E : 0;
            RowVec<T, E>::load(p.k_pool, row, kx[u]);
            RowVec<T, E>::load(p.v_pool, row, vx[u]);
        }
#pragma unroll
        for (int u = 0; u < kUnroll; ++u) pages[u] = page_of_token(t0 + (kUnroll + u) * kGroups);
        // a token that is not there: its weight will be zero, and its V must not reach the sums (0 * NaN)
#pragma unroll
        for (int u = 0; u < kUnroll; ++u)
#pragma unroll
            for (int i = 0; i < E; ++i) vx[u][i] = live[u] ? vx[u][i] : 0.f;
#pragma unroll
        for (int g = 0; g < GMAX; ++g) {
            if (g >= G) break;
            float s[kUnroll];
#pragma unroll
            for (int u = 0; u < kUnroll; ++u) {
                float dot = 0.f;
#pragma unroll
                for (int i = 0; i < E; ++i) dot = fmaf(q[g][i], kx[u][i], dot);
                s[u] = live[u] ? row16_sum(dot) : -INFINITY;
            }
            float m_new = m[g];
#pragma unroll
            for (int u = 0; u < kUnroll; ++u) m_new = fmaxf(m_new, s[u]);
            if (m_new == -INFINITY) continue;                    // nothing live in this turn, nothing before
            const float corr = ex(m[g] - m_new);                 // exp(-inf) = 0 on the first live token
            float w[kUnroll], wsum = 0.f;
#pragma unroll
            for (int u = 0; u < kUnroll; ++u) {
                w[u] = ex(s[u] - m_new);                         // exp(-inf) = 0 for a token that is not there
                wsum += w[u];
            }
            l[g] = l[g] * corr + wsum;
#pragma unroll
            for (int i = 0; i < E; ++i) {
                float a = acc[g][i] * corr;
#pragma unroll
                for (int u = 0; u < kUnroll; ++u) a = fmaf(w[u], vx[u][i], a);
                acc[g][i] = a;
            }
            m[g] = m_new;
        }
    }

    // the four groups of a wave first (lanes 16 and 32 apart hold the same dims of the same head) ...
#pragma unroll
    for (int g = 0; g < GMAX; ++g) {
        if (g >= G) break;
#pragma unroll
        for (int d = 16; d <= 32; d <<= 1) {
            const float m_o = __shfl_xor(m[g], d), l_o = __shfl_xor(l[g], d);
            const float m_new = fmaxf(m[g], m_o);
            const float f_me = m[g] == -INFINITY ? 0.f : ex(m[g] - m_new);
            const float f_o = m_o == -INFINITY ? 0.f : ex(m_o - m_new);
            l[g] = l[g] * f_me + l_o * f_o;
#pragma unroll
            for (int i = 0; i < E; ++i) acc[g][i] = acc[g][i] * f_me + __shfl_xor(acc[g][i], d) * f_o;
            m[g] = m_new;
        }
    }
    // ... then the four waves through LDS
    extern __shared__ float sh[];                                // [kWaves][G] m, [kWaves][G] l, [kWaves][G][D] acc
    float* sh_m = sh;
    float* sh_l = sh + kWaves * G;
    float* sh_acc = sh + 2 * kWaves * G;
    if (lane < 16) {
#pragma unroll
        for (int g = 0; g < GMAX; ++g) {
            if (g >= G) break;
            if (sub == 0) { sh_m[wave * G + g] = m[g]; sh_l[wave * G + g] = l[g]; }
#pragma unroll
            for (int i = 0; i < E; ++i) sh_acc[(wave * G + g) * D + sub * E + i] = acc[g][i];
        }
    }
    __syncthreads();

    const bool final_row = seq_direct && chunk == 0;
    const bool partial_row = !seq_direct || p.max_chunks == 1;     // a one-slot call keeps the partial as well
    for (int idx = threadIdx.x; idx < G * D; idx += kWaves * kWave) {
        const int g = idx / D, dim = idx - g * D;
        float mm = -INFINITY;
#pragma unroll
        for (int w = 0; w < kWaves; ++w) mm = fmaxf(mm, sh_m[w * G + g]);
        const long long prow = ((long long)seq * p.max_chunks + chunk) * p.hq + head0 + g;
        const long long orow = (long long)seq * p.hq + head0 + g;
        float o = 0.f, lse = -INFINITY;
        if (mm != -INFINITY) {
            float ll = 0.f, oo = 0.f;
#pragma unroll
            for (int w = 0; w < kWaves; ++w) {
                const float mw = sh_m[w * G + g];
                const float f = (mw == -INFINITY) ? 0.f : ex(mw - mm);
                ll += f * sh_l[w * G + g];
                oo += f * sh_acc[(w * G + g) * D + dim];
            }
            o = oo / ll;
            lse = (mm + __builtin_amdgcn_logf(ll)) * kLn2;                              // (v_log_f32 is log2)
            if (p.part_o && partial_row) p.part_o[prow * D + dim] = o;
        }
        if (p.part_lse && dim == 0) p.part_lse[prow] = partial_row ? lse : -INFINITY;
        if (final_row) {
            if (p.out_bf16) static_cast<uint16_t*>(p.out_o)[orow * D + dim] = f32_to_bf16(o);
            else static_cast<float*>(p.out_o)[orow * D + dim] = o;
            if (p.out_lse && dim == 0) p.out_lse[orow] = lse;
        }
    }
}

template <typename T, int D, bool listed>
hipError_t launch_for_group(const DecodeParams& p, const WorkEntry* entries, hipStream_t s)
{
    const int per = p.group <= 1 ? 1 : (p.group <= 4 ? 4 : 8);            // heads a workgroup serves at most
    const int splits = (p.group + per - 1) / per;
    const long long listed_blocks = (long long)p.batch * p.max_chunks * p.hkv * splits;
    if (listed && listed_blocks > 0x7fffffffLL) return hipErrorInvalidValue;       // (a list of that size: > 32 GB of entries)
    const dim3 grid = listed ? dim3((unsigned)listed_blocks, 1, 1) : dim3(p.hkv * splits, p.max_chunks, p.batch);
    const dim3 block(kWaves * kWave);
    const size_t lds = (size_t)(2 * kWaves * per + kWaves * per * D) * sizeof(float);
    if (per == 1) hipLaunchKernelGGL((decode_vector_kernel<T, D, 1, listed>), grid, block, lds, s, p, entries);
    else if (per == 4) hipLaunchKernelGGL((decode_vector_kernel<T, D, 4, listed>), grid, block, lds, s, p, entries);
    else hipLaunchKernelGGL((decode_vector_kernel<T, D, 8, listed>), grid, block, lds, s, p, entries);
    return hipGetLastError();
}

template <bool listed>
hipError_t launch_for_type(const DecodeParams& p, bool bf16, const WorkEntry* entries, hipStream_t s)
{
    if (bf16) return p.d == 64 ? launch_for_group<uint16_t, 64, listed>(p, entries, s)
                               : launch_for_group<uint16_t, 128, listed>(p, entries, s);
    return p.d == 64 ? launch_for_group<float, 64, listed>(p, entries, s) : launch_for_group<float, 128, listed>(p, entries, s);
}

}  // namespace

// With a workspace the launch goes by the work list in it (built here unless `planned` says it is there).
hipError_t launch_decode_vector(const DecodeParams& p, bool bf16, void* workspace, bool planned, hipStream_t s)
{
    if (!workspace) return launch_for_type<false>(p, bf16, nullptr, s);
    if (!planned) {
        const hipError_t e = launch_decode_plan(p, workspace, s);
        if (e != hipSuccess) return e;
    }
    const WorkEntry* entries = reinterpret_cast<const WorkEntry*>(static_cast<const unsigned*>(workspace) + kHeaderWords);
    return launch_for_type<true>(p, bf16, entries, s);
}

}  // namespace omni
