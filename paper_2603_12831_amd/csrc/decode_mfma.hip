// Matrix-core decode attention for bf16 KV, head_dim 128, GQA ratio G <= 16.
//
// One workgroup of four waves per (sequence, chunk, kv head): every KV byte of
// the chunk is read exactly once and serves all G query heads that share the
// kv head (Eq. 1 of the paper's Background section for G queries at a time).
// The chunk's pages are taken two at a time (a 32-token step); the steps are
// dealt round-robin to the four waves.  Per step a wave computes, with
// v_mfma_f32_16x16x32_bf16,
//
//   S^T[token, g]  = K[token, :] . Q[g, :]         (A = K tile, B = Q^T)
//   O^T[dim, g]   += V^T[dim, token] . P^T[token, g]  (A = V^T tile, B = P^T)
//
// Operand layouts of the 16x16x32 instruction: lane l supplies row/col l%16
// and eight consecutive k of group l/16; the result puts col l%16, rows
// 4*(l/16)+i in register i.
//
//   * K is loaded straight into the A layout: lane l reads 16 bytes of token
//     row tau(l%16) at dims kb*32 + (l/16)*8, tau(r) = 4*(r%4) + r/4.
//   * With that token order the S^T result registers of a lane (tokens
//     4i + l/16, i = 0..3, of each page) are exactly the k-slots the lane must
//     supply for P^T, so softmax weights never cross lanes.
//   * V is loaded with fully contiguous wave loads (lane l reads bytes
//     l*16 .. l*16+15 of each KiB of the page: token 4i + l/16, dims
//     (l%16)*8 .. +7) and transposed inside the lane with byte permutes into
//     V^T operands (row = dim group l%16, k = the lane's eight tokens).
//   * P is split into a bf16 head and a bf16 remainder (two MFMAs), which keeps
//     the weights to ~2^-17 relative error; the products with bf16 V and the
//     accumulation are fp32.
//
// The online softmax works in the log2 domain (logits pre-multiplied by
// sm_scale * log2 e), keeps one running maximum per query head (max over the
// lane's registers, then across the four lane groups) and rescales the
// accumulator only when some maximum of the wave moved.  The four waves'
// states are combined through LDS with the log-sum-exp rule.
#include "omni_internal.hpp"

namespace omni {
namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

constexpr int kWaves = 4;
constexpr int kD = 128;
constexpr int kPageBytes = kBlockSize * kD * 2;        // one (page, kv head) tile of K or of V
constexpr float kLog2e = 1.4426950408889634f;
constexpr float kLn2 = 0.6931471805599453f;

struct PageRegs {            // raw registers of one page: 4 KiB of K and 4 KiB of V across the wave
    u32x4 k[4];
    u32x4 v[4];
};

__device__ __forceinline__ uint32_t pack_lo(uint32_t x, uint32_t y) { return __builtin_amdgcn_perm(y, x, 0x05040100u); }
__device__ __forceinline__ uint32_t pack_hi(uint32_t x, uint32_t y) { return __builtin_amdgcn_perm(y, x, 0x07060302u); }

__device__ __forceinline__ uint32_t pack_bf16(float a, float b)
{
    f32x2 p = {a, b};
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(p, bf16x2));
}

// One 4 KiB tile (K or V of one page and kv head) into four 16-byte registers per lane; `stride` is
// the byte distance between the lane's four loads.  An absent page (< 0) reads page 0 instead, so the
// load is always in bounds; the caller masks every token of such a page.
__device__ __forceinline__ void load_tile(const void* __restrict__ pool, int hkv, long long page, int kvh,
                                          int lane_off, int stride, u32x4 (&r)[4])
{
    const long long pg = page < 0 ? 0 : page;
    const char* src = static_cast<const char*>(pool) + (pg * hkv + kvh) * (long long)kPageBytes + lane_off;
#pragma unroll
    for (int i = 0; i < 4; ++i) r[i] = *reinterpret_cast<const u32x4*>(src + i * stride);
}

// physical page of logical page index `lp` (wave-uniform) if it lies in [.., lp_last] and names a pool
// page, else -1
__device__ __forceinline__ long long page_of(const DecodeParams& p, const int* __restrict__ table, int lp,
                                             int lp_last)
{
    lp = __builtin_amdgcn_readfirstlane(lp);
    if (lp > lp_last) return -1;
    long long pg = table[lp];
    return (pg >= 0 && pg < p.num_blocks) ? pg : -1;
}

__global__ __launch_bounds__(kWaves * kWave, 2) void decode_mfma_kernel(DecodeParams p, const int* __restrict__ block_table)
{
    const int item = blockIdx.x;
    const int kvh = item % p.hkv;
    const int seq = (item / p.hkv) % p.batch;
    const int chunk = item / (p.hkv * p.batch);
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int col = lane & 15;                 // query head of the group (S^T / O^T column), or dim group for V
    const int kg = lane >> 4;                  // k group
    const int G = p.group;

    int b, e, cb, ce;
    seq_range(p, seq, b, e);
    chunk_range(p, b, e, chunk, cb, ce);
    const bool final_row = p.out_o != nullptr;                 // only set when max_chunks == 1
    const long long prow0 = ((long long)seq * p.max_chunks + chunk) * p.hq + (long long)kvh * G;
    const long long orow0 = (long long)seq * p.hq + (long long)kvh * G;

    if (ce <= cb) {                            // empty chunk: LSE = -inf, partial O left unwritten
        if (threadIdx.x < G) {
            if (p.part_lse) p.part_lse[prow0 + threadIdx.x] = -INFINITY;
            if (final_row && p.out_lse) p.out_lse[orow0 + threadIdx.x] = -INFINITY;
        }
        if (final_row) {
            for (int i = threadIdx.x; i < G * kD; i += kWaves * kWave) {
                if (p.out_bf16) static_cast<uint16_t*>(p.out_o)[orow0 * kD + i] = 0;
                else static_cast<float*>(p.out_o)[orow0 * kD + i] = 0.f;
            }
        }
        return;
    }

    // Q^T operands: lane supplies head `col`, dims kb*32 + kg*8 .. +7; heads beyond G are zero columns
    u32x4 qb[4];
    {
        const u32x4 z = {0, 0, 0, 0};
        const char* qp = static_cast<const char*>(p.q) + ((orow0 + col) * kD + kg * 8) * 2;
#pragma unroll
        for (int kb = 0; kb < 4; ++kb) qb[kb] = (col < G) ? *reinterpret_cast<const u32x4*>(qp + kb * 64) : z;
    }

    const int* __restrict__ table = block_table + (long long)seq * p.max_blocks;
    const int lp_first = cb >> 4, lp_last = (ce - 1) >> 4;
    const int n_steps = (lp_last - lp_first + 2) >> 1;
    const int tau = 4 * (col & 3) + (col >> 2);            // token row this lane loads of K
    const int k_lane_off = tau * (kD * 2) + kg * 16;
    const int v_lane_off = lane * 16;
    const float scale2 = p.sm_scale * kLog2e;

    f32x4 acc[8];                                          // acc[j][i] = O^T[dim (4*kg+i)*8 + j][head col]
#pragma unroll
    for (int j = 0; j < 8; ++j) acc[j] = f32x4{0.f, 0.f, 0.f, 0.f};
    float m_run = -INFINITY;                               // running max (log2 domain) of head `col`
    float l_run = 0.f;                                     // this lane's share of the running sum

    PageRegs pa, pb;                                       // the two pages of the current step
    int s = wave;
    long long pgA = -1, pgB = -1;                          // physical pages of the step in registers
    if (s < n_steps) {
        pgA = page_of(p, table, lp_first + 2 * s, lp_last);
        pgB = page_of(p, table, lp_first + 2 * s + 1, lp_last);
        load_tile(p.k_pool, p.hkv, pgA, kvh, k_lane_off, 64, pa.k);      // dims i*32 + kg*8 .. of token tau
        load_tile(p.k_pool, p.hkv, pgB, kvh, k_lane_off, 64, pb.k);
        load_tile(p.v_pool, p.hkv, pgA, kvh, v_lane_off, 1024, pa.v);    // token 4i + kg, dims col*8 ..
        load_tile(p.v_pool, p.hkv, pgB, kvh, v_lane_off, 1024, pb.v);
    }
    while (s < n_steps) {
        const int lp0 = lp_first + 2 * s;
        const bool okA = pgA >= 0, okB = pgB >= 0;
        const int sn = s + kWaves;
        if (sn < n_steps) {
            pgA = page_of(p, table, lp_first + 2 * sn, lp_last);
            pgB = page_of(p, table, lp_first + 2 * sn + 1, lp_last);
        }

        // ---- S^T = K . Q^T for both pages -------------------------------------------------
        f32x4 sa = {0.f, 0.f, 0.f, 0.f}, sb = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int kb = 0; kb < 4; ++kb) {
            sa = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, pa.k[kb]),
                                                         __builtin_bit_cast(bf16x8, qb[kb]), sa, 0, 0, 0);
            sb = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, pb.k[kb]),
                                                         __builtin_bit_cast(bf16x8, qb[kb]), sb, 0, 0, 0);
        }
        __builtin_amdgcn_sched_barrier(0);
        if (sn < n_steps) {                                // K registers are free again: prefetch next K
            load_tile(p.k_pool, p.hkv, pgA, kvh, k_lane_off, 64, pa.k);
            load_tile(p.k_pool, p.hkv, pgB, kvh, k_lane_off, 64, pb.k);
        }
        __builtin_amdgcn_sched_barrier(0);
        // ---- V^T operands of this step (then the V registers are free for the prefetch) ----
        // word j/2, half j%2 of load i holds dim (l%16)*8 + j of token 4i + kg
        u32x4 vt[8];
#pragma unroll
        for (int jj = 0; jj < 4; ++jj) {
            vt[2 * jj] = u32x4{pack_lo(pa.v[0][jj], pa.v[1][jj]), pack_lo(pa.v[2][jj], pa.v[3][jj]),
                               pack_lo(pb.v[0][jj], pb.v[1][jj]), pack_lo(pb.v[2][jj], pb.v[3][jj])};
            vt[2 * jj + 1] = u32x4{pack_hi(pa.v[0][jj], pa.v[1][jj]), pack_hi(pa.v[2][jj], pa.v[3][jj]),
                                   pack_hi(pb.v[0][jj], pb.v[1][jj]), pack_hi(pb.v[2][jj], pb.v[3][jj])};
        }
        __builtin_amdgcn_sched_barrier(0);
        if (sn < n_steps) {
            load_tile(p.v_pool, p.hkv, pgA, kvh, v_lane_off, 1024, pa.v);
            load_tile(p.v_pool, p.hkv, pgB, kvh, v_lane_off, 1024, pb.v);
        }
        __builtin_amdgcn_sched_barrier(0);

        // ---- logits to the log2 domain, masking on boundary steps ---------------------------
        const int t0 = lp0 << 4;                           // first token of page A; register i is token 4i + kg
        const bool interior = okA && okB && t0 >= cb && t0 + 32 <= ce;
#pragma unroll
        for (int i = 0; i < 4; ++i) { sa[i] *= scale2; sb[i] *= scale2; }
        if (!interior) {
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const int ta = t0 + 4 * i + kg, tb = ta + 16;
                const bool va = okA && ta >= cb && ta < ce;
                const bool vb = okB && tb >= cb && tb < ce;
                sa[i] = va ? sa[i] : -INFINITY;
                sb[i] = vb ? sb[i] : -INFINITY;
                // a masked token's V must not reach the MFMA (0 * NaN): V^T slot i (page A), 4+i (page B).
                // slots 2w, 2w+1 share word w of every vt[j]
                if (!va) {
#pragma unroll
                    for (int j = 0; j < 8; ++j) vt[j][i >> 1] &= (i & 1) ? 0x0000ffffu : 0xffff0000u;
                }
                if (!vb) {
#pragma unroll
                    for (int j = 0; j < 8; ++j) vt[j][2 + (i >> 1)] &= (i & 1) ? 0x0000ffffu : 0xffff0000u;
                }
            }
        }
        // ---- online softmax ------------------------------------------------------------------
        float mx = fmaxf(fmaxf(fmaxf(sa[0], sa[1]), fmaxf(sa[2], sa[3])),
                         fmaxf(fmaxf(sb[0], sb[1]), fmaxf(sb[2], sb[3])));
        mx = fmaxf(mx, __shfl_xor(mx, 16));
        mx = fmaxf(mx, __shfl_xor(mx, 32));
        const float m_new = fmaxf(m_run, mx);
        const float m_use = (m_new == -INFINITY) ? 0.f : m_new;      // nothing seen yet: avoid inf - inf
        if (__any(m_new > m_run)) {
            const float corr = __builtin_amdgcn_exp2f(m_run - m_use);   // 0 when m_run = -inf
            l_run *= corr;
#pragma unroll
            for (int j = 0; j < 8; ++j) acc[j] *= corr;
        }
        m_run = m_new;
        float pw[8];
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            pw[i] = __builtin_amdgcn_exp2f(sa[i] - m_use);
            pw[4 + i] = __builtin_amdgcn_exp2f(sb[i] - m_use);
        }
        l_run += ((pw[0] + pw[1]) + (pw[2] + pw[3])) + ((pw[4] + pw[5]) + (pw[6] + pw[7]));
        // P^T operand: bf16 head and bf16 remainder of every weight
        u32x4 ph, pl;
#pragma unroll
        for (int w = 0; w < 4; ++w) {
            const uint32_t h = pack_bf16(pw[2 * w], pw[2 * w + 1]);
            ph[w] = h;
            pl[w] = pack_bf16(pw[2 * w] - bf16lo_to_f32(h), pw[2 * w + 1] - bf16hi_to_f32(h));
        }
        // ---- O^T += V^T . P^T ------------------------------------------------------------------
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            acc[j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, vt[j]),
                                                             __builtin_bit_cast(bf16x8, ph), acc[j], 0, 0, 0);
            acc[j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, vt[j]),
                                                             __builtin_bit_cast(bf16x8, pl), acc[j], 0, 0, 0);
        }
        s = sn;
    }

    // ---- combine the four waves ------------------------------------------------------------------
    l_run += __shfl_xor(l_run, 16);
    l_run += __shfl_xor(l_run, 32);
    extern __shared__ float lds[];                         // [kWaves][G][kD] accumulators, then m and l
    float* sh_acc = lds;
    float* sh_m = lds + kWaves * G * kD;
    float* sh_l = sh_m + kWaves * 16;
    if (col < G) {
        float* dst = sh_acc + (wave * G + col) * kD;
#pragma unroll
        for (int j = 0; j < 8; ++j)
#pragma unroll
            for (int i = 0; i < 4; ++i) dst[(4 * kg + i) * 8 + j] = acc[j][i];
        if (kg == 0) { sh_m[wave * 16 + col] = m_run; sh_l[wave * 16 + col] = l_run; }
    }
    __syncthreads();
    for (int idx = threadIdx.x; idx < G * kD; idx += kWaves * kWave) {
        const int g = idx >> 7, d = idx & (kD - 1);
        float mm = -INFINITY;
#pragma unroll
        for (int w = 0; w < kWaves; ++w) mm = fmaxf(mm, sh_m[w * 16 + g]);
        float o = 0.f, lse = -INFINITY;
        if (mm != -INFINITY) {
            float ll = 0.f, oo = 0.f;
#pragma unroll
            for (int w = 0; w < kWaves; ++w) {
                const float mw = sh_m[w * 16 + g];
                const float f = (mw == -INFINITY) ? 0.f : __builtin_amdgcn_exp2f(mw - mm);
                ll += f * sh_l[w * 16 + g];
                oo += f * sh_acc[(w * G + g) * kD + d];
            }
            o = oo / ll;
            lse = (mm + __builtin_amdgcn_logf(ll)) * kLn2;           // v_log_f32 is log2
            if (p.part_o) p.part_o[(prow0 + g) * kD + d] = o;
        }
        if (p.part_lse && d == 0) p.part_lse[prow0 + g] = lse;
        if (final_row) {
            if (p.out_bf16) static_cast<uint16_t*>(p.out_o)[(orow0 + g) * kD + d] = f32_to_bf16(o);
            else static_cast<float*>(p.out_o)[(orow0 + g) * kD + d] = o;
            if (p.out_lse && d == 0) p.out_lse[orow0 + g] = lse;
        }
    }
}

}  // namespace

bool decode_mfma_supports(const DecodeParams& p, bool bf16)
{
    return bf16 && p.d == kD && p.group <= 16 &&
           (long long)p.batch * p.max_chunks * p.hkv <= 0x7fffffffLL;
}

hipError_t launch_decode_mfma(const DecodeParams& p, hipStream_t s)
{
    const unsigned grid = (unsigned)((long long)p.batch * p.max_chunks * p.hkv);
    const size_t lds = (size_t)(kWaves * p.group * kD + 2 * kWaves * 16) * sizeof(float);
    hipLaunchKernelGGL(decode_mfma_kernel, dim3(grid), dim3(kWaves * kWave), lds, s, p, p.block_table);
    return hipGetLastError();
}

}  // namespace omni
