// Host-side producer of partial attention rows (the paper's System Implementation, "CPU Attention":
// threads on the host's cores each compute a part of the attention load over KV held in host memory,
// vectorised inside a core, and the intermediate results are aggregated).
//
// A row is one (sequence, token range); for each of its query heads the producer writes the partial
// (O normalised inside the range, LSE natural log of the scaled logits) in the format
// omni_merge_partials takes as a CSR source.  Work is cut into units of one (row, kv head, slice of at
// most kSliceTokens tokens): a unit streams its K and V once for the G query heads that share the kv
// head, keeping (max, sum, accumulator) per head in fp32; worker threads draw units from an atomic
// counter and a second pass folds the slices of a (row, kv head) together with the log-sum-exp rule.
// Everything here is plain C++ on host memory: no HIP call is made.
#include "omni_attn.h"

#include <immintrin.h>

#include <algorithm>
#include <atomic>
#include <cmath>
#include <cstdint>
#include <cstring>
#include <limits>
#include <memory>
#include <thread>
#include <vector>

namespace {

constexpr int kPage = 16;
constexpr int kSliceTokens = 512;                      // a multiple of the page size
constexpr int kMaxGroup = 16;

struct HostParams {
    int n_rows, batch, hq, hkv, group, d, max_blocks;
    long long num_blocks;
    bool bf16;
    float sm_scale;
    const void *q, *k_pool, *v_pool;
    const int32_t *block_table, *row_seq, *row_begin, *row_end;
    float *part_o, *part_lse;
};

struct Unit { int row, kvh, t0, t1; };                 // tokens [t0, t1) of the row's sequence

inline float bf16_to_f32(uint16_t h)
{
    const uint32_t u = (uint32_t)h << 16;
    float f;
    std::memcpy(&f, &u, sizeof f);
    return f;
}

// The compute of a unit exists for three instruction-set levels (plain x86-64, AVX2 + FMA, AVX-512) and the
// level is chosen once per call from what the CPU reports (or by the caller).  The first two are the plain
// loops below, which the compiler vectorises for each level; the AVX-512 level is written out further down.
#define OMNI_HOST_INLINE static inline __attribute__((always_inline))

// e^x for x <= 0 (a weight exp(s - max)) from plain arithmetic, so that a loop over the tokens of a page
// vectorises: n = round(x log2 e), r = x - n ln 2 in two pieces, a degree-6 polynomial for e^r on
// |r| <= ln 2 / 2 (relative error ~1e-7), and 2^n put into the exponent field.  Below -87 the result is 0.
OMNI_HOST_INLINE float exp_nonpos(float x)
{
    const float xc = x < -87.0f ? -87.0f : x;
    const float t = xc * 1.44269504088896341f;
    const int n = (int)(t - 0.5f);                         // round to nearest for t <= 0
    const float nf = (float)n;
    float r = xc - nf * 0.693145751953125f;                // ln 2, high part (exact product for |n| < 2^11)
    r = r - nf * 1.42860682030941723e-6f;                  //       low part
    float p = 1.0f / 720.0f;
    p = p * r + 1.0f / 120.0f;
    p = p * r + 1.0f / 24.0f;
    p = p * r + 1.0f / 6.0f;
    p = p * r + 0.5f;
    p = p * r + 1.0f;
    p = p * r + 1.0f;
    const uint32_t bits = (uint32_t)(n + 127) << 23;
    float scale;
    std::memcpy(&scale, &bits, sizeof scale);
    return x < -87.0f ? 0.0f : p * scale;
}

// 16 x D tile of one (page, kv head) as fp32
template <int D>
OMNI_HOST_INLINE void load_tile(const void* pool, bool bf16, long long page, int hkv, int kvh, float (&out)[kPage][D])
{
    const size_t tile = ((size_t)page * hkv + kvh) * (size_t)(kPage * D);
    if (bf16) {
        const uint16_t* src = static_cast<const uint16_t*>(pool) + tile;
        for (int t = 0; t < kPage; ++t)
            for (int i = 0; i < D; ++i) out[t][i] = bf16_to_f32(src[t * D + i]);
    } else {
        std::memcpy(out, static_cast<const float*>(pool) + tile, sizeof(float) * kPage * D);
    }
}

// One unit: running (m, l, acc) of G heads over the unit's tokens.  m in natural-log units of the
// scaled logits; acc is the un-normalised sum of exp(s - m) v.
template <int D>
OMNI_HOST_INLINE void run_unit(const HostParams& p, const Unit& u, float* m, float* l, float* acc /* [G][D] */)
{
    const int G = p.group;
    const int seq = p.row_seq[u.row];
    float qf[kMaxGroup][D];
    for (int g = 0; g < G; ++g) {
        const size_t off = ((size_t)seq * p.hq + (size_t)u.kvh * G + g) * D;
        for (int i = 0; i < D; ++i)
            qf[g][i] = (p.bf16 ? bf16_to_f32(static_cast<const uint16_t*>(p.q)[off + i])
                               : static_cast<const float*>(p.q)[off + i]) * p.sm_scale;
        m[g] = -std::numeric_limits<float>::infinity();
        l[g] = 0.f;
        for (int i = 0; i < D; ++i) acc[g * D + i] = 0.f;
    }
    const int32_t* table = p.block_table + (size_t)seq * p.max_blocks;
    alignas(64) float kf[kPage][D], vf[kPage][D];
    for (int lp = u.t0 / kPage; lp * kPage < u.t1; ++lp) {
        const long long page = table[lp];
        if (page < 0 || page >= p.num_blocks) continue;            // absent page: its tokens do not count
        const int s0 = std::max(u.t0 - lp * kPage, 0), s1 = std::min(u.t1 - lp * kPage, kPage);
        load_tile<D>(p.k_pool, p.bf16, page, p.hkv, u.kvh, kf);
        load_tile<D>(p.v_pool, p.bf16, page, p.hkv, u.kvh, vf);
        for (int g = 0; g < G; ++g) {
            float s[kPage] = {0.f};
            float mx = m[g];
            for (int t = s0; t < s1; ++t) {
                float lanes[16] = {0.f};                           // 16 running sums: vectorises as is
                for (int i = 0; i < D; i += 16)
                    for (int j = 0; j < 16; ++j) lanes[j] += qf[g][i + j] * kf[t][i + j];
                for (int w = 8; w > 0; w >>= 1)
                    for (int j = 0; j < w; ++j) lanes[j] += lanes[j + w];
                const float dot = lanes[0];
                s[t] = dot;
                mx = std::max(mx, dot);
            }
            const float corr = (m[g] == -std::numeric_limits<float>::infinity()) ? 0.f : exp_nonpos(m[g] - mx);
            float* a = acc + g * D;
            for (int i = 0; i < D; ++i) a[i] *= corr;
            float sum = l[g] * corr;
            float w[kPage];
            for (int t = 0; t < kPage; ++t) w[t] = (t >= s0 && t < s1) ? exp_nonpos(s[t] - mx) : 0.f;
            for (int t = s0; t < s1; ++t) {
                sum += w[t];
                for (int i = 0; i < D; ++i) a[i] += w[t] * vf[t][i];
            }
            m[g] = mx;
            l[g] = sum;
        }
    }
}

// ---- the AVX-512 level, written out --------------------------------------------------------------------
// The plain loops above leave three things on the table that decide this path's rate on a host with
// 512-bit vectors: the eight multiply-adds of a logit form one dependent chain, every logit ends in a
// horizontal sum of its own, and the exponentials are scalar.  Here a page's 16 logits of a head are
// 16 partial-sum vectors (up to four heads at a time, so four independent chains per K row) that are
// reduced together by a transposing tree (45 shuffles and adds for 16 sums), the softmax of the page is
// one vector, and the output rows of two to four heads stay in registers over the page's tokens.
#define OMNI_AVX512_TARGET __attribute__((target("avx512f,avx512vl,avx512bw,avx512dq,fma")))
#define OMNI_AVX512_INLINE static inline __attribute__((always_inline)) OMNI_AVX512_TARGET

// 16 values from element `idx` on, widened to fp32
OMNI_AVX512_INLINE __m512 load16_f32(const void* base, bool bf16, size_t idx)
{
    if (bf16) {
        const __m256i h = _mm256_loadu_si256(reinterpret_cast<const __m256i*>(static_cast<const uint16_t*>(base) + idx));
        return _mm512_castsi512_ps(_mm512_slli_epi32(_mm512_cvtepu16_epi32(h), 16));
    }
    return _mm512_loadu_ps(static_cast<const float*>(base) + idx);
}

// e^x for x <= 0 or -inf, 16 at a time (as exp_nonpos: two-piece ln 2, degree-6 polynomial)
OMNI_AVX512_INLINE __m512 exp_nonpos16(__m512 x)
{
    const __m512 lo = _mm512_set1_ps(-87.0f);
    const __mmask16 live = _mm512_cmp_ps_mask(x, lo, _CMP_GE_OQ);
    const __m512 xc = _mm512_max_ps(x, lo);
    const __m512 nf = _mm512_roundscale_ps(_mm512_mul_ps(xc, _mm512_set1_ps(1.44269504088896341f)),
                                           _MM_FROUND_TO_NEAREST_INT | _MM_FROUND_NO_EXC);
    __m512 r = _mm512_fnmadd_ps(nf, _mm512_set1_ps(0.693145751953125f), xc);
    r = _mm512_fnmadd_ps(nf, _mm512_set1_ps(1.42860682030941723e-6f), r);
    __m512 p = _mm512_set1_ps(1.0f / 720.0f);
    p = _mm512_fmadd_ps(p, r, _mm512_set1_ps(1.0f / 120.0f));
    p = _mm512_fmadd_ps(p, r, _mm512_set1_ps(1.0f / 24.0f));
    p = _mm512_fmadd_ps(p, r, _mm512_set1_ps(1.0f / 6.0f));
    p = _mm512_fmadd_ps(p, r, _mm512_set1_ps(0.5f));
    p = _mm512_fmadd_ps(p, r, _mm512_set1_ps(1.0f));
    p = _mm512_fmadd_ps(p, r, _mm512_set1_ps(1.0f));
    return _mm512_maskz_mov_ps(live, _mm512_scalef_ps(p, nf));
}

// sums of four vectors inside each 128-bit lane: lane L of the result holds, for i = 0..3, the sum of the
// four elements of lane L of v[i]
OMNI_AVX512_INLINE __m512 lane_sums4(__m512 v0, __m512 v1, __m512 v2, __m512 v3)
{
    const __m512 ab = _mm512_add_ps(_mm512_unpacklo_ps(v0, v1), _mm512_unpackhi_ps(v0, v1));
    const __m512 cd = _mm512_add_ps(_mm512_unpacklo_ps(v2, v3), _mm512_unpackhi_ps(v2, v3));
    return _mm512_add_ps(_mm512_shuffle_ps(ab, cd, 0x44), _mm512_shuffle_ps(ab, cd, 0xEE));
}

// element t of the result = sum of the 16 elements of rows[t]
OMNI_AVX512_INLINE __m512 row_sums16(const float (&rows)[kPage][16])
{
    __m512 r[4];
    for (int q = 0; q < 4; ++q)
        r[q] = lane_sums4(_mm512_load_ps(rows[4 * q]), _mm512_load_ps(rows[4 * q + 1]), _mm512_load_ps(rows[4 * q + 2]),
                          _mm512_load_ps(rows[4 * q + 3]));
    // lane q of the result = sum over the four lanes of r[q]
    const __m512 u01 = _mm512_add_ps(_mm512_shuffle_f32x4(r[0], r[1], 0x44), _mm512_shuffle_f32x4(r[0], r[1], 0xEE));
    const __m512 u23 = _mm512_add_ps(_mm512_shuffle_f32x4(r[2], r[3], 0x44), _mm512_shuffle_f32x4(r[2], r[3], 0xEE));
    return _mm512_add_ps(_mm512_shuffle_f32x4(u01, u23, 0x88), _mm512_shuffle_f32x4(u01, u23, 0xDD));
}

// partial sums of the logits of heads g0 .. g0+HB-1 against the 16 K rows of a page: part[h][t] = the 16
// running sums of q_h . k_t, one per 16-dim chunk position
template <int D, int HB>
OMNI_AVX512_INLINE void logit_parts(const float (&kf)[kPage][D], const float (*qf)[D], int g0, float (*part)[kPage][16])
{
    for (int t = 0; t < kPage; ++t) {
        __m512 a[HB];
        for (int h = 0; h < HB; ++h) a[h] = _mm512_setzero_ps();
        for (int c = 0; c < D / 16; ++c) {
            const __m512 kz = _mm512_load_ps(&kf[t][16 * c]);
            for (int h = 0; h < HB; ++h) a[h] = _mm512_fmadd_ps(kz, _mm512_load_ps(&qf[g0 + h][16 * c]), a[h]);
        }
        for (int h = 0; h < HB; ++h) _mm512_store_ps(part[h][t], a[h]);
    }
}

// acc rows of heads g0 .. g0+HB-1 (in memory, [G][D]): scaled by corr[g], plus w[g][t] v_t over tokens s0 .. s1-1
template <int D, int HB>
OMNI_AVX512_INLINE void accumulate_rows(const float (&vf)[kPage][D], const float (*w)[kPage], const float* corr, int g0,
                                        int s0, int s1, float* acc)
{
    constexpr int C = D / 16;
    __m512 a[HB][C];
    for (int h = 0; h < HB; ++h) {
        const __m512 f = _mm512_set1_ps(corr[g0 + h]);
        for (int c = 0; c < C; ++c) a[h][c] = _mm512_mul_ps(_mm512_loadu_ps(acc + (size_t)(g0 + h) * D + 16 * c), f);
    }
    for (int t = s0; t < s1; ++t) {
        __m512 wb[HB];
        for (int h = 0; h < HB; ++h) wb[h] = _mm512_set1_ps(w[g0 + h][t]);
        for (int c = 0; c < C; ++c) {
            const __m512 vz = _mm512_load_ps(&vf[t][16 * c]);
            for (int h = 0; h < HB; ++h) a[h][c] = _mm512_fmadd_ps(wb[h], vz, a[h][c]);
        }
    }
    for (int h = 0; h < HB; ++h)
        for (int c = 0; c < C; ++c) _mm512_storeu_ps(acc + (size_t)(g0 + h) * D + 16 * c, a[h][c]);
}

template <int D>
OMNI_AVX512_TARGET static void run_unit_avx512(const HostParams& p, const Unit& u, float* m, float* l, float* acc /* [G][D] */)
{
    constexpr int C = D / 16;
    constexpr int VB = D == 128 ? 2 : 4;                   // heads whose output rows fit the registers together
    const int G = p.group;
    const int seq = p.row_seq[u.row];
    const float ninf = -std::numeric_limits<float>::infinity();
    alignas(64) float qf[kMaxGroup][D];
    const __m512 scale = _mm512_set1_ps(p.sm_scale);
    for (int g = 0; g < G; ++g) {
        const size_t off = ((size_t)seq * p.hq + (size_t)u.kvh * G + g) * D;
        for (int c = 0; c < C; ++c) _mm512_store_ps(&qf[g][16 * c], _mm512_mul_ps(load16_f32(p.q, p.bf16, off + 16 * c), scale));
        m[g] = ninf;
        l[g] = 0.f;
        for (int i = 0; i < D; ++i) acc[g * D + i] = 0.f;
    }
    const int32_t* table = p.block_table + (size_t)seq * p.max_blocks;
    alignas(64) float kf[kPage][D], vf[kPage][D];
    alignas(64) float part[4][kPage][16];
    alignas(64) float w[kMaxGroup][kPage];
    float corr[kMaxGroup];
    for (int lp = u.t0 / kPage; lp * kPage < u.t1; ++lp) {
        const long long page = table[lp];
        if (page < 0 || page >= p.num_blocks) continue;            // absent page: its tokens do not count
        const int s0 = std::max(u.t0 - lp * kPage, 0), s1 = std::min(u.t1 - lp * kPage, kPage);
        const __mmask16 in_range = (__mmask16)(((1u << s1) - 1u) & ~((1u << s0) - 1u));
        const size_t tile = ((size_t)page * p.hkv + u.kvh) * (size_t)(kPage * D);
        for (int t = 0; t < kPage; ++t)
            for (int c = 0; c < C; ++c) {
                _mm512_store_ps(&kf[t][16 * c], load16_f32(p.k_pool, p.bf16, tile + (size_t)t * D + 16 * c));
                _mm512_store_ps(&vf[t][16 * c], load16_f32(p.v_pool, p.bf16, tile + (size_t)t * D + 16 * c));
            }
        // logits and weights, up to four heads at a time (rows outside the range hold whatever the page holds:
        // their logits are replaced before they are used)
        for (int g0 = 0; g0 < G;) {
            const int hb = G - g0 >= 4 ? 4 : (G - g0 >= 2 ? 2 : 1);
            if (hb == 4) logit_parts<D, 4>(kf, qf, g0, part);
            else if (hb == 2) logit_parts<D, 2>(kf, qf, g0, part);
            else logit_parts<D, 1>(kf, qf, g0, part);
            for (int h = 0; h < hb; ++h) {
                const int g = g0 + h;
                const __m512 s = _mm512_mask_mov_ps(_mm512_set1_ps(ninf), in_range, row_sums16(part[h]));
                const float mx = std::max(m[g], _mm512_reduce_max_ps(s));
                const __m512 wv = exp_nonpos16(_mm512_sub_ps(s, _mm512_set1_ps(mx)));
                _mm512_store_ps(w[g], wv);
                corr[g] = m[g] == ninf ? 0.f : exp_nonpos(m[g] - mx);
                l[g] = l[g] * corr[g] + _mm512_reduce_add_ps(wv);
                m[g] = mx;
            }
            g0 += hb;
        }
        for (int g0 = 0; g0 < G;) {
            const int hb = G - g0 >= VB ? VB : (G - g0 >= 2 ? 2 : 1);
            if (hb == 4) accumulate_rows<D, 4>(vf, w, corr, g0, s0, s1, acc);
            else if (hb == 2) accumulate_rows<D, 2>(vf, w, corr, g0, s0, s1, acc);
            else accumulate_rows<D, 1>(vf, w, corr, g0, s0, s1, acc);
            g0 += hb;
        }
    }
}

typedef void (*UnitFn)(const HostParams&, const Unit&, float*, float*, float*);

#define OMNI_HOST_UNIT(name, D, target_attr)                                                        \
    target_attr static void name(const HostParams& p, const Unit& u, float* m, float* l, float* acc) \
    {                                                                                               \
        run_unit<D>(p, u, m, l, acc);                                                               \
    }
OMNI_HOST_UNIT(unit_base_64, 64, )
OMNI_HOST_UNIT(unit_base_128, 128, )
OMNI_HOST_UNIT(unit_avx2_64, 64, __attribute__((target("avx2,fma"))))
OMNI_HOST_UNIT(unit_avx2_128, 128, __attribute__((target("avx2,fma"))))
OMNI_AVX512_TARGET static void unit_avx512_64(const HostParams& p, const Unit& u, float* m, float* l, float* acc)
{
    run_unit_avx512<64>(p, u, m, l, acc);
}
OMNI_AVX512_TARGET static void unit_avx512_128(const HostParams& p, const Unit& u, float* m, float* l, float* acc)
{
    run_unit_avx512<128>(p, u, m, l, acc);
}

// level: 0 = best available, 1 = plain, 2 = AVX2 + FMA, 3 = AVX-512; null if the CPU lacks the level
UnitFn pick_unit_fn(int d, int level)
{
    __builtin_cpu_init();
    const bool avx512 = __builtin_cpu_supports("avx512f") && __builtin_cpu_supports("avx512vl") &&
                        __builtin_cpu_supports("avx512bw") && __builtin_cpu_supports("avx512dq");
    const bool avx2 = __builtin_cpu_supports("avx2") && __builtin_cpu_supports("fma");
    if (level == 0) level = avx512 ? 3 : (avx2 ? 2 : 1);
    if (level == 3) return avx512 ? (d == 128 ? unit_avx512_128 : unit_avx512_64) : nullptr;
    if (level == 2) return avx2 ? (d == 128 ? unit_avx2_128 : unit_avx2_64) : nullptr;
    return d == 128 ? unit_base_128 : unit_base_64;
}

template <int D>
void produce(const HostParams& p, int n_threads, UnitFn unit_fn)
{
    // units, grouped by (row, kv head) in order
    std::vector<Unit> units;
    std::vector<size_t> first_unit((size_t)p.n_rows * p.hkv + 1, 0);
    const int cap = p.max_blocks * kPage;
    for (int r = 0; r < p.n_rows; ++r) {
        const int b = std::max(p.row_begin ? p.row_begin[r] : 0, 0), e = std::min(p.row_end[r], cap);
        for (int h = 0; h < p.hkv; ++h) {
            first_unit[(size_t)r * p.hkv + h] = units.size();
            for (int t = b; t < e;) {
                const int stop = std::min(e, (t / kSliceTokens + 1) * kSliceTokens);
                units.push_back(Unit{r, h, t, stop});
                t = stop;
            }
        }
    }
    first_unit.back() = units.size();
    const int G = p.group;
    const size_t stride = (size_t)G * (D + 2);                    // per unit: m[G], l[G], acc[G][D]
    // (not a std::vector: that would fill tens of megabytes with zeros on one thread before any work starts;
    // every unit writes all of its slot)
    std::unique_ptr<float[]> partial_mem(new float[units.size() * stride]);
    float* const partial = partial_mem.get();

    auto run_parallel = [&](size_t count, auto&& body) {
        std::atomic<size_t> next{0};
        auto worker = [&] {
            for (size_t i; (i = next.fetch_add(1, std::memory_order_relaxed)) < count;) body(i);
        };
        const int n = (int)std::min<size_t>(std::max(n_threads, 1), std::max<size_t>(count, 1));
        std::vector<std::thread> pool;
        for (int t = 1; t < n; ++t) pool.emplace_back(worker);
        worker();
        for (auto& th : pool) th.join();
    };

    // longest units first would not matter (all are at most kSliceTokens); draw in order
    run_parallel(units.size(), [&](size_t i) {
        float* res = partial + i * stride;
        unit_fn(p, units[i], res, res + G, res + 2 * G);
    });

    // fold the slices of each (row, kv head) and write the rows
    run_parallel((size_t)p.n_rows * p.hkv, [&](size_t rk) {
        const int r = (int)(rk / p.hkv), h = (int)(rk % p.hkv);
        const size_t u0 = first_unit[rk], u1 = first_unit[rk + 1];
        for (int g = 0; g < G; ++g) {
            const size_t row = ((size_t)r * p.hq + (size_t)h * G + g);
            float mm = -std::numeric_limits<float>::infinity();
            for (size_t u = u0; u < u1; ++u) mm = std::max(mm, partial[u * stride + g]);
            float* out = p.part_o + row * D;
            if (mm == -std::numeric_limits<float>::infinity()) {
                p.part_lse[row] = mm;
                for (int i = 0; i < D; ++i) out[i] = 0.f;
                continue;
            }
            float ll = 0.f;
            float o[D];
            for (int i = 0; i < D; ++i) o[i] = 0.f;
            for (size_t u = u0; u < u1; ++u) {
                const float* res = partial + u * stride;
                if (res[g] == -std::numeric_limits<float>::infinity()) continue;
                const float f = std::exp(res[g] - mm);
                ll += f * res[G + g];
                const float* a = res + 2 * G + (size_t)g * D;
                for (int i = 0; i < D; ++i) o[i] += f * a[i];
            }
            const float inv = 1.f / ll;
            for (int i = 0; i < D; ++i) out[i] = o[i] * inv;
            p.part_lse[row] = mm + std::log(ll);
        }
    });
}

}  // namespace

extern "C" omni_status omni_host_partial_attn(const omni_host_attn_args* a)
{
    if (!a) return OMNI_ERR_NULL;
    if (a->n_rows < 0 || a->batch < 0 || a->isa_level < 0 || a->isa_level > 3) return OMNI_ERR_SHAPE;
    if (a->n_rows == 0) return OMNI_OK;
    if (!a->q || !a->k_pool || !a->v_pool || !a->block_table || !a->row_seq || !a->row_end || !a->part_o ||
        !a->part_lse)
        return OMNI_ERR_NULL;
    if (a->qkv_dtype != OMNI_F32 && a->qkv_dtype != OMNI_BF16) return OMNI_ERR_DTYPE;
    if (a->batch <= 0 || a->num_q_heads <= 0 || a->num_kv_heads <= 0 || a->max_blocks_per_seq <= 0 ||
        a->num_blocks <= 0 || a->num_q_heads % a->num_kv_heads != 0)
        return OMNI_ERR_SHAPE;
    if (a->block_size != kPage || (a->head_dim != 64 && a->head_dim != 128) ||
        a->num_q_heads / a->num_kv_heads > kMaxGroup)
        return OMNI_ERR_UNSUPPORTED;
    for (int r = 0; r < a->n_rows; ++r)
        if (a->row_seq[r] < 0 || a->row_seq[r] >= a->batch) return OMNI_ERR_SHAPE;

    HostParams p;
    p.n_rows = a->n_rows;
    p.batch = a->batch;
    p.hq = a->num_q_heads;
    p.hkv = a->num_kv_heads;
    p.group = p.hq / p.hkv;
    p.d = a->head_dim;
    p.max_blocks = a->max_blocks_per_seq;
    p.num_blocks = a->num_blocks;
    p.bf16 = a->qkv_dtype == OMNI_BF16;
    p.sm_scale = a->sm_scale;
    p.q = a->q;
    p.k_pool = a->k_pool;
    p.v_pool = a->v_pool;
    p.block_table = a->block_table;
    p.row_seq = a->row_seq;
    p.row_begin = a->row_begin;
    p.row_end = a->row_end;
    p.part_o = a->part_o;
    p.part_lse = a->part_lse;
    int n_threads = a->n_threads;
    if (n_threads <= 0) n_threads = (int)std::max(1u, std::thread::hardware_concurrency());
    const UnitFn unit_fn = pick_unit_fn(p.d, a->isa_level);
    if (!unit_fn) return OMNI_ERR_UNSUPPORTED;
    if (p.d == 128) produce<128>(p, n_threads, unit_fn);
    else produce<64>(p, n_threads, unit_fn);
    return OMNI_OK;
}

// Measurement aid: `n_threads` threads read `bytes` bytes of host memory once, each a contiguous slab, and
// fold them into *sink (so that the reads cannot be dropped): what the host's memory gives threads that only
// read - the streaming reference the producer above is set against.
extern "C" omni_status omni_debug_host_stream_read(const void* src, size_t bytes, int32_t n_threads, uint64_t* sink)
{
    if (!src || !sink) return OMNI_ERR_NULL;
    if (bytes % 8 != 0) return OMNI_ERR_SHAPE;
    int n = n_threads > 0 ? n_threads : (int)std::max(1u, std::thread::hardware_concurrency());
    const size_t words = bytes / 8;
    const size_t per = (words + (size_t)n - 1) / (size_t)n;
    std::vector<uint64_t> folds((size_t)n, 0);
    auto worker = [&](int t) {
        const uint64_t* w = static_cast<const uint64_t*>(src);
        const size_t lo = std::min(words, (size_t)t * per), hi = std::min(words, lo + per);
        uint64_t lanes[8] = {0, 0, 0, 0, 0, 0, 0, 0};              // eight running sums: vectorises as is
        size_t i = lo;
        for (; i + 8 <= hi; i += 8)
            for (int j = 0; j < 8; ++j) lanes[j] += w[i + j];
        for (; i < hi; ++i) lanes[0] += w[i];
        uint64_t f = 0;
        for (int j = 0; j < 8; ++j) f ^= lanes[j];
        folds[(size_t)t] = f;
    };
    std::vector<std::thread> pool;
    for (int t = 1; t < n; ++t) pool.emplace_back(worker, t);
    worker(0);
    for (auto& th : pool) th.join();
    uint64_t f = 0;
    for (uint64_t x : folds) f ^= x;
    *sink = f;
    return OMNI_OK;
}
