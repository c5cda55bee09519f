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

#include <algorithm>
#include <atomic>
#include <cmath>
#include <cstdint>
#include <cstring>
#include <limits>
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

// The compute of a unit is instantiated for three instruction-set levels (baseline x86-64, AVX2 + FMA,
// AVX-512) and the level is chosen once per call from what the CPU reports; the bodies below are plain
// loops over whole rows that the compiler vectorises for each level.
#define OMNI_HOST_INLINE static inline __attribute__((always_inline))

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
            float s[kPage];
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
            const float corr = (m[g] == -std::numeric_limits<float>::infinity()) ? 0.f : std::exp(m[g] - mx);
            float* a = acc + g * D;
            for (int i = 0; i < D; ++i) a[i] *= corr;
            float sum = l[g] * corr;
            for (int t = s0; t < s1; ++t) {
                const float w = std::exp(s[t] - mx);
                sum += w;
                for (int i = 0; i < D; ++i) a[i] += w * vf[t][i];
            }
            m[g] = mx;
            l[g] = sum;
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
OMNI_HOST_UNIT(unit_avx512_64, 64, __attribute__((target("avx512f,avx512vl,avx512bw,avx512dq,fma"))))
OMNI_HOST_UNIT(unit_avx512_128, 128, __attribute__((target("avx512f,avx512vl,avx512bw,avx512dq,fma"))))

UnitFn pick_unit_fn(int d)
{
    __builtin_cpu_init();
    if (__builtin_cpu_supports("avx512f") && __builtin_cpu_supports("avx512vl") &&
        __builtin_cpu_supports("avx512bw") && __builtin_cpu_supports("avx512dq"))
        return d == 128 ? unit_avx512_128 : unit_avx512_64;
    if (__builtin_cpu_supports("avx2") && __builtin_cpu_supports("fma"))
        return d == 128 ? unit_avx2_128 : unit_avx2_64;
    return d == 128 ? unit_base_128 : unit_base_64;
}

template <int D>
void produce(const HostParams& p, int n_threads)
{
    const UnitFn unit_fn = pick_unit_fn(D);
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
    std::vector<float> partial(units.size() * stride);

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
        float* res = partial.data() + i * stride;
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
                const float* res = partial.data() + u * stride;
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
    if (a->n_rows < 0 || a->batch < 0) return OMNI_ERR_SHAPE;
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
    if (p.d == 128) produce<128>(p, n_threads);
    else produce<64>(p, n_threads);
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
