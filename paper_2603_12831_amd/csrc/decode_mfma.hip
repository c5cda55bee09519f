// Matrix-core decode attention for bf16 KV: head_dim 128 with GQA ratio G <= 16, and head_dim 64 with
// G <= 4 as pairs of kv heads (further down).
//
// A work item is one (sequence, chunk, kv head): every KV byte of the chunk is
// read exactly once and serves all G query heads that share the kv head (Eq. 1
// of the paper's Background section for G queries at a time).  A workgroup of
// four waves handles an item; the chunk's pages are taken two at a time (a
// 32-token step) and the steps are dealt round-robin to the waves.  Per step a
// wave computes, with v_mfma_f32_16x16x32_bf16,
//
//   S^T[token, g]  = K[token, :] . Q[g, :]            (A = K tile, B = Q^T)
//   O^T[dim, g]   += V^T[dim, token] . P^T[token, g]  (A = V^T tile, B = P^T)
//
// Operand layouts of the 16x16x32 instruction: lane l supplies row/col l%16
// and eight consecutive k of group l/16; the result puts col l%16, rows
// 4*(l/16)+i in register i.
//
//   * K goes from memory straight into a per-wave LDS staging area (direct-to-LDS
//     16-byte loads, whole 256-byte rows per 16 lanes, XOR-swizzled image) and is
//     read from there in the A layout: lane l takes token row tau(l%16) at dims
//     kb*32 + (l/16)*8, tau(r) = 4*(r%4) + r/4, conflict-free.
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
//   * K and V loads both carry the non-temporal hint (measured: both plain is 8 % slower; K plain is
//     1-2 % slower on ragged batches and 1-3 % faster only on very long uniform contexts).
//
// The online softmax works in the log2 domain (logits pre-multiplied by
// sm_scale * log2 e), keeps one running maximum per query head (max over the
// lane's registers, then across the four lane groups) and rescales the
// accumulator only when some maximum of the wave moved.  The four waves'
// states are combined through LDS with the log-sum-exp rule.
//
// head_dim 64 rides on the same tiles ("half" instances): the 2 KiB tiles of two neighbouring kv heads of a
// page are one contiguous 4 KiB run, which read as sixteen 256-byte rows holds in row r the tokens 2 (r % 8)
// and 2 (r % 8) + 1 of kv head r / 8, side by side.  A query head of either kv head then becomes two columns
// of the Q^T operand, its 64 dims in the even-token or in the odd-token half of the 128 and zeros in the
// other, so that S^T[r, column] is the logit of one token of one head (entries whose row belongs to the
// other kv head are masked), the weights enter P^T exactly as before, and O^T comes out with the even
// tokens' sum in dims 0..63 of one column and the odd tokens' in dims 64..127 of its neighbour, added up at
// the end.  Four columns per query head pair up to G = 4; the streaming of K and V is untouched.
//
// Two launch forms share the per-step code:
//   * grid form: one workgroup per (sequence, chunk, kv head) slot of the
//     partial buffers, empty slots exit at once; needs no workspace.
//   * persistent form (caller gave a workspace): a one-workgroup pass lists the
//     non-empty (sequence, chunk) ranges longest-first and the empty ones apart;
//     one workgroup per CU then draws items from that list with atomic tickets,
//     and in its last step of an item already requests the first step of its next
//     item, so the memory pipe never drains between items and the longest items
//     cannot end up last.  A fifth wave combines the four streaming waves' states
//     and does all global stores, one item behind them.  Short ranges, when there
//     are many, are taken four at a time, one whole item per wave.
#include <mutex>

#include "omni_internal.hpp"

namespace omni {
namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

constexpr int kWaves = 4;
constexpr int kThreads = kWaves * kWave;
// persistent form: four streaming waves and a writer wave - two in the fused form, where a writer's work on a
// ticket of four short items (each item's rows folded with the rows from elsewhere: ~700 instructions an
// item) otherwise takes longer than the streaming waves take for the ticket
__host__ __device__ constexpr int persistent_writers(bool fused) { return fused ? 2 : 1; }
__host__ __device__ constexpr int persistent_threads(bool fused) { return kThreads + persistent_writers(fused) * kWave; }
constexpr int kD = 128;
constexpr int kPageBytes = kBlockSize * kD * 2;        // one (page, kv head) tile of K or of V
constexpr float kLog2e = 1.4426950408889634f;
constexpr float kLn2 = 0.6931471805599453f;
constexpr int kSortBins = 256;

struct StepRegs {            // raw V registers of one 32-token step (pages A and B); K waits in LDS
    u32x4 va[4], vb[4];
};

constexpr int kStageBytes = 2 * kPageBytes;            // per-wave LDS staging of a step's two K tiles

typedef __attribute__((address_space(3))) void lds_void;
typedef const __attribute__((address_space(1))) void global_void;

// wait until at most n vector-memory operations of this wave are outstanding (they retire in order)
#define OMNI_WAIT_VMCNT(n) __builtin_amdgcn_s_waitcnt((((n) >> 4) << 14) | 0x0F70 | ((n) & 0xF))

struct Item {                // wave-uniform description of a work item
    int seq, chunk, kvh, cb, ce, lp_first, lp_last, n_steps;
    // `chunk`: the chunk index in the low 16 bits, the number of non-empty chunks of the item's sequence (its
    // own included) in the high 16 (one word, to keep the streaming loop's scalar registers down)
    int s0, ds;              // this wave's steps of the item: s0, s0 + ds, ... (ds = 1: the item is this wave's alone)
    const int* __restrict__ table;
};

// Data no kernel of a launch writes (block table, work list) is read through the constant address space:
// a wave-uniform read then always becomes a scalar load, whatever else the kernel stores or updates.
__device__ __forceinline__ int load_invariant(const int* ptr)
{
    return *(const __attribute__((address_space(4))) int*)ptr;
}

__device__ __forceinline__ WorkEntry load_invariant(const WorkEntry* ptr)
{
    typedef int i32x4 __attribute__((ext_vector_type(4)));
    const i32x4 v = *(const __attribute__((address_space(4))) i32x4*)ptr;
    return WorkEntry{v[0], v[1], v[2], v[3]};
}


struct Pages { long long a, b; };                      // physical pages of a step, -1 = absent

__device__ __forceinline__ uint32_t pack_lo(uint32_t x, uint32_t y) { return __builtin_amdgcn_perm(y, x, 0x05040100u); }
__device__ __forceinline__ uint32_t pack_hi(uint32_t x, uint32_t y) { return __builtin_amdgcn_perm(y, x, 0x07060302u); }

__device__ __forceinline__ uint32_t pack_bf16(float a, float b)
{
    f32x2 p = {a, b};
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(p, bf16x2));
}

// A step's pages travel as 64-bit words: the physical page in the low 48 bits and, above bit 56, how many
// 128-byte units from the start of its tile the item needs (the item's last page may end early); a
// negative word is an absent page.  Loads of a page go through a buffer resource that ends with the last
// attended token, so the rows behind it (and all of an absent page) are neither fetched nor written: they
// read as zero, and the caller masks those tokens anyway.  A tile of 128-wide rows needs two units per
// token; a pair of 64-wide tiles (`half`) needs all of the first tile and one unit per token of the second.
constexpr int kPageTokenShift = 56;
template <bool half>
__device__ __forceinline__ long long page_word(long long page, int tokens)
{
    return page | ((long long)(half ? kBlockSize + tokens : 2 * tokens) << kPageTokenShift);
}
__device__ __forceinline__ long long page_of(long long word) { return word < 0 ? 0 : (word & ((1ll << 48) - 1)); }
__device__ __forceinline__ int page_bytes(long long word) { return word < 0 ? 0 : (int)(word >> kPageTokenShift) * kD; }

// One 4 KiB tile (V of one page and kv head) into four 16-byte registers per lane: lane l reads bytes
// lane_off .. +15 of each KiB (non-temporal).
__device__ __forceinline__ void load_tile(const void* __restrict__ pool, int hkv, long long word, int kvh,
                                          int lane_off, u32x4 (&r)[4])
{
    constexpr int kNonTemporal = 2;
    const char* src = static_cast<const char*>(pool) + (page_of(word) * hkv + kvh) * (long long)kPageBytes;
    const __amdgpu_buffer_rsrc_t rs = __builtin_amdgcn_make_buffer_rsrc(const_cast<char*>(src), 0, page_bytes(word), 0x00020000);
#pragma unroll
    for (int i = 0; i < 4; ++i) r[i] = __builtin_amdgcn_raw_buffer_load_b128(rs, lane_off + i * 1024, 0, kNonTemporal);
}

// physical pages of step s of an item (s wave-uniform); pages past the item's last page, or whose
// table entry does not name a pool page, come back as -1
template <bool half>
__device__ __forceinline__ Pages step_pages(const DecodeParams& p, const Item& it, int s)
{
    Pages r = {-1, -1};
    const int lp = __builtin_amdgcn_readfirstlane(it.lp_first + 2 * s);
    if (lp <= it.lp_last) {
        long long pg = load_invariant(it.table + lp);
        r.a = (pg >= 0 && pg < p.num_blocks) ? page_word<half>(pg, min(kBlockSize, it.ce - (lp << 4))) : -1;
    }
    if (lp + 1 <= it.lp_last) {
        long long pg = load_invariant(it.table + lp + 1);
        r.b = (pg >= 0 && pg < p.num_blocks) ? page_word<half>(pg, min(kBlockSize, it.ce - ((lp + 1) << 4))) : -1;
    }
    return r;
}

// Raw buffer descriptor over `bytes` bytes at `base` (offsets past the end read as zero).
__device__ __forceinline__ __amdgpu_buffer_rsrc_t byte_buffer(const void* base, int bytes)
{
    return __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(base), 0, bytes, 0x00020000);
}

constexpr int kAuxK = 2;                               // cache policy of the K loads: non-temporal, like V (load_tile)

// K tiles of a step go from HBM straight into the wave's LDS staging area (no registers while in
// flight).  A wave-wide 16-byte direct load puts lane s's data at base + 16 s, so for KiB i of a page
// lane s fetches token 4i + s/16, 16-byte chunk (s%16) ^ token: the global side stays whole 256-byte
// rows per 16 lanes, and the LDS image is XOR-swizzled so that the later operand reads (16 lanes =
// 16 different tokens, same chunk) touch every bank once.
// Buffer-addressed direct loads are used (not flat/global ones): the compiler then keeps exact counts of
// the vector-memory operations in flight instead of draining them all at the next register-load wait.
__device__ __forceinline__ void issue_k(const DecodeParams& p, int kvh, Pages pg, int lane, char* stage)
{
    const int row = lane >> 4, chunk = lane & 15;
    const int v0 = row * (kD * 2) + ((chunk ^ row) & 15) * 16;          // byte offset in KiB 0; KiB i: ^ (i << 6)
#pragma unroll
    for (int half = 0; half < 2; ++half) {
        const long long word = half ? pg.b : pg.a;
        const char* src = static_cast<const char*>(p.k_pool) + (page_of(word) * p.hkv + kvh) * (long long)kPageBytes;
        const __amdgpu_buffer_rsrc_t rs = byte_buffer(src, page_bytes(word));
        char* dst = stage + half * kPageBytes;
        // the instruction's immediate offset moves both the memory address and the LDS address
        __builtin_amdgcn_raw_ptr_buffer_load_lds(rs, (lds_void*)dst, 16, v0, 0, 0, kAuxK);
        __builtin_amdgcn_raw_ptr_buffer_load_lds(rs, (lds_void*)dst, 16, v0 ^ (1 << 6), 0, 1024, kAuxK);
        __builtin_amdgcn_raw_ptr_buffer_load_lds(rs, (lds_void*)dst, 16, v0 ^ (2 << 6), 0, 2048, kAuxK);
        __builtin_amdgcn_raw_ptr_buffer_load_lds(rs, (lds_void*)dst, 16, v0 ^ (3 << 6), 0, 3072, kAuxK);
    }
}

// operand kb of page `half` for the S^T product: lane (row r = l%16, k group kg) needs token tau(r),
// 16-byte chunk kb*4 + kg, found at the swizzled position written by issue_k
__device__ __forceinline__ u32x4 read_k(const char* stage, int half, int kb, int tau, int kg)
{
    const int chunk = kb * 4 + kg;
    return *reinterpret_cast<const u32x4*>(stage + half * kPageBytes + tau * (kD * 2) + ((chunk ^ tau) & 15) * 16);
}

__device__ __forceinline__ void issue_v(const DecodeParams& p, int kvh, Pages pg, int v_lane_off, StepRegs& r)
{
    load_tile(p.v_pool, p.hkv, pg.a, kvh, v_lane_off, r.va);            // token 4i + kg, dims col*8 ..
    load_tile(p.v_pool, p.hkv, pg.b, kvh, v_lane_off, r.vb);
}

// Request a whole step: the 8 K loads strictly before the 8 V loads (the in-order counting of
// attend_step relies on that order, so the scheduler must not swap them).
__device__ __forceinline__ void issue_step(const DecodeParams& p, int kvh, Pages pg, int lane, char* stage,
                                           int v_lane_off, StepRegs& r)
{
    __builtin_amdgcn_sched_barrier(0);
    issue_k(p, kvh, pg, lane, stage);
    __builtin_amdgcn_sched_barrier(0);
    issue_v(p, kvh, pg, v_lane_off, r);
    __builtin_amdgcn_sched_barrier(0);
}

// Q^T operands: lane supplies head `col`, dims kb*32 + kg*8 .. +7; heads beyond G are zero columns.
// `half`: column c stands for query row c / 2 of the kv-head pair (2 G rows of 64 dims) and token parity
// c % 2: its 64 dims sit in that parity's half of the 128, the other half is zero.
template <bool half>
__device__ __forceinline__ void load_q(const DecodeParams& p, const Item& it, int col, int kg, u32x4 (&qb)[4])
{
    const u32x4 z = {0, 0, 0, 0};
    const long long row0 = (long long)it.seq * p.hq + (long long)it.kvh * p.group;       // in 256-byte rows
    const char* q0 = static_cast<const char*>(p.q) + row0 * (kD * 2);
#pragma unroll
    for (int kb = 0; kb < 4; ++kb) {
        if (half) {
            const bool on = col < 4 * p.group && (kb >> 1) == (col & 1);
            qb[kb] = on ? *reinterpret_cast<const u32x4*>(q0 + (col >> 1) * kD + ((kb & 1) * 4 + kg) * 16) : z;
        } else {
            qb[kb] = (col < p.group) ? *reinterpret_cast<const u32x4*>(q0 + col * (kD * 2) + (kb * 4 + kg) * 16) : z;
        }
    }
}

__device__ __forceinline__ void finish_item(Item& it, const int* __restrict__ block_table, int max_blocks)
{
    it.table = block_table + (long long)it.seq * max_blocks;
    it.lp_first = it.cb >> 4;
    it.lp_last = (it.ce - 1) >> 4;
    it.n_steps = (it.lp_last - it.lp_first + 2) >> 1;
}

// Tell the compiler that every field of an item is the same in all lanes (it is: items are derived from
// wave-uniform tickets), where its own analysis gives up; otherwise the fields move to vector registers
// and the table reads become vector loads with full waits.
__device__ __forceinline__ int uniform(int v) { return __builtin_amdgcn_readfirstlane(v); }
__device__ __forceinline__ void make_uniform(Item& it)
{
    it.seq = uniform(it.seq); it.chunk = uniform(it.chunk); it.kvh = uniform(it.kvh);
    it.cb = uniform(it.cb); it.ce = uniform(it.ce);
    it.lp_first = uniform(it.lp_first); it.lp_last = uniform(it.lp_last); it.n_steps = uniform(it.n_steps);
    it.s0 = uniform(it.s0); it.ds = uniform(it.ds);
    const unsigned long long t = reinterpret_cast<unsigned long long>(it.table);
    const unsigned lo = (unsigned)uniform((int)(unsigned)t), hi = (unsigned)uniform((int)(unsigned)(t >> 32));
    it.table = reinterpret_cast<const int*>(((unsigned long long)hi << 32) | (unsigned long long)lo);
}

struct WaveState {
    f32x4 acc[8];            // acc[j][i] = O^T[dim (4*kg+i)*8 + j][head col]
    float m_run;             // running max (log2 domain) of head `col`
    float l_run;             // this lane's share of the running sum
    __device__ __forceinline__ void reset()
    {
#pragma unroll
        for (int j = 0; j < 8; ++j) acc[j] = f32x4{0.f, 0.f, 0.f, 0.f};
        m_run = -INFINITY;
        l_run = 0.f;
    }
};

struct LaneIds {
    int lane, wave, col, kg, tau, v_lane_off;
    char* stage;             // this wave's K staging area in LDS
    __device__ __forceinline__ LaneIds(char* stage_base)
    {
        lane = threadIdx.x & 63;
        wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
        col = lane & 15;                                   // head column of S^T / O^T, dim group of V
        kg = lane >> 4;                                    // k group
        tau = 4 * (col & 3) + (col >> 2);                  // token whose K row this lane feeds to the MFMA
        v_lane_off = lane * 16;
        stage = stage_base + wave * kStageBytes;
    }
};

// One 32-token step: K from the wave's LDS staging area, V from the registers in `r`.  When `more`
// (compile-time) says the wave has a further step (pages `next` of kv head `next_kvh`: the same item's, or the first
// step of the workgroup's next item), its K tiles are requested into the staging area as soon as this
// step's K operands have been read out, and its V tiles into `r` after the PV products.
//
// Vector-memory operations retire in order, and every request for a step is "8 K loads, then 8 V
// loads": once at most 8 operations are outstanding the K tiles have landed, whatever was issued
// after them.
// `before_v` runs right before the V request that ends the step: requests made there are older than that V
// and younger than everything this step still waits for, so they delay nothing in it.
template <bool more, bool half, class BeforeV>
__device__ __forceinline__ void attend_step(const DecodeParams& p, const Item& it, WaveState& st, StepRegs& r,
                                            const u32x4 (&qb)[4], const LaneIds& id, int s, bool ok_a, bool ok_b,
                                            Pages next, int next_kvh, float scale2, BeforeV&& before_v)
{
    const int kg = id.kg;
    // ---- S^T = K . Q^T for both pages ----------------------------------------------------------
    OMNI_WAIT_VMCNT(8);
    __builtin_amdgcn_sched_barrier(0);
    u32x4 ka[4], kb_[4];
#pragma unroll
    for (int kb = 0; kb < 4; ++kb) {
        ka[kb] = read_k(id.stage, 0, kb, id.tau, kg);
        kb_[kb] = read_k(id.stage, 1, kb, id.tau, kg);
    }
    f32x4 sa = {0.f, 0.f, 0.f, 0.f}, sb = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int kb = 0; kb < 4; ++kb) {
        sa = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, ka[kb]),
                                                     __builtin_bit_cast(bf16x8, qb[kb]), sa, 0, 0, 0);
        sb = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, kb_[kb]),
                                                     __builtin_bit_cast(bf16x8, qb[kb]), sb, 0, 0, 0);
    }
    __builtin_amdgcn_sched_barrier(0);
    if (more) issue_k(p, next_kvh, next, id.lane, id.stage);
    __builtin_amdgcn_sched_barrier(0);

    // ---- logits to the log2 domain, masking on boundary steps -----------------------------------
    const int t0 = (it.lp_first + 2 * s) << 4;             // first token of page A; register i is tile row 4i + kg
    const bool interior = ok_a && ok_b && t0 >= it.cb && t0 + 32 <= it.ce;
    uint32_t vmask[4] = {0xffffffffu, 0xffffffffu, 0xffffffffu, 0xffffffffu};
#pragma unroll
    for (int i = 0; i < 4; ++i) { sa[i] *= scale2; sb[i] *= scale2; }
    if (!half) {
        if (!interior) {
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const int ta = t0 + 4 * i + kg, tb = ta + 16;  // (tile row = token of the page)
                const bool va = ok_a && ta >= it.cb && ta < it.ce;
                const bool vb = ok_b && tb >= it.cb && tb < it.ce;
                sa[i] = va ? sa[i] : -INFINITY;
                sb[i] = vb ? sb[i] : -INFINITY;
                // a masked token's V must not reach the MFMA (0 * NaN): V^T k-slot i (page A) or 4+i (page B);
                // slots 2w, 2w+1 are the two halves of operand word w
                const uint32_t keep = (i & 1) ? 0x0000ffffu : 0xffff0000u;
                if (!va) vmask[i >> 1] &= keep;
                if (!vb) vmask[2 + (i >> 1)] &= keep;
            }
        }
    } else {
        // tile row 4i + kg holds, of kv head i / 2 of the pair, the tokens 2 (4 (i % 2) + kg) + parity; a
        // logit is real where the row's kv head is the column's and the column's token parity is attended
        const int par = id.col & 1, kvsel = id.col >= 2 * p.group ? 1 : 0, par_v = id.col >> 3;
        const bool col_on = id.col < 4 * p.group;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int ta = t0 + 2 * (4 * (i & 1) + kg) + par, tb = ta + 16;
            const bool mine = col_on && (i >> 1) == kvsel;
            sa[i] = (mine && ok_a && ta >= it.cb && ta < it.ce) ? sa[i] : -INFINITY;
            sb[i] = (mine && ok_b && tb >= it.cb && tb < it.ce) ? sb[i] : -INFINITY;
            if (!interior) {
                // this lane's V^T rows are dims of the even-token (lanes 0..7 of 16) or odd-token half
                const int tva = t0 + 2 * (4 * (i & 1) + kg) + par_v, tvb = tva + 16;
                const uint32_t keep = (i & 1) ? 0x0000ffffu : 0xffff0000u;
                if (!(ok_a && tva >= it.cb && tva < it.ce)) vmask[i >> 1] &= keep;
                if (!(ok_b && tvb >= it.cb && tvb < it.ce)) vmask[2 + (i >> 1)] &= keep;
            }
        }
    }
    // ---- online softmax ----------------------------------------------------------------------------
    float mx = fmaxf(fmaxf(fmaxf(sa[0], sa[1]), fmaxf(sa[2], sa[3])), fmaxf(fmaxf(sb[0], sb[1]), fmaxf(sb[2], sb[3])));
    mx = fmaxf(mx, __shfl_xor(mx, 16));
    mx = fmaxf(mx, __shfl_xor(mx, 32));
    if (half) mx = fmaxf(mx, __shfl_xor(mx, 1));           // the two token parities of a head share its maximum
    const float m_new = fmaxf(st.m_run, mx);
    const float m_use = (m_new == -INFINITY) ? 0.f : m_new;          // nothing seen yet: avoid inf - inf
    if (__any(m_new > st.m_run)) {
        const float corr = __builtin_amdgcn_exp2f(st.m_run - m_use);   // 0 when m_run = -inf
        st.l_run *= corr;
#pragma unroll
        for (int j = 0; j < 8; ++j) st.acc[j] *= corr;
    }
    st.m_run = m_new;
    float pw[8];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        pw[i] = __builtin_amdgcn_exp2f(sa[i] - m_use);
        pw[4 + i] = __builtin_amdgcn_exp2f(sb[i] - m_use);
    }
    st.l_run += ((pw[0] + pw[1]) + (pw[2] + pw[3])) + ((pw[4] + pw[5]) + (pw[6] + pw[7]));
    // P^T operand: bf16 head and bf16 remainder of every weight
    u32x4 ph, pl;
#pragma unroll
    for (int w = 0; w < 4; ++w) {
        const uint32_t h = pack_bf16(pw[2 * w], pw[2 * w + 1]);
        ph[w] = h;
        pl[w] = pack_bf16(pw[2 * w] - bf16lo_to_f32(h), pw[2 * w + 1] - bf16hi_to_f32(h));
    }
    // ---- O^T += V^T . P^T: word j/2, half j%2 of load i holds dim (l%16)*8 + j of token 4i + kg ----
#pragma unroll
    for (int jj = 0; jj < 4; ++jj) {
        u32x4 lo = {pack_lo(r.va[0][jj], r.va[1][jj]), pack_lo(r.va[2][jj], r.va[3][jj]),
                    pack_lo(r.vb[0][jj], r.vb[1][jj]), pack_lo(r.vb[2][jj], r.vb[3][jj])};
        u32x4 hi = {pack_hi(r.va[0][jj], r.va[1][jj]), pack_hi(r.va[2][jj], r.va[3][jj]),
                    pack_hi(r.vb[0][jj], r.vb[1][jj]), pack_hi(r.vb[2][jj], r.vb[3][jj])};
        if (!interior) {
#pragma unroll
            for (int w = 0; w < 4; ++w) { lo[w] &= vmask[w]; hi[w] &= vmask[w]; }
        }
        f32x4 a0 = st.acc[2 * jj], a1 = st.acc[2 * jj + 1];
        a0 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, lo), __builtin_bit_cast(bf16x8, ph), a0, 0, 0, 0);
        a1 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, hi), __builtin_bit_cast(bf16x8, ph), a1, 0, 0, 0);
        a0 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, lo), __builtin_bit_cast(bf16x8, pl), a0, 0, 0, 0);
        a1 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, hi), __builtin_bit_cast(bf16x8, pl), a1, 0, 0, 0);
        st.acc[2 * jj] = a0;
        st.acc[2 * jj + 1] = a1;
    }
    __builtin_amdgcn_sched_barrier(0);
    before_v();
    if (more) issue_v(p, next_kvh, next, id.v_lane_off, r);
    __builtin_amdgcn_sched_barrier(0);
}

// What a wave streams after its last step of the current item: the first step of the workgroup's next
// item (persistent form), or nothing.
struct Tail {
    bool valid;
    int kvh;
    Pages pages;
};

// All steps of an item that belong to this wave.  On entry the loads of the wave's first step are
// already requested (if it has one).  `at_penult(true)` runs right before and `at_penult(false)` right
// after the wave's second-to-last step (if it has two or more).  The wave's last step is peeled off:
// `before_last` runs right before it and returns what the wave requests during it instead of a further
// step of this item, `after_last` runs right after it.
template <bool chained, bool half, class Penult, class Before, class Mid, class After>
__device__ __forceinline__ void run_item(const DecodeParams& p, const Item& it, WaveState& st, StepRegs& r,
                                         const u32x4 (&qb)[4], const LaneIds& id, float scale2, Pages cur, Pages nxt,
                                         Penult&& at_penult, Before&& before_last, Mid&& in_last, After&& after_last)
{
    int s = it.s0;
    // everything older than the first step's 8 K + 8 V requests has landed
    OMNI_WAIT_VMCNT(16);
    while (s + it.ds < it.n_steps) {
        const bool penult = s + 2 * it.ds >= it.n_steps;
        Pages nn = {-1, -1};
        if (!penult) nn = step_pages<half>(p, it, s + 2 * it.ds);                        // table reads run a step ahead
        else at_penult(true);
        attend_step<true, half>(p, it, st, r, qb, id, s, cur.a >= 0, cur.b >= 0, nxt, it.kvh, scale2, [] {});
        if (penult) at_penult(false);
        cur = nxt;
        nxt = nn;
        s += it.ds;
    }
    if (s < it.n_steps) {
        const Tail tail = before_last();
        // `chained`: the step always ends with a request (the next item's first step, or, when there is
        // none, the same loads on two absent pages, which fetch nothing), so that one copy of the step code with exact load
        // counts serves; a second copy for "nothing follows" cost registers to the point of spilling
        if (chained) attend_step<true, half>(p, it, st, r, qb, id, s, cur.a >= 0, cur.b >= 0,
                                       tail.valid ? tail.pages : Pages{-1, -1}, tail.valid ? tail.kvh : 0, scale2, in_last);
        else attend_step<false, half>(p, it, st, r, qb, id, s, cur.a >= 0, cur.b >= 0, tail.pages, tail.kvh, scale2, in_last);
        after_last();
    }
}

// Workgroup barrier that orders LDS traffic only: vector-memory loads already in flight (the prefetch of
// the next step or item) stay in flight across it.
__device__ __forceinline__ void lds_barrier()
{
    // LDS writes of this wave done (lgkmcnt), then the barrier; the memory clobber keeps the compiler from
    // moving LDS accesses across.  A fence would also wait for the direct-to-LDS loads in flight, which
    // only ever target the issuing wave's own staging area.
    asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
}

// A word in LDS that one thread posts and waves of the same workgroup poll between barriers.  Written
// as instructions of their own: an LDS access the compiler knows of makes it wait first for every
// direct-to-LDS load in flight (it cannot tell the staging areas from this word), which would drain the
// wave's memory pipe at each poll.
__device__ __forceinline__ unsigned lds_peek(const unsigned* word)
{
    const unsigned addr = (unsigned)(uintptr_t)(const __attribute__((address_space(3))) unsigned*)word;
    unsigned v;
    asm volatile("ds_read_b32 %0, %1\n\ts_waitcnt lgkmcnt(0)" : "=v"(v) : "v"(addr));
    return v;
}
__device__ __forceinline__ void lds_post(unsigned* word, unsigned value)
{
    const unsigned addr = (unsigned)(uintptr_t)(__attribute__((address_space(3))) unsigned*)word;
    asm volatile("ds_write_b32 %0, %1" : : "v"(addr), "v"(value) : "memory");
}

// Q rows of an item's G heads into an LDS buffer ([g][256 bytes]) by one wave's direct-to-LDS loads:
// lane l moves 16 bytes of row 4i + l/16 in round i; lanes of rows >= G stay idle.
__device__ __forceinline__ void issue_q(const DecodeParams& p, const Item& it, int lane, char* qbuf)
{
    const long long row0 = (long long)it.seq * p.hq + (long long)it.kvh * p.group;
    const __amdgpu_buffer_rsrc_t rs = byte_buffer(static_cast<const char*>(p.q) + row0 * (kD * 2), p.group * kD * 2);
    for (int i = 0; 4 * i < p.group; ++i) {
        if (4 * i + (lane >> 4) < p.group)
            __builtin_amdgcn_raw_ptr_buffer_load_lds(rs, (lds_void*)(qbuf + i * 1024), 16, lane * 16, i * 1024, 0, 0);
    }
}

// Q^T operands from the LDS copy: lane supplies head `col`, dims kb*32 + kg*8 .. +7; heads beyond G are
// zero columns (`half`: as in load_q)
template <bool half>
__device__ __forceinline__ void read_q(const char* qbuf, int group, int col, int kg, u32x4 (&qb)[4])
{
    const u32x4 z = {0, 0, 0, 0};
#pragma unroll
    for (int kb = 0; kb < 4; ++kb) {
        if (half) {
            const bool on = col < 4 * group && (kb >> 1) == (col & 1);
            qb[kb] = on ? *reinterpret_cast<const u32x4*>(qbuf + (col >> 1) * kD + ((kb & 1) * 4 + kg) * 16) : z;
        } else {
            qb[kb] = (col < group) ? *reinterpret_cast<const u32x4*>(qbuf + col * (kD * 2) + (kb * 4 + kg) * 16) : z;
        }
    }
}

// Dynamic LDS of a workgroup: the cross-wave combine area ([kWaves][G][kD] accumulators, then
// [kWaves][16] m and l), the waves' K staging areas and, in the persistent form (which has two combine
// areas), two sets of per-wave Q buffers.
__host__ __device__ __forceinline__ size_t combine_bytes(int group)
{
    return (size_t)(kWaves * group * kD + 2 * kWaves * 16) * sizeof(float);
}

// Position of dim d (a multiple of 4) of head row g inside that row of the combine area.  A lane holds,
// for each i, eight consecutive dims 32 kg + 8 i .. + 7 of head `col`; rows are 128 floats apart, so
// without a swizzle the 16 lanes of a 16-byte store (4 heads x 4 k groups, more heads for larger G) would
// all start in the same bank.  XOR-ing bits 3-4 with the head and bit 2 with the upper k-group bit
// spreads them over all banks and keeps groups of four dims together for the 16-byte reads of the combine.
__device__ __forceinline__ int combine_slot(int g, int d) { return d ^ ((g & 3) << 3) ^ ((d >> 6 & 1) << 2); }

__device__ __forceinline__ void stage_wave_state(const WaveState& st, float* lds, int G, int wave, int col, int kg)
{
    float l = st.l_run;
    l += __shfl_xor(l, 16);
    l += __shfl_xor(l, 32);
    float* sh_acc = lds;
    float* sh_m = lds + kWaves * G * kD;
    float* sh_l = sh_m + kWaves * 16;
    if (col < G) {
        float* dst = sh_acc + (wave * G + col) * kD;
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
            for (int h = 0; h < 2; ++h) {
                const f32x4 v = {st.acc[4 * h][i], st.acc[4 * h + 1][i], st.acc[4 * h + 2][i], st.acc[4 * h + 3][i]};
                *reinterpret_cast<f32x4*>(dst + combine_slot(col, (4 * kg + i) * 8 + 4 * h)) = v;
            }
        if (kg == 0) { sh_m[wave * 16 + col] = st.m_run; sh_l[wave * 16 + col] = l; }
    }
}

// four dims of a final row (row = sequence * Hq + head, of `dout` dims)
__device__ __forceinline__ void store_final_quad(void* out_o, float* out_lse, bool out_bf16, long long row, int d,
                                                 f32x4 o, float lse, int dout = kD)
{
    if (out_bf16) {
        uint2 pk;
        pk.x = (uint32_t)f32_to_bf16(o[0]) | ((uint32_t)f32_to_bf16(o[1]) << 16);
        pk.y = (uint32_t)f32_to_bf16(o[2]) | ((uint32_t)f32_to_bf16(o[3]) << 16);
        *reinterpret_cast<uint2*>(static_cast<uint16_t*>(out_o) + row * dout + d) = pk;
    } else {
        *reinterpret_cast<f32x4*>(static_cast<float*>(out_o) + row * dout + d) = o;
    }
    if (out_lse && d == 0) out_lse[row] = lse;
}

// What becomes of an item's rows: a partial row for a later merge; the sequence's final row (the item is
// the sequence's only non-empty chunk); the final row after folding in the rows other sources hold for
// the sequence; a partial row that another workgroup of this launch will read (the fused form: whoever
// finishes a sequence's last chunk merges them all).
enum RowMode { kRowPartial = 0, kRowFinal = 1, kRowFinalFold = 2, kRowShared = 3 };

__device__ __forceinline__ int row_mode(const DecodeParams& p, int n_live)
{
    if (p.out_o == nullptr) return kRowPartial;
    if (n_live > 1) return p.fuse ? kRowShared : kRowPartial;
    return (p.fuse && p.n_ext > 0) ? kRowFinalFold : kRowFinal;
}

// Partial rows that cross from one workgroup to another inside a launch are stored and loaded at device
// scope (each XCD has an L2 of its own; a device-scope store is written through it, a device-scope load
// does not take a line another XCD may have changed from it), so no cache-wide write-back or invalidate is
// needed: those cost a third of the read rate when issued per item.  `base` + `bytes` bound the buffer
// resource, `off` is the lane's byte offset in it.
__device__ __forceinline__ void store_shared4(float* base, int bytes, int off, f32x4 v)
{
    constexpr int kDeviceScopeNt = (1 << 4) | (1 << 1);
    __builtin_amdgcn_raw_buffer_store_b128(__builtin_bit_cast(u32x4, v), byte_buffer(base, bytes), off, 0, kDeviceScopeNt);
}

// after a barrier: the states of waves w0 .. w1-1 merged with the log-sum-exp rule into four dims of one
// head of the item's row, at position idx of the G x 32 (G = columns of the combine area).  `half`: position
// idx of the (G / 2) x 16 - row idx / 16 of the kv-head pair, whose even-token sums are dims 0..63 of column
// 2 row and whose odd-token sums are dims 64..127 of column 2 row + 1 (the two share their maximum).
template <bool half = false>
__device__ __forceinline__ void combine_quad(const float* lds, int G, int idx, int w0, int w1, f32x4& o, float& lse)
{
    const float* sh_acc = lds;
    const float* sh_m = lds + kWaves * G * kD;
    const float* sh_l = sh_m + kWaves * 16;
    const int g = half ? 2 * (idx >> 4) : idx >> 5, d = half ? (idx & 15) * 4 : (idx & 31) * 4;
    float mm = -INFINITY;
    for (int w = w0; w < w1; ++w) mm = fmaxf(mm, sh_m[w * 16 + g]);
    o = f32x4{0.f, 0.f, 0.f, 0.f};
    lse = -INFINITY;
    if (mm != -INFINITY) {
        float ll = 0.f;
        f32x4 oo = {0.f, 0.f, 0.f, 0.f};
        for (int w = w0; w < w1; ++w) {
            const float mw = sh_m[w * 16 + g];
            const float f = (mw == -INFINITY) ? 0.f : __builtin_amdgcn_exp2f(mw - mm);
            ll += f * sh_l[w * 16 + g];
            oo += f * *reinterpret_cast<const f32x4*>(sh_acc + (w * G + g) * kD + combine_slot(g, d));
            if (half) {
                ll += f * sh_l[w * 16 + g + 1];
                oo += f * *reinterpret_cast<const f32x4*>(sh_acc + (w * G + g + 1) * kD + combine_slot(g + 1, 64 + d));
            }
        }
#pragma unroll
        for (int i = 0; i < 4; ++i) o[i] = oo[i] / ll;
        lse = (mm + __builtin_amdgcn_logf(ll)) * kLn2;           // v_log_f32 is log2
    }
}

// ---- the merges inside the launch (fused form) ----------------------------------------------------------
// One routine turns everything that is known about G heads of a sequence into their final rows: the item's own state still in LDS (if any), the
// partial rows of the sequence's chunks written by this and other workgroups (if any), and the rows other
// sources hold for the sequence.  Rule: the disjoint-union identity of Eq. 1 in incremental form,
// acc = sum w_r O_r and wsum = sum w_r with w_r = exp(LSE_r - m), in a fixed order of rows, so the result
// does not depend on which workgroup runs it.
struct MergeJob {
    void* out_o;                   // final rows
    float* out_lse;                // may be null
    const float* part_o;           // chunk rows of the call (n_chunks > 0)
    const float* part_lse;
    const float* ext_o[3];         // rows computed elsewhere: rows r0 .. r1-1 of each source
    const float* ext_lse[3];
    int r0[3], r1[3];
    const float* own_lds;          // combine area holding the item's own state (null: none)
    int w0, w1;                    //   waves whose states make it up
    int hq, max_chunks, out_bf16, n_ext;
    int seq, head0, heads, group;  // rows [head0, head0 + heads) of the sequence; `group` = G of the launch
    int n_chunks;                  // chunks 0 .. n_chunks-1 of (seq, kv head head0 / G) hold partial rows
};

struct RowAcc {
    float m, wsum;
    f32x4 acc;
};

constexpr int kMergeLanes = 2;     // (head, four dims) positions a lane merges side by side
constexpr int kMergeTile = 8;      // rows per round trip

// Adds rows 0 .. n-1 (n <= kMergeTile) of one source to the kMergeLanes running merges of a lane: row r of
// position k has its LSE at lse[k] + r * lse_stride and its four dims at byte offset off[k] + r * o_stride
// of the buffer resource `rows`.  All LSE values and all O pieces of the tile are requested before anything
// is used: one memory round trip per tile, whatever the weights turn out to be (these merges are chains of
// such trips, and their number is what they cost).  Loads are device-scope ones, which is what the chunk
// rows need and does no harm to the others.  A row of weight zero (LSE = -inf) is fetched like the others
// but never enters the sums, so whatever its O holds (it may never have been written) does no harm.
__device__ __forceinline__ void merge_tile(RowAcc (&a)[kMergeLanes], const bool (&on)[kMergeLanes], int n,
                                           const float* const (&lse)[kMergeLanes], long long lse_stride,
                                           __amdgpu_buffer_rsrc_t rows, const int (&off)[kMergeLanes], int o_stride)
{
    constexpr int kDeviceScope = 1 << 4;
    float l[kMergeLanes][kMergeTile];
    f32x4 x[kMergeLanes][kMergeTile];
#pragma unroll
    for (int k = 0; k < kMergeLanes; ++k)
#pragma unroll
        for (int u = 0; u < kMergeTile; ++u)
            l[k][u] = (on[k] && u < n) ? __hip_atomic_load(lse[k] + u * lse_stride, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT)
                                       : -INFINITY;
#pragma unroll
    for (int k = 0; k < kMergeLanes; ++k)
#pragma unroll
        for (int u = 0; u < kMergeTile; ++u) {
            x[k][u] = f32x4{0.f, 0.f, 0.f, 0.f};
            if (on[k] && u < n)
                x[k][u] = __builtin_bit_cast(f32x4, __builtin_amdgcn_raw_buffer_load_b128(rows, off[k] + u * o_stride, 0, kDeviceScope));
        }
#pragma unroll
    for (int k = 0; k < kMergeLanes; ++k) {
        float m_new = a[k].m;
#pragma unroll
        for (int u = 0; u < kMergeTile; ++u) m_new = fmaxf(m_new, l[k][u]);
        // (nothing live so far: m_new = -inf, every weight below is zero and the state stays as it is)
        const float keep = a[k].m == -INFINITY ? 0.f : __builtin_amdgcn_exp2f((a[k].m - m_new) * kLog2e);
        a[k].acc *= keep;
        a[k].wsum *= keep;
        a[k].m = m_new;
#pragma unroll
        for (int u = 0; u < kMergeTile; ++u) {
            const bool live = l[k][u] != -INFINITY;
            const float w = live ? __builtin_amdgcn_exp2f((l[k][u] - m_new) * kLog2e) : 0.f;
            a[k].wsum += w;
#pragma unroll
            for (int c = 0; c < 4; ++c) a[k].acc[c] += live ? w * x[k][u][c] : 0.f;
        }
    }
}

// a pointer that is the same in all lanes, said so to the compiler (arguments of an out-of-line function
// arrive in vector registers)
__device__ __forceinline__ const float* uniform_ptr(const float* ptr)
{
    const unsigned long long t = reinterpret_cast<unsigned long long>(ptr);
    const unsigned lo = (unsigned)uniform((int)(unsigned)t), hi = (unsigned)uniform((int)(unsigned)(t >> 32));
    return reinterpret_cast<const float*>(((unsigned long long)hi << 32) | (unsigned long long)lo);
}

// rows of one sequence in a source are addressed through a buffer resource with 32-bit offsets: at most
// this many bytes of them are merged (2 GiB: more rows than any batch holds)
constexpr long long kMergeSpanBytes = 0x7fffffffLL;

// (jobs sit in LDS and the persistent kernel has exactly one call of this routine, in a loop over the jobs
// of a ticket: inlined several times, its unrolled tiles tripled the kernel's size and pushed scalar
// registers of the streaming loop into spills; as a real call it would need scratch memory)
__device__ __forceinline__ void merge_and_store_final(const MergeJob* job, int lane)
{
    const MergeJob& j = *job;
    void* const out_o = const_cast<float*>(uniform_ptr(static_cast<const float*>(j.out_o)));
    float* const out_lse_ptr = const_cast<float*>(uniform_ptr(j.out_lse));
    const bool out_bf16 = uniform(j.out_bf16) != 0;
    const int hq = uniform(j.hq), seq = uniform(j.seq), head0 = uniform(j.head0), heads = uniform(j.heads);
    const int n_chunks = uniform(j.n_chunks), n_ext = uniform(j.n_ext), max_chunks = uniform(j.max_chunks);
    const long long orow0 = (long long)seq * hq + head0;
    const long long prow0 = (long long)seq * max_chunks * hq + head0;
    const int row_bytes = hq * kD * 4;                                   // between consecutive rows of a source
    for (int base = lane; base < heads * (kD / 4); base += kWave * kMergeLanes) {
        RowAcc a[kMergeLanes];
        bool on[kMergeLanes];
        int g[kMergeLanes], d[kMergeLanes], off[kMergeLanes];
        const float* lse[kMergeLanes];
#pragma unroll
        for (int k = 0; k < kMergeLanes; ++k) {
            const int idx = base + k * kWave;
            on[k] = idx < heads * (kD / 4);
            g[k] = on[k] ? idx >> 5 : 0;
            d[k] = (idx & 31) * 4;
            off[k] = (g[k] * kD + d[k]) * 4;
            f32x4 own = {0.f, 0.f, 0.f, 0.f};
            float own_lse = -INFINITY;
            if (j.own_lds && on[k]) combine_quad(j.own_lds, uniform(j.group), idx, uniform(j.w0), uniform(j.w1), own, own_lse);
            a[k].m = own_lse;
            a[k].wsum = own_lse == -INFINITY ? 0.f : 1.f;
            a[k].acc = own;
        }
        // the sequence's chunk rows, in chunk order
        if (n_chunks > 0) {
            const float* rows = uniform_ptr(j.part_o) + prow0 * kD;
            const long long span = (long long)n_chunks * row_bytes;
            const __amdgpu_buffer_rsrc_t rs = byte_buffer(rows, (int)(span < kMergeSpanBytes ? span : kMergeSpanBytes));
            for (int c = 0; c < n_chunks; c += kMergeTile) {
                int at[kMergeLanes];
#pragma unroll
                for (int k = 0; k < kMergeLanes; ++k) {
                    lse[k] = j.part_lse + prow0 + g[k] + (long long)c * hq;
                    at[k] = off[k] + c * row_bytes;
                }
                merge_tile(a, on, min(kMergeTile, n_chunks - c), lse, hq, rs, at, row_bytes);
            }
        }
        // the rows computed elsewhere, source by source
        for (int s = 0; s < n_ext; ++s) {
            const int r0 = uniform(j.r0[s]), r1 = uniform(j.r1[s]);
            if (r1 <= r0) continue;
            const float* rows = uniform_ptr(j.ext_o[s]) + ((long long)r0 * hq + head0) * kD;
            const long long span = (long long)(r1 - r0) * row_bytes;
            const __amdgpu_buffer_rsrc_t rs = byte_buffer(rows, (int)(span < kMergeSpanBytes ? span : kMergeSpanBytes));
            for (int r = r0; r < r1; r += kMergeTile) {
                int at[kMergeLanes];
#pragma unroll
                for (int k = 0; k < kMergeLanes; ++k) {
                    lse[k] = j.ext_lse[s] + (long long)r * hq + head0 + g[k];
                    at[k] = off[k] + (r - r0) * row_bytes;
                }
                merge_tile(a, on, min(kMergeTile, r1 - r), lse, hq, rs, at, row_bytes);
            }
        }
#pragma unroll
        for (int k = 0; k < kMergeLanes; ++k) {
            f32x4 out = {0.f, 0.f, 0.f, 0.f};
            float out_lse = -INFINITY;
            if (a[k].m != -INFINITY) {
                out = a[k].acc * (1.f / a[k].wsum);
                out_lse = a[k].m + __builtin_amdgcn_logf(a[k].wsum) * kLn2;
            }
            if (on[k]) store_final_quad(out_o, out_lse_ptr, out_bf16, orow0 + g[k], d[k], out, out_lse);
        }
    }
}

// Final rows of a sequence that has no resident token at all: whatever the other sources hold for it, one
// row at a time (rare, and kept small: this sits in the writer wave's prologue).
__device__ __forceinline__ void fold_rows_plain(const DecodeParams& p, int seq, int lane)
{
    for (int idx = lane; idx < p.hq * (kD / 4); idx += kWave) {
        const int head = idx >> 5, d = (idx & 31) * 4;
        float m = -INFINITY, wsum = 0.f;
        f32x4 acc = {0.f, 0.f, 0.f, 0.f};
        for (int s = 0; s < p.n_ext; ++s) {
            int r0, r1;
            src_rows(p.ext[s], seq, r0, r1);
            for (int r = r0; r < r1; ++r) {
                const float l = p.ext[s].lse[(long long)r * p.hq + head];
                if (l == -INFINITY) continue;
                const f32x4 x = *reinterpret_cast<const f32x4*>(p.ext[s].o + ((long long)r * p.hq + head) * kD + d);
                const float m_new = fmaxf(m, l);
                const float keep = m == -INFINITY ? 0.f : __builtin_amdgcn_exp2f((m - m_new) * kLog2e);
                const float w = __builtin_amdgcn_exp2f((l - m_new) * kLog2e);
                acc = acc * keep + w * x;
                wsum = wsum * keep + w;
                m = m_new;
            }
        }
        f32x4 o = {0.f, 0.f, 0.f, 0.f};
        float lse = -INFINITY;
        if (m != -INFINITY) {
            o = acc * (1.f / wsum);
            lse = m + __builtin_amdgcn_logf(wsum) * kLn2;
        }
        store_final_quad(p.out_o, p.out_lse, p.out_bf16 != 0, (long long)seq * p.hq + head, d, o, lse);
    }
}

// a job for rows [head0, head0 + heads) of `seq`: outputs and the rows other sources hold for the sequence;
// written by one wave into its slot in LDS (every lane stores the same values)
__device__ __forceinline__ void merge_job(MergeJob& j, const DecodeParams& p, int seq, int head0, int heads)
{
    j.out_o = p.out_o; j.out_lse = p.out_lse; j.part_o = p.part_o; j.part_lse = p.part_lse;
    j.hq = p.hq; j.max_chunks = p.max_chunks; j.out_bf16 = p.out_bf16; j.n_ext = p.n_ext;
    j.seq = seq; j.head0 = head0; j.heads = heads; j.group = p.group;
    j.own_lds = nullptr; j.w0 = 0; j.w1 = 0; j.n_chunks = 0;
#pragma unroll
    for (int s = 0; s < 3; ++s) {
        j.ext_o[s] = p.ext[s].o;
        j.ext_lse[s] = p.ext[s].lse;
        j.r0[s] = j.r1[s] = 0;
        if (s < p.n_ext) {
            src_rows(p.ext[s], seq, j.r0[s], j.r1[s]);
            const long long most = kMergeSpanBytes / ((long long)p.hq * kD * 4);      // rows a resource can span
            if ((long long)j.r1[s] - j.r0[s] > most) j.r1[s] = j.r0[s] + (int)most;
        }
    }
}

// Rows computed elsewhere for an item that finishes its sequence, brought into LDS while the item streams:
// up to kExtLdsRows rows of the item's G heads (G <= kExtLdsGroup) from the call's single external source.
// A slot holds [row][G][128] floats of O and behind them [row][G] LSE values.  The loads are direct-to-LDS
// ones issued by the wave that also requests the item's Q rows, right after those: they need no registers,
// are older than the item's first K / V requests and have landed with Q.  Always kExtLdsRows row requests:
// rows beyond `n` lie outside the buffer resource and fetch nothing (fixed instruction count).
constexpr int kExtLdsRows = 4, kExtLdsGroup = 4;
__host__ __device__ __forceinline__ size_t ext_slot_bytes(int group)
{
    return (size_t)kExtLdsRows * group * kD * 4 + 64;
}
__device__ __forceinline__ void issue_ext(const DecodeParams& p, const Item& it, int r0, int n, int lane, char* slot)
{
    const int G = p.group, row_lds = G * kD * 4, row_bytes = p.hq * kD * 4;
    const float* o0 = p.ext[0].o + ((long long)r0 * p.hq + (long long)it.kvh * G) * kD;
    const __amdgpu_buffer_rsrc_t rs = byte_buffer(o0, (n - 1) * row_bytes + row_lds);
#pragma unroll
    for (int e = 0; e < kExtLdsRows; ++e)
        for (int i = 0; i * 1024 < row_lds; ++i)
            if (lane * 16 + i * 1024 < row_lds)
                __builtin_amdgcn_raw_ptr_buffer_load_lds(rs, (lds_void*)(slot + e * row_lds + i * 1024), 16,
                                                         lane * 16 + i * 1024 + e * row_bytes, 0, 0, 0);
    const float* l0 = p.ext[0].lse + (long long)r0 * p.hq + (long long)it.kvh * G;
    const __amdgpu_buffer_rsrc_t rl = byte_buffer(l0, ((n - 1) * p.hq + G) * 4);
    if (lane < kExtLdsRows * G) {                          // lane = row * G + head
        const int e = lane / G, g = lane - e * G;
        __builtin_amdgcn_raw_ptr_buffer_load_lds(rl, (lds_void*)(slot + kExtLdsRows * row_lds), 4, (e * p.hq + g) * 4, 0, 0, 0);
    }
}

// after a barrier: the final rows of an item whose sequence ends here, from the states of waves w0 .. w1-1
// and the n rows waiting in the item's LDS slot (own state first, then the rows in order)
template <int n>
__device__ __forceinline__ void combine_fold_store(const DecodeParams& p, const Item& it, const float* area,
                                                   int lane, int w0, int w1, const char* slot)
{
    const int G = p.group;
    const long long orow0 = (long long)it.seq * p.hq + (long long)it.kvh * G;
    const float* e_o = reinterpret_cast<const float*>(slot);
    const float* e_lse = reinterpret_cast<const float*>(slot + (size_t)kExtLdsRows * G * kD * 4);
    // Two (head, four dims) positions per lane and turn, and every LDS read of a turn before anything is used:
    // this wave works alone and in order, so what its work costs is its chains of waits.
    constexpr int kSide = 2;
    for (int base = lane; base < G * (kD / 4); base += kSide * kWave) {
        int g[kSide], d[kSide];
        bool on[kSide];
        float le[kSide][n], lse[kSide];
        f32x4 x[kSide][n], o[kSide];
#pragma unroll
        for (int k = 0; k < kSide; ++k) {
            const int idx = base + k * kWave;
            on[k] = idx < G * (kD / 4);
            g[k] = on[k] ? idx >> 5 : 0;
            d[k] = (idx & 31) * 4;
#pragma unroll
            for (int e = 0; e < n; ++e) {
                le[k][e] = on[k] ? e_lse[e * G + g[k]] : -INFINITY;
                x[k][e] = *reinterpret_cast<const f32x4*>(e_o + (size_t)(e * G + g[k]) * kD + d[k]);
            }
        }
#pragma unroll
        for (int k = 0; k < kSide; ++k) combine_quad<false>(area, G, on[k] ? base + k * kWave : 0, w0, w1, o[k], lse[k]);
#pragma unroll
        for (int k = 0; k < kSide; ++k) {
            float m = lse[k];
#pragma unroll
            for (int e = 0; e < n; ++e) m = fmaxf(m, le[k][e]);
            f32x4 out = {0.f, 0.f, 0.f, 0.f};
            float out_lse = -INFINITY;
            if (m != -INFINITY) {
                // own state first, then the rows in order; a row without weight may hold anything and is left out
                float wsum = lse[k] == -INFINITY ? 0.f : __builtin_amdgcn_exp2f((lse[k] - m) * kLog2e);
                f32x4 acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
                for (int c = 0; c < 4; ++c) acc[c] = lse[k] == -INFINITY ? 0.f : wsum * o[k][c];
#pragma unroll
                for (int e = 0; e < n; ++e) {
                    const bool live = le[k][e] != -INFINITY;
                    const float w = live ? __builtin_amdgcn_exp2f((le[k][e] - m) * kLog2e) : 0.f;
                    wsum += w;
#pragma unroll
                    for (int c = 0; c < 4; ++c) acc[c] += live ? w * x[k][e][c] : 0.f;
                }
                out = acc * (1.f / wsum);
                out_lse = m + __builtin_amdgcn_logf(wsum) * kLn2;
            }
            if (on[k]) store_final_quad(p.out_o, p.out_lse, p.out_bf16 != 0, orow0 + g[k], d[k], out, out_lse);
        }
    }
}

// after a barrier: the item's rows from the states of waves w0 .. w1-1, and their stores (only seq, chunk and
// kvh of `it` are used); thread `tid` of `nthreads` takes four dims of one head per turn.  The fold of rows
// from other sources is the out-of-line merge's (one wave calls this then).
template <bool can_fold, bool half = false>
__device__ __forceinline__ void combine_and_store(const DecodeParams& p, const Item& it, const float* lds, int G,
                                                  int tid, int nthreads, int mode, MergeJob* job = nullptr,
                                                  int w0 = 0, int w1 = kWaves)
{
    if (can_fold && mode == kRowFinalFold) {           // left to the merge routine: the caller runs the job
        merge_job(*job, p, it.seq, it.kvh * G, G);
        job->own_lds = lds; job->w0 = w0; job->w1 = w1;
        return;
    }
    const bool final_row = mode == kRowFinal;
    // a final row is also kept as a partial one when the call has a single chunk slot and a partial buffer
    const bool partial_row = !final_row || p.max_chunks == 1;
    // `half`: the item's rows are the 2 G heads of a kv-head pair, 64 dims each, among 2 p.hq heads; its
    // combine area has 4 G columns
    constexpr int dout = half ? kD / 2 : kD;
    const int heads = half ? 2 * G : G, hq = half ? 2 * p.hq : p.hq, cols = half ? 4 * G : G;
    const long long prow0 = ((long long)it.seq * p.max_chunks + chunk_index(it.chunk)) * hq + (long long)it.kvh * heads;
    const long long orow0 = (long long)it.seq * hq + (long long)it.kvh * heads;
    for (int idx = tid; idx < heads * (dout / 4); idx += nthreads) {
        const int g = half ? idx >> 4 : idx >> 5, d = half ? (idx & 15) * 4 : (idx & 31) * 4;
        f32x4 o;
        float lse;
        combine_quad<half>(lds, cols, idx, w0, w1, o, lse);
        if (p.part_o && partial_row && lse != -INFINITY) {
            if (mode == kRowShared) store_shared4(p.part_o + prow0 * dout, heads * dout * 4, (g * dout + d) * 4, o);
            else __builtin_nontemporal_store(o, reinterpret_cast<f32x4*>(p.part_o + (prow0 + g) * dout + d));
        }
        // 4 G bytes: a plain store, so that the L2 can fill the line; the slot of a row that went out as a
        // final row holds no partial
        if (p.part_lse && d == 0) {
            if (mode == kRowShared) __hip_atomic_store(p.part_lse + prow0 + g, lse, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            else p.part_lse[prow0 + g] = partial_row ? lse : -INFINITY;
        }
        if (final_row) store_final_quad(p.out_o, p.out_lse, p.out_bf16 != 0, orow0 + g, d, o, lse, dout);
    }
}

// rows of an empty range: LSE = -inf, partial O left unwritten; `heads` rows from `head0`.  `final_here`:
// the range is the sequence's whole (empty) range and the call writes final rows: O = 0 and LSE = -inf
// (what other sources hold for such a sequence is the out-of-line merge's, see the persistent form).
__device__ __forceinline__ void store_empty(const DecodeParams& p, int seq, int chunk, int head0, int heads,
                                            int tid, int nthreads, bool final_here, int hq, int dout)
{
    const long long prow0 = ((long long)seq * p.max_chunks + chunk) * hq + head0;
    const long long orow0 = (long long)seq * hq + head0;
    if (p.part_lse)
        for (int h = tid; h < heads; h += nthreads) p.part_lse[prow0 + h] = -INFINITY;
    if (final_here) {
        const int quads = dout / 4;
        for (int idx = tid; idx < heads * quads; idx += nthreads)
            store_final_quad(p.out_o, p.out_lse, p.out_bf16 != 0, orow0 + idx / quads, (idx % quads) * 4,
                             f32x4{0.f, 0.f, 0.f, 0.f}, -INFINITY, dout);
    }
}

// ---------------------------------------------------------------------------------------------------
// grid form
// ---------------------------------------------------------------------------------------------------
template <bool half>
__global__ __launch_bounds__(kThreads, 3) void decode_mfma_grid_kernel(DecodeParams p, const int* __restrict__ block_table)
{
    // the K staging areas and the combine area share the same LDS: the combine starts after a barrier
    // behind every wave's last K read, and nothing is in flight by then in this form
    extern __shared__ __attribute__((aligned(16))) float lds[];
    const LaneIds id(reinterpret_cast<char*>(lds));
    Item it;
    const int item = blockIdx.x;
    it.kvh = item % p.hkv;
    it.seq = (item / p.hkv) % p.batch;
    const int chunk = item / (p.hkv * p.batch);
    int b, e;
    seq_range(p, it.seq, b, e);
    chunk_range(p, b, e, chunk, it.cb, it.ce);
    const int n_live = seq_parts(p, it.seq, b, e);
    it.chunk = pack_chunk(chunk, n_live);
    if (p.seq_final && chunk == 0 && it.kvh == 0 && threadIdx.x == 0)
        p.seq_final[it.seq] = (p.out_o != nullptr && n_live <= 1) ? 1 : 0;
    if (it.ce <= it.cb) {
        constexpr int per = half ? 2 : 1;                  // heads per kv head of the launch's geometry
        store_empty(p, it.seq, chunk, it.kvh * p.group * per, p.group * per, threadIdx.x, kThreads,
                    p.out_o != nullptr && chunk == 0 && n_live <= 1, p.hq * per, kD / per);
        return;
    }
    finish_item(it, block_table, p.max_blocks);
    it.s0 = id.wave;
    it.ds = kWaves;
    const float scale2 = p.sm_scale * kLog2e;
    u32x4 qb[4];
    load_q<half>(p, it, id.col, id.kg, qb);
    WaveState st;
    st.reset();
    StepRegs r;
    Pages cur = {-1, -1}, second = {-1, -1};              // pages of the wave's first and second step of the item
    if (id.wave < it.n_steps) {
        cur = step_pages<half>(p, it, id.wave);
        issue_step(p, it.kvh, cur, id.lane, id.stage, id.v_lane_off, r);
    }
    if (id.wave + kWaves < it.n_steps) second = step_pages<half>(p, it, id.wave + kWaves);
    run_item<false, half>(p, it, st, r, qb, id, scale2, cur, second, [](bool) {}, [] { return Tail{false, 0, Pages{-1, -1}}; },
                          [] {}, [] {});
    __syncthreads();
    stage_wave_state(st, lds, half ? 4 * p.group : p.group, id.wave, id.col, id.kg);
    __syncthreads();
    combine_and_store<false, half>(p, it, lds, p.group, threadIdx.x, kThreads, row_mode(p, n_live));
}

// ---------------------------------------------------------------------------------------------------
// persistent form
// ---------------------------------------------------------------------------------------------------
// (workspace layout: omni_internal.hpp)

// Ranges of up to kShortTokens tokens ("short") are dealt out one per wave, four to a ticket; the sort keeps
// them apart from the longer ones: bins 0 .. kLongBins-1 hold the longer ranges by scaled page count (bin 0
// the longest), then comes one bin per page count of the short ones, so that the first short entry of the
// sorted list is known exactly.
constexpr int kShortTokens = 256;
constexpr int kShortPages = kShortTokens / kBlockSize;
constexpr int kLongBins = kSortBins - kShortPages;

__host__ __device__ __forceinline__ float sort_bins_per_page(int chunk_tokens)
{
    const int max_pages = chunk_tokens / kBlockSize > 0 ? chunk_tokens / kBlockSize : 1;
    return (float)(kLongBins - 1) / (float)max_pages;
}

__host__ __device__ __forceinline__ int sort_bin(int tokens, float bins_per_page)
{
    const int pages = (tokens + kBlockSize - 1) / kBlockSize;
    if (tokens <= kShortTokens) return kSortBins - pages;
    int b = (int)((float)pages * bins_per_page);
    if (b > kLongBins - 1) b = kLongBins - 1;
    return (kLongBins - 1) - b;
}

// Every active lane takes one slot of counters[key].  The two keys that whole waves tend to share (`hot_a`:
// full chunks, `hot_b`: empty ones) are served by one LDS atomic per wave; the other keys, which differ
// from lane to lane, by one atomic per lane.  Must be called by all lanes of the wave together.
__device__ __forceinline__ unsigned wave_take_slot(unsigned* counters, int key, bool active, int hot_a, int hot_b)
{
    const int lane = threadIdx.x & 63;
    const unsigned long long below = (1ull << lane) - 1ull;
    unsigned slot = 0;
    bool served = !active;
#pragma unroll
    for (int h = 0; h < 2; ++h) {
        const int hot = h ? hot_b : hot_a;
        const bool mine = active && key == hot;
        const unsigned long long grp = __ballot(mine);
        if (grp) {
            const int leader = __builtin_ctzll(grp);
            unsigned base = 0;
            if (lane == leader) base = atomicAdd(&counters[hot], (unsigned)__popcll(grp));
            base = __builtin_amdgcn_readlane(base, leader);
            if (mine) { slot = base + (unsigned)__popcll(grp & below); served = true; }
        }
    }
    if (!served) slot = atomicAdd(&counters[key], 1u);
    return slot;
}

// Work list of a call: the non-empty (sequence, chunk) ranges, longest first, from the front of
// `entries`; the empty ones from the back.  Header: word 0 ticket counter (zeroed here), word 1 number
// of non-empty entries, word 2 number of empty ones, word 3 count of departed workgroups (zeroed here),
// word 5 number of waves that ever gave up waiting for a ticket (zeroed here; stays zero), word 6 number
// of non-empty entries longer than kShortTokens (they come first).
// Depends only on the ranges and the chunking, so a list can serve every call that shares them (all
// layers of one decoding iteration).
constexpr int kListCachedSeqs = 2048;                  // sequences whose ranges the list kernel keeps in LDS

__global__ __launch_bounds__(1024) void decode_list_kernel(DecodeParams p, unsigned* __restrict__ header,
                                                           WorkEntry* __restrict__ entries, unsigned* __restrict__ arrivals)
{
    __shared__ unsigned hist[kSortBins + 1];               // last counter: empty entries
    __shared__ int sh_b[kListCachedSeqs], sh_e[kListCachedSeqs];
    const int total = p.batch * p.max_chunks;
    const int max_pages = p.chunk_tokens / kBlockSize > 0 ? p.chunk_tokens / kBlockSize : 1;
    const float bins_per_page = sort_bins_per_page(p.chunk_tokens);
    const int full_bin = sort_bin(max_pages * kBlockSize, bins_per_page);     // the key whole waves tend to share
    const bool cached = p.batch <= kListCachedSeqs;        // one trip to memory for the ranges, then LDS
    for (int i = threadIdx.x; i < kSortBins + 1; i += blockDim.x) hist[i] = 0;
    if (cached) {
        for (int i = threadIdx.x; i < p.batch; i += blockDim.x) {
            int b, en;
            seq_range(p, i, b, en);
            sh_b[i] = b;
            sh_e[i] = en;
        }
    }
    __syncthreads();
    auto entry_range = [&](int e, int& seq, int& chunk, int& cb, int& ce) {
        seq = e / p.max_chunks;
        chunk = e - seq * p.max_chunks;
        int b, en;
        if (cached) { b = sh_b[seq]; en = sh_e[seq]; }
        else seq_range(p, seq, b, en);
        chunk_range(p, b, en, chunk, cb, ce);
        return seq_parts(p, seq, b, en);
    };
    for (int i = threadIdx.x; i < p.batch * p.hkv; i += blockDim.x) arrivals[i] = 0;
    for (int base = 0; base < total; base += blockDim.x) {
        const int e = base + threadIdx.x;
        int seq, chunk, cb = 0, ce = 0;
        if (e < total) entry_range(e, seq, chunk, cb, ce);
        const bool live = ce > cb;
        wave_take_slot(hist, live ? sort_bin(ce - cb, bins_per_page) : kSortBins, e < total, full_bin, kSortBins);
    }
    __syncthreads();
    if (threadIdx.x < kWave) {                             // exclusive scan by one wave: bin -> first output slot
        constexpr int kPer = kSortBins / kWave;
        unsigned c[kPer], sum = 0;
#pragma unroll
        for (int i = 0; i < kPer; ++i) { c[i] = hist[threadIdx.x * kPer + i]; sum += c[i]; }
        unsigned incl = sum;
#pragma unroll
        for (int d = 1; d < kWave; d <<= 1) {
            const unsigned up = __shfl_up(incl, d);
            if ((int)threadIdx.x >= d) incl += up;
        }
        unsigned run = incl - sum;
#pragma unroll
        for (int i = 0; i < kPer; ++i) {
            if (threadIdx.x * kPer + i == kLongBins) header[6] = run;      // entries before the first short one
            hist[threadIdx.x * kPer + i] = run;
            run += c[i];
        }
        if (threadIdx.x == kWave - 1) {
            header[0] = 0;
            header[1] = incl;
            header[2] = hist[kSortBins];
            header[3] = 0;
            header[5] = 0;
            hist[kSortBins] = 0;
        }
    }
    __syncthreads();
    for (int base = 0; base < total; base += blockDim.x) {
        const int e = base + threadIdx.x;
        int seq = 0, chunk = 0, cb = 0, ce = 0, n_live = 0;
        if (e < total) n_live = entry_range(e, seq, chunk, cb, ce);
        const bool live = ce > cb;
        const unsigned slot = wave_take_slot(hist, live ? sort_bin(ce - cb, bins_per_page) : kSortBins, e < total,
                                             full_bin, kSortBins);
        if (e < total) entries[live ? slot : (unsigned)(total - 1) - slot] = WorkEntry{seq, pack_chunk(chunk, n_live), cb, ce};
    }
}

// What the tickets of a launch stand for, in list order (longest ranges first).  Tickets below t_long are
// one item each: its steps are dealt round-robin to the four streaming waves.  Every further ticket
// stands for four consecutive items, one per wave: a wave takes all steps of its item, so the workgroup
// keeps four steps in flight where a short item alone has fewer steps than waves, and one ticket draw
// serves four items (measured on batches of 32..128-token ranges: 1.3-2.2 x the rate).  Only ranges of up
// to kShortTokens tokens are grouped, and only if there are enough of them to give every workgroup a
// grouped ticket: fewer are just the tail of the launch, where the smaller one-item tickets keep the
// workgroups' finishing times closer together (config 3: grouping its ~800 short ranges costs 1.4 %).
struct TicketSpace {
    unsigned n_items, t_long, n_tickets;
};

// n_live non-empty list entries, the first n_long of them longer than kShortTokens, hkv items per entry,
// n_workgroups workgroups in the launch
__host__ __device__ __forceinline__ TicketSpace make_ticket_space(unsigned n_live, unsigned n_long, unsigned hkv,
                                                                  unsigned n_workgroups)
{
    TicketSpace ts;
    ts.n_items = n_live * hkv;
    ts.t_long = (n_long < n_live ? n_long : n_live) * hkv;
    if (ts.n_items - ts.t_long < (unsigned)kWaves * n_workgroups) ts.t_long = ts.n_items;
    ts.n_tickets = ts.t_long + (ts.n_items - ts.t_long + (unsigned)kWaves - 1u) / (unsigned)kWaves;
    return ts;
}

// list item (entry index * hkv + kv head) of wave `wave` under `ticket`; false if the wave has none
__host__ __device__ __forceinline__ bool ticket_index(const TicketSpace& ts, unsigned ticket, int wave, unsigned& idx,
                                                      bool& grouped)
{
    grouped = ticket >= ts.t_long;
    idx = grouped ? ts.t_long + (unsigned)kWaves * (ticket - ts.t_long) + (unsigned)wave : ticket;
    return idx < ts.n_items;
}

// this wave's item under a ticket (ticket < n_tickets); n_steps = 0 if the wave has none
__device__ __forceinline__ Item ticket_item(const DecodeParams& p, const WorkEntry* __restrict__ entries,
                                            const int* __restrict__ block_table, const TicketSpace& ts,
                                            unsigned ticket, int wave)
{
    bool grouped;
    unsigned idx;
    const bool valid = ticket_index(ts, ticket, wave, idx, grouped);
    idx = valid ? idx : ts.n_items - 1u;
    const WorkEntry w = load_invariant(entries + idx / (unsigned)p.hkv);
    Item it;
    it.kvh = (int)(idx % (unsigned)p.hkv);
    // A list that was planned for these very ranges holds only values that pass unchanged; one reused
    // against the contract (other batch, other chunking) is forced into bounds, so that wrong rows are the
    // worst that can come of it, never an access outside the table or the output buffers.
    const int cap = p.max_blocks * kBlockSize;
    it.seq = min(max(w.seq, 0), p.batch - 1);
    it.chunk = pack_chunk(min(chunk_index(w.chunk), p.max_chunks - 1), min(max(chunk_live(w.chunk), 1), p.max_chunks + 1 - p.fuse));  // (parts: chunks, + 1 for rows from elsewhere)
    it.cb = min(max(w.cb, 0), cap - 1);
    it.ce = min(max(w.ce, it.cb + 1), cap);
    finish_item(it, block_table, p.max_blocks);
    it.s0 = grouped ? 0 : wave;
    it.ds = grouped ? 1 : kWaves;
    if (!valid) it.n_steps = 0;
    return it;
}

// what the streaming waves tell the writer about an item: [0] last ticket, [1] grouped, then per wave (seq,
// chunk word, kv head, rows from elsewhere as bring_ext returns them)
constexpr int kItemWords = 2 + 4 * kWaves;

// `fused`: the launch may finish sequences by merging (p.fuse); the plain instance carries none of that code,
// whose register needs change how the compiler schedules the streaming loop (2 % of the launch).
// `timed`: the instance behind omni_debug_decode_timeline, which stamps the constant-rate clock into
// p.stamps (kStampWords per workgroup) as the workgroup goes along.
constexpr int kStampWords = 32, kStampTickets = kStampWords - 8;

template <bool fused, bool half, bool timed>
__device__ __forceinline__ void persistent_body(
    const DecodeParams& p, const int* __restrict__ block_table, unsigned* ticket_counter,
    const unsigned* __restrict__ counts, const WorkEntry* __restrict__ entries, unsigned* arrivals)
{
    extern __shared__ __attribute__((aligned(16))) float lds[];
    __shared__ unsigned sh_ticket[3];
    // by ticket parity: [0] 1 if the workgroup's last, [1] 1 if one item per wave, then (seq, chunk, kvh,
    // non-empty chunks of the sequence) of the item (slot 0) or of each wave's item (seq < 0: the wave had none)
    __shared__ int sh_item[2][kItemWords];
    __shared__ MergeJob sh_job[kWaves];                    // the writer wave's jobs for the merge routine, per ticket
    const int comb_cols = half ? 4 * p.group : p.group;    // columns of the Q^T operand that are in use
    const size_t comb_bytes = combine_bytes(comb_cols);    // two combine areas, by ticket parity
    char* const stage_base = reinterpret_cast<char*>(lds) + 2 * comb_bytes;
    char* const q_base = stage_base + kWaves * kStageBytes;          // [parity][wave] buffers of G rows
    const int q_bytes = p.group * kD * 2;
    // fused form with one external source and few heads: [ticket % 3][wave] slots for the rows of items that
    // finish their sequence (see issue_ext).  Three deep: while the rows for ticket k+2 arrive (requested in
    // the last step of ticket k+1), the writer wave may still be reading those of ticket k.
    const bool ext_lds = fused && p.n_ext == 1 && p.group <= kExtLdsGroup;
    char* const ext_base = q_base + 2 * kWaves * q_bytes;
    const size_t ext_bytes = ext_slot_bytes(p.group);
    const LaneIds id(stage_base);
    const unsigned total = (unsigned)(p.batch * p.max_chunks);
    const TicketSpace ts = make_ticket_space(min(counts[0], total), counts[5], (unsigned)p.hkv, gridDim.x);
    const unsigned n_tickets = ts.n_tickets;
    const float scale2 = p.sm_scale * kLog2e;
    // [0] start, [1] first Q landed, [2] streaming waves done, [3] last store done, [4] tickets, [5] steps of wave 0,
    // [8 + k] the workgroup's meeting after ticket k
    unsigned long long* const stamp = timed ? p.stamps + (size_t)blockIdx.x * kStampWords : nullptr;
    if (timed && threadIdx.x == 0) stamp[0] = wall_clock64();
    int n_steps_wave0 = 0;

    // rows of empty chunks: LSE = -inf, and the final row of a sequence whose whole range is empty (stores
    // only, shared out over the resident workgroups); and which sequences this call finishes
    auto store_empty_share = [&] {
        auto empty_slot = [&](int seq, int chunk, int n_parts) {
            const bool final_here = p.out_o != nullptr && chunk == 0 && n_parts <= 1;
            store_empty(p, seq, chunk, 0, half ? 2 * p.hq : p.hq, id.lane, kWave, final_here && !(fused && p.n_ext > 0),
                        half ? 2 * p.hq : p.hq, half ? kD / 2 : kD);
            if (fused && final_here && p.n_ext > 0) fold_rows_plain(p, seq, id.lane);
        };
        const unsigned n_empty = min(counts[1], total);
        for (unsigned i = blockIdx.x; i < n_empty; i += gridDim.x) {
            const WorkEntry w = load_invariant(entries + (total - 1u - i));
            empty_slot(uniform(min(max(w.seq, 0), p.batch - 1)), uniform(min(chunk_index(w.chunk), p.max_chunks - 1)),
                       uniform(chunk_live(w.chunk)));
        }
        if (p.seq_final) {
            for (int i = blockIdx.x * kWave + id.lane; i < p.batch; i += gridDim.x * kWave) {
                int b, e;
                seq_range(p, i, b, e);
                p.seq_final[i] = (p.out_o != nullptr && (p.fuse || seq_parts(p, i, b, e) <= 1)) ? 1 : 0;
            }
        }
    };

    // A workgroup's first ticket is fixed by its index; every further one is drawn from the ticket counter
    // as late as the latencies allow, so that a workgroup that gets little of the memory bandwidth (the
    // CU favours its oldest waves) does not sit on items claimed long ago while the others run dry.
    // Slot j % 3 of sh_ticket holds the workgroup's j-th ticket once thread 0 knows it (kPending before).
    // Ticket k+1 is drawn by thread 0 before its second-to-last step of ticket k and published after that
    // step; if its wave has fewer than two steps under ticket k, it is drawn a whole ticket earlier, in the
    // last step of ticket k-1 (for k = 0: at the start).  Every wave picks the ticket up right before its
    // own last step of ticket k (waiting, if it got there first, for thread 0, which never waits for
    // anybody between barriers), reads its item's description and first pages, and in that last step
    // streams the first step of its next item instead of a further step of this one, so the memory pipe
    // does not drain between items.
    constexpr unsigned kPending = 0xffffffffu, kPollLimit = 1u << 24;
    bool gave_up = false;
    const unsigned first_dynamic = gridDim.x;
    auto short_item = [](const Item& x) { return x.n_steps <= x.s0 + x.ds; };      // fewer than two steps for this wave
    auto has_steps = [](const Item& x) { return x.s0 < x.n_steps; };
    // who brings an item's Q rows into LDS, and where: wave 0 for all, or every wave for its own item
    auto brings_q = [&](const Item& x) { return x.ds == 1 ? x.n_steps > 0 : id.wave == 0; };
    auto q_buffer = [&](int parity, const Item& x) {
        return q_base + (parity * kWaves + (x.ds == 1 ? id.wave : 0)) * q_bytes;
    };
    // What an item's final row still needs from the call's external sources, for the wave that brings its Q
    // rows: `rows` = 0: nothing (not the sequence's only part, or no rows there), n > 0: n rows from row `first`
    // on that go through the item's LDS slot, -1: rows that do not (the merge routine fetches them).
    struct ExtRows { int rows, first; };
    auto ext_slot = [&](int third, int wave) { return ext_base + (size_t)(third * kWaves + wave) * ext_bytes; };
    auto ext_rows = [&](const Item& x) {                   // (scalar loads: call it where the item's pages are read)
        if (!fused || row_mode(p, chunk_live(x.chunk)) != kRowFinalFold) return ExtRows{0, 0};
        int n_all = 0, r0 = 0, r1 = 0;
        for (int s = 0; s < p.n_ext; ++s) {
            if (p.ext[s].row_offsets) {
                r0 = load_invariant(p.ext[s].row_offsets + x.seq);
                r1 = load_invariant(p.ext[s].row_offsets + x.seq + 1);
            } else {
                r0 = x.seq * p.ext[s].dense_rows_per_seq;
                r1 = r0 + p.ext[s].dense_rows_per_seq;
            }
            n_all += max(r1 - r0, 0);
        }
        n_all = uniform(n_all);
        if (n_all == 0) return ExtRows{0, 0};
        if (!ext_lds || n_all > kExtLdsRows) return ExtRows{-1, 0};
        return ExtRows{n_all, uniform(r0)};
    };
    auto bring_ext = [&](int third, const Item& x, ExtRows e) {
        if (fused && e.rows > 0) issue_ext(p, x, e.first, e.rows, id.lane, ext_slot(third, x.ds == 1 ? id.wave : 0));
    };
    // The workgroup's last ticket has nothing to stream behind it.  When its items are one per wave, each
    // wave stores the rows of its own item instead of leaving the four to the writer wave one after the
    // other: on batches of short items those four combines in a row are the end of the launch (measured on
    // the hybrid batch: the writer finished 3.2 us after the streaming waves, 6.4 us in the fused form).
    // Only rows that need nothing beyond the item's own state and its LDS slot go this way (`own_store`,
    // decided from the ticket's staged words alike by the wave and by the writer); rows that are shared with
    // other workgroups or go through the merge routine stay with the writer.
    auto staged_item = [&](const int* si, int w, Item& x, int& mode, int& ext) {
        x.seq = uniform(si[2 + 4 * w]);
        x.chunk = uniform(si[3 + 4 * w]);
        x.kvh = uniform(si[4 + 4 * w]);
        mode = row_mode(p, chunk_live(x.chunk));
        ext = 0;
        if (fused && mode == kRowFinalFold) {
            // rows from elsewhere: none (a plain final row), waiting in the item's LDS slot, or the merge routine's
            ext = uniform(si[5 + 4 * w]);
            if (ext == 0) mode = kRowFinal;
        }
    };
    auto own_store = [&](int mode, int ext) { return !fused || mode == kRowFinal || (mode == kRowFinalFold && ext > 0); };
    // the rows of wave w's item under a one-item-per-wave ticket k (own_store(mode, ext) holds)
    auto store_item = [&](int k, int w, const Item& x, int mode, int ext, const float* area) {
        if (fused && mode == kRowFinalFold) {
            const char* slot = ext_slot(k % 3, w);
            // (the row count as a constant: the rows' loads and weights are straight-line code)
            if (ext == 1) combine_fold_store<1>(p, x, area, id.lane, w, w + 1, slot);
            else if (ext == 2) combine_fold_store<2>(p, x, area, id.lane, w, w + 1, slot);
            else if (ext == 3) combine_fold_store<3>(p, x, area, id.lane, w, w + 1, slot);
            else combine_fold_store<4>(p, x, area, id.lane, w, w + 1, slot);
        } else {
            combine_and_store<false, half>(p, x, area, p.group, id.lane, kWave, mode, nullptr, w, w + 1);
        }
    };
    auto store_own_item = [&](int k, const int* si, const float* area) {
        Item x;
        int mode, ext;
        staged_item(si, id.wave, x, mode, ext);
        if (x.seq >= 0 && own_store(mode, ext)) store_item(k, id.wave, x, mode, ext, area);
    };
    unsigned tk = blockIdx.x;
    const int writer_id = id.wave - kWaves;                // the waves behind the streaming ones
    const bool writer = writer_id >= 0;
    constexpr bool two_writers = persistent_writers(fused) == 2;
    if (writer_id == 0) store_empty_share();
    if (tk >= n_tickets) return;

    // The writer wave does every global store of the workgroup: the rows of empty chunks now, then, ticket
    // after ticket, the combine of the four streaming waves' states and the rows of the item (or of the
    // waves' four items, which need no combine).  A store counts in the issuing wave's vector-memory
    // counter until the L2 has taken it, and the counter retires in order, so a store between a streaming
    // wave's loads holds back its waits on younger loads; the writer has no loads to wait for (measured:
    // 0.5-2 % on batches of short items, nothing on long ones).  It meets the streaming waves at one
    // barrier per ticket; the combine areas alternate, so it works on ticket k while the others stream
    // ticket k+1.  The partial O rows (whole 128-byte lines) carry the non-temporal hint: plain stores of
    // these few bytes (0.5 % of the traffic) cost 3-4 % of the read rate on long contexts with many chunks,
    // whichever wave issues them.  An item's LSE values are 4 G bytes of a line that several items share:
    // they go out as plain stores, which the L2 gathers (with the hint each is a partial-line write to
    // memory: 1-1.5 % of the launch on configs 3 and 5).
    if (writer) {
        lds_barrier();
        for (int k = 0;; ++k) {
            lds_barrier();                                 // ticket k is staged
            const int* si = sh_item[k & 1];
            const bool last = si[0] != 0, grouped = si[1] != 0;
            const float* area = reinterpret_cast<const float*>(reinterpret_cast<const char*>(lds) + (k & 1) * comb_bytes);
            // The second writer takes the odd items of a one-item-per-wave ticket, those that `own_store`
            // says need nothing but their own state and LDS slot; everything else is the first writer's.
            if (two_writers && writer_id == 1) {
                if (grouped && !last) {
                    for (int w = 1; w < kWaves; w += 2) {
                        Item x;
                        int mode, ext;
                        staged_item(si, w, x, mode, ext);
                        if (x.seq >= 0 && own_store(mode, ext)) store_item(k, w, x, mode, ext, area);
                    }
                }
                if (last) break;
                continue;
            }
            // An item's rows are stored at once, unless they still have to be merged with rows from
            // elsewhere: those become jobs of the merge routine (at most one per item), run at the end.
            Item done;
            bool shared = false;
            int n_jobs = 0;
            const int n_done = grouped ? kWaves : 1;
            for (int w = 0; w < n_done; ++w) {
                int mode, ext;
                staged_item(si, w, done, mode, ext);
                if (done.seq < 0) continue;
                if (grouped && own_store(mode, ext)) {
                    if (last) continue;                                    // the item's own wave stores these
                    if (two_writers && (w & 1)) continue;                  // the second writer does
                }
                shared |= mode == kRowShared;
                if (fused && mode == kRowFinalFold) {
                    if (ext > 0) {
                        const int w0 = grouped ? w : 0, w1 = grouped ? w + 1 : kWaves;
                        const char* slot = ext_slot(k % 3, w);
                        // (the row count as a constant: the rows' loads and weights are straight-line code)
                        if (ext == 1) combine_fold_store<1>(p, done, area, id.lane, w0, w1, slot);
                        else if (ext == 2) combine_fold_store<2>(p, done, area, id.lane, w0, w1, slot);
                        else if (ext == 3) combine_fold_store<3>(p, done, area, id.lane, w0, w1, slot);
                        else combine_fold_store<4>(p, done, area, id.lane, w0, w1, slot);
                        continue;
                    }
                }
                MergeJob* job = &sh_job[n_jobs];
                if (grouped) combine_and_store<fused, half>(p, done, area, p.group, id.lane, kWave, mode, job, w, w + 1);
                else combine_and_store<fused, half>(p, done, area, p.group, id.lane, kWave, mode, job);
                if (fused && mode == kRowFinalFold) ++n_jobs;
            }
            if (fused && shared) {
                // The fused form.  The rows just stored (at device scope) have left this wave for good once
                // its vector-memory counter is back to zero; only then does the item count as arrived.
                // Whoever brings a (sequence, kv head)'s count to the number of its non-empty chunks finds
                // every one of those rows in place, merges them and puts the counter back to zero.
                __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
                OMNI_WAIT_VMCNT(0);
                for (int w = 0; w < n_done; ++w) {
                    const int seq = uniform(si[2 + 4 * w]), kvh = uniform(si[4 + 4 * w]);
                    const int n_live = chunk_live(uniform(si[3 + 4 * w]));
                    if (seq < 0 || row_mode(p, n_live) != kRowShared) continue;
                    unsigned* counter = arrivals + (long long)seq * p.hkv + kvh;
                    unsigned before = 0;
                    if (id.lane == 0) before = __hip_atomic_fetch_add(counter, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                    before = (unsigned)uniform((int)before);
                    if (before + 1u == (unsigned)n_live) {
                        if (id.lane == 0) __hip_atomic_store(counter, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                        merge_job(sh_job[n_jobs], p, seq, kvh * p.group, p.group);
                        sh_job[n_jobs].n_chunks = n_live;
                        ++n_jobs;
                    }
                }
                __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup");
            }
            if (fused)
                for (int i = 0; i < n_jobs; ++i) merge_and_store_final(&sh_job[i], id.lane);
            if (last) break;
        }
        if (timed && id.lane == 0) {
            OMNI_WAIT_VMCNT(0);
            atomicMax(&stamp[3], wall_clock64());          // (the streaming waves may store last, see below)
        }
        return;
    }

    // first ticket: Q goes into LDS, every wave requests its first step, then all read Q; the stores for
    // the empty rows go out while those first loads are on their way
    Item it = ticket_item(p, entries, block_table, ts, tk, id.wave);
    if (threadIdx.x == 0) {
        sh_ticket[0] = kPending;
        sh_ticket[2] = kPending;
        sh_ticket[1] = short_item(it) ? first_dynamic + atomicAdd(ticket_counter, 1u) : kPending;
    }
    int it_ext = 0;                                        // ext_rows(...).rows of the current item (in the wave that brings its Q)
    if (brings_q(it)) {
        issue_q(p, it, id.lane, q_buffer(0, it));
        const ExtRows e = ext_rows(it);
        bring_ext(0, it, e);
        it_ext = e.rows;
    }
    StepRegs r;
    Pages cur = {-1, -1}, second = {-1, -1};              // pages of the wave's first and second step of the item
    if (has_steps(it)) {
        cur = step_pages<half>(p, it, it.s0);
        issue_step(p, it.kvh, cur, id.lane, id.stage, id.v_lane_off, r);
    }
    if (it.s0 + it.ds < it.n_steps) second = step_pages<half>(p, it, it.s0 + it.ds);
    OMNI_WAIT_VMCNT(16);                                   // Q is older than the 16 K/V requests
    lds_barrier();
    u32x4 qb[4];
    read_q<half>(q_buffer(0, it), p.group, id.col, id.kg, qb);
    WaveState st;
    st.reset();
    if (timed && threadIdx.x == 0) stamp[1] = wall_clock64();

    for (int k = 0;; ++k) {
        make_uniform(it);                                  // (the loop-carried copy is where the analysis gives up)
        unsigned* const slot_next = &sh_ticket[(k + 1) % 3];
        const int parity_next = (k + 1) & 1;
        const bool late_draw = !short_item(it);
        const bool streamed = has_steps(it);
        Item nx = it;
        Tail tail = {false, 0, Pages{-1, -1}};
        Pages next_second = {-1, -1};
        bool has_next = false, q_coming = false;
        ExtRows nx_ext = {0, 0};
        unsigned t1 = 0, t2 = 0;
        bool draw2 = false;

        // the next ticket, this wave's item under it and the item's first pages
        auto acquire = [&] {
            // (the poll is bounded, about a second: should the ticket never come, the wave takes that as
            // "no further ticket", which ends the workgroup after this one instead of hanging the GPU)
            unsigned tn = kPending;
            for (unsigned n = 0; n < kPollLimit; ++n) {
                tn = __builtin_amdgcn_readfirstlane(lds_peek(slot_next));
                if (tn != kPending) break;
                __builtin_amdgcn_s_sleep(1);
            }
            if (tn == kPending) gave_up = true;
            has_next = tn < n_tickets;
            if (has_next) {
                nx = ticket_item(p, entries, block_table, ts, tn, id.wave);
                if (has_steps(nx)) tail = Tail{true, nx.kvh, step_pages<half>(p, nx, nx.s0)};
                // the table reads for the wave's second step of that item go out now as well: at the
                // item's start they would be a cold round trip in front of its second request
                next_second = Pages{-1, -1};
                if (nx.s0 + nx.ds < nx.n_steps) next_second = step_pages<half>(p, nx, nx.s0 + nx.ds);
                q_coming = brings_q(nx);
                if (fused && q_coming) nx_ext = ext_rows(nx);
            } else {
                nx.n_steps = 0;
            }
        };

        run_item<true, half>(p, it, st, r, qb, id, scale2, cur, second,
                 [&](bool before) {
                     if (threadIdx.x == 0 && late_draw) {
                         if (before) t1 = atomicAdd(ticket_counter, 1u);
                         else lds_post(slot_next, first_dynamic + t1);
                     }
                 },
                 [&] {
                     acquire();
                     // the next Q goes into the other set of Q buffers; if thread 0's wave has no
                     // second-to-last step under the next ticket to draw its successor in, it draws it now
                     if (q_coming) issue_q(p, nx, id.lane, q_buffer(parity_next, nx));
                     draw2 = has_next && short_item(nx);
                     if (threadIdx.x == 0 && draw2) t2 = atomicAdd(ticket_counter, 1u);
                     return tail;
                 },
                 [&] { bring_ext((k + 1) % 3, nx, nx_ext); },
                 [&] {
                     if (threadIdx.x == 0 && draw2) lds_post(&sh_ticket[(k + 2) % 3], first_dynamic + t2);
                 });
        // waves that had no step under this ticket request their Q and first step of the next one now
        if (!streamed) {
            acquire();
            if (q_coming) {
                issue_q(p, nx, id.lane, q_buffer(parity_next, nx));
                bring_ext((k + 1) % 3, nx, nx_ext);
            }
        }

        // accumulators go to LDS (the ticket's combine area); whoever requested Q rows makes sure they have
        // landed (they are older than the 16 K/V requests behind them); the waves say which items these
        // were; then the workgroup meets, with all those loads still in flight, and the writer wave takes
        // over
        float* const area = reinterpret_cast<float*>(reinterpret_cast<char*>(lds) + (k & 1) * comb_bytes);
        stage_wave_state(st, area, comb_cols, id.wave, id.col, id.kg);
        cur = tail.pages;
        second = next_second;
        if (tail.valid && !streamed) {
            issue_step(p, nx.kvh, cur, id.lane, id.stage, id.v_lane_off, r);
        }
        if (q_coming) {
            // Q is older than the 16 K / V requests behind it - and than the requests for rows from elsewhere,
            // when those went out between that K and that V (4 rows of one or two KiB, and the LSE values)
            const int between = (fused && streamed && nx_ext.rows > 0) ? kExtLdsRows * ((p.group * kD * 4 + 1023) / 1024) + 1 : 0;
            if (between == 9) OMNI_WAIT_VMCNT(25);
            else if (between == 5) OMNI_WAIT_VMCNT(21);
            else OMNI_WAIT_VMCNT(16);
        }
        const bool grouped = it.ds == 1;
        if (id.lane == 0 && (grouped || id.wave == 0)) {
            int* si = sh_item[k & 1];
            if (id.wave == 0) {
                si[0] = has_next ? 0 : 1;
                si[1] = grouped ? 1 : 0;
            }
            si[2 + 4 * id.wave] = streamed ? it.seq : -1;
            si[3 + 4 * id.wave] = it.chunk;
            si[4 + 4 * id.wave] = it.kvh;
            if (fused) si[5 + 4 * id.wave] = it_ext;
        }
        lds_barrier();
        if (timed && threadIdx.x == 0) {
            if (k < kStampTickets) stamp[8 + k] = wall_clock64();
            if (streamed) n_steps_wave0 += (it.n_steps - it.s0 + it.ds - 1) / it.ds;
            stamp[4] = (unsigned long long)(k + 1);
            stamp[5] = (unsigned long long)n_steps_wave0;
        }
        if (!has_next) {
            if (timed && threadIdx.x == 0) stamp[2] = wall_clock64();
            if (uniform(sh_item[k & 1][1]) != 0) {         // (the word the writer wave goes by)
                store_own_item(k, sh_item[k & 1], area);
                if (timed && id.lane == 0) {
                    OMNI_WAIT_VMCNT(0);
                    atomicMax(&stamp[3], wall_clock64());
                }
            }
            break;
        }
        if (threadIdx.x == 0) lds_post(slot_next, kPending);   // every wave has read it; next used by ticket k+4
        read_q<half>(q_buffer(parity_next, nx), p.group, id.col, id.kg, qb);
        st.reset();
        it = nx;
        it_ext = nx_ext.rows;
    }
    OMNI_WAIT_VMCNT(0);                                    // no direct-to-LDS load may outlive the workgroup
    if (gave_up && id.lane == 0) atomicAdd(ticket_counter + 5, 1u);
}

// Header words 0 (ticket counter) and 3 (workgroups that have left) are the only mutable state of a work
// list; the last workgroup to leave puts them back to zero, so the same list can serve the next call.
template <bool fused, bool half, bool timed = false>
__global__ __launch_bounds__(persistent_threads(fused), 1) void decode_mfma_persistent_kernel(
    DecodeParams p, const int* __restrict__ block_table, unsigned* header,
    const unsigned* __restrict__ counts, const WorkEntry* __restrict__ entries, unsigned* arrivals)
{
    persistent_body<fused, half, timed>(p, block_table, header, counts, entries, arrivals);
    if (threadIdx.x == 0) {
        const unsigned gone = atomicAdd(header + 3, 1u);   // after this workgroup's last ticket draw
        if (gone == gridDim.x - 1) {
            atomicExch(header + 3, 0u);
            atomicExch(header, 0u);
        }
    }
}

size_t lds_bytes(int group, bool persistent, bool fused = false)
{
    if (!persistent) {
        const size_t a = combine_bytes(group), b = (size_t)kWaves * kStageBytes;
        return a > b ? a : b;
    }
    const size_t ext = (fused && group <= kExtLdsGroup) ? 3 * (size_t)kWaves * ext_slot_bytes(group) : 0;
    return 2 * combine_bytes(group) + (size_t)kWaves * kStageBytes + 2 * (size_t)kWaves * group * kD * 2 + ext;
}

}  // namespace

// head_dim 64 runs as kv-head pairs (see the top of the file): an even number of kv heads, G <= 4
bool decode_mfma_half(const DecodeParams& p) { return p.d == kD / 2; }

bool decode_mfma_supports(const DecodeParams& p, bool bf16)
{
    const bool shape = (p.d == kD && p.group <= 16) || (p.d == kD / 2 && p.group <= 4 && p.hkv % 2 == 0);
    return bf16 && shape && (long long)p.batch * p.max_chunks * p.hkv <= 0x7fffffffLL;
}

size_t decode_workspace_bytes(long long batch, long long max_chunks, long long hkv)
{
    const size_t counters = ((size_t)(batch * hkv) * sizeof(unsigned) + 15) / 16 * 16;
    return (size_t)kHeaderWords * sizeof(unsigned) + (size_t)(batch * max_chunks) * sizeof(WorkEntry) + counters;
}

// Host-side views of the work-list logic, for tests: the sort bin of a range, and which list item every
// streaming wave takes under every ticket.
int decode_list_sort_bin(int tokens, int chunk_tokens)
{
    return tokens > 0 ? sort_bin(tokens, sort_bins_per_page(chunk_tokens)) : kSortBins;
}

unsigned decode_ticket_map(unsigned n_entries, unsigned n_long_entries, unsigned hkv, unsigned n_workgroups,
                           int* items, size_t capacity)
{
    const TicketSpace ts = make_ticket_space(n_entries, n_long_entries, hkv, n_workgroups);
    for (unsigned t = 0; t < ts.n_tickets && ((size_t)t + 1) * 2 * kWaves <= capacity; ++t)
        for (int w = 0; w < kWaves; ++w) {
            unsigned idx;
            bool grouped;
            const bool valid = ticket_index(ts, t, w, idx, grouped);
            items[((size_t)t * kWaves + w) * 2] = valid ? (int)idx : -1;
            items[((size_t)t * kWaves + w) * 2 + 1] = grouped ? 1 : 0;
        }
    return ts.n_tickets;
}

hipError_t launch_decode_plan(const DecodeParams& p, void* workspace, hipStream_t s)
{
    unsigned* header = static_cast<unsigned*>(workspace);
    WorkEntry* entries = reinterpret_cast<WorkEntry*>(header + kHeaderWords);
    unsigned* arrivals = reinterpret_cast<unsigned*>(entries + (size_t)p.batch * p.max_chunks);
    hipLaunchKernelGGL(decode_list_kernel, dim3(1), dim3(1024), 0, s, p, header, entries, arrivals);
    return hipGetLastError();
}

namespace {

// What a launch needs to know about the current device, found out once per device: the number of CUs, and
// that the persistent kernel fits a CU even with its largest LDS request (G = 16), for which both kernels
// are given the large LDS window.  Later calls only look the entry up.
struct DeviceFacts { int cus; hipError_t status; bool known; };

hipError_t device_facts(int& cus)
{
    constexpr int kMaxDevices = 64;
    static DeviceFacts facts[kMaxDevices] = {};
    static std::mutex mu;
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    if (dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice;
    std::lock_guard<std::mutex> lock(mu);
    DeviceFacts& f = facts[dev];
    if (!f.known) {
        f.status = hipDeviceGetAttribute(&f.cus, hipDeviceAttributeMultiprocessorCount, dev);
        const int lds_p = (int)std::max(lds_bytes(16, true), lds_bytes(kExtLdsGroup, true, true));
        const int lds_g = (int)lds_bytes(16, false);
        if (f.status == hipSuccess) {
            const void* forms[5] = {(const void*)decode_mfma_persistent_kernel<false, false>,
                                    (const void*)decode_mfma_persistent_kernel<true, false>,
                                    (const void*)decode_mfma_persistent_kernel<false, true>,
                                    (const void*)decode_mfma_persistent_kernel<false, false, true>,
                                    (const void*)decode_mfma_persistent_kernel<true, false, true>};
            for (int i = 0; i < 5 && f.status == hipSuccess; ++i)
                f.status = hipFuncSetAttribute(forms[i], hipFuncAttributeMaxDynamicSharedMemorySize, lds_p);
        }
        if (f.status == hipSuccess && lds_g > 64 * 1024) {
            f.status = hipFuncSetAttribute((const void*)decode_mfma_grid_kernel<false>,
                                           hipFuncAttributeMaxDynamicSharedMemorySize, lds_g);
            if (f.status == hipSuccess)
                f.status = hipFuncSetAttribute((const void*)decode_mfma_grid_kernel<true>,
                                               hipFuncAttributeMaxDynamicSharedMemorySize, lds_g);
        }
        int per_cu = 0;
        if (f.status == hipSuccess)
            f.status = hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, decode_mfma_persistent_kernel<true, false>,
                                                                    persistent_threads(true), lds_p);
        if (f.status == hipSuccess && (per_cu < 1 || f.cus < 1)) f.status = hipErrorLaunchOutOfResources;
        f.known = true;
    }
    cus = f.cus;
    return f.status;
}

}  // namespace

// Workgroups of a persistent launch on this device (the stamps of a timed launch: kStampWords each)
hipError_t decode_timeline_shape(int& n_workgroups, int& words_per_workgroup)
{
    words_per_workgroup = kStampWords;
    return device_facts(n_workgroups);
}

hipError_t launch_decode_mfma(const DecodeParams& given, void* workspace, bool planned, hipStream_t s)
{
    // head_dim 64: the kernels see kv-head pairs as kv heads of 128-wide rows, half as many of them and of
    // the 256-byte query rows, and 4 G columns of the Q^T operand in use
    const bool half = decode_mfma_half(given);
    DecodeParams p = given;
    if (half) {
        p.hq = given.hq / 2;
        p.hkv = given.hkv / 2;
        if (p.fuse) return hipErrorInvalidValue;           // (the API layer does not let this through)
    }
    const size_t lds = lds_bytes(half ? 4 * p.group : p.group, workspace != nullptr, p.fuse != 0);
    int cus = 0;
    hipError_t e = device_facts(cus);
    if (e != hipSuccess) return e;
    if (!workspace) {
        const unsigned grid = (unsigned)((long long)p.batch * p.max_chunks * p.hkv);
        if (half) hipLaunchKernelGGL(decode_mfma_grid_kernel<true>, dim3(grid), dim3(kThreads), lds, s, p, p.block_table);
        else hipLaunchKernelGGL(decode_mfma_grid_kernel<false>, dim3(grid), dim3(kThreads), lds, s, p, p.block_table);
        return hipGetLastError();
    }
    unsigned* header = static_cast<unsigned*>(workspace);
    WorkEntry* entries = reinterpret_cast<WorkEntry*>(header + kHeaderWords);
    if (!planned) {
        e = launch_decode_plan(p, workspace, s);
        if (e != hipSuccess) return e;
    }
    // One workgroup per CU.  More would fit (three), but the memory system is saturated by four waves
    // per CU already, and a CU serves its oldest waves first: a second and third workgroup get a
    // fraction of the first one's bandwidth, start late and finish late, which costs more at both ends
    // of the launch than their overlap gains in between (measured on every configuration).
    long long want = (long long)cus, cap = (long long)p.batch * p.max_chunks * p.hkv;
    const unsigned grid = (unsigned)(want < cap ? want : cap);
    unsigned* arrivals = reinterpret_cast<unsigned*>(entries + (size_t)p.batch * p.max_chunks);
    if (p.stamps && half) return hipErrorInvalidValue;                   // (the API layer does not let this through)
    auto kernel = half ? decode_mfma_persistent_kernel<false, true>
                       : (p.fuse ? (p.stamps ? decode_mfma_persistent_kernel<true, false, true> : decode_mfma_persistent_kernel<true, false>)
                                 : (p.stamps ? decode_mfma_persistent_kernel<false, false, true>
                                             : decode_mfma_persistent_kernel<false, false>));
    hipLaunchKernelGGL(kernel, dim3(grid), dim3(persistent_threads(p.fuse != 0)), lds, s, p, p.block_table, header, header + 1,
                       entries, arrivals);
    return hipGetLastError();
}

}  // namespace omni
