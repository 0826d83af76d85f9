// Fused Predict+Verify attention for bfloat16 caches with head_dim 128 and at most 64 query rows
// per KV head (rows = queries x grouped heads): the streaming kernel for gfx950.
//
// What is computed: see attention.hip (MemoSight paper, Sections 2.1.1 and 2.3).  How:
//   * The host cuts the batch's cached tokens, flattened over sequences in 32-token tiles, into
//     equal contiguous shares, one workgroup per (share, KV head).  A share that crosses sequence
//     boundaries is processed as several segments.
//   * Each of a workgroup's 8 waves streams tiles of a segment on its own: K goes from
//     HBM straight into MFMA operand registers, V is staged through a wave-private LDS tile and
//     read back transposed (ds_read_b64_tr_b16); a wave refills its registers for its next tile as
//     soon as the current tile has consumed them.  There is no barrier inside the stream.
//   * Scores are computed transposed, S^T = K . Q^T (v_mfma_f32_32x32x16_bf16), so a lane owns one
//     query row: the online softmax needs one cross-lane exchange per tile and the rescale of the
//     O^T = V^T . P^T accumulators is a per-lane scalar.  Rescaling is lazy (only when a row's
//     maximum grows by more than 2^24), scores are kept in log2 units.
//   * The step's own (in-flight) verify / foresight keys are one more tile: the workgroup that owns
//     a sequence's first segment rotates them into an LDS K tile and one of its waves runs the
//     tile with the visibility rule applied to the scores.
//   * Each segment takes a ticket in the finishing order of its (sequence, KV head) pair.  All but
//     the last leave a partial (row maxima, row sums, unnormalised O) in the workspace; the last
//     one folds the others' partials into its own registers, normalises and writes the bf16 output
//     rows.  One launch per call.
//   * Each wave's first tile of a segment is fixed; by default the waves then take further tiles
//     first come, first served (results reproducible to rounding), optionally every 8th tile each
//     (bit-reproducible).
#include <math.h>
#include <string.h>

#include <algorithm>
#include <mutex>
#include <vector>

#include "attention.h"
#include "ms_device.h"
#include "ms_internal.h"

namespace ms {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8_t;
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2_t;
typedef __attribute__((ext_vector_type(2))) float f32x2_t;
typedef __attribute__((ext_vector_type(16))) float f32x16_t;
typedef __attribute__((ext_vector_type(4))) short s16x4_t;
typedef __attribute__((ext_vector_type(8))) short s16x8_t;
typedef __attribute__((address_space(3))) s16x4_t lds_s16x4_t;

constexpr int kD = 128;
constexpr int kRows = 64;               // query rows per KV head (padded)
constexpr int kVRowBytes = 320;         // LDS bytes per V row: 256 + 64.  The transposed 8-byte reads of the PV operand
                                        // take 64 bytes of 4 consecutive rows per 32 lanes: with a stride of 16 banks
                                        // (mod 64) those fall on disjoint banks (288 left 22 % of the LDS cycles as conflicts)
constexpr int kQRowBytes = 272;         // LDS bytes per rotated-Q row
constexpr int kVTileBytes = kTile * kVRowBytes;
constexpr float kRescaleThreshold = 24.0f;  // log2 units: P stays below 2^24
constexpr int kPartFloats = 2 * kRows + kRows * kD;  // m[64], l[64], O[128 regs][64 lanes]

// LDS map.  Stream phase: [Q tile][cos/sin table][in-flight K tile][one V tile per wave].  Merge
// phase (overlays it): per wave 64 accumulator registers (two d blocks of both row blocks) + 4
// softmax scalars per lane.
//
// This is the decode kernel: all of a step's queries in one launch, at most 16 queries and 64 rows.
// Wider steps (memory-token pass, prompt chunks, per-position foresight: up to 64 queries) run
// pv_attn_mfma_wide further down.
constexpr int kDecodeQueries = 16;
constexpr int kMergeRegionBytes = (64 + 4) * 64 * 4;                     // 17408
constexpr int kLdsMerge = kWaves * kMergeRegionBytes;                    // 139264
struct Lds {
    static constexpr int kQueries = kDecodeQueries;   // rows of the cos/sin table
    static constexpr int kNewTiles = 1;
    static constexpr int kQ = 0;
    static constexpr int kCs = kQ + kRows * kQRowBytes;                  // 17408
    static constexpr int kKn = kCs + kQueries * 64 * 8;                  // + 8192
    static constexpr int kV = kKn + kNewTiles * kTile * kQRowBytes;      // + 8704
    static constexpr int kStream = kV + kWaves * kVTileBytes;            // + 73728 = 108032
    static constexpr int kFlag = kLdsMerge > kStream ? kLdsMerge : kStream;  // one word: "last arriver"
    static constexpr int kBytes = kFlag + 16;
    static_assert(kBytes <= 160 * 1024, "LDS budget of one compute unit");
};
constexpr int kThreads = kWaves * 64;
static_assert(kThreads == kRows * 8, "the Q prologue maps one thread to one row and 8 rotation pairs");
static_assert(MS_MAX_QUERIES * 8 <= kThreads, "the K prologue maps one thread to one in-flight key and 8 rotation pairs");

struct MfmaArgs {
    const uint16_t* pool_layer;
    const int* d_pt;
    const int* d_len;       // [max_seqs] lengths on the device: what the kernel goes by
    const float* inv_freq;
    const uint16_t* q;
    const uint16_t* k_new;
    const uint16_t* v_new;
    const int* pos;
    const int* ctx_new;
    uint16_t* out;
    float* ws;
    const Seg* item_first;  // [n_items]: first segment of every work item
    const Seg* segs;        // all segments in item order
    const int* part_begin;  // [B + 1]
    int* arrive;            // [B][n_kv_heads][2] counters (shares finished, partials published), zero between calls
    int* error_word;        // host memory the device can write: set when a closing workgroup gave up waiting
    int poll_limit;         // polls of the published counter before a closing workgroup gives up
    int n_q, n_verify, n_q_heads, n_kv_heads, group, max_pages;
    int q0, n_qc;           // wide kernel: this launch computes queries q0 .. q0 + n_qc
    long page_elems;
    float scale_log2;       // softmax scale * log2(e)
};

__device__ __forceinline__ uint32_t pack_bf16x2(float a, float b) {
    f32x2_t f = {a, b};
    bf16x2_t h = __builtin_convertvector(f, bf16x2_t);
    return __builtin_bit_cast(uint32_t, h);
}

typedef __attribute__((ext_vector_type(4))) unsigned int u32x4_t;

// sin and cos of an fp32 angle of any size (RoPE angles reach 1e5 rad): the reduction by pi/2 is
// done in fp64 (two-term constant), the kernels on [-pi/4, pi/4] are the classic single-precision
// minimax polynomials.  About 1e-7 absolute error, far below the bf16 rounding of the rotated rows,
// and much cheaper than the library routine's large-argument path.
__device__ __forceinline__ void sincos_reduced(float x, float* sn, float* cs) {
    const double xd = (double)x;
    const double n = rint(xd * 0.63661977236758134308);
    double r = fma(n, -1.57079632679489655800e+00, xd);
    r = fma(n, -6.12323399573676603587e-17, r);
    const float t = (float)r, t2 = t * t;
    const float sp = t + t * t2 * (-1.6666654611e-1f + t2 * (8.3321608736e-3f + t2 * -1.9515295891e-4f));
    const float cp = 1.0f - 0.5f * t2 + t2 * t2 * (4.166664568298827e-2f + t2 * (-1.388731625493765e-3f + t2 * 2.443315711809948e-5f));
    const int q = (int)n & 3;
    const float s1 = (q & 1) ? cp : sp, c1 = (q & 1) ? sp : cp;
    *sn = (q & 2) ? -s1 : s1;
    *cs = ((q + 1) & 2) ? -c1 : c1;
}

// 16-byte non-temporal global load.
__device__ __forceinline__ uint4 load_stream(const char* p) {
    const u32x4_t t = __builtin_nontemporal_load(reinterpret_cast<const u32x4_t*>(p));
    return make_uint4(t.x, t.y, t.z, t.w);
}

// Partials travel between workgroups on different XCDs, whose L2 caches are not coherent with each
// other.  They are written and read with device-scope relaxed atomic accesses (write-through /
// cache-bypassing), which needs no cache write-back or invalidation; ordering comes from waiting
// for the stores (workgroup barrier) before the arrival count is bumped.
__device__ __forceinline__ void store_coherent(float* p, float v) {
    __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ float load_coherent(const float* p) {
    return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
// 16-byte accesses with the same cache policy (the bit device-scope atomics carry: the other XCDs'
// L2s are bypassed), through a buffer descriptor over the partials: one instruction per float4
// instead of two 8-byte atomics.  byte_off < 2 GiB.
typedef uint32_t pv_u32x4_t __attribute__((ext_vector_type(4)));
constexpr int kCoherentPolicy = 16;   // sc1
__device__ __forceinline__ __amdgpu_buffer_rsrc_t partials_descriptor(float* ws) {
    return __builtin_amdgcn_make_buffer_rsrc(ws, 0, 0x7fffffff, 0x00020000);
}
__device__ __forceinline__ float4 load_coherent4(__amdgpu_buffer_rsrc_t rs, uint32_t byte_off) {
    const pv_u32x4_t v = __builtin_amdgcn_raw_buffer_load_b128(rs, (int)byte_off, 0, kCoherentPolicy);
    return make_float4(__uint_as_float(v.x), __uint_as_float(v.y), __uint_as_float(v.z), __uint_as_float(v.w));
}
__device__ __forceinline__ void store_coherent4(__amdgpu_buffer_rsrc_t rs, uint32_t byte_off, float4 f) {
    pv_u32x4_t v = {__float_as_uint(f.x), __float_as_uint(f.y), __float_as_uint(f.z), __float_as_uint(f.w)};
    __builtin_amdgcn_raw_buffer_store_b128(v, rs, (int)byte_off, 0, kCoherentPolicy);
}

// Read-only, wave-uniform control data (the work plan, position ids) is read through the constant
// address space: scalar loads, which return out of order with respect to the vector loads and so do
// not queue behind the tile loads in flight.
template <typename T>
__device__ __forceinline__ T uniform_load(const T* p) {
    return *reinterpret_cast<const __attribute__((address_space(4))) T*>(reinterpret_cast<uintptr_t>(p));
}

// Workgroup barrier that orders LDS traffic only.  __syncthreads() also waits for every outstanding
// global load, which would stall the set-up phases on the tile loads already in flight.
__device__ __forceinline__ void lds_barrier() {
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup", "local");
    __builtin_amdgcn_s_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup", "local");
}

// Registers of one 32-token tile in flight.
struct TileRegs {
    uint4 k[8];  // K operand: token = lane % 32, d = 16 kk + 8 (lane / 32) .. + 8
    uint4 v[8];  // V rows as loaded: token = 4 r + lane / 16, d = 8 (lane % 16) .. + 8
};

// Page ids of a tile's two pages.  `tile` may lie past the segment: it is clamped, so that loads
// stay unconditional (a fixed number of loads in flight lets the waits stay partial).
__device__ __forceinline__ void tile_pages(const int* __restrict__ pt, int tile, int n_tiles, int t0, int last_page,
                                           int& pa, int& pb) {
    const int tc = tile < n_tiles ? tile : n_tiles - 1;
    const int pg0 = (t0 >> 4) + 2 * tc;
    pa = __builtin_amdgcn_readfirstlane(pt[pg0 < last_page ? pg0 : last_page]);
    pb = __builtin_amdgcn_readfirstlane(pt[pg0 + 1 < last_page ? pg0 + 1 : last_page]);
}

// K operand of a tile straight from the pool.  Addresses are a uniform base plus a 32-bit byte
// offset per lane (page_bytes * page id + lane part), which keeps the per-lane address state to one
// register; layer pools of 4 GiB and more take the kBigPool build below.
template <bool kBigPool>
__device__ __forceinline__ void load_k(uint4 (&k)[8], const char* __restrict__ pool, int pa, int pb,
                                       uint32_t page_bytes, uint32_t lane_off_k, int lane) {
    if (!kBigPool) {
        const uint32_t off = (uint32_t)((lane & 16) ? pb : pa) * page_bytes + lane_off_k;
#pragma unroll
        for (int kk = 0; kk < 8; ++kk) k[kk] = *reinterpret_cast<const uint4*>(pool + off + 32 * kk);
    } else {
        // layer pools of 4 GiB and more: the page's base is a 64-bit (wave-uniform) address, the
        // half-waves pick theirs, the lane part stays a 32-bit offset
        const char* base_a = pool + (size_t)(uint32_t)pa * page_bytes;
        const char* base_b = pool + (size_t)(uint32_t)pb * page_bytes;
        const char* base = (lane & 16) ? base_b : base_a;
#pragma unroll
        for (int kk = 0; kk < 8; ++kk) k[kk] = *reinterpret_cast<const uint4*>(base + lane_off_k + 32 * kk);
    }
}

// V rows of a tile: tokens 4 rr + lane / 16 of page a (rr < 4) and of page b.  V is read exactly once
// per call: streaming (non-temporal) loads keep it out of the caches.
template <bool kBigPool>
__device__ __forceinline__ void load_v(uint4 (&v)[8], const char* __restrict__ pool, int pa, int pb,
                                       uint32_t page_bytes, uint32_t lane_off_v) {
    if (kBigPool) {
        const char* base_a = pool + (size_t)(uint32_t)pa * page_bytes;
        const char* base_b = pool + (size_t)(uint32_t)pb * page_bytes;
#pragma unroll
        for (int rr = 0; rr < 4; ++rr) v[rr] = load_stream(base_a + lane_off_v + 4 * rr * kD * 2);
#pragma unroll
        for (int rr = 0; rr < 4; ++rr) v[4 + rr] = load_stream(base_b + lane_off_v + 4 * rr * kD * 2);
        return;
    }
    const uint32_t oa = (uint32_t)pa * page_bytes + lane_off_v, ob = (uint32_t)pb * page_bytes + lane_off_v;
#pragma unroll
    for (int rr = 0; rr < 4; ++rr) v[rr] = load_stream(pool + oa + 4 * rr * kD * 2);
#pragma unroll
    for (int rr = 0; rr < 4; ++rr) v[4 + rr] = load_stream(pool + ob + 4 * rr * kD * 2);
}

struct WaveState {
    f32x16_t o[2][4];   // O^T accumulators: [row block][d block]; lane column = query row
    float m[2];         // row maximum in use (log2 units), per row block
    float l[2];         // this lane's share of the row sum
};

// P = 2^(S - m) of one 32-row block, its row sums, and O^T += V^T . P^T.
__device__ __forceinline__ void exp_and_pv(WaveState& st, f32x16_t& s, const int rb, const char* vbase) {
    float sum = 0.f;
#pragma unroll
    for (int i = 0; i < 16; ++i) {
        s[i] = __builtin_amdgcn_exp2f(s[i] - st.m[rb]);
        sum += s[i];
    }
    st.l[rb] += sum;
    bf16x8_t pb[2];
#pragma unroll
    for (int ks = 0; ks < 2; ++ks) {
        uint4 w;
        w.x = pack_bf16x2(s[8 * ks + 0], s[8 * ks + 1]);
        w.y = pack_bf16x2(s[8 * ks + 2], s[8 * ks + 3]);
        w.z = pack_bf16x2(s[8 * ks + 4], s[8 * ks + 5]);
        w.w = pack_bf16x2(s[8 * ks + 6], s[8 * ks + 7]);
        pb[ks] = __builtin_bit_cast(bf16x8_t, w);
    }
#pragma unroll
    for (int ks = 0; ks < 2; ++ks) {
        // keep the second half's operand reads below the first half's MFMAs (fewer live registers)
        if (ks == 1) __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int db = 0; db < 4; ++db) {
            const char* p0 = vbase + (16 * ks) * kVRowBytes + 64 * db;
            const s16x4_t lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4_t*)(p0));
            const s16x4_t hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4_t*)(p0 + 8 * kVRowBytes));
            const s16x8_t both = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
            st.o[rb][db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8_t, both), pb[ks],
                                                                   st.o[rb][db], 0, 0, 0);
        }
    }
}

// Softmax and PV of one 32-row block of a tile whose scores are in `s`.  The accumulators are only
// rescaled when some row's maximum outgrows the one in use by more than the threshold (always on a
// wave's first tile).
__device__ __forceinline__ void softmax_pv(WaveState& st, f32x16_t& s, const int rb, const char* vbase) {
    float t = s[0];
#pragma unroll
    for (int i = 1; i < 16; ++i) t = fmaxf(t, s[i]);
    const float tmax = fmaxf(t, __shfl_xor(t, 32, 64));
    const bool grow = tmax > st.m[rb] + kRescaleThreshold;
    if (__any(grow)) {
        const float mn = grow ? tmax : st.m[rb];
        const float f = __builtin_amdgcn_exp2f(st.m[rb] - mn);  // 2^-inf = 0 on the first tile
        st.m[rb] = mn;
        st.l[rb] *= f;
#pragma unroll
        for (int db = 0; db < 4; ++db)
#pragma unroll
            for (int i = 0; i < 16; ++i) st.o[rb][db][i] *= f;
    }
    exp_and_pv(st, s, rb, vbase);
}

// S^T block = K . Q^T for the 32 query rows of row block rb.
__device__ __forceinline__ void qk_block(f32x16_t& s, const uint4 (&k)[8], const char* qbase, const int rb) {
#pragma unroll
    for (int i = 0; i < 16; ++i) s[i] = 0.f;
#pragma unroll
    for (int kk = 0; kk < 8; ++kk) {
        // at most four Q operands in registers at a time
        if (kk == 4) __builtin_amdgcn_sched_barrier(0);
        const bf16x8_t qb =
            __builtin_bit_cast(bf16x8_t, *reinterpret_cast<const uint4*>(qbase + rb * 32 * kQRowBytes + 32 * kk));
        s = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8_t, k[kk]), qb, s, 0, 0, 0);
    }
}

// Same with the K operand read from an LDS tile (row stride kQRowBytes) instead of registers.
__device__ __forceinline__ void qk_block_lds(f32x16_t& s, const char* kbase, const char* qbase, const int rb) {
#pragma unroll
    for (int i = 0; i < 16; ++i) s[i] = 0.f;
#pragma unroll
    for (int kk = 0; kk < 8; ++kk) {
        const bf16x8_t ka = __builtin_bit_cast(bf16x8_t, *reinterpret_cast<const uint4*>(kbase + 32 * kk));
        const bf16x8_t qb =
            __builtin_bit_cast(bf16x8_t, *reinterpret_cast<const uint4*>(qbase + rb * 32 * kQRowBytes + 32 * kk));
        s = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ka, qb, s, 0, 0, 0);
    }
}

// Accumulator i of a lane holds token 8 (i / 4) + 4 (lane / 32) + i % 4 of the tile.
__device__ __forceinline__ void mask_tail(f32x16_t& s, int valid, int hf) {
#pragma unroll
    for (int i = 0; i < 16; ++i)
        if (8 * (i >> 2) + 4 * hf + (i & 3) >= valid) s[i] = -INFINITY;
}

// Visibility of the in-flight tile (token j = in-flight query/key j): a row sees tokens below `lim`
// and token `self` (lim = min(ctx, n_q), self = its own query index; padding rows: lim 0, self 0).
__device__ __forceinline__ void mask_inflight(f32x16_t& s, int lim, int self, int hf) {
#pragma unroll
    for (int i = 0; i < 16; ++i) {
        const int tok = 8 * (i >> 2) + 4 * hf + (i & 3);
        s[i] = (tok < lim || tok == self) ? s[i] : -INFINITY;
    }
}

// Closing a (sequence, KV head) pair: the workgroup that finished its share last keeps its own merged
// state in registers (`own`, laid out as the LDS merge leaves it: wave w, pass p, u holds register
// group reg4 = 16 (w / 4) + 4 (2 p + (w / 2) % 2) + 2 (w % 2) + u of row block w / 4), reads the other
// partials p_begin .. p_end of the pair, folds everything in partial-index order (so the result does
// not depend on who closes), normalises and writes the bf16 output rows.  Partials are taken four
// at a time so that their loads overlap.
__device__ __forceinline__ void close_pair(const MfmaArgs& a, int q0, int n_rows, int b, int g, int p_begin, int p_end,
                                           int p_own, const float4 (&own)[2][2], float own_m, float own_l, int w, int lane) {
    const int rb = w >> 2, d2 = (w >> 1) & 1, i4b = 2 * (w & 1), l32 = lane & 31, hf = lane >> 5;
    const int row = 32 * rb + l32;
    float m = -INFINITY, lsum = 0.f;
    float4 o[2][2];
#pragma unroll
    for (int ps = 0; ps < 2; ++ps)
#pragma unroll
        for (int u = 0; u < 2; ++u) o[ps][u] = make_float4(0.f, 0.f, 0.f, 0.f);
    const __amdgpu_buffer_rsrc_t rs = partials_descriptor(a.ws);
    constexpr int kBatch = 8;   // partials requested together: one memory round trip per batch
    for (int p0 = p_begin; p0 < p_end; p0 += kBatch) {
        float pm[kBatch], pl[kBatch];
        float4 px[kBatch][2][2];
#pragma unroll
        for (int k = 0; k < kBatch; ++k) {
            const int p = p0 + k;
            if (p < p_end && p != p_own) {
                const uint32_t base = (uint32_t)(((size_t)p * a.n_kv_heads + g) * kPartFloats * sizeof(float));
                const float* part = a.ws + ((size_t)p * a.n_kv_heads + g) * kPartFloats;
                pm[k] = load_coherent(part + row);
                pl[k] = load_coherent(part + kRows + row);
#pragma unroll
                for (int ps = 0; ps < 2; ++ps)
#pragma unroll
                    for (int u = 0; u < 2; ++u)
                        px[k][ps][u] = load_coherent4(rs, base + (2 * kRows + ((rb * 16 + (2 * ps + d2) * 4 + i4b + u) * 64 + lane) * 4) * 4);
            } else {
                const bool mine = p == p_own;
                pm[k] = mine ? own_m : -INFINITY;   // past the end: weight 2^-inf = 0
                pl[k] = mine ? own_l : 0.f;
#pragma unroll
                for (int ps = 0; ps < 2; ++ps)
#pragma unroll
                    for (int u = 0; u < 2; ++u) px[k][ps][u] = mine ? own[ps][u] : make_float4(0.f, 0.f, 0.f, 0.f);
            }
        }
#pragma unroll
        for (int k = 0; k < kBatch; ++k) {
            if (p0 + k >= p_end) continue;                          // (uniform) nothing in this slot
            const float mn = fmaxf(m, pm[k]);                       // the first partial exists and is finite
            const float fo = __builtin_amdgcn_exp2f(m - mn);
            const float fp = __builtin_amdgcn_exp2f(pm[k] - mn);
            m = mn;
            lsum = lsum * fo + pl[k] * fp;
#pragma unroll
            for (int ps = 0; ps < 2; ++ps)
#pragma unroll
                for (int u = 0; u < 2; ++u) {
                    o[ps][u].x = o[ps][u].x * fo + px[k][ps][u].x * fp;
                    o[ps][u].y = o[ps][u].y * fo + px[k][ps][u].y * fp;
                    o[ps][u].z = o[ps][u].z * fo + px[k][ps][u].z * fp;
                    o[ps][u].w = o[ps][u].w * fo + px[k][ps][u].w * fp;
                }
        }
    }
    if (row < n_rows) {
        const float inv = 1.f / lsum;
        uint16_t* op = a.out + (((size_t)b * a.n_q + q0 + row / a.group) * a.n_q_heads + g * a.group + row % a.group) * kD;
#pragma unroll
        for (int ps = 0; ps < 2; ++ps)
#pragma unroll
            for (int u = 0; u < 2; ++u) {
                // register group -> d = 32 (2 ps + d2) + 8 (i4b + u) + 4 (lane / 32) .. + 4
                uint2 pk;
                pk.x = pack_bf16x2(o[ps][u].x * inv, o[ps][u].y * inv);
                pk.y = pack_bf16x2(o[ps][u].z * inv, o[ps][u].w * inv);
                *reinterpret_cast<uint2*>(op + 32 * (2 * ps + d2) + 8 * (i4b + u) + 4 * hf) = pk;
            }
    }
}

// Next tile of the segment for the calling wave: one lane bumps the workgroup's counter in LDS.
__device__ __forceinline__ int claim_tile(int* counter, int lane) {
    int v = 0;
    if (lane == 0) v = __hip_atomic_fetch_add(counter, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
    return __builtin_amdgcn_readfirstlane(v);
}

// kWide: see the LDS map.  kClaim: the waves of a workgroup take the segment's tiles first come,
// first served instead of every 8th tile each; this evens out the waves' finishing times, at the
// price of results that depend on the order the tiles happened to be taken in (rounding only).
template <bool kClaim, bool kBigPool = false>
__global__ __launch_bounds__(kThreads) void pv_attn_mfma_stream(MfmaArgs a) {
    extern __shared__ __attribute__((aligned(16))) char smem[];
    typedef Lds L;
    const int q0 = 0, n_qc = a.n_q;
    const int item = blockIdx.x, g = blockIdx.y;
    const int tid = threadIdx.x;
    const int w = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int lane = tid & 63, hf = lane >> 5, l32 = lane & 31, l16 = lane & 15;
    const int n_rows = n_qc * a.group;
    char* vl = smem + L::kV + w * kVTileBytes;
    float2* cs_tab = reinterpret_cast<float2*>(smem + L::kCs);
    // V^T operand addressing.  Within a 16-lane group the transposing load gives lane i, element j
    // the value M[4 j + i / 4][i % 4] of the 16 x 4 block whose row r is addressed by lane r.
    // Source lane r points at token T[r / 4], columns d0 + 4 (r % 4) .. + 4, so result lane i holds
    // V[T[0..3]][d0 + i]; T[j] = 16 ks + 8 w + 4 (lane / 32) + j matches the k-order of P^T, whose
    // operand element 4 w + j is score accumulator 8 ks + 4 w + j.
    const char* vbase = vl + (4 * hf + (l16 >> 2)) * kVRowBytes + (16 * ((lane >> 4) & 1) + 4 * (l16 & 3)) * 2;
    // Q^T operand: column = query row 32 rb + lane % 32, k = 16 kk + 8 (lane / 32) .. + 8
    const char* qbase = smem + L::kQ + l32 * kQRowBytes + 16 * hf;
    char* vwrite = vl + (lane >> 4) * kVRowBytes + l16 * 16;
    // byte offsets inside a page: K operand row = token lane % 16 of the page, 16 bytes at d = 8 (lane / 32);
    // V row = token lane / 16 (+ 4 rr), 16 bytes at d = 8 (lane % 16)
    const char* pool = reinterpret_cast<const char*>(a.pool_layer);
    const uint32_t page_bytes = (uint32_t)a.page_elems * 2;
    const uint32_t lane_off_k = ((uint32_t)g * 2 * MS_PAGE_SIZE * kD + (lane & 15) * kD + 8 * hf) * 2;
    const uint32_t lane_off_v = (((uint32_t)g * 2 + 1) * MS_PAGE_SIZE * kD + (lane >> 4) * kD + 8 * l16) * 2;
    // The item's first segment record also holds the item's segment range and the page ids of the
    // first tiles, so the first loads depend on this one record only.
    const float inv_f = a.inv_freq[lane];   // rotation pair `lane`; issued before anything else
    const int seg_begin = uniform_load(&a.item_first[item].seg_begin), seg_end = uniform_load(&a.item_first[item].seg_end);
    for (int si = seg_begin; si < seg_end; ++si) {
        const Seg* sp = si == seg_begin ? a.item_first + item : a.segs + si;
        const int sg_b = uniform_load(&sp->b), sg_t0 = uniform_load(&sp->t0), sg_part = uniform_load(&sp->part);
        const int sg_seq = uniform_load(&sp->seq);
        const int* pt = a.d_pt + (size_t)sg_seq * a.max_pages;
        // The plan was cut from the lengths the host knew.  Rows committed on the device since then
        // (the host has not been told how many) belong to the sequence's last segment, the one that
        // ended at the length the plan knew: it runs to the length the device holds.
        const int len_plan = uniform_load(&sp->len), t1_plan = uniform_load(&sp->t1);
        const int len_dev = uniform_load(a.d_len + sg_seq);
        const int last_page = (len_dev - 1) >> 4;
        const int n_tok = (t1_plan == len_plan ? len_dev : t1_plan) - sg_t0;
        const int n_tiles = (n_tok + kTile - 1) / kTile;
        const bool first_seg = sg_t0 == 0;   // this workgroup also runs the sequence's in-flight tile
        int pa = uniform_load(&sp->pages[2 * w]), pb = uniform_load(&sp->pages[2 * w + 1]);
        // the record's page ids hold for tiles below the last page the plan knew; a first tile that
        // reaches past it is looked up in the page table (written by the device-side commit)
        if (len_dev != len_plan && (sg_t0 >> 4) + 2 * w + 1 > ((len_plan - 1) >> 4)) tile_pages(pt, w, n_tiles, sg_t0, last_page, pa, pb);

        // ---- set-up loads.  Order matters: waiting for a load also waits for every load issued
        // before it, so the small loads the Q rotation needs go first and this wave's first tile
        // (16 loads, left in flight) goes last.  Thread t owns query row t / 8, rotation pairs
        // 8 (t % 8) .. + 8; in a first segment, threads below 256 do the same for in-flight key t / 8
        // (keys and queries share position ids, hence one cos/sin table).
        // (lane-derived values of the set-up and merge phases are rebuilt from an opaque copy of the
        // thread id, so that they are not computed at kernel entry and kept -- or spilled -- across
        // the stream loop)
        int tid_p = tid;
        asm volatile("" : "+v"(tid_p));
        const int qr = tid_p >> 3, qc = tid_p & 7;
        // all of these loads are unconditional (out-of-range rows read row 0 and are zeroed by their
        // rotation factors) so that the number of loads in flight is known and waits stay partial
        const int qi = q0 + (qr < n_rows ? qr / a.group : 0);
        const int qh = qr < n_rows ? qr % a.group : 0;
        const uint16_t* qp = a.q + (((size_t)sg_b * a.n_q + qi) * a.n_q_heads + g * a.group + qh) * kD + 8 * qc;
        const uint4 x0v = *reinterpret_cast<const uint4*>(qp);
        const uint4 x1v = *reinterpret_cast<const uint4*>(qp + 64);
        const uint16_t* kp = a.k_new + (((size_t)sg_b * a.n_q + (qr < a.n_q ? qr : 0)) * a.n_kv_heads + g) * kD + 8 * qc;
        const uint4 k0v = *reinterpret_cast<const uint4*>(kp);
        const uint4 k1v = *reinterpret_cast<const uint4*>(kp + 64);
        // position ids of queries w, w + 8, ... (wave-uniform: scalar loads)
        constexpr int kPosPerWave = L::kQueries / kWaves;
        int pos_w[kPosPerWave];
#pragma unroll
        for (int k = 0; k < kPosPerWave; ++k) pos_w[k] = w + 8 * k < a.n_q ? uniform_load(a.pos + sg_b * a.n_q + w + 8 * k) : 0;
        TileRegs r;   // (an empty segment's record names page 0: loaded, never used)
        load_v<kBigPool>(r.v, pool, pa, pb, page_bytes, lane_off_v);
        load_k<kBigPool>(r.k, pool, pa, pb, page_bytes, lane_off_k, lane);
        int* tile_counter = reinterpret_cast<int*>(smem + L::kFlag + 4);
        if (kClaim && tid_p == 0) *tile_counter = kWaves;   // tiles 0 .. 7 are the waves' first ones
        // cos/sin table: wave w fills the rows of queries w, w + 8, ..., lane = rotation pair
#pragma unroll
        for (int k = 0; k < kPosPerWave; ++k)
            if (w + 8 * k < a.n_q) {
                float sn, cs;
                sincos_reduced((float)pos_w[k] * inv_f, &sn, &cs);
                cs_tab[(w + 8 * k) * 64 + (tid_p & 63)] = make_float2(cs, sn);
            }
        lds_barrier();
        {
            const uint32_t w0[4] = {x0v.x, x0v.y, x0v.z, x0v.w}, w1[4] = {x1v.x, x1v.y, x1v.z, x1v.w};
            const uint32_t u0[4] = {k0v.x, k0v.y, k0v.z, k0v.w}, u1[4] = {k1v.x, k1v.y, k1v.z, k1v.w};
            uint32_t y0[4], y1[4], z0[4], z1[4];
#pragma unroll
            for (int e2 = 0; e2 < 4; ++e2) {
                float r0[2], r1[2], s0[2], s1[2];
#pragma unroll
                for (int hh = 0; hh < 2; ++hh) {
                    const float x0 = hh ? __uint_as_float(w0[e2] & 0xffff0000u) : __uint_as_float(w0[e2] << 16);
                    const float x1 = hh ? __uint_as_float(w1[e2] & 0xffff0000u) : __uint_as_float(w1[e2] << 16);
                    const float2 c = qr < n_rows ? cs_tab[qi * 64 + 8 * qc + 2 * e2 + hh] : make_float2(0.f, 0.f);
                    r0[hh] = (x0 * c.x - x1 * c.y) * a.scale_log2;
                    r1[hh] = (x1 * c.x + x0 * c.y) * a.scale_log2;
                    const float k0 = hh ? __uint_as_float(u0[e2] & 0xffff0000u) : __uint_as_float(u0[e2] << 16);
                    const float k1 = hh ? __uint_as_float(u1[e2] & 0xffff0000u) : __uint_as_float(u1[e2] << 16);
                    const float2 ck = qr < a.n_q ? cs_tab[qr * 64 + 8 * qc + 2 * e2 + hh] : make_float2(0.f, 0.f);
                    s0[hh] = k0 * ck.x - k1 * ck.y;
                    s1[hh] = k1 * ck.x + k0 * ck.y;
                }
                y0[e2] = pack_bf16x2(r0[0], r0[1]);
                y1[e2] = pack_bf16x2(r1[0], r1[1]);
                z0[e2] = pack_bf16x2(s0[0], s0[1]);
                z1[e2] = pack_bf16x2(s1[0], s1[1]);
            }
            char* qrow = smem + L::kQ + qr * kQRowBytes + 16 * qc;
            *reinterpret_cast<uint4*>(qrow) = make_uint4(y0[0], y0[1], y0[2], y0[3]);
            *reinterpret_cast<uint4*>(qrow + 128) = make_uint4(y1[0], y1[1], y1[2], y1[3]);
            if (first_seg && qr < L::kNewTiles * kTile) {   // rows at and past n_q are zeros
                char* krow = smem + L::kKn + qr * kQRowBytes + 16 * qc;
                *reinterpret_cast<uint4*>(krow) = make_uint4(z0[0], z0[1], z0[2], z0[3]);
                *reinterpret_cast<uint4*>(krow + 128) = make_uint4(z1[0], z1[1], z1[2], z1[3]);
            }
        }
        lds_barrier();
        WaveState st;
#pragma unroll
        for (int rb = 0; rb < 2; ++rb) {
            st.m[rb] = -INFINITY;
            st.l[rb] = 0.f;
#pragma unroll
            for (int db = 0; db < 4; ++db)
#pragma unroll
                for (int i = 0; i < 16; ++i) st.o[rb][db][i] = 0.f;
        }

        // ---- the in-flight tile: the step's own keys and values, visibility rule on the scores;
        // run by the last wave (it has the fewest stream tiles) of the first segment's workgroup,
        // ahead of the stream so that nothing it needs stays live across the stream loop ----
        if (first_seg && w == kWaves - 1) {
            int ln = lane;
            asm volatile("" : "+v"(ln));
            const int l16 = ln & 15, l32 = ln & 31, hf = ln >> 5;
            const int new_tiles = 1;
            for (int it = 0; it < new_tiles; ++it) {
#pragma unroll
                for (int rr = 0; rr < 8; ++rr) {
                    const int tok = kTile * it + 4 * rr + (ln >> 4);
                    const int tc = tok < a.n_q ? tok : a.n_q - 1;   // clamped: the load is unconditional
                    const uint4 val = *reinterpret_cast<const uint4*>(a.v_new + (((size_t)sg_b * a.n_q + tc) * a.n_kv_heads + g) * kD + 8 * l16);
                    *reinterpret_cast<uint4*>(vwrite + 4 * rr * kVRowBytes) = tok < a.n_q ? val : make_uint4(0, 0, 0, 0);
                }
#pragma unroll
                for (int rb = 0; rb < 2; ++rb) {
                    const int row = 32 * rb + l32;
                    const bool pad_row = row >= n_rows;
                    const int i = q0 + (pad_row ? 0 : row / a.group);
                    int ctx = a.ctx_new ? a.ctx_new[sg_b * a.n_q + i] : (i < a.n_verify ? i : a.n_verify);
                    ctx = pad_row ? 0 : (ctx < a.n_q ? ctx : a.n_q);
                    f32x16_t s;
                    qk_block_lds(s, smem + L::kKn + (kTile * it + l32) * kQRowBytes + 16 * hf, qbase, rb);
                    // a tile none of whose tokens a row may see leaves that row's state untouched:
                    // its scores are all minus infinity and its running maximum is already finite
                    // or, on the first tile, made finite by the row's own token or an earlier one
                    mask_inflight(s, ctx - kTile * it, i - kTile * it, hf);
                    softmax_pv(st, s, rb, vbase);
                }
            }
        }

        // ---- the stream: full tiles w, w + 8, ...; the next tile's loads are issued as soon as the
        // registers of the current one have been consumed.  Refills are unconditional (clamped to
        // the last tile), so a wave leaves the loop holding its next tile -- the segment's partial
        // tail tile, if that one is its to do ----
        const int full_tiles = n_tok / kTile;
        int cur = w;   // every wave's first tile is fixed: its loads were issued during the set-up
        for (int turn = 0; cur < full_tiles; ++turn) {
            int nxt = cur + kWaves;
            if (kClaim) nxt = claim_tile(tile_counter, lane);
            // the two waves of a SIMD take turns at the higher issue priority, tile by tile; with
            // equal priorities the older wave always wins and the younger one finishes late
            if ((turn ^ (w >> 2)) & 1) __builtin_amdgcn_s_setprio(1);
            else __builtin_amdgcn_s_setprio(0);
#pragma unroll
            for (int rr = 0; rr < 8; ++rr) *reinterpret_cast<uint4*>(vwrite + 4 * rr * kVRowBytes) = r.v[rr];
            tile_pages(pt, nxt, n_tiles, sg_t0, last_page, pa, pb);
            load_v<kBigPool>(r.v, pool, pa, pb, page_bytes, lane_off_v);
            f32x16_t s;
            qk_block(s, r.k, qbase, 0);
            softmax_pv(st, s, 0, vbase);
            qk_block(s, r.k, qbase, 1);
            load_k<kBigPool>(r.k, pool, pa, pb, page_bytes, lane_off_k, lane);
            softmax_pv(st, s, 1, vbase);
            cur = nxt;
        }
        __builtin_amdgcn_s_setprio(0);
        // ---- the tail tile (fewer than 32 tokens), for the wave whose next tile it is: V rows past
        // the end become zeros, their scores minus infinity ----
        if (full_tiles < n_tiles && cur == full_tiles) {
            const int valid = n_tok - full_tiles * kTile;
#pragma unroll
            for (int rr = 0; rr < 8; ++rr)
                *reinterpret_cast<uint4*>(vwrite + 4 * rr * kVRowBytes) =
                    4 * rr + (lane >> 4) < valid ? r.v[rr] : make_uint4(0, 0, 0, 0);
#pragma unroll
            for (int rb = 0; rb < 2; ++rb) {
                f32x16_t s;
                qk_block(s, r.k, qbase, rb);
                mask_tail(s, valid, hf);
                softmax_pv(st, s, rb, vbase);
            }
        }

        // ---- merge the waves' states through LDS (overlays the stream buffers), two d blocks per
        // pass: every wave stores its 64 registers of the pair, then wave w reduces two float4 per
        // lane over all waves and writes them to the segment's partial ----
        float* part = a.ws + ((size_t)sg_part * a.n_kv_heads + g) * kPartFloats;
        const int p_begin = uniform_load(a.part_begin + sg_b), p_end = uniform_load(a.part_begin + sg_b + 1);
        int* ctr = a.arrive + 2 * (sg_b * a.n_kv_heads + g);   // [0] shares finished, [1] partials published
        int lane_m = lane;
        asm volatile("" : "+v"(lane_m));
        int ticket = 0;
        float4 own[2][2];
        float own_m = 0.f, own_l = 0.f;
#pragma unroll
        for (int pass = 0; pass < 2; ++pass) {
            lds_barrier();
            // every wave has left the stream: take this share's place in the pair's finishing order.
            // The answer is not needed before the merge is done, which hides the round trip.
            if (pass == 0 && tid == 0) ticket = __hip_atomic_fetch_add(ctr, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            {
                float* reg = reinterpret_cast<float*>(smem + w * kMergeRegionBytes);
#pragma unroll
                for (int rb = 0; rb < 2; ++rb)
#pragma unroll
                    for (int d2 = 0; d2 < 2; ++d2)
#pragma unroll
                        for (int i4 = 0; i4 < 4; ++i4) {
                            const f32x16_t& o = st.o[rb][2 * pass + d2];
                            *reinterpret_cast<float4*>(reg + (((rb * 2 + d2) * 4 + i4) * 64 + lane_m) * 4) =
                                make_float4(o[4 * i4], o[4 * i4 + 1], o[4 * i4 + 2], o[4 * i4 + 3]);
                        }
                if (pass == 0)
                    *reinterpret_cast<float4*>(reg + (16 * 64 + lane_m) * 4) = make_float4(st.m[0], st.m[1], st.l[0], st.l[1]);
            }
            lds_barrier();
            {
                // wave w reduces slots 2 w and 2 w + 1 of the 16: slot = (rb * 2 + d2) * 4 + i4
                const int rb = w >> 2;
                float mn = -INFINITY;    // some wave had a tile (or the in-flight tile): finite
                float mo[kWaves], lo[kWaves];
#pragma unroll
                for (int ow = 0; ow < kWaves; ++ow) {
                    const float4 ml = *reinterpret_cast<const float4*>(smem + ow * kMergeRegionBytes + (16 * 64 + lane_m) * 16);
                    mo[ow] = rb ? ml.y : ml.x;
                    lo[ow] = rb ? ml.w : ml.z;
                    mn = fmaxf(mn, mo[ow]);
                }
                float4 acc[2];
                acc[0] = acc[1] = make_float4(0.f, 0.f, 0.f, 0.f);
                float lt = 0.f;
#pragma unroll
                for (int ow = 0; ow < kWaves; ++ow) {
                    const float f = __builtin_amdgcn_exp2f(mo[ow] - mn);   // idle wave: 2^-inf = 0
                    lt += f * lo[ow];
#pragma unroll
                    for (int u = 0; u < 2; ++u) {
                        const float4 x =
                            *reinterpret_cast<const float4*>(smem + ow * kMergeRegionBytes + ((2 * w + u) * 64 + lane_m) * 16);
                        acc[u].x += f * x.x;
                        acc[u].y += f * x.y;
                        acc[u].z += f * x.z;
                        acc[u].w += f * x.w;
                    }
                }
                own[pass][0] = acc[0];
                own[pass][1] = acc[1];
                if (pass == 0) {
                    own_m = mn;
                    own_l = lt + __shfl_xor(lt, 32, 64);   // the two half-waves hold the two halves of a row's sum
                }
            }
        }
        // ---- closing the pair.  The share that finished last (by ticket) folds the others' partials
        // into its registers and writes the output; every other share publishes its partial.  The
        // closing workgroup only ever waits for workgroups that took their ticket before it, and those
        // publish without waiting for anything, so the wait is bounded by their store latency ----
        if (tid == 0) *reinterpret_cast<volatile int*>(smem + L::kFlag) = ticket;
        lds_barrier();
        const bool closing = *reinterpret_cast<volatile int*>(smem + L::kFlag) == p_end - p_begin - 1;
        if (!closing) {
            const int rb = w >> 2;
            const __amdgpu_buffer_rsrc_t rs = partials_descriptor(a.ws);
            const uint32_t base = (uint32_t)(((size_t)sg_part * a.n_kv_heads + g) * kPartFloats * sizeof(float));
#pragma unroll
            for (int pass = 0; pass < 2; ++pass)
#pragma unroll
                for (int u = 0; u < 2; ++u) {
                    const int slot = 2 * w + u, d2 = (slot >> 2) & 1, i4 = slot & 3;
                    const int reg4 = rb * 16 + (2 * pass + d2) * 4 + i4;
                    store_coherent4(rs, base + (2 * kRows + (reg4 * 64 + lane_m) * 4) * 4, own[pass][u]);
                }
            if ((w & 3) == 0 && (lane_m >> 5) == 0) {
                store_coherent(part + 32 * rb + (lane_m & 31), own_m);
                store_coherent(part + kRows + 32 * rb + (lane_m & 31), own_l);
            }
            __syncthreads();   // waits for every thread's partial stores
            if (tid == 0) __hip_atomic_fetch_add(ctr + 1, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        } else {
            if (tid == 0) {
                const int others = p_end - p_begin - 1;
                // The wait ends when the shares that took their tickets earlier have published; they
                // wait for nothing, so this takes a few microseconds.  The bound (about a second by
                // default) only guards against counters left in a bad state: then nothing is folded
                // from the workspace, the output rows of the pair stay unwritten, and the host is
                // told through the error word -- the next call on the cache fails and resets them.
                int seen = __hip_atomic_load(ctr + 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                for (int spin = 0; spin < a.poll_limit && seen != others; ++spin) {
                    __builtin_amdgcn_s_sleep(2);
                    seen = __hip_atomic_load(ctr + 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                }
                const bool complete = seen == others;
                if (complete) {
                    __hip_atomic_store(ctr, 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);       // ready for the next call
                    __hip_atomic_store(ctr + 1, 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                } else {
                    __hip_atomic_store(a.error_word, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM);
                }
                *reinterpret_cast<volatile int*>(smem + L::kFlag + 8) = complete ? 1 : 0;
            }
            lds_barrier();
            asm volatile("" ::: "memory");   // the partials are read after the wait, also in the compiler's order
            if (*reinterpret_cast<volatile int*>(smem + L::kFlag + 8))
                close_pair(a, q0, n_rows, sg_b, g, p_begin, p_end, sg_part, own, own_m, own_l, w, lane_m);
        }
        lds_barrier();  // the next segment reuses the LDS
    }
}


// ---------------------------------------------------------------------------------------------
// Wide steps: more than 16 queries or more than 64 rows per KV head (the memory-token pass of a
// closed step with its l + 1 causal queries, prompt chunks, per-position foresight).
//
// The queries are cut into chunks of 64 / group queries (at most 64 rows) and wave w of a workgroup
// owns chunk w: its rotated Q rows are its Q^T operand (rows 0 .. 31 in registers, rows 32 .. 63 in
// a wave-private LDS tile: both in registers do not fit beside the accumulators), its O^T
// accumulators are its own.  All eight waves walk over the SAME tiles of the share, so a tile leaves HBM once per
// call however many queries there are: the 512 threads load a tile's K and V rows together (16
// bytes of each per thread, one tile ahead, through registers) into a double-buffered pair of LDS
// tiles, one workgroup barrier per tile.  With eight times the arithmetic per byte the stream is
// bound by the matrix cores and LDS, not by HBM.  No wave shares rows with another, so there is no
// merge at the end: every wave leaves (or folds) the partial of its own chunk.  The work plan, the
// tickets and the page handling are the decode kernel's.  Results do not depend on timing.
// ---------------------------------------------------------------------------------------------
struct WideLds {
    static constexpr int kCs = 0;                                   // cos/sin of every query's position id: 32768
    static constexpr int kKn = kCs + MS_MAX_QUERIES * 64 * 8;       // rotated in-flight keys, two tiles: 17408
    static constexpr int kQ1 = kKn + 2 * kTile * kQRowBytes;        // every wave's rotated Q rows 32 .. 63: 69632
    static constexpr int kK = kQ1 + kWaves * kTile * kQRowBytes;    // K tiles, two buffers: 17408
    static constexpr int kV = kK + 2 * kTile * kQRowBytes;          // V tiles, two buffers: 20480
    static constexpr int kFlag = kV + 2 * kVTileBytes;
    static constexpr int kBytes = kFlag + 16;
    static_assert(kBytes <= 160 * 1024, "LDS budget of one compute unit");
};
constexpr int kWideChunks = kWaves;   // chunks per launch: one per wave

// S^T block = K . Q^T with K read from an LDS tile and the Q^T operand held in registers.
// The K operands are asked for two ahead of their use: one LDS round trip per multiplication would
// otherwise be all a wave does.
__device__ __forceinline__ void qk_block_qreg(f32x16_t& s, const char* kbase, const bf16x8_t (&q)[8]) {
#pragma unroll
    for (int i = 0; i < 16; ++i) s[i] = 0.f;
    uint4 ka[8];
#pragma unroll
    for (int kk = 0; kk < 2; ++kk) ka[kk] = *reinterpret_cast<const uint4*>(kbase + 32 * kk);
#pragma unroll
    for (int kk = 0; kk < 8; ++kk) {
        if (kk + 2 < 8) ka[kk + 2] = *reinterpret_cast<const uint4*>(kbase + 32 * (kk + 2));
        __builtin_amdgcn_sched_barrier(0);
        s = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8_t, ka[kk]), q[kk], s, 0, 0, 0);
    }
}

// Both operands from LDS (K tile rows, a wave's Q rows), one pair ahead of their use.
__device__ __forceinline__ void qk_block_lds2(f32x16_t& s, const char* kbase, const char* qbase) {
#pragma unroll
    for (int i = 0; i < 16; ++i) s[i] = 0.f;
    uint4 ka[8], qa[8];
    ka[0] = *reinterpret_cast<const uint4*>(kbase);
    qa[0] = *reinterpret_cast<const uint4*>(qbase);
#pragma unroll
    for (int kk = 0; kk < 8; ++kk) {
        if (kk + 1 < 8) {
            ka[kk + 1] = *reinterpret_cast<const uint4*>(kbase + 32 * (kk + 1));
            qa[kk + 1] = *reinterpret_cast<const uint4*>(qbase + 32 * (kk + 1));
        }
        __builtin_amdgcn_sched_barrier(0);
        s = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8_t, ka[kk]), __builtin_bit_cast(bf16x8_t, qa[kk]), s, 0, 0, 0);
    }
}

// 16 bytes of K and of V of one token of a tile, as one thread loads them.
struct WideStage {
    uint4 k, v;
};

__global__ __launch_bounds__(kThreads) void pv_attn_mfma_wide(MfmaArgs a) {
    extern __shared__ __attribute__((aligned(16))) char smem[];
    typedef WideLds L;
    const int item = blockIdx.x, g = blockIdx.y;
    const int tid = threadIdx.x;
    const int w = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int lane = tid & 63, hf = lane >> 5, l32 = lane & 31, l16 = lane & 15;
    // this wave's chunk of queries
    const int per = kRows / a.group;
    const int cq0 = a.q0 + w * per;
    const int cq_left = a.q0 + a.n_qc - cq0;
    const int cn = cq_left < 0 ? 0 : (cq_left < per ? cq_left : per);
    const int n_rows = cn * a.group;
    float2* cs_tab = reinterpret_cast<float2*>(smem + L::kCs);
    const char* pool = reinterpret_cast<const char*>(a.pool_layer);
    const size_t page_bytes = (size_t)a.page_elems * 2;
    // a thread's part of a tile: token tid / 16, 16 bytes at d = 8 (tid % 16)
    const int my_tok = tid >> 4, my_col = tid & 15;
    const uint32_t off_k = ((uint32_t)g * 2 * MS_PAGE_SIZE * kD + (my_tok & 15) * kD + 8 * my_col) * 2;
    const uint32_t off_v = off_k + MS_PAGE_SIZE * kD * 2;
    char* k_store = smem + L::kK + my_tok * kQRowBytes + my_col * 16;
    char* v_store = smem + L::kV + my_tok * kVRowBytes + my_col * 16;
    // operand addressing as in the decode kernel
    const char* k_read = smem + L::kK + l32 * kQRowBytes + 16 * hf;
    const char* v_read = smem + L::kV + (4 * hf + (l16 >> 2)) * kVRowBytes + (16 * ((lane >> 4) & 1) + 4 * (l16 & 3)) * 2;
    const float inv_f = a.inv_freq[lane];
    const int seg_begin = uniform_load(&a.item_first[item].seg_begin), seg_end = uniform_load(&a.item_first[item].seg_end);
    for (int si = seg_begin; si < seg_end; ++si) {
        const Seg* sp = si == seg_begin ? a.item_first + item : a.segs + si;
        const int sg_b = uniform_load(&sp->b), sg_t0 = uniform_load(&sp->t0), sg_part = uniform_load(&sp->part);
        const int sg_seq = uniform_load(&sp->seq);
        const int* pt = a.d_pt + (size_t)sg_seq * a.max_pages;
        const int len_plan = uniform_load(&sp->len), t1_plan = uniform_load(&sp->t1);
        const int len_dev = uniform_load(a.d_len + sg_seq);     // see the decode kernel: the device's length counts
        const int last_page = (len_dev - 1) >> 4;
        const int n_tok = (t1_plan == len_plan ? len_dev : t1_plan) - sg_t0;
        const int n_tiles = (n_tok + kTile - 1) / kTile;
        const bool first_seg = sg_t0 == 0;

        // page id of this thread's token of tile T (clamped: loads are unconditional and stay inside the sequence)
        auto page_of = [&](int T) {
            const int tc = T < n_tiles ? T : n_tiles - 1;
            const int pg = (sg_t0 >> 4) + 2 * tc + (my_tok >> 4);
            return pt[pg < last_page ? pg : last_page];
        };
        auto load_stage = [&](int page) {
            WideStage st_;
            const char* base = pool + (size_t)(uint32_t)page * page_bytes;
            st_.k = *reinterpret_cast<const uint4*>(base + off_k);
            st_.v = load_stream(base + off_v);
            return st_;
        };

        // ---- set-up: cos/sin of every query's position id (wave w: queries w, w + 8, ...), this
        // wave's raw Q rows, and for a sequence's first segment its in-flight keys ----
        WideStage sa;
        int pid_c = 0;
        if (n_tiles > 0) {
            const int p0 = page_of(0);
            pid_c = page_of(1);
            sa = load_stage(p0);
        }
        uint4 xq[2][8];
#pragma unroll
        for (int rb = 0; rb < 2; ++rb) {
            const int row = 32 * rb + l32;
            const bool live = row < n_rows;
            const int qi = cq0 + (live ? row / a.group : 0), qh = live ? row % a.group : 0;
            const uint16_t* qp = a.q + (((size_t)sg_b * a.n_q + (cn > 0 ? qi : 0)) * a.n_q_heads + g * a.group + qh) * kD + 8 * hf;
#pragma unroll
            for (int kk = 0; kk < 8; ++kk) xq[rb][kk] = *reinterpret_cast<const uint4*>(qp + 16 * kk);
        }
        const int kr = tid >> 3, kc = tid & 7;     // in-flight key kr, rotation pairs 8 kc .. + 8
        const uint16_t* kp = a.k_new + (((size_t)sg_b * a.n_q + (kr < a.n_q ? kr : 0)) * a.n_kv_heads + g) * kD + 8 * kc;
        const uint4 k0v = *reinterpret_cast<const uint4*>(kp);
        const uint4 k1v = *reinterpret_cast<const uint4*>(kp + 64);
#pragma unroll
        for (int k = 0; k < MS_MAX_QUERIES / kWaves; ++k)
            if (w + 8 * k < a.n_q) {
                float sn, cs;
                sincos_reduced((float)uniform_load(a.pos + sg_b * a.n_q + w + 8 * k) * inv_f, &sn, &cs);
                cs_tab[(w + 8 * k) * 64 + lane] = make_float2(cs, sn);
            }
        lds_barrier();
        // rotate: the lane holds elements 16 kk + 8 hf .. + 8 of its row; element i pairs with i + 64
        bf16x8_t qreg[8];
        char* q1_row = smem + L::kQ1 + (w * kTile + l32) * kQRowBytes + 16 * hf;
#pragma unroll
        for (int rb = 0; rb < 2; ++rb) {
            const int row = 32 * rb + l32;
            const bool live = row < n_rows;
            const int qi = cq0 + (live ? row / a.group : 0);
#pragma unroll
            for (int kk = 0; kk < 4; ++kk) {
                const uint32_t w0[4] = {xq[rb][kk].x, xq[rb][kk].y, xq[rb][kk].z, xq[rb][kk].w};
                const uint32_t w1[4] = {xq[rb][kk + 4].x, xq[rb][kk + 4].y, xq[rb][kk + 4].z, xq[rb][kk + 4].w};
                uint32_t y0[4], y1[4];
#pragma unroll
                for (int e2 = 0; e2 < 4; ++e2) {
                    float r0[2], r1[2];
#pragma unroll
                    for (int hh = 0; hh < 2; ++hh) {
                        const float x0 = hh ? __uint_as_float(w0[e2] & 0xffff0000u) : __uint_as_float(w0[e2] << 16);
                        const float x1 = hh ? __uint_as_float(w1[e2] & 0xffff0000u) : __uint_as_float(w1[e2] << 16);
                        const float2 c = live ? cs_tab[qi * 64 + 16 * kk + 8 * hf + 2 * e2 + hh] : make_float2(0.f, 0.f);
                        r0[hh] = (x0 * c.x - x1 * c.y) * a.scale_log2;
                        r1[hh] = (x1 * c.x + x0 * c.y) * a.scale_log2;
                    }
                    y0[e2] = pack_bf16x2(r0[0], r0[1]);
                    y1[e2] = pack_bf16x2(r1[0], r1[1]);
                }
                if (rb == 0) {
                    qreg[kk] = __builtin_bit_cast(bf16x8_t, make_uint4(y0[0], y0[1], y0[2], y0[3]));
                    qreg[kk + 4] = __builtin_bit_cast(bf16x8_t, make_uint4(y1[0], y1[1], y1[2], y1[3]));
                } else {
                    *reinterpret_cast<uint4*>(q1_row + 32 * kk) = make_uint4(y0[0], y0[1], y0[2], y0[3]);
                    *reinterpret_cast<uint4*>(q1_row + 32 * (kk + 4)) = make_uint4(y1[0], y1[1], y1[2], y1[3]);
                }
            }
        }
        if (first_seg) {   // the in-flight keys, rotated, as up to two K tiles (rows at and past n_q are zeros)
            const uint32_t u0[4] = {k0v.x, k0v.y, k0v.z, k0v.w}, u1[4] = {k1v.x, k1v.y, k1v.z, k1v.w};
            uint32_t z0[4], z1[4];
#pragma unroll
            for (int e2 = 0; e2 < 4; ++e2) {
                float s0[2], s1[2];
#pragma unroll
                for (int hh = 0; hh < 2; ++hh) {
                    const float x0 = hh ? __uint_as_float(u0[e2] & 0xffff0000u) : __uint_as_float(u0[e2] << 16);
                    const float x1 = hh ? __uint_as_float(u1[e2] & 0xffff0000u) : __uint_as_float(u1[e2] << 16);
                    const float2 ck = kr < a.n_q ? cs_tab[kr * 64 + 8 * kc + 2 * e2 + hh] : make_float2(0.f, 0.f);
                    s0[hh] = x0 * ck.x - x1 * ck.y;
                    s1[hh] = x1 * ck.x + x0 * ck.y;
                }
                z0[e2] = pack_bf16x2(s0[0], s0[1]);
                z1[e2] = pack_bf16x2(s1[0], s1[1]);
            }
            char* krow = smem + L::kKn + kr * kQRowBytes + 16 * kc;
            *reinterpret_cast<uint4*>(krow) = make_uint4(z0[0], z0[1], z0[2], z0[3]);
            *reinterpret_cast<uint4*>(krow + 128) = make_uint4(z1[0], z1[1], z1[2], z1[3]);
        }
        WaveState st;
#pragma unroll
        for (int rb = 0; rb < 2; ++rb) {
            // an in-flight tile may be wholly invisible to a row whose state is still empty: a finite
            // floor keeps 2^(s - m) at zero there instead of 2^(inf - inf)
            st.m[rb] = -1e30f;
            st.l[rb] = 0.f;
#pragma unroll
            for (int db = 0; db < 4; ++db)
#pragma unroll
                for (int i = 0; i < 16; ++i) st.o[rb][db][i] = 0.f;
        }

        // ---- the stream: every wave takes every tile.  Tile t is computed from LDS buffer t % 2
        // while tile t + 1 is on its way into registers ----
        if (n_tiles > 0) {
            *reinterpret_cast<uint4*>(k_store) = sa.k;
            *reinterpret_cast<uint4*>(v_store) = my_tok < n_tok ? sa.v : make_uint4(0, 0, 0, 0);
        }
        lds_barrier();
        for (int t = 0; t < n_tiles; ++t) {
            const int buf = t & 1;
            // the next tile's loads go out before this tile is computed and are stored behind it; the
            // page id after that is asked for first, so that waiting for it leaves the tile's loads in flight
            const int pid_n = page_of(t + 2);
            sa = load_stage(pid_c);          // tile t + 1
            pid_c = pid_n;
            const int valid = n_tok - t * kTile;
#pragma unroll
            for (int rb = 0; rb < 2; ++rb)
                if (32 * rb < n_rows) {
                    f32x16_t s;
                    if (rb == 0) qk_block_qreg(s, k_read + buf * (kTile * kQRowBytes), qreg);
                    else qk_block_lds2(s, k_read + buf * (kTile * kQRowBytes), q1_row);
                    if (valid < kTile) mask_tail(s, valid, hf);
                    softmax_pv(st, s, rb, v_read + buf * kVTileBytes);
                }
            // into the other buffer: every wave has finished with tile t - 1 (barrier of the last trip)
            *reinterpret_cast<uint4*>(k_store + (buf ^ 1) * (kTile * kQRowBytes)) = sa.k;
            *reinterpret_cast<uint4*>(v_store + (buf ^ 1) * kVTileBytes) =
                (t + 1) * kTile + my_tok < n_tok ? sa.v : make_uint4(0, 0, 0, 0);     // rows past the end: zeros (stale pool bytes may be NaN)
            lds_barrier();
        }
        // ---- the in-flight tiles (first segment only): keys from the rotated tiles, values from v_new,
        // the visibility rule on the scores ----
        if (first_seg) {
            const int new_tiles = (a.n_q + kTile - 1) / kTile;
            for (int it = 0; it < new_tiles; ++it) {
                const int tok = kTile * it + my_tok;
                const int tc = tok < a.n_q ? tok : a.n_q - 1;
                const uint4 val = *reinterpret_cast<const uint4*>(a.v_new + (((size_t)sg_b * a.n_q + tc) * a.n_kv_heads + g) * kD + 8 * my_col);
                *reinterpret_cast<uint4*>(v_store) = tok < a.n_q ? val : make_uint4(0, 0, 0, 0);
                lds_barrier();
#pragma unroll
                for (int rb = 0; rb < 2; ++rb)
                    if (32 * rb < n_rows) {
                        const int row = 32 * rb + l32;
                        const bool pad_row = row >= n_rows;
                        const int i = cq0 + (pad_row ? 0 : row / a.group);
                        int ctx = a.ctx_new ? a.ctx_new[sg_b * a.n_q + i] : (i < a.n_verify ? i : a.n_verify);
                        ctx = pad_row ? 0 : (ctx < a.n_q ? ctx : a.n_q);
                        f32x16_t s;
                        if (rb == 0) qk_block_qreg(s, smem + L::kKn + (kTile * it + l32) * kQRowBytes + 16 * hf, qreg);
                        else qk_block_lds2(s, smem + L::kKn + (kTile * it + l32) * kQRowBytes + 16 * hf, q1_row);
                        mask_inflight(s, ctx - kTile * it, i - kTile * it, hf);
                        softmax_pv(st, s, rb, v_read);
                    }
                lds_barrier();
            }
        }

        // ---- the pair's finishing order; this wave's chunk goes to, or is folded with, the partials
        // [partial][kv head][chunk]: m[64], l[64], then O as [row block][d block][4 registers][lane] ----
        const int p_begin = uniform_load(a.part_begin + sg_b), p_end = uniform_load(a.part_begin + sg_b + 1);
        int* ctr = a.arrive + 2 * (sg_b * a.n_kv_heads + g);
        int lane_t = lane;     // (an opaque copy: what the tail derives from the lane is not kept across the stream)
        asm volatile("" : "+v"(lane_t));
        const int lane = lane_t, hf = lane >> 5, l32 = lane & 31;
        if (tid == 0) *reinterpret_cast<volatile int*>(smem + L::kFlag) = __hip_atomic_fetch_add(ctr, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        float lsum[2];
#pragma unroll
        for (int rb = 0; rb < 2; ++rb) lsum[rb] = st.l[rb] + __shfl_xor(st.l[rb], 32, 64);   // the half-waves hold halves of a row's sum
        lds_barrier();
        const bool closing = *reinterpret_cast<volatile int*>(smem + L::kFlag) == p_end - p_begin - 1;
        const __amdgpu_buffer_rsrc_t rs = partials_descriptor(a.ws);
        auto part_floats = [&](int p) { return (((size_t)p * a.n_kv_heads + g) * kWideChunks + w) * kPartFloats; };
        if (!closing) {
            if (n_rows > 0) {
                float* part = a.ws + part_floats(sg_part);
                const uint32_t base = (uint32_t)(part_floats(sg_part) * sizeof(float));
#pragma unroll
                for (int rb = 0; rb < 2; ++rb) {
                    if (hf == 0) {
                        store_coherent(part + 32 * rb + l32, st.m[rb]);
                        store_coherent(part + kRows + 32 * rb + l32, lsum[rb]);
                    }
#pragma unroll
                    for (int db = 0; db < 4; ++db)
#pragma unroll
                        for (int i4 = 0; i4 < 4; ++i4)
                            store_coherent4(rs, base + (2 * kRows + (((rb * 4 + db) * 4 + i4) * 64 + lane) * 4) * 4,
                                            make_float4(st.o[rb][db][4 * i4], st.o[rb][db][4 * i4 + 1], st.o[rb][db][4 * i4 + 2], st.o[rb][db][4 * i4 + 3]));
                }
            }
            __syncthreads();   // waits for every thread's partial stores
            if (tid == 0) __hip_atomic_fetch_add(ctr + 1, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        } else {
            if (tid == 0) {
                const int others = p_end - p_begin - 1;
                int seen = __hip_atomic_load(ctr + 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                for (int spin = 0; spin < a.poll_limit && seen != others; ++spin) {
                    __builtin_amdgcn_s_sleep(2);
                    seen = __hip_atomic_load(ctr + 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                }
                if (seen == others) {
                    __hip_atomic_store(ctr, 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                    __hip_atomic_store(ctr + 1, 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                } else {
                    __hip_atomic_store(a.error_word, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM);   // see the decode kernel
                }
                *reinterpret_cast<volatile int*>(smem + L::kFlag + 8) = seen == others ? 1 : 0;
            }
            lds_barrier();
            asm volatile("" ::: "memory");
            if (*reinterpret_cast<volatile int*>(smem + L::kFlag + 8) && n_rows > 0) {
                // fold in partial-index order (this share's own state at its index), so that the
                // result does not depend on which share closes; the partials' loads go out four at a time
                constexpr int kFold = 4;
#pragma unroll
                for (int rb = 0; rb < 2; ++rb) {
                    const int row = 32 * rb + l32;
                    float m_all = -INFINITY;
                    for (int p0 = p_begin; p0 < p_end; p0 += kFold) {
                        float mp[kFold];
#pragma unroll
                        for (int k = 0; k < kFold; ++k) {
                            const int p = p0 + k;
                            mp[k] = p >= p_end ? -INFINITY : (p == sg_part ? st.m[rb] : load_coherent(a.ws + part_floats(p) + row));
                        }
#pragma unroll
                        for (int k = 0; k < kFold; ++k) m_all = fmaxf(m_all, mp[k]);
                    }
                    float l_all = 0.f;
                    for (int p0 = p_begin; p0 < p_end; p0 += kFold) {
                        float mp[kFold], lp[kFold];
#pragma unroll
                        for (int k = 0; k < kFold; ++k) {
                            const int p = p0 + k;
                            const bool mine = p == sg_part, none = p >= p_end;
                            mp[k] = none ? -INFINITY : (mine ? st.m[rb] : load_coherent(a.ws + part_floats(p) + row));
                            lp[k] = none ? 0.f : (mine ? lsum[rb] : load_coherent(a.ws + part_floats(p) + kRows + row));
                        }
#pragma unroll
                        for (int k = 0; k < kFold; ++k) l_all += lp[k] * __builtin_amdgcn_exp2f(mp[k] - m_all);   // past the end: 0 * 2^-inf
                    }
                    const float inv = 1.f / l_all;
                    const bool live = row < n_rows;
                    const int qi = cq0 + (live ? row / a.group : 0), qh = live ? row % a.group : 0;
                    uint16_t* op = a.out + (((size_t)sg_b * a.n_q + qi) * a.n_q_heads + g * a.group + qh) * kD;
#pragma unroll
                    for (int db = 0; db < 4; ++db) {
                        float4 acc[4];
#pragma unroll
                        for (int i4 = 0; i4 < 4; ++i4) acc[i4] = make_float4(0.f, 0.f, 0.f, 0.f);
                        for (int p0 = p_begin; p0 < p_end; p0 += kFold) {
                            float f[kFold];
                            float4 x[kFold][4];
#pragma unroll
                            for (int k = 0; k < kFold; ++k) {
                                const int p = p0 + k;
                                if (p < p_end && p != sg_part) {
                                    const uint32_t base = (uint32_t)(part_floats(p) * sizeof(float));
                                    f[k] = load_coherent(a.ws + part_floats(p) + row);
#pragma unroll
                                    for (int i4 = 0; i4 < 4; ++i4)
                                        x[k][i4] = load_coherent4(rs, base + (2 * kRows + (((rb * 4 + db) * 4 + i4) * 64 + lane) * 4) * 4);
                                } else {
                                    const bool mine = p == sg_part;
                                    f[k] = mine ? st.m[rb] : -INFINITY;
#pragma unroll
                                    for (int i4 = 0; i4 < 4; ++i4)
                                        x[k][i4] = mine ? make_float4(st.o[rb][db][4 * i4], st.o[rb][db][4 * i4 + 1], st.o[rb][db][4 * i4 + 2], st.o[rb][db][4 * i4 + 3])
                                                        : make_float4(0.f, 0.f, 0.f, 0.f);
                                }
                            }
#pragma unroll
                            for (int k = 0; k < kFold; ++k) {
                                const float fk = __builtin_amdgcn_exp2f(f[k] - m_all);
#pragma unroll
                                for (int i4 = 0; i4 < 4; ++i4) {
                                    acc[i4].x += fk * x[k][i4].x;
                                    acc[i4].y += fk * x[k][i4].y;
                                    acc[i4].z += fk * x[k][i4].z;
                                    acc[i4].w += fk * x[k][i4].w;
                                }
                            }
                        }
                        if (live)
#pragma unroll
                            for (int i4 = 0; i4 < 4; ++i4) {   // registers 4 i4 .. + 4 hold d = 32 db + 8 i4 + 4 (lane / 32) .. + 4
                                uint2 pk;
                                pk.x = pack_bf16x2(acc[i4].x * inv, acc[i4].y * inv);
                                pk.y = pack_bf16x2(acc[i4].z * inv, acc[i4].w * inv);
                                *reinterpret_cast<uint2*>(op + 32 * db + 8 * i4 + 4 * hf) = pk;
                            }
                    }
                }
            }
        }
        lds_barrier();  // the next segment reuses the LDS
    }
}

// ---------------------------------------------------------------------------------------------
// host side
// ---------------------------------------------------------------------------------------------

// bf16, head_dim 128, at most 64 grouped heads per KV head; at most 128 KV heads keeps the partials
// of the largest batch below the 2 GiB a buffer descriptor's 32-bit offsets reach.
bool mfma_eligible(const ms_cache* c, int n_q) {
    return c->d.dtype == MS_BF16 && c->d.head_dim == kD && c->group <= kRows && n_q <= MS_MAX_QUERIES && c->d.n_kv_heads <= 128;
}

// Layer pools below 4 GiB are addressed with 32-bit byte offsets from the layer base (one register
// per lane); larger ones take the build with 64-bit page bases.
static bool big_pool(const ms_cache* c) { return (unsigned long long)c->layer_elems * 2ull >= (1ull << 32); }

static int mfma_items(const ms_cache* c) {
    int target = c->n_cus / c->d.n_kv_heads;
    if (target < 1) target = 1;
    return target > kMaxMfmaItems ? kMaxMfmaItems : target;
}

// steps the decode kernel does not take: more than 16 queries or more than 64 rows per KV head
static bool mfma_wide_step(const ms_cache* c, int n_q) { return n_q > kDecodeQueries || n_q * c->group > kRows; }

// every share contributes one partial plus one per sequence boundary inside it; in a wide step one
// per chunk of queries
size_t mfma_workspace_bytes(const ms_cache* c, int B, int n_q) {
    return (size_t)(mfma_items(c) + B) * c->d.n_kv_heads * kPartFloats * sizeof(float) * (mfma_wide_step(c, n_q) ? kWideChunks : 1);
}

constexpr int kMaxAttrDevices = 64;
constexpr int kDefaultPollLimit = 1 << 22;   // about a second

__global__ void fill_arrival_counters(int* ctr, int n_pairs, int finished, int published) {
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n_pairs) {
        ctr[2 * i] = finished;
        ctr[2 * i + 1] = published;
    }
}

// Sets every pair's counters (a fill kernel: safe under stream capture, ordered behind earlier launches).
int reset_arrival_counters(ms_cache* c, int published, hipStream_t stream) {
    const int n_pairs = MS_MAX_BATCH * c->d.n_kv_heads;
    c->launches++;
    hipLaunchKernelGGL(fill_arrival_counters, dim3((n_pairs + 255) / 256), dim3(256), 0, stream, c->d_arrive, n_pairs, 0, published);
    MS_HIP_TRY(hipGetLastError());
    return MS_OK;
}

int launch_mfma(ms_cache* c, const AttnArgs& ga, const BatchMeta& bm, int B, hipStream_t stream) {
    // the kernels' LDS size is a per-device attribute: set once for every device the library meets
    static std::once_flag attr_once[kMaxAttrDevices];
    static hipError_t attr_result[kMaxAttrDevices];
    if (c->device < 0 || c->device >= kMaxAttrDevices) MS_FAIL(MS_ERR_UNSUPPORTED, "device index %d outside [0, %d)", c->device, kMaxAttrDevices);
    std::call_once(attr_once[c->device], [&] {
        hipError_t e = hipSuccess;
        const void* decode_builds[] = {(const void*)pv_attn_mfma_stream<false, false>, (const void*)pv_attn_mfma_stream<true, false>,
                                       (const void*)pv_attn_mfma_stream<false, true>, (const void*)pv_attn_mfma_stream<true, true>};
        for (const void* f : decode_builds)
            if (e == hipSuccess) e = hipFuncSetAttribute(f, hipFuncAttributeMaxDynamicSharedMemorySize, Lds::kBytes);
        if (e == hipSuccess) e = hipFuncSetAttribute((const void*)pv_attn_mfma_wide, hipFuncAttributeMaxDynamicSharedMemorySize, WideLds::kBytes);
        attr_result[c->device] = e;
    });
    if (attr_result[c->device] != hipSuccess)
        MS_FAIL(MS_ERR_HIP, "hipFuncSetAttribute(MaxDynamicSharedMemorySize) failed: %s", hipGetErrorString(attr_result[c->device]));
    // A closing workgroup of an earlier launch on this cache gave up waiting for partial results
    // (arrival counters in a bad state): that launch left output rows unwritten.  Report it once,
    // and put the counters back to zero behind everything queued so far.
    if (__atomic_load_n(c->h_error, __ATOMIC_RELAXED) != 0) {
        __atomic_store_n(c->h_error, 0, __ATOMIC_RELAXED);
        int rc = reset_arrival_counters(c, 0, stream);
        if (rc != MS_OK) return rc;
        MS_FAIL(MS_ERR_HIP, "an earlier attention launch on this cache timed out waiting for split-KV partial results and left "
                            "output rows unwritten; the arrival counters have been reset, repeat the step");
    }
    // plan: rebuilt only when the batch (ids, lengths) changed since the last call on this cache
    std::vector<int> key;
    // Smallest share.  Decode steps: two tiles per wave.  Wide steps: 32 tiles.  A share that does not
    // close its pair writes one partial per chunk of queries (33 KB each, read back once), which
    // argues for long shares; but a wide pass is bound by the work inside a workgroup, not by HBM,
    // so what counts is that every compute unit has a share: shares of 24 tiles per chunk (partials
    // below a tenth of the traffic) left three quarters of the chip idle on a batch of 8 sequences of
    // 4096 tokens and took 250 us where shares of 32 tiles take 95 us.
    const int n_q = ga.n_q;
    const int wide_chunks = !mfma_wide_step(c, n_q) ? 0 : std::min(kWideChunks, (n_q + kRows / ga.group - 1) / (kRows / ga.group));
    const long min_tiles = wide_chunks ? 32L : 2L * kWaves;
    key.reserve(B + 3);
    key.push_back(B);
    key.push_back((int)min_tiles);
    key.push_back((int)c->version);   // any change of lengths or page tables bumps the version
    for (int b = 0; b < B; ++b) key.push_back(bm.seq[b]);
    if (key != c->plan_key) {
        std::vector<int> blob;
        build_plan(c->pt, bm.seq, bm.len, B, mfma_items(c), min_tiles, blob, &c->plan_items, &c->plan_parts);
        const size_t bytes = blob.size() * sizeof(int);
        if (bytes > StageRing::kSlotBytes) MS_FAIL(MS_ERR_UNSUPPORTED, "attention plan of %zu bytes too large", bytes);
        int rc = c->stage.upload_to(c->d_plan, blob.data(), bytes, stream);
        if (rc != MS_OK) return rc;
        c->plan_key = key;
        c->plan_B = B;
    }
    MfmaArgs a;
    a.pool_layer = (const uint16_t*)ga.pool_layer;
    a.d_pt = ga.d_pt;
    a.d_len = ga.d_len;
    a.inv_freq = ga.inv_freq;
    a.q = (const uint16_t*)ga.q;
    a.k_new = (const uint16_t*)ga.k_new;
    a.v_new = (const uint16_t*)ga.v_new;
    a.pos = ga.pos;
    a.ctx_new = ga.ctx_new;
    a.out = (uint16_t*)ga.out;
    a.ws = ga.ws;
    a.item_first = reinterpret_cast<const Seg*>(c->d_plan);
    a.segs = reinterpret_cast<const Seg*>(c->d_plan + (size_t)c->plan_items * kSegInts);
    a.part_begin = c->d_plan + (size_t)(c->plan_items + c->plan_parts) * kSegInts;
    a.arrive = c->d_arrive;
    a.error_word = c->d_error;
    a.poll_limit = c->poll_limit > 0 ? c->poll_limit : kDefaultPollLimit;
    a.n_q = ga.n_q;
    a.n_verify = ga.n_verify;
    a.n_q_heads = ga.n_q_heads;
    a.n_kv_heads = ga.n_kv_heads;
    a.group = ga.group;
    a.max_pages = ga.max_pages;
    a.page_elems = ga.page_elems;
    a.scale_log2 = ga.scale * 1.44269504088896340736f;
    {
        // every prof_stride-th call opens a timed span of prof_span consecutive calls
        if (c->prof_open == 0 && c->prof_count < (int)c->prof_start.size() && c->prof_seen % c->prof_stride == 0) {
            MS_HIP_TRY(hipEventRecord(c->prof_start[c->prof_count], stream));
            c->prof_open = c->prof_span;
        }
        c->prof_seen++;
        const dim3 grid(c->plan_items, a.n_kv_heads);
        if (!mfma_wide_step(c, a.n_q)) {
            a.q0 = 0;
            a.n_qc = a.n_q;
            const bool big = big_pool(c);
            auto kern = c->deterministic ? (big ? pv_attn_mfma_stream<false, true> : pv_attn_mfma_stream<false, false>)
                                         : (big ? pv_attn_mfma_stream<true, true> : pv_attn_mfma_stream<true, false>);
            c->launches++;
            hipLaunchKernelGGL(kern, grid, dim3(kThreads), Lds::kBytes, stream, a);
        } else {
            // wide steps: a launch takes eight chunks of 64 / group queries, one per wave (with more than
            // eight query heads per KV head a step of 64 queries has more chunks than that: further
            // launches, which run in order on the stream and share the workspace and the counters)
            const int per_launch = kWideChunks * (kRows / a.group);
            for (a.q0 = 0; a.q0 < a.n_q; a.q0 += per_launch) {
                a.n_qc = a.n_q - a.q0 < per_launch ? a.n_q - a.q0 : per_launch;
                c->launches++;
                hipLaunchKernelGGL(pv_attn_mfma_wide, grid, dim3(kThreads), WideLds::kBytes, stream, a);
            }
        }
        MS_HIP_TRY(hipGetLastError());
        if (c->prof_open > 0 && --c->prof_open == 0) MS_HIP_TRY(hipEventRecord(c->prof_stop[c->prof_count++], stream));
    }
    return MS_OK;
}

}  // namespace ms

extern "C" int ms_profile_attention(ms_cache* c, int capacity, int stride, int span) {
    if (!c || capacity < 0 || stride < 1 || span < 1 || span > stride)
        MS_FAIL(MS_ERR_INVALID, "ms_profile_attention: bad argument");
    c->prof_stride = stride;
    c->prof_span = span;
    c->prof_seen = 0;
    c->prof_open = 0;
    for (hipEvent_t e : c->prof_start) (void)hipEventDestroy(e);
    for (hipEvent_t e : c->prof_stop) (void)hipEventDestroy(e);
    c->prof_start.clear();
    c->prof_stop.clear();
    c->prof_count = 0;
    for (int i = 0; i < capacity; ++i) {
        hipEvent_t a = nullptr, b = nullptr;
        MS_HIP_TRY(hipEventCreate(&a));
        c->prof_start.push_back(a);
        MS_HIP_TRY(hipEventCreate(&b));
        c->prof_stop.push_back(b);
    }
    return MS_OK;
}

extern "C" int ms_profile_read(ms_cache* c, float* ms_out, int cap, int* n) {
    if (!c || !n || (cap > 0 && !ms_out)) MS_FAIL(MS_ERR_INVALID, "ms_profile_read: null argument");
    *n = c->prof_count;
    for (int i = 0; i < c->prof_count && i < cap; ++i) {
        MS_HIP_TRY(hipEventSynchronize(c->prof_stop[i]));
        MS_HIP_TRY(hipEventElapsedTime(&ms_out[i], c->prof_start[i], c->prof_stop[i]));
        ms_out[i] /= (float)c->prof_span;
    }
    c->prof_count = 0;
    c->prof_open = 0;   // a span still open is dropped
    return MS_OK;
}

extern "C" int ms_attention_fault_injection(ms_cache* c, int poll_limit, int published_bias, void* stream) {
    if (!c || poll_limit < 0) MS_FAIL(MS_ERR_INVALID, "ms_attention_fault_injection: bad argument");
    c->poll_limit = poll_limit;
    return ms::reset_arrival_counters(c, published_bias, (hipStream_t)stream);
}
