// Fused Predict+Verify attention for bfloat16 caches with head_dim 128 and at most 64 query rows
// per KV head (rows = queries x grouped heads): the streaming kernel for gfx950.
//
// What is computed: see attention.hip (MemoSight paper, Sections 2.1.1 and 2.3).  How:
//   * The host cuts the batch's cached tokens, flattened over sequences in 32-token tiles, into
//     equal contiguous shares, one workgroup per (share, KV head).  A share that crosses sequence
//     boundaries is processed as several segments.
//   * Each of a workgroup's 8 waves streams every 8th tile of a segment on its own: K goes from
//     HBM straight into MFMA operand registers, V is staged through a wave-private LDS tile and
//     read back transposed (ds_read_b64_tr_b16); a wave refills its registers for its next tile as
//     soon as the current tile has consumed them.  There is no barrier inside the stream.
//   * Scores are computed transposed, S^T = K . Q^T (v_mfma_f32_32x32x16_bf16), so a lane owns one
//     query row: the online softmax needs one cross-lane exchange per tile and the rescale of the
//     O^T = V^T . P^T accumulators is a per-lane scalar.  Rescaling is lazy (only when a row's
//     maximum grows by more than 2^24), scores are kept in log2 units.
//   * Each segment leaves one partial (row maxima, row sums, unnormalised O) in the workspace; the
//     combine kernel merges the partials of a (sequence, KV head) with the in-flight block -- the
//     step's own verify / foresight keys under the visibility rule -- in fp32 and writes bf16.
#include <math.h>

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
constexpr int kTile = 32;               // tokens per MFMA tile
constexpr int kRows = 64;               // query rows per KV head (padded)
constexpr int kWaves = 8;               // waves per workgroup (2 per SIMD: at most 256 registers each)
constexpr int kVRowBytes = 288;         // LDS bytes per V row: 256 + 32 so 4 consecutive rows hit distinct banks
constexpr int kQRowBytes = 272;         // LDS bytes per rotated-Q row
constexpr int kVTileBytes = kTile * kVRowBytes;
constexpr float kRescaleThreshold = 24.0f;  // log2 units: P stays below 2^24
constexpr int kPartFloats = 2 * kRows + kRows * kD;  // m[64], l[64], O[128 regs][64 lanes]

// LDS map.  Stream phase: [Q tile][cos/sin table][one V tile per wave].  Merge phase (overlays it):
// per wave 32 accumulator registers (one d block of both row blocks) + 4 softmax scalars per lane.
constexpr int kLdsQ = 0;
constexpr int kLdsCs = kLdsQ + kRows * kQRowBytes;                       // 17408
constexpr int kLdsV = kLdsCs + MS_MAX_QUERIES * 64 * 8;                  // + 8192
constexpr int kLdsStream = kLdsV + kWaves * kVTileBytes;                 // + 73728 = 99328
constexpr int kMergeRegionBytes = (32 + 4) * 64 * 4;                     // 9216
constexpr int kLdsMerge = kWaves * kMergeRegionBytes;                    // 73728
constexpr int kLdsBytes = kLdsMerge > kLdsStream ? kLdsMerge : kLdsStream;
constexpr int kThreads = kWaves * 64;
static_assert(kThreads == kRows * 8, "the Q prologue maps one thread to one row and 8 rotation pairs");

struct Seg {
    int b;      // index in the call's batch
    int seq;    // sequence id
    int t0;     // first token (multiple of 32)
    int t1;     // one past the last token
    int part;   // partial slot (per KV head)
    int len;    // sequence length
    int pad0, pad1;
};

struct MfmaArgs {
    const uint16_t* pool_layer;
    const int* d_pt;
    const float* inv_freq;
    const uint16_t* q;
    const uint16_t* k_new;
    const uint16_t* v_new;
    const int* pos;
    const int* ctx_new;
    uint16_t* out;
    float* ws;
    const int* item_seg;    // [n_items + 1]
    const Seg* segs;
    const int* part_begin;  // [B + 1]
    int n_q, n_verify, n_q_heads, n_kv_heads, group, max_pages;
    long page_elems;
    float scale_log2;       // softmax scale * log2(e)
};

__device__ __forceinline__ uint32_t pack_bf16x2(float a, float b) {
    f32x2_t f = {a, b};
    bf16x2_t h = __builtin_convertvector(f, bf16x2_t);
    return __builtin_bit_cast(uint32_t, h);
}

typedef __attribute__((ext_vector_type(4))) unsigned int u32x4_t;

// 16-byte non-temporal global load.
__device__ __forceinline__ uint4 load_stream(const uint16_t* p) {
    const u32x4_t t = __builtin_nontemporal_load(reinterpret_cast<const u32x4_t*>(p));
    return make_uint4(t.x, t.y, t.z, t.w);
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

__device__ __forceinline__ void load_k(uint4 (&k)[8], const uint16_t* __restrict__ pool, int pa, int pb, long page_elems,
                                       int g, int lane) {
    const int tok = lane & 31;
    const uint16_t* kp = pool + (size_t)(tok < 16 ? pa : pb) * page_elems + (size_t)g * 2 * MS_PAGE_SIZE * kD +
                         (tok & 15) * kD + 8 * (lane >> 5);
#pragma unroll
    for (int kk = 0; kk < 8; ++kk) k[kk] = *reinterpret_cast<const uint4*>(kp + 16 * kk);
}

__device__ __forceinline__ void load_v(uint4 (&v)[8], const uint16_t* __restrict__ pool, int pa, int pb, long page_elems,
                                       int g, int lane) {
    const size_t off = ((size_t)g * 2 + 1) * MS_PAGE_SIZE * kD + (lane >> 4) * kD + 8 * (lane & 15);
    const uint16_t* va = pool + (size_t)pa * page_elems + off;
    const uint16_t* vb = pool + (size_t)pb * page_elems + off;
    // V is read exactly once per call: streaming (non-temporal) loads keep it out of the caches
#pragma unroll
    for (int rr = 0; rr < 4; ++rr) v[rr] = load_stream(va + 4 * rr * kD);
#pragma unroll
    for (int rr = 0; rr < 4; ++rr) v[4 + rr] = load_stream(vb + 4 * rr * kD);
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
        const bf16x8_t qb =
            __builtin_bit_cast(bf16x8_t, *reinterpret_cast<const uint4*>(qbase + rb * 32 * kQRowBytes + 32 * kk));
        s = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8_t, k[kk]), qb, s, 0, 0, 0);
    }
}

// Accumulator i of a lane holds token 8 (i / 4) + 4 (lane / 32) + i % 4 of the tile.
__device__ __forceinline__ void mask_tail(f32x16_t& s, int valid, int hf) {
#pragma unroll
    for (int i = 0; i < 16; ++i)
        if (8 * (i >> 2) + 4 * hf + (i & 3) >= valid) s[i] = -INFINITY;
}

__global__ __launch_bounds__(kThreads) void pv_attn_mfma_stream(MfmaArgs a) {
    extern __shared__ __attribute__((aligned(16))) char smem[];
    const int item = blockIdx.x, g = blockIdx.y;
    const int tid = threadIdx.x;
    const int w = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int lane = tid & 63, hf = lane >> 5, l32 = lane & 31, l16 = lane & 15;
    const int n_rows = a.n_q * a.group;
    char* vl = smem + kLdsV + w * kVTileBytes;
    float2* cs_tab = reinterpret_cast<float2*>(smem + kLdsCs);
    // V^T operand addressing.  Within a 16-lane group the transposing load gives lane i, element j
    // the value M[4 j + i / 4][i % 4] of the 16 x 4 block whose row r is addressed by lane r.
    // Source lane r points at token T[r / 4], columns d0 + 4 (r % 4) .. + 4, so result lane i holds
    // V[T[0..3]][d0 + i]; T[j] = 16 ks + 8 w + 4 (lane / 32) + j matches the k-order of P^T, whose
    // operand element 4 w + j is score accumulator 8 ks + 4 w + j.
    const char* vbase = vl + (4 * hf + (l16 >> 2)) * kVRowBytes + (16 * ((lane >> 4) & 1) + 4 * (l16 & 3)) * 2;
    // Q^T operand: column = query row 32 rb + lane % 32, k = 16 kk + 8 (lane / 32) .. + 8
    const char* qbase = smem + kLdsQ + l32 * kQRowBytes + 16 * hf;
    char* vwrite = vl + (lane >> 4) * kVRowBytes + l16 * 16;

    const int seg_end = a.item_seg[item + 1];
    for (int si = a.item_seg[item]; si < seg_end; ++si) {
        const Seg sg = a.segs[si];
        const int* pt = a.d_pt + (size_t)sg.seq * a.max_pages;
        const int last_page = (sg.len - 1) >> 4;
        const int n_tok = sg.t1 - sg.t0;
        const int n_tiles = (n_tok + kTile - 1) / kTile;

        // this wave's first tile goes in flight before anything else
        TileRegs r;
        int pa, pb;
        tile_pages(pt, w, n_tiles, sg.t0, last_page, pa, pb);
        load_v(r.v, a.pool_layer, pa, pb, a.page_elems, g, lane);
        load_k(r.k, a.pool_layer, pa, pb, a.page_elems, g, lane);

        // ---- rotate this (sequence, KV head)'s queries into the LDS Q tile: thread t owns row
        // t / 8, rotation pairs 8 (t % 8) .. + 8; its two 16-byte loads are issued before the
        // cos/sin table is built ----
        const int qr = tid >> 3, qc = tid & 7;
        uint4 x0v = make_uint4(0, 0, 0, 0), x1v = make_uint4(0, 0, 0, 0);
        const int qi = qr / a.group;
        if (qr < n_rows) {
            const uint16_t* qp = a.q + (((size_t)sg.b * a.n_q + qi) * a.n_q_heads + g * a.group + qr % a.group) * kD + 8 * qc;
            x0v = *reinterpret_cast<const uint4*>(qp);
            x1v = *reinterpret_cast<const uint4*>(qp + 64);
        }
        for (int idx = tid; idx < a.n_q * 64; idx += kThreads) {
            float sn, cs;
            sincosf((float)a.pos[sg.b * a.n_q + (idx >> 6)] * a.inv_freq[idx & 63], &sn, &cs);
            cs_tab[idx] = make_float2(cs, sn);
        }
        __syncthreads();
        {
            const uint32_t w0[4] = {x0v.x, x0v.y, x0v.z, x0v.w}, w1[4] = {x1v.x, x1v.y, x1v.z, x1v.w};
            uint32_t y0[4], y1[4];
#pragma unroll
            for (int e2 = 0; e2 < 4; ++e2) {
                float r0[2], r1[2];
#pragma unroll
                for (int hh = 0; hh < 2; ++hh) {
                    const float x0 = hh ? __uint_as_float(w0[e2] & 0xffff0000u) : __uint_as_float(w0[e2] << 16);
                    const float x1 = hh ? __uint_as_float(w1[e2] & 0xffff0000u) : __uint_as_float(w1[e2] << 16);
                    const float2 c = qr < n_rows ? cs_tab[qi * 64 + 8 * qc + 2 * e2 + hh] : make_float2(0.f, 0.f);
                    r0[hh] = (x0 * c.x - x1 * c.y) * a.scale_log2;
                    r1[hh] = (x1 * c.x + x0 * c.y) * a.scale_log2;
                }
                y0[e2] = pack_bf16x2(r0[0], r0[1]);
                y1[e2] = pack_bf16x2(r1[0], r1[1]);
            }
            char* qrow = smem + kLdsQ + qr * kQRowBytes + 16 * qc;
            *reinterpret_cast<uint4*>(qrow) = make_uint4(y0[0], y0[1], y0[2], y0[3]);
            *reinterpret_cast<uint4*>(qrow + 128) = make_uint4(y1[0], y1[1], y1[2], y1[3]);
        }
        __syncthreads();

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

        // ---- the stream: tiles w, w + 8, ...; the next tile's loads are issued as soon as the
        // registers of the current one have been consumed ----
        for (int j = w; j < n_tiles; j += kWaves) {
            const int valid = n_tok - j * kTile;   // >= 32 except in the tail tile
            // V rows -> wave-private LDS tile; rows past the segment end become zeros
#pragma unroll
            for (int rr = 0; rr < 8; ++rr) *reinterpret_cast<uint4*>(vwrite + 4 * rr * kVRowBytes) = r.v[rr];
            if (valid < kTile) {
                for (int rr = 0; rr < 8; ++rr)
                    if (4 * rr + (lane >> 4) >= valid)
                        *reinterpret_cast<uint4*>(vwrite + 4 * rr * kVRowBytes) = make_uint4(0, 0, 0, 0);
            }
            tile_pages(pt, j + kWaves, n_tiles, sg.t0, last_page, pa, pb);
            load_v(r.v, a.pool_layer, pa, pb, a.page_elems, g, lane);
            f32x16_t s;
            qk_block(s, r.k, qbase, 0);
            if (valid < kTile) mask_tail(s, valid, hf);
            softmax_pv(st, s, 0, vbase);
            qk_block(s, r.k, qbase, 1);
            load_k(r.k, a.pool_layer, pa, pb, a.page_elems, g, lane);
            if (valid < kTile) mask_tail(s, valid, hf);
            softmax_pv(st, s, 1, vbase);
        }

        // ---- merge the waves' states through LDS (overlays the stream buffers), one d block per
        // pass: every wave stores its 32 registers of the block, then wave w reduces one float4 per
        // lane over all waves and writes it to the segment's partial ----
        float* part = a.ws + ((size_t)sg.part * a.n_kv_heads + g) * kPartFloats;
        float fw[2] = {0.f, 0.f};   // this wave's reduction weights are rebuilt per pass from m
        (void)fw;
#pragma unroll
        for (int db = 0; db < 4; ++db) {
            __syncthreads();
            {
                float* reg = reinterpret_cast<float*>(smem + w * kMergeRegionBytes);
#pragma unroll
                for (int rb = 0; rb < 2; ++rb)
#pragma unroll
                    for (int i4 = 0; i4 < 4; ++i4)
                        *reinterpret_cast<float4*>(reg + ((rb * 4 + i4) * 64 + lane) * 4) =
                            make_float4(st.o[rb][db][4 * i4], st.o[rb][db][4 * i4 + 1], st.o[rb][db][4 * i4 + 2],
                                        st.o[rb][db][4 * i4 + 3]);
                if (db == 0)
                    *reinterpret_cast<float4*>(reg + (8 * 64 + lane) * 4) = make_float4(st.m[0], st.m[1], st.l[0], st.l[1]);
            }
            __syncthreads();
            {
                // wave w reduces float4 slot w: row block w / 4, accumulators 4 (w % 4) .. + 4
                const int rb = w >> 2, i4 = w & 3;
                float mn = -INFINITY;    // wave 0 always has a tile, so the maximum is finite
                float mo[kWaves], lo[kWaves];
#pragma unroll
                for (int ow = 0; ow < kWaves; ++ow) {
                    const float4 ml = *reinterpret_cast<const float4*>(smem + ow * kMergeRegionBytes + (8 * 64 + lane) * 16);
                    mo[ow] = rb ? ml.y : ml.x;
                    lo[ow] = rb ? ml.w : ml.z;
                    mn = fmaxf(mn, mo[ow]);
                }
                float4 acc = make_float4(0.f, 0.f, 0.f, 0.f);
                float lt = 0.f;
#pragma unroll
                for (int ow = 0; ow < kWaves; ++ow) {
                    const float f = __builtin_amdgcn_exp2f(mo[ow] - mn);   // idle wave: 2^-inf = 0
                    lt += f * lo[ow];
                    const float4 x =
                        *reinterpret_cast<const float4*>(smem + ow * kMergeRegionBytes + ((rb * 4 + i4) * 64 + lane) * 16);
                    acc.x += f * x.x;
                    acc.y += f * x.y;
                    acc.z += f * x.z;
                    acc.w += f * x.w;
                }
                const int reg4 = rb * 16 + db * 4 + i4;
                *reinterpret_cast<float4*>(part + 2 * kRows + (reg4 * 64 + lane) * 4) = acc;
                if (db == 0 && i4 == 0) {
                    lt += __shfl_xor(lt, 32, 64);
                    if (hf == 0) {
                        part[32 * rb + l32] = mn;
                        part[kRows + 32 * rb + l32] = lt;
                    }
                }
            }
        }
        __syncthreads();  // the next segment reuses the LDS
    }
}

// One workgroup per (sequence of the call, KV head): merges that pair's partials with the in-flight
// block and writes the normalised bf16 output rows.  Wave w owns d block w; lanes own the same
// (row, d) pairs as in the stream kernel's accumulator layout.  All global loads of a phase are
// issued together: the kernel is a chain of a few memory latencies, not a stream.
__global__ __launch_bounds__(256) void pv_attn_mfma_combine(MfmaArgs a) {
    __shared__ float2 cs_tab[MS_MAX_QUERIES * 64];
    __shared__ float k_rot[MS_MAX_QUERIES][kD + 4];
    __shared__ float s_new[kRows][MS_MAX_QUERIES + 1];
    const int b = blockIdx.x, g = blockIdx.y;
    const int tid = threadIdx.x, w = tid >> 6, lane = tid & 63, hf = lane >> 5, l32 = lane & 31;
    const int n_q = a.n_q, n_rows = n_q * a.group;

    // phase 0: raw loads -- this thread's 16 rotation pairs of query row tid / 4, and (threads
    // below 8 n_q) 8 rotation pairs of one in-flight key
    const int r = tid >> 2, qtr = tid & 3;
    const int qi = r / a.group;
    uint4 qx0[2], qx1[2];
    qx0[0] = qx0[1] = qx1[0] = qx1[1] = make_uint4(0, 0, 0, 0);
    if (r < n_rows) {
        const uint16_t* qp = a.q + (((size_t)b * n_q + qi) * a.n_q_heads + g * a.group + r % a.group) * kD + 16 * qtr;
        qx0[0] = *reinterpret_cast<const uint4*>(qp);
        qx0[1] = *reinterpret_cast<const uint4*>(qp + 8);
        qx1[0] = *reinterpret_cast<const uint4*>(qp + 64);
        qx1[1] = *reinterpret_cast<const uint4*>(qp + 72);
    }
    const int kj = tid >> 3, kc = tid & 7;
    uint4 kx0 = make_uint4(0, 0, 0, 0), kx1 = make_uint4(0, 0, 0, 0);
    if (kj < n_q) {
        const uint16_t* kp = a.k_new + (((size_t)b * n_q + kj) * a.n_kv_heads + g) * kD + 8 * kc;
        kx0 = *reinterpret_cast<const uint4*>(kp);
        kx1 = *reinterpret_cast<const uint4*>(kp + 64);
    }
    for (int idx = tid; idx < n_q * 64; idx += 256) {
        float sn, cs;
        sincosf((float)a.pos[b * n_q + (idx >> 6)] * a.inv_freq[idx & 63], &sn, &cs);
        cs_tab[idx] = make_float2(cs, sn);
    }
    __syncthreads();
    if (kj < n_q) {
        const uint32_t w0[4] = {kx0.x, kx0.y, kx0.z, kx0.w}, w1[4] = {kx1.x, kx1.y, kx1.z, kx1.w};
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            const float x0 = (e & 1) ? __uint_as_float(w0[e >> 1] & 0xffff0000u) : __uint_as_float(w0[e >> 1] << 16);
            const float x1 = (e & 1) ? __uint_as_float(w1[e >> 1] & 0xffff0000u) : __uint_as_float(w1[e >> 1] << 16);
            const float2 c = cs_tab[kj * 64 + 8 * kc + e];
            k_rot[kj][8 * kc + e] = x0 * c.x - x1 * c.y;
            k_rot[kj][8 * kc + e + 64] = x1 * c.x + x0 * c.y;
        }
    }
    __syncthreads();
    {
        // scores of the in-flight keys: thread (row, quarter) covers 16 rotation pairs of its row
        float acc[MS_MAX_QUERIES];
#pragma unroll
        for (int j = 0; j < MS_MAX_QUERIES; ++j) acc[j] = 0.f;
        if (r < n_rows) {
            const uint32_t w0[8] = {qx0[0].x, qx0[0].y, qx0[0].z, qx0[0].w, qx0[1].x, qx0[1].y, qx0[1].z, qx0[1].w};
            const uint32_t w1[8] = {qx1[0].x, qx1[0].y, qx1[0].z, qx1[0].w, qx1[1].x, qx1[1].y, qx1[1].z, qx1[1].w};
#pragma unroll
            for (int e = 0; e < 16; ++e) {
                const int dd = 16 * qtr + e;
                const float x0 = (e & 1) ? __uint_as_float(w0[e >> 1] & 0xffff0000u) : __uint_as_float(w0[e >> 1] << 16);
                const float x1 = (e & 1) ? __uint_as_float(w1[e >> 1] & 0xffff0000u) : __uint_as_float(w1[e >> 1] << 16);
                const float2 c = cs_tab[qi * 64 + dd];
                const float y0 = x0 * c.x - x1 * c.y, y1 = x1 * c.x + x0 * c.y;
#pragma unroll
                for (int j = 0; j < MS_MAX_QUERIES; ++j)
                    if (j < n_q) acc[j] += y0 * k_rot[j][dd] + y1 * k_rot[j][dd + 64];
            }
        }
#pragma unroll
        for (int j = 0; j < MS_MAX_QUERIES; ++j) {
            float v = acc[j];
            v += __shfl_xor(v, 1, 64);
            v += __shfl_xor(v, 2, 64);
            if (qtr == 0 && j < n_q) s_new[r][j] = v * a.scale_log2;
        }
    }
    __syncthreads();

    const int p_begin = a.part_begin[b], p_end = a.part_begin[b + 1];
#pragma unroll
    for (int rb = 0; rb < 2; ++rb) {
        const int row = 32 * rb + l32;
        if (row >= n_rows) continue;
        const int i = row / a.group, h = g * a.group + row % a.group;
        const int ctx = a.ctx_new ? a.ctx_new[b * n_q + i] : (i < a.n_verify ? i : a.n_verify);
        float m = -INFINITY;
        for (int p = p_begin; p < p_end; ++p) m = fmaxf(m, a.ws[((size_t)p * a.n_kv_heads + g) * kPartFloats + row]);
        for (int j = 0; j < n_q; ++j)
            if (j < ctx || j == i) m = fmaxf(m, s_new[row][j]);
        float lsum = 0.f;
        float o[16];
#pragma unroll
        for (int e = 0; e < 16; ++e) o[e] = 0.f;
        for (int p = p_begin; p < p_end; ++p) {
            const float* part = a.ws + ((size_t)p * a.n_kv_heads + g) * kPartFloats;
            const float f = __builtin_amdgcn_exp2f(part[row] - m);
            lsum += f * part[kRows + row];
#pragma unroll
            for (int i4 = 0; i4 < 4; ++i4) {
                const int reg4 = rb * 16 + w * 4 + i4;
                const float4 x = *reinterpret_cast<const float4*>(part + 2 * kRows + (reg4 * 64 + lane) * 4);
                o[4 * i4 + 0] += f * x.x;
                o[4 * i4 + 1] += f * x.y;
                o[4 * i4 + 2] += f * x.z;
                o[4 * i4 + 3] += f * x.w;
            }
        }
        for (int j = 0; j < n_q; ++j) {
            if (!(j < ctx || j == i)) continue;
            const float pj = __builtin_amdgcn_exp2f(s_new[row][j] - m);
            lsum += pj;
            const uint16_t* vp = a.v_new + (((size_t)b * n_q + j) * a.n_kv_heads + g) * kD + 32 * w + 4 * hf;
#pragma unroll
            for (int i4 = 0; i4 < 4; ++i4) {
                const uint2 raw = *reinterpret_cast<const uint2*>(vp + 8 * i4);
                o[4 * i4 + 0] += pj * bf16_bits_to_float(raw.x & 0xffffu);
                o[4 * i4 + 1] += pj * bf16_bits_to_float(raw.x >> 16);
                o[4 * i4 + 2] += pj * bf16_bits_to_float(raw.y & 0xffffu);
                o[4 * i4 + 3] += pj * bf16_bits_to_float(raw.y >> 16);
            }
        }
        const float inv = 1.f / lsum;
        uint16_t* op = a.out + (((size_t)b * n_q + i) * a.n_q_heads + h) * kD + 32 * w + 4 * hf;
#pragma unroll
        for (int i4 = 0; i4 < 4; ++i4) {
            uint2 pk;
            pk.x = pack_bf16x2(o[4 * i4 + 0] * inv, o[4 * i4 + 1] * inv);
            pk.y = pack_bf16x2(o[4 * i4 + 2] * inv, o[4 * i4 + 3] * inv);
            *reinterpret_cast<uint2*>(op + 8 * i4) = pk;
        }
    }
}

// ---------------------------------------------------------------------------------------------
// host side
// ---------------------------------------------------------------------------------------------

bool mfma_eligible(const ms_cache* c, int n_q) {
    return c->d.dtype == MS_BF16 && c->d.head_dim == kD && n_q * c->group <= kRows;
}

static int mfma_items(const ms_cache* c) {
    int target = c->n_cus / c->d.n_kv_heads;
    if (target < 1) target = 1;
    return target > kMaxMfmaItems ? kMaxMfmaItems : target;
}

// every share contributes one partial plus one per sequence boundary inside it
size_t mfma_workspace_bytes(const ms_cache* c, int B) {
    return (size_t)(mfma_items(c) + B) * c->d.n_kv_heads * kPartFloats * sizeof(float);
}

int mfma_plan_ints(int B) { return (kMaxMfmaItems + 1) + (kMaxMfmaItems + B) * (int)(sizeof(Seg) / sizeof(int)) + (B + 1); }

// Splits the batch's tiles into equal contiguous shares and lists each share's segments.
static void build_plan(const ms_cache* c, const BatchMeta& bm, int B, int n_items_target, std::vector<int>& blob,
                       int* n_items_out, int* n_parts_out) {
    std::vector<long> tile_prefix(B + 1, 0);
    for (int b = 0; b < B; ++b) tile_prefix[b + 1] = tile_prefix[b] + (bm.len[b] + kTile - 1) / kTile;
    const long nt = tile_prefix[B];
    int n_items = n_items_target;
    const long min_tiles = 2 * kWaves;  // at least two tiles per wave in a share
    if ((long)n_items * min_tiles > nt) n_items = (int)(nt / min_tiles);
    if (n_items < 1) n_items = nt > 0 ? 1 : 0;
    std::vector<int> item_seg(n_items + 1, 0);
    std::vector<Seg> segs;
    std::vector<int> part_begin(B + 1, 0);
    std::vector<int> part_count(B, 0);
    int b = 0;
    for (int it = 0; it < n_items; ++it) {
        const long lo = nt * it / n_items, hi = nt * (it + 1) / n_items;
        item_seg[it] = (int)segs.size();
        long cur = lo;
        while (cur < hi) {
            while (tile_prefix[b + 1] <= cur) ++b;
            const long end = hi < tile_prefix[b + 1] ? hi : tile_prefix[b + 1];
            Seg s;
            s.b = b;
            s.seq = bm.seq[b];
            s.t0 = (int)(cur - tile_prefix[b]) * kTile;
            s.t1 = (int)(end - tile_prefix[b]) * kTile;
            if (s.t1 > bm.len[b]) s.t1 = bm.len[b];
            s.part = 0;
            s.len = bm.len[b];
            s.pad0 = s.pad1 = 0;
            part_count[b]++;
            segs.push_back(s);
            cur = end;
        }
    }
    item_seg[n_items] = (int)segs.size();
    for (int i = 0; i < B; ++i) part_begin[i + 1] = part_begin[i] + part_count[i];
    // segments are generated in sequence order, so partial slots are simply their running index
    for (size_t i = 0; i < segs.size(); ++i) segs[i].part = (int)i;
    blob.clear();
    blob.insert(blob.end(), item_seg.begin(), item_seg.end());
    blob.resize(kMaxMfmaItems + 1, 0);
    const int* sp = reinterpret_cast<const int*>(segs.data());
    blob.insert(blob.end(), sp, sp + segs.size() * (sizeof(Seg) / sizeof(int)));
    blob.resize((kMaxMfmaItems + 1) + (size_t)(kMaxMfmaItems + B) * (sizeof(Seg) / sizeof(int)), 0);
    blob.insert(blob.end(), part_begin.begin(), part_begin.end());
    *n_items_out = n_items;
    *n_parts_out = (int)segs.size();
}

int launch_mfma(ms_cache* c, const AttnArgs& ga, const BatchMeta& bm, int B, hipStream_t stream) {
    static bool attr_set = false;
    if (!attr_set) {
        MS_HIP_TRY(hipFuncSetAttribute((const void*)pv_attn_mfma_stream, hipFuncAttributeMaxDynamicSharedMemorySize, kLdsBytes));
        attr_set = true;
    }
    // plan: rebuilt only when the batch (ids, lengths) changed since the last call on this cache
    std::vector<int> key;
    key.reserve(2 * B + 1);
    key.push_back(B);
    for (int b = 0; b < B; ++b) {
        key.push_back(bm.seq[b]);
        key.push_back(bm.len[b]);
    }
    if (key != c->plan_key) {
        std::vector<int> blob;
        build_plan(c, bm, B, mfma_items(c), blob, &c->plan_items, &c->plan_parts);
        const size_t bytes = blob.size() * sizeof(int);
        if (bytes > StageRing::kSlotBytes) MS_FAIL(MS_ERR_UNSUPPORTED, "attention plan of %zu bytes too large", bytes);
        void* dev = nullptr;
        int rc = c->stage.upload(blob.data(), bytes, stream, &dev);
        if (rc != MS_OK) return rc;
        MS_HIP_TRY(hipMemcpyAsync(c->d_plan, dev, bytes, hipMemcpyDeviceToDevice, stream));
        c->plan_key = key;
        c->plan_B = B;
    }
    MfmaArgs a;
    a.pool_layer = (const uint16_t*)ga.pool_layer;
    a.d_pt = ga.d_pt;
    a.inv_freq = ga.inv_freq;
    a.q = (const uint16_t*)ga.q;
    a.k_new = (const uint16_t*)ga.k_new;
    a.v_new = (const uint16_t*)ga.v_new;
    a.pos = ga.pos;
    a.ctx_new = ga.ctx_new;
    a.out = (uint16_t*)ga.out;
    a.ws = ga.ws;
    a.item_seg = c->d_plan;
    a.segs = reinterpret_cast<const Seg*>(c->d_plan + (kMaxMfmaItems + 1));
    a.part_begin = c->d_plan + (kMaxMfmaItems + 1) + (size_t)(kMaxMfmaItems + B) * (sizeof(Seg) / sizeof(int));
    a.n_q = ga.n_q;
    a.n_verify = ga.n_verify;
    a.n_q_heads = ga.n_q_heads;
    a.n_kv_heads = ga.n_kv_heads;
    a.group = ga.group;
    a.max_pages = ga.max_pages;
    a.page_elems = ga.page_elems;
    a.scale_log2 = ga.scale * 1.44269504088896340736f;
    if (c->plan_items > 0) {
        const bool prof = c->prof_count < (int)c->prof_start.size();
        if (prof) MS_HIP_TRY(hipEventRecord(c->prof_start[c->prof_count], stream));
        hipLaunchKernelGGL(pv_attn_mfma_stream, dim3(c->plan_items, a.n_kv_heads), dim3(kThreads), kLdsBytes, stream, a);
        MS_HIP_TRY(hipGetLastError());
        if (prof) MS_HIP_TRY(hipEventRecord(c->prof_stop[c->prof_count++], stream));
    }
    hipLaunchKernelGGL(pv_attn_mfma_combine, dim3(B, a.n_kv_heads), dim3(256), 0, stream, a);
    MS_HIP_TRY(hipGetLastError());
    return MS_OK;
}

}  // namespace ms

extern "C" int ms_profile_attention(ms_cache* c, int capacity) {
    if (!c || capacity < 0) MS_FAIL(MS_ERR_INVALID, "ms_profile_attention: bad argument");
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
    }
    c->prof_count = 0;
    return MS_OK;
}
