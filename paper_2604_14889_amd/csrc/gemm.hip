// bf16 GEMM for the decode step's dense projections: C[M][N] = A[M][K] . W[N][K]^T (+ bias),
// fp32 accumulation on the matrix cores (MemoSight paper, Appendix A, Algorithm 1: SpeculativeStep
// runs the model's projections over the few hundred tokens of a step; Section 4.1 names the models).
//
// Shape of the problem: M is small (batch x queries, a few hundred rows), N and K are the model's
// widths, both operands are K-contiguous.  One workgroup of 8 waves computes a 256 (M) x 128 (N)
// tile over a K range; grid = (column tiles x row tiles, 1, split_k).  K is walked in steps of 32:
// both tiles go global -> registers -> LDS (row stride 80 bytes: conflict-free for the 16-byte
// operand reads); the global loads run three steps ahead of the multiplication, one LDS-only
// barrier per step.  A wave owns 64 (M) x 64 (N): 2 x 2 accumulator tiles of
// v_mfma_f32_32x32x16_bf16 with W as the A operand (rows = n) and the activations as the B operand
// (columns = m), so a lane ends up with four consecutive n of one row m per register quad.
// split_k > 1 (deep K, few output tiles: the MLP down projection) writes fp32 partials that a
// second kernel sums, adds the bias to and rounds.  With split_k = 1 and more tiles than the chip
// holds at once, the tiles of the last, partly filled round are split over K inside the same launch
// (their workgroups start as soon as slots free up), so that a round with few tiles does not cost a
// whole tile's time.  The gate/up projection of the MLP can apply SwiGLU in the epilogue: with the
// weight rows interleaved in blocks of 32 (gate block, up block), a lane holds gate and up of the
// same output element in two accumulators and writes silu(gate) * up directly.
#include <stdint.h>

#include "ms_device.h"
#include "ms_internal.h"

namespace ms {

typedef __attribute__((ext_vector_type(8))) __bf16 g_bf16x8_t;
typedef __attribute__((ext_vector_type(16))) float g_f32x16_t;

constexpr int kGemmBM = 256, kGemmBN = 128, kGemmBK = 32;
constexpr int kGemmThreads = 512;
constexpr int kGemmRowBytes = kGemmBK * 2 + 16;                      // 80
constexpr int kGemmStageBytes = (kGemmBM + kGemmBN) * kGemmRowBytes;  // 30720
constexpr int kGemmMaxOut = 4;

struct GemmArgs {
    const uint16_t* a;      // [M][K]
    const uint16_t* w;      // [N][K]
    const uint16_t* bias;   // [N] or null
    int M, N, K, k_per_split;
    int n_out;
    uint16_t* out[kGemmMaxOut];     // destination of columns out_col[i] .. out_col[i + 1]
    int out_col[kGemmMaxOut + 1];
    float* partial;         // split_k > 1: [split_k][M][N]; K-split last round: [tail_split][M][N - tail_col0]
    // K-split last round (split_k == 1 only): blocks from tail_first on compute K part
    // (block - tail_first) / tail_blocks of tile tail_first + (block - tail_first) % tail_blocks
    int tail_first, tail_blocks, tail_k, tail_col0;
    // greedy-token mode: no C is written; every group of columns leaves its best (value, column) per
    // row as a 64-bit key in keys[group][M], and argmax_finish picks the best key of each row
    unsigned long long* keys;
};

enum GemmMode { kGemmPlain = 0, kGemmAllPartial = 1, kGemmSwiglu = 2, kGemmArgmax = 3 };

// Destination of column n: base pointer, first column and width.  Written as a chain of selects
// over constant indices (a run-time index into the argument arrays would move them to memory).
__device__ __forceinline__ void pick_destination(const GemmArgs& g, int n, uint16_t*& dst, int& col0, int& ld) {
    dst = g.out[0];
    col0 = 0;
    int col1 = g.out_col[1];
#pragma unroll
    for (int t = 1; t < kGemmMaxOut; ++t)
        if (t < g.n_out && n >= g.out_col[t]) {
            dst = g.out[t];
            col0 = g.out_col[t];
            col1 = g.out_col[t + 1];
        }
    ld = col1 - col0;
}

__device__ __forceinline__ uint32_t g_pack_bf16x2(float a, float b) {
    return (uint32_t)float_to_bf16_bits(a) | ((uint32_t)float_to_bf16_bits(b) << 16);
}

// silu(gate) * up in fp32 (SwiGLU of the models' MLP)
__device__ __forceinline__ float swiglu_value(float gate, float up) { return gate / (1.f + __expf(-gate)) * up; }

// Greedy token over fp32 sums: a 64-bit key orders by value first, then by lower column; NaN never
// wins (key 0).  max over keys = the largest value, the lowest column among equals.
__device__ __forceinline__ unsigned long long argmax_key(float v, int n) {
    if (v != v) return 0ull;
    uint32_t u = __float_as_uint(v);
    u = (u & 0x80000000u) ? ~u : (u | 0x80000000u);
    return ((unsigned long long)u << 32) | (0xffffffffu - (uint32_t)n);
}
__device__ __forceinline__ unsigned long long key_max(unsigned long long a, unsigned long long b) { return a > b ? a : b; }

// Workgroup barrier that orders LDS traffic only (a plain __syncthreads() would also wait for the
// global loads of the steps ahead).
__device__ __forceinline__ void gemm_lds_barrier() {
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup", "local");
    __builtin_amdgcn_s_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup", "local");
}

template <int kMode>
__global__ __launch_bounds__(kGemmThreads, 4) void gemm_tn_bf16(GemmArgs g) {
    constexpr bool kSplit = kMode == kGemmAllPartial;
    __shared__ __attribute__((aligned(16))) char smem[2 * kGemmStageBytes];
    const int tid = threadIdx.x, lane = tid & 63, l32 = lane & 31, hf = lane >> 5;
    const int w = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm = w >> 1, wn = w & 1;                  // wave tile: rows 64 wm .. + 64, columns 64 wn .. + 64
    // Tile mapping.  Workgroups are handed to the 8 XCDs (each with its own L2) round robin, so
    // workgroups 8 apart share an L2: the row tiles of one column tile are placed 8 apart, and the
    // weight tile they share comes from HBM once.
    const int m_tiles = (g.M + kGemmBM - 1) / kGemmBM, n_tiles = g.N / kGemmBN;
    int block = blockIdx.x, k_part = blockIdx.z, k_len = g.k_per_split;
    bool to_partial = kSplit;
    if (!kSplit && block >= g.tail_first) {   // a K part of a tile of the last round
        const int t = block - g.tail_first;
        k_part = t / g.tail_blocks;
        block = g.tail_first + t % g.tail_blocks;
        k_len = g.tail_k;
        to_partial = true;
    }
    const int in_group = block % (8 * m_tiles);
    const int n_tile = block / (8 * m_tiles) * 8 + in_group % 8, m_tile = in_group / 8;
    if (n_tile >= n_tiles) return;   // padding of the last group (the whole workgroup leaves)
    const int n0 = n_tile * kGemmBN, m0 = m_tile * kGemmBM;
    const int k_begin = k_part * k_len;
    const int steps = k_len / kGemmBK;

    // global -> LDS staging.  Four consecutive threads bring the 64 bytes one row contributes to a
    // step, so a load instruction of a wave covers 16 rows x 64 contiguous bytes; thread t handles
    // chunk t % 4 of activation rows r and r + 128 and of weight row r, r = t / 4 up to the order below.
    // Rows past M are clamped (read again, never stored).
    // Within each block of 16 rows the 4 x 4 (lane group, row) order is transposed: the 16 lanes that
    // store together then hold rows r, r + 4, r + 8, r + 12, whose 80-byte strides put their four
    // 16-byte chunks on 16 different groups of 4 banks (rows r .. r + 3 would collide two ways).
    const int sr_lin = tid >> 2, sc = tid & 3;
    const int sr = (sr_lin & ~15) | ((sr_lin & 3) << 2) | ((sr_lin >> 2) & 3);
    const uint16_t* a_src[2];
#pragma unroll
    for (int i = 0; i < 2; ++i) {
        const int row = m0 + sr + 128 * i < g.M ? m0 + sr + 128 * i : g.M - 1;
        a_src[i] = g.a + (size_t)row * g.K + k_begin + 8 * sc;
    }
    const uint16_t* w_src = g.w + (size_t)(n0 + sr) * g.K + k_begin + 8 * sc;
    char* a_dst = smem + sr * kGemmRowBytes + 16 * sc;
    char* w_dst = smem + kGemmBM * kGemmRowBytes + sr * kGemmRowBytes + 16 * sc;

    // Three register sets of staged tiles: while step s is multiplied out of LDS, the tiles of
    // steps s + 1 and s + 2 are in registers or on their way and those of s + 3 are requested.  Only
    // LDS traffic is ordered by the barriers, so a step waits for the oldest loads alone.
    // (plain named registers: aggregates handed around by name ended up in scratch memory)
    uint4 r0a0, r0a1, r0w0;
    uint4 r1a0, r1a1, r1w0;
    uint4 r2a0, r2a1, r2w0;
#define MS_GEMM_FETCH(R, step_)                                                 \
    do {                                                                        \
        const int ko_ = (step_) * kGemmBK;                                      \
        R##a0 = *reinterpret_cast<const uint4*>(a_src[0] + ko_);                \
        R##a1 = *reinterpret_cast<const uint4*>(a_src[1] + ko_);                \
        R##w0 = *reinterpret_cast<const uint4*>(w_src + ko_);                   \
    } while (0)
#define MS_GEMM_STASH(R, buf_)                                                  \
    do {                                                                        \
        char* ad_ = a_dst + (buf_) * kGemmStageBytes;                           \
        char* wd_ = w_dst + (buf_) * kGemmStageBytes;                           \
        *reinterpret_cast<uint4*>(ad_) = R##a0;                                 \
        *reinterpret_cast<uint4*>(ad_ + 128 * kGemmRowBytes) = R##a1;           \
        *reinterpret_cast<uint4*>(wd_) = R##w0;                                 \
    } while (0)

    g_f32x16_t acc[2][2];
#pragma unroll
    for (int ni = 0; ni < 2; ++ni)
#pragma unroll
        for (int mi = 0; mi < 2; ++mi)
#pragma unroll
            for (int i = 0; i < 16; ++i) acc[ni][mi][i] = 0.f;

    // operand addresses inside a stage: 16 bytes at k = 16 kk + 8 (lane / 32) of row (lane % 32)
    const int a_op = (64 * wm + l32) * kGemmRowBytes + 16 * hf;
    const int w_op = kGemmBM * kGemmRowBytes + (64 * wn + l32) * kGemmRowBytes + 16 * hf;

    // steps past the end re-read the last one (clamped): loads stay unconditional, nothing is used
    const int last = steps - 1;
#define MS_GEMM_CLAMP(s_) ((s_) < last ? (s_) : last)
    MS_GEMM_FETCH(r0, 0);
    MS_GEMM_FETCH(r1, MS_GEMM_CLAMP(1));
    MS_GEMM_FETCH(r2, MS_GEMM_CLAMP(2));
    MS_GEMM_STASH(r0, 0);
    gemm_lds_barrier();
    // one pipeline turn: multiply step s out of LDS[s & 1], request step s + 3 into the set that
    // step s came from (FREE), move step s + 1 (NEXT) into the other LDS stage
#define MS_GEMM_TURN(step_, FREE, NEXT)                                                                                     \
    do {                                                                                                                    \
        MS_GEMM_FETCH(FREE, MS_GEMM_CLAMP((step_) + 3));                                                                    \
        const char* base_ = smem + ((step_) & 1) * kGemmStageBytes;                                                         \
        _Pragma("unroll") for (int kk = 0; kk < 2; ++kk) {                                                                  \
            g_bf16x8_t wf[2], af[2];                                                                                        \
            _Pragma("unroll") for (int ni = 0; ni < 2; ++ni) wf[ni] = __builtin_bit_cast(                                   \
                g_bf16x8_t, *reinterpret_cast<const uint4*>(base_ + w_op + ni * 32 * kGemmRowBytes + 32 * kk));             \
            _Pragma("unroll") for (int mi = 0; mi < 2; ++mi) af[mi] = __builtin_bit_cast(                                   \
                g_bf16x8_t, *reinterpret_cast<const uint4*>(base_ + a_op + mi * 32 * kGemmRowBytes + 32 * kk));             \
            _Pragma("unroll") for (int ni = 0; ni < 2; ++ni) _Pragma("unroll") for (int mi = 0; mi < 2; ++mi)               \
                acc[ni][mi] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wf[ni], af[mi], acc[ni][mi], 0, 0, 0);                \
        }                                                                                                                   \
        MS_GEMM_STASH(NEXT, ((step_) + 1) & 1); /* that stage was last read before the previous barrier */                  \
        gemm_lds_barrier();                                                                                                 \
    } while (0)
    int step = 0;
    for (; step + 3 <= steps; step += 3) {
        MS_GEMM_TURN(step, r0, r1);
        MS_GEMM_TURN(step + 1, r1, r2);
        MS_GEMM_TURN(step + 2, r2, r0);
    }
    if (step < steps) {
        MS_GEMM_TURN(step, r0, r1);
        if (step + 1 < steps) MS_GEMM_TURN(step + 1, r1, r2);
    }
#undef MS_GEMM_TURN
#undef MS_GEMM_CLAMP
#undef MS_GEMM_FETCH
#undef MS_GEMM_STASH

    // accumulator i of a lane: n = 8 (i / 4) + 4 (lane / 32) + i % 4, m = lane % 32 (within the 32 x 32 tile)
    if (to_partial) {
        const int p_col0 = kSplit ? 0 : g.tail_col0, p_ld = g.N - p_col0;
#pragma unroll
        for (int mi = 0; mi < 2; ++mi) {
            const int m = m0 + 64 * wm + 32 * mi + l32;
            if (m >= g.M) continue;
#pragma unroll
            for (int ni = 0; ni < 2; ++ni)
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    const int n = n0 + 64 * wn + 32 * ni + 8 * q + 4 * hf;
                    *reinterpret_cast<float4*>(g.partial + ((size_t)k_part * g.M + m) * p_ld + (n - p_col0)) =
                        make_float4(acc[ni][mi][4 * q], acc[ni][mi][4 * q + 1], acc[ni][mi][4 * q + 2], acc[ni][mi][4 * q + 3]);
                }
        }
        return;
    }
    if (kMode == kGemmArgmax) {
        // group = (column tile, wave column): 64 columns; a lane first folds its 32 of them, then the
        // two half-waves (same row m, the other 4-column pieces) are folded through a lane exchange
#pragma unroll
        for (int mi = 0; mi < 2; ++mi) {
            unsigned long long best = 0ull;
#pragma unroll
            for (int ni = 0; ni < 2; ++ni)
#pragma unroll
                for (int i = 0; i < 16; ++i)
                    best = key_max(best, argmax_key(acc[ni][mi][i], n0 + 64 * wn + 32 * ni + 8 * (i >> 2) + 4 * hf + (i & 3)));
            const uint32_t lo = __shfl_xor((int)(uint32_t)best, 32, 64), hi = __shfl_xor((int)(uint32_t)(best >> 32), 32, 64);
            best = key_max(best, ((unsigned long long)hi << 32) | lo);
            const int m = m0 + 64 * wm + 32 * mi + l32;
            if (m < g.M && hf == 0) g.keys[(size_t)(n_tile * 2 + wn) * g.M + m] = best;
        }
        return;
    }
    if (kMode == kGemmSwiglu) {
        // weight rows 64 wn .. + 32 of the tile are gate rows, the next 32 the matching up rows:
        // accumulators [0][mi] and [1][mi] hold gate and up of output column n0 / 2 + 32 wn + ...
#pragma unroll
        for (int mi = 0; mi < 2; ++mi) {
            const int m = m0 + 64 * wm + 32 * mi + l32;
            if (m >= g.M) continue;
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                float o[4];
#pragma unroll
                for (int i = 0; i < 4; ++i) o[i] = swiglu_value(acc[0][mi][4 * q + i], acc[1][mi][4 * q + i]);
                uint2 pk;
                pk.x = g_pack_bf16x2(o[0], o[1]);
                pk.y = g_pack_bf16x2(o[2], o[3]);
                *reinterpret_cast<uint2*>(g.out[0] + (size_t)m * (g.N / 2) + n0 / 2 + 32 * wn + 8 * q + 4 * hf) = pk;
            }
        }
        return;
    }
    uint16_t* dst = nullptr;   // the whole tile goes to one destination: boundaries are multiples of 128
    int col0 = 0, ld = 0;
    pick_destination(g, n0, dst, col0, ld);
#pragma unroll
    for (int mi = 0; mi < 2; ++mi) {
        const int m = m0 + 64 * wm + 32 * mi + l32;
        if (m >= g.M) continue;
#pragma unroll
        for (int ni = 0; ni < 2; ++ni)
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const int n = n0 + 64 * wn + 32 * ni + 8 * q + 4 * hf;
                float4 v = make_float4(acc[ni][mi][4 * q], acc[ni][mi][4 * q + 1], acc[ni][mi][4 * q + 2], acc[ni][mi][4 * q + 3]);
                if (g.bias) {
                    const uint2 b = *reinterpret_cast<const uint2*>(g.bias + n);
                    v.x += bf16_bits_to_float(b.x & 0xffffu);
                    v.y += bf16_bits_to_float(b.x >> 16);
                    v.z += bf16_bits_to_float(b.y & 0xffffu);
                    v.w += bf16_bits_to_float(b.y >> 16);
                }
                uint2 pk;
                pk.x = g_pack_bf16x2(v.x, v.y);
                pk.y = g_pack_bf16x2(v.z, v.w);
                *reinterpret_cast<uint2*>(dst + (size_t)m * ld + (n - col0)) = pk;
            }
    }
}

// Sums the K parts of columns col0 .. N (partials [parts][M][N - col0]), adds the bias, rounds to
// bf16 and writes to the destination(s); in SwiGLU mode a thread sums four gate columns and the four
// matching up columns and writes silu(gate) * up.
template <bool kSwiglu>
__global__ __launch_bounds__(256) void gemm_reduce(GemmArgs g, int parts, int col0) {
    const int width = g.N - col0;
    const size_t quad = (size_t)blockIdx.x * 256 + threadIdx.x;   // 4 consecutive columns (of the output in SwiGLU mode)
    const int row_quads = (kSwiglu ? width / 2 : width) / 4;
    if (quad >= (size_t)g.M * row_quads) return;
    const int m = (int)(quad / row_quads), c = (int)(quad % row_quads) * 4;
    // SwiGLU: output column c of this range <- gate column 64 (c / 32) + c % 32 and the up column 32 further
    const int n_rel = kSwiglu ? 64 * (c / 32) + c % 32 : c;
    float4 s = make_float4(0.f, 0.f, 0.f, 0.f), u = s;
    for (int z = 0; z < parts; ++z) {
        const float* p = g.partial + ((size_t)z * g.M + m) * width + n_rel;
        const float4 a = *reinterpret_cast<const float4*>(p);
        s.x += a.x; s.y += a.y; s.z += a.z; s.w += a.w;
        if (kSwiglu) {
            const float4 b = *reinterpret_cast<const float4*>(p + 32);
            u.x += b.x; u.y += b.y; u.z += b.z; u.w += b.w;
        }
    }
    uint2 pk;
    if (kSwiglu) {
        pk.x = g_pack_bf16x2(swiglu_value(s.x, u.x), swiglu_value(s.y, u.y));
        pk.y = g_pack_bf16x2(swiglu_value(s.z, u.z), swiglu_value(s.w, u.w));
        *reinterpret_cast<uint2*>(g.out[0] + (size_t)m * (g.N / 2) + col0 / 2 + c) = pk;
        return;
    }
    const int n = col0 + c;
    if (g.bias) {
        const uint2 b = *reinterpret_cast<const uint2*>(g.bias + n);
        s.x += bf16_bits_to_float(b.x & 0xffffu);
        s.y += bf16_bits_to_float(b.x >> 16);
        s.z += bf16_bits_to_float(b.y & 0xffffu);
        s.w += bf16_bits_to_float(b.y >> 16);
    }
    uint16_t* dst;
    int dcol0, ld;
    pick_destination(g, n, dst, dcol0, ld);
    pk.x = g_pack_bf16x2(s.x, s.y);
    pk.y = g_pack_bf16x2(s.z, s.w);
    *reinterpret_cast<uint2*>(dst + (size_t)m * ld + (n - dcol0)) = pk;
}

// out[m] = column of the best key among keys[0 .. groups)[m]; a row without any key (all NaN) gives 0.
__global__ __launch_bounds__(256) void argmax_finish(const unsigned long long* keys, int groups, int M, int* out) {
    __shared__ unsigned long long red[256];
    const int m = blockIdx.x;
    unsigned long long best = 0ull;
    for (int gI = threadIdx.x; gI < groups; gI += 256) best = key_max(best, keys[(size_t)gI * M + m]);
    red[threadIdx.x] = best;
    __syncthreads();
    for (int s_ = 128; s_ > 0; s_ >>= 1) {
        if ((int)threadIdx.x < s_) red[threadIdx.x] = key_max(red[threadIdx.x], red[threadIdx.x + s_]);
        __syncthreads();
    }
    if (threadIdx.x == 0) out[m] = red[0] ? (int)(0xffffffffu - (uint32_t)red[0]) : 0;
}

typedef __attribute__((ext_vector_type(4))) uint32_t g_u32x4_t;

// ---------------------------------------------------------------------------------------------
// At most 8 rows (the step of a single sequence).  The product is bound by reading W once; tiles
// and matrix cores buy nothing.  A wave owns kR weight rows; per K step of 512 a lane takes 16
// bytes of each of them, so that one load instruction reads 1 KB of one row, and multiplies them
// with the activations' same 8 elements (from LDS, where the workgroup keeps its K range of all
// rows of A; read and widened once per step for all kR rows) with fp32 FMAs into sums per lane
// (v_dot2c_f32_bf16 was slower: the kernel became bound by it at 8 rows).
// The 64 lanes' sums are added at the end (DPP), lane 63 writes.  A workgroup's K range is what fits
// 64 KB of LDS with all rows of A (at most 16 steps): deeper K is divided over `parts` workgroups
// (fp32 partials, summed by gemm_reduce).
// ---------------------------------------------------------------------------------------------
constexpr int kGemvStepK = 512;            // 64 lanes x 8 elements
constexpr int kGemvThreads = 512;          // 8 waves share the staged activations
constexpr int kGemvLdsBytes = 64 * 1024;

// the 8 bf16 of a 16-byte chunk as fp32 (a shift or a mask each)
__device__ __forceinline__ void unpack8_bf16(uint4 v, float (&f)[8]) {
    f[0] = __uint_as_float(v.x << 16);
    f[1] = __uint_as_float(v.x & 0xffff0000u);
    f[2] = __uint_as_float(v.y << 16);
    f[3] = __uint_as_float(v.y & 0xffff0000u);
    f[4] = __uint_as_float(v.z << 16);
    f[5] = __uint_as_float(v.z & 0xffff0000u);
    f[6] = __uint_as_float(v.w << 16);
    f[7] = __uint_as_float(v.w & 0xffff0000u);
}

// Sum over the wave; the total arrives in lane 63.  Within rows of 16 lanes: the other lane of a
// pair, the other pair of a quad, the mirrored half row, the mirrored row; then lane 15 of rows 0
// and 2 into rows 1 and 3, lane 31 into rows 2 and 3.
__device__ __forceinline__ float wave_sum_to_last_lane(float v) {
    v += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), 0xB1, 0xF, 0xF, false));
    v += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), 0x4E, 0xF, 0xF, false));
    v += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), 0x141, 0xF, 0xF, false));
    v += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), 0x140, 0xF, 0xF, false));
    v += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), 0x142, 0xA, 0xF, false));
    v += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), 0x143, 0xC, 0xF, false));
    return v;
}

template <int kM, int kR>   // rows of A (1 .. 8), weight rows per wave
__global__ __launch_bounds__(kGemvThreads) void gemv_rows_bf16(GemmArgs g, int parts) {
    extern __shared__ __attribute__((aligned(16))) char a_lds[];
    const int tid = threadIdx.x, lane = tid & 63;
    const int w = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int steps_total = g.K / kGemvStepK;
    const int part = blockIdx.y;
    const int s_lo = (int)((long)steps_total * part / parts), s_hi = (int)((long)steps_total * (part + 1) / parts);
    const int steps = s_hi - s_lo, kp = steps * kGemvStepK;
    // the workgroup's K range of A: [kM][kp] bf16 (kM = M)
    for (int c = tid; c < kM * (kp / 8); c += kGemvThreads) {
        const int m = c / (kp / 8), kc = c % (kp / 8);
        uint4 v = make_uint4(0u, 0u, 0u, 0u);
        if (m < g.M) v = *reinterpret_cast<const uint4*>(g.a + (size_t)m * g.K + (size_t)s_lo * kGemvStepK + 8 * kc);
        *reinterpret_cast<uint4*>(a_lds + ((size_t)m * kp + 8 * kc) * 2) = v;
    }
    const int n0 = (blockIdx.x * (kGemvThreads / 64) + w) * kR;
    const uint16_t* wp = g.w + (size_t)n0 * g.K + (size_t)s_lo * kGemvStepK + 8 * lane;
    uint4 w0[kR], w1[kR];
    const int last = steps - 1;
#pragma unroll
    for (int r = 0; r < kR; ++r) {
        w0[r] = __builtin_bit_cast(uint4, __builtin_nontemporal_load(reinterpret_cast<const g_u32x4_t*>(wp + (size_t)r * g.K)));
        w1[r] = __builtin_bit_cast(uint4, __builtin_nontemporal_load(
            reinterpret_cast<const g_u32x4_t*>(wp + (size_t)r * g.K + (1 < last ? 1 : last) * kGemvStepK)));
    }
    float acc[kR][kM];
#pragma unroll
    for (int r = 0; r < kR; ++r)
#pragma unroll
        for (int m = 0; m < kM; ++m) acc[r][m] = 0.f;
    __syncthreads();
#define MS_GEMV_STEP(WV, s_)                                                                                  \
    do {                                                                                                      \
        float af[kM][8];                                                                                      \
        _Pragma("unroll") for (int m = 0; m < kM; ++m) unpack8_bf16(                                          \
            *reinterpret_cast<const uint4*>(a_lds + ((size_t)m * kp + (s_) * kGemvStepK + 8 * lane) * 2), af[m]); \
        _Pragma("unroll") for (int r = 0; r < kR; ++r) {                                                      \
            float wf[8];                                                                                      \
            unpack8_bf16(WV[r], wf);                                                                          \
            _Pragma("unroll") for (int m = 0; m < kM; ++m)                                                    \
                _Pragma("unroll") for (int e = 0; e < 8; ++e) acc[r][m] = fmaf(wf[e], af[m][e], acc[r][m]);   \
        }                                                                                                     \
    } while (0)
#define MS_GEMV_LOAD(WV, s_)                                                                                  \
    do {                                                                                                      \
        const int sc_ = (s_) < last ? (s_) : last; /* past the end: the last step again, unused */            \
        _Pragma("unroll") for (int r = 0; r < kR; ++r) WV[r] = __builtin_bit_cast(uint4, __builtin_nontemporal_load( \
            reinterpret_cast<const g_u32x4_t*>(wp + (size_t)r * g.K + sc_ * kGemvStepK)));                    \
    } while (0)
    for (int s = 0; s < steps; s += 2) {
        MS_GEMV_STEP(w0, s);
        MS_GEMV_LOAD(w0, s + 2);
        if (s + 1 < steps) MS_GEMV_STEP(w1, s + 1);
        MS_GEMV_LOAD(w1, s + 3);
    }
#undef MS_GEMV_STEP
#undef MS_GEMV_LOAD
#pragma unroll
    for (int r = 0; r < kR; ++r)
#pragma unroll
        for (int m = 0; m < kM; ++m) acc[r][m] = wave_sum_to_last_lane(acc[r][m]);
    if (lane != 63) return;
    if (g.keys) {   // greedy-token mode (parts == 1): the best of this wave's rows per row of A
#pragma unroll
        for (int m = 0; m < kM; ++m) {
            unsigned long long best = 0ull;
#pragma unroll
            for (int r = 0; r < kR; ++r) best = key_max(best, argmax_key(acc[r][m], n0 + r));
            g.keys[(size_t)(n0 / kR) * g.M + m] = best;
        }
        return;
    }
#pragma unroll
    for (int r = 0; r < kR; ++r) {
        const int n = n0 + r;
        uint16_t* dst = nullptr;
        int col0 = 0, ld = 0;
        if (parts == 1) pick_destination(g, n, dst, col0, ld);
        const float b = parts == 1 && g.bias ? bf16_bits_to_float(g.bias[n]) : 0.f;
#pragma unroll
        for (int m = 0; m < kM; ++m) {
            if (m >= g.M) continue;
            if (parts > 1) g.partial[((size_t)part * g.M + m) * g.N + n] = acc[r][m];
            else dst[(size_t)m * ld + (n - col0)] = float_to_bf16_bits(acc[r][m] + b);
        }
    }
}

static bool g_aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

// Workgroups the chip holds at once (two per compute unit), for the current device.
static int gemm_slots() {
    static int cached[64] = {};
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return 512;
    if (!cached[dev]) {
        int cus = 0;
        if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus < 1) cus = 256;
        cached[dev] = 2 * cus;
    }
    return cached[dev];
}

// The launch shape.  Blocks come in groups of 8 column tiles x m_tiles row tiles.  When the groups
// fill the chip at least once and the last round is at most 60 % full, the groups of that round are
// split over K: tail_split parts, chosen so that the round still fits the chip.
struct GemmPlan {
    int m_tiles, n_groups, group_blocks;
    int main_groups, tail_groups, tail_split;
    size_t workspace_bytes;
};

static GemmPlan gemm_plan(int M, int N, int K, int split_k) {
    GemmPlan p;
    p.m_tiles = (M + kGemmBM - 1) / kGemmBM;
    p.n_groups = (N / kGemmBN + 7) / 8;
    p.group_blocks = 8 * p.m_tiles;
    p.main_groups = p.n_groups;
    p.tail_groups = 0;
    p.tail_split = 1;
    p.workspace_bytes = split_k > 1 ? (size_t)split_k * M * N * sizeof(float) : 0;
    if (split_k != 1) return p;
    const int per_round = gemm_slots() / p.group_blocks;
    if (per_round < 1 || p.n_groups <= per_round) return p;
    const int rem = p.n_groups % per_round;
    if (rem == 0 || 10 * rem > 6 * per_round) return p;
    const int steps = K / kGemmBK;
    for (int s = 8; s >= 2; s >>= 1)
        if (steps % s == 0 && steps / s >= 8 && rem * s <= per_round) {
            p.tail_split = s;
            break;
        }
    if (p.tail_split == 1) return p;
    p.tail_groups = rem;
    p.main_groups = p.n_groups - rem;
    const long tail_cols = (long)N - (long)p.main_groups * 8 * kGemmBN;
    p.workspace_bytes = (size_t)p.tail_split * M * tail_cols * sizeof(float);
    return p;
}

// At most 8 rows: the row-streaming kernel's launch shape (0 parts: shape not eligible).
constexpr int kGemvMaxRows = 8;
struct GemvPlan {
    int parts, km, kr, lds_bytes;
    size_t workspace_bytes;
};
static GemvPlan gemv_plan(int M, int N, int K) {
    GemvPlan p = {0, 0, 0, 0, 0};
    if (M > kGemvMaxRows || K % kGemvStepK) return p;
    p.km = M;
    int max_steps = kGemvLdsBytes / (p.km * kGemvStepK * 2);         // K steps whose rows of A fit the LDS share
    if (max_steps > 16) max_steps = 16;
    const int steps = K / kGemvStepK;
    p.parts = (steps + max_steps - 1) / max_steps;
    p.lds_bytes = p.km * ((steps + p.parts - 1) / p.parts) * kGemvStepK * 2;
    const int want = gemm_slots();                                   // workgroups the chip holds two of per CU
    p.kr = N / 64 >= want ? 8 : N / 32 >= want ? 4 : 2;              // weight rows per wave, 8 waves per workgroup
    p.workspace_bytes = p.parts > 1 ? (size_t)p.parts * M * N * sizeof(float) : 0;
    return p;
}

static int gemm_check_shape(const char* what, int M, int N, int K, int split_k) {
    if (M < 0 || N < 1 || K < 1 || split_k < 1) MS_FAIL(MS_ERR_INVALID, "%s: bad size", what);
    if (N % kGemmBN || K % (kGemmBK * split_k))
        MS_FAIL(MS_ERR_UNSUPPORTED, "%s: N must be a multiple of %d and K of %d x split_k", what, kGemmBN, kGemmBK);
    if ((long long)M * N >= (1ll << 40) || split_k > 64 ||
        (long long)((N / kGemmBN + 7) / 8) * 8 * ((M + kGemmBM - 1) / kGemmBM) * 9 > 2000000000ll)
        MS_FAIL(MS_ERR_UNSUPPORTED, "%s: shape too large", what);
    return MS_OK;
}

// Launches the tiles (and the reduction of the parts, if any).  g holds operands and destinations.
template <int kM>
static void gemv_dispatch(const GemmArgs& g, const GemvPlan& v, hipStream_t stream) {
    const dim3 grid((unsigned)(g.N / (kGemvThreads / 64 * v.kr)), (unsigned)v.parts);
    if (v.kr == 8)
        hipLaunchKernelGGL((gemv_rows_bf16<kM, 8>), grid, dim3(kGemvThreads), v.lds_bytes, stream, g, v.parts);
    else if (v.kr == 4)
        hipLaunchKernelGGL((gemv_rows_bf16<kM, 4>), grid, dim3(kGemvThreads), v.lds_bytes, stream, g, v.parts);
    else
        hipLaunchKernelGGL((gemv_rows_bf16<kM, 2>), grid, dim3(kGemvThreads), v.lds_bytes, stream, g, v.parts);
}

static int gemm_launch(GemmArgs& g, int split_k, bool swiglu, void* workspace, size_t ws_bytes, hipStream_t stream) {
    if (!swiglu) {
        const GemvPlan v = gemv_plan(g.M, g.N, g.K);
        if (v.parts == 1 || (v.parts > 1 && workspace && ws_bytes >= v.workspace_bytes && g_aligned16(workspace))) {
            g.k_per_split = g.K;
            g.partial = v.parts > 1 ? (float*)workspace : nullptr;
            g.tail_first = g.tail_blocks = g.tail_k = g.tail_col0 = 0;
            switch (v.km) {
                case 1: gemv_dispatch<1>(g, v, stream); break;
                case 2: gemv_dispatch<2>(g, v, stream); break;
                case 3: gemv_dispatch<3>(g, v, stream); break;
                case 4: gemv_dispatch<4>(g, v, stream); break;
                case 5: gemv_dispatch<5>(g, v, stream); break;
                case 6: gemv_dispatch<6>(g, v, stream); break;
                case 7: gemv_dispatch<7>(g, v, stream); break;
                default: gemv_dispatch<8>(g, v, stream); break;
            }
            if (v.parts > 1) {
                const size_t quads = (size_t)g.M * g.N / 4;
                hipLaunchKernelGGL((gemm_reduce<false>), dim3((unsigned)((quads + 255) / 256)), dim3(256), 0, stream, g, v.parts, 0);
            }
            MS_HIP_TRY(hipGetLastError());
            return MS_OK;
        }
    }
    GemmPlan p = gemm_plan(g.M, g.N, g.K, split_k);
    if (split_k == 1 && p.tail_groups && (!workspace || ws_bytes < p.workspace_bytes || !g_aligned16(workspace))) {
        p.main_groups = p.n_groups;   // no room for the parts: whole tiles throughout
        p.tail_groups = 0;
        p.tail_split = 1;
    }
    g.k_per_split = g.K / split_k;
    g.partial = nullptr;
    const int main_blocks = p.main_groups * p.group_blocks;
    g.tail_first = main_blocks;
    g.tail_blocks = p.tail_groups * p.group_blocks;
    g.tail_k = g.K / p.tail_split;
    g.tail_col0 = p.main_groups * 8 * kGemmBN;
    const dim3 grid((unsigned)(main_blocks + g.tail_blocks * p.tail_split), 1, (unsigned)split_k);
    if (split_k > 1) {
        if (!workspace || ws_bytes < p.workspace_bytes || !g_aligned16(workspace))
            MS_FAIL(MS_ERR_WORKSPACE, "ms_gemm_bf16: split-K workspace of %zu bytes needed", p.workspace_bytes);
        g.partial = (float*)workspace;
        g.tail_first = (int)grid.x;   // unused by this build of the kernel
        hipLaunchKernelGGL((gemm_tn_bf16<kGemmAllPartial>), grid, dim3(kGemmThreads), 0, stream, g);
        const size_t quads = (size_t)g.M * g.N / 4;
        hipLaunchKernelGGL((gemm_reduce<false>), dim3((unsigned)((quads + 255) / 256)), dim3(256), 0, stream, g, split_k, 0);
    } else {
        if (p.tail_groups) g.partial = (float*)workspace;
        if (swiglu)
            hipLaunchKernelGGL((gemm_tn_bf16<kGemmSwiglu>), grid, dim3(kGemmThreads), 0, stream, g);
        else
            hipLaunchKernelGGL((gemm_tn_bf16<kGemmPlain>), grid, dim3(kGemmThreads), 0, stream, g);
        if (p.tail_groups) {
            const size_t quads = (size_t)g.M * (g.N - g.tail_col0) / (swiglu ? 8 : 4);
            const dim3 rgrid((unsigned)((quads + 255) / 256));
            if (swiglu)
                hipLaunchKernelGGL((gemm_reduce<true>), rgrid, dim3(256), 0, stream, g, p.tail_split, g.tail_col0);
            else
                hipLaunchKernelGGL((gemm_reduce<false>), rgrid, dim3(256), 0, stream, g, p.tail_split, g.tail_col0);
        }
    }
    MS_HIP_TRY(hipGetLastError());
    return MS_OK;
}

}  // namespace ms

extern "C" size_t ms_gemm_workspace_bytes(int M, int N, int K, int split_k) {
    if (M < 1 || N < 1 || K < 1 || split_k < 1 || N % ms::kGemmBN || K % (ms::kGemmBK * split_k)) return 0;
    const size_t tiled = ms::gemm_plan(M, N, K, split_k).workspace_bytes;
    const size_t rows = ms::gemv_plan(M, N, K).workspace_bytes;   // enough for either kernel
    return tiled > rows ? tiled : rows;
}

extern "C" int ms_gemm_bf16(const void* a, const void* w, const void* bias, int M, int N, int K, int n_out, void* const* out,
                            const int* out_col, int split_k, void* workspace, size_t ws_bytes, void* stream) {
    using namespace ms;
    if (n_out < 1 || n_out > kGemmMaxOut || !out || !out_col) MS_FAIL(MS_ERR_INVALID, "ms_gemm_bf16: bad destination table");
    int rc = gemm_check_shape("ms_gemm_bf16", M, N, K, split_k);
    if (rc != MS_OK) return rc;
    if (M == 0) return MS_OK;
    if (!a || !w || !g_aligned16(a) || !g_aligned16(w) || (bias && (reinterpret_cast<uintptr_t>(bias) & 7u)))
        MS_FAIL(MS_ERR_INVALID, "ms_gemm_bf16: null or misaligned operand");
    GemmArgs g;
    g.a = (const uint16_t*)a;
    g.w = (const uint16_t*)w;
    g.bias = (const uint16_t*)bias;
    g.M = M;
    g.N = N;
    g.K = K;
    g.n_out = n_out;
    g.keys = nullptr;
    if (out_col[0] != 0 || out_col[n_out] != N) MS_FAIL(MS_ERR_INVALID, "ms_gemm_bf16: destinations must cover columns 0 .. N");
    for (int i = 0; i < n_out; ++i) {
        if (out_col[i + 1] <= out_col[i] || out_col[i] % kGemmBN || !out[i] || (reinterpret_cast<uintptr_t>(out[i]) & 7u) ||
            (out_col[i + 1] - out_col[i]) % 4)
            MS_FAIL(MS_ERR_INVALID, "ms_gemm_bf16: destination %d: boundaries must rise in multiples of %d, pointers be 8-byte aligned", i, kGemmBN);
        g.out[i] = (uint16_t*)out[i];
        g.out_col[i] = out_col[i];
    }
    g.out_col[n_out] = N;
    for (int i = n_out; i < kGemmMaxOut; ++i) {
        g.out[i] = nullptr;
        g.out_col[i + 1] = N;
    }
    return gemm_launch(g, split_k, false, workspace, ws_bytes, (hipStream_t)stream);
}

extern "C" int ms_gemm_swiglu_bf16(const void* a, const void* w_gate_up, int M, int inter, int K, void* out, void* workspace,
                                   size_t ws_bytes, void* stream) {
    using namespace ms;
    if (inter < 1 || inter > (1 << 29)) MS_FAIL(MS_ERR_INVALID, "ms_gemm_swiglu_bf16: bad size");
    if (inter % 64) MS_FAIL(MS_ERR_UNSUPPORTED, "ms_gemm_swiglu_bf16: the MLP width must be a multiple of 64");
    const int N = 2 * inter;
    int rc = gemm_check_shape("ms_gemm_swiglu_bf16", M, N, K, 1);
    if (rc != MS_OK) return rc;
    if (M == 0) return MS_OK;
    if (!a || !w_gate_up || !out || !g_aligned16(a) || !g_aligned16(w_gate_up) || (reinterpret_cast<uintptr_t>(out) & 7u))
        MS_FAIL(MS_ERR_INVALID, "ms_gemm_swiglu_bf16: null or misaligned operand");
    GemmArgs g;
    g.a = (const uint16_t*)a;
    g.w = (const uint16_t*)w_gate_up;
    g.bias = nullptr;
    g.keys = nullptr;
    g.M = M;
    g.N = N;
    g.K = K;
    g.n_out = 1;
    g.out[0] = (uint16_t*)out;
    g.out_col[0] = 0;
    for (int i = 1; i < kGemmMaxOut; ++i) g.out[i] = nullptr;
    for (int i = 1; i <= kGemmMaxOut; ++i) g.out_col[i] = N;
    return gemm_launch(g, 1, true, workspace, ws_bytes, (hipStream_t)stream);
}

// Column groups that leave a key per row in greedy-token mode, for the kernel the shape runs on.
static int argmax_groups(int M, int N, int K) {
    const ms::GemvPlan v = ms::gemv_plan(M, N, K);
    return v.parts == 1 ? N / v.kr : N / ms::kGemmBN * 2;
}

extern "C" size_t ms_lm_head_argmax_workspace_bytes(int M, int vocab, int K) {
    if (M < 1 || vocab < 1 || K < 1 || vocab % ms::kGemmBN || K % ms::kGemmBK) return 0;
    return (size_t)argmax_groups(M, vocab, K) * M * sizeof(unsigned long long);
}

extern "C" int ms_lm_head_argmax_bf16(const void* a, const void* w, int M, int vocab, int K, int* out, void* workspace,
                                      size_t ws_bytes, void* stream_) {
    using namespace ms;
    hipStream_t stream = (hipStream_t)stream_;
    int rc = gemm_check_shape("ms_lm_head_argmax_bf16", M, vocab, K, 1);
    if (rc != MS_OK) return rc;
    if (M == 0) return MS_OK;
    if (!a || !w || !out || !g_aligned16(a) || !g_aligned16(w)) MS_FAIL(MS_ERR_INVALID, "ms_lm_head_argmax_bf16: null or misaligned operand");
    const size_t need = ms_lm_head_argmax_workspace_bytes(M, vocab, K);
    if (!workspace || ws_bytes < need || !g_aligned16(workspace))
        MS_FAIL(MS_ERR_WORKSPACE, "ms_lm_head_argmax_bf16: workspace of %zu bytes needed", need);
    GemmArgs g;
    g.a = (const uint16_t*)a;
    g.w = (const uint16_t*)w;
    g.bias = nullptr;
    g.M = M;
    g.N = vocab;
    g.K = K;
    g.k_per_split = K;
    g.n_out = 1;
    for (int i = 0; i < kGemmMaxOut; ++i) g.out[i] = nullptr;
    g.out_col[0] = 0;
    for (int i = 1; i <= kGemmMaxOut; ++i) g.out_col[i] = vocab;
    g.partial = nullptr;
    g.keys = (unsigned long long*)workspace;
    const int groups = argmax_groups(M, vocab, K);
    const GemvPlan v = gemv_plan(M, vocab, K);
    if (v.parts == 1) {
        g.tail_first = g.tail_blocks = g.tail_k = g.tail_col0 = 0;
        switch (v.km) {
            case 1: gemv_dispatch<1>(g, v, stream); break;
            case 2: gemv_dispatch<2>(g, v, stream); break;
            case 3: gemv_dispatch<3>(g, v, stream); break;
            case 4: gemv_dispatch<4>(g, v, stream); break;
            case 5: gemv_dispatch<5>(g, v, stream); break;
            case 6: gemv_dispatch<6>(g, v, stream); break;
            case 7: gemv_dispatch<7>(g, v, stream); break;
            default: gemv_dispatch<8>(g, v, stream); break;
        }
    } else {
        const GemmPlan p = gemm_plan(M, vocab, K, 1);
        const int blocks = p.n_groups * p.group_blocks;   // whole tiles throughout
        g.tail_first = blocks;
        g.tail_blocks = 0;
        g.tail_k = K;
        g.tail_col0 = vocab;
        hipLaunchKernelGGL((gemm_tn_bf16<kGemmArgmax>), dim3((unsigned)blocks), dim3(kGemmThreads), 0, stream, g);
    }
    hipLaunchKernelGGL(argmax_finish, dim3((unsigned)M), dim3(256), 0, stream, (const unsigned long long*)workspace, groups, M, out);
    MS_HIP_TRY(hipGetLastError());
    return MS_OK;
}
