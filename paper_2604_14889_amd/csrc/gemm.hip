// bf16 GEMM for the decode step's dense projections: C[M][N] = A[M][K] . W[N][K]^T (+ bias),
// fp32 accumulation on the matrix cores (MemoSight paper, Appendix A, Algorithm 1: SpeculativeStep
// runs the model's projections over the few hundred tokens of a step; Section 3.1 names the models).
//
// Shape of the problem: M is small (batch x queries, a few hundred rows), N and K are the model's
// widths, both operands are K-contiguous.  One workgroup of 8 waves computes a 256 (M) x 256 (N)
// tile over a K range; grid = (column tiles x row tiles, 1, split_k); one workgroup per compute
// unit (two waves per SIMD, up to 256 registers each).  K is walked in steps of 32: both tiles go
// global -> registers -> LDS (two stages; row stride 80 bytes: conflict-free for the 16-byte
// operand reads), the global loads requested two steps before they are stored.  A wave owns
// 128 (M) x 64 (N): 2 x 4 accumulator tiles of v_mfma_f32_32x32x16_bf16 with W as the A operand
// (rows = n) and the activations as the B operand (columns = m), so a lane ends up with four
// consecutive n of one row m per register quad; 12 operand reads of 16 bytes feed 16
// multiplications.
// The two waves of a SIMD take turns: a wave's step is a data phase (its operands out of LDS into
// registers, the staged tiles of the next step into the other LDS stage, new global loads) and a
// multiply phase (16 matrix instructions and nothing else), with a workgroup barrier after each;
// waves 4 .. 7 start half a step after waves 0 .. 3, so that on every SIMD one wave multiplies
// while the other moves data.  (With all waves in the same phase at the same time, as in a plain
// double-buffered loop, the memory instructions' time added to the matrix cores' instead of hiding
// under it.)  Row blocks past M and column groups past N are not multiplied.
// split_k > 1 (deep K, few output tiles: the MLP down projection) writes fp32 partials that a
// second kernel sums, adds the bias to and rounds.  With split_k = 1 and more tiles than the chip
// holds at once, the tiles of the last, partly filled round are split over K inside the same launch
// (their workgroups start as soon as slots free up), so that a round with few tiles does not cost a
// whole tile's time.  The gate/up projection of the MLP can apply SwiGLU in the epilogue: with the
// weight rows interleaved in blocks of 32 (gate block, up block), a lane holds gate and up of the
// same output element in two accumulators and writes silu(gate) * up directly.
// Steps of at most 16 rows (one or two sequences) are bound by reading W once and run on a second
// kernel, further down, that streams 16 weight rows per wave through the matrix cores.
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>

#include <mutex>

#include "ms_device.h"
#include "ms_internal.h"

namespace ms {

typedef __attribute__((ext_vector_type(8))) __bf16 g_bf16x8_t;
typedef __attribute__((ext_vector_type(16))) float g_f32x16_t;

constexpr int kGemmBM = 256, kGemmBN = 256, kGemmBK = 32;
constexpr int kGemmThreads = 512;
constexpr int kGemmRowBytes = kGemmBK * 2 + 16;                      // 80
constexpr int kGemmStageBytes = (kGemmBM + kGemmBN) * kGemmRowBytes;  // 40960
constexpr int kGemmLdsBytes = 2 * kGemmStageBytes;                   // above the 64 KB a kernel gets without asking
constexpr int kGemmColGroup = 64;                                    // columns of a wave: granularity of N and of the destinations
constexpr int kGemmMaxOut = 4;
constexpr int kGemmNUnit = 128;   // N and the destinations' boundaries are multiples of this

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

// The K loop of one wave for kMi row blocks of 32 that hold rows of the product (0: the wave only
// moves data and keeps the barriers' count).
template <int kMi>
__device__ __forceinline__ void gemm_k_loop(char* smem, const uint16_t* const (&a_src)[2], const uint16_t* const (&w_src)[2], char* a_dst,
                                            char* w_dst, int a_op, int w_op, int steps, int late, g_f32x16_t (&acc)[2][4]) {
    // Two register sets of staged tiles: while step s is multiplied, the tiles of step s + 1 are
    // stored to LDS and those of steps s + 2 and s + 3 are on their way.  Only LDS traffic is ordered
    // by the barriers, so a data phase waits for the oldest loads alone.
    // (plain named registers: aggregates handed around by name ended up in scratch memory)
    uint4 r0a0, r0a1, r0w0, r0w1;
    uint4 r1a0, r1a1, r1w0, r1w1;
#define MS_GEMM_FETCH(R, step_)                                                 \
    do {                                                                        \
        const int ko_ = (step_) * kGemmBK;                                      \
        R##a0 = *reinterpret_cast<const uint4*>(a_src[0] + ko_);                \
        R##a1 = *reinterpret_cast<const uint4*>(a_src[1] + ko_);                \
        R##w0 = *reinterpret_cast<const uint4*>(w_src[0] + ko_);                \
        R##w1 = *reinterpret_cast<const uint4*>(w_src[1] + ko_);                \
    } while (0)
#define MS_GEMM_STASH(R, buf_)                                                  \
    do {                                                                        \
        char* ad_ = a_dst + (buf_) * kGemmStageBytes;                           \
        char* wd_ = w_dst + (buf_) * kGemmStageBytes;                           \
        *reinterpret_cast<uint4*>(ad_) = R##a0;                                 \
        *reinterpret_cast<uint4*>(ad_ + 128 * kGemmRowBytes) = R##a1;           \
        *reinterpret_cast<uint4*>(wd_) = R##w0;                                 \
        *reinterpret_cast<uint4*>(wd_ + 128 * kGemmRowBytes) = R##w1;           \
    } while (0)
    // steps past the end re-read the last one (clamped): loads stay unconditional, nothing is used
    const int last = steps - 1;
#define MS_GEMM_CLAMP(s_) ((s_) < last ? (s_) : last)
    MS_GEMM_FETCH(r0, 0);
    MS_GEMM_FETCH(r1, MS_GEMM_CLAMP(1));
    MS_GEMM_STASH(r0, 0);
    MS_GEMM_FETCH(r0, MS_GEMM_CLAMP(2));
    gemm_lds_barrier();
    if (late) gemm_lds_barrier();   // waves 4 .. 7 run half a step behind waves 0 .. 3
    // One turn of a wave.  Data phase: the operands of step s out of LDS stage s & 1, the staged
    // tiles of step s + 1 (set NEXT) into the other stage - last read, as stage s - 1, by the late
    // waves one barrier ago -, the loads of step s + 3 requested into the freed set.  Barrier.
    // Multiply phase.  Barrier.  Every wave passes the same number of barriers (the early waves one
    // more at the end), and between two barriers one half of the waves is in its data phase, the
    // other in its multiply phase.  Stage s + 1 is complete one barrier after the late waves'
    // data phase of step s, which is when the early waves first read it.
    g_bf16x8_t wf[2][2], af[2][kMi > 0 ? kMi : 1];
#define MS_GEMM_TURN(step_, NEXT)                                                                                           \
    do {                                                                                                                    \
        const char* base_ = smem + ((step_) & 1) * kGemmStageBytes;                                                         \
        if (kMi > 0) {                                                                                                      \
            _Pragma("unroll") for (int kk = 0; kk < 2; ++kk) {                                                              \
                _Pragma("unroll") for (int ni = 0; ni < 2; ++ni) wf[kk][ni] = __builtin_bit_cast(                           \
                    g_bf16x8_t, *reinterpret_cast<const uint4*>(base_ + w_op + ni * 32 * kGemmRowBytes + 32 * kk));         \
                _Pragma("unroll") for (int mi = 0; mi < kMi; ++mi) af[kk][mi] = __builtin_bit_cast(                         \
                    g_bf16x8_t, *reinterpret_cast<const uint4*>(base_ + a_op + mi * 32 * kGemmRowBytes + 32 * kk));         \
            }                                                                                                               \
        }                                                                                                                   \
        MS_GEMM_STASH(NEXT, ((step_) + 1) & 1);                                                                             \
        MS_GEMM_FETCH(NEXT, MS_GEMM_CLAMP((step_) + 3));                                                                    \
        __builtin_amdgcn_sched_barrier(0);                                                                                  \
        gemm_lds_barrier();                                                                                                 \
        __builtin_amdgcn_sched_barrier(0);                                                                                  \
        __builtin_amdgcn_s_setprio(1);                                                                                      \
        _Pragma("unroll") for (int kk = 0; kk < 2; ++kk)                                                                    \
            _Pragma("unroll") for (int ni = 0; ni < 2; ++ni) _Pragma("unroll") for (int mi = 0; mi < kMi; ++mi)             \
                acc[ni][mi] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wf[kk][ni], af[kk][mi], acc[ni][mi], 0, 0, 0);        \
        __builtin_amdgcn_s_setprio(0);                                                                                      \
        __builtin_amdgcn_sched_barrier(0);                                                                                  \
        gemm_lds_barrier();                                                                                                 \
        __builtin_amdgcn_sched_barrier(0);                                                                                  \
    } while (0)
    int step = 0;
    for (; step + 2 <= steps; step += 2) {
        MS_GEMM_TURN(step, r1);
        MS_GEMM_TURN(step + 1, r0);
    }
    if (step < steps) MS_GEMM_TURN(step, r1);
    if (!late) gemm_lds_barrier();
#undef MS_GEMM_TURN
#undef MS_GEMM_CLAMP
#undef MS_GEMM_FETCH
#undef MS_GEMM_STASH
}

template <int kMode>
__global__ __launch_bounds__(kGemmThreads) void gemm_tn_bf16(GemmArgs g) {
    constexpr bool kSplit = kMode == kGemmAllPartial;
    extern __shared__ __attribute__((aligned(16))) char smem[];
    const int tid = threadIdx.x, lane = tid & 63, l32 = lane & 31, hf = lane >> 5;
    const int w = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm = w >> 2, wn = w & 3;                  // wave tile: rows 128 wm .. + 128, columns 64 wn .. + 64
    // Waves w and w + 4 of a workgroup share a SIMD (the hardware deals a workgroup's waves out to the
    // four SIMDs in turn): the two halves take turns at the matrix cores.
    const int late = wm;
    // Tile mapping.  Workgroups are handed to the 8 XCDs (each with its own L2) round robin, so
    // workgroups 8 apart share an L2: the row tiles of one column tile are placed 8 apart, and the
    // weight tile they share comes from HBM once.
    const int m_tiles = (g.M + kGemmBM - 1) / kGemmBM, n_tiles = (g.N + kGemmBN - 1) / kGemmBN;
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
    // 32-row blocks of this wave that hold rows of the product (0 if its columns lie past N)
    int mi_n = (g.M - m0 - 128 * wm + 31) / 32;
    mi_n = mi_n < 0 ? 0 : (mi_n > 4 ? 4 : mi_n);
    if (n0 + kGemmColGroup * wn >= g.N) mi_n = 0;

    // global -> LDS staging.  Four consecutive threads bring the 64 bytes one row contributes to a
    // step, so a load instruction of a wave covers 16 rows x 64 contiguous bytes; thread t handles
    // chunk t % 4 of activation rows r and r + 128 and of weight rows r and r + 128, r = t / 4 up to the
    // order below.  Rows past M or N are clamped (read again, never stored to the product).
    // Within each block of 16 rows the 4 x 4 (lane group, row) order is transposed: the 16 lanes that
    // store together then hold rows r, r + 4, r + 8, r + 12, whose 80-byte strides put their four
    // 16-byte chunks on 16 different groups of 4 banks (rows r .. r + 3 would collide two ways).
    const int sr_lin = tid >> 2, sc = tid & 3;
    const int sr = (sr_lin & ~15) | ((sr_lin & 3) << 2) | ((sr_lin >> 2) & 3);
    const uint16_t* a_src[2];
    const uint16_t* w_src[2];
#pragma unroll
    for (int i = 0; i < 2; ++i) {
        const int row = m0 + sr + 128 * i < g.M ? m0 + sr + 128 * i : g.M - 1;
        a_src[i] = g.a + (size_t)row * g.K + k_begin + 8 * sc;
        const int col = n0 + sr + 128 * i < g.N ? n0 + sr + 128 * i : g.N - 1;
        w_src[i] = g.w + (size_t)col * g.K + k_begin + 8 * sc;
    }
    char* a_dst = smem + sr * kGemmRowBytes + 16 * sc;
    char* w_dst = smem + kGemmBM * kGemmRowBytes + sr * kGemmRowBytes + 16 * sc;

    g_f32x16_t acc[2][4];
#pragma unroll
    for (int ni = 0; ni < 2; ++ni)
#pragma unroll
        for (int mi = 0; mi < 4; ++mi)
#pragma unroll
            for (int i = 0; i < 16; ++i) acc[ni][mi][i] = 0.f;

    // operand addresses inside a stage: 16 bytes at k = 16 kk + 8 (lane / 32) of row (lane % 32)
    const int a_op = (128 * wm + l32) * kGemmRowBytes + 16 * hf;
    const int w_op = kGemmBM * kGemmRowBytes + (kGemmColGroup * wn + l32) * kGemmRowBytes + 16 * hf;

    switch (mi_n) {   // uniform in the wave
        case 4: gemm_k_loop<4>(smem, a_src, w_src, a_dst, w_dst, a_op, w_op, steps, late, acc); break;
        case 3: gemm_k_loop<3>(smem, a_src, w_src, a_dst, w_dst, a_op, w_op, steps, late, acc); break;
        case 2: gemm_k_loop<2>(smem, a_src, w_src, a_dst, w_dst, a_op, w_op, steps, late, acc); break;
        case 1: gemm_k_loop<1>(smem, a_src, w_src, a_dst, w_dst, a_op, w_op, steps, late, acc); break;
        default: gemm_k_loop<0>(smem, a_src, w_src, a_dst, w_dst, a_op, w_op, steps, late, acc); break;
    }
    if (mi_n == 0) return;   // nothing of the product in this wave's tile (no barrier follows)

    // accumulator i of a lane: n = 8 (i / 4) + 4 (lane / 32) + i % 4, m = lane % 32 (within the 32 x 32 tile)
    if (to_partial) {
        const int p_col0 = kSplit ? 0 : g.tail_col0, p_ld = g.N - p_col0;
#pragma unroll
        for (int mi = 0; mi < 4; ++mi) {
            const int m = m0 + 128 * wm + 32 * mi + l32;
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
        for (int mi = 0; mi < 4; ++mi) {
            unsigned long long best = 0ull;
#pragma unroll
            for (int ni = 0; ni < 2; ++ni)
#pragma unroll
                for (int i = 0; i < 16; ++i)
                    best = key_max(best, argmax_key(acc[ni][mi][i], n0 + 64 * wn + 32 * ni + 8 * (i >> 2) + 4 * hf + (i & 3)));
            const uint32_t lo = __shfl_xor((int)(uint32_t)best, 32, 64), hi = __shfl_xor((int)(uint32_t)(best >> 32), 32, 64);
            best = key_max(best, ((unsigned long long)hi << 32) | lo);
            const int m = m0 + 128 * wm + 32 * mi + l32;
            if (m < g.M && hf == 0) g.keys[(size_t)(n_tile * 4 + wn) * g.M + m] = best;
        }
        return;
    }
    if (kMode == kGemmSwiglu) {
        // weight rows 64 wn .. + 32 of the tile are gate rows, the next 32 the matching up rows:
        // accumulators [0][mi] and [1][mi] hold gate and up of output column n0 / 2 + 32 wn + ...
#pragma unroll
        for (int mi = 0; mi < 4; ++mi) {
            const int m = m0 + 128 * wm + 32 * mi + l32;
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
    uint16_t* dst = nullptr;   // a wave's columns go to one destination: boundaries are multiples of 64
    int col0 = 0, ld = 0;
    pick_destination(g, n0 + kGemmColGroup * wn, dst, col0, ld);
#pragma unroll
    for (int mi = 0; mi < 4; ++mi) {
        const int m = m0 + 128 * wm + 32 * mi + l32;
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
    const float* p0 = g.partial + (size_t)m * width + n_rel;
    const size_t part_stride = (size_t)g.M * width;
    int z = 0;
    for (; z + 4 <= parts; z += 4) {   // four parts per memory round trip, added in their order
        float4 a[4], b[4];
#pragma unroll
        for (int t = 0; t < 4; ++t) {
            a[t] = *reinterpret_cast<const float4*>(p0 + (z + t) * part_stride);
            if (kSwiglu) b[t] = *reinterpret_cast<const float4*>(p0 + (z + t) * part_stride + 32);
        }
#pragma unroll
        for (int t = 0; t < 4; ++t) {
            s.x += a[t].x; s.y += a[t].y; s.z += a[t].z; s.w += a[t].w;
            if (kSwiglu) { u.x += b[t].x; u.y += b[t].y; u.z += b[t].z; u.w += b[t].w; }
        }
    }
    for (; z < parts; ++z) {
        const float4 a = *reinterpret_cast<const float4*>(p0 + z * part_stride);
        s.x += a.x; s.y += a.y; s.z += a.z; s.w += a.w;
        if (kSwiglu) {
            const float4 b = *reinterpret_cast<const float4*>(p0 + z * part_stride + 32);
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

// gemm_reduce over whole rows (no bias) and the decoder block's residual add + RMSNorm in one pass:
// delta = the K parts' sum rounded to bf16, h[row] += delta, out[row] = h[row] / sqrt(mean(h[row]^2)
// + eps) * weight.  One workgroup per row; same arithmetic in the same order as the two kernels it
// replaces (the same bits).  N a multiple of 8, at most 8192.
__global__ __launch_bounds__(kNormThreads) void reduce_add_rmsnorm(const float* __restrict__ partial, int parts, int M, int N,
                                                                    float* __restrict__ h, const uint16_t* __restrict__ weight,
                                                                    float eps, uint16_t* __restrict__ out) {
    __shared__ float red[kNormThreads / 64];
    const int row = blockIdx.x;
    float* hr = h + (size_t)row * N;
    float x[kNormMaxPerThread][8];
    uint4 wv[kNormMaxPerThread];
    float ss = 0.f;
#pragma unroll
    for (int t = 0; t < kNormMaxPerThread; ++t) {
        const int i = (t * kNormThreads + (int)threadIdx.x) * 8;
        if (i < N) {
            const float4 ha = *reinterpret_cast<const float4*>(hr + i), hb = *reinterpret_cast<const float4*>(hr + i + 4);
            wv[t] = *reinterpret_cast<const uint4*>(weight + i);
            float s[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
            const float* p = partial + (size_t)row * N + i;
            const size_t part_stride = (size_t)M * N;
            int z = 0;
            for (; z + 8 <= parts; z += 8) {   // eight parts per memory round trip, added in their order
                float4 a[8], b[8];
#pragma unroll
                for (int u = 0; u < 8; ++u) {
                    a[u] = *reinterpret_cast<const float4*>(p + (z + u) * part_stride);
                    b[u] = *reinterpret_cast<const float4*>(p + (z + u) * part_stride + 4);
                }
#pragma unroll
                for (int u = 0; u < 8; ++u) {
                    s[0] += a[u].x; s[1] += a[u].y; s[2] += a[u].z; s[3] += a[u].w;
                    s[4] += b[u].x; s[5] += b[u].y; s[6] += b[u].z; s[7] += b[u].w;
                }
            }
            for (; z < parts; ++z) {
                const float4 a = *reinterpret_cast<const float4*>(p + z * part_stride), b = *reinterpret_cast<const float4*>(p + z * part_stride + 4);
                s[0] += a.x; s[1] += a.y; s[2] += a.z; s[3] += a.w;
                s[4] += b.x; s[5] += b.y; s[6] += b.z; s[7] += b.w;
            }
            x[t][0] = ha.x; x[t][1] = ha.y; x[t][2] = ha.z; x[t][3] = ha.w;
            x[t][4] = hb.x; x[t][5] = hb.y; x[t][6] = hb.z; x[t][7] = hb.w;
#pragma unroll
            for (int e = 0; e < 8; ++e) x[t][e] += bf16_bits_to_float(float_to_bf16_bits(s[e]));
            *reinterpret_cast<float4*>(hr + i) = make_float4(x[t][0], x[t][1], x[t][2], x[t][3]);
            *reinterpret_cast<float4*>(hr + i + 4) = make_float4(x[t][4], x[t][5], x[t][6], x[t][7]);
#pragma unroll
            for (int e = 0; e < 8; ++e) ss += x[t][e] * x[t][e];
        }
    }
    const float rs = 1.0f / sqrtf(block_sum<kNormThreads>(ss, red) / (float)N + eps);
#pragma unroll
    for (int t = 0; t < kNormMaxPerThread; ++t) {
        const int i = (t * kNormThreads + (int)threadIdx.x) * 8;
        if (i < N) {
            const uint32_t w[4] = {wv[t].x, wv[t].y, wv[t].z, wv[t].w};
            uint32_t o[4];
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const float lo = x[t][2 * e] * rs * bf16_bits_to_float(w[e] & 0xffffu);
                const float hi = x[t][2 * e + 1] * rs * bf16_bits_to_float(w[e] >> 16);
                o[e] = (uint32_t)float_to_bf16_bits(lo) | ((uint32_t)float_to_bf16_bits(hi) << 16);
            }
            *reinterpret_cast<uint4*>(out + (size_t)row * N + i) = make_uint4(o[0], o[1], o[2], o[3]);
        }
    }
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
// At most 16 rows on the matrix cores (the step of one or two sequences).  The product is bound by
// reading W once, and the vector ALUs cannot keep up with 7 or more FMAs per weight (a kernel with
// fp32 FMAs per lane and a wave reduction at the end reached 2.2 to 3.9 TB/s at 7 rows), so W goes
// through v_mfma_f32_16x16x32_bf16: 16 weight rows are the A operand, the activations the B
// operand (columns = rows of A, padded to 16 by repeating the last one; from LDS, where the
// workgroup keeps its K range of A).  A tile of 16 weight rows x 128 K is loaded with four 16-byte
// loads per lane, each covering 256 contiguous bytes of four rows (loading the operand layout
// directly - one row per lane - ran at half the rate: every lane of a load then touches another
// cache line), passes through a wave-private LDS tile (row stride 272 bytes) and is read back in
// the operand layout (row = lane % 16, k = 8 (lane / 16) + 32 j for the j-th MFMA).  Per tile: four
// loads, four LDS writes, four (+ four for the activations) LDS reads, four MFMAs.  A workgroup is
// 4 waves: kWK of them split the K range of the same weight rows (summed through LDS at the end),
// 4 / kWK take different rows; a wave owns kNT tiles of 16 rows and keeps 16 loads (16 KB) in
// flight.  K ranges too long for the LDS are divided over `parts` workgroups (fp32 partials, summed
// by gemm_reduce).  kSwiglu (four tiles per wave = one gate block and one up block of the
// interleaved gate/up weight): the wave writes silu(gate) * up.
// ---------------------------------------------------------------------------------------------
constexpr int kSkinnyMaxRows = 16;
constexpr int kSkinnyStepK = 128;
constexpr int kSkinnyThreads = 256;
constexpr int kSkinnyTileRowBytes = kSkinnyStepK * 2 + 16;        // 272
constexpr int kSkinnyTileBytes = 16 * kSkinnyTileRowBytes;        // 4352 per wave
constexpr int kSkinnyLdsBytes = 76 * 1024;                        // two workgroups per compute unit
constexpr int kSkinnyLdsForA = kSkinnyLdsBytes - 4 * kSkinnyTileBytes;
// One workgroup per compute unit: room for all rows of A over the whole K of a wide projection at 9 to
// 16 rows (K = 3584: 115 KB), which then needs no K parts (and can apply SwiGLU in its epilogue).
constexpr int kSkinnyLdsBytesWide = 152 * 1024;
constexpr int kSkinnyLdsForAWide = kSkinnyLdsBytesWide - 4 * kSkinnyTileBytes;
typedef __attribute__((ext_vector_type(4))) float g_f32x4_t;

template <int kNT, int kWK, bool kSwiglu = false>
__global__ __launch_bounds__(kSkinnyThreads) void skinny_mfma_bf16(GemmArgs g, int parts) {
    static_assert(!kSwiglu || (kNT == 4 && kWK == 1), "SwiGLU: a wave owns 64 consecutive weight rows");
    constexpr int kDepth = 4 / kNT;            // K steps in flight: 16 loads per wave
    constexpr int kWN = 4 / kWK;
    extern __shared__ __attribute__((aligned(16))) char a_lds[];
    const int tid = threadIdx.x, lane = tid & 63, r = lane & 15, q = lane >> 4;
    const int w = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wn = w / kWK, wk = w % kWK;
    const int steps_total = g.K / kSkinnyStepK;
    const int part = blockIdx.y;
    const int p_lo = (int)((long)steps_total * part / parts), p_hi = (int)((long)steps_total * (part + 1) / parts);
    const int p_steps = p_hi - p_lo, kp = p_steps * kSkinnyStepK;
    // this wave's steps of the part
    const int s_lo = p_steps * wk / kWK, s_hi = p_steps * (wk + 1) / kWK;
    const int steps = s_hi - s_lo, last = steps > 0 ? steps - 1 : 0;
    const int n0 = ((int)blockIdx.x * kWN + wn) * (16 * kNT);
    // (a wave without steps, which the launch shapes in use never leave, would load the part's first step)
    // load i of a tile: row 4 i + lane / 16, 16 bytes at k = 8 (lane % 16)
    const uint16_t* wp = g.w + (size_t)(n0 + q) * g.K + (size_t)(p_lo + (steps > 0 ? s_lo : 0)) * kSkinnyStepK + 8 * r;
    const size_t tile_stride = (size_t)16 * g.K, quad_stride = (size_t)4 * g.K;
    // The workgroup's K range of A goes to LDS: [M][kp] bf16, rows 16 bytes further apart than their
    // length.  Its loads are issued first and the weight loads right behind them, so that waiting
    // for A (loads return in order) leaves the weights in flight.
    const int row_bytes = kp * 2 + 16;
    const int lds_a_bytes = (g.M * row_bytes + 15) & ~15;
    const int chunks = g.M * (kp / 8), row_chunks = kp / 8;
    constexpr int kStage = 16;                 // 16-byte chunks per thread in the first round (all of A at the sizes in use)
    uint4 sv[kStage];
#pragma unroll
    for (int u = 0; u < kStage; ++u) {
        const int c = tid + u * kSkinnyThreads < chunks ? tid + u * kSkinnyThreads : 0;
        sv[u] = *reinterpret_cast<const uint4*>(g.a + (size_t)(c / row_chunks) * g.K + (size_t)p_lo * kSkinnyStepK + 8 * (c % row_chunks));
    }
    uint4 wv[kDepth][kNT][4];
#define MS_SKINNY_LOAD(d_, s_)                                                                                 \
    do {                                                                                                       \
        const int sc_ = (s_) < last ? (s_) : last; /* past the end: the last step again, unused */             \
        _Pragma("unroll") for (int t = 0; t < kNT; ++t) _Pragma("unroll") for (int j = 0; j < 4; ++j)          \
            wv[d_][t][j] = __builtin_bit_cast(uint4, __builtin_nontemporal_load(reinterpret_cast<const g_u32x4_t*>( \
                wp + t * tile_stride + j * quad_stride + (size_t)sc_ * kSkinnyStepK)));                        \
    } while (0)
#pragma unroll
    for (int d = 0; d < kDepth; ++d) MS_SKINNY_LOAD(d, d);
#pragma unroll
    for (int u = 0; u < kStage; ++u) {
        const int c = tid + u * kSkinnyThreads;
        if (c < chunks) *reinterpret_cast<uint4*>(a_lds + (size_t)(c / row_chunks) * row_bytes + 16 * (c % row_chunks)) = sv[u];
    }
    for (int c0 = tid + kStage * kSkinnyThreads; c0 < chunks; c0 += 8 * kSkinnyThreads) {   // longer ranges: the rest, eight chunks a round
        uint4 v[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) {
            const int c = c0 + u * kSkinnyThreads < chunks ? c0 + u * kSkinnyThreads : c0;
            v[u] = *reinterpret_cast<const uint4*>(g.a + (size_t)(c / row_chunks) * g.K + (size_t)p_lo * kSkinnyStepK + 8 * (c % row_chunks));
        }
#pragma unroll
        for (int u = 0; u < 8; ++u) {
            const int c = c0 + u * kSkinnyThreads;
            if (c < chunks) *reinterpret_cast<uint4*>(a_lds + (size_t)(c / row_chunks) * row_bytes + 16 * (c % row_chunks)) = v[u];
        }
    }
    g_f32x4_t acc[kNT];
#pragma unroll
    for (int t = 0; t < kNT; ++t) acc[t] = g_f32x4_t{0.f, 0.f, 0.f, 0.f};
    __syncthreads();
    const char* ap = a_lds + (size_t)(r < g.M ? r : g.M - 1) * row_bytes + ((size_t)s_lo * kSkinnyStepK + 8 * q) * 2;
    char* tile = a_lds + lds_a_bytes + w * kSkinnyTileBytes;       // this wave's own
    char* tile_in = tile + q * kSkinnyTileRowBytes + 16 * r;       // as loaded: + 4 i rows
    const char* tile_out = tile + r * kSkinnyTileRowBytes + 16 * q;  // as multiplied: + 64 j bytes
#define MS_SKINNY_STEP(d_, s_)                                                                                 \
    do {                                                                                                       \
        g_bf16x8_t af[4];                                                                                      \
        _Pragma("unroll") for (int j = 0; j < 4; ++j)                                                          \
            af[j] = *reinterpret_cast<const g_bf16x8_t*>(ap + ((size_t)(s_) * kSkinnyStepK + 32 * j) * 2);     \
        _Pragma("unroll") for (int t = 0; t < kNT; ++t) {                                                      \
            _Pragma("unroll") for (int i = 0; i < 4; ++i)                                                      \
                *reinterpret_cast<uint4*>(tile_in + 4 * i * kSkinnyTileRowBytes) = wv[d_][t][i];               \
            g_bf16x8_t wf[4];                                                                                  \
            _Pragma("unroll") for (int j = 0; j < 4; ++j) wf[j] = *reinterpret_cast<const g_bf16x8_t*>(tile_out + 64 * j); \
            _Pragma("unroll") for (int j = 0; j < 4; ++j)                                                      \
                acc[t] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(wf[j], af[j], acc[t], 0, 0, 0);               \
        }                                                                                                      \
    } while (0)
    for (int s = 0; s < steps; s += kDepth) {
#pragma unroll
        for (int d = 0; d < kDepth; ++d) {
            if (s + d < steps) MS_SKINNY_STEP(d, s + d);
            MS_SKINNY_LOAD(d, s + d + kDepth);
        }
    }
#undef MS_SKINNY_STEP
#undef MS_SKINNY_LOAD
    if (kWK > 1) {   // the waves that split K: sums to the first of them, through the LDS
        __syncthreads();
        float* red = reinterpret_cast<float*>(a_lds);
        if (wk > 0) {
#pragma unroll
            for (int t = 0; t < kNT; ++t)
                *reinterpret_cast<g_f32x4_t*>(red + ((size_t)((wn * (kWK - 1) + wk - 1) * kNT + t) * 64 + lane) * 4) = acc[t];
        }
        __syncthreads();
        if (wk > 0) return;
#pragma unroll
        for (int o = 0; o < kWK - 1; ++o)
#pragma unroll
            for (int t = 0; t < kNT; ++t)
                acc[t] += *reinterpret_cast<const g_f32x4_t*>(red + ((size_t)((wn * (kWK - 1) + o) * kNT + t) * 64 + lane) * 4);
    }
    // lane: row m = r of A, columns n0 + 16 t + 4 q .. + 3
    const int m = r;
    if (g.keys) {   // greedy-token mode (parts == 1): the best of this wave's columns per row of A
        unsigned long long best = 0ull;
#pragma unroll
        for (int t = 0; t < kNT; ++t)
#pragma unroll
            for (int i = 0; i < 4; ++i) best = key_max(best, argmax_key(acc[t][i], n0 + 16 * t + 4 * q + i));
        best = key_max(best, __shfl_xor(best, 16));
        best = key_max(best, __shfl_xor(best, 32));
        if (q == 0 && m < g.M) g.keys[(size_t)(n0 / (16 * kNT)) * g.M + m] = best;
        return;
    }
    if (m >= g.M) return;
    if (kSwiglu) {   // rows n0 .. n0 + 31: gate of output columns n0 / 2 .. + 31, rows n0 + 32 .. + 63: up of the same
#pragma unroll
        for (int t = 0; t < 2; ++t) {
            uint2 pk;
            pk.x = g_pack_bf16x2(swiglu_value(acc[t][0], acc[t + 2][0]), swiglu_value(acc[t][1], acc[t + 2][1]));
            pk.y = g_pack_bf16x2(swiglu_value(acc[t][2], acc[t + 2][2]), swiglu_value(acc[t][3], acc[t + 2][3]));
            *reinterpret_cast<uint2*>(g.out[0] + (size_t)m * (g.N / 2) + n0 / 2 + 16 * t + 4 * q) = pk;
        }
        return;
    }
#pragma unroll
    for (int t = 0; t < kNT; ++t) {
        const int n = n0 + 16 * t + 4 * q;
        if (parts > 1) {
            *reinterpret_cast<g_f32x4_t*>(g.partial + ((size_t)part * g.M + m) * g.N + n) = acc[t];
            continue;
        }
        uint16_t* dst = nullptr;
        int col0 = 0, ld = 0;
        pick_destination(g, n, dst, col0, ld);
        float4 v = make_float4(acc[t][0], acc[t][1], acc[t][2], acc[t][3]);
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

static bool g_aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

// Twice the compute units of the current device (the few-row kernel's workgroups per round; the
// tiled kernel runs one workgroup per compute unit).
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
    p.n_groups = ((N + kGemmBN - 1) / kGemmBN + 7) / 8;
    p.group_blocks = 8 * p.m_tiles;
    p.main_groups = p.n_groups;
    p.tail_groups = 0;
    p.tail_split = 1;
    p.workspace_bytes = split_k > 1 ? (size_t)split_k * M * N * sizeof(float) : 0;
    if (split_k != 1) return p;
    const int per_round = gemm_slots() / 2 / p.group_blocks;
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

// At most 16 rows: the few-row kernel's launch shape (0 parts: shape not eligible).
struct SkinnyPlan {
    int parts, nt, wk, lds_bytes;
    size_t workspace_bytes;
};
static SkinnyPlan skinny_plan(int M, int N, int K, int min_parts = 1) {
    SkinnyPlan p = {0, 0, 0, 0, 0};
    if (M < 1 || M > kSkinnyMaxRows || K % kSkinnyStepK || N % 64) return p;
    const int steps = K / kSkinnyStepK;
    if (steps < min_parts) return p;
    // fewest K parts (from min_parts up) whose rows of A fit the LDS share
    int parts = min_parts;
    while (parts < steps && (long)M * (((steps + parts - 1) / parts) * kSkinnyStepK * 2 + 16) > kSkinnyLdsForA) ++parts;
    const int want = 2 * gemm_slots();   // waves that fill the memory pipeline with 16 KB in flight each
    const int n_tiles = N / 16;
    int nt = 1, wk = 1;
    // wide outputs whose rows of A fit a whole compute unit's LDS: one K part, one workgroup per compute unit
    const bool wide = parts > 1 && min_parts == 1 && N % 256 == 0 && N / 16 >= 2048 &&
                      (long)M * (K * 2 + 16) <= kSkinnyLdsForAWide;
    if (wide) {
        parts = 1;
        const int cus = gemm_slots() / 2;
        // workgroups of 64 nt rows: all at once if four tiles per wave allow it, else the split with the fullest last round
        double best = 0.0;
        for (int cand = 4; cand >= 1; cand /= 2) {
            const int wgs = N / (64 * cand);
            if (cand == 4 && wgs <= cus) { nt = 4; break; }
            const double fill = (double)wgs / ((wgs + cus - 1) / cus * cus);
            if (fill > best + 1e-9) { best = fill; nt = cand; }
        }
    } else if (parts > 1) {   // partials and a second kernel anyway: enough parts for about 1.75 x want waves (measured)
        const int more = (int)((7L * want / 4 + n_tiles - 1) / n_tiles);
        if (more > parts) parts = more < steps / 4 ? more : (steps / 4 > parts ? steps / 4 : parts);
    }
    if (wide) {
    } else if (N % 128 == 0 && (long)n_tiles / 2 * parts >= 4 * want) nt = 2;
    else if ((long)n_tiles * parts < want) wk = (long)n_tiles * parts * 2 >= want ? 2 : 4;
    while (wk > 1 && steps / parts < wk) wk /= 2;   // every wave gets a step
    p.parts = parts;
    p.nt = nt;
    p.wk = wk;
    const int a_bytes = ((M * (((steps + parts - 1) / parts) * kSkinnyStepK * 2 + 16) + 15) & ~15) + 4 * kSkinnyTileBytes;
    const int red_bytes = (4 / wk) * (wk - 1) * nt * 64 * 16;
    p.lds_bytes = a_bytes > red_bytes ? a_bytes : red_bytes;
    p.workspace_bytes = parts > 1 ? (size_t)parts * M * N * sizeof(float) : 0;
    return p;
}

static int skinny_dispatch(const GemmArgs& g, const SkinnyPlan& v, hipStream_t stream, bool swiglu = false) {
    static bool lds_allowed[64] = {};   // per device: the builds may use more than the default 64 KB of dynamic LDS
    int dev = 0;
    MS_HIP_TRY(hipGetDevice(&dev));
    if (dev < 0 || dev >= 64) MS_FAIL(MS_ERR_UNSUPPORTED, "ms_gemm_bf16: device index %d", dev);
    if (!lds_allowed[dev]) {
        const void* builds[] = {(const void*)skinny_mfma_bf16<4, 1>, (const void*)skinny_mfma_bf16<2, 1>, (const void*)skinny_mfma_bf16<1, 4>,
                                (const void*)skinny_mfma_bf16<1, 2>, (const void*)skinny_mfma_bf16<1, 1>,
                                (const void*)skinny_mfma_bf16<4, 1, true>};
        for (const void* f : builds) MS_HIP_TRY(hipFuncSetAttribute(f, hipFuncAttributeMaxDynamicSharedMemorySize, kSkinnyLdsBytesWide));
        lds_allowed[dev] = true;
    }
    const dim3 grid((unsigned)(g.N / (4 / v.wk * 16 * v.nt)), (unsigned)v.parts);
    const dim3 block(kSkinnyThreads);
    if (swiglu) hipLaunchKernelGGL((skinny_mfma_bf16<4, 1, true>), grid, block, v.lds_bytes, stream, g, v.parts);
    else if (v.nt == 4) hipLaunchKernelGGL((skinny_mfma_bf16<4, 1>), grid, block, v.lds_bytes, stream, g, v.parts);
    else if (v.nt == 2) hipLaunchKernelGGL((skinny_mfma_bf16<2, 1>), grid, block, v.lds_bytes, stream, g, v.parts);
    else if (v.wk == 4) hipLaunchKernelGGL((skinny_mfma_bf16<1, 4>), grid, block, v.lds_bytes, stream, g, v.parts);
    else if (v.wk == 2) hipLaunchKernelGGL((skinny_mfma_bf16<1, 2>), grid, block, v.lds_bytes, stream, g, v.parts);
    else hipLaunchKernelGGL((skinny_mfma_bf16<1, 1>), grid, block, v.lds_bytes, stream, g, v.parts);
    return MS_OK;
}

static int gemm_check_shape(const char* what, int M, int N, int K, int split_k) {
    if (M < 0 || N < 1 || K < 1 || split_k < 1) MS_FAIL(MS_ERR_INVALID, "%s: bad size", what);
    if (N % kGemmNUnit || K % (kGemmBK * split_k))
        MS_FAIL(MS_ERR_UNSUPPORTED, "%s: N must be a multiple of %d and K of %d x split_k", what, kGemmNUnit, kGemmBK);
    if ((long long)M * N >= (1ll << 40) || split_k > 64 ||
        (long long)((N / kGemmNUnit + 7) / 8) * 8 * ((M + kGemmBM - 1) / kGemmBM) * 9 > 2000000000ll)
        MS_FAIL(MS_ERR_UNSUPPORTED, "%s: shape too large", what);
    return MS_OK;
}

// What follows the down projection in a decoder block: with it, the product always goes through fp32
// partials and reduce_add_rmsnorm takes the place of gemm_reduce.
struct NormTail {
    float* h;
    const uint16_t* weight;
    float eps;
    uint16_t* out;
};

// The tiled kernel's two LDS stages (80 KB) are above the default limit: allowed once per device.
static int gemm_allow_lds() {
    static std::once_flag once[64];
    static hipError_t result[64];
    int dev = 0;
    MS_HIP_TRY(hipGetDevice(&dev));
    if (dev < 0 || dev >= 64) MS_FAIL(MS_ERR_UNSUPPORTED, "device index %d outside [0, 64)", dev);
    std::call_once(once[dev], [&] {
        hipError_t e = hipSuccess;
        const void* builds[] = {(const void*)gemm_tn_bf16<kGemmPlain>, (const void*)gemm_tn_bf16<kGemmAllPartial>,
                                (const void*)gemm_tn_bf16<kGemmSwiglu>, (const void*)gemm_tn_bf16<kGemmArgmax>};
        for (const void* f : builds)
            if (e == hipSuccess) e = hipFuncSetAttribute(f, hipFuncAttributeMaxDynamicSharedMemorySize, kGemmLdsBytes);
        result[dev] = e;
    });
    if (result[dev] != hipSuccess) MS_FAIL(MS_ERR_HIP, "hipFuncSetAttribute(MaxDynamicSharedMemorySize) failed: %s", hipGetErrorString(result[dev]));
    return MS_OK;
}

// Launches the tiles (and the reduction of the parts, if any).  g holds operands and destinations.
static int gemm_launch(GemmArgs& g, int split_k, bool swiglu, void* workspace, size_t ws_bytes, hipStream_t stream,
                       const NormTail* norm = nullptr) {
    if (swiglu) {   // few rows: four tiles per wave, the whole K in one part
        SkinnyPlan sk = skinny_plan(g.M, g.N, g.K);
        if (sk.parts == 1 && g.N % 256 == 0) {
            sk.nt = 4;
            sk.wk = 1;
            g.k_per_split = g.K;
            g.partial = nullptr;
            g.tail_first = g.tail_blocks = g.tail_k = g.tail_col0 = 0;
            if (int rc = skinny_dispatch(g, sk, stream, true)) return rc;
            MS_HIP_TRY(hipGetLastError());
            return MS_OK;
        }
    } else {
        const SkinnyPlan sk = skinny_plan(g.M, g.N, g.K, norm ? 2 : 1);
        if (sk.parts == 1 || (sk.parts > 1 && workspace && ws_bytes >= sk.workspace_bytes && g_aligned16(workspace))) {
            g.k_per_split = g.K;
            g.partial = sk.parts > 1 ? (float*)workspace : nullptr;
            g.tail_first = g.tail_blocks = g.tail_k = g.tail_col0 = 0;
            if (int rc = skinny_dispatch(g, sk, stream)) return rc;
            if (norm) {
                hipLaunchKernelGGL(reduce_add_rmsnorm, dim3((unsigned)g.M), dim3(kNormThreads), 0, stream, (const float*)g.partial,
                                   sk.parts, g.M, g.N, norm->h, norm->weight, norm->eps, norm->out);
            } else if (sk.parts > 1) {
                const size_t quads = (size_t)g.M * g.N / 4;
                hipLaunchKernelGGL((gemm_reduce<false>), dim3((unsigned)((quads + 255) / 256)), dim3(256), 0, stream, g, sk.parts, 0);
            }
            MS_HIP_TRY(hipGetLastError());
            return MS_OK;
        }
    }
    if (int rc = gemm_allow_lds()) return rc;
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
        hipLaunchKernelGGL((gemm_tn_bf16<kGemmAllPartial>), grid, dim3(kGemmThreads), kGemmLdsBytes, stream, g);
        if (norm) {
            hipLaunchKernelGGL(reduce_add_rmsnorm, dim3((unsigned)g.M), dim3(kNormThreads), 0, stream, (const float*)g.partial, split_k,
                               g.M, g.N, norm->h, norm->weight, norm->eps, norm->out);
        } else {
            const size_t quads = (size_t)g.M * g.N / 4;
            hipLaunchKernelGGL((gemm_reduce<false>), dim3((unsigned)((quads + 255) / 256)), dim3(256), 0, stream, g, split_k, 0);
        }
    } else {
        if (norm) MS_FAIL(MS_ERR_INVALID, "ms_gemm_add_rmsnorm_bf16: split_k >= 2 needed above %d rows", kSkinnyMaxRows);
        if (p.tail_groups) g.partial = (float*)workspace;
        if (swiglu)
            hipLaunchKernelGGL((gemm_tn_bf16<kGemmSwiglu>), grid, dim3(kGemmThreads), kGemmLdsBytes, stream, g);
        else
            hipLaunchKernelGGL((gemm_tn_bf16<kGemmPlain>), grid, dim3(kGemmThreads), kGemmLdsBytes, stream, g);
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
    if (M < 1 || N < 1 || K < 1 || split_k < 1 || N % ms::kGemmNUnit || K % (ms::kGemmBK * split_k)) return 0;
    const size_t tiled = ms::gemm_plan(M, N, K, split_k).workspace_bytes;
    const size_t few = ms::skinny_plan(M, N, K).workspace_bytes;   // enough for either kernel
    return tiled > few ? tiled : few;
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
        if (out_col[i + 1] <= out_col[i] || out_col[i] % kGemmNUnit || !out[i] || (reinterpret_cast<uintptr_t>(out[i]) & 7u) ||
            (out_col[i + 1] - out_col[i]) % 4)
            MS_FAIL(MS_ERR_INVALID, "ms_gemm_bf16: destination %d: boundaries must rise in multiples of %d, pointers be 8-byte aligned", i, kGemmNUnit);
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

extern "C" size_t ms_gemm_add_rmsnorm_workspace_bytes(int M, int N, int K, int split_k) {
    if (M < 1 || N < 1 || K < 1 || split_k < 1 || N % ms::kGemmNUnit || K % (ms::kGemmBK * split_k)) return 0;
    const size_t tiled = split_k > 1 ? ms::gemm_plan(M, N, K, split_k).workspace_bytes : 0;
    const size_t few = ms::skinny_plan(M, N, K, 2).workspace_bytes;
    return tiled > few ? tiled : few;
}

extern "C" int ms_gemm_add_rmsnorm_bf16(const void* a, const void* w, int M, int N, int K, int split_k, float* h,
                                        const void* norm_weight, float eps, void* out, void* workspace, size_t ws_bytes,
                                        void* stream) {
    using namespace ms;
    int rc = gemm_check_shape("ms_gemm_add_rmsnorm_bf16", M, N, K, split_k);
    if (rc != MS_OK) return rc;
    if (N > kNormMaxPerThread * kNormThreads * 8 || !(eps >= 0.f))
        MS_FAIL(MS_ERR_INVALID, "ms_gemm_add_rmsnorm_bf16: need N up to %d and eps >= 0", kNormMaxPerThread * kNormThreads * 8);
    if (M == 0) return MS_OK;
    if (!a || !w || !h || !norm_weight || !out || !g_aligned16(a) || !g_aligned16(w) || !g_aligned16(h) ||
        !g_aligned16(norm_weight) || !g_aligned16(out))
        MS_FAIL(MS_ERR_INVALID, "ms_gemm_add_rmsnorm_bf16: null or misaligned (16 bytes) argument");
    const size_t need = ms_gemm_add_rmsnorm_workspace_bytes(M, N, K, split_k);
    if (!need) MS_FAIL(MS_ERR_INVALID, "ms_gemm_add_rmsnorm_bf16: split_k >= 2 needed for this shape");
    if (!workspace || ws_bytes < need || !g_aligned16(workspace))
        MS_FAIL(MS_ERR_WORKSPACE, "ms_gemm_add_rmsnorm_bf16: workspace of %zu bytes needed", need);
    GemmArgs g;
    g.a = (const uint16_t*)a;
    g.w = (const uint16_t*)w;
    g.bias = nullptr;
    g.keys = nullptr;
    g.M = M;
    g.N = N;
    g.K = K;
    g.n_out = 1;
    g.out[0] = (uint16_t*)out;   // not written by the product itself
    g.out_col[0] = 0;
    for (int i = 1; i < kGemmMaxOut; ++i) g.out[i] = nullptr;
    for (int i = 1; i <= kGemmMaxOut; ++i) g.out_col[i] = N;
    const NormTail tail = {h, (const uint16_t*)norm_weight, eps, (uint16_t*)out};
    return gemm_launch(g, split_k, false, workspace, ws_bytes, (hipStream_t)stream, &tail);
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
    const ms::SkinnyPlan sk = ms::skinny_plan(M, N, K);
    return sk.parts == 1 ? N / (16 * sk.nt) : N / ms::kGemmColGroup;
}

extern "C" size_t ms_lm_head_argmax_workspace_bytes(int M, int vocab, int K) {
    if (M < 1 || vocab < 1 || K < 1 || vocab % ms::kGemmNUnit || K % ms::kGemmBK) return 0;
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
    const SkinnyPlan sk = skinny_plan(M, vocab, K);
    if (sk.parts == 1) {
        g.tail_first = g.tail_blocks = g.tail_k = g.tail_col0 = 0;
        rc = skinny_dispatch(g, sk, stream);
        if (rc != MS_OK) return rc;
    } else {
        rc = gemm_allow_lds();
        if (rc != MS_OK) return rc;
        const GemmPlan p = gemm_plan(M, vocab, K, 1);
        const int blocks = p.n_groups * p.group_blocks;   // whole tiles throughout
        g.tail_first = blocks;
        g.tail_blocks = 0;
        g.tail_k = K;
        g.tail_col0 = vocab;
        hipLaunchKernelGGL((gemm_tn_bf16<kGemmArgmax>), dim3((unsigned)blocks), dim3(kGemmThreads), kGemmLdsBytes, stream, g);
    }
    hipLaunchKernelGGL(argmax_finish, dim3((unsigned)M), dim3(256), 0, stream, (const unsigned long long*)workspace, groups, M, out);
    MS_HIP_TRY(hipGetLastError());
    return MS_OK;
}
