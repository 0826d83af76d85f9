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
// second kernel sums, adds the bias to and rounds.
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
    float* partial;         // [split_k][M][N] when split_k > 1
};

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

// Workgroup barrier that orders LDS traffic only (a plain __syncthreads() would also wait for the
// global loads of the steps ahead).
__device__ __forceinline__ void gemm_lds_barrier() {
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup", "local");
    __builtin_amdgcn_s_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup", "local");
}

template <bool kSplit>
__global__ __launch_bounds__(kGemmThreads, 2) void gemm_tn_bf16(GemmArgs g) {
    __shared__ __attribute__((aligned(16))) char smem[2 * kGemmStageBytes];
    const int tid = threadIdx.x, lane = tid & 63, l32 = lane & 31, hf = lane >> 5;
    const int w = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm = w >> 1, wn = w & 1;                  // wave tile: rows 64 wm .. + 64, columns 64 wn .. + 64
    // Tile mapping.  Workgroups are handed to the 8 XCDs (each with its own L2) round robin, so
    // workgroups 8 apart share an L2: the row tiles of one column tile are placed 8 apart, and the
    // weight tile they share comes from HBM once.
    const int m_tiles = (g.M + kGemmBM - 1) / kGemmBM, n_tiles = g.N / kGemmBN;
    const int in_group = blockIdx.x % (8 * m_tiles);
    const int n_tile = blockIdx.x / (8 * m_tiles) * 8 + in_group % 8, m_tile = in_group / 8;
    if (n_tile >= n_tiles) return;   // padding of the last group (the whole workgroup leaves)
    const int n0 = n_tile * kGemmBN, m0 = m_tile * kGemmBM;
    const int k_begin = blockIdx.z * g.k_per_split;
    const int steps = g.k_per_split / kGemmBK;

    // global -> LDS staging.  Four consecutive threads bring the 64 bytes one row contributes to a
    // step, so a load instruction of a wave covers 16 rows x 64 contiguous bytes; thread t handles
    // chunk t % 4 of activation rows t / 4 and t / 4 + 128 and of weight row t / 4.
    // Rows past M are clamped (read again, never stored).
    const int sr = tid >> 2, sc = tid & 3;
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
    uint16_t* dst = nullptr;   // the whole tile goes to one destination: boundaries are multiples of 128
    int col0 = 0, ld = 0;
    if (!kSplit) pick_destination(g, n0, dst, col0, ld);
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
                if (kSplit) {
                    *reinterpret_cast<float4*>(g.partial + ((size_t)blockIdx.z * g.M + m) * g.N + n) = v;
                } else {
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
}

// Sums the split-K partials, adds the bias, rounds to bf16 and writes to the destination(s).
__global__ __launch_bounds__(256) void gemm_reduce(GemmArgs g, int split_k) {
    const size_t idx = ((size_t)blockIdx.x * 256 + threadIdx.x) * 4;   // 4 consecutive columns
    if (idx >= (size_t)g.M * g.N) return;
    const int m = (int)(idx / g.N), n = (int)(idx % g.N);
    float4 s = make_float4(0.f, 0.f, 0.f, 0.f);
    for (int z = 0; z < split_k; ++z) {
        const float4 p = *reinterpret_cast<const float4*>(g.partial + ((size_t)z * g.M + m) * g.N + n);
        s.x += p.x; s.y += p.y; s.z += p.z; s.w += p.w;
    }
    if (g.bias) {
        const uint2 b = *reinterpret_cast<const uint2*>(g.bias + n);
        s.x += bf16_bits_to_float(b.x & 0xffffu);
        s.y += bf16_bits_to_float(b.x >> 16);
        s.z += bf16_bits_to_float(b.y & 0xffffu);
        s.w += bf16_bits_to_float(b.y >> 16);
    }
    uint16_t* dst;
    int col0, ld;
    pick_destination(g, n, dst, col0, ld);
    uint2 pk;
    pk.x = g_pack_bf16x2(s.x, s.y);
    pk.y = g_pack_bf16x2(s.z, s.w);
    *reinterpret_cast<uint2*>(dst + (size_t)m * ld + (n - col0)) = pk;
}

static bool g_aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

}  // namespace ms

extern "C" size_t ms_gemm_workspace_bytes(int M, int N, int split_k) {
    if (M < 1 || N < 1 || split_k < 2) return 0;
    return (size_t)split_k * M * N * sizeof(float);
}

extern "C" int ms_gemm_bf16(const void* a, const void* w, const void* bias, int M, int N, int K, int n_out, void* const* out,
                            const int* out_col, int split_k, void* workspace, size_t ws_bytes, void* stream) {
    using namespace ms;
    if (M < 0 || N < 1 || K < 1 || split_k < 1 || n_out < 1 || n_out > kGemmMaxOut || !out || !out_col)
        MS_FAIL(MS_ERR_INVALID, "ms_gemm_bf16: bad size or null table");
    if (M == 0) return MS_OK;
    if (N % kGemmBN || K % (kGemmBK * split_k))
        MS_FAIL(MS_ERR_UNSUPPORTED, "ms_gemm_bf16: N must be a multiple of %d and K of %d x split_k", kGemmBN, kGemmBK);
    if ((long long)M * N >= (1ll << 40) || split_k > 64 ||
        (long long)((N / kGemmBN + 7) / 8) * 8 * ((M + kGemmBM - 1) / kGemmBM) > 2000000000ll)
        MS_FAIL(MS_ERR_UNSUPPORTED, "ms_gemm_bf16: shape too large");
    if (!a || !w || !g_aligned16(a) || !g_aligned16(w) || (bias && (reinterpret_cast<uintptr_t>(bias) & 7u)))
        MS_FAIL(MS_ERR_INVALID, "ms_gemm_bf16: null or misaligned operand");
    GemmArgs g;
    g.a = (const uint16_t*)a;
    g.w = (const uint16_t*)w;
    g.bias = (const uint16_t*)bias;
    g.M = M;
    g.N = N;
    g.K = K;
    g.k_per_split = K / split_k;
    g.n_out = n_out;
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
    g.partial = nullptr;
    const int m_tiles = (M + kGemmBM - 1) / kGemmBM, n_groups = (N / kGemmBN + 7) / 8;
    const dim3 grid((unsigned)(n_groups * 8 * m_tiles), 1, split_k);
    if (split_k == 1) {
        hipLaunchKernelGGL(gemm_tn_bf16<false>, grid, dim3(kGemmThreads), 0, (hipStream_t)stream, g);
    } else {
        const size_t need = ms_gemm_workspace_bytes(M, N, split_k);
        if (!workspace || ws_bytes < need || !g_aligned16(workspace))
            MS_FAIL(MS_ERR_WORKSPACE, "ms_gemm_bf16: split-K workspace of %zu bytes needed", need);
        g.partial = (float*)workspace;
        hipLaunchKernelGGL(gemm_tn_bf16<true>, grid, dim3(kGemmThreads), 0, (hipStream_t)stream, g);
        const size_t quads = (size_t)M * N / 4;
        hipLaunchKernelGGL(gemm_reduce, dim3((unsigned)((quads + 255) / 256)), dim3(256), 0, (hipStream_t)stream, g, split_k);
    }
    MS_HIP_TRY(hipGetLastError());
    return MS_OK;
}
