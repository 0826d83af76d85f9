// Memory-bound pieces of the decoder block around the attention, for the full decode step
// (MemoSight paper, Appendix A, Algorithm 1: SpeculativeStep runs the model once over the verify
// and foresight tokens; Section 3.1 names the models, whose block is pre-norm RMSNorm, attention,
// SwiGLU MLP): embedding rows, residual add + RMSNorm, SiLU(gate) * up, and the greedy token of
// every logits row.  The dense projections are GEMMs and live outside this file.
//
// Activations are bf16, the residual stream is kept in fp32, all arithmetic is fp32.
#include <math.h>

#include "ms_device.h"
#include "ms_internal.h"

namespace ms {

constexpr int kRowThreads = 256;

// h[row] = table[tokens[row]] widened to fp32.  One workgroup per row, 8 elements per thread and turn.
__global__ __launch_bounds__(kRowThreads) void embed_rows(const uint16_t* __restrict__ table, int vocab, int hidden,
                                                           const int* __restrict__ tokens, float* __restrict__ h) {
    const int row = blockIdx.x;
    int tok = tokens[row];
    tok = tok < 0 ? 0 : (tok >= vocab ? vocab - 1 : tok);   // ids are validated by the caller; never read outside
    const uint16_t* src = table + (size_t)tok * hidden;
    float* dst = h + (size_t)row * hidden;
    for (int i = threadIdx.x * 8; i < hidden; i += kRowThreads * 8) {
        const uint4 v = *reinterpret_cast<const uint4*>(src + i);
        const uint32_t w[4] = {v.x, v.y, v.z, v.w};
        float4 lo, hi;
        lo.x = bf16_bits_to_float(w[0] & 0xffffu);
        lo.y = bf16_bits_to_float(w[0] >> 16);
        lo.z = bf16_bits_to_float(w[1] & 0xffffu);
        lo.w = bf16_bits_to_float(w[1] >> 16);
        hi.x = bf16_bits_to_float(w[2] & 0xffffu);
        hi.y = bf16_bits_to_float(w[2] >> 16);
        hi.z = bf16_bits_to_float(w[3] & 0xffffu);
        hi.w = bf16_bits_to_float(w[3] >> 16);
        *reinterpret_cast<float4*>(dst + i) = lo;
        *reinterpret_cast<float4*>(dst + i + 4) = hi;
    }
}

// h[row] += delta[row] (if given); out[row] = h[row] / sqrt(mean(h[row]^2) + eps) * weight.
// One workgroup per row; the row is read once (kept in registers between the two passes); all loads
// are issued before the first wait (with a few rows the kernel is one memory round trip long).
__global__ __launch_bounds__(kNormThreads) void add_rmsnorm(float* __restrict__ h, const uint16_t* __restrict__ delta,
                                                             const uint16_t* __restrict__ weight, float eps,
                                                             uint16_t* __restrict__ out, int hidden) {
    __shared__ float red[kNormThreads / 64];
    const int row = blockIdx.x;
    float* hr = h + (size_t)row * hidden;
    float x[kNormMaxPerThread][8];
    uint4 wv[kNormMaxPerThread], dv[kNormMaxPerThread];
#pragma unroll
    for (int t = 0; t < kNormMaxPerThread; ++t) {
        const int i = (t * kNormThreads + (int)threadIdx.x) * 8;
        if (i < hidden) {
            const float4 a = *reinterpret_cast<const float4*>(hr + i), b = *reinterpret_cast<const float4*>(hr + i + 4);
            x[t][0] = a.x; x[t][1] = a.y; x[t][2] = a.z; x[t][3] = a.w;
            x[t][4] = b.x; x[t][5] = b.y; x[t][6] = b.z; x[t][7] = b.w;
            wv[t] = *reinterpret_cast<const uint4*>(weight + i);
            if (delta) dv[t] = *reinterpret_cast<const uint4*>(delta + (size_t)row * hidden + i);
        }
    }
    float ss = 0.f;
#pragma unroll
    for (int t = 0; t < kNormMaxPerThread; ++t) {
        const int i = (t * kNormThreads + (int)threadIdx.x) * 8;
        if (i < hidden) {
            if (delta) {
                const uint32_t w[4] = {dv[t].x, dv[t].y, dv[t].z, dv[t].w};
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    x[t][2 * e] += bf16_bits_to_float(w[e] & 0xffffu);
                    x[t][2 * e + 1] += bf16_bits_to_float(w[e] >> 16);
                }
                *reinterpret_cast<float4*>(hr + i) = make_float4(x[t][0], x[t][1], x[t][2], x[t][3]);
                *reinterpret_cast<float4*>(hr + i + 4) = make_float4(x[t][4], x[t][5], x[t][6], x[t][7]);
            }
#pragma unroll
            for (int e = 0; e < 8; ++e) ss += x[t][e] * x[t][e];
        }
    }
    const float rs = 1.0f / sqrtf(block_sum<kNormThreads>(ss, red) / (float)hidden + eps);
#pragma unroll
    for (int t = 0; t < kNormMaxPerThread; ++t) {
        const int i = (t * kNormThreads + (int)threadIdx.x) * 8;
        if (i < hidden) {
            const uint32_t w[4] = {wv[t].x, wv[t].y, wv[t].z, wv[t].w};
            uint32_t o[4];
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const float lo = x[t][2 * e] * rs * bf16_bits_to_float(w[e] & 0xffffu);
                const float hi = x[t][2 * e + 1] * rs * bf16_bits_to_float(w[e] >> 16);
                o[e] = (uint32_t)float_to_bf16_bits(lo) | ((uint32_t)float_to_bf16_bits(hi) << 16);
            }
            *reinterpret_cast<uint4*>(out + (size_t)row * hidden + i) = make_uint4(o[0], o[1], o[2], o[3]);
        }
    }
}

// out[row][i] = silu(gate_up[row][i]) * gate_up[row][inter + i], 8 elements per thread.
__global__ __launch_bounds__(kRowThreads) void swiglu(const uint16_t* __restrict__ gate_up, uint16_t* __restrict__ out,
                                                       int inter) {
    const int row = blockIdx.y;
    const int i = (blockIdx.x * kRowThreads + threadIdx.x) * 8;
    if (i >= inter) return;
    const uint16_t* g = gate_up + (size_t)row * 2 * inter + i;
    const uint4 gv = *reinterpret_cast<const uint4*>(g), uv = *reinterpret_cast<const uint4*>(g + inter);
    const uint32_t gw[4] = {gv.x, gv.y, gv.z, gv.w}, uw[4] = {uv.x, uv.y, uv.z, uv.w};
    uint32_t o[4];
#pragma unroll
    for (int e = 0; e < 4; ++e) {
        float r[2];
#pragma unroll
        for (int hh = 0; hh < 2; ++hh) {
            const float a = bf16_bits_to_float(hh ? gw[e] >> 16 : gw[e] & 0xffffu);
            const float b = bf16_bits_to_float(hh ? uw[e] >> 16 : uw[e] & 0xffffu);
            r[hh] = a / (1.0f + expf(-a)) * b;
        }
        o[e] = (uint32_t)float_to_bf16_bits(r[0]) | ((uint32_t)float_to_bf16_bits(r[1]) << 16);
    }
    *reinterpret_cast<uint4*>(out + (size_t)row * inter + i) = make_uint4(o[0], o[1], o[2], o[3]);
}

// Greedy token of a logits row: the largest value, the lowest index among equals; NaN never wins.
__device__ __forceinline__ void take_better(float& bv, int& bi, float v, int i) {
    if (v > bv || (v == bv && i < bi)) {
        bv = v;
        bi = i;
    }
}
__global__ __launch_bounds__(kRowThreads) void argmax_rows(const uint16_t* __restrict__ logits, int vocab, long ld,
                                                            int* __restrict__ out) {
    __shared__ float rv[kRowThreads / 64];
    __shared__ int ri[kRowThreads / 64];
    const uint16_t* row = logits + (size_t)blockIdx.x * ld;
    float bv = -INFINITY;
    int bi = 0x7fffffff;
    const int vec_end = vocab & ~7;
    // four chunks per turn, each with a candidate of its own: four loads in flight and four
    // independent compare chains instead of one (take_better keeps the lower index among equals,
    // so the order in which candidates are folded does not matter)
    constexpr int kWays = 4;
    float cv[kWays];
    int ci[kWays];
#pragma unroll
    for (int u = 0; u < kWays; ++u) {
        cv[u] = -INFINITY;
        ci[u] = 0x7fffffff;
    }
    int i = threadIdx.x * 8;
    for (; i + (kWays - 1) * kRowThreads * 8 < vec_end; i += kWays * kRowThreads * 8) {
        uint4 v[kWays];
#pragma unroll
        for (int u = 0; u < kWays; ++u) v[u] = *reinterpret_cast<const uint4*>(row + i + u * kRowThreads * 8);
#pragma unroll
        for (int u = 0; u < kWays; ++u) {
            const uint32_t w[4] = {v[u].x, v[u].y, v[u].z, v[u].w};
            const int at = i + u * kRowThreads * 8;
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                take_better(cv[u], ci[u], bf16_bits_to_float(w[e] & 0xffffu), at + 2 * e);
                take_better(cv[u], ci[u], bf16_bits_to_float(w[e] >> 16), at + 2 * e + 1);
            }
        }
    }
#pragma unroll
    for (int u = 0; u < kWays; ++u) take_better(bv, bi, cv[u], ci[u]);
    for (; i < vec_end; i += kRowThreads * 8) {
        const uint4 v = *reinterpret_cast<const uint4*>(row + i);
        const uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            take_better(bv, bi, bf16_bits_to_float(w[e] & 0xffffu), i + 2 * e);
            take_better(bv, bi, bf16_bits_to_float(w[e] >> 16), i + 2 * e + 1);
        }
    }
    for (int i = vec_end + threadIdx.x; i < vocab; i += kRowThreads) take_better(bv, bi, bf16_bits_to_float(row[i]), i);
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) take_better(bv, bi, __shfl_xor(bv, o, 64), __shfl_xor(bi, o, 64));
    const int w = threadIdx.x >> 6;
    if ((threadIdx.x & 63) == 0) {
        rv[w] = bv;
        ri[w] = bi;
    }
    __syncthreads();
    if (threadIdx.x == 0) {
#pragma unroll
        for (int k = 1; k < kRowThreads / 64; ++k) take_better(bv, bi, rv[k], ri[k]);
        out[blockIdx.x] = bi == 0x7fffffff ? 0 : bi;   // a row of NaN / -inf only: token 0
    }
}

static bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

}  // namespace ms

extern "C" int ms_embed_rows(const void* table, int vocab, int hidden, const int* tokens, int n, float* h_out, void* stream) {
    if (n < 0 || vocab < 1 || hidden < 8 || hidden % 8) MS_FAIL(MS_ERR_INVALID, "ms_embed_rows: need hidden a multiple of 8, vocab >= 1");
    if (n == 0) return MS_OK;
    if (!table || !tokens || !h_out || !ms::aligned16(table) || !ms::aligned16(h_out))
        MS_FAIL(MS_ERR_INVALID, "ms_embed_rows: null or misaligned (16 bytes) argument");
    hipLaunchKernelGGL(ms::embed_rows, dim3(n), dim3(ms::kRowThreads), 0, (hipStream_t)stream, (const uint16_t*)table, vocab,
                       hidden, tokens, h_out);
    MS_HIP_TRY(hipGetLastError());
    return MS_OK;
}

extern "C" int ms_add_rmsnorm(float* h, const void* delta, const void* weight, float eps, void* out, int n, int hidden,
                              void* stream) {
    if (n < 0 || hidden < 8 || hidden % 8 || hidden > ms::kNormMaxPerThread * ms::kNormThreads * 8 || !(eps >= 0.f))
        MS_FAIL(MS_ERR_INVALID, "ms_add_rmsnorm: need hidden a multiple of 8 up to %d and eps >= 0",
                ms::kNormMaxPerThread * ms::kNormThreads * 8);
    if (n == 0) return MS_OK;
    if (!h || !weight || !out || !ms::aligned16(h) || !ms::aligned16(weight) || !ms::aligned16(out) || !ms::aligned16(delta))
        MS_FAIL(MS_ERR_INVALID, "ms_add_rmsnorm: null or misaligned (16 bytes) argument");
    hipLaunchKernelGGL(ms::add_rmsnorm, dim3(n), dim3(ms::kNormThreads), 0, (hipStream_t)stream, h, (const uint16_t*)delta,
                       (const uint16_t*)weight, eps, (uint16_t*)out, hidden);
    MS_HIP_TRY(hipGetLastError());
    return MS_OK;
}

extern "C" int ms_swiglu(const void* gate_up, void* out, int n, int inter, void* stream) {
    if (n < 0 || inter < 8 || inter % 8) MS_FAIL(MS_ERR_INVALID, "ms_swiglu: need the MLP width a multiple of 8");
    if (n == 0) return MS_OK;
    if (n > 65535) MS_FAIL(MS_ERR_INVALID, "ms_swiglu: at most 65535 rows per call");
    if (!gate_up || !out || !ms::aligned16(gate_up) || !ms::aligned16(out))
        MS_FAIL(MS_ERR_INVALID, "ms_swiglu: null or misaligned (16 bytes) argument");
    const int per_block = ms::kRowThreads * 8;
    hipLaunchKernelGGL(ms::swiglu, dim3((inter + per_block - 1) / per_block, n), dim3(ms::kRowThreads), 0, (hipStream_t)stream,
                       (const uint16_t*)gate_up, (uint16_t*)out, inter);
    MS_HIP_TRY(hipGetLastError());
    return MS_OK;
}

extern "C" int ms_argmax_rows(const void* logits, int n, int vocab, long ld, int* out, void* stream) {
    if (n < 0 || vocab < 1 || ld < vocab || ld % 8) MS_FAIL(MS_ERR_INVALID, "ms_argmax_rows: need ld >= vocab >= 1, ld a multiple of 8");
    if (n == 0) return MS_OK;
    if (!logits || !out || !ms::aligned16(logits)) MS_FAIL(MS_ERR_INVALID, "ms_argmax_rows: null or misaligned (16 bytes) argument");
    hipLaunchKernelGGL(ms::argmax_rows, dim3(n), dim3(ms::kRowThreads), 0, (hipStream_t)stream, (const uint16_t*)logits, vocab,
                       ld, out);
    MS_HIP_TRY(hipGetLastError());
    return MS_OK;
}
