// Fused Predict+Verify attention: host entry point, the general one-wave-per-row kernel (any
// supported dtype / head_dim / head grouping) and the split-KV combine.
//
// What is computed (MemoSight paper, Section 2.1.1 Predict and Verify; Section 2.3 "Compression
// Attention" and "MTP Attention"): every query of the step -- the verify block followed by the
// foresight tokens -- attends to all cached tokens of its sequence (the cache holds only what
// compression kept), to the in-flight tokens its ctx_new entry allows, and to itself; nothing but
// a foresight token itself ever attends to a foresight token.
#include <math.h>

#include <mutex>

#include "attention.h"
#include "ms_device.h"
#include "ms_internal.h"

namespace ms {

__device__ __forceinline__ float wave_max(float x) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) x = fmaxf(x, __shfl_xor(x, o, 64));
    return x;
}
__device__ __forceinline__ float wave_sum(float x) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) x += __shfl_xor(x, o, 64);
    return x;
}

template <int D>
__device__ __forceinline__ float dot_row(const float* __restrict__ k, const float* q_s) {
    float acc = 0.f;
#pragma unroll 4
    for (int d = 0; d < D; d += 4) {
        const float4 kv = *reinterpret_cast<const float4*>(k + d);
        acc += kv.x * q_s[d] + kv.y * q_s[d + 1] + kv.z * q_s[d + 2] + kv.w * q_s[d + 3];
    }
    return acc;
}
template <int D>
__device__ __forceinline__ float dot_row(const bf16_t* __restrict__ k, const float* q_s) {
    float acc = 0.f;
#pragma unroll 4
    for (int d = 0; d < D; d += 8) {
        const uint4 kv = *reinterpret_cast<const uint4*>(k + d);
        const uint32_t w[4] = {kv.x, kv.y, kv.z, kv.w};
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            acc += __uint_as_float(w[e] << 16) * q_s[d + 2 * e];
            acc += __uint_as_float(w[e] & 0xffff0000u) * q_s[d + 2 * e + 1];
        }
    }
    return acc;
}

// One wave per (kv split, query row (i, h), sequence).  Lanes run over tokens for the scores and
// over head_dim for the value accumulation.
template <typename T, int D>
__global__ __launch_bounds__(64) void pv_attn_rowwave(AttnArgs a, BatchMeta bm) {
    const int sp = blockIdx.x, row = blockIdx.y, b = blockIdx.z, lane = threadIdx.x;
    const int i = row / a.n_q_heads, h = row % a.n_q_heads, g = h / a.group;
    const int seq = bm.seq[b], L = a.d_len[seq];
    const int* pt = a.d_pt + (size_t)seq * a.max_pages;
    const T* pool = (const T*)a.pool_layer;
    constexpr int H2 = D / 2;
    constexpr int EPL = D / 64;  // accumulator elements per lane
    __shared__ float q_s[D];
    __shared__ float p_s[64];

    // rotate the query by its own position id and fold the softmax scale in
    if (lane < H2) {
        const T* qp = (const T*)a.q + (((size_t)b * a.n_q + i) * a.n_q_heads + h) * D;
        const float x0 = to_float(qp[lane]), x1 = to_float(qp[lane + H2]);
        float sn, cs;
        sincosf((float)a.pos[b * a.n_q + i] * a.inv_freq[lane], &sn, &cs);
        q_s[lane] = (x0 * cs - x1 * sn) * a.scale;
        q_s[lane + H2] = (x1 * cs + x0 * sn) * a.scale;
    }
    __syncthreads();

    float m = -INFINITY, l = 0.f, acc[EPL];
#pragma unroll
    for (int e = 0; e < EPL; ++e) acc[e] = 0.f;

    const int t_begin = sp * a.chunk;
    // (the chunks were cut from the lengths the host knew; rows committed on the device since then
    // fall to the last split)
    const int t_end = sp == a.n_splits - 1 ? L : min(L, t_begin + a.chunk);
    for (int t0 = t_begin; t0 < t_end; t0 += 64) {
        const int t = t0 + lane;
        const bool valid = t < t_end;
        float s = -INFINITY;
        if (valid) {
            const int page = pt[t >> 4];
            s = dot_row<D>(pool + (size_t)page * a.page_elems + ((size_t)g * 2) * MS_PAGE_SIZE * D + (t & 15) * D, q_s);
        }
        const float m_new = fmaxf(m, wave_max(s));
        const float p = valid ? expf(s - m_new) : 0.f;
        const float corr = expf(m - m_new);
        l = l * corr + wave_sum(p);
#pragma unroll
        for (int e = 0; e < EPL; ++e) acc[e] *= corr;
        m = m_new;
        p_s[lane] = p;
        __syncthreads();
        const int cnt = min(64, t_end - t0);
        for (int tt = 0; tt < cnt; ++tt) {
            const int tok = t0 + tt;
            const int page = pt[tok >> 4];
            const T* vp = pool + (size_t)page * a.page_elems + ((size_t)g * 2 + 1) * MS_PAGE_SIZE * D + (tok & 15) * D;
            const float pp = p_s[tt];
#pragma unroll
            for (int e = 0; e < EPL; ++e) acc[e] += pp * to_float(vp[lane + 64 * e]);
        }
        __syncthreads();
    }

    if (sp == 0) {
        // in-flight block: lane j holds in-flight token j
        const int ctx = a.ctx_new ? a.ctx_new[b * a.n_q + i] : (i < a.n_verify ? i : a.n_verify);
        const bool valid = lane < a.n_q && (lane < ctx || lane == i);
        float s = -INFINITY;
        if (valid) {
            const T* kp = (const T*)a.k_new + (((size_t)b * a.n_q + lane) * a.n_kv_heads + g) * D;
            const float posf = (float)a.pos[b * a.n_q + lane];
            float dot = 0.f;
            for (int d = 0; d < H2; ++d) {
                float sn, cs;
                sincosf(posf * a.inv_freq[d], &sn, &cs);
                const float x0 = to_float(kp[d]), x1 = to_float(kp[d + H2]);
                dot += q_s[d] * (x0 * cs - x1 * sn) + q_s[d + H2] * (x1 * cs + x0 * sn);
            }
            s = dot;
        }
        const float m_new = fmaxf(m, wave_max(s));  // the query always sees itself: finite
        const float p = valid ? expf(s - m_new) : 0.f;
        const float corr = expf(m - m_new);
        l = l * corr + wave_sum(p);
#pragma unroll
        for (int e = 0; e < EPL; ++e) acc[e] *= corr;
        m = m_new;
        p_s[lane] = p;
        __syncthreads();
        for (int j = 0; j < a.n_q; ++j) {
            const float pp = p_s[j];
            if (pp == 0.f) continue;
            const T* vp = (const T*)a.v_new + (((size_t)b * a.n_q + j) * a.n_kv_heads + g) * D;
#pragma unroll
            for (int e = 0; e < EPL; ++e) acc[e] += pp * to_float(vp[lane + 64 * e]);
        }
    }

    const size_t orow = ((size_t)b * a.n_q + i) * a.n_q_heads + h;
    if (a.n_splits == 1) {
        T* op = (T*)a.out + orow * D;
        const float inv = 1.f / l;
#pragma unroll
        for (int e = 0; e < EPL; ++e) op[lane + 64 * e] = from_float<T>(acc[e] * inv);
    } else {
        float* wp = a.ws + (orow * a.n_splits + sp) * (D + 2);
        if (lane == 0) {
            wp[0] = m;
            wp[1] = l;
        }
#pragma unroll
        for (int e = 0; e < EPL; ++e) wp[2 + lane + 64 * e] = acc[e];
    }
}

// out = sum_s e^{m_s - m} acc_s / sum_s e^{m_s - m} l_s ; one wave per output row.
template <typename T, int D>
__global__ __launch_bounds__(64) void pv_attn_combine(const float* __restrict__ ws, void* __restrict__ out, int n_splits) {
    const size_t orow = blockIdx.x;
    const int lane = threadIdx.x;
    constexpr int EPL = D / 64;
    const float* wp = ws + orow * n_splits * (D + 2);
    float m = -INFINITY;
    for (int s = 0; s < n_splits; ++s) m = fmaxf(m, wp[s * (D + 2)]);
    float l = 0.f, acc[EPL];
#pragma unroll
    for (int e = 0; e < EPL; ++e) acc[e] = 0.f;
    for (int s = 0; s < n_splits; ++s) {
        const float* p = wp + s * (D + 2);
        const float w = expf(p[0] - m);  // empty splits carry m = -inf, l = 0
        l += w * p[1];
#pragma unroll
        for (int e = 0; e < EPL; ++e) acc[e] += w * p[2 + lane + 64 * e];
    }
    T* op = (T*)out + orow * D;
    const float inv = 1.f / l;
#pragma unroll
    for (int e = 0; e < EPL; ++e) op[lane + 64 * e] = from_float<T>(acc[e] * inv);
}

static int rowwave_splits(int rows, int max_len, int* chunk) {
    int want = (4096 + rows - 1) / rows;           // aim for a few thousand waves in flight
    int by_len = (max_len + 255) / 256;            // at least 256 tokens per split
    int s = want < by_len ? want : by_len;
    if (s < 1) s = 1;
    if (s > kMaxRowwaveSplits) s = kMaxRowwaveSplits;
    int c = (max_len + s - 1) / s;
    c = ((c + 63) / 64) * 64;
    if (c < 64) c = 64;
    *chunk = c;
    return s;
}

template <typename T, int D>
static int launch_rowwave(ms_cache* c, AttnArgs& a, const BatchMeta& bm, int B, int max_len, hipStream_t stream) {
    const int rows = a.n_q * a.n_q_heads;
    a.n_splits = rowwave_splits(B * rows, max_len, &a.chunk);
    c->launches += a.n_splits > 1 ? 2 : 1;
    hipLaunchKernelGGL((pv_attn_rowwave<T, D>), dim3(a.n_splits, rows, B), dim3(64), 0, stream, a, bm);
    MS_HIP_TRY(hipGetLastError());
    if (a.n_splits > 1) {
        hipLaunchKernelGGL((pv_attn_combine<T, D>), dim3((unsigned)((size_t)B * rows)), dim3(64), 0, stream, a.ws, a.out,
                           a.n_splits);
        MS_HIP_TRY(hipGetLastError());
    }
    return MS_OK;
}

size_t rowwave_workspace_bytes(const ms_cache* c, int B, int n_q) {
    return (size_t)B * n_q * c->d.n_q_heads * kMaxRowwaveSplits * (c->d.head_dim + 2) * sizeof(float);
}

// ---------------------------------------------------------------------------------------------
// Library-owned workspace for callers that cannot allocate (ms_predict_verify_attention_static):
// the split-KV partials live in a fixed array of device memory that every GPU the library runs on
// holds until the process ends.  In host code the array's name is only a handle for
// hipGetSymbolAddress: the address the kernels get is resolved once per device, with that device
// current, and kept in g_scratch_ptr.
// ---------------------------------------------------------------------------------------------
static __device__ __align__(256) unsigned char scratch[MS_STATIC_SCRATCH_BYTES];

constexpr int kMaxDevices = 64;
static std::mutex g_scratch_mutex;
static void* g_scratch_ptr[kMaxDevices] = {};

// Address of `scratch` on `device`, which must be the current device.  Resolved on the first call
// per device (ms_cache_create makes that call).
int static_scratch(int device, void** ptr) {
    if (device < 0 || device >= kMaxDevices) MS_FAIL(MS_ERR_UNSUPPORTED, "device index %d outside [0, %d)", device, kMaxDevices);
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[device]) {
        int cur = -1;
        MS_HIP_TRY(hipGetDevice(&cur));
        if (cur != device) MS_FAIL(MS_ERR_INVALID, "static workspace: device %d is not the current device (%d)", device, cur);
        void* p = nullptr;
        MS_HIP_TRY(hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)));
        if (!p || ((uintptr_t)p & 255) != 0) MS_FAIL(MS_ERR_HIP, "static workspace: bad symbol address %p", p);
        g_scratch_ptr[device] = p;
    }
    *ptr = g_scratch_ptr[device];
    return MS_OK;
}

}  // namespace ms

using namespace ms;

extern "C" int ms_attention_set_deterministic(ms_cache* c, int on) {
    if (!c) MS_FAIL(MS_ERR_INVALID, "ms_attention_set_deterministic: null cache");
    c->deterministic = on != 0;
    return MS_OK;
}

extern "C" size_t ms_attention_workspace_bytes(ms_cache* c, int B, int n_q) {
    if (!c || B < 1 || B > MS_MAX_BATCH || n_q < 1 || n_q > MS_MAX_QUERIES) return 0;
    size_t need = mfma_eligible(c, n_q) ? mfma_workspace_bytes(c, B, n_q) : rowwave_workspace_bytes(c, B, n_q);
    return (need + 255) & ~(size_t)255;
}

extern "C" int ms_predict_verify_attention(ms_cache* c, int layer, int B, const int* seq_ids, int n_verify,
                                           int n_foresight, const void* q, const void* k_new, const void* v_new,
                                           const int* pos_ids, const int* ctx_new, float scale, void* out,
                                           void* workspace, size_t ws_bytes, void* stream_) {
    hipStream_t stream = (hipStream_t)stream_;
    if (!c) MS_FAIL(MS_ERR_INVALID, "ms_predict_verify_attention: null cache");
    if (B == 0) return MS_OK;
    if (B < 0 || B > MS_MAX_BATCH) MS_FAIL(MS_ERR_INVALID, "ms_predict_verify_attention: B %d outside [0, %d]", B, MS_MAX_BATCH);
    if (layer < 0 || layer >= c->d.n_layers) MS_FAIL(MS_ERR_INVALID, "ms_predict_verify_attention: layer %d out of range", layer);
    const int n_q = n_verify + n_foresight;
    if (n_verify < 0 || n_foresight < 0 || n_q < 1 || n_q > MS_MAX_QUERIES)
        MS_FAIL(MS_ERR_INVALID, "ms_predict_verify_attention: n_verify %d + n_foresight %d outside [1, %d]", n_verify,
                n_foresight, MS_MAX_QUERIES);
    if (!seq_ids || !q || !k_new || !v_new || !pos_ids || !out)
        MS_FAIL(MS_ERR_INVALID, "ms_predict_verify_attention: null argument");
    const size_t need = ms_attention_workspace_bytes(c, B, n_q);
    if (!workspace || ws_bytes < need)
        MS_FAIL(MS_ERR_WORKSPACE, "ms_predict_verify_attention: workspace needs %zu bytes, has %zu", need,
                workspace ? ws_bytes : (size_t)0);
    if (((uintptr_t)workspace & 255) != 0) MS_FAIL(MS_ERR_WORKSPACE, "ms_predict_verify_attention: workspace not 256-byte aligned");
    if (!c->pending_pt.empty()) {   // lengths of sequences created or freed since the last call with a stream
        int rc = flush_page_table_patches(c, stream);
        if (rc != MS_OK) return rc;
    }
    BatchMeta bm;
    int max_len = 0;
    for (int b = 0; b < B; ++b) {
        int rc = check_seq(c, seq_ids[b], "ms_predict_verify_attention");
        if (rc != MS_OK) return rc;
        bm.seq[b] = seq_ids[b];
        bm.len[b] = c->len[seq_ids[b]];
        if (bm.len[b] > max_len) max_len = bm.len[b];
    }
    AttnArgs a;
    a.pool_layer = (const char*)c->d.pool + (size_t)layer * c->layer_elems * c->esize;
    a.d_pt = c->d_pt;
    a.d_len = c->d_len;
    a.inv_freq = c->d_inv_freq;
    a.q = q;
    a.k_new = k_new;
    a.v_new = v_new;
    a.pos = pos_ids;
    a.ctx_new = ctx_new;
    a.out = out;
    a.ws = (float*)workspace;
    a.n_q = n_q;
    a.n_verify = n_verify;
    a.n_q_heads = c->d.n_q_heads;
    a.n_kv_heads = c->d.n_kv_heads;
    a.group = c->group;
    a.max_pages = c->d.max_pages_per_seq;
    a.page_elems = (long)c->page_elems;
    a.n_splits = 1;
    a.chunk = 0;
    a.scale = scale != 0.f ? scale : 1.0f / sqrtf((float)c->d.head_dim);
    if ((((uintptr_t)q | (uintptr_t)k_new | (uintptr_t)v_new | (uintptr_t)out) & 15) != 0)
        MS_FAIL(MS_ERR_INVALID, "ms_predict_verify_attention: q, k_new, v_new and out must be 16-byte aligned");
    if (mfma_eligible(c, n_q)) return launch_mfma(c, a, bm, B, stream);
    const int D = c->d.head_dim;
    if (c->d.dtype == MS_F32)
        return D == 64 ? launch_rowwave<float, 64>(c, a, bm, B, max_len, stream) : launch_rowwave<float, 128>(c, a, bm, B, max_len, stream);
    return D == 64 ? launch_rowwave<bf16_t, 64>(c, a, bm, B, max_len, stream) : launch_rowwave<bf16_t, 128>(c, a, bm, B, max_len, stream);
}

extern "C" int ms_predict_verify_attention_static(ms_cache* c, int layer, int B, const int* seq_ids, int n_verify,
                                                  int n_foresight, const void* q, const void* k_new, const void* v_new,
                                                  const int* pos_ids, const int* ctx_new, float scale, void* out,
                                                  void* stream) {
    if (!c) MS_FAIL(MS_ERR_INVALID, "ms_predict_verify_attention_static: null cache");
    if (B == 0) return MS_OK;
    const int n_q = n_verify + n_foresight;
    if (B < 0 || B > MS_MAX_BATCH || n_verify < 0 || n_foresight < 0 || n_q < 1 || n_q > MS_MAX_QUERIES)
        MS_FAIL(MS_ERR_INVALID, "ms_predict_verify_attention_static: B %d, n_verify %d, n_foresight %d out of range", B, n_verify,
                n_foresight);
    const size_t need = ms_attention_workspace_bytes(c, B, n_q);
    if (need > (size_t)MS_STATIC_SCRATCH_BYTES)
        MS_FAIL(MS_ERR_WORKSPACE,
                "ms_predict_verify_attention_static: this call needs %zu bytes of workspace, the library's fixed one has %zu; "
                "use ms_predict_verify_attention with a workspace of the caller's",
                need, (size_t)MS_STATIC_SCRATCH_BYTES);
    void* ws = nullptr;
    const int rc = static_scratch(c->device, &ws);   // resolved in ms_cache_create: a table look-up here
    if (rc != MS_OK) return rc;
    // nothing in the workspace has to start at zero: every partial is written before it is read
    return ms_predict_verify_attention(c, layer, B, seq_ids, n_verify, n_foresight, q, k_new, v_new, pos_ids, ctx_new, scale,
                                       out, ws, (size_t)MS_STATIC_SCRATCH_BYTES, stream);
}
