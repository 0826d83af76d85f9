// Paged KV cache: host-side page tables and allocator, device mirror, and the row scatter /
// gather kernels behind append, commit and segment compaction (Algorithm 1: "S <- S (+) A" and
// "UpdateCache"; Section 2.1.2 of the MemoSight paper).
#include <math.h>
#include <stdarg.h>
#include <stdio.h>
#include <string.h>

#include <algorithm>
#include <iterator>
#include <new>

#include "attention.h"
#include "ms_device.h"
#include "ms_internal.h"

// ---------------------------------------------------------------------------------------------
// errors
// ---------------------------------------------------------------------------------------------
namespace ms {

static thread_local char g_err[512] = "";

void set_error(const char* fmt, ...) {
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof(g_err), fmt, ap);
    va_end(ap);
}
void clear_error() { g_err[0] = 0; }

// ---------------------------------------------------------------------------------------------
// staging ring
// ---------------------------------------------------------------------------------------------
int StageRing::init() {
    MS_HIP_TRY(hipHostMalloc((void**)&h, kSlots * kSlotBytes, hipHostMallocDefault));
    MS_HIP_TRY(hipMalloc((void**)&d, kSlots * kSlotBytes));
    for (int i = 0; i < kSlots; ++i) {
        MS_HIP_TRY(hipEventCreateWithFlags(&ev[i], hipEventDisableTiming));
        used[i] = false;
    }
    next = 0;
    return MS_OK;
}

void StageRing::destroy() {
    for (int i = 0; i < kSlots; ++i)
        if (ev[i]) (void)hipEventDestroy(ev[i]);
    if (h) (void)hipHostFree(h);
    if (d) (void)hipFree(d);
    h = d = nullptr;
}

int StageRing::upload(const void* src, size_t bytes, hipStream_t stream, void** dev) {
    if (bytes > kSlotBytes) MS_FAIL(MS_ERR_INVALID, "internal: staging upload of %zu bytes", bytes);
    int s = next;
    next = (next + 1) % kSlots;
    if (used[s]) MS_HIP_TRY(hipEventSynchronize(ev[s]));
    memcpy(h + s * kSlotBytes, src, bytes);
    MS_HIP_TRY(hipMemcpyAsync(d + s * kSlotBytes, h + s * kSlotBytes, bytes, hipMemcpyHostToDevice,
                              stream));
    MS_HIP_TRY(hipEventRecord(ev[s], stream));
    used[s] = true;
    *dev = d + s * kSlotBytes;
    return MS_OK;
}

int StageRing::upload_to(void* dst, const void* src, size_t bytes, hipStream_t stream) {
    if (bytes > kSlotBytes) MS_FAIL(MS_ERR_INVALID, "internal: staging upload of %zu bytes", bytes);
    int s = next;
    next = (next + 1) % kSlots;
    if (used[s]) MS_HIP_TRY(hipEventSynchronize(ev[s]));
    memcpy(h + s * kSlotBytes, src, bytes);
    MS_HIP_TRY(hipMemcpyAsync(dst, h + s * kSlotBytes, bytes, hipMemcpyHostToDevice, stream));
    MS_HIP_TRY(hipEventRecord(ev[s], stream));
    used[s] = true;
    return MS_OK;
}

// ---------------------------------------------------------------------------------------------
// kernels
// ---------------------------------------------------------------------------------------------

// Writes (seq, index, page) triples into the device page-table mirror; a triple with index -1
// carries the sequence's new length instead.
__global__ void patch_page_table(int* __restrict__ d_pt, int* __restrict__ d_len, const int* __restrict__ triples, int n,
                                 int max_pages) {
    int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= n) return;
    const int seq = triples[3 * i], idx = triples[3 * i + 1], val = triples[3 * i + 2];
    if (idx < 0) d_len[seq] = val;
    else d_pt[(size_t)seq * max_pages + idx] = val;
}

struct ScatterArgs {
    void* pool;
    const int* d_pt;
    int* d_len;
    const float* inv_freq;
    const RowDesc* desc;
    int n_seq;
    int total_rows;
    const void* k;
    const void* v;
    const int* pos;        // indexed by buffer row; may be null when !rope
    long buf_layer_rows;   // rows per layer in the packed buffers
    int n_kv_heads;
    int max_pages;
    long page_elems;
    long layer_elems;
    int rope;
};

__device__ __forceinline__ int find_seq(const RowDesc* desc, int n_seq, int r) {
    int lo = 0, hi = n_seq - 1;  // last b with prefix <= r
    while (lo < hi) {
        int mid = (lo + hi + 1) >> 1;
        if (desc[mid].prefix <= r) lo = mid; else hi = mid - 1;
    }
    return lo;
}

// One workgroup per (row, layer): stores one token's K (rotated on request) and V for every KV
// head into its page slot.
template <typename T, int D>
__global__ __launch_bounds__(256) void kv_scatter(ScatterArgs a) {
    const int r = blockIdx.x, layer = blockIdx.y;
    const int b = find_seq(a.desc, a.n_seq, r);
    const RowDesc de = a.desc[b];
    const int j = r - de.prefix;
    const long src_row = (long)layer * a.buf_layer_rows + de.buf_first + j;
    const int t = de.cache_begin + j;
    const int page = a.d_pt[(size_t)de.seq * a.max_pages + t / MS_PAGE_SIZE];
    const int slot = t % MS_PAGE_SIZE;
    T* pool = (T*)a.pool + (size_t)layer * a.layer_elems + (size_t)page * a.page_elems;
    const T* ks = (const T*)a.k + src_row * a.n_kv_heads * D;
    const T* vs = (const T*)a.v + src_row * a.n_kv_heads * D;
    const float posf = a.rope ? (float)a.pos[de.buf_first + j] : 0.f;
    constexpr int H2 = D / 2;
    for (int e = threadIdx.x; e < a.n_kv_heads * H2; e += blockDim.x) {
        const int g = e / H2, i = e % H2;
        float x0 = to_float(ks[g * D + i]), x1 = to_float(ks[g * D + i + H2]);
        if (a.rope) {
            float sn, cs;
            sincosf(posf * a.inv_freq[i], &sn, &cs);
            const float y0 = x0 * cs - x1 * sn, y1 = x1 * cs + x0 * sn;
            x0 = y0;
            x1 = y1;
        }
        T* kd = pool + ((size_t)g * 2 + 0) * MS_PAGE_SIZE * D + slot * D;
        T* vd = pool + ((size_t)g * 2 + 1) * MS_PAGE_SIZE * D + slot * D;
        kd[i] = from_float<T>(x0);
        kd[i + H2] = from_float<T>(x1);
        vd[i] = vs[g * D + i];
        vd[i + H2] = vs[g * D + i + H2];
    }
}

// Small calls (the decode-step case) carry their row descriptors and page-table patches in the
// kernel arguments: one launch, no staging copy.  A workgroup finds its destination page among the
// call's patches first (the mirror does not hold them yet) and in the mirror otherwise; workgroup
// (0, 0) writes the patches into the mirror for the launches that follow.
constexpr int kInlineSeqs = 64;
constexpr int kInlinePatches = 160;
struct InlineTables {
    RowDesc desc[kInlineSeqs];
    int patch[3 * kInlinePatches];
    int n_patch;
};

template <typename T, int D>
__global__ __launch_bounds__(256) void kv_scatter_inline(ScatterArgs a, InlineTables tb) {
    const int r = blockIdx.x, layer = blockIdx.y;
    const int b = find_seq(tb.desc, a.n_seq, r);
    const RowDesc de = tb.desc[b];
    const int j = r - de.prefix;
    const long src_row = (long)layer * a.buf_layer_rows + de.buf_first + j;
    const int t = de.cache_begin + j;
    int page = -1;
    for (int i = 0; i < tb.n_patch; ++i)
        if (tb.patch[3 * i] == de.seq && tb.patch[3 * i + 1] == t / MS_PAGE_SIZE) page = tb.patch[3 * i + 2];
    if (page < 0) page = a.d_pt[(size_t)de.seq * a.max_pages + t / MS_PAGE_SIZE];
    if (r == 0 && layer == 0)
        for (int i = threadIdx.x; i < tb.n_patch; i += blockDim.x) {
            if (tb.patch[3 * i + 1] < 0) a.d_len[tb.patch[3 * i]] = tb.patch[3 * i + 2];     // a sequence's new length
            else const_cast<int*>(a.d_pt)[(size_t)tb.patch[3 * i] * a.max_pages + tb.patch[3 * i + 1]] = tb.patch[3 * i + 2];
        }
    const int slot = t % MS_PAGE_SIZE;
    T* pool = (T*)a.pool + (size_t)layer * a.layer_elems + (size_t)page * a.page_elems;
    const T* ks = (const T*)a.k + src_row * a.n_kv_heads * D;
    const T* vs = (const T*)a.v + src_row * a.n_kv_heads * D;
    const float posf = a.rope ? (float)a.pos[de.buf_first + j] : 0.f;
    constexpr int H2 = D / 2;
    for (int e = threadIdx.x; e < a.n_kv_heads * H2; e += blockDim.x) {
        const int g = e / H2, i = e % H2;
        float x0 = to_float(ks[g * D + i]), x1 = to_float(ks[g * D + i + H2]);
        if (a.rope) {
            float sn, cs;
            sincosf(posf * a.inv_freq[i], &sn, &cs);
            const float y0 = x0 * cs - x1 * sn, y1 = x1 * cs + x0 * sn;
            x0 = y0;
            x1 = y1;
        }
        T* kd = pool + ((size_t)g * 2 + 0) * MS_PAGE_SIZE * D + slot * D;
        T* vd = pool + ((size_t)g * 2 + 1) * MS_PAGE_SIZE * D + slot * D;
        kd[i] = from_float<T>(x0);
        kd[i + H2] = from_float<T>(x1);
        vd[i] = vs[g * D + i];
        vd[i + H2] = vs[g * D + i + H2];
    }
}

// Inverse of kv_scatter without rotation: copies cache rows into packed buffers.
template <typename T, int D>
__global__ __launch_bounds__(256) void kv_gather(ScatterArgs a) {
    const int r = blockIdx.x, layer = blockIdx.y;
    const int b = find_seq(a.desc, a.n_seq, r);
    const RowDesc de = a.desc[b];
    const int j = r - de.prefix;
    const long dst_row = (long)layer * a.buf_layer_rows + de.buf_first + j;
    const int t = de.cache_begin + j;
    const int page = a.d_pt[(size_t)de.seq * a.max_pages + t / MS_PAGE_SIZE];
    const int slot = t % MS_PAGE_SIZE;
    const T* pool = (const T*)a.pool + (size_t)layer * a.layer_elems + (size_t)page * a.page_elems;
    T* kd = (T*)a.k + dst_row * a.n_kv_heads * D;
    T* vd = (T*)a.v + dst_row * a.n_kv_heads * D;
    for (int e = threadIdx.x; e < a.n_kv_heads * D; e += blockDim.x) {
        const int g = e / D, i = e % D;
        kd[e] = pool[((size_t)g * 2 + 0) * MS_PAGE_SIZE * D + slot * D + i];
        vd[e] = pool[((size_t)g * 2 + 1) * MS_PAGE_SIZE * D + slot * D + i];
    }
}

// ---- commit with the accept lengths read on the device ------------------------------------------
//
// The host does not know how many rows each sequence keeps, so it cannot name pages: it hands over
// an ascending list of free pages, and the kernel gives them out in the order the host would (the
// sequences in argument order, a page whenever a row's index is a multiple of 16, always the lowest
// free one).  state[0] counts the list entries used so far; arrival counters tell when every
// workgroup has read the lengths, and the last one to arrive writes the new lengths, the new
// page-table entries and, per page taken, the sequence that took it (for the host to catch up later).
struct CommitArgs {
    void* pool;
    int* d_pt;
    int* d_len;
    const float* inv_freq;
    const int* d_free;
    int* state;
    const int* accept_len;   // device [B]
    int* first_pid;          // device [B] or null: advanced by the accepted count
    const void* k;
    const void* v;
    const int* pos;
    int B, n_q, n_max, n_kv_heads, max_pages;
    long page_elems, layer_elems, buf_layer_rows;
};
struct SeqIds {
    int seq[MS_MAX_BATCH];
};

__device__ __forceinline__ int clamp_accept(int a, int n_max) { return a < 0 ? 0 : (a > n_max ? n_max : a); }
// pages a sequence of length len takes when it grows by acc rows
__device__ __forceinline__ int pages_taken(int len, int acc) { return ((len + acc + MS_PAGE_SIZE - 1) >> 4) - ((len + MS_PAGE_SIZE - 1) >> 4); }

template <typename T, int D>
__global__ __launch_bounds__(256) void kv_commit_device(CommitArgs a, SeqIds ids) {
    __shared__ int red[8];
    const int r = blockIdx.x, layer = blockIdx.y, tid = threadIdx.x;
    const int b = r / a.n_max, j = r % a.n_max;
    // pages taken by the sequences listed before this one
    int mine = 0;
    for (int bb = tid; bb < b; bb += 256) mine += pages_taken(a.d_len[ids.seq[bb]], clamp_accept(a.accept_len[bb], a.n_max));
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) mine += __shfl_xor(mine, o, 64);
    if ((tid & 63) == 0) red[tid >> 6] = mine;
    const int seq = ids.seq[b];
    const int len0 = a.d_len[seq], acc = clamp_accept(a.accept_len[b], a.n_max), cursor = a.state[0];
    __syncthreads();
    const int rank = red[0] + red[1] + red[2] + red[3];
    if (j < acc) {
        const int t = len0 + j, pi = t >> 4, had = (len0 + MS_PAGE_SIZE - 1) >> 4;
        const int page = pi < had ? a.d_pt[(size_t)seq * a.max_pages + pi] : a.d_free[cursor + rank + (pi - had)];
        const int slot = t & (MS_PAGE_SIZE - 1);
        const long src_row = (long)layer * a.buf_layer_rows + (long)b * a.n_q + j;
        T* pool = (T*)a.pool + (size_t)layer * a.layer_elems + (size_t)page * a.page_elems;
        const T* ks = (const T*)a.k + src_row * a.n_kv_heads * D;
        const T* vs = (const T*)a.v + src_row * a.n_kv_heads * D;
        const float posf = (float)a.pos[b * a.n_q + j];
        constexpr int H2 = D / 2;
        for (int e = tid; e < a.n_kv_heads * H2; e += 256) {
            const int g = e / H2, i = e % H2;
            const float x0 = to_float(ks[g * D + i]), x1 = to_float(ks[g * D + i + H2]);
            float sn, cs;
            sincosf(posf * a.inv_freq[i], &sn, &cs);
            T* kd = pool + ((size_t)g * 2 + 0) * MS_PAGE_SIZE * D + slot * D;
            T* vd = pool + ((size_t)g * 2 + 1) * MS_PAGE_SIZE * D + slot * D;
            kd[i] = from_float<T>(x0 * cs - x1 * sn);
            kd[i + H2] = from_float<T>(x1 * cs + x0 * sn);
            vd[i] = vs[g * D + i];
            vd[i + H2] = vs[g * D + i + H2];
        }
    }
    // every thread has used the lengths and the list position it read: count this workgroup in.
    // Two levels (a counter per layer, 256 bytes apart, then one over the layers): thousands of
    // arrivals at a single address would take tens of microseconds.
    __syncthreads();
    if (tid == 0) {
        int* layer_ctr = a.state + 2 + kFreeListCap + 64 * layer;
        int last = 0;
        if (__hip_atomic_fetch_add(layer_ctr, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) == (int)gridDim.x - 1) {
            __hip_atomic_store(layer_ctr, 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            last = __hip_atomic_fetch_add(a.state + 1, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) == (int)gridDim.y - 1;
        }
        red[4] = last;
    }
    __syncthreads();
    if (!red[4]) return;
    // ---- the last workgroup: thread bb brings sequence bb of the call up to date ----
    int len_b = 0, acc_b = 0, take = 0, seq_b = 0;
    if (tid < a.B) {
        seq_b = ids.seq[tid];
        len_b = a.d_len[seq_b];
        acc_b = clamp_accept(a.accept_len[tid], a.n_max);
        take = pages_taken(len_b, acc_b);
    }
    int incl = take;   // inclusive scan over the 256 threads: within waves, then over the waves' totals
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) {
        const int up = __shfl_up(incl, o, 64);
        if ((tid & 63) >= o) incl += up;
    }
    __syncthreads();
    if ((tid & 63) == 63) red[tid >> 6] = incl;
    __syncthreads();
    int before = incl - take;
    for (int w = 0; w < (tid >> 6); ++w) before += red[w];
    if (tid < a.B) {
        const int had = (len_b + MS_PAGE_SIZE - 1) >> 4;
        for (int k = 0; k < take; ++k) {
            const int at = cursor + before + k;
            a.d_pt[(size_t)seq_b * a.max_pages + had + k] = a.d_free[at];
            a.state[2 + at] = seq_b;
        }
        a.d_len[seq_b] = len_b + acc_b;
        if (a.first_pid) a.first_pid[tid] += acc_b;
    }
    if (tid == 255) {   // holds the grand total
        a.state[0] = cursor + before + take;
        __hip_atomic_store(a.state + 1, 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
}

// pos[b][i] = first_pid[b] + i: the verify block's consecutive position ids followed by the
// foresight tokens' (Section 2.1.1), from a device array of first position ids.
__global__ void step_positions_device(int B, const int* __restrict__ first_pid, int n_q, int* __restrict__ out) {
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < B * n_q) out[i] = first_pid[i / n_q] + i % n_q;
}

// ---------------------------------------------------------------------------------------------
// host helpers
// ---------------------------------------------------------------------------------------------

int check_seq(const ms_cache* c, int seq, const char* what) {
    if (seq < 0 || seq >= c->d.max_seqs || !c->live[seq])
        MS_FAIL(MS_ERR_INVALID, "%s: unknown sequence id %d", what, seq);
    return MS_OK;
}

int flush_page_table_patches(ms_cache* c, hipStream_t stream) {
    const size_t per = StageRing::kSlotBytes / (3 * sizeof(int));
    size_t n = c->pending_pt.size() / 3, done = 0;
    while (done < n) {
        size_t cnt = std::min(per, n - done);
        void* dev = nullptr;
        int rc = c->stage.upload(c->pending_pt.data() + 3 * done, cnt * 3 * sizeof(int), stream, &dev);
        if (rc != MS_OK) return rc;
        c->launches++;
        hipLaunchKernelGGL(patch_page_table, dim3((unsigned)((cnt + 255) / 256)), dim3(256), 0, stream,
                           c->d_pt, c->d_len, (const int*)dev, (int)cnt, c->d.max_pages_per_seq);
        MS_HIP_TRY(hipGetLastError());
        done += cnt;
    }
    c->pending_pt.clear();
    return MS_OK;
}

int reconcile(ms_cache* c) {
    if (!c->deferred) return MS_OK;
    MS_HIP_TRY(hipStreamSynchronize(c->deferred_stream));
    int used = 0;
    MS_HIP_TRY(hipMemcpy(&used, c->d_commit_state, sizeof(int), hipMemcpyDeviceToHost));
    if (used < 0 || used > (int)c->free_list.size()) MS_FAIL(MS_ERR_HIP, "device-side commit state is corrupt (%d pages taken of %zu listed)", used, c->free_list.size());
    std::vector<int> who(used), lens(c->d.max_seqs);
    if (used > 0) MS_HIP_TRY(hipMemcpy(who.data(), c->d_commit_state + 2, used * sizeof(int), hipMemcpyDeviceToHost));
    MS_HIP_TRY(hipMemcpy(lens.data(), c->d_len, lens.size() * sizeof(int), hipMemcpyDeviceToHost));
    if (!c->apply_device_commits(who.data(), used, c->free_list, lens.data()))
        MS_FAIL(MS_ERR_HIP, "device-side commit state is corrupt (a page of the log is not free, or its sequence is not live)");
    c->pending_growth.assign(c->d.max_seqs, 0);
    c->reserved_pages = 0;
    c->free_list_valid = false;
    c->deferred = false;
    return MS_OK;
}

#define MS_RECONCILE(c)                      \
    do {                                     \
        int rc_ = ::ms::reconcile(c);        \
        if (rc_ != MS_OK) return rc_;        \
        (c)->free_list_valid = false;        \
    } while (0)

static inline int pages_for(long n) { return HostTables::pages_for(n); }

template <typename F>
static int dispatch(const ms_cache* c, F&& f) {
    const int D = c->d.head_dim;
    if (c->d.dtype == MS_F32) return D == 64 ? f((float*)0, std::integral_constant<int, 64>()) : f((float*)0, std::integral_constant<int, 128>());
    return D == 64 ? f((bf16_t*)0, std::integral_constant<int, 64>()) : f((bf16_t*)0, std::integral_constant<int, 128>());
}

static int launch_rows(ms_cache* c, bool gather, const std::vector<RowDesc>& desc, int total_rows,
                       const void* k, const void* v, const int* pos, long buf_layer_rows, int rope,
                       hipStream_t stream) {
    if (total_rows == 0) return MS_OK;
    void* dev = nullptr;
    int rc = c->stage.upload(desc.data(), desc.size() * sizeof(RowDesc), stream, &dev);
    if (rc != MS_OK) return rc;
    ScatterArgs a;
    a.pool = c->d.pool;
    a.d_pt = c->d_pt;
    a.d_len = c->d_len;
    a.inv_freq = c->d_inv_freq;
    a.desc = (const RowDesc*)dev;
    a.n_seq = (int)desc.size();
    a.total_rows = total_rows;
    a.k = k;
    a.v = v;
    a.pos = pos;
    a.buf_layer_rows = buf_layer_rows;
    a.n_kv_heads = c->d.n_kv_heads;
    a.max_pages = c->d.max_pages_per_seq;
    a.page_elems = (long)c->page_elems;
    a.layer_elems = (long)c->layer_elems;
    a.rope = rope;
    dim3 grid((unsigned)total_rows, (unsigned)c->d.n_layers);
    return dispatch(c, [&](auto* tp, auto dc) -> int {
        using T = std::remove_pointer_t<decltype(tp)>;
        constexpr int D = decltype(dc)::value;
        c->launches++;
        if (gather)
            hipLaunchKernelGGL((kv_gather<T, D>), grid, dim3(256), 0, stream, a);
        else
            hipLaunchKernelGGL((kv_scatter<T, D>), grid, dim3(256), 0, stream, a);
        MS_HIP_TRY(hipGetLastError());
        return (int)MS_OK;
    });
}

// Patches the mirror and scatters rows in one launch when the call is small enough for its tables
// to travel in the kernel arguments; otherwise patch launch(es) + staged descriptors + scatter.
static int patch_and_scatter(ms_cache* c, const std::vector<RowDesc>& desc, int total_rows, const void* k,
                             const void* v, const int* pos, long buf_layer_rows, int rope, hipStream_t stream) {
    const size_t n_patch = c->pending_pt.size() / 3;
    if (total_rows == 0 || desc.size() > (size_t)kInlineSeqs || n_patch > (size_t)kInlinePatches) {
        int rc = flush_page_table_patches(c, stream);
        if (rc != MS_OK) return rc;
        return launch_rows(c, false, desc, total_rows, k, v, pos, buf_layer_rows, rope, stream);
    }
    InlineTables tb;
    memset(&tb, 0, sizeof(tb));
    memcpy(tb.desc, desc.data(), desc.size() * sizeof(RowDesc));
    memcpy(tb.patch, c->pending_pt.data(), n_patch * 3 * sizeof(int));
    tb.n_patch = (int)n_patch;
    c->pending_pt.clear();
    ScatterArgs a;
    a.pool = c->d.pool;
    a.d_pt = c->d_pt;
    a.d_len = c->d_len;
    a.inv_freq = c->d_inv_freq;
    a.desc = nullptr;
    a.n_seq = (int)desc.size();
    a.total_rows = total_rows;
    a.k = k;
    a.v = v;
    a.pos = pos;
    a.buf_layer_rows = buf_layer_rows;
    a.n_kv_heads = c->d.n_kv_heads;
    a.max_pages = c->d.max_pages_per_seq;
    a.page_elems = (long)c->page_elems;
    a.layer_elems = (long)c->layer_elems;
    a.rope = rope;
    dim3 grid((unsigned)total_rows, (unsigned)c->d.n_layers);
    return dispatch(c, [&](auto* tp, auto dc) -> int {
        using T = std::remove_pointer_t<decltype(tp)>;
        constexpr int D = decltype(dc)::value;
        c->launches++;
        hipLaunchKernelGGL((kv_scatter_inline<T, D>), grid, dim3(256), 0, stream, a, tb);
        MS_HIP_TRY(hipGetLastError());
        return (int)MS_OK;
    });
}

static int validate_desc(const ms_cache_desc* d) {
    if (!d) MS_FAIL(MS_ERR_INVALID, "descriptor is null");
    if (d->n_layers < 1 || d->n_kv_heads < 1 || d->n_q_heads < 1 || d->n_pages < 1 || d->max_seqs < 1 ||
        d->max_pages_per_seq < 1)
        MS_FAIL(MS_ERR_INVALID, "descriptor: counts must be positive");
    if (d->n_q_heads % d->n_kv_heads) MS_FAIL(MS_ERR_INVALID, "n_q_heads must be a multiple of n_kv_heads");
    if (d->head_dim != 64 && d->head_dim != 128) MS_FAIL(MS_ERR_UNSUPPORTED, "head_dim must be 64 or 128");
    if (d->page_size != MS_PAGE_SIZE) MS_FAIL(MS_ERR_UNSUPPORTED, "page_size must be %d", MS_PAGE_SIZE);
    if (d->dtype != MS_F32 && d->dtype != MS_BF16) MS_FAIL(MS_ERR_INVALID, "unknown dtype %d", d->dtype);
    if (!(d->rope_base > 1.0f)) MS_FAIL(MS_ERR_INVALID, "rope_base must be > 1");
    return MS_OK;
}

}  // namespace ms

using namespace ms;

// ---------------------------------------------------------------------------------------------
// C ABI
// ---------------------------------------------------------------------------------------------
extern "C" {

const char* ms_last_error(void) { return g_err; }

size_t ms_pool_bytes(const ms_cache_desc* d) {
    if (validate_desc(d) != MS_OK) return 0;
    size_t es = d->dtype == MS_F32 ? 4 : 2;
    return (size_t)d->n_layers * d->n_pages * d->n_kv_heads * 2 * MS_PAGE_SIZE * d->head_dim * es;
}

int ms_cache_create(const ms_cache_desc* desc, ms_cache** out) {
    if (!out) MS_FAIL(MS_ERR_INVALID, "out is null");
    *out = nullptr;
    int rc = validate_desc(desc);
    if (rc != MS_OK) return rc;
    if (!desc->pool) MS_FAIL(MS_ERR_INVALID, "pool is null");
    if (desc->pool_bytes < ms_pool_bytes(desc))
        MS_FAIL(MS_ERR_INVALID, "pool has %zu bytes, needs %zu", desc->pool_bytes, ms_pool_bytes(desc));
    ms_cache* c = new (std::nothrow) ms_cache();
    if (!c) MS_FAIL(MS_ERR_INVALID, "out of host memory");
    c->d = *desc;
    c->group = desc->n_q_heads / desc->n_kv_heads;
    c->esize = desc->dtype == MS_F32 ? 4 : 2;
    c->page_elems = (size_t)desc->n_kv_heads * 2 * MS_PAGE_SIZE * desc->head_dim;
    c->layer_elems = c->page_elems * desc->n_pages;
    c->init_tables(desc->n_pages, desc->max_seqs, desc->max_pages_per_seq);
    auto fail = [&](int code) {
        ms_cache_destroy(c);
        return code;
    };
    if (hipGetDevice(&c->device) != hipSuccess) {
        set_error("hipGetDevice failed");
        return fail(MS_ERR_HIP);
    }
    size_t pt_bytes = (size_t)desc->max_seqs * desc->max_pages_per_seq * sizeof(int);
    if (hipMalloc((void**)&c->d_pt, pt_bytes) != hipSuccess || hipMemset(c->d_pt, 0, pt_bytes) != hipSuccess) {
        set_error("allocating the page-table mirror (%zu bytes) failed", pt_bytes);
        return fail(MS_ERR_HIP);
    }
    const size_t len_bytes = (size_t)desc->max_seqs * sizeof(int), state_bytes = (size_t)(2 + kFreeListCap + 64 * desc->n_layers) * sizeof(int);
    if (hipMalloc((void**)&c->d_len, len_bytes) != hipSuccess || hipMemset(c->d_len, 0, len_bytes) != hipSuccess ||
        hipMalloc((void**)&c->d_free, (size_t)kFreeListCap * sizeof(int)) != hipSuccess ||
        hipMalloc((void**)&c->d_commit_state, state_bytes) != hipSuccess || hipMemset(c->d_commit_state, 0, state_bytes) != hipSuccess) {
        set_error("allocating the device-side lengths and free-page list failed");
        return fail(MS_ERR_HIP);
    }
    c->pending_growth.assign(desc->max_seqs, 0);
    // inv_freq_i = float(base^(-2i/D)), evaluated in double and rounded once
    std::vector<float> inv(desc->head_dim / 2);
    for (int i = 0; i < desc->head_dim / 2; ++i)
        inv[i] = (float)pow((double)desc->rope_base, -2.0 * i / desc->head_dim);
    if (hipMalloc((void**)&c->d_inv_freq, inv.size() * sizeof(float)) != hipSuccess ||
        hipMemcpy(c->d_inv_freq, inv.data(), inv.size() * sizeof(float), hipMemcpyHostToDevice) != hipSuccess) {
        set_error("allocating the inv_freq table failed");
        return fail(MS_ERR_HIP);
    }
    rc = c->stage.init();
    if (rc != MS_OK) return fail(rc);
    void* fixed_ws = nullptr;   // this device's copy of the library's fixed attention workspace
    rc = static_scratch(c->device, &fixed_ws);
    if (rc != MS_OK) return fail(rc);
    int cus = 0;
    if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, c->device) == hipSuccess && cus > 0) c->n_cus = cus;
    if (hipMalloc((void**)&c->d_plan, (size_t)mfma_plan_ints(MS_MAX_BATCH) * sizeof(int)) != hipSuccess) {
        set_error("allocating the attention plan buffer failed");
        return fail(MS_ERR_HIP);
    }
    const size_t arrive_bytes = (size_t)2 * MS_MAX_BATCH * desc->n_kv_heads * sizeof(int);   // two counters per (sequence, KV head)
    if (hipMalloc((void**)&c->d_arrive, arrive_bytes) != hipSuccess || hipMemset(c->d_arrive, 0, arrive_bytes) != hipSuccess) {
        set_error("allocating the arrival counters failed");
        return fail(MS_ERR_HIP);
    }
    if (hipHostMalloc((void**)&c->h_error, sizeof(int), hipHostMallocMapped) != hipSuccess ||
        hipHostGetDevicePointer((void**)&c->d_error, c->h_error, 0) != hipSuccess) {
        set_error("allocating the error word failed");
        return fail(MS_ERR_HIP);
    }
    *c->h_error = 0;
    *out = c;
    return MS_OK;
}

int ms_cache_destroy(ms_cache* c) {
    if (!c) return MS_OK;
    (void)hipDeviceSynchronize();
    c->stage.destroy();
    if (c->d_pt) (void)hipFree(c->d_pt);
    if (c->d_len) (void)hipFree(c->d_len);
    if (c->d_free) (void)hipFree(c->d_free);
    if (c->d_commit_state) (void)hipFree(c->d_commit_state);
    if (c->d_inv_freq) (void)hipFree(c->d_inv_freq);
    if (c->d_plan) (void)hipFree(c->d_plan);
    if (c->d_arrive) (void)hipFree(c->d_arrive);
    if (c->h_error) (void)hipHostFree(c->h_error);
    for (hipEvent_t e : c->prof_start) (void)hipEventDestroy(e);
    for (hipEvent_t e : c->prof_stop) (void)hipEventDestroy(e);
    delete c;
    return MS_OK;
}

int ms_seq_create(ms_cache* c, int* seq_id) {
    if (!c || !seq_id) MS_FAIL(MS_ERR_INVALID, "ms_seq_create: null argument");
    MS_RECONCILE(c);
    const int s = c->create_seq();
    if (s >= 0) {
        *seq_id = s;
        return MS_OK;
    }
    MS_FAIL(MS_ERR_INVALID, "ms_seq_create: all %d sequence ids are in use", c->d.max_seqs);
}

int ms_seq_import(ms_cache* c, int length, const int* pages, int n_pages, int* seq_id, void* stream) {
    if (!c || !seq_id || (n_pages > 0 && !pages)) MS_FAIL(MS_ERR_INVALID, "ms_seq_import: null argument");
    if (length < 0 || n_pages != pages_for(length))
        MS_FAIL(MS_ERR_INVALID, "ms_seq_import: %d pages do not match length %d", n_pages, length);
    MS_RECONCILE(c);
    if (n_pages > c->d.max_pages_per_seq)
        MS_FAIL(MS_ERR_OOM_PAGES, "ms_seq_import: %d pages exceed max_pages_per_seq %d", n_pages, c->d.max_pages_per_seq);
    if (!c->pages_importable(pages, n_pages)) MS_FAIL(MS_ERR_INVALID, "ms_seq_import: a listed page is not free, out of range or listed twice");
    int s = -1;
    int rc = ms_seq_create(c, &s);
    if (rc != MS_OK) return rc;
    c->import_seq(s, pages, n_pages, length);
    *seq_id = s;
    return flush_page_table_patches(c, (hipStream_t)stream);
}

int ms_seq_free(ms_cache* c, int seq_id) {
    if (!c) MS_FAIL(MS_ERR_INVALID, "ms_seq_free: null cache");
    int rc = check_seq(c, seq_id, "ms_seq_free");
    if (rc != MS_OK) return rc;
    MS_RECONCILE(c);
    c->free_seq(seq_id);
    return MS_OK;
}

// Shared by ms_append_kv and ms_commit_accepted: counts[b] rows per sequence, taken from buffer
// rows src_first[b] .. of a packed buffer with `buf_layer_rows` rows per layer.
static int append_rows(ms_cache* c, const char* what, int B, const int* seq_ids, const int* counts,
                       const std::vector<int>& src_first, long buf_layer_rows, const void* k,
                       const void* v, const int* pos, int rope, hipStream_t stream) {
    MS_RECONCILE(c);
    long need = 0;
    std::vector<int> extra(c->d.max_seqs, 0);  // a sequence may appear more than once in a call
    for (int b = 0; b < B; ++b) {
        int rc = check_seq(c, seq_ids[b], what);
        if (rc != MS_OK) return rc;
        if (counts[b] < 0) MS_FAIL(MS_ERR_INVALID, "%s: negative row count", what);
        extra[seq_ids[b]] += counts[b];
    }
    need = c->pages_needed(extra);
    if (need < 0)
        MS_FAIL(MS_ERR_OOM_PAGES, "%s: sequence %ld would need more than max_pages_per_seq %d pages", what, -1 - need, c->d.max_pages_per_seq);
    if (need > (long)c->free_pages.size())
        MS_FAIL(MS_ERR_OOM_PAGES, "%s: needs %ld pages, %zu free", what, need, c->free_pages.size());
    std::vector<RowDesc> desc;
    int total = 0;
    for (int b = 0; b < B; ++b) {
        if (counts[b] == 0) continue;
        RowDesc de{seq_ids[b], c->len[seq_ids[b]], src_first[b], total};
        desc.push_back(de);
        c->grow(seq_ids[b], counts[b]);
        total += counts[b];
    }
    return patch_and_scatter(c, desc, total, k, v, pos, buf_layer_rows, rope, stream);
}

int ms_append_kv(ms_cache* c, int B, const int* seq_ids, const int* n_tok, const void* k, const void* v,
                 const int* pos_ids, int flags, void* stream) {
    if (!c || B < 0 || (B > 0 && (!seq_ids || !n_tok))) MS_FAIL(MS_ERR_INVALID, "ms_append_kv: null argument");
    if (B > MS_MAX_BATCH) MS_FAIL(MS_ERR_INVALID, "ms_append_kv: B %d exceeds %d", B, MS_MAX_BATCH);
    if (flags != MS_PRE_ROTATED && flags != MS_ROPE_APPLY) MS_FAIL(MS_ERR_INVALID, "ms_append_kv: bad flags %d", flags);
    long total = 0;
    std::vector<int> first(B);
    for (int b = 0; b < B; ++b) {
        first[b] = (int)total;
        total += n_tok[b] > 0 ? n_tok[b] : 0;
    }
    if (total > 0 && (!k || !v)) MS_FAIL(MS_ERR_INVALID, "ms_append_kv: k or v is null");
    if (total > 0 && flags == MS_ROPE_APPLY && !pos_ids) MS_FAIL(MS_ERR_INVALID, "ms_append_kv: pos_ids is null");
    return append_rows(c, "ms_append_kv", B, seq_ids, n_tok, first, total, k, v, pos_ids, flags == MS_ROPE_APPLY,
                       (hipStream_t)stream);
}

int ms_commit_accepted(ms_cache* c, int B, const int* seq_ids, const int* accept_len, int n_q, const void* k_new,
                       const void* v_new, const int* pos_ids, void* stream) {
    if (!c || B < 0 || (B > 0 && (!seq_ids || !accept_len))) MS_FAIL(MS_ERR_INVALID, "ms_commit_accepted: null argument");
    if (B > MS_MAX_BATCH) MS_FAIL(MS_ERR_INVALID, "ms_commit_accepted: B %d exceeds %d", B, MS_MAX_BATCH);
    if (n_q < 1 || n_q > MS_MAX_QUERIES) MS_FAIL(MS_ERR_INVALID, "ms_commit_accepted: n_q %d out of range", n_q);
    std::vector<int> first(B);
    bool any = false;
    for (int b = 0; b < B; ++b) {
        if (accept_len[b] < 0 || accept_len[b] > n_q)
            MS_FAIL(MS_ERR_RANGE, "ms_commit_accepted: accept_len[%d] = %d outside [0, %d]", b, accept_len[b], n_q);
        first[b] = b * n_q;
        any |= accept_len[b] > 0;
    }
    if (any && (!k_new || !v_new || !pos_ids)) MS_FAIL(MS_ERR_INVALID, "ms_commit_accepted: null tensor");
    return append_rows(c, "ms_commit_accepted", B, seq_ids, accept_len, first, (long)B * n_q, k_new, v_new, pos_ids, 1,
                       (hipStream_t)stream);
}

int ms_commit_accepted_device(ms_cache* c, int B, const int* seq_ids, const int* accept_len, int n_q, int n_max,
                              const void* k_new, const void* v_new, const int* pos_ids, int* first_pid, void* stream_) {
    hipStream_t stream = (hipStream_t)stream_;
    if (!c || B < 0 || (B > 0 && (!seq_ids || !accept_len || !k_new || !v_new || !pos_ids)))
        MS_FAIL(MS_ERR_INVALID, "ms_commit_accepted_device: null argument");
    if (B == 0) return MS_OK;
    if (B > MS_MAX_BATCH) MS_FAIL(MS_ERR_INVALID, "ms_commit_accepted_device: B %d exceeds %d", B, MS_MAX_BATCH);
    if (n_q < 1 || n_q > MS_MAX_QUERIES || n_max < 1 || n_max > n_q || n_max > MS_PAGE_SIZE)
        MS_FAIL(MS_ERR_INVALID, "ms_commit_accepted_device: need 1 <= n_max <= min(n_q, %d), n_q <= %d", MS_PAGE_SIZE, MS_MAX_QUERIES);
    std::vector<char> seen(c->d.max_seqs, 0);
    for (int b = 0; b < B; ++b) {
        int rc = check_seq(c, seq_ids[b], "ms_commit_accepted_device");
        if (rc != MS_OK) return rc;
        if (seen[seq_ids[b]]) MS_FAIL(MS_ERR_INVALID, "ms_commit_accepted_device: sequence %d is listed twice", seq_ids[b]);
        seen[seq_ids[b]] = 1;
    }
    if (c->deferred && c->deferred_stream != stream) {   // the device-side state is ordered by one stream at a time
        int rc = reconcile(c);
        if (rc != MS_OK) return rc;
    }
    // Room for the worst case (every sequence keeps n_max rows: at most one more page each).  First
    // against the bounds the host has; if those do not suffice, against the exact state.
    for (int attempt = 0; attempt < 2; ++attempt) {
        bool fits = c->free_list_valid && c->reserved_pages + B <= (int)c->free_list.size();
        for (int b = 0; b < B && fits; ++b) {
            const int s = seq_ids[b];
            fits = pages_for((long)c->len[s] + c->pending_growth[s] + n_max) <= c->d.max_pages_per_seq;
        }
        if (fits) break;
        if (attempt == 1) {
            for (int b = 0; b < B; ++b)
                if (pages_for((long)c->len[seq_ids[b]] + n_max) > c->d.max_pages_per_seq)
                    MS_FAIL(MS_ERR_OOM_PAGES, "ms_commit_accepted_device: sequence %d could need more than max_pages_per_seq %d pages",
                            seq_ids[b], c->d.max_pages_per_seq);
            MS_FAIL(MS_ERR_OOM_PAGES, "ms_commit_accepted_device: needs room for %d pages, %zu free", B, c->free_pages.size());
        }
        int rc = reconcile(c);
        if (rc != MS_OK) return rc;
        rc = flush_page_table_patches(c, stream);
        if (rc != MS_OK) return rc;
        // hand the device the lowest free pages in ascending order and start counting from zero
        c->free_list.assign(c->free_pages.begin(), c->free_pages.size() > (size_t)kFreeListCap
                                                        ? std::next(c->free_pages.begin(), kFreeListCap) : c->free_pages.end());
        if (!c->free_list.empty()) {
            rc = c->stage.upload_to(c->d_free, c->free_list.data(), c->free_list.size() * sizeof(int), stream);
            if (rc != MS_OK) return rc;
        }
        const int zero[2] = {0, 0};
        rc = c->stage.upload_to(c->d_commit_state, zero, sizeof(zero), stream);
        if (rc != MS_OK) return rc;
        c->free_list_valid = true;
        c->reserved_pages = 0;
    }
    int rc = flush_page_table_patches(c, stream);
    if (rc != MS_OK) return rc;
    CommitArgs a;
    a.pool = c->d.pool;
    a.d_pt = c->d_pt;
    a.d_len = c->d_len;
    a.inv_freq = c->d_inv_freq;
    a.d_free = c->d_free;
    a.state = c->d_commit_state;
    a.accept_len = accept_len;
    a.first_pid = first_pid;
    a.k = k_new;
    a.v = v_new;
    a.pos = pos_ids;
    a.B = B;
    a.n_q = n_q;
    a.n_max = n_max;
    a.n_kv_heads = c->d.n_kv_heads;
    a.max_pages = c->d.max_pages_per_seq;
    a.page_elems = (long)c->page_elems;
    a.layer_elems = (long)c->layer_elems;
    a.buf_layer_rows = (long)B * n_q;
    SeqIds ids;
    memset(&ids, 0, sizeof(ids));
    for (int b = 0; b < B; ++b) {
        ids.seq[b] = seq_ids[b];
        c->pending_growth[seq_ids[b]] += n_max;
    }
    c->reserved_pages += B;
    c->deferred = true;
    c->deferred_stream = stream;
    c->launches++;
    const dim3 grid((unsigned)(B * n_max), (unsigned)c->d.n_layers);
    return dispatch(c, [&](auto* tp, auto dc) -> int {
        using T = std::remove_pointer_t<decltype(tp)>;
        constexpr int D = decltype(dc)::value;
        hipLaunchKernelGGL((kv_commit_device<T, D>), grid, dim3(256), 0, stream, a, ids);
        MS_HIP_TRY(hipGetLastError());
        return (int)MS_OK;
    });
}

int ms_cache_sync(ms_cache* c) {
    if (!c) MS_FAIL(MS_ERR_INVALID, "ms_cache_sync: null cache");
    return reconcile(c);
}

int ms_step_positions_device(int B, const int* first_pid, int n_verify, int n_foresight, int* out, void* stream) {
    const int n_q = n_verify + n_foresight;
    if (B < 0 || n_verify < 0 || n_foresight < 0 || n_q < 1) MS_FAIL(MS_ERR_INVALID, "ms_step_positions_device: bad size");
    if (B == 0) return MS_OK;
    if (!first_pid || !out) MS_FAIL(MS_ERR_INVALID, "ms_step_positions_device: null argument");
    hipLaunchKernelGGL(step_positions_device, dim3((unsigned)((B * n_q + 255) / 256)), dim3(256), 0, (hipStream_t)stream, B, first_pid,
                       n_q, out);
    MS_HIP_TRY(hipGetLastError());
    return MS_OK;
}

size_t ms_compact_workspace_bytes(ms_cache* c, int B, const int* seq_ids, const int* seg_begin, const int* seg_len) {
    if (!c || B < 0 || (B > 0 && (!seq_ids || !seg_begin || !seg_len))) return 0;
    if (reconcile(c) != MS_OK) return 0;
    std::vector<int> cur(c->len);
    long tail = 0;
    for (int b = 0; b < B; ++b) {
        int s = seq_ids[b];
        if (s < 0 || s >= c->d.max_seqs || !c->live[s]) return 0;
        long t = (long)cur[s] - seg_begin[b] - seg_len[b];
        if (t > 0) tail += t;
    }
    return (size_t)tail * 2 * c->d.n_layers * c->d.n_kv_heads * c->d.head_dim * c->esize;
}

int ms_compact_segment(ms_cache* c, int B, const int* seq_ids, const int* seg_begin, const int* seg_len,
                       const int* n_mem, const void* mem_k, const void* mem_v, const int* mem_pos, int flags,
                       void* workspace, size_t ws_bytes, void* stream_) {
    hipStream_t stream = (hipStream_t)stream_;
    if (!c || B < 0 || (B > 0 && (!seq_ids || !seg_begin || !seg_len || !n_mem)))
        MS_FAIL(MS_ERR_INVALID, "ms_compact_segment: null argument");
    if (B > MS_MAX_BATCH) MS_FAIL(MS_ERR_INVALID, "ms_compact_segment: B %d exceeds %d", B, MS_MAX_BATCH);
    if (flags != MS_PRE_ROTATED && flags != MS_ROPE_APPLY) MS_FAIL(MS_ERR_INVALID, "ms_compact_segment: bad flags %d", flags);
    MS_RECONCILE(c);
    // ---- validate everything on a simulated copy of the lengths / page counts ----
    std::vector<int> sim_len(c->len);
    std::vector<int> sim_pages(c->d.max_seqs);
    for (int s = 0; s < c->d.max_seqs; ++s) sim_pages[s] = (int)c->pt[s].size();
    long sim_free = (long)c->free_pages.size();
    long total_mem = 0, total_tail = 0;
    for (int b = 0; b < B; ++b) {
        int rc = check_seq(c, seq_ids[b], "ms_compact_segment");
        if (rc != MS_OK) return rc;
        const int s = seq_ids[b], L = sim_len[s];
        if (seg_begin[b] < 0 || seg_len[b] < 0 || n_mem[b] < 0 || (long)seg_begin[b] + seg_len[b] > L)
            MS_FAIL(MS_ERR_RANGE, "ms_compact_segment: segment [%d, %d+%d) outside sequence %d of length %d", seg_begin[b],
                    seg_begin[b], seg_len[b], s, L);
        const int keep = pages_for(seg_begin[b]);
        const int new_len = L - seg_len[b] + n_mem[b];
        const int np = pages_for(new_len);
        if (np > c->d.max_pages_per_seq)
            MS_FAIL(MS_ERR_OOM_PAGES, "ms_compact_segment: sequence %d would need %d pages", s, np);
        sim_free += sim_pages[s] - keep;
        sim_free -= np - keep;
        if (sim_free < 0) MS_FAIL(MS_ERR_OOM_PAGES, "ms_compact_segment: pool exhausted");
        sim_pages[s] = np;
        sim_len[s] = new_len;
        total_mem += n_mem[b];
        total_tail += L - seg_begin[b] - seg_len[b];
    }
    if (total_mem > 0 && (!mem_k || !mem_v)) MS_FAIL(MS_ERR_INVALID, "ms_compact_segment: mem_k or mem_v is null");
    if (total_mem > 0 && flags == MS_ROPE_APPLY && !mem_pos) MS_FAIL(MS_ERR_INVALID, "ms_compact_segment: mem_pos is null");
    const size_t row_bytes = (size_t)c->d.n_kv_heads * c->d.head_dim * c->esize;
    const size_t need_ws = (size_t)total_tail * 2 * c->d.n_layers * row_bytes;
    if (total_tail > 0 && (!workspace || ws_bytes < need_ws))
        MS_FAIL(MS_ERR_WORKSPACE, "ms_compact_segment: rows follow a segment; workspace needs %zu bytes, has %zu", need_ws,
                workspace ? ws_bytes : (size_t)0);
    char* tail_k = (char*)workspace;
    char* tail_v = tail_k + (size_t)total_tail * c->d.n_layers * row_bytes;

    // ---- 1. save rows that follow each segment (old page tables still in the mirror) ----
    // A sequence listed twice would need its first splice applied before its second gather.
    std::vector<char> seen(c->d.max_seqs, 0);
    for (int b = 0; b < B; ++b) {
        if (seen[seq_ids[b]]) MS_FAIL(MS_ERR_INVALID, "ms_compact_segment: sequence %d is listed twice", seq_ids[b]);
        seen[seq_ids[b]] = 1;
    }
    std::vector<RowDesc> tails;
    int tprefix = 0;
    for (int b = 0; b < B; ++b) {
        const int s = seq_ids[b];
        const int t = c->len[s] - seg_begin[b] - seg_len[b];
        if (t > 0) {
            tails.push_back(RowDesc{s, seg_begin[b] + seg_len[b], tprefix, tprefix});
            tprefix += t;
        }
    }
    int rc = launch_rows(c, true, tails, (int)total_tail, tail_k, tail_v, nullptr, total_tail, 0, stream);
    if (rc != MS_OK) return rc;

    // ---- 2. host page tables: release, then re-grow (memory rows, then tail rows) ----
    std::vector<RowDesc> mems;
    std::vector<RowDesc> tails_dst;
    int mprefix = 0, moff = 0, tp2 = 0;
    for (int b = 0; b < B; ++b) {
        const int s = seq_ids[b];
        const int L = c->len[s];
        const int t = L - seg_begin[b] - seg_len[b];
        c->cut_to(s, seg_begin[b]);
        if (n_mem[b] > 0) {
            mems.push_back(RowDesc{s, c->len[s], moff, mprefix});
            mprefix += n_mem[b];
        }
        c->grow(s, n_mem[b]);
        moff += n_mem[b];
        if (t > 0) {
            tails_dst.push_back(RowDesc{s, c->len[s], tp2, tp2});
            tp2 += t;
        }
        c->grow(s, t);
        c->note_len(s);
    }
    // ---- 3. scatter memory rows (rotated at their UPL position ids), then the saved tails ----
    if (total_tail == 0 && total_mem > 0)
        return patch_and_scatter(c, mems, (int)total_mem, mem_k, mem_v, mem_pos, total_mem, flags == MS_ROPE_APPLY, stream);
    rc = flush_page_table_patches(c, stream);
    if (rc != MS_OK) return rc;
    rc = launch_rows(c, false, mems, (int)total_mem, mem_k, mem_v, mem_pos, total_mem, flags == MS_ROPE_APPLY, stream);
    if (rc != MS_OK) return rc;
    return launch_rows(c, false, tails_dst, (int)total_tail, tail_k, tail_v, nullptr, total_tail, 0, stream);
}

int ms_seq_len(ms_cache* c, int seq_id, int* len) {
    if (!c || !len) MS_FAIL(MS_ERR_INVALID, "ms_seq_len: null argument");
    int rc = check_seq(c, seq_id, "ms_seq_len");
    if (rc != MS_OK) return rc;
    rc = reconcile(c);
    if (rc != MS_OK) return rc;
    *len = c->len[seq_id];
    return MS_OK;
}

int ms_seq_page_table(ms_cache* c, int seq_id, int* out, int cap, int* n) {
    if (!c || !n || (cap > 0 && !out)) MS_FAIL(MS_ERR_INVALID, "ms_seq_page_table: null argument");
    int rc = check_seq(c, seq_id, "ms_seq_page_table");
    if (rc != MS_OK) return rc;
    rc = reconcile(c);
    if (rc != MS_OK) return rc;
    *n = (int)c->pt[seq_id].size();
    for (int i = 0; i < *n && i < cap; ++i) out[i] = c->pt[seq_id][i];
    return MS_OK;
}

int ms_free_page_count(ms_cache* c, int* n) {
    if (!c || !n) MS_FAIL(MS_ERR_INVALID, "ms_free_page_count: null argument");
    if (int rc = reconcile(c)) return rc;
    *n = (int)c->free_pages.size();
    return MS_OK;
}

int ms_peak_pages(ms_cache* c, int* n) {
    if (!c || !n) MS_FAIL(MS_ERR_INVALID, "ms_peak_pages: null argument");
    if (int rc = reconcile(c)) return rc;
    *n = c->peak_pages;
    return MS_OK;
}

int ms_launch_count(ms_cache* c, long long* n) {
    if (!c || !n) MS_FAIL(MS_ERR_INVALID, "ms_launch_count: null argument");
    *n = c->launches;
    return MS_OK;
}

int ms_check_integrity(ms_cache* c, void* stream) {
    if (!c) MS_FAIL(MS_ERR_INVALID, "ms_check_integrity: null cache");
    if (int rc = reconcile(c)) return rc;
    if (int rc = flush_page_table_patches(c, (hipStream_t)stream)) return rc;   // lengths of sequences created or freed since
    const std::string fault = c->check_tables();
    if (!fault.empty()) MS_FAIL(MS_ERR_INVALID, "integrity: %s", fault.c_str());
    if (!c->pending_pt.empty()) MS_FAIL(MS_ERR_INVALID, "integrity: page-table patches not flushed");
    MS_HIP_TRY(hipStreamSynchronize((hipStream_t)stream));
    if (__atomic_load_n(c->h_error, __ATOMIC_RELAXED) != 0)   // left set: the next attention call reports and clears it too
        MS_FAIL(MS_ERR_HIP, "integrity: an attention launch timed out waiting for split-KV partial results");
    std::vector<int> dev_len(c->d.max_seqs);
    MS_HIP_TRY(hipMemcpy(dev_len.data(), c->d_len, dev_len.size() * sizeof(int), hipMemcpyDeviceToHost));
    for (int s = 0; s < c->d.max_seqs; ++s)
        if (c->live[s] && dev_len[s] != c->len[s])
            MS_FAIL(MS_ERR_INVALID, "integrity: device copy of sequence %d's length is %d, host has %d", s, dev_len[s], c->len[s]);
    std::vector<int> row(c->d.max_pages_per_seq);
    for (int s = 0; s < c->d.max_seqs; ++s) {
        if (!c->live[s] || c->pt[s].empty()) continue;
        MS_HIP_TRY(hipMemcpy(row.data(), c->d_pt + (size_t)s * c->d.max_pages_per_seq, c->pt[s].size() * sizeof(int),
                             hipMemcpyDeviceToHost));
        for (size_t i = 0; i < c->pt[s].size(); ++i)
            if (row[i] != c->pt[s][i])
                MS_FAIL(MS_ERR_INVALID, "integrity: device mirror of sequence %d differs at page %zu (%d vs %d)", s, i, row[i],
                        c->pt[s][i]);
    }
    return MS_OK;
}

}  // extern "C"
