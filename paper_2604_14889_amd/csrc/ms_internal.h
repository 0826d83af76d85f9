// Internal declarations shared by the library's translation units (not part of the C ABI).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include <set>
#include <vector>

#include "host_tables.h"
#include "memosight.h"

namespace ms {

void set_error(const char* fmt, ...) __attribute__((format(printf, 1, 2)));
void clear_error();

#define MS_FAIL(code, ...)          \
    do {                            \
        ::ms::set_error(__VA_ARGS__); \
        return (code);              \
    } while (0)

#define MS_HIP_TRY(expr)                                                               \
    do {                                                                               \
        hipError_t e_ = (expr);                                                        \
        if (e_ != hipSuccess) {                                                        \
            ::ms::set_error("%s failed: %s", #expr, hipGetErrorString(e_));            \
            return MS_ERR_HIP;                                                         \
        }                                                                              \
    } while (0)

// Pinned-host + device staging ring for small control uploads.  A slot's pinned half may be
// rewritten once the event recorded after its copy has completed; the device half is only
// rewritten by a later copy on the same stream, i.e. after every kernel that read it.
struct StageRing {
    static constexpr int kSlots = 16;
    static constexpr size_t kSlotBytes = 256 * 1024;
    char* h = nullptr;
    char* d = nullptr;
    hipEvent_t ev[kSlots] = {};
    bool used[kSlots] = {};
    int next = 0;
    int init();
    void destroy();
    // Copies `bytes` (<= kSlotBytes) to a device slot on `stream`; *dev receives the slot address.
    int upload(const void* src, size_t bytes, hipStream_t stream, void** dev);
    // Same through a pinned slot, but to a device address of the caller's.
    int upload_to(void* dst, const void* src, size_t bytes, hipStream_t stream);
};

// Which rows of a packed [rows][Hkv][D] buffer go to / come from which logical cache rows.
struct RowDesc {
    int seq;          // sequence id
    int cache_begin;  // logical cache row of this sequence's first row in the call
    int buf_first;    // row index of that first row in the packed buffer (per layer)
    int prefix;       // number of rows of earlier sequences in this call
};

}  // namespace ms

// The host tables (page tables, free pages, lengths, queued mirror updates, version) are the base
// class: plain C++ that also builds for the CPU alone.
struct ms_cache : ms::HostTables {
    ms_cache_desc d;
    int device = 0;
    int group = 1;               // query heads per KV head
    size_t esize = 2;            // bytes per element
    size_t page_elems = 0;       // elements per page (all heads, K and V)
    size_t layer_elems = 0;      // elements per layer
    int* d_pt = nullptr;         // device mirror [max_seqs][max_pages_per_seq]
    int* d_len = nullptr;        // device [max_seqs]: the sequences' lengths as the kernels see them
    // ---- device-side commits (ms_commit_accepted_device): the kernels take pages from an ordered
    // list of free pages and advance d_len; the host tables below are stale until reconciled
    int* d_free = nullptr;       // device [kFreeListCap]: free pages in ascending order, as uploaded at the last reconcile
    int* d_commit_state = nullptr;  // device: {pages taken from d_free so far, layers arrived}, then [kFreeListCap] the sequence
                                 // that took each page, in order, then one arrival counter per layer (64 ints apart)
    std::vector<int> free_list;  // host copy of what d_free holds
    bool free_list_valid = false;
    int reserved_pages = 0;      // upper bound of the pages device-side commits may have taken since the last reconcile
    std::vector<int> pending_growth;   // per sequence: upper bound of the rows added on the device since the last reconcile
    bool deferred = false;       // device-side commits are outstanding: host lengths / page tables are stale
    hipStream_t deferred_stream = nullptr;
    float* d_inv_freq = nullptr; // device [head_dim / 2]
    ms::StageRing stage;
    int n_cus = 256;             // compute units of the device
    int* d_plan = nullptr;       // device copy of the streaming kernel's work plan
    int* d_arrive = nullptr;     // [MS_MAX_BATCH][n_kv_heads][2] counters of the streaming kernel: shares finished, partials published
    int* h_error = nullptr;      // pinned host word the streaming kernel sets when a closing workgroup times out
    int* d_error = nullptr;      // the same word as the device sees it
    int poll_limit = 0;          // polls before a closing workgroup gives up; 0 = the default (about a second)
    std::vector<int> plan_key;   // batch (ids, lengths) the plan was built for
    int plan_items = 0, plan_parts = 0, plan_B = 0;
    std::vector<hipEvent_t> prof_start, prof_stop;  // event pairs around the streaming kernel
    bool deterministic = false;   // attention: fixed tile-to-wave assignment (bitwise reproducible)
    int prof_count = 0;
    int prof_stride = 1;   // every prof_stride-th eligible call opens a timed span
    int prof_span = 1;     // consecutive calls one event pair covers
    int prof_open = 0;     // calls the open span still waits for
    int prof_seen = 0;
    long long launches = 0;   // kernels launched by calls on this cache so far
};

namespace ms {

constexpr int kFreeListCap = 16384;   // entries of the device-side free-page list

// cache.hip
int flush_page_table_patches(ms_cache* c, hipStream_t stream);
// Brings the host tables up to date with device-side commits (synchronises their stream); a no-op otherwise.
int reconcile(ms_cache* c);
int check_seq(const ms_cache* c, int seq, const char* what);

}  // namespace ms
