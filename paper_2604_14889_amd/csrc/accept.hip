// Greedy longest-prefix acceptance (footnote of Section 2.1.1 of the MemoSight paper: the accepted
// tokens are the leading drafts that coincide with the model's argmax predictions; Algorithm 1 ends
// a step when the boundary token is among the accepted ones).
#include "ms_internal.h"

namespace ms {

// One lane per sequence; n is at most a handful, so the scan is serial per lane.
__global__ void accept_prefix(int B, int n, const int* __restrict__ draft, const int* __restrict__ target,
                              const int* __restrict__ stop_ids, int n_stop, int* __restrict__ accept_len,
                              int* __restrict__ next_token) {
    const int b = blockIdx.x * blockDim.x + threadIdx.x;
    if (b >= B) return;
    const int* dr = draft + (size_t)b * n;
    const int* tg = target + (size_t)b * n;
    int a = 0;
    while (a < n && dr[a] == tg[a]) {
        const int tok = dr[a];
        ++a;
        bool stop = false;
        for (int s = 0; s < n_stop; ++s) stop |= (stop_ids[s] == tok);
        if (stop) break;
    }
    accept_len[b] = a;
    next_token[b] = a < n ? tg[a] : -1;
}

}  // namespace ms

extern "C" int ms_accept(int B, int n, const int* draft, const int* target, const int* stop_ids, int n_stop,
                         int* accept_len, int* next_token, void* stream) {
    if (B < 0 || n < 0 || n_stop < 0) MS_FAIL(MS_ERR_INVALID, "ms_accept: negative size");
    if (B == 0) return MS_OK;
    if (!accept_len || !next_token || (n > 0 && (!draft || !target)) || (n_stop > 0 && !stop_ids))
        MS_FAIL(MS_ERR_INVALID, "ms_accept: null argument");
    hipLaunchKernelGGL(ms::accept_prefix, dim3((unsigned)((B + 63) / 64)), dim3(64), 0, (hipStream_t)stream, B, n, draft,
                       target, stop_ids, n_stop, accept_len, next_token);
    MS_HIP_TRY(hipGetLastError());
    return MS_OK;
}
