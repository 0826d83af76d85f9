// Position-layout helpers: pure integer functions of the MemoSight paper's rules.
//   AMA  -- Section 2.1.2 "Adaptive Memory Allocation": l = ceil(|R_i| / c)
//   UPL  -- Section 2.1.2 "Uniform Position Layout" and Section 2.2 "Position ID Assignment":
//           each memory token takes the centre PID of its group of c step tokens
//   <o>  -- Section 2.2: the output token takes the PID after the step's last token
//   <f>  -- Section 2.1.1: foresight PIDs increase by one from the prefix's last PID; a foresight
//           token holds the PID just before the token it predicts
//   per-position foresight -- Section 2.2 "CoT Augmentation" / Section 2.3 "MTP Attention": the
//           training layout (foresight tokens at every position of the step) as a decode step
//   ablation layouts -- Appendix B: consecutive memory PIDs (w/o UPL), fixed budget (w/o AMA)
#include "memosight.h"

extern "C" {

int ms_ama_count(int n_tokens, int c) {
    if (n_tokens < 0 || c <= 0) return MS_ERR_INVALID;
    return (int)(((long)n_tokens + c - 1) / c);
}

int ms_upl_positions(int first_pid, int n_tokens, int c, int* out, int cap) {
    const int groups = ms_ama_count(n_tokens, c);
    if (groups < 0) return groups;
    for (int g = 0; g < groups && g < cap; ++g) {
        const long first = (long)g * c;                                   // step-local, inclusive
        const long last = (first + c < n_tokens ? first + c : n_tokens) - 1;
        // middle member of the group; the lower one when the group has an even size
        out[g] = first_pid + (int)((first + last) / 2);
    }
    return groups;
}

int ms_output_token_pid(int last_pid) { return last_pid + 1; }

int ms_foresight_pids(int last_prefix_pid, int d, int* out, int cap) {
    if (d < 0) return MS_ERR_INVALID;
    for (int j = 0; j < d && j < cap; ++j) out[j] = last_prefix_pid + 1 + j;
    return d;
}

int ms_step_positions(int B, const int* first_pid, int n_verify, int n_foresight, int* out) {
    if (B < 0 || n_verify < 0 || n_foresight < 0 || (B > 0 && (!first_pid || !out))) return MS_ERR_INVALID;
    const int n_q = n_verify + n_foresight;
    for (int b = 0; b < B; ++b) {
        int* row = out + (long)b * n_q;
        for (int i = 0; i < n_verify; ++i) row[i] = first_pid[b] + i;
        // the prefix ends at the last verify token (or just before first_pid if there is none)
        ms_foresight_pids(first_pid[b] + n_verify - 1, n_foresight, row + n_verify, n_foresight);
    }
    return B * n_q;
}

int ms_default_ctx_new(int n_verify, int n_foresight, int* out, int cap) {
    if (n_verify < 0 || n_foresight < 0) return MS_ERR_INVALID;
    const int n = n_verify + n_foresight;
    for (int i = 0; i < n && i < cap; ++i) out[i] = i < n_verify ? i : n_verify;
    return n;
}

int ms_per_position_layout(int first_pid, int n_verify, int d, int* pos_out, int* ctx_out, int cap) {
    if (n_verify < 0 || d < 0) return MS_ERR_INVALID;
    const long n = (long)n_verify * (1 + d);
    if (n > 0x7fffffffL) return MS_ERR_INVALID;
    int at = 0;
    auto put = [&](int pid, int ctx) {
        if (at < cap) {
            if (pos_out) pos_out[at] = pid;
            if (ctx_out) ctx_out[at] = ctx;
        }
        ++at;
    };
    for (int j = 0; j < n_verify; ++j) put(first_pid + j, j);
    for (int j = 0; j < n_verify; ++j)
        for (int k = 1; k <= d; ++k) put(first_pid + j + k, j + 1);
    return at;
}

int ms_consecutive_memory_positions(int last_pid, int n_mem, int* out, int cap) {
    if (n_mem < 0) return MS_ERR_INVALID;
    for (int j = 0; j < n_mem && j < cap; ++j) out[j] = last_pid + 1 + j;
    return n_mem;
}

int ms_upl_positions_fixed(int first_pid, int n_tokens, int n_mem, int* out, int cap) {
    if (n_tokens < 1 || n_mem < 1) return MS_ERR_INVALID;
    for (int g = 0; g < n_mem && g < cap; ++g) {
        const long lo = (long)g * n_tokens / n_mem;
        long hi = (long)(g + 1) * n_tokens / n_mem - 1;
        if (hi < lo) hi = lo;   // more memory tokens than step tokens: the group is its boundary token
        out[g] = first_pid + (int)((lo + hi) / 2);
    }
    return n_mem;
}

}  // extern "C"
