// Position-layout helpers: pure integer functions of the MemoSight paper's rules.
//   AMA  -- Section 2.1.2 "Adaptive Memory Allocation": l = ceil(|R_i| / c)
//   UPL  -- Section 2.1.2 "Uniform Position Layout" and Section 2.2 "Position ID Assignment":
//           each memory token takes the centre PID of its group of c step tokens
//   <o>  -- Section 2.2: the output token takes the PID after the step's last token
//   <f>  -- Section 2.1.1: foresight PIDs increase by one from the prefix's last PID; a foresight
//           token holds the PID just before the token it predicts
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

int ms_default_ctx_new(int n_verify, int n_foresight, int* out, int cap) {
    if (n_verify < 0 || n_foresight < 0) return MS_ERR_INVALID;
    const int n = n_verify + n_foresight;
    for (int i = 0; i < n && i < cap; ++i) out[i] = i < n_verify ? i : n_verify;
    return n;
}

}  // extern "C"
