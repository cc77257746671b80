// Retrieval drafter over the token history (paper Sec. 3: drafts come from the context; Sec. 5.1:
// suffix-automaton retrieval): host code only, no device work.  The draft is what followed the most
// recent earlier occurrence of the longest suffix of the history.  Histories here are a few
// thousand tokens and suffixes a handful, so the search is the plain one: candidate end positions
// from the most recent back, extended backwards while they agree with the suffix; the best length
// so far is kept, and a full-length match ends the search.
#include "vf_internal.h"

int vf_draft_suffix_match(const int32_t *history_host, int n, int max_suffix, int min_suffix, int k,
                          int32_t *drafts_host) {
    if (n < 0 || (n > 0 && !history_host) || max_suffix < 1 || min_suffix < 1 || min_suffix > max_suffix || k < 0 ||
        k > VF_MAX_DRAFTS || (k > 0 && !drafts_host))
        return vf_fail(VF_ERR_ARG, "vf_draft_suffix_match: n %d, suffix %d..%d, k %d", n, min_suffix, max_suffix, k);
    if (k == 0 || n < 2) return 0;
    const int cap = max_suffix < n - 1 ? max_suffix : n - 1;
    int best_len = 0, best_end = -1;  // the occurrence covers history[best_end - best_len + 1 .. best_end]
    for (int end = n - 2; end >= 0 && best_len < cap; --end) {
        int len = 0;
        while (len < cap && len <= end && history_host[end - len] == history_host[n - 1 - len]) ++len;
        if (len > best_len) {  // strictly longer only: among equal lengths the most recent (first seen) stays
            best_len = len;
            best_end = end;
        }
    }
    if (best_len < min_suffix) return 0;
    int out = 0;
    for (int p = best_end + 1; p < n && out < k; ++p) drafts_host[out++] = history_host[p];
    return out;
}
