/* The public header must be plain C (C99): compiled, not run.  Takes the address of every
 * entry point so that a declaration that does not parse, or a missing one, fails the build. */
#include "../../include/skipffn.h"

typedef void (*fn)(void);
fn skipffn_entry_points[] = {
    (fn)skipffn_compact_workspace_bytes, (fn)skipffn_compact,
    (fn)skipffn_saved_bytes, (fn)skipffn_forward_workspace_bytes, (fn)skipffn_forward,
    (fn)skipffn_backward_workspace_bytes, (fn)skipffn_backward,
    (fn)skipffn_gather_rows, (fn)skipffn_kv_compact,
    (fn)skipffn_summary_saved_bytes, (fn)skipffn_summary_workspace_bytes,
    (fn)skipffn_summary_forward, (fn)skipffn_summary_backward,
    (fn)skipffn_select_retained,
    (fn)skipffn_token_merge_workspace_bytes, (fn)skipffn_token_merge,
    (fn)skipffn_token_merge_backward,
    (fn)skipffn_probe_mfma,
    (fn)skipffn_saved_layout, (fn)skipffn_status_string, (fn)skipffn_last_hip_error,
    (fn)skipffn_version, (fn)skipffn_profile_begin, (fn)skipffn_profile_end,
};
