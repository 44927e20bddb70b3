// Internal declarations shared by the translation units of libxkv.
#ifndef XKV_INTERNAL_H
#define XKV_INTERNAL_H

#include <stddef.h>
#include <stdint.h>

#include "xkv.h"

namespace xkv {

// Granularity of the work split of a stream: strips are multiples of this many slots.
constexpr int kChunk = 256;
// Longest strip one workgroup of the streaming kernel handles.
constexpr int kMaxStripRows = 4096;
// (layer, sequence) regions described in the kernel arguments of one launch.
constexpr int kMaxPairs = 128;

inline int64_t ceil_div(int64_t a, int64_t b) { return (a + b - 1) / b; }

// Checks everything about a cache descriptor that can be checked on the host.
xkv_status check_cache(const xkv_cache* c);
// Checks a layer range against a checked cache.
xkv_status check_layers(const xkv_cache* c, int32_t layer_begin, int32_t layer_end);

// Workspace needs, in bytes, for `layers` layers in the worst case (by cap).
size_t attend_workspace_bytes(const xkv_cache* c, int32_t layers);
size_t evict_workspace_bytes(const xkv_cache* c, int32_t layers);

// What xkv_evict_compact checks of its arguments before it enqueues anything, for a
// cache whose regions will hold extra_rows more tokens each by then.
xkv_status evict_check_args(const xkv_cache* cache, int32_t layer_begin, int32_t layer_end, const int32_t* budgets,
                            int32_t pool_size, int32_t n_protect, int32_t extra_rows, const void* workspace,
                            size_t workspace_bytes);

// Remembers the control words of the most recent launch that waits inside a kernel
// (word 1: some workgroup gave up its wait), for xkv_fused_status; null: the most
// recent call had no such launch.
void note_waiting_launch(const unsigned* control, void* stream);
// XKV_CFG_FUSED_SPIN_LIMIT as it stands.
uint32_t fused_spin_limit();

// Per-kernel event timing (xkv_profile_*).  begin() returns a token >= 0 when
// timing is on and records the start event on the stream; end() records the
// stop event.  Both are no-ops when timing is off.
int profile_begin(int kernel_index, void* stream);
void profile_end(int token, void* stream);

}  // namespace xkv

#endif  // XKV_INTERNAL_H
