// Configuration selection: which compiled kernel (and split-K factor) runs a problem when
// no override is active.  The table of shape classes below is the outcome of the on-device
// parameter sweep (paper Section 3.3: tuned parameters looked up by the routine's host code).
#pragma once
#include "internal.h"

namespace mg {

// Sets *kernel (-1 if nothing applies) and *split.  workspace_bytes: what the caller can offer for split-K
// partial sums (a configuration that needs more is not chosen).
void select_config(const std::vector<KernelEntry> &table, const Problem &p, int64_t alignment, size_t workspace_bytes,
                   int32_t *kernel, int32_t *split);
// Returns the kernel id for a batched problem, or -1.
int32_t select_batched(const std::vector<KernelEntry> &table, const BatchedProblem &p);

}  // namespace mg
