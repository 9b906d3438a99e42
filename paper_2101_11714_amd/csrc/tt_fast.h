// Specialised kernels for the shapes the paper uses (placeholder: none yet).
#pragma once

#include "tt_common.h"

namespace tt {

// Returns 0 if a specialised forward kernel was launched, -1 if the shape has none.
static inline int fast_fwd(const Params &, const float *, const float *, const float *, const int64_t *,
                           const int64_t *, int, const float *, const CacheDev &, float *, hipStream_t)
{
    return -1;
}

static inline bool fast_bwd_supported(const Params &) { return false; }

static inline void fast_bwd(const Params &, const float *, const float *, const float *, const int64_t *, int,
                            const int64_t *, int, const float *, const int32_t *, const float *, float *, float *,
                            float *, hipStream_t)
{
}

}  // namespace tt
