// IVFADC search (Section 2.3.2; Index, Tables and Scan steps of Section 2.3.3).
#include "pq_internal.h"

namespace pq {

int launch_ivf(pq_ctx *ctx, const ivf_lists *, const float *, int, int, int, const float *, int, int, int, float *,
               int64_t *, int32_t *) {
    return fail(ctx, PQ_EUNSUPPORTED, "ivf_adc_search: not built yet");
}

}  // namespace pq
