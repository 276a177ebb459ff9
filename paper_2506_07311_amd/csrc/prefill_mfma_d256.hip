// Paged prefill on the matrix cores: the head_dim 256 kernels.
#include "prefill_mfma_impl.h"

namespace pa {

template pa_status launch_prefill_mfma_dim<256>(const AttnArgs&, const prefill::PrefillPlan&, int64_t, int64_t,
                                                hipStream_t);

}  // namespace pa
