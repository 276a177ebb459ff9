#include "common.h"
namespace pa {
bool prefill_mfma_supported(const AttnArgs&) { return false; }
pa_status launch_prefill_mfma(const AttnArgs&, hipStream_t) { return PA_ERR_UNSUPPORTED; }
}
