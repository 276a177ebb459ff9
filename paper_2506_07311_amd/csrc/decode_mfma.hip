#include "common.h"
namespace pa {
bool decode_mfma_supported(const AttnArgs&) { return false; }
pa_status launch_decode_mfma(const AttnArgs&, hipStream_t) { return PA_ERR_UNSUPPORTED; }
}
