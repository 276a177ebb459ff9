// Paged decode on the matrix cores: the head_dim 256 kernels.
#include "decode_mfma_impl.h"

namespace pa {

template void launch_decode_mfma_dim<256>(const AttnArgs&, hipStream_t);
template void launch_decode_short_dim<256>(const AttnArgs&, hipStream_t);

}  // namespace pa
