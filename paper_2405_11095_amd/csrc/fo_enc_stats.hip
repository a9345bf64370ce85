// The dither + sign + pack kernels with the diagnostic counters of fo_stats compiled in (see fo_set_stats).
#include "fo_enc_pack.h"

namespace fo_host {

template int launch_pack_s<IN_GRAD, true>(fo_plan *, int, dim3, hipStream_t, const ContigArgs &, const PtrTab &);
template int launch_pack_s<IN_F32, true>(fo_plan *, int, dim3, hipStream_t, const ContigArgs &, const PtrTab &);

} // namespace fo_host
