// bf16 forward kernels for head dimension C = 16: the C = 32 tiles of the four-wave kernel with
// channels 16..31 zero-filled on the way in and never stored.
#include "fb_fwd_bf16_impl.h"

int fb_launch_fwd_bf16_c16(const FwdParams& p, int rp, bool dense, int qb, hipStream_t stream) {
    return fwd_bf16_dispatch_c16(p, rp, dense, qb, stream);
}
