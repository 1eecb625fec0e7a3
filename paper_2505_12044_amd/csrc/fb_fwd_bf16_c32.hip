// bf16 forward kernels for head dimension C = 32 (one translation unit per C so they build in parallel).
#include "fb_fwd_bf16_impl.h"

int fb_launch_fwd_bf16_c32(const FwdParams& p, int rp, bool dense, int qb, hipStream_t stream) {
    return fwd_bf16_dispatch<32>(p, rp, dense, qb, stream);
}
