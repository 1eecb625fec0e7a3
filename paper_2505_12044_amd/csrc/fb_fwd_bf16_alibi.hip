// bf16 forward with the ALiBi bias generated inside the kernel (factor mode 4 of the four-wave
// kernel in fb_fwd_bf16_impl.h): instantiations for every head dimension.
#include "fb_fwd_bf16_impl.h"

int fb_launch_fwd_bf16_alibi(const FwdParams& p, int C, int qb, hipStream_t stream) {
    switch (C) {
        case 16: return dispatch_qb<32, 16, 4, false, 16>(p, qb, stream);
        case 32: return dispatch_qb<32, 16, 4, false>(p, qb, stream);
        case 64: return dispatch_qb<64, 16, 4, false>(p, qb, stream);
        case 128: return dispatch_qb<128, 16, 4, false>(p, qb, stream);
        default: return -1;
    }
}
