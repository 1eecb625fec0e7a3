// bf16 forward kernels for head dimension C = 16: the C = 32 tiles of the four-wave kernel with
// channels 16..31 zero-filled on the way in and never stored.
#include "fb_fwd_bf16_impl.h"

namespace {

// Head dimension 16 on the C = 32 tiles of the four-wave kernel (qb = 1 or 2).
int fwd_bf16_dispatch_c16(const FwdParams& p, int rp, bool dense, int qb, hipStream_t stream) {
    if (qb != 2) qb = 1;
    if (dense) return dispatch_qb<32, 0, 0, true, 16>(p, qb, stream);
    switch (rp) {
        case 0: return dispatch_qb<32, 0, 0, false, 16>(p, qb, stream);
        case 16: return dispatch_pm<32, 16, 16>(p, qb, stream);
        case 32: return dispatch_pm<32, 32, 16>(p, qb, stream);
        case 48: return dispatch_pm<32, 48, 16>(p, qb, stream);
        case 64: return dispatch_pm<32, 64, 16>(p, qb, stream);
        default: break;
    }
    // wider blocks of extra channels (multiplicative form): bf16 columns in whole 16-byte chunks
    if (p.phi_f32 || (p.R % 8) != 0) return -1;
    if (rp == 96) return dispatch_causal<32, 96, 1, 1, false, 16>(p, stream);
    if (rp == 128) return dispatch_causal<32, 128, 1, 1, false, 16>(p, stream);
    return -1;
}

}  // namespace

int fb_launch_fwd_bf16_c16(const FwdParams& p, int rp, bool dense, int qb, hipStream_t stream) {
    return fwd_bf16_dispatch_c16(p, rp, dense, qb, stream);
}
