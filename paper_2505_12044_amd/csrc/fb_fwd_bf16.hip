// Head-dimension switch of the bf16 forward; the kernels live in fb_fwd_bf16_impl.h and are
// instantiated per C in fb_fwd_bf16_c{16,32,64,128}.hip.
#include "fb_launch.h"

int fb_launch_fwd_bf16_c16(const FwdParams& p, int rp, bool dense, int qb, hipStream_t stream);
int fb_launch_fwd_bf16_c32(const FwdParams& p, int rp, bool dense, int qb, hipStream_t stream);
int fb_launch_fwd_bf16_c64(const FwdParams& p, int rp, bool dense, int qb, hipStream_t stream);
int fb_launch_fwd_bf16_c128(const FwdParams& p, int rp, bool dense, int qb, hipStream_t stream);

int fb_launch_fwd_bf16(const FwdParams& p, int C, int rp, bool dense, int qb, hipStream_t stream) {
    switch (C) {
        case 16: return fb_launch_fwd_bf16_c16(p, rp, dense, qb, stream);
        case 32: return fb_launch_fwd_bf16_c32(p, rp, dense, qb, stream);
        case 64: return fb_launch_fwd_bf16_c64(p, rp, dense, qb, stream);
        case 128: return fb_launch_fwd_bf16_c128(p, rp, dense, qb, stream);
        default: return -1;
    }
}
