// Placeholder until the backward kernels land: reports "no instantiation".
#include "fb_launch.h"
int fb_launch_bwd_bf16(const BwdParams&, int, int, hipStream_t) { return -1; }
