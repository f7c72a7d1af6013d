// Backward bf16 kernels for head dimension 64.
#include "sattn_bwd_launch.hpp"

template int sattn::launch_bwd_bf16<64>(sattn::BwdParams, bool, bool, int, bool, int, bool, hipStream_t);
