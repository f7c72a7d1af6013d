// Backward bf16 kernels for head dimension 128.
#include "sattn_bwd_launch.hpp"

template int sattn::launch_bwd_bf16<128>(sattn::BwdParams, bool, bool, int, bool, int, bool, hipStream_t);
