// Forward bf16 kernels for head dimension 128.
#include "sattn_fwd_launch.hpp"

template int sattn::launch_fwd_bf16<128>(sattn::FwdParams, int, int, bool, bool, int, bool, hipStream_t);
