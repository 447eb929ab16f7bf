// placeholder (replaced below)
#pragma once
#include "tv_common.hpp"
namespace tvk {
inline hipError_t launch_fwd_long(const FwdParams &, hipStream_t) { return hipErrorNotSupported; }
inline hipError_t launch_bwd_long(const BwdParams &, hipStream_t) { return hipErrorNotSupported; }
}
