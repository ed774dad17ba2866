#include "fm_common.h"
#include "fm_kernels.h"
hipError_t fm_launch_dvec(const FmBwdArgs& a, hipStream_t stream) { return hipErrorNotSupported; }
hipError_t fm_launch_bwd_dq(const FmBwdArgs& a, hipStream_t stream) { return hipErrorNotSupported; }
hipError_t fm_launch_bwd_dkdv(const FmBwdArgs& a, hipStream_t stream) { return hipErrorNotSupported; }
