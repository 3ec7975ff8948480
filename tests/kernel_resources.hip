// Instantiations of the decode kernel for the headline shape only (with and without the code for short pairs),
// compiled by test_kernel_resources.py to read the compiler's resource report: seconds instead of the minutes of
// the whole library.
#include "decode_mfma.h"
template __global__ void fairkv::fairkv_decode_mfma_kernel<128, 8, false, false, false, false>(fairkv::DecodeArgs);
template __global__ void fairkv::fairkv_decode_mfma_kernel<128, 8, false, false, true, false>(fairkv::DecodeArgs);
template __global__ void fairkv::fairkv_decode_mfma_kernel<128, 4, true, true, true, false>(fairkv::DecodeArgs);
