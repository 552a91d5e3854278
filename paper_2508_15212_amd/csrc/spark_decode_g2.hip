// Decode-attention kernels for query groups of 2 heads per KV head.
#include "spark_decode_kernel.h"

namespace spark {
template hipError_t launch_g<2>(const DecodeParams &, int, hipStream_t);
}
