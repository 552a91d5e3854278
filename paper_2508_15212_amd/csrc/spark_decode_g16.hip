// Decode-attention kernels for query groups of 16 heads per KV head.
#include "spark_decode_kernel.h"

namespace spark {
template hipError_t launch_g<16>(const DecodeParams &, int, hipStream_t);
}
