// Decode-attention kernels for query groups of 1 head per KV head.
#include "spark_decode_kernel.h"

namespace spark {
template hipError_t launch_g<1>(const DecodeParams &, int, hipStream_t);
}
