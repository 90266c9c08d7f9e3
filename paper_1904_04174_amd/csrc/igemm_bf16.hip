// bf16 implicit-GEMM convolution (placeholder until the MFMA kernel lands).
#include "conv2d_internal.h"

namespace conv2d {
int igemm_bf16_num_tiles() { return 0; }
const char* igemm_bf16_tile_name(int) { return ""; }
void igemm_bf16_tile_shape(int, int* bm, int* bn, int* bk) { *bm = *bn = *bk = 0; }
hipError_t launch_igemm_bf16(const Problem&, int, hipStream_t) { return hipErrorNotSupported; }
}  // namespace conv2d
