// i8 MFMA GEMM, tile 192x256 with 8 waves: all epilogue instantiations of this shape.
#include "q8_gemm_kernel.h"

namespace q8 {

int launch_tile_192x256_w8(const int8_t* xq, const int8_t* wq, int M, int N, int K, int group_m, const Epilogue& ep,
                       hipStream_t st)
{
    return launch_tile<192, 256, 2, 4, 3>(xq, wq, M, N, K, group_m, ep, st);
}

}  // namespace q8
