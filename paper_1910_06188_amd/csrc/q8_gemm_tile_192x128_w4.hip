// i8 MFMA GEMM, tile 192x128 with 4 waves, two workgroups per compute unit: all epilogue instantiations of this shape.
#include "q8_gemm_kernel.h"

namespace q8 {

int launch_tile_192x128_w4(const int8_t* xq, const int8_t* wq, int M, int N, int K, int group_m, const Epilogue& ep,
                       hipStream_t st)
{
    return launch_tile<192, 128, 2, 2, 2>(xq, wq, M, N, K, group_m, ep, st);
}

}  // namespace q8
