// Per-column constants and the per-element epilogue of the quantized FC layer (Section 3:
// Int32 bias at scale S_x S_W, dequantize; optional fp32 GELU, requantize), shared by the
// MFMA kernel and the generic kernel so that both give identical results.
#pragma once
#include "q8_device.h"
#include "q8_launch.h"

namespace q8 {

__device__ __forceinline__ unsigned f32_abs_bits(float v) { return __float_as_uint(v) & 0x7fffffffu; }

struct ColConst {
    int bq;    // quantized bias of this column
    float r;   // 1 / (S_x * S_W[group])
};

__device__ __forceinline__ ColConst col_const(const Epilogue& ep, int n, float sx)
{
    float sw = ep.sw[n / ep.cols_per_group];
    ColConst c;
    c.bq = ep.bias ? quantize_bias(ep.bias[n], sx, sw) : 0;
    c.r = dequant_factor(sx, sw);
    return c;
}

// One output element: dequantize, optional GELU, optional residual addition (one fp32 add),
// optional requantize; returns the bit pattern of |y| for the optional abs-max.
__device__ __forceinline__ unsigned epilogue_store(const Epilogue& ep, int64_t idx, int acc, float r, float next_scale)
{
    if (ep.acc_out) ep.acc_out[idx] = acc;
    float y = (float)acc * r;
    if (ep.flags & 1u) y = gelu_erf(y);
    if (ep.residual) y = __fadd_rn(y, ep.residual[idx]);
    if (ep.flags & 4u)
        reinterpret_cast<int8_t*>(ep.y)[idx] = (int8_t)quantize_code(y, next_scale);
    else
        reinterpret_cast<float*>(ep.y)[idx] = y;
    return f32_abs_bits(y);
}

}  // namespace q8
