// Elementary operations the codec's arithmetic rests on, one per launch, for the test that compares
// them bit for bit with the host's IEEE arithmetic (see slicer_arith_probe in include/slicer.h).
// Every operation is written exactly as the kernels write it (same operators, same helpers, same
// compiler flags), so a change of a flag or of the compiler's defaults (division not correctly rounded,
// a contracted multiply-add, flushed denormals) shows up here before it shows up as a parity failure.
#include "../../include/slicer.h"

#include <hip/hip_runtime.h>

#include "slicer_common.hpp"

using namespace slicer;

namespace {

__global__ __launch_bounds__(256) void arith_probe_kernel(int op, const u32* __restrict__ a, const u32* __restrict__ b,
                                                          u32* __restrict__ out, int64_t n)
{
    const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (i >= n) return;
    const float x = __uint_as_float(a[i]), y = __uint_as_float(b[i]);
    u32 r = 0;
    switch (op) {
        case 0: r = __float_as_uint(x / y); break;                               // quantiser scale L / range
        case 1: r = __float_as_uint(__fdiv_rn(x, y)); break;                     // decoder step
        case 2: r = __float_as_uint(x * y); break;
        case 3: r = __float_as_uint(x + y); break;
        case 4: r = __float_as_uint(x - y); break;
        case 5: r = __float_as_uint(rintf(x)); break;                            // codes: round half to even
        case 6: r = __float_as_uint(ldexpf(x, (int)(b[i] % 301u) - 150)); break; // block scale, energy grid
        case 7: r = __float_as_uint(x * y + 8388608.0f); break;                  // residual: multiply, then add (no contraction)
        case 8: r = f32_to_bf16_rne(x); break;                                   // bf16 output
        case 9: r = __float_as_uint(__fadd_rn(x, __fmul_rn(y, y))); break;       // decoder: vmin + c * step
        case 10: {                                                               // energy grid on the significand
            const u32 bits = a[i] & 0x7FFFFFFFu;
            const int e = ilogb_bits(bits ? bits : 1u) + 1 + (int)(b[i] % 3u);
            r = bits ? energy_grid(bits, e) : 0u;
            break;
        }
        case 11: {                                                               // feasibility side: products in double
            const double d = ((double)x * (double)x) * (double)(b[i]) * 0x1p-30;
            r = (u32)(__double_as_longlong(d) >> 32) ^ (u32)__double_as_longlong(d);
            break;
        }
        default: break;
    }
    out[i] = r;
}

}  // namespace

extern "C" int slicer_arith_probe(int op, const void* a, const void* b, void* out, int64_t n, void* hip_stream)
{
    if (op < 0 || op > 11 || !a || !b || !out || n <= 0) return SLICER_EINVAL;
    hipLaunchKernelGGL(arith_probe_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, (hipStream_t)hip_stream, op,
                       (const u32*)a, (const u32*)b, (u32*)out, n);
    return hipGetLastError() == hipSuccess ? SLICER_OK : SLICER_EHIP;
}
