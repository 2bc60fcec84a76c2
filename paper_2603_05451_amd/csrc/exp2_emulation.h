// Software 2^x on the vector ALU (paper Sec. 3.1.3), device function only; shared by the
// elementwise entry point of the library (exp2_emulated.hip) and by the rate probes (probes.hip).
//
// Steps of the section: clamp to >= -127; floor (v_floor_f32 here; the section's
// add-and-subtract of 2^23 + 2^22 in round-down mode computes the same function); fractional
// part; polynomial with p0 = 1 by Horner's rule with FMAs; integer part shifted into the exponent
// field and added to the polynomial's bits.  Coefficients: minimax relative error on [0, 1),
// from gen_exp2_coeffs.py (Remez exchange); the section prints none.
#pragma once
#include <hip/hip_runtime.h>

namespace attn {

template <int DEG> struct Exp2Poly;
template <> struct Exp2Poly<3> { static constexpr float p[3] = {6.951167583e-01f, 2.276449949e-01f, 7.706703991e-02f}; };
template <> struct Exp2Poly<4> { static constexpr float p[4] = {6.930448413e-01f, 2.412801981e-01f, 5.224247277e-02f, 1.342668384e-02f}; };
template <> struct Exp2Poly<5> { static constexpr float p[5] = {6.931512952e-01f, 2.401644439e-01f, 5.579991266e-02f, 9.017030708e-03f, 1.867130050e-03f}; };

template <int DEG>
__device__ __forceinline__ float exp2_emulated(float x)
{
    x = fmaxf(x, -127.0f);
    const float fl = __builtin_floorf(x);
    const float f = x - fl;
    float acc = Exp2Poly<DEG>::p[DEG - 1];
#pragma unroll
    for (int i = DEG - 2; i >= 0; --i) acc = __builtin_fmaf(acc, f, Exp2Poly<DEG>::p[i]);
    acc = __builtin_fmaf(acc, f, 1.0f);
    return __int_as_float(__float_as_int(acc) + ((int)fl << 23));
}

}  // namespace attn
