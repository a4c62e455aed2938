// The counter-based draw of eps shared by the libhot translation units (gfx950 only).
#ifndef HOT_DRAW_H
#define HOT_DRAW_H

#include "hot.h"
#include "vec.h"

namespace {

typedef unsigned int u4 __attribute__((ext_vector_type(4)));

// ---------------------------------------------------------------------------------
// Counter-based draw of eps ~ N(0, I) (Algorithm 2, sampling line; every GPU has to draw
// samples no other GPU draws).  The paper names no generator; this one is fixed here:
//   integer stage  Philox-4x32 with 10 rounds (Salmon, Moraes, Dror, Shaw, SC'11):
//                  key = the two halves of the seed, counter = (q lo, q hi, t, step) with
//                  q = i div 4 the quad of weight i and t the global sample index; the four
//                  output words belong to weights 4q .. 4q+3;
//   float stage    Box-Muller on the word pairs (x0,x1) and (x2,x3):
//                  u = ((xa >> 8) + 1) 2^-24 in (0,1], f = (xb >> 8) 2^-24 in [0,1) turns,
//                  r = sqrt(-2 ln u), outputs r cos(2 pi f), r sin(2 pi f).
// u and f are exact in fp32.  log2, sqrt, sin and cos are the hardware's transcendental
// instructions (sin and cos take their argument in turns, so no range reduction is
// needed); each operation is rounded on its own (no contraction), so the forward and the
// backward kernel regenerate bit-identical values.
// ---------------------------------------------------------------------------------
struct Rng {
    unsigned k0, k1;        // key
    unsigned first_sample;  // global index of local sample 0
    unsigned step;
};

__device__ __forceinline__ u4 philox4x32_10(unsigned c0, unsigned c1, unsigned c2, unsigned c3,
                                            unsigned k0, unsigned k1)
{
    constexpr unsigned kM0 = 0xD2511F53u, kM1 = 0xCD9E8D57u, kW0 = 0x9E3779B9u, kW1 = 0xBB67AE85u;
#pragma unroll
    for (int r = 0; r < 10; ++r) {
        const unsigned long long p0 = (unsigned long long)kM0 * c0;
        const unsigned long long p1 = (unsigned long long)kM1 * c2;
        const unsigned n0 = (unsigned)(p1 >> 32) ^ c1 ^ k0;
        const unsigned n2 = (unsigned)(p0 >> 32) ^ c3 ^ k1;
        c1 = (unsigned)p1;
        c3 = (unsigned)p0;
        c0 = n0;
        c2 = n2;
        k0 += kW0;
        k1 += kW1;
    }
    u4 x;
    x[0] = c0;
    x[1] = c1;
    x[2] = c2;
    x[3] = c3;
    return x;
}

__device__ __forceinline__ u4 eps_words(long quad, int s, const Rng &rng)
{
    return philox4x32_10((unsigned)((unsigned long long)quad & 0xFFFFFFFFull),
                         (unsigned)((unsigned long long)quad >> 32), rng.first_sample + (unsigned)s, rng.step,
                         rng.k0, rng.k1);
}

__device__ __forceinline__ f4 eps_from_words(u4 x)
{
#pragma clang fp contract(off)
    f4 e;
#pragma unroll
    for (int p = 0; p < 2; ++p) {
        const float u = (float)((x[2 * p] >> 8) + 1u) * 0x1p-24f;
        const float f = (float)(x[2 * p + 1] >> 8) * 0x1p-24f;
        // -2 ln u = (-2 ln 2) log2 u
        const float r = __builtin_amdgcn_sqrtf(-1.3862943611198906f * __builtin_amdgcn_logf(u));
        e[2 * p] = r * __builtin_amdgcn_cosf(f);
        e[2 * p + 1] = r * __builtin_amdgcn_sinf(f);
    }
    return e;
}

__device__ __forceinline__ f4 eps_quad(long quad, int s, const Rng &rng)
{
    return eps_from_words(eps_words(quad, s, rng));
}

// Host side: the generator state of a call from its public description; false if the global
// sample indices first_sample .. first_sample + s_local - 1 do not fit in 32 bits.
inline bool make_rng(const hot_rng *r, int s_local, Rng &out)
{
    if (!r) return false;
    if ((unsigned long long)r->first_sample + (unsigned long long)s_local > 0x100000000ull) return false;
    out.k0 = (unsigned)(r->seed & 0xFFFFFFFFull);
    out.k1 = (unsigned)(r->seed >> 32);
    out.first_sample = r->first_sample;
    out.step = r->step;
    return true;
}

}  // namespace

#endif  // HOT_DRAW_H
