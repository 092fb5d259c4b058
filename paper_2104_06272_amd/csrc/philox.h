// Counter-based random numbers for the actor: Philox4x32 with 10 rounds
// (Salmon et al., SC'11).  The paper (section 3.1) asks for self-contained,
// deterministic experiments; a counter keyed by (env, global step, purpose)
// makes every draw independent of grid shape, batch size and call order.
#pragma once
#include <stdint.h>
#include <hip/hip_runtime.h>

#define ANK_HD __host__ __device__ __forceinline__

namespace ank {

// what a draw is used for (fourth counter word)
enum : uint32_t { DOM_ACTION = 0, DOM_RESET = 1, DOM_INIT = 2, DOM_PARAM = 3, DOM_MAZE = 4 };

struct u32x4 { uint32_t x, y, z, w; };

ANK_HD uint32_t mulhi32(uint32_t a, uint32_t b)
{
#if defined(__HIP_DEVICE_COMPILE__)
    return __umulhi(a, b);
#else
    return (uint32_t)(((uint64_t)a * b) >> 32);
#endif
}

// counter = (index, t_low, t_high, domain), key = seed
ANK_HD u32x4 philox(uint64_t seed, uint32_t index, uint64_t t, uint32_t domain)
{
    uint32_t c0 = index, c1 = (uint32_t)t, c2 = (uint32_t)(t >> 32), c3 = domain;
    uint32_t k0 = (uint32_t)seed, k1 = (uint32_t)(seed >> 32);
#pragma unroll
    for (int r = 0; r < 10; ++r) {
        const uint32_t hi0 = mulhi32(0xD2511F53u, c0), lo0 = 0xD2511F53u * c0;
        const uint32_t hi1 = mulhi32(0xCD9E8D57u, c2), lo1 = 0xCD9E8D57u * c2;
        c0 = hi1 ^ c1 ^ k0;
        c1 = lo1;
        c2 = hi0 ^ c3 ^ k1;
        c3 = lo0;
        k0 += 0x9E3779B9u;
        k1 += 0xBB67AE85u;
    }
    return u32x4{c0, c1, c2, c3};
}

// 24-bit uniforms: [0,1) and (0,1]
ANK_HD float u01(uint32_t x) { return (float)(x >> 8) * 0x1p-24f; }
ANK_HD float u01_plus(uint32_t x) { return (float)((x >> 8) + 1u) * 0x1p-24f; }
// integer in [0,n) by multiply-shift
ANK_HD uint32_t bounded(uint32_t x, uint32_t n) { return mulhi32(x, n); }

}  // namespace ank
