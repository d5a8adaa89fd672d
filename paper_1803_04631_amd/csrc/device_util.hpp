// Device helpers for gfx950: counter-based uniforms and wave64 cross-lane primitives.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace mlda {

constexpr int kWave = 64;

// ---------------------------------------------------------------- Philox4x32-10
// Salmon et al., SC'11: each round multiplies two counter words by fixed odd
// constants, xors the high halves with the remaining words and the round key, and the
// key advances by two Weyl constants.  Only the first two output words are used.
__device__ __forceinline__ void philox4x32_10(uint32_t c0, uint32_t c1, uint32_t c2, uint32_t c3,
                                              uint32_t k0, uint32_t k1,
                                              uint32_t& r0, uint32_t& r1) {
#pragma unroll
    for (int r = 0; r < 10; ++r) {
        const uint32_t hi0 = __umulhi(0xD2511F53u, c0), lo0 = 0xD2511F53u * c0;
        const uint32_t hi1 = __umulhi(0xCD9E8D57u, c2), lo1 = 0xCD9E8D57u * c2;
        c0 = hi1 ^ c1 ^ k0;
        c1 = lo1;
        c2 = hi0 ^ c3 ^ k1;
        c3 = lo0;
        k0 += 0x9E3779B9u;
        k1 += 0xBB67AE85u;
    }
    r0 = c0;
    r1 = c1;
}

// u in [0,1): top 53 bits of (r0:r1); counter (token lo, token hi, iteration, 0).
__device__ __forceinline__ double token_uniform(uint64_t seed, uint32_t iter, uint64_t token) {
    uint32_t r0, r1;
    philox4x32_10((uint32_t)token, (uint32_t)(token >> 32), iter, 0u,
                  (uint32_t)seed, (uint32_t)(seed >> 32), r0, r1);
    const uint64_t bits = (((uint64_t)r0 << 32) | (uint64_t)r1) >> 11;
    return (double)bits * (1.0 / 9007199254740992.0);
}

// ---------------------------------------------------------------- cross-lane
__device__ __forceinline__ int lane_id() { return (int)(threadIdx.x & (kWave - 1)); }

// Value of lane `src` (wave-uniform index) as a wave-uniform value.
__device__ __forceinline__ int read_lane(int v, int src) { return __builtin_amdgcn_readlane(v, src); }
__device__ __forceinline__ float read_lane(float v, int src) {
    return __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), src));
}
__device__ __forceinline__ double read_lane(double v, int src) {
    const int lo = __builtin_amdgcn_readlane(__double2loint(v), src);
    const int hi = __builtin_amdgcn_readlane(__double2hiint(v), src);
    return __hiloint2double(hi, lo);
}

// One DPP move of a double; lanes without a source (or outside the row mask) get 0.0.
template <int kCtrl, int kRowMask>
__device__ __forceinline__ double dpp_move0(double v) {
    const int lo = __builtin_amdgcn_update_dpp(0, __double2loint(v), kCtrl, kRowMask, 0xf, false);
    const int hi = __builtin_amdgcn_update_dpp(0, __double2hiint(v), kCtrl, kRowMask, 0xf, false);
    return __hiloint2double(hi, lo);
}

// Inclusive prefix sum over the 64 lanes of a wave.  Every lane must be active.
// Four shifts inside each row of 16 lanes, then lane 15 of rows 0/2 is added to rows
// 1/3 and lane 31 to rows 2 and 3.
__device__ __forceinline__ double wave_inclusive_sum(double v) {
    v += dpp_move0<0x111, 0xf>(v);   // row_shr:1
    v += dpp_move0<0x112, 0xf>(v);   // row_shr:2
    v += dpp_move0<0x114, 0xf>(v);   // row_shr:4
    v += dpp_move0<0x118, 0xf>(v);   // row_shr:8
    v += dpp_move0<0x142, 0xa>(v);   // row_bcast:15 into rows 1 and 3
    v += dpp_move0<0x143, 0xc>(v);   // row_bcast:31 into rows 2 and 3
    return v;
}

__device__ __forceinline__ int wave_inclusive_sum(int v) {
    v += __builtin_amdgcn_update_dpp(0, v, 0x111, 0xf, 0xf, false);
    v += __builtin_amdgcn_update_dpp(0, v, 0x112, 0xf, 0xf, false);
    v += __builtin_amdgcn_update_dpp(0, v, 0x114, 0xf, 0xf, false);
    v += __builtin_amdgcn_update_dpp(0, v, 0x118, 0xf, 0xf, false);
    v += __builtin_amdgcn_update_dpp(0, v, 0x142, 0xa, 0xf, false);
    v += __builtin_amdgcn_update_dpp(0, v, 0x143, 0xc, 0xf, false);
    return v;
}

__device__ __forceinline__ int wave_sum(int v) {
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off, kWave);
    return v;
}

__device__ __forceinline__ double wave_sum(double v) {
    return read_lane(wave_inclusive_sum(v), kWave - 1);
}

__device__ __forceinline__ uint64_t lanes_below() {   // mask of lanes with a smaller id
    return (1ull << lane_id()) - 1ull;
}

}  // namespace mlda
