// Wave-level device helpers shared by the kernels of libppv_hip.so (gfx950, wave64).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

constexpr int WAVE = 64;

// wave-level helpers on DPP (data-parallel primitives: a lane reads a neighbour's register inside
// the VALU instruction, no LDS round trip).  Reductions return a wave-uniform value.
constexpr int DPP_QUAD_XOR1 = 0xB1;     // quad_perm [1,0,3,2]
constexpr int DPP_QUAD_XOR2 = 0x4E;     // quad_perm [2,3,0,1]
constexpr int DPP_ROW_SHR1 = 0x111, DPP_ROW_SHR2 = 0x112, DPP_ROW_SHR3 = 0x113, DPP_ROW_SHR4 = 0x114,
              DPP_ROW_SHR8 = 0x118;
constexpr int DPP_ROW_MIRROR = 0x140, DPP_ROW_HALF_MIRROR = 0x141, DPP_ROW_BCAST15 = 0x142, DPP_ROW_BCAST31 = 0x143;

// source lane's value, or 0 where the lane has no source or is masked off
template <int CTRL, int ROW_MASK = 0xF, int BANK_MASK = 0xF> __device__ inline int dpp0(int x) {
    return __builtin_amdgcn_update_dpp(0, x, CTRL, ROW_MASK, BANK_MASK, true);
}
template <int CTRL, int ROW_MASK = 0xF, int BANK_MASK = 0xF> __device__ inline uint32_t dpp0(uint32_t x) {
    return (uint32_t)dpp0<CTRL, ROW_MASK, BANK_MASK>((int)x);
}
template <int CTRL, int ROW_MASK = 0xF, int BANK_MASK = 0xF> __device__ inline float dpp0(float x) {
    return __int_as_float(dpp0<CTRL, ROW_MASK, BANK_MASK>(__float_as_int(x)));
}
template <int CTRL, int ROW_MASK = 0xF, int BANK_MASK = 0xF> __device__ inline double dpp0(double x) {
    return __hiloint2double(dpp0<CTRL, ROW_MASK, BANK_MASK>(__double2hiint(x)),
                            dpp0<CTRL, ROW_MASK, BANK_MASK>(__double2loint(x)));
}
// source lane's value, or the lane's own value where it has no source or is masked off
template <int CTRL, int ROW_MASK = 0xF, int BANK_MASK = 0xF> __device__ inline float dpp_self(float x) {
    return __int_as_float(
        __builtin_amdgcn_update_dpp(__float_as_int(x), __float_as_int(x), CTRL, ROW_MASK, BANK_MASK, false));
}
__device__ inline float last_lane(float x) { return __int_as_float(__builtin_amdgcn_readlane(__float_as_int(x), 63)); }
__device__ inline int last_lane(int x) { return __builtin_amdgcn_readlane(x, 63); }
__device__ inline uint32_t last_lane(uint32_t x) { return (uint32_t)__builtin_amdgcn_readlane((int)x, 63); }
__device__ inline double last_lane(double x) {
    return __hiloint2double(__builtin_amdgcn_readlane(__double2hiint(x), 63),
                            __builtin_amdgcn_readlane(__double2loint(x), 63));
}

// value held by lane l (l must be wave-uniform)
__device__ inline int lane_value(int x, int l) { return __builtin_amdgcn_readlane(x, l); }
__device__ inline uint32_t lane_value(uint32_t x, int l) { return (uint32_t)__builtin_amdgcn_readlane((int)x, l); }
__device__ inline double lane_value(double x, int l) {
    return __hiloint2double(__builtin_amdgcn_readlane(__double2hiint(x), l),
                            __builtin_amdgcn_readlane(__double2loint(x), l));
}

__device__ inline float wave_max(float x) {
    x = fmaxf(x, dpp_self<DPP_QUAD_XOR1>(x));
    x = fmaxf(x, dpp_self<DPP_QUAD_XOR2>(x));
    x = fmaxf(x, dpp_self<DPP_ROW_HALF_MIRROR>(x));
    x = fmaxf(x, dpp_self<DPP_ROW_MIRROR>(x));           // every lane: maximum of its row of 16
    x = fmaxf(x, dpp_self<DPP_ROW_BCAST15, 0xA>(x));     // rows 1, 3 take in rows 0, 2
    x = fmaxf(x, dpp_self<DPP_ROW_BCAST31, 0xC>(x));     // rows 2, 3 take in lane 31
    return last_lane(x);
}
template <int CTRL, int ROW_MASK = 0xF, int BANK_MASK = 0xF> __device__ inline uint32_t dpp_self(uint32_t x) {
    return (uint32_t)__builtin_amdgcn_update_dpp((int)x, (int)x, CTRL, ROW_MASK, BANK_MASK, false);
}
__device__ inline uint32_t wave_max(uint32_t x) {
    x = max(x, dpp_self<DPP_QUAD_XOR1>(x));
    x = max(x, dpp_self<DPP_QUAD_XOR2>(x));
    x = max(x, dpp_self<DPP_ROW_HALF_MIRROR>(x));
    x = max(x, dpp_self<DPP_ROW_MIRROR>(x));
    x = max(x, dpp_self<DPP_ROW_BCAST15, 0xA>(x));
    x = max(x, dpp_self<DPP_ROW_BCAST31, 0xC>(x));
    return last_lane(x);
}
template <typename V> __device__ inline V wave_sum(V x) {
    x += dpp0<DPP_QUAD_XOR1>(x);
    x += dpp0<DPP_QUAD_XOR2>(x);
    x += dpp0<DPP_ROW_HALF_MIRROR>(x);
    x += dpp0<DPP_ROW_MIRROR>(x);
    x += dpp0<DPP_ROW_BCAST15, 0xA>(x);
    x += dpp0<DPP_ROW_BCAST31, 0xC>(x);
    return last_lane(x);
}
// inclusive prefix sum over the 64 lanes (lane order)
template <typename V> __device__ inline V wave_incl_scan(V x) {
    V t = x;
    t += dpp0<DPP_ROW_SHR1>(x);
    t += dpp0<DPP_ROW_SHR2>(x);
    t += dpp0<DPP_ROW_SHR3>(x);                          // up to 4 consecutive lanes of the row
    t += dpp0<DPP_ROW_SHR4, 0xF, 0xE>(t);
    t += dpp0<DPP_ROW_SHR8, 0xF, 0xC>(t);                // prefix inside each row of 16
    t += dpp0<DPP_ROW_BCAST15, 0xA>(t);
    t += dpp0<DPP_ROW_BCAST31, 0xC>(t);
    return t;
}
