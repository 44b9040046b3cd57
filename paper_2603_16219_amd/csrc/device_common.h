// Device-side helpers shared by the kernels of this library (gfx950, 64-lane wavefronts):
// cross-lane reductions and scans built on DPP, and the logit loads.  Included by each .hip
// file inside its own anonymous namespace; nothing here has external linkage.
#pragma once

#include <hip/hip_runtime.h>

#include <atomic>

#include <cstdint>

#include "specsteer.h"

namespace {

constexpr int kWave = 64;

// ------------------------------------------------------------------ wave primitives

// Cross-lane moves inside a row of 16 lanes use DPP; all four patterns below read a valid
// lane for every destination lane, so neither `old` nor bound_ctrl matters.
template <int CTRL>
__device__ __forceinline__ int dpp_mov(int v) {
    return __builtin_amdgcn_update_dpp(v, v, CTRL, 0xF, 0xF, false);
}
constexpr int kDppXor1 = 0xB1;        // quad_perm [1,0,3,2]
constexpr int kDppXor2 = 0x4E;        // quad_perm [2,3,0,1]
constexpr int kDppHalfMirror = 0x141; // lane i <-> 7-i inside each 8
constexpr int kDppMirror = 0x140;     // lane i <-> 15-i inside each 16

__device__ __forceinline__ int wave_max_i32(int v) {
    v = max(v, dpp_mov<kDppXor1>(v));
    v = max(v, dpp_mov<kDppXor2>(v));
    v = max(v, dpp_mov<kDppHalfMirror>(v));
    v = max(v, dpp_mov<kDppMirror>(v));
    // every lane of a 16-lane row now holds its row's maximum
    const int a = __builtin_amdgcn_readlane(v, 0), b = __builtin_amdgcn_readlane(v, 16);
    const int c = __builtin_amdgcn_readlane(v, 32), d = __builtin_amdgcn_readlane(v, 48);
    return max(max(a, b), max(c, d));
}

__device__ __forceinline__ int wave_sum_i32(int v) {
    v += dpp_mov<kDppXor1>(v);
    v += dpp_mov<kDppXor2>(v);
    v += dpp_mov<kDppHalfMirror>(v);
    v += dpp_mov<kDppMirror>(v);
    return __builtin_amdgcn_readlane(v, 0) + __builtin_amdgcn_readlane(v, 16) +
           __builtin_amdgcn_readlane(v, 32) + __builtin_amdgcn_readlane(v, 48);
}

__device__ __forceinline__ float wave_sum_f32(float x) {
    x += __int_as_float(dpp_mov<kDppXor1>(__float_as_int(x)));
    x += __int_as_float(dpp_mov<kDppXor2>(__float_as_int(x)));
    x += __int_as_float(dpp_mov<kDppHalfMirror>(__float_as_int(x)));
    x += __int_as_float(dpp_mov<kDppMirror>(__float_as_int(x)));
    const int v = __float_as_int(x);
    const float a = __int_as_float(__builtin_amdgcn_readlane(v, 0));
    const float b = __int_as_float(__builtin_amdgcn_readlane(v, 16));
    const float c = __int_as_float(__builtin_amdgcn_readlane(v, 32));
    const float d = __int_as_float(__builtin_amdgcn_readlane(v, 48));
    return (a + b) + (c + d);
}

// One DPP move of a double (both halves); lanes the pattern leaves without a source, or that
// row_mask disables, receive 0.0.
template <int CTRL, int ROW_MASK>
__device__ __forceinline__ double dpp_f64_or_zero(double x) {
    const long long b = __double_as_longlong(x);
    const int lo = __builtin_amdgcn_update_dpp(0, (int)(b & 0xFFFFFFFFll), CTRL, ROW_MASK, 0xF, false);
    const int hi = __builtin_amdgcn_update_dpp(0, (int)(b >> 32), CTRL, ROW_MASK, 0xF, false);
    return __longlong_as_double(((long long)hi << 32) | (unsigned int)lo);
}
constexpr int kDppRowShr1 = 0x111, kDppRowShr2 = 0x112, kDppRowShr4 = 0x114, kDppRowShr8 = 0x118;
constexpr int kDppRowBcast15 = 0x142;  // lane 15 of each row -> every lane of the next row
constexpr int kDppRowBcast31 = 0x143;  // lane 31 -> every lane of rows 2 and 3
constexpr int kDppWaveShr1 = 0x138;    // lane i-1 -> lane i across the whole wave

// Inclusive prefix sum over the 64 lanes: Hillis-Steele inside each row of 16, then the row totals.
__device__ __forceinline__ double wave_incl_scan_f64(double x) {
    x += dpp_f64_or_zero<kDppRowShr1, 0xF>(x);
    x += dpp_f64_or_zero<kDppRowShr2, 0xF>(x);
    x += dpp_f64_or_zero<kDppRowShr4, 0xF>(x);
    x += dpp_f64_or_zero<kDppRowShr8, 0xF>(x);
    x += dpp_f64_or_zero<kDppRowBcast15, 0xA>(x);  // rows 1 and 3 take in the row before them
    x += dpp_f64_or_zero<kDppRowBcast31, 0xC>(x);  // rows 2 and 3 take in the first half
    return x;
}

// Exclusive companion of an inclusive scan result (lane 0 gets 0) and the wave total.
__device__ __forceinline__ double wave_shift_up_f64(double incl) { return dpp_f64_or_zero<kDppWaveShr1, 0xF>(incl); }
__device__ __forceinline__ double wave_last_f64(double incl) {
    const long long b = __double_as_longlong(incl);
    const int lo = __builtin_amdgcn_readlane((int)(b & 0xFFFFFFFFll), 63);
    const int hi = __builtin_amdgcn_readlane((int)(b >> 32), 63);
    return __longlong_as_double(((long long)hi << 32) | (unsigned int)lo);
}

__device__ __forceinline__ int first_lane(unsigned long long mask) { return __ffsll((long long)mask) - 1; }

// ------------------------------------------------------------------ logit loads

template <int DT, int VEC> struct RawT;
template <> struct RawT<SS_BF16, 8> { using type = uint4; };
template <> struct RawT<SS_F32, 4> { using type = float4; };

// Logit rows are streamed once and never reused by the same kernel: non-temporal loads keep
// them from displacing each other in L2 / Infinity Cache and measure ~12 % faster than plain
// loads on a pure read of this size.
// The vector types only promise element alignment (2 bytes for bf16, 4 for fp32): gfx950 under ROCm runs
// with unaligned access enabled, so the same 16-byte load instruction serves rows that start anywhere
// (an odd vocabulary size with dense rows) at the cost of an extra cache line per wave-load.
typedef unsigned int u32x4 __attribute__((ext_vector_type(4), aligned(2)));
typedef float f32x4 __attribute__((ext_vector_type(4), aligned(4)));

template <int DT, int VEC>
__device__ __forceinline__ typename RawT<DT, VEC>::type ld_raw(const void* row, long vec);
template <>
__device__ __forceinline__ uint4 ld_raw<SS_BF16, 8>(const void* row, long vec) {
    const u32x4 t = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(row) + vec);
    return make_uint4(t.x, t.y, t.z, t.w);
}
template <>
__device__ __forceinline__ float4 ld_raw<SS_F32, 4>(const void* row, long vec) {
    const f32x4 t = __builtin_nontemporal_load(reinterpret_cast<const f32x4*>(row) + vec);
    return make_float4(t.x, t.y, t.z, t.w);
}

__device__ __forceinline__ float bf16_lo(unsigned w) { return __uint_as_float(w << 16); }
__device__ __forceinline__ float bf16_hi(unsigned w) { return __uint_as_float(w & 0xFFFF0000u); }

__device__ __forceinline__ void unpack(const uint4& r, float (&h)[8]) {
    h[0] = bf16_lo(r.x); h[1] = bf16_hi(r.x);
    h[2] = bf16_lo(r.y); h[3] = bf16_hi(r.y);
    h[4] = bf16_lo(r.z); h[5] = bf16_hi(r.z);
    h[6] = bf16_lo(r.w); h[7] = bf16_hi(r.w);
}
__device__ __forceinline__ void unpack(const float4& r, float (&h)[4]) {
    h[0] = r.x; h[1] = r.y; h[2] = r.z; h[3] = r.w;
}

template <int DT>
__device__ __forceinline__ float ld_elem(const void* row, long e) {
    if (DT == SS_BF16) return __uint_as_float((unsigned)reinterpret_cast<const unsigned short*>(row)[e] << 16);
    return reinterpret_cast<const float*>(row)[e];
}

template <int DT>
__device__ __forceinline__ const void* row_ptr(const void* base, long elem_off) {
    return reinterpret_cast<const char*>(base) + elem_off * (DT == SS_BF16 ? 2 : 4);
}

// ------------------------------------------------------------------ host helpers

// Compute units of the current device (MI355X: 256), looked up once per device; callers on
// several host threads may race to fill an entry, all with the same value.
inline int device_cu_count() {
    static std::atomic<int> cached[64];
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return 256;
    int n = cached[dev].load(std::memory_order_relaxed);
    if (n == 0) {
        if (hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n <= 0) n = 256;
        cached[dev].store(n, std::memory_order_relaxed);
    }
    return n;
}

}  // namespace
