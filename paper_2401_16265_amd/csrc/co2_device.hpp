// Device-side helpers shared by the gfx950 kernels of libco2: launch geometry,
// wavefront (64-lane) reductions through DPP, segment lookup.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "co2.h"

#ifndef CO2_SWEEP_U
#define CO2_SWEEP_U 2          // 16-byte vectors per lane and stream in the fused sweep
#endif
#ifndef CO2_NT
#define CO2_NT 0               // 1: non-temporal loads/stores on the streaming buffers
#endif

namespace co2 {

constexpr int kBlock = 256;                       // 4 wavefronts
constexpr int kWave = 64;
constexpr int kWavesPerBlock = kBlock / kWave;
constexpr int64_t kNormTile = 8192;               // elements per workgroup, norm pass
constexpr int64_t kSweepTile = int64_t(kBlock) * 4 * CO2_SWEEP_U;   // fused sweep
constexpr int64_t kAdamTile = int64_t(kBlock) * 4 * 2;              // AdamW step

struct DeltaPtrs {
  const float* p[CO2_MAX_K];
};

// Section 3.3: Clip(chi, phi) = max{-phi, min{chi, phi}}.
__device__ __forceinline__ float clip_coord(float chi, float phi) {
  return fmaxf(-phi, fminf(chi, phi));
}

// Index s of the segment that holds flat index j, 0 <= j < off[S]:
// off[s] <= j < off[s+1].  Empty segments are skipped.
__device__ __forceinline__ int seg_of(const int64_t* __restrict__ off, int S, int64_t j) {
  int lo = 0, hi = S;                              // off[lo] <= j < off[hi]
  while (hi - lo > 1) {
    const int mid = (lo + hi) >> 1;
    if (off[mid] <= j) lo = mid; else hi = mid;
  }
  return lo;
}

// One DPP lane exchange of a double (two 32-bit halves).  Needs all 64 lanes
// of the wavefront active.
template <int CTRL>
__device__ __forceinline__ double dpp_move(double v) {
  int lo = __double2loint(v), hi = __double2hiint(v);
  lo = __builtin_amdgcn_update_dpp(0, lo, CTRL, 0xF, 0xF, false);
  hi = __builtin_amdgcn_update_dpp(0, hi, CTRL, 0xF, 0xF, false);
  return __hiloint2double(hi, lo);
}

__device__ __forceinline__ double read_lane(double v, int lane) {
  const int lo = __builtin_amdgcn_readlane(__double2loint(v), lane);
  const int hi = __builtin_amdgcn_readlane(__double2hiint(v), lane);
  return __hiloint2double(hi, lo);
}

// Sum over the 64 lanes of a wavefront, identical in every lane and for every
// run: a butterfly inside each row of 16 lanes (quad_perm [1,0,3,2], quad_perm
// [2,3,0,1], row_half_mirror, row_mirror), then the four row sums added in
// row order.
__device__ __forceinline__ double wave_sum(double v) {
  v += dpp_move<0xB1>(v);
  v += dpp_move<0x4E>(v);
  v += dpp_move<0x141>(v);
  v += dpp_move<0x140>(v);
  const double r0 = read_lane(v, 0), r1 = read_lane(v, 16);
  const double r2 = read_lane(v, 32), r3 = read_lane(v, 48);
  return ((r0 + r1) + r2) + r3;
}

// Sum over the workgroup; every thread must call it.  Result valid in all
// threads.  `lds` holds kWavesPerBlock doubles per concurrent reduction.
__device__ __forceinline__ double block_sum(double v, double* lds) {
  const double w = wave_sum(v);
  const int wave = threadIdx.x / kWave;
  __syncthreads();                                 // previous use of lds is over
  if ((threadIdx.x & (kWave - 1)) == 0) lds[wave] = w;
  __syncthreads();
  double t = lds[0];
#pragma unroll
  for (int i = 1; i < kWavesPerBlock; ++i) t += lds[i];
  return t;
}

__device__ __forceinline__ float4 ld4(const float* p) {
#if CO2_NT
  return __builtin_nontemporal_load(reinterpret_cast<const float4*>(p));
#else
  return *reinterpret_cast<const float4*>(p);
#endif
}
__device__ __forceinline__ void st4(float* p, float4 v) {
#if CO2_NT
  __builtin_nontemporal_store(v, reinterpret_cast<float4*>(p));
#else
  *reinterpret_cast<float4*>(p) = v;
#endif
}

__device__ __forceinline__ double sq(float v) {
  const double d = static_cast<double>(v);
  return d * d;                                    // exact: 24-bit x 24-bit
}

}  // namespace co2
