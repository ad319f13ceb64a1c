// Host-side launch interface between the C ABI (co2_api.hip) and the kernels.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "co2_device.hpp"

namespace co2 {

struct SweepArgs {
  float* x;                 // params (nullable: split form)
  const float* a_in;        // anchor
  float* a_out;             // next anchor (may equal a_in)
  float* m;                 // momentum
  DeltaPtrs d;              // K worker pseudo-gradients
  float* dout;              // delta_out (nullable with x)
  const float* inv;         // 1/Lambda per segment
  const int64_t* off_dev;   // segment table on the device
  int S;
  int64_t n;
  float alpha, beta, phi, rK;
  double* part_m;           // per-slot sums of Clip(m',phi)^2 for the next round
  double* part_d;           // per-slot sums of delta_out^2 for the next round
};

struct AdamArgs {
  int64_t n;
  const float* p_in;
  float* p_out;
  const uint16_t* grad;
  float* exp_avg;
  float* exp_avg_sq;
  float beta1, beta2, omb1, omb2, decay, step_size, sqrt_bc2, eps;
  const float* anchor;      // nullable
  float* dout;              // nullable
  const int64_t* off_dev;   // nullable (with part)
  int S;
  double* part;             // per-slot sums of (p' - p_in)^2, nullable
};

hipError_t launch_sqnorm_partials(int nb, const float* b0, float phi0, const float* b1,
                                  float phi1, const int64_t* off_dev, int S, int64_t n,
                                  double* part0, double* part1, hipStream_t st);
hipError_t launch_segment_totals(const double* part, const int64_t* off_dev, int S,
                                 int64_t tile_elems, double* out, hipStream_t st);
hipError_t launch_lambda_stage2(const double* part_m, const double* part_d,
                                const int64_t* off_dev, int S, int64_t tile_elems,
                                const float* first_step_norm, float c, float alpha, int tau,
                                double* seg_sq, float* inv, float* lambda_out, hipStream_t st);
hipError_t launch_sqrt_to_f32(const double* sq_in, float* out, int S, hipStream_t st);
hipError_t launch_fused_sweep(int K, bool has_x, const SweepArgs& g, hipStream_t st);
hipError_t launch_first_round(bool has_x, const SweepArgs& g, hipStream_t st);
hipError_t launch_copy_f32(const float* src, float* dst, int64_t n, hipStream_t st);
hipError_t launch_adamw(const AdamArgs& g, hipStream_t st);

}  // namespace co2
