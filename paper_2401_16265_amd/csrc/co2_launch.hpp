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
  DeltaPtrs d;              // K worker pseudo-gradients (fp32, or bf16 bits if bf16)
  void* dout;               // delta_out (nullable with x), same element type as d
  bool bf16;                // pseudo-gradient buffers hold bf16 bit patterns
  const float* inv;         // 1/Lambda per segment
  const int64_t* off_dev;   // segment table on the device
  int S;
  int64_t n;
  float alpha, beta, phi, rK;
  SlotRec* slots;           // per-slot sums of Clip(m',phi)^2 and delta_out^2 for the next
                            // round's gap, and the count of |m'| > phi
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
  SlotRec* slots;           // per-slot sums of (p' - p_in)^2 in column 0, nullable
};

// Resident wavefronts per compute unit each streaming kernel is capped to
// (0 = no cap).  Defaults come from bandwidth sweeps on MI355X; the environment
// variables CO2_SWEEP_WAVES, CO2_NORM_WAVES, CO2_ADAM_WAVES and CO2_COPY_WAVES
// override them (read at every launch) for tuning runs.
struct Tuning {
  int sweep_waves_per_cu[CO2_MAX_K + 1];
  int norm_waves_per_cu[3];     // by number of buffers read (1 or 2)
  int adam_waves_per_cu[2];     // [1]: the step that also reads the anchor and writes delta_out
  int copy_waves_per_cu;
};
const Tuning& tuning();
// Records `e` as this thread's most recent HIP error (what co2_last_hip_error() returns).
void note_hip_error(hipError_t e);
// Dynamic LDS bytes to request per single-wavefront workgroup so that at most
// `waves_per_cu` of them fit on a compute unit.
unsigned throttle_lds_bytes(int waves_per_cu);

// b1 (optional second buffer) may hold bf16 bit patterns (b1_bf16).
hipError_t launch_sqnorm_partials(int nb, const float* b0, float phi0, const void* b1,
                                  float phi1, bool b1_bf16, const int64_t* off_dev, int S,
                                  int64_t n, SlotRec* slots, hipStream_t st);
// Sums column `col` (and col+1 if two) of each segment's slot records into
// out_a (and out_b), `split` sub-sums per segment.
hipError_t launch_slot_sums(const SlotRec* slots, int col, bool two, const int64_t* off_dev,
                            int S, int64_t tile_elems, int split, double* out_a, double* out_b,
                            hipStream_t st);
hipError_t launch_totals_finish(const double* sub, int S, int split, double* out, hipStream_t st);
hipError_t launch_counts_finish(const double* sub, int S, int split, int64_t* out, hipStream_t st);
hipError_t launch_lambda_finish(const double* sub_m, const double* sub_d, int S, int split,
                                const float* first_step_norm, float c, float alpha, int tau,
                                double* seg_sq, float* inv, float* lambda_out, hipStream_t st);
hipError_t launch_sqrt_to_f32(const double* sq_in, float* out, int S, hipStream_t st);
hipError_t launch_fused_sweep(int K, bool has_x, const SweepArgs& g, hipStream_t st);   // g.bf16 selects the variant
hipError_t launch_first_round(bool has_x, const SweepArgs& g, hipStream_t st);
hipError_t launch_copy_f32(const float* src, float* dst, int64_t n, hipStream_t st);
hipError_t launch_adamw(const AdamArgs& g, hipStream_t st);

}  // namespace co2
