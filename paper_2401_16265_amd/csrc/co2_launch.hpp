// Host-side launch interface between the C ABI (co2_api.hip) and the kernels.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "co2_device.hpp"

namespace co2 {

// Run-time switches of the sweep (wavefront-uniform; see co2_sweep.hip).
struct SweepMode {
  bool own_current;         // the worker's own current pseudo-gradient leads the mean
  bool pull;                // params = x - rho*(x - x') instead of x'
  bool defer_iterate;       // norm-rescale clip: x' is written by apply_iterate afterwards
  float rho;
};

struct SweepArgs {
  float* x;                 // params (nullable: split form)
  const float* a_in;        // anchor
  float* a_out;             // next anchor (may equal a_in)
  float* m;                 // momentum
  DeltaPtrs d;              // the pseudo-gradient buffers read (element type `dtype`)
  void* dout;               // delta_out (nullable with x), same element type as d
  int dtype;                // DeltaType of d and dout
  SweepMode mode;
  int waves_per_cu;         // resident-wavefront cap for the sweep; 0 = the library's default
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

// Resident wavefronts per compute unit each streaming kernel is capped to.
// Measured optima on MI355X at 1.3B parameters, averaged over several buffer
// placements: about 56-64 KB of loads in flight per compute unit.  A sweep
// wavefront holds 1 KB per stream read (3 + buffers), a norm-pass wavefront (which stays for 16 pieces) 4 KB
// per buffer, an AdamW wavefront 3.5 KB (4.5 KB with the anchor).
// `delta_kb`: KB of pseudo-gradient loads one sweep wavefront issues (1 per fp32 buffer, 0.5 per
// 16-bit buffer), beside its 3 KB of anchor, momentum and params.
inline int default_sweep_waves(float delta_kb) {
  if (delta_kb <= 0.5f) return 12;                 // K = 1 with 16-bit transport
  if (delta_kb <= 1.0f) return 10;                 // K = 1, or K = 2 with 16-bit transport
  return delta_kb <= 4.0f ? 8 : delta_kb <= 9.0f ? 7 : 6;   // 11 and more: two load phases, see co2_sweep.hip
}
constexpr int kNormWavesOneBuffer = 5;
constexpr int kNormWavesTwoBuffers = 5;
constexpr int kAdamWavesPerCu = 16;
constexpr int kAdamWavesWithAnchor = 12;  // the step that also reads the anchor and writes delta_out
constexpr int kAdamWavesNoStore = 10;     // ... and does not store the parameters
constexpr int kCopyWavesPerCu = 7;
constexpr int kApplyWavesPerCu = 16;      // deferred outer iterate: 2-3 KB of loads per wavefront
// Records `e` as this thread's most recent HIP error (what co2_last_hip_error() returns).
void note_hip_error(hipError_t e);
// Dynamic LDS bytes to request per single-wavefront workgroup so that at most
// `waves_per_cu` of them fit on a compute unit.
unsigned throttle_lds_bytes(int waves_per_cu);

// b1 (optional second buffer) has element type b1_dtype (a DeltaType).
hipError_t launch_sqnorm_partials(int nb, const float* b0, float phi0, const void* b1,
                                  float phi1, int b1_dtype, const int64_t* off_dev, int S,
                                  int64_t n, SlotRec* slots, hipStream_t st);
// Sums column `col` (and col+1 if two) of each segment's slot records into
// out_a (and out_b), `split` sub-sums per segment.
hipError_t launch_slot_sums(const SlotRec* slots, int col, bool two, const int64_t* off_dev,
                            int S, int64_t tile_elems, int split, double* out_a, double* out_b,
                            hipStream_t st);
hipError_t launch_totals_finish(const double* sub, int S, int split, double* out, hipStream_t st);
hipError_t launch_counts_finish(const double* sub, int S, int split, int64_t* out, hipStream_t st);
// `use_d`: the denominator is sqrt of the sums in sub_d (else tau*first_step_norm, or
// none at all: Lambda = 1).  `numer_cap`: upper bound of the numerator's norm (+inf: none).
hipError_t launch_lambda_finish(const double* sub_m, const double* sub_d, bool use_d, int S, int split,
                                const float* first_step_norm, float c, float alpha, int tau,
                                double numer_cap, double* seg_sq, float* inv, float* lambda_out,
                                hipStream_t st);
// Stage 2 in ONE launch for tables whose segments are short: each workgroup adds
// its segment's slots and evaluates Lambda itself.
hipError_t launch_lambda_direct(const SlotRec* slots, const int64_t* off_dev, int S, int64_t tile_elems,
                                bool use_d, const float* first_step_norm, float c, float alpha, int tau,
                                double numer_cap, double* seg_sq, float* inv, float* lambda_out,
                                hipStream_t st);
// scale[s] = min(1, phi/sqrt(sum)) from the per-segment sub-sums of m'^2.
hipError_t launch_scale_finish(const double* sub, int S, int split, float phi, float* scale, hipStream_t st);
hipError_t launch_sqrt_to_f32(const double* sq_in, float* out, int S, hipStream_t st);
hipError_t launch_fused_sweep(int nbuf, bool has_x, const SweepArgs& g, hipStream_t st);  // nbuf buffers in g.d
hipError_t launch_apply_iterate(bool has_x, const SweepArgs& g, const float* scale, hipStream_t st);
hipError_t launch_first_round(bool has_x, const SweepArgs& g, hipStream_t st);
hipError_t launch_copy_f32(const float* src, float* dst, int64_t n, hipStream_t st);
hipError_t launch_adamw(const AdamArgs& g, hipStream_t st);

}  // namespace co2
