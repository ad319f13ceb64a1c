// Segmented sums of squares for the two norms of the staleness gap
// (CO2 paper, Definition 3.1 / Eq. 3) and the per-segment scalar Lambda.
//
// Pass 1 (sqnorm_partials): the flat index space is cut into aligned tiles of
// kNormTile elements, one workgroup each.  A tile that lies inside one segment
// is read with 16-byte loads, squared and accumulated in fp64 per lane, reduced
// through DPP + LDS, and leaves ONE partial in slot (tile + segment).  A tile
// that holds a segment boundary (or the ragged end) gives each of its segments
// to one wavefront, which leaves one partial per (tile, segment) pair.  The
// slot index tile+segment is unique per pair because both indices only grow
// along the flat vector, so no atomics and no zero-fill are needed.
//
// Stage 2 (segment_totals / lambda_stage2): one workgroup per segment adds
// that segment's slots in a fixed order and, for the outer step, evaluates
// Lambda in fp64.  Everything is deterministic.
#include "co2_device.hpp"
#include "co2_launch.hpp"

namespace co2 {

template <int NB>
__global__ __launch_bounds__(kBlock) void sqnorm_partials(
    const float* __restrict__ b0, float phi0, const float* __restrict__ b1, float phi1,
    const int64_t* __restrict__ off, int S, int64_t n,
    double* __restrict__ part0, double* __restrict__ part1) {
  __shared__ double lds[2][kWavesPerBlock];
  const int64_t tile = blockIdx.x;
  const int64_t base = tile * kNormTile;
  const int64_t end = (base + kNormTile < n) ? base + kNormTile : n;
  const int s_lo = seg_of(off, S, base);

  if (end <= off[s_lo + 1]) {
    // Whole tile inside segment s_lo.
    double a0 = 0.0, a1 = 0.0;
    const int64_t nvec = (end - base) >> 2;                 // full 16-byte vectors
    for (int64_t v = threadIdx.x; v < nvec; v += kBlock) {
      const int64_t j = base + (v << 2);
      float4 q = ld4(b0 + j);
      if (phi0 > 0.0f) {
        q.x = clip_coord(q.x, phi0); q.y = clip_coord(q.y, phi0);
        q.z = clip_coord(q.z, phi0); q.w = clip_coord(q.w, phi0);
      }
      a0 += sq(q.x); a0 += sq(q.y); a0 += sq(q.z); a0 += sq(q.w);
      if (NB == 2) {
        float4 r = ld4(b1 + j);
        if (phi1 > 0.0f) {
          r.x = clip_coord(r.x, phi1); r.y = clip_coord(r.y, phi1);
          r.z = clip_coord(r.z, phi1); r.w = clip_coord(r.w, phi1);
        }
        a1 += sq(r.x); a1 += sq(r.y); a1 += sq(r.z); a1 += sq(r.w);
      }
    }
    for (int64_t j = base + (nvec << 2) + threadIdx.x; j < end; j += kBlock) {   // ragged end
      float q = b0[j];
      if (phi0 > 0.0f) q = clip_coord(q, phi0);
      a0 += sq(q);
      if (NB == 2) {
        float r = b1[j];
        if (phi1 > 0.0f) r = clip_coord(r, phi1);
        a1 += sq(r);
      }
    }
    const double t0 = block_sum(a0, lds[0]);
    double t1 = 0.0;
    if (NB == 2) t1 = block_sum(a1, lds[1]);
    if (threadIdx.x == 0) {
      part0[tile + s_lo] = t0;
      if (NB == 2) part1[tile + s_lo] = t1;
    }
    return;
  }

  // Boundary tile: wavefront w takes segments s_lo+w, s_lo+w+4, ...
  const int s_hi = seg_of(off, S, end - 1);
  const int wave = threadIdx.x / kWave, lane = threadIdx.x & (kWave - 1);
  for (int s = s_lo + wave; s <= s_hi; s += kWavesPerBlock) {
    const int64_t lo = off[s] > base ? off[s] : base;
    const int64_t hi = off[s + 1] < end ? off[s + 1] : end;
    if (lo >= hi) continue;                                  // empty segment: no slot is read
    double a0 = 0.0, a1 = 0.0;
    for (int64_t j = lo + lane; j < hi; j += kWave) {
      float q = b0[j];
      if (phi0 > 0.0f) q = clip_coord(q, phi0);
      a0 += sq(q);
      if (NB == 2) {
        float r = b1[j];
        if (phi1 > 0.0f) r = clip_coord(r, phi1);
        a1 += sq(r);
      }
    }
    const double t0 = wave_sum(a0);
    double t1 = 0.0;
    if (NB == 2) t1 = wave_sum(a1);
    if (lane == 0) {
      part0[tile + s] = t0;
      if (NB == 2) part1[tile + s] = t1;
    }
  }
}

// Sum of segment s's slots, in a fixed order; every thread of the block calls.
__device__ __forceinline__ double segment_total(const double* __restrict__ part, int s,
                                                int64_t lo, int64_t hi, int64_t tile_elems,
                                                double* lds) {
  double acc = 0.0;
  if (hi > lo) {
    const int64_t t0 = lo / tile_elems, t1 = (hi - 1) / tile_elems;
    for (int64_t t = t0 + threadIdx.x; t <= t1; t += kBlock) acc += part[t + s];
  }
  return block_sum(acc, lds);
}

__global__ __launch_bounds__(kBlock) void segment_totals(
    const double* __restrict__ part, const int64_t* __restrict__ off, int S,
    int64_t tile_elems, double* __restrict__ out) {
  __shared__ double lds[kWavesPerBlock];
  for (int s = blockIdx.x; s < S; s += gridDim.x) {
    const double t = segment_total(part, s, off[s], off[s + 1], tile_elems, lds);
    if (threadIdx.x == 0) out[s] = t;
  }
}

// Lambda_t per segment (Algorithm 1, gap update; Eq. 3), fp64:
//   numerator   alpha*sqrt(M2),  M2 = sum Clip(m_{t-1},phi)^2   (slots part_m)
//   denominator tau*first_step_norm[s], or sqrt(P2), P2 = sum d_0^2 (slots part_d)
//   Lambda = (c == 0 || T == 0) ? 1 : (c*alpha)*sqrt(M2)/T + 1;  inv = (float)(1/Lambda)
__global__ __launch_bounds__(kBlock) void lambda_stage2(
    const double* __restrict__ part_m, const double* __restrict__ part_d,
    const int64_t* __restrict__ off, int S, int64_t tile_elems,
    const float* __restrict__ first_step_norm, float c, float alpha, int tau,
    double* __restrict__ seg_sq, float* __restrict__ inv, float* __restrict__ lambda_out) {
  __shared__ double lds[2][kWavesPerBlock];
  for (int s = blockIdx.x; s < S; s += gridDim.x) {
    const int64_t lo = off[s], hi = off[s + 1];
    const double M2 = segment_total(part_m, s, lo, hi, tile_elems, lds[0]);
    double P2 = 0.0;
    if (first_step_norm == nullptr) P2 = segment_total(part_d, s, lo, hi, tile_elems, lds[1]);
    if (threadIdx.x == 0) {
      const double T = first_step_norm
                           ? static_cast<double>(tau) * static_cast<double>(first_step_norm[s])
                           : sqrt(P2);
      double Lam = 1.0;
      if (c != 0.0f && T != 0.0) {
        Lam = (static_cast<double>(c) * static_cast<double>(alpha)) * sqrt(M2) / T + 1.0;
      }
      seg_sq[s] = M2;
      seg_sq[S + s] = first_step_norm ? T * T : P2;
      inv[s] = static_cast<float>(1.0 / Lam);
      if (lambda_out) lambda_out[s] = static_cast<float>(Lam);
    }
  }
}

__global__ __launch_bounds__(kBlock) void sqrt_to_f32(const double* __restrict__ sq_in,
                                                      float* __restrict__ out, int S) {
  const int s = blockIdx.x * kBlock + threadIdx.x;
  if (s < S) out[s] = static_cast<float>(sqrt(sq_in[s]));
}

// ---------------------------------------------------------------- launches

static inline unsigned tiles_of(int64_t n, int64_t tile) {
  return static_cast<unsigned>((n + tile - 1) / tile);
}

hipError_t launch_sqnorm_partials(int nb, const float* b0, float phi0, const float* b1,
                                  float phi1, const int64_t* off_dev, int S, int64_t n,
                                  double* part0, double* part1, hipStream_t st) {
  const dim3 grid(tiles_of(n, kNormTile)), block(kBlock);
  if (nb == 2) {
    hipLaunchKernelGGL(sqnorm_partials<2>, grid, block, 0, st, b0, phi0, b1, phi1, off_dev, S, n,
                       part0, part1);
  } else {
    hipLaunchKernelGGL(sqnorm_partials<1>, grid, block, 0, st, b0, phi0, b0, 0.0f, off_dev, S, n,
                       part0, part0);
  }
  return hipGetLastError();
}

static inline unsigned seg_grid(int S) { return static_cast<unsigned>(S < 65536 ? S : 65536); }

hipError_t launch_segment_totals(const double* part, const int64_t* off_dev, int S,
                                 int64_t tile_elems, double* out, hipStream_t st) {
  hipLaunchKernelGGL(segment_totals, dim3(seg_grid(S)), dim3(kBlock), 0, st, part, off_dev, S,
                     tile_elems, out);
  return hipGetLastError();
}

hipError_t launch_lambda_stage2(const double* part_m, const double* part_d,
                                const int64_t* off_dev, int S, int64_t tile_elems,
                                const float* first_step_norm, float c, float alpha, int tau,
                                double* seg_sq, float* inv, float* lambda_out, hipStream_t st) {
  hipLaunchKernelGGL(lambda_stage2, dim3(seg_grid(S)), dim3(kBlock), 0, st, part_m, part_d,
                     off_dev, S, tile_elems, first_step_norm, c, alpha, tau, seg_sq, inv,
                     lambda_out);
  return hipGetLastError();
}

hipError_t launch_sqrt_to_f32(const double* sq_in, float* out, int S, hipStream_t st) {
  hipLaunchKernelGGL(sqrt_to_f32, dim3((S + kBlock - 1) / kBlock), dim3(kBlock), 0, st, sq_in,
                     out, S);
  return hipGetLastError();
}

}  // namespace co2
