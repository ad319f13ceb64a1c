// The fused elementwise sweep of one CO2 outer update (CO2 paper, Algorithm 1:
// momentum and outer-iterate lines; Section 3.3 for Clip), the first-round
// kernel, and a plain copy kernel used as the bandwidth yardstick.
//
// Per coordinate j of segment s (fp32, every operation rounded once):
//   delta_out[j] = anchor[j] - params[j]                       (this round's pseudo-gradient)
//   dbar  = (((d_0[j] + d_1[j]) + ...) + d_{K-1}[j]) * (1/K)    (mean over workers, round t-1)
//   m'    = beta*m[j] + dbar*inv[s]                             (inv = 1/Lambda_t)
//   x'    = anchor[j] - alpha*Clip(m', phi)
//   m[j] = m';  params[j] = anchor_out[j] = x'
// 3+K read streams and 4 write streams, 28+4K bytes per coordinate, nothing
// staged through HBM in between.  The flat index space is cut into aligned
// tiles of kSweepTile elements, one workgroup each.  A tile inside one segment
// issues all its 16-byte loads first (U per lane and stream), with 1/Lambda a
// workgroup-uniform scalar; a tile holding a segment boundary or the ragged end
// gives each of its segments to one wavefront, element by element.
//
// While it writes m' and delta_out the sweep also accumulates, in fp64, the sums
// of Clip(m',phi)^2 and delta_out^2 per (tile, segment) slot: they are the two
// sums of squares the NEXT round's gap needs, so a steady-state caller can skip
// the separate norm pass.
#include "co2_device.hpp"
#include "co2_launch.hpp"

namespace co2 {

struct SweepScalars {
  float alpha, beta, phi, rK;
};

template <int K>
__device__ __forceinline__ float mean_of_workers(const float (&d)[K], float rK) {
  float sum = d[0];
#pragma unroll
  for (int k = 1; k < K; ++k) sum = sum + d[k];
  return sum * rK;
}

// One coordinate of the update.  Returns x'; m is updated in place.
__device__ __forceinline__ float outer_coord(float a, float& m, float dbar, float inv,
                                             const SweepScalars& h) {
  const float bm = h.beta * m;
  const float pen = dbar * inv;
  m = bm + pen;
  const float stepv = h.alpha * clip_coord(m, h.phi);
  return a - stepv;
}

template <int K, int U, bool HAS_X>
__global__ __launch_bounds__(kBlock) void fused_sweep(
    float* x, const float* a_in, float* a_out, float* m, DeltaPtrs d, float* dout,
    const float* __restrict__ inv_tab, const int64_t* __restrict__ off, int S, int64_t n,
    SweepScalars h, double* __restrict__ part_m, double* __restrict__ part_d) {
  __shared__ double lds[2][kWavesPerBlock];
  constexpr int64_t kTile = int64_t(kBlock) * 4 * U;
  const int64_t tile = blockIdx.x;
  const int64_t base = tile * kTile;
  const int s_lo = seg_of(off, S, base);

  if (base + kTile <= n && base + kTile <= off[s_lo + 1]) {
    // Full tile inside segment s_lo: vector path.
    float4 va[U], vm[U], vx[U], vd[K][U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int64_t j = base + ((int64_t(u) * kBlock + threadIdx.x) << 2);
      va[u] = ld4(a_in + j);
      vm[u] = ld4(m + j);
      if (HAS_X) vx[u] = ld4(x + j);
#pragma unroll
      for (int k = 0; k < K; ++k) vd[k][u] = ld4(d.p[k] + j);
    }
    const float inv = inv_tab[s_lo];
    double acc_m = 0.0, acc_d = 0.0;
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int64_t j = base + ((int64_t(u) * kBlock + threadIdx.x) << 2);
      const float ac[4] = {va[u].x, va[u].y, va[u].z, va[u].w};
      float mc[4] = {vm[u].x, vm[u].y, vm[u].z, vm[u].w};
      float xc[4], dc[4];
      if (HAS_X) {
        const float xin[4] = {vx[u].x, vx[u].y, vx[u].z, vx[u].w};
#pragma unroll
        for (int e = 0; e < 4; ++e) dc[e] = ac[e] - xin[e];
      }
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        float dk[K];
#pragma unroll
        for (int k = 0; k < K; ++k) {
          const float4 q = vd[k][u];
          dk[k] = e == 0 ? q.x : e == 1 ? q.y : e == 2 ? q.z : q.w;
        }
        xc[e] = outer_coord(ac[e], mc[e], mean_of_workers<K>(dk, h.rK), inv, h);
        acc_m += sq(clip_coord(mc[e], h.phi));
        if (HAS_X) acc_d += sq(dc[e]);
      }
      const float4 xo = make_float4(xc[0], xc[1], xc[2], xc[3]);
      if (HAS_X) {
        st4(dout + j, make_float4(dc[0], dc[1], dc[2], dc[3]));
        st4(x + j, xo);
      }
      st4(m + j, make_float4(mc[0], mc[1], mc[2], mc[3]));
      st4(a_out + j, xo);
    }
    const double tm = block_sum(acc_m, lds[0]);
    double td = 0.0;
    if (HAS_X) td = block_sum(acc_d, lds[1]);
    if (threadIdx.x == 0) {
      part_m[tile + s_lo] = tm;
      if (HAS_X) part_d[tile + s_lo] = td;
    }
    return;
  }

  // Boundary or ragged tile: wavefront w takes segments s_lo+w, s_lo+w+4, ...
  const int64_t end = (base + kTile < n) ? base + kTile : n;
  const int s_hi = seg_of(off, S, end - 1);
  const int wave = threadIdx.x / kWave, lane = threadIdx.x & (kWave - 1);
  for (int s = s_lo + wave; s <= s_hi; s += kWavesPerBlock) {
    const int64_t lo = off[s] > base ? off[s] : base;
    const int64_t hi = off[s + 1] < end ? off[s + 1] : end;
    if (lo >= hi) continue;
    const float inv = inv_tab[s];
    double acc_m = 0.0, acc_d = 0.0;
    for (int64_t j = lo + lane; j < hi; j += kWave) {
      const float a = a_in[j];
      float mj = m[j];
      float dk[K];
#pragma unroll
      for (int k = 0; k < K; ++k) dk[k] = d.p[k][j];
      float dj = 0.0f;
      if (HAS_X) dj = a - x[j];
      const float xn = outer_coord(a, mj, mean_of_workers<K>(dk, h.rK), inv, h);
      acc_m += sq(clip_coord(mj, h.phi));
      if (HAS_X) {
        acc_d += sq(dj);
        dout[j] = dj;
        x[j] = xn;
      }
      m[j] = mj;
      a_out[j] = xn;
    }
    const double tm = wave_sum(acc_m);
    double td = 0.0;
    if (HAS_X) td = wave_sum(acc_d);
    if (lane == 0) {
      part_m[tile + s] = tm;
      if (HAS_X) part_d[tile + s] = td;
    }
  }
}

// First outer round (Section 3.1: the gap/momentum/iterate lines are skipped):
// delta_out = anchor - params; params = anchor_out = anchor.  Also leaves the
// sums of Clip(m,phi)^2 and delta_out^2 per slot for the next round's gap.
template <bool HAS_X>
__global__ __launch_bounds__(kBlock) void first_round(
    float* x, const float* a_in, float* a_out, const float* __restrict__ m, float* dout,
    const int64_t* __restrict__ off, int S, int64_t n, float phi,
    double* __restrict__ part_m, double* __restrict__ part_d) {
  constexpr int64_t kTile = kSweepTile;
  const int64_t tile = blockIdx.x;
  const int64_t base = tile * kTile;
  const int64_t end = (base + kTile < n) ? base + kTile : n;
  const int s_lo = seg_of(off, S, base);
  const int s_hi = seg_of(off, S, end - 1);
  const int wave = threadIdx.x / kWave, lane = threadIdx.x & (kWave - 1);
  // Same (tile, segment) slot layout as the sweep; one wavefront per segment
  // piece.  This kernel runs once per training run, so it is kept simple.
  for (int s = s_lo + wave; s <= s_hi; s += kWavesPerBlock) {
    const int64_t lo = off[s] > base ? off[s] : base;
    const int64_t hi = off[s + 1] < end ? off[s + 1] : end;
    if (lo >= hi) continue;
    double acc_m = 0.0, acc_d = 0.0;
    for (int64_t j = lo + lane; j < hi; j += kWave) {
      const float a = a_in[j];
      acc_m += sq(clip_coord(m[j], phi));
      if (HAS_X) {
        const float dj = a - x[j];
        acc_d += sq(dj);
        dout[j] = dj;
        x[j] = a;
      }
      if (a_out != a_in) a_out[j] = a;
    }
    const double tm = wave_sum(acc_m);
    double td = 0.0;
    if (HAS_X) td = wave_sum(acc_d);
    if (lane == 0) {
      part_m[tile + s] = tm;
      if (HAS_X) part_d[tile + s] = td;
    }
  }
}

__global__ __launch_bounds__(kBlock) void copy_f32(const float* __restrict__ src,
                                                   float* __restrict__ dst, int64_t n) {
  constexpr int U = 4;
  constexpr int64_t kTile = int64_t(kBlock) * 4 * U;
  const int64_t base = blockIdx.x * kTile;
  if (base + kTile <= n) {
    float4 v[U];
#pragma unroll
    for (int u = 0; u < U; ++u) v[u] = ld4(src + base + ((int64_t(u) * kBlock + threadIdx.x) << 2));
#pragma unroll
    for (int u = 0; u < U; ++u) st4(dst + base + ((int64_t(u) * kBlock + threadIdx.x) << 2), v[u]);
  } else {
    for (int64_t j = base + threadIdx.x; j < n; j += kBlock) dst[j] = src[j];
  }
}

// ---------------------------------------------------------------- launches

template <int K>
static hipError_t launch_sweep_k(bool has_x, const SweepArgs& g, hipStream_t st) {
  const unsigned tiles = static_cast<unsigned>((g.n + kSweepTile - 1) / kSweepTile);
  const SweepScalars h{g.alpha, g.beta, g.phi, g.rK};
  if (has_x) {
    hipLaunchKernelGGL((fused_sweep<K, CO2_SWEEP_U, true>), dim3(tiles), dim3(kBlock), 0, st,
                       g.x, g.a_in, g.a_out, g.m, g.d, g.dout, g.inv, g.off_dev, g.S, g.n, h,
                       g.part_m, g.part_d);
  } else {
    hipLaunchKernelGGL((fused_sweep<K, CO2_SWEEP_U, false>), dim3(tiles), dim3(kBlock), 0, st,
                       g.x, g.a_in, g.a_out, g.m, g.d, g.dout, g.inv, g.off_dev, g.S, g.n, h,
                       g.part_m, g.part_d);
  }
  return hipGetLastError();
}

hipError_t launch_fused_sweep(int K, bool has_x, const SweepArgs& g, hipStream_t st) {
  switch (K) {
#define CO2_CASE(k) case k: return launch_sweep_k<k>(has_x, g, st);
    CO2_CASE(1) CO2_CASE(2) CO2_CASE(3) CO2_CASE(4) CO2_CASE(5) CO2_CASE(6) CO2_CASE(7)
    CO2_CASE(8) CO2_CASE(9) CO2_CASE(10) CO2_CASE(11) CO2_CASE(12) CO2_CASE(13) CO2_CASE(14)
    CO2_CASE(15) CO2_CASE(16)
#undef CO2_CASE
    default: return hipErrorInvalidValue;
  }
}

hipError_t launch_first_round(bool has_x, const SweepArgs& g, hipStream_t st) {
  const unsigned tiles = static_cast<unsigned>((g.n + kSweepTile - 1) / kSweepTile);
  if (has_x) {
    hipLaunchKernelGGL(first_round<true>, dim3(tiles), dim3(kBlock), 0, st, g.x, g.a_in, g.a_out,
                       g.m, g.dout, g.off_dev, g.S, g.n, g.phi, g.part_m, g.part_d);
  } else {
    hipLaunchKernelGGL(first_round<false>, dim3(tiles), dim3(kBlock), 0, st, g.x, g.a_in,
                       g.a_out, g.m, g.dout, g.off_dev, g.S, g.n, g.phi, g.part_m, g.part_d);
  }
  return hipGetLastError();
}

hipError_t launch_copy_f32(const float* src, float* dst, int64_t n, hipStream_t st) {
  constexpr int64_t kTile = int64_t(kBlock) * 16;
  hipLaunchKernelGGL(copy_f32, dim3(static_cast<unsigned>((n + kTile - 1) / kTile)),
                     dim3(kBlock), 0, st, src, dst, n);
  return hipGetLastError();
}

}  // namespace co2
