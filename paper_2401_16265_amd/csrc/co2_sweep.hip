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
// staged through HBM in between.  One single-wavefront workgroup per aligned
// tile of 256 coordinates: the lane issues its 3+K 16-byte loads at once, the
// segment lookup (a short scalar binary search) runs while they are in flight,
// and 1/Lambda is then a wavefront-uniform scalar.  A tile that holds a segment
// boundary or the ragged end walks its segments element by element instead.
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

__device__ __forceinline__ float comp(const float4& q, int e) {
  return e == 0 ? q.x : e == 1 ? q.y : e == 2 ? q.z : q.w;
}

template <int K, bool HAS_X, bool BF16>
struct SubTile {
  float4 va, vm, vx;
  typename DeltaIO<BF16>::Vec vd[K];
};

template <int K, bool HAS_X, bool BF16>
__device__ __forceinline__ void load_sub(SubTile<K, HAS_X, BF16>& t, const float* x,
                                         const float* a_in, const float* m, const DeltaPtrs& d,
                                         int64_t base, int lane) {
  t.va = ld4_stream(a_in + base, lane);
  t.vm = ld4_stream(m + base, lane);
  if (HAS_X) t.vx = ld4_stream(x + base, lane);
#pragma unroll
  for (int k = 0; k < K; ++k) t.vd[k] = DeltaIO<BF16>::load4(d.p[k], base, lane);
}

// Update and store one 256-coordinate tile held in registers.
template <int K, bool HAS_X, bool BF16>
__device__ __forceinline__ void finish_sub(const SubTile<K, HAS_X, BF16>& t, float* x,
                                           float* a_out, float* m, void* dout, int64_t base,
                                           int lane, float inv, const SweepScalars& h,
                                           double& acc_m, double& acc_d, int& nclip) {
  using IO = DeltaIO<BF16>;
  float mc[4], xc[4], dc[4];
#pragma unroll
  for (int e = 0; e < 4; ++e) {
    const float ae = comp(t.va, e);
    float dk[K];
#pragma unroll
    for (int k = 0; k < K; ++k) dk[k] = IO::get(t.vd[k], e);
    if (HAS_X) {
      dc[e] = IO::stored(ae - comp(t.vx, e));
      acc_d += sq(dc[e]);
    }
    mc[e] = comp(t.vm, e);
    xc[e] = outer_coord(ae, mc[e], mean_of_workers<K>(dk, h.rK), inv, h);
    acc_m += sq(clip_coord(mc[e], h.phi));
    nclip += __popcll(__ballot(fabsf(mc[e]) > h.phi));   // wavefront-uniform count
  }
  constexpr int kTileBytes = kWave * 16;
  const float4 xo = make_float4(xc[0], xc[1], xc[2], xc[3]);
  if (HAS_X) {
    IO::store4(dout, base, lane, dc);
    st4_stream(x + base, kTileBytes, lane, xo);
  }
  st4_stream(m + base, kTileBytes, lane, make_float4(mc[0], mc[1], mc[2], mc[3]));
  st4_stream(a_out + base, kTileBytes, lane, xo);
}

template <int K, bool HAS_X, bool BF16>
__global__ __launch_bounds__(kWave) void fused_sweep(
    float* x, const float* a_in, float* a_out, float* m, DeltaPtrs d, void* dout,
    const float* __restrict__ inv_tab, const int64_t* __restrict__ off, int S, int64_t n,
    SweepScalars h, SlotRec* __restrict__ slots) {
  using IO = DeltaIO<BF16>;
  const int64_t tile = blockIdx.x;
  const int64_t base = tile * kSweepTile;
  const int lane = threadIdx.x;
  const bool full = base + kSweepTile <= n;

  // The tile's loads go out before the segment lookup, which does not depend
  // on them and runs while they are in flight.
  SubTile<K, HAS_X, BF16> cur;
  if (full) load_sub<K, HAS_X, BF16>(cur, x, a_in, m, d, base, lane);
  const int s_lo = seg_of(off, S, base);

  if (full && base + kSweepTile <= off[s_lo + 1]) {
    const float inv = inv_tab[s_lo];
    double acc_m = 0.0, acc_d = 0.0;
    int nclip = 0;
    finish_sub<K, HAS_X, BF16>(cur, x, a_out, m, dout, base, lane, inv, h, acc_m, acc_d, nclip);
    const double tm = wave_sum(acc_m);
    double td = 0.0;
    if (HAS_X) td = wave_sum(acc_d);
    write_slot(slots, tile + s_lo, lane, tm, td, static_cast<double>(nclip));
    return;
  }

  // Boundary or ragged tile: one segment piece after the other.
  const int64_t end = (base + kSweepTile < n) ? base + kSweepTile : n;
  const int s_hi = seg_of(off, S, end - 1);
  for (int s = s_lo; s <= s_hi; ++s) {
    const int64_t lo = off[s] > base ? off[s] : base;
    const int64_t hi = off[s + 1] < end ? off[s + 1] : end;
    if (lo >= hi) continue;
    const float inv = inv_tab[s];
    double acc_m = 0.0, acc_d = 0.0, acc_c = 0.0;
    for (int64_t j = lo + lane; j < hi; j += kWave) {
      const float a = a_in[j];
      float mj = m[j];
      float dk[K];
#pragma unroll
      for (int k = 0; k < K; ++k) dk[k] = IO::load1(d.p[k], j);
      float dj = 0.0f;
      if (HAS_X) dj = IO::stored(a - x[j]);
      const float xn = outer_coord(a, mj, mean_of_workers<K>(dk, h.rK), inv, h);
      acc_m += sq(clip_coord(mj, h.phi));
      if (fabsf(mj) > h.phi) acc_c += 1.0;
      if (HAS_X) {
        acc_d += sq(dj);
        IO::store1(dout, j, dj);
        x[j] = xn;
      }
      m[j] = mj;
      a_out[j] = xn;
    }
    const double tm = wave_sum(acc_m);
    const double tc = wave_sum(acc_c);
    double td = 0.0;
    if (HAS_X) td = wave_sum(acc_d);
    write_slot(slots, tile + s, lane, tm, td, tc);
  }
}

// First outer round (Section 3.1: the gap/momentum/iterate lines are skipped):
// delta_out = anchor - params; params = anchor_out = anchor.  Also leaves the
// sums of Clip(m,phi)^2 and delta_out^2 per slot for the next round's gap.
// Same tile structure as the sweep.
template <bool HAS_X, bool BF16>
__global__ __launch_bounds__(kWave) void first_round(
    float* x, const float* a_in, float* a_out, const float* __restrict__ m, void* dout,
    const int64_t* __restrict__ off, int S, int64_t n, float phi, SlotRec* __restrict__ slots) {
  using IO = DeltaIO<BF16>;
  const int64_t tile = blockIdx.x;
  const int64_t base = tile * kSweepTile;
  const int64_t end = (base + kSweepTile < n) ? base + kSweepTile : n;
  const int lane = threadIdx.x;
  const bool full = base + kSweepTile <= n;
  float4 va, vm, vx;
  if (full) {
    va = ld4_stream(a_in + base, lane);
    vm = ld4_stream(m + base, lane);
    if (HAS_X) vx = ld4_stream(x + base, lane);
  }
  const int s_lo = seg_of(off, S, base);

  if (full && base + kSweepTile <= off[s_lo + 1]) {
    double acc_m = 0.0, acc_d = 0.0;
    float dc[4];
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      acc_m += sq(clip_coord(comp(vm, e), phi));
      if (HAS_X) {
        dc[e] = IO::stored(comp(va, e) - comp(vx, e));
        acc_d += sq(dc[e]);
      }
    }
    if (HAS_X) {
      IO::store4(dout, base, lane, dc);
      st4_stream(x + base, kWave * 16, lane, va);
    }
    if (a_out != a_in) st4_stream(a_out + base, kWave * 16, lane, va);
    const double tm = wave_sum(acc_m);
    double td = 0.0;
    if (HAS_X) td = wave_sum(acc_d);
    write_slot(slots, tile + s_lo, lane, tm, td, 0.0);   // no outer iterate in the first round
    return;
  }

  const int s_hi = seg_of(off, S, end - 1);
  for (int s = s_lo; s <= s_hi; ++s) {
    const int64_t lo = off[s] > base ? off[s] : base;
    const int64_t hi = off[s + 1] < end ? off[s + 1] : end;
    if (lo >= hi) continue;
    double acc_m = 0.0, acc_d = 0.0;
    for (int64_t j = lo + lane; j < hi; j += kWave) {
      const float a = a_in[j];
      acc_m += sq(clip_coord(m[j], phi));
      if (HAS_X) {
        const float dj = IO::stored(a - x[j]);
        acc_d += sq(dj);
        IO::store1(dout, j, dj);
        x[j] = a;
      }
      if (a_out != a_in) a_out[j] = a;
    }
    const double tm = wave_sum(acc_m);
    double td = 0.0;
    if (HAS_X) td = wave_sum(acc_d);
    write_slot(slots, tile + s, lane, tm, td, 0.0);   // no outer iterate in the first round
  }
}

__global__ __launch_bounds__(kWave) void copy_f32(const float* __restrict__ src,
                                                  float* __restrict__ dst, int64_t n) {
  constexpr int U = 4;
  constexpr int64_t kTile = int64_t(kWave) * 4 * U;
  const int64_t base = blockIdx.x * kTile;
  if (base + kTile <= n) {
    float4 v[U];
#pragma unroll
    for (int u = 0; u < U; ++u) v[u] = ld4_stream(src + base + int64_t(u) * kWave * 4, threadIdx.x);
#pragma unroll
    for (int u = 0; u < U; ++u) st4_stream(dst + base + int64_t(u) * kWave * 4, kWave * 16, threadIdx.x, v[u]);
  } else {
    for (int64_t j = base + threadIdx.x; j < n; j += kWave) dst[j] = src[j];
  }
}

// ---------------------------------------------------------------- launches

template <int K, bool HAS_X, bool BF16>
static hipError_t launch_sweep_v(const SweepArgs& g, hipStream_t st) {
  const unsigned tiles = static_cast<unsigned>((g.n + kSweepTile - 1) / kSweepTile);
  // bf16 pseudo-gradients put half the bytes per stream in flight: cap like K/2 fp32 streams
  const unsigned lds = throttle_lds_bytes(tuning().sweep_waves_per_cu[BF16 ? (K + 1) / 2 : K]);
  const SweepScalars h{g.alpha, g.beta, g.phi, g.rK};
  hipLaunchKernelGGL((fused_sweep<K, HAS_X, BF16>), dim3(tiles), dim3(kWave), lds, st, g.x, g.a_in,
                     g.a_out, g.m, g.d, g.dout, g.inv, g.off_dev, g.S, g.n, h, g.slots);
  return hipGetLastError();
}

template <int K>
static hipError_t launch_sweep_k(bool has_x, const SweepArgs& g, hipStream_t st) {
  if (g.bf16) return has_x ? launch_sweep_v<K, true, true>(g, st) : launch_sweep_v<K, false, true>(g, st);
  return has_x ? launch_sweep_v<K, true, false>(g, st) : launch_sweep_v<K, false, false>(g, st);
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

template <bool HAS_X, bool BF16>
static hipError_t launch_first_v(const SweepArgs& g, hipStream_t st) {
  const unsigned tiles = static_cast<unsigned>((g.n + kSweepTile - 1) / kSweepTile);
  const unsigned lds = throttle_lds_bytes(tuning().sweep_waves_per_cu[1]);
  hipLaunchKernelGGL((first_round<HAS_X, BF16>), dim3(tiles), dim3(kWave), lds, st, g.x, g.a_in,
                     g.a_out, g.m, g.dout, g.off_dev, g.S, g.n, g.phi, g.slots);
  return hipGetLastError();
}

hipError_t launch_first_round(bool has_x, const SweepArgs& g, hipStream_t st) {
  if (g.bf16) return has_x ? launch_first_v<true, true>(g, st) : launch_first_v<false, true>(g, st);
  return has_x ? launch_first_v<true, false>(g, st) : launch_first_v<false, false>(g, st);
}

hipError_t launch_copy_f32(const float* src, float* dst, int64_t n, hipStream_t st) {
  constexpr int64_t kTile = int64_t(kWave) * 16;
  const unsigned lds = throttle_lds_bytes(tuning().copy_waves_per_cu);
  hipLaunchKernelGGL(copy_f32, dim3(static_cast<unsigned>((n + kTile - 1) / kTile)), dim3(kWave),
                     lds, st, src, dst, n);
  return hipGetLastError();
}

}  // namespace co2
