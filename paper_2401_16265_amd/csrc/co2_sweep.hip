// The fused elementwise sweep of one CO2 outer update (CO2 paper, Algorithm 1:
// momentum and outer-iterate lines; Section 3.3 for Clip), the first-round
// kernel, the deferred outer-iterate kernel of the norm-rescale variant, and a
// plain copy kernel used as the bandwidth yardstick.
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
//
// Variants of the rule (wavefront-uniform run-time switches, SweepMode):
//   own_current    the mean runs over THIS round's pseudo-gradients (Section 3.2's
//                  recursion before the staleness): the worker's own anchor - params
//                  formed here comes first in the sum, followed by the buffers read;
//   pull           the local parameters are pulled towards the new outer iterate,
//                  params = x - rho*(x - x'), instead of restarting from it (the
//                  anchor-model rule of the overlap variant of local SGD);
//   defer_iterate  clipping by norm rescale: x' needs ||m'||_s, so this kernel only
//                  writes m' and delta_out (and the slot sums, taken without the
//                  coordinate clamp), and apply_iterate writes x' afterwards.
#include "co2_device.hpp"
#include "co2_launch.hpp"

namespace co2 {

struct SweepScalars {
  float alpha, beta, phi, rK;
};

// Sum over the workers, left to right, times 1/K.  With `own_first` the
// worker's own current pseudo-gradient `own` is the first term and the NB
// buffers follow; otherwise the NB buffers are all the terms (NB >= 1).
template <int NB>
__device__ __forceinline__ float mean_of_workers(const float* d, float own, bool own_first, float rK) {
  float sum;
  if constexpr (NB == 0) {
    sum = own;
  } else {
    sum = own_first ? own + d[0] : d[0];
#pragma unroll
    for (int k = 1; k < NB; ++k) sum = sum + d[k];
  }
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

// What the local parameters become: the new outer iterate, or a step of rho
// from the old local value towards it.
__device__ __forceinline__ float local_after(float x_old, float x_new, bool pull, float rho) {
  if (!pull) return x_new;
  const float gap = x_old - x_new;
  const float step = rho * gap;
  return x_old - step;
}

__device__ __forceinline__ float comp(const float4& q, int e) {
  return e == 0 ? q.x : e == 1 ? q.y : e == 2 ? q.z : q.w;
}

// With many worker buffers the tile's loads go out in two phases: the first
// phase_a_buffers buffers together with anchor, momentum and params, the rest once
// those have arrived (their partial sum is formed while the second phase is in
// flight).  A wavefront then never holds more than about 11 KB of loads in
// flight, as at K = 8, and the compute unit can keep as many wavefronts resident
// as there; with all 3 + NB loads in flight at once it could keep only 4, too
// few to cover each other's compute and store phases.  The order of the sum is
// unchanged (left to right over the buffers).
constexpr int kTwoPhaseFrom = 11;                  // fp32 buffers read; below this one phase is faster
template <int NB, int DT>
constexpr int phase_a_buffers() { return (DT == kDeltaF32 && NB >= kTwoPhaseFrom) ? (NB + 1) / 2 : NB; }

template <int NB, bool HAS_X, int DT>
struct SubTile {
  float4 va, vm, vx;
  typename DeltaIO<DT>::Vec vd[NB > 0 ? NB : 1];
};

// Loads of anchor, momentum, params and pseudo-gradient buffers [0, phase_a_buffers).
template <int NB, bool HAS_X, int DT>
__device__ __forceinline__ void load_sub(SubTile<NB, HAS_X, DT>& t, const float* x,
                                         const float* a_in, const float* m, const DeltaPtrs& d,
                                         int64_t base, int lane) {
  t.va = ld4_stream(a_in + base, lane);
  t.vm = ld4_stream(m + base, lane);
  if (HAS_X) t.vx = ld4_stream(x + base, lane);
#pragma unroll
  for (int k = 0; k < phase_a_buffers<NB, DT>(); ++k) t.vd[k] = DeltaIO<DT>::load4(d.p[k], base, lane);
}

// Update and store one 256-coordinate tile held in registers.
template <int NB, bool HAS_X, int DT>
__device__ __forceinline__ void finish_sub(SubTile<NB, HAS_X, DT>& t, float* x,
                                           float* a_out, float* m, const DeltaPtrs& d, void* dout,
                                           int64_t base, int lane, float inv, const SweepScalars& h,
                                           const SweepMode& mode,
                                           double& acc_m, double& acc_d, int& nclip) {
  using IO = DeltaIO<DT>;
  constexpr int NA = phase_a_buffers<NB, DT>();
  float mc[4], xc[4], dc[4], lc[4], sum[4];
  if constexpr (NA < NB) {
    // second phase: wait for the first, then issue the remaining buffers' loads
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
#pragma unroll
    for (int k = NA; k < NB; ++k) t.vd[k] = IO::load4(d.p[k], base, lane);
  }
#pragma unroll
  for (int e = 0; e < 4; ++e) {
    dc[e] = 0.0f;
    if (HAS_X) {
      dc[e] = IO::stored(comp(t.va, e) - comp(t.vx, e));
      acc_d += sq(dc[e]);
    }
    // sum over the workers, left to right; in the current-round order the worker's own
    // pseudo-gradient formed above leads
    if constexpr (NB == 0) {
      sum[e] = dc[e];
    } else {
      const float d0 = IO::get(t.vd[0], e);
      sum[e] = mode.own_current ? dc[e] + d0 : d0;
#pragma unroll
      for (int k = 1; k < NA; ++k) sum[e] = sum[e] + IO::get(t.vd[k], e);
    }
  }
#pragma unroll
  for (int e = 0; e < 4; ++e) {
#pragma unroll
    for (int k = NA; k < NB; ++k) sum[e] = sum[e] + IO::get(t.vd[k], e);
    mc[e] = comp(t.vm, e);
    xc[e] = outer_coord(comp(t.va, e), mc[e], sum[e] * h.rK, inv, h);
    if (HAS_X) lc[e] = local_after(comp(t.vx, e), xc[e], mode.pull, mode.rho);
    // the term carried to the next round's gap: Clip(m', phi)^2, or under norm rescale m'^2
    // itself (a clamp at phi = inf would turn a NaN into inf)
    acc_m += sq(mode.defer_iterate ? mc[e] : clip_coord(mc[e], h.phi));
    nclip += __popcll(__ballot(fabsf(mc[e]) > h.phi));   // wavefront-uniform count
  }
  constexpr int kTileBytes = kWave * 16;
  if (HAS_X) IO::store4(dout, base, lane, dc);
  st4_stream(m + base, kTileBytes, lane, make_float4(mc[0], mc[1], mc[2], mc[3]));
  if (mode.defer_iterate) return;
  if (HAS_X) st4_stream(x + base, kTileBytes, lane, make_float4(lc[0], lc[1], lc[2], lc[3]));
  st4_stream(a_out + base, kTileBytes, lane, make_float4(xc[0], xc[1], xc[2], xc[3]));
}

template <int NB, bool HAS_X, int DT>
__global__ __launch_bounds__(kWave) void fused_sweep(
    float* x, const float* a_in, float* a_out, float* m, DeltaPtrs d, void* dout,
    const float* __restrict__ inv_tab, const int64_t* __restrict__ off, int S, int64_t n,
    SweepScalars h, SweepMode mode, SlotRec* __restrict__ slots) {
  using IO = DeltaIO<DT>;
  const int64_t tile = blockIdx.x;
  const int64_t base = tile * kSweepTile;
  const int lane = threadIdx.x;
  const bool full = base + kSweepTile <= n;

  // The tile's loads go out before the segment lookup, which does not depend
  // on them and runs while they are in flight.
  SubTile<NB, HAS_X, DT> cur;
  if (full) load_sub<NB, HAS_X, DT>(cur, x, a_in, m, d, base, lane);
  const int s_lo = seg_of(off, S, base);

  if (full && base + kSweepTile <= off[s_lo + 1]) {
    const float inv = inv_tab[s_lo];
    double acc_m = 0.0, acc_d = 0.0;
    int nclip = 0;
    finish_sub<NB, HAS_X, DT>(cur, x, a_out, m, d, dout, base, lane, inv, h, mode, acc_m, acc_d, nclip);
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
      float dk[NB > 0 ? NB : 1];
#pragma unroll
      for (int k = 0; k < NB; ++k) dk[k] = IO::load1(d.p[k], j);
      float dj = 0.0f, xj = 0.0f;
      if (HAS_X) {
        xj = x[j];
        dj = IO::stored(a - xj);
      }
      const float xn = outer_coord(a, mj, mean_of_workers<NB>(dk, dj, mode.own_current, h.rK), inv, h);
      acc_m += sq(mode.defer_iterate ? mj : clip_coord(mj, h.phi));
      if (fabsf(mj) > h.phi) acc_c += 1.0;
      if (HAS_X) {
        acc_d += sq(dj);
        IO::store1(dout, j, dj);
        if (!mode.defer_iterate) x[j] = local_after(xj, xn, mode.pull, mode.rho);
      }
      m[j] = mj;
      if (!mode.defer_iterate) a_out[j] = xn;
    }
    const double tm = wave_sum(acc_m);
    const double tc = wave_sum(acc_c);
    double td = 0.0;
    if (HAS_X) td = wave_sum(acc_d);
    write_slot(slots, tile + s, lane, tm, td, tc);
  }
}

// Outer iterate of the norm-rescale variant, after the sweep has written m':
//   x' = anchor - alpha*(m'*scale[s]),  scale[s] = min(1, phi/||m'||_s);
//   anchor_out = x';  params = x' (or pulled towards it).
// Same tile structure as the sweep; 8 (12 with params) bytes read and 4 (8)
// written per coordinate.
template <bool HAS_X>
__global__ __launch_bounds__(kWave) void apply_iterate(
    float* x, const float* a_in, float* a_out, const float* __restrict__ m,
    const float* __restrict__ scale_tab, const int64_t* __restrict__ off, int S, int64_t n,
    float alpha, SweepMode mode) {
  const int64_t tile = blockIdx.x;
  const int64_t base = tile * kSweepTile;
  const int64_t end = (base + kSweepTile < n) ? base + kSweepTile : n;
  const int lane = threadIdx.x;
  const bool full = base + kSweepTile <= n;
  const bool need_x = HAS_X && mode.pull;
  float4 va, vm, vx = make_float4(0.0f, 0.0f, 0.0f, 0.0f);
  if (full) {
    va = ld4_stream(a_in + base, lane);
    vm = ld4_stream(m + base, lane);
    if (need_x) vx = ld4_stream(x + base, lane);
  }
  const int s_lo = seg_of(off, S, base);

  if (full && base + kSweepTile <= off[s_lo + 1]) {
    const float scale = scale_tab[s_lo];
    float xc[4], lc[4];
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      const float cm = comp(vm, e) * scale;
      const float stepv = alpha * cm;
      xc[e] = comp(va, e) - stepv;
      lc[e] = local_after(comp(vx, e), xc[e], need_x, mode.rho);
    }
    if (HAS_X) st4_stream(x + base, kWave * 16, lane, make_float4(lc[0], lc[1], lc[2], lc[3]));
    st4_stream(a_out + base, kWave * 16, lane, make_float4(xc[0], xc[1], xc[2], xc[3]));
    return;
  }

  const int s_hi = seg_of(off, S, end - 1);
  for (int s = s_lo; s <= s_hi; ++s) {
    const int64_t lo = off[s] > base ? off[s] : base;
    const int64_t hi = off[s + 1] < end ? off[s + 1] : end;
    if (lo >= hi) continue;
    const float scale = scale_tab[s];
    for (int64_t j = lo + lane; j < hi; j += kWave) {
      const float cm = m[j] * scale;
      const float stepv = alpha * cm;
      const float xn = a_in[j] - stepv;
      if (HAS_X) x[j] = local_after(need_x ? x[j] : 0.0f, xn, need_x, mode.rho);
      a_out[j] = xn;
    }
  }
}

// First outer round (Section 3.1: the gap/momentum/iterate lines are skipped):
// delta_out = anchor - params; params = anchor_out = anchor.  Also leaves the
// sums of Clip(m,phi)^2 and delta_out^2 per slot for the next round's gap.
// Same tile structure as the sweep.
template <bool HAS_X, int DT>
__global__ __launch_bounds__(kWave) void first_round(
    float* x, const float* a_in, float* a_out, const float* __restrict__ m, void* dout,
    const int64_t* __restrict__ off, int S, int64_t n, float phi, SlotRec* __restrict__ slots) {
  using IO = DeltaIO<DT>;
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

template <int NB, bool HAS_X, int DT>
static hipError_t launch_sweep_v(const SweepArgs& g, hipStream_t st) {
  const unsigned tiles = static_cast<unsigned>((g.n + kSweepTile - 1) / kSweepTile);
  // 16-bit pseudo-gradients put half the bytes per stream in flight: two of them count as one
  // fp32 stream (K = 1 and 2 apart, which run fastest with more wavefronts: measured at 1.3B,
  // 12 at K = 1 and 10 at K = 2 against 8: +8 % and +3 %).
  // Kernels with two load phases hold at most ~11 KB in flight per wavefront like K = 8, but run
  // fastest with slightly fewer wavefronts (measured at 1.3B: 6 at K = 12, 5 at K = 16).
  constexpr bool kTwoPhase = phase_a_buffers<NB, DT>() < NB;
  const float delta_kb = DT == kDeltaF32 ? float(NB) : NB <= 2 ? 0.5f * float(NB) : float((NB + 1) / 2);
  const int dflt = !kTwoPhase ? default_sweep_waves(delta_kb) : NB > 12 ? 5 : 6;
  const unsigned lds = throttle_lds_bytes(g.waves_per_cu > 0 ? g.waves_per_cu : dflt);
  const SweepScalars h{g.alpha, g.beta, g.phi, g.rK};
  hipLaunchKernelGGL((fused_sweep<NB, HAS_X, DT>), dim3(tiles), dim3(kWave), lds, st, g.x, g.a_in,
                     g.a_out, g.m, g.d, g.dout, g.inv, g.off_dev, g.S, g.n, h, g.mode, g.slots);
  return hipGetLastError();
}

template <int NB>
static hipError_t launch_sweep_k(bool has_x, const SweepArgs& g, hipStream_t st) {
  if (g.dtype == kDeltaBF16)
    return has_x ? launch_sweep_v<NB, true, kDeltaBF16>(g, st) : launch_sweep_v<NB, false, kDeltaBF16>(g, st);
  if (g.dtype == kDeltaF16)
    return has_x ? launch_sweep_v<NB, true, kDeltaF16>(g, st) : launch_sweep_v<NB, false, kDeltaF16>(g, st);
  return has_x ? launch_sweep_v<NB, true, kDeltaF32>(g, st) : launch_sweep_v<NB, false, kDeltaF32>(g, st);
}

hipError_t launch_fused_sweep(int nbuf, bool has_x, const SweepArgs& g, hipStream_t st) {
  switch (nbuf) {
    // no buffer at all: a single worker in the current-round order (fp32, fused form only)
    case 0:
      if (!has_x || g.dtype != kDeltaF32 || !g.mode.own_current) return hipErrorInvalidValue;
      return launch_sweep_v<0, true, kDeltaF32>(g, st);
#define CO2_CASE(k) case k: return launch_sweep_k<k>(has_x, g, st);
    CO2_CASE(1) CO2_CASE(2) CO2_CASE(3) CO2_CASE(4) CO2_CASE(5) CO2_CASE(6) CO2_CASE(7)
    CO2_CASE(8) CO2_CASE(9) CO2_CASE(10) CO2_CASE(11) CO2_CASE(12) CO2_CASE(13) CO2_CASE(14)
    CO2_CASE(15) CO2_CASE(16)
#undef CO2_CASE
    default: return hipErrorInvalidValue;
  }
}

hipError_t launch_apply_iterate(bool has_x, const SweepArgs& g, const float* scale, hipStream_t st) {
  const unsigned tiles = static_cast<unsigned>((g.n + kSweepTile - 1) / kSweepTile);
  const unsigned lds = throttle_lds_bytes(kApplyWavesPerCu);
  if (has_x) {
    hipLaunchKernelGGL((apply_iterate<true>), dim3(tiles), dim3(kWave), lds, st, g.x, g.a_in, g.a_out,
                       g.m, scale, g.off_dev, g.S, g.n, g.alpha, g.mode);
  } else {
    hipLaunchKernelGGL((apply_iterate<false>), dim3(tiles), dim3(kWave), lds, st, g.x, g.a_in, g.a_out,
                       g.m, scale, g.off_dev, g.S, g.n, g.alpha, g.mode);
  }
  return hipGetLastError();
}

template <bool HAS_X, int DT>
static hipError_t launch_first_v(const SweepArgs& g, hipStream_t st) {
  const unsigned tiles = static_cast<unsigned>((g.n + kSweepTile - 1) / kSweepTile);
  const unsigned lds = throttle_lds_bytes(default_sweep_waves(1));
  hipLaunchKernelGGL((first_round<HAS_X, DT>), dim3(tiles), dim3(kWave), lds, st, g.x, g.a_in,
                     g.a_out, g.m, g.dout, g.off_dev, g.S, g.n, g.phi, g.slots);
  return hipGetLastError();
}

hipError_t launch_first_round(bool has_x, const SweepArgs& g, hipStream_t st) {
  if (g.dtype == kDeltaBF16)
    return has_x ? launch_first_v<true, kDeltaBF16>(g, st) : launch_first_v<false, kDeltaBF16>(g, st);
  if (g.dtype == kDeltaF16)
    return has_x ? launch_first_v<true, kDeltaF16>(g, st) : launch_first_v<false, kDeltaF16>(g, st);
  return has_x ? launch_first_v<true, kDeltaF32>(g, st) : launch_first_v<false, kDeltaF32>(g, st);
}

hipError_t launch_copy_f32(const float* src, float* dst, int64_t n, hipStream_t st) {
  constexpr int64_t kTile = int64_t(kWave) * 16;
  const unsigned lds = throttle_lds_bytes(kCopyWavesPerCu);
  hipLaunchKernelGGL(copy_f32, dim3(static_cast<unsigned>((n + kTile - 1) / kTile)), dim3(kWave),
                     lds, st, src, dst, n);
  return hipGetLastError();
}

}  // namespace co2
