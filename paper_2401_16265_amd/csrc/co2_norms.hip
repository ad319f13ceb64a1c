// Segmented sums of squares for the two norms of the staleness gap
// (CO2 paper, Definition 3.1 / Eq. 3) and the per-segment scalar Lambda.
//
// Pass 1 (sqnorm_partials): the flat index space is cut into aligned tiles of
// kNormTile elements, one single-wavefront workgroup each, which reads its tile
// in pieces of kNormSub elements: 16-byte loads, squares accumulated in fp64
// per lane.  When the segment changes inside the tile (and at the tile's end)
// the lane sums are reduced across the wavefront through DPP and leave ONE
// partial in slot (tile + segment).  The slot index tile+segment is unique per
// pair because both indices only grow along the flat vector, so no atomics and
// no zero-fill are needed.  (Tiles are this long because even a thin stream of
// stores beside the loads costs bandwidth: one record per 1024 elements held
// the pass at 6.5-6.7 TB/s, one per 16384 lets it run at 6.85.)
//
// Stage 2: slot_sums adds each segment's slots in a fixed order (large segments
// are split over several workgroups), then lambda_finish / totals_finish adds
// those few sub-sums in order and, for the outer step, evaluates Lambda in fp64.
// Everything is deterministic: same inputs, same bits.
#include "co2_device.hpp"
#include "co2_launch.hpp"

namespace co2 {

__device__ __forceinline__ void acc4(double& acc, float4 q, float phi) {
  if (phi > 0.0f) {
    q.x = clip_coord(q.x, phi); q.y = clip_coord(q.y, phi);
    q.z = clip_coord(q.z, phi); q.w = clip_coord(q.w, phi);
  }
  acc += sq(q.x); acc += sq(q.y); acc += sq(q.z); acc += sq(q.w);
}

// NB buffers (1 or 2); the second has element type B1_DT (a DeltaType).
//
// One wavefront walks its tile in kNormSubs pieces of kNormSub elements.  A
// piece that lies inside the current segment is read with 16-byte loads and
// accumulated per lane; any other piece (segment boundary inside it, ragged
// end) is walked element by element, segment after segment.  Whenever the
// current segment ends, its lane sums are reduced and leave the record of
// (tile, segment); the last segment's record is written at the end of the tile.
template <int NB, int B1_DT>
__global__ __launch_bounds__(kWave) void sqnorm_partials(
    const float* __restrict__ b0, float phi0, const void* __restrict__ b1, float phi1,
    const int64_t* __restrict__ off, int S, int64_t n, SlotRec* __restrict__ slots) {
  using IO1 = DeltaIO<B1_DT>;
  const int64_t tile = blockIdx.x;
  const int64_t base = tile * kNormTile;
  const int64_t end = (base + kNormTile < n) ? base + kNormTile : n;
  const int lane = threadIdx.x;

  auto load_piece = [&](float4 (&r0)[kNormU], typename IO1::Vec (&r1)[kNormU], int64_t at) {
#pragma unroll
    for (int u = 0; u < kNormU; ++u) {
      const int64_t row = at + int64_t(u) * kWave * 4;
      r0[u] = ld4_stream(b0 + row, lane);
      if (NB == 2) r1[u] = IO1::load4(b1, row, lane);
    }
  };
  // The first piece's loads go out before the segment lookup, which does not
  // depend on them and runs while they are in flight.
  float4 q0[kNormU];
  typename IO1::Vec q1[kNormU];
  const bool first_full = base + kNormSub <= end;
  if (first_full) load_piece(q0, q1, base);
  int cur = seg_of(off, S, base);                  // off[cur] <= base < off[cur + 1]
  int64_t cur_end = off[cur + 1];
  double a0 = 0.0, a1 = 0.0;

  auto flush = [&]() {
    const double t0 = wave_sum(a0);
    double t1 = 0.0;
    if (NB == 2) t1 = wave_sum(a1);
    write_slot(slots, tile + cur, lane, t0, t1, 0.0);
    a0 = 0.0;
    a1 = 0.0;
  };
  // moves on to the segment that holds `pos` (pos < n, so one exists); empty segments are skipped
  auto advance_to = [&](int64_t pos) {
    flush();
    do {
      cur = uniform(cur + 1);
      cur_end = uniform(off[cur + 1]);
    } while (cur_end <= pos);
  };

  auto add_piece = [&](const float4 (&r0)[kNormU], const typename IO1::Vec (&r1)[kNormU]) {
#pragma unroll
    for (int u = 0; u < kNormU; ++u) {
      acc4(a0, r0[u], phi0);
      if (NB == 2) {
        acc4(a1, make_float4(IO1::get(r1[u], 0), IO1::get(r1[u], 1), IO1::get(r1[u], 2),
                             IO1::get(r1[u], 3)), phi1);
      }
    }
  };

  int64_t sb = base;                               // start of the next piece (a multiple of kNormSub)
  while (sb < end) {
    sb = uniform(sb);
    if (sb >= cur_end) advance_to(sb);
    const int64_t lim = cur_end < end ? cur_end : end;
    const int64_t run = (lim - sb) / kNormSub;     // whole pieces inside the current segment
    if (run > 0) {
      // Software pipeline over the run: the next piece's loads go out before this piece's
      // arithmetic, so the wavefront always has loads in flight.  Two register sets take
      // turns (copying one into the other would have to wait for the loads just issued).
      float4 r0[kNormU];
      typename IO1::Vec r1[kNormU];
      if (!(first_full && sb == base)) load_piece(q0, q1, sb);
      int64_t i = 1;
      for (; i + 1 < run; i += 2) {
        load_piece(r0, r1, sb + i * kNormSub);
        add_piece(q0, q1);
        load_piece(q0, q1, sb + (i + 1) * kNormSub);
        add_piece(r0, r1);
      }
      if (i < run) {
        load_piece(r0, r1, sb + i * kNormSub);
        add_piece(q0, q1);
        add_piece(r0, r1);
      } else {
        add_piece(q0, q1);
      }
      sb += run * kNormSub;
      continue;
    }
    // A piece with a segment boundary in it, or the ragged end: element by element.
    const int64_t se = (sb + kNormSub < end) ? sb + kNormSub : end;
    int64_t pos = sb;
    while (pos < se) {
      pos = uniform(pos);
      if (pos >= cur_end) advance_to(pos);
      const int64_t hi = cur_end < se ? cur_end : se;
      for (int64_t j = pos + lane; j < hi; j += kWave) {
        float v = b0[j];
        if (phi0 > 0.0f) v = clip_coord(v, phi0);
        a0 += sq(v);
        if (NB == 2) {
          float r = IO1::load1(b1, j);
          if (phi1 > 0.0f) r = clip_coord(r, phi1);
          a1 += sq(r);
        }
      }
      pos = hi;
    }
    sb = se;
  }
  flush();
}

// a += rec[t].v[col] (and b += rec[t].v[col + 1] with `two`) for t = first, first + kReduceBlock,
// ... <= last, in that order.  The records of kSlotBatch steps are loaded before the first of them
// is added, so that a thread has several loads in flight instead of one (a long segment is
// otherwise a chain of dependent memory latencies); a step beyond `last` contributes +0.0, which
// changes no sum of squares.
constexpr int kSlotBatch = 8;
__device__ __forceinline__ void add_slots(const SlotRec* __restrict__ rec, int col, bool two,
                                          int64_t first, int64_t last, double& a, double& b) {
  for (int64_t t = first; t <= last; t += int64_t(kSlotBatch) * kReduceBlock) {
    double va[kSlotBatch], vb[kSlotBatch];
#pragma unroll
    for (int u = 0; u < kSlotBatch; ++u) {
      const int64_t tt = t + int64_t(u) * kReduceBlock;
      const bool in = tt <= last;
      va[u] = in ? rec[tt].v[col] : 0.0;
      vb[u] = (in && two) ? rec[tt].v[col + 1] : 0.0;
    }
#pragma unroll
    for (int u = 0; u < kSlotBatch; ++u) {
      a += va[u];
      b += vb[u];
    }
  }
}

// Sub-sum g of `split` over segment s's slots (tiles t0..t1 of the producing
// kernel), in a fixed order.  grid = (segments, split); out[q][s*split + g].
__global__ __launch_bounds__(kReduceBlock) void slot_sums(
    const SlotRec* __restrict__ slots, int col, bool two,
    const int64_t* __restrict__ off, int S, int64_t tile_elems, int split,
    double* __restrict__ out_a, double* __restrict__ out_b) {
  __shared__ double lds[2][kReduceWaves];
  const int g = blockIdx.y;
  for (int s = blockIdx.x; s < S; s += gridDim.x) {
    const int64_t lo = off[s], hi = off[s + 1];
    double a = 0.0, b = 0.0;
    if (hi > lo) {
      const int64_t t0 = lo / tile_elems, t1 = (hi - 1) / tile_elems;
      const int64_t chunk = (t1 - t0 + split) / split;       // ceil(count / split)
      const int64_t c0 = t0 + g * chunk;
      const int64_t c1 = (c0 + chunk - 1 < t1) ? c0 + chunk - 1 : t1;
      add_slots(slots + s, col, two, c0 + threadIdx.x, c1, a, b);
    }
    const double ta = block_sum(a, lds[0]);
    double tb = 0.0;
    if (two) tb = block_sum(b, lds[1]);
    if (threadIdx.x == 0) {
      out_a[int64_t(s) * split + g] = ta;
      if (two) out_b[int64_t(s) * split + g] = tb;
    }
  }
}

__device__ __forceinline__ double add_in_order(const double* __restrict__ v, int64_t first,
                                               int count) {
  double t = v[first];
  for (int i = 1; i < count; ++i) t += v[first + i];
  return t;
}

__global__ __launch_bounds__(kReduceBlock) void totals_finish(
    const double* __restrict__ sub, int S, int split, double* __restrict__ out) {
  const int s = blockIdx.x * kReduceBlock + threadIdx.x;
  if (s < S) out[s] = add_in_order(sub, int64_t(s) * split, split);
}

// Per-segment counts (exact integers carried as doubles) to int64.
__global__ __launch_bounds__(kReduceBlock) void counts_finish(
    const double* __restrict__ sub, int S, int split, int64_t* __restrict__ out) {
  const int s = blockIdx.x * kReduceBlock + threadIdx.x;
  if (s < S) out[s] = static_cast<int64_t>(add_in_order(sub, int64_t(s) * split, split));
}

// Lambda_t per segment (Algorithm 1, gap update; Eq. 3), fp64:
//   numerator   alpha*min(sqrt(M2), cap),  M2 = sum Clip(m_{t-1},phi)^2  (cap = +inf unless
//               clipping rescales by norm: then the previous step's norm is at most phi)
//   denominator tau*first_step_norm[s], or sqrt(P2) with P2 = sum d_0^2, or none (Lambda = 1)
//   Lambda = (c == 0 || T == 0) ? 1 : (c*alpha)*numerator_norm/T + 1;  inv = (float)(1/Lambda)
__device__ __forceinline__ void lambda_of(double M2, double P2_sum, bool use_d,
                                          const float* __restrict__ first_step_norm, int s, float c,
                                          float alpha, int tau, double numer_cap, int S,
                                          double* __restrict__ seg_sq, float* __restrict__ inv,
                                          float* __restrict__ lambda_out) {
  double P2 = 0.0, T = 0.0;
  if (first_step_norm) {
    T = static_cast<double>(tau) * static_cast<double>(first_step_norm[s]);
    P2 = T * T;
  } else if (use_d) {
    P2 = P2_sum;
    T = sqrt(P2);
  }
  double moved = sqrt(M2);
  if (moved > numer_cap) moved = numer_cap;
  double Lam = 1.0;
  if (c != 0.0f && T != 0.0) {
    Lam = (static_cast<double>(c) * static_cast<double>(alpha)) * moved / T + 1.0;
  }
  seg_sq[s] = M2;
  seg_sq[S + s] = P2;
  inv[s] = static_cast<float>(1.0 / Lam);
  if (lambda_out) lambda_out[s] = static_cast<float>(Lam);
}

__global__ __launch_bounds__(kReduceBlock) void lambda_finish(
    const double* __restrict__ sub_m, const double* __restrict__ sub_d, bool use_d, int S, int split,
    const float* __restrict__ first_step_norm, float c, float alpha, int tau, double numer_cap,
    double* __restrict__ seg_sq, float* __restrict__ inv, float* __restrict__ lambda_out) {
  const int s = blockIdx.x * kReduceBlock + threadIdx.x;
  if (s >= S) return;
  const double M2 = add_in_order(sub_m, int64_t(s) * split, split);
  const double P2 = use_d ? add_in_order(sub_d, int64_t(s) * split, split) : 0.0;
  lambda_of(M2, P2, use_d, first_step_norm, s, c, alpha, tau, numer_cap, S, seg_sq, inv, lambda_out);
}

// Stage 2 in one launch, for tables whose segments span few slots: workgroup s
// adds the slots of segment s (fixed order) and evaluates Lambda itself.
__global__ __launch_bounds__(kReduceBlock) void lambda_direct(
    const SlotRec* __restrict__ slots, const int64_t* __restrict__ off, int S, int64_t tile_elems,
    bool use_d, const float* __restrict__ first_step_norm, float c, float alpha, int tau,
    double numer_cap, double* __restrict__ seg_sq, float* __restrict__ inv,
    float* __restrict__ lambda_out) {
  __shared__ double lds[2][kReduceWaves];
  for (int s = blockIdx.x; s < S; s += gridDim.x) {
    const int64_t lo = off[s], hi = off[s + 1];
    double a = 0.0, b = 0.0;
    if (hi > lo) {
      const int64_t t0 = lo / tile_elems, t1 = (hi - 1) / tile_elems;
      add_slots(slots + s, 0, use_d, t0 + threadIdx.x, t1, a, b);
    }
    const double M2 = block_sum(a, lds[0]);
    double P2 = 0.0;
    if (use_d) P2 = block_sum(b, lds[1]);
    if (threadIdx.x == 0)
      lambda_of(M2, P2, use_d, first_step_norm, s, c, alpha, tau, numer_cap, S, seg_sq, inv, lambda_out);
  }
}

// Norm-rescale clipping: scale[s] = min(1, phi/||m_t||_s) from the sub-sums of m_t^2.
__global__ __launch_bounds__(kReduceBlock) void scale_finish(
    const double* __restrict__ sub, int S, int split, float phi, float* __restrict__ scale) {
  const int s = blockIdx.x * kReduceBlock + threadIdx.x;
  if (s >= S) return;
  const double nrm = sqrt(add_in_order(sub, int64_t(s) * split, split));
  float f = 1.0f;
  if (nrm > static_cast<double>(phi)) f = static_cast<float>(static_cast<double>(phi) / nrm);
  scale[s] = f;
}

__global__ __launch_bounds__(kReduceBlock) void sqrt_to_f32(const double* __restrict__ sq_in,
                                                            float* __restrict__ out, int S) {
  const int s = blockIdx.x * kReduceBlock + threadIdx.x;
  if (s < S) out[s] = static_cast<float>(sqrt(sq_in[s]));
}

// ---------------------------------------------------------------- launches

hipError_t launch_sqnorm_partials(int nb, const float* b0, float phi0, const void* b1,
                                  float phi1, int b1_dtype, const int64_t* off_dev, int S,
                                  int64_t n, SlotRec* slots, hipStream_t st) {
  const dim3 grid(static_cast<unsigned>((n + kNormTile - 1) / kNormTile)), block(kWave);
  const unsigned lds = throttle_lds_bytes(nb == 2 ? kNormWavesTwoBuffers : kNormWavesOneBuffer);
  if (nb == 2 && b1_dtype == kDeltaBF16) {
    hipLaunchKernelGGL((sqnorm_partials<2, kDeltaBF16>), grid, block, lds, st, b0, phi0, b1, phi1,
                       off_dev, S, n, slots);
  } else if (nb == 2 && b1_dtype == kDeltaF16) {
    hipLaunchKernelGGL((sqnorm_partials<2, kDeltaF16>), grid, block, lds, st, b0, phi0, b1, phi1,
                       off_dev, S, n, slots);
  } else if (nb == 2) {
    hipLaunchKernelGGL((sqnorm_partials<2, kDeltaF32>), grid, block, lds, st, b0, phi0, b1, phi1,
                       off_dev, S, n, slots);
  } else {
    hipLaunchKernelGGL((sqnorm_partials<1, kDeltaF32>), grid, block, lds, st, b0, phi0,
                       static_cast<const void*>(b0), 0.0f, off_dev, S, n, slots);
  }
  return hipGetLastError();
}

hipError_t launch_slot_sums(const SlotRec* slots, int col, bool two, const int64_t* off_dev,
                            int S, int64_t tile_elems, int split, double* out_a, double* out_b,
                            hipStream_t st) {
  const dim3 grid(static_cast<unsigned>(S < 32768 ? S : 32768), static_cast<unsigned>(split));
  hipLaunchKernelGGL(slot_sums, grid, dim3(kReduceBlock), 0, st, slots, col, two, off_dev, S,
                     tile_elems, split, out_a, out_b);
  return hipGetLastError();
}

hipError_t launch_totals_finish(const double* sub, int S, int split, double* out,
                                hipStream_t st) {
  hipLaunchKernelGGL(totals_finish, dim3((S + kReduceBlock - 1) / kReduceBlock),
                     dim3(kReduceBlock), 0, st, sub, S, split, out);
  return hipGetLastError();
}

hipError_t launch_counts_finish(const double* sub, int S, int split, int64_t* out,
                                hipStream_t st) {
  hipLaunchKernelGGL(counts_finish, dim3((S + kReduceBlock - 1) / kReduceBlock),
                     dim3(kReduceBlock), 0, st, sub, S, split, out);
  return hipGetLastError();
}

hipError_t launch_lambda_finish(const double* sub_m, const double* sub_d, bool use_d, int S, int split,
                                const float* first_step_norm, float c, float alpha, int tau,
                                double numer_cap, double* seg_sq, float* inv, float* lambda_out,
                                hipStream_t st) {
  hipLaunchKernelGGL(lambda_finish, dim3((S + kReduceBlock - 1) / kReduceBlock),
                     dim3(kReduceBlock), 0, st, sub_m, sub_d, use_d, S, split, first_step_norm, c,
                     alpha, tau, numer_cap, seg_sq, inv, lambda_out);
  return hipGetLastError();
}

hipError_t launch_lambda_direct(const SlotRec* slots, const int64_t* off_dev, int S, int64_t tile_elems,
                                bool use_d, const float* first_step_norm, float c, float alpha, int tau,
                                double numer_cap, double* seg_sq, float* inv, float* lambda_out,
                                hipStream_t st) {
  hipLaunchKernelGGL(lambda_direct, dim3(static_cast<unsigned>(S < 32768 ? S : 32768)),
                     dim3(kReduceBlock), 0, st, slots, off_dev, S, tile_elems, use_d, first_step_norm,
                     c, alpha, tau, numer_cap, seg_sq, inv, lambda_out);
  return hipGetLastError();
}

hipError_t launch_scale_finish(const double* sub, int S, int split, float phi, float* scale,
                               hipStream_t st) {
  hipLaunchKernelGGL(scale_finish, dim3((S + kReduceBlock - 1) / kReduceBlock), dim3(kReduceBlock), 0,
                     st, sub, S, split, phi, scale);
  return hipGetLastError();
}

hipError_t launch_sqrt_to_f32(const double* sq_in, float* out, int S, hipStream_t st) {
  hipLaunchKernelGGL(sqrt_to_f32, dim3((S + kReduceBlock - 1) / kReduceBlock),
                     dim3(kReduceBlock), 0, st, sq_in, out, S);
  return hipGetLastError();
}

}  // namespace co2
