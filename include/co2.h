/* co2.h -- C ABI of the MI355X (gfx950) CO2 outer-update library (libco2.so).
 *
 * One data-parallel worker of CO2 (Sun et al., "CO2: Efficient Distributed
 * Training with Full Communication-Computation Overlap") runs, once per outer
 * round t and after its tau local steps, the update of Algorithm 1:
 *
 *     Lambda_t = ||x_{t,0} - x_{t-1,0}|| / (tau ||x_{t-1,1} - x_{t-1,0}||) + 1     (Def. 3.1, Eq. 3)
 *     m_t      = beta m_{t-1} + (1/Lambda_t) (x_{t-1,0} - x_{t-1,tau})            (Sec. 3.2)
 *     x_{t+1,0}= x_{t,0} - alpha Clip(m_t, phi),  Clip = max{-phi, min{., phi}}   (Sec. 3.3)
 *
 * where x_{t-1,tau} is the average over the workers delivered by the previous
 * round's asynchronous all-reduce.  On one GPU that average is taken inside the
 * kernel over K device buffers holding the workers' pseudo-gradients
 * x_{t-1,0} - x^{(k)}_{t-1,tau}.  All buffers are flat fp32 vectors of n elements;
 * a segment table (one segment per parameter tensor) says over which index
 * ranges the two norms of Eq. 3 are taken.
 *
 * Conventions
 *   - Pointers marked DEVICE point to GPU memory owned by the caller; pointers
 *     marked HOST point to ordinary host memory.  Nothing declared in this
 *     header allocates (the optional memory-layout service that does is in
 *     co2_layout.h), reads the environment or keeps state between calls
 *     (co2_outer_step_static alone works in a scratch array of the library's
 *     own), and nothing synchronises: every call
 *     validates its arguments on the host, enqueues kernels on `hip_stream`
 *     (a hipStream_t; NULL = the null stream) and returns.  The launches hold
 *     no memset and no host callback, so a caller may capture them into a HIP
 *     graph (leave the timing events of co2_params NULL then): `step` only
 *     tells the first round from the later ones, so two captured steady-state
 *     rounds -- the two halves of a delta_out ping-pong -- can be replayed for
 *     the rest of a run (one captured round suffices when delta_out is
 *     deltas[0] itself).
 *   - Every DEVICE buffer must be 16-byte aligned.  Layout advice: the sweep
 *     streams all flat buffers of one worker (params, anchor, momentum, the K
 *     pseudo-gradient buffers, delta_out) in lock step, and on MI355X its
 *     duration depends on which physical pages lie behind them, by up to 10 %
 *     between otherwise identical plain allocations (fixed for an allocation's
 *     life).  A buffer set of co2_layout.h with its default 64 MiB pieces has
 *     measured fast every time (84 % of the HBM peak at K = 4 ... 16, where
 *     plain allocations gave 77-84 %); failing that, carve the buffers out of
 *     ONE device allocation, 4 KiB aligned (2-5 % faster than scattered
 *     buffers), and a long-running caller can time the sweep on a few
 *     candidate allocations held together and keep the fastest.  On a device
 *     that the process has to itself and whose memory has been through many
 *     allocate/free cycles it also pays to allocate nearly all free memory in
 *     one piece and free it again first (the driver then merges its free
 *     blocks; never do this on a device shared with other processes).
 *   - Return value: CO2_OK or a negative error code.  Arguments are checked
 *     before the first launch: on CO2_EINVAL or CO2_EWORKSPACE nothing has
 *     been enqueued and no buffer has been touched.  CO2_EHIP reports a HIP
 *     call of the launch sequence that failed; launches enqueued before it
 *     still run.  No exceptions, no aborts.
 *   - All fp32 arithmetic is unfused (no FMA contraction) and evaluated in the
 *     order documented per call, so results are reproducible bit for bit.
 */
#ifndef CO2_H_
#define CO2_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define CO2_MAX_K 16            /* most worker buffers one call can average   */
#define CO2_MAX_NORM_BUFS 32    /* most buffers one co2_pseudo_grad_norms call */

enum {
  CO2_OK = 0,
  CO2_EINVAL = -1,      /* bad argument (NULL, range, alignment, aliasing)  */
  CO2_EWORKSPACE = -2,  /* workspace NULL or smaller than co2_workspace_bytes */
  CO2_EHIP = -3,        /* a HIP call failed (a launch; an allocation in
                           co2_layout.h's calls); see co2_last_hip_error()   */
  CO2_ESCRATCH = -4     /* co2_outer_step_static: the sizes need more scratch than
                           CO2_STATIC_SCRATCH_BYTES                          */
};

/* Bits of co2_params.flags */
#define CO2_FLAG_NONE 0u
/* Steady-state single pass: take this round's two sums of squares (clipped
 * m_{t-1} and deltas[0]) from the partial sums the PREVIOUS co2_outer_step on
 * the same workspace left there while it wrote m_{t-1} and delta_out, instead
 * of re-reading both vectors.  The caller promises that since that call the
 * momentum buffer is unchanged, deltas[0] holds exactly the delta_out it wrote,
 * and n, the segment table and clip_phi are the same.  Results are identical to
 * the two-pass form up to the summation order of the fp64 norms. */
#define CO2_FLAG_CARRIED_NORMS 1u
/* Variants of the outer rule (the family CO2 is built on or compared with).
 * They combine freely with each other and with the penalty and the clipping;
 * only the fp32 entry points (co2_outer_step, co2_outer_step_static) take them.
 *
 * CO2_FLAG_CURRENT_ROUND: the momentum line in the order of Section 3.2's
 *   recursion m_{t+1} = beta m_t + (x_{t,0} - x_{t,tau}) before the staleness is
 *   introduced: the mean is taken over THIS round's pseudo-gradients, the
 *   worker's own anchor - params (formed in this call) first, then
 *   deltas[1..K-1], which must hold the peers' pseudo-gradients of this round.
 *   deltas[0] is not read (may be NULL).  Round 0 is an ordinary round.  With
 *   penalty_c = 0 and clip_phi = +INF this is the slow-momentum update.  Needs
 *   params; a penalty (penalty_c != 0) needs first_step_norm.
 * CO2_FLAG_ANCHOR_PULL: the local parameters do not restart from the new outer
 *   iterate but are pulled towards it, params = x - pull_rho*(x - x_{t+1,0})
 *   (the anchor-model rule of the overlap variant of local SGD discussed in the
 *   paper's Discussions section); anchor_out still receives x_{t+1,0}.  Needs
 *   params; pull_rho in (0,1], 1 being the plain restart.
 * CO2_FLAG_NORM_CLIP: clipping by rescaling instead of Section 3.3's coordinate-
 *   wise clamp (not in the paper): per segment Clip_norm(m, phi) = m*min(1,
 *   phi/||m||_s), and Eq. 3's numerator ||x_{t,0} - x_{t-1,0}||_s becomes
 *   alpha*min(||m_{t-1}||_s, phi).  The outer iterate needs ||m_t||_s, so it is
 *   written by a second, lighter kernel (36+4K instead of 28+4K bytes per
 *   coordinate).  clipped_out is not available. */
#define CO2_FLAG_CURRENT_ROUND 2u
#define CO2_FLAG_ANCHOR_PULL 4u
#define CO2_FLAG_NORM_CLIP 8u

/* Hyper-parameters and shape of one outer update (Algorithm 1's inputs).
 * Passed by pointer, read on the host only. */
typedef struct co2_params {
  int64_t n;                  /* elements in every flat buffer (this GPU's shard), >= 1 */
  int32_t S;                  /* number of segments, >= 1                          */
  int32_t K;                  /* workers whose pseudo-gradients are averaged, 1..CO2_MAX_K */
  const int64_t* seg_off;     /* HOST, S+1 entries: seg_off[0]=0, seg_off[S]=n, non-decreasing.
                                 Segment s is [seg_off[s], seg_off[s+1]); may be empty. */
  const int64_t* seg_off_dev; /* DEVICE copy of the same S+1 values (caller uploads once) */
  float alpha;                /* outer learning rate alpha, finite                 */
  float beta;                 /* outer momentum factor beta, in [0,1)              */
  float clip_phi;             /* clipping threshold phi > 0; +INF disables clipping */
  float penalty_c;            /* c >= 0 scaling the ratio in Eq. 3: Lambda = c*ratio + 1.
                                 1 = the paper; 0 = its "w/o penalty" ablation      */
  int32_t tau;                /* inner steps per round, >= 1                       */
  uint32_t flags;             /* CO2_FLAG_*                                        */
  int64_t step;               /* outer round index t >= 0.  t = 0 is the first round, in
                                 which only the pseudo-gradient is formed (Sec. 3.1) */
  void* ev_sweep_begin;       /* optional hipEvent_t recorded on the stream right before */
  void* ev_sweep_end;         /* / right after the fused sweep kernel (timing only)      */
  int64_t* clipped_out;       /* optional DEVICE int64[S]: per segment, the number of coordinates
                                 with |m_t| > phi, i.e. clamped in the outer iterate (0 at
                                 step 0).  Costs two small extra launches when set.       */
  float pull_rho;             /* CO2_FLAG_ANCHOR_PULL: rho in (0,1]; ignored otherwise     */
  int32_t sweep_waves_per_cu; /* tuning: resident wavefronts per compute unit the sweep kernel
                                 is capped to; 0 = the library's measured default (5..8 by K),
                                 which was also the fastest beside another bandwidth-bound
                                 kernel on a second stream.  Range 0..32.                 */
} co2_params;

/* Bytes of DEVICE workspace the calls below need for these sizes (256-byte
 * aligned regions: per-tile partial sums, per-segment sums, 1/Lambda).  Returns
 * 0 for invalid sizes. */
size_t co2_workspace_bytes(int64_t n, int32_t S, int32_t K);

/* One outer update of Algorithm 1 (gap, momentum and outer-iterate lines) for
 * round p->step, plus the pseudo-gradient x_{t,0} - x^{(i)}_{t,tau} that the
 * all-reduce launched in the same round carries.
 *
 *   params      DEVICE fp32[n]. in: x^{(i)}_{t,tau}; out: x_{t+1,0}.  May be NULL
 *               ("split form" for the side stream: only m_t and the next anchor
 *               are produced); then delta_out must be NULL too.
 *   anchor      DEVICE fp32[n]. in: x_{t,0}.
 *   anchor_out  DEVICE fp32[n]. out: x_{t+1,0}.  Either == anchor (in place) or a
 *               disjoint buffer (anchor is then left untouched).
 *   momentum    DEVICE fp32[n]. in: m_{t-1}; out: m_t.
 *   deltas      HOST array of K DEVICE fp32[n] pointers: round t-1's
 *               pseudo-gradients of the K workers; deltas[0] is this worker's own.
 *               Ignored (may be NULL) when p->step == 0.
 *   delta_out   DEVICE fp32[n]. out: anchor - params, taken before either changes.
 *   first_step_norm  DEVICE fp32[S] or NULL: ||x_{t-1,1} - x_{t-1,0}||_s, the norm
 *               of the first inner step of the previous round per segment.  The
 *               denominator of Eq. 3 is tau times it.  NULL: the denominator is
 *               ||deltas[0]||_s (own previous pseudo-gradient, which equals
 *               tau*||first step|| when the tau inner steps are equal).
 *   lambda_out  DEVICE fp32[S] or NULL: receives Lambda_t per segment.
 *   workspace   DEVICE, >= co2_workspace_bytes(n,S,K) bytes, 256-byte aligned.
 *
 * Arithmetic per coordinate j of segment s, fp32, each operation rounded once:
 *   delta_out[j] = anchor[j] - params[j]
 *   dbar   = (((d_0[j] + d_1[j]) + d_2[j]) + ... + d_{K-1}[j]) * (float)(1.0/K)
 *   m'     = beta*momentum[j] + dbar*inv[s]
 *   x'     = anchor[j] - alpha*Clip(m', phi)
 *   momentum[j] = m';  params[j] = anchor_out[j] = x'
 * and per segment, fp64:
 *   M2 = sum_j Clip(momentum_in[j], phi)^2 ;  T = tau*first_step_norm[s] or sqrt(sum_j d_0[j]^2)
 *   Lambda = (c == 0 || T == 0) ? 1 : (c*alpha)*sqrt(M2)/T + 1 ;  inv[s] = (float)(1/Lambda)
 * (x_{t,0} - x_{t-1,0} = -alpha*Clip(m_{t-1},phi) by the outer-iterate line one round
 * earlier, which is why the numerator is read from the momentum buffer.)
 * step == 0: delta_out = anchor - params; params = anchor_out = anchor; momentum
 * is only read (its clipped sum of squares is left in the workspace for round 1).
 *
 * With CO2_FLAG_* variants (see the flags): dbar leads with the worker's own
 * anchor[j] - params[j] and continues over deltas[1..K-1] (CURRENT_ROUND);
 * params[j] = x - pull_rho*(x - x') with x the incoming params[j] (ANCHOR_PULL);
 * per segment scale = (||m'||_s > phi) ? (float)(phi/||m'||_s) : 1 in fp64 and
 * x' = anchor[j] - alpha*(m'*scale), M2 = sum_j momentum_in[j]^2 and the
 * numerator of Lambda is alpha*min(sqrt(M2), phi) (NORM_CLIP).
 *
 * Buffers must not overlap, with two exceptions: anchor_out == anchor, and
 * delta_out == deltas[0] (the worker's own pseudo-gradient replaced in place,
 * one buffer instead of a ping-pong pair: each coordinate's old value is read
 * before the new one is stored).  No other output, small or large, may overlap
 * any other argument or the workspace.  Errors: CO2_EINVAL
 * for NULL/misaligned/overlapping buffers, n<1, S<1, K outside 1..CO2_MAX_K, a
 * bad segment table, beta outside [0,1), phi<=0 or NaN, c<0, tau<1, step<0,
 * non-finite alpha, unknown or inconsistent flags, pull_rho outside (0,1],
 * sweep_waves_per_cu outside 0..32; CO2_EWORKSPACE; CO2_EHIP. */
int co2_outer_step(const co2_params* p,
                   float* params, const float* anchor, float* anchor_out,
                   float* momentum, const float* const* deltas, float* delta_out,
                   const float* first_step_norm, float* lambda_out,
                   void* workspace, size_t workspace_bytes, void* hip_stream);

/* co2_outer_step for callers that cannot allocate device memory and have no
 * workspace to pass: code under HIP graph capture, tight serving-style loops,
 * harnesses that forbid hipMalloc.  Same arguments, arithmetic, flags and
 * results (bit for bit) as co2_outer_step, minus the workspace: the per-tile
 * partial sums, per-segment sums and 1/Lambda live in a scratch array of
 * CO2_STATIC_SCRATCH_BYTES that is part of the library's device image (one
 * copy per GPU, occupied on every GPU the library is used on until the process
 * ends).  The call itself never calls hipMalloc, hipFree or any allocating
 * routine; the first call made on a GPU looks up that GPU's copy of the array
 * (make that call outside a graph capture), later calls only enqueue kernels.
 *
 *   - Limit: co2_workspace_bytes(p->n, p->S, p->K) <= CO2_STATIC_SCRATCH_BYTES
 *     (about 1.3e8 elements with a few hundred segments); beyond it the call
 *     returns CO2_ESCRATCH before anything is enqueued.
 *   - The GPU that hip_stream belongs to must be the current device.
 *   - All calls on one GPU share that GPU's array, which keeps what the last
 *     call left in it.  Nothing in it has to start at zero (every record a
 *     round reads is written earlier in the same round or, with
 *     CO2_FLAG_CARRIED_NORMS, by the previous call), so the library clears
 *     nothing.  Consequences: calls that may run at the same time on one GPU
 *     (different streams without ordering between them) race on the array and
 *     must be serialised by the caller; CO2_FLAG_CARRIED_NORMS is only valid
 *     if the previous call of this entry point on this GPU was the previous
 *     round of the same problem.
 * Errors: as co2_outer_step (no CO2_EWORKSPACE), plus CO2_ESCRATCH. */
#define CO2_STATIC_SCRATCH_BYTES (32u << 20)
int co2_outer_step_static(const co2_params* p,
                          float* params, const float* anchor, float* anchor_out,
                          float* momentum, const float* const* deltas, float* delta_out,
                          const float* first_step_norm, float* lambda_out,
                          void* hip_stream);

/* The same update with the pseudo-gradients transported in bf16 (the paper's
 * Section 2, "Efficient Communication": compression of what the all-reduce
 * carries is orthogonal to CO2 and can be combined with it).  Differences from
 * co2_outer_step:
 *   deltas_bf16     HOST array of K DEVICE uint16[n] pointers, bf16 bit patterns,
 *                   widened exactly to fp32 before the (fp32) mean;
 *   delta_out_bf16  DEVICE uint16[n]: bf16(anchor - params), the fp32 difference
 *                   rounded once to nearest-even; the sum of squares carried to
 *                   the next round is taken over these rounded values.
 * Everything else (arithmetic order, Lambda, flags, errors) is unchanged.  26+2K
 * bytes per coordinate instead of 28+4K.  Carried sums (CO2_FLAG_CARRIED_NORMS)
 * must come from a previous call of this same entry point. */
int co2_outer_step_bf16(const co2_params* p,
                        float* params, const float* anchor, float* anchor_out,
                        float* momentum, const uint16_t* const* deltas_bf16,
                        uint16_t* delta_out_bf16,
                        const float* first_step_norm, float* lambda_out,
                        void* workspace, size_t workspace_bytes, void* hip_stream);

/* As co2_outer_step_bf16 with IEEE fp16 bit patterns (round to nearest even,
 * gradual underflow, overflow to infinity): 11 bits of significand instead of
 * 8, but pseudo-gradient coordinates below 6e-8 in magnitude vanish and those
 * below 6.1e-5 lose precision gradually. */
int co2_outer_step_f16(const co2_params* p,
                       float* params, const float* anchor, float* anchor_out,
                       float* momentum, const uint16_t* const* deltas_f16,
                       uint16_t* delta_out_f16,
                       const float* first_step_norm, float* lambda_out,
                       void* workspace, size_t workspace_bytes, void* hip_stream);

/* Segmented sums of squares (the quantities under the roots of Eq. 3's norms).
 * Uses p->n, p->S, p->seg_off, p->seg_off_dev and p->clip_phi only.
 *
 *   bufs        HOST array of nbuf DEVICE fp32[n] pointers, 0 <= nbuf <= CO2_MAX_NORM_BUFS.
 *   momentum    DEVICE fp32[n] or NULL.  If given, one more row is produced:
 *               sum_j Clip(momentum[j], phi)^2 (Eq. 3's numerator over alpha^2).
 *   sqnorm_out  DEVICE fp64[(nbuf + (momentum?1:0)) * S], row-major [buffer][segment];
 *               the momentum row is last.  Sums of squares, not roots, so that
 *               shards of one tensor can be added before the root is taken.
 * fp64 accumulation in a fixed order: results are deterministic, and equal to
 * an ascending-index fp64 sum up to fp64 rounding.  The call works in a part of
 * the workspace of its own: sums that a previous co2_outer_step left there for
 * CO2_FLAG_CARRIED_NORMS stay valid.  Errors as above. */
int co2_pseudo_grad_norms(const co2_params* p, const float* const* bufs, int32_t nbuf,
                          const float* momentum, double* sqnorm_out,
                          void* workspace, size_t workspace_bytes, void* hip_stream);

/* One local update (Algorithm 1, "LU") with AdamW (decoupled weight decay) as
 * the base optimizer, fp32 master weights and bf16 gradients, for the inner
 * step with 1-based index adam_step:
 *   g  = bf16 -> fp32 (exact)
 *   m1 = beta1*exp_avg + (1-beta1)*g ;  v = beta2*exp_avg_sq + ((1-beta2)*g)*g
 *   p' = p_in*(1 - lr*wd) - (float)(lr/(1-beta1^k)) * (m1 / (sqrt(v)/(float)sqrt(1-beta2^k) + eps))
 * every fp32 operation rounded once (IEEE sqrt and division).
 *
 *   p_in, p_out DEVICE fp32[n]; p_out may equal p_in.  p_out may be NULL if delta_out
 *               is given: p' is then only used to form delta_out (the last local
 *               step of a round whose parameters restart from the next anchor
 *               need not store x_{t,tau}: 30 bytes per coordinate instead of 34).
 *   grad_bf16   DEVICE uint16[n] (bf16 bit patterns).
 *   exp_avg, exp_avg_sq  DEVICE fp32[n], updated in place.
 *   anchor, delta_out    both NULL, or DEVICE fp32[n]: delta_out = anchor - p'
 *               (the round's pseudo-gradient, fused into the last inner step).
 *   seg_off_dev, S, step_sq_out: all unset (NULL,0,NULL) or DEVICE int64[S+1],
 *               S >= 1 and DEVICE fp64[S]: step_sq_out[s] = sum_{j in s} (p' - p_in)^2,
 *               whose root at the first inner step of a round is Eq. 3's
 *               ||x_{t,1} - x_{t,0}||_s.  Needs seg_off (HOST) for validation.
 *   workspace   needed only with step_sq_out (co2_workspace_bytes(n,S,1)).
 */
int co2_inner_adamw(int64_t n, const float* p_in, float* p_out,
                    const uint16_t* grad_bf16, float* exp_avg, float* exp_avg_sq,
                    float lr, float beta1, float beta2, float eps, float weight_decay,
                    int64_t adam_step,
                    const float* anchor, float* delta_out,
                    const int64_t* seg_off, const int64_t* seg_off_dev, int32_t S,
                    double* step_sq_out,
                    void* workspace, size_t workspace_bytes, void* hip_stream);

/* Square roots of S fp64 sums, written as fp32 (turns step_sq_out into the
 * first_step_norm argument of co2_outer_step without leaving the stream).
 *   sq DEVICE fp64[S]; out DEVICE fp32[S]. */
int co2_sqrt_to_f32(const double* sq, float* out, int32_t S, void* hip_stream);

/* Plain device-to-device copy kernel (n fp32 elements, 16-byte vectors), the
 * yardstick for attainable HBM bandwidth and for calibrating byte counters.
 * Moves 8 bytes per element. */
int co2_copy_f32(const float* src, float* dst, int64_t n, void* hip_stream);

/* Text for an error code (static string, never NULL). */
const char* co2_strerror(int code);

/* hipError_t value of the most recent failed HIP call in this thread (0 if none). */
int co2_last_hip_error(void);

#ifdef __cplusplus
}
#endif
#endif /* CO2_H_ */
