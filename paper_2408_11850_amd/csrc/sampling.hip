// Fused logits -> probability kernels (gfx950): the draft's draw x_i ~ q_i and the target's
// accept / reject with residual resampling (paper Section 2, Eq. (1); Algorithm 2).
//
// A distribution is softmax(mult * logits) in fp32 (mult = logit_scale / temperature), or the
// one-hot at the arg-max (lowest id on ties) for greedy decoding.  A draw is an inverse-CDF walk in
// ascending token id with one uniform u: the first k whose running sum (fp64) exceeds u * total.
// The acceptance test is evaluated without a division, in fp64: accept iff r * q[x] <= p[x].
// One workgroup of 1024 threads handles one vocabulary row.  With a single compute unit per row the kernels are
// bound by its vector ALU and by the latency of dependent passes, so rows of up to 32768 ids are held in
// registers and read once (the reg_* functions); longer rows take the generic multi-pass kernels.
#include <cstring>

#include "spec_internal.h"

#define SAMP_THREADS 1024
#define SAMP_WAVES (SAMP_THREADS / 64)

struct MaxIdx { float v; int i; };

__device__ __forceinline__ MaxIdx better(MaxIdx a, MaxIdx b) {
  // larger value wins; on equal values the lower index wins
  if (b.v > a.v || (b.v == a.v && b.i < a.i)) return b;
  return a;
}

__device__ MaxIdx block_argmax(MaxIdx m, MaxIdx* sh) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) {
    MaxIdx t;
    t.v = __shfl_xor(m.v, o);
    t.i = __shfl_xor(m.i, o);
    m = better(m, t);
  }
  const int w = threadIdx.x >> 6;
  if ((threadIdx.x & 63) == 0) sh[w] = m;
  __syncthreads();
  MaxIdx r = sh[0];
  for (int i = 1; i < SAMP_WAVES; ++i) r = better(r, sh[i]);
  __syncthreads();
  return r;
}

__device__ double block_sum_d(double v, double* sh) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o);
  const int w = threadIdx.x >> 6;
  if ((threadIdx.x & 63) == 0) sh[w] = v;
  __syncthreads();
  double r = 0.0;
  for (int i = 0; i < SAMP_WAVES; ++i) r += sh[i];
  __syncthreads();
  return r;
}

// Row statistics: arg-max of the logits and sum_j exp(mult*(l_j - max)).
__device__ void row_stats(const float* __restrict__ logits, int V, float mult, MaxIdx* shm, double* shd,
                          MaxIdx& top, float& sum) {
  MaxIdx m;
  m.v = -INFINITY; m.i = 0x7fffffff;
  for (int j = threadIdx.x; j < V; j += SAMP_THREADS) {
    MaxIdx t; t.v = logits[j]; t.i = j;
    m = better(m, t);
  }
  top = block_argmax(m, shm);
  float acc = 0.f;
  const float zmax = top.v * mult;
  for (int j = threadIdx.x; j < V; j += SAMP_THREADS) acc += expf(logits[j] * mult - zmax);
  sum = (float)block_sum_d((double)acc, shd);
}

// Inverse-CDF draw from the non-negative weights w[0..V) (device memory, fp32) with uniform u.
// Thread t owns the contiguous ids [t*C, (t+1)*C).  Returns the token to every thread.
__device__ int block_inverse_cdf(const float* __restrict__ w, int V, float u, double* shd, int* shi, double* total_out) {
  const int C = (V + SAMP_THREADS - 1) / SAMP_THREADS;
  const int b = threadIdx.x * C;
  int e = b + C;
  if (e > V) e = V;
  double local = 0.0;
  for (int j = b; j < e; ++j) local += (double)w[j];
  // inclusive scan over threads: wave scan, then scan of the wave totals
  double incl = local;
#pragma unroll
  for (int o = 1; o < 64; o <<= 1) {
    double t = __shfl_up(incl, o);
    if ((threadIdx.x & 63) >= o) incl += t;
  }
  const int wv = threadIdx.x >> 6;
  if ((threadIdx.x & 63) == 63) shd[wv] = incl;
  if (threadIdx.x == 0) shi[0] = 0x7fffffff;
  __syncthreads();
  double base = 0.0, total = 0.0;
  for (int i = 0; i < SAMP_WAVES; ++i) {
    if (i < wv) base += shd[i];
    total += shd[i];
  }
  incl += base;
  const double target = (double)u * total;
  if (incl > target && local > 0.0) atomicMin(&shi[0], (int)threadIdx.x);
  __syncthreads();
  const int owner = shi[0];
  __syncthreads();
  if ((int)threadIdx.x == owner) {
    double run = incl - local;
    int k = -1, lastpos = -1;
    for (int j = b; j < e; ++j) {
      const double wj = (double)w[j];
      run += wj;
      if (wj > 0.0) lastpos = j;
      if (run > target && wj > 0.0) { k = j; break; }
    }
    shi[1] = k >= 0 ? k : lastpos;
  }
  __syncthreads();
  int tok = shi[1];
  if (owner == 0x7fffffff) tok = -1;   // no mass at all
  if (total_out) *total_out = total;
  __syncthreads();
  return tok;
}

// ---- draft: q = softmax(mult*logits), x = invCDF(q, u) -------------------------------------
__global__ __launch_bounds__(SAMP_THREADS) void sample_row_kernel(const float* __restrict__ logits, int V, float mult,
                                                                  int greedy, float u, float* __restrict__ q_out,
                                                                  int* __restrict__ tok_out) {
  __shared__ MaxIdx shm[SAMP_WAVES];
  __shared__ double shd[SAMP_WAVES];
  __shared__ int shi[2];
  MaxIdx top;
  float sum;
  if (greedy) {
    MaxIdx m;
    m.v = -INFINITY; m.i = 0x7fffffff;
    for (int j = threadIdx.x; j < V; j += SAMP_THREADS) {
      MaxIdx t; t.v = logits[j]; t.i = j;
      m = better(m, t);
    }
    top = block_argmax(m, shm);
    for (int j = threadIdx.x; j < V; j += SAMP_THREADS) q_out[j] = (j == top.i) ? 1.0f : 0.0f;
    if (threadIdx.x == 0) tok_out[0] = top.i;
    return;
  }
  row_stats(logits, V, mult, shm, shd, top, sum);
  const float zmax = top.v * mult;
  for (int j = threadIdx.x; j < V; j += SAMP_THREADS) q_out[j] = expf(logits[j] * mult - zmax) / sum;
  __threadfence_block();
  __syncthreads();
  const int tok = block_inverse_cdf(q_out, V, u, shd, shi, nullptr);
  if (threadIdx.x == 0) tok_out[0] = tok;
}

// The same draw for vocabularies of up to 32768 ids with the row held in registers: wave w owns the ids
// [w R 64, (w+1) R 64) (R = rows of 64 ids per wave), lane l of it the ids w R 64 + 64 k + l, so every load and
// store is a coalesced 256-byte run and the logits are read once.  The inverse-CDF walk is three nested searches
// in ascending id order, all sums in fp64: wave (scan of the 16 wave totals), row of 64 ids (scan of the wave's
// row totals), lane (scan of the row).  The row totals come from one transposing butterfly (32 exchanges for 32
// rows instead of 6 per row): each exchange halves the rows a lane still carries.
#define SAMP_ROWS_MAX 32
__device__ __forceinline__ double scan_up_d(double v, int lane, int width) {
#pragma unroll
  for (int o = 1; o < 64; o <<= 1) {
    const double t = __shfl_up(v, o);
    if (o < width && lane >= o) v += t;
  }
  return v;
}
struct RegGeom {          // which ids a thread owns: row0 + 64 k + lane, k < R
  int R, w, lane, row0, j0;
};
__device__ __forceinline__ RegGeom reg_geom(int V) {
  RegGeom g;
  g.R = (V + SAMP_THREADS - 1) / SAMP_THREADS;
  g.w = threadIdx.x >> 6;
  g.lane = threadIdx.x & 63;
  g.row0 = g.w * g.R * 64;
  g.j0 = g.row0 + g.lane;
  return g;
}
// probability of a logit given the row's statistics: hardware exp2 (1 ulp) of a product rounded once, times the
// reciprocal of the sum: relative error below 1e-5 for exponents down to -100, two orders under what the bf16
// logits carry.  Every kernel of the register path forms p and q with this one expression.
__device__ __forceinline__ float reg_prob(float l, float mult, float zmax, float inv) { return __expf(l * mult - zmax) * inv; }

// Loads the row once; returns the arg-max, sum_j exp(mult l_j - zmax) and e[k] = exp(mult l - zmax) (0 outside V).
__device__ __forceinline__ void reg_softmax(const float* __restrict__ row, int V, float mult, const RegGeom& g,
                                            float (&e)[SAMP_ROWS_MAX], MaxIdx& top, float& sum, MaxIdx* shm,
                                            double* shd) {
  MaxIdx m;
  m.v = -INFINITY; m.i = 0x7fffffff;
#pragma unroll
  for (int k = 0; k < SAMP_ROWS_MAX; ++k) {
    const int j = g.j0 + 64 * k;
    const bool in = k < g.R && j < V;
    e[k] = in ? row[j] : -INFINITY;
    if (in && e[k] > m.v) { m.v = e[k]; m.i = j; }   // ids ascend with k: a strict test keeps the lowest id on ties
  }
  top = block_argmax(m, shm);
  const float zmax = top.v * mult;
  float acc = 0.f;
#pragma unroll
  for (int k = 0; k < SAMP_ROWS_MAX; ++k) {
    const int j = g.j0 + 64 * k;
    e[k] = (k < g.R && j < V) ? __expf(e[k] * mult - zmax) : 0.f;
    acc += e[k];
  }
  sum = (float)block_sum_d((double)acc, shd);
}

// Inverse-CDF draw over the non-negative weights e[] (0 outside V).  Returns the id to every thread, -1 if the
// weights have no mass; *total_out = their fp64 sum.  rt: [SAMP_WAVES][SAMP_ROWS_MAX + 1] doubles, shi: 1 int.
// Every thread of the workgroup must call it (two barriers inside).
__device__ __forceinline__ int reg_draw(const float (&e)[SAMP_ROWS_MAX], const RegGeom& g, float u,
                                        double (*rt)[SAMP_ROWS_MAX + 1], int* shi, double* total_out) {
  const int lane = g.lane, w = g.w;
  // transposing butterfly: after the exchange over lane bit b a lane carries half of its rows, summed over both
  // partners; after bits 5..1 it carries row (lane >> 1), after bit 0 both lanes of a pair hold that row's total
  double a[SAMP_ROWS_MAX / 2];
  {
    const bool hi = (lane & 32) != 0;
#pragma unroll
    for (int i = 0; i < SAMP_ROWS_MAX / 2; ++i) {
      const float x = e[i], y = e[i + SAMP_ROWS_MAX / 2];
      asm volatile("" ::"v"(x), "v"(y));        // a second use keeps the choice a select of values, not of indices
      const double send = (double)(hi ? x : y);
      const double keep = (double)(hi ? y : x);
      a[i] = keep + __shfl_xor(send, 32);
    }
  }
#pragma unroll
  for (int half = SAMP_ROWS_MAX / 4, off = 16; half >= 1; half >>= 1, off >>= 1) {
    const bool hi = (lane & off) != 0;
#pragma unroll
    for (int i = 0; i < half; ++i) {
      const double x = a[i], y = a[i + half];
      asm volatile("" ::"v"(x), "v"(y));
      const double send = hi ? x : y;
      const double keep = hi ? y : x;
      a[i] = keep + __shfl_xor(send, off);
    }
  }
  a[0] += __shfl_xor(a[0], 1);
  if ((lane & 1) == 0) rt[w][lane >> 1] = a[0];
  __syncthreads();
  // every wave: the 16 wave totals (lane i < 16 sums wave i's rows in order), their scan, the owner wave
  double wt = 0.0;
  if (lane < SAMP_WAVES) {
    for (int k = 0; k < SAMP_ROWS_MAX; ++k) wt += rt[lane][k];
  }
  const double wincl = scan_up_d(wt, lane, SAMP_WAVES);
  const double total = __shfl(wincl, SAMP_WAVES - 1);
  if (total_out) *total_out = total;
  const double target = (double)u * total;
  const unsigned long long wmass = __ballot(lane < SAMP_WAVES && wt > 0.0);
  const unsigned long long whit = __ballot(lane < SAMP_WAVES && wt > 0.0 && wincl > target);
  // rounding can leave the target at or beyond the total: then the draw is the last id with mass
  const bool clamp = whit == 0;
  const int owner = !wmass ? -1 : (clamp ? 63 - __clzll((long long)wmass) : __ffsll((long long)whit) - 1);
  if (threadIdx.x == 0 && owner < 0) shi[0] = -1;      // no mass at all
  if (w == owner) {
    double wexcl = __shfl_up(wincl, 1);
    if (lane == 0) wexcl = 0.0;
    const double base = __shfl(wexcl, owner);
    // the last id of this wave with mass (the fallback wherever rounding lets a search run off its end)
    int lastpos = -1;
#pragma unroll
    for (int k = 0; k < SAMP_ROWS_MAX; ++k)
      if (e[k] > 0.f) lastpos = g.j0 + 64 * k;
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) lastpos = max(lastpos, __shfl_xor(lastpos, o));
    // row search: lane k < 32 holds row k's total
    const double rtk = lane < SAMP_ROWS_MAX ? rt[w][lane] : 0.0;
    const double rincl = scan_up_d(rtk, lane, SAMP_ROWS_MAX);
    const unsigned long long rhit = __ballot(lane < SAMP_ROWS_MAX && rtk > 0.0 && base + rincl > target);
    int tok = lastpos;
    if (!clamp && rhit) {
      const int row = __ffsll((long long)rhit) - 1;
      double rexcl = __shfl_up(rincl, 1);
      if (lane == 0) rexcl = 0.0;
      const double rbase = base + __shfl(rexcl, row);
      float qf = 0.f;
#pragma unroll
      for (int k = 0; k < SAMP_ROWS_MAX; ++k) qf = (k == row) ? e[k] : qf;
      const double qk = (double)qf;
      const double incl = scan_up_d(qk, lane, 64);
      const unsigned long long pos = __ballot(qk > 0.0);
      const unsigned long long hit = __ballot(qk > 0.0 && rbase + incl > target);
      const int l = hit ? __ffsll((long long)hit) - 1 : 63 - __clzll((long long)pos);   // pos != 0: the row has mass
      tok = g.row0 + 64 * row + l;
    }
    if (lane == 0) shi[0] = tok;
  }
  __syncthreads();
  return shi[0];
}

__global__ __launch_bounds__(SAMP_THREADS) void sample_row_reg_kernel(const float* __restrict__ logits, int V, float mult,
                                                                      float u, float* __restrict__ q_out,
                                                                      int* __restrict__ tok_out) {
  __shared__ MaxIdx shm[SAMP_WAVES];
  __shared__ double shd[SAMP_WAVES];
  __shared__ double rt[SAMP_WAVES][SAMP_ROWS_MAX + 1];   // row totals, one padded line per wave
  __shared__ int shi[1];
  const RegGeom g = reg_geom(V);
  float e[SAMP_ROWS_MAX];
  MaxIdx top;
  float sum;
  reg_softmax(logits, V, mult, g, e, top, sum, shm, shd);
  const float inv = 1.0f / sum;
#pragma unroll
  for (int k = 0; k < SAMP_ROWS_MAX; ++k) {
    const int j = g.j0 + 64 * k;
    e[k] = e[k] * inv;
    if (k < g.R && j < V) q_out[j] = e[k];
  }
  const int tok = reg_draw(e, g, u, rt, shi, nullptr);
  if (threadIdx.x == 0) tok_out[0] = tok;
}

hipError_t launch_sample_row(const float* logits, int V, float mult, int greedy, float u, float* q_out, int* tok_out,
                             hipStream_t st) {
  if (!greedy && V <= SAMP_ROWS_MAX * SAMP_THREADS) {
    sample_row_reg_kernel<<<1, SAMP_THREADS, 0, st>>>(logits, V, mult, u, q_out, tok_out);
  } else {
    sample_row_kernel<<<1, SAMP_THREADS, 0, st>>>(logits, V, mult, greedy, u, q_out, tok_out);
  }
  return hipGetLastError();
}

// ---- target: per-row test, then first rejection + resampling ---------------------------------
// stats layout per row i: [0] = max logit, [1] = sum exp, [2] = arg-max (as int bits), [3] = accept flag
__global__ __launch_bounds__(SAMP_THREADS) void accept_rows_kernel(const float* __restrict__ logits, int V, float mult,
                                                                   int greedy, const float* __restrict__ qcache,
                                                                   const int* __restrict__ ring,
                                                                   const int* __restrict__ x_direct, AcceptArgs a,
                                                                   float* __restrict__ stats) {
  __shared__ MaxIdx shm[SAMP_WAVES];
  __shared__ double shd[SAMP_WAVES];
  const int i = blockIdx.x;
  const float* row = logits + (size_t)i * V;
  const bool reg = V <= SAMP_ROWS_MAX * SAMP_THREADS;   // the row fits the registers of the workgroup
  MaxIdx top;
  float sum = 1.f;
  if (greedy) {
    MaxIdx m;
    m.v = -INFINITY; m.i = 0x7fffffff;
    for (int j = threadIdx.x; j < V; j += SAMP_THREADS) {
      MaxIdx t; t.v = row[j]; t.i = j;
      m = better(m, t);
    }
    top = block_argmax(m, shm);
  } else if (reg) {
    float e[SAMP_ROWS_MAX];
    reg_softmax(row, V, mult, reg_geom(V), e, top, sum, shm, shd);
  } else {
    row_stats(row, V, mult, shm, shd, top, sum);
  }
  if (threadIdx.x == 0) {
    int acc = 0;
    if (i < a.n_test) {
      const int x = x_direct ? x_direct[i] : ring[a.slot[i]];
      const float* qrow = x_direct ? qcache + (size_t)i * V : qcache + (size_t)a.slot[i] * V;
      if (greedy) {
        acc = (x == top.i);
      } else {
        const float px = reg ? reg_prob(row[x], mult, top.v * mult, 1.0f / sum) : expf(row[x] * mult - top.v * mult) / sum;
        acc = ((double)a.r[i] * (double)qrow[x] <= (double)px);
      }
      if (a.force_mask >= 0) acc = (int)((a.force_mask >> i) & 1);
    }
    stats[i * 4 + 0] = top.v;
    stats[i * 4 + 1] = sum;
    stats[i * 4 + 2] = __int_as_float(top.i);
    stats[i * 4 + 3] = __int_as_float(acc);
  }
}

// One workgroup: n = first rejection; draw from norm(max(0, p_n - q_n)) (from p_n if that has no
// mass), or the bonus / autoregressive token from the row after the last test.  `wbuf` is a
// scratch row of V floats holding the weights the draw walks over.
__global__ __launch_bounds__(SAMP_THREADS) void accept_finish_kernel(const float* __restrict__ logits, int V,
                                                                     float mult, int greedy,
                                                                     const float* __restrict__ qcache,
                                                                     const int* __restrict__ ring,
                                                                     const int* __restrict__ x_direct, AcceptArgs a,
                                                                     const float* __restrict__ stats,
                                                                     float* __restrict__ wbuf,
                                                                     AcceptResult* __restrict__ res,
                                                                     int* __restrict__ out2) {
  __shared__ double shd[SAMP_WAVES];
  __shared__ int shi[2];
  __shared__ double rt[SAMP_WAVES][SAMP_ROWS_MAX + 1];
  int n = 0;
  bool off_path = false;   // guided tests: row n is the target's distribution after x_1..x_n only if those are the guesses
  while (n < a.n_test) {
    if (a.guided && n >= 1 && ring[a.slot[n - 1]] != a.guess[n - 1]) {
      off_path = true;
      break;
    }
    if (__float_as_int(stats[n * 4 + 3]) == 0) break;
    ++n;
  }
  const bool rejected = !off_path && n < a.n_test;
  int token = -1;
  if (rejected || (!a.guided && n < a.n_rows)) {   // a row to draw from exists: the rejecting row, or the bonus row
    const float* row = logits + (size_t)n * V;
    const float vmax = stats[n * 4 + 0], sum = stats[n * 4 + 1];
    const int amax = __float_as_int(stats[n * 4 + 2]);
    if (greedy) {
      token = amax;   // residual of two one-hots, or the one-hot itself, is the target's arg-max
    } else {
      const float* qrow = nullptr;
      if (rejected) qrow = x_direct ? qcache + (size_t)n * V : qcache + (size_t)a.slot[n] * V;
      const float zmax = vmax * mult;
      if (V <= SAMP_ROWS_MAX * SAMP_THREADS) {
        // the row in registers: residual weights (or p itself for the bonus / autoregressive token), one draw
        const RegGeom g = reg_geom(V);
        const float inv = 1.0f / sum;
        float e[SAMP_ROWS_MAX];
#pragma unroll
        for (int k = 0; k < SAMP_ROWS_MAX; ++k) {
          const int j = g.j0 + 64 * k;
          float wj = 0.f;
          if (k < g.R && j < V) {
            const float p = reg_prob(row[j], mult, zmax, inv);
            wj = qrow ? (float)fmax((double)p - (double)qrow[j], 0.0) : p;
          }
          e[k] = wj;
        }
        double total = 0.0;
        token = reg_draw(e, g, a.u_resample, rt, shi, &total);
        if (rejected && !(total > 0.0)) {   // no residual mass in floating point: draw from p itself
#pragma unroll
          for (int k = 0; k < SAMP_ROWS_MAX; ++k) {
            const int j = g.j0 + 64 * k;
            e[k] = (k < g.R && j < V) ? reg_prob(row[j], mult, zmax, inv) : 0.f;
          }
          token = reg_draw(e, g, a.u_resample, rt, shi, nullptr);
        }
      } else {
      for (int j = threadIdx.x; j < V; j += SAMP_THREADS) {
        const float p = expf(row[j] * mult - zmax) / sum;
        wbuf[j] = qrow ? (float)fmax((double)p - (double)qrow[j], 0.0) : p;
      }
      __threadfence_block();
      __syncthreads();
      double total = 0.0;
      token = block_inverse_cdf(wbuf, V, a.u_resample, shd, shi, &total);
      if (rejected && !(total > 0.0)) {   // no residual mass in floating point: draw from p itself
        __syncthreads();
        for (int j = threadIdx.x; j < V; j += SAMP_THREADS) wbuf[j] = expf(row[j] * mult - zmax) / sum;
        __threadfence_block();
        __syncthreads();
        token = block_inverse_cdf(wbuf, V, a.u_resample, shd, shi, nullptr);
      }
      }
    }
  }
  if (threadIdx.x == 0) {
    res->n_accepted = n;
    res->token = token;
    res->rejected = rejected ? 1 : 0;
    res->off_path = off_path ? 1 : 0;
    if (out2) {   // callers that want the outcome in device memory of their own
      out2[0] = n;
      out2[1] = token;
    }
  }
  if (ring && threadIdx.x < SPEC_RING_MAX) res->ring[threadIdx.x] = ring[threadIdx.x];
}

hipError_t launch_accept(const float* logits, int V, float mult, int greedy, const float* qcache, const int* ring,
                         const int* x_direct, AcceptArgs a, float* stats_scratch, AcceptResult* result_dev,
                         hipStream_t st, int* out2) {
  // stats_scratch: 4 floats per row, followed (at a 256-float offset) by one scratch row of V floats
  if (a.guided && !ring) return hipErrorInvalidValue;   // guided tests compare ring tokens with the guesses
  accept_rows_kernel<<<a.n_rows, SAMP_THREADS, 0, st>>>(logits, V, mult, greedy, qcache, ring, x_direct, a,
                                                        stats_scratch);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  accept_finish_kernel<<<1, SAMP_THREADS, 0, st>>>(logits, V, mult, greedy, qcache, ring, x_direct, a, stats_scratch,
                                                   stats_scratch + 256, result_dev, out2);
  return hipGetLastError();
}

// ---- acceptance without any allocation ---------------------------------------------------------
// The scratch of the two acceptance kernels (row statistics, one row of draw weights, the result record) in a
// file-scope device array instead of memory from hipMalloc: for callers that must not allocate (code under HIP
// graph capture, tight serving loops).  Every GPU the library runs on holds its own copy of the array until the
// process ends; its address on a device is looked up once, with that device current.  All calls on one GPU share
// the array, so calls that overlap on one GPU (two streams, two threads) race; nothing in it has to start at zero
// (every word a call reads was written by that call before).
#define ACCEPT_STATIC_STATS_FLOATS 256
#define ACCEPT_STATIC_BYTES ((ACCEPT_STATIC_STATS_FLOATS + SPEC_STATIC_VOCAB_MAX) * 4 + 512)
static __device__ __align__(256) unsigned char scratch[ACCEPT_STATIC_BYTES];

#include <mutex>
#define ACCEPT_STATIC_MAX_DEVICES 64
static void* g_scratch_ptr[ACCEPT_STATIC_MAX_DEVICES];
static std::mutex g_scratch_mutex;

// device address of `scratch` on the current device (nullptr and an error message on failure)
static void* static_scratch_ptr() {
  int dev = -1;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess || dev < 0 || dev >= ACCEPT_STATIC_MAX_DEVICES) {
    spec_set_error("hipGetDevice failed or device id %d above %d: %s", dev, ACCEPT_STATIC_MAX_DEVICES - 1,
                   hipGetErrorString(e));
    return nullptr;
  }
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (!g_scratch_ptr[dev]) {
    void* p = nullptr;
    e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
    if (e != hipSuccess || !p) {
      spec_set_error("hipGetSymbolAddress(scratch) failed on device %d: %s", dev, hipGetErrorString(e));
      return nullptr;
    }
    g_scratch_ptr[dev] = p;
  }
  return g_scratch_ptr[dev];
}

extern "C" int spec_accept_rows_static(const float* p_logits, int n_rows, const float* q_rows, const int32_t* x,
                                       int n_test, int vocab, float temperature, float logit_scale, const float* r,
                                       float u_resample, int32_t* result_dev, void* stream) {
  if (!p_logits || !result_dev || vocab < 1 || n_rows < 1 || n_rows > SPEC_MAX_TOKENS || n_test < 0 || n_test > n_rows) {
    spec_set_error("bad argument");
    return SPEC_E_INVAL;
  }
  if (vocab > SPEC_STATIC_VOCAB_MAX) {
    spec_set_error("vocabulary of %d ids is above the %d the static scratch holds; use spec_accept_rows", vocab,
                   SPEC_STATIC_VOCAB_MAX);
    return SPEC_E_INVAL;
  }
  if (n_test > 0 && (!q_rows || !x || !r)) {
    spec_set_error("null pointer");
    return SPEC_E_INVAL;
  }
  if (!(temperature >= 0.0f) || !(logit_scale > 0.0f) || !(u_resample >= 0.0f && u_resample < 1.0f)) {
    spec_set_error("bad temperature / logit_scale / uniform");
    return SPEC_E_INVAL;
  }
  static_assert(4 * SPEC_MAX_TOKENS <= ACCEPT_STATIC_STATS_FLOATS, "four statistics per row");
  static_assert(sizeof(AcceptResult) <= 512, "the result record sits in the last 512 bytes");
  unsigned char* base = (unsigned char*)static_scratch_ptr();
  if (!base) return SPEC_E_HIP;
  AcceptArgs a;
  memset(&a, 0, sizeof(a));
  a.n_rows = n_rows;
  a.n_test = n_test;
  a.u_resample = u_resample;
  a.force_mask = -1;
  for (int i = 0; i < n_test; ++i) {
    if (!(r[i] >= 0.0f && r[i] < 1.0f)) {
      spec_set_error("uniform outside [0,1)");
      return SPEC_E_INVAL;
    }
    a.r[i] = r[i];
  }
  const bool greedy = temperature == 0.0f;
  float* stats = (float*)base;
  AcceptResult* res = (AcceptResult*)(base + (size_t)(ACCEPT_STATIC_STATS_FLOATS + SPEC_STATIC_VOCAB_MAX) * 4);
  hipError_t e = launch_accept(p_logits, vocab, greedy ? 1.0f : logit_scale / temperature, greedy ? 1 : 0, q_rows,
                               nullptr, x, a, stats, res, (hipStream_t)stream, result_dev);
  if (e != hipSuccess) {
    spec_set_error("accept kernels failed to launch: %s", hipGetErrorString(e));
    return SPEC_E_HIP;
  }
  return SPEC_OK;
}
