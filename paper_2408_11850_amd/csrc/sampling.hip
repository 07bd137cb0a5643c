// Fused logits -> probability kernels (gfx950): the draft's draw x_i ~ q_i and the target's
// accept / reject with residual resampling (paper Section 2, Eq. (1); Algorithm 2).
//
// A distribution is softmax(mult * logits) in fp32 (mult = logit_scale / temperature), or the
// one-hot at the arg-max (lowest id on ties) for greedy decoding.  A draw is an inverse-CDF walk in
// ascending token id with one uniform u: the first k whose running sum (fp64) exceeds u * total.
// The acceptance test is evaluated without a division, in fp64: accept iff r * q[x] <= p[x].
// One workgroup of 1024 threads handles one vocabulary row; these kernels are latency-bound.
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

hipError_t launch_sample_row(const float* logits, int V, float mult, int greedy, float u, float* q_out, int* tok_out,
                             hipStream_t st) {
  sample_row_kernel<<<1, SAMP_THREADS, 0, st>>>(logits, V, mult, greedy, u, q_out, tok_out);
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
        const float px = expf(row[x] * mult - top.v * mult) / sum;
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
                                                                     AcceptResult* __restrict__ res) {
  __shared__ double shd[SAMP_WAVES];
  __shared__ int shi[2];
  int n = 0;
  while (n < a.n_test && __float_as_int(stats[n * 4 + 3]) != 0) ++n;
  const bool rejected = n < a.n_test;
  int token = -1;
  if (rejected || n < a.n_rows) {   // a row to draw from exists: the rejecting row, or the bonus row
    const float* row = logits + (size_t)n * V;
    const float vmax = stats[n * 4 + 0], sum = stats[n * 4 + 1];
    const int amax = __float_as_int(stats[n * 4 + 2]);
    if (greedy) {
      token = amax;   // residual of two one-hots, or the one-hot itself, is the target's arg-max
    } else {
      const float* qrow = nullptr;
      if (rejected) qrow = x_direct ? qcache + (size_t)n * V : qcache + (size_t)a.slot[n] * V;
      const float zmax = vmax * mult;
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
  if (threadIdx.x == 0) {
    res->n_accepted = n;
    res->token = token;
    res->rejected = rejected ? 1 : 0;
    res->pad = 0;
  }
  if (ring && threadIdx.x < SPEC_RING_MAX) res->ring[threadIdx.x] = ring[threadIdx.x];
}

hipError_t launch_accept(const float* logits, int V, float mult, int greedy, const float* qcache, const int* ring,
                         const int* x_direct, AcceptArgs a, float* stats_scratch, AcceptResult* result_dev,
                         hipStream_t st) {
  // stats_scratch: 4 floats per row, followed (at a 256-float offset) by one scratch row of V floats
  accept_rows_kernel<<<a.n_rows, SAMP_THREADS, 0, st>>>(logits, V, mult, greedy, qcache, ring, x_direct, a,
                                                        stats_scratch);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  accept_finish_kernel<<<1, SAMP_THREADS, 0, st>>>(logits, V, mult, greedy, qcache, ring, x_direct, a, stats_scratch,
                                                   stats_scratch + 256, result_dev);
  return hipGetLastError();
}
