// Small per-token kernels between the projections (gfx950): token gather, embedding,
// residual add + RMSNorm, RoPE + KV append, SiLU*mul.  All of them read the fp32 K-slice
// partials of the preceding projection and add the slices in ascending order.
#include "spec_internal.h"

__global__ void gather_tokens_kernel(int* tok_out, const int* ring, TokenSrc src) {
  int i = threadIdx.x;
  if (i < src.n) tok_out[i] = src.imm[i] >= 0 ? src.imm[i] : ring[src.slot[i]];
}
hipError_t launch_gather_tokens(int* tok_out, const int* ring, TokenSrc src, hipStream_t st) {
  gather_tokens_kernel<<<1, 64, 0, st>>>(tok_out, ring, src);
  return hipGetLastError();
}

__global__ void set_int_kernel(int* dst, int v) { dst[0] = v; }
__global__ void add_int_kernel(int* dst, int d) { dst[0] += d; }
hipError_t launch_set_int(int* dst, int value, hipStream_t st) {
  set_int_kernel<<<1, 1, 0, st>>>(dst, value);
  return hipGetLastError();
}
hipError_t launch_add_int(int* dst, int delta, hipStream_t st) {
  add_int_kernel<<<1, 1, 0, st>>>(dst, delta);
  return hipGetLastError();
}
__global__ void set_pages_kernel(int* bt, PageUpdate u) {
  int i = threadIdx.x;
  if (i < u.count) bt[u.first + i] = u.page[i];
}
hipError_t launch_set_pages(int* block_table, PageUpdate u, hipStream_t st) {
  set_pages_kernel<<<1, 64, 0, st>>>(block_table, u);
  return hipGetLastError();
}

// h[m][:] = float(E[tok[m]][:]); an id outside the vocabulary reads row 0 (ids are validated on the host)
__global__ void embed_kernel(float* __restrict__ h, const bf16* __restrict__ E, const int* __restrict__ tok, int d,
                             int vocab) {
  const int m = blockIdx.x;
  int t = tok[m];
  if (t < 0 || t >= vocab) t = 0;
  const bf16* row = E + (size_t)t * d;
  for (int i = threadIdx.x; i < d; i += blockDim.x) h[(size_t)m * d + i] = __bfloat162float(row[i]);
}
hipError_t launch_embed(float* h, const bf16* embed, const int* tok, int M, int d, int vocab, hipStream_t st) {
  embed_kernel<<<M, 256, 0, st>>>(h, embed, tok, d, vocab);
  return hipGetLastError();
}

__device__ __forceinline__ float block_sum(float v, float* sh) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o);
  const int w = threadIdx.x >> 6;
  if ((threadIdx.x & 63) == 0) sh[w] = v;
  __syncthreads();
  float t = 0.f;
  const int nw = blockDim.x >> 6;
  for (int i = 0; i < nw; ++i) t += sh[i];
  __syncthreads();
  return t;
}

// h[m] += sum_s P[s][m] ; a[m] = h[m] * rsqrt(mean(h[m]^2) + eps) * gain.
// One workgroup of 1024 threads per row; a thread keeps its (at most 4) float4 pieces of the row in
// registers, and the S slice loads of a piece are independent, so the row is read in a few round trips.
#define ADDNORM_THREADS 1024
#define ADDNORM_PIECES 4      // d_model <= 4 * 4 * 1024
__global__ __launch_bounds__(ADDNORM_THREADS) void addnorm_kernel(float* __restrict__ h, const float* __restrict__ P,
                                                                  int S, const bf16* __restrict__ gain,
                                                                  bf16* __restrict__ a, int M, int d, float eps) {
  __shared__ float sh[ADDNORM_THREADS / 64];
  const int m = blockIdx.x;
  const int d4 = d >> 2;
  f32x4* hr = reinterpret_cast<f32x4*>(h + (size_t)m * d);
  const f32x4* P4 = reinterpret_cast<const f32x4*>(P);
  f32x4 v[ADDNORM_PIECES];
  float ss = 0.f;
#pragma unroll
  for (int it = 0; it < ADDNORM_PIECES; ++it) {
    const int i = threadIdx.x + it * ADDNORM_THREADS;
    v[it] = f32x4{0.f, 0.f, 0.f, 0.f};
    if (i < d4) {
      f32x4 t = hr[i];
      if (P) {
        int s = 0;
        for (; s + 4 <= S; s += 4) {   // four independent loads in flight, added in ascending slice order
          const f32x4 p0 = P4[((size_t)(s + 0) * M + m) * d4 + i], p1 = P4[((size_t)(s + 1) * M + m) * d4 + i];
          const f32x4 p2 = P4[((size_t)(s + 2) * M + m) * d4 + i], p3 = P4[((size_t)(s + 3) * M + m) * d4 + i];
          t += p0; t += p1; t += p2; t += p3;
        }
        for (; s < S; ++s) t += P4[((size_t)s * M + m) * d4 + i];
      }
      hr[i] = t;
      v[it] = t;
      ss += t.x * t.x + t.y * t.y + t.z * t.z + t.w * t.w;
    }
  }
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) ss += __shfl_xor(ss, o);
  if ((threadIdx.x & 63) == 0) sh[threadIdx.x >> 6] = ss;
  __syncthreads();
  float tot = 0.f;
#pragma unroll
  for (int i = 0; i < ADDNORM_THREADS / 64; ++i) tot += sh[i];
  const float inv = 1.0f / sqrtf(tot / (float)d + eps);
#pragma unroll
  for (int it = 0; it < ADDNORM_PIECES; ++it) {
    const int i = threadIdx.x + it * ADDNORM_THREADS;
    if (i < d4) {
      const bf16* g = gain + (size_t)i * 4;
      bf16* dst = a + (size_t)m * d + (size_t)i * 4;
      dst[0] = __float2bfloat16(v[it].x * inv * __bfloat162float(g[0]));
      dst[1] = __float2bfloat16(v[it].y * inv * __bfloat162float(g[1]));
      dst[2] = __float2bfloat16(v[it].z * inv * __bfloat162float(g[2]));
      dst[3] = __float2bfloat16(v[it].w * inv * __bfloat162float(g[3]));
    }
  }
}
hipError_t launch_addnorm(float* h, const float* partials, int S, const bf16* gain, bf16* a, int M, int d, float eps,
                          hipStream_t st) {
  addnorm_kernel<<<M, ADDNORM_THREADS, 0, st>>>(h, partials, S, gain, a, M, d, eps);
  return hipGetLastError();
}

// The residual add alone, spread over d/1024 workgroups per row (one compute unit cannot pull the S slices of a
// long row fast enough): h += sum_s P[s] in the same order as addnorm_kernel, and the sum of squares of each
// 1024-column piece, plus x' = bf16(h * gain) for the next projection (whose consumers apply 1/rms).
#define ADDSQ_THREADS 256
__global__ __launch_bounds__(ADDSQ_THREADS) void add_sumsq_kernel(float* __restrict__ h, const float* __restrict__ P,
                                                                  int S, const bf16* __restrict__ gain,
                                                                  bf16* __restrict__ a, float* __restrict__ ssq, int M,
                                                                  int d, int W) {
  __shared__ float sh[ADDSQ_THREADS / 64];
  const int m = blockIdx.y, w = blockIdx.x;
  const int d4 = d >> 2;
  const int i = w * ADDSQ_THREADS + threadIdx.x;
  float ss = 0.f;
  if (i < d4) {
    f32x4* hr = reinterpret_cast<f32x4*>(h + (size_t)m * d);
    const f32x4* P4 = reinterpret_cast<const f32x4*>(P);
    f32x4 t = hr[i];
    if (P) {
      int s = 0;
      for (; s + 4 <= S; s += 4) {
        const f32x4 p0 = P4[((size_t)(s + 0) * M + m) * d4 + i], p1 = P4[((size_t)(s + 1) * M + m) * d4 + i];
        const f32x4 p2 = P4[((size_t)(s + 2) * M + m) * d4 + i], p3 = P4[((size_t)(s + 3) * M + m) * d4 + i];
        t += p0; t += p1; t += p2; t += p3;
      }
      for (; s < S; ++s) t += P4[((size_t)s * M + m) * d4 + i];
      hr[i] = t;
    }
    ss = t.x * t.x + t.y * t.y + t.z * t.z + t.w * t.w;
    const bf16* g = gain + (size_t)i * 4;
    bf16* dst = a + (size_t)m * d + (size_t)i * 4;
    dst[0] = __float2bfloat16(t.x * __bfloat162float(g[0]));
    dst[1] = __float2bfloat16(t.y * __bfloat162float(g[1]));
    dst[2] = __float2bfloat16(t.z * __bfloat162float(g[2]));
    dst[3] = __float2bfloat16(t.w * __bfloat162float(g[3]));
  }
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) ss += __shfl_xor(ss, o);
  if ((threadIdx.x & 63) == 0) sh[threadIdx.x >> 6] = ss;
  __syncthreads();
  if (threadIdx.x == 0) {
    float tot = 0.f;
#pragma unroll
    for (int k = 0; k < ADDSQ_THREADS / 64; ++k) tot += sh[k];
    ssq[m * SSQ_STRIDE + w] = tot;
  }
}
hipError_t launch_add_sumsq(float* h, const float* partials, int S, const bf16* gain, bf16* a, float* ssq, int M,
                            int d, int* W_out, hipStream_t st) {
  const int W = ((d >> 2) + ADDSQ_THREADS - 1) / ADDSQ_THREADS;
  if ((d & 3) || W > ADDSQ_MAX_PIECES) return hipErrorInvalidValue;
  add_sumsq_kernel<<<dim3(W, M), ADDSQ_THREADS, 0, st>>>(h, partials, S, gain, a, ssq, M, d, W);
  *W_out = W;
  return hipGetLastError();
}

// One 64-thread slice of a workgroup per (token, head) of the fused QKV output (ROPE_HPB heads per workgroup);
// thread e of the slice handles the pair (e, e + dh/2).
// q heads: rotate, store bf16 [M][Hq][dh].  k heads: rotate, store into the page in K-operand order.
// v heads: store into the page in V-operand order.  Position of token i is len + i.
#define ROPE_HPB 4
// (cos, sin) of the rotation angle of pair e at position len + i, for all tokens of a prompt block: the same
// expression as in rope_append_kernel, evaluated once per block instead of once per layer and head.
__global__ void rope_table_kernel(float2* __restrict__ tab, const int* __restrict__ len_ptr, int dh, float theta) {
  const int i = blockIdx.x, e = threadIdx.x, half = dh >> 1;
  if (e >= half) return;
  const int pos = len_ptr[0] + i;
  const double ang = (double)pos * pow((double)theta, -2.0 * (double)e / (double)dh);
  tab[(size_t)i * half + e] = make_float2((float)cos(ang), (float)sin(ang));
}
hipError_t launch_rope_table(float2* tab, const int* len_ptr, int M, int dh, float theta, hipStream_t st) {
  rope_table_kernel<<<M, 64, 0, st>>>(tab, len_ptr, dh, theta);
  return hipGetLastError();
}

__global__ void rope_append_kernel(const float* __restrict__ P, int S, bf16* __restrict__ q, bf16* __restrict__ pool,
                                   const int* __restrict__ block_table, const int* __restrict__ len_ptr, KvGeom g,
                                   int layer, int M, int Hq, float theta, const float2* __restrict__ tab, RowScale rs) {
  const int i = blockIdx.x, head = blockIdx.y * ROPE_HPB + (threadIdx.x >> 6);
  const int dh = g.head_dim, half = dh >> 1, Hkv = g.n_kv_heads;
  const int N = (Hq + 2 * Hkv) * dh;
  const int e = threadIdx.x & 63;
  if (e >= half || head >= Hq + 2 * Hkv) return;
  const int pos = len_ptr[0] + i;
  // The kernel is one chain of latencies, so every load goes out before anything waits: the first four K slices,
  // the row's sums of squares, the position; the fp64 angle is worked out while they are in flight.  Slices are
  // added in ascending order whatever the grouping.
  const float* base = P + (size_t)i * N + (size_t)head * dh;
  const size_t sstride = (size_t)M * N;
  float a0[4], a1[4];
#pragma unroll
  for (int k = 0; k < 4; ++k) {
    a0[k] = (k < S) ? base[k * sstride + e] : 0.f;
    a1[k] = (k < S) ? base[k * sstride + e + half] : 0.f;
  }
  const float inv = rs.inv(i);
  float cs = 1.f, sn = 0.f;
  if (head < Hq + Hkv) {   // rotation of pair (e, e + dh/2) by pos * theta^(-2e/dh)
    if (tab) {
      const float2 t = tab[(size_t)i * half + e];
      cs = t.x; sn = t.y;
    } else {
      const double ang = (double)pos * pow((double)theta, -2.0 * (double)e / (double)dh);
      cs = (float)cos(ang); sn = (float)sin(ang);
    }
  }
  float x0 = 0.f, x1 = 0.f;
#pragma unroll
  for (int k = 0; k < 4; ++k)
    if (k < S) { x0 += a0[k]; x1 += a1[k]; }
  for (int s0 = 4; s0 < S; s0 += 4) {
#pragma unroll
    for (int k = 0; k < 4; ++k) {
      a0[k] = (s0 + k < S) ? base[(s0 + k) * sstride + e] : 0.f;
      a1[k] = (s0 + k < S) ? base[(s0 + k) * sstride + e + half] : 0.f;
    }
#pragma unroll
    for (int k = 0; k < 4; ++k)
      if (s0 + k < S) { x0 += a0[k]; x1 += a1[k]; }
  }
  x0 *= inv;
  x1 *= inv;
  if (head < Hq + Hkv) {
    const float y0 = x0 * cs - x1 * sn, y1 = x0 * sn + x1 * cs;
    x0 = y0; x1 = y1;
  }
  if (head < Hq) {
    bf16* dst = q + ((size_t)i * Hq + head) * dh;
    dst[e] = __float2bfloat16(x0);
    dst[e + half] = __float2bfloat16(x1);
    return;
  }
  const int page = block_table[pos / SPEC_PAGE_TOKENS];
  const int r = pos % SPEC_PAGE_TOKENS;
  if (head < Hq + Hkv) {
    bf16* blk = pool + g.offset(page, layer, 0, head - Hq);
    const int tile = r >> 4, rr = r & 15, nsteps = dh >> 5;
    for (int t = 0; t < 2; ++t) {
      const int ee = t ? e + half : e;
      const size_t off = ((size_t)((tile * nsteps + (ee >> 5)) * 64 + ((ee & 31) >> 3) * 16 + rr)) * 8 + (ee & 7);
      blk[off] = __float2bfloat16(t ? x1 : x0);
    }
  } else {
    bf16* blk = pool + g.offset(page, layer, 1, head - Hq - Hkv);
    const int chunk = r >> 5, r32 = r & 31;
    const int slot = ((r32 & 15) >> 2) * 8 + (r32 >> 4) * 4 + (r32 & 3);
    blk[((size_t)chunk * dh + e) * 32 + slot] = __float2bfloat16(x0);
    blk[((size_t)chunk * dh + e + half) * 32 + slot] = __float2bfloat16(x1);
  }
}
hipError_t launch_rope_append(const float* partials, int S, bf16* q, bf16* pool, const int* block_table,
                              const int* len_ptr, KvGeom g, int layer, int M, int Hq, float theta, hipStream_t st,
                              const float2* tab, RowScale rs) {
  dim3 grid(M, (Hq + 2 * g.n_kv_heads + ROPE_HPB - 1) / ROPE_HPB), block(64 * ROPE_HPB);
  rope_append_kernel<<<grid, block, 0, st>>>(partials, S, q, pool, block_table, len_ptr, g, layer, M, Hq, theta, tab,
                                             rs);
  return hipGetLastError();
}

// z[m][f] = silu(gate) * up, gate/up panels interleaved in the fused projection output (width 2F)
__global__ void silu_mul_kernel(const float* __restrict__ P, int S, bf16* __restrict__ z, int M, int F, RowScale rs) {
  const int m = blockIdx.y;
  const int f = blockIdx.x * blockDim.x + threadIdx.x;
  if (f >= F) return;
  const int gc = (f >> 4) * 32 + (f & 15);
  // all loads of the first four K slices and of the row's sums of squares go out together (one round trip);
  // slices are added in ascending order whatever the grouping
  const float* base = P + (size_t)m * (2 * (size_t)F) + gc;
  const size_t sstride = (size_t)M * (2 * (size_t)F);
  float g4[4], u4[4];
#pragma unroll
  for (int k = 0; k < 4; ++k) {
    g4[k] = (k < S) ? base[k * sstride] : 0.f;
    u4[k] = (k < S) ? base[k * sstride + 16] : 0.f;
  }
  const float inv = rs.inv(m);
  float gv = 0.f, uv = 0.f;
#pragma unroll
  for (int k = 0; k < 4; ++k)
    if (k < S) { gv += g4[k]; uv += u4[k]; }
  for (int s0 = 4; s0 < S; s0 += 4) {
#pragma unroll
    for (int k = 0; k < 4; ++k) {
      g4[k] = (s0 + k < S) ? base[(s0 + k) * sstride] : 0.f;
      u4[k] = (s0 + k < S) ? base[(s0 + k) * sstride + 16] : 0.f;
    }
#pragma unroll
    for (int k = 0; k < 4; ++k)
      if (s0 + k < S) { gv += g4[k]; uv += u4[k]; }
  }
  gv *= inv;
  uv *= inv;
  const float sg = gv / (1.0f + __expf(-gv));
  z[(size_t)m * F + f] = __float2bfloat16(sg * uv);
}
hipError_t launch_silu_mul(const float* partials, int S, bf16* z, int M, int F, hipStream_t st, RowScale rs) {
  dim3 grid((F + 255) / 256, M), block(256);
  silu_mul_kernel<<<grid, block, 0, st>>>(partials, S, z, M, F, rs);
  return hipGetLastError();
}
