// Small per-token kernels around the projections (gfx950): token gather, embedding, RoPE + KV append.
// (RMSNorm, the residual adds and SiLU*mul are fused into the projection kernel.)  The RoPE kernel reads the
// fp32 K-slice partials of the QKV projection and adds the slices in ascending order.
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

// h[m][:] = float(E[tok[m]][:]) and sumsq[m] = sum_i h[m][i]^2 (added in a fixed order); an id outside the
// vocabulary reads row 0 (ids are validated on the host)
__global__ __launch_bounds__(256) void embed_kernel(float* __restrict__ h, float* __restrict__ sumsq,
                                                    const bf16* __restrict__ E, const int* __restrict__ tok, int d,
                                                    int vocab) {
  __shared__ float sh[4];
  const int m = blockIdx.x;
  int t = tok[m];
  if (t < 0 || t >= vocab) t = 0;
  const bf16* row = E + (size_t)t * d;
  float ss = 0.f;
  for (int i = threadIdx.x; i < d; i += 256) {
    const float v = __bfloat162float(row[i]);
    h[(size_t)m * d + i] = v;
    ss += v * v;
  }
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) ss += __shfl_xor(ss, o);
  if ((threadIdx.x & 63) == 0) sh[threadIdx.x >> 6] = ss;
  __syncthreads();
  if (threadIdx.x == 0) sumsq[m] = sh[0] + sh[1] + sh[2] + sh[3];
}
hipError_t launch_embed(float* h, float* sumsq, const bf16* embed, const int* tok, int M, int d, int vocab,
                        hipStream_t st) {
  embed_kernel<<<M, 256, 0, st>>>(h, sumsq, embed, tok, d, vocab);
  return hipGetLastError();
}

// One workgroup per (token, head) of the fused QKV output; thread e handles the pair (e, e + dh/2).
// q heads: rotate, store bf16 [M][Hq][dh].  k heads: rotate, store into the page in K-operand order.
// v heads: store into the page in V-operand order.  Position of token i is len + i.
__global__ void rope_append_kernel(const float* __restrict__ P, int S, bf16* __restrict__ q, bf16* __restrict__ pool,
                                   const int* __restrict__ block_table, const int* __restrict__ len_ptr, KvGeom g,
                                   int layer, int M, int Hq, float theta) {
  const int i = blockIdx.x, head = blockIdx.y;
  const int dh = g.head_dim, half = dh >> 1, Hkv = g.n_kv_heads;
  const int N = (Hq + 2 * Hkv) * dh;
  const int e = threadIdx.x;
  if (e >= half) return;
  const int pos = len_ptr[0] + i;
  float x0 = 0.f, x1 = 0.f;
  for (int s = 0; s < S; ++s) {
    const float* row = P + ((size_t)s * M + i) * N + (size_t)head * dh;
    x0 += row[e];
    x1 += row[e + half];
  }
  if (head < Hq + Hkv) {   // rotate pair (e, e + dh/2) by pos * theta^(-2e/dh)
    const double ang = (double)pos * pow((double)theta, -2.0 * (double)e / (double)dh);
    const float cs = (float)cos(ang), sn = (float)sin(ang);
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
                              const int* len_ptr, KvGeom g, int layer, int M, int Hq, float theta, hipStream_t st) {
  dim3 grid(M, Hq + 2 * g.n_kv_heads), block(64);
  rope_append_kernel<<<grid, block, 0, st>>>(partials, S, q, pool, block_table, len_ptr, g, layer, M, Hq, theta);
  return hipGetLastError();
}
