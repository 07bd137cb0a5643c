// Skinny projection kernels for gfx950: y[M][N] = x[M][K] W^T with M <= 32 new tokens.
//
// Every weight is read exactly once per forward, so the kernel is HBM-bound (M flop per weight
// byte pair); the MFMA unit is only the cheapest way to apply up to 32 activations to each
// streamed weight.  W is stored panel-packed: a panel is 16 output rows, cut into 32-wide
// K steps, and the 16x32 block of one step is laid out exactly as the A operand of
// v_mfma_f32_16x16x32_bf16 (lane l = 16*(k/8) + row holds 8 consecutive k), 1 KiB per step.
// A wave therefore reads its share of a panel as consecutive fully-coalesced 1 KiB loads.
//
// Work split: the K axis is cut into S slices; a workgroup of 8 waves owns one slice and a
// contiguous range of panels; wave w owns `spw` <= 8 consecutive steps of the slice and keeps the
// matching activation fragments (the B operand) in registers for the whole kernel.  After every
// round of 4 panels the 8 wave-partials are summed through LDS in a fixed order.
//
// What happens to the sums (EPI) and where the activations come from (PRO) is fused in:
//   PRO_BF16  x is bf16 [M][K];            PRO_NORM  x = rmsnorm(h) * gain computed while loading h (fp32)
//   EPI_PARTIAL  write the K-slice partial P[s][m][n] (the consumer adds the slices)
//   EPI_F32      y[m][n] = sum            EPI_RESID  h[m][n] += sum, and sum_n h^2 per row for the next norm
//   EPI_SILU     z[m][f] = silu(gate) * up with gate / up in alternating panels
// With S > 1 the fused epilogues need all K slices: every workgroup writes its partial, and the last of the
// S workgroups that share a panel range to arrive (an atomic counter, no waiting) adds the slices in ascending
// order and applies the epilogue.  All additions happen in an order fixed by the shape, so results are
// bit-reproducible and do not depend on which workgroup arrives last.
#include "spec_internal.h"

#define GEMM_WAVES 8
#define GEMM_THREADS (GEMM_WAVES * 64)
#define GEMM_SPW 8    // most K steps per wave (32 VGPRs of activation fragments per 16 rows)
#define GEMM_RP 4     // panels per reduction round
#define GEMM_LOAD(p) __builtin_nontemporal_load(p)

GemmPlan gemm_plan(int M, int N, int K, int wgs_per_cu) {
  GemmPlan p;
  p.M = M; p.N = N; p.K = K;
  p.steps = (K + 31) / 32;
  p.NT = N / 16;
  p.MT = M > 16 ? 2 : 1;
  if (p.MT == 2 || wgs_per_cu < 1) wgs_per_cu = 1;     // the 32-row variant needs a whole CU
  if (wgs_per_cu > 2) wgs_per_cu = 2;
  const int slots = SPEC_NUM_CU * wgs_per_cu;
  p.S = (p.steps + GEMM_WAVES * GEMM_SPW - 1) / (GEMM_WAVES * GEMM_SPW);
  // small matrices: cut K finer until every workgroup slot (at two per CU) has work.  The K split depends
  // on the shape only, never on wgs_per_cu, so both launch modes add the same numbers in the same order.
  while (p.S * p.NT < 2 * SPEC_NUM_CU && (p.steps + GEMM_WAVES * p.S * 2 - 1) / (GEMM_WAVES * p.S * 2) >= 2) p.S *= 2;
  p.spw = (p.steps + GEMM_WAVES * p.S - 1) / (GEMM_WAVES * p.S);
  p.Gs = slots / p.S;
  if (p.Gs < 1) p.Gs = 1;
  if (p.Gs > p.NT / 2) p.Gs = p.NT / 2 > 0 ? p.NT / 2 : 1;   // at least one gate/up panel pair per workgroup
  return p;
}

__device__ __forceinline__ void load_chunk(u32x4 (&a)[GEMM_SPW], const u32x4* __restrict__ wp, int nst) {
#pragma unroll
  for (int j = 0; j < GEMM_SPW; ++j)
    if (j < nst) a[j] = GEMM_LOAD(wp + (size_t)j * 64);
}

template <int MT>
__device__ __forceinline__ void mma_chunk(f32x4 (&acc)[MT], const u32x4 (&a)[GEMM_SPW],
                                          const bf16x8 (&b)[MT][GEMM_SPW], int nst) {
#pragma unroll
  for (int j = 0; j < GEMM_SPW; ++j)
    if (j < nst) {
      bf16x8 av = __builtin_bit_cast(bf16x8, a[j]);
#pragma unroll
      for (int mt = 0; mt < MT; ++mt) acc[mt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(av, b[mt][j], acc[mt], 0, 0, 0);
    }
}

// Epilogue of one (row m, panel p, quad q) group: t holds the sums of columns 16 p + 4 q .. + 3 (t2: the same
// columns of panel p + 1 for EPI_SILU).
template <int EPI>
__device__ __forceinline__ void epi_store(const GemmArgs& a, int m, int p, int q, f32x4 t, f32x4 t2, float& ss) {
  const size_t n = (size_t)p * 16 + q * 4;
  if (EPI == EPI_F32) {
    *reinterpret_cast<f32x4*>(static_cast<float*>(a.out) + (size_t)m * a.N + n) = t;
  } else if (EPI == EPI_RESID) {
    f32x4* hp = reinterpret_cast<f32x4*>(static_cast<float*>(a.out) + (size_t)m * a.N + n);
    f32x4 v = *hp;
    v += t;
    *hp = v;
    ss += v.x * v.x + v.y * v.y + v.z * v.z + v.w * v.w;
  } else if (EPI == EPI_SILU) {
    const size_t f = (size_t)(p >> 1) * 16 + q * 4;
    bf16* dst = static_cast<bf16*>(a.out) + (size_t)m * (a.N >> 1) + f;
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      const float g = t[e];
      dst[e] = __float2bfloat16(g / (1.0f + __expf(-g)) * t2[e]);
    }
  }
}

// TAG only names the instantiation (0 = target model, 1 = draft model, 2 = stand-alone call) so that profilers
// list the two models' launches separately.  WPE = waves per SIMD the register budget is sized for: the 16-row
// variant is held to 128 VGPRs (WPE 4) so that two workgroups share a CU: 16 waves per CU hide the HBM latency
// far better than 8 (measured 6.9 vs 5.9 TB/s on the gate/up matrix), and the second slot can also go to the
// other stream's kernel.
template <int MT, int TAG, int WPE, int EPI, int PRO>
__global__ __launch_bounds__(GEMM_THREADS, WPE) void gemm_kernel(const GemmArgs a) {
  constexpr int NBUF = (MT == 1) ? 2 : 1;    // LDS reduction buffers: two let a round end with a single barrier
  __shared__ f32x4 red[NBUF][GEMM_WAVES][GEMM_RP][MT][64];
  __shared__ int s_last;
  const int M = a.M, N = a.N, K = a.K, S = a.S, Gs = a.Gs;
  const int s = blockIdx.x % S;
  const int idx = blockIdx.x / S;
  const int units = a.NT >> 1;               // panel ranges are cut at even panels (gate/up pairs stay together)
  int p0 = 2 * (int)((long long)idx * units / Gs);
  int p1 = 2 * (int)((long long)(idx + 1) * units / Gs);
  if (idx == Gs - 1) p1 = a.NT;              // an odd panel count: the last range takes the odd one
  const int w = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int c = lane & 15, kb = lane >> 4;
  const int step0 = (s * GEMM_WAVES + w) * a.spw;
  int nst = a.steps - step0;
  if (nst > a.spw) nst = a.spw;
  if (nst < 0) nst = 0;

  // activation fragments of this wave's K range, kept for the whole kernel
  bf16x8 b[MT][GEMM_SPW];
#pragma unroll
  for (int mt = 0; mt < MT; ++mt) {
    const int m = mt * 16 + c;
    float inv = 0.f;
    if (PRO == PRO_NORM && m < M) inv = 1.0f / sqrtf(a.sumsq_in[m] / (float)K + a.eps);
#pragma unroll
    for (int j = 0; j < GEMM_SPW; ++j) {
      const int k = (step0 + j) * 32 + kb * 8;
      u32x4 v = {0u, 0u, 0u, 0u};
      if (j < nst && m < M && k < K) {
        if (PRO == PRO_BF16) {
          v = *reinterpret_cast<const u32x4*>(static_cast<const bf16*>(a.X) + (size_t)m * K + k);
        } else {
          const float* hp = static_cast<const float*>(a.X) + (size_t)m * K + k;
          const f32x4 h0 = *reinterpret_cast<const f32x4*>(hp), h1 = *reinterpret_cast<const f32x4*>(hp + 4);
          const bf16x8 g = __builtin_bit_cast(bf16x8, *reinterpret_cast<const u32x4*>(a.gain + k));
          bf16x8 o;
#pragma unroll
          for (int e = 0; e < 4; ++e) {
            o[e] = (__bf16)(h0[e] * inv * (float)g[e]);
            o[e + 4] = (__bf16)(h1[e] * inv * (float)g[e + 4]);
          }
          v = __builtin_bit_cast(u32x4, o);
        }
      }
      b[mt][j] = __builtin_bit_cast(bf16x8, v);
    }
  }

  const u32x4* wbase = a.Wp + (size_t)step0 * 64 + lane;
  const size_t pstride = (size_t)a.steps * 64;   // 16-byte units per panel
  // Two-deep software pipeline over the panels: the chunks of panels q and q+1 are in flight; once a chunk is
  // consumed its buffer is refilled with panel q+2.  The sequence runs on across reduction rounds, so the
  // loads never drain at a round's barrier.
  u32x4 av[2][GEMM_SPW];
#pragma unroll
  for (int q = 0; q < 2; ++q)
    if (p0 + q < p1) load_chunk(av[q], wbase + (size_t)(p0 + q) * pstride, nst);

  float ss = 0.f;
  int rb = 0;
  for (int pr = p0; pr < p1; pr += GEMM_RP) {
    f32x4 acc[GEMM_RP][MT];
#pragma unroll
    for (int rp = 0; rp < GEMM_RP; ++rp)
#pragma unroll
      for (int mt = 0; mt < MT; ++mt) acc[rp][mt] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int u = 0; u < GEMM_RP; ++u) {
      if (pr + u < p1) mma_chunk<MT>(acc[u], av[u & 1], b, nst);
      if (pr + u + 2 < p1) load_chunk(av[u & 1], wbase + (size_t)(pr + u + 2) * pstride, nst);
    }

#pragma unroll
    for (int rp = 0; rp < GEMM_RP; ++rp)
#pragma unroll
      for (int mt = 0; mt < MT; ++mt) red[rb][w][rp][mt][lane] = acc[rp][mt];
    __syncthreads();
    for (int item = threadIdx.x; item < GEMM_RP * MT * 64; item += GEMM_THREADS) {
      const int l2 = item & 63, mt = (item >> 6) % MT, rp = item / (64 * MT);
      const int p = pr + rp;
      const int m = mt * 16 + (l2 & 15);
      const bool pair = (EPI == EPI_SILU) && S == 1;   // gate and up sums are needed in one thread
      if (pair && (rp & 1)) continue;
      if (p < p1 && m < M) {
        f32x4 t = red[rb][0][rp][mt][l2], t2 = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int ww = 1; ww < GEMM_WAVES; ++ww) t += red[rb][ww][rp][mt][l2];
        if (pair) {
          t2 = red[rb][0][rp + 1][mt][l2];
#pragma unroll
          for (int ww = 1; ww < GEMM_WAVES; ++ww) t2 += red[rb][ww][rp + 1][mt][l2];
        }
        if (EPI != EPI_PARTIAL && S == 1)
          epi_store<EPI>(a, m, p, l2 >> 4, t, t2, ss);
        else
          *reinterpret_cast<f32x4*>(a.P + ((size_t)s * M + m) * N + (size_t)p * 16 + (l2 >> 4) * 4) = t;
      }
    }
    // with two buffers the next round writes the other one, and nobody can reach the round after that
    // before every thread has passed the next barrier, i.e. has finished reading this buffer
    if (NBUF == 2) rb ^= 1;
    else __syncthreads();
  }
  if (EPI == EPI_PARTIAL) return;

  if (S > 1) {
    // The last of the S workgroups of this panel range to get here adds the slices.  Release our partials,
    // count arrivals, and (last one only) acquire the others' partials.
    __threadfence();
    __syncthreads();
    if (threadIdx.x == 0) {
      const int old = atomicAdd(&a.cnt[idx], 1);
      s_last = (old == S - 1);
      if (old == S - 1) a.cnt[idx] = 0;   // ready for the next launch
    }
    __syncthreads();
    if (!s_last) return;
    __threadfence();
    const int step = (EPI == EPI_SILU) ? 2 : 1;
    for (int item = threadIdx.x; item < (p1 - p0) * MT * 64; item += GEMM_THREADS) {
      const int l2 = item & 63, mt = (item >> 6) % MT, pp = item / (64 * MT);
      if (step == 2 && (pp & 1)) continue;
      const int p = p0 + pp;
      const int m = mt * 16 + (l2 & 15);
      if (m < M) {
        const size_t off = (size_t)m * N + (size_t)p * 16 + (l2 >> 4) * 4;
        f32x4 t = f32x4{0.f, 0.f, 0.f, 0.f}, t2 = f32x4{0.f, 0.f, 0.f, 0.f};
        for (int sl = 0; sl < S; ++sl) {
          const float* ps = a.P + (size_t)sl * M * N + off;
          t += *reinterpret_cast<const f32x4*>(ps);
          if (step == 2) t2 += *reinterpret_cast<const f32x4*>(ps + 16);
        }
        epi_store<EPI>(a, m, p, l2 >> 4, t, t2, ss);
      }
    }
  }

  if (EPI == EPI_RESID) {
    // sum of squares of the updated rows: per workgroup in a fixed order, then across workgroups by the last
    // one to finish (again a counter, no waiting)
    float* sred = reinterpret_cast<float*>(&red[0][0][0][0][0]);
    __syncthreads();
    sred[threadIdx.x] = ss;
    __syncthreads();
    if (threadIdx.x < 16 * MT) {
      const int cc = threadIdx.x & 15, mt = threadIdx.x >> 4;
      float tot = 0.f;
      for (int t = 0; t < GEMM_THREADS; ++t)
        if ((t & 15) == cc && ((t >> 6) % MT) == mt) tot += sred[t];
      a.slots[(size_t)idx * SPEC_MAX_TOKENS + threadIdx.x] = tot;
    }
    __threadfence();
    __syncthreads();
    if (threadIdx.x == 0) {
      const int old = atomicAdd(a.done, 1);
      s_last = (old == Gs - 1);
      if (old == Gs - 1) a.done[0] = 0;
    }
    __syncthreads();
    if (!s_last) return;
    __threadfence();
    if (threadIdx.x < M) {
      float tot = 0.f;
      for (int i = 0; i < Gs; ++i) tot += a.slots[(size_t)i * SPEC_MAX_TOKENS + threadIdx.x];
      a.sumsq_out[threadIdx.x] = tot;
    }
  }
}

template <int TAG, int EPI, int PRO>
static void launch_variant(const GemmPlan& p, const GemmArgs& a, hipStream_t st) {
  dim3 grid(p.Gs * p.S), block(GEMM_THREADS);
  if (p.MT == 1)
    gemm_kernel<1, TAG, 4, EPI, PRO><<<grid, block, 0, st>>>(a);
  else
    gemm_kernel<2, TAG, 2, EPI, PRO><<<grid, block, 0, st>>>(a);
}

hipError_t launch_gemm(const GemmPlan& p, GemmArgs a, int epi, int pro, int tag, hipStream_t st) {
  a.M = p.M; a.N = p.N; a.K = p.K; a.NT = p.NT; a.steps = p.steps; a.S = p.S; a.spw = p.spw; a.Gs = p.Gs;
  const int key = epi * 2 + pro;
  if (tag == 2 && key == EPI_PARTIAL * 2 + PRO_BF16) launch_variant<2, EPI_PARTIAL, PRO_BF16>(p, a, st);
#define GEMM_CASE(T, E, Pm) else if (tag == T && key == E * 2 + Pm) launch_variant<T, E, Pm>(p, a, st);
  GEMM_CASE(0, EPI_PARTIAL, PRO_NORM) GEMM_CASE(1, EPI_PARTIAL, PRO_NORM)
  GEMM_CASE(0, EPI_RESID, PRO_BF16) GEMM_CASE(1, EPI_RESID, PRO_BF16)
  GEMM_CASE(0, EPI_SILU, PRO_NORM) GEMM_CASE(1, EPI_SILU, PRO_NORM)
  GEMM_CASE(0, EPI_F32, PRO_NORM) GEMM_CASE(1, EPI_F32, PRO_NORM)
#undef GEMM_CASE
  else return hipErrorInvalidValue;
  return hipGetLastError();
}

// y[i] = sum_s partials[s][i], slices added in ascending order
__global__ void reduce_partials_kernel(float* __restrict__ y, const float* __restrict__ P, int S, size_t n4) {
  size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= n4) return;
  const f32x4* p = reinterpret_cast<const f32x4*>(P);
  f32x4 t = p[i];
  for (int s = 1; s < S; ++s) t += p[(size_t)s * n4 + i];
  reinterpret_cast<f32x4*>(y)[i] = t;
}

hipError_t launch_reduce_partials(float* y, const float* partials, int S, size_t n, hipStream_t st) {
  size_t n4 = n / 4;   // n = M*N with N % 16 == 0
  reduce_partials_kernel<<<dim3((unsigned)((n4 + 255) / 256)), dim3(256), 0, st>>>(y, partials, S, n4);
  return hipGetLastError();
}

// dst block (panel, step) lane l=(kb*16+r): W[16*panel + r][32*step + 8*kb .. +7]
__global__ void pack_weight_kernel(u32x4* __restrict__ dst, const bf16* __restrict__ src, int N, int K, int steps,
                                   int panel_start, int panel_step) {
  size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;   // 16-byte chunk index within this matrix
  size_t total = (size_t)(N / 16) * steps * 64;
  if (i >= total) return;
  const int lane = (int)(i & 63);
  const size_t blk = i >> 6;
  const int step = (int)(blk % steps);
  const int panel = (int)(blk / steps);
  const int r = lane & 15, kb = lane >> 4;
  const int k = step * 32 + kb * 8;
  u32x4 v = {0u, 0u, 0u, 0u};
  if (k < K) v = *reinterpret_cast<const u32x4*>(src + (size_t)(panel * 16 + r) * K + k);
  const size_t dpanel = (size_t)panel_start + (size_t)panel * panel_step;
  dst[(dpanel * steps + step) * 64 + lane] = v;
}

hipError_t launch_pack_weight(void* dst, const void* src, int N, int K, int panel_start, int panel_step,
                              hipStream_t st) {
  const int steps = (K + 31) / 32;
  size_t total = (size_t)(N / 16) * steps * 64;
  pack_weight_kernel<<<dim3((unsigned)((total + 255) / 256)), dim3(256), 0, st>>>((u32x4*)dst, (const bf16*)src, N, K,
                                                                                  steps, panel_start, panel_step);
  return hipGetLastError();
}

// Streaming-read probe: every workgroup sums a contiguous share with 16-byte loads.
__global__ __launch_bounds__(512) void read_probe_kernel(const u32x4* __restrict__ src, size_t n16, unsigned* out) {
  const size_t per = (n16 + gridDim.x - 1) / gridDim.x;
  size_t b = (size_t)blockIdx.x * per, e = b + per;
  if (e > n16) e = n16;
  unsigned acc = 0;
  size_t i = b + threadIdx.x;
  for (; i + 3 * 512 < e; i += 4 * 512) {
    u32x4 v0 = __builtin_nontemporal_load(src + i), v1 = __builtin_nontemporal_load(src + i + 512);
    u32x4 v2 = __builtin_nontemporal_load(src + i + 1024), v3 = __builtin_nontemporal_load(src + i + 1536);
    acc += v0.x ^ v0.y ^ v0.z ^ v0.w ^ v1.x ^ v1.y ^ v1.z ^ v1.w ^ v2.x ^ v2.y ^ v2.z ^ v2.w ^ v3.x ^ v3.y ^ v3.z ^ v3.w;
  }
  for (; i < e; i += 512) {
    u32x4 v = __builtin_nontemporal_load(src + i);
    acc += v.x ^ v.y ^ v.z ^ v.w;
  }
  if (acc == 0x9E3779B9u) out[0] = acc;   // practically never: keeps the loads alive without a store per thread
}

hipError_t launch_read_probe(const void* src, size_t bytes, void* out, hipStream_t st) {
  read_probe_kernel<<<dim3(SPEC_NUM_CU * 4), dim3(512), 0, st>>>((const u32x4*)src, bytes / 16, (unsigned*)out);
  return hipGetLastError();
}
