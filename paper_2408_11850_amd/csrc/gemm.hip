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
// contiguous range of panels; the slice's steps are dealt evenly to its 8 waves (at most 8 consecutive steps
// each), and a wave keeps the matching activation fragments (the B operand) in registers for the whole kernel.  After every
// round of 4 panels the 8 wave-partials are summed through LDS in a fixed order and written to
// P[s][m][n] (fp32).  Consumers add the S slices in ascending order, so results do not depend
// on timing.
#include <cstring>

#include "spec_internal.h"

#define GEMM_WAVES 8
static_assert(GEMM_WAVES == GEMM_WAVES_PER_GROUP, "consumers of the fused projections count 8 S sums of squares");
#define GEMM_THREADS (GEMM_WAVES * 64)
#ifndef GEMM_RP
#define GEMM_RP 4   // panels per reduction round
#endif
#ifndef GEMM_LOAD
#define GEMM_LOAD(p) __builtin_nontemporal_load(p)
#endif

static int g_num_cu = 256;
int spec_num_cu() { return g_num_cu; }
void spec_set_num_cu(int n) {
  if (n >= 1) g_num_cu = n;
}

GemmPlan gemm_plan(int M, int N, int K, int wgs_per_cu) {
  const int ncu = spec_num_cu();
  GemmPlan p;
  p.M = M; p.N = N; p.K = K;
  p.steps = (K + 31) / 32;
  p.NT = N / 16;
  p.MT = M > 16 ? 2 : 1;
  if (p.MT == 2 || wgs_per_cu < 1) wgs_per_cu = 1;     // the 32-row variant needs a whole CU
  if (wgs_per_cu > 2) wgs_per_cu = 2;
  const int slots = ncu * wgs_per_cu;
  const int spwmax = 8;
  // The K split depends on the shape only, never on wgs_per_cu (always planned for two workgroups per CU), so both
  // launch modes add the same numbers in the same order.  The fewest slices a wave's 8 steps allow are not always
  // the best: K = 28672 gives 14 slices, 36 groups of workgroups for 512 panels and a tail of groups with 15
  // panels instead of 14.2; 16 slices of 7 steps give 32 groups of 16 panels.  Among S .. 2 S slices (at least 4
  // steps per wave) the split with the least work for the busiest wave is taken: panels per group x steps per wave.
  const int smin = (p.steps + GEMM_WAVES * spwmax - 1) / (GEMM_WAVES * spwmax);
  long long best = -1;
  p.S = smin;
  for (int S = smin; S <= 2 * smin; ++S) {
    const int spw = (p.steps + GEMM_WAVES * S - 1) / (GEMM_WAVES * S);
    if (S > smin && spw < 4) break;
    int Gs = 2 * ncu / S;
    if (Gs < 1) Gs = 1;
    if (Gs > p.NT) Gs = p.NT;
    const long long cost = (long long)((p.NT + Gs - 1) / Gs) * spw;
    if (best < 0 || cost < best) best = cost, p.S = S;
  }
  // small matrices: cut K finer until every workgroup slot (at two per CU) has work
  while (p.S * p.NT < 2 * ncu && (p.steps + GEMM_WAVES * p.S * 2 - 1) / (GEMM_WAVES * p.S * 2) >= 2) p.S *= 2;
  p.spw = (p.steps + GEMM_WAVES * p.S - 1) / (GEMM_WAVES * p.S);   // most steps a wave takes
  p.Gs = slots / p.S;
  if (p.Gs < 1) p.Gs = 1;
  if (p.Gs > p.NT) p.Gs = p.NT;
  return p;
}

// Loads / multiplies one chunk of 8 K-steps (steps CH*8 .. CH*8+7 of the wave's range) of one panel.
__device__ __forceinline__ void load_chunk(u32x4 (&a)[8], const u32x4* __restrict__ wp, int first, int nst) {
#pragma unroll
  for (int j = 0; j < 8; ++j)
    if (first + j < nst) a[j] = GEMM_LOAD(wp + (size_t)(first + j) * 64);
}

template <int MT, int SPWMAX, int CH>
__device__ __forceinline__ void mma_chunk(f32x4 (&acc)[MT], const u32x4 (&a)[8], const bf16x8 (&b)[MT][SPWMAX],
                                          int nst) {
#pragma unroll
  for (int j = 0; j < 8; ++j)
    if (CH * 8 + j < nst) {
      bf16x8 av = __builtin_bit_cast(bf16x8, a[j]);
#pragma unroll
      for (int mt = 0; mt < MT; ++mt)
        acc[mt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(av, b[mt][CH * 8 + j], acc[mt], 0, 0, 0);
    }
}

// TAG only names the instantiation (0 = target model, 1 = draft model, 2 = stand-alone call) so
// that profilers list the two models' launches separately.
// WPE = waves per SIMD the register budget is sized for.  The 16-row variant is held to 128 VGPRs (WPE 4) so
// that two workgroups share a CU: 16 waves per CU hide the HBM latency far better than 8 (measured 6.9 vs
// 5.9 TB/s on the gate/up matrix), and the second slot can also go to the other stream's kernel.
// ---- prologues of the single-token projections (PRO != PRO_NONE, M = 1) ------------------------------------
// A wave forms the activation values of its own K range (at most 256 columns): lane l the four columns
// k0 + 4 l .. + 3, all loads of a lane independent of each other.  The bf16 results go through LDS into operand
// order.  Every sum runs in the order the stand-alone kernels use (K slices ascending), so the values are the ones
// the three-kernel chain would produce.
__device__ __forceinline__ unsigned pack_bf16x2(float a, float b) {
  const bf16 x = __float2bfloat16(a), y = __float2bfloat16(b);
  return (unsigned)__builtin_bit_cast(unsigned short, x) | ((unsigned)__builtin_bit_cast(unsigned short, y) << 16);
}

// h_in + sum of the K slices (ascending), four independent loads in flight
__device__ __forceinline__ f32x4 sum_slices(f32x4 t, const f32x4* __restrict__ P4, size_t sstride4, int S) {
  int s = 0;
  for (; s + 4 <= S; s += 4) {
    const f32x4 p0 = P4[(size_t)(s + 0) * sstride4], p1 = P4[(size_t)(s + 1) * sstride4];
    const f32x4 p2 = P4[(size_t)(s + 2) * sstride4], p3 = P4[(size_t)(s + 3) * sstride4];
    t += p0; t += p1; t += p2; t += p3;
  }
  for (; s < S; ++s) t += P4[(size_t)s * sstride4];
  return t;
}

template <int PRO>
__device__ __forceinline__ void prologue_values(const GemmPro& pro, int K, int k, bool valid, bool first_group, int ws,
                                                int lane, uint2* __restrict__ dst) {
  f32x4 r = {0.f, 0.f, 0.f, 0.f};
  if (PRO == PRO_ADDNORM) {
    // residual add, sums of squares, x' = bf16(h * gain) (the consumers of this projection apply 1 / rms)
    f32x4 t = {0.f, 0.f, 0.f, 0.f};
    if (valid) {
      t = *reinterpret_cast<const f32x4*>(pro.h_in + k);
      if (pro.part) t = sum_slices(t, reinterpret_cast<const f32x4*>(pro.part) + (k >> 2), (size_t)(K >> 2), pro.S);
      const bf16* g = pro.gain + k;
      r = f32x4{t.x * __bfloat162float(g[0]), t.y * __bfloat162float(g[1]), t.z * __bfloat162float(g[2]),
                t.w * __bfloat162float(g[3])};
    }
    if (first_group) {
      if (valid) *reinterpret_cast<f32x4*>(pro.h_out + k) = t;
      float ss = t.x * t.x + t.y * t.y + t.z * t.z + t.w * t.w;
#pragma unroll
      for (int o = 32; o > 0; o >>= 1) ss += __shfl_xor(ss, o);
      if (lane == 0) pro.ssq_out[ws] = ss;
    }
  } else if (PRO == PRO_SWIGLU) {
    if (valid) {
      const int gc = (k >> 4) * 32 + (k & 15);          // gate panel of 16 columns, then the up panel
      const f32x4 zero = {0.f, 0.f, 0.f, 0.f};
      const f32x4* P4 = reinterpret_cast<const f32x4*>(pro.part + gc);
      const f32x4 g = sum_slices(zero, P4, (size_t)(K >> 1), pro.S);
      const f32x4 u = sum_slices(zero, P4 + 4, (size_t)(K >> 1), pro.S);
      const float inv = pro.rs.inv(0);
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const float gv = g[i] * inv, uv = u[i] * inv;
        r[i] = gv / (1.0f + __expf(-gv)) * uv;
      }
    }
  }
  dst[0] = make_uint2(pack_bf16x2(r.x, r.y), pack_bf16x2(r.z, r.w));
}

template <int MT, int SPWMAX, int TAG, int WPE, int PRO>
__global__ __launch_bounds__(GEMM_THREADS, WPE) void gemm_partial_kernel(const bf16* __restrict__ X,
                                                                    const u32x4* __restrict__ Wp,
                                                                    float* __restrict__ P, int M, int N, int K,
                                                                    int NT, int steps, int S, int spw, int Gs,
                                                                    GemmPro pro) {
  static_assert(PRO == PRO_NONE || MT == 1, "the fused prologues exist for single-token forwards only");
  constexpr int NCH = SPWMAX / 8;            // chunks per panel
  constexpr int UNITS = GEMM_RP * NCH;       // chunks per reduction round (even)
  constexpr int NBUF = (MT == 1) ? 2 : 1;    // LDS reduction buffers: two let a round end with a single barrier
  __shared__ f32x4 red[NBUF][GEMM_WAVES][GEMM_RP][MT][64];
  const int s = blockIdx.x % S;
  const int idx = blockIdx.x / S;
  const int p0 = (int)((long long)idx * NT / Gs);
  const int p1 = (int)((long long)(idx + 1) * NT / Gs);
  const int w = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int c = lane & 15, kb = lane >> 4;
  if (pro.stamp && threadIdx.x == 0)
    atomicMax(pro.stamp + 2 * (blockIdx.x % STAMP_WAYS), ~(unsigned long long)wall_clock64());
  // the K steps are dealt evenly to the S * 8 waves that share a panel: floor / ceil of steps / (8 S) each
  const int ws = s * GEMM_WAVES + w, nws = S * GEMM_WAVES;
  const int step0 = (int)((long long)ws * steps / nws);
  const int nst = (int)((long long)(ws + 1) * steps / nws) - step0;   // <= spw <= SPWMAX

  const u32x4* wbase = Wp + (size_t)step0 * 64 + lane;
  const size_t pstride = (size_t)steps * 64;   // 16-byte units per panel
  // Two-deep software pipeline over the chunk sequence (panel-major, NCH chunks per panel): chunks q and
  // q+1 are in flight; once chunk q is consumed its buffer is refilled with chunk q+2.  The sequence runs on
  // across reduction rounds, so the loads never drain at a round's barrier.  The first two chunks are requested
  // before anything else: whatever the activations cost (a plain load, or a fused prologue with dependent loads
  // of its own) then runs under the start of the weight stream.
  u32x4 a[2][8];
#pragma unroll
  for (int q = 0; q < 2; ++q)
    if (p0 + q / NCH < p1) load_chunk(a[q], wbase + (size_t)(p0 + q / NCH) * pstride, (q % NCH) * 8, nst);

  // activation fragments of this wave's K range, kept for the whole kernel
  bf16x8 b[MT][SPWMAX];
  if (PRO == PRO_NONE) {
#pragma unroll
    for (int mt = 0; mt < MT; ++mt)
#pragma unroll
      for (int j = 0; j < SPWMAX; ++j) {
        const int m = mt * 16 + c;
        const int k = (step0 + j) * 32 + kb * 8;
        u32x4 v = {0u, 0u, 0u, 0u};
        if (j < nst && m < M && k < K) v = *reinterpret_cast<const u32x4*>(X + (size_t)m * K + k);
        b[mt][j] = __builtin_bit_cast(bf16x8, v);
      }
  } else {
    // the wave's (at most) 256 columns: formed four per lane, handed over in operand order through LDS (the
    // reduction buffer is not in use yet)
    unsigned short* stage = reinterpret_cast<unsigned short*>(&red[0][0][0][0][0]) + w * (SPWMAX * 32);
    const int kk = step0 * 32 + 4 * lane;
    const bool valid = 4 * lane < nst * 32 && kk < K;
    prologue_values<PRO>(pro, K, kk, valid, idx == 0, ws, lane, reinterpret_cast<uint2*>(stage) + lane);
    __syncthreads();
#pragma unroll
    for (int j = 0; j < SPWMAX; ++j) {
      u32x4 v = {0u, 0u, 0u, 0u};
      if (j < nst && c == 0) v = *reinterpret_cast<const u32x4*>(stage + j * 32 + kb * 8);
      b[0][j] = __builtin_bit_cast(bf16x8, v);
    }
    __syncthreads();   // the staging area is the reduction buffer of the first round
  }

  int rb = 0;
  for (int pr = p0; pr < p1; pr += GEMM_RP) {
    f32x4 acc[GEMM_RP][MT];
#pragma unroll
    for (int rp = 0; rp < GEMM_RP; ++rp)
#pragma unroll
      for (int mt = 0; mt < MT; ++mt) acc[rp][mt] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int u = 0; u < UNITS; ++u) {
      if (pr + u / NCH < p1) {
        if (u % NCH == 0) mma_chunk<MT, SPWMAX, 0>(acc[u / NCH], a[u & 1], b, nst);
        else mma_chunk<MT, SPWMAX, (NCH > 1 ? 1 : 0)>(acc[u / NCH], a[u & 1], b, nst);
      }
      const int pn = pr + (u + 2) / NCH;
      if (pn < p1) load_chunk(a[u & 1], wbase + (size_t)pn * pstride, ((u + 2) % NCH) * 8, nst);
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
      if (p < p1 && m < M) {
        f32x4 t = red[rb][0][rp][mt][l2];
#pragma unroll
        for (int ww = 1; ww < GEMM_WAVES; ++ww) t += red[rb][ww][rp][mt][l2];
        *reinterpret_cast<f32x4*>(P + ((size_t)s * M + m) * N + (size_t)p * 16 + (l2 >> 4) * 4) = t;
      }
    }
    // with two buffers the next round writes the other one, and nobody can reach the round after that
    // before every thread has passed the next barrier, i.e. has finished reading this buffer
    if (NBUF == 2) rb ^= 1;
    else __syncthreads();
  }
  if (pro.stamp && threadIdx.x == 0)
    atomicMax(pro.stamp + 2 * (blockIdx.x % STAMP_WAYS) + 1, (unsigned long long)wall_clock64());
}

template <int TAG, int PRO>
static void launch_tagged(const GemmPlan& p, const bf16* x, const void* wp, float* partials, hipStream_t st,
                          const GemmPro& pro) {
  dim3 grid(p.Gs * p.S), block(GEMM_THREADS);
  if (p.MT == 1)
    gemm_partial_kernel<1, 8, TAG, 4, PRO><<<grid, block, 0, st>>>(x, (const u32x4*)wp, partials, p.M, p.N, p.K, p.NT,
                                                                     p.steps, p.S, p.spw, p.Gs, pro);
  else if (PRO == PRO_NONE)
    gemm_partial_kernel<2, 8, TAG, 2, PRO_NONE><<<grid, block, 0, st>>>(x, (const u32x4*)wp, partials, p.M, p.N, p.K,
                                                                          p.NT, p.steps, p.S, p.spw, p.Gs, pro);
}

hipError_t launch_gemm_partials(const GemmPlan& p, const bf16* x, const void* wp, float* partials, hipStream_t st,
                                int tag, unsigned long long* stamp) {
  GemmPro none;
  memset(&none, 0, sizeof(none));
  none.stamp = stamp;
  if (tag == 0) launch_tagged<0, PRO_NONE>(p, x, wp, partials, st, none);
  else if (tag == 1) launch_tagged<1, PRO_NONE>(p, x, wp, partials, st, none);
  else launch_tagged<2, PRO_NONE>(p, x, wp, partials, st, none);
  return hipGetLastError();
}

template <int TAG>
static void launch_fused_tagged(const GemmPlan& p, const GemmPro& pro, const void* wp, float* partials, hipStream_t st) {
  if (pro.kind == PRO_ADDNORM) launch_tagged<TAG, PRO_ADDNORM>(p, nullptr, wp, partials, st, pro);
  else launch_tagged<TAG, PRO_SWIGLU>(p, nullptr, wp, partials, st, pro);
}

hipError_t launch_gemm_fused(const GemmPlan& p, const GemmPro& pro, const void* wp, float* partials, hipStream_t st,
                             int tag) {
  if (p.M != 1 || p.MT != 1 || pro.kind < PRO_ADDNORM || pro.kind > PRO_SWIGLU || (p.K & 3)) return hipErrorInvalidValue;
  if (tag == 0) launch_fused_tagged<0>(p, pro, wp, partials, st);
  else launch_fused_tagged<1>(p, pro, wp, partials, st);
  return hipGetLastError();
}

// y[i] = sum_s partials[s][i], slices added in ascending order; with a row scale, row i / N of the sum is
// multiplied by it (N % 4 == 0)
__global__ void reduce_partials_kernel(float* __restrict__ y, const float* __restrict__ P, int S, size_t n4, RowScale rs,
                                       int N4) {
  size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= n4) return;
  const f32x4* p = reinterpret_cast<const f32x4*>(P);
  // slices in groups of four independent loads, added in ascending order
  f32x4 v[4];
#pragma unroll
  for (int k = 0; k < 4; ++k) v[k] = (k < S) ? p[(size_t)k * n4 + i] : f32x4{0.f, 0.f, 0.f, 0.f};
  const float inv = rs.ssq ? rs.inv((int)(i / (size_t)N4)) : 1.0f;
  f32x4 t = v[0];
#pragma unroll
  for (int k = 1; k < 4; ++k)
    if (k < S) t += v[k];
  for (int s0 = 4; s0 < S; s0 += 4) {
#pragma unroll
    for (int k = 0; k < 4; ++k) v[k] = (s0 + k < S) ? p[(size_t)(s0 + k) * n4 + i] : f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int k = 0; k < 4; ++k)
      if (s0 + k < S) t += v[k];
  }
  if (rs.ssq) t *= inv;
  reinterpret_cast<f32x4*>(y)[i] = t;
}

hipError_t launch_reduce_partials(float* y, const float* partials, int S, size_t n, hipStream_t st, RowScale rs, int N) {
  size_t n4 = n / 4;   // n = M*N with N % 16 == 0
  if (rs.ssq && N < 4) return hipErrorInvalidValue;
  reduce_partials_kernel<<<dim3((unsigned)((n4 + 255) / 256)), dim3(256), 0, st>>>(y, partials, S, n4, rs,
                                                                                   rs.ssq ? N / 4 : 1);
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
  read_probe_kernel<<<dim3(spec_num_cu() * 4), dim3(512), 0, st>>>((const u32x4*)src, bytes / 16, (unsigned*)out);
  return hipGetLastError();
}
