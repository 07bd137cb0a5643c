// Prompt (prefill) kernels for gfx950: the only compute-bound part of the decoding workload.
//
// A prompt of C tokens goes through every projection as one dense GEMM Y[C][N] = X[C][K] W^T, so the
// contraction has C flop per weight byte pair and belongs on the matrix cores at full tile size,
// unlike the decode-time projections (<= 32 rows, HBM-bound).  W stays in the panel-packed order the decode
// kernels stream (16 output rows x 32 k per 1 KiB block = one A operand of v_mfma_f32_16x16x32_bf16), so a
// wave loads its weight fragments straight from global memory into registers, three K steps ahead of their
// use.  X is row-major bf16; a 16-token x 32-k block of it gathered with one 16-byte load per lane is exactly
// one B operand, and since the four waves that share a token range all need it, it goes global -> LDS with the
// LDS-direct loads of gfx950 (global_load_lds_dwordx4: lane l lands at base + 16 l, i.e. already in operand
// order) and is read back with one conflict-free ds_read_b128 per fragment.  Keeping the weights out of LDS
// matters: with both operands staged there the kernel was bound by LDS bandwidth.
//
// Tiling: workgroup = 8 waves = 256 tokens x 256 outputs, wave = 128 tokens x 64 outputs (8 x 4 MFMA tiles,
// 128 accumulator registers, two waves per SIMD), K advances 32 per step; X steps go through a ring of
// DG_STAGES LDS buffers of 16 KiB, W steps through a ring of DG_STAGES - 1 register sets.
#include "spec_internal.h"

#define DG_BM 256
#define DG_BN 256
#define DG_THREADS 512
#define DG_STAGES 4
#define DG_STAGE_U4 (16 * 64)          // 16-byte units per LDS stage: 16 activation blocks

enum { DG_EPI_STORE = 0, DG_EPI_RESID = 1, DG_EPI_SWIGLU = 2 };

// EPI: STORE  Y[m][n] = acc (fp32);  RESID  Y[m][n] += acc;  SWIGLU  Z[m][f] = silu(gate) * up (bf16) with the
// gate / up panels interleaved (even panel = gate rows of f-tile j, odd = the matching up rows), N = 2F.
template <int EPI>
__global__ __launch_bounds__(DG_THREADS, 2) void dense_gemm_kernel(const bf16* __restrict__ X,
                                                                   const u32x4* __restrict__ Wp,
                                                                   float* __restrict__ Y, bf16* __restrict__ Z, int M,
                                                                   int N, int K, int NT, int steps, int TM, int cx) {
  __shared__ u32x4 lds[DG_STAGES * DG_STAGE_U4];
  const int w = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), lane = threadIdx.x & 63;   // w: wave-uniform
  // Workgroups are dealt to the 8 XCDs round-robin; XCD x owns tile columns [x cx, (x+1) cx) and walks them in
  // groups of 4 columns x all row tiles, so the 32 workgroups an XCD runs together share 8 x 4 operand strips
  // in its L2.
  const int x = blockIdx.x & 7, j = blockIdx.x >> 3;
  const int TN = (NT + 15) >> 4;
  int nx = TN - x * cx;
  if (nx > cx) nx = cx;
  const int grp = j / (TM * 4), idx = j % (TM * 4);
  int gw = nx - grp * 4;          // columns in this group; its tiles are numbered row-major over them
  if (gw > 4) gw = 4;
  if (gw <= 0 || idx >= TM * gw) return;
  const int tm = idx / gw, tn = x * cx + grp * 4 + idx % gw;

  const int c = lane & 15, kb = lane >> 4;
  const int wn = w & 3, wm = w >> 2;      // wave grid: 4 along the outputs x 2 along the tokens
  // Addresses are a wave-uniform base (scalar registers) plus a 32-bit per-lane offset, which keeps them out of
  // the vector registers the accumulators and fragment rings need.
  const char* wbase[4];                   // this wave's 4 weight panels (clamped rows are computed, never stored)
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    int panel = tn * 16 + wn * 4 + i;
    if (panel > NT - 1) panel = NT - 1;
    wbase[i] = reinterpret_cast<const char*>(Wp + (size_t)panel * steps * 64);
  }
  const unsigned woff = lane * 16;
  const char* xbase = reinterpret_cast<const char*>(X);
  unsigned xoff[2];                       // the 2 activation blocks this wave brings into every LDS stage
#pragma unroll
  for (int i = 0; i < 2; ++i) {
    int m = tm * DG_BM + (w * 2 + i) * 16 + c;
    if (m > M - 1) m = M - 1;
    xoff[i] = (unsigned)m * (unsigned)K * 2u + kb * 16;     // < 2^32: checked by the launcher
  }

  f32x4 acc[4][8];
#pragma unroll
  for (int a = 0; a < 4; ++a)
#pragma unroll
    for (int b = 0; b < 8; ++b) acc[a][b] = f32x4{0.f, 0.f, 0.f, 0.f};

  // Every step issues 2 LDS-direct loads and 4 register loads per wave, in this order, DG_STAGES - 1 steps ahead.
  // Steps past the end reload the last step (into a free buffer / a dead register set), which keeps the count
  // of outstanding loads uniform so that one vmcnt threshold serves every iteration.
  u32x4 wq[DG_STAGES - 1][4];
#define DG_ISSUE(STEP, SET)                                                                                  \
  {                                                                                                          \
    const int st_ = (STEP) < steps ? (STEP) : steps - 1;                                                     \
    u32x4* dst_ = lds + ((STEP) % DG_STAGES) * DG_STAGE_U4 + (w * 2) * 64;                                   \
    const char* xs_ = xbase + (size_t)st_ * 64;                                                              \
    __builtin_amdgcn_global_load_lds(xs_ + xoff[0], dst_, 16, 0, 0);                                         \
    __builtin_amdgcn_global_load_lds(xs_ + xoff[1], dst_ + 64, 16, 0, 0);                                    \
    _Pragma("unroll") for (int i = 0; i < 4; ++i)                                                            \
      asm volatile("global_load_dwordx4 %0, %1, %2"                                                          \
                   : "=v"(wq[SET][i]) : "v"(woff), "s"(wbase[i] + (size_t)st_ * 1024) : "memory");           \
  }
  // The weight loads are inline asm and the barrier is a bare s_barrier behind an explicit vmcnt wait, because
  // the compiler's own bookkeeping would drain every load in flight (it orders nothing behind an LDS-direct
  // load short of vmcnt(0), and so does the fence of __syncthreads).  The wait statement names the register set
  // of the next step as read-write, which is what makes every use of those weights depend on it.
  //
  // One iteration = 32 MFMAs in two halves (tokens 0..63 and 64..127 of the wave's rows).  All 8 waves meet at
  // one barrier per step, so the two waves of a SIMD run in phase and cannot hide each other's LDS latency;
  // instead all activation fragments of step KS + 1 are read from LDS between the halves of step KS (the low
  // half into the registers the first half has just consumed, the high half into a second set), so that their
  // latency passes behind the 16 MFMAs of the second half.
#define DG_ITER(KS, SET, NSET, HC, HN)                                                                       \
  {                                                                                                          \
    bf16x8 a[4];                                                                                             \
    _Pragma("unroll") for (int i = 0; i < 4; ++i) a[i] = __builtin_bit_cast(bf16x8, wq[SET][i]);             \
    _Pragma("unroll") for (int nt = 0; nt < 4; ++nt)                                                         \
      _Pragma("unroll") for (int mt = 0; mt < 4; ++mt)                                                       \
        acc[nt][mt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a[nt], blo[mt], acc[nt][mt], 0, 0, 0);         \
    __builtin_amdgcn_sched_barrier(0);                                                                       \
    /* step KS+1: X is in LDS for all waves, this wave's weights are in wq[NSET] */                          \
    asm volatile("s_waitcnt vmcnt(6)\n\ts_barrier"                                                            \
                 : "+v"(wq[NSET][0]), "+v"(wq[NSET][1]), "+v"(wq[NSET][2]), "+v"(wq[NSET][3])::"memory");    \
    const u32x4* fb = lds + (((KS) + 1) % DG_STAGES) * DG_STAGE_U4 + (wm * 8) * 64 + lane;                   \
    _Pragma("unroll") for (int i = 0; i < 4; ++i) blo[i] = __builtin_bit_cast(bf16x8, fb[i * 64]);           \
    _Pragma("unroll") for (int i = 0; i < 4; ++i) bhi[HN][i] = __builtin_bit_cast(bf16x8, fb[(4 + i) * 64]); \
    __builtin_amdgcn_sched_barrier(0);                                                                       \
    _Pragma("unroll") for (int nt = 0; nt < 4; ++nt)                                                         \
      _Pragma("unroll") for (int mt = 0; mt < 4; ++mt)                                                       \
        acc[nt][4 + mt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a[nt], bhi[HC][mt], acc[nt][4 + mt], 0, 0, 0); \
    __builtin_amdgcn_sched_barrier(0);                                                                       \
    DG_ISSUE((KS) + DG_STAGES - 1, SET)                                                                      \
    __builtin_amdgcn_sched_barrier(0);                                                                       \
  }
  DG_ISSUE(0, 0)
  DG_ISSUE(1, 1)
  DG_ISSUE(2, 2)
  bf16x8 blo[4], bhi[2][4];
  asm volatile("s_waitcnt vmcnt(12)\n\ts_barrier"
               : "+v"(wq[0][0]), "+v"(wq[0][1]), "+v"(wq[0][2]), "+v"(wq[0][3])::"memory");
  {
    const u32x4* fb = lds + (wm * 8) * 64 + lane;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      blo[i] = __builtin_bit_cast(bf16x8, fb[i * 64]);
      bhi[0][i] = __builtin_bit_cast(bf16x8, fb[(4 + i) * 64]);
    }
  }
  int ks = 0;
  for (; ks + 6 <= steps; ks += 6) {
    DG_ITER(ks, 0, 1, 0, 1)
    DG_ITER(ks + 1, 1, 2, 1, 0)
    DG_ITER(ks + 2, 2, 0, 0, 1)
    DG_ITER(ks + 3, 0, 1, 1, 0)
    DG_ITER(ks + 4, 1, 2, 0, 1)
    DG_ITER(ks + 5, 2, 0, 1, 0)
  }
  if (ks < steps) DG_ITER(ks, 0, 1, 0, 1)
  if (ks + 1 < steps) DG_ITER(ks + 1, 1, 2, 1, 0)
  if (ks + 2 < steps) DG_ITER(ks + 2, 2, 0, 0, 1)
  if (ks + 3 < steps) DG_ITER(ks + 3, 0, 1, 1, 0)
  if (ks + 4 < steps) DG_ITER(ks + 4, 1, 2, 0, 1)
#undef DG_ITER
#undef DG_ISSUE
  // The redundant tail loads must not outlive the workgroup's LDS, and their destination registers must not be
  // handed to anything else while they are in flight: naming every set here keeps them allocated until now.
  asm volatile("s_waitcnt vmcnt(0)"
               : "+v"(wq[0][0]), "+v"(wq[0][1]), "+v"(wq[0][2]), "+v"(wq[0][3]), "+v"(wq[1][0]), "+v"(wq[1][1]),
                 "+v"(wq[1][2]), "+v"(wq[1][3]), "+v"(wq[2][0]), "+v"(wq[2][1]), "+v"(wq[2][2]), "+v"(wq[2][3])::"memory");

  // acc[nt][mt][r] = Y[m0 + 16 mt + c][n0 + 16 nt + 4 kb + r]
  const int m0 = tm * DG_BM + wm * 128, n0 = tn * DG_BN + wn * 64;
#pragma unroll
  for (int mt = 0; mt < 8; ++mt) {
    const int m = m0 + mt * 16 + c;
    if (m >= M) continue;
    if (EPI == DG_EPI_SWIGLU) {
      const int F = N >> 1;
#pragma unroll
      for (int nt = 0; nt < 4; nt += 2) {
        const int n = n0 + nt * 16;
        if (n + 32 > N) continue;
        const int f = (n >> 1) + kb * 4;
        const f32x4 g = acc[nt][mt], u = acc[nt + 1][mt];
        bf16 out[4];
#pragma unroll
        for (int q = 0; q < 4; ++q) out[q] = __float2bfloat16(g[q] / (1.0f + __expf(-g[q])) * u[q]);
        *reinterpret_cast<uint2*>(Z + (size_t)m * F + f) = *reinterpret_cast<const uint2*>(out);
      }
    } else {
#pragma unroll
      for (int nt = 0; nt < 4; ++nt) {
        const int n = n0 + nt * 16 + kb * 4;
        if (n >= N) continue;
        f32x4* dst = reinterpret_cast<f32x4*>(Y + (size_t)m * N + n);
        if (EPI == DG_EPI_RESID) *dst = *dst + acc[nt][mt];
        else *dst = acc[nt][mt];
      }
    }
  }
}

hipError_t launch_dense_gemm(const bf16* x, const void* wp, int M, int N, int K, int epi, float* y, bf16* z,
                             hipStream_t st) {
  if ((double)M * K * 2.0 >= 4294967296.0) return hipErrorInvalidValue;   // per-lane activation offsets are 32-bit
  const int NT = N / 16, steps = K / 32;
  const int TM = (M + DG_BM - 1) / DG_BM, TN = (NT + 15) / 16;
  const int cx = (TN + 7) / 8;
  const int groups = (cx + 3) / 4;
  dim3 grid(8 * groups * TM * 4), block(DG_THREADS);
  if (epi == DG_EPI_STORE)
    dense_gemm_kernel<DG_EPI_STORE><<<grid, block, 0, st>>>(x, (const u32x4*)wp, y, z, M, N, K, NT, steps, TM, cx);
  else if (epi == DG_EPI_RESID)
    dense_gemm_kernel<DG_EPI_RESID><<<grid, block, 0, st>>>(x, (const u32x4*)wp, y, z, M, N, K, NT, steps, TM, cx);
  else
    dense_gemm_kernel<DG_EPI_SWIGLU><<<grid, block, 0, st>>>(x, (const u32x4*)wp, y, z, M, N, K, NT, steps, TM, cx);
  return hipGetLastError();
}

// ---------------------------------------------------------------------------------------------------------
// Causal attention of a block of M prompt tokens over the paged KV cache (positions 0 .. len + M - 1, the
// block's own K / V already appended).  Rows are the M*G (token, query head) pairs of one KV head, token-major,
// as in the decode kernel; a workgroup of 8 waves owns 256 consecutive rows, a wave 2 tiles of 16 (two waves
// per SIMD, so that one wave's softmax arithmetic overlaps the other's MFMAs).  K and V pages are in MFMA
// operand order, so every 64-position chunk (= one page) is 32 KiB (head_dim 128) that the workgroup brings
// into LDS once with LDS-direct loads and each wave reads as ready-made fragments: S^T = K Q^T, online softmax
// per query row in the base-2 domain, O^T += V^T P^T.  Chunks beyond the last position a workgroup's rows may
// see are never touched (causal skip), and the workgroups with the longest ranges are scheduled first.
// ---------------------------------------------------------------------------------------------------------
#define PA_WAVES 8
#define PA_QT 2                                  // 16-row tiles per wave
#define PA_ROWS (PA_WAVES * PA_QT * 16)          // rows per workgroup
#define PA_STAGES 2
#define PA_NEG_BIG (-1.0e30f)

// Brings chunk `ch` (64 positions = page block_table[ch]) of one KV head into an LDS stage.  Block b of a chunk:
// b < KB -> K block b (lane-linear in the page), else V block b - KB, whose lane (c, g4) sits at byte
// c*64 + g4*16 of the block.
template <int DH>
__device__ __forceinline__ void pa_issue(const bf16* __restrict__ pool, const int* __restrict__ block_table,
                                         const KvGeom& g, int layer, int kvh, int ch, u32x4* lds_stage, int w,
                                         int lane) {
  constexpr int KB = 4 * (DH / 32), VB = 2 * (DH / 16), LPW = (KB + VB) / PA_WAVES;
  const int c = lane & 15, g4 = lane >> 4;
  const int page = block_table[ch];
  const u32x4* kblk = reinterpret_cast<const u32x4*>(pool + g.offset(page, layer, 0, kvh)) + lane;
  const bf16* vblk = pool + g.offset(page, layer, 1, kvh);
#pragma unroll
  for (int i = 0; i < LPW; ++i) {
    const int b = w * LPW + i;
    const void* src = (b < KB) ? (const void*)(kblk + (size_t)b * 64)
                               : (const void*)(vblk + ((size_t)((b - KB) * 16 + c) * 32 + g4 * 8));
    __builtin_amdgcn_global_load_lds(src, lds_stage + b * 64, 16, 0, 0);
  }
}

template <int DH>
__global__ __launch_bounds__(PA_WAVES * 64, 2) void prefill_attn_kernel(const bf16* __restrict__ q,
                                                                        const bf16* __restrict__ pool,
                                                                        const int* __restrict__ block_table,
                                                                        const int* __restrict__ len_ptr, KvGeom g,
                                                                        int layer, int M, int Hq, float scale_log2e,
                                                                        bf16* __restrict__ out) {
  constexpr int KS = DH / 32;                    // K steps per 16-position tile
  constexpr int KB = 4 * KS;                     // K blocks (1 KiB) per chunk
  constexpr int VB = 2 * (DH / 16);              // V blocks per chunk
  constexpr int NB = KB + VB;
  __shared__ u32x4 lds[PA_STAGES][NB][64];
  const int kvh = blockIdx.y;
  const int rb = gridDim.x - 1 - blockIdx.x;     // longest ranges first
  const int w = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), lane = threadIdx.x & 63;
  const int c = lane & 15, g4 = lane >> 4;
  const int Hkv = g.n_kv_heads, G = Hq / Hkv, R = M * G;
  const int len = len_ptr[0];
  const int r0 = rb * PA_ROWS;
  int rlast = r0 + PA_ROWS - 1;
  if (rlast > R - 1) rlast = R - 1;
  const int nch = ((len + rlast / G) >> 6) + 1;  // chunks this workgroup needs
  int wlast = r0 + (w + 1) * PA_QT * 16 - 1;
  if (wlast > R - 1) wlast = R - 1;
  const int wave_limit = (r0 + w * PA_QT * 16 < R) ? len + wlast / G : -1;

  // per q tile: row of this lane, its visibility limit and its Q fragments.  Rows past the end behave like
  // unmasked rows of zeros (finite arithmetic, never stored).
  int limit[PA_QT];
  bf16x8 qf[PA_QT][KS];
#pragma unroll
  for (int t = 0; t < PA_QT; ++t) {
    const int Rr = r0 + (w * PA_QT + t) * 16 + c;
    const bool valid = Rr < R;
    const int tok = valid ? Rr / G : 0;
    const int head = kvh * G + (valid ? Rr % G : 0);
    limit[t] = valid ? len + tok : 0x7fffffff;
#pragma unroll
    for (int j = 0; j < KS; ++j) {
      u32x4 v = {0u, 0u, 0u, 0u};
      if (valid) v = *reinterpret_cast<const u32x4*>(q + ((size_t)tok * Hq + head) * DH + j * 32 + g4 * 8);
      qf[t][j] = __builtin_bit_cast(bf16x8, v);
    }
  }

  float m_run[PA_QT], l_run[PA_QT];             // running max (base-2 domain) and sum per query row
  f32x4 o[PA_QT][DH / 16];
#pragma unroll
  for (int t = 0; t < PA_QT; ++t) {
    m_run[t] = PA_NEG_BIG;
    l_run[t] = 0.f;
#pragma unroll
    for (int dt = 0; dt < DH / 16; ++dt) o[t][dt] = f32x4{0.f, 0.f, 0.f, 0.f};
  }

  pa_issue<DH>(pool, block_table, g, layer, kvh, 0, &lds[0][0][0], w, lane);
  for (int ch = 0; ch < nch; ++ch) {
    // chunk ch has landed for this wave, then for everybody; all waves are done with the other stage
    asm volatile("s_waitcnt vmcnt(0)\n\ts_barrier" ::: "memory");
    pa_issue<DH>(pool, block_table, g, layer, kvh, ch + 1 < nch ? ch + 1 : nch - 1, &lds[(ch + 1) % PA_STAGES][0][0], w,
                 lane);
    const int pos0 = ch << 6;
    if (pos0 > wave_limit) continue;           // nothing visible for this wave's rows (uniform per wave)
    const u32x4(*st)[64] = lds[ch % PA_STAGES];

    // scores of the 64 positions: s[t][t4][r] = position pos0 + 16 t4 + 4 g4 + r for query row c of tile t
    f32x4 s[PA_QT][4];
#pragma unroll
    for (int t4 = 0; t4 < 4; ++t4) {
      bf16x8 kf[KS];
#pragma unroll
      for (int j = 0; j < KS; ++j) kf[j] = __builtin_bit_cast(bf16x8, st[t4 * KS + j][lane]);
#pragma unroll
      for (int t = 0; t < PA_QT; ++t) {
        s[t][t4] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int j = 0; j < KS; ++j)
          s[t][t4] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(kf[j], qf[t][j], s[t][t4], 0, 0, 0);
      }
    }
    bf16x8 pf[PA_QT][2];                        // P fragments of the two 32-position halves
#pragma unroll
    for (int t = 0; t < PA_QT; ++t) {
      float mx = PA_NEG_BIG;
#pragma unroll
      for (int t4 = 0; t4 < 4; ++t4)
#pragma unroll
        for (int r = 0; r < 4; ++r) {
          const int pos = pos0 + t4 * 16 + g4 * 4 + r;
          const float v = (pos <= limit[t]) ? s[t][t4][r] * scale_log2e : PA_NEG_BIG;
          s[t][t4][r] = v;
          mx = fmaxf(mx, v);
        }
      mx = fmaxf(mx, __shfl_xor(mx, 16));
      mx = fmaxf(mx, __shfl_xor(mx, 32));
      // position 0 is visible to every row, so after the first chunk the running max is a real score and a
      // masked entry (-1e30) underflows to exactly 0
      const float m_new = fmaxf(m_run[t], mx);
      const float corr = __builtin_amdgcn_exp2f(m_run[t] - m_new);
      float psum = 0.f;
#pragma unroll
      for (int t4 = 0; t4 < 4; ++t4)
#pragma unroll
        for (int r = 0; r < 4; ++r) {
          const float pv = __builtin_amdgcn_exp2f(s[t][t4][r] - m_new);
          psum += pv;
          pf[t][t4 >> 1][(t4 & 1) * 4 + r] = (__bf16)pv;
        }
      l_run[t] = l_run[t] * corr + psum;
      m_run[t] = m_new;
#pragma unroll
      for (int dt = 0; dt < DH / 16; ++dt) o[t][dt] *= corr;
    }
#pragma unroll
    for (int h = 0; h < 2; ++h)
#pragma unroll
      for (int dt = 0; dt < DH / 16; ++dt) {
        const bf16x8 vf = __builtin_bit_cast(bf16x8, st[KB + h * (DH / 16) + dt][lane]);
#pragma unroll
        for (int t = 0; t < PA_QT; ++t)
          o[t][dt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(vf, pf[t][h], o[t][dt], 0, 0, 0);
      }
  }
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");   // the redundant tail loads must not outlive the workgroup's LDS

#pragma unroll
  for (int t = 0; t < PA_QT; ++t) {
    float l = l_run[t];
    l += __shfl_xor(l, 16);
    l += __shfl_xor(l, 32);
    const int Rr = r0 + (w * PA_QT + t) * 16 + c;
    if (Rr >= R) continue;
    const int tok = Rr / G, head = kvh * G + Rr % G;
    const float inv = 1.0f / l;
    bf16* dst = out + ((size_t)tok * Hq + head) * DH + g4 * 4;
#pragma unroll
    for (int dt = 0; dt < DH / 16; ++dt) {
      bf16 v4[4];
#pragma unroll
      for (int r = 0; r < 4; ++r) v4[r] = __float2bfloat16(o[t][dt][r] * inv);
      *reinterpret_cast<uint2*>(dst + dt * 16) = *reinterpret_cast<const uint2*>(v4);
    }
  }
}

hipError_t launch_prefill_attention(const bf16* q, const bf16* pool, const int* block_table, const int* len_ptr,
                                    KvGeom g, int layer, int M, int Hq, bf16* out, hipStream_t st) {
  const int Hkv = g.n_kv_heads, G = Hq / Hkv, R = M * G, dh = g.head_dim;
  dim3 grid((R + PA_ROWS - 1) / PA_ROWS, Hkv), block(PA_WAVES * 64);
  const float scale_log2e = 1.4426950408889634f / sqrtf((float)dh);
  if (dh == 128)
    prefill_attn_kernel<128><<<grid, block, 0, st>>>(q, pool, block_table, len_ptr, g, layer, M, Hq, scale_log2e, out);
  else
    prefill_attn_kernel<64><<<grid, block, 0, st>>>(q, pool, block_table, len_ptr, g, layer, M, Hq, scale_log2e, out);
  return hipGetLastError();
}
