// Prompt (prefill) kernels for gfx950: the only compute-bound part of the decoding workload.
//
// A prompt of C tokens goes through every projection as one dense GEMM Y[C][N] = X[C][K] W^T, so the
// contraction has C flop per weight byte pair and belongs on the matrix cores at full tile size,
// unlike the decode-time projections (<= 32 rows, HBM-bound).  W stays in the panel-packed order the decode
// kernels stream (16 output rows x 32 k per 1 KiB block = one A operand of v_mfma_f32_16x16x32_bf16); X is
// row-major bf16, and a 16-token x 32-k block of it gathered with one 16-byte load per lane is exactly one
// B operand.
//
// Tiling: workgroup = 4 waves (one per SIMD, 512 registers each) = 256 tokens x 256 outputs; wave w owns the
// outputs 64 w .. 64 w + 63 for all 256 tokens: 4 x 16 MFMA tiles whose 256 accumulator registers fill the
// AGPR file.  Measured on this part, a CU moves about 25 bytes per clock from L2 and about 62 from LDS, so the
// tile is built to need the least of both per MFMA:
//   * every weight fragment is used by exactly one wave, which loads it straight from global memory into
//     registers three K steps ahead (no LDS traffic, no duplicate loads), through a ring of four register sets;
//   * X is needed by all four waves and goes global -> LDS once per workgroup with the LDS-direct loads of
//     gfx950 (global_load_lds_dwordx4: lane l lands at base + 16 l), whole 128-byte lines at a time (8 token
//     rows x 64 k per instruction, so L2 is asked for every line once); a wave reads each of its 16 fragments
//     back with one ds_read_b128 (free of bank conflicts).
// Per 32-wide K step that is 32 KiB from L2 and 80 KiB through LDS for 64 MFMAs per wave (1024 MFMA cycles).
//
// The inner loop is inline asm with hand-placed waits.  The compiler cannot be trusted with it: it drains every
// load in flight behind an LDS-direct load (vmcnt(0)), shuffles accumulators between register files when all
// 256 AGPRs are live, and sinks LDS reads to just before their use.  Every asm statement names the registers
// it defines or that a wait makes valid, so the compiler still sees all data flow.
#include "spec_internal.h"

#define DG_BM 256
#define DG_BN 256
#define DG_THREADS 256
// LDS ring of X: a stage holds two K steps (64 k) of the 256 tokens.  Per 16-token tile two 1 KiB blocks (rows
// 0-7 and rows 8-15, each [8 k-chunks of 16 bytes][8 rows]).  A fragment read takes 128 contiguous bytes from
// each block per 16 lanes; SQ_LDS_BANK_CONFLICT is 0 for this layout (and for the blocks 1280 bytes apart), while
// blocks 1088 or 1152 bytes apart double the LDS cycles.
#define DG_STAGES 3
#define DG_HALF_BYTES 1024
#define DG_TILE_BYTES (2 * DG_HALF_BYTES)
#define DG_STAGE_BYTES (16 * DG_TILE_BYTES)

enum { DG_EPI_STORE = 0, DG_EPI_RESID = 1, DG_EPI_SWIGLU = 2, DG_EPI_ROPE128 = 3, DG_EPI_ROPE64 = 4 };

// What the QKV epilogue needs to rotate q and k and to append k and v to the paged cache.
struct DenseRope {
  bf16* q;                    // [M][Hq][dh]
  bf16* pool;                 // KV pages
  const int* block_table;
  const int* len_ptr;         // position of token 0 of the block
  const float2* tab;          // [M][dh/2] (cos, sin) for positions len .. len + M - 1
  KvGeom g;
  int layer, Hq;
};

typedef __attribute__((address_space(3))) u32x4 dg_lds_u32x4;

// EPI: STORE  Y[m][n] = acc (fp32);  RESID  Y[m][n] += acc;  SWIGLU  Z[m][f] = silu(gate) * up (bf16) with the
// gate / up panels interleaved (even panel = gate rows of f-tile j, odd = the matching up rows), N = 2F;
// ROPE128 / ROPE64 (fused QKV projection, head_dim 128 / 64): rotate the q and k heads, store q as bf16 and
// k, v into the paged cache in operand order.  For the rotation a wave must hold columns e and e + dh/2 of a
// head: with head_dim 64 its 64 columns are one head; with head_dim 128 the two waves of a head take the
// 16-column panels {0, 1, 4, 5} and {2, 3, 6, 7}.  Either way accumulator tiles nt and nt + 2 pair up.
template <int EPI>
__global__ __launch_bounds__(DG_THREADS, 1) void dense_gemm_kernel(const bf16* __restrict__ X,
                                                                   const u32x4* __restrict__ Wp,
                                                                   float* __restrict__ Y, bf16* __restrict__ Z, int M,
                                                                   int N, int K, int NT, int steps, int TM, int cx,
                                                                   DenseRope ra) {
  extern __shared__ u32x4 lds[];          // DG_STAGES * DG_STAGE_BYTES
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
  // Addresses are a wave-uniform base (scalar registers) plus a 32-bit per-lane offset.
  const char* wbase[4];                   // this wave's 4 weight panels (clamped rows are computed, never stored)
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    int panel = tn * 16 + w * 4 + i;
    if (EPI == DG_EPI_ROPE128) panel = tn * 16 + (w >> 1) * 8 + (w & 1) * 2 + (i & 1) + (i >> 1) * 4;
    if (panel > NT - 1) panel = NT - 1;
    wbase[i] = reinterpret_cast<const char*>(Wp + (size_t)panel * steps * 64);
  }
  const unsigned woff = lane * 16;
  const char* xbase = reinterpret_cast<const char*>(X);
  // X moves global -> LDS in whole 128-byte lines: one LDS-direct load covers 8 token rows x 64 k (lane = k-chunk
  // * 8 + row), so that L2 sees every line of X once (a 16-row x 32-k load would ask for each line twice, half
  // used).  Per stage the wave issues 8 of them: token tiles 4w .. 4w+3, rows 0-7 and 8-15 of each.
  unsigned xoff[8];
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    int m = tm * DG_BM + (w * 4 + i / 2) * 16 + (i & 1) * 8 + (lane & 7);
    if (m > M - 1) m = M - 1;
    xoff[i] = (unsigned)m * (unsigned)K * 2u + (lane >> 3) * 16;     // < 2^32: checked by the launcher
  }
  // fragment (tile mt, step half h) of lane (c, kb): tile mt, block c / 8, chunk 4 h + kb, row c % 8
  const unsigned lds_rd = (unsigned)(size_t)(dg_lds_u32x4*)lds + (c >> 3) * DG_HALF_BYTES + kb * 128 + (c & 7) * 16;

  f32x4 acc[4][16];
#pragma unroll
  for (int a = 0; a < 4; ++a)
#pragma unroll
    for (int b = 0; b < 16; ++b) acc[a][b] = f32x4{0.f, 0.f, 0.f, 0.f};

  // Load schedule per wave: iteration j issues 4 of the 8 LDS-direct loads of X stage j/2 + 2 (K steps 2(j/2)+4
  // and +5) and the 4 register loads of W step j+3, alternating, one after every second token tile, i.e. 8 MFMAs
  // apart: the address unit takes about 30 cycles per 1 KiB wave load, and a wave that issues loads back to back
  // sits in the issue stage (issuing no MFMAs) until the unit has taken them all.  Vector-memory operations
  // complete in order.  Steps past the end reload the last step (into a free buffer / a dead register set),
  // which keeps the count of outstanding loads uniform so that one vmcnt threshold serves every iteration.
  u32x4 wq[4][4];      // W fragments of steps j .. j+3 (set = step % 4)
  u32x4 bq[16];        // X fragments of the current step; each is refilled for the next step once consumed
  const unsigned xfix = (lane >> 5) * 64;   // lanes of the second K step of a stage: fall back to the first one
#define DG_LOAD_X(PG, J)   /* instruction J (0..7) of X stage PG: token tile 4w + J/2, rows 8 (J%2) .. + 7 */    \
  {                                                                                                          \
    const int st_ = 2 * (PG) < steps ? 2 * (PG) : (steps - 1) & ~1;                                          \
    const unsigned fix_ = st_ + 1 < steps ? 0u : xfix;   /* odd K-step count: never read past the row's end */ \
    __builtin_amdgcn_global_load_lds(                                                                        \
        xbase + (size_t)st_ * 64 + (xoff[J] - fix_),                                                         \
        lds + (((PG) % DG_STAGES) * DG_STAGE_BYTES + (w * 4 + (J) / 2) * DG_TILE_BYTES + ((J) & 1) * DG_HALF_BYTES) / 16, \
        16, 0, 0);                                                                                           \
  }
#define DG_LOAD_W(STEP, SET, I)                                                                              \
  {                                                                                                          \
    const int st_ = (STEP) < steps ? (STEP) : steps - 1;                                                     \
    asm volatile("global_load_dwordx4 %0, %1, %2"                                                            \
                 : "=v"(wq[SET][I]) : "v"(woff), "s"(wbase[I] + (size_t)st_ * 1024) : "memory");             \
  }
#define DG_MFMA(ACC, A, B)                                                                                   \
  asm volatile("v_mfma_f32_16x16x32_bf16 %0, %1, %2, %0" : "+a"(ACC) : "v"(A), "v"(B))
  // One iteration = K step KS (KS % 4 == U, so that the register sets are compile-time names).  At its top: this
  // wave's loads issued up to iteration KS-2 have landed (the 8 of iteration KS-1 may be in flight), i.e. W step
  // KS+1 and X step KS+1's stage, then the barrier: that stage is in LDS for everybody, and everybody is past
  // reading the stage this iteration's LDS-direct loads refill.  The 16 token tiles follow; fragment mt of step
  // KS was read 16 LDS reads ago (lgkmcnt(15)), feeds 4 MFMAs and is at once re-read for step KS+1, so that every
  // LDS read has 60 MFMAs to arrive.
#define DG_ITER(KS, U)                                                                                       \
  {                                                                                                          \
    asm volatile("s_waitcnt vmcnt(8)\n\ts_barrier"                                                            \
                 : "+v"(wq[((U) + 1) % 4][0]), "+v"(wq[((U) + 1) % 4][1]), "+v"(wq[((U) + 1) % 4][2]),       \
                   "+v"(wq[((U) + 1) % 4][3])::"memory");                                                    \
    const unsigned rd_ = lds_rd + ((((KS) + 1) >> 1) % DG_STAGES) * DG_STAGE_BYTES + (((KS) + 1) & 1) * 512;  \
    _Pragma("unroll") for (int mt = 0; mt < 16; ++mt) {                                                      \
      asm volatile("s_waitcnt lgkmcnt(15)" : "+v"(bq[mt]));                                                  \
      _Pragma("unroll") for (int nt = 0; nt < 4; ++nt) DG_MFMA(acc[nt][mt], wq[U][nt], bq[mt]);              \
      asm volatile("ds_read_b128 %0, %1 offset:%2" : "=v"(bq[mt]) : "v"(rd_), "n"(mt * DG_TILE_BYTES));      \
      if (mt % 4 == 1) DG_LOAD_X((KS) / 2 + 2, ((U) & 1) * 4 + mt / 4)                                       \
      if (mt % 4 == 3) DG_LOAD_W((KS) + 3, ((U) + 3) % 4, mt / 4)                                            \
    }                                                                                                        \
  }
  // prologue: X stages 0 and 1 (K steps 0..3) and W steps 0..2, all landed before the first iteration
#pragma unroll
  for (int j8 = 0; j8 < 8; ++j8) {
    DG_LOAD_X(0, j8)
    DG_LOAD_X(1, j8)
  }
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    DG_LOAD_W(0, 0, i)
    DG_LOAD_W(1, 1, i)
    DG_LOAD_W(2, 2, i)
  }
  asm volatile("s_waitcnt vmcnt(0)\n\ts_barrier"
               : "+v"(wq[0][0]), "+v"(wq[0][1]), "+v"(wq[0][2]), "+v"(wq[0][3]), "+v"(wq[1][0]), "+v"(wq[1][1]),
                 "+v"(wq[1][2]), "+v"(wq[1][3]), "+v"(wq[2][0]), "+v"(wq[2][1]), "+v"(wq[2][2]), "+v"(wq[2][3])::"memory");
#pragma unroll
  for (int mt = 0; mt < 16; ++mt)
    asm volatile("ds_read_b128 %0, %1 offset:%2" : "=v"(bq[mt]) : "v"(lds_rd), "n"(mt * DG_TILE_BYTES));
  int ks = 0;
  for (; ks + 4 <= steps; ks += 4) {
    DG_ITER(ks, 0)
    DG_ITER(ks + 1, 1)
    DG_ITER(ks + 2, 2)
    DG_ITER(ks + 3, 3)
  }
  if (ks < steps) DG_ITER(ks, 0)
  if (ks + 1 < steps) DG_ITER(ks + 1, 1)
  if (ks + 2 < steps) DG_ITER(ks + 2, 2)
#undef DG_ITER
#undef DG_MFMA
#undef DG_LOAD_X
#undef DG_LOAD_W
  // The redundant tail loads must not outlive the workgroup's LDS, and the registers they (and the last LDS
  // reads) target must not be handed to anything else while they are in flight: naming them here keeps them
  // allocated until everything has landed.  The s_nops cover the distance the hardware wants between the last
  // MFMA and a read of its accumulator; the compiler does not know that the asm statements above are MFMAs and
  // would otherwise be free to read an accumulator right behind the one that wrote it, so every accumulator is
  // passed through a statement that follows the s_nops.
  asm volatile("s_waitcnt vmcnt(0) lgkmcnt(0)\n\ts_nop 15\n\ts_nop 15"
               : "+v"(wq[0][0]), "+v"(wq[0][1]), "+v"(wq[0][2]), "+v"(wq[0][3]), "+v"(wq[1][0]), "+v"(wq[1][1]),
                 "+v"(wq[1][2]), "+v"(wq[1][3]), "+v"(wq[2][0]), "+v"(wq[2][1]), "+v"(wq[2][2]), "+v"(wq[2][3])::"memory");
  asm volatile("" : "+v"(wq[3][0]), "+v"(wq[3][1]), "+v"(wq[3][2]), "+v"(wq[3][3]));
  asm volatile("" : "+v"(bq[0]), "+v"(bq[1]), "+v"(bq[2]), "+v"(bq[3]), "+v"(bq[4]), "+v"(bq[5]), "+v"(bq[6]),
               "+v"(bq[7]), "+v"(bq[8]), "+v"(bq[9]), "+v"(bq[10]), "+v"(bq[11]), "+v"(bq[12]), "+v"(bq[13]),
               "+v"(bq[14]), "+v"(bq[15]));
#pragma unroll
  for (int nt = 0; nt < 4; ++nt)
    asm volatile("" : "+a"(acc[nt][0]), "+a"(acc[nt][1]), "+a"(acc[nt][2]), "+a"(acc[nt][3]), "+a"(acc[nt][4]),
                 "+a"(acc[nt][5]), "+a"(acc[nt][6]), "+a"(acc[nt][7]), "+a"(acc[nt][8]), "+a"(acc[nt][9]),
                 "+a"(acc[nt][10]), "+a"(acc[nt][11]), "+a"(acc[nt][12]), "+a"(acc[nt][13]), "+a"(acc[nt][14]),
                 "+a"(acc[nt][15]));

  // acc[nt][mt][r] = Y[m0 + 16 mt + c][n0 + 16 nt + 4 kb + r]
  const int m0 = tm * DG_BM, n0 = tn * DG_BN + w * 64;
  if (EPI == DG_EPI_ROPE128 || EPI == DG_EPI_ROPE64) {
    constexpr int DH = EPI == DG_EPI_ROPE128 ? 128 : 64;
    const int Hkv = ra.g.n_kv_heads;
    const int head = tn * (DG_BN / DH) + (DH == 128 ? (w >> 1) : w);
    if (head >= ra.Hq + 2 * Hkv) return;
    const int len = ra.len_ptr[0];
    const int ebase = (DH == 128 ? (w & 1) * 32 : 0) + kb * 4;     // + 16 nt + r: column inside the head, < dh/2
#pragma unroll
    for (int mt = 0; mt < 16; ++mt) {
      const int m = m0 + mt * 16 + c;
      if (m >= M) continue;
      const int pos = len + m;
#pragma unroll
      for (int nt = 0; nt < 2; ++nt) {
        const int e0 = ebase + nt * 16;
        f32x4 x0 = acc[nt][mt], x1 = acc[nt + 2][mt];               // columns e0 + r and e0 + r + dh/2
        if (head < ra.Hq + Hkv) {
#pragma unroll
          for (int r = 0; r < 4; ++r) {
            const float2 cs = ra.tab[(size_t)m * (DH / 2) + e0 + r];
            const float y0 = x0[r] * cs.x - x1[r] * cs.y, y1 = x0[r] * cs.y + x1[r] * cs.x;
            x0[r] = y0; x1[r] = y1;
          }
        }
        bf16 o0[4], o1[4];
#pragma unroll
        for (int r = 0; r < 4; ++r) o0[r] = __float2bfloat16(x0[r]), o1[r] = __float2bfloat16(x1[r]);
        if (head < ra.Hq) {
          bf16* dst = ra.q + ((size_t)m * ra.Hq + head) * DH + e0;
          *reinterpret_cast<uint2*>(dst) = *reinterpret_cast<const uint2*>(o0);
          *reinterpret_cast<uint2*>(dst + DH / 2) = *reinterpret_cast<const uint2*>(o1);
          continue;
        }
        const int page = ra.block_table[pos / SPEC_PAGE_TOKENS];
        const int rr = pos % SPEC_PAGE_TOKENS;
        if (head < ra.Hq + Hkv) {       // K block: [16-token tile][dh/32 steps][64 lanes][8]
          bf16* blk = ra.pool + ra.g.offset(page, ra.layer, 0, head - ra.Hq);
#pragma unroll
          for (int t = 0; t < 2; ++t) {
            const int e = e0 + t * (DH / 2);
            const size_t off = ((size_t)(((rr >> 4) * (DH / 32) + (e >> 5)) * 64 + ((e & 31) >> 3) * 16 + (rr & 15))) * 8 + (e & 7);
            *reinterpret_cast<uint2*>(blk + off) = *reinterpret_cast<const uint2*>(t ? o1 : o0);
          }
        } else {                        // V block: [32-token chunk][dh][32 slots]
          bf16* blk = ra.pool + ra.g.offset(page, ra.layer, 1, head - ra.Hq - Hkv);
          const int r32 = rr & 31;
          const int slot = ((r32 & 15) >> 2) * 8 + (r32 >> 4) * 4 + (r32 & 3);
          bf16* base = blk + ((size_t)(rr >> 5) * DH + e0) * 32 + slot;
#pragma unroll
          for (int r = 0; r < 4; ++r) {
            base[(size_t)r * 32] = o0[r];
            base[(size_t)(r + DH / 2) * 32] = o1[r];
          }
        }
      }
    }
    return;
  }
#pragma unroll
  for (int mt = 0; mt < 16; ++mt) {
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

static hipError_t dense_gemm_launch(const bf16* x, const void* wp, int M, int N, int K, int epi, float* y, bf16* z,
                                    const DenseRope& ra, hipStream_t st) {
  if ((double)M * K * 2.0 >= 4294967296.0) return hipErrorInvalidValue;   // per-lane activation offsets are 32-bit
  const int NT = N / 16, steps = K / 32;
  const int TM = (M + DG_BM - 1) / DG_BM, TN = (NT + 15) / 16;
  const int cx = (TN + 7) / 8;
  const int groups = (cx + 3) / 4;
  dim3 grid(8 * groups * TM * 4), block(DG_THREADS);
  static bool attr_set = false;
  const size_t lds_bytes = (size_t)DG_STAGES * DG_STAGE_BYTES;   // 96 KiB: above the default dynamic-LDS limit
  if (!attr_set) {
    const void* fns[5] = {(const void*)dense_gemm_kernel<DG_EPI_STORE>, (const void*)dense_gemm_kernel<DG_EPI_RESID>,
                          (const void*)dense_gemm_kernel<DG_EPI_SWIGLU>, (const void*)dense_gemm_kernel<DG_EPI_ROPE128>,
                          (const void*)dense_gemm_kernel<DG_EPI_ROPE64>};
    for (const void* f : fns) {
      hipError_t e = hipFuncSetAttribute(f, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds_bytes);
      if (e != hipSuccess) return e;
    }
    attr_set = true;
  }
  const u32x4* w4 = (const u32x4*)wp;
  switch (epi) {
    case DG_EPI_STORE: dense_gemm_kernel<DG_EPI_STORE><<<grid, block, lds_bytes, st>>>(x, w4, y, z, M, N, K, NT, steps, TM, cx, ra); break;
    case DG_EPI_RESID: dense_gemm_kernel<DG_EPI_RESID><<<grid, block, lds_bytes, st>>>(x, w4, y, z, M, N, K, NT, steps, TM, cx, ra); break;
    case DG_EPI_SWIGLU: dense_gemm_kernel<DG_EPI_SWIGLU><<<grid, block, lds_bytes, st>>>(x, w4, y, z, M, N, K, NT, steps, TM, cx, ra); break;
    case DG_EPI_ROPE128: dense_gemm_kernel<DG_EPI_ROPE128><<<grid, block, lds_bytes, st>>>(x, w4, y, z, M, N, K, NT, steps, TM, cx, ra); break;
    default: dense_gemm_kernel<DG_EPI_ROPE64><<<grid, block, lds_bytes, st>>>(x, w4, y, z, M, N, K, NT, steps, TM, cx, ra); break;
  }
  return hipGetLastError();
}

hipError_t launch_dense_gemm(const bf16* x, const void* wp, int M, int N, int K, int epi, float* y, bf16* z,
                             hipStream_t st) {
  DenseRope none = {};
  return dense_gemm_launch(x, wp, M, N, K, epi, y, z, none, st);
}

// The fused QKV projection of a prompt block: q (rotated, bf16) to `q`, k (rotated) and v into the pages of
// positions len .. len + M - 1.  `tab` from launch_rope_table for the same block.
hipError_t launch_dense_qkv_rope(const bf16* x, const void* wp, int M, int K, bf16* q, bf16* pool, const int* block_table,
                                 const int* len_ptr, const float2* tab, KvGeom g, int layer, int Hq, hipStream_t st) {
  DenseRope ra = {q, pool, block_table, len_ptr, tab, g, layer, Hq};
  const int N = (Hq + 2 * g.n_kv_heads) * g.head_dim;
  return dense_gemm_launch(x, wp, M, N, K, g.head_dim == 128 ? DG_EPI_ROPE128 : DG_EPI_ROPE64, nullptr, nullptr, ra, st);
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
