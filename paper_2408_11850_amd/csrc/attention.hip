// Multi-token decode attention over the paged KV cache (gfx950), grouped-query, causal inside
// the block of M new tokens.
//
// The M*G query rows that share one KV head (G = query heads per KV head) form the column
// dimension of 16x16x32 MFMAs: S^T = K Q^T per 16 positions, then O^T += V^T P^T per 32
// positions.  K and V pages are stored in MFMA operand order (see KvGeom), so a wave streams a
// page with consecutive fully-coalesced 1 KiB loads and nothing is staged through LDS.  One wave
// owns one 16-row tile of queries and one contiguous range of 32-position chunks (split-KV);
// a second kernel merges the splits with their running max / sum.  The causal mask only bites in
// the last chunks: query row of token i sees positions 0 .. len + i.
#include "spec_internal.h"

#define NEG_BIG (-1.0e30f)

template <int DH>
__global__ __launch_bounds__(256) void attn_split_kernel(const bf16* __restrict__ q, const bf16* __restrict__ pool,
                                                         const int* __restrict__ block_table,
                                                         const int* __restrict__ len_ptr, KvGeom g, int layer, int M,
                                                         int Hq, int nsplit, int Rpad, float scale,
                                                         float* __restrict__ opart, float* __restrict__ mlpart) {
  const int kvh = blockIdx.y, split = blockIdx.z;
  const int w = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int Hkv = g.n_kv_heads, G = Hq / Hkv, R = M * G;
  const int rtile = blockIdx.x * (blockDim.x >> 6) + w;
  if (rtile * 16 >= R) return;
  const int c = lane & 15, g4 = lane >> 4;
  const int len = len_ptr[0];
  const int T = len + M;
  const int nchunks = (T + 31) >> 5;
  const int cps = (nchunks + nsplit - 1) / nsplit;
  const int c0 = split * cps;
  const int c1 = (c0 + cps < nchunks) ? c0 + cps : nchunks;

  const int Rr = rtile * 16 + c;
  const bool valid = Rr < R;
  const int tok = valid ? Rr / G : 0;
  const int head = kvh * G + (valid ? Rr % G : 0);
  const int limit = valid ? len + tok : -1;   // last visible position

  bf16x8 qf[DH / 32];
#pragma unroll
  for (int j = 0; j < DH / 32; ++j) {
    u32x4 v = {0u, 0u, 0u, 0u};
    if (valid) v = *reinterpret_cast<const u32x4*>(q + ((size_t)tok * Hq + head) * DH + j * 32 + g4 * 8);
    qf[j] = __builtin_bit_cast(bf16x8, v);
  }

  float m_run = NEG_BIG, l_run = 0.f;
  f32x4 o[DH / 16];
#pragma unroll
  for (int dt = 0; dt < DH / 16; ++dt) o[dt] = f32x4{0.f, 0.f, 0.f, 0.f};

  // K / V fragments of two chunks: while one chunk is multiplied the loads of the next are already in flight
  // (a wave owns only a handful of chunks, so its run time is a chain of load latencies unless they overlap).
  u32x4 ka[2][2][DH / 32], va[2][DH / 16];
#define ATT_LOAD(B, CH)                                                                                       \
  {                                                                                                           \
    const int pos0_ = (CH) << 5;                                                                              \
    const int page_ = block_table[pos0_ / SPEC_PAGE_TOKENS];                                                  \
    const int inpage_ = pos0_ % SPEC_PAGE_TOKENS;                                                             \
    const u32x4* kblk_ = reinterpret_cast<const u32x4*>(pool + g.offset(page_, layer, 0, kvh)) +              \
                         (size_t)(inpage_ >> 4) * (DH / 32) * 64 + lane;                                      \
    const bf16* vblk_ = pool + g.offset(page_, layer, 1, kvh) + (size_t)(inpage_ >> 5) * DH * 32;             \
    _Pragma("unroll") for (int t = 0; t < 2; ++t)                                                             \
      _Pragma("unroll") for (int j = 0; j < DH / 32; ++j) ka[B][t][j] = kblk_[(size_t)(t * (DH / 32) + j) * 64]; \
    _Pragma("unroll") for (int dt = 0; dt < DH / 16; ++dt)                                                    \
      va[B][dt] = *reinterpret_cast<const u32x4*>(vblk_ + ((size_t)(dt * 16 + c) * 32 + g4 * 8));             \
  }
#define ATT_COMPUTE(B, CH)                                                                                    \
  {                                                                                                           \
    const int pos0 = (CH) << 5;                                                                               \
    f32x4 s[2];                                                                                               \
    _Pragma("unroll") for (int t = 0; t < 2; ++t) {                                                           \
      s[t] = f32x4{0.f, 0.f, 0.f, 0.f};                                                                       \
      _Pragma("unroll") for (int j = 0; j < DH / 32; ++j)                                                     \
        s[t] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, ka[B][t][j]), qf[j], s[t], 0, 0, 0); \
    }                                                                                                         \
    /* s[t][r] = score of position pos0 + 16 t + 4 g4 + r for query row c */                                  \
    float mx = NEG_BIG;                                                                                       \
    _Pragma("unroll") for (int t = 0; t < 2; ++t)                                                             \
      _Pragma("unroll") for (int r = 0; r < 4; ++r) {                                                         \
        const int pos = pos0 + t * 16 + g4 * 4 + r;                                                           \
        const float v = (pos <= limit) ? s[t][r] * scale : NEG_BIG;                                           \
        s[t][r] = v;                                                                                          \
        mx = fmaxf(mx, v);                                                                                    \
      }                                                                                                       \
    mx = fmaxf(mx, __shfl_xor(mx, 16));                                                                       \
    mx = fmaxf(mx, __shfl_xor(mx, 32));                                                                       \
    const float m_new = fmaxf(m_run, mx);                                                                     \
    const float corr = __expf(m_run - m_new);                                                                 \
    float psum = 0.f;                                                                                         \
    bf16x8 pf;                                                                                                \
    _Pragma("unroll") for (int t = 0; t < 2; ++t)                                                             \
      _Pragma("unroll") for (int r = 0; r < 4; ++r) {                                                         \
        const float p = (s[t][r] > 0.5f * NEG_BIG) ? __expf(s[t][r] - m_new) : 0.f;                           \
        psum += p;                                                                                            \
        pf[t * 4 + r] = (__bf16)p;                                                                            \
      }                                                                                                       \
    l_run = l_run * corr + psum;                                                                              \
    m_run = m_new;                                                                                            \
    _Pragma("unroll") for (int dt = 0; dt < DH / 16; ++dt) {                                                  \
      o[dt] *= corr;                                                                                          \
      o[dt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, va[B][dt]), pf, o[dt], 0, 0, 0); \
    }                                                                                                         \
  }
  if (c0 < c1) ATT_LOAD(0, c0)
  int ch = c0;
  for (; ch + 2 <= c1; ch += 2) {
    ATT_LOAD(1, ch + 1)
    ATT_COMPUTE(0, ch)
    if (ch + 2 < c1) ATT_LOAD(0, ch + 2)
    ATT_COMPUTE(1, ch + 1)
  }
  if (ch < c1) ATT_COMPUTE(0, ch)
#undef ATT_LOAD
#undef ATT_COMPUTE
  l_run += __shfl_xor(l_run, 16);
  l_run += __shfl_xor(l_run, 32);
  if (valid) {
    const size_t row = ((size_t)kvh * Rpad + Rr) * nsplit + split;   // the splits of a query row lie side by side
#pragma unroll
    for (int dt = 0; dt < DH / 16; ++dt)
      *reinterpret_cast<f32x4*>(opart + row * DH + dt * 16 + g4 * 4) = o[dt];
    if (g4 == 0) {
      mlpart[row * 2] = m_run;
      mlpart[row * 2 + 1] = l_run;
    }
  }
}

// out[i][head][e] = sum_s w_s O_s[e] / sum_s w_s l_s,  w_s = exp(m_s - max_s m_s).
// Workgroup = (dh, 8): the eight thread rows take every eighth split and fold them into a running (max, numerator,
// denominator) triple - no pass for the maximum first, and eight splits' loads in flight per thread, so up to 64
// splits cost one memory round trip - then the eight triples are combined through LDS in a fixed order.
#define MERGE_WAYS 8
#define MERGE_UNROLL 8
__global__ __launch_bounds__(128 * MERGE_WAYS) void attn_merge_kernel(const float* __restrict__ opart,
                                                                      const float* __restrict__ mlpart,
                                                                      bf16* __restrict__ out, int M, int Hq, int Hkv,
                                                                      int dh, int nsplit, int Rpad) {
  __shared__ float sm[MERGE_WAYS], snum[MERGE_WAYS][128], sden[MERGE_WAYS];
  const int i = blockIdx.x, head = blockIdx.y, e = threadIdx.x, y = threadIdx.y;
  const int G = Hq / Hkv, kvh = head / G, Rr = i * G + head % G;
  float mrun = NEG_BIG, num = 0.f, den = 0.f;
  for (int s = y; s < nsplit; s += MERGE_UNROLL * MERGE_WAYS) {
    float ms[MERGE_UNROLL], ls[MERGE_UNROLL], os[MERGE_UNROLL];
#pragma unroll
    for (int k = 0; k < MERGE_UNROLL; ++k) {
      const int sk = s + k * MERGE_WAYS;
      const size_t row = ((size_t)kvh * Rpad + Rr) * nsplit + (sk < nsplit ? sk : s);
      const bool in = sk < nsplit;
      ms[k] = in ? mlpart[row * 2] : NEG_BIG;
      ls[k] = in ? mlpart[row * 2 + 1] : 0.f;
      os[k] = in ? opart[row * dh + e] : 0.f;
    }
#pragma unroll
    for (int k = 0; k < MERGE_UNROLL; ++k) {
      const float mnew = fmaxf(mrun, ms[k]);
      const float c0 = __expf(mrun - mnew), c1 = __expf(ms[k] - mnew);
      num = num * c0 + c1 * os[k];
      den = den * c0 + c1 * ls[k];
      mrun = mnew;
    }
  }
  snum[y][e] = num;
  if (e == 0) sm[y] = mrun, sden[y] = den;
  __syncthreads();
  if (y == 0) {
    float mstar = sm[0];
#pragma unroll
    for (int k = 1; k < MERGE_WAYS; ++k) mstar = fmaxf(mstar, sm[k]);
    float n = 0.f, dd = 0.f;
#pragma unroll
    for (int k = 0; k < MERGE_WAYS; ++k) {
      const float c = __expf(sm[k] - mstar);    // a thread row that took no split holds (NEG_BIG, 0, 0): weight 0 or 0 * 1
      n += c * snum[k][e];
      dd += c * sden[k];
    }
    out[((size_t)i * Hq + head) * dh + e] = __float2bfloat16(n / dd);
  }
}

static int attn_nsplit(int Hkv, int nrt, int T) {
  const int nchunks = (T + 31) / 32;
  int ns = (3 * spec_num_cu() + Hkv * nrt - 1) / (Hkv * nrt);   // about three waves per compute unit ...
  if (ns > (nchunks + 1) / 2) ns = (nchunks + 1) / 2;           // ... but at least two chunks per split
  if (ns < 1) ns = 1;
  return ns;
}

size_t attention_workspace_floats(int Hq, int Hkv, int dh, int max_seq) {
  const int G = Hq / Hkv;
  const int Rpad = ((SPEC_MAX_TOKENS * G + 15) / 16) * 16;
  // the split count is largest for a single query tile
  int ns_max = attn_nsplit(Hkv, 1, max_seq + SPEC_MAX_TOKENS);
  return (size_t)ns_max * Hkv * Rpad * (dh + 2);
}

hipError_t launch_attention(const bf16* q, const bf16* pool, const int* block_table, const int* len_ptr, KvGeom g,
                            int layer, int M, int Hq, int split_tokens, float* opart, float* mlpart, bf16* out,
                            hipStream_t st) {
  const int Hkv = g.n_kv_heads, G = Hq / Hkv, R = M * G, dh = g.head_dim;
  const int nrt = (R + 15) / 16;
  const int Rpad = ((SPEC_MAX_TOKENS * G + 15) / 16) * 16;
  // the split count is sized for the longest context, not the current one, so that the launch is replayable
  const int nsplit = attn_nsplit(Hkv, nrt, split_tokens);
  const int wpb = nrt < 4 ? nrt : 4;
  dim3 grid((nrt + wpb - 1) / wpb, Hkv, nsplit), block(64 * wpb);
  const float scale = 1.0f / sqrtf((float)dh);
  if (dh == 128)
    attn_split_kernel<128><<<grid, block, 0, st>>>(q, pool, block_table, len_ptr, g, layer, M, Hq, nsplit, Rpad, scale,
                                                   opart, mlpart);
  else
    attn_split_kernel<64><<<grid, block, 0, st>>>(q, pool, block_table, len_ptr, g, layer, M, Hq, nsplit, Rpad, scale,
                                                  opart, mlpart);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  attn_merge_kernel<<<dim3(M, Hq), dim3(dh, MERGE_WAYS), 0, st>>>(opart, mlpart, out, M, Hq, Hkv, dh, nsplit, Rpad);
  return hipGetLastError();
}
