// Internal declarations shared by the kernel files and the host runtime (gfx950 only).
#pragma once
#include <hip/hip_runtime.h>
#include <hip/hip_bf16.h>
#include <stdint.h>
#include <stddef.h>

#include "../../include/spec.h"

typedef __hip_bfloat16 bf16;
typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(4))) unsigned u32x4;

#define SPEC_PAGE_TOKENS 64      // tokens per KV page
#define SPEC_RING_MAX 64         // most slots of the draft-token / q-row ring
// Compute units of the device the library runs on: 256 (MI355X) until spec_init has asked the device.
int spec_num_cu();
void spec_set_num_cu(int n);
#define SPEC_PEARL_WGS_PER_CU 1   // projection workgroups per CU and stream while draft and target overlap

// ---------------------------------------------------------------------------------------
// Projection (skinny GEMM) plan: y[M][N] = x[M][K] W^T, W panel-packed.
// The K axis is cut into S slices (one per group of workgroups) and each slice into 8
// wave-slices of `spw` 32-wide steps; partial sums of slice s go to P[s][M][N] (fp32).
// ---------------------------------------------------------------------------------------
struct GemmPlan {
  int M, N, K;
  int steps;   // K rounded up to 32, divided by 32
  int NT;      // N / 16 panels
  int MT;      // 16-row tiles of x (1 or 2)
  int S;       // K slices
  int spw;     // steps per wave
  int Gs;      // workgroups per slice
  size_t partial_bytes() const { return (size_t)S * M * N * sizeof(float); }
  size_t weight_bytes() const { return (size_t)NT * steps * 1024; }
};
// wgs_per_cu: 2 = fill both workgroup slots of every CU (a stream running alone), 1 = leave one slot to
// the other stream's kernels.  The K split (S, spw) does not depend on it.
GemmPlan gemm_plan(int M, int N, int K, int wgs_per_cu = 2);
// stamp: optional pair of device words that receives the launch's time stamps (see GemmPro::stamp)
hipError_t launch_gemm_partials(const GemmPlan& p, const bf16* x, const void* wp, float* partials, hipStream_t st,
                                int tag, unsigned long long* stamp = nullptr);

// The RMSNorm of the decode path is split in three: the residual-add kernel stores x' = bf16(h * gain) and the
// rows' sums of squares (W pieces per row); the projection runs on x' unchanged; whoever adds the projection's K
// slices multiplies the sum by inv_m = 1 / sqrt(sum_w ssq[m][w] / d + eps) (the projection is linear in its rows
// and bf16 keeps the same relative precision at any scale).  ssq == nullptr: no scaling.
#define SSQ_STRIDE 128                     // floats per row of sums of squares
static_assert(SSQ_STRIDE % 4 == 0, "RowScale::inv reads the pieces as 16-byte vectors");
struct RowScale {
  const float* ssq;    // [rows][SSQ_STRIDE], W pieces in use (whatever lies behind them is ignored)
  int W, d;
  float eps;
#ifdef __HIPCC__
  // the row's pieces come in independent 16-byte loads, four in flight (one round trip for up to 16 pieces), and
  // are added in ascending order
  __device__ __forceinline__ float inv(int m) const {
    if (!ssq) return 1.0f;
    const f32x4* p = reinterpret_cast<const f32x4*>(ssq + (size_t)m * SSQ_STRIDE);
    const int nv = (W + 3) >> 2;
    float tot = 0.f;
    for (int k0 = 0; k0 < nv; k0 += 4) {
      f32x4 v[4];
#pragma unroll
      for (int k = 0; k < 4; ++k) v[k] = (k0 + k < nv) ? p[k0 + k] : f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
      for (int k = 0; k < 4; ++k) {
        const int i0 = (k0 + k) * 4;
        tot += (i0 + 0 < W) ? v[k].x : 0.f; tot += (i0 + 1 < W) ? v[k].y : 0.f;
        tot += (i0 + 2 < W) ? v[k].z : 0.f; tot += (i0 + 3 < W) ? v[k].w : 0.f;
      }
    }
    return 1.0f / sqrtf(tot / (float)d + eps);
  }
#endif
};

// ---------------------------------------------------------------------------------------
// Single-token forwards (M = 1: every draft step, autoregressive and pre-verify target forwards) fold the residual
// add + RMSNorm input and the SiLU * mul into the prologue of the projection that consumes them: a wave forms the
// activation fragments of its own K range itself, after its first weight loads are on their way, so the dependent
// loads hide behind the start of the weight stream and three kernel boundaries per layer disappear.
// ---------------------------------------------------------------------------------------
enum { PRO_NONE = 0, PRO_ADDNORM = 1, PRO_SWIGLU = 2 };
#define STAMP_WAYS 16
#define GEMM_WAVES_PER_GROUP 8   // waves of a projection workgroup: a PRO_ADDNORM launch leaves 8 S sums of squares
struct GemmPro {
  int kind;
  // Optional time stamps of the launch (any kind): STAMP_WAYS pairs (workgroup b uses pair b % STAMP_WAYS, so that
  // the atomics of a launch do not queue on one address: one pair cost 3.5 us per launch), stamp[2 i] = max over its
  // workgroups of ~(start), stamp[2 i + 1] = max of their end, in ticks of the constant-rate wall clock; all start at
  // 0.  The kernel's own duration, first workgroup in to last workgroup out, without the dispatch overhead that
  // events around a launch include.
  unsigned long long* stamp;
  // PRO_ADDNORM: x' = bf16((h_in + sum_s part[s]) * gain); the workgroups of the first panel range also store the new
  // residual stream to h_out (another buffer than h_in: the other workgroups still read h_in) and one sum of
  // squares per wave to ssq[0 .. 8 S)
  const float* h_in;
  float* h_out;
  const bf16* gain;
  float* ssq_out;
  // PRO_ADDNORM, PRO_SWIGLU: K-slice partial sums of the producing projection, [S][width]
  const float* part;
  int S;
  // PRO_SWIGLU: z = bf16(silu(g * inv) * (u * inv)), gate / up panels interleaved in `part` (width 2 K)
  RowScale rs;
};
// the same projection for M = 1 with the activation formed in the prologue (pro.kind != PRO_NONE)
hipError_t launch_gemm_fused(const GemmPlan& p, const GemmPro& pro, const void* wp, float* partials, hipStream_t st,
                             int tag);


// n = M * N elements; rs scales row i / N (N given) of the sum
hipError_t launch_reduce_partials(float* y, const float* partials, int S, size_t n, hipStream_t st,
                                  RowScale rs = RowScale{nullptr, 0, 0, 0.f}, int N = 0);
hipError_t launch_pack_weight(void* dst, const void* src, int N, int K, int panel_start, int panel_step, hipStream_t st);
hipError_t launch_read_probe(const void* src, size_t bytes, void* out, hipStream_t st);

// ---------------------------------------------------------------------------------------
// KV cache geometry.  Pool element order: [page][layer][k|v][kv_head][page block], where a K
// block is [P/16 tiles][dh/32 steps][64 lanes][8] and a V block is [P/32 chunks][dh][32 slots]
// (both already in the operand order of the 16x16x32 MFMA).
// ---------------------------------------------------------------------------------------
struct KvGeom {
  int n_layers, n_kv_heads, head_dim;
  __host__ __device__ size_t head_block() const { return (size_t)SPEC_PAGE_TOKENS * head_dim; }
  __host__ __device__ size_t page_elems() const { return (size_t)n_layers * 2 * n_kv_heads * head_block(); }
  __host__ __device__ size_t offset(int page, int layer, int kv, int head) const {
    return (((size_t)page * n_layers + layer) * 2 + kv) * n_kv_heads * head_block() + (size_t)head * head_block();
  }
};

struct TokenSrc {           // by-value kernel argument: where each input token of a forward comes from
  int n;
  int imm[SPEC_MAX_TOKENS];   // token id, or -1 to read ring[slot]
  int slot[SPEC_MAX_TOKENS];
};
struct PageUpdate {         // by-value kernel argument: new block-table entries
  int first, count;
  int page[8];
};

hipError_t launch_gather_tokens(int* tok_out, const int* ring, TokenSrc src, hipStream_t st);
hipError_t launch_set_int(int* dst, int value, hipStream_t st);
hipError_t launch_add_int(int* dst, int delta, hipStream_t st);
hipError_t launch_set_pages(int* block_table, PageUpdate u, hipStream_t st);
hipError_t launch_embed(float* h, const bf16* embed, const int* tok, int M, int d, int vocab, hipStream_t st);
// h += sum_s partials[s] (if partials), a = rmsnorm(h) * gain
hipError_t launch_addnorm(float* h, const float* partials, int S, const bf16* gain, bf16* a, int M, int d,
                          float eps, hipStream_t st);
// h += sum_s partials[s] (if partials), a = bf16(h * gain) (not normalised), ssq[m][w] = sum of h^2 over the w-th
// piece of 1024 columns of row m (row stride SSQ_STRIDE; pieces beyond W
// are never written); returns the number of pieces W through *W_out
#define ADDSQ_MAX_PIECES 16
static_assert(ADDSQ_MAX_PIECES <= SSQ_STRIDE, "a row of sums of squares holds every piece");
hipError_t launch_add_sumsq(float* h, const float* partials, int S, const bf16* gain, bf16* a, float* ssq, int M,
                            int d, int* W_out, hipStream_t st);
// tab: optional [M][dh/2] (cos, sin) table from launch_rope_table for the same len; nullptr = compute in place
hipError_t launch_rope_append(const float* partials, int S, bf16* q, bf16* pool, const int* block_table,
                              const int* len_ptr, KvGeom g, int layer, int M, int Hq, float theta, hipStream_t st,
                              const float2* tab = nullptr, RowScale rs = RowScale{nullptr, 0, 0, 0.f});
hipError_t launch_rope_table(float2* tab, const int* len_ptr, int M, int dh, float theta, hipStream_t st);
hipError_t launch_attention(const bf16* q, const bf16* pool, const int* block_table, const int* len_ptr, KvGeom g,
                            int layer, int M, int Hq, int split_tokens, float* opart, float* mlpart, bf16* out,
                            hipStream_t st);
size_t attention_workspace_floats(int Hq, int Hkv, int dh, int max_seq);
hipError_t launch_silu_mul(const float* partials, int S, bf16* z, int M, int F, hipStream_t st,
                           RowScale rs = RowScale{nullptr, 0, 0, 0.f});

// prompt-sized (matrix-core bound) kernels: epilogue 0 = store fp32, 1 = add into fp32, 2 = silu(gate)*up -> bf16
#define SPEC_PREFILL_BLOCK_MAX 4096   // most prompt tokens one dense pass takes
hipError_t launch_dense_gemm(const bf16* x, const void* wp, int M, int N, int K, int epi, float* y, bf16* z,
                             hipStream_t st);
// fused QKV projection of a prompt block with RoPE and the paged K / V append in its epilogue
hipError_t launch_dense_qkv_rope(const bf16* x, const void* wp, int M, int K, bf16* q, bf16* pool, const int* block_table,
                                 const int* len_ptr, const float2* tab, KvGeom g, int layer, int Hq, hipStream_t st);
hipError_t launch_prefill_attention(const bf16* q, const bf16* pool, const int* block_table, const int* len_ptr,
                                    KvGeom g, int layer, int M, int Hq, bf16* out, hipStream_t st);

// sampling / acceptance
struct AcceptArgs {
  int kind;                 // SPEC_ACCEPT_*
  int n_rows;               // rows of target logits available
  int n_test;               // draft tokens to test
  int slot[SPEC_MAX_TOKENS];// ring slot of the token / q row tested against logits row i
  float r[SPEC_MAX_TOKENS];
  float u_resample;
  long long force_mask;     // < 0: none
  int guided;               // 1: row i >= 1 exists only if the drafts tested by rows 0..i-1 equal guess[0..i-1]; no bonus row
  int guess[SPEC_MAX_TOKENS];
};
struct AcceptResult {       // device -> pinned host
  int n_accepted;
  int token;                // corrected / bonus / autoregressive token, -1 if none
  int rejected;             // 1 if a rejection happened
  int off_path;             // 1 if a guided test ended at a draft that left the guessed path (no rejection)
  int ring[SPEC_RING_MAX];  // snapshot of the draft-token ring
};
hipError_t launch_sample_row(const float* logits, int V, float mult, int greedy, float u, float* q_out, int* tok_out,
                             hipStream_t st);
hipError_t launch_accept(const float* logits, int V, float mult, int greedy, const float* qcache, const int* ring,
                         const int* x_direct, AcceptArgs a, float* stats_scratch, AcceptResult* result_dev,
                         hipStream_t st, int* out2 = nullptr);

void spec_set_error(const char* fmt, ...);
