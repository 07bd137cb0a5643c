// Host runtime of the speculative-decoding library: contexts, the paged KV allocator, the
// forward pass as a chain of kernel launches, the draft-token ring with its q-row cache, the
// accept step's bookkeeping and the three decoding loops (paper Section 2 and Algorithms 1, 2).
#include <chrono>
#include <cstdarg>
#include <cstdio>
#include <cstring>
#include <new>
#include <vector>

#include "spec_internal.h"

static thread_local char g_err[512] = "";
void spec_set_error(const char* fmt, ...) {
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(g_err, sizeof(g_err), fmt, ap);
  va_end(ap);
}
extern "C" const char* spec_last_error(void) { return g_err; }

#define HIPCHK(expr)                                                                        \
  do {                                                                                      \
    hipError_t e_ = (expr);                                                                 \
    if (e_ != hipSuccess) {                                                                 \
      spec_set_error("%s failed: %s (%s:%d)", #expr, hipGetErrorString(e_), __FILE__, __LINE__); \
      return SPEC_E_HIP;                                                                    \
    }                                                                                       \
  } while (0)
#define FAIL(code, ...)        \
  do {                         \
    spec_set_error(__VA_ARGS__); \
    return (code);             \
  } while (0)

#define SPEC_GRAPH_PARTS 24                          // graphs a forward may be cut into (see ModelRt::graphs)
#define SPEC_TAIL_CHUNKS_MAX (SPEC_GRAPH_PARTS - 2)

namespace {

struct ModelRt {
  spec_model_desc d;
  const void *tok_embed = nullptr, *final_norm = nullptr, *lm_head = nullptr;
  std::vector<const void*> attn_norm, wqkv, wo, ffn_norm, wgu, wdown;
  hipStream_t stream = nullptr;
  KvGeom geom;
  bf16* pool = nullptr;
  int n_pages = 0;
  int* block_table_dev = nullptr;
  std::vector<int> block_table;   // pages of the sequence, in order
  std::vector<int> free_pages;
  int len = 0;                    // host mirror of *len_dev
  int* len_dev = nullptr;
  int* tok_in = nullptr;
  float* h = nullptr;
  float* h2 = nullptr;            // second residual buffer of the single-token path (its projections read one, write the other)
  float* partials2 = nullptr;     // and second buffer of K-slice sums
  float2* rope_tab = nullptr;     // (cos, sin) of the new position of a single-token forward
  float* ssq = nullptr;           // sums of squares of the rows of h, SSQ_STRIDE floats per row
  bf16 *a = nullptr, *qbuf = nullptr, *attn_out = nullptr, *z = nullptr;
  float *partials = nullptr, *opart = nullptr, *mlpart = nullptr, *logits = nullptr;
  long long n_forwards = 0;
  int split_tokens = 0;           // context length the attention split count is sized for (fixed per context)
  // captured forwards, keyed [tokens][logit mode 0/1/2][projection workgroups per CU][part]; part 0 = the first
  // layers, 1 = all the rest, 2 + i = chunk i of the rest (forwards whose trailing chunks launch in another mode)
  hipGraphExec_t graphs[SPEC_MAX_TOKENS + 1][3][3][SPEC_GRAPH_PARTS] = {};
  // activation buffers of the dense prompt path, allocated at its first use for pf_cap tokens
  int pf_cap = 0;
  int* pf_tok = nullptr;
  float* pf_h = nullptr;
  bf16 *pf_a = nullptr, *pf_q = nullptr, *pf_attn = nullptr, *pf_z = nullptr;
  float2* pf_rope = nullptr;      // (cos, sin) per token and rotation pair of the current block
};

struct ProfStamps {               // per profiled projection launch: the kernel's own (start, end) stamps
  unsigned long long* dev = nullptr;   // [cap][STAMP_WAYS][2], zeroed; see GemmPro::stamp
  size_t cap = 0, used = 0;
  double bytes = 0.0;
  double tick_s = 0.0;            // seconds per tick of the device's wall clock
};

}  // namespace

struct spec_ctx {
  spec_config cfg;
  ModelRt m[2];
  int ring_n = 0;
  float* qcache = nullptr;        // [ring_n][vocab]
  int* ring = nullptr;            // [SPEC_RING_MAX] draft tokens
  hipEvent_t ev_slot[SPEC_RING_MAX];
  bool ev_slot_valid[SPEC_RING_MAX];
  float* accept_scratch = nullptr;
  AcceptResult* res_dev = nullptr;
  AcceptResult* res_host = nullptr;
  std::vector<int> committed;
  int n_prompt = 0;
  int ring_base = 0, n_drafted = 0;
  bool first_verified = false;    // x_1 of the ring is already committed (it is the frontier)
  int last_verify_rows = 0;
  int n_guess = -1;               // >= 0: the last target forward was spec_verify_guess over the frontier + guess[0..n_guess)
  int guess[SPEC_MAX_TOKENS];
  int guess_opt = -1;             // most guesses per pre-verify step of the loop: -1 = gamma - 1
  bool prefilled = false;
  int mode = SPEC_MODE_PRE;       // strategy of the next PEARL step
  int profile_flags = 0;
  bool use_graphs = true;         // replay captured forwards instead of launching ~10 kernels per layer
  int wgs_opt = -1;               // projection workgroups per CU: -1 = automatic, 1, 2
  int wgs = 2;                    // what the next forward uses
  int tail_opt = -1;              // trailing target layers that launch with two workgroups per CU while wgs == 1:
                                  // -1 = chosen by spec_generate from the two chains' end times, >= 0 fixed
  int tail_layers = 0;            // what the next target forward uses
  hipEvent_t ev_t0[2] = {}, ev_tend[2] = {}, ev_dend[2] = {};   // start of a PEARL step, ends of its target / draft chain (timed), two sets in turn
  bool bal_valid[2] = {false, false};   // set holds a step's three events
  bool fuse_single = true;        // single-token forwards through the projections with fused prologues
  int prefill_opt = -1;           // -1 automatic, 0 = 32-token verify forwards, 1 = dense path
  int fail_prefill_after = 0;     // test hook: > 0 = the next spec_prefill gives up after that many forwards
  ProfStamps prof;
};

namespace {

inline int slot_of(const spec_ctx* c, int i /* 1-based draft index */) { return (c->ring_base + i - 1) % c->ring_n; }

int check_desc(const spec_model_desc& d, const char* name) {
  if (d.n_layers < 1 || d.d_model < 32 || d.n_heads < 1 || d.n_kv_heads < 1 || d.d_ffn < 16 || d.vocab < 16)
    FAIL(SPEC_E_INVAL, "%s: non-positive model dimension", name);
  if (d.head_dim != 64 && d.head_dim != 128) FAIL(SPEC_E_INVAL, "%s: head_dim must be 64 or 128", name);
  if (d.n_heads % d.n_kv_heads) FAIL(SPEC_E_INVAL, "%s: n_heads must be a multiple of n_kv_heads", name);
  if (d.d_model % 16 || d.d_ffn % 16 || d.vocab % 16) FAIL(SPEC_E_INVAL, "%s: d_model, d_ffn, vocab must be multiples of 16", name);
  if (d.d_model > 1024 * ADDSQ_MAX_PIECES) FAIL(SPEC_E_INVAL, "%s: d_model above %d", name, 1024 * ADDSQ_MAX_PIECES);
  if (!(d.rope_theta > 1.0f) || !(d.rms_eps >= 0.0f)) FAIL(SPEC_E_INVAL, "%s: bad rope_theta / rms_eps", name);
  return SPEC_OK;
}

template <typename T>
int dev_alloc(T** p, size_t count) {
  void* v = nullptr;
  hipError_t e = hipMalloc(&v, count * sizeof(T) + 256);
  if (e != hipSuccess) {
    (void)hipGetLastError();
    FAIL(SPEC_E_NOMEM, "hipMalloc of %zu bytes failed: %s", count * sizeof(T), hipGetErrorString(e));
  }
  *p = (T*)v;
  return SPEC_OK;
}

int init_model(ModelRt& m, const spec_model_desc& d, const spec_weights& w, const spec_config& cfg, hipStream_t st) {
  m.d = d;
  m.stream = st;
  m.tok_embed = w.tok_embed; m.final_norm = w.final_norm; m.lm_head = w.lm_head;
  if (!w.tok_embed || !w.final_norm || !w.lm_head || !w.attn_norm || !w.wqkv || !w.wo || !w.ffn_norm || !w.w_gateup ||
      !w.w_down)
    FAIL(SPEC_E_INVAL, "null weight pointer");
  for (int l = 0; l < d.n_layers; ++l) {
    if (!w.attn_norm[l] || !w.wqkv[l] || !w.wo[l] || !w.ffn_norm[l] || !w.w_gateup[l] || !w.w_down[l])
      FAIL(SPEC_E_INVAL, "null weight pointer in layer %d", l);
    m.attn_norm.push_back(w.attn_norm[l]); m.wqkv.push_back(w.wqkv[l]); m.wo.push_back(w.wo[l]);
    m.ffn_norm.push_back(w.ffn_norm[l]); m.wgu.push_back(w.w_gateup[l]); m.wdown.push_back(w.w_down[l]);
  }
  m.geom.n_layers = d.n_layers; m.geom.n_kv_heads = d.n_kv_heads; m.geom.head_dim = d.head_dim;
  m.n_pages = (cfg.max_seq + SPEC_PAGE_TOKENS - 1) / SPEC_PAGE_TOKENS + 1;
  m.split_tokens = m.n_pages * SPEC_PAGE_TOKENS;
  int rc;
  const size_t pool_elems = (size_t)m.n_pages * m.geom.page_elems();
  if ((rc = dev_alloc(&m.pool, pool_elems))) return rc;
  // stale slots are read (then masked) by the attention kernel: they must hold finite numbers
  HIPCHK(hipMemset(m.pool, 0, pool_elems * sizeof(bf16)));
  if ((rc = dev_alloc(&m.block_table_dev, (size_t)m.n_pages))) return rc;
  HIPCHK(hipMemset(m.block_table_dev, 0, m.n_pages * sizeof(int)));
  if ((rc = dev_alloc(&m.len_dev, 4))) return rc;
  HIPCHK(hipMemset(m.len_dev, 0, 16));
  for (int p = m.n_pages - 1; p >= 0; --p) m.free_pages.push_back(p);
  const int MX = SPEC_MAX_TOKENS;
  const int qkvN = (d.n_heads + 2 * d.n_kv_heads) * d.head_dim;
  const int kmax = d.d_model > d.d_ffn ? d.d_model : d.d_ffn;
  const int amax = kmax > d.n_heads * d.head_dim ? kmax : d.n_heads * d.head_dim;
  if ((rc = dev_alloc(&m.tok_in, (size_t)MX))) return rc;
  if ((rc = dev_alloc(&m.h, (size_t)MX * d.d_model))) return rc;
  if ((rc = dev_alloc(&m.ssq, (size_t)MX * SSQ_STRIDE))) return rc;
  HIPCHK(hipMemset(m.ssq, 0, (size_t)MX * SSQ_STRIDE * sizeof(float)));
  if ((rc = dev_alloc(&m.a, (size_t)MX * amax))) return rc;
  if ((rc = dev_alloc(&m.qbuf, (size_t)MX * d.n_heads * d.head_dim))) return rc;
  if ((rc = dev_alloc(&m.attn_out, (size_t)MX * d.n_heads * d.head_dim))) return rc;
  if ((rc = dev_alloc(&m.z, (size_t)MX * d.d_ffn))) return rc;
  size_t pb = 0;
  const int shapes[5][2] = {{qkvN, d.d_model}, {d.d_model, d.n_heads * d.head_dim}, {2 * d.d_ffn, d.d_model},
                            {d.d_model, d.d_ffn}, {d.vocab, d.d_model}};
  for (int mm : {1, 16, MX})
    for (auto& s : shapes) {
      size_t b = gemm_plan(mm, s[0], s[1]).partial_bytes();
      if (b > pb) pb = b;
    }
  if ((rc = dev_alloc(&m.partials, pb / sizeof(float)))) return rc;
  if ((rc = dev_alloc(&m.partials2, pb / sizeof(float)))) return rc;
  if ((rc = dev_alloc(&m.h2, (size_t)MX * d.d_model))) return rc;
  if ((rc = dev_alloc(&m.rope_tab, (size_t)MX * (d.head_dim / 2)))) return rc;
  const size_t aw = attention_workspace_floats(d.n_heads, d.n_kv_heads, d.head_dim, m.n_pages * SPEC_PAGE_TOKENS);
  if ((rc = dev_alloc(&m.opart, aw))) return rc;
  m.mlpart = m.opart + (aw / (d.head_dim + 2)) * d.head_dim;
  if ((rc = dev_alloc(&m.logits, (size_t)MX * d.vocab))) return rc;
  return SPEC_OK;
}

void free_model(ModelRt& m) {
  for (auto& a : m.graphs)
    for (auto& b : a)
      for (auto& cc : b)
        for (hipGraphExec_t& g : cc)
          if (g) {
            (void)hipGraphExecDestroy(g);
            g = nullptr;
          }
  void* ptrs[] = {m.h2, m.partials2, m.rope_tab,
                  m.pool, m.block_table_dev, m.len_dev, m.tok_in, m.h, m.ssq, m.a, m.qbuf, m.attn_out, m.z, m.partials,
                  m.opart, m.logits, m.pf_tok, m.pf_h, m.pf_a, m.pf_q, m.pf_attn, m.pf_z, m.pf_rope};
  for (void* p : ptrs)
    if (p) (void)hipFree(p);
}

// make sure pages exist for positions [0, new_len)
int ensure_pages(ModelRt& m, int new_len) {
  const int need = (new_len + SPEC_PAGE_TOKENS - 1) / SPEC_PAGE_TOKENS;
  const int have = (int)m.block_table.size();
  if (need <= have) return SPEC_OK;
  if ((size_t)(need - have) > m.free_pages.size())
    FAIL(SPEC_E_NOMEM, "KV cache full: %d tokens need %d pages, %d in use, %zu free", new_len, need, have,
         m.free_pages.size());
  int first = have;
  while ((int)m.block_table.size() < need) {
    PageUpdate u;
    u.first = (int)m.block_table.size();
    u.count = 0;
    while (u.count < 8 && (int)m.block_table.size() < need) {
      const int pg = m.free_pages.back();
      m.free_pages.pop_back();
      m.block_table.push_back(pg);
      u.page[u.count++] = pg;
    }
    HIPCHK(launch_set_pages(m.block_table_dev, u, m.stream));
  }
  (void)first;
  return SPEC_OK;
}

#define PROF_MAX_LAUNCHES 65536
// the stamp words of the next profiled projection launch (nullptr once the buffer is full: later launches run untimed)
int prof_slot(spec_ctx* c, double bytes, unsigned long long** slot) {
  ProfStamps& p = c->prof;
  *slot = nullptr;
  if (!p.dev) {
    int rc = dev_alloc(&p.dev, (size_t)PROF_MAX_LAUNCHES * 2 * STAMP_WAYS);
    if (rc) return rc;
    HIPCHK(hipMemset(p.dev, 0, (size_t)PROF_MAX_LAUNCHES * 2 * STAMP_WAYS * sizeof(unsigned long long)));
    int dev = 0, khz = 0;
    HIPCHK(hipGetDevice(&dev));
    HIPCHK(hipDeviceGetAttribute(&khz, hipDeviceAttributeWallClockRate, dev));
    if (khz < 1) FAIL(SPEC_E_HIP, "device reports a wall clock rate of %d kHz", khz);
    p.tick_s = 1.0 / (1e3 * khz);
    p.cap = PROF_MAX_LAUNCHES;
  }
  if (p.used >= p.cap) return SPEC_OK;
  *slot = p.dev + (size_t)2 * STAMP_WAYS * p.used;
  p.used++;
  p.bytes += bytes;
  return SPEC_OK;
}

int run_gemm(spec_ctx* c, int which, ModelRt& m, int M, int N, int K, const bf16* x, const void* w, GemmPlan* plan_out) {
  GemmPlan p = gemm_plan(M, N, K, c->wgs);
  const bool prof = (c->profile_flags & 1) && which == SPEC_TARGET;
  unsigned long long* slot = nullptr;
  int rc;
  if (prof && (rc = prof_slot(c, (double)p.weight_bytes(), &slot))) return rc;
  HIPCHK(launch_gemm_partials(p, x, w, m.partials, m.stream, which, slot));
  *plan_out = p;
  return SPEC_OK;
}

// The kernel chain of one forward over the M tokens in m.tok_in.  Nothing here depends on host state other
// than M, logit_rows and the launch mode: positions come from *len_dev, pages from the device block table,
// so the chain can be captured once into a HIP graph and replayed.
// Layers [l0, l1) of the chain: the embedding goes with layer 0, the LM head and the length update with the last layer.
int enqueue_forward(spec_ctx* c, int which, int M, int logit_rows, int l0, int l1) {
  ModelRt& m = c->m[which];
  const spec_model_desc& d = m.d;
  hipStream_t st = m.stream;
  int rc;
  if (l0 == 0) HIPCHK(launch_embed(m.h, (const bf16*)m.tok_embed, m.tok_in, M, d.d_model, d.vocab, st));
  const int qkvN = (d.n_heads + 2 * d.n_kv_heads) * d.head_dim;
  const int HD = d.n_heads * d.head_dim;
  GemmPlan p;
  // a chain that starts behind layer 0 first adds the K slices the previous layer's down projection left
  const float* prev = l0 > 0 ? m.partials : nullptr;
  int prevS = l0 > 0 ? gemm_plan(M, d.d_model, d.d_ffn, c->wgs).S : 0;
  // Every RMSNorm is split in three: a residual add spread over several workgroups per row, which leaves the
  // rows' sums of squares and x' = bf16(h * gain); the projection of x'; and the factor 1/rms, applied to the
  // projection's output rows by the kernel that adds its K slices.
  RowScale rs{m.ssq, 0, d.d_model, d.rms_eps};
  for (int l = l0; l < l1; ++l) {
    HIPCHK(launch_add_sumsq(m.h, prev, prevS, (const bf16*)m.attn_norm[l], m.a, m.ssq, M, d.d_model, &rs.W, st));
    if ((rc = run_gemm(c, which, m, M, qkvN, d.d_model, m.a, m.wqkv[l], &p))) return rc;
    HIPCHK(launch_rope_append(m.partials, p.S, m.qbuf, m.pool, m.block_table_dev, m.len_dev, m.geom, l, M, d.n_heads,
                              d.rope_theta, st, nullptr, rs));
    HIPCHK(launch_attention(m.qbuf, m.pool, m.block_table_dev, m.len_dev, m.geom, l, M, d.n_heads, m.split_tokens,
                            m.opart, m.mlpart, m.attn_out, st));
    if ((rc = run_gemm(c, which, m, M, d.d_model, HD, m.attn_out, m.wo[l], &p))) return rc;
    HIPCHK(launch_add_sumsq(m.h, m.partials, p.S, (const bf16*)m.ffn_norm[l], m.a, m.ssq, M, d.d_model, &rs.W, st));
    if ((rc = run_gemm(c, which, m, M, 2 * d.d_ffn, d.d_model, m.a, m.wgu[l], &p))) return rc;
    HIPCHK(launch_silu_mul(m.partials, p.S, m.z, M, d.d_ffn, st, rs));
    if ((rc = run_gemm(c, which, m, M, d.d_model, d.d_ffn, m.z, m.wdown[l], &p))) return rc;
    prev = m.partials;
    prevS = p.S;
  }
  if (l1 < d.n_layers) return SPEC_OK;
  if (logit_rows > 0) {
    HIPCHK(launch_add_sumsq(m.h, prev, prevS, (const bf16*)m.final_norm, m.a, m.ssq, M, d.d_model, &rs.W, st));
    const int rows = logit_rows >= M ? M : 1;
    const bf16* x = m.a + (size_t)(M - rows) * d.d_model;
    if ((rc = run_gemm(c, which, m, rows, d.vocab, d.d_model, x, m.lm_head, &p))) return rc;
    RowScale rl = rs;
    rl.ssq = m.ssq + (size_t)(M - rows) * SSQ_STRIDE;
    HIPCHK(launch_reduce_partials(m.logits, m.partials, p.S, (size_t)rows * d.vocab, st, rl, d.vocab));
  }
  HIPCHK(launch_add_int(m.len_dev, M, st));
  return SPEC_OK;
}

// a plain projection into a given buffer of K-slice sums
int run_gemm_into(spec_ctx* c, int which, ModelRt& m, const GemmPlan& p, const bf16* x, const void* w, float* out) {
  const bool prof = (c->profile_flags & 1) && which == SPEC_TARGET;
  unsigned long long* slot = nullptr;
  int rc;
  if (prof && (rc = prof_slot(c, (double)p.weight_bytes(), &slot))) return rc;
  HIPCHK(launch_gemm_partials(p, x, w, out, m.stream, which, slot));
  return SPEC_OK;
}

int run_gemm_fused(spec_ctx* c, int which, ModelRt& m, const GemmPlan& p, GemmPro pro, const void* w, float* out) {
  const bool prof = (c->profile_flags & 1) && which == SPEC_TARGET;
  int rc;
  if (prof && (rc = prof_slot(c, (double)p.weight_bytes(), &pro.stamp))) return rc;
  HIPCHK(launch_gemm_fused(p, pro, w, out, m.stream, which));
  return SPEC_OK;
}

bool single_token_path(const spec_ctx* c, const ModelRt& m, int M) {
  return c->fuse_single && M == 1;
}

// The same layers for a single token (every draft step, autoregressive and pre-verify target forwards) in seven
// kernels per layer instead of ten: the QKV, gate/up and down projections (and the LM head) form their own input in
// their prologue (residual add + gain + sums of squares; SiLU(gate) * up).  Those projections read the residual
// stream and the K-slice sums from one buffer and write the other.  Entry state of a layer: residual in h,
// pending K-slice sums of the previous down projection in partials2.  Measured on the 70B/7B shapes: draft forward
// 3.46 -> 3.26 ms, single-token target forward 23.30 -> 22.97 ms.
int enqueue_forward_single(spec_ctx* c, int which, int logit_rows, int l0, int l1) {
  ModelRt& m = c->m[which];
  const spec_model_desc& d = m.d;
  hipStream_t st = m.stream;
  int rc;
  if (l0 == 0) {
    HIPCHK(launch_embed(m.h, (const bf16*)m.tok_embed, m.tok_in, 1, d.d_model, d.vocab, st));
    HIPCHK(launch_rope_table(m.rope_tab, m.len_dev, 1, d.head_dim, d.rope_theta, st));
  }
  const int qkvN = (d.n_heads + 2 * d.n_kv_heads) * d.head_dim;
  const int HD = d.n_heads * d.head_dim;
  const float* prev = l0 > 0 ? m.partials2 : nullptr;
  int prevS = l0 > 0 ? gemm_plan(1, d.d_model, d.d_ffn, c->wgs).S : 0;
  GemmPro pro;
  for (int l = l0; l < l1; ++l) {
    const GemmPlan pq = gemm_plan(1, qkvN, d.d_model, c->wgs);
    memset(&pro, 0, sizeof(pro));
    pro.kind = PRO_ADDNORM; pro.h_in = m.h; pro.h_out = m.h2; pro.gain = (const bf16*)m.attn_norm[l]; pro.ssq_out = m.ssq;
    pro.part = prev; pro.S = prevS;
    if ((rc = run_gemm_fused(c, which, m, pq, pro, m.wqkv[l], m.partials))) return rc;
    RowScale rs{m.ssq, GEMM_WAVES_PER_GROUP * pq.S, d.d_model, d.rms_eps};
    const GemmPlan po = gemm_plan(1, d.d_model, HD, c->wgs);
    HIPCHK(launch_rope_append(m.partials, pq.S, m.qbuf, m.pool, m.block_table_dev, m.len_dev, m.geom, l, 1, d.n_heads,
                              d.rope_theta, st, m.rope_tab, rs));
    HIPCHK(launch_attention(m.qbuf, m.pool, m.block_table_dev, m.len_dev, m.geom, l, 1, d.n_heads, m.split_tokens,
                            m.opart, m.mlpart, m.attn_out, st));
    if ((rc = run_gemm_into(c, which, m, po, m.attn_out, m.wo[l], m.partials2))) return rc;
    const GemmPlan pg = gemm_plan(1, 2 * d.d_ffn, d.d_model, c->wgs);
    memset(&pro, 0, sizeof(pro));
    pro.kind = PRO_ADDNORM; pro.h_in = m.h2; pro.h_out = m.h; pro.gain = (const bf16*)m.ffn_norm[l]; pro.ssq_out = m.ssq;
    pro.part = m.partials2; pro.S = po.S;
    if ((rc = run_gemm_fused(c, which, m, pg, pro, m.wgu[l], m.partials))) return rc;
    const GemmPlan pd = gemm_plan(1, d.d_model, d.d_ffn, c->wgs);
    memset(&pro, 0, sizeof(pro));
    pro.kind = PRO_SWIGLU; pro.part = m.partials; pro.S = pg.S;
    pro.rs = RowScale{m.ssq, GEMM_WAVES_PER_GROUP * pg.S, d.d_model, d.rms_eps};
    if ((rc = run_gemm_fused(c, which, m, pd, pro, m.wdown[l], m.partials2))) return rc;
    prev = m.partials2;
    prevS = pd.S;
  }
  if (l1 < d.n_layers) return SPEC_OK;
  if (logit_rows > 0) {
    const GemmPlan pl = gemm_plan(1, d.vocab, d.d_model, c->wgs);
    memset(&pro, 0, sizeof(pro));
    pro.kind = PRO_ADDNORM; pro.h_in = m.h; pro.h_out = m.h2; pro.gain = (const bf16*)m.final_norm; pro.ssq_out = m.ssq;
    pro.part = prev; pro.S = prevS;
    if ((rc = run_gemm_fused(c, which, m, pl, pro, m.lm_head, m.partials))) return rc;
    RowScale rl{m.ssq, GEMM_WAVES_PER_GROUP * pl.S, d.d_model, d.rms_eps};
    HIPCHK(launch_reduce_partials(m.logits, m.partials, pl.S, (size_t)d.vocab, st, rl, d.vocab));
  }
  HIPCHK(launch_add_int(m.len_dev, 1, st));
  return SPEC_OK;
}

// Layers per chunk when a forward is cut into chunks behind its first layers (0: the model is too shallow to cut).
int tail_chunk_layers(int L) {
  const int Lh = L >= 8 ? 4 : L;
  if (Lh >= L) return 0;
  const int ch = (L - Lh + SPEC_TAIL_CHUNKS_MAX - 1) / SPEC_TAIL_CHUNKS_MAX;
  return ch < 4 ? 4 : ch;
}

// One forward of model `which` over M tokens.  logit_rows: 0 = none (prefill), 1 = last row only, M = all rows.
int forward(spec_ctx* c, int which, const TokenSrc& src, int logit_rows) {
  ModelRt& m = c->m[which];
  const int M = src.n;
  if (M < 1 || M > SPEC_MAX_TOKENS) FAIL(SPEC_E_INVAL, "forward over %d tokens (1..%d allowed)", M, SPEC_MAX_TOKENS);
  int rc;
  if ((rc = ensure_pages(m, m.len + M))) return rc;
  hipStream_t st = m.stream;
  HIPCHK(launch_gather_tokens(m.tok_in, c->ring, src, st));
  const int L = m.d.n_layers;
  // Cut of the layers into launch units.  Two graphs per forward: launching ~10 nodes per layer costs the host
  // about 0.45 us per node (0.45 ms for the 80-layer target), during which the stream would sit idle; a short graph
  // of the first layers is on the GPU in tens of microseconds and runs while the host launches the rest.
  // While draft and target overlap with one projection workgroup per CU and stream, the target's last layers may
  // launch with two (tail_layers): the chain that would end later is favoured, and once the draft chain has
  // ended the target has the GPU to itself, where one workgroup per CU streams at half the rate.  The rest is
  // then cut into chunks so that the boundary can move without capturing anything again.  The K split of a
  // projection does not depend on the launch mode, so the numbers are the same bit for bit.
  const int Lh = L >= 8 ? 4 : L;
  struct Unit { int l0, l1, wgs, part; } units[SPEC_GRAPH_PARTS];
  int n_units = 0;
  units[n_units++] = Unit{0, Lh, c->wgs, 0};
  const int tail = (which == SPEC_TARGET && c->wgs == 1 && Lh < L) ? c->tail_layers : 0;
  if (Lh < L && tail <= 0) {
    units[n_units++] = Unit{Lh, L, c->wgs, 1};
  } else if (Lh < L) {
    const int ch = tail_chunk_layers(L);
    const int tail_from = L - tail;       // chunks that start at or behind this layer launch with two workgroups per CU
    for (int l0 = Lh, i = 0; l0 < L; l0 += ch, ++i)
      units[n_units++] = Unit{l0, l0 + ch < L ? l0 + ch : L, l0 >= tail_from ? 2 : 1, 2 + i};
  }
  const int wgs_saved = c->wgs;
  rc = SPEC_OK;
  for (int u = 0; u < n_units && !rc; ++u) {
    const Unit& un = units[u];
    c->wgs = un.wgs;
    if (c->use_graphs && !(c->profile_flags & 1)) {
      const int lm = logit_rows == 0 ? 0 : (logit_rows >= M ? 2 : 1);
      hipGraphExec_t& ge = m.graphs[M][lm][un.wgs][un.part];
      if (!ge) {
        hipError_t e = hipStreamBeginCapture(st, hipStreamCaptureModeRelaxed);
        if (e != hipSuccess) {
          spec_set_error("hipStreamBeginCapture failed: %s", hipGetErrorString(e));
          rc = SPEC_E_HIP;
          break;
        }
        rc = single_token_path(c, m, M) ? enqueue_forward_single(c, which, logit_rows, un.l0, un.l1)
                                        : enqueue_forward(c, which, M, logit_rows, un.l0, un.l1);
        hipGraph_t g = nullptr;
        e = hipStreamEndCapture(st, &g);   // always leave capture mode, also after a failed launch
        if (rc || e != hipSuccess) {
          if (g) (void)hipGraphDestroy(g);
          if (!rc) {
            spec_set_error("hipStreamEndCapture failed: %s", hipGetErrorString(e));
            rc = SPEC_E_HIP;
          }
          break;
        }
        e = hipGraphInstantiate(&ge, g, nullptr, nullptr, 0);
        (void)hipGraphDestroy(g);
        if (e != hipSuccess) {
          ge = nullptr;
          spec_set_error("hipGraphInstantiate failed: %s", hipGetErrorString(e));
          rc = SPEC_E_HIP;
          break;
        }
      }
      hipError_t e = hipGraphLaunch(ge, st);
      if (e != hipSuccess) {
        spec_set_error("hipGraphLaunch failed: %s", hipGetErrorString(e));
        rc = SPEC_E_HIP;
      }
    } else {
      rc = single_token_path(c, m, M) ? enqueue_forward_single(c, which, logit_rows, un.l0, un.l1)
                                      : enqueue_forward(c, which, M, logit_rows, un.l0, un.l1);
    }
  }
  c->wgs = wgs_saved;
  if (rc) return rc;
  m.len += M;
  m.n_forwards++;
  return SPEC_OK;
}

bool dense_shapes_ok(const spec_model_desc& d) {
  return d.d_model % 32 == 0 && (d.n_heads * d.head_dim) % 32 == 0 && d.d_ffn % 32 == 0;
}

int ensure_prefill_buffers(ModelRt& m) {
  if (m.pf_cap) return SPEC_OK;
  const spec_model_desc& d = m.d;
  int cap = m.n_pages * SPEC_PAGE_TOKENS;
  if (cap > SPEC_PREFILL_BLOCK_MAX) cap = SPEC_PREFILL_BLOCK_MAX;
  const size_t C = (size_t)cap;
  const int HD = d.n_heads * d.head_dim, qkvN = (d.n_heads + 2 * d.n_kv_heads) * d.head_dim;
  const int amax = d.d_model > HD ? d.d_model : HD;
  int rc;
  if ((rc = dev_alloc(&m.pf_tok, C))) return rc;
  if ((rc = dev_alloc(&m.pf_h, C * d.d_model))) return rc;
  if ((rc = dev_alloc(&m.pf_a, C * amax))) return rc;
  if ((rc = dev_alloc(&m.pf_q, C * HD))) return rc;
  if ((rc = dev_alloc(&m.pf_attn, C * HD))) return rc;
  if ((rc = dev_alloc(&m.pf_z, C * d.d_ffn))) return rc;
  if ((rc = dev_alloc(&m.pf_rope, C * (d.head_dim / 2)))) return rc;
  m.pf_cap = cap;
  return SPEC_OK;
}

// One dense pass of model `which` over C prompt tokens (host ids `tok`) at positions len .. len + C - 1:
// the same chain of operations as enqueue_forward without the LM head, every projection one matrix-core GEMM.
int prefill_dense_block(spec_ctx* c, int which, const int32_t* tok, int C) {
  ModelRt& m = c->m[which];
  const spec_model_desc& d = m.d;
  hipStream_t st = m.stream;
  int rc;
  if ((rc = ensure_pages(m, m.len + C))) return rc;
  HIPCHK(hipMemcpyAsync(m.pf_tok, tok, (size_t)C * sizeof(int), hipMemcpyHostToDevice, st));
  HIPCHK(launch_embed(m.pf_h, (const bf16*)m.tok_embed, m.pf_tok, C, d.d_model, d.vocab, st));
  HIPCHK(launch_rope_table(m.pf_rope, m.len_dev, C, d.head_dim, d.rope_theta, st));
  const int qkvN = (d.n_heads + 2 * d.n_kv_heads) * d.head_dim;
  const int HD = d.n_heads * d.head_dim;
  for (int l = 0; l < d.n_layers; ++l) {
    HIPCHK(launch_addnorm(m.pf_h, nullptr, 0, (const bf16*)m.attn_norm[l], m.pf_a, C, d.d_model, d.rms_eps, st));
    HIPCHK(launch_dense_qkv_rope(m.pf_a, m.wqkv[l], C, d.d_model, m.pf_q, m.pool, m.block_table_dev, m.len_dev,
                                 m.pf_rope, m.geom, l, d.n_heads, st));
    HIPCHK(launch_prefill_attention(m.pf_q, m.pool, m.block_table_dev, m.len_dev, m.geom, l, C, d.n_heads, m.pf_attn,
                                    st));
    HIPCHK(launch_dense_gemm(m.pf_attn, m.wo[l], C, d.d_model, HD, 1, m.pf_h, nullptr, st));
    HIPCHK(launch_addnorm(m.pf_h, nullptr, 0, (const bf16*)m.ffn_norm[l], m.pf_a, C, d.d_model, d.rms_eps, st));
    HIPCHK(launch_dense_gemm(m.pf_a, m.wgu[l], C, 2 * d.d_ffn, d.d_model, 2, nullptr, m.pf_z, st));
    HIPCHK(launch_dense_gemm(m.pf_z, m.wdown[l], C, d.d_model, d.d_ffn, 1, m.pf_h, nullptr, st));
  }
  HIPCHK(launch_add_int(m.len_dev, C, st));
  m.len += C;
  m.n_forwards++;
  return SPEC_OK;
}

void reset_ring(spec_ctx* c) {
  c->ring_base = 0;
  c->n_drafted = 0;
  c->first_verified = false;
}

int rollback_model(spec_ctx* c, int which, int new_len) {
  ModelRt& m = c->m[which];
  if (new_len < 0 || new_len > m.len) FAIL(SPEC_E_INVAL, "rollback to %d outside [0, %d]", new_len, m.len);
  if (new_len == m.len) return SPEC_OK;
  m.len = new_len;
  HIPCHK(launch_set_int(m.len_dev, new_len, m.stream));
  const int keep = (new_len + SPEC_PAGE_TOKENS - 1) / SPEC_PAGE_TOKENS;
  while ((int)m.block_table.size() > keep) {
    m.free_pages.push_back(m.block_table.back());
    m.block_table.pop_back();
  }
  return SPEC_OK;
}

}  // namespace

// -------------------------------------------------------------------------------------------
extern "C" int spec_init(const spec_config* cfg, const spec_model_desc* target, const spec_weights* tw,
                         const spec_model_desc* draft, const spec_weights* dw, spec_ctx** out) {
  if (!cfg || !target || !tw || !draft || !dw || !out) FAIL(SPEC_E_INVAL, "null argument");
  *out = nullptr;
  int rc;
  if ((rc = check_desc(*target, "target")) || (rc = check_desc(*draft, "draft"))) return rc;
  if (target->vocab != draft->vocab) FAIL(SPEC_E_INVAL, "target and draft vocabularies differ");
  if (cfg->gamma_max < 1 || cfg->gamma_max > SPEC_MAX_TOKENS - 1) FAIL(SPEC_E_INVAL, "gamma_max outside 1..%d", SPEC_MAX_TOKENS - 1);
  if (cfg->page_tokens != SPEC_PAGE_TOKENS) FAIL(SPEC_E_INVAL, "page_tokens must be %d", SPEC_PAGE_TOKENS);
  if (cfg->max_seq < 1) FAIL(SPEC_E_INVAL, "max_seq must be positive");
  if (!(cfg->temperature >= 0.0f) || !(cfg->logit_scale > 0.0f)) FAIL(SPEC_E_INVAL, "bad temperature / logit_scale");
  {
    // the work splits (K slices of the projections, attention splits) are sized for the device's compute units
    int dev = 0, ncu = 0;
    HIPCHK(hipGetDevice(&dev));
    HIPCHK(hipDeviceGetAttribute(&ncu, hipDeviceAttributeMultiprocessorCount, dev));
    if (ncu < 1) FAIL(SPEC_E_HIP, "device reports %d compute units", ncu);
    spec_set_num_cu(ncu);
  }
  spec_ctx* c = new (std::nothrow) spec_ctx();
  if (!c) FAIL(SPEC_E_NOMEM, "out of host memory");
  c->cfg = *cfg;
  for (int i = 0; i < SPEC_RING_MAX; ++i) c->ev_slot_valid[i] = false, c->ev_slot[i] = nullptr;
  c->ring_n = 2 * cfg->gamma_max;
  if (c->ring_n > SPEC_RING_MAX) c->ring_n = SPEC_RING_MAX;
  rc = init_model(c->m[SPEC_TARGET], *target, *tw, *cfg, (hipStream_t)cfg->stream_target);
  if (!rc) rc = init_model(c->m[SPEC_DRAFT], *draft, *dw, *cfg, (hipStream_t)cfg->stream_draft);
  if (!rc) rc = dev_alloc(&c->qcache, (size_t)c->ring_n * target->vocab);
  if (!rc) rc = dev_alloc(&c->ring, (size_t)SPEC_RING_MAX);
  if (!rc) rc = dev_alloc(&c->accept_scratch, (size_t)256 + target->vocab);
  if (!rc) rc = dev_alloc(&c->res_dev, (size_t)1);
  if (!rc) {
    hipError_t e = hipMemset(c->ring, 0, SPEC_RING_MAX * sizeof(int));
    if (e == hipSuccess) e = hipHostMalloc((void**)&c->res_host, sizeof(AcceptResult), hipHostMallocDefault);
    for (int i = 0; i < c->ring_n && e == hipSuccess; ++i) e = hipEventCreateWithFlags(&c->ev_slot[i], hipEventDisableTiming);
    for (int i = 0; i < 2; ++i) {
      if (e == hipSuccess) e = hipEventCreate(&c->ev_t0[i]);
      if (e == hipSuccess) e = hipEventCreate(&c->ev_tend[i]);
      if (e == hipSuccess) e = hipEventCreate(&c->ev_dend[i]);
    }
    if (e == hipSuccess) e = hipDeviceSynchronize();
    if (e != hipSuccess) {
      spec_set_error("context set-up failed: %s", hipGetErrorString(e));
      rc = SPEC_E_HIP;
    }
  }
  if (rc) {
    spec_free(c);
    return rc;
  }
  *out = c;
  return SPEC_OK;
}

extern "C" void spec_free(spec_ctx* c) {
  if (!c) return;
  (void)hipDeviceSynchronize();
  free_model(c->m[0]);
  free_model(c->m[1]);
  if (c->qcache) (void)hipFree(c->qcache);
  if (c->ring) (void)hipFree(c->ring);
  if (c->accept_scratch) (void)hipFree(c->accept_scratch);
  if (c->res_dev) (void)hipFree(c->res_dev);
  if (c->res_host) (void)hipHostFree(c->res_host);
  for (int i = 0; i < SPEC_RING_MAX; ++i)
    if (c->ev_slot[i]) (void)hipEventDestroy(c->ev_slot[i]);
  if (c->prof.dev) (void)hipFree(c->prof.dev);
  for (int i = 0; i < 2; ++i) {
    if (c->ev_t0[i]) (void)hipEventDestroy(c->ev_t0[i]);
    if (c->ev_tend[i]) (void)hipEventDestroy(c->ev_tend[i]);
    if (c->ev_dend[i]) (void)hipEventDestroy(c->ev_dend[i]);
  }
  delete c;
}

extern "C" int spec_prefill(spec_ctx* c, const int32_t* prompt, int n_prompt, int which_mask) {
  if (!c || !prompt) FAIL(SPEC_E_INVAL, "null argument");
  if (n_prompt < 1) FAIL(SPEC_E_INVAL, "the prompt must hold at least one token");
  if (!(which_mask & 3)) FAIL(SPEC_E_INVAL, "which_mask selects no model");
  const int V = c->m[0].d.vocab;
  for (int i = 0; i < n_prompt; ++i)
    if (prompt[i] < 0 || prompt[i] >= V) FAIL(SPEC_E_INVAL, "prompt[%d] = %d outside the vocabulary", i, prompt[i]);
  for (int w = 0; w < 2; ++w)
    if (n_prompt - 1 + 2 * c->cfg.gamma_max > c->m[w].n_pages * SPEC_PAGE_TOKENS)
      FAIL(SPEC_E_NOMEM, "prompt of %d tokens does not fit max_seq", n_prompt);
  for (int w = 0; w < 2; ++w)
    if (((which_mask >> w) & 1) && c->prefill_opt == 1 && !dense_shapes_ok(c->m[w].d))
      FAIL(SPEC_E_INVAL, "dense prefill needs d_model, n_heads*head_dim and d_ffn to be multiples of 32");
  int rc;
  // from here on the caches are being rebuilt: until the call has succeeded the context takes no decoding call
  // (a prompt pass that fails half way, e.g. for lack of KV pages, must not leave a usable-looking context)
  c->prefilled = false;
  HIPCHK(hipStreamSynchronize(c->m[0].stream));
  HIPCHK(hipStreamSynchronize(c->m[1].stream));
  for (int w = 0; w < 2; ++w)
    if ((rc = rollback_model(c, w, 0))) return rc;
  reset_ring(c);
  c->committed.assign(prompt, prompt + n_prompt);
  c->n_prompt = n_prompt;
  c->last_verify_rows = 0;
  c->n_guess = -1;
  c->mode = SPEC_MODE_PRE;
  int fail_after = c->fail_prefill_after;   // one-shot test hook (SPEC_OPT_TEST_FAIL_PREFILL)
  c->fail_prefill_after = 0;
  auto injected_failure = [&]() {
    if (fail_after > 0 && --fail_after == 0) {
      spec_set_error("prompt pass abandoned half way (SPEC_OPT_TEST_FAIL_PREFILL)");
      return true;
    }
    return false;
  };
  for (int w = 0; w < 2; ++w) {
    if (!((which_mask >> w) & 1)) continue;
    if (c->prefill_opt == 1 || (c->prefill_opt < 0 && dense_shapes_ok(c->m[w].d) && n_prompt - 1 > 64)) {
      if ((rc = ensure_prefill_buffers(c->m[w]))) return rc;
      // the ids are copied from the context's own copy of the prompt, which outlives the asynchronous copy
      for (int s = 0; s < n_prompt - 1; s += c->m[w].pf_cap) {
        const int n = (n_prompt - 1 - s) < c->m[w].pf_cap ? (n_prompt - 1 - s) : c->m[w].pf_cap;
        if ((rc = prefill_dense_block(c, w, c->committed.data() + s, n))) return rc;
        if (injected_failure()) return SPEC_E_NOMEM;
      }
      continue;
    }
    for (int s = 0; s < n_prompt - 1; s += SPEC_MAX_TOKENS) {
      TokenSrc src;
      src.n = (n_prompt - 1 - s) < SPEC_MAX_TOKENS ? (n_prompt - 1 - s) : SPEC_MAX_TOKENS;
      for (int i = 0; i < src.n; ++i) src.imm[i] = prompt[s + i], src.slot[i] = 0;
      if ((rc = forward(c, w, src, 0))) return rc;
      if (injected_failure()) return SPEC_E_NOMEM;
    }
  }
  HIPCHK(hipStreamSynchronize(c->m[0].stream));
  HIPCHK(hipStreamSynchronize(c->m[1].stream));
  c->prefilled = true;
  return SPEC_OK;
}

extern "C" int spec_draft_step(spec_ctx* c, float u, int32_t* tok_out) {
  if (!c) FAIL(SPEC_E_INVAL, "null context");
  if (!c->prefilled) FAIL(SPEC_E_STATE, "spec_prefill has not run");
  if (!(u >= 0.0f && u < 1.0f)) FAIL(SPEC_E_INVAL, "uniform outside [0,1)");
  if (c->n_drafted >= c->ring_n) FAIL(SPEC_E_STATE, "%d unverified drafts already pending", c->n_drafted);
  ModelRt& m = c->m[SPEC_DRAFT];
  int rc;
  TokenSrc src;
  if (c->n_drafted == 0) {
    // feed every committed token the draft cache lacks; the last one is the frontier
    int missing = (int)c->committed.size() - m.len;
    if (missing < 1) FAIL(SPEC_E_STATE, "draft cache holds %d tokens but only %zu are committed", m.len, c->committed.size());
    while (missing > SPEC_MAX_TOKENS) {
      src.n = SPEC_MAX_TOKENS;
      for (int i = 0; i < src.n; ++i) src.imm[i] = c->committed[m.len + i], src.slot[i] = 0;
      if ((rc = forward(c, SPEC_DRAFT, src, 0))) return rc;
      missing -= SPEC_MAX_TOKENS;
    }
    src.n = missing;
    const int base = m.len;
    for (int i = 0; i < missing; ++i) src.imm[i] = c->committed[base + i], src.slot[i] = 0;
  } else {
    src.n = 1;
    src.imm[0] = -1;
    src.slot[0] = slot_of(c, c->n_drafted);
  }
  if ((rc = forward(c, SPEC_DRAFT, src, 1))) return rc;
  const int slot = slot_of(c, c->n_drafted + 1);
  const bool greedy = c->cfg.temperature == 0.0f;
  const float mult = greedy ? 1.0f : c->cfg.logit_scale / c->cfg.temperature;
  HIPCHK(launch_sample_row(m.logits, m.d.vocab, mult, greedy ? 1 : 0, u, c->qcache + (size_t)slot * m.d.vocab,
                           c->ring + slot, m.stream));
  HIPCHK(hipEventRecord(c->ev_slot[slot], m.stream));
  c->ev_slot_valid[slot] = true;
  c->n_drafted++;
  if (tok_out) {
    HIPCHK(hipStreamSynchronize(m.stream));
    HIPCHK(hipMemcpy(tok_out, c->ring + slot, sizeof(int), hipMemcpyDeviceToHost));
  }
  return SPEC_OK;
}

extern "C" int spec_verify(spec_ctx* c, const int32_t* tokens, int n_tokens, float* logits_out) {
  if (!c) FAIL(SPEC_E_INVAL, "null context");
  if (!c->prefilled) FAIL(SPEC_E_STATE, "spec_prefill has not run");
  if (n_tokens < 1 || n_tokens > SPEC_MAX_TOKENS) FAIL(SPEC_E_INVAL, "n_tokens outside 1..%d", SPEC_MAX_TOKENS);
  ModelRt& m = c->m[SPEC_TARGET];
  TokenSrc src;
  src.n = n_tokens;
  if (tokens) {
    for (int i = 0; i < n_tokens; ++i) {
      if (tokens[i] < 0 || tokens[i] >= m.d.vocab) FAIL(SPEC_E_INVAL, "tokens[%d] outside the vocabulary", i);
      src.imm[i] = tokens[i];
      src.slot[i] = 0;
    }
  } else {
    if (m.len != (int)c->committed.size() - 1)
      FAIL(SPEC_E_STATE, "target cache holds %d tokens, expected %zu", m.len, c->committed.size() - 1);
    // the frontier, then unverified drafts: x_2.. if x_1 is the frontier, else x_1..
    const int first = c->first_verified ? 2 : 1;
    const int n_dr = n_tokens - 1;
    if (first + n_dr - 1 > c->n_drafted) FAIL(SPEC_E_STATE, "%d drafts requested, %d pending", n_dr, c->n_drafted - first + 1);
    src.imm[0] = c->committed.back();
    src.slot[0] = 0;
    for (int i = 0; i < n_dr; ++i) src.imm[1 + i] = -1, src.slot[1 + i] = slot_of(c, first + i);
    if (n_dr > 0) {
      // The rows need draft tokens that may still be in the making (vanilla SD; PEARL verifies earlier steps' drafts,
      // which exist).  A target stream parked on a device-side wait makes every kernel launch of the running draft
      // stream about 1 us slower (measured: 3.91 instead of 3.64 ms per 7B-shape draft forward), so the host waits
      // for the draft chain instead and the target stream stays empty until it can run.
      hipEvent_t ev = c->ev_slot[slot_of(c, first + n_dr - 1)];
      if (hipEventQuery(ev) == hipErrorNotReady) HIPCHK(hipEventSynchronize(ev));
      HIPCHK(hipStreamWaitEvent(m.stream, ev, 0));
    }
  }
  int rc = forward(c, SPEC_TARGET, src, n_tokens);
  if (rc) return rc;
  c->last_verify_rows = n_tokens;
  c->n_guess = -1;
  if (logits_out) {
    HIPCHK(hipStreamSynchronize(m.stream));
    HIPCHK(hipMemcpy(logits_out, m.logits, (size_t)n_tokens * m.d.vocab * sizeof(float), hipMemcpyDeviceToHost));
  }
  return SPEC_OK;
}

// The library's candidate pool: the committed text as an n-gram cache.  Writes up to k tokens that followed the
// most recent earlier occurrence of the frontier token; returns how many (0 if the token has not occurred before).
static int pool_guesses(const std::vector<int>& text, int k, int* out) {
  const int n = (int)text.size();
  if (k <= 0 || n < 2) return 0;
  const int frontier = text[n - 1];
  int at = n - 2;
  while (at >= 0 && text[at] != frontier) --at;
  if (at < 0) return 0;
  int m = 0;
  for (int j = at + 1; j < n && m < k; ++j) out[m++] = text[j];
  return m;
}

extern "C" int spec_verify_guess(spec_ctx* c, const int32_t* guess, int n_guess, int* n_fed, float* logits_out) {
  if (!c) FAIL(SPEC_E_INVAL, "null context");
  if (!c->prefilled) FAIL(SPEC_E_STATE, "spec_prefill has not run");
  if (n_guess < 0 || n_guess > c->cfg.gamma_max - 1) FAIL(SPEC_E_INVAL, "n_guess outside 0..gamma_max-1 = %d", c->cfg.gamma_max - 1);
  ModelRt& m = c->m[SPEC_TARGET];
  if (c->first_verified) FAIL(SPEC_E_STATE, "pre-verify needs fresh drafts, but x_1 is already committed");
  if (m.len != (int)c->committed.size() - 1)
    FAIL(SPEC_E_STATE, "target cache holds %d tokens, expected %zu", m.len, c->committed.size() - 1);
  int g[SPEC_MAX_TOKENS];
  int ng = 0;
  if (guess) {
    for (int i = 0; i < n_guess; ++i) {
      if (guess[i] < 0 || guess[i] >= m.d.vocab) FAIL(SPEC_E_INVAL, "guess[%d] outside the vocabulary", i);
      g[i] = guess[i];
    }
    ng = n_guess;
  } else {
    ng = pool_guesses(c->committed, n_guess, g);
  }
  TokenSrc src;
  src.n = ng + 1;
  src.imm[0] = c->committed.back();
  src.slot[0] = 0;
  for (int i = 0; i < ng; ++i) src.imm[1 + i] = g[i], src.slot[1 + i] = 0;
  int rc = forward(c, SPEC_TARGET, src, ng + 1);
  if (rc) return rc;
  c->last_verify_rows = ng + 1;
  c->n_guess = ng;
  for (int i = 0; i < ng; ++i) c->guess[i] = g[i];
  if (n_fed) *n_fed = ng;
  if (logits_out) {
    HIPCHK(hipStreamSynchronize(m.stream));
    HIPCHK(hipMemcpy(logits_out, m.logits, (size_t)(ng + 1) * m.d.vocab * sizeof(float), hipMemcpyDeviceToHost));
  }
  return SPEC_OK;
}

extern "C" int spec_accept(spec_ctx* c, int kind, const float* r, int n_r, float u_resample, long long force_mask,
                           int* n_accepted, int32_t* tokens_out, int* n_out, int* next_mode, int* keep_len) {
  if (!c || !n_accepted || !tokens_out || !n_out || !next_mode || !keep_len) FAIL(SPEC_E_INVAL, "null argument");
  if (!(u_resample >= 0.0f && u_resample < 1.0f)) FAIL(SPEC_E_INVAL, "uniform outside [0,1)");
  ModelRt& mt = c->m[SPEC_TARGET];
  AcceptArgs a;
  memset(&a, 0, sizeof(a));
  a.kind = kind;
  a.u_resample = u_resample;
  a.force_mask = force_mask;
  a.n_rows = c->last_verify_rows;
  // draft index tested by logits row 0: x_2 when x_1 is already committed (it was the first token fed), else x_1
  const int first = c->first_verified ? 2 : 1;
  switch (kind) {
    case SPEC_ACCEPT_AR: a.n_test = 0; break;
    case SPEC_ACCEPT_SD: a.n_test = c->last_verify_rows - 1; break;    // the last row draws the bonus token
    case SPEC_ACCEPT_PRE: a.n_test = 1; break;
    case SPEC_ACCEPT_POST: a.n_test = c->last_verify_rows; break;      // every row tests a draft, no bonus
    case SPEC_ACCEPT_PRE_GUESS: a.n_test = c->last_verify_rows; break; // row i tests x_{i+1} while the drafts follow the guesses
    default: FAIL(SPEC_E_INVAL, "unknown accept kind %d", kind);
  }
  if (c->last_verify_rows < 1) FAIL(SPEC_E_STATE, "no target forward to accept against");
  if (kind == SPEC_ACCEPT_PRE && c->last_verify_rows != 1) FAIL(SPEC_E_STATE, "pre-verify needs a one-token target forward");
  if (kind == SPEC_ACCEPT_PRE_GUESS) {
    if (c->n_guess < 0 || c->last_verify_rows != c->n_guess + 1)
      FAIL(SPEC_E_STATE, "pre-verify over guesses needs the target forward of spec_verify_guess");
    if (c->first_verified) FAIL(SPEC_E_STATE, "pre-verify needs fresh drafts, but x_1 is already committed");
    a.guided = 1;
    for (int i = 0; i < c->n_guess; ++i) a.guess[i] = c->guess[i];
  }
  if (kind == SPEC_ACCEPT_PRE && c->first_verified) FAIL(SPEC_E_STATE, "pre-verify needs fresh drafts, but x_1 is already committed");
  if (first + a.n_test - 1 > c->n_drafted) FAIL(SPEC_E_STATE, "%d drafts to test, %d drafted", a.n_test, c->n_drafted);
  if (a.n_test > 0 && (!r || n_r < a.n_test)) FAIL(SPEC_E_INVAL, "%d acceptance uniforms needed", a.n_test);
  for (int i = 0; i < a.n_test; ++i) {
    if (!(r[i] >= 0.0f && r[i] < 1.0f)) FAIL(SPEC_E_INVAL, "uniform outside [0,1)");
    a.r[i] = r[i];
    a.slot[i] = slot_of(c, first + i);
  }
  if (a.n_test > 0) HIPCHK(hipStreamWaitEvent(mt.stream, c->ev_slot[a.slot[a.n_test - 1]], 0));
  const bool greedy = c->cfg.temperature == 0.0f;
  const float mult = greedy ? 1.0f : c->cfg.logit_scale / c->cfg.temperature;
  HIPCHK(launch_accept(mt.logits, mt.d.vocab, mult, greedy ? 1 : 0, c->qcache, c->ring, nullptr, a, c->accept_scratch,
                       c->res_dev, mt.stream));
  HIPCHK(hipMemcpyAsync(c->res_host, c->res_dev, sizeof(AcceptResult), hipMemcpyDeviceToHost, mt.stream));
  HIPCHK(hipStreamSynchronize(mt.stream));
  const AcceptResult& res = *c->res_host;
  const int n = res.n_accepted;
  int no = 0;
  *keep_len = -1;
  c->last_verify_rows = 0;
  c->n_guess = -1;
  bool cut_target = false;
  switch (kind) {
    case SPEC_ACCEPT_AR:
      tokens_out[no++] = res.token;
      *next_mode = SPEC_MODE_PRE;
      break;
    case SPEC_ACCEPT_SD:
      for (int i = 0; i < n; ++i) tokens_out[no++] = res.ring[a.slot[i]];
      tokens_out[no++] = res.token;
      *next_mode = SPEC_MODE_PRE;
      reset_ring(c);
      break;
    case SPEC_ACCEPT_PRE:
      if (n == 1) {
        tokens_out[no++] = res.ring[a.slot[0]];
        c->first_verified = true;
        *next_mode = SPEC_MODE_POST;
      } else {
        tokens_out[no++] = res.token;
        reset_ring(c);
        *next_mode = SPEC_MODE_PRE;
      }
      break;
    case SPEC_ACCEPT_POST:
      for (int i = 0; i < n; ++i) tokens_out[no++] = res.ring[a.slot[i]];
      if (n == a.n_test) {
        // the last accepted draft x_L (L = first + n_test - 1) is the new frontier and becomes x_1
        const int shift = first + a.n_test - 2;
        c->ring_base = (c->ring_base + shift) % c->ring_n;
        c->n_drafted -= shift;
        c->first_verified = true;
        *next_mode = SPEC_MODE_POST;
      } else {
        tokens_out[no++] = res.token;
        reset_ring(c);
        *next_mode = SPEC_MODE_PRE;
      }
      break;
    case SPEC_ACCEPT_PRE_GUESS:
      for (int i = 0; i < n; ++i) tokens_out[no++] = res.ring[a.slot[i]];
      if (res.rejected) {
        tokens_out[no++] = res.token;
        reset_ring(c);
        *next_mode = SPEC_MODE_PRE;
      } else {
        // x_n (n >= 1: row 0 always tests x_1) is the new frontier and becomes x_1; x_{n+1}.. stay pending
        c->ring_base = (c->ring_base + n - 1) % c->ring_n;
        c->n_drafted -= n - 1;
        c->first_verified = true;
        cut_target = true;   // the guess rows behind the new frontier leave the target cache
        *next_mode = SPEC_MODE_POST;
      }
      break;
  }
  for (int i = 0; i < no; ++i) c->committed.push_back(tokens_out[i]);
  if (cut_target && mt.len > (int)c->committed.size() - 1) {
    int rc = rollback_model(c, SPEC_TARGET, (int)c->committed.size() - 1);
    if (rc) return rc;
  }
  if (kind == SPEC_ACCEPT_SD || res.rejected) *keep_len = (int)c->committed.size() - 1;
  *n_accepted = n;
  *n_out = no;
  c->mode = *next_mode;
  return SPEC_OK;
}

extern "C" int spec_rollback_kv(spec_ctx* c, int which, int new_len) {
  if (!c || (which != SPEC_TARGET && which != SPEC_DRAFT)) FAIL(SPEC_E_INVAL, "bad argument");
  return rollback_model(c, which, new_len);
}

extern "C" int spec_drop_drafts(spec_ctx* c) {
  if (!c) FAIL(SPEC_E_INVAL, "null context");
  reset_ring(c);
  c->mode = SPEC_MODE_PRE;
  return SPEC_OK;
}

extern "C" int spec_rewind(spec_ctx* c, int committed_len) {
  if (!c) FAIL(SPEC_E_INVAL, "null context");
  if (!c->prefilled) FAIL(SPEC_E_STATE, "spec_prefill has not run");
  if (committed_len < 1 || committed_len > (int)c->committed.size())
    FAIL(SPEC_E_INVAL, "rewind to %d outside [1, %zu]", committed_len, c->committed.size());
  c->committed.resize(committed_len);
  reset_ring(c);
  c->mode = SPEC_MODE_PRE;
  c->last_verify_rows = 0;
  c->n_guess = -1;
  for (int w = 0; w < 2; ++w)
    if (c->m[w].len > committed_len - 1) {
      int rc = rollback_model(c, w, committed_len - 1);
      if (rc) return rc;
    }
  return SPEC_OK;
}

extern "C" int spec_kv_len(const spec_ctx* c, int which) {
  if (!c || (which != SPEC_TARGET && which != SPEC_DRAFT)) return SPEC_E_INVAL;
  return c->m[which].len;
}
extern "C" int spec_pending_rows(const spec_ctx* c) {
  if (!c) return SPEC_E_INVAL;
  if (c->n_drafted == 0) return 0;
  return c->first_verified ? c->n_drafted : c->n_drafted + 1;
}
extern "C" int spec_committed_len(const spec_ctx* c) { return c ? (int)c->committed.size() : SPEC_E_INVAL; }
extern "C" int spec_kv_free_pages(const spec_ctx* c, int which) {
  if (!c || (which != SPEC_TARGET && which != SPEC_DRAFT)) return SPEC_E_INVAL;
  return (int)c->m[which].free_pages.size();
}
extern "C" long long spec_forward_count(const spec_ctx* c, int which) {
  if (!c || (which != SPEC_TARGET && which != SPEC_DRAFT)) return SPEC_E_INVAL;
  return c->m[which].n_forwards;
}

// -------------------------------------------------------------------------------------------
// Loops (host control flow over the calls above)
// -------------------------------------------------------------------------------------------
extern "C" int spec_generate(spec_ctx* c, int algo, int gamma, int n_generate, int max_steps, const float* u_draft,
                             const float* r_accept, const float* u_resample, const uint8_t* force_bits,
                             int32_t* out_tokens, double* stats) {
  if (!c || !out_tokens || !u_resample) FAIL(SPEC_E_INVAL, "null argument");
  if (algo < 0 || algo > 5)
    FAIL(SPEC_E_INVAL, "algo must be 0 (AR), 1 (SD), 2 (PEARL), 3 (PEARL w/o pre-verify), 4 (PEARL w/o post-verify) or "
                       "5 (PEARL with pre-verify over guesses)");
  if (algo > 0 && (gamma < 1 || gamma > c->cfg.gamma_max || !u_draft || !r_accept)) FAIL(SPEC_E_INVAL, "bad gamma / uniforms");
  if (n_generate < 1) FAIL(SPEC_E_INVAL, "n_generate must be positive");
  if (!c->prefilled) FAIL(SPEC_E_STATE, "spec_prefill has not run");
  // Drafts left pending by an earlier call belong to that call's loop and window: autoregressive and vanilla
  // speculative decoding start from none, the PEARL variants may go on where a PEARL call with the same window stopped.
  if (algo <= 1 && c->n_drafted > 0)
    FAIL(SPEC_E_STATE, "%d unverified drafts pending: drop them (spec_drop_drafts + spec_rollback_kv, or spec_rewind) first",
         c->n_drafted);
  if (algo >= 2 && algo != 5 && c->n_drafted != 0 && c->n_drafted != gamma)
    FAIL(SPEC_E_STATE, "%d unverified drafts pending do not fit a window of %d", c->n_drafted, gamma);
  // pre-verify over guesses leaves 1..gamma drafts pending, the first of them committed
  if (algo == 5 && c->n_drafted != 0 && (c->n_drafted > gamma || !c->first_verified))
    FAIL(SPEC_E_STATE, "%d unverified drafts pending do not fit a window of %d", c->n_drafted, gamma);
  const int k_guess = (c->guess_opt < 0 || c->guess_opt > gamma - 1) ? gamma - 1 : c->guess_opt;
  const int g1 = gamma + 1;
  // the launch mode is put back on every way out of the loop, errors included
  struct WgsGuard {
    spec_ctx* c;
    int saved;
    ~WgsGuard() { c->wgs = saved; }
  } wgs_guard{c, c->wgs};
  // while the two streams overlap, one projection workgroup per CU and stream is better from gamma 6 on (long draft chains),
  // two per CU below that (measured on the 70B/7B-shape pair)
  if (c->wgs_opt < 0) c->wgs = ((algo >= 2) && (c->m[0].stream != c->m[1].stream) && gamma >= 6) ? SPEC_PEARL_WGS_PER_CU : 2;
  int mode = c->mode;
  int produced = 0, rc = 0;
  long long steps = 0, accepted = 0, tested = 0, post_steps = 0;
  const long long f0t = c->m[0].n_forwards, f0d = c->m[1].n_forwards;
  const size_t base = c->committed.size();
  auto t0 = std::chrono::steady_clock::now();
  int toks[SPEC_MAX_TOKENS + 1];
  while (produced < n_generate && (max_steps <= 0 || steps < max_steps)) {
    const long long t = steps;
    int n_acc = 0, n_out = 0, next_mode = SPEC_MODE_PRE, keep = -1, kind;
    // where both chains of the step start and end (timed events): the balance of the next steps is set from it
    const bool balance = (algo == 2 || algo == 5) && c->wgs == 1 && c->tail_opt < 0 && c->m[0].stream != c->m[1].stream;
    const int bset = (int)(steps & 1);
    if (balance) {
      c->bal_valid[bset] = false;
      HIPCHK(hipEventRecord(c->ev_t0[bset], c->m[SPEC_TARGET].stream));
    }
    long long fm = -1;
    int n_test = 0;
    if (algo == 0) {
      kind = SPEC_ACCEPT_AR;
      if ((rc = spec_verify(c, nullptr, 1, nullptr))) return rc;
    } else if (algo == 1) {
      kind = SPEC_ACCEPT_SD;
      n_test = gamma;
      for (int i = 0; i < gamma; ++i)
        if ((rc = spec_draft_step(c, u_draft[t * gamma + i], nullptr))) return rc;
      if ((rc = spec_verify(c, nullptr, gamma + 1, nullptr))) return rc;
    } else if (algo == 3) {
      // PEARL without pre-verify: after a rejection one step only drafts; every other step verifies what is
      // pending (the first time together with the frontier: gamma + 1 rows) while the draft goes on
      if (c->n_drafted == 0) {
        for (int i = 0; i < gamma; ++i)
          if ((rc = spec_draft_step(c, u_draft[t * gamma + i], nullptr))) return rc;
        steps++;
        continue;
      }
      kind = SPEC_ACCEPT_POST;
      n_test = c->first_verified ? gamma : gamma + 1;
      post_steps++;
      if ((rc = spec_verify(c, nullptr, n_test, nullptr))) return rc;
      for (int i = 0; i < gamma; ++i)
        if ((rc = spec_draft_step(c, u_draft[t * gamma + i], nullptr))) return rc;
    } else if (algo == 4 && mode == SPEC_MODE_POST) {
      // PEARL without post-verify: x_1 was accepted early; the target verifies x_2..x_gamma (bonus token from the
      // last row) while the draft model idles
      kind = SPEC_ACCEPT_SD;
      n_test = gamma - 1;
      post_steps++;
      if ((rc = spec_verify(c, nullptr, gamma, nullptr))) return rc;
    } else if (algo == 5 && mode == SPEC_MODE_PRE) {
      // pre-verify over the frontier and up to k guessed tokens (closing remark of Section 4.3)
      kind = SPEC_ACCEPT_PRE_GUESS;
      int fed = 0;
      if ((rc = spec_verify_guess(c, nullptr, k_guess, &fed, nullptr))) return rc;
      n_test = fed + 1;
      for (int i = 0; i < gamma; ++i)
        if ((rc = spec_draft_step(c, u_draft[t * gamma + i], nullptr))) return rc;
    } else if (algo == 5) {
      // post-verify of what the pre-verify step left of the window: the frontier x_1 and the drafts behind it
      kind = SPEC_ACCEPT_POST;
      n_test = c->n_drafted;
      post_steps++;
      if ((rc = spec_verify(c, nullptr, n_test, nullptr))) return rc;
      for (int i = 0; i < gamma; ++i)
        if ((rc = spec_draft_step(c, u_draft[t * gamma + i], nullptr))) return rc;
    } else if (mode == SPEC_MODE_PRE) {
      kind = SPEC_ACCEPT_PRE;
      n_test = 1;
      if ((rc = spec_verify(c, nullptr, 1, nullptr))) return rc;
      for (int i = 0; i < gamma; ++i)
        if ((rc = spec_draft_step(c, u_draft[t * gamma + i], nullptr))) return rc;
    } else {
      kind = SPEC_ACCEPT_POST;
      n_test = gamma;
      post_steps++;
      if ((rc = spec_verify(c, nullptr, gamma, nullptr))) return rc;
      for (int i = 0; i < gamma; ++i)
        if ((rc = spec_draft_step(c, u_draft[t * gamma + i], nullptr))) return rc;
    }
    if (balance) {
      HIPCHK(hipEventRecord(c->ev_tend[bset], c->m[SPEC_TARGET].stream));
      HIPCHK(hipEventRecord(c->ev_dend[bset], c->m[SPEC_DRAFT].stream));
      c->bal_valid[bset] = true;
    }
    if (force_bits && n_test > 0) {
      fm = 0;
      for (int i = 0; i < n_test; ++i)
        if (force_bits[t * g1 + i]) fm |= (1LL << i);
    }
    if ((rc = spec_accept(c, kind, algo ? r_accept + t * g1 : nullptr, g1, u_resample[t], fm, &n_acc, toks, &n_out,
                          &next_mode, &keep)))
      return rc;
    if (keep >= 0)
      for (int w = 0; w < 2; ++w) {
        const int len = c->m[w].len;
        if (len > keep && (rc = rollback_model(c, w, keep))) return rc;
      }
    if (balance && c->bal_valid[bset ^ 1]) {
      // The step before this one: both its chains have ended by now (this step's accept waited for a draft that
      // the draft stream produced behind them), whereas this step's draft chain may still be running - PEARL does
      // not wait for it.  Target chain later than the draft chain: more trailing target layers launch with two
      // workgroups per CU; the other way round: fewer.  A chunk that changes mode moves the two ends apart by
      // 0.4 - 1.3 ms of a 42 ms step (measured on the 70B/7B shapes; a chunk is 1 / 20 of the target chain); the
      // boundary moves by the lag counted in chunk times, at most 4 chunks a step, which errs on the slow side.
      // Both ends are timed from the step's start: the time between two events is only defined forwards.
      const int o = bset ^ 1;
      c->bal_valid[o] = false;
      float span_ms = 0.f, draft_ms = 0.f;
      const int L = c->m[SPEC_TARGET].d.n_layers, ch = tail_chunk_layers(L);
      if (ch > 0 && hipEventElapsedTime(&span_ms, c->ev_t0[o], c->ev_tend[o]) == hipSuccess &&
          hipEventElapsedTime(&draft_ms, c->ev_t0[o], c->ev_dend[o]) == hipSuccess && span_ms > 0.f) {
        const float late_ms = span_ms - draft_ms;             // > 0: the target chain ended later
        const int most = (L - (L >= 8 ? 4 : L)) / ch * ch;
        const float unit = span_ms * (float)ch / (float)L;
        int move = (int)(late_ms / unit);                     // towards zero
        if (move == 0 && late_ms > 0.3f * unit) move = 1;
        if (move == 0 && late_ms < -0.3f * unit) move = -1;
        if (move > 4) move = 4;
        if (move < -4) move = -4;
        const int t2 = c->tail_layers + move * ch;
        c->tail_layers = t2 < 0 ? 0 : (t2 > most ? most : t2);
      } else {
        (void)hipGetLastError();
      }
    }
    accepted += n_acc;
    // tokens actually tested: up to and including the first rejection (a pre-verify over guesses may stop earlier
    // without one: keep >= 0 tells a rejection there)
    if (kind == SPEC_ACCEPT_PRE_GUESS) tested += n_acc + (keep >= 0 ? 1 : 0);
    else tested += (n_acc < n_test) ? n_acc + 1 : n_test;
    produced += n_out;
    mode = next_mode;
    steps++;
  }
  HIPCHK(hipStreamSynchronize(c->m[0].stream));
  HIPCHK(hipStreamSynchronize(c->m[1].stream));
  auto t1 = std::chrono::steady_clock::now();
  for (int i = 0; i < n_generate && i < produced; ++i) out_tokens[i] = c->committed[base + i];
  if (stats) {
    stats[0] = (double)steps;
    stats[1] = (double)produced;
    stats[2] = (double)(c->m[1].n_forwards - f0d);
    stats[3] = (double)(c->m[0].n_forwards - f0t);
    stats[4] = (double)accepted;
    stats[5] = (double)tested;
    stats[6] = (double)post_steps;
    stats[7] = std::chrono::duration<double>(t1 - t0).count();
  }
  return SPEC_OK;
}

// Window size gamma = round(c), c = T(target forward) / T(draft forward) (Section 4.4.1).
extern "C" int spec_calibrate_gamma(spec_ctx* c, int n_iter, int cap, int concurrent, int* gamma_out,
                                    double* t_target_s, double* t_draft_s) {
  if (!c || !gamma_out || !t_target_s || !t_draft_s) FAIL(SPEC_E_INVAL, "null argument");
  if (n_iter < 1 || cap < 1) FAIL(SPEC_E_INVAL, "n_iter and cap must be positive");
  if (!c->prefilled) FAIL(SPEC_E_STATE, "spec_prefill has not run");
  if (c->n_drafted > 0 || c->last_verify_rows > 0)
    FAIL(SPEC_E_STATE, "calibration needs a context between steps with no drafts pending");
  ModelRt &mt = c->m[SPEC_TARGET], &md = c->m[SPEC_DRAFT];
  if (mt.len != (int)c->committed.size() - 1 || md.len > (int)c->committed.size() - 1)
    FAIL(SPEC_E_STATE, "caches do not match the committed tokens");
  const int lt = mt.len, ld = md.len;
  int rc = SPEC_OK;
  // the forwards of the timed runs append to the caches: never more than fits
  const int room_t = mt.n_pages * SPEC_PAGE_TOKENS - lt, room_d = md.n_pages * SPEC_PAGE_TOKENS - (int)c->committed.size();
  int nt = n_iter < room_t ? n_iter : room_t;
  int nd = n_iter < c->ring_n ? n_iter : c->ring_n;
  if (nd > room_d) nd = room_d;
  if (nt < 1 || nd < 1) FAIL(SPEC_E_NOMEM, "no room in the caches for a timed forward");
  struct WgsGuard {
    spec_ctx* c;
    int saved;
    ~WgsGuard() { c->wgs = saved; }
  } wgs_guard{c, c->wgs};
  if (concurrent && c->wgs_opt < 0) c->wgs = SPEC_PEARL_WGS_PER_CU;
  TokenSrc src;
  src.n = 1;
  src.imm[0] = c->committed.back();
  src.slot[0] = 0;
  auto restore = [&]() -> int {   // leave caches, ring and mode as they were found
    int r2;
    HIPCHK(hipStreamSynchronize(mt.stream));
    HIPCHK(hipStreamSynchronize(md.stream));
    reset_ring(c);
    c->last_verify_rows = 0;
    if ((r2 = rollback_model(c, SPEC_TARGET, lt))) return r2;
    if ((r2 = rollback_model(c, SPEC_DRAFT, ld))) return r2;
    HIPCHK(hipStreamSynchronize(mt.stream));
    HIPCHK(hipStreamSynchronize(md.stream));
    return SPEC_OK;
  };
  auto fail = [&](int code) {
    (void)restore();
    return code;
  };
  // untimed: the first forward of a shape also captures its graphs
  if ((rc = forward(c, SPEC_TARGET, src, 1))) return fail(rc);
  if ((rc = spec_draft_step(c, 0.5f, nullptr))) return fail(rc);
  if ((rc = restore())) return rc;
  using clk = std::chrono::steady_clock;
  double tp = 0.0, tq = 0.0;
  if (!concurrent) {
    auto t0 = clk::now();
    for (int i = 0; i < nt; ++i)
      if ((rc = forward(c, SPEC_TARGET, src, 1))) return fail(rc);
    HIPCHK(hipStreamSynchronize(mt.stream));
    tp = std::chrono::duration<double>(clk::now() - t0).count() / nt;
    if ((rc = restore())) return rc;
    t0 = clk::now();
    for (int i = 0; i < nd; ++i)
      if ((rc = spec_draft_step(c, 0.5f, nullptr))) return fail(rc);
    HIPCHK(hipStreamSynchronize(md.stream));
    tq = std::chrono::duration<double>(clk::now() - t0).count() / nd;
  } else {
    // Both streams busy at once, as inside a PEARL step: A target forwards beside B draft steps, B chosen from a
    // first round so that the two chains end about together; each chain's time per forward is taken from its own
    // start and end events.
    if (mt.stream == md.stream) return fail((spec_set_error("concurrent calibration needs two streams"), SPEC_E_STATE));
    hipEvent_t ev[4] = {nullptr, nullptr, nullptr, nullptr};
    auto destroy = [&]() {
      for (hipEvent_t& e : ev)
        if (e) (void)hipEventDestroy(e), e = nullptr;
    };
    for (hipEvent_t& e : ev)
      if (hipEventCreate(&e) != hipSuccess) {
        destroy();
        return fail((spec_set_error("hipEventCreate failed"), SPEC_E_HIP));
      }
    int A = 1, B = nd < 4 ? nd : 4;
    for (int round = 0; round < 2; ++round) {
      hipError_t e = hipEventRecord(ev[0], mt.stream);
      if (e == hipSuccess) e = hipEventRecord(ev[2], md.stream);
      for (int i = 0; i < A && !rc && e == hipSuccess; ++i) rc = forward(c, SPEC_TARGET, src, 1);
      for (int i = 0; i < B && !rc && e == hipSuccess; ++i) rc = spec_draft_step(c, 0.5f, nullptr);
      if (e == hipSuccess && !rc) e = hipEventRecord(ev[1], mt.stream);
      if (e == hipSuccess && !rc) e = hipEventRecord(ev[3], md.stream);
      if (e == hipSuccess && !rc) e = hipEventSynchronize(ev[1]);
      if (e == hipSuccess && !rc) e = hipEventSynchronize(ev[3]);
      float ms_t = 0.f, ms_d = 0.f;
      if (e == hipSuccess && !rc) e = hipEventElapsedTime(&ms_t, ev[0], ev[1]);
      if (e == hipSuccess && !rc) e = hipEventElapsedTime(&ms_d, ev[2], ev[3]);
      if (rc || e != hipSuccess) {
        destroy();
        if (!rc) spec_set_error("concurrent calibration failed: %s", hipGetErrorString(e)), rc = SPEC_E_HIP;
        return fail(rc);
      }
      tp = ms_t * 1e-3 / A;
      tq = ms_d * 1e-3 / B;
      if ((rc = restore())) {
        destroy();
        return rc;
      }
      // second round: two target forwards beside as many draft steps as take about the same time
      A = nt < 2 ? nt : 2;
      long long want = (long long)(A * tp / (tq > 0 ? tq : 1e-9) + 0.5);
      B = (int)(want < 1 ? 1 : (want > nd ? nd : want));
    }
    destroy();
  }
  if ((rc = restore())) return rc;
  double cc = tq > 0 ? tp / tq : (double)cap;
  int g = (int)(cc + 0.5);
  if (g < 1) g = 1;
  if (g > cap) g = cap;
  if (g > c->cfg.gamma_max) g = c->cfg.gamma_max;
  *gamma_out = g;
  *t_target_s = tp;
  *t_draft_s = tq;
  return SPEC_OK;
}

// -------------------------------------------------------------------------------------------
// Set-up helpers and single kernels
// -------------------------------------------------------------------------------------------
extern "C" size_t spec_packed_bytes(int N, int K) { return (size_t)(N / 16) * ((K + 31) / 32) * 1024; }

extern "C" int spec_pack_weight(void* dst, const void* src, int N, int K, int panel_start, int panel_step, void* stream) {
  if (!dst || !src) FAIL(SPEC_E_INVAL, "null pointer");
  if (N < 16 || N % 16 || K < 8 || K % 8 || panel_start < 0 || panel_step < 1) FAIL(SPEC_E_INVAL, "N %% 16, K %% 8 required");
  HIPCHK(launch_pack_weight(dst, src, N, K, panel_start, panel_step, (hipStream_t)stream));
  return SPEC_OK;
}

static int check_gemm_args(int M, int N, int K) {
  if (M < 1 || M > SPEC_MAX_TOKENS || N < 16 || N % 16 || K < 8 || K % 8)
    FAIL(SPEC_E_INVAL, "gemm needs 1 <= M <= %d, N %% 16 == 0, K %% 8 == 0", SPEC_MAX_TOKENS);
  return SPEC_OK;
}
extern "C" size_t spec_gemm_workspace_bytes(int M, int N, int K) {
  if (check_gemm_args(M, N, K)) return 0;
  return gemm_plan(M, N, K).partial_bytes();
}
extern "C" int spec_gemm_plan_query(int M, int N, int K, int workgroups_per_cu, int* out6) {
  if (!out6) FAIL(SPEC_E_INVAL, "null pointer");
  if (workgroups_per_cu != 1 && workgroups_per_cu != 2) FAIL(SPEC_E_INVAL, "workgroups_per_cu must be 1 or 2");
  int rc = check_gemm_args(M, N, K);
  if (rc) return rc;
  const GemmPlan p = gemm_plan(M, N, K, workgroups_per_cu);
  out6[0] = p.S; out6[1] = p.spw; out6[2] = p.Gs; out6[3] = p.NT; out6[4] = p.steps; out6[5] = p.MT;
  return SPEC_OK;
}
extern "C" int spec_gemm_partials(const void* x, const void* w, int M, int N, int K, void* work, void* stream) {
  if (!x || !w || !work) FAIL(SPEC_E_INVAL, "null pointer");
  int rc = check_gemm_args(M, N, K);
  if (rc) return rc;
  GemmPlan p = gemm_plan(M, N, K);
  HIPCHK(launch_gemm_partials(p, (const bf16*)x, w, (float*)work, (hipStream_t)stream, 2));
  return SPEC_OK;
}
extern "C" int spec_gemm(float* y, const void* x, const void* w, int M, int N, int K, void* work, void* stream) {
  if (!y) FAIL(SPEC_E_INVAL, "null pointer");
  int rc = spec_gemm_partials(x, w, M, N, K, work, stream);
  if (rc) return rc;
  GemmPlan p = gemm_plan(M, N, K);
  HIPCHK(launch_reduce_partials(y, (const float*)work, p.S, (size_t)M * N, (hipStream_t)stream));
  return SPEC_OK;
}

extern "C" int spec_dense_gemm(float* y, void* z, const void* x, const void* w, int M, int N, int K, int epilogue,
                               void* stream) {
  if (!x || !w) FAIL(SPEC_E_INVAL, "null pointer");
  if (epilogue < 0 || epilogue > 2) FAIL(SPEC_E_INVAL, "epilogue must be 0, 1 or 2");
  if (M < 1 || N < 16 || N % 16 || K < 32 || K % 32) FAIL(SPEC_E_INVAL, "need M >= 1, N %% 16 == 0, K %% 32 == 0");
  if (epilogue == 2 ? (!z || N % 32) : !y) FAIL(SPEC_E_INVAL, "output pointer missing (or N %% 32 != 0 for epilogue 2)");
  HIPCHK(launch_dense_gemm((const bf16*)x, w, M, N, K, epilogue, y, (bf16*)z, (hipStream_t)stream));
  return SPEC_OK;
}

extern "C" int spec_read_probe(const void* src, size_t bytes, void* out, void* stream) {
  if (!src || !out || bytes < 16) FAIL(SPEC_E_INVAL, "bad argument");
  HIPCHK(launch_read_probe(src, bytes, out, (hipStream_t)stream));
  return SPEC_OK;
}

extern "C" int spec_sample_row(const float* logits, int vocab, float temperature, float logit_scale, float u,
                               float* q_out, int32_t* tok_out, void* stream) {
  if (!logits || !q_out || !tok_out || vocab < 1) FAIL(SPEC_E_INVAL, "bad argument");
  if (!(u >= 0.0f && u < 1.0f) || !(temperature >= 0.0f)) FAIL(SPEC_E_INVAL, "bad uniform / temperature");
  const bool greedy = temperature == 0.0f;
  HIPCHK(launch_sample_row(logits, vocab, greedy ? 1.0f : logit_scale / temperature, greedy ? 1 : 0, u, q_out, tok_out,
                           (hipStream_t)stream));
  return SPEC_OK;
}

extern "C" int spec_accept_rows(const float* p_logits, int n_rows, const float* q_rows, const int32_t* x, int n_test,
                                int vocab, float temperature, float logit_scale, const float* r, float u_resample,
                                int32_t* result, void* stream) {
  if (!p_logits || !result || vocab < 1 || n_rows < 1 || n_rows > SPEC_MAX_TOKENS || n_test < 0 || n_test > n_rows)
    FAIL(SPEC_E_INVAL, "bad argument");
  if (n_test > 0 && (!q_rows || !x || !r)) FAIL(SPEC_E_INVAL, "null pointer");
  AcceptArgs a;
  memset(&a, 0, sizeof(a));
  a.n_rows = n_rows;
  a.n_test = n_test;
  a.u_resample = u_resample;
  a.force_mask = -1;
  for (int i = 0; i < n_test; ++i) a.r[i] = r[i];
  float* scratch = nullptr;
  AcceptResult* res = nullptr;
  hipStream_t st = (hipStream_t)stream;
  if (hipMalloc((void**)&scratch, (256 + (size_t)vocab) * sizeof(float)) != hipSuccess ||
      hipMalloc((void**)&res, sizeof(AcceptResult)) != hipSuccess) {
    if (scratch) (void)hipFree(scratch);
    FAIL(SPEC_E_NOMEM, "hipMalloc failed");
  }
  const bool greedy = temperature == 0.0f;
  AcceptResult host;
  hipError_t e = launch_accept(p_logits, vocab, greedy ? 1.0f : logit_scale / temperature, greedy ? 1 : 0, q_rows,
                               nullptr, x, a, scratch, res, st);
  if (e == hipSuccess) e = hipStreamSynchronize(st);
  if (e == hipSuccess) e = hipMemcpy(&host, res, sizeof(host), hipMemcpyDeviceToHost);
  (void)hipFree(scratch);
  (void)hipFree(res);
  if (e != hipSuccess) FAIL(SPEC_E_HIP, "accept kernels failed: %s", hipGetErrorString(e));
  result[0] = host.n_accepted;
  result[1] = host.token;
  return SPEC_OK;
}

extern "C" int spec_set_option(spec_ctx* c, int option, int value) {
  if (!c) FAIL(SPEC_E_INVAL, "null context");
  if (option == SPEC_OPT_GEMM_WGS_PER_CU) {
    if (value != -1 && value != 1 && value != 2) FAIL(SPEC_E_INVAL, "SPEC_OPT_GEMM_WGS_PER_CU takes -1, 1 or 2");
    c->wgs_opt = value;
    c->wgs = value < 0 ? 2 : value;
    return SPEC_OK;
  }
  if (option == SPEC_OPT_GRAPHS) {
    if (value != 0 && value != 1) FAIL(SPEC_E_INVAL, "SPEC_OPT_GRAPHS takes 0 or 1");
    c->use_graphs = value == 1;
    return SPEC_OK;
  }
  if (option == SPEC_OPT_FUSE_SINGLE) {
    if (value != 0 && value != 1) FAIL(SPEC_E_INVAL, "SPEC_OPT_FUSE_SINGLE takes 0 or 1");
    if (c->fuse_single != (value == 1)) {
      // captured single-token forwards belong to the other kernel chain
      HIPCHK(hipStreamSynchronize(c->m[0].stream));
      HIPCHK(hipStreamSynchronize(c->m[1].stream));
      for (ModelRt& m : c->m)
        for (auto& b : m.graphs[1])
          for (auto& cc : b)
            for (hipGraphExec_t& g : cc)
              if (g) {
                (void)hipGraphExecDestroy(g);
                g = nullptr;
              }
    }
    c->fuse_single = value == 1;
    return SPEC_OK;
  }
  if (option == SPEC_OPT_PREFILL) {
    if (value < -1 || value > 1) FAIL(SPEC_E_INVAL, "SPEC_OPT_PREFILL takes -1, 0 or 1");
    c->prefill_opt = value;
    return SPEC_OK;
  }
  if (option == SPEC_OPT_TARGET_TAIL_LAYERS) {
    if (value < -1) FAIL(SPEC_E_INVAL, "SPEC_OPT_TARGET_TAIL_LAYERS takes -1 or a layer count");
    const int L = c->m[SPEC_TARGET].d.n_layers, most = L - (L >= 8 ? 4 : L);
    c->tail_opt = value;
    c->tail_layers = value < 0 ? 0 : (value > most ? most : value);
    return SPEC_OK;
  }
  if (option == SPEC_OPT_GUESS_TOKENS) {
    if (value < -1 || value > SPEC_MAX_TOKENS - 2) FAIL(SPEC_E_INVAL, "SPEC_OPT_GUESS_TOKENS takes -1 or 0..%d", SPEC_MAX_TOKENS - 2);
    c->guess_opt = value;
    return SPEC_OK;
  }
  if (option == SPEC_OPT_TEST_FAIL_PREFILL) {
    if (value < 0) FAIL(SPEC_E_INVAL, "SPEC_OPT_TEST_FAIL_PREFILL takes a count >= 0");
    c->fail_prefill_after = value;
    return SPEC_OK;
  }
  FAIL(SPEC_E_INVAL, "unknown option %d", option);
}

extern "C" int spec_get_option(const spec_ctx* c, int option, int* value) {
  if (!c || !value) FAIL(SPEC_E_INVAL, "null argument");
  switch (option) {
    case SPEC_OPT_GEMM_WGS_PER_CU: *value = c->wgs; return SPEC_OK;       // what the next forward launches with
    case SPEC_OPT_GRAPHS: *value = c->use_graphs ? 1 : 0; return SPEC_OK;
    case SPEC_OPT_PREFILL: *value = c->prefill_opt; return SPEC_OK;
    case SPEC_OPT_FUSE_SINGLE: *value = c->fuse_single ? 1 : 0; return SPEC_OK;
    case SPEC_OPT_TEST_FAIL_PREFILL: *value = c->fail_prefill_after; return SPEC_OK;
    case SPEC_OPT_GUESS_TOKENS: *value = c->guess_opt; return SPEC_OK;
    case SPEC_OPT_TARGET_TAIL_LAYERS: *value = c->tail_layers; return SPEC_OK;   // what the next target forward uses
  }
  FAIL(SPEC_E_INVAL, "unknown option %d", option);
}

extern "C" int spec_set_profile(spec_ctx* c, int flags) {
  if (!c) FAIL(SPEC_E_INVAL, "null context");
  c->profile_flags = flags;
  return SPEC_OK;
}

extern "C" int spec_profile_read(spec_ctx* c, double* ms_total, long long* n_launches, double* bytes_total) {
  if (!c || !ms_total || !n_launches || !bytes_total) FAIL(SPEC_E_INVAL, "null argument");
  HIPCHK(hipStreamSynchronize(c->m[0].stream));
  ProfStamps& p = c->prof;
  double ms = 0.0;
  if (p.used) {
    std::vector<unsigned long long> host((size_t)2 * STAMP_WAYS * p.used);
    HIPCHK(hipMemcpy(host.data(), p.dev, host.size() * sizeof(unsigned long long), hipMemcpyDeviceToHost));
    for (size_t i = 0; i < p.used; ++i) {
      unsigned long long a = 0, b = 0;     // max of ~start = earliest start, max of end
      for (int k = 0; k < STAMP_WAYS; ++k) {
        const unsigned long long* s2 = &host[((size_t)i * STAMP_WAYS + k) * 2];
        if (s2[0] > a) a = s2[0];
        if (s2[1] > b) b = s2[1];
      }
      const unsigned long long t0 = ~a;
      if (a && b > t0) ms += (double)(b - t0) * p.tick_s * 1e3;
    }
    HIPCHK(hipMemset(p.dev, 0, host.size() * sizeof(unsigned long long)));
  }
  *ms_total = ms;
  *n_launches = (long long)p.used;
  *bytes_total = p.bytes;
  p.used = 0;
  p.bytes = 0.0;
  return SPEC_OK;
}
