// Host side of the C ABI: validation, workspace layout, weight pre-tiling at init, and the launch
// sequence of one decoding step (Algorithm 1 of the Cerberus paper in streaming form: the gate and
// the heads run at the end of a forward pass and shape the next one).
#include <cmath>
#include <cstdarg>
#include <cstdio>
#include <cstring>
#include <new>
#include <string>
#include <vector>

#include "step_kernels.h"

using namespace cerb;

namespace {

thread_local char g_err[512] = "";

int fail(int code, const char* fmt, ...) {
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(g_err, sizeof g_err, fmt, ap);
  va_end(ap);
  return code;
}

#define HIP_TRY(expr)                                                                              \
  do {                                                                                             \
    hipError_t e_ = (expr);                                                                        \
    if (e_ != hipSuccess) return fail(CERBERUS_ERR_HIP, "%s: %s", #expr, hipGetErrorString(e_));   \
  } while (0)

inline size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }
inline int ceil_div(int a, int b) { return (a + b - 1) / b; }

struct Bump {
  unsigned char* base;
  size_t off;
  template <typename T>
  T* take(size_t n) {
    off = align_up(off, 256);
    T* p = reinterpret_cast<T*>(base + off);  // base may be null when only sizing
    off += n * sizeof(T);
    return p;
  }
};

}  // namespace

struct cerberus_ctx {
  cerberus_config cfg;
  Dims D;
  int device = 0;
  int elem = 2;  // bytes per stored element
  std::vector<int> parent, rank, depth;
  std::vector<unsigned long long> anc;
  TreeDev chain{};   // tables of a chain of T nodes (node i's parent is i-1): the causal mask of a prompt pass

  // device memory, all inside the workspace
  TreeDev tree{};
  RowMap rm{};
  double* inv_freq = nullptr;
  float2* rope_cs = nullptr;   // [rows][dh/2] (cos, sin) of this launch's row positions
  int *last_row = nullptr, *path = nullptr, *g = nullptr;
  float* topk_v = nullptr;   // per-slice candidate lists of the heads' top-k: [Hc][Bmax][TOPK_MAX_PARTS][CERBERUS_MAX_TOPK]
  int* topk_i = nullptr;
  float *x = nullptr, *h_last = nullptr, *part = nullptr, *attn_po = nullptr, *attn_ml = nullptr, *ssq = nullptr;
  void *xn = nullptr, *q = nullptr, *attn = nullptr, *act = nullptr, *ktree = nullptr, *vtree = nullptr;
  void* hsA[2] = {nullptr, nullptr};
  float* hsF[2] = {nullptr, nullptr};
  float* final_norm = nullptr;
  std::vector<float*> attn_norm, ffn_norm, res_b;
  std::vector<void*> pk_qkv, pk_o, pk_gu, pk_down, pk_res, pk_fc;
  std::vector<void*> st_qkv, st_gu;      // stream-order copies of the QKV and gate/up weights for the whole-K kernels
  void* pk_lm = nullptr;
  size_t small_bytes = 0;  // everything before the packed weights

  // weights as the kernels read them (packed copies in bf16 mode, the caller's in fp32 mode)
  const void* embed = nullptr;
  std::vector<const void*> wqkv, wo, wgu, wdown, res_w, head_fc;
  const void* lm_head = nullptr;

  size_t part_floats = 0;
  int n_chunks_max = 0, R64 = 0, prompt_rows = 0;
  cerberus_taps taps{};
  int use_mfma_attn = 1, target_wgs = 768, max_split = 8, gemm_nsub = 2, gemm_nsub_rows = 0, gemm_team = 3, act_split = 1, attn_chunk = 128, attn_target_wgs = 1024, uneven_split = 0, wg_slots = 512;
  std::vector<GemmBatch> p_qkv, p_o, p_gu, p_down, p_res;
  GemmBatch p_lm{}, p_fc{};

  // whole-K fused GEMMs (bf16 mode, launches of up to 64 rows): which slabs every workgroup owns
  int fused_grid = 0;                    // workgroups of a whole-K launch (0: not set up)
  int *slabs_qkv = nullptr, *slabs_gu = nullptr;   // device tables [kFusedMaxGrid][ns]
  int ns_qkv = 0, ns_gu = 0;             // positions per workgroup; 0 = that GEMM stays on the split-K path
  int use_fused = 1;
  void* workspace = nullptr;
  size_t workspace_bytes = 0;
};

namespace {

constexpr int kFusedMaxGrid = 512, kFusedMaxNs = 6;
constexpr int kFusedGrid = 256;          // one workgroup per compute unit of an MI355X; fixed, so that the workspace
                                         // (which holds weight copies laid out for this grid) can be sized without a device

// Scratch of cerberus_accept_noalloc (the acceptance entry point for callers that cannot pass or
// allocate a workspace): the row map, the accepted path and the last-row list, for up to
// kNoAllocBatch sequences and kNoAllocRows tree rows in all.  One copy of the array per GPU, held
// until the process ends; its address on a device is resolved once, at cerberus_init on that device.
constexpr int kNoAllocBatch = CERBERUS_MAX_BATCH;
constexpr int kNoAllocRows = 1024;
constexpr int kNoAllocPath = CERBERUS_MAX_HEADS + 1;
constexpr size_t kNoAllocScratchBytes = 32768;
static __device__ __align__(256) unsigned char scratch[kNoAllocScratchBytes];
constexpr int kMaxDevices = 64;
unsigned char* g_scratch_ptr[kMaxDevices] = {};

// with the context's device current
int resolve_static_scratch(int device) {
  if (device < 0 || device >= kMaxDevices) return fail(CERBERUS_ERR_ARG, "device index %d out of 0..%d", device, kMaxDevices - 1);
  if (g_scratch_ptr[device]) return CERBERUS_OK;
  void* p = nullptr;
  hipError_t e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
  if (e != hipSuccess || !p) return fail(CERBERUS_ERR_HIP, "hipGetSymbolAddress(scratch): %s", hipGetErrorString(e));
  g_scratch_ptr[device] = reinterpret_cast<unsigned char*>(p);
  return CERBERUS_OK;
}

int head_width(const cerberus_config& c, int i, int s) {
  return (i >= 1 && c.special_block >= 0 && s >= c.special_block) ? 2 * c.d_model : c.d_model;
}

int kpad(const cerberus_config& c, int K) { return c.dtype == CERBERUS_BF16 ? (int)align_up(K, 256) : K; }

int validate(const cerberus_config* c, const cerberus_tree* t) {
  if (!c || !t) return fail(CERBERUS_ERR_ARG, "null config or tree");
  if (c->dtype != CERBERUS_F32 && c->dtype != CERBERUS_BF16) return fail(CERBERUS_ERR_ARG, "dtype must be 0 (fp32) or 1 (bf16)");
  if (c->n_layers < 1 || c->d_model < 1 || c->n_heads < 1 || c->d_ffn < 1 || c->vocab < 1)
    return fail(CERBERUS_ERR_ARG, "non-positive model dimension");
  if (c->head_dim != 64 && c->head_dim != 128) return fail(CERBERUS_ERR_SHAPE, "head_dim must be 64 or 128");
  if (c->d_model != c->n_heads * c->head_dim) return fail(CERBERUS_ERR_SHAPE, "d_model != n_heads * head_dim");
  if (c->d_ffn % 8 || c->vocab % 16) return fail(CERBERUS_ERR_SHAPE, "d_ffn must be a multiple of 8 and vocab of 16");
  if (c->d_model > 8192 || c->vocab > 65536) return fail(CERBERUS_ERR_SHAPE, "d_model above 8192 or vocab above 65536");
  if (c->dtype == CERBERUS_BF16 && c->d_model % 256) return fail(CERBERUS_ERR_SHAPE, "bf16 mode needs d_model to be a multiple of 256");
  if (c->n_cerb_heads < 1 || c->n_cerb_heads > CERBERUS_MAX_HEADS) return fail(CERBERUS_ERR_SHAPE, "n_cerb_heads out of 1..%d", CERBERUS_MAX_HEADS);
  if (c->n_resblocks < 1 || c->n_resblocks > 16) return fail(CERBERUS_ERR_SHAPE, "n_resblocks out of 1..16");
  if (c->special_block >= c->n_resblocks) return fail(CERBERUS_ERR_SHAPE, "special_block >= n_resblocks");
  if (c->max_batch < 1 || c->max_batch > CERBERUS_MAX_BATCH) return fail(CERBERUS_ERR_SHAPE, "max_batch out of 1..%d", CERBERUS_MAX_BATCH);
  if (c->topk < 1 || c->topk > CERBERUS_MAX_TOPK || c->topk > c->vocab) return fail(CERBERUS_ERR_SHAPE, "topk out of 1..%d", CERBERUS_MAX_TOPK);
  if (c->kv_capacity < 1) return fail(CERBERUS_ERR_ARG, "kv_capacity < 1");
  if (!(c->rms_eps > 0.f) || !(c->rope_theta > 0.f)) return fail(CERBERUS_ERR_ARG, "rms_eps and rope_theta must be positive");
  if (std::isnan(c->entropy_threshold)) return fail(CERBERUS_ERR_ARG, "entropy_threshold is NaN");
  if (t->n_nodes < 1 || t->n_nodes > CERBERUS_MAX_TREE) return fail(CERBERUS_ERR_SHAPE, "tree size out of 1..%d", CERBERUS_MAX_TREE);
  if (t->n_nodes > c->kv_capacity) return fail(CERBERUS_ERR_SHAPE, "tree larger than kv_capacity");
  if (!t->parent || !t->rank) return fail(CERBERUS_ERR_ARG, "null tree arrays");
  if (t->parent[0] != -1) return fail(CERBERUS_ERR_SHAPE, "parent[0] must be -1");
  std::vector<int> depth(t->n_nodes, 0);
  for (int n = 1; n < t->n_nodes; ++n) {
    if (t->parent[n] < 0 || t->parent[n] >= n) return fail(CERBERUS_ERR_SHAPE, "parent[%d] must lie in 0..%d", n, n - 1);
    depth[n] = depth[t->parent[n]] + 1;
    if (depth[n] > c->n_cerb_heads) return fail(CERBERUS_ERR_SHAPE, "node %d is deeper than the number of heads", n);
    if (t->rank[n] < 0 || t->rank[n] >= c->topk) return fail(CERBERUS_ERR_SHAPE, "rank[%d] must lie in 0..topk-1", n);
  }
  return CERBERUS_OK;
}

void fill_dims(cerberus_ctx* c, const cerberus_config* cfg, const cerberus_tree* t) {
  c->cfg = *cfg;
  Dims& D = c->D;
  D.n_layers = cfg->n_layers; D.d = cfg->d_model; D.nH = cfg->n_heads; D.dh = cfg->head_dim; D.F = cfg->d_ffn;
  D.Fpad = kpad(*cfg, cfg->d_ffn); D.V = cfg->vocab; D.Hc = cfg->n_cerb_heads; D.R = cfg->n_resblocks;
  D.sb = cfg->special_block; D.dtype = cfg->dtype; D.Bmax = cfg->max_batch; D.cap = cfg->kv_capacity;
  D.topk = cfg->topk; D.T = t->n_nodes; D.eps = cfg->rms_eps; D.threshold = cfg->entropy_threshold;
  c->elem = cfg->dtype == CERBERUS_F32 ? 4 : 2;
  // A prompt pass is a chain of up to prompt_rows rows of one sequence, whatever the tree's size: room
  // for it in the row buffers, the row map and the attention partials.
  c->prompt_rows = CERBERUS_MAX_TREE;
  c->R64 = (int)align_up((size_t)std::max(cfg->max_batch * t->n_nodes, c->prompt_rows), 64);
  D.R64 = c->R64;
  c->n_chunks_max = ceil_div(cfg->kv_capacity, 128) + ceil_div(std::max(t->n_nodes, c->prompt_rows), 64);  // committed-row chunks + tree chunks
}

int fused_tables(const Dims& D, int grid, std::vector<int>& qkv, int& ns_qkv, std::vector<int>& gu, int& ns_gu);

// Assigns every workspace pointer of the context; with base == nullptr it only measures.
size_t layout(cerberus_ctx* c, unsigned char* base) {
  const Dims& D = c->D;
  const cerberus_config& cfg = c->cfg;
  Bump b{base, 0};
  const int T = D.T, B = D.Bmax, Rmax = std::max(B * T, c->prompt_rows), R64 = c->R64, d = D.d, el = c->elem;
  const int P = c->prompt_rows;
  c->tree.T = T;
  c->tree.parent = b.take<int>(T);
  c->tree.rank = b.take<int>(T);
  c->tree.depth = b.take<int>(T);
  c->tree.aw = ceil_div(T, 64);
  c->tree.anc = b.take<unsigned long long>((size_t)T * c->tree.aw);
  c->chain.T = P;
  c->chain.parent = c->tree.parent;   // not read in a prompt pass
  c->chain.rank = c->tree.rank;       // not read in a prompt pass
  c->chain.depth = b.take<int>(P);
  c->chain.aw = ceil_div(P, 64);
  c->chain.anc = b.take<unsigned long long>((size_t)P * c->chain.aw);
  c->inv_freq = b.take<double>(D.dh / 2);
  c->rope_cs = b.take<float2>((size_t)std::max(B * T, c->prompt_rows) * (D.dh / 2));
  c->rm.n_rows = b.take<int>(1);
  c->rm.seq_row0 = b.take<int>(B);
  c->rm.seq_T = b.take<int>(B);
  c->rm.seq_L = b.take<int>(B);
  c->rm.row_seq = b.take<int>(Rmax);
  c->rm.row_node = b.take<int>(Rmax);
  c->rm.row_pos = b.take<int>(Rmax);
  c->rm.row_tok = b.take<int>(Rmax);
  c->rm.att_item = b.take<int4>((size_t)B * c->n_chunks_max);
  c->rm.seq_npi = b.take<int>(B);
  c->last_row = b.take<int>(B);
  c->path = b.take<int>((size_t)B * (D.Hc + 1));
  c->topk_v = b.take<float>((size_t)D.Hc * B * TOPK_MAX_PARTS * CERBERUS_MAX_TOPK);
  c->topk_i = b.take<int>((size_t)D.Hc * B * TOPK_MAX_PARTS * CERBERUS_MAX_TOPK);
  c->g = b.take<int>(Rmax);
  c->x = b.take<float>((size_t)R64 * d);
  c->h_last = b.take<float>((size_t)R64 * d);
  c->ssq = b.take<float>((size_t)R64 * add_gain_blocks(d));
  const int planes = cfg.dtype == CERBERUS_BF16 ? 2 : 1;  // GEMM inputs: hi and lo plane in bf16 mode
  c->xn = b.take<unsigned char>((size_t)planes * R64 * d * el);
  c->q = b.take<unsigned char>((size_t)planes * R64 * d * el);
  c->attn = b.take<unsigned char>((size_t)planes * R64 * d * el);
  if (cfg.dtype == CERBERUS_BF16) {  // this step's K/V rows as hi + lo planes (the cache keeps one bf16)
    c->ktree = b.take<unsigned char>((size_t)2 * R64 * d * el);
    c->vtree = b.take<unsigned char>((size_t)2 * R64 * d * el);
  } else {
    c->ktree = c->vtree = nullptr;
  }
  c->act = b.take<unsigned char>((size_t)planes * R64 * D.Fpad * el);
  const size_t nmax = (size_t)std::max(std::max(3 * d, 2 * D.F), D.V);
  c->part_floats = 16 * std::max((size_t)R64 * nmax, (size_t)16 * D.Hc * std::max((size_t)2 * d, (size_t)D.V));
  c->part = b.take<float>(c->part_floats);
  const size_t slots = (size_t)B * D.nH * c->n_chunks_max * align_up((size_t)std::max(D.T, P), 64);
  c->attn_po = b.take<float>(slots * D.dh);
  c->attn_ml = b.take<float>(slots * 2);
  for (int i = 0; i < 2; ++i) {
    c->hsA[i] = b.take<unsigned char>((size_t)planes * D.Hc * 16 * 2 * d * el);
    c->hsF[i] = b.take<float>((size_t)D.Hc * 16 * 2 * d);
  }
  c->final_norm = b.take<float>(d);
  c->attn_norm.assign(D.n_layers, nullptr);
  c->ffn_norm.assign(D.n_layers, nullptr);
  for (int l = 0; l < D.n_layers; ++l) { c->attn_norm[l] = b.take<float>(d); c->ffn_norm[l] = b.take<float>(d); }
  c->res_b.assign((size_t)D.Hc * D.R, nullptr);
  for (int i = 0; i < D.Hc; ++i)
    for (int s = 0; s < D.R; ++s) c->res_b[i * D.R + s] = b.take<float>(head_width(cfg, i, s));
  if (cfg.dtype == CERBERUS_BF16) {
    c->slabs_qkv = b.take<int>((size_t)kFusedMaxGrid * kFusedMaxNs);
    c->slabs_gu = b.take<int>((size_t)kFusedMaxGrid * kFusedMaxNs);
  }
  c->small_bytes = align_up(b.off, 256);
  if (cfg.dtype == CERBERUS_BF16) {
    auto pk = [&](int N, int K) { return (void*)b.take<bf16_t>((size_t)N * kpad(cfg, K)); };
    c->pk_qkv.assign(D.n_layers, nullptr); c->pk_o.assign(D.n_layers, nullptr);
    c->pk_gu.assign(D.n_layers, nullptr); c->pk_down.assign(D.n_layers, nullptr);
    for (int l = 0; l < D.n_layers; ++l) {
      c->pk_qkv[l] = pk(3 * d, d); c->pk_o[l] = pk(d, d); c->pk_gu[l] = pk(2 * D.F, d); c->pk_down[l] = pk(d, D.F);
    }
    c->pk_lm = pk(D.V, d);
    {
      // whole-K kernels: slab tables for the fixed grid, and a copy of the QKV and gate/up weights in their stream order
      std::vector<int> tq, tg;
      fused_tables(D, kFusedGrid, tq, c->ns_qkv, tg, c->ns_gu);
      const int ksteps = kpad(cfg, d) / 32;
      c->st_qkv.assign(D.n_layers, nullptr); c->st_gu.assign(D.n_layers, nullptr);
      for (int l = 0; l < D.n_layers; ++l) {
        if (c->ns_qkv) c->st_qkv[l] = b.take<uint4>(fused_stream_pieces(c->ns_qkv, kFusedGrid, ksteps));
        if (c->ns_gu) c->st_gu[l] = b.take<uint4>(fused_stream_pieces(c->ns_gu, kFusedGrid, ksteps));
      }
    }
    c->pk_res.assign((size_t)D.Hc * D.R, nullptr);
    c->pk_fc.assign(D.Hc, nullptr);
    for (int i = 0; i < D.Hc; ++i) {
      for (int s = 0; s < D.R; ++s) { const int w = head_width(cfg, i, s); c->pk_res[i * D.R + s] = pk(w, w); }
      c->pk_fc[i] = pk(D.V, head_width(cfg, i, D.R - 1));
    }
  }
  return align_up(b.off, 256);
}

// Split-K choice: enough workgroups to cover the chip a few times over, whole LDS chunks of k per
// split.  A launch over more than 64 rows has a workgroup per 64-row block of every (column tile,
// split) and writes a partial of every row per split, so the split count goes down with the rows:
// the workgroup target is shared among the row blocks.
int choose_split(const cerberus_ctx* c, int total_tiles, int chunks, int rows_max) {
  const int cap = std::min(c->max_split, chunks);
  if (rows_max <= 64) {
    // resident workgroups: two per CU of the 32- and 64-row instances, three of the 16-row one
    const int slots = rows_max <= 16 ? c->wg_slots * 3 / 2 : c->wg_slots;
    // A launch that fits the chip in one round of resident workgroups (two 64-row workgroups per CU)
    // and fills at least 90 % of it beats one and a half rounds of shorter workgroups: it writes
    // fewer partials and has no half-empty second round (QKV at d = 4096: 480 workgroups with 5
    // splits, 29.5 us, against 768 with 8 splits, 31.1 us).  The ranges need not divide the chunks.
    const int one_round = slots / total_tiles;
    if (one_round >= 1 && one_round <= cap && total_tiles * one_round * 10 >= slots * 9) return one_round;
    int S = std::max(1, (c->target_wgs + total_tiles / 2) / total_tiles);
    S = std::min(S, cap);
    if (c->uneven_split) return S;
    // an uneven split leaves some workgroups with less to do and costs a whole extra partial: take
    // the next lower split that divides the chunks, if there is one nearby
    for (int s2 = S; s2 * 5 >= S * 3 && s2 >= 1; --s2)
      if (chunks % s2 == 0) return s2;
    return S;
  }
  // the split nearest (in ratio) to the ideal one; a split that does not divide the chunks pays for
  // the idle time of the workgroups with the short last range
  const double ideal = std::max(1.0, (double)c->target_wgs * 64.0 / ((double)total_tiles * rows_max));
  int best = 1;
  double best_cost = std::fabs(std::log(1.0 / ideal));
  for (int s2 = 2; s2 <= cap; ++s2) {
    const int cps = ceil_div(chunks, s2);
    const double imbalance = (double)cps * s2 / chunks - 1.0;
    const double cost = std::fabs(std::log((double)s2 / ideal)) + 3.0 * imbalance;
    if (cost < best_cost) { best = s2; best_cost = cost; }
  }
  return best;
}

// (Re)computes split, tile numbering and partial buffers of a plan for a launch of up to rows_max rows.
void split_plan(const cerberus_ctx* c, GemmBatch& g, int rows_max) {
  const int cols = gemm_cols_per_wg(c->cfg.dtype, g.nsub);
  int total_tiles = 0;
  for (int p = 0; p < g.n_prob; ++p) total_tiles += ceil_div(g.p[p].N, cols);
  float* out = c->part;
  int wg = 0;
  for (int p = 0; p < g.n_prob; ++p) {
    GemmProb& P = g.p[p];
    if (c->cfg.dtype == CERBERUS_F32) {
      P.S = 1; P.kps = 0; P.rem = 0;
    } else {
      // unit of a split: one LDS chunk of the kernel, 4 k-steps (128 columns of K) with both activation
      // planes, 8 with one (K is padded to 256, so either divides it)
      const int unit = g.split ? 4 : 8;
      const int chunks = P.K / (32 * unit);
      const int S = g.fixed_s1 ? 1 : choose_split(c, total_tiles, chunks, rows_max);
      P.S = S;                              // S <= chunks
      P.kps = (chunks / S) * unit;          // as even as whole chunks allow: the first chunks % S splits take one more
      P.rem = chunks % S;
    }
    P.out = out;
    out += (size_t)P.S * P.out_rows * P.N;
    g.tile0[p] = wg;
    wg += ceil_div(P.N, cols) * P.S;
  }
  g.tile0[g.n_prob] = wg;
}

void plan_gemm(const cerberus_ctx* c, GemmBatch& g, int nprob, const void* const* A, const int* lda, size_t lo_off,
               const void* const* W, const int* N, const int* K, int out_rows, bool force_s1) {
  std::memset(&g, 0, sizeof g);
  g.n_prob = nprob;
  g.nsub = c->gemm_nsub;
  g.split = c->act_split;
  g.fixed_s1 = force_s1 ? 1 : 0;
  for (int p = 0; p < nprob; ++p) {
    GemmProb& P = g.p[p];
    P.A = A[p]; P.lo_off = lo_off; P.W = W[p]; P.N = N[p]; P.lda = lda[p]; P.out_rows = out_rows;
    P.K = c->cfg.dtype == CERBERUS_F32 ? K[p] : kpad(c->cfg, K[p]);
  }
  split_plan(c, g, 64);
}

// Slab tables of the whole-K fused GEMMs for a grid of `grid` workgroups.  Positions (2p, 2p+1) of a
// workgroup hold what its epilogue needs together: slabs i and i + dh/32 of a q or k head (RoPE rotates column
// j with j + dh/2), one or two v slabs, or the gate and the up slab of 16 FFN columns.  Work is dealt so that
// the workgroups' slab counts differ by as little as the pairing allows.  Returns the positions per workgroup
// (0 if more than kFusedMaxNs would be needed).
int fused_tables(const Dims& D, int grid, std::vector<int>& qkv, int& ns_qkv, std::vector<int>& gu, int& ns_gu) {
  const int spd = D.d / 16, sph = D.dh / 16;
  std::vector<std::vector<int>> pos(grid);       // per workgroup: flat list of positions
  auto load = [&](int w) { int n = 0; for (int v : pos[w]) n += v >= 0; return n; };
  auto lightest = [&]() { int best = 0; for (int w = 1; w < grid; ++w) if (load(w) < load(best)) best = w; return best; };
  int w = 0;
  for (int sec = 0; sec < 2; ++sec)
    for (int h = 0; h < D.nH; ++h)
      for (int i = 0; i < sph / 2; ++i) {
        const int lo = sec * spd + h * sph + i;
        pos[w].push_back(lo); pos[w].push_back(lo + sph / 2);
        w = (w + 1) % grid;
      }
  for (int t = 0; t < spd; ++t) {
    const int sv = 2 * spd + t, best = lightest();
    std::vector<int>& P = pos[best];
    if (P.size() % 2 == 1) P.push_back(sv);      // joins the v slab that stood alone at the end
    else P.push_back(sv);                        // stands alone at the end (an odd number of positions) for now
  }
  // a list of odd length ends in a single v slab; lists are padded with -1 up to the common width
  size_t mx = 0;
  for (auto& P : pos) mx = std::max(mx, P.size());
  ns_qkv = mx <= (size_t)kFusedMaxNs ? (int)std::max<size_t>(mx, 2) : 0;
  qkv.assign((size_t)grid * std::max(ns_qkv, 1), -1);
  if (ns_qkv)
    for (int g = 0; g < grid; ++g) std::copy(pos[g].begin(), pos[g].end(), qkv.begin() + (size_t)g * ns_qkv);

  ns_gu = 0;
  gu.clear();
  if (D.F % 16 == 0) {
    const int fs = D.F / 16, per = ceil_div(fs, grid);
    if (2 * per <= kFusedMaxNs) {
      ns_gu = 2 * per;
      gu.assign((size_t)grid * ns_gu, -1);
      for (int s2 = 0; s2 < fs; ++s2) {
        const int g = s2 % grid, p = s2 / grid;
        gu[(size_t)g * ns_gu + 2 * p] = s2;
        gu[(size_t)g * ns_gu + 2 * p + 1] = fs + s2;
      }
    }
  }
  return ns_qkv;
}

void build_plans(cerberus_ctx* c) {
  const Dims& D = c->D;
  const int d = D.d, L = D.n_layers;
  c->p_qkv.resize(L); c->p_o.resize(L); c->p_gu.resize(L); c->p_down.resize(L);
  for (int l = 0; l < L; ++l) {
    { const void* A = c->xn; int lda = d, N = 3 * d, K = d; plan_gemm(c, c->p_qkv[l], 1, &A, &lda, (size_t)c->R64 * d, &c->wqkv[l], &N, &K, 64, false); c->p_qkv[l].team_rows = 2; }
    { const void* A = c->attn; int lda = d, N = d, K = d; plan_gemm(c, c->p_o[l], 1, &A, &lda, (size_t)c->R64 * d, &c->wo[l], &N, &K, 64, false); }
    { const void* A = c->xn; int lda = d, N = 2 * D.F, K = d; plan_gemm(c, c->p_gu[l], 1, &A, &lda, (size_t)c->R64 * d, &c->wgu[l], &N, &K, 64, false); c->p_gu[l].team_rows = 1; }
    { const void* A = c->act; int lda = D.Fpad, N = d, K = D.F; plan_gemm(c, c->p_down[l], 1, &A, &lda, (size_t)c->R64 * D.Fpad, &c->wdown[l], &N, &K, 64, false); c->p_down[l].wide_rows = 1; }
  }
  { const void* A = c->xn; int lda = d, N = D.V, K = d; plan_gemm(c, c->p_lm, 1, &A, &lda, (size_t)c->R64 * d, &c->lm_head, &N, &K, 64, false); c->p_lm.wide_rows = 1; c->p_lm.team_rows = 3; }
  c->p_res.resize(D.R);
  const void* A[CERBERUS_MAX_HEADS]; const void* W[CERBERUS_MAX_HEADS];
  int lda[CERBERUS_MAX_HEADS], N[CERBERUS_MAX_HEADS], K[CERBERUS_MAX_HEADS];
  for (int s = 0; s < D.R; ++s) {
    for (int i = 0; i < D.Hc; ++i) {
      A[i] = (const unsigned char*)c->hsA[s & 1] + (size_t)i * 16 * 2 * d * c->elem;
      W[i] = c->res_w[i * D.R + s];
      lda[i] = 2 * d;
      N[i] = K[i] = head_width(c->cfg, i, s);
    }
    plan_gemm(c, c->p_res[s], D.Hc, A, lda, (size_t)D.Hc * 16 * 2 * d, W, N, K, 16, false);
  }
  for (int i = 0; i < D.Hc; ++i) {
    A[i] = (const unsigned char*)c->hsA[D.R & 1] + (size_t)i * 16 * 2 * d * c->elem;
    W[i] = c->head_fc[i];
    lda[i] = 2 * d;
    N[i] = D.V;
    K[i] = head_width(c->cfg, i, D.R - 1);
  }
  plan_gemm(c, c->p_fc, D.Hc, A, lda, (size_t)D.Hc * 16 * 2 * d, W, N, K, 16, true);
}

int check_state(const cerberus_ctx* c, const cerberus_state* st, int batch) {
  if (!c || !st) return fail(CERBERUS_ERR_ARG, "null context or state");
  if (batch < 1 || batch > c->cfg.max_batch) return fail(CERBERUS_ERR_ARG, "batch %d out of 1..%d", batch, c->cfg.max_batch);
  if (!st->kv || !st->kv_len || !st->root_token || !st->cand || !st->gate_flag || !st->entropy || !st->accept_len ||
      !st->accepted_tokens || !st->accepted_nodes || !st->status)
    return fail(CERBERUS_ERR_ARG, "null pointer in cerberus_state");
  return CERBERUS_OK;
}

// Launches a planned GEMM over up to rows_max rows and returns the first problem as launched (its
// split count and partial buffer are what the consumer of the partials needs).
int run_gemm(const cerberus_ctx* c, const GemmBatch& plan, const int* n_rows, int rows_static, int rows_max,
             const int* skip_flags, int n_skip, hipStream_t s, GemmProb* launched = nullptr) {
  GemmBatch g = plan;
  // Above 128 rows the problems the planner marked (wide weights: gate/up, QKV, the LM head, in the order of what
  // they gain; the knob says how far down that list to go) run on the team kernel, which streams the weights once
  // per team of row blocks; its partial planes are the split of the launch.  Narrow weights (O, down) would need
  // more planes than the consumers sum and stay on the 64-row blocks (the plan refuses them).  QKV and the LM head
  // change over only past 256 rows: with two row blocks their extra planes cost what the kernel gains.
  TeamPlan tp;
  if (launched && plan.team_rows && c->gemm_team >= plan.team_rows && (plan.team_rows == 1 || rows_max > 256) && c->cfg.dtype == CERBERUS_BF16 && g.split && g.n_prob == 1 && !skip_flags &&
      c->fused_grid >= 8 && g.p[0].lda >= g.p[0].K &&   // (the kernel reads whole padded rows)
      plan_team_gemm(rows_max, g.p[0].N, g.p[0].K, c->fused_grid, c->max_split, &tp) &&
      (size_t)tp.planes * align_up((size_t)rows_max, 64) * g.p[0].N <= c->part_floats) {
    GemmProb& P = g.p[0];
    P.out_rows = (int)align_up((size_t)rows_max, 64);
    P.S = tp.planes; P.kps = 0; P.rem = 0;
    P.out = c->part;
    TeamGemmArgs ta{};
    ta.W = reinterpret_cast<const uint4*>(P.W); ta.A = reinterpret_cast<const bf16_t*>(P.A); ta.lo_off = P.lo_off; ta.lda = P.lda;
    ta.out = P.out; ta.out_rows = P.out_rows; ta.N = P.N; ta.ksteps = P.K / 32;
    ta.n_rows = n_rows; ta.rows_static = rows_static; ta.rows_cap = rows_max; ta.rb_min = tp.rb_min; ta.P = tp.planes;
    *launched = P;
    HIP_TRY(launch_team_gemm(ta, tp, s));
    return CERBERUS_OK;
  }
  // plans are made for 17..64 rows; other row counts run other kernel instances or several row
  // blocks and get their own split (only where the caller takes the launched description back)
  if (launched && (rows_max > 64 || rows_max <= 16)) {
    // several row blocks: 2 slabs per wave, or the 4-slab one-workgroup-per-CU instance.  Measured at the 7B
    // shapes: the 4-slab instance wins only past 256 rows and only where the planner marked the problem
    // (long K against few columns, or the vocabulary-wide LM head); the knob forces either one.
    if (rows_max > 64) g.nsub = c->gemm_nsub_rows ? c->gemm_nsub_rows : (rows_max > 256 && plan.wide_rows) ? 4 : 2;
    for (int p = 0; p < g.n_prob; ++p) g.p[p].out_rows = (int)align_up((size_t)rows_max, 64);   // partials packed for this launch
    split_plan(c, g, rows_max);
  }
  if (launched) *launched = g.p[0];
  g.n_rows = n_rows;
  g.rows_static = rows_static;
  g.skip_flags = skip_flags;
  g.n_skip = n_skip;
  HIP_TRY(launch_gemm(g, c->cfg.dtype, rows_max, s));
  return CERBERUS_OK;
}

#define TRY(expr)                     \
  do {                                \
    int rc_ = (expr);                 \
    if (rc_ != CERBERUS_OK) return rc_; \
  } while (0)

// whole-K fused launches of layer l over the rows of the current row map (kv_layer may be null: no cache write)
int run_fused_qkv(const cerberus_ctx* c, int l, void* kv_layer, hipStream_t s) {
  const Dims& D = c->D;
  FusedQkvArgs fa{};
  fa.W = c->st_qkv[l]; fa.At = c->xn; fa.slabs = c->slabs_qkv; fa.ksteps = kpad(c->cfg, D.d) / 32; fa.ssq = c->ssq;
  fa.nb = add_gain_blocks(D.d); fa.rope_cs = c->rope_cs; fa.rm = c->rm; fa.q = (bf16_t*)c->q; fa.kv_layer = (bf16_t*)kv_layer;
  fa.ktree = (bf16_t*)c->ktree; fa.vtree = (bf16_t*)c->vtree; fa.lo_off = (size_t)c->R64 * D.d; fa.D = D;
  HIP_TRY(launch_qkv_rope(fa, c->ns_qkv, c->fused_grid, s));
  return CERBERUS_OK;
}

int run_fused_gate_up(const cerberus_ctx* c, int l, hipStream_t s) {
  const Dims& D = c->D;
  FusedGateUpArgs ga{};
  ga.W = c->st_gu[l]; ga.At = c->xn; ga.slabs = c->slabs_gu; ga.ksteps = kpad(c->cfg, D.d) / 32; ga.ssq = c->ssq;
  ga.nb = add_gain_blocks(D.d); ga.d = D.d; ga.eps = D.eps; ga.rm = c->rm; ga.act = (bf16_t*)c->act;
  ga.lo_off = (size_t)c->R64 * D.Fpad; ga.Fpad = D.Fpad;
  HIP_TRY(launch_gate_up_swiglu(ga, c->ns_gu, c->fused_grid, s));
  return CERBERUS_OK;
}

// Embedding, the decoder layers and, with `head`, final norm + LM head + per-row argmax, over the
// rows the assembly kernel laid out; `tr` supplies the attention mask (candidate tree, or a chain).
int forward_rows(cerberus_ctx* c, const cerberus_state* st, int batch, int rows_max, const TreeDev& tr, bool head,
                 hipStream_t s) {
  const Dims& D = c->D;
  const RowMap& rm = c->rm;
  const size_t kv_layer_bytes = (size_t)2 * D.Bmax * D.nH * D.cap * D.dh * c->elem;
  HIP_TRY(launch_embed(D, rm, c->embed, c->x, c->inv_freq, c->rope_cs, rows_max, s));

  GemmProb pd{};                   // GEMM whose partials are the pending residual
  const GemmProb* prev = nullptr;
  // launches of up to 64 rows: QKV + RoPE + KV write and gate/up + SwiGLU as one whole-K launch each
  const bool fused = c->use_fused && D.dtype == CERBERUS_BF16 && rows_max <= 64 && c->fused_grid > 0 && c->act_split == 1;
  const bool fq = fused && c->ns_qkv > 0, fg = fused && c->ns_gu > 0;
  for (int l = 0; l < D.n_layers; ++l) {
    HIP_TRY(launch_add_gain(D, rm, c->x, prev ? prev->out : nullptr, prev ? prev->S : 0,
                            prev ? (size_t)prev->out_rows * prev->N : 0, c->attn_norm[l], c->xn, c->ssq, rows_max, s, fq));
    GemmProb pq, po, pg;
    void* kv_layer = (unsigned char*)st->kv + (size_t)l * kv_layer_bytes;
    if (fq) {
      TRY(run_fused_qkv(c, l, kv_layer, s));
    } else {
      TRY(run_gemm(c, c->p_qkv[l], rm.n_rows, 0, rows_max, nullptr, 0, s, &pq));
      HIP_TRY(launch_rope_kv(D, rm, pq.out, pq.S, (size_t)pq.out_rows * pq.N, c->rope_cs, c->q, kv_layer, c->ktree, c->vtree,
                             c->ssq, rows_max, s));
    }
    AttnArgs aa{};
    aa.q = c->q; aa.q_lo_off = D.dtype == CERBERUS_BF16 ? (size_t)c->R64 * D.d : 0; aa.kv = kv_layer; aa.ktree = c->ktree; aa.vtree = c->vtree; aa.out = c->attn; aa.out_lo_off = (size_t)c->R64 * D.d; aa.part_o = c->attn_po; aa.part_ml = c->attn_ml; aa.rm = rm;
    aa.anc = tr.anc; aa.aw = tr.aw; aa.Tpad = (int)align_up((size_t)tr.T, 64); aa.tc_max = ceil_div(tr.T, 64); aa.batch = batch; aa.Bmax = D.Bmax; aa.nH = D.nH; aa.dh = D.dh; aa.cap = D.cap; aa.T = tr.T;
    aa.chunk = c->attn_chunk; aa.n_chunks_max = ceil_div(D.cap, c->attn_chunk) + aa.tc_max;   // <= c->n_chunks_max, which sized the partial buffers
    // every item gets a workgroup per head: at most target / nH cache-range items plus one per sequence from
    // rounding, and the tree chunks
    aa.att_cap = D.Bmax * c->n_chunks_max;
    aa.grid_x = std::min(batch * aa.n_chunks_max, std::max(1, c->attn_target_wgs / D.nH) + batch * (1 + aa.tc_max));
    aa.rows_max = rows_max; aa.status = st->status;
    HIP_TRY(launch_attention(aa, D.dtype, c->use_mfma_attn, s));
    TRY(run_gemm(c, c->p_o[l], rm.n_rows, 0, rows_max, nullptr, 0, s, &po));
    HIP_TRY(launch_add_gain(D, rm, c->x, po.out, po.S, (size_t)po.out_rows * po.N, c->ffn_norm[l], c->xn, c->ssq, rows_max, s, fg));
    if (fg) {
      TRY(run_fused_gate_up(c, l, s));
    } else {
      TRY(run_gemm(c, c->p_gu[l], rm.n_rows, 0, rows_max, nullptr, 0, s, &pg));
      HIP_TRY(launch_swiglu(D, rm, pg.out, pg.S, (size_t)pg.out_rows * pg.N, c->act, c->ssq, rows_max, s));
    }
    TRY(run_gemm(c, c->p_down[l], rm.n_rows, 0, rows_max, nullptr, 0, s, &pd));
    prev = &pd;
  }
  if (!head) return CERBERUS_OK;
  HIP_TRY(launch_add_rmsnorm(D, rm, c->x, prev->out, prev->S, (size_t)prev->out_rows * prev->N, c->final_norm, c->xn,
                             c->h_last, c->taps.h_last, rows_max, s));
  GemmProb pl;
  TRY(run_gemm(c, c->p_lm, rm.n_rows, 0, rows_max, nullptr, 0, s, &pl));
  HIP_TRY(launch_row_argmax(D, rm, pl.out, pl.S, (size_t)pl.out_rows * pl.N, c->g, c->taps, rows_max, s));

  return CERBERUS_OK;
}

// the gate launch also writes the heads' stage-0 state (the gated row)
HeadsPrep heads_prep(const cerberus_ctx* c) {
  const Dims& D = c->D;
  return HeadsPrep{c->hsF[0], c->hsA[0], D.dtype == CERBERUS_BF16 ? (size_t)D.Hc * 16 * 2 * D.d : 0, D.Hc, D.sb};
}

// heads: skipped on the device when every sequence's gate chose the auto-regressive step
int run_heads(cerberus_ctx* c, const cerberus_state* st, int batch, hipStream_t s) {
  const Dims& D = c->D;
  const RowMap& rm = c->rm;
  for (int st_i = 0; st_i < D.R; ++st_i) {
    TRY(run_gemm(c, c->p_res[st_i], nullptr, batch, batch, st->gate_flag, batch, s));
    ResFinishArgs ra{};
    for (int i = 0; i < D.Hc; ++i) {
      const GemmProb& P = c->p_res[st_i].p[i];
      ra.part[i] = P.out; ra.S[i] = P.S; ra.pstride[i] = (size_t)P.out_rows * P.N; ra.width[i] = P.N;
      ra.bias[i] = c->res_b[i * D.R + st_i];
    }
    HIP_TRY(launch_resblock_finish(D, ra, c->hsF[st_i & 1], c->hsF[(st_i + 1) & 1], c->hsA[(st_i + 1) & 1],
                                   (st_i + 1 == D.sb) ? 1 : 0, batch, s));
  }
  TRY(run_gemm(c, c->p_fc, nullptr, batch, batch, st->gate_flag, batch, s));
  TopkArgs ta{};
  ta.seq_T = rm.seq_T;
  ta.part_v = c->topk_v;
  ta.part_i = c->topk_i;
  for (int i = 0; i < D.Hc; ++i) ta.logits[i] = c->p_fc.p[i].out;
  HIP_TRY(launch_topk(D, ta, *st, c->taps, batch, s));
  return CERBERUS_OK;
}

// the attention work list is built only for the MFMA kernel; the plain one walks rows and heads
AttnPlanCfg attn_plan_cfg(const cerberus_ctx* c) {
  const bool mfma = c->cfg.dtype == CERBERUS_BF16 && c->use_mfma_attn;
  return AttnPlanCfg{mfma ? c->attn_chunk : 0, c->attn_target_wgs, c->D.Bmax * c->n_chunks_max};
}

int run_step(cerberus_ctx* c, const cerberus_state* st, int batch, void* stream, int mode) {
  TRY(check_state(c, st, batch));
  hipStream_t s = reinterpret_cast<hipStream_t>(stream);
  const Dims& D = c->D;
  const RowMap& rm = c->rm;
  const int rows_max = (mode == ASSEMBLE_FORCE_AR) ? batch : batch * D.T;

  HIP_TRY(launch_assemble(D, c->tree, rm, *st, c->taps, batch, mode, PromptArgs{}, attn_plan_cfg(c), s));
  TRY(forward_rows(c, st, batch, rows_max, c->tree, true, s));

  HIP_TRY(launch_accept(D, c->tree, rm, c->g, rm.row_tok, *st, c->path, c->last_row, batch, s));
  if (mode != ASSEMBLE_FORCE_AR) HIP_TRY(launch_compact(D, rm, *st, c->path, batch, s));
  HIP_TRY(launch_gate(D.d, D.threshold, c->h_last, c->last_row, c->taps.forced_gate_hidden, rm.seq_T, batch, st->entropy,
                      st->gate_flag, heads_prep(c), D.dtype, s));
  return run_heads(c, st, batch, s);
}

// Prompt phase for one sequence: passes of up to prompt_rows rows, each a chain (causal mask, positions
// L, L+1, ...) whose K/V rows land where they stay.
int run_prompt(cerberus_ctx* c, const cerberus_state* st, int batch, int seq, const int* tokens, int n_tokens, hipStream_t s) {
  const Dims& D = c->D;
  const RowMap& rm = c->rm;
  // output taps see the prompt rows like any others; values forced for decoding steps do not apply here
  struct Restore {
    cerberus_taps& t; cerberus_taps saved;
    ~Restore() { t = saved; }
  } restore{c->taps, c->taps};
  c->taps.forced_node_argmax = nullptr;
  c->taps.forced_gate_hidden = nullptr;
  for (int off = 0; off < n_tokens; off += c->chain.T) {
    const int n = std::min(c->chain.T, n_tokens - off);
    const bool last = off + n >= n_tokens;
    HIP_TRY(launch_assemble(D, c->chain, rm, *st, c->taps, batch, ASSEMBLE_PROMPT, PromptArgs{tokens + off, n, seq}, attn_plan_cfg(c), s));
    TRY(forward_rows(c, st, batch, n, c->chain, last, s));
    HIP_TRY(launch_prompt_commit(rm, *st, c->g, c->last_row, batch, seq, last ? 1 : 0, s));
    if (last) {
      HIP_TRY(launch_gate(D.d, D.threshold, c->h_last, c->last_row, nullptr, rm.seq_T, batch, st->entropy, st->gate_flag,
                          heads_prep(c), D.dtype, s));
      TRY(run_heads(c, st, batch, s));
    }
  }
  return CERBERUS_OK;
}

}  // namespace

extern "C" {

const char* cerberus_last_error(void) { return g_err; }

size_t cerberus_workspace_bytes(const cerberus_config* cfg, const cerberus_tree* tree) {
  if (validate(cfg, tree) != CERBERUS_OK) return 0;
  cerberus_ctx tmp;
  fill_dims(&tmp, cfg, tree);
  return layout(&tmp, nullptr);
}

int cerberus_init(cerberus_ctx** out, const cerberus_config* cfg, const cerberus_weights* w, const cerberus_tree* tree,
                  void* workspace, size_t workspace_bytes) {
  if (!out) return fail(CERBERUS_ERR_ARG, "null out pointer");
  *out = nullptr;
  TRY(validate(cfg, tree));
  if (!w || !workspace) return fail(CERBERUS_ERR_ARG, "null weights or workspace");
  if (reinterpret_cast<uintptr_t>(workspace) % 256) return fail(CERBERUS_ERR_ARG, "workspace must be 256-byte aligned");
  if (!w->embed || !w->final_norm || !w->lm_head || !w->attn_norm || !w->wqkv || !w->wo || !w->ffn_norm || !w->w_gate_up ||
      !w->w_down || !w->res_w || !w->res_b || !w->head_fc)
    return fail(CERBERUS_ERR_ARG, "null pointer in cerberus_weights");
  for (int l = 0; l < cfg->n_layers; ++l)
    if (!w->attn_norm[l] || !w->wqkv[l] || !w->wo[l] || !w->ffn_norm[l] || !w->w_gate_up[l] || !w->w_down[l])
      return fail(CERBERUS_ERR_ARG, "null weight pointer in layer %d", l);
  for (int i = 0; i < cfg->n_cerb_heads; ++i) {
    if (!w->head_fc[i]) return fail(CERBERUS_ERR_ARG, "null head_fc[%d]", i);
    for (int s = 0; s < cfg->n_resblocks; ++s)
      if (!w->res_w[i * cfg->n_resblocks + s] || !w->res_b[i * cfg->n_resblocks + s])
        return fail(CERBERUS_ERR_ARG, "null Resblock weight of head %d block %d", i, s);
  }

  cerberus_ctx* c = new (std::nothrow) cerberus_ctx;
  if (!c) return fail(CERBERUS_ERR_ARG, "out of host memory");
  fill_dims(c, cfg, tree);
  const size_t need = layout(c, reinterpret_cast<unsigned char*>(workspace));
  if (workspace_bytes < need) {
    delete c;
    return fail(CERBERUS_ERR_CAPACITY, "workspace of %zu bytes, %zu needed", workspace_bytes, need);
  }
  c->workspace = workspace;
  c->workspace_bytes = workspace_bytes;
  const Dims& D = c->D;
  const int T = D.T, d = D.d;

  c->parent.assign(tree->parent, tree->parent + T);
  c->rank.assign(tree->rank, tree->rank + T);
  c->depth.assign(T, 0);
  const int aw = ceil_div(T, 64);
  c->anc.assign((size_t)T * aw, 0ull);
  for (int n = 0; n < T; ++n) {
    if (n > 0) {
      c->depth[n] = c->depth[c->parent[n]] + 1;
      for (int w = 0; w < aw; ++w) c->anc[(size_t)n * aw + w] = c->anc[(size_t)c->parent[n] * aw + w];
    }
    c->anc[(size_t)n * aw + (n >> 6)] |= 1ull << (n & 63);
  }
  std::vector<double> inv(D.dh / 2);
  for (int j = 0; j < D.dh / 2; ++j) inv[j] = std::pow((double)cfg->rope_theta, -2.0 * j / D.dh);

  auto cleanup = [&](int rc) { delete c; return rc; };
#define HIP_INIT(expr)                                                                                      \
  do {                                                                                                      \
    hipError_t e_ = (expr);                                                                                 \
    if (e_ != hipSuccess) return cleanup(fail(CERBERUS_ERR_HIP, "%s: %s", #expr, hipGetErrorString(e_)));   \
  } while (0)

  HIP_INIT(hipGetDevice(&c->device));
  { const int rc = resolve_static_scratch(c->device); if (rc != CERBERUS_OK) return cleanup(rc); }
  HIP_INIT(hipMemset(workspace, 0, c->small_bytes));
  HIP_INIT(hipMemcpy((void*)c->tree.parent, c->parent.data(), T * sizeof(int), hipMemcpyHostToDevice));
  HIP_INIT(hipMemcpy((void*)c->tree.rank, c->rank.data(), T * sizeof(int), hipMemcpyHostToDevice));
  HIP_INIT(hipMemcpy((void*)c->tree.depth, c->depth.data(), T * sizeof(int), hipMemcpyHostToDevice));
  HIP_INIT(hipMemcpy((void*)c->tree.anc, c->anc.data(), c->anc.size() * sizeof(unsigned long long), hipMemcpyHostToDevice));
  HIP_INIT(hipMemcpy(c->inv_freq, inv.data(), inv.size() * sizeof(double), hipMemcpyHostToDevice));
  {
    const int P = c->chain.T, caw = c->chain.aw;
    std::vector<int> cd(P);
    std::vector<unsigned long long> ca((size_t)P * caw, 0ull);
    for (int n = 0; n < P; ++n) {
      cd[n] = n;
      for (int m = 0; m <= n; ++m) ca[(size_t)n * caw + (m >> 6)] |= 1ull << (m & 63);
    }
    HIP_INIT(hipMemcpy((void*)c->chain.depth, cd.data(), P * sizeof(int), hipMemcpyHostToDevice));
    HIP_INIT(hipMemcpy((void*)c->chain.anc, ca.data(), ca.size() * sizeof(unsigned long long), hipMemcpyHostToDevice));
  }

  hipStream_t s0 = nullptr;
  HIP_INIT(launch_to_f32(w->final_norm, c->final_norm, d, D.dtype, s0));
  for (int l = 0; l < D.n_layers; ++l) {
    HIP_INIT(launch_to_f32(w->attn_norm[l], c->attn_norm[l], d, D.dtype, s0));
    HIP_INIT(launch_to_f32(w->ffn_norm[l], c->ffn_norm[l], d, D.dtype, s0));
  }
  for (int i = 0; i < D.Hc; ++i)
    for (int s = 0; s < D.R; ++s)
      HIP_INIT(launch_to_f32(w->res_b[i * D.R + s], c->res_b[i * D.R + s], head_width(*cfg, i, s), D.dtype, s0));

  c->embed = w->embed;
  c->wqkv.assign(D.n_layers, nullptr); c->wo.assign(D.n_layers, nullptr);
  c->wgu.assign(D.n_layers, nullptr); c->wdown.assign(D.n_layers, nullptr);
  c->res_w.assign((size_t)D.Hc * D.R, nullptr); c->head_fc.assign(D.Hc, nullptr);
  if (D.dtype == CERBERUS_F32) {
    for (int l = 0; l < D.n_layers; ++l) {
      c->wqkv[l] = w->wqkv[l]; c->wo[l] = w->wo[l]; c->wgu[l] = w->w_gate_up[l]; c->wdown[l] = w->w_down[l];
    }
    c->lm_head = w->lm_head;
    for (int i = 0; i < D.Hc; ++i) {
      for (int s = 0; s < D.R; ++s) c->res_w[i * D.R + s] = w->res_w[i * D.R + s];
      c->head_fc[i] = w->head_fc[i];
    }
  } else {
    auto pack = [&](const void* src, void* dst, int N, int K) {
      return launch_pack_weight(reinterpret_cast<const bf16_t*>(src), dst, N, K, kpad(*cfg, K), s0);
    };
    for (int l = 0; l < D.n_layers; ++l) {
      HIP_INIT(pack(w->wqkv[l], c->pk_qkv[l], 3 * d, d));
      HIP_INIT(pack(w->wo[l], c->pk_o[l], d, d));
      HIP_INIT(pack(w->w_gate_up[l], c->pk_gu[l], 2 * D.F, d));
      HIP_INIT(pack(w->w_down[l], c->pk_down[l], d, D.F));
      c->wqkv[l] = c->pk_qkv[l]; c->wo[l] = c->pk_o[l]; c->wgu[l] = c->pk_gu[l]; c->wdown[l] = c->pk_down[l];
    }
    HIP_INIT(pack(w->lm_head, c->pk_lm, D.V, d));
    c->lm_head = c->pk_lm;
    for (int i = 0; i < D.Hc; ++i) {
      for (int s = 0; s < D.R; ++s) {
        const int wd = head_width(*cfg, i, s);
        HIP_INIT(pack(w->res_w[i * D.R + s], c->pk_res[i * D.R + s], wd, wd));
        c->res_w[i * D.R + s] = c->pk_res[i * D.R + s];
      }
      HIP_INIT(pack(w->head_fc[i], c->pk_fc[i], D.V, head_width(*cfg, i, D.R - 1)));
      c->head_fc[i] = c->pk_fc[i];
    }
  }
  if (D.dtype == CERBERUS_BF16) {
    c->fused_grid = kFusedGrid;
    HIP_INIT(init_team_gemm());
    std::vector<int> tq, tg;
    fused_tables(D, c->fused_grid, tq, c->ns_qkv, tg, c->ns_gu);     // the same tables the workspace was laid out for
    if (c->ns_qkv) HIP_INIT(hipMemcpy(c->slabs_qkv, tq.data(), tq.size() * sizeof(int), hipMemcpyHostToDevice));
    if (c->ns_gu) HIP_INIT(hipMemcpy(c->slabs_gu, tg.data(), tg.size() * sizeof(int), hipMemcpyHostToDevice));
    const int ksteps = kpad(*cfg, d) / 32;
    for (int l = 0; l < D.n_layers; ++l) {
      if (c->ns_qkv) HIP_INIT(launch_pack_stream(c->pk_qkv[l], c->st_qkv[l], c->slabs_qkv, c->ns_qkv, c->fused_grid, ksteps, s0));
      if (c->ns_gu) HIP_INIT(launch_pack_stream(c->pk_gu[l], c->st_gu[l], c->slabs_gu, c->ns_gu, c->fused_grid, ksteps, s0));
    }
  }
  HIP_INIT(hipDeviceSynchronize());
#undef HIP_INIT
  build_plans(c);
  *out = c;
  return CERBERUS_OK;
}

int cerberus_verify_step(cerberus_ctx* ctx, const cerberus_state* st, int32_t batch, void* stream) {
  return run_step(ctx, st, batch, stream, ASSEMBLE_BY_FLAG);
}

int cerberus_ar_step(cerberus_ctx* ctx, const cerberus_state* st, int32_t batch, void* stream) {
  return run_step(ctx, st, batch, stream, ASSEMBLE_FORCE_AR);
}

int cerberus_prefill(cerberus_ctx* ctx, const cerberus_state* st, int32_t batch, int32_t seq, const int32_t* tokens,
                     int32_t n_tokens, void* stream) {
  TRY(check_state(ctx, st, batch));
  if (seq < 0 || seq >= batch) return fail(CERBERUS_ERR_ARG, "sequence index out of 0..batch-1");
  if (!tokens || n_tokens < 1) return fail(CERBERUS_ERR_ARG, "empty prompt");
  return run_prompt(ctx, st, batch, seq, tokens, n_tokens, reinterpret_cast<hipStream_t>(stream));
}

int cerberus_decode(cerberus_ctx* ctx, const cerberus_state* st, int32_t batch, int32_t n_steps, int32_t* out_tokens,
                    int32_t out_capacity, int32_t* out_count, void* stream) {
  TRY(check_state(ctx, st, batch));
  if (!out_tokens || !out_count) return fail(CERBERUS_ERR_ARG, "null token log");
  if (n_steps < 0 || out_capacity < 0) return fail(CERBERUS_ERR_ARG, "negative step count or log capacity");
  for (int i = 0; i < n_steps; ++i) {
    TRY(run_step(ctx, st, batch, stream, ASSEMBLE_BY_FLAG));
    HIP_TRY(launch_log_tokens(ctx->D, *st, batch, out_tokens, out_capacity, out_count, reinterpret_cast<hipStream_t>(stream)));
  }
  return CERBERUS_OK;
}

int cerberus_gate(cerberus_ctx* ctx, const float* hidden, int32_t rows, float* entropy_out, int32_t* flag_out, void* stream) {
  if (!ctx || !hidden || !entropy_out || !flag_out) return fail(CERBERUS_ERR_ARG, "null argument");
  if (rows < 0) return fail(CERBERUS_ERR_ARG, "rows < 0");
  if (rows == 0) return CERBERUS_OK;
  HIP_TRY(launch_gate(ctx->D.d, ctx->D.threshold, hidden, nullptr, nullptr, nullptr, rows, entropy_out, flag_out, HeadsPrep{}, ctx->D.dtype,
                      reinterpret_cast<hipStream_t>(stream)));
  return CERBERUS_OK;
}

int cerberus_accept(cerberus_ctx* ctx, const int32_t* node_argmax, const int32_t* node_token, const cerberus_state* st,
                    int32_t batch, void* stream) {
  TRY(check_state(ctx, st, batch));
  if (!node_argmax || !node_token) return fail(CERBERUS_ERR_ARG, "null node arrays");
  hipStream_t s = reinterpret_cast<hipStream_t>(stream);
  cerberus_taps none{};
  HIP_TRY(launch_assemble(ctx->D, ctx->tree, ctx->rm, *st, none, batch, ASSEMBLE_FULL_TREE, PromptArgs{}, AttnPlanCfg{0, 0, 0}, s));
  HIP_TRY(launch_accept(ctx->D, ctx->tree, ctx->rm, node_argmax, node_token, *st, ctx->path, ctx->last_row, batch, s));
  HIP_TRY(launch_compact(ctx->D, ctx->rm, *st, ctx->path, batch, s));
  return CERBERUS_OK;
}

int cerberus_accept_noalloc(cerberus_ctx* ctx, const int32_t* node_argmax, const int32_t* node_token, const cerberus_state* st,
                            int32_t batch, void* stream) {
  TRY(check_state(ctx, st, batch));
  if (!node_argmax || !node_token) return fail(CERBERUS_ERR_ARG, "null node arrays");
  const Dims& D = ctx->D;
  if (batch > kNoAllocBatch || batch * D.T > kNoAllocRows || D.Hc + 1 > kNoAllocPath)
    return fail(CERBERUS_ERR_CAPACITY, "cerberus_accept_noalloc takes up to %d sequences, %d tree rows in all and %d heads; got %d x %d rows, %d heads",
                kNoAllocBatch, kNoAllocRows, kNoAllocPath - 1, batch, D.T, D.Hc);
  if (ctx->device < 0 || ctx->device >= kMaxDevices || !g_scratch_ptr[ctx->device])
    return fail(CERBERUS_ERR_HIP, "the static scratch array of device %d was not resolved at cerberus_init", ctx->device);
  // carve the row map, the path and the last-row list out of this device's copy of the array
  Bump b{g_scratch_ptr[ctx->device], 0};
  RowMap rm{};
  rm.n_rows = b.take<int>(1);
  rm.seq_row0 = b.take<int>(kNoAllocBatch);
  rm.seq_T = b.take<int>(kNoAllocBatch);
  rm.seq_L = b.take<int>(kNoAllocBatch);
  rm.row_seq = b.take<int>(kNoAllocRows);
  rm.row_node = b.take<int>(kNoAllocRows);
  rm.row_pos = b.take<int>(kNoAllocRows);
  rm.row_tok = b.take<int>(kNoAllocRows);
  int* path = b.take<int>((size_t)kNoAllocBatch * kNoAllocPath);
  int* last_row = b.take<int>(kNoAllocBatch);
  if (b.off > kNoAllocScratchBytes) return fail(CERBERUS_ERR_CAPACITY, "static scratch layout exceeds the array");
  hipStream_t s = reinterpret_cast<hipStream_t>(stream);
  cerberus_taps none{};
  // every word the three kernels read from the array is written by an earlier one of them in this call
  // (the assembly writes the map of all `batch` sequences), so nothing has to start at zero
  HIP_TRY(launch_assemble(D, ctx->tree, rm, *st, none, batch, ASSEMBLE_FULL_TREE, PromptArgs{}, AttnPlanCfg{0, 0, 0}, s));
  HIP_TRY(launch_accept(D, ctx->tree, rm, node_argmax, node_token, *st, path, last_row, batch, s));
  HIP_TRY(launch_compact(D, rm, *st, path, batch, s));
  return CERBERUS_OK;
}

int cerberus_bench_gemm(cerberus_ctx* ctx, int32_t kind, int32_t rows, void* stream, double* bytes) {
  if (!ctx) return fail(CERBERUS_ERR_ARG, "null context");
  const Dims& D = ctx->D;
  if (kind >= 100 && kind <= 106) {   // query: would a step of this many rows run the kind as a whole-K fused launch?
    const bool f = ctx->use_fused && D.dtype == CERBERUS_BF16 && rows >= 1 && rows <= 64 && ctx->fused_grid > 0 && ctx->act_split == 1 &&
                   ((kind == 100 && ctx->ns_qkv) || (kind == 102 && ctx->ns_gu));
    TeamPlan tp;   // (2 + NT: the team kernel with NT row tiles per workgroup)
    const int level = kind == 102 ? 1 : kind == 100 ? 2 : kind == 104 ? 3 : 99, N = kind == 102 ? 2 * D.F : kind == 100 ? 3 * D.d : D.V;
    const bool team = ctx->gemm_team >= level && (level == 1 || rows > 256) && D.dtype == CERBERUS_BF16 && ctx->act_split == 1 && ctx->fused_grid >= 8 &&
                      plan_team_gemm(rows, N, kpad(ctx->cfg, D.d), ctx->fused_grid, ctx->max_split, &tp);
    if (bytes) *bytes = f ? 1.0 : team ? 2.0 + tp.NT : 0.0;
    return CERBERUS_OK;
  }
  const bool head_kind = kind == 5 || kind == 6;
  if (kind < 0 || kind > 6) return fail(CERBERUS_ERR_ARG, "kind out of 0..6");
  if (rows < 1 || rows > (head_kind ? D.Bmax : D.Bmax * D.T)) return fail(CERBERUS_ERR_ARG, "rows out of range");
  hipStream_t s = reinterpret_cast<hipStream_t>(stream);
  double total = 0.0;
  auto run = [&](const GemmBatch& g) -> int {
    for (int p = 0; p < g.n_prob; ++p)
      total += ((double)g.p[p].N * g.p[p].K + (double)rows * g.p[p].K * (g.split && ctx->elem == 2 ? 2 : 1)) * ctx->elem;
    GemmProb launched;   // layer and LM-head launches choose their split by row count, as in a step
    return run_gemm(ctx, g, nullptr, rows, rows, nullptr, 0, s, head_kind ? nullptr : &launched);
  };
  const bool fused = ctx->use_fused && D.dtype == CERBERUS_BF16 && rows <= 64 && ctx->fused_grid > 0 && ctx->act_split == 1;
  if (kind == 0 && fused && ctx->ns_qkv) {
    // what a step of this many rows launches for the QKV projection: the whole-K kernel with its RoPE
    // epilogue, over the rows of the last step's row map (which must hold `rows` rows), minus the cache write
    for (int l = 0; l < D.n_layers; ++l) TRY(run_fused_qkv(ctx, l, nullptr, s));
    total = (double)D.n_layers * ((double)3 * D.d * D.d + (double)rows * D.d * 2) * ctx->elem;
  } else if (kind == 2 && fused && ctx->ns_gu) {
    for (int l = 0; l < D.n_layers; ++l) TRY(run_fused_gate_up(ctx, l, s));
    total = (double)D.n_layers * ((double)2 * D.F * D.d + (double)rows * D.d * 2) * ctx->elem;
  } else if (kind <= 3) {
    const std::vector<GemmBatch>& v = kind == 0 ? ctx->p_qkv : kind == 1 ? ctx->p_o : kind == 2 ? ctx->p_gu : ctx->p_down;
    for (int l = 0; l < D.n_layers; ++l) TRY(run(v[l]));
  } else if (kind == 4) {
    TRY(run(ctx->p_lm));
  } else if (kind == 5) {
    for (int st_i = 0; st_i < D.R; ++st_i) TRY(run(ctx->p_res[st_i]));
  } else {
    TRY(run(ctx->p_fc));
  }
  if (bytes) *bytes = total;
  return CERBERUS_OK;
}

int cerberus_set_taps(cerberus_ctx* ctx, const cerberus_taps* taps) {
  if (!ctx) return fail(CERBERUS_ERR_ARG, "null context");
  if (taps) ctx->taps = *taps;
  else std::memset(&ctx->taps, 0, sizeof ctx->taps);
  return CERBERUS_OK;
}

int cerberus_set_param(cerberus_ctx* ctx, const char* name, int32_t value) {
  if (!ctx || !name) return fail(CERBERUS_ERR_ARG, "null argument");
  const std::string n(name);
  if (n == "attn_mfma") {
    if (value != 0 && value != 1) return fail(CERBERUS_ERR_ARG, "attn_mfma must be 0 or 1");
    ctx->use_mfma_attn = value;
  } else if (n == "attn_chunk") {
    if (value != 128 && value != 256) return fail(CERBERUS_ERR_ARG, "attn_chunk must be 128 or 256");
    ctx->attn_chunk = value;
  } else if (n == "gemm_wg_slots") {
    if (value < 0 || value > 65536) return fail(CERBERUS_ERR_ARG, "gemm_wg_slots out of 0..65536");
    ctx->wg_slots = value;
    build_plans(ctx);
  } else if (n == "gemm_uneven_split") {
    if (value != 0 && value != 1) return fail(CERBERUS_ERR_ARG, "gemm_uneven_split must be 0 or 1");
    ctx->uneven_split = value;
    build_plans(ctx);
  } else if (n == "gemm_target_wgs") {
    if (value < 1 || value > 65536) return fail(CERBERUS_ERR_ARG, "gemm_target_wgs out of 1..65536");
    ctx->target_wgs = value;
    build_plans(ctx);
  } else if (n == "gemm_nsub") {
    if (value != 2 && value != 4) return fail(CERBERUS_ERR_ARG, "gemm_nsub must be 2 or 4");
    ctx->gemm_nsub = value;
    build_plans(ctx);
  } else if (n == "attn_target_wgs") {
    if (value < 1 || value > 65536) return fail(CERBERUS_ERR_ARG, "attn_target_wgs out of 1..65536");
    ctx->attn_target_wgs = value;
  } else if (n == "gemm_team") {
    if (value < 0 || value > 3) return fail(CERBERUS_ERR_ARG, "gemm_team must be 0..3");
    ctx->gemm_team = value;
  } else if (n == "gemm_nsub_rows") {
    if (value != 0 && value != 2 && value != 4) return fail(CERBERUS_ERR_ARG, "gemm_nsub_rows must be 0, 2 or 4");
    ctx->gemm_nsub_rows = value;
  } else if (n == "act_split") {
    if (value != 0 && value != 1) return fail(CERBERUS_ERR_ARG, "act_split must be 0 or 1");
    ctx->act_split = value;
    build_plans(ctx);
  } else if (n == "gemm_fused") {
    if (value != 0 && value != 1) return fail(CERBERUS_ERR_ARG, "gemm_fused must be 0 or 1");
    ctx->use_fused = value;
  } else if (n == "gemm_max_split") {
    if (value < 1 || value > 16) return fail(CERBERUS_ERR_ARG, "gemm_max_split out of 1..16");
    ctx->max_split = value;
    build_plans(ctx);
  } else {
    return fail(CERBERUS_ERR_ARG, "unknown parameter '%s'", name);
  }
  return CERBERUS_OK;
}

void cerberus_destroy(cerberus_ctx* ctx) { delete ctx; }

}  // extern "C"
