// Launchers of the small kernels of the verify step (see step_kernels.hip).
#pragma once
#include "../../include/cerberus.h"
#include "common.h"

namespace cerb {

struct Dims {
  int n_layers, d, nH, dh, F, Fpad, V, Hc, R, sb, dtype, Bmax, cap, topk, T;
  int R64;  // rows allocated per activation plane
  float eps, threshold;
};

enum { ASSEMBLE_BY_FLAG = 0, ASSEMBLE_FORCE_AR = 1, ASSEMBLE_FULL_TREE = 2, ASSEMBLE_PROMPT = 3 };

// prompt pass: sequence `seq` runs `n` rows carrying tokens[0..n), every other sequence sits out
struct PromptArgs {
  const int* tokens;
  int n, seq;
};

struct ResFinishArgs {
  const float* part[CERBERUS_MAX_HEADS];   // GEMM partials of head i: [S][16][width]
  const float* bias[CERBERUS_MAX_HEADS];   // fp32 [width]
  size_t pstride[CERBERUS_MAX_HEADS];
  int S[CERBERUS_MAX_HEADS];
  int width[CERBERUS_MAX_HEADS];
};

enum { TOPK_MAX_PARTS = 16 };               // vocabulary slices of 4096 entries: up to 65536
struct TopkArgs {
  const float* logits[CERBERUS_MAX_HEADS];  // head i: [16][V]
  const int* seq_T;                         // [B] rows of each sequence this step (0: sat out)
  float* part_v;                            // [Hc][B][TOPK_MAX_PARTS][CERBERUS_MAX_TOPK] best entries of every slice, in order
  int* part_i;
};

hipError_t launch_assemble(const Dims& D, const TreeDev& tr, const RowMap& rm, const cerberus_state& st,
                           const cerberus_taps& tp, int batch, int mode, const PromptArgs& pa, const AttnPlanCfg& ap, hipStream_t s);
hipError_t launch_prompt_commit(const RowMap& rm, const cerberus_state& st, const int* g, int* last_row, int batch, int seq,
                                int last_pass, hipStream_t s);
// also fills rope_cs[row][j] = (cos, sin)(pos(row) * inv_freq[j]), j < dh/2, the angle formed in double
hipError_t launch_embed(const Dims& D, const RowMap& rm, const void* embed, float* x, const double* inv_freq, float2* rope_cs,
                        int rows_max, hipStream_t s);
hipError_t launch_add_rmsnorm(const Dims& D, const RowMap& rm, float* x, const float* part, int S, size_t pstride,
                              const float* gain, void* out, float* out_f32, float* tap, int rows_max, hipStream_t s);
// residual add + x * gain + per-block sums of x^2 (the RMSNorm scalar is applied by the consumer of the next GEMM)
int add_gain_blocks(int d);   // sums per row
// a_tiled: write the GEMM input in MFMA A-fragment order (64 rows, see FusedQkvArgs) instead of row-major planes
hipError_t launch_add_gain(const Dims& D, const RowMap& rm, float* x, const float* part, int S, size_t pstride,
                           const float* gain, void* out, float* ssq, int rows_max, hipStream_t s, bool a_tiled = false);
hipError_t launch_rope_kv(const Dims& D, const RowMap& rm, const float* part, int S, size_t pstride,
                          const float2* rope_cs, void* q, void* kv_layer, void* ktree, void* vtree, const float* ssq,
                          int rows_max, hipStream_t s);
// Whole-K GEMMs with fused epilogues (gemm_fused.hip), launches of up to 64 rows in bf16 mode.
// At: the GEMM input in MFMA A-fragment order, piece [((ks * 2 + plane) * 4 + mt) * 64 + lane] = the 8 values
// of row mt*16 + lane%16 at columns ks*32 + (lane/16)*8.., plane 0 = hi, 1 = lo (written by launch_add_gain
// with a_tiled).  slabs: [grid][ns] 16-column slabs of every workgroup, -1 = none; positions (2p, 2p+1) form a pair.
struct FusedQkvArgs {
  const void* W;            // [3d][K] in the stream order of this kernel's grid and slab table (launch_pack_stream)
  const void* At;
  const int* slabs;         // pairs: slabs i and i + dh/32 of a q or k head; or one or two v slabs
  int ksteps;               // padded K / 32
  const float* ssq;         // block sums of x^2 of the pending attention norm
  int nb;
  const float2* rope_cs;    // [rows][dh/2] (cos, sin) of every row's rotation angles (written by launch_embed)
  RowMap rm;
  bf16_t* q;                // [rows][d] hi, lo plane lo_off later
  bf16_t* kv_layer;         // [2][Bmax][nH][cap][dh]
  bf16_t* ktree;
  bf16_t* vtree;
  size_t lo_off;
  Dims D;
};
struct FusedGateUpArgs {
  const void* W;            // [2F][K] (gate rows first) in the stream order of this kernel's grid and slab table
  const void* At;
  const int* slabs;         // pairs: (gate slab s, up slab F/16 + s): the same 16 FFN columns
  int ksteps;
  const float* ssq;
  int nb, d;
  float eps;
  RowMap rm;
  bf16_t* act;              // [rows][Fpad] hi, lo plane lo_off later
  size_t lo_off;
  int Fpad;
};
hipError_t launch_qkv_rope(const FusedQkvArgs& a, int ns, int grid, hipStream_t s);
hipError_t launch_gate_up_swiglu(const FusedGateUpArgs& a, int ns, int grid, hipStream_t s);
size_t fused_stream_pieces(int ns, int grid, int ksteps);   // 16-byte pieces of a stream-order weight copy
hipError_t launch_pack_stream(const void* packed, void* dst, const int* table, int ns, int grid, int ksteps, hipStream_t s);
hipError_t launch_swiglu(const Dims& D, const RowMap& rm, const float* part, int S, size_t pstride, void* act,
                         const float* ssq, int rows_max, hipStream_t s);
hipError_t launch_row_argmax(const Dims& D, const RowMap& rm, const float* part, int S, size_t pstride, int* g,
                             const cerberus_taps& tp, int rows_max, hipStream_t s);
hipError_t launch_accept(const Dims& D, const TreeDev& tr, const RowMap& rm, const int* g, const int* tok,
                         const cerberus_state& st, int* path, int* last_row, int batch, hipStream_t s);
hipError_t launch_compact(const Dims& D, const RowMap& rm, const cerberus_state& st, const int* path, int batch,
                          hipStream_t s);
// entropy of `rows` vectors: vector r is forced[r] if forced != nullptr, else base[row_index ? row_index[r] : r];
// rows with seq_T[r] <= 0 (when seq_T != nullptr) are left untouched.
// Seeding of the decoding heads' stage-0 state by the gate launch; hsF == nullptr: none.
struct HeadsPrep {
  float* hsF;     // [Hc][16][2d] fp32 state
  void* hsA;      // same as the GEMM input type (bf16: lo plane lo_off elements later)
  size_t lo_off;
  int Hc, sb;     // number of heads; index of the special block
};
hipError_t launch_gate(int d, float threshold, const float* base, const int* row_index, const float* forced,
                       const int* seq_T, int rows, float* entropy, int* flag, const HeadsPrep& hp, int dtype, hipStream_t s);
hipError_t launch_resblock_finish(const Dims& D, const ResFinishArgs& a, const float* curF, float* nxtF, void* nxtA,
                                  int link_next, int batch, hipStream_t s);
hipError_t launch_topk(const Dims& D, const TopkArgs& a, const cerberus_state& st, const cerberus_taps& tp, int batch,
                       hipStream_t s);
hipError_t launch_log_tokens(const Dims& D, const cerberus_state& st, int batch, int* out, int cap, int* count,
                             hipStream_t s);
hipError_t launch_to_f32(const void* in, float* out, int n, int dtype, hipStream_t s);

}  // namespace cerb
