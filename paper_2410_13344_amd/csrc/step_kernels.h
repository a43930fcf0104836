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
                           const cerberus_taps& tp, int batch, int mode, const PromptArgs& pa, hipStream_t s);
hipError_t launch_prompt_commit(const RowMap& rm, const cerberus_state& st, const int* g, int* last_row, int batch, int seq,
                                int last_pass, hipStream_t s);
hipError_t launch_embed(const Dims& D, const RowMap& rm, const void* embed, float* x, int rows_max, hipStream_t s);
hipError_t launch_add_rmsnorm(const Dims& D, const RowMap& rm, float* x, const float* part, int S, size_t pstride,
                              const float* gain, void* out, float* out_f32, float* tap, int rows_max, hipStream_t s);
// residual add + x * gain + per-block sums of x^2 (the RMSNorm scalar is applied by the consumer of the next GEMM)
int add_gain_blocks(int d);   // sums per row
hipError_t launch_add_gain(const Dims& D, const RowMap& rm, float* x, const float* part, int S, size_t pstride,
                           const float* gain, void* out, float* ssq, int rows_max, hipStream_t s);
hipError_t launch_rope_kv(const Dims& D, const RowMap& rm, const float* part, int S, size_t pstride,
                          const double* inv_freq, void* q, void* kv_layer, void* ktree, void* vtree, const float* ssq,
                          int rows_max, hipStream_t s);
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
