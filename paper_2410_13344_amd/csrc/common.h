// Shared declarations of the Cerberus verify-step kernels (gfx950 only).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace cerb {

typedef uint16_t bf16_t;  // raw bfloat16 bits

typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef float f32x4_t __attribute__((ext_vector_type(4)));
typedef unsigned u32x4_t __attribute__((ext_vector_type(4)));

__device__ __forceinline__ float bf16_to_f32(bf16_t v) { return __uint_as_float(((uint32_t)v) << 16); }

// round-to-nearest-even (v_cvt_pk_bf16_f32 on gfx950)
__device__ __forceinline__ bf16_t f32_to_bf16(float f) { return __builtin_bit_cast(bf16_t, static_cast<__bf16>(f)); }

// 16 bytes of a weight matrix that a launch streams through: loaded with the streaming hint, so that the lines
// leave the caches first and the activation fragments every workgroup re-reads stay.
__device__ __forceinline__ uint4 ld_weight_once(const uint4* p) {
  const u32x4_t t = __builtin_nontemporal_load(reinterpret_cast<const u32x4_t*>(p));
  return make_uint4(t[0], t[1], t[2], t[3]);
}

template <bool ONCE> __device__ __forceinline__ uint4 ld_w(const uint4* p) { return ONCE ? ld_weight_once(p) : *p; }

template <typename T> __device__ __forceinline__ float ld_f(const T* p);
template <> __device__ __forceinline__ float ld_f<float>(const float* p) { return *p; }
template <> __device__ __forceinline__ float ld_f<bf16_t>(const bf16_t* p) { return bf16_to_f32(*p); }
template <typename T> __device__ __forceinline__ void st_f(T* p, float v);
template <> __device__ __forceinline__ void st_f<float>(float* p, float v) { *p = v; }
template <> __device__ __forceinline__ void st_f<bf16_t>(bf16_t* p, float v) { *p = f32_to_bf16(v); }

// Store of a GEMM input.  In bf16 mode an activation v is kept as two bf16 planes `lo_off` elements
// apart, hi = bf16(v) and lo = bf16(v - hi): the GEMM multiplies both by the same weight fragment, so
// activations carry about 16 significant bits at no extra HBM traffic (the MFMA units idle most of
// the time in this weight-streaming regime).  bf16-rounded GEMM inputs alone put ~4e-2 rms error on
// the logits of a 32-layer random-init model.
template <typename T> __device__ __forceinline__ void st_a(T* p, size_t lo_off, float v);
template <> __device__ __forceinline__ void st_a<float>(float* p, size_t, float v) { *p = v; }
template <> __device__ __forceinline__ void st_a<bf16_t>(bf16_t* p, size_t lo_off, float v) {
  const bf16_t hi = f32_to_bf16(v);
  *p = hi;
  p[lo_off] = f32_to_bf16(v - bf16_to_f32(hi));
}

// four consecutive values of a GEMM input row; p (and the lo plane) aligned to the four elements
template <typename T> __device__ __forceinline__ void st_a4(T* p, size_t lo_off, const float (&v)[4]);
template <> __device__ __forceinline__ void st_a4<float>(float* p, size_t, const float (&v)[4]) {
  *reinterpret_cast<float4*>(p) = make_float4(v[0], v[1], v[2], v[3]);
}
template <> __device__ __forceinline__ void st_a4<bf16_t>(bf16_t* p, size_t lo_off, const float (&v)[4]) {
  union { bf16_t h[4]; uint2 u; } hi, lo;
#pragma unroll
  for (int e = 0; e < 4; ++e) {
    hi.h[e] = f32_to_bf16(v[e]);
    lo.h[e] = f32_to_bf16(v[e] - bf16_to_f32(hi.h[e]));
  }
  *reinterpret_cast<uint2*>(p) = hi.u;
  *reinterpret_cast<uint2*>(p + lo_off) = lo.u;
}

// ---------------------------------------------------------------------------------------------
// per-step row map: packed rows of all sequences (sequence b owns rows seq_row0[b] .. +seq_T[b])
// ---------------------------------------------------------------------------------------------
struct RowMap {
  int* n_rows;    // [1]
  int* seq_row0;  // [B]
  int* seq_T;     // [B] tree size used this step: T or 1
  int* seq_L;     // [B] kv_len at the start of the step
  int* row_seq;   // [Rmax]
  int* row_node;  // [Rmax]
  int* row_pos;   // [Rmax]
  int* row_tok;   // [Rmax]
  // work list of the MFMA attention kernel, written with the row map (null where no attention follows)
  int4* att_item; // [att_cap] x = (sequence << 16) | index j of the item within its sequence (first the sequence's
                  // cache-range items, then its tree chunks), y = kv_len, z = (rows of the sequence << 16) | its
                  // first row, w = (cache-range items of the sequence << 16) | chunks per cache-range item;
                  // x = -1 from the end of the list on
  int* seq_npi;   // [B] cache-range items of the sequence
};

struct AttnPlanCfg {
  int chunk;       // committed cache rows per chunk: cache-range items are cut in these units (0: no work list)
  int target_wgs;  // the work list aims at this many workgroups over all heads
  int att_cap;     // entries of the list
};

struct TreeDev {
  int T;
  const int* parent;            // [T]
  const int* rank;              // [T]
  const int* depth;             // [T]
  const unsigned long long* anc;  // [T][aw] bit m of the words of node n set: node m is n itself or an ancestor of n
  int aw;                         // 64-bit words per node, ceil(T / 64)
};

// ---------------------------------------------------------------------------------------------
// GEMM launch description: out[split][row][n] = sum_k A[row][k] * W[n][k] over the split's k range
// ---------------------------------------------------------------------------------------------
struct GemmProb {
  const void* A;  // [rows_alloc][lda], element type of the mode; bf16: the lo plane follows lo_off elements later
  size_t lo_off;
  const void* W;  // bf16 mode: MFMA-tile packed; f32 mode: row-major [N][K]
  float* out;     // [S][out_rows][N]
  int N, K;       // bf16 mode: K is the padded K (multiple of 32)
  int lda;
  int out_rows;
  int S;          // split-K factor
  int kps;        // k-steps (of 32) per split, a multiple of the kernel's LDS chunk (4 with both activation planes, 8 with one)
  int rem;        // the first `rem` splits take one LDS chunk more than kps (a split count that does not divide the chunks)
};

enum { GEMM_MAX_PROB = 8 };

struct GemmBatch {
  GemmProb p[GEMM_MAX_PROB];
  int n_prob;
  int tile0[GEMM_MAX_PROB + 1];  // first workgroup of every problem
  const int* n_rows;             // device row count, or nullptr -> rows_static
  int rows_static;
  const int* skip_flags;         // if non-null and all n_skip flags are non-zero: nothing to do
  int n_skip;
  int nsub;                      // bf16: 16-column slabs per wave (2 or 4); a workgroup covers 64*nsub columns
  int split;                     // bf16: 1 = multiply the hi and the lo activation plane, 0 = hi only
  int row_blocks;                // bf16: blocks of 64 rows in the launch (set by the launcher)
  int fixed_s1;                  // host side: the planner keeps split-K off (the consumer reads out[0] as the result)
  int wide_rows;                 // host side: launches of more than 256 rows take the 4-slab instance (down projection, LM head)
  int team_rows;                 // host side: launches of more than 128 rows go to the team kernel (gate/up projection)
};

// GEMM of one problem over more than 128 rows by teams of workgroups (gemm_team.hip)
struct TeamGemmArgs {
  const uint4* W;        // pre-tiled weights: piece (slab, k-step) at (slab * ksteps + ks) * 64 sixteen-byte pieces
  const bf16_t* A;       // [rows][lda] hi plane, the lo plane lo_off elements later
  size_t lo_off;
  int lda;
  float* out;            // [P][out_rows][N]
  int out_rows, N, ksteps;
  const int* n_rows;     // device row count, or nullptr -> rows_static
  int rows_static;
  int rows_cap;          // upper bound of the row count the plan was made for
  int rb_min;            // least number of row blocks (>= 2)
  int P;                 // partial planes the consumer sums (an upper bound of what any row count needs)
};
struct TeamPlan {
  int NT, planes, grid;    // row tiles per workgroup, partial planes, workgroups
  int rb_min;              // least number of row blocks the device may form
  int RB, rows_per, T;     // row blocks, rows per block and teams if the launch has as many rows as the plan allows
};
bool plan_team_gemm(int rows_max, int N, int Kpad, int cus, int max_planes, TeamPlan* tp);
hipError_t init_team_gemm();
hipError_t launch_team_gemm(const TeamGemmArgs& a, const TeamPlan& tp, hipStream_t s);

// launchers (defined next to their kernels)
hipError_t launch_gemm(const GemmBatch& g, int dtype, int rows_max, hipStream_t s);
hipError_t launch_pack_weight(const bf16_t* W, void* packed, int N, int K, int Kpad, hipStream_t s);
int gemm_cols_per_wg(int dtype, int nsub);

struct AttnArgs {
  const void* q;     // [rows][nH*dh]; bf16: lo plane q_lo_off elements later (0 in fp32 mode)
  size_t q_lo_off;
  const void* kv;    // layer base: [2][Bmax][nH][cap][dh]
  const void* ktree; // bf16 mode: this step's K rows as hi + lo planes [rows][nH*dh] (lo plane q_lo_off later);
  const void* vtree; //            the tree keys are read from here, the cache only serves rows < L
  void* out;         // [rows][nH*dh] attention output (GEMM A operand; bf16: lo plane out_lo_off elements later)
  size_t out_lo_off;
  float* part_o;     // [B][nH][n_chunks_max][Tpad][dh]; slot j of a (seq, head) belongs to the sequence's work item j
  float* part_ml;    // [B][nH][n_chunks_max][Tpad][2]
  RowMap rm;
  const unsigned long long* anc;   // [T][aw]
  int aw;            // mask words per node
  int Tpad;          // tree size rounded up to 64: query rows per partial slot
  int tc_max;        // tree chunks (64 of this step's rows each) at the end of the chunk grid, ceil(T / 64)
  int batch, Bmax, nH, dh, cap, T;
  int chunk;         // committed cache rows per chunk of the work list
  int n_chunks_max;
  int grid_x;        // workgroups along the item axis (the kernel strides over the list if it is longer)
  int att_cap;       // entries of the work list
  int rows_max;
  int* status;
};
hipError_t launch_attention(const AttnArgs& a, int dtype, int use_mfma, hipStream_t s);

}  // namespace cerb
