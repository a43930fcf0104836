// Skinny GEMMs of the verify step: out[row][n] = sum_k A[row][k] * W[n][k] for 1..64 tree-token
// rows (per row block) against weight matrices that are read exactly once per step.  The work is
// weight streaming: every wave pulls its own 16-column slab of the pre-tiled weights straight from
// HBM into registers in 1 KB fully coalesced loads, several loads in flight, while the few
// activation rows are staged through LDS and shared by the four waves of the workgroup.
#include "common.h"

namespace cerb {

// ---------------------------------------------------------------------------------------------
// Weight pre-tiling (init time).  Packed layout, in 16-byte pieces:
//   piece[(sub * ksteps + ks) * 64 + lane] = W[sub*16 + lane%16][ks*32 + (lane/16)*8 .. +8]
// i.e. one 1 KB block per (16 output columns, 32 k) holds exactly the B operand of one
// v_mfma_f32_16x16x32_bf16, lane by lane; consecutive k-steps of a column slab are contiguous.
// Columns k >= K (padding up to Kpad) are zero.
// ---------------------------------------------------------------------------------------------
__global__ void k_pack_weight(const bf16_t* __restrict__ W, uint4* __restrict__ out, int N, int K, int Kpad) {
  const int ksteps = Kpad / 32;
  const size_t total = (size_t)(N / 16) * ksteps * 64;
  for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < total; i += (size_t)gridDim.x * blockDim.x) {
    const int lane = (int)(i % 64);
    const size_t blk = i / 64;
    const int ks = (int)(blk % ksteps);
    const int sub = (int)(blk / ksteps);
    const int n = sub * 16 + (lane % 16);
    const int k = ks * 32 + (lane / 16) * 8;
    uint4 v = make_uint4(0, 0, 0, 0);
    if (k < K) v = *reinterpret_cast<const uint4*>(W + (size_t)n * K + k);  // K % 8 == 0
    out[i] = v;
  }
}

hipError_t launch_pack_weight(const bf16_t* W, void* packed, int N, int K, int Kpad, hipStream_t s) {
  const size_t total = (size_t)(N / 16) * (Kpad / 32) * 64;
  int blocks = (int)((total + 255) / 256);
  if (blocks > 65535) blocks = 65535;
  hipLaunchKernelGGL(k_pack_weight, dim3(blocks), dim3(256), 0, s, W, reinterpret_cast<uint4*>(packed), N, K, Kpad);
  return hipGetLastError();
}

// ---------------------------------------------------------------------------------------------
// bf16 MFMA GEMM.  Workgroup = 4 waves; wave w owns NSUB adjacent 16-column slabs; a workgroup
// covers 64*NSUB columns, MT*16 rows and one split of K.  A is staged through a double-buffered LDS
// tile of 512-byte rows: 8 k-steps of one plane, or with SPLIT 4 k-steps of the hi plane followed by
// the same 4 k-steps of the lo plane.  16-byte pieces are XOR-swizzled by the row index so the 16
// lanes of an MFMA row group hit 64 distinct banks.  The main loop has no branches, so the weight
// loads stay in flight across chunk boundaries.
// ---------------------------------------------------------------------------------------------
constexpr int kLdsRow = 512;
#ifndef CERB_ROWS_RING
#define CERB_ROWS_RING 8
#endif
#ifndef CERB_KRING
#define CERB_KRING 8
#endif
constexpr int kRingSplit = CERB_KRING;  // k-steps of weights in flight per wave (half as many in the one-plane instances:
                                         // their 8-k-step chunks need the registers, else the 64-row one spills)

__device__ __forceinline__ bool gemm_skip(const GemmBatch& g) {
  if (g.skip_flags == nullptr) return false;
  bool all = true;
  for (int i = 0; i < g.n_skip; ++i) all = all && (g.skip_flags[i] != 0);
  return all;
}

// ONCE: the launch has a single row block, every weight byte is read by exactly one workgroup: streaming loads.
// (With several row blocks the repeats are meant to hit in L2, and the streaming hint costs 10-20 %.)
template <int MT, int NSUB, int SPLIT, bool ONCE>
__device__ __forceinline__ void gemm_bf16_body(const GemmBatch& g) {
  if (gemm_skip(g)) return;
  const int rows = g.n_rows ? *g.n_rows : g.rows_static;
  // One-dimensional grid, numbered so that the row blocks of one (column tile, split) have ids 8
  // apart: consecutive workgroup ids go to the 8 XCDs in turn, so those workgroups land on one XCD
  // at about the same time and the weight tile comes from HBM once and from that XCD's L2 afterwards.
  // (Should the hardware map ids differently, only the reuse is lost.)  With one row block the
  // numbering is the identity.
  const int RB = g.row_blocks;
  const int grp = (int)blockIdx.x / (8 * RB), within = (int)blockIdx.x - grp * 8 * RB;
  const int tile_id = grp * 8 + (within & 7);
  const int m0 = (within >> 3) * (MT * 16);
  if (tile_id >= g.tile0[g.n_prob] || m0 >= rows) return;

  int pi = 0;
  while (pi + 1 < g.n_prob && tile_id >= g.tile0[pi + 1]) ++pi;
  const GemmProb P = g.p[pi];
  const int local = tile_id - g.tile0[pi];
  const int split = local % P.S;
  const int ntile = local / P.S;
  constexpr int KSC = SPLIT ? 4 : 8;         // k-steps per LDS chunk
  constexpr int kRing = (MT == 4 && NSUB == 4) ? CERB_ROWS_RING : SPLIT ? kRingSplit : kRingSplit / 2;
  static_assert((2 * KSC) % kRing == 0 && (kRing % KSC == 0 || KSC % kRing == 0),
                "ring slots must be compile-time constants: k-step (chunk parity * KSC + s) lives in slot of that index mod kRing");
  const int ksteps = P.K / 32;               // K is a multiple of 256
  const int ks0 = split * P.kps + min(split, P.rem) * KSC;   // kps is a multiple of KSC
  const int ks1 = min(ks0 + P.kps + (split < P.rem ? KSC : 0), ksteps);
  const int nchunks = (ks1 - ks0) / KSC;
  if (nchunks <= 0) return;                  // uniform over the workgroup

  const int wave = threadIdx.x >> 6;
  const int lane = threadIdx.x & 63;
  const int nsub_total = P.N / 16;

  constexpr int kBuf = MT * 16 * kLdsRow;
  __shared__ __attribute__((aligned(16))) unsigned char lds[2 * kBuf];

  const uint4* wp[NSUB];
  int sub[NSUB];
#pragma unroll
  for (int j = 0; j < NSUB; ++j) {
    sub[j] = (ntile * 4 + wave) * NSUB + j;
    const int sc = min(sub[j], nsub_total - 1);  // clamp: out-of-range slabs load valid memory, store nothing
    wp[j] = reinterpret_cast<const uint4*>(P.W) + (size_t)sc * ksteps * 64 + lane;
  }

  // row tiles that hold rows at all (uniform): a launch sized for whole trees may carry a single row
  const int mt_n = min(MT, (rows - m0 + 15) / 16);
  const int a_n = 2 * mt_n;                  // staging passes that touch live rows (a pass covers 8 rows)
  f32x4_t acc[MT][NSUB];
#pragma unroll
  for (int mt = 0; mt < MT; ++mt)
#pragma unroll
    for (int j = 0; j < NSUB; ++j) acc[mt][j] = f32x4_t{0.f, 0.f, 0.f, 0.f};

  // Activation chunks travel global -> registers -> LDS two chunks ahead of their use: the loads of
  // chunk c+2 are issued before chunk c is multiplied and are written to LDS after chunk c+1's
  // buffer has been freed, so an L2 round trip (about three chunks of MFMA time) is covered.
  // Thread t owns 16-byte piece t%32 of rows t/32 + 8i.  The staging registers are named scalars
  // (P0..7 / Q0..7) on purpose: arrays that live across the loop back-edge, or are touched through
  // a lambda, end up in scratch memory, and a scratch round trip inside the loop serialises the
  // whole in-order load queue.
  constexpr int kApt = MT * 2;  // pieces per thread per chunk
  const int a_r0 = threadIdx.x >> 5, a_pc = threadIdx.x & 31;
  const bf16_t* a_src = reinterpret_cast<const bf16_t*>(P.A) + (size_t)(m0 + a_r0) * P.lda + (size_t)ks0 * 32 +
                        (SPLIT ? (size_t)(a_pc >> 4) * P.lo_off + (a_pc & 15) * 8 : (size_t)a_pc * 8);
  const size_t a_step = (size_t)8 * P.lda;                 // row r0 + 8i
  const int a_q = a_pc ^ (a_r0 & 15);                      // (r0 + 8i) & 15 flips bit 3 for odd i
  const int a_dst_e = a_r0 * kLdsRow + a_q * 16, a_dst_o = a_r0 * kLdsRow + (a_q ^ 8) * 16;

#define CERB_A_LD(X, CH, FULL)                                                                                      \
  {                                                                                                           \
    const bf16_t* sp = a_src + (size_t)(CH) * (KSC * 32);                                                     \
    if (kApt > 0 && (FULL || 0 < a_n)) X##0 = *reinterpret_cast<const uint4*>(sp);                                                 \
    if (kApt > 1 && (FULL || 1 < a_n)) X##1 = *reinterpret_cast<const uint4*>(sp + a_step);                                        \
    if (kApt > 2 && (FULL || 2 < a_n)) X##2 = *reinterpret_cast<const uint4*>(sp + 2 * a_step);                                    \
    if (kApt > 3 && (FULL || 3 < a_n)) X##3 = *reinterpret_cast<const uint4*>(sp + 3 * a_step);                                    \
    if (kApt > 4 && (FULL || 4 < a_n)) X##4 = *reinterpret_cast<const uint4*>(sp + 4 * a_step);                                    \
    if (kApt > 5 && (FULL || 5 < a_n)) X##5 = *reinterpret_cast<const uint4*>(sp + 5 * a_step);                                    \
    if (kApt > 6 && (FULL || 6 < a_n)) X##6 = *reinterpret_cast<const uint4*>(sp + 6 * a_step);                                    \
    if (kApt > 7 && (FULL || 7 < a_n)) X##7 = *reinterpret_cast<const uint4*>(sp + 7 * a_step);                                    \
  }
#define CERB_A_ST(X, BUF, FULL)                                                                                     \
  {                                                                                                           \
    unsigned char* dp = lds + (BUF) * kBuf;                                                                   \
    if (kApt > 0 && (FULL || 0 < a_n)) *reinterpret_cast<uint4*>(dp + a_dst_e) = X##0;                                             \
    if (kApt > 1 && (FULL || 1 < a_n)) *reinterpret_cast<uint4*>(dp + a_dst_o + 8 * kLdsRow) = X##1;                               \
    if (kApt > 2 && (FULL || 2 < a_n)) *reinterpret_cast<uint4*>(dp + a_dst_e + 16 * kLdsRow) = X##2;                              \
    if (kApt > 3 && (FULL || 3 < a_n)) *reinterpret_cast<uint4*>(dp + a_dst_o + 24 * kLdsRow) = X##3;                              \
    if (kApt > 4 && (FULL || 4 < a_n)) *reinterpret_cast<uint4*>(dp + a_dst_e + 32 * kLdsRow) = X##4;                              \
    if (kApt > 5 && (FULL || 5 < a_n)) *reinterpret_cast<uint4*>(dp + a_dst_o + 40 * kLdsRow) = X##5;                              \
    if (kApt > 6 && (FULL || 6 < a_n)) *reinterpret_cast<uint4*>(dp + a_dst_e + 48 * kLdsRow) = X##6;                              \
    if (kApt > 7 && (FULL || 7 < a_n)) *reinterpret_cast<uint4*>(dp + a_dst_o + 56 * kLdsRow) = X##7;                              \
  }

  uint4 P0, P1, P2, P3, P4, P5, P6, P7, Q0, Q1, Q2, Q3, Q4, Q5, Q6, Q7;
  P0 = P1 = P2 = P3 = P4 = P5 = P6 = P7 = Q0 = Q1 = Q2 = Q3 = Q4 = Q5 = Q6 = Q7 = make_uint4(0, 0, 0, 0);
  CERB_A_LD(P, 0, 0)
  uint4 ring[kRing][NSUB];
#pragma unroll
  for (int i = 0; i < kRing; ++i)     // slot kRing - 1 is filled by the first k-step of the loop (its load below is not waited for)
#pragma unroll
    for (int j = 0; j < NSUB; ++j) ring[i][j] = ld_w<ONCE>(wp[j] + (size_t)min(ks0 + min(i, kRing - 2), ks1 - 1) * 64);
  CERB_A_ST(P, 0, 0)
  CERB_A_LD(P, min(1, nchunks - 1), 0)
  __syncthreads();

  const int a_row = lane & 15, a_grp = lane >> 4;  // (mt*16 + a_row) & 15 == a_row

#define CERB_GEMM_CHUNK(C, PAR, NEXT2, NEXT1, FULL)                                                                                \
  {                                                                                                                       \
    CERB_A_LD(NEXT2, min((C) + 2, nchunks - 1), FULL)                                                                           \
    __builtin_amdgcn_sched_barrier(0);                                                                                    \
    const unsigned char* L = lds + ((C) & 1) * kBuf + a_row * kLdsRow;                                                    \
    const int kb = ks0 + (C) * KSC;                                                                                       \
    _Pragma("unroll") for (int s = 0; s < KSC; ++s) {                                                                     \
      /* The slot multiplied in the previous k-step takes the load for kRing - 1 k-steps ahead; this k-step's slot */       \
      /* is read in place.  (Refilling the slot being read needs a copy of it first, and the copies of a whole     */       \
      /* chunk get hoisted to its top, where they wait for every load in flight.)  The scheduling barrier keeps   */       \
      /* the load here instead of wherever the scheduler would sink it.                                           */       \
      _Pragma("unroll") for (int j = 0; j < NSUB; ++j)                                                                    \
        ring[((PAR) * KSC + s + kRing - 1) % kRing][j] = ld_w<ONCE>(wp[j] + (size_t)min(kb + s + kRing - 1, ks1 - 1) * 64);   \
      __builtin_amdgcn_sched_barrier(0);                                                                                  \
      const uint4* b = ring[((PAR) * KSC + s) % kRing];                                                                   \
      _Pragma("unroll") for (int mt = 0; mt < MT; ++mt) if (FULL || mt < mt_n) {                                                  \
        const uint4 a = *reinterpret_cast<const uint4*>(L + mt * 16 * kLdsRow + (((s * 4 + a_grp) ^ a_row) * 16));        \
        _Pragma("unroll") for (int j = 0; j < NSUB; ++j) acc[mt][j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(            \
            __builtin_bit_cast(bf16x8_t, a), __builtin_bit_cast(bf16x8_t, b[j]), acc[mt][j], 0, 0, 0);                    \
        if (SPLIT) {                                                                                                      \
          const uint4 al =                                                                                                \
              *reinterpret_cast<const uint4*>(L + mt * 16 * kLdsRow + (((16 + s * 4 + a_grp) ^ a_row) * 16));             \
          _Pragma("unroll") for (int j = 0; j < NSUB; ++j) acc[mt][j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(          \
              __builtin_bit_cast(bf16x8_t, al), __builtin_bit_cast(bf16x8_t, b[j]), acc[mt][j], 0, 0, 0);                 \
        }                                                                                                                 \
      }                                                                                                                   \
    }                                                                                                                     \
    CERB_A_ST(NEXT1, ((C) + 1) & 1, FULL)                                                                                       \
    __syncthreads();                                                                                                      \
  }

  // Two copies of the loop: the usual one for a full tile, without a single branch in it, and one
  // that skips the staging and the MFMAs of row tiles without rows (a launch sized for whole trees
  // when every sequence took the one-token step).
  if (MT == 1 || mt_n == MT) {
    for (int c = 0; c < nchunks; c += 2) {
      CERB_GEMM_CHUNK(c, 0, Q, P, 1)            // P holds chunk c+1, Q receives chunk c+2
      if (c + 1 >= nchunks) break;              // uniform over the workgroup
      CERB_GEMM_CHUNK(c + 1, 1, P, Q, 1)        // Q holds chunk c+2, P receives chunk c+3
    }
  } else {
    for (int c = 0; c < nchunks; c += 2) {
      CERB_GEMM_CHUNK(c, 0, Q, P, 0)
      if (c + 1 >= nchunks) break;
      CERB_GEMM_CHUNK(c + 1, 1, P, Q, 0)
    }
  }
#undef CERB_GEMM_CHUNK
#undef CERB_A_LD
#undef CERB_A_ST

  // D layout: lane holds column lane%16, rows 4*(lane/16) + v
  float* out = P.out + (size_t)split * P.out_rows * P.N;
#pragma unroll
  for (int j = 0; j < NSUB; ++j) {
    if (sub[j] >= nsub_total) continue;
    const int col = sub[j] * 16 + (lane & 15);
#pragma unroll
    for (int mt = 0; mt < MT; ++mt)
#pragma unroll
      for (int v = 0; v < 4; ++v) {
        const int row = m0 + mt * 16 + (lane >> 4) * 4 + v;
        if (row < rows) out[(size_t)row * P.N + col] = acc[mt][j][v];
      }
  }
}

// Two workgroups per CU: the weight-streaming instances, whose time goes to loads in flight.
template <int MT, int NSUB, int SPLIT, bool ONCE>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(2))) void k_gemm_bf16(const GemmBatch g) {
  gemm_bf16_body<MT, NSUB, SPLIT, ONCE>(g);
}

// One workgroup per CU with the whole register file: 64 rows x 4 slabs per wave.  Launches of several
// row blocks are bound by MFMA issue and by the LDS reads of the activation fragments; a fragment read
// once serves four slabs here instead of two.
template <int SPLIT>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(1, 1))) void k_gemm_bf16_rows(const GemmBatch g) {
  gemm_bf16_body<4, 4, SPLIT, false>(g);
}

// ---------------------------------------------------------------------------------------------
// fp32 reference-mode GEMM (small models only): one thread per output column, 4 rows per block
// pass, plain sequential fp32 accumulation.  Workgroup = 64 columns x 16 rows.
// ---------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void k_gemm_f32(const GemmBatch g) {
  if (gemm_skip(g)) return;
  const int rows = g.n_rows ? *g.n_rows : g.rows_static;
  const int m0 = blockIdx.y * 16;
  if (m0 >= rows) return;
  int pi = 0;
  while (pi + 1 < g.n_prob && (int)blockIdx.x >= g.tile0[pi + 1]) ++pi;
  const GemmProb P = g.p[pi];
  const int ntile = (int)blockIdx.x - g.tile0[pi];
  const int col = ntile * 64 + (threadIdx.x & 63);
  if (col >= P.N) return;
  const float* A = reinterpret_cast<const float*>(P.A);
  const float* Wr = reinterpret_cast<const float*>(P.W) + (size_t)col * P.K;
  for (int r = m0 + (threadIdx.x >> 6); r < min(m0 + 16, rows); r += 4) {
    const float* a = A + (size_t)r * P.lda;
    float acc = 0.f;
    for (int k = 0; k < P.K; ++k) acc = fmaf(a[k], Wr[k], acc);
    P.out[(size_t)r * P.N + col] = acc;
  }
}

int gemm_cols_per_wg(int dtype, int nsub) { return dtype == 0 ? 64 : 64 * nsub; }

template <int MT>
static void launch_bf16(const GemmBatch& g, dim3 grid, hipStream_t s) {
  if (MT == 4 && g.nsub == 4) {
    if (g.split) hipLaunchKernelGGL((k_gemm_bf16_rows<1>), grid, dim3(256), 0, s, g);
    else hipLaunchKernelGGL((k_gemm_bf16_rows<0>), grid, dim3(256), 0, s, g);
  } else if (g.nsub == 4) {        // (MT < 4 here: one row block)
    if (g.split) hipLaunchKernelGGL((k_gemm_bf16<MT, 4, 1, true>), grid, dim3(256), 0, s, g);
    else hipLaunchKernelGGL((k_gemm_bf16<MT, 4, 0, true>), grid, dim3(256), 0, s, g);
  } else if (MT < 4 || g.row_blocks == 1) {
    if (g.split) hipLaunchKernelGGL((k_gemm_bf16<MT, 2, 1, true>), grid, dim3(256), 0, s, g);
    else hipLaunchKernelGGL((k_gemm_bf16<MT, 2, 0, true>), grid, dim3(256), 0, s, g);
  } else {
    if (g.split) hipLaunchKernelGGL((k_gemm_bf16<4, 2, 1, false>), grid, dim3(256), 0, s, g);
    else hipLaunchKernelGGL((k_gemm_bf16<4, 2, 0, false>), grid, dim3(256), 0, s, g);
  }
}

hipError_t launch_gemm(const GemmBatch& plan, int dtype, int rows_max, hipStream_t s) {
  const int wgs = plan.tile0[plan.n_prob];
  if (wgs <= 0 || rows_max <= 0) return hipSuccess;
  if (dtype == 0) {
    hipLaunchKernelGGL(k_gemm_f32, dim3(wgs, (rows_max + 15) / 16), dim3(256), 0, s, plan);
    return hipGetLastError();
  }
  GemmBatch g = plan;
  g.row_blocks = rows_max <= 64 ? 1 : (rows_max + 63) / 64;
  const dim3 grid((unsigned)((wgs + 7) / 8 * 8 * g.row_blocks));
  if (rows_max <= 16) launch_bf16<1>(g, grid, s);
  else if (rows_max <= 32) launch_bf16<2>(g, grid, s);
  else launch_bf16<4>(g, grid, s);
  return hipGetLastError();
}

}  // namespace cerb
