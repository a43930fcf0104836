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
#ifndef CERB_KRING
#define CERB_KRING 4
#endif
constexpr int kRing = CERB_KRING;  // k-steps of weights in flight per wave

__device__ __forceinline__ bool gemm_skip(const GemmBatch& g) {
  if (g.skip_flags == nullptr) return false;
  bool all = true;
  for (int i = 0; i < g.n_skip; ++i) all = all && (g.skip_flags[i] != 0);
  return all;
}

template <int MT, int NSUB, int SPLIT>
__global__ __launch_bounds__(256) void k_gemm_bf16(const GemmBatch g) {
  if (gemm_skip(g)) return;
  const int rows = g.n_rows ? *g.n_rows : g.rows_static;
  const int m0 = blockIdx.y * (MT * 16);
  if (m0 >= rows) return;

  int pi = 0;
  while (pi + 1 < g.n_prob && (int)blockIdx.x >= g.tile0[pi + 1]) ++pi;
  const GemmProb P = g.p[pi];
  const int local = (int)blockIdx.x - g.tile0[pi];
  const int split = local % P.S;
  const int ntile = local / P.S;
  constexpr int KSC = SPLIT ? 4 : 8;         // k-steps per LDS chunk
  const int ksteps = P.K / 32;               // K is a multiple of 256
  const int ks0 = split * P.kps;             // kps is a multiple of 8
  const int ks1 = min(ks0 + P.kps, ksteps);
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

  f32x4_t acc[MT][NSUB];
#pragma unroll
  for (int mt = 0; mt < MT; ++mt)
#pragma unroll
    for (int j = 0; j < NSUB; ++j) acc[mt][j] = f32x4_t{0.f, 0.f, 0.f, 0.f};

  // activation chunk c+1 travels global -> registers while chunk c is consumed from LDS.
  // (Plain unrolled loops with constant indices on purpose: staging arrays touched through a
  // lambda end up in scratch memory, and a scratch round trip inside the loop serialises the whole
  // in-order load queue.)
  constexpr int kApt = MT * 2;  // 16-byte pieces per thread per chunk
  const bf16_t* A = reinterpret_cast<const bf16_t*>(P.A);
  const bf16_t* a_src[kApt];
  int a_dst[kApt];
#pragma unroll
  for (int i = 0; i < kApt; ++i) {
    const int idx = threadIdx.x + i * 256;
    const int r = idx >> 5, pc = idx & 31;
    a_src[i] = A + (size_t)(m0 + r) * P.lda + (size_t)ks0 * 32 +
               (SPLIT ? (size_t)(pc >> 4) * P.lo_off + (pc & 15) * 8 : (size_t)pc * 8);
    a_dst[i] = r * kLdsRow + ((pc ^ (r & 15)) * 16);
  }
  uint4 areg[kApt];
#pragma unroll
  for (int i = 0; i < kApt; ++i) areg[i] = *reinterpret_cast<const uint4*>(a_src[i]);
  uint4 ring[kRing][NSUB];
#pragma unroll
  for (int i = 0; i < kRing; ++i)
#pragma unroll
    for (int j = 0; j < NSUB; ++j) ring[i][j] = wp[j][(size_t)min(ks0 + i, ks1 - 1) * 64];
#pragma unroll
  for (int i = 0; i < kApt; ++i) *reinterpret_cast<uint4*>(lds + a_dst[i]) = areg[i];
  __syncthreads();

  const int a_row = lane & 15, a_grp = lane >> 4;  // (mt*16 + a_row) & 15 == a_row
  for (int c = 0; c < nchunks; ++c) {
    const int cn = min(c + 1, nchunks - 1);
#pragma unroll
    for (int i = 0; i < kApt; ++i) areg[i] = *reinterpret_cast<const uint4*>(a_src[i] + (size_t)cn * (KSC * 32));
    const unsigned char* L = lds + (c & 1) * kBuf + a_row * kLdsRow;
    const int kb = ks0 + c * KSC;
#pragma unroll
    for (int s = 0; s < KSC; ++s) {
      uint4 b[NSUB];
#pragma unroll
      for (int j = 0; j < NSUB; ++j) {
        b[j] = ring[s % kRing][j];
        ring[s % kRing][j] = wp[j][(size_t)min(kb + s + kRing, ks1 - 1) * 64];
      }
#pragma unroll
      for (int mt = 0; mt < MT; ++mt) {
        const uint4 a = *reinterpret_cast<const uint4*>(L + mt * 16 * kLdsRow + (((s * 4 + a_grp) ^ a_row) * 16));
#pragma unroll
        for (int j = 0; j < NSUB; ++j)
          acc[mt][j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8_t, a),
                                                               __builtin_bit_cast(bf16x8_t, b[j]), acc[mt][j], 0, 0, 0);
        if (SPLIT) {
          const uint4 al = *reinterpret_cast<const uint4*>(L + mt * 16 * kLdsRow + (((16 + s * 4 + a_grp) ^ a_row) * 16));
#pragma unroll
          for (int j = 0; j < NSUB; ++j)
            acc[mt][j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8_t, al),
                                                                 __builtin_bit_cast(bf16x8_t, b[j]), acc[mt][j], 0, 0, 0);
        }
      }
    }
    unsigned char* Ln = lds + ((c + 1) & 1) * kBuf;
#pragma unroll
    for (int i = 0; i < kApt; ++i) *reinterpret_cast<uint4*>(Ln + a_dst[i]) = areg[i];
    __syncthreads();
  }

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
  if (g.nsub == 4) {
    if (g.split) hipLaunchKernelGGL((k_gemm_bf16<MT, 4, 1>), grid, dim3(256), 0, s, g);
    else hipLaunchKernelGGL((k_gemm_bf16<MT, 4, 0>), grid, dim3(256), 0, s, g);
  } else {
    if (g.split) hipLaunchKernelGGL((k_gemm_bf16<MT, 2, 1>), grid, dim3(256), 0, s, g);
    else hipLaunchKernelGGL((k_gemm_bf16<MT, 2, 0>), grid, dim3(256), 0, s, g);
  }
}

hipError_t launch_gemm(const GemmBatch& g, int dtype, int rows_max, hipStream_t s) {
  const int wgs = g.tile0[g.n_prob];
  if (wgs <= 0 || rows_max <= 0) return hipSuccess;
  if (dtype == 0) {
    hipLaunchKernelGGL(k_gemm_f32, dim3(wgs, (rows_max + 15) / 16), dim3(256), 0, s, g);
  } else if (rows_max <= 16) {
    launch_bf16<1>(g, dim3(wgs, 1), s);
  } else if (rows_max <= 32) {
    launch_bf16<2>(g, dim3(wgs, 1), s);
  } else {
    launch_bf16<4>(g, dim3(wgs, (rows_max + 63) / 64), s);
  }
  return hipGetLastError();
}

}  // namespace cerb
