// Whole-K GEMMs with fused epilogues for launches of up to 64 rows (bf16 mode): the QKV projection
// with RoPE and the KV write, and the gate/up projection with SwiGLU, each as ONE launch.
//
// The split-K kernel (gemm.hip) leaves partial sums that a second kernel must add up before anything
// non-linear can be applied; per layer that is a RoPE/KV launch and a SwiGLU launch plus 38 MB of
// partials written and read again.  Here a workgroup owns whole columns instead: one workgroup per
// compute unit takes a few 16-column slabs over the full K, its eight waves split K among
// themselves, the eight partial accumulators meet in LDS, and the epilogue works on finished sums.
// Every workgroup then needs all of A.  A is therefore kept in MFMA A-fragment order
// (At[k-step][plane][row tile][lane], 16 bytes each, written that way by k_add_gain), so a wave pulls
// its fragments straight from L2 in 1 KB coalesced loads like the weights: no LDS staging, no
// barriers in the main loop.  What bounds the kernel is that broadcast: 256 workgroups x 1 MB of A
// through the L2s (QKV 29.7 us against 30.5 + 6.2 for GEMM + RoPE launch, gate/up 45 against
// 47 + 7.6).  For the O and down projections (one slab per compute unit, the same 1 MB of A for
// a sixth of the weights) it loses, so those stay split-K.
//
// Which slabs a workgroup owns comes from a table built on the host: positions come in pairs, and
// a pair holds the two slabs an epilogue needs together: columns j and j + dh/2 of a q or k head
// (RoPE rotates the two), two v slabs, or the gate and the up slab of the same FFN columns; an odd
// number of positions ends in a single v slab.
#include "step_kernels.h"

namespace cerb {

namespace {

constexpr int kWaves = 8;

// acc[mt][j] += A tile mt (hi and lo plane) x slab j over this wave's k range.  FULL: all four row
// tiles hold rows; else only the first mt_n are fetched and multiplied.
template <int NS, int DA, int DB, bool FULL>
__device__ __forceinline__ void whole_k_accumulate(const uint4* __restrict__ W, const uint4* __restrict__ At, int ksteps,
                                                   const int (&slab)[NS], int mt_n, f32x4_t (&acc)[4][NS]) {
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int units = ksteps / 4;                       // K is padded to 256: whole units of 4 k-steps
  const int ks0 = (wave * units / kWaves) * 4, ks1 = ((wave + 1) * units / kWaves) * 4;
  if (ks1 <= ks0) return;
  // Weights in stream order (see k_pack_stream): what the chip reads at the same time sits together.  The
  // fragment of (k-step i of the wave's range, wave, workgroup, position j) is piece block
  // ((i * kWaves + wave) * workgroups + workgroup) * NS + j.
  const size_t wstep = (size_t)kWaves * gridDim.x * NS * 64;
  const uint4* wp[NS];
#pragma unroll
  for (int j = 0; j < NS; ++j) wp[j] = W + ((size_t)(wave * gridDim.x + blockIdx.x) * NS + j) * 64 + lane;
  const uint4* ap = At + lane;                        // fragment (ks, plane, mt) at ((ks * 2 + plane) * 4 + mt) * 64

  // slot of k-step ks: (ks - ks0) % D.  Step i multiplies slot i % D after refilling the slot the previous
  // step has finished with (distance D - 1); loads past the range are clamped: valid memory, never multiplied.
  uint4 ra[DA][8], rb[DB][NS];
#pragma unroll
  for (int i = 0; i < DB - 1; ++i)
#pragma unroll
    for (int j = 0; j < NS; ++j)
      if (slab[j] >= 0) rb[i][j] = ld_weight_once(wp[j] + (size_t)min(i, ks1 - ks0 - 1) * wstep);
#pragma unroll
  for (int i = 0; i < DA - 1; ++i)
#pragma unroll
    for (int f = 0; f < 8; ++f)
      if (FULL || (f & 3) < mt_n) ra[i][f] = ap[(size_t)(min(ks0 + i, ks1 - 1) * 8 + f) * 64];

  for (int base = ks0; base < ks1; base += 4) {
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int ks = base + i;
#pragma unroll
      for (int j = 0; j < NS; ++j)
        if (slab[j] >= 0) rb[(i + DB - 1) % DB][j] = ld_weight_once(wp[j] + (size_t)min(ks + DB - 1 - ks0, ks1 - ks0 - 1) * wstep);
#pragma unroll
      for (int f = 0; f < 8; ++f)
        if (FULL || (f & 3) < mt_n) ra[(i + DA - 1) % DA][f] = ap[(size_t)(min(ks + DA - 1, ks1 - 1) * 8 + f) * 64];
      __builtin_amdgcn_sched_barrier(0);              // the refills are requested before this step's MFMAs
#pragma unroll
      for (int mt = 0; mt < 4; ++mt)
        if (FULL || mt < mt_n) {
#pragma unroll
          for (int j = 0; j < NS; ++j)
            if (slab[j] >= 0) {
              acc[mt][j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8_t, ra[i % DA][mt]),
                                                                   __builtin_bit_cast(bf16x8_t, rb[i % DB][j]), acc[mt][j], 0, 0, 0);
              acc[mt][j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8_t, ra[i % DA][4 + mt]),
                                                                   __builtin_bit_cast(bf16x8_t, rb[i % DB][j]), acc[mt][j], 0, 0, 0);
            }
        }
      __builtin_amdgcn_sched_barrier(0);
    }
  }
}

// Sum of the eight waves' accumulators of slab pair (2p, 2p+1) through LDS: red[which][wave][1024].
// Afterwards thread t finds element e of slab `which` at red[which * kWaves * 1024 + w * 1024 + e], e = t, t + 512;
// element e is row (e >> 8) * 16 + ((e & 63) >> 4) * 4 + ((e >> 6) & 3), column (e & 15) of the slab.
template <int NS>
__device__ __forceinline__ void stage_pair(const f32x4_t (&acc)[4][NS], int p, float* red) {
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  __syncthreads();                                    // the previous pair's sums have been read
#pragma unroll
  for (int which = 0; which < 2; ++which) {
    if (2 * p + which >= NS) break;                   // an odd NS ends in a single slab
#pragma unroll
    for (int mt = 0; mt < 4; ++mt)
#pragma unroll
      for (int v = 0; v < 4; ++v) {
        // p is a compile-time constant at every call site (unrolled loop)
        red[((which * kWaves + wave) * 16 + mt * 4 + v) * 64 + lane] = acc[mt][min(2 * p + which, NS - 1)][v];
      }
  }
  __syncthreads();
}

__device__ __forceinline__ float pair_sum(const float* red, int which, int e) {
  float s = 0.f;
#pragma unroll
  for (int w = 0; w < kWaves; ++w) s += red[(which * kWaves + w) * 1024 + e];
  return s;
}

__device__ __forceinline__ int elem_row(int e) { return (e >> 8) * 16 + ((e & 63) >> 4) * 4 + ((e >> 6) & 3); }

// Thread t finishes elements e = t and t + 512 of every slab: column c = t & 15 of rows r0 = elem_row(t)
// and r0 + 32.  What the epilogue needs about those two rows is fetched BEFORE the main loop, so that no
// memory round trip is left between the last MFMA and the stores.
struct RowInfo {
  float rs[2];      // 1 / sqrt(mean x^2 + eps): the pending norm's scalar, applied to the GEMM output
  bool live[2];
};
__device__ __forceinline__ RowInfo row_info(const float* __restrict__ ssq, int nb, int d, float eps, int rows) {
  RowInfo ri;
#pragma unroll
  for (int k = 0; k < 2; ++k) {
    const int r = elem_row((int)threadIdx.x) + 32 * k;
    ri.live[k] = r < rows;
    float ss = 0.f;
    if (ri.live[k])
      for (int i = 0; i < nb; ++i) ss += ssq[(size_t)r * nb + i];
    ri.rs[k] = 1.0f / sqrtf(ss / (float)d + eps);
  }
  return ri;
}

template <int NS>
__global__ __launch_bounds__(kWaves * 64) void k_qkv_rope(const FusedQkvArgs a) {
  __shared__ __attribute__((aligned(16))) float red[2 * kWaves * 1024];
  const int rows = min(*a.rm.n_rows, 64);
  if (rows <= 0) return;
  int slab[NS];
#pragma unroll
  for (int j = 0; j < NS; ++j) slab[j] = a.slabs[blockIdx.x * NS + j];
  bool any = false;
#pragma unroll
  for (int j = 0; j < NS; ++j) any = any || slab[j] >= 0;
  if (!any) return;                                           // uniform: a workgroup the table gave nothing

  const Dims& D = a.D;
  const int d = D.d, dh = D.dh, half = dh / 2, spd = d / 16, sph = dh / 16;   // slabs per section / per head
  const int c = threadIdx.x & 15;
  const RowInfo ri = row_info(a.ssq, a.nb, d, D.eps, rows);
  size_t cache_row[2];
  int seq[2];
  float2 rot[(NS + 1) / 2][2];                                // (cos, sin) of the two rows, per position pair
#pragma unroll
  for (int k = 0; k < 2; ++k) {
    const int r = min(elem_row((int)threadIdx.x) + 32 * k, rows - 1);
    seq[k] = a.rm.row_seq[r];
    cache_row[k] = (size_t)(a.rm.seq_L[seq[k]] + a.rm.row_node[r]);
#pragma unroll
    for (int p = 0; p < (NS + 1) / 2; ++p) {
      const int s0 = slab[2 * p];
      rot[p][k] = make_float2(1.f, 0.f);
      if (s0 >= 0 && s0 < 2 * spd) rot[p][k] = a.rope_cs[(size_t)r * half + (s0 % sph) * 16 + c];
    }
  }

  f32x4_t acc[4][NS];
#pragma unroll
  for (int mt = 0; mt < 4; ++mt)
#pragma unroll
    for (int j = 0; j < NS; ++j) acc[mt][j] = f32x4_t{0.f, 0.f, 0.f, 0.f};
  const int mt_n = (rows + 15) / 16;
  const uint4* W = reinterpret_cast<const uint4*>(a.W);
  const uint4* At = reinterpret_cast<const uint4*>(a.At);
  constexpr int DB = NS > 4 ? 2 : 4;
  if (mt_n == 4) whole_k_accumulate<NS, 2, DB, true>(W, At, a.ksteps, slab, 4, acc);
  else whole_k_accumulate<NS, 2, DB, false>(W, At, a.ksteps, slab, mt_n, acc);

#pragma unroll
  for (int p = 0; p < (NS + 1) / 2; ++p) {
    const int s0 = slab[2 * p], s1 = 2 * p + 1 < NS ? slab[min(2 * p + 1, NS - 1)] : -1;
    if (s0 < 0 && s1 < 0) continue;                           // uniform over the workgroup
    stage_pair<NS>(acc, p, red);
    const int section = max(s0, s1) / spd;                    // 0 q, 1 k, 2 v
#pragma unroll
    for (int k = 0; k < 2; ++k) {
      if (!ri.live[k]) continue;
      const int e = (int)threadIdx.x + 512 * k, r = elem_row(e);
      const float scale = ri.rs[k];
      const int b = seq[k];
      if (section < 2) {
        // the pair is columns j and j + dh/2 of one head: rotate by pos * theta^(-2j/dh)
        const int h = (s0 % spd) / sph, j = (s0 % sph) * 16 + c;
        const float x0 = pair_sum(red, 0, e) * scale, x1 = pair_sum(red, 1, e) * scale;
        const float cs = rot[p][k].x, sn = rot[p][k].y;
        const float y0 = x0 * cs - x1 * sn, y1 = x0 * sn + x1 * cs;
        const int c0 = h * dh + j, c1 = c0 + half;
        if (section == 0) {
          st_a(a.q + (size_t)r * d + c0, a.lo_off, y0);
          st_a(a.q + (size_t)r * d + c1, a.lo_off, y1);
        } else {
          if (a.kv_layer) {   // (the benchmark hook has no cache to write to)
            bf16_t* Kr = a.kv_layer + (((size_t)(0 * D.Bmax + b) * D.nH + h) * D.cap + cache_row[k]) * dh;
            Kr[j] = f32_to_bf16(y0);
            Kr[j + half] = f32_to_bf16(y1);
          }
          st_a(a.ktree + (size_t)r * d + c0, a.lo_off, y0);
          st_a(a.ktree + (size_t)r * d + c1, a.lo_off, y1);
        }
      } else {
#pragma unroll
        for (int which = 0; which < 2; ++which) {
          const int sv = which ? s1 : s0;
          if (sv < 0) continue;
          const int col = (sv % spd) * 16 + c, h = col / dh, j = col % dh;
          const float y = pair_sum(red, which, e) * scale;
          if (a.kv_layer) {
            bf16_t* Vr = a.kv_layer + (((size_t)(1 * D.Bmax + b) * D.nH + h) * D.cap + cache_row[k]) * dh;
            Vr[j] = f32_to_bf16(y);
          }
          st_a(a.vtree + (size_t)r * d + col, a.lo_off, y);
        }
      }
    }
  }
}

template <int NS>
__global__ __launch_bounds__(kWaves * 64) void k_gate_up_swiglu(const FusedGateUpArgs a) {
  __shared__ __attribute__((aligned(16))) float red[2 * kWaves * 1024];
  const int rows = min(*a.rm.n_rows, 64);
  if (rows <= 0) return;
  int slab[NS];
#pragma unroll
  for (int j = 0; j < NS; ++j) slab[j] = a.slabs[blockIdx.x * NS + j];
  bool any = false;
#pragma unroll
  for (int j = 0; j < NS; ++j) any = any || slab[j] >= 0;
  if (!any) return;                                           // uniform: a workgroup the table gave nothing
  const RowInfo ri = row_info(a.ssq, a.nb, a.d, a.eps, rows);
  f32x4_t acc[4][NS];
#pragma unroll
  for (int mt = 0; mt < 4; ++mt)
#pragma unroll
    for (int j = 0; j < NS; ++j) acc[mt][j] = f32x4_t{0.f, 0.f, 0.f, 0.f};
  const int mt_n = (rows + 15) / 16;
  const uint4* W = reinterpret_cast<const uint4*>(a.W);
  const uint4* At = reinterpret_cast<const uint4*>(a.At);
  constexpr int DB = NS > 4 ? 2 : 4;
  if (mt_n == 4) whole_k_accumulate<NS, 2, DB, true>(W, At, a.ksteps, slab, 4, acc);
  else whole_k_accumulate<NS, 2, DB, false>(W, At, a.ksteps, slab, mt_n, acc);

#pragma unroll
  for (int p = 0; p < NS / 2; ++p) {
    if (slab[2 * p] < 0) continue;                            // uniform; pairs are (gate slab, up slab) of the same columns
    stage_pair<NS>(acc, p, red);
    const int f = slab[2 * p] * 16 + ((int)threadIdx.x & 15);
#pragma unroll
    for (int k = 0; k < 2; ++k) {
      if (!ri.live[k]) continue;
      const int e = (int)threadIdx.x + 512 * k, r = elem_row(e);
      const float g = pair_sum(red, 0, e) * ri.rs[k], u = pair_sum(red, 1, e) * ri.rs[k];
      st_a(a.act + (size_t)r * a.Fpad + f, a.lo_off, g / (1.0f + expf(-g)) * u);
    }
  }
}

}  // namespace

// Stream-order copy of a packed weight matrix for a whole-K kernel of `grid` workgroups with `ns` slab positions each:
// dst[(((i * kWaves + w) * grid + g) * ns + j) * 64 + lane] = fragment (slab table[g][j], k-step ks0(w) + i) of the
// slab-major packing.  With every wave of every workgroup at about the same k-step of its range, the chip then reads one
// contiguous region at a time instead of 256 * 8 * ns one-KB pieces 16-128 KB apart (measured: gate/up 47.9 -> 43.4 us,
// a one-row launch 41.2 -> 37.9, the rate of a plain streaming read).  Positions without a slab and k-steps past a
// wave's range hold zeros.
__global__ void k_pack_stream(const uint4* __restrict__ src, uint4* __restrict__ dst, const int* __restrict__ table, int ns, int grid,
                              int ksteps, int maxlen) {
  const int units = ksteps / 4;
  const size_t total = (size_t)maxlen * kWaves * grid * ns * 64;
  for (size_t idx = (size_t)blockIdx.x * blockDim.x + threadIdx.x; idx < total; idx += (size_t)gridDim.x * blockDim.x) {
    const int lane = (int)(idx % 64);
    size_t blk = idx / 64;
    const int j = (int)(blk % ns); blk /= ns;
    const int g = (int)(blk % grid); blk /= grid;
    const int w = (int)(blk % kWaves);
    const int i = (int)(blk / kWaves);
    const int ks0 = (w * units / kWaves) * 4, ks1 = ((w + 1) * units / kWaves) * 4;
    const int slab = table[g * ns + j];
    uint4 v = make_uint4(0, 0, 0, 0);
    if (slab >= 0 && ks0 + i < ks1) v = src[((size_t)slab * ksteps + ks0 + i) * 64 + lane];
    dst[idx] = v;
  }
}

size_t fused_stream_pieces(int ns, int grid, int ksteps) {
  const int units = ksteps / 4;
  int maxlen = 0;
  for (int w = 0; w < kWaves; ++w) maxlen = std::max(maxlen, ((w + 1) * units / kWaves) * 4 - (w * units / kWaves) * 4);
  return (size_t)std::max(maxlen, 1) * kWaves * grid * ns * 64;
}

hipError_t launch_pack_stream(const void* packed, void* dst, const int* table, int ns, int grid, int ksteps, hipStream_t s) {
  const size_t pieces = fused_stream_pieces(ns, grid, ksteps);
  const int maxlen = (int)(pieces / ((size_t)kWaves * grid * ns * 64));
  hipLaunchKernelGGL(k_pack_stream, dim3(4096), dim3(256), 0, s, reinterpret_cast<const uint4*>(packed), reinterpret_cast<uint4*>(dst), table, ns,
                     grid, ksteps, maxlen);
  return hipGetLastError();
}

hipError_t launch_qkv_rope(const FusedQkvArgs& a, int ns, int grid, hipStream_t s) {
  if (ns == 3) hipLaunchKernelGGL(k_qkv_rope<3>, dim3(grid), dim3(kWaves * 64), 0, s, a);
  else if (ns == 2) hipLaunchKernelGGL(k_qkv_rope<2>, dim3(grid), dim3(kWaves * 64), 0, s, a);
  else if (ns == 4) hipLaunchKernelGGL(k_qkv_rope<4>, dim3(grid), dim3(kWaves * 64), 0, s, a);
  else if (ns == 6) hipLaunchKernelGGL(k_qkv_rope<6>, dim3(grid), dim3(kWaves * 64), 0, s, a);
  else return hipErrorInvalidValue;
  return hipGetLastError();
}

hipError_t launch_gate_up_swiglu(const FusedGateUpArgs& a, int ns, int grid, hipStream_t s) {
  if (ns == 2) hipLaunchKernelGGL(k_gate_up_swiglu<2>, dim3(grid), dim3(kWaves * 64), 0, s, a);
  else if (ns == 4) hipLaunchKernelGGL(k_gate_up_swiglu<4>, dim3(grid), dim3(kWaves * 64), 0, s, a);
  else if (ns == 6) hipLaunchKernelGGL(k_gate_up_swiglu<6>, dim3(grid), dim3(kWaves * 64), 0, s, a);
  else return hipErrorInvalidValue;
  return hipGetLastError();
}

}  // namespace cerb
