// Small kernels of the verify step: tree assembly and embedding, residual + RMSNorm, RoPE and KV
// write, SwiGLU, per-node argmax, acceptance walk, KV compaction, entropy gate, the element-wise
// half of the Cerberus heads' Resblocks, and per-head top-k.  All are bandwidth-trivial next to
// the weight stream; each is written for clarity and coalesced access.
#include "step_kernels.h"

#include <limits.h>

namespace cerb {

// ---------------------------------------------------------------------------------------------
// block reductions (blockDim.x a multiple of 64, at most 1024: sh holds one entry per wave)
// ---------------------------------------------------------------------------------------------
template <typename V>
__device__ __forceinline__ V block_sum(V v, V* sh) {
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off, 64);
  const int wave = threadIdx.x >> 6, nw = (blockDim.x + 63) >> 6;
  __syncthreads();
  if ((threadIdx.x & 63) == 0) sh[wave] = v;
  __syncthreads();
  V t = sh[0];
  for (int w = 1; w < nw; ++w) t += sh[w];
  return t;
}

__device__ __forceinline__ float block_max(float v, float* sh) {
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) v = fmaxf(v, __shfl_xor(v, off, 64));
  const int wave = threadIdx.x >> 6, nw = (blockDim.x + 63) >> 6;
  __syncthreads();
  if ((threadIdx.x & 63) == 0) sh[wave] = v;
  __syncthreads();
  float t = sh[0];
  for (int w = 1; w < nw; ++w) t = fmaxf(t, sh[w]);
  return t;
}

// best = larger value, ties to the lower index
__device__ __forceinline__ void better(float& bv, int& bi, float v, int i) {
  const bool take = (v > bv) | ((v == bv) & (i < bi));   // bitwise on purpose: selects, not branches, per element
  bv = take ? v : bv;
  bi = take ? i : bi;
}

__device__ __forceinline__ void block_argmax(float& bv, int& bi, float* shv, int* shi) {
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) {
    const float ov = __shfl_xor(bv, off, 64);
    const int oi = __shfl_xor(bi, off, 64);
    better(bv, bi, ov, oi);
  }
  const int wave = threadIdx.x >> 6, nw = (blockDim.x + 63) >> 6;
  __syncthreads();
  if ((threadIdx.x & 63) == 0) { shv[wave] = bv; shi[wave] = bi; }
  __syncthreads();
  bv = shv[0]; bi = shi[0];
  for (int w = 1; w < nw; ++w) better(bv, bi, shv[w], shi[w]);
}

// ---------------------------------------------------------------------------------------------
// Split-K partials are summed by their consumer, in split order.  All MAXS loads are issued before
// the first add: a loop with a run-time trip count makes the compiler wait for every load in turn,
// S memory round trips in a row, which is what these kernels' run time would consist of.  Splits
// >= S re-read the last valid split (a cache hit) and are dropped by a select.  MAXS == 0: no loads.
// ---------------------------------------------------------------------------------------------
template <int MAXS, typename V>
struct Parts {
  V v[MAXS > 0 ? MAXS : 1];
  __device__ __forceinline__ void load(const float* p, size_t pstride, int S) {
#pragma unroll
    for (int s = 0; s < MAXS; ++s) v[s] = *reinterpret_cast<const V*>(p + (size_t)min(s, S - 1) * pstride);
  }
};
template <int MAXS>
__device__ __forceinline__ float add_parts(float a, const Parts<MAXS, float>& P, int S) {
#pragma unroll
  for (int s = 0; s < MAXS; ++s) a += (s < S) ? P.v[s] : 0.f;
  return a;
}
template <int MAXS>
__device__ __forceinline__ float4 add_parts(float4 a, const Parts<MAXS, float4>& P, int S) {
#pragma unroll
  for (int s = 0; s < MAXS; ++s) {
    const bool on = s < S;
    a.x += on ? P.v[s].x : 0.f; a.y += on ? P.v[s].y : 0.f; a.z += on ? P.v[s].z : 0.f; a.w += on ? P.v[s].w : 0.f;
  }
  return a;
}

// smallest compiled bucket that holds S splits
#define CERB_S_BUCKET(S, CALL)                                                                     \
  do {                                                                                             \
    if ((S) <= 0) { CALL(0); } else if ((S) <= 2) { CALL(2); } else if ((S) <= 4) { CALL(4); }     \
    else if ((S) <= 8) { CALL(8); } else { CALL(16); }                                             \
  } while (0)

// ---------------------------------------------------------------------------------------------
// Tree assembly (Algorithm 1 line 1 and the Candidates tuple of lines 11-12): which rows this step
// has, and the token / position of each.  One block; sequences pack their rows back to back.
// ---------------------------------------------------------------------------------------------
__global__ __launch_bounds__(64) void k_assemble(const Dims D, const TreeDev tr, const RowMap rm, const cerberus_state st,
                                                 const cerberus_taps tp, int batch, int mode, const PromptArgs pa,
                                                 const AttnPlanCfg ap) {
  __shared__ int sT[CERBERUS_MAX_BATCH], sL[CERBERUS_MAX_BATCH], sRow0[CERBERUS_MAX_BATCH];
  const int t = threadIdx.x;
  if (t < batch) {
    const int L = st.kv_len[t];
    int Tb = tr.T;
    if (mode == ASSEMBLE_FORCE_AR || (mode == ASSEMBLE_BY_FLAG && st.gate_flag[t] != 0)) Tb = 1;
    if (mode == ASSEMBLE_PROMPT) Tb = (t == pa.seq) ? pa.n : 0;   // a chain of prompt tokens (tr is the chain's tables)
    if (Tb > 0 && (L < 0 || L + Tb > D.cap)) {  // the sequence sits this step out
      Tb = 0;
      atomicOr(st.status, (int)CERBERUS_DEV_KV_OVERFLOW);
    }
    sT[t] = Tb;
    sL[t] = L;
  }
  __syncthreads();
  if (t == 0) {
    // rows pack back to back; with the caller's per-node arrays of the acceptance entry point
    // (ASSEMBLE_FULL_TREE) sequence b owns rows b*T.. whether or not an earlier sequence sits out
    int r = 0;
    for (int b = 0; b < batch; ++b) {
      sRow0[b] = mode == ASSEMBLE_FULL_TREE ? b * tr.T : r;
      r += sT[b];
    }
    *rm.n_rows = mode == ASSEMBLE_FULL_TREE ? batch * tr.T : r;
  }
  __syncthreads();
  if (rm.att_item != nullptr && ap.chunk > 0) {
    // Work list of the attention kernel, sized by the lengths the sequences have now, not by the cache
    // capacity: a cache-range item covers `cps` chunks of one sequence's committed rows, a tree item 64 of
    // the step's own rows.  cps grows with the total length so that the list stays near the workgroup
    // target: a long cache is walked inside a workgroup (one partial result per item) instead of being cut
    // into a partial per chunk.  Every thread derives the same plan; thread i writes entries i, i + 64, ...
    int chunks = 0;
    for (int b = 0; b < batch; ++b)
      if (sT[b] > 0) chunks += (sL[b] + ap.chunk - 1) / ap.chunk;
    const int per_head = max(1, ap.target_wgs / D.nH);
    const int cps = min(0xffff, max(1, (chunks + per_head - 1) / per_head));
    int n = 0;
    for (int b = 0; b < batch; ++b) {
      const int npi = sT[b] > 0 ? ((sL[b] + ap.chunk - 1) / ap.chunk + cps - 1) / cps : 0;
      const int ntree = (sT[b] + 63) / 64;
      if (t == 0) rm.seq_npi[b] = npi;
      for (int j = t; j < npi + ntree; j += blockDim.x)
        if (n + j < ap.att_cap) rm.att_item[n + j] = make_int4((b << 16) | j, sL[b], (sT[b] << 16) | sRow0[b], (npi << 16) | cps);
      n += npi + ntree;
    }
    for (int i = n + t; i < ap.att_cap; i += blockDim.x) rm.att_item[i] = make_int4(-1, 0, 0, 0);
  }
  __syncthreads();
  if (t < batch) { rm.seq_T[t] = sT[t]; rm.seq_L[t] = sL[t]; rm.seq_row0[t] = sRow0[t]; }
  for (int b = 0; b < batch; ++b) {
    for (int node = t; node < sT[b]; node += blockDim.x) {
      const int r = sRow0[b] + node;
      const int dep = tr.depth[node];
      rm.row_seq[r] = b;
      rm.row_node[r] = node;
      rm.row_pos[r] = sL[b] + dep;
      if (mode != ASSEMBLE_FULL_TREE) {
        int tok;
        if (mode == ASSEMBLE_PROMPT) tok = pa.tokens[node];
        else tok = node == 0 ? st.root_token[b] : st.cand[(b * D.Hc + dep - 1) * D.topk + tr.rank[node]];
        if (tok < 0 || tok >= D.V) { atomicOr(st.status, (int)CERBERUS_DEV_BAD_TOKEN); tok = 0; }
        rm.row_tok[r] = tok;
        if (tp.node_token && node < D.T) tp.node_token[b * D.T + node] = tok;   // the taps hold T rows per sequence
      }
    }
  }
}

hipError_t launch_assemble(const Dims& D, const TreeDev& tr, const RowMap& rm, const cerberus_state& st,
                           const cerberus_taps& tp, int batch, int mode, const PromptArgs& pa, const AttnPlanCfg& ap, hipStream_t s) {
  hipLaunchKernelGGL(k_assemble, dim3(1), dim3(64), 0, s, D, tr, rm, st, tp, batch, mode, pa, ap);
  return hipGetLastError();
}

// End of a prompt pass: the rows are where they belong already (row L + i), so committing them is
// advancing kv_len.  After the last pass the pending token is the base model's choice at the last
// prompt position, and that row feeds the gate and the heads.
__global__ void k_prompt_commit(const RowMap rm, const cerberus_state st, const int* __restrict__ g, int* __restrict__ last_row,
                                int batch, int seq, int last_pass) {
  const int b = threadIdx.x;
  if (b >= batch) return;
  const int n = rm.seq_T[b];              // 0 for every sequence but `seq` (and for `seq` when it did not fit)
  last_row[b] = -1;
  if (b != seq || n <= 0) return;
  st.kv_len[b] = rm.seq_L[b] + n;
  st.accept_len[b] = 0;
  if (last_pass) {
    const int r = rm.seq_row0[b] + n - 1;
    st.root_token[b] = g[r];
    last_row[b] = r;
  }
}

hipError_t launch_prompt_commit(const RowMap& rm, const cerberus_state& st, const int* g, int* last_row, int batch, int seq,
                                int last_pass, hipStream_t s) {
  hipLaunchKernelGGL(k_prompt_commit, dim3(1), dim3(64), 0, s, rm, st, g, last_row, batch, seq, last_pass);
  return hipGetLastError();
}

// x[row] = embedding of the row's token, widened to fp32; 512 threads, 8 consecutive elements each
// per pass (d % 8 == 0)
template <typename T>
__global__ __launch_bounds__(512) void k_embed(const T* __restrict__ embed, const RowMap rm, float* __restrict__ x, int d,
                                               const double* __restrict__ inv_freq, float2* __restrict__ rope_cs, int half) {
  const int r = blockIdx.x;
  if (r >= *rm.n_rows) return;
  // the row's RoPE rotations, the same in every layer: angle in double (at position ~4000 an fp32 product is
  // already off by 1e-4 rad), stored as float
  if ((int)threadIdx.x < half) {
    double snd, csd;
    sincos((double)rm.row_pos[r] * inv_freq[threadIdx.x], &snd, &csd);
    rope_cs[(size_t)r * half + threadIdx.x] = make_float2((float)csd, (float)snd);
  }
  const T* e = embed + (size_t)rm.row_tok[r] * d;
  for (int c = threadIdx.x * 8; c < d; c += 512 * 8) {
    float v[8];
    if (sizeof(T) == 2) {
      const uint4 w = *reinterpret_cast<const uint4*>(e + c);
      const uint32_t u[4] = {w.x, w.y, w.z, w.w};
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        v[2 * i] = __uint_as_float(u[i] << 16);
        v[2 * i + 1] = __uint_as_float(u[i] & 0xffff0000u);
      }
    } else {
#pragma unroll
      for (int i = 0; i < 8; ++i) v[i] = ld_f(e + c + i);
    }
    float* o = x + (size_t)r * d + c;
    *reinterpret_cast<float4*>(o) = make_float4(v[0], v[1], v[2], v[3]);
    *reinterpret_cast<float4*>(o + 4) = make_float4(v[4], v[5], v[6], v[7]);
  }
}

hipError_t launch_embed(const Dims& D, const RowMap& rm, const void* embed, float* x, const double* inv_freq, float2* rope_cs,
                        int rows_max, hipStream_t s) {
  if (D.dtype == 0) hipLaunchKernelGGL((k_embed<float>), dim3(rows_max), dim3(512), 0, s, (const float*)embed, rm, x, D.d, inv_freq, rope_cs, D.dh / 2);
  else hipLaunchKernelGGL((k_embed<bf16_t>), dim3(rows_max), dim3(512), 0, s, (const bf16_t*)embed, rm, x, D.d, inv_freq, rope_cs, D.dh / 2);
  return hipGetLastError();
}

// ---------------------------------------------------------------------------------------------
// x += sum of the previous GEMM's split-K partials (the residual add), then RMSNorm:
// out = x * gain / sqrt(mean(x^2) + eps), rounded to the GEMM input type.  d <= 8192, d % 4 == 0.
// One workgroup of 1024 threads per row; a thread owns up to two float4 column groups and has x and
// every partial of a group in flight together, so the row is read exactly once, in one round trip.
template <typename T, int MAXS>
__global__ __launch_bounds__(1024) void k_add_rmsnorm(float* __restrict__ x, const float* __restrict__ part, int S,
                                                      size_t pstride, const float* __restrict__ gain, float eps,
                                                      T* __restrict__ out, size_t lo_off, float* __restrict__ out_f32,
                                                      float* __restrict__ tap, const RowMap rm, int d, int T_tree) {
  __shared__ float sh[16];
  const int r = blockIdx.x;
  if (r >= *rm.n_rows) return;
  float* xr = x + (size_t)r * d;
  float4 v[2], g[2];
  float ss = 0.f;
#pragma unroll
  for (int it = 0; it < 2; ++it) {
    const int c = (it * 1024 + threadIdx.x) * 4;
    v[it] = make_float4(0.f, 0.f, 0.f, 0.f);
    g[it] = v[it];
    if (c < d) {
      Parts<MAXS, float4> P;
      P.load(part + (size_t)r * d + c, pstride, S);
      v[it] = *reinterpret_cast<const float4*>(xr + c);
      g[it] = *reinterpret_cast<const float4*>(gain + c);
      v[it] = add_parts(v[it], P, S);
      if (MAXS > 0) *reinterpret_cast<float4*>(xr + c) = v[it];
      ss += v[it].x * v[it].x + v[it].y * v[it].y + v[it].z * v[it].z + v[it].w * v[it].w;
    }
  }
  ss = block_sum(ss, sh);
  const float sc = 1.0f / sqrtf(ss / (float)d + eps);
  float* tp = (tap && rm.row_node[r] < T_tree) ? tap + ((size_t)rm.row_seq[r] * T_tree + rm.row_node[r]) * d : nullptr;   // T rows per sequence
#pragma unroll
  for (int it = 0; it < 2; ++it) {
    const int c = (it * 1024 + threadIdx.x) * 4;
    if (c < d) {
      const float o[4] = {v[it].x * g[it].x * sc, v[it].y * g[it].y * sc, v[it].z * g[it].z * sc, v[it].w * g[it].w * sc};
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        st_a(out + (size_t)r * d + c + e, lo_off, o[e]);
        if (out_f32) out_f32[(size_t)r * d + c + e] = o[e];
        if (tp) tp[c + e] = o[e];
      }
    }
  }
}

hipError_t launch_add_rmsnorm(const Dims& D, const RowMap& rm, float* x, const float* part, int S, size_t pstride,
                              const float* gain, void* out, float* out_f32, float* tap, int rows_max, hipStream_t s) {
#define CERB_CALL(MS)                                                                                                   \
  if (D.dtype == 0)                                                                                                     \
    hipLaunchKernelGGL((k_add_rmsnorm<float, MS>), dim3(rows_max), dim3(1024), 0, s, x, part, S, pstride, gain, D.eps,  \
                       (float*)out, (size_t)0, out_f32, tap, rm, D.d, D.T);                                             \
  else                                                                                                                  \
    hipLaunchKernelGGL((k_add_rmsnorm<bf16_t, MS>), dim3(rows_max), dim3(1024), 0, s, x, part, S, pstride, gain, D.eps, \
                       (bf16_t*)out, (size_t)D.R64 * D.d, out_f32, tap, rm, D.d, D.T)
  CERB_S_BUCKET(S, CERB_CALL);
#undef CERB_CALL
  return hipGetLastError();
}

// ---------------------------------------------------------------------------------------------
// The per-layer norms, split so that more than one workgroup can work on a row.  RMSNorm is a
// per-row scalar times x * gain, and a GEMM is linear in its input rows, so the scalar can be applied
// to the GEMM's output instead: this kernel does the residual add and writes x * gain as the GEMM
// input plus, per (row, 1024-column block), the block's sum of x^2; the kernel that sums the GEMM's
// split-K partials (k_rope_kv, k_swiglu) forms 1 / sqrt(mean x^2 + eps) from those sums and scales.
// Four workgroups per row at d = 4096 instead of one.
// ---------------------------------------------------------------------------------------------
// TILED (bf16 only): the GEMM input goes out in MFMA A-fragment order for the whole-K GEMMs: the 8 values of
// row r at columns ks*32 + g*8.. form 16-byte piece ((ks*2 + plane)*4 + r/16)*64 + r%16 + 16*g, 64 rows in all.
template <typename T, int MAXS, bool TILED>
__global__ __launch_bounds__(256) void k_add_gain(float* __restrict__ x, const float* __restrict__ part, int S, size_t pstride,
                                                  const float* __restrict__ gain, T* __restrict__ out, size_t lo_off,
                                                  float* __restrict__ ssq, const RowMap rm, int d) {
  __shared__ float sh[4];
  const int r = blockIdx.x, nb = gridDim.y;
  if (r >= *rm.n_rows) return;
  const int c = (blockIdx.y * 256 + threadIdx.x) * 4;
  float ss = 0.f;
  if (c < d) {
    float* xr = x + (size_t)r * d + c;
    Parts<MAXS, float4> P;
    P.load(part + (size_t)r * d + c, pstride, S);
    float4 v = *reinterpret_cast<const float4*>(xr);
    const float4 g = *reinterpret_cast<const float4*>(gain + c);
    v = add_parts(v, P, S);
    if (MAXS > 0) *reinterpret_cast<float4*>(xr) = v;
    ss = v.x * v.x + v.y * v.y + v.z * v.z + v.w * v.w;
    const float o[4] = {v.x * g.x, v.y * g.y, v.z * g.z, v.w * g.w};
    if (TILED && sizeof(T) == 2) {
      union { bf16_t h[4]; uint2 u; } hi, lo;
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        hi.h[e] = f32_to_bf16(o[e]);
        lo.h[e] = f32_to_bf16(o[e] - bf16_to_f32(hi.h[e]));
      }
      const size_t piece = ((size_t)(c >> 5) * 8 + (r >> 4)) * 64 + (r & 15) + 16 * ((c & 31) >> 3);   // hi plane; lo: + 4 * 64
      unsigned char* base = reinterpret_cast<unsigned char*>(out) + (c & 7) * 2;
      *reinterpret_cast<uint2*>(base + piece * 16) = hi.u;
      *reinterpret_cast<uint2*>(base + (piece + 256) * 16) = lo.u;
    } else {
      st_a4(out + (size_t)r * d + c, lo_off, o);       // d % 4 == 0: aligned
    }
  }
  ss = block_sum(ss, sh);
  if (threadIdx.x == 0) ssq[(size_t)r * nb + blockIdx.y] = ss;
}

int add_gain_blocks(int d) { return (d + 1023) / 1024; }

hipError_t launch_add_gain(const Dims& D, const RowMap& rm, float* x, const float* part, int S, size_t pstride,
                           const float* gain, void* out, float* ssq, int rows_max, hipStream_t s, bool a_tiled) {
  const dim3 grid(rows_max, add_gain_blocks(D.d));
  if (a_tiled && (D.dtype == 0 || rows_max > 64)) return hipErrorInvalidValue;
#define CERB_CALL(MS)                                                                                                  \
  if (D.dtype == 0)                                                                                                    \
    hipLaunchKernelGGL((k_add_gain<float, MS, false>), grid, dim3(256), 0, s, x, part, S, pstride, gain, (float*)out,  \
                       (size_t)0, ssq, rm, D.d);                                                                       \
  else if (a_tiled)                                                                                                    \
    hipLaunchKernelGGL((k_add_gain<bf16_t, MS, true>), grid, dim3(256), 0, s, x, part, S, pstride, gain, (bf16_t*)out, \
                       (size_t)D.R64 * D.d, ssq, rm, D.d);                                                             \
  else                                                                                                                 \
    hipLaunchKernelGGL((k_add_gain<bf16_t, MS, false>), grid, dim3(256), 0, s, x, part, S, pstride, gain, (bf16_t*)out,\
                       (size_t)D.R64 * D.d, ssq, rm, D.d)
  CERB_S_BUCKET(S, CERB_CALL);
#undef CERB_CALL
  return hipGetLastError();
}

// 1 / sqrt(mean x^2 + eps) of row r from the block sums k_add_gain left (summed in block order)
__device__ __forceinline__ float row_rms_scale(const float* __restrict__ ssq, int r, int nb, int d, float eps) {
  float ss = 0.f;
  for (int i = 0; i < nb; ++i) ss += ssq[(size_t)r * nb + i];
  return 1.0f / sqrtf(ss / (float)d + eps);
}

// ---------------------------------------------------------------------------------------------
// Sum the QKV partials, rotate q and k (pair (j, j + dh/2) by pos * theta^(-2j/dh)), write q for the
// attention kernel and k, v into the cache at row L + node.
// ---------------------------------------------------------------------------------------------
template <typename T>
__global__ void k_rope_kv(const float* __restrict__ part, int S, size_t pstride, const float2* __restrict__ rope_cs,
                          const RowMap rm, T* __restrict__ q, size_t q_lo_off, T* __restrict__ kv_layer,
                          T* __restrict__ ktree, T* __restrict__ vtree, const float* __restrict__ ssq, int nb, const Dims D) {
  const int r = blockIdx.x, h = blockIdx.y, j = threadIdx.x;
  if (r >= *rm.n_rows) return;
  const float rs = row_rms_scale(ssq, r, nb, D.d, D.eps);   // the layer input's RMSNorm scalar, applied to the GEMM output
  const int b = rm.row_seq[r], node = rm.row_node[r];
  const int d = D.d, dh = D.dh, half = dh / 2, N = 3 * d;
  const int c0 = h * dh + j, c1 = c0 + half;
  // (a plain loop: these partials are still in L2 and the kernel is bound by their volume, so having
  // every split's loads in flight at once gains nothing here)
  float v[6] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
  for (int s = 0; s < S; ++s) {
    const float* p = part + s * pstride + (size_t)r * N;
    v[0] += p[c0]; v[1] += p[c1]; v[2] += p[d + c0]; v[3] += p[d + c1]; v[4] += p[2 * d + c0]; v[5] += p[2 * d + c1];
  }
#pragma unroll
  for (int e = 0; e < 6; ++e) v[e] *= rs;
  const float2 rot = rope_cs[(size_t)r * half + j];   // (cos, sin), formed once per step by the embedding kernel
  const float cs = rot.x, sn = rot.y;
  st_a(q + (size_t)r * d + c0, q_lo_off, v[0] * cs - v[1] * sn);
  st_a(q + (size_t)r * d + c1, q_lo_off, v[0] * sn + v[1] * cs);
  const float k0 = v[2] * cs - v[3] * sn, k1 = v[2] * sn + v[3] * cs;
  const size_t row = (size_t)(rm.seq_L[b] + node);
  T* Kr = kv_layer + (((size_t)(0 * D.Bmax + b) * D.nH + h) * D.cap + row) * dh;
  T* Vr = kv_layer + (((size_t)(1 * D.Bmax + b) * D.nH + h) * D.cap + row) * dh;
  st_f(Kr + j, k0);
  st_f(Kr + j + half, k1);
  st_f(Vr + j, v[4]);
  st_f(Vr + j + half, v[5]);
  if (ktree) {
    // This step's attention reads the tree rows from these hi+lo planes instead: rounding a new
    // row to one bf16 before its own step uses it is the largest single error of the bf16 path
    // (4.8e-2 of logits at the 13B shape against 1e-2 from everything else).
    st_a(ktree + (size_t)r * d + c0, q_lo_off, k0);
    st_a(ktree + (size_t)r * d + c1, q_lo_off, k1);
    st_a(vtree + (size_t)r * d + c0, q_lo_off, v[4]);
    st_a(vtree + (size_t)r * d + c1, q_lo_off, v[5]);
  }
}

hipError_t launch_rope_kv(const Dims& D, const RowMap& rm, const float* part, int S, size_t pstride,
                          const float2* rope_cs, void* q, void* kv_layer, void* ktree, void* vtree, const float* ssq,
                          int rows_max, hipStream_t s) {
  const int nb = add_gain_blocks(D.d);
  dim3 grid(rows_max, D.nH), block(D.dh / 2);
  if (D.dtype == 0)
    hipLaunchKernelGGL((k_rope_kv<float>), grid, block, 0, s, part, S, pstride, rope_cs, rm, (float*)q, (size_t)0,
                       (float*)kv_layer, (float*)nullptr, (float*)nullptr, ssq, nb, D);
  else
    hipLaunchKernelGGL((k_rope_kv<bf16_t>), grid, block, 0, s, part, S, pstride, rope_cs, rm, (bf16_t*)q,
                       (size_t)D.R64 * D.d, (bf16_t*)kv_layer, (bf16_t*)ktree, (bf16_t*)vtree, ssq, nb, D);
  return hipGetLastError();
}

// act = SiLU(gate) * up from the gate/up partials ([.., 2F]: gate columns first)
template <typename T>
__global__ __launch_bounds__(256) void k_swiglu(const float* __restrict__ part, int S, size_t pstride, T* __restrict__ act,
                                                size_t lo_off, const RowMap rm, int F, int Fpad,
                                                const float* __restrict__ ssq, int nb, int d, float eps) {
  const int r = blockIdx.x;
  if (r >= *rm.n_rows) return;
  const int f = blockIdx.y * 256 + threadIdx.x;
  if (f >= F) return;
  const float rs = row_rms_scale(ssq, r, nb, d, eps);   // the FFN input's RMSNorm scalar
  float g = 0.f, u = 0.f;
  for (int s = 0; s < S; ++s) {
    const float* p = part + s * pstride + (size_t)r * 2 * F;
    g += p[f];
    u += p[F + f];
  }
  g *= rs;
  u *= rs;
  st_a(act + (size_t)r * Fpad + f, lo_off, g / (1.0f + expf(-g)) * u);
}

// The same for four consecutive FFN columns per thread (F % 4 == 0): 16-byte loads, 8-byte stores.  Launches of
// several row blocks move enough bytes for this form to win; at up to 64 rows the scalar form, with four times
// the waves to hide the latency of the one round trip, is the faster one.
template <typename T>
__global__ __launch_bounds__(256) void k_swiglu4(const float* __restrict__ part, int S, size_t pstride, T* __restrict__ act,
                                                 size_t lo_off, const RowMap rm, int F, int Fpad,
                                                 const float* __restrict__ ssq, int nb, int d, float eps) {
  const int r = blockIdx.x;
  if (r >= *rm.n_rows) return;
  const int f = (blockIdx.y * 256 + threadIdx.x) * 4;
  if (f >= F) return;
  const float rs = row_rms_scale(ssq, r, nb, d, eps);
  float4 g = make_float4(0.f, 0.f, 0.f, 0.f), u = g;
  for (int s = 0; s < S; ++s) {
    const float* p = part + s * pstride + (size_t)r * 2 * F;
    const float4 a = *reinterpret_cast<const float4*>(p + f), b = *reinterpret_cast<const float4*>(p + F + f);
    g.x += a.x; g.y += a.y; g.z += a.z; g.w += a.w;
    u.x += b.x; u.y += b.y; u.z += b.z; u.w += b.w;
  }
  const float gg[4] = {g.x * rs, g.y * rs, g.z * rs, g.w * rs}, uu[4] = {u.x * rs, u.y * rs, u.z * rs, u.w * rs};
  float o[4];
#pragma unroll
  for (int e = 0; e < 4; ++e) o[e] = gg[e] / (1.0f + expf(-gg[e])) * uu[e];
  st_a4(act + (size_t)r * Fpad + f, lo_off, o);
}

hipError_t launch_swiglu(const Dims& D, const RowMap& rm, const float* part, int S, size_t pstride, void* act,
                         const float* ssq, int rows_max, hipStream_t s) {
  const int nb = add_gain_blocks(D.d);
  if (rows_max > 64 && D.F % 4 == 0 && D.Fpad % 4 == 0 && pstride % 4 == 0) {
    dim3 grid4(rows_max, (D.F / 4 + 255) / 256);
    if (D.dtype == 0) hipLaunchKernelGGL((k_swiglu4<float>), grid4, dim3(256), 0, s, part, S, pstride, (float*)act, (size_t)0, rm, D.F, D.Fpad, ssq, nb, D.d, D.eps);
    else hipLaunchKernelGGL((k_swiglu4<bf16_t>), grid4, dim3(256), 0, s, part, S, pstride, (bf16_t*)act, (size_t)D.R64 * D.Fpad, rm, D.F, D.Fpad, ssq, nb, D.d, D.eps);
    return hipGetLastError();
  }
  dim3 grid(rows_max, (D.F + 255) / 256);
  if (D.dtype == 0) hipLaunchKernelGGL((k_swiglu<float>), grid, dim3(256), 0, s, part, S, pstride, (float*)act, (size_t)0, rm, D.F, D.Fpad, ssq, nb, D.d, D.eps);
  else hipLaunchKernelGGL((k_swiglu<bf16_t>), grid, dim3(256), 0, s, part, S, pstride, (bf16_t*)act, (size_t)D.R64 * D.Fpad, rm, D.F, D.Fpad, ssq, nb, D.d, D.eps);
  return hipGetLastError();
}

// ---------------------------------------------------------------------------------------------
// g[row] = argmax over the vocabulary of the LM-head logits (Algorithm 1 line 9 at every node),
// lowest id on ties.
// ---------------------------------------------------------------------------------------------
__global__ __launch_bounds__(1024) void k_row_argmax(const float* __restrict__ part, int S, size_t pstride, int* __restrict__ g,
                                                     const cerberus_taps tp, const RowMap rm, int V, int T_tree) {
  __shared__ float shv[16];
  __shared__ int shi[16];
  const int r = blockIdx.x;
  if (r >= *rm.n_rows) return;
  const size_t slot = (size_t)rm.row_seq[r] * T_tree + rm.row_node[r];
  const bool tapped = rm.row_node[r] < T_tree;   // the taps hold T rows per sequence; a prompt pass can be longer
  float bv = -INFINITY;
  int bi = INT_MAX;
  for (int v = threadIdx.x * 4; v < V; v += 4096) {   // V % 16 == 0
    float4 val = make_float4(0.f, 0.f, 0.f, 0.f);
    for (int s = 0; s < S; ++s) {
      const float4 p = *reinterpret_cast<const float4*>(part + s * pstride + (size_t)r * V + v);
      val.x += p.x; val.y += p.y; val.z += p.z; val.w += p.w;
    }
    if (tp.logits && tapped) *reinterpret_cast<float4*>(tp.logits + slot * V + v) = val;
    better(bv, bi, val.x, v); better(bv, bi, val.y, v + 1); better(bv, bi, val.z, v + 2); better(bv, bi, val.w, v + 3);
  }
  block_argmax(bv, bi, shv, shi);
  if (threadIdx.x == 0) {
    int best = bi == INT_MAX ? 0 : bi;
    if (tp.node_argmax && tapped) tp.node_argmax[slot] = best;
    if (tp.forced_node_argmax && tapped) best = tp.forced_node_argmax[slot];
    g[r] = best;
  }
}

hipError_t launch_row_argmax(const Dims& D, const RowMap& rm, const float* part, int S, size_t pstride, int* g,
                             const cerberus_taps& tp, int rows_max, hipStream_t s) {
  hipLaunchKernelGGL(k_row_argmax, dim3(rows_max), dim3(1024), 0, s, part, S, pstride, g, tp, rm, D.V, D.T);
  return hipGetLastError();
}

// ---------------------------------------------------------------------------------------------
// Acceptance (tree verification's outcome): walk down from the root while a child carries the
// token the base model itself produced at the current node; lowest child index on duplicates.
// One wave per sequence; the walk is at most Hc levels.
// ---------------------------------------------------------------------------------------------
__global__ __launch_bounds__(64) void k_accept(const Dims D, const TreeDev tr, const RowMap rm, const int* __restrict__ g,
                                               const int* __restrict__ tok, const cerberus_state st, int* __restrict__ path,
                                               int* __restrict__ last_row, int batch) {
  // one wave per sequence: at every level the 64 lanes test 64 candidate children at once and the
  // lowest matching node index wins (ballot), so a level costs one pass over the tree's nodes
  const int b = blockIdx.x, lane = threadIdx.x;
  const int Tb = rm.seq_T[b];
  if (Tb <= 0) {
    if (lane == 0) { st.accept_len[b] = 0; last_row[b] = -1; }
    return;
  }
  const int row0 = rm.seq_row0[b], W = D.Hc + 1;
  int cur = 0, a = 1, mine = 0;   // lane j keeps the j-th node of the path
  while (a < W) {
    const int want = g[row0 + cur];
    int nxt = -1;
    for (int c0 = cur + 1; c0 < Tb && nxt < 0; c0 += 64) {
      const int c = c0 + lane;
      const bool hit = c < Tb && tr.parent[c] == cur && tok[row0 + c] == want;
      const unsigned long long m = __ballot(hit);
      if (m) nxt = c0 + __ffsll((long long)m) - 1;
    }
    if (nxt < 0) break;
    if (lane == a) mine = nxt;
    ++a;
    cur = nxt;
  }
  if (lane < a) {
    path[b * W + lane] = mine;
    st.accepted_nodes[b * W + lane] = mine;
    st.accepted_tokens[b * W + lane] = tok[row0 + mine];
  }
  if (lane == 0) {
    st.accept_len[b] = a;
    st.root_token[b] = g[row0 + cur];
    st.kv_len[b] = rm.seq_L[b] + a;
    last_row[b] = row0 + cur;
  }
}

hipError_t launch_accept(const Dims& D, const TreeDev& tr, const RowMap& rm, const int* g, const int* tok,
                         const cerberus_state& st, int* path, int* last_row, int batch, hipStream_t s) {
  hipLaunchKernelGGL(k_accept, dim3(batch), dim3(64), 0, s, D, tr, rm, g, tok, st, path, last_row, batch);
  return hipGetLastError();
}

// ---------------------------------------------------------------------------------------------
// KV compaction: cache row L + path[j] -> row L + j for j = 1..a-1, in every layer, K and V, head.
// A workgroup owns one (layer, K|V, head) slice; thread (t, j) moves the t-th 16-byte piece of source
// row j.  A source row of one copy can be the destination of another (path[1] = 3 and j = 3), so
// every thread first loads its piece into a register, the whole workgroup waits for those loads and
// meets at a barrier, and only then are the pieces stored: no store can overtake a load.
// ---------------------------------------------------------------------------------------------
__global__ __launch_bounds__(512) void k_compact(const Dims D, const RowMap rm, const cerberus_state st,
                                                 const int* __restrict__ path, int elem_bytes) {
  const int lk = blockIdx.x, h = blockIdx.y, b = blockIdx.z;
  const int a = st.accept_len[b];
  if (a <= 1) return;                       // uniform over the workgroup
  const int pieces = D.dh * elem_bytes / 16;
  const int t = threadIdx.x, j = threadIdx.y + 1;
  const bool active = t < pieces && j < a;
  const int L = rm.seq_L[b], W = D.Hc + 1;
  const size_t row_bytes = (size_t)D.dh * elem_bytes;
  unsigned char* base = reinterpret_cast<unsigned char*>(st.kv) + (((size_t)lk * D.Bmax + b) * D.nH + h) * D.cap * row_bytes;
  uint4 v = make_uint4(0, 0, 0, 0);
  if (active) v = reinterpret_cast<const uint4*>(base + (size_t)(L + path[b * W + j]) * row_bytes)[t];
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");   // the row is in registers before anyone stores
  __syncthreads();
  if (active) reinterpret_cast<uint4*>(base + (size_t)(L + j) * row_bytes)[t] = v;
}

hipError_t launch_compact(const Dims& D, const RowMap& rm, const cerberus_state& st, const int* path, int batch,
                          hipStream_t s) {
  hipLaunchKernelGGL(k_compact, dim3(D.n_layers * 2, D.nH, batch), dim3(64, D.Hc), 0, s, D, rm, st, path,
                     D.dtype == 0 ? 4 : 2);
  return hipGetLastError();
}

// ---------------------------------------------------------------------------------------------
// Entropy gate (Section 4.2): P = softmax(h) over the d components of one hidden vector,
// S = -sum P log2 P = (ln Z - sum_i e_i z_i / Z) / ln 2 with z = h - max h, e = exp(z), Z = sum e.
// flag = 1 (auto-regressive) iff S > T; equality and only equality-or-below keeps the parallel
// path, and a NaN entropy takes the auto-regressive one.
// ---------------------------------------------------------------------------------------------
// One workgroup of 1024 threads per row keeps the row in registers (d <= 8192, d % 4 == 0): one pass
// over memory, one block-wide max and one block-wide sum of the three accumulators.
// With `hp`, the same launch also seeds the decoding heads: the row the gate looks at (the last
// accepted node's hidden state, Section 4.1) becomes the stage-0 state of every head, and where the
// first stage is the special block, [d..2d) of head i >= 1 as well (head i-1's state is the same
// vector there).  A sequence that sat the step out gets a zero state and no gate decision.
template <typename T>
__global__ __launch_bounds__(1024) void k_gate(int d, float threshold, const float* __restrict__ base,
                                               const int* __restrict__ row_index, const float* __restrict__ forced,
                                               const int* __restrict__ seq_T, float* __restrict__ entropy, int* __restrict__ flag,
                                               const HeadsPrep hp) {
  __shared__ float shf[16];
  __shared__ double shd[3][16];
  const int r = blockIdx.x;
  const bool sat_out = seq_T && seq_T[r] <= 0;
  const int ri = row_index ? row_index[r] : r;
  const float* hb = base + (size_t)max(ri, 0) * d;
  const float* h = forced ? forced + (size_t)r * d : hb;
  float4 v[2];
#pragma unroll
  for (int it = 0; it < 2; ++it) {
    const int c = (it * 1024 + threadIdx.x) * 4;
    v[it] = make_float4(-INFINITY, -INFINITY, -INFINITY, -INFINITY);
    if (c < d) {
      v[it] = *reinterpret_cast<const float4*>(h + c);
      if (hp.hsF) {
        float4 s = forced ? *reinterpret_cast<const float4*>(hb + c) : v[it];
        if (sat_out || ri < 0) s = make_float4(0.f, 0.f, 0.f, 0.f);
        const float e[4] = {s.x, s.y, s.z, s.w};
        const int ld = 2 * d;
        for (int i = 0; i < hp.Hc; ++i) {
          const size_t o = ((size_t)i * 16 + r) * ld + c;
          *reinterpret_cast<float4*>(hp.hsF + o) = s;
#pragma unroll
          for (int j = 0; j < 4; ++j) st_a(reinterpret_cast<T*>(hp.hsA) + o + j, hp.lo_off, e[j]);
          if (hp.sb == 0 && i >= 1) {
            *reinterpret_cast<float4*>(hp.hsF + o + d) = s;
#pragma unroll
            for (int j = 0; j < 4; ++j) st_a(reinterpret_cast<T*>(hp.hsA) + o + d + j, hp.lo_off, e[j]);
          }
        }
      }
    }
  }
  if (sat_out) return;   // uniform over the workgroup
  float m = fmaxf(fmaxf(fmaxf(v[0].x, v[0].y), fmaxf(v[0].z, v[0].w)), fmaxf(fmaxf(v[1].x, v[1].y), fmaxf(v[1].z, v[1].w)));
  m = block_max(m, shf);
  double Z = 0.0, A = 0.0, nbad = 0.0;
#pragma unroll
  for (int it = 0; it < 2; ++it) {
    const int c = (it * 1024 + threadIdx.x) * 4;
    if (c < d) {
      const float e4[4] = {v[it].x, v[it].y, v[it].z, v[it].w};
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        const float z = e4[j] - m;
        const float e = expf(z);
        Z += (double)e;
        if (e > 0.f) A += (double)e * (double)z;
        if (e4[j] != e4[j]) nbad += 1.0;
      }
    }
  }
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) {
    Z += __shfl_xor(Z, off, 64);
    A += __shfl_xor(A, off, 64);
    nbad += __shfl_xor(nbad, off, 64);
  }
  const int wave = threadIdx.x >> 6;
  __syncthreads();
  if ((threadIdx.x & 63) == 0) { shd[0][wave] = Z; shd[1][wave] = A; shd[2][wave] = nbad; }
  __syncthreads();
  if (threadIdx.x == 0) {
    Z = A = nbad = 0.0;
    for (int w = 0; w < 16; ++w) { Z += shd[0][w]; A += shd[1][w]; nbad += shd[2][w]; }
    double S = (log(Z) - A / Z) / 0.6931471805599453;
    if (nbad > 0.0) S = NAN;
    entropy[r] = (float)S;
    flag[r] = (S <= (double)threshold) ? 0 : 1;
  }
}

hipError_t launch_gate(int d, float threshold, const float* base, const int* row_index, const float* forced,
                       const int* seq_T, int rows, float* entropy, int* flag, const HeadsPrep& hp, int dtype, hipStream_t s) {
  if (dtype == 0)
    hipLaunchKernelGGL((k_gate<float>), dim3(rows), dim3(1024), 0, s, d, threshold, base, row_index, forced, seq_T, entropy, flag, hp);
  else
    hipLaunchKernelGGL((k_gate<bf16_t>), dim3(rows), dim3(1024), 0, s, d, threshold, base, row_index, forced, seq_T, entropy, flag, hp);
  return hipGetLastError();
}

// ---------------------------------------------------------------------------------------------
// Cerberus heads (Section 4.1).  State of head i before stage s lives in hsF/hsA[s & 1][i][b][0..w);
// where the coming stage is the special block, [d..2d) of head i holds head i-1's state, so the
// stage's GEMM simply sees the concatenation (own state first).
// ---------------------------------------------------------------------------------------------
// Resblock tail: Output = SiLU((W h + b) + h) from the GEMM partials of W h (Section 4.1).
template <typename T>
__global__ __launch_bounds__(256) void k_resblock_finish(const ResFinishArgs a, const float* __restrict__ curF,
                                                         float* __restrict__ nxtF, T* __restrict__ nxtA, size_t lo_off, int d,
                                                         int Hc, int link_next) {
  const int i = blockIdx.x, b = blockIdx.y;
  const int col = blockIdx.z * 256 + threadIdx.x;
  const int w = a.width[i], ld = 2 * d;
  if (col >= w) return;
  const size_t o = ((size_t)i * 16 + b) * ld + col;
  float v = a.bias[i][col] + curF[o];
  for (int s = 0; s < a.S[i]; ++s) v += a.part[i][s * a.pstride[i] + (size_t)b * w + col];
  v = v / (1.0f + expf(-v));
  nxtF[o] = v;
  st_a(nxtA + o, lo_off, v);
  if (link_next && i + 1 < Hc && col < d) {
    const size_t o2 = ((size_t)(i + 1) * 16 + b) * ld + d + col;
    nxtF[o2] = v;
    st_a(nxtA + o2, lo_off, v);
  }
}

hipError_t launch_resblock_finish(const Dims& D, const ResFinishArgs& a, const float* curF, float* nxtF, void* nxtA,
                                  int link_next, int batch, hipStream_t s) {
  dim3 grid(D.Hc, batch, (2 * D.d + 255) / 256);
  if (D.dtype == 0)
    hipLaunchKernelGGL((k_resblock_finish<float>), grid, dim3(256), 0, s, a, curF, nxtF, (float*)nxtA, (size_t)0, D.d, D.Hc, link_next);
  else
    hipLaunchKernelGGL((k_resblock_finish<bf16_t>), grid, dim3(256), 0, s, a, curF, nxtF, (bf16_t*)nxtA, (size_t)D.Hc * 16 * 2 * D.d, D.d, D.Hc, link_next);
  return hipGetLastError();
}

// ---------------------------------------------------------------------------------------------
// Per-head top-k (the heads' token candidates), in the order (value descending, id ascending).
// Two launches.  k_topk_slice: a workgroup owns 4096 consecutive vocabulary entries of one (head,
// sequence), four per thread.  Each wave lists the topk best of its 256 entries (a round is a
// wave-wide argmax over the lanes' best entries not taken yet, no barrier; only the winner's lane
// looks for its next one), the first wave merges the 16 sorted lists and writes the slice's list.
// k_topk_merge: one wave per (head, sequence) merges the slices' lists head by head.
// Sequences whose gate chose the auto-regressive step keep their old candidates.
// ---------------------------------------------------------------------------------------------
__device__ __forceinline__ void wave_argmax(float& bv, int& bi) {
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) {
    const float ov = __shfl_xor(bv, off, 64);
    const int oi = __shfl_xor(bi, off, 64);
    better(bv, bi, ov, oi);
  }
}

// Merge of n <= 64 lists sorted in the order, list w at lv/li[w * stride ..]: lane w walks list w;
// the best of the lists' heads is the next entry overall.  Calls out(r, id) on lane 0.
template <typename Out>
__device__ __forceinline__ void merge_lists(const float* lv, const int* li, int n, int stride, int topk, int lane, Out out) {
  int pos = 0;
  for (int r = 0; r < topk; ++r) {
    const bool live = (lane < n) & (pos < topk);
    const float hv = live ? lv[lane * stride + pos] : -INFINITY;
    const int hi = live ? li[lane * stride + pos] : INT_MAX;
    float bv = hv;
    int bi = hi;
    wave_argmax(bv, bi);
    if (lane == 0) out(r, bv, bi);
    if (live && hi == bi && bi != INT_MAX) ++pos;   // ids are unique: this lane's list held the winner
  }
}

__global__ __launch_bounds__(1024) void k_topk_slice(const TopkArgs a, const cerberus_state st, const cerberus_taps tp, int V, int Hc,
                                                     int B, int topk) {
  __shared__ float cv[16 * CERBERUS_MAX_TOPK];
  __shared__ int ci[16 * CERBERUS_MAX_TOPK];
  const int i = blockIdx.x, b = blockIdx.y, part = blockIdx.z;
  if (st.gate_flag[b] != 0 || a.seq_T[b] <= 0) return;
  const float* lg = a.logits[i] + (size_t)b * V;
  const int v0 = (part * 1024 + threadIdx.x) * 4;         // V % 4 == 0
  float e[4] = {-INFINITY, -INFINITY, -INFINITY, -INFINITY};
  if (v0 < V) {
    const float4 val = *reinterpret_cast<const float4*>(lg + v0);
    if (tp.head_logits) *reinterpret_cast<float4*>(tp.head_logits + ((size_t)b * Hc + i) * V + v0) = val;
    e[0] = val.x; e[1] = val.y; e[2] = val.z; e[3] = val.w;
  }
  // best of this lane's entries strictly after (pv, pi) in the order; (-inf, INT_MAX) if none
  auto scan = [&](float pv, int pi, float& lv, int& li) {
    lv = -INFINITY;
    li = INT_MAX;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const bool el = (v0 < V) & ((e[j] < pv) | ((e[j] == pv) & (v0 + j > pi)));
      better(lv, li, el ? e[j] : -INFINITY, el ? v0 + j : INT_MAX);
    }
  };
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  float lv;
  int li;
  scan(INFINITY, -1, lv, li);
  for (int r = 0; r < topk; ++r) {
    float bv = lv;
    int bi = li;
    wave_argmax(bv, bi);
    if (lane == 0) { cv[wave * topk + r] = bv; ci[wave * topk + r] = bi; }
    if (li == bi && bi != INT_MAX) scan(bv, bi, lv, li);
  }
  __syncthreads();
  if (wave != 0) return;
  float* pv = a.part_v + (((size_t)i * B + b) * TOPK_MAX_PARTS + part) * CERBERUS_MAX_TOPK;
  int* pi = a.part_i + (((size_t)i * B + b) * TOPK_MAX_PARTS + part) * CERBERUS_MAX_TOPK;
  merge_lists(cv, ci, 16, topk, topk, lane, [&](int r, float v, int id) { pv[r] = v; pi[r] = id; });
}

__global__ __launch_bounds__(64) void k_topk_merge(const TopkArgs a, const cerberus_state st, int Hc, int B, int topk, int parts) {
  const int i = blockIdx.x, b = blockIdx.y, lane = threadIdx.x;
  if (st.gate_flag[b] != 0 || a.seq_T[b] <= 0) return;
  const float* pv = a.part_v + ((size_t)i * B + b) * TOPK_MAX_PARTS * CERBERUS_MAX_TOPK;
  const int* pi = a.part_i + ((size_t)i * B + b) * TOPK_MAX_PARTS * CERBERUS_MAX_TOPK;
  int* cand = st.cand + ((size_t)b * Hc + i) * topk;
  merge_lists(pv, pi, parts, CERBERUS_MAX_TOPK, topk, lane, [&](int r, float, int id) { cand[r] = id == INT_MAX ? 0 : id; });
}

hipError_t launch_topk(const Dims& D, const TopkArgs& a, const cerberus_state& st, const cerberus_taps& tp, int batch,
                       hipStream_t s) {
  const int parts = (D.V + 4095) / 4096;   // V <= 65536
  hipLaunchKernelGGL(k_topk_slice, dim3(D.Hc, batch, parts), dim3(1024), 0, s, a, st, tp, D.V, D.Hc, D.Bmax, D.topk);
  hipLaunchKernelGGL(k_topk_merge, dim3(D.Hc, batch), dim3(64), 0, s, a, st, D.Hc, D.Bmax, D.topk, parts);
  return hipGetLastError();
}

// ---------------------------------------------------------------------------------------------
// Token log of the multi-step driver: append what the step committed (Algorithm 1 line 16).
// ---------------------------------------------------------------------------------------------
__global__ __launch_bounds__(64) void k_log_tokens(const cerberus_state st, int W, int batch, int* __restrict__ out,
                                                   int cap, int* __restrict__ count) {
  const int b = threadIdx.x;
  if (b >= batch) return;
  const int a = st.accept_len[b];      // 0 when the sequence sat the step out
  const int n0 = count[b];
  int n = n0;
  for (int j = 0; j < a; ++j) {
    if (n < cap) out[(size_t)b * cap + n++] = st.accepted_tokens[b * W + j];
  }
  if (n - n0 < a) atomicOr(st.status, (int)CERBERUS_DEV_LOG_FULL);
  count[b] = n;
}

hipError_t launch_log_tokens(const Dims& D, const cerberus_state& st, int batch, int* out, int cap, int* count,
                             hipStream_t s) {
  hipLaunchKernelGGL(k_log_tokens, dim3(1), dim3(64), 0, s, st, D.Hc + 1, batch, out, cap, count);
  return hipGetLastError();
}

// ---------------------------------------------------------------------------------------------
// init-time helpers
// ---------------------------------------------------------------------------------------------
template <typename T>
__global__ void k_to_f32(const T* __restrict__ in, float* __restrict__ out, int n) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) out[i] = ld_f(in + i);
}

hipError_t launch_to_f32(const void* in, float* out, int n, int dtype, hipStream_t s) {
  if (dtype == 0) hipLaunchKernelGGL((k_to_f32<float>), dim3((n + 255) / 256), dim3(256), 0, s, (const float*)in, out, n);
  else hipLaunchKernelGGL((k_to_f32<bf16_t>), dim3((n + 255) / 256), dim3(256), 0, s, (const bf16_t*)in, out, n);
  return hipGetLastError();
}

}  // namespace cerb
