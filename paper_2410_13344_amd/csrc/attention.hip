// Tree-masked attention of the verify step.  Row n of a sequence (a tree node) attends to every
// committed cache row 0..L-1 and to the tree rows L+m whose node m is n itself or an ancestor of n;
// the ancestor sets are bit masks, ceil(T / 64) words per node.  Tree attention is only named in the paper
// (Sections 1 and 5.1); this is the ancestor-mask reading, with position L + depth(n).
#include "common.h"

namespace cerb {

typedef short short4v __attribute__((ext_vector_type(4)));
typedef short4v __attribute__((address_space(3))) lds_short4v;

// ---------------------------------------------------------------------------------------------
// Plain kernel, any element type: one wave per (row, head), lanes over the head dimension, online
// softmax over the visible keys.  Used in fp32 reference mode and as a cross-check of the MFMA one.
// ---------------------------------------------------------------------------------------------
template <typename T, int EPL>
__global__ __launch_bounds__(64) void k_attn_simple(const AttnArgs a) {
  const int r = blockIdx.x, h = blockIdx.y;
  if (r >= *a.rm.n_rows) return;
  const int b = a.rm.row_seq[r], node = a.rm.row_node[r];
  const int L = a.rm.seq_L[b], Tb = a.rm.seq_T[b];
  const int dh = a.dh, lane = threadIdx.x;
  const unsigned long long* mask = a.anc + (size_t)node * a.aw;
  const T* q = reinterpret_cast<const T*>(a.q) + (size_t)r * a.nH * dh + h * dh;
  const T* Kb = reinterpret_cast<const T*>(a.kv) + ((size_t)(0 * a.Bmax + b) * a.nH + h) * a.cap * dh;
  const T* Vb = reinterpret_cast<const T*>(a.kv) + ((size_t)(1 * a.Bmax + b) * a.nH + h) * a.cap * dh;
  const float scale = rsqrtf((float)dh);
  float qv[EPL], o[EPL];
#pragma unroll
  for (int e = 0; e < EPL; ++e) {
    float qe = ld_f(q + lane + 64 * e);
    if (a.q_lo_off) qe += ld_f(q + a.q_lo_off + lane + 64 * e);
    qv[e] = qe * scale;
    o[e] = 0.f;
  }
  float m = -INFINITY, l = 0.f;
  const int row0 = a.rm.seq_row0[b];
  const T* Kt = reinterpret_cast<const T*>(a.ktree);
  const T* Vt = reinterpret_cast<const T*>(a.vtree);
  for (int p = 0; p < L + Tb; ++p) {
    if (p >= L && !((mask[(p - L) >> 6] >> ((p - L) & 63)) & 1ull)) continue;
    const bool side = Kt != nullptr && p >= L;    // this step's rows at hi + lo precision
    const size_t so = (size_t)(row0 + p - L) * a.nH * dh + h * dh;
    float kv[EPL], vv[EPL];
#pragma unroll
    for (int e = 0; e < EPL; ++e) {
      if (side) {
        kv[e] = ld_f(Kt + so + lane + 64 * e) + ld_f(Kt + a.q_lo_off + so + lane + 64 * e);
        vv[e] = ld_f(Vt + so + lane + 64 * e) + ld_f(Vt + a.q_lo_off + so + lane + 64 * e);
      } else {
        kv[e] = ld_f(Kb + (size_t)p * dh + lane + 64 * e);
        vv[e] = ld_f(Vb + (size_t)p * dh + lane + 64 * e);
      }
    }
    float s = 0.f;
#pragma unroll
    for (int e = 0; e < EPL; ++e) s += qv[e] * kv[e];
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) s += __shfl_xor(s, off, 64);
    const float mn = fmaxf(m, s);
    const float corr = expf(m - mn);   // first key: exp(-inf) = 0
    const float pw = expf(s - mn);
    l = l * corr + pw;
#pragma unroll
    for (int e = 0; e < EPL; ++e) o[e] = o[e] * corr + pw * vv[e];
    m = mn;
  }
  T* out = reinterpret_cast<T*>(a.out) + (size_t)r * a.nH * dh + h * dh;
#pragma unroll
  for (int e = 0; e < EPL; ++e) st_a(out + lane + 64 * e, a.out_lo_off, o[e] / l);
}

// ---------------------------------------------------------------------------------------------
// MFMA kernel (bf16).  Workgroup (chunk c, head h, sequence b) stages 128 keys of K and V in LDS
// (16-byte pieces XOR-swizzled by the key index, so neither the row-wise K reads nor the transposed
// V reads conflict), wave w takes query tile w (16 tree nodes).
//   S^T = K Q^T      A = K rows (keys), B = Q (queries)  -> lane: query lane%16, keys 4*(lane/16)+v
//   softmax stats per query: lane-local over its keys, then across the 4 lane groups
//   O^T = V^T P^T    B = P^T taken straight from the S^T accumulators: contraction slot (g, e) of a
//                    32-key block is key 4g+e (e<4) or 16+4g+e-4 (e>=4); A = V^T taken from the
//                    row-major LDS tile with transposing reads, in the same slot order.
// Writes unnormalised partial outputs with (max, sum) per query; k_attn_combine merges the chunks.
// ---------------------------------------------------------------------------------------------
template <int DH, int CK>   // CK: committed cache rows per workgroup, 128 or 256
__global__ __launch_bounds__(256) void k_attn_mfma(const AttnArgs a) {
  constexpr int PPR = DH / 8;   // 16-byte pieces per row
  constexpr int KS = DH / 32;
  constexpr int DT = DH / 16;
  constexpr int ROWB = DH * 2;
  __shared__ __attribute__((aligned(16))) unsigned char sK[CK * ROWB];
  __shared__ __attribute__((aligned(16))) unsigned char sV[CK * ROWB];

  const int h = blockIdx.y;
  const int qb_max = a.tc_max;                      // query blocks of 64 tree nodes, as many as tree chunks
  const int b = blockIdx.z / qb_max, qb = blockIdx.z % qb_max;
  const int L = a.rm.seq_L[b], Tb = a.rm.seq_T[b], row0 = a.rm.seq_row0[b];
  if (Tb <= 0 || qb * 64 >= Tb) return;
  // The last tc_max workgroups of a (head, sequence, query block) take the tree chunks: 64 of the
  // step's own rows each, read from the hi + lo side planes (LDS rows 0..63 = hi, 64..127 = lo of
  // the same key; rows 128.. stay unused when CK = 256).  The others take CK committed cache rows each.
  const int tci = (int)blockIdx.x - ((int)gridDim.x - a.tc_max);   // >= 0: index of the tree chunk
  const bool tree = tci >= 0;
  const int nprefix = (L + CK - 1) / CK;
  if (tree ? tci * 64 >= Tb : (int)blockIdx.x >= nprefix) return;
  const int c = tree ? nprefix + tci : blockIdx.x;  // partial slot
  const int key0 = c * CK;                          // first cache row of a prefix chunk

  // One source description for both kinds of chunk, so the staging below is straight-line code with
  // every global load (K, V and the wave's q fragments) issued before the first LDS write: a loop of
  // load-then-store pairs would pay one memory round trip per iteration.
  const bf16_t *Kb, *Vb;
  size_t rstride;
  int nvalid;                                      // rows of this chunk that exist
  if (tree) {
    Kb = reinterpret_cast<const bf16_t*>(a.ktree) + (size_t)(row0 + tci * 64) * a.nH * DH + h * DH;
    Vb = reinterpret_cast<const bf16_t*>(a.vtree) + (size_t)(row0 + tci * 64) * a.nH * DH + h * DH;
    rstride = (size_t)a.nH * DH;
    nvalid = min(64, Tb - tci * 64);
  } else {
    Kb = reinterpret_cast<const bf16_t*>(a.kv) + (((size_t)(0 * a.Bmax + b) * a.nH + h) * a.cap + key0) * DH;
    Vb = reinterpret_cast<const bf16_t*>(a.kv) + (((size_t)(1 * a.Bmax + b) * a.nH + h) * a.cap + key0) * DH;
    rstride = DH;
    nvalid = min(CK, L - key0);                    // >= 1: the block index is below ceil(L / CK)
  }
  const size_t lo_plane = tree ? a.q_lo_off : 0;   // LDS rows 64..127 of the tree chunk: lo halves of rows 0..63
  const int rmask = tree ? 63 : CK - 1;
  const int nkt = tree ? 8 : CK / 16;              // 16-key tiles in use (uniform)
  constexpr int NI = CK * PPR / 256;
  uint4 kk[NI], vv[NI];
#pragma unroll
  for (int it = 0; it < NI; ++it) {
    const int i = it * 256 + threadIdx.x;
    const int key = i / PPR, pc = i % PPR;
    const int m = key & rmask;
    const size_t off = (size_t)min(m, nvalid - 1) * rstride + ((key & 64 & ~rmask) ? lo_plane : 0);
    kk[it] = reinterpret_cast<const uint4*>(Kb + off)[pc];
    vv[it] = reinterpret_cast<const uint4*>(Vb + off)[pc];
  }

  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int lq = lane & 15, g = lane >> 4;
  const int qnode = qb * 64 + wave * 16 + lq;
  const bool qvalid = qnode < Tb;
  const bf16_t* qrow = reinterpret_cast<const bf16_t*>(a.q) + (size_t)(row0 + min(qnode, Tb - 1)) * (a.nH * DH) + h * DH;
  uint4 qf[KS], qfl[KS];   // hi and lo plane of q
#pragma unroll
  for (int ks = 0; ks < KS; ++ks) {
    qf[ks] = *reinterpret_cast<const uint4*>(qrow + ks * 32 + g * 8);
    qfl[ks] = *reinterpret_cast<const uint4*>(qrow + a.q_lo_off + ks * 32 + g * 8);
  }

  const unsigned long long amask = a.anc[(size_t)min(qnode, Tb - 1) * a.aw + max(tci, 0)] & (qvalid ? ~0ull : 0ull);

#pragma unroll
  for (int it = 0; it < NI; ++it) {
    const int i = it * 256 + threadIdx.x;
    const int key = i / PPR, pc = i % PPR;
    const unsigned ok = (((key & rmask) < nvalid) & (key < nkt * 16)) ? 0xffffffffu : 0u;   // rows that do not exist are staged as zeros
    const int sw = pc ^ (key & (PPR - 1));
    *reinterpret_cast<uint4*>(sK + key * ROWB + sw * 16) = make_uint4(kk[it].x & ok, kk[it].y & ok, kk[it].z & ok, kk[it].w & ok);
    *reinterpret_cast<uint4*>(sV + key * ROWB + sw * 16) = make_uint4(vv[it].x & ok, vv[it].y & ok, vv[it].z & ok, vv[it].w & ok);
  }
  __syncthreads();
  if (qb * 64 + wave * 16 >= Tb) return;
  const float scale = rsqrtf((float)DH);

  float s[CK / 16][4];
#pragma unroll
  for (int kt = 0; kt < CK / 16; ++kt) {
    f32x4_t acc = {0.f, 0.f, 0.f, 0.f};
    const int key = kt * 16 + lq;
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) {
      if (CK > 128 && kt >= nkt) break;
      const int sw = (ks * 4 + g) ^ (key & (PPR - 1));
      const uint4 kf = *reinterpret_cast<const uint4*>(sK + key * ROWB + sw * 16);
      acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8_t, kf), __builtin_bit_cast(bf16x8_t, qf[ks]),
                                                    acc, 0, 0, 0);
      acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8_t, kf), __builtin_bit_cast(bf16x8_t, qfl[ks]),
                                                    acc, 0, 0, 0);
    }
#pragma unroll
    for (int v = 0; v < 4; ++v) s[kt][v] = acc[v];
  }
  if (tree) {   // LDS rows 64.. hold the lo halves of keys 0..63: their products belong to the same scores
#pragma unroll
    for (int kt = 0; kt < 4; ++kt)
#pragma unroll
      for (int v = 0; v < 4; ++v) s[kt][v] += s[kt + 4][v];
  }
  float m = -INFINITY;
#pragma unroll
  for (int kt = 0; kt < CK / 16; ++kt)
#pragma unroll
    for (int v = 0; v < 4; ++v) {
      const int kin = kt * 16 + 4 * g + v;   // key within the chunk
      const bool vis = tree ? (kt < 4 && ((amask >> (kin & 63)) & 1ull)) : (key0 + kin < L);
      s[kt][v] = (vis && qvalid) ? s[kt][v] * scale : -INFINITY;
      m = fmaxf(m, s[kt][v]);
    }
  m = fmaxf(m, __shfl_xor(m, 16, 64));
  m = fmaxf(m, __shfl_xor(m, 32, 64));
  const float msafe = (m == -INFINITY) ? 0.f : m;
  float lsum = 0.f;
#pragma unroll
  for (int kt = 0; kt < CK / 16; ++kt)
#pragma unroll
    for (int v = 0; v < 4; ++v) {
      const float p = __expf(s[kt][v] - msafe);   // masked: exp(-inf) = 0
      s[kt][v] = p;
      lsum += p;
    }
  lsum += __shfl_xor(lsum, 16, 64);
  lsum += __shfl_xor(lsum, 32, 64);
  if (tree) {   // the lo halves of the V rows take the same probabilities
#pragma unroll
    for (int kt = 0; kt < 4; ++kt)
#pragma unroll
      for (int v = 0; v < 4; ++v) s[kt + 4][v] = s[kt][v];
  }

  f32x4_t o[DT];
#pragma unroll
  for (int dt = 0; dt < DT; ++dt) o[dt] = f32x4_t{0.f, 0.f, 0.f, 0.f};
#pragma unroll
  for (int kp = 0; kp < CK / 32; ++kp) {
    if (CK > 128 && 2 * kp >= nkt) break;
    union { bf16_t u[8]; uint4 q; } pb, pl;   // probabilities as hi + lo bf16, like every GEMM input
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      pb.u[e] = f32_to_bf16(s[2 * kp][e]);
      pl.u[e] = f32_to_bf16(s[2 * kp][e] - bf16_to_f32(pb.u[e]));
      pb.u[4 + e] = f32_to_bf16(s[2 * kp + 1][e]);
      pl.u[4 + e] = f32_to_bf16(s[2 * kp + 1][e] - bf16_to_f32(pb.u[4 + e]));
    }
    // A operand = V^T: lane (dh = dt*16 + lq, group g) needs V[key][dh] for the 8 keys of its slots, a
    // column of the row-major LDS tile.  The transposing LDS read of gfx950 delivers exactly that: within
    // a group of 16 lanes, lane i receives element i % 4 of the 8-byte chunks that lanes 4j + i/4
    // (j = 0..3) point at (layout checked on the device).  So lane c of the group points at the four
    // dh values dt*16 + 4*(c%4) .. +3 of key 4g + c/4, and lane i gets keys 4g .. 4g+3 at dh dt*16 + i.
    const int keyA = kp * 32 + 4 * g + (lq >> 2), keyB = keyA + 16;
#pragma unroll
    for (int dt = 0; dt < DT; ++dt) {
      const int dh = dt * 16 + 4 * (lq & 3);
      const unsigned char* pa = sV + keyA * ROWB + (((dh >> 3) ^ (keyA & (PPR - 1))) * 16) + (dh & 7) * 2;
      const unsigned char* pb2 = sV + keyB * ROWB + (((dh >> 3) ^ (keyB & (PPR - 1))) * 16) + (dh & 7) * 2;
      union { short4v h[2]; uint4 q; } va;
      va.h[0] = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_short4v*)pa);
      va.h[1] = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_short4v*)pb2);
      o[dt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8_t, va.q), __builtin_bit_cast(bf16x8_t, pb.q),
                                                      o[dt], 0, 0, 0);
      o[dt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8_t, va.q), __builtin_bit_cast(bf16x8_t, pl.q),
                                                      o[dt], 0, 0, 0);
    }
  }

  if (qvalid) {
    const size_t slot = (((size_t)b * a.nH + h) * a.n_chunks_max + c) * a.Tpad + qnode;
    float* po = a.part_o + slot * DH;
#pragma unroll
    for (int dt = 0; dt < DT; ++dt)
      *reinterpret_cast<float4*>(po + dt * 16 + 4 * g) = make_float4(o[dt][0], o[dt][1], o[dt][2], o[dt][3]);
    if (g == 0) {
      a.part_ml[slot * 2 + 0] = m;
      a.part_ml[slot * 2 + 1] = lsum;
    }
  }
}

// Merges the chunk partials of one (row, head): out = sum_c w_c o_c / sum_c w_c l_c with
// w_c = exp(m_c - max m).  Chunks are taken eight at a time, all loads of a batch in flight together,
// with a running maximum between batches.
template <int DH>
__global__ __launch_bounds__(DH) void k_attn_combine(const AttnArgs a) {
  const int r = blockIdx.x, h = blockIdx.y, t = threadIdx.x;
  if (r >= *a.rm.n_rows) return;
  const int b = a.rm.row_seq[r], node = a.rm.row_node[r];
  const int nch = (a.rm.seq_L[b] + a.chunk - 1) / a.chunk + (a.rm.seq_T[b] + 63) / 64;   // committed-row chunks + tree chunks
  const size_t base = (((size_t)b * a.nH + h) * a.n_chunks_max) * a.Tpad + node;
  constexpr int NB = 8;
  float M = -INFINITY, num = 0.f, den = 0.f;
  for (int c0 = 0; c0 < nch; c0 += NB) {
    float mv[NB], lv[NB], ov[NB];
#pragma unroll
    for (int j = 0; j < NB; ++j) {
      const size_t slot = base + (size_t)min(c0 + j, nch - 1) * a.Tpad;
      const float2 ml = *reinterpret_cast<const float2*>(a.part_ml + slot * 2);
      mv[j] = ml.x;
      lv[j] = ml.y;
      ov[j] = a.part_o[slot * DH + t];
    }
    float Mn = M;
#pragma unroll
    for (int j = 0; j < NB; ++j) Mn = fmaxf(Mn, (c0 + j < nch) ? mv[j] : -INFINITY);
    // every query sees at least itself in the tree chunk, but a batch of fully masked chunks keeps M = -inf
    const float corr = (M == -INFINITY) ? 0.f : __expf(M - Mn);
    num *= corr;
    den *= corr;
#pragma unroll
    for (int j = 0; j < NB; ++j) {
      const float w = (c0 + j < nch && mv[j] != -INFINITY) ? __expf(mv[j] - Mn) : 0.f;
      den += w * lv[j];
      num += w * ov[j];
    }
    M = Mn;
  }
  st_a(reinterpret_cast<bf16_t*>(a.out) + (size_t)r * a.nH * DH + h * DH + t, a.out_lo_off, num / den);
}

hipError_t launch_attention(const AttnArgs& a, int dtype, int use_mfma, hipStream_t s) {
  if (dtype == 0 || !use_mfma) {
    dim3 grid(a.rows_max, a.nH);
    if (dtype == 0) {
      if (a.dh == 64) hipLaunchKernelGGL((k_attn_simple<float, 1>), grid, dim3(64), 0, s, a);
      else hipLaunchKernelGGL((k_attn_simple<float, 2>), grid, dim3(64), 0, s, a);
    } else {
      if (a.dh == 64) hipLaunchKernelGGL((k_attn_simple<bf16_t, 1>), grid, dim3(64), 0, s, a);
      else hipLaunchKernelGGL((k_attn_simple<bf16_t, 2>), grid, dim3(64), 0, s, a);
    }
    return hipGetLastError();
  }
  if (a.chunk != 128 && a.chunk != 256) return hipErrorInvalidValue;
  if (a.n_chunks_max != (a.cap + a.chunk - 1) / a.chunk + a.tc_max) return hipErrorInvalidValue;
  dim3 grid(a.n_chunks_max, a.nH, a.batch * a.tc_max);   // x: ceil(cap / chunk) prefix chunks, then tc_max tree chunks; z: (sequence, query block)
  dim3 cgrid(a.rows_max, a.nH);
  if (a.dh == 64) {
    if (a.chunk == 128) hipLaunchKernelGGL((k_attn_mfma<64, 128>), grid, dim3(256), 0, s, a);
    else hipLaunchKernelGGL((k_attn_mfma<64, 256>), grid, dim3(256), 0, s, a);
    hipLaunchKernelGGL((k_attn_combine<64>), cgrid, dim3(64), 0, s, a);
  } else {
    if (a.chunk == 128) hipLaunchKernelGGL((k_attn_mfma<128, 128>), grid, dim3(256), 0, s, a);
    else hipLaunchKernelGGL((k_attn_mfma<128, 256>), grid, dim3(256), 0, s, a);
    hipLaunchKernelGGL((k_attn_combine<128>), cgrid, dim3(128), 0, s, a);
  }
  return hipGetLastError();
}

}  // namespace cerb
