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
// MFMA kernel (bf16).  A workgroup takes one item of the step's work list for one head and one block of
// 64 queries: either a range of one sequence's committed cache rows, walked in stages of 64 rows with a
// running softmax, or 64 of the step's own rows (a tree chunk: its hi plane is one stage, its lo plane
// the other, and both feed one softmax).  Wave w takes query tile w (16 tree nodes).
//
// Staging: LDS holds two stages of K and of V (rows 0..63 and 64..127 of a 128-row tile each).  The rows
// go from global memory straight into LDS (16 bytes per lane, a wave instruction fills 1 KB of LDS in lane
// order), so no registers are tied up and the load of stage s+2 is in flight while stage s+1 is
// multiplied.  A row's 16-byte pieces sit XOR-swizzled by the row index (neither the row-wise K reads
// nor the transposed V reads conflict); the swizzle is applied on the global side, by the choice of the
// piece a lane asks for.  Rows past the end of a ragged stage are re-reads of its last row: finite
// values whose scores are masked.
//   S^T = K Q^T      A = K rows (keys), B = Q (queries)  -> lane: query lane%16, keys 4*(lane/16)+v
//   softmax stats per query: lane-local over its keys, then across the 4 lane groups
//   O^T = V^T P^T    B = P^T taken straight from the S^T accumulators: contraction slot (g, e) of a
//                    32-key block is key 4g+e (e<4) or 16+4g+e-4 (e>=4); A = V^T taken from the
//                    row-major LDS tile with transposing reads, in the same slot order.
// Writes one unnormalised partial output with (max, sum) per query and item; k_attn_combine merges the
// items of a sequence.  The list is sized by the sequences' present lengths, so a launch over a large,
// mostly empty cache starts few workgroups that find nothing to do, and a long cache costs one partial
// per range instead of one per chunk.
// ---------------------------------------------------------------------------------------------
// Direct global -> LDS load, 16 bytes per lane: lane l of the wave writes LDS bytes lds_base + 16*l .. +15
// (lds_base uniform over the wave; lane layout checked on the device).  Written as inline assembly on purpose:
// for the builtin form the compiler waits for every such load in flight before any later LDS read, which would
// take the next stage's loads out of the shadow of this stage's arithmetic.  The kernel counts these loads
// itself (s_waitcnt vmcnt); the compiler's own counts for the loads it knows stay safe, because the counter
// retires in order and extra loads in flight only make its waits longer.
__device__ __forceinline__ void lds_dma16(const void* gptr, unsigned lds_base) {
  asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, off" ::"s"(lds_base), "v"(gptr) : "memory", "m0");
}
__device__ __forceinline__ unsigned lds_offset_of(const void* p) {
  return (unsigned)(unsigned long)((__attribute__((address_space(3))) const unsigned char*)p);
}
__device__ __forceinline__ void wg_barrier() {
  __syncthreads();
}

template <int DH>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(2))) void k_attn_mfma(const AttnArgs a) {
  constexpr int PPR = DH / 8;     // 16-byte pieces per row
  constexpr int KS = DH / 32;
  constexpr int DT = DH / 16;
  constexpr int ROWB = DH * 2;
  constexpr int RPI = 64 / PPR;   // rows a wave instruction of the staging covers
  constexpr int NI = PPR / 4;     // staging instructions per thread, stage and matrix
  __shared__ __attribute__((aligned(16))) unsigned char sK[128 * ROWB];
  __shared__ __attribute__((aligned(16))) unsigned char sV[128 * ROWB];

  const int h = blockIdx.y, qb = blockIdx.z;        // head; block of 64 queries
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int lq = lane & 15, g = lane >> 4;
  const int st_row = lane / PPR, st_sw = lane % PPR;   // staging: row within the instruction's rows, LDS piece slot
  const float scale = rsqrtf((float)DH);
  const unsigned sK_base = lds_offset_of(sK), sV_base = lds_offset_of(sV);

  for (int item = blockIdx.x; item < a.att_cap; item += gridDim.x) {   // the grid covers the list; the stride is a safety net
    const int4 e = a.rm.att_item[item];
    if (e.x < 0) break;                               // end of the list (uniform)
    const int b = e.x >> 16, j = e.x & 0xffff;
    const int L = e.y, Tb = e.z >> 16, row0 = e.z & 0xffff;
    const int npi = e.w >> 16, cps = e.w & 0xffff;
    if (qb * 64 >= Tb) continue;                      // uniform over the workgroup
    // Items npi.. of a sequence are its tree chunks.
    const bool tree = j >= npi;
    const int tci = tree ? j - npi : 0;
    const int k_begin = tree ? 0 : j * cps * a.chunk;                  // first cache row of a cache-range item
    const int k_end = tree ? 0 : min(L, k_begin + cps * a.chunk);
    const int ns = tree ? 2 : (k_end - k_begin + 63) / 64;             // stages (>= 1)
    const bool wave_live = qb * 64 + wave * 16 < Tb;

    const int qnode = qb * 64 + wave * 16 + lq;
    const bool qvalid = qnode < Tb;
    const bf16_t* qrow = reinterpret_cast<const bf16_t*>(a.q) + (size_t)(row0 + min(qnode, Tb - 1)) * (a.nH * DH) + h * DH;
    uint4 qf[KS], qfl[KS];   // hi and lo plane of q
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) {
      qf[ks] = *reinterpret_cast<const uint4*>(qrow + ks * 32 + g * 8);
      qfl[ks] = *reinterpret_cast<const uint4*>(qrow + a.q_lo_off + ks * 32 + g * 8);
    }
    const unsigned long long amask = a.anc[(size_t)min(qnode, Tb - 1) * a.aw + tci] & (qvalid ? ~0ull : 0ull);

    // stage `si` of the item -> LDS rows 64*buf .. 64*buf+63
    const bf16_t* Kc = reinterpret_cast<const bf16_t*>(a.kv) + (((size_t)(0 * a.Bmax + b) * a.nH + h) * a.cap) * DH;
    const bf16_t* Vc = reinterpret_cast<const bf16_t*>(a.kv) + (((size_t)(1 * a.Bmax + b) * a.nH + h) * a.cap) * DH;
    const bf16_t* Kt = reinterpret_cast<const bf16_t*>(a.ktree) + (size_t)(row0 + tci * 64) * a.nH * DH + h * DH;
    const bf16_t* Vt = reinterpret_cast<const bf16_t*>(a.vtree) + (size_t)(row0 + tci * 64) * a.nH * DH + h * DH;
    auto issue = [&](int si, int buf) {
      const bf16_t *Kb, *Vb;
      size_t rstride;
      int nvalid;                                    // rows of this stage that exist (>= 1)
      if (tree) {
        Kb = Kt + (si ? a.q_lo_off : 0);
        Vb = Vt + (si ? a.q_lo_off : 0);
        rstride = (size_t)a.nH * DH;
        nvalid = min(64, Tb - tci * 64);
      } else {
        const int key0 = k_begin + si * 64;
        Kb = Kc + (size_t)key0 * DH;
        Vb = Vc + (size_t)key0 * DH;
        rstride = DH;
        nvalid = min(64, k_end - key0);
      }
#pragma unroll
      for (int it = 0; it < NI; ++it) {
        const int r0 = (it * 4 + wave) * RPI;        // first row of the wave's instruction (uniform over the wave)
        const int r = r0 + st_row;
        const size_t off = (size_t)min(r, nvalid - 1) * rstride + (size_t)((st_sw ^ (r & (PPR - 1))) * 8);
        const unsigned lds_off = __builtin_amdgcn_readfirstlane((buf * 64 + r0) * ROWB);
        lds_dma16(Kb + off, sK_base + lds_off);
        lds_dma16(Vb + off, sV_base + lds_off);
      }
    };
    // S^T of the 64 keys of a stage, added to acc (4 key tiles)
    auto qk = [&](int buf, f32x4_t (&acc)[4]) {
#pragma unroll
      for (int kt = 0; kt < 4; ++kt) {
        const int key = buf * 64 + kt * 16 + lq;
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
          const int sw = (ks * 4 + g) ^ (key & (PPR - 1));
          const uint4 kf = *reinterpret_cast<const uint4*>(sK + key * ROWB + sw * 16);
          acc[kt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8_t, kf), __builtin_bit_cast(bf16x8_t, qf[ks]),
                                                            acc[kt], 0, 0, 0);
          acc[kt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8_t, kf), __builtin_bit_cast(bf16x8_t, qfl[ks]),
                                                            acc[kt], 0, 0, 0);
        }
      }
    };
    f32x4_t o[DT];
#pragma unroll
    for (int dt = 0; dt < DT; ++dt) o[dt] = f32x4_t{0.f, 0.f, 0.f, 0.f};
    // O^T += V^T P^T over the 64 keys of a stage; p holds the probabilities of the lane's keys
    auto pv = [&](int buf, const f32x4_t (&p)[4]) {
#pragma unroll
      for (int kp = 0; kp < 2; ++kp) {
        union { bf16_t u[8]; uint4 q; } pb, pl;   // probabilities as hi + lo bf16, like every GEMM input
#pragma unroll
        for (int e2 = 0; e2 < 4; ++e2) {
          pb.u[e2] = f32_to_bf16(p[2 * kp][e2]);
          pl.u[e2] = f32_to_bf16(p[2 * kp][e2] - bf16_to_f32(pb.u[e2]));
          pb.u[4 + e2] = f32_to_bf16(p[2 * kp + 1][e2]);
          pl.u[4 + e2] = f32_to_bf16(p[2 * kp + 1][e2] - bf16_to_f32(pb.u[4 + e2]));
        }
        // A operand = V^T: lane (dh = dt*16 + lq, group g) needs V[key][dh] for the 8 keys of its slots, a
        // column of the row-major LDS tile.  The transposing LDS read of gfx950 delivers exactly that: within
        // a group of 16 lanes, lane i receives element i % 4 of the 8-byte chunks that lanes 4j + i/4
        // (j = 0..3) point at (layout checked on the device).  So lane c of the group points at the four
        // dh values dt*16 + 4*(c%4) .. +3 of key 4g + c/4, and lane i gets keys 4g .. 4g+3 at dh dt*16 + i.
        const int keyA = buf * 64 + kp * 32 + 4 * g + (lq >> 2), keyB = keyA + 16;
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
    };

    float m_run = -INFINITY, l_run = 0.f;
    // masks the scores of 64 keys, folds them into the running softmax and leaves the probabilities in acc
    auto softmax_update = [&](f32x4_t (&acc)[4], int key0, bool first) {
      float m = -INFINITY;
#pragma unroll
      for (int kt = 0; kt < 4; ++kt)
#pragma unroll
        for (int v = 0; v < 4; ++v) {
          const int kin = kt * 16 + 4 * g + v;   // key within the stage
          const bool vis = tree ? (((amask >> kin) & 1ull) != 0) : (key0 + kin < L);
          acc[kt][v] = (vis && qvalid) ? acc[kt][v] * scale : -INFINITY;
          m = fmaxf(m, acc[kt][v]);
        }
      m = fmaxf(m, __shfl_xor(m, 16, 64));
      m = fmaxf(m, __shfl_xor(m, 32, 64));
      const float m_new = fmaxf(m_run, m);
      const float msafe = (m_new == -INFINITY) ? 0.f : m_new;
      const float corr = __expf(m_run - msafe);   // first stage: exp(-inf) = 0
      float lsum = 0.f;
#pragma unroll
      for (int kt = 0; kt < 4; ++kt)
#pragma unroll
        for (int v = 0; v < 4; ++v) {
          const float p = __expf(acc[kt][v] - msafe);   // masked: exp(-inf) = 0
          acc[kt][v] = p;
          lsum += p;
        }
      lsum += __shfl_xor(lsum, 16, 64);
      lsum += __shfl_xor(lsum, 32, 64);
      l_run = l_run * corr + lsum;
      m_run = m_new;
      if (!first) {
#pragma unroll
        for (int dt = 0; dt < DT; ++dt)
#pragma unroll
          for (int v = 0; v < 4; ++v) o[dt][v] *= corr;   // a lane's outputs all belong to its query lq
      }
    };

    // Loads in flight, oldest first: (q, mask,) stage s, stage s+1.  Waiting for stage s leaves the 2*NI
    // instructions of stage s+1 outstanding.
    issue(0, 0);
    if (ns > 1) issue(1, 1);
    // The compiler counts only the loads it knows (q and the mask).  Taking them as used here puts its wait for
    // them in front of the stage loop (it lets the first two stages land as well); left pending, they would be
    // waited for again in every round of the loop, with a count that also drains the stage just issued.
    typedef unsigned u32x4_t __attribute__((ext_vector_type(4)));
#pragma unroll
    for (int ks = 0; ks < KS; ++ks)
      asm volatile("" ::"v"(__builtin_bit_cast(u32x4_t, qf[ks])), "v"(__builtin_bit_cast(u32x4_t, qfl[ks])));
    asm volatile("" ::"v"(amask));
    if (tree) {
      asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
      wg_barrier();
      if (wave_live) {
        f32x4_t acc[4];
#pragma unroll
        for (int kt = 0; kt < 4; ++kt) acc[kt] = f32x4_t{0.f, 0.f, 0.f, 0.f};
        qk(0, acc);            // hi halves of the 64 keys
        qk(1, acc);            // lo halves: their products belong to the same scores
        softmax_update(acc, 0, true);
        pv(0, acc);
        pv(1, acc);            // the lo halves of the V rows take the same probabilities
      }
      wg_barrier();         // the tile is free for the next item
    } else {
      for (int si = 0; si < ns; ++si) {
        if (si + 1 < ns) {
          if (NI == 2) asm volatile("s_waitcnt vmcnt(4)" ::: "memory");
          else asm volatile("s_waitcnt vmcnt(8)" ::: "memory");
        } else {
          asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        }
        wg_barrier();       // every wave's part of stage si has landed
        if (wave_live) {
          f32x4_t acc[4];
#pragma unroll
          for (int kt = 0; kt < 4; ++kt) acc[kt] = f32x4_t{0.f, 0.f, 0.f, 0.f};
          qk(si & 1, acc);
          softmax_update(acc, k_begin + si * 64, si == 0);
          pv(si & 1, acc);
        }
        wg_barrier();       // stage si has been read by every wave: its rows can be refilled
        if (si + 2 < ns) issue(si + 2, si & 1);
      }
    }

    if (wave_live && qvalid) {
      const size_t slot = (((size_t)b * a.nH + h) * a.n_chunks_max + j) * a.Tpad + qnode;
      float* po = a.part_o + slot * DH;
#pragma unroll
      for (int dt = 0; dt < DT; ++dt)
        *reinterpret_cast<float4*>(po + dt * 16 + 4 * g) = make_float4(o[dt][0], o[dt][1], o[dt][2], o[dt][3]);
      if (g == 0) {
        a.part_ml[slot * 2 + 0] = m_run;
        a.part_ml[slot * 2 + 1] = l_run;
      }
    }
  }
}

// Merges the item partials of one (row, head): out = sum_c w_c o_c / sum_c w_c l_c with
// w_c = exp(m_c - max m).  Items are taken eight at a time, all loads of a batch in flight together,
// with a running maximum between batches.
template <int DH>
__global__ __launch_bounds__(DH) void k_attn_combine(const AttnArgs a) {
  const int r = blockIdx.x, h = blockIdx.y, t = threadIdx.x;
  if (r >= *a.rm.n_rows) return;
  const int b = a.rm.row_seq[r], node = a.rm.row_node[r];
  const int nch = a.rm.seq_npi[b] + (a.rm.seq_T[b] + 63) / 64;   // the sequence's cache-range items + tree chunks
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
  if (a.rm.att_item == nullptr || a.grid_x <= 0 || a.grid_x > a.att_cap) return hipErrorInvalidValue;
  dim3 grid(a.grid_x, a.nH, a.tc_max);   // x: items of the work list; z: block of 64 queries
  dim3 cgrid(a.rows_max, a.nH);
  if (a.dh == 64) {
    hipLaunchKernelGGL((k_attn_mfma<64>), grid, dim3(256), 0, s, a);
    hipLaunchKernelGGL((k_attn_combine<64>), cgrid, dim3(64), 0, s, a);
  } else {
    hipLaunchKernelGGL((k_attn_mfma<128>), grid, dim3(256), 0, s, a);
    hipLaunchKernelGGL((k_attn_combine<128>), cgrid, dim3(128), 0, s, a);
  }
  return hipGetLastError();
}

}  // namespace cerb
