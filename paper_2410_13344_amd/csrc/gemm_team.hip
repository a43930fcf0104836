// GEMM for launches of more than 128 rows whose weights are wide (the gate/up projection): out[p] += A W^T, bf16
// hi + lo activation planes, pre-tiled bf16 weights, fp32 partial planes for the consumer to sum.
//
// One workgroup of 8 waves per CU.  The rows are cut into RB row blocks of at most 128 rows; a wave owns all
// 16 * NT rows of its workgroup's row block and 64 columns (NT x 4 accumulators), the 8 waves sit side by side: a
// workgroup tile is 512 columns.  The activation rows of a row block go global -> LDS by direct loads that land in
// MFMA fragment order (2 k-steps per stage, 4 stages), shared by the 8 waves; the weights go global -> registers
// through a ring of 4 k-steps that the wave issues and counts by hand.
//
// Work is dealt in units (column block, stage): teams of RB workgroups, one per row block, walk contiguous unit
// ranges of equal length, so the workgroups of a team stream the same weights at the same time (they sit on one
// XCD: the weights come from HBM once and from that L2 for the other row blocks) and every CU gets the same amount
// of work whatever the shape.  A column block that several teams touch lands in several partial planes
// out[p][row][col], p = the team's rank among the teams of that block; the team that finishes a block also clears
// the planes above the last one written there, so a consumer sums `planes` planes everywhere.
#include "common.h"

#include <algorithm>

namespace cerb {

namespace {

constexpr int kKC = 2;    // k-steps per stage
constexpr int kDST = 4;   // stages in LDS
constexpr int kRW = 4;    // weight ring slots (k-steps)
constexpr int kSPT = 32;  // slabs per workgroup tile (8 waves x 4)

__device__ __forceinline__ void team_dma16(const void* gptr, unsigned lds_addr) {
  asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, off" ::"s"(lds_addr), "v"(gptr) : "memory", "m0");
}
// 16 bytes per lane from a wave-uniform base.  The destination is an in/out operand on purpose: the register then
// stays reserved for its ring slot from one load to the next, also while a load whose value nobody will use (a
// clamped repeat at the end of a range) is in flight.  A destination the compiler believes dead would be handed
// to other values and overwritten when the data arrives.
__device__ __forceinline__ void team_wload(u32x4_t& d, unsigned voff, const void* sbase) {
  asm volatile("global_load_dwordx4 %0, %1, %2" : "+v"(d) : "v"(voff), "s"(sbase) : "memory");
}
// waits until at most N of this wave's loads are in flight; the slot's registers are operands so that nothing
// that reads them moves above the wait
template <int N>
__device__ __forceinline__ void team_wwait(u32x4_t (&w)[4]) {
  asm volatile("s_waitcnt vmcnt(%4)" : "+v"(w[0]), "+v"(w[1]), "+v"(w[2]), "+v"(w[3]) : "n"(N) : "memory");
}
__device__ __forceinline__ const char* uniform_ptr(const char* p) {
  const unsigned long v = reinterpret_cast<unsigned long>(p);
  const unsigned lo = __builtin_amdgcn_readfirstlane((unsigned)v), hi = __builtin_amdgcn_readfirstlane((unsigned)(v >> 32));
  return reinterpret_cast<const char*>(((unsigned long)hi << 32) | lo);
}

template <int NT>
__global__ __launch_bounds__(512) __attribute__((amdgpu_waves_per_eu(2, 2))) void k_gemm_team(const TeamGemmArgs a) {
  constexpr int NQ = (NT + 1) / 2;         // direct-to-LDS loads per wave and stage
  constexpr int SBQ = kKC * NT * 2 * 64;   // 16-byte pieces per stage buffer
  // loads of this wave that may still be in flight (they complete in issue order) when ... has landed.  Per stage a
  // wave issues, in this order: NQ direct loads (stage n + 3), 4 weight loads (k-step 2n + 3), 4 more (k-step 2n + 4).
  constexpr int N_DMA = 2 * NQ + 24;       // ... the fragments of stage n, at the top of stage n
  constexpr int N_W0 = 2 * NQ + 12;        // ... the weights of k-step 2n, after the issues before its products
  constexpr int N_W1 = NQ + 12;            // ... the weights of k-step 2n + 1
  extern __shared__ __attribute__((aligned(16))) u32x4_t team_lds[];
  const int rows = min(a.n_rows ? *a.n_rows : a.rows_static, a.rows_cap);
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), lane = threadIdx.x & 63;
  // The row count is known on the device only (the gate decides how many rows a sequence brings), so the row
  // blocks and teams are formed here, by the same rule the host used for its bound (team_shape): as few row
  // blocks as the NT row tiles of a workgroup allow, at least rb_min; the teams share the grid's workgroups.
  const int RB = max(a.rb_min, (rows + NT * 16 - 1) / (NT * 16));
  const int rows_per = ((rows + RB - 1) / RB + 15) / 16 * 16;
  const int nst = a.ksteps / kKC;
  const int nslab = a.N >> 4;
  const int CB = (nslab + kSPT - 1) / kSPT;
  const long long V = (long long)CB * nst;
  const int T = (int)min((long long)((int)gridDim.x / RB), V);
  // consecutive workgroup ids go to the 8 XCDs in turn: logical ids put a team's workgroups on one XCD
  const int G = gridDim.x;                 // a multiple of 8
  const int L = ((int)blockIdx.x & 7) * (G >> 3) + ((int)blockIdx.x >> 3);
  const int team = L / RB, rb = L - team * RB;
  if (team >= T) return;
  const int v0 = (int)(V * team / T), v1 = (int)(V * (team + 1) / T);
  const int len = v1 - v0;
  if (len <= 0) return;
  const int m0 = rb * rows_per, m1 = min(rows, m0 + rows_per);
  if (m0 >= m1) return;                    // (uniform over the workgroup: nobody is left at a barrier)
  const int nt_live = (m1 - m0 + 15) >> 4; // row tiles of this workgroup that hold rows

  int cb = v0 / nst, st = v0 - cb * nst;   // the unit being multiplied
  // rank of this team among the teams of its first column block; any later block starts inside this team's range
  int plane = team - ((int)((((long long)cb * nst + 1) * T + V - 1) / V) - 1);

  // ---- activations: fragment f = q * 8 + wave of a stage: row tile f >> 2, plane (f >> 1) & 1, k-step f & 1
  const unsigned lds_base = (unsigned)(unsigned long)((__attribute__((address_space(3))) const unsigned char*)team_lds);
  const int dp = (wave >> 1) & 1, dk = wave & 1;
  unsigned aoff[NQ];                       // element offset of this lane's 16 bytes at stage 0
  unsigned foff[NQ];                       // byte offset of the fragment in a stage buffer
#pragma unroll
  for (int q = 0; q < NQ; ++q) {
    const int i = min(q * 2 + (wave >> 2), NT - 1);              // (a clamped repeat rewrites the same bytes)
    const int r = min(m0 + i * 16 + (lane & 15), m1 - 1);
    aoff[q] = (unsigned)(dp * a.lo_off + (size_t)r * a.lda + dk * 32 + (lane >> 4) * 8);
    foff[q] = (unsigned)(((dk * NT + i) * 2 + dp) * 1024);
  }
  int sta = st, aissued = 0;               // issues past the range repeat its last stage: valid memory, never multiplied
#define TEAM_DMA_ISSUE(buf)                                                                                     \
  {                                                                                                             \
    _Pragma("unroll") for (int q = 0; q < NQ; ++q)                                                              \
      team_dma16(a.A + aoff[q] + sta * (kKC * 32), lds_base + (unsigned)(buf) * (SBQ * 16) + foff[q]);          \
    if (aissued + 1 < len) { ++aissued; sta = sta + 1 == nst ? 0 : sta + 1; }                                   \
  }

  // ---- weights: piece (slab, k-step) of the pre-tiled matrix is 1 KB at (slab * ksteps + ks) * 1024
  const unsigned wlane = lane * 16;
  const char* wsl[4];
  int cbw = cb, ksw = st * kKC, wissued = 0;
#define TEAM_W_BASES()                                                                                          \
  _Pragma("unroll") for (int j = 0; j < 4; ++j)                                                                 \
    wsl[j] = uniform_ptr(reinterpret_cast<const char*>(a.W) + ((size_t)min(cbw * kSPT + wave * 4 + j, nslab - 1) * a.ksteps) * 1024);
  TEAM_W_BASES()
  u32x4_t Wr[kRW][4];
#pragma unroll
  for (int r = 0; r < kRW; ++r)
#pragma unroll
    for (int j = 0; j < 4; ++j) Wr[r][j] = u32x4_t{0u, 0u, 0u, 0u};
#define TEAM_W_ISSUE(slot, advance)                                                                             \
  {                                                                                                             \
    _Pragma("unroll") for (int j = 0; j < 4; ++j) team_wload(Wr[slot][j], wlane, wsl[j] + (size_t)ksw * 1024);  \
    if ((advance) && wissued + 1 < len * kKC) {                                                                 \
      ++wissued;                                                                                                \
      if (++ksw >= a.ksteps) { ksw = 0; ++cbw; TEAM_W_BASES() }                                                 \
    }                                                                                                           \
  }

  f32x4_t acc[NT][4];
#pragma unroll
  for (int i = 0; i < NT; ++i)
#pragma unroll
    for (int j = 0; j < 4; ++j) acc[i][j] = f32x4_t{0.f, 0.f, 0.f, 0.f};

  // ---- what stages -3, -2, -1 would have issued, in their order (the three loads before k-step 0 repeat it)
  TEAM_DMA_ISSUE(0) TEAM_W_ISSUE(1, false) TEAM_W_ISSUE(2, false)
  TEAM_DMA_ISSUE(1) TEAM_W_ISSUE(3, false) TEAM_W_ISSUE(0, true)
  TEAM_DMA_ISSUE(2) TEAM_W_ISSUE(1, true) TEAM_W_ISSUE(2, true)

  const u32x4_t* ldsA = team_lds + lane;
#define TEAM_KSTEP(slot, sA)                                                                                    \
  {                                                                                                             \
    u32x4_t ah = (sA)[0], al = (sA)[64];                                                                        \
    _Pragma("unroll") for (int i = 0; i < NT; ++i) {                                                            \
      u32x4_t nh = ah, nl = al;                                                                                 \
      if (i + 1 < NT) { nh = (sA)[((i + 1) * 2) * 64]; nl = (sA)[((i + 1) * 2 + 1) * 64]; }                     \
      if (i < nt_live) {                                                                                        \
        _Pragma("unroll") for (int j = 0; j < 4; ++j) {                                                         \
          acc[i][j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8_t, ah), __builtin_bit_cast(bf16x8_t, Wr[slot][j]), acc[i][j], 0, 0, 0); \
          acc[i][j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8_t, al), __builtin_bit_cast(bf16x8_t, Wr[slot][j]), acc[i][j], 0, 0, 0); \
        }                                                                                                       \
      }                                                                                                         \
      __builtin_amdgcn_sched_barrier(0);                                                                        \
      ah = nh; al = nl;                                                                                         \
    }                                                                                                           \
  }

  for (int n0 = 0; n0 < len; n0 += 2) {    // two stages per trip: the ring slots come out static
#pragma unroll
    for (int u = 0; u < 2; ++u) {
      const int n = n0 + u;
      if (n >= len) break;
      asm volatile("s_waitcnt vmcnt(%0)" ::"n"(N_DMA) : "memory");   // this wave's part of stage n has landed
      asm volatile("s_barrier" ::: "memory");                        // ... everyone's; and everyone is done with stage n - 1
      TEAM_DMA_ISSUE((n + 3) & 3)
      const u32x4_t* sbuf = ldsA + (n & 3) * SBQ;
      TEAM_W_ISSUE((u * 2 + 3) % kRW, true)
      team_wwait<N_W0>(Wr[(u * 2) % kRW]);
      TEAM_KSTEP((u * 2) % kRW, sbuf)
      TEAM_W_ISSUE((u * 2 + 4) % kRW, true)
      team_wwait<N_W1>(Wr[(u * 2 + 1) % kRW]);
      TEAM_KSTEP((u * 2 + 1) % kRW, sbuf + NT * 2 * 64)
      const bool tile_end = st == nst - 1;
      if (tile_end || n == len - 1) {
        // ---- this team's part of column block cb is complete: it goes to plane `plane`.  A lane holds rows
        // i*16 + (ln >> 4)*4 + v, column ln & 15 of slab j.
        int ln = lane;
        asm volatile("" : "+v"(ln));                                 // (keeps the address arithmetic inside this branch)
        const unsigned rowbase = (unsigned)(m0 + (ln >> 4) * 4) * (unsigned)a.N + (unsigned)(cb * kSPT + wave * 4) * 16 + (ln & 15);
        const int rlim = m1 - m0 - (ln >> 4) * 4;                    // rows i*16 + v below this are live for the lane
        const int jlim = min(4, nslab - (cb * kSPT + wave * 4));     // slabs of the wave that exist (<= 0: none)
        {
          float* o = a.out + (size_t)plane * a.out_rows * a.N;
#pragma unroll
          for (int j = 0; j < 4; ++j) {
            if (j >= jlim) continue;
#pragma unroll
            for (int i = 0; i < NT; ++i)
#pragma unroll
              for (int v = 0; v < 4; ++v)
                if (i * 16 + v < rlim) o[rowbase + (unsigned)((i * 16 + v) * a.N + j * 16)] = acc[i][j][v];
          }
        }
        if (tile_end) {   // the team that finishes a block clears the planes nobody writes there
          for (int pp = plane + 1; pp < a.P; ++pp) {
            float* o = a.out + (size_t)pp * a.out_rows * a.N;
#pragma unroll 1
            for (int j = 0; j < jlim; ++j)
#pragma unroll 1
              for (int r = 0; r < NT * 16; r += 16)
#pragma unroll
                for (int v = 0; v < 4; ++v)
                  if (r + v < rlim) o[rowbase + (unsigned)((r + v) * a.N + j * 16)] = 0.f;
          }
        }
#pragma unroll
        for (int i = 0; i < NT; ++i)
#pragma unroll
          for (int j = 0; j < 4; ++j) acc[i][j] = f32x4_t{0.f, 0.f, 0.f, 0.f};
        plane = 0;
      }
      if (tile_end) { st = 0; ++cb; } else { ++st; }
    }
  }
#undef TEAM_DMA_ISSUE
#undef TEAM_W_BASES
#undef TEAM_W_ISSUE
#undef TEAM_KSTEP
  // nothing of this wave is in flight any more when it ends (the ring registers stay reserved until here)
#pragma unroll
  for (int r = 0; r < kRW; ++r) team_wwait<0>(Wr[r]);
}

int team_of(long long v, int T, long long V) { return (int)(((v + 1) * T + V - 1) / V) - 1; }

template <int NT>
hipError_t size_nt() {   // the kernel takes more than the default 64 KB of LDS
  return hipFuncSetAttribute((const void*)k_gemm_team<NT>, hipFuncAttributeMaxDynamicSharedMemorySize, kDST * kKC * NT * 2 * 1024);
}
template <int NT>
hipError_t launch_nt(const TeamGemmArgs& a, int grid, hipStream_t s) {
  hipLaunchKernelGGL((k_gemm_team<NT>), dim3(grid), dim3(512), kDST * kKC * NT * 2 * 1024, s, a);
  return hipGetLastError();
}

}  // namespace

// The shape a launch takes for `rows` rows with NT row tiles per workgroup on `cus` workgroups (the kernel forms the
// same on the device): row blocks, rows per block, teams, partial planes.
static void team_shape(int rows, int NT, int rb_min, int N, int Kpad, int cus, int* RB, int* rows_per, int* T, int* planes) {
  *RB = std::max(rb_min, (rows + NT * 16 - 1) / (NT * 16));
  *rows_per = ((rows + *RB - 1) / *RB + 15) / 16 * 16;
  const int nst = Kpad / 32 / kKC, CB = (N / 16 + kSPT - 1) / kSPT;
  const long long V = (long long)CB * nst;
  *T = (int)std::min<long long>(cus / *RB, V);
  *planes = 1;
  if (*T < 1) return;
  for (int c = 0; c < CB; ++c)
    *planes = std::max(*planes, team_of((long long)c * nst + nst - 1, *T, V) - team_of((long long)c * nst, *T, V) + 1);
}

// Plan for a launch of up to rows_max rows on `cus` compute units (a multiple of 8): the row tiles per workgroup and
// the number of partial planes a consumer has to sum whatever the row count turns out to be; false where the kernel
// does not apply (few rows, a shape it cannot tile, more planes than max_planes).
bool plan_team_gemm(int rows_max, int N, int Kpad, int cus, int max_planes, TeamPlan* tp) {
  if (rows_max <= 128 || N % 16 != 0 || Kpad % (32 * kKC) != 0 || cus < 8 || cus % 8 != 0) return false;
  const int RBmax = (rows_max + 127) / 128;
  const int NT = (((rows_max + RBmax - 1) / RBmax) + 15) / 16;
  if (NT < 5 || NT > 8 || cus / RBmax < 1) return false;      // (NT < 5 cannot happen above 128 rows)
  // the planes depend on the teams only, and the teams on the row blocks: every count the device may choose
  // fewer row blocks mean more teams and more planes: small row counts keep nearly as many row blocks as the bound
  const int rb_min = std::max(2, RBmax - 1);
  int planes = 1;
  for (int RB = rb_min; RB <= std::max(rb_min, (rows_max + NT * 16 - 1) / (NT * 16)); ++RB) {
    int rb, rp, T, pl;
    team_shape(RB * NT * 16, NT, rb_min, N, Kpad, cus, &rb, &rp, &T, &pl);
    if (T < 1) return false;
    planes = std::max(planes, pl);
  }
  if (planes > max_planes) return false;
  tp->NT = NT; tp->planes = planes; tp->grid = cus; tp->rb_min = rb_min;
  team_shape(rows_max, NT, rb_min, N, Kpad, cus, &tp->RB, &tp->rows_per, &tp->T, &planes);   // (the shape at the bound, for reference)
  return true;
}

// once per process, before the first launch (not a stream operation: kept out of any capture)
hipError_t init_team_gemm() {
  hipError_t e = size_nt<5>();
  if (e == hipSuccess) e = size_nt<6>();
  if (e == hipSuccess) e = size_nt<7>();
  if (e == hipSuccess) e = size_nt<8>();
  return e;
}

hipError_t launch_team_gemm(const TeamGemmArgs& a, const TeamPlan& tp, hipStream_t s) {
  switch (tp.NT) {
    case 5: return launch_nt<5>(a, tp.grid, s);
    case 6: return launch_nt<6>(a, tp.grid, s);
    case 7: return launch_nt<7>(a, tp.grid, s);
    case 8: return launch_nt<8>(a, tp.grid, s);
    default: return hipErrorInvalidValue;
  }
}

}  // namespace cerb
