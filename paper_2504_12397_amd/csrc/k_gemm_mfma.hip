// bf16 MFMA GEMM for gfx950:  C[M,N] = A[M,K] B[N,K]^T  (both operands K-contiguous, which is
// how activations [tokens, in] and weights [out, in] are stored).
//
// * v_mfma_f32_32x32x16_bf16.  Operand layout (checked on hardware): lane l feeds row l%32 with
//   the 8 consecutive k values 8*(l/32)..+7; accumulator register v of lane l is
//   C[8*(v/4) + 4*(l/32) + v%4][l%32].
// * Block tile BM x BN x 64, four waves, each WM x WN.  Tiles go global -> registers -> LDS with a
//   two-tile register prefetch and two LDS buffers (one barrier per k-tile).  LDS rows are 128 B
//   (8 chunks of 16 B); chunk c of row r sits at position c ^ ((r >> 1) & 7): LDS serves a
//   16-byte-per-lane access 16 lanes at a time over 64 banks, and with this swizzle 16 consecutive
//   rows of one chunk (operand reads) as well as 2 rows x 8 chunks (stores) hit 64 distinct banks.
// * Gated low-rank term of Eq.6 as extra k-steps BEFORE the main loop (or, when the reduction is split anyway, in
//   workgroups of its own that hold one more partial sum: its loads are two dependent round trips that would
//   otherwise make the workgroups of split 0 the last to finish): for every adapter present
//   in the row tile, A-operand = t = s*A_a x (as a bf16 pair hi + lo, zero for rows that are not
//   adapted by a), B-operand = B_{a,p} (twice).  Rows that are not adapted accumulate exact zeros into zero
//   accumulators, so their results are bitwise what a base-only call gives.
// * Epilogues: fp32 partial sums (split-K capable, summed later in a fixed order), bf16 store
//   (+ residual), SwiGLU (gate and up columns interleaved in 32-column blocks inside the tile).
#include <type_traits>

#include "mfma_kernels.h"

namespace alora {

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float f32x16;

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

__device__ __forceinline__ bf16x8 as_bf16x8(u32x4 u) { return __builtin_bit_cast(bf16x8, u); }

// PF = tiles kept in flight in registers (2: for the weight-streaming shapes; 1: for the large
// tiles whose accumulators leave no room for a second one).
// WEAVE: tile loads and LDS stores issued between the k-steps of the running tile (pays with many row tiles:
// operands come from L2 and two workgroups share a compute unit) instead of in blocks around them (better
// for weight streaming, where the loads want the longest time in flight).
// SEG: the reduction axis is cut into g.k_segments equal segments; the workgroup accumulates each from zero
// and adds the segment sums in ascending order in fp32 -- bit for bit what the split-reduction path
// (one segment per workgroup, partial sums added in the same order by the kernel that consumes them)
// produces, so a row's result does not depend on how many rows share the call.
template <int BM, int BN, int WM, int WN, int EPI, int PF, bool WEAVE = false, bool SEG = false>
__global__ __launch_bounds__(64 * (BM / WM) * (BN / WN))
// the woven 128x128 kernel is built for two workgroups per compute unit (two waves per SIMD): hold the
// register allocator to that also when the segment sums take 64 more registers
__attribute__((amdgpu_waves_per_eu((WEAVE && SEG) ? 2 : 1))) void gemm_mfma_kernel(GemmArgs g) {
  constexpr int BK = 64;
  constexpr int WAVES_N = BN / WN;
  constexpr int NT = 64 * (BM / WM) * WAVES_N;
  static_assert(NT == 128 || NT == 256 || NT == 512, "two, four or eight waves per block");
  constexpr int TM = WM / 32, TN = WN / 32;
  static_assert(EPI != GEMM_EPI_SWIGLU || TN % 2 == 0, "the SwiGLU epilogue pairs the 32-column blocks of a wave");
  constexpr int A_CHUNKS = BM * 8 / NT, B_CHUNKS = BN * 8 / NT;
  extern __shared__ u32x4 smem[];
  __shared__ unsigned long long s_present;
  u32x4 *As0 = smem, *Bs0 = smem + BM * 8, *As1 = smem + (BM + BN) * 8, *Bs1 = As1 + BM * 8;

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm0 = (wave / WAVES_N) * WM, wn0 = (wave % WAVES_N) * WN;
  const int M = g.M, N = g.N, K = g.K;
  // Workgroups are dealt round-robin to the 8 XCDs (each with its own L2): XCD x takes the
  // column tiles x, x+8, ... with all their row tiles and splits, so a weight tile is fetched
  // into one L2 only.  Few row tiles (weight streaming): row tile fastest, the row tiles that
  // share a weight tile run together.  Many row tiles: column tile fastest.
  const int tiles_m = (M + BM - 1) / BM, tiles_n = (N + BN - 1) / BN;
  const int per_xcd_n = (tiles_n + 7) / 8;
  const int xcd = blockIdx.x & 7;
  int q = blockIdx.x >> 3;
  int tm, nl;
  if (tiles_m <= 4) { tm = q % tiles_m; q /= tiles_m; nl = q % per_xcd_n; q /= per_xcd_n; }
  else { nl = q % per_xcd_n; q /= per_xcd_n; tm = q % tiles_m; q /= tiles_m; }
  const int split = q;
  const int tn = xcd + 8 * nl;
  if (tn >= tiles_n) return;
  const int m0 = tm * BM, n0 = tn * BN;
  // with lora_split the workgroups of split number k_splits carry only the low-rank term (no k-tiles)
  const bool lora_only = g.lora_split && split == g.k_splits;
  const int k_len = K / g.k_splits, k_beg = split * k_len, nk = lora_only ? 0 : k_len / BK;
  const int l32 = lane & 31, lhi = lane >> 5;

  f32x16 acc[TM][TN];
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;
  // running sum of the finished segments (SEG only)
  // (starts at +0: an accumulator that began at +0 is never -0, so 0 + p0 is p0 bit for bit)
  f32x16 tot[SEG ? TM : 1][SEG ? TN : 1];
  if constexpr (SEG) {
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
      for (int j = 0; j < TN; ++j)
#pragma unroll
        for (int v = 0; v < 16; ++v) tot[i][j][v] = 0.f;
  }
  const int seg_tiles = SEG ? nk / g.k_segments : 0;
  int seg_left = seg_tiles;       // k-tiles until the running segment ends
  // called after every k-tile: at a segment end the accumulators join the running sum and restart from zero
  auto segment_end = [&](int) {
    if constexpr (SEG) {
      if (--seg_left != 0) return;
      seg_left = seg_tiles;
#pragma unroll
      for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
          for (int v = 0; v < 16; ++v) {
            tot[i][j][v] += acc[i][j][v];
            acc[i][j][v] = 0.f;
          }
    }
  };

  // ---- main loop --------------------------------------------------------------------------
  // Two tiles are kept in flight in registers (R0, R1) on top of the one being consumed from
  // LDS: with HBM latency in the microseconds, a single prefetched tile leaves the loads exposed.
  u32x4 ra0[A_CHUNKS], rb0[B_CHUNKS], ra1[PF == 2 ? A_CHUNKS : 1], rb1[PF == 2 ? B_CHUNKS : 1];
  auto b_src_row = [&](int j) -> int {      // LDS row j of the B tile -> row of the weight matrix
    if (EPI == GEMM_EPI_SWIGLU) {
      int blk = j >> 5;
      int src = (n0 >> 1) + (blk >> 1) * 32 + (j & 31);
      return src < (N >> 1) ? src : (N >> 1) - 1;
    }
    int src = n0 + j;
    return src < N ? src : N - 1;
  };
  // loads / stores of a tile, chunk by chunk: part p of 4 takes the chunks i with i % 4 == p, so that the work
  // can be spread over the four k-steps of the tile being multiplied
  auto load_part = [&](int kt, int p, u32x4 (&ra)[A_CHUNKS], u32x4 (&rb)[B_CHUNKS]) {
    const int k0 = k_beg + kt * BK;
#pragma unroll
    for (int i = 0; i < A_CHUNKS; ++i) {
      if ((i & 3) != p) continue;
      int q2 = tid + i * NT, row = q2 >> 3, c = q2 & 7;
      int gr = m0 + row;
      gr = gr < M ? gr : M - 1;
      ra[i] = *reinterpret_cast<const u32x4 *>(g.A + (int64_t)gr * g.lda + k0 + c * 8);
    }
#pragma unroll
    for (int i = 0; i < B_CHUNKS; ++i) {
      if (((i + A_CHUNKS) & 3) != p) continue;
      int q2 = tid + i * NT, row = q2 >> 3, c = q2 & 7;
      const bf16 *base = g.B;
      if (EPI == GEMM_EPI_SWIGLU && ((row >> 5) & 1)) base = g.B2;
      rb[i] = *reinterpret_cast<const u32x4 *>(base + (int64_t)b_src_row(row) * g.ldb + k0 + c * 8);
    }
  };
  auto store_part = [&](u32x4 *As, u32x4 *Bs, int p, const u32x4 (&ra)[A_CHUNKS], const u32x4 (&rb)[B_CHUNKS]) {
#pragma unroll
    for (int i = 0; i < A_CHUNKS; ++i) {
      if ((i & 3) != p) continue;
      int q2 = tid + i * NT, row = q2 >> 3, c = q2 & 7;
      As[row * 8 + (c ^ ((row >> 1) & 7))] = ra[i];
    }
#pragma unroll
    for (int i = 0; i < B_CHUNKS; ++i) {
      if (((i + A_CHUNKS) & 3) != p) continue;
      int q2 = tid + i * NT, row = q2 >> 3, c = q2 & 7;
      Bs[row * 8 + (c ^ ((row >> 1) & 7))] = rb[i];
    }
  };
  auto load_tiles = [&](int kt, u32x4 (&ra)[A_CHUNKS], u32x4 (&rb)[B_CHUNKS]) {
#pragma unroll
    for (int p = 0; p < 4; ++p) load_part(kt, p, ra, rb);
  };
  auto store_tiles = [&](u32x4 *As, u32x4 *Bs, const u32x4 (&ra)[A_CHUNKS], const u32x4 (&rb)[B_CHUNKS]) {
#pragma unroll
    for (int p = 0; p < 4; ++p) store_part(As, Bs, p, ra, rb);
  };
  // One k-tile = four k-steps of 16.  The fragments of step ks+1 are read from LDS before the
  // MFMAs of step ks are issued, so the LDS latency hides behind matrix work.
  auto read_frags = [&](const u32x4 *As, const u32x4 *Bs, int ks, bf16x8 (&af)[TM], bf16x8 (&bfr)[TN]) {
    const int c = 2 * ks + lhi;
#pragma unroll
    for (int mi = 0; mi < TM; ++mi) {
      int row = wm0 + mi * 32 + l32;
      af[mi] = as_bf16x8(As[row * 8 + (c ^ ((row >> 1) & 7))]);
    }
#pragma unroll
    for (int ni = 0; ni < TN; ++ni) {
      int row = wn0 + ni * 32 + l32;
      bfr[ni] = as_bf16x8(Bs[row * 8 + (c ^ ((row >> 1) & 7))]);
    }
  };
  auto mma = [&](const bf16x8 (&af)[TM], const bf16x8 (&bfr)[TN]) {
#pragma unroll
    for (int mi = 0; mi < TM; ++mi)
#pragma unroll
      for (int ni = 0; ni < TN; ++ni)
        acc[mi][ni] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[mi], bfr[ni], acc[mi][ni], 0, 0, 0);
  };
  auto compute = [&](const u32x4 *As, const u32x4 *Bs) {
    bf16x8 a0[TM], b0[TN], a1[TM], b1[TN];
    read_frags(As, Bs, 0, a0, b0);
    read_frags(As, Bs, 1, a1, b1);
    mma(a0, b0);
    read_frags(As, Bs, 2, a0, b0);
    mma(a1, b1);
    read_frags(As, Bs, 3, a1, b1);
    mma(a0, b0);
    mma(a1, b1);
  };
  // The same with the tile traffic woven in: the loads of the tile two ahead (kt_load -> rl) and the LDS
  // stores of the next tile (rs -> An, Bn) are issued a quarter at a time between the four k-steps, fenced so
  // that the compiler keeps them there.  A workgroup often has a compute unit to itself (weight streaming,
  // one wave per SIMD): issued in a block before or after the MFMAs these instructions would leave the
  // matrix unit idle, here they run under it.
  auto compute_weave = [&](auto early, const u32x4 *As, const u32x4 *Bs, int kt_load, u32x4 (&rla)[A_CHUNKS],
                           u32x4 (&rlb)[B_CHUNKS], u32x4 *An, u32x4 *Bn, const u32x4 (&rsa)[A_CHUNKS],
                           const u32x4 (&rsb)[B_CHUNKS]) {
    // early: all loads of the tile two ahead go out before the first MFMA (weights streamed from HBM want the
    // longest possible time in flight), only the LDS stores are woven in; otherwise both are
    constexpr bool EARLY = decltype(early)::value;
    bf16x8 a0[TM], b0[TN], a1[TM], b1[TN];
    if (EARLY) load_tiles(kt_load, rla, rlb);
    read_frags(As, Bs, 0, a0, b0);
    read_frags(As, Bs, 1, a1, b1);
    if (!EARLY) load_part(kt_load, 0, rla, rlb);
    __builtin_amdgcn_sched_barrier(0);
    mma(a0, b0);
    read_frags(As, Bs, 2, a0, b0);
    if (!EARLY) load_part(kt_load, 1, rla, rlb);
    store_part(An, Bn, 0, rsa, rsb);
    __builtin_amdgcn_sched_barrier(0);
    mma(a1, b1);
    read_frags(As, Bs, 3, a1, b1);
    if (!EARLY) load_part(kt_load, 2, rla, rlb);
    store_part(An, Bn, 1, rsa, rsb);
    __builtin_amdgcn_sched_barrier(0);
    mma(a0, b0);
    if (!EARLY) load_part(kt_load, 3, rla, rlb);
    store_part(An, Bn, 2, rsa, rsb);
    __builtin_amdgcn_sched_barrier(0);
    mma(a1, b1);
    store_part(An, Bn, 3, rsa, rsb);
  };

  // The loop is free of conditional loads and stores (tile indices are clamped instead: the last
  // tile may be fetched and stored once more, into a buffer nobody reads again), so that the
  // compiler can count outstanding loads exactly and wait only for the tile it is about to store.
  if (nk > 0) {
    load_tiles(0, ra0, rb0);
    if constexpr (PF == 2) load_tiles(min(1, nk - 1), ra1, rb1);
  }

  // ---- gated low-rank extension (Eq.6), split 0 only --------------------------------------
  // (runs while the first two main-loop tiles are already on their way from memory; its own loads
  // are issued two k-steps at a time before the MFMAs that use them)
  if (g.tlow != nullptr && (g.lora_split ? lora_only : split == 0)) {
    // the adapters among this tile's rows: from the per-16-row masks the row preparation left (uniform
    // addresses, no barrier), else collected here from the rows' adapter ids
    unsigned long long present = 0ull;
    if (g.present16 != nullptr) {
      const int t_end = min((m0 + BM) / 16, (M + 15) / 16);
      for (int t = m0 / 16; t < t_end; ++t) present |= g.present16[t];
    } else {
      if (tid == 0) s_present = 0ull;
      __syncthreads();
      for (int r = tid; r < BM; r += NT) {
        int row = m0 + r;
        if (row < M) {
          int a = g.row_adapter[row];
          if (a >= 0) atomicOr(&s_present, 1ull << a);
        }
      }
      __syncthreads();
      present = s_present;
    }
    const int r = g.rank;
    int a_row[TM];
#pragma unroll
    for (int mi = 0; mi < TM; ++mi) {
      int row = m0 + wm0 + mi * 32 + l32;
      a_row[mi] = row < M ? g.row_adapter[row] : -1;
    }
    // per 32-column block: which part (q / k / v; gate / up; the only one) it belongs to, the row of the
    // up-matrix B it reads, and the distance between adapters in that matrix
    const int parts = g.lr_parts;
    int p_of[TN];
    const bf16 *brow[TN];
    int64_t a_stride[TN];
    bool col_ok[TN];
#pragma unroll
    for (int ni = 0; ni < TN; ++ni) {
      if (EPI == GEMM_EPI_SWIGLU) {
        // accumulator blocks alternate gate, up; both belong to column (n0 + wn0) / 2 + 32 (ni / 2) + l32 of act
        const int col = (n0 >> 1) + (wn0 >> 1) + (ni >> 1) * 32 + l32;
        p_of[ni] = ni & 1;
        col_ok[ni] = col < (N >> 1);
        const int cc = col_ok[ni] ? col : (N >> 1) - 1;
        brow[ni] = ((ni & 1) ? g.Bk : g.Bq) + (int64_t)cc * r;
        a_stride[ni] = (int64_t)(N >> 1) * r;
      } else {
        const int colb = n0 + wn0 + ni * 32, col = colb + l32;
        p_of[ni] = colb < g.n_q ? 0 : (colb < g.n_q + g.n_kv ? 1 : 2);
        col_ok[ni] = col < N;
        const int cc = col < N ? col : N - 1;
        if (cc < g.n_q) brow[ni] = g.Bq + (int64_t)cc * r;
        else if (cc < g.n_q + g.n_kv) brow[ni] = g.Bk + (int64_t)(cc - g.n_q) * r;
        else brow[ni] = g.Bv + (int64_t)(cc - g.n_q - g.n_kv) * r;
        a_stride[ni] = (int64_t)(p_of[ni] == 0 ? g.n_q : g.n_kv) * r;
      }
    }
    while (present) {
      const int a = __builtin_ctzll(present);
      present &= present - 1;
      constexpr int PB = TM * TN > 4 ? 1 : 2;         // k-steps whose loads are issued together
      for (int kb2 = 0; kb2 < 2 * r; kb2 += 16 * PB) {     // k runs over [t_hi | t_lo] against [B | B]
        u32x4 bu[PB][TN], au[PB][TM][TN];
#pragma unroll
        for (int h2 = 0; h2 < PB; ++h2) {
          const int ks2 = kb2 + 16 * h2;
          const bool live = ks2 < 2 * r;
          const int ks = ks2 < r ? ks2 : ks2 - r;
#pragma unroll
          for (int ni = 0; ni < TN; ++ni) {
            bu[h2][ni] = u32x4{0, 0, 0, 0};
            if (live && col_ok[ni])
              bu[h2][ni] = *reinterpret_cast<const u32x4 *>(brow[ni] + (int64_t)a * a_stride[ni] + ks + lhi * 8);
          }
#pragma unroll
          for (int mi = 0; mi < TM; ++mi) {
            // every row's t is requested (rows past the end: the last row's) and the rows of other adapters are
            // zeroed afterwards, so the request does not wait for the rows' adapter ids
            const int row = min(m0 + wm0 + mi * 32 + l32, M - 1);
#pragma unroll
            for (int ni = 0; ni < TN; ++ni) {
              au[h2][mi][ni] = u32x4{0, 0, 0, 0};
              if (live)
                au[h2][mi][ni] =
                    *reinterpret_cast<const u32x4 *>(g.tlow + ((int64_t)row * parts + p_of[ni]) * 2 * r + ks2 + lhi * 8);
            }
          }
        }
#pragma unroll
        for (int h2 = 0; h2 < PB; ++h2)
#pragma unroll
          for (int mi = 0; mi < TM; ++mi)
#pragma unroll
            for (int ni = 0; ni < TN; ++ni)
              if (a_row[mi] != a) au[h2][mi][ni] = u32x4{0, 0, 0, 0};
#pragma unroll
        for (int h2 = 0; h2 < PB; ++h2)
#pragma unroll
          for (int mi = 0; mi < TM; ++mi)
#pragma unroll
            for (int ni = 0; ni < TN; ++ni)
              acc[mi][ni] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(as_bf16x8(au[h2][mi][ni]), as_bf16x8(bu[h2][ni]),
                                                                    acc[mi][ni], 0, 0, 0);
      }
    }
  }

  if (nk > 0) store_tiles(As0, Bs0, ra0, rb0);
  __syncthreads();
  if constexpr (PF == 2) {
    if constexpr (WEAVE) {
      for (int kt = 0; kt < nk; kt += 2) {
        compute_weave(std::false_type{}, As0, Bs0, min(kt + 2, nk - 1), ra0, rb0, As1, Bs1, ra1, rb1);
        segment_end(kt + 1);
        __syncthreads();
        if (kt + 1 < nk) {
          compute_weave(std::false_type{}, As1, Bs1, min(kt + 3, nk - 1), ra1, rb1, As0, Bs0, ra0, rb0);
          segment_end(kt + 2);
        } else {
          load_tiles(nk - 1, ra1, rb1);
          store_tiles(As0, Bs0, ra0, rb0);
        }
        __syncthreads();
      }
    } else {
      for (int kt = 0; kt < nk; kt += 2) {
        load_tiles(min(kt + 2, nk - 1), ra0, rb0);
        compute(As0, Bs0);
        segment_end(kt + 1);
        store_tiles(As1, Bs1, ra1, rb1);
        __syncthreads();
        load_tiles(min(kt + 3, nk - 1), ra1, rb1);
        if (kt + 1 < nk) {
          compute(As1, Bs1);
          segment_end(kt + 2);
        }
        store_tiles(As0, Bs0, ra0, rb0);
        __syncthreads();
      }
    }
  } else {
    for (int kt = 0; kt < nk; ++kt) {
      u32x4 *Ac = (kt & 1) ? As1 : As0, *Bc = (kt & 1) ? Bs1 : Bs0;
      u32x4 *An = (kt & 1) ? As0 : As1, *Bn = (kt & 1) ? Bs0 : Bs1;
      load_tiles(min(kt + 1, nk - 1), ra0, rb0);
      compute(Ac, Bc);
      segment_end(kt + 1);
      store_tiles(An, Bn, ra0, rb0);
      __syncthreads();
    }
  }
  if constexpr (SEG) {      // the last segment has joined the sum: the epilogues read acc
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
      for (int j = 0; j < TN; ++j) acc[i][j] = tot[i][j];
  }

  // ---- epilogue ---------------------------------------------------------------------------
  if constexpr (EPI == GEMM_EPI_ROPE) {
    // The 128-column tile is one head.  The accumulators go to LDS as fp32 (the k-tiles are done with it), then
    // each wave takes 32 rows, a lane the rotation pair (c, c + 64): the same arithmetic, in the same order,
    // as the rotary kernel applies to the fp32 projection it reads from memory.
    static_assert(EPI != GEMM_EPI_ROPE || (BM == 128 && BN == 128 && NT == 256), "one head per tile, four waves");
    float *ys = reinterpret_cast<float *>(smem);       // [128][128]
    __syncthreads();
#pragma unroll
    for (int mi = 0; mi < TM; ++mi)
#pragma unroll
      for (int ni = 0; ni < TN; ++ni)
#pragma unroll
        for (int v = 0; v < 16; ++v)
          ys[(wm0 + mi * 32 + 8 * (v >> 2) + 4 * lhi + (v & 3)) * 128 + wn0 + ni * 32 + l32] = acc[mi][ni][v];
    __syncthreads();
    const int kind = n0 < g.n_q ? 0 : (n0 < g.n_q + g.n_kv ? 1 : 2);          // q, k or v head
    const int hcol = kind == 0 ? n0 : (kind == 1 ? n0 - g.n_q : n0 - g.n_q - g.n_kv);
    // lanes 0..31 take one row, lanes 32..63 the next; a lane the columns (2j, 2j+1) and their partners
    // (64 + 2j, 64 + 2j + 1): 4-byte stores, and the table entries of four row pairs are requested together
    const int my_row = m0 + wave * 32 + (lane & 31);
    const bool my_ok = my_row < M;
    const int my_pos = my_ok ? g.rope_pos[my_row] : 0;
    const int64_t my_slot = (my_ok && kind != 0) ? g.rope_slot[my_row] : 0;
    const float qs = kind == 0 ? g.q_scale : 1.0f;
    const int j2 = 2 * (lane & 31), half = lane >> 5;
    typedef __attribute__((__vector_size__(2 * sizeof(__bf16)))) __bf16 bf16x2_t;
    for (int r0 = 0; r0 < 32; r0 += 8) {
      if (m0 + wave * 32 + r0 >= M) break;
      float4 cs[4];
      int pos[4];
      int64_t slot[4];
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const int rr = r0 + 2 * i + half;
        pos[i] = __shfl(my_pos, rr, 64);
        slot[i] = ((int64_t)__shfl((int)(my_slot >> 32), rr, 64) << 32) | (uint32_t)__shfl((int)my_slot, rr, 64);
        cs[i] = make_float4(1.f, 0.f, 1.f, 0.f);
        if (kind != 2) cs[i] = *reinterpret_cast<const float4 *>(g.rope_table + (int64_t)pos[i] * 64 + j2);
      }
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const int rr = r0 + 2 * i + half, row = m0 + wave * 32 + rr;
        if (row >= M) continue;
        const float2 u = *reinterpret_cast<const float2 *>(ys + (wave * 32 + rr) * 128 + j2);
        const float2 w = *reinterpret_cast<const float2 *>(ys + (wave * 32 + rr) * 128 + 64 + j2);
        bf16 *dst = kind == 0 ? g.Qout + (int64_t)row * g.n_q + hcol
                              : (kind == 1 ? g.cacheK : g.cacheV) + slot[i] * g.n_kv + hcol;
        bf16x2_t lo, hi;
        if (kind == 2) {
          lo[0] = (bf16)u.x; lo[1] = (bf16)u.y;
          hi[0] = (bf16)w.x; hi[1] = (bf16)w.y;
        } else if (kind == 0 && g.q_half) {
          // queries as fp16 for the MFMA prefill attention kernel: same arithmetic, same two bytes per element
          typedef _Float16 half2_t __attribute__((ext_vector_type(2)));
          half2_t l2, h2;
          l2[0] = (_Float16)((u.x * cs[i].x - w.x * cs[i].y) * qs);
          l2[1] = (_Float16)((u.y * cs[i].z - w.y * cs[i].w) * qs);
          h2[0] = (_Float16)((w.x * cs[i].x + u.x * cs[i].y) * qs);
          h2[1] = (_Float16)((w.y * cs[i].z + u.y * cs[i].w) * qs);
          lo = __builtin_bit_cast(bf16x2_t, l2);
          hi = __builtin_bit_cast(bf16x2_t, h2);
        } else {
          lo[0] = (bf16)((u.x * cs[i].x - w.x * cs[i].y) * qs);
          lo[1] = (bf16)((u.y * cs[i].z - w.y * cs[i].w) * qs);
          hi[0] = (bf16)((w.x * cs[i].x + u.x * cs[i].y) * qs);
          hi[1] = (bf16)((w.y * cs[i].z + u.y * cs[i].w) * qs);
        }
        *reinterpret_cast<bf16x2_t *>(dst + j2) = lo;
        *reinterpret_cast<bf16x2_t *>(dst + 64 + j2) = hi;
      }
    }
    return;
  }
#pragma unroll
  for (int mi = 0; mi < TM; ++mi) {
#pragma unroll
    for (int v = 0; v < 16; ++v) {
      const int row = m0 + wm0 + mi * 32 + 8 * (v >> 2) + 4 * lhi + (v & 3);
      if (row >= M) continue;
      if (EPI == GEMM_EPI_SWIGLU) {
#pragma unroll
        for (int q = 0; q < TN / 2; ++q) {
          int col = (n0 >> 1) + (wn0 >> 1) + q * 32 + l32;
          if (col < (N >> 1)) {
            float gv = acc[mi][2 * q][v], uv = acc[mi][2 * q + 1][v];
            g.C[(int64_t)row * g.ldc + col] = (bf16)(gv / (1.0f + __expf(-gv)) * uv);
          }
        }
      } else {
#pragma unroll
        for (int ni = 0; ni < TN; ++ni) {
          int col = n0 + wn0 + ni * 32 + l32;
          if (col >= N) continue;
          float val = acc[mi][ni][v];
          if (EPI == GEMM_EPI_PARTIAL) {
            g.Cpart[((int64_t)split * M + row) * N + col] = val;
          } else {
            if (g.R) val += (float)g.R[(int64_t)row * g.ldc + col];
            g.C[(int64_t)row * g.ldc + col] = (bf16)val;
          }
        }
      }
    }
  }
}

template <int BM, int BN, int WM, int WN, int EPI, int PF = 2, bool WEAVE = false, bool SEG = false>
static void launch_cfg(const GemmArgs &g, hipStream_t s) {
  const int tiles_m = (g.M + BM - 1) / BM, tiles_n = (g.N + BN - 1) / BN;
  dim3 grid(8 * ((tiles_n + 7) / 8) * tiles_m * (g.k_splits + (g.lora_split ? 1 : 0)));
  size_t smem = (size_t)2 * (BM + BN) * 8 * sizeof(u32x4);
  auto kern = gemm_mfma_kernel<BM, BN, WM, WN, EPI, PF, WEAVE, SEG>;
  constexpr int NT = 64 * (BM / WM) * (BN / WN);
  // set on every launch: a host-side attribute write, safe from any thread and on any device
  (void)hipFuncSetAttribute((const void *)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
  hipLaunchKernelGGL(kern, grid, dim3(NT), smem, s, g);
}

// Sum of the partial sums of one group of four columns, in split order.  The first eight partials are requested
// together before any is added (a loop over a run-time count would take one memory round trip per split).
__device__ __forceinline__ float4 sum_partials(const float *__restrict__ p, int splits, int64_t stride) {
  float4 v[8];
#pragma unroll
  for (int sp = 0; sp < 8; ++sp)
    if (sp < splits) v[sp] = *reinterpret_cast<const float4 *>(p + (int64_t)sp * stride);
  float4 acc = v[0];
#pragma unroll
  for (int sp = 1; sp < 8; ++sp)
    if (sp < splits) { acc.x += v[sp].x; acc.y += v[sp].y; acc.z += v[sp].z; acc.w += v[sp].w; }
  for (int sp = 8; sp < splits; ++sp) {
    const float4 w = *reinterpret_cast<const float4 *>(p + (int64_t)sp * stride);
    acc.x += w.x; acc.y += w.y; acc.z += w.z; acc.w += w.w;
  }
  return acc;
}

typedef __attribute__((__vector_size__(4 * sizeof(__bf16)))) __bf16 bf16x4_t;
__device__ __forceinline__ float4 load_bf16x4(const bf16 *p) {
  const bf16x4_t r = *reinterpret_cast<const bf16x4_t *>(p);
  return make_float4((float)r[0], (float)r[1], (float)r[2], (float)r[3]);
}
__device__ __forceinline__ void store_bf16x4(bf16 *p, float a, float b, float c, float d) {
  bf16x4_t o;
  o[0] = (bf16)a; o[1] = (bf16)b; o[2] = (bf16)c; o[3] = (bf16)d;
  *reinterpret_cast<bf16x4_t *>(p) = o;
}

// C = bf16( sum over splits of partial sums (fixed order) + residual )
__global__ __launch_bounds__(256) void splitk_reduce_kernel(const float *__restrict__ part, int splits, int64_t mn,
                                                            const bf16 *__restrict__ R, bf16 *__restrict__ C) {
  const int64_t i = ((int64_t)blockIdx.x * 256 + threadIdx.x) * 4;
  if (i >= mn) return;
  float4 res = make_float4(0.f, 0.f, 0.f, 0.f);
  if (R != nullptr) res = load_bf16x4(R + i);
  float4 acc = sum_partials(part + i, splits, mn);
  acc.x += res.x; acc.y += res.y; acc.z += res.z; acc.w += res.w;
  store_bf16x4(C + i, acc.x, acc.y, acc.z, acc.w);
}

void launch_splitk_reduce(const float *part, int splits, int64_t mn, const bf16 *R, bf16 *C, hipStream_t s) {
  if (mn == 0) return;
  const int64_t threads = (mn + 3) / 4;
  hipLaunchKernelGGL(splitk_reduce_kernel, dim3((unsigned)((threads + 255) / 256)), dim3(256), 0, s, part, splits, mn,
                     R, C);
}

// The same sum for whole rows, followed by the RMSNorm of the row (h = sum + residual is normalised from its
// fp32 value): C = bf16(h), Cn = bf16(h * gain / rms(h)).  One workgroup per row, N <= 16384, N % 4 == 0.
__global__ __launch_bounds__(256) void splitk_reduce_norm_kernel(const float *__restrict__ part, int splits, int M,
                                                                 int N, const bf16 *__restrict__ R,
                                                                 const bf16 *__restrict__ gain, float eps,
                                                                 bf16 *__restrict__ C, bf16 *__restrict__ Cn) {
  __shared__ float s_red[4];
  const int row = blockIdx.x, tid = threadIdx.x;
  const int64_t mn = (int64_t)M * N, ro = (int64_t)row * N;
  float4 h[16], res[16];
  float ssq = 0.f;
#pragma unroll
  for (int u = 0; u < 16; ++u) {
    const int c = (u * 256 + tid) * 4;
    res[u] = make_float4(0.f, 0.f, 0.f, 0.f);
    if (c < N && R != nullptr) res[u] = load_bf16x4(R + ro + c);
  }
#pragma unroll
  for (int u = 0; u < 16; ++u) {
    const int c = (u * 256 + tid) * 4;
    h[u] = make_float4(0.f, 0.f, 0.f, 0.f);
    if (c < N) {
      float4 acc = sum_partials(part + ro + c, splits, mn);
      acc.x += res[u].x; acc.y += res[u].y; acc.z += res[u].z; acc.w += res[u].w;
      h[u] = acc;
      ssq += acc.x * acc.x + acc.y * acc.y + acc.z * acc.z + acc.w * acc.w;
    }
  }
  ssq = wave_sum(ssq);
  if ((tid & 63) == 0) s_red[tid >> 6] = ssq;
  __syncthreads();
  const float rinv = 1.0f / sqrtf((s_red[0] + s_red[1] + s_red[2] + s_red[3]) / (float)N + eps);
#pragma unroll
  for (int u = 0; u < 16; ++u) {
    const int c = (u * 256 + tid) * 4;
    if (c < N) {
      const float4 gn = load_bf16x4(gain + c);
      store_bf16x4(C + ro + c, h[u].x, h[u].y, h[u].z, h[u].w);
      store_bf16x4(Cn + ro + c, h[u].x * gn.x * rinv, h[u].y * gn.y * rinv, h[u].z * gn.z * rinv, h[u].w * gn.w * rinv);
    }
  }
}

__global__ __launch_bounds__(256) void tlow_select_kernel(const float *__restrict__ Y, int splits, int M, int n_adapters,
                                                          int parts, int rank, const int32_t *__restrict__ row_adapter,
                                                          const float *__restrict__ scale, bf16 *__restrict__ tlow) {
  const int row = blockIdx.x;
  const int a = row_adapter[row];
  if (a < 0) return;
  const int N = n_adapters * parts * rank;
  const float sc = scale[a];
  for (int i = threadIdx.x; i < parts * rank; i += 256) {
    const int p = i / rank, j = i - p * rank;
    float t = 0.f;
    for (int sp = 0; sp < splits; ++sp) t += Y[((int64_t)sp * M + row) * N + (a * parts + p) * rank + j];
    t *= sc;
    const bf16 hi = (bf16)t;
    bf16 *dst = tlow + (((int64_t)row * parts + p) * 2) * rank + j;
    dst[0] = hi;
    dst[rank] = (bf16)(t - (float)hi);
  }
}

void launch_tlow_select(const float *Y, int splits, int M, int n_adapters, int parts, int rank,
                        const int32_t *row_adapter, const float *scale, bf16 *tlow, hipStream_t s) {
  if (M == 0) return;
  hipLaunchKernelGGL(tlow_select_kernel, dim3(M), dim3(256), 0, s, Y, splits, M, n_adapters, parts, rank, row_adapter,
                     scale, tlow);
}

bool splitk_reduce_norm_supported(int N) { return N % 4 == 0 && N <= 16384; }

void launch_splitk_reduce_norm(const float *part, int splits, int M, int N, const bf16 *R, const bf16 *gain, float eps,
                               bf16 *C, bf16 *Cn, hipStream_t s) {
  if (M == 0) return;
  hipLaunchKernelGGL(splitk_reduce_norm_kernel, dim3(M), dim3(256), 0, s, part, splits, M, N, R, gain, eps, C, Cn);
}

bool gemm_mfma_supported(int M, int N, int K) { return M > 0 && N > 0 && K >= 64 && K % 64 == 0; }

int gemm_mfma_pick_splits(int M, int N, int K, int n_cu) {
  // split the reduction only while the grid underfills the chip (every split adds a pass of
  // fp32 partial sums), in chunks of at least 512
  int tiles = ((M + 127) / 128) * ((N + 127) / 128);
  int s = 1;
  while (4 * tiles * s < 3 * n_cu && s < 8 && K % (s * 2 * 64) == 0 && K / (s * 2) >= 512) s *= 2;
  return s;
}

// The number of equal segments the reduction axis of a linear with weights [N, K] is ALWAYS cut in: a function
// of the weight shape (and the chip) alone, never of the number of rows, so that a row's result has one
// summation order whatever else is in the call (Proposition 1 in its strong form: the rows before the
// invocation point come out bit-identical from a long prefill, a short one and a decode step).  Enough
// segments that a call with one row tile fills the chip when every segment gets a workgroup of its own.
int gemm_mfma_fixed_segments(int N, int K, int n_cu) {
  const int tiles_n = (N + 127) / 128;
  int s = 1;
  while (4 * tiles_n * s < 3 * n_cu && s < 8 && K % (s * 2 * 64) == 0 && K / (s * 2) >= 512) s *= 2;
  return s;
}

// Whether the segments go to workgroups of their own (their sums travel as fp32 partials and are added in
// order by the consumer) or one workgroup walks through all of them (and adds them in the same order).
// Only a scheduling choice: few row tiles underfill the chip, many make the partials expensive.
bool gemm_mfma_split_segments(int M, int N, int n_cu) {
  const int tiles_m = (M + 127) / 128, tiles_n = (N + 127) / 128;
  return tiles_m <= 2 && 2 * tiles_m * tiles_n <= n_cu;
}

bool gemm_mfma_rope_supported(const GemmArgs &g, int head_dim) {
  return head_dim == 128 && g.k_splits == 1 && g.lora_split == 0 && g.n_q % 128 == 0 && g.n_kv % 128 == 0 &&
         g.N == g.n_q + 2 * g.n_kv && g.M > 2 * 128;
}

void launch_gemm_mfma(GemmArgs g, int epi, hipStream_t s) {
  if (g.M <= 0 || g.N <= 0) return;
  if (g.k_segments < 1) g.k_segments = 1;
  if (epi == GEMM_EPI_SWIGLU) {
    g.k_splits = 1;
    g.lora_split = 0;
    g.k_segments = 1;
  }
  // one workgroup per output tile and a segmented reduction: the kernel adds the segment sums itself.  (The
  // tile shapes behind tile_hint are tuning experiments and do not carry that code.)
  const bool seg = g.k_splits == 1 && g.k_segments > 1 && g.tile_hint == 0 && (g.K / 64) % g.k_segments == 0;
  if (!seg && g.k_splits == 1) g.k_segments = 1;
  if (epi == GEMM_EPI_ROPE) {
    if (seg) launch_cfg<128, 128, 64, 64, GEMM_EPI_ROPE, 2, true, true>(g, s);
    else launch_cfg<128, 128, 64, 64, GEMM_EPI_ROPE, 2, true>(g, s);
    return;
  }
  if (epi == GEMM_EPI_PARTIAL) {
    if (g.tile_hint == 2) launch_cfg<256, 128, 128, 64, GEMM_EPI_PARTIAL>(g, s);
    else if (g.tile_hint == 3) launch_cfg<256, 256, 64, 128, GEMM_EPI_PARTIAL, 1>(g, s);
    else if (g.tile_hint == 4) launch_cfg<128, 64, 32, 64, GEMM_EPI_PARTIAL>(g, s);
    else if (g.tile_hint == 5) launch_cfg<128, 128, 32, 64, GEMM_EPI_PARTIAL>(g, s);
    else if (g.tile_hint == 6) launch_cfg<128, 128, 64, 32, GEMM_EPI_PARTIAL>(g, s);
    else if (g.tile_hint == 1) launch_cfg<128, 128, 64, 64, GEMM_EPI_PARTIAL>(g, s);
    else if (seg) launch_cfg<128, 128, 64, 64, GEMM_EPI_PARTIAL, 2, true, true>(g, s);
    else if (g.M > 4 * 128) launch_cfg<128, 128, 64, 64, GEMM_EPI_PARTIAL, 2, true>(g, s);
    // up to 32 rows (a decode step of a few sequences): a 32-row block does a quarter of the matrix and
    // fragment work per weight tile and several workgroups share a compute unit
    else if (g.M <= 32) launch_cfg<32, 128, 32, 32, GEMM_EPI_PARTIAL>(g, s);
    // few row tiles: the kernel streams weights and eight waves (two per SIMD) hide its LDS and barrier
    // latencies better than four.  The block is cut into 64x32 wave tiles: that variant stays under 128
    // registers, so two workgroups share a compute unit -- with two row tiles and four reduction segments
    // there are more workgroups than compute units (the 32x64 cut needs 131 registers: one workgroup per unit,
    // a second round of workgroups, 34 instead of 31 us for a 256-row projection)
    else launch_cfg<128, 128, 64, 32, GEMM_EPI_PARTIAL>(g, s);
  } else if (epi == GEMM_EPI_SWIGLU) {
    if (g.tile_hint == 4) launch_cfg<128, 64, 32, 64, GEMM_EPI_SWIGLU>(g, s);
    // (a wave needs a gate block and its up block: at least two 32-column blocks, so no 64x32 wave tiles here)
    else if (g.tile_hint == 5 || g.tile_hint == 6) launch_cfg<128, 128, 32, 64, GEMM_EPI_SWIGLU>(g, s);
    else if (g.tile_hint == 1) launch_cfg<128, 128, 64, 64, GEMM_EPI_SWIGLU>(g, s);
    else if (g.M <= 32) launch_cfg<32, 128, 32, 64, GEMM_EPI_SWIGLU>(g, s);
    else if (g.M <= 128) launch_cfg<128, 128, 32, 64, GEMM_EPI_SWIGLU>(g, s);
    else if (g.tile_hint == 2 || g.M <= 512) launch_cfg<256, 128, 128, 64, GEMM_EPI_SWIGLU>(g, s);
    // many row tiles: the woven 128x128 block, two workgroups per compute unit, as in the QKV projection
    else launch_cfg<128, 128, 64, 64, GEMM_EPI_SWIGLU, 2, true>(g, s);
  } else {
    g.k_splits = 1;
    g.lora_split = 0;
    if (g.tile_hint == 4) launch_cfg<128, 64, 32, 64, GEMM_EPI_BF16>(g, s);
    else if (g.tile_hint == 5) launch_cfg<128, 128, 32, 64, GEMM_EPI_BF16>(g, s);
    else if (g.tile_hint == 6) launch_cfg<128, 128, 64, 32, GEMM_EPI_BF16>(g, s);
    else if (g.tile_hint == 1) launch_cfg<128, 128, 64, 64, GEMM_EPI_BF16>(g, s);
    else if (g.M <= 32) {
      if (seg) launch_cfg<32, 128, 32, 32, GEMM_EPI_BF16, 2, false, true>(g, s);
      else launch_cfg<32, 128, 32, 32, GEMM_EPI_BF16>(g, s);
    } else if (g.M <= 128) {
      if (seg) launch_cfg<128, 128, 64, 32, GEMM_EPI_BF16, 2, false, true>(g, s);
      else launch_cfg<128, 128, 64, 32, GEMM_EPI_BF16>(g, s);
    } else {
      if (seg) launch_cfg<128, 128, 64, 64, GEMM_EPI_BF16, 2, true, true>(g, s);
      else launch_cfg<256, 128, 128, 64, GEMM_EPI_BF16>(g, s);
    }
  }
}

}  // namespace alora
