// Row preparation with MFMA (bf16): per-row metadata, RMSNorm, and the low-rank down projection
// t = s_a * A_a x_hat (Eq.6, Delta applied right to left) for 16 packed rows per workgroup.
//
// Eight waves split the hidden dimension (d = 512, 1024, 2048 or 4096); each lane owns 8 consecutive
// elements of one row at a time, which is both the 16-byte global access and the A-operand layout of
// v_mfma_f32_16x16x32_bf16 (lane l: row l%16, k = 8*(l/16)..+7), so the normalised row goes from
// registers straight into the MFMA and into the x_hat store; LDS is used only for the row
// statistics and the fixed-order sum of the eight partial accumulators.
#include "mfma_kernels.h"

namespace alora {

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(4 * sizeof(float)))) float f32x4;
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

constexpr int PREP_ROWS = 16;
constexpr int PREP_WAVES = 8;

// Sum of squares of a row, in ONE order for every kernel that normalises rows (a row's x_hat must not depend on
// which of them ran -- the base rows of a long prefill and of a decode step are compared bit for bit): the
// row is cut into 16-byte chunks, chunk index c = 64 w + 4 u + g (w < 8, u < d / 256, g < 4); a chunk's eight
// squares are added in order starting from zero; the chunk sums of one (w, g) go through a balanced tree over u
// (neighbours first), the four g of a w through a tree (g ^ 1, then g ^ 2), the eight w are added in order.
__device__ __forceinline__ float chunk_ssq(u32x4 c) {
  const bf16x8 v = __builtin_bit_cast(bf16x8, c);
  float s = 0.f;
#pragma unroll
  for (int e = 0; e < 8; ++e) { const float f = (float)v[e]; s = __builtin_fmaf(f, f, s); }
  return s;
}
__device__ __forceinline__ float row_rinv(float ssq, int d, float eps) { return 1.0f / sqrtf(ssq / (float)d + eps); }
__device__ __forceinline__ u32x4 norm_chunk(u32x4 x, u32x4 g, float rinv) {
  const bf16x8 xv = __builtin_bit_cast(bf16x8, x), gv = __builtin_bit_cast(bf16x8, g);
  bf16x8 xh;
#pragma unroll
  for (int e = 0; e < 8; ++e) xh[e] = (bf16)((float)xv[e] * (float)gv[e] * rinv);
  return __builtin_bit_cast(u32x4, xh);
}
// Metadata of the rows [row0, tile_end) of one tile: a thread takes a sequence, fetches its record once and fills
// in the rows of the tile that belong to it -- one memory round trip, where a search over the sequence table
// per row costs log2(n_seqs) dependent ones.  s_adapter / s_scale may be nullptr.
__device__ __forceinline__ void fill_row_meta(const PrepArgs &a, const SeqMeta &sm, int sq, int mrow, int row0, bool write,
                                              int *s_adapter, float *s_scale, unsigned long long *s_present) {
  const int pos = sm.P + a.pos_shift + (mrow - sm.row_start);
  int adapter = -1;
  float scale = 0.f;
  if (sm.adapter >= 0 && pos >= sm.k) { adapter = sm.adapter; scale = sm.scale; }
  if (write) {
    a.rm.seq[mrow] = sq;
    a.rm.pos[mrow] = pos;
    a.rm.adapter[mrow] = adapter;
    a.rm.slot[mrow] = sm.pool_off + pos;
  }
  if (s_adapter != nullptr) { s_adapter[mrow - row0] = adapter; s_scale[mrow - row0] = scale; }
  if (adapter >= 0) atomicOr(s_present, 1ull << adapter);
}

// NF = 16-column fragments of t this workgroup computes (0: no adapter work).  The 3*rank columns
// of t are spread over gridDim.y workgroups so that short batches still fill the chip; group 0
// also writes x_hat and the row metadata.  CH = d / 256: 16-byte chunks of its row each lane
// holds.  x is read from memory once: the chunks stay in registers from the sum of squares to the
// normalised store and the MFMAs, and every phase issues all its loads before the first use, so
// the kernel pays about three memory round trips in total.
// EARLY (single-sequence batches with NF == 1): the sequence record comes with the kernel arguments, so the
// adapter of the tile is known at once and its A fragments are requested together with x instead of after
// the metadata and normalisation phases -- one dependent memory round trip less on a kernel that is nothing
// but round trips at these sizes.
template <int NF, int CH, bool EARLY = false>
__global__ __launch_bounds__(512, 2) void prep_rows_mfma_kernel(PrepArgs a) {
  __shared__ float s_ssq[PREP_WAVES][PREP_ROWS];
  __shared__ int s_adapter[PREP_ROWS];
  __shared__ float s_scale[PREP_ROWS];
  __shared__ unsigned long long s_present;
  __shared__ u32x4 s_gain[CH * 32];          // d / 8 chunks of the gain
  extern __shared__ float s_part[];          // [PREP_WAVES][PREP_ROWS][16 * NF]

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int r16 = lane & 15, kg = lane >> 4;
  const int row0 = blockIdx.x * PREP_ROWS;
  const int d = a.d;                            // = CH * 256
  const int col0 = blockIdx.y * 16 * NF;       // first column of t handled here
  // gridDim.z > 1 (short batches of several sequences): workgroup z does the pass of adapter z only -- the passes
  // of the adapters present in a row tile, each a memory round trip of its own, then run side by side
  const int only = gridDim.z > 1 ? (int)blockIdx.z : -1;
  const bool lead = blockIdx.y == 0 && blockIdx.z == 0;
  const int row = min(row0 + r16, a.T - 1);
  const bool row_ok = row0 + r16 < a.T;
  const int k_lo = wave * (CH * 32) + kg * 8;  // this lane's first element; chunk u is at k_lo + 32 u

  // ---- all of this lane's x (and gain) chunks, issued at once ----------------------------------
  // (the gain goes through LDS: one 16-byte chunk per thread instead of CH of them in every lane's registers)
  u32x4 xr[CH], gown = u32x4{0, 0, 0, 0};
  const bf16 *xrow = a.x + (int64_t)row * d + k_lo;
#pragma unroll
  for (int u = 0; u < CH; ++u) xr[u] = *reinterpret_cast<const u32x4 *>(xrow + 32 * u);
  if (a.gain != nullptr && tid < d / 8) gown = *reinterpret_cast<const u32x4 *>(a.gain + tid * 8);

  // EARLY: A fragments of the sequence's adapter, if any row of the tile is adapted
  u32x4 bpre[EARLY ? CH : 1][EARLY && NF > 0 ? NF : 1];
  bool pre_loaded = false;
  if constexpr (EARLY && NF > 0) {
    const SeqMeta &o = a.one;
    const int last = min(row0 + PREP_ROWS, a.T) - 1;
    pre_loaded = o.adapter >= 0 && o.P + a.pos_shift + (last - o.row_start) >= o.k;
    if (pre_loaded) {
      const bf16 *Ab = a.A + ((int64_t)o.adapter * 3 * a.rank + col0 + r16) * d + k_lo;
#pragma unroll
      for (int u = 0; u < CH; ++u)
#pragma unroll
        for (int j = 0; j < NF; ++j) bpre[u][j] = *reinterpret_cast<const u32x4 *>(Ab + (int64_t)j * 16 * d + 32 * u);
    }
  }

  if (tid == 0) s_present = 0ull;
  if (tid < PREP_ROWS) { s_adapter[tid] = -1; s_scale[tid] = 0.f; }
  __syncthreads();
  // Row metadata.  With one sequence (EARLY: its record came with the arguments) a thread takes a row.
  // Otherwise a thread takes a sequence: it fetches the sequence record once and fills in the rows of this
  // tile that belong to it -- one memory round trip, where a search over the sequence table per row costs
  // log2(n_seqs) dependent ones.
  const int tile_end = min(row0 + PREP_ROWS, a.T);
  auto fill_row = [&](const SeqMeta &sm, int sq, int mrow) {
    fill_row_meta(a, sm, sq, mrow, row0, a.write_meta && lead, s_adapter, s_scale, &s_present);
  };
  if constexpr (EARLY) {
    if (tid < PREP_ROWS && row0 + tid < tile_end) fill_row(a.one, 0, row0 + tid);
  } else {
    for (int sq = tid; sq < (a.seqs != nullptr ? a.n_seqs : 0); sq += 512) {
      const SeqMeta sm = a.seqs[sq];
      const int lo = max(sm.row_start, row0), hi = min(sm.row_start + sm.n_new, tile_end);
      for (int mrow = lo; mrow < hi; ++mrow) fill_row(sm, sq, mrow);
    }
  }

  // ---- sum of squares: lane -> the 4 lanes of a row -> the 8 waves (fixed order) ------------------
  float rinv = 1.f;
  if (a.gain != nullptr) {
    float cs[CH];
#pragma unroll
    for (int u = 0; u < CH; ++u) cs[u] = chunk_ssq(xr[u]);
#pragma unroll
    for (int st = 1; st < CH; st *= 2)
#pragma unroll
      for (int u = 0; u < CH; u += 2 * st) cs[u] += cs[u + st];
    float ssq = cs[0];
    ssq += __shfl_xor(ssq, 16, 64);
    ssq += __shfl_xor(ssq, 32, 64);
    if (kg == 0) s_ssq[wave][r16] = ssq;
    if (tid < d / 8) s_gain[tid] = gown;
  }
  __syncthreads();
  if (lead && tid == 0 && a.rm.present16 != nullptr) a.rm.present16[blockIdx.x] = s_present;
  if (a.gain != nullptr) {
    float t = 0.f;
#pragma unroll
    for (int w = 0; w < PREP_WAVES; ++w) t += s_ssq[w][r16];
    rinv = row_rinv(t, d, a.eps);
    // normalise in place: x_hat = bf16(x * g * rinv)
#pragma unroll
    for (int u = 0; u < CH; ++u) xr[u] = norm_chunk(xr[u], s_gain[(k_lo >> 3) + 4 * u], rinv);
  }
  if (lead && row_ok) {
    bf16 *dst = a.xh + (int64_t)row * d + k_lo;
#pragma unroll
    for (int u = 0; u < CH; ++u) *reinterpret_cast<u32x4 *>(dst + 32 * u) = xr[u];
  }

  // ---- t partials over this wave's slice of d, one pass per adapter present in the row tile -------
  const int my_adapter = s_adapter[r16];
  const unsigned long long present = NF > 0 ? (only >= 0 ? s_present & (1ull << only) : s_present) : 0ull;
  const int rank = a.rank;
  f32x4 acc[NF > 0 ? NF : 1];
#pragma unroll
  for (int j = 0; j < (NF > 0 ? NF : 1); ++j) acc[j] = f32x4{0.f, 0.f, 0.f, 0.f};
  if (NF > 0) {
    constexpr int NFX = NF > 0 ? NF : 1;
    // chunks per load batch: about 16 fragments, a power of two so that it divides CH
    constexpr int UBN = NFX >= 9 ? 1 : NFX >= 5 ? 2 : NFX >= 3 ? 4 : NFX == 2 ? 8 : 16;
    constexpr int UB0 = UBN > CH ? CH : UBN;
    constexpr int UB = UB0;
    if constexpr (EARLY) {
      if (pre_loaded) {
        const bool mine = my_adapter == a.one.adapter;
#pragma unroll
        for (int u = 0; u < CH; ++u) {
          const u32x4 au = mine ? xr[u] : u32x4{0, 0, 0, 0};
#pragma unroll
          for (int j = 0; j < NFX; ++j)
            acc[j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, au),
                                                             __builtin_bit_cast(bf16x8, bpre[u][j]), acc[j], 0, 0, 0);
        }
      }
    }
    // One pass over the lane's chunks per adapter present in the tile, in batches of UB chunks.  Every batch
    // of A fragments is a memory round trip, so two register buffers alternate: the next batch -- the next
    // adapter's first one at the end of a pass -- is requested before the current one is multiplied.
    unsigned long long todo = EARLY ? 0ull : present;
    auto next_adapter = [&]() {
      if (!todo) return -1;
      const int ad = __builtin_ctzll(todo);
      todo &= todo - 1;
      return ad;
    };
    auto load_batch = [&](int ad, int u0, u32x4 (&br)[UB][NFX]) {
      const bf16 *Ab = a.A + ((int64_t)ad * 3 * rank + col0 + r16) * d + k_lo;     // row col0 + 16 j + r16
#pragma unroll
      for (int u = 0; u < UB; ++u)
#pragma unroll
        for (int j = 0; j < NFX; ++j)
          br[u][j] = *reinterpret_cast<const u32x4 *>(Ab + (int64_t)j * 16 * d + 32 * (u0 + u));
    };
    auto mma_batch = [&](int ad, int u0, const u32x4 (&br)[UB][NFX]) {
      const bool mine = my_adapter == ad;
#pragma unroll
      for (int u = 0; u < UB; ++u) {
        const u32x4 au = mine ? xr[u0 + u] : u32x4{0, 0, 0, 0};
#pragma unroll
        for (int j = 0; j < NFX; ++j)
          acc[j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, au),
                                                           __builtin_bit_cast(bf16x8, br[u][j]), acc[j], 0, 0, 0);
      }
    };
    constexpr int NB = CH / UB;        // batches per pass
    static_assert(CH % UB == 0, "batches cover the lane's chunks exactly");
    if constexpr (NB % 2 == 0) {
      u32x4 br0[UB][NFX], br1[UB][NFX];
      int ad = next_adapter();
      if (ad >= 0) load_batch(ad, 0, br0);
      while (ad >= 0) {
        const int nx = next_adapter();
#pragma unroll
        for (int u0 = 0; u0 < CH; u0 += 2 * UB) {
          load_batch(ad, u0 + UB, br1);
          mma_batch(ad, u0, br0);
          if (u0 + 2 * UB < CH) load_batch(ad, u0 + 2 * UB, br0);
          else if (nx >= 0) load_batch(nx, 0, br0);
          mma_batch(ad, u0 + UB, br1);
        }
        ad = nx;
      }
    } else {
      static_assert(NB == 1, "batches per pass: one or an even number");
      u32x4 br0[UB][NFX], br1[UB][NFX];      // one batch per pass: adapters alternate between the buffers
      int ad = next_adapter();
      if (ad >= 0) load_batch(ad, 0, br0);
      while (ad >= 0) {
        const int nx = next_adapter();
        if (nx >= 0) load_batch(nx, 0, br1);
        mma_batch(ad, 0, br0);
        if (nx < 0) break;
        ad = next_adapter();
        if (ad >= 0) load_batch(ad, 0, br0);
        mma_batch(nx, 0, br1);
      }
    }
  }

  if (NF > 0 && present) {
    // accumulator register v of lane l is T[row 4*(l/16) + v][column 16*j + l%16]
    float *mine = s_part + (size_t)wave * PREP_ROWS * 16 * NF;
#pragma unroll
    for (int j = 0; j < NF; ++j)
#pragma unroll
      for (int v = 0; v < 4; ++v) mine[(4 * kg + v) * 16 * NF + j * 16 + r16] = acc[j][v];
    __syncthreads();
    const int n_out = PREP_ROWS * 16 * NF;       // 16 rows x 3*rank columns
    for (int i = tid; i < n_out; i += 512) {
      const int lr = i / (16 * NF), col = i % (16 * NF);
      const int orow = row0 + lr;
      if (orow >= a.T || s_adapter[lr] < 0 || (only >= 0 && s_adapter[lr] != only)) continue;
      float t = 0.f;
#pragma unroll
      for (int w = 0; w < PREP_WAVES; ++w) t += s_part[(size_t)w * n_out + i];
      t *= s_scale[lr];
      const int p = (col0 + col) / rank, jj = (col0 + col) % rank;
      const bf16 hi = (bf16)t;
      bf16 *dst = a.tlow16 + (((int64_t)orow * 3 + p) * 2) * rank + jj;
      dst[0] = hi;
      dst[rank] = (bf16)(t - (float)hi);
    }
  }
}

// Many rows at d = 4096 and no adapter in the call (a base-model prefill): metadata and RMSNorm only.  A wave takes
// four consecutive rows whole -- every load and store instruction covers 1 KB of one row, 32 KB are in flight per
// wave -- sixteen rows per workgroup of four waves, several workgroups per compute unit; the 16-rows-per-tile
// kernel above holds a whole tile in registers, runs one workgroup per compute unit and needs a second round of
// workgroups from 4097 rows on.  Same arithmetic in the same order: lane l holds the chunks c = l + 64 j, so
// l = 4 u + g and j = w in the terms of chunk_ssq's order.
__global__ __launch_bounds__(256) void norm_rows_kernel(PrepArgs a) {
  __shared__ unsigned long long s_present;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int row0 = blockIdx.x * PREP_ROWS;
  constexpr int D = 4096, NJ = D / 512, RW = PREP_ROWS / 4;      // rows per wave
  const int wrow0 = row0 + wave * RW;
  u32x4 xr[RW][NJ], gr[NJ];
#pragma unroll
  for (int i = 0; i < RW; ++i) {
    const int row = min(wrow0 + i, a.T - 1);      // rows past the end repeat the last one and are not stored
    const bf16 *xrow = a.x + (int64_t)row * D + lane * 8;
#pragma unroll
    for (int j = 0; j < NJ; ++j) xr[i][j] = *reinterpret_cast<const u32x4 *>(xrow + 512 * j);
  }
  if (a.gain != nullptr) {
#pragma unroll
    for (int j = 0; j < NJ; ++j) gr[j] = *reinterpret_cast<const u32x4 *>(a.gain + lane * 8 + 512 * j);
  }
  if (tid == 0) s_present = 0ull;
  __syncthreads();
  const int tile_end = min(row0 + PREP_ROWS, a.T);
  for (int sq = tid; sq < (a.seqs != nullptr ? a.n_seqs : 0); sq += 256) {
    const SeqMeta sm = a.seqs[sq];
    const int lo = max(sm.row_start, row0), hi = min(sm.row_start + sm.n_new, tile_end);
    for (int mrow = lo; mrow < hi; ++mrow) fill_row_meta(a, sm, sq, mrow, row0, a.write_meta != 0, nullptr, nullptr, &s_present);
  }
  __syncthreads();
  if (tid == 0 && a.rm.present16 != nullptr) a.rm.present16[blockIdx.x] = s_present;
#pragma unroll
  for (int i = 0; i < RW; ++i) {
    if (a.gain != nullptr) {
      float t = 0.f;
#pragma unroll
      for (int j = 0; j < NJ; ++j) {
        float v = chunk_ssq(xr[i][j]);
        v += __shfl_xor(v, 4, 64);       // tree over u (lane bits 2..5), neighbours first
        v += __shfl_xor(v, 8, 64);
        v += __shfl_xor(v, 16, 64);
        v += __shfl_xor(v, 32, 64);
        v += __shfl_xor(v, 1, 64);       // tree over g (lane bits 0, 1)
        v += __shfl_xor(v, 2, 64);
        t += v;                          // the eight w in order
      }
      const float rinv = row_rinv(t, D, a.eps);
#pragma unroll
      for (int j = 0; j < NJ; ++j) xr[i][j] = norm_chunk(xr[i][j], gr[j], rinv);
    }
    if (wrow0 + i < a.T) {
      bf16 *dst = a.xh + (int64_t)(wrow0 + i) * D + lane * 8;
#pragma unroll
      for (int j = 0; j < NJ; ++j) *reinterpret_cast<u32x4 *>(dst + 512 * j) = xr[i][j];
    }
  }
}

bool norm_rows_mfma_supported(int d) { return d == 4096; }
void launch_norm_rows_mfma(const PrepArgs &a, hipStream_t s) {
  if (a.T == 0) return;
  hipLaunchKernelGGL(norm_rows_kernel, dim3((a.T + PREP_ROWS - 1) / PREP_ROWS), dim3(256), 0, s, a);
}

bool prep_rows_mfma_supported(int d, int rank) {
  return (d == 4096 || d == 2048 || d == 1024 || d == 512) && (rank == 0 || rank == 16 || rank == 32 || rank == 64);
}

template <int NF, int CH, bool EARLY = false>
static void launch_prep_cfg(const PrepArgs &a, int groups, hipStream_t s) {
  const int row_tiles = (a.T + PREP_ROWS - 1) / PREP_ROWS;
  // few row tiles, several sequences, several adapters: one workgroup per (row tile, column group, adapter)
  const int per_adapter = (!EARLY && NF > 0 && a.n_adapters > 1 && a.n_adapters <= 16 && a.n_seqs > 1 &&
                           row_tiles * groups * a.n_adapters <= 1024) ? a.n_adapters : 1;
  const dim3 grid(row_tiles, groups, per_adapter);
  const size_t smem = (size_t)PREP_WAVES * PREP_ROWS * 16 * NF * sizeof(float);
  auto kern = prep_rows_mfma_kernel<NF, CH, EARLY>;
  // set on every launch that needs it: a host-side attribute write, safe from any thread and on any device
  if (smem > 48 * 1024)
    (void)hipFuncSetAttribute((const void *)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
  hipLaunchKernelGGL(kern, grid, dim3(512), smem, s, a);
}

template <int NF>
static void launch_prep_nf(const PrepArgs &a, int groups, hipStream_t s) {
  if (NF == 1 && a.seqs != nullptr && a.n_seqs == 1) {
    switch (a.d) {
      case 4096: launch_prep_cfg<1, 16, true>(a, groups, s); return;
      case 2048: launch_prep_cfg<1, 8, true>(a, groups, s); return;
      case 1024: launch_prep_cfg<1, 4, true>(a, groups, s); return;
      case 512: launch_prep_cfg<1, 2, true>(a, groups, s); return;
      default: break;
    }
  }
  switch (a.d) {
    case 4096: launch_prep_cfg<NF, 16>(a, groups, s); break;
    case 2048: launch_prep_cfg<NF, 8>(a, groups, s); break;
    case 1024: launch_prep_cfg<NF, 4>(a, groups, s); break;
    case 512: launch_prep_cfg<NF, 2>(a, groups, s); break;
    default: break;
  }
}

void launch_prep_rows_mfma(const PrepArgs &a, hipStream_t s) {
  if (a.T == 0) return;
  const int nf = (a.rank > 0 && a.A != nullptr) ? 3 * a.rank / 16 : 0;     // 3, 6 or 12
  if (nf == 0) { launch_prep_nf<0>(a, 1, s); return; }
  // fragments per workgroup: as few as it takes to reach ~256 workgroups, out of {nf, nf/2, 3, 1}
  const int row_tiles = (a.T + PREP_ROWS - 1) / PREP_ROWS;
  int per = nf;
  if (row_tiles * (nf / per) < 256 && per % 2 == 0 && per > 3) per /= 2;      // 12 -> 6, 6 -> 3
  if (row_tiles * (nf / per) < 256 && per % 2 == 0 && per > 3) per /= 2;      // 6 -> 3
  if (row_tiles * (nf / per) < 256 && per == 3) per = 1;
  const int groups = nf / per;
  switch (per) {
    case 1: launch_prep_nf<1>(a, groups, s); break;
    case 3: launch_prep_nf<3>(a, groups, s); break;
    case 6: launch_prep_nf<6>(a, groups, s); break;
    case 12: launch_prep_nf<12>(a, groups, s); break;
    default: break;
  }
}

}  // namespace alora
