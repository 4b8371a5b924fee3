// Decode attention (Eq.4: one new query per sequence over its whole cache), memory-bound:
// every cached key/value byte is read exactly once and everything else is kept out of the way.
//
// Work item: one workgroup of eight waves = (rows, key split), listed by the host.  Wave w takes kv head
// g0 + w % HW and sub-range w / HW of the item's keys (HW = kv heads per workgroup, 8 for eight or more kv heads):
// the waves of a workgroup walk the same token rows of the cache at the same time, each its own 256-byte head
// slice, so that between them they fetch whole rows of the token-major cache (2 KB at 8 kv heads) -- HBM delivers
// 6.2 TB/s to that pattern and 5.6 TB/s when the heads of a row are fetched by unrelated workgroups.  The waves
// never synchronise until the final merge of the sub-ranges.  Normally an item is one row
// (one sequence's new token) over that sequence's own cache rows.  Sequences that name the same
// shared prefix (Section 2, "Cache reuse patterns": several adapters on one context) are packed 16 / G to an item for the
// prefix part: their heads fill the MFMA columns a single sequence leaves empty, and the prefix
// is read from memory once for all of them.  A wave consumes 32 keys per step:
//   * K rows go from global memory straight into the A operand of v_mfma_f32_16x16x32_bf16
//     (lane l: key l%16, head-dim slice 8*(l/16)..+7 of the current 32-wide k-step), the G query
//     heads of the group are the (zero padded) 16 B-operand columns: S^T[key][head].
//   * Accumulator register v of lane l is S^T[key 4*(l/16)+v][head l%16]: a lane owns one head, so
//     max / sum / rescale are per-lane scalars, and the two key blocks' probabilities
//     p[16u + 4*(l/16) + v] are, as they sit, the B operand (k = 32 keys) of O^T += V^T P^T.
//   * V rows are loaded as 8 columns x 1 key per lane (16 B) for exactly those 8 keys and
//     transposed inside the lane with byte permutes: MFMA number c uses column 8*i + c of lane
//     row i, so O^T_c[i][head] = O[column 8*i + c][head].  No LDS, no cross-lane traffic.
// Every MFMA operand is fp16, as in the prefill kernel: the queries arrive as fp16, the bf16 cache rows are
// converted in registers on their way into the operands (exact; the V conversion packs two keys of one column into
// a word, which is the transposition) and the probabilities are packed to fp16.  The kernel waits for memory, the
// vector ALU has the time, and the rounding of bf16 queries and probabilities was most of the error.
// Partials (acc, max, sum) per (row, head, split) are merged by the log-sum-exp merge kernel.
#include "mfma_kernels.h"

namespace alora {

typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));
typedef __attribute__((__vector_size__(4 * sizeof(float)))) float f32x4;
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

// two floats as an fp16 pair (round toward zero: finite stays finite; exact for bf16 values)
__device__ __forceinline__ uint32_t dec_pack2(float a, float b) {
  return __builtin_bit_cast(uint32_t, __builtin_amdgcn_cvt_pkrtz(a, b));
}
__device__ __forceinline__ float dec_lo(uint32_t w) { return __builtin_bit_cast(float, w << 16); }
__device__ __forceinline__ float dec_hi(uint32_t w) { return __builtin_bit_cast(float, w & 0xffff0000u); }
__device__ __forceinline__ u32x4 dec_bf16x8_to_f16x8(u32x4 r) {
  return u32x4{dec_pack2(dec_lo(r.x), dec_hi(r.x)), dec_pack2(dec_lo(r.y), dec_hi(r.y)),
               dec_pack2(dec_lo(r.z), dec_hi(r.z)), dec_pack2(dec_lo(r.w), dec_hi(r.w))};
}

// acc + lo + hi of a packed fp16 pair
__device__ __forceinline__ float dec_sum2(uint32_t pair, float acc) {
  typedef _Float16 half2_t __attribute__((ext_vector_type(2)));
  return __builtin_amdgcn_fdot2(__builtin_bit_cast(half2_t, pair), __builtin_bit_cast(half2_t, 0x3c003c00u), acc, false);
}

constexpr float DEC_LOG2E = 1.4426950408889634f;
constexpr float DEC_LN2 = 0.6931471805599453f;

__global__ __launch_bounds__(512) void attn_decode_mfma_kernel(DecodeArgs a) {
  constexpr int H = 128;
  extern __shared__ float s_o[];           // [wave][column < cols_max][acc..., m, l]

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int j = lane & 15, kg = lane >> 4;           // j: head column / key row / V row; kg: k group
  const DecItem *it = a.items + blockIdx.x;
  const int HW = a.heads_per_wg, KR = a.ranges_per_wg, CM = a.cols_max;
  const int hw = wave % HW, sub = wave / HW;
  const bool active = sub < KR && it->g + hw < a.n_kv_heads;      // (a workgroup may hold fewer than eight (head, range) pairs)
  const int g = min(it->g + hw, a.n_kv_heads - 1), split = it->split;
  const int G = a.n_q_heads / a.n_kv_heads;
  const int n_cols = it->n_rows * G;                 // MFMA columns in use: column = row index * G + head
  const int row_first = it->rows[0];
  const SeqMeta sm = a.seqs[a.rm.seq[row_first]];
  // the item's keys are pool rows key_row0 .. key_row0 + n_keys - 1
  const int n_keys = it->shared ? sm.prefix_len : a.rm.pos[row_first] + 1 - sm.prefix_len;
  const int64_t key_row0 = it->shared ? sm.prefix_off : sm.pool_off + sm.prefix_len;
  // keys of this (split, sub-range): contiguous, multiple of 32
  const int n_ranges = it->n_splits * KR;
  int per = (n_keys + n_ranges - 1) / n_ranges;
  per = (per + 31) & ~31;
  const int kbeg = active ? (split * KR + sub) * per : 0;
  const int kend = active ? min(n_keys, kbeg + per) : 0;
  const bf16 *Kp = a.K + key_row0 * a.n_kv + g * H;
  const bf16 *Vp = a.V + key_row0 * a.n_kv + g * H;

  // queries: B operand columns = (row, head of the group) pairs (zero for padding columns)
  u32x4 qf[4];
  {
    const int rj = j / G, hj = j - rj * G;
    const int qrow = it->rows[j < n_cols ? rj : 0];
#pragma unroll
    for (int s = 0; s < 4; ++s) {
      qf[s] = u32x4{0, 0, 0, 0};
      if (j < n_cols) qf[s] = *reinterpret_cast<const u32x4 *>(a.Q + (int64_t)qrow * a.n_q + (g * G + hj) * H + 32 * s + 8 * kg);
    }
  }

  f32x4 o[8];
#pragma unroll
  for (int c = 0; c < 8; ++c) o[c] = f32x4{0.f, 0.f, 0.f, 0.f};
  float m_run = -INFINITY, l_run = 0.f;
  const float c_scale = a.sm_scale * DEC_LOG2E;

  u32x4 kr[2][4], vr[2][4];      // [key block u][k-step s] and [u][n]: key 16u + 4kg + n
  auto load_step = [&](int k0) {
#pragma unroll
    for (int u = 0; u < 2; ++u) {
      const int kk = min(k0 + 16 * u + j, n_keys - 1);
#pragma unroll
      for (int s = 0; s < 4; ++s)
        kr[u][s] = *reinterpret_cast<const u32x4 *>(Kp + (int64_t)kk * a.n_kv + 32 * s + 8 * kg);
#pragma unroll
      for (int n = 0; n < 4; ++n) {
        const int kv = min(k0 + 16 * u + 4 * kg + n, n_keys - 1);
        vr[u][n] = *reinterpret_cast<const u32x4 *>(Vp + (int64_t)kv * a.n_kv + 8 * j);
      }
    }
  };

  if (kbeg < kend) load_step(kbeg);
  for (int k0 = kbeg; k0 < kend; k0 += 32) {
    // consume the registers of this step, then refill them for the next one
    u32x4 kc[2][4], vc[2][4];
#pragma unroll
    for (int u = 0; u < 2; ++u)
#pragma unroll
      for (int s = 0; s < 4; ++s) { kc[u][s] = kr[u][s]; vc[u][s] = vr[u][s]; }
    load_step(k0 + 32);      // unconditional: key indices are clamped to the last valid row

    f32x4 sc[2];
#pragma unroll
    for (int u = 0; u < 2; ++u) {
      sc[u] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
      for (int s = 0; s < 4; ++s)
        sc[u] = __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(f16x8, dec_bf16x8_to_f16x8(kc[u][s])),
                                                       __builtin_bit_cast(f16x8, qf[s]), sc[u], 0, 0, 0);
    }
    if (k0 + 32 > kend) {
#pragma unroll
      for (int u = 0; u < 2; ++u)
#pragma unroll
        for (int v = 0; v < 4; ++v)
          if (k0 + 16 * u + 4 * kg + v >= kend) sc[u][v] = -INFINITY;
    }
    float mx = -INFINITY;
#pragma unroll
    for (int u = 0; u < 2; ++u)
#pragma unroll
      for (int v = 0; v < 4; ++v) mx = fmaxf(mx, sc[u][v]);
    mx = fmaxf(mx, __shfl_xor(mx, 16, 64));
    mx = fmaxf(mx, __shfl_xor(mx, 32, 64));
    const float m_new = fmaxf(m_run, mx * c_scale);       // finite: every step has at least one valid key
    const float alpha = __builtin_amdgcn_exp2f(m_run - m_new);
    m_run = m_new;
    float p[2][4];
#pragma unroll
    for (int u = 0; u < 2; ++u)
#pragma unroll
      for (int v = 0; v < 4; ++v) p[u][v] = __builtin_amdgcn_exp2f(fmaf(sc[u][v], c_scale, -m_new));
    const uint32_t d0 = dec_pack2(p[0][0], p[0][1]), d1 = dec_pack2(p[0][2], p[0][3]);
    const uint32_t d2 = dec_pack2(p[1][0], p[1][1]), d3 = dec_pack2(p[1][2], p[1][3]);
    // row sum from the rounded probabilities, so numerator and denominator carry the same rounding
    const float rs = dec_sum2(d3, dec_sum2(d2, dec_sum2(d1, dec_sum2(d0, 0.f))));
    const u32x4 pf = u32x4{d0, d1, d2, d3};
    l_run = l_run * alpha + rs;
#pragma unroll
    for (int c = 0; c < 8; ++c) {
      // column 8*j + c of the 8 keys this lane loaded: element c of each 16-byte row
      const int w = c >> 1;
      auto el = [&](uint32_t word) { return (c & 1) ? dec_hi(word) : dec_lo(word); };
      const u32x4 vf = u32x4{dec_pack2(el(vc[0][0][w]), el(vc[0][1][w])), dec_pack2(el(vc[0][2][w]), el(vc[0][3][w])),
                             dec_pack2(el(vc[1][0][w]), el(vc[1][1][w])), dec_pack2(el(vc[1][2][w]), el(vc[1][3][w]))};
      f32x4 oc = o[c];
#pragma unroll
      for (int v = 0; v < 4; ++v) oc[v] *= alpha;
      o[c] = __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(f16x8, vf), __builtin_bit_cast(f16x8, pf),
                                                    oc, 0, 0, 0);
    }
  }

  // ---- merge the sub-ranges of every head (fixed order) and write the partials ----------------------
  const float l_tot = l_run + __shfl_xor(l_run, 16, 64) + __shfl_xor(l_run, 32, 64) +
                      __shfl_xor(__shfl_xor(l_run, 16, 64), 32, 64);
  // o[c][v] of lane (j, kg) is O[column 8*(4*kg + v) + c][head j]
  if (j < CM) {
    float *mine = s_o + ((size_t)wave * CM + j) * (H + 2);
#pragma unroll
    for (int c = 0; c < 8; ++c)
#pragma unroll
      for (int v = 0; v < 4; ++v) mine[8 * (4 * kg + v) + c] = o[c][v];
    if (kg == 0) { mine[H] = m_run; mine[H + 1] = l_tot; }
  }
  __syncthreads();
  for (int i = tid; i < HW * n_cols * H; i += 512) {
    const int hwi = i / (n_cols * H), rem = i - hwi * (n_cols * H);
    const int hd = rem / H, col = rem % H;
    const int gi = it->g + hwi;
    if (gi >= a.n_kv_heads) continue;
    const int rj = hd / G, hj = hd - rj * G;
    const int orow = it->rows[rj];
    // wave kr2 * HW + hwi holds sub-range kr2 of this head
    float M = -INFINITY;
    for (int kr2 = 0; kr2 < KR; ++kr2) M = fmaxf(M, s_o[((size_t)(kr2 * HW + hwi) * CM + hd) * (H + 2) + H]);
    float acc = 0.f, den = 0.f;
    for (int kr2 = 0; kr2 < KR; ++kr2) {
      const float *src = s_o + ((size_t)(kr2 * HW + hwi) * CM + hd) * (H + 2);
      const float mw = src[H];
      const float wgt = (mw == -INFINITY) ? 0.f : __builtin_amdgcn_exp2f(mw - M);
      acc += wgt * src[col];
      den += wgt * src[H + 1];
    }
    float *pp = a.partials + (((int64_t)orow * a.n_q_heads + gi * G + hj) * a.n_parts + it->part) * (H + 2);
    pp[col] = acc;
    if (col == 0) {
      pp[H] = (M == -INFINITY) ? -INFINITY : M * DEC_LN2;     // natural-log domain for the merge kernel
      pp[H + 1] = den;
    }
  }
}

bool attn_decode_mfma_supported(const LayerDims &L) {
  const int G = L.n_q_heads / L.n_kv_heads;
  return L.head_dim == 128 && G <= 16;
}

void decode_mfma_shape(int n_kv_heads, int *heads_per_wg, int *ranges_per_wg) {
  const int hw = n_kv_heads < 8 ? n_kv_heads : 8;
  *heads_per_wg = hw;
  *ranges_per_wg = 8 / hw;
}

void launch_attn_decode_mfma(const DecodeArgs &a, int n_items, hipStream_t s) {
  if (n_items == 0) return;
  const size_t smem = (size_t)8 * a.cols_max * (128 + 2) * sizeof(float);
  // set on every launch that needs it: a host-side attribute write, safe from any thread and on any device
  if (smem > 48 * 1024)
    (void)hipFuncSetAttribute((const void *)attn_decode_mfma_kernel, hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
  hipLaunchKernelGGL(attn_decode_mfma_kernel, dim3(n_items), dim3(512), smem, s, a);
}

}  // namespace alora
