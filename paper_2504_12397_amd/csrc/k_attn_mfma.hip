// Flash-style causal attention of new queries over [cached prefix ; new suffix] (Eq.1 with the
// causal mask, rows as in Eq.6) on the gfx950 matrix cores, head_dim 128, grouped-query sharing.
//
// Operand precision.  The cache holds bf16 keys and values (storage), but inside this kernel every MFMA
// operand is fp16: the queries arrive as fp16 from the rotation step, K/V tiles are converted bf16 -> fp16 on
// their way into LDS (exact: 8 significant bits fit in 11; magnitudes beyond 65504 saturate, values below
// 2^-24 vanish), and the probabilities are packed to fp16.  With bf16 operands the rounding of q (2^-9 per
// element, amplified through the exponential) and of p dominated the error against the float64 oracle --
// 1.5e-3 and 1.2e-3 rms of the row scale, with maxima of 1-2.3e-2 over 10^6 elements, right at the 2e-2
// bar; fp16 operands cut both by 8x at the price of ~40 conversion instructions per thread and tile.
//
// Work item: one workgroup = (q-tile of 256/G tokens of one sequence, kv head, key split).
// The G query heads of the kv group are packed next to the tokens into 256 "packed rows"
// (packed row = token * G + head), 32 per wave and eight waves per workgroup, so every K/V tile
// fetched from HBM serves all heads of the group.  Two waves share a SIMD, so the softmax of one
// (exponentials and rescaling on the vector ALU) can in principle run under the matrix work of the
// other; measured, the tile time is close to the sum of its parts (MFMAs 1.59 us, softmax 0.35,
// tile loads 0.27, LDS reads 0.17, LDS stores 0.14 of 2.37 us per 256 x 64 tile).
//
// Per 64-key tile, each wave computes S^T = K Q^T (keys are MFMA rows, packed query rows are
// MFMA columns).  In that orientation a lane owns one query row (column l%32) in every
// accumulator register, so the online-softmax state (running max, running sum, rescale
// factor) is one scalar per lane and the probabilities can be fed straight back, from
// registers, as the B operand of O^T += V^T P^T.  The only data that needs a transpose is V:
// the loader threads turn 4 keys x 8 columns into 8 columns x 4 keys in registers (byte
// permutes) and store V^T tiles to LDS in the exact k-order the P registers have.
//
// K tile in LDS: [64 keys][16 chunks of 16 B], chunk c of key r at c ^ (r & 15).
// V^T tile in LDS: [128 columns][8 chunks of 16 B]; chunk (2*s4 + kh) of a column holds keys
//   32*(s4/2) + 16*(s4%2) + {4kh..4kh+3, 8+4kh..8+4kh+3}  (s4 = k-step 0..3, kh = lane/32),
//   stored at chunk ^ v_swz(column).
#include <type_traits>

#include "mfma_kernels.h"

namespace alora {

typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float f32x16;

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

__device__ __forceinline__ f16x8 u4_as_f16x8(u32x4 u) { return __builtin_bit_cast(f16x8, u); }

__device__ __forceinline__ uint32_t pack_bf16x2(float a, float b) {
  typedef __attribute__((__vector_size__(2 * sizeof(__bf16)))) __bf16 bf16x2;
  bf16x2 p;
  p[0] = (bf16)a;
  p[1] = (bf16)b;
  return __builtin_bit_cast(uint32_t, p);
}

// two floats as an fp16 pair (v_cvt_pkrtz_f16_f32: one instruction, round toward zero, so a finite value
// never becomes infinite).  Used for the probabilities -- numerator and denominator of the softmax are both
// taken from the packed values, so the rounding direction cancels -- and for bf16 values, where it is exact.
__device__ __forceinline__ uint32_t pack_f16x2(float a, float b) {
  return __builtin_bit_cast(uint32_t, __builtin_amdgcn_cvt_pkrtz(a, b));
}
// the two bf16 halves of a word as floats
__device__ __forceinline__ float bf16_lo(uint32_t w) { return __builtin_bit_cast(float, w << 16); }
__device__ __forceinline__ float bf16_hi(uint32_t w) { return __builtin_bit_cast(float, w & 0xffff0000u); }
// a word of two bf16 -> a word of two fp16
__device__ __forceinline__ uint32_t bf16x2_to_f16x2(uint32_t w) { return pack_f16x2(bf16_lo(w), bf16_hi(w)); }

// chunk swizzle of the V^T tile (128-byte rows).  LDS serves 16 lanes at a time over 64 banks:
// 16 consecutive columns of one chunk (operand reads) must land on 16 distinct 16-byte slots
// modulo 256 B, which (col >> 1) & 7 together with the row parity gives; the extra col >> 4 term
// spreads the transposing 8-byte stores (columns 4 apart) to a 2-way conflict at worst.
__device__ __forceinline__ int v_swz(int col) { return ((col >> 1) ^ (col >> 4)) & 7; }

// max of a value with the one held by the lane 32 away.  v_permlane32_swap trades lanes 32..63 of its
// first register with lanes 0..31 of its second; given two copies of x, the first then holds the low
// half's values in both halves and the second the high half's.  Written as inline assembly because
// the compiler builtin hands back its first result for both (the maximum then silently covers one
// half only); the s_nop's are the wait states between a vector write and this instruction's read.
__device__ __forceinline__ float max_with_other_half(float x) {
  float lo = x, hi = x;
  asm volatile("s_nop 1\n\tv_permlane32_swap_b32 %0, %1\n\ts_nop 1\n\tv_max_f32 %0, %0, %1" : "+v"(lo), "+v"(hi));
  return lo;
}

// acc + lo + hi of a packed fp16 pair (v_dot2_f32_f16 against (1, 1)): products and sum in fp32
__device__ __forceinline__ float sum_f16x2(uint32_t pair, float acc) {
  typedef _Float16 half2_t __attribute__((ext_vector_type(2)));
  return __builtin_amdgcn_fdot2(__builtin_bit_cast(half2_t, pair), __builtin_bit_cast(half2_t, 0x3c003c00u), acc, false);
}

// Waits for every outstanding global load (s_waitcnt vmcnt(0); the other counters left alone).
// Used once before the key loops: the query fragments are loaded before a conditional prologue,
// and unless their loads are known to be complete on every path into the loop the compiler guards
// each use of them inside the loop with a vmcnt wait -- which, the counter being in-order, also
// drains the K/V prefetches that are supposed to stay in flight.
__device__ __forceinline__ void wait_all_global_loads() { __builtin_amdgcn_s_waitcnt(0x0F70); }

constexpr int ATT_BN = 64;        // keys per tile
constexpr float LOG2E = 1.4426950408889634f;
constexpr float LN2 = 0.6931471805599453f;

// PFX: tile loads with full 64-bit address arithmetic (items whose keys lie beyond 2 GB from their first row)
// instead of buffer loads with 32-bit offsets
//
// FOLD: the queries arrive premultiplied by sm_scale * log2(e) (the rotation kernel does it while it
// rounds them), and the softmax bookkeeping moves onto the matrix unit:
//   * the accumulator of the first K Q^T product starts at -m_ref (the row's reference exponent,
//     replicated over the lane's 16 registers), so the scores come out as s - m_ref, ready for exp2;
//   * the row sums are taken on the vector ALU from the packed probabilities (v_dot2_f32_f16 against (1, 1)),
//     so numerator and denominator see the same rounded values; each half of the wave sums the keys it holds and
//     the two halves are added once, at the end (they share the reference exponent);
//   * m_ref is set to the exact maximum of the first block in which the row sees a key, and later moves
//     only when a block's maximum exceeds it by more than `lazy`, in a branch that is rare.
// The softmax is the same function: numerator and denominator share the reference exponent.
template <int G, int NW, bool PFX, bool FOLD>      // NW waves per workgroup (8 or 4), 32 packed rows each
__global__ __launch_bounds__(64 * NW) void attn_prefill_mfma_kernel(AttnArgs a) {
  constexpr int H = 128;
  constexpr int NT = 64 * NW;
  constexpr int NB = 1;             // 32-row query blocks per wave
  __shared__ u32x4 Ks[2][ATT_BN * 16];
  __shared__ u32x4 Vs[2][H * 8];

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int l32 = lane & 31, kh = lane >> 5;
  // work list built by the host: one item per workgroup -- up to TQ consecutive packed rows against one range of
  // key positions of one kv head -- ordered so that the items that stream the same keys and values sit on one XCD
  // (one L2) together.  The rows of an item belong to one sequence (the causal mask uses pos0 + token), or to
  // several consecutive sequences over the shared prefix they all name (no mask needed: pos0 is out of reach).
  const AttnItem wk = a.work[blockIdx.x];
  if (wk.ntok <= 0) return;
  const int g = wk.g, split = wk.part;
  const int ntok = wk.ntok;
  const int row0 = wk.row0;
  const int n_visible = wk.n_addr;                   // key positions addressable from key_row0
  const int kbeg = wk.kbeg, kend = wk.kend;
  const int ntiles = kend > kbeg ? (kend - kbeg + ATT_BN - 1) / ATT_BN : 0;
  const bf16 *Kp = a.K + wk.key_row0 * a.n_kv + g * H;
  const bf16 *Vp = a.V + wk.key_row0 * a.n_kv + g * H;
  const int first_pos = wk.pos0;                     // smallest query position in the tile

  // ---- this wave's queries as B operands: 2 column blocks x 8 k-steps ---------------------
  u32x4 qf[NB][8];
  int pos[NB], tok[NB], head[NB];
#pragma unroll
  for (int nb = 0; nb < NB; ++nb) {
    const int pr = wave * (32 * NB) + nb * 32 + l32;
    tok[nb] = pr / G;
    head[nb] = g * G + pr % G;
    const int tc = min(tok[nb], ntok - 1);
    pos[nb] = tok[nb] < ntok ? first_pos + tok[nb] : -1;       // -1: padding row, sees nothing
    const _Float16 *qp = a.Q + (int64_t)(row0 + tc) * a.n_q + head[nb] * H + kh * 8;
#pragma unroll
    for (int ks = 0; ks < 8; ++ks) qf[nb][ks] = *reinterpret_cast<const u32x4 *>(qp + ks * 16);
  }

  f32x16 o[4][NB];
#pragma unroll
  for (int cb = 0; cb < 4; ++cb)
#pragma unroll
    for (int nb = 0; nb < NB; ++nb)
#pragma unroll
      for (int v = 0; v < 16; ++v) o[cb][nb][v] = 0.f;
  const float c_scale = a.sm_scale * LOG2E;
  // softmax state of the lane's query row: the reference exponent m_ref (exp2 domain), the sum l_run of the
  // probabilities of the keys this half of the wave holds (for FOLD the score accumulators start at -m_ref)
  float m_ref = FOLD ? 0.f : -INFINITY;
  float l_run = 0.f;
  bool seen = false;        // the row has met a visible key (the same in both halves: derived from the shared maximum)

  // ---- tile loader: K rows as they are, V transposed in registers -------------------------
  // 512 threads: K = 1024 chunks of 16 B, two per thread; V = 16 key quads x 32 column groups of
  // 4, one (quad, group) per thread: four 8-byte loads become four columns x four keys.
  // Two tiles are kept in flight in registers (sets 0 and 1) on top of the one being consumed
  // from LDS: one tile of compute is shorter than the HBM latency.
  constexpr int KC = 1024 / NT;          // 16-byte K chunks per thread and tile
  constexpr int CW = 2048 / NT;          // V columns per thread (for 4 keys): 4 or 8
  constexpr int VW = CW / 2;             // 32-bit words per key
  typedef uint32_t vword __attribute__((ext_vector_type(VW)));
  u32x4 rk0[KC], rk1[KC];
  vword rv0[4], rv1[4];
  const int v_qd = tid / (H / CW), v_cg = tid % (H / CW);
  // Without shared prefixes the tile loads are buffer loads: a resource that covers exactly the rows
  // [0, n_visible) of this sequence and kv head, per-lane byte offsets that never change, and the tile's
  // first row as the scalar offset -- no address arithmetic per load, and rows past the end read as zero
  // (the range check of the buffer resource) instead of needing a clamp.  (The host takes the other path
  // when a sequence is too long for 32-bit byte offsets.)
  const uint32_t row_bytes = (uint32_t)a.n_kv * 2u;
  __amdgpu_buffer_rsrc_t k_rsrc, v_rsrc;
  uint32_t k_off[KC], v_off[4];
  if constexpr (!PFX) {
    const int n_rec = (int)(((uint32_t)max(n_visible, 1) - 1u) * row_bytes + H * 2u);
    k_rsrc = __builtin_amdgcn_make_buffer_rsrc((void *)Kp, 0, n_rec, 0x00020000);
    v_rsrc = __builtin_amdgcn_make_buffer_rsrc((void *)Vp, 0, n_rec, 0x00020000);
#pragma unroll
    for (int i = 0; i < KC; ++i) {
      const int q = tid + i * NT;
      k_off[i] = (uint32_t)(q >> 4) * row_bytes + (q & 15) * 16u;
    }
#pragma unroll
    for (int i = 0; i < 4; ++i) v_off[i] = (uint32_t)(v_qd * 4 + i) * row_bytes + v_cg * (CW * 2u);
  }
  auto load_tile = [&](int t, u32x4 (&rk)[KC], vword (&rv)[4]) {
    const int k0 = kbeg + t * ATT_BN;
    if constexpr (!PFX) {
      const int s_off = __builtin_amdgcn_readfirstlane((int)((uint32_t)k0 * row_bytes));
#pragma unroll
      for (int i = 0; i < KC; ++i)
        rk[i] = __builtin_bit_cast(u32x4, __builtin_amdgcn_raw_buffer_load_b128(k_rsrc, (int)k_off[i], s_off, 0));
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        if constexpr (VW == 2) rv[i] = __builtin_bit_cast(vword, __builtin_amdgcn_raw_buffer_load_b64(v_rsrc, (int)v_off[i], s_off, 0));
        else rv[i] = __builtin_bit_cast(vword, __builtin_amdgcn_raw_buffer_load_b128(v_rsrc, (int)v_off[i], s_off, 0));
      }
    } else {
#pragma unroll
      for (int i = 0; i < KC; ++i) {
        const int q = tid + i * NT, key = q >> 4, c = q & 15;
        const int kidx = min(k0 + key, n_visible - 1);
        const int64_t e = (int64_t)kidx * a.n_kv + c * 8;
        rk[i] = *reinterpret_cast<const u32x4 *>(Kp + e);
      }
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const int kidx = min(k0 + v_qd * 4 + i, n_visible - 1);
        const int64_t e = (int64_t)kidx * a.n_kv + v_cg * CW;
        rv[i] = *reinterpret_cast<const vword *>(Vp + e);
      }
    }
  };
  auto store_k = [&](int buf, const u32x4 (&rk)[KC]) {
#pragma unroll
    for (int i = 0; i < KC; ++i) {
      const int q = tid + i * NT, key = q >> 4, c = q & 15;
      Ks[buf][key * 16 + (c ^ (key & 15))] = u32x4{bf16x2_to_f16x2(rk[i].x), bf16x2_to_f16x2(rk[i].y),
                                                   bf16x2_to_f16x2(rk[i].z), bf16x2_to_f16x2(rk[i].w)};
    }
  };
  auto store_v = [&](int buf, const vword (&rv)[4]) {
    // V: this thread holds keys 4*v_qd..+3 for columns CW*v_cg..+CW-1
    const int grp16 = v_qd >> 2, qi = v_qd & 3;
    const int vkh = qi & 1, halfpos = qi >> 1;
    const int vchunk = grp16 * 2 + vkh;
    u32x2 *vs2 = reinterpret_cast<u32x2 *>(Vs[buf]);
#pragma unroll
    for (int j = 0; j < VW; ++j) {
      // even column 2j: low halves; odd column 2j+1: high halves.  The conversion to fp16 packs two keys of one
      // column into a word, which is the transposition.
      u32x2 ev, od;
      ev.x = pack_f16x2(bf16_lo(rv[0][j]), bf16_lo(rv[1][j]));
      ev.y = pack_f16x2(bf16_lo(rv[2][j]), bf16_lo(rv[3][j]));
      od.x = pack_f16x2(bf16_hi(rv[0][j]), bf16_hi(rv[1][j]));
      od.y = pack_f16x2(bf16_hi(rv[2][j]), bf16_hi(rv[3][j]));
      const int c0 = v_cg * CW + 2 * j, c1 = c0 + 1;
      vs2[(c0 * 8 + (vchunk ^ v_swz(c0))) * 2 + halfpos] = ev;
      vs2[(c1 * 8 + (vchunk ^ v_swz(c1))) * 2 + halfpos] = od;
    }
  };

  // A 64-key tile is consumed as two 32-key blocks, each with its own softmax update, so that only one
  // block of scores and probabilities is live at a time.  The three steps of a block:
  f32x16 sv;            // scores of the block in flight, then its probabilities
  u32x4 pf[2];          // the probabilities as fp16: [half of the block's keys] x 8
  // ---- S^T = K Q^T ------------------------------------------------------------------------------
  auto qk = [&](int buf, int kb) {
    // all eight K fragments of this key block are fetched from LDS first: with one MFMA per
    // fragment there is nothing else to hide the LDS latency behind
    f16x8 kf[8];
    const int key = kb * 32 + l32;
#pragma unroll
    for (int ks = 0; ks < 8; ++ks) kf[ks] = u4_as_f16x8(Ks[buf][key * 16 + ((2 * ks + kh) ^ (key & 15))]);
    if constexpr (FOLD) {
      const float neg_m = -m_ref;
#pragma unroll
      for (int v = 0; v < 16; ++v) sv[v] = neg_m;
    } else {
#pragma unroll
      for (int v = 0; v < 16; ++v) sv[v] = 0.f;
    }
#pragma unroll
    for (int ks = 0; ks < 8; ++ks) sv = __builtin_amdgcn_mfma_f32_32x32x16_f16(kf[ks], u4_as_f16x8(qf[0][ks]), sv, 0, 0, 0);
  };
  // ---- causal mask and online softmax (log2 domain), one query row per lane -----------------------
  auto softmax = [&](int t, int kb) {
    const int k0 = kbeg + t * ATT_BN;
    // only tiles that reach past the first query position or the split end need the mask
    if ((k0 + ATT_BN - 1 > first_pos) || (k0 + ATT_BN > kend)) {
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        const int key = k0 + kb * 32 + 8 * (v >> 2) + 4 * kh + (v & 3);
        if (key > pos[0] || key >= kend) sv[v] = -INFINITY;
      }
    }
    float mx = sv[0];
#pragma unroll
    for (int v = 1; v < 16; ++v) mx = fmaxf(mx, sv[v]);
    if constexpr (!FOLD) mx = max_with_other_half(mx);
    // The reference exponent of a row moves (and its 64 output accumulators and row sum are rescaled)
    // only in blocks where some row of the wave needs it -- a wave-uniform, rare branch: with random
    // scores a third of all blocks would otherwise move the maximum of some row.  The softmax is
    // mathematically unchanged (numerator and denominator share the reference); probabilities reach
    // 2^lazy instead of 1, with the same relative bf16 rounding.
    if constexpr (FOLD) {
      // sv holds s - m_ref.  A row's first keys set the reference to their exact maximum (the largest
      // probability is then exactly 1, which matters most for rows that see few keys).
      // mx covers the keys of this half of the wave.  Whether ANY row of the wave has to move is decided from the
      // half maxima (some half exceeds the threshold exactly when its row does); the exchange between the two
      // halves of a row is needed only inside the rare branch.  A row's `seen` flag changes only there too: a half
      // that meets its first key wants the branch, and both halves then take the row's maximum.
      if (__any(mx > a.lazy || (!seen && mx > -INFINITY))) {
        mx = max_with_other_half(mx);
        const bool fresh = !seen;              // nothing accumulated for this row yet
        const bool want = mx > a.lazy || (fresh && mx > -INFINITY);
        seen = seen || mx > -INFINITY;
        const float delta = want ? mx : 0.f;
        const float alpha = fresh ? 1.0f : __builtin_amdgcn_exp2f(-delta);
        m_ref += delta;
        l_run *= alpha;
#pragma unroll
        for (int v = 0; v < 16; ++v) sv[v] -= delta;
#pragma unroll
        for (int cb = 0; cb < 4; ++cb)
#pragma unroll
          for (int v = 0; v < 16; ++v) o[cb][0][v] *= alpha;
      }
#pragma unroll
      for (int v = 0; v < 16; ++v) sv[v] = __builtin_amdgcn_exp2f(sv[v]);
    } else {
      // sv holds raw scores; m_ref is in the exp2 domain (score * sm_scale * log2 e)
      const float m_blk = mx * c_scale;
      const bool move = __any(m_blk > m_ref + a.lazy);
      const float m_new = move ? fmaxf(m_ref, m_blk) : m_ref;
      const float m_safe = (m_new == -INFINITY) ? 0.f : m_new;
      if (move) {
        const float alpha = __builtin_amdgcn_exp2f(m_ref - m_safe);
        l_run *= alpha;
#pragma unroll
        for (int cb = 0; cb < 4; ++cb)
#pragma unroll
          for (int v = 0; v < 16; ++v) o[cb][0][v] *= alpha;
      }
      m_ref = m_new;
#pragma unroll
      for (int v = 0; v < 16; ++v) sv[v] = __builtin_amdgcn_exp2f(fmaf(sv[v], c_scale, -m_safe));
    }
#pragma unroll
    for (int hf = 0; hf < 2; ++hf) {
      const int e = 8 * hf;
      pf[hf] = u32x4{pack_f16x2(sv[e], sv[e + 1]), pack_f16x2(sv[e + 2], sv[e + 3]), pack_f16x2(sv[e + 4], sv[e + 5]),
                     pack_f16x2(sv[e + 6], sv[e + 7])};
      // row sum of the PACKED probabilities (the values the products below use)
      l_run = sum_f16x2(pf[hf].x, l_run);
      l_run = sum_f16x2(pf[hf].y, l_run);
      l_run = sum_f16x2(pf[hf].z, l_run);
      l_run = sum_f16x2(pf[hf].w, l_run);
    }
  };
  // ---- O^T += V^T P^T ----------------------------------------------------------------------------------
  auto pv = [&](int buf, int kb) {
    f16x8 vf[2][4];
#pragma unroll
    for (int hf = 0; hf < 2; ++hf)
#pragma unroll
      for (int cb = 0; cb < 4; ++cb) {
        const int col = cb * 32 + l32, c = 2 * (kb * 2 + hf) + kh;
        vf[hf][cb] = u4_as_f16x8(Vs[buf][col * 8 + (c ^ v_swz(col))]);
      }
#pragma unroll
    for (int hf = 0; hf < 2; ++hf)
#pragma unroll
      for (int cb = 0; cb < 4; ++cb)
        o[cb][0] = __builtin_amdgcn_mfma_f32_32x32x16_f16(vf[hf][cb], u4_as_f16x8(pf[hf]), o[cb][0], 0, 0, 0);
  };

  {
    auto compute_tile = [&](int buf, int t) {
#pragma unroll
      for (int kb = 0; kb < 2; ++kb) {
        qk(buf, kb);
        softmax(t, kb);
        pv(buf, kb);
      }
    };
    // Loads and stores in the loop are unconditional (tile indices clamped) so that the compiler's
    // count of outstanding loads is exact and it waits only for the tile it is about to store.
    if (ntiles > 0) {
      load_tile(0, rk0, rv0);
      load_tile(min(1, ntiles - 1), rk1, rv1);
      store_k(0, rk0);
      store_v(0, rv0);
    }
    __syncthreads();
    wait_all_global_loads();
    for (int t = 0; t < ntiles; t += 2) {
      load_tile(min(t + 2, ntiles - 1), rk0, rv0);
      compute_tile(0, t);
      store_k(1, rk1);
      store_v(1, rv1);
      __syncthreads();
      load_tile(min(t + 3, ntiles - 1), rk1, rv1);
      if (t + 1 < ntiles) compute_tile(1, t + 1);
      store_k(0, rk0);
      store_v(0, rv0);
      __syncthreads();
    }
  }

  // ---- write the partial (or final) result ----------------------------------------------------
#pragma unroll
  for (int nb = 0; nb < NB; ++nb) {
    const float l_tot = l_run + __shfl_xor(l_run, 32, 64);      // the two halves of the wave hold disjoint keys
    if (tok[nb] >= ntok) continue;
    const int64_t row = row0 + tok[nb];
    if (a.out != nullptr) {
      const float inv = 1.0f / l_tot;
      bf16 *op = a.out + row * a.n_q + head[nb] * H;
#pragma unroll
      for (int cb = 0; cb < 4; ++cb)
#pragma unroll
        for (int v4 = 0; v4 < 4; ++v4) {
          const int col = cb * 32 + 8 * v4 + 4 * kh;
          uint2 w;
          w.x = pack_bf16x2(o[cb][nb][4 * v4] * inv, o[cb][nb][4 * v4 + 1] * inv);
          w.y = pack_bf16x2(o[cb][nb][4 * v4 + 2] * inv, o[cb][nb][4 * v4 + 3] * inv);
          *reinterpret_cast<uint2 *>(op + col) = w;
        }
    } else if (a.compact) {
      // compact partial record (ATTN_REC16 bytes): the unnormalised accumulators of the row divided by their
      // largest magnitude, as 128 fp16 values (relative precision 2^-11, finer than the bf16 the merged result
      // is rounded to; no overflow whatever the values), then that magnitude, the reference and the row sum.
      // Half the bytes of the fp32 record -- and these records are most of what a short call writes and reads.
      float amax = 0.f;
#pragma unroll
      for (int cb = 0; cb < 4; ++cb)
#pragma unroll
        for (int v = 0; v < 16; ++v) amax = fmaxf(amax, fabsf(o[cb][nb][v]));
      amax = max_with_other_half(amax);
      const float rs = amax > 0.f ? 1.0f / amax : 0.f;
      char *rec = reinterpret_cast<char *>(a.partials) +
                  ((row * a.n_q_heads + head[nb]) * a.n_parts + split) * (int64_t)ATTN_REC16;
      typedef __attribute__((__vector_size__(4 * sizeof(_Float16)))) _Float16 half4_t;
#pragma unroll
      for (int cb = 0; cb < 4; ++cb)
#pragma unroll
        for (int v4 = 0; v4 < 4; ++v4) {
          const int col = cb * 32 + 8 * v4 + 4 * kh;
          half4_t hv;
#pragma unroll
          for (int i = 0; i < 4; ++i) hv[i] = (_Float16)(o[cb][nb][4 * v4 + i] * rs);
          *reinterpret_cast<half4_t *>(rec + col * 2) = hv;
        }
      if (kh == 0) {
        float *tail = reinterpret_cast<float *>(rec + 2 * H);
        tail[0] = (l_tot == 0.f || m_ref == -INFINITY) ? -INFINITY : m_ref * LN2;
        tail[1] = l_tot;
        tail[2] = amax;
      }
    } else {
      float *pp = a.partials + ((row * a.n_q_heads + head[nb]) * a.n_parts + split) * (H + 2);
#pragma unroll
      for (int cb = 0; cb < 4; ++cb)
#pragma unroll
        for (int v4 = 0; v4 < 4; ++v4) {
          const int col = cb * 32 + 8 * v4 + 4 * kh;
          // (H + 2) floats per record keeps 8-byte, not 16-byte, alignment
          *reinterpret_cast<float2 *>(pp + col) = make_float2(o[cb][nb][4 * v4], o[cb][nb][4 * v4 + 1]);
          *reinterpret_cast<float2 *>(pp + col + 2) = make_float2(o[cb][nb][4 * v4 + 2], o[cb][nb][4 * v4 + 3]);
        }
      if (kh == 0) {
        // natural-log domain; a row that saw no key keeps -inf so that the merge gives it no weight
        pp[H] = (l_tot == 0.f || m_ref == -INFINITY) ? -INFINITY : m_ref * LN2;
        pp[H + 1] = l_tot;
      }
    }
  }
}



bool attn_prefill_mfma_supported(const LayerDims &L) {
  const int G = L.n_q_heads / L.n_kv_heads;
  return L.head_dim == 128 && (G == 1 || G == 2 || G == 4 || G == 8);
}

int attn_prefill_mfma_tokens_per_tile(const LayerDims &L, int waves) {
  return 32 * waves / (L.n_q_heads / L.n_kv_heads);
}

template <int NW, bool PFX, bool FOLD>
static void launch_attn_nw(const AttnArgs &a, int n_work, int G, hipStream_t s) {
  dim3 grid(n_work);
  switch (G) {
    case 1: hipLaunchKernelGGL((attn_prefill_mfma_kernel<1, NW, PFX, FOLD>), grid, dim3(64 * NW), 0, s, a); break;
    case 2: hipLaunchKernelGGL((attn_prefill_mfma_kernel<2, NW, PFX, FOLD>), grid, dim3(64 * NW), 0, s, a); break;
    case 4: hipLaunchKernelGGL((attn_prefill_mfma_kernel<4, NW, PFX, FOLD>), grid, dim3(64 * NW), 0, s, a); break;
    case 8: hipLaunchKernelGGL((attn_prefill_mfma_kernel<8, NW, PFX, FOLD>), grid, dim3(64 * NW), 0, s, a); break;
    default: break;
  }
}

template <int NW>
static void launch_attn_nw_any(const AttnArgs &a, int n_work, int G, bool prefix, hipStream_t s) {
  if (a.q_prescaled) {
    if (prefix) launch_attn_nw<NW, true, true>(a, n_work, G, s);
    else launch_attn_nw<NW, false, true>(a, n_work, G, s);
  } else {
    if (prefix) launch_attn_nw<NW, true, false>(a, n_work, G, s);
    else launch_attn_nw<NW, false, false>(a, n_work, G, s);
  }
}

// Log-sum-exp merge of the compact partial records (Eq.1 over the union of the key splits): one wave per
// (row, head), a lane two columns.  out = sum_i w_i amax_i u_i / sum_i w_i l_i with w_i = exp(m_i - max m).
__global__ __launch_bounds__(256) void attn_merge16_kernel(const char *__restrict__ part, int n_splits, int64_t n_rh,
                                                           bf16 *__restrict__ out) {
  const int lane = threadIdx.x & 63;
  const int64_t rh = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
  if (rh >= n_rh) return;
  const char *p = part + rh * n_splits * (int64_t)ATTN_REC16;
  typedef __attribute__((__vector_size__(2 * sizeof(_Float16)))) _Float16 half2_t;
  float M = -INFINITY;
  for (int s0 = 0; s0 < n_splits; s0 += 64) {
    const int sp = s0 + lane;
    M = fmaxf(M, sp < n_splits ? *reinterpret_cast<const float *>(p + sp * (int64_t)ATTN_REC16 + 256) : -INFINITY);
  }
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) M = fmaxf(M, __shfl_xor(M, o, 64));
  float denom = 0.f, a0 = 0.f, a1 = 0.f;
  for (int s0 = 0; s0 < n_splits; s0 += 8) {       // eight records requested together
    float ms[8], ls[8], am[8];
    half2_t u[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      const char *r = p + min(s0 + i, n_splits - 1) * (int64_t)ATTN_REC16;
      const float *tail = reinterpret_cast<const float *>(r + 256);
      ms[i] = tail[0]; ls[i] = tail[1]; am[i] = tail[2];
      u[i] = *reinterpret_cast<const half2_t *>(r + lane * 4);
    }
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      const float w = (s0 + i >= n_splits || ms[i] == -INFINITY) ? 0.f : __expf(ms[i] - M);
      denom += w * ls[i];
      a0 += w * am[i] * (float)u[i][0];
      a1 += w * am[i] * (float)u[i][1];
    }
  }
  const float inv = 1.0f / denom;
  typedef __attribute__((__vector_size__(2 * sizeof(__bf16)))) __bf16 bf16x2_t;
  bf16x2_t ov;
  ov[0] = (bf16)(a0 * inv);
  ov[1] = (bf16)(a1 * inv);
  *reinterpret_cast<bf16x2_t *>(out + rh * 128 + lane * 2) = ov;
}

void launch_attn_merge16(const float *partials, const LayerDims &L, int T_rows, int n_splits, bf16 *out, hipStream_t s) {
  if (T_rows == 0) return;
  const int64_t n_rh = (int64_t)T_rows * L.n_q_heads;
  hipLaunchKernelGGL(attn_merge16_kernel, dim3((unsigned)((n_rh + 3) / 4)), dim3(256), 0, s, (const char *)partials,
                     n_splits, n_rh, out);
}

void launch_attn_prefill_mfma(const AttnArgs &a, int n_work, int G, int waves, bool prefix, hipStream_t s) {
  if (n_work == 0) return;
  if (waves == 4) launch_attn_nw_any<4>(a, n_work, G, prefix, s);
  else launch_attn_nw_any<8>(a, n_work, G, prefix, s);
}

// What the rotation kernel multiplies the queries by: the folded softmax wants them in the exp2 domain,
// otherwise the kernel applies sm_scale itself.
float attn_prefill_mfma_q_scale(const LayerDims &L, bool fold) {
  return fold ? LOG2E / sqrtf((float)L.head_dim) : 1.0f;
}

}  // namespace alora
