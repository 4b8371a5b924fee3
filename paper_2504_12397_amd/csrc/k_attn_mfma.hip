// Flash-style causal attention of new queries over [cached prefix ; new suffix] (Eq.1 with the
// causal mask, rows as in Eq.6) with bf16 MFMA on gfx950, head_dim 128, grouped-query sharing.
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

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float f32x16;

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

__device__ __forceinline__ bf16x8 u4_as_bf16x8(u32x4 u) { return __builtin_bit_cast(bf16x8, u); }

__device__ __forceinline__ uint32_t pack_bf16x2(float a, float b) {
  typedef __attribute__((__vector_size__(2 * sizeof(__bf16)))) __bf16 bf16x2;
  bf16x2 p;
  p[0] = (bf16)a;
  p[1] = (bf16)b;
  return __builtin_bit_cast(uint32_t, p);
}

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

// acc + lo + hi of a packed bf16 pair (v_dot2c_f32_bf16 against (1, 1))
__device__ __forceinline__ float sum_bf16x2(uint32_t pair, float acc) {
  typedef __attribute__((__vector_size__(2 * sizeof(__bf16)))) __bf16 bf16x2;
  return __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2, pair), __builtin_bit_cast(bf16x2, 0x3f803f80u), acc,
                                         false);
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

// PFX: some sequence of the call reads a shared prefix (cached position j < prefix_len lives in
// another place of the pool than the sequence's own rows)
//
// FOLD: the queries arrive premultiplied by sm_scale * log2(e) (the rotation kernel does it while it
// rounds them), and the softmax bookkeeping moves onto the matrix unit:
//   * the accumulator of the first K Q^T product starts at -m_ref (the row's reference exponent,
//     replicated over the lane's 16 registers), so the scores come out as s - m_ref, ready for exp2;
//   * the row sums are two more MFMAs per 32-key block, an all-ones A operand against the rounded
//     probabilities, which leave the sum over all 32 keys in every register of `lacc` (no
//     cross-half exchange, and numerator and denominator see the same rounded values);
//   * m_ref is set to the exact maximum of the first block in which the row sees a key, and later moves
//     only when a block's maximum exceeds it by more than `lazy`, in a branch that is rare.
// The softmax is the same function: numerator and denominator share the reference exponent.
template <int G, int NW, bool PFX, bool FOLD>      // NW waves per workgroup (8 or 4), 32 packed rows each
__global__ __launch_bounds__(64 * NW) void attn_prefill_mfma_kernel(AttnArgs a) {
  constexpr int H = 128;
  constexpr int NT = 64 * NW;
  constexpr int TQ = 32 * NW / G;
  constexpr int NB = 1;             // 32-row query blocks per wave
  __shared__ u32x4 Ks[2][ATT_BN * 16];
  __shared__ u32x4 Vs[2][H * 8];

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int l32 = lane & 31, kh = lane >> 5;
  // work list built by the host: (sequence, first token of the q-tile, kv head, key split), ordered
  // so that the q-tiles that stream the same keys and values sit on one XCD (one L2) together
  const int4 wk = a.work[blockIdx.x];
  if (wk.x < 0) return;
  const int g = wk.z, split = wk.w;
  const SeqMeta sm = a.seqs[wk.x];
  const int q0 = wk.y;
  const int ntok = min(TQ, sm.n_new - q0);
  const int row0 = sm.row_start + q0;
  const int n_visible = sm.P + q0 + ntok;            // keys visible to the tile's last token
  int chunk = (n_visible + a.n_splits - 1) / a.n_splits;
  chunk = (chunk + ATT_BN - 1) & ~(ATT_BN - 1);
  const int kbeg = split * chunk, kend = min(n_visible, kbeg + chunk);
  const int ntiles = kend > kbeg ? (kend - kbeg + ATT_BN - 1) / ATT_BN : 0;
  const bf16 *Kp = a.K + sm.pool_off * a.n_kv + g * H;
  const bf16 *Vp = a.V + sm.pool_off * a.n_kv + g * H;
  // offset (in elements) that turns an own-row address into the shared-prefix address of the same position
  const int64_t pfx_delta = PFX ? (sm.prefix_off - sm.pool_off) * a.n_kv : 0;
  const int pfx_len = PFX ? sm.prefix_len : 0;
  const int first_pos = sm.P + q0;                   // smallest query position in the tile

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
    const bf16 *qp = a.Q + (int64_t)(row0 + tc) * a.n_q + head[nb] * H + kh * 8;
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
  // softmax state of the lane's query row: the reference exponent m_ref (exp2 domain), the row sum in
  // every register of lacc (it is the accumulator of an MFMA), and for FOLD -m_ref in every register of negm
  f32x16 negm, lacc;
  float m_ref = FOLD ? 0.f : -INFINITY;
#pragma unroll
  for (int v = 0; v < 16; ++v) { negm[v] = 0.f; lacc[v] = 0.f; }
  const bf16x8 ones = u4_as_bf16x8(u32x4{0x3f803f80u, 0x3f803f80u, 0x3f803f80u, 0x3f803f80u});

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
        const int64_t e = (int64_t)kidx * a.n_kv + c * 8 + (kidx < pfx_len ? pfx_delta : 0);
        rk[i] = *reinterpret_cast<const u32x4 *>(Kp + e);
      }
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const int kidx = min(k0 + v_qd * 4 + i, n_visible - 1);
        const int64_t e = (int64_t)kidx * a.n_kv + v_cg * CW + (kidx < pfx_len ? pfx_delta : 0);
        rv[i] = *reinterpret_cast<const vword *>(Vp + e);
      }
    }
  };
  auto store_k = [&](int buf, const u32x4 (&rk)[KC]) {
#pragma unroll
    for (int i = 0; i < KC; ++i) {
      const int q = tid + i * NT, key = q >> 4, c = q & 15;
      Ks[buf][key * 16 + (c ^ (key & 15))] = rk[i];
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
      // even column 2j: low halves; odd column 2j+1: high halves
      u32x2 ev, od;
      ev.x = __builtin_amdgcn_perm(rv[1][j], rv[0][j], 0x05040100u);
      ev.y = __builtin_amdgcn_perm(rv[3][j], rv[2][j], 0x05040100u);
      od.x = __builtin_amdgcn_perm(rv[1][j], rv[0][j], 0x07060302u);
      od.y = __builtin_amdgcn_perm(rv[3][j], rv[2][j], 0x07060302u);
      const int c0 = v_cg * CW + 2 * j, c1 = c0 + 1;
      vs2[(c0 * 8 + (vchunk ^ v_swz(c0))) * 2 + halfpos] = ev;
      vs2[(c1 * 8 + (vchunk ^ v_swz(c1))) * 2 + halfpos] = od;
    }
  };

  // A 64-key tile is consumed as two 32-key blocks, each with its own softmax update, so that only one
  // block of scores and probabilities is live at a time.  The three steps of a block:
  f32x16 sv;            // scores of the block in flight, then its probabilities
  u32x4 pf[2];          // the probabilities as bf16: [half of the block's keys] x 8
  // ---- S^T = K Q^T ------------------------------------------------------------------------------
  auto qk = [&](int buf, int kb) {
    // all eight K fragments of this key block are fetched from LDS first: with one MFMA per
    // fragment there is nothing else to hide the LDS latency behind
    bf16x8 kf[8];
    const int key = kb * 32 + l32;
#pragma unroll
    for (int ks = 0; ks < 8; ++ks) kf[ks] = u4_as_bf16x8(Ks[buf][key * 16 + ((2 * ks + kh) ^ (key & 15))]);
    if constexpr (FOLD) {
      sv = negm;
    } else {
#pragma unroll
      for (int v = 0; v < 16; ++v) sv[v] = 0.f;
    }
#pragma unroll
    for (int ks = 0; ks < 8; ++ks) sv = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[ks], u4_as_bf16x8(qf[0][ks]), sv, 0, 0, 0);
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
    mx = max_with_other_half(mx);
    // The reference exponent of a row moves (and its 64 output accumulators and row sum are rescaled)
    // only in blocks where some row of the wave needs it -- a wave-uniform, rare branch: with random
    // scores a third of all blocks would otherwise move the maximum of some row.  The softmax is
    // mathematically unchanged (numerator and denominator share the reference); probabilities reach
    // 2^lazy instead of 1, with the same relative bf16 rounding.
    if constexpr (FOLD) {
      // sv holds s - m_ref.  A row's first keys set the reference to their exact maximum (the largest
      // probability is then exactly 1, which matters most for rows that see few keys).
      const bool fresh = lacc[0] == 0.f;       // nothing accumulated for this row yet
      const bool want = mx > a.lazy || (fresh && mx > -INFINITY);
      if (__any(want)) {
        const float delta = want ? mx : 0.f;
        const float alpha = fresh ? 1.0f : __builtin_amdgcn_exp2f(-delta);
        m_ref += delta;
#pragma unroll
        for (int v = 0; v < 16; ++v) { sv[v] -= delta; negm[v] -= delta; lacc[v] *= alpha; }
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
#pragma unroll
        for (int v = 0; v < 16; ++v) lacc[v] *= alpha;
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
      pf[hf] = u32x4{pack_bf16x2(sv[e], sv[e + 1]), pack_bf16x2(sv[e + 2], sv[e + 3]), pack_bf16x2(sv[e + 4], sv[e + 5]),
                     pack_bf16x2(sv[e + 6], sv[e + 7])};
    }
  };
  // ---- O^T += V^T P^T and the row sums ----------------------------------------------------------------
  auto pv = [&](int buf, int kb) {
    bf16x8 vf[2][4];
#pragma unroll
    for (int hf = 0; hf < 2; ++hf)
#pragma unroll
      for (int cb = 0; cb < 4; ++cb) {
        const int col = cb * 32 + l32, c = 2 * (kb * 2 + hf) + kh;
        vf[hf][cb] = u4_as_bf16x8(Vs[buf][col * 8 + (c ^ v_swz(col))]);
      }
#pragma unroll
    for (int hf = 0; hf < 2; ++hf)
#pragma unroll
      for (int cb = 0; cb < 4; ++cb)
        o[cb][0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf[hf][cb], u4_as_bf16x8(pf[hf]), o[cb][0], 0, 0, 0);
    // row sums of the ROUNDED probabilities (the values the products above use, so numerator and
    // denominator of the softmax carry the same rounding): an all-ones A operand leaves the sum over
    // the block's 32 keys in every register of lacc
#pragma unroll
    for (int hf = 0; hf < 2; ++hf)
      lacc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ones, u4_as_bf16x8(pf[hf]), lacc, 0, 0, 0);
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
    const float l_tot = lacc[0];
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
                  ((row * a.n_q_heads + head[nb]) * a.n_splits + split) * (int64_t)ATTN_REC16;
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
      float *pp = a.partials + ((row * a.n_q_heads + head[nb]) * a.n_splits + split) * (H + 2);
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


// ------------------------------------------------------------------------------------------------
// Software-pipelined variant (option attn_pipeline = 0; the default is the kernel above).  Same work item, layouts and arithmetic as the kernel
// above; what changes is the order in which one wave issues its work.  The loop advances in
// 32-key blocks, and in step j a wave issues, as three independent instruction streams,
//     matrix unit:  S(j+1) = K(j+1) Q^T   and   O^T += V(j-1)^T P(j-1)^T        (16 MFMAs)
//     vector ALU :  online softmax of S(j) -> P(j)
//     memory     :  LDS fragment reads for the MFMAs above, one half tile stored to LDS, one half
//                   tile requested from global memory (two tiles ahead)
// so the exponentials of one block run while the matrix unit works on its neighbours, inside the
// wave, instead of relying on another wave being in a different phase.  The rescaling of O by
// exp2(m_old - m_new) (Eq.1's softmax computed online) is applied after P(j-1) V(j-1) has been
// accumulated, which is the same value: O_j = (O_{j-2} + P_{j-1} V_{j-1}) * alpha_j.
//
// LDS buffers are double: K(t+1) is stored during the first step of tile t (its slot was last
// read two steps earlier), V(t+1) during the second (its slot was last read one step earlier);
// one barrier per step orders them.
template <int G, bool PFX>
__global__ __launch_bounds__(512) void attn_prefill_pipe_kernel(AttnArgs a) {
  constexpr int H = 128;
  constexpr int NT = 512;
  constexpr int TQ = 256 / G;
#ifndef ATT_AHEAD
#define ATT_AHEAD 6
#endif
  constexpr int AH = ATT_AHEAD;      // LDS fragment reads in flight per wave
  __shared__ u32x4 Ks[2][ATT_BN * 16];
  __shared__ u32x4 Vs[2][H * 8];

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int l32 = lane & 31, kh = lane >> 5;
  const int4 wk = a.work[blockIdx.x];
  if (wk.x < 0) return;
  const int g = wk.z, split = wk.w;
  const SeqMeta sm = a.seqs[wk.x];
  const int q0 = wk.y;
  const int ntok = min(TQ, sm.n_new - q0);
  const int row0 = sm.row_start + q0;
  const int n_visible = sm.P + q0 + ntok;
  int chunk = (n_visible + a.n_splits - 1) / a.n_splits;
  chunk = (chunk + ATT_BN - 1) & ~(ATT_BN - 1);
  const int kbeg = split * chunk, kend = min(n_visible, kbeg + chunk);
  const int ntiles = kend > kbeg ? (kend - kbeg + ATT_BN - 1) / ATT_BN : 0;
  const bf16 *Kp = a.K + sm.pool_off * a.n_kv + g * H;
  const bf16 *Vp = a.V + sm.pool_off * a.n_kv + g * H;
  // offset (in elements) that turns an own-row address into the shared-prefix address of the same position
  const int64_t pfx_delta = PFX ? (sm.prefix_off - sm.pool_off) * a.n_kv : 0;
  const int pfx_len = PFX ? sm.prefix_len : 0;
  const int first_pos = sm.P + q0;

  const int pr = wave * 32 + l32;
  const int tok = pr / G, head = g * G + pr % G;
  const int pos = tok < ntok ? first_pos + tok : -1;
  u32x4 qf[8];
  {
    const bf16 *qp = a.Q + (int64_t)(row0 + min(tok, ntok - 1)) * a.n_q + head * H + kh * 8;
#pragma unroll
    for (int ks = 0; ks < 8; ++ks) qf[ks] = *reinterpret_cast<const u32x4 *>(qp + ks * 16);
  }
  f32x16 o[4];
#pragma unroll
  for (int cb = 0; cb < 4; ++cb)
#pragma unroll
    for (int v = 0; v < 16; ++v) o[cb][v] = 0.f;
  float m_run = -INFINITY, l_run = 0.f;
  const float c_scale = a.sm_scale * LOG2E;

  // ---- loaders: as in the kernel above, K and V handled separately ----------------------------
  u32x4 rkA[2];
  u32x2 rvA[4];
  const int v_qd = tid >> 5, v_cg = tid & 31;
  auto load_k = [&](int t, u32x4 (&rk)[2]) {
    const int k0 = kbeg + min(t, ntiles - 1) * ATT_BN;
#pragma unroll
    for (int i = 0; i < 2; ++i) {
      const int q = tid + i * NT, key = q >> 4, c = q & 15;
      const int kidx = min(k0 + key, n_visible - 1);
      const int64_t e = (int64_t)kidx * a.n_kv + c * 8 + (PFX && kidx < pfx_len ? pfx_delta : 0);
      rk[i] = *reinterpret_cast<const u32x4 *>(Kp + e);
    }
  };
  auto load_v = [&](int t, u32x2 (&rv)[4]) {
    const int k0 = kbeg + min(t, ntiles - 1) * ATT_BN;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int kidx = min(k0 + v_qd * 4 + i, n_visible - 1);
      const int64_t e = (int64_t)kidx * a.n_kv + v_cg * 4 + (PFX && kidx < pfx_len ? pfx_delta : 0);
      rv[i] = *reinterpret_cast<const u32x2 *>(Vp + e);
    }
  };
  auto store_k = [&](int buf, const u32x4 (&rk)[2]) {
#pragma unroll
    for (int i = 0; i < 2; ++i) {
      const int q = tid + i * NT, key = q >> 4, c = q & 15;
      Ks[buf][key * 16 + (c ^ (key & 15))] = rk[i];
    }
  };
  auto store_v = [&](int buf, const u32x2 (&rv)[4]) {
    const int grp16 = v_qd >> 2, qi = v_qd & 3;
    const int vkh = qi & 1, halfpos = qi >> 1;
    const int vchunk = grp16 * 2 + vkh;
    u32x2 *vs2 = reinterpret_cast<u32x2 *>(Vs[buf]);
#pragma unroll
    for (int j = 0; j < 2; ++j) {
      u32x2 ev, od;
      ev.x = __builtin_amdgcn_perm(rv[1][j], rv[0][j], 0x05040100u);
      ev.y = __builtin_amdgcn_perm(rv[3][j], rv[2][j], 0x05040100u);
      od.x = __builtin_amdgcn_perm(rv[1][j], rv[0][j], 0x07060302u);
      od.y = __builtin_amdgcn_perm(rv[3][j], rv[2][j], 0x07060302u);
      const int c0 = v_cg * 4 + 2 * j, c1 = c0 + 1;
      vs2[(c0 * 8 + (vchunk ^ v_swz(c0))) * 2 + halfpos] = ev;
      vs2[(c1 * 8 + (vchunk ^ v_swz(c1))) * 2 + halfpos] = od;
    }
  };

  f32x16 s_cur;          // S of the block whose softmax is next
  u32x4 pf[2];           // P of the previous block (two k-steps of 16 keys), zero before the first
  pf[0] = u32x4{0, 0, 0, 0};
  pf[1] = u32x4{0, 0, 0, 0};

  // S(block kb of the K tile in buffer kbuf)
  auto qk_block = [&](int kbuf, int kb, f32x16 &s) {
    const int key = kb * 32 + l32;
    const u32x4 *kp = &Ks[kbuf][key * 16];
#pragma unroll
    for (int v = 0; v < 16; ++v) s[v] = 0.f;
#pragma unroll
    for (int ks = 0; ks < 8; ++ks)
      s = __builtin_amdgcn_mfma_f32_32x32x16_bf16(u4_as_bf16x8(kp[(2 * ks + kh) ^ (key & 15)]), u4_as_bf16x8(qf[ks]), s, 0, 0, 0);
  };
  // O^T += V^T P^T for block kb of the V tile in buffer vbuf
  auto pv_block = [&](int vbuf, int kb) {
#pragma unroll
    for (int hf = 0; hf < 2; ++hf)
#pragma unroll
      for (int cb = 0; cb < 4; ++cb) {
        const int col = cb * 32 + l32, c = 2 * (kb * 2 + hf) + kh;
        o[cb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(u4_as_bf16x8(Vs[vbuf][col * 8 + (c ^ v_swz(col))]),
                                                        u4_as_bf16x8(pf[hf]), o[cb], 0, 0, 0);
      }
  };

  const uint32_t k_base = (uint32_t)(l32 * 256 + ((kh ^ (l32 & 15)) << 4));
  const uint32_t v_base = (uint32_t)(l32 * 128 + ((kh ^ v_swz(l32)) << 4));

  // One pipeline step, written as 16 chunks of {one MFMA, one LDS fragment read three chunks ahead,
  // a slice of vector work}; scheduling fences between the chunks keep the compiler from
  // regrouping them, so the matrix unit gets a new instruction about every eight vector ones and
  // only a few fragments are live at a time.
  //   MFMA c < 8: O^T[cb] += V^T fragment (hf, cb) P(j-1)[hf] ; c >= 8: S(j+1) += K fragment c-8
  //   (S(j) has been consumed by then, so S(j+1) takes over its registers)
  //   vector slices: block maximum and rescale factor before the first MFMA (the fragment reads
  //   are in flight meanwhile), two exponentials + pack + row-sum per chunk, then the LDS store
  //   and the global prefetch that belong to this step (st, ld).
  auto step_m = [&](auto need_mask, int k0, int kbuf, auto kb_c, int vbuf, auto vb_c, auto &&st, auto &&ld) {
    constexpr int kb = decltype(kb_c)::value, vb = decltype(vb_c)::value;
    // fragment addresses: one per-lane base each for K and V^T, the chunk swizzles are XORs with
    // constants (bits 5..7 of the byte address) and everything else is an immediate offset
    // (the bases pass through an empty asm so that the XORs stay inside the step, one
    // instruction next to each read, instead of being hoisted into sixteen registers)
    uint32_t k_bs = k_base + (uint32_t)(kbuf * (ATT_BN * 256)), v_bs = v_base + (uint32_t)(vbuf * (H * 128));
    asm volatile("" : "+v"(k_bs), "+v"(v_bs));
    auto rd = [&](int c) -> u32x4 {
      const int i = c & 7;
      if (c >= 8) {
        // K chunk (2i + kh) ^ (key & 15) of row key = 32 kb + l32
        const uint32_t ad = (k_bs ^ (uint32_t)(i << 5)) + (uint32_t)(kb * (32 * 256));
        return *reinterpret_cast<const u32x4 *>(reinterpret_cast<const char *>(&Ks[0][0]) + ad);
      }
      // V^T chunk (2 (2 vb + hf) + kh) ^ v_swz(col) of row col = 32 cb + l32
      const int hf = i >> 2, cb = i & 3;
      const uint32_t ad = (v_bs ^ (uint32_t)(((2 * vb + hf) ^ cb) << 5)) + (uint32_t)(cb * (32 * 128));
      return *reinterpret_cast<const u32x4 *>(reinterpret_cast<const char *>(&Vs[0][0]) + ad);
    };
    // fragments are requested AH chunks before their MFMA: with eight waves sharing the LDS a read
    // takes a few hundred cycles to come back, so several per wave have to be in flight
    u32x4 fr[16];
#pragma unroll
    for (int c = 0; c < AH; ++c) fr[c] = rd(c);
    __builtin_amdgcn_sched_barrier(0);
    if constexpr (decltype(need_mask)::value) {
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        const int kk = k0 + 8 * (v >> 2) + 4 * kh + (v & 3);
        if (kk > pos || kk >= kend) s_cur[v] = -INFINITY;
      }
    }
    float mx = s_cur[0];
#pragma unroll
    for (int v = 1; v < 16; ++v) mx = fmaxf(mx, s_cur[v]);
    mx = max_with_other_half(mx);
    const float m_blk = mx * c_scale;
    const bool move = __any(m_blk > m_run + a.lazy);
    const float m_new = move ? fmaxf(m_run, m_blk) : m_run;
    const float m_safe = (m_new == -INFINITY) ? 0.f : m_new;
    float alpha = __builtin_amdgcn_exp2f(m_run - m_safe);      // 1 exactly where the maximum stays
    m_run = m_new;
    asm volatile("" : "+v"(alpha));
    __builtin_amdgcn_sched_barrier(0);
    f32x16 s_nxt;
#pragma unroll
    for (int v = 0; v < 16; ++v) s_nxt[v] = 0.f;
    uint32_t pw[8];
    float rs = 0.f;
#pragma unroll
    for (int c = 0; c < 16; ++c) {
      if (c + AH < 16) fr[c + AH] = rd(c + AH);
      const int i = c & 7;
      if (c >= 8) {
        s_nxt = __builtin_amdgcn_mfma_f32_32x32x16_bf16(u4_as_bf16x8(fr[c]), u4_as_bf16x8(qf[i]), s_nxt, 0, 0, 0);
      } else {
        o[i & 3] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(u4_as_bf16x8(fr[c]), u4_as_bf16x8(pf[i >> 2]), o[i & 3], 0, 0, 0);
      }
      if (c < 8) {
        // probabilities 2c, 2c+1 as a bf16 pair; the row sum is taken from the ROUNDED values so
        // that numerator and denominator of the softmax carry the same rounding
        const float e0 = __builtin_amdgcn_exp2f(fmaf(s_cur[2 * c], c_scale, -m_safe));
        const float e1 = __builtin_amdgcn_exp2f(fmaf(s_cur[2 * c + 1], c_scale, -m_safe));
        pw[c] = pack_bf16x2(e0, e1);
        rs = sum_bf16x2(pw[c], rs);
        asm volatile("" : "+v"(pw[c]), "+v"(rs));      // keeps this slice in this chunk
      } else if (c == 8) {
        l_run = l_run * alpha + rs;
      } else if (c == 10) {
        st();
      } else if (c == 12) {
        ld();
      }
      __builtin_amdgcn_sched_barrier(0);
    }
    if (move) {     // after P(j-1) V(j-1) has been accumulated: O_j = (O + P V) * alpha
#pragma unroll
      for (int cb = 0; cb < 4; ++cb)
#pragma unroll
        for (int v = 0; v < 16; ++v) o[cb][v] *= alpha;
    }
    s_cur = s_nxt;
    pf[0] = u32x4{pw[0], pw[1], pw[2], pw[3]};
    pf[1] = u32x4{pw[4], pw[5], pw[6], pw[7]};
  };
  if (ntiles > 0) {
    load_k(0, rkA); load_v(0, rvA);
    store_k(0, rkA); store_v(0, rvA);
    // the first step multiplies a zero P with whatever V buffer 1 holds: make that finite
    for (int i = tid; i < H * 8; i += NT) Vs[1][i] = u32x4{0, 0, 0, 0};
    load_k(1, rkA); load_v(1, rvA);
    __syncthreads();
    qk_block(0, 0, s_cur);
  }
  // Tile t sits in LDS buffer t & 1.  Its two steps: S(t, block 1) with V(t-1, block 1), then
  // S(t+1, block 0) with V(t, block 0).  The causal / split-end mask is compiled into a second copy
  // of the loop that takes over at the first tile that needs it (a branch inside a step would cut
  // the region the three streams share).
  auto tile_steps = [&](auto need_mask, int t) {
    const int b = t & 1;
    step_m(need_mask, kbeg + t * ATT_BN, b, std::integral_constant<int, 1>{}, b ^ 1, std::integral_constant<int, 1>{},
           [&] { store_k(b ^ 1, rkA); }, [&] { load_k(t + 2, rkA); });
    __syncthreads();
    step_m(need_mask, kbeg + t * ATT_BN + 32, b ^ 1, std::integral_constant<int, 0>{}, b, std::integral_constant<int, 0>{},
           [&] { store_v(b ^ 1, rvA); }, [&] { load_v(t + 2, rvA); });
    __syncthreads();
  };
  // tiles [0, t_mask) lie entirely below the tile's first query position and inside the split
  int t_mask = min(ntiles, max(0, (first_pos + 1 - kbeg) / ATT_BN));
  if (kbeg + t_mask * ATT_BN > kend) --t_mask;
  t_mask = max(t_mask, 0);
  wait_all_global_loads();
  for (int t = 0; t < t_mask; ++t) tile_steps(std::false_type{}, t);
  for (int t = t_mask; t < ntiles; ++t) tile_steps(std::true_type{}, t);
  // drain: the last block's probabilities still wait for their V
  if (ntiles > 0) pv_block((ntiles - 1) & 1, 1);

  const float l_tot = l_run + __shfl_xor(l_run, 32, 64);
  if (tok >= ntok) return;
  const int64_t row = row0 + tok;
  if (a.out != nullptr) {
    const float inv = 1.0f / l_tot;
    bf16 *op = a.out + row * a.n_q + head * H;
#pragma unroll
    for (int cb = 0; cb < 4; ++cb)
#pragma unroll
      for (int v4 = 0; v4 < 4; ++v4) {
        const int col = cb * 32 + 8 * v4 + 4 * kh;
        uint2 w;
        w.x = pack_bf16x2(o[cb][4 * v4] * inv, o[cb][4 * v4 + 1] * inv);
        w.y = pack_bf16x2(o[cb][4 * v4 + 2] * inv, o[cb][4 * v4 + 3] * inv);
        *reinterpret_cast<uint2 *>(op + col) = w;
      }
  } else {
    float *pp = a.partials + ((row * a.n_q_heads + head) * a.n_splits + split) * (H + 2);
#pragma unroll
    for (int cb = 0; cb < 4; ++cb)
#pragma unroll
      for (int v4 = 0; v4 < 4; ++v4) {
        const int col = cb * 32 + 8 * v4 + 4 * kh;
        *reinterpret_cast<float2 *>(pp + col) = make_float2(o[cb][4 * v4], o[cb][4 * v4 + 1]);
        *reinterpret_cast<float2 *>(pp + col + 2) = make_float2(o[cb][4 * v4 + 2], o[cb][4 * v4 + 3]);
      }
    if (kh == 0) {
      pp[H] = m_run == -INFINITY ? -INFINITY : m_run * LN2;
      pp[H + 1] = l_tot;
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

template <bool PFX>
static void launch_attn_pipe(const AttnArgs &a, int n_work, int G, hipStream_t s) {
  dim3 grid(n_work);
  switch (G) {
    case 1: hipLaunchKernelGGL((attn_prefill_pipe_kernel<1, PFX>), grid, dim3(512), 0, s, a); break;
    case 2: hipLaunchKernelGGL((attn_prefill_pipe_kernel<2, PFX>), grid, dim3(512), 0, s, a); break;
    case 4: hipLaunchKernelGGL((attn_prefill_pipe_kernel<4, PFX>), grid, dim3(512), 0, s, a); break;
    case 8: hipLaunchKernelGGL((attn_prefill_pipe_kernel<8, PFX>), grid, dim3(512), 0, s, a); break;
    default: break;
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

// compact records are written by the unpipelined kernels only
bool attn_prefill_mfma_compact(int waves, int schedule) { return !(schedule == ATTN_SCHED_PIPELINED && waves == 8); }

void launch_attn_prefill_mfma(const AttnArgs &a, int n_work, int G, int waves, int schedule, bool prefix,
                              hipStream_t s) {
  if (n_work == 0) return;
  if (schedule == ATTN_SCHED_PIPELINED && waves == 8) {
    if (prefix) launch_attn_pipe<true>(a, n_work, G, s);
    else launch_attn_pipe<false>(a, n_work, G, s);
  } else if (waves == 4) {
    launch_attn_nw_any<4>(a, n_work, G, prefix, s);
  } else {
    launch_attn_nw_any<8>(a, n_work, G, prefix, s);
  }
}

// What the rotation kernel multiplies the queries by for the variant the arguments select: the folded
// softmax wants them in the exp2 domain, every other kernel applies sm_scale itself.
float attn_prefill_mfma_q_scale(const LayerDims &L, int waves, int schedule, bool fold) {
  if (!fold || (schedule == ATTN_SCHED_PIPELINED && waves == 8)) return 1.0f;
  return LOG2E / sqrtf((float)L.head_dim);
}

}  // namespace alora
