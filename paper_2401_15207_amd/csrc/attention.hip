// Fused attention for gfx950, three kernels:
//   attn_k<.., BWD = false>  forward: scores, softmax and the product with V; the scores never reach HBM.  The
//                            probabilities do (bf16, [B, H, S, S]): the backward pass reads them.
//   attn_k<.., BWD = true>   query-major half of the backward: dP, the softmax derivative and dQ (same body, K and V
//                            exchanged); writes dS for the other half.
//   attn_bwd_kv_k            key-major half of the backward: dV and dK, sums over the queries.
//
// Forward: one workgroup = 32 NW query rows of one (batch, head), NW = 2 or 4 wavefronts; each wavefront owns
// 32 rows from start to end, so the softmax of a row never leaves its wavefront.  Keys and values pass
// through LDS in tiles of 64 keys; the next tile is on its way from HBM (direct-to-LDS loads) while the
// current one is used.  When the probabilities are wanted: two passes over the keys, the first finds each
// row's maximum and normaliser (online), the second recomputes the scores, writes the normalised
// probabilities and accumulates P.V from the bf16-rounded probabilities, which is exactly what separate
// softmax and contraction kernels compute.  When they are not (the model's case: the backward kernels form
// them again from the rows' log-sums): one pass with running sums, normalised at the end.
//
// MFMA (v_mfma_f32_32x32x16_bf16) conventions, as in gemm.hip: an operand fragment gives lane l row
// l%32 and the eight k-values 8*(l/32)..+7; acc = mfma(X, Y, acc) leaves in lane l, element e the
// entry (Y row l%32, X row 8*(e/4) + 4*(l/32) + e%4).
//   scores: Y = Q rows, X = K rows.  The K rows of a 32-key block are fed in the order
//   pi(r) = r with bits 2 and 3 swapped; then element e of lane l is key 16*(e/8) + 8*(l/32) + e%8 of
//   the block: elements 0..7 and 8..15 are, as they lie in registers, the two operand fragments of
//   P for the next product, and 16 contiguous bytes of a probability row each.
//   P.V: Y = P (rows = queries, k = keys), X = V^T (rows = head columns, k = keys), read from the
//   row-major V tile with transposing LDS reads (ds_read_b64_tr_b16: lane i of a group of 16 gets,
//   as element e, what lane i/4 + 4e of the group addressed as its element i%4).
#include <type_traits>

#include "common.h"
#include "kernels.h"

namespace hift {
namespace {

typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) __bf16 bf16x4;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef short v4i16 __attribute__((ext_vector_type(4)));

constexpr int KTILE = 64;  // keys per LDS tile

__device__ __forceinline__ int pi_row(int r) { return (r & ~12) | ((r & 4) << 1) | ((r & 8) >> 1); }

// 16 bytes per lane straight from memory into LDS: M0 carries the LDS address of lane 0's piece, lane l
// lands 16 l bytes further; reads past the buffer's end deliver zeros.
__device__ __forceinline__ void dma_b128(u32x4 rsrc, uint32_t lds_addr, uint32_t voff, uint32_t soff) {
  asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tbuffer_load_dwordx4 %1, %2, %3 offen lds"
               :
               : "s"(lds_addr), "v"(voff), "s"(rsrc), "s"(soff)
               : "memory");
}

// Adjoint of the rotary embedding on a row held as NB accumulator blocks of 32 columns (lane: columns
// 8 g + 4 fh + e of each block): the pair (c, c + HD/2) is (block nb, block nb + NB/2), same lane and element;
// cs: the row's position in the table, [HD/2] pairs (cos, sin).  d x1 = d y1 cos + d y2 sin, d x2 = d y2 cos - d y1 sin.
template <int NB>
__device__ __forceinline__ void unrotate(f32x16 (&acc)[NB], const float2* __restrict__ cs, int fh) {
#pragma unroll
  for (int nb = 0; nb < NB / 2; ++nb)
#pragma unroll
    for (int g = 0; g < 4; ++g)
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        const float2 c = cs[nb * 32 + 8 * g + 4 * fh + e];
        const float y1 = acc[nb][4 * g + e], y2 = acc[nb + NB / 2][4 * g + e];
        acc[nb][4 * g + e] = y1 * c.x + y2 * c.y;
        acc[nb + NB / 2][4 * g + e] = y2 * c.x - y1 * c.y;
      }
}

// Rows that a wavefront holds as accumulators (lane l: row l % 32 of its 32 rows, as 4-column pieces: element e of
// block nb is column 32 nb + 8 (e / 4) + 4 (l / 32) + e % 4) go to memory through LDS.  The output's rows lie a whole
// row of the caller's matrix apart; written from the registers, every store instruction would touch 32 lines for 16
// bytes each (measured: 3.8 of the key-major backward kernel's 48 microseconds).  Staged as [32 rows][32 NB columns]
// in a region of the wavefront's own (32 (64 NB + 16) bytes; the pad spreads the rows over the banks), a store
// instruction writes whole rows, 16 bytes per lane.  A wavefront reads back only what it wrote itself and its LDS
// accesses complete in order: no barrier in here; the caller makes sure nobody else still uses the region.
template <int NB>
__device__ __forceinline__ void store_rows_staged(const f32x16 (&acc)[NB], float mul, unsigned char* stage, bf16* dst, int64_t ld,
                                                  int rows_valid, int lane) {
  constexpr int PITCH = NB * 64 + 16, LPR = NB * 4, RPI = 64 / LPR;  // bytes per staged row; lanes per row; rows per store
  const int fr = lane & 31, fh = lane >> 5;
#pragma unroll
  for (int nb = 0; nb < NB; ++nb)
#pragma unroll
    for (int g = 0; g < 4; ++g) {
      bf16x4 o4;
#pragma unroll
      for (int e = 0; e < 4; ++e) o4[e] = static_cast<__bf16>(acc[nb][4 * g + e] * mul);
      *reinterpret_cast<bf16x4*>(stage + fr * PITCH + (nb * 32 + 8 * g + 4 * fh) * 2) = o4;
    }
  const int pr = lane / LPR, pc = lane % LPR;
#pragma unroll
  for (int r0 = 0; r0 < 32; r0 += RPI) {
    const int rr = r0 + pr;
    if (rr < rows_valid) *reinterpret_cast<u32x4*>(dst + (int64_t)rr * ld + pc * 8) = *reinterpret_cast<const u32x4*>(stage + rr * PITCH + pc * 16);
  }
}

// LDS tiles are [64 keys][HD] bf16 without padding; the 16-byte piece c of row r sits at piece position
// c ^ swz(r), which spreads both the fragment reads (sixteen rows, one piece) and the transposing
// reads over the banks.  A tile is filled by loads that write 1 KB of consecutive LDS bytes each, so
// the swizzle is applied by choosing which piece of its row a lane fetches.
//
// BWD = false: the forward kernel.  `scale` is log2(e) / sqrt(HD); writes ctx, the probabilities if prob is
// given, and lse (if given): log2 of each row's sum of exponentials, m + log2(l) in the notation below.
// BWD = true: the query-major half of the backward pass, on the same tiling.  Reads ctx (O), dctx (dO) and lse;
// `scale` is 1 / sqrt(HD).  Per row i:
//   D_i = sum_e dO[i,e] O[i,e]   (= sum_j P[i,j] dP[i,j], since O = P V); written to dsum for the other half
//   P[i,j] = exp2(S[i,j] scale log2(e) - lse_i) with S = Q K^T formed again tile by tile,
//   dP[i,j] = dO[i,:] . V[j,:],  dS[i,j] = scale * P[i,j] * (dP[i,j] - D_i),  dQ[i,:] = sum_j dS[i,j] K[j,:]
// dQ goes to the q columns of dqkv (row stride ld, like qkv), un-rotated if cos_sin is given.  Neither P nor dS
// is stored: the key-major kernel below forms its own.
template <int HD, bool CAUSAL, int NW, bool BWD>
__global__ void __launch_bounds__(64 * NW, NW == 4 ? 2 : 1) attn_k(const bf16* __restrict__ qkv, int64_t ld, int S, int H, int BH, float scale,
                                                   bf16* __restrict__ prob, bf16* __restrict__ ctx, int64_t ldc,
                                                   const bf16* __restrict__ dctx, float* __restrict__ lse, float* __restrict__ dsum,
                                                   bf16* __restrict__ dqkv, const float2* __restrict__ cos_sin) {
  const float scale_log2e = BWD ? scale * 1.4426950408889634f : scale;
  constexpr int QB = 32 * NW;       // query rows per workgroup
  constexpr int ROWB = HD * 2;      // bytes per LDS row
  constexpr int PPR = HD / 8;       // 16-byte pieces per row: 16 or 8
  constexpr int TILEB = KTILE * ROWB;
  constexpr int KS = HD / 16;       // k-steps of a score block
  constexpr int NB = HD / 32;       // 32-column blocks of the output
  constexpr int IPW = KTILE * PPR / 64 / NW;  // load instructions per wavefront and tile
  __shared__ __attribute__((aligned(1024))) unsigned char lds[4 * TILEB];  // [buffer][K | V]
  auto swz = [](int r) { return PPR == 16 ? (r & 15) : ((r >> 1) & 7); };

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int fr = lane & 31, fh = lane >> 5;
  // Causal rows get longer towards the end of the sequence.  Workgroups are handed out in the order of
  // their index, two fit a compute unit: the first half of the grid takes the long row blocks, the second
  // half their short counterparts, so that the two that share a compute unit add up to the same work.
  const int nqb = (S + QB - 1) / QB;
  int bh, qb;
  if (CAUSAL) {
    const int n_long = (nqb + 1) / 2, n_short = nqb - n_long;
    const int L = (int)blockIdx.x, first = n_long * BH;
    if (L < first) {
      bh = L / n_long;
      qb = nqb - 1 - L % n_long;
    } else {
      bh = (L - first) / n_short;
      qb = (L - first) % n_short;
    }
  } else {
    bh = (int)blockIdx.x / nqb;
    qb = (int)blockIdx.x % nqb;
  }
  const int b = bh / H, h = bh % H;
  const int64_t d = (int64_t)H * HD;
  const bf16* q = qkv + (int64_t)b * S * ld + (int64_t)h * HD;
  const bf16* k = q + d;
  const bf16* v = q + 2 * d;
  bf16* P = prob ? prob + (int64_t)bh * S * S : nullptr;
  bf16* O = ctx + (int64_t)b * S * ldc + (int64_t)h * HD;

  const int q0 = qb * QB + wave * 32;  // this wavefront's first row
  const int row = q0 + fr;
  const bool row_ok = row < S;

  bf16x8 qf[KS];  // fragments of the wavefront's 32 rows: Q (forward) or dO (backward)
  bf16x8 qq[BWD ? KS : 1];  // backward: the Q rows as well
  float Drow = 0.f;  // backward: D of this lane's row
  if (BWD) {
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) {
      u32x4 t = {0u, 0u, 0u, 0u};
      if (row_ok) t = *reinterpret_cast<const u32x4*>(q + (int64_t)row * ld + ks * 16 + fh * 8);
      qq[ks] = __builtin_bit_cast(bf16x8, t);
    }
  }
  {
    const bf16* src = BWD ? dctx + (int64_t)b * S * ldc + (int64_t)h * HD + (int64_t)row * ldc : q + (int64_t)row * ld;
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) {
      u32x4 t = {0u, 0u, 0u, 0u};
      if (row_ok) t = *reinterpret_cast<const u32x4*>(src + ks * 16 + fh * 8);
      qf[ks] = __builtin_bit_cast(bf16x8, t);
    }
    if (BWD) {
#pragma unroll
      for (int ks = 0; ks < KS; ++ks) {
        u32x4 t = {0u, 0u, 0u, 0u};
        if (row_ok) t = *reinterpret_cast<const u32x4*>(O + (int64_t)row * ldc + ks * 16 + fh * 8);
        const bf16x8 of = __builtin_bit_cast(bf16x8, t);
#pragma unroll
        for (int e = 0; e < 8; ++e) Drow = __builtin_fmaf((float)qf[ks][e], (float)of[e], Drow);
      }
      Drow += __shfl_xor(Drow, 32, 64);  // the two lanes of a row hold the two halves of every 16 columns
    }
  }

  const int last_row = min(S, qb * QB + QB) - 1;
  const int n_tiles = CAUSAL ? last_row / KTILE + 1 : (S + KTILE - 1) / KTILE;  // key tiles with unmasked keys
  const int all_tiles = (S + KTILE - 1) / KTILE;

  // tile loads
  const uint32_t rec = (uint32_t)((((int64_t)S - 1) * ld + HD) * 2);  // bytes of K (or V) of this head from its first row
  const uint64_t ka = reinterpret_cast<uint64_t>(k), va = reinterpret_cast<uint64_t>(v);
  const u32x4 rsK = {(uint32_t)ka, (uint32_t)(ka >> 32) & 0xFFFFu, rec, 0x00020000u};
  const u32x4 rsV = {(uint32_t)va, (uint32_t)(va >> 32) & 0xFFFFu, rec, 0x00020000u};
  uint32_t vo[IPW];
#pragma unroll
  for (int jj = 0; jj < IPW; ++jj) {
    const int pc = (wave * IPW + jj) * 64 + lane, r = pc / PPR, c = (pc % PPR) ^ swz(r);
    vo[jj] = (uint32_t)((r * ld + c * 8) * 2);
  }
  const uint32_t lds0 = (uint32_t)reinterpret_cast<uintptr_t>(lds);
  auto request = [&](int kt, bool with_v) __attribute__((always_inline)) {
    const uint32_t so = (uint32_t)((int64_t)kt * KTILE * ld * 2);
    const uint32_t dst = lds0 + (uint32_t)(kt & 1) * (2 * TILEB) + (uint32_t)wave * (IPW * 1024);
#pragma unroll
    for (int jj = 0; jj < IPW; ++jj) dma_b128(rsK, dst + jj * 1024, vo[jj], so);
    if (with_v) {
#pragma unroll
      for (int jj = 0; jj < IPW; ++jj) dma_b128(rsV, dst + TILEB + jj * 1024, vo[jj], so);
    }
  };

  // Addresses inside a tile, computed once (the swizzle makes them irregular; recomputing them per tile
  // would cost more instructions than the arithmetic of the softmax).
  int kaddr[2][KS];  // K fragment of block blk, k-step ks
#pragma unroll
  for (int blk = 0; blk < 2; ++blk) {
    const int r = blk * 32 + pi_row(fr);
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) kaddr[blk][ks] = r * ROWB + (((2 * ks + fh) ^ swz(r)) * 16);
  }
  // transposing reads of V for k-step t (16 keys): lane -> key row 16 t + 8 fh + sl/4 (+4 for the second
  // half) and columns nb*32 + 16*((lane/16)%2) + 4*(sl%4) ..+3; swz(row) does not depend on t
  const int sl = lane & 15;
  int vaddr[NB][2];
#pragma unroll
  for (int nb = 0; nb < NB; ++nb)
#pragma unroll
    for (int hh = 0; hh < 2; ++hh) {
      const int krow = 8 * fh + (sl >> 2) + 4 * hh;
      const int col = nb * 32 + 16 * ((lane >> 4) & 1) + 4 * (sl & 3);
      vaddr[nb][hh] = krow * ROWB + (((col >> 3) ^ swz(krow)) * 16) + (col & 7) * 2;
    }
  static_assert(KTILE == 64 && (16 * ROWB) % (PPR == 16 ? 16 * ROWB : 2 * ROWB) == 0, "swz(row + 16 t) = swz(row)");

  // raw scores (unscaled) of the tile's two 32-key blocks; MASKED: masked positions become -inf
  auto scores = [&](auto MASKED_, const unsigned char* Kb, int kt, float (&s)[32], const bf16x8* yf) __attribute__((always_inline)) {
    constexpr bool MASKED = decltype(MASKED_)::value;
    f32x16 a0, a1;
#pragma unroll
    for (int e = 0; e < 16; ++e) a0[e] = a1[e] = 0.f;
#pragma unroll
    for (int hf = 0; hf < 2; ++hf) {
      bf16x8 f0[KS / 2], f1[KS / 2];
#pragma unroll
      for (int i = 0; i < KS / 2; ++i) {
        f0[i] = *reinterpret_cast<const bf16x8*>(Kb + kaddr[0][hf * (KS / 2) + i]);
        f1[i] = *reinterpret_cast<const bf16x8*>(Kb + kaddr[1][hf * (KS / 2) + i]);
      }
      __builtin_amdgcn_sched_barrier(0);  // all fragment reads of this half before its MFMAs
#pragma unroll
      for (int i = 0; i < KS / 2; ++i) {
        const int ks = hf * (KS / 2) + i;
        a0 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(f0[i], yf[ks], a0, 0, 0, 0);
        a1 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(f1[i], yf[ks], a1, 0, 0, 0);
      }
    }
#pragma unroll
    for (int e = 0; e < 16; ++e) {
      s[e] = a0[e];
      s[16 + e] = a1[e];
    }
    if (MASKED) {
      const int key0 = kt * KTILE + 8 * fh;
#pragma unroll
      for (int e = 0; e < 32; ++e) {
        const int key = key0 + 32 * (e / 16) + 16 * ((e % 16) / 8) + (e % 8);
        const bool ok = key < S && (!CAUSAL || key <= row);
        s[e] = ok ? s[e] : -INFINITY;
      }
    }
  };
  // true when no key of tile kt is masked for any row of this wavefront
  auto tile_plain = [&](int kt) { return kt * KTILE + KTILE <= S && (!CAUSAL || kt * KTILE + KTILE - 1 <= q0); };
  using std::false_type;
  using std::true_type;

  if constexpr (!BWD) {
    if (prob == nullptr) {
      // ---- one pass (nobody reads the probabilities): exponentials against a reference maximum m_ref of the row
      // (log2 domain), which is raised, and the sums so far rescaled, only when a score exceeds it by more than
      // 2^8: the unnormalised probabilities then stay below 2^8, which costs bf16 (a relative format) nothing.
      // O = (sum_j p_j V_j) / (sum_j p_j) at the end. ----
      float m = -INFINITY, l = 0.f;
      f32x16 oacc[NB];
#pragma unroll
      for (int nb = 0; nb < NB; ++nb)
#pragma unroll
        for (int e = 0; e < 16; ++e) oacc[nb][e] = 0.f;
      request(0, true);
      for (int kt = 0; kt < n_tiles; ++kt) {
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        __syncthreads();
        if (kt + 1 < n_tiles) request(kt + 1, true);
        if (CAUSAL && kt * KTILE > q0 + 31) continue;  // wholly above the diagonal for this wavefront
        const unsigned char* Kb = lds + (kt & 1) * (2 * TILEB);
        const unsigned char* Vb = Kb + TILEB;
        float s[32];
        if (tile_plain(kt)) scores(false_type{}, Kb, kt, s, qf);
        else scores(true_type{}, Kb, kt, s, qf);
        float mr = s[0];
#pragma unroll
        for (int e = 1; e < 32; ++e) mr = fmaxf(mr, s[e]);
        mr = fmaxf(mr, __shfl_xor(mr, 32, 64));  // the two lanes of a row must agree on the reference
        const float cand = mr * scale_log2e;     // finite: every row has an unmasked key in every tile it visits
        if (__builtin_amdgcn_ballot_w64(cand > m + 8.0f) != 0) {
          const float mn = fmaxf(m, cand);
          const float alpha = __builtin_amdgcn_exp2f(m - mn);  // 0 on the first tile (m = -inf)
          l *= alpha;
#pragma unroll
          for (int nb = 0; nb < NB; ++nb)
#pragma unroll
            for (int e = 0; e < 16; ++e) oacc[nb][e] *= alpha;
          m = mn;
        }
        u32x4 pk[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          bf16x8 t;
#pragma unroll
          for (int e = 0; e < 8; ++e) {
            const float pr = __builtin_amdgcn_exp2f(__builtin_fmaf(s[8 * i + e], scale_log2e, -m));  // exp2(-inf) = 0
            l += pr;
            t[e] = static_cast<__bf16>(pr);
          }
          pk[i] = __builtin_bit_cast(u32x4, t);
        }
#pragma unroll
        for (int t = 0; t < 4; ++t) {
          bf16x8 vt[NB];
#pragma unroll
          for (int nb = 0; nb < NB; ++nb) {
            const unsigned char* a0 = Vb + t * 16 * ROWB + vaddr[nb][0];
            const unsigned char* a1 = Vb + t * 16 * ROWB + vaddr[nb][1];
            const v4i16 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((v4i16 __attribute__((address_space(3)))*)(a0));
            const v4i16 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((v4i16 __attribute__((address_space(3)))*)(a1));
            typedef short v8i16 __attribute__((ext_vector_type(8)));
            const v8i16 both = {lo[0], lo[1], lo[2], lo[3], hi[0], hi[1], hi[2], hi[3]};
            vt[nb] = __builtin_bit_cast(bf16x8, both);
          }
          __builtin_amdgcn_sched_barrier(0);
          const bf16x8 pf = __builtin_bit_cast(bf16x8, pk[t]);
#pragma unroll
          for (int nb = 0; nb < NB; ++nb) oacc[nb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vt[nb], pf, oacc[nb], 0, 0, 0);
        }
      }
      l += __shfl_xor(l, 32, 64);  // the two lanes of a row summed different keys
      const float inv = l > 0.f ? 1.0f / l : 0.f;
      if (lse && row_ok && fh == 0) lse[(int64_t)bh * S + row] = m + __builtin_amdgcn_logf(l);
      asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
      __syncthreads();  // every wavefront is done with the tiles: the context rows leave through their buffers
      static_assert(NW * 32 * (ROWB + 16) <= 4 * TILEB, "staging fits the tile buffers");
      store_rows_staged<NB>(oacc, inv, lds + wave * (32 * (ROWB + 16)), O + (int64_t)q0 * ldc, ldc, S - q0, lane);
      return;
    }
    // ---- pass 1: row maximum and normaliser (m in the log2 domain: raw score * scale_log2e) ----
    float m = -INFINITY, l = 0.f;
    request(0, false);
    for (int kt = 0; kt < n_tiles; ++kt) {
      asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
      __syncthreads();  // tile kt is complete; nobody reads the other buffer any more
      if (kt + 1 < n_tiles) request(kt + 1, false);
      if (CAUSAL && kt * KTILE > q0 + 31) continue;  // wholly above the diagonal for this wavefront
      const unsigned char* Kb = lds + (kt & 1) * (2 * TILEB);
      float s[32];
      if (tile_plain(kt)) scores(false_type{}, Kb, kt, s, qf);
      else scores(true_type{}, Kb, kt, s, qf);
      float mr = s[0];
  #pragma unroll
      for (int e = 1; e < 32; ++e) mr = fmaxf(mr, s[e]);
      const float mx = fmaxf(m, mr * scale_log2e);  // scale > 0
      if (mx > -INFINITY) {
        float add = 0.f;
  #pragma unroll
        for (int e = 0; e < 32; ++e) add += __builtin_amdgcn_exp2f(__builtin_fmaf(s[e], scale_log2e, -mx));
        l = l * __builtin_amdgcn_exp2f(m - mx) + add;
        m = mx;
      }
    }
    {  // the two lanes that share a row
      const float m2 = __shfl_xor(m, 32, 64), l2 = __shfl_xor(l, 32, 64);
      const float mm = fmaxf(m, m2);  // finite for every row < S: key 0 is never masked
      l = (m > -INFINITY ? l * __builtin_amdgcn_exp2f(m - mm) : 0.f) + (m2 > -INFINITY ? l2 * __builtin_amdgcn_exp2f(m2 - mm) : 0.f);
      m = mm;
    }
    const float inv = l > 0.f ? 1.0f / l : 0.f;
    // log2 of the row's sum of exponentials: what the backward kernels need to form a probability again
    if (lse && row_ok && fh == 0) lse[(int64_t)bh * S + row] = m + __builtin_amdgcn_logf(l);
    __syncthreads();  // pass 1 has left the buffers

    // ---- pass 2: probabilities and P.V ----
    f32x16 oacc[NB];
  #pragma unroll
    for (int nb = 0; nb < NB; ++nb)
  #pragma unroll
      for (int e = 0; e < 16; ++e) oacc[nb][e] = 0.f;
    // probabilities leave as 16-byte pieces (S is a multiple of 8); pieces of rows or keys past S get the
    // offset 2^31, which is beyond the buffer (at most 2^31 bytes) with or without the small scalar
    // offset added, and are dropped by the store
    const __amdgpu_buffer_rsrc_t rsP = __builtin_amdgcn_make_buffer_rsrc(P, 0, (int)(uint32_t)((int64_t)S * S * 2), 0x00020000);
    const uint32_t prow = row_ok ? (uint32_t)((int64_t)row * S * 2) + 16u * fh : 0x80000000u;
    const bool keep_p = prob != nullptr;  // null: nobody will read the probabilities (no backward through this layer)
    auto store_p = [&](int kt, const u32x4(&pk)[4]) __attribute__((always_inline)) {
      if (!keep_p) return;
      // whole tiles inside S (the usual case): the row offset plus a scalar; else per piece
      if (kt * KTILE + KTILE <= S) {
  #pragma unroll
        for (int i = 0; i < 4; ++i) __builtin_amdgcn_raw_buffer_store_b128(pk[i], rsP, (int)prow, (kt * KTILE + 16 * i) * 2, 0);
      } else {
  #pragma unroll
        for (int i = 0; i < 4; ++i) {
          const int key = kt * KTILE + 16 * i + 8 * fh;
          const uint32_t off = (row_ok && key < S) ? prow + (uint32_t)(kt * KTILE + 16 * i) * 2 : 0x80000000u;
          __builtin_amdgcn_raw_buffer_store_b128(pk[i], rsP, (int)off, 0, 0);
        }
      }
    };
    request(0, true);
    for (int kt = 0; kt < n_tiles; ++kt) {
      asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
      __syncthreads();
      if (kt + 1 < n_tiles) request(kt + 1, true);
      u32x4 pk[4];  // the wavefront's probabilities of this tile: four 16-byte pieces per row
      if (CAUSAL && kt * KTILE > q0 + 31) {
  #pragma unroll
        for (int i = 0; i < 4; ++i) pk[i] = u32x4{0u, 0u, 0u, 0u};
        store_p(kt, pk);
        continue;
      }
      const unsigned char* Kb = lds + (kt & 1) * (2 * TILEB);
      const unsigned char* Vb = Kb + TILEB;
      float s[32];
      if (tile_plain(kt)) scores(false_type{}, Kb, kt, s, qf);
      else scores(true_type{}, Kb, kt, s, qf);
  #pragma unroll
      for (int i = 0; i < 4; ++i) {
        bf16x8 t;
  #pragma unroll
        for (int e = 0; e < 8; ++e)
          t[e] = static_cast<__bf16>(__builtin_amdgcn_exp2f(__builtin_fmaf(s[8 * i + e], scale_log2e, -m)) * inv);  // exp2(-inf) = 0
        pk[i] = __builtin_bit_cast(u32x4, t);
      }
      store_p(kt, pk);
      // P.V over the tile's 64 keys: four k-steps of 16
  #pragma unroll
      for (int t = 0; t < 4; ++t) {
        bf16x8 vt[NB];
  #pragma unroll
        for (int nb = 0; nb < NB; ++nb) {
          const unsigned char* a0 = Vb + t * 16 * ROWB + vaddr[nb][0];
          const unsigned char* a1 = Vb + t * 16 * ROWB + vaddr[nb][1];
          const v4i16 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((v4i16 __attribute__((address_space(3)))*)(a0));
          const v4i16 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((v4i16 __attribute__((address_space(3)))*)(a1));
          typedef short v8i16 __attribute__((ext_vector_type(8)));
          const v8i16 both = {lo[0], lo[1], lo[2], lo[3], hi[0], hi[1], hi[2], hi[3]};
          vt[nb] = __builtin_bit_cast(bf16x8, both);
        }
        __builtin_amdgcn_sched_barrier(0);
        const bf16x8 pf = __builtin_bit_cast(bf16x8, pk[t]);
  #pragma unroll
        for (int nb = 0; nb < NB; ++nb) oacc[nb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vt[nb], pf, oacc[nb], 0, 0, 0);
      }
    }
    // keys past the last unmasked tile: zeros, so that every entry of the probability matrix is defined
    {
      u32x4 z[4];
  #pragma unroll
      for (int i = 0; i < 4; ++i) z[i] = u32x4{0u, 0u, 0u, 0u};
      for (int kt = n_tiles; kt < all_tiles; ++kt) store_p(kt, z);
    }
    // ---- output rows ----
    if (row_ok) {
  #pragma unroll
      for (int nb = 0; nb < NB; ++nb)
  #pragma unroll
        for (int g = 0; g < 4; ++g) {
          bf16x4 o4;
  #pragma unroll
          for (int e = 0; e < 4; ++e) o4[e] = static_cast<__bf16>(oacc[nb][4 * g + e]);
          *reinterpret_cast<bf16x4*>(O + (int64_t)row * ldc + nb * 32 + 8 * g + 4 * fh) = o4;
        }
    }
  } else {
    // P is formed again from the scores and the row's stored log-sum; neither P nor dS touches memory
    const float lrow = row_ok ? lse[(int64_t)bh * S + row] : 0.f;
    if (row_ok && fh == 0) dsum[(int64_t)bh * S + row] = Drow;  // the key-major kernel needs it per query
    auto above = [&](int kt) { return CAUSAL && kt * KTILE > q0 + 31; };  // wholly above the diagonal for this wavefront
    f32x16 qacc[NB];
#pragma unroll
    for (int nb = 0; nb < NB; ++nb)
#pragma unroll
      for (int e = 0; e < 16; ++e) qacc[nb][e] = 0.f;
    request(0, true);
    for (int kt = 0; kt < n_tiles; ++kt) {
      asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
      __syncthreads();
      if (kt + 1 < n_tiles) request(kt + 1, true);
      if (above(kt)) continue;
      const unsigned char* Kb = lds + (kt & 1) * (2 * TILEB);
      const unsigned char* Vb = Kb + TILEB;
      float s[32], dp[32];
      if (tile_plain(kt)) scores(false_type{}, Kb, kt, s, qq);
      else scores(true_type{}, Kb, kt, s, qq);
      scores(false_type{}, Vb, kt, dp, qf);  // dO . V^T; masked positions get P = 0 below
      u32x4 pk[4];
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        bf16x8 t;
#pragma unroll
        for (int e = 0; e < 8; ++e) {
          const float pr = __builtin_amdgcn_exp2f(__builtin_fmaf(s[8 * i + e], scale_log2e, -lrow));  // exp2(-inf) = 0
          t[e] = static_cast<__bf16>(scale * pr * (dp[8 * i + e] - Drow));
        }
        pk[i] = __builtin_bit_cast(u32x4, t);
      }
      // dQ += dS . K over the tile's 64 keys: four k-steps of 16, K^T by transposing reads
#pragma unroll
      for (int t = 0; t < 4; ++t) {
        bf16x8 kt_[NB];
#pragma unroll
        for (int nb = 0; nb < NB; ++nb) {
          const unsigned char* a0 = Kb + t * 16 * ROWB + vaddr[nb][0];
          const unsigned char* a1 = Kb + t * 16 * ROWB + vaddr[nb][1];
          const v4i16 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((v4i16 __attribute__((address_space(3)))*)(a0));
          const v4i16 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((v4i16 __attribute__((address_space(3)))*)(a1));
          typedef short v8i16 __attribute__((ext_vector_type(8)));
          const v8i16 both = {lo[0], lo[1], lo[2], lo[3], hi[0], hi[1], hi[2], hi[3]};
          kt_[nb] = __builtin_bit_cast(bf16x8, both);
        }
        __builtin_amdgcn_sched_barrier(0);
        const bf16x8 df = __builtin_bit_cast(bf16x8, pk[t]);
#pragma unroll
        for (int nb = 0; nb < NB; ++nb) qacc[nb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kt_[nb], df, qacc[nb], 0, 0, 0);
      }
    }
    if (row_ok && cos_sin) unrotate<NB>(qacc, cos_sin + (int64_t)row * (HD / 2), fh);  // q was rotated after its projection
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __syncthreads();  // every wavefront is done with the tiles: dQ leaves through their buffers
    store_rows_staged<NB>(qacc, 1.0f, lds + wave * (32 * (ROWB + 16)), dqkv + (int64_t)b * S * ld + (int64_t)h * HD + (int64_t)q0 * ld, ld,
                          S - q0, lane);
  }
}

// Key-major half of the attention backward: dV = P^T dO and dK = dS^T Q, both sums over the queries.  A workgroup
// owns 128 keys of one (batch, head), a wavefront 32 of them from start to end with their K and V rows in
// registers; queries pass through LDS in tiles of 64 (Q and dO rows, double-buffered direct-to-LDS loads).  Per
// tile a wavefront forms S^T = K Q^T and dP^T = V dO^T (Y = its key rows, X = the tile's rows in the pi order of
// the forward kernel), from them P^T = exp2(S^T c - lse[query]) and dS^T = scale P^T (dP^T - D[query]); in
// that order of rows the 16 values a lane holds per 32 queries are, as they lie in registers, the operand
// fragments of the two sums, whose other operands (dO^T, Q^T) come from the same tiles by transposing LDS
// reads.  Nothing of size S x S is read or written.  One workgroup per compute unit (the accumulators of four
// products and 64 K / V registers); workgroups are issued longest first under the causal mask.
// lse: log2 of each query's sum of exponentials (forward kernel); dsum: D = dO . O per query (query-major kernel).
// cos_sin, if given, un-rotates dK (k was rotated after its projection).
template <int HD, bool CAUSAL>
__global__ void __launch_bounds__(256, 1) attn_bwd_kv_k(const bf16* __restrict__ qkv, int64_t ld, int S, int H, int BH, float scale,
                                                         const float* __restrict__ lse, const float* __restrict__ dsum,
                                                         const bf16* __restrict__ dctx, int64_t ldc, bf16* __restrict__ dqkv,
                                                         const float2* __restrict__ cos_sin) {
  constexpr int KB = 128;           // keys per workgroup
  constexpr int QT = 64;            // queries per tile
  constexpr int ROWB = HD * 2, PPR = HD / 8, NB = HD / 32, KS = HD / 16;
  constexpr int TQ = QT * ROWB;     // bytes of the Q (or dO) tile
  constexpr int IQ = QT * PPR / 64 / 4;  // load instructions per wavefront, tile and operand
  constexpr int BUF = 2 * TQ + 2048;  // Q | dO | lse (1 KB, 256 bytes used) | D (same)
  __shared__ __attribute__((aligned(1024))) unsigned char lds[2 * BUF];
  auto swq = [](int r) { return PPR == 16 ? (r & 15) : ((r >> 1) & 7); };

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int fr = lane & 31, fh = lane >> 5;
  // key blocks early in the sequence see the most queries under the causal mask and go first
  const int nkb = (S + KB - 1) / KB;
  const int kb = (int)blockIdx.x / BH, bh = (int)blockIdx.x % BH;
  const int b = bh / H, h = bh % H;
  const int64_t d = (int64_t)H * HD;
  const bf16* q = qkv + (int64_t)b * S * ld + (int64_t)h * HD;
  const bf16* dO = dctx + (int64_t)b * S * ldc + (int64_t)h * HD;
  const int j0 = kb * KB + wave * 32;  // this wavefront's first key
  const int row = j0 + fr;
  const bool row_ok = row < S;
  const float scale_log2e = scale * 1.4426950408889634f;
  (void)nkb;

  bf16x8 kf[KS], vf[KS];  // this lane's key row: fragments of K and V
#pragma unroll
  for (int ks = 0; ks < KS; ++ks) {
    u32x4 tk = {0u, 0u, 0u, 0u}, tv = tk;
    if (row_ok) {
      tk = *reinterpret_cast<const u32x4*>(q + d + (int64_t)row * ld + ks * 16 + fh * 8);
      tv = *reinterpret_cast<const u32x4*>(q + 2 * d + (int64_t)row * ld + ks * 16 + fh * 8);
    }
    kf[ks] = __builtin_bit_cast(bf16x8, tk);
    vf[ks] = __builtin_bit_cast(bf16x8, tv);
  }

  const uint64_t qa = reinterpret_cast<uint64_t>(q), oa = reinterpret_cast<uint64_t>(dO);
  const uint32_t recq = (uint32_t)((((int64_t)S - 1) * ld + HD) * 2), reco = (uint32_t)((((int64_t)S - 1) * ldc + HD) * 2);
  const u32x4 rsQ = {(uint32_t)qa, (uint32_t)(qa >> 32) & 0xFFFFu, recq, 0x00020000u};
  const u32x4 rsO = {(uint32_t)oa, (uint32_t)(oa >> 32) & 0xFFFFu, reco, 0x00020000u};
  // per-query scalars travel with the tile (64 floats each; the lanes past them, and queries past the sequence
  // end, fetch zeros)
  const uint64_t la = reinterpret_cast<uint64_t>(lse + (int64_t)bh * S), da = reinterpret_cast<uint64_t>(dsum + (int64_t)bh * S);
  const u32x4 rsL = {(uint32_t)la, (uint32_t)(la >> 32) & 0xFFFFu, (uint32_t)S * 4u, 0x00020000u};
  const u32x4 rsD = {(uint32_t)da, (uint32_t)(da >> 32) & 0xFFFFu, (uint32_t)S * 4u, 0x00020000u};
  const uint32_t vos = lane < 16 ? (uint32_t)lane * 16u : 0x80000000u;
  uint32_t voq[IQ], voo[IQ];
#pragma unroll
  for (int jj = 0; jj < IQ; ++jj) {
    const int pc = (wave * IQ + jj) * 64 + lane, r = pc / PPR, c = (pc % PPR) ^ swq(r);
    voq[jj] = (uint32_t)((r * ld + c * 8) * 2);
    voo[jj] = (uint32_t)((r * ldc + c * 8) * 2);
  }
  const uint32_t lds0 = (uint32_t)reinterpret_cast<uintptr_t>(lds);
  auto request = [&](int it) __attribute__((always_inline)) {
    const uint32_t sq = (uint32_t)((int64_t)it * QT * ld * 2), so = (uint32_t)((int64_t)it * QT * ldc * 2);
    const uint32_t buf = lds0 + (uint32_t)(it & 1) * BUF, dst = buf + (uint32_t)wave * (IQ * 1024);
#pragma unroll
    for (int jj = 0; jj < IQ; ++jj) dma_b128(rsQ, dst + jj * 1024, voq[jj], sq);
#pragma unroll
    for (int jj = 0; jj < IQ; ++jj) dma_b128(rsO, dst + TQ + jj * 1024, voo[jj], so);
    if (wave == 0) dma_b128(rsL, buf + 2 * TQ, vos, (uint32_t)(it * QT * 4));
    if (wave == 1) dma_b128(rsD, buf + 2 * TQ + 1024, vos, (uint32_t)(it * QT * 4));
  };

  // fragment of tile rows in pi order (block blk of 32 queries, k-step ks) and transposing reads (k-step t = 16
  // queries, rows 16 t + 8 fh + sl/4 (+4), column block nb), as in the forward kernel
  int faddr[2][KS];
#pragma unroll
  for (int blk = 0; blk < 2; ++blk) {
    const int r = blk * 32 + pi_row(fr);
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) faddr[blk][ks] = r * ROWB + (((2 * ks + fh) ^ swq(r)) * 16);
  }
  const int sl = lane & 15;
  int xaddr[NB][2];
#pragma unroll
  for (int hh = 0; hh < 2; ++hh) {
    const int krow = 8 * fh + (sl >> 2) + 4 * hh;
#pragma unroll
    for (int nb = 0; nb < NB; ++nb) {
      const int col = nb * 32 + 16 * ((lane >> 4) & 1) + 4 * (sl & 3);
      xaddr[nb][hh] = krow * ROWB + (((col >> 3) ^ swq(krow)) * 16) + (col & 7) * 2;
    }
  }
  auto tr_frag = [&](const unsigned char* base, int a0, int a1) __attribute__((always_inline)) {
    const v4i16 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((v4i16 __attribute__((address_space(3)))*)(base + a0));
    const v4i16 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((v4i16 __attribute__((address_space(3)))*)(base + a1));
    typedef short v8i16 __attribute__((ext_vector_type(8)));
    const v8i16 both = {lo[0], lo[1], lo[2], lo[3], hi[0], hi[1], hi[2], hi[3]};
    return __builtin_bit_cast(bf16x8, both);
  };

  f32x16 vacc[NB], kacc[NB];
#pragma unroll
  for (int nb = 0; nb < NB; ++nb)
#pragma unroll
    for (int e = 0; e < 16; ++e) vacc[nb][e] = kacc[nb][e] = 0.f;

  const int all_tiles = (S + QT - 1) / QT;
  const int it0 = CAUSAL ? kb * KB / QT : 0;  // earlier tiles hold no query at or after this block's first key
  request(it0);
  for (int it = it0; it < all_tiles; ++it) {
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __syncthreads();  // tile `it` has landed for everyone; nobody reads the other buffer any more
    if (it + 1 < all_tiles) request(it + 1);
    if (CAUSAL && it * QT + QT - 1 < j0) continue;  // every query of the tile precedes this wavefront's keys
    const unsigned char* Qb = lds + (it & 1) * BUF;
    const unsigned char* Ob = Qb + TQ;
    // The tile's two blocks of 32 queries go through three phases each -- A: S^T and dP^T (2 KS products), B: the
    // probabilities and dS^T from them (an exponential and a handful of VALU instructions per element), C: the
    // sums into dV and dK (4 NB products) -- software-pipelined so that the VALU work of one block issues in the
    // shadow of the other block's products: A(0); A(1) with B(0); C(0) with B(1); C(1).  A wavefront issues in
    // order and a product holds the matrix pipe for 32 cycles, about what one element of phase B costs.
    f32x4 lq[2][4], dq4[2][4];  // per-query scalars: element e of a lane is query qb0 + 16 (e / 8) + 8 fh + e % 8
#pragma unroll
    for (int blk = 0; blk < 2; ++blk)
#pragma unroll
      for (int c = 0; c < 4; ++c) {
        const int off = (blk * 32 + 16 * (c >> 1) + 8 * fh + 4 * (c & 1)) * 4;
        lq[blk][c] = *reinterpret_cast<const f32x4*>(Qb + 2 * TQ + off);
        dq4[blk][c] = *reinterpret_cast<const f32x4*>(Qb + 2 * TQ + 1024 + off);
      }
    f32x16 st[2], dpt[2];
    bf16x8 pf[2][2], sf[2][2];
    bool plain[2];
#pragma unroll
    for (int blk = 0; blk < 2; ++blk) {
      const int qb0 = it * QT + blk * 32;
      // no query of the block is masked for any key of this wavefront: all inside the sequence and, under the
      // causal mask, at or after its last key
      plain[blk] = qb0 + 32 <= S && (!CAUSAL || qb0 >= j0 + 31);
#pragma unroll
      for (int e = 0; e < 16; ++e) st[blk][e] = dpt[blk][e] = 0.f;
    }
    auto element = [&](int blk, int e) __attribute__((always_inline)) {  // phase B for one element
      const int qi = it * QT + blk * 32 + 16 * (e / 8) + 8 * fh + e % 8;
      // (bitwise, not short-circuit: a branch per element would break the interleaving up)
      const bool ok = plain[blk] | ((qi < S) & (!CAUSAL | (qi >= row)));
      const float ex = __builtin_amdgcn_exp2f(__builtin_fmaf(st[blk][e], scale_log2e, -lq[blk][e / 4][e % 4]));
      const float pr = ok ? ex : 0.f;
      pf[blk][e / 8][e % 8] = static_cast<__bf16>(pr);
      sf[blk][e / 8][e % 8] = static_cast<__bf16>(scale * pr * (dpt[blk][e] - dq4[blk][e / 4][e % 4]));
    };
    constexpr int EA = 16 / KS, EC = 16 / (2 * NB);  // elements of phase B per pair of products of phase A / C
    auto phase_a = [&](int blk, int other) __attribute__((always_inline)) {  // other >= 0: phase B of that block rides along
      bf16x8 xq[2], xo[2];
      xq[0] = *reinterpret_cast<const bf16x8*>(Qb + faddr[blk][0]);
      xo[0] = *reinterpret_cast<const bf16x8*>(Ob + faddr[blk][0]);
#pragma unroll
      for (int ks = 0; ks < KS; ++ks) {
        if (ks + 1 < KS) {
          xq[(ks + 1) & 1] = *reinterpret_cast<const bf16x8*>(Qb + faddr[blk][ks + 1]);
          xo[(ks + 1) & 1] = *reinterpret_cast<const bf16x8*>(Ob + faddr[blk][ks + 1]);
        }
        st[blk] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(xq[ks & 1], kf[ks], st[blk], 0, 0, 0);
        if (other >= 0)
#pragma unroll
          for (int e = 0; e < EA / 2; ++e) element(other, ks * EA + e);
        __builtin_amdgcn_sched_barrier(0);
        dpt[blk] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(xo[ks & 1], vf[ks], dpt[blk], 0, 0, 0);
        if (other >= 0)
#pragma unroll
          for (int e = EA / 2; e < EA; ++e) element(other, ks * EA + e);
        __builtin_amdgcn_sched_barrier(0);
      }
    };
    auto phase_c = [&](int blk, int other) __attribute__((always_inline)) {
      bf16x8 xo[2][NB], xq[2][NB];
#pragma unroll
      for (int nb = 0; nb < NB; ++nb) {
        xo[0][nb] = tr_frag(Ob + (2 * blk) * 16 * ROWB, xaddr[nb][0], xaddr[nb][1]);
        xq[0][nb] = tr_frag(Qb + (2 * blk) * 16 * ROWB, xaddr[nb][0], xaddr[nb][1]);
      }
#pragma unroll
      for (int t2 = 0; t2 < 2; ++t2) {
#pragma unroll
        for (int nb = 0; nb < NB; ++nb) {
          if (t2 == 0) {  // the second k-step's fragments are read under the first one's products
            xo[1][nb] = tr_frag(Ob + (2 * blk + 1) * 16 * ROWB, xaddr[nb][0], xaddr[nb][1]);
            xq[1][nb] = tr_frag(Qb + (2 * blk + 1) * 16 * ROWB, xaddr[nb][0], xaddr[nb][1]);
          }
          vacc[nb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(xo[t2][nb], pf[blk][t2], vacc[nb], 0, 0, 0);
          if (other >= 0)
#pragma unroll
            for (int e = 0; e < EC / 2; ++e) element(other, (t2 * NB + nb) * EC + e);
          __builtin_amdgcn_sched_barrier(0);
          kacc[nb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(xq[t2][nb], sf[blk][t2], kacc[nb], 0, 0, 0);
          if (other >= 0)
#pragma unroll
            for (int e = EC / 2; e < EC; ++e) element(other, (t2 * NB + nb) * EC + e);
          __builtin_amdgcn_sched_barrier(0);
        }
      }
    };
    static_assert(EA >= 2 && EC >= 2 && EA * KS == 16 && EC * 2 * NB == 16, "all 16 elements of a block ride along");
    phase_a(0, -1);
    phase_a(1, 0);
    phase_c(0, 1);
    phase_c(1, -1);
  }
  // dK and dV leave through LDS (store_rows_staged), in the tile buffers
  if (row_ok && cos_sin) unrotate<NB>(kacc, cos_sin + (int64_t)row * (HD / 2), fh);
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
  __syncthreads();  // every wavefront is done with the tiles
  constexpr int OSTG = 32 * (ROWB + 16);
  static_assert(4 * 2 * OSTG <= 2 * BUF, "staging fits the tile buffers");
  bf16* dk0 = dqkv + (int64_t)b * S * ld + d + (int64_t)h * HD + (int64_t)j0 * ld;
  store_rows_staged<NB>(kacc, 1.0f, lds + (2 * wave) * OSTG, dk0, ld, S - j0, lane);
  store_rows_staged<NB>(vacc, 1.0f, lds + (2 * wave + 1) * OSTG, dk0 + d, ld, S - j0, lane);
}

inline bool al16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15) == 0; }

}  // namespace

// prob may be null for the forward (the probabilities are then not stored)
bool attention_fwd_fused_applies(int dt, int S, int hd, int64_t ld, int64_t ldc, const void* qkv, const void* prob, const void* ctx) {
  return dt == DT_BF16 && (hd == 64 || hd == 128) && S >= 8 && S % 8 == 0 && ld % 8 == 0 && ldc % 8 == 0 && al16(qkv) && al16(prob) &&
         (int64_t)S * ld * 2 < (int64_t(1) << 32) && (int64_t)S * S * 2 <= (int64_t(1) << 31) && al16(ctx);
}

namespace {
template <bool BWD_>
hipError_t attn_launch(int B, int H, int S, int hd, bool causal, const void* qkv, int64_t ld, void* prob, void* ctx, int64_t ldc,
                       const void* dctx, float* lse, float* dsum, void* dqkv, const float* cos_sin, hipStream_t st) {
  if (B == 0 || H == 0 || S == 0) return hipSuccess;
  const float2* cs = reinterpret_cast<const float2*>(cos_sin);
  const float sc = (1.0f / sqrtf((float)hd)) * (BWD_ ? 1.0f : 1.4426950408889634f);
  // 128-row workgroups when there are enough of them to give every compute unit two; else 64-row ones
  const bool big = (int64_t)B * H * ((S + 127) / 128) >= 512;
  const int qb = big ? 128 : 64;
  const int64_t nblk = (int64_t)((S + qb - 1) / qb) * B * H;
  if (nblk > 0x7FFFFFFF) return hipErrorInvalidValue;
  const dim3 grid((unsigned)nblk);
  const bf16* x = reinterpret_cast<const bf16*>(qkv);
  bf16* p = reinterpret_cast<bf16*>(prob);
  bf16* o = reinterpret_cast<bf16*>(ctx);
  const bf16* dO = reinterpret_cast<const bf16*>(dctx);
  bf16* dq = reinterpret_cast<bf16*>(dqkv);
#define ATTN_LAUNCH(HD_, C_)                                                                                       \
  do {                                                                                                             \
    if (big) attn_k<HD_, C_, 4, BWD_><<<grid, 256, 0, st>>>(x, ld, S, H, B * H, sc, p, o, ldc, dO, lse, dsum, dq, cs); \
    else attn_k<HD_, C_, 2, BWD_><<<grid, 128, 0, st>>>(x, ld, S, H, B * H, sc, p, o, ldc, dO, lse, dsum, dq, cs);     \
  } while (0)
  if (hd == 128) {
    if (causal) ATTN_LAUNCH(128, true); else ATTN_LAUNCH(128, false);
  } else if (hd == 64) {
    if (causal) ATTN_LAUNCH(64, true); else ATTN_LAUNCH(64, false);
  } else {
    return hipErrorInvalidValue;
  }
#undef ATTN_LAUNCH
  return hipGetLastError();
}
}  // namespace

hipError_t attention_fwd_fused(int B, int H, int S, int hd, bool causal, const void* qkv, int64_t ld, void* prob, void* ctx,
                               int64_t ldc, float* lse, hipStream_t st) {
  return attn_launch<false>(B, H, S, hd, causal, qkv, ld, prob, ctx, ldc, nullptr, lse, nullptr, nullptr, nullptr, st);
}

bool attention_bwd_fused_applies(int dt, int S, int hd, int64_t ld, int64_t ldc, const void* qkv, const void* ctx, const void* dctx,
                                 const void* dqkv) {
  return attention_fwd_fused_applies(dt, S, hd, ld, ldc, qkv, nullptr, ctx) && ldc % 8 == 0 && al16(ctx) && al16(dctx) &&
         (reinterpret_cast<uintptr_t>(dqkv) & 15) == 0;
}

hipError_t attention_bwd_fused(int B, int H, int S, int hd, bool causal, const void* qkv, int64_t ld, const void* ctx,
                               const float* lse, const void* dctx, int64_t ldc, float* dsum, void* dqkv, const float* cos_sin,
                               hipStream_t st) {
  if (!lse || !dsum) return hipErrorInvalidValue;
  hipError_t e = attn_launch<true>(B, H, S, hd, causal, qkv, ld, nullptr, const_cast<void*>(ctx), ldc, dctx, const_cast<float*>(lse),
                                   dsum, dqkv, cos_sin, st);
  if (e != hipSuccess || B == 0 || H == 0 || S == 0) return e;
  const int64_t nblk = (int64_t)((S + 127) / 128) * B * H;
  if (nblk > 0x7FFFFFFF) return hipErrorInvalidValue;
  const dim3 grid((unsigned)nblk);
  const bf16* x = reinterpret_cast<const bf16*>(qkv);
  const bf16* dO = reinterpret_cast<const bf16*>(dctx);
  bf16* dq = reinterpret_cast<bf16*>(dqkv);
  const float2* cs = reinterpret_cast<const float2*>(cos_sin);
  const float sc = 1.0f / sqrtf((float)hd);
  if (hd == 128) {
    if (causal) attn_bwd_kv_k<128, true><<<grid, 256, 0, st>>>(x, ld, S, H, B * H, sc, lse, dsum, dO, ldc, dq, cs);
    else attn_bwd_kv_k<128, false><<<grid, 256, 0, st>>>(x, ld, S, H, B * H, sc, lse, dsum, dO, ldc, dq, cs);
  } else if (hd == 64) {
    if (causal) attn_bwd_kv_k<64, true><<<grid, 256, 0, st>>>(x, ld, S, H, B * H, sc, lse, dsum, dO, ldc, dq, cs);
    else attn_bwd_kv_k<64, false><<<grid, 256, 0, st>>>(x, ld, S, H, B * H, sc, lse, dsum, dO, ldc, dq, cs);
  } else {
    return hipErrorInvalidValue;
  }
  return hipGetLastError();
}

}  // namespace hift
