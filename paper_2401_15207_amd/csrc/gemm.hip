// Contractions of the HiFT step for gfx950:  C[M,N] = A[M,K] . B[N,K]^T (+ bias) (+ residual).
//
// One kernel family serves every linear layer of the forward pass, the activation gradients
// (dX = dY . W) and the weight gradients of the active group (dW = dY^T . X), because each
// operand may be stored contraction-major ("k-major", the 8 values an MFMA lane needs are
// contiguous) or transposed; a transposed operand is turned around in registers on its way
// from HBM to LDS, so no transposed copy of a weight or activation is ever materialised.
//
//   * bf16: LDS-staged, double-buffered BMxBNx64 macro-tiles, four wavefronts in a 2x2 grid,
//     each computing (BM/2)x(BN/2) with v_mfma_f32_32x32x16_bf16, fp32 accumulation.
//     LDS rows are 128 bytes (64 bf16) with the 16-byte chunk index XOR-swizzled by the row so
//     that both the 16-byte stores and the MFMA fragment reads spread over all banks.
//   * bf16 with the weight operand pre-packed in MFMA fragment order (forward and dX of the large layers, the
//     dominant kernel of a step): 128x256 tiles, weight fragments straight from memory into registers, the
//     activation operand through a ring of direct-to-LDS stages, epilogues (bias, residual, RoPE, SwiGLU and GELU
//     forward and backward, folded RMS normalisation) straight from the accumulators.  See further down.
//   * fp32 and odd shapes: a plain 64x64x16 LDS-tiled FMA kernel with arbitrary strides.
#include <type_traits>

#include "common.h"
#include "kernels.h"

namespace hift {
namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;  // a 16-byte piece held in registers

struct GemmP {
  int64_t M, N, K;
  const void* A; int64_t lda;
  const void* B; int64_t ldb;
  void* C; int64_t ldc;
  const void* bias;
  const void* R; int64_t ldr;
  int nh;
  int64_t sa1, sa2, sb1, sb2, sc1, sc2;
  int tiles_m, tiles_n;
  int band = 0;
  // fused epilogues of the packed-operand kernel
  void* C2 = nullptr; int64_t ldc2 = 0;
  const float2* cos_sin = nullptr; int S = 1; int64_t rot_cols = 0;
  // split tail of the packed-operand kernel: workgroups from split_from on work in groups of `split` on one
  // tile each, every member a share of the k range; ws: counters (first 1 KB) and partial tiles
  int split_from = 0x7FFFFFFF, split = 1;
  unsigned char* ws = nullptr;
  // row normalisation folded into the packed-operand kernel (see Gemm in kernels.h)
  float* rowsq_out = nullptr;
  const float* rowsq = nullptr; int rowsq_n = 0; float norm_eps = 0.f; float* norm_stats = nullptr;
};

// ------------------------------------------------------------------------------------------
// bf16 MFMA kernel
// ------------------------------------------------------------------------------------------
constexpr int KT = 64;  // k extent of a macro-tile

// 16-byte chunk c of LDS row r lives at chunk position c ^ f(r), f(r) = (r ^ (r >> 3)) & 7.
// Both the fragment reads (32 rows, one chunk) and the staging stores (k-major: one row, 8 chunks;
// transposed: rows 8 apart, one chunk) then spread over all banks.  f(r + 64) = f(r) and
// f(r + 32) = f(r) ^ 4, so the fragment addresses of a lane are two registers (even and odd
// 32-row blocks) plus immediates.
__device__ __forceinline__ int swz_f(int row) { return (row ^ (row >> 3)) & 7; }
__device__ __forceinline__ int swz(int row, int chunk) { return chunk ^ swz_f(row); }

// Staging of one operand tile (ROWS x 64 bf16) from HBM through registers into LDS, in 16-byte
// pieces.  Loads are raw buffer loads: a 32-bit byte offset per lane plus a scalar offset that
// advances along k, and reads past the end of the operand return zero.  That covers rows past
// the edge and, for transposed sources, the ragged k edge; a k-major ragged k edge (KTAIL) is
// zeroed by hand, because there the next row's data follows in memory.
// k-major source: thread t owns chunk (t % 8) of rows t/8 + 32 i.
// transposed source ([K][rows]): thread t owns 8x8 blocks; block b = t + 256 i covers rows
// 8 (b % (ROWS/8))..+7 and k-chunk b / (ROWS/8); it is loaded as 8 source rows and turned
// around in registers, so LDS always holds [row][k].
template <int ROWS, bool KMAJOR, bool KTAIL>
struct Stage {
  static constexpr int NBLK = ROWS >= 256 ? ROWS / 256 : 1;
  static constexpr int NPIECE = KMAJOR ? ROWS / 32 : 8 * NBLK;
  __amdgpu_buffer_rsrc_t rsrc;
  uint32_t voff;   // byte offset of this lane's first piece at k = 0
  uint32_t step;   // k-major: bytes between pieces (32 rows); transposed: bytes per source row
  uint32_t step2;  // transposed: bytes between this lane's blocks
  int64_t K;
  int kpos;  // first k of this lane's pieces inside a tile (k-major)

  __device__ __forceinline__ void init(const bf16* src, int64_t ld, int64_t row0, int64_t nrows, int64_t K_, int tid) {
    K = K_;
    const int64_t lines = KMAJOR ? nrows : K_, width = KMAJOR ? K_ : nrows;
    const int64_t bytes = lines > 0 ? ((lines - 1) * ld + width) * 2 : 0;
    rsrc = __builtin_amdgcn_make_buffer_rsrc(const_cast<bf16*>(src), 0, (int)(uint32_t)bytes, 0x00020000);
    if (KMAJOR) {
      kpos = (tid & 7) * 8;
      int64_t row = row0 + (tid >> 3);
      // a row past the edge must stay past the end of the buffer after 32-bit wrap: clamp to the first such row
      row = row < nrows ? row : nrows;
      voff = (uint32_t)((row * ld + kpos) * 2);
      step = (uint32_t)(32 * ld * 2);
      step2 = 0;
    } else {
      constexpr int RB = ROWS / 8;
      const int b = tid % ROWS;  // ROWS < 256: the upper threads repeat the lower ones' loads
      int64_t row = row0 + (int64_t)(b % RB) * 8;
      kpos = (b / RB) * 8;
      // rows past the edge: point the lane past the end of the buffer (reads as zero)
      voff = row + 8 <= nrows ? (uint32_t)(((int64_t)kpos * ld + row) * 2) : 0xFFFFFFF0u;
      step = (uint32_t)(ld * 2);
      step2 = (uint32_t)((256 / RB) * 8 * ld * 2);
    }
  }

  __device__ __forceinline__ void load(int64_t kt, u32x4 (&r)[NPIECE]) const {
    if (KMAJOR) {
      const uint32_t so = (uint32_t)(kt * KT * 2);
      const bool live = !KTAIL || kt * KT + kpos < K;
#pragma unroll
      for (int i = 0; i < NPIECE; ++i) {
        r[i] = __builtin_amdgcn_raw_buffer_load_b128(rsrc, (int)(voff + i * step), (int)so, 0);
        if (KTAIL && !live) r[i] = u32x4{0, 0, 0, 0};
      }
    } else {
#pragma unroll
      for (int i = 0; i < NBLK; ++i)
#pragma unroll
        for (int j = 0; j < 8; ++j) {
          const uint32_t so = (uint32_t)(kt * KT + j) * step;
          r[i * 8 + j] = __builtin_amdgcn_raw_buffer_load_b128(rsrc, (int)(voff + i * step2), (int)so, 0);
        }
    }
  }

  __device__ __forceinline__ void store(unsigned char* lds, int tid, const u32x4 (&r)[NPIECE]) const {
    if (KMAJOR) {
      const int row = tid >> 3;
      unsigned char* dst0 = lds + row * 128 + swz(row, tid & 7) * 16;
      unsigned char* dst1 = lds + row * 128 + swz(row + 32, tid & 7) * 16;
#pragma unroll
      for (int i = 0; i < NPIECE; ++i) *reinterpret_cast<u32x4*>(((i & 1) ? dst1 : dst0) + i * 4096) = r[i];
    } else {
      constexpr int RB = ROWS / 8;
#pragma unroll
      for (int i = 0; i < NBLK; ++i) {
        const int b = (tid + 256 * i) % ROWS;
        const int rowb = (b % RB) * 8, c = b / RB;
        // r[i*8 + j] holds, for k = j, the 8 rows rowb..rowb+7 (two per dword).  Turn the 8x8
        // block around: output row m gets k = 0..7.
#pragma unroll
        for (int m = 0; m < 8; ++m) {
          u32x4 o;
#pragma unroll
          for (int q = 0; q < 4; ++q) {  // r[i*8 + j][q'] holds k = j, rows 2q', 2q'+1
            const uint32_t lo = r[i * 8 + 2 * q][m >> 1], hi = r[i * 8 + 2 * q + 1][m >> 1];
            o[q] = (m & 1) ? __builtin_amdgcn_perm(hi, lo, 0x07060302u) : __builtin_amdgcn_perm(hi, lo, 0x05040100u);
          }
          const int row = rowb + m;
          *reinterpret_cast<u32x4*>(lds + row * 128 + swz(row, c) * 16) = o;
        }
      }
    }
  }
};


// Epilogue shared by the contraction kernels: accumulators (transposed sub-tiles, see above) ->
// C (+bias)(+residual), through LDS when rows can be moved as 16-byte pieces.
template <int WM, int WN, bool VEC_EPI, typename OutT>
__device__ __forceinline__ void store_tile(const GemmP& p, f32x16 (&acc)[WM / 32][WN / 32], unsigned char* smem,
                                           int64_t m0, int64_t n0, int wm, int wn, int wave, int lane, int zb, int zh) {
  constexpr int MT = WM / 32, NT = WN / 32;
  const int frow = lane & 31, fhalf = lane >> 5;
  // ---- epilogue ----
  OutT* C = reinterpret_cast<OutT*>(p.C) + zb * p.sc1 + zh * p.sc2;
  const OutT* R = p.R ? reinterpret_cast<const OutT*>(p.R) + zb * p.sc1 + zh * p.sc2 : nullptr;
  const bf16* bias = reinterpret_cast<const bf16*>(p.bias);
  if (VEC_EPI) {
    // Stage up to 64 rows of the wave's tile in LDS as fp32 [rows][WN] (+16 bytes per row), then
    // walk whole rows: bias and residual are added in fp32 before the one rounding, and every
    // global access is a 16-byte piece of a contiguous row segment.
    constexpr int RP = WM < 64 ? WM : 64;
    constexpr int PITCH = WN * 4 + 16;
    constexpr int CPR = WN / 8;    // 8-column chunks per row
    constexpr int RPI = 64 / CPR;  // rows per sweep of the wave
    unsigned char* reg = smem + wave * (RP * PITCH);
    const int cc = lane % CPR, rr = lane / CPR;
    const int64_t col = n0 + wn * WN + cc * 8;
    float bv[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) bv[e] = 0.f;
    if (bias && col < p.N) {
      const bf16x8 t = *reinterpret_cast<const bf16x8*>(bias + col);
#pragma unroll
      for (int e = 0; e < 8; ++e) bv[e] = static_cast<float>(t[e]);
    }
#pragma unroll
    for (int pass = 0; pass < WM / RP; ++pass) {
      __syncthreads();  // operand tiles (first pass) or the previous pass are no longer read
#pragma unroll
      for (int ii = 0; ii < RP / 32; ++ii)
#pragma unroll
        for (int j = 0; j < NT; ++j)
#pragma unroll
          for (int g = 0; g < 4; ++g) {
            const int i = pass * (RP / 32) + ii;
            const f32x4 v = {acc[i][j][4 * g], acc[i][j][4 * g + 1], acc[i][j][4 * g + 2], acc[i][j][4 * g + 3]};
            *reinterpret_cast<f32x4*>(reg + (ii * 32 + frow) * PITCH + (j * 32 + 8 * g + 4 * fhalf) * 4) = v;
          }
      __syncthreads();
#pragma unroll 2
      for (int it = 0; it < RP / RPI; ++it) {
        const int lr = it * RPI + rr;
        const int64_t row = m0 + wm * WM + pass * RP + lr;
        if (row >= p.M || col >= p.N) continue;
        f32x4 lo = *reinterpret_cast<const f32x4*>(reg + lr * PITCH + cc * 32);
        f32x4 hi = *reinterpret_cast<const f32x4*>(reg + lr * PITCH + cc * 32 + 16);
#pragma unroll
        for (int e = 0; e < 4; ++e) { lo[e] += bv[e]; hi[e] += bv[4 + e]; }
        if (sizeof(OutT) == 2) {
          if (R) {
            const bf16x8 rv = *reinterpret_cast<const bf16x8*>(reinterpret_cast<const bf16*>(R) + row * p.ldr + col);
#pragma unroll
            for (int e = 0; e < 4; ++e) { lo[e] += static_cast<float>(rv[e]); hi[e] += static_cast<float>(rv[4 + e]); }
          }
          bf16x8 t;
#pragma unroll
          for (int e = 0; e < 4; ++e) { t[e] = static_cast<__bf16>(lo[e]); t[4 + e] = static_cast<__bf16>(hi[e]); }
          *reinterpret_cast<bf16x8*>(reinterpret_cast<bf16*>(C) + row * p.ldc + col) = t;
        } else {
          float* cp = reinterpret_cast<float*>(C) + row * p.ldc + col;
          if (R) {
            const float* rp = reinterpret_cast<const float*>(R) + row * p.ldr + col;
            lo += *reinterpret_cast<const f32x4*>(rp);
            hi += *reinterpret_cast<const f32x4*>(rp + 4);
          }
          *reinterpret_cast<f32x4*>(cp) = lo;
          *reinterpret_cast<f32x4*>(cp + 4) = hi;
        }
      }
    }
  } else {
#pragma unroll
    for (int i = 0; i < MT; ++i) {
      const int64_t row = m0 + wm * WM + i * 32 + frow;
      if (row >= p.M) continue;
#pragma unroll
      for (int j = 0; j < NT; ++j)
#pragma unroll
        for (int g = 0; g < 4; ++g) {
          const int64_t col = n0 + wn * WN + j * 32 + 8 * g + 4 * fhalf;
          {
#pragma unroll
            for (int e = 0; e < 4; ++e) {
              if (col + e >= p.N) continue;
              float v = acc[i][j][4 * g + e] + (bias ? to_f32(bias[col + e]) : 0.f);
              if (R) v += to_f32(R[row * p.ldr + col + e]);
              C[row * p.ldc + col + e] = from_f32<OutT>(v);
            }
          }
        }
    }
  }
}

// Four wavefronts in a 2x2 grid, each (BM/2)x(BN/2).  The accumulators hold the transposed
// tile (the weight-side operand is fed as MFMA's first operand), so that one lane owns four
// consecutive output columns of one output row and the epilogue can store vectors.
// Lane l, accumulator element e of sub-tile (i, j): output row i*32 + l%32,
// column j*32 + 8*(e/4) + 4*(l/32) + e%4.
template <int BM, int BN, bool AK, bool BKM, bool KTAIL, bool VEC_EPI, typename OutT>
__global__ void __launch_bounds__(256) gemm_mfma_k(GemmP p) {
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  constexpr int WM = BM / 2, WN = BN / 2, MT = WM / 32, NT = WN / 32;
  constexpr int A_BYTES = BM * 128, B_BYTES = BN * 128, BUF = A_BYTES + B_BYTES;

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave >> 1, wn = wave & 1;
  // Workgroups are dealt round-robin to the 8 XCDs, each with its own L2.  Give every XCD a
  // contiguous run of tiles, ordered so that neighbours share the same B (weight) tile.
  int tile = blockIdx.x;
  const int ntile = p.tiles_m * p.tiles_n;
  if ((ntile & 7) == 0) tile = (tile & 7) * (ntile >> 3) + (tile >> 3);
  const int tm = tile % p.tiles_m, tn = tile / p.tiles_m;
  const int z = blockIdx.y, zb = z / p.nh, zh = z % p.nh;
  const bf16* A = reinterpret_cast<const bf16*>(p.A) + zb * p.sa1 + zh * p.sa2;
  const bf16* B = reinterpret_cast<const bf16*>(p.B) + zb * p.sb1 + zh * p.sb2;
  const int64_t m0 = (int64_t)tm * BM, n0 = (int64_t)tn * BN;

  f32x16 acc[MT][NT];
#pragma unroll
  for (int i = 0; i < MT; ++i)
#pragma unroll
    for (int j = 0; j < NT; ++j)
#pragma unroll
      for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;

  typedef Stage<BM, AK, KTAIL> StA;
  typedef Stage<BN, BKM, KTAIL> StB;
  StA sa;
  StB sb;
  sa.init(A, p.lda, m0, p.M, p.K, tid);
  sb.init(B, p.ldb, n0, p.N, p.K, tid);
  const int64_t nk = (p.K + KT - 1) / KT;
  // k-tiles [kb, ke) of this output tile; a band hint (causal attention) shortens the range
  int64_t kb = 0, ke = nk;
  if (p.band == BAND_SKIP_UPPER && n0 >= m0 + BM) return;  // uniform over the workgroup
  if (p.band == BAND_K_UPTO_ROW) ke = (m0 + BM + KT - 1) / KT < nk ? (m0 + BM + KT - 1) / KT : nk;
  if (p.band == BAND_K_FROM_ROW) kb = m0 / KT < nk - 1 ? m0 / KT : nk - 1;
  u32x4 ra[StA::NPIECE], rb[StB::NPIECE];  // the next tile on its way from HBM to LDS

  sa.load(kb, ra);
  sb.load(kb, rb);
  sa.store(smem + (kb & 1) * BUF, tid, ra);
  sb.store(smem + (kb & 1) * BUF + A_BYTES, tid, rb);
  __syncthreads();

  const int frow = lane & 31, fhalf = lane >> 5;
  bf16x8 fa[2][MT], fb[2][NT];
  // byte offset of this lane's fragment chunk for each k-step; rows 32 apart add 4096 bytes
  int foff[KT / 16][2];  // [k-step][parity of the 32-row block]
#pragma unroll
  for (int ks = 0; ks < KT / 16; ++ks) {
    foff[ks][0] = frow * 128 + swz(frow, ks * 2 + fhalf) * 16;
    foff[ks][1] = frow * 128 + swz(frow + 32, ks * 2 + fhalf) * 16;
  }
  static_assert(WM % 64 == 0 && WN % 64 == 0, "wave tiles start at multiples of 64 rows");
  const int a_base = wm * WM * 128, b_base = A_BYTES + wn * WN * 128;
  auto read_frags = [&](bf16x8(&a)[MT], bf16x8(&b)[NT], const unsigned char* buf, int ks) __attribute__((always_inline)) {
#pragma unroll
    for (int i = 0; i < MT; ++i) a[i] = *reinterpret_cast<const bf16x8*>(buf + foff[ks][i & 1] + (a_base + i * 4096));
#pragma unroll
    for (int j = 0; j < NT; ++j) b[j] = *reinterpret_cast<const bf16x8*>(buf + foff[ks][j & 1] + (b_base + j * 4096));
  };
  read_frags(fa[0], fb[0], smem + (kb & 1) * BUF, 0);

  // One pass over a k-tile held in one of the two LDS buffers.  Every k-step is its own scheduling region.
  // A wavefront cannot issue anything while it waits for the matrix pipe to take its next MFMA,
  // so the memory instructions of a region are dealt out between its MFMAs:
  //   step 0     global loads of tile kt+1 into registers, fragment reads of step 1
  //   steps 1,2  fragment reads of the next step
  //   step 3a    LDS stores of tile kt+1 into the other buffer, which was last read before the
  //              previous barrier; first half of the MFMAs
  //   barrier
  //   step 3b    fragment reads of step 0 of tile kt+1; second half of the MFMAs
  // Tiles past the end are the last tile again: loaded, stored, never used.
  constexpr bool HINT = AK && BKM;  // the counts describe k-major staging; transposed staging schedules freely
  constexpr int NM = MT * NT, NR = MT + NT, NL = StA::NPIECE + StB::NPIECE;
  for (int64_t kt = kb; kt < ke; ++kt) {
    unsigned char* cur = smem + (kt & 1) * BUF;
    unsigned char* nxt = smem + ((kt + 1) & 1) * BUF;
    const int64_t kt2 = kt + 1 < ke ? kt + 1 : ke - 1;
#pragma unroll
    for (int ks = 0; ks < KT / 16 - 1; ++ks) {
      if (ks == 0) {
        sa.load(kt2, ra);
        sb.load(kt2, rb);
      }
      read_frags(fa[(ks + 1) & 1], fb[(ks + 1) & 1], cur, ks + 1);
#pragma unroll
      for (int i = 0; i < MT; ++i)
#pragma unroll
        for (int j = 0; j < NT; ++j)
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fb[ks & 1][j], fa[ks & 1][i], acc[i][j], 0, 0, 0);
      if (HINT) {
#pragma unroll
        for (int q = 0; q < NM; ++q) {
          __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
          if (ks == 0 && q < NL) __builtin_amdgcn_sched_group_barrier(0x020, (NL + NM - 1) / NM, 0);
          if (q < NR) __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
        }
      }
      __builtin_amdgcn_sched_barrier(0);
    }
    constexpr int KL = KT / 16 - 1, HM = MT / 2;
    sa.store(nxt, tid, ra);
    sb.store(nxt + A_BYTES, tid, rb);
#pragma unroll
    for (int i = 0; i < HM; ++i)
#pragma unroll
      for (int j = 0; j < NT; ++j)
        acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fb[KL & 1][j], fa[KL & 1][i], acc[i][j], 0, 0, 0);
    if (HINT) {
#pragma unroll
      for (int q = 0; q < HM * NT; ++q) {
        __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
        __builtin_amdgcn_sched_group_barrier(0x200, (NL + HM * NT - 1) / (HM * NT), 0);
      }
    }
    __builtin_amdgcn_sched_barrier(0);
    __syncthreads();
    __builtin_amdgcn_sched_barrier(0);
    read_frags(fa[0], fb[0], nxt, 0);
#pragma unroll
    for (int i = HM; i < MT; ++i)
#pragma unroll
      for (int j = 0; j < NT; ++j)
        acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fb[KL & 1][j], fa[KL & 1][i], acc[i][j], 0, 0, 0);
    if (HINT) {
#pragma unroll
      for (int q = 0; q < (MT - HM) * NT; ++q) {
        __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
        __builtin_amdgcn_sched_group_barrier(0x100, (NR + (MT - HM) * NT - 1) / ((MT - HM) * NT), 0);
      }
    }
    __builtin_amdgcn_sched_barrier(0);
  }

  store_tile<WM, WN, VEC_EPI, OutT>(p, acc, smem, m0, n0, wm, wn, wave, lane, zb, zh);
}

// Direct-to-LDS load of 16 bytes per lane: M0 carries the LDS address of lane 0's piece and lane l
// lands 16 l bytes further.  Inline assembly, with hand-placed s_waitcnt where the data is read:
// the compiler cannot see which LDS reads depend on which load and would otherwise wait for all
// of them before every read.
__device__ __forceinline__ void load_to_lds_b128(u32x4 rsrc, uint32_t lds_addr, uint32_t voff, uint32_t soff) {
  asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tbuffer_load_dwordx4 %1, %2, %3 offen lds"
               :
               : "s"(lds_addr), "v"(voff), "s"(rsrc), "s"(soff)
               : "memory");
}

// ------------------------------------------------------------------------------------------
// bf16 MFMA kernel with the weight operand pre-packed in MFMA fragment order
// ------------------------------------------------------------------------------------------
// Weights do not change inside a step, so the library keeps a second copy of every large weight
// matrix in the order the MFMA wants it: block (nb, kk) of 1 KB holds, for lane l, the 8 values
// B[nb*32 + pi(l%32)][kk*16 + (l/32)*8 ..+7] (pi_row below: why the rows of a block are permuted).  A wavefront loads its B fragments straight from
// HBM/L2 into registers with fully coalesced 1 KB loads, eight k-steps ahead; only the activation
// operand goes through LDS.  Rows of the packed copy are padded to a multiple of 256, so no load
// leaves the buffer.
constexpr int PKF = 8;  // k-steps of B fragments in flight per wavefront

// Position in the packed copy of the 32-row block s of B (half = blocks in half of B).
__device__ __forceinline__ int64_t pk_block_pos(int64_t s, int order, int64_t half) {
  if (order == PK_ORDER_HALVES) {
    if (s >= 2 * half) return s;  // no such block: N is a multiple of 256 in this order
    const int64_t h = s >= half ? 1 : 0, i = s - h * half;
    return (i >> 2) * 8 + (i & 3) * 2 + h;
  }
  if (order == PK_ORDER_PAIR64) {
    const int64_t q = s & 3;
    return (s & ~int64_t(3)) | (q == 1 ? 2 : q == 2 ? 1 : q);
  }
  return s;
}

// Row r of a 32-row block of B sits where row pi(r) would (bits 2 and 3 of the index exchanged).  acc = mfma(B
// fragment, A fragment, acc) leaves in lane l, element e the entry (A row l % 32, B row 8 (e / 4) + 4 (l / 32) + e % 4);
// with the rows fed in this order, element e belongs to column 16 (e / 8) + 8 (l / 32) + e % 8 of the block: elements
// 0..7 and 8..15 are eight consecutive columns each, 16 bytes of a bf16 output row, and the epilogues of the
// packed-operand kernel write rows straight from the registers.
__device__ __forceinline__ int pi_row(int r) { return (r & ~12) | ((r & 4) << 1) | ((r & 8) >> 1); }

// Product of eight bf16 pairs, each rounded once.
__device__ __forceinline__ u32x4 scale8(u32x4 a, u32x4 b) {
  bf16x8 x = __builtin_bit_cast(bf16x8, a);
  const bf16x8 y = __builtin_bit_cast(bf16x8, b);
#pragma unroll
  for (int e = 0; e < 8; ++e) x[e] = static_cast<__bf16>(static_cast<float>(x[e]) * static_cast<float>(y[e]));
  return __builtin_bit_cast(u32x4, x);
}

// Eight consecutive values of the source as bf16: a 16-byte load, or, for an fp32 source (the master weights), two
// loads and eight roundings to nearest even -- the bf16 model is by definition that rounding of the master.
__device__ __forceinline__ u32x4 load8_bf16(const bf16* p) { return *reinterpret_cast<const u32x4*>(p); }
__device__ __forceinline__ u32x4 load8_bf16(const float* p) {
  const f32x4 a = *reinterpret_cast<const f32x4*>(p), b = *reinterpret_cast<const f32x4*>(p + 4);
  bf16x8 t;
#pragma unroll
  for (int e = 0; e < 4; ++e) { t[e] = static_cast<__bf16>(a[e]); t[4 + e] = static_cast<__bf16>(b[e]); }
  return __builtin_bit_cast(u32x4, t);
}
__device__ __forceinline__ bf16 load1_bf16(const bf16* p) { return *p; }
__device__ __forceinline__ bf16 load1_bf16(const float* p) { return static_cast<__bf16>(*p); }

// The packers take an optional gain [K]: the copy then holds B[n][k] gain[k] (a row normalisation's gain folded
// into the weight that consumes the normalised rows).
// Generic packer (any alignment): one wavefront per 1 KB block, element-wise reads.
template <typename SrcT>
__global__ void __launch_bounds__(256) pack_b_k(const SrcT* __restrict__ B, int64_t ldb, int64_t N, int64_t K,
                                                 bool b_kmajor, u32x4* __restrict__ Bp, int64_t n_blocks, int64_t k_steps,
                                                 int order, int64_t half, const bf16* __restrict__ gain) {
  const int64_t w = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
  if (w >= n_blocks * k_steps) return;
  const int lane = threadIdx.x & 63;
  const int64_t nb = w / k_steps, kk = w % k_steps;
  const int64_t n = nb * 32 + pi_row(lane & 31), k0 = kk * 16 + (lane >> 5) * 8;
  bf16x8 v;
#pragma unroll
  for (int e = 0; e < 8; ++e) {
    const int64_t k = k0 + e;
    float x = 0.f;
    if (n < N && k < K) x = static_cast<float>(load1_bf16(b_kmajor ? B + n * ldb + k : B + k * ldb + n));
    if (gain && k < K) x *= static_cast<float>(gain[k]);
    v[e] = static_cast<__bf16>(x);
  }
  Bp[(pk_block_pos(nb, order, half) * k_steps + kk) * 64 + lane] = __builtin_bit_cast(u32x4, v);
}

// Packer for 16-byte aligned sources: a workgroup moves a 16 KB tile through LDS so that both the
// reads of the source and the writes of the 1 KB blocks are whole contiguous runs.
//   KMAJOR: tile = 32 rows (one n-block) x 256 k (16 k-steps); source rows are contiguous in k.
//   else:   tile = 32 k (two k-steps) x 256 n (eight n-blocks); source rows are contiguous in n.
template <bool KMAJOR, typename SrcT>
__global__ void __launch_bounds__(256) pack_b_tile_k(const SrcT* __restrict__ B, int64_t ldb, int64_t N, int64_t K,
                                                      u32x4* __restrict__ Bp, int64_t k_steps, int tiles_inner, int order,
                                                      int64_t half, const bf16* __restrict__ gain) {
  constexpr int PITCH = 512 + 16;  // bytes per tile row in LDS; the pad spreads 16-byte reads of one column over the banks
  __shared__ __attribute__((aligned(16))) unsigned char tile[32 * PITCH];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int64_t to = blockIdx.x / tiles_inner, ti = blockIdx.x % tiles_inner;
  const u32x4 zero = {0u, 0u, 0u, 0u};
  if (KMAJOR) {
    const int64_t nb = to, k00 = ti * 256;
#pragma unroll
    for (int ps = 0; ps < 4; ++ps) {
      const int r = ps * 8 + (tid >> 5), c = (tid & 31) * 8;
      const int64_t n = nb * 32 + r, k = k00 + c;
      u32x4 v = zero;
      if (n < N && k < K) v = load8_bf16(B + n * ldb + k);
      if (gain && n < N && k < K) v = scale8(v, *reinterpret_cast<const u32x4*>(gain + k));  // K % 8 == 0 here
      *reinterpret_cast<u32x4*>(tile + r * PITCH + c * 2) = v;
    }
    __syncthreads();
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const int kkl = wave * 4 + j;
      const int64_t kk = ti * 16 + kkl;
      if (kk < k_steps)
        Bp[(pk_block_pos(nb, order, half) * k_steps + kk) * 64 + lane] =
            *reinterpret_cast<const u32x4*>(tile + pi_row(lane & 31) * PITCH + (kkl * 16 + (lane >> 5) * 8) * 2);
    }
  } else {
    const int64_t kk0 = to * 2, n00 = ti * 256;
#pragma unroll
    for (int ps = 0; ps < 4; ++ps) {
      const int r = ps * 8 + (tid >> 5), c = (tid & 31) * 8;
      const int64_t k = kk0 * 16 + r, n = n00 + c;
      u32x4 v = zero;
      if (n + 8 <= N) {
        v = load8_bf16(B + k * ldb + n);
      } else if (n < N) {
        bf16x8 t;
#pragma unroll
        for (int e = 0; e < 8; ++e) t[e] = n + e < N ? load1_bf16(B + k * ldb + n + e) : static_cast<__bf16>(0.f);
        v = __builtin_bit_cast(u32x4, t);
      }
      if (gain && k < K) {
        const float gk = static_cast<float>(gain[k]);
        bf16x8 t = __builtin_bit_cast(bf16x8, v);
#pragma unroll
        for (int e = 0; e < 8; ++e) t[e] = static_cast<__bf16>(static_cast<float>(t[e]) * gk);
        v = __builtin_bit_cast(u32x4, t);
      }
      *reinterpret_cast<u32x4*>(tile + r * PITCH + c * 2) = v;
    }
    __syncthreads();
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const int idx = wave * 4 + j, nbl = idx >> 1, kkl = idx & 1;
      bf16x8 t;
#pragma unroll
      for (int e = 0; e < 8; ++e)
        t[e] = *reinterpret_cast<const bf16*>(tile + (kkl * 16 + (lane >> 5) * 8 + e) * PITCH + (nbl * 32 + pi_row(lane & 31)) * 2);
      Bp[(pk_block_pos(ti * 8 + nbl, order, half) * k_steps + kk0 + kkl) * 64 + lane] = __builtin_bit_cast(u32x4, t);
    }
  }
}

// ------------------------------------------------------------------------------------------
// The contraction kernel: a (32 MT) x 256 tile; the four wavefronts sit side by side along N, each
// (32 MT) x 64, and a stage of A is 64 k wide.  Every 128-byte line of either operand is then
// requested exactly once per compute unit: no wavefront shares a B fragment with another, and an A
// row piece is a whole line (half lines and fragments shared by two wavefronts cost a third of the
// speed in earlier layouts).  All wavefronts read all of A from LDS: MT 1 KB fragment reads per
// 2 MT MFMAs, a quarter of what LDS delivers (about 240 bytes per clock per compute unit, measured).
//   A stages arrive by direct-to-LDS loads into a ring of four, requested three stages ahead.
//   LDS row = 128 bytes = eight 16-byte pieces; piece c of tile row r sits at r*128 + (c ^ ((r>>1)&7))*16,
//   so that sixteen consecutive rows of one piece fall into sixteen different 16-byte bank groups;
//   a load instruction fills 8 rows (lane l -> row l/8, position l%8), so the swizzle is applied by
//   choosing which global piece a lane fetches.
// MT = 4 (128 x 256 tiles) is the instantiation in use: at M = 2048 it gives the 7B shapes whole
// numbers of rounds over 256 compute units more often than 256 x 256 does, and ran faster.
constexpr int PK_DK = 64, PK_STAGES = 4, PK_RD = 3, PK_ROW = 128;
constexpr int PK_SQ_MAX = 12;  // folded normalisation: 16-byte pieces of row partials a thread holds (K <= 6144)

// Fused epilogues of the packed-operand kernel (bf16 output).  The packed copy holds B's 32-row blocks in
// an order (PK_ORDER_*) that puts, side by side in a wavefront's two accumulator columns, the blocks
// that are combined element by element: gate and up block of the same features (EPI_SWIGLU), or a
// block and the one 64 columns further in the same head (EPI_ROPE): both values then sit in the same
// lane and element of the two accumulators.
// x / (1 + e^-x) with the hardware's base-2 exponential and reciprocal (about 1e-7 relative each; the
// library's expf and the IEEE division cost more than the memory traffic of the elementwise kernels).
// e^-x = inf for x < -88: 1 / inf = 0 and the result is -0.
__device__ __forceinline__ float silu_fast(float x) {
  return x * __builtin_amdgcn_rcpf(1.0f + __builtin_amdgcn_exp2f(-1.4426950408889634f * x));
}

// erf by formula 7.1.26 of Abramowitz and Stegun (absolute error below 1.5e-7, far inside bf16), with the hardware's
// reciprocal and base-2 exponential: the library's erff would make an epilogue issue-bound.
__device__ __forceinline__ float erf_fast(float z) {
  const float a = fabsf(z);
  const float t = __builtin_amdgcn_rcpf(1.0f + 0.3275911f * a);
  const float poly = t * (0.254829592f + t * (-0.284496736f + t * (1.421413741f + t * (-1.453152027f + t * 1.061405429f))));
  return copysignf(1.0f - poly * __builtin_amdgcn_exp2f(-1.4426950408889634f * a * a), z);
}
// x Phi(x) and its derivative Phi(x) + x phi(x)
__device__ __forceinline__ float gelu_fast(float x) { return 0.5f * x * (1.0f + erf_fast(0.70710678118654752f * x)); }
__device__ __forceinline__ float gelu_grad_fast(float x) {
  return 0.5f * (1.0f + erf_fast(0.70710678118654752f * x)) +
         x * 0.3989422804014327f * __builtin_amdgcn_exp2f(-0.72134752044448170f * x * x);
}

// Epilogues of the packed-operand kernel, straight from the registers (see pi_row): lane (frow, fh) holds, of tile rows
// 32 i + frow and each of its wavefront's two 32-column blocks j, the columns 16 h + 8 fh ..+7 (h = 0, 1) as elements
// 8 h ..+7 of acc[i][j]: a 16-byte piece of a bf16 row.  The four pieces of a row's 64 columns are stored by
// consecutive instructions and meet again in the L2 line.  No LDS, no barrier.
//   EPI_NONE        C = acc (+ bias) (+ R), bf16 or fp32; with rowsq_out also the sum of squares of the row's 64 stored values
//   EPI_SWIGLU      blocks j = 0 / 1 are gate / up of the same features (PK_ORDER_HALVES)
//   EPI_ROPE        block j = 1 lies 64 columns after block j = 0 in the same head (PK_ORDER_PAIR64)
//   EPI_SWIGLU_BWD  acc = d act; with the forward's pre-activations g | u (C2, [M, 2 N]) writes d g = d act u s (1 + g (1 - s))
//                   and d u = d act g s, s = 1 / (1 + e^-g), to C [M, 2 N]
//   EPI_GELU        pre = acc + bias to C (if given), gelu of the rounded pre to C2
//   EPI_GELU_BWD    acc = d act; with the forward's pre-activations (C2) writes d act gelu'(pre) to C
// row_rstd (forward epilogues, or null): the folded row normalisation's factor per tile row.
template <int MT, typename OutT, int EPI>
__device__ __forceinline__ void store_tile_regs(const GemmP& p, f32x16 (&acc)[MT][2], int64_t m0, int64_t n0, int tn, int wave,
                                                int lane, const float* row_rstd) {
  const int frow = lane & 31, fh = lane >> 5;
  bf16* C = reinterpret_cast<bf16*>(p.C);
  auto round8 = [](const float (&x)[8]) __attribute__((always_inline)) {
    bf16x8 t;
#pragma unroll
    for (int e = 0; e < 8; ++e) t[e] = static_cast<__bf16>(x[e]);
    return t;
  };
#pragma unroll
  for (int i = 0; i < MT; ++i) {
    const int64_t row = m0 + 32 * i + frow;
    const bool ok = row < p.M;
    const float rs = row_rstd ? row_rstd[32 * i + frow] : 1.0f;
    if constexpr (EPI == EPI_NONE) {
      float q = 0.f;
#pragma unroll
      for (int j = 0; j < 2; ++j)
#pragma unroll
        for (int h = 0; h < 2; ++h) {
          const int64_t col = n0 + wave * 64 + j * 32 + 16 * h + 8 * fh;
          if (!ok || col >= p.N) continue;
          float x[8];
#pragma unroll
          for (int e = 0; e < 8; ++e) x[e] = acc[i][j][8 * h + e];
          if (p.bias) {
            const bf16x8 bv = *reinterpret_cast<const bf16x8*>(reinterpret_cast<const bf16*>(p.bias) + col);
#pragma unroll
            for (int e = 0; e < 8; ++e) x[e] += static_cast<float>(bv[e]);
          }
          if constexpr (sizeof(OutT) == 2) {
            if (p.R) {
              const bf16x8 rv = *reinterpret_cast<const bf16x8*>(reinterpret_cast<const bf16*>(p.R) + row * p.ldr + col);
#pragma unroll
              for (int e = 0; e < 8; ++e) x[e] += static_cast<float>(rv[e]);
            }
            const bf16x8 t = round8(x);
            *reinterpret_cast<bf16x8*>(C + row * p.ldc + col) = t;
#pragma unroll
            for (int e = 0; e < 8; ++e) q += static_cast<float>(t[e]) * static_cast<float>(t[e]);
          } else {
            float* cp = reinterpret_cast<float*>(p.C) + row * p.ldc + col;
            if (p.R) {
              const float* rp = reinterpret_cast<const float*>(p.R) + row * p.ldr + col;
              const f32x4 r0 = *reinterpret_cast<const f32x4*>(rp), r1 = *reinterpret_cast<const f32x4*>(rp + 4);
#pragma unroll
              for (int e = 0; e < 4; ++e) { x[e] += r0[e]; x[4 + e] += r1[e]; }
            }
            *reinterpret_cast<f32x4*>(cp) = f32x4{x[0], x[1], x[2], x[3]};
            *reinterpret_cast<f32x4*>(cp + 4) = f32x4{x[4], x[5], x[6], x[7]};
          }
        }
      if constexpr (sizeof(OutT) == 2) {
        if (p.rowsq_out) {  // N is a whole number of strips here; the row's other half is in lane + 32
          q += __shfl_xor(q, 32, 64);
          if (ok && fh == 0) p.rowsq_out[row * (p.N / 64) + (n0 >> 6) + wave] = q;
        }
      }
    } else if constexpr (EPI == EPI_SWIGLU) {
#pragma unroll
      for (int h = 0; h < 2; ++h) {
        const int64_t feat = 128 * (int64_t)tn + 32 * wave + 16 * h + 8 * fh;
        if (!ok) continue;
        float g[8], u[8];
#pragma unroll
        for (int e = 0; e < 8; ++e) { g[e] = acc[i][0][8 * h + e] * rs; u[e] = acc[i][1][8 * h + e] * rs; }
        const bf16x8 gb = round8(g), ub = round8(u);
        if (C) {
          *reinterpret_cast<bf16x8*>(C + row * p.ldc + feat) = gb;
          *reinterpret_cast<bf16x8*>(C + row * p.ldc + p.N / 2 + feat) = ub;
        }
        float a[8];  // the activation from the values as they are stored
#pragma unroll
        for (int e = 0; e < 8; ++e) a[e] = silu_fast(static_cast<float>(gb[e])) * static_cast<float>(ub[e]);
        *reinterpret_cast<bf16x8*>(reinterpret_cast<bf16*>(p.C2) + row * p.ldc2 + feat) = round8(a);
      }
    } else if constexpr (EPI == EPI_ROPE) {
#pragma unroll
      for (int h = 0; h < 2; ++h) {
        const int fq = 32 * (wave & 1) + 16 * h + 8 * fh;  // frequency index = column within the first half of the head
        const int64_t c1 = 256 * (int64_t)tn + 128 * (wave >> 1) + fq;  // x1's column; x2's is 64 further
        if (!ok) continue;
        float x1[8], x2[8];
#pragma unroll
        for (int e = 0; e < 8; ++e) { x1[e] = acc[i][0][8 * h + e] * rs; x2[e] = acc[i][1][8 * h + e] * rs; }
        if (c1 < p.rot_cols) {
          // pairs (x1, x2):  x1' = x1 cos - x2 sin,  x2' = x2 cos + x1 sin
          const float2* cs = p.cos_sin + (int64_t)((uint32_t)row % (uint32_t)p.S) * 64 + fq;
#pragma unroll
          for (int e = 0; e < 8; ++e) {
            const float2 c = cs[e];
            const float y1 = x1[e] * c.x - x2[e] * c.y, y2 = x2[e] * c.x + x1[e] * c.y;
            x1[e] = y1;
            x2[e] = y2;
          }
        }
        *reinterpret_cast<bf16x8*>(C + row * p.ldc + c1) = round8(x1);
        *reinterpret_cast<bf16x8*>(C + row * p.ldc + c1 + 64) = round8(x2);
      }
    } else if constexpr (EPI == EPI_GELU || EPI == EPI_GELU_BWD) {
      bf16* C2 = reinterpret_cast<bf16*>(p.C2);
#pragma unroll
      for (int j = 0; j < 2; ++j)
#pragma unroll
        for (int h = 0; h < 2; ++h) {
          const int64_t col = n0 + wave * 64 + j * 32 + 16 * h + 8 * fh;
          if (!ok || col >= p.N) continue;
          float x[8];
#pragma unroll
          for (int e = 0; e < 8; ++e) x[e] = acc[i][j][8 * h + e];
          if constexpr (EPI == EPI_GELU) {
            if (p.bias) {
              const bf16x8 bv = *reinterpret_cast<const bf16x8*>(reinterpret_cast<const bf16*>(p.bias) + col);
#pragma unroll
              for (int e = 0; e < 8; ++e) x[e] += static_cast<float>(bv[e]);
            }
            const bf16x8 pb = round8(x);
            if (C) *reinterpret_cast<bf16x8*>(C + row * p.ldc + col) = pb;
#pragma unroll
            for (int e = 0; e < 8; ++e) x[e] = gelu_fast(static_cast<float>(pb[e]));  // from the values as they are stored
            *reinterpret_cast<bf16x8*>(C2 + row * p.ldc2 + col) = round8(x);
          } else {
            const bf16x8 pv = *reinterpret_cast<const bf16x8*>(C2 + row * p.ldc2 + col);
#pragma unroll
            for (int e = 0; e < 8; ++e) x[e] *= gelu_grad_fast(static_cast<float>(pv[e]));
            *reinterpret_cast<bf16x8*>(C + row * p.ldc + col) = round8(x);
          }
        }
    } else {
      const bf16* GU = reinterpret_cast<const bf16*>(p.C2);
#pragma unroll
      for (int j = 0; j < 2; ++j)
#pragma unroll
        for (int h = 0; h < 2; ++h) {
          const int64_t col = n0 + wave * 64 + j * 32 + 16 * h + 8 * fh;
          if (!ok || col >= p.N) continue;
          const bf16x8 gv = *reinterpret_cast<const bf16x8*>(GU + row * p.ldc2 + col);
          const bf16x8 uv = *reinterpret_cast<const bf16x8*>(GU + row * p.ldc2 + p.N + col);
          float dg[8], du[8];
#pragma unroll
          for (int e = 0; e < 8; ++e) {
            const float da = acc[i][j][8 * h + e];
            const float g = static_cast<float>(gv[e]), u = static_cast<float>(uv[e]);
            const float sg = __builtin_amdgcn_rcpf(1.0f + __builtin_amdgcn_exp2f(-1.4426950408889634f * g));
            dg[e] = da * u * sg * (1.0f + g * (1.0f - sg));
            du[e] = da * g * sg;
          }
          *reinterpret_cast<bf16x8*>(C + row * p.ldc + col) = round8(dg);
          *reinterpret_cast<bf16x8*>(C + row * p.ldc + p.N + col) = round8(du);
        }
    }
  }
}

template <int MT, bool VEC_EPI, typename OutT, int EPI = EPI_NONE>
__global__ void __launch_bounds__(256) gemm_pk_k(GemmP p, const u32x4* __restrict__ Bp, int64_t k_steps) {
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  constexpr int BM = 32 * MT, BN = 256, NT = 2;
  constexpr int STG = BM * PK_ROW;  // one stage of A
  constexpr int NP = MT;            // 1 KB pieces (8 rows) of a stage each wavefront requests

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  // Whole tiles first (a multiple of 256 of them when the tail is split, else all), then the tiles of the
  // last, partial round, each shared by `split` workgroups that take consecutive shares of the k range.
  int tile = blockIdx.x, part = 0, unit = -1;
  const bool shared_tile = tile >= p.split_from;
  if (shared_tile) {
    unit = tile - p.split_from;
    part = unit % p.split;
    tile = p.split_from + unit / p.split;
  } else {
    const int ntile = p.split > 1 ? p.split_from : p.tiles_m * p.tiles_n;
    if ((ntile & 7) == 0) tile = (tile & 7) * (ntile >> 3) + (tile >> 3);  // contiguous run of tiles per XCD
  }
  const int band = tile / (8 * p.tiles_n), in_band = tile - band * 8 * p.tiles_n;
  const int band_rows = min(8, p.tiles_m - band * 8);
  const int tm = band * 8 + in_band % band_rows, tn = in_band / band_rows;
  const bf16* A = reinterpret_cast<const bf16*>(p.A);
  const int64_t m0 = (int64_t)tm * BM, n0 = (int64_t)tn * BN;
  const int64_t nk = p.K / PK_DK;
  const int64_t kt0 = shared_tile ? nk * part / p.split : 0, kt1 = shared_tile ? nk * (part + 1) / p.split : nk;

  f32x16 acc[MT][NT];
#pragma unroll
  for (int i = 0; i < MT; ++i)
#pragma unroll
    for (int j = 0; j < NT; ++j)
#pragma unroll
      for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;

  // A: direct-to-LDS; lane l of piece gi carries LDS bytes [16 l, 16 l + 16) of rows gi*8 .. gi*8+7
  const uint64_t aa = reinterpret_cast<uint64_t>(A);
  const u32x4 rsA = {(uint32_t)aa, (uint32_t)(aa >> 32) & 0xFFFFu, (uint32_t)(((p.M - 1) * p.lda + p.K) * 2), 0x00020000u};
  uint32_t voA[NP];
#pragma unroll
  for (int gi = 0; gi < NP; ++gi) {
    const int r = wave * (BM / 4) + gi * 8 + (lane >> 3);  // row in the tile
    const int c = (lane & 7) ^ ((r >> 1) & 7);             // which 16 bytes of the row's 128 this lane fetches
    const int64_t ra = m0 + r;
    voA[gi] = (uint32_t)(((ra < p.M ? ra : p.M) * p.lda + c * 8) * 2);  // rows past M start past the buffer: zeros
  }
  const uint32_t lds0 = (uint32_t)reinterpret_cast<uintptr_t>(smem);
  auto request_piece = [&](int64_t stage, int gi) __attribute__((always_inline)) {
    const uint32_t so = (uint32_t)(stage * PK_DK * 2);
    const uint32_t dst = lds0 + (uint32_t)(stage & (PK_STAGES - 1)) * STG + (uint32_t)wave * (BM / 4 * PK_ROW);
    load_to_lds_b128(rsA, dst + gi * 1024, voA[gi], so);
  };

  // B: packed fragments, straight into registers
  const int64_t pk_bytes = (int64_t)p.tiles_n * 8 * k_steps * 1024;
  const __amdgpu_buffer_rsrc_t rsB = __builtin_amdgcn_make_buffer_rsrc(const_cast<u32x4*>(Bp), 0, (int)(uint32_t)pk_bytes, 0x00020000);
  const uint32_t vb = (uint32_t)lane * 16;
  const uint32_t nb0 = (uint32_t)((n0 >> 5) + wave * NT);
  // Inline assembly, like the direct-to-LDS loads of A: the compiler counts only the loads it knows of, so with this
  // one a builtin it waited, before every use of a fragment, until no more than the 15 younger B loads were
  // outstanding -- but the requests for A lie between them, which made the fragments wait for loads issued five
  // k-steps after them instead of eight.  The waits are placed by hand in kstep, with the true counts.
  auto load_b1 = [&](u32x4& dst, int64_t kk, int j) __attribute__((always_inline)) {
    const int64_t kc = kk < k_steps ? kk : k_steps - 1;  // past the end: the last block again
    const uint32_t so = (uint32_t)(((nb0 + j) * k_steps + kc) * 1024);
    asm volatile("buffer_load_dwordx4 %0, %1, %2, %3 offen" : "=v"(dst) : "v"(vb), "s"(rsB), "s"(so) : "memory");
  };

  const int frow = lane & 31, fhalf = lane >> 5;
  int foff[4];
#pragma unroll
  for (int ks = 0; ks < 4; ++ks) foff[ks] = frow * PK_ROW + (((ks * 2 + fhalf) ^ ((frow >> 1) & 7)) * 16);
  bf16x8 fa[2][MT];
  auto read_a1 = [&](bf16x8& a, const unsigned char* buf, int ks, int i) __attribute__((always_inline)) {
    a = *reinterpret_cast<const bf16x8*>(buf + foff[ks] + i * 32 * PK_ROW);
  };
  u32x4 bq[PKF][NT];

#pragma unroll
  for (int s = 0; s < PK_RD; ++s)
#pragma unroll
    for (int gi = 0; gi < NP; ++gi) request_piece(kt0 + s, gi);
  // The first fragments and the wait for them in one statement: between a load and its wait the registers hold
  // nothing yet, and the compiler, which takes them for defined, may move them elsewhere when registers are short
  // (seen in a variant of this kernel: copies into accumulator registers right behind the loads).  Four k-steps
  // lie 1 KB apart behind one scalar offset; a k range of fewer than PKF k-steps (loads past the end repeat the
  // last fragment) takes them one by one.
  static_assert(PKF == 8 && NT == 2, "operands of the statement below");
  if (kt0 * 4 + PKF <= k_steps) {
    const uint32_t o0 = (uint32_t)((nb0 * k_steps + kt0 * 4) * 1024), o1 = o0 + (uint32_t)(k_steps * 1024);
    const uint32_t o2 = o0 + 4096u, o3 = o1 + 4096u;
    asm volatile(
        "buffer_load_dwordx4 %0, %16, %17, %18 offen\n\t"
        "buffer_load_dwordx4 %1, %16, %17, %19 offen\n\t"
        "buffer_load_dwordx4 %2, %16, %17, %18 offen offset:1024\n\t"
        "buffer_load_dwordx4 %3, %16, %17, %19 offen offset:1024\n\t"
        "buffer_load_dwordx4 %4, %16, %17, %18 offen offset:2048\n\t"
        "buffer_load_dwordx4 %5, %16, %17, %19 offen offset:2048\n\t"
        "buffer_load_dwordx4 %6, %16, %17, %18 offen offset:3072\n\t"
        "buffer_load_dwordx4 %7, %16, %17, %19 offen offset:3072\n\t"
        "buffer_load_dwordx4 %8, %16, %17, %20 offen\n\t"
        "buffer_load_dwordx4 %9, %16, %17, %21 offen\n\t"
        "buffer_load_dwordx4 %10, %16, %17, %20 offen offset:1024\n\t"
        "buffer_load_dwordx4 %11, %16, %17, %21 offen offset:1024\n\t"
        "buffer_load_dwordx4 %12, %16, %17, %20 offen offset:2048\n\t"
        "buffer_load_dwordx4 %13, %16, %17, %21 offen offset:2048\n\t"
        "buffer_load_dwordx4 %14, %16, %17, %20 offen offset:3072\n\t"
        "buffer_load_dwordx4 %15, %16, %17, %21 offen offset:3072\n\t"
        "s_waitcnt vmcnt(0)"
        : "=&v"(bq[0][0]), "=&v"(bq[0][1]), "=&v"(bq[1][0]), "=&v"(bq[1][1]), "=&v"(bq[2][0]), "=&v"(bq[2][1]),
          "=&v"(bq[3][0]), "=&v"(bq[3][1]), "=&v"(bq[4][0]), "=&v"(bq[4][1]), "=&v"(bq[5][0]), "=&v"(bq[5][1]),
          "=&v"(bq[6][0]), "=&v"(bq[6][1]), "=&v"(bq[7][0]), "=&v"(bq[7][1])
        : "v"(vb), "s"(rsB), "s"(o0), "s"(o1), "s"(o2), "s"(o3)
        : "memory");
  } else {
#pragma unroll
    for (int s = 0; s < PKF; ++s)
#pragma unroll
      for (int j = 0; j < NT; ++j) {
        const int64_t kk = kt0 * 4 + s;
        const uint32_t so = (uint32_t)(((nb0 + j) * k_steps + (kk < k_steps ? kk : k_steps - 1)) * 1024);
        asm volatile("buffer_load_dwordx4 %0, %1, %2, %3 offen\n\ts_waitcnt vmcnt(0)"
                     : "=&v"(bq[s][j]) : "v"(vb), "s"(rsB), "s"(so) : "memory");
      }
  }
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
  __syncthreads();
#pragma unroll
  for (int i = 0; i < MT; ++i) read_a1(fa[0][i], smem + (kt0 & (PK_STAGES - 1)) * STG, 0, i);

  // Folded row normalisation: A holds the rows before normalisation and B the weight times the gain, so the
  // product only lacks each row's 1 / sqrt(mean of squares + eps).  The producer of A left the sums of squares
  // as K / 64 partials per row; two threads fetch a row's partials here (they arrive under the main loop; older
  // than every load of the loop, they are covered by its first wait) and add them up after it.
  __shared__ float row_rstd[BM];
  constexpr bool NORM_EPI = EPI == EPI_SWIGLU || EPI == EPI_ROPE;
  f32x4 sqv[NORM_EPI ? PK_SQ_MAX : 1];
  if constexpr (NORM_EPI) {
    static_assert(BM == 128, "two threads per row");
    if (p.rowsq) {
      const int hn4 = p.rowsq_n >> 3;  // 16-byte pieces per thread
      const int64_t row = m0 + (tid >> 1);
      const f32x4* src = reinterpret_cast<const f32x4*>(p.rowsq + (row < p.M ? row : 0) * p.rowsq_n) + (tid & 1) * hn4;
#pragma unroll
      for (int c = 0; c < PK_SQ_MAX; ++c) sqv[c] = c < hn4 ? src[c] : f32x4{0.f, 0.f, 0.f, 0.f};
    }
  }

  // One k-step: 2 MT MFMAs in the order (j, i); after the q-th one: q < MT: A fragment q of the next
  // k-step; q == MT: refill of B fragment 0; then (first two k-steps of a stage) NP / 2 pieces of the
  // request for a later stage; last: refill of B fragment 1.  A wavefront issues in order and an MFMA
  // holds the matrix pipe for 32 cycles, so every memory instruction sits in the shadow of one.
  auto kstep = [&](auto KS_, auto SLOT_, auto MAIN_, int64_t kt, const unsigned char* src_next) __attribute__((always_inline)) {
    constexpr int KS = decltype(KS_)::value, SLOT = decltype(SLOT_)::value;
    constexpr bool refill = decltype(MAIN_)::value != 0, read_next = decltype(MAIN_)::value != 2;  // 1: in the loop; 0, 2: tail
    // Loads issued since the fragment about to be used was requested (PKF k-steps = PKF / 4 stages ago; a stage
    // issues 8 B fragments and NP pieces of A): everything of those stages but the fragment itself (first B
    // fragment, used from q = 0) or but this k-step's share, which is not issued yet (second one, from q = MT).
    // In the tail nothing is requested any more: wait for everything.
    constexpr int W0 = refill ? (PKF / 4) * (8 + NP) - 1 : 0;
    constexpr int W1 = refill ? (PKF / 4) * (8 + NP) - 2 - (KS < 2 ? NP / 2 : 0) : 0;
#pragma unroll
    for (int q = 0; q < NT * MT; ++q) {
      const int j = q / MT, i = q % MT;
      // the fragment is an operand of the wait, so that the product cannot be moved in front of it
      if (q == 0) asm volatile("s_waitcnt vmcnt(%1)" : "+v"(bq[SLOT][0]) : "n"(W0) : "memory");
      if (q == MT) asm volatile("s_waitcnt vmcnt(%1)" : "+v"(bq[SLOT][1]) : "n"(W1) : "memory");
      acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, bq[SLOT][j]), fa[KS & 1][i], acc[i][j], 0, 0, 0);
      if (read_next && q < MT) read_a1(fa[(KS + 1) & 1][q], src_next, (KS + 1) & 3, q);
      if (refill) {
        if (q == MT) load_b1(bq[SLOT][0], kt * 4 + KS + PKF, 0);
        if (KS < 2 && q > MT && q <= MT + NP / 2) request_piece(kt + PK_RD, KS * (NP / 2) + q - MT - 1);
        if (q == NT * MT - 1) load_b1(bq[SLOT][1], kt * 4 + KS + PKF, 1);
      }
      __builtin_amdgcn_sched_barrier(0);
    }
  };
  static_assert(PKF == 8 && NP % 2 == 0 && MT + NP / 2 < NT * MT && 19 + 2 * MT <= 63 && (PKF / 4) * (8 + NP) - 1 <= 63,
                "slot rotation and wait counts");
  auto stage = [&](auto S0_, int64_t kt) __attribute__((always_inline)) {
    constexpr int S0 = decltype(S0_)::value;
    const unsigned char* cur = smem + (kt & (PK_STAGES - 1)) * STG;
    const unsigned char* nxt = smem + ((kt + 1) & (PK_STAGES - 1)) * STG;
    kstep(std::integral_constant<int, 0>{}, std::integral_constant<int, S0>{}, std::integral_constant<int, 1>{}, kt, cur);
    kstep(std::integral_constant<int, 1>{}, std::integral_constant<int, S0 + 1>{}, std::integral_constant<int, 1>{}, kt, cur);
    kstep(std::integral_constant<int, 2>{}, std::integral_constant<int, S0 + 2>{}, std::integral_constant<int, 1>{}, kt, cur);
    // Stage kt+1 is read from here on: its request (issued two stages ago) must have landed for every
    // wavefront.  Loads issued after its last piece: 5 of that stage, MT + 8 of the next, 6 + MT of this.
    asm volatile("s_waitcnt vmcnt(%0)" ::"n"(19 + 2 * MT) : "memory");
    __syncthreads();
    __builtin_amdgcn_sched_barrier(0);
    kstep(std::integral_constant<int, 3>{}, std::integral_constant<int, S0 + 3>{}, std::integral_constant<int, 1>{}, kt, nxt);
  };
  int64_t kt = kt0;
  for (; kt + 1 < kt1; kt += 2) {
    stage(std::integral_constant<int, 0>{}, kt);
    stage(std::integral_constant<int, 4>{}, kt + 1);
  }
  if (kt < kt1) {
    stage(std::integral_constant<int, 0>{}, kt++);
    if (p.K % PK_DK) {  // 32 columns left: two k-steps of the next stage (its A rows are half valid)
      const unsigned char* cur = smem + (kt & (PK_STAGES - 1)) * STG;
      kstep(std::integral_constant<int, 0>{}, std::integral_constant<int, 4>{}, std::integral_constant<int, 0>{}, kt, cur);
      kstep(std::integral_constant<int, 1>{}, std::integral_constant<int, 5>{}, std::integral_constant<int, 2>{}, kt, cur);
    }
  } else if (p.K % PK_DK) {
    const unsigned char* cur = smem + (kt & (PK_STAGES - 1)) * STG;
    kstep(std::integral_constant<int, 0>{}, std::integral_constant<int, 0>{}, std::integral_constant<int, 0>{}, kt, cur);
    kstep(std::integral_constant<int, 1>{}, std::integral_constant<int, 1>{}, std::integral_constant<int, 2>{}, kt, cur);
  }
  // Stray requests must land before LDS is reused -- and before the registers of the B fragments are: the last
  // refills are still on their way, and only as operands of this wait are those registers known to be taken.
#pragma unroll
  for (int s = 0; s < PKF; ++s) asm volatile("" : "+v"(bq[s][0]), "+v"(bq[s][1]));
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
#pragma unroll
  for (int s = 0; s < PKF; ++s) asm volatile("" : "+v"(bq[s][0]), "+v"(bq[s][1]));
  if constexpr (NORM_EPI) {
    if (p.rowsq) {
      const int r = tid >> 1;
      const int64_t row = m0 + r;
      float q = 0.f;
#pragma unroll
      for (int c = 0; c < PK_SQ_MAX; ++c) q += (sqv[c][0] + sqv[c][1]) + (sqv[c][2] + sqv[c][3]);
      q += __shfl_xor(q, 1);
      const float rstd = 1.0f / sqrtf(q / (float)p.K + p.norm_eps);
      if ((tid & 1) == 0) {
        row_rstd[r] = rstd;
        if (p.norm_stats && tn == 0 && part == 0 && row < p.M) {  // what the normalisation's backward reads
          p.norm_stats[2 * row] = 0.f;
          p.norm_stats[2 * row + 1] = rstd;
        }
      }
    }
  }

  if (shared_tile) {
    // Every member leaves its partial tile in its own slot (register order: 4 KB per wavefront and store)
    // and counts itself in; the member that finds all the others counted adds the slots up in their fixed
    // order (its own included: the sum must not depend on who came last) and goes on to the epilogue.
    // Nobody waits for anybody.  The members of a tile run on different XCDs, whose L2s do not see each
    // other's lines: slots are written and read with device-scope accesses (sc1: written through to memory,
    // read past the L2), which costs nothing but these accesses -- a device-scope fence instead writes back
    // and invalidates the whole L2 under the workgroups still computing and made the shared round slower
    // than a whole one.
    __shared__ int is_last;
    unsigned* count = reinterpret_cast<unsigned*>(p.ws) + (tile - p.split_from);
    constexpr int SLOTB = BM * BN * 4;  // bytes of a partial tile
    constexpr int SC1 = 16;             // cache-policy bit of the buffer instructions: device scope
    const __amdgpu_buffer_rsrc_t rsW = __builtin_amdgcn_make_buffer_rsrc(p.ws + 1024, 0, (int)(p.split * (p.tiles_m * p.tiles_n - p.split_from) * SLOTB), 0x00020000);
    const int mine = unit * SLOTB + tid * 16;
#pragma unroll
    for (int i = 0; i < MT; ++i)
#pragma unroll
      for (int j = 0; j < NT; ++j)
#pragma unroll
        for (int g = 0; g < 4; ++g) {
          const f32x4 v = {acc[i][j][4 * g], acc[i][j][4 * g + 1], acc[i][j][4 * g + 2], acc[i][j][4 * g + 3]};
          __builtin_amdgcn_raw_buffer_store_b128(__builtin_bit_cast(u32x4, v), rsW, mine, ((i * NT + j) * 4 + g) * 4096, SC1);
        }
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");  // this lane's part of the slot has reached memory
    __syncthreads();
    if (tid == 0) {
      const unsigned before = __hip_atomic_fetch_add(count, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      is_last = before == (unsigned)p.split - 1;
      if (is_last) __hip_atomic_store(count, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);  // every member has counted
    }
    __syncthreads();
    if (!is_last) return;
    const int first = (unit - part) * SLOTB + tid * 16;
#pragma unroll
    for (int i = 0; i < MT; ++i)
#pragma unroll
      for (int j = 0; j < NT; ++j)
#pragma unroll
        for (int g = 0; g < 4; ++g) {
          f32x4 sum = __builtin_bit_cast(f32x4, __builtin_amdgcn_raw_buffer_load_b128(rsW, first, ((i * NT + j) * 4 + g) * 4096, SC1));
          for (int q = 1; q < p.split; ++q)
            sum += __builtin_bit_cast(f32x4, __builtin_amdgcn_raw_buffer_load_b128(rsW, first + q * SLOTB, ((i * NT + j) * 4 + g) * 4096, SC1));
#pragma unroll
          for (int e = 0; e < 4; ++e) acc[i][j][4 * g + e] = sum[e];
        }
  }

  if constexpr (NORM_EPI) {
    if (p.rowsq) __syncthreads();  // row_rstd is complete
  }
  store_tile_regs<MT, OutT, EPI>(p, acc, m0, n0, tn, wave, lane, NORM_EPI && p.rowsq ? row_rstd : nullptr);
}

// ------------------------------------------------------------------------------------------
// bf16 MFMA kernel for two operands that are both stored contraction-index first: the weight gradient
// ------------------------------------------------------------------------------------------
// dW[out, in] = dY^T . X with dY [T, out] and X [T, in] as the backward pass leaves them: C[M, N] = sum_k A[k][m] B[k][n].
// The operands go from memory into LDS as they are (rows of k, m contiguous), by direct-to-LDS loads, and the
// MFMA fragments (lane l: row l % 32 of a 32-row block, the eight k-values 8 (l / 32) ..+7) are formed by
// transposing LDS reads (ds_read_b64_tr_b16: within a group of 16 lanes, lane i receives as element e what lane
// i/4 + 4e addressed as its element i%4), two per fragment.  No register staging and no in-register turn, which
// is what holds gemm_mfma_k back on these operands.
//   Tile 256 x 256, four wavefronts in a 2 x 2 grid, each 128 x 128 (256 accumulators); a stage is 32 k of both
//   operands (2 x 16 KB), a ring of four stages, requested three ahead, one barrier per stage in the middle of
//   the stage's second k-step.
//   LDS row = 512 bytes = 32 pieces of 16 bytes; piece c of k-row r sits at position c ^ ((r & 3) << 2): one
//   transposing read touches eight k-rows (r0 ..+3 and r0 + 8 ..+11), 64 bytes of each, which then fall into the
//   four 64-byte bank groups two by two -- the 512 bytes of the instruction in the two cycles they need anyway.
//   A load instruction fills two k-rows (lanes 0..31 and 32..63), so the swizzle is applied by choosing which
//   piece a lane fetches.
// Needs M and N multiples of 256 and K a multiple of 32 (every weight of the benchmark shapes); fp32 output.
constexpr int TT_BK = 32, TT_STAGES = 4, TT_ROWB = 512, TT_OPB = TT_BK * TT_ROWB, TT_STG = 2 * TT_OPB;

template <typename OutT>
__global__ void __launch_bounds__(256) gemm_tt_k(GemmP p) {
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  constexpr int BM = 256, BN = 256, WM = 128, WN = 128, MT = 4, NT = 4;
  typedef short v4i16 __attribute__((ext_vector_type(4)));
  typedef short v8i16 __attribute__((ext_vector_type(8)));
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wm = wave >> 1, wn = wave & 1;
  int tile = blockIdx.x;
  const int ntile = p.tiles_m * p.tiles_n;
  if ((ntile & 7) == 0) tile = (tile & 7) * (ntile >> 3) + (tile >> 3);  // a contiguous run of tiles per XCD
  // Bands of 8 tile rows, walked down the rows first: the 32 tiles an XCD works on at a time are an 8 x 4 block,
  // which shares each operand column 4 or 8 times in its L2 (a plain column of 32 tiles shares one operand only,
  // and 2.7 times as much came over the fabric).
  const int band = tile / (8 * p.tiles_n), in_band = tile - band * 8 * p.tiles_n;
  const int band_rows = min(8, p.tiles_m - band * 8);
  const int tm = band * 8 + in_band % band_rows, tn = in_band / band_rows;
  const int64_t m0 = (int64_t)tm * BM, n0 = (int64_t)tn * BN;
  const int64_t nst = p.K / TT_BK;

  f32x16 acc[MT][NT];
#pragma unroll
  for (int i = 0; i < MT; ++i)
#pragma unroll
    for (int j = 0; j < NT; ++j)
#pragma unroll
      for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;

  // ---- requests: wavefront w brings k-rows 8 w ..+7 of both operands of a stage, two rows per instruction
  const uint64_t aa = reinterpret_cast<uint64_t>(p.A), ba = reinterpret_cast<uint64_t>(p.B);
  const u32x4 rsA = {(uint32_t)aa, (uint32_t)(aa >> 32) & 0xFFFFu, (uint32_t)(((p.K - 1) * p.lda + p.M) * 2), 0x00020000u};
  const u32x4 rsB = {(uint32_t)ba, (uint32_t)(ba >> 32) & 0xFFFFu, (uint32_t)(((p.K - 1) * p.ldb + p.N) * 2), 0x00020000u};
  uint32_t voA[4], voB[4];
#pragma unroll
  for (int q = 0; q < 4; ++q) {
    const int kr = wave * 8 + q * 2 + (lane >> 5);             // k-row within the stage
    const int c = (lane & 31) ^ ((kr & 3) << 2);               // the piece this lane fetches
    voA[q] = (uint32_t)(((int64_t)kr * p.lda + m0 + c * 8) * 2);
    voB[q] = (uint32_t)(((int64_t)kr * p.ldb + n0 + c * 8) * 2);
  }
  const uint32_t lds0 = (uint32_t)reinterpret_cast<uintptr_t>(smem);
  const uint32_t stepA = (uint32_t)(TT_BK * p.lda * 2), stepB = (uint32_t)(TT_BK * p.ldb * 2);
  auto request = [&](int64_t st, int q) __attribute__((always_inline)) {  // q in 0..7: A pairs then B pairs
    const int64_t sc = st < nst ? st : nst - 1;                            // past the end: the last stage again
    const uint32_t dst = lds0 + (uint32_t)(st & (TT_STAGES - 1)) * TT_STG + (uint32_t)wave * 4096 + (q & 3) * 1024;
    if (q < 4) load_to_lds_b128(rsA, dst, voA[q], (uint32_t)sc * stepA);
    else load_to_lds_b128(rsB, dst + TT_OPB, voB[q & 3], (uint32_t)sc * stepB);
  };

  // ---- fragment addresses (k-step 0 of a stage; k-step 1 is 16 rows further)
  const int sl = lane & 15, fh = lane >> 5;
  int adA[MT][2], adB[NT][2];
#pragma unroll
  for (int i = 0; i < MT; ++i)
#pragma unroll
    for (int hh = 0; hh < 2; ++hh) {
      const int kr = 8 * fh + (sl >> 2) + 4 * hh;
      const int colA = wm * WM + i * 32 + 16 * ((lane >> 4) & 1) + 4 * (sl & 3);
      const int colB = wn * WN + i * 32 + 16 * ((lane >> 4) & 1) + 4 * (sl & 3);
      adA[i][hh] = kr * TT_ROWB + (((colA >> 3) ^ ((kr & 3) << 2)) * 16) + (colA & 7) * 2;
      adB[i][hh] = TT_OPB + kr * TT_ROWB + (((colB >> 3) ^ ((kr & 3) << 2)) * 16) + (colB & 7) * 2;
    }
  bf16x8 fa[2][MT], fb[2][NT];
  auto read_frag = [&](bf16x8& f, const unsigned char* base, const int (&ad)[2]) __attribute__((always_inline)) {
    const v4i16 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((v4i16 __attribute__((address_space(3)))*)(base + ad[0]));
    const v4i16 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((v4i16 __attribute__((address_space(3)))*)(base + ad[1]));
    const v8i16 both = {lo[0], lo[1], lo[2], lo[3], hi[0], hi[1], hi[2], hi[3]};
    f = __builtin_bit_cast(bf16x8, both);
  };

  // ---- prologue: three stages on their way, the first one landed
#pragma unroll
  for (int st = 0; st < TT_STAGES - 1; ++st)
#pragma unroll
    for (int q = 0; q < 8; ++q) request(st, q);
  asm volatile("s_waitcnt vmcnt(16)" ::: "memory");
  __syncthreads();
  {
    const unsigned char* cur = smem;
#pragma unroll
    for (int i = 0; i < MT; ++i) read_frag(fa[0][i], cur, adA[i]);
#pragma unroll
    for (int j = 0; j < NT; ++j) read_frag(fb[0][j], cur, adB[j]);
#pragma unroll
    for (int q = 0; q < 8; ++q) request(TT_STAGES - 1, q);
  }

  // ---- main loop.  At the top fa[0], fb[0] hold (or are about to receive) the fragments of the stage's first k-step.
  for (int64_t st = 0; st < nst; ++st) {
    const unsigned char* cur = smem + (st & (TT_STAGES - 1)) * TT_STG;
    const unsigned char* nxt = smem + ((st + 1) & (TT_STAGES - 1)) * TT_STG;
    // first k-step: one fragment of the second k-step is read after each of the first eight products
#pragma unroll
    for (int q = 0; q < MT * NT; ++q) {
      const int i = q / NT, j = q % NT;
      acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fb[0][j], fa[0][i], acc[i][j], 0, 0, 0);
      if (q < MT) read_frag(fa[1][q], cur + 16 * TT_ROWB, adA[q]);
      else if (q < MT + NT) read_frag(fb[1][q - MT], cur + 16 * TT_ROWB, adB[q - MT]);
      __builtin_amdgcn_sched_barrier(0);
    }
    // second k-step, first half
#pragma unroll
    for (int q = 0; q < MT * NT / 2; ++q) {
      const int i = q / NT, j = q % NT;
      acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fb[1][j], fa[1][i], acc[i][j], 0, 0, 0);
      __builtin_amdgcn_sched_barrier(0);
    }
    // The next stage is read from here on, and this stage's buffer is free once every wavefront is here: its own
    // requests for the next stage have landed when at most the 16 younger ones (two stages) are outstanding.
    asm volatile("s_waitcnt vmcnt(16)" ::: "memory");
    __syncthreads();
    __builtin_amdgcn_sched_barrier(0);
    // second half, with the first fragments of the next stage and the requests for the stage after the ring
#pragma unroll
    for (int q = MT * NT / 2; q < MT * NT; ++q) {
      const int i = q / NT, j = q % NT, r = q - MT * NT / 2;
      acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fb[1][j], fa[1][i], acc[i][j], 0, 0, 0);
      if (r < MT) read_frag(fa[0][r], nxt, adA[r]);
      else read_frag(fb[0][r - MT], nxt, adB[r - MT]);
      request(st + TT_STAGES, r);
      __builtin_amdgcn_sched_barrier(0);
    }
  }
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");  // stray requests must land before LDS is reused
  // epilogue shared with gemm_mfma_k (accumulator layout is the same: the B-side fragment is the first MFMA operand)
  store_tile<WM, WN, true, OutT>(p, acc, smem, m0, n0, wm, wn, wave, lane, 0, 0);
}

// ------------------------------------------------------------------------------------------
// plain FMA kernel: any strides, any element type, fp32 accumulation
// ------------------------------------------------------------------------------------------
template <typename T, typename OutT>
__global__ void __launch_bounds__(256) gemm_fma_k(GemmP p, int64_t sam, int64_t sak, int64_t sbn, int64_t sbk) {
  __shared__ float As[16][64 + 4];
  __shared__ float Bs[16][64 + 4];
  const int tid = threadIdx.x;
  const int tile = blockIdx.x;
  const int tm = tile % p.tiles_m, tn = tile / p.tiles_m;
  const int z = blockIdx.y, zb = z / p.nh, zh = z % p.nh;
  const T* A = reinterpret_cast<const T*>(p.A) + zb * p.sa1 + zh * p.sa2;
  const T* B = reinterpret_cast<const T*>(p.B) + zb * p.sb1 + zh * p.sb2;
  const int64_t m0 = (int64_t)tm * 64, n0 = (int64_t)tn * 64;
  const int tx = tid & 15, ty = tid >> 4;  // thread computes rows ty*4..+3, cols tx*4..+3
  float acc[4][4] = {};
  for (int64_t k0 = 0; k0 < p.K; k0 += 16) {
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int e = tid + 256 * i;
      int r, k;
      if (sak == 1) { k = e & 15; r = e >> 4; } else { r = e & 63; k = e >> 6; }
      const int64_t gm = m0 + r, gk = k0 + k;
      As[k][r] = (gm < p.M && gk < p.K) ? to_f32(A[gm * sam + gk * sak]) : 0.f;
      if (sbk == 1) { k = e & 15; r = e >> 4; } else { r = e & 63; k = e >> 6; }
      const int64_t gn = n0 + r, gk2 = k0 + k;
      Bs[k][r] = (gn < p.N && gk2 < p.K) ? to_f32(B[gn * sbn + gk2 * sbk]) : 0.f;
    }
    __syncthreads();
#pragma unroll
    for (int k = 0; k < 16; ++k) {
      float a[4], b[4];
#pragma unroll
      for (int i = 0; i < 4; ++i) { a[i] = As[k][ty * 4 + i]; b[i] = Bs[k][tx * 4 + i]; }
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) acc[i][j] = fmaf(a[i], b[j], acc[i][j]);
    }
    __syncthreads();
  }
  OutT* C = reinterpret_cast<OutT*>(p.C) + zb * p.sc1 + zh * p.sc2;
  const OutT* R = p.R ? reinterpret_cast<const OutT*>(p.R) + zb * p.sc1 + zh * p.sc2 : nullptr;
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int64_t row = m0 + ty * 4 + i;
    if (row >= p.M) continue;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const int64_t col = n0 + tx * 4 + j;
      if (col >= p.N) continue;
      float v = acc[i][j] + (p.bias ? to_f32(reinterpret_cast<const T*>(p.bias)[col]) : 0.f);
      if (R) v += to_f32(R[row * p.ldr + col]);
      C[row * p.ldc + col] = from_f32<OutT>(v);
    }
  }
}

template <int BM, int BN, bool AK, bool BKM, bool KTAIL, bool VEC, typename OutT>
hipError_t launch_mfma(GemmP& p, int nz, hipStream_t st) {
  constexpr int OPER = 2 * (BM + BN) * 128;                 // two buffers of both operand tiles
  constexpr int RP = BM / 2 < 64 ? BM / 2 : 64;
  constexpr int STAGE = 4 * RP * (BN / 2 * 4 + 16);         // fp32 epilogue staging, 4 waves
  constexpr int LDS = (VEC && STAGE > OPER) ? STAGE : OPER;
  static_assert(LDS <= 160 * 1024, "LDS of a gfx950 compute unit");
  static bool attr_done = false;  // one flag per instantiation
  auto kern = gemm_mfma_k<BM, BN, AK, BKM, KTAIL, VEC, OutT>;
  if (!attr_done) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, LDS);
    if (e != hipSuccess) return e;
    attr_done = true;
  }
  p.tiles_m = (int)((p.M + BM - 1) / BM);
  p.tiles_n = (int)((p.N + BN - 1) / BN);
  kern<<<dim3((unsigned)(p.tiles_m * p.tiles_n), (unsigned)nz), 256, LDS, st>>>(p);
  return hipGetLastError();
}

template <int BM, int BN, bool AK, bool BKM, typename OutT>
hipError_t launch_mfma_tail(GemmP& p, bool ktail, bool vec, int nz, hipStream_t st) {
  if (!ktail && vec) return launch_mfma<BM, BN, AK, BKM, false, true, OutT>(p, nz, st);
  if (!ktail) return launch_mfma<BM, BN, AK, BKM, false, false, OutT>(p, nz, st);
  return launch_mfma<BM, BN, AK, BKM, true, false, OutT>(p, nz, st);  // ragged k: rare, scalar epilogue
}

template <int BM, int BN, typename OutT>
hipError_t launch_mfma_layout(GemmP& p, bool ak, bool bk, bool ktail, bool vec, int nz, hipStream_t st) {
  if (ak && bk) return launch_mfma_tail<BM, BN, true, true, OutT>(p, ktail, vec, nz, st);
  if (ak && !bk) return launch_mfma_tail<BM, BN, true, false, OutT>(p, ktail, vec, nz, st);
  if (!ak && bk) return launch_mfma_tail<BM, BN, false, true, OutT>(p, ktail, vec, nz, st);
  return launch_mfma_tail<BM, BN, false, false, OutT>(p, ktail, vec, nz, st);
}

inline bool al16(const void* q) { return (reinterpret_cast<uintptr_t>(q) & 15) == 0; }

}  // namespace

// Size in bytes of the packed copy of a B operand with N rows and K columns (zero if the shape
// cannot be packed).
size_t packed_b_bytes(int64_t N, int64_t K) {
  if (N < 256 || K < 32 || K % 32 != 0) return 0;
  return (size_t)((N + 255) / 256) * 8 * (size_t)(K / 16) * 1024;
}

namespace {
template <typename SrcT>
hipError_t pack_b_from(const SrcT* Bs, int64_t ldb, int64_t N, int64_t K, bool b_kmajor, void* Bp, hipStream_t st, int order,
                       const void* gain) {
  const int64_t half = N / 64;  // 32-row blocks in half of B
  const int64_t n_blocks = ((N + 255) / 256) * 8, k_steps = K / 16;
  const bf16* gn = reinterpret_cast<const bf16*>(gain);
  u32x4* out = reinterpret_cast<u32x4*>(Bp);
  constexpr int PER16 = 16 / (int)sizeof(SrcT);  // source values per 16 bytes
  const bool src_ok = (reinterpret_cast<uintptr_t>(Bs) & 15) == 0 && ldb % PER16 == 0 && ldb % 8 == 0;
  if (src_ok && (!gain || (al16(gain) && K % 8 == 0))) {
    if (b_kmajor) {
      const int ti = (int)((K + 255) / 256);
      pack_b_tile_k<true, SrcT><<<dim3((unsigned)(n_blocks * ti)), 256, 0, st>>>(Bs, ldb, N, K, out, k_steps, ti, order, half, gn);
    } else {
      const int ti = (int)(n_blocks / 8);
      pack_b_tile_k<false, SrcT><<<dim3((unsigned)((K / 32) * ti)), 256, 0, st>>>(Bs, ldb, N, K, out, k_steps, ti, order, half, gn);
    }
  } else {
    const int64_t blocks = n_blocks * k_steps;
    pack_b_k<SrcT><<<dim3((unsigned)((blocks + 3) / 4)), 256, 0, st>>>(Bs, ldb, N, K, b_kmajor, out, n_blocks, k_steps, order, half, gn);
  }
  return hipGetLastError();
}
}  // namespace

hipError_t pack_b(const void* B, int64_t ldb, int64_t N, int64_t K, bool b_kmajor, void* Bp, hipStream_t st, int order,
                  const void* gain, bool src_f32) {
  if (packed_b_bytes(N, K) == 0) return hipErrorInvalidValue;
  if (order == PK_ORDER_HALVES ? N % 256 != 0 : order == PK_ORDER_PAIR64 ? N % 128 != 0 : order != PK_ORDER_PLAIN)
    return hipErrorInvalidValue;
  if (src_f32) return pack_b_from(reinterpret_cast<const float*>(B), ldb, N, K, b_kmajor, Bp, st, order, gain);
  return pack_b_from(reinterpret_cast<const bf16*>(B), ldb, N, K, b_kmajor, Bp, st, order, gain);
}

constexpr int PK_MT = 4;  // 128 x 256 tiles

bool packed_gemm_applies(const Gemm& g, bool any_tile_count) {
  if (g.dtype != DT_BF16 || !g.a_kmajor || g.nb * g.nh != 1 || packed_b_bytes(g.N, g.K) == 0) return false;
  const bool vec = g.N % 8 == 0 && g.ldc % 8 == 0 && al16(g.C) && (!g.R || (g.ldr % 8 == 0 && al16(g.R))) &&
                   (!g.bias || al16(g.bias));
  // 32-bit byte offsets, also for the rows past the edge of the last tile and the stages requested past K
  const bool fits = (g.M + 256) * g.lda * 2 < (int64_t(1) << 32) && al16(g.A) && g.lda % 8 == 0 &&
                    packed_b_bytes(g.N, g.K) < (size_t(1) << 32);
  if (!(vec && fits)) return false;
  // enough tiles to fill the chip -- unless the caller has no other kernel to go to (no row-major copy of the weight)
  return any_tile_count || ((g.M + 32 * PK_MT - 1) / (32 * PK_MT)) * ((g.N + 255) / 256) >= 200;
}

namespace {
// Launch of a packed-operand kernel with its dynamic LDS size enabled once per kernel.
template <auto Kern>
hipError_t launch_pk(dim3 grid, int threads, int lds, hipStream_t st, const GemmP& p, const u32x4* bp) {
  static bool attr_done = false;
  if (!attr_done) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(Kern), hipFuncAttributeMaxDynamicSharedMemorySize, lds);
    if (e != hipSuccess) return e;
    attr_done = true;
  }
  Kern<<<grid, threads, lds, st>>>(p, bp, p.K / 16);
  return hipGetLastError();
}

}  // namespace

// How many workgroups share each tile of the last round of a problem of `blocks` tiles (1: the round is not shared):
// 2 to 4 when at most half the compute units would have a tile, every share at least 8 stages of K long.
static int shared_round_split(int blocks, int64_t K) {
  const int rem = blocks % 256;
  if (rem == 0 || rem > 128 || K % PK_DK != 0) return 1;
  int split = 256 / rem;
  if (split > 4) split = 4;
  while (split > 1 && K / PK_DK < 8 * split) --split;
  return split;
}

size_t packed_ws_needed(const Gemm& g) {
  const int blocks = (int)((g.M + 32 * PK_MT - 1) / (32 * PK_MT)) * (int)((g.N + 255) / 256);
  const int split = shared_round_split(blocks, g.K);
  return split > 1 ? 1024 + (size_t)split * (blocks % 256) * (32 * PK_MT * 256 * 4) : 0;
}

hipError_t gemm_packed(const Gemm& g, const void* Bp, hipStream_t st) {
  if (!packed_gemm_applies(g, true)) return hipErrorInvalidValue;
  GemmP p;
  p.M = g.M; p.N = g.N; p.K = g.K;
  p.A = g.A; p.lda = g.lda; p.B = nullptr; p.ldb = 0; p.C = g.C; p.ldc = g.ldc;
  p.bias = g.bias; p.R = g.R; p.ldr = g.ldr;
  p.nh = 1; p.sa1 = p.sa2 = p.sb1 = p.sb2 = p.sc1 = p.sc2 = 0;
  if (g.epi != EPI_NONE) {
    // the fused epilogues write bf16 rows in 16-byte pieces and take neither bias (but for EPI_GELU) nor residual
    if (g.out_f32 || (g.bias && g.epi != EPI_GELU) || g.R) return hipErrorInvalidValue;
    if (g.epi == EPI_SWIGLU) {
      if (g.N % 256 != 0 || !g.C2 || !al16(g.C2) || g.ldc2 % 8 != 0 || g.ldc2 < g.N / 2) return hipErrorInvalidValue;
    } else if (g.epi == EPI_ROPE) {
      if (g.N % 256 != 0 || !g.C || !g.cos_sin || g.S < 1 || g.rot_cols % 128 != 0 || g.rot_cols > g.N ||
          (reinterpret_cast<uintptr_t>(g.cos_sin) & 7) != 0)
        return hipErrorInvalidValue;
    } else if (g.epi == EPI_SWIGLU_BWD) {
      if (g.N % 8 != 0 || !g.C || !g.C2 || !al16(g.C2) || g.ldc2 % 8 != 0 || g.ldc2 < 2 * g.N || g.ldc < 2 * g.N)
        return hipErrorInvalidValue;
    } else if (g.epi == EPI_GELU || g.epi == EPI_GELU_BWD) {
      if (g.N % 8 != 0 || !g.C2 || !al16(g.C2) || g.ldc2 % 8 != 0 || g.ldc2 < g.N || (g.epi == EPI_GELU_BWD && !g.C))
        return hipErrorInvalidValue;
    } else {
      return hipErrorInvalidValue;
    }
    p.C2 = g.C2; p.ldc2 = g.ldc2;
    p.cos_sin = reinterpret_cast<const float2*>(g.cos_sin); p.S = g.S > 0 ? g.S : 1; p.rot_cols = g.rot_cols;
  }
  if (g.rowsq_out) {  // one partial per row and 64-column strip: bf16 rows, plain epilogue, whole strips
    if (g.out_f32 || g.epi != EPI_NONE || g.N % 256 != 0) return hipErrorInvalidValue;
    p.rowsq_out = g.rowsq_out;
  }
  if (g.rowsq) {  // K / 64 partials per row, read in 16-byte pieces by two threads per row
    if ((g.epi != EPI_SWIGLU && g.epi != EPI_ROPE) || g.K % 512 != 0 || g.K > 512 * PK_SQ_MAX || !al16(g.rowsq))
      return hipErrorInvalidValue;
    p.rowsq = g.rowsq; p.rowsq_n = (int)(g.K / 64); p.norm_eps = g.norm_eps; p.norm_stats = g.norm_stats;
  }
  const u32x4* bp = reinterpret_cast<const u32x4*>(Bp);
  p.tiles_n = (int)((p.N + 255) / 256);
  constexpr int LDS = PK_STAGES * 32 * PK_MT * PK_ROW;  // ring of A stages
  static_assert(LDS <= 160 * 1024, "LDS of a gfx950 compute unit");
  p.tiles_m = (int)((p.M + 32 * PK_MT - 1) / (32 * PK_MT));
  // The last round: if at most half the compute units would have a tile and the caller gave a work space,
  // 2 to 4 workgroups share each
  int blocks = p.tiles_m * p.tiles_n;
  const int rem = blocks % 256;
  if (g.ws && (reinterpret_cast<uintptr_t>(g.ws) & 15) == 0) {
    const int split = shared_round_split(blocks, g.K);
    if (split > 1) {
      p.split = split;
      p.split_from = blocks - rem;
      p.ws = reinterpret_cast<unsigned char*>(g.ws);
      blocks = p.split_from + rem * split;
    }
  }
  const dim3 grid((unsigned)blocks);
  if (g.out_f32) return launch_pk<gemm_pk_k<PK_MT, true, float>>(grid, 256, LDS, st, p, bp);
  if (g.epi == EPI_SWIGLU) return launch_pk<gemm_pk_k<PK_MT, true, bf16, EPI_SWIGLU>>(grid, 256, LDS, st, p, bp);
  if (g.epi == EPI_ROPE) return launch_pk<gemm_pk_k<PK_MT, true, bf16, EPI_ROPE>>(grid, 256, LDS, st, p, bp);
  if (g.epi == EPI_SWIGLU_BWD) return launch_pk<gemm_pk_k<PK_MT, true, bf16, EPI_SWIGLU_BWD>>(grid, 256, LDS, st, p, bp);
  if (g.epi == EPI_GELU) return launch_pk<gemm_pk_k<PK_MT, true, bf16, EPI_GELU>>(grid, 256, LDS, st, p, bp);
  if (g.epi == EPI_GELU_BWD) return launch_pk<gemm_pk_k<PK_MT, true, bf16, EPI_GELU_BWD>>(grid, 256, LDS, st, p, bp);
  return launch_pk<gemm_pk_k<PK_MT, true, bf16>>(grid, 256, LDS, st, p, bp);
}

hipError_t gemm(const Gemm& g, hipStream_t st, int* variant) {
  if (variant) *variant = 0;
  if (g.M <= 0 || g.N <= 0 || g.nb <= 0 || g.nh <= 0) return hipSuccess;
  GemmP p;
  p.M = g.M; p.N = g.N; p.K = g.K;
  p.A = g.A; p.lda = g.lda; p.B = g.B; p.ldb = g.ldb; p.C = g.C; p.ldc = g.ldc;
  p.bias = g.bias; p.R = g.R; p.ldr = g.ldr;
  p.nh = g.nh; p.sa1 = g.sa1; p.sa2 = g.sa2; p.sb1 = g.sb1; p.sb2 = g.sb2; p.sc1 = g.sc1; p.sc2 = g.sc2;
  p.band = g.band;  // only the MFMA kernel uses it; the FMA kernel computes everything, which is also correct
  const int nz = g.nb * g.nh;
  if (nz > 65535) return hipErrorInvalidValue;

  if (g.dtype == DT_BF16) {
    // the MFMA path moves 16-byte pieces: 8 bf16 along the contiguous direction of each operand
    const bool a_ok = al16(g.A) && g.lda % 8 == 0 && g.sa1 % 8 == 0 && g.sa2 % 8 == 0 &&
                      (g.a_kmajor ? g.K % 8 == 0 : g.M % 8 == 0);
    const bool b_ok = al16(g.B) && g.ldb % 8 == 0 && g.sb1 % 8 == 0 && g.sb2 % 8 == 0 &&
                      (g.b_kmajor ? g.K % 8 == 0 : g.N % 8 == 0);
    // operands are addressed with 32-bit byte offsets from the (batch-adjusted) base
    const int64_t ext_a = (g.a_kmajor ? g.M * g.lda : g.K * g.lda) * 2, ext_b = (g.b_kmajor ? g.N * g.ldb : g.K * g.ldb) * 2;
    const bool fits = ext_a < (int64_t(1) << 32) && ext_b < (int64_t(1) << 32) &&
                      (g.a_kmajor || g.M >= 8) && (g.b_kmajor || g.N >= 8) && g.K >= 8;
    if (a_ok && b_ok && fits && !g.a_kmajor && !g.b_kmajor && nz == 1 && g.band == BAND_NONE && g.M % 256 == 0 &&
        g.N % 256 == 0 && g.K % TT_BK == 0 && (g.M / 256) * (g.N / 256) >= 128 && g.N % 8 == 0 && g.ldc % 8 == 0 &&
        al16(g.C) && (!g.R || (g.ldr % 8 == 0 && al16(g.R))) && (!g.bias || al16(g.bias))) {
      // both operands contraction-index first (the weight gradient): direct-to-LDS loads and transposing LDS reads
      constexpr int LDS_TT = TT_STAGES * TT_STG > 4 * 64 * (128 * 4 + 16) ? TT_STAGES * TT_STG : 4 * 64 * (128 * 4 + 16);
      static_assert(LDS_TT <= 160 * 1024, "LDS of a gfx950 compute unit");
      p.tiles_m = (int)(g.M / 256);
      p.tiles_n = (int)(g.N / 256);
      if (variant) *variant = 3;
      static bool attr_f = false, attr_h = false;
      if (g.out_f32) {
        if (!attr_f) {
          hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(gemm_tt_k<float>), hipFuncAttributeMaxDynamicSharedMemorySize, LDS_TT);
          if (e != hipSuccess) return e;
          attr_f = true;
        }
        gemm_tt_k<float><<<dim3((unsigned)(p.tiles_m * p.tiles_n)), 256, LDS_TT, st>>>(p);
      } else {
        if (!attr_h) {
          hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(gemm_tt_k<bf16>), hipFuncAttributeMaxDynamicSharedMemorySize, LDS_TT);
          if (e != hipSuccess) return e;
          attr_h = true;
        }
        gemm_tt_k<bf16><<<dim3((unsigned)(p.tiles_m * p.tiles_n)), 256, LDS_TT, st>>>(p);
      }
      return hipGetLastError();
    }
    if (a_ok && b_ok && fits) {
      const bool ktail = g.K % KT != 0;
      const int64_t t256 = ((g.M + 255) / 256) * ((g.N + 255) / 256) * (int64_t)nz;
      const bool big = g.M >= 256 && g.N >= 256 && t256 >= 200;
      const bool vec = g.N % 8 == 0 && g.ldc % 8 == 0 && al16(g.C) && (!g.R || (g.ldr % 8 == 0 && al16(g.R))) &&
                       g.sc1 % 8 == 0 && g.sc2 % 8 == 0 && (!g.bias || al16(g.bias));
      if (variant) *variant = big ? 2 : 1;
      if (g.out_f32) {
        if (big) return launch_mfma_layout<256, 256, float>(p, g.a_kmajor, g.b_kmajor, ktail, vec, nz, st);
        return launch_mfma_layout<128, 128, float>(p, g.a_kmajor, g.b_kmajor, ktail, vec, nz, st);
      }
      if (big) return launch_mfma_layout<256, 256, bf16>(p, g.a_kmajor, g.b_kmajor, ktail, vec, nz, st);
      return launch_mfma_layout<128, 128, bf16>(p, g.a_kmajor, g.b_kmajor, ktail, vec, nz, st);
    }
  }
  p.tiles_m = (int)((g.M + 63) / 64);
  p.tiles_n = (int)((g.N + 63) / 64);
  const dim3 grid((unsigned)(p.tiles_m * p.tiles_n), (unsigned)nz);
  const int64_t sam = g.a_kmajor ? g.lda : 1, sak = g.a_kmajor ? 1 : g.lda;
  const int64_t sbn = g.b_kmajor ? g.ldb : 1, sbk = g.b_kmajor ? 1 : g.ldb;
  if (g.dtype == DT_F32)
    gemm_fma_k<float, float><<<grid, 256, 0, st>>>(p, sam, sak, sbn, sbk);
  else if (g.out_f32)
    gemm_fma_k<bf16, float><<<grid, 256, 0, st>>>(p, sam, sak, sbn, sbk);
  else
    gemm_fma_k<bf16, bf16><<<grid, 256, 0, st>>>(p, sam, sak, sbn, sbk);
  return hipGetLastError();
}

}  // namespace hift
