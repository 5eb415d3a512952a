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
//   * fp32 and odd shapes: a plain 64x64x16 LDS-tiled FMA kernel with arbitrary strides.
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
};

// ------------------------------------------------------------------------------------------
// bf16 MFMA kernel
// ------------------------------------------------------------------------------------------
constexpr int KT = 64;  // k extent of a macro-tile

// 16-byte chunk c of LDS row r lives at chunk position c ^ f(r), f(r) = (r & 7) ^ ((r >> 3) & 3).
// f depends on r mod 32 only, so rows 32 apart differ by a constant byte offset and the
// addresses of all MFMA fragments of a lane are one register plus immediates.
__device__ __forceinline__ int swz_f(int row) { return (row & 7) ^ ((row >> 3) & 3); }
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
      unsigned char* dst = lds + row * 128 + swz(row, tid & 7) * 16;
#pragma unroll
      for (int i = 0; i < NPIECE; ++i) *reinterpret_cast<u32x4*>(dst + i * 4096) = r[i];
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

__device__ __forceinline__ uint32_t pack_bf16x2(float a, float b) {
  typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
  bf16x2 v = {static_cast<__bf16>(a), static_cast<__bf16>(b)};
  return *reinterpret_cast<uint32_t*>(&v);
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
  u32x4 ra[StA::NPIECE], rb[StB::NPIECE];  // the next tile on its way from HBM to LDS

  sa.load(0, ra);
  sb.load(0, rb);
  sa.store(smem, tid, ra);
  sb.store(smem + A_BYTES, tid, rb);
  __syncthreads();

  const int frow = lane & 31, fhalf = lane >> 5;
  bf16x8 fa[2][MT], fb[2][NT];
  // byte offset of this lane's fragment chunk for each k-step; rows 32 apart add 4096 bytes
  int foff[KT / 16];
#pragma unroll
  for (int ks = 0; ks < KT / 16; ++ks) foff[ks] = frow * 128 + swz(frow, ks * 2 + fhalf) * 16;
  const int a_base = wm * WM * 128, b_base = A_BYTES + wn * WN * 128;
  auto read_frags = [&](bf16x8(&a)[MT], bf16x8(&b)[NT], const unsigned char* buf, int ks) __attribute__((always_inline)) {
#pragma unroll
    for (int i = 0; i < MT; ++i) a[i] = *reinterpret_cast<const bf16x8*>(buf + foff[ks] + (a_base + i * 4096));
#pragma unroll
    for (int j = 0; j < NT; ++j) b[j] = *reinterpret_cast<const bf16x8*>(buf + foff[ks] + (b_base + j * 4096));
  };
  read_frags(fa[0], fb[0], smem, 0);

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
  for (int64_t kt = 0; kt < nk; ++kt) {
    unsigned char* cur = smem + (kt & 1) * BUF;
    unsigned char* nxt = smem + ((kt + 1) & 1) * BUF;
    const int64_t kt2 = kt + 1 < nk ? kt + 1 : nk - 1;
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

  // ---- epilogue ----
  const int z_c = zb * 0;  // (batch offsets below)
  (void)z_c;
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

hipError_t gemm(const Gemm& g, hipStream_t st, int* variant) {
  if (variant) *variant = 0;
  if (g.M <= 0 || g.N <= 0 || g.nb <= 0 || g.nh <= 0) return hipSuccess;
  GemmP p;
  p.M = g.M; p.N = g.N; p.K = g.K;
  p.A = g.A; p.lda = g.lda; p.B = g.B; p.ldb = g.ldb; p.C = g.C; p.ldc = g.ldc;
  p.bias = g.bias; p.R = g.R; p.ldr = g.ldr;
  p.nh = g.nh; p.sa1 = g.sa1; p.sa2 = g.sa2; p.sb1 = g.sb1; p.sb2 = g.sb2; p.sc1 = g.sc1; p.sc2 = g.sc2;
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
