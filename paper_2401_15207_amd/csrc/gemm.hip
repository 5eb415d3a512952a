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

__device__ __forceinline__ int swz(int row, int chunk) { return chunk ^ ((row ^ (row >> 3)) & 7); }

// Stage registers of one operand tile: ROWS x 64 bf16, 16-byte pieces.
// k-major source: thread t owns chunk (t % 8) of rows t/8 + 32 i.
// transposed source: thread t owns 8x8 blocks; block b = t + 256 i covers rows 8 (b % (ROWS/8))..+7
// and k-chunk b / (ROWS/8), loaded as 8 rows of the [K][rows] source.
template <int ROWS, bool KMAJOR>
struct Stage {
  static constexpr int NPIECE = KMAJOR ? ROWS / 32 : (ROWS >= 256 ? ROWS / 256 * 8 : 8);
  uint4 r[NPIECE];

  __device__ __forceinline__ void load(const bf16* __restrict__ src, int64_t ld, int64_t row0, int64_t nrows,
                                       int64_t k0, int64_t K, int tid) {
    if (KMAJOR) {
      const int c = tid & 7;
#pragma unroll
      for (int i = 0; i < ROWS / 32; ++i) {
        const int64_t row = row0 + (tid >> 3) + 32 * i, k = k0 + c * 8;
        if (row < nrows && k < K)
          r[i] = *reinterpret_cast<const uint4*>(src + row * ld + k);
        else
          r[i] = make_uint4(0, 0, 0, 0);
      }
    } else {
      constexpr int RB = ROWS / 8;  // row blocks
#pragma unroll
      for (int i = 0; i < NPIECE / 8; ++i) {
        const int b = tid + 256 * i;
        const bool live = b < ROWS;   // ROWS/8 * 8 blocks in total
        const int64_t row = row0 + (int64_t)(b % RB) * 8;
        const int64_t k = k0 + (int64_t)(b / RB) * 8;
#pragma unroll
        for (int j = 0; j < 8; ++j) {
          if (live && row < nrows && k + j < K)
            r[i * 8 + j] = *reinterpret_cast<const uint4*>(src + (k + j) * ld + row);
          else
            r[i * 8 + j] = make_uint4(0, 0, 0, 0);
        }
      }
    }
  }

  __device__ __forceinline__ void store(unsigned char* lds, int tid) const {
    if (KMAJOR) {
      const int c = tid & 7;
#pragma unroll
      for (int i = 0; i < ROWS / 32; ++i) {
        const int row = (tid >> 3) + 32 * i;
        *reinterpret_cast<uint4*>(lds + row * 128 + swz(row, c) * 16) = r[i];
      }
    } else {
      constexpr int RB = ROWS / 8;
#pragma unroll
      for (int i = 0; i < NPIECE / 8; ++i) {
        const int b = tid + 256 * i;
        if (b >= ROWS) continue;
        const int rowb = (b % RB) * 8, c = b / RB;
        // r[i*8 + j] holds, for k = j, the 8 rows rowb..rowb+7 (two per dword).  Turn the 8x8
        // block around: output row m gets k = 0..7.
        const uint32_t* in = reinterpret_cast<const uint32_t*>(&r[i * 8]);  // in[j*4 + q]: k=j, rows 2q,2q+1
#pragma unroll
        for (int m = 0; m < 8; ++m) {
          uint4 o;
          uint32_t* ow = reinterpret_cast<uint32_t*>(&o);
#pragma unroll
          for (int q = 0; q < 4; ++q) {
            const uint32_t lo = in[(2 * q) * 4 + (m >> 1)], hi = in[(2 * q + 1) * 4 + (m >> 1)];
            ow[q] = (m & 1) ? __builtin_amdgcn_perm(hi, lo, 0x07060302u) : __builtin_amdgcn_perm(hi, lo, 0x05040100u);
          }
          const int row = rowb + m;
          *reinterpret_cast<uint4*>(lds + row * 128 + swz(row, c) * 16) = o;
        }
      }
    }
  }
};

template <int BM, int BN, bool AK, bool BKM, typename OutT>
__global__ void __launch_bounds__(256) gemm_mfma_k(GemmP p) {
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  constexpr int WM = BM / 2, WN = BN / 2, MT = WM / 32, NT = WN / 32;
  constexpr int A_BYTES = BM * 128, B_BYTES = BN * 128, BUF = A_BYTES + B_BYTES;

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave >> 1, wn = wave & 1;
  const int tile = blockIdx.x;
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

  Stage<BM, AK> sa;
  Stage<BN, BKM> sb;
  const int64_t nk = (p.K + KT - 1) / KT;

  sa.load(A, p.lda, m0, p.M, 0, p.K, tid);
  sb.load(B, p.ldb, n0, p.N, 0, p.K, tid);
  sa.store(smem, tid);
  sb.store(smem + A_BYTES, tid);
  __syncthreads();

  const int frow = lane & 31, fhalf = lane >> 5;
  for (int64_t kt = 0; kt < nk; ++kt) {
    unsigned char* cur = smem + (kt & 1) * BUF;
    unsigned char* nxt = smem + ((kt + 1) & 1) * BUF;
    const bool more = kt + 1 < nk;
    if (more) {
      sa.load(A, p.lda, m0, p.M, (kt + 1) * KT, p.K, tid);
      sb.load(B, p.ldb, n0, p.N, (kt + 1) * KT, p.K, tid);
    }
#pragma unroll
    for (int ks = 0; ks < KT / 16; ++ks) {
      bf16x8 af[MT], bfr[NT];
#pragma unroll
      for (int i = 0; i < MT; ++i) {
        const int row = wm * WM + i * 32 + frow;
        af[i] = *reinterpret_cast<const bf16x8*>(cur + row * 128 + swz(row, ks * 2 + fhalf) * 16);
      }
#pragma unroll
      for (int j = 0; j < NT; ++j) {
        const int row = wn * WN + j * 32 + frow;
        bfr[j] = *reinterpret_cast<const bf16x8*>(cur + A_BYTES + row * 128 + swz(row, ks * 2 + fhalf) * 16);
      }
#pragma unroll
      for (int i = 0; i < MT; ++i)
#pragma unroll
        for (int j = 0; j < NT; ++j)
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[i], bfr[j], acc[i][j], 0, 0, 0);
    }
    if (more) {
      sa.store(nxt, tid);
      sb.store(nxt + A_BYTES, tid);
    }
    __syncthreads();
  }

  // epilogue: accumulator element e of lane l is row 8*(e/4) + 4*(l/32) + e%4, column l%32
  OutT* C = reinterpret_cast<OutT*>(p.C) + zb * p.sc1 + zh * p.sc2;
  const OutT* R = p.R ? reinterpret_cast<const OutT*>(p.R) + zb * p.sc1 + zh * p.sc2 : nullptr;
#pragma unroll
  for (int i = 0; i < MT; ++i)
#pragma unroll
    for (int j = 0; j < NT; ++j) {
      const int64_t col = n0 + wn * WN + j * 32 + frow;
      if (col >= p.N) continue;
      const float bias = p.bias ? to_f32(reinterpret_cast<const bf16*>(p.bias)[col]) : 0.f;
#pragma unroll
      for (int e = 0; e < 16; ++e) {
        const int64_t row = m0 + wm * WM + i * 32 + 8 * (e >> 2) + 4 * fhalf + (e & 3);
        if (row >= p.M) continue;
        float v = acc[i][j][e] + bias;
        if (R) v += to_f32(R[row * p.ldr + col]);
        C[row * p.ldc + col] = from_f32<OutT>(v);
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

template <int BM, int BN, bool AK, bool BKM, typename OutT>
hipError_t launch_mfma(GemmP& p, int nz, hipStream_t st) {
  constexpr int LDS = 2 * (BM + BN) * 128;
  static bool attr_done = false;  // one flag per instantiation
  auto kern = gemm_mfma_k<BM, BN, AK, BKM, OutT>;
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

template <int BM, int BN, typename OutT>
hipError_t launch_mfma_layout(GemmP& p, bool ak, bool bk, int nz, hipStream_t st) {
  if (ak && bk) return launch_mfma<BM, BN, true, true, OutT>(p, nz, st);
  if (ak && !bk) return launch_mfma<BM, BN, true, false, OutT>(p, nz, st);
  if (!ak && bk) return launch_mfma<BM, BN, false, true, OutT>(p, nz, st);
  return launch_mfma<BM, BN, false, false, OutT>(p, nz, st);
}

inline bool al16(const void* q) { return (reinterpret_cast<uintptr_t>(q) & 15) == 0; }

}  // namespace

hipError_t gemm(const Gemm& g, hipStream_t st) {
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
    if (a_ok && b_ok && g.K > 0) {
      const bool big = g.M >= 256 && g.N >= 256 &&
                       ((g.M + 255) / 256) * ((g.N + 255) / 256) * (int64_t)nz >= 128;
      if (g.out_f32) {
        if (big) return launch_mfma_layout<256, 256, float>(p, g.a_kmajor, g.b_kmajor, nz, st);
        return launch_mfma_layout<128, 128, float>(p, g.a_kmajor, g.b_kmajor, nz, st);
      }
      if (big) return launch_mfma_layout<256, 256, bf16>(p, g.a_kmajor, g.b_kmajor, nz, st);
      return launch_mfma_layout<128, 128, bf16>(p, g.a_kmajor, g.b_kmajor, nz, st);
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
