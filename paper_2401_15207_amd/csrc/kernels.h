// Host-side launchers of the HIP kernels of the HiFT step (gfx950).  Internal interface
// between the model code and the kernel sources; the public C ABI is include/hift.h.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace hift {

enum { DT_F32 = 0, DT_BF16 = 1 };
inline size_t dt_size(int dt) { return dt == DT_F32 ? 4 : 2; }

// ---- contraction -------------------------------------------------------------------------
struct Gemm {
  int dtype = DT_BF16;      // element type of A, B, R and (unless out_f32) C
  bool a_kmajor = true;     // A(m,k) at A[m*lda + k]; false: at A[k*lda + m]
  bool b_kmajor = true;     // B(n,k) at B[n*ldb + k]; false: at B[k*ldb + n]
  bool out_f32 = false;
  int64_t M = 0, N = 0, K = 0;
  const void* A = nullptr; int64_t lda = 0;
  const void* B = nullptr; int64_t ldb = 0;
  void* C = nullptr; int64_t ldc = 0;
  const void* bias = nullptr;           // [N], element type of A, or null
  const void* R = nullptr; int64_t ldr = 0;  // residual added in the epilogue, C's type, or null
  // two-level batch: problem z = b * nh + h uses offsets b*s?1 + h*s?2 (elements)
  int nb = 1, nh = 1;
  int64_t sa1 = 0, sa2 = 0, sb1 = 0, sb2 = 0, sc1 = 0, sc2 = 0;
  // Structure the caller vouches for (causal attention), used only to skip work that cannot matter:
  //   BAND_SKIP_UPPER   C(m,n) with n > m is never read: tiles wholly above the diagonal are not computed
  //                     (their part of C keeps whatever it held)
  //   BAND_K_UPTO_ROW   A(m,k) = 0 for k > m: the contraction of a tile stops at its last row
  //   BAND_K_FROM_ROW   A(m,k) = 0 for k < m: the contraction of a tile starts at its first row
  int band = 0;
  // Fused epilogue of the packed-operand kernel (gemm_packed only; the packed copy must have been built
  // with the matching column order, see pack_b):
  //   EPI_SWIGLU  B = gate | up, N = 2 f.  C [M, N] (may be null: not kept) receives the pre-activations as
  //               usual; C2 [M, f] (ldc2) receives silu(gate) * up computed from the rounded pre-activations.
  //   EPI_ROPE    B = q | k | v of heads of width 128.  Columns below rot_cols are rotated pairwise
  //               (i, i + 64 within a head) by the angle of position (row % S) before the one rounding;
  //               cos_sin: [>= S, 64] pairs (cos, sin), fp32.
  //   EPI_SWIGLU_BWD  (plain block order) the product is d act [M, N]; C2 holds the forward's pre-activations
  //               gate | up [M, 2 N] (ldc2, read only); C [M, 2 N] (ldc) receives d gate | d up.  d act is not stored.
  //   EPI_GELU    (plain block order; bias allowed) C [M, N] (may be null: not kept) receives the pre-activations
  //               A . B^T + bias; C2 [M, N] (ldc2) receives gelu of the rounded pre-activations (erf form; erf by a
  //               formula with absolute error below 1.5e-7).
  //   EPI_GELU_BWD  (plain block order) the product is d act [M, N]; C2 holds the forward's pre-activations [M, N]
  //               (ldc2, read only); C [M, N] receives d act * gelu'(pre).  d act is not stored.
  int epi = 0;
  void* C2 = nullptr; int64_t ldc2 = 0;
  const void* cos_sin = nullptr; int S = 0; int64_t rot_cols = 0;
  // Work space of the packed-operand kernel (gemm_packed only; optional): PACKED_WS_BYTES of device memory,
  // zero before its first use and left zero-counted by every launch.  With it, the tiles of a last, partial
  // round over the 256 compute units are shared by 2 to 4 workgroups each, every one taking a share of the
  // k range; launches that use the same work space must not overlap.
  void* ws = nullptr;
  // Row normalisation without a kernel of its own (gemm_packed only).  y = (x / rms(x)) gain . W^T is computed
  // as rstd(x) (x . (W gain)^T): the packed copy is built with the gain (pack_b), and
  //   rowsq_out  (plain epilogue, bf16 C, N a multiple of 256) the kernel that writes the rows x also leaves
  //              the sums of squares of the values it stored, [M, N / 64]: one partial per row and 64-column strip;
  //   rowsq      (EPI_ROPE and EPI_SWIGLU, K a multiple of 512 up to 6144) the consumer adds a row's K / 64 partials up,
  //              multiplies its accumulators by rstd = 1 / sqrt(sum / K + norm_eps) before anything else, and, if
  //              norm_stats is given, leaves (0, rstd) per row there, as the RMS normalisation kernel does.
  float* rowsq_out = nullptr;
  const float* rowsq = nullptr; float norm_eps = 0.f; float* norm_stats = nullptr;
};
constexpr size_t PACKED_WS_BYTES = 1024 + size_t(256) * 128 * 256 * 4;
enum { EPI_NONE = 0, EPI_SWIGLU = 1, EPI_ROPE = 2, EPI_SWIGLU_BWD = 3, EPI_GELU = 4, EPI_GELU_BWD = 5 };
enum { BAND_NONE = 0, BAND_SKIP_UPPER = 1, BAND_K_UPTO_ROW = 2, BAND_K_FROM_ROW = 3 };
// variant (optional) receives which kernel ran: 0 plain FMA, 1 MFMA 128x128 tiles, 2 MFMA 256x256 tiles
hipError_t gemm(const Gemm& g, hipStream_t st, int* variant = nullptr);

// Weight operand pre-packed in MFMA fragment order (see gemm.hip).  packed_b_bytes: size of the packed
// copy of a [N, K] operand, 0 if the shape cannot be packed.  pack_b: builds it from B given as in Gemm
// (b_kmajor or transposed).  gemm_packed: C = A . B^T with A k-major and B packed; only for problems
// packed_gemm_applies() accepts (g.B / g.ldb are ignored).
// The packed copy may hold the 32-row blocks of B in another order, so that the two blocks a wavefront
// multiplies side by side are the ones a fused epilogue combines element by element:
//   PK_ORDER_HALVES  block i of the first half of B next to block i of the second half (EPI_SWIGLU;
//                    N / 2 must be a multiple of 128)
//   PK_ORDER_PAIR64  within every four blocks the middle two exchanged: a block next to the one 64
//                    rows further (EPI_ROPE; N must be a multiple of 128)
enum { PK_ORDER_PLAIN = 0, PK_ORDER_HALVES = 1, PK_ORDER_PAIR64 = 2 };
size_t packed_b_bytes(int64_t N, int64_t K);
// gain (optional, bf16 [K]): the copy holds B[n][k] gain[k], each product rounded once.
// src_f32: B holds fp32 values (the master weights); each is rounded to bf16 (nearest even) first, which is by
// definition the value of the bf16 model, so the copy is the same as from a bf16 source.
hipError_t pack_b(const void* B, int64_t ldb, int64_t N, int64_t K, bool b_kmajor, void* Bp, hipStream_t st,
                  int order = PK_ORDER_PLAIN, const void* gain = nullptr, bool src_f32 = false);
// any_tile_count: also problems with too few tiles to fill the chip (for weights that have no row-major copy to fall back on)
bool packed_gemm_applies(const Gemm& g, bool any_tile_count = false);
hipError_t gemm_packed(const Gemm& g, const void* Bp, hipStream_t st);
// Bytes of work space gemm_packed would use for this problem if given one (0: its last round is not shared).
size_t packed_ws_needed(const Gemm& g);

// ---- row-wise and elementwise kernels ------------------------------------------------------
hipError_t embed_fwd(int dt, const int32_t* tokens, int64_t T, int S, int d, int V,
                     const void* tok_emb, const void* pos_emb, void* x, hipStream_t st);
// bf16 rows [rows, d] (d a multiple of 8): out[row][0] = sum of squares, out[row][1 .. n) = 0 (see Gemm::rowsq)
hipError_t row_sumsq(int64_t rows, int d, const void* x, int n, float* out, hipStream_t st);
hipError_t norm_fwd(int dt, bool rms, int64_t rows, int d, float eps, const void* x, const void* g,
                    const void* b, void* y, float* stats, hipStream_t st);
// dx = (dres ? dres : 0) + d norm / d x applied to dy
hipError_t norm_bwd_dx(int dt, bool rms, int64_t rows, int d, const void* dy, const void* x,
                       const void* g, const float* stats, const void* dres, void* dx, hipStream_t st);
// dg[j] = sum_r dy[r,j] * xhat[r,j];  db[j] = sum_r dy[r,j]  (db may be null); fp32 outputs.
// part: fp32 scratch of 2 * ceil(rows/64) * d floats.
hipError_t norm_bwd_params(int dt, bool rms, int64_t rows, int d, const void* dy, const void* x,
                           const float* stats, float* part, float* dg, float* db, hipStream_t st);
// out[j] = sum_r y[r*ld + j], fp32 output; part: scratch of ceil(rows/64) * n floats
hipError_t col_sum(int dt, int64_t rows, int64_t n, const void* y, int64_t ld, float* part,
                   float* out, hipStream_t st);
// rotary embedding in place on the q and k parts of qkv [T, 3d]; sign = +1 forward, -1 adjoint
hipError_t rope(int dt, void* qkv, int64_t T, int S, int H, int hd, const float* cos_sin, int sign,
                hipStream_t st);
hipError_t gelu_fwd(int dt, int64_t n, const void* pre, void* act, hipStream_t st);
hipError_t gelu_bwd(int dt, int64_t n, const void* dact, const void* pre, void* dpre, hipStream_t st);
// gu [T, 2f] = gate | up  ->  act [T, f]
hipError_t swiglu_fwd(int dt, int64_t T, int f, const void* gu, void* act, hipStream_t st);
hipError_t swiglu_bwd(int dt, int64_t T, int f, const void* dact, const void* gu, void* dgu, hipStream_t st);
// Fused attention (attention.hip): qkv [B*S, ld] holds q | k | v of every head side by side (head h at columns
// h*hd, d + h*hd, 2d + h*hd, d = H*hd).  bf16 only, hd 64 or 128.
// Forward: writes the context [B*S, ldc] (head h at columns h*hd); the probabilities [B, H, S, S] if prob is
// given; lse [B*H*S] fp32 if given: log2 of each row's sum of exponentials, what the backward needs.
bool attention_fwd_fused_applies(int dt, int S, int hd, int64_t ld, int64_t ldc, const void* qkv, const void* prob, const void* ctx);
hipError_t attention_fwd_fused(int B, int H, int S, int hd, bool causal, const void* qkv, int64_t ld, void* prob, void* ctx,
                               int64_t ldc, float* lse, hipStream_t st);
// Backward in two kernels, query-major (dq; leaves D = dO . O per query in dsum [B*H*S] fp32) and key-major
// (dk, dv); both form the probabilities again from q, k and lse, so nothing of size S x S is read or written.
// All of dqkv [B*S, ld] is written.  cos_sin: fp32 [>= S, hd/2] pairs (cos, sin) or null; if given, dq and dk
// are un-rotated on the way out (the adjoint of the rotary embedding applied to q and k after their projection).
bool attention_bwd_fused_applies(int dt, int S, int hd, int64_t ld, int64_t ldc, const void* qkv, const void* ctx, const void* dctx,
                                 const void* dqkv);
hipError_t attention_bwd_fused(int B, int H, int S, int hd, bool causal, const void* qkv, int64_t ld, const void* ctx,
                               const float* lse, const void* dctx, int64_t ldc, float* dsum, void* dqkv, const float* cos_sin,
                               hipStream_t st);
// in place over scores [nbh, S, S]: p = softmax(scale * s + causal mask)
hipError_t softmax_fwd(int dt, int64_t nbh, int S, float scale, bool causal, void* s, hipStream_t st);
// in place over dp: ds = scale * p * (dp - sum_j dp p)
hipError_t softmax_bwd(int dt, int64_t nbh, int S, float scale, bool causal, const void* p, void* dp, hipStream_t st);
// logits [rows, V] -> d loss / d logits in place; loss = mean over labels >= 0
hipError_t cross_entropy(int dt, int64_t rows, int V, void* logits, const int32_t* labels,
                         float* row_loss, float* loss_out, hipStream_t st);
// its three launches one by one (row_loss: rows + 1 floats): the number of rows with a target into row_loss[rows];
// the rows (per-row loss into row_loss[r], gradient over the logits); the mean of the per-row losses
hipError_t cross_entropy_count(int64_t rows, const int32_t* labels, float* row_loss, hipStream_t st);
hipError_t cross_entropy_rows(int dt, int64_t rows, int V, void* logits, const int32_t* labels, float* row_loss,
                              hipStream_t st);
hipError_t cross_entropy_mean(int64_t rows, const float* row_loss, float* loss_out, hipStream_t st);
// g_tok[v, :] = (add ? g_tok[v, :] : as zeroed by the caller) + sum over positions t holding token v of dx[t, :],
// in position order (no atomics: the first position holding a token does its row);  g_pos[s, :] = sum_b dx[b*S+s, :]
hipError_t embed_bwd(int dt, const int32_t* tokens, int64_t T, int S, int d, int V, const void* dx,
                     float* g_tok, float* g_pos, bool add, hipStream_t st);
// rows of x at positions b*S (first token of every sequence) -> y [B, d], and the adjoint
hipError_t gather_first(int dt, int B, int S, int d, const void* x, void* y, hipStream_t st);
hipError_t scatter_first(int dt, int B, int S, int d, const void* dy, void* dx, hipStream_t st);
// x[i] = a x[i] (one rounding in the storage type); for the small operands of the low-rank adapters
hipError_t scale_inplace(int dt, int64_t n, float a, void* x, hipStream_t st);
hipError_t cast_f32_to(int dt, int64_t n, const float* src, void* dst, hipStream_t st);
hipError_t cast_to_f32(int dt, int64_t n, const void* src, float* dst, hipStream_t st);
hipError_t fill_zero(void* p, size_t bytes, hipStream_t st);
// copy of a multiple of 16 bytes by a grid of `blocks` workgroups; either side may be pinned host memory
hipError_t copy_stream(void* dst, const void* src, size_t bytes, int blocks, hipStream_t st);

// ---- optimizer ---------------------------------------------------------------------------
struct OptArgs {
  int kind; double lr, beta1, beta2, eps, wd, momentum;
};
hipError_t optimizer_update(const OptArgs& o, int64_t n, bool decay, int64_t t, float* master,
                            const float* grad, float* s1, float* s2, void* compute_copy /* bf16 or null */,
                            hipStream_t st);

// Adafactor on one tensor (Shazeer and Stern 2018, Algorithm 4 without momentum, external step
// size; constants: epsilon_1 1e-30, clipping threshold 1, decay exponent 0.8).
//   rows x cols matrix: fac = [R (rows) | C (cols)];  vector (cols == 1): fac = V (rows).
//   work: floats, at least adafactor_work_floats(rows, cols).
size_t adafactor_work_floats(int64_t rows, int64_t cols);
hipError_t adafactor_update(double lr, double wd, bool decay, int64_t t, int64_t rows, int64_t cols, float* master,
                            const float* grad, float* fac, float* work, void* compute_copy /* bf16 or null */,
                            hipStream_t st);

}  // namespace hift
