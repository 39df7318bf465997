// fa_select_dims: which head dimensions to compress (paper, Section 3.4).
//
// Every head dimension of a token segment is compressed onto the first M basis functions
// and rebuilt (Eq. 3, then Eq. 6); the Dc dimensions with the lowest mean squared
// reconstruction error are the ones to compress.  The segment spans exactly one period
// (T = N, positions 0 .. N-1), where the basis is orthogonal and compress -> rebuild is
// the orthogonal projector onto its span, so the error needs no rebuilt row:
//     mse[d] = ( sum_j x[j,d]^2  -  sum_m w_m C[m,d]^2 ) / N .
// The difference of two sums is only as good as the coefficients, so they are formed in
// fp32 throughout (bf16 segments are widened first, which is exact), not with the bf16
// basis of the production compress kernel.  Three stages on the caller's stream:
//   1. select_energy : one pass over X: per-dim sums of squares per token chunk, the fp32
//      copy of a bf16 segment, an all-ones mask row
//   2. fa_compress   : all D dims, fp32 path, coefficients into the workspace
//   3. select_rank   : per (sequence, head): errors, ranks (ties to the lower dim), mask

#include "fa_common.hpp"
#include "fa_mma.hpp"

namespace fa {

constexpr int kSBlock = 256;
constexpr int kSChunk = 1024;   // tokens per workgroup of the energy pass

struct SelectParams {
  const void* x;
  int64_t sx_b, sx_h, sx_n;
  float* xf;          // fp32 copy [B,H,N,D] (bf16 input only)
  uint8_t* ones;      // [B,H,D]
  float* epart;       // [chunks][B*H][D]
  const float* coeffs;   // [B,H,M,D]
  uint8_t* mask_out;  // [B,H,D]
  float* mse_out;     // [B,H,D] or null
  int B, H, N, D, M, Dc, chunks;
};

// grid (chunks, B*H).  Thread (vector of 8 dims, row group): strided over the chunk's tokens.
template <typename T>
__global__ __launch_bounds__(kSBlock) void select_energy(SelectParams p) {
  __shared__ float red[kSBlock * 8];
  const int tid = threadIdx.x;
  const int bh = blockIdx.y, b = bh / p.H, h = bh % p.H;
  const int nch = p.D / 8, nrow = kSBlock / nch;          // D / 8 <= 32 vectors per row; threads past nrow * nch idle
  const int ch = tid % nch, row = tid / nch;
  const int j0 = blockIdx.x * kSChunk, jend = min(p.N, j0 + kSChunk);
  const T* xs = static_cast<const T*>(p.x) + b * p.sx_b + h * p.sx_h + ch * 8;
  float* xf = p.xf ? p.xf + (static_cast<size_t>(bh) * p.N) * p.D + ch * 8 : nullptr;
  float acc[8];
#pragma unroll
  for (int e = 0; e < 8; ++e) acc[e] = 0.0f;
  if (row < nrow) {
    for (int j = j0 + row; j < jend; j += nrow) {
      float v[8];
      if constexpr (sizeof(T) == 2) {
        Frag<T> f;
        f.load(xs + static_cast<int64_t>(j) * p.sx_n);
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          v[2 * e] = __builtin_bit_cast(float, f.v[e] << 16);
          v[2 * e + 1] = __builtin_bit_cast(float, f.v[e] & 0xffff0000u);
        }
        float* o = xf + static_cast<size_t>(j) * p.D;
        *reinterpret_cast<f32x4*>(o) = f32x4{v[0], v[1], v[2], v[3]};
        *reinterpret_cast<f32x4*>(o + 4) = f32x4{v[4], v[5], v[6], v[7]};
      } else {
        const float* src = reinterpret_cast<const float*>(xs) + static_cast<int64_t>(j) * p.sx_n;
        const f32x4 a = *reinterpret_cast<const f32x4*>(src), c = *reinterpret_cast<const f32x4*>(src + 4);
        v[0] = a[0]; v[1] = a[1]; v[2] = a[2]; v[3] = a[3];
        v[4] = c[0]; v[5] = c[1]; v[6] = c[2]; v[7] = c[3];
      }
#pragma unroll
      for (int e = 0; e < 8; ++e) acc[e] += v[e] * v[e];
    }
  }
  if (row < nrow) {
#pragma unroll
    for (int e = 0; e < 8; ++e) red[row * p.D + ch * 8 + e] = acc[e];
  }
  __syncthreads();
  if (tid < p.D) {
    float s = 0.0f;
    for (int r = 0; r < nrow; ++r) s += red[r * p.D + tid];
    p.epart[(static_cast<size_t>(blockIdx.x) * gridDim.y + bh) * p.D + tid] = s;
    if (blockIdx.x == 0) p.ones[static_cast<size_t>(bh) * p.D + tid] = 1;
  }
}

// grid (B*H), 1024 threads: thread (dim d, row group g) sums its share of the chunk energies and of
// the weighted squared coefficients (independent loads, several in flight), the groups meet in
// LDS, then thread d ranks its dim
constexpr int kRBlock = 1024;
__global__ __launch_bounds__(kRBlock) void select_rank(SelectParams p) {
  __shared__ double ex_s[kRBlock], ec_s[kRBlock];
  __shared__ float err[FA_MAX_HEAD_DIM];
  const int tid = threadIdx.x, bh = blockIdx.x;
  const int D = p.D, M = p.M, N = p.N;
  const int ng = kRBlock / D;                  // row groups (4 .. 128)
  const int d = tid % D, g = tid / D;
  double ex = 0.0, ec = 0.0;
  if (g < ng) {
    for (int c = g; c < p.chunks; c += ng) ex += p.epart[(static_cast<size_t>(c) * gridDim.x + bh) * D + d];
    const float* C = p.coeffs + static_cast<size_t>(bh) * M * D + d;
#pragma unroll 8
    for (int m = g; m < M; m += ng) {
      const double cm = C[static_cast<size_t>(m) * D];
      ec += static_cast<double>(basis_weight((m + 1) / 2, N)) * cm * cm;
    }
  }
  ex_s[tid] = ex;
  ec_s[tid] = ec;
  __syncthreads();
  float e = 0.0f;
  if (tid < D) {
    double sx = 0.0, sc = 0.0;
    for (int k = 0; k < ng; ++k) {             // fixed order: reproducible
      sx += ex_s[k * D + tid];
      sc += ec_s[k * D + tid];
    }
    e = static_cast<float>(fmax(sx - sc, 0.0) / N);
    err[tid] = e;
    if (p.mse_out) p.mse_out[static_cast<size_t>(bh) * D + tid] = e;
  }
  __syncthreads();
  if (tid < D) {
    int rank = 0;
    for (int o = 0; o < D; ++o) {
      const float eo = err[o];
      rank += (eo < e || (eo == e && o < tid)) ? 1 : 0;
    }
    p.mask_out[static_cast<size_t>(bh) * D + tid] = rank < p.Dc ? 1 : 0;
  }
}

struct SelectPlan {
  int chunks;
  size_t off_ones, off_epart, off_coeffs, off_xf, off_cws, cws_bytes, total;
};

static size_t align256(size_t x) { return (x + 255) & ~static_cast<size_t>(255); }

static int check_select_shapes(int dtype, int B, int H, int N, int D, int M, int Dc) {
  if (dtype != FA_F32 && dtype != FA_BF16) return FA_ERR_UNSUPPORTED;
  if (B <= 0 || H <= 0 || N < 1 || D <= 0 || Dc < 0 || Dc > D) return FA_ERR_SHAPE;
  if (M < 1 || M > N) return FA_ERR_SHAPE;
  if (D % 8 != 0 || D > FA_MAX_HEAD_DIM || M > FA_MAX_STATES) return FA_ERR_UNSUPPORTED;
  if (static_cast<long>(B) * H > 65535) return FA_ERR_UNSUPPORTED;
  return FA_OK;
}

static SelectPlan make_select_plan(int dtype, int B, int H, int N, int D, int M) {
  SelectPlan pl{};
  const size_t BH = static_cast<size_t>(B) * H;
  pl.chunks = (N + kSChunk - 1) / kSChunk;
  size_t off = 0;
  pl.off_ones = off;   off = align256(off + BH * D);
  pl.off_epart = off;  off = align256(off + static_cast<size_t>(pl.chunks) * BH * D * sizeof(float));
  pl.off_coeffs = off; off = align256(off + BH * M * D * sizeof(float));
  pl.off_xf = off;
  if (dtype == FA_BF16) off = align256(off + BH * N * D * sizeof(float));
  pl.off_cws = off;
  pl.cws_bytes = fa_compress_workspace_bytes(B, H, N, D, D, M);
  pl.total = align256(off + pl.cws_bytes);
  return pl;
}

}  // namespace fa

extern "C" {

size_t fa_select_workspace_bytes(int dtype, int B, int H, int N, int D, int M) {
  if (fa::check_select_shapes(dtype, B, H, N, D, M, 0) != FA_OK) return 0;
  return fa::make_select_plan(dtype, B, H, N, D, M).total;
}

int fa_select_dims(const void* x, int dtype, int64_t sx_b, int64_t sx_h, int64_t sx_n, int B, int H,
                   int N, int D, int M, int Dc, uint8_t* dim_mask, float* mse, void* workspace,
                   size_t workspace_bytes, void* hip_stream) {
  using namespace fa;
  const hipError_t prior = hipPeekAtLastError();   // (an error left by earlier, unrelated calls is not this call's)
  const int st = check_select_shapes(dtype, B, H, N, D, M, Dc);
  if (st != FA_OK) return st;
  if (!x || !dim_mask || !workspace) return FA_ERR_NULL;
  if (sx_n < D || (sx_n % 8) || (sx_h % 8) || (sx_b % 8)) return FA_ERR_SHAPE;
  if (reinterpret_cast<uintptr_t>(x) & 15u) return FA_ERR_SHAPE;
  const SelectPlan pl = make_select_plan(dtype, B, H, N, D, M);
  if (workspace_bytes < pl.total || (reinterpret_cast<uintptr_t>(workspace) & 255u)) return FA_ERR_WORKSPACE;

  char* ws = static_cast<char*>(workspace);
  SelectParams p{};
  p.x = x; p.sx_b = sx_b; p.sx_h = sx_h; p.sx_n = sx_n;
  p.xf = dtype == FA_BF16 ? reinterpret_cast<float*>(ws + pl.off_xf) : nullptr;
  p.ones = reinterpret_cast<uint8_t*>(ws + pl.off_ones);
  p.epart = reinterpret_cast<float*>(ws + pl.off_epart);
  float* coeffs = reinterpret_cast<float*>(ws + pl.off_coeffs);
  p.coeffs = coeffs;
  p.mask_out = dim_mask; p.mse_out = mse;
  p.B = B; p.H = H; p.N = N; p.D = D; p.M = M; p.Dc = Dc; p.chunks = pl.chunks;

  hipStream_t stream = static_cast<hipStream_t>(hip_stream);
  const dim3 g1(pl.chunks, B * H);
  if (dtype == FA_BF16) hipLaunchKernelGGL(select_energy<bf16_t>, g1, dim3(kSBlock), 0, stream, p);
  else hipLaunchKernelGGL(select_energy<float>, g1, dim3(kSBlock), 0, stream, p);
  if (hipPeekAtLastError() != hipSuccess && prior == hipSuccess) return FA_ERR_HIP;

  // all D dims, period T = N, fp32 arithmetic
  int rc;
  if (dtype == FA_BF16) {
    const int64_t dn = D, dh = static_cast<int64_t>(N) * D, db = dh * H;
    rc = fa_compress(p.xf, FA_F32, db, dh, dn, B, H, N, D, p.ones, D, M, N, 0, 0, coeffs, nullptr,
                     FA_KEEP_ROWS, 0, 0, ws + pl.off_cws, pl.cws_bytes, hip_stream);
  } else {
    rc = fa_compress(x, FA_F32, sx_b, sx_h, sx_n, B, H, N, D, p.ones, D, M, N, 0, 0, coeffs, nullptr,
                     FA_KEEP_ROWS, 0, 0, ws + pl.off_cws, pl.cws_bytes, hip_stream);
  }
  if (rc != FA_OK) return rc;

  hipLaunchKernelGGL(select_rank, dim3(B * H), dim3(kRBlock), 0, stream, p);
  return (hipPeekAtLastError() == hipSuccess || prior != hipSuccess) ? FA_OK : FA_ERR_HIP;
}

}  // extern "C"
