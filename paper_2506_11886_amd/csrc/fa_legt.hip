// fa_legt_*: the translated-Legendre (HiPPO-LegT) alternative basis (paper, Sections 3.2 and 5.1).
//
// The paper compares its Fourier basis with Legendre polynomials on the same window by how well
// each rebuilds a KV dimension from the same number of states.  These kernels are that
// comparison's two halves for a token segment x[b,h] of N rows:
//   fa_legt_compress : C[m,d] = sum_j P_m(x_j) x[j,d],  x_j = (2j+1)/N - 1 (cell midpoints of [-1,1])
//   fa_legt_mse      : mse[d] = mean_j ( x[j,d] - sum_m (2m+1)/N C[m,d] P_m(x_j) )^2
// A polynomial basis has no shift structure (no angle addition), so nothing of the Fourier
// kernels' table-and-rotation scheme carries over: the basis values are produced per token by
// Bonnet's recurrence (in fp64: its rounding grows with the degree) and meet the data in plain
// fp32 vector arithmetic through LDS.  This is a calibration / ablation tool, not part of a
// decode step; it is bound by the fp32 vector rate.
//
// Launches on the caller's stream:
//   legt_project  grid (groups of 32 degrees, B*H, token chunks): partial states per chunk
//   legt_error    grid (tiles of 64 tokens, B*H): squared errors per tile and dim
//   legt_sum      out[i] = scale * sum_s part[s][i], fixed order, fp64 running sum

#include "fa_common.hpp"
#include "fa_mma.hpp"

namespace fa {

constexpr int kLBlock = 256;
constexpr int kLDeg = 32;       // degrees per group
constexpr int kLTile = 256;     // tokens per recurrence pass of legt_project
constexpr int kLSub = 16;       // tokens per LDS tile of X in legt_project
constexpr int kLErr = 64;       // tokens per workgroup of legt_error
constexpr int kLChunkTiles = 8; // recurrence passes per workgroup of legt_project (2048 tokens)

struct LegtParams {
  const void* x;
  int64_t sx_b, sx_h, sx_n;
  int B, H, N, D, M, Sc, tiles;
  float* part;          // projection: [Sc][B*H][M][D]; error: [tiles][B*H][D]
  const float* coeffs;  // [B,H,M,D]
};

template <typename T>
__device__ __forceinline__ float legt_elem(const T* p) { return Elem<T>::load(p); }

// position of token j among N: midpoint of its cell of [-1, 1]
__device__ __forceinline__ double legt_pos(int j, int N) {
  return (2.0 * static_cast<double>(j) + 1.0) / static_cast<double>(N) - 1.0;
}

// ---------------------------------------------------------------------------
// C[m,d] partial over a token chunk, degrees 32 g .. 32 g + 31
// ---------------------------------------------------------------------------
// Thread t of a pass owns token t of 256: it runs the recurrence from degree 0 up to the group's
// last degree and leaves the group's 32 values in LDS.  Then the 256 threads are (degree o, dim
// residue dg): each multiplies its degree's values with the dims dg, dg + 8, ... of the X tile.
template <typename T>
__global__ __launch_bounds__(kLBlock) void legt_project(LegtParams p) {
  __shared__ float pb[kLDeg][kLTile];                       // basis values of the group, per token of the pass
  __shared__ float xt[kLSub][FA_MAX_HEAD_DIM];              // X tile, fp32 (every thread of a step reads the same row)
  const int tid = threadIdx.x;
  const int g = blockIdx.x, bh = blockIdx.y, sc = blockIdx.z;
  const int b = bh / p.H, h = bh % p.H;
  const int D = p.D, N = p.N, nd = D / 8;
  const int m0 = g * kLDeg;
  const int j0 = sc * kLChunkTiles * kLTile, jend = min(N, j0 + kLChunkTiles * kLTile);
  const T* xs = static_cast<const T*>(p.x) + b * p.sx_b + h * p.sx_h;
  const int o = tid >> 3, dg = tid & 7;

  float acc[FA_MAX_HEAD_DIM / 8];
#pragma unroll
  for (int k = 0; k < FA_MAX_HEAD_DIM / 8; ++k) acc[k] = 0.0f;

  for (int jt = j0; jt < jend; jt += kLTile) {
    // -- recurrence of this thread's token (tokens past the segment get zeros) --------------
    {
      const int j = jt + tid;
      const double xj = legt_pos(min(j, N - 1), N);
      double pm1 = 0.0, pm = 1.0;                            // P_{m-1}, P_m at m = 0
      for (int m = 0; m < m0 + kLDeg; ++m) {
        if (m >= m0) pb[m - m0][tid] = (j < N && m < p.M) ? static_cast<float>(pm) : 0.0f;
        const double pn = ((2.0 * m + 1.0) * xj * pm - static_cast<double>(m) * pm1) / (m + 1.0);
        pm1 = pm;
        pm = pn;
      }
    }
    for (int js = 0; js < kLTile && jt + js < jend; js += kLSub) {
      __syncthreads();                                       // pb is complete / the previous X tile has been used
      for (int it = tid; it < kLSub * D; it += kLBlock) {
        const int r = it / D, d = it - r * D;
        const int j = min(jt + js + r, N - 1);               // rows past the segment meet zero basis values
        xt[r][d] = legt_elem<T>(xs + static_cast<int64_t>(j) * p.sx_n + d);
      }
      __syncthreads();
      for (int r = 0; r < kLSub; ++r) {
        const float bv = pb[o][js + r];
#pragma unroll
        for (int k = 0; k < FA_MAX_HEAD_DIM / 8; ++k)
          if (k < nd) acc[k] += bv * xt[r][dg + 8 * k];
      }
    }
    __syncthreads();                                         // pb is rewritten by the next pass
  }
  const int m = m0 + o;
  if (m < p.M) {
    float* dst = p.part + ((static_cast<size_t>(sc) * p.B * p.H + bh) * p.M + m) * D;
#pragma unroll
    for (int k = 0; k < FA_MAX_HEAD_DIM / 8; ++k)
      if (k < nd) dst[dg + 8 * k] = acc[k];
  }
}

// ---------------------------------------------------------------------------
// squared reconstruction errors of a tile of 64 tokens, per dim
// ---------------------------------------------------------------------------
// Thread (token t, dim residue dq): dims dq, dq + 4, ...  The token's recurrence state lives in
// the registers of its dq = 0 thread across the degree groups.
template <typename T>
__global__ __launch_bounds__(kLBlock) void legt_error(LegtParams p) {
  __shared__ float pb[kLDeg][kLErr];                         // (2m+1)/N P_m(x_j)
  __shared__ float cs[kLDeg][FA_MAX_HEAD_DIM + 1];           // states of the group
  __shared__ float er[kLBlock / 64][FA_MAX_HEAD_DIM];        // squared errors summed over a wave's 16 tokens
  const int tid = threadIdx.x;
  const int tile = blockIdx.x, bh = blockIdx.y;
  const int b = bh / p.H, h = bh % p.H;
  const int D = p.D, N = p.N, M = p.M, nd = D / 4;
  const int t = tid >> 2, dq = tid & 3;
  const int j = tile * kLErr + t;
  const T* xs = static_cast<const T*>(p.x) + b * p.sx_b + h * p.sx_h;
  const float* cf = p.coeffs + static_cast<size_t>(bh) * M * D;

  float acc[FA_MAX_HEAD_DIM / 4];
#pragma unroll
  for (int k = 0; k < FA_MAX_HEAD_DIM / 4; ++k) acc[k] = 0.0f;
  const double xj = legt_pos(min(j, N - 1), N);
  const double invN = 1.0 / static_cast<double>(N);
  double pm1 = 0.0, pm = 1.0;

  for (int m0 = 0; m0 < M; m0 += kLDeg) {
    __syncthreads();                                         // the previous group has been used
    if (dq == 0) {
      for (int mm = 0; mm < kLDeg; ++mm) {
        const int m = m0 + mm;
        pb[mm][t] = (m < M) ? static_cast<float>((2.0 * m + 1.0) * invN * pm) : 0.0f;
        const double pn = ((2.0 * m + 1.0) * xj * pm - static_cast<double>(m) * pm1) / (m + 1.0);
        pm1 = pm;
        pm = pn;
      }
    }
    for (int it = tid; it < kLDeg * D; it += kLBlock) {
      const int mm = it / D, d = it - mm * D;
      cs[mm][d] = cf[static_cast<size_t>(min(m0 + mm, M - 1)) * D + d];   // degrees past M meet zero basis values
    }
    __syncthreads();
    for (int mm = 0; mm < kLDeg; ++mm) {
      const float bv = pb[mm][t];
#pragma unroll
      for (int k = 0; k < FA_MAX_HEAD_DIM / 4; ++k)
        if (k < nd) acc[k] += bv * cs[mm][dq + 4 * k];
    }
  }
  // squared errors of this token; a wave holds 16 tokens x 4 dim residues: its tokens meet by lane
  // exchange (a fixed tree), the four waves in LDS, in order
  const int wave = tid >> 6, lane = tid & 63;
#pragma unroll
  for (int k = 0; k < FA_MAX_HEAD_DIM / 4; ++k) {
    if (k < nd) {
      const int d = dq + 4 * k;
      float e = 0.0f;
      if (j < N) {
        const float xv = legt_elem<T>(xs + static_cast<int64_t>(j) * p.sx_n + d);
        e = (xv - acc[k]) * (xv - acc[k]);
      }
#pragma unroll
      for (int o = 4; o < 64; o <<= 1) e += __shfl_xor(e, o, kWave);
      if (lane < 4) er[wave][d] = e;
    }
  }
  __syncthreads();
  for (int d = tid; d < D; d += kLBlock) {
    float s = 0.0f;
#pragma unroll
    for (int w = 0; w < kLBlock / 64; ++w) s += er[w][d];
    p.part[(static_cast<size_t>(tile) * p.B * p.H + bh) * D + d] = s;
  }
}

// out[i] = scale * sum_s part[s * n + i]
__global__ __launch_bounds__(kLBlock) void legt_sum(const float* part, float* out, size_t n, int S, float scale) {
  const size_t i = static_cast<size_t>(blockIdx.x) * kLBlock + threadIdx.x;
  if (i >= n) return;
  double s = 0.0;
  for (int k = 0; k < S; ++k) s += static_cast<double>(part[static_cast<size_t>(k) * n + i]);
  out[i] = static_cast<float>(s * static_cast<double>(scale));
}

static int check_legt(const void* x, int dtype, int64_t sx_b, int64_t sx_h, int64_t sx_n, int B, int H, int N,
                      int D, int M) {
  if (dtype != FA_F32 && dtype != FA_BF16) return FA_ERR_UNSUPPORTED;
  if (B <= 0 || H <= 0 || N <= 0 || D <= 0 || M < 1 || M > N) return FA_ERR_SHAPE;
  if (D % 8 != 0 || D > FA_MAX_HEAD_DIM || M > FA_MAX_STATES) return FA_ERR_UNSUPPORTED;
  if (static_cast<long>(B) * H > 65535) return FA_ERR_UNSUPPORTED;
  if (!x) return FA_ERR_NULL;
  if (sx_n < D || sx_h < 0 || sx_b < 0) return FA_ERR_SHAPE;
  (void)sx_b; (void)sx_h;
  return FA_OK;
}

static int legt_chunks(int N) { return (N + kLChunkTiles * kLTile - 1) / (kLChunkTiles * kLTile); }
static int legt_tiles(int N) { return (N + kLErr - 1) / kLErr; }

}  // namespace fa

extern "C" {

size_t fa_legt_workspace_bytes(int B, int H, int N, int D, int M) {
  if (B <= 0 || H <= 0 || N <= 0 || D <= 0 || M < 1) return 0;
  const size_t a = static_cast<size_t>(fa::legt_chunks(N)) * B * H * M * D * sizeof(float);
  const size_t b = static_cast<size_t>(fa::legt_tiles(N)) * B * H * D * sizeof(float);
  return fa::align_up(a > b ? a : b, 256);
}

int fa_legt_compress(const void* x, int dtype, int64_t sx_b, int64_t sx_h, int64_t sx_n, int B, int H, int N,
                     int D, int M, float* coeffs, void* workspace, size_t workspace_bytes, void* hip_stream) {
  using namespace fa;
  const int st = check_legt(x, dtype, sx_b, sx_h, sx_n, B, H, N, D, M);
  if (st != FA_OK) return st;
  if (!coeffs || !workspace) return FA_ERR_NULL;
  if (workspace_bytes < fa_legt_workspace_bytes(B, H, N, D, M) || (reinterpret_cast<uintptr_t>(workspace) & 255u))
    return FA_ERR_WORKSPACE;
  LegtParams p{};
  p.x = x; p.sx_b = sx_b; p.sx_h = sx_h; p.sx_n = sx_n;
  p.B = B; p.H = H; p.N = N; p.D = D; p.M = M;
  p.Sc = legt_chunks(N);
  p.part = static_cast<float*>(workspace);
  hipStream_t stream = static_cast<hipStream_t>(hip_stream);
  const hipError_t prior = hipPeekAtLastError();
  const dim3 grid((M + kLDeg - 1) / kLDeg, B * H, p.Sc);
  if (dtype == FA_F32) hipLaunchKernelGGL(legt_project<float>, grid, dim3(kLBlock), 0, stream, p);
  else hipLaunchKernelGGL(legt_project<bf16_t>, grid, dim3(kLBlock), 0, stream, p);
  const size_t n = static_cast<size_t>(B) * H * M * D;
  hipLaunchKernelGGL(legt_sum, dim3(static_cast<unsigned>((n + kLBlock - 1) / kLBlock)), dim3(kLBlock), 0, stream,
                     p.part, coeffs, n, p.Sc, 1.0f);
  return (hipPeekAtLastError() == hipSuccess || prior != hipSuccess) ? FA_OK : FA_ERR_HIP;
}

int fa_legt_mse(const void* x, int dtype, int64_t sx_b, int64_t sx_h, int64_t sx_n, int B, int H, int N, int D,
                int M, const float* coeffs, float* mse, void* workspace, size_t workspace_bytes, void* hip_stream) {
  using namespace fa;
  const int st = check_legt(x, dtype, sx_b, sx_h, sx_n, B, H, N, D, M);
  if (st != FA_OK) return st;
  if (!coeffs || !mse || !workspace) return FA_ERR_NULL;
  if (workspace_bytes < fa_legt_workspace_bytes(B, H, N, D, M) || (reinterpret_cast<uintptr_t>(workspace) & 255u))
    return FA_ERR_WORKSPACE;
  LegtParams p{};
  p.x = x; p.sx_b = sx_b; p.sx_h = sx_h; p.sx_n = sx_n;
  p.B = B; p.H = H; p.N = N; p.D = D; p.M = M;
  p.tiles = legt_tiles(N);
  p.part = static_cast<float*>(workspace);
  p.coeffs = coeffs;
  hipStream_t stream = static_cast<hipStream_t>(hip_stream);
  const hipError_t prior = hipPeekAtLastError();
  const dim3 grid(p.tiles, B * H);
  if (dtype == FA_F32) hipLaunchKernelGGL(legt_error<float>, grid, dim3(kLBlock), 0, stream, p);
  else hipLaunchKernelGGL(legt_error<bf16_t>, grid, dim3(kLBlock), 0, stream, p);
  const size_t n = static_cast<size_t>(B) * H * D;
  hipLaunchKernelGGL(legt_sum, dim3(static_cast<unsigned>((n + kLBlock - 1) / kLBlock)), dim3(kLBlock), 0, stream,
                     p.part, mse, n, p.tiles, 1.0f / static_cast<float>(N));
  return (hipPeekAtLastError() == hipSuccess || prior != hipSuccess) ? FA_OK : FA_ERR_HIP;
}

}  // extern "C"
