// fa_compress: Fourier projection of the compressed head dimensions of a token
// segment (Eq. 2-3; Eq. 5 with accumulate) on the gfx950 matrix cores.
//
//   C[m,i] = sum_j phi_m(t0+j) X[j, idx_c[i]]         (a contraction over tokens)
//   X_keep[j,i'] = X[j, idx_u[i']]                     (packed kept dimensions)
//
// One workgroup owns (sequence, head, token chunk, block of 256 basis rows,
// block of 128 compressed columns).  Per 32-token step it
//   * reads the [32, D] slab of X once with 128-bit loads, scatters the
//     compressed columns transposed into LDS ([column][token]) and writes the
//     kept columns straight to x_keep,
//   * produces the [256, 32] slab of the basis in LDS by advancing per-thread
//     (cos, sin) pairs with one complex rotation per entry (exact integer-
//     reduced phases at the start of the chunk and every 32 steps),
//   * issues 16x16x32 MFMAs with the basis slab as A and the X slab as B.
// Token chunks are reduced in a second, deterministic pass.
//
// Internal row order of the basis block (so that every (cos, sin) pair is two
// adjacent rows owned by one thread): row 0 = constant, row 1 = cosine of order
// M/2 when M is even (it has no sine partner in the kept set), rows 2n, 2n+1 =
// cos, sin of order n for n = 1 .. (M-1)/2.

#include "fa_common.hpp"
#include "fa_mma.hpp"

namespace fa {

constexpr int kCBlock = 256;
constexpr int kKT = 32;         // tokens per MFMA step
constexpr int kLd = kKT + 8;    // LDS row pitch in elements (keeps 16-byte alignment, spreads banks)
constexpr int kRows = 256;      // basis rows per workgroup
constexpr int kCols = 128;      // compressed columns per workgroup
constexpr int kReanchor = 32;   // steps between exact re-evaluations of the rotating basis

struct CompressParams {
  const void* x;
  int64_t sx_b, sx_h, sx_n;
  int B, H, N, D, Dc, Du, M, T, t0, accumulate;
  const uint8_t* mask;
  float* coeffs;
  void* keep;
  int keep_layout;
  int keep_pitch;   // FA_KEEP_ROWS: elements per row, Du rounded up to 8
  int64_t keep_stride;
  int keep_offset;
  int Sc, chunk;  // token chunks and their length (multiple of kKT)
  int MC, DCn;    // row blocks, column blocks
  int P;          // (M-1)/2 complete (cos, sin) pairs
  float* part;    // [Sc][B*H][M][Dc] when Sc > 1
};

template <typename T> struct Pack16;
template <> struct Pack16<bf16_t> {
  // 16 consecutive tokens of one basis row -> two 128-bit LDS stores
  __device__ static __forceinline__ void store(bf16_t* dst, const float* v) {
    u32x4 a, b;
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      a[e] = static_cast<uint32_t>(f32_to_bf16(v[2 * e])) |
             (static_cast<uint32_t>(f32_to_bf16(v[2 * e + 1])) << 16);
      b[e] = static_cast<uint32_t>(f32_to_bf16(v[8 + 2 * e])) |
             (static_cast<uint32_t>(f32_to_bf16(v[8 + 2 * e + 1])) << 16);
    }
    *reinterpret_cast<u32x4*>(dst) = a;
    *reinterpret_cast<u32x4*>(dst + 8) = b;
  }
};
template <> struct Pack16<float> {
  __device__ static __forceinline__ void store(float* dst, const float* v) {
#pragma unroll
    for (int e = 0; e < 4; ++e)
      *reinterpret_cast<f32x4*>(dst + 4 * e) = f32x4{v[4 * e], v[4 * e + 1], v[4 * e + 2], v[4 * e + 3]};
  }
};

// 8 consecutive elements of a row of X (16-byte aligned)
__device__ __forceinline__ void load8(const bf16_t* p, bf16_t* out) {
  *reinterpret_cast<u32x4*>(out) = *reinterpret_cast<const u32x4*>(p);
}
__device__ __forceinline__ void load8(const float* p, float* out) {
  *reinterpret_cast<f32x4*>(out) = *reinterpret_cast<const f32x4*>(p);
  *reinterpret_cast<f32x4*>(out + 4) = *reinterpret_cast<const f32x4*>(p + 4);
}
__device__ __forceinline__ bf16_t zero_elem(const bf16_t*) { return bf16_t{0}; }
__device__ __forceinline__ float zero_elem(const float*) { return 0.0f; }

template <typename T>
__global__ __launch_bounds__(kCBlock) void compress_project(CompressParams p) {
  __shared__ __attribute__((aligned(16))) T phi_s[kRows * kLd];
  __shared__ __attribute__((aligned(16))) T xc_s[kCols * kLd];
  __shared__ int16_t cpos[FA_MAX_HEAD_DIM];
  __shared__ uint8_t mask_s[FA_MAX_HEAD_DIM];

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int s = blockIdx.x, mc = blockIdx.y % p.MC, dc = blockIdx.y / p.MC;
  const int bh = blockIdx.z, b = bh / p.H, h = bh % p.H;
  const int D = p.D, M = p.M;
  const int j0 = s * p.chunk, jend = min(p.N, j0 + p.chunk);
  const bool write_keep = (blockIdx.y == 0) && p.keep != nullptr && p.Du > 0;
  const bool project = p.Dc > 0;

  // cpos[d]: >= 0 index among kept dims, < 0: -(1 + index among compressed dims)
  for (int d = tid; d < D; d += kCBlock) mask_s[d] = p.mask[static_cast<size_t>(bh) * D + d] ? 1 : 0;
  __syncthreads();
  for (int d = tid; d < D; d += kCBlock) {
    int nc = 0;
    for (int e = 0; e < d; ++e) nc += mask_s[e];
    cpos[d] = mask_s[d] ? static_cast<int16_t>(-(1 + nc)) : static_cast<int16_t>(d - nc);
  }
  // unused columns of the X slab stay zero for the whole kernel
  for (int it = tid; it < kCols * kLd; it += kCBlock) xc_s[it] = zero_elem(xc_s);
  __syncthreads();

  // ---- rotating basis state: thread owns pair pl of this row block, 16 tokens
  const int pl = tid >> 1, half = tid & 1;
  const int pg = mc * (kRows / 2) + pl;           // global pair index
  const bool pair_live = project && pg <= p.P;
  const int order = (pg == 0) ? (M / 2) : pg;     // pair 0 carries the unpaired cosine
  float bc[16], bs[16], tc = 1.0f, ts = 0.0f;
  if (pair_live) unit_phase(order, kKT, p.T, &tc, &ts);

  const int rows_here = min(kRows, 2 * (p.P + 1) - mc * kRows);  // live internal rows
  const int cols_here = min(kCols, p.Dc - dc * kCols);
  const int DT = (cols_here + 15) / 16;

  f32x4 acc[4][8];
#pragma unroll
  for (int mt = 0; mt < 4; ++mt)
#pragma unroll
    for (int dt = 0; dt < 8; ++dt) acc[mt][dt] = f32x4{0.f, 0.f, 0.f, 0.f};

  const T* xbase = static_cast<const T*>(p.x) + b * p.sx_b + h * p.sx_h;
  T* keep = static_cast<T*>(p.keep) + static_cast<int64_t>(bh) * p.keep_stride;
  const int nch = D / 8;
  const int q = lane >> 4, r16 = lane & 15;

  int step = 0;
  for (int js = j0; js < jend; js += kKT, ++step) {
    // -- basis slab for tokens js .. js+31 (in registers until the LDS is free)
    if (pair_live) {
      if (step % kReanchor == 0) {
#pragma unroll
        for (int u = 0; u < 16; ++u) unit_phase(order, p.t0 + js + 16 * half + u, p.T, &bc[u], &bs[u]);
      } else {
#pragma unroll
        for (int u = 0; u < 16; ++u) {
          const float c = bc[u] * tc - bs[u] * ts;
          const float sn = bs[u] * tc + bc[u] * ts;
          bc[u] = c;
          bs[u] = sn;
        }
      }
    }
    __syncthreads();  // previous step's MFMAs have consumed the LDS slabs

    // -- X slab: 128-bit loads, compressed columns transposed into LDS, kept ones to x_keep
    for (int it = tid; it < kKT * nch; it += kCBlock) {
      const int jt = it / nch, ch = it % nch;
      const int j = js + jt;
      T v[8];
      if (j < jend) {
        load8(xbase + static_cast<int64_t>(j) * p.sx_n + ch * 8, v);
      } else {
#pragma unroll
        for (int e = 0; e < 8; ++e) v[e] = zero_elem(v);
      }
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        const int cp = cpos[ch * 8 + e];
        if (cp < 0) {
          const int rank = -cp - 1 - dc * kCols;
          if (rank >= 0 && rank < kCols) xc_s[rank * kLd + jt] = v[e];
        } else if (write_keep && j < jend) {
          const int64_t tok = static_cast<int64_t>(p.keep_offset) + j;
          const int64_t off = (p.keep_layout == FA_KEEP_ROWS)
                                  ? tok * p.keep_pitch + cp
                                  : ((tok >> 3) * p.Du + cp) * 8 + (tok & 7);
          keep[off] = v[e];
        }
      }
    }
    if (write_keep && p.keep_layout == FA_KEEP_ROWS && p.keep_pitch > p.Du) {
      const int npad = p.keep_pitch - p.Du;
      for (int it = tid; it < kKT * npad; it += kCBlock) {
        const int j = js + it / npad;
        if (j < jend)
          keep[(static_cast<int64_t>(p.keep_offset) + j) * p.keep_pitch + p.Du + it % npad] = zero_elem(keep);
      }
    }
    if (project) {
      float row0[16], row1[16];
#pragma unroll
      for (int u = 0; u < 16; ++u) {
        if (!pair_live) { row0[u] = 0.0f; row1[u] = 0.0f; }
        else if (pg == 0) { row0[u] = 1.0f; row1[u] = (M % 2 == 0) ? bc[u] : 0.0f; }
        else { row0[u] = bc[u]; row1[u] = bs[u]; }
      }
      Pack16<T>::store(&phi_s[(2 * pl) * kLd + 16 * half], row0);
      Pack16<T>::store(&phi_s[(2 * pl + 1) * kLd + 16 * half], row1);
    }
    __syncthreads();

    // -- MFMA: wave owns rows [64*wave, 64*wave+64) of the block
    if (project && wave * 64 < rows_here) {
      Frag<T> a[4];
#pragma unroll
      for (int mt = 0; mt < 4; ++mt) a[mt].load(&phi_s[(wave * 64 + mt * 16 + r16) * kLd + 8 * q]);
#pragma unroll
      for (int dt = 0; dt < 8; ++dt) {
        if (dt < DT) {
          Frag<T> bfr;
          bfr.load(&xc_s[(dt * 16 + r16) * kLd + 8 * q]);
#pragma unroll
          for (int mt = 0; mt < 4; ++mt) mma_k32(acc[mt][dt], a[mt], bfr);
        }
      }
    }
  }

  // ---- epilogue: accumulator rows back to the caller's basis order
  if (!project) return;
  const size_t BH = static_cast<size_t>(p.B) * p.H;
  float* dst = (p.Sc == 1) ? p.coeffs + static_cast<size_t>(bh) * M * p.Dc
                           : p.part + (static_cast<size_t>(s) * BH + bh) * M * p.Dc;
  const bool add = (p.Sc == 1) && p.accumulate;
#pragma unroll
  for (int mt = 0; mt < 4; ++mt) {
#pragma unroll
    for (int v = 0; v < 4; ++v) {
      const int rho = mc * kRows + wave * 64 + mt * 16 + 4 * q + v;  // internal row
      int m;
      if (rho == 0) m = 0;
      else if (rho == 1) m = (M % 2 == 0) ? M - 1 : -1;   // unpaired cosine of order M/2
      else m = 2 * (rho >> 1) - 1 + (rho & 1);            // rows 2n, 2n+1 -> m = 2n-1, 2n
      if (m < 0 || (rho >= 2 && (rho >> 1) > p.P)) continue;
#pragma unroll
      for (int dt = 0; dt < 8; ++dt) {
        const int i = dc * kCols + dt * 16 + r16;
        if (dt < DT && i < p.Dc) {
          float* o = dst + static_cast<size_t>(m) * p.Dc + i;
          const float val = acc[mt][dt][v];
          *o = add ? (*o + val) : val;
        }
      }
    }
  }
}

// sum of the token-chunk partials (fixed order, so results are reproducible)
__global__ __launch_bounds__(256) void compress_reduce(const float* part, float* coeffs, size_t total,
                                                       int Sc, int accumulate) {
  const size_t idx = static_cast<size_t>(blockIdx.x) * 256 + threadIdx.x;
  if (idx >= total) return;
  float v = accumulate ? coeffs[idx] : 0.0f;
  for (int s = 0; s < Sc; ++s) v += part[static_cast<size_t>(s) * total + idx];
  coeffs[idx] = v;
}

struct CompressPlan {
  int Sc, chunk, MC, DCn, P;
  size_t total;  // workspace bytes
};

static CompressPlan make_compress_plan(int B, int H, int N, int Dc, int M) {
  CompressPlan pl{};
  pl.P = (M - 1) / 2;
  const int rows = 2 * (pl.P + 1);
  pl.MC = Dc > 0 ? (rows + kRows - 1) / kRows : 1;
  pl.DCn = Dc > 0 ? (Dc + kCols - 1) / kCols : 1;
  const long groups = static_cast<long>(B) * H * pl.MC * pl.DCn;
  long want = (512 + groups - 1) / groups;  // token chunks needed to fill the chip
  const long steps = (N + kKT - 1) / kKT;
  if (want > steps) want = steps;
  if (want < 1) want = 1;
  if (want > 1024) want = 1024;
  const long per = N > 0 ? (steps + want - 1) / want : 1;
  pl.chunk = static_cast<int>(per) * kKT;
  pl.Sc = N > 0 ? (N + pl.chunk - 1) / pl.chunk : 0;
  pl.total = (pl.Sc > 1 && Dc > 0)
                 ? align_up(static_cast<size_t>(pl.Sc) * B * H * M * Dc * sizeof(float), 256)
                 : 0;
  return pl;
}

static int check_compress_shapes(int dtype, int B, int H, int N, int D, int Dc, int M, int T, int t0) {
  if (dtype != FA_F32 && dtype != FA_BF16) return FA_ERR_UNSUPPORTED;
  if (B <= 0 || H <= 0 || N < 0 || D <= 0 || Dc < 0 || Dc > D) return FA_ERR_SHAPE;
  if (M < 1 || T < 1 || M > T || t0 < 0 || static_cast<long>(t0) + N > T) return FA_ERR_SHAPE;
  if (D % 8 != 0 || D > FA_MAX_HEAD_DIM || M > FA_MAX_STATES) return FA_ERR_UNSUPPORTED;
  if (static_cast<long>(B) * H > 65535) return FA_ERR_UNSUPPORTED;
  return FA_OK;
}

}  // namespace fa

extern "C" {

size_t fa_compress_workspace_bytes(int B, int H, int N, int D, int Dc, int M) {
  if (fa::check_compress_shapes(FA_BF16, B, H, N, D, Dc, M, M > N ? M : N, 0) != FA_OK) return 0;
  const size_t t = fa::make_compress_plan(B, H, N, Dc, M).total;
  return t ? t : 256;
}

static int compress_impl(const void* x, int dtype, int64_t sx_b, int64_t sx_h, int64_t sx_n, int B,
                         int H, int N, int D, const uint8_t* dim_mask, int Dc, int M, int T, int t0,
                         int accumulate, float* coeffs, void* x_keep, int keep_layout,
                         int64_t keep_stride_bh, int keep_offset, void* workspace,
                         size_t workspace_bytes, void* hip_stream, hipEvent_t* ev) {
  using namespace fa;
  const int st = check_compress_shapes(dtype, B, H, N, D, Dc, M, T, t0);
  if (st != FA_OK) return st;
  if (!dim_mask || (Dc > 0 && !coeffs) || (N > 0 && !x)) return FA_ERR_NULL;
  if (keep_layout != FA_KEEP_ROWS && keep_layout != FA_KEEP_TOK8) return FA_ERR_SHAPE;
  if (keep_offset < 0) return FA_ERR_SHAPE;
  const int Du = D - Dc;
  if (N > 0) {
    if (sx_n < D || (sx_n % 8) || (sx_h % 8) || (sx_b % 8)) return FA_ERR_SHAPE;
    if (reinterpret_cast<uintptr_t>(x) & 15u) return FA_ERR_SHAPE;
  }
  const int64_t tokens = static_cast<int64_t>(keep_offset) + N;
  const int keep_pitch = (Du + 7) & ~7;
  const int64_t dense = (keep_layout == FA_KEEP_ROWS) ? tokens * keep_pitch : ((tokens + 7) / 8) * 8 * Du;
  if (keep_stride_bh == 0) keep_stride_bh = dense;
  if (x_keep && keep_stride_bh < dense) return FA_ERR_SHAPE;

  const CompressPlan pl = make_compress_plan(B, H, N, Dc, M);
  if (pl.total > 0) {
    if (!workspace) return FA_ERR_NULL;
    if (workspace_bytes < pl.total || (reinterpret_cast<uintptr_t>(workspace) & 255u))
      return FA_ERR_WORKSPACE;
  }

  CompressParams p{};
  p.x = x; p.sx_b = sx_b; p.sx_h = sx_h; p.sx_n = sx_n;
  p.B = B; p.H = H; p.N = N; p.D = D; p.Dc = Dc; p.Du = Du; p.M = M; p.T = T; p.t0 = t0;
  p.accumulate = accumulate ? 1 : 0;
  p.mask = dim_mask; p.coeffs = coeffs;
  p.keep = x_keep; p.keep_layout = keep_layout; p.keep_pitch = keep_pitch; p.keep_stride = keep_stride_bh; p.keep_offset = keep_offset;
  p.Sc = pl.Sc; p.chunk = pl.chunk; p.MC = pl.MC; p.DCn = pl.DCn; p.P = pl.P;
  p.part = static_cast<float*>(workspace);

  hipStream_t stream = static_cast<hipStream_t>(hip_stream);
  const size_t total = static_cast<size_t>(B) * H * M * Dc;
  if (ev) (void)hipEventRecord(ev[0], stream);
  if (pl.Sc > 0) {
    dim3 grid(pl.Sc, pl.MC * pl.DCn, B * H);
    if (dtype == FA_F32) hipLaunchKernelGGL(compress_project<float>, grid, dim3(kCBlock), 0, stream, p);
    else hipLaunchKernelGGL(compress_project<bf16_t>, grid, dim3(kCBlock), 0, stream, p);
  }
  if (ev) (void)hipEventRecord(ev[1], stream);
  if (total > 0 && (pl.Sc > 1 || (pl.Sc == 0 && !accumulate))) {
    const unsigned blocks = static_cast<unsigned>((total + 255) / 256);
    hipLaunchKernelGGL(compress_reduce, dim3(blocks), dim3(256), 0, stream, p.part, coeffs, total,
                       pl.Sc, p.accumulate);
  }
  if (ev) (void)hipEventRecord(ev[2], stream);
  return hipGetLastError() == hipSuccess ? FA_OK : FA_ERR_HIP;
}

int fa_compress(const void* x, int dtype, int64_t sx_b, int64_t sx_h, int64_t sx_n, int B, int H,
                int N, int D, const uint8_t* dim_mask, int Dc, int M, int T, int t0, int accumulate,
                float* coeffs, void* x_keep, int keep_layout, int64_t keep_stride_bh,
                int keep_offset, void* workspace, size_t workspace_bytes, void* hip_stream) {
  return compress_impl(x, dtype, sx_b, sx_h, sx_n, B, H, N, D, dim_mask, Dc, M, T, t0, accumulate,
                       coeffs, x_keep, keep_layout, keep_stride_bh, keep_offset, workspace,
                       workspace_bytes, hip_stream, nullptr);
}

int fa_compress_timed(const void* x, int dtype, int64_t sx_b, int64_t sx_h, int64_t sx_n, int B,
                      int H, int N, int D, const uint8_t* dim_mask, int Dc, int M, int T, int t0,
                      int accumulate, float* coeffs, void* x_keep, int keep_layout,
                      int64_t keep_stride_bh, int keep_offset, void* workspace,
                      size_t workspace_bytes, void* hip_stream, float* kernel_ms) {
  if (!kernel_ms) return FA_ERR_NULL;
  hipEvent_t ev[3];
  for (int i = 0; i < 3; ++i)
    if (hipEventCreate(&ev[i]) != hipSuccess) return FA_ERR_HIP;
  int st = compress_impl(x, dtype, sx_b, sx_h, sx_n, B, H, N, D, dim_mask, Dc, M, T, t0, accumulate,
                         coeffs, x_keep, keep_layout, keep_stride_bh, keep_offset, workspace,
                         workspace_bytes, hip_stream, ev);
  if (st == FA_OK) {
    if (hipEventSynchronize(ev[2]) != hipSuccess) st = FA_ERR_HIP;
    for (int i = 0; i < 2 && st == FA_OK; ++i)
      if (hipEventElapsedTime(&kernel_ms[i], ev[i], ev[i + 1]) != hipSuccess) st = FA_ERR_HIP;
  }
  for (int i = 0; i < 3; ++i) (void)hipEventDestroy(ev[i]);
  return st;
}

const char* fa_status_string(int status) {
  switch (status) {
    case FA_OK: return "ok";
    case FA_ERR_NULL: return "a required pointer is NULL";
    case FA_ERR_SHAPE: return "inconsistent or out-of-range sizes";
    case FA_ERR_UNSUPPORTED: return "outside the compiled limits";
    case FA_ERR_WORKSPACE: return "workspace too small or misaligned";
    case FA_ERR_HIP: return "HIP launch error";
    default: return "unknown status";
  }
}

}  // extern "C"
