// fa_compress: Fourier projection of the compressed head dimensions of a token
// segment (Eq. 2-3; Eq. 5 with accumulate) on the gfx950 matrix cores.
//
//   C[m,i] = sum_j phi_m(t0+j) X[j, idx_c[i]]         (a contraction over tokens)
//   X_keep[j,i'] = X[j, idx_u[i']]                     (packed kept dimensions)
//
// The basis never exists as a matrix.  With j = tau + u (tau = start of a
// 64-token block, u < 64) the angle-addition identity gives, per harmonic n,
//   [C_cos; C_sin] = sum_blocks Rot(omega_n tau) [E_cos X_blk; E_sin X_blk],
// where E[rho,u] = cos|sin(omega_n u) is a 64-column table that every wave keeps
// in registers as its MFMA A operand for the whole kernel.  Instead of rotating
// each block's product, the accumulators live in a frame that moves with the
// blocks: before a block is added they are rotated by -omega_n * 64 (four FMAs
// per (cos, sin) pair, in place in the MFMA accumulator registers), and once at
// the end by the exact phase of the last block.
//
// One workgroup owns (sequence, head, token chunk, 128 harmonics = 256 basis
// rows, 128 compressed columns).  Per block it reads the [64, D] slab of X once
// with 128-bit loads (the next slab is in flight while the current one is
// multiplied), scatters the compressed columns transposed into LDS and the kept
// columns into an LDS staging tile that is written out with 128-bit stores.
// The constant function (m = 0) is a plain column sum.  Token chunks are reduced
// in a second, deterministic pass.

#include "fa_common.hpp"
#include "fa_mma.hpp"

namespace fa {

constexpr int kCBlock = 512;      // 8 waves (generic kernel: 4 row groups of 64 basis rows x 2 column halves)
constexpr int kTB = 64;          // tokens per block
constexpr int kLdX = kTB + 8;    // LDS pitch (elements) of a transposed column: 16-byte aligned, bank-spread
constexpr int kPairs = 128;      // harmonics per workgroup (256 basis rows)
constexpr int kCols = 128;       // compressed columns per workgroup
constexpr unsigned kMaxCLds = 160 * 1024 - 8192;


typedef float f32x2c __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x2c __attribute__((ext_vector_type(2)));
typedef uint32_t u32x2c __attribute__((ext_vector_type(2)));

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
  int stage_keep;   // kept dims go through an LDS tile and leave as 128-bit stores
  int Sc, chunk;    // token chunks and their length (multiple of kTB)
  int MC, DCn;      // row blocks (128 harmonics each), column blocks
  int nmax;         // highest harmonic: M / 2
  uint32_t kv_magic;   // ceil(2^16 / kept-dim vectors per token (rows) or kept dims (groups of 8 tokens))
  unsigned ks_elems;   // elements of one keep-staging buffer
  double ph_scale;  // 2^32 / T
  float* part;      // [Sc][part_stride] when Sc > 1, chunk s holds [B*H][M][Dc]
  size_t part_stride;   // B*H*M*Dc rounded up to 4 floats
};

__device__ __forceinline__ void load8(const bf16_t* p, Frag<bf16_t>& f) { f.load(p); }
__device__ __forceinline__ void load8(const float* p, Frag<float>& f) { f.load(p); }
__device__ __forceinline__ bf16_t felem(const Frag<bf16_t>& f, int e) {
  return bf16_t{static_cast<uint16_t>((f.v[e >> 1] >> (16 * (e & 1))) & 0xffffu)};
}
__device__ __forceinline__ float felem(const Frag<float>& f, int e) { return f.v[e]; }
__device__ __forceinline__ float tof(bf16_t x) { return bf16_to_f32(x.bits); }
__device__ __forceinline__ float tof(float x) { return x; }
__device__ __forceinline__ bf16_t zero_elem(const bf16_t*) { return bf16_t{0}; }
__device__ __forceinline__ float zero_elem(const float*) { return 0.0f; }

// position -> phase in units of 2^-32 turns (wraps), and its cosine / sine.  An
// integer multiple n * phase wraps exactly, so harmonics cost one multiply.
__device__ __forceinline__ uint32_t fixed_phase(int pos, double ph_scale) {
  return static_cast<uint32_t>(static_cast<uint64_t>(static_cast<double>(pos) * ph_scale));
}
template <typename T>
__device__ __forceinline__ void fixed_phase_cs(uint32_t ph, float* c, float* s) {
  const float x = static_cast<float>(static_cast<int32_t>(ph)) * 2.3283064365386963e-10f;  // turns in [-0.5, 0.5)
  if constexpr (sizeof(T) == 4) {
    sincospif(2.0f * x, s, c);
  } else {
    *s = __builtin_amdgcn_sinf(x);
    *c = __builtin_amdgcn_cosf(x);
  }
}

template <typename T>
__device__ __forceinline__ void set_elem(Frag<T>& f, int e, float x);
template <>
__device__ __forceinline__ void set_elem<bf16_t>(Frag<bf16_t>& f, int e, float x) { f.set(e, x); }
template <>
__device__ __forceinline__ void set_elem<float>(Frag<float>& f, int e, float x) { f.v[e] = x; }

// DT: 16-column tiles of compressed dims per wave (a workgroup covers 2 * DT); kXR:
// 8-element vectors of X per thread and block (2 covers head dims up to 128, 4 up to 256)
// kFast: the row vectors divide the workgroup evenly (head dim 64 / 128 / 256) and
// kept dims are staged, so every thread routes the same 8 dims in every block.
// kSplit (bf16 only): the basis is held as a bf16 head plus a bf16 remainder (two products per
// operand, 2^-17 relative instead of 2^-9).  Used for short segments, where the matrix work is
// negligible and the rounding errors of a short period's few distinct basis values would not
// average out.
template <typename T, int DT, int kXR, bool kFast, bool kSplit>
__global__ __launch_bounds__(kCBlock) void compress_project(CompressParams p) {
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  __shared__ int16_t cpos[FA_MAX_HEAD_DIM];
  __shared__ float dcred[kCBlock];

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int q4 = lane >> 4, r16 = lane & 15;
  const int s = blockIdx.x, mc = blockIdx.y % p.MC, dc = blockIdx.y / p.MC;
  const int bh = blockIdx.z, b = bh / p.H, h = bh % p.H;
  const int D = p.D, M = p.M, Du = p.Du;
  const int j0 = s * p.chunk, jend = min(p.N, j0 + p.chunk);
  const int nb = (jend - j0 + kTB - 1) / kTB;
  const bool write_keep = (blockIdx.y == 0) && p.keep != nullptr && Du > 0;
  const bool stage = write_keep && p.stage_keep;
  const bool project = p.Dc > 0;
  const bool do_dc = project && mc == 0;

  // two buffers of [compressed columns kCols x kLdX | keep staging ks_elems | 8 spare elements]
  T* lds = reinterpret_cast<T*>(smem);
  const uint32_t bufe = kCols * kLdX + p.ks_elems + 8;      // elements per buffer

  // ---- first X block is requested before anything else --------------------------------
  const T* xbase = static_cast<const T*>(p.x) + b * p.sx_b + h * p.sx_h;
  const int nch = D / 8;
  const int nx = (kTB * nch + kCBlock - 1) / kCBlock;      // vectors per thread and block (<= kXR)
  Frag<T> xr[kXR];
  auto load_x = [&](int blk) {
    const int js = j0 + blk * kTB;
#pragma unroll
    for (int i = 0; i < kXR; ++i) {
      if (i < nx) {
        const int it = tid + i * kCBlock;
        const int jt = it / nch, ch = it % nch;
        const int j = min(js + min(jt, kTB - 1), p.N - 1);
        load8(xbase + static_cast<int64_t>(j) * p.sx_n + ch * 8, xr[i]);
      }
    }
  };
  load_x(0);

  // ---- dimension ranks: >= 0 index among kept dims, < 0: -(1 + index among compressed) ------
  {
    uint8_t mb[4];
#pragma unroll
    for (int j = 0; j < 4; ++j) mb[j] = p.mask[static_cast<size_t>(bh) * D + min(lane + 64 * j, D - 1)];
    uint64_t bal[4];
#pragma unroll
    for (int j = 0; j < 4; ++j) bal[j] = __ballot(mb[j] != 0 && lane + 64 * j < D);
    if (tid < D) {
      const int w = tid >> 6;
      const uint64_t bit = 1ull << (tid & 63);
      int nc = 0;
      uint64_t hit = 0;
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        const uint64_t below = (j < w) ? ~0ull : ((j == w) ? (bit - 1ull) : 0ull);
        nc += __popcll(bal[j] & below);
        hit |= bal[j] & ((j == w) ? bit : 0ull);
      }
      cpos[tid] = hit ? static_cast<int16_t>(-(1 + nc)) : static_cast<int16_t>(tid - nc);
    }
  }
  // unused columns / pad columns of the LDS tiles stay zero for the whole kernel
  for (int it = tid; it < static_cast<int>(2 * bufe * sizeof(T) / 16); it += kCBlock)
    reinterpret_cast<u32x4*>(smem)[it] = u32x4{0u, 0u, 0u, 0u};

  // ---- per-wave constants: E fragments (A operand) and frame twiddles -------------------
  const int rows_here = 2 * min(kPairs, p.nmax - mc * kPairs);   // live basis rows of this row block
  const int rgw = wave & 3, chw = wave >> 2;       // row group (64 basis rows), column half of this wave
  const int cols_here = min(kCols, p.Dc - dc * kCols);
  const int ndt = (cols_here + 15) / 16 - chw * DT;   // live column tiles of this wave (may be <= 0)
  const bool wave_live = project && rgw * 64 < rows_here && ndt > 0;

  Frag<T> ea[4][2];          // [m tile][32-token half]
  Frag<T> el[kSplit ? 4 : 1][2];   // remainders of the split basis
  float twc[4][2], tws[4][2];   // cos/sin(omega_n * 64) of the two pairs a lane owns in every m tile
  const uint32_t ph_blk = fixed_phase(kTB, p.ph_scale);   // 64 positions, as a 2^-32-turn phase
  if (wave_live) {
    const float invT = 1.0f / static_cast<float>(p.T);
#pragma unroll
    for (int mt = 0; mt < 4; ++mt) {
      const int rho = rgw * 64 + mt * 16 + r16;               // A-operand row of this lane
      const int n = mc * kPairs + (rho >> 1) + 1;
      const bool live = n <= p.nmax;
#pragma unroll
      for (int ksx = 0; ksx < 2; ++ksx) {
        const int u0 = 32 * ksx + 8 * q4;
#pragma unroll
        for (int e = 0; e < 8; ++e) {
          float c, sn;
          if constexpr (sizeof(T) == 4) {
            unit_phase(n, u0 + e, p.T, &c, &sn);
          } else {
            // n * u < 2^24: the float quotient estimate is exact to +-1
            const int prod = n * (u0 + e);
            int ph = prod - static_cast<int>(static_cast<float>(prod) * invT) * p.T;
            if (ph < 0) ph += p.T;
            if (ph >= p.T) ph -= p.T;
            const float x = static_cast<float>(ph) * invT;
            sn = __builtin_amdgcn_sinf(x);
            c = __builtin_amdgcn_cosf(x);
          }
          const float val = live ? ((rho & 1) ? sn : c) : 0.0f;
          set_elem<T>(ea[mt][ksx], e, val);
          if constexpr (kSplit) {
            const float head = bf16_to_f32(f32_to_bf16(val));
            set_elem<T>(el[mt][ksx], e, val - head);
          }
        }
      }
#pragma unroll
      for (int pr = 0; pr < 2; ++pr) {
        const int n2 = mc * kPairs + ((rgw * 64 + mt * 16 + 4 * q4) >> 1) + pr + 1;   // accumulator rows 4*q4 + 2*pr
        fixed_phase_cs<T>(static_cast<uint32_t>(n2) * ph_blk, &twc[mt][pr], &tws[mt][pr]);
      }
    }
  }

  f32x4 acc[4][DT];
#pragma unroll
  for (int mt = 0; mt < 4; ++mt)
#pragma unroll
    for (int dt = 0; dt < DT; ++dt) acc[mt][dt] = f32x4{0.f, 0.f, 0.f, 0.f};
  float dcs = 0.0f;   // column sum of this thread's (column, token half)

  T* keep = static_cast<T*>(p.keep) + static_cast<int64_t>(bh) * p.keep_stride;
  const int kp = p.keep_pitch;
  __syncthreads();   // cpos and the zero fills are visible

  // Where each of a thread's 8 dims goes inside a buffer is decided once (kFast).
  const int tstride = kCBlock / nch;            // tokens between a thread's consecutive vectors
  uint32_t sc_off[8], sc_step[8];               // byte offset inside a buffer, step per vector
  if constexpr (kFast) {
    const int ch = tid % nch, jt0 = tid / nch;
    const uint32_t es = sizeof(T);
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      const int cp = cpos[ch * 8 + e];
      const int rank = -cp - 1 - dc * kCols;
      if (cp < 0 && rank >= 0 && rank < kCols) {
        sc_off[e] = (rank * kLdX + jt0) * es;
        sc_step[e] = tstride * es;
      } else if (cp >= 0 && stage) {
        const bool rows = p.keep_layout == FA_KEEP_ROWS;
        sc_off[e] = (kCols * kLdX + (rows ? jt0 * (kp + 8) + cp : cp * kLdX + jt0)) * es;
        sc_step[e] = (rows ? tstride * (kp + 8) : tstride) * es;
      } else {
        sc_off[e] = (kCols * kLdX + p.ks_elems) * es;   // spare slot: the value is not needed here
        sc_step[e] = 0;
      }
    }
  }

  for (int blk = 0; blk < nb; ++blk) {
    const int buf = blk & 1;
    const int js = j0 + blk * kTB;
    T* xcb = lds + buf * bufe;
    T* ksb = xcb + kCols * kLdX;

    // -- scatter the block held in registers: compressed columns transposed, kept ones staged
    if constexpr (kFast) {
      const bool ragged = js + kTB > jend;
      unsigned char* bb = reinterpret_cast<unsigned char*>(xcb);
#pragma unroll
      for (int i = 0; i < kXR; ++i) {
        if (i < nx) {
          const bool valid = !ragged || js + tid / nch + i * tstride < jend;
#pragma unroll
          for (int e = 0; e < 8; ++e) {
            const T val = valid ? felem(xr[i], e) : zero_elem(lds);
            *reinterpret_cast<T*>(bb + sc_off[e] + i * sc_step[e]) = val;
          }
        }
      }
    } else {
#pragma unroll
      for (int i = 0; i < kXR; ++i) {
        if (i < nx) {
          const int it = tid + i * kCBlock;
          const int jt = it / nch, ch = it % nch;
          const bool valid = jt < kTB && js + jt < jend;
          if (jt < kTB) {
#pragma unroll
            for (int e = 0; e < 8; ++e) {
              const int cp = cpos[ch * 8 + e];
              const T val = valid ? felem(xr[i], e) : zero_elem(lds);
              if (cp < 0) {
                const int rank = -cp - 1 - dc * kCols;
                if (rank >= 0 && rank < kCols) xcb[rank * kLdX + jt] = val;
              } else if (stage) {
                if (p.keep_layout == FA_KEEP_ROWS) ksb[jt * (kp + 8) + cp] = val;
                else ksb[cp * kLdX + jt] = val;
              } else if (write_keep && valid) {
                const int64_t tok = static_cast<int64_t>(p.keep_offset) + js + jt;
                const int64_t off = (p.keep_layout == FA_KEEP_ROWS) ? tok * kp + cp
                                                                    : ((tok >> 3) * Du + cp) * 8 + (tok & 7);
                keep[off] = val;
              }
            }
          }
        }
      }
    }
    if (write_keep && !stage && p.keep_layout == FA_KEEP_ROWS && kp > Du) {
      const int npad = kp - Du;   // zero pad columns of the rows layout
      for (int it = tid; it < kTB * npad; it += kCBlock) {
        const int j = js + it / npad;
        if (j < jend) keep[(static_cast<int64_t>(p.keep_offset) + j) * kp + Du + it % npad] = zero_elem(keep);
      }
    }
    // -- the next block travels while this one is multiplied
    if (blk + 1 < nb) load_x(blk + 1);
    __syncthreads();

    // -- kept dims: staging tile -> 128-bit stores
    if (stage) {
      const int64_t tok0 = static_cast<int64_t>(p.keep_offset) + js;
      if (p.keep_layout == FA_KEEP_ROWS) {
        const int c8n = kp / 8;
        for (int it = tid; it < kTB * c8n; it += kCBlock) {
          const int jt = it / c8n, c8 = it % c8n;
          if (js + jt < jend) {
            Frag<T> f;
            f.load(ksb + jt * (kp + 8) + 8 * c8);
            *reinterpret_cast<Frag<T>*>(keep + (tok0 + jt) * kp + 8 * c8) = f;
          }
        }
      } else {
        for (int it = tid; it < Du * (kTB / 8); it += kCBlock) {
          const int dim = it / (kTB / 8), g = it % (kTB / 8);
          if (js + 8 * g < jend) {
            Frag<T> f;
            f.load(ksb + dim * kLdX + 8 * g);
            *reinterpret_cast<Frag<T>*>(keep + (((tok0 >> 3) + g) * Du + dim) * 8) = f;
          }
        }
      }
    }
    // -- constant function: column sums
    if (do_dc) {
      const int col = tid & (kCols - 1), th = tid / kCols;   // four token quarters per column
#pragma unroll
      for (int g = 0; g < 2; ++g) {
        Frag<T> f;
        f.load(xcb + col * kLdX + 16 * th + 8 * g);
#pragma unroll
        for (int e = 0; e < 8; ++e) dcs += tof(felem(f, e));
      }
    }
    // -- harmonics: move the frame to this block, then accumulate E * X_blk
    if (wave_live) {
      if (blk > 0) {
#pragma unroll
        for (int mt = 0; mt < 4; ++mt)
#pragma unroll
          for (int pr = 0; pr < 2; ++pr) {
            const float c = twc[mt][pr], sn = tws[mt][pr];
#pragma unroll
            for (int dt = 0; dt < DT; ++dt) {
              const float ac = acc[mt][dt][2 * pr], as = acc[mt][dt][2 * pr + 1];
              acc[mt][dt][2 * pr] = c * ac + sn * as;
              acc[mt][dt][2 * pr + 1] = c * as - sn * ac;
            }
          }
      }
#pragma unroll
      for (int dt = 0; dt < DT; ++dt) {
        if (dt < ndt) {
#pragma unroll
          for (int ksx = 0; ksx < 2; ++ksx) {
            Frag<T> bx;
            bx.load(xcb + ((chw * DT + dt) * 16 + r16) * kLdX + 32 * ksx + 8 * q4);
#pragma unroll
            for (int mt = 0; mt < 4; ++mt) {
              mma_k32(acc[mt][dt], ea[mt][ksx], bx);
              if constexpr (kSplit) mma_k32(acc[mt][dt], el[mt][ksx], bx);
            }
          }
        }
      }
    }
  }

  // ---- epilogue -----------------------------------------------------------------------------
  if (!project) return;
  float* dst = (p.Sc == 1) ? p.coeffs + static_cast<size_t>(bh) * M * p.Dc
                           : p.part + static_cast<size_t>(s) * p.part_stride + static_cast<size_t>(bh) * M * p.Dc;
  const bool add = (p.Sc == 1) && p.accumulate;
  if (do_dc) {   // uniform per workgroup
    dcred[tid] = dcs;
    __syncthreads();
    if (tid < kCols) {
      const int i = dc * kCols + tid;
      if (tid < cols_here) {
        const float v = (dcred[tid] + dcred[tid + kCols]) + (dcred[tid + 2 * kCols] + dcred[tid + 3 * kCols]);
        dst[i] = add ? dst[i] + v : v;
      }
    }
  }
  if (wave_live) {
    const uint32_t ph_last = fixed_phase(p.t0 + j0 + (nb - 1) * kTB, p.ph_scale);   // frame origin
#pragma unroll
    for (int mt = 0; mt < 4; ++mt)
#pragma unroll
      for (int pr = 0; pr < 2; ++pr) {
        const int n = mc * kPairs + ((rgw * 64 + mt * 16 + 4 * q4) >> 1) + pr + 1;
        if (n > p.nmax) continue;
        float c, sn;
        fixed_phase_cs<T>(static_cast<uint32_t>(n) * ph_last, &c, &sn);
        const int m_cos = 2 * n - 1, m_sin = 2 * n;
#pragma unroll
        for (int dt = 0; dt < DT; ++dt) {
          const int i = dc * kCols + (chw * DT + dt) * 16 + r16;
          if (dt < ndt && i < p.Dc) {
            const float ac = acc[mt][dt][2 * pr], as = acc[mt][dt][2 * pr + 1];
            const float vc = c * ac - sn * as, vs = sn * ac + c * as;
            float* oc = dst + static_cast<size_t>(m_cos) * p.Dc + i;
            *oc = add ? (*oc + vc) : vc;
            if (m_sin < M) {
              float* os = dst + static_cast<size_t>(m_sin) * p.Dc + i;
              *os = add ? (*os + vs) : vs;
            }
          }
        }
      }
  }
}

// ---------------------------------------------------------------------------
// bf16, head dim 128: blocks of 128 tokens
// ---------------------------------------------------------------------------
// Same decomposition as compress_project, specialised for the common shape.  A thread
// loads 8 dims of 4 consecutive tokens, so that every dim leaves as ONE 64-bit LDS
// write into the transposed tiles (compressed dims: MFMA B operands; kept dims: a
// staging tile in the same [dim][token] layout that serves both output layouts).  Each
// of the 8 waves owns 32 basis rows and all compressed columns; it holds the basis of a
// PAIR of blocks (256 tokens) in registers, so the frame moves once per 256 tokens.  The
// constant function rides on the matrix cores as a row of ones, and all addressing is
// decided before the loop.
constexpr int kSplitTokens = 512;      // bf16 segments up to this length take the split basis
constexpr long kF32ChunkBlocks = 4;    // fp32 inputs: at most this many 128-token blocks per chunk
constexpr int kFB = 128;            // tokens per block
constexpr int kFP = kFB + 8;        // LDS pitch (elements) of a transposed column
constexpr int kFK = kFB / 32;       // 32-token contraction steps per block

__device__ __forceinline__ uint32_t pack_lo(uint32_t a, uint32_t b) {   // (a.lo, b.lo)
  return __builtin_amdgcn_perm(b, a, 0x05040100u);
}
__device__ __forceinline__ uint32_t pack_hi(uint32_t a, uint32_t b) {   // (a.hi, b.hi)
  return __builtin_amdgcn_perm(b, a, 0x07060302u);
}

// KM selects the block step: 0 / 1 / 2 = the straight-line step with no kept dims to write /
// kept dims as rows / kept dims in groups of 8 tokens (at most one 128-bit vector of kept dims
// per thread and block); 3 = 1 or 2 by the call's layout (the K | V pair launch); -1 = the general
// step (any number of kept dims, or nothing to project).
template <int DT, int KM>
__device__ __forceinline__ void project_fast_body(const CompressParams& p, const int bh) {
  using T = bf16_t;
  constexpr int NW = kCBlock / 64;    // 8 waves
  constexpr int kThreads = kCBlock;
  constexpr int MT = 2;               // 16-row basis tiles per wave
  constexpr int CH = 1;               // column groups of DT tiles: every wave multiplies all columns
  constexpr int TOK = 32 / NW;        // consecutive tokens a thread loads: 4
  constexpr int RG = NW / CH;         // row groups of 16 MT = 32 basis rows
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int q4 = lane >> 4, r16 = lane & 15;
  const int s = blockIdx.x, mc = blockIdx.y;
  const int b = bh / p.H, h = bh % p.H;
  constexpr int D = 128;
  const int M = p.M, Du = p.Du, kp = p.keep_pitch;
  const int j0 = s * p.chunk, jend = min(p.N, j0 + p.chunk);
  const int nb = (jend - j0 + kFB - 1) / kFB;
  const bool write_keep = (blockIdx.y == 0) && p.keep != nullptr && Du > 0;
  const bool project = p.Dc > 0;
  const bool do_dc = project && mc == 0;
  const bool rows_layout = p.keep_layout == FA_KEEP_ROWS;

  // two buffers of [compressed columns kCols x kFP | kept dims kp x kFP | 8 spare elements]
  const uint32_t bufb = (kCols * kFP + static_cast<uint32_t>(kp) * kFP + 8) * 2;   // bytes per buffer
  const uint32_t ks_off = kCols * kFP * 2;

  // ---- first X block is requested before anything else --------------------------------
  // 8 dims (vector ch of a row), TOK consecutive tokens (group quad).  Sixteen consecutive lanes
  // hold 4 vectors x 4 token groups: each token's 64 bytes still load as one segment, and the
  // transposed writes of one instruction spread over the LDS banks (16 different columns of
  // one token group would land 8 columns apart on the same banks)
  const int ch = (lane & 3) | ((lane >> 4) << 2), quad = ((lane >> 2) & 3) | (wave << 2);
  const T* xthr = static_cast<const T*>(p.x) + b * p.sx_b + h * p.sx_h + ch * 8;
  Frag<T> xra[TOK], xrb[TOK];   // even / odd blocks: two blocks are in flight
  // Loads are never predicated: a load under a condition is merged with the old register contents
  // right after it, i.e. waited for at once.  Blocks past the chunk re-read its last block and rows
  // past the segment its last row; both are ignored downstream.
  auto load_x = [&](Frag<T> (&xr)[TOK], int blk) {
    const int js = j0 + min(blk, nb - 1) * kFB + TOK * quad;
#pragma unroll
    for (int i = 0; i < TOK; ++i) xr[i].load(xthr + static_cast<int64_t>(min(js + i, p.N - 1)) * p.sx_n);
  };
  // the mask row first (it is waited for first), then the first two X blocks
  uint8_t mb[2];
#pragma unroll
  for (int j = 0; j < 2; ++j) mb[j] = p.mask[static_cast<size_t>(bh) * D + lane + 64 * j];
  load_x(xra, 0);
  load_x(xrb, 1);

  // ---- per-wave constants: E fragments (A operand) and frame twiddles -------------------
  const int rows_here = 2 * min(kPairs, p.nmax - mc * kPairs);   // live basis rows of this row block
  const int rgw = wave % RG, chw = wave / RG;      // row group (16 MT basis rows), column group (always 0 for CH = 1)
  const int ndt = (p.Dc + 15) / 16 - chw * DT;     // live column tiles of this wave (may be <= 0)
  const bool wave_live = project && rgw * 16 * MT < rows_here && ndt > 0;
  const bool wave_dc = do_dc && rgw < ndt && rgw < DT;   // this wave sums column tile rgw

  // Two basis sets: tokens 0..127 and 128..255 of a pair of blocks.  The frame then moves once per
  // PAIR of blocks (by 256 tokens), which halves the turning arithmetic per token.
  Frag<T> ea[2][MT][kFK];          // [block of the pair][m tile][32-token step]
  float twc[MT][2], tws[MT][2];    // cos/sin(omega_n * 256) of the two pairs a lane owns in every m tile
  const uint32_t ph_blk = fixed_phase(2 * kFB, p.ph_scale);
  if (wave_live) {
    // phase of token u as a 2^-32-turn fixed-point number; times n it wraps exactly, and the
    // rounding of the unit (< 2^-32 turn) grows to at most n * 2^-32 turn: far below a bf16 ulp
    const uint32_t ph_1 = fixed_phase(1, p.ph_scale);
    uint32_t ph_u[2 * kFK];
#pragma unroll
    for (int ksx = 0; ksx < 2 * kFK; ++ksx) ph_u[ksx] = fixed_phase(32 * ksx + 8 * q4, p.ph_scale);
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) {
      const int rho = rgw * 16 * MT + mt * 16 + r16;               // A-operand row of this lane
      const int n = mc * kPairs + (rho >> 1) + 1;
      const bool live = n <= p.nmax;
      // A lane needs ONE sequence per 32-token step: cos (even row) or sin (odd row) of 8
      // consecutive tokens.  Two evaluations start it; the rest follows from the three-term
      // recurrence v[e+1] = 2 cos(step) v[e] - v[e-1], written in differences
      //   d[e+1] = d[e] - kappa v[e],  v[e+1] = v[e] + d[e+1],  kappa = 4 sin^2(step / 2),
      // which keeps its accuracy for the tiny steps of low harmonics (2 cos(step) would round
      // to 2).  Over 8 steps the rounding stays far below a bf16 ulp.
      const uint32_t stepn = static_cast<uint32_t>(n) * ph_1;   // <= half a turn: n <= T / 2
      const uint32_t quarter = (rho & 1) ? 0x40000000u : 0u;    // sin x = cos(x - 1/4 turn)
      const float sh = sinpif(static_cast<float>(stepn) * 2.3283064365386963e-10f);   // sin(step / 2)
      const float kappa = 4.0f * sh * sh;
#pragma unroll
      for (int ksx = 0; ksx < 2 * kFK; ++ksx) {
        const uint32_t ph0 = static_cast<uint32_t>(n) * ph_u[ksx] - quarter;
        float vals[8];
        vals[0] = __builtin_amdgcn_cosf(static_cast<float>(static_cast<int32_t>(ph0)) * 2.3283064365386963e-10f);
        vals[1] = __builtin_amdgcn_cosf(static_cast<float>(static_cast<int32_t>(ph0 + stepn)) * 2.3283064365386963e-10f);
        if (!live) vals[0] = vals[1] = 0.0f;   // rows past the highest harmonic: the recurrence keeps them zero
        float dv = vals[1] - vals[0];
#pragma unroll
        for (int e = 2; e < 8; ++e) {
          dv -= kappa * vals[e - 1];
          vals[e] = vals[e - 1] + dv;
        }
#pragma unroll
        for (int e = 0; e < 4; ++e)
          ea[ksx / kFK][mt][ksx % kFK].v[e] =
              __builtin_bit_cast(uint32_t, __builtin_convertvector(f32x2c{vals[2 * e], vals[2 * e + 1]}, bf16x2c));
      }
#pragma unroll
      for (int pr = 0; pr < 2; ++pr) {
        const int n2 = mc * kPairs + ((rgw * 16 * MT + mt * 16 + 4 * q4) >> 1) + pr + 1;   // accumulator rows 4*q4 + 2*pr
        fixed_phase_cs<T>(static_cast<uint32_t>(n2) * ph_blk, &twc[mt][pr], &tws[mt][pr]);
      }
    }
  }
  // ---- dimension ranks, wave-local (no LDS, no barrier): the mask bits of all 128 dims sit in two
  // ballots; a lane's 8 dims are consecutive, so one byte of a ballot holds their bits and the
  // rank of its first dim is a population count below it
  uint32_t sc_off[8];   // where each of the thread's 8 dims goes inside a buffer (bytes)
  {
    const uint64_t bal0 = __ballot(mb[0] != 0), bal1 = __ballot(mb[1] != 0);
    const int d0 = ch * 8;                                   // first dim of this lane
    const uint64_t word = d0 < 64 ? bal0 : bal1;
    const uint32_t bits = static_cast<uint32_t>(word >> (d0 & 63)) & 0xffu;
    const int below0 = __popcll(word & ((1ull << (d0 & 63)) - 1ull)) + (d0 < 64 ? 0 : __popcll(bal0));
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      const int nc = below0 + __popc(bits & ((1u << e) - 1u));   // compressed dims below dim d0 + e
      const bool hit = (bits >> e) & 1u;
      if (hit) sc_off[e] = (static_cast<uint32_t>(nc) * kFP + TOK * quad) * 2;
      else if (write_keep) sc_off[e] = ks_off + (static_cast<uint32_t>(d0 + e - nc) * kFP + TOK * quad) * 2;
      else sc_off[e] = ks_off + static_cast<uint32_t>(kp) * kFP * 2;   // spare slot: the value is not needed
    }
  }
  // The pad rows of the kept-dim staging tiles (dims Du .. kp-1, which leave as the zero pad of the
  // rows layout) are zero for the whole kernel.  Nothing else needs clearing: every token of a used
  // column is written before it is read, and columns past Dc only feed accumulator columns that
  // are never stored (a matrix product keeps columns apart).
  {
    const uint32_t pad_words = static_cast<uint32_t>(kp - Du) * kFP / 2;   // 32-bit words per buffer
    for (uint32_t it = tid; it < 2 * pad_words; it += kThreads) {
      const uint32_t bsel = it >= pad_words ? 1u : 0u;
      reinterpret_cast<uint32_t*>(smem + bsel * bufb + ks_off + static_cast<uint32_t>(Du) * kFP * 2)[it - bsel * pad_words] = 0u;
    }
  }

  Frag<T> ones;
  ones.v = u32x4{0x3f803f80u, 0x3f803f80u, 0x3f803f80u, 0x3f803f80u};

  f32x4 acc[MT][DT];
#pragma unroll
  for (int mt = 0; mt < MT; ++mt)
#pragma unroll
    for (int dt = 0; dt < DT; ++dt) acc[mt][dt] = f32x4{0.f, 0.f, 0.f, 0.f};
  f32x4 acc_dc = {0.f, 0.f, 0.f, 0.f};   // rows are identical: the column sums of tile rgw

  T* keep = static_cast<T*>(p.keep) + static_cast<int64_t>(bh) * p.keep_stride;
  // (no barrier here: the first scatter touches no pad row, and the barrier after it also orders
  // the zero fill before the first read of the staging tile)
  // ---- kept dims leave the staging tile as 128-bit stores: one or more vectors per thread ------
  // rows layout: vector (token jt, 8 dims 8 c8..): gathered from 8 tile rows; tok8 layout: vector
  // (dim, 8 tokens 8 g..): contiguous in the tile
  const int nvec = rows_layout ? kFB * (kp / 8) : Du * (kFB / 8);
  const int c8n = max(kp / 8, 1), dun = max(Du, 1);
  const int kv_0 = max(min(tid, nvec - 1), 0);                   // first vector of this thread
  // (division by the layout's vectors per token / dims per group through the host's 16-bit reciprocal:
  // exact for indices below 512 and divisors up to 64)
  const int kv_d = rows_layout ? c8n : dun;
  int kv_a;   // token (rows) or 8-token group (tok8)
  if constexpr (KM >= 0) kv_a = static_cast<int>((static_cast<uint32_t>(kv_0) * p.kv_magic) >> 16);   // (one vector per thread: d <= 32)
  else kv_a = kv_0 / kv_d;
  const int kv_b = kv_0 - kv_a * kv_d;                           // 8-dim group (rows) or dim (tok8)

  auto scatter_block = [&](Frag<T> (&xr)[TOK], int blk) {   // this thread's 4 tokens x 8 dims of block blk -> LDS
    const int js = j0 + blk * kFB;
    unsigned char* bb = smem + (blk & 1) * bufb;
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      const int w = e >> 1;
      uint32_t lo, hi;
      if (e & 1) {
        lo = pack_hi(xr[0].v[w], xr[1].v[w]);
        hi = pack_hi(xr[2].v[w], xr[3].v[w]);
      } else {
        lo = pack_lo(xr[0].v[w], xr[1].v[w]);
        hi = pack_lo(xr[2].v[w], xr[3].v[w]);
      }
      *reinterpret_cast<u32x2c*>(bb + sc_off[e]) = u32x2c{lo, hi};
    }
    if (js + kFB > jend) {   // ragged last block: tokens past the end count as zeros (written over)
#pragma unroll
      for (int i = 0; i < TOK; ++i)
        if (js + TOK * quad + i >= jend) {
#pragma unroll
          for (int e = 0; e < 8; ++e) *reinterpret_cast<uint16_t*>(bb + sc_off[e] + 2 * i) = 0;
        }
    }
  };
  auto keep_out = [&](int blk) {   // kept dims of block blk: staging tile -> 128-bit stores (general step)
    const int js = j0 + blk * kFB;
    const T* ks = reinterpret_cast<const T*>(smem + (blk & 1) * bufb + ks_off);
    const int64_t tok0 = static_cast<int64_t>(p.keep_offset) + js;
    const int it0 = tid;
    if (rows_layout) {
      for (int it = it0; it < nvec; it += kThreads) {
        const int jt = (it == it0) ? kv_a : it / c8n, c8 = (it == it0) ? kv_b : it - (it / c8n) * c8n;
        if (js + jt < jend) {
          const uint16_t* src = reinterpret_cast<const uint16_t*>(ks) + (8 * c8) * kFP + jt;
          u32x4 v;
#pragma unroll
          for (int k = 0; k < 4; ++k)
            v[k] = static_cast<uint32_t>(src[(2 * k) * kFP]) | (static_cast<uint32_t>(src[(2 * k + 1) * kFP]) << 16);
          *reinterpret_cast<u32x4*>(keep + (tok0 + jt) * kp + 8 * c8) = v;
        }
      }
    } else {
      for (int it = it0; it < nvec; it += kThreads) {
        const int g = (it == it0) ? kv_a : it / dun, dim = (it == it0) ? kv_b : it - (it / dun) * dun;
        if (js + 8 * g < jend) {
          Frag<T> f;
          f.load(ks + dim * kFP + 8 * g);
          *reinterpret_cast<Frag<T>*>(keep + (((tok0 >> 3) + g) * Du + dim) * 8) = f;
        }
      }
    }
  };
  auto multiply_block = [&](int blk, auto odd_c) {
    constexpr int kOdd = decltype(odd_c)::value;   // second block of a pair: second basis set, no turn
    if (!wave_live && !wave_dc) return;
    const T* xcb = reinterpret_cast<const T*>(smem + (blk & 1) * bufb);
    const T* bcol = xcb + (chw * DT * 16 + r16) * kFP + 8 * q4;   // this lane's column in tile 0
    // The B operands of column tile dt + 1 are requested before the products of tile dt are
    // issued, and the turn of the frame runs while the first tile's operands travel.
    Frag<T> bxa[kFK], bxb[kFK];
#pragma unroll
    for (int ksx = 0; ksx < kFK; ++ksx) bxa[ksx].load(bcol + 32 * ksx);
    if (wave_live && !kOdd) {
      // (also for the first block: the accumulators are zero then, and an unconditional turn keeps
      // them in place in their registers)
#pragma unroll
      for (int mt = 0; mt < MT; ++mt)
#pragma unroll
        for (int pr = 0; pr < 2; ++pr) {
          const float c = twc[mt][pr], sn = tws[mt][pr];
#pragma unroll
          for (int dt = 0; dt < DT; ++dt) {
            const float ac = acc[mt][dt][2 * pr], as = acc[mt][dt][2 * pr + 1];
            acc[mt][dt][2 * pr] = c * ac + sn * as;
            acc[mt][dt][2 * pr + 1] = c * as - sn * ac;
          }
        }
    }
#pragma unroll
    for (int dt = 0; dt < DT; ++dt) {
      Frag<T> (&cur)[kFK] = (dt & 1) ? bxb : bxa;
      Frag<T> (&nxt)[kFK] = (dt & 1) ? bxa : bxb;
      if (dt + 1 < DT) {   // (tiles past the last compressed column are zero-filled, never written)
#pragma unroll
        for (int ksx = 0; ksx < kFK; ++ksx) nxt[ksx].load(bcol + (dt + 1) * 16 * kFP + 32 * ksx);
      }
      __builtin_amdgcn_sched_barrier(0);
      if (wave_live && dt < ndt) {
#pragma unroll
        for (int ksx = 0; ksx < kFK; ++ksx)
#pragma unroll
          for (int mt = 0; mt < MT; ++mt) mma_k32(acc[mt][dt], ea[kOdd][mt][ksx], cur[ksx]);
      }
      // constant function: a row of ones against column tile rgw
      if (wave_dc && dt == rgw) {
#pragma unroll
        for (int ksx = 0; ksx < kFK; ++ksx) mma_k32(acc_dc, ones, cur[ksx]);
      }
      __builtin_amdgcn_sched_barrier(0);
    }
  };
  // One straight-line pass over block blk for a wave with live basis rows: the products of block
  // blk, the scatter of block blk + 1 (into the other buffer) and the kept dims of block blk leave
  // in ONE instruction stream without branches, so that the scatter and the frame turn issue in
  // the shadow of the matrix instructions.  Ragged edges are handled by value: tokens past the
  // chunk are masked to zero, vectors past the end re-store the last valid one.
  const int dcl = min(rgw, DT - 1);   // column tile whose sums this wave forms (used if wave_dc)
  auto fused_step = [&](Frag<T> (&xnext)[TOK], int blk, auto odd_c, auto mode_c) {
    constexpr int kOdd = decltype(odd_c)::value;   // second block of a pair: second basis set, no turn
    constexpr int kMode = decltype(mode_c)::value;   // kept dims: 0 none to write, 1 rows, 2 groups of 8 tokens
    const int js = j0 + blk * kFB;
    const unsigned char* cb = smem + (blk & 1) * bufb;
    unsigned char* fb = smem + ((blk & 1) ^ 1) * bufb;
    const T* bcol = reinterpret_cast<const T*>(cb) + (chw * DT * 16 + r16) * kFP + 8 * q4;
    Frag<T> bxa[kFK], bxb[kFK];
#pragma unroll
    for (int ksx = 0; ksx < kFK; ++ksx) bxa[ksx].load(bcol + 32 * ksx);
    // kept dims of block blk: out of the staging tile
    u32x4 kvv = {0u, 0u, 0u, 0u};
    T* kdst = keep;
    if (kMode == 1 || (kMode == 3 && rows_layout)) {   // (kMode 3: decided per launch half, a uniform branch)
      const int jt = max(min(kv_a, jend - js - 1), 0);
      const uint16_t* src = reinterpret_cast<const uint16_t*>(cb + ks_off) + (8 * kv_b) * kFP + jt;
#pragma unroll
      for (int k = 0; k < 4; ++k)
        kvv[k] = static_cast<uint32_t>(src[(2 * k) * kFP]) | (static_cast<uint32_t>(src[(2 * k + 1) * kFP]) << 16);
      kdst = keep + (static_cast<int64_t>(p.keep_offset) + js + jt) * kp + 8 * kv_b;
    } else if (kMode == 2 || kMode == 3) {
      const int g = max(min(kv_a, (jend - js - 1) >> 3), 0);
      kvv = *reinterpret_cast<const u32x4*>(reinterpret_cast<const T*>(cb + ks_off) + kv_b * kFP + 8 * g);
      kdst = keep + ((((static_cast<int64_t>(p.keep_offset) + js) >> 3) + g) * Du + kv_b) * 8;
    }
    // the frame turns by 128 tokens (also before the first block: the accumulators are zero then);
    // tile dt + 1 turns while tile dt is multiplied
    auto turn = [&](int dt) {
#pragma unroll
      for (int mt = 0; mt < MT; ++mt)
#pragma unroll
        for (int pr = 0; pr < 2; ++pr) {
          const float c = twc[mt][pr], sn = tws[mt][pr];
          const float ac = acc[mt][dt][2 * pr], as = acc[mt][dt][2 * pr + 1];
          acc[mt][dt][2 * pr] = c * ac + sn * as;
          acc[mt][dt][2 * pr + 1] = c * as - sn * ac;
        }
    };
    // this thread's tokens of block blk + 1, zeros past the end of the chunk
    const int left = jend - (js + kFB) - TOK * quad;
    uint32_t vm[TOK / 2];
#pragma unroll
    for (int i = 0; i < TOK / 2; ++i)
      vm[i] = (left > 2 * i ? 0x0000ffffu : 0u) | (left > 2 * i + 1 ? 0xffff0000u : 0u);
    auto scatter_dim = [&](int e) {
      const int w = e >> 1;
      uint32_t pk[TOK / 2];
#pragma unroll
      for (int i = 0; i < TOK / 2; ++i)
        pk[i] = ((e & 1) ? pack_hi(xnext[2 * i].v[w], xnext[2 * i + 1].v[w])
                         : pack_lo(xnext[2 * i].v[w], xnext[2 * i + 1].v[w])) & vm[i];
      *reinterpret_cast<u32x2c*>(fb + sc_off[e]) = u32x2c{pk[0], pk[1]};
    };
    if constexpr (!kOdd) turn(0);
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int dt = 0; dt < DT; ++dt) {
      Frag<T> (&cur)[kFK] = (dt & 1) ? bxb : bxa;
      Frag<T> (&nxt)[kFK] = (dt & 1) ? bxa : bxb;
      // next tile's operands; after the last tile the tile whose column sums this wave forms
      const T* nsrc = bcol + ((dt + 1 < DT) ? (dt + 1) * 16 * kFP : dcl * 16 * kFP);
#pragma unroll
      for (int ksx = 0; ksx < kFK; ++ksx) nxt[ksx].load(nsrc + 32 * ksx);
      if constexpr (!kOdd) {
        if (dt + 1 < DT) turn(dt + 1);
      }
      if (dt == 0) {
        // the whole scatter rides on the first tile, so that the registers can be refilled at once:
        // the block after next is requested a full block and a half before its turn
#pragma unroll
        for (int e = 0; e < 8; ++e) scatter_dim(e);
        load_x(xnext, blk + 3);
      }
#pragma unroll
      for (int ksx = 0; ksx < kFK; ++ksx)
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) mma_k32(acc[mt][dt], ea[kOdd][mt][ksx], cur[ksx]);
#pragma unroll
      for (int i = 0; i < MT * kFK; ++i) {
        __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);   // one matrix instruction,
        __builtin_amdgcn_sched_group_barrier(0x002, 3, 0);   // three vector instructions,
        __builtin_amdgcn_sched_group_barrier(0x300, 1, 0);   // one LDS access
      }
      __builtin_amdgcn_sched_barrier(0);
    }
    {
      Frag<T> (&dcx)[kFK] = (DT & 1) ? bxb : bxa;
#pragma unroll
      for (int ksx = 0; ksx < kFK; ++ksx) mma_k32(acc_dc, ones, dcx[ksx]);
    }
    if constexpr (kMode > 0) {
      if (write_keep && blk < nb) __builtin_nontemporal_store(kvv, reinterpret_cast<u32x4*>(kdst));   // streamed: nobody reads it soon
    }
  };
  auto two_slots = [&](Frag<T> (&xnext)[TOK], int blk, auto odd_c) {   // block blk; xnext holds block blk + 1
    if constexpr (KM >= 0) {
      fused_step(xnext, blk, odd_c, std::integral_constant<int, KM>{});
    } else {
      multiply_block(blk, odd_c);
      if (blk + 1 < nb) scatter_block(xnext, blk + 1);
      if (write_keep) keep_out(blk);
    }
    __syncthreads();
  };
  // Loads are issued where every wave passes, never under a condition (the result would have to be
  // merged with the other path, i.e. waited for at once): as soon as a register set has been
  // scattered, the block two ahead is requested into it.
  scatter_block(xra, 0);
  load_x(xra, 2);
  __syncthreads();
  if constexpr (KM >= 0) {
    // blocks go in pairs without a branch in between; an odd chunk ends with a block of zeros
    // (the scatter past the chunk writes zeros), which only turns the frame once more
    for (int blk = 0; blk < nb; blk += 2) {
      two_slots(xrb, blk, std::integral_constant<int, 0>{});
      two_slots(xra, blk + 1, std::integral_constant<int, 1>{});
    }
  } else {
    for (int blk = 0; blk < nb; blk += 2) {
      two_slots(xrb, blk, std::integral_constant<int, 0>{});
      load_x(xrb, blk + 3);
      if (blk + 1 < nb) two_slots(xra, blk + 1, std::integral_constant<int, 1>{});
      load_x(xra, blk + 4);
    }
  }

  // ---- epilogue -----------------------------------------------------------------------------
  if (!project) return;
  float* dst = (p.Sc == 1) ? p.coeffs + static_cast<size_t>(bh) * M * p.Dc
                           : p.part + static_cast<size_t>(s) * p.part_stride + static_cast<size_t>(bh) * M * p.Dc;
  const bool add = (p.Sc == 1) && p.accumulate;
  if (wave_dc && q4 == 0) {
    const int i = (chw * DT + rgw) * 16 + r16;
    if (i < p.Dc) dst[i] = add ? dst[i] + acc_dc[0] : acc_dc[0];
  }
  if (wave_live) {
    // the frame's origin is the first block of the last pair (an odd chunk of the straight-line
    // step ends with a block of zeros, which belongs to the last pair)
    const int last_even = (nb - 1) & ~1;
    const uint32_t ph_last = fixed_phase(p.t0 + j0 + last_even * kFB, p.ph_scale);
    // Rows whose length is a multiple of 4 leave as 128-bit stores: a lane owns 4 ROWS of one column,
    // so each 16-row tile set goes through a wave-private piece of LDS (the token tiles are done
    // with) and comes back as 4 consecutive columns of one row per lane.
    if ((p.Dc & 3) == 0 && !add) {
      constexpr int P = DT * 16 + 4;   // floats per LDS row: keeps the 4-row groups of a write on distinct banks
      float* ep = reinterpret_cast<float*>(smem) + wave * (16 * P);
#pragma unroll
      for (int mt = 0; mt < MT; ++mt) {
#pragma unroll
        for (int pr = 0; pr < 2; ++pr) {
          const int n = mc * kPairs + ((rgw * 16 * MT + mt * 16 + 4 * q4) >> 1) + pr + 1;
          float c, sn;
          fixed_phase_cs<T>(static_cast<uint32_t>(n) * ph_last, &c, &sn);   // (rows past the highest harmonic are not stored)
#pragma unroll
          for (int dt = 0; dt < DT; ++dt) {
            const float ac = acc[mt][dt][2 * pr], as = acc[mt][dt][2 * pr + 1];
            ep[(4 * q4 + 2 * pr) * P + dt * 16 + r16] = c * ac - sn * as;
            ep[(4 * q4 + 2 * pr + 1) * P + dt * 16 + r16] = sn * ac + c * as;
          }
        }
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");   // this wave's LDS writes before its reads
        __builtin_amdgcn_wave_barrier();
#pragma unroll
        for (int k = 0; k < DT; ++k) {   // 16 rows x 4 DT vectors = DT per lane
          const int v = lane + 64 * k;
          const int row = v / (DT * 4), c4 = v - row * (DT * 4);
          const int rho = rgw * 16 * MT + mt * 16 + row;
          const int n = mc * kPairs + (rho >> 1) + 1;
          const int m = (rho & 1) ? 2 * n : 2 * n - 1;
          const f32x4 val = *reinterpret_cast<const f32x4*>(ep + row * P + 4 * c4);
          if (n <= p.nmax && m < M && 4 * c4 < p.Dc)
            *reinterpret_cast<f32x4*>(dst + static_cast<size_t>(m) * p.Dc + 4 * c4) = val;
        }
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
        __builtin_amdgcn_wave_barrier();
      }
      return;
    }
#pragma unroll
    for (int mt = 0; mt < MT; ++mt)
#pragma unroll
      for (int pr = 0; pr < 2; ++pr) {
        const int n = mc * kPairs + ((rgw * 16 * MT + mt * 16 + 4 * q4) >> 1) + pr + 1;
        if (n > p.nmax) continue;
        float c, sn;
        fixed_phase_cs<T>(static_cast<uint32_t>(n) * ph_last, &c, &sn);
        const int m_cos = 2 * n - 1, m_sin = 2 * n;
#pragma unroll
        for (int dt = 0; dt < DT; ++dt) {
          const int i = (chw * DT + dt) * 16 + r16;
          if (dt < ndt && i < p.Dc) {
            const float ac = acc[mt][dt][2 * pr], as = acc[mt][dt][2 * pr + 1];
            const float vc = c * ac - sn * as, vs = sn * ac + c * as;
            float* oc = dst + static_cast<size_t>(m_cos) * p.Dc + i;
            *oc = add ? (*oc + vc) : vc;
            if (m_sin < M) {
              float* os = dst + static_cast<size_t>(m_sin) * p.Dc + i;
              *os = add ? (*os + vs) : vs;
            }
          }
        }
      }
  }
}

template <int DT, int KM>
__global__ __launch_bounds__(kCBlock) void compress_project_fast(CompressParams p) {
  project_fast_body<DT, KM>(p, blockIdx.z);
}

// K and V of the same tokens in one launch: grid z covers the (sequence, head) pairs of K, then
// those of V; each half runs with its own arguments
struct CompressParamsKV {
  CompressParams k, v;
};
template <int DT>
__global__ __launch_bounds__(kCBlock) void compress_project_fast_kv(CompressParamsKV pp) {
  const int BH = pp.k.B * pp.k.H;
  const bool second = static_cast<int>(blockIdx.z) >= BH;
  const CompressParams& p = second ? pp.v : pp.k;
  project_fast_body<DT, 3>(p, static_cast<int>(blockIdx.z) - (second ? BH : 0));
}

// Sum of the token-chunk partials of four consecutive coefficients, in chunk order (reproducible) and
// in fp64: the partials of a slow out-of-band tone are individually large and cancel, and an fp32
// running sum over many chunks would lose what the chunks themselves resolved.
__device__ __forceinline__ void reduce_chunks(const float* part, float* coeffs, size_t total, size_t stride,
                                              int Sc, int accumulate, size_t idx) {
  if (idx + 4 <= total) {
    double v0 = 0.0, v1 = 0.0, v2 = 0.0, v3 = 0.0;
    if (accumulate) {
      const f32x4 c = *reinterpret_cast<const f32x4*>(coeffs + idx);
      v0 = c[0], v1 = c[1], v2 = c[2], v3 = c[3];
    }
#pragma unroll 8
    for (int s = 0; s < Sc; ++s) {
      const f32x4 t = *reinterpret_cast<const f32x4*>(part + static_cast<size_t>(s) * stride + idx);
      v0 += t[0], v1 += t[1], v2 += t[2], v3 += t[3];
    }
    *reinterpret_cast<f32x4*>(coeffs + idx) =
        f32x4{static_cast<float>(v0), static_cast<float>(v1), static_cast<float>(v2), static_cast<float>(v3)};
  } else {
    for (size_t k = idx; k < total; ++k) {
      double v = accumulate ? coeffs[k] : 0.0f;
      for (int s = 0; s < Sc; ++s) v += part[static_cast<size_t>(s) * stride + k];
      coeffs[k] = static_cast<float>(v);
    }
  }
}

// the chunk reduction of both tensors in one launch (grid y: 0 = K, 1 = V)
struct ReducePair {
  const float* part[2];
  float* coeffs[2];
  size_t total[2], stride[2];
  int Sc, accumulate;
};
__global__ __launch_bounds__(256) void compress_reduce_kv(ReducePair r) {
  const int y = blockIdx.y;
  const float* part = y ? r.part[1] : r.part[0];
  float* coeffs = y ? r.coeffs[1] : r.coeffs[0];
  const size_t total = y ? r.total[1] : r.total[0], stride = y ? r.stride[1] : r.stride[0];
  const size_t idx = (static_cast<size_t>(blockIdx.x) * 256 + threadIdx.x) * 4;
  if (idx >= total) return;
  reduce_chunks(part, coeffs, total, stride, r.Sc, r.accumulate, idx);
}

// the chunk reduction of one tensor
__global__ __launch_bounds__(256) void compress_reduce(const float* part, float* coeffs, size_t total,
                                                       size_t stride, int Sc, int accumulate) {
  const size_t idx = (static_cast<size_t>(blockIdx.x) * 256 + threadIdx.x) * 4;
  if (idx >= total) return;
  reduce_chunks(part, coeffs, total, stride, Sc, accumulate, idx);
}

struct CompressPlan {
  int Sc, chunk, MC, DCn, nmax, stage;
  unsigned ks_elems, lds;
  size_t total;  // workspace bytes
};

// tensors: how many tensors share the projection launch (2 for the K | V pair: each then aims at half
// the chip, so that the pair is ONE round of workgroups - half the chunk partials, one fixed cost)
static CompressPlan make_compress_plan(int dtype, int B, int H, int N, int D, int Dc, int M,
                                       int keep_layout, int keep_offset, int tensors = 1) {
  CompressPlan pl{};
  pl.nmax = M / 2;
  pl.MC = (Dc > 0 && pl.nmax > 0) ? (pl.nmax + kPairs - 1) / kPairs : 1;
  pl.DCn = Dc > 0 ? (Dc + kCols - 1) / kCols : 1;
  const long groups = static_cast<long>(B) * H * pl.MC * pl.DCn;
  const long nblocks = (N + kFB - 1) / kFB;       // 128-token blocks (two blocks of the generic kernel)
  // Token chunks: one workgroup per compute unit (a projection workgroup takes a whole unit: 87 KB of
  // LDS, 256 registers).  A second round of workgroups costs more (its fixed prologue / epilogue,
  // twice the chunk partials) than the idle tail of one round (measured: 256 vs 512 targets: step
  // -7 % on 16 x 8K, -15 % on 8 x 4K MHA where the reduction disappears altogether).
  const long kTargetWgs = 256 / tensors;
  long want = (kTargetWgs + groups - 1) / groups;
  const long cap = nblocks / 8 > 0 ? nblocks / 8 : 1;     // but at least 1024 tokens per chunk: the
  if (want > cap) want = cap;                             // chunk partials cost memory traffic
  if (want < 1) want = 1;
  long per = N > 0 ? (nblocks + want - 1) / want : 1;
  // fp32 inputs: an fp32 accumulator that runs over n tokens of a slow tone the band misses ends
  // with an error of about 2^-24 * n / 11 of sqrt(N) * rms(x), the scale the 1e-5 parity bound is
  // taken against; 512 tokens per chunk keep that three times below the bound for any N
  if (dtype == FA_F32 && per > kF32ChunkBlocks) per = kF32ChunkBlocks;
  pl.chunk = static_cast<int>(per) * kFB;
  pl.Sc = N > 0 ? (N + pl.chunk - 1) / pl.chunk : 0;
  pl.total = (pl.Sc > 1 && Dc > 0)
                 ? align_up(static_cast<size_t>(pl.Sc) * ((static_cast<size_t>(B) * H * M * Dc + 3) & ~size_t(3)) *
                                sizeof(float), 256)
                 : 0;
  const unsigned es = dtype == FA_F32 ? 4 : 2;
  const int Du = D - Dc, kp = (Du + 7) & ~7;
  const unsigned rows_elems = kTB * (kp + 8), tok8_elems = static_cast<unsigned>(Du) * kLdX;
  pl.ks_elems = keep_layout == FA_KEEP_ROWS ? rows_elems : tok8_elems;
  const unsigned base = 2u * (kCols * kLdX + 8u) * es;
  pl.stage = Du > 0 && (keep_layout == FA_KEEP_ROWS || keep_offset % 8 == 0) &&
             base + 2u * pl.ks_elems * es <= kMaxCLds;
  if (!pl.stage) pl.ks_elems = 0;
  pl.lds = base + 2u * pl.ks_elems * es;
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

template <int DT, int KM>
static int launch_project_fast(const CompressParams& p, const CompressPlan& pl, unsigned lds, hipStream_t st,
                               KernelTimers* tm) {
  auto kern = compress_project_fast<DT, KM>;
  // the dynamic-LDS ceiling belongs to the kernel as loaded on the current device: raised whenever a
  // launch needs it (a host-side table write, no stream operation)
  if (lds > 48u * 1024u &&
      hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize,
                          static_cast<int>(kMaxCLds)) != hipSuccess)
    return FA_ERR_HIP;
  dim3 grid(pl.Sc, pl.MC, p.B * p.H);
  FA_LAUNCH_TIMED(tm, 0, kern, grid, dim3(kCBlock), lds, st, p);
  return FA_OK;
}

template <typename T, int DT, int kXR, bool kFast, bool kSplit>
static int launch_project(const CompressParams& p, const CompressPlan& pl, hipStream_t st, KernelTimers* tm) {
  auto kern = compress_project<T, DT, kXR, kFast, kSplit>;
  if (pl.lds > 48u * 1024u &&
      hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize,
                          static_cast<int>(kMaxCLds)) != hipSuccess)
    return FA_ERR_HIP;
  dim3 grid(pl.Sc, pl.MC * pl.DCn, p.B * p.H);
  FA_LAUNCH_TIMED(tm, 0, kern, grid, dim3(kCBlock), pl.lds, st, p);
  return FA_OK;
}

}  // namespace fa

extern "C" {

size_t fa_compress_workspace_bytes_for(int dtype, int B, int H, int N, int D, int Dc, int M) {
  if (dtype != FA_F32 && dtype != FA_BF16) return 0;
  if (fa::check_compress_shapes(dtype, B, H, N, D, Dc, M, M > N ? M : N, 0) != FA_OK) return 0;
  const size_t t = fa::make_compress_plan(dtype, B, H, N, D, Dc, M, FA_KEEP_ROWS, 0).total;
  return t ? t : 256;
}

size_t fa_compress_workspace_bytes(int B, int H, int N, int D, int Dc, int M) {
  // enough for either element type (fp32 inputs use shorter token chunks, hence more partials)
  const size_t tb = fa_compress_workspace_bytes_for(FA_BF16, B, H, N, D, Dc, M);
  const size_t tf = fa_compress_workspace_bytes_for(FA_F32, B, H, N, D, Dc, M);
  return tb > tf ? tb : tf;
}

static int compress_impl(const void* x, int dtype, int64_t sx_b, int64_t sx_h, int64_t sx_n, int B,
                         int H, int N, int D, const uint8_t* dim_mask, int Dc, int M, int T, int t0,
                         int accumulate, float* coeffs, void* x_keep, int keep_layout,
                         int64_t keep_stride_bh, int keep_offset, void* workspace,
                         size_t workspace_bytes, void* hip_stream, fa::KernelTimers* tm,
                         fa::CompressParams* only_params = nullptr, fa::CompressPlan* only_plan = nullptr,
                         int tensors = 1) {
  using namespace fa;
  const hipError_t prior = hipPeekAtLastError();   // (an error left by earlier, unrelated calls is not this call's)
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
  if (x_keep && (keep_stride_bh < dense || (keep_stride_bh % 8) ||
                 (reinterpret_cast<uintptr_t>(x_keep) & 15u)))
    return FA_ERR_SHAPE;
  if (reinterpret_cast<uintptr_t>(coeffs) & 15u) return FA_ERR_SHAPE;

  const CompressPlan pl = make_compress_plan(dtype, B, H, N, D, Dc, M, keep_layout, keep_offset, tensors);
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
  p.keep = x_keep; p.keep_layout = keep_layout; p.keep_pitch = keep_pitch;
  p.keep_stride = keep_stride_bh; p.keep_offset = keep_offset; p.stage_keep = pl.stage;
  p.Sc = pl.Sc; p.chunk = pl.chunk; p.MC = pl.MC; p.DCn = pl.DCn; p.nmax = pl.nmax;
  p.ks_elems = pl.ks_elems;
  {
    const int kv_d = (keep_layout == FA_KEEP_ROWS) ? (keep_pitch / 8 > 0 ? keep_pitch / 8 : 1) : (Du > 0 ? Du : 1);
    p.kv_magic = static_cast<uint32_t>((65536 + kv_d - 1) / kv_d);
  }
  p.ph_scale = 4294967296.0 / static_cast<double>(T);
  p.part = static_cast<float*>(workspace);
  p.part_stride = (static_cast<size_t>(B) * H * M * Dc + 3) & ~size_t(3);

  if (only_params) {   // the caller launches (the K | V pair entry)
    *only_params = p;
    *only_plan = pl;
    return FA_OK;
  }
  hipStream_t stream = static_cast<hipStream_t>(hip_stream);
  const size_t total = static_cast<size_t>(B) * H * M * Dc;
  if (pl.Sc > 0) {
    const int cols = Dc < kCols ? Dc : kCols;
    int rc;
    const bool narrow = cols <= 96, small_d = D <= 128;
    // every thread routes fixed dims when the row vectors divide the workgroup and kept dims are staged
    const bool fast = (kCBlock % (D / 8)) == 0 && (pl.stage || Du == 0 || x_keep == nullptr);
#define FA_LAUNCH_PROJECT2(T_, F_, S_)                                                              \
  rc = narrow ? (small_d ? launch_project<T_, 3, 2, F_, S_>(p, pl, stream, tm) : launch_project<T_, 3, 4, F_, S_>(p, pl, stream, tm)) \
              : (small_d ? launch_project<T_, 4, 2, F_, S_>(p, pl, stream, tm) : launch_project<T_, 4, 4, F_, S_>(p, pl, stream, tm))
#define FA_LAUNCH_PROJECT(T_, S_)       \
  do {                                  \
    if (fast) {                         \
      FA_LAUNCH_PROJECT2(T_, true, S_); \
    } else {                            \
      FA_LAUNCH_PROJECT2(T_, false, S_);\
    }                                   \
  } while (0)
    // short bf16 segments: split basis in the generic kernel (see compress_project)
    const bool short_seg = dtype == FA_BF16 && N <= kSplitTokens;
    // bf16 with head dim 128 and staged (or no) kept dims: the specialised kernel
    const unsigned fast_lds = 2u * (kCols * kFP + static_cast<unsigned>(keep_pitch) * kFP + 8u) * 2u;
    const bool staged_ok = x_keep == nullptr || Du == 0 || keep_layout == FA_KEEP_ROWS || keep_offset % 8 == 0;
    if (dtype == FA_BF16 && D == 128 && staged_ok && fast_lds <= kMaxCLds && !short_seg) {
      // straight-line block step when every thread has at most one vector of kept dims to store
      const int nvec = (x_keep == nullptr || Du == 0) ? 0 : (keep_layout == FA_KEEP_ROWS ? kFB * (keep_pitch / 8) : Du * (kFB / 8));
      const int km = (Dc == 0 || nvec > kCBlock) ? -1 : (nvec == 0 ? 0 : (keep_layout == FA_KEEP_ROWS ? 1 : 2));
      // (column tiles compiled in: 6, 7 or 8 - a tile without compressed columns would still be multiplied)
#define FA_LAUNCH_FAST(KM_) \
  rc = narrow ? launch_project_fast<6, KM_>(p, pl, fast_lds, stream, tm) \
     : (Dc <= 112 ? launch_project_fast<7, KM_>(p, pl, fast_lds, stream, tm) : launch_project_fast<8, KM_>(p, pl, fast_lds, stream, tm))
      if (km == 0) FA_LAUNCH_FAST(0);
      else if (km == 1) FA_LAUNCH_FAST(1);
      else if (km == 2) FA_LAUNCH_FAST(2);
      else FA_LAUNCH_FAST(-1);
#undef FA_LAUNCH_FAST
    } else if (dtype == FA_F32) {
      FA_LAUNCH_PROJECT(float, false);
    } else if (short_seg) {
      FA_LAUNCH_PROJECT(bf16_t, true);
    } else {
      FA_LAUNCH_PROJECT(bf16_t, false);
    }
#undef FA_LAUNCH_PROJECT2
#undef FA_LAUNCH_PROJECT
    if (rc != FA_OK) return rc;
  }
  if (total > 0 && (pl.Sc > 1 || (pl.Sc == 0 && !accumulate))) {
    const unsigned blocks = static_cast<unsigned>((total / 4 + 1 + 255) / 256);
    FA_LAUNCH_TIMED(tm, 1, compress_reduce, dim3(blocks), dim3(256), 0, stream, p.part, coeffs, total,
                    p.part_stride, pl.Sc, p.accumulate);
  }
  return (hipPeekAtLastError() == hipSuccess || prior != hipSuccess) ? FA_OK : FA_ERR_HIP;
}

int fa_compress(const void* x, int dtype, int64_t sx_b, int64_t sx_h, int64_t sx_n, int B, int H,
                int N, int D, const uint8_t* dim_mask, int Dc, int M, int T, int t0, int accumulate,
                float* coeffs, void* x_keep, int keep_layout, int64_t keep_stride_bh,
                int keep_offset, void* workspace, size_t workspace_bytes, void* hip_stream) {
  return compress_impl(x, dtype, sx_b, sx_h, sx_n, B, H, N, D, dim_mask, Dc, M, T, t0, accumulate,
                       coeffs, x_keep, keep_layout, keep_stride_bh, keep_offset, workspace,
                       workspace_bytes, hip_stream, nullptr);
}

size_t fa_compress_kv_workspace_bytes_for(int dtype, int B, int H, int N, int D, int Dkc, int Dvc, int M) {
  const size_t a = fa_compress_workspace_bytes_for(dtype, B, H, N, D, Dkc, M);
  const size_t b = fa_compress_workspace_bytes_for(dtype, B, H, N, D, Dvc, M);
  if (a == 0 || b == 0) return 0;
  return ((a + 255) & ~size_t(255)) + b;
}

size_t fa_compress_kv_workspace_bytes(int B, int H, int N, int D, int Dkc, int Dvc, int M) {
  const size_t tb = fa_compress_kv_workspace_bytes_for(FA_BF16, B, H, N, D, Dkc, Dvc, M);
  const size_t tf = fa_compress_kv_workspace_bytes_for(FA_F32, B, H, N, D, Dkc, Dvc, M);
  return tb > tf ? tb : tf;
}

// tm / tm2 (optional): event pairs for the timed entry point; tm2 is used only when the call falls
// back to two projections
static int compress_kv_impl(const void* k, const void* v, int dtype, int64_t sx_b, int64_t sx_h, int64_t sx_n,
                            int B, int H, int N, int D, const uint8_t* kmask, int Dkc, const uint8_t* vmask,
                            int Dvc, int M, int T, int t0, int accumulate, float* ck, float* cv, void* k_keep,
                            int64_t kk_stride_bh, void* v_keep, int64_t vk_stride_bh, int keep_offset,
                            void* workspace, size_t workspace_bytes, void* hip_stream, fa::KernelTimers* tm,
                            fa::KernelTimers* tm2) {
  using namespace fa;
  const hipError_t prior = hipPeekAtLastError();   // (an error left by earlier, unrelated calls is not this call's)
  if (dtype != FA_F32 && dtype != FA_BF16) return FA_ERR_UNSUPPORTED;
  const size_t wk = (fa_compress_workspace_bytes_for(dtype, B, H, N, D, Dkc, M) + 255) & ~size_t(255);
  const size_t wv = fa_compress_workspace_bytes_for(dtype, B, H, N, D, Dvc, M);
  if (wk == 0 || wv == 0) return FA_ERR_SHAPE;
  if (!workspace) return FA_ERR_NULL;
  if (workspace_bytes < wk + wv || (reinterpret_cast<uintptr_t>(workspace) & 255u)) return FA_ERR_WORKSPACE;
  char* ws = static_cast<char*>(workspace);
  CompressParams pk{}, pv{};
  CompressPlan plk{}, plv{};
  int rc = compress_impl(k, dtype, sx_b, sx_h, sx_n, B, H, N, D, kmask, Dkc, M, T, t0, accumulate, ck, k_keep,
                         FA_KEEP_ROWS, kk_stride_bh, keep_offset, ws, wk, hip_stream, nullptr, &pk, &plk, 2);
  if (rc != FA_OK) return rc;
  rc = compress_impl(v, dtype, sx_b, sx_h, sx_n, B, H, N, D, vmask, Dvc, M, T, t0, accumulate, cv, v_keep,
                     FA_KEEP_TOK8, vk_stride_bh, keep_offset, ws + wk, wv, hip_stream, nullptr, &pv, &plv, 2);
  if (rc != FA_OK) return rc;
  // One launch for both when each side takes the straight-line step with kept dims to write
  // (bf16, head dim 128, at most one kept vector per thread and block) and they split the tokens
  // alike; otherwise one call after the other.
  auto nvec_of = [&](const CompressParams& p) {
    return p.keep_layout == FA_KEEP_ROWS ? kFB * (p.keep_pitch / 8) : p.Du * (kFB / 8);
  };
  const unsigned lds_k = 2u * (kCols * kFP + static_cast<unsigned>(pk.keep_pitch) * kFP + 8u) * 2u;
  const unsigned lds_v = 2u * (kCols * kFP + static_cast<unsigned>(pv.keep_pitch) * kFP + 8u) * 2u;
  const unsigned lds = lds_k > lds_v ? lds_k : lds_v;
  const bool pair = dtype == FA_BF16 && D == 128 && N > kSplitTokens && Dkc > 0 && Dvc > 0 && k_keep && v_keep &&
                    pk.Du > 0 && pv.Du > 0 && nvec_of(pk) <= kCBlock && nvec_of(pv) <= kCBlock &&
                    keep_offset % 8 == 0 && lds <= kMaxCLds && plk.Sc == plv.Sc && plk.chunk == plv.chunk &&
                    plk.MC == plv.MC && plk.Sc > 0;
  if (!pair) {
    rc = compress_impl(k, dtype, sx_b, sx_h, sx_n, B, H, N, D, kmask, Dkc, M, T, t0, accumulate, ck, k_keep,
                       FA_KEEP_ROWS, kk_stride_bh, keep_offset, ws, wk, hip_stream, tm);
    if (rc != FA_OK) return rc;
    return compress_impl(v, dtype, sx_b, sx_h, sx_n, B, H, N, D, vmask, Dvc, M, T, t0, accumulate, cv, v_keep,
                         FA_KEEP_TOK8, vk_stride_bh, keep_offset, ws + wk, wv, hip_stream, tm2);
  }
  hipStream_t stream = static_cast<hipStream_t>(hip_stream);
  CompressParamsKV pp{pk, pv};
  // column tiles compiled in: 6, 7 or 8 (a tile without compressed columns would still be multiplied)
  const int dmax = Dkc > Dvc ? Dkc : Dvc;
  const void* kern = dmax <= 96 ? reinterpret_cast<const void*>(compress_project_fast_kv<6>)
                   : (dmax <= 112 ? reinterpret_cast<const void*>(compress_project_fast_kv<7>)
                                  : reinterpret_cast<const void*>(compress_project_fast_kv<8>));
  if (lds > 48u * 1024u &&
      hipFuncSetAttribute(kern,
                          hipFuncAttributeMaxDynamicSharedMemorySize, static_cast<int>(kMaxCLds)) != hipSuccess)
    return FA_ERR_HIP;
  const dim3 grid(plk.Sc, plk.MC, 2 * B * H);
  if (dmax <= 96) FA_LAUNCH_TIMED(tm, 0, compress_project_fast_kv<6>, grid, dim3(kCBlock), lds, stream, pp);
  else if (dmax <= 112) FA_LAUNCH_TIMED(tm, 0, compress_project_fast_kv<7>, grid, dim3(kCBlock), lds, stream, pp);
  else FA_LAUNCH_TIMED(tm, 0, compress_project_fast_kv<8>, grid, dim3(kCBlock), lds, stream, pp);
  if (plk.Sc > 1) {
    ReducePair r{};
    r.part[0] = pk.part; r.part[1] = pv.part;
    r.coeffs[0] = ck; r.coeffs[1] = cv;
    r.total[0] = static_cast<size_t>(B) * H * M * Dkc; r.total[1] = static_cast<size_t>(B) * H * M * Dvc;
    r.stride[0] = pk.part_stride; r.stride[1] = pv.part_stride;
    r.Sc = plk.Sc; r.accumulate = accumulate ? 1 : 0;
    const size_t tmax = r.total[0] > r.total[1] ? r.total[0] : r.total[1];
    FA_LAUNCH_TIMED(tm, 1, compress_reduce_kv, dim3(static_cast<unsigned>((tmax / 4 + 1 + 255) / 256), 2), dim3(256), 0, stream, r);
  }
  return (hipPeekAtLastError() == hipSuccess || prior != hipSuccess) ? FA_OK : FA_ERR_HIP;
}

int fa_compress_kv(const void* k, const void* v, int dtype, int64_t sx_b, int64_t sx_h, int64_t sx_n,
                   int B, int H, int N, int D, const uint8_t* kmask, int Dkc, const uint8_t* vmask,
                   int Dvc, int M, int T, int t0, int accumulate, float* ck, float* cv, void* k_keep,
                   int64_t kk_stride_bh, void* v_keep, int64_t vk_stride_bh, int keep_offset,
                   void* workspace, size_t workspace_bytes, void* hip_stream) {
  return compress_kv_impl(k, v, dtype, sx_b, sx_h, sx_n, B, H, N, D, kmask, Dkc, vmask, Dvc, M, T, t0, accumulate,
                          ck, cv, k_keep, kk_stride_bh, v_keep, vk_stride_bh, keep_offset, workspace,
                          workspace_bytes, hip_stream, nullptr, nullptr);
}

int fa_compress_kv_timed(const void* k, const void* v, int dtype, int64_t sx_b, int64_t sx_h, int64_t sx_n,
                         int B, int H, int N, int D, const uint8_t* kmask, int Dkc, const uint8_t* vmask,
                         int Dvc, int M, int T, int t0, int accumulate, float* ck, float* cv, void* k_keep,
                         int64_t kk_stride_bh, void* v_keep, int64_t vk_stride_bh, int keep_offset,
                         void* workspace, size_t workspace_bytes, void* hip_stream, float* kernel_ms) {
  if (!kernel_ms) return FA_ERR_NULL;
  fa::KernelTimers tm, tm2;
  int st = tm.create();
  if (st == FA_OK) st = tm2.create();
  if (st == FA_OK)
    st = compress_kv_impl(k, v, dtype, sx_b, sx_h, sx_n, B, H, N, D, kmask, Dkc, vmask, Dvc, M, T, t0, accumulate,
                          ck, cv, k_keep, kk_stride_bh, v_keep, vk_stride_bh, keep_offset, workspace,
                          workspace_bytes, hip_stream, &tm, &tm2);
  float a[2] = {0.f, 0.f}, b[2] = {0.f, 0.f};
  if (st == FA_OK) st = tm.read(2, a);
  if (st == FA_OK) st = tm2.read(2, b);
  if (st == FA_OK && hipStreamSynchronize(static_cast<hipStream_t>(hip_stream)) != hipSuccess) st = FA_ERR_HIP;
  kernel_ms[0] = a[0] + b[0];   // projection(s)
  kernel_ms[1] = a[1] + b[1];   // chunk reduction(s)
  tm.destroy();
  tm2.destroy();
  return st;
}

int fa_compress_timed(const void* x, int dtype, int64_t sx_b, int64_t sx_h, int64_t sx_n, int B,
                      int H, int N, int D, const uint8_t* dim_mask, int Dc, int M, int T, int t0,
                      int accumulate, float* coeffs, void* x_keep, int keep_layout,
                      int64_t keep_stride_bh, int keep_offset, void* workspace,
                      size_t workspace_bytes, void* hip_stream, float* kernel_ms) {
  if (!kernel_ms) return FA_ERR_NULL;
  fa::KernelTimers tm;
  int st = tm.create();
  if (st == FA_OK)
    st = compress_impl(x, dtype, sx_b, sx_h, sx_n, B, H, N, D, dim_mask, Dc, M, T, t0, accumulate,
                       coeffs, x_keep, keep_layout, keep_stride_bh, keep_offset, workspace,
                       workspace_bytes, hip_stream, &tm);
  if (st == FA_OK) st = tm.read(2, kernel_ms);
  if (st == FA_OK && hipStreamSynchronize(static_cast<hipStream_t>(hip_stream)) != hipSuccess) st = FA_ERR_HIP;
  tm.destroy();
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
    case FA_ERR_SCRATCH: return "problem needs more split-K state than the library's static scratch array holds";
    default: return "unknown status";
  }
}

}  // extern "C"
