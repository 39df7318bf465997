// fa_decode: fused decode attention over a Fourier-compressed KV cache (Eq. 6).
//
// Eq. 6 rebuilds the compressed dimensions of every middle row from the
// coefficients and then attends.  Both products with the rebuilt rows commute
// with the (linear) reconstruction, so the rows are never formed:
//
//   K side:  q . K~[j, D^kc] = sum_m phi_m(j) g_m,     g = diag(w) C_k q[D^kc]
//   V side:  sum_j p_j V~[j, D^vc] = (diag(w) C_v)^T r,   r_m = sum_j p_j phi_m(j)
//
// and the series over the basis is evaluated on the matrix cores through the
// angle-addition identity: with j = tau + u (tau = tile origin, u < 64),
//   sum_m phi_m(tau+u) g_m = sum_m E[u,m] g'_m(tau),
// where E[u,m] = phi_m(u) is a fixed 64-row table (LDS resident, built once
// per workgroup) and g'(tau) is g with every (cos, sin) pair rotated by
// omega_n tau.  One 16-column MFMA tile covers (up to 4 token tiles) x (query
// heads of the group), so the table is shared by the heads and by both sides.
// The V side is the mirror image: r' = P^T E per tile, rotated back once per
// chunk.
//
// The kernels are latency-shaped: a decode step moves only tens of megabytes,
// so every kernel requests all of its global-memory operands up front (one
// dependent round trip) and hides them behind table construction and MFMAs.
//
// Launches on the caller's stream:
//   1. decode_prepare : g (series order) for every query head, from C_k and q.
//   2. decode_partial : one workgroup per (sequence, KV head, token chunk);
//      chunks of middle rows and chunks of full-width sink/window rows; emits
//      a flash-decoding partial (max, sum, acc[D], r[Mint]) per query head.
//   3. decode_finish  : one workgroup per query head merges the partials,
//      applies diag(w) C_v to r and normalises.

#include "fa_common.hpp"
#include "fa_mma.hpp"

namespace fa {

constexpr int kBlock = 256;
constexpr int kWaves = 4;
constexpr int kMaxG = FA_MAX_GROUP;
constexpr int kTJ = 64;            // tokens per tile (rows of the E table)
constexpr int kRB = kTJ / 16;      // 16-row blocks per tile
constexpr int kXN = kTJ / 32;      // 32-token contraction steps per tile on the V side
constexpr int kMaxKT = 4;          // tiles per wave step
constexpr int kWChunk = 64;        // full-width rows per workgroup
constexpr int kMaxDvTiles = 8;     // kept V dims handled per middle row: 8 * 16
constexpr int kMaxPartials = 1024; // partial records per query head
constexpr unsigned kMaxDynLds = 160 * 1024 - 4096;   // dynamic LDS a workgroup may ask for
constexpr int kFinBlock = 1024;    // threads of decode_finish

typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef _Float16 f16x2 __attribute__((ext_vector_type(2)));
typedef float f32x2 __attribute__((ext_vector_type(2)));

// Developer aid (compiled out unless FA_TRACE is defined): per-wave cycle stamps
// at phase boundaries, written behind the partial records of the workspace.
#ifdef FA_TRACE
#define FA_STAMP(i)                                                                          \
  do {                                                                                       \
    if ((threadIdx.x & 63) == 0)                                                             \
      p.trace[((static_cast<size_t>(blockIdx.y) * gridDim.x + blockIdx.x) * 4 +              \
               (threadIdx.x >> 6)) * 16 + (i)] = clock64();                                  \
  } while (0)
#else
#define FA_STAMP(i) do {} while (0)
#endif

struct DecodeParams {
  const void* q;
  const float* ck;
  const float* cv;
  const uint8_t* kmask;
  const uint8_t* vmask;
  const void* k_keep;
  const void* v_keep;
  const void* k_full;
  const void* v_full;
  int64_t kk_stride, vk_stride, full_stride;
  int B, Hq, Hkv, G, D, Dkc, Dvc, Dku, Dvu, M, T, t0, N, W;
  int Gp, KT;       // group size padded to a power of two, tiles per wave step
  int Mint;         // series length: 2 * (M/2) padded to a compiled size
  int Sw, Sm;       // chunks of full-width rows / of middle rows (middle chunks come first)
  int chunk_m;      // middle rows per chunk (multiple of the workgroup step)
  int rec;          // floats per partial record: 2 + D + Mint
  unsigned lds_tab; // bytes of the E-table region
  float scale;
  double ph_scale;  // 2^32 / T
  float* gs;        // [B,Hq,Mint] series coefficients, K-side order
  float* g0;        // [B,Hq]      constant-term coefficient
  float* part;      // [B,Hq,Sm+Sw,rec]
  float* out;       // [B,Hq,D]
#ifdef FA_TRACE
  long long* trace;
#endif
};

// ---------------------------------------------------------------------------
// small helpers
// ---------------------------------------------------------------------------
template <typename T> struct SeriesType;
template <> struct SeriesType<bf16_t> { using type = f16_t; };   // E, g', p on the series side
template <> struct SeriesType<float> { using type = float; };

__device__ __forceinline__ void pack8(Frag<f16_t>& f, const float* v) {
#pragma unroll
  for (int e = 0; e < 4; ++e)
    f.v[e] = __builtin_bit_cast(uint32_t, __builtin_convertvector(f32x2{v[2 * e], v[2 * e + 1]}, f16x2));
}
__device__ __forceinline__ void pack8(Frag<bf16_t>& f, const float* v) {
#pragma unroll
  for (int e = 0; e < 4; ++e)
    f.v[e] = __builtin_bit_cast(uint32_t, __builtin_convertvector(f32x2{v[2 * e], v[2 * e + 1]}, bf16x2));
}
__device__ __forceinline__ void pack8(Frag<float>& f, const float* v) {
#pragma unroll
  for (int e = 0; e < 8; ++e) f.v[e] = v[e];
}

__device__ __forceinline__ void unpack8(const Frag<bf16_t>& f, float* v) {
#pragma unroll
  for (int e = 0; e < 4; ++e) {
    v[2 * e] = __uint_as_float(f.v[e] << 16);
    v[2 * e + 1] = __uint_as_float(f.v[e] & 0xffff0000u);
  }
}
__device__ __forceinline__ void unpack8(const Frag<float>& f, float* v) {
#pragma unroll
  for (int e = 0; e < 8; ++e) v[e] = f.v[e];
}
// element e of a fragment, as stored
__device__ __forceinline__ bf16_t frag_elem(const Frag<bf16_t>& f, int e) {
  return bf16_t{static_cast<uint16_t>((f.v[e >> 1] >> (16 * (e & 1))) & 0xffffu)};
}
__device__ __forceinline__ float frag_elem(const Frag<float>& f, int e) { return f.v[e]; }
__device__ __forceinline__ float to_f32(bf16_t x) { return bf16_to_f32(x.bits); }
__device__ __forceinline__ float to_f32(float x) { return x; }

// keep the first `nvalid` (<= 8, may be <= 0) elements, zero the rest
__device__ __forceinline__ void mask_tail(Frag<bf16_t>& f, int nvalid) {
#pragma unroll
  for (int e = 0; e < 4; ++e) {
    const uint32_t lo = (2 * e < nvalid) ? 0x0000ffffu : 0u;
    const uint32_t hi = (2 * e + 1 < nvalid) ? 0xffff0000u : 0u;
    f.v[e] &= (lo | hi);
  }
}
__device__ __forceinline__ void mask_tail(Frag<float>& f, int nvalid) {
#pragma unroll
  for (int e = 0; e < 8; ++e)
    if (e >= nvalid) f.v[e] = 0.0f;
}

// cos / sin of a 32-bit fixed-point phase (2^32 = one turn)
template <typename T>
__device__ __forceinline__ void phase_cs(uint32_t ph, float* c, float* s) {
  const float x = static_cast<float>(static_cast<int32_t>(ph)) * 2.3283064365386963e-10f;  // turns in [-0.5, 0.5)
  if constexpr (sizeof(T) == 4) {
    sincospif(2.0f * x, s, c);          // fp32 inputs: full-accuracy evaluation
  } else {
    *s = __builtin_amdgcn_sinf(x);      // hardware sin/cos take turns
    *c = __builtin_amdgcn_cosf(x);
  }
}

// fixed-point phase of position pos: frac(pos / T) * 2^32 (wraps for pos >= T)
__device__ __forceinline__ uint32_t phase_of(int pos, double ph_scale) {
  return static_cast<uint32_t>(static_cast<uint64_t>(static_cast<double>(pos) * ph_scale));
}

// value held by lane i of the caller's quad (4 consecutive lanes)
__device__ __forceinline__ float quad_bcast(float v, int i) {
  const int x = __float_as_int(v);
  int r;
  switch (i) {
    case 0: r = __builtin_amdgcn_mov_dpp(x, 0x00, 0xf, 0xf, true); break;
    case 1: r = __builtin_amdgcn_mov_dpp(x, 0x55, 0xf, 0xf, true); break;
    case 2: r = __builtin_amdgcn_mov_dpp(x, 0xaa, 0xf, 0xf, true); break;
    default: r = __builtin_amdgcn_mov_dpp(x, 0xff, 0xf, 0xf, true); break;
  }
  return __int_as_float(r);
}

// every wave reads the whole mask row (D <= 256) and keeps it as 4 ballot words
__device__ __forceinline__ void mask_ballots(const uint8_t* mask, int D, int lane, uint64_t* bal) {
  uint8_t b[4];
#pragma unroll
  for (int j = 0; j < 4; ++j) b[j] = mask[min(lane + 64 * j, D - 1)];
#pragma unroll
  for (int j = 0; j < 4; ++j) bal[j] = __ballot(b[j] != 0 && lane + 64 * j < D);
}

// rank of dimension d among the kept dims (>= 0) or -(1 + rank among the
// compressed dims), from the ballot words of the mask
__device__ __forceinline__ int dim_rank(const uint64_t* bal, int d) {
  const int w = d >> 6;
  const uint64_t bit = 1ull << (d & 63);
  int nc = 0;
  uint64_t hit = 0;
#pragma unroll
  for (int j = 0; j < 4; ++j) {   // static indices only: the words stay in registers
    const uint64_t below = (j < w) ? ~0ull : ((j == w) ? (bit - 1ull) : 0ull);
    nc += __popcll(bal[j] & below);
    hit |= bal[j] & ((j == w) ? bit : 0ull);
  }
  return hit ? -(1 + nc) : d - nc;
}

// ---------------------------------------------------------------------------
// 1. g = diag(w) C_k q_c, written in series order: slot s <-> basis function s+1
// ---------------------------------------------------------------------------
constexpr int kPrepRows = 8;                       // basis rows per workgroup
constexpr int kPrepLoads = kPrepRows * FA_MAX_HEAD_DIM / kBlock;   // C_k loads per thread (worst case)

template <typename T>
__global__ __launch_bounds__(kBlock) void decode_prepare(DecodeParams p) {
  __shared__ float qc[kMaxG * FA_MAX_HEAD_DIM];            // [G][Dkc] query at the compressed dims
  __shared__ float crow[kPrepRows * (FA_MAX_HEAD_DIM + 1)];

  const int tid = threadIdx.x, lane = tid & 63;
  const int bh = blockIdx.y, b = bh / p.Hkv, hkv = bh % p.Hkv;
  const int m0 = blockIdx.x * kPrepRows;
  const int Dkc = p.Dkc, D = p.D, G = p.G, Gp = p.Gp;
  const int ld = Dkc + 1;

  // all global operands first: C_k rows, the mask row, q of the group
  const float* ck = p.ck + static_cast<size_t>(bh) * p.M * Dkc;
  const int nck = kPrepRows * Dkc;
  float cval[kPrepLoads];
#pragma unroll
  for (int i = 0; i < kPrepLoads; ++i) {
    const int it = min(tid + i * kBlock, max(nck - 1, 0));
    const int r = it / max(Dkc, 1), col = it % max(Dkc, 1);
    const int m = min(m0 + r, p.M - 1);
    cval[i] = (Dkc > 0) ? ck[static_cast<size_t>(m) * Dkc + col] : 0.0f;
  }
  uint64_t kbal[4];
  mask_ballots(p.kmask + static_cast<size_t>(bh) * D, D, lane, kbal);
  const T* q = static_cast<const T*>(p.q) + (static_cast<size_t>(b) * p.Hq + hkv * G) * D;
  constexpr int kQLoads = kMaxG * FA_MAX_HEAD_DIM / 8 / kBlock;   // 8-element vectors per thread
  Frag<T> qv[kQLoads];
  const int nq8 = G * D / 8;
#pragma unroll
  for (int i = 0; i < kQLoads; ++i) qv[i].load(q + 8 * min(tid + i * kBlock, nq8 - 1));

#pragma unroll
  for (int i = 0; i < kPrepLoads; ++i) {
    const int it = tid + i * kBlock;
    if (it < nck) {
      const int r = it / Dkc, col = it % Dkc;
      crow[r * ld + col] = (m0 + r < p.M) ? cval[i] : 0.0f;
    }
  }
#pragma unroll
  for (int i = 0; i < kQLoads; ++i) {
    const int v8 = tid + i * kBlock;
    if (v8 < nq8) {
      const int h = (8 * v8) / D, d0 = (8 * v8) % D;
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        const int r = dim_rank(kbal, d0 + e);
        if (r < 0) qc[h * Dkc + (-r - 1)] = to_f32(frag_elem(qv[i], e));
      }
    }
  }
  __syncthreads();

  // (row, head) dot products; nseg consecutive lanes share one of them
  const int nseg = kBlock / (kPrepRows * Gp);   // power of two, >= 2
  const int seg = tid % nseg, item = tid / nseg;
  const int r = item % kPrepRows, h = item / kPrepRows;
  float acc = 0.0f;
  if (h < G)
    for (int i = seg; i < Dkc; i += nseg) acc += crow[r * ld + i] * qc[h * Dkc + i];
  for (int o = nseg >> 1; o > 0; o >>= 1) acc += __shfl_xor(acc, o, kWave);
  const int m = m0 + r;
  if (seg == 0 && h < G && m <= p.Mint) {
    const float g = (m < p.M) ? acc * basis_weight((m + 1) / 2, p.T) : 0.0f;
    const size_t hq = static_cast<size_t>(b) * p.Hq + hkv * G + h;
    if (m == 0) p.g0[hq] = g;
    else p.gs[hq * p.Mint + (m - 1)] = g;
  }
}

// ---------------------------------------------------------------------------
// 2a. full-width sink/window rows: plain single-query attention partial
// ---------------------------------------------------------------------------
template <typename T>
__device__ __forceinline__ void partial_full_rows(const DecodeParams& p, unsigned char* smem) {
  const int s = blockIdx.x - p.Sm, bh = blockIdx.y, b = bh / p.Hkv, hkv = bh % p.Hkv;
  const int G = p.G, D = p.D;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int q4 = lane >> 4, r16 = lane & 15;
  const size_t hq0 = static_cast<size_t>(b) * p.Hq + hkv * G;
  const int j0 = s * kWChunk, n = min(kWChunk, p.W - j0);

  // LDS carve-up
  T* qf = reinterpret_cast<T*>(smem);                                             // [16][D]
  float* sc = reinterpret_cast<float*>(smem + 16 * FA_MAX_HEAD_DIM * sizeof(T));  // [64][16]
  float* red = sc + kWChunk * kMaxG;                                              // [slices*4][D]
  __shared__ float mx[kMaxG], lsum[kMaxG];

  FA_STAMP(0);
  // ---- all global operands first ---------------------------------------------------
  constexpr int kQLoads = kMaxG * FA_MAX_HEAD_DIM / 8 / kBlock;
  const T* q = static_cast<const T*>(p.q) + hq0 * D;
  const int nq8 = G * D / 8;
  Frag<T> qv[kQLoads];
#pragma unroll
  for (int i = 0; i < kQLoads; ++i) qv[i].load(q + 8 * min(tid + i * kBlock, nq8 - 1));
  // K rows of this wave (16 rows), 32 dims per fragment
  constexpr int kKF = FA_MAX_HEAD_DIM / 32;
  const int tok = wave * 16 + r16;
  const T* krow = static_cast<const T*>(p.k_full) + bh * p.full_stride +
                  static_cast<int64_t>(j0 + min(tok, n - 1)) * D;
  Frag<T> ka[kKF];
#pragma unroll
  for (int cc = 0; cc < kKF; ++cc)
    if (cc * 32 < D) ka[cc].load(krow + min(cc * 32 + 8 * q4, D - 8));
  // V rows: thread owns 8 dims of every nts-th row
  const int nch = D / 8;
  const int nts = kBlock / nch;
  const int dc = tid % nch, ts = tid / nch;
  const bool active = ts < nts;
  constexpr int kMaxRows = 8;   // ceil(64 / nts) <= 8 for D <= 256
  Frag<T> vf[kMaxRows];
  {
    const T* vb = static_cast<const T*>(p.v_full) + bh * p.full_stride +
                  static_cast<int64_t>(j0) * D + dc * 8;
#pragma unroll
    for (int r = 0; r < kMaxRows; ++r) {
      const int j = ts + r * nts;
      if (r * nts < kWChunk) vf[r].load(vb + static_cast<int64_t>(min(j, n - 1)) * D);
    }
  }

  FA_STAMP(1);
  // ---- q into LDS (rows >= G zero) ---------------------------------------------------
  for (int it = tid; it < (16 - G) * D; it += kBlock) qf[G * D + it] = T{};
#pragma unroll
  for (int i = 0; i < kQLoads; ++i) {
    const int v8 = tid + i * kBlock;
    if (v8 < nq8) *reinterpret_cast<Frag<T>*>(qf + 8 * v8) = qv[i];
  }
  __syncthreads();

  FA_STAMP(2);
  // scores of 16 rows per wave: A = K rows, B = q (one column per head)
  {
    f32x4 acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int cc = 0; cc < kKF; ++cc) {
      if (cc * 32 < D) {
        const int d0 = cc * 32 + 8 * q4;
        Frag<T> a = ka[cc], bq;
        if (d0 < D) {
          bq.load(qf + r16 * D + d0);
        } else {
          bq.zero();
          a.zero();
        }
        mma_k32(acc, a, bq);
      }
    }
    // lane holds column h = r16, rows 4*q4 + v
    if (r16 < G) {
#pragma unroll
      for (int v = 0; v < 4; ++v) {
        const int t = wave * 16 + 4 * q4 + v;
        sc[t * kMaxG + r16] = (t < n) ? acc[v] * p.scale : -INFINITY;
      }
    }
  }
  __syncthreads();
  FA_STAMP(3);
  if (wave == 0) {
    for (int h = 0; h < G; ++h) {
      const float sv = sc[lane * kMaxG + h];
      const float m = wave_max(sv);
      const float e = __expf(sv - m);   // rows >= n hold -inf -> 0
      const float l = wave_sum(e);
      sc[lane * kMaxG + h] = e;
      if (lane == 0) {
        mx[h] = m;
        lsum[h] = l;
      }
    }
  }
  __syncthreads();

  float* part = p.part + (hq0 * (p.Sw + p.Sm) + blockIdx.x) * p.rec;
  const size_t part_h = static_cast<size_t>(p.Sw + p.Sm) * p.rec;
  if (tid < G) {
    part[tid * part_h + 0] = mx[tid];
    part[tid * part_h + 1] = lsum[tid];
  }

  FA_STAMP(4);
  // sum_j p_j V[j,:]
  for (int hg = 0; hg < G; hg += 4) {
    float acc[4][8];
#pragma unroll
    for (int hh = 0; hh < 4; ++hh)
#pragma unroll
      for (int e = 0; e < 8; ++e) acc[hh][e] = 0.0f;
    if (active) {
#pragma unroll
      for (int r = 0; r < kMaxRows; ++r) {
        const int j = ts + r * nts;
        if (r * nts < kWChunk && j < n) {
          float x[8];
          unpack8(vf[r], x);
#pragma unroll
          for (int hh = 0; hh < 4; ++hh) {
            const float pj = (hg + hh < G) ? sc[j * kMaxG + hg + hh] : 0.0f;
#pragma unroll
            for (int e = 0; e < 8; ++e) acc[hh][e] += pj * x[e];
          }
        }
      }
    }
    __syncthreads();   // previous head group's reduction is finished with `red`
    if (active) {
#pragma unroll
      for (int hh = 0; hh < 4; ++hh)
#pragma unroll
        for (int e = 0; e < 8; ++e) red[(ts * 4 + hh) * D + dc * 8 + e] = acc[hh][e];
    }
    __syncthreads();
    for (int it = tid; it < 4 * D; it += kBlock) {
      const int hh = it / D, d = it % D;
      if (hg + hh < G) {
        float v = 0.0f;
#pragma unroll 8
        for (int k = 0; k < nts; ++k) v += red[(k * 4 + hh) * D + d];
        part[(hg + hh) * part_h + 2 + d] = v;
      }
    }
  }
  FA_STAMP(5);
}

// ---------------------------------------------------------------------------
// 2b. middle rows: kept dims streamed, compressed dims through the series
// ---------------------------------------------------------------------------
template <typename T, int NCH, int DVTM>
__device__ __forceinline__ void partial_middle_rows(const DecodeParams& p, unsigned char* smem) {
  using ES = typename SeriesType<T>::type;
  constexpr int Mint = NCH * 32;
  constexpr int kPitchA = Mint * sizeof(ES) + 16;   // bytes per E_A row
  constexpr int kPitchB = kTJ * sizeof(ES) + 16;    // bytes per E_B row
  constexpr int kQLoads = kMaxG * FA_MAX_HEAD_DIM / 8 / kBlock;
  constexpr int kGLoads = kMaxG * Mint / 4 / kBlock;   // >= 1 since Mint >= 64
  // V^mu operands of a whole step are requested at once when they fit in registers (they reuse
  // the registers of the K^mu operands, which are consumed by then)
  constexpr bool kPrefetchV = DVTM <= 2;

  const int sm_idx = blockIdx.x, bh = blockIdx.y, b = bh / p.Hkv, hkv = bh % p.Hkv;
  const int G = p.G, Gp = p.Gp, KT = p.KT, D = p.D;
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);   // uniform: keeps step offsets scalar
  const int q4 = lane >> 4, r16 = lane & 15;
  const size_t hq0 = static_cast<size_t>(b) * p.Hq + hkv * G;
  const int c0 = sm_idx * p.chunk_m, c1 = min(p.N, c0 + p.chunk_m);   // chunk of middle rows
  const int wstep = KT * kTJ;                                          // rows per wave step
  const int stride = kWaves * wstep;

  // ---- LDS carve-up -------------------------------------------------------
  unsigned char* eA = smem;                                   // [kRB*16][pitchA]
  unsigned char* eB = smem + kTJ * kPitchA;                   // [Mint][pitchB]
  float* red = reinterpret_cast<float*>(smem);                // aliases everything after the loop
  unsigned char* aux = smem + p.lds_tab;
  float* gs_s = reinterpret_cast<float*>(aux);                // [Gp][Mint]
  T* qk_s = reinterpret_cast<T*>(aux + Gp * Mint * 4);        // [Gp][FA_MAX_HEAD_DIM]
  __shared__ float g0_s[kMaxG];
  __shared__ float stat_m[kWaves * 16], stat_l[kWaves * 16], mstar[kMaxG], lstar[kMaxG];

  // ---- per-lane roles ---------------------------------------------------------
  const int col_k = r16 / Gp, col_h = r16 % Gp;      // S column = (tile, head)
  const bool col_live = col_k < KT && col_h < G;
  const int DVT = (p.Dvu + 15) / 16;
  const int kpitch = (p.Dku + 7) & ~7;               // K^mu rows are padded to 8 columns
  const int kchunks = (kpitch + 31) / 32;
  const bool kragged = (kpitch & 31) != 0, vragged = (p.Dvu & 15) != 0;
  const T* kk = static_cast<const T*>(p.k_keep) + bh * p.kk_stride;
  const T* vk = static_cast<const T*>(p.v_keep) + bh * p.vk_stride;
  const int Nm1 = p.N - 1;

  // K^mu rows of one wave step, dims [32*cc, 32*cc+32): 4 tiles x 4 row blocks.
  // A step that lies wholly inside the chunk addresses its operands as (uniform
  // offset) + (one per-lane offset); the last, ragged step clamps every row into
  // the slab instead (rows past the chunk are masked at the softmax).  Columns
  // past the row pitch are zeroed in both cases.
  const uint32_t lane_k = (8u * (r16 >> 2) + (r16 & 3)) * static_cast<uint32_t>(kpitch);
  auto load_k = [&](Frag<T> (&kf)[kMaxKT][kRB], int base, int cc) {
    const int d0 = cc * 32 + 8 * q4;
    const uint32_t dcl = static_cast<uint32_t>(min(d0, kpitch - 8));
    const bool dead = kragged && d0 >= kpitch;
    if (base + wstep <= c1) {
      const T* lp = kk + (lane_k + dcl);
#pragma unroll
      for (int k = 0; k < kMaxKT; ++k) {
        if (k < KT) {
#pragma unroll
          for (int rb = 0; rb < kRB; ++rb) {
            const uint32_t urow = static_cast<uint32_t>(base + k * kTJ + 32 * (rb >> 1) + 4 * (rb & 1));
            kf[k][rb].load(lp + urow * static_cast<uint32_t>(kpitch));
            if (dead) kf[k][rb].zero();
          }
        }
      }
    } else {
#pragma unroll
      for (int k = 0; k < kMaxKT; ++k) {
        if (k < KT) {
#pragma unroll
          for (int rb = 0; rb < kRB; ++rb) {
            const int u = 32 * (rb >> 1) + 8 * (r16 >> 2) + 4 * (rb & 1) + (r16 & 3);
            const int j = min(base + k * kTJ + u, Nm1);
            kf[k][rb].load(kk + (static_cast<uint32_t>(j) * static_cast<uint32_t>(kpitch) + dcl));
            if (dead) kf[k][rb].zero();
          }
        }
      }
    }
  };
  // V^mu operand of tile k, contraction step x, dim tile dt: 8 consecutive rows of one dim.
  // Rows past the chunk are zeroed (their softmax weight is 0, but 0 * garbage must stay 0).
  const uint32_t lane_v = (static_cast<uint32_t>(q4) * static_cast<uint32_t>(p.Dvu) + r16) * 8u;
  auto load_v = [&](Frag<T>& bv, int base, bool tail, int k, int x, int dt) {
    if (!tail && !vragged) {
      const uint32_t ug = static_cast<uint32_t>((base + k * kTJ + 32 * x) >> 3);
      bv.load(vk + lane_v + (ug * static_cast<uint32_t>(p.Dvu) + 16u * dt) * 8u);
    } else {
      const int tok0 = base + k * kTJ + 32 * x + 8 * q4;   // multiple of 8
      const int dim = 16 * dt + r16;
      const uint32_t g8 = static_cast<uint32_t>(min(tok0, Nm1) >> 3);
      bv.load(vk + (g8 * static_cast<uint32_t>(p.Dvu) + static_cast<uint32_t>(min(dim, p.Dvu - 1))) * 8u);
      if (vragged && dim >= p.Dvu) bv.zero();
      if (tail && tok0 + 8 > c1) mask_tail(bv, c1 - tok0);
    }
  };

  FA_STAMP(0);
  // ---- (0) everything that comes from global memory is requested first ------------
  const int base0 = c0 + wave * wstep;
  uint8_t kmb[4], vmb[4];
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    kmb[j] = p.kmask[static_cast<size_t>(bh) * D + min(lane + 64 * j, D - 1)];
    vmb[j] = p.vmask[static_cast<size_t>(bh) * D + min(lane + 64 * j, D - 1)];
  }
  const T* q = static_cast<const T*>(p.q) + hq0 * D;
  const int nq8 = G * D / 8;
  Frag<T> qv[kQLoads];
#pragma unroll
  for (int i = 0; i < kQLoads; ++i) qv[i].load(q + 8 * min(tid + i * kBlock, nq8 - 1));
  // series coefficients of the group: G * Mint contiguous floats
  const int ng4 = G * Mint / 4;
  f32x4 gv[kGLoads];
#pragma unroll
  for (int i = 0; i < kGLoads; ++i)
    gv[i] = *reinterpret_cast<const f32x4*>(p.gs + hq0 * Mint + 4 * min(tid + i * kBlock, ng4 - 1));
  const float g0v = p.g0[hq0 + min(tid, G - 1)];
  Frag<T> kf[kMaxKT][kRB];
  if (kchunks > 0 && base0 < c1) load_k(kf, base0, 0);

  FA_STAMP(1);
  // ---- zero fills that do not depend on anything loaded ---------------------------------
  for (int it = tid; it < Gp * FA_MAX_HEAD_DIM; it += kBlock) qk_s[it] = T{};
  for (int it = tid; it < (Gp - G) * Mint; it += kBlock) gs_s[G * Mint + it] = 0.0f;

  // ---- E tables: E[u][slot] = cos/sin(2 pi n u / T), n = slot/2 + 1 ----------
  // E_A rows are stored row-block-major (row 16*rb + i holds u(rb,i)); E_B rows
  // are V-side series indices, columns are u.
  {
    const int n_max = p.M / 2;
    const float invT = 1.0f / static_cast<float>(p.T);
    for (int it = tid; it < (Mint / 2) * (kTJ / 8); it += kBlock) {
      const int o = it % (Mint / 2), ug = it / (Mint / 2);
      const int n = o + 1;
      float cs[8], sn[8];
      if (n <= n_max) {
        // phase numerator (n * u) mod T; n * u < 2^24, so one float quotient estimate is exact to +-1
        const int prod = n * (8 * ug);
        int ph = prod - static_cast<int>(static_cast<float>(prod) * invT) * p.T;
        if (ph < 0) ph += p.T;
        if (ph >= p.T) ph -= p.T;
#pragma unroll
        for (int e = 0; e < 8; ++e) {
          if constexpr (sizeof(T) == 4) {
            sincospif(2.0f * (static_cast<float>(ph) / static_cast<float>(p.T)), &sn[e], &cs[e]);
          } else {
            const float x = static_cast<float>(ph) * invT;
            sn[e] = __builtin_amdgcn_sinf(x);
            cs[e] = __builtin_amdgcn_cosf(x);
          }
          ph += n;
          if (ph >= p.T) ph -= p.T;
        }
      } else {
#pragma unroll
        for (int e = 0; e < 8; ++e) cs[e] = sn[e] = 0.0f;
      }
      // E_A: (cos, sin) of order n are slots 2o, 2o+1 of row u
      const int x = ug >> 2, a = ug & 3;
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        const int row = 16 * (2 * x + (e >> 2)) + 4 * a + (e & 3);
        ES* dst = reinterpret_cast<ES*>(eA + row * kPitchA) + 2 * o;
        if constexpr (sizeof(ES) == 4) {
          dst[0] = cs[e];
          dst[1] = sn[e];
        } else {
          *reinterpret_cast<uint32_t*>(dst) =
              __builtin_bit_cast(uint32_t, __builtin_convertvector(f32x2{cs[e], sn[e]}, f16x2));
        }
      }
      // E_B: rows iota = 32*(o/16) + (o%16) [cos], +16 [sin]; 8 consecutive u
      const int iota = 32 * (o >> 4) + (o & 15);
      Frag<ES> fc, fs;
      pack8(fc, cs);
      pack8(fs, sn);
      ES* bc = reinterpret_cast<ES*>(eB + iota * kPitchB) + 8 * ug;
      ES* bs = reinterpret_cast<ES*>(eB + (iota + 16) * kPitchB) + 8 * ug;
      if constexpr (sizeof(ES) == 4) {
#pragma unroll
        for (int e = 0; e < 8; ++e) {
          bc[e] = fc.v[e];
          bs[e] = fs.v[e];
        }
      } else {
        *reinterpret_cast<u32x4*>(bc) = fc.v;
        *reinterpret_cast<u32x4*>(bs) = fs.v;
      }
    }
  }
  FA_STAMP(2);
  uint64_t kbal[4], vbal[4];
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    kbal[j] = __ballot(kmb[j] != 0 && lane + 64 * j < D);
    vbal[j] = __ballot(vmb[j] != 0 && lane + 64 * j < D);
  }
  __syncthreads();   // the qk_s zero fill is complete before the gather below
  FA_STAMP(3);

  // ---- loaded operands into LDS ---------------------------------------------------------
#pragma unroll
  for (int i = 0; i < kQLoads; ++i) {
    const int v8 = tid + i * kBlock;
    if (v8 < nq8) {
      const int h = (8 * v8) / D, d0 = (8 * v8) % D;
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        const int r = dim_rank(kbal, d0 + e);
        if (r >= 0) qk_s[h * FA_MAX_HEAD_DIM + r] = frag_elem(qv[i], e);
      }
    }
  }
#pragma unroll
  for (int i = 0; i < kGLoads; ++i) {
    const int v4 = tid + i * kBlock;
    if (v4 < ng4) *reinterpret_cast<f32x4*>(gs_s + 4 * v4) = gv[i];
  }
  if (tid < kMaxG) g0_s[tid] = (tid < G) ? g0v : 0.0f;
  __syncthreads();
  FA_STAMP(4);

  f32x4 racc[2 * NCH];          // r' = P^T E, frame of the current step
  f32x4 oacc[DVTM];             // sum_j p_j V^mu[j,:]
#pragma unroll
  for (int t = 0; t < 2 * NCH; ++t) racc[t] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
  for (int t = 0; t < DVTM; ++t) oacc[t] = f32x4{0.f, 0.f, 0.f, 0.f};
  float m_run = -INFINITY, l_run = 0.0f;   // per S column (replicated over q4); l is a per-lane partial
  int last_base = c0;                       // origin of this wave's latest step
  const bool quad_share = Gp >= 4;          // the 4 lanes of a quad then share (tile, q4)

  bool first = true;
  for (int base = base0; base < c1; base += stride) {
    const bool tail = base + wstep > c1;
    const int next = base + stride;
    f32x4 sacc[kRB];
#pragma unroll
    for (int rb = 0; rb < kRB; ++rb) sacc[rb] = f32x4{0.f, 0.f, 0.f, 0.f};

    // -- (a) series on the K side: S += E g'(tile origin) --------------------------
    const uint32_t ph_k = phase_of(p.t0 + base + col_k * kTJ, p.ph_scale);
#pragma unroll 2
    for (int c = 0; c < NCH; ++c) {
      float gp[8];
      const float* gsrc = gs_s + col_h * Mint + 32 * c + 8 * q4;
      const uint32_t n0 = 16 * c + 4 * q4 + 1;
      float csv[4], snv[4];
      if (quad_share) {
        float cs, sn;
        phase_cs<T>((n0 + (lane & 3)) * ph_k, &cs, &sn);
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          csv[i] = quad_bcast(cs, i);
          snv[i] = quad_bcast(sn, i);
        }
      } else {
#pragma unroll
        for (int i = 0; i < 4; ++i) phase_cs<T>((n0 + i) * ph_k, &csv[i], &snv[i]);
      }
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const float gc = gsrc[2 * i], gsn = gsrc[2 * i + 1];
        gp[2 * i] = gc * csv[i] + gsn * snv[i];
        gp[2 * i + 1] = gsn * csv[i] - gc * snv[i];
      }
      Frag<ES> bg;
      pack8(bg, gp);
      if (!col_live) bg.zero();
#pragma unroll
      for (int rb = 0; rb < kRB; ++rb) {
        Frag<ES> a;
        a.load(reinterpret_cast<const ES*>(eA + (16 * rb + r16) * kPitchA) + 32 * c + 8 * q4);
        mma_k32(sacc[rb], a, bg);
      }
    }

    FA_STAMP(5);
    // -- (b) kept K dims: A = K^mu rows, B = q masked to the tile's columns ------
    for (int cc = 0; cc < kchunks; ++cc) {
      if (cc > 0) load_k(kf, base, cc);
      Frag<T> bq;
      bq.load(qk_s + col_h * FA_MAX_HEAD_DIM + cc * 32 + 8 * q4);
#pragma unroll
      for (int k = 0; k < kMaxKT; ++k) {
        if (k < KT) {
          Frag<T> bk = bq;
          if (col_k != k) bk.zero();
#pragma unroll
          for (int rb = 0; rb < kRB; ++rb) mma_k32(sacc[rb], kf[k][rb], bk);
        }
      }
    }
    // V^mu operands travel while the softmax and the V-side series run
    Frag<T> vf[kPrefetchV ? kMaxKT : 1][kXN][kPrefetchV ? DVTM : 1];
    if constexpr (kPrefetchV) {
      if (DVT > 0) {
#pragma unroll
        for (int k = 0; k < kMaxKT; ++k)
          if (k < KT)
#pragma unroll
            for (int x = 0; x < kXN; ++x)
#pragma unroll
              for (int dt = 0; dt < DVTM; ++dt)
                if (dt < DVT) load_v(vf[k][x][dt], base, tail, k, x, dt);
      }
    }

    FA_STAMP(6);
    // -- (c) online softmax per column -----------------------------------------------
    // lane (column, q4) holds rows u = 32x + 8*q4 + 4y + v  (rb = 2x + y)
    float pv[kRB][4];
    float m_tile = -INFINITY;
    const float g0 = g0_s[col_h];
#pragma unroll
    for (int rb = 0; rb < kRB; ++rb)
#pragma unroll
      for (int v = 0; v < 4; ++v) {
        const int u = 32 * (rb >> 1) + 8 * q4 + 4 * (rb & 1) + v;
        const int j = base + col_k * kTJ + u;
        const float s = (col_live && j < c1) ? (sacc[rb][v] + g0) * p.scale : -INFINITY;
        pv[rb][v] = s;
        m_tile = fmaxf(m_tile, s);
      }
    m_tile = fmaxf(m_tile, __shfl_xor(m_tile, 16, kWave));
    m_tile = fmaxf(m_tile, __shfl_xor(m_tile, 32, kWave));
    const float m_new = fmaxf(m_run, m_tile);
    const float m_ref = (m_new == -INFINITY) ? 0.0f : m_new;
    const float alpha = __expf(m_run - m_ref);   // m_run = -inf -> 0
    float l_add = 0.0f;
#pragma unroll
    for (int rb = 0; rb < kRB; ++rb)
#pragma unroll
      for (int v = 0; v < 4; ++v) {
        pv[rb][v] = __expf(pv[rb][v] - m_ref);
        l_add += pv[rb][v];
      }
    l_run = l_run * alpha + l_add;
    m_run = m_new;

    FA_STAMP(7);
    // -- (d) bring the accumulators into this step's frame --------------------------------
    if (!first) {
      // accumulator rows are S columns 4*q4 + v: fetch their rescale factors
      float al[4];
#pragma unroll
      for (int v = 0; v < 4; ++v) al[v] = __shfl(alpha, 4 * q4 + v, kWave);
#pragma unroll
      for (int t = 0; t < DVTM; ++t)
#pragma unroll
        for (int v = 0; v < 4; ++v) oacc[t][v] *= al[v];
      // r' moves to the new origin: rotate every (cos, sin) pair by -omega_n * stride
      const uint32_t ph_d = phase_of(stride, p.ph_scale);
#pragma unroll
      for (int t = 0; t < NCH; ++t) {
        float cs, sn;
        phase_cs<T>(static_cast<uint32_t>(16 * t + r16 + 1) * ph_d, &cs, &sn);
#pragma unroll
        for (int v = 0; v < 4; ++v) {
          const float rc = racc[2 * t][v], rs = racc[2 * t + 1][v];
          racc[2 * t][v] = al[v] * (cs * rc + sn * rs);
          racc[2 * t + 1][v] = al[v] * (cs * rs - sn * rc);
        }
      }
    }
    first = false;
    last_base = base;

    // -- (e) V side: r' += P^T E, O += P^T V^mu ---------------------------------------------
    Frag<T> pt[kXN];
#pragma unroll
    for (int x = 0; x < kXN; ++x) {
      float pe[8];
#pragma unroll
      for (int e = 0; e < 8; ++e) pe[e] = pv[2 * x + (e >> 2)][e & 3];
      Frag<ES> ps;
      pack8(ps, pe);
      pack8(pt[x], pe);
#pragma unroll
      for (int t = 0; t < 2 * NCH; ++t) {
        Frag<ES> eb;
        eb.load(reinterpret_cast<const ES*>(eB + (16 * t + r16) * kPitchB) + 32 * x + 8 * q4);
        mma_k32(racc[t], ps, eb);
        // keep the table reads next to their MFMAs: hoisting all of them costs ~4 registers each
        if ((t & 3) == 3) __builtin_amdgcn_sched_barrier(0);
      }
    }
    FA_STAMP(8);
    if (DVT > 0) {
#pragma unroll
      for (int k = 0; k < kMaxKT; ++k) {
        if (k < KT) {
#pragma unroll
          for (int x = 0; x < kXN; ++x) {
            Frag<T> ak = pt[x];
            if (col_k != k) ak.zero();
            if constexpr (kPrefetchV) {
#pragma unroll
              for (int dt = 0; dt < DVTM; ++dt)
                if (dt < DVT) mma_k32(oacc[dt], ak, vf[k][x][dt]);
            } else {
              Frag<T> bv[DVTM];
#pragma unroll
              for (int dt = 0; dt < DVTM; ++dt)
                if (dt < DVT) load_v(bv[dt], base, tail, k, x, dt);
#pragma unroll
              for (int dt = 0; dt < DVTM; ++dt)
                if (dt < DVT) mma_k32(oacc[dt], ak, bv[dt]);
            }
          }
        }
      }
    }
    // the K operands of this wave's next step travel during its series evaluation
    if (kchunks > 0 && next < c1) load_k(kf, next, 0);
  }

  FA_STAMP(9);
  // ---- merge tiles and waves --------------------------------------------------------------
  l_run += __shfl_xor(l_run, 16, kWave);
  l_run += __shfl_xor(l_run, 32, kWave);
  if (q4 == 0) {
    stat_m[wave * 16 + r16] = col_live ? m_run : -INFINITY;
    stat_l[wave * 16 + r16] = col_live ? l_run : 0.0f;
  }
  __syncthreads();   // also: every wave is done with the E tables and the aux region
  FA_STAMP(10);
  if (tid < G) {
    float m = -INFINITY;
    for (int w = 0; w < kWaves; ++w)
      for (int k = 0; k < KT; ++k) m = fmaxf(m, stat_m[w * 16 + k * Gp + tid]);
    float l = 0.0f;
    for (int w = 0; w < kWaves; ++w)
      for (int k = 0; k < KT; ++k) {
        const float mm = stat_m[w * 16 + k * Gp + tid];
        if (mm != -INFINITY) l += stat_l[w * 16 + k * Gp + tid] * __expf(mm - m);
      }
    mstar[tid] = m;
    lstar[tid] = l;
  }
  __syncthreads();

  // every wave rotates its r' rows to the global frame, scales rows to the chunk
  // maximum and parks them in LDS: red[wave][row][Mint + 16*DVT]
  const int redw = Mint + 16 * DVT;
  {
    float f[4];
    uint32_t phr[4];
#pragma unroll
    for (int v = 0; v < 4; ++v) {
      const int row = 4 * q4 + v, k = row / Gp, h = row % Gp;
      const float mm = stat_m[wave * 16 + row];
      f[v] = (k < KT && h < G && mm != -INFINITY) ? __expf(mm - mstar[h]) : 0.0f;
      phr[v] = phase_of(p.t0 + last_base + k * kTJ, p.ph_scale);
    }
    float* dst = red + static_cast<size_t>(wave) * 16 * redw;
#pragma unroll
    for (int t = 0; t < NCH; ++t) {
      const uint32_t n = 16 * t + r16 + 1;
      float cs[4], sn[4];
      phase_cs<T>(n * phr[0], &cs[0], &sn[0]);
      if (quad_share) {   // rows 4*q4 .. 4*q4+3 belong to one tile
#pragma unroll
        for (int v = 1; v < 4; ++v) {
          cs[v] = cs[0];
          sn[v] = sn[0];
        }
      } else {
#pragma unroll
        for (int v = 1; v < 4; ++v) phase_cs<T>(n * phr[v], &cs[v], &sn[v]);
      }
#pragma unroll
      for (int v = 0; v < 4; ++v) {
        const float rc = racc[2 * t][v], rs = racc[2 * t + 1][v];
        const int row = 4 * q4 + v;
        dst[row * redw + 32 * t + r16] = f[v] * (cs[v] * rc - sn[v] * rs);
        dst[row * redw + 32 * t + 16 + r16] = f[v] * (sn[v] * rc + cs[v] * rs);
      }
    }
#pragma unroll
    for (int dt = 0; dt < DVTM; ++dt)
      if (dt < DVT)
#pragma unroll
        for (int v = 0; v < 4; ++v)
          dst[(4 * q4 + v) * redw + Mint + 16 * dt + r16] = f[v] * oacc[dt][v];
  }
  __syncthreads();
  FA_STAMP(11);

  float* part = p.part + (hq0 * (p.Sw + p.Sm) + blockIdx.x) * p.rec;
  const size_t part_h = static_cast<size_t>(p.Sw + p.Sm) * p.rec;
  if (tid < G) {
    part[tid * part_h + 0] = mstar[tid];
    part[tid * part_h + 1] = lstar[tid];
  }
  // r[h][iota] and acc[h][dim] = sum over waves and tiles
  for (int it = tid; it < G * (D + Mint); it += kBlock) {
    const int h = it / (D + Mint), x = it % (D + Mint);
    int src;   // column of the reduction rows, or -1 for a dim that middle rows do not carry
    if (x < D) {
      const int r = dim_rank(vbal, x);
      src = (r >= 0) ? Mint + r : -1;
    } else {
      src = x - D;
    }
    float v = 0.0f;
    if (src >= 0) {
#pragma unroll
      for (int w = 0; w < kWaves; ++w)
#pragma unroll
        for (int k = 0; k < kMaxKT; ++k)
          if (k < KT) v += red[(w * 16 + k * Gp + h) * redw + src];
    }
    part[h * part_h + 2 + x] = v;
  }
  FA_STAMP(12);
}

template <typename T, int NCH, int DVTM>
__global__ __launch_bounds__(kBlock) void decode_partial(DecodeParams p) {
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  if (static_cast<int>(blockIdx.x) < p.Sm) partial_middle_rows<T, NCH, DVTM>(p, smem);
  else partial_full_rows<T>(p, smem);
}

// ---------------------------------------------------------------------------
// 3. merge partials, apply diag(w) C_v, normalise: one workgroup per query head
// ---------------------------------------------------------------------------
template <typename T>
__global__ __launch_bounds__(kFinBlock) void decode_finish(DecodeParams p) {
  __shared__ float rr[FA_MAX_DECODE_STATES];   // r in basis order, weighted
  __shared__ float accs[FA_MAX_HEAD_DIM];
  __shared__ float es[kMaxPartials];
  __shared__ float red[kFinBlock];
  __shared__ float wred[kFinBlock / 64];
  __shared__ float stat[2];

  const int hq = blockIdx.x, b = hq / p.Hq, hkv = (hq % p.Hq) / p.G;
  const int bh = b * p.Hkv + hkv;
  const int D = p.D, M = p.M, S = p.Sw + p.Sm, Dvc = p.Dvc;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  constexpr int kNW = kFinBlock / 64;
  const float* part = p.part + static_cast<size_t>(hq) * S * p.rec;
  const size_t rec = p.rec;

  // ---- every global operand is requested before anything is consumed -------------------
  // (1) chunk maxima and sums
  const int s_me = min(tid, S - 1);
  const float ms_me = part[s_me * rec], ls_me = part[s_me * rec + 1];
  // (2) acc[d] over chunks: thread (d, group ga) takes chunks ga, ga+nga, ...
  constexpr int kU = 8;
  const int nga = kFinBlock / D;
  const int d_a = tid % D, ga = tid / D;
  float av[kU];
#pragma unroll
  for (int u = 0; u < kU; ++u) av[u] = part[min(ga + u * nga, S - 1) * rec + 2 + d_a];
  // (3) r[m] over middle chunks: thread (m, group gr)
  const int ngr = kFinBlock / M;   // M <= 512
  const int m_r = tid % M, gr = tid / M;
  int col_r;   // record column of basis function m_r
  if (m_r == 0) {
    col_r = 1;   // constant function: r_0 = sum of p over the middle rows = the chunk sums
  } else {
    const int n = (m_r + 1) / 2, cs = (m_r & 1) ? 0 : 1;   // odd m: cosine
    col_r = 2 + D + 32 * ((n - 1) >> 4) + 16 * cs + ((n - 1) & 15);
  }
  float rv[kU];
#pragma unroll
  for (int u = 0; u < kU; ++u) rv[u] = part[min(gr + u * ngr, max(p.Sm - 1, 0)) * rec + col_r];
  // (4) C_v rows: thread (4 columns c4, row group) takes rows rg, rg+nrg, ...
  const bool vec4 = (Dvc % 4) == 0 && Dvc > 0;
  const int ncol = vec4 ? Dvc / 4 : max(Dvc, 1);
  const int nrg = kFinBlock / ncol;
  const int c4 = tid % ncol, rg = tid / ncol;
  const float* cv = p.cv + static_cast<size_t>(bh) * M * Dvc;
  constexpr int kCU = 16;
  f32x4 cvv[kCU];
  const bool do_cv = p.Sm > 0 && Dvc > 0;
  if (do_cv) {
#pragma unroll
    for (int u = 0; u < kCU; ++u) {
      const int mm = min(rg + u * nrg, M - 1);
      if (vec4) cvv[u] = *reinterpret_cast<const f32x4*>(cv + static_cast<size_t>(mm) * Dvc + 4 * c4);
      else cvv[u] = f32x4{cv[static_cast<size_t>(mm) * Dvc + c4], 0.f, 0.f, 0.f};
    }
  }
  uint64_t vbal[4];
  mask_ballots(p.vmask + static_cast<size_t>(bh) * D, D, lane, vbal);

  // ---- global max and per-chunk factors ---------------------------------------------------
  float m = (tid < S) ? ms_me : -INFINITY;
  for (int s = tid + kFinBlock; s < S; s += kFinBlock) m = fmaxf(m, part[s * rec]);
  m = wave_max(m);
  if (lane == 0) wred[wave] = m;
  __syncthreads();
  m = wred[0];
#pragma unroll
  for (int w = 1; w < kNW; ++w) m = fmaxf(m, wred[w]);
  float l = 0.0f;
  if (tid < S) {
    const float e = (ms_me == -INFINITY) ? 0.0f : __expf(ms_me - m);
    es[tid] = e;
    l = e * ls_me;
  }
  l = wave_sum(l);
  __syncthreads();   // wred reads above are finished
  if (lane == 0) wred[wave] = l;
  __syncthreads();
  if (tid == 0) {
    float t = 0.0f;
    for (int w = 0; w < kNW; ++w) t += wred[w];
    stat[0] = t;
  }

  // ---- acc[d] ---------------------------------------------------------------------------------
  {
    float a = 0.0f;
#pragma unroll
    for (int u = 0; u < kU; ++u) {
      const int s = ga + u * nga;
      if (s < S) a += es[s] * av[u];
    }
    for (int s = ga + kU * nga; s < S; s += nga) a += es[s] * part[s * rec + 2 + d_a];
    red[tid] = (ga < nga) ? a : 0.0f;
  }
  __syncthreads();
  if (tid < D) {
    float a = 0.0f;
    for (int g = 0; g < nga; ++g) a += red[g * D + tid];
    accs[tid] = a;
  }
  __syncthreads();
  // ---- r[m] -----------------------------------------------------------------------------------
  {
    float a = 0.0f;
#pragma unroll
    for (int u = 0; u < kU; ++u) {
      const int s = gr + u * ngr;
      if (s < p.Sm) a += es[s] * rv[u];
    }
    for (int s = gr + kU * ngr; s < p.Sm; s += ngr) a += es[s] * part[s * rec + col_r];
    red[tid] = (gr < ngr) ? a : 0.0f;
  }
  __syncthreads();
  if (tid < M) {
    float a = 0.0f;
    for (int g = 0; g < ngr; ++g) a += red[g * M + tid];
    rr[tid] = a * basis_weight((tid + 1) / 2, p.T);
  }
  __syncthreads();

  // ---- o[idx_vc[i]] += sum_m rr[m] C_v[m,i] ---------------------------------------------------
  if (do_cv) {
    f32x4 a = {0.f, 0.f, 0.f, 0.f};
    if (rg < nrg) {
#pragma unroll
      for (int u = 0; u < kCU; ++u) {
        const int mm = rg + u * nrg;
        if (mm < M) a += rr[mm] * cvv[u];
      }
      for (int mm = rg + kCU * nrg; mm < M; mm += nrg) {
        if (vec4) a += rr[mm] * *reinterpret_cast<const f32x4*>(cv + static_cast<size_t>(mm) * Dvc + 4 * c4);
        else a[0] += rr[mm] * cv[static_cast<size_t>(mm) * Dvc + c4];
      }
    }
    // reduce over row groups, one component at a time
    const int ncomp = vec4 ? 4 : 1;
    for (int comp = 0; comp < ncomp; ++comp) {
      __syncthreads();
      red[tid] = (rg < nrg) ? a[comp] : 0.0f;
      __syncthreads();
      if (tid < D) {
        const int r = dim_rank(vbal, tid);
        if (r < 0) {
          const int ci = -r - 1;
          const bool mine = vec4 ? ((ci & 3) == comp) : true;
          if (mine) {
            const int col = vec4 ? (ci >> 2) : ci;
            float v = 0.0f;
            for (int g = 0; g < nrg; ++g) v += red[g * ncol + col];
            accs[tid] += v;
          }
        }
      }
    }
  }
  __syncthreads();
  if (tid < D) p.out[static_cast<size_t>(hq) * D + tid] = accs[tid] / stat[0];
}

// ---------------------------------------------------------------------------
// host side
// ---------------------------------------------------------------------------
struct DecodePlan {
  int Gp, KT, Mint, nch, Sw, Sm, chunk_m, rec;
  unsigned lds_tab, lds_total;
  size_t off_gs, off_g0, off_part, total;
};

static int round_up(int x, int a) { return (x + a - 1) / a * a; }

static int series_chunks(int M) {   // compiled series lengths: 64, 128, 256, 512
  const int slots = 2 * (M / 2);
  const int need = slots > 0 ? (slots + 31) / 32 : 1;
  for (int n : {2, 4, 8, 16})
    if (need <= n) return n;
  return 0;
}

static int default_steps_per_chunk(int B, int Hkv, int N, int wg_step) {
  const long total_steps = static_cast<long>(B) * Hkv * ((N + wg_step - 1) / wg_step);
  long spc = (total_steps + 128) / 256;   // about one workgroup per compute unit
  if (spc < 1) spc = 1;
  if (spc > 16) spc = 16;
  return static_cast<int>(spc);
}

static bool make_plan(DecodePlan& pl, int dtype, int B, int Hq, int Hkv, int D, int Dvc, int M,
                      int N, int W, int num_splits) {
  const int G = Hq / Hkv;
  pl.Gp = 1;
  while (pl.Gp < G) pl.Gp *= 2;
  pl.KT = 16 / pl.Gp < kMaxKT ? 16 / pl.Gp : kMaxKT;
  pl.nch = series_chunks(M);
  if (pl.nch == 0) return false;
  pl.Mint = pl.nch * 32;
  const int wg_step = kWaves * pl.KT * kTJ;
  pl.Sw = (W + kWChunk - 1) / kWChunk;
  if (N > 0) {
    int chunk;
    if (num_splits > 0) chunk = round_up((N + num_splits - 1) / num_splits, wg_step);
    else chunk = default_steps_per_chunk(B, Hkv, N, wg_step) * wg_step;
    pl.chunk_m = chunk;
    pl.Sm = (N + chunk - 1) / chunk;
  } else {
    pl.chunk_m = wg_step;
    pl.Sm = 0;
  }
  if (pl.Sw + pl.Sm > kMaxPartials) return false;
  pl.rec = 2 + D + pl.Mint;
  const unsigned es = (dtype == FA_F32) ? 4 : 2;   // bytes of a table entry
  const unsigned ts = (dtype == FA_F32) ? 4 : 2;   // bytes of a K/V element
  const unsigned tab = kTJ * (pl.Mint * es + 16) + pl.Mint * (kTJ * es + 16);
  pl.lds_tab = (tab + 255u) & ~255u;
  const unsigned mid = pl.lds_tab + pl.Gp * pl.Mint * 4 + pl.Gp * FA_MAX_HEAD_DIM * ts;
  const unsigned DVT = (D - Dvc + 15) / 16;
  const unsigned redb = kWaves * 16 * (pl.Mint + 16 * DVT) * 4;
  const unsigned wpath = 16 * FA_MAX_HEAD_DIM * ts + kWChunk * kMaxG * 4 + kBlock * 8 * 4 * 4;
  unsigned t = mid > redb ? mid : redb;
  if (wpath > t) t = wpath;
  pl.lds_total = (t + 255u) & ~255u;
  if (pl.lds_total > kMaxDynLds) return false;
  pl.off_gs = 0;
  pl.off_g0 = align_up(static_cast<size_t>(B) * Hq * pl.Mint * sizeof(float), 256);
  pl.off_part = pl.off_g0 + align_up(static_cast<size_t>(B) * Hq * sizeof(float), 256);
  pl.total = pl.off_part +
             align_up(static_cast<size_t>(B) * Hq * (pl.Sw + pl.Sm) * pl.rec * sizeof(float), 256);
#ifdef FA_TRACE
  pl.total += static_cast<size_t>(B) * Hkv * (pl.Sw + pl.Sm) * 4 * 16 * sizeof(long long);
#endif
  return true;
}

static int check_decode_shapes(int dtype, int B, int Hq, int Hkv, int D, int Dkc, int Dvc, int M,
                               int T, int t0, int N, int W, int num_splits) {
  if (dtype != FA_F32 && dtype != FA_BF16) return FA_ERR_UNSUPPORTED;
  if (B <= 0 || Hq <= 0 || Hkv <= 0 || D <= 0 || Hq % Hkv != 0) return FA_ERR_SHAPE;
  if (Dkc < 0 || Dkc > D || Dvc < 0 || Dvc > D) return FA_ERR_SHAPE;
  if (N < 0 || W < 0 || static_cast<long>(N) + W <= 0) return FA_ERR_SHAPE;
  if (M < 1 || T < 1 || M > T || t0 < 0 || static_cast<long>(t0) + N > T) return FA_ERR_SHAPE;
  if (num_splits < 0) return FA_ERR_SHAPE;
  if (D % 8 != 0 || D > FA_MAX_HEAD_DIM) return FA_ERR_UNSUPPORTED;
  if (Hq / Hkv > FA_MAX_GROUP || M > FA_MAX_DECODE_STATES || num_splits > FA_MAX_SPLITS)
    return FA_ERR_UNSUPPORTED;
  if (dtype == FA_F32 && M > FA_MAX_DECODE_STATES / 2) return FA_ERR_UNSUPPORTED;
  if (D - Dvc > 16 * kMaxDvTiles) return FA_ERR_UNSUPPORTED;
  if (static_cast<long>(B) * Hkv > 65535) return FA_ERR_UNSUPPORTED;
  return FA_OK;
}

template <typename T, int NCH, int DVTM>
static int launch_partial(const DecodeParams& p, unsigned lds, hipStream_t st) {
  auto kern = decode_partial<T, NCH, DVTM>;
  // raising the dynamic-LDS ceiling is a property of the loaded kernel: do it once
  static unsigned granted = 48 * 1024;
  if (lds > granted) {
    if (hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                            hipFuncAttributeMaxDynamicSharedMemorySize,
                            static_cast<int>(kMaxDynLds)) != hipSuccess)
      return FA_ERR_HIP;
    granted = kMaxDynLds;
  }
  dim3 g2(p.Sw + p.Sm, p.B * p.Hkv);
  hipLaunchKernelGGL(kern, g2, dim3(kBlock), lds, st, p);
  return FA_OK;
}

// ev (optional): 4 events recorded before/after each kernel, for fa_decode_timed
template <typename T>
static int launch_decode(const DecodeParams& p, const DecodePlan& pl, hipStream_t st, hipEvent_t* ev) {
  const int BH = p.B * p.Hkv;
  if (ev) (void)hipEventRecord(ev[0], st);
  if (p.Sm > 0) {
    dim3 g1((p.Mint + 1 + kPrepRows - 1) / kPrepRows, BH);
    hipLaunchKernelGGL(decode_prepare<T>, g1, dim3(kBlock), 0, st, p);
  }
  if (ev) (void)hipEventRecord(ev[1], st);
  int rc;
  const bool narrow = p.Dvu <= 32;   // kept V dims fit two MFMA column tiles
#define FA_LAUNCH_PARTIAL(NCH_)                                                     \
  rc = narrow ? launch_partial<T, NCH_, 2>(p, pl.lds_total, st)                     \
              : launch_partial<T, NCH_, kMaxDvTiles>(p, pl.lds_total, st)
  switch (pl.nch) {
    case 2: FA_LAUNCH_PARTIAL(2); break;
    case 4: FA_LAUNCH_PARTIAL(4); break;
    case 8: FA_LAUNCH_PARTIAL(8); break;
    default:
      if constexpr (sizeof(T) == 2) {
        FA_LAUNCH_PARTIAL(16);
      } else {
        rc = FA_ERR_UNSUPPORTED;
      }
      break;
  }
#undef FA_LAUNCH_PARTIAL
  if (rc != FA_OK) return rc;
  if (ev) (void)hipEventRecord(ev[2], st);
  hipLaunchKernelGGL(decode_finish<T>, dim3(p.B * p.Hq), dim3(kFinBlock), 0, st, p);
  if (ev) (void)hipEventRecord(ev[3], st);
  return hipGetLastError() == hipSuccess ? FA_OK : FA_ERR_HIP;
}

}  // namespace fa

extern "C" {

int fa_decode_default_splits(int B, int Hq, int Hkv, int N) {
  if (B <= 0 || Hq <= 0 || Hkv <= 0 || N <= 0 || Hq % Hkv != 0 || Hq / Hkv > FA_MAX_GROUP) return 0;
  fa::DecodePlan pl{};
  if (!fa::make_plan(pl, FA_BF16, B, Hq, Hkv, 128, 0, 2, N, 0, 0)) return 0;
  return pl.Sm;
}

size_t fa_decode_workspace_bytes(int B, int Hq, int Hkv, int D, int Dkc, int Dvc, int M, int N,
                                 int W, int num_splits) {
  if (fa::check_decode_shapes(FA_BF16, B, Hq, Hkv, D, Dkc, Dvc, M, M > N ? M : N, 0, N, W,
                              num_splits) != FA_OK)
    return 0;
  fa::DecodePlan pl{};
  if (!fa::make_plan(pl, FA_BF16, B, Hq, Hkv, D, Dvc, M, N, W, num_splits)) return 0;
  return pl.total;
}

static int decode_impl(const void* q, int dtype, int B, int Hq, int Hkv, int D, const float* ck,
                       const uint8_t* kmask, int Dkc, const float* cv, const uint8_t* vmask, int Dvc,
                       int M, int T, int t0, int N, const void* k_keep, int64_t kk_stride_bh,
                       const void* v_keep, int64_t vk_stride_bh, const void* k_full,
                       const void* v_full, int W, int64_t full_stride_bh, float scale,
                       int num_splits, float* out, void* workspace, size_t workspace_bytes,
                       void* hip_stream, hipEvent_t* ev) {
  using namespace fa;
  const int st = check_decode_shapes(dtype, B, Hq, Hkv, D, Dkc, Dvc, M, T, t0, N, W, num_splits);
  if (st != FA_OK) return st;
  if (!q || !kmask || !vmask || !out || !workspace) return FA_ERR_NULL;
  const int Dku = D - Dkc, Dvu = D - Dvc;
  if (N > 0) {
    if ((Dkc > 0 && !ck) || (Dvc > 0 && !cv)) return FA_ERR_NULL;
    if ((Dku > 0 && !k_keep) || (Dvu > 0 && !v_keep)) return FA_ERR_NULL;
  }
  if (W > 0 && (!k_full || !v_full)) return FA_ERR_NULL;
  const int64_t kk_dense = static_cast<int64_t>(N) * ((Dku + 7) & ~7);
  const int64_t vk_dense = static_cast<int64_t>((N + 7) / 8) * 8 * Dvu;
  const int64_t full_dense = static_cast<int64_t>(W) * D;
  if (kk_stride_bh == 0) kk_stride_bh = kk_dense;
  if (vk_stride_bh == 0) vk_stride_bh = vk_dense;
  if (full_stride_bh == 0) full_stride_bh = full_dense;
  if (kk_stride_bh < kk_dense || vk_stride_bh < vk_dense || full_stride_bh < full_dense)
    return FA_ERR_SHAPE;
  // vector loads need 16-byte aligned slabs
  if ((vk_stride_bh % 8) || (full_stride_bh % 8) || (kk_stride_bh % 8)) return FA_ERR_SHAPE;
  if ((reinterpret_cast<uintptr_t>(k_keep) | reinterpret_cast<uintptr_t>(v_keep) |
       reinterpret_cast<uintptr_t>(k_full) | reinterpret_cast<uintptr_t>(v_full) |
       reinterpret_cast<uintptr_t>(q) | reinterpret_cast<uintptr_t>(cv)) & 15u)
    return FA_ERR_SHAPE;
  // kernels index slabs with 32-bit element offsets
  if (kk_dense > 0x7fffffffLL || vk_dense > 0x7fffffffLL || full_dense > 0x7fffffffLL)
    return FA_ERR_UNSUPPORTED;

  DecodePlan pl{};
  if (!make_plan(pl, dtype, B, Hq, Hkv, D, Dvc, M, N, W, num_splits)) return FA_ERR_UNSUPPORTED;
  if (workspace_bytes < pl.total || (reinterpret_cast<uintptr_t>(workspace) & 255u))
    return FA_ERR_WORKSPACE;

  DecodeParams p{};
  p.q = q; p.ck = ck; p.cv = cv; p.kmask = kmask; p.vmask = vmask;
  p.k_keep = k_keep; p.v_keep = v_keep; p.k_full = k_full; p.v_full = v_full;
  p.kk_stride = kk_stride_bh; p.vk_stride = vk_stride_bh; p.full_stride = full_stride_bh;
  p.B = B; p.Hq = Hq; p.Hkv = Hkv; p.G = Hq / Hkv; p.D = D;
  p.Dkc = Dkc; p.Dvc = Dvc; p.Dku = Dku; p.Dvu = Dvu;
  p.M = M; p.T = T; p.t0 = t0; p.N = N; p.W = W;
  p.Gp = pl.Gp; p.KT = pl.KT; p.Mint = pl.Mint;
  p.Sw = pl.Sw; p.Sm = pl.Sm; p.chunk_m = pl.chunk_m; p.rec = pl.rec;
  p.lds_tab = pl.lds_tab;
  p.scale = scale > 0.0f ? scale : 1.0f / sqrtf(static_cast<float>(D));
  p.ph_scale = 4294967296.0 / static_cast<double>(T);
  char* ws = static_cast<char*>(workspace);
  p.gs = reinterpret_cast<float*>(ws + pl.off_gs);
  p.g0 = reinterpret_cast<float*>(ws + pl.off_g0);
  p.part = reinterpret_cast<float*>(ws + pl.off_part);
  p.out = out;
#ifdef FA_TRACE
  p.trace = reinterpret_cast<long long*>(
      ws + pl.off_part + align_up(static_cast<size_t>(B) * Hq * (pl.Sw + pl.Sm) * pl.rec * sizeof(float), 256));
#endif
  hipStream_t stream = static_cast<hipStream_t>(hip_stream);
  return dtype == FA_F32 ? launch_decode<float>(p, pl, stream, ev)
                         : launch_decode<bf16_t>(p, pl, stream, ev);
}

int fa_decode(const void* q, int dtype, int B, int Hq, int Hkv, int D, const float* ck,
              const uint8_t* kmask, int Dkc, const float* cv, const uint8_t* vmask, int Dvc, int M,
              int T, int t0, int N, const void* k_keep, int64_t kk_stride_bh, const void* v_keep,
              int64_t vk_stride_bh, const void* k_full, const void* v_full, int W,
              int64_t full_stride_bh, float scale, int num_splits, float* out, void* workspace,
              size_t workspace_bytes, void* hip_stream) {
  return decode_impl(q, dtype, B, Hq, Hkv, D, ck, kmask, Dkc, cv, vmask, Dvc, M, T, t0, N, k_keep,
                     kk_stride_bh, v_keep, vk_stride_bh, k_full, v_full, W, full_stride_bh, scale,
                     num_splits, out, workspace, workspace_bytes, hip_stream, nullptr);
}

int fa_decode_timed(const void* q, int dtype, int B, int Hq, int Hkv, int D, const float* ck,
                    const uint8_t* kmask, int Dkc, const float* cv, const uint8_t* vmask, int Dvc,
                    int M, int T, int t0, int N, const void* k_keep, int64_t kk_stride_bh,
                    const void* v_keep, int64_t vk_stride_bh, const void* k_full,
                    const void* v_full, int W, int64_t full_stride_bh, float scale, int num_splits,
                    float* out, void* workspace, size_t workspace_bytes, void* hip_stream,
                    float* kernel_ms) {
  if (!kernel_ms) return FA_ERR_NULL;
  hipEvent_t ev[4];
  for (int i = 0; i < 4; ++i)
    if (hipEventCreate(&ev[i]) != hipSuccess) return FA_ERR_HIP;
  int st = decode_impl(q, dtype, B, Hq, Hkv, D, ck, kmask, Dkc, cv, vmask, Dvc, M, T, t0, N, k_keep,
                       kk_stride_bh, v_keep, vk_stride_bh, k_full, v_full, W, full_stride_bh, scale,
                       num_splits, out, workspace, workspace_bytes, hip_stream, ev);
  if (st == FA_OK) {
    if (hipEventSynchronize(ev[3]) != hipSuccess) st = FA_ERR_HIP;
    for (int i = 0; i < 3 && st == FA_OK; ++i)
      if (hipEventElapsedTime(&kernel_ms[i], ev[i], ev[i + 1]) != hipSuccess) st = FA_ERR_HIP;
  }
  for (int i = 0; i < 4; ++i) (void)hipEventDestroy(ev[i]);
  return st;
}

}  // extern "C"
