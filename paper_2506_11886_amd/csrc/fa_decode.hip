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
// chunk.  The table is split by harmonics over the four waves of a workgroup
// and lives in registers.
//
// The kernels are latency-shaped: a decode step moves only tens of megabytes,
// so every kernel requests all of its global-memory operands up front (one
// dependent round trip) and hides them behind table construction and MFMAs.
//
// Launches on the caller's stream:
//   1. decode_prepare : g (series order) for every query head, from C_k and q;
//      q at the kept K dims, packed.
//   2. decode_partial : one workgroup per (sequence, KV head, token chunk);
//      chunks of middle rows and chunks of full-width sink/window rows; emits
//      a flash-decoding partial per query head: (max, sum, acc[kept dims],
//      r[Mint]) for middle rows, (max, sum, acc[D]) for full-width rows.
//   3. decode_finish  : a few workgroups per query head (one per slice of output dims) merge the partials,
//      applies diag(w) C_v to r and normalises.

#include <cstdlib>
#include <mutex>
#include <type_traits>

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
constexpr int kWChunk = 256;       // full-width rows per workgroup
constexpr int kMaxDvTiles = 8;     // kept V dims handled per middle row: 8 * 16
constexpr int kMaxPartials = 1024; // partial records per query head
constexpr unsigned kMaxDynLds = 160 * 1024 - 4096;   // dynamic LDS a workgroup may ask for
constexpr int kFinBlock = 256;     // threads of decode_finish

typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef _Float16 f16x2 __attribute__((ext_vector_type(2)));
typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef uint32_t u32x2d __attribute__((ext_vector_type(2)));


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
  int Tq, Gq;       // query tokens per sequence (1: plain decode) and query heads per KV head and token
  int Gp, KT;       // group size padded to a power of two, tiles per wave step
  int Mint;         // series length: 2 * (M/2) padded to a compiled size
  int Sw, Sm;       // chunks of full-width rows / of middle rows (middle chunks come first)
  int nprep, Swp;   // workgroups per head of the series-coefficient part when the full-width rows share its launch;
                    // chunks of full-width rows inside the middle-row launch (0 when they ran with the coefficients)
  int chunk_m;      // middle rows per chunk (multiple of the workgroup step)
  int recm, recw;   // floats per partial record: 4 + 16 ceil(Dvu/16) + Mint (middle), 4 + D (full rows)
  unsigned lds_tab; // bytes of the exchange / reduction region of a middle-row workgroup
  float scale;
  double ph_scale;  // 2^32 / T
  float* gs;        // [B,Hq,Mint] series coefficients, K-side order
  float* g0;        // [B,Hq]      constant-term coefficient
  void* qkeep;      // [B,Hq,Dkq]  q at the kept K dims, zero padded to Dkq = 32 ceil(Dku/32)
  float* part_m;    // [B,Hq,Sm,recm]
  float* part_w;    // [B,Hq,Sw,recw]
  float* out;       // [B,Hq,D]
  const int32_t* seq_n;   // [B] middle rows of each sequence (<= N), or null: N for all
  const int32_t* seq_w;   // [B] full-width rows of each sequence (<= W), or null: W for all
  int Sw_rec;       // full-row records reserved per query head (= Sw of the longest sequence)
  int wrb;          // 16-row blocks per wave of a full-width-row workgroup: 4 (256 rows per workgroup) or 1 (64)
};

// What a workgroup uses of one sequence: its row counts, the chunking that follows from them and
// where its records go.  The three-launch kernels take the call's own values; the one-launch form
// resolves them per sequence.
struct SeqView {
  int N, W, Sm, Sw, chunk_m;
  float* part_m;
  float* part_w;
};
// rows of sequence b: the call's counts, or the sequence's own (clamped into them) when the caller gave lists
__device__ __forceinline__ int seq_middle_rows(const DecodeParams& p, int b) {
  return p.seq_n ? min(max(p.seq_n[b], 0), p.N) : p.N;
}
__device__ __forceinline__ int seq_full_rows(const DecodeParams& p, int b) {
  return p.seq_w ? min(max(p.seq_w[b], 0), p.W) : p.W;
}
__device__ __forceinline__ SeqView call_view(const DecodeParams& p, int b) {
  return SeqView{seq_middle_rows(p, b), seq_full_rows(p, b), p.Sm, p.Sw, p.chunk_m, p.part_m, p.part_w};
}

// Middle-row chunks [chunk_lo, chunk_hi) of a (sequence, KV head) that lie past the sequence's rows:
// records that say "nothing here" (maximum -inf, everything else zero), for every query head.
__device__ __forceinline__ void write_empty_middle(const DecodeParams& p, size_t hq0, int chunk_lo, int chunk_hi,
                                                   int nthreads) {
  const int recm = p.recm, G = p.G;
  const int per = (chunk_hi - chunk_lo) * recm;
  for (int it = threadIdx.x; it < G * per; it += nthreads) {
    const int h = it / per, x = it - h * per;
    p.part_m[((hq0 + h) * p.Sm + chunk_lo) * recm + x] = (x % recm == 0) ? -INFINITY : 0.0f;
  }
}

// LDS of a workgroup of the one-launch form, after the exchange region of the middle-row phase:
// series coefficients [G][Mint + 32] | packed kept q [G][32] | constant-term coefficients | the
// middle-row record [G][recm] | the full-row record [G][recw] | C_v of the pair [M][Dvc] (1 KB aligned)
struct FusedLds {
  unsigned gs, qk, g0, recm, recw, cv, total;
};
__host__ __device__ __forceinline__ FusedLds fused_lds(unsigned lds_tab, int G, int Mint, int recm, int recw, int M,
                                                       int Dvc) {
  FusedLds L;
  L.gs = lds_tab;
  L.qk = L.gs + G * (Mint + 32) * 4;
  L.g0 = L.qk + G * 32 * 2;
  L.recm = L.g0 + 64;
  L.recw = L.recm + G * recm * 4;
  L.cv = (L.recw + G * recw * 4 + 1023u) & ~1023u;
  L.total = L.cv + ((static_cast<unsigned>(M) * Dvc * 4 + 1023u) & ~1023u);
  return L;
}

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

// rotation by N lanes within each row of 16 lanes (lane i receives lane (i + N) % 16 of its row)
template <int N>
__device__ __forceinline__ float row_ror(float v) {
  return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), 0x120 + N, 0xf, 0xf, false));
}
// sum / max over the lanes of a row whose indices differ by a multiple of `stride` (a power of two)
__device__ __forceinline__ float row_stride_sum(float v, int stride) {
  if (stride <= 8) v += row_ror<8>(v);
  if (stride <= 4) v += row_ror<4>(v);
  if (stride <= 2) v += row_ror<2>(v);
  if (stride <= 1) v += row_ror<1>(v);
  return v;
}
__device__ __forceinline__ float row_stride_max(float v, int stride) {
  if (stride <= 8) v = fmaxf(v, row_ror<8>(v));
  if (stride <= 4) v = fmaxf(v, row_ror<4>(v));
  if (stride <= 2) v = fmaxf(v, row_ror<2>(v));
  if (stride <= 1) v = fmaxf(v, row_ror<1>(v));
  return v;
}

// value of lane `src` (compile-time) broadcast to the wave
template <int SRC>
__device__ __forceinline__ float lane_value(float v) {
  return __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), SRC));
}
// wave-wide sum / max, result in every lane: rotations inside the rows, then the four row totals
__device__ __forceinline__ float wave_sum_fast(float v) {
  v = row_stride_sum(v, 1);
  return (lane_value<0>(v) + lane_value<16>(v)) + (lane_value<32>(v) + lane_value<48>(v));
}
__device__ __forceinline__ float wave_max_fast(float v) {
  v = row_stride_max(v, 1);
  return fmaxf(fmaxf(lane_value<0>(v), lane_value<16>(v)), fmaxf(lane_value<32>(v), lane_value<48>(v)));
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
// LDS of decode_prepare is sized by the launch (rows of C_k at a pitch of Dkc rounded up to 4, plus 4
// floats; then the group's queries at the compressed dims), so that many workgroups fit a unit
static inline int prep_pitch(int Dkc) { return ((Dkc + 3) & ~3) + 4; }
static inline unsigned prep_lds_bytes(int rows, int G, int Dkc) {
  return static_cast<unsigned>(rows * prep_pitch(Dkc) + ((G * Dkc + 3) & ~3)) * sizeof(float);
}

// kPrepRows: basis rows per workgroup (8 when the launch would otherwise not fill the chip, else 32)
template <typename T, int kPrepRows>
__global__ __launch_bounds__(kBlock) void decode_prepare(DecodeParams p) {
  extern __shared__ __attribute__((aligned(16))) unsigned char prep_smem[];
  const int kPrepLd = ((p.Dkc + 3) & ~3) + 4;                          // LDS pitch of a C_k row (floats)
  float* crow = reinterpret_cast<float*>(prep_smem);                   // [kPrepRows][kPrepLd]
  float* qc = crow + kPrepRows * kPrepLd;                              // [G][Dkc] query at the compressed dims

  const int tid = threadIdx.x, lane = tid & 63;
  const int bh = blockIdx.y, b = bh / p.Hkv, hkv = bh % p.Hkv;
  const int m0 = blockIdx.x * kPrepRows;
  const int Dkc = p.Dkc, D = p.D, G = p.G;

  // all global operands first (clamped, never predicated): C_k rows, the mask row, q of the group
  const float* ck = p.ck + static_cast<size_t>(bh) * p.M * Dkc;
  const bool vec4 = (Dkc & 3) == 0 && Dkc > 0;
  constexpr int kV4 = (kPrepRows * FA_MAX_HEAD_DIM / 4 + kBlock - 1) / kBlock;   // float4 per thread, worst case
  const int c4n = vec4 ? Dkc / 4 : 1;
  const int nv4 = vec4 ? kPrepRows * c4n : 0;
  f32x4 cv4[kV4];
  if (vec4) {
#pragma unroll
    for (int i = 0; i < kV4; ++i) {
      const int it = min(tid + i * kBlock, nv4 - 1);
      const int r = it / c4n, c4 = it - r * c4n;
      cv4[i] = *reinterpret_cast<const f32x4*>(ck + static_cast<size_t>(min(m0 + r, p.M - 1)) * Dkc + 4 * c4);
    }
  }
  uint64_t kbal[4];
  mask_ballots(p.kmask + static_cast<size_t>(bh) * D, D, lane, kbal);
  const size_t hq0 = static_cast<size_t>(b) * p.Hq + hkv * G;
  const T* q = static_cast<const T*>(p.q) + hq0 * D;
  constexpr int kQElems = kMaxG * FA_MAX_HEAD_DIM / kBlock;   // query elements per thread (worst case)
  const int nqe = G * D;
  T qe[kQElems];
#pragma unroll
  for (int i = 0; i < kQElems; ++i) qe[i] = q[min(tid + i * kBlock, nqe - 1)];

  if (vec4) {
#pragma unroll
    for (int i = 0; i < kV4; ++i) {
      const int it = tid + i * kBlock;
      if (it < nv4) {
        const int r = it / c4n, c4 = it - r * c4n;
        *reinterpret_cast<f32x4*>(crow + r * kPrepLd + 4 * c4) = cv4[i];
      }
    }
  } else {   // odd column counts: element by element
    for (int it = tid; it < kPrepRows * Dkc; it += kBlock) {
      const int r = it / Dkc, col = it - r * Dkc;
      crow[r * kPrepLd + col] = ck[static_cast<size_t>(min(m0 + r, p.M - 1)) * Dkc + col];
    }
  }
  // q splits into its compressed dims (fp32, for the products below) and its kept dims (packed and
  // zero padded for the K^mu products of decode_partial; written by the first workgroup of the row)
  const int kpitch = (p.Dku + 7) & ~7;
  const int Dkq = (kpitch + 31) / 32 * 32;
  T* qkeep = static_cast<T*>(p.qkeep) + hq0 * Dkq;
#pragma unroll
  for (int i = 0; i < kQElems; ++i) {
    const int it = tid + i * kBlock;
    if (it < nqe) {
      const int h = it / D, d = it % D;
      const int r = dim_rank(kbal, d);
      if (r < 0) qc[h * Dkc + (-r - 1)] = to_f32(qe[i]);
      else if (blockIdx.x == 0) qkeep[h * Dkq + r] = qe[i];
    }
  }
  if (blockIdx.x == 0) {
    const int npad = Dkq - p.Dku;
    for (int it = tid; it < G * npad; it += kBlock) qkeep[(it / npad) * Dkq + p.Dku + it % npad] = T{};
  }
  __syncthreads();

  // (row, head) dot products, nseg lanes each (a power of two that fills the workgroup)
  int nseg = 1;
  while (nseg < 64 && kPrepRows * G * nseg * 2 <= kBlock) nseg *= 2;
  for (int item0 = 0; item0 < kPrepRows * G; item0 += kBlock / nseg) {
    const int item = item0 + tid / nseg, seg = tid % nseg;
    const int r = item % kPrepRows, h = item / kPrepRows;
    float acc = 0.0f;
    if (h < G) {
      const float* cr = crow + r * kPrepLd;
      const float* qh = qc + h * Dkc;
      for (int i = seg; i < Dkc; i += nseg) acc += cr[i] * qh[i];
    }
    for (int o = nseg >> 1; o > 0; o >>= 1) acc += __shfl_xor(acc, o, kWave);
    const int m = m0 + r;
    if (seg == 0 && h < G && m <= p.Mint) {
      const float g = (m < p.M) ? acc * basis_weight((m + 1) / 2, p.T) : 0.0f;
      if (m == 0) p.g0[hq0 + h] = g;
      else p.gs[(hq0 + h) * p.Mint + (m - 1)] = g;
    }
  }
}

// ---------------------------------------------------------------------------
// 1b. g = diag(w) C_k q_c for compressed counts that are a multiple of 4: the streaming form
// ---------------------------------------------------------------------------
// TPR threads share a row of C_k and read it as interleaved 128-bit vectors, all requested
// before anything else happens (rows are independent of the mask); the group's queries at the
// compressed dims go through LDS once, each thread forms its share of the G dot products from
// registers, and the TPR shares meet by lane rotation.  256 / TPR rows per workgroup: 64 when
// the (sequence, head) pairs alone fill the chip, 16 when there are few of them.
template <typename T, int TPR>
__device__ __forceinline__ void prepare2_rows(const DecodeParams& p, const int bh, const int blk) {
  constexpr int kRows = kBlock / TPR;
  constexpr int kV4 = (FA_MAX_HEAD_DIM / 4 + TPR - 1) / TPR;
  __shared__ __attribute__((aligned(16))) float qc[kMaxG * FA_MAX_HEAD_DIM];   // [G][Dkc] query at the compressed dims

  const int tid = threadIdx.x, lane = tid & 63;
  const int b = bh / p.Hkv, hkv = bh % p.Hkv;
  const int Dkc = p.Dkc, D = p.D, G = p.G;
  const int row = tid / TPR, seg = tid % TPR;
  const int m = blk * kRows + row;            // basis function of this thread's row (0 .. Mint)
  const int c4n = Dkc / 4;

  // C_k row, the mask row and q of the group: all requested up front, clamped, never predicated
  const float* ck = p.ck + static_cast<size_t>(bh) * p.M * Dkc + static_cast<size_t>(min(m, p.M - 1)) * Dkc;
  f32x4 cv4[kV4];
#pragma unroll
  for (int i = 0; i < kV4; ++i)
    if (i * TPR < c4n) cv4[i] = *reinterpret_cast<const f32x4*>(ck + 4 * min(seg + i * TPR, c4n - 1));
  uint64_t kbal[4];
  mask_ballots(p.kmask + static_cast<size_t>(bh) * D, D, lane, kbal);
  const size_t hq0 = static_cast<size_t>(b) * p.Hq + hkv * G;
  const T* q = static_cast<const T*>(p.q) + hq0 * D;
  constexpr int kQElems = kMaxG * FA_MAX_HEAD_DIM / kBlock;
  const int nqe = G * D;
  T qe[kQElems];
#pragma unroll
  for (int i = 0; i < kQElems; ++i)
    if (i * kBlock < nqe) qe[i] = q[min(tid + i * kBlock, nqe - 1)];

  // q splits into its compressed dims (fp32, for the products below) and its kept dims (packed and
  // zero padded for the K^mu products of decode_partial; written by the first workgroup of the row)
  const int kpitch = (p.Dku + 7) & ~7;
  const int Dkq = (kpitch + 31) / 32 * 32;
  T* qkeep = static_cast<T*>(p.qkeep) + hq0 * Dkq;
#pragma unroll
  for (int i = 0; i < kQElems; ++i) {
    const int it = tid + i * kBlock;
    if (it < nqe) {
      const int h = it / D, d = it % D;
      const int r = dim_rank(kbal, d);
      if (r < 0) qc[h * Dkc + (-r - 1)] = to_f32(qe[i]);
      else if (blk == 0) qkeep[h * Dkq + r] = qe[i];
    }
  }
  if (blk == 0) {
    const int npad = Dkq - p.Dku;
    for (int it = tid; it < G * npad; it += kBlock) qkeep[(it / npad) * Dkq + p.Dku + it % npad] = T{};
  }
  __syncthreads();

  const float w = (m < p.M) ? basis_weight((m + 1) / 2, p.T) : 0.0f;
  for (int h = 0; h < G; ++h) {
    const float* qh = qc + h * Dkc;
    float acc = 0.0f;
#pragma unroll
    for (int i = 0; i < kV4; ++i) {
      if (i * TPR < c4n) {
        const int c4 = seg + i * TPR;
        const f32x4 qv = *reinterpret_cast<const f32x4*>(qh + 4 * min(c4, c4n - 1));
        const float d4 = (cv4[i][0] * qv[0] + cv4[i][1] * qv[1]) + (cv4[i][2] * qv[2] + cv4[i][3] * qv[3]);
        acc += (c4 < c4n) ? d4 : 0.0f;
      }
    }
    if constexpr (TPR == 16) {
      acc = row_stride_sum(acc, 1);
    } else {
      static_assert(TPR == 4, "threads per row");
      acc += __shfl_xor(acc, 1, kWave);
      acc += __shfl_xor(acc, 2, kWave);
    }
    if (seg == 0 && m <= p.Mint) {
      const float g = acc * w;
      if (m == 0) p.g0[hq0 + h] = g;
      else p.gs[(hq0 + h) * p.Mint + (m - 1)] = g;
    }
  }
}

template <typename T, int TPR>
__global__ __launch_bounds__(kBlock) void decode_prepare2(DecodeParams p) {
  prepare2_rows<T, TPR>(p, blockIdx.y, blockIdx.x);
}

// ---------------------------------------------------------------------------
// 2a. full-width sink/window rows: plain single-query attention partial
// ---------------------------------------------------------------------------
// A workgroup takes 256 rows, 64 per wave.  A wave multiplies its rows with q on the matrix
// cores (A = K rows, B = q, one column per head), normalises its 64 scores per head in registers
// and accumulates sum_j p_j V[j,:] on the vector unit, each lane owning 8 dims of every nrg-th
// row; the per-lane partial sums of all waves meet once in LDS.
constexpr int kWRows = 64;      // rows per wave
constexpr int kWBatch = 8;      // V rows a lane has in flight

template <typename T>
__device__ __forceinline__ void partial_full_rows(const DecodeParams& p, unsigned char* smem, int s) {
  const int bh = blockIdx.y, b = bh / p.Hkv, hkv = bh % p.Hkv;
  const int G = p.G, D = p.D;
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int q4 = lane >> 4, r16 = lane & 15;
  const size_t hq0 = static_cast<size_t>(b) * p.Hq + hkv * G;
  const int jw = s * kWChunk + wave * kWRows;          // first row of this wave
  const int Wb = seq_full_rows(p, b);
  const int nw = max(0, min(kWRows, Wb - jw));         // its valid rows (0: the wave only joins the barriers)
  const int jlast = max(Wb - 1, 0);
  const int jvis = Wb - p.Tq + r16 / p.Gq;             // last row the query token of column r16 may see

  // LDS carve-up: q [16][D] | p tiles [4][64][16] | partial sums [parts][4][D]
  T* qf = reinterpret_cast<T*>(smem);
  float* pw = reinterpret_cast<float*>(smem + 16 * FA_MAX_HEAD_DIM * sizeof(T)) + wave * kWRows * kMaxG;
  float* red = reinterpret_cast<float*>(smem + 16 * FA_MAX_HEAD_DIM * sizeof(T)) + kWaves * kWRows * kMaxG;
  __shared__ float wm[kWaves][kMaxG], wl[kWaves][kMaxG];

  // ---- global operands: q of the group, this wave's K rows (rows past the end re-read the last) --
  constexpr int kQLoads = kMaxG * FA_MAX_HEAD_DIM / 8 / kBlock;
  const T* q = static_cast<const T*>(p.q) + hq0 * D;
  const int nq8 = G * D / 8;
  Frag<T> qv[kQLoads];
#pragma unroll
  for (int i = 0; i < kQLoads; ++i) qv[i].load(q + 8 * min(tid + i * kBlock, nq8 - 1));
  const int kcn = (D + 31) / 32;                        // 32-dim steps (the last may be partial)
  const T* kbase = static_cast<const T*>(p.k_full) + bh * p.full_stride;
  const T* vbase = static_cast<const T*>(p.v_full) + bh * p.full_stride;
  const T* krow[kRB];
#pragma unroll
  for (int rb = 0; rb < kRB; ++rb) krow[rb] = kbase + static_cast<int64_t>(min(jw + 16 * rb + r16, jlast)) * D;
  Frag<T> ka[4][kRB];                                   // dims [0, 128)
#pragma unroll
  for (int cc = 0; cc < 4; ++cc)
#pragma unroll
    for (int rb = 0; rb < kRB; ++rb) ka[cc][rb].load(krow[rb] + min(cc * 32 + 8 * q4, D - 8));

  // ---- q into LDS (rows >= G zero) ---------------------------------------------------
  {
    const int nz = (16 - G) * D * static_cast<int>(sizeof(T)) / 16;
    for (int it = tid; it < nz; it += kBlock) reinterpret_cast<u32x4*>(qf + G * D)[it] = u32x4{0u, 0u, 0u, 0u};
  }
#pragma unroll
  for (int i = 0; i < kQLoads; ++i) {
    const int v8 = tid + i * kBlock;
    if (v8 < nq8) *reinterpret_cast<Frag<T>*>(qf + 8 * v8) = qv[i];
  }
  __syncthreads();

  // ---- scores of the wave's 64 rows: lane (head r16, q4) gets rows 16 rb + 4 q4 + v ----------------
  f32x4 sacc[kRB];
#pragma unroll
  for (int rb = 0; rb < kRB; ++rb) sacc[rb] = f32x4{0.f, 0.f, 0.f, 0.f};
  auto score_steps = [&](int c0) {   // four 32-dim steps from step c0 on, operands in ka
#pragma unroll
    for (int cc = 0; cc < 4; ++cc) {
      const int dd = (c0 + cc) * 32 + 8 * q4;
      Frag<T> bq;
      bq.load(qf + r16 * D + min(dd, D - 8));
      if (dd >= D) bq.zero();            // a step past the head dim multiplies re-read dims by zero
#pragma unroll
      for (int rb = 0; rb < kRB; ++rb) mma_k32(sacc[rb], ka[cc][rb], bq);
    }
  };
  score_steps(0);
  if (kcn > 4) {                         // head dims 136 .. 256
#pragma unroll
    for (int cc = 0; cc < 4; ++cc)
#pragma unroll
      for (int rb = 0; rb < kRB; ++rb) ka[cc][rb].load(krow[rb] + min((4 + cc) * 32 + 8 * q4, D - 8));
    score_steps(4);
  }
  // V rows of this lane: 8 dims (dc) of rows rg, rg + nrg, ...; the first batch travels during the softmax
  const int nch = D / 8, nrg = max(64 / nch, 1);
  const bool lane_on = lane < nch * nrg;
  const int dc = lane % nch, rg = min(lane / nch, nrg - 1);
  const int vrows = (kWRows + nrg - 1) / nrg;
  const T* vlane = vbase + dc * 8;
  Frag<T> vf0[kWBatch];
#pragma unroll
  for (int i = 0; i < kWBatch; ++i) vf0[i].load(vlane + static_cast<int64_t>(min(jw + rg + i * nrg, jlast)) * D);

  // ---- softmax over the wave's rows, per head -----------------------------------------------------
  float m_w = -INFINITY;
#pragma unroll
  for (int rb = 0; rb < kRB; ++rb)
#pragma unroll
    for (int v = 0; v < 4; ++v) {
      const int r = 16 * rb + 4 * q4 + v;
      const float sv = (r < nw && r16 < G && jw + r <= jvis) ? sacc[rb][v] * p.scale : -INFINITY;
      sacc[rb][v] = sv;
      m_w = fmaxf(m_w, sv);
    }
  m_w = fmaxf(m_w, __shfl_xor(m_w, 16, kWave));
  m_w = fmaxf(m_w, __shfl_xor(m_w, 32, kWave));
  const float m_ref = (m_w == -INFINITY) ? 0.0f : m_w;
  float l_w = 0.0f;
#pragma unroll
  for (int rb = 0; rb < kRB; ++rb)
#pragma unroll
    for (int v = 0; v < 4; ++v) {
      const float e = __expf(sacc[rb][v] - m_ref);   // masked rows hold -inf -> 0
      l_w += e;
      pw[(16 * rb + 4 * q4 + v) * kMaxG + r16] = e;
    }
  l_w += __shfl_xor(l_w, 16, kWave);
  l_w += __shfl_xor(l_w, 32, kWave);
  if (q4 == 0) {
    wm[wave][r16] = m_w;
    wl[wave][r16] = l_w;
  }
  __syncthreads();   // statistics of all waves (and this wave's p tile) are visible

  // record of head h: [max, sum, -, -, acc[D]]
  float* part = p.part_w + (hq0 * p.Sw + s) * p.recw;
  const size_t part_h = static_cast<size_t>(p.Sw) * p.recw;
  for (int hg = 0; hg < G; hg += 4) {
    float acc[4][8];
#pragma unroll
    for (int hh = 0; hh < 4; ++hh)
#pragma unroll
      for (int e = 0; e < 8; ++e) acc[hh][e] = 0.0f;
    // factors that bring every wave to the workgroup's maximum
    float fw[4];
#pragma unroll
    for (int hh = 0; hh < 4; ++hh) {
      const int h = min(hg + hh, kMaxG - 1);
      float ms = wm[0][h];
#pragma unroll
      for (int w = 1; w < kWaves; ++w) ms = fmaxf(ms, wm[w][h]);
      const float mine = wm[wave][h];
      fw[hh] = (mine == -INFINITY) ? 0.0f : __expf(mine - ms);
      if (tid == hh && hg + hh < G) {
        float l = 0.0f;
#pragma unroll
        for (int w = 0; w < kWaves; ++w) l += (wm[w][h] == -INFINITY) ? 0.0f : wl[w][h] * __expf(wm[w][h] - ms);
        part[(hg + hh) * part_h + 0] = ms;
        part[(hg + hh) * part_h + 1] = l;
      }
    }
    // sum_j p_j V[j,:] over this lane's rows
    auto accumulate = [&](const Frag<T> (&vf)[kWBatch], int i0) {
#pragma unroll
      for (int i = 0; i < kWBatch; ++i) {
        const int r = rg + (i0 + i) * nrg;
        if (i0 + i < vrows && r < nw && lane_on) {
          const f32x4 p4 = *reinterpret_cast<const f32x4*>(pw + r * kMaxG + hg);
          float x[8];
          unpack8(vf[i], x);
#pragma unroll
          for (int hh = 0; hh < 4; ++hh)
#pragma unroll
            for (int e = 0; e < 8; ++e) acc[hh][e] += p4[hh] * x[e];
        }
        if ((i & 3) == 3) __builtin_amdgcn_sched_barrier(0);   // keep the p reads next to their rows
      }
    };
    if (hg == 0) {
      accumulate(vf0, 0);
    } else {
      Frag<T> vf[kWBatch];
#pragma unroll
      for (int i = 0; i < kWBatch; ++i) vf[i].load(vlane + static_cast<int64_t>(min(jw + rg + i * nrg, jlast)) * D);
      accumulate(vf, 0);
    }
    for (int i0 = kWBatch; i0 < vrows; i0 += kWBatch) {   // head dims above 128 only
      Frag<T> vf[kWBatch];
#pragma unroll
      for (int i = 0; i < kWBatch; ++i) vf[i].load(vlane + static_cast<int64_t>(min(jw + rg + (i0 + i) * nrg, jlast)) * D);
      accumulate(vf, i0);
    }
    // park the scaled partial sums: red[wave * nrg + rg][hh][D]
    if (hg > 0) __syncthreads();   // the previous head group's sums have been read
    if (lane_on) {
      float* dst = red + ((wave * nrg + rg) * 4) * D + dc * 8;
#pragma unroll
      for (int hh = 0; hh < 4; ++hh) {
        *reinterpret_cast<f32x4*>(dst + hh * D) = f32x4{fw[hh] * acc[hh][0], fw[hh] * acc[hh][1], fw[hh] * acc[hh][2], fw[hh] * acc[hh][3]};
        *reinterpret_cast<f32x4*>(dst + hh * D + 4) = f32x4{fw[hh] * acc[hh][4], fw[hh] * acc[hh][5], fw[hh] * acc[hh][6], fw[hh] * acc[hh][7]};
      }
    }
    __syncthreads();
    const int nparts = kWaves * nrg;
    for (int it = tid; it < D; it += kBlock) {   // 4 heads x D dims, four floats per item
      const int hh = (4 * it) / D, d = (4 * it) % D;
      if (hg + hh < G) {
        f32x4 v = {0.f, 0.f, 0.f, 0.f};
        for (int k = 0; k < nparts; ++k) v += *reinterpret_cast<const f32x4*>(red + (k * 4 + hh) * D + d);
        *reinterpret_cast<f32x4*>(part + (hg + hh) * part_h + 4 + d) = v;
      }
    }
  }
}

// ---------------------------------------------------------------------------
// 2b. middle rows: kept dims streamed, compressed dims through the series
// ---------------------------------------------------------------------------
// The four waves of a workgroup walk the same steps (KT tiles of 64 rows x the
// query heads of the group) and divide the work of every step:
//   * the series by harmonics: wave w owns orders 16 CW w + 1 .. 16 CW (w + 1)
//     on both sides; its slices of the E table (K side: A operands, V side: B
//     operands) are built once and stay in registers;
//   * the kept dims by rows: wave w multiplies a quarter of the step's K^mu row
//     blocks and a quarter of its V^mu token blocks.
// The partial scores meet in LDS; wave w then sums and exponentiates the four
// columns 4 w .. 4 w + 3 (one token tile when the group has four heads), keeps
// their running maximum and sum, and hands the probabilities back through LDS
// as ready-made MFMA operands: two barriers per step, no work done twice.
constexpr int kVU = 2;                                        // V^mu token blocks per wave and step
constexpr unsigned kXchgBytes = 32 * 1024;   // score exchange, probability tiles, statistics; E transpose tiles

// cos / sin of 2 pi n u / T for a table entry (n u < 2^24): exact integer phase
template <typename T>
__device__ __forceinline__ void table_cs(int n, int u, int period, float inv_period, float* c, float* s) {
  const int prod = n * u;
  int ph = prod - static_cast<int>(static_cast<float>(prod) * inv_period) * period;   // quotient exact to +-1
  if (ph < 0) ph += period;
  if (ph >= period) ph -= period;
  if constexpr (sizeof(T) == 4) {
    sincospif(2.0f * (static_cast<float>(ph) / static_cast<float>(period)), s, c);
  } else {
    const float x = static_cast<float>(ph) * inv_period;
    *s = __builtin_amdgcn_sinf(x);
    *c = __builtin_amdgcn_cosf(x);
  }
}

// KC1: the kept K dims fit one 32-dim MFMA step (the usual case), so that all K^mu operands of
// a step are requested ahead and none on demand.
template <typename T, int CW, int DVTM, bool KC1>
__device__ __forceinline__ void partial_middle_rows(const DecodeParams& p, unsigned char* smem) {
  using ES = typename SeriesType<T>::type;
  constexpr int Mint = kWaves * CW * 32;
  constexpr int kQLoads = kMaxG * FA_MAX_HEAD_DIM / 8 / kBlock;
  // V^mu operands are requested a step ahead when they fit in registers
  constexpr bool kPrefetchV = DVTM <= 2;
  constexpr int kVR = kPrefetchV ? DVTM : 1;

  const int sm_idx = blockIdx.x, bh = blockIdx.y, b = bh / p.Hkv, hkv = bh % p.Hkv;
  const int G = p.G, Gp = p.Gp, KT = p.KT;
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);   // uniform: keeps unit ids scalar
  const int q4 = lane >> 4, r16 = lane & 15;
  const size_t hq0 = static_cast<size_t>(b) * p.Hq + hkv * G;
  const int Nb = seq_middle_rows(p, b);
  const int c0 = sm_idx * p.chunk_m, c1 = min(Nb, c0 + p.chunk_m);    // chunk of middle rows
  if (c0 >= Nb) {   // (only with per-sequence counts) nothing of this chunk belongs to the sequence
    write_empty_middle(p, hq0, sm_idx, sm_idx + 1, kBlock);
    return;
  }
  const int step = KT * kTJ;                                           // rows per step
  const int col_k = r16 / Gp, col_h = r16 % Gp;                        // S column = (tile, head)
  const bool col_live = col_k < KT && col_h < G;
  const int hsafe = min(col_h, G - 1);
  const int DVT = (p.Dvu + 15) / 16;
  const int kpitch = (p.Dku + 7) & ~7;               // K^mu rows are padded to 8 columns
  const int kchunks = (kpitch + 31) / 32;
  const int Dkq = kchunks * 32;                      // pitch of the packed query rows (zero padded)
  const bool vragged = (p.Dvu & 15) != 0;
  const T* kk = static_cast<const T*>(p.k_keep) + bh * p.kk_stride;
  const T* vk = static_cast<const T*>(p.v_keep) + bh * p.vk_stride;
  const int Nm1 = Nb - 1;
  const int NV = KT >= 2 ? KT / 2 : 1;               // V^mu token blocks of this wave per step

  // ---- LDS carve-up -------------------------------------------------------
  f32x4* xs = reinterpret_cast<f32x4*>(smem);                   // [kWaves][kRB][64] partial scores
  constexpr unsigned kXsBytes = kWaves * kRB * 64 * 16;
  ES* pse = reinterpret_cast<ES*>(smem + kXsBytes);             // [kXN][16][4][8] probabilities, series type
  T* pte = reinterpret_cast<T*>(smem + kXsBytes + kXN * 16 * 4 * 8 * sizeof(ES));   // same, element type
  // what the element-type rounding of the probabilities dropped (16-bit element types only): the kept-V
  // product takes both tiles, so a diffuse softmax does not see 2^-9 rounding noise in its output
  T* ptl = reinterpret_cast<T*>(smem + kXsBytes + kXN * 16 * 4 * 8 * (sizeof(ES) + sizeof(T)));
  float* alpha_s = reinterpret_cast<float*>(smem + kXsBytes + kXN * 16 * 4 * 8 * (sizeof(ES) + 2 * sizeof(T)));   // [16]
  float* st_m = alpha_s + 16;                                   // [16] column maxima (after the loop)
  float* st_l = st_m + 16;                                      // [16] column sums
  float* red_r = reinterpret_cast<float*>(smem);                // after the loop: [16][Mint + 4]
  const int pr = Mint + 4, po = 16 * DVT + 4;
  float* red_o = red_r + 16 * pr;                               // [kWaves][16][16 DVT + 4]
  constexpr int kPitchG = Mint + 32;                            // floats per row of gs_s
  float* gs_s = reinterpret_cast<float*>(smem + p.lds_tab);     // [G][kPitchG] series coefficients
  T* qk_s = reinterpret_cast<T*>(gs_s + G * kPitchG);           // [G][Dkq]

  // K^mu row block uid of the step at `base` (tile uid / 4, row block uid % 4), dims
  // [32 cc, 32 cc + 32).  Rows are clamped into the slab (rows past the chunk are
  // masked at the softmax); columns past the row pitch re-read the row's last 8
  // columns, where the packed query is zero.
  auto k_ptr = [&](int base, int uid, int cc) -> const T* {
    const int k = uid >> 2, rb = uid & 3;
    const int u = 32 * (rb >> 1) + 8 * (r16 >> 2) + 4 * (rb & 1) + (r16 & 3);
    const int j = min(base + k * kTJ + u, Nm1);
    const int dcl = min(cc * 32 + 8 * q4, kpitch - 8);
    return kk + (static_cast<uint32_t>(j) * static_cast<uint32_t>(kpitch) + static_cast<uint32_t>(dcl));
  };
  // V^mu token block vid (tile vid / 2, half vid % 2), dim tile dt: 8 consecutive rows of one dim
  auto v_ptr = [&](int base, int vid, int dt) -> const T* {
    const int tok0 = base + (vid >> 1) * kTJ + 32 * (vid & 1) + 8 * q4;   // multiple of 8
    const int dim = min(16 * dt + r16, p.Dvu - 1);
    const uint32_t g8 = static_cast<uint32_t>(min(tok0, Nm1)) >> 3;
    return vk + (g8 * static_cast<uint32_t>(p.Dvu) + static_cast<uint32_t>(dim)) * 8u;
  };
  // applied when the operand is consumed, so that the loads stay asynchronous: rows past
  // the chunk and dims past Dvu are zeroed (their weight is 0, but 0 * garbage must stay 0)
  auto fix_v = [&](Frag<T>& bv, int base, int vid, int dt) {
    const int tok0 = base + (vid >> 1) * kTJ + 32 * (vid & 1) + 8 * q4;
    if (16 * dt + r16 >= p.Dvu) bv.zero();
    if (tok0 + 8 > c1) mask_tail(bv, c1 - tok0);
  };
  auto load_step = [&](Frag<T> (&kf)[kMaxKT], Frag<T> (&vf)[kVU][kVR], int base) {
    if (kchunks > 0) {
#pragma unroll
      for (int i = 0; i < kMaxKT; ++i)
        if (i < KT) kf[i].load(k_ptr(base, wave * KT + i, 0));
    }
    if constexpr (kPrefetchV) {
      if (DVT > 0) {
#pragma unroll
        for (int i = 0; i < kVU; ++i) {
          const int vid = wave * NV + i;
          if (i < NV && vid < 2 * KT) {
#pragma unroll
            for (int dt = 0; dt < DVTM; ++dt)
              if (dt < DVT) vf[i][dt].load(v_ptr(base, vid, dt));
          }
        }
      }
    }
  };

  // ---- (0) everything that comes from global memory is requested first ------------
  // series coefficients of the group: G * Mint contiguous floats
  constexpr int kGLoads = kMaxG * Mint / 4 / kBlock;
  const int ng4 = G * Mint / 4;
  f32x4 gv[kGLoads];
#pragma unroll
  for (int i = 0; i < kGLoads; ++i)
    gv[i] = *reinterpret_cast<const f32x4*>(p.gs + hq0 * Mint + 4 * min(tid + i * kBlock, ng4 - 1));
  // this lane's share of the softmax: column ocol, rows 16 orb + 4 oq4 + v of the tile
  const int ocol = 4 * wave + (lane & 3), orb = lane >> 4, oq4 = (lane >> 2) & 3;
  const int ocol_k = ocol / Gp, ocol_h = ocol % Gp;
  const bool olive = ocol_k < KT && ocol_h < G;
  const float g0 = p.g0[hq0 + min(ocol_h, G - 1)];
  const int nq8 = G * Dkq / 8;
  Frag<T> qv[kQLoads];
  if (nq8 > 0) {
    const T* qsrc = static_cast<const T*>(p.qkeep) + hq0 * Dkq;
#pragma unroll
    for (int i = 0; i < kQLoads; ++i) qv[i].load(qsrc + 8 * min(tid + i * kBlock, nq8 - 1));
  }
  Frag<T> kfA[kMaxKT], kfB[kMaxKT];
  Frag<T> vfA[kVU][kVR], vfB[kVU][kVR];
  load_step(kfA, vfA, c0);

  // ---- this wave's slices of the E table ------------------------------------------------------
  // K side, A operand of (own chunk i, row block rb): row u(rb, r16), slots 8 q4 .. 8 q4 + 7 of the
  // chunk = (cos, sin) of 4 consecutive orders.  V side, B operand of (own chunk i, cos | sin,
  // half x): order 16 c + r16 + 1 at the 8 consecutive rows 32 x + 8 q4 ...
  Frag<ES> eA[CW][kRB], eB[CW][2][kXN];
  {
    const int n_max = p.M / 2;
    const float invT = 1.0f / static_cast<float>(p.T);
    if constexpr (sizeof(ES) == 4) {
      // fp32 tables: every entry evaluated on its own
#pragma unroll
      for (int i = 0; i < CW; ++i) {
        const int c = wave * CW + i;
#pragma unroll
        for (int rb = 0; rb < kRB; ++rb) {
          const int u = 32 * (rb >> 1) + 8 * (r16 >> 2) + 4 * (rb & 1) + (r16 & 3);
          float vals[8];
#pragma unroll
          for (int hp = 0; hp < 4; ++hp) {
            const int n = 16 * c + 4 * q4 + hp + 1;
            vals[2 * hp] = vals[2 * hp + 1] = 0.0f;
            if (n <= n_max) table_cs<T>(n, u, p.T, invT, &vals[2 * hp], &vals[2 * hp + 1]);
          }
          pack8(eA[i][rb], vals);
        }
        const int n = 16 * c + r16 + 1;
#pragma unroll
        for (int x = 0; x < kXN; ++x) {
          float cs[8], sn[8];
#pragma unroll
          for (int e = 0; e < 8; ++e) {
            cs[e] = sn[e] = 0.0f;
            if (n <= n_max) table_cs<T>(n, 32 * x + 8 * q4 + e, p.T, invT, &cs[e], &sn[e]);
          }
          pack8(eB[i][0][x], cs);
          pack8(eB[i][1][x], sn);
        }
      }
    } else {
      // 16-bit tables.  K side: the first of a lane's 4 consecutive orders is evaluated, the others
      // follow by the angle-addition step of its row.  V side: the same entries, transposed through a
      // wave-private LDS tile [slot][row] one chunk at a time.
      constexpr int kPitchT = 2 * kTJ + 16;   // bytes per slot row of the transpose tile
      unsigned char* et = smem + wave * (32 * kPitchT);
      int urow[kRB];
      float cd[kRB], sd[kRB];
#pragma unroll
      for (int rb = 0; rb < kRB; ++rb) {
        urow[rb] = 32 * (rb >> 1) + 8 * (r16 >> 2) + 4 * (rb & 1) + (r16 & 3);
        table_cs<T>(1, urow[rb], p.T, invT, &cd[rb], &sd[rb]);
      }
#pragma unroll
      for (int i = 0; i < CW; ++i) {
        const int n0 = 16 * (wave * CW + i) + 4 * q4 + 1;
#pragma unroll
        for (int rb = 0; rb < kRB; ++rb) {
          float vals[8];
          table_cs<T>(n0, urow[rb], p.T, invT, &vals[0], &vals[1]);
#pragma unroll
          for (int hp = 1; hp < 4; ++hp) {
            vals[2 * hp] = vals[2 * hp - 2] * cd[rb] - vals[2 * hp - 1] * sd[rb];
            vals[2 * hp + 1] = vals[2 * hp - 1] * cd[rb] + vals[2 * hp - 2] * sd[rb];
          }
#pragma unroll
          for (int hp = 0; hp < 4; ++hp)
            if (n0 + hp > n_max) vals[2 * hp] = vals[2 * hp + 1] = 0.0f;
          pack8(eA[i][rb], vals);
#pragma unroll
          for (int e = 0; e < 8; ++e)
            *reinterpret_cast<uint16_t*>(et + (8 * q4 + e) * kPitchT + 2 * urow[rb]) =
                static_cast<uint16_t>(eA[i][rb].v[e >> 1] >> (16 * (e & 1)));
        }
        __syncthreads();
#pragma unroll
        for (int cs = 0; cs < 2; ++cs)
#pragma unroll
          for (int x = 0; x < kXN; ++x)
            eB[i][cs][x].load(reinterpret_cast<const ES*>(et + (2 * r16 + cs) * kPitchT) + 32 * x + 8 * q4);
        if (i + 1 < CW) __syncthreads();
      }
    }
  }
  // the accumulators of the V side live in a frame that moves with the steps: per step
  // every (cos, sin) pair turns by -omega_n * step, a fixed twiddle per order
  float tc[CW], ts[CW];
  {
    const uint32_t ph_step = phase_of(step, p.ph_scale);
#pragma unroll
    for (int i = 0; i < CW; ++i)
      phase_cs<T>(static_cast<uint32_t>(16 * (wave * CW + i) + r16 + 1) * ph_step, &tc[i], &ts[i]);
  }

  // ---- series coefficients and packed query into LDS ---------------------------------------------
#pragma unroll
  for (int i = 0; i < kGLoads; ++i) {
    const int v4 = tid + i * kBlock;
    if (v4 < ng4) *reinterpret_cast<f32x4*>(gs_s + (4 * v4 / Mint) * kPitchG + (4 * v4) % Mint) = gv[i];
  }
#pragma unroll
  for (int i = 0; i < kQLoads; ++i) {
    const int v8 = tid + i * kBlock;
    if (v8 < nq8) *reinterpret_cast<Frag<T>*>(qk_s + 8 * v8) = qv[i];
  }
  __syncthreads();
  // the second step's operands are requested only now: a wave that asks for more than the memory
  // pipeline holds stalls at the request, and the table above is better built before that
  if (c0 + step < c1) load_step(kfB, vfB, c0 + step);

  f32x4 racc[2 * CW];           // r' = P^T E (own orders), frame of the current step
  f32x4 oacc[DVTM];             // sum_j p_j V^mu[j,:] over this wave's token blocks
#pragma unroll
  for (int t = 0; t < 2 * CW; ++t) racc[t] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
  for (int t = 0; t < DVTM; ++t) oacc[t] = f32x4{0.f, 0.f, 0.f, 0.f};
  float m_run = -INFINITY, l_run = 0.0f;   // per S column (replicated over q4 and waves); l is a per-lane partial
  int last_base = c0;                       // origin of the latest step
  const bool quad_share = Gp >= 4;          // the 4 lanes of a quad then share (tile, q4)
  bool first = true;

  auto do_step = [&](Frag<T> (&kf)[kMaxKT], Frag<T> (&vf)[kVU][kVR], int base) {
    const bool tail = base + step > c1;
    f32x4 sacc[kRB];
#pragma unroll
    for (int rb = 0; rb < kRB; ++rb) sacc[rb] = f32x4{0.f, 0.f, 0.f, 0.f};

    // -- (a) series on the K side, own orders: S += E g'(tile origin) -----------------
    const uint32_t ph_k = phase_of(p.t0 + base + col_k * kTJ, p.ph_scale);
#pragma unroll
    for (int i = 0; i < CW; ++i) {
      const uint32_t n0 = 16 * (wave * CW + i) + 4 * q4 + 1;
      float csv[4], snv[4];
      if (quad_share) {
        float cs, sn;
        phase_cs<T>((n0 + (lane & 3)) * ph_k, &cs, &sn);
#pragma unroll
        for (int j = 0; j < 4; ++j) {
          csv[j] = quad_bcast(cs, j);
          snv[j] = quad_bcast(sn, j);
        }
      } else {
#pragma unroll
        for (int j = 0; j < 4; ++j) phase_cs<T>((n0 + j) * ph_k, &csv[j], &snv[j]);
      }
      const float* gl = gs_s + hsafe * kPitchG + 32 * (wave * CW + i) + 8 * q4;
      const f32x4 ga = *reinterpret_cast<const f32x4*>(gl), gb = *reinterpret_cast<const f32x4*>(gl + 4);
      float gp[8];
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        const float gc = (j < 2) ? ga[2 * (j & 1)] : gb[2 * (j & 1)];
        const float gsn = (j < 2) ? ga[2 * (j & 1) + 1] : gb[2 * (j & 1) + 1];
        gp[2 * j] = gc * csv[j] + gsn * snv[j];
        gp[2 * j + 1] = gsn * csv[j] - gc * snv[j];
      }
      Frag<ES> bg;
      pack8(bg, gp);
      if (!col_live) bg.zero();
#pragma unroll
      for (int rb = 0; rb < kRB; ++rb) mma_k32(sacc[rb], eA[i][rb], bg);
    }

    // -- (b) kept K dims, own row blocks: A = K^mu rows, B = q masked to the tile's columns --
    if (kchunks > 0) {
#pragma unroll
      for (int i = 0; i < kMaxKT; ++i) {
        if (i < KT) {
          const int uid = wave * KT + i, k = uid >> 2, rbd = uid & 3;
          f32x4 ka = {0.f, 0.f, 0.f, 0.f};
          {
            Frag<T> bq;
            bq.load(qk_s + hsafe * Dkq + 8 * q4);
            if (col_k != k || !col_live) bq.zero();
            mma_k32(ka, kf[i], bq);
          }
          if constexpr (!KC1) {
            for (int cc = 1; cc < kchunks; ++cc) {
              Frag<T> a, bq;
              a.load(k_ptr(base, uid, cc));
              bq.load(qk_s + hsafe * Dkq + cc * 32 + 8 * q4);
              if (col_k != k || !col_live) bq.zero();
              mma_k32(ka, a, bq);
            }
          }
          if (rbd == 0) sacc[0] += ka;
          else if (rbd == 1) sacc[1] += ka;
          else if (rbd == 2) sacc[2] += ka;
          else sacc[3] += ka;
        }
      }
    }

    // -- (c) the partial scores of the four waves meet; this wave sums its four columns --------
    {
      f32x4* xw = xs + (wave * kRB) * 64 + lane;
#pragma unroll
      for (int rb = 0; rb < kRB; ++rb) xw[rb * 64] = sacc[rb];
    }
    __syncthreads();
    f32x4 sv;
    {
      const f32x4* xr = xs + orb * 64 + oq4 * 16 + ocol;
      sv = ((xr[0 * kRB * 64] + xr[1 * kRB * 64]) + xr[2 * kRB * 64]) + xr[3 * kRB * 64];
    }
    // -- (d) online softmax of the own columns: lane holds rows u = 32x + 8 oq4 + 4y + v (orb = 2x + y)
    float pv[4];
    float m_tile = -INFINITY;
#pragma unroll
    for (int v = 0; v < 4; ++v) {
      const int u = 32 * (orb >> 1) + 8 * oq4 + 4 * (orb & 1) + v;
      const int j = base + ocol_k * kTJ + u;
      const float sc = (olive && j < c1) ? (sv[v] + g0) * p.scale : -INFINITY;
      pv[v] = sc;
      m_tile = fmaxf(m_tile, sc);
    }
    m_tile = row_stride_max(m_tile, 4);                      // the 16 lanes of a column are 4 apart
    m_tile = fmaxf(m_tile, __shfl_xor(m_tile, 16, kWave));
    m_tile = fmaxf(m_tile, __shfl_xor(m_tile, 32, kWave));
    const float m_new = fmaxf(m_run, m_tile);
    const float m_ref = (m_new == -INFINITY) ? 0.0f : m_new;
    const float alpha = __expf(m_run - m_ref);   // m_run = -inf -> 0
    float l_add = 0.0f;
#pragma unroll
    for (int v = 0; v < 4; ++v) {
      pv[v] = __expf(pv[v] - m_ref);
      l_add += pv[v];
    }
    l_run = l_run * alpha + l_add;
    m_run = m_new;
    // probabilities back as A operands: reader lane (column c, q4) takes rows 32x + 8 q4 + e, e < 8
    {
      const int slot = (((orb >> 1) * 16 + ocol) * 4 + oq4) * 8 + 4 * (orb & 1);
      if constexpr (sizeof(ES) == 4) {
        *reinterpret_cast<f32x4*>(reinterpret_cast<float*>(pse) + slot) = f32x4{pv[0], pv[1], pv[2], pv[3]};
      } else {
        u32x2d w;
        w[0] = __builtin_bit_cast(uint32_t, __builtin_convertvector(f32x2{pv[0], pv[1]}, f16x2));
        w[1] = __builtin_bit_cast(uint32_t, __builtin_convertvector(f32x2{pv[2], pv[3]}, f16x2));
        *reinterpret_cast<u32x2d*>(reinterpret_cast<uint16_t*>(pse) + slot) = w;
        w[0] = __builtin_bit_cast(uint32_t, __builtin_convertvector(f32x2{pv[0], pv[1]}, bf16x2));
        w[1] = __builtin_bit_cast(uint32_t, __builtin_convertvector(f32x2{pv[2], pv[3]}, bf16x2));
        *reinterpret_cast<u32x2d*>(reinterpret_cast<uint16_t*>(pte) + slot) = w;
        float lo[4];
#pragma unroll
        for (int v = 0; v < 4; ++v)
          lo[v] = pv[v] - __builtin_bit_cast(float, ((w[v >> 1] >> (16 * (v & 1))) & 0xffffu) << 16);
        w[0] = __builtin_bit_cast(uint32_t, __builtin_convertvector(f32x2{lo[0], lo[1]}, bf16x2));
        w[1] = __builtin_bit_cast(uint32_t, __builtin_convertvector(f32x2{lo[2], lo[3]}, bf16x2));
        *reinterpret_cast<u32x2d*>(reinterpret_cast<uint16_t*>(ptl) + slot) = w;
      }
      if (lane < 4) alpha_s[ocol] = alpha;
    }
    __syncthreads();
    // -- (e) bring the accumulators into this step's frame --------------------------------
    if (!first) {
      // accumulator rows are S columns 4*q4 + v
      const f32x4 al = *reinterpret_cast<const f32x4*>(alpha_s + 4 * q4);
#pragma unroll
      for (int t = 0; t < DVTM; ++t)
#pragma unroll
        for (int v = 0; v < 4; ++v) oacc[t][v] *= al[v];
#pragma unroll
      for (int i = 0; i < CW; ++i)
#pragma unroll
        for (int v = 0; v < 4; ++v) {
          const float rc = racc[2 * i][v], rs = racc[2 * i + 1][v];
          racc[2 * i][v] = al[v] * (tc[i] * rc + ts[i] * rs);
          racc[2 * i + 1][v] = al[v] * (tc[i] * rs - ts[i] * rc);
        }
    }
    first = false;
    last_base = base;

    // -- (f) V side, own orders: r' += P^T E ------------------------------------------------------
    Frag<T> pt[kXN], pl[kXN];
#pragma unroll
    for (int x = 0; x < kXN; ++x) {
      Frag<ES> ps;
      ps.load(pse + ((x * 16 + r16) * 4 + q4) * 8);
      if constexpr (sizeof(ES) == 4) pt[x].load(reinterpret_cast<const T*>(pse) + ((x * 16 + r16) * 4 + q4) * 8);
      else {
        pt[x].load(pte + ((x * 16 + r16) * 4 + q4) * 8);
        if (DVT > 0) pl[x].load(ptl + ((x * 16 + r16) * 4 + q4) * 8);
      }
#pragma unroll
      for (int i = 0; i < CW; ++i) {
        mma_k32(racc[2 * i], ps, eB[i][0][x]);
        mma_k32(racc[2 * i + 1], ps, eB[i][1][x]);
      }
    }
    // -- (g) kept V dims, own token blocks: O += P^T V^mu -----------------------------------------
    if (DVT > 0) {
#pragma unroll
      for (int i = 0; i < kVU; ++i) {
        const int vid = wave * NV + i;
        if (i < NV && vid < 2 * KT) {
          Frag<T> ak = pt[0];   // select by value: an lvalue choice would put both fragments in memory
          const Frag<T> p1 = pt[1];
          if (vid & 1) ak = p1;
          if (col_k != (vid >> 1)) ak.zero();
          Frag<T> al;
          if constexpr (sizeof(ES) != 4) {
            al = pl[0];
            const Frag<T> l1 = pl[1];
            if (vid & 1) al = l1;
            if (col_k != (vid >> 1)) al.zero();
          }
#pragma unroll
          for (int dt = 0; dt < DVTM; ++dt) {
            if (dt < DVT) {
              Frag<T> bv;
              if constexpr (kPrefetchV) bv = vf[i][dt];
              else bv.load(v_ptr(base, vid, dt));
              if (tail || vragged) fix_v(bv, base, vid, dt);
              mma_k32(oacc[dt], ak, bv);
              if constexpr (sizeof(ES) != 4) mma_k32(oacc[dt], al, bv);
            }
          }
        }
      }
    }
  };

  // two steps per trip: the operands of a step are requested while the step before it runs
  for (int base = c0; base < c1; base += 2 * step) {
    do_step(kfA, vfA, base);
    if (base + 2 * step < c1) load_step(kfA, vfA, base + 2 * step);
    if (base + step < c1) {
      do_step(kfB, vfB, base + step);
      if (base + 3 * step < c1) load_step(kfB, vfB, base + 3 * step);
    }
  }

  // ---- merge the tiles of a head --------------------------------------------------------------
  // the owners publish the statistics of their columns; then every lane takes those of its S column
  l_run = row_stride_sum(l_run, 4);
  l_run += __shfl_xor(l_run, 16, kWave);
  l_run += __shfl_xor(l_run, 32, kWave);
  if (lane < 4) {
    st_m[ocol] = m_run;
    st_l[ocol] = l_run;
  }
  __syncthreads();
  const float mc = col_live ? st_m[r16] : -INFINITY;
  const float lcol = st_l[r16];
  const float mstar = row_stride_max(mc, Gp);   // the columns of one head are Gp lanes apart
  const float fc = (mc != -INFINITY) ? __expf(mc - mstar) : 0.0f;
  const float lstar = row_stride_sum(col_live ? lcol * fc : 0.0f, Gp);
  __syncthreads();   // every wave is done with the exchange regions: they are reused below

  // every wave rotates its r' rows to the global frame, scales rows to the head's maximum and
  // parks them in LDS: red_r[row][own orders], red_o[wave][row][kept dims]
  {
    float f[4];
    uint32_t phr[4];
#pragma unroll
    for (int v = 0; v < 4; ++v) {
      const int row = 4 * q4 + v;
      f[v] = __shfl(fc, row, kWave);
      phr[v] = phase_of(p.t0 + last_base + (row / Gp) * kTJ, p.ph_scale);
    }
#pragma unroll
    for (int i = 0; i < CW; ++i) {
      const int c = wave * CW + i;
      const uint32_t n = 16 * c + r16 + 1;
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
        const float rc = racc[2 * i][v], rs = racc[2 * i + 1][v];
        float* dst = red_r + (4 * q4 + v) * pr + 32 * c + r16;
        dst[0] = f[v] * (cs[v] * rc - sn[v] * rs);
        dst[16] = f[v] * (sn[v] * rc + cs[v] * rs);
      }
    }
    float* ro = red_o + wave * 16 * po;
#pragma unroll
    for (int dt = 0; dt < DVTM; ++dt)
      if (dt < DVT)
#pragma unroll
        for (int v = 0; v < 4; ++v) ro[(4 * q4 + v) * po + 16 * dt + r16] = f[v] * oacc[dt][v];
  }
  __syncthreads();

  // record of head h: [max, sum, -, -, acc over the kept dims (16 DVT), r (Mint, V-side order)]
  const size_t rec_h = static_cast<size_t>(p.Sm) * p.recm;
  float* rec0 = p.part_m + (hq0 * p.Sm + sm_idx) * p.recm;
  if (wave == 0 && lane < G) {   // lane = column (tile 0, head lane): holds the head's merged statistics
    rec0[lane * rec_h + 0] = mstar;
    rec0[lane * rec_h + 1] = lstar;
  }
  const int no4 = 4 * DVT, nr4 = Mint / 4, per = no4 + nr4;
  for (int it = tid; it < G * per; it += kBlock) {
    {
      const int h = it / per, x4 = it - h * per;
      f32x4 v = {0.f, 0.f, 0.f, 0.f};
      if (x4 < no4) {
#pragma unroll
        for (int w = 0; w < kWaves; ++w)
#pragma unroll
          for (int k = 0; k < kMaxKT; ++k)
            if (k < KT) v += *reinterpret_cast<const f32x4*>(red_o + ((w * 16 + k * Gp + h) * po + 4 * x4));
      } else {
        const int y = x4 - no4;
#pragma unroll
        for (int k = 0; k < kMaxKT; ++k)
          if (k < KT) v += *reinterpret_cast<const f32x4*>(red_r + ((k * Gp + h) * pr + 4 * y));
      }
      *reinterpret_cast<f32x4*>(rec0 + h * rec_h + 4 + 4 * x4) = v;
    }
  }
}

// ---------------------------------------------------------------------------
// 2c. middle rows, specialised: bf16, groups of at most four query heads, at most 32 kept dims
// ---------------------------------------------------------------------------
// The same algorithm and the same LDS layouts as partial_middle_rows, with every shape that
// decides control flow fixed at compile time (four tiles per step, CW series chunks per wave,
// DVT column tiles of kept V dims, GP = 1 or 4 score columns per tile), so that a step is one
// straight-line instruction stream: no branch sits between a load and its use, every wait
// names the exact number of younger requests, and the loads of the step after next are
// issued unconditionally (clamped into the chunk) right after a step.  The V-side table
// slices are evaluated directly (a rotation recurrence along the eight consecutive rows a
// lane holds) instead of being transposed through LDS, which takes the barriers out of the
// prologue.  The wave-wide maximum of the softmax uses the half- and row-swap lane permutes.

constexpr float kSoftmaxSlack = 8.0f;   // how far a score may exceed its column's reference before the reference moves

// max over the four 16-lane rows of a wave, per lane position, result in every lane
__device__ __forceinline__ float cross_row_max(float v) {
  auto a = __builtin_amdgcn_permlane32_swap(__float_as_uint(v), __float_as_uint(v), false, false);
  v = fmaxf(__uint_as_float(a[0]), __uint_as_float(a[1]));
  auto b = __builtin_amdgcn_permlane16_swap(__float_as_uint(v), __float_as_uint(v), false, false);
  return fmaxf(__uint_as_float(b[0]), __uint_as_float(b[1]));
}
__device__ __forceinline__ float cross_row_sum(float v) {
  auto a = __builtin_amdgcn_permlane32_swap(__float_as_uint(v), __float_as_uint(v), false, false);
  v = __uint_as_float(a[0]) + __uint_as_float(a[1]);
  auto b = __builtin_amdgcn_permlane16_swap(__float_as_uint(v), __float_as_uint(v), false, false);
  return __uint_as_float(b[0]) + __uint_as_float(b[1]);
}

// ---------------------------------------------------------------------------
// 2a'. full-width rows, specialised: bf16, head dim 128, at most four query columns
// ---------------------------------------------------------------------------
// Same arithmetic as partial_full_rows (256 rows per workgroup, 64 per wave).  Everything a wave
// needs from global memory - its 64 K rows, its 64 V rows and the queries, which go straight into
// B operands - is requested at the start, the softmax of a wave stays inside the wave, and the
// waves meet once, at the end.
// RB: 16-row blocks per wave (4: 256 rows per workgroup; 1: 64 rows, for launches with few workgroups)
template <typename T, int RB = kRB>
__device__ __forceinline__ void partial_full_fast(const DecodeParams& p, const SeqView& sv, unsigned char* smem, const int bh, int s) {
  static_assert(sizeof(T) == 2, "16-bit elements");
  constexpr int D = 128, kH = 4;                        // head dim, query columns
  const int b = bh / p.Hkv, hkv = bh % p.Hkv;
  const int G = p.G;
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int q4 = lane >> 4, r16 = lane & 15;
  const size_t hq0 = static_cast<size_t>(b) * p.Hq + hkv * G;
  constexpr int kRowsW = 16 * RB;                      // rows per wave
  const int jw = (s * kWaves + wave) * kRowsW;
  const int nw = max(0, min(kRowsW, sv.W - jw));
  const int jlast = max(sv.W - 1, 0);
  const int jvis = sv.W - p.Tq + r16 / p.Gq;             // last row the query token of column r16 may see

  float* pw = reinterpret_cast<float*>(smem) + wave * kWRows * kH;          // [64 rows][4 columns] probabilities
  float* red = reinterpret_cast<float*>(smem) + kWaves * kWRows * kH;      // [waves][4 columns][128 dims]
  float* wm = red + kWaves * kH * D;                                        // [waves][4] maxima
  float* wl = wm + kWaves * kH;                                             // [waves][4] sums

  // ---- global operands ------------------------------------------------------------------------
  const T* kbase = static_cast<const T*>(p.k_full) + bh * p.full_stride;
  const T* vbase = static_cast<const T*>(p.v_full) + bh * p.full_stride;
  Frag<T> ka[4][RB];
#pragma unroll
  for (int rb = 0; rb < RB; ++rb) {
    const T* krow = kbase + static_cast<int64_t>(min(jw + 16 * rb + r16, jlast)) * D + 8 * q4;
#pragma unroll
    for (int cc = 0; cc < 4; ++cc) ka[cc][rb].load(krow + cc * 32);
  }
  Frag<T> qb[4];
  {
    const T* q = static_cast<const T*>(p.q) + (hq0 + min(r16, G - 1)) * D + 8 * q4;
#pragma unroll
    for (int cc = 0; cc < 4; ++cc) qb[cc].load(q + cc * 32);
  }
  // V rows of this lane: 8 dims (dc) of rows rg, rg + 4, ...
  const int dc = lane & 15, rg = lane >> 4;
  Frag<T> vf[4 * RB];
#pragma unroll
  for (int i = 0; i < 4 * RB; ++i) vf[i].load(vbase + static_cast<int64_t>(min(jw + rg + 4 * i, jlast)) * D + dc * 8);

  // ---- scores of the wave's 64 rows: lane (column r16, q4) gets rows 16 rb + 4 q4 + v -----------
  if (r16 >= G) {
#pragma unroll
    for (int cc = 0; cc < 4; ++cc) qb[cc].zero();
  }
  f32x4 sacc[RB];
#pragma unroll
  for (int rb = 0; rb < RB; ++rb) sacc[rb] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
  for (int cc = 0; cc < 4; ++cc)
#pragma unroll
    for (int rb = 0; rb < RB; ++rb) mma_k32(sacc[rb], ka[cc][rb], qb[cc]);

  // ---- softmax over the wave's rows, per column ---------------------------------------------------
  float m_w = -INFINITY;
#pragma unroll
  for (int rb = 0; rb < RB; ++rb)
#pragma unroll
    for (int v = 0; v < 4; ++v) {
      const int r = 16 * rb + 4 * q4 + v;
      const float sv = (r < nw && r16 < G && jw + r <= jvis) ? sacc[rb][v] * p.scale : -INFINITY;
      sacc[rb][v] = sv;
      m_w = fmaxf(m_w, sv);
    }
  m_w = cross_row_max(m_w);
  const float m_ref = (m_w == -INFINITY) ? 0.0f : m_w;
  float l_w = 0.0f;
#pragma unroll
  for (int rb = 0; rb < RB; ++rb)
#pragma unroll
    for (int v = 0; v < 4; ++v) {
      const float e = __expf(sacc[rb][v] - m_ref);   // masked rows hold -inf -> 0
      l_w += e;
      if (r16 < kH) pw[(16 * rb + 4 * q4 + v) * kH + r16] = e;
    }
  l_w = cross_row_sum(l_w);
  if (lane < kH) {
    wm[wave * kH + lane] = m_w;
    wl[wave * kH + lane] = l_w;
  }
  // the probabilities were written by this wave and are read by this wave: no barrier, the LDS
  // operations of a wave complete in order
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
  __builtin_amdgcn_wave_barrier();
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");

  // ---- sum_j p_j V[j,:] over this lane's rows ---------------------------------------------------
  float acc[kH][8];
#pragma unroll
  for (int h = 0; h < kH; ++h)
#pragma unroll
    for (int e = 0; e < 8; ++e) acc[h][e] = 0.0f;
#pragma unroll
  for (int i = 0; i < 4 * RB; ++i) {
    const int r = rg + 4 * i;
    const f32x4 p4 = *reinterpret_cast<const f32x4*>(pw + r * kH);   // rows past the end hold zeros
    float x[8];
    unpack8(vf[i], x);
#pragma unroll
    for (int h = 0; h < kH; ++h)
#pragma unroll
      for (int e = 0; e < 8; ++e) acc[h][e] += p4[h] * x[e];
  }
  // the four row groups of the wave meet in its first 16 lanes
#pragma unroll
  for (int h = 0; h < kH; ++h)
#pragma unroll
    for (int e = 0; e < 8; ++e) acc[h][e] = cross_row_sum(acc[h][e]);
  if (rg == 0) {
#pragma unroll
    for (int h = 0; h < kH; ++h) {
      float* dst = red + (wave * kH + h) * D + dc * 8;
      *reinterpret_cast<f32x4*>(dst) = f32x4{acc[h][0], acc[h][1], acc[h][2], acc[h][3]};
      *reinterpret_cast<f32x4*>(dst + 4) = f32x4{acc[h][4], acc[h][5], acc[h][6], acc[h][7]};
    }
  }
  __syncthreads();

  // ---- the waves meet: record of column h = [max, sum, -, -, acc[128]] ---------------------------
  if (tid < kH * (D / 4)) {
    const int h = tid / (D / 4), d4 = tid % (D / 4);
    if (h < G) {
      float ms = wm[h];
#pragma unroll
      for (int w = 1; w < kWaves; ++w) ms = fmaxf(ms, wm[w * kH + h]);
      f32x4 v = {0.f, 0.f, 0.f, 0.f};
      float l = 0.0f;
#pragma unroll
      for (int w = 0; w < kWaves; ++w) {
        const float mw = wm[w * kH + h];
        const float f = (mw == -INFINITY) ? 0.0f : __expf(mw - ms);
        l += f * wl[w * kH + h];
        v += f * *reinterpret_cast<const f32x4*>(red + (w * kH + h) * D + 4 * d4);
      }
      float* rec = sv.part_w + ((hq0 + h) * sv.Sw + s) * p.recw;
      *reinterpret_cast<f32x4*>(rec + 4 + 4 * d4) = v;
      if (d4 == 0) {
        rec[0] = ms;
        rec[1] = l;
      }
    }
  }
}

// One launch for the two parts of a call that do not depend on each other: the series
// coefficients g (the first p.nprep workgroups of a row of the grid) and the partial records of
// the full-width rows (the others).  The first is a chain of round trips that leaves the chip
// idle, the second is a stream: together they take about as long as the longer of the two.
template <typename T, int TPR>
__global__ __launch_bounds__(kBlock) void decode_prepare_window(DecodeParams p) {
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  if (static_cast<int>(blockIdx.x) < p.nprep) {
    prepare2_rows<T, TPR>(p, blockIdx.y, blockIdx.x);
  } else {
    const int s = blockIdx.x - p.nprep;
    if constexpr (sizeof(T) == 2) {
      if (p.D == 128 && p.G <= 4) {
        if (p.wrb == 1) partial_full_fast<T, 1>(p, call_view(p, blockIdx.y / p.Hkv), smem, blockIdx.y, s);
        else partial_full_fast<T>(p, call_view(p, blockIdx.y / p.Hkv), smem, blockIdx.y, s);
      } else {
        partial_full_rows<T>(p, smem, s);
      }
    } else {
      partial_full_rows<T>(p, smem, s);
    }
  }
}

// g = diag(w) C_k q[D^kc], the constant-term coefficient and q at the kept K dims, formed by the
// workgroup that uses them and left in the LDS places the middle-row phase reads.  Four threads
// share a row of C_k (interleaved 128-bit vectors); the rows of all NP passes of 64 rows are
// requested by issue(), before anything is waited for; finish() runs after the caller's own
// independent work (the table build of the middle-row phase).  The query at the compressed dims is
// staged at the start of the exchange region, which the middle-row phase only writes after its
// own barrier.
template <int NP>
struct FusedCoeffs {
  using T = bf16_t;
  static constexpr int D = 128, kV = D / 16;   // 128-bit vectors of a row per thread (compressed dims <= 124)
  static constexpr int Mint = (NP - 1) * 64, kPitchG = Mint + 32;
  f32x4 cv4[NP][kV];
  uint8_t mb[2];
  T qe[2];

  __device__ __forceinline__ void issue(const DecodeParams& p, const int bh) {
    const int tid = threadIdx.x, lane = tid & 63;
    const int b = bh / p.Hkv, hkv = bh % p.Hkv;
    const int Dkc = p.Dkc, M = p.M;
    const int row = tid >> 2, seg = tid & 3, c4n = Dkc / 4;
    const float* ck0 = p.ck + static_cast<size_t>(bh) * M * Dkc;
#pragma unroll
    for (int ps = 0; ps < NP; ++ps) {
      const float* ckr = ck0 + static_cast<size_t>(min(row + 64 * ps, M - 1)) * Dkc;
#pragma unroll
      for (int i = 0; i < kV; ++i)
        if (4 * i < c4n) cv4[ps][i] = *reinterpret_cast<const f32x4*>(ckr + 4 * min(seg + 4 * i, c4n - 1));
    }
#pragma unroll
    for (int j = 0; j < 2; ++j) mb[j] = p.kmask[static_cast<size_t>(bh) * D + lane + 64 * j];
    const size_t hq0 = static_cast<size_t>(b) * p.Hq + hkv * p.G;
    const T* q = static_cast<const T*>(p.q) + hq0 * D;
    const int nqe = p.G * D;   // <= 512
#pragma unroll
    for (int i = 0; i < 2; ++i) qe[i] = q[min(tid + i * kBlock, nqe - 1)];
  }

  __device__ __forceinline__ void finish(const DecodeParams& p, unsigned char* smem) {
    const int tid = threadIdx.x;
    const int Dkc = p.Dkc, G = p.G, M = p.M;
    const int row = tid >> 2, seg = tid & 3, c4n = Dkc / 4;
    float* qc = reinterpret_cast<float*>(smem);                    // [G][Dkc]
    float* gs_s = reinterpret_cast<float*>(smem + p.lds_tab);      // [G][Mint + 32]
    T* qk_s = reinterpret_cast<T*>(gs_s + G * kPitchG);            // [G][32]
    float* g0_s = reinterpret_cast<float*>(qk_s + G * 32);         // [G]
    uint64_t kbal[4];
    kbal[0] = __ballot(mb[0] != 0);
    kbal[1] = __ballot(mb[1] != 0);
    kbal[2] = kbal[3] = 0;
    const int nqe = G * D;
#pragma unroll
    for (int i = 0; i < 2; ++i) {
      const int it = tid + i * kBlock;
      if (it < nqe) {
        const int h = it >> 7, d = it & 127;
        const int r = dim_rank(kbal, d);
        if (r < 0) qc[h * Dkc + (-r - 1)] = to_f32(qe[i]);
        else qk_s[h * 32 + r] = qe[i];
      }
    }
    {
      const int npad = 32 - p.Dku;
      if (tid < G * npad) qk_s[(tid / npad) * 32 + p.Dku + tid % npad] = T{};
    }
    __syncthreads();
#pragma unroll
    for (int ps = 0; ps < NP; ++ps) {
      const int m = row + 64 * ps;
      const float w = (m < M) ? basis_weight((m + 1) / 2, p.T) : 0.0f;
      for (int h = 0; h < G; ++h) {
        const float* qh = qc + h * Dkc;
        float acc = 0.0f;
#pragma unroll
        for (int i = 0; i < kV; ++i) {
          if (4 * i < c4n) {
            const int c4 = seg + 4 * i;
            const f32x4 qv = *reinterpret_cast<const f32x4*>(qh + 4 * min(c4, c4n - 1));
            const f32x4 c = cv4[ps][i];
            const float d4 = (c[0] * qv[0] + c[1] * qv[1]) + (c[2] * qv[2] + c[3] * qv[3]);
            acc += (c4 < c4n) ? d4 : 0.0f;
          }
        }
        acc += __shfl_xor(acc, 1, kWave);
        acc += __shfl_xor(acc, 2, kWave);
        if (seg == 0 && m <= Mint) {
          if (m == 0) g0_s[h] = acc * w;
          else gs_s[h * kPitchG + (m - 1)] = acc * w;
        }
      }
    }
    // (the barrier that publishes g is the caller's)
  }
};

// C_v of the pair goes straight from global memory into LDS (no registers, nothing waits for it
// here): every wave copies 1 KB blocks, lane i of a block supplying bytes 16 i .. 16 i + 15.  The
// last block may reach past the matrix: its lanes re-read the last vector (the stash is padded).
__device__ __forceinline__ void fused_stash_cv(const DecodeParams& p, unsigned char* smem, const int bh,
                                               const unsigned lds_cv) {
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const unsigned bytes = static_cast<unsigned>(p.M) * p.Dvc * 4u;
  const unsigned nblk = (bytes + 1023u) >> 10;
  const char* src = reinterpret_cast<const char*>(p.cv + static_cast<size_t>(bh) * p.M * p.Dvc);
  for (unsigned blk = wave; blk < nblk; blk += kWaves) {
    const unsigned off = min(blk * 1024u + 16u * lane, bytes - 16u);
    __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)(src + off),
                                     (__attribute__((address_space(3))) void*)(smem + lds_cv + blk * 1024u), 16, 0, 0);
  }
}

// FUSED (the one-launch form): the series coefficients, the constant-term coefficient and the packed
// query are formed here, around the table build, and C_v is sent on its way into LDS
template <int CW, int DVT, int GP, bool FUSED = false>
__device__ __forceinline__ void partial_middle_fast(const DecodeParams& p, const SeqView& sv, unsigned char* smem,
                                                    const int bh, const int sm_idx) {
  using T = bf16_t;
  using ES = f16_t;
  constexpr int Mint = kWaves * CW * 32;
  constexpr int KT = 4, step = KT * kTJ;
  static_assert(GP == 1 || GP == 4, "score columns per tile");
  static_assert(DVT == 1 || DVT == 2, "kept V column tiles");

  const int b = bh / p.Hkv, hkv = bh % p.Hkv;
  const int G = p.G;
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int q4 = lane >> 4, r16 = lane & 15;
  const size_t hq0 = static_cast<size_t>(b) * p.Hq + hkv * G;
  const int c0 = sm_idx * sv.chunk_m, c1 = min(sv.N, c0 + sv.chunk_m);
  if constexpr (!FUSED) {
    if (c0 >= sv.N) {   // (only with per-sequence counts) nothing of this chunk belongs to the sequence
      write_empty_middle(p, hq0, sm_idx, sm_idx + 1, kBlock);
      return;
    }
  }
  const int nsteps = (c1 - c0 + step - 1) / step;
  const int col_k = r16 / GP, col_h = r16 % GP;
  const bool col_live = col_k < KT && col_h < G;
  const int hsafe = min(col_h, G - 1);
  const int kpitch = (p.Dku + 7) & ~7;               // 8 .. 32
  constexpr int Dkq = 32;                             // pitch of the packed query rows
  const int Dvu = p.Dvu;
  const T* kk = static_cast<const T*>(p.k_keep) + bh * p.kk_stride;
  const T* vk = static_cast<const T*>(p.v_keep) + bh * p.vk_stride;
  const int Nm1 = sv.N - 1;

  // ---- LDS carve-up (as partial_middle_rows) -------------------------------
  f32x4* xs = reinterpret_cast<f32x4*>(smem);
  constexpr unsigned kXsBytes = kWaves * kRB * 64 * 16;
  ES* pse = reinterpret_cast<ES*>(smem + kXsBytes);
  T* pte = reinterpret_cast<T*>(smem + kXsBytes + kXN * 16 * 4 * 8 * sizeof(ES));
  T* ptl = reinterpret_cast<T*>(smem + kXsBytes + kXN * 16 * 4 * 8 * (sizeof(ES) + sizeof(T)));
  float* alpha_s = reinterpret_cast<float*>(smem + kXsBytes + kXN * 16 * 4 * 8 * (sizeof(ES) + 2 * sizeof(T)));
  float* st_m = alpha_s + 16;
  float* st_l = st_m + 16;
  float* red_r = reinterpret_cast<float*>(smem);
  constexpr int pr = Mint + 4, po = 16 * DVT + 4;
  float* red_o = red_r + 16 * pr;
  constexpr int kPitchG = Mint + 32;
  float* gs_s = reinterpret_cast<float*>(smem + p.lds_tab);
  T* qk_s = reinterpret_cast<T*>(gs_s + G * kPitchG);
  const float* g0_s = reinterpret_cast<const float*>(qk_s + G * 32);

  // this wave's kept operands of the step at `base`: the four row blocks and the two token
  // blocks of tile `wave`.  Rows are clamped into the slab (rows past the chunk are masked at the
  // softmax); K columns past the row pitch re-read the row's last 8 columns, where q is zero.
  const int urow_lane = 8 * (r16 >> 2) + (r16 & 3);
  const uint32_t kcol = static_cast<uint32_t>(min(8 * q4, kpitch - 8));
  auto load_step = [&](Frag<T> (&kf)[4], Frag<T> (&vf)[2][DVT], int base) {
#pragma unroll
    for (int rb = 0; rb < 4; ++rb) {
      const int u = 32 * (rb >> 1) + 4 * (rb & 1) + urow_lane;
      const int j = min(base + wave * kTJ + u, Nm1);
      kf[rb].load(kk + (static_cast<uint32_t>(j) * static_cast<uint32_t>(kpitch) + kcol));
    }
#pragma unroll
    for (int i = 0; i < 2; ++i) {
      const int tok0 = base + wave * kTJ + 32 * i + 8 * q4;
      const uint32_t g8 = static_cast<uint32_t>(min(tok0, Nm1)) >> 3;
#pragma unroll
      for (int dt = 0; dt < DVT; ++dt) {
        const int dim = min(16 * dt + r16, Dvu - 1);
        vf[i][dt].load(vk + (g8 * static_cast<uint32_t>(Dvu) + static_cast<uint32_t>(dim)) * 8u);
      }
    }
  };

  // ---- (0) everything that comes from global memory is requested first ------------
  constexpr int kGLoads = (Mint + kBlock - 1) / kBlock;   // G <= 4 heads of Mint floats, as float4
  const int ng4 = G * Mint / 4;
  f32x4 gv[kGLoads];
  if constexpr (!FUSED) {
#pragma unroll
    for (int i = 0; i < kGLoads; ++i)
      gv[i] = *reinterpret_cast<const f32x4*>(p.gs + hq0 * Mint + 4 * min(tid + i * kBlock, ng4 - 1));
  }
  const int ocol = 4 * wave + (lane & 3), orb = lane >> 4, oq4 = (lane >> 2) & 3;
  const int ocol_k = ocol / GP, ocol_h = ocol % GP;
  const bool olive = ocol_k < KT && ocol_h < G;
  float g0 = 0.0f;
  // packed query at the kept K dims: G rows of 32 elements = at most 16 vectors of 8
  Frag<T> qv;
  FusedCoeffs<FUSED ? 2 * CW + 1 : 1> coeffs;
  if constexpr (!FUSED) {
    g0 = p.g0[hq0 + min(ocol_h, G - 1)];
    qv.load(static_cast<const T*>(p.qkeep) + hq0 * Dkq + 8 * min(tid, G * 4 - 1));
  } else {
    coeffs.issue(p, bh);
    if (p.Dvc > 0) fused_stash_cv(p, smem, bh, fused_lds(p.lds_tab, G, Mint, p.recm, p.recw, p.M, p.Dvc).cv);
  }
  Frag<T> kfA[4], kfB[4];
  Frag<T> vfA[2][DVT], vfB[2][DVT];
  load_step(kfA, vfA, c0);
  load_step(kfB, vfB, c0 + min(1, nsteps - 1) * step);

  // ---- this wave's slices of the E table, evaluated in registers -----------------------------
  Frag<ES> eA[CW][kRB], eB[CW][2][kXN];
  float tc[CW], ts[CW];
  {
    const int n_max = p.M / 2;
    const float invT = 1.0f / static_cast<float>(p.T);
    // K side: row u(rb, r16), slots = (cos, sin) of the 4 consecutive orders n0 .. n0 + 3; the first
    // order is evaluated, the others follow by the angle-addition step of the row
    float cd[kRB], sd[kRB];
    int urow[kRB];
#pragma unroll
    for (int rb = 0; rb < kRB; ++rb) {
      urow[rb] = 32 * (rb >> 1) + 4 * (rb & 1) + urow_lane;
      table_cs<T>(1, urow[rb], p.T, invT, &cd[rb], &sd[rb]);
    }
#pragma unroll
    for (int i = 0; i < CW; ++i) {
      const int n0 = 16 * (wave * CW + i) + 4 * q4 + 1;
#pragma unroll
      for (int rb = 0; rb < kRB; ++rb) {
        float vals[8];
        table_cs<T>(n0, urow[rb], p.T, invT, &vals[0], &vals[1]);
#pragma unroll
        for (int hp = 1; hp < 4; ++hp) {
          vals[2 * hp] = vals[2 * hp - 2] * cd[rb] - vals[2 * hp - 1] * sd[rb];
          vals[2 * hp + 1] = vals[2 * hp - 1] * cd[rb] + vals[2 * hp - 2] * sd[rb];
        }
#pragma unroll
        for (int hp = 0; hp < 4; ++hp)
          if (n0 + hp > n_max) vals[2 * hp] = vals[2 * hp + 1] = 0.0f;
        pack8(eA[i][rb], vals);
      }
    }
    // V side: order n = 16 c + r16 + 1 at the 8 consecutive rows 32 x + 8 q4 + e: the first row is
    // evaluated, the others follow by the angle-addition step of the order
#pragma unroll
    for (int i = 0; i < CW; ++i) {
      const int n = 16 * (wave * CW + i) + r16 + 1;
      float cn, sn;
      table_cs<T>(n, 1, p.T, invT, &cn, &sn);
#pragma unroll
      for (int x = 0; x < kXN; ++x) {
        float cs[8], ss[8];
        table_cs<T>(n, 32 * x + 8 * q4, p.T, invT, &cs[0], &ss[0]);
#pragma unroll
        for (int e = 1; e < 8; ++e) {
          cs[e] = cs[e - 1] * cn - ss[e - 1] * sn;
          ss[e] = ss[e - 1] * cn + cs[e - 1] * sn;
        }
        if (n > n_max) {
#pragma unroll
          for (int e = 0; e < 8; ++e) cs[e] = ss[e] = 0.0f;
        }
        pack8(eB[i][0][x], cs);
        pack8(eB[i][1][x], ss);
      }
    }
    // the V-side accumulators live in a frame that moves with the steps
    const uint32_t ph_step = phase_of(step, p.ph_scale);
#pragma unroll
    for (int i = 0; i < CW; ++i)
      phase_cs<T>(static_cast<uint32_t>(16 * (wave * CW + i) + r16 + 1) * ph_step, &tc[i], &ts[i]);
  }

  // ---- series coefficients and packed query into LDS ---------------------------------------------
  if constexpr (!FUSED) {
#pragma unroll
    for (int i = 0; i < kGLoads; ++i) {
      const int v4 = tid + i * kBlock;
      if (v4 < ng4) *reinterpret_cast<f32x4*>(gs_s + (4 * v4 / Mint) * kPitchG + (4 * v4) % Mint) = gv[i];
    }
    if (tid < G * 4) *reinterpret_cast<Frag<T>*>(qk_s + 8 * tid) = qv;
  } else {
    coeffs.finish(p, smem);
  }
  __syncthreads();
  if constexpr (FUSED) g0 = g0_s[min(ocol_h, G - 1)];
  // this lane's B operand of the kept-K products: q of its column's head, only in the columns of tile `wave`
  Frag<T> bq;
  bq.load(qk_s + hsafe * Dkq + 8 * q4);
  if (col_k != wave || !col_live) bq.zero();

  f32x4 racc[2 * CW];
  f32x4 oacc[DVT];
#pragma unroll
  for (int t = 0; t < 2 * CW; ++t) racc[t] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
  for (int t = 0; t < DVT; ++t) oacc[t] = f32x4{0.f, 0.f, 0.f, 0.f};
  float m_run = -INFINITY, l_run = 0.0f;

  // FUSED (a wave has the registers): the K-side coefficients of this lane's column (tile, head), four
  // orders per slice, stay in registers rotated to the tile origin of the current step and are
  // turned on by one step's angle after use (angle addition, four multiply-adds per order), instead
  // of being evaluated from g in every step; they are taken afresh from g every 32 steps, so that the
  // rounding of the turns never builds up over a long sequence.
  float gk[FUSED ? CW : 1][8], tkc[FUSED ? CW : 1][4], tks[FUSED ? CW : 1][4];
  auto seed_gk = [&](int base) {
    if constexpr (FUSED) {
      const uint32_t ph_k = phase_of(p.t0 + base + col_k * kTJ, p.ph_scale);
#pragma unroll
      for (int i = 0; i < CW; ++i) {
        const uint32_t n0 = 16 * (wave * CW + i) + 4 * q4 + 1;
        const float* gl = gs_s + hsafe * kPitchG + 32 * (wave * CW + i) + 8 * q4;
        const f32x4 ga = *reinterpret_cast<const f32x4*>(gl), gb = *reinterpret_cast<const f32x4*>(gl + 4);
#pragma unroll
        for (int j = 0; j < 4; ++j) {
          float cs, sn;
          phase_cs<T>((n0 + j) * ph_k, &cs, &sn);
          const float gc = (j < 2) ? ga[2 * (j & 1)] : gb[2 * (j & 1)];
          const float gsn = (j < 2) ? ga[2 * (j & 1) + 1] : gb[2 * (j & 1) + 1];
          gk[i][2 * j] = gc * cs + gsn * sn;
          gk[i][2 * j + 1] = gsn * cs - gc * sn;
        }
      }
    }
  };
  if constexpr (FUSED) {
    const uint32_t ph_step = phase_of(step, p.ph_scale);
#pragma unroll
    for (int i = 0; i < CW; ++i)
#pragma unroll
      for (int j = 0; j < 4; ++j)
        phase_cs<T>(static_cast<uint32_t>(16 * (wave * CW + i) + 4 * q4 + 1 + j) * ph_step, &tkc[i][j], &tks[i][j]);
    seed_gk(c0);
  }

  auto do_step = [&](Frag<T> (&kf)[4], Frag<T> (&vf)[2][DVT], int base, auto tail_tag) {
    constexpr bool kTail = decltype(tail_tag)::value;
    f32x4 sacc[kRB];
#pragma unroll
    for (int rb = 0; rb < kRB; ++rb) sacc[rb] = f32x4{0.f, 0.f, 0.f, 0.f};

    // -- (a) series on the K side, own orders: S += E g'(tile origin) -----------------
    if constexpr (FUSED) {
#pragma unroll
      for (int i = 0; i < CW; ++i) {
        Frag<ES> bg;   // (columns without a query head get some head's values: their scores are never used)
        pack8(bg, gk[i]);
#pragma unroll
        for (int rb = 0; rb < kRB; ++rb) mma_k32(sacc[rb], eA[i][rb], bg);
#pragma unroll
        for (int j = 0; j < 4; ++j) {
          const float gc = gk[i][2 * j], gsn = gk[i][2 * j + 1];
          gk[i][2 * j] = tkc[i][j] * gc + tks[i][j] * gsn;
          gk[i][2 * j + 1] = tkc[i][j] * gsn - tks[i][j] * gc;
        }
      }
    } else {
      const uint32_t ph_k = phase_of(p.t0 + base + col_k * kTJ, p.ph_scale);
#pragma unroll
      for (int i = 0; i < CW; ++i) {
        const uint32_t n0 = 16 * (wave * CW + i) + 4 * q4 + 1;
        float csv[4], snv[4];
        if constexpr (GP >= 4) {          // the 4 lanes of a quad share (tile, q4): one evaluation each
          float cs, sn;
          phase_cs<T>((n0 + (lane & 3)) * ph_k, &cs, &sn);
#pragma unroll
          for (int j = 0; j < 4; ++j) {
            csv[j] = quad_bcast(cs, j);
            snv[j] = quad_bcast(sn, j);
          }
        } else {
#pragma unroll
          for (int j = 0; j < 4; ++j) phase_cs<T>((n0 + j) * ph_k, &csv[j], &snv[j]);
        }
        const float* gl = gs_s + hsafe * kPitchG + 32 * (wave * CW + i) + 8 * q4;
        const f32x4 ga = *reinterpret_cast<const f32x4*>(gl), gb = *reinterpret_cast<const f32x4*>(gl + 4);
        float gp[8];
#pragma unroll
        for (int j = 0; j < 4; ++j) {
          const float gc = (j < 2) ? ga[2 * (j & 1)] : gb[2 * (j & 1)];
          const float gsn = (j < 2) ? ga[2 * (j & 1) + 1] : gb[2 * (j & 1) + 1];
          gp[2 * j] = gc * csv[j] + gsn * snv[j];
          gp[2 * j + 1] = gsn * csv[j] - gc * snv[j];
        }
        Frag<ES> bg;   // (columns without a query head get some head's values: their scores are never used)
        pack8(bg, gp);
#pragma unroll
        for (int rb = 0; rb < kRB; ++rb) mma_k32(sacc[rb], eA[i][rb], bg);
      }
    }
    // -- (b) kept K dims of tile `wave`: A = K^mu rows, B = q masked to the tile's columns --
#pragma unroll
    for (int rb = 0; rb < kRB; ++rb) mma_k32(sacc[rb], kf[rb], bq);

    // -- (c) the partial scores of the four waves meet; this wave sums its four columns --------
    {
      f32x4* xw = xs + (wave * kRB) * 64 + lane;
#pragma unroll
      for (int rb = 0; rb < kRB; ++rb) xw[rb * 64] = sacc[rb];
    }
    __syncthreads();
    f32x4 sv;
    {
      const f32x4* xr = xs + orb * 64 + oq4 * 16 + ocol;
      sv = ((xr[0 * kRB * 64] + xr[1 * kRB * 64]) + xr[2 * kRB * 64]) + xr[3 * kRB * 64];
    }
    // -- (d) online softmax of the own columns: lane holds rows u = 32x + 8 oq4 + 4y + v (orb = 2x + y)
    float pv[4];
    float m_tile = -INFINITY;
#pragma unroll
    for (int v = 0; v < 4; ++v) {
      float sc = (sv[v] + g0) * p.scale;
      if constexpr (kTail) {
        const int u = 32 * (orb >> 1) + 8 * oq4 + 4 * (orb & 1) + v;
        if (base + ocol_k * kTJ + u >= c1) sc = -INFINITY;
      }
      if (!olive) sc = -INFINITY;
      pv[v] = sc;
      m_tile = fmaxf(m_tile, sc);
    }
    // The reference m_run of a column only has to keep exp(score - m_run) inside the range of the
    // 16-bit probabilities, not to be the maximum: it moves when a score of one of the wave's columns
    // exceeds it by more than kSoftmaxSlack (always in a chunk's first step), and only then is there a
    // maximum to reduce and a factor to apply.
    float alpha = 1.0f;
    if (__builtin_amdgcn_ballot_w64(m_tile > m_run + kSoftmaxSlack) != 0) {   // (uniform over the wave)
      m_tile = row_stride_max(m_tile, 4);                    // the 16 lanes of a column are 4 apart
      m_tile = cross_row_max(m_tile);
      const float m_new = fmaxf(m_run, m_tile);
      alpha = __expf(m_run - ((m_new == -INFINITY) ? 0.0f : m_new));   // m_run = -inf -> 0
      m_run = m_new;
    }
    const float m_ref = (m_run == -INFINITY) ? 0.0f : m_run;
    float l_add = 0.0f;
#pragma unroll
    for (int v = 0; v < 4; ++v) {
      pv[v] = __expf(pv[v] - m_ref);
      l_add += pv[v];
    }
    l_run = l_run * alpha + l_add;
    {
      const int slot = (((orb >> 1) * 16 + ocol) * 4 + oq4) * 8 + 4 * (orb & 1);
      u32x2d w;
      w[0] = __builtin_bit_cast(uint32_t, __builtin_convertvector(f32x2{pv[0], pv[1]}, f16x2));
      w[1] = __builtin_bit_cast(uint32_t, __builtin_convertvector(f32x2{pv[2], pv[3]}, f16x2));
      *reinterpret_cast<u32x2d*>(reinterpret_cast<uint16_t*>(pse) + slot) = w;
      w[0] = __builtin_bit_cast(uint32_t, __builtin_convertvector(f32x2{pv[0], pv[1]}, bf16x2));
      w[1] = __builtin_bit_cast(uint32_t, __builtin_convertvector(f32x2{pv[2], pv[3]}, bf16x2));
      *reinterpret_cast<u32x2d*>(reinterpret_cast<uint16_t*>(pte) + slot) = w;
      float lo[4];
#pragma unroll
      for (int v = 0; v < 4; ++v)
        lo[v] = pv[v] - __builtin_bit_cast(float, ((w[v >> 1] >> (16 * (v & 1))) & 0xffffu) << 16);
      w[0] = __builtin_bit_cast(uint32_t, __builtin_convertvector(f32x2{lo[0], lo[1]}, bf16x2));
      w[1] = __builtin_bit_cast(uint32_t, __builtin_convertvector(f32x2{lo[2], lo[3]}, bf16x2));
      *reinterpret_cast<u32x2d*>(reinterpret_cast<uint16_t*>(ptl) + slot) = w;
      if (lane < 4) alpha_s[ocol] = alpha;
    }
    __syncthreads();
    // -- (e) bring the accumulators into this step's frame (the first step scales zeros by zero) --
    {
      const f32x4 al = *reinterpret_cast<const f32x4*>(alpha_s + 4 * q4);
      const bool moved = al[0] != 1.0f || al[1] != 1.0f || al[2] != 1.0f || al[3] != 1.0f;
      if (__builtin_amdgcn_ballot_w64(moved) != 0) {   // some column's reference moved: factors to apply
#pragma unroll
        for (int t = 0; t < DVT; ++t)
#pragma unroll
          for (int v = 0; v < 4; ++v) oacc[t][v] *= al[v];
#pragma unroll
        for (int i = 0; i < CW; ++i)
#pragma unroll
          for (int v = 0; v < 4; ++v) {
            racc[2 * i][v] *= al[v];
            racc[2 * i + 1][v] *= al[v];
          }
      }
#pragma unroll
      for (int i = 0; i < CW; ++i)
#pragma unroll
        for (int v = 0; v < 4; ++v) {
          const float rc = racc[2 * i][v], rs = racc[2 * i + 1][v];
          racc[2 * i][v] = tc[i] * rc + ts[i] * rs;
          racc[2 * i + 1][v] = tc[i] * rs - ts[i] * rc;
        }
    }
    // -- (f) V side, own orders: r' += P^T E;  (g) kept V dims of tile `wave`: O += P^T V^mu -------
#pragma unroll
    for (int x = 0; x < kXN; ++x) {
      Frag<ES> ps;
      Frag<T> pt, pl;
      ps.load(pse + ((x * 16 + r16) * 4 + q4) * 8);
      pt.load(pte + ((x * 16 + r16) * 4 + q4) * 8);
      pl.load(ptl + ((x * 16 + r16) * 4 + q4) * 8);
#pragma unroll
      for (int i = 0; i < CW; ++i) {
        mma_k32(racc[2 * i], ps, eB[i][0][x]);
        mma_k32(racc[2 * i + 1], ps, eB[i][1][x]);
      }
      if (col_k != wave) {   // this wave's token blocks belong to tile `wave`: other columns contribute nothing
        pt.zero();
        pl.zero();
      }
#pragma unroll
      for (int dt = 0; dt < DVT; ++dt) {
        Frag<T> bv = vf[x][dt];
        if ((Dvu & 15) != 0 && 16 * dt + r16 >= Dvu) bv.zero();
        if constexpr (kTail) {
          const int tok0 = base + wave * kTJ + 32 * x + 8 * q4;
          if (tok0 + 8 > c1) mask_tail(bv, c1 - tok0);
        }
        mma_k32(oacc[dt], pt, bv);
        mma_k32(oacc[dt], pl, bv);
      }
    }
  };

  // (four steps of operands in flight, which the one-launch form has the registers for, made its
  // 4 K-token chunks slower: 38.5 -> 41.5 us; the loop does not wait for memory)
  const int last_base = c0 + (nsteps - 1) * step;
  {
    // two steps per trip: the operands of a step are requested two steps ahead, clamped into the chunk
    int s = 0;
    for (; s + 2 < nsteps; s += 2) {
      const int base = c0 + s * step;
      if constexpr (FUSED) {
        if ((s & 31) == 0 && s > 0) seed_gk(base);
      }
      do_step(kfA, vfA, base, std::false_type{});
      load_step(kfA, vfA, min(base + 2 * step, last_base));
      do_step(kfB, vfB, base + step, std::false_type{});
      load_step(kfB, vfB, min(base + 3 * step, last_base));
    }
    const int base = c0 + s * step;
    if (nsteps - s == 2) {
      do_step(kfA, vfA, base, std::false_type{});
      do_step(kfB, vfB, base + step, std::true_type{});
    } else {
      do_step(kfA, vfA, base, std::true_type{});
    }
  }

  // ---- merge the tiles of a head --------------------------------------------------------------
  l_run = row_stride_sum(l_run, 4);
  l_run = cross_row_sum(l_run);
  if (lane < 4) {
    st_m[ocol] = m_run;
    st_l[ocol] = l_run;
  }
  __syncthreads();
  const float mc = col_live ? st_m[r16] : -INFINITY;
  const float lcol = st_l[r16];
  const float mstar = row_stride_max(mc, GP);   // the columns of one head are GP lanes apart
  const float fc = (mc != -INFINITY) ? __expf(mc - mstar) : 0.0f;
  const float lstar = row_stride_sum(col_live ? lcol * fc : 0.0f, GP);
  __syncthreads();   // every wave is done with the exchange regions: they are reused below

  {
    float f[4];
    uint32_t phr[4];
#pragma unroll
    for (int v = 0; v < 4; ++v) {
      const int row = 4 * q4 + v;
      f[v] = __shfl(fc, row, kWave);
      phr[v] = phase_of(p.t0 + last_base + (row / GP) * kTJ, p.ph_scale);
    }
#pragma unroll
    for (int i = 0; i < CW; ++i) {
      const int c = wave * CW + i;
      const uint32_t n = 16 * c + r16 + 1;
      float cs[4], sn[4];
      phase_cs<T>(n * phr[0], &cs[0], &sn[0]);
      if constexpr (GP >= 4) {   // rows 4*q4 .. 4*q4+3 belong to one tile
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
        const float rc = racc[2 * i][v], rs = racc[2 * i + 1][v];
        float* dst = red_r + (4 * q4 + v) * pr + 32 * c + r16;
        dst[0] = f[v] * (cs[v] * rc - sn[v] * rs);
        dst[16] = f[v] * (sn[v] * rc + cs[v] * rs);
      }
    }
    float* ro = red_o + wave * 16 * po;
#pragma unroll
    for (int dt = 0; dt < DVT; ++dt)
#pragma unroll
      for (int v = 0; v < 4; ++v) ro[(4 * q4 + v) * po + 16 * dt + r16] = f[v] * oacc[dt][v];
  }
  __syncthreads();

  // record of head h: [max, sum, -, -, acc over the kept dims (16 DVT), r (Mint, V-side order)]
  // (FUSED: the record stays in LDS, past the regions read here)
  const size_t rec_h = FUSED ? static_cast<size_t>(p.recm) : static_cast<size_t>(sv.Sm) * p.recm;
  float* rec0 = FUSED ? reinterpret_cast<float*>(smem + fused_lds(p.lds_tab, G, Mint, p.recm, p.recw, p.M, p.Dvc).recm)
                      : sv.part_m + (hq0 * sv.Sm + sm_idx) * p.recm;
  if (wave == 0 && lane < G) {
    rec0[lane * rec_h + 0] = mstar;
    rec0[lane * rec_h + 1] = lstar;
  }
  constexpr int no4 = 4 * DVT, nr4 = Mint / 4, per = no4 + nr4;
  for (int it = tid; it < G * per; it += kBlock) {
    const int h = it / per, x4 = it - h * per;
    f32x4 v = {0.f, 0.f, 0.f, 0.f};
    if (x4 < no4) {
      // kept dims of tile k were accumulated by wave k alone
#pragma unroll
      for (int k = 0; k < KT; ++k) v += *reinterpret_cast<const f32x4*>(red_o + ((k * 16 + k * GP + h) * po + 4 * x4));
    } else {
      const int y = x4 - no4;
#pragma unroll
      for (int k = 0; k < KT; ++k) v += *reinterpret_cast<const f32x4*>(red_r + ((k * GP + h) * pr + 4 * y));
    }
    *reinterpret_cast<f32x4*>(rec0 + h * rec_h + 4 + 4 * x4) = v;
  }
}

template <int CW, int DVT, int GP>
__global__ __launch_bounds__(kBlock, CW <= 2 ? 2 : 1) void decode_partial_fast(DecodeParams p) {
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  if (static_cast<int>(blockIdx.x) < p.Sm) partial_middle_fast<CW, DVT, GP>(p, call_view(p, blockIdx.y / p.Hkv), smem, blockIdx.y, blockIdx.x);
  else if (p.D == 128) partial_full_fast<bf16_t>(p, call_view(p, blockIdx.y / p.Hkv), smem, blockIdx.y, blockIdx.x - p.Sm);
  else partial_full_rows<bf16_t>(p, smem, blockIdx.x - p.Sm);
}

// ---------------------------------------------------------------------------
// 2d. middle rows, specialised, eight waves: the long series (up to 512 slots) at two waves per SIMD
// ---------------------------------------------------------------------------
// With 512 series slots the table slices of a four-wave workgroup fill its registers (one wave
// per SIMD, nothing to overlap a wait with).  Here eight waves split the harmonics (CW chunks of
// 32 slots each: CW = 2 for 512 slots), so a wave's slices take 64 registers and two waves share
// a SIMD.  A step is still four tiles of 64 rows; of its kept operands a wave takes two row blocks
// of K^mu and one token block of V^mu (tile wave / 2); of the softmax it owns two score columns,
// two rows per lane.  The score exchange is padded so that the eight-byte reads of the owners
// fall in distinct LDS banks.
constexpr int kWaves8 = 8;
constexpr int kBlock8 = 64 * kWaves8;
constexpr int kXs8Q4 = 18;                    // f32x4 cells per (row block, lane / 16): 16 columns + 2 pad cells
constexpr int kXs8Rb = 4 * kXs8Q4;            // per row block
constexpr int kXs8Wave = kRB * kXs8Rb;        // per wave
constexpr unsigned kXs8Bytes = kWaves8 * kXs8Wave * 16;

template <int CW, int DVT, int GP>
__device__ __forceinline__ void partial_middle_fast8(const DecodeParams& p, unsigned char* smem) {
  using T = bf16_t;
  using ES = f16_t;
  constexpr int Mint = kWaves8 * CW * 32;
  constexpr int KT = 4, step = KT * kTJ;
  static_assert(GP == 1 || GP == 4, "score columns per tile");
  static_assert(DVT == 1 || DVT == 2, "kept V column tiles");

  const int sm_idx = blockIdx.x, bh = blockIdx.y, b = bh / p.Hkv, hkv = bh % p.Hkv;
  const int G = p.G;
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int q4 = lane >> 4, r16 = lane & 15;
  const size_t hq0 = static_cast<size_t>(b) * p.Hq + hkv * G;
  // the workgroup's chunk of its head: rows [w0, w1)
  const int Nb = seq_middle_rows(p, b);
  const int w0 = sm_idx * p.chunk_m, w1 = min(Nb, w0 + p.chunk_m);
  const int total = (w1 - w0 + step - 1) / step;
  if (w0 >= Nb) {   // (only with per-sequence counts) nothing of this chunk belongs to the sequence
    write_empty_middle(p, hq0, sm_idx, sm_idx + 1, kBlock8);
    return;
  }
  const int c1 = w1;                                  // rows at or past it are masked (only the last step can hold any)
  const int col_k = r16 / GP, col_h = r16 % GP;
  const bool col_live = col_k < KT && col_h < G;
  const int hsafe = min(col_h, G - 1);
  const int kpitch = (p.Dku + 7) & ~7;
  constexpr int Dkq = 32;
  const int Dvu = p.Dvu;
  const T* kk = static_cast<const T*>(p.k_keep) + bh * p.kk_stride;
  const T* vk = static_cast<const T*>(p.v_keep) + bh * p.vk_stride;
  const int Nm1 = Nb - 1;
  const int my_tile = wave >> 1, my_half = wave & 1;   // kept operands: tile, and which half of it

  // ---- LDS carve-up ----------------------------------------------------------------------------
  f32x4* xs = reinterpret_cast<f32x4*>(smem);                   // [8 waves][4 rb][4][18] partial scores
  ES* pse = reinterpret_cast<ES*>(smem + kXs8Bytes);
  T* pte = reinterpret_cast<T*>(smem + kXs8Bytes + kXN * 16 * 4 * 8 * sizeof(ES));
  T* ptl = reinterpret_cast<T*>(smem + kXs8Bytes + kXN * 16 * 4 * 8 * (sizeof(ES) + sizeof(T)));
  float* alpha_s = reinterpret_cast<float*>(smem + kXs8Bytes + kXN * 16 * 4 * 8 * (sizeof(ES) + 2 * sizeof(T)));
  float* st_m = alpha_s + 16;
  float* st_l = st_m + 16;
  float* red_r = reinterpret_cast<float*>(smem);                // after the loop: [16][Mint + 4]
  constexpr int pr = Mint + 4, po = 16 * DVT + 4;
  float* red_o = red_r + 16 * pr;                               // [8 waves][16][16 DVT + 4]
  constexpr int kPitchG = Mint + 32;
  float* gs_s = reinterpret_cast<float*>(smem + p.lds_tab);
  T* qk_s = reinterpret_cast<T*>(gs_s + G * kPitchG);

  const int urow_lane = 8 * (r16 >> 2) + (r16 & 3);
  const uint32_t kcol = static_cast<uint32_t>(min(8 * q4, kpitch - 8));
  // this wave's kept operands of the step at `base`: row blocks 2 my_half, 2 my_half + 1 and token block
  // my_half of tile my_tile
  auto load_step = [&](Frag<T> (&kf)[2], Frag<T> (&vf)[DVT], int base) {
#pragma unroll
    for (int i = 0; i < 2; ++i) {
      const int rb = 2 * my_half + i;
      const int u = 32 * (rb >> 1) + 4 * (rb & 1) + urow_lane;
      const int j = min(base + my_tile * kTJ + u, Nm1);
      kf[i].load(kk + (static_cast<uint32_t>(j) * static_cast<uint32_t>(kpitch) + kcol));
    }
    const int tok0 = base + my_tile * kTJ + 32 * my_half + 8 * q4;
    const uint32_t g8 = static_cast<uint32_t>(min(tok0, Nm1)) >> 3;
#pragma unroll
    for (int dt = 0; dt < DVT; ++dt) {
      const int dim = min(16 * dt + r16, Dvu - 1);
      vf[dt].load(vk + (g8 * static_cast<uint32_t>(Dvu) + static_cast<uint32_t>(dim)) * 8u);
    }
  };

  // ---- (0) everything that comes from global memory is requested first ------------
  constexpr int kGLoads = (Mint + kBlock8 - 1) / kBlock8;   // G <= 4 heads of Mint floats, as float4
  const int ng4 = G * Mint / 4;
  f32x4 gv[kGLoads];
#pragma unroll
  for (int i = 0; i < kGLoads; ++i)
    gv[i] = *reinterpret_cast<const f32x4*>(p.gs + hq0 * Mint + 4 * min(tid + i * kBlock8, ng4 - 1));
  // this lane's share of the softmax: column ocol, rows 32 x + 8 oq4 + 4 y + 2 ohalf + {0, 1} (orb = 2 x + y)
  const int ocol = 2 * wave + (lane & 1), ohalf = (lane >> 1) & 1, oq4 = (lane >> 2) & 3, orb = lane >> 4;
  const int ocol_k = ocol / GP, ocol_h = ocol % GP;
  const bool olive = ocol_k < KT && ocol_h < G;
  const float g0 = p.g0[hq0 + min(ocol_h, G - 1)];
  Frag<T> qv;
  qv.load(static_cast<const T*>(p.qkeep) + hq0 * Dkq + 8 * min(tid, G * 4 - 1));
  Frag<T> kfA[2], kfB[2];
  Frag<T> vfA[DVT], vfB[DVT];
  load_step(kfA, vfA, w0);
  load_step(kfB, vfB, w0 + min(1, total - 1) * step);

  // ---- this wave's slices of the E table, evaluated in registers -----------------------------
  Frag<ES> eA[CW][kRB], eB[CW][2][kXN];
  float tc[CW], ts[CW];
  {
    const int n_max = p.M / 2;
    const float invT = 1.0f / static_cast<float>(p.T);
    // The wave's accumulators hold the row blocks of a tile in an order of their own: local block l is row
    // block (l + 2 my_half) & 3, so that the two blocks whose kept K rows this wave multiplies are always
    // accumulators 0 and 1 (no branch on the wave's half in the steps).
    float cd[kRB], sd[kRB];
    int urow[kRB];
#pragma unroll
    for (int l = 0; l < kRB; ++l) {
      const int rb = (l + 2 * my_half) & 3;
      urow[l] = 32 * (rb >> 1) + 4 * (rb & 1) + urow_lane;
      table_cs<T>(1, urow[l], p.T, invT, &cd[l], &sd[l]);
    }
#pragma unroll
    for (int i = 0; i < CW; ++i) {
      const int n0 = 16 * (wave * CW + i) + 4 * q4 + 1;
#pragma unroll
      for (int rb = 0; rb < kRB; ++rb) {
        float vals[8];
        table_cs<T>(n0, urow[rb], p.T, invT, &vals[0], &vals[1]);
#pragma unroll
        for (int hp = 1; hp < 4; ++hp) {
          vals[2 * hp] = vals[2 * hp - 2] * cd[rb] - vals[2 * hp - 1] * sd[rb];
          vals[2 * hp + 1] = vals[2 * hp - 1] * cd[rb] + vals[2 * hp - 2] * sd[rb];
        }
#pragma unroll
        for (int hp = 0; hp < 4; ++hp)
          if (n0 + hp > n_max) vals[2 * hp] = vals[2 * hp + 1] = 0.0f;
        pack8(eA[i][rb], vals);
      }
    }
#pragma unroll
    for (int i = 0; i < CW; ++i) {
      const int n = 16 * (wave * CW + i) + r16 + 1;
      float cn, sn;
      table_cs<T>(n, 1, p.T, invT, &cn, &sn);
#pragma unroll
      for (int x = 0; x < kXN; ++x) {
        float cs[8], ss[8];
        table_cs<T>(n, 32 * x + 8 * q4, p.T, invT, &cs[0], &ss[0]);
#pragma unroll
        for (int e = 1; e < 8; ++e) {
          cs[e] = cs[e - 1] * cn - ss[e - 1] * sn;
          ss[e] = ss[e - 1] * cn + cs[e - 1] * sn;
        }
        if (n > n_max) {
#pragma unroll
          for (int e = 0; e < 8; ++e) cs[e] = ss[e] = 0.0f;
        }
        pack8(eB[i][0][x], cs);
        pack8(eB[i][1][x], ss);
      }
    }
    const uint32_t ph_step = phase_of(step, p.ph_scale);
#pragma unroll
    for (int i = 0; i < CW; ++i)
      phase_cs<T>(static_cast<uint32_t>(16 * (wave * CW + i) + r16 + 1) * ph_step, &tc[i], &ts[i]);
  }

  // ---- series coefficients and packed query into LDS ---------------------------------------------
#pragma unroll
  for (int i = 0; i < kGLoads; ++i) {
    const int v4 = tid + i * kBlock8;
    if (v4 < ng4) *reinterpret_cast<f32x4*>(gs_s + (4 * v4 / Mint) * kPitchG + (4 * v4) % Mint) = gv[i];
  }
  if (tid < G * 4) *reinterpret_cast<Frag<T>*>(qk_s + 8 * tid) = qv;
  __syncthreads();
  Frag<T> bq;
  bq.load(qk_s + hsafe * Dkq + 8 * q4);
  if (col_k != my_tile || !col_live) bq.zero();

  // K-side series coefficients of this lane's column (tile, head) and four orders per slice, rotated to
  // the origin of the column's tile in the first step; every later step turns them on by the angle of
  // one step (angle addition, four multiply-adds per order: no table look-up, no evaluation in the loop)
  float gk[CW][8], tkc[CW][4], tks[CW][4];
  {
    const uint32_t ph_k = phase_of(p.t0 + w0 + col_k * kTJ, p.ph_scale);
    const uint32_t ph_step = phase_of(step, p.ph_scale);
#pragma unroll
    for (int i = 0; i < CW; ++i) {
      const uint32_t n0 = 16 * (wave * CW + i) + 4 * q4 + 1;
      const float* gl = gs_s + hsafe * kPitchG + 32 * (wave * CW + i) + 8 * q4;
      const f32x4 ga = *reinterpret_cast<const f32x4*>(gl), gb = *reinterpret_cast<const f32x4*>(gl + 4);
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        float cs, sn;
        phase_cs<T>((n0 + j) * ph_k, &cs, &sn);
        const float gc = (j < 2) ? ga[2 * (j & 1)] : gb[2 * (j & 1)];
        const float gsn = (j < 2) ? ga[2 * (j & 1) + 1] : gb[2 * (j & 1) + 1];
        gk[i][2 * j] = gc * cs + gsn * sn;
        gk[i][2 * j + 1] = gsn * cs - gc * sn;
        phase_cs<T>((n0 + j) * ph_step, &tkc[i][j], &tks[i][j]);
      }
    }
  }

  // where the local row blocks go in the score exchange: blocks 0, 1 are row blocks 2 my_half, 2 my_half + 1
  f32x4* const xw_lo = xs + wave * kXs8Wave + q4 * kXs8Q4 + r16 + 2 * my_half * kXs8Rb;
  f32x4* const xw_hi = xs + wave * kXs8Wave + q4 * kXs8Q4 + r16 + 2 * (1 - my_half) * kXs8Rb;

  f32x4 racc[2 * CW];
  f32x4 oacc[DVT];
  float m_run = -INFINITY, l_run = 0.0f;
#pragma unroll
  for (int t = 0; t < 2 * CW; ++t) racc[t] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
  for (int t = 0; t < DVT; ++t) oacc[t] = f32x4{0.f, 0.f, 0.f, 0.f};

  auto do_step = [&](Frag<T> (&kf)[2], Frag<T> (&vf)[DVT], int base, auto tail_tag) {
    constexpr bool kTail = decltype(tail_tag)::value;
    f32x4 sacc[kRB];
#pragma unroll
    for (int rb = 0; rb < kRB; ++rb) sacc[rb] = f32x4{0.f, 0.f, 0.f, 0.f};

    // -- (a) series on the K side, own orders: S += E g'(tile origin); g' moves on to the next step ---
#pragma unroll
    for (int i = 0; i < CW; ++i) {
      Frag<ES> bg;   // (columns without a query head get some head's values: their scores are never used)
      pack8(bg, gk[i]);
#pragma unroll
      for (int rb = 0; rb < kRB; ++rb) mma_k32(sacc[rb], eA[i][rb], bg);
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        const float gc = gk[i][2 * j], gsn = gk[i][2 * j + 1];
        gk[i][2 * j] = tkc[i][j] * gc + tks[i][j] * gsn;
        gk[i][2 * j + 1] = tkc[i][j] * gsn - tks[i][j] * gc;
      }
    }
    // -- (b) kept K dims: two row blocks of tile my_tile (local blocks 0 and 1) ----------------------
    mma_k32(sacc[0], kf[0], bq);
    mma_k32(sacc[1], kf[1], bq);

    // -- (c) the partial scores of the eight waves meet; this wave sums its two columns --------
    xw_lo[0] = sacc[0];
    xw_lo[kXs8Rb] = sacc[1];
    xw_hi[0] = sacc[2];
    xw_hi[kXs8Rb] = sacc[3];
    __syncthreads();
    f32x2 sv;
    {
      const f32x2* xr = reinterpret_cast<const f32x2*>(xs + orb * kXs8Rb + oq4 * kXs8Q4 + ocol) + ohalf;
      f32x2 a0 = xr[0 * 2 * kXs8Wave] + xr[1 * 2 * kXs8Wave], a1 = xr[2 * 2 * kXs8Wave] + xr[3 * 2 * kXs8Wave];
      f32x2 a2 = xr[4 * 2 * kXs8Wave] + xr[5 * 2 * kXs8Wave], a3 = xr[6 * 2 * kXs8Wave] + xr[7 * 2 * kXs8Wave];
      sv = (a0 + a1) + (a2 + a3);
    }
    // -- (d) online softmax of the own columns -----------------------------------------------------
    // The reference m_run of a column only has to keep exp(score - m_run) inside the range of the
    // 16-bit probabilities, not to be the maximum: it moves when a score of one of the wave's columns
    // exceeds it by more than kSoftmaxSlack (always in a chunk's first step), and only then is there a
    // maximum to reduce and a factor to apply.
    float pv[2];
    float m_tile = -INFINITY;
#pragma unroll
    for (int v = 0; v < 2; ++v) {
      float sc = (sv[v] + g0) * p.scale;
      if constexpr (kTail) {
        const int u = 32 * (orb >> 1) + 8 * oq4 + 4 * (orb & 1) + 2 * ohalf + v;
        if (base + ocol_k * kTJ + u >= c1) sc = -INFINITY;
      }
      if (!olive) sc = -INFINITY;
      pv[v] = sc;
      m_tile = fmaxf(m_tile, sc);
    }
    float alpha = 1.0f;
    if (__builtin_amdgcn_ballot_w64(m_tile > m_run + kSoftmaxSlack) != 0) {   // (uniform over the wave)
      m_tile = row_stride_max(m_tile, 2);                    // the 32 lanes of a column are 2 apart
      m_tile = cross_row_max(m_tile);
      const float m_new = fmaxf(m_run, m_tile);
      alpha = __expf(m_run - ((m_new == -INFINITY) ? 0.0f : m_new));
      m_run = m_new;
    }
    const float m_ref = (m_run == -INFINITY) ? 0.0f : m_run;
    pv[0] = __expf(pv[0] - m_ref);
    pv[1] = __expf(pv[1] - m_ref);
    l_run = l_run * alpha + (pv[0] + pv[1]);
    {
      const int slot = (((orb >> 1) * 16 + ocol) * 4 + oq4) * 8 + 4 * (orb & 1) + 2 * ohalf;
      uint32_t w = __builtin_bit_cast(uint32_t, __builtin_convertvector(f32x2{pv[0], pv[1]}, f16x2));
      *reinterpret_cast<uint32_t*>(reinterpret_cast<uint16_t*>(pse) + slot) = w;
      w = __builtin_bit_cast(uint32_t, __builtin_convertvector(f32x2{pv[0], pv[1]}, bf16x2));
      *reinterpret_cast<uint32_t*>(reinterpret_cast<uint16_t*>(pte) + slot) = w;
      const float lo0 = pv[0] - __builtin_bit_cast(float, (w & 0xffffu) << 16);
      const float lo1 = pv[1] - __builtin_bit_cast(float, w & 0xffff0000u);
      w = __builtin_bit_cast(uint32_t, __builtin_convertvector(f32x2{lo0, lo1}, bf16x2));
      *reinterpret_cast<uint32_t*>(reinterpret_cast<uint16_t*>(ptl) + slot) = w;
      if (lane < 2) alpha_s[ocol] = alpha;
    }
    __syncthreads();
    // -- (e) bring the accumulators into this step's frame ------------------------------------------
    {
      const f32x4 al = *reinterpret_cast<const f32x4*>(alpha_s + 4 * q4);
      const bool moved = al[0] != 1.0f || al[1] != 1.0f || al[2] != 1.0f || al[3] != 1.0f;
      if (__builtin_amdgcn_ballot_w64(moved) != 0) {   // some column's reference moved: factors to apply
#pragma unroll
        for (int t = 0; t < DVT; ++t)
#pragma unroll
          for (int v = 0; v < 4; ++v) oacc[t][v] *= al[v];
#pragma unroll
        for (int i = 0; i < CW; ++i)
#pragma unroll
          for (int v = 0; v < 4; ++v) {
            racc[2 * i][v] *= al[v];
            racc[2 * i + 1][v] *= al[v];
          }
      }
#pragma unroll
      for (int i = 0; i < CW; ++i)
#pragma unroll
        for (int v = 0; v < 4; ++v) {
          const float rc = racc[2 * i][v], rs = racc[2 * i + 1][v];
          racc[2 * i][v] = tc[i] * rc + ts[i] * rs;
          racc[2 * i + 1][v] = tc[i] * rs - ts[i] * rc;
        }
    }
    // -- (f) V side, own orders: r' += P^T E ----------------------------------------------------------
#pragma unroll
    for (int x = 0; x < kXN; ++x) {
      Frag<ES> ps;
      ps.load(pse + ((x * 16 + r16) * 4 + q4) * 8);
#pragma unroll
      for (int i = 0; i < CW; ++i) {
        mma_k32(racc[2 * i], ps, eB[i][0][x]);
        mma_k32(racc[2 * i + 1], ps, eB[i][1][x]);
      }
    }
    // -- (g) kept V dims: token block my_half of tile my_tile -----------------------------------------
    {
      Frag<T> pt, pl;
      pt.load(pte + ((my_half * 16 + r16) * 4 + q4) * 8);
      pl.load(ptl + ((my_half * 16 + r16) * 4 + q4) * 8);
      if (col_k != my_tile) {
        pt.zero();
        pl.zero();
      }
#pragma unroll
      for (int dt = 0; dt < DVT; ++dt) {
        Frag<T> bv = vf[dt];
        if ((Dvu & 15) != 0 && 16 * dt + r16 >= Dvu) bv.zero();
        if constexpr (kTail) {
          const int tok0 = base + my_tile * kTJ + 32 * my_half + 8 * q4;
          if (tok0 + 8 > c1) mask_tail(bv, c1 - tok0);
        }
        mma_k32(oacc[dt], pt, bv);
        mma_k32(oacc[dt], pl, bv);
      }
    }
  };

  // the chunk's record from the accumulators: its last step started at last_base
  auto finish_chunk = [&](int chunk, int last_base) {
    // ---- merge the tiles of a head --------------------------------------------------------------
    float l_tot = row_stride_sum(l_run, 2);
    l_tot = cross_row_sum(l_tot);
    if (lane < 2) {
      st_m[ocol] = m_run;
      st_l[ocol] = l_tot;
    }
    __syncthreads();
    const float mc = col_live ? st_m[r16] : -INFINITY;
    const float lcol = st_l[r16];
    const float mstar = row_stride_max(mc, GP);
    const float fc = (mc != -INFINITY) ? __expf(mc - mstar) : 0.0f;
    const float lstar = row_stride_sum(col_live ? lcol * fc : 0.0f, GP);
    __syncthreads();

    {
      float f[4];
      uint32_t phr[4];
#pragma unroll
      for (int v = 0; v < 4; ++v) {
        const int row = 4 * q4 + v;
        f[v] = __shfl(fc, row, kWave);
        phr[v] = phase_of(p.t0 + last_base + (row / GP) * kTJ, p.ph_scale);
      }
#pragma unroll
      for (int i = 0; i < CW; ++i) {
        const int c = wave * CW + i;
        const uint32_t n = 16 * c + r16 + 1;
        float cs[4], sn[4];
        phase_cs<T>(n * phr[0], &cs[0], &sn[0]);
        if constexpr (GP >= 4) {
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
          const float rc = racc[2 * i][v], rs = racc[2 * i + 1][v];
          float* dst = red_r + (4 * q4 + v) * pr + 32 * c + r16;
          dst[0] = f[v] * (cs[v] * rc - sn[v] * rs);
          dst[16] = f[v] * (sn[v] * rc + cs[v] * rs);
        }
      }
      float* ro = red_o + wave * 16 * po;
#pragma unroll
      for (int dt = 0; dt < DVT; ++dt)
#pragma unroll
        for (int v = 0; v < 4; ++v) ro[(4 * q4 + v) * po + 16 * dt + r16] = f[v] * oacc[dt][v];
    }
    __syncthreads();

    const size_t rec_h = static_cast<size_t>(p.Sm) * p.recm;
    float* rec0 = p.part_m + (hq0 * p.Sm + chunk) * p.recm;
    if (wave == 0 && lane < G) {
      rec0[lane * rec_h + 0] = mstar;
      rec0[lane * rec_h + 1] = lstar;
    }
    constexpr int no4 = 4 * DVT, nr4 = Mint / 4, per = no4 + nr4;
    for (int it = tid; it < G * per; it += kBlock8) {
      const int h = it / per, x4 = it - h * per;
      f32x4 v = {0.f, 0.f, 0.f, 0.f};
      if (x4 < no4) {
        // kept dims of tile k were accumulated by waves 2 k and 2 k + 1
#pragma unroll
        for (int k = 0; k < KT; ++k) {
          v += *reinterpret_cast<const f32x4*>(red_o + (((2 * k) * 16 + k * GP + h) * po + 4 * x4));
          v += *reinterpret_cast<const f32x4*>(red_o + (((2 * k + 1) * 16 + k * GP + h) * po + 4 * x4));
        }
      } else {
        const int y = x4 - no4;
#pragma unroll
        for (int k = 0; k < KT; ++k) v += *reinterpret_cast<const f32x4*>(red_r + ((k * GP + h) * pr + 4 * y));
      }
      *reinterpret_cast<f32x4*>(rec0 + h * rec_h + 4 + 4 * x4) = v;
    }
  };

  const int wlast = w0 + (total - 1) * step;            // first row of the workgroup's last step
  {
    int s = 0;
    for (; s + 2 < total; s += 2) {
      const int base = w0 + s * step;
      do_step(kfA, vfA, base, std::false_type{});
      load_step(kfA, vfA, min(base + 2 * step, wlast));
      do_step(kfB, vfB, base + step, std::false_type{});
      load_step(kfB, vfB, min(base + 3 * step, wlast));
    }
    const int base = w0 + s * step;
    if (total - s == 2) {
      do_step(kfA, vfA, base, std::false_type{});
      do_step(kfB, vfB, base + step, std::true_type{});
    } else {
      do_step(kfA, vfA, base, std::true_type{});
    }
    finish_chunk(sm_idx, wlast);
  }
}

template <int CW, int DVT, int GP>
__global__ __launch_bounds__(kBlock8, 1) void decode_partial_fast8(DecodeParams p) {
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  if (static_cast<int>(blockIdx.x) < p.Sm) {
    partial_middle_fast8<CW, DVT, GP>(p, smem);
  } else {
    if (threadIdx.x >= kBlock) return;   // the full-row path is written for four waves; the others leave before any barrier
    if (p.D == 128) partial_full_fast<bf16_t>(p, call_view(p, blockIdx.y / p.Hkv), smem, blockIdx.y, blockIdx.x - p.Sm);
    else partial_full_rows<bf16_t>(p, smem, blockIdx.x - p.Sm);
  }
}

template <typename T, int CW, int DVTM, bool KC1>
__global__ __launch_bounds__(kBlock, (CW <= 2 && sizeof(T) == 2) ? 2 : 1) void decode_partial(DecodeParams p) {
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  if (static_cast<int>(blockIdx.x) < p.Sm) partial_middle_rows<T, CW, DVTM, KC1>(p, smem);
  else partial_full_rows<T>(p, smem, blockIdx.x - p.Sm);
}

// ---------------------------------------------------------------------------
// 3. merge partials, apply diag(w) C_v, normalise
// ---------------------------------------------------------------------------
// A query head is shared by ceil(D / 32) workgroups, one per slice of 32 output
// dims.  Every slice merges the statistics and the series sums r of the head's
// records (replicated work, a few tens of KB), then finishes its own dims: kept
// dims from the accumulators, compressed dims from r and its columns of C_v.
// Nothing is exchanged between workgroups.
// kFinDims: output dims per workgroup.  Every workgroup of a head re-reads the head's statistics and
// series sums, so few wide slices read less and many narrow slices fill the chip sooner: 32 dims
// when there are few query heads, 64 once the heads alone give enough workgroups.
template <typename T, int kFinDims>
__global__ __launch_bounds__(kFinBlock) void decode_finish(DecodeParams p) {
  constexpr int kNW = kFinBlock / 64;
  constexpr int kSP = kMaxPartials / kFinBlock;   // records per thread when reading statistics
  constexpr int kCG = kFinBlock / kFinDims;       // row / record groups of the per-dim passes
  __shared__ float es[kMaxPartials];              // e^{m_s - m} per record
  __shared__ f32x4 red4[kFinBlock];
  __shared__ float rr[FA_MAX_DECODE_STATES];      // r in basis order, weighted
  __shared__ f32x4 redw4[kFinBlock];
  __shared__ float redc[kFinBlock];
  __shared__ float outw[kFinDims];
  __shared__ float wmax[kNW], wsum[kNW], wsum_m[kNW];

  const int sl = blockIdx.x, hq = blockIdx.y;
  const int b = hq / p.Hq, hkv = (hq % p.Hq) / p.G, bh = b * p.Hkv + hkv;
  const int D = p.D, M = p.M, Sm = p.Sm, Sw = p.Sw, S = Sm + Sw, Dvc = p.Dvc;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int Dva = 16 * ((p.Dvu + 15) / 16);
  const int recm = p.recm, recw = p.recw;
  const float* pm = p.part_m + static_cast<size_t>(hq) * Sm * recm;
  const float* pw = p.part_w + static_cast<size_t>(hq) * Sw * recw;
  const bool do_cv = Sm > 0 && Dvc > 0;
  const int d0 = kFinDims * sl;

  // ---- global operands, in the order they are needed -----------------------------------------
  // (0) the mask row: it decides which columns of C_v and of the accumulators this slice reads
  uint8_t vmb[4];
#pragma unroll
  for (int i = 0; i < 4; ++i) vmb[i] = p.vmask[static_cast<size_t>(bh) * D + min(lane + 64 * i, D - 1)];
  // (1) chunk maxima and sums
  float ms[kSP], ls[kSP];
#pragma unroll
  for (int i = 0; i < kSP; ++i) {
    const int s = min(tid + i * kFinBlock, S - 1);
    const float* r = (s < Sm) ? pm + static_cast<size_t>(s) * recm : pw + static_cast<size_t>(s - Sm) * recw;
    ms[i] = r[0];
    ls[i] = r[1];
  }
  // (2) series sums of the middle records: thread (4 columns, group of records)
  const int cr4 = p.Mint / 4, ngr = kFinBlock / cr4;
  const int c4r = tid % cr4, gr = tid / cr4;
  const float* pr = pm + 4 + Dva + 4 * c4r;
  constexpr int kUr = 12;
  f32x4 rv[kUr];
  if (do_cv) {
#pragma unroll
    for (int u = 0; u < kUr; ++u)   // lanes are clamped, never predicated (a predicated load is waited for
      if (u * ngr < Sm)             // at once); rounds no lane needs are skipped by the whole workgroup
        rv[u] = *reinterpret_cast<const f32x4*>(pr + static_cast<size_t>(min(gr + u * ngr, Sm - 1)) * recm);
  }
  // (3) this slice's columns of the full-row records: thread (4 columns, group of records)
  constexpr int kW4 = kFinDims / 4, kWG = kFinBlock / kW4;
  const int c4w = tid % kW4, gw = tid / kW4;
  const bool w_ok = d0 + 4 * c4w < D;
  const int dw = min(d0 + 4 * c4w, D - 4);
  constexpr int kUw = 2;
  f32x4 wv[kUw];
  if (Sw > 0) {
#pragma unroll
    for (int u = 0; u < kUw; ++u)
      if (u * kWG < Sw)
        wv[u] = *reinterpret_cast<const f32x4*>(pw + static_cast<size_t>(min(gw + u * kWG, Sw - 1)) * recw + 4 + dw);
  }
  // ranks of this slice's dims (needs only the mask)
  uint64_t vbal[4];
#pragma unroll
  for (int i = 0; i < 4; ++i) vbal[i] = __ballot(vmb[i] != 0 && lane + 64 * i < D);
  const int col = tid % kFinDims, cg = tid / kFinDims;
  const int dme = d0 + col;
  const int rk = (dme < D) ? dim_rank(vbal, dme) : 0;
  const bool is_c = dme < D && rk < 0, is_k = dme < D && rk >= 0;
  // (4) C_v.  The compressed dims of a slice have consecutive ranks r0 .. r0 + nc - 1, i.e. the slice
  // needs a contiguous band of C_v's columns.  With Dvc a multiple of 4 the band is read as 128-bit
  // vectors: thread (column quad cq, row group rg) takes rows rg, rg + ngrp, ...  Otherwise every
  // thread reads its own dim's column element by element (rows cg, cg + kCG, ...).
  constexpr int kUc = 64, kUk = 6, kUv = 16;
  const bool vec_cv = do_cv && (Dvc & 3) == 0;
  int r0 = 0, nc = 0;
  {
    const int w0 = d0 >> 6, sh = d0 & 63;   // kFinDims divides 64: the slice lies inside one ballot word
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      if (j < w0) r0 += __popcll(vbal[j]);
      if (j == w0) {
        r0 += __popcll(vbal[j] & ((1ull << sh) - 1ull));
        nc = __popcll((vbal[j] >> sh) & (kFinDims == 64 ? ~0ull : ((1ull << kFinDims) - 1ull)));
      }
    }
  }
  const int q0 = r0 >> 2, nq = nc > 0 ? ((r0 + nc + 3) >> 2) - q0 : 1;   // column quads of the band
  const int ngrp = kFinBlock / nq;                                       // row groups
  const int rgv = tid / nq, cqv = tid - rgv * nq;
  const float* cvb = p.cv + static_cast<size_t>(bh) * M * Dvc;
  const float* cvc = cvb + (is_c ? -rk - 1 : 0);
  float cvv[kUc];
  f32x4 cv4[kUv];
  if (vec_cv) {
    const float* cq_ptr = cvb + 4 * min(q0 + cqv, Dvc / 4 - 1);
#pragma unroll
    for (int u = 0; u < kUv; ++u)
      if (u * ngrp < M) cv4[u] = *reinterpret_cast<const f32x4*>(cq_ptr + static_cast<size_t>(min(rgv + u * ngrp, M - 1)) * Dvc);
  } else if (do_cv) {
#pragma unroll
    for (int u = 0; u < kUc; ++u)
      if (u * kCG < M) cvv[u] = cvc[static_cast<size_t>(min(cg + u * kCG, M - 1)) * Dvc];
  }
  const float* pk = pm + 4 + (is_k ? rk : 0);
  float kv[kUk];
  if (Sm > 0) {
#pragma unroll
    for (int u = 0; u < kUk; ++u)
      if (u * kCG < Sm) kv[u] = pk[static_cast<size_t>(min(cg + u * kCG, Sm - 1)) * recm];
  }

  // ---- global max, per-record factors, normaliser ---------------------------------------------
  float m = -INFINITY;
#pragma unroll
  for (int i = 0; i < kSP; ++i)
    if (tid + i * kFinBlock < S) m = fmaxf(m, ms[i]);
  m = wave_max_fast(m);
  if (lane == 0) wmax[wave] = m;
  __syncthreads();
  m = wmax[0];
#pragma unroll
  for (int w = 1; w < kNW; ++w) m = fmaxf(m, wmax[w]);
  float l = 0.0f, lm = 0.0f;
#pragma unroll
  for (int i = 0; i < kSP; ++i) {
    const int s = tid + i * kFinBlock;
    if (s < S) {
      const float e = (ms[i] == -INFINITY) ? 0.0f : __expf(ms[i] - m);
      es[s] = e;
      l += e * ls[i];
      if (s < Sm) lm += e * ls[i];   // the middle rows' share: r of the constant basis function
    }
  }
  l = wave_sum_fast(l);
  lm = wave_sum_fast(lm);
  if (lane == 0) {
    wsum[wave] = l;
    wsum_m[wave] = lm;
  }
  __syncthreads();
  float L = 0.0f, Lm = 0.0f;
#pragma unroll
  for (int w = 0; w < kNW; ++w) {
    L += wsum[w];
    Lm += wsum_m[w];
  }

  // ---- r in basis order, weighted by the inverse squared norms ---------------------------------
  if (do_cv) {
    f32x4 a = {0.f, 0.f, 0.f, 0.f};
    if (gr < ngr) {
#pragma unroll
      for (int u = 0; u < kUr; ++u) {
        const int s = gr + u * ngr;
        if (s < Sm) a += es[s] * rv[u];
      }
      for (int s = gr + kUr * ngr; s < Sm; s += ngr)
        a += es[s] * *reinterpret_cast<const f32x4*>(pr + static_cast<size_t>(s) * recm);
    }
    red4[tid] = a;
  }
  // this slice's full-row columns
  {
    f32x4 c = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int u = 0; u < kUw; ++u) {
      const int s = gw + u * kWG;
      if (s < Sw && w_ok) c += es[Sm + s] * wv[u];
    }
    if (w_ok)
      for (int s = gw + kUw * kWG; s < Sw; s += kWG)
        c += es[Sm + s] * *reinterpret_cast<const f32x4*>(pw + static_cast<size_t>(s) * recw + 4 + dw);
    redw4[tid] = c;   // [record group][column quad]
  }
  __syncthreads();
  if (tid < kFinDims) {
    const float* src = reinterpret_cast<const float*>(redw4) + tid;
    float v = 0.0f;
#pragma unroll
    for (int g = 0; g < kWG; ++g) v += src[g * kFinDims];
    outw[tid] = v;
  }
  if (do_cv) {
    for (int ig = tid; ig < p.Mint; ig += kFinBlock) {   // record order: 32 * chunk + 16 * (cos | sin) + order
      const float* src = reinterpret_cast<const float*>(red4) + ig;
      float v = 0.0f;
      for (int g = 0; g < ngr; ++g) v += src[g * p.Mint];
      const int n = 16 * (ig >> 5) + (ig & 15) + 1, cs = (ig >> 4) & 1;
      const int mm = 2 * n - 1 + cs;
      if (mm < M) rr[mm] = v * basis_weight(n, p.T);
    }
    if (tid == kFinBlock - 1) rr[0] = Lm * basis_weight(0, p.T);   // constant function: sum of p over the middle rows
  }
  __syncthreads();

  // ---- per dim: sum_m rr[m] C_v[m, i] (compressed) or the merged accumulator (kept) ------------
  if (vec_cv) {   // band of C_v: partial sums per (row group, column quad); red4 is free again
    f32x4 o4 = {0.f, 0.f, 0.f, 0.f};
    if (rgv < ngrp) {
#pragma unroll
      for (int u = 0; u < kUv; ++u) {
        const int mm = rgv + u * ngrp;
        if (mm < M) o4 += rr[mm] * cv4[u];
      }
      const float* cq_ptr = cvb + 4 * min(q0 + cqv, Dvc / 4 - 1);
      for (int mm = rgv + kUv * ngrp; mm < M; mm += ngrp)
        o4 += rr[mm] * *reinterpret_cast<const f32x4*>(cq_ptr + static_cast<size_t>(mm) * Dvc);
    }
    red4[tid] = o4;
  }
  {
    float o = 0.0f;
    if (do_cv && is_c && !vec_cv) {
#pragma unroll
      for (int u = 0; u < kUc; ++u) {
        const int mm = cg + u * kCG;
        if (mm < M) o += rr[mm] * cvv[u];
      }
      for (int mm = cg + kUc * kCG; mm < M; mm += kCG) o += rr[mm] * cvc[static_cast<size_t>(mm) * Dvc];
    }
    if (is_k && Sm > 0) {
#pragma unroll
      for (int u = 0; u < kUk; ++u) {
        const int s = cg + u * kCG;
        if (s < Sm) o += es[s] * kv[u];
      }
      for (int s = cg + kUk * kCG; s < Sm; s += kCG) o += es[s] * pk[static_cast<size_t>(s) * recm];
    }
    redc[tid] = o;
  }
  __syncthreads();
  if (tid < kFinDims && d0 + tid < D) {
    float v = outw[tid];
#pragma unroll
    for (int g = 0; g < kCG; ++g) v += redc[g * kFinDims + tid];
    if (vec_cv && is_c) {   // (tid < kFinDims: col == tid, so rk is this dim's rank)
      const int c = (-rk - 1) - 4 * q0;
      const float* src = reinterpret_cast<const float*>(red4) + 4 * (c >> 2) + (c & 3);
      for (int g = 0; g < ngrp; ++g) v += src[4 * g * nq];
    }
    p.out[static_cast<size_t>(hq) * D + d0 + tid] = L > 0.0f ? v / L : 0.0f;   // (a sequence without rows)
  }
}

// ---------------------------------------------------------------------------
// 3b. merge partials, apply diag(w) C_v, normalise: the pipelined form
// ---------------------------------------------------------------------------
// Same arithmetic as decode_finish, organised so that a workgroup's large reads depend on
// nothing but the kernel arguments: a query head is shared by NS workgroups that divide the
// output dims by RANK (compressed dims cb0 .. cb0 + cbw - 1 and kept dims kb0 .. kb0 + kbw - 1 in
// mask order) instead of by position, so the band of C_v columns and the kept-dim columns of the
// records are known before the mask row arrives; only the few full-row records are read after
// it.  Every load is issued in batches of independent requests (no load waits for another one's
// data), and the workgroups of one KV head are numbered so that they run on one XCD and share
// its L2 (workgroup ids go round the eight XCDs).  Needs Dvc to be a multiple of 4.
constexpr int kFin2Batch = 4;    // independent requests per batch: narrow columns (kept dims, full-row records)
// kFin2Wide: independent 128-bit requests per batch of the series sums and of the C_v band: 16 when a
// launch has few workgroups (long record lists, registers to spare), 8 with four workgroups per unit
template <int kFin2Wide>
__device__ __forceinline__ void finish2_slice(const DecodeParams& p, const SeqView& sv, const int NS, const int bh,
                                              const int g, const int sl) {
  constexpr int kNW = kFinBlock / 64;
  constexpr int kSP = kMaxPartials / kFinBlock;
  __shared__ float es[kMaxPartials];
  __shared__ f32x4 red4[kFinBlock];                 // series sums per record group, then C_v partial sums per row group
  __shared__ float redk[2 * kFinBlock];             // kept-dim and full-row partial sums per record group
  __shared__ float rr[FA_MAX_DECODE_STATES + 4];
  __shared__ int dim_of[FA_MAX_HEAD_DIM];           // output dim of each rank of this slice
  __shared__ float wmax[kNW], wsum[kNW], wsum_m[kNW];

  const int b = bh / p.Hkv, hkv = bh % p.Hkv;
  const int hq = b * p.Hq + hkv * p.G + g;

  const int D = p.D, M = p.M, Sm = sv.Sm, Sw = sv.Sw, S = Sm + Sw, Dvc = p.Dvc, Dvu = p.Dvu, Mint = p.Mint;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int Dva = 16 * ((Dvu + 15) / 16);
  const int recm = p.recm, recw = p.recw;
  const float* pm = sv.part_m + static_cast<size_t>(hq) * Sm * recm;
  const float* pw = sv.part_w + static_cast<size_t>(hq) * Sw * recw;
  const bool do_cv = Sm > 0 && Dvc > 0;
  // this slice's ranks
  const int cbw = (((Dvc + NS - 1) / NS) + 3) & ~3, cb0 = sl * cbw, cbn = max(0, min(cbw, Dvc - cb0));
  const int kbw = (Dvu + NS - 1) / NS, kb0 = sl * kbw, kbn = max(0, min(kbw, Dvu - kb0));

  // ---- loads that depend on nothing ------------------------------------------------------------
  uint8_t vmb[4];
#pragma unroll
  for (int i = 0; i < 4; ++i) vmb[i] = p.vmask[static_cast<size_t>(bh) * D + min(lane + 64 * i, D - 1)];
  float ms[kSP], ls[kSP];
#pragma unroll
  for (int i = 0; i < kSP; ++i) {
    if (i * kFinBlock < S) {
      const int s = min(tid + i * kFinBlock, S - 1);
      const float* r = (s < Sm) ? pm + static_cast<size_t>(s) * recm : pw + static_cast<size_t>(s - Sm) * recw;
      ms[i] = r[0];
      ls[i] = r[1];
    }
  }
  // first batch of the series sums: thread (4 slots c4r, record group gr)
  const int cr4 = Mint / 4, ngr = max(kFinBlock / cr4, 1);
  const int c4r = tid % cr4, gr = tid / cr4;
  const bool r_on = do_cv && tid < cr4 * ngr;
  const float* pr = pm + 4 + Dva + 4 * c4r;
  f32x4 rv[kFin2Wide];
  if (do_cv) {
#pragma unroll
    for (int u = 0; u < kFin2Wide; ++u)
      if (u * ngr < Sm) rv[u] = *reinterpret_cast<const f32x4*>(pr + static_cast<size_t>(min(gr + u * ngr, Sm - 1)) * recm);
  }
  // first batch of the C_v band: thread (column quad cqv, row group rgv)
  const int nq = max(cbn / 4, 1), ngrp = kFinBlock / nq;
  const int cqv = tid % nq, rgv = tid / nq;
  const bool cv_on = do_cv && cbn > 0 && tid < nq * ngrp;
  const float* cvb = p.cv + static_cast<size_t>(bh) * M * Dvc + cb0 + 4 * cqv;
  f32x4 cv4[kFin2Wide];
  if (do_cv && cbn > 0) {
#pragma unroll
    for (int u = 0; u < kFin2Wide; ++u)
      if (u * ngrp < M) cv4[u] = *reinterpret_cast<const f32x4*>(cvb + static_cast<size_t>(min(rgv + u * ngrp, M - 1)) * Dvc);
  }
  // kept-dim accumulators of the middle records: thread (kept rank kc, record group kg)
  const int kcn = max(kbn, 1), nkg = kFinBlock / kcn;
  const int kc = tid % kcn, kg = tid / kcn;
  const bool k_on = Sm > 0 && kbn > 0 && tid < kcn * nkg;
  const float* pk = pm + 4 + kb0 + kc;
  float kv[kFin2Batch];
  if (Sm > 0 && kbn > 0) {
#pragma unroll
    for (int u = 0; u < kFin2Batch; ++u)
      if (u * nkg < Sm) kv[u] = pk[static_cast<size_t>(min(kg + u * nkg, Sm - 1)) * recm];
  }

  // ---- which dims this slice writes (needs the mask row) ---------------------------------------
  uint64_t vbal[4];
#pragma unroll
  for (int i = 0; i < 4; ++i) vbal[i] = __ballot(vmb[i] != 0 && lane + 64 * i < D);
  if (tid < D) {
    const int rk = dim_rank(vbal, tid);
    if (rk < 0) {
      const int c = -rk - 1 - cb0;
      if (c >= 0 && c < cbn) dim_of[c] = tid;
    } else {
      const int k = rk - kb0;
      if (k >= 0 && k < kbn) dim_of[cbw + k] = tid;
    }
  }

  // ---- global max, per-record factors, normaliser ---------------------------------------------
  float m = -INFINITY;
#pragma unroll
  for (int i = 0; i < kSP; ++i)
    if (tid + i * kFinBlock < S) m = fmaxf(m, ms[i]);
  m = wave_max_fast(m);
  if (lane == 0) wmax[wave] = m;
  __syncthreads();   // also publishes dim_of
  m = wmax[0];
#pragma unroll
  for (int w = 1; w < kNW; ++w) m = fmaxf(m, wmax[w]);
  float l = 0.0f, lm = 0.0f;
#pragma unroll
  for (int i = 0; i < kSP; ++i) {
    const int s = tid + i * kFinBlock;
    if (s < S) {
      const float e = (ms[i] == -INFINITY) ? 0.0f : __expf(ms[i] - m);
      es[s] = e;
      l += e * ls[i];
      if (s < Sm) lm += e * ls[i];
    }
  }
  // the full-row records at this slice's dims: thread (rank j of the slice, record group)
  const int nj = cbw + kbw, njn = max(nj, 1), nwg = kFinBlock / njn;
  const int wj = tid % njn, wg = tid / njn;
  const bool wj_live = (wj < cbn) || (wj >= cbw && wj < cbw + kbn);
  const bool w_on = Sw > 0 && nj > 0 && tid < njn * nwg && wj_live;
  const int wdim = wj_live && nj > 0 ? dim_of[wj] : 0;
  float wv[kFin2Batch];
  if (Sw > 0) {
#pragma unroll
    for (int u = 0; u < kFin2Batch; ++u)
      if (u * nwg < Sw) wv[u] = pw[static_cast<size_t>(min(wg + u * nwg, Sw - 1)) * recw + 4 + wdim];
  }
  l = wave_sum_fast(l);
  lm = wave_sum_fast(lm);
  if (lane == 0) {
    wsum[wave] = l;
    wsum_m[wave] = lm;
  }
  __syncthreads();
  float Lsum = 0.0f, Lm = 0.0f;
#pragma unroll
  for (int w = 0; w < kNW; ++w) {
    Lsum += wsum[w];
    Lm += wsum_m[w];
  }

  // ---- kept dims of the slice and the full-row records: per-thread partial sums ------------------
  {
    float o = 0.0f;
    if (k_on) {
#pragma unroll
      for (int u = 0; u < kFin2Batch; ++u) {
        const int s = kg + u * nkg;
        if (s < Sm) o += es[s] * kv[u];
      }
      for (int s = kg + kFin2Batch * nkg; s < Sm; s += nkg) o += es[s] * pk[static_cast<size_t>(s) * recm];
    }
    redk[tid] = o;
    float ow = 0.0f;
    if (w_on) {
#pragma unroll
      for (int u = 0; u < kFin2Batch; ++u) {
        const int s = wg + u * nwg;
        if (s < Sw) ow += es[Sm + s] * wv[u];
      }
      for (int s = wg + kFin2Batch * nwg; s < Sw; s += nwg) ow += es[Sm + s] * pw[static_cast<size_t>(s) * recw + 4 + wdim];
    }
    redk[kFinBlock + tid] = ow;
  }
  // ---- r in basis order, weighted by the inverse squared norms ---------------------------------
  if (do_cv) {
    f32x4 a = {0.f, 0.f, 0.f, 0.f};
    if (r_on) {
#pragma unroll
      for (int u = 0; u < kFin2Wide; ++u) {
        const int s = gr + u * ngr;
        if (s < Sm) a += es[s] * rv[u];
      }
      for (int s0 = kFin2Wide * ngr; s0 < Sm; s0 += kFin2Wide * ngr) {   // further batches: requests first, sums after
        f32x4 t[kFin2Wide];
#pragma unroll
        for (int u = 0; u < kFin2Wide; ++u)
          t[u] = *reinterpret_cast<const f32x4*>(pr + static_cast<size_t>(min(s0 + gr + u * ngr, Sm - 1)) * recm);
#pragma unroll
        for (int u = 0; u < kFin2Wide; ++u) {
          const int s = s0 + gr + u * ngr;
          if (s < Sm) a += es[s] * t[u];
        }
      }
    }
    red4[tid] = a;
  }
  __syncthreads();
  if (do_cv) {
    for (int ig = tid; ig < Mint; ig += kFinBlock) {   // record order: 32 * chunk + 16 * (cos | sin) + order
      const float* src = reinterpret_cast<const float*>(red4) + ig;
      float v = 0.0f;
      for (int gi = 0; gi < ngr; ++gi) v += src[gi * Mint];
      const int n = 16 * (ig >> 5) + (ig & 15) + 1, cs = (ig >> 4) & 1;
      const int mm = 2 * n - 1 + cs;
      if (mm < M) rr[mm] = v * basis_weight(n, p.T);
    }
    if (tid == kFinBlock - 1) rr[0] = Lm * basis_weight(0, p.T);
  }
  __syncthreads();

  // ---- compressed dims of the slice: sum_m rr[m] C_v[m, rank] -----------------------------------
  {
    f32x4 o4 = {0.f, 0.f, 0.f, 0.f};
    if (cv_on) {
#pragma unroll
      for (int u = 0; u < kFin2Wide; ++u) {
        const int mm = rgv + u * ngrp;
        if (mm < M) o4 += rr[mm] * cv4[u];
      }
      for (int m0 = kFin2Wide * ngrp; m0 < M; m0 += kFin2Wide * ngrp) {
        f32x4 t[kFin2Wide];
#pragma unroll
        for (int u = 0; u < kFin2Wide; ++u)
          t[u] = *reinterpret_cast<const f32x4*>(cvb + static_cast<size_t>(min(m0 + rgv + u * ngrp, M - 1)) * Dvc);
#pragma unroll
        for (int u = 0; u < kFin2Wide; ++u) {
          const int mm = m0 + rgv + u * ngrp;
          if (mm < M) o4 += rr[mm] * t[u];
        }
      }
    }
    red4[tid] = o4;   // [row group][column quad]
  }
  __syncthreads();
  if (tid < nj) {
    const bool live = (tid < cbn) || (tid >= cbw && tid < cbw + kbn);
    if (live) {
      float v = 0.0f;
      if (do_cv && tid < cbn) {
        const float* src = reinterpret_cast<const float*>(red4) + tid;   // band column tid = quad tid / 4, element tid % 4
        for (int gi = 0; gi < ngrp; ++gi) v += src[4 * gi * nq];
      }
      if (tid >= cbw && Sm > 0)
        for (int gi = 0; gi < nkg; ++gi) v += redk[gi * kcn + (tid - cbw)];
      if (Sw > 0)
        for (int gi = 0; gi < nwg; ++gi) v += redk[kFinBlock + gi * njn + tid];
      p.out[static_cast<size_t>(hq) * D + dim_of[tid]] = Lsum > 0.0f ? v / Lsum : 0.0f;   // (a sequence without rows)
    }
  }
}

template <int kFin2Wide>
__global__ __launch_bounds__(kFinBlock, kFin2Wide == 16 ? 2 : 4) void decode_finish2(DecodeParams p, int NS) {
  // workgroup -> (KV head, query head of the group, slice): the G * NS workgroups of a KV head share an XCD
  const int per_kv = p.G * NS;
  const int L = blockIdx.x, xcd = L & 7, slot = L >> 3;
  const int bh = (slot / per_kv) * 8 + xcd;
  if (bh >= p.B * p.Hkv) return;
  const int within = slot % per_kv;
  finish2_slice<kFin2Wide>(p, SeqView{p.N, p.W, p.Sm, p.Sw, p.chunk_m, p.part_m, p.part_w}, NS, bh, within / NS, within % NS);
}

// ---------------------------------------------------------------------------
// 4. the whole call in one launch: one workgroup per (sequence, KV head)
// ---------------------------------------------------------------------------
// With many (sequence, KV head) pairs nothing has to be split to fill the chip, and a call of
// three launches is mostly launch latency and dependent round trips.  Here a workgroup runs the
// phases of its pair back to back - series coefficients, all middle rows as one chunk, the
// full-width rows, the merge with diag(w) C_v - and the pieces of state that the three-launch
// form passes through the workspace (g, packed q, one record per phase) stay with the workgroup
// that wrote them (same compute unit, same first-level cache).  Sequences may differ in length:
// a workgroup takes its own counts from seq_n / seq_w.
// All full-width rows of a pair in one pass: wave w takes rows 256 s + 64 w .. + 63 of every chunk
// s, keeps a running (max, sum, accumulator) of its own across the chunks, and requests the rows
// of the next chunk as soon as the registers of the current one are free.  The waves meet once,
// at the end, and leave ONE record.  Same arithmetic per chunk as partial_full_fast.
// kH: query columns carried through the V side (1 for one query head per KV head, else 4).
template <typename T, int kH>
__device__ __forceinline__ void fused_full_rows(const DecodeParams& p, const SeqView& sv, unsigned char* smem,
                                                const int bh, const unsigned lds_recw) {
  static_assert(sizeof(T) == 2, "16-bit elements");
  constexpr int D = 128, kHP = 4;   // (LDS pitches stay those of four columns)
  const int b = bh / p.Hkv, hkv = bh % p.Hkv;
  const int G = p.G;
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int q4 = lane >> 4, r16 = lane & 15;
  const size_t hq0 = static_cast<size_t>(b) * p.Hq + hkv * G;
  const int W = sv.W, jlast = max(W - 1, 0);
  const int nch = (W + kWChunk - 1) / kWChunk;
  const int jvis = W - p.Tq + r16 / p.Gq;

  float* pw = reinterpret_cast<float*>(smem) + wave * kWRows * kHP;          // [64 rows][4 columns] probabilities
  float* red = reinterpret_cast<float*>(smem) + kWaves * kWRows * kHP;      // [waves][4 columns][128 dims]
  float* wm = red + kWaves * kHP * D;                                        // [waves][4] maxima
  float* wl = wm + kWaves * kHP;                                             // [waves][4] sums
  float* wa = wl + kWaves * kHP;                                             // [waves][4] rescale factors of a chunk

  const T* kbase = static_cast<const T*>(p.k_full) + bh * p.full_stride;
  const T* vbase = static_cast<const T*>(p.v_full) + bh * p.full_stride;
  const int dc = lane & 15, rg = lane >> 4;
  Frag<T> ka[4][kRB], vf[16];
  auto load_k = [&](int s) {
    const int jw = s * kWChunk + wave * kWRows;
#pragma unroll
    for (int rb = 0; rb < kRB; ++rb) {
      const T* krow = kbase + static_cast<int64_t>(min(jw + 16 * rb + r16, jlast)) * D + 8 * q4;
#pragma unroll
      for (int cc = 0; cc < 4; ++cc) ka[cc][rb].load(krow + cc * 32);
    }
  };
  auto load_v = [&](int s) {
    const int jw = s * kWChunk + wave * kWRows;
#pragma unroll
    for (int i = 0; i < 16; ++i) vf[i].load(vbase + static_cast<int64_t>(min(jw + rg + 4 * i, jlast)) * D + dc * 8);
  };
  load_k(0);
  Frag<T> qb[4];
  {
    const T* q = static_cast<const T*>(p.q) + (hq0 + min(r16, G - 1)) * D + 8 * q4;
#pragma unroll
    for (int cc = 0; cc < 4; ++cc) qb[cc].load(q + cc * 32);
  }
  load_v(0);
  if (r16 >= G) {
#pragma unroll
    for (int cc = 0; cc < 4; ++cc) qb[cc].zero();
  }
  float m_run = -INFINITY, l_run = 0.0f;
  float acc[kH][8];
#pragma unroll
  for (int h = 0; h < kH; ++h)
#pragma unroll
    for (int e = 0; e < 8; ++e) acc[h][e] = 0.0f;

  for (int s = 0; s < nch; ++s) {
    const int jw = s * kWChunk + wave * kWRows;
    const int nw = max(0, min(kWRows, W - jw));
    f32x4 sacc[kRB];
#pragma unroll
    for (int rb = 0; rb < kRB; ++rb) sacc[rb] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int cc = 0; cc < 4; ++cc)
#pragma unroll
      for (int rb = 0; rb < kRB; ++rb) mma_k32(sacc[rb], ka[cc][rb], qb[cc]);
    load_k(min(s + 1, nch - 1));   // (the last chunk is asked for once more: never used, never waited for alone)
    float m_w = -INFINITY;
#pragma unroll
    for (int rb = 0; rb < kRB; ++rb)
#pragma unroll
      for (int v = 0; v < 4; ++v) {
        const int r = 16 * rb + 4 * q4 + v;
        const float scv = (r < nw && r16 < G && jw + r <= jvis) ? sacc[rb][v] * p.scale : -INFINITY;
        sacc[rb][v] = scv;
        m_w = fmaxf(m_w, scv);
      }
    m_w = cross_row_max(m_w);
    const float m_new = fmaxf(m_run, m_w);
    const float m_ref = (m_new == -INFINITY) ? 0.0f : m_new;
    const float alpha = __expf(m_run - m_ref);   // m_run = -inf -> 0
    float l_w = 0.0f;
#pragma unroll
    for (int rb = 0; rb < kRB; ++rb)
#pragma unroll
      for (int v = 0; v < 4; ++v) {
        const float e = __expf(sacc[rb][v] - m_ref);   // masked rows hold -inf -> 0
        l_w += e;
        if (r16 < kH) pw[(16 * rb + 4 * q4 + v) * kHP + r16] = e;
      }
    l_w = cross_row_sum(l_w);
    l_run = l_run * alpha + l_w;
    m_run = m_new;
    if (lane < kH) wa[wave * kHP + lane] = alpha;
    // written by this wave, read by this wave: the LDS operations of a wave complete in order
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
    const f32x4 al = *reinterpret_cast<const f32x4*>(wa + wave * kHP);
#pragma unroll
    for (int h = 0; h < kH; ++h)
#pragma unroll
      for (int e = 0; e < 8; ++e) acc[h][e] *= al[h];
#pragma unroll
    for (int i = 0; i < 16; ++i) {
      const int r = rg + 4 * i;
      const f32x4 p4 = *reinterpret_cast<const f32x4*>(pw + r * kHP);   // rows past the end hold zeros
      float x[8];
      unpack8(vf[i], x);
#pragma unroll
      for (int h = 0; h < kH; ++h)
#pragma unroll
        for (int e = 0; e < 8; ++e) acc[h][e] += p4[h] * x[e];
    }
    load_v(min(s + 1, nch - 1));
    // the next chunk's probabilities overwrite pw: this wave's reads above come first (in-order LDS)
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
  }
  // the four row groups of the wave meet in its first 16 lanes
#pragma unroll
  for (int h = 0; h < kH; ++h)
#pragma unroll
    for (int e = 0; e < 8; ++e) acc[h][e] = cross_row_sum(acc[h][e]);
  if (rg == 0) {
#pragma unroll
    for (int h = 0; h < kH; ++h) {
      float* dst = red + (wave * kHP + h) * D + dc * 8;
      *reinterpret_cast<f32x4*>(dst) = f32x4{acc[h][0], acc[h][1], acc[h][2], acc[h][3]};
      *reinterpret_cast<f32x4*>(dst + 4) = f32x4{acc[h][4], acc[h][5], acc[h][6], acc[h][7]};
    }
  }
  if (lane < kH) {
    wm[wave * kHP + lane] = m_run;
    wl[wave * kHP + lane] = l_run;
  }
  __syncthreads();
  if (tid < kH * (D / 4)) {
    const int h = tid / (D / 4), d4 = tid % (D / 4);
    if (h < G) {
      float ms = wm[h];
#pragma unroll
      for (int w = 1; w < kWaves; ++w) ms = fmaxf(ms, wm[w * kHP + h]);
      f32x4 v = {0.f, 0.f, 0.f, 0.f};
      float l = 0.0f;
#pragma unroll
      for (int w = 0; w < kWaves; ++w) {
        const float mw = wm[w * kHP + h];
        const float f = (mw == -INFINITY) ? 0.0f : __expf(mw - ms);
        l += f * wl[w * kHP + h];
        v += f * *reinterpret_cast<const f32x4*>(red + (w * kHP + h) * D + 4 * d4);
      }
      float* rec = reinterpret_cast<float*>(smem + lds_recw) + h * p.recw;   // past everything this phase uses
      *reinterpret_cast<f32x4*>(rec + 4 + 4 * d4) = v;
      if (d4 == 0) {
        rec[0] = ms;
        rec[1] = l;
      }
    }
  }
}

// Merge of the pair's two records (middle rows, full-width rows) with diag(w) C_v, all out of
// LDS: out[d] = (e_m (C_v^T diag(w) r | kept accumulator) + e_w acc_w[d]) / (e_m l_m + e_w l_w).
__device__ __forceinline__ void fused_finish(const DecodeParams& p, unsigned char* smem, const int bh,
                                             const FusedLds& L, const bool has_m, const bool has_w) {
  constexpr int D = 128;
  const int tid = threadIdx.x, lane = tid & 63;
  const int b = bh / p.Hkv, hkv = bh % p.Hkv;
  const int G = p.G, M = p.M, Dvc = p.Dvc, Mint = p.Mint;
  const size_t hq0 = static_cast<size_t>(b) * p.Hq + hkv * G;
  const float* recm = reinterpret_cast<const float*>(smem + L.recm);
  const float* recw = reinterpret_cast<const float*>(smem + L.recw);
  const float* cv_s = reinterpret_cast<const float*>(smem + L.cv);
  const int Dva = 16 * ((p.Dvu + 15) / 16);
  const int pitch_r = M + 4;
  float* rr = reinterpret_cast<float*>(smem);                       // [G][M + 4] weighted series sums, basis order
  f32x4* part4 = reinterpret_cast<f32x4*>(smem + 8192);             // [G][row groups][column quads]

  uint64_t vbal[4];
  mask_ballots(p.vmask + static_cast<size_t>(bh) * D, D, lane, vbal);

  const bool do_cv = has_m && Dvc > 0;
  const int nq = max(Dvc / 4, 1), ngrp = kBlock / nq;
  if (do_cv) {
    for (int it = tid; it < G * Mint; it += kBlock) {   // record order: 32 * chunk + 16 * (cos | sin) + order
      const int h = it / Mint, ig = it - h * Mint;
      const int n = 16 * (ig >> 5) + (ig & 15) + 1, cs = (ig >> 4) & 1;
      const int mm = 2 * n - 1 + cs;
      if (mm < M) rr[h * pitch_r + mm] = recm[h * p.recm + 4 + Dva + ig] * basis_weight(n, p.T);
    }
    if (tid < G) rr[tid * pitch_r] = recm[tid * p.recm + 1] * basis_weight(0, p.T);   // the sum of the probabilities
  }
  // (the waits of this barrier also cover the stash: it was requested before the middle-row phase)
  __builtin_amdgcn_s_waitcnt(0);
  __syncthreads();
  if (do_cv) {
    const int cq = tid % nq, rg = tid / nq;
    f32x4 o4[4];
#pragma unroll
    for (int h = 0; h < 4; ++h) o4[h] = f32x4{0.f, 0.f, 0.f, 0.f};
    if (rg < ngrp) {
      for (int mm = rg; mm < M; mm += ngrp) {
        const f32x4 c = *reinterpret_cast<const f32x4*>(cv_s + mm * Dvc + 4 * cq);
#pragma unroll
        for (int h = 0; h < 4; ++h)
          if (h < G) o4[h] += rr[h * pitch_r + mm] * c;
      }
#pragma unroll
      for (int h = 0; h < 4; ++h)
        if (h < G) part4[(h * ngrp + rg) * nq + cq] = o4[h];
    }
  }
  __syncthreads();
  if (tid < D) {
    const int r = dim_rank(vbal, tid);
    for (int h = 0; h < G; ++h) {
      const float mm_ = has_m ? recm[h * p.recm + 0] : -INFINITY, lm = has_m ? recm[h * p.recm + 1] : 0.0f;
      const float mw = has_w ? recw[h * p.recw + 0] : -INFINITY, lw = has_w ? recw[h * p.recw + 1] : 0.0f;
      const float mx = fmaxf(mm_, mw);
      const float em = (mm_ == -INFINITY) ? 0.0f : __expf(mm_ - mx);
      const float ew = (mw == -INFINITY) ? 0.0f : __expf(mw - mx);
      float v = 0.0f;
      if (has_m) {
        if (r < 0) {
          const int c = -r - 1;
          const float* src = reinterpret_cast<const float*>(part4 + h * ngrp * nq) + c;   // column c = quad c / 4, element c % 4
          float a = 0.0f;
          for (int gi = 0; gi < ngrp; ++gi) a += src[4 * gi * nq];
          v = em * a;
        } else {
          v = em * recm[h * p.recm + 4 + r];
        }
      }
      if (has_w) v += ew * recw[h * p.recw + 4 + tid];
      const float lsum = em * lm + ew * lw;
      p.out[(hq0 + h) * D + tid] = lsum > 0.0f ? v / lsum : 0.0f;   // (a sequence without rows)
    }
  }
}

template <int CW, int DVT, int GP>
__global__ __launch_bounds__(kBlock, 1) void decode_fused(DecodeParams p) {
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  using T = bf16_t;
  constexpr int Mint = kWaves * CW * 32;
  const int bh = blockIdx.x, b = bh / p.Hkv;
  SeqView sv;
  sv.N = seq_middle_rows(p, b);
  sv.W = seq_full_rows(p, b);
  sv.Sm = sv.N > 0 ? 1 : 0;
  sv.Sw = sv.W > 0 ? 1 : 0;
  sv.chunk_m = max(sv.N, 1);
  sv.part_m = nullptr;   // the records of both phases stay in LDS
  sv.part_w = nullptr;
  const FusedLds L = fused_lds(p.lds_tab, p.G, Mint, p.recm, p.recw, p.M, p.Dvc);
  if (sv.N > 0) {
    partial_middle_fast<CW, DVT, GP, true>(p, sv, smem, bh, 0);
  }
  if (sv.W > 0) {
    __syncthreads();
    if constexpr (GP == 1) fused_full_rows<T, 1>(p, sv, smem, bh, L.recw);
    else fused_full_rows<T, 4>(p, sv, smem, bh, L.recw);
  }
  __syncthreads();
  fused_finish(p, smem, bh, L, sv.N > 0, sv.W > 0);
}

// ---------------------------------------------------------------------------
// host side
// ---------------------------------------------------------------------------
struct DecodePlan {
  int Gp, KT, Mint, cw, Sw, Sm, chunk_m, recm, recw;
  int wrb;        // 16-row blocks per wave of a full-width-row workgroup
  int Swp;        // chunks of full-width rows that run inside the middle-row launch
  unsigned lds_window;   // dynamic LDS of a full-width-row workgroup
  int fast;   // 0: general middle-row kernel; 4 / 8: the specialised one with that many waves
  bool fused; // the whole call as one launch (one workgroup per (sequence, KV head))
  unsigned lds_tab, lds_total;
  unsigned lds_fused;    // dynamic LDS of a workgroup of the one-launch form
  size_t off_gs, off_g0, off_qk, off_pm, off_pw, total;
};

static int round_up(int x, int a) { return (x + a - 1) / a * a; }

static int series_chunks_per_wave(int M) {   // compiled series lengths: 128, 256, 512, 1024 slots
  const int slots = 2 * (M / 2);
  for (int cw : {1, 2, 4, 8})
    if (slots <= kWaves * cw * 32) return cw;
  return 0;
}

// Steps per chunk when the caller leaves the split to the library.  With few (sequence, head)
// pairs the chunks are sized so that all workgroups of the launch (middle chunks and full-row
// chunks) are resident at once, two per compute unit when two fit (short series), else one.
// With many pairs that would make long chunks and a ragged last round: short chunks balance
// better (measured: 3-5 steps per chunk is the flat optimum at two workgroups per unit).
static int default_steps_per_chunk(int B, int Hkv, int N, int step, int cw, int Sw) {
  const long total_steps = static_cast<long>(B) * Hkv * ((N + step - 1) / step);
  // a launch small enough for ONE workgroup per compute unit with at most six steps each runs
  // faster that way than spread over two per unit (32 K tokens: 25 chunks per head 12.0 us, 42 chunks 13.1 us)
  if (cw <= 2) {
    const long one_each = 256 - static_cast<long>(B) * Hkv * Sw;
    if (one_each >= 128) {
      const long spc1 = (total_steps + one_each - 1) / one_each;
      if (spc1 >= 1 && spc1 <= 6) return static_cast<int>(spc1);
    }
  }
  const long slots = cw <= 2 ? 512 : 256;
  long target = slots - static_cast<long>(B) * Hkv * Sw;
  if (target < 3 * slots / 4) target = 3 * slots / 4;
  long spc = (total_steps + target - 1) / target;
  const long cap = cw <= 2 ? 5 : 16;
  if (spc > cap) spc = cap;
  if (spc < 1) spc = 1;
  return static_cast<int>(spc);
}

// shapes the one-launch form covers: those of the specialised four-wave middle-row kernel whose
// other phases have a streaming form (head dim 128, compressed counts in multiples of 4)
static bool fused_shape(int dtype, int Hq, int Hkv, int D, int Dkc, int Dvc, int M, int N) {
  const int G = Hq / Hkv, Dku = D - Dkc, Dvu = D - Dvc;
  const int cw = series_chunks_per_wave(M);
  return dtype == FA_BF16 && D == 128 && G <= 4 && cw >= 1 && cw <= 2 && N > 0 && Dku > 0 && Dku <= 32 &&
         Dvu > 0 && Dvu <= 32 && Dkc > 0 && (Dkc & 3) == 0 && (Dvc & 3) == 0;
}
constexpr int kFusedMinPairs = 192;   // (sequence, KV head) pairs from which the one-launch form is the default

static bool make_plan(DecodePlan& pl, int dtype, int B, int Hq, int Hkv, int D, int Dkc, int Dvc, int M,
                      int N, int W, int num_splits, int fused_mode = 0) {   // fused_mode: 0 by shape, -1 never
  const int G = Hq / Hkv;
  pl.Gp = 1;
  while (pl.Gp < G) pl.Gp *= 2;
  pl.KT = 16 / pl.Gp < kMaxKT ? 16 / pl.Gp : kMaxKT;
  pl.cw = series_chunks_per_wave(M);
  if (pl.cw == 0 || (dtype == FA_F32 && pl.cw > 2)) return false;
  pl.Mint = kWaves * pl.cw * 32;
  const int step = pl.KT * kTJ;
  pl.Sw = (W + kWChunk - 1) / kWChunk;
  pl.fused = fused_shape(dtype, Hq, Hkv, D, Dkc, Dvc, M, N) &&
             fused_mode >= 0 && (num_splits == 1 || (num_splits == 0 && static_cast<long>(B) * Hkv >= kFusedMinPairs));
  if (pl.fused) {   // one middle chunk and one record of full-width rows per (sequence, KV head)
    num_splits = 1;
    pl.Sw = W > 0 ? 1 : 0;
  }
  // full-width rows that ride in the launch of the series coefficients (see Swp below) take no
  // compute unit away from the middle rows
  const bool window_rides = dtype == FA_BF16 && N > 0 && pl.cw == 4 && G <= 4 && D - Dkc > 0 && D - Dkc <= 32 &&
                            D - Dvc > 0 && D - Dvc <= 32 && Dkc > 0 && (Dkc & 3) == 0;
  // ... and when they would be few workgroups of 256 rows each, every one of them bound by what a single
  // compute unit can keep in flight, they go in workgroups of 64 rows instead (four times as many units)
  pl.wrb = 4;
  // (inside the middle-row launch they are better off as few long workgroups: 32 K tokens 13.6 -> 16.6 us with 64-row ones)
  if (window_rides && D == 128 && static_cast<long>(B) * Hkv * pl.Sw < 128 && (W + 63) / 64 <= kMaxPartials / 2) {
    pl.wrb = 1;
    pl.Sw = (W + 63) / 64;
  }
  if (N > 0) {
    int chunk;
    if (num_splits > 0) chunk = round_up((N + num_splits - 1) / num_splits, step);
    else chunk = default_steps_per_chunk(B, Hkv, N, step, pl.cw, window_rides ? 0 : pl.Sw) * step;
    // a record list has room for kMaxPartials entries per query head: very long contexts (or a
    // caller's very fine split) take longer chunks instead of being refused
    if (pl.Sw < kMaxPartials) {
      const int room = kMaxPartials - pl.Sw;
      const int least = round_up((N + room - 1) / room, step);
      if (chunk < least) chunk = least;
    }
    pl.chunk_m = chunk;
    pl.Sm = (N + chunk - 1) / chunk;
  } else {
    pl.chunk_m = step;
    pl.Sm = 0;
  }
  if (pl.Sw + pl.Sm > kMaxPartials) return false;
  const unsigned ts = (dtype == FA_F32) ? 4 : 2;   // bytes of a q/K/V element
  const int Dvu = D - Dvc, Dku = D - Dkc;
  const unsigned DVT = (Dvu + 15) / 16;
  const unsigned Dkq = (((Dku + 7) & ~7) + 31) / 32 * 32;
  pl.recm = 4 + 16 * DVT + pl.Mint;
  pl.recw = 4 + D;
  // the specialised kernels: bf16, groups of at most four query heads, 1 .. 32 kept dims on both sides,
  // at most 512 series slots (eight waves once the series is that long)
  pl.fast = 0;
  if (dtype == FA_BF16 && N > 0 && pl.cw <= 4 && G <= 4 && Dku > 0 && Dku <= 32 && Dvu > 0 && Dvu <= 32)
    pl.fast = pl.cw == 4 ? 8 : 4;
  // an eight-wave workgroup takes a whole compute unit: when the caller's split makes more chunks than
  // units, the chunks that would share a workgroup are joined (tables built once; the running maximum,
  // sum and accumulators simply carry on, and the final merge reads one record instead of several:
  // 128 K tokens in 64 chunks per head, 8 heads: partial + finish 39.3 -> 36.7 us)
  if (pl.fast == 8) {
    const long chunks = static_cast<long>(B) * Hkv * pl.Sm;
    if (chunks > 256) {
      const int per = static_cast<int>((chunks + 255) / 256);
      pl.chunk_m *= per;
      pl.Sm = (N + pl.chunk_m - 1) / pl.chunk_m;
    }
  }
  const unsigned nwaves = pl.fast == 8 ? kWaves8 : kWaves;
  const unsigned redb = (16 * (pl.Mint + 4) + nwaves * 16 * (16 * DVT + 4)) * 4;
  const unsigned xchg = pl.fast == 8 ? kXs8Bytes + 8 * 1024 : kXchgBytes;
  const unsigned tab = redb > xchg ? redb : xchg;
  pl.lds_tab = (tab + 255u) & ~255u;
  const unsigned mid = pl.lds_tab + G * (pl.Mint + 32) * 4 + G * Dkq * ts + 64;   // (+ constant-term coefficients)
  const unsigned wpath = 16 * FA_MAX_HEAD_DIM * ts + kWChunk * kMaxG * 4 + kWaves * 512 * 4 * 4;   // q, p tiles, partial sums
  // the specialised full-row path keeps only probabilities, per-wave sums and statistics there
  const bool wfast = dtype == FA_BF16 && D == 128 && G <= 4;
  pl.lds_window = wfast ? (kWaves * kWRows * 4 + kWaves * 4 * 128 + 64) * 4 : wpath;   // (64: maxima, sums, factors)
  // The eight-wave middle-row workgroups take a compute unit each, so full-width-row workgroups in their
  // launch would run as a tail behind them: they run in the launch that forms the series coefficients
  // instead (independent work that fills the chip while that chain of round trips is in flight).  With
  // two middle-row workgroups per unit the full-width rows overlap with them and stay where they are
  // (measured: moving them costs 1.5 us on 32 K tokens, 12 us on 8 x 4 K MHA).
  pl.Swp = (pl.fast == 8 && Dkc > 0 && (Dkc & 3) == 0) ? 0 : pl.Sw;   // (= window_rides)
  {
    const FusedLds L = fused_lds(pl.lds_tab, G, pl.Mint, pl.recm, pl.recw, M, Dvc);
    pl.lds_fused = L.total > pl.lds_window ? L.total : pl.lds_window;
    // a stash of C_v that does not fit next to the other regions: the three-launch form
    if (pl.fused && pl.lds_fused > kMaxDynLds)
      return make_plan(pl, dtype, B, Hq, Hkv, D, Dkc, Dvc, M, N, W, num_splits, -1);
  }
  const unsigned t = mid > wpath ? mid : wpath;
  pl.lds_total = (t + 255u) & ~255u;
  if (pl.lds_total > kMaxDynLds) return false;
  const size_t BHq = static_cast<size_t>(B) * Hq;
  pl.off_gs = 0;
  pl.off_g0 = align_up(BHq * pl.Mint * sizeof(float), 256);
  pl.off_qk = pl.off_g0 + align_up(BHq * sizeof(float), 256);
  pl.off_pm = pl.off_qk + align_up(BHq * Dkq * 4 + 16, 256);   // sized for fp32: the size query has no dtype
  pl.off_pw = pl.off_pm + align_up(BHq * pl.Sm * pl.recm * sizeof(float) + 16, 256);
  pl.total = pl.off_pw + align_up(BHq * pl.Sw * pl.recw * sizeof(float) + 16, 256);
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
  if (dtype == FA_F32 && M > FA_MAX_DECODE_STATES_F32) return FA_ERR_UNSUPPORTED;
  if (D - Dvc > 16 * kMaxDvTiles) return FA_ERR_UNSUPPORTED;
  if (static_cast<long>(B) * Hkv > 65535) return FA_ERR_UNSUPPORTED;
  return FA_OK;
}

template <typename T, int CW, int DVTM, bool KC1>
static int launch_partial(const DecodeParams& p, unsigned lds, hipStream_t st, KernelTimers* tm) {
  auto kern = decode_partial<T, CW, DVTM, KC1>;
  // the dynamic-LDS ceiling is a property of the kernel as loaded on the current device: raised
  // whenever a launch needs it (a host-side table write, no stream operation)
  if (lds > 48u * 1024u &&
      hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize,
                          static_cast<int>(kMaxDynLds)) != hipSuccess)
    return FA_ERR_HIP;
  dim3 g2(p.Swp + p.Sm, p.B * p.Hkv);
  FA_LAUNCH_TIMED(tm, 1, kern, g2, dim3(kBlock), lds, st, p);
  return FA_OK;
}

template <typename T>
static int launch_finish(const DecodeParams& p, hipStream_t st, KernelTimers* tm, hipError_t prior) {
  if ((p.Dvc & 3) == 0) {
    // slices per query head: as many as keep the launch within one round of resident workgroups
    const int BH = p.B * p.Hkv;
    const long heads = static_cast<long>(p.B) * p.Hq;
    int NS = p.D <= 32 ? 1 : (p.D <= 64 ? 2 : (p.D <= 128 ? 4 : 8));
    while (NS > 1 && heads * NS > 1024) NS /= 2;
    const dim3 grid((BH + 7) / 8 * 8 * p.G * NS);
    if (heads * NS <= 512) FA_LAUNCH_TIMED(tm, 2, decode_finish2<16>, grid, dim3(kFinBlock), 0, st, p, NS);
    else FA_LAUNCH_TIMED(tm, 2, decode_finish2<8>, grid, dim3(kFinBlock), 0, st, p, NS);
  } else if (static_cast<long>(p.B) * p.Hq >= 256) {
    FA_LAUNCH_TIMED(tm, 2, (decode_finish<T, 64>), dim3((p.D + 63) / 64, p.B * p.Hq), dim3(kFinBlock), 0, st, p);
  } else {
    FA_LAUNCH_TIMED(tm, 2, (decode_finish<T, 32>), dim3((p.D + 31) / 32, p.B * p.Hq), dim3(kFinBlock), 0, st, p);
  }
  // only this call's launches are reported: an error some earlier, unrelated HIP call of the
  // application left behind is neither returned nor cleared
  return (hipPeekAtLastError() == hipSuccess || prior != hipSuccess) ? FA_OK : FA_ERR_HIP;
}

template <int CW, int DVT, int GP>
static int launch_partial_fast_one(const DecodeParams& p, unsigned lds, hipStream_t st, KernelTimers* tm) {
  auto kern = decode_partial_fast<CW, DVT, GP>;
  if (lds > 48u * 1024u &&
      hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize,
                          static_cast<int>(kMaxDynLds)) != hipSuccess)
    return FA_ERR_HIP;
  dim3 g2(p.Swp + p.Sm, p.B * p.Hkv);
  FA_LAUNCH_TIMED(tm, 1, kern, g2, dim3(kBlock), lds, st, p);
  return FA_OK;
}

template <int CW, int DVT, int GP>
static int launch_partial_fast8_one(const DecodeParams& p, unsigned lds, hipStream_t st, KernelTimers* tm) {
  auto kern = decode_partial_fast8<CW, DVT, GP>;
  if (lds > 48u * 1024u &&
      hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize,
                          static_cast<int>(kMaxDynLds)) != hipSuccess)
    return FA_ERR_HIP;
  dim3 g2(p.Swp + p.Sm, p.B * p.Hkv);
  FA_LAUNCH_TIMED(tm, 1, kern, g2, dim3(kBlock8), lds, st, p);
  return FA_OK;
}

static int launch_partial_fast(const DecodeParams& p, const DecodePlan& pl, hipStream_t st, KernelTimers* tm) {
  const bool one_tile = p.Dvu <= 16, one_head = p.G == 1;
#define FA_FAST(CW_)                                                                              \
  return one_tile ? (one_head ? launch_partial_fast_one<CW_, 1, 1>(p, pl.lds_total, st, tm)        \
                              : launch_partial_fast_one<CW_, 1, 4>(p, pl.lds_total, st, tm))       \
                  : (one_head ? launch_partial_fast_one<CW_, 2, 1>(p, pl.lds_total, st, tm)        \
                              : launch_partial_fast_one<CW_, 2, 4>(p, pl.lds_total, st, tm))
  switch (pl.cw) {
    case 1: FA_FAST(1);
    case 2: FA_FAST(2);
    default: break;
  }
#undef FA_FAST
  // 512 slots: eight waves, two chunks each
  return one_tile ? (one_head ? launch_partial_fast8_one<2, 1, 1>(p, pl.lds_total, st, tm)
                              : launch_partial_fast8_one<2, 1, 4>(p, pl.lds_total, st, tm))
                  : (one_head ? launch_partial_fast8_one<2, 2, 1>(p, pl.lds_total, st, tm)
                              : launch_partial_fast8_one<2, 2, 4>(p, pl.lds_total, st, tm));
}

template <int CW, int DVT, int GP>
static int launch_fused_one(const DecodeParams& p, unsigned lds, hipStream_t st, KernelTimers* tm) {
  auto kern = decode_fused<CW, DVT, GP>;
  if (lds > 32u * 1024u &&
      hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize,
                          static_cast<int>(lds)) != hipSuccess)
    return FA_ERR_HIP;
  FA_LAUNCH_TIMED(tm, 1, kern, dim3(p.B * p.Hkv), dim3(kBlock), lds, st, p);
  return FA_OK;
}

static int launch_fused(const DecodeParams& p, const DecodePlan& pl, hipStream_t st, KernelTimers* tm) {
  const hipError_t prior = hipPeekAtLastError();
  const bool one_tile = p.Dvu <= 16, one_head = p.G == 1;
  const unsigned lds = pl.lds_fused;
  int rc;
#define FA_FUSED(CW_)                                                                  \
  rc = one_tile ? (one_head ? launch_fused_one<CW_, 1, 1>(p, lds, st, tm)               \
                            : launch_fused_one<CW_, 1, 4>(p, lds, st, tm))              \
                : (one_head ? launch_fused_one<CW_, 2, 1>(p, lds, st, tm)               \
                            : launch_fused_one<CW_, 2, 4>(p, lds, st, tm))
  if (pl.cw == 1) FA_FUSED(1);
  else FA_FUSED(2);
#undef FA_FUSED
  if (rc != FA_OK) return rc;
  return (hipPeekAtLastError() == hipSuccess || prior != hipSuccess) ? FA_OK : FA_ERR_HIP;
}

// tm (optional): per-kernel event pairs, for fa_decode_timed
template <typename T>
static int launch_decode(const DecodeParams& p, const DecodePlan& pl, hipStream_t st, KernelTimers* tm) {
  const int BH = p.B * p.Hkv;
  if constexpr (sizeof(T) == 2) {
    if (pl.fused) return launch_fused(p, pl, st, tm);
  }
  const hipError_t prior = hipPeekAtLastError();
  if (p.Sm > 0 && p.Dkc > 0 && (p.Dkc & 3) == 0) {
    const bool wide = static_cast<long>(BH) * (p.Mint / 64 + 1) >= 256;
    const int nprep = wide ? p.Mint / 64 + 1 : p.Mint / 16 + 1;
    if (p.Sw > 0 && p.Swp == 0) {   // the full-width rows ride along
      DecodeParams pp = p;
      pp.nprep = nprep;
      const unsigned lds = pl.lds_window;
      auto kern = wide ? decode_prepare_window<T, 4> : decode_prepare_window<T, 16>;
      // (the kernel also holds 16 KB of static LDS: the ceiling asked for is what this launch needs)
      if (lds > 32u * 1024u &&
          hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize,
                              static_cast<int>(lds)) != hipSuccess)
        return FA_ERR_HIP;
      FA_LAUNCH_TIMED(tm, 0, kern, dim3(nprep + p.Sw, BH), dim3(kBlock), lds, st, pp);
    } else if (wide) {
      FA_LAUNCH_TIMED(tm, 0, (decode_prepare2<T, 4>), dim3(nprep, BH), dim3(kBlock), 0, st, p);
    } else {
      FA_LAUNCH_TIMED(tm, 0, (decode_prepare2<T, 16>), dim3(nprep, BH), dim3(kBlock), 0, st, p);
    }
  } else if (p.Sm > 0) {
    if (static_cast<long>(BH) * ((p.Mint + 32) / 32) >= 512) {
      dim3 g1((p.Mint + 32) / 32, BH);
      FA_LAUNCH_TIMED(tm, 0, (decode_prepare<T, 32>), g1, dim3(kBlock), prep_lds_bytes(32, p.G, p.Dkc), st, p);
    } else {
      dim3 g1((p.Mint + 8) / 8, BH);
      FA_LAUNCH_TIMED(tm, 0, (decode_prepare<T, 8>), g1, dim3(kBlock), prep_lds_bytes(8, p.G, p.Dkc), st, p);
    }
  }
  int rc;
  if constexpr (sizeof(T) == 2) {
    // the specialised kernel: groups of at most four query heads, 1 .. 32 kept dims on both sides
    if (pl.fast != 0) {
      rc = launch_partial_fast(p, pl, st, tm);
      if (rc != FA_OK) return rc;
      return launch_finish<T>(p, st, tm, prior);
    }
  }
  const bool narrow = p.Dvu <= 32;   // kept V dims fit two MFMA column tiles
  const bool kc1 = p.Dku <= 32;      // kept K dims fit one MFMA step
#define FA_LAUNCH_PARTIAL(CW_)                                                                      \
  rc = (narrow && kc1) ? launch_partial<T, CW_, 2, true>(p, pl.lds_total, st, tm)                       \
       : narrow        ? launch_partial<T, CW_, 2, false>(p, pl.lds_total, st, tm)                      \
                       : launch_partial<T, CW_, kMaxDvTiles, false>(p, pl.lds_total, st, tm)
  switch (pl.cw) {
    case 1: FA_LAUNCH_PARTIAL(1); break;
    case 2: FA_LAUNCH_PARTIAL(2); break;
    default:
      if constexpr (sizeof(T) == 2) {   // fp32 inputs stop at 256 states (two chunks per wave)
        if (pl.cw == 4) FA_LAUNCH_PARTIAL(4);
        else FA_LAUNCH_PARTIAL(8);
      } else {
        rc = FA_ERR_UNSUPPORTED;
      }
      break;
  }
#undef FA_LAUNCH_PARTIAL
  if (rc != FA_OK) return rc;
  return launch_finish<T>(p, st, tm, prior);
}

}  // namespace fa

extern "C" {

int fa_decode_default_splits(int B, int Hq, int Hkv, int M, int N, int W) {
  if (B <= 0 || Hq <= 0 || Hkv <= 0 || N <= 0 || W < 0 || M < 1 || Hq % Hkv != 0 ||
      Hq / Hkv > FA_MAX_GROUP)
    return 0;
  fa::DecodePlan pl{};
  if (!fa::make_plan(pl, FA_BF16, B, Hq, Hkv, 128, 0, 0, M, N, W, 0)) return 0;
  return pl.Sm;
}

size_t fa_decode_workspace_bytes(int B, int Hq, int Hkv, int D, int Dkc, int Dvc, int M, int N,
                                 int W, int num_splits) {
  if (fa::check_decode_shapes(FA_BF16, B, Hq, Hkv, D, Dkc, Dvc, M, M > N ? M : N, 0, N, W,
                              num_splits) != FA_OK)
    return 0;
  fa::DecodePlan pl{};
  if (!fa::make_plan(pl, FA_BF16, B, Hq, Hkv, D, Dkc, Dvc, M, N, W, num_splits)) return 0;
  return pl.total;
}

static int decode_impl(const void* q, int dtype, int B, int Hq, int Hkv, int D, const float* ck,
                       const uint8_t* kmask, int Dkc, const float* cv, const uint8_t* vmask, int Dvc,
                       int M, int T, int t0, int N, const void* k_keep, int64_t kk_stride_bh,
                       const void* v_keep, int64_t vk_stride_bh, const void* k_full,
                       const void* v_full, int W, int64_t full_stride_bh, float scale,
                       int num_splits, float* out, void* workspace, size_t workspace_bytes,
                       void* hip_stream, fa::KernelTimers* tm, int Tq = 1, const int32_t* seq_n = nullptr,
                       const int32_t* seq_w = nullptr) {
  using namespace fa;
  if ((seq_n || seq_w) && Tq != 1) return FA_ERR_UNSUPPORTED;
  // Tq query tokens per sequence are Tq * Hq query heads to every kernel (group index = token * G +
  // head); only the full-width rows know about tokens: the last Tq rows are the new tokens, and
  // query t sees new tokens 0 .. t
  if (Tq < 1 || (Tq > 1 && Tq > W) || Hq <= 0 || Hkv <= 0 || Hq % Hkv != 0) return FA_ERR_SHAPE;
  const int Gq = Hq / Hkv;
  if (static_cast<long>(Hq) * Tq / Hkv > FA_MAX_GROUP) return FA_ERR_UNSUPPORTED;
  Hq *= Tq;
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
       reinterpret_cast<uintptr_t>(q) | reinterpret_cast<uintptr_t>(cv) | reinterpret_cast<uintptr_t>(ck)) & 15u)
    return FA_ERR_SHAPE;
  // kernels index slabs with 32-bit element offsets
  if (kk_dense > 0x7fffffffLL || vk_dense > 0x7fffffffLL || full_dense > 0x7fffffffLL)
    return FA_ERR_UNSUPPORTED;

  DecodePlan pl{};
  if (!make_plan(pl, dtype, B, Hq, Hkv, D, Dkc, Dvc, M, N, W, num_splits)) return FA_ERR_UNSUPPORTED;
  if (workspace_bytes < pl.total || (reinterpret_cast<uintptr_t>(workspace) & 255u))
    return FA_ERR_WORKSPACE;

  DecodeParams p{};
  p.q = q; p.ck = ck; p.cv = cv; p.kmask = kmask; p.vmask = vmask;
  p.k_keep = k_keep; p.v_keep = v_keep; p.k_full = k_full; p.v_full = v_full;
  p.kk_stride = kk_stride_bh; p.vk_stride = vk_stride_bh; p.full_stride = full_stride_bh;
  p.B = B; p.Hq = Hq; p.Hkv = Hkv; p.G = Hq / Hkv; p.D = D;
  p.Tq = Tq; p.Gq = Gq > 0 ? Gq : 1;
  p.Dkc = Dkc; p.Dvc = Dvc; p.Dku = Dku; p.Dvu = Dvu;
  p.M = M; p.T = T; p.t0 = t0; p.N = N; p.W = W;
  p.Gp = pl.Gp; p.KT = pl.KT; p.Mint = pl.Mint;
  p.Sw = pl.Sw; p.Sm = pl.Sm; p.chunk_m = pl.chunk_m; p.recm = pl.recm; p.recw = pl.recw;
  p.Swp = pl.Swp; p.nprep = 0;
  p.lds_tab = pl.lds_tab;
  p.seq_n = seq_n; p.seq_w = seq_w; p.Sw_rec = pl.Sw; p.wrb = pl.wrb;
  p.scale = scale > 0.0f ? scale : 1.0f / sqrtf(static_cast<float>(D));
  p.ph_scale = 4294967296.0 / static_cast<double>(T);
  char* ws = static_cast<char*>(workspace);
  p.gs = reinterpret_cast<float*>(ws + pl.off_gs);
  p.g0 = reinterpret_cast<float*>(ws + pl.off_g0);
  p.qkeep = ws + pl.off_qk;
  p.part_m = reinterpret_cast<float*>(ws + pl.off_pm);
  p.part_w = reinterpret_cast<float*>(ws + pl.off_pw);
  p.out = out;
  hipStream_t stream = static_cast<hipStream_t>(hip_stream);
  return dtype == FA_F32 ? launch_decode<float>(p, pl, stream, tm)
                         : launch_decode<bf16_t>(p, pl, stream, tm);
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

int fa_decode_varlen(const void* q, int dtype, int B, int Hq, int Hkv, int D, const float* ck,
                     const uint8_t* kmask, int Dkc, const float* cv, const uint8_t* vmask, int Dvc, int M,
                     int T, int t0, int N_max, const int32_t* seq_n, const void* k_keep, int64_t kk_stride_bh,
                     const void* v_keep, int64_t vk_stride_bh, const void* k_full, const void* v_full,
                     int W_max, const int32_t* seq_w, int64_t full_stride_bh, float scale, int num_splits,
                     float* out, void* workspace, size_t workspace_bytes, void* hip_stream) {
  return decode_impl(q, dtype, B, Hq, Hkv, D, ck, kmask, Dkc, cv, vmask, Dvc, M, T, t0, N_max, k_keep,
                     kk_stride_bh, v_keep, vk_stride_bh, k_full, v_full, W_max, full_stride_bh, scale,
                     num_splits, out, workspace, workspace_bytes, hip_stream, nullptr, 1, seq_n, seq_w);
}

int fa_decode_mq(const void* q, int dtype, int B, int Tq, int Hq, int Hkv, int D, const float* ck,
                 const uint8_t* kmask, int Dkc, const float* cv, const uint8_t* vmask, int Dvc, int M,
                 int T, int t0, int N, const void* k_keep, int64_t kk_stride_bh, const void* v_keep,
                 int64_t vk_stride_bh, const void* k_full, const void* v_full, int W,
                 int64_t full_stride_bh, float scale, int num_splits, float* out, void* workspace,
                 size_t workspace_bytes, void* hip_stream) {
  return decode_impl(q, dtype, B, Hq, Hkv, D, ck, kmask, Dkc, cv, vmask, Dvc, M, T, t0, N, k_keep,
                     kk_stride_bh, v_keep, vk_stride_bh, k_full, v_full, W, full_stride_bh, scale,
                     num_splits, out, workspace, workspace_bytes, hip_stream, nullptr, Tq);
}

// ---------------------------------------------------------------------------
// fa_decode_static: fa_decode with the split-K state in a static device array
// ---------------------------------------------------------------------------
// One array per GPU (every device that loads this code object holds its own copy
// at its own address).  In host code the array's name only stands for the symbol;
// the device address is asked for once per device and kept.
static __device__ __align__(256) unsigned char scratch[FA_STATIC_SCRATCH_BYTES];

namespace {
constexpr int kMaxDevices = 64;
std::mutex scratch_mutex;
void* scratch_ptr[kMaxDevices] = {};   // device address of `scratch` on device i (nullptr: not asked yet)

// address of the current device's copy of `scratch`, or nullptr
void* static_scratch() {
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return nullptr;
  std::lock_guard<std::mutex> lock(scratch_mutex);
  if (!scratch_ptr[dev]) {
    void* ptr = nullptr;
    if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess) return nullptr;
    scratch_ptr[dev] = ptr;
  }
  return scratch_ptr[dev];
}
}  // namespace

int fa_decode_static(const void* q, int dtype, int B, int Hq, int Hkv, int D, const float* ck,
                     const uint8_t* kmask, int Dkc, const float* cv, const uint8_t* vmask, int Dvc,
                     int M, int T, int t0, int N, const void* k_keep, int64_t kk_stride_bh,
                     const void* v_keep, int64_t vk_stride_bh, const void* k_full, const void* v_full,
                     int W, int64_t full_stride_bh, float scale, int num_splits, float* out,
                     void* hip_stream) {
  // sizes first: a problem whose split-K state does not fit the array is refused before anything else
  if (Hq > 0 && Hkv > 0 && Hq % Hkv == 0 &&
      fa::check_decode_shapes(dtype, B, Hq, Hkv, D, Dkc, Dvc, M, T, t0, N, W, num_splits) == FA_OK) {
    fa::DecodePlan pl{};
    if (fa::make_plan(pl, dtype, B, Hq, Hkv, D, Dkc, Dvc, M, N, W, num_splits) &&
        pl.total > static_cast<size_t>(FA_STATIC_SCRATCH_BYTES))
      return FA_ERR_SCRATCH;
  }
  void* ws = static_scratch();
  if (!ws) return FA_ERR_HIP;
  // every float of the state that a kernel reads is written by an earlier kernel of the same call,
  // so nothing has to be cleared between calls
  return decode_impl(q, dtype, B, Hq, Hkv, D, ck, kmask, Dkc, cv, vmask, Dvc, M, T, t0, N, k_keep,
                     kk_stride_bh, v_keep, vk_stride_bh, k_full, v_full, W, full_stride_bh, scale,
                     num_splits, out, ws, FA_STATIC_SCRATCH_BYTES, hip_stream, nullptr);
}

int fa_decode_timed(const void* q, int dtype, int B, int Hq, int Hkv, int D, const float* ck,
                    const uint8_t* kmask, int Dkc, const float* cv, const uint8_t* vmask, int Dvc,
                    int M, int T, int t0, int N, const void* k_keep, int64_t kk_stride_bh,
                    const void* v_keep, int64_t vk_stride_bh, const void* k_full,
                    const void* v_full, int W, int64_t full_stride_bh, float scale, int num_splits,
                    float* out, void* workspace, size_t workspace_bytes, void* hip_stream,
                    float* kernel_ms) {
  if (!kernel_ms) return FA_ERR_NULL;
  fa::KernelTimers tm;
  int st = tm.create();
  if (st == FA_OK)
    st = decode_impl(q, dtype, B, Hq, Hkv, D, ck, kmask, Dkc, cv, vmask, Dvc, M, T, t0, N, k_keep,
                     kk_stride_bh, v_keep, vk_stride_bh, k_full, v_full, W, full_stride_bh, scale,
                     num_splits, out, workspace, workspace_bytes, hip_stream, &tm);
  if (st == FA_OK) st = tm.read(3, kernel_ms);
  if (st == FA_OK && hipStreamSynchronize(static_cast<hipStream_t>(hip_stream)) != hipSuccess) st = FA_ERR_HIP;
  tm.destroy();
  return st;
}

}  // extern "C"
