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
// Launches on the caller's stream:
//   1. decode_prepare : g (series order) for every query head, from C_k and q.
//   2. decode_partial : one workgroup per (sequence, KV head, token chunk);
//      chunks of full-width sink/window rows and chunks of middle rows; emits
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

typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef _Float16 f16x2 __attribute__((ext_vector_type(2)));
typedef float f32x2 __attribute__((ext_vector_type(2)));

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
  int Sw, Sm;       // chunks of full-width rows / of middle rows
  int chunk_m;      // middle rows per chunk (multiple of the workgroup step)
  int rec;          // floats per partial record: 2 + D + Mint
  unsigned lds_tab; // bytes of the E-table region
  float scale;
  double ph_scale;  // 2^32 / T
  float* gs;        // [B,Hq,Mint] series coefficients, K-side order
  float* g0;        // [B,Hq]      constant-term coefficient
  float* part;      // [B,Hq,Sw+Sm,rec]
  float* out;       // [B,Hq,D]
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

// keep the first `nvalid` (0..8) elements, zero the rest
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

// 8 consecutive elements from global memory; vector load when the address is
// 16-byte aligned, element loads otherwise; elements >= nvalid read as zero.
template <typename T>
__device__ __forceinline__ void load_frag(Frag<T>& f, const T* p, int nvalid, bool vec_ok) {
  if (nvalid <= 0) {
    f.zero();
  } else if (vec_ok && nvalid >= 8) {
    f.load(p);
  } else {
    f.zero();
    for (int e = 0; e < 8; ++e)
      if (e < nvalid) f.set(e, Elem<T>::load(p + e));
  }
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

// rank tables of a dimension mask: pos[d] >= 0 index among kept dims,
// pos[d] < 0: -(1 + index among compressed dims)
__device__ __forceinline__ void build_dim_table(const uint8_t* mask, int D, int16_t* pos,
                                                uint8_t* mask_s) {
  for (int d = threadIdx.x; d < D; d += kBlock) mask_s[d] = mask[d] ? 1 : 0;
  __syncthreads();
  for (int d = threadIdx.x; d < D; d += kBlock) {
    int nc = 0;
    for (int e = 0; e < d; ++e) nc += mask_s[e];
    pos[d] = mask_s[d] ? static_cast<int16_t>(-(1 + nc)) : static_cast<int16_t>(d - nc);
  }
  __syncthreads();
}

// ---------------------------------------------------------------------------
// 1. g = diag(w) C_k q_c, written in series order: slot s <-> basis function s+1
// ---------------------------------------------------------------------------
constexpr int kPrepRows = 32;

template <typename T>
__global__ __launch_bounds__(kBlock) void decode_prepare(DecodeParams p) {
  __shared__ float qc[kMaxG * FA_MAX_HEAD_DIM];
  __shared__ float crow[kPrepRows * (FA_MAX_HEAD_DIM + 1)];
  __shared__ int16_t kpos[FA_MAX_HEAD_DIM];
  __shared__ uint8_t mask_s[FA_MAX_HEAD_DIM];

  const int bh = blockIdx.y, b = bh / p.Hkv, hkv = bh % p.Hkv;
  const int m0 = blockIdx.x * kPrepRows;
  const int ld = p.Dkc + 1;
  build_dim_table(p.kmask + static_cast<size_t>(bh) * p.D, p.D, kpos, mask_s);

  const T* q = static_cast<const T*>(p.q) + (static_cast<size_t>(b) * p.Hq + hkv * p.G) * p.D;
  for (int it = threadIdx.x; it < p.G * p.D; it += kBlock) {
    const int h = it / p.D, d = it % p.D;
    if (kpos[d] < 0) qc[h * p.Dkc + (-kpos[d] - 1)] = Elem<T>::load(q + h * p.D + d);
  }
  const float* ck = p.ck + static_cast<size_t>(bh) * p.M * p.Dkc;
  for (int it = threadIdx.x; it < kPrepRows * p.Dkc; it += kBlock) {
    const int r = it / p.Dkc, i = it % p.Dkc;
    const int m = m0 + r;
    crow[r * ld + i] = (m < p.M) ? ck[static_cast<size_t>(m) * p.Dkc + i] : 0.0f;
  }
  __syncthreads();
  for (int it = threadIdx.x; it < kPrepRows * p.G; it += kBlock) {
    const int r = it % kPrepRows, h = it / kPrepRows;
    const int m = m0 + r;
    if (m > p.Mint) continue;
    float acc = 0.0f;
    if (m < p.M) {
      for (int i = 0; i < p.Dkc; ++i) acc += crow[r * ld + i] * qc[h * p.Dkc + i];
      acc *= basis_weight((m + 1) / 2, p.T);
    }
    const size_t hq = static_cast<size_t>(b) * p.Hq + hkv * p.G + h;
    if (m == 0) p.g0[hq] = acc;
    else p.gs[hq * p.Mint + (m - 1)] = acc;
  }
}

// ---------------------------------------------------------------------------
// 2a. full-width sink/window rows: plain single-query attention partial
// ---------------------------------------------------------------------------
template <typename T>
__device__ __forceinline__ void partial_full_rows(const DecodeParams& p, unsigned char* smem) {
  const int s = blockIdx.x, bh = blockIdx.y, b = bh / p.Hkv, hkv = bh % p.Hkv;
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

  {
    const T* q = static_cast<const T*>(p.q) + hq0 * D;
    for (int it = tid; it < 16 * D; it += kBlock) {
      const int h = it / D;
      qf[it] = (h < G) ? q[it] : T{};
    }
  }
  __syncthreads();

  // scores of 16 rows per wave: A = K rows, B = q (one column per head)
  {
    const int tok = wave * 16 + r16;
    const T* krow = static_cast<const T*>(p.k_full) + bh * p.full_stride +
                    static_cast<int64_t>(j0 + min(tok, n - 1)) * D;
    f32x4 acc = {0.f, 0.f, 0.f, 0.f};
    for (int cc = 0; cc * 32 < D; ++cc) {
      const int d0 = cc * 32 + 8 * q4;
      Frag<T> a, bq;
      load_frag(a, krow + d0, (tok < n) ? D - d0 : 0, true);
      if (d0 < D) bq.load(qf + r16 * D + d0); else bq.zero();
      mma_k32(acc, a, bq);
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
  if (wave == 0) {
    for (int h = 0; h < G; ++h) {
      const float sv = sc[lane * kMaxG + h];
      const float m = wave_max(sv);
      const float e = __expf(sv - m);   // rows >= n hold -inf -> 0
      const float l = wave_sum(e);
      sc[lane * kMaxG + h] = e;
      if (lane == 0) { mx[h] = m; lsum[h] = l; }
    }
  }
  __syncthreads();

  float* part = p.part + (hq0 * (p.Sw + p.Sm) + s) * p.rec;
  const size_t part_h = static_cast<size_t>(p.Sw + p.Sm) * p.rec;
  if (tid < G) {
    part[tid * part_h + 0] = mx[tid];
    part[tid * part_h + 1] = lsum[tid];
  }

  // sum_j p_j V[j,:]: thread owns 8 dims of every nts-th row
  const int nch = D / 8;
  const int nts = kBlock / nch;
  const int dc = tid % nch, ts = tid / nch;
  const bool active = ts < nts;
  constexpr int kMaxRows = 8;   // ceil(64 / nts) <= 8 for D <= 256
  Frag<T> vf[kMaxRows];
  if (active) {
    const T* vb = static_cast<const T*>(p.v_full) + bh * p.full_stride +
                  static_cast<int64_t>(j0) * D + dc * 8;
#pragma unroll
    for (int r = 0; r < kMaxRows; ++r) {
      const int j = ts + r * nts;
      if (j < n) vf[r].load(vb + static_cast<int64_t>(j) * D); else vf[r].zero();
    }
  }
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
        if (j < n) {
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
        for (int k = 0; k < nts; ++k) v += red[(k * 4 + hh) * D + d];
        part[(hg + hh) * part_h + 2 + d] = v;
      }
    }
  }
}

// ---------------------------------------------------------------------------
// 2b. middle rows: kept dims streamed, compressed dims through the series
// ---------------------------------------------------------------------------
template <typename T, int NCH>
__device__ __forceinline__ void partial_middle_rows(const DecodeParams& p, unsigned char* smem) {
  using ES = typename SeriesType<T>::type;
  constexpr int Mint = NCH * 32;
  constexpr int kPitchA = Mint * sizeof(ES) + 16;   // bytes per E_A row
  constexpr int kPitchB = kTJ * sizeof(ES) + 16;    // bytes per E_B row

  const int sm_idx = blockIdx.x - p.Sw, bh = blockIdx.y, b = bh / p.Hkv, hkv = bh % p.Hkv;
  const int G = p.G, Gp = p.Gp, KT = p.KT, D = p.D;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int q4 = lane >> 4, r16 = lane & 15;
  const size_t hq0 = static_cast<size_t>(b) * p.Hq + hkv * G;
  const int c0 = sm_idx * p.chunk_m, c1 = min(p.N, c0 + p.chunk_m);   // chunk of middle rows
  const int wstep = KT * kTJ;                                          // rows per wave step

  // ---- LDS carve-up -------------------------------------------------------
  unsigned char* eA = smem;                                   // [kRB*16][pitchA]
  unsigned char* eB = smem + kTJ * kPitchA;                   // [Mint][pitchB]
  float* red = reinterpret_cast<float*>(smem);                // aliases everything after the loop
  unsigned char* aux = smem + p.lds_tab;
  float* gs_s = reinterpret_cast<float*>(aux);                // [Gp][Mint]
  T* qk_s = reinterpret_cast<T*>(aux + Gp * Mint * 4);        // [Gp][FA_MAX_HEAD_DIM]
  __shared__ float g0_s[kMaxG];
  __shared__ float stat_m[kWaves * 16], stat_l[kWaves * 16], mstar[kMaxG], lstar[kMaxG];
  __shared__ int16_t kpos[FA_MAX_HEAD_DIM], vpos[FA_MAX_HEAD_DIM];
  __shared__ uint8_t mask_s[FA_MAX_HEAD_DIM];

  build_dim_table(p.kmask + static_cast<size_t>(bh) * D, D, kpos, mask_s);
  build_dim_table(p.vmask + static_cast<size_t>(bh) * D, D, vpos, mask_s);

  // q of the kept K dims (zero padded), series coefficients
  for (int it = tid; it < Gp * FA_MAX_HEAD_DIM; it += kBlock) qk_s[it] = T{};
  for (int it = tid; it < Gp * Mint; it += kBlock) {
    const int h = it / Mint, sl = it % Mint;
    gs_s[it] = (h < G && sl < p.Mint) ? p.gs[(hq0 + h) * p.Mint + sl] : 0.0f;
  }
  if (tid < kMaxG) g0_s[tid] = (tid < G) ? p.g0[hq0 + tid] : 0.0f;
  __syncthreads();
  {
    const T* q = static_cast<const T*>(p.q) + hq0 * D;
    for (int it = tid; it < G * D; it += kBlock) {
      const int h = it / D, d = it % D;
      if (kpos[d] >= 0) qk_s[h * FA_MAX_HEAD_DIM + kpos[d]] = q[it];
    }
  }

  // ---- E tables: E[u][slot] = cos/sin(2 pi n u / T), n = slot/2 + 1 ----------
  // E_A rows are stored row-block-major (row 16*rb + i holds u(rb,i)); E_B rows
  // are V-side series indices, columns are u.
  {
    const int n_max = p.M / 2;
    for (int it = tid; it < (Mint / 2) * (kTJ / 8); it += kBlock) {
      const int o = it % (Mint / 2), ug = it / (Mint / 2);
      const int n = o + 1;
      float cs[8], sn[8];
      if (n <= n_max) {
        uint32_t ph = static_cast<uint32_t>((static_cast<uint64_t>(n) * (8 * ug)) % p.T);
        const float invT = 1.0f / static_cast<float>(p.T);
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
          if (ph >= static_cast<uint32_t>(p.T)) ph -= p.T;
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
  __syncthreads();

  // ---- per-lane roles ---------------------------------------------------------
  const int col_k = r16 / Gp, col_h = r16 % Gp;      // S column = (tile, head)
  const bool col_live = col_k < KT && col_h < G;
  const int DVT = (p.Dvu + 15) / 16;
  const int kchunks = (p.Dku + 31) / 32;
  const bool kvec = (p.Dku % 8) == 0;
  const T* kk = static_cast<const T*>(p.k_keep) + bh * p.kk_stride;
  const T* vk = static_cast<const T*>(p.v_keep) + bh * p.vk_stride;

  f32x4 racc[2 * NCH];          // r' = P^T E, frame of the current step
  f32x4 oacc[kMaxDvTiles];      // sum_j p_j V^mu[j,:]
#pragma unroll
  for (int t = 0; t < 2 * NCH; ++t) racc[t] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
  for (int t = 0; t < kMaxDvTiles; ++t) oacc[t] = f32x4{0.f, 0.f, 0.f, 0.f};
  float m_run = -INFINITY, l_run = 0.0f;   // per S column (replicated over q4); l is a per-lane partial
  int last_base = c0;                       // origin of this wave's latest step

  const int stride = kWaves * wstep;
  bool first = true;
  for (int base = c0 + wave * wstep; base < c1; base += stride) {
    // -- (a) kept K dims: A = K^mu rows, B = q masked to the tile's columns ------
    f32x4 sacc[kRB];
#pragma unroll
    for (int rb = 0; rb < kRB; ++rb) sacc[rb] = f32x4{0.f, 0.f, 0.f, 0.f};
    for (int cc = 0; cc < kchunks; ++cc) {
      const int d0 = cc * 32 + 8 * q4;
      Frag<T> bq;
      bq.load(qk_s + col_h * FA_MAX_HEAD_DIM + d0);
      for (int k = 0; k < KT; ++k) {
        Frag<T> bk = bq;
        if (col_k != k) bk.zero();
        Frag<T> a[kRB];
#pragma unroll
        for (int rb = 0; rb < kRB; ++rb) {
          const int u = 32 * (rb >> 1) + 8 * (r16 >> 2) + 4 * (rb & 1) + (r16 & 3);
          const int j = base + k * kTJ + u;
          load_frag(a[rb], kk + static_cast<int64_t>(min(j, p.N - 1)) * p.Dku + d0,
                    (j < c1) ? p.Dku - d0 : 0, kvec);
        }
#pragma unroll
        for (int rb = 0; rb < kRB; ++rb) mma_k32(sacc[rb], a[rb], bk);
      }
    }

    // -- (b) series on the K side: S += E g'(tile origin) --------------------------
    const uint32_t ph_k = phase_of(p.t0 + base + col_k * kTJ, p.ph_scale);
#pragma unroll 2
    for (int c = 0; c < NCH; ++c) {
      float gp[8];
      const float* gsrc = gs_s + col_h * Mint + 32 * c + 8 * q4;
      const int n0 = 16 * c + 4 * q4 + 1;
      uint32_t ph = static_cast<uint32_t>(n0) * ph_k;
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        float cs, sn;
        phase_cs<T>(ph, &cs, &sn);
        ph += ph_k;
        const float gc = gsrc[2 * i], gsn = gsrc[2 * i + 1];
        gp[2 * i] = gc * cs + gsn * sn;
        gp[2 * i + 1] = gsn * cs - gc * sn;
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

    // -- (c) online softmax per column -----------------------------------------------
    // lane (column, q4) holds rows u = 32x + 8*q4 + 4y + v  (rb = 2x + y)
    float sv[kRB][4];
    float m_tile = -INFINITY;
    const float g0 = g0_s[col_h];
#pragma unroll
    for (int rb = 0; rb < kRB; ++rb)
#pragma unroll
      for (int v = 0; v < 4; ++v) {
        const int u = 32 * (rb >> 1) + 8 * q4 + 4 * (rb & 1) + v;
        const int j = base + col_k * kTJ + u;
        const float s = (col_live && j < c1) ? (sacc[rb][v] + g0) * p.scale : -INFINITY;
        sv[rb][v] = s;
        m_tile = fmaxf(m_tile, s);
      }
    m_tile = fmaxf(m_tile, __shfl_xor(m_tile, 16, kWave));
    m_tile = fmaxf(m_tile, __shfl_xor(m_tile, 32, kWave));
    const float m_new = fmaxf(m_run, m_tile);
    const float m_ref = (m_new == -INFINITY) ? 0.0f : m_new;
    const float alpha = __expf(m_run - m_ref);   // m_run = -inf -> 0
    float pv[kRB][4];
    float l_add = 0.0f;
#pragma unroll
    for (int rb = 0; rb < kRB; ++rb)
#pragma unroll
      for (int v = 0; v < 4; ++v) {
        pv[rb][v] = __expf(sv[rb][v] - m_ref);
        l_add += pv[rb][v];
      }
    l_run = l_run * alpha + l_add;
    m_run = m_new;

    // -- (d) bring the accumulators into this step's frame --------------------------------
    if (!first) {
      // accumulator rows are S columns 4*q4 + v: fetch their rescale factors
      float al[4];
#pragma unroll
      for (int v = 0; v < 4; ++v) al[v] = __shfl(alpha, 4 * q4 + v, kWave);
#pragma unroll
      for (int t = 0; t < kMaxDvTiles; ++t)
        if (t < DVT)
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
#pragma unroll
    for (int x = 0; x < kXN; ++x) {
      float pe[8];
#pragma unroll
      for (int e = 0; e < 8; ++e) pe[e] = pv[2 * x + (e >> 2)][e & 3];
      Frag<ES> ps;
      pack8(ps, pe);
#pragma unroll
      for (int t = 0; t < 2 * NCH; ++t) {
        Frag<ES> eb;
        eb.load(reinterpret_cast<const ES*>(eB + (16 * t + r16) * kPitchB) + 32 * x + 8 * q4);
        mma_k32(racc[t], ps, eb);
        // keep the table reads next to their MFMAs: hoisting all of them costs ~4 registers each
        if ((t & 3) == 3) __builtin_amdgcn_sched_barrier(0);
      }
      if (DVT > 0) {
        Frag<T> pt;
        pack8(pt, pe);
        for (int k = 0; k < KT; ++k) {
          Frag<T> ak = pt;
          if (col_k != k) ak.zero();
          const int tok0 = base + k * kTJ + 32 * x + 8 * q4;   // 8 consecutive rows, multiple of 8
#pragma unroll
          for (int dt = 0; dt < kMaxDvTiles; ++dt) {
            if (dt < DVT) {
              const int dim = 16 * dt + r16;
              Frag<T> bv;
              if (dim < p.Dvu && tok0 < c1) {
                bv.load(vk + (static_cast<int64_t>(tok0 >> 3) * p.Dvu + dim) * 8);
                if (tok0 + 8 > c1) mask_tail(bv, c1 - tok0);
              } else {
                bv.zero();
              }
              mma_k32(oacc[dt], ak, bv);
            }
          }
        }
      }
    }
  }

  // ---- merge tiles and waves --------------------------------------------------------------
  l_run += __shfl_xor(l_run, 16, kWave);
  l_run += __shfl_xor(l_run, 32, kWave);
  if (q4 == 0) {
    stat_m[wave * 16 + r16] = col_live ? m_run : -INFINITY;
    stat_l[wave * 16 + r16] = col_live ? l_run : 0.0f;
  }
  __syncthreads();   // also: every wave is done with the E tables and the aux region
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
#pragma unroll
      for (int v = 0; v < 4; ++v) {
        float cs, sn;
        phase_cs<T>(n * phr[v], &cs, &sn);
        const float rc = racc[2 * t][v], rs = racc[2 * t + 1][v];
        const int row = 4 * q4 + v;
        dst[row * redw + 32 * t + r16] = f[v] * (cs * rc - sn * rs);
        dst[row * redw + 32 * t + 16 + r16] = f[v] * (sn * rc + cs * rs);
      }
    }
#pragma unroll
    for (int dt = 0; dt < kMaxDvTiles; ++dt)
      if (dt < DVT)
#pragma unroll
        for (int v = 0; v < 4; ++v)
          dst[(4 * q4 + v) * redw + Mint + 16 * dt + r16] = f[v] * oacc[dt][v];
  }
  __syncthreads();

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
    if (x < D) src = (vpos[x] >= 0) ? Mint + vpos[x] : -1;
    else src = x - D;
    float v = 0.0f;
    if (src >= 0)
      for (int w = 0; w < kWaves; ++w)
        for (int k = 0; k < KT; ++k) v += red[(w * 16 + k * Gp + h) * redw + src];
    part[h * part_h + 2 + x] = v;
  }
}

// Series lengths up to 256 leave room (registers and LDS) for two workgroups per
// compute unit; the 512-long series takes the whole unit.
template <typename T, int NCH>
__global__ __launch_bounds__(kBlock, (NCH <= 8 && sizeof(T) == 2) ? 2 : 1) void decode_partial(DecodeParams p) {
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  if (static_cast<int>(blockIdx.x) < p.Sw) partial_full_rows<T>(p, smem);
  else partial_middle_rows<T, NCH>(p, smem);
}

// ---------------------------------------------------------------------------
// 3. merge partials, apply diag(w) C_v, normalise: one workgroup per query head
// ---------------------------------------------------------------------------
template <typename T>
__global__ __launch_bounds__(kBlock) void decode_finish(DecodeParams p) {
  __shared__ float rr[FA_MAX_DECODE_STATES];   // r in basis order, weighted
  __shared__ float accs[FA_MAX_HEAD_DIM];
  __shared__ float es[kMaxPartials];
  __shared__ float red[kBlock];
  __shared__ float stat[2];
  __shared__ int16_t vpos[FA_MAX_HEAD_DIM];
  __shared__ uint8_t mask_s[FA_MAX_HEAD_DIM];

  const int hq = blockIdx.x, b = hq / p.Hq, hkv = (hq % p.Hq) / p.G;
  const int bh = b * p.Hkv + hkv;
  const int D = p.D, M = p.M, S = p.Sw + p.Sm;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  build_dim_table(p.vmask + static_cast<size_t>(bh) * D, D, vpos, mask_s);
  const float* part = p.part + static_cast<size_t>(hq) * S * p.rec;

  // global max and per-chunk factors
  float m = -INFINITY;
  for (int s = tid; s < S; s += kBlock) m = fmaxf(m, part[static_cast<size_t>(s) * p.rec]);
  m = wave_max(m);
  if (lane == 0) red[wave] = m;
  __syncthreads();
  m = fmaxf(fmaxf(red[0], red[1]), fmaxf(red[2], red[3]));
  float l = 0.0f;
  for (int s = tid; s < S; s += kBlock) {
    const float ms = part[static_cast<size_t>(s) * p.rec];
    const float e = (ms == -INFINITY) ? 0.0f : __expf(ms - m);
    es[s] = e;
    l += e * part[static_cast<size_t>(s) * p.rec + 1];
  }
  l = wave_sum(l);
  __syncthreads();
  if (lane == 0) red[wave] = l;
  __syncthreads();
  if (tid == 0) stat[0] = red[0] + red[1] + red[2] + red[3];
  __syncthreads();

  for (int d = tid; d < D; d += kBlock) {
    float a = 0.0f;
    for (int s = 0; s < S; ++s) a += es[s] * part[static_cast<size_t>(s) * p.rec + 2 + d];
    accs[d] = a;
  }
  // r: merge middle chunks, convert series order -> basis order, apply weights
  for (int m_i = tid; m_i < M; m_i += kBlock) {
    float a = 0.0f;
    if (m_i == 0) {
      // constant function: r_0 = sum of p over the middle rows = their partial sums
      for (int s = p.Sw; s < S; ++s) a += es[s] * part[static_cast<size_t>(s) * p.rec + 1];
    } else {
      const int n = (m_i + 1) / 2, cs = (m_i & 1) ? 0 : 1;   // odd m: cosine
      const int iota = 32 * ((n - 1) >> 4) + 16 * cs + ((n - 1) & 15);
      for (int s = p.Sw; s < S; ++s) a += es[s] * part[static_cast<size_t>(s) * p.rec + 2 + D + iota];
    }
    rr[m_i] = a * basis_weight((m_i + 1) / 2, p.T);
  }
  __syncthreads();

  // o[idx_vc[i]] += sum_m rr[m] C_v[m,i]
  const int Dvc = p.Dvc;
  if (p.Sm > 0 && Dvc > 0) {
    const float* cv = p.cv + static_cast<size_t>(bh) * M * Dvc;
    const int nsl = kBlock / Dvc;   // >= 1 since Dvc <= 256
    const int i = tid % Dvc, sl = tid / Dvc;
    float a = 0.0f;
    if (sl < nsl)
      for (int mm = sl; mm < M; mm += nsl) a += rr[mm] * cv[static_cast<size_t>(mm) * Dvc + i];
    red[tid] = (sl < nsl) ? a : 0.0f;
    __syncthreads();
    for (int d = tid; d < D; d += kBlock) {
      if (vpos[d] < 0) {
        const int ci = -vpos[d] - 1;
        float v = 0.0f;
        for (int k = 0; k < nsl; ++k) v += red[k * Dvc + ci];
        accs[d] += v;
      }
    }
  }
  __syncthreads();
  const float inv_l = 1.0f / stat[0];
  for (int d = tid; d < D; d += kBlock) p.out[static_cast<size_t>(hq) * D + d] = accs[d] * inv_l;
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
  long spc = (total_steps + 256) / 512;   // about two workgroups per compute unit
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

template <typename T, int NCH>
static int launch_partial(const DecodeParams& p, unsigned lds, hipStream_t st) {
  auto kern = decode_partial<T, NCH>;
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
  switch (pl.nch) {
    case 2: rc = launch_partial<T, 2>(p, pl.lds_total, st); break;
    case 4: rc = launch_partial<T, 4>(p, pl.lds_total, st); break;
    case 8: rc = launch_partial<T, 8>(p, pl.lds_total, st); break;
    default:
      if constexpr (sizeof(T) == 2) rc = launch_partial<T, 16>(p, pl.lds_total, st);
      else rc = FA_ERR_UNSUPPORTED;
      break;
  }
  if (rc != FA_OK) return rc;
  if (ev) (void)hipEventRecord(ev[2], st);
  hipLaunchKernelGGL(decode_finish<T>, dim3(p.B * p.Hq), dim3(kBlock), 0, st, p);
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
  const int64_t kk_dense = static_cast<int64_t>(N) * Dku;
  const int64_t vk_dense = static_cast<int64_t>((N + 7) / 8) * 8 * Dvu;
  const int64_t full_dense = static_cast<int64_t>(W) * D;
  if (kk_stride_bh == 0) kk_stride_bh = kk_dense;
  if (vk_stride_bh == 0) vk_stride_bh = vk_dense;
  if (full_stride_bh == 0) full_stride_bh = full_dense;
  if (kk_stride_bh < kk_dense || vk_stride_bh < vk_dense || full_stride_bh < full_dense)
    return FA_ERR_SHAPE;
  // vector loads need 16-byte aligned slabs
  if ((vk_stride_bh % 8) || (full_stride_bh % 8) || (Dku % 8 == 0 && (kk_stride_bh % 8)))
    return FA_ERR_SHAPE;
  if ((reinterpret_cast<uintptr_t>(k_keep) | reinterpret_cast<uintptr_t>(v_keep) |
       reinterpret_cast<uintptr_t>(k_full) | reinterpret_cast<uintptr_t>(v_full) |
       reinterpret_cast<uintptr_t>(q)) & 15u)
    return FA_ERR_SHAPE;

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
