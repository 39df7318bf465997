// fa_decode: fused decode attention over a Fourier-compressed KV cache (Eq. 6).
//
// Three launches on the caller's stream:
//   1. decode_prepare : g[b,hq,m] = w_m * sum_i C_k[m,i] q[idx_kc[i]]
//      (the K-side reconstruction of Eq. 6 commuted with the q.K product:
//       q_c . K~[j, D^kc] = sum_m phi_m(j) g_m);
//   2. decode_partial : one workgroup per (sequence, KV head, token chunk);
//      chunks of the full-width sink/window rows and chunks of the middle rows.
//      Emits a flash-decoding partial (max, sum, acc[D], r[M]) per query head,
//      where r_m = sum_j p_j phi_m(j) carries the V-side series;
//   3. decode_finish  : merges the partials and applies
//      o[idx_vc[i]] += sum_m w_m r_m C_v[m,i]  (V-side reconstruction of Eq. 6
//      commuted with the p.V product), then normalises.
// Reconstructed K~/V~ rows are never formed in memory.

#include "fa_common.hpp"

namespace fa {

constexpr int kBlock = 256;
constexpr int kMaxG = FA_MAX_GROUP;
constexpr int kScoreFloats = 2048;  // LDS floats for scores of one chunk (chunk * G)
constexpr int kRedFloats = 8192;    // LDS floats for cross-slice reductions

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
  int Sw, Sm, chunk_w, chunk_m;
  int rec;  // floats per partial record: 2 + D + M
  float scale;
  float* gq;    // [B,Hq,M]
  float* part;  // [B,Hq,Sw+Sm,rec]
  float* out;   // [B,Hq,D]
};

// rank of every dimension inside its (compressed | kept) list; pos[d] >= 0 is
// the index among kept dims, -(1 + index among compressed dims) otherwise.
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
// 1. g = diag(w) C_k q_c
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
    if (m >= p.M) continue;
    float acc = 0.0f;
    for (int i = 0; i < p.Dkc; ++i) acc += crow[r * ld + i] * qc[h * p.Dkc + i];
    p.gq[(static_cast<size_t>(b) * p.Hq + hkv * p.G + h) * p.M + m] =
        acc * basis_weight((m + 1) / 2, p.T);
  }
}

// ---------------------------------------------------------------------------
// 2. per-chunk partial attention
// ---------------------------------------------------------------------------
template <typename T>
__global__ __launch_bounds__(kBlock) void decode_partial(DecodeParams p) {
  __shared__ float sc[kScoreFloats];
  __shared__ float qs[kMaxG * FA_MAX_HEAD_DIM];
  __shared__ float red[kRedFloats];
  __shared__ float wred[4 * kMaxG];
  __shared__ float mx[kMaxG], lsum[kMaxG];
  __shared__ int16_t kpos[FA_MAX_HEAD_DIM], vpos[FA_MAX_HEAD_DIM];
  __shared__ uint8_t mask_s[FA_MAX_HEAD_DIM];

  const int s = blockIdx.x, bh = blockIdx.y, b = bh / p.Hkv, hkv = bh % p.Hkv;
  const int G = p.G, D = p.D, M = p.M;
  const bool is_w = s < p.Sw;
  const int j0 = is_w ? s * p.chunk_w : (s - p.Sw) * p.chunk_m;
  const int jend = is_w ? min(p.W, j0 + p.chunk_w) : min(p.N, j0 + p.chunk_m);
  const int n = jend - j0;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const size_t hq0 = static_cast<size_t>(b) * p.Hq + hkv * G;

  build_dim_table(p.kmask + static_cast<size_t>(bh) * D, D, kpos, mask_s);
  build_dim_table(p.vmask + static_cast<size_t>(bh) * D, D, vpos, mask_s);

  const int ncol = is_w ? D : p.Dku;
  {
    const T* q = static_cast<const T*>(p.q) + hq0 * D;
    for (int it = tid; it < G * D; it += kBlock) {
      const int h = it / D, d = it % D;
      const float v = Elem<T>::load(q + it);
      if (is_w) qs[h * D + d] = v;
      else if (kpos[d] >= 0) qs[h * D + kpos[d]] = v;
    }
  }
  __syncthreads();

  // ---- pass 1: scores ----------------------------------------------------
  const int n_max = M / 2;  // highest harmonic order present
  for (int jl = tid; jl < n; jl += kBlock) {
    float acc[kMaxG];
#pragma unroll
    for (int h = 0; h < kMaxG; ++h) acc[h] = 0.0f;
    const T* row = is_w ? static_cast<const T*>(p.k_full) + bh * p.full_stride +
                              static_cast<size_t>(j0 + jl) * D
                        : static_cast<const T*>(p.k_keep) + bh * p.kk_stride +
                              static_cast<size_t>(j0 + jl) * p.Dku;
    for (int c = 0; c < ncol; ++c) {
      const float x = Elem<T>::load(row + c);
#pragma unroll
      for (int h = 0; h < kMaxG; ++h)
        if (h < G) acc[h] += x * qs[h * D + c];
    }
    if (!is_w) {
      const int pos = p.t0 + j0 + jl;
      const float* g = p.gq + hq0 * M;
#pragma unroll
      for (int h = 0; h < kMaxG; ++h)
        if (h < G) acc[h] += g[h * M];
      for (int o = 1; o <= n_max; ++o) {
        float c, sn;
        unit_phase(o, pos, p.T, &c, &sn);
        const bool has_sin = 2 * o < M;
#pragma unroll
        for (int h = 0; h < kMaxG; ++h)
          if (h < G) {
            acc[h] += g[h * M + 2 * o - 1] * c;
            if (has_sin) acc[h] += g[h * M + 2 * o] * sn;
          }
      }
    }
#pragma unroll
    for (int h = 0; h < kMaxG; ++h)
      if (h < G) sc[jl * G + h] = acc[h] * p.scale;
  }
  __syncthreads();

  // ---- softmax statistics of the chunk ------------------------------------
  for (int h = 0; h < G; ++h) {
    float m = -INFINITY;
    for (int jl = tid; jl < n; jl += kBlock) m = fmaxf(m, sc[jl * G + h]);
    m = wave_max(m);
    if (lane == 0) wred[wave * kMaxG + h] = m;
  }
  __syncthreads();
  if (tid < G) mx[tid] = fmaxf(fmaxf(wred[tid], wred[kMaxG + tid]),
                               fmaxf(wred[2 * kMaxG + tid], wred[3 * kMaxG + tid]));
  __syncthreads();
  for (int h = 0; h < G; ++h) {
    float l = 0.0f;
    const float m = mx[h];
    for (int jl = tid; jl < n; jl += kBlock) {
      const float e = __expf(sc[jl * G + h] - m);
      sc[jl * G + h] = e;
      l += e;
    }
    l = wave_sum(l);
    if (lane == 0) wred[wave * kMaxG + h] = l;
  }
  __syncthreads();
  if (tid < G) lsum[tid] = wred[tid] + wred[kMaxG + tid] + wred[2 * kMaxG + tid] + wred[3 * kMaxG + tid];
  __syncthreads();

  float* part = p.part + ((hq0) * (p.Sw + p.Sm) + s) * p.rec;
  const size_t part_h = static_cast<size_t>(p.Sw + p.Sm) * p.rec;  // stride between heads
  if (tid < G) {
    part[tid * part_h + 0] = mx[tid];
    part[tid * part_h + 1] = lsum[tid];
  }

  // ---- pass 2: sum_j p_j V[j,:] -------------------------------------------
  const int Dv = is_w ? D : p.Dvu;  // columns streamed from V
  if (Dv > 0) {
    const int nsl = kBlock / Dv;
    const int i = tid % Dv, sl = tid / Dv;
    float acc[kMaxG];
#pragma unroll
    for (int h = 0; h < kMaxG; ++h) acc[h] = 0.0f;
    if (sl < nsl) {
      if (is_w) {
        const T* v = static_cast<const T*>(p.v_full) + bh * p.full_stride +
                     static_cast<size_t>(j0) * D + i;
        for (int j = sl; j < n; j += nsl) {
          const float x = Elem<T>::load(v + static_cast<size_t>(j) * D);
#pragma unroll
          for (int h = 0; h < kMaxG; ++h)
            if (h < G) acc[h] += sc[j * G + h] * x;
        }
      } else {
        // token-interleaved-by-8 layout: [group][dim][8]
        const T* v = static_cast<const T*>(p.v_keep) + bh * p.vk_stride;
        const int g0 = j0 / 8, ng = (n + 7) / 8;
        for (int gi = sl; gi < ng; gi += nsl) {
          const T* grp = v + (static_cast<size_t>(g0 + gi) * Dv + i) * 8;
          for (int e = 0; e < 8; ++e) {
            const int j = gi * 8 + e;
            if (j < n) {
              const float x = Elem<T>::load(grp + e);
#pragma unroll
              for (int h = 0; h < kMaxG; ++h)
                if (h < G) acc[h] += sc[j * G + h] * x;
            }
          }
        }
      }
#pragma unroll
      for (int h = 0; h < kMaxG; ++h)
        if (h < G) red[(sl * Dv + i) * G + h] = acc[h];
    }
    __syncthreads();
    for (int it = tid; it < D * G; it += kBlock) {
      const int d = it % D, h = it / D;
      const int col = is_w ? d : vpos[d];
      float v = 0.0f;
      if (col >= 0)
        for (int k = 0; k < nsl; ++k) v += red[(k * Dv + col) * G + h];
      part[h * part_h + 2 + d] = v;
    }
    __syncthreads();
  } else {
    for (int it = tid; it < D * G; it += kBlock) part[(it / D) * part_h + 2 + (it % D)] = 0.0f;
  }

  // ---- pass 2b: r_m = sum_j p_j phi_m(j) (middle chunks only) ---------------
  if (!is_w) {
    if (tid < G) part[tid * part_h + 2 + D] = lsum[tid];  // constant function
    const int P = n_max;
    if (P > 0) {
      const int Pc = min(P, kBlock);
      const int nsl = kBlock / Pc;
      const int pi = tid % Pc, sl = tid / Pc;
      for (int pb = 0; pb < P; pb += Pc) {
        const int o = 1 + pb + pi;
        float rc[kMaxG], rs[kMaxG];
#pragma unroll
        for (int h = 0; h < kMaxG; ++h) rc[h] = rs[h] = 0.0f;
        if (sl < nsl && o <= P) {
          for (int j = sl; j < n; j += nsl) {
            float c, sn;
            unit_phase(o, p.t0 + j0 + j, p.T, &c, &sn);
#pragma unroll
            for (int h = 0; h < kMaxG; ++h)
              if (h < G) {
                const float pj = sc[j * G + h];
                rc[h] += pj * c;
                rs[h] += pj * sn;
              }
          }
        }
        __syncthreads();
        if (sl < nsl) {
#pragma unroll
          for (int h = 0; h < kMaxG; ++h)
            if (h < G) {
              red[((sl * Pc + pi) * 2 + 0) * G + h] = rc[h];
              red[((sl * Pc + pi) * 2 + 1) * G + h] = rs[h];
            }
        }
        __syncthreads();
        for (int it = tid; it < Pc * 2 * G; it += kBlock) {
          const int h = it % G, cs = (it / G) % 2, q = it / (2 * G);
          const int oo = 1 + pb + q;
          const int m = 2 * oo - 1 + cs;
          if (oo <= P && m < M) {
            float v = 0.0f;
            for (int k = 0; k < nsl; ++k) v += red[((k * Pc + q) * 2 + cs) * G + h];
            part[h * part_h + 2 + D + m] = v;
          }
        }
      }
    }
  }
}

// ---------------------------------------------------------------------------
// 3. merge partials, apply C_v, normalise
// ---------------------------------------------------------------------------
template <typename T>
__global__ __launch_bounds__(kBlock) void decode_finish(DecodeParams p) {
  __shared__ float rr[FA_MAX_STATES];
  __shared__ float accs[FA_MAX_HEAD_DIM];
  __shared__ float stat[2];
  __shared__ int16_t vpos[FA_MAX_HEAD_DIM];
  __shared__ uint8_t mask_s[FA_MAX_HEAD_DIM];

  const int bh = blockIdx.x, b = bh / p.Hkv, hkv = bh % p.Hkv;
  const int D = p.D, M = p.M, S = p.Sw + p.Sm;
  const int tid = threadIdx.x;
  build_dim_table(p.vmask + static_cast<size_t>(bh) * D, D, vpos, mask_s);
  const float* cv = p.cv + static_cast<size_t>(bh) * M * p.Dvc;

  for (int h = 0; h < p.G; ++h) {
    const size_t hq = static_cast<size_t>(b) * p.Hq + hkv * p.G + h;
    const float* part = p.part + hq * S * p.rec;
    if (tid == 0) {
      float m = -INFINITY;
      for (int s = 0; s < S; ++s) m = fmaxf(m, part[static_cast<size_t>(s) * p.rec]);
      float l = 0.0f;
      for (int s = 0; s < S; ++s)
        l += __expf(part[static_cast<size_t>(s) * p.rec] - m) * part[static_cast<size_t>(s) * p.rec + 1];
      stat[0] = l;
      stat[1] = m;
    }
    __syncthreads();
    const float mstar = stat[1];
    for (int d = tid; d < D; d += kBlock) {
      float a = 0.0f;
      for (int s = 0; s < S; ++s) {
        const float* rec = part + static_cast<size_t>(s) * p.rec;
        a += __expf(rec[0] - mstar) * rec[2 + d];
      }
      accs[d] = a;
    }
    for (int m = tid; m < M; m += kBlock) {
      float a = 0.0f;
      for (int s = p.Sw; s < S; ++s) {
        const float* rec = part + static_cast<size_t>(s) * p.rec;
        a += __expf(rec[0] - mstar) * rec[2 + D + m];
      }
      rr[m] = a * basis_weight((m + 1) / 2, p.T);
    }
    __syncthreads();
    const float inv_l = 1.0f / stat[0];
    for (int d = tid; d < D; d += kBlock) {
      float a = accs[d];
      if (vpos[d] < 0 && p.Sm > 0) {
        const int i = -vpos[d] - 1;
        for (int m = 0; m < M; ++m) a += rr[m] * cv[static_cast<size_t>(m) * p.Dvc + i];
      }
      p.out[hq * D + d] = a * inv_l;
    }
    __syncthreads();
  }
}

// ---------------------------------------------------------------------------
// host side
// ---------------------------------------------------------------------------
struct DecodePlan {
  int Sw, Sm, chunk_w, chunk_m, rec;
  size_t off_gq, off_part, total;
};

static int round_up(int x, int a) { return (x + a - 1) / a * a; }

static int default_chunk_m(int B, int Hkv, int N, int G) {
  const int cap = kScoreFloats / (G > 0 ? G : 1) / 64 * 64;  // tokens whose scores fit in LDS
  // aim at >= 512 workgroups over the chip, never more than `cap` tokens each
  long want = (static_cast<long>(N) * B * Hkv + 511) / 512;
  int chunk = round_up(static_cast<int>(want > 64 ? want : 64), 64);
  if (chunk > cap) chunk = cap;
  return chunk;
}

static DecodePlan make_plan(int B, int Hq, int Hkv, int D, int M, int N, int W, int num_splits) {
  DecodePlan pl{};
  const int G = Hq / Hkv;
  const int cap = kScoreFloats / G / 64 * 64;
  pl.chunk_w = 64 < cap ? 64 : cap;
  pl.Sw = (W + pl.chunk_w - 1) / pl.chunk_w;
  if (N > 0) {
    int chunk = default_chunk_m(B, Hkv, N, G);
    if (num_splits > 0) {
      chunk = round_up((N + num_splits - 1) / num_splits, 64);
      if (chunk > cap) chunk = cap;
    }
    pl.chunk_m = chunk;
    pl.Sm = (N + chunk - 1) / chunk;
  } else {
    pl.chunk_m = 64;
    pl.Sm = 0;
  }
  pl.rec = 2 + D + M;
  pl.off_gq = 0;
  pl.off_part = align_up(static_cast<size_t>(B) * Hq * M * sizeof(float), 256);
  pl.total = pl.off_part +
             align_up(static_cast<size_t>(B) * Hq * (pl.Sw + pl.Sm) * pl.rec * sizeof(float), 256);
  return pl;
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
  if (Hq / Hkv > FA_MAX_GROUP || M > FA_MAX_STATES || num_splits > FA_MAX_SPLITS)
    return FA_ERR_UNSUPPORTED;
  return FA_OK;
}

// ev (optional): 4 events recorded before/after each kernel, for fa_decode_timed
template <typename T>
static int launch_decode(const DecodeParams& p, hipStream_t st, hipEvent_t* ev) {
  const int BH = p.B * p.Hkv;
  if (ev) (void)hipEventRecord(ev[0], st);
  if (p.Sm > 0) {
    dim3 g1((p.M + kPrepRows - 1) / kPrepRows, BH);
    hipLaunchKernelGGL(decode_prepare<T>, g1, dim3(kBlock), 0, st, p);
  }
  if (ev) (void)hipEventRecord(ev[1], st);
  dim3 g2(p.Sw + p.Sm, BH);
  hipLaunchKernelGGL(decode_partial<T>, g2, dim3(kBlock), 0, st, p);
  if (ev) (void)hipEventRecord(ev[2], st);
  hipLaunchKernelGGL(decode_finish<T>, dim3(BH), dim3(kBlock), 0, st, p);
  if (ev) (void)hipEventRecord(ev[3], st);
  return hipGetLastError() == hipSuccess ? FA_OK : FA_ERR_HIP;
}

}  // namespace fa

extern "C" {

int fa_decode_default_splits(int B, int Hkv, int N) {
  if (B <= 0 || Hkv <= 0 || N <= 0) return 0;
  const int chunk = fa::default_chunk_m(B, Hkv, N, 1);
  return (N + chunk - 1) / chunk;
}

size_t fa_decode_workspace_bytes(int B, int Hq, int Hkv, int D, int Dkc, int Dvc, int M, int N,
                                 int W, int num_splits) {
  if (fa::check_decode_shapes(FA_BF16, B, Hq, Hkv, D, Dkc, Dvc, M, M > N ? M : N, 0, N, W,
                              num_splits) != FA_OK)
    return 0;
  return fa::make_plan(B, Hq, Hkv, D, M, N, W, num_splits).total;
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

  const DecodePlan pl = make_plan(B, Hq, Hkv, D, M, N, W, num_splits);
  if (workspace_bytes < pl.total || (reinterpret_cast<uintptr_t>(workspace) & 255u))
    return FA_ERR_WORKSPACE;

  DecodeParams p{};
  p.q = q; p.ck = ck; p.cv = cv; p.kmask = kmask; p.vmask = vmask;
  p.k_keep = k_keep; p.v_keep = v_keep; p.k_full = k_full; p.v_full = v_full;
  p.kk_stride = kk_stride_bh; p.vk_stride = vk_stride_bh; p.full_stride = full_stride_bh;
  p.B = B; p.Hq = Hq; p.Hkv = Hkv; p.G = Hq / Hkv; p.D = D;
  p.Dkc = Dkc; p.Dvc = Dvc; p.Dku = Dku; p.Dvu = Dvu;
  p.M = M; p.T = T; p.t0 = t0; p.N = N; p.W = W;
  p.Sw = pl.Sw; p.Sm = pl.Sm; p.chunk_w = pl.chunk_w; p.chunk_m = pl.chunk_m; p.rec = pl.rec;
  p.scale = scale > 0.0f ? scale : 1.0f / sqrtf(static_cast<float>(D));
  p.gq = reinterpret_cast<float*>(static_cast<char*>(workspace) + pl.off_gq);
  p.part = reinterpret_cast<float*>(static_cast<char*>(workspace) + pl.off_part);
  p.out = out;
  hipStream_t stream = static_cast<hipStream_t>(hip_stream);
  return dtype == FA_F32 ? launch_decode<float>(p, stream, ev) : launch_decode<bf16_t>(p, stream, ev);
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
