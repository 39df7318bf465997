// fa_append: per-token cache maintenance during decoding (Eq. 5 and the window of Eq. 1).
//
// The recent window is a ring inside the full-width row buffers.  When it is full, the row that
// holds its oldest token is folded into the compressed state before the new token takes it:
//   C[m,i] += phi_m(n_mid) * x[idx_c[i]]     (Eq. 5: one basis column times the evicted row)
//   X_keep[n_mid, :] = x[idx_u]              (kept dims appended at middle position n_mid)
// for K and for V.  Two launches on the caller's stream: the fold reads the old row from many
// workgroups, so the overwrite with the new token has to wait for all of them.

#include "fa_common.hpp"

namespace fa {

constexpr int kABlock = 256;
constexpr int kARows = 32;   // basis rows per workgroup of the fold

struct AppendParams {
  const void* k_new;
  const void* v_new;
  void* k_full;
  void* v_full;
  int64_t full_stride;
  const uint8_t* kmask;
  const uint8_t* vmask;
  float* ck;
  float* cv;
  void* k_keep;
  void* v_keep;
  int64_t kk_stride, vk_stride;
  int B, Hkv, D, W, slot, Dkc, Dvc, M, T, n_mid;
  // per-sequence lists (fa_append_varlen), or null: `slot` / `n_mid` for all
  const int32_t* seq_slot;   // [B] ring row of each sequence; out of [0, W): the sequence is left alone
  const int32_t* seq_nmid;   // [B] middle position of the evicted token; < 0 or >= n_cap: nothing is folded
  int n_cap;                 // tokens the middle slabs have room for
};

// this sequence's ring row and fold position (-1: no fold; slot -1: nothing at all)
__device__ __forceinline__ void seq_append(const AppendParams& p, int b, int* slot, int* n_mid) {
  int s = p.slot, n = p.n_mid;
  if (p.seq_slot) {
    s = p.seq_slot[b];
    if (s < 0 || s >= p.W) s = -1;
  }
  if (p.seq_nmid) {
    n = p.seq_nmid[b];
    if (n < 0 || n >= p.n_cap || n >= p.T || s < 0) n = -1;
  }
  *slot = s;
  *n_mid = n;
}

// grid (row blocks, K | V, sequences x heads)
template <typename T>
__global__ __launch_bounds__(kABlock) void append_fold(AppendParams p) {
  __shared__ float xc[FA_MAX_HEAD_DIM];     // the evicted row at the compressed dims
  __shared__ float phi[kARows];
  const int tid = threadIdx.x, lane = tid & 63;
  const int bh = blockIdx.z, is_v = blockIdx.y, m0 = blockIdx.x * kARows;
  int slot, n_mid;
  seq_append(p, bh / p.Hkv, &slot, &n_mid);
  if (n_mid < 0) return;   // (only with per-sequence lists) this sequence's window is still filling
  const int D = p.D, Dc = is_v ? p.Dvc : p.Dkc, Du = D - Dc;
  const uint8_t* mask = (is_v ? p.vmask : p.kmask) + static_cast<size_t>(bh) * D;
  const T* row = static_cast<const T*>(is_v ? p.v_full : p.k_full) + bh * p.full_stride +
                 static_cast<int64_t>(slot) * D;
  float* C = (is_v ? p.cv : p.ck) + static_cast<size_t>(bh) * p.M * Dc;

  // ranks of the dims: every wave reads the whole mask row
  uint8_t mb[4];
#pragma unroll
  for (int j = 0; j < 4; ++j) mb[j] = mask[min(lane + 64 * j, D - 1)];
  const float xv = (tid < D) ? Elem<T>::load(row + tid) : 0.0f;
  const T xraw = row[min(tid, D - 1)];
  uint64_t bal[4];
#pragma unroll
  for (int j = 0; j < 4; ++j) bal[j] = __ballot(mb[j] != 0 && lane + 64 * j < D);
  if (tid < D) {
    const int w = tid >> 6;
    const uint64_t bit = 1ull << (tid & 63);
    int nc = 0;
    bool hit = false;
#pragma unroll
    for (int j = 0; j < 4; ++j) {   // static indices only: the words stay in registers
      const uint64_t below = (j < w) ? ~0ull : ((j == w) ? (bit - 1ull) : 0ull);
      nc += __popcll(bal[j] & below);
      hit = hit || (j == w && (bal[j] & bit) != 0);
    }
    if (hit) {
      xc[nc] = xv;
    } else if (blockIdx.x == 0) {   // kept dims: appended once, at middle position n_mid
      const int cp = tid - nc;
      if (is_v) {   // [ceil(n/8), Du, 8]
        T* keep = static_cast<T*>(p.v_keep) + bh * p.vk_stride;
        keep[(static_cast<int64_t>(n_mid >> 3) * Du + cp) * 8 + (n_mid & 7)] = xraw;
      } else {      // [n, Du rounded up to 8]
        T* keep = static_cast<T*>(p.k_keep) + bh * p.kk_stride;
        keep[static_cast<int64_t>(n_mid) * ((Du + 7) & ~7) + cp] = xraw;
      }
    }
  }
  if (blockIdx.x == 0 && !is_v && Du > 0) {   // zero pad columns of the new K^mu row
    const int kp = (Du + 7) & ~7;
    T* keep = static_cast<T*>(p.k_keep) + bh * p.kk_stride;
    if (tid < kp - Du) keep[static_cast<int64_t>(n_mid) * kp + Du + tid] = T{};
  }
  if (tid < kARows) {
    const int m = m0 + tid;
    float c = 1.0f, s = 0.0f;
    if (m > 0 && m < p.M) unit_phase((m + 1) / 2, n_mid, p.T, &c, &s);
    phi[tid] = (m & 1) || m == 0 ? c : s;   // odd m: cosine, even m > 0: sine
  }
  __syncthreads();
  const int rows = min(kARows, p.M - m0);
  for (int it = tid; it < rows * Dc; it += kABlock) {
    const int r = it / Dc, i = it - r * Dc;
    float* dst = C + static_cast<size_t>(m0 + r) * Dc + i;
    *dst += phi[r] * xc[i];
  }
}

// the new token takes the ring slot: grid (K | V, sequences x heads)
template <typename T>
__global__ __launch_bounds__(kABlock) void append_store(AppendParams p) {
  const int bh = blockIdx.y, is_v = blockIdx.x, tid = threadIdx.x;
  int slot, n_mid;
  seq_append(p, bh / p.Hkv, &slot, &n_mid);
  if (slot < 0) return;
  const T* src = static_cast<const T*>(is_v ? p.v_new : p.k_new) + static_cast<size_t>(bh) * p.D;
  T* dst = static_cast<T*>(is_v ? p.v_full : p.k_full) + bh * p.full_stride + static_cast<int64_t>(slot) * p.D;
  if (tid < p.D) dst[tid] = src[tid];
}

}  // namespace fa

static int append_impl(const void* k_new, const void* v_new, int dtype, int B, int Hkv, int D,
                       void* k_full, void* v_full, int W, int64_t full_stride_bh, int slot, int evict,
                       const uint8_t* kmask, int Dkc, const uint8_t* vmask, int Dvc, int M, int T,
                       int n_mid, float* ck, float* cv, void* k_keep, int64_t kk_stride_bh,
                       void* v_keep, int64_t vk_stride_bh, void* hip_stream, const int32_t* seq_slot,
                       const int32_t* seq_nmid, int n_cap) {
  using namespace fa;
  if (dtype != FA_F32 && dtype != FA_BF16) return FA_ERR_UNSUPPORTED;
  if (B <= 0 || Hkv <= 0 || D <= 0 || W <= 0 || slot < 0 || slot >= W) return FA_ERR_SHAPE;
  if (D % 8 != 0 || D > FA_MAX_HEAD_DIM || static_cast<long>(B) * Hkv > 65535) return FA_ERR_UNSUPPORTED;
  if (!k_new || !v_new || !k_full || !v_full) return FA_ERR_NULL;
  if (full_stride_bh == 0) full_stride_bh = static_cast<int64_t>(W) * D;
  if (full_stride_bh < static_cast<int64_t>(W) * D) return FA_ERR_SHAPE;
  AppendParams p{};
  p.k_new = k_new; p.v_new = v_new; p.k_full = k_full; p.v_full = v_full;
  p.full_stride = full_stride_bh; p.B = B; p.Hkv = Hkv; p.D = D; p.W = W; p.slot = slot;
  p.seq_slot = seq_slot; p.seq_nmid = seq_nmid; p.n_cap = n_cap; p.T = T;
  hipStream_t st = static_cast<hipStream_t>(hip_stream);
  const hipError_t prior = hipPeekAtLastError();
  if (evict) {
    if (Dkc < 0 || Dkc > D || Dvc < 0 || Dvc > D) return FA_ERR_SHAPE;
    if (M < 1 || T < 1 || M > T || n_mid < 0 || n_mid >= T) return FA_ERR_SHAPE;
    if (M > FA_MAX_STATES) return FA_ERR_UNSUPPORTED;
    if (!kmask || !vmask) return FA_ERR_NULL;
    if ((Dkc > 0 && !ck) || (Dvc > 0 && !cv) || (Dkc < D && !k_keep) || (Dvc < D && !v_keep)) return FA_ERR_NULL;
    // the slabs hold every token that may be written: n_mid + 1 of them, or the stated capacity
    const int64_t tokens = seq_nmid ? n_cap : n_mid + 1;
    const int64_t kk_dense = tokens * ((D - Dkc + 7) & ~7);
    const int64_t vk_dense = (tokens + 7) / 8 * 8 * (D - Dvc);
    if (kk_stride_bh == 0) kk_stride_bh = kk_dense;
    if (vk_stride_bh == 0) vk_stride_bh = vk_dense;
    if (kk_stride_bh < kk_dense || vk_stride_bh < vk_dense) return FA_ERR_SHAPE;
    p.kmask = kmask; p.vmask = vmask; p.ck = ck; p.cv = cv; p.k_keep = k_keep; p.v_keep = v_keep;
    p.kk_stride = kk_stride_bh; p.vk_stride = vk_stride_bh;
    p.Dkc = Dkc; p.Dvc = Dvc; p.M = M; p.n_mid = n_mid;
    const dim3 grid((M + kARows - 1) / kARows, 2, B * Hkv);
    if (dtype == FA_F32) hipLaunchKernelGGL(append_fold<float>, grid, dim3(kABlock), 0, st, p);
    else hipLaunchKernelGGL(append_fold<bf16_t>, grid, dim3(kABlock), 0, st, p);
  } else {
    p.n_mid = -1;
  }
  const dim3 g2(2, B * Hkv);
  if (dtype == FA_F32) hipLaunchKernelGGL(append_store<float>, g2, dim3(kABlock), 0, st, p);
  else hipLaunchKernelGGL(append_store<bf16_t>, g2, dim3(kABlock), 0, st, p);
  // only this call's launches are reported: an error an earlier, unrelated HIP call left behind is
  // neither returned nor cleared
  return (hipPeekAtLastError() == hipSuccess || prior != hipSuccess) ? FA_OK : FA_ERR_HIP;
}

extern "C" int fa_append(const void* k_new, const void* v_new, int dtype, int B, int Hkv, int D,
                         void* k_full, void* v_full, int W, int64_t full_stride_bh, int slot, int evict,
                         const uint8_t* kmask, int Dkc, const uint8_t* vmask, int Dvc, int M, int T,
                         int n_mid, float* ck, float* cv, void* k_keep, int64_t kk_stride_bh,
                         void* v_keep, int64_t vk_stride_bh, void* hip_stream) {
  return append_impl(k_new, v_new, dtype, B, Hkv, D, k_full, v_full, W, full_stride_bh, slot, evict, kmask, Dkc,
                     vmask, Dvc, M, T, n_mid, ck, cv, k_keep, kk_stride_bh, v_keep, vk_stride_bh, hip_stream,
                     nullptr, nullptr, 0);
}

extern "C" int fa_append_varlen(const void* k_new, const void* v_new, int dtype, int B, int Hkv, int D,
                                void* k_full, void* v_full, int W, int64_t full_stride_bh,
                                const int32_t* seq_slot, const uint8_t* kmask, int Dkc, const uint8_t* vmask,
                                int Dvc, int M, int T, const int32_t* seq_nmid, int n_cap, float* ck, float* cv,
                                void* k_keep, int64_t kk_stride_bh, void* v_keep, int64_t vk_stride_bh,
                                void* hip_stream) {
  if (!seq_slot || !seq_nmid) return FA_ERR_NULL;
  if (n_cap < 1 || n_cap > T) return FA_ERR_SHAPE;
  return append_impl(k_new, v_new, dtype, B, Hkv, D, k_full, v_full, W, full_stride_bh, 0, 1, kmask, Dkc, vmask,
                     Dvc, M, T, 0, ck, cv, k_keep, kk_stride_bh, v_keep, vk_stride_bh, hip_stream, seq_slot,
                     seq_nmid, n_cap);
}
