// k-means clustering of queries / keys (Lloyd iterations) for every head.
// Paper: Methodology, "Problem Formulation" (Q and K are clustered, a centroid is the mean
// of its cluster); "Linear Compensation" (V is averaged under K's assignment).
//
// Assignment arithmetic (fixed so that labels are reproducible bit for bit):
//   score(c) = fma(-2, dot(x, c), |c|^2), dot and |c|^2 each ONE fp32 fma chain over
//   t = 0..d-1 in index order; argmin with strict '<' scanning c upward (lowest index wins).
// Update: members are brought into cluster order by the stable counting sort, then summed
// in a fixed order (8 interleaved partial sums per cluster, combined 0..7) -- no float
// atomics, so the centroids are run-to-run deterministic.
#include "common.h"

namespace svgear {
namespace {

constexpr int kAssignThreads = 256;
constexpr int kCentChunk = 64;  // centroids staged in LDS per pass

// |c|^2 of every centroid, one chain per centroid.
__global__ void cnorm_kernel(const float* __restrict__ cent, int64_t total, int d, float* __restrict__ cn) {
  const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= total) return;
  const float* c = cent + i * d;
  float acc = 0.f;
  for (int t = 0; t < d; ++t) acc = __builtin_fmaf(c[t], c[t], acc);
  cn[i] = acc;
}

// One thread per row: the row lives in registers, centroids stream through LDS (uniform
// 16-byte reads, broadcast to the wave).
template <typename T, int D>
__global__ void __launch_bounds__(kAssignThreads)
assign_kernel(const T* __restrict__ x, Strides st, int H, int64_t nv, const float* __restrict__ cent,
              const float* __restrict__ cn, int C, int32_t* __restrict__ labels) {
  __shared__ float4 cs[kCentChunk * D / 4];
  __shared__ float cns[kCentChunk];
  const int bh = blockIdx.y;
  const int64_t row = (int64_t)blockIdx.x * kAssignThreads + threadIdx.x;
  const int64_t lrow = row < nv ? row : nv - 1;
  const T* xr = x + head_base(st, bh, H) + lrow * st.n;
  float xv[D];
#pragma unroll
  for (int t = 0; t < D; t += 4) {
    float4 v = load4(xr + t);
    xv[t] = v.x; xv[t + 1] = v.y; xv[t + 2] = v.z; xv[t + 3] = v.w;
  }
  const float* cbase = cent + (int64_t)bh * C * D;
  const float* cnb = cn + (int64_t)bh * C;
  float best = 0.f;
  int arg = 0;
  for (int c0 = 0; c0 < C; c0 += kCentChunk) {
    const int nc = min(kCentChunk, C - c0);
    __syncthreads();
    const float4* src = reinterpret_cast<const float4*>(cbase + (int64_t)c0 * D);
    for (int i = threadIdx.x; i < nc * D / 4; i += kAssignThreads) cs[i] = src[i];
    if (threadIdx.x < nc) cns[threadIdx.x] = cnb[c0 + threadIdx.x];
    __syncthreads();
    for (int c = 0; c < nc; ++c) {
      const float4* cc = cs + c * (D / 4);
      float dot = 0.f;
#pragma unroll
      for (int q = 0; q < D / 4; ++q) {
        const float4 v = cc[q];
        dot = __builtin_fmaf(xv[4 * q], v.x, dot);
        dot = __builtin_fmaf(xv[4 * q + 1], v.y, dot);
        dot = __builtin_fmaf(xv[4 * q + 2], v.z, dot);
        dot = __builtin_fmaf(xv[4 * q + 3], v.w, dot);
      }
      const float score = __builtin_fmaf(-2.0f, dot, cns[c]);
      if ((c0 + c) == 0 || score < best) {
        best = score;
        arg = c0 + c;
      }
    }
  }
  if (row < nv) labels[(int64_t)bh * nv + row] = arg;
}

// Mean of the members of one cluster. 256 threads = 8 member slots x 32 lanes; lane l owns
// dims [l*D/32, (l+1)*D/32). Slot s sums members s, s+8, ... in order; slots are then added
// 0..7 in order.
template <typename T, int D>
__global__ void __launch_bounds__(256)
means_kernel(const T* __restrict__ x, Strides st, int H, const int32_t* __restrict__ perm, int64_t N,
             const int32_t* __restrict__ offsets, int C, float* __restrict__ cent,
             int32_t* __restrict__ counts) {
  constexpr int PER = D / 32;
  __shared__ float red[8][D];
  const int c = blockIdx.x, bh = blockIdx.y;
  const int slot = threadIdx.x >> 5, lane = threadIdx.x & 31;
  const int32_t* off = offsets + (int64_t)bh * (C + 2);
  const int start = off[c], end = off[c + 1];
  const int32_t* pm = perm + (int64_t)bh * N;
  const T* xb = x + head_base(st, bh, H);
  float acc[PER];
#pragma unroll
  for (int k = 0; k < PER; ++k) acc[k] = 0.f;
  for (int m = start + slot; m < end; m += 8) {
    const T* r = xb + (int64_t)pm[m] * st.n + lane * PER;
#pragma unroll
    for (int k = 0; k < PER; ++k) acc[k] += Elem<T>::load(r + k);
  }
#pragma unroll
  for (int k = 0; k < PER; ++k) red[slot][lane * PER + k] = acc[k];
  __syncthreads();
  const int cnt = end - start;
  if (threadIdx.x < D && cnt > 0) {
    float s = red[0][threadIdx.x];
#pragma unroll
    for (int k = 1; k < 8; ++k) s += red[k][threadIdx.x];
    cent[((int64_t)bh * C + c) * D + threadIdx.x] = s / (float)cnt;
  }
  if (threadIdx.x == 0 && counts) counts[(int64_t)bh * C + c] = cnt;
}

template <typename T, int D>
int run_kmeans(const T* x, const T* x2, int BH, int H, int64_t N, int64_t n_tail, Strides st, int C, int iters,
               float* cent, float* cent2, int32_t* labels, int32_t* counts, Workspace& ws, hipStream_t s) {
  const int64_t nv = N - n_tail;
  int32_t* chunk_hist = ws.take<int32_t>((size_t)BH * sort_chunks(nv) * (C + 1));
  int32_t* perm = ws.take<int32_t>((size_t)BH * nv);
  int32_t* offsets = ws.take<int32_t>((size_t)BH * (C + 2));
  float* cn = ws.take<float>((size_t)BH * C);
  if (!ws.ok()) return SVGEAR_ERR_WORKSPACE;
  const int64_t total = (int64_t)BH * C;
  for (int it = 0; it < iters; ++it) {
    cnorm_kernel<<<(unsigned)ceil_div(total, 256), 256, 0, s>>>(cent, total, D, cn);
    SVGEAR_LAUNCH_CHECK();
    dim3 ga((unsigned)ceil_div(nv, kAssignThreads), BH);
    assign_kernel<T, D><<<ga, kAssignThreads, 0, s>>>(x, st, H, nv, cent, cn, C, labels);
    SVGEAR_LAUNCH_CHECK();
    int rc = sort_labels(labels, BH, nv, 0, C, perm, offsets, chunk_hist, s);
    if (rc != SVGEAR_OK) return rc;
    means_kernel<T, D><<<dim3(C, BH), 256, 0, s>>>(x, st, H, perm, nv, offsets, C, cent, counts);
    SVGEAR_LAUNCH_CHECK();
  }
  if (x2) {
    means_kernel<T, D><<<dim3(C, BH), 256, 0, s>>>(x2, st, H, perm, nv, offsets, C, cent2, nullptr);
    SVGEAR_LAUNCH_CHECK();
  }
  return SVGEAR_OK;
}

}  // namespace
}  // namespace svgear

using namespace svgear;

extern "C" size_t svgear_kmeans_workspace(int B, int H, int64_t N, int d, int C) {
  if (B <= 0 || H <= 0 || N <= 0 || C <= 0 || d <= 0) return 0;
  const size_t BH = (size_t)B * H;
  return align_up(BH * sort_chunks(N) * (C + 1) * 4, 256) + align_up(BH * N * 4, 256) +
         align_up(BH * (C + 2) * 4, 256) + align_up(BH * C * 4, 256);
}

extern "C" int svgear_kmeans(const void* x, const void* x2, svgear_dtype dt, int B, int H, int64_t N,
                             int64_t n_tail, int d, const int64_t xstride[3], int C, int iters, float* centroids,
                             float* centroids2, int32_t* labels, int32_t* counts, void* ws, size_t ws_bytes,
                             void* stream) {
  if (!x || !xstride || !centroids || !labels || !counts || B <= 0 || H <= 0 || N <= 0 || n_tail < 0 ||
      n_tail >= N || C <= 0 || C > N - n_tail || C > 8192 || iters < 1 || N > INT32_MAX / 2 ||
      (d != 64 && d != 128) || (dt != SVGEAR_F32 && dt != SVGEAR_BF16) || ((x2 == nullptr) != (centroids2 == nullptr)))
    return SVGEAR_ERR_INVALID;
  const size_t es = esize(dt);
  for (int i = 0; i < 3; ++i)
    if (xstride[i] < 0 || (xstride[i] * (int64_t)es) % 16) return SVGEAR_ERR_INVALID;
  if (reinterpret_cast<uintptr_t>(x) % 16 || reinterpret_cast<uintptr_t>(x2) % 16) return SVGEAR_ERR_INVALID;
  if (!ws || ws_bytes < svgear_kmeans_workspace(B, H, N, d, C)) return SVGEAR_ERR_WORKSPACE;
  Workspace w(ws, ws_bytes);
  hipStream_t s = static_cast<hipStream_t>(stream);
  Strides st{xstride[0], xstride[1], xstride[2]};
  const int BH = B * H;
#define SVGEAR_KM(T, D)                                                                                   \
  return run_kmeans<T, D>(static_cast<const T*>(x), static_cast<const T*>(x2), BH, H, N, n_tail, st, C, iters, \
                          centroids, centroids2, labels, counts, w, s)
  if (dt == SVGEAR_F32) {
    if (d == 64) SVGEAR_KM(float, 64);
    SVGEAR_KM(float, 128);
  } else {
    if (d == 64) SVGEAR_KM(bf16_t, 64);
    SVGEAR_KM(bf16_t, 128);
  }
#undef SVGEAR_KM
}
