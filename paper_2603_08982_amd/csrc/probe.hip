// Error probe: estimated compensation error of every (query cluster, key cluster) block.
// Paper: Eq. (7) (value-aware estimate), Eq. (5) (plain estimate), Algorithm 1 (row
// stabiliser m_a = max_b Sbar_ab; streaming over the keys of a cluster without writing
// logits to memory), "Error-Aware Routing" (error-to-size ratio).
//
// One workgroup per (head, key cluster b); lane a of the workgroup owns query centroid a,
// holds qbar_a in registers and streams the cluster's keys once. The squared difference of
// Eq. (7) is expanded around the cluster mean instead of around zero:
//   W vbar - w v_j = (W - w) vbar - w delta_j,   delta_j = v_j - vbar
//   || . ||^2 = (W-w)^2 |vbar|^2 - 2 (W-w) w (vbar.delta_j) + w^2 |delta_j|^2
// so each key contributes O(1) work per query centroid after its logit, and no term
// cancels catastrophically when the cluster is tight. |delta_j|^2 and vbar.delta_j do not
// depend on a and are computed once per key by the whole workgroup.
#include "common.h"

namespace svgear {
namespace {

constexpr int kKeyChunk = 64;
constexpr float kMaxExponent = 40.0f;  // e^40 squared still fits fp32

// Sbar[a][b] = qbar_a . kbar_b * scale; mrow[a] = max over non-empty b.
template <int D>
__global__ void __launch_bounds__(256)
sbar_kernel(const float* __restrict__ qbar, const float* __restrict__ kbar, const int32_t* __restrict__ k_offsets,
            int Cq, int Ck, float scale, float* __restrict__ sbar, float* __restrict__ mrow) {
  __shared__ float q[D];
  __shared__ float red[256];
  const int a = blockIdx.x, bh = blockIdx.y;
  const float* qa = qbar + ((int64_t)bh * Cq + a) * D;
  for (int t = threadIdx.x; t < D; t += 256) q[t] = qa[t];
  __syncthreads();
  const int32_t* off = k_offsets + (int64_t)bh * (Ck + 2);
  float mx = -INFINITY;
  for (int b = threadIdx.x; b < Ck; b += 256) {
    const float4* kb = reinterpret_cast<const float4*>(kbar + ((int64_t)bh * Ck + b) * D);
    float dot = 0.f;
#pragma unroll 8
    for (int t = 0; t < D / 4; ++t) {
      const float4 v = kb[t];
      dot = __builtin_fmaf(q[4 * t], v.x, dot);
      dot = __builtin_fmaf(q[4 * t + 1], v.y, dot);
      dot = __builtin_fmaf(q[4 * t + 2], v.z, dot);
      dot = __builtin_fmaf(q[4 * t + 3], v.w, dot);
    }
    const float s = dot * scale;
    sbar[((int64_t)bh * Cq + a) * Ck + b] = s;
    if (off[b + 1] > off[b]) mx = fmaxf(mx, s);
  }
  red[threadIdx.x] = mx;
  __syncthreads();
  for (int w = 128; w > 0; w >>= 1) {
    if (threadIdx.x < w) red[threadIdx.x] = fmaxf(red[threadIdx.x], red[threadIdx.x + w]);
    __syncthreads();
  }
  if (threadIdx.x == 0) mrow[(int64_t)bh * Cq + a] = red[0];
}

template <typename T, int D, bool VALUE_AWARE>
__global__ void __launch_bounds__(256)
block_error_kernel(const float* __restrict__ qbar, const float* __restrict__ vbar,
                                   const T* __restrict__ kp, const T* __restrict__ vp,
                                   const int32_t* __restrict__ k_offsets, const float* __restrict__ sbar,
                                   const float* __restrict__ mrow, int64_t Nk, int Cq, int Ck, float scale,
                                   float* __restrict__ scores) {
  __shared__ float kf[kKeyChunk][D];  // keys of the chunk, widened to fp32
  __shared__ float nd[kKeyChunk];     // |delta_j|^2
  __shared__ float dd[kKeyChunk];     // vbar . delta_j
  const int b = blockIdx.x, bh = blockIdx.y;
  const int a = blockIdx.z * 256 + threadIdx.x;
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63, nwaves = blockDim.x >> 6;
  const int32_t* off = k_offsets + (int64_t)bh * (Ck + 2);
  const int start = off[b], end = off[b + 1];
  const bool live = a < Cq;
  float* out = scores + ((int64_t)bh * Cq + (live ? a : 0)) * Ck + b;
  if (end <= start) {  // empty key cluster: score 0, never routed nor compensated
    if (live) *out = 0.f;
    return;
  }
  float q[D];
  {
    const float4* qa = reinterpret_cast<const float4*>(qbar + ((int64_t)bh * Cq + (live ? a : 0)) * D);
#pragma unroll
    for (int t = 0; t < D / 4; ++t) {
      const float4 v = qa[t];
      q[4 * t] = v.x; q[4 * t + 1] = v.y; q[4 * t + 2] = v.z; q[4 * t + 3] = v.w;
    }
  }
  const float m_a = live ? mrow[(int64_t)bh * Cq + a] : 0.f;
  const float W = live ? __expf(fminf(sbar[((int64_t)bh * Cq + a) * Ck + b] - m_a, kMaxExponent)) : 0.f;
  constexpr int PER = D / 64;
  const float* vb = vbar + ((int64_t)bh * Ck + b) * D;
  float vbl[PER];
  float nvb = 0.f;
#pragma unroll
  for (int k = 0; k < PER; ++k) vbl[k] = vb[lane * PER + k];
  if (VALUE_AWARE) {
    float part = 0.f;
#pragma unroll
    for (int k = 0; k < PER; ++k) part = __builtin_fmaf(vbl[k], vbl[k], part);
    for (int o = 32; o > 0; o >>= 1) part += __shfl_xor(part, o);
    nvb = part;
  }
  const T* kh = kp + (int64_t)bh * Nk * D;
  const T* vh = vp + (int64_t)bh * Nk * D;
  float E = 0.f;
  for (int j0 = start; j0 < end; j0 += kKeyChunk) {
    const int nk = min(kKeyChunk, end - j0);
    __syncthreads();
    for (int kk = wave; kk < nk; kk += nwaves) {
      const T* kr = kh + (int64_t)(j0 + kk) * D + lane * PER;
#pragma unroll
      for (int k = 0; k < PER; ++k) kf[kk][lane * PER + k] = Elem<T>::load(kr + k);
      if (VALUE_AWARE) {
        const T* vr = vh + (int64_t)(j0 + kk) * D + lane * PER;
        float p_nd = 0.f, p_dd = 0.f;
#pragma unroll
        for (int k = 0; k < PER; ++k) {
          const float dl = Elem<T>::load(vr + k) - vbl[k];
          p_nd = __builtin_fmaf(dl, dl, p_nd);
          p_dd = __builtin_fmaf(dl, vbl[k], p_dd);
        }
        for (int o = 32; o > 0; o >>= 1) {
          p_nd += __shfl_xor(p_nd, o);
          p_dd += __shfl_xor(p_dd, o);
        }
        if (lane == 0) {
          nd[kk] = p_nd;
          dd[kk] = p_dd;
        }
      }
    }
    __syncthreads();
    for (int kk = 0; kk < nk; ++kk) {
      const float4* kr = reinterpret_cast<const float4*>(&kf[kk][0]);
      float dot = 0.f;
#pragma unroll
      for (int t = 0; t < D / 4; ++t) {
        const float4 v = kr[t];
        dot = __builtin_fmaf(q[4 * t], v.x, dot);
        dot = __builtin_fmaf(q[4 * t + 1], v.y, dot);
        dot = __builtin_fmaf(q[4 * t + 2], v.z, dot);
        dot = __builtin_fmaf(q[4 * t + 3], v.w, dot);
      }
      const float w = __expf(fminf(dot * scale - m_a, kMaxExponent));
      const float g = W - w;
      if (VALUE_AWARE) {
        E = __builtin_fmaf(g * g, nvb, E);
        E = __builtin_fmaf(-2.0f * g * w, dd[kk], E);
        E = __builtin_fmaf(w * w, nd[kk], E);
      } else {
        E = __builtin_fmaf(g, g, E);
      }
    }
  }
  if (live) *out = E / (float)(end - start);
}

}  // namespace

int run_probe(const float* qbar, const float* kbar, const float* vbar, const void* kp, const void* vp,
              svgear_dtype dt, const int32_t* k_offsets, int BH, int64_t Nk, int d, int Cq, int Ck, float scale,
              bool value_aware, float* scores, float* sbar, float* mrow, hipStream_t s) {
  if (d == 64)
    sbar_kernel<64><<<dim3(Cq, BH), 256, 0, s>>>(qbar, kbar, k_offsets, Cq, Ck, scale, sbar, mrow);
  else
    sbar_kernel<128><<<dim3(Cq, BH), 256, 0, s>>>(qbar, kbar, k_offsets, Cq, Ck, scale, sbar, mrow);
  SVGEAR_LAUNCH_CHECK();
  const int threads = Cq >= 256 ? 256 : (int)align_up(Cq, 64);
  dim3 grid(Ck, BH, (unsigned)ceil_div(Cq, 256));
#define SVGEAR_PB(T, D, VA)                                                                                   \
  block_error_kernel<T, D, VA><<<grid, threads, 0, s>>>(qbar, vbar, static_cast<const T*>(kp),                \
                                                        static_cast<const T*>(vp), k_offsets, sbar, mrow, Nk, \
                                                        Cq, Ck, scale, scores)
  if (dt == SVGEAR_F32) {
    if (d == 64) { if (value_aware) SVGEAR_PB(float, 64, true); else SVGEAR_PB(float, 64, false); }
    else { if (value_aware) SVGEAR_PB(float, 128, true); else SVGEAR_PB(float, 128, false); }
  } else {
    if (d == 64) { if (value_aware) SVGEAR_PB(bf16_t, 64, true); else SVGEAR_PB(bf16_t, 64, false); }
    else { if (value_aware) SVGEAR_PB(bf16_t, 128, true); else SVGEAR_PB(bf16_t, 128, false); }
  }
#undef SVGEAR_PB
  SVGEAR_LAUNCH_CHECK();
  return SVGEAR_OK;
}

}  // namespace svgear
