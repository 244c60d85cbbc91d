// k-means clustering of queries / keys (Lloyd iterations) for every head.
// Paper: Methodology, "Problem Formulation" (Q and K are clustered, a centroid is the mean
// of its cluster); "Linear Compensation" (V is averaged under K's assignment).
//
// Assignment arithmetic (fixed so that labels are reproducible bit for bit):
//   score(c) = fma(-2, dot(x, c), |c|^2), dot and |c|^2 each ONE fp32 fma chain over
//   t = 0..d-1 in index order; argmin with strict '<' scanning c upward (lowest index wins).
// The dot products run on the fp32 matrix cores: a chain of v_mfma_f32_32x32x2_f32 over
// k-steps accumulates every (centroid, row) pair in exactly that order (one fused
// multiply-add with one rounding per element of the contraction, k ascending), which was
// checked bit for bit against a scalar fmaf chain on gfx950.
// Update: members are brought into cluster order by the stable counting sort, then summed
// in a fixed order (interleaved partial sums per cluster, combined in slot order) -- no float
// atomics, so the centroids are run-to-run deterministic.
#include "common.h"

namespace svgear {
namespace {

constexpr int kAssignWaves = 8;                 // 32 rows per wave
constexpr int kAssignRows = 32 * kAssignWaves;  // rows per workgroup
constexpr int kCentChunk = 64;                  // centroids per LDS stage (two 32-blocks)

typedef __attribute__((__vector_size__(16 * sizeof(float)))) float f32x16;

// Prepares the centroids of one iteration for the matrix cores:
//  * cn[c] = |c|^2 as ONE fp32 fma chain over t = 0..d-1 (+inf for the padding centroids that
//    round C up to a multiple of 64, so they never win the argmin);
//  * cperm: the centroid table re-laid in MFMA operand order. For v_mfma_f32_32x32x2_f32 the
//    A operand of k-step s is one float per lane: A[i = lane%32][k = 2s + lane/32]. Block
//    blk (32 centroids), group q (4 consecutive k-steps), lane, j hold
//    cent[32 blk + lane%32][2 (4q + j) + lane/32], so a lane fetches the operands of four
//    MFMAs with one 16-byte read and a wave reads 1 KB contiguously.
__global__ void __launch_bounds__(256)
prep_centroids_kernel(const float* __restrict__ cent, int C, int Cpad, int d, float* __restrict__ cperm,
                      float* __restrict__ cn) {
  const int bh = blockIdx.y;
  const float* cb = cent + (int64_t)bh * C * d;
  const int64_t n = (int64_t)Cpad * d;
  for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < n; i += (int64_t)gridDim.x * 256) {
    const int j = (int)(i & 3), lane = (int)((i >> 2) & 63);
    const int64_t rest = i >> 8;  // blk * (d/8) + q
    const int q = (int)(rest % (d / 8)), blk = (int)(rest / (d / 8));
    const int c = 32 * blk + (lane & 31), k = 2 * (4 * q + j) + (lane >> 5);
    cperm[(int64_t)bh * n + i] = c < C ? cb[(int64_t)c * d + k] : 0.f;
  }
  for (int c = blockIdx.x * 256 + threadIdx.x; c < Cpad; c += gridDim.x * 256) {
    float acc = INFINITY;
    if (c < C) {
      acc = 0.f;
      const float* cr = cb + (int64_t)c * d;
      for (int t = 0; t < d; ++t) acc = __builtin_fmaf(cr[t], cr[t], acc);
    }
    cn[(int64_t)bh * Cpad + c] = acc;
  }
}

// 16 bytes per lane from global memory straight into LDS (lane l lands at lds_addr + 16 l).
// Inline assembly keeps the compiler from serialising later LDS reads behind the copy;
// completion is tracked by hand with vmcnt.
__device__ __forceinline__ void async_copy_16B(const void* gptr, uint32_t lds_addr) {
  asm volatile("s_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, off\n"
               :
               : "v"(gptr), "s"(lds_addr)
               : "memory", "m0");
}
#define SVGEAR_WAIT_VMCNT(n) __builtin_amdgcn_s_waitcnt(((n) & 0xF) | (((n) >> 4) << 14) | (7 << 4) | (15 << 8))

// x[row][2s + h] for s = 0..D/2-1 into xb[] (the B operand of k-step s for lane (row, h))
template <int D>
__device__ __forceinline__ void load_row_operands(const float* xr, int h, float (&xb)[D / 2]) {
#pragma unroll
  for (int t = 0; t < D / 4; ++t) {
    const float4 v = *reinterpret_cast<const float4*>(xr + 4 * t);
    xb[2 * t] = h ? v.y : v.x;
    xb[2 * t + 1] = h ? v.w : v.z;
  }
}
template <int D>
__device__ __forceinline__ void load_row_operands(const bf16_t* xr, int h, float (&xb)[D / 2]) {
#pragma unroll
  for (int t = 0; t < D / 8; ++t) {
    const uint4 v = *reinterpret_cast<const uint4*>(xr + 8 * t);
    const uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
    for (int i = 0; i < 4; ++i) xb[4 * t + i] = __uint_as_float(h ? (w[i] & 0xffff0000u) : (w[i] << 16));
  }
}

// Nearest centroid of every row. The score tile is computed transposed (centroids x rows):
// a lane then holds 16 centroids of ONE row per 32x32 block and keeps a private running
// (min, argmin) in ascending centroid order; the two lanes of a row merge once at the end.
// Centroid chunks (64 centroids, in operand order) stream through two LDS stages with
// asynchronous global-to-LDS copies shared by the 8 waves (256 rows) of the workgroup.
template <typename T, int D>
__global__ void __launch_bounds__(64 * kAssignWaves)
assign_mfma_kernel(const T* __restrict__ x, Strides st, int H, int64_t nv, const float* __restrict__ cperm,
                   const float* __restrict__ cn, int Cpad, int32_t* __restrict__ labels) {
  constexpr int QG = D / 8;                        // 16-byte operand groups per block
  constexpr int CHUNK_BYTES = kCentChunk * D * 4;  // one LDS stage of centroids
  constexpr int COPIES = CHUNK_BYTES / 1024 / kAssignWaves;
  static_assert(CHUNK_BYTES % (1024 * kAssignWaves) == 0, "chunk copies must split over the waves");
  extern __shared__ __attribute__((aligned(256))) unsigned char smem[];
  float* cns = reinterpret_cast<float*>(smem + 2 * CHUNK_BYTES);  // [2][kCentChunk]
  const int bh = blockIdx.y;
  const int tid = threadIdx.x, lane = tid & 63, li = lane & 31, lh = lane >> 5;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int64_t row = (int64_t)blockIdx.x * kAssignRows + 32 * wave + li;
  const int64_t lrow = row < nv ? row : nv - 1;
  float xb[D / 2];
  load_row_operands<D>(x + head_base(st, bh, H) + lrow * st.n, lh, xb);
  SVGEAR_WAIT_VMCNT(0);  // rows are in registers before the asynchronous copies start

  const unsigned char* cp = reinterpret_cast<const unsigned char*>(cperm + (int64_t)bh * Cpad * D);
  const float* cnb = cn + (int64_t)bh * Cpad;
  const uint32_t lds0 = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) unsigned char*)smem;
  const int nchunks = Cpad / kCentChunk;
  auto issue_chunk = [&](int ch) {
    const unsigned char* src = cp + (int64_t)ch * CHUNK_BYTES;
    const uint32_t dst = lds0 + (ch & 1) * CHUNK_BYTES;
#pragma unroll
    for (int i = 0; i < COPIES; ++i) {
      const int inst = wave + i * kAssignWaves;
      async_copy_16B(src + inst * 1024 + lane * 16, __builtin_amdgcn_readfirstlane(dst + inst * 1024));
    }
  };

  float best = INFINITY;
  int arg = 0;
  issue_chunk(0);
  if (tid < kCentChunk) cns[tid] = cnb[tid];
  SVGEAR_WAIT_VMCNT(0);
  __syncthreads();
  for (int ch = 0; ch < nchunks; ++ch) {
    float cn_next = 0.f;
    if (ch + 1 < nchunks) {
      issue_chunk(ch + 1);
      if (tid < kCentChunk) cn_next = cnb[(ch + 1) * kCentChunk + tid];
    }
    const unsigned char* cb = smem + (ch & 1) * CHUNK_BYTES + lane * 16;
    const float* cnc = cns + (ch & 1) * kCentChunk;
    f32x16 acc0, acc1;
#pragma unroll
    for (int r = 0; r < 16; ++r) acc0[r] = acc1[r] = 0.f;
#pragma unroll
    for (int q = 0; q < QG; ++q) {
      const float4 a0 = *reinterpret_cast<const float4*>(cb + q * 1024);
      const float4 a1 = *reinterpret_cast<const float4*>(cb + (QG + q) * 1024);
      acc0 = __builtin_amdgcn_mfma_f32_32x32x2f32(a0.x, xb[4 * q + 0], acc0, 0, 0, 0);
      acc1 = __builtin_amdgcn_mfma_f32_32x32x2f32(a1.x, xb[4 * q + 0], acc1, 0, 0, 0);
      acc0 = __builtin_amdgcn_mfma_f32_32x32x2f32(a0.y, xb[4 * q + 1], acc0, 0, 0, 0);
      acc1 = __builtin_amdgcn_mfma_f32_32x32x2f32(a1.y, xb[4 * q + 1], acc1, 0, 0, 0);
      acc0 = __builtin_amdgcn_mfma_f32_32x32x2f32(a0.z, xb[4 * q + 2], acc0, 0, 0, 0);
      acc1 = __builtin_amdgcn_mfma_f32_32x32x2f32(a1.z, xb[4 * q + 2], acc1, 0, 0, 0);
      acc0 = __builtin_amdgcn_mfma_f32_32x32x2f32(a0.w, xb[4 * q + 3], acc0, 0, 0, 0);
      acc1 = __builtin_amdgcn_mfma_f32_32x32x2f32(a1.w, xb[4 * q + 3], acc1, 0, 0, 0);
    }
    // register r of a block is centroid 8(r/4) + 4 lh + r%4 of the block, row li
#pragma unroll
    for (int g = 0; g < 4; ++g) {
      const float4 n4 = *reinterpret_cast<const float4*>(cnc + 8 * g + 4 * lh);
      const float nn[4] = {n4.x, n4.y, n4.z, n4.w};
#pragma unroll
      for (int r = 0; r < 4; ++r) {
        const float score = __builtin_fmaf(-2.0f, acc0[4 * g + r], nn[r]);
        const int idx = ch * kCentChunk + 8 * g + 4 * lh + r;
        if (score < best) { best = score; arg = idx; }
      }
    }
#pragma unroll
    for (int g = 0; g < 4; ++g) {
      const float4 n4 = *reinterpret_cast<const float4*>(cnc + 32 + 8 * g + 4 * lh);
      const float nn[4] = {n4.x, n4.y, n4.z, n4.w};
#pragma unroll
      for (int r = 0; r < 4; ++r) {
        const float score = __builtin_fmaf(-2.0f, acc1[4 * g + r], nn[r]);
        const int idx = ch * kCentChunk + 32 + 8 * g + 4 * lh + r;
        if (score < best) { best = score; arg = idx; }
      }
    }
    if (ch + 1 < nchunks && tid < kCentChunk) cns[((ch + 1) & 1) * kCentChunk + tid] = cn_next;
    SVGEAR_WAIT_VMCNT(0);
    __syncthreads();
  }
  const float ob = __shfl_xor(best, 32);
  const int oa = __shfl_xor(arg, 32);
  if (ob < best || (ob == best && oa < arg)) arg = oa;
  if (lh == 0 && row < nv) labels[(int64_t)bh * nv + row] = arg;
}

// Mean of the members of one cluster. A row is covered by LPR lanes of 16 bytes each; the
// 256 threads form 256/LPR member slots. Slot s sums members s, s+SLOTS, ... in order;
// slots are then added in slot order.
template <typename T, int D>
__global__ void __launch_bounds__(256)
means_kernel(const T* __restrict__ x, Strides st, int H, const int32_t* __restrict__ perm, int64_t N,
             const int32_t* __restrict__ offsets, int C, float* __restrict__ cent,
             int32_t* __restrict__ counts) {
  constexpr int VEC = 16 / sizeof(T);  // elements per lane
  constexpr int LPR = D / VEC;         // lanes per row
  constexpr int SLOTS = 256 / LPR;
  __shared__ float red[SLOTS][D];
  const int c = blockIdx.x, bh = blockIdx.y;
  const int slot = threadIdx.x / LPR, lane = threadIdx.x % LPR;
  const int32_t* off = offsets + (int64_t)bh * (C + 2);
  const int start = off[c], end = off[c + 1];
  const int32_t* pm = perm + (int64_t)bh * N;
  const T* xb = x + head_base(st, bh, H) + lane * VEC;
  float acc[VEC];
#pragma unroll
  for (int k = 0; k < VEC; ++k) acc[k] = 0.f;
  auto add_row = [&](const T* r) {
    if constexpr (sizeof(T) == 4) {
      const float4 v = *reinterpret_cast<const float4*>(r);
      acc[0] += v.x; acc[1] += v.y; acc[2] += v.z; acc[3] += v.w;
    } else {
      const uint4 v = *reinterpret_cast<const uint4*>(r);
      const uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        acc[2 * i] += __uint_as_float(w[i] << 16);
        acc[2 * i + 1] += __uint_as_float(w[i] & 0xffff0000u);
      }
    }
  };
  int m = start + slot;
  for (; m + 3 * SLOTS < end; m += 4 * SLOTS) {  // four independent row fetches in flight
    const T* r0 = xb + (int64_t)pm[m] * st.n;
    const T* r1 = xb + (int64_t)pm[m + SLOTS] * st.n;
    const T* r2 = xb + (int64_t)pm[m + 2 * SLOTS] * st.n;
    const T* r3 = xb + (int64_t)pm[m + 3 * SLOTS] * st.n;
    add_row(r0); add_row(r1); add_row(r2); add_row(r3);
  }
  for (; m < end; m += SLOTS) add_row(xb + (int64_t)pm[m] * st.n);
#pragma unroll
  for (int k = 0; k < VEC; ++k) red[slot][lane * VEC + k] = acc[k];
  __syncthreads();
  const int cnt = end - start;
  if (threadIdx.x < D && cnt > 0) {
    float s = red[0][threadIdx.x];
#pragma unroll
    for (int k = 1; k < SLOTS; ++k) s += red[k][threadIdx.x];
    cent[((int64_t)bh * C + c) * D + threadIdx.x] = s / (float)cnt;
  }
  if (threadIdx.x == 0 && counts) counts[(int64_t)bh * C + c] = cnt;
}

template <typename T, int D>
int run_kmeans(const T* x, const T* x2, int BH, int H, int64_t N, int64_t n_tail, Strides st, int C, int iters,
               float* cent, float* cent2, int32_t* labels, int32_t* counts, Workspace& ws, hipStream_t s) {
  const int64_t nv = N - n_tail;
  const int Cpad = (int)align_up(C, kCentChunk);
  int32_t* chunk_hist = ws.take<int32_t>((size_t)BH * sort_chunks(nv) * (C + 1));
  int32_t* perm = ws.take<int32_t>((size_t)BH * nv);
  int32_t* offsets = ws.take<int32_t>((size_t)BH * (C + 2));
  float* cn = ws.take<float>((size_t)BH * Cpad);
  float* cperm = ws.take<float>((size_t)BH * Cpad * D);
  if (!ws.ok()) return SVGEAR_ERR_WORKSPACE;
  const size_t lds = 2 * (size_t)kCentChunk * D * 4 + 2 * kCentChunk * sizeof(float);
  auto assign = assign_mfma_kernel<T, D>;
  SVGEAR_HIP_TRY(hipFuncSetAttribute(reinterpret_cast<const void*>(assign),
                                     hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));
  const dim3 gp((unsigned)ceil_div((int64_t)Cpad * D, 256 * 4), BH);
  const dim3 ga((unsigned)ceil_div(nv, kAssignRows), BH);
  for (int it = 0; it < iters; ++it) {
    prep_centroids_kernel<<<gp, 256, 0, s>>>(cent, C, Cpad, D, cperm, cn);
    SVGEAR_LAUNCH_CHECK();
    assign<<<ga, 64 * kAssignWaves, lds, s>>>(x, st, H, nv, cperm, cn, Cpad, labels);
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
  const size_t Cpad = align_up(C, kCentChunk);
  return align_up(BH * sort_chunks(N) * (C + 1) * 4, 256) + align_up(BH * N * 4, 256) +
         align_up(BH * (C + 2) * 4, 256) + align_up(BH * Cpad * 4, 256) + align_up(BH * Cpad * d * 4, 256);
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
