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
// For bf16 inputs a cheap FILTER runs first: the same scores from bf16 MFMAs (the centroid
// split exactly into two bf16 pieces plus a residual below 2^-16), with the best and the
// second-best score tracked per row. A row whose margin exceeds a rigorous bound on
// |filter score - fixed-order score| keeps the filter's label (the fixed-order argmin is
// provably the same); the few remaining rows are re-assigned by the fp32 kernel, so the
// labels are always those of the fixed-order definition.
// From the second iteration on only the rows whose distance bounds (Hamerly's: one upper, one
// lower bound per row, widened by the centroids' moves) do not prove that the fixed-order label
// stays are assigned again; with many centroids each such row is tested only against the
// centroids near its cluster (lists built from centroid-to-centroid distances, with the same
// kind of proof). Neither changes a label.
// Update: members are brought into cluster order by the stable counting sort, then summed
// in a fixed order (interleaved partial sums per cluster, combined in slot order) -- no float
// atomics, so the centroids are run-to-run deterministic.
#include <atomic>

#include "common.h"

namespace svgear {
namespace {

constexpr int kAssignWaves = 8;                 // 32 rows per wave
constexpr int kAssignRows = 32 * kAssignWaves;  // rows per workgroup
constexpr int kCentChunk = 64;                  // centroids per LDS stage (two 32-blocks)
// per head: [0] rows queued for assign_filter_kernel; as float bits: [1] max |x| of the flagged rows, [2] max |c|^2
constexpr int kHeadState = 4;
constexpr int kListMax = 128;                   // longest candidate list of a cluster (longer: every centroid)
constexpr int kListTile = 64;                   // sorted positions per step of a wave of assign_list_kernel
constexpr int kListChunk = 4 * kListTile;       // sorted positions per wave (one cluster's)
constexpr int kMaxCentroids = 8192;             // most centroids per head the entry point accepts
// Candidate lists pay when there are many centroids: with fewer than this, testing every
// centroid (shared through LDS by 256 rows, streaming) costs no more than the lists' gathers.
std::atomic<int> g_list_min_centroids{400};
// (in the second iteration of a cold start the radii still reach every centroid, so no cluster gets
// a list: the lists start one iteration later)
#ifndef SVGEAR_LIST_FROM
#define SVGEAR_LIST_FROM 2
#endif
constexpr int kListFromIteration = SVGEAR_LIST_FROM;

typedef __attribute__((__vector_size__(16 * sizeof(float)))) float f32x16;

// Prepares the centroids of one iteration for the matrix cores:
//  * cn[c] = |c|^2 as ONE fp32 fma chain over t = 0..d-1 (+inf for the padding centroids that
//    round C up to a multiple of 64, so they never win the argmin);
//  * cperm: the centroid table re-laid in MFMA operand order. For v_mfma_f32_32x32x2_f32 the
//    A operand of k-step s is one float per lane: A[i = lane%32][k = 2s + lane/32]. Block
//    blk (32 centroids), group q (4 consecutive k-steps), lane, j hold
//    cent[32 blk + lane%32][2 (4q + j) + lane/32], so a lane fetches the operands of four
//    MFMAs with one 16-byte read and a wave reads 1 KB contiguously.
//  * chl (optional): the bf16 split c = hi + lo + residual, hi = bf16(c), lo = bf16(c - hi), in
//    the operand order of v_mfma_f32_32x32x16_bf16 (A[i = lane%32][k = 16s + 8(lane/32) + e]):
//    [blk][piece][s][lane][e], 16 bytes per lane; crow (with chl): the same two pieces row by row,
//    [c][piece][d], for the kernel that fetches single centroids;
//  * amb_count, head_state, rmax (optional): the per-iteration counters and maxima are reset.
__global__ void __launch_bounds__(256)
prep_centroids_kernel(const float* __restrict__ cent, int C, int Cpad, int d, float* __restrict__ cperm,
                      float* __restrict__ cn, bf16_t* __restrict__ chl, bf16_t* __restrict__ crow,
                      int32_t* __restrict__ amb_count, int32_t* __restrict__ head_state, int32_t* __restrict__ rmax,
                      int32_t* __restrict__ dirty) {
  const int bh = blockIdx.y;
  const float* cb = cent + (int64_t)bh * C * d;
  const int64_t n = (int64_t)Cpad * d;
  if (amb_count && blockIdx.x == 0 && threadIdx.x == 0) amb_count[bh] = 0;
  if (head_state && blockIdx.x == 0 && threadIdx.x < kHeadState) head_state[bh * kHeadState + threadIdx.x] = 0;
  // both operand tables are written 16 bytes per thread from 32 contiguous bytes of a centroid row
  if (chl) {
    const int ksn = d / 16;
    for (int64_t u = (int64_t)blockIdx.x * 256 + threadIdx.x; u < n / 8; u += (int64_t)gridDim.x * 256) {
      const int lane = (int)(u & 63);
      const int64_t rest = u >> 6;  // blk * ksn + s
      const int sidx = (int)(rest % ksn), blk = (int)(rest / ksn);
      const int c = 32 * blk + (lane & 31), k0 = 16 * sidx + 8 * (lane >> 5);
      float v[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
      if (c < C) {
        const float4* src = reinterpret_cast<const float4*>(cb + (int64_t)c * d + k0);
        const float4 v0 = src[0], v1 = src[1];
        v[0] = v0.x; v[1] = v0.y; v[2] = v0.z; v[3] = v0.w;
        v[4] = v1.x; v[5] = v1.y; v[6] = v1.z; v[7] = v1.w;
      }
      uint32_t hw[4], lw[4];
#pragma unroll
      for (int e = 0; e < 8; e += 2) {
        const bf16_t h0 = f32_to_bf16(v[e]), h1 = f32_to_bf16(v[e + 1]);
        const bf16_t l0 = f32_to_bf16(v[e] - bf16_to_f32(h0)), l1 = f32_to_bf16(v[e + 1] - bf16_to_f32(h1));
        hw[e >> 1] = (uint32_t)h0 | ((uint32_t)h1 << 16);
        lw[e >> 1] = (uint32_t)l0 | ((uint32_t)l1 << 16);
      }
      const int64_t base = (int64_t)bh * 2 * n + (((int64_t)blk * 2) * ksn + sidx) * 512 + lane * 8;
      *reinterpret_cast<uint4*>(chl + base) = uint4{hw[0], hw[1], hw[2], hw[3]};
      *reinterpret_cast<uint4*>(chl + base + (int64_t)ksn * 512) = uint4{lw[0], lw[1], lw[2], lw[3]};
      const int64_t rbase = (int64_t)bh * 2 * n + (int64_t)c * 2 * d + k0;
      *reinterpret_cast<uint4*>(crow + rbase) = uint4{hw[0], hw[1], hw[2], hw[3]};
      *reinterpret_cast<uint4*>(crow + rbase + d) = uint4{lw[0], lw[1], lw[2], lw[3]};
    }
  }
  for (int64_t u = (int64_t)blockIdx.x * 256 + threadIdx.x; u < n / 4; u += (int64_t)gridDim.x * 256) {
    const int lane = (int)(u & 63);
    const int64_t rest = u >> 6;  // blk * (d/8) + q
    const int q = (int)(rest % (d / 8)), blk = (int)(rest / (d / 8));
    const int c = 32 * blk + (lane & 31), h = lane >> 5;
    float4 out = make_float4(0.f, 0.f, 0.f, 0.f);
    if (c < C) {  // dims 8q + 2j + h, j = 0..3
      const float4* src = reinterpret_cast<const float4*>(cb + (int64_t)c * d + 8 * q);
      const float4 v0 = src[0], v1 = src[1];
      out = h ? make_float4(v0.y, v0.w, v1.y, v1.w) : make_float4(v0.x, v0.z, v1.x, v1.z);
    }
    *reinterpret_cast<float4*>(cperm + (int64_t)bh * n + u * 4) = out;
  }
  for (int c = blockIdx.x * 256 + threadIdx.x; c < Cpad; c += gridDim.x * 256) {
    if (dirty) dirty[(int64_t)bh * Cpad + c] = 0;  // no cluster has gained or lost a member yet
    if (rmax) rmax[(int64_t)bh * Cpad + c] = 0;    // nor has any of its rows been flagged
    float acc = INFINITY;
    if (c < C) {
      acc = 0.f;
      const float4* cr = reinterpret_cast<const float4*>(cb + (int64_t)c * d);
      for (int t0 = 0; t0 < d / 4; t0 += 8) {  // 8 independent 16-byte loads, then the chain in order
        float4 v[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) v[u] = cr[t0 + u];
#pragma unroll
        for (int u = 0; u < 8; ++u) {
          acc = __builtin_fmaf(v[u].x, v[u].x, acc);
          acc = __builtin_fmaf(v[u].y, v[u].y, acc);
          acc = __builtin_fmaf(v[u].z, v[u].z, acc);
          acc = __builtin_fmaf(v[u].w, v[u].w, acc);
        }
      }
    }
    cn[(int64_t)bh * Cpad + c] = acc;
  }
}


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
// (Every row of fp32 inputs goes through this kernel; of bf16 inputs only the rows the filter
// below cannot decide, through assign_few_kernel.)
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
  const int64_t pos = (int64_t)blockIdx.x * kAssignRows + 32 * wave + li;
  const int64_t row = pos < nv ? pos : nv - 1;
  float xb[D / 2];
  load_row_operands<D>(x + head_base(st, bh, H) + row * st.n, lh, xb);
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
  if (lh == 0 && pos < nv) labels[(int64_t)bh * nv + row] = arg;
}

// The same assignment for a short list of rows (the filter's ambiguous ones): with few rows
// the kernel above leaves most of the chip idle while each of its waves walks every centroid, so
// here the centroids of a 32-row tile are dealt to the 4 waves of the workgroup (32-blocks
// round-robin), every wave fetches its operand fragments straight from the table (1 KB
// contiguous per fetch; no LDS stage, no barrier inside the walk), and the four partial
// (min, argmin) meet in LDS at the end. Every score is the same chain of matrix-core
// instructions as above, and ties still go to the lowest index.
template <typename T, int D>
__global__ void __launch_bounds__(256)
assign_few_kernel(const T* __restrict__ x, Strides st, int H, int64_t nv, const float* __restrict__ cperm,
                  const float* __restrict__ cn, int Cpad, int32_t* __restrict__ labels,
                  const int32_t* __restrict__ row_list, const int32_t* __restrict__ row_count,
                  int32_t* __restrict__ dirty) {
  constexpr int QG = D / 8;  // 16-byte operand groups per 32-block
  __shared__ float s_best[4][32];
  __shared__ int s_arg[4][32];
  const int bh = blockIdx.y;
  const int tid = threadIdx.x, lane = tid & 63, li = lane & 31, lh = lane >> 5;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int64_t n_rows = row_count[bh];
  const float* cp = cperm + (int64_t)bh * Cpad * D;
  const float* cnb = cn + (int64_t)bh * Cpad;
  for (int64_t tile = blockIdx.x; tile * 32 < n_rows; tile += gridDim.x) {
    const int64_t pos = tile * 32 + li;
    const int64_t row = row_list[(int64_t)bh * nv + (pos < n_rows ? pos : n_rows - 1)];
    float xb[D / 2];
    load_row_operands<D>(x + head_base(st, bh, H) + row * st.n, lh, xb);
    float best = INFINITY;
    int arg = 0;
    for (int blk = wave; blk < Cpad / 32; blk += 4) {
      const float* cb = cp + (int64_t)blk * 32 * D + lane * 4;
      f32x16 acc;
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[r] = 0.f;
#pragma unroll
      for (int q0 = 0; q0 < QG; q0 += 8) {  // 8 fetches in flight, then their 32 MFMAs in k order
        float4 a[8];
#pragma unroll
        for (int q = 0; q < 8; ++q) a[q] = *reinterpret_cast<const float4*>(cb + (q0 + q) * 256);
#pragma unroll
        for (int q = 0; q < 8; ++q) {
          acc = __builtin_amdgcn_mfma_f32_32x32x2f32(a[q].x, xb[4 * (q0 + q) + 0], acc, 0, 0, 0);
          acc = __builtin_amdgcn_mfma_f32_32x32x2f32(a[q].y, xb[4 * (q0 + q) + 1], acc, 0, 0, 0);
          acc = __builtin_amdgcn_mfma_f32_32x32x2f32(a[q].z, xb[4 * (q0 + q) + 2], acc, 0, 0, 0);
          acc = __builtin_amdgcn_mfma_f32_32x32x2f32(a[q].w, xb[4 * (q0 + q) + 3], acc, 0, 0, 0);
        }
      }
      // register r is centroid 32 blk + 8(r/4) + 4 lh + r%4, row li
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        const float4 n4 = *reinterpret_cast<const float4*>(cnb + 32 * blk + 8 * g + 4 * lh);
        const float nn[4] = {n4.x, n4.y, n4.z, n4.w};
#pragma unroll
        for (int r = 0; r < 4; ++r) {
          const float score = __builtin_fmaf(-2.0f, acc[4 * g + r], nn[r]);
          const int idx = 32 * blk + 8 * g + 4 * lh + r;
          if (score < best) { best = score; arg = idx; }
        }
      }
    }
    const float ob = __shfl_xor(best, 32);
    const int oa = __shfl_xor(arg, 32);
    if (ob < best || (ob == best && oa < arg)) { best = ob; arg = oa; }
    if (lh == 0) {
      s_best[wave][li] = best;
      s_arg[wave][li] = arg;
    }
    __syncthreads();
    if (wave == 0 && lh == 0 && pos < n_rows) {
#pragma unroll
      for (int w = 1; w < 4; ++w) {
        const float wb = s_best[w][li];
        const int wa = s_arg[w][li];
        if (wb < best || (wb == best && wa < arg)) { best = wb; arg = wa; }
      }
      if (dirty) {  // a row that moves marks the cluster it leaves and the one it joins
        const int cur = labels[(int64_t)bh * nv + row];
        if (cur != arg) {
          dirty[(int64_t)bh * Cpad + cur] = 1;
          dirty[(int64_t)bh * Cpad + arg] = 1;
        }
      }
      labels[(int64_t)bh * nv + row] = arg;
    }
    __syncthreads();  // the LDS slots are written again by the next tile
  }
}

// ---- bf16 filter -----------------------------------------------------------------------
typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
__device__ __forceinline__ bf16x8 as_bf16x8(uint4 v) {
  union { uint4 u; bf16x8 b; } c;
  c.u = v;
  return c.b;
}

// 4 waves x 64 rows per workgroup: two workgroups share a CU (registers allow two waves per
// SIMD either way), so one's set-up - row loads, |c|^2 table, first centroid chunk - overlaps
// the other's steady state (measured 6 % faster than one 8-wave workgroup per CU)
constexpr int kFilterWaves = 4;
// waves that issue the centroid chunk copies (all of them when the 32 copies split evenly)
constexpr int kFilterCopyWaves = 32 % kFilterWaves == 0 ? kFilterWaves : 4;
constexpr int kFilterRowsPerWave = 64;  // two 32-row operand sets share every centroid fragment
constexpr int kFilterRows = kFilterWaves * kFilterRowsPerWave;
constexpr int kFilterGroups = 8;  // row groups per workgroup when every centroid fits the two LDS stages

// Distance of a fixed-order fp32 score fma(-2, x.c, |c|^2) (both sums fmaf chains over d
// terms) from the real number |c|^2 - 2 x.c, for |x| <= X and |c| <= Cm: d 2^-24 relative on
// each chain plus the final rounding, with head room.
template <int D>
__device__ __forceinline__ float fixed_order_error(float X, float Cm) {
  return (D + 2) * 5.9604644775390625e-08f * 1.001f * (Cm * Cm + 2.0f * X * Cm);
}

// Per-row state between iterations: bnd[row] = (ub, lb), an upper bound of the row's distance
// to its centroid and a lower bound of its distance to every other centroid; xnorm[row] = |x|_2
// rounded up.
//
// What a filter kernel does with a row once its lanes have ranked the centroids they tested:
// (best, second, arg) are the lowest and second-lowest approximate score and the position of the
// lowest seen by THIS lane; the two lanes of a row (lane, lane ^ 32) each saw half of the
// centroids of every 32-block and are merged here. `positions` (optional) maps a position in the
// tested list to a centroid index. far_lb: a lower bound of the row's distance to every centroid
// that was not tested (+inf if all were). cur: the row's present label if the caller knows it
// (-1: read it). Writes the label if it changes, queues the row for the exact kernel if the
// margin does not exceed the bound B on the filter's error (see assign_filter_kernel), flags the
// clusters the row leaves and joins, and stores the row's bounds for the next iterations: with F
// the distance of a filter score from the real |c|^2 - 2 x.c, the assigned centroid is at most
// sqrt(best + F + |x|^2) away and every other one at least sqrt(second - F + |x|^2) (tested) or
// far_lb (not tested). A row whose label the exact kernel decides gets no lower bound (it is
// assigned again next iteration).
template <int D>
__device__ __forceinline__ void settle_row(float best, float second, int arg, bool valid, int64_t row, float X,
                                           float Cm, float far_lb, const int32_t* __restrict__ positions, int cur,
                                           int bh, int64_t nv, int Cpad, int32_t* __restrict__ labels,
                                           int32_t* __restrict__ amb_rows, int32_t* __restrict__ amb_count,
                                           float2* __restrict__ bnd, int32_t* __restrict__ dirty) {
  constexpr float kappa = 1.52587890625e-05f + (2 * D + 1) * 1.1920928955078125e-07f + D * 5.9604644775390625e-08f;
  const int lane = threadIdx.x & 63, lh = lane >> 5;
  const float ob = __shfl_xor(best, 32), os = __shfl_xor(second, 32);
  const int oa = __shfl_xor(arg, 32);
  const float lo = fminf(best, ob), hi = fmaxf(best, ob);
  const float sec = fminf(hi, fminf(second, os));
  int a = (ob < best || (ob == best && oa < arg)) ? oa : arg;
  if (lh == 0 && valid) {
    if (positions) a = positions[a];
    const float B = 2.0f * X * Cm * kappa + 1.1920928955078125e-07f * (Cm * Cm + 2.0f * X * Cm);
    if (dirty) {  // a row that moves marks the cluster it leaves and the one it joins
      if (cur < 0) cur = labels[(int64_t)bh * nv + row];
      if (cur != a) {
        dirty[(int64_t)bh * Cpad + cur] = 1;
        dirty[(int64_t)bh * Cpad + a] = 1;
      }
    }
    if (cur != a) labels[(int64_t)bh * nv + row] = a;
    const bool ambiguous = !(sec - lo > 2.0f * B * 1.0001f);  // also catches NaN / inf margins
    if (ambiguous) {
      // one counter update for the ambiguous rows of the wave (the active lanes here)
      const unsigned long long am = __ballot(1);
      const int leader = __ffsll((long long)am) - 1;
      int slot = 0;
      if (lane == leader) slot = atomicAdd(&amb_count[bh], __popcll(am));
      slot = __shfl(slot, leader) + __popcll(am & ((1ull << lane) - 1ull));
      amb_rows[(int64_t)bh * nv + slot] = (int32_t)row;
    }
    if (bnd) {
      const float F = B + fixed_order_error<D>(X, Cm);
      const float x2_hi = X * X, x2_lo = X * X * 0.9999f;
      const float u2 = lo + (ambiguous ? 2.0002f * B : 0.f) + F + x2_hi;
      const float l2 = sec - F + x2_lo;
      float lbv = (ambiguous || !(l2 > 0.f)) ? 0.f : sqrtf(l2) * 0.999999f;
      lbv = fminf(lbv, fmaxf(far_lb, 0.f));
      bnd[(int64_t)bh * nv + row] = make_float2(sqrtf(fmaxf(u2, 0.f)) * 1.000001f, lbv);
    }
  }
}

// Approximate scores s~(c) = fma(-2, x.hi_c + x.lo_c, |c|^2) on bf16 MFMAs, with the best and
// second-best kept per row. With X = |x|_2, Cm = max_c |c|_2 and d the head dimension,
//   |x.c(filter) - x.c(fixed order)| <= X Cm (2^-16 + (2d+1) 2^-23 + d 2^-24) =: X Cm kappa
// (split residual below 2^-16 |c| per element; every fp32 addition inside the matrix core
// charged 2^-23 relative, twice the round-to-nearest unit, over 2d+1 terms in any order; the
// fixed-order chain charged the usual d 2^-24), the two final fmas add 2^-23 (Cm^2 + 2 X Cm),
// so two scores differ from their fixed-order values by at most
//   B = 2 X Cm kappa + 2^-23 (Cm^2 + 2 X Cm).
// If second - best > 2B the fixed-order argmin is the filter's argmin; otherwise the row is
// queued for the exact kernel. With row_list != nullptr only the rows listed there
// (row_count[kHeadState bh] of them, in any order) are assigned.
template <int D, bool RESIDENT>
__global__ void __launch_bounds__(64 * kFilterWaves) __attribute__((amdgpu_waves_per_eu(2)))
assign_filter_kernel(const bf16_t* __restrict__ x, Strides st, int H, int64_t nv, const bf16_t* __restrict__ chl,
                     const float* __restrict__ cn, float* __restrict__ xnorm, int C, int Cpad,
                     int32_t* __restrict__ labels, int32_t* __restrict__ amb_rows, int32_t* __restrict__ amb_count,
                     const int32_t* __restrict__ row_list, const int32_t* __restrict__ row_count,
                     float2* __restrict__ bnd, int32_t* __restrict__ dirty) {
  constexpr int KSN = D / 16;
  constexpr int CHUNK_BYTES = kCentChunk * D * 2 * 2;  // 64 centroids, hi and lo pieces
  constexpr int COPIES = CHUNK_BYTES / 1024 / kFilterCopyWaves;
  static_assert(CHUNK_BYTES % (1024 * kFilterCopyWaves) == 0, "chunk copies must split over the copying waves");
  extern __shared__ __attribute__((aligned(256))) unsigned char smem[];
  float* cns = reinterpret_cast<float*>(smem + 2 * CHUNK_BYTES);  // [Cpad] |c|^2 of every centroid
  float* red = cns + Cpad;                                        // [64 * kFilterWaves]
  const int bh = blockIdx.y;
  const int64_t n_rows = row_list ? row_count[bh * kHeadState] : nv;
  if ((int64_t)blockIdx.x * kFilterRows >= n_rows) return;
  const int tid = threadIdx.x, lane = tid & 63, li = lane & 31, lh = lane >> 5;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const float* cnb = cn + (int64_t)bh * Cpad;

  // |c|^2 table into LDS; Cm^2 = max |c|^2 over the real centroids
  float cm2 = 0.f;
  for (int c = tid; c < Cpad; c += 64 * kFilterWaves) {
    const float v = cnb[c];
    cns[c] = v;
    if (c < C) cm2 = fmaxf(cm2, v);
  }
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) cm2 = fmaxf(cm2, __shfl_xor(cm2, o));
  if (lane == 0) red[wave] = cm2;
  __syncthreads();
  cm2 = red[0];
#pragma unroll
  for (int w = 1; w < kFilterWaves; ++w) cm2 = fmaxf(cm2, red[w]);
  const float Cm = sqrtf(cm2) * 1.00002f;  // upper bound

  // RESIDENT (the caller's choice when Cpad <= 2 kCentChunk: both LDS stages hold their chunk of
  // centroids for good): the workgroup takes several groups of rows, one after the other - the
  // table above, the chunk copies and the barriers are paid once, and while one workgroup of a
  // CU fetches its next rows the other one computes. Otherwise the grid has one workgroup per
  // group of rows.
  int64_t grp = blockIdx.x;
  do {
  // B operands: rows of two 32-row sets, dims 16s + 8 lh .. +7
  int64_t rows[2];
  bool valid[2];
  int cur[2] = {-1, -1};  // the rows' present labels, fetched with the rows (the epilogue compares them)
  bf16x8 bx[2][KSN];
#pragma unroll
  for (int rs = 0; rs < 2; ++rs) {
    const int64_t pos = grp * kFilterRows + kFilterRowsPerWave * wave + 32 * rs + li;
    valid[rs] = pos < n_rows;
    const int64_t lpos = valid[rs] ? pos : n_rows - 1;
    rows[rs] = row_list ? row_list[(int64_t)bh * nv + lpos] : lpos;
    const bf16_t* xr = x + head_base(st, bh, H) + rows[rs] * st.n;
#pragma unroll
    for (int s = 0; s < KSN; ++s) bx[rs][s] = as_bf16x8(*reinterpret_cast<const uint4*>(xr + 16 * s + 8 * lh));
    if (dirty && lh == 0) cur[rs] = labels[(int64_t)bh * nv + rows[rs]];
  }
  SVGEAR_WAIT_VMCNT(0);
  // |x|_2 of the rows, rounded up, computed from the operands the lane holds - each lane squares
  // its half of the row, the halves meet across lane^32 - and stored for the later iterations;
  // an fp32 sum of d squares in any order is within d 2^-24 of the exact one, which the factor
  // covers
  float xn[2];
#pragma unroll
  for (int rs = 0; rs < 2; ++rs) {
    float acc = 0.f;
#pragma unroll
    for (int s = 0; s < KSN; ++s) {
      union { bf16x8 b; uint4 u; } c;
      c.b = bx[rs][s];
      const uint32_t w[4] = {c.u.x, c.u.y, c.u.z, c.u.w};
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const float lo = __uint_as_float(w[i] << 16), hi = __uint_as_float(w[i] & 0xffff0000u);
        acc = __builtin_fmaf(lo, lo, acc);
        acc = __builtin_fmaf(hi, hi, acc);
      }
    }
    acc += __shfl_xor(acc, 32);
    xn[rs] = sqrtf(acc) * 1.00002f;
    if (!row_list && lh == 0 && valid[rs]) xnorm[(int64_t)bh * nv + rows[rs]] = xn[rs];
  }

  const unsigned char* cp = reinterpret_cast<const unsigned char*>(chl + (int64_t)bh * 2 * Cpad * D);
  const uint32_t lds0 = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) unsigned char*)smem;
  const int nchunks = Cpad / kCentChunk;
  auto issue_chunk = [&](int ch) {
    if (kFilterCopyWaves < kFilterWaves && wave >= kFilterCopyWaves) return;
    const unsigned char* src = cp + (int64_t)ch * CHUNK_BYTES;
    const uint32_t dst = lds0 + (ch & 1) * CHUNK_BYTES;
#pragma unroll
    for (int i = 0; i < COPIES; ++i) {
      const int inst = wave + i * kFilterCopyWaves;
      async_copy_16B(src + inst * 1024 + lane * 16, __builtin_amdgcn_readfirstlane(dst + inst * 1024));
    }
  };

  float best[2] = {INFINITY, INFINITY}, second[2] = {INFINITY, INFINITY};
  int arg[2] = {0, 0};

  // Software pipeline over 32-centroid blocks g = 0 .. 2 nchunks - 1 (block g lives in LDS
  // stage (g/2)&1): while the VALU ranks the scores of block g, the matrix cores already
  // accumulate block g+1. The slices are written in issue order and fenced, because a wave
  // blocks at its next MFMA while the matrix core is busy: VALU work overlaps only if it sits
  // between the MFMAs in program order.
  //   slice i of a step: the two MFMAs of operand fragment i of block g+1 (one per row set),
  //                      then the score / best / second-best update of register i of block g.
  f32x16 accA0, accA1, accB0, accB1;  // two block accumulators per row set, used alternately
  auto block_base = [&](int g) { return smem + ((g >> 1) & 1) * CHUNK_BYTES + (g & 1) * (2 * KSN * 1024) + lane * 16; };
  auto rank_slice = [&](int g, int r, float nn, const f32x16& a0, const f32x16& a1) {
    // register r of block g is centroid 32 g + 8(r/4) + 4 lh + r%4, row li of the set
    const int idx = 32 * g + 8 * (r >> 2) + 4 * lh + (r & 3);
    const float s0 = __builtin_fmaf(-2.0f, a0[r], nn);
    const float s1 = __builtin_fmaf(-2.0f, a1[r], nn);
    second[0] = __builtin_amdgcn_fmed3f(s0, best[0], second[0]);
    second[1] = __builtin_amdgcn_fmed3f(s1, best[1], second[1]);
    if (s0 < best[0]) { best[0] = s0; arg[0] = idx; }
    if (s1 < best[1]) { best[1] = s1; arg[1] = idx; }
  };
  // one pipeline step: MFMAs of block g+1 (if any) interleaved with the ranking of block g
  auto step = [&](int g, bool has_next, const f32x16& cur0, const f32x16& cur1, f32x16& nxt0, f32x16& nxt1) {
    // |c|^2 of the 16 centroids this lane ranks, fetched up front (no LDS wait inside the slices)
    float nn[16];
    if (g >= 0) {
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        const float4 v = *reinterpret_cast<const float4*>(cns + 32 * g + 8 * q + 4 * lh);
        nn[4 * q] = v.x; nn[4 * q + 1] = v.y; nn[4 * q + 2] = v.z; nn[4 * q + 3] = v.w;
      }
    }
    if (has_next) {
      const unsigned char* nb = block_base(g + 1);
#pragma unroll
      for (int r = 0; r < 16; ++r) nxt0[r] = nxt1[r] = 0.f;
      bf16x8 a[2 * KSN];
#pragma unroll
      for (int i = 0; i < 4; ++i) a[i] = as_bf16x8(*reinterpret_cast<const uint4*>(nb + i * 1024));
      __builtin_amdgcn_sched_barrier(0);
#pragma unroll
      for (int i = 0; i < 2 * KSN; ++i) {
        if (i + 4 < 2 * KSN) a[i + 4] = as_bf16x8(*reinterpret_cast<const uint4*>(nb + (i + 4) * 1024));
        nxt0 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[i], bx[0][i % KSN], nxt0, 0, 0, 0);
        nxt1 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[i], bx[1][i % KSN], nxt1, 0, 0, 0);
        if (g >= 0) {
          // 16 registers spread over the 2 KSN slices
#pragma unroll
          for (int r = i * 16 / (2 * KSN); r < (i + 1) * 16 / (2 * KSN); ++r) rank_slice(g, r, nn[r], cur0, cur1);
        }
        __builtin_amdgcn_sched_barrier(0);
      }
    } else {
#pragma unroll
      for (int r = 0; r < 16; ++r) rank_slice(g, r, nn[r], cur0, cur1);
    }
  };

  // prologue: chunks 0 and 1 in flight, block 0 accumulated
  if (!RESIDENT || grp == blockIdx.x) {
    issue_chunk(0);
    if (nchunks > 1) issue_chunk(1);
    SVGEAR_WAIT_VMCNT(0);
    __syncthreads();
  }
  step(-1, true, accB0, accB1, accA0, accA1);  // accumulates block 0 into A (nothing to rank yet)
  for (int ch = 0; ch < nchunks; ++ch) {
    // block 2ch+1 (same chunk) into B while ranking block 2ch from A
    step(2 * ch, true, accA0, accA1, accB0, accB1);
    if (!RESIDENT) {
      // stage ch&1 is now free for chunk ch+2, and chunk ch+1 (issued one iteration ago) has landed
      SVGEAR_WAIT_VMCNT(0);
      __syncthreads();
      if (ch + 2 < nchunks) issue_chunk(ch + 2);
    }
    // block 2ch+2 (next chunk) into A while ranking block 2ch+1 from B
    step(2 * ch + 1, ch + 1 < nchunks, accB0, accB1, accA0, accA1);
  }
#pragma unroll
  for (int rs = 0; rs < 2; ++rs)
    settle_row<D>(best[rs], second[rs], arg[rs], valid[rs], rows[rs], xn[rs], Cm, INFINITY, nullptr, cur[rs], bh, nv,
                  Cpad, labels, amb_rows, amb_count, bnd, dirty);
  grp += gridDim.x;
  } while (RESIDENT && grp * kFilterRows < n_rows);
}

constexpr int kBoundRows = 8;  // rows per thread of bounds_update_kernel

// Per head: Cm^2 = max |c|^2, the largest and second largest centroid move, and whose the
// largest is. Every workgroup of bounds_update_kernel works them out for itself from the
// per-centroid tables (a few hundred loads; a kernel of its own cost a launch per iteration).
// Called by all 256 threads; the same code on the same tables gives every workgroup the same
// answer, also among equal moves.
__device__ __forceinline__ void head_stats(const float* __restrict__ cn, const float* __restrict__ drift, int C,
                                           float& cm2_out, float& d1_out, float& d2_out, int& a1_out) {
  __shared__ float s_cm2[4], s_d1[4], s_d2[4];
  __shared__ int s_a1[4];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  float cm2 = 0.f, d1 = 0.f, d2 = 0.f;
  int a1 = -1;
  // (d1, a1, d2) of two disjoint sets of centroids -> of their union
  auto merge = [&](float e1, int b1, float e2) {
    if (e1 > d1) {
      d2 = fmaxf(d1, e2);
      d1 = e1;
      a1 = b1;
    } else {
      d2 = fmaxf(d2, e1);
    }
  };
  for (int c = tid; c < C; c += 256) {
    cm2 = fmaxf(cm2, cn[c]);
    merge(drift[c], c, 0.f);
  }
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) {
    cm2 = fmaxf(cm2, __shfl_xor(cm2, o));
    const float e1 = __shfl_xor(d1, o), e2 = __shfl_xor(d2, o);
    const int b1 = __shfl_xor(a1, o);
    merge(e1, b1, e2);
  }
  if (lane == 0) { s_cm2[wave] = cm2; s_d1[wave] = d1; s_d2[wave] = d2; s_a1[wave] = a1; }
  __syncthreads();
  cm2 = s_cm2[0]; d1 = s_d1[0]; d2 = s_d2[0]; a1 = s_a1[0];
  for (int w = 1; w < 4; ++w) {
    cm2 = fmaxf(cm2, s_cm2[w]);
    merge(s_d1[w], s_a1[w], s_d2[w]);
  }
  cm2_out = cm2; d1_out = d1; d2_out = d2; a1_out = a1;
}

// Which rows need a new assignment (Hamerly's bounds). bnd[row] holds ub, an upper bound of the
// row's distance to its centroid, and lb, a lower bound of its distance to every other centroid,
// both for the centroids of the previous assignment. The centroids have since moved by at most
// drift[c]; by the triangle inequality the row's centroid is now at most u = ub + drift[label]
// away and every other at least l = lb - (largest drift among the others). If l^2 - u^2
// exceeds twice the error E of a fixed-order fp32 score, the fixed-order argmin is the old
// label, strictly, so the row is skipped and keeps its label with the widened bounds;
// otherwise it is flagged. Skipping never changes a label, so the result is the same as
// assigning every row in every iteration.
// LISTS = false: the flagged rows are queued (act_rows, counted in head_state[kHeadState bh])
// for assign_filter_kernel.
// LISTS = true: they are left to assign_list_kernel: prow, indexed by the row's position in the
// sorted order of the previous iteration, holds the row's index (-1 for a skipped row); per
// cluster the kernel records rmax = the largest u among its flagged rows (the radius the
// cluster's candidate list is built for; non-negative floats order like their bit patterns),
// per head the largest |x| among the flagged rows and max |c|^2.
template <int D, bool LISTS>
__global__ void __launch_bounds__(256)
bounds_update_kernel(const int32_t* __restrict__ labels, const float* __restrict__ xnorm,
                     const float* __restrict__ cn, const float* __restrict__ drift, int C, int Cpad, int64_t nv,
                     float2* __restrict__ bnd, int32_t* __restrict__ act_rows, const int32_t* __restrict__ rank,
                     int32_t* __restrict__ prow, int32_t* __restrict__ rmax, int32_t* __restrict__ head_state) {
  const int bh = blockIdx.y, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  float cm2, d1, d2;
  int a1;
  head_stats(cn + (int64_t)bh * Cpad, drift + (int64_t)bh * Cpad, C, cm2, d1, d2, a1);
  const float Cm = sqrtf(cm2) * 1.00002f;
  if (LISTS && blockIdx.x == 0 && tid == 0) head_state[bh * kHeadState + 2] = __float_as_int(cm2);

  // kBoundRows rows per thread, 256 apart (a launch of one-row threads is bound by the rate at
  // which workgroups start, not by memory)
  float xmax = 0.f;
  unsigned qmask = 0;
#pragma unroll
  for (int j = 0; j < kBoundRows; ++j) {
    const int64_t row = ((int64_t)blockIdx.x * kBoundRows + j) * 256 + tid;
    if (row < nv) {
      const int a = labels[(int64_t)bh * nv + row];
      const float2 st = bnd[(int64_t)bh * nv + row];
      const float X = xnorm[(int64_t)bh * nv + row];
      const float u = (st.x + drift[(int64_t)bh * Cpad + a]) * 1.000001f;
      const float l = (st.y - (a == a1 ? d2 : d1)) * 0.999999f;
      const float E = fixed_order_error<D>(X, Cm);
      const bool keep = l > u && (l - u) * (l + u) > 2.002f * E;  // false for NaN
      bnd[(int64_t)bh * nv + row] = make_float2(u, l > 0.f ? l : 0.f);
      if constexpr (LISTS) {
        prow[(int64_t)bh * nv + rank[(int64_t)bh * nv + row]] = keep ? -1 : (int32_t)row;
        if (!keep) {
          const int ubits = __float_as_int(u);
          // (the plain read only saves atomics: most rows find a radius that already covers them)
          if (ubits > rmax[(int64_t)bh * Cpad + a]) atomicMax(&rmax[(int64_t)bh * Cpad + a], ubits);
          xmax = fmaxf(xmax, X);
        }
      }
      if (!LISTS && !keep) qmask |= 1u << j;
    }
  }
  if constexpr (LISTS) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) xmax = fmaxf(xmax, __shfl_xor(xmax, o));
    if (lane == 0 && xmax > 0.f) atomicMax(&head_state[bh * kHeadState + 1], __float_as_int(xmax));
  } else {
    // queue the rows of this workgroup with one counter update: exclusive scan of the per-thread
    // counts (wave shuffles, then the four wave totals)
    __shared__ int s_cnt[4], s_base;
    const int cnt = __popc(qmask);
    int incl = cnt;
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) {
      const int t = __shfl_up(incl, o);
      if (lane >= o) incl += t;
    }
    if (lane == 63) s_cnt[wave] = incl;
    __syncthreads();
    if (tid == 0) {
      const int total = s_cnt[0] + s_cnt[1] + s_cnt[2] + s_cnt[3];
      s_base = total ? atomicAdd(&head_state[bh * kHeadState], total) : 0;
    }
    __syncthreads();
    int pos = s_base + incl - cnt;
    for (int w = 0; w < wave; ++w) pos += s_cnt[w];
#pragma unroll
    for (int j = 0; j < kBoundRows; ++j)
      if (qmask & (1u << j))
        act_rows[(int64_t)bh * nv + pos++] = (int32_t)(((int64_t)blockIdx.x * kBoundRows + j) * 256 + tid);
  }
}

// Candidate lists. For cluster a whose flagged rows are all within R of its centroid, a
// centroid c at distance d from centroid a cannot be the fixed-order argmin of any of those rows
// if (d - R)^2 - R^2 = d (d - 2R) exceeds twice the error E of a fixed-order fp32 score: the
// row is at least d - R from c and at most R from a, so in real numbers c's score exceeds a's
// by more than 2E and its fixed-order score is strictly larger. Every other centroid joins
// the list (a itself always does). dout[a] is a lower bound of the distance from centroid a to
// the nearest centroid left out (+inf if none): the rows' lower bounds need it. A list longer
// than kListMax is dropped (nlen = -1: the cluster's rows are tested against every centroid).
// The centroid-to-centroid products run on the bf16 matrix cores from the operand table of the
// filter (c = hi + lo + a residual below 2^-16 |c|), which serves as A operand (centroid c of a
// 32-block = row lane % 32) and as B operand (cluster a = column lane % 32) alike: a.c ~
// hi.hi + hi.lo + lo.hi, and d^2 = |a|^2 + |c|^2 - 2 a.c is lowered by 1.2e-4 (|a|^2 + |c|^2), more
// than the split residuals, the dropped lo.lo term and the fp32 roundings together.
// One workgroup per 32 clusters; its 4 waves take the 32-blocks of centroids round-robin. A
// lane owns one cluster (column) and 16 centroids of a block. First pass: which centroids stay
// (16 bits per lane and block, kept in LDS) and how many; then every wave knows where its part of
// each list starts (wave order, inside a wave ascending centroid index: the order is fixed,
// and no result depends on it -- equal approximate scores send a row to the exact kernel);
// second pass: the entries are written.
template <int D>
__global__ void __launch_bounds__(256)
nlist_kernel(const bf16_t* __restrict__ chl, const float* __restrict__ cn, int C, int Cpad,
             const int32_t* __restrict__ rmax, const int32_t* __restrict__ head_state, int32_t* __restrict__ nlist,
             int32_t* __restrict__ nlen, float* __restrict__ dout) {
  constexpr int KSN = D / 16;
  __shared__ uint16_t s_keep[kMaxCentroids / 32][64];
  __shared__ int s_cnt[4][32];
  __shared__ float s_dmin[4][32];
  const int bh = blockIdx.y, lane = threadIdx.x & 63, li = lane & 31, lh = lane >> 5;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int ab = blockIdx.x;  // block of 32 clusters
  const int a = ab * 32 + li;
  const bf16_t* tab = chl + (int64_t)bh * 2 * Cpad * D;
  const float* cnb = cn + (int64_t)bh * Cpad;
  bf16x8 bhi[KSN], blo[KSN];
#pragma unroll
  for (int s = 0; s < KSN; ++s) {
    const bf16_t* frag = tab + ((int64_t)(ab * 2) * KSN + s) * 512 + lane * 8;  // hi piece; lo: KSN fragments on
    bhi[s] = as_bf16x8(*reinterpret_cast<const uint4*>(frag));
    blo[s] = as_bf16x8(*reinterpret_cast<const uint4*>(frag + (int64_t)KSN * 512));
  }
  const float cna = a < C ? cnb[a] : 0.f;
  const float r2 = a < C ? 2.0f * __int_as_float(rmax[(int64_t)bh * Cpad + a]) * 1.000001f : 0.f;
  const float Cm = sqrtf(__int_as_float(head_state[bh * kHeadState + 2])) * 1.00002f;
  const float E2 = 2.002f * fixed_order_error<D>(__int_as_float(head_state[bh * kHeadState + 1]), Cm);
  int mine = 0;  // entries of cluster a this lane contributes
  float dmin = INFINITY;
  for (int cb = wave; cb * 32 < C; cb += 4) {
    f32x16 acc;
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[r] = 0.f;
#pragma unroll
    for (int s = 0; s < KSN; ++s) {
      const bf16_t* frag = tab + ((int64_t)(cb * 2) * KSN + s) * 512 + lane * 8;
      const bf16x8 ahi = as_bf16x8(*reinterpret_cast<const uint4*>(frag));
      const bf16x8 alo = as_bf16x8(*reinterpret_cast<const uint4*>(frag + (int64_t)KSN * 512));
      acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ahi, bhi[s], acc, 0, 0, 0);
      acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ahi, blo[s], acc, 0, 0, 0);
      acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(alo, bhi[s], acc, 0, 0, 0);
    }
    // register r is centroid 32 cb + 8 (r/4) + 4 lh + r%4, cluster a
    unsigned keep = 0;
#pragma unroll
    for (int g = 0; g < 4; ++g) {
      const float4 n4 = *reinterpret_cast<const float4*>(cnb + 32 * cb + 8 * g + 4 * lh);
      const float nn[4] = {n4.x, n4.y, n4.z, n4.w};
#pragma unroll
      for (int r = 0; r < 4; ++r) {
        const int c = 32 * cb + 8 * g + 4 * lh + r;
        const float nsum = cna + nn[r];
        const float dd2 = nsum - 2.0f * acc[4 * g + r] - 1.2e-4f * nsum;  // lower bound of |a - c|^2
        const float d = sqrtf(fmaxf(dd2, 0.f)) * 0.999999f;               // lower bound of |a - c|
        const bool out_c = d > r2 && d * (d - r2) * 0.9999f > E2;         // false for NaN: kept
        const bool k = c < C && (!out_c || c == a);
        if (c < C && !k) dmin = fminf(dmin, d);
        if (k) keep |= 1u << (4 * g + r);
      }
    }
    s_keep[cb][lane] = (uint16_t)keep;
    mine += __popc(keep);
  }
  mine += __shfl_xor(mine, 32);
  dmin = fminf(dmin, __shfl_xor(dmin, 32));
  if (lh == 0) {
    s_cnt[wave][li] = mine;
    s_dmin[wave][li] = dmin;
  }
  __syncthreads();
  int run = 0, total = 0;
#pragma unroll
  for (int w = 0; w < 4; ++w) {
    if (w < wave) run += s_cnt[w][li];
    total += s_cnt[w][li];
    dmin = fminf(dmin, s_dmin[w][li]);
  }
  if (a < C && total <= kListMax) {  // (a list that is dropped is not written either)
    int32_t* out = nlist + ((int64_t)bh * C + a) * kListMax;
    for (int cb = wave; cb * 32 < C; cb += 4) {
      // (each lane reads back what it wrote itself, and its partner's after the barrier above)
      const unsigned keep = s_keep[cb][lane], theirs = s_keep[cb][lane ^ 32];
      // inside the block ascending: group g of the lower lane half (centroids 8g .. 8g+3), then
      // group g of the upper half (8g+4 .. 8g+7)
      int pos = run;
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        const int tg = __popc((theirs >> (4 * g)) & 15u);
        if (lh) pos += tg;  // the lower half's group comes first
#pragma unroll
        for (int r = 0; r < 4; ++r)
          if (keep & (1u << (4 * g + r))) out[pos++] = 32 * cb + 8 * g + 4 * lh + r;
        if (!lh) pos += tg;
      }
      run = pos;  // both lanes of a cluster arrive at the same total
    }
  }
  if (wave == 0 && lh == 0 && a < C) {
    nlen[(int64_t)bh * C + a] = total <= kListMax ? total : -1;
    dout[(int64_t)bh * C + a] = total <= kListMax ? dmin : INFINITY;
  }
}

// Later iterations: the flagged rows against the candidate list of the cluster they are in -- a
// centroid outside the list provably has a larger fixed-order score than the row's old
// centroid, so the argmin over the list is the argmin over all centroids. A few clusters (wide
// ones, whose radius reaches most centroids) have no list (nlen < 0): their flagged rows are
// only queued here, for assign_filter_kernel, which tests every centroid and shares the
// centroids among 256 rows. One wave takes a chunk of at most kListChunk positions of ONE cluster in
// the sorted order (chunk table of sort_labels), 64 positions per step. Lists are short (a
// handful to a few dozen centroids once the clustering settles), so there is nothing to share
// between waves: no LDS, no barrier. What bounds the kernel is the number of cache lines its
// fetches touch (every row and every candidate lies somewhere else), so
//  * a list of at most 32 candidates is fetched once per wave and stays in registers;
//  * a lane reads half a row / half a piece of "its" candidate (position lane % 32 of the list's
//    32-block) as whole cache lines: the contraction index is permuted (the filter's scores are
//    approximate and their error bound holds for any order of the additions), in k-step s lane
//    (i, h) holds dims D/2 h + 8 s .. + 7 of centroid / row i;
//  * rows that are not flagged are not fetched, and nothing of a flagged row's state is read:
//    every 4 bytes read or written at a row's index cost a whole memory transaction, as much as
//    a quarter of the row itself. |x| is computed again from the row, the row's old upper bound
//    is replaced by the cluster's radius, and which rows are flagged comes in position order;
//  * the chain of dependent fetches is three long (tile -> rows and list -> operands), and the
//    rows of the next step are looked up while this step's are ranked.
template <int D>
__global__ void __launch_bounds__(64)
assign_list_kernel(const bf16_t* __restrict__ x, Strides st, int H, int64_t nv, const bf16_t* __restrict__ crow,
                   const float* __restrict__ cn, int C, int Cpad, int32_t* __restrict__ labels,
                   int32_t* __restrict__ amb_rows, int32_t* __restrict__ amb_count,
                   const int32_t* __restrict__ prow, const int4* __restrict__ tiles, int tile_cap,
                   const int32_t* __restrict__ rmax, const int32_t* __restrict__ nlist,
                   const int32_t* __restrict__ nlen, const float* __restrict__ dout,
                   int32_t* __restrict__ head_state, int32_t* __restrict__ act_rows, float2* __restrict__ bnd,
                   int32_t* __restrict__ dirty) {
  constexpr int KSN = D / 16;
  const int bh = blockIdx.y, lane = threadIdx.x & 63, li = lane & 31, lh = lane >> 5;
  const int4 tile = tiles[(int64_t)bh * tile_cap + blockIdx.x];
  const int a_old = tile.x, p_begin = tile.y, p_end = tile.z;
  if (a_old < 0) return;
  const int n_list = nlen[(int64_t)bh * C + a_old];
  if (n_list < 0) {  // no list: queue the flagged rows (all fetches first, then one counter update)
    int r[kListChunk / 64];
#pragma unroll
    for (int j = 0; j < kListChunk / 64; ++j) {
      const int p = p_begin + 64 * j + lane;
      r[j] = p < p_end ? prow[(int64_t)bh * nv + p] : -1;
    }
    int mine = 0;
#pragma unroll
    for (int j = 0; j < kListChunk / 64; ++j) mine += r[j] >= 0;
    int incl = mine;
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) {
      const int t = __shfl_up(incl, o);
      if (lane >= o) incl += t;
    }
    const int total = __shfl(incl, 63);
    if (total == 0) return;
    int base = 0;
    if (lane == 0) base = atomicAdd(&head_state[bh * kHeadState], total);
    int slot = __shfl(base, 0) + incl - mine;
#pragma unroll
    for (int j = 0; j < kListChunk / 64; ++j)
      if (r[j] >= 0) act_rows[(int64_t)bh * nv + slot++] = r[j];
    return;
  }
  // a centroid outside the list is at least |a_old - c| - |x - a_old| away from a flagged row x of
  // the cluster, and the list was built for |x - a_old| <= rmax
  const float far = dout[(int64_t)bh * C + a_old] * 0.99999f -
                    __int_as_float(rmax[(int64_t)bh * Cpad + a_old]) * 1.000001f;
  const float Cm = sqrtf(__int_as_float(head_state[bh * kHeadState + 2])) * 1.00002f;
  const int nblk = (n_list + 31) / 32;
  const int32_t* lst = nlist + ((int64_t)bh * C + a_old) * kListMax;
  const bf16_t* tab = crow + (int64_t)bh * 2 * Cpad * D;
  const float* cnb = cn + (int64_t)bh * Cpad;

  // this lane's candidate of block g (both lane halves hold the same one): operands and |c|^2
  bf16x8 av[2 * KSN];
  float cnv;
  auto fetch_candidates = [&](int g) {
    // (the entry is fetched whether or not the list reaches it, so that the fetch does not wait for
    // the list's length; an entry beyond the length is whatever the memory holds and is not used)
    const int entry = lst[32 * g + li];
    const int ci = 32 * g + li < n_list ? entry : -1;
    const int cc = ci < 0 ? 0 : ci;  // padding: any centroid's bits, its |c|^2 entry is +inf
    cnv = ci < 0 ? INFINITY : cnb[cc];
    const bf16_t* src = tab + (int64_t)cc * 2 * D + (D / 2) * lh;
#pragma unroll
    for (int i = 0; i < 2 * KSN; ++i)  // hi piece (k-steps 0 .. KSN-1), then lo piece
      av[i] = as_bf16x8(*reinterpret_cast<const uint4*>(src + (i / KSN) * D + 8 * (i % KSN)));
  };
  // rows of the step at positions p .. p + 63 (row set rs, lane li: position p + 32 rs + li) and
  // whether they are flagged
  auto fetch_rows = [&](int p, int64_t (&rows)[2], int (&flag)[2]) {
#pragma unroll
    for (int rs = 0; rs < 2; ++rs) {
      const int pos = p + 32 * rs + li;
      const int r = pos < p_end ? prow[(int64_t)bh * nv + pos] : -1;
      rows[rs] = r < 0 ? 0 : r;
      flag[rs] = r >= 0;
    }
  };

  int64_t rows[2], rows_next[2];
  int flag[2], flag_next[2];
  fetch_rows(p_begin, rows, flag);
  fetch_candidates(0);
  for (int p = p_begin; p < p_end; p += kListTile) {
    const bool more = p + kListTile < p_end;
    if (more) fetch_rows(p + kListTile, rows_next, flag_next);
    const bool valid[2] = {flag[0] != 0, flag[1] != 0};
    if (__any(valid[0] || valid[1])) {  // else nothing flagged in this step (whole wave)
      bf16x8 bx[2][KSN];
      float xn[2];
#pragma unroll
      for (int rs = 0; rs < 2; ++rs) {
#pragma unroll
        for (int s = 0; s < KSN; ++s) bx[rs][s] = as_bf16x8(uint4{0u, 0u, 0u, 0u});
        if (valid[rs]) {
          const bf16_t* xr = x + head_base(st, bh, H) + rows[rs] * st.n + (D / 2) * lh;
#pragma unroll
          for (int s = 0; s < KSN; ++s) bx[rs][s] = as_bf16x8(*reinterpret_cast<const uint4*>(xr + 8 * s));
        }
        // |x|_2 rounded up, as in assign_filter_kernel
        float acc = 0.f;
#pragma unroll
        for (int s = 0; s < KSN; ++s) {
          union { bf16x8 b; uint4 u; } c;
          c.b = bx[rs][s];
          const uint32_t w[4] = {c.u.x, c.u.y, c.u.z, c.u.w};
#pragma unroll
          for (int i = 0; i < 4; ++i) {
            const float lo = __uint_as_float(w[i] << 16), hi = __uint_as_float(w[i] & 0xffff0000u);
            acc = __builtin_fmaf(lo, lo, acc);
            acc = __builtin_fmaf(hi, hi, acc);
          }
        }
        acc += __shfl_xor(acc, 32);
        xn[rs] = sqrtf(acc) * 1.00002f;
      }
      float best[2] = {INFINITY, INFINITY}, second[2] = {INFINITY, INFINITY};
      int arg[2] = {0, 0};
      for (int g = 0; g < nblk; ++g) {
        if (nblk > 1) fetch_candidates(g);  // (a single block is already in registers)
        f32x16 acc0, acc1;
#pragma unroll
        for (int r = 0; r < 16; ++r) acc0[r] = acc1[r] = 0.f;
#pragma unroll
        for (int i = 0; i < 2 * KSN; ++i) {
          acc0 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(av[i], bx[0][i % KSN], acc0, 0, 0, 0);
          acc1 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(av[i], bx[1][i % KSN], acc1, 0, 0, 0);
        }
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          // register r is the candidate at position 32 g + 8(r/4) + 4 lh + r%4 of the list
          const int k = 8 * (r >> 2) + 4 * lh + (r & 3);
          const float nn = __shfl(cnv, k);
          const int idx = 32 * g + k;
          const float s0 = __builtin_fmaf(-2.0f, acc0[r], nn);
          const float s1 = __builtin_fmaf(-2.0f, acc1[r], nn);
          second[0] = __builtin_amdgcn_fmed3f(s0, best[0], second[0]);
          second[1] = __builtin_amdgcn_fmed3f(s1, best[1], second[1]);
          if (s0 < best[0]) { best[0] = s0; arg[0] = idx; }
          if (s1 < best[1]) { best[1] = s1; arg[1] = idx; }
        }
      }
#pragma unroll
      for (int rs = 0; rs < 2; ++rs)
        settle_row<D>(best[rs], second[rs], arg[rs], valid[rs], rows[rs], xn[rs], Cm, far, lst, a_old, bh, nv, Cpad,
                      labels, amb_rows, amb_count, bnd, dirty);
    }
    if (more) {
#pragma unroll
      for (int rs = 0; rs < 2; ++rs) {
        rows[rs] = rows_next[rs];
        flag[rs] = flag_next[rs];
      }
    }
  }
}

// Mean of the members of one cluster. A row is covered by LPR lanes of 16 bytes each; the
// 256 threads form 256/LPR member slots. Slot s sums members s, s+SLOTS, ... in order;
// slots are then added in slot order. With gridDim.z = P > 1 the members are cut into P
// contiguous parts (a fixed function of the cluster's size), part z writes its sum to
// `partial` [BH][C][P][D] and means_finish_kernel adds the parts in order: a few very large
// clusters no longer set the kernel's duration, and the result stays run-to-run identical.
template <typename T, int D>
__global__ void __launch_bounds__(256)
means_kernel(const T* __restrict__ x, Strides st, int H, const int32_t* __restrict__ perm, int64_t N,
             const int32_t* __restrict__ offsets, int C, float* __restrict__ cent,
             int32_t* __restrict__ counts, float* __restrict__ partial, const int32_t* __restrict__ dirty,
             int Cpad, float* __restrict__ drift) {
  constexpr int VEC = 16 / sizeof(T);  // elements per lane
  constexpr int LPR = D / VEC;         // lanes per row
  constexpr int SLOTS = 256 / LPR;
  __shared__ float red[SLOTS][D];
  const int c = blockIdx.x, bh = blockIdx.y;
  // a cluster whose membership did not change keeps its centroid and count (same sum)
  if (dirty && !dirty[(int64_t)bh * Cpad + c]) {
    if (drift && gridDim.z == 1 && threadIdx.x == 0) drift[(int64_t)bh * Cpad + c] = 0.f;  // it did not move
    return;
  }
  const int slot = threadIdx.x / LPR, lane = threadIdx.x % LPR;
  const int32_t* off = offsets + (int64_t)bh * (C + 2);
  const int c_start = off[c], c_end = off[c + 1];
  const int P = gridDim.z, part = blockIdx.z;
  const int part_len = (((c_end - c_start + P - 1) / P) + SLOTS - 1) / SLOTS * SLOTS;
  const int start = c_start + part * part_len < c_end ? c_start + part * part_len : c_end;
  const int end = start + part_len < c_end ? start + part_len : c_end;
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
  const int cnt = c_end - c_start;
  float dv2 = 0.f;  // this dimension's share of the centroid's squared move
  if (threadIdx.x < D && (cnt > 0 || P > 1)) {
    float s = red[0][threadIdx.x];
#pragma unroll
    for (int k = 1; k < SLOTS; ++k) s += red[k][threadIdx.x];
    if (P == 1) {
      const int64_t ci = ((int64_t)bh * C + c) * D + threadIdx.x;
      const float v = s / (float)cnt;
      if (drift) {
        const float dv = v - cent[ci];
        dv2 = dv * dv;
      }
      cent[ci] = v;
    } else {
      partial[(((int64_t)bh * C + c) * P + part) * D + threadIdx.x] = s;
    }
  }
  if (P == 1 && threadIdx.x == 0 && counts) counts[(int64_t)bh * C + c] = cnt;
  if (P == 1 && drift) {
    // how far the centroid moved, rounded up (an fp32 sum of D non-negative terms is within
    // D 2^-23 of the exact one): the row bounds of the next iteration need it
    __shared__ float dpart[D / 64];
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) dv2 += __shfl_xor(dv2, o);
    if (threadIdx.x < D && (threadIdx.x & 63) == 0) dpart[threadIdx.x >> 6] = dv2;
    __syncthreads();
    if (threadIdx.x == 0) {
      float t = dpart[0];
#pragma unroll
      for (int w = 1; w < D / 64; ++w) t += dpart[w];
      drift[(int64_t)bh * Cpad + c] = sqrtf(t) * 1.0001f;
    }
  }
}

// Adds the P partial sums of every cluster in part order and divides by the member count; a
// cluster without members keeps its centroid. With drift != nullptr it also records how far
// every centroid moved (rounded up; 0 for the clusters that were not touched). D is 64 or 128,
// so the D threads of a centroid are whole waves of one workgroup.
__global__ void __launch_bounds__(256)
means_finish_kernel(const float* __restrict__ partial, const int32_t* __restrict__ offsets, int C, int P, int D,
                    float* __restrict__ cent, int32_t* __restrict__ counts, const int32_t* __restrict__ dirty,
                    int Cpad, float* __restrict__ drift) {
  __shared__ float dpart[4];
  const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;  // (bh, c, dim)
  const int bh = blockIdx.y;
  const bool in = i < (int64_t)C * D;
  const int c = in ? (int)(i / D) : 0, dim = in ? (int)(i % D) : 1;
  float dv2 = 0.f;
  if (in && !(dirty && !dirty[(int64_t)bh * Cpad + c])) {
    const int32_t* off = offsets + (int64_t)bh * (C + 2);
    const int cnt = off[c + 1] - off[c];
    if (cnt > 0) {
      const float* pp = partial + (((int64_t)bh * C + c) * P) * D + dim;
      float s = pp[0];
      for (int k = 1; k < P; ++k) s += pp[(int64_t)k * D];
      const int64_t ci = ((int64_t)bh * C + c) * D + dim;
      const float v = s / (float)cnt;
      if (drift) {
        const float dv = v - cent[ci];
        dv2 = dv * dv;
      }
      cent[ci] = v;
    }
    if (dim == 0 && counts) counts[(int64_t)bh * C + c] = cnt;
  }
  if (drift) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) dv2 += __shfl_xor(dv2, o);
    const int wave = threadIdx.x >> 6;
    if ((threadIdx.x & 63) == 0) dpart[wave] = dv2;
    __syncthreads();
    if (in && dim == 0) {
      float t = dpart[wave];
      for (int w = 1; w < D / 64; ++w) t += dpart[wave + w];
      drift[(int64_t)bh * Cpad + c] = sqrtf(t) * 1.0001f;
    }
  }
}

// Parts per cluster of the centroid update: about 128 members per part on average, at most 8.
static inline int means_parts(int64_t n, int C) {
  const int64_t p = (n / C + 64) / 128;
  return (int)(p < 1 ? 1 : (p > 8 ? 8 : p));
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
  constexpr bool kFilter = sizeof(T) == 2;  // bf16 input: filter on bf16 MFMAs, then exact on the ambiguous rows
  bf16_t* chl = kFilter ? ws.take<bf16_t>((size_t)BH * 2 * Cpad * D) : nullptr;
  bf16_t* crow = kFilter ? ws.take<bf16_t>((size_t)BH * 2 * Cpad * D) : nullptr;
  int32_t* amb_rows = kFilter ? ws.take<int32_t>((size_t)BH * nv) : nullptr;
  int32_t* amb_count = kFilter ? ws.take<int32_t>((size_t)BH) : nullptr;
  const int P = means_parts(nv, C);
  float* partial = P > 1 ? ws.take<float>((size_t)BH * C * P * D) : nullptr;
  // row skipping between iterations (bf16 input): distance bounds and flags per row, centroid
  // moves, per-cluster radii and candidate lists, the tile table of the sorted order
  const bool use_lists = kFilter && C >= g_list_min_centroids.load(std::memory_order_relaxed);
  const int tile_cap = (int)(nv / kListChunk) + C + 1;
  float2* bnd = kFilter ? ws.take<float2>((size_t)BH * nv) : nullptr;
  float* xnorm = kFilter ? ws.take<float>((size_t)BH * nv) : nullptr;
  int32_t* rank = kFilter ? ws.take<int32_t>((size_t)BH * nv) : nullptr;
  int32_t* prow = kFilter ? ws.take<int32_t>((size_t)BH * nv) : nullptr;
  int32_t* act_rows = kFilter ? ws.take<int32_t>((size_t)BH * nv) : nullptr;
  int32_t* head_state = kFilter ? ws.take<int32_t>((size_t)BH * kHeadState) : nullptr;
  float* drift = kFilter ? ws.take<float>((size_t)BH * Cpad) : nullptr;
  int32_t* rmax = kFilter ? ws.take<int32_t>((size_t)BH * Cpad) : nullptr;
  int32_t* dirty = kFilter ? ws.take<int32_t>((size_t)BH * Cpad) : nullptr;
  int32_t* nlist = kFilter ? ws.take<int32_t>((size_t)BH * C * kListMax) : nullptr;
  int32_t* nlen = kFilter ? ws.take<int32_t>((size_t)BH * C) : nullptr;
  float* dout = kFilter ? ws.take<float>((size_t)BH * C) : nullptr;
  int4* tiles = kFilter ? ws.take<int4>((size_t)BH * tile_cap) : nullptr;
  if (!ws.ok()) return SVGEAR_ERR_WORKSPACE;
  const size_t lds = 2 * (size_t)kCentChunk * D * 4 + 2 * kCentChunk * sizeof(float);
  auto assign = assign_mfma_kernel<T, D>;
  SVGEAR_HIP_TRY(hipFuncSetAttribute(reinterpret_cast<const void*>(assign),
                                     hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));
  const size_t lds_f = 2 * (size_t)kCentChunk * D * 4 + ((size_t)Cpad + 64 * kFilterWaves) * sizeof(float);
  if constexpr (kFilter) {
    SVGEAR_HIP_TRY(hipFuncSetAttribute(reinterpret_cast<const void*>(assign_filter_kernel<D, false>),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds_f));
    SVGEAR_HIP_TRY(hipFuncSetAttribute(reinterpret_cast<const void*>(assign_filter_kernel<D, true>),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds_f));
  }
  const dim3 gp((unsigned)ceil_div((int64_t)Cpad * D, 256 * 4), BH);
  const dim3 ga((unsigned)ceil_div(nv, kAssignRows), BH);
  // only_changed: clusters that neither gained nor lost a member in this iteration keep their
  // centroid (flags set by the assignment kernels; null = every cluster)
  // moves: where the update records how far every centroid moved (null = not needed)
  auto update = [&](const T* src, float* dst, int32_t* cnt_out, const int32_t* only_changed, float* moves) -> int {
    means_kernel<T, D><<<dim3(C, BH, P), 256, 0, s>>>(src, st, H, perm, nv, offsets, C, dst, cnt_out, partial,
                                                      only_changed, Cpad, moves);
    SVGEAR_LAUNCH_CHECK();
    if (P > 1) {
      means_finish_kernel<<<dim3((unsigned)ceil_div((int64_t)C * D, 256), BH), 256, 0, s>>>(
          partial, offsets, C, P, D, dst, cnt_out, only_changed, Cpad, moves);
      SVGEAR_LAUNCH_CHECK();
    }
    return SVGEAR_OK;
  };
  for (int it = 0; it < iters; ++it) {
    prep_centroids_kernel<<<gp, 256, 0, s>>>(cent, C, Cpad, D, cperm, cn, chl, crow, amb_count, head_state, rmax,
                                             dirty);
    SVGEAR_LAUNCH_CHECK();
    if constexpr (kFilter) {
      // (with at most two chunks of centroids a workgroup of the filter takes several groups of rows)
      const bool resident = Cpad <= 2 * kCentChunk;
      auto filter = resident ? assign_filter_kernel<D, true> : assign_filter_kernel<D, false>;
      const dim3 gf((unsigned)ceil_div(ceil_div(nv, kFilterRows), resident ? kFilterGroups : 1), BH);
      const dim3 gb((unsigned)ceil_div(nv, 256 * kBoundRows), BH);
      const bf16_t* xb = reinterpret_cast<const bf16_t*>(x);
      if (it == 0) {
        // every row against every centroid
        filter<<<gf, 64 * kFilterWaves, lds_f, s>>>(xb, st, H, nv, chl, cn, xnorm, C, Cpad, labels, amb_rows, amb_count,
                                                    nullptr, nullptr, bnd, nullptr);
        SVGEAR_LAUNCH_CHECK();
      } else {
        // only the rows whose bounds do not prove that their label stays
        if (use_lists && it >= kListFromIteration) {
          // ... each against the centroids near its cluster
          bounds_update_kernel<D, true><<<gb, 256, 0, s>>>(labels, xnorm, cn, drift, C, Cpad, nv, bnd, act_rows, rank,
                                                           prow, rmax, head_state);
          SVGEAR_LAUNCH_CHECK();
          nlist_kernel<D><<<dim3((unsigned)ceil_div(C, 32), BH), 256, 0, s>>>(chl, cn, C, Cpad, rmax, head_state,
                                                                               nlist, nlen, dout);
          SVGEAR_LAUNCH_CHECK();
          assign_list_kernel<D><<<dim3((unsigned)tile_cap, BH), 64, 0, s>>>(
              xb, st, H, nv, crow, cn, C, Cpad, labels, amb_rows, amb_count, prow, tiles, tile_cap, rmax, nlist, nlen,
              dout, head_state, act_rows, bnd, dirty);
          SVGEAR_LAUNCH_CHECK();
        } else {
          bounds_update_kernel<D, false><<<gb, 256, 0, s>>>(labels, xnorm, cn, drift, C, Cpad, nv, bnd, act_rows,
                                                            nullptr, nullptr, nullptr, head_state);
          SVGEAR_LAUNCH_CHECK();
        }
        // the queued rows (all flagged rows, or those of the clusters without a list) against
        // every centroid; the grid covers every row, workgroups beyond the queue's length leave
        // at once
        filter<<<gf, 64 * kFilterWaves, lds_f, s>>>(xb, st, H, nv, chl, cn, xnorm, C, Cpad, labels, amb_rows, amb_count,
                                                    act_rows, head_state, bnd, dirty);
        SVGEAR_LAUNCH_CHECK();
      }
      assign_few_kernel<T, D><<<dim3((unsigned)ceil_div(nv, 32 * 8), BH), 256, 0, s>>>(
          x, st, H, nv, cperm, cn, Cpad, labels, amb_rows, amb_count, it > 0 ? dirty : nullptr);
    } else {
      assign<<<ga, 64 * kAssignWaves, lds, s>>>(x, st, H, nv, cperm, cn, Cpad, labels);
    }
    SVGEAR_LAUNCH_CHECK();
    int rc = sort_labels(labels, BH, nv, 0, C, perm, offsets, chunk_hist, s, use_lists ? tiles : nullptr, tile_cap,
                         kListChunk, use_lists ? rank : nullptr);
    if (rc != SVGEAR_OK) return rc;
    rc = update(x, cent, counts, (kFilter && it > 0) ? dirty : nullptr, drift);
    if (rc != SVGEAR_OK) return rc;
  }
  if (x2) {
    const int rc = update(x2, cent2, nullptr, nullptr, nullptr);
    if (rc != SVGEAR_OK) return rc;
  }
  return SVGEAR_OK;
}

}  // namespace
}  // namespace svgear

using namespace svgear;

extern "C" int svgear_kmeans_list_threshold(int min_centroids) {
  if (min_centroids <= 0) return g_list_min_centroids.load(std::memory_order_relaxed);
  return g_list_min_centroids.exchange(min_centroids, std::memory_order_relaxed);
}

extern "C" size_t svgear_kmeans_workspace(int B, int H, int64_t N, int d, int C) {
  if (B <= 0 || H <= 0 || N <= 0 || C <= 0 || d <= 0) return 0;
  const size_t BH = (size_t)B * H;
  const size_t Cpad = align_up(C, kCentChunk);
  return align_up(BH * sort_chunks(N) * (C + 1) * 4, 256) + align_up(BH * N * 4, 256) +
         align_up(BH * (C + 2) * 4, 256) + align_up(BH * Cpad * 4, 256) + align_up(BH * Cpad * d * 4, 256) +
         // bf16 filter: hi/lo operand tables (two layouts), ambiguous-row list and counter
         2 * align_up(BH * 2 * Cpad * d * 2, 256) + align_up(BH * N * 4, 256) + align_up(BH * 4, 256) +
         // partial sums of the split centroid update
         (means_parts(N, C) > 1 ? align_up(BH * C * means_parts(N, C) * d * 4, 256) : 0) +
         // row skipping: per row two bounds, the norm, the sorted position, the flagged-row table and
         // the queue; per-head maxima, centroid moves, radii,
         // membership-changed flags, candidate lists with their lengths and outer distances, chunk table
         align_up(BH * N * 8, 256) + 4 * align_up(BH * N * 4, 256) +
         align_up(BH * kHeadState * 4, 256) + 3 * align_up(BH * Cpad * 4, 256) +
         align_up(BH * C * kListMax * 4, 256) + 2 * align_up(BH * C * 4, 256) +
         align_up(BH * (N / kListChunk + C + 1) * 16, 256);
}

extern "C" int svgear_kmeans(const void* x, const void* x2, svgear_dtype dt, int B, int H, int64_t N,
                             int64_t n_tail, int d, const int64_t xstride[3], int C, int iters, float* centroids,
                             float* centroids2, int32_t* labels, int32_t* counts, void* ws, size_t ws_bytes,
                             void* stream) {
  if (!x || !xstride || !centroids || !labels || !counts || B <= 0 || H <= 0 || N <= 0 || n_tail < 0 ||
      n_tail >= N || C <= 0 || C > N - n_tail || C > kMaxCentroids || iters < 1 || N > INT32_MAX / 2 ||
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
