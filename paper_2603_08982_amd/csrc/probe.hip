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
#include <type_traits>

#include "common.h"

namespace svgear {
namespace {

constexpr int kKeyChunk = 64;
constexpr float kMaxExponent = 40.0f;  // e^40 squared still fits fp32

// Sbar[a][b] = qbar_a . kbar_b * scale; mrow[a] = max over non-empty b.
// With q3 != nullptr (grid.x = Cq rounded up to 32) it also writes qbar split into three bf16
// pieces q = hi + mid + lo (exact: 3 x 8 significant bits), laid out as B operands of
// v_mfma_f32_32x32x16_bf16: [a-block][piece][s][lane = a%32 + 32*((k%16)/8)][k%8], zero rows
// for a >= Cq.
constexpr int kSbarRows = 4;  // query centroids per workgroup: each kbar row fetched serves all of them

template <int D>
__global__ void __launch_bounds__(256)
sbar_kernel(const float* __restrict__ qbar, const float* __restrict__ kbar, const int32_t* __restrict__ k_offsets,
            int Cq, int Ck, float scale, float* __restrict__ sbar, float* __restrict__ mrow,
            bf16_t* __restrict__ q3) {
  __shared__ float q[kSbarRows][D];
  __shared__ float red[kSbarRows][4];
  const int a0 = blockIdx.x * kSbarRows, bh = blockIdx.y;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  for (int i = threadIdx.x; i < kSbarRows * D; i += 256) {
    const int a = a0 + i / D;
    q[i / D][i % D] = a < Cq ? qbar[((int64_t)bh * Cq + a) * D + i % D] : 0.f;
  }
  __syncthreads();
  if (q3) {
    constexpr int KSN = D / 16;
    for (int i = threadIdx.x; i < kSbarRows * D; i += 256) {
      const int a = a0 + i / D, k = i % D, ab = a >> 5, nab = (Cq + 31) >> 5;
      const float v = q[i / D][k];
      const bf16_t hi = f32_to_bf16(v);
      const float r1 = v - bf16_to_f32(hi);
      const bf16_t mid = f32_to_bf16(r1);
      const bf16_t lo = f32_to_bf16(r1 - bf16_to_f32(mid));
      const int ln = (a & 31) + 32 * ((k & 15) >> 3);
      bf16_t* dst = q3 + ((((int64_t)bh * nab + ab) * 3) * KSN + (k >> 4)) * 512 + ln * 8 + (k & 7);
      dst[0] = hi;
      dst[(int64_t)KSN * 512] = mid;
      dst[(int64_t)2 * KSN * 512] = lo;
    }
  }
  if (a0 >= Cq) return;
  const int32_t* off = k_offsets + (int64_t)bh * (Ck + 2);
  float mx[kSbarRows];
#pragma unroll
  for (int r = 0; r < kSbarRows; ++r) mx[r] = -INFINITY;
  for (int b = threadIdx.x; b < Ck; b += 256) {
    const float4* kb = reinterpret_cast<const float4*>(kbar + ((int64_t)bh * Ck + b) * D);
    float dot[kSbarRows];
#pragma unroll
    for (int r = 0; r < kSbarRows; ++r) dot[r] = 0.f;
#pragma unroll 8
    for (int t = 0; t < D / 4; ++t) {
      const float4 v = kb[t];
#pragma unroll
      for (int r = 0; r < kSbarRows; ++r) {  // one fma chain per (a, b), dims in order
        dot[r] = __builtin_fmaf(q[r][4 * t], v.x, dot[r]);
        dot[r] = __builtin_fmaf(q[r][4 * t + 1], v.y, dot[r]);
        dot[r] = __builtin_fmaf(q[r][4 * t + 2], v.z, dot[r]);
        dot[r] = __builtin_fmaf(q[r][4 * t + 3], v.w, dot[r]);
      }
    }
    const bool live = off[b + 1] > off[b];
#pragma unroll
    for (int r = 0; r < kSbarRows; ++r) {
      if (a0 + r >= Cq) break;
      const float sv = dot[r] * scale;
      sbar[((int64_t)bh * Cq + a0 + r) * Ck + b] = sv;
      if (live) mx[r] = fmaxf(mx[r], sv);
    }
  }
#pragma unroll
  for (int r = 0; r < kSbarRows; ++r) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) mx[r] = fmaxf(mx[r], __shfl_xor(mx[r], o));
    if (lane == 0) red[r][wave] = mx[r];
  }
  __syncthreads();
  if (threadIdx.x < kSbarRows && a0 + threadIdx.x < Cq) {
    const int r = threadIdx.x;
    mrow[(int64_t)bh * Cq + a0 + r] = fmaxf(fmaxf(red[r][0], red[r][1]), fmaxf(red[r][2], red[r][3]));
  }
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

// ---- bf16 inputs: the probe on the matrix cores -----------------------------------------
typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float f32x16;
__device__ __forceinline__ bf16x8 as_bf16x8(uint4 v) {
  union { uint4 u; bf16x8 b; } c;
  c.u = v;
  return c.b;
}

// |delta_j|^2 and -2 vbar . delta_j of every clustered key (delta_j = v_j - vbar of its cluster).
// One workgroup per (head, key cluster): 16 key slots x 16 lanes of 8 dims.
template <int D>
__global__ void __launch_bounds__(256)
value_stats_kernel(const float* __restrict__ vbar, const bf16_t* __restrict__ vp,
                   const int32_t* __restrict__ k_offsets, int64_t Nk, int64_t stat_stride, int Ck,
                   float* __restrict__ nd, float* __restrict__ dd) {
  constexpr int LPK = D / 8;  // lanes per key
  constexpr int SLOTS = 256 / LPK;
  const int b = blockIdx.x, bh = blockIdx.y;
  const int slot = threadIdx.x / LPK, lane = threadIdx.x % LPK;
  const int32_t* off = k_offsets + (int64_t)bh * (Ck + 2);
  const int start = off[b], end = off[b + 1];
  const float* vb = vbar + ((int64_t)bh * Ck + b) * D + lane * 8;
  float vbl[8];
#pragma unroll
  for (int k = 0; k < 8; ++k) vbl[k] = vb[k];
  const bf16_t* vh = vp + (int64_t)bh * Nk * D + lane * 8;
  constexpr int INFLIGHT = 4;  // independent key fetches per lane group
  for (int j0 = start + slot; j0 < end; j0 += INFLIGHT * SLOTS) {
    uint4 raw[INFLIGHT];
#pragma unroll
    for (int u = 0; u < INFLIGHT; ++u) {
      const int j = j0 + u * SLOTS;
      raw[u] = j < end ? *reinterpret_cast<const uint4*>(vh + (int64_t)j * D) : uint4{0u, 0u, 0u, 0u};
    }
#pragma unroll
    for (int u = 0; u < INFLIGHT; ++u) {
      const int j = j0 + u * SLOTS;
      const uint32_t w[4] = {raw[u].x, raw[u].y, raw[u].z, raw[u].w};
      float p_nd = 0.f, p_dd = 0.f;
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const float d0 = __uint_as_float(w[i] << 16) - vbl[2 * i];
        const float d1 = __uint_as_float(w[i] & 0xffff0000u) - vbl[2 * i + 1];
        p_nd = __builtin_fmaf(d0, d0, p_nd);
        p_dd = __builtin_fmaf(d0, vbl[2 * i], p_dd);
        p_nd = __builtin_fmaf(d1, d1, p_nd);
        p_dd = __builtin_fmaf(d1, vbl[2 * i + 1], p_dd);
      }
#pragma unroll
      for (int o = LPK / 2; o > 0; o >>= 1) {
        p_nd += __shfl_xor(p_nd, o);
        p_dd += __shfl_xor(p_dd, o);
      }
      if (lane == 0 && j < end) {
        nd[(int64_t)bh * stat_stride + j] = p_nd;
        dd[(int64_t)bh * stat_stride + j] = -2.0f * p_dd;
      }
    }
  }
}


// Block errors with the logits qbar_a . k_j on bf16 MFMAs (qbar in three exact bf16 pieces,
// so the logits carry fp32-level accuracy). One workgroup per (head, kProbeClusters consecutive
// key clusters, group of 128 query centroids); wave w owns query centroids 32w..32w+31 of the
// group and keeps their operand fragments in registers across those key clusters. The score
// tile is keys x centroids: a lane holds 16 keys of ONE query centroid per 32-key block, so
// the block error accumulates lane-locally.
// The 32-key blocks of the workgroup's key clusters form one sequence. Each block is copied
// once by the whole workgroup, straight from global memory into a ring of kProbeStages LDS
// buffers, kProbeStages - 1 blocks ahead of the one being computed (the kernel streams every
// key once and has few workgroups per CU: without that depth too few bytes are in flight),
// together with its per-key value statistics; the 16-byte chunks of a row are XOR-swizzled
// with the row index so that the operand reads of 32 rows do not collide. One barrier per
// block.
constexpr int kProbeClusters = 4;  // key clusters per workgroup
constexpr int kProbeStages = 4;    // LDS ring buffers

template <int D, bool VALUE_AWARE>
__global__ void __launch_bounds__(256)
block_error_mfma_kernel(const bf16_t* __restrict__ q3, const float* __restrict__ vbar, const bf16_t* __restrict__ kp,
                        const int32_t* __restrict__ k_offsets, const float* __restrict__ sbar,
                        const float* __restrict__ mrow, const float* __restrict__ nd, const float* __restrict__ dd,
                        int64_t Nk, int64_t stat_stride, int Cq, int Ck, float scale, float* __restrict__ scores) {
  constexpr int KSN = D / 16;
  constexpr int CPR = D / 8;             // 16-byte chunks per key row
  constexpr int RPI = 64 / CPR;          // key rows per copy instruction of a wave
  constexpr int NCH = 32 / RPI / 4;      // copy instructions per wave per block
  constexpr int TILE_B = 32 * D * 2;     // bytes of a block in LDS
  constexpr int LPB = NCH + (VALUE_AWARE ? 1 : 0);  // loads per wave per block
  constexpr int PF = kProbeStages - 1;   // blocks in flight ahead of the one computed
  static_assert(32 % (RPI * 4) == 0 && (CPR == 16 || CPR == 8), "tile split / swizzle assume d = 64 or 128");
  __shared__ __attribute__((aligned(1024))) unsigned char ktile[kProbeStages][TILE_B];
  __shared__ __attribute__((aligned(256))) float stat[kProbeStages][64];  // [|delta|^2 x 32, vbar.delta x 32]
  // scores of the workgroup's key clusters, per wave [query centroid][key cluster]: a row leaves
  // as ONE 16-byte store at the end instead of kProbeClusters 4-byte stores a score row apart
  __shared__ __attribute__((aligned(16))) float sc[4][32][kProbeClusters];
  const int bh = blockIdx.y, tid = threadIdx.x;
  const int lane = tid & 63, li = lane & 31, lh = lane >> 5;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int ab = blockIdx.z * 4 + wave, nab = (Cq + 31) >> 5;
  const bool wave_on = ab < nab;  // waves past the last centroid block still help copying
  const int a = 32 * ab + li;
  const bool live = wave_on && a < Cq;
  const int32_t* off = k_offsets + (int64_t)bh * (Ck + 2);
  const int b_lo = blockIdx.x * kProbeClusters, b_end = min(b_lo + kProbeClusters, Ck);
  // empty key clusters score 0 (each wave reads and writes its own part of sc only)
  if (lh == 0) {
#pragma unroll
    for (int i = 0; i < kProbeClusters; ++i) sc[wave][li][i] = 0.f;
  }
  auto flush = [&]() {  // the wave's scores to global memory
    if (!live || lh != 0) return;
    float* dst = scores + ((int64_t)bh * Cq + a) * Ck + b_lo;
    if (b_end - b_lo == kProbeClusters && (Ck % 4) == 0) {
      *reinterpret_cast<float4*>(dst) = *reinterpret_cast<const float4*>(&sc[wave][li][0]);
    } else {
      for (int i = 0; i < b_end - b_lo; ++i) dst[i] = sc[wave][li][i];
    }
  };
  bf16x8 bq[3][KSN];
  if (wave_on) {
    const bf16_t* src = q3 + (((int64_t)bh * nab + ab) * 3 * KSN) * 512 + lane * 8;
#pragma unroll
    for (int pc = 0; pc < 3; ++pc)
#pragma unroll
      for (int s = 0; s < KSN; ++s)
        bq[pc][s] = as_bf16x8(*reinterpret_cast<const uint4*>(src + (pc * KSN + s) * 512));
  }
  const float m_a = live ? mrow[(int64_t)bh * Cq + a] : 0.f;
  // exponentials as exp2 with the constants folded: e^(x scale - m) = 2^(x scale2 - m2)
  constexpr float kLog2e = 1.4426950408889634f;
  const float scale2 = scale * kLog2e, neg_m2 = -m_a * kLog2e, cap2 = kMaxExponent * kLog2e;
  SVGEAR_WAIT_VMCNT(0);  // from here on vmcnt counts the block copies only
  const bf16_t* kh = kp + (int64_t)bh * Nk * D;
  const float* ndh = nd + (int64_t)bh * stat_stride;
  const float* ddh = dd + (int64_t)bh * stat_stride;
  const uint32_t lds_k = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) unsigned char*)&ktile[0][0];
  const uint32_t lds_s = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) float*)&stat[0][0];

  // position in the sequence of blocks: cluster b, keys j0 .. of [start, end)
  struct Cursor { int b, start, end, j0; };
  auto seek = [&](Cursor& c) {  // first non-empty cluster at or after c.b
    while (c.b < b_end) {
      c.start = off[c.b];
      c.end = off[c.b + 1];
      if (c.end > c.start) break;
      ++c.b;
    }
    c.j0 = c.start;
  };
  auto advance = [&](Cursor& c) {
    c.j0 += 32;
    if (c.j0 >= c.end) {
      ++c.b;
      seek(c);
    }
  };
  // row r of a block keeps its 16-byte chunk c at position c ^ swz(r)
  auto swz = [](int r) { return CPR == 16 ? (r & 15) : ((r >> 1) & 7); };
  auto issue = [&](const Cursor& c, int buf) {  // rows past the cluster's end repeat its last key
#pragma unroll
    for (int i = 0; i < NCH; ++i) {
      const int inst = wave * NCH + i;
      const int row = inst * RPI + lane / CPR;
      const int chunk = (lane % CPR) ^ swz(row);
      const int jr = min(c.j0 + row, c.end - 1);
      async_copy_16B(kh + (int64_t)jr * D + chunk * 8,
                     __builtin_amdgcn_readfirstlane(lds_k + buf * TILE_B + inst * 1024));
    }
    if (VALUE_AWARE) {  // every wave copies the 64 statistics (same values to the same words)
      const int j = min(c.j0 + li, c.end - 1);
      async_copy_4B((lh ? ddh : ndh) + j, __builtin_amdgcn_readfirstlane(lds_s + buf * 256));
    }
  };

  Cursor fc{b_lo, 0, 0, 0};  // next block to copy
  seek(fc);
  if (fc.b >= b_end) {  // nothing but empty clusters (uniform over the workgroup)
    flush();
    return;
  }
  Cursor cc = fc;             // block being computed
  int issued = 0;
  for (; issued < PF && fc.b < b_end; ++issued) {
    issue(fc, issued);
    advance(fc);
  }
  float E = 0.f, W = 0.f, nvb = 0.f;
  for (int k = 0; cc.b < b_end; ++k) {
    // block k has landed once at most the copies of the later blocks are outstanding
    const int ahead = issued - k - 1;
    if (ahead >= 2) SVGEAR_WAIT_VMCNT(2 * LPB);
    else if (ahead == 1) SVGEAR_WAIT_VMCNT(LPB);
    else SVGEAR_WAIT_VMCNT(0);
    __syncthreads();  // everyone's part of block k is in LDS; everyone is done with block k - 1
    if (fc.b < b_end) {
      issue(fc, issued % kProbeStages);
      advance(fc);
      ++issued;
    }
    const int buf = k % kProbeStages;
    if (cc.j0 == cc.start) {  // first block of key cluster cc.b
      E = 0.f;
      W = live ? __expf(fminf(sbar[((int64_t)bh * Cq + a) * Ck + cc.b] - m_a, kMaxExponent)) : 0.f;
      nvb = 0.f;
      if (VALUE_AWARE) {  // |vbar_b|^2: D/64 dims per lane, then across the wave
        const float* vb = vbar + ((int64_t)bh * Ck + cc.b) * D;
#pragma unroll
        for (int t = 0; t < D / 64; ++t) nvb = __builtin_fmaf(vb[lane + 64 * t], vb[lane + 64 * t], nvb);
#pragma unroll
        for (int o = 32; o > 0; o >>= 1) nvb += __shfl_xor(nvb, o);
      }
    }
    if (wave_on) {
      // A operand: key row li of the block, dims 16s + 8lh .. = chunk 2s + lh
      const unsigned char* kr = &ktile[buf][li * (D * 2)];
      const int key = swz(li);
      f32x16 acc;
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[r] = 0.f;
#pragma unroll
      for (int s = 0; s < KSN; ++s) {
        const bf16x8 ak = as_bf16x8(*reinterpret_cast<const uint4*>(kr + (((2 * s + lh) ^ key) << 4)));
#pragma unroll
        for (int pc = 0; pc < 3; ++pc) acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ak, bq[pc][s], acc, 0, 0, 0);
      }
      // register r is key j0 + 8(r/4) + 4lh + r%4, query centroid a. Per key, with u = W - w:
      //   |W vbar - w v_j|^2 = u (u |vbar|^2 - 2 w vbar.delta_j) + w^2 |delta_j|^2
      auto rank = [&](auto tail_tag) __attribute__((always_inline)) {
        constexpr bool TAIL = decltype(tail_tag)::value;  // only a cluster's last block has unused rows
#pragma unroll
        for (int g = 0; g < 4; ++g) {
          const int jb = cc.j0 + 8 * g + 4 * lh;
          float nn[4] = {0.f, 0.f, 0.f, 0.f}, dl[4] = {0.f, 0.f, 0.f, 0.f};
          if (VALUE_AWARE) {
            const float4 n4 = *reinterpret_cast<const float4*>(&stat[buf][8 * g + 4 * lh]);
            const float4 d4 = *reinterpret_cast<const float4*>(&stat[buf][32 + 8 * g + 4 * lh]);
            nn[0] = n4.x; nn[1] = n4.y; nn[2] = n4.z; nn[3] = n4.w;
            dl[0] = d4.x; dl[1] = d4.y; dl[2] = d4.z; dl[3] = d4.w;
          }
#pragma unroll
          for (int r = 0; r < 4; ++r) {
            if (!TAIL || jb + r < cc.end) {
              const float w = __builtin_amdgcn_exp2f(fminf(__builtin_fmaf(acc[4 * g + r], scale2, neg_m2), cap2));
              const float u = W - w;
              if (VALUE_AWARE) {
                E = __builtin_fmaf(u, __builtin_fmaf(w, dl[r], u * nvb), E);
                E = __builtin_fmaf(w * w, nn[r], E);
              } else {
                E = __builtin_fmaf(u, u, E);
              }
            }
          }
        }
      };
      if (cc.j0 + 32 <= cc.end) rank(std::false_type{});
      else rank(std::true_type{});
      if (cc.j0 + 32 >= cc.end) {  // last block of the cluster
        const float Et = E + __shfl_xor(E, 32);
        if (lh == 0) sc[wave][li][cc.b - b_lo] = Et / (float)(cc.end - cc.start);
      }
    }
    advance(cc);
  }
  flush();
}

}  // namespace

// Centroid logits and their row maxima alone (no block errors).
int run_sbar(const float* qbar, const float* kbar, const int32_t* k_offsets, int BH, int d, int Cq, int Ck,
             float scale, float* sbar, float* mrow, hipStream_t s) {
  if (d == 64)
    sbar_kernel<64><<<dim3((unsigned)ceil_div(Cq, kSbarRows), BH), 256, 0, s>>>(qbar, kbar, k_offsets, Cq, Ck, scale,
                                                                              sbar, mrow, nullptr);
  else
    sbar_kernel<128><<<dim3((unsigned)ceil_div(Cq, kSbarRows), BH), 256, 0, s>>>(qbar, kbar, k_offsets, Cq, Ck, scale,
                                                                               sbar, mrow, nullptr);
  SVGEAR_LAUNCH_CHECK();
  return SVGEAR_OK;
}

int run_probe(const float* qbar, const float* kbar, const float* vbar, const void* kp, const void* vp,
              svgear_dtype dt, const int32_t* k_offsets, int BH, int64_t Nk, int d, int Cq, int Ck, float scale,
              bool value_aware, float* scores, float* sbar, float* mrow, bf16_t* q3, float* nd, float* dd,
              hipStream_t s) {
  const bool mfma = dt == SVGEAR_BF16;
  const int rows = mfma ? (int)align_up(Cq, 32) : Cq;
  if (d == 64)
    sbar_kernel<64><<<dim3((unsigned)ceil_div(rows, kSbarRows), BH), 256, 0, s>>>(qbar, kbar, k_offsets, Cq, Ck, scale,
                                                                                sbar, mrow, mfma ? q3 : nullptr);
  else
    sbar_kernel<128><<<dim3((unsigned)ceil_div(rows, kSbarRows), BH), 256, 0, s>>>(qbar, kbar, k_offsets, Cq, Ck, scale,
                                                                                 sbar, mrow, mfma ? q3 : nullptr);
  SVGEAR_LAUNCH_CHECK();
  if (mfma) {
    const int64_t stat_stride = probe_stat_stride(Nk);
    const bf16_t* k16 = static_cast<const bf16_t*>(kp);
    const bf16_t* v16 = static_cast<const bf16_t*>(vp);
    const dim3 gs(Ck, BH), gb((unsigned)ceil_div(Ck, kProbeClusters), BH, (unsigned)ceil_div(ceil_div(Cq, 32), 4));
    if (value_aware) {
      if (d == 64) value_stats_kernel<64><<<gs, 256, 0, s>>>(vbar, v16, k_offsets, Nk, stat_stride, Ck, nd, dd);
      else value_stats_kernel<128><<<gs, 256, 0, s>>>(vbar, v16, k_offsets, Nk, stat_stride, Ck, nd, dd);
      SVGEAR_LAUNCH_CHECK();
    }
#define SVGEAR_PM(D, VA)                                                                                     \
  block_error_mfma_kernel<D, VA><<<gb, 256, 0, s>>>(q3, vbar, k16, k_offsets, sbar, mrow, nd, dd, Nk, stat_stride, \
                                                    Cq, Ck, scale, scores)
    if (d == 64) { if (value_aware) SVGEAR_PM(64, true); else SVGEAR_PM(64, false); }
    else { if (value_aware) SVGEAR_PM(128, true); else SVGEAR_PM(128, false); }
#undef SVGEAR_PM
    SVGEAR_LAUNCH_CHECK();
    return SVGEAR_OK;
  }
  const int threads = Cq >= 256 ? 256 : (int)align_up(Cq, 64);
  dim3 grid(Ck, BH, (unsigned)ceil_div(Cq, 256));
#define SVGEAR_PB(T, D, VA)                                                                                   \
  block_error_kernel<T, D, VA><<<grid, threads, 0, s>>>(qbar, vbar, static_cast<const T*>(kp),                \
                                                        static_cast<const T*>(vp), k_offsets, sbar, mrow, Nk, \
                                                        Cq, Ck, scale, scores)
  if (d == 64) { if (value_aware) SVGEAR_PB(float, 64, true); else SVGEAR_PB(float, 64, false); }
  else { if (value_aware) SVGEAR_PB(float, 128, true); else SVGEAR_PB(float, 128, false); }
#undef SVGEAR_PB
  SVGEAR_LAUNCH_CHECK();
  return SVGEAR_OK;
}

}  // namespace svgear
