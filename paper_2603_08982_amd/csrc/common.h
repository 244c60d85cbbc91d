// Internal helpers shared by the gfx950 kernels of libsvgear. Not part of the C ABI.
#pragma once

#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include "../../include/svgear.h"

namespace svgear {

// ---- host-side error plumbing --------------------------------------------------------
void set_last_hip_error(hipError_t e);

#define SVGEAR_HIP_TRY(expr)                \
  do {                                      \
    hipError_t _e = (expr);                 \
    if (_e != hipSuccess) {                 \
      ::svgear::set_last_hip_error(_e);     \
      return SVGEAR_ERR_HIP;                \
    }                                       \
  } while (0)

#define SVGEAR_LAUNCH_CHECK() SVGEAR_HIP_TRY(hipGetLastError())

static inline size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }
static inline int64_t ceil_div(int64_t a, int64_t b) { return (a + b - 1) / b; }

// Bump allocator over the caller's workspace (256-byte granules).
struct Workspace {
  char* base;
  size_t size;
  size_t used = 0;
  Workspace(void* p, size_t n) : base(static_cast<char*>(p)), size(n) {}
  template <typename T>
  T* take(size_t count) {
    size_t bytes = align_up(count * sizeof(T), 256);
    T* r = reinterpret_cast<T*>(base + used);
    used += bytes;
    return r;
  }
  bool ok() const { return used <= size; }
};

static inline size_t esize(svgear_dtype dt) { return dt == SVGEAR_F32 ? 4 : 2; }

// ---- device-side element access ------------------------------------------------------
typedef uint16_t bf16_t;  // raw bf16 bit pattern

__device__ __forceinline__ float bf16_to_f32(bf16_t v) { return __uint_as_float(((uint32_t)v) << 16); }

// round-to-nearest-even fp32 -> bf16 (NaN kept quiet)
__device__ __forceinline__ bf16_t f32_to_bf16(float f) {
  uint32_t u = __float_as_uint(f);
  if ((u & 0x7fffffffu) > 0x7f800000u) return (bf16_t)((u >> 16) | 0x40);
  u += 0x7fffu + ((u >> 16) & 1u);
  return (bf16_t)(u >> 16);
}

template <typename T>
struct Elem;
template <>
struct Elem<float> {
  static __device__ __forceinline__ float load(const float* p) { return *p; }
  static __device__ __forceinline__ void store(float* p, float v) { *p = v; }
};
template <>
struct Elem<bf16_t> {
  static __device__ __forceinline__ float load(const bf16_t* p) { return bf16_to_f32(*p); }
  static __device__ __forceinline__ void store(bf16_t* p, float v) { *p = f32_to_bf16(v); }
};

// Loads 4 consecutive elements as floats (p must be 16-byte aligned for float, 8 for bf16).
__device__ __forceinline__ float4 load4(const float* p) { return *reinterpret_cast<const float4*>(p); }
__device__ __forceinline__ float4 load4(const bf16_t* p) {
  uint2 r = *reinterpret_cast<const uint2*>(p);
  return make_float4(__uint_as_float(r.x << 16), __uint_as_float(r.x & 0xffff0000u),
                     __uint_as_float(r.y << 16), __uint_as_float(r.y & 0xffff0000u));
}

// Batch*head decomposition for strided [B,H,N,d] tensors.
struct Strides {
  int64_t b, h, n;
};
__device__ __forceinline__ int64_t head_base(const Strides& s, int bh, int H) {
  return (int64_t)(bh / H) * s.b + (int64_t)(bh % H) * s.h;
}

// ---- asynchronous global -> LDS copies -------------------------------------------------
// 16 (4) bytes per lane from global memory straight into LDS: the wave's 64 lanes fill 1 KB
// (256 B) starting at the wave-uniform LDS byte address `lds_addr`, lane l at lds_addr + 16 l
// (4 l). Written as inline assembly so that the compiler does not treat every later LDS read
// as dependent on the copy (it would drain the copies before the first read of each tile);
// completion is tracked by hand with SVGEAR_WAIT_VMCNT.
__device__ __forceinline__ void async_copy_16B(const void* gptr, uint32_t lds_addr) {
  asm volatile("s_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, off\n"
               :
               : "v"(gptr), "s"(lds_addr)
               : "memory", "m0");
}
// Same copy with the global address given as a wave-uniform base plus a 32-bit byte offset
// per lane (no 64-bit vector arithmetic).
__device__ __forceinline__ void async_copy_16B(const void* gbase, uint32_t byte_off, uint32_t lds_addr) {
  asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1\n"
               :
               : "v"(byte_off), "s"(gbase), "s"(lds_addr)
               : "memory", "m0");
}
__device__ __forceinline__ void async_copy_4B(const void* gptr, uint32_t lds_addr) {
  asm volatile("s_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dword %0, off\n"
               :
               : "v"(gptr), "s"(lds_addr)
               : "memory", "m0");
}
// vmcnt(n) with expcnt and lgkmcnt left unconstrained (gfx9 s_waitcnt encoding)
#define SVGEAR_WAIT_VMCNT(n) __builtin_amdgcn_s_waitcnt(((n) & 0xF) | (((n) >> 4) << 14) | (7 << 4) | (15 << 8))

// ---- internal cross-file entry points ------------------------------------------------
// Stable counting sort of token indices by label (tail tokens = pseudo-cluster C).
// chunk_hist: scratch of BH * sort_chunks(N) * (C+1) int32.
constexpr int kSortChunk = 2048;
static inline int64_t sort_chunks(int64_t N) { return ceil_div(N, kSortChunk); }
// tiles (optional, [BH][tile_cap], tile_cap >= N / tile_len + C + 1): the sorted order cut into
// tiles of at most tile_len positions that never straddle a cluster: tile
// t = floor(offsets[c] / tile_len) + c + j is positions offsets[c] + tile_len j .. of cluster c, stored
// as (c, first position, end position, 0); indices no cluster uses hold c = -1.
// rank (optional, [BH][N]): the position of every token in the sorted order (perm's inverse).
int sort_labels(const int32_t* labels, int BH, int64_t N, int64_t n_tail, int C, int32_t* perm,
                int32_t* offsets, int32_t* chunk_hist, hipStream_t s, int4* tiles = nullptr, int tile_cap = 0,
                int tile_len = 64, int32_t* rank = nullptr);


// Per-head length of the probe's per-key statistic arrays (padded so that 16-byte reads
// starting at any key stay inside the array).
static inline int64_t probe_stat_stride(int64_t Nk) { return (int64_t)align_up((size_t)Nk + 64, 64); }

}  // namespace svgear
