// Cluster permutation: stable counting sort of token indices by cluster label, row
// gather into cluster-contiguous order, and the inverse row scatter.
// Paper: Motivation, "Structured Redundancy in Attention Computation" (tokens of a cluster
// are laid out contiguously so the attention map becomes a grid of blocks).
//
// The sort is integer-only and deterministic: per-chunk histograms (LDS integer atomics),
// an exclusive scan over (cluster, chunk), then a stable in-chunk ranking without atomics.
#include "common.h"

#include <mutex>

namespace svgear {

namespace {

constexpr int kThreads = 256;

__device__ __forceinline__ int token_label(const int32_t* labels, int64_t i, int64_t nv, int C) {
  if (i >= nv) return C;  // tail pseudo-cluster
  int l = labels[i];
  return l < 0 ? 0 : (l >= C ? C - 1 : l);  // out-of-range labels are clamped
}

__global__ void __launch_bounds__(kThreads)
hist_kernel(const int32_t* __restrict__ labels, int64_t N, int64_t nv, int C, int nchunks,
            int32_t* __restrict__ chunk_hist) {
  extern __shared__ int32_t h[];
  const int bh = blockIdx.y, chunk = blockIdx.x;
  for (int c = threadIdx.x; c <= C; c += kThreads) h[c] = 0;
  __syncthreads();
  const int64_t lo = (int64_t)chunk * kSortChunk;
  const int64_t hi = min(N, lo + kSortChunk);
  const int32_t* lab = labels + (int64_t)bh * nv;
  for (int64_t i = lo + threadIdx.x; i < hi; i += kThreads) atomicAdd(&h[token_label(lab, i, nv, C)], 1);
  __syncthreads();
  int32_t* out = chunk_hist + ((int64_t)bh * nchunks + chunk) * (C + 1);
  for (int c = threadIdx.x; c <= C; c += kThreads) out[c] = h[c];
}

// Turns per-chunk histograms into per-chunk start positions and writes the offsets.
__global__ void __launch_bounds__(kThreads)
scan_kernel(int32_t* __restrict__ chunk_hist, int64_t N, int C, int nchunks,
            int32_t* __restrict__ offsets, int4* __restrict__ tiles, int tile_cap, int tile_len) {
  extern __shared__ int32_t tot[];  // C+1 totals, then C+1 exclusive offsets
  int32_t* offs = tot + (C + 1);
  const int bh = blockIdx.x;
  int32_t* hist = chunk_hist + (int64_t)bh * nchunks * (C + 1);
  // label totals: loads only, eight in flight per thread
  for (int c = threadIdx.x; c <= C; c += kThreads) {
    int32_t run = 0;
    int k = 0;
    for (; k + 8 <= nchunks; k += 8) {
      int32_t v[8];
#pragma unroll
      for (int u = 0; u < 8; ++u) v[u] = hist[(int64_t)(k + u) * (C + 1) + c];
#pragma unroll
      for (int u = 0; u < 8; ++u) run += v[u];
    }
    for (; k < nchunks; ++k) run += hist[(int64_t)k * (C + 1) + c];
    tot[c] = run;
  }
  __syncthreads();
  // exclusive scan of the C+1 totals: each thread takes a contiguous run of labels
  {
    const int per = (C + 1 + kThreads - 1) / kThreads;
    const int lo = threadIdx.x * per, hi = lo + per < C + 1 ? lo + per : C + 1;
    int32_t sum = 0;
    for (int c = lo; c < hi; ++c) sum += tot[c];
    __shared__ int32_t part[kThreads];
    part[threadIdx.x] = sum;
    __syncthreads();
    for (int o = 1; o < kThreads; o <<= 1) {
      const int32_t t = threadIdx.x >= o ? part[threadIdx.x - o] : 0;
      __syncthreads();
      part[threadIdx.x] += t;
      __syncthreads();
    }
    int32_t run = part[threadIdx.x] - sum;
    for (int c = lo; c < hi; ++c) {
      offs[c] = run;
      run += tot[c];
    }
  }
  __syncthreads();
  // start of every (chunk, label) segment: offset of the label plus the label's count in the
  // earlier chunks; eight chunks per round (loads first, then the stores)
  int32_t* o = offsets + (int64_t)bh * (C + 2);
  for (int c = threadIdx.x; c <= C; c += kThreads) {
    int32_t run = offs[c];
    o[c] = run;
    int k = 0;
    for (; k + 8 <= nchunks; k += 8) {
      int32_t v[8];
#pragma unroll
      for (int u = 0; u < 8; ++u) v[u] = hist[(int64_t)(k + u) * (C + 1) + c];
#pragma unroll
      for (int u = 0; u < 8; ++u) {
        hist[(int64_t)(k + u) * (C + 1) + c] = run;
        run += v[u];
      }
    }
    for (; k < nchunks; ++k) {
      const int32_t v = hist[(int64_t)k * (C + 1) + c];
      hist[(int64_t)k * (C + 1) + c] = run;
      run += v;
    }
  }
  if (threadIdx.x == 0) o[C + 1] = (int32_t)N;
  if (tiles) {  // tiles of the clusters (see sort_labels in common.h)
    int4* ta = tiles + (int64_t)bh * tile_cap;
    for (int c = threadIdx.x; c < C; c += kThreads) {
      const int start = offs[c] / tile_len + c, nt = (tot[c] + tile_len - 1) / tile_len;
      const int next = c + 1 < C ? offs[c + 1] / tile_len + c + 1 : tile_cap;
      const int end = offs[c] + tot[c];
      for (int j = 0; j < nt; ++j) {
        const int p0 = offs[c] + j * tile_len;
        ta[start + j] = make_int4(c, p0, p0 + tile_len < end ? p0 + tile_len : end, 0);
      }
      for (int j = start + nt; j < next; ++j) ta[j] = make_int4(-1, 0, 0, 0);
    }
  }
}

// Stable placement: tokens of a chunk are taken 256 at a time; inside a wave the rank of a
// token among the lanes with the same label comes from ballots over the label bits, and the
// four waves of the workgroup claim their positions one after the other (wave order = token
// order), so equal labels keep ascending token order without any atomic.
__global__ void __launch_bounds__(kThreads)
scatter_kernel(const int32_t* __restrict__ labels, int64_t N, int64_t nv, int C, int nchunks,
               const int32_t* __restrict__ chunk_hist, int32_t* __restrict__ perm, int32_t* __restrict__ rank_out) {
  extern __shared__ int32_t base[];  // C+1 next free position per label
  const int bh = blockIdx.y, chunk = blockIdx.x;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int32_t* hist = chunk_hist + ((int64_t)bh * nchunks + chunk) * (C + 1);
  for (int c = threadIdx.x; c <= C; c += kThreads) base[c] = hist[c];
  const int32_t* lab = labels + (int64_t)bh * nv;
  int32_t* out = perm + (int64_t)bh * N;
  const int64_t lo = (int64_t)chunk * kSortChunk;
  const int nbits = 32 - __clz(C + 1);
  const uint64_t below = (1ull << lane) - 1ull;
  __syncthreads();
  for (int sub = 0; sub < kSortChunk / kThreads; ++sub) {
    if (lo + (int64_t)sub * kThreads >= N) break;
    const int64_t i = lo + (int64_t)sub * kThreads + threadIdx.x;
    const bool valid = i < N;
    const int my = valid ? token_label(lab, i, nv, C) : (C + 1);
    uint64_t same = ~0ull;
    for (int bit = 0; bit < nbits; ++bit) {
      const uint64_t vote = __ballot((my >> bit) & 1);
      same &= ((my >> bit) & 1) ? vote : ~vote;
    }
    const int rank = __popcll(same & below);
    const int total = __popcll(same);
    for (int w = 0; w < kThreads / 64; ++w) {
      if (wave == w && valid) {
        const int b = base[my];
        out[b + rank] = (int32_t)i;
        if (rank_out) rank_out[(int64_t)bh * N + i] = b + rank;
        if (rank == total - 1) base[my] = b + total;  // issued after every lane's read of base
      }
      __syncthreads();
    }
  }
}

// dst[bh][p][:] = src[b,h,perm[p],:] in 16-byte units.
__global__ void __launch_bounds__(kThreads)
gather_rows_kernel(const uint4* __restrict__ src, Strides st_units, int H, const int32_t* __restrict__ perm,
                   int64_t N, int row_units, uint4* __restrict__ dst) {
  const int bh = blockIdx.y;
  const int64_t u = (int64_t)blockIdx.x * kThreads + threadIdx.x;
  if (u >= N * row_units) return;
  const int64_t p = u / row_units;
  const int v = (int)(u % row_units);
  const int64_t row = perm[(int64_t)bh * N + p];
  dst[((int64_t)bh * N + p) * row_units + v] = src[head_base(st_units, bh, H) + row * st_units.n + v];
}

// dst[b,h,perm[p],:] = src[bh][p][:]
__global__ void __launch_bounds__(kThreads)
scatter_rows_kernel(const uint4* __restrict__ src, const int32_t* __restrict__ perm, int64_t N,
                    int row_units, uint4* __restrict__ dst, Strides st_units, int H) {
  const int bh = blockIdx.y;
  const int64_t u = (int64_t)blockIdx.x * kThreads + threadIdx.x;
  if (u >= N * row_units) return;
  const int64_t p = u / row_units;
  const int v = (int)(u % row_units);
  const int64_t row = perm[(int64_t)bh * N + p];
  dst[head_base(st_units, bh, H) + row * st_units.n + v] = src[((int64_t)bh * N + p) * row_units + v];
}

bool strides_ok(const int64_t st[3], size_t es, const void* p) {
  if (!st) return false;
  for (int i = 0; i < 3; ++i)
    if (st[i] < 0 || (st[i] * (int64_t)es) % 16 != 0) return false;
  return (reinterpret_cast<uintptr_t>(p) % 16) == 0;
}

}  // namespace

int sort_labels(const int32_t* labels, int BH, int64_t N, int64_t n_tail, int C, int32_t* perm,
                int32_t* offsets, int32_t* chunk_hist, hipStream_t s, int4* tiles, int tile_cap, int tile_len,
                int32_t* rank) {
  const int nchunks = (int)sort_chunks(N);
  const int64_t nv = N - n_tail;
  dim3 grid(nchunks, BH);
  hist_kernel<<<grid, kThreads, (C + 1) * sizeof(int32_t), s>>>(labels, N, nv, C, nchunks, chunk_hist);
  SVGEAR_LAUNCH_CHECK();
  // two tables of C+1 counters: a few bytes over the default 64 KB at the largest C
  SVGEAR_HIP_TRY(hipFuncSetAttribute(reinterpret_cast<const void*>(scan_kernel),
                                     hipFuncAttributeMaxDynamicSharedMemorySize,
                                     (int)(2 * (C + 1) * sizeof(int32_t))));
  if (tiles && (tile_len < 1 || tile_cap < (int)(N / tile_len) + C + 1)) return SVGEAR_ERR_INVALID;
  scan_kernel<<<BH, kThreads, 2 * (C + 1) * sizeof(int32_t), s>>>(chunk_hist, N, C, nchunks, offsets, tiles, tile_cap,
                                                                  tile_len);
  SVGEAR_LAUNCH_CHECK();
  scatter_kernel<<<grid, kThreads, (C + 1) * sizeof(int32_t), s>>>(labels, N, nv, C, nchunks,
                                                                            chunk_hist, perm, rank);
  SVGEAR_LAUNCH_CHECK();
  return SVGEAR_OK;
}

}  // namespace svgear

using namespace svgear;

extern "C" size_t svgear_permute_workspace(int B, int H, int64_t N, int C) {
  if (B <= 0 || H <= 0 || N <= 0 || C <= 0) return 0;
  return align_up((size_t)B * H * sort_chunks(N) * (C + 1) * sizeof(int32_t), 256);
}

namespace svgear {
namespace {

// dst[k][bh][p][:] = src[k][b,h,perm[p],:] for every tensor k
int gather_tensors(const int32_t* perm, int BH, int H, int64_t N, int n_tensors, const void* const* src,
                   const int64_t (*sstride)[3], void* const* dst, svgear_dtype dt, int d, hipStream_t s) {
  const int row_units = (int)(d * esize(dt) / 16);
  const int upe = (int)(16 / esize(dt));  // elements per 16-byte unit
  for (int k = 0; k < n_tensors; ++k) {
    Strides st{sstride[k][0] / upe, sstride[k][1] / upe, sstride[k][2] / upe};
    dim3 grid((unsigned)ceil_div(N * row_units, kThreads), BH);
    gather_rows_kernel<<<grid, kThreads, 0, s>>>(static_cast<const uint4*>(src[k]), st, H, perm, N, row_units,
                                                 static_cast<uint4*>(dst[k]));
    SVGEAR_LAUNCH_CHECK();
  }
  return SVGEAR_OK;
}

}  // namespace
}  // namespace svgear

extern "C" int svgear_permute(const int32_t* labels, int B, int H, int64_t N, int64_t n_tail, int C,
                              int32_t* perm, int32_t* offsets, int n_tensors, const void* const* src,
                              const int64_t (*sstride)[3], void* const* dst, svgear_dtype dt, int d,
                              void* ws, size_t ws_bytes, void* stream) {
  if (!labels || !perm || !offsets || B <= 0 || H <= 0 || N <= 0 || n_tail < 0 || n_tail >= N || C <= 0 ||
      C > N - n_tail || N > INT32_MAX / 2 || n_tensors < 0 || n_tensors > 4 || C > 8192)
    return SVGEAR_ERR_INVALID;
  if (dt != SVGEAR_F32 && dt != SVGEAR_BF16) return SVGEAR_ERR_INVALID;
  if (n_tensors > 0) {
    if (!src || !dst || !sstride || (d != 64 && d != 128)) return SVGEAR_ERR_INVALID;
    for (int k = 0; k < n_tensors; ++k)
      if (!src[k] || !dst[k] || !strides_ok(sstride[k], esize(dt), src[k]) ||
          reinterpret_cast<uintptr_t>(dst[k]) % 16)
        return SVGEAR_ERR_INVALID;
  }
  if (!ws || ws_bytes < svgear_permute_workspace(B, H, N, C)) return SVGEAR_ERR_WORKSPACE;
  hipStream_t s = static_cast<hipStream_t>(stream);
  const int BH = B * H;
  int rc = sort_labels(labels, BH, N, n_tail, C, perm, offsets, static_cast<int32_t*>(ws), s);
  if (rc != SVGEAR_OK) return rc;
  return gather_tensors(perm, BH, H, N, n_tensors, src, sstride, dst, dt, d, s);
}

// ---- the same call for callers that cannot allocate -----------------------------------------
// The sort's chunk histograms live in a file-scope device array instead of a caller workspace.
// In host code the array's NAME is only a stand-in for the symbol; its device address is taken
// once per device with hipGetSymbolAddress and that address is what the kernels receive.
namespace svgear {
namespace {

constexpr size_t kStaticScratchBytes = (size_t)8 << 20;
constexpr int kMaxDevices = 64;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];
std::mutex g_scratch_mutex;
void* g_scratch_ptr[kMaxDevices] = {};

// Device address of `scratch` on the current device (looked up on the first call there).
int static_scratch(void** out) {
  int dev = -1;
  SVGEAR_HIP_TRY(hipGetDevice(&dev));
  if (dev < 0 || dev >= kMaxDevices) return SVGEAR_ERR_UNSUPPORTED;
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (!g_scratch_ptr[dev]) {
    void* p = nullptr;
    SVGEAR_HIP_TRY(hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)));
    if (!p) return SVGEAR_ERR_HIP;
    g_scratch_ptr[dev] = p;
  }
  *out = g_scratch_ptr[dev];
  return SVGEAR_OK;
}

}  // namespace
}  // namespace svgear

extern "C" size_t svgear_permute_static_capacity(void) { return kStaticScratchBytes; }

extern "C" int svgear_permute_static(const int32_t* labels, int B, int H, int64_t N, int64_t n_tail, int C,
                                     int32_t* perm, int32_t* offsets, int n_tensors, const void* const* src,
                                     const int64_t (*sstride)[3], void* const* dst, svgear_dtype dt, int d,
                                     void* stream) {
  if (B <= 0 || H <= 0 || N <= 0 || C <= 0) return SVGEAR_ERR_INVALID;
  if (svgear_permute_workspace(B, H, N, C) > kStaticScratchBytes) return SVGEAR_ERR_WORKSPACE;
  void* ptr = nullptr;
  const int rc = static_scratch(&ptr);
  if (rc != SVGEAR_OK) return rc;
  // every counter of the histogram area in use is written by hist_kernel before it is read,
  // so what an earlier call left in the array does not matter
  return svgear_permute(labels, B, H, N, n_tail, C, perm, offsets, n_tensors, src, sstride, dst, dt, d, ptr,
                        kStaticScratchBytes, stream);
}

extern "C" int svgear_permute_rows(const int32_t* perm, int B, int H, int64_t N, int n_tensors,
                                   const void* const* src, const int64_t (*sstride)[3], void* const* dst,
                                   svgear_dtype dt, int d, void* stream) {
  if (!perm || B <= 0 || H <= 0 || N <= 0 || N > INT32_MAX / 2 || n_tensors < 1 || n_tensors > 4 || !src || !dst ||
      !sstride || (d != 64 && d != 128) || (dt != SVGEAR_F32 && dt != SVGEAR_BF16))
    return SVGEAR_ERR_INVALID;
  for (int k = 0; k < n_tensors; ++k)
    if (!src[k] || !dst[k] || !strides_ok(sstride[k], esize(dt), src[k]) || reinterpret_cast<uintptr_t>(dst[k]) % 16)
      return SVGEAR_ERR_INVALID;
  return gather_tensors(perm, B * H, H, N, n_tensors, src, sstride, dst, dt, d, static_cast<hipStream_t>(stream));
}

extern "C" int svgear_unpermute(const void* op, const int32_t* perm, svgear_dtype dt, int B, int H, int64_t N,
                                int d, void* o, const int64_t ostride[3], void* stream) {
  if (!op || !perm || !o || B <= 0 || H <= 0 || N <= 0 || N > INT32_MAX / 2 || (d != 64 && d != 128))
    return SVGEAR_ERR_INVALID;
  if (dt != SVGEAR_F32 && dt != SVGEAR_BF16) return SVGEAR_ERR_INVALID;
  if (!strides_ok(ostride, esize(dt), o) || reinterpret_cast<uintptr_t>(op) % 16) return SVGEAR_ERR_INVALID;
  hipStream_t s = static_cast<hipStream_t>(stream);
  const int row_units = (int)(d * esize(dt) / 16);
  const int upe = (int)(16 / esize(dt));
  Strides st{ostride[0] / upe, ostride[1] / upe, ostride[2] / upe};
  dim3 grid((unsigned)ceil_div(N * row_units, kThreads), B * H);
  scatter_rows_kernel<<<grid, kThreads, 0, s>>>(static_cast<const uint4*>(op), perm, N, row_units,
                                                static_cast<uint4*>(o), st, H);
  SVGEAR_LAUNCH_CHECK();
  return SVGEAR_OK;
}
