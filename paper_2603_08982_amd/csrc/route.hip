// Greedy error-to-cost routing under a cost budget, and the svgear_probe_route entry point.
// Paper: "Error-Aware Routing" (blocks are taken in descending order of error-to-size ratio
// until the budget is exhausted; the rest go to linear compensation); Experiments,
// "Implementation" (per-query-cluster budgets).
//
// "Sort, prefix-sum the costs, cut at the budget" is done without a sort: the cut is the
// first block, in (score desc, index asc) order, whose inclusive cumulative cost exceeds
// the budget. Each block gets a unique 64-bit key that is monotone in that order; an
// 8-pass, most-significant-byte-first radix descent over cost histograms finds the key K*
// of the cut exactly (integer arithmetic only), and block (a,b) is routed iff key > K*.
//
// The adaptive per-query-cluster budgets (a reading of the top-p allocation the paper
// inherits and does not define) use the same descent over integer mass weights.
#include "common.h"

namespace svgear {

int run_probe(const float* qbar, const float* kbar, const float* vbar, const void* kp, const void* vp,
              svgear_dtype dt, const int32_t* k_offsets, int BH, int64_t Nk, int d, int Cq, int Ck, float scale,
              bool value_aware, float* scores, float* sbar, float* mrow, bf16_t* q3, float* nd, float* dd,
              hipStream_t s);

int run_sbar(const float* qbar, const float* kbar, const int32_t* k_offsets, int BH, int d, int Cq, int Ck,
             float scale, float* sbar, float* mrow, hipStream_t s);

namespace {

constexpr int kSelThreads = 1024;
constexpr int kTopPThreads = 256;
constexpr int kTopPWeightBits = 20;  // masses are counted in units of 2^-20
constexpr int kTopPIndexBits = 13;   // Ck <= 8192

// Larger score -> larger key; among equal scores lower linear index -> larger key.
__device__ __forceinline__ uint64_t block_key(float score, uint32_t idx) {
  if (score != score) score = INFINITY;  // NaN ranks first
  if (score == 0.f) score = 0.f;         // -0 and +0 tie
  uint32_t u = __float_as_uint(score);
  u = (u & 0x80000000u) ? ~u : (u | 0x80000000u);
  return ((uint64_t)u << 32) | (uint64_t)(0xFFFFFFFFu - idx);
}

struct CutState {
  unsigned long long hist[256];
  unsigned long long prefix;
  long long remaining;
  long long wave_total[4];
  unsigned int count[256];  // items per digit
  int crossed[2];           // per pass parity: some digit's cumulative weight exceeded what is left
  int single;               // the digit that crossed holds one item: that item is the cut
};

// Walks n_items items in descending key order (keys unique) and returns the key of the first
// one whose inclusive cumulative weight exceeds rem, or 0 if every item fits. visit(it, key,
// weight) returns false for items that do not take part. Called by all threads of the block
// (THREADS >= 256, a multiple of 64).
// Items are visited four at a time per thread, all their loads issued before the first
// histogram update; the digit of the cut is found by a 256-wide scan of the histogram from
// the top digit down (four waves, shuffles), not by one thread walking it. As soon as the
// digit that crosses holds a single item, that item is the cut and one more walk fetches its
// key (scores are mostly distinct, so this happens after three or four of the eight digits).
template <int THREADS, class Visit>
__device__ __forceinline__ unsigned long long radix_cut(CutState& st, long long rem, int n_items, Visit visit) {
  constexpr int U = 4;
  static_assert(THREADS >= 256 && THREADS % 64 == 0, "the histogram scan uses the first four waves");
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  if (threadIdx.x == 0) {
    st.remaining = rem > 0 ? rem : 0;
    st.prefix = 0ull;
  }
  for (int pass = 0; pass < 8; ++pass) {
    const int shift = 56 - 8 * pass;
    for (int i = threadIdx.x; i < 256; i += THREADS) {
      st.hist[i] = 0ull;
      st.count[i] = 0u;
    }
    if (threadIdx.x == 0) {
      st.crossed[pass & 1] = 0;
      st.single = 0;
    }
    __syncthreads();
    const unsigned long long prefix = st.prefix;
    const long long left = st.remaining;
    for (int base = 0; base < n_items; base += U * THREADS) {  // same trip count for every thread
      uint64_t key[U];
      unsigned long long weight[U];
      bool on[U];
#pragma unroll
      for (int u = 0; u < U; ++u) {
        const int it = base + u * THREADS + (int)threadIdx.x;
        on[u] = it < n_items && visit(it, key[u], weight[u]);
        on[u] = on[u] && (pass == 0 || (key[u] >> (shift + 8)) == prefix);
      }
#pragma unroll
      for (int u = 0; u < U; ++u) {
        if (!on[u]) continue;
        const int digit = (int)((key[u] >> shift) & 255u);
        atomicAdd(&st.hist[digit], weight[u]);
        atomicAdd(&st.count[digit], 1u);
      }
    }
    __syncthreads();
    // thread i < 256 owns digit 255 - i: inclusive sums in descending digit order
    long long h = 0, incl = 0;
    if (threadIdx.x < 256) {
      h = (long long)st.hist[255 - threadIdx.x];
      incl = h;
#pragma unroll
      for (int o = 1; o < 64; o <<= 1) {
        const long long t = __shfl_up(incl, o);
        if (lane >= o) incl += t;
      }
      if (lane == 63) st.wave_total[wave] = incl;
    }
    __syncthreads();
    if (threadIdx.x < 256) {
      for (int w = 0; w < wave; ++w) incl += st.wave_total[w];
      if (incl > left && incl - h <= left) {  // the first digit that does not fit: one thread at most
        st.remaining = left - (incl - h);
        st.prefix = (prefix << 8) | (unsigned long long)(255 - threadIdx.x);
        st.crossed[pass & 1] = 1;
        st.single = st.count[255 - threadIdx.x] == 1u;
      }
    }
    __syncthreads();
    if (!st.crossed[pass & 1]) return 0ull;  // everything fits (can only happen on the first pass)
    if (st.single && pass < 7) {
      const unsigned long long found = st.prefix;  // the leading 8 (pass + 1) bits of the cut
      __syncthreads();
      for (int base = 0; base < n_items; base += THREADS) {
        const int it = base + (int)threadIdx.x;
        uint64_t key;
        unsigned long long weight;
        if (it < n_items && visit(it, key, weight) && (key >> shift) == found) st.prefix = key;
      }
      __syncthreads();
      return st.prefix;
    }
  }
  return st.prefix;
}

// grid (nseg, BH): nseg = 1 (one budget per head) or Cq (one per query cluster; row_budget,
// if given, holds each cluster's budget for its clustered blocks, the tail column on top).
__global__ void __launch_bounds__(kSelThreads)
select_kernel(const float* __restrict__ scores, const int32_t* __restrict__ q_offsets,
              const int32_t* __restrict__ k_offsets, int Cq, int Ck, int64_t budget, int per_row,
              const int64_t* __restrict__ row_budget, uint64_t* __restrict__ kstar) {
  __shared__ CutState st;
  const int seg = blockIdx.x, bh = blockIdx.y;
  const int32_t* qo = q_offsets + (int64_t)bh * (Cq + 2);
  const int32_t* ko = k_offsets + (int64_t)bh * (Ck + 2);
  const float* sc = scores + (int64_t)bh * Cq * Ck;
  const int64_t Nq = qo[Cq + 1], Nk = ko[Ck + 1];
  const int64_t tq = qo[Cq + 1] - qo[Cq], tk = ko[Ck + 1] - ko[Ck];
  const int a_lo = per_row ? seg : 0, a_hi = per_row ? seg + 1 : Cq;
  const int n_items = (a_hi - a_lo) * Ck;  // (Cq + 1)(Ck + 1) fits 31 bits (checked by the caller)
  long long rem;
  if (row_budget) {
    rem = row_budget[(int64_t)bh * Cq + seg];
  } else if (per_row) {
    const int64_t qa = qo[seg + 1] - qo[seg];
    rem = (budget * qa) / (Nq > 0 ? Nq : 1) - qa * tk;
  } else {
    rem = budget - (tq * Nk + (Nq - tq) * tk);
  }
  const unsigned long long cut = radix_cut<kSelThreads>(st, rem, n_items, [&](int it, uint64_t& key,
                                                                              unsigned long long& weight) {
    const int ar = (int)((unsigned)it / (unsigned)Ck);
    const int a = a_lo + ar, b = it - ar * Ck;
    const int64_t cost = (int64_t)(qo[a + 1] - qo[a]) * (int64_t)(ko[b + 1] - ko[b]);
    if (cost <= 0) return false;
    key = block_key(sc[(int64_t)a * Ck + b], (uint32_t)(a * Ck + b));
    weight = (unsigned long long)cost;
    return true;
  });
  if (threadIdx.x == 0) kstar[(int64_t)bh * (per_row ? Cq : 1) + seg] = cut;
}

// Adaptive budget of query cluster a (grid (Cq, BH)): the non-empty key clusters carry the
// centroid attention mass |k_b| exp(Sbar_ab - m_a), counted in integer units of 2^-20 so that
// sums are exact in any order; ordered by weight descending (ties: lower b first), the
// shortest prefix whose weight reaches ceil(top_p * total) is kept, and the budget is the
// cost |q_a| * sum |k_b| of exact attention over it.
__global__ void __launch_bounds__(kTopPThreads)
top_p_budget_kernel(const float* __restrict__ sbar, const float* __restrict__ mrow,
                    const int32_t* __restrict__ q_offsets, const int32_t* __restrict__ k_offsets, int Cq, int Ck,
                    float top_p, int64_t* __restrict__ row_budget) {
  extern __shared__ unsigned long long wgt[];  // Ck
  __shared__ CutState st;
  __shared__ unsigned long long sh_total, sh_keys;
  const int a = blockIdx.x, bh = blockIdx.y;
  const int32_t* qo = q_offsets + (int64_t)bh * (Cq + 2);
  const int32_t* ko = k_offsets + (int64_t)bh * (Ck + 2);
  const int64_t qa = qo[a + 1] - qo[a];
  if (qa <= 0) {
    if (threadIdx.x == 0) row_budget[(int64_t)bh * Cq + a] = 0;
    return;
  }
  if (threadIdx.x == 0) {
    sh_total = 0ull;
    sh_keys = 0ull;
  }
  __syncthreads();
  const float* sr = sbar + ((int64_t)bh * Cq + a) * Ck;
  const float m = mrow[(int64_t)bh * Cq + a];
  unsigned long long part = 0ull;
  for (int b = threadIdx.x; b < Ck; b += kTopPThreads) {
    const int32_t kb = ko[b + 1] - ko[b];
    unsigned long long w = 0ull;
    if (kb > 0) {
      const float mass = (float)kb * expf(sr[b] - m) * (float)(1 << kTopPWeightBits);
      if (mass >= 1.f) w = (unsigned long long)mass;  // also drops NaN
    }
    wgt[b] = w;
    part += w;
  }
  if (part) atomicAdd(&sh_total, part);
  __syncthreads();
  const unsigned long long total = sh_total;
  const double want = ceil((double)top_p * (double)total);
  const long long need = want >= 1.0 ? (long long)want : 1ll;
  auto key_of = [&](int b) { return (wgt[b] << kTopPIndexBits) | (unsigned long long)((1 << kTopPIndexBits) - 1 - b); };
  const unsigned long long cut = radix_cut<kTopPThreads>(st, need - 1, Ck, [&](int it, uint64_t& key,
                                                                               unsigned long long& weight) {
    const int b = it;
    if (ko[b + 1] <= ko[b]) return false;
    key = key_of(b);
    weight = wgt[b];
    return true;
  });
  unsigned long long keys = 0ull;
  for (int b = threadIdx.x; b < Ck; b += kTopPThreads) {
    const int32_t kb = ko[b + 1] - ko[b];
    if (kb > 0 && key_of(b) >= cut) keys += (unsigned long long)kb;
  }
  if (keys) atomicAdd(&sh_keys, keys);
  __syncthreads();
  if (threadIdx.x == 0) row_budget[(int64_t)bh * Cq + a] = qa * (int64_t)sh_keys;
}

constexpr int kBuildThreads = 1024;

// grid (BH). Builds the bit mask, the CSR lists and the routed cost from K*. A wave takes a
// row of blocks at a time, 64 consecutive key clusters per step (coalesced score loads), and
// forms two mask words with one ballot.
__global__ void __launch_bounds__(kBuildThreads)
build_kernel(const float* __restrict__ scores, const int32_t* __restrict__ q_offsets,
             const int32_t* __restrict__ k_offsets, int Cq, int Ck, int per_row,
             const uint64_t* __restrict__ kstar, uint32_t* __restrict__ mask_bits, int32_t* __restrict__ row_ptr,
             int32_t* __restrict__ col_idx, int64_t* __restrict__ routed_cost) {
  extern __shared__ int32_t rowcnt[];  // Cq+2
  __shared__ unsigned long long cost_sum;
  const int bh = blockIdx.x, lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  constexpr int NWAVES = kBuildThreads / 64;
  const int R = Cq + 1, Cc = Ck + 1, W = (Cc + 31) / 32;
  const int32_t* qo = q_offsets + (int64_t)bh * (Cq + 2);
  const int32_t* ko = k_offsets + (int64_t)bh * (Ck + 2);
  const float* sc = scores + (int64_t)bh * Cq * Ck;
  uint32_t* mb = mask_bits + (int64_t)bh * R * W;
  if (threadIdx.x == 0) cost_sum = 0ull;
  __syncthreads();
  long long my_cost = 0;
  for (int a = wave; a < R; a += NWAVES) {
    const int64_t qa = qo[a + 1] - qo[a];
    const uint64_t ks = (a < Cq) ? kstar[(int64_t)bh * (per_row ? Cq : 1) + (per_row ? a : 0)] : 0ull;
    int cnt = 0;
    for (int b0 = 0; b0 < W * 32; b0 += 64) {
      const int b = b0 + lane;
      bool on = false;
      if (qa > 0 && b < Cc) {
        const int64_t kb = ko[b + 1] - ko[b];
        if (kb > 0) {
          on = (a == Cq) || (b == Ck);
          if (!on) on = block_key(sc[(int64_t)a * Ck + b], (uint32_t)(a * Ck + b)) > ks;
          if (on) my_cost += qa * kb;
        }
      }
      const unsigned long long bits = __ballot(on);
      cnt += __popcll(bits);
      if (lane == 0) {
        mb[a * W + (b0 >> 5)] = (uint32_t)bits;
        if ((b0 >> 5) + 1 < W) mb[a * W + (b0 >> 5) + 1] = (uint32_t)(bits >> 32);
      }
    }
    if (lane == 0) rowcnt[a] = cnt;
  }
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) my_cost += __shfl_xor(my_cost, o);
  if (lane == 0 && my_cost) atomicAdd(&cost_sum, (unsigned long long)my_cost);
  __threadfence_block();
  __syncthreads();
  int32_t* rp = row_ptr + (int64_t)bh * (R + 1);
  if (threadIdx.x == 0) {
    int32_t run = 0;
    for (int a = 0; a < R; ++a) {
      const int32_t c = rowcnt[a];
      rowcnt[a] = run;
      rp[a] = run;
      run += c;
    }
    rp[R] = run;
    routed_cost[bh] = (int64_t)cost_sum;
  }
  __syncthreads();
  // routed key clusters of every row, ascending: a wave per row, a lane per set bit
  int32_t* ci = col_idx + (int64_t)bh * R * Cc;
  for (int a = wave; a < R; a += NWAVES) {
    int32_t pos = rowcnt[a];
    for (int w0 = 0; w0 < W; w0 += 2) {
      unsigned long long bits = mb[a * W + w0];
      if (w0 + 1 < W) bits |= (unsigned long long)mb[a * W + w0 + 1] << 32;
      if ((bits >> lane) & 1ull) ci[pos + __popcll(bits & ((1ull << lane) - 1ull))] = w0 * 32 + lane;
      pos += __popcll(bits);
    }
  }
}

}  // namespace
}  // namespace svgear

using namespace svgear;

extern "C" size_t svgear_probe_route_workspace(int B, int H, int64_t Nk, int d, int Cq, int Ck) {
  if (B <= 0 || H <= 0 || Cq <= 0 || Ck <= 0 || Nk <= 0 || d <= 0) return 0;
  const size_t BH = (size_t)B * H;
  return align_up(BH * Cq * Ck * 4, 256) + align_up(BH * Cq * 4, 256) + align_up(BH * (Cq + 1) * 8, 256) +
         // bf16 probe: qbar in three bf16 pieces (operand order), per-key value statistics
         align_up(BH * align_up(Cq, 32) * d * 3 * 2, 256) + 2 * align_up(BH * probe_stat_stride(Nk) * 4, 256);
}

namespace {

// top_p < 0: budget_cost rules (per head or per query cluster); otherwise adaptive row budgets.
int probe_route_impl(const float* qbar, const float* kbar, const float* vbar, const void* kp, const void* vp,
                     svgear_dtype dt, const int32_t* q_offsets, const int32_t* k_offsets, int B, int H, int64_t Nq,
                     int64_t Nk, int d, int Cq, int Ck, int64_t budget_cost, float top_p, float scale, unsigned flags,
                     float* scores, uint32_t* mask_bits, int32_t* row_ptr, int32_t* col_idx, int64_t* routed_cost,
                     int64_t* row_budget, void* ws, size_t ws_bytes, void* stream) {
  const bool given = flags & SVGEAR_USE_GIVEN_SCORES;
  const bool adaptive = top_p >= 0.f;
  if (!q_offsets || !k_offsets || !scores || !mask_bits || !row_ptr || !col_idx || !routed_cost || B <= 0 ||
      H <= 0 || Nq <= 0 || Nk <= 0 || Cq <= 0 || Ck <= 0 || Cq > 8192 || Ck > 8192 || budget_cost < 0 ||
      Nq > INT32_MAX / 2 || Nk > INT32_MAX / 2 || (flags & ~7u) || (int64_t)(Cq + 1) * (Ck + 1) > INT32_MAX / 2)
    return SVGEAR_ERR_INVALID;
  if (adaptive && (!row_budget || !(top_p > 0.f && top_p <= 1.f))) return SVGEAR_ERR_INVALID;
  if (!given || adaptive) {
    if (!qbar || !kbar || (d != 64 && d != 128) || reinterpret_cast<uintptr_t>(qbar) % 16 ||
        reinterpret_cast<uintptr_t>(kbar) % 16)
      return SVGEAR_ERR_INVALID;
  }
  if (!given) {
    if (!vbar || !kp || !vp || (dt != SVGEAR_F32 && dt != SVGEAR_BF16) || reinterpret_cast<uintptr_t>(kp) % 16 ||
        reinterpret_cast<uintptr_t>(vp) % 16)
      return SVGEAR_ERR_INVALID;
  }
  if (!ws || ws_bytes < svgear_probe_route_workspace(B, H, Nk, d, Cq, Ck)) return SVGEAR_ERR_WORKSPACE;
  const int BH = B * H;
  Workspace w(ws, ws_bytes);
  float* sbar = w.take<float>((size_t)BH * Cq * Ck);
  float* mrow = w.take<float>((size_t)BH * Cq);
  uint64_t* kstar = w.take<uint64_t>((size_t)BH * (Cq + 1));
  bf16_t* q3 = w.take<bf16_t>((size_t)BH * align_up(Cq, 32) * (d > 0 ? d : 1) * 3);
  float* nd = w.take<float>((size_t)BH * probe_stat_stride(Nk));
  float* dd = w.take<float>((size_t)BH * probe_stat_stride(Nk));
  if (!w.ok()) return SVGEAR_ERR_WORKSPACE;
  hipStream_t s = static_cast<hipStream_t>(stream);
  if (!given) {
    int rc = run_probe(qbar, kbar, vbar, kp, vp, dt, k_offsets, BH, Nk, d, Cq, Ck, scale,
                       !(flags & SVGEAR_PROBE_PLAIN), scores, sbar, mrow, q3, nd, dd, s);
    if (rc != SVGEAR_OK) return rc;
  } else if (adaptive) {
    int rc = run_sbar(qbar, kbar, k_offsets, BH, d, Cq, Ck, scale, sbar, mrow, s);
    if (rc != SVGEAR_OK) return rc;
  }
  const int per_row = (adaptive || (flags & SVGEAR_ROUTE_PER_ROW)) ? 1 : 0;
  if (adaptive) {
    // up to 64 KB of weights for the largest Ck, beside the kernel's static LDS
    SVGEAR_HIP_TRY(hipFuncSetAttribute(reinterpret_cast<const void*>(top_p_budget_kernel),
                                       hipFuncAttributeMaxDynamicSharedMemorySize,
                                       (int)((size_t)Ck * sizeof(unsigned long long))));
    top_p_budget_kernel<<<dim3(Cq, BH), kTopPThreads, (size_t)Ck * sizeof(unsigned long long), s>>>(
        sbar, mrow, q_offsets, k_offsets, Cq, Ck, top_p, row_budget);
    SVGEAR_LAUNCH_CHECK();
  }
  select_kernel<<<dim3(per_row ? Cq : 1, BH), kSelThreads, 0, s>>>(scores, q_offsets, k_offsets, Cq, Ck, budget_cost,
                                                                  per_row, adaptive ? row_budget : nullptr, kstar);
  SVGEAR_LAUNCH_CHECK();
  build_kernel<<<BH, kBuildThreads, (Cq + 2) * sizeof(int32_t), s>>>(scores, q_offsets, k_offsets, Cq, Ck, per_row, kstar,
                                                          mask_bits, row_ptr, col_idx, routed_cost);
  SVGEAR_LAUNCH_CHECK();
  return SVGEAR_OK;
}

}  // namespace

extern "C" int svgear_probe_route(const float* qbar, const float* kbar, const float* vbar, const void* kp,
                                  const void* vp, svgear_dtype dt, const int32_t* q_offsets,
                                  const int32_t* k_offsets, int B, int H, int64_t Nq, int64_t Nk, int d, int Cq,
                                  int Ck, int64_t budget_cost, float scale, unsigned flags, float* scores,
                                  uint32_t* mask_bits, int32_t* row_ptr, int32_t* col_idx, int64_t* routed_cost,
                                  void* ws, size_t ws_bytes, void* stream) {
  return probe_route_impl(qbar, kbar, vbar, kp, vp, dt, q_offsets, k_offsets, B, H, Nq, Nk, d, Cq, Ck, budget_cost,
                          -1.f, scale, flags, scores, mask_bits, row_ptr, col_idx, routed_cost, nullptr, ws, ws_bytes,
                          stream);
}

extern "C" int svgear_probe_route_top_p(const float* qbar, const float* kbar, const float* vbar, const void* kp,
                                        const void* vp, svgear_dtype dt, const int32_t* q_offsets,
                                        const int32_t* k_offsets, int B, int H, int64_t Nq, int64_t Nk, int d,
                                        int Cq, int Ck, float top_p, float scale, unsigned flags, float* scores,
                                        uint32_t* mask_bits, int32_t* row_ptr, int32_t* col_idx,
                                        int64_t* routed_cost, int64_t* row_budget, void* ws, size_t ws_bytes,
                                        void* stream) {
  if (!(top_p > 0.f && top_p <= 1.f) || (flags & SVGEAR_ROUTE_PER_ROW)) return SVGEAR_ERR_INVALID;
  return probe_route_impl(qbar, kbar, vbar, kp, vp, dt, q_offsets, k_offsets, B, H, Nq, Nk, d, Cq, Ck, 0, top_p,
                          scale, flags, scores, mask_bits, row_ptr, col_idx, routed_cost, row_budget, ws, ws_bytes,
                          stream);
}
