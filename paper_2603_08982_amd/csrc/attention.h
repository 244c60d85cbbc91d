// Shared declarations of the fused attention kernels (internal).
#pragma once
#include "common.h"

namespace svgear {

constexpr float kLog2e = 1.4426950408889634f;
constexpr float kLn2 = 0.6931471805599453f;
constexpr int BN = 64;  // keys per tile

struct AttnArgs {
  const void* qp;
  const void* kp;
  const void* vp;
  const float* kbar;
  const float* vbar;
  const bf16_t* kbar16;
  const bf16_t* vbar16;
  const int32_t* q_offsets;
  const int32_t* k_offsets;
  const uint32_t* mask_bits;
  const int32_t* row_ptr;
  const int32_t* col_idx;
  const int32_t* tile_a;
  const int32_t* tile_row0;
  const int32_t* n_tiles;
  // work lists of the d = 128 bf16 kernel (see plan_d128): tiles sorted longest first and
  // dealt to 8 lists, one per XCD; sched_x = [8] first slot, [8] tile count, [8] next counter
  const int32_t* sched_bh;
  const int32_t* sched_a;
  const int32_t* sched_row0;
  const int32_t* sched_rend;  // tile = rows [sched_row0, sched_rend) of query cluster sched_a
  int32_t* sched_x;
  int64_t Nq, Nk;
  int BH, Cq, Ck, max_tiles;
  float scale;
  void* op;
  float* lse;
  int part;  // 0: routed blocks and compensation (fused); 1: routed blocks only; 2: compensation only
  // token order at both ends (the queries' permutation folded into the kernel, whose lanes read
  // and write whole rows anyway): row r of head bh is token tok_perm[bh*Nq + r] of the query
  // tensor (element strides q_st) and of the output tensor (out_st), both [B,H,Nq,d];
  // null = qp and op are permuted and dense
  const int32_t* tok_perm;
  Strides q_st, out_st;
  int H;
};

// Element offset of query row `row` of head bh.
__device__ __forceinline__ int64_t q_row_offset(const AttnArgs& p, int bh, int64_t row, int D) {
  if (!p.tok_perm) return ((int64_t)bh * p.Nq + row) * D;
  return head_base(p.q_st, bh, p.H) + (int64_t)p.tok_perm[(int64_t)bh * p.Nq + row] * p.q_st.n;
}

// Element offset of output row `row` of head bh (and the index of its lse entry).
__device__ __forceinline__ int64_t out_row_offset(const AttnArgs& p, int bh, int64_t row, int D, int64_t& lse_idx) {
  if (!p.tok_perm) {
    lse_idx = (int64_t)bh * p.Nq + row;
    return lse_idx * D;
  }
  const int64_t tok = p.tok_perm[(int64_t)bh * p.Nq + row];
  lse_idx = (int64_t)bh * p.Nq + tok;
  return head_base(p.out_st, bh, p.H) + tok * p.out_st.n;
}

__device__ __forceinline__ bool mask_bit(const uint32_t* mrow, int b) { return (mrow[b >> 5] >> (b & 31)) & 1u; }


// Waves per workgroup of the generic bf16 kernel (32 query rows per wave).
constexpr int kBf16Waves = 4;
// Query rows per workgroup tile of the bf16 kernel used for head dimension d.
int attn_bf16_bm(int d);

// Workspace of the d = 128 work lists (bytes) and their construction on stream s.
size_t plan_d128_workspace(int BH, int Cq, int64_t Nq);
int plan_d128(AttnArgs& a, void* ws, size_t ws_bytes, hipStream_t s);

// LDS bytes the bf16 kernel needs for head dimension d and Ck key clusters.
size_t attn_bf16_lds_bytes(int d, int Ck);
// Launches the bf16 MFMA kernel over `total` (multiple of 8) workgroups.
int launch_attn_bf16(const AttnArgs& a, int d, unsigned total, hipStream_t s);

// out = merge of (o1, lse1) and (o2, lse2), partial softmax results over disjoint key sets.
int launch_merge(const bf16_t* o1, const float* lse1, const bf16_t* o2, const float* lse2, int64_t rows, int d,
                 bf16_t* out, float* lse, hipStream_t s);

}  // namespace svgear
