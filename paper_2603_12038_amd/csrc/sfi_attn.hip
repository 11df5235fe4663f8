// Split single-query GQA attention for gfx950: dense over a position range, or gathered by index.
//
// What it computes (paper Sec. 3.1): for one (sequence b, KV head h) and the G query heads that
// share it, logits l_g(j) = scale * <q_g, k_j> over a list of positions, and the flash-style
// partial  (m, sum_j e^{l-m}, sum_j e^{l-m} v_j)  of a share of that list, in the log2 domain
// (y = log2(e) * l, weights 2^(y - m)).
//   dense  kernel (slow step; in the ragged step with the launch planned on the device, attn_dense_items_kernel):
//          the waves of n_split workgroups share the tiles of the allowed set
//          J = [n_sink, L - recent), for which y is also exposed to the Selector (Eq. window_logits,
//          W = 1), followed by the tiles of the sink and recent rows, which the Selector never ranks
//          (Eq. allowed_set).  A wave keeps the two kinds in separate records, so the J-only softmax
//          normaliser of Eq. selector_pt is just the merge of the J records.  Every wave writes its
//          own records: waves never wait for each other.
//   gather kernels (fast step): the list is  sink ++ sel_idx[0:n_sel] ++ [recent_start, L)
//          (Eq. index_set_head), strided over n_split workgroups; the four waves of a workgroup
//          are combined into one record (fewer records for the merge that follows).  One tile per
//          wave, or a pipelined walk over several for large launches.
//   compact kernel (fast step, two-segment layout of Sec. 4.2) and the Reorg copy that feeds it.
//
// Mapping to the matrix cores.  A wave owns 32 positions per iteration, as two 16-row blocks.
//   S^T = K_blk (16 rows x 128) . Q^T (128 x 16 heads, heads >= G are zero): 4 x mfma 16x16x32 bf16
//         per block.  Lane (jg = lane/16, n = lane%16) feeds K row n, dims kblk*32 + 8*jg .. +8
//         (one 16-byte load) and gets back S[row 4*jg+i][head n], i = 0..3.
//   O   += P (16 heads x 32 rows) . V (32 rows x 128): the contraction slot (jg, i') of the PV
//         product is mapped to row 4*jg+i' of block A (i' < 4) or block B (i' >= 4), which is
//         exactly where the S^T result left this lane's probabilities, so P never crosses lanes.
//         Lane (jg, n) loads V rows 4*jg+i' at dims 8n..8n+7 (16-byte, row-contiguous across the
//         16 lanes) and issues 8 products, one per dim offset e, taking element e of each row.
//         P is split into two bf16 terms (hi + lo) so the weights keep ~16 bits.
// bf16 x bf16 products are exact in fp32, so logits differ from an fp64 evaluation only by the
// fp32 accumulation inside the matrix core.
#include "sfi_internal.h"
#include "sfi_merge.h"

namespace sfi {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) float f32x4;

__device__ __forceinline__ bf16x8 as_bf16x8(uint4 v) { return __builtin_bit_cast(bf16x8, v); }

__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

// two fp32 -> one dword of two truncated bf16 (low half = a)
__device__ __forceinline__ uint32_t pack_hi16(float a, float b) {
  return (__float_as_uint(a) >> 16) | (__float_as_uint(b) & 0xffff0000u);
}

// K and V rows are read once per step: stream them past the caches.  base is uniform over the
// workgroup, off a 32-bit byte offset (the API rejects layouts whose per-head extent exceeds 4 GiB).
__device__ __forceinline__ uint4 load_row16(const char* base, uint32_t off) {
  typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
  const u32x4 v = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(base + off));
  return make_uint4(v.x, v.y, v.z, v.w);
}
// The same with a 64-bit byte offset: block pools of a paged cache may exceed 4 GiB.
__device__ __forceinline__ uint4 load_row16(const char* base, uint64_t off) {
  typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
  const u32x4 v = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(base + off));
  return make_uint4(v.x, v.y, v.z, v.w);
}
// Offset type of a row address: 32 bits for a flat cache, 64 for a paged one.
template <bool PAGED> struct RowOff { typedef uint32_t type; };
template <> struct RowOff<true> { typedef uint64_t type; };

struct Tile {
  uint4 ka[4], kb[4];  // K rows of blocks A / B: row n, dims kblk*32 + 8*jg .. +8  (WIDE: see below)
  uint4 v[8];          // V rows 4*jg + i of block A (i < 4) and block B (i >= 4), dims 8n .. 8n+7
};

// WIDE (the gather and compact kernels, query groups of at most 8 heads): a K row's 256 bytes go out as two requests
// for whole 128-byte lines instead of four for 64 bytes -- a compute unit's bandwidth is the requests it
// keeps in flight times their size.  (The dense kernel stays with the plain layout: it measured 1-4 % slower
// with this one, whichever way the lanes exchange their halves.)  The operand layout gives a row of the matrix product to four lanes of 16 bytes, so
// a row of the product is made half a K row: the tile is four blocks of 8 positions, product row
// n = 8 * half + r of block blk is position 8 * blk + r, dims 64 * kb + 32 * half + 8 * jg .. + 8 in
// step kb (two steps), and its column 8 * half' + head is the same half of q[head].  The halves
// meet where half == half': lane (jg < 2, n < 8) and its mirror (jg + 2, n + 8), 40 lanes up.
// K registers: ka[2 * blk + kb] for blk < 2, kb[2 * (blk - 2) + kb] above.
// Position of V slot i (and of logit y[i]) of lane row jg within the tile:
template <bool WIDE>
__device__ __forceinline__ int slot_pos(int jg, int i) {
  return WIDE ? 16 * (jg >> 1) + 8 * (i >> 2) + 4 * (jg & 1) + (i & 3) : 16 * (i >> 2) + 4 * jg + (i & 3);
}
__device__ __forceinline__ uint4& wide_k(Tile& T, int blk, int kb) { return blk < 2 ? T.ka[2 * blk + kb] : T.kb[2 * (blk - 2) + kb]; }
__device__ __forceinline__ const uint4& wide_k(const Tile& T, int blk, int kb) { return blk < 2 ? T.ka[2 * blk + kb] : T.kb[2 * (blk - 2) + kb]; }
// Lane exchanges of the WIDE layout on the vector ALU (no trip through the LDS crossbar): the lane 8
// further round the same row of 16 (row rotate by 8), and the lane 40 up or down (the same, then the
// two halves of the wave swapped).
__device__ __forceinline__ int lane_xor8(int v) { return __builtin_amdgcn_update_dpp(0, v, 0x128, 0xf, 0xf, false); }
__device__ __forceinline__ float lane_xor8(float v) { return __int_as_float(lane_xor8(__float_as_int(v))); }
__device__ __forceinline__ float lane_xor40(float v) {
  const unsigned w = (unsigned)lane_xor8(__float_as_int(v));
  const auto sw = __builtin_amdgcn_permlane32_swap(w, w, false, false);  // [0]: lower half twice, [1]: upper half twice
  return __uint_as_float((threadIdx.x & 32) != 0 ? sw[0] : sw[1]);
}
// this lane's byte offset into a K row
template <bool WIDE>
__device__ __forceinline__ uint32_t k_lane_of(int jg, int n) { return WIDE ? (uint32_t)((n >> 3) * 64 + jg * 16) : (uint32_t)(jg * 16); }

// Per-wave addressing of one (sequence, KV head): uniform bases, per-lane byte offsets.
struct Rows {
  const char* Kb;
  const char* Vb;
  uint32_t k_st, v_st;    // row strides in bytes
  uint32_t k_lane, v_lane;  // jg * 16, n * 16
  int jg, n;
};

// Paged cache: K and V are pools of blocks of 2^lg consecutive rows (row stride as in Rows); blocks
// start every rpb row strides (rpb = 2^lg when the blocks lie back to back).  A sequence's logical
// row r lives in block tbl[r >> lg] at row r & mask of that block, i.e. at row number
// tbl[r >> lg] * rpb + (r & mask) of the pool's row space.  Everything downstream of a row number
// is unchanged: kernels translate logical rows to physical ones and hand those to the same loads.
struct Pages {
  const int32_t* tbl;  // this sequence's row of the block table
  int lg, mask, rpb;
  int last;            // n_blocks - 1: a block id outside [0, last] is clamped and noted in the caller's flags
  bool live;           // ctx_len > 0 (an empty context has no valid table entry; its padding reads go to row 0 of
                       // whatever block the clamp yields and are not reported)
  __device__ __forceinline__ int page_of(int row) const { return tbl[row >> lg]; }
  __device__ __forceinline__ int phys(int row, int page, int& bad) const {
    const int pc = min(max(page, 0), last);
    bad |= (pc != page && live) ? kGuardBlock : 0;
    return pc * rpb + (row & mask);
  }
};
__device__ __forceinline__ Pages pages_of(const AttnArgs& a, int b, int L) {
  Pages P;
  P.tbl = a.table + (int64_t)b * a.table_stride;
  P.lg = a.page_lg;
  P.mask = (1 << a.page_lg) - 1;
  P.rpb = a.page_rpb;
  P.last = a.n_blocks - 1;
  P.live = L > 0;
  return P;
}

// ctx_len[b] clamped to what the launch may touch.
__device__ __forceinline__ int guarded_len(int L0, int cap, int& bad) {
  const int L = min(max(L0, 0), cap);
  bad |= L != L0 ? kGuardCtxLen : 0;
  return L;
}
// A lane that had to clamp an input says so, once, as the last thing the kernel does: a store inside the
// loop would sit in the in-order memory counter the pipelined loops wait on, and even the untaken branch,
// placed between the loop and the record write, cost the fast step 0.2 us.
__device__ __forceinline__ void report_guard(int32_t* guard, int bad) {
  if (bad != 0 && guard != nullptr) atomicOr(guard, bad);
}

// Row loads of a tile whose positions map to consecutive cache rows: block A row n is cache row
// r0 + n; rows above r_max are replaced by r_max (they carry no weight).  K and V separately, so
// that each half of the tile buffer can be refilled as soon as its consumer is done with it.
template <bool WIDE = false>
__device__ __forceinline__ void issue_k_affine(Tile& T, const Rows& R, int r0, int r_max) {
  if (WIDE) {
#pragma unroll
    for (int blk = 0; blk < 4; ++blk) {
      const uint32_t o = (uint32_t)min(r0 + 8 * blk + (R.n & 7), r_max) * R.k_st + R.k_lane;
      wide_k(T, blk, 0) = load_row16(R.Kb, o);
      wide_k(T, blk, 1) = load_row16(R.Kb, o + 128u);
    }
    return;
  }
  const uint32_t oa = (uint32_t)min(r0 + R.n, r_max) * R.k_st + R.k_lane;
  const uint32_t ob = (uint32_t)min(r0 + 16 + R.n, r_max) * R.k_st + R.k_lane;
#pragma unroll
  for (int kb = 0; kb < 4; ++kb) {
    T.ka[kb] = load_row16(R.Kb, oa + kb * 64);
    T.kb[kb] = load_row16(R.Kb, ob + kb * 64);
  }
}
template <bool WIDE = false>
__device__ __forceinline__ void issue_v_affine(Tile& T, const Rows& R, int r0, int r_max) {
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    T.v[i] = load_row16(R.Vb, (uint32_t)min(r0 + slot_pos<WIDE>(R.jg, i), r_max) * R.v_st + R.v_lane);
    T.v[4 + i] = load_row16(R.Vb, (uint32_t)min(r0 + slot_pos<WIDE>(R.jg, 4 + i), r_max) * R.v_st + R.v_lane);
  }
}
template <bool WIDE = false>
__device__ __forceinline__ void issue_affine(Tile& T, const Rows& R, int r0, int r_max) {
  issue_k_affine<WIDE>(T, R, r0, r_max);
  issue_v_affine<WIDE>(T, R, r0, r_max);
}

// Row loads of a tile with arbitrary rows: ra / rb are the cache rows of this lane's K rows in
// blocks A / B; the V rows 4*jg + i are the ones lanes 4*jg + i resolved for K.  OffT: RowOff<>::type.
template <typename OffT = uint32_t, bool WIDE = false>
__device__ __forceinline__ void issue_k_rows(Tile& T, const Rows& R, int ra, int rb) {
  if (WIDE) {  // positions 8 * blk + (n & 7): held by this lane or by the lane 8 further round its row of 16
    const int xa = lane_xor8(ra), xb = lane_xor8(rb);
    const bool lo = R.n < 8;
    const int r[4] = {lo ? ra : xa, lo ? xa : ra, lo ? rb : xb, lo ? xb : rb};
#pragma unroll
    for (int blk = 0; blk < 4; ++blk) {
      const OffT o = (OffT)(uint32_t)r[blk] * R.k_st + R.k_lane;
      wide_k(T, blk, 0) = load_row16(R.Kb, (OffT)o);
      wide_k(T, blk, 1) = load_row16(R.Kb, (OffT)(o + 128u));
    }
    return;
  }
  const OffT oa = (OffT)(uint32_t)ra * R.k_st + R.k_lane, ob = (OffT)(uint32_t)rb * R.k_st + R.k_lane;
#pragma unroll
  for (int kb = 0; kb < 4; ++kb) {
    T.ka[kb] = load_row16(R.Kb, (OffT)(oa + kb * 64));
    T.kb[kb] = load_row16(R.Kb, (OffT)(ob + kb * 64));
  }
}
template <typename OffT = uint32_t, bool WIDE = false>
__device__ __forceinline__ void issue_v_rows(Tile& T, const Rows& R, int ra, int rb) {
  if (WIDE) {  // slot i is position slot_pos(jg, i): index 4 * (jg & 1) + (i & 3) + 8 * (i >> 2) of ra (jg < 2) or rb,
               // taken from the lane of this lane's own row of 16 that resolved it
    const int sel = R.jg < 2 ? ra : rb;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      T.v[i] = load_row16(R.Vb, (OffT)((OffT)(uint32_t)__shfl(sel, 16 * R.jg + 4 * (R.jg & 1) + i) * R.v_st + R.v_lane));
      T.v[4 + i] = load_row16(R.Vb, (OffT)((OffT)(uint32_t)__shfl(sel, 16 * R.jg + 8 + 4 * (R.jg & 1) + i) * R.v_st + R.v_lane));
    }
    return;
  }
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    T.v[i] = load_row16(R.Vb, (OffT)((OffT)(uint32_t)__shfl(ra, 4 * R.jg + i) * R.v_st + R.v_lane));
    T.v[4 + i] = load_row16(R.Vb, (OffT)((OffT)(uint32_t)__shfl(rb, 4 * R.jg + i) * R.v_st + R.v_lane));
  }
}
template <typename OffT = uint32_t, bool WIDE = false>
__device__ __forceinline__ void issue_rows(Tile& T, const Rows& R, int ra, int rb) {
  issue_k_rows<OffT, WIDE>(T, R, ra, rb);
  issue_v_rows<OffT, WIDE>(T, R, ra, rb);
}

// Q^T operand: head n, dims kblk*32 + 8*jg .. +8; zero for heads >= G (no branch around the loads).
template <bool WIDE = false>
__device__ __forceinline__ void load_q(bf16x8 (&qreg)[4], const uint16_t* q, int64_t head0, int G, int jg, int n) {
  if (WIDE) {  // column n = 8 * half + head: dims 64 * kb + 32 * half + 8 * jg .. + 8 of q[head]; qreg[2], qreg[3] unused
    const int head = n & 7;
    const uint16_t* qw = q + (head0 + (head < G ? head : 0)) * kHeadDim + (n >> 3) * 32 + jg * 8;
    const uint32_t kp = head < G ? 0xffffffffu : 0u;
#pragma unroll
    for (int kb = 0; kb < 2; ++kb) {
      uint4 t = *reinterpret_cast<const uint4*>(qw + kb * 64);
      t.x &= kp; t.y &= kp; t.z &= kp; t.w &= kp;
      qreg[kb] = as_bf16x8(t);
      qreg[2 + kb] = as_bf16x8(make_uint4(0u, 0u, 0u, 0u));
    }
    return;
  }
  const uint16_t* qp = q + (head0 + (n < G ? n : 0)) * kHeadDim + jg * 8;
  const uint32_t keep = n < G ? 0xffffffffu : 0u;
#pragma unroll
  for (int kb = 0; kb < 4; ++kb) {
    uint4 t = *reinterpret_cast<const uint4*>(qp + kb * 32);
    t.x &= keep; t.y &= keep; t.z &= keep; t.w &= keep;
    qreg[kb] = as_bf16x8(t);
  }
}

// One 32-position tile in three phases: S^T = K Q^T, online softmax in the log2 domain, O += P V.
// y = c2 * <q, k> with c2 = scale * log2(e); m_run / l_run are the running max of y and the running
// sum of 2^(y - m_run) of this lane's rows; acc[e][i] is O[head 4*jg+i][dim 8n+e].
// Lanes of heads >= G see q = 0; their state stays finite and is never written out: no mask needed.

// Phase 1: y[i] = logit (log2 domain) of head n, row 4*jg+i of block A (i < 4) / block B (i >= 4).
// WIDE, first half: the eight products of a tile; after them the K registers are free for the next tile's rows.
__device__ __forceinline__ void qk_products_wide(const Tile& T, const bf16x8 (&qreg)[4], f32x4 (&s)[4]) {
#pragma unroll
  for (int blk = 0; blk < 4; ++blk) {
    s[blk] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int kb = 0; kb < 2; ++kb)
      s[blk] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(as_bf16x8(wide_k(T, blk, kb)), qreg[kb], s[blk], 0, 0, 0);
  }
}
// WIDE, second half: the half-row sums meet.
// s[blk][i] of lane (jg, n): product row 4 * jg + i, column n.  Lane (jg < 2, n < 8) holds the first-half
// sums of positions 8 * blk + 4 * jg + i for head n, its mirror 40 lanes up the second-half sums.  The
// lower lane keeps blocks 0 and 1, the mirror blocks 2 and 3: each sends the other the half it lacks.
// Then lane (jg >= 2, n < 8) fetches its logits from the mirror (jg, n + 8) in its own row of 16.
__device__ __forceinline__ void qk_join_wide(const f32x4 (&s)[4], float c2, float (&y)[8]) {
  const int lane = threadIdx.x & 63, jg = lane >> 4, n = lane & 15;
  const bool low = jg < 2;
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const float u0 = (low ? s[0][i] : s[2][i]) + lane_xor40(low ? s[2][i] : s[0][i]);
    const float u1 = (low ? s[1][i] : s[3][i]) + lane_xor40(low ? s[3][i] : s[1][i]);
    const float x0 = lane_xor8(u0), x1 = lane_xor8(u1);
    y[i] = n < 8 ? (low ? u0 : x0) * c2 : 0.f;
    y[4 + i] = n < 8 ? (low ? u1 : x1) * c2 : 0.f;
  }
}

template <bool WIDE = false>
__device__ __forceinline__ void qk_phase(const Tile& T, const bf16x8 (&qreg)[4], float c2, float (&y)[8]) {
  if (WIDE) {
    f32x4 s[4];
    qk_products_wide(T, qreg, s);
    qk_join_wide(s, c2, y);
    return;
  }
  f32x4 sa = {0.f, 0.f, 0.f, 0.f}, sb = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
  for (int kb = 0; kb < 4; ++kb) {
    sa = __builtin_amdgcn_mfma_f32_16x16x32_bf16(as_bf16x8(T.ka[kb]), qreg[kb], sa, 0, 0, 0);
    sb = __builtin_amdgcn_mfma_f32_16x16x32_bf16(as_bf16x8(T.kb[kb]), qreg[kb], sb, 0, 0, 0);
  }
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    y[i] = sa[i] * c2;
    y[4 + i] = sb[i] * c2;
  }
}

// Squared norms of the tile's K rows from the matrix cores: K K^T of block A (B), whose diagonal
// element (row m, row m) sits in lane (jg, n) = (m / 4, m), slot m % 4.  Products of bf16 pairs are
// exact in fp32.  The lane with jg == n / 4 gets ||row n||^2 of block A in k2a and of block B in k2b.
__device__ __forceinline__ void knorm_phase(const Tile& T, int jg, int n, float& k2a, float& k2b) {
  f32x4 sa = {0.f, 0.f, 0.f, 0.f}, sb = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
  for (int kb = 0; kb < 4; ++kb) {
    sa = __builtin_amdgcn_mfma_f32_16x16x32_bf16(as_bf16x8(T.ka[kb]), as_bf16x8(T.ka[kb]), sa, 0, 0, 0);
    sb = __builtin_amdgcn_mfma_f32_16x16x32_bf16(as_bf16x8(T.kb[kb]), as_bf16x8(T.kb[kb]), sb, 0, 0, 0);
  }
  const int i = n & 3;
  k2a = i == 0 ? sa[0] : i == 1 ? sa[1] : i == 2 ? sa[2] : sa[3];
  k2b = i == 0 ? sb[0] : i == 1 ? sb[1] : i == 2 ? sb[2] : sb[3];
  (void)jg;
}

// y of head n, rows 0..31 of the tile, goes to stage[n * 32 ..] (this wave's LDS patch).
template <bool WIDE = false>
__device__ __forceinline__ void stage_logits(float* stage, const float (&y)[8], int jg, int n, int G) {
  if (n < G) {
    *reinterpret_cast<float4*>(stage + n * kTile + slot_pos<WIDE>(jg, 0)) = make_float4(y[0], y[1], y[2], y[3]);
    *reinterpret_cast<float4*>(stage + n * kTile + slot_pos<WIDE>(jg, 4)) = make_float4(y[4], y[5], y[6], y[7]);
  }
}

// Ragged last tile: positions >= N carry no weight; their V rows may hold anything, so zero them
// to keep 0 * v finite.
template <bool WITH_V = true, bool WIDE = false>  // WITH_V false: the tile holds no V rows (evidence-only pass)
__device__ __forceinline__ void mask_tail(Tile& T, float (&y)[8], int jg, int p0, int N) {
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const bool oka = p0 + slot_pos<WIDE>(jg, i) < N, okb = p0 + slot_pos<WIDE>(jg, 4 + i) < N;
    y[i] = oka ? y[i] : kNeg;
    y[4 + i] = okb ? y[4 + i] : kNeg;
    if (WITH_V && !oka) T.v[i] = make_uint4(0u, 0u, 0u, 0u);
    if (WITH_V && !okb) T.v[4 + i] = make_uint4(0u, 0u, 0u, 0u);
  }
}

// Phase 2: running max / sum update (accumulators rescaled only when some head's maximum moved,
// which is rare after the first tiles) and the weights as two bf16 terms, hi + lo ~ 16 bits.
// Masked rows carry y = kNeg; every tile handed in has at least one unmasked row, so each head's
// maximum is finite and 2^(kNeg - max) is exactly 0.
__device__ __forceinline__ void softmax_phase(const float (&y)[8], f32x4 (&acc)[8], float& m_run, float& l_run, int jg,
                                              bf16x8& a_hi, bf16x8& a_lo) {
  float mt = fmaxf(fmaxf(fmaxf(y[0], y[1]), fmaxf(y[2], y[3])), fmaxf(fmaxf(y[4], y[5]), fmaxf(y[6], y[7])));
  mt = fmaxf(mt, __shfl_xor(mt, 16));
  mt = fmaxf(mt, __shfl_xor(mt, 32));
  const float m_new = fmaxf(m_run, mt);
  if (__ballot(m_new > m_run) != 0ull) {
    const float alpha = fast_exp2(m_run - m_new);
    l_run *= alpha;
    float al[4];  // this lane's accumulators belong to heads 4*jg + i
#pragma unroll
    for (int i = 0; i < 4; ++i) al[i] = __shfl(alpha, 4 * jg + i);
#pragma unroll
    for (int e = 0; e < 8; ++e) {
#pragma unroll
      for (int i = 0; i < 4; ++i) acc[e][i] *= al[i];
    }
    m_run = m_new;
  }
  float pr[8], lo[8], ps = 0.f;
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    pr[i] = fast_exp2(y[i] - m_run);
    ps += pr[i];
    lo[i] = pr[i] - __uint_as_float(__float_as_uint(pr[i]) & 0xffff0000u);
  }
  l_run += ps;
  a_hi = as_bf16x8(make_uint4(pack_hi16(pr[0], pr[1]), pack_hi16(pr[2], pr[3]), pack_hi16(pr[4], pr[5]),
                              pack_hi16(pr[6], pr[7])));
  a_lo = as_bf16x8(make_uint4(pack_hi16(lo[0], lo[1]), pack_hi16(lo[2], lo[3]), pack_hi16(lo[4], lo[5]),
                              pack_hi16(lo[6], lo[7])));
}

// Phase 3: O += P V, one product per dim offset e: element e of each of the 8 rows this lane holds.
__device__ __forceinline__ void pv_phase(const Tile& T, const bf16x8& a_hi, const bf16x8& a_lo, f32x4 (&acc)[8]) {
#pragma unroll
  for (int e = 0; e < 8; ++e) {
    uint32_t c[8];
#pragma unroll
    for (int i = 0; i < 8; ++i)
      c[i] = (e >> 1) == 0 ? T.v[i].x : (e >> 1) == 1 ? T.v[i].y : (e >> 1) == 2 ? T.v[i].z : T.v[i].w;
    uint4 bv;
    if ((e & 1) == 0) {
      bv = make_uint4((c[0] & 0xffffu) | (c[1] << 16), (c[2] & 0xffffu) | (c[3] << 16),
                      (c[4] & 0xffffu) | (c[5] << 16), (c[6] & 0xffffu) | (c[7] << 16));
    } else {
      bv = make_uint4((c[0] >> 16) | (c[1] & 0xffff0000u), (c[2] >> 16) | (c[3] & 0xffff0000u),
                      (c[4] >> 16) | (c[5] & 0xffff0000u), (c[6] >> 16) | (c[7] & 0xffff0000u));
    }
    const bf16x8 b_e = as_bf16x8(bv);
    acc[e] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a_hi, b_e, acc[e], 0, 0, 0);
    acc[e] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a_lo, b_e, acc[e], 0, 0, 0);
  }
}

// All three phases on a tile that is already in registers.  MASKED: ragged last tile of a list.
template <bool MASKED, bool WIDE = false>
__device__ __forceinline__ void tile_math(Tile& T, const bf16x8 (&qreg)[4], float c2, f32x4 (&acc)[8],
                                          float& m_run, float& l_run, int jg, int p0, int N) {
  float y[8];
  qk_phase<WIDE>(T, qreg, c2, y);
  if (MASKED) mask_tail<true, WIDE>(T, y, jg, p0, N);
  bf16x8 a_hi, a_lo;
  softmax_phase(y, acc, m_run, l_run, jg, a_hi, a_lo);
  pv_phase(T, a_hi, a_lo, acc);
}

// Device-scope accesses: visible to / from every compute unit of the device whatever L2 it sits behind,
// without a fence (records that one workgroup hands to another inside a launch).  They go through a buffer
// descriptor, 16 bytes at a time: the records of one (b, h) pair as a raw buffer
// (byte offsets, out-of-range accesses dropped by the hardware), every access with the device-scope cache policy.
typedef unsigned int u32x4_t __attribute__((ext_vector_type(4)));
typedef unsigned int u32x2_t __attribute__((ext_vector_type(2)));
constexpr int kScopeDevice = 16;  // cache-policy bit sc1 of the buffer instructions
__device__ __forceinline__ __amdgpu_buffer_rsrc_t pair_records(float* base, int bytes) {
  return __builtin_amdgcn_make_buffer_rsrc(base, 0, bytes, 0x00020000);
}
__device__ __forceinline__ void store_device4(__amdgpu_buffer_rsrc_t r, int byte_off, float4 v) {
  __builtin_amdgcn_raw_buffer_store_b128(u32x4_t{__float_as_uint(v.x), __float_as_uint(v.y), __float_as_uint(v.z), __float_as_uint(v.w)},
                                         r, byte_off, 0, kScopeDevice);
}
__device__ __forceinline__ void store_device2(__amdgpu_buffer_rsrc_t r, int byte_off, float v0, float v1) {
  __builtin_amdgcn_raw_buffer_store_b64(u32x2_t{__float_as_uint(v0), __float_as_uint(v1)}, r, byte_off, 0, kScopeDevice);
}
__device__ __forceinline__ float4 load_device4(__amdgpu_buffer_rsrc_t r, int byte_off) {
  const u32x4_t v = __builtin_amdgcn_raw_buffer_load_b128(r, byte_off, 0, kScopeDevice);
  return make_float4(__uint_as_float(v.x), __uint_as_float(v.y), __uint_as_float(v.z), __uint_as_float(v.w));
}
__device__ __forceinline__ float2 load_device2(__amdgpu_buffer_rsrc_t r, int byte_off) {
  const u32x2_t v = __builtin_amdgcn_raw_buffer_load_b64(r, byte_off, 0, kScopeDevice);
  return make_float2(__uint_as_float(v.x), __uint_as_float(v.y));
}

// Merge inside the attention kernel.  Called by every thread of every workgroup of a (b, h) pair after
// the workgroup's record went out in device-scope stores.  Every thread waits for its stores to be
// acknowledged, then one thread counts the workgroup in on *arrive.  The workgroup that finds all
// n_wgs - 1 others there before it merges the pair's n_wgs records per head with device-scope loads:
//   out[b, head, :] = sum_s 2^(m_s - M) acc_s / sum_s 2^(m_s - M) l_s,
// and puts the counter back to zero.  Nothing waits on anything, and no cache is written back or
// invalidated as a whole (a device-scope fence costs tens of microseconds here).
// One thread per (head, four output dims); records eight at a time, all loads of the eight in flight.
template <int NW = kWaves>  // waves of the calling workgroup
__device__ __forceinline__ void finish_pair(const float* part, int64_t head0, int G, int n_wgs, uint32_t* arrive,
                                            float* out, bool out_bf16, int slot_cap) {
  const int tid = threadIdx.x;
  __shared__ uint32_t s_before;
  // s_waitcnt vmcnt(0): a workgroup barrier by itself only orders the stores within the compute unit
  __builtin_amdgcn_s_waitcnt(0x0F70);
  __syncthreads();
  if (tid == 0) s_before = __hip_atomic_fetch_add(arrive, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  __syncthreads();
  if (s_before != (uint32_t)(n_wgs - 1)) return;
  if (tid == 0) __hip_atomic_store(arrive, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  const __amdgpu_buffer_rsrc_t R = pair_records(const_cast<float*>(part) + head0 * slot_cap * kPartStride,
                                                G * slot_cap * kPartStride * (int)sizeof(float));
  for (int idx = tid; idx < G * (kHeadDim / 4); idx += NW * 64) {
    const int hh = idx >> 5, c = idx & 31;
    const int P = hh * slot_cap * kPartStride * (int)sizeof(float);  // byte offset of the head's records
    float M = kNeg, Z = 0.f;
    float4 o = make_float4(0.f, 0.f, 0.f, 0.f);
    for (int s0 = 0; s0 < n_wgs; s0 += 8) {
      float2 ml[8];
      float4 r4[8];
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        const int rec = P + min(s0 + i, n_wgs - 1) * kPartStride * (int)sizeof(float);
        ml[i] = load_device2(R, rec);
        r4[i] = load_device4(R, rec + (4 + 4 * c) * (int)sizeof(float));
      }
      float Mn = M;
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        if (s0 + i >= n_wgs) ml[i] = make_float2(kNeg, 0.f);
        Mn = fmaxf(Mn, ml[i].x);
      }
      const float f = fast_exp2(M - Mn);
      Z *= f;
      o.x *= f; o.y *= f; o.z *= f; o.w *= f;
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        const float wgt = fast_exp2(ml[i].x - Mn);
        Z += wgt * ml[i].y;
        o.x += wgt * r4[i].x; o.y += wgt * r4[i].y; o.z += wgt * r4[i].z; o.w += wgt * r4[i].w;
      }
      M = Mn;
    }
    const float inv = Z > 0.f ? 1.0f / Z : 0.f;
    store_out4(out, (head0 + hh) * kHeadDim + 4 * c, make_float4(o.x * inv, o.y * inv, o.z * inv, o.w * inv), out_bf16);
  }
}

// record of (b, head, slot): { max of y, sum 2^(y - max), -, -, O[128] }, written by one wave
__device__ __forceinline__ void write_wave_record(float* part, int64_t head0, int G, int wslot, const f32x4 (&acc)[8],
                                                  float m_run, float l_run, int lane, bool with_acc = true) {
  const int jg = lane >> 4, n = lane & 15;
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int hh = 4 * jg + i;
    if (with_acc && hh < G) {
      float* dst = part + ((head0 + hh) * kSlotCap + wslot) * kPartStride + 4 + n * 8;
      *reinterpret_cast<float4*>(dst) = make_float4(acc[0][i], acc[1][i], acc[2][i], acc[3][i]);
      *reinterpret_cast<float4*>(dst + 4) = make_float4(acc[4][i], acc[5][i], acc[6][i], acc[7][i]);
    }
  }
  if (lane < G) {
    float* r = part + ((head0 + lane) * kSlotCap + wslot) * kPartStride;
    *reinterpret_cast<float2*>(r) = make_float2(m_run, l_run);
  }
}

// Walks a position list whose rows are not consecutive: sink ++ sel ++ recent (gather), or
// sink ++ recent (the dense kernel's last workgroup, n_sel = 0).  Position p < nS is row p, then
// nSel selected rows, then rows rs, rs + 1, ...; positions past the list read row 0 with weight 0.
struct ListWalk {
  const int32_t* sel;  // row of sel_idx of this (b, h), or nullptr
  int sel_cap;         // sel_stride - 1
  int n_sink;
  int nS, nSel, rs, N;
  int r_hi;            // last readable row, max(L, 1) - 1: a stored index outside [0, r_hi] reads as r_hi
  int bad;
  __device__ __forceinline__ void set_counts(int L, int n_sel, int recent_start, int sel_stride) {
    nS = min(n_sink, L);
    nSel = min(max(n_sel, 0), sel_stride);
    bad |= nSel != n_sel ? kGuardNSel : 0;
    rs = min(max(recent_start, nS), L);
    N = nS + nSel + (L - rs);
    r_hi = max(L, 1) - 1;
  }
  __device__ __forceinline__ int sel_at(int p) const {  // index stored for list position p (valid inside the sel part)
    return sel_cap >= 0 ? sel[min(max(p - n_sink, 0), sel_cap)] : 0;
  }
  __device__ __forceinline__ int sel_at_nonempty(int p) const {  // the same without the branch; needs sel_cap >= 0
    return sel[min(max(p - n_sink, 0), sel_cap)];
  }
  __device__ __forceinline__ int row_of(int p, int s) {
    const int i = p - nS;
    int r = i < nSel ? s : rs + (i - nSel);
    r = p < nS ? p : r;
    r = p < N ? r : 0;
    // Sink and recent rows are inside the context by construction, so only a stored index can change here.
    // One clamp for both ends: a negative row reads as a huge one.
    const int rc = (int)min((uint32_t)r, (uint32_t)r_hi);
    bad |= rc != r ? kGuardSelIdx : 0;
    return rc;
  }
};

// ------------------------------------------------------------------------------------------------
// dense kernel
// ------------------------------------------------------------------------------------------------
// PAGED: K / V are block pools addressed through the sequence's block table.
// EXPOSE 1: also write y over J for the Selector; 2: y and the squared key norms.
// BIG: twice the logits stash per wave, which leaves room for one workgroup per compute unit only
// (launches where every sequence is dense, and the ragged step's planned launch, run one per unit anyway; the ragged
// step's launch with a workgroup per cell keeps two).
// NOV: evidence only -- no V row is read, no P V product, the records carry the softmax statistics alone.
template <int EXPOSE, bool PAGED, bool BIG = false, bool NOV = false, bool WIDE = false>
__device__ __forceinline__ void dense_body(const AttnArgs& a, const int n_split, const int slot, const int h, const int b,
                                           const int tid_bias = 0) {
  constexpr int kStash = BIG ? 2 * kStashFloats : kStashFloats;
  __shared__ float s_stash[EXPOSE != 0 ? kWaves : 1][EXPOSE != 0 ? kStash : 1];  // per-wave logits stash
  if (a.is_slow != nullptr && a.is_slow[b * a.fs] == 0) return;
  const int tid = threadIdx.x + tid_bias;  // (tid_bias: zero; see attn_dense_items_kernel)
  const int lane = tid & 63, w = tid >> 6;
  const int jg = lane >> 4, n = lane & 15;
  const int G = a.G;
  const int bh = b * a.Hkv + h;
  const int64_t head0 = (int64_t)b * a.Hq + h * G;
  Rows R;
  R.Kb = reinterpret_cast<const char*>(a.K + b * a.k_sb + h * a.k_sh);
  R.Vb = reinterpret_cast<const char*>(a.V + b * a.v_sb + h * a.v_sh);
  R.k_st = (uint32_t)a.k_st * 2u;
  R.v_st = (uint32_t)a.v_st * 2u;
  R.k_lane = k_lane_of<WIDE>(jg, n);
  R.v_lane = n * 16;
  R.jg = jg;
  R.n = n;

  // The prefix of (b, h) is cut into 32-row tiles in two runs: tiles [0, nTJ) cover the allowed set J
  // (tile t, position i is cache row n_sink + 32 t + i), tiles [nTJ, nTJ + nTS) cover the sink rows
  // followed by the recent window, which the Selector never ranks.  The n_split * 4 waves of the
  // (b, h) pair own tiles first, first + step, ... of that sequence, so every wave of every workgroup
  // carries an equal share.  A wave's J tiles come first; it keeps two records, one for each run
  // (the J-only softmax statistics the Selector needs are merged from the J records alone).
  // The rows of the wave's first tile follow from the block index alone (almost always a J tile):
  // their loads go out before ctx_len arrives, clamped to the launch's row bound.
  const int n_waves = n_split * kWaves;
  const int first = slot * kWaves + w, step = n_waves;
  Tile T;
  // (a paged cache has valid blocks only up to ctx_len: no load before ctx_len is known)
  if (!PAGED && first < a.max_tiles) {
    issue_k_affine<WIDE>(T, R, a.n_sink + first * kTile, a.row_cap);
    if (!NOV) issue_v_affine<WIDE>(T, R, a.n_sink + first * kTile, a.row_cap);
  }
  bf16x8 qreg[4];
  load_q<WIDE>(qreg, a.q, head0, G, jg, n);
  int bad = 0;
  int L, recent;  // a window query under the causal mask sees a shorter context with what is left of the recent window
  window_view(a.q_len, b, guarded_len(a.ctx_len[b * a.ms], a.len_cap, bad), a.recent, L, recent);
  if (slot == 0 && a.hist1 != nullptr) {  // fresh Selector state for this (b, h)
    uint32_t* hh = a.hist1 + (int64_t)bh * kHist1Bins;
    for (int i = tid; i < kHist1Bins; i += kAttnThreads) hh[i] = 0u;
    if (tid < kStateWords) a.state[(int64_t)bh * kStateWords + tid] = 0u;
  }
  const int NJ = max(0, L - recent - a.n_sink);
  const int nTJ = (NJ + kTile - 1) / kTile;
  const int rJ_max = a.n_sink + NJ - 1;
  const int nS = min(a.n_sink, L);
  const int rs = min(max(a.n_sink, L - recent), L);
  const int NS = nS + (L - rs);
  const int nTS = (NS + kTile - 1) / kTile;
  const int nT = nTJ + nTS;
  const int K = first < nT ? (nT - first + step - 1) / step : 0;      // tiles of this wave
  const int KJ = first < nTJ ? (nTJ - first + step - 1) / step : 0;   // ... of which in J
  const int d_rs = rs - nS, r_last = max(L, 1) - 1;
  // cache row of position i of tile t; tiles past the end (the refill after the last tile) read row L - 1
  // (row 0 of an empty context: the cache holds max_ctx >= 1 rows)
  auto row_for = [&](int t, int i) -> int {
    const int xj = a.n_sink + t * kTile + i;
    const int xs = (t - nTJ) * kTile + i;
    const int r_s = min(xs < nS ? xs : xs + d_rs, r_last);
    return t < nTJ ? min(xj, rJ_max) : r_s;
  };
  auto issue_k_tile = [&](Tile& T, int t) {
    if (WIDE) {  // whole 128-byte lines: position 8 * blk + (n & 7), the half of the row this lane's column belongs to
#pragma unroll
      for (int blk = 0; blk < 4; ++blk) {
        const uint32_t o = (uint32_t)row_for(t, 8 * blk + (n & 7)) * R.k_st + R.k_lane;
        wide_k(T, blk, 0) = load_row16(R.Kb, o);
        wide_k(T, blk, 1) = load_row16(R.Kb, o + 128u);
      }
      return;
    }
    const uint32_t oa = (uint32_t)row_for(t, n) * R.k_st + R.k_lane;
    const uint32_t ob = (uint32_t)row_for(t, 16 + n) * R.k_st + R.k_lane;
#pragma unroll
    for (int kb = 0; kb < 4; ++kb) {
      T.ka[kb] = load_row16(R.Kb, oa + kb * 64);
      T.kb[kb] = load_row16(R.Kb, ob + kb * 64);
    }
  };
  auto issue_v_tile = [&](Tile& T, int t) {
    if (NOV) return;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      T.v[i] = load_row16(R.Vb, (uint32_t)row_for(t, slot_pos<WIDE>(jg, i)) * R.v_st + R.v_lane);
      T.v[4 + i] = load_row16(R.Vb, (uint32_t)row_for(t, slot_pos<WIDE>(jg, 4 + i)) * R.v_st + R.v_lane);
    }
  };
  Pages P;
  int pa_n = 0, pb_n = 0;  // PAGED: block-table entries of the next tile's K rows (this lane's rows n and 16 + n)
  if (PAGED) {
    // Same order of memory instructions as an iteration of the loop: K rows, the table entries of the
    // tile after, V rows.  Waves without tiles read row L - 1.
    P = pages_of(a, b, L);
    const int ra = row_for(first, n), rb = row_for(first, 16 + n);
    const int pra = P.phys(ra, P.page_of(ra), bad), prb = P.phys(rb, P.page_of(rb), bad);
    __builtin_amdgcn_sched_barrier(0);
    issue_k_rows<uint64_t>(T, R, pra, prb);
    __builtin_amdgcn_sched_barrier(0);
    pa_n = P.page_of(row_for(first + step, n));
    pb_n = P.page_of(row_for(first + step, 16 + n));
    __builtin_amdgcn_sched_barrier(0);
    if (!NOV) issue_v_rows<uint64_t>(T, R, pra, prb);
    __builtin_amdgcn_sched_barrier(0);
  } else if (K > 0 && first >= nTJ) {  // short context: the first tile is a sink / recent tile after all
    issue_k_tile(T, first);
    issue_v_tile(T, first);
  }
  // A flat cache keeps two tiles in flight per wave: the second buffer takes the wave's second tile now.
  Tile T2;
  constexpr int NB = PAGED ? 1 : 2;  // tile buffers; a tile's refill is the wave's tile NB further on
  if (!PAGED) {
    __builtin_amdgcn_sched_barrier(0);
    issue_k_tile(T2, first + step);
    issue_v_tile(T2, first + step);
    __builtin_amdgcn_sched_barrier(0);
  }

  float m_run = kNeg, l_run = 0.f;
  f32x4 acc[8];
#pragma unroll
  for (int e = 0; e < 8; ++e) acc[e] = f32x4{0.f, 0.f, 0.f, 0.f};

  // Exposing y.  The logits of (b, h) are stored tile-major, [tile][G heads][32 positions], so a
  // tile's G x 128 bytes are one contiguous run.  A wave does not store a tile's logits when it
  // has them: a store acknowledged late would sit in front of the next rows in the in-order
  // memory counter.  It parks them in its LDS stash, laid out as they go to memory, and writes the
  // stash out in one burst when it is full and once more after its last tile, when nothing is
  // left to wait for.
  // With EXPOSE == 2 a tile has one more row: ||k_j||^2 of its 32 positions, for the key-norm factor of
  // the Selector's prior (Eq. selector_prior_kn).
  const int rows_exp = G + (EXPOSE == 2 ? 1 : 0);
  float* stash = EXPOSE != 0 ? &s_stash[w][0] : nullptr;
  float* lg_base = EXPOSE != 0 ? a.logits + (int64_t)bh * rows_exp * a.ld_pos : nullptr;
  const int tile_f4 = rows_exp * (kTile / 4);        // float4 per tile
  const int stash_cap = kStash / (rows_exp * kTile);  // tiles the stash holds
  int n_stashed = 0, k_flushed = 0;
  auto flush_stash = [&]() {
    __builtin_amdgcn_wave_barrier();
    const int n_f4 = n_stashed * tile_f4;
    for (int f = lane; f < n_f4; f += 64) {
      const int i = f / tile_f4, rem = f - i * tile_f4;
      const int t = first + (k_flushed + i) * step;
      *reinterpret_cast<float4*>(lg_base + ((int64_t)t * tile_f4 + rem) * 4) = *reinterpret_cast<const float4*>(stash + f * 4);
    }
    __builtin_amdgcn_wave_barrier();
    k_flushed += n_stashed;
    n_stashed = 0;
  };
  auto write_record = [&](int wslot) {
    float lr = l_run;
    lr += __shfl_xor(lr, 16);
    lr += __shfl_xor(lr, 32);
    write_wave_record(a.part, head0, G, wslot, acc, m_run, lr, lane, !NOV);
  };

  // One loop for all of the wave's tiles.  A tile buffer's K half is refilled with the rows of the
  // tile that uses the buffer next as soon as the logits are out, its V half as soon as P V is done,
  // so rows are on their way during all of the math (with two buffers, a whole tile more than with
  // one).  The refill is unconditional -- past the wave's last tile it degenerates to re-reading row
  // L - 1 -- so that no branch surrounds a load and every wait can name exactly the loads it needs.
  auto tile_step = [&](Tile& T, int k) {
    const int t = first + k * step;
    const bool inJ = k < KJ;
    if (k == KJ) {  // the J tiles are done (or there were none): close the J record, start the other one
      write_record(first);
#pragma unroll
      for (int e = 0; e < 8; ++e) acc[e] = f32x4{0.f, 0.f, 0.f, 0.f};
      m_run = kNeg;
      l_run = 0.f;
    }
    float y[8];
    f32x4 s4[4];
    if (WIDE) qk_products_wide(T, qreg, s4);  // the refill of the K half below goes out before the lane exchanges
    else qk_phase(T, qreg, a.scale_log2, y);
    float k2a = 0.f, k2b = 0.f;
    if (EXPOSE == 2) knorm_phase(T, jg, n, k2a, k2b);
    int pra = 0, prb = 0;
    if (PAGED) {
      pra = P.phys(row_for(t + step, n), pa_n, bad);
      prb = P.phys(row_for(t + step, 16 + n), pb_n, bad);
      issue_k_rows<uint64_t>(T, R, pra, prb);
      pa_n = P.page_of(row_for(t + 2 * step, n));
      pb_n = P.page_of(row_for(t + 2 * step, 16 + n));
    } else {
      issue_k_tile(T, t + NB * step);
    }
    if (WIDE) {
      __builtin_amdgcn_sched_barrier(0);
      qk_join_wide(s4, a.scale_log2, y);
    }
    if (EXPOSE != 0 && inJ) {  // positions past |J| land in the padding of the last tile, never used
      float* st = stash + n_stashed * (rows_exp * kTile);
      stage_logits<WIDE>(st, y, jg, n, G);
      if (EXPOSE == 2 && jg == (n >> 2)) {
        st[G * kTile + n] = k2a;
        st[G * kTile + 16 + n] = k2b;
      }
      if (++n_stashed == stash_cap) flush_stash();
    }
    const int p0 = (inJ ? t : t - nTJ) * kTile;
    const int N = inJ ? NJ : NS;
    if (p0 + kTile > N) mask_tail<!NOV, WIDE>(T, y, jg, p0, N);
    bf16x8 a_hi, a_lo;
    softmax_phase(y, acc, m_run, l_run, jg, a_hi, a_lo);
    if (!NOV) pv_phase(T, a_hi, a_lo, acc);
    if (PAGED && !NOV) issue_v_rows<uint64_t>(T, R, pra, prb);
    else if (!PAGED) issue_v_tile(T, t + NB * step);
  };
  if (PAGED) {
    for (int k = 0; k < K; ++k) tile_step(T, k);
  } else {
    // (an odd last tile is taken after the loop: a way out of the middle of the loop body would put a
    // path from the first buffer's refill straight to its next use into the flow graph, and the waits
    // would be placed for that path)
    int k = 0;
    for (; k + 1 < K; k += 2) {
      tile_step(T, k);
      tile_step(T2, k + 1);
    }
    if (k < K) tile_step(T, k);
  }
  if (EXPOSE != 0) flush_stash();
  // the record still open: the J record if the wave had no other tile (slot first), else the record of
  // its sink / recent tiles, slot n_waves + e with e the rank of its first such tile among them
  write_record(K == KJ ? first : n_waves + (first + KJ * step - nTJ));
  report_guard(a.guard, bad);
}
// One workgroup per (split, KV head, sequence) cell ...
template <int EXPOSE, bool PAGED, bool BIG = false, bool NOV = false, bool WIDE = false>
__global__ __launch_bounds__(kAttnThreads, BIG ? 1 : 2) void attn_dense_kernel(const AttnArgs a) {
  dense_body<EXPOSE, PAGED, BIG, NOV, WIDE>(a, a.n_split, blockIdx.x, blockIdx.y, blockIdx.z);
}
// ... or, in the ragged step (sfi_mixed_step*), one workgroup per compute unit that plans the launch on the device.
// Which sequences are slow is only known there, so the host cannot size the launch for them: one workgroup per (split,
// KV head, sequence) cell with the finest split and an early exit for fast sequences leaves the kernel with a handful
// of tiles per wave (a wave's start and end weigh as much as its tiles), thousands of empty workgroups, and shares
// that follow the sequences' lengths.  Here every workgroup builds the same plan from the flags and lengths: the slow
// sequences' ids; for each its tiles T_r (the body's own count: tiles of J plus tiles of sink ++ recent) and its splits
// s_r = T_r x (grid / Hkv) / sum T rounded down, at least 1 and at most the host's bound a.n_split or one tile per
// wave, what the rounding left over going one by one to the sequence with the most tiles per split -- so that the cells
// (r, h, slot < s_r) number one per workgroup and hold the same number of tiles whatever the sequences' lengths (with
// many slow sequences: about four splits each, dealt round robin).  Workgroup i takes cells i, i + grid, ...; workgroup
// 0 leaves s_r in a.seq_splits for the launches that merge the records.
// The waves of a workgroup share no LDS in the body, so a wave may be on the workgroup's next cell while another is
// still on this one.  A cell's coordinates are made scalars again (they come out of LDS), so that the body's addressing
// stays on the scalar unit as it is with block indices.
template <int EXPOSE, bool PAGED>
__global__ __launch_bounds__(kAttnThreads, 1) void attn_dense_items_kernel(const AttnArgs a) {
  __shared__ int s_list[kListCap];       // slow sequence ids, ascending
  __shared__ int s_tiles[kListCap];      // their tiles
  __shared__ int s_split[kListCap];      // their splits
  __shared__ int s_first[kListCap + 1];  // cells in front of sequence r (prefix of s_r * Hkv)
  __shared__ int s_scr[8];
  const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
  // flags and lengths of this thread's four sequences, all requested together
  int flag[4], len[4], c = 0;
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    const int b = min(4 * tid + j, a.item_batch - 1);
    flag[j] = a.is_slow[(int64_t)b * a.fs];
    len[j] = a.ctx_len[(int64_t)b * a.ms];
  }
  int tiles = 0;
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    flag[j] = 4 * tid + j < a.item_batch && flag[j] != 0;
    const int L = min(max(len[j], 0), a.len_cap);
    const int NJ = max(0, L - a.recent - a.n_sink);
    const int nS = min(a.n_sink, L), rs = min(max(a.n_sink, L - a.recent), L);
    len[j] = (NJ + kTile - 1) / kTile + (nS + (L - rs) + kTile - 1) / kTile;  // from here on: the sequence's tiles
    c += flag[j];
    tiles += flag[j] ? len[j] : 0;
  }
  int inc = c;
#pragma unroll
  for (int d = 1; d < 64; d <<= 1) {
    const int t = __shfl_up(inc, d);
    if (lane >= d) inc += t;
  }
#pragma unroll
  for (int d = 32; d >= 1; d >>= 1) tiles += __shfl_xor(tiles, d);
  if (lane == 63) s_scr[w] = inc;
  if (lane == 0) s_scr[4 + w] = tiles;
  __syncthreads();
  int base = 0, n_slow = 0;
#pragma unroll
  for (int i = 0; i < kWaves; ++i) {
    const int t = s_scr[i];
    if (i < w) base += t;
    n_slow += t;
  }
  n_slow = __builtin_amdgcn_readfirstlane(n_slow);
  if (n_slow == 0) return;
  const int total = max(1, s_scr[4] + s_scr[5] + s_scr[6] + s_scr[7]);
  // splits to hand out among the slow sequences: one cell per workgroup, or, with many slow sequences, about four
  // splits each, so that dealing the cells round robin still balances
  const int per_head = max(max(1, (int)gridDim.x / a.Hkv), 4 * n_slow);
  {
    int o = base + inc - c;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      if (flag[j]) {
        s_list[o] = 4 * tid + j;
        s_tiles[o] = len[j];
        const int want = (int)((int64_t)len[j] * per_head / total);  // rounded down: the sum must not pass per_head
        s_split[o] = max(1, min(want, min(a.n_split, (len[j] + kWaves - 1) / kWaves)));
        ++o;
      }
    }
  }
  __syncthreads();
  if (tid == 0) {  // (a few dozen sequences at most in practice; done by one thread, the plan is the same everywhere)
    int acc = 0;
    for (int r = 0; r < n_slow; ++r) acc += s_split[r];
    // what rounding down left over goes, one split at a time, to the sequence with the most tiles per split
    for (int left = per_head - acc; left > 0 && n_slow <= 64; --left) {
      int best = -1;
      float worst = 0.f;
      for (int r = 0; r < n_slow; ++r) {
        const int cap = min(a.n_split, (s_tiles[r] + kWaves - 1) / kWaves);
        const float load = (float)s_tiles[r] / (float)s_split[r];
        if (s_split[r] < cap && load > worst) {
          worst = load;
          best = r;
        }
      }
      if (best < 0) break;
      ++s_split[best];
    }
    acc = 0;
    for (int r = 0; r < n_slow; ++r) {
      s_first[r] = acc;
      acc += s_split[r] * a.Hkv;
    }
    s_first[n_slow] = acc;
  }
  __syncthreads();
  if (blockIdx.x == 0)
    for (int r = tid; r < n_slow; r += kAttnThreads) a.seq_splits[s_list[r]] = s_split[r];
  const int n_items = __builtin_amdgcn_readfirstlane(s_first[n_slow]);
  for (int item = blockIdx.x; item < n_items; item += gridDim.x) {
    int lo = 0, hi = n_slow;  // the sequence whose cells include this one: s_first[lo] <= item < s_first[lo + 1]
    while (hi - lo > 1) {
      const int mid = (lo + hi) >> 1;
      if (s_first[mid] <= item) lo = mid;
      else hi = mid;
    }
    const int r = lo;
    const int ns = __builtin_amdgcn_readfirstlane(s_split[r]);
    const int rem = item - __builtin_amdgcn_readfirstlane(s_first[r]);
    const int h = rem / ns;
    const int b = __builtin_amdgcn_readfirstlane(s_list[r]);
    // A zero the compiler cannot see through: without it everything the body derives from the thread index is
    // computed once in front of this loop and kept in registers across the body.
    int zero = 0;
    asm volatile("" : "+s"(zero));
    dense_body<EXPOSE, PAGED, true, false, false>(a, ns, rem - h * ns, h, b, zero);
  }
}

// Where a fast-step workgroup's result goes.
struct WgOut {
  float* out_direct;   // the workgroup is the only one of its (b, h) pair: it writes O / l straight to out[b, head, :]
  float* out_merge;    // or: records go out in device-scope stores and the pair's last workgroup merges them into this
  uint32_t* arrive;    //   (finish_pair); arrive counts the pair's workgroups that have sent theirs
  float* part;         // the records (with neither pointer above: a merge launch follows)
  int n_split, slot_cap;
  bool out_bf16;
};
__device__ __forceinline__ WgOut wg_out_of(const AttnArgs& a, int bh) {
  WgOut o;
  o.out_direct = a.out_direct;
  o.out_merge = a.out_merge;
  o.arrive = a.arrive != nullptr ? a.arrive + bh : nullptr;
  o.part = a.part;
  o.n_split = a.n_split;
  o.slot_cap = a.slot_cap;
  o.out_bf16 = a.out_bf16 != 0;
  return o;
}
// The four waves' partial results combined through LDS, then sent where WgOut says.
template <int NW = kWaves, int HMAX = 16>  // waves of the workgroup; query heads the reduction buffer has room for (>= G)
__device__ __forceinline__ void write_wg_record(const WgOut& o, int64_t head0, int G, int slot, const f32x4 (&acc)[8],
                                                float m_run, float l_run) {
  const int tid = threadIdx.x;
  const int lane = tid & 63, w = tid >> 6;
  const int jg = lane >> 4, n = lane & 15;
  __shared__ float s_m[NW][16];
  __shared__ float s_l[NW][16];
  __shared__ __align__(16) float s_red[NW][HMAX][kHeadDim];
  if (lane < 16) {
    s_m[w][lane] = m_run;
    s_l[w][lane] = l_run;
  }
  __syncthreads();
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int hh = 4 * jg + i;
    if (hh < G) {
      float M = s_m[0][hh];
#pragma unroll
      for (int ww = 1; ww < NW; ++ww) M = fmaxf(M, s_m[ww][hh]);
      const float f = fast_exp2(s_m[w][hh] - M);
      float* dst = &s_red[w][hh][n * 8];
      *reinterpret_cast<float4*>(dst) = make_float4(acc[0][i] * f, acc[1][i] * f, acc[2][i] * f, acc[3][i] * f);
      *reinterpret_cast<float4*>(dst + 4) = make_float4(acc[4][i] * f, acc[5][i] * f, acc[6][i] * f, acc[7][i] * f);
    }
  }
  __syncthreads();
  if (o.out_direct != nullptr) {  // block-uniform
    for (int idx = tid; idx < G * kHeadDim; idx += NW * 64) {
      const int hh = idx >> 7, dim = idx & 127;
      float M = s_m[0][hh];
#pragma unroll
      for (int ww = 1; ww < NW; ++ww) M = fmaxf(M, s_m[ww][hh]);
      float ls = 0.f, sum = 0.f;
#pragma unroll
      for (int ww = 0; ww < NW; ++ww) {
        ls += s_l[ww][hh] * fast_exp2(s_m[ww][hh] - M);
        sum += s_red[ww][hh][dim];
      }
      store_out(o.out_direct, (head0 + hh) * kHeadDim + dim, ls > 0.f ? sum / ls : 0.f, o.out_bf16);
    }
    return;
  }
  const bool tail = o.out_merge != nullptr;  // block-uniform
  // slot_cap: records each query head has room for (kSlotCap in a caller's workspace, fewer in the static scratch)
  float* const pair_base = o.part + head0 * o.slot_cap * kPartStride;
  const __amdgpu_buffer_rsrc_t R = pair_records(pair_base, G * o.slot_cap * kPartStride * (int)sizeof(float));
  for (int idx = tid; idx < G * (kHeadDim / 4); idx += NW * 64) {  // one thread per (head, four dims): 16-byte stores
    const int hh = idx >> 5, c = idx & 31;
    float4 s = *reinterpret_cast<const float4*>(&s_red[0][hh][4 * c]);
#pragma unroll
    for (int ww = 1; ww < NW; ++ww) {
      const float4 t = *reinterpret_cast<const float4*>(&s_red[ww][hh][4 * c]);
      s.x += t.x; s.y += t.y; s.z += t.z; s.w += t.w;
    }
    const int off = (hh * o.slot_cap + slot) * kPartStride + 4 + 4 * c;  // in floats, from the pair's first record
    if (tail) store_device4(R, off * (int)sizeof(float), s);
    else *reinterpret_cast<float4*>(pair_base + off) = s;
  }
  if (tid < G) {
    float M = s_m[0][tid];
#pragma unroll
    for (int ww = 1; ww < NW; ++ww) M = fmaxf(M, s_m[ww][tid]);
    float ls = 0.f;
#pragma unroll
    for (int ww = 0; ww < NW; ++ww) ls += s_l[ww][tid] * fast_exp2(s_m[ww][tid] - M);
    const int off = (tid * o.slot_cap + slot) * kPartStride;
    if (tail) store_device2(R, off * (int)sizeof(float), M, ls);
    else *reinterpret_cast<float2*>(pair_base + off) = make_float2(M, ls);
  }
  if (tail) finish_pair<NW>(o.part, head0, G, o.n_split, o.arrive, o.out_merge, o.out_bf16, o.slot_cap);
}

// ------------------------------------------------------------------------------------------------
// gather kernel
// ------------------------------------------------------------------------------------------------
template <bool PAGED, bool WIDE>
__global__ __launch_bounds__(kAttnThreads, 3) void attn_gather_kernel(const AttnArgs a) {
  constexpr int NW = kWaves;
  const int slot = blockIdx.x, h = blockIdx.y, b = blockIdx.z;
  if (a.is_slow != nullptr && a.is_slow[b * a.fs] != 0) return;
  const int tid = threadIdx.x;
  const int lane = tid & 63, w = tid >> 6;
  const int jg = lane >> 4, n = lane & 15;
  const int G = a.G;
  const int bh = b * a.Hkv + h;
  const int64_t head0 = (int64_t)b * a.Hq + h * G;
  const int first = slot * NW + w, step = a.n_split * NW;
  // The step's three scalars are requested together, ahead of everything else: read one by one where
  // they are used, the wait for the first would hold back the requests for the others (a round trip each).
  const int L_in = a.ctx_len[b * a.ms], n_sel_in = a.n_sel[bh], rs_in = a.recent_start[b * a.ms];

  // ---- first round of loads, none depending on another: the selected indices of this wave's first
  // tile (read before the list length is known, clamped to the row of sel_idx), q, the scalars.
  ListWalk W;
  W.sel = a.sel_idx + (int64_t)bh * a.sel_stride;
  W.sel_cap = (int)a.sel_stride - 1;
  W.n_sink = a.n_sink;
  int sA = W.sel_at(first * kTile + n);
  int sB = W.sel_at(first * kTile + 16 + n);
  bf16x8 qreg[4];
  load_q<WIDE>(qreg, a.q, head0, G, jg, n);
  W.bad = 0;
  const int L = guarded_len(L_in, a.len_cap, W.bad);
  W.set_counts(L, n_sel_in, rs_in, (int)a.sel_stride);

  Rows R;
  R.Kb = reinterpret_cast<const char*>(a.K + b * a.k_sb + h * a.k_sh);
  R.Vb = reinterpret_cast<const char*>(a.V + b * a.v_sb + h * a.v_sh);
  R.k_st = (uint32_t)a.k_st * 2u;
  R.v_st = (uint32_t)a.v_st * 2u;
  R.k_lane = k_lane_of<WIDE>(jg, n);
  R.v_lane = n * 16;
  R.jg = jg;
  R.n = n;

  Tile T;
  float m_run = kNeg, l_run = 0.f;
  f32x4 acc[8];
#pragma unroll
  for (int e = 0; e < 8; ++e) acc[e] = f32x4{0.f, 0.f, 0.f, 0.f};

  const int nT = (W.N + kTile - 1) / kTile;
  for (int t = first; t < nT; t += step) {  // normally a single trip
    const int p0 = t * kTile;
    if (t != first) {
      sA = W.sel_at(p0 + n);
      sB = W.sel_at(p0 + 16 + n);
    }
    int ra = W.row_of(p0 + n, sA), rb = W.row_of(p0 + 16 + n, sB);
    if (PAGED) {  // one more dependent round: row -> block-table entry -> physical row
      const Pages P = pages_of(a, b, L);
      ra = P.phys(ra, P.page_of(ra), W.bad);
      rb = P.phys(rb, P.page_of(rb), W.bad);
    }
    issue_rows<typename RowOff<PAGED>::type, WIDE>(T, R, ra, rb);
    if (p0 + kTile <= W.N) tile_math<false, WIDE>(T, qreg, a.scale_log2, acc, m_run, l_run, jg, p0, W.N);
    else tile_math<true, WIDE>(T, qreg, a.scale_log2, acc, m_run, l_run, jg, p0, W.N);
  }
  l_run += __shfl_xor(l_run, 16);
  l_run += __shfl_xor(l_run, 32);
  write_wg_record(wg_out_of(a, bh), head0, G, slot, acc, m_run, l_run);
  report_guard(a.guard, W.bad);  // last: the way to the record and the merge is the launch's critical path
}

// ------------------------------------------------------------------------------------------------
// gather kernel, pipelined: for launches whose index lists are long or many enough that one tile
// per wave would take several rounds of workgroups (large batches, large budgets).  Few workgroups
// per (b, h), each wave walks tiles first, first + step, ... with the dense kernel's loop: one tile
// buffer whose K half is refilled with the next tile's rows right after S^T, the V half right
// after P V; the selected indices are read two tiles ahead.  Loads past the wave's last tile fall
// on row 0 (no branch around a load, so every wait names exactly the loads it needs).
// ------------------------------------------------------------------------------------------------
template <bool PAGED, bool WIDE>
__global__ __launch_bounds__(kAttnThreads, 3) void attn_gather_stream_kernel(const AttnArgs a) {
  const int slot = blockIdx.x, h = blockIdx.y, b = blockIdx.z;
  if (a.is_slow != nullptr && a.is_slow[b * a.fs] != 0) return;
  const int tid = threadIdx.x;
  const int lane = tid & 63, w = tid >> 6;
  const int jg = lane >> 4, n = lane & 15;
  const int G = a.G;
  const int bh = b * a.Hkv + h;
  const int64_t head0 = (int64_t)b * a.Hq + h * G;
  const int first = slot * kWaves + w, step = a.n_split * kWaves;
  const int pstep = step * kTile;
  // The step's three scalars are requested together, ahead of everything else: read one by one where
  // they are used, the wait for the first would hold back the requests for the others (a round trip each).
  const int L_in = a.ctx_len[b * a.ms], n_sel_in = a.n_sel[bh], rs_in = a.recent_start[b * a.ms];

  ListWalk W;
  W.sel = a.sel_idx + (int64_t)bh * a.sel_stride;
  W.sel_cap = max((int)a.sel_stride - 1, 0);  // sel_stride = 0: the host points sel_idx at one readable word
  W.n_sink = a.n_sink;
  const int p_first = first * kTile;
  const int sA = W.sel_at_nonempty(p_first + n), sB = W.sel_at_nonempty(p_first + 16 + n);
  bf16x8 qreg[4];
  load_q<WIDE>(qreg, a.q, head0, G, jg, n);
  W.bad = 0;
  const int L = guarded_len(L_in, a.len_cap, W.bad);
  W.set_counts(L, n_sel_in, rs_in, (int)a.sel_stride);

  Rows R;
  R.Kb = reinterpret_cast<const char*>(a.K + b * a.k_sb + h * a.k_sh);
  R.Vb = reinterpret_cast<const char*>(a.V + b * a.v_sb + h * a.v_sh);
  R.k_st = (uint32_t)a.k_st * 2u;
  R.v_st = (uint32_t)a.v_st * 2u;
  R.k_lane = k_lane_of<WIDE>(jg, n);
  R.v_lane = n * 16;
  R.jg = jg;
  R.n = n;

  Tile T;
  float m_run = kNeg, l_run = 0.f;
  f32x4 acc[8];
#pragma unroll
  for (int e = 0; e < 8; ++e) acc[e] = f32x4{0.f, 0.f, 0.f, 0.f};

  const int nT = (W.N + kTile - 1) / kTile;
  const int K = first < nT ? (nT - first + step - 1) / step : 0;
  // Memory instructions go out in the same order here as in an iteration of the loop below -- K rows,
  // the indices of the tile after, V rows -- so the in-order load counter reads the same on both ways
  // into the loop.  A wave without tiles reads row 0 and skips the loop.
  // PAGED adds one stage to the pipeline: indices are read two tiles ahead, the block-table entries
  // of the rows they name one tile ahead (order: K rows, table entries, indices, V rows).
  int sAn, sBn;            // !PAGED: indices of the next tile; PAGED: of the tile after the next
  int ra_n = 0, rb_n = 0;  // PAGED: logical rows of the next tile and their block-table entries
  int pa_n = 0, pb_n = 0;
  Pages P;
  if (PAGED) {
    P = pages_of(a, b, L);
    const int sA1 = W.sel_at_nonempty(p_first + pstep + n), sB1 = W.sel_at_nonempty(p_first + pstep + 16 + n);
    int ra = W.row_of(p_first + n, sA), rb = W.row_of(p_first + 16 + n, sB);
    ra = P.phys(ra, P.page_of(ra), W.bad);
    rb = P.phys(rb, P.page_of(rb), W.bad);
    __builtin_amdgcn_sched_barrier(0);
    issue_k_rows<typename RowOff<PAGED>::type, WIDE>(T, R, ra, rb);
    __builtin_amdgcn_sched_barrier(0);
    ra_n = W.row_of(p_first + pstep + n, sA1);
    rb_n = W.row_of(p_first + pstep + 16 + n, sB1);
    pa_n = P.page_of(ra_n);
    pb_n = P.page_of(rb_n);
    __builtin_amdgcn_sched_barrier(0);
    sAn = W.sel_at_nonempty(p_first + 2 * pstep + n);
    sBn = W.sel_at_nonempty(p_first + 2 * pstep + 16 + n);
    __builtin_amdgcn_sched_barrier(0);
    issue_v_rows<typename RowOff<PAGED>::type, WIDE>(T, R, ra, rb);
    __builtin_amdgcn_sched_barrier(0);
  } else {
    const int ra = W.row_of(p_first + n, sA), rb = W.row_of(p_first + 16 + n, sB);
    __builtin_amdgcn_sched_barrier(0);  // the compiler's scheduler must not reorder the three groups
    issue_k_rows<typename RowOff<PAGED>::type, WIDE>(T, R, ra, rb);
    __builtin_amdgcn_sched_barrier(0);
    sAn = W.sel_at_nonempty(p_first + pstep + n);
    sBn = W.sel_at_nonempty(p_first + pstep + 16 + n);
    __builtin_amdgcn_sched_barrier(0);
    issue_v_rows<typename RowOff<PAGED>::type, WIDE>(T, R, ra, rb);
    __builtin_amdgcn_sched_barrier(0);
  }
  // The last tile is taken after the loop, without the refill: no rows are requested for a tile that does not
  // exist, and nothing is in flight when the wave reaches the record write (worth 0.05 us at most: the tail
  // waits for its own stores far longer than for such rows).
  for (int k = 0; k + 1 < K; ++k) {
    const int p0 = p_first + k * pstep;
    const int pn = p0 + pstep;
    float y[8];
    qk_phase<WIDE>(T, qreg, a.scale_log2, y);
    int ra, rb;
    if (PAGED) {
      ra = P.phys(ra_n, pa_n, W.bad);
      rb = P.phys(rb_n, pb_n, W.bad);
      issue_k_rows<typename RowOff<PAGED>::type, WIDE>(T, R, ra, rb);
      ra_n = W.row_of(pn + pstep + n, sAn);  // row 0 past the list
      rb_n = W.row_of(pn + pstep + 16 + n, sBn);
      pa_n = P.page_of(ra_n);
      pb_n = P.page_of(rb_n);
      sAn = W.sel_at_nonempty(pn + 2 * pstep + n);
      sBn = W.sel_at_nonempty(pn + 2 * pstep + 16 + n);
    } else {
      ra = W.row_of(pn + n, sAn);  // row 0 past the list
      rb = W.row_of(pn + 16 + n, sBn);
      issue_k_rows<typename RowOff<PAGED>::type, WIDE>(T, R, ra, rb);
      sAn = W.sel_at_nonempty(pn + pstep + n);
      sBn = W.sel_at_nonempty(pn + pstep + 16 + n);
    }
    if (p0 + kTile > W.N) mask_tail<true, WIDE>(T, y, jg, p0, W.N);
    bf16x8 a_hi, a_lo;
    softmax_phase(y, acc, m_run, l_run, jg, a_hi, a_lo);
    pv_phase(T, a_hi, a_lo, acc);
    issue_v_rows<typename RowOff<PAGED>::type, WIDE>(T, R, ra, rb);
  }
  if (K > 0) {
    const int p0 = p_first + (K - 1) * pstep;
    float y[8];
    qk_phase<WIDE>(T, qreg, a.scale_log2, y);
    if (p0 + kTile > W.N) mask_tail<true, WIDE>(T, y, jg, p0, W.N);
    bf16x8 a_hi, a_lo;
    softmax_phase(y, acc, m_run, l_run, jg, a_hi, a_lo);
    pv_phase(T, a_hi, a_lo, acc);
  }
  l_run += __shfl_xor(l_run, 16);
  l_run += __shfl_xor(l_run, 32);
  write_wg_record(wg_out_of(a, bh), head0, G, slot, acc, m_run, l_run);
  report_guard(a.guard, W.bad);  // last: the way to the record and the merge is the launch's critical path
}

// ------------------------------------------------------------------------------------------------
// Memory skeleton of the fast step -- a measurement aid, not part of the path.  Same grid, same three
// scalars, same index loads and the same row loads as the gather kernels, but no arithmetic: what
// arrives is folded into one word per lane.  It answers what a launch of this shape costs when the
// matrix and vector units do nothing, i.e. the floor the real kernel can be held against.
//   TAIL   the workgroup's record goes through the same LDS combine, device-scope record stores,
//          arrival counter and last-workgroup merge as in the real kernel (the numbers are junk);
//          without it every workgroup ends with one plain 4-byte store.
//   BURST  instead of walking its tiles with one register buffer (K half and V half refilled as the
//          real loop does), a wave requests the rows of all its tiles at once, straight into LDS
//          (global_load_lds, 16 bytes per lane), and waits once: the most requests in flight the
//          launch shape allows.  The workgroup owns tiles [slot * tpw, (slot + 1) * tpw) of the list,
//          wave w the tiles w, w + 4, ... of that range; tpw * 16 KB of dynamic LDS.
// ------------------------------------------------------------------------------------------------
__device__ __forceinline__ uint32_t fold16(const uint4& v) { return v.x ^ v.y ^ v.z ^ v.w; }

//   depth  1: stop after the scalars and indices; 2: load nothing at all (the cost of the bare launch).
template <bool WIDE, bool TAIL, bool BURST>
__global__ __launch_bounds__(kAttnThreads, BURST ? 1 : 3) void attn_gather_floor_kernel(const AttnArgs a, int tpw, int depth) {
  extern __shared__ uint4 s_rows[];  // BURST: [tpw][16 instructions][64 lanes]
  const int slot = blockIdx.x, h = blockIdx.y, b = blockIdx.z;
  const int tid = threadIdx.x;
  const int lane = tid & 63, w = tid >> 6;
  const int jg = lane >> 4, n = lane & 15;
  const int G = a.G;
  const int bh = b * a.Hkv + h;
  const int64_t head0 = (int64_t)b * a.Hq + h * G;
  uint32_t fold = 0u;
  if (!TAIL && !BURST && depth == 2) {  // wave-uniform: the bare launch
    if (lane == 0) reinterpret_cast<uint32_t*>(a.part)[((head0 * a.slot_cap + slot) * kPartStride) + w] = (uint32_t)slot;
    return;
  }
  const int L_in = a.ctx_len[b * a.ms], n_sel_in = a.n_sel[bh], rs_in = a.recent_start[b * a.ms];
  ListWalk W;
  W.sel = a.sel_idx + (int64_t)bh * a.sel_stride;
  W.sel_cap = max((int)a.sel_stride - 1, 0);
  W.n_sink = a.n_sink;
  W.bad = 0;
  Rows R;
  R.Kb = reinterpret_cast<const char*>(a.K + b * a.k_sb + h * a.k_sh);
  R.Vb = reinterpret_cast<const char*>(a.V + b * a.v_sb + h * a.v_sh);
  R.k_st = (uint32_t)a.k_st * 2u;
  R.v_st = (uint32_t)a.v_st * 2u;
  R.k_lane = k_lane_of<WIDE>(jg, n);
  R.v_lane = n * 16;
  R.jg = jg;
  R.n = n;
  if (!TAIL && !BURST && depth == 1) {  // wave-uniform: scalars and the first tile's indices, nothing else
    const int first = slot * kWaves + w;
    const int sA = W.sel_at_nonempty(first * kTile + n), sB = W.sel_at_nonempty(first * kTile + 16 + n);
    fold = (uint32_t)(L_in ^ n_sel_in ^ rs_in ^ sA ^ sB);
#pragma unroll
    for (int d = 32; d >= 1; d >>= 1) fold ^= __shfl_xor(fold, d);
    if (lane == 0) reinterpret_cast<uint32_t*>(a.part)[((head0 * a.slot_cap + slot) * kPartStride) + w] = fold;
    return;
  }
  if (BURST) {
    // indices of all of this wave's tiles first (rows n and 16 + n of each), then the scalars
    constexpr int kMaxT = 4;  // tiles per wave: tpw <= 16
    int sA[kMaxT], sB[kMaxT];
#pragma unroll
    for (int k = 0; k < kMaxT; ++k) {
      const int p0 = (slot * tpw + w + kWaves * k) * kTile;
      sA[k] = W.sel_at_nonempty(p0 + n);
      sB[k] = W.sel_at_nonempty(p0 + 16 + n);
    }
    const int L = guarded_len(L_in, a.len_cap, W.bad);
    W.set_counts(L, n_sel_in, rs_in, (int)a.sel_stride);
    const int nT = (W.N + kTile - 1) / kTile;
#pragma unroll
    for (int k = 0; k < kMaxT; ++k) {
      const int lt = w + kWaves * k;            // tile within the workgroup's range
      const int t = slot * tpw + lt;
      if (lt < tpw && t < nT) {                 // wave-uniform
        const int p0 = t * kTile;
        const int ra = W.row_of(p0 + n, sA[k]), rb = W.row_of(p0 + 16 + n, sB[k]);
        uint4* dst = s_rows + (size_t)lt * 16 * 64;
#pragma unroll
        for (int i = 0; i < 8; ++i) {           // instruction i: rows 4 i .. 4 i + 3 of the tile, 16 lanes x 16 bytes each
          const int row = __shfl(i < 4 ? ra : rb, (4 * i + jg) & 15);  // resolved by the lane that holds that position
          const char* gk = R.Kb + (size_t)((uint32_t)row * R.k_st + (uint32_t)n * 16u);
          const char* gv = R.Vb + (size_t)((uint32_t)row * R.v_st + (uint32_t)n * 16u);
          __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)gk,
                                           (__attribute__((address_space(3))) void*)(dst + i * 64), 16, 0, 0);
          __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)gv,
                                           (__attribute__((address_space(3))) void*)(dst + (8 + i) * 64), 16, 0, 0);
        }
      }
    }
    __builtin_amdgcn_s_waitcnt(0x0F70);  // vmcnt(0): every row of this wave has landed in LDS
#pragma unroll
    for (int k = 0; k < kMaxT; ++k) {
      const int lt = w + kWaves * k;
      const int t = slot * tpw + lt;
      if (lt < tpw && t < nT) {
        const uint4* src = s_rows + (size_t)lt * 16 * 64;
        for (int i = 0; i < 16; ++i) fold ^= fold16(src[i * 64 + lane]);
      }
    }
  } else {
    const int first = slot * kWaves + w, step = a.n_split * kWaves;
    const int pstep = step * kTile;
    const int p_first = first * kTile;
    const int sA = W.sel_at_nonempty(p_first + n), sB = W.sel_at_nonempty(p_first + 16 + n);
    const int L = guarded_len(L_in, a.len_cap, W.bad);
    W.set_counts(L, n_sel_in, rs_in, (int)a.sel_stride);
    Tile T;
    const int nT = (W.N + kTile - 1) / kTile;
    const int K = first < nT ? (nT - first + step - 1) / step : 0;
    int ra = W.row_of(p_first + n, sA), rb = W.row_of(p_first + 16 + n, sB);
    __builtin_amdgcn_sched_barrier(0);
    issue_k_rows<uint32_t, WIDE>(T, R, ra, rb);
    __builtin_amdgcn_sched_barrier(0);
    int sAn = W.sel_at_nonempty(p_first + pstep + n), sBn = W.sel_at_nonempty(p_first + pstep + 16 + n);
    __builtin_amdgcn_sched_barrier(0);
    issue_v_rows<uint32_t, WIDE>(T, R, ra, rb);
    __builtin_amdgcn_sched_barrier(0);
    for (int k = 0; k + 1 < K; ++k) {
      const int pn = p_first + (k + 1) * pstep;
#pragma unroll
      for (int i = 0; i < 4; ++i) fold ^= fold16(T.ka[i]) ^ fold16(T.kb[i]);   // the K half is consumed ...
      ra = W.row_of(pn + n, sAn);
      rb = W.row_of(pn + 16 + n, sBn);
      issue_k_rows<uint32_t, WIDE>(T, R, ra, rb);                              // ... and refilled,
      sAn = W.sel_at_nonempty(pn + pstep + n);
      sBn = W.sel_at_nonempty(pn + pstep + 16 + n);
#pragma unroll
      for (int i = 0; i < 8; ++i) fold ^= fold16(T.v[i]);                      // then the V half
      issue_v_rows<uint32_t, WIDE>(T, R, ra, rb);
    }
    if (K > 0) {
#pragma unroll
      for (int i = 0; i < 4; ++i) fold ^= fold16(T.ka[i]) ^ fold16(T.kb[i]);
#pragma unroll
      for (int i = 0; i < 8; ++i) fold ^= fold16(T.v[i]);
    }
  }
  if (TAIL) {
    f32x4 acc[8];
    const float v = (float)(fold & 0xffu);
#pragma unroll
    for (int e = 0; e < 8; ++e) acc[e] = f32x4{v, v, v, v};
    write_wg_record(wg_out_of(a, bh), head0, G, slot, acc, 0.f, 1.f);
  } else {
    fold ^= __shfl_xor(fold, 32);
    if (lane == 0) reinterpret_cast<uint32_t*>(a.part)[((head0 * a.slot_cap + slot) * kPartStride) + w] = fold;
  }
  report_guard(a.guard, W.bad);
}

hipError_t launch_attn_gather_floor(const AttnArgs& a, int B, int n_slots, int tail, int burst, int tpw, int depth, hipStream_t s) {
  const dim3 grid(n_slots, a.Hkv, B);
  const size_t lds = burst ? (size_t)tpw * 16 * 64 * sizeof(uint4) : 0;
#define SFI_FLOOR(WIDE, TAIL, BURST)                                                                                   \
  do {                                                                                                                 \
    if (lds > 0 && hipFuncSetAttribute(reinterpret_cast<const void*>(&attn_gather_floor_kernel<WIDE, TAIL, BURST>),   \
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds) != hipSuccess)            \
      return hipGetLastError();                                                                                        \
    hipLaunchKernelGGL((attn_gather_floor_kernel<WIDE, TAIL, BURST>), grid, dim3(kAttnThreads), lds, s, a, tpw, depth);       \
  } while (0)
  const bool wide = a.G <= 8;
  if (wide && tail && burst) SFI_FLOOR(true, true, true);
  else if (wide && tail) SFI_FLOOR(true, true, false);
  else if (wide && burst) SFI_FLOOR(true, false, true);
  else if (wide) SFI_FLOOR(true, false, false);
  else if (tail && burst) SFI_FLOOR(false, true, true);
  else if (tail) SFI_FLOOR(false, true, false);
  else if (burst) SFI_FLOOR(false, false, true);
  else SFI_FLOOR(false, false, false);
#undef SFI_FLOOR
  return hipGetLastError();
}

// ------------------------------------------------------------------------------------------------
// Memory skeleton of the dense kernel -- a measurement aid, not part of the path: the dense launch's grid and
// tile dealing (tiles first, first + step, ... of the prefix per wave, two tile buffers in flight, K half and V
// half of a buffer refilled separately; tile t starts at row n_sink + 32 t as the kernel's tiles of J do), nontemporal
// 16-byte loads, nothing computed: what arrives is folded
// into one word per wave.  WIDE: K rows requested as whole 128-byte lines (the gather kernels' layout) instead
// of the four 64-byte pieces the dense kernel's operand layout asks for.  No logits are written.
// The eight loads of a half go out back to back, as the kernel issues them (left to itself the compiler refills
// register by register as the fold frees them, and that order of requests is 10 % slower).  idle_units > 0: the wave
// sleeps idle_units x 64 cycles where the kernel has its two blocks of arithmetic (after the K half and after the V
// half of every tile), to show what time between the waits costs when the memory side is the same.
// writer > 0: the workgroup has a fifth wave that does nothing but store what the kernel would expose (G x 128 bytes
// per tile, the kernel's addresses; writer == 2: always the same 2 KB of them), at about the readers' pace, while the
// four waves read: what store instructions cost a compute unit that is streaming rows.
// ------------------------------------------------------------------------------------------------
__device__ __forceinline__ void idle(int units) {
  for (int i = 0; i < units; ++i) __builtin_amdgcn_s_sleep(1);
}
template <bool WIDE>
__global__ __launch_bounds__(kAttnThreads + 64, 1) void attn_dense_floor_kernel(const AttnArgs a, int idle_units, int writer) {
  const int slot = blockIdx.x, h = blockIdx.y, b = blockIdx.z;
  const int tid = threadIdx.x;
  const int lane = tid & 63, w = tid >> 6;
  const int jg = lane >> 4, n = lane & 15;
  if (w == kWaves) {  // the writer wave (only launched with writer > 0)
    int bad0 = 0;
    const int L0 = guarded_len(a.ctx_len[b * a.ms], a.len_cap, bad0);
    const int nT0 = (L0 + kTile - 1) / kTile;
    const int step0 = a.n_split * kWaves;
    float* lg = a.logits + (int64_t)(b * a.Hkv + h) * a.G * a.ld_pos;
    const int tile_floats = a.G * kTile;
    const int k_max = slot * kWaves < nT0 ? (nT0 - slot * kWaves + step0 - 1) / step0 : 0;
    for (int k = 0; k < k_max; ++k) {
      __builtin_amdgcn_s_sleep(90);  // 5760 cycles: a little less than the four waves take per tile
      for (int ww = 0; ww < kWaves; ++ww) {
        const int t = slot * kWaves + ww + k * step0;
        if (t < a.max_tiles && lane * 4 < tile_floats)
          *reinterpret_cast<float4*>(lg + (int64_t)(writer == 2 ? ww : t) * tile_floats + lane * 4) = make_float4((float)lane, 0.f, 0.f, 0.f);
      }
    }
    return;
  }
  Rows R;
  R.Kb = reinterpret_cast<const char*>(a.K + b * a.k_sb + h * a.k_sh);
  R.Vb = reinterpret_cast<const char*>(a.V + b * a.v_sb + h * a.v_sh);
  R.k_st = (uint32_t)a.k_st * 2u;
  R.v_st = (uint32_t)a.v_st * 2u;
  R.k_lane = k_lane_of<WIDE>(jg, n);
  R.v_lane = n * 16;
  R.jg = jg;
  R.n = n;
  const int first = slot * kWaves + w, step = a.n_split * kWaves;
  Tile T, T2;
  issue_affine<WIDE>(T, R, a.n_sink + first * kTile, a.row_cap);  // before ctx_len arrives, as the kernel does
  issue_affine<WIDE>(T2, R, a.n_sink + (first + step) * kTile, a.row_cap);
  int bad = 0;
  const int L = guarded_len(a.ctx_len[b * a.ms], a.len_cap, bad);
  const int r_last = max(L, 1) - 1;
  const int nT = (L + kTile - 1) / kTile;
  const int K = first < nT ? (nT - first + step - 1) / step : 0;
  uint32_t fold = 0u;
  auto use = [&](Tile& B, int k) {
    const int t_next = first + (k + 2) * step;
#pragma unroll
    for (int i = 0; i < 4; ++i) fold ^= fold16(B.ka[i]) ^ fold16(B.kb[i]);
    __builtin_amdgcn_sched_barrier(0);
    idle(idle_units);
    __builtin_amdgcn_sched_barrier(0);
    issue_k_affine<WIDE>(B, R, a.n_sink + t_next * kTile, r_last);
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int i = 0; i < 8; ++i) fold ^= fold16(B.v[i]);
    __builtin_amdgcn_sched_barrier(0);
    idle(idle_units);
    __builtin_amdgcn_sched_barrier(0);
    issue_v_affine<WIDE>(B, R, a.n_sink + t_next * kTile, r_last);
    __builtin_amdgcn_sched_barrier(0);
  };
  int k = 0;
  for (; k + 1 < K; k += 2) {
    use(T, k);
    use(T2, k + 1);
  }
  if (k < K) use(T, k);
#pragma unroll
  for (int i = 0; i < 4; ++i) fold ^= fold16(T.ka[i]) ^ fold16(T.kb[i]) ^ fold16(T2.ka[i]) ^ fold16(T2.kb[i]);  // the refills past the end
#pragma unroll
  for (int i = 0; i < 8; ++i) fold ^= fold16(T.v[i]) ^ fold16(T2.v[i]);
#pragma unroll
  for (int d = 32; d >= 1; d >>= 1) fold ^= __shfl_xor(fold, d);
  const int64_t head0 = (int64_t)b * a.Hq + h * a.G;
  if (lane == 0) reinterpret_cast<uint32_t*>(a.part)[((head0 * kSlotCap + slot) * kPartStride) + w] = fold;
}
hipError_t launch_attn_dense_floor(const AttnArgs& a, int B, int n_slots, int wide, int idle_units, int writer, hipStream_t s) {
  const dim3 grid(n_slots, a.Hkv, B);
  const dim3 block(writer != 0 ? kAttnThreads + 64 : kAttnThreads);
  if (wide) hipLaunchKernelGGL(attn_dense_floor_kernel<true>, grid, block, 0, s, a, idle_units, writer);
  else hipLaunchKernelGGL(attn_dense_floor_kernel<false>, grid, block, 0, s, a, idle_units, writer);
  return hipGetLastError();
}

// ------------------------------------------------------------------------------------------------
// compact kernel: the fast step over the two-segment layout (Sec. "Memory-coalesced Kernel Design
// and Selector Maintenance"): sink ++ selected rows from the compact buffers the Reorg kernel filled,
// the recent window in place from the cache.  Both segments are runs of consecutive rows, so no
// index is read: a wave's first tile is on its way before any scalar of the step has arrived.
// Tiles never straddle the two segments: the compact segment ends with a ragged tile of its own.
// ------------------------------------------------------------------------------------------------
template <bool PAGED, bool WIDE>  // PAGED: the recent window is read from a paged cache (the compact buffers are always flat)
__global__ __launch_bounds__(kAttnThreads, PAGED ? 2 : 3) void attn_compact_kernel(const AttnArgs a) {
  const int slot = blockIdx.x, h = blockIdx.y, b = blockIdx.z;
  if (a.is_slow != nullptr && a.is_slow[b * a.fs] != 0) return;
  const int tid = threadIdx.x;
  const int lane = tid & 63, w = tid >> 6;
  const int jg = lane >> 4, n = lane & 15;
  const int G = a.G;
  const int bh = b * a.Hkv + h;
  const int64_t head0 = (int64_t)b * a.Hq + h * G;
  const int first = slot * kWaves + w, step = a.n_split * kWaves;

  Rows Rc;  // compact segment
  Rc.Kb = reinterpret_cast<const char*>(a.Kc + b * a.c_sb + h * a.c_sh);
  Rc.Vb = reinterpret_cast<const char*>(a.Vc + b * a.c_sb + h * a.c_sh);
  Rc.k_st = Rc.v_st = kHeadDim * 2u;
  Rc.k_lane = k_lane_of<WIDE>(jg, n);
  Rc.v_lane = n * 16;
  Rc.jg = jg;
  Rc.n = n;
  Rows R = Rc;  // recent segment, in the cache
  R.Kb = reinterpret_cast<const char*>(a.K + b * a.k_sb + h * a.k_sh);
  R.Vb = reinterpret_cast<const char*>(a.V + b * a.v_sb + h * a.v_sh);
  R.k_st = (uint32_t)a.k_st * 2u;
  R.v_st = (uint32_t)a.v_st * 2u;

  Tile T;
  const bool spec = first * kTile < a.c_rows;  // almost every wave's tile lies in the compact segment
  if (spec) issue_affine<WIDE>(T, Rc, first * kTile, a.c_rows - 1);
  bf16x8 qreg[4];
  load_q<WIDE>(qreg, a.q, head0, G, jg, n);
  int bad = 0;
  const int L_in = a.ctx_len[b * a.ms], nSel0 = a.n_sel[bh], rs_in = a.recent_start[b * a.ms];  // one round trip for the three
  const int L = guarded_len(L_in, a.len_cap, bad);
  const int nSel = min(max(nSel0, 0), (int)a.sel_stride);
  bad |= nSel != nSel0 ? kGuardNSel : 0;
  const int nS = min(a.n_sink, L);
  // A context that still lies inside the sink range has nothing selected, and the rows appended since
  // the reorganisation are sink rows the compact buffers do not hold: all of it is read in place.
  const bool all_sink = L <= a.n_sink;
  const int rs = all_sink ? 0 : min(max(rs_in, nS), L);
  const int Nc = all_sink ? 0 : a.n_sink + nSel;  // compact rows in use
  const int Tc = (Nc + kTile - 1) / kTile;
  const int Nr = L - rs;
  const int nT = Tc + (Nr + kTile - 1) / kTile;

  float m_run = kNeg, l_run = 0.f;
  f32x4 acc[8];
#pragma unroll
  for (int e = 0; e < 8; ++e) acc[e] = f32x4{0.f, 0.f, 0.f, 0.f};

  // Tile t < Tc is rows 32 t .. of the compact segment, tile t >= Tc rows rs + 32 (t - Tc) .. of the cache
  // (clamped to L - 1, which is also what the refill past the wave's last tile reads).  The branch is
  // wave-uniform and both sides issue the same number of loads.
  int pra_n = 0, prb_n = 0;  // PAGED: physical rows of the recent tile whose K half was issued last
  auto issue_k_tile = [&](int t) {
    if (t < Tc) {
      issue_k_affine<WIDE>(T, Rc, t * kTile, a.c_rows - 1);
    } else if (PAGED) {
      const Pages P = pages_of(a, b, L);
      const int ra = min(rs + (t - Tc) * kTile + n, L - 1), rb = min(rs + (t - Tc) * kTile + 16 + n, L - 1);
      pra_n = P.phys(ra, P.page_of(ra), bad);
      prb_n = P.phys(rb, P.page_of(rb), bad);
      issue_k_rows<uint64_t, WIDE>(T, R, pra_n, prb_n);
    } else {
      issue_k_affine<WIDE>(T, R, rs + (t - Tc) * kTile, L - 1);
    }
  };
  auto issue_v_tile = [&](int t) {
    if (t < Tc) issue_v_affine<WIDE>(T, Rc, t * kTile, a.c_rows - 1);
    else if (PAGED) issue_v_rows<uint64_t, WIDE>(T, R, pra_n, prb_n);
    else issue_v_affine<WIDE>(T, R, rs + (t - Tc) * kTile, L - 1);
  };
  const int K = first < nT ? (nT - first + step - 1) / step : 0;
  if (K > 0 && !(spec && first < Tc)) {  // the first tile is not the compact tile requested up front
    issue_k_tile(first);
    issue_v_tile(first);
  }
  // the dense kernel's loop: K half refilled after S^T, V half after P V
  for (int k = 0; k < K; ++k) {
    const int t = first + k * step;
    const int p0 = (t < Tc ? t : t - Tc) * kTile;
    const int N = t < Tc ? Nc : Nr;
    float y[8];
    qk_phase<WIDE>(T, qreg, a.scale_log2, y);
    issue_k_tile(t + step);
    if (p0 + kTile > N) mask_tail<true, WIDE>(T, y, jg, p0, N);
    bf16x8 a_hi, a_lo;
    softmax_phase(y, acc, m_run, l_run, jg, a_hi, a_lo);
    pv_phase(T, a_hi, a_lo, acc);
    issue_v_tile(t + step);
  }
  l_run += __shfl_xor(l_run, 16);
  l_run += __shfl_xor(l_run, 32);
  write_wg_record(wg_out_of(a, bh), head0, G, slot, acc, m_run, l_run);
  report_guard(a.guard, bad);
}

// ------------------------------------------------------------------------------------------------
// Reorg (Sec. "Hiding Slow-step Overhead via Layer-wise Asynchronous Execution": Reorg_i): compact row
// i < n_sink is cache row i, compact row n_sink + i is cache row sel_idx[i], i < n_sel.  A workgroup
// moves kReorgRows compact rows of one (b, h), 16 lanes x 16 bytes per row, K and V; the indices
// are read before the list length is known, and all of a thread's row loads precede its stores.
// ------------------------------------------------------------------------------------------------
template <bool PAGED>
__global__ __launch_bounds__(kAttnThreads) void reorg_kernel(const ReorgArgs a) {
  const int chunk = blockIdx.x, h = blockIdx.y, b = blockIdx.z;
  if (a.is_slow != nullptr && a.is_slow[b * a.fs] == 0) return;
  const int bh = b * a.Hkv + h;
  const int tid = threadIdx.x;
  const int sub = tid & 15, r = tid >> 4;
  constexpr int kPass = kReorgRows / 16;
  const int32_t* sel = a.sel_idx + (int64_t)bh * a.sel_stride;
  const int sel_cap = (int)a.sel_stride - 1;
  int src[kPass];
#pragma unroll
  for (int p = 0; p < kPass; ++p) {
    const int i = chunk * kReorgRows + p * 16 + r;
    src[p] = sel_cap >= 0 ? sel[min(max(i - a.n_sink, 0), sel_cap)] : 0;
  }
  int bad = 0;
  const int L_in = a.ctx_len[b * a.ms], nSel0 = a.n_sel[bh];
  const int L = guarded_len(L_in, a.len_cap, bad);
  const int nSel = min(max(nSel0, 0), (int)a.sel_stride);
  bad |= nSel != nSel0 ? kGuardNSel : 0;
  const int nS = min(a.n_sink, L);
  const int r_hi = max(L, 1) - 1;
  const char* Kb = reinterpret_cast<const char*>(a.K + b * a.k_sb + h * a.k_sh);
  const char* Vb = reinterpret_cast<const char*>(a.V + b * a.v_sb + h * a.v_sh);
  char* Kc = reinterpret_cast<char*>(a.Kc + b * a.c_sb + h * a.c_sh);
  char* Vc = reinterpret_cast<char*>(a.Vc + b * a.c_sb + h * a.c_sh);
  uint4 kr[kPass], vr[kPass];
  bool ok[kPass];
#pragma unroll
  for (int p = 0; p < kPass; ++p) {
    const int i = chunk * kReorgRows + p * 16 + r;
    ok[p] = i < nS || (i >= a.n_sink && i < a.n_sink + nSel);
    int row = i < a.n_sink ? i : src[p];
    if (ok[p]) {  // a stored index outside the context reads as the context's last row (as in the gather kernels)
      const int rc = (int)min((uint32_t)row, (uint32_t)r_hi);
      bad |= rc != row ? kGuardSelIdx : 0;
      row = rc;
    }
    if (PAGED && ok[p]) {
      const int32_t* tbl = a.table + (int64_t)b * a.table_stride;
      const int page = tbl[row >> a.page_lg];
      const int pc = min(max(page, 0), a.n_blocks - 1);
      bad |= pc != page ? kGuardBlock : 0;
      row = pc * a.page_rpb + (row & ((1 << a.page_lg) - 1));
    }
    if (ok[p]) {
      typedef typename RowOff<PAGED>::type OffT;
      kr[p] = load_row16(Kb, (OffT)((OffT)(uint32_t)row * ((uint32_t)a.k_st * 2u) + sub * 16));
      vr[p] = load_row16(Vb, (OffT)((OffT)(uint32_t)row * ((uint32_t)a.v_st * 2u) + sub * 16));
    }
  }
#pragma unroll
  for (int p = 0; p < kPass; ++p) {
    const int i = chunk * kReorgRows + p * 16 + r;
    if (ok[p]) {
      *reinterpret_cast<uint4*>(Kc + (int64_t)i * (kHeadDim * 2) + sub * 16) = kr[p];
      *reinterpret_cast<uint4*>(Vc + (int64_t)i * (kHeadDim * 2) + sub * 16) = vr[p];
    }
  }
  report_guard(a.guard, bad);
}

// Stand-alone merge: one workgroup per (sequence, query head).
__global__ __launch_bounds__(kMergeThreads) void merge_kernel(const MergeArgs a) {
  const int bg = blockIdx.x;
  const int b = bg / a.Hq;
  int n_slots;
  if (a.mode == 2 && a.slots_fast == 0 && a.is_slow[b * a.fs] == 0) return;  // fast sequences wrote their output themselves
  if (a.mode == 0) n_slots = a.slots_slow;
  else if (a.mode == 1) n_slots = a.slots_fast;
  else n_slots = a.is_slow[b * a.fs] ? a.slots_slow : a.slots_fast;
  const bool dense = a.mode == 0 || (a.mode == 2 && a.is_slow[b * a.fs]);
  if (dense) {
    // dense records: slots_slow waves' J records, then one record per wave that owned sink / recent tiles
    int L, recent;
    window_view(a.q_len, b, min(max(a.ctx_len[b * a.ms], 0), a.len_cap), a.recent, L, recent);  // the dense launch's view
    const int nS = min(a.n_sink, L);
    const int rs = min(max(a.n_sink, L - recent), L);
    const int nTS = (nS + (L - rs) + kTile - 1) / kTile;
    n_slots = a.slots_slow + min(a.slots_slow, nTS);
  }
  merge_records(a.part, a.out, bg, n_slots, dense ? a.jstat : nullptr, a.n_j, a.G, a.alpha, a.out_bf16 != 0);
}

__global__ void advance_kernel(int32_t* ctx_len, int32_t* recent_start, int B, int n_sink, int recent) {
  const int b = blockIdx.x * blockDim.x + threadIdx.x;
  if (b < B) {
    const int L = ctx_len[b] + 1;
    ctx_len[b] = L;
    recent_start[b] = max(n_sink, L - recent);
  }
}

__global__ void trigger_kernel(const int32_t* last_token, const uint32_t* bitmap, int vocab, int t_max, int32_t* since_slow,
                               uint8_t* is_slow, int B) {
  const int b = blockIdx.x * blockDim.x + threadIdx.x;
  if (b < B) {
    const int tok = last_token[b];
    const int c = since_slow[b];
    const bool hit = tok >= 0 && tok < vocab && ((bitmap[tok >> 5] >> (tok & 31)) & 1u) != 0u;
    const bool slow = hit || c >= t_max;
    is_slow[b] = slow ? 1 : 0;
    since_slow[b] = slow ? 0 : c + 1;
  }
}

// The packed per-step descriptor (Sec. "Memory-coalesced Kernel Design and Selector Maintenance": built once per
// decoding step, read by every kernel of the step): state update and trigger decision of every sequence in one launch.
__global__ void step_begin_kernel(sfi_step_desc* desc, const int32_t* last_token, const uint32_t* bitmap, int vocab, int t_max,
                                  int advance, int B, int n_sink, int recent) {
  const int b = blockIdx.x * blockDim.x + threadIdx.x;
  if (b < B) {
    sfi_step_desc d = desc[b];
    if (advance) d.ctx_len += 1;
    d.recent_start = max(n_sink, d.ctx_len - recent);
    const int tok = last_token != nullptr ? last_token[b] : -1;
    const bool hit = bitmap != nullptr && tok >= 0 && tok < vocab && ((bitmap[tok >> 5] >> (tok & 31)) & 1u) != 0u;
    const bool slow = hit || d.since_slow >= t_max;
    d.is_slow = slow ? 1 : 0;
    d.since_slow = slow ? 0 : d.since_slow + 1;
    desc[b] = d;
  }
}
hipError_t launch_step_begin(sfi_step_desc* desc, const int32_t* last_token, const uint32_t* bitmap, int vocab, int t_max,
                             int advance, int B, int n_sink, int recent, hipStream_t s) {
  hipLaunchKernelGGL(step_begin_kernel, dim3((B + 63) / 64), dim3(64), 0, s, desc, last_token, bitmap, vocab, t_max, advance, B,
                     n_sink, recent);
  return hipGetLastError();
}

hipError_t launch_trigger(const int32_t* last_token, const uint32_t* bitmap, int vocab, int t_max, int32_t* since_slow,
                          uint8_t* is_slow, int B, hipStream_t s) {
  hipLaunchKernelGGL(trigger_kernel, dim3((B + 63) / 64), dim3(64), 0, s, last_token, bitmap, vocab, t_max, since_slow,
                     is_slow, B);
  return hipGetLastError();
}

template <bool PAGED>
static void launch_dense_t(const AttnArgs& a, dim3 grid, hipStream_t s) {
  if (a.item_batch > 0) {  // ragged step (logits always exposed, never the big stash, never evidence-only)
    if (a.with_knorm) hipLaunchKernelGGL((attn_dense_items_kernel<2, PAGED>), grid, dim3(kAttnThreads), 0, s, a);
    else hipLaunchKernelGGL((attn_dense_items_kernel<1, PAGED>), grid, dim3(kAttnThreads), 0, s, a);
    return;
  }
  if constexpr (!PAGED) {
    if (a.dense_wide && a.G <= 8 && !a.with_knorm && !a.no_v) {
      if (a.logits != nullptr && a.big_stash) hipLaunchKernelGGL((attn_dense_kernel<1, false, true, false, true>), grid, dim3(kAttnThreads), 0, s, a);
      else if (a.logits != nullptr) hipLaunchKernelGGL((attn_dense_kernel<1, false, false, false, true>), grid, dim3(kAttnThreads), 0, s, a);
      else hipLaunchKernelGGL((attn_dense_kernel<0, false, false, false, true>), grid, dim3(kAttnThreads), 0, s, a);
      return;
    }
  }
  if (a.logits != nullptr && a.no_v && a.with_knorm)  // evidence only (always with the big stash)
    hipLaunchKernelGGL((attn_dense_kernel<2, PAGED, true, true>), grid, dim3(kAttnThreads), 0, s, a);
  else if (a.logits != nullptr && a.no_v)
    hipLaunchKernelGGL((attn_dense_kernel<1, PAGED, true, true>), grid, dim3(kAttnThreads), 0, s, a);
  else if (a.logits != nullptr && a.with_knorm && a.big_stash)
    hipLaunchKernelGGL((attn_dense_kernel<2, PAGED, true>), grid, dim3(kAttnThreads), 0, s, a);
  else if (a.logits != nullptr && a.with_knorm)
    hipLaunchKernelGGL((attn_dense_kernel<2, PAGED>), grid, dim3(kAttnThreads), 0, s, a);
  else if (a.logits != nullptr && a.big_stash)
    hipLaunchKernelGGL((attn_dense_kernel<1, PAGED, true>), grid, dim3(kAttnThreads), 0, s, a);
  else if (a.logits != nullptr)
    hipLaunchKernelGGL((attn_dense_kernel<1, PAGED>), grid, dim3(kAttnThreads), 0, s, a);
  else
    hipLaunchKernelGGL((attn_dense_kernel<0, PAGED>), grid, dim3(kAttnThreads), 0, s, a);
}
hipError_t launch_attn_dense(const AttnArgs& a, int B, int n_slots, hipStream_t s) {
  // ragged step: a fixed number of workgroups (no more than there are cells)
  const dim3 grid = a.item_batch > 0 ? dim3((unsigned)min((int64_t)n_slots * a.Hkv * B, (int64_t)a.item_wgs)) : dim3(n_slots, a.Hkv, B);
  if (a.table != nullptr) launch_dense_t<true>(a, grid, s);
  else launch_dense_t<false>(a, grid, s);
  return hipGetLastError();
}
hipError_t launch_attn_compact(const AttnArgs& a, int B, int n_slots, hipStream_t s) {
  const dim3 grid(n_slots, a.Hkv, B);
  if (a.G <= 8) {
    if (a.table != nullptr) hipLaunchKernelGGL((attn_compact_kernel<true, true>), grid, dim3(kAttnThreads), 0, s, a);
    else hipLaunchKernelGGL((attn_compact_kernel<false, true>), grid, dim3(kAttnThreads), 0, s, a);
  } else {
    if (a.table != nullptr) hipLaunchKernelGGL((attn_compact_kernel<true, false>), grid, dim3(kAttnThreads), 0, s, a);
    else hipLaunchKernelGGL((attn_compact_kernel<false, false>), grid, dim3(kAttnThreads), 0, s, a);
  }
  return hipGetLastError();
}
hipError_t launch_reorg(const ReorgArgs& a, int B, int rows, hipStream_t s) {
  const dim3 grid((rows + kReorgRows - 1) / kReorgRows, a.Hkv, B);
  if (a.table != nullptr) hipLaunchKernelGGL(reorg_kernel<true>, grid, dim3(kAttnThreads), 0, s, a);
  else hipLaunchKernelGGL(reorg_kernel<false>, grid, dim3(kAttnThreads), 0, s, a);
  return hipGetLastError();
}
template <bool WIDE>
static void launch_gather_t(const AttnArgs& a, dim3 grid, hipStream_t s) {
  if (a.pipelined) {
    if (a.table != nullptr) hipLaunchKernelGGL((attn_gather_stream_kernel<true, WIDE>), grid, dim3(kAttnThreads), 0, s, a);
    else hipLaunchKernelGGL((attn_gather_stream_kernel<false, WIDE>), grid, dim3(kAttnThreads), 0, s, a);
    return;
  }
  if (a.table != nullptr) hipLaunchKernelGGL((attn_gather_kernel<true, WIDE>), grid, dim3(kAttnThreads), 0, s, a);
  else hipLaunchKernelGGL((attn_gather_kernel<false, WIDE>), grid, dim3(kAttnThreads), 0, s, a);
}
hipError_t launch_attn_gather(const AttnArgs& a, int B, int n_slots, hipStream_t s) {
  const dim3 grid(n_slots, a.Hkv, B);
  if (a.G <= 8) launch_gather_t<true>(a, grid, s);
  else launch_gather_t<false>(a, grid, s);
  return hipGetLastError();
}
hipError_t launch_merge(const MergeArgs& a, int B, hipStream_t s) {
  hipLaunchKernelGGL(merge_kernel, dim3(B * a.Hq), dim3(kMergeThreads), 0, s, a);
  return hipGetLastError();
}
hipError_t launch_advance(int32_t* ctx_len, int32_t* recent_start, int B, int n_sink, int recent, hipStream_t s) {
  hipLaunchKernelGGL(advance_kernel, dim3((B + 63) / 64), dim3(64), 0, s, ctx_len, recent_start, B, n_sink, recent);
  return hipGetLastError();
}

}  // namespace sfi
