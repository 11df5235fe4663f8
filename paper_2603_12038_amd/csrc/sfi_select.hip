// Selector on the GPU (paper Algorithm 2) for gfx950.
//
// Per (sequence b, KV head h), over the allowed set J (Eq. allowed_set), positions p = j - n_sink:
//   p_g(j) = softmax over J of the logits of query head g          (Eq. selector_pt); the dense
//            kernel left y = log2(e) * logit, so e^{l - M} is 2^{y - M_y}
//   mu(j)  = (1/G) sum_g p_g(j)^alpha, f = mu^(1/alpha) / sum      (Eqs. selector_mu, selector_f; the G
//            heads of the group are the observation window; alpha = 1: f is the mean of the p_g)
// Mode 0 ranks by f alone: z = log(f + eps) is monotone in mu, so the Top-K of Eq. topk_out is taken
// on mu itself.  Mode 1 goes through the prior, the reverse-KL fusion with lambda*, Soft-NMS and the
// cross-head exclusivity first (three kernels further down) and ranks by e^z_adj.
// Top-K is a radix select on the fp32 bit pattern of the ranking value (positive floats order like
// unsigned integers): a 12-bit histogram over all of J (stage 1, with the scoring), the keys of the
// threshold bin collected with the segment they came from (stage 2), and, in one launch (stage 3), an
// exact 19-bit refinement among those few keys followed by an index-ordered compaction that takes every
// key above the threshold and the lowest-index keys equal to it.  Integer atomics only count, so the result
// does not depend on scheduling.
#include "sfi_internal.h"
#include "sfi_merge.h"

namespace sfi {

__device__ __forceinline__ float fast_exp2s(float x) { return __builtin_amdgcn_exp2f(x); }

// Exclusive prefix sum of one value per thread over a 256-thread block; returns the exclusive
// prefix and leaves the block total in *total.  scratch: 8 words of LDS.
__device__ __forceinline__ uint32_t block_excl_scan(uint32_t v, uint32_t* scratch, uint32_t* total) {
  const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
  uint32_t inc = v;
#pragma unroll
  for (int d = 1; d < 64; d <<= 1) {
    const uint32_t t = __shfl_up(inc, d);
    if (lane >= d) inc += t;
  }
  __syncthreads();  // scratch may still be read from a previous call
  if (lane == 63) scratch[w] = inc;
  __syncthreads();
  uint32_t base = 0, tot = 0;
#pragma unroll
  for (int i = 0; i < kSelThreads / 64; ++i) {
    const uint32_t s = scratch[i];
    if (i < w) base += s;
    tot += s;
  }
  *total = tot;
  return base + inc - v;
}

// Finds, scanning bins from the highest down, the bin holding the k-th largest key (1-based k,
// k <= total count).  Writes res[0] = bin, res[1] = how many keys of that bin are still needed.
// hist may live in LDS or global memory; nbins is a multiple of 256.
__device__ __forceinline__ void find_kth_desc(const uint32_t* hist, int nbins, uint32_t k, uint32_t* res,
                                              uint32_t* scratch) {
  const int per = nbins / kSelThreads;
  const int hi = nbins - (int)threadIdx.x * per;  // exclusive upper bin of this thread
  if (threadIdx.x == 0) res[0] = res[1] = 0u;      // defined result even if k exceeds the total
  uint32_t c = 0;
  for (int i = 1; i <= per; ++i) c += hist[hi - i];
  uint32_t total;
  const uint32_t above = block_excl_scan(c, scratch, &total);
  if (above < k && k <= above + c) {
    uint32_t cum = above;
    for (int i = 1; i <= per; ++i) {
      const uint32_t hv = hist[hi - i];
      if (cum + hv >= k) {
        res[0] = (uint32_t)(hi - i);
        res[1] = k - cum;
        break;
      }
      cum += hv;
    }
  }
  __syncthreads();
}

// The same with the thread's bins already in registers: hv[i] is bin (nbins - tid * N) - 1 - i.
template <int N>
__device__ __forceinline__ void find_kth_desc_regs(const uint32_t (&hv)[N], int nbins, uint32_t k, uint32_t* res,
                                                   uint32_t* scratch) {
  const int hi = nbins - (int)threadIdx.x * N;
  if (threadIdx.x == 0) res[0] = res[1] = 0u;
  uint32_t c = 0;
#pragma unroll
  for (int i = 0; i < N; ++i) c += hv[i];
  uint32_t total;
  const uint32_t above = block_excl_scan(c, scratch, &total);
  if (above < k && k <= above + c) {
    uint32_t cum = above;
    bool found = false;
#pragma unroll
    for (int i = 0; i < N; ++i) {
      if (!found && cum + hv[i] >= k) {
        res[0] = (uint32_t)(hi - 1 - i);
        res[1] = k - cum;
        found = true;
      }
      cum += hv[i];
    }
  }
  __syncthreads();
}

struct Problem {
  int nJ;        // |J|
  uint32_t ksel; // min(budget, |J|)
};

__device__ __forceinline__ Problem problem_of(const SelArgs& a, int b) {
  Problem p;
  p.nJ = max(0, min(a.ctx_len[b * a.ms], a.len_cap) - a.recent - a.n_sink);  // the dense launch's clamp of ctx_len
  p.ksel = (uint32_t)min(a.budget, p.nJ);
  return p;
}

// The slow step without a merge launch (SelArgs::part != nullptr).  The launch that reads the exposed
// logits first carries G extra workgroups per (b, h); each merges the dense kernel's records of one
// query head into the attention output (J records of all waves, then one record per wave that owned
// sink / recent tiles).
// J records per query head of sequence b: one per wave of the dense launch's workgroups of that sequence (the ragged
// step's dense launch chooses the splits per sequence on the device and leaves them in the workspace)
__device__ __forceinline__ int n_jrec_of(const SelArgs& a, int b) {
  return a.seq_splits != nullptr ? a.seq_splits[b] * kWaves : a.n_jrec;
}
__device__ __forceinline__ void merge_head(const SelArgs& a, int b, int h, int g) {
  const int n_jrec = n_jrec_of(a, b);
  const int L = min(max(a.ctx_len[b * a.ms], 0), a.len_cap);
  const int nS = min(a.n_sink, L);
  const int rs = min(max(a.n_sink, L - a.recent), L);
  const int nTS = (nS + (L - rs) + 31) / 32;
  const int n_slots = n_jrec + min(n_jrec, nTS);
  merge_records(a.part, a.merge_out, b * a.Hq + h * a.G + g, n_slots, nullptr, 0, a.G, a.alpha, a.out_bf16 != 0);
}

// ... and every other workgroup takes the J-only softmax statistics of the group's heads from the
// headers of the J records itself: one wave per head, a lane takes records lane, lane + 64, ... (at
// most kSlotCap = 256).  sM[g] = max of y over J, sc[g] = Z^(-alpha) / G; valid after the next barrier.
__device__ __forceinline__ void group_jstat(const SelArgs& a, int b, int h, float* sM, float* sc) {
  const int lane = threadIdx.x & 63;
  const int n_jrec = n_jrec_of(a, b);
  for (int g = threadIdx.x >> 6; g < a.G; g += kSelThreads / 64) {
    const float* P = a.part + (int64_t)(b * a.Hq + h * a.G + g) * kSlotCap * kPartStride;
    float2 ml[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int sl = lane + 64 * i;
      ml[i] = sl < n_jrec ? *reinterpret_cast<const float2*>(P + (int64_t)sl * kPartStride) : make_float2(kNeg, 0.f);
    }
    float M = fmaxf(fmaxf(ml[0].x, ml[1].x), fmaxf(ml[2].x, ml[3].x));
#pragma unroll
    for (int d = 32; d >= 1; d >>= 1) M = fmaxf(M, __shfl_xor(M, d));
    float Z = 0.f;
#pragma unroll
    for (int i = 0; i < 4; ++i) Z += ml[i].y * fast_exp2s(ml[i].x - M);
#pragma unroll
    for (int d = 32; d >= 1; d >>= 1) Z += __shfl_xor(Z, d);
    if (lane == 0) {
      const float zpow = a.alpha == 1.0f ? Z : fast_exp2s(a.alpha * __builtin_amdgcn_logf(Z));
      sM[g] = M;
      sc[g] = 1.0f / ((float)a.G * zpow);
    }
  }
}

// ---- stage 1: evidence f, its key, and the 12-bit histogram ------------------------------------
// ACCUM: windowed evidence (Eq. selector_mu over several queries): instead of ranking, add this
// query's head-mean to the accumulator mu (or start it, a.accum_first); sel_finalize_kernel ranks later.
template <bool ACCUM>
__global__ __launch_bounds__(kSelThreads) void sel_score_kernel(const SelArgs a) {
  const int seg = blockIdx.x, h = blockIdx.y, b = blockIdx.z;
  if (a.is_slow != nullptr && a.is_slow[b * a.fs] == 0) return;
  Problem pb = problem_of(a, b);
  int n_all = pb.nJ;  // ACCUM under the causal mask: |J| of the whole window; pb.nJ becomes the part this query sees
  if (ACCUM && a.q_len != nullptr) {
    int Lq, rec;
    window_view(a.q_len, b, min(max(a.ctx_len[b * a.ms], 0), a.len_cap), a.recent, Lq, rec);
    pb.nJ = max(0, Lq - rec - a.n_sink);
  }
  const int tid = threadIdx.x;
  const int bh = b * a.Hkv + h;
  const int G = a.G;
  const bool fused = !ACCUM && a.part != nullptr;  // grid-uniform
  if (fused && seg >= (int)gridDim.x - G) {
    merge_head(a, b, h, seg - ((int)gridDim.x - G));
    return;
  }
  const int p_lo = seg * kSelSeg;
  if (ACCUM && a.accum_first && n_all > pb.nJ) {  // the first query of a window starts the accumulator: zero where it sees nothing
    float* mu0 = a.mu + (int64_t)bh * a.ld_pos;
    // (from the next whole quad on: the quad that straddles the edge is written by the thread that owns it)
    for (int p = max(p_lo, (pb.nJ + 3) & ~3) + tid; p < min(p_lo + kSelSeg, n_all); p += kSelThreads) mu0[p] = 0.f;
  }
  if (p_lo >= pb.nJ) return;

  __shared__ float s_jM[16], s_jc[16];
  if (fused) group_jstat(a, b, h, s_jM, s_jc);

  __shared__ uint32_t s_hist[kHist1Bins];
  for (int i = tid; i < kHist1Bins; i += kSelThreads) s_hist[i] = 0u;

  // logits of (b, h): tile-major, [tile of 32 positions][G heads][32].  A thread owns two quads of
  // positions, half a segment apart; for G <= 8 all its loads are issued before any is used.
  const int rows = a.lg_rows;  // G, or G + 1 when the dense kernel also exposed the key norms
  const float* lg = a.logits + (int64_t)bh * rows * a.ld_pos;
  uint32_t* keys = a.keys + (int64_t)bh * a.ld_pos;
  constexpr int kHalf = kSelSeg / 2;
  const int pq[2] = {p_lo + tid * 4, p_lo + kHalf + tid * 4};
  float4 lq[2][8];
  if (G <= 8) {
#pragma unroll
    for (int r = 0; r < 2; ++r)
#pragma unroll
      for (int g = 0; g < 8; ++g)
        lq[r][g] = (pq[r] < pb.nJ && g < G)
                       ? *reinterpret_cast<const float4*>(lg + (int64_t)(pq[r] >> 5) * rows * kTile + g * kTile + (pq[r] & 31))
                       : make_float4(0.f, 0.f, 0.f, 0.f);
  }
  // J-only softmax statistics of the heads of this group, left by the merge kernel:
  // f(j) = sum_g c_g 2^(y_g(j) - M_g) with (M_g, c_g) = jstat[head g]
  const float al = a.alpha;  // mu(j) = sum_g sc[g] 2^(alpha (y_g(j) - sM[g]))  (Eq. selector_mu)
  float sM[16], sc[16];
  if (!fused) {
#pragma unroll
    for (int g = 0; g < 16; ++g) {
      const float2 t = g < G ? a.jstat[b * a.Hq + h * G + g] : make_float2(0.f, 0.f);
      sM[g] = t.x;
      sc[g] = t.y;
    }
  }
  __syncthreads();  // histogram cleared, statistics in place
  if (fused) {
#pragma unroll
    for (int g = 0; g < 16; ++g) {
      sM[g] = g < G ? s_jM[g] : 0.f;
      sc[g] = g < G ? s_jc[g] : 0.f;
    }
  }
#pragma unroll
  for (int r = 0; r < 2; ++r) {
    const int p = pq[r];
    if (p >= pb.nJ) continue;
    float f0 = 0.f, f1 = 0.f, f2 = 0.f, f3 = 0.f;
    if (G <= 8) {
#pragma unroll
      for (int g = 0; g < 8; ++g) {
        if (g < G) {
          f0 += sc[g] * fast_exp2s(al * (lq[r][g].x - sM[g]));
          f1 += sc[g] * fast_exp2s(al * (lq[r][g].y - sM[g]));
          f2 += sc[g] * fast_exp2s(al * (lq[r][g].z - sM[g]));
          f3 += sc[g] * fast_exp2s(al * (lq[r][g].w - sM[g]));
        }
      }
    } else {
      const float* lt = lg + (int64_t)(p >> 5) * rows * kTile + (p & 31);
#pragma unroll
      for (int g = 0; g < 16; ++g) {
        if (g < G) {
          const float4 l4 = *reinterpret_cast<const float4*>(lt + g * kTile);
          f0 += sc[g] * fast_exp2s(al * (l4.x - sM[g]));
          f1 += sc[g] * fast_exp2s(al * (l4.y - sM[g]));
          f2 += sc[g] * fast_exp2s(al * (l4.z - sM[g]));
          f3 += sc[g] * fast_exp2s(al * (l4.w - sM[g]));
        }
      }
    }
    if (ACCUM) {
      float4* mp = reinterpret_cast<float4*>(a.mu + (int64_t)bh * a.ld_pos + p);
      float4 m4 = a.accum_first ? make_float4(0.f, 0.f, 0.f, 0.f) : *mp;
      m4.x += f0;                       // positions of the quad past the part this query sees take nothing from it
      m4.y += p + 1 < pb.nJ ? f1 : 0.f;
      m4.z += p + 2 < pb.nJ ? f2 : 0.f;
      m4.w += p + 3 < pb.nJ ? f3 : 0.f;
      *mp = m4;
      continue;
    }
    const uint4 k4 = make_uint4(__float_as_uint(f0), __float_as_uint(f1), __float_as_uint(f2), __float_as_uint(f3));
    *reinterpret_cast<uint4*>(keys + p) = k4;
    atomicAdd(&s_hist[k4.x >> 19], 1u);
    if (p + 1 < pb.nJ) atomicAdd(&s_hist[k4.y >> 19], 1u);
    if (p + 2 < pb.nJ) atomicAdd(&s_hist[k4.z >> 19], 1u);
    if (p + 3 < pb.nJ) atomicAdd(&s_hist[k4.w >> 19], 1u);
  }
  if (ACCUM) return;
  __syncthreads();
  uint32_t* gh = a.hist1 + (int64_t)bh * kHist1Bins;
  for (int i = tid; i < kHist1Bins; i += kSelThreads) {
    const uint32_t c = s_hist[i];
    if (c) atomicAdd(&gh[i], c);
  }
}

// Windowed evidence, mode 0: the accumulated mu times 1 / (number of queries added) is the ranking value.
__global__ __launch_bounds__(kSelThreads) void sel_finalize_kernel(const SelArgs a) {
  const int seg = blockIdx.x, h = blockIdx.y, b = blockIdx.z;
  if (a.is_slow != nullptr && a.is_slow[b * a.fs] == 0) return;
  const Problem pb = problem_of(a, b);
  const int p_lo = seg * kSelSeg;
  if (p_lo >= pb.nJ) return;
  const int tid = threadIdx.x;
  const int bh = b * a.Hkv + h;
  __shared__ uint32_t s_hist[kHist1Bins];
  for (int i = tid; i < kHist1Bins; i += kSelThreads) s_hist[i] = 0u;
  __syncthreads();
  uint32_t* keys = a.keys + (int64_t)bh * a.ld_pos;
  const float* mu = a.mu + (int64_t)bh * a.ld_pos;
#pragma unroll
  for (int r = 0; r < 2; ++r) {
    const int p = p_lo + r * (kSelSeg / 2) + tid * 4;
    if (p >= pb.nJ) continue;
    const float4 m4 = *reinterpret_cast<const float4*>(mu + p);
    const uint4 k4 = make_uint4(__float_as_uint(m4.x * a.mu_scale), __float_as_uint(m4.y * a.mu_scale),
                                __float_as_uint(m4.z * a.mu_scale), __float_as_uint(m4.w * a.mu_scale));
    *reinterpret_cast<uint4*>(keys + p) = k4;
    atomicAdd(&s_hist[k4.x >> 19], 1u);
    if (p + 1 < pb.nJ) atomicAdd(&s_hist[k4.y >> 19], 1u);
    if (p + 2 < pb.nJ) atomicAdd(&s_hist[k4.z >> 19], 1u);
    if (p + 3 < pb.nJ) atomicAdd(&s_hist[k4.w >> 19], 1u);
  }
  __syncthreads();
  uint32_t* gh = a.hist1 + (int64_t)bh * kHist1Bins;
  for (int i = tid; i < kHist1Bins; i += kSelThreads) {
    const uint32_t c = s_hist[i];
    if (c) atomicAdd(&gh[i], c);
  }
}

// ---- full Selector (mode 1): three kernels in place of stage 1 -------------------------------------
// All scores of this part live in the log2 domain, Z = log2(s + eps) = z / ln 2: Soft-NMS is
// homogeneous of degree one in z, the head softmax of z / T is 2^(Z / T) normalised, and the
// adjustment alpha_cross * log(r) becomes alpha_cross * log2(r); the ranking key is 2^Z_adj = e^z_adj,
// a positive fp32 whose bit pattern orders like z_adj, so stages 2-4 are shared with mode 0.
__device__ __forceinline__ float fast_log2s(float x) { return __builtin_amdgcn_logf(x); }

// Deterministic block sums of kSegStats doubles per thread (fixed tree, one pair of barriers for all of
// them); results valid in every thread.  scratch: [kSelThreads / 64][kSegStats] doubles of LDS.
__device__ __forceinline__ void block_sums_f64(double (&v)[kSegStats], double (*scratch)[kSegStats]) {
#pragma unroll
  for (int i = 0; i < kSegStats; ++i) {
#pragma unroll
    for (int d = 32; d >= 1; d >>= 1) v[i] += __shfl_xor(v[i], d);
  }
  __syncthreads();
  if ((threadIdx.x & 63) == 0) {
#pragma unroll
    for (int i = 0; i < kSegStats; ++i) scratch[threadIdx.x >> 6][i] = v[i];
  }
  __syncthreads();
#pragma unroll
  for (int i = 0; i < kSegStats; ++i) v[i] = (scratch[0][i] + scratch[1][i]) + (scratch[2][i] + scratch[3][i]);
}

// (1a) evidence f (as in mode 0) and the unnormalised prior pi_kn * pi_pos (Eqs. selector_prior_kn,
// selector_u, selector_prior_pos) of one segment, and the segment's sums for lambda*.
__global__ __launch_bounds__(kSelThreads) void sel_prior_kernel(const SelArgs a) {
  const int seg = blockIdx.x, h = blockIdx.y, b = blockIdx.z;
  if (a.is_slow != nullptr && a.is_slow[b * a.fs] == 0) return;
  const Problem pb = problem_of(a, b);
  const int G = a.G, rows = G + 1;
  const bool fused = a.part != nullptr;  // grid-uniform: no merge launch has run
  if (fused && seg >= (int)gridDim.x - G) {
    merge_head(a, b, h, seg - ((int)gridDim.x - G));
    return;
  }
  const int p_lo = seg * kSelSeg;
  if (p_lo >= pb.nJ) return;
  const int tid = threadIdx.x;
  const int bh = b * a.Hkv + h;
  const float* lg = a.logits + (int64_t)bh * rows * a.ld_pos;  // [tile][G heads + key norms][32]
  float* fbuf = reinterpret_cast<float*>(a.keys) + (int64_t)bh * a.ld_pos;
  float* prior = a.prior + (int64_t)bh * a.ld_pos;
  const float al = a.alpha;  // mu(j) = sum_g sc[g] 2^(alpha (y_g(j) - sM[g]))  (Eq. selector_mu)
  __shared__ float s_jM[16], s_jc[16];
  if (fused) {
    group_jstat(a, b, h, s_jM, s_jc);
    __syncthreads();
  }
  float sM[16], sc[16];
#pragma unroll
  for (int g = 0; g < 16; ++g) {
    const float2 t = g >= G ? make_float2(0.f, 0.f) : fused ? make_float2(s_jM[g], s_jc[g]) : a.jstat[b * a.Hq + h * G + g];
    sM[g] = t.x;
    sc[g] = t.y;
  }
  // u(j) = p / D, 1 - u(j) + eps = ((|J| - 1 - p) + eps) / D + eps with D = |J| - 1 + eps: the second
  // form keeps full relative precision near the tail, where 1 - u cancels.
  const float D = (float)(pb.nJ - 1) + a.eps;
  const float inv_D = 1.0f / D;
  const float beta2 = a.beta * 1.4426950408889634f;
  double sums[kSegStats] = {0.0, 0.0, 0.0, 0.0, 0.0};
#pragma unroll
  for (int r = 0; r < 2; ++r) {
    const int p = p_lo + r * (kSelSeg / 2) + tid * 4;
    if (p >= pb.nJ) continue;
    const float* lt = lg + (int64_t)(p >> 5) * rows * kTile + (p & 31);
    float f[4] = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int g = 0; g < 16; ++g) {
      if (g < G) {
        const float4 l4 = *reinterpret_cast<const float4*>(lt + g * kTile);
        f[0] += sc[g] * fast_exp2s(al * (l4.x - sM[g]));
        f[1] += sc[g] * fast_exp2s(al * (l4.y - sM[g]));
        f[2] += sc[g] * fast_exp2s(al * (l4.z - sM[g]));
        f[3] += sc[g] * fast_exp2s(al * (l4.w - sM[g]));
      }
    }
    if (a.f_from_mu) {  // windowed evidence: mu was accumulated over the window's queries
      const float4 m4 = *reinterpret_cast<const float4*>(a.mu + (int64_t)bh * a.ld_pos + p);
      f[0] = m4.x * a.mu_scale; f[1] = m4.y * a.mu_scale; f[2] = m4.z * a.mu_scale; f[3] = m4.w * a.mu_scale;
    }
    if (al != 1.0f) {  // f = mu^(1/alpha) up to the normalisation done with the segment sums (Eq. selector_f)
#pragma unroll
      for (int c = 0; c < 4; ++c) f[c] = fast_exp2s(a.inv_alpha * fast_log2s(f[c]));
    }
    const float4 k4 = *reinterpret_cast<const float4*>(lt + G * kTile);
    const float k2[4] = {k4.x, k4.y, k4.z, k4.w};
    float rr[4];
#pragma unroll
    for (int c = 0; c < 4; ++c) {
      const int pc = p + c;
      const float pi_kn = fast_exp2s(-a.gamma * fast_log2s(sqrtf(k2[c]) + a.eps));
      const float u = (float)pc * inv_D;
      const float omu = ((float)(pb.nJ - 1 - pc) + a.eps) * inv_D + a.eps;
      const float up = u > 0.f ? fast_exp2s(a.p * fast_log2s(u)) : 0.f;
      const float pi_pos = fast_exp2s(-beta2 * up + a.eta * fast_log2s(omu));
      const bool ok = pc < pb.nJ;
      rr[c] = ok ? pi_kn * pi_pos : 0.f;
      f[c] = ok ? f[c] : 0.f;
      sums[0] += (double)f[c];
      sums[1] += (double)rr[c];
      sums[2] += (double)f[c] * (double)f[c];
      sums[3] += (double)f[c] * (double)rr[c];
      sums[4] += (double)rr[c] * (double)rr[c];
    }
    *reinterpret_cast<float4*>(fbuf + p) = make_float4(f[0], f[1], f[2], f[3]);
    *reinterpret_cast<float4*>(prior + p) = make_float4(rr[0], rr[1], rr[2], rr[3]);
  }
  __shared__ double s_scr[kSelThreads / 64][kSegStats];
  double* out = a.segstat + ((int64_t)bh * a.n_seg_cap + seg) * kSegStats;
  block_sums_f64(sums, s_scr);
  if (tid == 0) {
#pragma unroll
    for (int i = 0; i < kSegStats; ++i) out[i] = sums[i];
  }
}

// (1b) lambda* (Eq. selector_lambda_closed) from the segment sums, the fused score (Eq. selector_closed),
// Z = log2(s + eps) (Eq. z_base) over the segment and a halo of nms_radius positions on either side,
// then Soft-NMS on the un-updated scores with the neighbourhood clipped to J (Eqs. nms_pool, nms).
__global__ __launch_bounds__(kSelThreads) void sel_fuse_kernel(const SelArgs a) {
  const int seg = blockIdx.x, h = blockIdx.y, b = blockIdx.z;
  if (a.is_slow != nullptr && a.is_slow[b * a.fs] == 0) return;
  const Problem pb = problem_of(a, b);
  const int p_lo = seg * kSelSeg;
  if (p_lo >= pb.nJ) return;
  const int tid = threadIdx.x;
  const int bh = b * a.Hkv + h;
  const float* fbuf = reinterpret_cast<const float*>(a.keys) + (int64_t)bh * a.ld_pos;
  const float* prior = a.prior + (int64_t)bh * a.ld_pos;
  float* zn = a.znms + (int64_t)bh * a.ld_pos;
  __shared__ double s_scr[kSelThreads / 64][kSegStats];
  __shared__ float s_z[kSelSeg + 2 * kMaxNmsRadius];
  const int n_seg = (pb.nJ + kSelSeg - 1) / kSelSeg;
  const double* st = a.segstat + (int64_t)bh * a.n_seg_cap * kSegStats;
  double tot[kSegStats];
#pragma unroll
  for (int i = 0; i < kSegStats; ++i) {
    double v = 0.0;
    for (int s = tid; s < n_seg; s += kSelThreads) v += st[(int64_t)s * kSegStats + i];
    tot[i] = v;
  }
  block_sums_f64(tot, s_scr);
  // f and r normalised to sum 1: |f|^2 = tot2 / F^2, f.r = tot3 / (F R), |r|^2 = tot4 / R^2
  const double F = tot[0], Rs = tot[1];
  const double ff = tot[2] / (F * F), fr = tot[3] / (F * Rs), rr = tot[4] / (Rs * Rs);
  const double den = ff - 2.0 * fr + rr;
  double lambda = den > 1e-300 ? (ff - fr) / den : 0.0;
  lambda = fmin(fmax(lambda, 0.0), (double)a.lambda_clip);
  const float wf = (float)((1.0 - lambda) / F), wr = (float)(lambda / Rs);
  const int rad = a.nms_radius;
  const int n_here = min(kSelSeg, pb.nJ - p_lo);
  for (int i = tid; i < n_here + 2 * rad; i += kSelThreads) {
    const int p = p_lo - rad + i;
    s_z[i] = (p >= 0 && p < pb.nJ) ? fast_log2s(wf * fbuf[p] + wr * prior[p] + a.eps) : -INFINITY;
  }
  __syncthreads();
  for (int i = tid; i < n_here; i += kSelThreads) {
    const float z = s_z[i + rad];
    float m = z;
    for (int d = 0; d <= 2 * rad; ++d) m = fmaxf(m, s_z[i + d]);
    zn[p_lo + i] = z - a.alpha_soft * fmaxf(m - z, 0.f);
  }
}

// (1c) cross-head exclusivity at each position over the Hkv heads of the sequence (Eqs. head_softmax,
// head_mutex), then the ranking key and the 12-bit histogram exactly as stage 1 of mode 0.
__global__ __launch_bounds__(kSelThreads) void sel_cross_kernel(const SelArgs a) {
  const int seg = blockIdx.x, h = blockIdx.y, b = blockIdx.z;
  if (a.is_slow != nullptr && a.is_slow[b * a.fs] == 0) return;
  const Problem pb = problem_of(a, b);
  const int p_lo = seg * kSelSeg;
  if (p_lo >= pb.nJ) return;
  const int tid = threadIdx.x;
  const int bh = b * a.Hkv + h;
  __shared__ uint32_t s_hist[kHist1Bins];
  for (int i = tid; i < kHist1Bins; i += kSelThreads) s_hist[i] = 0u;
  __syncthreads();
  const float* zb = a.znms + (int64_t)b * a.Hkv * a.ld_pos;
  uint32_t* keys = a.keys + (int64_t)bh * a.ld_pos;
  const float log2_eps = fast_log2s(a.eps);
#pragma unroll
  for (int r = 0; r < 2; ++r) {
    const int p = p_lo + r * (kSelSeg / 2) + tid * 4;
    if (p >= pb.nJ) continue;
    const float4 own4 = *reinterpret_cast<const float4*>(zb + (int64_t)h * a.ld_pos + p);
    const float own[4] = {own4.x, own4.y, own4.z, own4.w};
    float mx[4] = {own[0], own[1], own[2], own[3]};
    for (int hh = 0; hh < a.Hkv; ++hh) {
      const float4 t = *reinterpret_cast<const float4*>(zb + (int64_t)hh * a.ld_pos + p);
      mx[0] = fmaxf(mx[0], t.x); mx[1] = fmaxf(mx[1], t.y); mx[2] = fmaxf(mx[2], t.z); mx[3] = fmaxf(mx[3], t.w);
    }
    float zs[4] = {0.f, 0.f, 0.f, 0.f};
    for (int hh = 0; hh < a.Hkv; ++hh) {
      const float4 t = *reinterpret_cast<const float4*>(zb + (int64_t)hh * a.ld_pos + p);
      zs[0] += fast_exp2s((t.x - mx[0]) * a.inv_temp);
      zs[1] += fast_exp2s((t.y - mx[1]) * a.inv_temp);
      zs[2] += fast_exp2s((t.z - mx[2]) * a.inv_temp);
      zs[3] += fast_exp2s((t.w - mx[3]) * a.inv_temp);
    }
    uint32_t k[4];
#pragma unroll
    for (int c = 0; c < 4; ++c) {
      // log2 of the responsibility, floored at log2(eps)
      const float lr = fmaxf((own[c] - mx[c]) * a.inv_temp - fast_log2s(zs[c]), log2_eps);
      k[c] = __float_as_uint(fast_exp2s(own[c] + a.alpha_cross * lr));
    }
    *reinterpret_cast<uint4*>(keys + p) = make_uint4(k[0], k[1], k[2], k[3]);
    atomicAdd(&s_hist[k[0] >> 19], 1u);
    if (p + 1 < pb.nJ) atomicAdd(&s_hist[k[1] >> 19], 1u);
    if (p + 2 < pb.nJ) atomicAdd(&s_hist[k[2] >> 19], 1u);
    if (p + 3 < pb.nJ) atomicAdd(&s_hist[k[3] >> 19], 1u);
  }
  __syncthreads();
  uint32_t* gh = a.hist1 + (int64_t)bh * kHist1Bins;
  for (int i = tid; i < kHist1Bins; i += kSelThreads) {
    const uint32_t c = s_hist[i];
    if (c) atomicAdd(&gh[i], c);
  }
}

// ---- stage 2: find the threshold bin, collect its keys -----------------------------------------
__global__ __launch_bounds__(kSelThreads) void sel_cand_kernel(const SelArgs a) {
  const int seg = blockIdx.x, h = blockIdx.y, b = blockIdx.z;
  if (a.is_slow != nullptr && a.is_slow[b * a.fs] == 0) return;
  const int p_lo = seg * kSelSeg;
  const int tid = threadIdx.x;
  const int bh = b * a.Hkv + h;
  uint32_t* st = a.state + (int64_t)bh * kStateWords;
  // Requested before ctx_len has arrived (all of it readable whatever the context is): the thread's 8
  // consecutive keys -- the key row is padded to a whole segment, so both 16-byte loads are always in
  // bounds -- and its 16 bins of the pair's histogram.
  constexpr int kPer = kSelSeg / kSelThreads;
  static_assert(kPer == 8, "two 16-byte key loads per thread");
  const int p0 = p_lo + tid * kPer;
  uint32_t key[kPer];
  {
    const uint32_t* keys = a.keys + (int64_t)bh * a.ld_pos;
    const uint4 k0 = *reinterpret_cast<const uint4*>(keys + p0);
    const uint4 k1 = *reinterpret_cast<const uint4*>(keys + p0 + 4);
    key[0] = k0.x; key[1] = k0.y; key[2] = k0.z; key[3] = k0.w;
    key[4] = k1.x; key[5] = k1.y; key[6] = k1.z; key[7] = k1.w;
  }
  constexpr int kBinsPer = kHist1Bins / kSelThreads;
  uint32_t hv[kBinsPer];  // bins hi - 1, hi - 2, ... of this thread, hi = kHist1Bins - tid * kBinsPer
  {
    const uint4* hq = reinterpret_cast<const uint4*>(a.hist1 + (int64_t)bh * kHist1Bins + (kHist1Bins - (tid + 1) * kBinsPer));
    static_assert(kBinsPer == 16, "four 16-byte histogram loads per thread");
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const uint4 q4 = hq[3 - i];
      hv[4 * i] = q4.w; hv[4 * i + 1] = q4.z; hv[4 * i + 2] = q4.y; hv[4 * i + 3] = q4.x;
    }
  }
  const Problem pb = problem_of(a, b);
  if (pb.ksel == 0 || pb.ksel == (uint32_t)pb.nJ) {
    if (seg == 0 && tid == 0) {
      st[ST_KSEL] = pb.ksel;
      st[ST_FLAGS] = pb.ksel == 0 ? kFlagNone : kFlagAll;
    }
    return;
  }
  if (p_lo >= pb.nJ) return;

  uint2* cand = reinterpret_cast<uint2*>(a.cand) + (int64_t)bh * a.ld_pos;  // (key, segment it came from)
  __shared__ uint32_t s_res[2];
  __shared__ uint32_t s_scr[8];
  find_kth_desc_regs(hv, kHist1Bins, pb.ksel, s_res, s_scr);
  const uint32_t bin1 = s_res[0];
  if (seg == 0 && tid == 0) {
    st[ST_BIN1] = bin1;
    st[ST_K1] = s_res[1];
    st[ST_KSEL] = pb.ksel;
    st[ST_FLAGS] = 0u;
  }
  uint32_t mine = 0;  // bit i: key i falls into the threshold bin
  uint32_t above = 0; // keys of this thread in a higher bin: selected whatever the exact threshold is
#pragma unroll
  for (int i = 0; i < kPer; ++i) {
    if (p0 + i < pb.nJ) {
      if ((key[i] >> 19) == bin1) mine |= 1u << i;
      above += (key[i] >> 19) > bin1;
    }
  }
  // One prefix sum over the workgroup gives both the segment's count of keys above the threshold bin (for
  // the write stage's prefix) and every thread's place in the segment's run of candidates; one atomic per
  // workgroup reserves the run in the pair's list (one per wave made the long-context launches crawl:
  // hundreds of atomics on one counter).
  uint32_t total;
  const uint32_t ex = block_excl_scan((uint32_t)__popc(mine) | (above << 16), s_scr, &total);
  __shared__ uint32_t s_base;
  if (tid == 0) {
    a.segcnt[(int64_t)bh * a.n_seg_cap + seg] = total >> 16;
    s_base = (total & 0xffffu) != 0u ? atomicAdd(&st[ST_CAND], total & 0xffffu) : 0u;
  }
  __syncthreads();
  uint32_t base = s_base + (ex & 0xffffu);
#pragma unroll
  for (int i = 0; i < kPer; ++i)
    if (mine & (1u << i)) cand[base++] = make_uint2(key[i], (uint32_t)seg);
}

// ---- stage 3: exact threshold among the candidates, index-ordered write of the selected set ------
__global__ __launch_bounds__(kSelThreads) void sel_write_kernel(const SelArgs a) {
  const int seg = blockIdx.x, h = blockIdx.y, b = blockIdx.z;
  if (a.is_slow != nullptr && a.is_slow[b * a.fs] == 0) return;
  const Problem pb = problem_of(a, b);
  const int tid = threadIdx.x;
  const int bh = b * a.Hkv + h;
  const uint32_t* st = a.state + (int64_t)bh * kStateWords;
  int32_t* out = a.sel_idx + (int64_t)bh * a.budget;
  const int n_seg = gridDim.x;
  // padding and n_sel, spread over the segments' workgroups
  for (int i = (int)pb.ksel + seg * kSelThreads + tid; i < a.budget; i += n_seg * kSelThreads) out[i] = -1;
  if (seg == 0 && tid == 0) a.n_sel[bh] = (int32_t)pb.ksel;
  const int p_lo = seg * kSelSeg;
  if (pb.ksel == 0 || p_lo >= pb.nJ) return;
  const int p_hi = min(p_lo + kSelSeg, pb.nJ);
  if (pb.ksel == (uint32_t)pb.nJ) {  // everything is selected
    for (int p = p_lo + tid; p < p_hi; p += kSelThreads) out[p] = a.n_sink + p;
    return;
  }

  __shared__ uint32_t s_h[1024];
  __shared__ uint32_t s_res[2];
  __shared__ uint32_t s_base[2];
  __shared__ uint32_t s_scr[8];
  const uint32_t bin1 = st[ST_BIN1], k1 = st[ST_K1], n_cand = st[ST_CAND];
  const uint2* cand = reinterpret_cast<const uint2*>(a.cand) + (int64_t)bh * a.ld_pos;
  const uint32_t* keys = a.keys + (int64_t)bh * a.ld_pos;
  constexpr int kPer = kSelSeg / kSelThreads;  // consecutive positions per thread
  const int p0 = p_lo + tid * kPer;
  static_assert(kPer == 8, "two 16-byte key loads per thread");
  uint32_t key[kPer];
  {  // fetched while the threshold is worked out; the key row is padded to a multiple of kSelSeg, so the
     // full 32 bytes are always readable
    const uint4 lo4 = *reinterpret_cast<const uint4*>(keys + p0);
    const uint4 hi4 = *reinterpret_cast<const uint4*>(keys + p0 + 4);
    key[0] = lo4.x; key[1] = lo4.y; key[2] = lo4.z; key[3] = lo4.w;
    key[4] = hi4.x; key[5] = hi4.y; key[6] = hi4.z; key[7] = hi4.w;
  }
  // Exact threshold tau and tie quota among the keys of the threshold bin (typically a few hundred):
  // two LDS radix passes, bits [18:9] then [8:0]; every workgroup of the pair does the same.
  for (int i = tid; i < 1024; i += kSelThreads) s_h[i] = 0u;
  if (tid < 2) s_base[tid] = 0u;
  __syncthreads();
  for (uint32_t i = tid; i < n_cand; i += kSelThreads) atomicAdd(&s_h[(cand[i].x >> 9) & 1023u], 1u);
  __syncthreads();
  find_kth_desc(s_h, 1024, k1, s_res, s_scr);
  const uint32_t bin2 = s_res[0], k2 = s_res[1];
  __syncthreads();
  for (int i = tid; i < 512; i += kSelThreads) s_h[i] = 0u;
  __syncthreads();
  for (uint32_t i = tid; i < n_cand; i += kSelThreads) {
    const uint32_t key = cand[i].x;
    if (((key >> 9) & 1023u) == bin2) atomicAdd(&s_h[key & 511u], 1u);
  }
  __syncthreads();
  find_kth_desc(s_h, 512, k2, s_res, s_scr);
  const uint32_t tau = (bin1 << 19) | (bin2 << 9) | s_res[0];
  const uint32_t take = s_res[1];
  {  // keys selected in the segments before this one: those above the threshold bin (counted by stage 2)
     // plus the bin's own keys above tau; and the ties before this segment
    uint32_t gt = 0, eq = 0;
    for (int sg = tid; sg < seg; sg += kSelThreads) gt += a.segcnt[(int64_t)bh * a.n_seg_cap + sg];
    for (uint32_t i = tid; i < n_cand; i += kSelThreads) {
      const uint2 c = cand[i];
      if ((int)c.y < seg) {
        gt += c.x > tau;
        eq += c.x == tau;
      }
    }
#pragma unroll
    for (int d = 32; d >= 1; d >>= 1) {
      gt += __shfl_xor(gt, d);
      eq += __shfl_xor(eq, d);
    }
    if ((tid & 63) == 0) {
      atomicAdd(&s_base[0], gt);
      atomicAdd(&s_base[1], eq);
    }
  }
  __syncthreads();
  const uint32_t base_gt = s_base[0], base_eq = s_base[1];

  uint32_t cg = 0, ce = 0;
#pragma unroll
  for (int i = 0; i < kPer; ++i) {
    if (p0 + i < p_hi) {
      cg += key[i] > tau;
      ce += key[i] == tau;
    }
  }
  uint32_t total;
  const uint32_t ex = block_excl_scan(cg | (ce << 16), s_scr, &total);
  uint32_t gt_before = base_gt + (ex & 0xffffu);
  uint32_t eq_before = base_eq + (ex >> 16);
#pragma unroll
  for (int i = 0; i < kPer; ++i) {
    if (p0 + i < p_hi) {
      const bool g = key[i] > tau, e = key[i] == tau;
      if (g || (e && eq_before < take)) {
        const uint32_t pos = gt_before + min(eq_before, take);
        if (pos < pb.ksel) out[pos] = a.n_sink + p0 + i;  // always true when ctx_len <= max_len held
      }
      gt_before += g;
      eq_before += e;
    }
  }
}

// Fresh Selector state (histogram, state words) for every (b, h) of the sequences taking part.  The dense
// kernel does this for the evidence it writes; a Selector pass that runs a second time on the same evidence
// (another budget, say) starts with this launch instead, or it would count into the first pass's histogram.
__global__ __launch_bounds__(kSelThreads) void sel_clear_kernel(const SelArgs a) {
  const int h = blockIdx.y, b = blockIdx.z;
  if (a.is_slow != nullptr && a.is_slow[b * a.fs] == 0) return;
  const int bh = b * a.Hkv + h;
  uint32_t* hh = a.hist1 + (int64_t)bh * kHist1Bins;
  for (int i = threadIdx.x; i < kHist1Bins; i += kSelThreads) hh[i] = 0u;
  if (threadIdx.x < kStateWords) a.state[(int64_t)bh * kStateWords + threadIdx.x] = 0u;
}
hipError_t launch_sel_clear(const SelArgs& a, int B, hipStream_t s) {
  hipLaunchKernelGGL(sel_clear_kernel, dim3(1, a.Hkv, B), dim3(kSelThreads), 0, s, a);
  return hipGetLastError();
}

hipError_t launch_sel_score(const SelArgs& a, int B, int n_seg, hipStream_t s) {
  // with the merge on board: one more workgroup per query head
  hipLaunchKernelGGL(sel_score_kernel<false>, dim3(n_seg + (a.part != nullptr ? a.G : 0), a.Hkv, B), dim3(kSelThreads), 0, s, a);
  return hipGetLastError();
}
hipError_t launch_sel_accum(const SelArgs& a, int B, int n_seg, hipStream_t s) {
  hipLaunchKernelGGL(sel_score_kernel<true>, dim3(n_seg, a.Hkv, B), dim3(kSelThreads), 0, s, a);
  return hipGetLastError();
}
hipError_t launch_sel_finalize(const SelArgs& a, int B, int n_seg, hipStream_t s) {
  hipLaunchKernelGGL(sel_finalize_kernel, dim3(n_seg, a.Hkv, B), dim3(kSelThreads), 0, s, a);
  return hipGetLastError();
}
hipError_t launch_sel_full(const SelArgs& a, int B, int n_seg, hipStream_t s) {
  hipLaunchKernelGGL(sel_prior_kernel, dim3(n_seg + (a.part != nullptr ? a.G : 0), a.Hkv, B), dim3(kSelThreads), 0, s, a);
  hipLaunchKernelGGL(sel_fuse_kernel, dim3(n_seg, a.Hkv, B), dim3(kSelThreads), 0, s, a);
  hipLaunchKernelGGL(sel_cross_kernel, dim3(n_seg, a.Hkv, B), dim3(kSelThreads), 0, s, a);
  return hipGetLastError();
}
hipError_t launch_sel_cand(const SelArgs& a, int B, int n_seg, hipStream_t s) {
  hipLaunchKernelGGL(sel_cand_kernel, dim3(n_seg, a.Hkv, B), dim3(kSelThreads), 0, s, a);
  return hipGetLastError();
}
hipError_t launch_sel_write(const SelArgs& a, int B, int n_seg, hipStream_t s) {
  hipLaunchKernelGGL(sel_write_kernel, dim3(n_seg, a.Hkv, B), dim3(kSelThreads), 0, s, a);
  return hipGetLastError();
}

}  // namespace sfi
