// Split single-query GQA attention for gfx950: dense over a position range, or gathered by index.
//
// What it computes (paper Sec. 3.1): for one (sequence b, KV head h) and the G query heads that
// share it, logits l_g(j) = scale * <q_g, k_j> over a list of positions, and the flash-style
// partial  (m, sum_j e^{l-m}, sum_j e^{l-m} v_j)  of every workgroup's share of that list.
//   dense  mode (slow step): workgroups 0..n_split-1 cover the allowed set J = [n_sink, L - recent)
//          and also expose the fp32 logits for the Selector (Eq. window_logits, W = 1);
//          workgroup n_split covers the sink and recent rows, which the Selector never ranks
//          (Eq. allowed_set).  Keeping J apart means the J-only softmax normaliser of
//          Eq. selector_pt is just the merge of the first n_split partials.
//   gather mode (fast step): the list is  sink ++ sel_idx[0:n_sel] ++ [recent_start, L)
//          (Eq. index_set_head), strided over n_split workgroups.
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

namespace sfi {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) float f32x4;

__device__ __forceinline__ bf16x8 as_bf16x8(uint4 v) { return __builtin_bit_cast(bf16x8, v); }

__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

// two fp32 -> one dword of two truncated bf16 (low half = a)
__device__ __forceinline__ uint32_t pack_hi16(float a, float b) {
  return (__float_as_uint(a) >> 16) | (__float_as_uint(b) & 0xffff0000u);
}

template <int MODE>  // 0: dense (slow step), 1: gather (fast step)
__global__ __launch_bounds__(kAttnThreads) void attn_split_kernel(const AttnArgs a) {
  const int slot = blockIdx.x, h = blockIdx.y, b = blockIdx.z;
  if (a.is_slow != nullptr && ((a.is_slow[b] != 0) != (MODE == 0))) return;

  const int tid = threadIdx.x;
  const int lane = tid & 63, w = tid >> 6;
  const int jg = lane >> 4, n = lane & 15;
  const int G = a.G;
  const int L = a.ctx_len[b];
  const int bh = b * a.Hkv + h;

  // ---- the position list of this workgroup -------------------------------------------------
  int N;          // number of positions
  int first, step;  // tile stride of this wave
  int nS = 0, nSel = 0, rs = 0;
  const int32_t* sel = nullptr;
  bool j_range = false;
  if (MODE == 0) {
    if (slot < a.n_split) {
      N = max(0, L - a.recent - a.n_sink);
      first = slot * kWaves + w;
      step = a.n_split * kWaves;
      j_range = true;
    } else {
      nS = min(a.n_sink, L);
      rs = min(max(a.n_sink, L - a.recent), L);
      N = nS + (L - rs);
      first = w;
      step = kWaves;
      if (a.hist1 != nullptr) {  // fresh Selector state for this (b, h)
        uint32_t* hh = a.hist1 + (int64_t)bh * kHist1Bins;
        for (int i = tid; i < kHist1Bins; i += kAttnThreads) hh[i] = 0u;
        if (tid < kStateWords) a.state[(int64_t)bh * kStateWords + tid] = 0u;
      }
    }
  } else {
    nS = min(a.n_sink, L);
    nSel = a.n_sel[bh];
    rs = min(max(a.recent_start[b], nS), L);
    N = nS + nSel + (L - rs);
    sel = a.sel_idx + (int64_t)bh * a.sel_stride;
    first = slot * kWaves + w;
    step = a.n_split * kWaves;
  }
  auto row_of = [&](int p) -> int64_t {
    if (MODE == 0) return j_range ? (int64_t)(a.n_sink + p) : (int64_t)(p < nS ? p : rs + (p - nS));
    if (p < nS) return p;
    if (p < nS + nSel) return sel[p - nS];
    return rs + (p - nS - nSel);
  };

  const uint16_t* Kb = a.K + b * a.k_sb + h * a.k_sh;
  const uint16_t* Vb = a.V + b * a.v_sb + h * a.v_sh;

  // ---- Q^T operand: head n, dims kblk*32 + 8*jg .. +8 ----------------------------------------
  bf16x8 qreg[4];
  {
    const uint16_t* qp = a.q + ((int64_t)b * a.Hq + h * G + (n < G ? n : 0)) * kHeadDim + jg * 8;
#pragma unroll
    for (int kb = 0; kb < 4; ++kb) {
      uint4 t = *reinterpret_cast<const uint4*>(qp + kb * 32);
      if (n >= G) t = make_uint4(0u, 0u, 0u, 0u);
      qreg[kb] = as_bf16x8(t);
    }
  }

  float m_run = kNeg, l_run = 0.f;
  f32x4 acc[8];
#pragma unroll
  for (int e = 0; e < 8; ++e) acc[e] = f32x4{0.f, 0.f, 0.f, 0.f};

  const int nT = (N + kTile - 1) / kTile;
  const bool head_ok = n < G;
  const float c_scale = a.scale;
  float* lg_row = (MODE == 0 && j_range && a.logits != nullptr && head_ok)
                      ? a.logits + ((int64_t)b * a.Hq + h * G + n) * a.ld_pos
                      : nullptr;

  for (int t = first; t < nT; t += step) {
    const int p0 = t * kTile;
    // K rows (A operand of S^T): block A row n, block B row n
    uint4 ka[4], kb4[4], v[8];
    {
      const int64_t ra = row_of(min(p0 + n, N - 1));
      const int64_t rb = row_of(min(p0 + 16 + n, N - 1));
      const uint16_t* pa = Kb + ra * a.k_st + jg * 8;
      const uint16_t* pb = Kb + rb * a.k_st + jg * 8;
#pragma unroll
      for (int kb = 0; kb < 4; ++kb) {
        ka[kb] = *reinterpret_cast<const uint4*>(pa + kb * 32);
        kb4[kb] = *reinterpret_cast<const uint4*>(pb + kb * 32);
      }
    }
    // V rows (B operand of O): rows 4*jg + i of block A, then of block B; dims 8n .. 8n+7
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int64_t r0 = row_of(min(p0 + 4 * jg + i, N - 1));
      const int64_t r1 = row_of(min(p0 + 16 + 4 * jg + i, N - 1));
      v[i] = *reinterpret_cast<const uint4*>(Vb + r0 * a.v_st + n * 8);
      v[4 + i] = *reinterpret_cast<const uint4*>(Vb + r1 * a.v_st + n * 8);
    }

    // ---- S^T = K . Q^T ------------------------------------------------------------------------
    f32x4 sa = {0.f, 0.f, 0.f, 0.f}, sb = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int kb = 0; kb < 4; ++kb) {
      sa = __builtin_amdgcn_mfma_f32_16x16x32_bf16(as_bf16x8(ka[kb]), qreg[kb], sa, 0, 0, 0);
      sb = __builtin_amdgcn_mfma_f32_16x16x32_bf16(as_bf16x8(kb4[kb]), qreg[kb], sb, 0, 0, 0);
    }
    float x[8];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      x[i] = sa[i] * c_scale;
      x[4 + i] = sb[i] * c_scale;
    }
    if (lg_row != nullptr) {  // expose logits of J (rows past N land in the padded tail, never read)
      *reinterpret_cast<float4*>(lg_row + p0 + 4 * jg) = make_float4(x[0], x[1], x[2], x[3]);
      *reinterpret_cast<float4*>(lg_row + p0 + 16 + 4 * jg) = make_float4(x[4], x[5], x[6], x[7]);
    }
    bool ok[8];
    float mt = kNeg;
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      const int p = p0 + (i < 4 ? 4 * jg + i : 16 + 4 * jg + (i - 4));
      ok[i] = head_ok && (p < N);
      x[i] = ok[i] ? x[i] : kNeg;
      mt = fmaxf(mt, x[i]);
    }
    mt = fmaxf(mt, __shfl_xor(mt, 16));
    mt = fmaxf(mt, __shfl_xor(mt, 32));
    const float m_new = fmaxf(m_run, mt);
    const float alpha = fast_exp2((m_run - m_new) * kLog2e);
    m_run = m_new;
    float pr[8], ps = 0.f;
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      pr[i] = ok[i] ? fast_exp2((x[i] - m_new) * kLog2e) : 0.f;
      ps += pr[i];
    }
    l_run = l_run * alpha + ps;

    // ---- rescale O: this lane's accumulators belong to heads 4*jg + i ---------------------------
    float al[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) al[i] = __shfl(alpha, 4 * jg + i);
#pragma unroll
    for (int e = 0; e < 8; ++e) {
#pragma unroll
      for (int i = 0; i < 4; ++i) acc[e][i] *= al[i];
    }

    // ---- P as two bf16 terms -------------------------------------------------------------------
    uint4 phi, plo;
    {
      float lo[8];
#pragma unroll
      for (int i = 0; i < 8; ++i) lo[i] = pr[i] - __uint_as_float(__float_as_uint(pr[i]) & 0xffff0000u);
      phi = make_uint4(pack_hi16(pr[0], pr[1]), pack_hi16(pr[2], pr[3]), pack_hi16(pr[4], pr[5]),
                       pack_hi16(pr[6], pr[7]));
      plo = make_uint4(pack_hi16(lo[0], lo[1]), pack_hi16(lo[2], lo[3]), pack_hi16(lo[4], lo[5]),
                       pack_hi16(lo[6], lo[7]));
    }
    const bf16x8 a_hi = as_bf16x8(phi), a_lo = as_bf16x8(plo);

    // ---- O += P . V, one product per dim offset e ------------------------------------------------
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      uint32_t c[8];
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        const uint32_t d = (e >> 1) == 0 ? v[i].x : (e >> 1) == 1 ? v[i].y : (e >> 1) == 2 ? v[i].z : v[i].w;
        c[i] = d;
      }
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

  // ---- combine the four waves and write this workgroup's partial ----------------------------------
  l_run += __shfl_xor(l_run, 16);
  l_run += __shfl_xor(l_run, 32);

  __shared__ float s_m[kWaves][16];
  __shared__ float s_l[kWaves][16];
  __shared__ float s_red[kWaves][16][kHeadDim];
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
      for (int ww = 1; ww < kWaves; ++ww) M = fmaxf(M, s_m[ww][hh]);
      const float f = fast_exp2((s_m[w][hh] - M) * kLog2e);
      float* dst = &s_red[w][hh][n * 8];
      *reinterpret_cast<float4*>(dst) = make_float4(acc[0][i] * f, acc[1][i] * f, acc[2][i] * f, acc[3][i] * f);
      *reinterpret_cast<float4*>(dst + 4) = make_float4(acc[4][i] * f, acc[5][i] * f, acc[6][i] * f, acc[7][i] * f);
    }
  }
  __syncthreads();
  const int64_t rec0 = (((int64_t)b * a.Hq + h * G) * kSlotCap + slot) * kPartStride;
  for (int idx = tid; idx < G * kHeadDim; idx += kAttnThreads) {
    const int hh = idx >> 7, dim = idx & 127;
    float s = s_red[0][hh][dim];
#pragma unroll
    for (int ww = 1; ww < kWaves; ++ww) s += s_red[ww][hh][dim];
    a.part[rec0 + (int64_t)hh * kSlotCap * kPartStride + 4 + dim] = s;
  }
  if (tid < G) {
    float M = s_m[0][tid];
#pragma unroll
    for (int ww = 1; ww < kWaves; ++ww) M = fmaxf(M, s_m[ww][tid]);
    float ls = 0.f;
#pragma unroll
    for (int ww = 0; ww < kWaves; ++ww) ls += s_l[ww][tid] * fast_exp2((s_m[ww][tid] - M) * kLog2e);
    float* r = a.part + rec0 + (int64_t)tid * kSlotCap * kPartStride;
    r[0] = M;
    r[1] = ls;
  }
}

// out[b, g, :] = sum_s e^{m_s - M} acc_s / sum_s e^{m_s - M} l_s over the split records of (b, g).
__global__ __launch_bounds__(kHeadDim) void merge_kernel(const MergeArgs a) {
  const int bg = blockIdx.x;
  const int b = bg / a.Hq;
  int n_slots;
  if (a.mode == 0) n_slots = a.slots_slow;
  else if (a.mode == 1) n_slots = a.slots_fast;
  else n_slots = a.is_slow[b] ? a.slots_slow : a.slots_fast;
  const float* P = a.part + (int64_t)bg * kSlotCap * kPartStride;
  const int dim = threadIdx.x;
  float M = kNeg;
  for (int s = 0; s < n_slots; ++s) M = fmaxf(M, P[s * kPartStride]);
  float Z = 0.f, o = 0.f;
#pragma unroll 8
  for (int s = 0; s < n_slots; ++s) {
    const float wgt = fast_exp2((P[s * kPartStride] - M) * kLog2e);
    Z += wgt * P[s * kPartStride + 1];
    o += wgt * P[s * kPartStride + 4 + dim];
  }
  a.out[(int64_t)bg * kHeadDim + dim] = Z > 0.f ? o / Z : 0.f;
}

__global__ void advance_kernel(int32_t* ctx_len, int32_t* recent_start, int B, int n_sink, int recent) {
  const int b = blockIdx.x * blockDim.x + threadIdx.x;
  if (b < B) {
    const int L = ctx_len[b] + 1;
    ctx_len[b] = L;
    recent_start[b] = max(n_sink, L - recent);
  }
}

hipError_t launch_attn_dense(const AttnArgs& a, int B, int n_slots, hipStream_t s) {
  hipLaunchKernelGGL(attn_split_kernel<0>, dim3(n_slots, a.Hkv, B), dim3(kAttnThreads), 0, s, a);
  return hipGetLastError();
}
hipError_t launch_attn_gather(const AttnArgs& a, int B, int n_slots, hipStream_t s) {
  hipLaunchKernelGGL(attn_split_kernel<1>, dim3(n_slots, a.Hkv, B), dim3(kAttnThreads), 0, s, a);
  return hipGetLastError();
}
hipError_t launch_merge(const MergeArgs& a, int B, hipStream_t s) {
  hipLaunchKernelGGL(merge_kernel, dim3(B * a.Hq), dim3(kHeadDim), 0, s, a);
  return hipGetLastError();
}
hipError_t launch_advance(int32_t* ctx_len, int32_t* recent_start, int B, int n_sink, int recent, hipStream_t s) {
  hipLaunchKernelGGL(advance_kernel, dim3((B + 63) / 64), dim3(64), 0, s, ctx_len, recent_start, B, n_sink, recent);
  return hipGetLastError();
}

}  // namespace sfi
