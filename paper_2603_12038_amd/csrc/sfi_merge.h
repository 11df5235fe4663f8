// Merge of split records into the attention output (device function, one workgroup per output row).
#pragma once
#include "sfi_internal.h"

namespace sfi {

constexpr int kMergeThreads = 256;
constexpr int kMergeLanes = 8;
static_assert(kSlotCap <= kMergeThreads, "one record header per thread");

// out[bg, :] = sum_s 2^{m_s - M} acc_s / sum_s 2^{m_s - M} l_s over the n_slots split records of
// (sequence, query head) bg.  One workgroup of 256 threads = 8 record lanes x 32 dim quads: every
// thread owns four output dims of every eighth record, so all of a thread's loads are independent
// and in flight together.
// If jstat != nullptr the first n_j records are the ones that cover the allowed set J (dense kernel):
// their merge gives the J-only softmax statistics of this head for the Selector (Eq. selector_pt),
// stored as jstat[bg] = { M = max of y over J, Z^(-alpha) / G } with Z = sum over J of 2^(y - M): the
// head's term of Eq. selector_mu is then p^alpha / G = (Z^(-alpha) / G) * 2^(alpha (y - M)).
__device__ __forceinline__ void merge_records(const float* part, float* out, int bg, int n_slots, float2* jstat,
                                              int n_j, int G, float alpha, bool out_bf16) {
  const float* P = part + (int64_t)bg * kSlotCap * kPartStride;
  const int tid = threadIdx.x;
  const int sl = tid >> 5, c = tid & 31;

  __shared__ float s_w[kSlotCap];          // 2^{m_s - M}
  __shared__ float s_wl[kSlotCap];         // 2^{m_s - M} l_s
  __shared__ float s_max[kMergeThreads / 64];
  __shared__ float4 s_acc[kMergeLanes][32];

  // the record headers: one per thread
  float m = kNeg, l = 0.f;
  if (tid < n_slots) {
    const float2 ml = *reinterpret_cast<const float2*>(P + tid * kPartStride);
    m = ml.x;
    l = ml.y;
  }
  float M = m;
#pragma unroll
  for (int d = 32; d >= 1; d >>= 1) M = fmaxf(M, __shfl_xor(M, d));
  if ((tid & 63) == 0) s_max[tid >> 6] = M;
  // meanwhile the accumulator loads of this thread's records
  constexpr int kPer = (kSlotCap + kMergeLanes - 1) / kMergeLanes;
  float4 r[kPer];
#pragma unroll
  for (int i = 0; i < kPer; ++i) {
    const int s = sl + i * kMergeLanes;
    r[i] = s < n_slots ? *reinterpret_cast<const float4*>(P + s * kPartStride + 4 + 4 * c) : make_float4(0.f, 0.f, 0.f, 0.f);
  }
  if (jstat != nullptr) {  // block-uniform
    __shared__ float s_jm[kMergeThreads / 64], s_jz[kMergeThreads / 64];
    float mj = tid < n_j ? m : kNeg;
#pragma unroll
    for (int d = 32; d >= 1; d >>= 1) mj = fmaxf(mj, __shfl_xor(mj, d));
    if ((tid & 63) == 0) s_jm[tid >> 6] = mj;
    __syncthreads();
    const float MJ = fmaxf(fmaxf(s_jm[0], s_jm[1]), fmaxf(s_jm[2], s_jm[3]));
    float zj = tid < n_j ? l * __builtin_amdgcn_exp2f(m - MJ) : 0.f;
#pragma unroll
    for (int d = 32; d >= 1; d >>= 1) zj += __shfl_xor(zj, d);
    if ((tid & 63) == 0) s_jz[tid >> 6] = zj;
    __syncthreads();
    if (tid == 0) {
      const float Z = s_jz[0] + s_jz[1] + s_jz[2] + s_jz[3];
      const float zpow = alpha == 1.0f ? Z : __builtin_amdgcn_exp2f(alpha * __builtin_amdgcn_logf(Z));
      jstat[bg] = make_float2(MJ, 1.0f / ((float)G * zpow));
    }
  }
  __syncthreads();
  M = fmaxf(fmaxf(s_max[0], s_max[1]), fmaxf(s_max[2], s_max[3]));
  if (tid < n_slots) {
    const float wgt = __builtin_amdgcn_exp2f(m - M);
    s_w[tid] = wgt;
    s_wl[tid] = wgt * l;
  }
  __syncthreads();
  float4 o = make_float4(0.f, 0.f, 0.f, 0.f);
#pragma unroll
  for (int i = 0; i < kPer; ++i) {
    const int s = sl + i * kMergeLanes;
    if (s < n_slots) {
      const float wgt = s_w[s];
      o.x += wgt * r[i].x;
      o.y += wgt * r[i].y;
      o.z += wgt * r[i].z;
      o.w += wgt * r[i].w;
    }
  }
  s_acc[sl][c] = o;
  __syncthreads();
  if (tid < 32) {
    float Z = 0.f;
    for (int s = 0; s < n_slots; ++s) Z += s_wl[s];
    float4 t = s_acc[0][tid];
#pragma unroll
    for (int j = 1; j < kMergeLanes; ++j) {
      const float4 u = s_acc[j][tid];
      t.x += u.x; t.y += u.y; t.z += u.z; t.w += u.w;
    }
    const float inv = Z > 0.f ? 1.0f / Z : 0.f;
    if (out != nullptr)  // nullptr: only the J statistics were wanted (evidence-only pass)
      store_out4(out, (int64_t)bg * kHeadDim + 4 * tid, make_float4(t.x * inv, t.y * inv, t.z * inv, t.w * inv),
                 out_bf16);
  }
}

}  // namespace sfi
