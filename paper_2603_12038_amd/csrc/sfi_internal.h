// Internal declarations shared by the HIP translation units of libsfi (gfx950 only).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "sfi.h"

namespace sfi {

constexpr int kHeadDim = 128;
constexpr int kTile = 32;          // KV positions per wave iteration (two 16-row MFMA blocks)
constexpr int kWaves = 4;          // waves per attention workgroup
constexpr int kAttnThreads = 64 * kWaves;
constexpr int kStashFloats = 4096;  // per-wave LDS stash for exposed logits (16 KB): 128 / G tiles; big variant: twice that
constexpr int kMaxNmsRadius = 64;
constexpr int kSegStats = 5;        // sum f, sum r, sum f^2, sum f r, sum r^2 of one segment
constexpr int kPartStride = 132;   // floats per split record: m, l, pad, pad, acc[128]
constexpr int kMaxSplits = 63;     // split workgroups per (sequence, KV head)
// records per (sequence, query head): the dense kernel writes one per wave, (splits + 1 sink/recent
// workgroup) x 4 waves; the gather kernel one per workgroup
constexpr int kSlotCap = (kMaxSplits + 1) * kWaves;
constexpr int kSelSeg = 2048;      // Selector positions per workgroup
constexpr int kSelThreads = 256;
constexpr int kHist1Bits = 12;     // first radix pass: bits [30:19] of the fp32 score
constexpr int kHist1Bins = 1 << kHist1Bits;
constexpr int kStateWords = 8;     // per (b, h) Selector state, see SelState
constexpr float kNeg = -1.0e30f;   // "minus infinity" that stays finite under subtraction
constexpr float kLog2e = 1.4426950408889634f;

// Output stores: fp32, or bf16 rounded to nearest even (results here are finite: no NaN handling).
__device__ __forceinline__ uint32_t bf16_rne(float v) {
  const uint32_t u = __float_as_uint(v);
  return (u + 0x7FFFu + ((u >> 16) & 1u)) >> 16;
}
__device__ __forceinline__ void store_out(float* out, int64_t elem, float v, bool as_bf16) {
  if (as_bf16) reinterpret_cast<uint16_t*>(out)[elem] = (uint16_t)bf16_rne(v);
  else out[elem] = v;
}
__device__ __forceinline__ void store_out4(float* out, int64_t elem, float4 v, bool as_bf16) {  // elem % 4 == 0
  if (as_bf16)
    *reinterpret_cast<uint2*>(reinterpret_cast<uint16_t*>(out) + elem) =
        make_uint2(bf16_rne(v.x) | (bf16_rne(v.y) << 16), bf16_rne(v.z) | (bf16_rne(v.w) << 16));
  else
    *reinterpret_cast<float4*>(out + elem) = v;
}

// Per (sequence, KV head) Selector state words.
enum SelState { ST_CAND = 0, ST_BIN1 = 1, ST_K1 = 2, ST_TAU = 3, ST_TAKE = 4, ST_FLAGS = 5, ST_KSEL = 6 };
constexpr uint32_t kFlagAll = 1u;   // budget >= |J|: take every position of J
constexpr uint32_t kFlagNone = 2u;  // nothing to select

// A window query under the causal mask (Eq. window_logits): the query sits at row q_len - 1 of a context that ends
// at row L_end - 1, sees rows [0, q_len) only, and its evidence covers the part of the allowed set
// J = [n_sink, L_end - recent) it sees.  For the kernels that is a dense step over a context of q_len rows whose
// recent window is what is left of the real one in front of the query: rec = max(0, recent - (L_end - q_len)).
// q_len == nullptr: an ordinary step (L = L_end, rec = recent).
__device__ __forceinline__ void window_view(const int32_t* q_len, int b, int L_end, int recent, int& L, int& rec) {
  L = L_end;
  rec = recent;
  if (q_len != nullptr) {
    L = min(max(q_len[b], 0), L_end);
    rec = max(0, recent - (L_end - L));
  }
}

constexpr int kListCap = 1024;  // sequences the ragged step's dense launch can plan for on the device (see attn_dense_items_kernel)

struct Workspace {
  float* part;        // [B*Hq][kSlotCap][kPartStride]
  float* logits;      // [B*Hq][ld_pos]   J-relative positions
  uint32_t* keys;     // [B*Hkv][ld_pos]  fp32 bit pattern of the evidence f
  uint32_t* cand;     // [B*Hkv][ld_pos][2]  keys falling into the threshold bin, each with its segment
  uint32_t* hist1;    // [B*Hkv][kHist1Bins]
  uint32_t* state;    // [B*Hkv][kStateWords]
  uint32_t* segcnt;   // [B*Hkv][n_seg_cap]  keys of each segment above the threshold bin
  int32_t* seq_splits;  // [B]  ragged step: splits per (sequence, KV head) the dense launch chose for each slow sequence
  float2* jstat;      // [B*Hq]  J-only softmax statistics of each query head (slow step)
  float* prior;       // [B*Hkv][ld]  full Selector: unnormalised prior pi_kn * pi_pos
  float* znms;        // [B*Hkv][ld]  full Selector: log2-domain score after Soft-NMS
  double* segstat;    // [B*Hkv][n_seg_cap][kSegStats]  full Selector: per-segment sums for lambda*
  float* mu;          // [B*Hkv][ld]  windowed evidence: accumulator over the window's queries
  uint32_t* arrive;   // [B*Hkv]  workgroups of a split fast-step launch that have written their record
  int32_t* guard;     // [1]  SFI_GUARD_* bits of device-side inputs the kernels found out of range and clamped
  int64_t ld_pos;     // multiple of kSelSeg
  int32_t n_seg_cap;
};

// Device-side inputs (lengths, counts, row indices, block ids) are clamped into the range the launch may
// touch before they address memory; a kernel that had to clamp ORs the matching bit into Workspace::guard
// once, on its way out.  The bit values are the public SFI_GUARD_* ones.
constexpr int kGuardCtxLen = 1, kGuardNSel = 2, kGuardSelIdx = 4, kGuardBlock = 8;

struct AttnArgs {
  const uint16_t* q;
  const uint16_t* K;
  const uint16_t* V;
  int64_t k_sb, k_sh, k_st, v_sb, v_sh, v_st;
  const int32_t* ctx_len;
  int32_t ms, fs;                // strides of the per-sequence entries: ctx_len / recent_start in int32, is_slow in bytes
                                 //   (1, 1 for plain arrays; 4, 16 when they are fields of a packed sfi_step_desc array)
  int32_t item_batch;            // dense mode, ragged step: > 0 = the launch is a fixed number of workgroups that deal the
                                 //   slow sequences' cells among themselves (attn_dense_items_kernel); the batch size
  int32_t item_wgs;              //   ... and that number of workgroups
  int32_t* seq_splits;           //   ... and where the splits chosen for each slow sequence are left, [batch]
  const int32_t* q_len;          // dense mode, nullptr or: rows each sequence's query sees (window query under the causal mask)
  const int32_t* recent_start;   // gather mode
  const int32_t* sel_idx;        // gather mode
  const int32_t* n_sel;          // gather mode
  int64_t sel_stride;
  const uint8_t* is_slow;        // nullptr: every sequence takes part
  float* part;
  int32_t slot_cap;              // gather / compact mode: records each query head has room for in part (kSlotCap in a
                                 //   caller's workspace)
  float* logits;                 // dense mode, nullptr: do not expose logits
  int32_t with_knorm;            // dense mode: also expose the squared key norms (full Selector)
  int32_t no_v;                  // dense mode with logits: evidence only -- V is not read, the records hold no output
  int32_t dense_wide;            // dense mode: K rows read as whole 128-byte lines (query groups of at most 8 heads, flat cache)
  int32_t big_stash;             // dense mode with logits: the variant with the 32 KB stash per wave (one workgroup per CU)
  int32_t pipelined;             // gather mode: few workgroups per (b, h), each wave walks several tiles
  float* out_direct;             // gather / compact mode with n_split == 1: write the output here, no record
  float* out_merge;              // gather / compact mode, nullptr or: the pair's last workgroup to finish merges
  uint32_t* arrive;              //   the pair's records into out_merge; arrive[b * Hkv + h] counts the finished
                                 //   workgroups of the pair (zero between launches)
  const int32_t* table;          // paged cache: block table [B][table_stride], logical page -> block of the pool
  int64_t table_stride;
  int32_t page_lg;               // log2 of the page size in rows
  int32_t page_rpb;              // row numbers a block spans in the pool's row space (block stride / row stride)
  uint32_t* hist1;               // dense mode with Selector: cleared by the sink/recent workgroup
  uint32_t* state;
  int64_t ld_pos;
  int32_t Hq, Hkv, G, n_sink, recent, n_split;
  int32_t max_tiles;             // dense mode: tiles of J the launch covers at most (from the host's max_len)
  int32_t row_cap;               // dense mode: max_len - 1, the last row the launch may touch
  float scale_log2;              // logit scale times log2(e): the kernels work on y = log2(e) * logit
  const uint16_t* Kc;            // compact mode: sink ++ selected rows of each (b, h), rows back to back
  const uint16_t* Vc;
  int64_t c_sb, c_sh;            // compact mode: strides between sequences / KV heads, in elements
  int32_t c_rows;                // compact mode: rows every (b, h) slice of Kc / Vc holds (all readable)
  int32_t out_bf16;              // out_direct / out_merge are bf16 (rounded to nearest even as stored), not fp32
  int32_t len_cap;               // ctx_len[b] is clamped to [0, len_cap]: the launch's max_len, else cfg.max_ctx
  int32_t n_blocks;              // paged cache: block ids are clamped to [0, n_blocks)
  int32_t* guard;                // Workspace::guard
};

// Reorg: gather the sink and the selected rows of every (b, h) into the compact buffers.
struct ReorgArgs {
  const uint16_t* K;
  const uint16_t* V;
  int64_t k_sb, k_sh, k_st, v_sb, v_sh, v_st;
  const int32_t* sel_idx;
  const int32_t* n_sel;
  const int32_t* ctx_len;
  const uint8_t* is_slow;        // nullptr: every sequence takes part
  int32_t ms, fs;                // strides of ctx_len (int32) and is_slow (bytes), see AttnArgs
  int64_t sel_stride;
  uint16_t* Kc;
  uint16_t* Vc;
  int64_t c_sb, c_sh;
  int32_t Hkv, n_sink;
  const int32_t* table;          // paged cache (see AttnArgs)
  int64_t table_stride;
  int32_t page_lg, page_rpb;
  int32_t len_cap, n_blocks;     // clamps of ctx_len and of the block ids (see AttnArgs)
  int32_t* guard;
};
constexpr int kReorgRows = 64;   // compact rows per workgroup of the Reorg kernel

struct MergeArgs {
  const float* part;
  float* out;
  const uint8_t* is_slow;
  int32_t Hq, slots_slow, slots_fast;  // slot counts for slow / fast sequences
  int32_t mode;                        // 0: all sequences use slots_slow, 1: all use slots_fast, 2: per is_slow
  float2* jstat;                       // dense records: also leave the J-only softmax statistics here (may be null)
  int32_t n_j, G;                      // records that cover J; query heads per KV head
  const int32_t* ctx_len;              // dense records: the number of sink / recent records follows from it
  const int32_t* q_len;                // the dense launch's (see window_view)
  int32_t n_sink, recent;
  float alpha;                         // power-mean exponent of the evidence (Eq. selector_mu)
  int32_t len_cap;                     // the clamp the dense launch applied to ctx_len
  int32_t out_bf16;                    // out is bf16
  int32_t ms = 1, fs = 1;              // strides of ctx_len (int32) and is_slow (bytes), see AttnArgs
};

struct SelArgs {
  const float2* jstat;
  const float* logits;
  uint32_t* keys;
  uint32_t* cand;
  uint32_t* hist1;
  uint32_t* state;
  uint32_t* segcnt;
  const int32_t* ctx_len;
  const int32_t* q_len;    // accumulation of a window query under the causal mask (see window_view), else nullptr
  const int32_t* seq_splits;  // ragged step: splits the dense launch chose per sequence (n_jrec = 4 x that), else nullptr
  int32_t ms, fs;          // strides of ctx_len (int32) and is_slow (bytes), see AttnArgs
  const uint8_t* is_slow;
  int32_t* sel_idx;
  int32_t* n_sel;
  int64_t ld_pos;
  int32_t n_seg_cap;
  int32_t Hq, Hkv, G, n_sink, recent, budget;
  int32_t n_jrec;          // dense records that cover J (one per wave of the dense launch)
  // full Selector (mode 1)
  float* prior;
  float* znms;
  double* segstat;
  float gamma, beta, p, eta, lambda_clip, alpha_soft, alpha_cross, inv_temp, eps;
  int32_t nms_radius;
  float alpha, inv_alpha;  // power-mean exponent of the evidence and its reciprocal
  // windowed evidence
  float* mu;               // [B*Hkv][ld] accumulator of the head-means of the window's queries
  float mu_scale;          // 1 / number of queries added
  int32_t accum_first;     // this query starts the accumulator
  int32_t f_from_mu;       // full Selector: take the evidence from the accumulator
  int32_t lg_rows;         // rows per tile of the exposed logits: G, or G + 1 with key norms
  // slow step in one go, mode 0: the scoring launch also merges the dense kernel's records (one more
  // workgroup per query head) and takes the J-only softmax statistics from the record headers itself
  const float* part;       // nullptr: a merge launch has run, jstat is valid
  float* merge_out;
  int32_t len_cap;         // the clamp the dense launch applied to ctx_len
  int32_t out_bf16;        // merge_out is bf16
};

hipError_t launch_attn_dense(const AttnArgs& a, int B, int n_slots, hipStream_t s);
hipError_t launch_attn_dense_floor(const AttnArgs& a, int B, int n_slots, int wide, int idle_units, int writer, hipStream_t s);
hipError_t launch_attn_compact(const AttnArgs& a, int B, int n_slots, hipStream_t s);
hipError_t launch_reorg(const ReorgArgs& a, int B, int rows, hipStream_t s);
hipError_t launch_attn_gather(const AttnArgs& a, int B, int n_slots, hipStream_t s);
hipError_t launch_attn_gather_floor(const AttnArgs& a, int B, int n_slots, int tail, int burst, int tpw, int depth, hipStream_t s);
hipError_t launch_merge(const MergeArgs& a, int B, hipStream_t s);
hipError_t launch_sel_clear(const SelArgs& a, int B, hipStream_t s);
hipError_t launch_sel_score(const SelArgs& a, int B, int n_seg, hipStream_t s);
hipError_t launch_sel_accum(const SelArgs& a, int B, int n_seg, hipStream_t s);
hipError_t launch_sel_finalize(const SelArgs& a, int B, int n_seg, hipStream_t s);
hipError_t launch_sel_full(const SelArgs& a, int B, int n_seg, hipStream_t s);
hipError_t launch_sel_cand(const SelArgs& a, int B, int n_seg, hipStream_t s);
hipError_t launch_sel_write(const SelArgs& a, int B, int n_seg, hipStream_t s);
hipError_t launch_trigger(const int32_t* last_token, const uint32_t* bitmap, int vocab, int t_max, int32_t* since_slow,
                          uint8_t* is_slow, int B, hipStream_t s);
hipError_t launch_advance(int32_t* ctx_len, int32_t* recent_start, int B, int n_sink, int recent, hipStream_t s);
hipError_t launch_step_begin(sfi_step_desc* desc, const int32_t* last_token, const uint32_t* bitmap, int vocab, int t_max,
                             int advance, int B, int n_sink, int recent, hipStream_t s);

}  // namespace sfi
