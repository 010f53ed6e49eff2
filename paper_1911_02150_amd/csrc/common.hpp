// Shared declarations of the gfx950 decode library: kernel parameter blocks and
// the host-side launchers each .hip file exports to the C-ABI layer.
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

namespace mqa {

constexpr int kMaxSplits = 64;          // upper bound on position ranges per sequence a caller can ask for
constexpr int kMaxAutoSplits = 256;     // ... and that the heuristics choose (one sequence alone fills the chip)
constexpr float kLog2e = 1.4426950408889634f;

// One decode launch.  "Sequences" here are KV groups: a multi-query call has
// nseq = b groups of G = h heads; a multi-head call has nseq = b*h groups of
// G = 1 head, and lens is indexed by seq / lens_div (lens_div = h).
// What differs between the two caches of a two-segment launch (see DecodeParams).
struct DecodeSegment {
  const void* K;
  const void* V;
  const int32_t* lens;
  int G, cap, chunk, S, HG, slot0, lens_div;
};

struct DecodeParams {
  const float* q;        // [nseq, G, k]
  const void* K;         // [nseq, cap, k]
  const void* V;         // [nseq, cap, v]
  const int32_t* lens;   // [nseq / lens_div]
  const int32_t* order;  // MFMA kernel: null, or a permutation of the groups, longest first (scheduling only)
  float* o;              // [nseq, G, v]
  // Partial softmax states, one per (row, slot): row = seq*G + head over the whole call,
  // slot = slot0 + range.  PS slots per row; PS = 0 means "no partials: write o directly".
  float* part_o;         // [nseq*G, PS, v]  un-normalised partial outputs
  float* part_m;         // [nseq*G, PS]     running maxima (log2 domain)
  float* part_l;         // [nseq*G, PS]     sums of 2^(logit - max)
  int PS, slot0;
  int nseq, G, cap, lens_div;
  int k, v;
  int window;            // > 0: attend only to the last `window` valid positions (0 = all)
  int causal_h;          // > 0 (MFMA kernel): the G rows of a group are n = G/causal_h consecutive queries
                         // x causal_h heads; query j sits at position L-n+j and sees positions <= its own
  int chunk;             // positions per range (multiple of 32)
  int S;                 // ranges per sequence
  int HG;                // head groups per sequence (MFMA kernel: ceil(G / (16*HB)))
  int merge_alias;       // MFMA kernel: 1 = the wave-merge buffers re-use the q operands' LDS
  int persist;           // MFMA kernel, 64-head form: > 0 = that many workgroups (the grid) each take several ranked
                         // sequences in turn instead of one workgroup per sequence; the ranking is `order`, or, if
                         // that is null, made by every workgroup for itself
  float qscale;          // scale * log2(e): logits are kept in the log2 domain
  // MFMA kernel, two-segment launches only: workgroups [nblocks0, grid) work on seg1 instead of
  // the fields above (same q, o and partial-state rows)
  int nblocks0;
  DecodeSegment seg1;
  __host__ __device__ DecodeSegment seg0() const { return DecodeSegment{K, V, lens, G, cap, chunk, S, HG, slot0, lens_div}; }
#ifdef MQA_TIMELINE
  long long* timeline;   // debug builds only: [waves][8] wall-clock stamps
#endif
};

// The merge of the partial states.  The slots of a row come from up to two launches
// ("segments": e.g. the memory shared by the hypotheses of a beam and each hypothesis' own
// rows); a segment wrote slot s only if its range s starts before the row's length there.
struct CombineSegment {
  const int32_t* lens;   // length of row r in this segment: lens[r / rows_per_len]
  int rows_per_len;
  int cap, window, chunk, S;
};
struct CombineParams {
  const float* part_o;   // [rows, PS, v]
  const float* part_m;   // [rows, PS]
  const float* part_l;   // [rows, PS]
  float* o;              // [rows, v]
  long long rows;
  int v, PS, nseg;
  CombineSegment seg[2]; // segment 0 owns slots [0, seg[0].S), segment 1 the next seg[1].S
};

struct Tuning {
  int splits = 0;
  int kernel = 0;
  int flags = 0;
};

// decode_mfma.hip: bf16 cache, k = v = 128; 16 or 32 heads per workgroup.
bool mfma_shape_ok(int G, int k, int v, int is_bf16, int cap);
int mfma_heads_per_block(int G, int flags, int causal);
int mfma_persistent_workgroups(int nseq, int G, int S, int HG, int window, int causal, int flags, int* inline_rank);
hipError_t launch_decode_mfma(const DecodeParams& p, int flags, hipStream_t st);
// both segments in one launch (p.seg1 filled in, 32 heads per workgroup in both); p.order must be null
hipError_t launch_decode_mfma_two(const DecodeParams& p, long long nblocks0, long long nblocks1, hipStream_t st);

// decode_generic.hip: any k, v <= 256, float32 or bf16 cache.
hipError_t launch_decode_generic(const DecodeParams& p, int is_bf16, hipStream_t st);

// small_kernels.hip
hipError_t launch_combine(const CombineParams& p, hipStream_t st);
hipError_t launch_length_order(const int32_t* lens, int lens_div, int nseq, int cap, int32_t* order, hipStream_t st);
constexpr int kMaxOrdered = 1 << 16;      // groups the single-workgroup length ranking handles
hipError_t launch_reorder(const void* K_src, const void* V_src, const int32_t* lens_src, const int32_t* parent,
                          void* K_dst, void* V_dst, int32_t* lens_dst, int n, int h_kv, int cap,
                          size_t k_row_bytes, size_t v_row_bytes, hipStream_t st);
hipError_t launch_append(void* K, void* V, const float* k_new, const float* v_new, int32_t* lens,
                         int b, int h_kv, int cap, int k, int v, int n, int is_bf16, hipStream_t st);
hipError_t launch_stream_read(const void* src, size_t bytes, float* sink, hipStream_t st);
hipError_t launch_stream_copy(const void* src, void* dst, size_t bytes, hipStream_t st);

// project.hip
// epilogue: 0 store, 1 store max(x, 0), 2 add to what out holds
hipError_t launch_project(int mode, const float* in, const float* P, float* out,
                          int rows, int d, int h, int kv, int epilogue, hipStream_t st);

// gemm.hip: the same GEMM for large row counts / wide outputs (hipErrorNotSupported: too small, use launch_project's own kernel)
hipError_t launch_gemm_tiled(int mode, const float* in, const float* P, float* out,
                             int rows, int d, int h, int kv, int epilogue, hipStream_t st);
hipError_t launch_project_qkv_append(const float* x, const float* P_q, const float* P_k, const float* P_v,
                                     float* q, void* K, void* V, const int32_t* lens_in, int32_t* lens_out,
                                     int rows, int d, int h, int h_kv, int cap, int k, int v, int is_bf16,
                                     int mem_rows, hipStream_t st);

// stack_kernels.hip
hipError_t launch_layernorm(const float* x, float* y, int rows, int d, float eps, hipStream_t st);
hipError_t launch_embed(const int32_t* tokens, const int32_t* pos, const float* E, const float* P, float* x,
                        int rows, int d, int vocab, int max_pos, hipStream_t st);
hipError_t launch_add(float* a, const float* b, size_t n, hipStream_t st);
hipError_t launch_relu(float* a, size_t n, hipStream_t st);
hipError_t launch_argmax(const float* x, int32_t* out, int rows, int n, hipStream_t st);

// ---------------------------------------------------------------- device helpers
// First position a sequence of length L attends to, and the 32-aligned position its ranges start from.
__device__ __forceinline__ int window_lo(int L, int window) { return window > 0 ? max(0, L - window) : 0; }
__device__ __forceinline__ int window_base(int L, int window) { return window_lo(L, window) & ~31; }

// what a GEMM does with a finished output element (see launch_project)
__device__ __forceinline__ float apply_epilogue(float x, const float* dst, int epilogue) {
  if (epilogue == 1) return fmaxf(x, 0.f);
  if (epilogue == 2) return x + *dst;
  return x;
}

__device__ __forceinline__ float bf16_bits_to_float(uint32_t bits16) {
  return __uint_as_float(bits16 << 16);
}

// float32 -> bf16 bits, round to nearest even; NaN stays NaN (quiet).
__device__ __forceinline__ uint32_t float_to_bf16_rne(float x) {
  uint32_t u = __float_as_uint(x);
  if ((u & 0x7fffffffu) > 0x7f800000u) return (u >> 16) | 0x40u;
  return (u + 0x7fffu + ((u >> 16) & 1u)) >> 16;
}

__device__ __forceinline__ float wave_max(float x) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) x = fmaxf(x, __shfl_xor(x, o));
  return x;
}
__device__ __forceinline__ float wave_sum(float x) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) x += __shfl_xor(x, o);
  return x;
}

}  // namespace mqa
