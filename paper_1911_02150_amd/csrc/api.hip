// C-ABI layer: argument validation on the host, choice of the position split
// and of the kernel, launches.  Validation happens before any HIP call, so the
// error paths run on a machine without a GPU.
#include "../../include/mqa.h"
#include "common.hpp"

#include <mutex>

using namespace mqa;

// Scratch memory of mqa_decode_step_noalloc: partial softmax states and the length schedule of
// one call.  One copy per GPU, held until the process ends.  In host code the array's name is
// only a handle for hipGetSymbolAddress; kernels are given the address that call returns.
constexpr size_t kScratchBytes = (size_t)MQA_NOALLOC_SCRATCH_BYTES;
static __device__ __align__(256) unsigned char scratch[kScratchBytes];

namespace {

inline bool misaligned(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) != 0; }

// Longest-first scheduling pays once the workgroups outnumber the compute units two to one and the
// launch is long enough to absorb the ranking pass (~10 us with its launch gap).
constexpr int kOrderedMinBlocks = 512;
constexpr long long kOrderedMinBytes = 128ll << 20;
constexpr int kTargetBlocks = 256;    // one workgroup per compute unit: measured best for the streaming pass

#ifdef MQA_TIMELINE
long long* g_timeline = nullptr;
#endif

// Device address of `scratch` on the current device, looked up once per device.
constexpr int kMaxDevices = 64;
void* g_scratch_ptr[kMaxDevices] = {};
std::mutex g_scratch_mutex;

int scratch_address(void** out) {
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return MQA_ERR_LAUNCH;
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (!g_scratch_ptr[dev]) {
    void* ptr = nullptr;
    if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess || !ptr) return MQA_ERR_LAUNCH;
    g_scratch_ptr[dev] = ptr;
  }
  *out = g_scratch_ptr[dev];
  return MQA_OK;
}

struct Plan {
  bool use_mfma;
  int S, chunk, HG;
};

// Split of the position axis.  Every range is a multiple of 32 positions; a
// range is at least 128 (MFMA: one tile per wave) or 256 (generic) positions.
int plan_decode(int nseq, int G, int cap_all, int window, int k, int v, int is_bf16, const Tuning& tn, Plan* pl,
                int causal = 0) {
  // with a window a sequence attends to at most window positions, lying in at most
  // ceil(window/32)+1 tiles counted from the 32-aligned start of the window
  int cap = cap_all;
  if (window > 0 && window < cap_all) {
    const long long span = (((long long)window + 31) & ~31ll) + 32;
    if (span < cap) cap = (int)span;
  }
  const bool ok = mfma_shape_ok(G, k, v, is_bf16, cap_all);
  if (tn.kernel == 2 && !ok) return MQA_ERR_SHAPE;
  pl->use_mfma = ok && tn.kernel != 1;
  pl->HG = 1;
  if (pl->use_mfma) pl->HG = (G + mfma_heads_per_block(G, tn.flags, causal) - 1) / mfma_heads_per_block(G, tn.flags, causal);
  const int min_chunk = pl->use_mfma ? 128 : 256;
  int max_s = (cap + min_chunk - 1) / min_chunk;
  if (max_s > kMaxAutoSplits) max_s = kMaxAutoSplits;
  if (max_s < 1) max_s = 1;
  int S;
  if (tn.splits > 0) {
    S = tn.splits > kMaxSplits ? kMaxSplits : tn.splits;
    const int by_len = (cap + 31) / 32;
    if (S > by_len) S = by_len;
  } else {
    const long long groups = (long long)nseq * pl->HG;
    S = (int)((kTargetBlocks + groups - 1) / groups);
    if (S > max_s) S = max_s;
  }
  if (S < 1) S = 1;
  int chunk = (cap + S - 1) / S;
  chunk = (chunk + 31) & ~31;
  pl->chunk = chunk;
  pl->S = (cap + chunk - 1) / chunk;
  if (!pl->use_mfma) {
    // generic kernel, few workgroups: split the heads of a sequence over workgroups as well
    // (heads are independent, so this needs no merge)
    const long long blocks = (long long)nseq * pl->S;
    if (blocks < 128) pl->HG = (int)(G < 256 / blocks ? G : 256 / blocks);
  }
  return MQA_OK;
}

size_t partial_bytes(long long rows, int slots, int v) {
  return (size_t)rows * slots * (v + 2) * sizeof(float);
}

void set_partials(DecodeParams* p, void* workspace, long long rows, int slots, int slot0) {
  p->part_o = static_cast<float*>(workspace);
  p->part_m = p->part_o ? p->part_o + (size_t)rows * slots * p->v : nullptr;
  p->part_l = p->part_m ? p->part_m + (size_t)rows * slots : nullptr;
  p->PS = slots;
  p->slot0 = slot0;
}

CombineSegment segment_of(const DecodeParams& p) {
  CombineSegment sg;
  sg.lens = p.lens;
  sg.rows_per_len = p.G * p.lens_div;
  sg.cap = p.cap; sg.window = p.window; sg.chunk = p.chunk; sg.S = p.S;
  return sg;
}

int check_decode_args(const float* q, const void* K, const void* V, const int32_t* lens, const float* o,
                      int b, int h, int cap, int k, int v, int dt, bool need_qkv) {
  if (!lens || !o || (need_qkv && (!q || !K || !V))) return MQA_ERR_NULL;
  if (dt != MQA_F32 && dt != MQA_BF16) return MQA_ERR_DTYPE;
  if (b <= 0 || h <= 0 || cap <= 0 || k <= 0 || v <= 0) return MQA_ERR_SHAPE;
  if ((k & 7) || (v & 7) || k > 256 || v > 256) return MQA_ERR_SHAPE;
  if ((long long)b * h > (1ll << 24) || cap > (1 << 24)) return MQA_ERR_SHAPE;
  if (misaligned(o) || misaligned(lens) || (need_qkv && (misaligned(q) || misaligned(K) || misaligned(V))))
    return MQA_ERR_ALIGN;
  return MQA_OK;
}

// phase bit 0: partial pass, bit 1: combine pass
int decode_impl(const float* q, const void* K, const void* V, const int32_t* lens, float* o,
                int b, int h, int cap, int k, int v, int dt, float scale,
                void* workspace, size_t workspace_bytes, void* stream, const mqa_tuning* tuning,
                bool multi_head, int phase, int window = 0, int causal_n = 0) {
  if (window < 0 || causal_n < 0) return MQA_ERR_SHAPE;
  const int h_true = h;
  if (causal_n > 0 && (long long)h * causal_n > (1 << 20)) return MQA_ERR_SHAPE;
  // n queries x h heads per sequence: multi-query, n*h rows sharing the sequence's K/V;
  // multi-head, b*h groups of n rows (the n queries of one head) over that head's K/V
  if (causal_n > 0 && !multi_head) h = h * causal_n;
  int rc = check_decode_args(q, K, V, lens, o, b, multi_head && causal_n > 0 ? h * causal_n : h, cap, k, v, dt,
                             (phase & 1) != 0);
  if (rc) return rc;
  Tuning tn;
  if (tuning) {
    tn.splits = tuning->splits;
    tn.kernel = tuning->kernel;
    tn.flags = tuning->flags;
  }
  const int nseq = multi_head ? b * h : b;
  const int G = multi_head ? (causal_n > 0 ? causal_n : 1) : h;
  Plan pl;
  if (causal_n > 0) tn.splits = 1;     // rows end at different positions: one range per workgroup, no merge pass
  rc = plan_decode(nseq, G, cap, window, k, v, dt == MQA_BF16, tn, &pl, causal_n > 0);
  if (rc) return rc;
  if (causal_n > 0 && !pl.use_mfma) return MQA_ERR_SHAPE;       // causal rows: MFMA kernel only
  if (pl.S > 1) {
    if (!workspace || workspace_bytes < partial_bytes((long long)nseq * G, pl.S, v)) return MQA_ERR_WORKSPACE;
    if (misaligned(workspace)) return MQA_ERR_ALIGN;
  }
  DecodeParams p = {};
  p.q = q; p.K = K; p.V = V; p.lens = lens; p.o = o;
  p.nseq = nseq; p.G = G; p.cap = cap; p.lens_div = multi_head ? h : 1;
  p.k = k; p.v = v; p.window = window; p.causal_h = causal_n > 0 ? (multi_head ? 1 : h_true) : 0; p.chunk = pl.chunk; p.S = pl.S; p.HG = pl.HG;
  p.qscale = scale * kLog2e;
  set_partials(&p, workspace, (long long)nseq * G, pl.S > 1 ? pl.S : 0, 0);
  // Ragged batches with several workgroups per compute unit: schedule the longest groups first
  // (a ranking pass writes the permutation behind the partial states).  Best effort: needs the
  // workspace; results do not depend on it.
  const size_t order_off = ((pl.S > 1 ? partial_bytes((long long)nseq * G, pl.S, v) : 0) + 15) & ~(size_t)15;
  const bool worth_it = (long long)nseq * pl.S * pl.HG >= kOrderedMinBlocks &&
                        (long long)nseq * cap * (k + v) * 2 >= kOrderedMinBytes;
  const bool rank_wanted = pl.use_mfma && window == 0 && causal_n == 0 && !(tn.flags & 32) && nseq <= kMaxOrdered &&
                           (worth_it || (tn.flags & 64));
  const bool order_fits = workspace && !misaligned(workspace) &&
                          workspace_bytes >= order_off + (size_t)nseq * sizeof(int32_t);
  // more than 32 heads and more sequences than compute units: one workgroup per compute unit goes over
  // several ranked sequences, and up to 1024 sequences it ranks them itself (no ranking launch, no workspace)
  int inline_rank = 0;
  const int persistent = rank_wanted ? mfma_persistent_workgroups(nseq, G, pl.S, pl.HG, window, causal_n, tn.flags, &inline_rank) : 0;
  const bool ordered = rank_wanted && !(persistent && inline_rank) && order_fits;
  int32_t* order = ordered ? reinterpret_cast<int32_t*>(static_cast<char*>(workspace) + order_off) : nullptr;
  p.order = order;
  p.persist = (persistent && (inline_rank || ordered)) ? persistent : 0;
#ifdef MQA_TIMELINE
  p.timeline = g_timeline;
#endif
  hipStream_t st = static_cast<hipStream_t>(stream);
  if (phase & 1) {
    if (order && launch_length_order(lens, p.lens_div, nseq, cap, order, st) != hipSuccess) return MQA_ERR_LAUNCH;
    hipError_t e = pl.use_mfma ? launch_decode_mfma(p, tn.flags, st)
                               : launch_decode_generic(p, dt == MQA_BF16, st);
    if (e != hipSuccess) return MQA_ERR_LAUNCH;
  }
  if ((phase & 2) && pl.S > 1) {
    CombineParams c;
    c.part_o = p.part_o; c.part_m = p.part_m; c.part_l = p.part_l; c.o = o;
    c.rows = (long long)nseq * G; c.v = v; c.PS = pl.S; c.nseg = 1;
    c.seg[0] = segment_of(p);
    c.seg[1] = c.seg[0];
    if (launch_combine(c, st) != hipSuccess) return MQA_ERR_LAUNCH;
  }
  return MQA_OK;
}

// Beam search step: the hypotheses of a source attend to the source's shared rows (beam*h rows per
// K/V group) and to their own rows (h rows per group); the two parts leave partial states in
// disjoint slots of the same rows (one launch for both when the MFMA kernel serves both, else
// two) and one merge pass finishes.
struct BeamPlan {
  Plan src, own;
  int slots;
};

int plan_beams(int b, int beam, int h, int cap_src, int cap_own, int k, int v, int dt, BeamPlan* bp) {
  if (dt != MQA_F32 && dt != MQA_BF16) return MQA_ERR_DTYPE;
  if (b <= 0 || beam <= 0 || h <= 0 || cap_src <= 0 || cap_own <= 0 || k <= 0 || v <= 0) return MQA_ERR_SHAPE;
  if ((k & 7) || (v & 7) || k > 256 || v > 256) return MQA_ERR_SHAPE;
  if ((long long)b * beam * h > (1ll << 24) || cap_src > (1 << 24) || cap_own > (1 << 24)) return MQA_ERR_SHAPE;
  Tuning tn;
  int rc = plan_decode(b, beam * h, cap_src, 0, k, v, dt == MQA_BF16, tn, &bp->src);
  if (rc) return rc;
  rc = plan_decode(b * beam, h, cap_own, 0, k, v, dt == MQA_BF16, tn, &bp->own);
  if (rc) return rc;
  bp->slots = bp->src.S + bp->own.S;
  return MQA_OK;
}

// the four projections, with what happens to a finished output element (0 store, 1 relu, 2 add to out)
int project_impl(int mode, const float* in, const float* P, float* out, int rows, int d, int h, int kv, int epilogue,
                 void* stream) {
  if (!in || !P || !out) return MQA_ERR_NULL;
  if (mode < 0 || mode > 4 || epilogue < 0 || epilogue > 2) return MQA_ERR_DTYPE;
  if (mode == MQA_PROJ_KV || mode == MQA_PROJ_LINEAR) h = 1;
  if (rows <= 0 || d <= 0 || h <= 0 || kv <= 0) return MQA_ERR_SHAPE;
  if ((d & 7) || (kv & 7)) return MQA_ERR_SHAPE;
  if (misaligned(in) || misaligned(P) || misaligned(out)) return MQA_ERR_ALIGN;
  if (launch_project(mode, in, P, out, rows, d, h, kv, epilogue, static_cast<hipStream_t>(stream)) != hipSuccess)
    return MQA_ERR_LAUNCH;
  return MQA_OK;
}

}  // namespace

extern "C" {

int mqa_decode_step(const float* q, const void* K, const void* V, const int32_t* lens, float* o,
                    int b, int h, int cap, int k, int v, mqa_dtype dt, float scale,
                    void* workspace, size_t workspace_bytes, void* stream) {
  return decode_impl(q, K, V, lens, o, b, h, cap, k, v, (int)dt, scale, workspace, workspace_bytes, stream,
                     nullptr, false, 3);
}

int mha_decode_step(const float* q, const void* K, const void* V, const int32_t* lens, float* o,
                    int b, int h, int cap, int k, int v, mqa_dtype dt, float scale,
                    void* workspace, size_t workspace_bytes, void* stream) {
  return decode_impl(q, K, V, lens, o, b, h, cap, k, v, (int)dt, scale, workspace, workspace_bytes, stream,
                     nullptr, true, 3);
}

int mqa_decode_step_window(const float* q, const void* K, const void* V, const int32_t* lens, float* o,
                           int b, int h, int cap, int k, int v, mqa_dtype dt, float scale, int window,
                           void* workspace, size_t workspace_bytes, void* stream) {
  if (window <= 0) return MQA_ERR_SHAPE;
  return decode_impl(q, K, V, lens, o, b, h, cap, k, v, (int)dt, scale, workspace, workspace_bytes, stream,
                     nullptr, false, 3, window);
}

int mha_decode_step_window(const float* q, const void* K, const void* V, const int32_t* lens, float* o,
                           int b, int h, int cap, int k, int v, mqa_dtype dt, float scale, int window,
                           void* workspace, size_t workspace_bytes, void* stream) {
  if (window <= 0) return MQA_ERR_SHAPE;
  return decode_impl(q, K, V, lens, o, b, h, cap, k, v, (int)dt, scale, workspace, workspace_bytes, stream,
                     nullptr, true, 3, window);
}

int mqa_decode_step_ex(const float* q, const void* K, const void* V, const int32_t* lens, float* o,
                       int b, int h, int cap, int k, int v, mqa_dtype dt, float scale,
                       void* workspace, size_t workspace_bytes, void* stream, const mqa_tuning* tuning) {
  return decode_impl(q, K, V, lens, o, b, h, cap, k, v, (int)dt, scale, workspace, workspace_bytes, stream,
                     tuning, false, 3);
}

int mha_decode_step_ex(const float* q, const void* K, const void* V, const int32_t* lens, float* o,
                       int b, int h, int cap, int k, int v, mqa_dtype dt, float scale,
                       void* workspace, size_t workspace_bytes, void* stream, const mqa_tuning* tuning) {
  return decode_impl(q, K, V, lens, o, b, h, cap, k, v, (int)dt, scale, workspace, workspace_bytes, stream,
                     tuning, true, 3);
}

int mqa_decode_partials(const float* q, const void* K, const void* V, const int32_t* lens, float* o,
                        int b, int h, int cap, int k, int v, mqa_dtype dt, float scale,
                        void* workspace, size_t workspace_bytes, void* stream, const mqa_tuning* tuning) {
  return decode_impl(q, K, V, lens, o, b, h, cap, k, v, (int)dt, scale, workspace, workspace_bytes, stream,
                     tuning, false, 1);
}

int mqa_decode_combine(const int32_t* lens, float* o, int b, int h, int cap, int k, int v, mqa_dtype dt,
                       void* workspace, size_t workspace_bytes, void* stream, const mqa_tuning* tuning) {
  return decode_impl(nullptr, nullptr, nullptr, lens, o, b, h, cap, k, v, (int)dt, 1.0f, workspace,
                     workspace_bytes, stream, tuning, false, 2);
}

size_t mqa_decode_workspace_bytes(int b, int h, int cap, int v) {
  if (b <= 0 || h <= 0 || cap <= 0 || v <= 0) return 0;
  // ranges: at most one per 32 positions; a caller may force up to kMaxSplits, the heuristics
  // choose up to ceil(256 / groups) <= ceil(256 / b)
  int S = (cap + 31) / 32;
  int most = (kTargetBlocks + b - 1) / b;
  if (most < kMaxSplits) most = kMaxSplits;
  if (S > most) S = most;
  return partial_bytes((long long)b * h, S, v) + 16 + (size_t)b * sizeof(int32_t);   // + the schedule of the groups
}

size_t mha_decode_workspace_bytes(int b, int h, int cap, int v) {
  if (b <= 0 || h <= 0 || cap <= 0 || v <= 0) return 0;
  // b*h groups of one head: the same number of partial states, one schedule entry per group
  return mqa_decode_workspace_bytes(b, h, cap, v) + (size_t)b * (h - 1) * sizeof(int32_t);
}

int mqa_decode_num_splits(int b, int h, int cap, int k, int v, mqa_dtype dt, int multi_head,
                          const mqa_tuning* tuning) {
  if (b <= 0 || h <= 0 || cap <= 0 || k <= 0 || v <= 0) return -MQA_ERR_SHAPE;
  Tuning tn;
  if (tuning) {
    tn.splits = tuning->splits;
    tn.kernel = tuning->kernel;
    tn.flags = tuning->flags;
  }
  Plan pl;
  const int rc = plan_decode(multi_head ? b * h : b, multi_head ? 1 : h, cap, 0, k, v, dt == MQA_BF16, tn, &pl);
  return rc ? -rc : pl.S;
}

int mqa_decode_plan(int b, int h, int cap, int k, int v, mqa_dtype dt, int multi_head, int window,
                    const mqa_tuning* tuning, int32_t* splits, int32_t* chunk, int32_t* head_groups) {
  if (b <= 0 || h <= 0 || cap <= 0 || k <= 0 || v <= 0 || window < 0) return MQA_ERR_SHAPE;
  if (dt != MQA_F32 && dt != MQA_BF16) return MQA_ERR_DTYPE;
  Tuning tn;
  if (tuning) {
    tn.splits = tuning->splits;
    tn.kernel = tuning->kernel;
    tn.flags = tuning->flags;
  }
  Plan pl;
  const int rc = plan_decode(multi_head ? b * h : b, multi_head ? 1 : h, cap, window, k, v, dt == MQA_BF16, tn, &pl);
  if (rc) return rc;
  if (splits) *splits = pl.S;
  if (chunk) *chunk = pl.chunk;
  if (head_groups) *head_groups = pl.HG;
  return MQA_OK;
}

size_t mqa_decode_workspace_bytes_default(int b, int h, int cap, int k, int v, mqa_dtype dt, int multi_head) {
  if (b <= 0 || h <= 0 || cap <= 0 || k <= 0 || v <= 0) return 0;
  Plan pl;
  const long long nseq = multi_head ? (long long)b * h : b;
  if (plan_decode((int)nseq, multi_head ? 1 : h, cap, 0, k, v, dt == MQA_BF16, Tuning{}, &pl)) return 0;
  const size_t part = pl.S > 1 ? partial_bytes((long long)b * h, pl.S, v) : 0;
  return ((part + 15) & ~(size_t)15) + (size_t)nseq * sizeof(int32_t);      // + the schedule of the groups
}

int mqa_decode_step_noalloc(const float* q, const void* K, const void* V, const int32_t* lens, float* o,
                            int b, int h, int cap, int k, int v, mqa_dtype dt, float scale, void* stream) {
  // validate first, so that a wrong call touches neither the device nor the stream
  int rc = check_decode_args(q, K, V, lens, o, b, h, cap, k, v, (int)dt, true);
  if (rc) return rc;
  if (mqa_decode_workspace_bytes_default(b, h, cap, k, v, dt, 0) > kScratchBytes) return MQA_ERR_SCRATCH_LIMIT;
  void* ws = nullptr;
  rc = scratch_address(&ws);
  if (rc) return rc;
  return decode_impl(q, K, V, lens, o, b, h, cap, k, v, (int)dt, scale, ws, kScratchBytes, stream, nullptr, false, 3);
}

int mqa_append_kv(void* K, void* V, const float* k_new, const float* v_new, int32_t* lens,
                  int b, int h_kv, int cap, int k, int v, mqa_dtype dt, void* stream) {
  if (!K || !V || !k_new || !v_new || !lens) return MQA_ERR_NULL;
  if (dt != MQA_F32 && dt != MQA_BF16) return MQA_ERR_DTYPE;
  if (b <= 0 || h_kv <= 0 || cap <= 0 || k <= 0 || v <= 0) return MQA_ERR_SHAPE;
  if ((k & 7) || (v & 7)) return MQA_ERR_SHAPE;
  if (misaligned(K) || misaligned(V) || misaligned(k_new) || misaligned(v_new) || misaligned(lens))
    return MQA_ERR_ALIGN;
  if (launch_append(K, V, k_new, v_new, lens, b, h_kv, cap, k, v, 1, dt == MQA_BF16,
                    static_cast<hipStream_t>(stream)) != hipSuccess)
    return MQA_ERR_LAUNCH;
  return MQA_OK;
}

int mqa_append_kv_rows(void* K, void* V, const float* k_new, const float* v_new, int32_t* lens,
                       int b, int n, int h_kv, int cap, int k, int v, mqa_dtype dt, void* stream) {
  if (!K || !V || !k_new || !v_new || !lens) return MQA_ERR_NULL;
  if (dt != MQA_F32 && dt != MQA_BF16) return MQA_ERR_DTYPE;
  if (b <= 0 || n <= 0 || h_kv <= 0 || cap <= 0 || k <= 0 || v <= 0 || n > cap) return MQA_ERR_SHAPE;
  if ((k & 7) || (v & 7)) return MQA_ERR_SHAPE;
  if (misaligned(K) || misaligned(V) || misaligned(k_new) || misaligned(v_new) || misaligned(lens))
    return MQA_ERR_ALIGN;
  if (launch_append(K, V, k_new, v_new, lens, b, h_kv, cap, k, v, n, dt == MQA_BF16,
                    static_cast<hipStream_t>(stream)) != hipSuccess)
    return MQA_ERR_LAUNCH;
  return MQA_OK;
}

int mqa_prefill_attention(const float* q, const void* K, const void* V, const int32_t* lens, float* o,
                          int b, int n, int h, int cap, int k, int v, mqa_dtype dt, float scale,
                          void* workspace, size_t workspace_bytes, void* stream) {
  if (n <= 0 || n > cap) return MQA_ERR_SHAPE;
  return decode_impl(q, K, V, lens, o, b, h, cap, k, v, (int)dt, scale, workspace, workspace_bytes, stream,
                     nullptr, false, 3, 0, n);
}

int mha_prefill_attention(const float* q, const void* K, const void* V, const int32_t* lens, float* o,
                          int b, int n, int h, int cap, int k, int v, mqa_dtype dt, float scale,
                          void* workspace, size_t workspace_bytes, void* stream) {
  if (n <= 0 || n > cap) return MQA_ERR_SHAPE;
  return decode_impl(q, K, V, lens, o, b, h, cap, k, v, (int)dt, scale, workspace, workspace_bytes, stream,
                     nullptr, true, 3, 0, n);
}

int mqa_decode_step_beams(const float* q, const void* K_src, const void* V_src, const int32_t* lens_src,
                          const void* K_own, const void* V_own, const int32_t* lens_own, float* o,
                          int b, int beam, int h, int cap_src, int cap_own, int k, int v, mqa_dtype dt,
                          float scale, void* workspace, size_t workspace_bytes, void* stream) {
  if (!q || !K_src || !V_src || !lens_src || !K_own || !V_own || !lens_own || !o) return MQA_ERR_NULL;
  BeamPlan bp;
  int rc = plan_beams(b, beam, h, cap_src, cap_own, k, v, (int)dt, &bp);
  if (rc) return rc;
  if (misaligned(q) || misaligned(K_src) || misaligned(V_src) || misaligned(lens_src) || misaligned(K_own) ||
      misaligned(V_own) || misaligned(lens_own) || misaligned(o))
    return MQA_ERR_ALIGN;
  const long long rows = (long long)b * beam * h;
  if (!workspace || workspace_bytes < partial_bytes(rows, bp.slots, v)) return MQA_ERR_WORKSPACE;
  if (misaligned(workspace)) return MQA_ERR_ALIGN;
  hipStream_t st = static_cast<hipStream_t>(stream);
  DecodeParams ps = {};
  ps.q = q; ps.K = K_src; ps.V = V_src; ps.lens = lens_src; ps.o = o;
  ps.nseq = b; ps.G = beam * h; ps.cap = cap_src; ps.lens_div = 1;
  ps.order = nullptr;
  ps.k = k; ps.v = v; ps.window = 0; ps.causal_h = 0;
  ps.chunk = bp.src.chunk; ps.S = bp.src.S; ps.HG = bp.src.HG; ps.merge_alias = 0;
  ps.qscale = scale * kLog2e;
  set_partials(&ps, workspace, rows, bp.slots, 0);
  DecodeParams po = ps;
  po.K = K_own; po.V = V_own; po.lens = lens_own;
  po.nseq = b * beam; po.G = h; po.cap = cap_own;
  po.chunk = bp.own.chunk; po.S = bp.own.S; po.HG = bp.own.HG;
  po.slot0 = bp.src.S;
#ifdef MQA_TIMELINE
  ps.timeline = po.timeline = nullptr;
#endif
  if (bp.src.use_mfma && bp.own.use_mfma) {
    // one launch for both caches: 32 heads per workgroup in both segments
    const int hg_src = (ps.G + 31) / 32, hg_own = (po.G + 31) / 32;
    ps.HG = hg_src;
    ps.seg1 = po.seg0();
    ps.seg1.HG = hg_own;
    if (launch_decode_mfma_two(ps, (long long)ps.nseq * ps.S * hg_src, (long long)po.nseq * po.S * hg_own, st) != hipSuccess)
      return MQA_ERR_LAUNCH;
  } else {
    hipError_t e = bp.src.use_mfma ? launch_decode_mfma(ps, 0, st) : launch_decode_generic(ps, dt == MQA_BF16, st);
    if (e != hipSuccess) return MQA_ERR_LAUNCH;
    e = bp.own.use_mfma ? launch_decode_mfma(po, 0, st) : launch_decode_generic(po, dt == MQA_BF16, st);
    if (e != hipSuccess) return MQA_ERR_LAUNCH;
  }
  CombineParams c;
  c.part_o = ps.part_o; c.part_m = ps.part_m; c.part_l = ps.part_l; c.o = o;
  c.rows = rows; c.v = v; c.PS = bp.slots; c.nseg = 2;
  c.seg[0] = segment_of(ps);
  c.seg[1] = segment_of(po);
  if (launch_combine(c, st) != hipSuccess) return MQA_ERR_LAUNCH;
  return MQA_OK;
}

size_t mqa_decode_beams_workspace_bytes(int b, int beam, int h, int cap_src, int cap_own, int k, int v, mqa_dtype dt) {
  BeamPlan bp;
  if (plan_beams(b, beam, h, cap_src, cap_own, k, v, (int)dt, &bp)) return 0;
  return partial_bytes((long long)b * beam * h, bp.slots, v);
}

int mqa_beam_reorder_kv(const void* K_src, const void* V_src, const int32_t* lens_src, const int32_t* parent,
                        void* K_dst, void* V_dst, int32_t* lens_dst,
                        int n, int h_kv, int cap, int k, int v, mqa_dtype dt, void* stream) {
  if (!K_src || !V_src || !lens_src || !parent || !K_dst || !V_dst || !lens_dst) return MQA_ERR_NULL;
  if (dt != MQA_F32 && dt != MQA_BF16) return MQA_ERR_DTYPE;
  if (n <= 0 || h_kv <= 0 || cap <= 0 || k <= 0 || v <= 0) return MQA_ERR_SHAPE;
  if ((k & 7) || (v & 7) || (long long)n * h_kv > (1ll << 24) || cap > (1 << 24)) return MQA_ERR_SHAPE;
  if (K_src == K_dst || V_src == V_dst || lens_src == lens_dst) return MQA_ERR_SHAPE;     // not an in-place operation
  if (misaligned(K_src) || misaligned(V_src) || misaligned(K_dst) || misaligned(V_dst) || misaligned(lens_src) ||
      misaligned(lens_dst) || misaligned(parent))
    return MQA_ERR_ALIGN;
  const size_t esz = dt == MQA_BF16 ? 2 : 4;
  const size_t rowmax = (size_t)(k > v ? k : v) * esz / 16;
  if (((size_t)cap * rowmax + 4095) / 4096 > 65535) return MQA_ERR_SHAPE;
  if (launch_reorder(K_src, V_src, lens_src, parent, K_dst, V_dst, lens_dst, n, h_kv, cap, (size_t)k * esz,
                     (size_t)v * esz, static_cast<hipStream_t>(stream)) != hipSuccess)
    return MQA_ERR_LAUNCH;
  return MQA_OK;
}

int mqa_project_qkvo(mqa_proj_mode mode, const float* in, const float* P, float* out,
                     int rows, int d, int h, int kv, void* stream) {
  return project_impl((int)mode, in, P, out, rows, d, h, kv, 0, stream);
}

int mqa_project_qkvo_ex(mqa_proj_mode mode, const float* in, const float* P, float* out,
                        int rows, int d, int h, int kv, mqa_proj_epilogue epilogue, void* stream) {
  return project_impl((int)mode, in, P, out, rows, d, h, kv, (int)epilogue, stream);
}

int mqa_project_append_qkv(const float* x, const float* P_q, const float* P_k, const float* P_v,
                           float* q, void* K, void* V, const int32_t* lens_in, int32_t* lens_out,
                           int b, int d, int h, int h_kv, int cap, int k, int v, mqa_dtype dt, void* stream) {
  if (!x || !P_q || !P_k || !P_v || !q || !K || !V || !lens_in || !lens_out) return MQA_ERR_NULL;
  if (dt != MQA_F32 && dt != MQA_BF16) return MQA_ERR_DTYPE;
  if (b <= 0 || d <= 0 || h <= 0 || cap <= 0 || k <= 0 || v <= 0) return MQA_ERR_SHAPE;
  if (h_kv != 1 && h_kv != h) return MQA_ERR_SHAPE;
  if ((d & 7) || (k & 15) || (v & 15)) return MQA_ERR_SHAPE;
  if (lens_in == lens_out) return MQA_ERR_SHAPE;
  if (misaligned(x) || misaligned(P_q) || misaligned(P_k) || misaligned(P_v) || misaligned(q) || misaligned(K) ||
      misaligned(V) || misaligned(lens_in) || misaligned(lens_out))
    return MQA_ERR_ALIGN;
  if (launch_project_qkv_append(x, P_q, P_k, P_v, q, K, V, lens_in, lens_out, b, d, h, h_kv, cap, k, v,
                                dt == MQA_BF16, 0, static_cast<hipStream_t>(stream)) != hipSuccess)
    return MQA_ERR_LAUNCH;
  return MQA_OK;
}

int mqa_project_memory_kv(const float* M, const float* P_k, const float* P_v, void* K, void* V,
                          const int32_t* mem_lens, int32_t* lens, int b, int m, int d, int h_kv, int cap,
                          int k, int v, mqa_dtype dt, void* stream) {
  if (!M || !P_k || !P_v || !K || !V || !lens) return MQA_ERR_NULL;
  if (dt != MQA_F32 && dt != MQA_BF16) return MQA_ERR_DTYPE;
  if (b <= 0 || m <= 0 || d <= 0 || h_kv <= 0 || cap <= 0 || k <= 0 || v <= 0 || m > cap) return MQA_ERR_SHAPE;
  if ((d & 7) || (k & 15) || (v & 15) || (long long)b * m > (1ll << 30)) return MQA_ERR_SHAPE;
  if (misaligned(M) || misaligned(P_k) || misaligned(P_v) || misaligned(K) || misaligned(V) || misaligned(lens) ||
      (mem_lens && misaligned(mem_lens)))
    return MQA_ERR_ALIGN;
  if (launch_project_qkv_append(M, nullptr, P_k, P_v, nullptr, K, V, mem_lens, lens, b * m, d, 0, h_kv, cap, k, v,
                                dt == MQA_BF16, m, static_cast<hipStream_t>(stream)) != hipSuccess)
    return MQA_ERR_LAUNCH;
  return MQA_OK;
}

int mqa_memory_decode_step(const float* q, const void* K, const void* V, const int32_t* lens, float* o,
                           int b, int queries, int h, int cap, int k, int v, mqa_dtype dt, float scale,
                           void* workspace, size_t workspace_bytes, void* stream) {
  if (queries <= 0 || h <= 0 || (long long)queries * h > (1 << 20)) return MQA_ERR_SHAPE;
  // the queries x h rows of a memory are query heads over one shared K/V: the multi-query step
  return decode_impl(q, K, V, lens, o, b, queries * h, cap, k, v, (int)dt, scale, workspace, workspace_bytes, stream,
                     nullptr, false, 3);
}

int mqa_stream_read(const void* src, size_t bytes, float* sink, void* stream) {
  if (!src || !sink) return MQA_ERR_NULL;
  if (bytes == 0 || (bytes & 15)) return MQA_ERR_SHAPE;
  if (misaligned(src)) return MQA_ERR_ALIGN;
  return launch_stream_read(src, bytes, sink, static_cast<hipStream_t>(stream)) == hipSuccess ? MQA_OK : MQA_ERR_LAUNCH;
}

int mqa_stream_copy(const void* src, void* dst, size_t bytes, void* stream) {
  if (!src || !dst) return MQA_ERR_NULL;
  if (bytes == 0 || (bytes & 15)) return MQA_ERR_SHAPE;
  if (misaligned(src) || misaligned(dst)) return MQA_ERR_ALIGN;
  return launch_stream_copy(src, dst, bytes, static_cast<hipStream_t>(stream)) == hipSuccess ? MQA_OK : MQA_ERR_LAUNCH;
}

#ifdef MQA_TIMELINE
void mqa_debug_timeline(long long* p) { g_timeline = p; }
#endif

int mqa_stack_layernorm(const float* x, float* y, int rows, int d, float eps, void* stream) {
  if (!x || !y) return MQA_ERR_NULL;
  if (rows <= 0 || d <= 0) return MQA_ERR_SHAPE;
  if (misaligned(x) || misaligned(y)) return MQA_ERR_ALIGN;
  return launch_layernorm(x, y, rows, d, eps, static_cast<hipStream_t>(stream)) == hipSuccess ? MQA_OK : MQA_ERR_LAUNCH;
}

int mqa_stack_embed(const int32_t* tokens, const int32_t* positions, const float* E, const float* P, float* x,
                    int rows, int d, int vocab, int max_pos, void* stream) {
  if (!tokens || !positions || !E || !P || !x) return MQA_ERR_NULL;
  if (rows <= 0 || d <= 0 || vocab <= 0 || max_pos <= 0) return MQA_ERR_SHAPE;
  if (misaligned(tokens) || misaligned(positions) || misaligned(E) || misaligned(P) || misaligned(x)) return MQA_ERR_ALIGN;
  return launch_embed(tokens, positions, E, P, x, rows, d, vocab, max_pos, static_cast<hipStream_t>(stream)) == hipSuccess
             ? MQA_OK : MQA_ERR_LAUNCH;
}

int mqa_stack_add(float* a, const float* b, size_t n, void* stream) {
  if (!a || !b) return MQA_ERR_NULL;
  if (n == 0) return MQA_ERR_SHAPE;
  if (misaligned(a) || misaligned(b)) return MQA_ERR_ALIGN;
  return launch_add(a, b, n, static_cast<hipStream_t>(stream)) == hipSuccess ? MQA_OK : MQA_ERR_LAUNCH;
}

int mqa_stack_relu(float* a, size_t n, void* stream) {
  if (!a) return MQA_ERR_NULL;
  if (n == 0) return MQA_ERR_SHAPE;
  if (misaligned(a)) return MQA_ERR_ALIGN;
  return launch_relu(a, n, static_cast<hipStream_t>(stream)) == hipSuccess ? MQA_OK : MQA_ERR_LAUNCH;
}

int mqa_stack_argmax(const float* x, int32_t* out, int rows, int n, void* stream) {
  if (!x || !out) return MQA_ERR_NULL;
  if (rows <= 0 || n <= 0) return MQA_ERR_SHAPE;
  if (misaligned(x)) return MQA_ERR_ALIGN;          // rows of n % 4 == 0 floats are read with 16-byte loads
  return launch_argmax(x, out, rows, n, static_cast<hipStream_t>(stream)) == hipSuccess ? MQA_OK : MQA_ERR_LAUNCH;
}

const char* mqa_status_string(int status) {
  switch (status) {
    case MQA_OK: return "ok";
    case MQA_ERR_NULL: return "null pointer";
    case MQA_ERR_SHAPE: return "unsupported or non-positive size";
    case MQA_ERR_ALIGN: return "pointer not 16-byte aligned";
    case MQA_ERR_WORKSPACE: return "workspace missing or too small";
    case MQA_ERR_DTYPE: return "unknown dtype or mode";
    case MQA_ERR_LAUNCH: return "HIP launch failed";
    case MQA_ERR_SCRATCH_LIMIT: return "problem needs more scratch than the library's static buffer holds";
    default: return "unknown status";
  }
}

}  // extern "C"
