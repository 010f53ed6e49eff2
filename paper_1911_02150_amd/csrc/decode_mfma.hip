// Decode attention for a bf16 cache with k = v = 128 on gfx950 matrix cores.
//
// Computes, per KV group ("sequence") and per position range, the three lines
// logits / weights / o of the paper's incremental listings (Section 3 for
// multi-query, Section 2.4 for multi-head with one head per group):
//   logits[j,p] = sum_c q[j,c] K[p,c];  weights = softmax_p;  o[j,:] = sum_p weights[j,p] V[p,:]
//
// Work decomposition
//   grid  = nseq * S * HG workgroups (sequence, position range, group of 16*HB heads; HB = 1 or 2).
//           More than 32 heads: the STAGE form (64 heads per workgroup, see the end of this
//           comment), or, for causal rows and by a tuning flag, head groups of 32 as neighbouring
//           work items on one XCD that read the same tiles at about the same time, so that with
//           cacheable loads the second read is served by L2.
//           With an order array (ragged batches) the sequences are taken longest first; the STAGE
//           form then runs one workgroup per compute unit over several sequences.
//   block = NW wavefronts (2, 4 or 8), independent of each other up to 32 heads; wave w takes the
//           32-position tiles w, w+NW, ... of the range, so the block streams its range front to back.
//   Each wave keeps, for all 16*HB heads, a running maximum, a running sum and
//   the un-normalised output O^T [128 x 16*HB] in MFMA accumulators.  At the end
//   the NW partial states are merged through LDS and written either as the
//   final o (S = 1) or as one partial state per range for the combine pass.
//
// Operand layouts (no LDS on the K/V path)
//   v_mfma_f32_16x16x32_bf16: D[16x16] += A[16x32] B[32x16]; lane l = i + 16 g
//   holds A[i][slots (g,0..7)], B[slots (g,0..7)][i] and D[4g+r][i], r = 0..3.
//   The contraction does not care which k index a slot denotes as long as A and
//   B agree, so slots are assigned to suit the memory layout:
//   * logits^T tile = K_tile[16 pos x 128] . q^T[128 x 16 heads], 4 MFMA steps.
//     Lane (i,g) loads 4 x 16 B of ONE K row; step s uses 16-byte column chunk
//     4s+g of the row for both K and q.  MFMA row i stands for position
//     p0 + 16u + 4(i%4) + i/4, which makes the result lane (head, g) hold
//     positions p0 + 16u + 4r + g.
//   * O^T[16 cols x 16 heads] += V^T[16 cols x 32 pos] . P^T[32 pos x 16 heads].
//     The 8 logits a lane owns (2 sub-tiles x 4) are exactly its 8 B-operand
//     slots, so the weights feed the second MFMA without leaving the lane.
//     For the A operand lane (c,g) loads 16 B (8 columns 8c..8c+7) of the 8 rows
//     p0 + 4e + g (each load instruction covers 4 whole rows = 1 KiB contiguous)
//     and transposes the 8x8 block inside the lane with 32 byte-permutes; MFMA j
//     then uses column 8c+j, and D_j row i stands for output column 8i+j.
//   q (fp32) and the weights are split into bf16 hi + lo terms (two MFMAs) so
//   that only K/V storage, not the arithmetic, is reduced precision.
//
// Rows at and beyond the sequence length are never used: their logits are set
// to -inf and their V registers to zero before the second MFMA, so the cache
// may hold anything (NaN included) there.  K and V are read through buffer
// descriptors that span the sequence's capacity (the hardware returns zeros
// beyond it), not its length, which lets the first tile be requested before the
// length has arrived from memory.
//
// More than 32 heads: two head groups of 32 as separate workgroups read every tile twice (the
// second read an L2 hit) and measured 4.5 TB/s where 32 heads reach 6.5; 64 heads in one wave
// (128 accumulator registers, one wave per SIMD) stalls on its own dependency chains (3.8 TB/s).
// The STAGE form below shares each tile between two teams of waves through LDS instead.
#include "common.hpp"

namespace mqa {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) float floatx4;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;
typedef __attribute__((ext_vector_type(2))) float floatx2;
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;

namespace {

constexpr int kD = 128;              // k = v = 128
constexpr int kRowU4 = kD * 2 / 16;  // 16-byte words per cache row (16)
constexpr int kOPitch = kD + 4;      // LDS row pitch (floats) of the merge buffers
// Buffer descriptors (CDNA3/4 ISA guide, buffer resource word 3): raw 32-bit-element buffer,
// no swizzle; kNoTile is an offset no cache reaches (capacities are below 2^23 rows of 256 B).
constexpr int kBufferWord3 = 0x00020000;
constexpr uint32_t kNoTile = 0x80000000u;
constexpr float kSlack = 8.f;        // log2 of the largest softmax weight kept before the running state is rescaled

__device__ __forceinline__ floatx4 mfma16(const u32x4& a, const u32x4& b, const floatx4& c) {
  return __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, a),
                                                 __builtin_bit_cast(bf16x8, b), c, 0, 0, 0);
}

// two floats -> packed bf16 pair (round to nearest even; one v_cvt_pk_bf16_f32)
__device__ __forceinline__ uint32_t pack_bf16(float a, float b) {
  return __builtin_bit_cast(uint32_t, __builtin_convertvector(floatx2{a, b}, bf16x2));
}
// hi + lo bf16 terms of a pair: hi = rne(x), lo = rne(x - hi) (the difference is exact in float32)
__device__ __forceinline__ void split_pair(float a, float b, uint32_t& hi, uint32_t& lo) {
  hi = pack_bf16(a, b);
  lo = pack_bf16(a - __uint_as_float(hi << 16), b - __uint_as_float(hi & 0xffff0000u));
}
__device__ __forceinline__ void split8(const float (&x)[8], u32x4& hi, u32x4& lo) {
#pragma unroll
  for (int d = 0; d < 4; ++d) {
    uint32_t h, l;
    split_pair(x[2 * d], x[2 * d + 1], h, l);
    hi[d] = h;
    lo[d] = l;
  }
}

// The persistent form without a ranking launch: every workgroup ranks the sequences by length for
// itself -- a counting sort over 1024 length classes in LDS, which is free before the first
// sequence is staged; equal classes by sequence index, so that all workgroups arrive at the same
// order whatever order their LDS atomics complete in -- and keeps the sequences of its own turns
// (ranks bid, 2N-1-bid, 2N+bid, ... for N workgroups).  512 threads, nseq <= 1024, at most
// kMaxTurns turns.  Batches of equal lengths (one class) keep the given order.
constexpr int kMaxTurns = 4;
constexpr int kMaxInlineRanked = 1024;
__device__ __forceinline__ void rank_own_sequences(const int32_t* lens, int lens_div, int nseq, int cap, int nwg,
                                                   int bid, unsigned char* smem, int (&mine)[kMaxTurns]) {
  int* s_cnt = reinterpret_cast<int*>(smem);   // [1024] members of a class, then the first rank of the class
  int* s_fill = s_cnt + 1024;                  // [1024] members placed so far
  int* s_bkt = s_fill + 1024;                  // [1024] the members class by class, in order of arrival
  int* s_ord = s_bkt + 1024;                   // [1024] the ranking
  int* s_tot = s_ord + 1024;                   // [8] wave totals of the prefix sum
  int* s_min = s_tot + 8;                      // [8], [8] smallest / largest class seen by a wave
  int* s_max = s_min + 8;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const float per_pos = 1023.0f / (float)cap;
  int cls[2];
  int lo = 1023, hi = 0;
#pragma unroll
  for (int u = 0; u < 2; ++u) {
    const int i = tid + 512 * u;
    cls[u] = -1;
    if (i < nseq) {
      int L = lens[i / lens_div];
      L = L < 0 ? 0 : (L > cap ? cap : L);
      cls[u] = 1023 - min(1023, (int)((float)L * per_pos));        // class 0 holds the longest
      lo = min(lo, cls[u]);
      hi = max(hi, cls[u]);
    }
    s_cnt[i] = 0;
    s_fill[i] = 0;
  }
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) {
    lo = min(lo, __shfl_xor(lo, off));
    hi = max(hi, __shfl_xor(hi, off));
  }
  if (lane == 0) { s_min[wave] = lo; s_max[wave] = hi; }
  __syncthreads();
#pragma unroll
  for (int w = 0; w < 8; ++w) { lo = min(lo, s_min[w]); hi = max(hi, s_max[w]); }
  auto rank_of_turn = [&](int t) { return t * nwg + ((t & 1) ? nwg - 1 - bid : bid); };
  if (lo >= hi) {                              // one class: the given order
#pragma unroll
    for (int t = 0; t < kMaxTurns; ++t) mine[t] = rank_of_turn(t) < nseq ? rank_of_turn(t) : -1;
    __syncthreads();                           // (s_min / s_max are read: LDS may be re-used)
    return;
  }
#pragma unroll
  for (int u = 0; u < 2; ++u)
    if (cls[u] >= 0) atomicAdd(&s_cnt[cls[u]], 1);
  __syncthreads();
  // exclusive prefix sum over the classes: thread t owns classes 2t and 2t+1
  const int x0 = s_cnt[2 * tid], x1 = s_cnt[2 * tid + 1];
  int incl = x0 + x1;
#pragma unroll
  for (int off = 1; off < 64; off <<= 1) {
    const int y = __shfl_up(incl, off);
    if (lane >= off) incl += y;
  }
  if (lane == 63) s_tot[wave] = incl;
  __syncthreads();
  int before = 0;
  for (int w = 0; w < wave; ++w) before += s_tot[w];
  const int excl = before + incl - (x0 + x1);
  s_cnt[2 * tid] = excl;
  s_cnt[2 * tid + 1] = excl + x0;
  __syncthreads();
#pragma unroll
  for (int u = 0; u < 2; ++u)
    if (cls[u] >= 0) s_bkt[s_cnt[cls[u]] + atomicAdd(&s_fill[cls[u]], 1)] = tid + 512 * u;
  __syncthreads();
#pragma unroll
  for (int u = 0; u < 2; ++u)
    if (cls[u] >= 0) {
      const int i = tid + 512 * u, base = s_cnt[cls[u]], n = s_fill[cls[u]];
      int r = base;
      for (int m2 = 0; m2 < n; ++m2) r += (s_bkt[base + m2] < i) ? 1 : 0;     // inside a class: by index
      s_ord[r] = i;
    }
  __syncthreads();
#pragma unroll
  for (int t = 0; t < kMaxTurns; ++t) mine[t] = rank_of_turn(t) < nseq ? s_ord[rank_of_turn(t)] : -1;
  __syncthreads();                             // LDS is handed on to the q operands and the staged rounds
}

#ifdef MQA_TIMELINE   // debug builds: per-wave wall-clock stamps (100 MHz counter shared by all CUs)
#define MQA_STAMP(i) do { if (p.timeline && lane == 0) p.timeline[((size_t)blockIdx.x * NW + (threadIdx.x >> 6)) * 8 + (i)] = wall_clock64(); } while (0)
#else
#define MQA_STAMP(i) do { } while (0)
#endif

// TWO_SEG: one launch covers two caches over the same q and output rows (beam search: the rows
// shared by the hypotheses of a source, then each hypothesis' own rows); workgroups from
// p.nblocks0 on take the second segment's cache, grouping and slots.
//
// STAGE: the 64-head form.  The workgroup is two teams of four waves; team e takes heads
// 32e .. 32e+31 and wave w of either team the tiles w, w+4, ... -- the two waves that need a
// tile read it from LDS, where all eight waves put a round of four tiles (128 positions, 64 KiB)
// with coalesced 16-byte loads of whole rows, one round ahead in registers.  Each byte of the
// cache is requested from L2 once per workgroup, whatever the number of heads.
//
// ROWS: the form for causal rows (a prompt's n queries x h heads per sequence).  Every wave is a
// team of its own: it takes 16*HB of the workgroup's NW*16*HB rows and all tiles up to those rows'
// limits, so nothing is merged between waves and a workgroup's fixed costs (launch, q staging,
// output) are spread over NW times the rows.
template <int HB, int NW, bool QSPLIT, bool PSPLIT, bool NTL, bool TWO_SEG = false, bool STAGE = false, bool ROWS = false>
__global__ __launch_bounds__(NW * 64, STAGE ? 1 : 2)
void decode_mfma_kernel(DecodeParams p) {
  extern __shared__ __align__(16) unsigned char smem_raw[];
  static_assert(!STAGE || (HB == 2 && NW == 8 && !TWO_SEG), "the staged form is two teams of four waves, 32 heads each");
  static_assert(!ROWS || (!STAGE && !TWO_SEG), "one form at a time");
  constexpr int TEAMS = STAGE ? 2 : ROWS ? NW : 1;
  constexpr int NWT = NW / TEAMS;             // waves per team: they share the team's heads and split the tiles
  constexpr int NT = NWT * 64;                // threads per team
  constexpr int NH = 16 * HB;                 // heads handled by a team
  const int lane = threadIdx.x & 63;
  const int team = TEAMS > 1 ? (int)threadIdx.x / NT : 0;
  const int tid = threadIdx.x - team * NT, wave = tid >> 6;      // thread and wave inside the team
  const int i16 = lane & 15, g = lane >> 4;

  // workgroup -> (sequence, range, head group); consecutive work items share an XCD
  int nb = gridDim.x, bid = blockIdx.x;
  DecodeSegment sg = p.seg0();
  if constexpr (TWO_SEG) {
    if (bid >= p.nblocks0) {
      sg = p.seg1;
      bid -= p.nblocks0;
      nb -= p.nblocks0;
    } else {
      nb = p.nblocks0;
    }
  }
  int hg, srange, seq;
  // Persistent form (64-head kernel over a ranked ragged batch, one range and one head group per
  // sequence): the grid is one workgroup per compute unit and workgroup j takes the sequences ranked
  // j, 2N-1-j, 2N+j, ... (N workgroups; back and forth over the ranking, so that a long first
  // sequence is followed by a short second one), requesting the next sequence's q and first rows
  // while the current one's last rows are still being worked on.
  const bool persist = STAGE && p.persist > 0;
  int pass = 0;
  int mine[kMaxTurns] = {-1, -1, -1, -1};       // persistent form without a ranking launch: this workgroup's sequences
  if (persist) {
    hg = srange = 0;
    if (p.order) {
      seq = p.order[bid];
    } else {
      if constexpr (STAGE) {
        rank_own_sequences(sg.lens, sg.lens_div, p.nseq, sg.cap, p.persist, bid, smem_raw, mine);
#pragma unroll
        for (int t = 0; t < kMaxTurns; ++t) mine[t] = __builtin_amdgcn_readfirstlane(mine[t]);      // (the same in every lane)
      }
      seq = mine[0];
    }
  } else if (p.order) {
    // Longest-first schedule: workgroups are dispatched in index order, round-robin over the
    // 8 XCDs, so XCD x takes the sequences ranked x, x+8, ... by length, longest first, and all
    // work items of a sequence stay on that XCD.
    const int j = bid >> 3, items = sg.S * sg.HG;
    const int t = (j / items) * 8 + (bid & 7);
    if (t >= p.nseq) return;                   // padding of the grid to a multiple of 8 sequences
    hg = j % sg.HG;
    srange = (j / sg.HG) % sg.S;
    seq = p.order[t];
  } else {
    const int wid = ((nb & 7) == 0) ? (bid & 7) * (nb >> 3) + (bid >> 3) : bid;
    hg = wid % sg.HG;
    srange = (wid / sg.HG) % sg.S;
    seq = wid / (sg.HG * sg.S);
  }
  const int head0 = (hg * TEAMS + team) * NH;
  int begin = srange * sg.chunk;                // < cap by construction of S and chunk; moved up below for a window
  const int krow_in_tile = 4 * (i16 & 3) + (i16 >> 2);

  // Tile loads go through buffer descriptors of the sequence's K and V (base, cap rows of 256 B):
  // a lane's address is a per-lane constant plus the tile's byte offset, both in the 32-bit VGPR
  // offset that the hardware checks against the buffer size, so rows at and beyond the capacity
  // read as zeros without touching memory.  That makes the tile that straddles the capacity, the
  // speculative first tile and the "tile" a wave requests after its last one (offset kNoTile:
  // nothing is fetched) all the same branch-free code, and leaves four integer additions per tile
  // as the whole address arithmetic.  (Keeping a second tile per wave in flight was measured
  // slower: the memory pipeline accepts the extra requests no sooner.)
  struct Tile { u32x4 kr[2][4]; u32x4 vr[8]; };
  Tile tb;
  // (the sequence index is the same in every lane; saying so keeps the descriptors in scalar registers)
  auto k_rows_of = [&](int s) {
    const size_t su = (size_t)__builtin_amdgcn_readfirstlane(s);
    return __builtin_amdgcn_make_buffer_rsrc(
        const_cast<u32x4*>(reinterpret_cast<const u32x4*>(sg.K) + su * sg.cap * kRowU4), 0, sg.cap * (kRowU4 * 16), kBufferWord3);
  };
  auto v_rows_of = [&](int s) {
    const size_t su = (size_t)__builtin_amdgcn_readfirstlane(s);
    return __builtin_amdgcn_make_buffer_rsrc(
        const_cast<u32x4*>(reinterpret_cast<const u32x4*>(sg.V) + su * sg.cap * kRowU4), 0, sg.cap * (kRowU4 * 16), kBufferWord3);
  };
  __amdgpu_buffer_rsrc_t Kbuf = k_rows_of(seq), Vbuf = v_rows_of(seq);
  const uint32_t klane = (uint32_t)(krow_in_tile * kRowU4 + g) * 16u;      // row krow_in_tile, 16-byte chunk g
  const uint32_t vlane = (uint32_t)(g * kRowU4 + i16) * 16u;               // row g, 16-byte chunk i16
  // Cache rows are read exactly once per step: the non-temporal hint keeps them from displacing
  // anything in L2 / Infinity Cache and measurably raises HBM read throughput.
  constexpr int kAuxK = NTL ? 2 : 0, kAuxV = NTL ? 2 : 0;
  auto tile_offset = [&](int t, bool wanted) -> uint32_t {                  // wave-uniform
    return wanted ? (uint32_t)(begin + 32 * t) * (uint32_t)(kRowU4 * 16) : kNoTile;
  };
  auto load_k = [&](Tile& tl, uint32_t toff) {
#pragma unroll
    for (int u = 0; u < 2; ++u) {
      const uint32_t off = klane + toff + (uint32_t)u * (16u * kRowU4 * 16u);        // rows 16u.. of the tile
#pragma unroll
      for (int s4 = 0; s4 < 4; ++s4)
        tl.kr[u][s4] = __builtin_amdgcn_raw_buffer_load_b128(Kbuf, off + 64u * s4, 0, kAuxK);
    }
  };
  auto load_v = [&](Tile& tl, uint32_t toff) {
#pragma unroll
    for (int e = 0; e < 8; ++e)
      tl.vr[e] = __builtin_amdgcn_raw_buffer_load_b128(Vbuf, vlane + toff + (uint32_t)e * (4u * kRowU4 * 16u), 0, kAuxV);
  };

  // STAGE: a round is 128 consecutive rows = 2048 16-byte chunks of K and as many of V; thread x
  // of the workgroup fetches chunks x, x+512, x+1024, x+1536 of each (consecutive lanes,
  // consecutive addresses) and stores chunk c of row r at position c ^ (r & 15) of the row's 16
  // slots, so that neither these stores nor the operand reads (16 lanes reading one chunk column
  // of 16 different rows) collide on LDS banks.
  constexpr int kStageBytes = 128 * kRowU4 * 16;                  // one tensor's round: 32 KiB
  unsigned char* stage0 = smem_raw + TEAMS * (HB * 4 * 64 * 16 * 2);     // two buffers of (K round, V round)
  unsigned char* stage_k = stage0;                                        // the buffer being read
  unsigned char* stage_v = stage0 + kStageBytes;
  struct Staged { u32x4 k[STAGE ? 4 : 1], v[STAGE ? 4 : 1]; };
  Staged st;                               // the round after the one in the other LDS buffer, on its way
  const uint32_t wg_tid = threadIdx.x;
  auto stage_load_from = [&](__amdgpu_buffer_rsrc_t kb, __amdgpu_buffer_rsrc_t vb, uint32_t toff) {
    if constexpr (STAGE) {
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        st.k[j] = __builtin_amdgcn_raw_buffer_load_b128(kb, wg_tid * 16u + toff + (uint32_t)j * 8192u, 0, kAuxK);
        st.v[j] = __builtin_amdgcn_raw_buffer_load_b128(vb, wg_tid * 16u + toff + (uint32_t)j * 8192u, 0, kAuxV);
      }
    }
  };
  auto stage_load = [&](uint32_t toff) { stage_load_from(Kbuf, Vbuf, toff); };
  auto stage_store = [&](int buf) {
    if constexpr (STAGE) {
      unsigned char* dst = stage0 + buf * (2 * kStageBytes) + (wg_tid >> 4) * 256u + (((wg_tid & 15u) ^ ((wg_tid >> 4) & 15u)) << 4);
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        *reinterpret_cast<u32x4*>(dst + j * 8192) = st.k[j];
        *reinterpret_cast<u32x4*>(dst + kStageBytes + j * 8192) = st.v[j];
      }
    }
  };
  // operand reads of the wave's tile (rows 32*wave .. +31 of the round)
  auto stage_read_k = [&](Tile& tl) {
    if constexpr (STAGE) {
      const uint32_t row = 32u * wave + krow_in_tile;                       // + 16u; row & 15 = krow_in_tile
#pragma unroll
      for (int s4 = 0; s4 < 4; ++s4) {
        const unsigned char* src = stage_k + row * 256u + ((((uint32_t)(4 * s4 + g)) ^ (uint32_t)krow_in_tile) << 4);
        tl.kr[0][s4] = *reinterpret_cast<const u32x4*>(src);
        tl.kr[1][s4] = *reinterpret_cast<const u32x4*>(src + 16 * 256);
      }
    }
  };
  auto stage_read_v = [&](Tile& tl) {
    if constexpr (STAGE) {
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        const uint32_t r15 = 4u * e + g;                                    // (row & 15) of rows 4e+g and 4(e+4)+g
        const unsigned char* src = stage_v + (32u * wave + r15) * 256u + ((((uint32_t)i16) ^ r15) << 4);
        tl.vr[e] = *reinterpret_cast<const u32x4*>(src);
        tl.vr[e + 4] = *reinterpret_cast<const u32x4*>(src + 16 * 256);
      }
    }
  };
  auto round_offset = [&](int r, bool wanted) -> uint32_t {
    return wanted ? (uint32_t)(begin + 128 * r) * (uint32_t)(kRowU4 * 16) : kNoTile;
  };

  // q is requested first (loads return in order, and q is needed first), then the wave's
  // first K/V tile -- both before the length is known, so the start-up latencies overlap.
  // (Rows are in bounds for any length.)
  constexpr int QITEMS = (NH * 16 + NT - 1) / NT;        // (head, 16-byte chunk) items per thread
  float4 qa[QITEMS], qb[QITEMS];
  // In the persistent form everything below runs once per sequence, so the compiler would compute
  // the per-thread addresses of the start-up and merge code once, before the first sequence, and
  // hold them in registers through the rounds, where registers are short.  An opaque copy of the
  // thread index keeps those computations where they are used.
  auto here = [&](int x) {
    if constexpr (STAGE) asm volatile("" : "+v"(x));
    return x;
  };
  auto load_q = [&](int s, bool wanted) {
    const int tid_q = here(tid);
#pragma unroll
    for (int it = 0; it < QITEMS; ++it) {
      const int idx = tid_q + it * NT;
      const int hl = idx >> 4, c = idx & 15;               // head in block, 8-float chunk of the row
      qa[it] = qb[it] = make_float4(0.f, 0.f, 0.f, 0.f);
      if (wanted && idx < NH * 16 && head0 + hl < sg.G) {
        const float4* src = reinterpret_cast<const float4*>(p.q + ((size_t)s * sg.G + head0 + hl) * kD + c * 8);
        qa[it] = src[0];
        qb[it] = src[1];
      }
    }
  };
  int seq_next = -1, L_next = 0;
  bool prefetched = false;    // persistent form: q, the length and the first round were requested during the previous sequence
  for (;;) {                  // one turn per sequence: a single one unless persistent
  MQA_STAMP(0);
  const bool started = prefetched;
  prefetched = false;
  if (!started) {
    load_q(seq, true);
    // All waves of the workgroup put their q requests into the CU's memory queue before any of
    // them queues its 16 KiB of K/V (plain s_barrier: no wait for the data), so q is not stuck
    // behind the other waves' tiles and can be converted while the tiles stream in.
    asm volatile("" ::: "memory");
    __builtin_amdgcn_s_barrier();
    asm volatile("" ::: "memory");
    if (p.window == 0) {
      if constexpr (STAGE) {
        stage_load(round_offset(0, true));
      } else {
        load_k(tb, tile_offset(wave, true));
        load_v(tb, tile_offset(wave, true));
      }
    }
  }
  MQA_STAMP(1);
  int L = started ? L_next : sg.lens[seq / sg.lens_div];
  if (persist) {              // which sequence comes after this one: asked for now, needed a round before this one ends
    ++pass;
    if (p.order) {
      const int rank = pass * p.persist + ((pass & 1) ? p.persist - 1 - bid : bid);
      seq_next = rank < p.nseq ? p.order[rank] : -1;
    } else {
      seq_next = pass == 1 ? mine[1] : pass == 2 ? mine[2] : pass == 3 ? mine[3] : -1;
    }
  }
  L = L < 0 ? 0 : (L > sg.cap ? sg.cap : L);
  // Local attention (the paper's Section 4.1 variant): only positions [lo, L) count; the ranges
  // then start at the 32-aligned position below lo, which is known only now.
  const int lo = window_lo(L, p.window);
  if (p.window > 0) {
    begin += window_base(L, p.window);
    if constexpr (STAGE) {
      stage_load(round_offset(0, true));
    } else {
      load_k(tb, tile_offset(wave, true));
      load_v(tb, tile_offset(wave, true));
    }
  }
  // Causal rows (prefill of n queries per sequence): row r = query r / h, at position L - n + r / h,
  // attends to positions <= its own.  `end` is the largest such limit in this workgroup.
  const int causal_h = STAGE ? 0 : p.causal_h;      // (the 64-head form is never used for causal rows)
  const int nq = causal_h > 0 ? sg.G / causal_h : 1;
  int lim[HB];                                   // first position the lane's row (per head block) must NOT see
  int lim_min = L, lim_max = L;
  if (causal_h > 0) {
#pragma unroll
    for (int hb = 0; hb < HB; ++hb) lim[hb] = max(0, L - nq + min(head0 + 16 * hb + i16, sg.G - 1) / causal_h + 1);
    lim_min = max(0, L - nq + head0 / causal_h + 1);
    lim_max = max(0, L - nq + (min(head0 + NH, sg.G) - 1) / causal_h + 1);
  } else {
#pragma unroll
    for (int hb = 0; hb < HB; ++hb) lim[hb] = L;
  }
  const int end = min(begin + sg.chunk, lim_max);
  const int mask_from = min(end, lim_min);        // tiles reaching beyond this position need masking
  // (ROWS: the other waves of the workgroup have their own limits and wait at the barriers below, so a wave
  // with nothing to see goes on with no tiles and writes its zero rows at the end like any other)
  if (!ROWS && end <= begin) {
    if (p.PS == 0) {          // empty sequence: zero output rows
      for (int idx = here(tid); idx < NH * (kD / 4); idx += NT) {
        int hl = idx / (kD / 4), c4 = idx % (kD / 4);
        if (head0 + hl < sg.G)
          reinterpret_cast<float4*>(p.o + ((size_t)seq * sg.G + head0 + hl) * kD)[c4] =
              make_float4(0.f, 0.f, 0.f, 0.f);
      }
    }
    // ranges past the length write nothing; the combine pass skips them
    if (!persist || seq_next < 0) return;
    seq = seq_next;
    Kbuf = k_rows_of(seq);
    Vbuf = v_rows_of(seq);
    continue;
  }
  const int ntiles = end > begin ? (end - begin + 31) >> 5 : 0;
  const int nrounds = (ntiles + 3) >> 2;           // (64-head form)
  // Load slot s of a sequence fetches its round s; the slot after the last round is used, in the
  // persistent form, for the next sequence's first round (its q and length are requested when the
  // rounds are done and the accumulators are about to leave the registers).
  auto issue_slot = [&](int s) {
    if (s < nrounds) {
      stage_load(round_offset(s, true));
    } else if (s == nrounds && persist && seq_next >= 0) {
      stage_load_from(k_rows_of(seq_next), v_rows_of(seq_next), 0u);
      prefetched = true;
    }
  };

  // ---- q -> LDS as MFMA B operands: qs[(hb*4 + s)*64 + lane] (hi), then lo
  constexpr int QOPS = HB * 4 * 64;
  u32x4* qs = reinterpret_cast<u32x4*>(smem_raw) + team * (2 * QOPS);
  const int tid_s = here(tid);
#pragma unroll
  for (int it = 0; it < QITEMS; ++it) {
    const int idx = tid_s + it * NT;
    if (idx >= NH * 16) break;
    const int hl = idx >> 4, c = idx & 15;
    const int s4 = c >> 2, gg = c & 3;              // chunk c = 4s + g
    float x[8] = {qa[it].x, qa[it].y, qa[it].z, qa[it].w, qb[it].x, qb[it].y, qb[it].z, qb[it].w};
#pragma unroll
    for (int e = 0; e < 8; ++e) x[e] *= p.qscale;
    u32x4 hi, lo;
    split8(x, hi, lo);
    const int slot = (((hl >> 4) * 4 + s4) * 64) + (hl & 15) + 16 * gg;
    qs[slot] = hi;
    qs[QOPS + slot] = lo;
  }
  stage_store(0);             // STAGE: round 0 of the range into the first buffer ...
  if constexpr (STAGE) issue_slot(1);     // ... and round 1 requested
  __syncthreads();
  MQA_STAMP(2);

  // Single-term weights (PSPLIT = false): the weights enter the second MFMA rounded to bf16, so the
  // sum that normalises them is taken over the same rounded values -- by one more MFMA whose A
  // operand is all ones (every row of its result is sum_p P[p][head]) -- and a rounding error then
  // only perturbs the weights relative to each other (2^-9 each, averaging out over the positions)
  // instead of biasing a sharply peaked row by the rounding of its one large weight.
  floatx4 acc[HB][8], accl[HB];
  float m_run[HB], l_run[HB];
#pragma unroll
  for (int hb = 0; hb < HB; ++hb) {
    m_run[hb] = -INFINITY;
    l_run[hb] = 0.f;
    accl[hb] = floatx4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int j = 0; j < 8; ++j) acc[hb][j] = floatx4{0.f, 0.f, 0.f, 0.f};
  }
  const u32x4 ones = u32x4{0x3f803f80u, 0x3f803f80u, 0x3f803f80u, 0x3f803f80u};      // bf16 1.0 in every slot

  // one tile: logits, online softmax, weighted sum; refills the tile's registers with tile tn
  auto process = [&](Tile& tl, int t, int tn) {
    const int p0 = begin + 32 * t;
    const bool tail = p0 + 32 > mask_from || p0 < lo;
    const bool more = tn < ntiles;

    // ---- logits^T tiles: sc[u][hb][r] = logit(head 16hb+i16, position p0+16u+4r+g)
    const u32x4* qs_t = qs;      // (loop invariant: the compiler keeps the q operands in registers)
    floatx4 sc[2][HB];
#pragma unroll
    for (int hb = 0; hb < HB; ++hb) {
      sc[0][hb] = floatx4{0.f, 0.f, 0.f, 0.f};
      sc[1][hb] = floatx4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
      for (int s4 = 0; s4 < 4; ++s4) {
        const u32x4 qh = qs_t[(hb * 4 + s4) * 64 + lane];
        sc[0][hb] = mfma16(tl.kr[0][s4], qh, sc[0][hb]);
        sc[1][hb] = mfma16(tl.kr[1][s4], qh, sc[1][hb]);
        if (QSPLIT) {
          const u32x4 ql = qs_t[QOPS + (hb * 4 + s4) * 64 + lane];
          sc[0][hb] = mfma16(tl.kr[0][s4], ql, sc[0][hb]);
          sc[1][hb] = mfma16(tl.kr[1][s4], ql, sc[1][hb]);
        }
      }
    }
    if constexpr (STAGE) stage_read_v(tl);
    else load_k(tl, tile_offset(tn, more)); // K registers are free: fetch the tile that will use them next
    if (t == wave) MQA_STAMP(3);

    if (__builtin_expect(tail, 0)) {   // ragged end of the range / start of a window: drop positions outside [lo, end)
#pragma unroll
      for (int u = 0; u < 2; ++u)
#pragma unroll
        for (int r = 0; r < 4; ++r) {
          const int pos = p0 + 16 * u + 4 * r + g;
#pragma unroll
          for (int hb = 0; hb < HB; ++hb)
            if (pos >= min(end, lim[hb]) || pos < lo) sc[u][hb][r] = -INFINITY;
        }
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        const int pos = p0 + 4 * e + g;
        if (pos >= end || pos < lo) tl.vr[e] = u32x4{0u, 0u, 0u, 0u};
      }
    }

    // ---- online softmax per head block; weights packed as MFMA B operands
    u32x4 phi[HB], plo[HB];
#pragma unroll
    for (int hb = 0; hb < HB; ++hb) {
      float mx = fmaxf(fmaxf(fmaxf(sc[0][hb][0], sc[0][hb][1]), fmaxf(sc[0][hb][2], sc[0][hb][3])),
                       fmaxf(fmaxf(sc[1][hb][0], sc[1][hb][1]), fmaxf(sc[1][hb][2], sc[1][hb][3])));
      mx = fmaxf(mx, __shfl_xor(mx, 16));
      mx = fmaxf(mx, __shfl_xor(mx, 32));
      // The reference value the exponentials are taken against is only moved up when some row's
      // maximum has grown by more than 2^kSlack (lazy rescaling): weights then reach at most
      // 2^kSlack instead of 1, which float32 sums and the bf16 hi/lo split carry without loss,
      // and the 32 accumulator registers are rescaled on a few tiles only, not on most of them.
      // Any reference is a valid softmax state: the merges below only need (reference, sum, acc).
      const float mnew = fmaxf(m_run[hb], mx);
      if (__any(mnew > m_run[hb] + kSlack)) {
        // a causal row may have seen nothing yet (maximum still -inf): subtract 0 instead, so that
        // its weights come out as 2^(-inf) = 0 rather than 2^(-inf + inf)
        const float alpha = __builtin_amdgcn_exp2f(m_run[hb] - (mnew == -INFINITY ? 0.f : mnew));
        if (PSPLIT) l_run[hb] *= alpha;
        else accl[hb] *= alpha;
#pragma unroll
        for (int j = 0; j < 8; ++j) acc[hb][j] *= alpha;
        m_run[hb] = mnew;
      }
      const float mref = m_run[hb] == -INFINITY ? 0.f : m_run[hb];
      float pe[8];
      float sum = 0.f;
#pragma unroll
      for (int u = 0; u < 2; ++u)
#pragma unroll
        for (int r = 0; r < 4; ++r) {
          pe[4 * u + r] = __builtin_amdgcn_exp2f(sc[u][hb][r] - mref);
          if (PSPLIT) sum += pe[4 * u + r];
        }
      if (PSPLIT) l_run[hb] += sum;
#pragma unroll
      for (int d = 0; d < 4; ++d) {
        if (PSPLIT) {
          uint32_t hh, ll;
          split_pair(pe[2 * d], pe[2 * d + 1], hh, ll);
          phi[hb][d] = hh;
          plo[hb][d] = ll;
        } else {
          phi[hb][d] = pack_bf16(pe[2 * d], pe[2 * d + 1]);
        }
      }
      if (!PSPLIT) accl[hb] = mfma16(ones, phi[hb], accl[hb]);
    }

    // ---- O^T += V^T . P^T, V transposed 8x8 inside the lane
#pragma unroll
    for (int w = 0; w < 4; ++w) {
#pragma unroll
      for (int par = 0; par < 2; ++par) {
        const int j = 2 * w + par;
        u32x4 a;
#pragma unroll
        for (int x = 0; x < 4; ++x)
          a[x] = __builtin_amdgcn_perm(tl.vr[2 * x + 1][w], tl.vr[2 * x][w], par ? 0x07060302u : 0x05040100u);
#pragma unroll
        for (int hb = 0; hb < HB; ++hb) {
          acc[hb][j] = mfma16(a, phi[hb], acc[hb][j]);
          if (PSPLIT) acc[hb][j] = mfma16(a, plo[hb], acc[hb][j]);
        }
      }
    }
    if constexpr (!STAGE) load_v(tl, tile_offset(tn, more));
    if (t == wave) MQA_STAMP(4);
  };
  if constexpr (STAGE) {
    // Round r is read from LDS buffer r & 1 while round r+1 arrives in registers; it is stored into
    // the other buffer (last read in round r-1, which the barrier at the end of that round closed)
    // as soon as this wave is done with its tile, round r+2 is requested into the freed registers,
    // and one barrier ends the round.
    for (int r = 0; r < nrounds; ++r) {
      stage_k = stage0 + (r & 1) * (2 * kStageBytes);
      stage_v = stage_k + kStageBytes;
      const int t = 4 * r + wave;
      if (t < ntiles) {
        stage_read_k(tb);
        process(tb, t, ntiles);
      }
      if (r + 1 < nrounds) {
        stage_store((r + 1) & 1);
        issue_slot(r + 2);
        __syncthreads();
      }
    }
  } else {
    for (int t = wave; t < ntiles; t += NWT) process(tb, t, t + NWT);
  }
  MQA_STAMP(5);
  if constexpr (STAGE) {      // (assigned either way, so that no old value has to be carried through the rounds)
    load_q(seq_next, prefetched);
    L_next = prefetched ? sg.lens[seq_next / sg.lens_div] : 0;
  }

  // ---- merge a team's NWT wave states through LDS.  When one workgroup per CU is all that runs, the
  // merge buffers follow the q operands and a wave that finishes early writes its state without
  // waiting for the others; when several workgroups should share a CU the buffers re-use the
  // q region (after a barrier), which halves the LDS footprint.
  if (!PSPLIT) {              // each of a head's four lanes holds the whole sum: a quarter each for the merge below
#pragma unroll
    for (int hb = 0; hb < HB; ++hb) l_run[hb] = 0.25f * accl[hb][0];
  }
  if (p.merge_alias || TEAMS > 1) __syncthreads();
  constexpr int kMergeFloats = NWT * NH * kOPitch + 5 * NWT * NH;                        // per team
  float* so = reinterpret_cast<float*>(smem_raw + ((p.merge_alias || TEAMS > 1) ? 0 : QOPS * 16 * 2)) + team * kMergeFloats;   // [NWT][NH][kOPitch]
  float* sm = so + NWT * NH * kOPitch;                      // [NH][NWT]  running maxima
  float* sl = sm + NWT * NH;                                // [NH][NWT]  sums
  const int lane_m = here(lane), i16m = lane_m & 15, gm = lane_m >> 4;
#pragma unroll
  for (int hb = 0; hb < HB; ++hb) {
    float* row = so + ((size_t)wave * NH + 16 * hb + i16m) * kOPitch;
#pragma unroll
    for (int r = 0; r < 4; ++r) {
      float4 lo4 = make_float4(acc[hb][0][r], acc[hb][1][r], acc[hb][2][r], acc[hb][3][r]);
      float4 hi4 = make_float4(acc[hb][4][r], acc[hb][5][r], acc[hb][6][r], acc[hb][7][r]);
      float4* dst = reinterpret_cast<float4*>(row + 8 * (4 * gm + r));
      dst[0] = lo4;
      dst[1] = hi4;
    }
    // the four lanes of a head share one maximum and hold a quarter of the sum each
    float lq = l_run[hb];
    lq += __shfl_xor(lq, 16);
    lq += __shfl_xor(lq, 32);
    if (gm == 0) {
      sm[(16 * hb + i16m) * NWT + wave] = m_run[hb];
      sl[(16 * hb + i16m) * NWT + wave] = lq;
    }
  }
  __syncthreads();
  constexpr int ITERS = NH * (kD / 4) / NT;                   // float4 outputs per thread
  float fw[ITERS][NWT], lw[ITERS][NWT];
  float4 xw[ITERS][NWT];
  const int tid_m = here(tid);
#pragma unroll
  for (int it = 0; it < ITERS; ++it) {                        // all LDS reads first: one latency
    const int idx = tid_m + it * NT;
    const int hl = idx / (kD / 4), c4 = idx % (kD / 4);
    if constexpr (NWT == 4) {                                 // a head's four maxima and four sums: one read each
      const float4 m4 = *reinterpret_cast<const float4*>(sm + hl * 4);
      const float4 l4 = *reinterpret_cast<const float4*>(sl + hl * 4);
      fw[it][0] = m4.x; fw[it][1] = m4.y; fw[it][2] = m4.z; fw[it][3] = m4.w;
      lw[it][0] = l4.x; lw[it][1] = l4.y; lw[it][2] = l4.z; lw[it][3] = l4.w;
    } else {
#pragma unroll
      for (int w = 0; w < NWT; ++w) {
        fw[it][w] = sm[hl * NWT + w];
        lw[it][w] = sl[hl * NWT + w];
      }
    }
#pragma unroll
    for (int w = 0; w < NWT; ++w) xw[it][w] = reinterpret_cast<const float4*>(so + ((size_t)w * NH + hl) * kOPitch)[c4];
  }
#pragma unroll
  for (int it = 0; it < ITERS; ++it) {
    const int idx = tid_m + it * NT;
    const int hl = idx / (kD / 4), c4 = idx % (kD / 4);
    if (head0 + hl >= sg.G) continue;
    float M = -INFINITY;
#pragma unroll
    for (int w = 0; w < NWT; ++w) M = fmaxf(M, fw[it][w]);
    float4 a = make_float4(0.f, 0.f, 0.f, 0.f);
    float lsum = 0.f;
#pragma unroll
    for (int w = 0; w < NWT; ++w) {
      const float f = M == -INFINITY ? 0.f : __builtin_amdgcn_exp2f(fw[it][w] - M);   // (a row that saw nothing)
      const float4 x = xw[it][w];
      a.x += f * x.x; a.y += f * x.y; a.z += f * x.z; a.w += f * x.w;
      lsum += f * lw[it][w];
    }
    const int head = head0 + hl;
    if (p.PS == 0) {
      const float inv = lsum > 0.f ? 1.0f / lsum : 0.f;      // (a causal row with nothing to see: zeros)
      a.x *= inv; a.y *= inv; a.z *= inv; a.w *= inv;
      reinterpret_cast<float4*>(p.o + ((size_t)seq * sg.G + head) * kD)[c4] = a;
    } else {
      const size_t pidx = ((size_t)seq * sg.G + head) * p.PS + sg.slot0 + srange;
      reinterpret_cast<float4*>(p.part_o + pidx * kD)[c4] = a;
      if (c4 == 0) {
        p.part_m[pidx] = M;
        p.part_l[pidx] = lsum;
      }
    }
  }
  MQA_STAMP(6);
  if (!persist || seq_next < 0) break;
  __syncthreads();            // the merge buffers are read: the next sequence's q operands and first round may overwrite them
  seq = seq_next;
  Kbuf = k_rows_of(seq);
  Vbuf = v_rows_of(seq);
  }
}

template <int HB, int NW, bool STAGE = false, bool ROWS = false>
hipError_t launch_hb(const DecodeParams& p_in, int flags, hipStream_t st) {
  DecodeParams p = p_in;
  size_t nblocks = (p.order ? (size_t)((p.nseq + 7) / 8) * 8 : (size_t)p.nseq) * p.S * p.HG;
  if (!STAGE) p.persist = 0;
  if (p.persist > 0) nblocks = (size_t)p.persist;      // one workgroup per compute unit, several sequences each
  constexpr int TEAMS = STAGE ? 2 : ROWS ? NW : 1;
  constexpr int NWT = NW / TEAMS;
  p.merge_alias = (nblocks > 256 || TEAMS > 1) ? 1 : 0;      // more workgroups than CUs: keep LDS small
  const size_t q_bytes = (size_t)TEAMS * HB * 4 * 64 * 16 * 2;
  const size_t merge_bytes = (size_t)TEAMS * ((size_t)NWT * 16 * HB * kOPitch + 5 * NWT * 16 * HB) * sizeof(float);
  const size_t work_bytes = q_bytes + (STAGE ? 4 * 128 * kRowU4 * 16 : 0);     // q operands (+ two rounds of K and V)
  const size_t lds = p.merge_alias ? (work_bytes > merge_bytes ? work_bytes : merge_bytes) : work_bytes + merge_bytes;
  const size_t most = STAGE ? lds : q_bytes + merge_bytes;
  const dim3 grid((unsigned)nblocks), block(NW * 64);
  void (*kern)(DecodeParams);
  // Non-temporal loads unless the tiles are meant to be found in L2 by a second head group.
  const bool ntl = !(flags & 4) && (p.HG == 1 || STAGE) && !ROWS;
#define MQA_PICK(QS, PS) (ntl ? decode_mfma_kernel<HB, NW, QS, PS, true, false, STAGE, ROWS> : decode_mfma_kernel<HB, NW, QS, PS, false, false, STAGE, ROWS>)
  switch (flags & 3) {
    case 0: kern = MQA_PICK(true, true); break;
    case 1: kern = MQA_PICK(false, true); break;
    case 2: kern = MQA_PICK(true, false); break;
    default: kern = MQA_PICK(false, false); break;
  }
#undef MQA_PICK
  if (most > 64 * 1024) {     // opt in to more than 64 KiB of LDS, once per device and kernel variant
    static bool done[64][8] = {};
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) dev = 0;
    const int slot = (flags & 3) | (ntl ? 4 : 0);
    if (!done[dev][slot]) {
      hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                                         hipFuncAttributeMaxDynamicSharedMemorySize, (int)most);
      if (e != hipSuccess) return e;
      done[dev][slot] = true;
    }
  }
  hipLaunchKernelGGL(kern, grid, block, lds, st, p);
  return hipGetLastError();
}

}  // namespace

bool mfma_shape_ok(int G, int k, int v, int is_bf16, int cap) {
  (void)G;
  return is_bf16 && k == kD && v == kD && cap < (1 << 23);      // a sequence's cache is addressed with 31-bit byte offsets
}

// 16 or 32 heads per workgroup; more than 32 heads: the staged form with 64 heads per workgroup
// (plain decode and local attention), or groups of 32 (causal rows, or by a tuning flag)
int mfma_heads_per_block(int G, int flags, int causal) {
  if (causal && G > 32 && !(flags & 4096)) return 128;      // causal rows: four waves of 32 rows each
  return G <= 16 ? 16 : (G > 32 && !(flags & 8) && !causal) ? 64 : 32;
}

// The persistent form of the 64-head kernel applies to a ranked batch of more sequences than
// compute units with one range and one head group per sequence: returns the number of workgroups
// (one per compute unit), else 0.  *inline_rank: the kernel can rank the sequences itself.
int mfma_persistent_workgroups(int nseq, int G, int S, int HG, int window, int causal, int flags, int* inline_rank) {
  *inline_rank = 0;
  if (mfma_heads_per_block(G, flags, causal) != 64 || S != 1 || HG != 1 || window != 0 || (flags & 1024)) return 0;
  static int ncu[64] = {};
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) dev = 0;
  if (ncu[dev] == 0) {
    int n = 0;
    if (hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n <= 0) n = -1;
    ncu[dev] = n;
  }
  if (ncu[dev] <= 0 || nseq <= ncu[dev]) return 0;
  *inline_rank = (nseq <= kMaxInlineRanked && nseq <= kMaxTurns * ncu[dev] && !(flags & 2048)) ? 1 : 0;
  return ncu[dev];
}

hipError_t launch_decode_mfma_two(const DecodeParams& p_in, long long nblocks0, long long nblocks1, hipStream_t st) {
  constexpr int HB = 2, NW = 4;
  DecodeParams p = p_in;
  p.nblocks0 = (int)nblocks0;
  p.order = nullptr;
  p.merge_alias = 1;                          // small LDS footprint: two workgroups per CU
  const size_t q_bytes = (size_t)HB * 4 * 64 * 16 * 2;
  const size_t merge_bytes = ((size_t)NW * 16 * HB * kOPitch + 5 * NW * 16 * HB) * sizeof(float);
  const size_t lds = q_bytes > merge_bytes ? q_bytes : merge_bytes;        // 68.5 KiB
  // non-temporal loads unless some head group is meant to find its tiles in L2
  const bool ntl = p.HG == 1 && p.seg1.HG == 1;
  void (*kern)(DecodeParams) = ntl ? decode_mfma_kernel<HB, NW, true, true, true, true>
                                   : decode_mfma_kernel<HB, NW, true, true, false, true>;
  {                                           // opt in to more than 64 KiB of LDS, once per device and variant
    static bool done[64][2] = {};
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) dev = 0;
    if (!done[dev][ntl]) {
      hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                                         hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
      if (e != hipSuccess) return e;
      done[dev][ntl] = true;
    }
  }
  hipLaunchKernelGGL(kern, dim3((unsigned)(nblocks0 + nblocks1)), dim3(NW * 64), lds, st, p);
  return hipGetLastError();
}

hipError_t launch_decode_mfma(const DecodeParams& p, int flags, hipStream_t st) {
  const bool wide = (flags & 16) != 0;       // 8 waves per workgroup instead of 4
  const int hpb = mfma_heads_per_block(p.G, flags, p.causal_h > 0);
  // Short ranges (at most one tile per wave of a 4-wave workgroup) in a launch of many workgroups: 2 waves
  // per workgroup, so that more of them are resident and less of each one's time is the merge of its waves.
  const long long nblocks = (long long)p.nseq * p.S * p.HG;
  const bool narrow = (flags & 256) || (!(flags & 512) && !wide && p.chunk <= 128 && nblocks >= 512);
  if (hpb == 16 && narrow) return launch_hb<1, 2>(p, flags, st);
  if (hpb == 16) return wide ? launch_hb<1, 8>(p, flags, st) : launch_hb<1, 4>(p, flags, st);
  // the staged form is bound by its arithmetic, not by HBM: single-term weights unless asked otherwise
  if (hpb == 64) return launch_hb<2, 8, true>(p, (flags & 128) ? flags : (flags | 2), st);
  if (hpb == 128) return launch_hb<2, 4, false, true>(p, flags, st);
  return wide ? launch_hb<2, 8>(p, flags, st) : launch_hb<2, 4>(p, flags, st);
}

}  // namespace mqa
