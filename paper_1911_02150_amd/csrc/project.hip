// The four linear projections of the incremental listings (paper Section 2.4
// and Section 3): q = einsum('bd,hdk->bhk'), the new K / V rows
// einsum('bd,dk->bk') (multi-head: 'bd,hdk->bhk') and y = einsum('bhv,hdv->bd').
// float32 in, float32 products and accumulation on the matrix cores
// (v_mfma_f32_16x16x4_f32), float32 out.  The new K / V rows are the exception: their
// products (exact in float64) are accumulated in float64 (v_mfma_f64_16x16x4_f64) and the sum
// is rounded once to float32, so that the value then rounded into a bf16 cache is the correctly
// rounded projection and does not depend on the summation order (a float32 sum within an ulp
// of a bf16 tie would round either way, and one flipped cache element moves an attention
// output by up to a bf16 ulp of V).
//
// All four are one GEMM out[rows, N] = in[rows, C] . B[C, N] with B addressed
// inside the projection tensor P [h, d, kv]:
//   Q / KV / KV_MH : C = d,    N = h*kv, B[t, n]  = P[n/kv][t][n%kv]   (N contiguous)
//   O              : C = h*kv, N = d,    B[c, t]  = P[c/kv][t][c%kv]   (C contiguous)
//
// One workgroup of 8 waves per output tile of RB x CB MFMA blocks of 16x16 (16x16 ... 32x64).
// The contraction axis is cut into groups of 2 or 4 chunks of 16; wave w takes groups
// w, w+8, ... (one group in flight while the previous one is multiplied) and the eight partial
// tiles are summed through LDS.  With at most a few hundred rows these GEMMs are far from
// HBM-bound (the weights are read once); what limits them is the number of operand loads per
// MFMA, so operands are read straight from global memory (L2-resident) in MFMA layout and
// shared between the blocks of a tile:
//   A operand: lane (i, kk) holds in[row0+i][c0 + 4kk + e], e = 0..3 (one 16-byte load),
//              and MFMA e of the chunk contracts slots {c0+e, c0+4+e, c0+8+e, c0+12+e};
//   B operand: N contiguous: lane (kk, i) holds B[c0 + 4kk + e][n0 + CB*i + j], j < CB (four
//              loads of 4*CB bytes; column block j is every CB-th column);
//              C contiguous: lane (kk, i) holds B[c0 + 4kk + e][n0 + 16 j + i] (CB 16-byte loads).
#include "common.hpp"

namespace mqa {
namespace {


constexpr int NWAVES = 8;

// B operands of one group of GC chunks: w[e][s][j] is the weight of contraction slot 4kk + s of
// chunk e for column block j (N contiguous: CB adjacent columns per load) or v[e][j] the four
// slots of column block j (C contiguous: four adjacent contraction indices per load).
template <bool OUT_PROJ, int GC, int CB> struct BFrag;
template <int GC, int CB> struct BFrag<false, GC, CB> {
  typedef float __attribute__((ext_vector_type(CB))) vec;
  vec w[GC][4];
};
template <int GC> struct BFrag<false, GC, 1> {
  struct vec { float x; __device__ __forceinline__ float operator[](int) const { return x; } };
  vec w[GC][4];
};
template <int GC, int CB> struct BFrag<true, GC, CB> { float4 v[GC][CB]; };

// One (RB*T) x (CB*T) output tile of out = in . B: RB x CB MFMA blocks per wave that share the
// A operand along a block row and the B operand along a block column (RB + CB operand loads feed
// RB*CB MFMAs), left as NWAVES partial tiles in `red` (the caller sums them after the barrier
// this function ends with).  B is addressed inside P [h, C or N, kv]; n0 is the tile's first
// column (OUT_PROJ: of d; else of h*kv), rows / columns past the end are clamped and must be
// discarded by the caller.  Column blocks: with C contiguous (OUT_PROJ) block j is columns
// n0 + j*T + i; with N contiguous block j is columns n0 + CB*i + j, i = 0..T-1, so that a lane's
// CB weights of one contraction index are adjacent in memory and arrive in one load.
template <bool OUT_PROJ, int T, int RB, int CB, typename ACC = float>
__device__ __forceinline__ void gemm_tile(const float* __restrict__ in, const float* __restrict__ P,
                                          int rows, int d, int h, int kv, int row0, int n0,
                                          ACC (*red)[RB * T * CB * T]) {
  static_assert(sizeof(ACC) == 4 || T == 16, "float64 accumulation uses the 16x16x4 blocks");
  constexpr int TN = CB * T;
  constexpr int GC = (CB == 4) ? 2 : 4;        // chunks of contraction indices fetched together
  constexpr int CH = 256 / T;                  // contraction indices per chunk (4 per lane group)
  constexpr int NACC = T * T / 64;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int i32 = lane % T, kk = lane / T;
  const int C = OUT_PROJ ? h * kv : d;
  const int N = OUT_PROJ ? d : h * kv;
  const size_t head_stride = (size_t)d * kv;

  // A: this lane's row in each of the RB row blocks (clamped; rows past the end are discarded at the store)
  const float* arow[RB];
#pragma unroll
  for (int r = 0; r < RB; ++r) arow[r] = in + (size_t)min(row0 + r * T + i32, rows - 1) * C + 4 * kk;
  // B: this lane's output column(s), clamped likewise; shared by the row blocks.
  // OUT_PROJ: column n[j] of block j, contiguous along c;  else: CB adjacent columns from nb
  // (inside one head: kv and N are multiples of CB), stride kv along the contraction index
  int ncol[CB];
#pragma unroll
  for (int j = 0; j < CB; ++j) ncol[j] = min(n0 + j * T + i32, N - 1);
  const int nb = min(n0 + CB * i32, N - CB);
  const float* bcol = P + (size_t)(nb / kv) * head_stride + (nb % kv) + (size_t)(4 * kk) * kv;

  typedef __attribute__((ext_vector_type(NACC))) ACC accv;
  accv acc[RB][CB];
#pragma unroll
  for (int r = 0; r < RB; ++r)
#pragma unroll
    for (int j = 0; j < CB; ++j)
#pragma unroll
      for (int e = 0; e < NACC; ++e) acc[r][j][e] = ACC(0);

  const int nchunks = C / CH;                  // C is a multiple of 8; a last half chunk (T = 16) is handled below
  const int tail = C - nchunks * CH;           // 0 or 8 (only when T = 16)
  const int ngroups = (nchunks + (tail ? 1 : 0) + GC - 1) / GC;
  typedef BFrag<OUT_PROJ, GC, CB> bfrag;
  auto load_group = [&](int grp, float4 (&a)[RB][GC], bfrag& b) {
#pragma unroll
    for (int e = 0; e < GC; ++e) {
      const int chunk = grp * GC + e;
      // the last, half-filled chunk of a 16-wide contraction: only lane groups kk < 2 hold data
      if (chunk < nchunks || (chunk == nchunks && tail && kk < 2)) {
        const int c0 = chunk * CH;
#pragma unroll
        for (int r = 0; r < RB; ++r) a[r][e] = *reinterpret_cast<const float4*>(arow[r] + c0);
        if constexpr (OUT_PROJ) {
          const int c = c0 + 4 * kk;                 // 4 consecutive c stay inside one head (kv % 8 == 0)
          const float* bp = P + (size_t)(c / kv) * head_stride + (c % kv);
#pragma unroll
          for (int j = 0; j < CB; ++j) b.v[e][j] = *reinterpret_cast<const float4*>(bp + (size_t)ncol[j] * kv);
        } else {
          const float* bp = bcol + (size_t)c0 * kv;
#pragma unroll
          for (int s = 0; s < 4; ++s) b.w[e][s] = *reinterpret_cast<const typename bfrag::vec*>(bp + s * (size_t)kv);
        }
      } else {
#pragma unroll
        for (int r = 0; r < RB; ++r) a[r][e] = make_float4(0.f, 0.f, 0.f, 0.f);
        if constexpr (OUT_PROJ) {
#pragma unroll
          for (int j = 0; j < CB; ++j) b.v[e][j] = make_float4(0.f, 0.f, 0.f, 0.f);
        } else {
#pragma unroll
          for (int s = 0; s < 4; ++s) b.w[e][s] = typename bfrag::vec{};
        }
      }
    }
  };
  auto mfma = [&](float x, float y, accv c) -> accv {
    if constexpr (sizeof(ACC) == 8) return __builtin_amdgcn_mfma_f64_16x16x4f64((double)x, (double)y, c, 0, 0, 0);
    else if constexpr (T == 32) return __builtin_amdgcn_mfma_f32_32x32x2f32(x, y, c, 0, 0, 0);
    else return __builtin_amdgcn_mfma_f32_16x16x4f32(x, y, c, 0, 0, 0);
  };
  auto multiply = [&](const float4 (&a)[RB][GC], const bfrag& b) {
#pragma unroll
    for (int e = 0; e < GC; ++e)
#pragma unroll
      for (int r = 0; r < RB; ++r)
#pragma unroll
        for (int j = 0; j < CB; ++j) {
          if constexpr (OUT_PROJ) {
            acc[r][j] = mfma(a[r][e].x, b.v[e][j].x, acc[r][j]);
            acc[r][j] = mfma(a[r][e].y, b.v[e][j].y, acc[r][j]);
            acc[r][j] = mfma(a[r][e].z, b.v[e][j].z, acc[r][j]);
            acc[r][j] = mfma(a[r][e].w, b.v[e][j].w, acc[r][j]);
          } else {
            acc[r][j] = mfma(a[r][e].x, b.w[e][0][j], acc[r][j]);
            acc[r][j] = mfma(a[r][e].y, b.w[e][1][j], acc[r][j]);
            acc[r][j] = mfma(a[r][e].z, b.w[e][2][j], acc[r][j]);
            acc[r][j] = mfma(a[r][e].w, b.w[e][3][j], acc[r][j]);
          }
        }
  };

  float4 a0[RB][GC], a1[RB][GC];
  bfrag b0, b1;
  int grp = wave;
  if (grp < ngroups) load_group(grp, a0, b0);
  while (grp < ngroups) {
    if (grp + NWAVES < ngroups) load_group(grp + NWAVES, a1, b1);
    multiply(a0, b0);
    grp += NWAVES;
    if (grp >= ngroups) break;
    if (grp + NWAVES < ngroups) load_group(grp + NWAVES, a0, b0);
    multiply(a1, b1);
    grp += NWAVES;
  }

  // D layout: register e of lane (i, g) is block element (8*(e/4) + 4*g + e%4, i) for the 32x32
  // block, (4*g + e, i) for the float32 16x16 block and (4*e + g, i) for the float64 16x16 block
  // (whose four result registers interleave the lane groups' rows); row block r adds r*T rows,
  // column block j maps to tile columns as described above
#pragma unroll
  for (int r = 0; r < RB; ++r)
#pragma unroll
    for (int j = 0; j < CB; ++j)
#pragma unroll
      for (int e = 0; e < NACC; ++e) {
        const int trow = r * T + ((T == 32) ? (8 * (e >> 2) + 4 * kk + (e & 3)) : sizeof(ACC) == 8 ? (4 * e + kk) : (4 * kk + e));
        const int tcol = OUT_PROJ ? j * T + i32 : CB * i32 + j;
        red[wave][trow * TN + tcol] = acc[r][j][e];
      }
  __syncthreads();
}

template <typename ACC>
__device__ __forceinline__ float sum_partials(const ACC* red0, int e, int stride) {
  return (float)(((red0[e] + red0[stride + e]) + (red0[2 * stride + e] + red0[3 * stride + e])) +
                 ((red0[4 * stride + e] + red0[5 * stride + e]) + (red0[6 * stride + e] + red0[7 * stride + e])));
}

// T = 16: 16x16 MFMA blocks (v_mfma_f32_16x16x4_f32, chunks of 16 contraction indices), the
// ones launched; T = 32: 32x32 blocks (v_mfma_f32_32x32x2_f32, chunks of 8).  A workgroup owns
// an (RB*T) x (CB*T) output tile.  Lane (i, kk): i = lane % T, kk = lane / T.
template <bool OUT_PROJ, int T, int RB, int CB, typename ACC = float>
__global__ __launch_bounds__(NWAVES * 64)
void project_mfma_kernel(const float* __restrict__ in, const float* __restrict__ P, float* out,
                         int rows, int d, int h, int kv, int epilogue) {
  constexpr int TM = RB * T, TN = CB * T;
  __shared__ ACC red[NWAVES][TM * TN];
  const int N = OUT_PROJ ? d : h * kv;
  const int row0 = blockIdx.y * TM, n0 = blockIdx.x * TN;
  gemm_tile<OUT_PROJ, T, RB, CB, ACC>(in, P, rows, d, h, kv, row0, n0, red);
  for (int e = threadIdx.x; e < TM * TN; e += NWAVES * 64) {
    const int r = e / TN, c = e % TN;
    if (row0 + r < rows && n0 + c < N) {
      float* dst = out + (size_t)(row0 + r) * N + n0 + c;
      *dst = apply_epilogue(sum_partials(&red[0][0], e, TM * TN), dst, epilogue);
    }
  }
}

template <typename CT> __device__ __forceinline__ CT cache_value(float x);
template <> __device__ __forceinline__ float cache_value<float>(float x) { return x; }
template <> __device__ __forceinline__ uint16_t cache_value<uint16_t>(float x) { return (uint16_t)float_to_bf16_rne(x); }

// The first three lines of the incremental listings in one launch: q = x . P_q to memory, the
// new K and V rows x . P_k, x . P_v straight into row lens_in[i] of the caches (accumulated in
// float64, rounded once to float32 and then to the cache type), and lens_out[i] = lens_in[i] + 1.
// Column tiles are numbered over q's h*k columns, then K's h_kv*k, then V's h_kv*v (k and v are
// multiples of the tile width, so a tile belongs to one of them); the launch covers the tiles from
// tile0 on (tile0 > 0: q was computed by another launch).  A K or V tile is worked off one row
// block at a time so that its float64 partial tiles fit the same LDS as a q tile's float32 ones.
// A sequence at capacity keeps its cache and its length.
// mem_rows > 0 is the form for a whole memory (encoder-decoder attention: the memory M of the
// Section 2.2 listing, projected once): input row r is row r % mem_rows of sequence r / mem_rows
// and goes to that position of the cache; lens_in, if given, holds the number of valid memory
// rows per sequence, and lens_out receives it clamped to [0, mem_rows] (mem_rows if not given).
template <int T, int RB, int CB, typename CT>
__global__ __launch_bounds__(NWAVES * 64)
void project_qkv_append_kernel(const float* __restrict__ x, const float* __restrict__ P_q,
                               const float* __restrict__ P_k, const float* __restrict__ P_v,
                               float* __restrict__ q, CT* __restrict__ K, CT* __restrict__ V,
                               const int32_t* __restrict__ lens_in, int32_t* __restrict__ lens_out,
                               int rows, int d, int h, int h_kv, int cap, int k, int v, int nq_tiles, int kv_narrow,
                               int mem_rows) {
  constexpr int TM = RB * T, TN = CB * T;
  __shared__ __align__(16) double red_raw[NWAVES * T * TN];       // = RB <= 2 float32 row blocks
  static_assert(RB <= 2, "a q tile's float32 partial tiles must fit the float64 buffer");
  const int row0 = blockIdx.y * TM;
  const int nq = h * k, nk = h_kv * k;
  if ((int)blockIdx.x < nq_tiles) {    // a tile of q
    const int n0 = blockIdx.x * TN;
    float (*red)[TM * TN] = reinterpret_cast<float (*)[TM * TN]>(red_raw);
    gemm_tile<false, T, RB, CB>(x, P_q, rows, d, h, k, row0, n0, red);
    for (int e = threadIdx.x; e < TM * TN; e += NWAVES * 64) {
      const int r = e / TN, c = e % TN;
      if (row0 + r < rows) q[(size_t)(row0 + r) * nq + n0 + c] = sum_partials(&red[0][0], e, TM * TN);
    }
    return;
  }
  // A tile of the K or V rows.  Their float64 products run at half the matrix rate, so for few
  // rows (a decode step) the tiles are a single block of 16 columns wide: four times the
  // workgroups, a quarter of the time each; for many rows (a prompt) they keep the q tiles' width
  // and with it the re-use of the input rows.
  const int kvt = blockIdx.x - nq_tiles;
  const int width = kv_narrow ? T : TN;
  int n0 = kvt * width;
  const int which = n0 >= nk ? 2 : 1;      // 1: K row, 2: V row
  if (which == 2) n0 -= nk;
  const int kv = which == 2 ? v : k;
  CT* dst = which == 1 ? K : V;
  const float* P = which == 1 ? P_k : P_v;
  for (int rb = 0; rb < RB && row0 + rb * T < rows; ++rb) {
    if (rb) __syncthreads();           // the previous row block's sums have been read
    if (kv_narrow) gemm_tile<false, T, 1, 1, double>(x, P, rows, d, h_kv, kv, row0 + rb * T, n0, reinterpret_cast<double (*)[T * T]>(red_raw));
    else gemm_tile<false, T, 1, CB, double>(x, P, rows, d, h_kv, kv, row0 + rb * T, n0, reinterpret_cast<double (*)[T * TN]>(red_raw));
    for (int e = threadIdx.x; e < T * width; e += NWAVES * 64) {
      const int row = row0 + rb * T + e / width, n = n0 + e % width;
      if (row >= rows) continue;
      const int seq = mem_rows > 0 ? row / mem_rows : row;
      const int L = mem_rows > 0 ? row - seq * mem_rows : lens_in[row];
      if (L < 0 || L >= cap) continue;
      dst[(((size_t)seq * h_kv + n / kv) * cap + L) * kv + (n % kv)] = cache_value<CT>(sum_partials(red_raw, e, T * width));
    }
  }
  if (kvt == 0 && threadIdx.x < TM && row0 + threadIdx.x < rows) {      // the first K tile of each row tile
    const int row = row0 + threadIdx.x;
    if (mem_rows > 0) {
      if (row % mem_rows == 0) {
        const int L = lens_in ? lens_in[row / mem_rows] : mem_rows;
        lens_out[row / mem_rows] = L < 0 ? 0 : (L > mem_rows ? mem_rows : L);
      }
    } else {
      const int L = lens_in[row];
      lens_out[row] = (L < 0 || L >= cap) ? L : L + 1;
    }
  }
}

}  // namespace

// Tile shapes of the split-contraction kernel: 16x16 MFMA blocks, RB x CB of them per wave.
// Larger tiles need fewer operand loads per MFMA (the kernel is bound by the rate of L1 / L2
// accesses, not by the matrix cores) but give fewer workgroups; the widest tile that still gives
// about 160 workgroups wins at the decode-sized shapes measured (rows = 128, contraction x
// columns, microseconds 16x16 -> chosen tile): 1024 x 4096: 33.9 -> 17.3 (32x64); 4096 x 1024:
// 29.5 -> 22.9 (16x32); 1024 x 1024: 9.5 -> 7.8 (16x32); fused q/K/V 1024 x 1280: 12.2 -> 10.3
// (16x64), multi-head 1024 x 3072: 21.8 -> 17.6 (32x64).  A second row block only pays when it
// holds real rows (rows > 16).  32x32 MFMA blocks (T = 32, which gemm_tile also supports) were
// slower than these at every such shape (1024 x 4096: 21.4) and are not instantiated.
struct Tile { int RB, CB; };
static inline long long tiles_of(const Tile& t, long long ncols, int rows) {
  const long long tm = t.RB * 16, tn = t.CB * 16;
  return ((ncols + tn - 1) / tn) * ((rows + tm - 1) / tm);
}
// colmult: the column width (in floats) that a tile must divide (the fused q/K/V launch: tiles
// must not straddle q / K / V; else 0)
static Tile pick_tile(long long ncols, int rows, int colmult) {
  static const Tile order[] = {{2, 4}, {1, 4}, {2, 2}, {1, 2}, {2, 1}, {1, 1}};
  for (const Tile& t : order) {
    if (t.RB == 2 && rows <= 16) continue;
    if (colmult && (colmult % (t.CB * 16))) continue;
    if (tiles_of(t, ncols, rows) >= 160) return t;
  }
  return (colmult && (colmult % 16)) ? Tile{0, 0} : Tile{1, 1};
}

#define MQA_TILES(X) X(2, 4) X(1, 4) X(2, 2) X(1, 2) X(2, 1) X(1, 1)

hipError_t launch_project(int mode, const float* in, const float* P, float* out,
                          int rows, int d, int h, int kv, int epilogue, hipStream_t st) {
  const bool outp = (mode == 3);
  const bool f64 = (mode == 1 || mode == 2);        // new K / V rows: float64 accumulation, split-contraction kernel only
  if (!f64) {
    const hipError_t big = launch_gemm_tiled(mode, in, P, out, rows, d, h, kv, epilogue, st);     // large GEMMs: LDS-tiled kernel
    if (big != hipErrorNotSupported) return big;
  }
  const int N = outp ? d : h * kv;
  const dim3 block(NWAVES * 64);
  Tile t = pick_tile(N, rows, 0);
  if (f64 && t.RB == 2 && t.CB == 4) t = Tile{1, 4};        // float64 partial tiles: at most 1024 elements in 64 KiB of LDS
  bool launched = false;
#define MQA_PROJ(RB_, CB_)                                                                                           \
  if (!launched && t.RB == RB_ && t.CB == CB_) {                                                                     \
    const dim3 grid((N + CB_ * 16 - 1) / (CB_ * 16), (rows + RB_ * 16 - 1) / (RB_ * 16));                            \
    if (outp) hipLaunchKernelGGL((project_mfma_kernel<true, 16, RB_, CB_>), grid, block, 0, st, in, P, out, rows, d, h, kv, epilogue); \
    else if (!f64) hipLaunchKernelGGL((project_mfma_kernel<false, 16, RB_, CB_>), grid, block, 0, st, in, P, out, rows, d, h, kv, epilogue); \
    else if constexpr (RB_ * CB_ <= 4)                                                                               \
      hipLaunchKernelGGL((project_mfma_kernel<false, 16, RB_, CB_, double>), grid, block, 0, st, in, P, out, rows, d, h, kv, epilogue); \
    launched = true;                                                                                                 \
  }
  MQA_TILES(MQA_PROJ)
#undef MQA_PROJ
  if (!launched) return hipErrorInvalidValue;
  return hipGetLastError();
}

hipError_t launch_project_qkv_append(const float* x, const float* P_q, const float* P_k, const float* P_v,
                                     float* q, void* K, void* V, const int32_t* lens_in, int32_t* lens_out,
                                     int rows, int d, int h, int h_kv, int cap, int k, int v, int is_bf16,
                                     int mem_rows, hipStream_t st) {
  // prompt-sized row counts: q through the LDS-tiled kernel, then only the K / V columns here
  // (h = 0: no q at all, the projection of a memory)
  const hipError_t big = h > 0 ? launch_gemm_tiled(0, x, P_q, q, rows, d, h, k, 0, st) : hipErrorNotSupported;
  if (big != hipErrorNotSupported && big != hipSuccess) return big;
  const bool q_done = (big == hipSuccess);
  const int nq = h * k;
  const int ntot = nq + h_kv * (k + v);
  // column tiles must not straddle q / K / V: the tile width divides k and v (both multiples of 16)
  int g = k, r = v;
  while (r) { const int t2 = g % r; g = r; r = t2; }
  const Tile t = pick_tile(q_done ? ntot - nq : ntot, rows, g);
  // a decode step's rows and K / V columns that are a small part of the product (multi-query): K / V tiles of
  // 16 columns (b=128, h=8: 14.2 -> 10.4 us; multi-head, where they are two thirds of it: 25.9 -> 31.6 us, so not there)
  const int kv_narrow = (rows <= 512 && 2 * (ntot - nq) <= nq) ? 1 : 0;
  const dim3 block(NWAVES * 64);
  bool launched = false;
#define MQA_QKV(RB_, CB_)                                                                                            \
  if (!launched && t.RB == RB_ && t.CB == CB_) {                                                                     \
    const int nq_tiles = q_done ? 0 : nq / (CB_ * 16);                                                               \
    const dim3 grid(nq_tiles + (ntot - nq) / (kv_narrow ? 16 : CB_ * 16), (rows + RB_ * 16 - 1) / (RB_ * 16));       \
    if (is_bf16) hipLaunchKernelGGL((project_qkv_append_kernel<16, RB_, CB_, uint16_t>), grid, block, 0, st, x, P_q, P_k, P_v, q, \
                                    (uint16_t*)K, (uint16_t*)V, lens_in, lens_out, rows, d, h, h_kv, cap, k, v, nq_tiles, kv_narrow, mem_rows); \
    else hipLaunchKernelGGL((project_qkv_append_kernel<16, RB_, CB_, float>), grid, block, 0, st, x, P_q, P_k, P_v, q, \
                            (float*)K, (float*)V, lens_in, lens_out, rows, d, h, h_kv, cap, k, v, nq_tiles, kv_narrow, mem_rows);  \
    launched = true;                                                                                                 \
  }
  MQA_TILES(MQA_QKV)
#undef MQA_QKV
  if (!launched) return hipErrorInvalidValue;
  return hipGetLastError();
}

}  // namespace mqa
