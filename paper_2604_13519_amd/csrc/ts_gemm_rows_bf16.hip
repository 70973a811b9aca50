// Many-row projection of a bf16 model for gfx950:  out[r][n] = sum_k X[r][k] * W[n][k]  for R > 80 rows
// (batched verification: the rows of all requests of a pass share one weight stream).
//
// With hundreds of rows the projection is no longer a weight stream but a matrix-core problem:
// every weight fragment is multiplied with R / 16 activation fragments.  The kernel keeps the
// arithmetic (IEEE half x half -> fp32) and the data path of the skinny kernel - weights
// pre-tiled in MFMA operand order and loaded straight from global memory into registers,
// activations shared through a double-buffered LDS chunk - and changes the tile a wave owns:
//  * 4 tiles of 16 output features per wave (the skinny kernel has 2).  One 1 KiB activation
//    fragment read from LDS then feeds 4 MFMAs, 64 matrix-pipe cycles against 8 LDS-pipe
//    cycles; with 8 waves the LDS pipe is half as busy as the four matrix pipes.
//  * 4 to 8 row tiles (up to 128 rows) per workgroup.  The rows of a pass are cut into equal
//    row blocks; the row blocks of one weight slab get consecutive places on the same XCD, so that
//    the slab comes from HBM once and from that XCD's L2 for the other blocks.
//  * 8 waves as CS column sets x KW k-waves (8x1: 512 columns, 4x2: 256, 2x4: 128) plus K
//    splits across workgroups; the planner takes the combination with the fewest rounds of
//    workgroups over the CUs.  The k-waves of a column set add their accumulators through LDS,
//    one row tile at a time, in the order kq = 0, 1, ...; K splits write fp32 partial sums
//    [split][row][col] for the next row-wise kernel (deterministic, no atomics).
//  * gate/up variant (SWIGLU): gate and up tiles alternate, a wave holds two (gate, up) pairs
//    and the epilogue stores SiLU(gate) * up as half.
//  * lm_head variant (ARGMAX, 8x1 only, no K split): the epilogue reduces each row's maximum over
//    the workgroup's 512 columns and emits one (value, index) partial per row and column group.
#include "ts_internal.h"
#include "ts_device_utils.h"
#include <algorithm>
#include <type_traits>

typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

namespace {

struct RowsArgs {
  const f16_t* X;      // [2 planes][x_rows][K] IEEE half (x = hi + lo)
  size_t x_plane;      // elements between the planes
  size_t act_plane;    // SWIGLU: elements between the planes of act_out
  unsigned long long* sat;   // counts gated products beyond half's range
  int x_rows;          // rows allocated (reads are clamped to them)
  const f16_t* Wt;     // tiled weights, IEEE half
  float* out;          // [split][R][N] partial sums
  f16_t* act_out;      // SWIGLU: [x_rows][N/2] IEEE half
  float* logits;       // ARGMAX: [R][N] or nullptr
  float* aval;         // ARGMAX: [R][amax_stride] partial maxima, one per column group
  int32_t* aidx;
  int amax_stride;
  int R, N, K;
  int kper;            // k elements per split
  int n_tiles;         // ceil(N / 16)
  int kt_count;        // K / 32
  size_t split_stride; // R * N
  int n_groups;        // column groups
  int n_units;         // column groups x K splits: one weight slab each
  int n_rblocks;       // row blocks
};

enum { MODE_PARTIAL = 0, MODE_ARGMAX = 1, MODE_SWIGLU = 2 };
constexpr int NT = 4;        // tiles of 16 output features per wave
constexpr int WAVES = 8;

template <int MT, int CS, int KW, int MODE>
__global__ __launch_bounds__(64 * WAVES) void k_gemm_rows_bf16(RowsArgs a) {
  static_assert(CS * KW == WAVES, "8 waves");
  static_assert(MODE != MODE_ARGMAX || KW == 1, "the arg-max epilogue expects one wave per column set");
  constexpr int KC = KW * 32;             // k elements per staged chunk: one k-step per wave
  constexpr int KSTEPS = KC / 32;
  constexpr int KSW = KSTEPS / KW;          // k-steps of a chunk this wave multiplies
  static_assert(KSW >= 1 && KSW * KW == KSTEPS, "k-steps of a chunk divide among the k-waves");
  constexpr int XS = KC + 8;                // LDS row stride in elements (+16 B: bank spread)
  constexpr int NTHR = 64 * WAVES;
  constexpr int PL = TS_ACT_PLANES;         // an activation is the sum of a hi and a lo half
  constexpr int XVP = MT * 16 * KC / 8;     // 16-byte vectors per plane of a chunk
  constexpr int XV = PL * XVP;
  constexpr int XPT = (XV + NTHR - 1) / NTHR;
  constexpr size_t XS_BYTES = sizeof(f16_t) * 2 * PL * MT * 16 * XS;
  constexpr size_t RED_BYTES = KW > 1 ? sizeof(float) * WAVES * 4 * NT * 64 : 0;   // the reduction reuses the activation buffers
  constexpr size_t AMAX_BYTES = MODE == MODE_ARGMAX ? (size_t)8 * WAVES * MT * 16 : 0;
  constexpr size_t SMEM_BYTES = XS_BYTES > RED_BYTES ? (XS_BYTES > AMAX_BYTES ? XS_BYTES : AMAX_BYTES) : (RED_BYTES > AMAX_BYTES ? RED_BYTES : AMAX_BYTES);
  __shared__ __attribute__((aligned(16))) char smem[SMEM_BYTES];
  f16_t (*xs)[PL][MT * 16][XS] = reinterpret_cast<f16_t (*)[PL][MT * 16][XS]>(smem);

  // place: XCD = blockIdx.x % 8; the row blocks of a weight slab follow each other on one XCD
  const int xcd = blockIdx.x & 7, rest = blockIdx.x >> 3;
  const int rb = rest % a.n_rblocks;
  const int unit = (rest / a.n_rblocks) * 8 + xcd;
  if (unit >= a.n_units) return;
  const int group = unit % a.n_groups, split = unit / a.n_groups;

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int l15 = lane & 15, g = lane >> 4;
  const int cs = wave / KW, kq = wave % KW;
  const int row0 = rb * (MT * 16);
  const int kbase0 = split * a.kper;
  const int n_chunks = a.kper / KC;

  const int cs_u = __builtin_amdgcn_readfirstlane(cs), kq_u = __builtin_amdgcn_readfirstlane(kq);
  const char* wbase[NT];
  int nt_idx[NT];
#pragma unroll
  for (int t = 0; t < NT; ++t) {
    nt_idx[t] = (group * CS + cs_u) * NT + t;
    const int c = nt_idx[t] < a.n_tiles ? nt_idx[t] : a.n_tiles - 1;   // idle waves re-read a valid tile
    wbase[t] = reinterpret_cast<const char*>(a.Wt) + ((size_t)c * a.kt_count + kbase0 / 32 + kq_u * KSW) * 1024;
  }
  const uint32_t w_lane = lane * 16;
  const char* xbase = reinterpret_cast<const char*>(a.X) + (size_t)kbase0 * 2;
  uint32_t x_off[XPT];                      // byte offset of each staged vector within a chunk
#pragma unroll
  for (int p = 0; p < XPT; ++p) {
    const int v = min(tid + p * NTHR, XV - 1);
    const int pl = v / XVP, row = min(row0 + (v % XVP) / (KC / 8), a.x_rows - 1), cv = v % (KC / 8);
    x_off[p] = (uint32_t)((pl * a.x_plane + (size_t)row * a.K + cv * 8) * 2);
  }

  f32x4 acc[MT][NT];
#pragma unroll
  for (int mt = 0; mt < MT; ++mt)
#pragma unroll
    for (int t = 0; t < NT; ++t) acc[mt][t] = f32x4{0.f, 0.f, 0.f, 0.f};

  // Pipeline depth.  With one workgroup per CU (2 waves per SIMD) the loads need more than one
  // chunk of matrix-core time to arrive: weights travel RD - 1 chunks ahead in a register ring,
  // activations XD chunks ahead in registers and one chunk ahead in LDS.  The 4-row-tile kernels
  // that run two workgroups per CU keep the short pipeline (their register budget is half).
  constexpr int RD = (MT <= 4 && KW <= 2) ? 2 : 4;
  constexpr int XD = (RD == 4 && KW == 1) ? 2 : 1;
  f16x8 w[RD][NT][KSW];
  u32x4 xr[XD][XPT];
  const int last_chunk = n_chunks - 1;

  // loads are never predicated (a load under an `if` would make every later wait a wait for
  // everything): past the end they re-request the last chunk
  auto load_w = [&](f16x8 (&dst)[NT][KSW], int chunk) {
    const size_t off = (size_t)min(chunk, last_chunk) * (KSTEPS * 1024);
#pragma unroll
    for (int t = 0; t < NT; ++t)
#pragma unroll
      for (int j = 0; j < KSW; ++j)
        dst[t][j] = *reinterpret_cast<const f16x8*>(wbase[t] + off + w_lane + j * 1024);
  };
  auto load_x = [&](u32x4 (&dst)[XPT], int chunk) {
    const char* xb = xbase + (size_t)min(chunk, last_chunk) * (KC * 2);
#pragma unroll
    for (int p = 0; p < XPT; ++p) dst[p] = *reinterpret_cast<const u32x4*>(xb + x_off[p]);
  };
  auto store_x = [&](const u32x4 (&src)[XPT], int buf) {
#pragma unroll
    for (int p = 0; p < XPT; ++p) {
      const int v = tid + p * NTHR;
      if (XV % NTHR == 0 || v < XV)
        *reinterpret_cast<u32x4*>(&xs[buf][v / XVP][(v % XVP) / (KC / 8)][(v % (KC / 8)) * 8]) = src[p];
    }
  };
  auto mma_chunk = [&](const f16x8 (&wc)[NT][KSW], int buf) {
#pragma unroll
    for (int ks = 0; ks < KSW; ++ks) {
      const int kk = (kq * KSW + ks) * 32 + g * 8;
#pragma unroll
      for (int mt = 0; mt < MT; ++mt) {
#pragma unroll
        for (int pl = 0; pl < PL; ++pl) {
          const f16x8 xa = *reinterpret_cast<const f16x8*>(&xs[buf][pl][mt * 16 + l15][kk]);
#pragma unroll
          for (int t = 0; t < NT; ++t) acc[mt][t] = __builtin_amdgcn_mfma_f32_16x16x32_f16(xa, wc[t][ks], acc[mt][t], 0, 0, 0);
        }
      }
    }
  };
  // Step c (I = c % RD at compile time).  On entry: weights of chunks c .. c+RD-2 requested,
  // activations of chunk c in LDS buffer c % 2, of chunks c+1 .. c+XD-1 requested into registers.
  auto step = [&](auto i_c, int c) {
    constexpr int I = decltype(i_c)::value;
    load_x(xr[I % XD], c + XD);
    load_w(w[(I + RD - 1) % RD], c + RD - 1);
    mma_chunk(w[I], I & 1);
    store_x(xr[(I + 1) % XD], (I + 1) & 1);
    __syncthreads();
  };

#pragma unroll
  for (int i = 0; i < XD; ++i) load_x(xr[i], i);
#pragma unroll
  for (int i = 0; i < RD - 1; ++i) load_w(w[i], i);
  store_x(xr[0], 0);
  __syncthreads();
  int c0 = 0;
  for (; c0 + RD <= n_chunks; c0 += RD) {
    step(std::integral_constant<int, 0>{}, c0);
    step(std::integral_constant<int, 1>{}, c0 + 1);
    if (RD == 4) {
      step(std::integral_constant<int, 2 % RD>{}, c0 + 2);
      step(std::integral_constant<int, 3 % RD>{}, c0 + 3);
    }
  }
  if (c0 < n_chunks) step(std::integral_constant<int, 0>{}, c0);
  if (RD == 4) {
    if (c0 + 1 < n_chunks) step(std::integral_constant<int, 1>{}, c0 + 1);
    if (c0 + 2 < n_chunks) step(std::integral_constant<int, 2 % RD>{}, c0 + 2);
  }

  if (MODE == MODE_ARGMAX) {
    // per row: maximum over the wave's 64 columns (in-lane over the 4 tiles, then over the 16
    // lanes of the row), then over the 8 waves through LDS (free after the loop's last barrier)
    float* rv = reinterpret_cast<float*>(smem);                    // [WAVES][MT * 16]
    int* ri = reinterpret_cast<int*>(smem) + WAVES * MT * 16;
#pragma unroll
    for (int mt = 0; mt < MT; ++mt)
#pragma unroll
      for (int r = 0; r < 4; ++r) {
        const int row = row0 + mt * 16 + g * 4 + r;
        float bv = -INFINITY;
        int bi = 0x7fffffff;
#pragma unroll
        for (int t = 0; t < NT; ++t) {
          const int col = nt_idx[t] * 16 + l15;
          if (nt_idx[t] < a.n_tiles && col < a.N) {
            const float v = acc[mt][t][r];
            if (a.logits != nullptr && row < a.R) a.logits[(size_t)row * a.N + col] = v;
            amax_take(bv, bi, v, col);
          }
        }
#pragma unroll
        for (int o = 8; o > 0; o >>= 1) {
          const float ov = __shfl_xor(bv, o, 64);
          const int oi = __shfl_xor(bi, o, 64);
          amax_take(bv, bi, ov, oi);
        }
        if (l15 == 0) { rv[wave * (MT * 16) + mt * 16 + g * 4 + r] = bv; ri[wave * (MT * 16) + mt * 16 + g * 4 + r] = bi; }
      }
    __syncthreads();
    if (tid < MT * 16 && row0 + tid < a.R) {
      float bv = rv[tid];
      int bi = ri[tid];
      for (int wv = 1; wv < WAVES; ++wv) amax_take(bv, bi, rv[wv * (MT * 16) + tid], ri[wv * (MT * 16) + tid]);
      a.aval[(size_t)(row0 + tid) * a.amax_stride + group] = bv;
      a.aidx[(size_t)(row0 + tid) * a.amax_stride + group] = bi;
    }
    return;
  }

  // value of output (row tile mt, row r of the lane group, tile t) goes to memory
  auto emit = [&](int mt, int r, const float (&v)[NT]) {
    const int row = row0 + mt * 16 + g * 4 + r;
    if (row >= a.R) return;
    if (MODE == MODE_SWIGLU) {
#pragma unroll
      for (int t = 0; t < NT; t += 2) {       // tiles 2j / 2j+1 = gate / up of features 16j..
        if (nt_idx[t + 1] < a.n_tiles) {
          const int f = (nt_idx[t] >> 1) * 16 + l15;
          const float gv = v[t], uv = v[t + 1];
          st_act_planes(a.act_out + (size_t)row * (a.N / 2) + f, a.act_plane, gv / (1.0f + expf(-gv)) * uv, a.sat);
        }
      }
    } else {
      float* o = a.out + (size_t)split * a.split_stride;
#pragma unroll
      for (int t = 0; t < NT; ++t) {
        const int col = nt_idx[t] * 16 + l15;
        if (nt_idx[t] < a.n_tiles && col < a.N) o[(size_t)row * a.N + col] = v[t];
      }
    }
  };
  if (KW == 1) {
#pragma unroll
    for (int mt = 0; mt < MT; ++mt)
#pragma unroll
      for (int r = 0; r < 4; ++r) {
        float v[NT];
#pragma unroll
        for (int t = 0; t < NT; ++t) v[t] = acc[mt][t][r];
        emit(mt, r, v);
      }
  } else {
    // one row tile at a time through LDS (the activation buffers are free after the loop's last
    // barrier): every wave stores its 16 values per lane, then k-wave kq finishes the rows
    // r = kq, kq + KW, .. of the tile, adding in the order kq = 0, 1, ...
    float* red = reinterpret_cast<float*>(smem);
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) {
#pragma unroll
      for (int r = 0; r < 4; ++r)
#pragma unroll
        for (int t = 0; t < NT; ++t) red[((wave * 4 + r) * NT + t) * 64 + lane] = acc[mt][t][r];
      __syncthreads();
      for (int r = kq; r < 4; r += KW) {
        float v[NT];
#pragma unroll
        for (int t = 0; t < NT; ++t) {
          float sum = 0.f;
#pragma unroll
          for (int k = 0; k < KW; ++k) sum += red[(((cs * KW + k) * 4 + r) * NT + t) * 64 + lane];
          v[t] = sum;
        }
        emit(mt, r, v);
      }
      __syncthreads();
    }
  }
}

// compiled (CS, KW) pairs; a chunk is one k-step per k-wave
constexpr int kNumCfg = 3;
constexpr int kMinMT = 4, kMaxMT = 8;   // compiled row tiles per workgroup
const int kCfgCS[kNumCfg] = {8, 4, 2};
const int kCfgKW[kNumCfg] = {1, 2, 4};
const int kCfgKC[kNumCfg] = {32, 64, 128};

template <int MT, int MODE>
void launch_cfg(int cfg, dim3 grid, hipStream_t s, const RowsArgs& a) {
  const dim3 block(64 * WAVES);
  if (MODE == MODE_ARGMAX) {                      // 8x1 only
    hipLaunchKernelGGL((k_gemm_rows_bf16<MT, 8, 1, MODE>), grid, block, 0, s, a);
    return;
  }
  switch (cfg) {
    case 0: hipLaunchKernelGGL((k_gemm_rows_bf16<MT, 8, 1, MODE>), grid, block, 0, s, a); break;
    case 1: hipLaunchKernelGGL((k_gemm_rows_bf16<MT, 4, 2, MODE == MODE_ARGMAX ? MODE_PARTIAL : MODE>), grid, block, 0, s, a); break;
    default: hipLaunchKernelGGL((k_gemm_rows_bf16<MT, 2, 4, MODE == MODE_ARGMAX ? MODE_PARTIAL : MODE>), grid, block, 0, s, a); break;
  }
}

template <int MODE>
void launch_mt(int mt, int cfg, dim3 grid, hipStream_t s, const RowsArgs& a) {
  switch (mt) {
    case 4: launch_cfg<4, MODE>(cfg, grid, s, a); break;
    case 5: launch_cfg<5, MODE>(cfg, grid, s, a); break;
    case 6: launch_cfg<6, MODE>(cfg, grid, s, a); break;
    case 7: launch_cfg<7, MODE>(cfg, grid, s, a); break;
    default: launch_cfg<8, MODE>(cfg, grid, s, a); break;
  }
}

}  // namespace

int gemm_rows_chunk(int cfg) { return kCfgKC[cfg]; }

// Row tiles per workgroup (4..8: the rows are cut into equal blocks), configuration and K
// splits with the least modelled time: rounds of workgroups over the CUs x (matrix-core time of
// a workgroup + a fixed start/finish cost) + traffic of the partial sums.  max_part_elems
// bounds splits x R x N.  Returns false if K fits no compiled chunk length.
bool gemm_rows_plan(const ts_model* m, int R, int N, int K, int mode, size_t max_part_elems, int* mt_out, int* cfg_out,
                    int* splits_out) {
  const int tiles = (R + 15) / 16;
  double best = 1e300;
  bool found = false;
  if ((size_t)TS_ACT_PLANES * (R + 2 * TS_MROWS_PER_BLOCK) * K * 2 >= ((size_t)1 << 32)) return false;   // 32-bit activation offsets
  for (int mt = kMinMT; mt <= kMaxMT; ++mt) {
    const int n_rblocks = (tiles + mt - 1) / mt;
    if (mt > kMinMT && n_rblocks == (tiles + mt - 2) / (mt - 1)) continue;   // same blocks, more idle rows
    for (int cfg = 0; cfg < kNumCfg; ++cfg) {
      if (mode == MODE_ARGMAX && cfg != 0) break;
      const int kc = kCfgKC[cfg];
      if (K % kc) continue;
      const int chunks = K / kc;
      const int cols = kCfgCS[cfg] * NT * 16;
      const int groups = (N + cols - 1) / cols;
      for (int s = 1; s <= chunks && s <= 8; ++s) {
        if (chunks % s) continue;
        if (mode != MODE_PARTIAL && s > 1) break;
        if (s > 1 && (size_t)s * R * N > max_part_elems) break;
        const long wgs = (long)((groups * s + 7) / 8) * 8 * n_rblocks;
        // the 4-row-tile kernels with one or two k-waves need half the registers and LDS of a CU:
        // two workgroups share one
        const int wg_per_cu = (cfg <= 1 && mt <= 4) ? 2 : 1;
        const long rounds = (wgs + (long)m->n_cu * wg_per_cu - 1) / ((long)m->n_cu * wg_per_cu);
        // MFMAs a SIMD issues for one workgroup (2 waves per SIMD), 16 cycles each at 2.4 GHz;
        // measured issue efficiency (one activation plane's worth): about 0.36 with four waves per
        // SIMD and the short pipeline, 0.40 with two waves and the deep one, a tenth less with k-waves
        // (their deeper activation registers leave no room for two chunks ahead)
        const double eff = wg_per_cu == 2 ? 0.36 : (cfg == 0 ? 0.40 : 0.36 * (cfg == 2 ? 0.9 : 1.0));
        const double mfma_us = 2.0 * (K / s / 32 / kCfgKW[cfg]) * mt * NT * 16 / 2400.0;
        double cost = rounds * (wg_per_cu * mfma_us / eff + 6.0);
        if (s > 1) cost += s * R * (double)N * 4.0 / 12.0e6;        // partial sums, mostly overlapped with the products
        if (cost < best) { best = cost; found = true; *mt_out = mt; *cfg_out = cfg; *splits_out = s; }
      }
    }
  }
  return found;
}

void launch_gemm_rows_bf16(ts_model* m, const f16_t* X, const f16_t* Wt, float* out, int R, int N, int K, int mt, int cfg,
                           int splits, int mode, f16_t* act_out, float* logits) {
  RowsArgs a;
  a.x_rows = m->ws_rows + TS_MROWS_PER_BLOCK;
  a.X = X; a.Wt = Wt; a.out = out;
  a.x_plane = (size_t)a.x_rows * K;
  a.act_plane = (size_t)a.x_rows * (N / 2);
  a.act_out = act_out;
  a.sat = m->sat_count;
  a.logits = logits; a.aval = m->amax_val; a.aidx = m->amax_idx; a.amax_stride = m->amax_parts;
  a.R = R; a.N = N; a.K = K;
  if (mode != MODE_PARTIAL) splits = 1;
  a.kper = K / splits;
  a.n_tiles = (N + 15) / 16;
  a.kt_count = K / 32;
  a.split_stride = (size_t)R * N;
  const int cols = kCfgCS[cfg] * NT * 16;
  a.n_groups = (N + cols - 1) / cols;
  a.n_units = a.n_groups * splits;
  a.n_rblocks = ((R + 15) / 16 + mt - 1) / mt;
  dim3 grid((unsigned)((a.n_units + 7) / 8) * 8 * a.n_rblocks);
  if (mode == MODE_ARGMAX) m->amax_used = a.n_groups;       // partials the combine kernel has to look at
  if (mode == MODE_SWIGLU) launch_mt<MODE_SWIGLU>(mt, cfg, grid, m->stream, a);
  else if (mode == MODE_ARGMAX) launch_mt<MODE_ARGMAX>(mt, cfg, grid, m->stream, a);
  else launch_mt<MODE_PARTIAL>(mt, cfg, grid, m->stream, a);
}
