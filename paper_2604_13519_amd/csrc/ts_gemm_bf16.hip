// Skinny-M bf16 projection for gfx950:  out[r][n] = sum_k X[r][k] * W[n][k],  r < R <= 80 per pass.
//
// With at most a few dozen rows the projection is a weight stream: every weight byte is
// used once, so the kernel is organised around the HBM read of W and nothing else.
//  * W is pre-tiled at model load into MFMA operand order (see k_repack_tiles): a wave's
//    16-byte-per-lane global load is one contiguous 1 KiB tile that feeds
//    v_mfma_f32_16x16x32_bf16 directly as the B operand - no LDS, no shuffles for weights.
//  * Each wave owns NT tiles of 16 output features and walks its K range in chunks of KC;
//    the weights of the next PF chunks are in flight (register ring) while the current one
//    is multiplied.
//  * The activations X (R x K, tiny) are shared by the WAVES waves of a workgroup through a
//    double-buffered LDS chunk and read as A operands with 16-byte LDS loads.  Each activation
//    is a (hi, lo) pair of bf16 values (about 16 significant bits): two MFMAs per weight
//    fragment.  The matrix cores idle most of the time in a weight-streaming kernel, so the
//    extra precision costs no bandwidth.
//  * K is split across workgroups (grid.y) so that every CU streams; partial sums go to a
//    fp32 [split][row][col] buffer that the next row-wise kernel adds up in a fixed order
//    (deterministic, no atomics).
//  * lm_head variant (ARGMAX): no split; the epilogue reduces each row's maximum over the
//    workgroup's columns and emits one (value, index) partial per row, so the full logits
//    never have to reach memory.
#include "ts_internal.h"
#include "ts_device_utils.h"

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

namespace {

struct GemmArgs {
  const bf16_t* X;     // [2][rows][K]: hi plane, then lo plane (x = hi + lo), rows padded in memory
  size_t x_plane;      // elements between the planes
  const bf16_t* Wt;    // tiled weights
  float* out;          // [split][R][N] partial sums (nullptr for ARGMAX)
  float* logits;       // [R][N] or nullptr (ARGMAX only)
  float* aval;         // [R][amax_parts]
  int32_t* aidx;
  int R, N, K;
  int kper;            // k elements per split
  int n_tiles;         // ceil(N / 16)
  int kt_count;        // K / 32
  size_t split_stride; // R * N
  int amax_parts;
};

template <int MT, int NT, int WAVES, int KC, int PF, bool ARGMAX, int XPAD = 8>
__global__ __launch_bounds__(64 * WAVES) void k_gemm_bf16(GemmArgs a) {
  constexpr int KSTEPS = KC / 32;           // MFMA k-steps per chunk
  constexpr int XS = KC + XPAD;             // LDS row stride in elements (+16 B: bank spread, keeps alignment)
  constexpr int NTHR = 64 * WAVES;
  constexpr int NBUF = PF + 1;              // weight register ring
  constexpr int XV1 = MT * 16 * KC / 8;     // 16-byte vectors per X chunk and plane
  constexpr int XV = 2 * XV1;               // both planes
  constexpr int XPT = (XV + NTHR - 1) / NTHR;
  __shared__ __attribute__((aligned(16))) bf16_t xs[2][2][MT * 16][XS];   // [buffer][plane][row][k]

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int l15 = lane & 15, g = lane >> 4;
  const int row0 = blockIdx.z * TS_MROWS_PER_BLOCK;
  const int kbase0 = blockIdx.y * a.kper;
  const int n_chunks = a.kper / KC;

  const bf16_t* wp[NT];                     // this lane's pointer into each owned tile row
  int nt_idx[NT];
#pragma unroll
  for (int t = 0; t < NT; ++t) {
    nt_idx[t] = (blockIdx.x * WAVES + wave) * NT + t;
    const int c = nt_idx[t] < a.n_tiles ? nt_idx[t] : a.n_tiles - 1;   // idle waves re-read a valid tile
    wp[t] = a.Wt + (((size_t)c * a.kt_count + kbase0 / 32) * 64 + lane) * 8;
  }

  f32x4 acc[MT][NT];
#pragma unroll
  for (int mt = 0; mt < MT; ++mt)
#pragma unroll
    for (int t = 0; t < NT; ++t) acc[mt][t] = f32x4{0.f, 0.f, 0.f, 0.f};

  bf16x8 w[NBUF][NT][KSTEPS];
  u32x4 xr[XPT];

  auto load_w = [&](bf16x8 (&dst)[NT][KSTEPS], int chunk) {
#pragma unroll
    for (int t = 0; t < NT; ++t)
#pragma unroll
      for (int j = 0; j < KSTEPS; ++j)
        dst[t][j] = __builtin_nontemporal_load(
            reinterpret_cast<const bf16x8*>(wp[t] + ((size_t)chunk * KSTEPS + j) * 512));
  };
  auto load_x = [&](int chunk) {
    const int kb = kbase0 + chunk * KC;
#pragma unroll
    for (int p = 0; p < XPT; ++p) {
      const int v = tid + p * NTHR;
      if (XV % NTHR == 0 || v < XV) {
        const int pl = v / XV1, u = v % XV1;
        const int row = u / (KC / 8), cv = u % (KC / 8);
        xr[p] = *reinterpret_cast<const u32x4*>(a.X + pl * a.x_plane + (size_t)(row0 + row) * a.K + kb + cv * 8);
      }
    }
  };
  auto store_x = [&](int buf) {
#pragma unroll
    for (int p = 0; p < XPT; ++p) {
      const int v = tid + p * NTHR;
      if (XV % NTHR == 0 || v < XV) {
        const int pl = v / XV1, u = v % XV1;
        const int row = u / (KC / 8), cv = u % (KC / 8);
        *reinterpret_cast<u32x4*>(&xs[buf][pl][row][cv * 8]) = xr[p];
      }
    }
  };
  // activations are (hi, lo) bf16 pairs: both planes multiply the same weight fragment and
  // add into the same fp32 accumulator
  auto mma_chunk = [&](const bf16x8 (&wc)[NT][KSTEPS], int buf) {
#pragma unroll
    for (int ks = 0; ks < KSTEPS; ++ks) {
      bf16x8 ah[MT], al[MT];
#pragma unroll
      for (int mt = 0; mt < MT; ++mt) {
        ah[mt] = *reinterpret_cast<const bf16x8*>(&xs[buf][0][mt * 16 + l15][ks * 32 + g * 8]);
        al[mt] = *reinterpret_cast<const bf16x8*>(&xs[buf][1][mt * 16 + l15][ks * 32 + g * 8]);
      }
#pragma unroll
      for (int t = 0; t < NT; ++t)
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) {
          acc[mt][t] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(ah[mt], wc[t][ks], acc[mt][t], 0, 0, 0);
          acc[mt][t] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(al[mt], wc[t][ks], acc[mt][t], 0, 0, 0);
        }
    }
  };

  // Vector-memory loads complete in issue order as far as the wait counter is concerned, so
  // the small X loads are always issued BEFORE the weight prefetch of the same step: waiting
  // for X then leaves the newest weight chunks in flight.
  load_x(0);
  __builtin_amdgcn_sched_barrier(0);        // keep the issue order
#pragma unroll
  for (int b = 0; b < PF; ++b)
    if (b < n_chunks) load_w(w[b], b);
  store_x(0);
  __syncthreads();

  // NBUF chunks per trip so that ring slots are compile-time register names
  for (int c0 = 0; c0 < n_chunks; c0 += NBUF) {
#pragma unroll
    for (int b = 0; b < NBUF; ++b) {
      const int c = c0 + b;
      if (c < n_chunks) {
        const bool more = c + 1 < n_chunks;
        if (more) load_x(c + 1);
        __builtin_amdgcn_sched_barrier(0);  // X loads first, then the weight prefetch
        if (c + PF < n_chunks) load_w(w[(b + PF) % NBUF], c + PF);
        __builtin_amdgcn_sched_barrier(0);
        mma_chunk(w[b], c & 1);
        if (more) store_x((c + 1) & 1);
        __syncthreads();
      }
    }
  }

  if (!ARGMAX) {
    float* o = a.out + (size_t)blockIdx.y * a.split_stride;
#pragma unroll
    for (int t = 0; t < NT; ++t) {
      const int col = nt_idx[t] * 16 + l15;
      if (nt_idx[t] < a.n_tiles && col < a.N) {
#pragma unroll
        for (int mt = 0; mt < MT; ++mt)
#pragma unroll
          for (int r = 0; r < 4; ++r) {
            const int row = row0 + mt * 16 + g * 4 + r;
            if (row < a.R) o[(size_t)row * a.N + col] = acc[mt][t][r];
          }
      }
    }
  } else {
    __shared__ float rv[WAVES][MT * 16];
    __shared__ int ri[WAVES][MT * 16];
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
        for (int o = 8; o > 0; o >>= 1) {       // reduce over the 16 lanes that hold this row
          const float ov = __shfl_xor(bv, o, 64);
          const int oi = __shfl_xor(bi, o, 64);
          amax_take(bv, bi, ov, oi);
        }
        if (l15 == 0) { rv[wave][mt * 16 + g * 4 + r] = bv; ri[wave][mt * 16 + g * 4 + r] = bi; }
      }
    __syncthreads();
    if (tid < MT * 16 && row0 + tid < a.R) {
      float bv = rv[0][tid];
      int bi = ri[0][tid];
      for (int wv = 1; wv < WAVES; ++wv) amax_take(bv, bi, rv[wv][tid], ri[wv][tid]);
      a.aval[(size_t)(row0 + tid) * a.amax_parts + blockIdx.x] = bv;
      a.aidx[(size_t)(row0 + tid) * a.amax_parts + blockIdx.x] = bi;
    }
  }
}

template <int NT, int WAVES, int KC, int PF, bool ARGMAX>
void launch_mt(int mt, dim3 grid, hipStream_t s, const GemmArgs& a) {
  switch (mt) {
    case 1: hipLaunchKernelGGL((k_gemm_bf16<1, NT, WAVES, KC, PF, ARGMAX>), grid, dim3(64 * WAVES), 0, s, a); break;
    case 2: hipLaunchKernelGGL((k_gemm_bf16<2, NT, WAVES, KC, PF, ARGMAX>), grid, dim3(64 * WAVES), 0, s, a); break;
    case 3: hipLaunchKernelGGL((k_gemm_bf16<3, NT, WAVES, KC, PF, ARGMAX>), grid, dim3(64 * WAVES), 0, s, a); break;
    case 4: hipLaunchKernelGGL((k_gemm_bf16<4, NT, WAVES, KC, PF, ARGMAX>), grid, dim3(64 * WAVES), 0, s, a); break;
    default: hipLaunchKernelGGL((k_gemm_bf16<5, NT, WAVES, KC, PF, ARGMAX>), grid, dim3(64 * WAVES), 0, s, a); break;
  }
}

// The compiled tile shapes.  shape id -> (NT, WAVES, KC, PF).  The LDS holds two buffers of
// two planes of the activation chunk, which keeps KC at 128 for 80 rows.
constexpr int kNumShapes = 4;
const int kShapeNT[kNumShapes] = {1, 2, 1, 2};
const int kShapeWaves[kNumShapes] = {4, 4, 8, 8};
const int kShapeKC[kNumShapes] = {128, 128, 128, 128};

template <bool ARGMAX>
void launch_shape(int shape, int mt, dim3 grid, hipStream_t s, const GemmArgs& a) {
  switch (shape) {
    case 0: launch_mt<1, 4, 128, 1, ARGMAX>(mt, grid, s, a); break;
    case 1: launch_mt<2, 4, 128, 1, ARGMAX>(mt, grid, s, a); break;
    case 2: launch_mt<1, 8, 128, 1, ARGMAX>(mt, grid, s, a); break;
    default: launch_mt<2, 8, 128, 1, ARGMAX>(mt, grid, s, a); break;
  }
}

}  // namespace

int gemm_bf16_cols_per_group(int shape) { return kShapeNT[shape] * kShapeWaves[shape] * 16; }
int gemm_bf16_chunk(int shape) { return kShapeKC[shape]; }

// Tile shape and K splits.  Measured on MI355X, the stream is fastest when the workgroups
// of a launch fit the chip in ONE round (one 8-wave workgroup per CU): a second round adds
// a tail and more partial-sum traffic than it gains.  So: the (shape, splits) pair with the
// most workgroups not exceeding the CU count, wider tiles winning ties; if even the
// coarsest split exceeds the chip (lm_head), the fewest workgroups.
GemmPlan gemm_bf16_plan(const ts_model* m, int N, int K, bool allow_split) {
  GemmPlan best{0, 1};
  long best_score = -1;
  for (int shape = 0; shape < kNumShapes; ++shape) {
    const int kc = kShapeKC[shape];
    if (K % kc) continue;
    const int chunks = K / kc;
    const int cols = gemm_bf16_cols_per_group(shape);
    const int groups = (N + cols - 1) / cols;
    for (int s = 1; s <= chunks && s <= 16; ++s) {
      if (chunks % s) continue;
      if (!allow_split && s > 1) break;
      const long wgs = (long)groups * s;
      // fits in one round: more workgroups is better; otherwise fewer is better
      long score = wgs <= m->n_cu ? (1L << 40) + wgs * 16 : (1L << 30) - wgs * 16;
      score += kShapeWaves[shape] + kShapeNT[shape];        // prefer 8 waves, 2 tiles on ties
      if (score > best_score) { best_score = score; best.shape = shape; best.splits = s; }
    }
  }
  return best;
}

void launch_gemm_bf16(ts_model* m, const bf16_t* X, const bf16_t* Wt, float* out, int R, int N, int K, GemmPlan plan,
                      bool argmax, float* logits) {
  GemmArgs a;
  a.x_plane = (size_t)(m->ws_rows + TS_MROWS_PER_BLOCK) * K;
  a.X = X; a.Wt = Wt; a.out = out; a.logits = logits;
  a.aval = m->amax_val; a.aidx = m->amax_idx;
  a.R = R; a.N = N; a.K = K;
  const int splits = argmax ? 1 : plan.splits;
  a.kper = K / splits;
  a.n_tiles = (N + 15) / 16;
  a.kt_count = K / 32;
  a.split_stride = (size_t)R * N;
  a.amax_parts = m->amax_parts;
  const int cols = gemm_bf16_cols_per_group(plan.shape);
  const int groups = (N + cols - 1) / cols;
  const int m_blocks = (R + TS_MROWS_PER_BLOCK - 1) / TS_MROWS_PER_BLOCK;
  const int mt = m_blocks > 1 ? 5 : (R + 15) / 16;
  dim3 grid(groups, splits, m_blocks);
  if (argmax) launch_shape<true>(plan.shape, mt, grid, m->stream, a);
  else launch_shape<false>(plan.shape, mt, grid, m->stream, a);
}
