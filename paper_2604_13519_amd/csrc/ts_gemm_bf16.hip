// Skinny-M bf16 projection for gfx950:  out[r][n] = sum_k X[r][k] * W[n][k],  r < R <= 80 per pass.
//
// With at most a few dozen rows the projection is a weight stream: every weight byte is
// used once, so the kernel is organised around the HBM read of W and nothing else.
//  * W is pre-tiled at model load into MFMA operand order (see k_repack_tiles): a wave's
//    16-byte-per-lane global load is one contiguous 1 KiB tile that feeds
//    v_mfma_f32_16x16x32_bf16 directly as the B operand - no LDS, no shuffles for weights.
//  * Each wave owns NT tiles of 16 output features and walks its K range in chunks of 128;
//    the next chunk's weights are in flight (register double buffer) while the current one
//    is multiplied.
//  * The activations X (R x K, tiny) are shared by the 4 waves of a workgroup through a
//    double-buffered LDS chunk and read as A operands with 16-byte LDS loads.
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

constexpr int KC = TS_GEMM_KC;   // k elements per chunk
constexpr int KSTEPS = KC / 32;  // MFMA k-steps per chunk
constexpr int XS = KC + 8;       // LDS row stride in elements (272 B, keeps 16 B alignment)

struct GemmArgs {
  const bf16_t* X;     // [rows][K] row-major, rows padded to a multiple of 16 in memory
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

template <int NT>
__device__ __forceinline__ void load_w(bf16x8 (&w)[NT][KSTEPS], const bf16_t* __restrict__ Wt, const size_t (&tile0)[NT],
                                       int kt, int lane) {
#pragma unroll
  for (int t = 0; t < NT; ++t)
#pragma unroll
    for (int j = 0; j < KSTEPS; ++j)
      w[t][j] = *reinterpret_cast<const bf16x8*>(Wt + ((tile0[t] + kt + j) * 64 + lane) * 8);
}

template <int MT>
__device__ __forceinline__ void load_x(u32x4 (&xr)[MT], const bf16_t* __restrict__ X, int row0, int K, int kbase, int tid) {
#pragma unroll
  for (int p = 0; p < MT; ++p)
    xr[p] = *reinterpret_cast<const u32x4*>(X + (size_t)(row0 + p * 16 + (tid >> 4)) * K + kbase + (tid & 15) * 8);
}

template <int MT>
__device__ __forceinline__ void store_x(bf16_t (*xs)[XS], const u32x4 (&xr)[MT], int tid) {
#pragma unroll
  for (int p = 0; p < MT; ++p) *reinterpret_cast<u32x4*>(&xs[p * 16 + (tid >> 4)][(tid & 15) * 8]) = xr[p];
}

template <int MT, int NT>
__device__ __forceinline__ void mma_chunk(f32x4 (&acc)[MT][NT], const bf16_t (*xs)[XS], const bf16x8 (&w)[NT][KSTEPS],
                                          int lane) {
  const int l15 = lane & 15, g = lane >> 4;
#pragma unroll
  for (int ks = 0; ks < KSTEPS; ++ks) {
    bf16x8 a[MT];
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) a[mt] = *reinterpret_cast<const bf16x8*>(&xs[mt * 16 + l15][ks * 32 + g * 8]);
#pragma unroll
    for (int t = 0; t < NT; ++t)
#pragma unroll
      for (int mt = 0; mt < MT; ++mt)
        acc[mt][t] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a[mt], w[t][ks], acc[mt][t], 0, 0, 0);
  }
}

template <int MT, int NT, bool ARGMAX>
__global__ __launch_bounds__(256) void k_gemm_bf16(GemmArgs a) {
  __shared__ __attribute__((aligned(16))) bf16_t xs[2][MT * 16][XS];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int row0 = blockIdx.z * TS_MROWS_PER_BLOCK;
  const int kbase0 = blockIdx.y * a.kper;
  const int n_chunks = a.kper / KC;

  size_t tile0[NT];
  int nt_idx[NT];
#pragma unroll
  for (int t = 0; t < NT; ++t) {
    nt_idx[t] = (blockIdx.x * 4 + wave) * NT + t;
    const int c = nt_idx[t] < a.n_tiles ? nt_idx[t] : a.n_tiles - 1;   // clamp: idle waves re-read a valid tile
    tile0[t] = (size_t)c * a.kt_count;
  }

  f32x4 acc[MT][NT];
#pragma unroll
  for (int mt = 0; mt < MT; ++mt)
#pragma unroll
    for (int t = 0; t < NT; ++t) acc[mt][t] = f32x4{0.f, 0.f, 0.f, 0.f};

  bf16x8 w0[NT][KSTEPS], w1[NT][KSTEPS];
  u32x4 xr[MT];

  load_w<NT>(w0, a.Wt, tile0, kbase0 / 32, lane);
  load_x<MT>(xr, a.X, row0, a.K, kbase0, tid);
  store_x<MT>(xs[0], xr, tid);
  __syncthreads();

  // two chunks per trip so that the weight register buffers swap without copies
  int c = 0;
  for (; c + 1 < n_chunks; c += 2) {
    const int kb1 = kbase0 + (c + 1) * KC;
    load_w<NT>(w1, a.Wt, tile0, kb1 / 32, lane);
    load_x<MT>(xr, a.X, row0, a.K, kb1, tid);
    mma_chunk<MT, NT>(acc, xs[0], w0, lane);
    store_x<MT>(xs[1], xr, tid);
    __syncthreads();
    const bool more = c + 2 < n_chunks;
    if (more) {
      const int kb2 = kbase0 + (c + 2) * KC;
      load_w<NT>(w0, a.Wt, tile0, kb2 / 32, lane);
      load_x<MT>(xr, a.X, row0, a.K, kb2, tid);
    }
    mma_chunk<MT, NT>(acc, xs[1], w1, lane);
    if (more) store_x<MT>(xs[0], xr, tid);
    __syncthreads();
  }
  if (c < n_chunks) mma_chunk<MT, NT>(acc, xs[0], w0, lane);   // odd chunk count: last chunk sits in buffer 0

  const int l15 = lane & 15, g = lane >> 4;
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
    __shared__ float rv[4][MT * 16];
    __shared__ int ri[4][MT * 16];
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
      for (int w = 1; w < 4; ++w) amax_take(bv, bi, rv[w][tid], ri[w][tid]);
      a.aval[(size_t)(row0 + tid) * a.amax_parts + blockIdx.x] = bv;
      a.aidx[(size_t)(row0 + tid) * a.amax_parts + blockIdx.x] = bi;
    }
  }
}

template <int NT, bool ARGMAX>
void launch_mt(int mt, dim3 grid, hipStream_t s, const GemmArgs& a) {
  switch (mt) {
    case 1: hipLaunchKernelGGL((k_gemm_bf16<1, NT, ARGMAX>), grid, dim3(256), 0, s, a); break;
    case 2: hipLaunchKernelGGL((k_gemm_bf16<2, NT, ARGMAX>), grid, dim3(256), 0, s, a); break;
    case 3: hipLaunchKernelGGL((k_gemm_bf16<3, NT, ARGMAX>), grid, dim3(256), 0, s, a); break;
    case 4: hipLaunchKernelGGL((k_gemm_bf16<4, NT, ARGMAX>), grid, dim3(256), 0, s, a); break;
    default: hipLaunchKernelGGL((k_gemm_bf16<5, NT, ARGMAX>), grid, dim3(256), 0, s, a); break;
  }
}

}  // namespace

// Tiles per wave and K splits: enough workgroups that every CU holds several, each still
// walking at least two chunks.
GemmPlan gemm_bf16_plan(const ts_model* m, int N, int K) {
  const int n_tiles = (N + 15) / 16;
  const int chunks = K / KC;
  GemmPlan p;
  p.nt = ((n_tiles + 7) / 8 >= m->n_cu) ? 2 : 1;
  const int groups = (n_tiles + 4 * p.nt - 1) / (4 * p.nt);
  p.splits = 1;
  for (int s = 1; s <= chunks; ++s) {
    if (chunks % s) continue;
    if (chunks / s < 2 && s > 1) break;
    p.splits = s;
    if (groups * s >= 2 * m->n_cu) break;
  }
  return p;
}

void launch_gemm_bf16(ts_model* m, const bf16_t* X, const bf16_t* Wt, float* out, int R, int N, int K, GemmPlan plan,
                      bool argmax, float* logits) {
  GemmArgs a;
  a.X = X; a.Wt = Wt; a.out = out; a.logits = logits;
  a.aval = m->amax_val; a.aidx = m->amax_idx;
  a.R = R; a.N = N; a.K = K;
  const int splits = argmax ? 1 : plan.splits;
  a.kper = K / splits;
  a.n_tiles = (N + 15) / 16;
  a.kt_count = K / 32;
  a.split_stride = (size_t)R * N;
  a.amax_parts = m->amax_parts;
  const int groups = (a.n_tiles + 4 * plan.nt - 1) / (4 * plan.nt);
  const int m_blocks = (R + TS_MROWS_PER_BLOCK - 1) / TS_MROWS_PER_BLOCK;
  const int mt = m_blocks > 1 ? 5 : (R + 15) / 16;
  dim3 grid(groups, splits, m_blocks);
  if (argmax) {
    if (plan.nt == 2) launch_mt<2, true>(mt, grid, m->stream, a); else launch_mt<1, true>(mt, grid, m->stream, a);
  } else {
    if (plan.nt == 2) launch_mt<2, false>(mt, grid, m->stream, a); else launch_mt<1, false>(mt, grid, m->stream, a);
  }
}
