// Skinny-M projection of a bf16 model for gfx950:  out[r][n] = sum_k X[r][k] * W[n][k],  r < R <= 80 per pass.
//
// With at most a few dozen rows the projection is a weight stream: every weight byte is
// used once, so the kernel is organised around the HBM read of W and nothing else.
//  * Arithmetic: IEEE half x IEEE half -> fp32 (v_mfma_f32_16x16x32_f16).  The bf16 weights are
//    re-encoded as half at model load (exact: half has more significand bits; the load rejects
//    magnitudes beyond half's range) and the activations arrive rounded to half - 11
//    significant bits where bf16 has 8, with one MFMA per weight fragment.
//  * W is pre-tiled at model load into MFMA operand order (see k_repack_tiles): a wave's
//    16-byte-per-lane global load is one contiguous 1 KiB tile that feeds the MFMA directly as
//    the B operand - no LDS, no shuffles for weights.
//  * Each wave owns NT tiles of 16 output features and walks its K range in chunks of KC;
//    the weights of the next PF chunks are in flight (register ring) while the current one
//    is multiplied.
//  * The activations X (R x K, tiny) are shared by the WAVES waves of a workgroup through a
//    double-buffered LDS chunk and read as A operands with 16-byte LDS loads.
//  * K is split two ways.  Inside a workgroup, KW waves share the same output columns and take
//    alternate k-steps of every chunk; their accumulators are added through LDS in a fixed
//    order at the end.  Across workgroups (grid.y), partial sums go to a fp32
//    [split][row][col] buffer that the next row-wise kernel adds up in a fixed order
//    (deterministic, no atomics).  The in-workgroup split costs no memory traffic, the
//    cross-workgroup one costs a write and a read of the partial sums, so the planner uses as
//    little of the second as still fills the chip.
//  * gate/up variant (SWIGLU): the weight tiles of gate and up alternate, so a wave that owns
//    two neighbouring tiles holds gate and up of the same 16 features; with no cross-workgroup
//    split the epilogue applies SiLU(gate) * up and stores the product as half directly.
//  * lm_head variant (ARGMAX): no split; the epilogue reduces each row's maximum over the
//    workgroup's columns and emits one (value, index) partial per row, so the full logits
//    never have to reach memory.
#include "ts_internal.h"
#include "ts_device_utils.h"

typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

namespace {

struct GemmArgs {
  const f16_t* X;      // [2 planes][rows][K] IEEE half (x = hi + lo), rows padded in memory
  size_t x_plane;      // elements between the hi and the lo plane
  const f16_t* Wt;     // tiled weights, IEEE half
  float* out;          // [split][R][N] partial sums (nullptr for ARGMAX)
  float* logits;       // [R][N] or nullptr (ARGMAX only)
  float* aval;         // [R][amax_parts]
  int32_t* aidx;
  f16_t* act_out;      // SWIGLU: [2 planes][rows][N/2] gated product, IEEE half hi + lo
  size_t act_plane;    // elements between its planes
  unsigned long long* sat;   // counts gated products beyond half's range
  int R, N, K;
  int kper;            // k elements per split
  int n_tiles;         // ceil(N / 16)
  int kt_count;        // K / 32
  size_t split_stride; // R * N
  int amax_parts;
};

enum { MODE_PARTIAL = 0, MODE_ARGMAX = 1, MODE_SWIGLU = 2 };

template <int MT, int NT, int CS, int KW, int KC, int PF, int MODE, int XPAD = 8>
__global__ __launch_bounds__(64 * CS * KW) void k_gemm_bf16(GemmArgs a) {
  constexpr int WAVES = CS * KW;            // CS column sets x KW k-step owners
  constexpr bool ARGMAX = MODE == MODE_ARGMAX;
  constexpr int KSTEPS = KC / 32;           // MFMA k-steps per chunk
  constexpr int KSW = KSTEPS / KW;          // ... of which this wave multiplies KSW
  static_assert(KSTEPS % KW == 0 && KSW >= 1, "k-steps of a chunk must divide among the k-waves");
  static_assert(!(ARGMAX && KW != 1), "the arg-max epilogue expects one wave per column set");
  static_assert(MODE != MODE_SWIGLU || NT == 2, "gate and up tiles alternate");
  constexpr int XS = KC + XPAD;             // LDS row stride in elements (+16 B: bank spread, keeps alignment)
  constexpr int NTHR = 64 * WAVES;
  constexpr int NBUF = PF + 1;              // weight register ring
  constexpr int PL = TS_ACT_PLANES;         // an activation is the sum of a hi and a lo half
  constexpr int XVP = MT * 16 * KC / 8;     // 16-byte vectors per plane of an X chunk
  constexpr int XV = PL * XVP;
  constexpr int XPT = (XV + NTHR - 1) / NTHR;
  // activation chunks [buffer][plane][row][k]; the same memory later serves the k-wave reduction
  constexpr size_t XS_BYTES = sizeof(f16_t) * 2 * PL * MT * 16 * XS;
  constexpr size_t RED_BYTES = KW > 1 ? sizeof(float) * WAVES * 4 * NT * 64 : 0;
  __shared__ __attribute__((aligned(16))) char smem[XS_BYTES > RED_BYTES ? XS_BYTES : RED_BYTES];
  f16_t (*xs)[PL][MT * 16][XS] = reinterpret_cast<f16_t (*)[PL][MT * 16][XS]>(smem);

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int l15 = lane & 15, g = lane >> 4;
  const int cs = wave / KW, kq = wave % KW;
  const int row0 = blockIdx.z * TS_MROWS_PER_BLOCK;
  const int kbase0 = blockIdx.y * a.kper;
  const int n_chunks = a.kper / KC;

  // Addresses are (uniform 64-bit base) + (32-bit per-lane byte offset that never changes):
  // the loads then need no vector address arithmetic inside the loop.
  const int cs_u = __builtin_amdgcn_readfirstlane(cs), kq_u = __builtin_amdgcn_readfirstlane(kq);
  const char* wbase[NT];                    // start of this wave's k range in each owned tile row
  int nt_idx[NT];
#pragma unroll
  for (int t = 0; t < NT; ++t) {
    nt_idx[t] = (blockIdx.x * CS + cs_u) * NT + t;
    const int c = nt_idx[t] < a.n_tiles ? nt_idx[t] : a.n_tiles - 1;   // idle waves re-read a valid tile
    wbase[t] = reinterpret_cast<const char*>(a.Wt) + ((size_t)c * a.kt_count + kbase0 / 32 + kq_u * KSW) * 1024;
  }
  const uint32_t w_lane = lane * 16;
  const char* xbase = reinterpret_cast<const char*>(a.X) + ((size_t)row0 * a.K + kbase0) * 2;
  uint32_t x_off[XPT];                      // byte offset of each staged vector within a chunk
#pragma unroll
  for (int p = 0; p < XPT; ++p) {
    const int v = min(tid + p * NTHR, XV - 1);      // surplus threads re-read the last vector
    const int pl = v / XVP, row = (v % XVP) / (KC / 8), cv = v % (KC / 8);
    x_off[p] = (uint32_t)((pl * a.x_plane + (size_t)row * a.K + cv * 8) * 2);
  }

  f32x4 acc[MT][NT];
#pragma unroll
  for (int mt = 0; mt < MT; ++mt)
#pragma unroll
    for (int t = 0; t < NT; ++t) acc[mt][t] = f32x4{0.f, 0.f, 0.f, 0.f};

  f16x8 w[NBUF][NT][KSW];
  u32x4 xr[NBUF][XPT];   // activation chunks travel the same register ring as the weights

  auto load_w = [&](f16x8 (&dst)[NT][KSW], int chunk) {
#pragma unroll
    for (int t = 0; t < NT; ++t)
#pragma unroll
      for (int j = 0; j < KSW; ++j)
        dst[t][j] = __builtin_nontemporal_load(
            reinterpret_cast<const f16x8*>(wbase[t] + (size_t)chunk * (KSTEPS * 1024) + w_lane + j * 1024));
  };
  auto load_x = [&](u32x4 (&dst)[XPT], int chunk) {
    const char* xb = xbase + (size_t)chunk * (KC * 2);
#pragma unroll
    for (int p = 0; p < XPT; ++p) dst[p] = *reinterpret_cast<const u32x4*>(xb + x_off[p]);   // never predicated, see below
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
#pragma unroll
      for (int pl = 0; pl < PL; ++pl) {
        f16x8 xa[MT];
#pragma unroll
        for (int mt = 0; mt < MT; ++mt)
          xa[mt] = *reinterpret_cast<const f16x8*>(&xs[buf][pl][mt * 16 + l15][(kq * KSW + ks) * 32 + g * 8]);
#pragma unroll
        for (int t = 0; t < NT; ++t)
#pragma unroll
          for (int mt = 0; mt < MT; ++mt)
            acc[mt][t] = __builtin_amdgcn_mfma_f32_16x16x32_f16(xa[mt], wc[t][ks], acc[mt][t], 0, 0, 0);
      }
    }
  };

  // Vector-memory loads complete in issue order as far as the wait counter is concerned, and
  // the compiler's wait for a load counts every later load that MIGHT not have been issued as
  // not issued.  Three consequences shape this loop.  The activation chunk of step c + PF is
  // requested together with the weights of step c + PF and waits in registers as long as they
  // do: were it requested one step ahead, storing it to LDS would first wait for every weight
  // load issued before it, and the weights would never be more than one step ahead either.  The
  // small X loads go out BEFORE the weight loads of the same step.  And no load is ever
  // predicated - a prefetch under an `if` would turn every wait into a wait for everything;
  // where nothing is left to prefetch the step re-requests the last chunk instead (an L2 hit
  // that is never used).
  const int last = n_chunks - 1;
  auto step = [&](f16x8 (&wcur)[NT][KSW], f16x8 (&wpf)[NT][KSW], u32x4 (&xpf)[XPT], const u32x4 (&xnext)[XPT], int c) {
    load_x(xpf, min(c + PF, last));
    __builtin_amdgcn_sched_barrier(0);
    load_w(wpf, min(c + PF, last));
    __builtin_amdgcn_sched_barrier(0);
    mma_chunk(wcur, c & 1);
    store_x(xnext, (c + 1) & 1);            // chunk c + 1, requested PF - 1 steps ago
    __syncthreads();
  };

#pragma unroll
  for (int b = 0; b < PF; ++b) {
    load_x(xr[b], min(b, last));
    __builtin_amdgcn_sched_barrier(0);
    load_w(w[b], min(b, last));
    __builtin_amdgcn_sched_barrier(0);
  }
  store_x(xr[0], 0);
  __syncthreads();

  // NBUF chunks per trip so that ring slots are compile-time register names
  int c0 = 0;
  for (; c0 + NBUF <= n_chunks; c0 += NBUF) {
#pragma unroll
    for (int b = 0; b < NBUF; ++b) step(w[b], w[(b + PF) % NBUF], xr[(b + PF) % NBUF], xr[(b + 1) % NBUF], c0 + b);
  }
#pragma unroll
  for (int b = 0; b < NBUF - 1; ++b)
    if (c0 + b < n_chunks) step(w[b], w[(b + PF) % NBUF], xr[(b + PF) % NBUF], xr[(b + 1) % NBUF], c0 + b);

  if (!ARGMAX) {
    // value of output (row tile mt, row r of the lane group, tile t) goes to memory
    auto emit = [&](int mt, int r, const float (&v)[NT]) {
      const int row = row0 + mt * 16 + g * 4 + r;
      if (row >= a.R) return;
      if (MODE == MODE_SWIGLU) {
        const int f = (nt_idx[0] >> 1) * 16 + l15;           // tiles 2j / 2j+1 = gate / up of features 16j..
        if (nt_idx[1] < a.n_tiles) {
          const float gv = v[0], uv = v[NT - 1];
          st_act_planes(a.act_out + (size_t)row * (a.N / 2) + f, a.act_plane, gv / (1.0f + expf(-gv)) * uv, a.sat);
        }
      } else {
        float* o = a.out + (size_t)blockIdx.y * a.split_stride;
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
      // add the KW accumulators of a column set through LDS (the activation buffers are free
      // after the loop's last barrier), one row tile at a time, always in the order kq = 0, 1, ...
      float* red = reinterpret_cast<float*>(smem);
#pragma unroll
      for (int mt = 0; mt < MT; ++mt) {
#pragma unroll
        for (int r = 0; r < 4; ++r)
#pragma unroll
          for (int t = 0; t < NT; ++t) red[((wave * 4 + r) * NT + t) * 64 + lane] = acc[mt][t][r];
        __syncthreads();
        for (int r = kq; r < 4; r += KW) {                 // this wave finishes rows r of the tile
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

template <int NT, int CS, int KW, int KC, int PF, int MODE>
void launch_mt(int mt, dim3 grid, hipStream_t s, const GemmArgs& a) {
  const dim3 block(64 * CS * KW);
  switch (mt) {
    case 1: hipLaunchKernelGGL((k_gemm_bf16<1, NT, CS, KW, KC, PF, MODE>), grid, block, 0, s, a); break;
    case 2: hipLaunchKernelGGL((k_gemm_bf16<2, NT, CS, KW, KC, PF, MODE>), grid, block, 0, s, a); break;
    case 3: hipLaunchKernelGGL((k_gemm_bf16<3, NT, CS, KW, KC, PF, MODE>), grid, block, 0, s, a); break;
    case 4: hipLaunchKernelGGL((k_gemm_bf16<4, NT, CS, KW, KC, PF, MODE>), grid, block, 0, s, a); break;
    default: hipLaunchKernelGGL((k_gemm_bf16<5, NT, CS, KW, KC, PF, MODE>), grid, block, 0, s, a); break;
  }
}

// The compiled tile shapes.  shape id -> (NT, CS, KW): tiles per wave, column sets and
// k-waves per workgroup.  All use chunks of 128 k (the LDS holds two buffers of the
// activation chunk, 43 KiB for 80 rows).  The k-wave shapes hold fewer weight registers
// per chunk and prefetch two chunks ahead instead of one.
constexpr int kNumShapes = 5;
const int kShapeNT[kNumShapes] = {1, 2, 1, 2, 2};
const int kShapeCS[kNumShapes] = {4, 4, 8, 8, 4};
const int kShapeKW[kNumShapes] = {1, 1, 1, 1, 2};
const int kShapeKC[kNumShapes] = {128, 128, 128, 128, 128};

template <int MODE>
void launch_shape(int shape, int mt, dim3 grid, hipStream_t s, const GemmArgs& a) {
  switch (shape) {
    case 0: if (MODE != MODE_SWIGLU) launch_mt<1, 4, 1, 128, 1, MODE == MODE_SWIGLU ? MODE_PARTIAL : MODE>(mt, grid, s, a); break;
    case 1: launch_mt<2, 4, 1, 128, 1, MODE>(mt, grid, s, a); break;
    case 2: if (MODE != MODE_SWIGLU) launch_mt<1, 8, 1, 128, 1, MODE == MODE_SWIGLU ? MODE_PARTIAL : MODE>(mt, grid, s, a); break;
    case 3: launch_mt<2, 8, 1, 128, 1, MODE>(mt, grid, s, a); break;
    case 4: if (MODE != MODE_ARGMAX) launch_mt<2, 4, 2, 128, 2, MODE == MODE_ARGMAX ? MODE_PARTIAL : MODE>(mt, grid, s, a); break;
    default: break;
  }
}

bool shape_supports(int shape, int mode) {
  if (mode == MODE_ARGMAX) return kShapeKW[shape] == 1;
  if (mode == MODE_SWIGLU) return kShapeNT[shape] == 2;
  return true;
}

// plan.shape values from here on name a many-row configuration: kRowsShape0 + 4 * row tiles + cfg
constexpr int kRowsShape0 = 100;
constexpr size_t kRowsPartCap = (size_t)64 << 20;   // partial-sum elements a plan may use before a workspace exists

}  // namespace

int gemm_bf16_cols_per_group(int shape) { return kShapeNT[shape] * kShapeCS[shape] * 16; }
int gemm_bf16_chunk(int shape) { return shape >= kRowsShape0 ? gemm_rows_chunk((shape - kRowsShape0) % 4) : kShapeKC[shape]; }

// Tile shape and cross-workgroup K splits, from a byte count per CU:
//   rounds x (weight bytes one workgroup streams)         rounds = ceil(workgroups / CUs)
// + write and read of the fp32 partial sums, shared by all CUs (only if splits > 1)
// + a quarter of the activation bytes (both planes) a workgroup stages from L2 per round.
// Measured on MI355X, a second round of workgroups costs a full round (the tail does not
// overlap), which the round count models.  mode: 0 partial sums, 1 arg-max (no split),
// 2 SwiGLU epilogue (no split).
GemmPlan gemm_bf16_plan(const ts_model* m, int R, int N, int K, int mode) {
  if (R > TS_MROWS_PER_BLOCK) {   // batches: the many-row kernel
    int mt, cfg, splits;
    const size_t max_part = m->part_elems ? m->part_elems : kRowsPartCap;
    if (gemm_rows_plan(m, R, N, K, mode, max_part, &mt, &cfg, &splits)) return GemmPlan{kRowsShape0 + mt * 4 + cfg, splits};
  }
  GemmPlan best{mode == MODE_SWIGLU ? 1 : 0, 1};
  double best_cost = 1e300;
  const int rows = R > TS_MROWS_PER_BLOCK ? TS_MROWS_PER_BLOCK : ((R + 15) / 16) * 16;
  const int m_blocks = (R + TS_MROWS_PER_BLOCK - 1) / TS_MROWS_PER_BLOCK;   // each streams the weights again
  for (int shape = 0; shape < kNumShapes; ++shape) {
    if (!shape_supports(shape, mode)) continue;
    const int kc = kShapeKC[shape];
    if (K % kc) continue;
    const int chunks = K / kc;
    const int cols = gemm_bf16_cols_per_group(shape);
    const int groups = (N + cols - 1) / cols;
    for (int s = 1; s <= chunks && s <= 16; ++s) {
      if (chunks % s) continue;
      if (mode != MODE_PARTIAL && s > 1) break;
      const long wgs = (long)groups * s * m_blocks;
      const long rounds = (wgs + m->n_cu - 1) / m->n_cu;
      const double kper = (double)K / s;
      double cost = rounds * cols * kper * 2.0;
      if (s > 1) cost += 2.0 * s * R * (double)N * 4.0 / m->n_cu;
      cost += 0.25 * rounds * rows * kper * 2.0 * TS_ACT_PLANES;
      // Measured (8B shape, 65 rows): over a long K range the k-wave shape wins by its deeper prefetch
      // (gate/up, 32 chunks: 56.2 us against 58.1 us for the 4-wave shape of the same columns); over
      // the short ranges of the split projections its longer prologue and the cross-wave reduction
      // are not amortised (O, 4 chunks: 17.0 against 15.2 us; QKV, 8 chunks: 21.9 against 21.2 us).
      if (kper / kc >= 16 ? kShapeCS[shape] * kShapeKW[shape] < 6 : kShapeKW[shape] > 1) cost *= 1.05;
      if (kShapeNT[shape] < 2) cost *= 1.05;                     // one tile per wave reads twice the LDS per weight byte
      if (cost < best_cost) { best_cost = cost; best.shape = shape; best.splits = s; }
    }
  }
  return best;
}

void launch_gemm_bf16(ts_model* m, const f16_t* X, const f16_t* Wt, float* out, int R, int N, int K, GemmPlan plan,
                      int mode, float* logits, f16_t* act_out) {
  if (plan.shape >= kRowsShape0) {
    const int code = plan.shape - kRowsShape0;
    launch_gemm_rows_bf16(m, X, Wt, out, R, N, K, code / 4, code % 4, plan.splits, mode, act_out, logits);
    return;
  }
  GemmArgs a;
  a.X = X; a.Wt = Wt; a.out = out; a.logits = logits;
  a.x_plane = (size_t)(m->ws_rows + TS_MROWS_PER_BLOCK) * K;
  a.act_plane = (size_t)(m->ws_rows + TS_MROWS_PER_BLOCK) * (N / 2);
  a.aval = m->amax_val; a.aidx = m->amax_idx;
  a.act_out = act_out;
  a.sat = m->sat_count;
  a.R = R; a.N = N; a.K = K;
  const int splits = mode == MODE_PARTIAL ? plan.splits : 1;
  a.kper = K / splits;
  a.n_tiles = (N + 15) / 16;
  a.kt_count = K / 32;
  a.split_stride = (size_t)R * N;
  a.amax_parts = m->amax_parts;
  if (mode == MODE_ARGMAX) m->amax_used = (N + gemm_bf16_cols_per_group(plan.shape) - 1) / gemm_bf16_cols_per_group(plan.shape);
  const int cols = gemm_bf16_cols_per_group(plan.shape);
  const int groups = (N + cols - 1) / cols;
  const int m_blocks = (R + TS_MROWS_PER_BLOCK - 1) / TS_MROWS_PER_BLOCK;
  const int mt = m_blocks > 1 ? 5 : (R + 15) / 16;
  dim3 grid(groups, splits, m_blocks);
  if (mode == MODE_ARGMAX) launch_shape<MODE_ARGMAX>(plan.shape, mt, grid, m->stream, a);
  else if (mode == MODE_SWIGLU) launch_shape<MODE_SWIGLU>(plan.shape, mt, grid, m->stream, a);
  else launch_shape<MODE_PARTIAL>(plan.shape, mt, grid, m->stream, a);
}
