// Tree-masked grouped-query attention of the draft rows over the paged KV cache (bf16, gfx950).
//
// Every row of a sequence attends to all committed positions [0, P), to the root row and
// to its own ancestors among the tree rows, whose K/V were just written to slots
// P .. P+M-1 (paper App. A.1: one forward pass with a tree-structured mask).  The mask is a
// 64-bit ancestor set per row plus "root is always visible"; it only matters for the key
// blocks that overlap [P, P+M).
//
// Work split: grid = (key splits, KV head x head group, sequence).  A workgroup streams
// its key range once in blocks of 64 keys (4 pages) through double-buffered LDS and serves
// up to 4 query heads of the same KV head, one wave per head, all M rows of that head per
// wave - so each K/V byte is read from HBM once per KV head.
//
// The two products run in IEEE half precision (v_mfma_f32_16x16x32_f16): the cache stays bf16
// and its entries are widened to half while they are staged into LDS (exact in half's normal
// range), Q arrives in half, and the probabilities are rounded to half - 11 significant bits
// instead of bf16's 8 where it matters most for the logits.
//
// MFMA formulation, chosen so that no operand needs a transpose or a cross-lane shuffle:
//   S^T[key][query] = K . Q^T     A = K tile from LDS (16 keys x 32 dims per step)
//                                 B = Q fragments, resident in registers
//   lane l then holds query (l % 16) and 4 keys of each 16-key tile, so the soft-max
//   maximum over keys is an in-lane max plus two lane swaps (16, 32), and the exponentials
//   of two 16-key tiles pack straight into the B operand of
//   O^T[dim][query] += V^T . P^T  A = V^T tile from LDS.  V pages are stored transposed in
//                                 the cache ([head_dim][16 tokens]) exactly for this.
// Soft-max is the running-max / rescale recurrence in fp32 on scores in log2 units, with a
// whole-number reference (the rounded-up maximum, followed lazily: see kRefSlack) so that every
// rescale is an exact power of two;
// probabilities 2^(s - ref) are rounded to half for the second product and the row sum
// accumulates those rounded values (an extra MFMA against an all-ones operand, fp32 exact).
// Partial (max, sum, O) per split are combined by k_attn_merge.
#include <type_traits>

#include "ts_internal.h"
#include "ts_device_utils.h"

typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

namespace {

constexpr int KB = TS_ATTN_KB;   // keys per block

struct AttnArgs {
  const bf16_t* Qb;          // [rows][Hq*HD], IEEE half bit patterns
  const uint64_t* row_anc;   // [rows]
  const SeqDesc* seqs;
  uint16_t* part_o;          // [R][Hq][splits][HD], IEEE half: the split's output divided by its row sum
  float* part_ml;            // [R][Hq][splits][2]
  int layer, Hq, Hkv, R, splits, n_seqs;
  float scale;               // 1/sqrt(head_dim) * log2(e): scores are kept in log2 units
};

// 8 cache entries bf16 -> half (exact in half's normal range), done while staging into LDS
__device__ __forceinline__ u32x4 to_half8(u32x4 v) {
  return u32x4{bf16x2_to_f16x2(v.x), bf16x2_to_f16x2(v.y), bf16x2_to_f16x2(v.z), bf16x2_to_f16x2(v.w)};
}

// The running soft-max reference of a row follows its maximum lazily: it moves only when the
// rounded-up maximum exceeds it by more than this many powers of two.  Probabilities then reach
// 2^kRefSlack at most (half holds 2^15), every rescale stays an exact power of two, and the O
// rescale - 32 multiplies per row tile whenever any row of the wave moves its reference - runs a
// few times per row instead of at most half blocks of a long context.
constexpr float kRefSlack = 8.f;

union Pack8 {
  f16x8 v;
  u32x2 h[2];
  uint32_t u[4];
};

// MT0 row tiles for the waves of the first row split, MT1 (0 = no second split) for the second
template <int HD, int MT0, int MT1, int HB>
__global__ __launch_bounds__(64 * HB * (MT1 > 0 ? 2 : 1), (HB * (MT1 > 0 ? 2 : 1) <= 4) ? 2 : 1) void k_attn_bf16(AttnArgs a) {
  constexpr int RS = MT1 > 0 ? 2 : 1;
  constexpr int KSQ = HD / 32;            // k-steps of the score product
  constexpr int DT = HD / 16;             // 16-dim tiles of the output
  constexpr int NTHR = 64 * HB * RS;
  constexpr int VPP = 2 * HD;             // 16-byte vectors per K page (and per V page)
  constexpr int VTS = 40;                 // LDS row stride of the V^T of a 32-key half block, in tokens
  constexpr int VPG = 2 * VPP;            // 16-byte vectors per page, K then V
  constexpr int JP = (VPG + NTHR - 1) / NTHR;   // staged vectors per thread and page
  constexpr int NV = 4 * JP;              // staged vectors per thread and key block
  __shared__ __attribute__((aligned(16))) bf16_t ks_[2][KB][HD + 8];
  // V^T of a half block (2 pages = 32 keys): per head-dim row, the keys in the order the second
  // MFMA wants them - lane group g holds tokens 4g..4g+3 of the first page, then of the second -
  // so that a lane's operand is one 16-byte read.  Rows are padded to 40 tokens (80 B): 16 lanes
  // reading 16 B from 16 consecutive rows then fall into 16 distinct groups of 4 banks.
  __shared__ __attribute__((aligned(16))) bf16_t vs_[2][2][HD][VTS];

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int l15 = lane & 15, g4 = lane >> 4;
  const int G = a.Hq / a.Hkv;
  const int subs = G / HB;
  // Workgroups are dealt to the 8 XCDs round-robin by linear id.  The `subs` workgroups that
  // share one (sequence, KV head, key split) read the same K/V, so they are given ids that
  // differ by 8: same XCD, same L2, dispatched back to back.
  const int bid = blockIdx.x;
  const int jj = bid >> 3;
  const int rest = (jj / subs) * 8 + (bid & 7);
  if (rest >= a.splits * a.Hkv * a.n_seqs) return;
  const int split = rest % a.splits;
  const int g = (rest / a.splits) % a.Hkv;
  const int h = g * G + (jj % subs) * HB + (wave % HB);
  const int tile0 = (wave / HB) * MT0;    // first 16-row tile of this wave
  const SeqDesc sd = a.seqs[rest / (a.splits * a.Hkv)];
  const int P = sd.P, M = sd.M, T = P + M;
  const int n_blk = (T + KB - 1) / KB;
  const int bps = (n_blk + a.splits - 1) / a.splits;
  const int b0 = split * bps;
  const int b1 = min(n_blk, b0 + bps);

  const size_t page_elems = (size_t)a.Hkv * 16 * HD;
  const TS_GLOBAL bf16_t* kl = (const TS_GLOBAL bf16_t*)sd.k_pool + (size_t)a.layer * sd.n_pages * page_elems + (size_t)g * 16 * HD;
  const TS_GLOBAL bf16_t* vl = (const TS_GLOBAL bf16_t*)sd.v_pool + (size_t)a.layer * sd.n_pages * page_elems + (size_t)g * 16 * HD;
  const TS_GLOBAL int32_t* ptab = (const TS_GLOBAL int32_t*)sd.page_table;

  // Staging of one key block (4 pages).  A thread always fetches the same vector of a page
  // (K vectors for the first VPP thread ids, V vectors after), so its source pointer is fixed
  // and a page only adds a wave-uniform offset: one scalar page-table load and no vector
  // address arithmetic per page.  Pages past the last key are clamped to the last one: their
  // keys are masked in the scores and their V entries (finite cache contents) meet zero
  // probabilities.
  const TS_GLOBAL bf16_t* my_src[JP];
#pragma unroll
  for (int j = 0; j < JP; ++j) {
    const int w = min(tid + j * NTHR, VPG - 1);
    my_src[j] = (w < VPP) ? (kl + (size_t)w * 8) : (vl + (size_t)(w - VPP) * 8);
  }
  // Page-table entries of a key block: one 16-byte load (the table is padded by four entries of
  // page 0), fetched a block ahead of the data loads that need it and moved to scalar registers
  // there.  Pages past the last key hold finite cache contents.
  typedef int32_t i32x4 __attribute__((ext_vector_type(4)));
  auto load_pt = [&](int blk) { return *reinterpret_cast<const TS_GLOBAL i32x4*>(ptab + blk * 4); };
  u32x4 stage[NV];
  auto load_block = [&](const i32x4& pt) {
#pragma unroll
    for (int p = 0; p < 4; ++p) {
      const size_t pg = (size_t)__builtin_amdgcn_readfirstlane(pt[p]) * page_elems;
#pragma unroll
      for (int j = 0; j < JP; ++j)
        if (VPG % NTHR == 0 || tid + j * NTHR < VPG) stage[p * JP + j] = *reinterpret_cast<const TS_GLOBAL u32x4*>(my_src[j] + pg);
    }
  };
  auto store_block = [&](int buf) {
#pragma unroll
    for (int p = 0; p < 4; ++p)
#pragma unroll
      for (int j = 0; j < JP; ++j) {
        const int w = tid + j * NTHR;
        if (VPG % NTHR != 0 && w >= VPG) continue;
        if (w < VPP) {
          const int t = w / (HD / 8), dv = w % (HD / 8);
          *reinterpret_cast<u32x4*>(&ks_[buf][p * 16 + t][dv * 8]) = to_half8(stage[p * JP + j]);
        } else {
          const int w2 = w - VPP;
          const u32x4 v = to_half8(stage[p * JP + j]);     // 8 tokens of one head-dim row
          // tokens 8 (w2 & 1) .. +8 of page p: two groups of 4, lane groups 2 (w2 & 1) and 2 (w2 & 1) + 1
          *reinterpret_cast<u32x2*>(&vs_[buf][p >> 1][w2 >> 1][(w2 & 1) * 16 + (p & 1) * 4]) = u32x2{v.x, v.y};
          *reinterpret_cast<u32x2*>(&vs_[buf][p >> 1][w2 >> 1][(w2 & 1) * 16 + 8 + (p & 1) * 4]) = u32x2{v.z, v.w};
        }
      }
  };

  // The main loop, compiled once per tile count: the waves of the second row split usually own
  // fewer tiles (5 tiles = 3 + 2) and run a copy without the empty one.  Both copies execute
  // the same barriers.
  auto body = [&](auto mt_c) {
    constexpr int MT = decltype(mt_c)::value;
    // LDS operand fragments requested ahead of the MFMAs that consume them; 0 leaves the order to
    // the compiler (which requests a pair, waits, multiplies).  The explicit pipeline pays in the
    // 8-wave variants with two row splits (65 rows: -4 % with 4 query heads per KV head, -9 %
    // with 8) and loses elsewhere (+8 % at 33 rows with one row split), measured.
    constexpr int FD = (RS == 2 && HB == 4) ? 3 : 0;
  // resident query fragments and ancestor masks of this wave's head
  f16x8 qf[MT][KSQ];
  uint64_t anc[MT];
#pragma unroll
  for (int mt = 0; mt < MT; ++mt) {
    const int lrow = (tile0 + mt) * 16 + l15;
    const bf16_t* qp = a.Qb + (size_t)(sd.row0 + lrow) * a.Hq * HD + (size_t)h * HD + g4 * 8;
#pragma unroll
    for (int ks = 0; ks < KSQ; ++ks) qf[mt][ks] = *reinterpret_cast<const f16x8*>(qp + ks * 32);
    anc[mt] = lrow < M ? a.row_anc[sd.row0 + lrow] : 0ull;
  }

  f32x4 o[DT][MT];
  float m_run[MT], l_run[MT];
#pragma unroll
  for (int mt = 0; mt < MT; ++mt) {
    m_run[mt] = -INFINITY;
    l_run[mt] = 0.f;
#pragma unroll
    for (int dt = 0; dt < DT; ++dt) o[dt][mt] = f32x4{0.f, 0.f, 0.f, 0.f};
  }

  Pack8 ones;
#pragma unroll
  for (int i = 0; i < 4; ++i) ones.u[i] = 0x3c003c00u;   // half 1.0 x 8

  i32x4 pt_next = i32x4{0, 0, 0, 0};
  if (b0 < b1) {
    load_block(load_pt(b0));
    if (b0 + 1 < b1) pt_next = load_pt(b0 + 1);
    store_block(0);
  }
  // Every load issued so far (query fragments, ancestor masks, first block) is complete past
  // this point.  Without the explicit wait the compiler has to assume, at the loop head, that
  // the query loads may still be in flight, and guards the first MFMA of every pass with a
  // wait for ALL vector loads - which would include the next block's K/V just requested.
  __builtin_amdgcn_s_waitcnt(0x0F70);       // vmcnt(0)
  __syncthreads();

  for (int blk = b0; blk < b1; ++blk) {
    const int cur = (blk - b0) & 1;
    const bool more = blk + 1 < b1;
    if (more) {
      load_block(pt_next);
      if (blk + 2 < b1) pt_next = load_pt(blk + 2);
    }

    // Two sub-blocks of 32 keys (2 pages) each: scores, mask, running soft-max, P.V.
    const int key0 = blk * KB;
    const bool masked = key0 + KB > P;
#pragma unroll 1   // keeping the two halves rolled holds the register need at 256
    for (int k2 = 0; k2 < 2; ++k2) {
      // ---- S^T = K . Q^T -----------------------------------------------------------
      // With FD > 0 the K fragments come from LDS through a short software pipeline, FD of them
      // in flight ahead of the MFMAs that consume them; the scheduling barriers keep the stages
      // in this order.
      f32x4 s[2][MT];
#pragma unroll
      for (int kt = 0; kt < 2; ++kt)
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) s[kt][mt] = f32x4{0.f, 0.f, 0.f, 0.f};
      constexpr int NKF = 2 * KSQ;
      static_assert(FD <= NKF && FD <= DT, "pipeline deeper than the fragment count");
      auto k_frag = [&](int i) {
        return *reinterpret_cast<const f16x8*>(&ks_[cur][(2 * k2 + i / KSQ) * 16 + l15][(i % KSQ) * 32 + g4 * 8]);
      };
      auto v_frag = [&](int dt) { return *reinterpret_cast<const f16x8*>(&vs_[cur][k2][dt * 16 + l15][g4 * 8]); };
      f16x8 kf[NKF];
#pragma unroll
      for (int i = 0; i < FD; ++i) kf[i] = k_frag(i);
      if (FD > 0) __builtin_amdgcn_sched_barrier(0);
#pragma unroll
      for (int i = 0; i < NKF; ++i) {
        if (FD == 0) kf[i] = k_frag(i);
        else if (i + FD < NKF) kf[i + FD] = k_frag(i + FD);
#pragma unroll
        for (int mt = 0; mt < MT; ++mt)
          s[i / KSQ][mt] = __builtin_amdgcn_mfma_f32_16x16x32_f16(kf[i], qf[mt][i % KSQ], s[i / KSQ][mt], 0, 0, 0);
        if (FD > 0) __builtin_amdgcn_sched_barrier(0);
      }
      // the first V^T fragments of the second product travel while the soft-max is computed
      f16x8 vf[DT];
#pragma unroll
      for (int dt = 0; dt < FD; ++dt) vf[dt] = v_frag(dt);
      if (FD > 0) __builtin_amdgcn_sched_barrier(0);

      // ---- mask (only blocks that reach past the committed context) ----------------------
      if (masked) {
#pragma unroll
        for (int kt = 0; kt < 2; ++kt)
#pragma unroll
          for (int r = 0; r < 4; ++r) {
            const int key = key0 + (2 * k2 + kt) * 16 + g4 * 4 + r;
            const int srow = key - P;                      // tree row of this key (if >= 0)
#pragma unroll
            for (int mt = 0; mt < MT; ++mt) {
              bool vis = key < T;
              if (vis && srow > 0) vis = (anc[mt] >> (srow - 1)) & 1ull;
              if (!vis) s[kt][mt][r] = -INFINITY;
            }
          }
      }

      // ---- running soft-max on raw scores; a.scale = log2(e)/sqrt(hd) folds into the exponent ---
      Pack8 pb[MT];
      float alpha[MT];
      bool rescale = false;
#pragma unroll
      for (int mt = 0; mt < MT; ++mt) {
        float mx = -INFINITY;
#pragma unroll
        for (int kt = 0; kt < 2; ++kt)
#pragma unroll
          for (int r = 0; r < 4; ++r) mx = fmaxf(mx, s[kt][mt][r]);
        mx = max_over_lane_groups(mx);
        // the running reference is a whole number (scores in log2 units) that follows the
        // rounded-up maximum lazily (kRefSlack): every rescale is an exact power of two, which
        // commutes with the half rounding of the probabilities, so blocking and splitting of the
        // keys can change a probability only where it falls into half's subnormal range (below
        // 2^-14 of the reference's scale)
        const float m_ceil = ceilf(mx * a.scale);
        const float m_new = (m_ceil > m_run[mt] + kRefSlack) ? m_ceil : m_run[mt];
        const float m_use = (m_new == -INFINITY) ? 0.f : m_new;
        alpha[mt] = __builtin_amdgcn_exp2f(m_run[mt] - m_use);
        rescale |= (m_new != m_run[mt]);
        m_run[mt] = m_new;
#pragma unroll
        for (int kt = 0; kt < 2; ++kt)
#pragma unroll
          for (int r = 0; r < 4; r += 2)
            pb[mt].u[kt * 2 + (r >> 1)] = pack_f16x2(__builtin_amdgcn_exp2f(fmaf(s[kt][mt][r], a.scale, -m_use)),
                                                      __builtin_amdgcn_exp2f(fmaf(s[kt][mt][r + 1], a.scale, -m_use)));
      }
      // the reference moves rarely after the first blocks: skip the O rescale when no row's did
      if (__builtin_amdgcn_ballot_w64(rescale) != 0ull) {
#pragma unroll
        for (int mt = 0; mt < MT; ++mt)
#pragma unroll
          for (int dt = 0; dt < DT; ++dt) o[dt][mt] *= alpha[mt];
      }

      // ---- O^T += V^T . P^T ; row sums of the rounded probabilities from an all-ones operand ---
#pragma unroll
      for (int mt = 0; mt < MT; ++mt) {
        const f32x4 ps = __builtin_amdgcn_mfma_f32_16x16x32_f16(ones.v, pb[mt].v, f32x4{0.f, 0.f, 0.f, 0.f}, 0, 0, 0);
        l_run[mt] = fmaf(l_run[mt], alpha[mt], ps[0]);
      }
      if (FD > 0) __builtin_amdgcn_sched_barrier(0);
#pragma unroll
      for (int dt = 0; dt < DT; ++dt) {
        if (FD == 0) vf[dt] = v_frag(dt);
        else if (dt + FD < DT) vf[dt + FD] = v_frag(dt + FD);
#pragma unroll
        for (int mt = 0; mt < MT; ++mt)
          o[dt][mt] = __builtin_amdgcn_mfma_f32_16x16x32_f16(vf[dt], pb[mt].v, o[dt][mt], 0, 0, 0);
        if (FD > 0) __builtin_amdgcn_sched_barrier(0);
      }
    }

    if (more) store_block(cur ^ 1);
    __syncthreads();
  }

  // ---- partial results of this split ---------------------------------------------------
  // (reference, row sum) in fp32 and the split's own normalised output O / l in half: a convex
  // combination of V rows, so it can neither overflow nor lose more than half's 11 bits, the
  // precision the probabilities already have.  Half the bytes of fp32 partials, which is what
  // bounds this epilogue and the merge kernel.
#pragma unroll
  for (int mt = 0; mt < MT; ++mt) {
    const float l = l_run[mt];     // already the sum over all keys (MFMA reduces over the lane groups)
    const int lrow = (tile0 + mt) * 16 + l15;
    if (lrow < M) {
      const size_t base = ((size_t)(sd.row0 + lrow) * a.Hq + h) * a.splits + split;
      if (g4 == 0) {
        a.part_ml[base * 2 + 0] = m_run[mt];
        a.part_ml[base * 2 + 1] = l;
      }
      const float inv = l > 0.f ? 1.0f / l : 0.f;
#pragma unroll
      for (int dt = 0; dt < DT; ++dt)
        *reinterpret_cast<u32x2*>(a.part_o + base * HD + dt * 16 + g4 * 4) =
            u32x2{pack_f16x2(o[dt][mt][0] * inv, o[dt][mt][1] * inv), pack_f16x2(o[dt][mt][2] * inv, o[dt][mt][3] * inv)};
    }
  }
  };
  if (RS == 1 || wave / HB == 0) body(std::integral_constant<int, MT0>{});
  else body(std::integral_constant<int, (MT1 > 0 ? MT1 : MT0)>{});
}

// Combine the splits: out = sum_s w_s (O_s / l_s) / sum_s w_s with w_s = 2^(m_s - m*) l_s, stored as IEEE half.
// One workgroup per (row, head): its 256 threads form 256/(HD/4) groups, group j takes splits
// j, j+groups, ... so that every partial of the slot is requested at once (the kernel is a
// single round of memory latency plus the transfer); the groups' sums are then added through
// LDS in a fixed order.
constexpr int kMergeMaxSplits = 512;

__global__ __launch_bounds__(256) void k_attn_merge(const uint16_t* __restrict__ part_o, const float* __restrict__ part_ml,
                                                    f16_t* __restrict__ Ab, size_t a_plane, int R, int Hq, int HD, int splits,
                                                    unsigned long long* __restrict__ sat) {
  __shared__ float s_m[kMergeMaxSplits], s_l[kMergeMaxSplits];
  __shared__ float4 r_num[256];
  __shared__ float r_den[256];
  const int tid = threadIdx.x;
  const int tpp = HD / 4;                  // threads per group: four dims of the head each
  const int groups = 256 / tpp;
  const int grp = tid / tpp, d4 = tid % tpp;
  const size_t slot = blockIdx.x;
  const float2* ml = reinterpret_cast<const float2*>(part_ml);
  const uint2* po = reinterpret_cast<const uint2*>(part_o);     // 4 halves
  for (int sp = tid; sp < splits; sp += 256) {
    const float2 v = ml[slot * splits + sp];
    s_m[sp] = v.x;
    s_l[sp] = v.y;
  }
  uint2 o4[4];
#pragma unroll
  for (int u = 0; u < 4; ++u) {
    const int sp = grp + u * groups;
    o4[u] = sp < splits ? po[(slot * splits + sp) * tpp + d4] : make_uint2(0u, 0u);
  }
  __syncthreads();
  float mstar = -INFINITY;
  for (int sp = 0; sp < splits; ++sp) mstar = fmaxf(mstar, s_m[sp]);
  float4 num = make_float4(0.f, 0.f, 0.f, 0.f);
  float den = 0.f;
  for (int s0 = 0; s0 < splits; s0 += 4 * groups) {
    if (s0 > 0) {
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        const int sp = s0 + grp + u * groups;
        o4[u] = sp < splits ? po[(slot * splits + sp) * tpp + d4] : make_uint2(0u, 0u);
      }
    }
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      const int sp = s0 + grp + u * groups;
      if (sp < splits && s_m[sp] != -INFINITY) {
        const float w = exp2f(s_m[sp] - mstar) * s_l[sp];   // whole-number references: an exact power of two
        den += w;
        const ts_f16x2 lo2 = __builtin_bit_cast(ts_f16x2, o4[u].x), hi2 = __builtin_bit_cast(ts_f16x2, o4[u].y);
        num.x += w * (float)lo2[0]; num.y += w * (float)lo2[1]; num.z += w * (float)hi2[0]; num.w += w * (float)hi2[1];
      }
    }
  }
  r_num[tid] = num;
  r_den[tid] = den;
  __syncthreads();
  if (grp != 0) return;
  for (int k = 1; k < groups; ++k) {
    const float4 t = r_num[k * tpp + d4];
    num.x += t.x; num.y += t.y; num.z += t.z; num.w += t.w;
    den += r_den[k * tpp + d4];
  }
  // the attention output feeds the O projection as a hi and a lo half
  st_act_planes4(Ab + slot * HD + d4 * 4, a_plane, num.x / den, num.y / den, num.z / den, num.w / den, sat);
}

// Rows are covered by RS waves per head, MT tiles of 16 rows each: (tiles -> RS x MT)
// 1 -> 1, 2 -> 2, 3 -> 3, 4 -> 2+2, 5 -> 3+2.  Two row-splits put two waves on every
// SIMD (256 registers each) and let one wave's soft-max arithmetic overlap the other's MFMAs.
template <int HD, int HB>
void launch_hb(int tiles, dim3 grid, hipStream_t s, const AttnArgs& a) {
  switch (tiles) {
    case 1: hipLaunchKernelGGL((k_attn_bf16<HD, 1, 0, HB>), grid, dim3(64 * HB), 0, s, a); break;
    case 2: hipLaunchKernelGGL((k_attn_bf16<HD, 2, 0, HB>), grid, dim3(64 * HB), 0, s, a); break;
    case 3: hipLaunchKernelGGL((k_attn_bf16<HD, 3, 0, HB>), grid, dim3(64 * HB), 0, s, a); break;
    case 4: hipLaunchKernelGGL((k_attn_bf16<HD, 2, 2, HB>), grid, dim3(128 * HB), 0, s, a); break;
    default: hipLaunchKernelGGL((k_attn_bf16<HD, 3, 2, HB>), grid, dim3(128 * HB), 0, s, a); break;
  }
}

template <int HD>
void launch_hd(int hb, int tiles, dim3 grid, hipStream_t s, const AttnArgs& a) {
  if (hb == 4) launch_hb<HD, 4>(tiles, grid, s, a);
  else if (hb == 2) launch_hb<HD, 2>(tiles, grid, s, a);
  else launch_hb<HD, 1>(tiles, grid, s, a);
}

// query heads of one KV head served by a workgroup (one wave each per row split)
int heads_per_block(int G) { return G >= 4 ? 4 : (G >= 2 ? 2 : 1); }

}  // namespace

// Number of key splits (every sequence is cut into the same number of splits, each covering
// ceil(blocks / splits) of ITS key blocks).  One sequence: enough workgroups to cover the CUs
// once.  Several sequences of different lengths: one round would be as slow as the longest
// sequence's share, so the splits are made fine enough that the longest workgroup carries at
// most half of a CU's average load and the dispatcher can even the rest out over a few rounds.
int attn_bf16_splits(const ts_model* m, int max_keys, int n_seqs, long sum_keys) {
  const int G = m->cfg.n_q_heads / m->cfg.n_kv_heads;
  const int subs = G / heads_per_block(G);
  const int per_split = m->cfg.n_kv_heads * subs * n_seqs;
  const int n_blk = (max_keys + KB - 1) / KB;
  const int wg_per_cu = heads_per_block(G) <= 2 ? 2 : 1;
  int want = (wg_per_cu * m->n_cu + per_split - 1) / per_split;
  if (n_seqs > 1) {
    const double avg_per_cu = (double)((sum_keys + KB - 1) / KB) * m->cfg.n_kv_heads * subs / m->n_cu;
    const int fine = (int)((double)n_blk / (avg_per_cu > 2.0 ? avg_per_cu / 2.0 : 1.0) + 0.999);
    if (fine > want) want = fine < 16 ? fine : 16;          // partial sums grow with the split count
  }
  if (want < 1) want = 1;
  if (want > n_blk) want = n_blk;
  if (want > kMergeMaxSplits) want = kMergeMaxSplits;      // the merge kernel keeps (max, sum) of every split in LDS
  const int bps = (n_blk + want - 1) / want;
  return (n_blk + bps - 1) / bps;
}

void launch_attn_bf16(ts_model* m, const RowMeta& rm, int R, int n_seqs, int layer, int splits, int max_M) {
  ProfScope ps(m, "attn_bf16");
  const ts_model_config& c = m->cfg;
  AttnArgs a;
  a.Qb = (const bf16_t*)m->Qb; a.row_anc = rm.anc; a.seqs = m->seq_dev;
  a.part_o = m->attn_part_o; a.part_ml = m->attn_part_ml;
  a.layer = layer; a.Hq = c.n_q_heads; a.Hkv = c.n_kv_heads; a.R = R; a.splits = splits;
  a.scale = (float)(1.4426950408889634 / sqrt((double)c.head_dim));   // 1/sqrt(hd) * log2(e)
  const int G = c.n_q_heads / c.n_kv_heads;
  const int hb = heads_per_block(G);
  a.n_seqs = n_seqs;
  const int units = splits * c.n_kv_heads * n_seqs;        // (sequence, KV head, key split) triples
  dim3 grid(((units + 7) / 8) * 8 * (G / hb));
  const int mt = (max_M + 15) / 16;
  if (c.head_dim == 128) launch_hd<128>(hb, mt, grid, m->stream, a);
  else launch_hd<64>(hb, mt, grid, m->stream, a);
}

void launch_attn_merge(ts_model* m, int R, int splits) {
  ProfScope ps(m, "attn_merge");
  const ts_model_config& c = m->cfg;
  hipLaunchKernelGGL(k_attn_merge, dim3(R * c.n_q_heads), dim3(256), 0, m->stream, m->attn_part_o, m->attn_part_ml,
                     (f16_t*)m->Ab, (size_t)(m->ws_rows + TS_MROWS_PER_BLOCK) * m->q_dim, R, c.n_q_heads, c.head_dim, splits, m->sat_count);
}
