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
// MFMA formulation (v_mfma_f32_16x16x32_bf16), chosen so that no operand needs a transpose
// or a cross-lane shuffle:
//   S^T[key][query] = K . Q^T     A = K tile from LDS (16 keys x 32 dims per step)
//                                 B = Q fragments, resident in registers
//   lane l then holds query (l % 16) and 4 keys of each 16-key tile, so the soft-max
//   maximum over keys is an in-lane max plus two xor-shuffles (16, 32), and the exponentials
//   of two 16-key tiles pack straight into the B operand of
//   O^T[dim][query] += V^T . P^T  A = V^T tile from LDS.  V pages are stored transposed in
//                                 the cache ([head_dim][16 tokens]) exactly for this.
// Soft-max is the running-max / rescale recurrence in fp32 on scores in log2 units, with the
// reference rounded up to a whole number so that every rescale is an exact power of two;
// probabilities 2^(s - ref) are rounded to bf16 for the second product and the row sum
// accumulates those rounded values.
// Partial (max, sum, O) per split are combined by k_attn_merge.
#include <stdlib.h>

#include "ts_internal.h"
#include "ts_device_utils.h"

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

namespace {

constexpr int KB = TS_ATTN_KB;   // keys per block

struct AttnArgs {
  const bf16_t* Qb;          // [rows][Hq*HD]
  const uint64_t* row_anc;   // [rows]
  const SeqDesc* seqs;
  float* part_o;             // [splits][R][Hq][HD]
  float* part_ml;            // [splits][R][Hq][2]
  int layer, Hq, Hkv, R, splits;
  float scale;               // 1/sqrt(head_dim) * log2(e): scores are kept in log2 units
};

union Pack8 {
  bf16x8 v;
  u32x2 h[2];
  uint32_t u[4];
};

template <int HD, int MT, int HB, int RS>
__global__ __launch_bounds__(64 * HB * RS) void k_attn_bf16(AttnArgs a) {
  constexpr int KSQ = HD / 32;            // k-steps of the score product
  constexpr int DT = HD / 16;             // 16-dim tiles of the output
  constexpr int NTHR = 64 * HB * RS;
  constexpr int VPP = 2 * HD;             // 16-byte vectors per K page (and per V page)
  constexpr int NVEC = 4 * 2 * VPP;       // 16-byte vectors per key block (K and V)
  constexpr int NV = (NVEC + NTHR - 1) / NTHR;  // staged vectors per thread and block
  __shared__ __attribute__((aligned(16))) bf16_t ks_[2][KB][HD + 8];
  __shared__ __attribute__((aligned(16))) bf16_t vs_[2][4][HD][16];

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int l15 = lane & 15, g4 = lane >> 4;
  const int G = a.Hq / a.Hkv;
  const int subs = G / HB;
  const int g = blockIdx.y / subs;
  const int h = g * G + (blockIdx.y % subs) * HB + (wave % HB);
  const int tile0 = (wave / HB) * MT;     // first 16-row tile of this wave
  const SeqDesc sd = a.seqs[blockIdx.z];
  const int P = sd.P, M = sd.M, T = P + M;
  const int n_blk = (T + KB - 1) / KB;
  const int bps = (n_blk + a.splits - 1) / a.splits;
  const int b0 = blockIdx.x * bps;
  const int b1 = min(n_blk, b0 + bps);

  const size_t page_elems = (size_t)a.Hkv * 16 * HD;
  const bf16_t* kl = (const bf16_t*)sd.k_pool + (size_t)a.layer * sd.n_pages * page_elems + (size_t)g * 16 * HD;
  const bf16_t* vl = (const bf16_t*)sd.v_pool + (size_t)a.layer * sd.n_pages * page_elems + (size_t)g * 16 * HD;

  // resident query fragments and ancestor masks of this wave's head
  bf16x8 qf[MT][KSQ];
  uint64_t anc[MT];
#pragma unroll
  for (int mt = 0; mt < MT; ++mt) {
    const int lrow = (tile0 + mt) * 16 + l15;
    const bf16_t* qp = a.Qb + (size_t)(sd.row0 + lrow) * a.Hq * HD + (size_t)h * HD + g4 * 8;
#pragma unroll
    for (int ks = 0; ks < KSQ; ++ks) qf[mt][ks] = *reinterpret_cast<const bf16x8*>(qp + ks * 32);
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

  u32x4 stage[NV];
  auto load_block = [&](int blk) {
#pragma unroll
    for (int i = 0; i < NV; ++i) {
      const int v = tid + i * NTHR;
      const int p = v / (2 * VPP), w = v % (2 * VPP);
      const int lp = blk * 4 + p;
      u32x4 val = u32x4{0u, 0u, 0u, 0u};
      if ((NVEC % NTHR == 0 || v < NVEC) && lp < sd.n_pages && lp * 16 < T) {
        const size_t pg = (size_t)sd.page_table[lp] * page_elems;
        const bf16_t* src = (w < VPP) ? (kl + pg + (size_t)w * 8) : (vl + pg + (size_t)(w - VPP) * 8);
        val = *reinterpret_cast<const u32x4*>(src);
      }
      stage[i] = val;
    }
  };
  auto store_block = [&](int buf) {
#pragma unroll
    for (int i = 0; i < NV; ++i) {
      const int v = tid + i * NTHR;
      const int p = v / (2 * VPP), w = v % (2 * VPP);
      if (NVEC % NTHR != 0 && v >= NVEC) continue;
      if (w < VPP) {
        const int t = w / (HD / 8), dv = w % (HD / 8);
        *reinterpret_cast<u32x4*>(&ks_[buf][p * 16 + t][dv * 8]) = stage[i];
      } else {
        const int w2 = w - VPP;
        *reinterpret_cast<u32x4*>(&vs_[buf][p][w2 >> 1][(w2 & 1) * 8]) = stage[i];
      }
    }
  };

  if (b0 < b1) {
    load_block(b0);
    store_block(0);
  }
  __syncthreads();

  for (int blk = b0; blk < b1; ++blk) {
    const int cur = (blk - b0) & 1;
    const bool more = blk + 1 < b1;
    if (more) load_block(blk + 1);

    // Two sub-blocks of 32 keys (2 pages) each: scores, mask, running soft-max, P.V.
    const int key0 = blk * KB;
    const bool masked = key0 + KB > P;
#pragma unroll 1   // keeping the two halves rolled holds the register need at 256
    for (int k2 = 0; k2 < 2; ++k2) {
      // ---- S^T = K . Q^T -----------------------------------------------------------
      f32x4 s[2][MT];
#pragma unroll
      for (int kt = 0; kt < 2; ++kt) {
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) s[kt][mt] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int ks = 0; ks < KSQ; ++ks) {
          const bf16x8 ka = *reinterpret_cast<const bf16x8*>(&ks_[cur][(2 * k2 + kt) * 16 + l15][ks * 32 + g4 * 8]);
#pragma unroll
          for (int mt = 0; mt < MT; ++mt)
            s[kt][mt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(ka, qf[mt][ks], s[kt][mt], 0, 0, 0);
        }
      }

      // ---- scale, mask ---------------------------------------------------------------
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
              s[kt][mt][r] = vis ? s[kt][mt][r] * a.scale : -INFINITY;
            }
          }
      } else {
#pragma unroll
        for (int kt = 0; kt < 2; ++kt)
#pragma unroll
          for (int mt = 0; mt < MT; ++mt) s[kt][mt] *= a.scale;
      }

      // ---- running soft-max ------------------------------------------------------------
      Pack8 pb[MT];
#pragma unroll
      for (int mt = 0; mt < MT; ++mt) {
        float mx = -INFINITY;
#pragma unroll
        for (int kt = 0; kt < 2; ++kt)
#pragma unroll
          for (int r = 0; r < 4; ++r) mx = fmaxf(mx, s[kt][mt][r]);
        mx = fmaxf(mx, __shfl_xor(mx, 16, 64));
        mx = fmaxf(mx, __shfl_xor(mx, 32, 64));
        // the running reference is a whole number (scores are in log2 units): rescaling by
        // exact powers of two commutes with the bf16 rounding of the probabilities, so the
        // result does not depend on how keys are blocked or split
        const float m_new = fmaxf(m_run[mt], ceilf(mx));
        const float m_use = (m_new == -INFINITY) ? 0.f : m_new;
        const float alpha = exp2f(m_run[mt] - m_use);
        m_run[mt] = m_new;
        float psum = 0.f;
#pragma unroll
        for (int kt = 0; kt < 2; ++kt)
#pragma unroll
          for (int r = 0; r < 4; r += 2) {
            const bf16_t p0 = f32_to_bf16(exp2f(s[kt][mt][r] - m_use));
            const bf16_t p1 = f32_to_bf16(exp2f(s[kt][mt][r + 1] - m_use));
            psum += bf16_to_f32(p0) + bf16_to_f32(p1);
            pb[mt].u[kt * 2 + (r >> 1)] = (uint32_t)p0 | ((uint32_t)p1 << 16);
          }
        l_run[mt] = l_run[mt] * alpha + psum;
#pragma unroll
        for (int dt = 0; dt < DT; ++dt) o[dt][mt] *= alpha;
      }

      // ---- O^T += V^T . P^T --------------------------------------------------------------
#pragma unroll
      for (int dt = 0; dt < DT; ++dt) {
        Pack8 va;
        va.h[0] = *reinterpret_cast<const u32x2*>(&vs_[cur][2 * k2][dt * 16 + l15][g4 * 4]);
        va.h[1] = *reinterpret_cast<const u32x2*>(&vs_[cur][2 * k2 + 1][dt * 16 + l15][g4 * 4]);
#pragma unroll
        for (int mt = 0; mt < MT; ++mt)
          o[dt][mt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(va.v, pb[mt].v, o[dt][mt], 0, 0, 0);
      }
    }

    if (more) store_block(cur ^ 1);
    __syncthreads();
  }

  // ---- partial results of this split ---------------------------------------------------
#pragma unroll
  for (int mt = 0; mt < MT; ++mt) {
    float l = l_run[mt];
    l += __shfl_xor(l, 16, 64);
    l += __shfl_xor(l, 32, 64);
    const int lrow = (tile0 + mt) * 16 + l15;
    if (lrow < M) {
      const size_t base = ((size_t)blockIdx.x * a.R + sd.row0 + lrow) * a.Hq + h;
      if (g4 == 0) {
        a.part_ml[base * 2 + 0] = m_run[mt];
        a.part_ml[base * 2 + 1] = l;
      }
#pragma unroll
      for (int dt = 0; dt < DT; ++dt)
        *reinterpret_cast<f32x4*>(a.part_o + base * HD + dt * 16 + g4 * 4) = o[dt][mt];
    }
  }
}

// Combine the splits: out = sum_s 2^(m_s - m*) O_s / sum_s 2^(m_s - m*) l_s, stored as bf16.
__global__ void k_attn_merge(const float* __restrict__ part_o, const float* __restrict__ part_ml,
                             bf16_t* __restrict__ Ab, int R, int Hq, int HD, int splits) {
  const int r = blockIdx.x, h = blockIdx.y, dd = threadIdx.x;
  float mstar = -INFINITY;
  for (int s = 0; s < splits; ++s) mstar = fmaxf(mstar, part_ml[(((size_t)s * R + r) * Hq + h) * 2]);
  float num = 0.f, den = 0.f;
  for (int s = 0; s < splits; ++s) {
    const size_t base = ((size_t)s * R + r) * Hq + h;
    const float ms = part_ml[base * 2];
    if (ms == -INFINITY) continue;
    const float w = exp2f(ms - mstar);      // both are whole numbers: an exact power of two
    den += w * part_ml[base * 2 + 1];
    num += w * part_o[base * HD + dd];
  }
  Ab[(size_t)r * Hq * HD + (size_t)h * HD + dd] = f32_to_bf16(num / den);
}

// Rows are covered by RS waves per head, MT tiles of 16 rows each: (tiles -> RS x MT)
// 1 -> 1x1, 2 -> 1x2, 3 -> 1x3, 4 -> 2x2, 5 -> 2x3.  Two row-splits put two waves on every
// SIMD (256 registers each) and let one wave's soft-max arithmetic overlap the other's MFMAs.
template <int HD, int HB>
void launch_hb(int tiles, dim3 grid, hipStream_t s, const AttnArgs& a) {
  switch (tiles) {
    case 1: hipLaunchKernelGGL((k_attn_bf16<HD, 1, HB, 1>), grid, dim3(64 * HB), 0, s, a); break;
    case 2: hipLaunchKernelGGL((k_attn_bf16<HD, 2, HB, 1>), grid, dim3(64 * HB), 0, s, a); break;
    case 3: hipLaunchKernelGGL((k_attn_bf16<HD, 3, HB, 1>), grid, dim3(64 * HB), 0, s, a); break;
    case 4: hipLaunchKernelGGL((k_attn_bf16<HD, 2, HB, 2>), grid, dim3(128 * HB), 0, s, a); break;
    default: hipLaunchKernelGGL((k_attn_bf16<HD, 3, HB, 2>), grid, dim3(128 * HB), 0, s, a); break;
  }
}

template <int HD>
void launch_hd(int hb, int tiles, dim3 grid, hipStream_t s, const AttnArgs& a) {
  if (hb == 4) launch_hb<HD, 4>(tiles, grid, s, a);
  else if (hb == 2) launch_hb<HD, 2>(tiles, grid, s, a);
  else launch_hb<HD, 1>(tiles, grid, s, a);
}

int heads_per_block(int G) { return G >= 4 ? 4 : (G >= 2 ? 2 : 1); }

}  // namespace

// Number of key splits: enough workgroups to cover the CUs, never more than key blocks.
int attn_bf16_splits(const ts_model* m, int max_keys, int n_seqs) {
  const int G = m->cfg.n_q_heads / m->cfg.n_kv_heads;
  const int per_split = m->cfg.n_kv_heads * (G / heads_per_block(G)) * n_seqs;
  const int n_blk = (max_keys + KB - 1) / KB;
  int want = (m->n_cu + per_split - 1) / per_split;
  if (want < 1) want = 1;
  if (want > n_blk) want = n_blk;
  if (const char* e = getenv("TS_ATTN_MAX_SPLITS")) {   // tuning / debugging knob
    const int cap = atoi(e);
    if (cap >= 1 && want > cap) want = cap;
  }
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
  dim3 grid(splits, c.n_kv_heads * (G / hb), n_seqs);
  const int mt = (max_M + 15) / 16;
  if (c.head_dim == 128) launch_hd<128>(hb, mt, grid, m->stream, a);
  else launch_hd<64>(hb, mt, grid, m->stream, a);
}

void launch_attn_merge(ts_model* m, int R, int splits) {
  ProfScope ps(m, "attn_merge");
  const ts_model_config& c = m->cfg;
  hipLaunchKernelGGL(k_attn_merge, dim3(R, c.n_q_heads), dim3(c.head_dim), 0, m->stream, m->attn_part_o, m->attn_part_ml,
                     (bf16_t*)m->Ab, R, c.n_q_heads, c.head_dim, splits);
}
