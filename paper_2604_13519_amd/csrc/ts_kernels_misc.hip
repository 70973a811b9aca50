// Row-wise and bookkeeping kernels of the verify pass, plus the fp32 compute path.
//
// Everything here is bandwidth-trivial next to the weight and K/V streams (a verify
// pass has at most a few hundred rows); the kernels are written for clarity and for
// few launches.  Storage type T is float (fp32 models) or bf16_t (bf16 models);
// arithmetic is fp32 everywhere, bf16 only when a value is stored.
#include "ts_internal.h"
#include "ts_device_utils.h"

// rotated queries: float, or IEEE half bits for bf16 models (the attention products run in
// half precision; bf16 K/V entries widen to half exactly)
__device__ __forceinline__ void st_q(float* p, float v) { *p = v; }
__device__ __forceinline__ void st_q(bf16_t* p, float v) { *p = f32_to_f16_bits(v); }

// store an activation that feeds a projection: float as is; for bf16 models as a hi and a lo
// IEEE half in two planes `plane` elements apart (hi saturating)
__device__ __forceinline__ void st_act(float* p, size_t, float v, unsigned long long*) { *p = v; }
__device__ __forceinline__ void st_act(f16_t* p, size_t plane, float v, unsigned long long* sat) { st_act_planes(p, plane, v, sat); }
// four consecutive activations (p 16-byte aligned in float terms): one vector store per plane
__device__ __forceinline__ void st_act4(float* p, size_t, const float4& v, unsigned long long*) { *reinterpret_cast<float4*>(p) = v; }
__device__ __forceinline__ void st_act4(f16_t* p, size_t plane, const float4& v, unsigned long long* sat) { st_act_planes4(p, plane, v.x, v.y, v.z, v.w, sat); }

// ---------------------------------------------------------------------------------
// weight re-tiling (model load): row-major [N][K] bf16 -> MFMA operand tiles of IEEE half.
// Tile (nt, kt) covers out-features [16 nt, 16 nt + 16) x in-features [32 kt, 32 kt + 32)
// and is stored as 64 lanes x 8 elements, lane l holding W[16 nt + l%16][32 kt + 8 (l/16) + e],
// i.e. exactly one wave-wide 16-byte-per-lane load.  Tiles of one nt are contiguous in kt.
// Destination tile index = n_tile0 + nt * n_tile_stride, which lets two matrices be
// interleaved tile by tile (gate / up).  Rows >= N are zero-filled.
// bf16 -> half is exact wherever half is normal (8 significand bits into 11); magnitudes below
// 2^-14 round to half's subnormal grid (absolute error below 3e-8).  A finite weight beyond
// half's range (> 65504) cannot be represented: *range_flag is set and the load fails.
// ---------------------------------------------------------------------------------
__global__ void k_repack_tiles(const bf16_t* __restrict__ src, f16_t* __restrict__ dst,
                               int N, int K, int n_tile0, int n_tile_stride, int* __restrict__ range_flag) {
  const int kt_count = K / 32;
  const size_t n_tiles = (size_t)((N + 15) / 16) * kt_count;
  bool bad = false;
  for (size_t v = (size_t)blockIdx.x * blockDim.x + threadIdx.x; v < n_tiles * 64;
       v += (size_t)gridDim.x * blockDim.x) {
    const int lane = (int)(v & 63);
    const size_t tile = v >> 6;
    const int nt = (int)(tile / kt_count), kt = (int)(tile % kt_count);
    const int n = nt * 16 + (lane & 15);
    const int k = kt * 32 + (lane >> 4) * 8;
    uint4 val = make_uint4(0, 0, 0, 0);
    if (n < N) val = *reinterpret_cast<const uint4*>(src + (size_t)n * K + k);
    const uint32_t w[4] = {val.x, val.y, val.z, val.w};
    uint32_t o[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const float a = __uint_as_float(w[i] << 16), b = __uint_as_float(w[i] & 0xffff0000u);
      bad |= (fabsf(a) > 65504.f && fabsf(a) < INFINITY) || (fabsf(b) > 65504.f && fabsf(b) < INFINITY);
      o[i] = pack_f16x2(a, b);
    }
    const size_t dtile = (size_t)(n_tile0 + nt * n_tile_stride) * kt_count + kt;
    *reinterpret_cast<uint4*>(dst + (dtile * 64 + lane) * 8) = make_uint4(o[0], o[1], o[2], o[3]);
  }
  if (bad) atomicOr(range_flag, 1);
}

void launch_repack_tiles(hipStream_t s, const bf16_t* src, f16_t* dst, int N, int K, int n_tile0,
                         int n_tile_stride, int* range_flag) {
  size_t vecs = (size_t)((N + 15) / 16) * (K / 32) * 64;
  int blocks = (int)((vecs + 255) / 256);
  if (blocks > 65535) blocks = 65535;
  hipLaunchKernelGGL(k_repack_tiles, dim3(blocks), dim3(256), 0, s, src, dst, N, K, n_tile0, n_tile_stride, range_flag);
}

// ---------------------------------------------------------------------------------
// Per-row set-up of a pass, one workgroup per row:
//  * embedding gather H[r][:] = E[tok[r]][:]  (the residual stream is fp32);
//  * rotary table (cos, sin)(pos[r] * theta^(-2j/hd)) for j < hd/2, evaluated in double so that
//    large positions lose no phase accuracy, stored as float;
//  * where the row's K and V go in its sequence's paged cache (layer 0; a layer adds
//    layer_stride elements), so that the per-layer QKV epilogue needs one load instead of the
//    chain row -> sequence -> page table.
// ---------------------------------------------------------------------------------
__device__ __forceinline__ void widen_store(float* h, const float* e) { *reinterpret_cast<float4*>(h) = *reinterpret_cast<const float4*>(e); }
__device__ __forceinline__ void widen_store(float* h, const bf16_t* e) {
  const uint2 v = *reinterpret_cast<const uint2*>(e);             // 4 bf16
  *reinterpret_cast<float4*>(h) = make_float4(__uint_as_float(v.x << 16), __uint_as_float(v.x & 0xffff0000u),
                                               __uint_as_float(v.y << 16), __uint_as_float(v.y & 0xffff0000u));
}

template <typename T>
__global__ __launch_bounds__(256) void k_embed_rope(const T* __restrict__ E, const int32_t* __restrict__ tok, float* __restrict__ H, int d,
                                                    const int32_t* __restrict__ pos, float2* __restrict__ cs, int half, double theta,
                                                    const int32_t* __restrict__ row_seq, const int32_t* __restrict__ row_lrow,
                                                    const SeqDesc* __restrict__ seqs, RowDst* __restrict__ dst, int Hkv) {
  const int r = blockIdx.x;
  const T* e = E + (size_t)tok[r] * d;
  if (d % 4 == 0) {
    for (int i = threadIdx.x * 4; i < d; i += blockDim.x * 4) widen_store(H + (size_t)r * d + i, e + i);
  } else {
    for (int i = threadIdx.x; i < d; i += blockDim.x) H[(size_t)r * d + i] = ld_f32(e + i);
  }
  for (int j = threadIdx.x; j < half; j += blockDim.x) {
    const double inv_freq = pow(theta, -(double)j / (double)half);
    const double ang = (double)pos[r] * inv_freq;
    cs[(size_t)r * half + j] = make_float2((float)cos(ang), (float)sin(ang));
  }
  if (threadIdx.x == blockDim.x - 1) {
    const SeqDesc sd = seqs[row_seq[r]];
    const int slot = sd.P + row_lrow[r];
    const int hd = 2 * half;
    const size_t page_elems = (size_t)Hkv * 16 * hd;
    const size_t pg = (size_t)sd.page_table[slot >> 4] * page_elems;
    RowDst o;
    o.k = (T*)sd.k_pool + pg + (size_t)(slot & 15) * hd;          // + g * 16 * hd + dim
    o.v = (T*)sd.v_pool + pg + (slot & 15);                        // + g * hd * 16 + dim * 16
    o.layer_stride = (size_t)sd.n_pages * page_elems;
    dst[r] = o;
  }
}

void launch_embed(ts_model* m, const RowMeta& rm, int R) {
  ProfScope ps(m, "embed_rope_table");
  const ts_model_config& c = m->cfg;
  if (c.dtype == TS_DTYPE_BF16)
    hipLaunchKernelGGL(k_embed_rope<bf16_t>, dim3(R), dim3(256), 0, m->stream, (const bf16_t*)m->embed, rm.tok, m->H, c.d_model, rm.pos,
                       m->rope_cs, c.head_dim / 2, (double)c.rope_theta, rm.seq, rm.lrow, m->seq_dev, m->row_dst, c.n_kv_heads);
  else
    hipLaunchKernelGGL(k_embed_rope<float>, dim3(R), dim3(256), 0, m->stream, (const float*)m->embed, rm.tok, m->H, c.d_model, rm.pos,
                       m->rope_cs, c.head_dim / 2, (double)c.rope_theta, rm.seq, rm.lrow, m->seq_dev, m->row_dst, c.n_kv_heads);
}

// ---------------------------------------------------------------------------------
// residual update + RMSNorm:  H[r] += sum_s part[s][r]  (skipped when n_parts = 0),
// Xn[r] = H[r] * rsqrt(mean(H[r]^2) + eps) * gain, stored as float (fp32 models) or as a hi and
// a lo IEEE half (bf16 models: every projection input is such a pair).
// One block of 1024 threads per row, 16-byte accesses; needs d_model % 4 == 0.
// ---------------------------------------------------------------------------------
template <typename T>
__global__ __launch_bounds__(1024) void k_norm(float* __restrict__ H, const float* __restrict__ part, int n_parts,
                                               size_t part_stride, const float* __restrict__ gain,
                                               T* __restrict__ Xn, size_t x_plane, int d, float eps,
                                               unsigned long long* __restrict__ sat) {
  __shared__ float red[16];
  const int r = blockIdx.x;
  float4* h4 = reinterpret_cast<float4*>(H + (size_t)r * d);
  const float4* p4 = reinterpret_cast<const float4*>(part + (size_t)r * d);
  const float4* g4 = reinterpret_cast<const float4*>(gain);
  const size_t stride4 = part_stride / 4;
  const int d4 = d / 4;
  // the first KEEP vectors of a thread stay in registers between the two passes (d_model up
  // to 8192 never re-reads the residual); their gains are requested together with the data
  constexpr int KEEP = 2;
  float4 keep[KEEP], gk[KEEP];
  float ss = 0.f;
  auto updated = [&](int i) {
    float4 v = h4[i];
    if (n_parts > 0) {
      // all partial loads of a batch are issued before the first add (fixed summation order)
      for (int s0 = 0; s0 < n_parts; s0 += 8) {
        float4 q[8];
#pragma unroll
        for (int j = 0; j < 8; ++j)
          q[j] = (s0 + j < n_parts) ? p4[(size_t)(s0 + j) * stride4 + i] : make_float4(0.f, 0.f, 0.f, 0.f);
#pragma unroll
        for (int j = 0; j < 8; ++j) { v.x += q[j].x; v.y += q[j].y; v.z += q[j].z; v.w += q[j].w; }
      }
      h4[i] = v;
    }
    ss += v.x * v.x + v.y * v.y + v.z * v.z + v.w * v.w;
    return v;
  };
#pragma unroll
  for (int k = 0; k < KEEP; ++k) {
    const int i = threadIdx.x + k * 1024;
    if (i < d4) { gk[k] = g4[i]; keep[k] = updated(i); }
  }
  for (int i = threadIdx.x + KEEP * 1024; i < d4; i += 1024) updated(i);
  ss = wave_sum(ss);
  if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = ss;
  __syncthreads();
  float tot = 0.f;
#pragma unroll
  for (int w = 0; w < 16; ++w) tot += red[w];
  const float inv = 1.0f / sqrtf(tot / (float)d + eps);
  auto emit = [&](int i, const float4& v, const float4& g) {
    st_act4(Xn + (size_t)r * d + 4 * i, x_plane, make_float4(v.x * inv * g.x, v.y * inv * g.y, v.z * inv * g.z, v.w * inv * g.w), sat);
  };
#pragma unroll
  for (int k = 0; k < KEEP; ++k) {
    const int i = threadIdx.x + k * 1024;
    if (i < d4) emit(i, keep[k], gk[k]);
  }
  for (int i = threadIdx.x + KEEP * 1024; i < d4; i += 1024) emit(i, h4[i], g4[i]);
}

void launch_norm(ts_model* m, int R, const float* gain, int n_parts, size_t part_stride, bool) {
  ProfScope ps(m, "residual_rmsnorm");
  if (m->cfg.dtype == TS_DTYPE_BF16)
    hipLaunchKernelGGL(k_norm<f16_t>, dim3(R), dim3(1024), 0, m->stream, m->H, m->part, n_parts, part_stride, gain,
                       (f16_t*)m->Xn, (size_t)(m->ws_rows + TS_MROWS_PER_BLOCK) * m->cfg.d_model, m->cfg.d_model, m->cfg.rms_eps, m->sat_count);
  else
    hipLaunchKernelGGL(k_norm<float>, dim3(R), dim3(1024), 0, m->stream, m->H, m->part, n_parts, part_stride, gain,
                       (float*)m->Xn, (size_t)0, m->cfg.d_model, m->cfg.rms_eps, (unsigned long long*)nullptr);
}

// ---------------------------------------------------------------------------------
// QKV epilogue: sum split-K partials, rotate Q and K at the row's position, store Q for
// the attention kernel and K / V into the row's tree slot (committed length + local row)
// of its sequence's paged cache.  K pages are [16 tokens][hd]; V pages are stored
// transposed, [hd][16 tokens], which is the operand order of the P.V product.
// A workgroup takes one row and 256 / (hd/8) heads; a thread owns the rotation pairs
// (j .. j+3, j+hd/2 .. j+hd/2+3) of one head: 16-byte loads of every partial, all in flight at once.
// Needs hd % 8 == 0.
// ---------------------------------------------------------------------------------
__device__ __forceinline__ void st_q4(float* p, const float4& v) { *reinterpret_cast<float4*>(p) = v; }
__device__ __forceinline__ void st_q4(bf16_t* p, const float4& v) {
  *reinterpret_cast<uint2*>(p) = make_uint2((uint32_t)f32_to_f16_bits(v.x) | ((uint32_t)f32_to_f16_bits(v.y) << 16),
                                            (uint32_t)f32_to_f16_bits(v.z) | ((uint32_t)f32_to_f16_bits(v.w) << 16));
}
__device__ __forceinline__ void st_kv4(float* p, const float4& v) { *reinterpret_cast<float4*>(p) = v; }
__device__ __forceinline__ void st_kv4(bf16_t* p, const float4& v) {
  *reinterpret_cast<uint2*>(p) = make_uint2((uint32_t)f32_to_bf16(v.x) | ((uint32_t)f32_to_bf16(v.y) << 16),
                                            (uint32_t)f32_to_bf16(v.z) | ((uint32_t)f32_to_bf16(v.w) << 16));
}

template <typename T>
__global__ __launch_bounds__(256) void k_rope_kv(const float* __restrict__ part, int n_parts, size_t part_stride,
                                                 const float2* __restrict__ cs, const RowDst* __restrict__ dst,
                                                 T* __restrict__ Qb, int layer, int Hq, int Hkv, int hd) {
  const int r = blockIdx.x;
  const int half = hd / 2, tph = half / 4;          // threads per head
  const int head = blockIdx.y * (256 / tph) + threadIdx.x / tph;      // heads: Hq query, then Hkv key, then Hkv value
  if (head >= Hq + 2 * Hkv) return;
  const int j = (threadIdx.x % tph) * 4;
  const int q_dim = Hq * hd, N = q_dim + 2 * Hkv * hd;
  const int c1 = head * hd + j, c2 = c1 + half;
  const RowDst rd = dst[r];
  const float4 w01 = *reinterpret_cast<const float4*>(cs + (size_t)r * half + j);        // (cos, sin) of j, j+1
  const float4 w23 = *reinterpret_cast<const float4*>(cs + (size_t)r * half + j + 2);
  const float* p0 = part + (size_t)r * N;
  float4 x1 = make_float4(0.f, 0.f, 0.f, 0.f), x2 = x1;
  for (int s0 = 0; s0 < n_parts; s0 += 8) {
    float4 a[8], b[8];
#pragma unroll
    for (int u = 0; u < 8; ++u) {
      const int su = min(s0 + u, n_parts - 1);
      a[u] = *reinterpret_cast<const float4*>(p0 + (size_t)su * part_stride + c1);
      b[u] = *reinterpret_cast<const float4*>(p0 + (size_t)su * part_stride + c2);
    }
#pragma unroll
    for (int u = 0; u < 8; ++u)
      if (s0 + u < n_parts) {
        x1.x += a[u].x; x1.y += a[u].y; x1.z += a[u].z; x1.w += a[u].w;
        x2.x += b[u].x; x2.y += b[u].y; x2.z += b[u].z; x2.w += b[u].w;
      }
  }
  if (head >= Hq + Hkv) {                             // V: transposed in-page, [dim][16 tokens]
    const int g = head - Hq - Hkv;
    T* vcol = (T*)rd.v + (size_t)layer * rd.layer_stride + (size_t)g * hd * 16;
    st_from_f32(vcol + (size_t)(j + 0) * 16, x1.x); st_from_f32(vcol + (size_t)(j + 1) * 16, x1.y);
    st_from_f32(vcol + (size_t)(j + 2) * 16, x1.z); st_from_f32(vcol + (size_t)(j + 3) * 16, x1.w);
    st_from_f32(vcol + (size_t)(j + half + 0) * 16, x2.x); st_from_f32(vcol + (size_t)(j + half + 1) * 16, x2.y);
    st_from_f32(vcol + (size_t)(j + half + 2) * 16, x2.z); st_from_f32(vcol + (size_t)(j + half + 3) * 16, x2.w);
    return;
  }
  const float4 lo = make_float4(x1.x * w01.x - x2.x * w01.y, x1.y * w01.z - x2.y * w01.w,
                                x1.z * w23.x - x2.z * w23.y, x1.w * w23.z - x2.w * w23.w);
  const float4 hi = make_float4(x2.x * w01.x + x1.x * w01.y, x2.y * w01.z + x1.y * w01.w,
                                x2.z * w23.x + x1.z * w23.y, x2.w * w23.z + x1.w * w23.w);
  if (head < Hq) {
    st_q4(Qb + (size_t)r * q_dim + c1, lo);
    st_q4(Qb + (size_t)r * q_dim + c2, hi);
  } else {
    T* krow = (T*)rd.k + (size_t)layer * rd.layer_stride + (size_t)(head - Hq) * 16 * hd;
    st_kv4(krow + j, lo);
    st_kv4(krow + j + half, hi);
  }
}

void launch_rope_kv(ts_model* m, const RowMeta&, int R, int layer, int n_parts, size_t part_stride) {
  ProfScope ps(m, "rope_kv_write");
  const ts_model_config& c = m->cfg;
  const int heads_per_wg = 256 / (c.head_dim / 8);
  const dim3 grid(R, (c.n_q_heads + 2 * c.n_kv_heads + heads_per_wg - 1) / heads_per_wg);
  if (c.dtype == TS_DTYPE_BF16)
    hipLaunchKernelGGL(k_rope_kv<bf16_t>, grid, dim3(256), 0, m->stream, m->part, n_parts, part_stride, m->rope_cs, m->row_dst,
                       (bf16_t*)m->Qb, layer, c.n_q_heads, c.n_kv_heads, c.head_dim);
  else
    hipLaunchKernelGGL(k_rope_kv<float>, grid, dim3(256), 0, m->stream, m->part, n_parts, part_stride, m->rope_cs, m->row_dst,
                       (float*)m->Qb, layer, c.n_q_heads, c.n_kv_heads, c.head_dim);
}

// ---------------------------------------------------------------------------------
// SwiGLU: Fb[r][f] = T( silu(gate) * up ), gate / up = sums of split-K partials of the
// fused projection whose 16-column tiles alternate gate, up, gate, up, ...
// ---------------------------------------------------------------------------------
template <typename T>
__global__ void k_swiglu(const float* __restrict__ part, int n_parts, size_t part_stride, T* __restrict__ Fb,
                         size_t f_plane, int R, int F, unsigned long long* __restrict__ sat) {
  const size_t total = (size_t)R * F;
  for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < total; i += (size_t)gridDim.x * blockDim.x) {
    const int r = (int)(i / F), f = (int)(i % F);
    const int cg = (f >> 4) * 32 + (f & 15);
    const float* p = part + (size_t)r * (2 * F) + cg;
    float g = 0.f, u = 0.f;
    for (int s = 0; s < n_parts; ++s) {
      g += p[(size_t)s * part_stride];
      u += p[(size_t)s * part_stride + 16];
    }
    st_act(Fb + i, f_plane, g / (1.0f + expf(-g)) * u, sat);
  }
}

void launch_swiglu(ts_model* m, int R, int n_parts, size_t part_stride) {
  ProfScope ps(m, "swiglu");
  const int F = m->cfg.d_ffn;
  size_t total = (size_t)R * F;
  int blocks = (int)((total + 255) / 256);
  if (blocks > 4096) blocks = 4096;
  if (m->cfg.dtype == TS_DTYPE_BF16)
    hipLaunchKernelGGL(k_swiglu<f16_t>, dim3(blocks), dim3(256), 0, m->stream, m->part, n_parts, part_stride, (f16_t*)m->Fb, (size_t)(m->ws_rows + TS_MROWS_PER_BLOCK) * F, R, F, m->sat_count);
  else
    hipLaunchKernelGGL(k_swiglu<float>, dim3(blocks), dim3(256), 0, m->stream, m->part, n_parts, part_stride, (float*)m->Fb, (size_t)0, R, F, (unsigned long long*)nullptr);
}

// ---------------------------------------------------------------------------------
// arg-max over a row of materialised logits (fp32 path): one block per row, one partial.
// Lowest index wins among equal values.
// ---------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void k_argmax_rows(const float* __restrict__ logits, int V, float* __restrict__ aval,
                                                     int32_t* __restrict__ aidx, int parts) {
  __shared__ float sv[4];
  __shared__ int si[4];
  const int r = blockIdx.x;
  const float* p = logits + (size_t)r * V;
  float bv = -INFINITY;
  int bi = 0x7fffffff;
  for (int i = threadIdx.x; i < V; i += 256) amax_take(bv, bi, p[i], i);
  wave_amax(bv, bi);
  if ((threadIdx.x & 63) == 0) { sv[threadIdx.x >> 6] = bv; si[threadIdx.x >> 6] = bi; }
  __syncthreads();
  if (threadIdx.x == 0) {
    for (int w = 1; w < 4; ++w) amax_take(bv, bi, sv[w], si[w]);
    aval[(size_t)r * parts] = bv;
    aidx[(size_t)r * parts] = bi;
  }
}

void launch_argmax_rows(ts_model* m, int R) {
  ProfScope ps(m, "argmax_rows");
  hipLaunchKernelGGL(k_argmax_rows, dim3(R), dim3(256), 0, m->stream, m->logits, m->cfg.vocab, m->amax_val, m->amax_idx, m->amax_parts);
}

// ---------------------------------------------------------------------------------
// greedy acceptance, two small kernels.
//  k_argmax_combine  one block per row: g[row] = arg-max token, combined from the `parts`
//                    (value, index) partials of the lm_head epilogue (lowest index on ties)
//  k_walk            one block per sequence:
//   valid[r] = valid[parent(r)] && tok[r] == g[parent(r)],  valid[root] = true
//   best     = deepest valid row, lowest row index among equals
// result: [0] accept_len, [1] bonus token g[best], [2] best row, [4+i] row of depth i+1,
//         [4+64+i] token of depth i+1.
// ---------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void k_argmax_combine(const float* __restrict__ aval, const int32_t* __restrict__ aidx,
                                                        int parts, int used_parts, int32_t* __restrict__ g) {
  __shared__ float sv[4];
  __shared__ int si[4];
  const size_t base = (size_t)blockIdx.x * parts;
  float bv = -INFINITY;
  int bi = 0x7fffffff;
  for (int p0 = 0; p0 < used_parts; p0 += 256 * 4) {   // 4 independent loads per thread in flight
    float v4[4];
    int i4[4];
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const int p = p0 + j * 256 + threadIdx.x;
      const bool ok = p < used_parts;
      v4[j] = ok ? aval[base + p] : -INFINITY;
      i4[j] = ok ? aidx[base + p] : 0x7fffffff;
    }
#pragma unroll
    for (int j = 0; j < 4; ++j) amax_take(bv, bi, v4[j], i4[j]);
  }
  wave_amax(bv, bi);
  if ((threadIdx.x & 63) == 0) { sv[threadIdx.x >> 6] = bv; si[threadIdx.x >> 6] = bi; }
  __syncthreads();
  if (threadIdx.x == 0) {
    for (int w = 1; w < 4; ++w) amax_take(bv, bi, sv[w], si[w]);
    g[blockIdx.x] = bi;
  }
}

__global__ __launch_bounds__(128) void k_walk(const int32_t* __restrict__ g_row, const int32_t* __restrict__ tok,
                                              const int32_t* __restrict__ par, const int32_t* __restrict__ depth,
                                              const SeqDesc* __restrict__ seqs) {
  __shared__ int g[TS_MAX_NODES + 1];
  __shared__ int s_tok[TS_MAX_NODES + 1], s_par[TS_MAX_NODES + 1], s_dep[TS_MAX_NODES + 1];
  __shared__ unsigned char valid[TS_MAX_NODES + 1];
  const SeqDesc sd = seqs[blockIdx.x];
  if (threadIdx.x < sd.M) {                           // the serial walk below reads the tree from LDS
    g[threadIdx.x] = g_row[sd.row0 + threadIdx.x];
    s_tok[threadIdx.x] = tok[sd.row0 + threadIdx.x];
    s_par[threadIdx.x] = par[sd.row0 + threadIdx.x];
    s_dep[threadIdx.x] = depth[sd.row0 + threadIdx.x];
  }
  __syncthreads();
  if (threadIdx.x == 0) {
    int best = 0;
    valid[0] = 1;
    for (int r = 1; r < sd.M; ++r) {
      const int p = s_par[r];
      const unsigned char v = valid[p] && (s_tok[r] == g[p]);
      valid[r] = v;
      if (v && s_dep[r] > s_dep[best]) best = r;
    }
    int32_t* res = sd.result;
    const int len = s_dep[best];
    res[0] = len;
    res[1] = g[best];
    res[2] = best;
    int r = best;
    for (int dd = len; dd >= 1; --dd) {
      res[4 + dd - 1] = r;
      res[4 + TS_MAX_NODES + dd - 1] = s_tok[r];
      r = s_par[r];
    }
  }
}

void launch_walk(ts_model* m, const RowMeta& rm, int R, int n_seqs) {
  ProfScope ps(m, "accept_walk");
  hipLaunchKernelGGL(k_argmax_combine, dim3(R), dim3(256), 0, m->stream, m->amax_val, m->amax_idx, m->amax_parts,
                     m->amax_used, m->samp_tok);
  hipLaunchKernelGGL(k_walk, dim3(n_seqs), dim3(128), 0, m->stream, m->samp_tok, rm.tok, rm.par, rm.depth, m->seq_dev);
}

// ---------------------------------------------------------------------------------
// Stochastic acceptance (speculative sampling with point-mass drafts; App. B.2 names the
// rule, Leviathan et al. 2023).  Two kernels over the materialised logits of one sequence:
//  k_sample_rows  per row: log-sum-exp of logits / T, and the residual sample the step would
//                 end with at this row: arg-max of logits / T + Gumbel noise over all tokens
//                 except those of the row's children (if the walk stops here, every child was
//                 rejected and its token removed from the distribution).
//  k_walk_sample  child c of row r is accepted with probability p_r(x_c) / (1 - mass of the
//                 siblings rejected before it), decided by the caller's uniform of that node.
// Noise: one splitmix64 output per (seed, row within the sequence, token); its top 23 bits
// (+ 0.5) / 2^23 are the uniform, exact in single precision.
// ---------------------------------------------------------------------------------
__device__ __forceinline__ float gumbel_noise(uint64_t seed, int lrow, int v) {
  uint64_t z = seed + (((uint64_t)(uint32_t)lrow << 32) | (uint32_t)v) + 0x9E3779B97F4A7C15ull;
  z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
  z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
  z = z ^ (z >> 31);
  const float u = ((float)(uint32_t)(z >> 41) + 0.5f) * (1.0f / 8388608.0f);
  return -logf(-logf(u));
}

__global__ __launch_bounds__(1024) void k_sample_rows(const float* __restrict__ logits, int V, float inv_t, uint64_t seed,
                                                      const int32_t* __restrict__ tok, const int32_t* __restrict__ par,
                                                      const int32_t* __restrict__ lrow, const int32_t* __restrict__ row_seq,
                                                      const SeqDesc* __restrict__ seqs, float* __restrict__ lse,
                                                      int32_t* __restrict__ samp_tok) {
  __shared__ int excl[TS_MAX_NODES + 1];
  __shared__ int n_excl;
  __shared__ float sm[16], ss[16], sv[16];
  __shared__ int si[16];
  const int row = blockIdx.x, tid = threadIdx.x;
  const SeqDesc sd = seqs[row_seq[row]];
  const int lr = lrow[row];
  if (tid == 0) n_excl = 0;
  __syncthreads();
  if (tid < sd.M && tid > 0 && par[sd.row0 + tid] == lr) excl[atomicAdd(&n_excl, 1)] = tok[sd.row0 + tid];
  __syncthreads();
  const int ne = n_excl;
  const float* p = logits + (size_t)row * V;
  float m = -INFINITY, s = 0.f, bv = -INFINITY;
  int bi = 0x7fffffff;
  for (int v = tid; v < V; v += 1024) {
    const float z = p[v] * inv_t;
    if (z > m) { s = s * expf(m - z) + 1.0f; m = z; } else { s += expf(z - m); }
    bool ex = false;
    for (int e = 0; e < ne; ++e) ex |= (excl[e] == v);
    if (!ex) amax_take(bv, bi, z + gumbel_noise(seed, lr, v), v);
  }
  // combine (max, sum of exponentials) and the best perturbed score over the wave, then over the block
  for (int o = 32; o > 0; o >>= 1) {
    const float om = __shfl_xor(m, o, 64), os = __shfl_xor(s, o, 64);
    const float mm = fmaxf(m, om);
    s = (m == -INFINITY ? 0.f : s * expf(m - mm)) + (om == -INFINITY ? 0.f : os * expf(om - mm));
    m = mm;
  }
  wave_amax(bv, bi);
  if ((tid & 63) == 0) { sm[tid >> 6] = m; ss[tid >> 6] = s; sv[tid >> 6] = bv; si[tid >> 6] = bi; }
  __syncthreads();
  if (tid == 0) {
    for (int w = 1; w < 16; ++w) {
      const float mm = fmaxf(m, sm[w]);
      s = (m == -INFINITY ? 0.f : s * expf(m - mm)) + (sm[w] == -INFINITY ? 0.f : ss[w] * expf(sm[w] - mm));
      m = mm;
      amax_take(bv, bi, sv[w], si[w]);
    }
    lse[row] = m + logf(s);
    samp_tok[row] = bi;
  }
}

__global__ __launch_bounds__(128) void k_walk_sample(const float* __restrict__ logits, int V, float inv_t,
                                                     const float* __restrict__ lse, const int32_t* __restrict__ samp_tok,
                                                     const float* __restrict__ node_u, const int32_t* __restrict__ tok,
                                                     const int32_t* __restrict__ par, const SeqDesc* __restrict__ seqs) {
  __shared__ float prob[TS_MAX_NODES + 1], uu[TS_MAX_NODES + 1];
  __shared__ int s_tok[TS_MAX_NODES + 1], s_par[TS_MAX_NODES + 1];
  const SeqDesc sd = seqs[blockIdx.x];
  const int t = threadIdx.x;
  if (t < sd.M) {
    s_tok[t] = tok[sd.row0 + t];
    s_par[t] = par[sd.row0 + t];
    if (t > 0) {                       // probability of this node's token under its parent's distribution
      const int pr = sd.row0 + s_par[t];
      prob[t] = expf(logits[(size_t)pr * V + s_tok[t]] * inv_t - lse[pr]);
      uu[t] = node_u[sd.row0 + t];
    }
  }
  __syncthreads();
  if (t != 0) return;
  int32_t* res = sd.result;
  int r = 0, len = 0;
  for (;;) {
    float rem = 1.0f;
    int rejected[TS_MAX_NODES];
    int n_rej = 0, nxt = -1;
    for (int c = 1; c < sd.M && nxt < 0; ++c) {
      if (s_par[c] != r) continue;
      bool dup = false;
      for (int e = 0; e < n_rej; ++e) dup |= (rejected[e] == s_tok[c]);
      if (dup) continue;               // its token was already removed from the distribution
      if (uu[c] < prob[c] / rem) {
        nxt = c;
      } else {
        rejected[n_rej++] = s_tok[c];
        rem -= prob[c];
      }
    }
    if (nxt < 0) break;
    res[4 + len] = nxt;
    res[4 + TS_MAX_NODES + len] = s_tok[nxt];
    ++len;
    r = nxt;
  }
  res[0] = len;
  res[1] = samp_tok[sd.row0 + r];
  res[2] = r;
}

void launch_sample(ts_model* m, const RowMeta& rm, int R, int n_seqs, float temperature, uint64_t seed) {
  ProfScope ps(m, "sample_accept");
  const float inv_t = 1.0f / temperature;
  hipLaunchKernelGGL(k_sample_rows, dim3(R), dim3(1024), 0, m->stream, m->logits, m->cfg.vocab, inv_t, seed, rm.tok, rm.par,
                     rm.lrow, rm.seq, m->seq_dev, m->samp_lse, m->samp_tok);
  hipLaunchKernelGGL(k_walk_sample, dim3(n_seqs), dim3(128), 0, m->stream, m->logits, m->cfg.vocab, inv_t, m->samp_lse,
                     m->samp_tok, rm.u, rm.tok, rm.par, m->seq_dev);
}

// ---------------------------------------------------------------------------------
// commit: move the K/V of the accepted row of depth d from tree slot P + row_d to slot
// P + d, for d = 1..l.  A thread owns one element column (one head-dim index of one KV
// head of one layer) across all depths and walks d upwards; since row_d >= d and rows
// increase with depth, a slot is always read before the step that overwrites it, and no
// two threads touch the same element, so the in-place move is race-free.
// ---------------------------------------------------------------------------------
template <typename T>
__global__ void k_commit(T* __restrict__ k_pool, T* __restrict__ v_pool, const int32_t* __restrict__ page_table,
                         const int32_t* __restrict__ result, int n_pages, int Hkv, int hd, int P, int len) {
  const int layer = blockIdx.x / Hkv, g = blockIdx.x % Hkv;
  const int dd = threadIdx.x;
  if (dd >= hd) return;
  const size_t page_elems = (size_t)Hkv * 16 * hd;
  for (int dep = 1; dep <= len; ++dep) {
    const int src = P + result[4 + dep - 1], dst = P + dep;
    if (src == dst) continue;
    const size_t sp = ((size_t)layer * n_pages + page_table[src >> 4]) * page_elems;
    const size_t dp = ((size_t)layer * n_pages + page_table[dst >> 4]) * page_elems;
    const int st = src & 15, dt = dst & 15;
    k_pool[dp + ((size_t)g * 16 + dt) * hd + dd] = k_pool[sp + ((size_t)g * 16 + st) * hd + dd];
    v_pool[dp + ((size_t)g * hd + dd) * 16 + dt] = v_pool[sp + ((size_t)g * hd + dd) * 16 + st];
  }
}

void launch_commit(ts_kv* kv, int accept_len) {
  ts_model* m = kv->model;
  const ts_model_config& c = m->cfg;
  dim3 grid(c.n_layers * c.n_kv_heads), block(c.head_dim <= 64 ? 64 : 128);
  if (c.dtype == TS_DTYPE_BF16)
    hipLaunchKernelGGL(k_commit<bf16_t>, grid, block, 0, m->stream, (bf16_t*)kv->k_pool, (bf16_t*)kv->v_pool,
                       kv->page_table, kv->result, kv->pool_pages, c.n_kv_heads, c.head_dim, kv->P, accept_len);
  else
    hipLaunchKernelGGL(k_commit<float>, grid, block, 0, m->stream, (float*)kv->k_pool, (float*)kv->v_pool,
                       kv->page_table, kv->result, kv->pool_pages, c.n_kv_heads, c.head_dim, kv->P, accept_len);
}

// ---------------------------------------------------------------------------------
// import / export between the position-major exchange layout [pos][Hkv][hd] (one layer,
// staged on the device) and the paged pools.
// ---------------------------------------------------------------------------------
template <typename T, bool IMPORT>
__global__ void k_kv_xfer(T* __restrict__ k_pool, T* __restrict__ v_pool, const int32_t* __restrict__ page_table,
                          T* __restrict__ sk, T* __restrict__ sv, int layer, int n_pages, int Hkv, int hd, int pos0,
                          int n_pos) {
  const size_t page_elems = (size_t)Hkv * 16 * hd;
  const size_t total = (size_t)n_pos * Hkv * hd;
  for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < total; i += (size_t)gridDim.x * blockDim.x) {
    const int dd = (int)(i % hd);
    const int g = (int)((i / hd) % Hkv);
    const int pos = pos0 + (int)(i / ((size_t)hd * Hkv));
    const size_t pg = ((size_t)layer * n_pages + page_table[pos >> 4]) * page_elems;
    const int t = pos & 15;
    const size_t ki = pg + ((size_t)g * 16 + t) * hd + dd;
    const size_t vi = pg + ((size_t)g * hd + dd) * 16 + t;
    if (IMPORT) { k_pool[ki] = sk[i]; v_pool[vi] = sv[i]; }
    else        { sk[i] = k_pool[ki]; sv[i] = v_pool[vi]; }
  }
}

template <bool IMPORT>
static void kv_xfer(ts_kv* kv, int pos0, int n_pos, void* sk, void* sv, int layer) {
  ts_model* m = kv->model;
  const ts_model_config& c = m->cfg;
  size_t total = (size_t)n_pos * c.n_kv_heads * c.head_dim;
  int blocks = (int)((total + 255) / 256);
  if (blocks > 8192) blocks = 8192;
  if (blocks < 1) blocks = 1;
  if (c.dtype == TS_DTYPE_BF16)
    hipLaunchKernelGGL((k_kv_xfer<bf16_t, IMPORT>), dim3(blocks), dim3(256), 0, m->stream, (bf16_t*)kv->k_pool,
                       (bf16_t*)kv->v_pool, kv->page_table, (bf16_t*)sk, (bf16_t*)sv, layer, kv->pool_pages,
                       c.n_kv_heads, c.head_dim, pos0, n_pos);
  else
    hipLaunchKernelGGL((k_kv_xfer<float, IMPORT>), dim3(blocks), dim3(256), 0, m->stream, (float*)kv->k_pool,
                       (float*)kv->v_pool, kv->page_table, (float*)sk, (float*)sv, layer, kv->pool_pages, c.n_kv_heads,
                       c.head_dim, pos0, n_pos);
}

void launch_kv_import(ts_kv* kv, int pos0, int n_pos, const void* sk, const void* sv, int layer) {
  kv_xfer<true>(kv, pos0, n_pos, const_cast<void*>(sk), const_cast<void*>(sv), layer);
}
void launch_kv_export(ts_kv* kv, int pos0, int n_pos, void* sk, void* sv, int layer) {
  kv_xfer<false>(kv, pos0, n_pos, sk, sv, layer);
}

// =================================================================================
// fp32 compute path (small models; launch-latency bound, written for exactness)
// =================================================================================

// out[M][N] = X[M][K] . W[N][K]^T, fp32 FMA in ascending k.  Block = 16 rows x 64 columns.
__global__ __launch_bounds__(256) void k_gemm_f32(const float* __restrict__ X, const float* __restrict__ W,
                                                  float* __restrict__ out, int M, int N, int K) {
  __shared__ float xs[16][33];
  __shared__ float ws[64][33];
  const int tx = threadIdx.x & 63, ty = threadIdx.x >> 6;
  const int n0 = blockIdx.x * 64, m0 = blockIdx.y * 16;
  float acc[4] = {0.f, 0.f, 0.f, 0.f};
  for (int k0 = 0; k0 < K; k0 += 32) {
    for (int i = threadIdx.x; i < 16 * 32; i += 256) {
      const int r = i >> 5, c = i & 31;
      xs[r][c] = (m0 + r < M && k0 + c < K) ? X[(size_t)(m0 + r) * K + k0 + c] : 0.f;
    }
    for (int i = threadIdx.x; i < 64 * 32; i += 256) {
      const int r = i >> 5, c = i & 31;
      ws[r][c] = (n0 + r < N && k0 + c < K) ? W[(size_t)(n0 + r) * K + k0 + c] : 0.f;
    }
    __syncthreads();
#pragma unroll
    for (int c = 0; c < 32; ++c) {
      const float w = ws[tx][c];
#pragma unroll
      for (int i = 0; i < 4; ++i) acc[i] = fmaf(xs[ty * 4 + i][c], w, acc[i]);
    }
    __syncthreads();
  }
  for (int i = 0; i < 4; ++i) {
    const int r = m0 + ty * 4 + i, n = n0 + tx;
    if (r < M && n < N) out[(size_t)r * N + n] = acc[i];
  }
}

void launch_gemm_f32(ts_model* m, const float* X, const float* W, float* out, int M, int N, int K) {
  ProfScope ps(m, "gemm_f32");
  hipLaunchKernelGGL(k_gemm_f32, dim3((N + 63) / 64, (M + 15) / 16), dim3(256), 0, m->stream, X, W, out, M, N, K);
}

// Tree-masked attention, fp32: one block per (row, query head).  Scores for all keys of
// the row's sequence live in LDS.  Key j < P is context (visible); key P + s is tree row s,
// visible iff s = 0 (root) or bit s-1 of the row's ancestor mask is set.
size_t attn_f32_max_keys() { return 15000; }

__global__ __launch_bounds__(256) void k_attn_f32(const float* __restrict__ Qb, float* __restrict__ Ab,
                                                  const int32_t* __restrict__ row_seq,
                                                  const int32_t* __restrict__ row_lrow,
                                                  const uint64_t* __restrict__ row_anc,
                                                  const SeqDesc* __restrict__ seqs, int layer, int Hq, int Hkv, int hd,
                                                  float scale) {
  extern __shared__ float smem[];
  __shared__ float red[4];
  const int r = blockIdx.x, h = blockIdx.y, g = h / (Hq / Hkv);
  const SeqDesc sd = seqs[row_seq[r]];
  const uint64_t anc = row_anc[r];
  const int T = sd.P + sd.M;
  float* q = smem;          // [hd]
  float* sc = smem + hd;    // [T]
  float* acc = sc + T;      // [256]
  const size_t page_elems = (size_t)Hkv * 16 * hd;
  const float* kl = (const float*)sd.k_pool + (size_t)layer * sd.n_pages * page_elems;
  const float* vl = (const float*)sd.v_pool + (size_t)layer * sd.n_pages * page_elems;
  for (int i = threadIdx.x; i < hd; i += 256) q[i] = Qb[(size_t)r * Hq * hd + h * hd + i];
  __syncthreads();
  float mx = -INFINITY;
  for (int j = threadIdx.x; j < T; j += 256) {
    bool vis = true;
    if (j >= sd.P) {
      const int s = j - sd.P;
      vis = (s == 0) || ((anc >> (s - 1)) & 1ull);
    }
    float v = -INFINITY;
    if (vis) {
      const float* kr = kl + (size_t)sd.page_table[j >> 4] * page_elems + ((size_t)g * 16 + (j & 15)) * hd;
      float a = 0.f;
      for (int i = 0; i < hd; ++i) a = fmaf(q[i], kr[i], a);
      v = a * scale;
    }
    sc[j] = v;
    mx = fmaxf(mx, v);
  }
  mx = wave_max(mx);
  if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = mx;
  __syncthreads();
  mx = fmaxf(fmaxf(red[0], red[1]), fmaxf(red[2], red[3]));
  __syncthreads();
  float sum = 0.f;
  for (int j = threadIdx.x; j < T; j += 256) {
    const float p = expf(sc[j] - mx);
    sc[j] = p;
    sum += p;
  }
  sum = wave_sum(sum);
  if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = sum;
  __syncthreads();
  sum = red[0] + red[1] + red[2] + red[3];
  // P.V: thread (dd, part) accumulates keys part, part + n_parts, ... for head-dim index dd
  const int n_parts = 256 / hd;
  const int dd = threadIdx.x % hd, part = threadIdx.x / hd;
  float a = 0.f;
  if (part < n_parts) {
    for (int j = part; j < T; j += n_parts) {
      const float p = sc[j];
      if (p != 0.f) {
        const float* vp = vl + (size_t)sd.page_table[j >> 4] * page_elems + ((size_t)g * hd + dd) * 16 + (j & 15);
        a = fmaf(p, *vp, a);
      }
    }
  }
  acc[threadIdx.x] = a;
  __syncthreads();
  if (threadIdx.x < hd) {
    float o = 0.f;
    for (int p = 0; p < n_parts; ++p) o += acc[p * hd + threadIdx.x];
    Ab[(size_t)r * Hq * hd + h * hd + threadIdx.x] = o / sum;
  }
}

void launch_attn_f32(ts_model* m, const RowMeta& rm, int R, int, int layer, int max_keys) {
  ProfScope ps(m, "attn_f32");
  const ts_model_config& c = m->cfg;
  size_t shmem = (size_t)(c.head_dim + max_keys + 256) * sizeof(float);
  hipLaunchKernelGGL(k_attn_f32, dim3(R, c.n_q_heads), dim3(256), shmem, m->stream, (const float*)m->Qb, (float*)m->Ab,
                     rm.seq, rm.lrow, rm.anc, m->seq_dev, layer, c.n_q_heads, c.n_kv_heads, c.head_dim,
                     1.0f / sqrtf((float)c.head_dim));
}

// ---------------------------------------------------------------------------------
// Plain streaming read of a weight tensor: what the memory system gives a kernel that does
// nothing but read, on the same bytes the fused gate/up projection streams.  One workgroup per
// CU, eight 16-byte loads in flight per thread, grid-strided (the fastest of the grids and
// patterns tried).  The xor of the words keeps the loads alive; nothing is written unless the
// xor hits one value in 2^32.
// ---------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void k_plain_read(const uint4* __restrict__ p, size_t n_vec, uint32_t* __restrict__ sink) {
  uint32_t acc = 0;
  const size_t stride = (size_t)gridDim.x * 256;
  size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
  for (; i + 7 * stride < n_vec; i += 8 * stride) {
    uint4 v[8];
#pragma unroll
    for (int u = 0; u < 8; ++u) v[u] = p[i + u * stride];
#pragma unroll
    for (int u = 0; u < 8; ++u) acc ^= v[u].x ^ v[u].w;
  }
  for (; i < n_vec; i += stride) acc ^= p[i].x;
  if (acc == 0x9e3779b9u) sink[0] = acc;
}

void launch_plain_read(ts_model* m, const void* src, size_t bytes, uint32_t* sink) {
  ProfScope ps(m, "plain_read");
  hipLaunchKernelGGL(k_plain_read, dim3(m->n_cu), dim3(256), 0, m->stream, (const uint4*)src, bytes / 16, sink);
}
