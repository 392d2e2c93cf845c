// Fast path for passes of at most 32 rows (tree verification at batch 1, the head's tree levels, vanilla
// decoding): weight-streaming GEMM with the reduction and the layer's element-wise work fused into it.
//
//   * A work-group owns (a group of 32-row weight blocks) x (one K slice).  Its K slice of the activations sits
//     in LDS in MFMA B-operand order; every wave streams its own weight tiles straight from HBM into the MFMA
//     A operand (one coalesced 1 KiB load per tile, many tiles in flight).
//   * Waves that share a weight block but split K are summed through LDS in a fixed order; work-groups that
//     split K write partials and the LAST one to arrive (an atomic counter, no waiting) sums them in split
//     order and runs the epilogue -- so results do not depend on timing.
//   * RMSNorm is folded around the GEMM: the producer writes h*gain (not normalised) plus per-row partial sums
//     of squares; the consumer multiplies its outputs by 1/rms, which commutes with the matrix product.
#pragma once
#include "kernels.h"

#define V2_THREADS 512

// Data that one work-group writes and another reads INSIDE one kernel (split-K partials, attention partials) goes
// through agent-scope relaxed atomics: such stores are written through to the device-coherent level and such
// loads never hit a stale line of another XCD's L2, so no cache write-back / invalidate is needed around the
// arrival counter -- a work-group-scope fence (a wait for the stores to be acknowledged) is enough.
__device__ inline void coh_store(float* p, float v) { __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT); }
__device__ inline float coh_load(const float* p) { return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT); }

// 16-byte agent-scope accesses: buffer instructions carry the scope bit (aux 16 = sc1); byte offsets below 2 GiB.
__device__ inline __amdgpu_buffer_rsrc_t coh_rsrc(const void* p) {
  return __builtin_amdgcn_make_buffer_rsrc((void*)p, 0, 0x7FFFFFFF, 0x00020000);
}
__device__ inline f32x4 coh_load16(const void* base, uint32_t byte_off) {
  return __builtin_bit_cast(f32x4, __builtin_amdgcn_raw_buffer_load_b128(coh_rsrc(base), byte_off, 0, 16));
}
__device__ inline void coh_store16(void* base, uint32_t byte_off, f32x4 v) {
  __builtin_amdgcn_raw_buffer_store_b128(__builtin_bit_cast(u32x4, v), coh_rsrc(base), byte_off, 0, 16);
}
// Split-K partials PT[s][n][m]: four consecutive weight rows n of one token m are adjacent (16 bytes), which is what
// one lane of the MFMA accumulator holds (registers 4i..4i+3) and what an epilogue thread consumes.
__device__ inline uint32_t pt_quad_bytes(int s, int Npad, int n4 /*multiple of 4*/, int m) {
  return (uint32_t)((((size_t)s * Npad + n4) * 32 + (size_t)m * 4) * 4);
}

struct RowScale {            // 1/rms of the rows that produced the GEMM input; ssq == nullptr -> 1
  const float* ssq;          // [groups][32] partial sums of squares
  int groups;
  float inv_d, eps;
};
// 1/rms of row m from the per-group partial sums of squares: 16 strided classes of groups, classes added in order
// (one fixed order for every caller).  The block shares the loads: threads 0..15 each own a class (at most 16 groups,
// all loads in flight), thread 0 adds the classes.  tmp: 17 floats of LDS.  Every thread of the block must call it.
__device__ inline float block_row_rstd(const float* ssq, int groups, float inv_d, float eps, int m, float* tmp) {
  if (!ssq) return 1.0f;
  if (threadIdx.x < 16) {
    float v[16];
#pragma unroll
    for (int i = 0; i < 16; ++i) {
      const int g = (int)threadIdx.x + 16 * i;
      v[i] = g < groups ? ssq[g * 32 + m] : 0.f;
    }
    float a = 0.f;
#pragma unroll
    for (int i = 0; i < 16; ++i) a += v[i];
    tmp[threadIdx.x] = a;
  }
  __syncthreads();
  if (threadIdx.x == 0) {
    float tot = 0.f;
    for (int c = 0; c < 16; ++c) tot += tmp[c];
    tmp[16] = 1.0f / sqrtf(tot * inv_d + eps);
  }
  __syncthreads();
  return tmp[16];
}
// The same value for all 32 rows at once, computed by a 512-thread block: thread (m, class c) loads its class's groups
// (at most 16, all in flight) early in the kernel (rstd_class_partial); the classes are combined through LDS when the
// epilogue needs the result (block_rstd_finish).
__device__ inline float rstd_class_partial(const RowScale& rs) {
  if (!rs.ssq) return 0.f;
  const int m = threadIdx.x & 31, c = threadIdx.x >> 5;
  float v[16];
#pragma unroll
  for (int i = 0; i < 16; ++i) {
    const int g = c + 16 * i;
    v[i] = g < rs.groups ? rs.ssq[g * 32 + m] : 0.f;
  }
  float a = 0.f;
#pragma unroll
  for (int i = 0; i < 16; ++i) a += v[i];
  return a;
}
__device__ inline void block_rstd_finish(const RowScale& rs, float part, float* out, float* tmp) {
  if (!rs.ssq) {
    if (threadIdx.x < 32) out[threadIdx.x] = 1.0f;
    __syncthreads();
    return;
  }
  tmp[(threadIdx.x >> 5) * 32 + (threadIdx.x & 31)] = part;
  __syncthreads();
  if (threadIdx.x < 32) {
    float tot = 0.f;
    for (int cc = 0; cc < 16; ++cc) tot += tmp[cc * 32 + threadIdx.x];
    out[threadIdx.x] = 1.0f / sqrtf(tot * rs.inv_d + rs.eps);
  }
  __syncthreads();
}

enum { EPI_QKV = 0, EPI_RESID = 1, EPI_SWIGLU = 2, EPI_LOGITS = 3 };

// Before a work-group announces its coherent stores through an arrival counter, every wave waits until its own
// vector-memory stores have been acknowledged.  A work-group-scope release fence alone does not do that on this
// target (waves of one work-group share a CU, so the compiler emits no vector-memory wait for it), and the stores
// go to other L2 channels than the counter: without the wait the counter can be seen before the data.
// s_waitcnt 0x0F70 = vmcnt(0), expcnt and lgkmcnt left alone.
__device__ __forceinline__ void publish_wait() {
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
  __builtin_amdgcn_s_waitcnt(0x0F70);
}

struct Gemm2 {
  const bf16_t* W; size_t wps; int NRB, KS, Npad, N;
  const bf16_t* XF;                       // NXP planes of KS tiles (one 32-row tile per k-step)
  int S, groups, lanes, kparts;
  float* PT; int* counters;
  int M, epi;
  RowScale in_scale;
  // EPI_QKV
  Pass pass; const TreeDev* tree; SeqState st; KVCache kv; int kv_f32; float* Q; const float* rope_cos; const float* rope_sin; int H;
  // EPI_RESID / EPI_SWIGLU
  const float* h_in; float* h_out; const float* bias; const float* gain_next; bf16_t* xf_out; int xf_KS; float* ssq_out; int d;
  // EPI_LOGITS
  float* logits; int out_kind, V, only_last_row;
  const bf16_t* SC; int NG;               // 4-bit weights: scales [NRB][NG][2][16] and groups along K (W then holds codes)
  const float* row_w;                     // MoE: per-row routing weight applied to this GEMM's result (nullptr = 1)
  const int* skip_flag;                   // MoE: the whole launch is a no-op when *skip_flag == 0 (no row uses the expert)
  unsigned long long* trace;              // profiling builds (-DEAGLE_TRACE) only: [work-group][8] time stamps of this launch
};

// out[0..3] = sum over the K splits of rows nA..nA+3, out[4..7] the same for rows nB..nB+3 (nA, nB multiples of 4,
// below Npad), token m.  All loads of a batch of splits are in flight together; splits are added in order.
template <int B>
__device__ inline void pt_sum8_b(const float* __restrict__ PT, int S, int Npad, int nA, int nB, int m, float* out) {
  for (int s0 = 0; s0 < S; s0 += B) {
    f32x4 va[B], vb[B];
#pragma unroll
    for (int u = 0; u < B; ++u) {
      const int s = min(s0 + u, S - 1);
      va[u] = coh_load16(PT, pt_quad_bytes(s, Npad, nA, m));
      vb[u] = coh_load16(PT, pt_quad_bytes(s, Npad, nB, m));
    }
#pragma unroll
    for (int u = 0; u < B; ++u)
      if (s0 + u < S) {
        out[0] += va[u].x; out[1] += va[u].y; out[2] += va[u].z; out[3] += va[u].w;
        out[4] += vb[u].x; out[5] += vb[u].y; out[6] += vb[u].z; out[7] += vb[u].w;
      }
  }
}
__device__ inline void pt_sum8(const float* __restrict__ PT, int S, int Npad, int nA, int nB, int m, float* out) {
#pragma unroll
  for (int t = 0; t < 8; ++t) out[t] = 0.f;
  // the batch size closest above S: loads beyond S would be wasted traffic in an epilogue that one CU's bandwidth bounds
  if (S <= 4) pt_sum8_b<4>(PT, S, Npad, nA, nB, m, out);
  else if (S <= 8) pt_sum8_b<8>(PT, S, Npad, nA, nB, m, out);
  else if (S <= 12) pt_sum8_b<12>(PT, S, Npad, nA, nB, m, out);
  else pt_sum8_b<16>(PT, S, Npad, nA, nB, m, out);
}

// four quads at once, S <= 4: 16 loads in flight; issue and summation are separate so that a caller can put the
// loads of several items in flight before it consumes the first
struct PtQuads4 { f32x4 v[4][4]; };
__device__ inline void pt_issue16(PtQuads4& b, const float* __restrict__ PT, int S, int Npad, int nA, int nB, int nC, int nD, int m) {
#pragma unroll
  for (int u = 0; u < 4; ++u) {
    const int sp = min(u, S - 1);
    b.v[u][0] = coh_load16(PT, pt_quad_bytes(sp, Npad, nA, m));
    b.v[u][1] = coh_load16(PT, pt_quad_bytes(sp, Npad, nB, m));
    b.v[u][2] = coh_load16(PT, pt_quad_bytes(sp, Npad, nC, m));
    b.v[u][3] = coh_load16(PT, pt_quad_bytes(sp, Npad, nD, m));
  }
}
__device__ inline void pt_finish16(const PtQuads4& b, int S, float* outAB, float* outCD) {
#pragma unroll
  for (int t = 0; t < 8; ++t) { outAB[t] = 0.f; outCD[t] = 0.f; }
#pragma unroll
  for (int u = 0; u < 4; ++u)
    if (u < S) {
      outAB[0] += b.v[u][0].x; outAB[1] += b.v[u][0].y; outAB[2] += b.v[u][0].z; outAB[3] += b.v[u][0].w;
      outAB[4] += b.v[u][1].x; outAB[5] += b.v[u][1].y; outAB[6] += b.v[u][1].z; outAB[7] += b.v[u][1].w;
      outCD[0] += b.v[u][2].x; outCD[1] += b.v[u][2].y; outCD[2] += b.v[u][2].z; outCD[3] += b.v[u][2].w;
      outCD[4] += b.v[u][3].x; outCD[5] += b.v[u][3].y; outCD[6] += b.v[u][3].z; outCD[7] += b.v[u][3].w;
    }
}
// the same for any S (more than 4 splits: two rounds of two quads)
__device__ inline void pt_sum16(const float* __restrict__ PT, int S, int Npad, int nA, int nB, int nC, int nD, int m, float* outAB, float* outCD) {
  if (S > 4) { pt_sum8(PT, S, Npad, nA, nB, m, outAB); pt_sum8(PT, S, Npad, nC, nD, m, outCD); return; }
  PtQuads4 b;
  pt_issue16(b, PT, S, Npad, nA, nB, nC, nD, m);
  pt_finish16(b, S, outAB, outCD);
}

// what a thread needs about "its" row in the epilogue, fetched before the streaming loop so that the loads are
// long finished when the last work-group gets there
struct RowPre { int valid, seq, pos, slot; long dst; float ssq_part; };

template <int NXP>
__device__ inline void epilogue_qkv(const Gemm2& g, int n0, int n1, const float* rstd_s, const RowPre& rp) {
  const int m = threadIdx.x & 31, slot = threadIdx.x >> 5;
  const int dh = g.kv.head_dim, half = dh >> 1, KVH = g.kv.n_kv_heads, H = g.H;
  const bool live = m < g.M;
  const float rs = live ? rstd_s[m] : 0.f;
  const int nquads = (n1 - n0) >> 2;                          // n0, n1 are multiples of 32 here (whole heads)
  constexpr int SL = V2_THREADS / 32;
  for (int q0 = slot; q0 < nquads; q0 += 4 * SL) {           // four quads = eight rotate-half pairs per batch of loads
    int nq[4];
#pragma unroll
    for (int c = 0; c < 4; ++c) nq[c] = n0 + 4 * min(q0 + c * SL, nquads - 1);
    float cs[8], sn[8];
#pragma unroll
    for (int u = 0; u < 8; ++u) {
      const int n = nq[u >> 1] + 2 * (u & 1);
      const int i = (n % dh) >> 1;                            // rotation angle index (unused for v heads)
      cs[u] = g.rope_cos[(size_t)rp.pos * half + i];
      sn[u] = g.rope_sin[(size_t)rp.pos * half + i];
    }
    float val[16];
    pt_sum16(g.PT, g.S, g.Npad, nq[0], nq[1], nq[2], nq[3], m, val, val + 8);
#pragma unroll
    for (int u = 0; u < 8; ++u) {
      if (q0 + (u >> 1) * SL >= nquads || !live) continue;
      const int n = nq[u >> 1] + 2 * (u & 1), hd = n / dh, pr = n % dh;
      float a = val[2 * u] * rs, b = val[2 * u + 1] * rs;
      int d1, d2;
      if (hd < H + KVH) {        // q or k head: the two rows are a rotate-half pair
        const int i = pr >> 1;
        const float a2 = a * cs[u] - b * sn[u], b2 = b * cs[u] + a * sn[u];
        a = a2; b = b2; d1 = i; d2 = i + half;
      } else { d1 = pr; d2 = pr + 1; }
      if (hd < H) {
        float* q = g.Q + ((size_t)m * H + hd) * dh;
        q[d1] = a; q[d2] = b;
      } else if (rp.valid) {
        const int kvh = (hd - H) % KVH;
        const size_t off = kv_offset(g.kv, rp.seq, rp.slot, kvh);
        void* base = hd < H + KVH ? g.kv.k : g.kv.v;
        if (g.kv_f32) { ((float*)base)[off + d1] = a; ((float*)base)[off + d2] = b; }
        else { ((bf16_t*)base)[off + d1] = f32_to_bf16(a); ((bf16_t*)base)[off + d2] = f32_to_bf16(b); }
      }
    }
  }
}

template <int NXP>
__device__ inline void epilogue_resid(const Gemm2& g, int grp, int n0, int n1, float* sh /*>= 16*32 floats*/) {
  const int m = threadIdx.x & 31, slot = threadIdx.x >> 5;
  const bool live = m < g.M;
  const int nchunks = (n1 - n0 + 7) >> 3;
  float ss = 0.f;
  for (int c = slot; c < nchunks; c += V2_THREADS / 32) {
    const int n = n0 + 8 * c;
    float x[8], pv[8], hv[8], bv[8], gv[8];
    int rows[8];
    const float rw = g.row_w ? g.row_w[m] : 1.0f;
#pragma unroll
    for (int t = 0; t < 8; ++t) {                            // everything that does not depend on the partials first
      rows[t] = min(n + t, n1 - 1);
      hv[t] = (g.h_in && live) ? g.h_in[(size_t)m * g.d + rows[t]] : 0.f;
      bv[t] = g.bias ? g.bias[rows[t]] : 0.f;
      gv[t] = g.gain_next ? g.gain_next[rows[t]] : 1.0f;
    }
    pt_sum8(g.PT, g.S, g.Npad, n, n + 4, m, pv);            // rows up to the padded end of the block exist (zero weights)
#pragma unroll
    for (int t = 0; t < 8; ++t) {
      float v = 0.f;
      if (n + t < n1) {
        v = g.row_w ? rw * pv[t] : pv[t];
        if (g.bias) v += bv[t];
        if (g.h_in && live) v += hv[t];
        if (live) g.h_out[(size_t)m * g.d + n + t] = v;
        ss += v * v;
        x[t] = g.gain_next ? v * gv[t] : v;
      } else x[t] = 0.f;
    }
    if (live) xf_store8(g.xf_out, m, n, 1, g.xf_KS, NXP, x);
  }
  __syncthreads();
  sh[slot * 32 + m] = ss;
  __syncthreads();
  if (threadIdx.x < 32 && g.ssq_out) {
    float a = 0.f;
    for (int i = 0; i < V2_THREADS / 32; ++i) a += sh[i * 32 + threadIdx.x];
    g.ssq_out[grp * 32 + threadIdx.x] = a;
  }
}

__device__ inline void swiglu8(const float* gv, const float* uv, float rs, float* x) {
#pragma unroll
  for (int t = 0; t < 8; ++t) {
    const float gg = gv[t] * rs, uu = uv[t] * rs;
    x[t] = gg / (1.0f + __expf(-gg)) * uu;
  }
}
template <int NXP>
__device__ inline void epilogue_swiglu(const Gemm2& g, int n0, int n1, const float* rstd_s) {
  const int m = threadIdx.x & 31, slot = threadIdx.x >> 5;
  const bool live = m < g.M;
  const float rs = live ? rstd_s[m] : 0.f;
  const int items = ((n1 - n0) >> 5) * 2;                    // 8 outputs each: gate rows nb..nb+7, up rows 16 further
  constexpr int SL = V2_THREADS / 32;
  if (g.S <= 4) {
    for (int it = slot; it < items; it += 2 * SL) {          // two items = 32 loads in flight
      const int it2 = min(it + SL, items - 1);
      const int nbA = n0 + (it >> 1) * 32 + 8 * (it & 1), nbB = n0 + (it2 >> 1) * 32 + 8 * (it2 & 1);
      PtQuads4 qa, qb;
      pt_issue16(qa, g.PT, g.S, g.Npad, nbA, nbA + 4, nbA + 16, nbA + 20, m);
      pt_issue16(qb, g.PT, g.S, g.Npad, nbB, nbB + 4, nbB + 16, nbB + 20, m);
      float x[8], gv[8], uv[8];
      pt_finish16(qa, g.S, gv, uv);
      swiglu8(gv, uv, rs, x);
      if (live) xf_store8(g.xf_out, m, ((n0 >> 5) + (it >> 1)) * 16 + 8 * (it & 1), 1, g.xf_KS, NXP, x);
      pt_finish16(qb, g.S, gv, uv);
      swiglu8(gv, uv, rs, x);
      if (live && it + SL < items) xf_store8(g.xf_out, m, ((n0 >> 5) + (it2 >> 1)) * 16 + 8 * (it2 & 1), 1, g.xf_KS, NXP, x);
    }
    return;
  }
  for (int it = slot; it < items; it += SL) {
    const int rb = it >> 1, c2 = it & 1;
    const int nb = n0 + rb * 32 + 8 * c2;
    const int f = ((n0 >> 5) + rb) * 16 + 8 * c2;
    float x[8], gv[8], uv[8];
    pt_sum16(g.PT, g.S, g.Npad, nb, nb + 4, nb + 16, nb + 20, m, gv, uv);
    swiglu8(gv, uv, rs, x);
    if (live) xf_store8(g.xf_out, m, f, 1, g.xf_KS, NXP, x);
  }
}

__device__ inline void epilogue_logits(const Gemm2& g, int n0, int n1, const float* rstd_s, const RowPre& rp) {
  const int m = threadIdx.x & 31, b = threadIdx.x >> 5;        // token m, quad b (and b + 16) of each 128-row batch
  const float rs = m < g.M ? rstd_s[m] : 0.f;
  const long dst = rp.dst;                                     // where token m's logits row starts, or -1
  const int nend = min(n1, g.V);
  const bool vec = (g.V & 3) == 0;                             // rows of the output are 16-byte aligned
  for (int nb0 = n0; nb0 < n1; nb0 += 128) {
    const int nA = nb0 + 4 * b, nB = nb0 + 64 + 4 * b;
    float val[8];
    pt_sum8(g.PT, g.S, g.Npad, min(nA, g.Npad - 4), min(nB, g.Npad - 4), m, val);
    if (dst < 0) continue;
#pragma unroll
    for (int h = 0; h < 2; ++h) {
      const int n = h ? nB : nA;
      if (n >= nend) continue;
      if (vec && n + 4 <= nend) {
        f32x4 o; o.x = val[4 * h] * rs; o.y = val[4 * h + 1] * rs; o.z = val[4 * h + 2] * rs; o.w = val[4 * h + 3] * rs;
        *(f32x4*)(g.logits + dst + n) = o;
      } else {
#pragma unroll
        for (int t = 0; t < 4; ++t) if (n + t < nend) g.logits[dst + n + t] = val[4 * h + t] * rs;
      }
    }
  }
}

// The streaming loop of one wave: NR weight blocks over k-steps [kb, ke), DEPTH k-steps (DEPTH*NR tiles of 1 KiB)
// in flight.  Loads are issued unconditionally (indices clamped to the last step) so that the number in flight is
// static and the compiler waits for exactly the tile it needs.  The first DEPTH steps are requested by
// k2_prologue BEFORE the block stages its X slice, so HBM is already busy while LDS is being filled.
// Tile registers: pre[(dd*NR + j)*NWP + p].
template <int NWP, int NR, int DEPTH>
__device__ __forceinline__ void k2_prologue(int kb, int ke, const u32x4* const* wp, size_t wps, u32x4* pre) {
  if (ke <= kb) return;
  const int klast = ke - 1;
#pragma unroll
  for (int dd = 0; dd < DEPTH; ++dd) {
    const int kk = min(kb + dd, klast);
#pragma unroll
    for (int j = 0; j < NR; ++j)
#pragma unroll
      for (int p = 0; p < NWP; ++p) pre[(dd * NR + j) * NWP + p] = *(const u32x4*)((const bf16_t*)(wp[j] + (size_t)kk * 64) + p * wps);
  }
}

template <int NWP, int NXP, int NR, int DEPTH>
__device__ __forceinline__ void k2_stream(const u32x4* __restrict__ xs, int kt, int kb, int ke, const u32x4* const* wp,
                                          size_t wps, f32x16* acc, int lane, u32x4* pre) {
  constexpr int PMAX = NWP > NXP ? NWP : NXP;
  if (ke <= kb) return;
  const int klast = ke - 1;
  int k = kb;
  for (; k + DEPTH < ke; k += DEPTH) {
#pragma unroll
    for (int dd = 0; dd < DEPTH; ++dd) {
      const int kk = k + dd;
      u32x4 bq[NXP];
#pragma unroll
      for (int q = 0; q < NXP; ++q) bq[q] = xs[((size_t)q * kt + kk) * 64 + lane];
#pragma unroll
      for (int j = 0; j < NR; ++j)
#pragma unroll
        for (int p = 0; p < NWP; ++p)
#pragma unroll
          for (int q = 0; q < NXP; ++q)
            if (p + q < PMAX)
              acc[j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, pre[(dd * NR + j) * NWP + p]),
                                                                __builtin_bit_cast(bf16x8, bq[q]), acc[j], 0, 0, 0);
      const int kn = min(kk + DEPTH, klast);
#pragma unroll
      for (int j = 0; j < NR; ++j)
#pragma unroll
        for (int p = 0; p < NWP; ++p) pre[(dd * NR + j) * NWP + p] = *(const u32x4*)((const bf16_t*)(wp[j] + (size_t)kn * 64) + p * wps);
      __builtin_amdgcn_sched_barrier(0);          // keep "use a slot, refill that slot" in program order
    }
  }
#pragma unroll
  for (int dd = 0; dd < DEPTH; ++dd) {
    const int kk = k + dd;
    if (kk < ke) {
      u32x4 bq[NXP];
#pragma unroll
      for (int q = 0; q < NXP; ++q) bq[q] = xs[((size_t)q * kt + kk) * 64 + lane];
#pragma unroll
      for (int j = 0; j < NR; ++j)
#pragma unroll
        for (int p = 0; p < NWP; ++p)
#pragma unroll
          for (int q = 0; q < NXP; ++q)
            if (p + q < PMAX)
              acc[j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, pre[(dd * NR + j) * NWP + p]),
                                                                __builtin_bit_cast(bf16x8, bq[q]), acc[j], 0, 0, 0);
    }
  }
}

// ---- 4-bit weights against an activation slice in LDS (layout and arithmetic: see k_pack_weight_q4 / fk_stream_q4) ------
// A wave owns NR row blocks over the groups [gb, ge) of the work-group's K slice (slice-relative group indices; the
// slice starts at group g0 of the matrix).  With a quarter of the weight bytes the activation fragments are what a CU
// fetches most of, so here they are fetched ONCE per work-group (into LDS) and every wave reads them from there.
template <int NXP, int NR>
__device__ __forceinline__ void k2_stream_q4(const u32x4* __restrict__ xs, int kt, int g0, int gb, int ge, const u32x4* const* wq,
                                             const u32x4* const* sq, f32x16* acc, int lane) {
  if (ge <= gb) return;
  const int glast = ge - 1;
  u32x4 a4[2][NR];
  const u32x4 ones = {0x3F803F80u, 0x3F803F80u, 0x3F803F80u, 0x3F803F80u};
#pragma unroll
  for (int st = 0; st < 2; ++st)
#pragma unroll
    for (int j = 0; j < NR; ++j) a4[st][j] = wq[j][(size_t)(2 * (g0 + gb) + st) * 64];
  for (int g = gb; g < ge; ++g) {
    f32x16 part[NR], sx;
#pragma unroll
    for (int r = 0; r < 16; ++r) sx[r] = 0.f;
#pragma unroll
    for (int j = 0; j < NR; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) part[j][r] = 0.f;
    u32x4 sraw[NR][2];
#pragma unroll
    for (int j = 0; j < NR; ++j) { sraw[j][0] = sq[j][(size_t)(g0 + g) * 4]; sraw[j][1] = sq[j][(size_t)(g0 + g) * 4 + 1]; }
    const int gn = min(g + 1, glast);
#pragma unroll
    for (int st = 0; st < 2; ++st) {
#pragma unroll
      for (int ks = 0; ks < 4; ++ks) {
        const int kk = 8 * g + 4 * st + ks;                    // k-step inside the slice
        u32x4 bq[NXP];
#pragma unroll
        for (int q = 0; q < NXP; ++q) bq[q] = xs[((size_t)q * kt + kk) * 64 + lane];
#pragma unroll
        for (int j = 0; j < NR; ++j) {
          const uint32_t wd = ks == 0 ? a4[st][j].x : ks == 1 ? a4[st][j].y : ks == 2 ? a4[st][j].z : a4[st][j].w;
          u32x4 av;
          av.x = (wd & 0x000F000Fu) | 0x43004300u;
          av.y = ((wd >> 4) & 0x000F000Fu) | 0x43004300u;
          av.z = ((wd >> 8) & 0x000F000Fu) | 0x43004300u;
          av.w = ((wd >> 12) & 0x000F000Fu) | 0x43004300u;
#pragma unroll
          for (int q = 0; q < NXP; ++q)
            part[j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, av), __builtin_bit_cast(bf16x8, bq[q]), part[j], 0, 0, 0);
        }
#pragma unroll
        for (int q = 0; q < NXP; ++q)
          sx = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, ones), __builtin_bit_cast(bf16x8, bq[q]), sx, 0, 0, 0);
      }
#pragma unroll
      for (int j = 0; j < NR; ++j) a4[st][j] = wq[j][(size_t)(2 * (g0 + gn) + st) * 64];
      __builtin_amdgcn_sched_barrier(0);
    }
#pragma unroll
    for (int j = 0; j < NR; ++j) {
      const uint32_t sw[8] = {sraw[j][0].x, sraw[j][0].y, sraw[j][0].z, sraw[j][0].w, sraw[j][1].x, sraw[j][1].y, sraw[j][1].z, sraw[j][1].w};
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const float sv = __builtin_bit_cast(float, (r & 1) ? (sw[r >> 1] & 0xFFFF0000u) : (sw[r >> 1] << 16));
        acc[j][r] += sv * (part[j][r] - 136.0f * sx[r]);
      }
    }
  }
}
template <int NXP, int RW, int NR>
__device__ __forceinline__ void k2_stream_q4_dispatch(int nr, const u32x4* xs, int kt, int g0, int gb, int ge, const u32x4* const* wq,
                                                      const u32x4* const* sq, f32x16* acc, int lane) {
  if (nr == NR) k2_stream_q4<NXP, NR>(xs, kt, g0, gb, ge, wq, sq, acc, lane);
  else if constexpr (NR > 1) k2_stream_q4_dispatch<NXP, RW, NR - 1>(nr, xs, kt, g0, gb, ge, wq, sq, acc, lane);
}

template <int NWP, int NXP, int RW, int NR, int DEPTH>
__device__ __forceinline__ void k2_prologue_dispatch(int nr, int kb, int ke, const u32x4* const* wp, size_t wps, u32x4* pre) {
  if (nr == NR) k2_prologue<NWP, NR, (DEPTH * RW) / NR>(kb, ke, wp, wps, pre);
  else if constexpr (NR > 1) k2_prologue_dispatch<NWP, NXP, RW, NR - 1, DEPTH>(nr, kb, ke, wp, wps, pre);
}
template <int NWP, int NXP, int RW, int NR, int DEPTH>
__device__ __forceinline__ void k2_stream_dispatch(int nr, const u32x4* xs, int kt, int kb, int ke, const u32x4* const* wp,
                                                   size_t wps, f32x16* acc, int lane, u32x4* pre) {
  if (nr == NR) k2_stream<NWP, NXP, NR, (DEPTH * RW) / NR>(xs, kt, kb, ke, wp, wps, acc, lane, pre);
  else if constexpr (NR > 1) k2_stream_dispatch<NWP, NXP, RW, NR - 1, DEPTH>(nr, xs, kt, kb, ke, wp, wps, acc, lane, pre);
}

template <int NWP, int NXP, int RW, int DEPTH, bool Q4 = false>
__global__ __launch_bounds__(V2_THREADS) void k2_gemm(Gemm2 g) {
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  __shared__ float sh_small[16 * 33];
  __shared__ int s_last;
  if (g.skip_flag && *g.skip_flag == 0) return;               // uniform over the whole grid
  u32x4* xs = (u32x4*)smem;
  const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
  // the work split in 32-bit arithmetic: every product stays far below 2^31 (<= 1024 groups x a few thousand row blocks)
  const unsigned uS = g.S, ugroups = g.groups, uNRB = g.NRB, uKS = g.KS, ulanes = g.lanes, ukparts = g.kparts;
  const int s = blockIdx.x % uS, grp = blockIdx.x / uS;
  const int rb0 = (unsigned)grp * uNRB / ugroups, rb1 = (unsigned)(grp + 1) * uNRB / ugroups;
  // K slice of the work-group and K part of the wave: in k-steps, or (4-bit weights) in whole groups of 8 k-steps
  const int gs0 = Q4 ? (int)((unsigned)s * (unsigned)g.NG / uS) : 0, gs1 = Q4 ? (int)((unsigned)(s + 1) * (unsigned)g.NG / uS) : 0;
  const int ks0 = Q4 ? 8 * gs0 : (int)((unsigned)s * uKS / uS), ks1 = Q4 ? 8 * gs1 : (int)((unsigned)(s + 1) * uKS / uS), kt = ks1 - ks0;
  const int la = (unsigned)w % ulanes, kb_i = (unsigned)w / ulanes;
  const int qgb = (unsigned)kb_i * (unsigned)(gs1 - gs0) / ukparts, qge = (unsigned)(kb_i + 1) * (unsigned)(gs1 - gs0) / ukparts;
  const int kb = Q4 ? 8 * qgb : (int)((unsigned)kb_i * (unsigned)kt / ukparts), ke = Q4 ? 8 * qge : (int)((unsigned)(kb_i + 1) * (unsigned)kt / ukparts);
  unsigned long long* tr = TRACE_PTR((g.trace && threadIdx.x == 0) ? g.trace + (size_t)blockIdx.x * 8 : nullptr);
  TRACE_STAMP(tr, 0);
  int nr = 0;
  for (int j = 0; j < RW; ++j) nr += (rb0 + la + j * g.lanes < rb1) ? 1 : 0;
  nr = __builtin_amdgcn_readfirstlane(nr);

  const u32x4* wp[RW];
#pragma unroll
  for (int j = 0; j < RW; ++j) {
    int rb = rb0 + la + j * g.lanes;
    if (rb >= rb1) rb = rb0;                                  // never dereferenced: only the first nr entries are used
    wp[j] = (const u32x4*)(g.W + ((size_t)rb * g.KS + ks0) * 512) + lane;
  }
  // the first weight tiles are requested before anything else (a wave with fewer row blocks keeps more k-steps in flight)
  u32x4 pre[DEPTH * RW * NWP];
  if constexpr (!Q4) k2_prologue_dispatch<NWP, NXP, RW, RW, DEPTH>(nr, kb, ke, wp, g.wps, pre);

  // row facts and the 1/rms inputs the epilogue will want: requested now, used (by the last work-group) much later
  RowPre rp;
  rp.valid = 0; rp.seq = 0; rp.pos = 0; rp.slot = 0; rp.dst = -1;
  rp.ssq_part = rstd_class_partial(g.in_scale);
  if (g.epi == EPI_QKV) {
    const int m = threadIdx.x & 31;
    if (m < g.M) {
      const RowInfo ri = row_info(g.pass, g.tree, g.st, m);
      rp.valid = ri.valid; rp.seq = ri.seq; rp.pos = ri.pos; rp.slot = ri.slot;
    }
  } else if (g.epi == EPI_LOGITS) {
    const int m = threadIdx.x & 31;
    if (m < g.M) {
      const RowInfo ri = row_info(g.pass, g.tree, g.st, m);
      if (ri.valid) {
        if (g.out_kind == 0) { if (ri.node >= 0) rp.dst = ((long)ri.seq * g.tree->M + ri.node) * g.V; }
        else if (!(g.only_last_row && ri.rel != g.pass.chunk_n - 1 && g.pass.kind != PASS_VANILLA)) rp.dst = (long)ri.seq * g.V;
      }
    }
  }

  // stage this work-group's K slice of X: per plane a contiguous run of kt tiles (8 loads in flight per thread)
  for (int p = 0; p < NXP; ++p) {
    const u32x4* src = (const u32x4*)(g.XF + ((size_t)p * g.KS + ks0) * 512);
    u32x4* dst = xs + (size_t)p * kt * 64;
    const int n = kt * 64;
    for (int i0 = 0; i0 < n; i0 += V2_THREADS * 8) {
      u32x4 v[8];
#pragma unroll
      for (int u = 0; u < 8; ++u) v[u] = src[min(i0 + u * V2_THREADS + (int)threadIdx.x, n - 1)];
#pragma unroll
      for (int u = 0; u < 8; ++u) {
        const int i = i0 + u * V2_THREADS + (int)threadIdx.x;
        if (i < n) dst[i] = v[u];
      }
    }
  }
  f32x16 acc[RW];
#pragma unroll
  for (int j = 0; j < RW; ++j)
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[j][r] = 0.f;
  __syncthreads();
  TRACE_STAMP(tr, 1);
  if constexpr (Q4) {
    const u32x4* wq[RW];
    const u32x4* sq[RW];
#pragma unroll
    for (int j = 0; j < RW; ++j) {
      int rb = rb0 + la + j * g.lanes;
      if (rb >= rb1) rb = rb0;
      wq[j] = (const u32x4*)g.W + (size_t)rb * (size_t)(g.KS / 4) * 64 + lane;
      sq[j] = (const u32x4*)g.SC + (size_t)rb * (size_t)g.NG * 4 + 2 * (lane >> 5);
    }
    k2_stream_q4_dispatch<NXP, RW, RW>(nr, xs, kt, gs0, qgb, qge, wq, sq, acc, lane);
  } else
  k2_stream_dispatch<NWP, NXP, RW, RW, DEPTH>(nr, xs, kt, kb, ke, wp, g.wps, acc, lane, pre);
  TRACE_STAMP(tr, 2);
  // waves that split K inside the work-group: sum through LDS in k-part order
  if (g.kparts > 1) {
    __syncthreads();                                          // the X slice is no longer needed
    float* red = (float*)smem;
    if (kb_i > 0) {
#pragma unroll
      for (int j = 0; j < RW; ++j)
        if (j < nr)
#pragma unroll
          for (int r = 0; r < 16; ++r)
            red[((((size_t)la * (g.kparts - 1) + (kb_i - 1)) * RW + j) * 16 + r) * 64 + lane] = acc[j][r];
    }
    __syncthreads();
    if (kb_i == 0) {
      for (int b = 1; b < g.kparts; ++b)
#pragma unroll
        for (int j = 0; j < RW; ++j)
          if (j < nr)
#pragma unroll
            for (int r = 0; r < 16; ++r)
              acc[j][r] += red[((((size_t)la * (g.kparts - 1) + (b - 1)) * RW + j) * 16 + r) * 64 + lane];
    }
  }
  if (kb_i == 0) {
#pragma unroll
    for (int j = 0; j < RW; ++j)
      if (j < nr) {
        const int rb = rb0 + la + j * g.lanes;
#pragma unroll
        for (int i = 0; i < 4; ++i) {                           // accumulator registers 4i..4i+3 = rows 8i + 4(lane/32) + 0..3
          f32x4 v; v.x = acc[j][4 * i]; v.y = acc[j][4 * i + 1]; v.z = acc[j][4 * i + 2]; v.w = acc[j][4 * i + 3];
          coh_store16(g.PT, pt_quad_bytes(s, g.Npad, rb * 32 + 8 * i + 4 * (lane >> 5), lane & 31), v);
        }
      }
  }
  // publish the partials; the last work-group of this row group to arrive finishes the job
  publish_wait();                                               // every coherent store above has been acknowledged
  __syncthreads();
  if (threadIdx.x == 0) {
    int old = __hip_atomic_fetch_add(g.counters + grp, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    s_last = (old == g.S - 1);
    if (s_last) __hip_atomic_store(g.counters + grp, 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);   // ready for the next launch
  }
  __syncthreads();
  TRACE_STAMP(tr, 3);
  if (!s_last) return;
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup");
  const int n0 = rb0 * 32, n1 = min(rb1 * 32, g.N);
  if (n1 <= n0) return;
  __shared__ float rstd_s[32];
  if (g.epi != EPI_RESID) block_rstd_finish(g.in_scale, rp.ssq_part, rstd_s, sh_small);
  switch (g.epi) {
    case EPI_QKV: epilogue_qkv<NXP>(g, n0, n1, rstd_s, rp); break;
    case EPI_RESID: epilogue_resid<NXP>(g, grp, n0, n1, sh_small); break;
    case EPI_SWIGLU: epilogue_swiglu<NXP>(g, n0, n1, rstd_s); break;
    default: epilogue_logits(g, n0, n1, rstd_s, rp); break;
  }
  TRACE_STAMP(tr, 4);
}

// ---- full-K variant for wide matrices (QKV, gate/up, LM head) ----------------------------------------------------------
// A work-group owns up to 4 whole row blocks over ALL of K: no partial sums leave the chip, no arrival counter, no
// last work-group.  The eight waves split K eight ways; a wave streams, per k-step, the weight tiles of the group's
// row blocks from HBM AND the activation fragments of that k-step straight from L2 (every work-group reads the whole
// X, 512 KB at d = 4096, which the 32 work-groups of an XCD share through its L2) -- no LDS staging, no barrier until
// the end.  The waves' sums meet in LDS (k-part order) and the epilogue runs on them in place.  Costs more bytes per
// CU than the split-K kernel and saves its publish / arrive / read-back round trips; pays off for matrices with at
// least as many row blocks as there are CUs.
// The activation fragments come through buffer loads: a lane whose row (lane % 32) is not a live row of the pass gets
// an offset beyond the buffer, which the hardware answers with zeros WITHOUT touching memory -- a pass of M rows moves
// M/32 of the fragment bytes (26/32 in a 26-node verify, 1/8 and less in the head's passes).
// Row-masked weight loads (half-block work split): the tiles of row block j come through a buffer resource over the
// whole matrix; vo[j] is the lane's byte offset inside a tile, or an out-of-range offset for lanes whose weight row
// is not this work-group's (zeros, no memory access); so[j] the byte offset of the block's first tile.
struct FkHalf { __amdgpu_buffer_rsrc_t rs; uint32_t vo[4]; uint32_t so[4]; };

template <int NWP, int NXP, int NR, int DEPTH, bool WB = false>
__device__ __forceinline__ void fk_stream(const bf16_t* __restrict__ XF, int KS, int M, int kb, int ke, const u32x4* const* wp,
                                          size_t wps, f32x16* acc, int lane, const FkHalf* hw = nullptr) {
  static_assert(!WB || NWP == 1, "row-masked weight loads exist for one weight plane only");
  constexpr int PMAX = NWP > NXP ? NWP : NXP;
  if (ke <= kb) return;
  const int klast = ke - 1;
  u32x4 ta[DEPTH][NR][NWP], tb[DEPTH][NXP];
  const __amdgpu_buffer_rsrc_t xrs = __builtin_amdgcn_make_buffer_rsrc((void*)XF, 0, NXP * KS * 1024, 0x00020000);
  const uint32_t xlane = (lane & 31) < M ? (uint32_t)lane * 16u : 0x80000000u;   // dead rows: out of range
#define FK_XLOAD(q, kk) __builtin_bit_cast(u32x4, __builtin_amdgcn_raw_buffer_load_b128(xrs, xlane, (uint32_t)(((q) * KS + (kk)) * 1024), 0))
  auto wload = [&](int j, int p, int kk) -> u32x4 {
    if constexpr (WB) return __builtin_bit_cast(u32x4, __builtin_amdgcn_raw_buffer_load_b128(hw->rs, hw->vo[j], hw->so[j] + (uint32_t)kk * 1024u, 0));
    else return *(const u32x4*)((const bf16_t*)(wp[j] + (size_t)kk * 64) + p * wps);
  };
#pragma unroll
  for (int dd = 0; dd < DEPTH; ++dd) {
    const int kk = min(kb + dd, klast);
#pragma unroll
    for (int j = 0; j < NR; ++j)
#pragma unroll
      for (int p = 0; p < NWP; ++p) ta[dd][j][p] = wload(j, p, kk);
#pragma unroll
    for (int q = 0; q < NXP; ++q) tb[dd][q] = FK_XLOAD(q, kk);
  }
  int k = kb;
  for (; k + DEPTH < ke; k += DEPTH) {
#pragma unroll
    for (int dd = 0; dd < DEPTH; ++dd) {
#pragma unroll
      for (int j = 0; j < NR; ++j)
#pragma unroll
        for (int p = 0; p < NWP; ++p)
#pragma unroll
          for (int q = 0; q < NXP; ++q)
            if (p + q < PMAX)
              acc[j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, ta[dd][j][p]),
                                                                __builtin_bit_cast(bf16x8, tb[dd][q]), acc[j], 0, 0, 0);
      const int kn = min(k + dd + DEPTH, klast);
#pragma unroll
      for (int j = 0; j < NR; ++j)
#pragma unroll
        for (int p = 0; p < NWP; ++p) ta[dd][j][p] = wload(j, p, kn);
#pragma unroll
      for (int q = 0; q < NXP; ++q) tb[dd][q] = FK_XLOAD(q, kn);
      __builtin_amdgcn_sched_barrier(0);
    }
  }
#pragma unroll
  for (int dd = 0; dd < DEPTH; ++dd) {
    if (k + dd < ke) {
#pragma unroll
      for (int j = 0; j < NR; ++j)
#pragma unroll
        for (int p = 0; p < NWP; ++p)
#pragma unroll
          for (int q = 0; q < NXP; ++q)
            if (p + q < PMAX)
              acc[j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, ta[dd][j][p]),
                                                                __builtin_bit_cast(bf16x8, tb[dd][q]), acc[j], 0, 0, 0);
    }
  }
}
#undef FK_XLOAD
template <int NWP, int NXP, int NR, bool WB = false>
__device__ __forceinline__ void fk_stream_dispatch(int nr, const bf16_t* XF, int KS, int M, int kb, int ke, const u32x4* const* wp,
                                                   size_t wps, f32x16* acc, int lane, const FkHalf* hw = nullptr) {
  constexpr int DEPTH = NWP == 1 ? (NR == 1 ? 8 : NR == 2 ? 6 : NR == 3 ? 5 : 4) : 2;   // ~24 KiB in flight per wave; deeper measured the same
  if (nr == NR) fk_stream<NWP, NXP, NR, DEPTH, WB>(XF, KS, M, kb, ke, wp, wps, acc, lane, hw);
  else if constexpr (NR > 1) fk_stream_dispatch<NWP, NXP, NR - 1, WB>(nr, XF, KS, M, kb, ke, wp, wps, acc, lane, hw);
}

// ---- the same stream over 4-bit weights (see k_pack_weight_q4 for the layout) -------------------------------------------
// A wave owns the groups [gb, ge) of 128 k.  Per group: two 16-byte loads per row block bring the codes of its 8 k-steps;
// a k-step's A operand is 128 + code (exact in bf16) -- two ALU operations per pair of codes, which run beside the MFMAs
// -- so the group's partial sums come out as sum_k x_k (128 + c_k); an MFMA against an all-ones tile gives sum_k x_k of
// the same k-steps, and the group is folded into the result as  acc += s_row * (partial - 136 * sum_x)  in fp32.
// Activation fragments are streamed from L2 as in fk_stream, one group (8 k-steps) ahead; the next group's codes are
// requested as soon as a super-tile's registers are free.
template <int NXP, int NR>
__device__ __forceinline__ void fk_stream_q4(const bf16_t* __restrict__ XF, int KS, int M, int gb, int ge, const u32x4* const* wq,
                                             const u32x4* const* sq /*scales of (block j, group 0), this lane's half*/, int NG,
                                             f32x16* acc, int lane) {
  if (ge <= gb) return;
  const int glast = ge - 1;
  const __amdgpu_buffer_rsrc_t xrs = __builtin_amdgcn_make_buffer_rsrc((void*)XF, 0, NXP * KS * 1024, 0x00020000);
  const uint32_t xlane = (lane & 31) < M ? (uint32_t)lane * 16u : 0x80000000u;   // dead rows: out of range -> zeros
#define Q4_XLOAD(q, kk) __builtin_bit_cast(u32x4, __builtin_amdgcn_raw_buffer_load_b128(xrs, xlane, (uint32_t)(((q) * KS + (kk)) * 1024), 0))
  u32x4 a4[2][NR], tb[8][NXP];                                 // codes of a group; activation fragments one group ahead
  const u32x4 ones = {0x3F803F80u, 0x3F803F80u, 0x3F803F80u, 0x3F803F80u};
#pragma unroll
  for (int st = 0; st < 2; ++st)
#pragma unroll
    for (int j = 0; j < NR; ++j) a4[st][j] = wq[j][(size_t)(2 * gb + st) * 64];
#pragma unroll
  for (int i = 0; i < 8; ++i)
#pragma unroll
    for (int q = 0; q < NXP; ++q) tb[i][q] = Q4_XLOAD(q, 8 * gb + i);
  for (int g = gb; g < ge; ++g) {
    f32x16 part[NR], sx;
#pragma unroll
    for (int r = 0; r < 16; ++r) sx[r] = 0.f;
#pragma unroll
    for (int j = 0; j < NR; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) part[j][r] = 0.f;
    u32x4 sraw[NR][2];                                          // this group's scales: needed after its 8 k-steps
#pragma unroll
    for (int j = 0; j < NR; ++j) { sraw[j][0] = sq[j][(size_t)g * 4]; sraw[j][1] = sq[j][(size_t)g * 4 + 1]; }
    const int gn = min(g + 1, glast);
#pragma unroll
    for (int st = 0; st < 2; ++st) {
#pragma unroll
      for (int ks = 0; ks < 4; ++ks) {
        const int kk = 8 * g + 4 * st + ks;
        auto expand = [&](int j) {
          const uint32_t wd = ks == 0 ? a4[st][j].x : ks == 1 ? a4[st][j].y : ks == 2 ? a4[st][j].z : a4[st][j].w;
          u32x4 av;
          av.x = (wd & 0x000F000Fu) | 0x43004300u;
          av.y = ((wd >> 4) & 0x000F000Fu) | 0x43004300u;
          av.z = ((wd >> 8) & 0x000F000Fu) | 0x43004300u;
          av.w = ((wd >> 12) & 0x000F000Fu) | 0x43004300u;
          return av;
        };
        if constexpr (NR <= 2) {
          // plane by plane, so that consecutive MFMAs write different accumulators (measured: QKV 20.4 -> 19.3 us, down
          // 19.0 -> 17.8 us); with three row blocks the expanded operands held across the planes spill, so they keep the
          // block-by-block order
          u32x4 av[NR];
#pragma unroll
          for (int j = 0; j < NR; ++j) av[j] = expand(j);
#pragma unroll
          for (int q = 0; q < NXP; ++q) {
#pragma unroll
            for (int j = 0; j < NR; ++j)
              part[j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, av[j]), __builtin_bit_cast(bf16x8, tb[4 * st + ks][q]), part[j], 0, 0, 0);
            sx = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, ones), __builtin_bit_cast(bf16x8, tb[4 * st + ks][q]), sx, 0, 0, 0);
          }
        } else {
#pragma unroll
          for (int j = 0; j < NR; ++j) {
            const u32x4 av = expand(j);
#pragma unroll
            for (int q = 0; q < NXP; ++q)
              part[j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, av), __builtin_bit_cast(bf16x8, tb[4 * st + ks][q]), part[j], 0, 0, 0);
          }
#pragma unroll
          for (int q = 0; q < NXP; ++q)
            sx = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, ones), __builtin_bit_cast(bf16x8, tb[4 * st + ks][q]), sx, 0, 0, 0);
        }
        // use a slot, refill that slot: the same k-step of the next group
        (void)kk;
#pragma unroll
        for (int q = 0; q < NXP; ++q) tb[4 * st + ks][q] = Q4_XLOAD(q, 8 * gn + 4 * st + ks);
      }
      // the super-tile's code registers are free: request the next group's
#pragma unroll
      for (int j = 0; j < NR; ++j) a4[st][j] = wq[j][(size_t)(2 * gn + st) * 64];
      __builtin_amdgcn_sched_barrier(0);
    }
#pragma unroll
    for (int j = 0; j < NR; ++j) {
      const uint32_t sw[8] = {sraw[j][0].x, sraw[j][0].y, sraw[j][0].z, sraw[j][0].w, sraw[j][1].x, sraw[j][1].y, sraw[j][1].z, sraw[j][1].w};
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const float sv = __builtin_bit_cast(float, (r & 1) ? (sw[r >> 1] & 0xFFFF0000u) : (sw[r >> 1] << 16));
        acc[j][r] += sv * (part[j][r] - 136.0f * sx[r]);
      }
    }
  }
#undef Q4_XLOAD
}
template <int NXP, int NR>
__device__ __forceinline__ void fk_stream_q4_dispatch(int nr, const bf16_t* XF, int KS, int M, int gb, int ge, const u32x4* const* wq,
                                                      const u32x4* const* sq, int NG, f32x16* acc, int lane) {
  if (nr == NR) fk_stream_q4<NXP, NR>(XF, KS, M, gb, ge, wq, sq, NG, acc, lane);
  else if constexpr (NR > 1) fk_stream_q4_dispatch<NXP, NR - 1>(nr, XF, KS, M, gb, ge, wq, sq, NG, acc, lane);
}

// sum over the 8 waves of element (row n_local of row block j, token m) of the per-wave accumulators parked in LDS
// as red[w][j][r][lane] (MFMA layout: r = 4*(n_local/8) + n_local%4, lane = m + 32*((n_local/4)%2)); k-part order
__device__ inline float fk_sum(const float* red, int nrmax, int j, int n_local, int m) {
  const int r = 4 * (n_local >> 3) + (n_local & 3), l = m + 32 * ((n_local >> 2) & 1);
  float a = 0.f;
#pragma unroll
  for (int w = 0; w < 8; ++w) a += red[(((size_t)w * nrmax + j) * 16 + r) * 64 + l];
  return a;
}

// HALF: the unit of the work split is half a row block (16 weight rows) instead of a whole one, for matrices whose
// row blocks do not divide evenly over the CUs (QKV at d = 4096: 384 blocks over 256 CUs = 1 or 2 each, but 3 halves
// each) and for matrices with fewer row blocks than CUs (O, down, FC at d = 4096: 128 blocks = one half per CU, which
// keeps them whole-K: no partial sums are exchanged).  A work-group then owns a run of halves; of a block it shares
// with a neighbour it loads and finishes only its own 16 rows (the other lanes of the tile load nothing and multiply
// zeros).  Rotate-half pairs are adjacent rows, so a half holds whole pairs.  Epilogues: QKV and the residual one.
template <int NWP, int NXP, int NRMAX, bool HALF = false, bool Q4 = false>
__global__ __launch_bounds__(V2_THREADS) void k2_gemm_fk(Gemm2 g) {
  static_assert(!Q4 || (!HALF && NWP == 1), "4-bit weights: whole row blocks, one plane");
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  __shared__ float sh_small[16 * 33];
  __shared__ float rstd_s[32];
  float* red = (float*)smem;                                    // [8][NRMAX][16][64]
  if (g.skip_flag && *g.skip_flag == 0) return;                 // MoE: no row selected this expert (uniform over the grid)
  const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
  unsigned long long* tr = TRACE_PTR((g.trace && threadIdx.x == 0) ? g.trace + (size_t)blockIdx.x * 8 : nullptr);
  TRACE_STAMP(tr, 0);
  const unsigned G = gridDim.x;
  int rb0, rb1, row_lo = 0, row_hi = 32;                        // rows [row_lo, 32) of the first block, [0, row_hi) of the last
  if constexpr (HALF) {
    const unsigned U = 2u * (unsigned)g.NRB;
    const unsigned u0 = (unsigned)blockIdx.x * U / G, u1 = (unsigned)(blockIdx.x + 1) * U / G;
    rb0 = (int)(u0 >> 1); rb1 = (int)((u1 + 1) >> 1);
    row_lo = (u0 & 1) ? 16 : 0; row_hi = (u1 & 1) ? 16 : 32;
  } else {
    rb0 = (unsigned)blockIdx.x * (unsigned)g.NRB / G; rb1 = (unsigned)(blockIdx.x + 1) * (unsigned)g.NRB / G;
  }
  const int nr = rb1 - rb0;                                     // <= NRMAX (host)
  const int kb = (unsigned)w * (unsigned)g.KS / 8u, ke = (unsigned)(w + 1) * (unsigned)g.KS / 8u;
  const u32x4* wp[NRMAX];
#pragma unroll
  for (int j = 0; j < NRMAX; ++j) wp[j] = (const u32x4*)(g.W + (size_t)min(rb0 + j, g.NRB - 1) * g.KS * 512) + lane;
  FkHalf hw;
  if constexpr (HALF) {
    hw.rs = __builtin_amdgcn_make_buffer_rsrc((void*)g.W, 0, (int)((unsigned)g.NRB * (unsigned)g.KS * 1024u), 0x00020000);
    const int row = lane & 31;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const bool mine = j < nr && row >= (j == 0 ? row_lo : 0) && row < (j == nr - 1 ? row_hi : 32);
      hw.vo[j] = mine ? (uint32_t)lane * 16u : 0x80000000u;
      hw.so[j] = (uint32_t)min(rb0 + j, g.NRB - 1) * (uint32_t)g.KS * 1024u;
    }
  }
  f32x16 acc[NRMAX];
#pragma unroll
  for (int j = 0; j < NRMAX; ++j)
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[j][r] = 0.f;
  // row facts and 1/rms inputs, requested before the stream
  RowPre rp;
  rp.valid = 0; rp.seq = 0; rp.pos = 0; rp.slot = 0; rp.dst = -1;
  rp.ssq_part = rstd_class_partial(g.in_scale);
  {
    const int m = threadIdx.x & 31;
    if (m < g.M) {
      const RowInfo ri = row_info(g.pass, g.tree, g.st, m);
      if (g.epi == EPI_QKV) { rp.valid = ri.valid; rp.seq = ri.seq; rp.pos = ri.pos; rp.slot = ri.slot; }
      else if (g.epi == EPI_LOGITS && ri.valid) {
        if (g.out_kind == 0) { if (ri.node >= 0) rp.dst = ((long)ri.seq * g.tree->M + ri.node) * g.V; }
        else if (!(g.only_last_row && ri.rel != g.pass.chunk_n - 1 && g.pass.kind != PASS_VANILLA)) rp.dst = (long)ri.seq * g.V;
      }
    }
  }
  if constexpr (Q4) {
    // K is split over the waves by groups of 128; pointers to the codes / scales of each row block
    const int gb = (unsigned)w * (unsigned)g.NG / 8u, ge = (unsigned)(w + 1) * (unsigned)g.NG / 8u;
    const u32x4* wq[NRMAX];
    const u32x4* sq[NRMAX];
#pragma unroll
    for (int j = 0; j < NRMAX; ++j) {
      const size_t rb = (size_t)min(rb0 + j, g.NRB - 1);
      wq[j] = (const u32x4*)g.W + rb * (size_t)(g.KS / 4) * 64 + lane;
      sq[j] = (const u32x4*)g.SC + rb * (size_t)g.NG * 4 + 2 * (lane >> 5);
    }
    fk_stream_q4_dispatch<NXP, NRMAX>(nr, g.XF, g.KS, g.M, gb, ge, wq, sq, g.NG, acc, lane);
  } else
  fk_stream_dispatch<NWP, NXP, NRMAX, HALF>(nr, g.XF, g.KS, g.M, kb, ke, wp, g.wps, acc, lane, &hw);
  TRACE_STAMP_AFTER(tr, 2, acc[0][0]);
  // park every wave's sums in LDS
#pragma unroll
  for (int j = 0; j < NRMAX; ++j)
    if (j < nr)
#pragma unroll
      for (int r = 0; r < 16; ++r) red[(((size_t)w * NRMAX + j) * 16 + r) * 64 + lane] = acc[j][r];
  block_rstd_finish(g.in_scale, rp.ssq_part, rstd_s, sh_small);   // (contains the barriers that publish `red`)
  __syncthreads();
  const int m = threadIdx.x & 31, slot = threadIdx.x >> 5;     // 16 slots of 32 tokens
  const bool live = m < g.M;
  const float rs = live ? rstd_s[m] : 0.f;
  if (g.epi == EPI_SWIGLU) {
    // item = (row block j, half c2): 8 outputs f = rb*16 + 8*c2 .. +7 from gate rows 8*c2.. and up rows 16 + 8*c2..
    for (int it = slot; it < nr * 2; it += 16) {
      const int j = it >> 1, c2 = it & 1;
      float x[8];
#pragma unroll
      for (int t = 0; t < 8; ++t) {
        const float gg = fk_sum(red, NRMAX, j, 8 * c2 + t, m) * rs, uu = fk_sum(red, NRMAX, j, 16 + 8 * c2 + t, m) * rs;
        x[t] = gg / (1.0f + __expf(-gg)) * uu;
      }
      if (live) xf_store8(g.xf_out, m, (rb0 + j) * 16 + 8 * c2, 1, g.xf_KS, NXP, x);
    }
  } else if (g.epi == EPI_QKV) {
    const int dh = g.kv.head_dim, half = dh >> 1, KVH = g.kv.n_kv_heads, H = g.H;
    // item = (row block j, rotate-half pair pp of 16): rows 2pp, 2pp + 1 of the block
    for (int it = slot; it < nr * 16; it += 16) {
      const int j = it >> 4, pp = it & 15;
      const int n = (rb0 + j) * 32 + 2 * pp;
      if (n >= g.N || !live) continue;
      if (HALF && (2 * pp < (j == 0 ? row_lo : 0) || 2 * pp >= (j == nr - 1 ? row_hi : 32))) continue;   // the neighbour's rows
      float a = fk_sum(red, NRMAX, j, 2 * pp, m) * rs, b = fk_sum(red, NRMAX, j, 2 * pp + 1, m) * rs;
      const int hd = n / dh, pr = n % dh;
      int d1, d2;
      if (hd < H + KVH) {        // q or k head: the two rows are a rotate-half pair
        const int i = pr >> 1;
        const float cs = g.rope_cos[(size_t)rp.pos * half + i], sn = g.rope_sin[(size_t)rp.pos * half + i];
        const float a2 = a * cs - b * sn, b2 = b * cs + a * sn;
        a = a2; b = b2; d1 = i; d2 = i + half;
      } else { d1 = pr; d2 = pr + 1; }
      if (hd < H) {
        float* q = g.Q + ((size_t)m * H + hd) * dh;
        q[d1] = a; q[d2] = b;
      } else if (rp.valid) {
        const int kvh = (hd - H) % KVH;
        const size_t off = kv_offset(g.kv, rp.seq, rp.slot, kvh);
        void* base = hd < H + KVH ? g.kv.k : g.kv.v;
        if (g.kv_f32) { ((float*)base)[off + d1] = a; ((float*)base)[off + d2] = b; }
        else { ((bf16_t*)base)[off + d1] = f32_to_bf16(a); ((bf16_t*)base)[off + d2] = f32_to_bf16(b); }
      }
    }
  } else if (g.epi == EPI_RESID) {
    // h_out = h_in + (routing weight *) W x + bias on this work-group's rows [n_lo, n_hi); per-token partial sums of
    // squares for the consumer's RMSNorm; x * gain of the next norm in fragment layout.  One output per thread and
    // round, parked in LDS behind `red`, then repacked in runs of 8 rows.
    float* xo = red + (size_t)8 * NRMAX * 16 * 64;              // [rows <= 32*NRMAX][33]
    const int n_lo = HALF ? rb0 * 32 + row_lo : rb0 * 32;
    const int n_hi = min(HALF ? (rb1 - 1) * 32 + row_hi : rb1 * 32, g.N);
    const float rw = g.row_w ? g.row_w[m] : 1.0f;
    float ss = 0.f;
    for (int nl = slot; nl < n_hi - n_lo; nl += 16) {
      const int n = n_lo + nl;
      float v = fk_sum(red, NRMAX, (n >> 5) - rb0, n & 31, m);
      if (g.row_w) v *= rw;
      if (g.bias) v += g.bias[n];
      if (g.h_in && live) v += g.h_in[(size_t)m * g.d + n];
      if (live) g.h_out[(size_t)m * g.d + n] = v;
      ss += v * v;
      xo[nl * 33 + m] = g.gain_next ? v * g.gain_next[n] : v;
    }
    sh_small[slot * 32 + m] = ss;
    __syncthreads();
    if (threadIdx.x < 32 && g.ssq_out) {
      float a = 0.f;
      for (int i = 0; i < 16; ++i) a += sh_small[i * 32 + threadIdx.x];
      g.ssq_out[blockIdx.x * 32 + threadIdx.x] = a;
    }
    for (int c = slot; c < (n_hi - n_lo + 7) >> 3; c += 16) {
      float x[8];
#pragma unroll
      for (int t = 0; t < 8; ++t) x[t] = 8 * c + t < n_hi - n_lo ? xo[(8 * c + t) * 33 + m] : 0.f;
      if (live) xf_store8(g.xf_out, m, n_lo + 8 * c, 1, g.xf_KS, NXP, x);
    }
  } else {                                                      // EPI_LOGITS
    const int nend = min(g.N, g.V);
    const bool vec = (g.V & 3) == 0;
    for (int it = slot; it < nr * 8; it += 16) {                // item = (row block j, quad of 4 rows)
      const int j = it >> 3, qd = it & 7;
      const int n = (rb0 + j) * 32 + 4 * qd;
      if (rp.dst < 0 || n >= nend) continue;
      float v[4];
#pragma unroll
      for (int t = 0; t < 4; ++t) v[t] = fk_sum(red, NRMAX, j, 4 * qd + t, m) * rs;
      if (vec && n + 4 <= nend) { f32x4 o; o.x = v[0]; o.y = v[1]; o.z = v[2]; o.w = v[3]; *(f32x4*)(g.logits + rp.dst + n) = o; }
      else {
#pragma unroll
        for (int t = 0; t < 4; ++t) if (n + t < nend) g.logits[rp.dst + n + t] = v[t];
      }
    }
  }
  TRACE_STAMP(tr, 4);
}

// ---- split-K with streamed activations (narrow matrices with a long K: O, down) ------------------------------------------
// The split-K kernel above keeps its X slice in LDS, so a long K forces many slices (11 at K = 11008) and the last
// work-group of a row group reads that many partials on one CU.  Here the slice is streamed from L2 like in the
// whole-K kernel (8 waves split the slice's k-steps, sums meet in LDS), so S is free: a few slices of a few row
// blocks each.  The work-group then costs its weights plus M/32 of its X slice in fetches, but exchanges only
// S x (row blocks) x 4 KiB per row group, and nothing waits for an LDS fill before the weight stream starts.
// Partials, arrival counter and epilogues are those of k2_gemm.
// Q4: 4-bit codes (k_pack_weight_q4); the slices are then whole groups of 128 columns (host: at least 8 groups a slice).
template <int NWP, int NXP, int NRMAX, bool Q4 = false>
__global__ __launch_bounds__(V2_THREADS) void k2_gemm_xk(Gemm2 g) {
  static_assert(!Q4 || NWP == 1, "4-bit weights: one plane");
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  __shared__ float sh_small[16 * 33];
  __shared__ float rstd_s[32];
  __shared__ int s_last;
  float* red = (float*)smem;                                    // [8][NRMAX][16][64]
  if (g.skip_flag && *g.skip_flag == 0) return;                 // uniform over the whole grid
  const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
  unsigned long long* tr = TRACE_PTR((g.trace && threadIdx.x == 0) ? g.trace + (size_t)blockIdx.x * 8 : nullptr);
  TRACE_STAMP(tr, 0);
  const unsigned uS = g.S, ugroups = g.groups, uNRB = g.NRB, uKS = g.KS;
  const int s = blockIdx.x % uS, grp = blockIdx.x / uS;
  const int rb0 = (unsigned)grp * uNRB / ugroups, rb1 = (unsigned)(grp + 1) * uNRB / ugroups;
  const int nr = rb1 - rb0;                                     // <= NRMAX (host)
  const int ks0 = (unsigned)s * uKS / uS, ks1 = (unsigned)(s + 1) * uKS / uS, kt = ks1 - ks0;
  const int kb = ks0 + (unsigned)w * (unsigned)kt / 8u, ke = ks0 + (unsigned)(w + 1) * (unsigned)kt / 8u;
  const u32x4* wp[NRMAX];
#pragma unroll
  for (int j = 0; j < NRMAX; ++j) wp[j] = (const u32x4*)(g.W + (size_t)min(rb0 + j, g.NRB - 1) * g.KS * 512) + lane;
  f32x16 acc[NRMAX];
#pragma unroll
  for (int j = 0; j < NRMAX; ++j)
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[j][r] = 0.f;
  RowPre rp;
  rp.valid = 0; rp.seq = 0; rp.pos = 0; rp.slot = 0; rp.dst = -1;
  rp.ssq_part = rstd_class_partial(g.in_scale);
  {
    const int m = threadIdx.x & 31;
    if (m < g.M && (g.epi == EPI_QKV || g.epi == EPI_LOGITS)) {
      const RowInfo ri = row_info(g.pass, g.tree, g.st, m);
      if (g.epi == EPI_QKV) { rp.valid = ri.valid; rp.seq = ri.seq; rp.pos = ri.pos; rp.slot = ri.slot; }
      else if (ri.valid) {
        if (g.out_kind == 0) { if (ri.node >= 0) rp.dst = ((long)ri.seq * g.tree->M + ri.node) * g.V; }
        else if (!(g.only_last_row && ri.rel != g.pass.chunk_n - 1 && g.pass.kind != PASS_VANILLA)) rp.dst = (long)ri.seq * g.V;
      }
    }
  }
  if constexpr (Q4) {
    const unsigned uNG = g.NG;
    const int G0 = (unsigned)s * uNG / uS, G1 = (unsigned)(s + 1) * uNG / uS, gt = G1 - G0;
    const int gb = G0 + (unsigned)w * (unsigned)gt / 8u, ge = G0 + (unsigned)(w + 1) * (unsigned)gt / 8u;
    const u32x4* wq[NRMAX];
    const u32x4* sq[NRMAX];
#pragma unroll
    for (int j = 0; j < NRMAX; ++j) {
      const size_t rb = (size_t)min(rb0 + j, g.NRB - 1);
      wq[j] = (const u32x4*)g.W + rb * (size_t)(g.KS / 4) * 64 + lane;
      sq[j] = (const u32x4*)g.SC + rb * (size_t)g.NG * 4 + 2 * (lane >> 5);
    }
    fk_stream_q4_dispatch<NXP, NRMAX>(nr, g.XF, g.KS, g.M, gb, ge, wq, sq, g.NG, acc, lane);
  } else
  fk_stream_dispatch<NWP, NXP, NRMAX>(nr, g.XF, g.KS, g.M, kb, ke, wp, g.wps, acc, lane);
  TRACE_STAMP_AFTER(tr, 2, acc[0][0]);
#pragma unroll
  for (int j = 0; j < NRMAX; ++j)
    if (j < nr)
#pragma unroll
      for (int r = 0; r < 16; ++r) red[(((size_t)w * NRMAX + j) * 16 + r) * 64 + lane] = acc[j][r];
  __syncthreads();
  // the waves share the sum and the publication: item = (row block j, register quad i) -> rows 8i + 4(lane/32) + 0..3
  for (int it = w; it < nr * 4; it += 8) {
    const int j = it >> 2, i = it & 3;
    float v[4];
#pragma unroll
    for (int t = 0; t < 4; ++t) {
      float a = 0.f;
#pragma unroll
      for (int ww = 0; ww < 8; ++ww) a += red[(((size_t)ww * NRMAX + j) * 16 + 4 * i + t) * 64 + lane];
      v[t] = a;
    }
    f32x4 o; o.x = v[0]; o.y = v[1]; o.z = v[2]; o.w = v[3];
    coh_store16(g.PT, pt_quad_bytes(s, g.Npad, (rb0 + j) * 32 + 8 * i + 4 * (lane >> 5), lane & 31), o);
  }
  TRACE_STAMP(tr, 3);
  publish_wait();
  __syncthreads();
  if (threadIdx.x == 0) {
    int old = __hip_atomic_fetch_add(g.counters + grp, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    s_last = (old == g.S - 1);
    if (s_last) __hip_atomic_store(g.counters + grp, 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  }
  __syncthreads();
  if (!s_last) return;
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup");
  const int n0 = rb0 * 32, n1 = min(rb1 * 32, g.N);
  if (n1 <= n0) return;
  if (g.epi != EPI_RESID) block_rstd_finish(g.in_scale, rp.ssq_part, rstd_s, sh_small);
  switch (g.epi) {
    case EPI_QKV: epilogue_qkv<NXP>(g, n0, n1, rstd_s, rp); break;
    case EPI_RESID: epilogue_resid<NXP>(g, grp, n0, n1, sh_small); break;
    case EPI_SWIGLU: epilogue_swiglu<NXP>(g, n0, n1, rstd_s); break;
    default: epilogue_logits(g, n0, n1, rstd_s, rp); break;
  }
  TRACE_STAMP(tr, 4);
}

// Rows of a pass that need no GEMM in front: h = embedding of the row's token.  Writes h, XF(h * gain) and the
// partial sums of squares, one column slab per block (the same outputs a residual epilogue produces).
template <typename EmbT, int NXP>
__global__ __launch_bounds__(256) void k2_embed(Pass pass, const TreeDev* tree, SeqState st, const int* tree_tok,
                                                const EmbT* __restrict__ embed, int vocab, int M, int d, float* h,
                                                const float* gain, bf16_t* xf_out, float* ssq_out) {
  __shared__ float sh[8 * 32];
  const int m = threadIdx.x & 31, slot = threadIdx.x >> 5;          // 8 slots
  const int grp = blockIdx.x, groups = gridDim.x;
  const int c0 = (int)((long)grp * (d / 8) / groups), c1 = (int)((long)(grp + 1) * (d / 8) / groups);
  const bool live = m < M;
  int tok = 0;
  if (live) {
    RowInfo ri = row_info(pass, tree, st, m);
    if (pass.kind == PASS_VERIFY) tok = tree_tok[ri.seq * tree->M + ri.node];
    else tok = st.tokens[(size_t)ri.seq * st.tok_stride + ri.pos];
    tok = min(max(tok, 0), vocab - 1);
  }
  float ss = 0.f;
  for (int c = c0 + slot; c < c1; c += 8) {
    float x[8];
    for (int t = 0; t < 8; ++t) {
      float v = 0.f;
      if (live) {
        if constexpr (sizeof(EmbT) == 4) v = ((const float*)embed)[(size_t)tok * d + 8 * c + t];
        else v = bf16_to_f32(((const bf16_t*)embed)[(size_t)tok * d + 8 * c + t]);
        h[(size_t)m * d + 8 * c + t] = v;
      }
      ss += v * v;
      x[t] = v * gain[8 * c + t];
    }
    if (live) xf_store8(xf_out, m, 8 * c, 1, d / 16, NXP, x);
  }
  sh[slot * 32 + m] = ss;
  __syncthreads();
  if (threadIdx.x < 32) {
    float a = 0.f;
    for (int i = 0; i < 8; ++i) a += sh[i * 32 + threadIdx.x];
    ssq_out[grp * 32 + threadIdx.x] = a;
  }
}

// features[m][k] = h[m][k] * rstd[m] * gain[k]   (the target's final RMSNorm, Sec. 2: f is what the LM head reads)
__global__ __launch_bounds__(256) void k2_features(const float* h, RowScale rs, const float* gain, int M, int d, float* out) {
  __shared__ float tmp[17];
  const int m = blockIdx.x;
  if (m >= M) return;
  const float r = block_row_rstd(rs.ssq, rs.groups, rs.inv_d, rs.eps, m, tmp);
  for (int k = threadIdx.x; k < d; k += blockDim.x) out[(size_t)m * d + k] = h[(size_t)m * d + k] * r * gain[k];
}

// ============================================================================ tree-masked paged attention, <= 32 rows per sequence
// Block = (kv split, query head, sequence), 4 waves.  Each wave runs flash attention on its own 32-token blocks
// entirely in registers on the MFMA units:
//   S^T[tok][q] = K[tok][:] . Q[q][:]      A = K block (32 tokens x 16 dims per step), B = Q fragments (kept in VGPRs)
//   O^T[d][q]  += V[tok][d] * P[q][tok]    A = V^T (gathered so that the token order matches the S^T accumulator
//                                          layout), B = P straight out of the accumulator registers
// fp32 cache values and probabilities are split into bf16 hi + lo on the fly (hi*hi + hi*lo + lo*hi), so the
// result keeps ~16 mantissa bits.  A lane always owns one query (column l%32): running max / sum and the rescale
// of O^T are lane-local, the only cross-lane traffic is one xor-32 shuffle per reduction.  Keys: cache slots
// [0, base) are visible to every row; slot base+j is visible iff bit j of the row's ancestor mask is set (tree
// passes) or j <= the row's own relative index (causal passes).  Waves are merged through LDS, splits through
// coherent partials and the last split to arrive, which writes XF layout for the output projection.
__device__ inline void split8(const float* x, bf16x8& hi, bf16x8& lo) {
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    hi[i] = (__bf16)x[i];
    lo[i] = (__bf16)(x[i] - (float)hi[i]);
  }
}
__device__ inline void load8(const float* p, float* x) {
  const f32x4 a = *(const f32x4*)p, b = *(const f32x4*)(p + 4);
  x[0] = a.x; x[1] = a.y; x[2] = a.z; x[3] = a.w; x[4] = b.x; x[5] = b.y; x[6] = b.z; x[7] = b.w;
}
__device__ inline void load8(const bf16_t* p, float* x) {
  const u32x4 r = *(const u32x4*)p;
  x[0] = __builtin_bit_cast(float, r.x << 16); x[1] = __builtin_bit_cast(float, r.x & 0xFFFF0000u);
  x[2] = __builtin_bit_cast(float, r.y << 16); x[3] = __builtin_bit_cast(float, r.y & 0xFFFF0000u);
  x[4] = __builtin_bit_cast(float, r.z << 16); x[5] = __builtin_bit_cast(float, r.z & 0xFFFF0000u);
  x[6] = __builtin_bit_cast(float, r.w << 16); x[7] = __builtin_bit_cast(float, r.w & 0xFFFF0000u);
}

// Folds NS splits (e, e+1, ...) of one (row, head) into the running (max, denominator, CW outputs): every load of the
// chunk is in flight before the first use.
template <int DH, int CW, int NS>
__device__ __forceinline__ void attn_merge_chunk(const float* part_o, const float* part_ml, size_t e0, int d0, float& mx, float& den, float* x) {
  constexpr int NQ = CW / 4;
  float msv[NS], lsv[NS];
  f32x4 ov[NS][NQ];
#pragma unroll
  for (int u = 0; u < NS; ++u) {
    const size_t e = e0 + u;
    msv[u] = coh_load(part_ml + e * 2);
    lsv[u] = coh_load(part_ml + e * 2 + 1);
#pragma unroll
    for (int qd = 0; qd < NQ; ++qd) ov[u][qd] = coh_load16(part_o, (uint32_t)((e * DH + d0 + 4 * qd) * 4));
  }
  float cmx = mx;
#pragma unroll
  for (int u = 0; u < NS; ++u) cmx = fmaxf(cmx, msv[u]);
  const float resc = (mx == -INFINITY) ? 0.f : __expf(mx - cmx);   // nothing to rescale on the first chunk
  den *= resc;
#pragma unroll
  for (int t = 0; t < CW; ++t) x[t] *= resc;
  mx = cmx;
#pragma unroll
  for (int u = 0; u < NS; ++u) {
    const float wv = (msv[u] != -INFINITY) ? __expf(msv[u] - mx) : 0.f;
    den += wv * lsv[u];
#pragma unroll
    for (int qd = 0; qd < NQ; ++qd) {
      x[4 * qd] += wv * ov[u][qd].x; x[4 * qd + 1] += wv * ov[u][qd].y;
      x[4 * qd + 2] += wv * ov[u][qd].z; x[4 * qd + 3] += wv * ov[u][qd].w;
    }
  }
}

template <typename CT, int DH>
__global__ __launch_bounds__(256) void k2_attn(Pass pass, const TreeDev* tree, SeqState st, KVCache kv,
                                               const float* __restrict__ Q, float* part_o, float* part_ml, int H,
                                               int n_splits, int n_new, float scale, int* counters, bf16_t* xf_out,
                                               int nplanes, unsigned long long* trace, int MT, int rblocks) {
  constexpr int KSN = DH / 16;              // k-steps of the QK product
  constexpr int DB = DH / 32;               // 32-wide blocks of the head dimension
  extern __shared__ __attribute__((aligned(16))) unsigned char smem_a[];
  float* o_s = (float*)smem_a;              // [4 waves][DH][32]
  float* ml_s = o_s + 4 * DH * 32;          // [4 waves][2][32]
  __shared__ int s_last;
  // blockIdx.z = (sequence of the pass, 32-row block of that sequence's rows); MT = 32-row tiles of the XF output
  const int split = blockIdx.x, hd = blockIdx.y, seq_l = blockIdx.z / rblocks, rblk = blockIdx.z % rblocks;
  // optional time stamps: 0 entered, 1 keys/values consumed, 2 waves merged + partials written, 3 arrived, 4 splits merged
  unsigned long long* tr = TRACE_PTR((trace && threadIdx.x == 0 && seq_l == 0) ? trace + ((size_t)hd * gridDim.x + split) * 8 : nullptr);
  TRACE_STAMP(tr, 0);
  const int r0 = seq_l * pass.rows_per_seq + 32 * rblk;
  const int R = min(32, pass.rows_per_seq - 32 * rblk);
  const int kvh = hd / (H / kv.n_kv_heads);
  const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
  const int q = lane & 31, hh = lane >> 5;
  const RowInfo r_first = row_info(pass, tree, st, r0);
  const int seq = r_first.seq, base = r_first.base;
  // this lane's query row
  int rel = 0, causal = 1;
  unsigned long long mask = 0ull;
  if (q < R) {
    const RowInfo ri = row_info(pass, tree, st, r0 + q);
    rel = ri.rel; causal = ri.causal; mask = ri.mask;
  }
  // The scaled queries as bf16 hi + lo B-operand fragments live in LDS, built once by the four waves together (wave w
  // converts k-steps w, w+4, ...); they share the memory of o_s, which is not written before every wave has left the
  // key loop.  (One load and one conversion of the queries per work-group instead of one per wave.)
  bf16x8* q_s = (bf16x8*)smem_a;                               // [2 planes][KSN][64 lanes]
  for (int ks = w; ks < KSN; ks += 4) {
    float x[8];
    if (q < R) {
      load8(Q + ((size_t)(r0 + q) * H + hd) * DH + 16 * ks + 8 * hh, x);
#pragma unroll
      for (int t = 0; t < 8; ++t) x[t] *= scale;
    } else {
#pragma unroll
      for (int t = 0; t < 8; ++t) x[t] = 0.f;
    }
    bf16x8 h8, l8;
    split8(x, h8, l8);
    q_s[(0 * KSN + ks) * 64 + lane] = h8;
    q_s[(1 * KSN + ks) * 64 + lane] = l8;
  }
  __syncthreads();
  // causal passes (prompt chunks, pending rows): the rows of this 32-row block see no new token beyond its own last row,
  // so the blocks of keys after it are not visited at all (they would contribute exp(-inf) = 0: same bits, less work)
  const int T = base + (r_first.causal ? min(n_new, 32 * rblk + R) : n_new);
  // the split boundaries depend on `base` only, so a row sees the same partition whatever else is in the pass
  const int span = base + max(64, (n_new + 63) / 64 * 64);   // passes with at most 64 new rows share one partition
  const int tps = ((span + n_splits - 1) / n_splits + 63) / 64 * 64;
  const int t_begin = split * tps, t_end = min(T, t_begin + tps);
  float m_run = -INFINITY, l_run = 0.f;
  f32x16 oacc[DB];
#pragma unroll
  for (int b = 0; b < DB; ++b)
#pragma unroll
    for (int r = 0; r < 16; ++r) oacc[b][r] = 0.f;

  // Wave w takes every 4th 32-token block.  A block starts on a multiple of 32 and therefore lies inside one 64-token
  // (or larger) page.  The keys of the NEXT block are requested as soon as the scores of the current one are done
  // (the registers are free then), after the current block's values, so that they travel while the softmax and the
  // P V product run: a wave that walks several blocks pays about one memory round trip per block.
  float kx[KSN][8];
  size_t blk = 0;
  {
    const int tok0 = t_begin + 32 * w;
    if (tok0 < t_end) {
      blk = kv_offset(kv, seq, tok0, kvh);
      const CT* kp = (const CT*)kv.k + blk + (size_t)(lane & 31) * DH + 8 * hh;
#pragma unroll
      for (int ks = 0; ks < KSN; ++ks) load8(kp + 16 * ks, kx[ks]);
    }
  }
  for (int tok0 = t_begin + 32 * w; tok0 < t_end; tok0 += 128) {
    const CT* vp = (const CT*)kv.v + blk;
    const bool more = tok0 + 128 < t_end;
    const size_t blk_next = more ? kv_offset(kv, seq, tok0 + 128, kvh) : 0;   // look-up in flight during the scores
    f32x16 sacc;
#pragma unroll
    for (int r = 0; r < 16; ++r) sacc[r] = 0.f;
#pragma unroll
    for (int ks = 0; ks < KSN; ++ks) {
      bf16x8 kh, kl;
      split8(kx[ks], kh, kl);
      const bf16x8 qh = q_s[(0 * KSN + ks) * 64 + lane], ql = q_s[(1 * KSN + ks) * 64 + lane];
      sacc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kh, qh, sacc, 0, 0, 0);
      sacc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kh, ql, sacc, 0, 0, 0);
      sacc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kl, qh, sacc, 0, 0, 0);
    }
    // V gathers go out before the softmax arithmetic: slot t of lane-half hh in k-step j is the token that
    // accumulator register 8j+t of the same lane-half holds
    float vx[2][DB][8];
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int b = 0; b < DB; ++b)
#pragma unroll
        for (int t = 0; t < 8; ++t) {
          const int tl = 16 * j + 8 * (t >> 2) + 4 * hh + (t & 3);
          vx[j][b][t] = cache_load(vp + (size_t)tl * DH + 32 * b + (lane & 31));
        }
    if (more) {
      const CT* kp = (const CT*)kv.k + blk_next + (size_t)(lane & 31) * DH + 8 * hh;
#pragma unroll
      for (int ks = 0; ks < KSN; ++ks) load8(kp + 16 * ks, kx[ks]);
    }
    blk = blk_next;
    // mask, running max and sum for this lane's query
    float bmax = -INFINITY;
#pragma unroll
    for (int r = 0; r < 16; ++r) {
      const int t = tok0 + 8 * (r >> 2) + 4 * hh + (r & 3);
      bool vis = t < base;
      if (!vis) {
        const int j = t - base;
        vis = causal ? (j <= rel) : (j < 64 && ((mask >> j) & 1ull));
      }
      vis = vis && t < t_end && q < R;
      sacc[r] = vis ? sacc[r] : -INFINITY;
      bmax = fmaxf(bmax, sacc[r]);
    }
    bmax = fmaxf(bmax, __shfl_xor(bmax, 32, 64));
    const float m_new = fmaxf(m_run, bmax);
    const float alpha = (m_run == -INFINITY) ? 0.f : __expf(m_run - m_new);
    float psum = 0.f, pv[2][8];                                // two arrays: a pointer into one of 16 ends up on the stack
#pragma unroll
    for (int r = 0; r < 16; ++r) {
      const float e = (m_new == -INFINITY) ? 0.f : __expf(sacc[r] - m_new);
      pv[r >> 3][r & 7] = e;
      psum += e;
    }
    psum += __shfl_xor(psum, 32, 64);
    l_run = l_run * alpha + psum;
    m_run = m_new;
#pragma unroll
    for (int b = 0; b < DB; ++b)
#pragma unroll
      for (int r = 0; r < 16; ++r) oacc[b][r] *= alpha;
#pragma unroll
    for (int j = 0; j < 2; ++j) {
      bf16x8 ph, pl;
      split8(pv[j], ph, pl);
#pragma unroll
      for (int b = 0; b < DB; ++b) {
        bf16x8 vh, vl;
        split8(vx[j][b], vh, vl);
        oacc[b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vh, ph, oacc[b], 0, 0, 0);
        oacc[b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vh, pl, oacc[b], 0, 0, 0);
        oacc[b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vl, ph, oacc[b], 0, 0, 0);
      }
    }
  }
  TRACE_STAMP(tr, 1);
  __syncthreads();                          // every wave is done with the query fragments that o_s overlays
  // merge the 4 waves through LDS: o_s[w][d][q], d = 32b + 8(r/4) + 4hh + r%4
#pragma unroll
  for (int b = 0; b < DB; ++b)
#pragma unroll
    for (int r = 0; r < 16; ++r) o_s[((size_t)w * DH + 32 * b + 8 * (r >> 2) + 4 * hh + (r & 3)) * 32 + q] = oacc[b][r];
  if (hh == 0) { ml_s[(w * 2 + 0) * 32 + q] = m_run; ml_s[(w * 2 + 1) * 32 + q] = l_run; }
  __syncthreads();
  // thread = (query q2, 8-wide chunks c = tid/32, tid/32 + 8, ... of the head dimension)
  const int q2 = tid & 31;
  float mm = -INFINITY;
#pragma unroll
  for (int ww = 0; ww < 4; ++ww) mm = fmaxf(mm, ml_s[(ww * 2) * 32 + q2]);
  float wgt[4], L = 0.f;
#pragma unroll
  for (int ww = 0; ww < 4; ++ww) {
    const float mw = ml_s[(ww * 2) * 32 + q2];
    wgt[ww] = (mw == -INFINITY) ? 0.f : __expf(mw - mm);
    L += wgt[ww] * ml_s[(ww * 2 + 1) * 32 + q2];
  }
  const int KSX = H * DH / 16;
  const float inv = L > 0.f ? 1.0f / L : 0.f;
  for (int c = tid >> 5; c < DH / 8; c += 8) {
    float o[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      float a = 0.f;
#pragma unroll
      for (int ww = 0; ww < 4; ++ww) a += wgt[ww] * o_s[((size_t)ww * DH + 8 * c + i) * 32 + q2];
      o[i] = a;
    }
    if (q2 >= R) continue;
    if (n_splits == 1) {
#pragma unroll
      for (int t = 0; t < 8; ++t) o[t] *= inv;
      xf_store8(xf_out, r0 + q2, hd * DH + 8 * c, MT, KSX, nplanes, o);
    } else {
      const uint32_t po = (uint32_t)(((((size_t)(r0 + q2) * H + hd) * n_splits + split) * DH + 8 * c) * 4);
      f32x4 v0, v1;
      v0.x = o[0]; v0.y = o[1]; v0.z = o[2]; v0.w = o[3]; v1.x = o[4]; v1.y = o[5]; v1.z = o[6]; v1.w = o[7];
      coh_store16(part_o, po, v0);
      coh_store16(part_o, po + 16, v1);
    }
  }
  TRACE_STAMP(tr, 2);
  if (n_splits == 1) return;
  if (q2 < R && tid < 32) {
    const size_t ofs = (((size_t)(r0 + q2) * H + hd) * n_splits + split) * 2;
    coh_store(part_ml + ofs, mm);
    coh_store(part_ml + ofs + 1, L);
  }
  publish_wait();
  __syncthreads();
  if (tid == 0) {
    int* cnt = counters + blockIdx.z * H + hd;
    int old = __hip_atomic_fetch_add(cnt, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    s_last = (old == n_splits - 1);
    if (s_last) __hip_atomic_store(cnt, 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  }
  __syncthreads();
  TRACE_STAMP(tr, 3);
  if (!s_last) return;
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup");
  // merge the splits of (sequence, head): thread = (row, CW-wide column chunk), one item per thread in the usual
  // shapes.  Every load of up to 8 splits -- (max, sum) pairs and partial outputs -- is in flight at once, so the
  // merge costs one memory round trip; more splits continue with a running rescale, in split order.
  constexpr int CW = DH >= 128 ? 16 : 8;
  for (int it = tid; it < R * (DH / CW); it += 256) {
    const int r = it / (DH / CW), d0 = (it % (DH / CW)) * CW;
    const size_t rowhead = ((size_t)(r0 + r) * H + hd) * n_splits;
    float mx = -INFINITY, den = 0.f, x[CW];
#pragma unroll
    for (int t = 0; t < CW; ++t) x[t] = 0.f;
    for (int sp0 = 0; sp0 < n_splits; sp0 += 8) {
      switch (min(n_splits - sp0, 8)) {                        // uniform: exactly the loads that are needed
        case 1: attn_merge_chunk<DH, CW, 1>(part_o, part_ml, rowhead + sp0, d0, mx, den, x); break;
        case 2: attn_merge_chunk<DH, CW, 2>(part_o, part_ml, rowhead + sp0, d0, mx, den, x); break;
        case 3: attn_merge_chunk<DH, CW, 3>(part_o, part_ml, rowhead + sp0, d0, mx, den, x); break;
        case 4: attn_merge_chunk<DH, CW, 4>(part_o, part_ml, rowhead + sp0, d0, mx, den, x); break;
        case 5: attn_merge_chunk<DH, CW, 5>(part_o, part_ml, rowhead + sp0, d0, mx, den, x); break;
        case 6: attn_merge_chunk<DH, CW, 6>(part_o, part_ml, rowhead + sp0, d0, mx, den, x); break;
        case 7: attn_merge_chunk<DH, CW, 7>(part_o, part_ml, rowhead + sp0, d0, mx, den, x); break;
        default: attn_merge_chunk<DH, CW, 8>(part_o, part_ml, rowhead + sp0, d0, mx, den, x); break;
      }
    }
    const float inv = den > 0.f ? 1.0f / den : 0.f;
#pragma unroll
    for (int t = 0; t < CW; ++t) x[t] *= inv;
#pragma unroll
    for (int h8 = 0; h8 < CW / 8; ++h8) xf_store8(xf_out, r0 + r, hd * DH + d0 + 8 * h8, MT, KSX, nplanes, x + 8 * h8);
  }
  TRACE_STAMP(tr, 4);
}
